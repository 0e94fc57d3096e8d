"""Helpers of the GPU parity tests: build the oracle and the engine from the same seeded weights,
teacher-force oracle states through the library, and apply the agreement rules.

Agreement rules (per step, on the oracle's state before the step):
  * logits: max|gpu - oracle| / max|oracle| <= tol  (1e-4 for fp32 models, 2e-2 for bf16 models);
  * greedy token: equal, unless the oracle's top-1 / top-2 logit gap at that position is below
    twice the measured absolute logit error (a near-tie the arithmetic cannot resolve);
  * unmask decision: equal, unless |p_j - tau| < 1e-3, or the position is a masked one whose oracle
    confidence is within the measured relative confidence error (x2; at least 1e-3) of the highest
    masked confidence, i.e. a candidate for the forced top-1 that the arithmetic cannot tell apart.
Exempt positions are counted and returned; everything else must match exactly.
"""
from __future__ import annotations

import types

import numpy as np
import torch

from oracle import l2pd_oracle as O
from paper_2509_25188_amd import binding as Bd
from paper_2509_25188_amd import synth


def oracle_model(shape: synth.ModelShape, weights, dtype=np.float32, gemm_input="fp32") -> O.Model:
    s = types.SimpleNamespace(**{k: getattr(shape, k) for k in
                                 ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "mask_id",
                                  "eos_id", "rope_base", "rms_eps")})
    return O.Model(s, {k: synth.to_numpy(v) for k, v in weights.items()}, dtype, gemm_input)


def to_dev(weights, device="cuda"):
    return {k: v.to(device) for k, v in weights.items()}


def np_filter(flt):
    return {k: v.detach().cpu().numpy() for k, v in flt.items()}


def tol_for(shape: synth.ModelShape) -> float:
    return 1e-4 if shape.dtype == "fp32" else 2e-2


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    return float(np.max(np.abs(gpu.astype(np.float64) - ref.astype(np.float64))) / np.max(np.abs(ref)))


def top2_gap(logits: np.ndarray, mask_id: int) -> np.ndarray:
    z = np.array(logits, dtype=np.float64, copy=True)
    z[:, mask_id] = -np.inf
    part = np.partition(z, -2, axis=-1)
    return part[:, -1] - part[:, -2]


class StepReport:
    def __init__(self):
        self.steps = 0
        self.max_logit_err = 0.0
        self.max_conf_err = 0.0
        self.max_p_err = 0.0
        self.exempt_tokens = 0
        self.exempt_decisions = 0
        self.positions = 0

    def __repr__(self):
        return (f"steps={self.steps} positions={self.positions} logit_err={self.max_logit_err:.3e} "
                f"conf_err={self.max_conf_err:.3e} p_err={self.max_p_err:.3e} "
                f"exempt_tokens={self.exempt_tokens} exempt_decisions={self.exempt_decisions}")


def check_step(rec, taps, b, shape, tau, tol, rep: StepReport, check_logits=True):
    """Compares one oracle step record with the library's taps for sequence b of the batch."""
    n = len(rec["conf"])     # fewer than block_len when step-granular EoTP has shortened the sequence
    conf = taps["conf"][b].cpu().numpy()[:n]
    pred = taps["pred"][b].cpu().numpy()[:n]
    p = taps["p"][b].cpu().numpy()[:n]
    sel = taps["sel"][b].cpu().numpy().astype(bool)
    assert not sel[n:].any(), "a discarded position was unmasked"
    sel = sel[:n]
    masked = rec["masked"]
    rep.steps += 1
    rep.positions += len(conf)
    abs_err = None
    if check_logits and "logits" in taps:
        lg = taps["logits"][b].cpu().numpy()[:n]
        e = rel_err(lg, rec["logits"])
        rep.max_logit_err = max(rep.max_logit_err, e)
        assert e <= tol, f"logits off by {e:.3e} (tol {tol})"
        abs_err = float(np.max(np.abs(lg - rec["logits"])))
    conf_err = float(np.max(np.abs(conf - rec["conf"]) / rec["conf"]))
    rep.max_conf_err = max(rep.max_conf_err, conf_err)
    assert conf_err <= max(20 * tol, 1e-3), f"confidence off by {conf_err:.3e}"
    # greedy tokens
    bad = np.nonzero(pred != rec["pre"])[0]
    if len(bad):
        gap = top2_gap(rec["logits"], shape.mask_id)
        lim = 2 * (abs_err if abs_err is not None else tol * float(np.max(np.abs(rec["logits"]))))
        for j in bad:
            assert gap[j] < lim, f"token mismatch at {j}: gap {gap[j]:.3e} >= {lim:.3e}"
            rep.exempt_tokens += 1
    # filter output
    p_err = float(np.max(np.abs(p - rec["p"])))
    rep.max_p_err = max(rep.max_p_err, p_err)
    assert p_err <= max(10 * tol, 1e-4), f"filter output off by {p_err:.3e}"
    # unmask decisions
    diff = np.nonzero(sel != rec["sel"])[0]
    if len(diff):
        # the forced position is the masked one of highest confidence: positions whose oracle
        # confidence lies within the measured confidence error of the top are interchangeable
        cm = np.where(masked, rec["conf"], -np.inf)
        c1 = float(np.max(cm))
        lim_c = max(2 * conf_err, 1e-3)
        for j in diff:
            near_top = bool(masked[j]) and (c1 - float(cm[j])) / c1 < lim_c
            ok = abs(float(rec["p"][j]) - tau) < 1e-3 or near_top
            assert ok, (f"unmask decision mismatch at {j}: p={rec['p'][j]:.6f} gpu p={p[j]:.6f} tau={tau} "
                        f"masked={bool(masked[j])} top conf {c1:.6f} conf[j] {cm[j]:.6f} gpu conf[j] {conf[j]:.6f} "
                        f"conf_err {conf_err:.3e} gpu sel {np.nonzero(sel)[0].tolist()} "
                        f"oracle sel {np.nonzero(rec['sel'])[0].tolist()}")
            rep.exempt_decisions += 1
    return len(bad) == 0 and len(diff) == 0


def teacher_forced(engine: Bd.Engine, trace_per_seq, prompt_len, cfg, flt_dev, shape, tau, rep: StepReport,
                   want_logits=True, sample=None):
    """Feeds every (or every `sample`-th) oracle step state through l2pd_denoise_step.

    trace_per_seq: list over sequences of oracle trace lists; sequences are stepped as a batch of one
    each (B = 1) so that every sequence's own state can be imposed."""
    tol = tol_for(shape)
    dev = "cuda"
    all_match = True
    for trace in trace_per_seq:
        for i, rec in enumerate(trace):
            if sample and i % sample and i != len(trace) - 1:
                continue
            X = torch.tensor(rec["X_before"], dtype=torch.int32, device=dev).view(1, -1)
            state = torch.tensor([[rec["block"], i, 0]], dtype=torch.int32, device=dev)
            # dual cache: the stored K/V are those of the block's first state; later steps of the
            # block must run on that store, not on one rebuilt from their own state
            first_of_block = i == 0 or trace[i - 1]["block"] != rec["block"]
            if cfg.kv_cache == Bd.CACHE_DUAL:
                assert not sample, "dual-cache steps depend on the block's earlier calls: no sampling"
                cfg.keep_kv = 0 if first_of_block else 1
            taps = engine.denoise_step(X, prompt_len, state, flt_dev, cfg, want_logits=want_logits)
            torch.cuda.synchronize()
            same = check_step(rec, taps, 0, shape, tau, tol, rep, check_logits=want_logits)
            all_match &= same
            if same:
                # the state after the step must be the oracle's next state
                lo = prompt_len + rec["block"] * cfg.block_len
                after = np.array(rec["X_before"], copy=True)
                idx = np.nonzero(rec["sel"])[0]
                after[lo + idx] = rec["pre"][idx]
                np.testing.assert_array_equal(X.cpu().numpy()[0], after)
                assert int(state[0, 1]) == i + 1
    return all_match


def oracle_generate(model, prompt_row, w: synth.Workload, flt_np, trace=None, tau=None):
    bias = (w.model.eos_id, w.bias_from, w.bias_value) if w.bias_value else None
    if w.eotp_step:
        assert not (w.prefix_cache or w.dual_cache)
        return O.generate_eotp_step(model, prompt_row, w.gen_len, w.block_len, w.model.mask_id, w.model.eos_id,
                                    flt_np, w.threshold if tau is None else tau, bias=bias, trace=trace)
    return O.generate(model, prompt_row, w.gen_len, w.block_len, w.model.mask_id, w.model.eos_id, flt_np,
                      w.threshold if tau is None else tau, eotp=w.eotp, bias=bias, prefix_cache=w.prefix_cache,
                      trace=trace, dual_cache=w.dual_cache)


def cfg_for(w: synth.Workload, tau=None):
    bias = (w.model.eos_id, w.bias_from, w.bias_value) if w.bias_value else None
    return Bd.Engine.cfg_struct(w.gen_len, w.block_len, w.threshold if tau is None else tau,
                                Bd.EOTP_STEP if w.eotp_step else w.eotp,
                                w.prefix_cache, bias, w.dual_cache)


def random_state(w: synth.Workload, seed: int, block: int, n_committed: int, b: int = 0):
    """A teacher-forced state: prompt of sequence b, blocks before `block` committed with random
    tokens, `n_committed` random positions of the active block committed, the rest masked."""
    rng = np.random.default_rng(seed)
    prompt = synth.make_prompt(1234, max(w.batch, b + 1), w.prompt_len, w.prompt_hi)[b].numpy()
    X = np.concatenate([prompt.astype(np.int64), np.full(w.gen_len, w.model.mask_id, dtype=np.int64)])
    lo = w.prompt_len + block * w.block_len
    X[w.prompt_len:lo] = rng.integers(0, w.prompt_hi, lo - w.prompt_len)
    idx = rng.choice(w.block_len, n_committed, replace=False)
    X[lo + idx] = rng.integers(0, w.prompt_hi, n_committed)
    return X


def oracle_step_record(model, X, w: synth.Workload, flt_np, block: int):
    """The oracle's record of one step taken from state X (X is not modified)."""
    bias = (w.model.eos_id, w.bias_from, w.bias_value) if w.bias_value else None
    Xc = np.array(X, copy=True)
    cache = model.prefix_kv(Xc[:w.prompt_len + block * w.block_len]) if w.prefix_cache else (
        model.full_kv(Xc) if w.dual_cache else None)
    rec = O.denoise_step(model, Xc, w.prompt_len, block, w.block_len, w.model.mask_id, flt_np, w.threshold, bias,
                         cache, w.dual_cache)
    rec.update(X_before=np.array(X, copy=True), block=block)
    return rec
