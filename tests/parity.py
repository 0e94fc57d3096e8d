"""Helpers of the GPU parity tests: build the oracle and the engine from the same seeded weights,
teacher-force oracle states through the library, and apply the agreement rules.

Agreement rules (per step, on the oracle's state before the step).  Every margin is a property of the
ORACLE at that step; nothing is widened by what the GPU path is measured to do.
  * logits: max|gpu - oracle| / max|oracle| <= tol  (1e-4 for fp32 models, 2e-2 for bf16 models);
  * resolution D of the step, in logit units: for bf16 models the largest difference between the logits
    of the two oracle evaluations of that state (bf16-rounded matrix-product inputs, the primary one, and
    float32 activations): two correct evaluations of the same model in the two number formats differ
    by that much, so no bf16 path can be asked to resolve less.  Where no second evaluation is at hand,
    and for fp32 models, D = tol * max|oracle logit| (what the stated tolerance permits);
  * confidence: |log conf_gpu - log conf_oracle| <= 2 * tol * max|oracle logit| (conf is exp(max - logsumexp),
    each term moves by at most the permitted logit error);
  * greedy token: equal, unless the oracle's best / second-best logit gap at that position is below 2 D;
  * filter output: |p_gpu - p_oracle| <= max(10 tol, 1e-4);
  * unmask decision: equal, unless |p_j - tau| < 1e-3, or the position is a masked one whose oracle
    log-confidence lies within 2 D of the highest masked one (a candidate for the forced most-confident
    position that the number format cannot tell from the winner).
Exempt positions are counted and returned; the caller bounds the count.  Everything else must match exactly.
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


def resolution(rec, shape, tol):
    """D of the rules above for one oracle step record (logit units)."""
    absmax = float(rec["absmax"]) if "absmax" in rec else float(np.max(np.abs(rec["logits"])))
    if shape.dtype != "fp32" and rec.get("fmt_abs") is not None:
        return float(rec["fmt_abs"]), absmax
    return tol * absmax, absmax


def check_step(rec, taps, b, shape, tau, tol, rep: StepReport, check_logits=True):
    """Compares one oracle step record with the library's taps for sequence b of the batch.

    `rec` holds conf / pre / p / sel / masked and either the block's `logits` or what a stored
    trajectory keeps of them (`absmax`, `gap`, and at sampled steps `cols_fixed` / `lg_fixed` /
    `cols_top` / `lg_top`); `fmt_abs`, if present, is the distance between the two oracle evaluations."""
    n = len(rec["conf"])     # fewer than block_len when step-granular EoTP has shortened the sequence
    conf = taps["conf"][b].cpu().numpy()[:n]
    pred = taps["pred"][b].cpu().numpy()[:n]
    p = taps["p"][b].cpu().numpy()[:n]
    sel = taps["sel"][b].cpu().numpy().astype(bool)
    assert not sel[n:].any(), "a discarded position was unmasked"
    sel = sel[:n]
    masked = np.asarray(rec["masked"]).astype(bool)
    rsel = np.asarray(rec["sel"]).astype(bool)
    rep.steps += 1
    rep.positions += len(conf)
    D, absmax = resolution(rec, shape, tol)
    if check_logits and "logits" in taps:
        if "logits" in rec:
            lg = taps["logits"][b].cpu().numpy()[:n]
            e = float(np.max(np.abs(lg.astype(np.float64) - rec["logits"]))) / absmax
        elif "lg_fixed" in rec:
            # stored trajectory: sampled columns (a fixed stride, and the oracle's largest logits of every row)
            tl = taps["logits"][b][:n]
            dev = tl.device
            got_f = tl[:, torch.as_tensor(rec["cols_fixed"], dtype=torch.long, device=dev)].cpu().numpy()
            got_t = torch.gather(tl, 1, torch.as_tensor(rec["cols_top"], dtype=torch.long, device=dev)).cpu().numpy()
            e = max(float(np.max(np.abs(got_f.astype(np.float64) - rec["lg_fixed"]))),
                    float(np.max(np.abs(got_t.astype(np.float64) - rec["lg_top"])))) / absmax
        else:
            e = None
        if e is not None:
            rep.max_logit_err = max(rep.max_logit_err, e)
            lim = rec.get("logit_tol", tol)
            assert e <= lim, f"logits off by {e:.3e} (tol {lim:.3e})"
    conf_err = float(np.max(np.abs(np.log(conf.astype(np.float64)) - np.log(np.asarray(rec["conf"], dtype=np.float64)))))
    rep.max_conf_err = max(rep.max_conf_err, conf_err)
    conf_lim = 2 * float(rec.get("logit_tol", tol)) * absmax
    assert conf_err <= conf_lim, f"log confidence off by {conf_err:.3e} (limit {conf_lim:.3e})"
    # greedy tokens
    bad = np.nonzero(pred != rec["pre"])[0]
    if len(bad):
        gap = rec["gap"] if "gap" in rec else top2_gap(rec["logits"], shape.mask_id)
        for j in bad:
            assert gap[j] < 2 * D, f"token mismatch at {j}: oracle gap {gap[j]:.3e} >= 2 D = {2 * D:.3e}"
            rep.exempt_tokens += 1
    # filter output
    p_err = float(np.max(np.abs(p - rec["p"])))
    rep.max_p_err = max(rep.max_p_err, p_err)
    assert p_err <= max(10 * tol, 1e-4), f"filter output off by {p_err:.3e}"
    # unmask decisions
    diff = np.nonzero(sel != rsel)[0]
    if len(diff):
        lc = np.where(masked, np.log(np.asarray(rec["conf"], dtype=np.float64)), -np.inf)
        l1 = float(np.max(lc))
        for j in diff:
            near_top = bool(masked[j]) and l1 - float(lc[j]) < 2 * D
            ok = abs(float(rec["p"][j]) - tau) < 1e-3 or near_top
            assert ok, (f"unmask decision mismatch at {j}: p={rec['p'][j]:.6f} gpu p={p[j]:.6f} tau={tau} "
                        f"masked={bool(masked[j])} top log conf {l1:.6f} log conf[j] {lc[j]:.6f} gpu conf[j] {conf[j]:.6f} "
                        f"D {D:.3e} gpu sel {np.nonzero(sel)[0].tolist()} "
                        f"oracle sel {np.nonzero(rsel)[0].tolist()}")
            rep.exempt_decisions += 1
    return len(bad) == 0 and len(diff) == 0


class Forced:
    """Outcome of teacher forcing: truthy when every step matched with no exemption; `first_exempt[k]` is
    the index of sequence k's first step with an exempt position (None if it has none)."""

    def __init__(self):
        self.first_exempt = []

    def __bool__(self):
        return all(f is None for f in self.first_exempt)


def alt_block_logits(alt, trace, i, w: synth.Workload):
    """Biased logits of step i's block from the same state under the oracle `alt` (the second evaluation
    that defines the resolution D).  Caches of the cached modes are rebuilt from the trace: the prefix
    tokens do not change within a block, and the dual store is that of the block's first state."""
    rec = trace[i]
    blk = rec["block"]
    lo = w.prompt_len + blk * w.block_len
    n = len(rec["conf"])
    X = np.asarray(rec["X_before"])
    if w.eotp_step:
        lg = alt.forward(X[:rec["t_eff"]], lo, n)
    elif w.prefix_cache:
        lg = alt.forward_block_cached(alt.prefix_kv(X[:lo]), X[lo:lo + w.block_len], lo)
    elif w.dual_cache:
        j = i
        while j > 0 and trace[j - 1]["block"] == blk:
            j -= 1
        lg = alt.forward_block_dual(alt.full_kv(np.asarray(trace[j]["X_before"])), X[lo:lo + w.block_len], lo)
    else:
        lg = alt.forward(X, lo, w.block_len)
    bias = (w.model.eos_id, w.bias_from, w.bias_value) if w.bias_value else None
    return O.apply_bias(lg, blk * w.block_len, bias)


def annotate_fmt(traces, alt, w: synth.Workload):
    """Adds rec["fmt_abs"] = max |logits - logits under `alt`| to every step record (bf16 models: `alt` is
    the oracle with float32 activations while the records come from the one with bf16-rounded inputs)."""
    for trace in traces:
        for i, rec in enumerate(trace):
            rec["fmt_abs"] = float(np.max(np.abs(alt_block_logits(alt, trace, i, w).astype(np.float64) - rec["logits"])))


def teacher_forced(engine: Bd.Engine, trace_per_seq, prompt_len, cfg, flt_dev, shape, tau, rep: StepReport,
                   want_logits=True, sample=None):
    """Feeds every (or every `sample`-th) oracle step state through l2pd_denoise_step.

    trace_per_seq: list over sequences of oracle trace lists; sequences are stepped as a batch of one
    each (B = 1) so that every sequence's own state can be imposed.  `want_logits` may be a callable
    (record -> bool): stored trajectories keep logits at sampled steps only."""
    tol = tol_for(shape)
    dev = "cuda"
    out = Forced()
    for trace in trace_per_seq:
        first_exempt = None
        for i, rec in enumerate(trace):
            if sample and i % sample and i != len(trace) - 1:
                continue
            X = torch.tensor(np.asarray(rec["X_before"]), dtype=torch.int32, device=dev).view(1, -1)
            state = torch.tensor([[rec["block"], i, 0]], dtype=torch.int32, device=dev)
            # dual cache: the stored K/V are those of the block's first state; later steps of the
            # block must run on that store, not on one rebuilt from their own state
            first_of_block = i == 0 or trace[i - 1]["block"] != rec["block"]
            if cfg.kv_cache == Bd.CACHE_DUAL:
                assert not sample, "dual-cache steps depend on the block's earlier calls: no sampling"
                cfg.keep_kv = 0 if first_of_block else 1
            wl = want_logits(rec) if callable(want_logits) else want_logits
            taps = engine.denoise_step(X, prompt_len, state, flt_dev, cfg, want_logits=wl)
            torch.cuda.synchronize()
            same = check_step(rec, taps, 0, shape, tau, tol, rep, check_logits=wl)
            if not same and first_exempt is None:
                first_exempt = i
            if same:
                # the state after the step must be the oracle's next state
                lo = prompt_len + rec["block"] * cfg.block_len
                after = np.array(rec["X_before"], copy=True)
                idx = np.nonzero(np.asarray(rec["sel"]))[0]
                after[lo + idx] = np.asarray(rec["pre"])[idx]
                np.testing.assert_array_equal(X.cpu().numpy()[0], after)
                assert int(state[0, 1]) == i + 1
        out.first_exempt.append(first_exempt)
    return out


def check_generate(tok_row, steps, dlen, trace, resp, o_steps, o_dlen, first_exempt, prompt_len, block_len, what=""):
    """l2pd_generate's result for one sequence against the oracle's.  With no exempt position on the
    oracle's trajectory the two must be identical.  Otherwise both trajectories coincide up to the first
    step with an exempt position, so everything the oracle committed before that step must be in the
    result, and the rest is reported."""
    tok_row = np.asarray(tok_row)
    if first_exempt is None:
        np.testing.assert_array_equal(tok_row, resp)
        assert int(steps) == int(o_steps) and int(dlen) == int(o_dlen)
        return True
    keep = min(int(dlen), int(o_dlen))     # step-granular EoTP discards what was committed behind the end-of-text
    for rec in trace[:first_exempt]:
        g0 = rec["block"] * block_len
        idx = np.nonzero(np.asarray(rec["sel"]))[0]
        idx = idx[g0 + idx < keep]
        np.testing.assert_array_equal(tok_row[g0 + idx], np.asarray(rec["pre"])[idx])
    same = bool(np.array_equal(tok_row, resp)) and int(steps) == int(o_steps)
    print(f"{what}: first exempt step {first_exempt} of {len(trace)}; free-running result identical to the oracle's: {same} "
          f"(steps {int(steps)} vs {int(o_steps)}, {int(np.sum(tok_row != np.asarray(resp)))} tokens differ)")
    return same


def load_trajectory(path):
    """A stored oracle trajectory (tests/golden/make_trajectories.py) as (meta, per-step records, result).
    Every record carries the file's largest fmt_abs as its resolution D (the distance between the two oracle
    evaluations is a property of model and depth; it is stored at sampled steps), and sampled steps carry
    their logit samples and, where the float64 evaluation was stored, the tolerance derived from it."""
    import json
    z = np.load(path)
    meta = json.loads(str(z["meta"]))
    recs = []
    if "block" in z:
        fmt = float(np.nanmax(z["fmt_abs"]))
        smp = {int(i): k for k, i in enumerate(z["smp_idx"])}
        floor = z["floor_abs"]
        have_floor = np.isfinite(floor)
        floor_rel = float(np.max(floor[have_floor] / z["absmax"][z["smp_idx"][have_floor]])) if have_floor.any() else 0.0
        for i in range(len(z["block"])):
            rec = dict(X_before=z["X_before"][i], block=int(z["block"][i]), conf=z["conf"][i], pre=z["pre"][i],
                       p=z["p"][i], sel=z["sel"][i].astype(bool), masked=z["masked"][i].astype(bool),
                       absmax=float(z["absmax"][i]), gap=z["gap"][i], fmt_abs=fmt)
            if i in smp:
                k = smp[i]
                rec.update(cols_fixed=z["cols_fixed"], lg_fixed=z["lg_fixed"][k], cols_top=z["cols_top"][k],
                           lg_top=z["lg_top"][k])
            recs.append(rec)
        meta["fmt_abs_max"] = fmt
        meta["floor_rel_max"] = floor_rel
    result = (z["tokens"], int(z["steps"]), int(z["decoded_len"])) if "tokens" in z else None
    return meta, recs, result


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


def oracle_step_record(model, X, w: synth.Workload, flt_np, block: int, alt=None):
    """The oracle's record of one step taken from state X (X is not modified).  With `alt` (the second
    oracle evaluation) the record also carries fmt_abs, the distance between the two sets of logits."""
    bias = (w.model.eos_id, w.bias_from, w.bias_value) if w.bias_value else None
    Xc = np.array(X, copy=True)
    cache = model.prefix_kv(Xc[:w.prompt_len + block * w.block_len]) if w.prefix_cache else (
        model.full_kv(Xc) if w.dual_cache else None)
    rec = O.denoise_step(model, Xc, w.prompt_len, block, w.block_len, w.model.mask_id, flt_np, w.threshold, bias,
                         cache, w.dual_cache)
    rec.update(X_before=np.array(X, copy=True), block=block)
    if alt is not None:
        assert not w.eotp_step
        rec["fmt_abs"] = float(np.max(np.abs(alt_block_logits(alt, [rec], 0, w).astype(np.float64) - rec["logits"])))
    return rec
