#!/usr/bin/env python3
"""Writes the stored oracle trajectories under tests/golden/ (one .npz per case).

Calls only the CPU oracle (oracle/l2pd_oracle.py) and the seeded input generator; nothing here
touches the HIP library or a GPU.  Each file holds, for one sequence of one named workload decoded
by the oracle (Alg. 2; Alg. 3 where the workload has End-of-Text Prediction; Sec. 4.3's prefix cache
where it has one), the state before every step and what the step computed, so that a GPU test can
impose every state on l2pd_denoise_step and compare (teacher forcing), and compare l2pd_generate's
tokens, step count and decoded length with the oracle's.

    python tests/golden/make_trajectories.py <case> [<case> ...]      (see CASES; "all-quick" = the cheap ones)
    python tests/golden/make_trajectories.py --fill-floor <case> ...  (float64 distance at every sampled step)

Oracle used: bf16 models are evaluated with every matrix-product input rounded to bf16 and float32
accumulation (the arithmetic of the path under test); at sampled steps (first and last step of every
block, plus every `every`-th step) two more evaluations of the same state are stored as distances:
  fmt_abs    max |logit difference| to the oracle with float32 activations (no bf16 rounding of
             activations): the error of the number format, which bounds what any bf16 path can resolve;
  floor_abs  max |logit difference| to the same bf16-input oracle accumulated in float64: the noise floor
             (roundings flipped by accumulation order), computed where `floor` says so.
Weights are widened from bf16 to float32 once per case (exact), instead of once per call.

Stored per file (n steps, block length s, m sampled steps, T = prompt + generation length):
  meta (JSON), prompt [P], tokens [G], steps, decoded_len,
  X_before [n, T], block [n], conf / p [n, s] f32, pre [n, s] i32, sel / masked [n, s] u8,
  absmax [n] (largest |logit| of the block's rows), gap [n, s] (best minus second-best logit over the
  data vocabulary), smp_idx [m], cols_fixed [C], lg_fixed [m, s, C], cols_top [m, s, 8], lg_top [m, s, 8],
  fmt_abs [m], floor_abs [m] (NaN where not computed).
Cases named *_eotp_off hold only the result of the same decode with EoTP off (tokens, steps).
Cases named *_states_from_* take their states from another case's file (the oracle's trajectory of the
same workload at reduced depth) and evaluate them at this case's depth: first and last step of every block.
"""
from __future__ import annotations

import dataclasses
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import l2pd_oracle as O                      # noqa: E402
from paper_2509_25188_amd import synth                   # noqa: E402  (seeded inputs only)

SEED = 1234
COL_STRIDE = 251          # fixed sampled logit columns: every 251st token id
N_TOP = 8                 # plus the oracle's eight largest logits of every row


@dataclasses.dataclass(frozen=True)
class Case:
    workload: str
    layers: int            # 0 = the workload's own depth
    seqs: tuple            # sequences of the workload's batch to decode (each alone, B = 1)
    every: int = 8         # sampled steps besides block boundaries; 0 = boundaries only
    floor: str = "sampled"  # "sampled": float64 evaluation at every sampled step; "few": at every sixth of them
    eotp_off: bool = False  # store only the result of the decode with EoTP switched off
    states_from: str = ""   # take states from this case's files instead of decoding


CASES = {
    # config 2: full depth (8 layers), two of the eight sequences
    "mid": Case("mid", 0, (0, 5)),
    # configs 3, 4, 5 at two layers, real widths and vocabulary, whole trajectory
    "8b_g256_L2": Case("8b_g256", 2, (0,), floor="few"),
    "8b_g1024_eotp_L2": Case("8b_g1024_eotp", 2, (0,), every=16, floor="few"),
    "8b_g1024_eotp_L2_eotp_off": Case("8b_g1024_eotp", 2, (0,), eotp_off=True),
    "8b_b32_prefix_L2": Case("8b_b32_prefix", 2, (0, 17), every=16, floor="few"),
    # config 3 at its real depth: the oracle's whole trajectory (hours of CPU)
    "8b_g256_full": Case("8b_g256", 0, (0,), every=0, floor="few"),
    # config 4 / 5 at their real depth: states of the two-layer trajectories, first and last step of every block
    "8b_g1024_eotp_full_states_from_L2": Case("8b_g1024_eotp", 0, (0,), every=0, floor="few",
                                              states_from="8b_g1024_eotp_L2"),
    "8b_b32_prefix_full_states_from_L2": Case("8b_b32_prefix", 0, (0,), every=0, floor="few",
                                              states_from="8b_b32_prefix_L2"),
}
QUICK = ("mid", "8b_g256_L2", "8b_b32_prefix_L2")


def path_of(case: str, seq: int) -> str:
    return os.path.join(HERE, f"traj_{case}_seq{seq}.npz")


def shape_ns(m: synth.ModelShape):
    import types
    return types.SimpleNamespace(**{k: getattr(m, k) for k in
                                    ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab", "mask_id",
                                     "eos_id", "rope_base", "rms_eps")})


def widened_weights(m: synth.ModelShape):
    """name -> float32 array (exact widening of the bf16 draws); the embedding stays as bit patterns
    (the oracle widens the gathered rows only)."""
    out = {}
    for name, shape, kind in synth.weight_specs(m):
        t = synth.to_numpy(synth.make_tensor(m, SEED, name, shape, kind, "cpu"))
        out[name] = t if name == "tok_emb" else O.widen(t, np.float32)
    return out


class LazyBits:
    """name -> the same weight as bf16 bit patterns, drawn again on every access (for the float64
    evaluation, which widens per call: nothing of the 16 GB model stays resident twice)."""

    def __init__(self, m: synth.ModelShape):
        self.m = m
        self.specs = {name: (shape, kind) for name, shape, kind in synth.weight_specs(m)}

    def __getitem__(self, name):
        shape, kind = self.specs[name]
        return synth.to_numpy(synth.make_tensor(self.m, SEED, name, shape, kind, "cpu"))


class Oracles:
    """The primary oracle and the two comparison evaluations of one model."""

    def __init__(self, w: synth.Workload, need_f64: bool):
        t0 = time.time()
        self.w = w
        ns = shape_ns(w.model)
        wide = widened_weights(w.model)
        self.main = O.Model(ns, wide, np.float32, "bf16")
        self.fp32act = O.Model(ns, wide, np.float32, "fp32")
        self.f64 = O.Model(ns, LazyBits(w.model), np.float64, "bf16") if need_f64 else None
        print(f"  weights ready in {time.time() - t0:.0f} s", flush=True)

    def block_logits(self, model, X_before, block, cache_store):
        """Biased logits of the active block from state X_before under `model` (full recompute or prefix cache)."""
        w = self.w
        lo = w.prompt_len + block * w.block_len
        if w.prefix_cache:
            key = (id(model), block)
            if key not in cache_store:
                cache_store.clear()
                cache_store[key] = model.prefix_kv(X_before[:lo])
            lg = model.forward_block_cached(cache_store[key], X_before[lo:lo + w.block_len], lo)
        else:
            lg = model.forward(X_before, lo, w.block_len)
        bias = (w.model.eos_id, w.bias_from, w.bias_value) if w.bias_value else None
        return O.apply_bias(lg, block * w.block_len, bias)


def top2_gap(logits, mask_id):
    z = np.array(logits, dtype=np.float64, copy=True)
    z[:, mask_id] = -np.inf
    part = np.partition(z, -2, axis=-1)
    return (part[:, -1] - part[:, -2]).astype(np.float32)


class Recorder(list):
    """Receives the oracle's per-step records, keeps the small arrays, and at sampled steps the
    sampled logits and the distances to the two comparison evaluations."""

    def __init__(self, ora: Oracles, case: Case, n_blocks: int):
        super().__init__()
        self.ora, self.case = ora, case
        m = ora.w.model
        self.cols_fixed = np.arange(0, m.vocab, COL_STRIDE, dtype=np.int64)
        self.rows = {k: [] for k in ("X_before", "block", "conf", "pre", "p", "sel", "masked", "absmax", "gap")}
        self.smp = {k: [] for k in ("smp_idx", "lg_fixed", "cols_top", "lg_top", "fmt_abs", "floor_abs")}
        self.caches = {"fp32act": {}, "f64": {}}
        self.n_blocks = n_blocks
        self.t0 = time.time()

    def append(self, d, force=False):
        i = len(self.rows["block"])
        lg = d["logits"]
        r = self.rows
        r["X_before"].append(np.asarray(d["X_before"], dtype=np.int32))
        r["block"].append(int(d["block"]))
        r["conf"].append(np.asarray(d["conf"], dtype=np.float32))
        r["pre"].append(np.asarray(d["pre"], dtype=np.int32))
        r["p"].append(np.asarray(d["p"], dtype=np.float32))
        r["sel"].append(np.asarray(d["sel"], dtype=np.uint8))
        r["masked"].append(np.asarray(d["masked"], dtype=np.uint8))
        r["absmax"].append(np.float32(np.max(np.abs(lg))))
        r["gap"].append(top2_gap(lg, self.ora.w.model.mask_id))
        first = i == 0 or r["block"][i - 1] != r["block"][i]
        last = not np.any(d["masked"] & ~d["sel"])
        if force or first or last or (self.case.every and i % self.case.every == 0):
            self.sample(i, d)
        if i % 16 == 0:
            print(f"    step {i} block {d['block']} ({time.time() - self.t0:.0f} s)", flush=True)

    def sample(self, i, d):
        lg = d["logits"]
        s = self.smp
        s["smp_idx"].append(i)
        s["lg_fixed"].append(np.asarray(lg[:, self.cols_fixed], dtype=np.float32))
        z = np.array(lg, copy=True)
        z[:, self.ora.w.model.mask_id] = -np.inf
        top = np.argsort(-z, axis=-1, kind="stable")[:, :N_TOP]
        s["cols_top"].append(top.astype(np.int32))
        s["lg_top"].append(np.take_along_axis(np.asarray(lg, dtype=np.float32), top, axis=-1))
        l2 = self.ora.block_logits(self.ora.fp32act, d["X_before"], d["block"], self.caches["fp32act"])
        s["fmt_abs"].append(np.float32(np.max(np.abs(l2.astype(np.float64) - lg))))
        # "few": the float64 evaluation at every sixth sampled step only (it takes minutes at the real depth)
        want64 = self.ora.f64 is not None and (self.case.floor == "sampled" or (len(s["smp_idx"]) - 1) % 6 == 0)
        if want64:
            l3 = self.ora.block_logits(self.ora.f64, d["X_before"], d["block"], self.caches["f64"])
            s["floor_abs"].append(np.float32(np.max(np.abs(l3 - lg.astype(np.float64)))))
        else:
            s["floor_abs"].append(np.float32(np.nan))

    def arrays(self):
        out = {k: np.stack(v) if k not in ("block", "absmax") else np.asarray(v) for k, v in self.rows.items()}
        out["block"] = out["block"].astype(np.int32)
        out["cols_fixed"] = self.cols_fixed.astype(np.int32)
        for k, v in self.smp.items():
            out[k] = np.stack(v) if k in ("lg_fixed", "cols_top", "lg_top") else np.asarray(v)
        out["smp_idx"] = out["smp_idx"].astype(np.int32)
        return out


def decode(ora: Oracles, prompt, flt, trace, eotp=None):
    w = ora.w
    bias = (w.model.eos_id, w.bias_from, w.bias_value) if w.bias_value else None
    return O.generate(ora.main, prompt, w.gen_len, w.block_len, w.model.mask_id, w.model.eos_id, flt, w.threshold,
                      eotp=w.eotp if eotp is None else eotp, bias=bias, prefix_cache=w.prefix_cache, trace=trace)


def run_case(name: str):
    case = CASES[name]
    w = synth.WORKLOADS[case.workload]
    if case.layers:
        w = synth.with_layers(w, case.layers)
    print(f"{name}: workload {w.name}, {w.model.n_layers} layers, sequences {case.seqs}", flush=True)
    flt = {k: v.numpy() for k, v in synth.make_filter(SEED, w.block_len, w.filter_hidden).items()}
    prompts = synth.make_prompt(SEED, max(w.batch, max(case.seqs) + 1), w.prompt_len, w.prompt_hi).numpy()
    ora = Oracles(w, need_f64=not case.eotp_off)
    n_blocks = w.gen_len // w.block_len
    for b in case.seqs:
        t0 = time.time()
        prompt = prompts[b].astype(np.int64)
        meta = dict(case=name, workload=case.workload, layers=w.model.n_layers, seq=b, seed=SEED,
                    threshold=w.threshold, block_len=w.block_len, gen_len=w.gen_len, prompt_len=w.prompt_len,
                    eotp=bool(w.eotp), prefix_cache=bool(w.prefix_cache), col_stride=COL_STRIDE,
                    oracle="bf16-rounded matrix-product inputs, float32 accumulation")
        if case.eotp_off:
            tokens, steps, dlen = decode(ora, prompt, flt, None, eotp=False)
            meta["eotp"] = False
            np.savez_compressed(path_of(name, b), meta=json.dumps(meta), prompt=prompt.astype(np.int32),
                                tokens=tokens.astype(np.int32), steps=np.int32(steps), decoded_len=np.int32(dlen))
        elif case.states_from:
            src = np.load(path_of(case.states_from, b))
            rec = Recorder(ora, case, n_blocks)
            blocks = src["block"]
            cache = {}
            for i in range(len(blocks)):
                first = i == 0 or blocks[i - 1] != blocks[i]
                last = i + 1 == len(blocks) or blocks[i + 1] != blocks[i]
                if not (first or last):
                    continue
                X = src["X_before"][i].astype(np.int64)
                lg = ora.block_logits(ora.main, X, int(blocks[i]), cache)
                lo = w.prompt_len + int(blocks[i]) * w.block_len
                d = O.decide(X[lo:lo + w.block_len], lg, w.model.mask_id, flt, w.threshold)
                d.update(logits=lg, X_before=X, block=int(blocks[i]))
                rec.append(d, force=True)
            meta["states_from"] = case.states_from
            meta["source_steps"] = [int(i) for i in range(len(blocks))
                                    if i == 0 or blocks[i - 1] != blocks[i] or i + 1 == len(blocks) or blocks[i + 1] != blocks[i]]
            np.savez_compressed(path_of(name, b), meta=json.dumps(meta), prompt=prompt.astype(np.int32), **rec.arrays())
        else:
            rec = Recorder(ora, case, n_blocks)
            tokens, steps, dlen = decode(ora, prompt, flt, rec)
            np.savez_compressed(path_of(name, b), meta=json.dumps(meta), prompt=prompt.astype(np.int32),
                                tokens=tokens.astype(np.int32), steps=np.int32(steps), decoded_len=np.int32(dlen),
                                **rec.arrays())
        print(f"  sequence {b}: written {path_of(name, b)} in {time.time() - t0:.0f} s", flush=True)


def fill_floor(name: str):
    """Computes the float64 distance (floor_abs) at every sampled step of an existing file that does not have
    it yet (the "few" cases store it at every sixth sampled step only) and rewrites the file."""
    case = CASES[name]
    w = synth.WORKLOADS[case.workload]
    if case.layers:
        w = synth.with_layers(w, case.layers)
    ora = Oracles(w, need_f64=True)
    for b in case.seqs:
        z = dict(np.load(path_of(name, b)))
        floor = z["floor_abs"].copy()
        caches = {"main": {}, "f64": {}}
        for k, i in enumerate(z["smp_idx"]):
            if np.isfinite(floor[k]):
                continue
            t0 = time.time()
            X, blk = z["X_before"][i].astype(np.int64), int(z["block"][i])
            lg = ora.block_logits(ora.main, X, blk, caches["main"])
            # the stored step again (BLAS may block differently with another thread count: equal up to that)
            np.testing.assert_allclose(lg[:, z["cols_fixed"]], z["lg_fixed"][k], rtol=0, atol=5e-2 * float(z["floor_abs"][0]))
            l3 = ora.block_logits(ora.f64, X, blk, caches["f64"])
            floor[k] = np.float32(np.max(np.abs(l3 - lg.astype(np.float64))))
            z["floor_abs"] = floor
            tmp = path_of(name, b) + ".tmp.npz"          # replace atomically: a kill must not leave half a file
            np.savez_compressed(tmp, **z)
            os.replace(tmp, path_of(name, b))
            print(f"  {name} seq {b}: sampled step {i}: floor {floor[k]:.4e} ({time.time() - t0:.0f} s)", flush=True)


if __name__ == "__main__":
    if len(sys.argv) > 2 and sys.argv[1] == "--fill-floor":
        for n in sys.argv[2:]:
            fill_floor(n)
        sys.exit(0)
    names = sys.argv[1:]
    if not names:
        print(__doc__)
        print("cases:", ", ".join(CASES))
        sys.exit(1)
    if names == ["all-quick"]:
        names = list(QUICK)
    for n in names:
        run_case(n)
