#!/usr/bin/env python3
"""Throughput of the Learn2PD denoising loop on one MI355X.

A "step" is one pass of the whole hot path over the batch: the full bidirectional forward of the
8B-shaped model over prompt + generation window, the fused vocabulary softmax-max / argmax of the
active block, the filter, and the on-device unmask / block-advance / EoTP update.  The timed region
runs exactly K such steps along the real decoding trajectory (the state is re-initialised on device
whenever a generation completes), with weights, prompt and state already resident in HBM.

Prints ONE JSON line.  `value` = generated tokens per second (tokens committed per step on this
trajectory x steps per second); `roofline` is for the dominant kernel (the gate/up SwiGLU GEMM),
timed live with HIP event pairs on the launch stream (no correction: a pair also sees the gap between
the events and the kernel, so the figure is a slight under-estimate of the kernel's rate); `cpu_baseline` is the CPU oracle timed on this
host on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0


def model_label(m):
    """'8B-shaped' for the 32-layer, 4096-wide shape the headline metric is quoted on, else the dimensions."""
    if (m.n_layers, m.d_model, m.d_ffn) == (32, 4096, 12288):
        return "8B-shaped"
    return f"{m.n_layers}-layer d{m.d_model}"


def step_flops(w):
    """Algorithmic flops of one denoising step (full recompute): linear layers on every row,
    bidirectional attention, LM head on the active block's rows only."""
    m = w.model
    rows = w.batch * (w.prompt_len + w.gen_len)
    T = w.prompt_len + w.gen_len
    lin = 2.0 * rows * m.n_layers * (4 * m.d_model * m.d_model + 3 * m.d_model * m.d_ffn)
    attn = 4.0 * w.batch * T * T * m.d_model * m.n_layers
    head = 2.0 * w.batch * w.block_len * m.d_model * m.vocab
    return lin, attn, head


def note(msg):
    """Progress line on stderr (the one JSON line stays alone on stdout)."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def cpu_baseline(w, tokens_per_step, seed, n_layers_sample=2):
    """Times the oracle as it stands on a bounded sample: `n_layers_sample` of the layers plus
    embedding + LM head + decode rule at full width and full sequence length, one sequence."""
    import numpy as np
    import torch
    from oracle import l2pd_oracle as O
    from paper_2509_25188_amd import synth
    from tests import parity as Pz

    m = w.model
    ws = synth.with_layers(w, n_layers_sample)
    t0 = time.time()
    weights = synth.make_weights(ws.model, seed, "cpu")
    ora = Pz.oracle_model(ws.model, weights)
    flt = Pz.np_filter(synth.make_filter(seed, w.block_len, w.filter_hidden))
    prompt = synth.make_prompt(seed, 1, w.prompt_len, w.prompt_hi)[0].numpy()
    gen_s = time.time() - t0
    X = np.concatenate([prompt.astype(np.int64), np.full(w.gen_len, m.mask_id, dtype=np.int64)])
    T = len(X)
    pos = np.arange(T)
    t0 = time.time()
    h = ora.embed(X)
    t_embed = time.time() - t0
    t_layers = 0.0
    for l in range(n_layers_sample):
        t0 = time.time()
        q, k, v = ora.qkv(l, h, pos)
        h = ora.finish_layer(l, h, O.attention(q, k, v))
        t_layers += time.time() - t0
    t0 = time.time()
    logits = ora.head(h[w.prompt_len:w.prompt_len + w.block_len])
    d = O.decide(X[w.prompt_len:w.prompt_len + w.block_len], logits, m.mask_id, flt, w.threshold)
    t_head = time.time() - t0
    per_step = t_embed + t_layers / n_layers_sample * m.n_layers + t_head
    per_step *= w.batch           # the oracle decodes one sequence at a time
    steps_per_s = 1.0 / per_step
    # threads the oracle's matrix products actually ran on: NumPy's BLAS pool
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        blas_threads = None
    return {
        "value": steps_per_s * tokens_per_step, "unit": "tokens/s", "cores": blas_threads or os.cpu_count(),
        "host_cpus": os.cpu_count(), "kind": "oracle", "steps_per_s": steps_per_s,
        "sample": (f"one denoising step of one sequence: embedding + {n_layers_sample} of {m.n_layers} layers "
                   f"+ LM head + decode rule at full width, T={T}, fp32 NumPy; layer time scaled to "
                   f"{m.n_layers} layers and to batch {w.batch} (measured {t_layers + t_embed + t_head:.1f} s of "
                   f"oracle work, {gen_s:.0f} s generating its weights)"),
    }


def cached_workload(args, w, eng, flt, prompt, cfg, f, X0, state0, traj_steps, tokens_total, gen_wall, setup_s):
    """KV-cache workloads (prefix or dual cache, Sec. 4.3): `value` is end-to-end, whole generations
    through l2pd_generate (store rebuilt at every block start, block-only steps in between);
    `ms_per_step` is one block-only step, timed over exactly K calls of l2pd_denoise_step that keep
    the store of the first call; the roofline is the weight stream of such a step (32 or 64 rows per
    sequence: every GEMM is bound by reading its weights once)."""
    import ctypes as C
    import torch
    from paper_2509_25188_amd import binding as Bd
    m = w.model
    lib = Bd.lib()
    stream = torch.cuda.current_stream().cuda_stream
    n_gen = max(1, -(-args.steps // traj_steps))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_gen):
        tok, st, dl = eng.generate(prompt, flt, cfg)
    torch.cuda.synchronize()
    gen_elapsed = time.perf_counter() - t0
    # block-only steps on the store built by the first call (state frozen at block 0: same shapes every call)
    X = X0.clone()
    state = state0.clone()

    def step(keep):
        cfg.keep_kv = keep
        state.copy_(state0)
        rc = lib.l2pd_denoise_step(eng._ctx, X.data_ptr(), w.batch, w.prompt_len, C.byref(cfg), C.byref(f),
                                   state.data_ptr(), None, None, None, None, None, stream)
        if rc:
            raise RuntimeError(f"l2pd_denoise_step: {rc}")

    step(0)
    for _ in range(args.warmup):
        step(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(1)
    torch.cuda.synchronize()
    step_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(4):
        step(0)
    torch.cuda.synchronize()
    refresh_ms = (time.perf_counter() - t0) * 1e3 / 4 - step_ms
    cfg.keep_kv = 0
    weight_bytes = sum(v.numel() * v.element_size() for k_, v in eng.weights.items() if k_ != "tok_emb")
    rows = w.batch * w.block_len
    # one block-only step: the linear layers on the block's rows, attention of those rows over the
    # keys the mode lets them see (the whole window is the upper figure), the LM head on the same rows
    keys = w.prompt_len + w.gen_len
    step_flop = (2.0 * rows * m.n_layers * (4 * m.d_model * m.d_model + 3 * m.d_model * m.d_ffn)
                 + 4.0 * rows * keys * m.d_model * m.n_layers + 2.0 * rows * m.d_model * m.vocab)
    # weights are read once per step whatever the batch: above 2.5e15 / 8e12 = 312 flop per weight byte the
    # matrix cores bound the step, below it the weight stream does
    if step_flop / weight_bytes > PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        tf = step_flop / (step_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": "all kernels of one block-only step (upper figure: every key counted)",
                "achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tf / PEAK_BF16_TFLOPS,
                "traffic": None, "flop_per_step": step_flop}
    else:
        achieved = weight_bytes / (step_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": "all GEMMs of one block-only step (weights read once)",
                "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                "traffic": None, "bytes_per_step": weight_bytes}
    return {
        "metric": f"generated tokens/sec (and denoising steps/sec), {model_label(m)} dLLM, KV-cache decode, "
                  f"bs={w.batch}, 1 MI355X",
        "value": n_gen * tokens_total / gen_elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if m.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "prompt_len": w.prompt_len, "gen_len": w.gen_len,
                   "block_len": w.block_len, "threshold": w.threshold, "eotp": bool(w.eotp),
                   "kv_cache": "dual" if w.dual_cache else "prefix", "layers": m.n_layers, "d_model": m.d_model,
                   "d_ffn": m.d_ffn, "vocab": m.vocab, "rows_per_step": w.batch * w.block_len},
        "steps_per_s": n_gen * traj_steps / gen_elapsed,
        "trajectory": {"generations_timed": n_gen, "steps_per_generation": traj_steps,
                       "tokens_per_generation": tokens_total, "generate_wall_s": gen_elapsed / n_gen,
                       "store_rebuild_ms_per_block": refresh_ms},
        "roofline": roof,
        "setup_s": setup_s,
        **({"eotp_steps_saved": eotp_on_off(w, eng, prompt, flt, cfg, traj_steps, tokens_total)} if w.eotp else {}),
        **({"batch_schedules": batch_schedules(w, eng, prompt, flt, cfg)} if args.batch_schedules else {}),
    }


def pipeline(w, eng, prompt, cfg, seed, dev, n_layers=2):
    """Alg. 1 end to end on the synthetic model: the model's own one-token-per-step answer is the
    reference (Sec. 3.1.2), an EGP rollout labels the confidences, the filter is trained on them
    (AdamW, lr 1e-3, 5,000 epochs as in Sec. 4.1), and the prompt is decoded again with it."""
    import torch
    from paper_2509_25188_amd import binding as Bd
    from paper_2509_25188_amd import synth
    flt = synth.make_filter(seed, w.block_len, w.filter_hidden, dev, n_layers=n_layers)
    vcfg = Bd.Engine.cfg_struct(w.gen_len, w.block_len, 1.0)           # tau = 1: only the forced position goes
    t0 = time.perf_counter()
    ref, st_v, _ = eng.generate(prompt, flt, vcfg)
    torch.cuda.synchronize()
    t_van = time.perf_counter() - t0
    rcfg = Bd.Engine.cfg_struct(w.gen_len, w.block_len, 0.5)
    t0 = time.perf_counter()
    C, Y, steps = eng.egp_rollout(prompt, ref, rcfg)
    torch.cuda.synchronize()
    t_roll = time.perf_counter() - t0
    rows_c = torch.cat([C[b, :int(steps[b])] for b in range(prompt.shape[0])]).contiguous()
    rows_y = torch.cat([Y[b, :int(steps[b])] for b in range(prompt.shape[0])]).contiguous()
    t0 = time.perf_counter()
    losses = Bd.train_filter(flt, rows_c, rows_y, 5000, lr=1e-3)
    torch.cuda.synchronize()
    t_train = time.perf_counter() - t0
    dcfg = Bd.Engine.cfg_struct(w.gen_len, w.block_len, 0.5)
    t0 = time.perf_counter()
    tok, st_f, _ = eng.generate(prompt, flt, dcfg)
    torch.cuda.synchronize()
    t_dec = time.perf_counter() - t0
    return {"vanilla_steps": int(st_v.max()), "vanilla_s": t_van, "egp_steps": int(steps.max()), "egp_rollout_s": t_roll,
            "filter_layers": n_layers, "filter_hidden": w.filter_hidden,
            "filter_params": sum(v.numel() for v in flt.values()),
            "training_rows": int(rows_c.shape[0]), "training_epochs": 5000, "training_s": t_train,
            "bce_first": float(losses[0]), "bce_last": float(losses[-1]),
            "trained_filter_steps": int(st_f.max()), "trained_filter_s": t_dec,
            "trained_filter_tokens_equal_to_reference": float((tok == ref).float().mean())}


def batch_schedules(w, eng, prompt, flt, cfg):
    """Whole generations of one batch under the three batch schedules (lock step, per-sequence block
    pointers, pointers + compaction of the live sequences): same tokens, different number and size
    of forwards."""
    import torch
    from paper_2509_25188_amd import binding as Bd
    out, ref = {}, None
    for name, mode in (("lock_step", Bd.RAGGED_OFF), ("own_blocks", Bd.RAGGED_BLOCKS), ("compact", Bd.RAGGED_COMPACT)):
        cfg.ragged = mode
        eng.generate(prompt, flt, cfg)
        torch.cuda.synchronize()
        note(f"batch schedule {name}: warm-up generation done")
        t0 = time.perf_counter()
        tok, st, dl = eng.generate(prompt, flt, cfg)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ref = tok if ref is None else ref
        n_steps, n_seq_steps = eng.generate_stats()
        note(f"batch schedule {name}: {dt:.1f} s, {n_steps} step launches, {n_seq_steps} sequence-steps")
        out[name] = {"generate_wall_s": dt, "tokens_per_s": int(dl.sum()) / dt,
                     "step_launches": n_steps, "sequence_steps": n_seq_steps,
                     "steps_per_sequence": st.cpu().tolist(), "tokens_equal_lock_step": bool(torch.equal(tok, ref))}
    cfg.ragged = Bd.RAGGED_OFF
    return out


def eotp_on_off(w, eng, prompt, flt, cfg, steps_on, tokens_on):
    """The same decode with End-of-Text Prediction switched off (every block of the window is decoded):
    steps and wall time against the EoTP run (Sec. 3.3; App. B counts the cost of the padding the same way)."""
    import torch
    from paper_2509_25188_amd import binding as Bd
    off = Bd.DecodeCfg.from_buffer_copy(cfg)
    off.eotp = Bd.EOTP_OFF
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tok, st, dl = eng.generate(prompt, flt, off)
    torch.cuda.synchronize()
    t_off = time.perf_counter() - t0
    note(f"EoTP off: {t_off:.1f} s")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.generate(prompt, flt, cfg)
    torch.cuda.synchronize()
    t_on = time.perf_counter() - t0
    steps_off = int(st.max())
    return {"steps_eotp_on": int(steps_on), "steps_eotp_off": steps_off,
            "steps_saved_fraction": 1.0 - steps_on / steps_off, "generate_wall_s_eotp_on": t_on,
            "generate_wall_s_eotp_off": t_off, "wall_time_ratio_off_over_on": t_off / t_on,
            "tokens_decoded_eotp_on": int(tokens_on), "tokens_decoded_eotp_off": int(dl.sum().item())}


TRAFFIC_WORKLOAD = "8b_g256"      # the workload the committed counter runs were taken on
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gate_up_gemm_hbm_traffic.txt")
GEMM_SOURCE = os.path.join(ROOT, "paper_2509_25188_amd", "csrc", "gemm_bf16.hip")


def measured_traffic():
    """HBM bytes per launch of the gate/up GEMM from the committed counter summary, or None when
    there is none or the kernel source has changed since the counters were taken."""
    import hashlib
    try:
        fields = {}
        with open(TRAFFIC_FILE) as fh:
            for line in fh:
                if ":" in line and not line.startswith("#"):
                    k, v = line.split(":", 1)
                    fields[k.strip()] = v.strip()
        with open(GEMM_SOURCE, "rb") as fh:
            sha = hashlib.sha256(fh.read()).hexdigest()
        if fields.get("kernel_source_sha256") != sha:
            return None
        return float(fields["hbm_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=96)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="8b_g256")
    ap.add_argument("--layers", type=int, default=0, help="reduced depth (debugging only; invalid as a result)")
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--decoder", default="learn2pd", choices=["learn2pd", "vanilla", "threshold"],
                    help="learn2pd: the workload's filter and threshold; vanilla: one token per step (the most "
                         "confident masked position); threshold: unmask where the confidence exceeds --conf-threshold")
    ap.add_argument("--conf-threshold", type=float, default=0.9)
    ap.add_argument("--lm-head-scale", type=float, default=1.0,
                    help="scales the synthetic LM head; 25 spreads the confidences over (0, 1) (not the headline config)")
    ap.add_argument("--pipeline", action="store_true",
                    help="also run the whole Learn2PD pipeline on the synthetic model: vanilla answer as reference, "
                         "EGP rollout, filter training, decode with the trained filter (adds a 'pipeline' object)")
    ap.add_argument("--filter-layers", type=int, default=2,
                    help="depth of the filter MLP (2 = the paper's; 1 and 4 are the variants of Table 3)")
    ap.add_argument("--filter-hidden", type=int, default=0, help="hidden width of the filter (0: the workload's)")
    ap.add_argument("--batch-schedules", action="store_true",
                    help="also time whole generations of the batch in lock step, with per-sequence block "
                         "pointers, and with batch compaction")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain device copy of known size (reference for HBM counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_25188_amd import binding as Bd
    from paper_2509_25188_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    if args.layers:
        w = synth.with_layers(w, args.layers)
    import dataclasses
    if args.filter_hidden:
        w = dataclasses.replace(w, filter_hidden=args.filter_hidden)
    m = w.model
    dev = "cuda"
    t0 = time.time()
    eng = Bd.engine_for(w, args.seed, dev, lm_head_scale=args.lm_head_scale)
    flt = synth.make_filter(args.seed, w.block_len, w.filter_hidden, dev, n_layers=args.filter_layers)
    if args.decoder == "vanilla":          # the filter never passes: only the forced most confident position goes
        w = dataclasses.replace(w, threshold=1.0)
    elif args.decoder == "threshold":
        flt = synth.threshold_filter(w.block_len, args.conf_threshold, device=dev)
        w = dataclasses.replace(w, threshold=0.5, filter_hidden=w.block_len)
    prompt = synth.make_prompt(args.seed, w.batch, w.prompt_len, w.prompt_hi, dev)
    bias = (m.eos_id, w.bias_from, w.bias_value) if w.bias_value else None
    cfg = Bd.Engine.cfg_struct(w.gen_len, w.block_len, w.threshold, Bd.EOTP_STEP if w.eotp_step else w.eotp,
                               w.prefix_cache, bias, w.dual_cache)
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    note(f"weights and engine ready in {setup_s:.1f} s")

    # The real trajectory once (also a warm-up): total steps and tokens of one generation.
    t0 = time.time()
    tok, st, dl = eng.generate(prompt, flt, cfg)
    torch.cuda.synchronize()
    gen_wall = time.time() - t0
    t0 = time.time()
    tok, st, dl = eng.generate(prompt, flt, cfg)
    torch.cuda.synchronize()
    gen_wall = time.time() - t0
    note(f"two generations done ({gen_wall:.1f} s each); timing steps")
    steps_per_seq = st.cpu().tolist()
    traj_steps = max(steps_per_seq)                 # lock-step batch: forwards of one generation
    tokens_total = int(dl.sum().item())
    tokens_per_step = tokens_total / traj_steps

    # K steps along that trajectory through l2pd_denoise_step; state reset on device at wrap-around.
    T = w.prompt_len + w.gen_len
    X0 = torch.cat([prompt, torch.full((w.batch, w.gen_len), m.mask_id, dtype=torch.int32, device=dev)], 1)
    X = X0.clone()
    state0 = torch.zeros((w.batch, 3), dtype=torch.int32, device=dev)
    state = state0.clone()
    f = eng.filter_struct(flt)
    import ctypes as C
    lib = Bd.lib()
    stream = torch.cuda.current_stream().cuda_stream

    def run(n, k0):
        for k in range(k0, k0 + n):
            if k % traj_steps == 0:
                X.copy_(X0)
                state.copy_(state0)
            rc = lib.l2pd_denoise_step(eng._ctx, X.data_ptr(), w.batch, w.prompt_len, C.byref(cfg), C.byref(f),
                                       state.data_ptr(), None, None, None, None, None, stream)
            if rc:
                raise RuntimeError(f"l2pd_denoise_step: {rc}")
        return k0 + n

    if w.prefix_cache or w.dual_cache:
        print(json.dumps(cached_workload(args, w, eng, flt, prompt, cfg, f, X0, state0, traj_steps, tokens_total,
                                         gen_wall, setup_s)))
        return
    k = run(args.warmup, 0)
    torch.cuda.synchronize()
    eng.profile_select(Bd.K_GEMM_GATEUP)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, k)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    n_launch, kern_ms = eng.profile_read()
    eng.profile_select(Bd.K_NONE)

    ms_per_step = elapsed * 1e3 / args.steps
    steps_per_s = args.steps / elapsed
    lin, attn, head = step_flops(w)
    total_flops = lin + attn + head
    rows = w.batch * T
    gu_flops = 2.0 * rows * m.d_model * 2 * m.d_ffn
    avg_kern_ms = kern_ms / max(n_launch, 1)
    achieved = gu_flops / (avg_kern_ms * 1e-3) / 1e12 if n_launch else None
    result = {
        "metric": f"generated tokens/sec (and denoising steps/sec), {model_label(m)} dLLM, bs={w.batch}, 1 MI355X",
        "value": tokens_per_step * steps_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if m.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "prompt_len": w.prompt_len, "gen_len": w.gen_len,
                   "block_len": w.block_len, "threshold": w.threshold,
                   "eotp": "step" if w.eotp_step else bool(w.eotp), "decoder": args.decoder,
                   "filter_layers": args.filter_layers, "filter_hidden": w.filter_hidden,
                   "lm_head_scale": args.lm_head_scale, "layers": m.n_layers, "d_model": m.d_model, "d_ffn": m.d_ffn,
                   "vocab": m.vocab, "full_recompute_rows": rows},
        "steps_per_s": steps_per_s,
        "trajectory": {"steps_per_generation": traj_steps, "tokens_per_generation": tokens_total,
                       "tokens_per_step": tokens_per_step, "generate_wall_s": gen_wall,
                       "generate_tokens_per_s": tokens_total / gen_wall},
        "step_tflop": total_flops / 1e12,
        "step_mfma_frac": total_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "step_weight_stream_gbs": (sum(v.numel() * v.element_size() for k_, v in eng.weights.items()
                                       if k_ != "tok_emb") / 1e9) / (ms_per_step * 1e-3),
        "roofline": {"bound": "mfma", "kernel": "k_gemm_bf16<SwiGLU gate/up>", "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": (achieved / PEAK_BF16_TFLOPS) if achieved else None, "traffic": measured_traffic() if w.name == TRAFFIC_WORKLOAD else None,
                     "launches": n_launch, "avg_launch_ms": avg_kern_ms, "flop_per_launch": gu_flops},
        "setup_s": setup_s,
    }
    if w.eotp and not w.eotp_step:
        result["eotp_steps_saved"] = eotp_on_off(w, eng, prompt, flt, cfg, traj_steps, tokens_total)
    if args.pipeline:
        result["pipeline"] = pipeline(w, eng, prompt, cfg, args.seed, dev, args.filter_layers)
    if args.batch_schedules:
        result["batch_schedules"] = batch_schedules(w, eng, prompt, flt, cfg)
    if args.copy_calibration:
        n = 1 << 28
        src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["copy_calibration"] = {"bytes_read_per_launch": n, "bytes_written_per_launch": n, "launches": 4}
    if not args.no_cpu_baseline:
        note("GPU legs done; timing the CPU oracle on a bounded sample")
        result["cpu_baseline"] = cpu_baseline(w, tokens_per_step, args.seed, n_layers_sample=min(m.n_layers, 32))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
