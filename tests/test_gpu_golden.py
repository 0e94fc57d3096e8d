"""GPU parity against the stored oracle trajectories of the named workloads (tests/golden/traj_*.npz,
written by tests/golden/make_trajectories.py from the CPU oracle alone).

Every stored step is imposed on l2pd_denoise_step (teacher forcing) and compared under the fixed rules of
tests/parity.py; then l2pd_generate decodes the same prompt freely and its tokens, step count and decoded
length are compared with the oracle's (identical when no position of the trajectory is exempt, else
identical up to the first exempt step, and reported)."""
import dataclasses
import os

import numpy as np
import pytest
import torch

from paper_2509_25188_amd import binding as Bd
from paper_2509_25188_amd import synth
from tests import parity as Pz

pytestmark = pytest.mark.gpu
SEED = 1234
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def path_of(case, seq):
    return os.path.join(GOLDEN, f"traj_{case}_seq{seq}.npz")


def engine(w, max_batch):
    eng = Bd.engine_for(w, SEED, "cuda", max_batch=max_batch)
    flt = synth.make_filter(SEED, w.block_len, w.filter_hidden, "cuda")
    return eng, flt


def forced_and_free(case, w, seqs, eng, flt, exempt_frac, batch_rows=None):
    """Teacher-forces every stored step of the sequences `seqs`, then compares a free-running decode.
    batch_rows: decode the workload's whole batch in one call and compare these rows (else one call per
    sequence at B = 1).  Returns the report."""
    cfg = Pz.cfg_for(w)
    prompts = synth.make_prompt(SEED, max(w.batch, max(seqs) + 1), w.prompt_len, w.prompt_hi, "cuda")
    rep = Pz.StepReport()
    loaded = {}
    for b in seqs:
        meta, recs, result = Pz.load_trajectory(path_of(case, b))
        assert meta["workload"] == (w.name.split("_L")[0]) and meta["layers"] == w.model.n_layers and meta["seq"] == b
        np.testing.assert_array_equal(np.load(path_of(case, b))["prompt"], prompts[b].cpu().numpy())
        # logits: the stated tolerance, or 2 x the stored noise floor where that is larger (the floor is the distance
        # of one float32 summation order, the oracle's, from exact accumulation; the HIP path is another order, so
        # floor + floor bounds their distance by the triangle inequality; deep random-init
        # models: the same oracle accumulated in float64 instead of float32 already moves the logits that far)
        lim = max(Pz.tol_for(w.model), 2.0 * meta["floor_rel_max"])
        for r in recs:
            r["logit_tol"] = lim
        forced = Pz.teacher_forced(eng, [recs], w.prompt_len, cfg, flt, w.model, w.threshold, rep,
                                   want_logits=lambda r: "lg_fixed" in r)
        loaded[b] = (recs, result, forced.first_exempt[0])
        print(f"{case} seq {b}: {len(recs)} stored steps, D = {meta['fmt_abs_max']:.3e} logit units, noise floor "
              f"{meta['floor_rel_max']:.3e}, logit tolerance {lim:.3e}, first exempt step {forced.first_exempt[0]}")
    print(f"{case} teacher-forced:", rep)
    assert rep.exempt_tokens + rep.exempt_decisions <= exempt_frac * rep.positions, rep
    if batch_rows is not None:
        tok, st, dl = eng.generate(prompts[:w.batch].contiguous(), flt, cfg)
        tok, st, dl = tok.cpu().numpy(), st.cpu().numpy(), dl.cpu().numpy()
        rows = {b: (tok[b], st[b], dl[b]) for b in batch_rows}
    else:
        rows = {}
        for b in seqs:
            tok, st, dl = eng.generate(prompts[b:b + 1].contiguous(), flt, cfg)
            rows[b] = (tok.cpu().numpy()[0], int(st[0]), int(dl[0]))
    for b in seqs:
        recs, result, first_exempt = loaded[b]
        if result is None:
            continue
        Pz.check_generate(rows[b][0], rows[b][1], rows[b][2], recs, *result, first_exempt, w.prompt_len,
                          w.block_len, f"{case} seq {b}")
    return rep, rows, loaded


def test_mid_workload_full_depth_trajectories():
    # the mid-size workload at its own depth (8 layers): sequences 0 and 5 of the batch of 8, every step of the
    # oracle's trajectories teacher-forced, then the whole batch decoded in one call
    w = synth.WORKLOADS["mid"]
    eng, flt = engine(w, w.batch)
    rep, rows, _ = forced_and_free("mid", w, (0, 5), eng, flt, exempt_frac=0.05, batch_rows=(0, 5))   # measured 3.3 % of the positions
    assert rep.max_logit_err < 2e-2


def test_8b_g256_two_layers_whole_trajectory():
    # the benchmarked workload's widths, vocabulary and decode arguments at two layers: every step of the
    # oracle's trajectory teacher-forced (512 rows, full recompute), then a free-running decode
    w = synth.with_layers(synth.WORKLOADS["8b_g256"], 2)
    eng, flt = engine(w, 1)
    rep, rows, _ = forced_and_free("8b_g256_L2", w, (0,), eng, flt, exempt_frac=0.05)
    assert rep.max_logit_err < 2e-2


def test_8b_b32_prefix_two_layers_trajectories_and_batch_of_32():
    # block 64, prefix cache, EoTP with the end-of-text bias from generation position 400: sequences 0 and 17
    # of the batch, each teacher-forced along its own stored trajectory and decoded alone; then the whole
    # batch of 32 DIFFERENT prompts in one call, rows 0 and 17 against the same stored results (a batched
    # block-only step has 2048 rows and takes other GEMM tiles and split depths than the 64-row step of a
    # single sequence, so the rows agree to rounding, not bit for bit: compared under the exemption rules)
    w = synth.with_layers(synth.WORKLOADS["8b_b32_prefix"], 2)
    eng, flt = engine(w, w.batch)
    rep, rows, loaded = forced_and_free("8b_b32_prefix_L2", w, (0, 17), eng, flt, exempt_frac=0.05)
    assert rep.max_logit_err < 2e-2
    cfg = Pz.cfg_for(w)
    prompts = synth.make_prompt(SEED, w.batch, w.prompt_len, w.prompt_hi, "cuda")
    assert len({tuple(r) for r in prompts.cpu().numpy().tolist()}) == w.batch          # 32 different prompts
    tok, st, dl = eng.generate(prompts, flt, cfg)
    tok, st, dl = tok.cpu().numpy(), st.cpu().numpy(), dl.cpu().numpy()
    stop = (w.bias_from // w.block_len + 1) * w.block_len
    # Alg. 3 for every row: decoding stops after the first block that holds an end-of-text token, which the bias
    # forces in the block of generation position 400; an untrained model may also pick the token by itself in an
    # earlier block (one chance in 126,464 per position), and then that block is the last
    for b in range(w.batch):
        n = int(dl[b])
        assert n % w.block_len == 0 and 0 < n <= stop
        assert not np.any(tok[b, :n] == w.model.mask_id) and np.all(tok[b, n:] == w.model.mask_id)
        assert np.any(tok[b, n - w.block_len:n] == w.model.eos_id) and not np.any(tok[b, :n - w.block_len] == w.model.eos_id)
    assert np.sum(dl == stop) >= w.batch - 2
    assert len(set(st.tolist())) > 1                                                    # sequences in different states
    for b in (0, 17):
        recs, result, first_exempt = loaded[b]
        Pz.check_generate(tok[b], st[b], dl[b], recs, *result, first_exempt, w.prompt_len, w.block_len,
                          f"8b_b32_prefix_L2 batch of 32, row {b}")


def have(case, seq=0):
    return os.path.exists(path_of(case, seq))


def needs(*cases):
    missing = [c for c in cases if not have(c)]
    return pytest.mark.skipif(bool(missing), reason=f"stored trajectory not generated: {missing} "
                                                    "(python tests/golden/make_trajectories.py <case>; hours of CPU)")


@needs("8b_g1024_eotp_L2")
def test_8b_g1024_eotp_two_layers_whole_trajectory_and_steps_saved():
    # generation length 1024 with EoTP (Alg. 3), the end-of-text bias from generation position 400, 1280 rows of
    # full recompute: every stored step teacher-forced, then the free-running decode; then the same decode with
    # EoTP off against the stored EoTP-off result: the steps EoTP saves (Sec. 3.3)
    w = synth.with_layers(synth.WORKLOADS["8b_g1024_eotp"], 2)
    eng, flt = engine(w, 1)
    rep, rows, loaded = forced_and_free("8b_g1024_eotp_L2", w, (0,), eng, flt, exempt_frac=0.05)
    assert rep.max_logit_err < 2e-2
    tok_on, st_on, dl_on = rows[0]
    recs, (o_tok, o_steps, o_dlen), first_exempt = loaded[0]
    stop = (w.bias_from // w.block_len + 1) * w.block_len
    assert dl_on == o_dlen == stop and np.all(tok_on[stop:] == w.model.mask_id)
    if not have("8b_g1024_eotp_L2_eotp_off"):
        pytest.skip("EoTP-off companion not generated")
    meta, _, (f_tok, f_steps, f_dlen) = Pz.load_trajectory(path_of("8b_g1024_eotp_L2_eotp_off", 0))
    cfg_off = Pz.cfg_for(dataclasses.replace(w, eotp=False))
    prompt = synth.make_prompt(SEED, 1, w.prompt_len, w.prompt_hi, "cuda")
    tok, st, dl = eng.generate(prompt, flt, cfg_off)
    tok, st, dl = tok.cpu().numpy()[0], int(st[0]), int(dl[0])
    assert dl == f_dlen == w.gen_len and not np.any(tok == w.model.mask_id)
    np.testing.assert_array_equal(f_tok[:stop], o_tok[:stop])          # the oracle's two runs coincide up to the stop
    np.testing.assert_array_equal(tok[:stop], tok_on[:stop])           # and so do the library's
    print(f"EoTP on: {st_on} steps (oracle {o_steps}); off: {st} steps (oracle {f_steps}); saved {st - st_on} "
          f"(oracle {f_steps - o_steps}) = {100.0 * (st - st_on) / st:.1f} % of the steps")
    assert st > st_on and f_steps > o_steps
    if first_exempt is None and np.array_equal(tok, f_tok):
        assert st == f_steps
    else:
        # a near-tie somewhere flips a decision and the later blocks differ; the count of steps stays close
        assert abs(st - f_steps) <= 0.1 * f_steps


@needs("8b_g256_full")
def test_8b_g256_full_depth_whole_trajectory():
    # the benchmarked workload itself: 32 layers, 512 rows, every step of the oracle's whole trajectory (242
    # steps) teacher-forced, logits compared at the first and last step of every block, then the free-running
    # decode.  The logit tolerance is 2 x the noise floor stored with the trajectory (the same oracle
    # accumulated in float64: 1.9e-2 of the largest logit at this depth), see forced_and_free; at this depth the
    # two oracle evaluations differ by 0.31 logit units, so more positions are near-ties than at two layers
    # (measured 6.8 % exempt).
    w = synth.WORKLOADS["8b_g256"]
    eng, flt = engine(w, 1)
    rep, rows, loaded = forced_and_free("8b_g256_full", w, (0,), eng, flt, exempt_frac=0.10)
    print("8b_g256 at 32 layers:", rep)


@needs("8b_g1024_eotp_full_states_from_L2")
def test_8b_g1024_eotp_full_depth_block_boundaries():
    # 32 layers, 1280 rows: the first and last state of every block of the two-layer trajectory, evaluated by the
    # oracle at full depth
    w = synth.WORKLOADS["8b_g1024_eotp"]
    eng, flt = engine(w, 1)
    rep, _, _ = forced_and_free("8b_g1024_eotp_full_states_from_L2", w, (0,), eng, flt, exempt_frac=0.15)
    print("8b_g1024_eotp at 32 layers:", rep)


@needs("8b_b32_prefix_full_states_from_L2")
def test_8b_b32_prefix_full_depth_block_boundaries():
    # 32 layers, block 64, prefix cache rebuilt from every imposed state (sequence 0 of the batch alone)
    w = synth.WORKLOADS["8b_b32_prefix"]
    eng, flt = engine(w, 1)
    rep, _, _ = forced_and_free("8b_b32_prefix_full_states_from_L2", w, (0,), eng, flt, exempt_frac=0.15)
    print("8b_b32_prefix at 32 layers:", rep)
