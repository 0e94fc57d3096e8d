"""GPU tests for per-sequence block pointers: every sequence of a batch works on its own block instead
of idling until the others finish the common one.  Tokens and per-sequence step counts must be what the
lock-step batch (and the oracle, sequence by sequence) gives; only the number of forwards falls."""
import numpy as np
import pytest
import torch

from paper_2509_25188_amd import binding as Bd
from paper_2509_25188_amd import synth
from tests import parity as Pz
from tests.test_gpu_parity import build, small_bf16

pytestmark = pytest.mark.gpu
TINY = synth.WORKLOADS["tiny"].model


def cfg_of(w, ragged):
    bias = (w.model.eos_id, w.bias_from, w.bias_value) if w.bias_value else None
    return Bd.Engine.cfg_struct(w.gen_len, w.block_len, w.threshold, Bd.EOTP_STEP if w.eotp_step else w.eotp,
                                w.prefix_cache, bias, w.dual_cache, ragged)


def forwards(eng, prompt, fdev, cfg):
    eng.profile_select(Bd.K_UPDATE)
    out = eng.generate(prompt, fdev, cfg)
    torch.cuda.synchronize()
    n, _ = eng.profile_read()
    eng.profile_select(Bd.K_NONE)
    return out, n


@pytest.mark.parametrize("mode", [Bd.RAGGED_BLOCKS, Bd.RAGGED_COMPACT])
@pytest.mark.parametrize("eotp,eotp_step", [(False, False), (True, False), (True, True)])
def test_ragged_batch_equals_lock_step_and_oracle_fp32(eotp, eotp_step, mode):
    w = synth.Workload("tiny_rag", TINY, 4, 13, 128, 32, 32, 0.5, eotp=eotp, eotp_step=eotp_step,
                       bias_from=70 if eotp else -1, bias_value=60.0 if eotp else 0.0, prompt_hi=1022)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    fdev = {k: v.cuda() for k, v in flt.items()}
    (t0, s0, d0), n_lock = forwards(eng, prompt.cuda(), fdev, cfg_of(w, False))
    (t1, s1, d1), n_rag = forwards(eng, prompt.cuda(), fdev, cfg_of(w, mode))
    launches, seq_steps = eng.generate_stats()
    assert torch.equal(t0, t1) and torch.equal(s0, s1) and torch.equal(d0, d1)
    # what the decode enqueued: without compaction every step runs over the whole batch; with it a finished
    # sequence is dropped once the host has seen it (one to two chunks of four steps late), never earlier
    assert launches == n_rag
    if mode == Bd.RAGGED_COMPACT and not eotp_step:
        assert int(s1.sum()) <= seq_steps <= w.batch * launches
    else:
        assert seq_steps == w.batch * launches
    for b in range(w.batch):
        resp, steps, dlen = Pz.oracle_generate(ora, prompt[b].numpy(), w, Pz.np_filter(flt))
        np.testing.assert_array_equal(t1.cpu().numpy()[b], resp)
        assert int(s1[b]) == steps and int(d1[b]) == dlen
    steps = s1.cpu().numpy()
    print(f"eotp={eotp} step={eotp_step}: steps per sequence {steps.tolist()}, forwards enqueued lock step {n_lock}, ragged {n_rag}")
    # the host enqueues steps in chunks of 4 until the device reports completion
    assert steps.max() <= n_rag <= steps.max() + 8
    assert n_rag <= n_lock


def test_ragged_denoise_step_sequences_at_different_blocks():
    # two sequences imposed at different blocks in one call: each must get its own block's step
    w = synth.Workload("tiny_rag2", TINY, 2, 13, 128, 32, 32, 0.5, bias_from=40, bias_value=5.0, prompt_hi=1022)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    fdev = {k: v.cuda() for k, v in flt.items()}
    blocks = [1, 3]
    X = np.stack([Pz.random_state(w, 5 + b, blocks[b], 7 + 3 * b, b) for b in range(2)])
    recs = [Pz.oracle_step_record(ora, X[b], w, Pz.np_filter(flt), blocks[b]) for b in range(2)]
    Xd = torch.tensor(X, dtype=torch.int32, device="cuda")
    state = torch.tensor([[blocks[0], 4, 0], [blocks[1], 9, 0]], dtype=torch.int32, device="cuda")
    taps = eng.denoise_step(Xd, w.prompt_len, state, fdev, cfg_of(w, True), want_logits=True)
    torch.cuda.synchronize()
    rep = Pz.StepReport()
    for b in range(2):
        assert Pz.check_step(recs[b], taps, b, w.model, w.threshold, 1e-4, rep)
        lo = w.prompt_len + blocks[b] * w.block_len
        after = X[b].copy()
        idx = np.nonzero(recs[b]["sel"])[0]
        after[lo + idx] = recs[b]["pre"][idx]
        np.testing.assert_array_equal(Xd.cpu().numpy()[b], after)
    assert state.cpu().numpy()[:, 1].tolist() == [5, 10]
    print("ragged denoise_step:", rep)


@pytest.mark.parametrize("mode", [Bd.RAGGED_BLOCKS, Bd.RAGGED_COMPACT])
def test_ragged_bf16_batch_rows_equal_lock_step(mode):
    w = small_bf16("bf_rag", 2, 256, 4, 64, 448, 2000, 5, 40, 128, 32, tau=0.7)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    fdev = {k: v.cuda() for k, v in flt.items()}
    (t0, s0, d0), n_lock = forwards(eng, prompt.cuda(), fdev, cfg_of(w, False))
    (t1, s1, d1), n_rag = forwards(eng, prompt.cuda(), fdev, cfg_of(w, mode))
    # same kernels on the same rows: the sequences do not interact, so the bits agree
    assert torch.equal(t0, t1) and torch.equal(s0, s1) and torch.equal(d0, d1)
    print(f"bf16 batch of 5: steps {s1.tolist()}, forwards lock step {n_lock}, ragged {n_rag}")
    assert n_rag <= n_lock


def test_ragged_forward_count_matches_the_oracle_traces():
    # fixed-threshold decoding spreads the per-block step counts of the sequences; the oracle's traces give
    # the forwards each schedule needs: lock step = sum over blocks of the slowest sequence's steps in that
    # block, own-block pointers = the slowest sequence's total
    w = synth.Workload("tiny_rag3", TINY, 6, 13, 128, 16, 16, 0.5, prompt_hi=1022)
    eng, ora, _, prompt = build(w, lm_head_scale=120.0)
    flt = synth.threshold_filter(w.block_len, 0.9)
    fdev = {k: v.cuda() for k, v in flt.items()}
    per_block = np.zeros((w.batch, w.gen_len // w.block_len), dtype=np.int64)
    want = []
    for b in range(w.batch):
        tr = []
        want.append(Pz.oracle_generate(ora, prompt[b].numpy(), w, Pz.np_filter(flt), trace=tr))
        for d in tr:
            per_block[b, d["block"]] += 1
    need_lock, need_rag = int(per_block.max(axis=0).sum()), int(per_block.sum(axis=1).max())
    (t0, s0, _), n_lock = forwards(eng, prompt.cuda(), fdev, cfg_of(w, False))
    (t1, s1, _), n_rag = forwards(eng, prompt.cuda(), fdev, cfg_of(w, Bd.RAGGED_BLOCKS))
    (t2, s2, d2), n_cmp = forwards(eng, prompt.cuda(), fdev, cfg_of(w, Bd.RAGGED_COMPACT))
    for b in range(w.batch):
        np.testing.assert_array_equal(t1.cpu().numpy()[b], want[b][0])
        np.testing.assert_array_equal(t2.cpu().numpy()[b], want[b][0])
        assert int(s1[b]) == want[b][1] == int(s0[b]) == int(s2[b])
        assert int(d2[b]) == want[b][2]
    assert torch.equal(t0, t1) and n_cmp == n_rag
    print(f"threshold decoding, batch of 6: steps {s1.tolist()}; forwards needed lock step {need_lock}, own blocks "
          f"{need_rag}; enqueued {n_lock}, {n_rag}")
    assert need_lock <= n_lock <= need_lock + 8 and need_rag <= n_rag <= need_rag + 8
    assert need_rag < need_lock


@pytest.mark.parametrize("dual", [False, True])
@pytest.mark.parametrize("eotp", [False, True])
def test_ragged_batch_with_kv_cache_equals_the_oracle_fp32(dual, eotp):
    # per-sequence block pointers with the prefix / dual cache (Sec. 4.3): every sequence's slice of the
    # K/V stores is rebuilt when that sequence enters a new block; fixed-threshold decoding on a peaked
    # model spreads the per-block step counts, so the sequences really sit in different blocks
    w = synth.Workload("tiny_ragkv", TINY, 4, 13, 96, 16, 16, 0.5, eotp=eotp, prefix_cache=not dual, dual_cache=dual,
                       bias_from=50 if eotp else -1, bias_value=60.0 if eotp else 0.0, prompt_hi=1022)
    eng, ora, _, prompt = build(w, lm_head_scale=120.0)
    flt = synth.threshold_filter(w.block_len, 0.9)
    fdev = {k: v.cuda() for k, v in flt.items()}
    per_block = np.zeros((w.batch, w.gen_len // w.block_len), dtype=np.int64)
    want = []
    for b in range(w.batch):
        tr = []
        want.append(Pz.oracle_generate(ora, prompt[b].numpy(), w, Pz.np_filter(flt), trace=tr))
        for d in tr:
            per_block[b, d["block"]] += 1
    need_lock, need_rag = int(per_block.max(axis=0).sum()), int(per_block.sum(axis=1).max())
    (t0, s0, d0), n_lock = forwards(eng, prompt.cuda(), fdev, cfg_of(w, False))
    (t1, s1, d1), n_rag = forwards(eng, prompt.cuda(), fdev, cfg_of(w, Bd.RAGGED_BLOCKS))
    rows_rag = eng.generate_stats()[1]
    (t2, s2, d2), n_cmp = forwards(eng, prompt.cuda(), fdev, cfg_of(w, Bd.RAGGED_COMPACT))   # live sequences moved to the front, their K/V slices with them
    steps_cmp, rows_cmp = eng.generate_stats()
    for b in range(w.batch):
        for t, st, dl in ((t0, s0, d0), (t1, s1, d1), (t2, s2, d2)):
            np.testing.assert_array_equal(t.cpu().numpy()[b], want[b][0])
            assert int(st[b]) == want[b][1] and int(dl[b]) == want[b][2]
    print(f"{'dual' if dual else 'prefix'} cache, eotp={eotp}: steps {s1.tolist()}; forwards needed lock step {need_lock}, "
          f"own blocks {need_rag}; enqueued {n_lock}, {n_rag}")
    assert n_rag == need_rag == n_cmp == steps_cmp   # the host looks before every step: not one forward too many
    assert need_rag <= need_lock and n_rag <= n_lock
    # compaction: a step runs over the sequences still decoding only, so the sequence-steps are the sum of the
    # sequences' own step counts once every finished sequence has been dropped at the host's next look
    print(f"sequence-steps: own blocks {rows_rag}, with compaction {rows_cmp}, sum of the step counts {int(s2.sum())}")
    assert rows_rag == w.batch * n_rag and rows_cmp == int(s2.sum())
    if len(set(s2.tolist())) > 1:
        assert rows_cmp < rows_rag
    if not eotp:
        assert need_rag < need_lock     # six blocks of spread step counts: own blocks really save forwards


def test_ragged_denoise_step_with_prefix_cache_sequences_at_different_blocks():
    # two sequences imposed at different blocks in one call, prefix cache: each gets its own store rebuild
    # (a forward over its own prefix) and its own block's step
    w = synth.Workload("tiny_rag4", TINY, 2, 13, 128, 32, 32, 0.5, prefix_cache=True, bias_from=40, bias_value=5.0,
                       prompt_hi=1022)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    fdev = {k: v.cuda() for k, v in flt.items()}
    blocks = [2, 0]
    X = np.stack([Pz.random_state(w, 15 + b, blocks[b], 5 + 4 * b, b) for b in range(2)])
    recs = [Pz.oracle_step_record(ora, X[b], w, Pz.np_filter(flt), blocks[b]) for b in range(2)]
    Xd = torch.tensor(X, dtype=torch.int32, device="cuda")
    state = torch.tensor([[blocks[0], 4, 0], [blocks[1], 9, 0]], dtype=torch.int32, device="cuda")
    taps = eng.denoise_step(Xd, w.prompt_len, state, fdev, cfg_of(w, True), want_logits=True)
    torch.cuda.synchronize()
    rep = Pz.StepReport()
    for b in range(2):
        assert Pz.check_step(recs[b], taps, b, w.model, w.threshold, 1e-4, rep)
    assert state.cpu().numpy()[:, 1].tolist() == [5, 10]
    print("ragged denoise_step with prefix cache:", rep)


@pytest.mark.parametrize("B,dual", [(5, False), (5, True), (2, False)])
def test_ragged_bf16_kv_cache_rows_match_lock_step(B, dual):
    # bf16, block-only steps of 160 rows (wide GEMM path) and of 64 rows (few-row path): the sequences go
    # through the same kernels in either schedule, only at other positions of the batch, so tokens agree
    w = small_bf16("bf_ragkv", 2, 256, 4, 64, 448, 2000, B, 40, 128, 32, tau=0.7, eotp=True, prefix_cache=not dual,
                   dual_cache=dual, bias_from=75, bias_value=60.0)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    fdev = {k: v.cuda() for k, v in flt.items()}
    (t0, s0, d0), n_lock = forwards(eng, prompt.cuda(), fdev, cfg_of(w, False))
    (t1, s1, d1), n_rag = forwards(eng, prompt.cuda(), fdev, cfg_of(w, Bd.RAGGED_BLOCKS))
    assert torch.equal(d0, d1) and d1.tolist() == [96] * B
    same = torch.equal(t0, t1) and torch.equal(s0, s1)
    print(f"bf16 {'dual' if dual else 'prefix'} cache batch of {B}: steps {s1.tolist()} (lock step {s0.tolist()}), "
          f"forwards lock step {n_lock}, own blocks {n_rag}, identical {same}")
    # a single-sequence store rebuild runs 40..136 rows through other GEMM tiles than the batched rebuild
    # (same K order per element on the wide path, another split depth on the few-row path), so identity is
    # expected whenever every rebuild stays on one path; the invariants hold regardless
    assert not torch.any(t1[:, :96] == w.model.mask_id) and torch.all(t1[:, 96:] == w.model.mask_id)
    assert n_rag <= n_lock
    # compaction on top: the live sequences and their slices of the stores move to the front; the same
    # invariants, and a step runs over the sequences still decoding only
    rows_rag = eng.generate_stats()[1]
    (t2, s2, d2), n_cmp = forwards(eng, prompt.cuda(), fdev, cfg_of(w, Bd.RAGGED_COMPACT))
    rows_cmp = eng.generate_stats()[1]
    assert torch.equal(d2, d1)
    assert not torch.any(t2[:, :96] == w.model.mask_id) and torch.all(t2[:, 96:] == w.model.mask_id)
    assert rows_cmp == int(s2.sum()) <= rows_rag
    print(f"  compaction: steps {s2.tolist()}, identical to own blocks {torch.equal(t1, t2) and torch.equal(s1, s2)}, "
          f"sequence-steps {rows_rag} -> {rows_cmp}")
