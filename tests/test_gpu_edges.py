"""GPU parity on the degenerate and extreme shapes of the decoding loop (Alg. 2 / Alg. 3): one
block only, blocks of one token, a one-token prompt, the largest block and filter the library
accepts, and an argument the library must refuse without launching anything."""
import numpy as np
import pytest
import torch

from paper_2509_25188_amd import binding as Bd
from paper_2509_25188_amd import synth
from tests import parity as Pz
from tests.test_gpu_parity import build, small_bf16

pytestmark = pytest.mark.gpu
TINY = synth.WORKLOADS["tiny"].model


def run_against_oracle(w, lm_head_scale=25.0):
    eng, ora, flt, prompt = build(w, lm_head_scale=lm_head_scale)
    fdev = {k: v.cuda() for k, v in flt.items()}
    tok, st, dl = eng.generate(prompt.cuda(), fdev, Pz.cfg_for(w))
    tok = tok.cpu().numpy()
    for b in range(w.batch):
        resp, steps, dlen = Pz.oracle_generate(ora, prompt[b].numpy(), w, Pz.np_filter(flt))
        np.testing.assert_array_equal(tok[b], resp)
        assert int(st[b]) == steps and int(dl[b]) == dlen
    return tok, st.cpu().numpy(), dl.cpu().numpy()


def test_single_block_generation():
    # gen_len == block_len: the loop over blocks degenerates to the inner loop alone
    w = synth.Workload("one_block", TINY, 2, 9, 32, 32, 16, 0.5, prompt_hi=1022)
    tok, st, dl = run_against_oracle(w)
    assert np.all(dl == 32) and np.all(st >= 1) and np.all(st <= 32)


def test_blocks_of_one_token():
    # block_len == 1: every step commits exactly the forced most-confident (only) position
    w = synth.Workload("unit_blocks", TINY, 1, 7, 12, 1, 4, 0.5, prompt_hi=1022)
    tok, st, dl = run_against_oracle(w)
    assert int(st[0]) == 12 and int(dl[0]) == 12


def test_one_token_prompt():
    w = synth.Workload("p1", TINY, 2, 1, 64, 32, 32, 0.5, prompt_hi=1022)
    run_against_oracle(w)


def test_largest_block_and_filter():
    # block_len 256 and 1024 hidden units are the limits of the update kernel's on-chip arrays
    w = synth.Workload("max_block", TINY, 1, 5, 256, 256, 1024, 0.6, prompt_hi=1022)
    tok, st, dl = run_against_oracle(w)
    assert int(dl[0]) == 256


def test_eotp_when_first_block_already_ends():
    # EOS forced everywhere: the first block completes with EOS in it and decoding stops there
    w = synth.Workload("eotp_first", TINY, 1, 8, 96, 32, 16, 0.5, eotp=True, bias_from=0, bias_value=60.0,
                       prompt_hi=1022)
    tok, st, dl = run_against_oracle(w)
    assert int(dl[0]) == 32
    assert np.all(tok[0, :32] == TINY.eos_id) and np.all(tok[0, 32:] == TINY.mask_id)


def test_bf16_decode_rows_not_multiple_of_four():
    # T = 37 + 32 = 69 rows per sequence, 3 sequences: ragged 4-row groups in the GEMM epilogues
    w = small_bf16("bf_ragged", 2, 256, 2, 128, 320, 1500, 3, 37, 32, 32, tau=0.7)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    fdev = {k: v.cuda() for k, v in flt.items()}
    cfg = Pz.cfg_for(w)
    traces = []
    for b in range(3):
        tr = []
        Pz.oracle_generate(ora, prompt[b].numpy(), w, Pz.np_filter(flt), tr)
        traces.append(tr)
    rep = Pz.StepReport()
    Pz.teacher_forced(eng, traces, w.prompt_len, cfg, fdev, w.model, w.threshold, rep)
    print("bf16 ragged rows:", rep)
    assert rep.max_logit_err < 2e-2


def test_refused_arguments_launch_nothing():
    w = synth.WORKLOADS["tiny"]
    eng, ora, flt, prompt = build(w)
    fdev = {k: v.cuda() for k, v in flt.items()}
    bad = Bd.Engine.cfg_struct(w.gen_len + 1, w.block_len, 0.5, False, False, None)   # not a multiple of the block
    with pytest.raises(Exception):
        eng.generate(prompt.cuda(), fdev, bad)
    too_long = Bd.Engine.cfg_struct(w.gen_len * 4, w.block_len, 0.5, False, False, None)   # exceeds max_seq
    with pytest.raises(Exception):
        eng.generate(prompt.cuda(), fdev, too_long)
    # the engine still works afterwards
    tok, st, dl = eng.generate(prompt.cuda(), fdev, Pz.cfg_for(w))
    assert int(dl[0]) == w.gen_len


def test_calls_follow_the_callers_stream():
    # everything a call enqueues (and the host's own polling of the control block) goes to the stream
    # it is given: a decode on a side stream gives the same result as on the default stream, and the
    # default stream stays free to do unrelated work meanwhile
    w = synth.Workload("tiny_stream", TINY, 2, 17, 64, 16, 32, 0.5, prompt_hi=1022)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    fdev = {k: v.cuda() for k, v in flt.items()}
    cfg = Pz.cfg_for(w)
    pd = prompt.cuda()
    ref = eng.generate(pd, fdev, cfg)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        got = eng.generate(pd, fdev, cfg)
        lg = eng.forward(torch.cat([pd, torch.full((2, 64), w.model.mask_id, dtype=torch.int32, device="cuda")], 1))
    busy = torch.ones(1 << 20, device="cuda").cumsum(0)          # the default stream does something else
    side.synchronize()
    torch.cuda.synchronize()
    for a, b in zip(ref, got):
        assert torch.equal(a, b)
    assert torch.isfinite(lg).all() and float(busy[-1]) == float(1 << 20)


@pytest.mark.parametrize("bf16", [False, True])
def test_denoise_step_can_be_captured_in_a_hip_graph(bf16):
    # a serving loop may capture the full-recompute step (no host synchronisation, no memset nodes: the
    # library clears with fill kernels) and replay it; every replay must equal the eager step, with the
    # program's own eager work and synchronisations between the replays
    if bf16:
        w = small_bf16("bf_graph", 2, 256, 4, 64, 448, 2000, 2, 40, 64, 32, tau=0.7)
    else:
        w = synth.Workload("tiny_graph", TINY, 2, 21, 64, 32, 32, 0.5, prompt_hi=1022)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    fdev = {k: v.cuda() for k, v in flt.items()}
    cfg = Pz.cfg_for(w)
    X0 = torch.cat([prompt, torch.full((w.batch, w.gen_len), w.model.mask_id, dtype=torch.int32)], 1).cuda()
    S0 = torch.zeros((w.batch, 3), dtype=torch.int32, device="cuda")
    # eager reference: the state after each of six steps
    Xe, Se = X0.clone(), S0.clone()
    want = []
    for _ in range(6):
        eng.denoise_step(Xe, w.prompt_len, Se, fdev, cfg)
        want.append((Xe.clone(), Se.clone()))
    torch.cuda.synchronize()
    Xg, Sg = X0.clone(), S0.clone()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        eng.denoise_step(Xg, w.prompt_len, Sg, fdev, cfg)          # warm-up on the capture stream, then rewind
        Xg.copy_(X0)
        Sg.copy_(S0)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            eng.denoise_step(Xg, w.prompt_len, Sg, fdev, cfg)
    torch.cuda.synchronize()
    for k in range(6):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Xg, want[k][0]) and torch.equal(Sg, want[k][1]), f"replay {k}"
        other = eng.forward(X0)                                     # eager work of the same context in between
        torch.cuda.synchronize()
        assert torch.isfinite(other).all()
