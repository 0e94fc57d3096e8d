"""Differential test over seeded random decode configurations on the tiny fp32 model: whole
generations on the GPU against the oracle, sequence by sequence.  Every case draws batch size,
prompt length, window, block size, threshold, filter depth and width, EoTP mode, cache mode, batch
schedule and the position of a forced end-of-text, so that combinations no hand-written test names
still get exercised."""
import numpy as np
import pytest
import torch

from paper_2509_25188_amd import binding as Bd
from paper_2509_25188_amd import synth
from tests import parity as Pz

pytestmark = pytest.mark.gpu
TINY = synth.WORKLOADS["tiny"].model


def draw(seed):
    r = np.random.default_rng(1000 + seed)
    s = int(r.choice([8, 16, 32]))
    n_blocks = int(r.integers(1, 5))
    G = s * n_blocks
    P = int(r.integers(1, 40))
    B = int(r.integers(1, 4))
    eotp_mode = int(r.integers(0, 3))                       # off, block, step
    cache = int(r.integers(0, 3)) if eotp_mode != 2 else 0   # step-granular EoTP is full recompute only
    ragged = int(r.integers(0, 3))                            # lock step, own blocks, own blocks + compaction
    bias_from = int(r.integers(0, G)) if eotp_mode and r.random() < 0.8 else -1
    w = synth.Workload(f"rand{seed}", TINY, B, P, G, s, int(r.choice([8, 32, 48])), float(r.choice([0.3, 0.5, 0.8])),
                       eotp=eotp_mode > 0, eotp_step=eotp_mode == 2, prefix_cache=cache == 1, dual_cache=cache == 2,
                       bias_from=bias_from, bias_value=60.0 if bias_from >= 0 else 0.0, prompt_hi=1022)
    return w, ragged, int(r.integers(1, 5))


@pytest.mark.parametrize("seed", range(48))
def test_random_configuration_against_the_oracle(seed):
    w, ragged, depth = draw(seed)
    weights = synth.make_weights(w.model, 77 + seed, "cpu", lm_head_scale=25.0)
    ora = Pz.oracle_model(w.model, weights)
    eng = Bd.Engine(w.model, Pz.to_dev(weights), w.batch, w.prompt_len + w.gen_len, w.prefix_cache or w.dual_cache)
    flt = synth.make_filter(500 + seed, w.block_len, w.filter_hidden, "cpu", n_layers=depth)
    prompt = synth.make_prompt(300 + seed, w.batch, w.prompt_len, w.prompt_hi, "cpu")
    cfg = Pz.cfg_for(w)
    cfg.ragged = ragged
    fdev = {k: v.cuda() for k, v in flt.items()}
    tok, st, dl = eng.generate(prompt.cuda(), fdev, cfg)
    torch.cuda.synchronize()
    tok, st, dl = tok.cpu().numpy(), st.cpu().numpy(), dl.cpu().numpy()
    what = (f"B={w.batch} P={w.prompt_len} G={w.gen_len} s={w.block_len} tau={w.threshold} depth={depth} "
            f"hidden={w.filter_hidden} eotp={'step' if w.eotp_step else w.eotp} cache="
            f"{'prefix' if w.prefix_cache else 'dual' if w.dual_cache else 'none'} ragged={ragged} bias_from={w.bias_from}")
    print(what, "steps", st.tolist(), "decoded", dl.tolist())
    for b in range(w.batch):
        resp, steps, dlen = Pz.oracle_generate(ora, prompt[b].numpy(), w, Pz.np_filter(flt))
        np.testing.assert_array_equal(tok[b], resp, err_msg=what)
        assert int(st[b]) == steps and int(dl[b]) == dlen, what


def test_one_context_serves_changing_calls():
    # one context (created with K/V stores) takes a run of calls that differ in batch, lengths, block,
    # cache mode, EoTP mode and batch schedule, with forwards and single steps in between: nothing a call
    # leaves behind (pending partials, stores, control block, compaction copies) may leak into the next
    weights = synth.make_weights(TINY, 911, "cpu", lm_head_scale=25.0)
    ora = Pz.oracle_model(TINY, weights)
    eng = Bd.Engine(TINY, Pz.to_dev(weights), 3, 40 + 128, True)
    for seed in (3, 7, 10, 12, 0, 17, 22, 9, 15, 1):
        w, ragged, depth = draw(seed)
        flt = synth.make_filter(500 + seed, w.block_len, w.filter_hidden, "cpu", n_layers=depth)
        fdev = {k: v.cuda() for k, v in flt.items()}
        prompt = synth.make_prompt(300 + seed, w.batch, w.prompt_len, w.prompt_hi, "cpu")
        cfg = Pz.cfg_for(w)
        cfg.ragged = ragged
        tok, st, dl = eng.generate(prompt.cuda(), fdev, cfg)
        tok, st, dl = tok.cpu().numpy(), st.cpu().numpy(), dl.cpu().numpy()
        for b in range(w.batch):
            resp, steps, dlen = Pz.oracle_generate(ora, prompt[b].numpy(), w, Pz.np_filter(flt))
            np.testing.assert_array_equal(tok[b], resp, err_msg=f"seed {seed}")
            assert int(st[b]) == steps and int(dl[b]) == dlen, seed
        # a forward and a teacher-forced step of another shape in between
        X = synth.make_prompt(seed, 2, 50 + seed, 1022, "cpu")
        got = eng.forward(X.cuda()).cpu().numpy()
        assert Pz.rel_err(got[1], ora.forward(X[1].numpy())) < 1e-4
        w2 = synth.Workload("mid_call", TINY, 1, 9, 64, 16, 32, 0.5, dual_cache=seed % 2 == 0, prompt_hi=1022)
        f2 = synth.make_filter(seed, 16, 32, "cpu")
        Xs = Pz.random_state(w2, seed, 2, 5)
        rec = Pz.oracle_step_record(ora, Xs, w2, Pz.np_filter(f2), 2)
        Xd = torch.tensor(Xs, dtype=torch.int32, device="cuda").view(1, -1)
        state = torch.tensor([[2, 1, 0]], dtype=torch.int32, device="cuda")
        taps = eng.denoise_step(Xd, w2.prompt_len, state, {k: v.cuda() for k, v in f2.items()}, Pz.cfg_for(w2),
                                want_logits=True)
        rep = Pz.StepReport()
        assert Pz.check_step(rec, taps, 0, TINY, w2.threshold, 1e-4, rep)
