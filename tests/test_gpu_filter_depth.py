"""GPU parity for the filter-depth variants of Table 3 (one, two and four layers): decoding with each,
teacher-forced and free-running, and training each, against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import l2pd_oracle as O
from paper_2509_25188_amd import binding as Bd
from paper_2509_25188_amd import synth
from tests import parity as Pz
from tests.test_gpu_parity import build

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_layers,hidden", [(1, 64), (2, 64), (4, 64), (4, 48), (3, 200)])
def test_decode_with_filters_of_each_depth_fp32(n_layers, hidden):
    w = synth.WORKLOADS["tiny"]
    eng, ora, _, prompt = build(w, lm_head_scale=25.0)
    flt = synth.make_filter(77, w.block_len, hidden, "cpu", n_layers=n_layers)
    assert len(flt) == 2 * n_layers
    trace = []
    resp, steps, dlen = Pz.oracle_generate(ora, prompt[0].numpy(), w, Pz.np_filter(flt), trace)
    fdev = {k: v.cuda() for k, v in flt.items()}
    cfg = Pz.cfg_for(w)
    rep = Pz.StepReport()
    same = Pz.teacher_forced(eng, [trace], w.prompt_len, cfg, fdev, w.model, w.threshold, rep)
    print(f"{n_layers}-layer filter (hidden {hidden}): {rep}; oracle steps {steps}")
    assert rep.max_p_err < 1e-4
    tok, st, dl = eng.generate(prompt.cuda(), fdev, cfg)
    if same:
        np.testing.assert_array_equal(tok.cpu().numpy()[0], resp)
        assert int(st[0]) == steps and int(dl[0]) == dlen


def test_single_layer_filter_equals_two_layer_with_identity_first_layer():
    # the reduction the oracle is pinned with, on the device: same decisions, same trajectory
    w = synth.WORKLOADS["tiny"]
    eng, ora, _, prompt = build(w, lm_head_scale=25.0)
    s = w.block_len
    one = synth.make_filter(78, s, s, "cuda", n_layers=1)
    two = {"w1": torch.eye(s, device="cuda"), "b1": torch.zeros(s, device="cuda"), "w2": one["w1"], "b2": one["b1"]}
    cfg = Pz.cfg_for(w)
    a = eng.generate(prompt.cuda(), one, cfg)
    b = eng.generate(prompt.cuda(), two, cfg)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("n_layers,s,h,n", [(1, 32, 32, 300), (4, 32, 32, 300), (4, 64, 64, 70), (3, 8, 5, 9),
                                            (1, 1, 1, 3)])
def test_training_filters_of_each_depth_matches_oracle(n_layers, s, h, n):
    r = np.random.default_rng(81)
    Cn = r.uniform(size=(n, s)).astype(np.float32)
    Yn = (r.uniform(size=(n, s)) < 0.2 + 0.6 * Cn).astype(np.float32)
    flt = synth.make_filter(82, s, h, "cpu", n_layers=n_layers)
    fdev = {k: v.clone().cuda() for k, v in flt.items()}
    Cd, Yd = torch.tensor(Cn).cuda(), torch.tensor(Yn).cuda()
    losses = Bd.train_filter(fdev, Cd, Yd, 20, lr=1e-3).cpu().numpy()
    ref, ref_losses = O.train_filter(Pz.np_filter(flt), Cn, Yn, 20, lr=1e-3)
    np.testing.assert_allclose(losses, ref_losses, rtol=1e-5, atol=1e-7)
    assert set(ref) == set(fdev)
    for k in ref:
        d = np.abs(fdev[k].cpu().numpy() - ref[k])
        assert np.mean(d < 1e-4) > 0.99 and d.max() < 2.5e-2, (k, d.max(), np.mean(d < 1e-4))
    # a longer run through losses and outputs (parameters may drift apart at equal loss once a ReLU
    # switches in one precision and not in the other)
    fdev = {k: v.clone().cuda() for k, v in flt.items()}
    losses = Bd.train_filter(fdev, Cd, Yd, 200, lr=3e-3).cpu().numpy()
    ref, ref_losses = O.train_filter(Pz.np_filter(flt), Cn, Yn, 200, lr=3e-3)
    print(f"{n_layers} layers, s {s}, hidden {h}, rows {n}: loss {losses[0]:.5f} -> {losses[-1]:.5f} "
          f"(oracle {ref_losses[0]:.5f} -> {ref_losses[-1]:.5f})")
    n_params = sum(v.numel() for v in flt.values())
    if n * s >= n_params:
        np.testing.assert_allclose(losses, ref_losses, rtol=1e-2, atol=1e-5)
    else:
        # more parameters than targets: the descent is ill-conditioned and the two precisions part ways
        # after some tens of steps; the first stretch still agrees, and both fit the rows
        np.testing.assert_allclose(losses[:40], ref_losses[:40], rtol=1e-2, atol=1e-5)
        assert abs(losses[-1] - ref_losses[-1]) < 0.15 * ref_losses[-1]
    assert losses[-1] < losses[0]


def test_filters_too_large_for_the_training_kernel_are_refused():
    flt = synth.make_filter(83, 64, 128, "cuda", n_layers=4)      # 49,600 parameters
    C = torch.rand(10, 64, device="cuda")
    with pytest.raises(RuntimeError):
        Bd.train_filter(flt, C, (C > 0.5).float(), 2)
