"""GPU parity for the Extremely Greedy Parallel rollout (Alg. 1's labelling) and the filter training
(Eq. 6 with AdamW), against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import l2pd_oracle as O
from paper_2509_25188_amd import binding as Bd
from paper_2509_25188_amd import synth
from tests import parity as Pz
from tests.test_gpu_parity import build, small_bf16

pytestmark = pytest.mark.gpu
TINY = synth.WORKLOADS["tiny"].model


def references(w, ora, flt, prompt, corrupt_every=0):
    """The model's own vanilla (one token per step) answers, optionally with every n-th token replaced
    so that some positions can never agree with the prediction."""
    refs = []
    for b in range(w.batch):
        resp, _, _ = O.generate(ora, prompt[b].numpy(), w.gen_len, w.block_len, w.model.mask_id, w.model.eos_id,
                                Pz.np_filter(flt), 2.0)
        if corrupt_every:
            resp = resp.copy()
            resp[::corrupt_every] = (resp[::corrupt_every] + 1) % 1000
        refs.append(resp)
    return np.stack(refs)


@pytest.mark.parametrize("corrupt_every", [0, 5])
def test_egp_rollout_fp32_matches_oracle(corrupt_every):
    w = synth.Workload("tiny_egp", TINY, 2, 11, 64, 32, 16, 0.5, prompt_hi=1022)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    ref = references(w, ora, flt, prompt, corrupt_every)
    cfg = Bd.Engine.cfg_struct(w.gen_len, w.block_len, 0.5)
    C, Y, steps = eng.egp_rollout(prompt.cuda(), torch.tensor(ref, dtype=torch.int32).cuda(), cfg)
    C, Y, steps = C.cpu().numpy(), Y.cpu().numpy(), steps.cpu().numpy()
    for b in range(2):
        Co, Yo, per_block = O.egp_rollout(ora, prompt[b].numpy(), ref[b], w.gen_len, w.block_len, w.model.mask_id)
        n = len(Co)
        print(f"EGP rollout (corrupt_every={corrupt_every}) seq {b}: steps per block {per_block}")
        assert steps[b] == n
        np.testing.assert_array_equal(Y[b, :n], Yo)
        np.testing.assert_allclose(C[b, :n], Co, rtol=1e-4, atol=1e-6)
        assert np.all(C[b, n:] == 0)
        if corrupt_every:
            assert (Yo == 0).any() and n > 2 * (w.gen_len // w.block_len)
    # lock-step batch: both sequences walk the blocks together, so a sequence never has more rows than gen_len
    assert steps.max() <= w.gen_len


def test_egp_rollout_bf16_rows_close_where_labels_agree():
    w = small_bf16("bf_egp", 2, 256, 4, 64, 512, 2000, 1, 40, 64, 32, tau=0.7)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    ref = references(w, ora, flt, prompt, 7)
    cfg = Bd.Engine.cfg_struct(w.gen_len, w.block_len, 0.5)
    C, Y, steps = eng.egp_rollout(prompt.cuda(), torch.tensor(ref, dtype=torch.int32).cuda(), cfg)
    Co, Yo, per_block = O.egp_rollout(ora, prompt[0].numpy(), ref[0], w.gen_len, w.block_len, w.model.mask_id)
    n = int(steps[0])
    C, Y = C.cpu().numpy()[0, :n], Y.cpu().numpy()[0, :n]
    # Both rollouts follow the same trajectory until a near-tie is resolved differently in bf16 (a prediction
    # that equals the reference in one arithmetic and not in the other).  Up to and including the first row
    # whose labels differ the two were computed from the same state, so those confidence rows must agree;
    # if no row differs the rollouts are identical throughout.
    m = min(n, len(Co))
    differ = [i for i in range(m) if not np.array_equal(Y[i], Yo[i])]
    k = min(differ[0] + 1, m) if differ else m
    print(f"bf16 EGP rollout: {n} rows, oracle {len(Co)}; first row with different labels: "
          f"{differ[0] if differ else None}; confidence rows compared: {k}")
    assert k >= 1
    assert np.max(np.abs(C[:k] - Co[:k]) / np.maximum(Co[:k], 1e-3)) < 0.4
    if not differ:
        assert n == len(Co)
    # invariants that hold whatever the rounding: labels are 0/1, committed entries are (1.0, 1), the last row of a
    # block has no masked position left afterwards, row count within bounds
    assert set(np.unique(Y)) <= {0.0, 1.0}
    assert np.all(Y[C == 1.0] == 1.0)
    assert w.gen_len // w.block_len <= n <= w.gen_len


def test_filter_training_matches_oracle():
    s, h, n = 32, 32, 300
    r = np.random.default_rng(61)
    Cn = r.uniform(size=(n, s)).astype(np.float32)
    Yn = (r.uniform(size=(n, s)) < 0.2 + 0.6 * Cn).astype(np.float32)       # labels correlated with the confidence
    flt = synth.make_filter(62, s, h, "cpu")
    fnp = Pz.np_filter(flt)
    Cd, Yd = torch.tensor(Cn).cuda(), torch.tensor(Yn).cuda()
    # a few epochs: parameter by parameter.  (Over hundreds of epochs a ReLU that switches for one row in
    # fp32 but not in fp64 changes a gradient entry by a finite amount, and Adam's normalisation turns
    # that into diverging parameters at equal loss: the long run is compared through losses and outputs.)
    fdev = {k: v.clone().cuda() for k, v in flt.items()}
    losses = Bd.train_filter(fdev, Cd, Yd, 20, lr=1e-3).cpu().numpy()
    ref, ref_losses = O.train_filter(fnp, Cn, Yn, 20, lr=1e-3)
    np.testing.assert_allclose(losses, ref_losses, rtol=1e-5, atol=1e-7)
    for k in ref:
        d = np.abs(fdev[k].cpu().numpy() - ref[k])
        assert np.mean(d < 1e-4) > 0.995 and d.max() < 2.5e-2, (k, d.max(), np.mean(d < 1e-4))   # 20 steps of 1e-3 at most
    fdev = {k: v.clone().cuda() for k, v in flt.items()}
    losses = Bd.train_filter(fdev, Cd, Yd, 300, lr=1e-2).cpu().numpy()
    ref, ref_losses = O.train_filter(fnp, Cn, Yn, 300, lr=1e-2)
    print(f"filter training: loss {losses[0]:.5f} -> {losses[-1]:.5f} (oracle {ref_losses[0]:.5f} -> {ref_losses[-1]:.5f})")
    np.testing.assert_allclose(losses, ref_losses, rtol=1e-3, atol=1e-6)
    assert losses[-1] < 0.9 * losses[0]
    p_gpu = np.stack([O.filter_prob(Cn[i], {k: v.cpu().numpy() for k, v in fdev.items()}) for i in range(32)])
    p_ref = np.stack([O.filter_prob(Cn[i].astype(np.float64), ref) for i in range(32)])
    assert np.max(np.abs(p_gpu - p_ref)) < 2e-2


@pytest.mark.parametrize("s,h,n", [(8, 4, 5), (64, 128, 70), (1, 1, 3)])
def test_filter_training_shapes(s, h, n):
    # rows fewer than a chunk, the largest filter the kernel accepts (ragged last chunk), the smallest one
    r = np.random.default_rng(63)
    Cn = r.uniform(size=(n, s)).astype(np.float32)
    Yn = (r.uniform(size=(n, s)) > 0.5).astype(np.float32)
    flt = synth.make_filter(64, s, h, "cpu")
    fdev = {k: v.clone().cuda() for k, v in flt.items()}
    losses = Bd.train_filter(fdev, torch.tensor(Cn).cuda(), torch.tensor(Yn).cuda(), 40, lr=1e-2)
    ref, ref_losses = O.train_filter(Pz.np_filter(flt), Cn, Yn, 40, lr=1e-2)
    np.testing.assert_allclose(losses.cpu().numpy(), ref_losses, rtol=5e-4, atol=1e-6)
    for k in ref:
        d = np.abs(fdev[k].cpu().numpy() - ref[k])
        assert np.mean(d < 1e-3) > 0.98, (k, d.max())


def test_rollout_then_training_lowers_the_loss_on_the_rollout_rows():
    w = synth.Workload("tiny_egp2", TINY, 1, 11, 64, 32, 32, 0.5, prompt_hi=1022)
    eng, ora, flt, prompt = build(w, lm_head_scale=25.0)
    ref = references(w, ora, flt, prompt, 4)
    cfg = Bd.Engine.cfg_struct(w.gen_len, w.block_len, 0.5)
    C, Y, steps = eng.egp_rollout(prompt.cuda(), torch.tensor(ref, dtype=torch.int32).cuda(), cfg)
    n = int(steps[0])
    rows_c, rows_y = C[0, :n].contiguous(), Y[0, :n].contiguous()
    fdev = {k: v.clone().cuda() for k, v in flt.items()}
    losses = Bd.train_filter(fdev, rows_c, rows_y, 500, lr=1e-2).cpu().numpy()
    print(f"rollout rows {n}; loss {losses[0]:.4f} -> {losses[-1]:.4f}")
    assert losses[-1] < 0.5 * losses[0]
