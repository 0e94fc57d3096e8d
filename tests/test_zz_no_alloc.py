"""The entry point that allocates nothing: l2pd_filter_train_static keeps the optimiser moments in a
device array of the library image.  Called through the C ABI with every buffer allocated beforehand,
it must reproduce l2pd_filter_train (same kernel, caller-provided moments) bit for bit: on two calls
in a row, the second on a smaller filter and fewer rows, so that whatever the first call left in the
shared array must not leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2509_25188_amd import binding as Bd
from paper_2509_25188_amd import synth

pytestmark = pytest.mark.gpu


def _case(seed, s, h, n_layers, n_rows, epochs):
    r = np.random.default_rng(seed)
    Cn = r.uniform(size=(n_rows, s)).astype(np.float32)
    Yn = (r.uniform(size=(n_rows, s)) < 0.2 + 0.6 * Cn).astype(np.float32)
    flt = synth.make_filter(seed, s, h, "cpu", n_layers=n_layers)
    return flt, torch.tensor(Cn).cuda(), torch.tensor(Yn).cuda(), epochs


def test_static_scratch_training_equals_caller_scratch_training_twice_in_a_row():
    lib = Bd.lib()
    cases = [_case(71, 64, 128, 2, 90, 60),      # 16,576 parameters: most of the static array is written
             _case(72, 32, 32, 2, 17, 25)]       # then a smaller filter on fewer rows
    # every buffer of the static calls exists before the first of them
    prepared = []
    for flt, Cd, Yd, epochs in cases:
        ref = {k: v.clone().cuda() for k, v in flt.items()}
        ref_losses = Bd.train_filter(ref, Cd, Yd, epochs, lr=1e-2)
        got = {k: v.clone().cuda() for k, v in flt.items()}
        losses = torch.zeros(epochs, dtype=torch.float32, device="cuda")
        prepared.append((ref, ref_losses, got, losses, Cd, Yd, epochs))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for ref, ref_losses, got, losses, Cd, Yd, epochs in prepared:
        f = Bd.Engine.filter_struct(got)
        tc = Bd.TrainCfg(1e-2, 0.9, 0.999, 1e-8, 0.01, epochs)
        rc = lib.l2pd_filter_train_static(C.byref(f), Cd.data_ptr(), Yd.data_ptr(), Cd.shape[0], C.byref(tc),
                                          losses.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert rc == Bd.L2PD_OK
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for ref, ref_losses, got, losses, Cd, Yd, epochs in prepared:
        assert torch.equal(losses, ref_losses)
        assert losses[-1] < losses[0]
        for k in ref:
            assert torch.equal(got[k], ref[k]), k


def test_static_scratch_limit_is_refused_before_any_launch():
    lib = Bd.lib()
    s, h = 64, 512                       # 2 * 64 * 512 + 576 = 66,112 parameters > 20,480
    flt = {k: v.cuda() for k, v in synth.make_filter(73, s, h, "cpu").items()}
    f = Bd.Engine.filter_struct(flt)
    rows = torch.zeros((4, s), dtype=torch.float32, device="cuda")
    tc = Bd.TrainCfg(1e-3, 0.9, 0.999, 1e-8, 0.01, 1)
    w1 = flt["w1"].clone()
    rc = lib.l2pd_filter_train_static(C.byref(f), rows.data_ptr(), rows.data_ptr(), 4, C.byref(tc), None,
                                      torch.cuda.current_stream().cuda_stream)
    assert rc == Bd.L2PD_ENOMEM
    assert b"static scratch" in lib.l2pd_strerror(rc)
    torch.cuda.synchronize()
    assert torch.equal(flt["w1"], w1)
