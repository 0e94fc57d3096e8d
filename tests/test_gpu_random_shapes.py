"""Seeded random model shapes on the bf16 path: logits of a full forward against the oracle.  Widths,
head size, FFN width, vocabulary, sequence length and batch are drawn so that the tile chooser of the
GEMMs, the ragged last tiles in rows and columns, both attention head sizes and ragged key tiles all get
hit by shapes nobody picked by hand."""
import numpy as np
import pytest
import torch

from paper_2509_25188_amd import binding as Bd
from paper_2509_25188_amd import synth
from tests import parity as Pz

pytestmark = pytest.mark.gpu


def draw(seed):
    r = np.random.default_rng(2000 + seed)
    Dh = int(r.choice([64, 128]))
    H = int(r.choice([1, 2, 3, 4, 6, 8]))
    d = H * Dh
    F = 64 * int(r.integers(1, 24))
    V = int(r.integers(130, 3000))
    L = int(r.integers(1, 4))
    T = int(r.choice([int(r.integers(1, 64)), int(r.integers(64, 300)), int(r.integers(300, 900))]))
    B = int(r.integers(1, 4))
    return synth.ModelShape(L, d, H, Dh, F, V, V - 1, V - 2, dtype="bf16"), B, T


@pytest.mark.parametrize("seed", range(20))
def test_random_bf16_shape_forward(seed):
    m, B, T = draw(seed)
    weights = synth.make_weights(m, 40 + seed, "cpu")
    ora = Pz.oracle_model(m, weights)
    eng = Bd.Engine(m, Pz.to_dev(weights), B, T)
    X = synth.make_prompt(60 + seed, B, T, m.vocab - 2, "cpu")
    got = eng.forward(X.cuda()).cpu().numpy()
    worst = 0.0
    for b in range(B):
        ref = ora.forward(X[b].numpy())
        assert got[b].shape == ref.shape
        worst = max(worst, Pz.rel_err(got[b], ref))
    print(f"L={m.n_layers} d={m.d_model} H={m.n_heads}x{m.head_dim} F={m.d_ffn} V={m.vocab} B={B} T={T}: {worst:.2e}")
    assert worst < 2e-2
    # rows of a batch do not interact: a sequence alone gives the same logits as inside the batch
    if B > 1:
        alone = eng.forward(X[B - 1:B].cuda()).cpu().numpy()[0]
        assert Pz.rel_err(alone, got[B - 1]) < 2e-2
