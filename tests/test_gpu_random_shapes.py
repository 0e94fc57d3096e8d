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


# Widths from 2048 up take the tiles that read their A operand into registers from quad-tiled activations
# (256 x 96 for Q/K/V, 256 x 192 for gate/up, 256 x 128 with K split four ways for the output and down
# projections where K is a multiple of 1024); the 8B-width tests cover one shape of them.  Others by hand:
# both head sizes, gate/up columns that no tile divides, depths that do and do not allow the four-way split,
# row counts that no tile divides, a batch whose row groups straddle sequences.
WIDE = [
    # (d, H, Dh, F, V, B, T)
    (2048, 32, 64, 4096, 1500, 1, 300),     # head size 64; O and down both split four ways
    (2048, 16, 128, 5632, 1100, 2, 261),    # F = 5.5 x 1024: down takes 128 x 128 tiles and a row-major act; 522 rows
    (2560, 20, 128, 6400, 900, 1, 515),     # K = 2560 for Q/K/V and gate/up; 12800 gate/up columns (66.7 tiles of 192)
    (3072, 24, 128, 3072, 700, 3, 171),     # three sequences of 171 rows: 513 rows, quads straddle sequences
]


@pytest.mark.parametrize("case", range(len(WIDE)))
def test_wide_bf16_shape_forward(case):
    d, H, Dh, F, V, B, T = WIDE[case]
    m = synth.ModelShape(1, d, H, Dh, F, V, V - 1, V - 2, dtype="bf16")
    weights = synth.make_weights(m, 140 + case, "cpu")
    ora = Pz.oracle_model(m, weights, gemm_input="bf16")
    eng = Bd.Engine(m, Pz.to_dev(weights), B, T)
    X = synth.make_prompt(160 + case, B, T, m.vocab - 2, "cpu")
    got = eng.forward(X.cuda()).cpu().numpy()
    again = eng.forward(X.cuda()).cpu().numpy()
    np.testing.assert_array_equal(got, again)                     # bit-reproducible
    worst = max(Pz.rel_err(got[b], ora.forward(X[b].numpy())) for b in range(B))
    print(f"d={d} H={H}x{Dh} F={F} V={V} B={B} T={T}: {worst:.2e}")
    assert worst < 2e-2
    if B > 1:
        # more than 256 rows in the batch, fewer in one sequence: other tiles, same arithmetic up to the split depth
        alone = eng.forward(X[B - 1:B].cuda()).cpu().numpy()[0]
        assert Pz.rel_err(alone, got[B - 1]) < 2e-2


def draw_step(seed):
    r = np.random.default_rng(3000 + seed)
    Dh = int(r.choice([64, 128]))
    H = int(r.choice([1, 2, 4]))
    m = synth.ModelShape(2, H * Dh, H, Dh, 64 * int(r.integers(2, 12)), int(r.integers(200, 2500)), 0, 0, dtype="bf16")
    m = synth.ModelShape(m.n_layers, m.d_model, H, Dh, m.d_ffn, m.vocab, m.vocab - 1, m.vocab - 2, dtype="bf16")
    s = int(r.choice([8, 16, 32, 64]))
    nb = int(r.integers(1, 5))
    cache = int(r.integers(0, 3))
    w = synth.Workload(f"rs{seed}", m, int(r.integers(1, 4)), int(r.integers(1, 200)), s * nb, s, int(r.choice([16, 64])),
                       float(r.choice([0.3, 0.6])), prefix_cache=cache == 1, dual_cache=cache == 2,
                       bias_from=int(r.integers(0, s * nb)), bias_value=float(r.choice([0.0, 4.0])),
                       prompt_hi=m.vocab - 2)
    return w, int(r.integers(0, nb)), int(r.integers(1, 5))


@pytest.mark.parametrize("seed", range(20))
def test_random_bf16_shape_denoise_step(seed):
    # one teacher-forced step of every sequence of a batch, all in the same block (lock step), each with
    # its own number of committed positions; cached modes rebuild their store from the given tokens first
    w, block, depth = draw_step(seed)
    weights = synth.make_weights(w.model, 90 + seed, "cpu", lm_head_scale=8.0)
    ora = Pz.oracle_model(w.model, weights, gemm_input="bf16")     # the arithmetic under test
    alt = Pz.oracle_model(w.model, weights)                         # float32 activations: defines the resolution D
    eng = Bd.Engine(w.model, Pz.to_dev(weights), w.batch, w.prompt_len + w.gen_len, w.prefix_cache or w.dual_cache)
    flt = synth.make_filter(70 + seed, w.block_len, w.filter_hidden, "cpu", n_layers=depth)
    fdev = {k: v.cuda() for k, v in flt.items()}
    r = np.random.default_rng(4000 + seed)
    X = np.stack([Pz.random_state(w, 100 * seed + b, block, int(r.integers(0, w.block_len)), b) for b in range(w.batch)])
    recs = [Pz.oracle_step_record(ora, X[b], w, Pz.np_filter(flt), block, alt=alt) for b in range(w.batch)]
    Xd = torch.tensor(X, dtype=torch.int32, device="cuda")
    state = torch.tensor([[block, 3, 0]] * w.batch, dtype=torch.int32, device="cuda")
    taps = eng.denoise_step(Xd, w.prompt_len, state, fdev, Pz.cfg_for(w), want_logits=True)
    torch.cuda.synchronize()
    rep = Pz.StepReport()
    for b in range(w.batch):
        Pz.check_step(recs[b], taps, b, w.model, w.threshold, Pz.tol_for(w.model), rep)
    m = w.model
    print(f"d={m.d_model} H={m.n_heads}x{m.head_dim} F={m.d_ffn} V={m.vocab} B={w.batch} P={w.prompt_len} G={w.gen_len} "
          f"s={w.block_len} block={block} cache={'prefix' if w.prefix_cache else 'dual' if w.dual_cache else 'none'} "
          f"depth={depth}: {rep}")
    assert rep.steps == w.batch and rep.max_logit_err < 2e-2
    assert rep.exempt_tokens + rep.exempt_decisions <= max(4, 0.06 * rep.positions), rep
