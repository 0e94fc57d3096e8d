"""Pins for the oracle's mask predictor M(X): scalar-loop brute force on tiny inputs,
closed forms and invariants (none of them call the oracle's own array code)."""
import math
import types

import numpy as np
import pytest

from oracle import l2pd_oracle as O


def tiny_shape(L=2, d=8, H=2, Dh=4, F=12, V=11):
    return types.SimpleNamespace(n_layers=L, d_model=d, n_heads=H, head_dim=Dh, d_ffn=F, vocab=V,
                                 mask_id=V - 1, eos_id=V - 2, rope_base=10000.0, rms_eps=1e-5)


def tiny_weights(s, seed=0, scale=0.5):
    r = np.random.default_rng(seed)
    w = {"tok_emb": r.normal(0, scale, (s.vocab, s.d_model)),
         "lm_head": r.normal(0, scale, (s.vocab, s.d_model)),
         "final_norm_g": r.normal(1, 0.1, s.d_model)}
    for l in range(s.n_layers):
        p = f"layers.{l}."
        w[p + "attn_norm_g"] = r.normal(1, 0.1, s.d_model)
        w[p + "ffn_norm_g"] = r.normal(1, 0.1, s.d_model)
        for n in ("wq", "wk", "wv", "wo"):
            w[p + n] = r.normal(0, scale, (s.d_model, s.d_model))
        w[p + "w_gate"] = r.normal(0, scale, (s.d_ffn, s.d_model))
        w[p + "w_up"] = r.normal(0, scale, (s.d_ffn, s.d_model))
        w[p + "w_down"] = r.normal(0, scale, (s.d_model, s.d_ffn))
    return w


# ----------------------------------------------------------------- scalar-loop reference
def bf_norm(x, g, eps):
    ms = sum(v * v for v in x) / len(x)
    return [v / math.sqrt(ms + eps) * gi for v, gi in zip(x, g)]


def bf_matvec(W, x):  # W[out][in]
    return [sum(W[o][i] * x[i] for i in range(len(x))) for o in range(len(W))]


def bf_rope_head(v, t, base):
    dh = len(v)
    half = dh // 2
    out = [0.0] * dh
    for i in range(half):
        a = t * base ** (-2.0 * i / dh)
        out[i] = v[i] * math.cos(a) - v[i + half] * math.sin(a)
        out[i + half] = v[i + half] * math.cos(a) + v[i] * math.sin(a)
    return out


def scalar_bf16(x):
    """Nearest bf16 value of one number (ties to even), through the bits of its float32 form."""
    import struct
    u = struct.unpack("<I", struct.pack("<f", x))[0]
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return struct.unpack("<f", struct.pack("<I", u))[0]


ROUND_POINTS = ("attn_norm", "q", "k", "v", "prob", "attn_out", "ffn_norm", "swiglu", "final_norm")


def bf_forward(s, w, tokens, key_limit=None, pos0=0, round_at=()):
    """Pure-Python forward.  key_limit (optional) restricts every query to keys < key_limit.
    `round_at` names the matrix-product inputs that are rounded to bf16 (any of ROUND_POINTS)."""
    def rnd(name, vec):
        return [scalar_bf16(x) for x in vec] if name in round_at else vec
    T = len(tokens)
    W = {k: np.asarray(v).tolist() for k, v in w.items()}
    h = [list(W["tok_emb"][t]) for t in tokens]
    H, Dh = s.n_heads, s.head_dim
    for l in range(s.n_layers):
        p = f"layers.{l}."
        a = [rnd("attn_norm", bf_norm(h[t], W[p + "attn_norm_g"], s.rms_eps)) for t in range(T)]
        q = [bf_matvec(W[p + "wq"], a[t]) for t in range(T)]
        k = [bf_matvec(W[p + "wk"], a[t]) for t in range(T)]
        v = [bf_matvec(W[p + "wv"], a[t]) for t in range(T)]
        for t in range(T):
            for hh in range(H):
                q[t][hh * Dh:(hh + 1) * Dh] = bf_rope_head(q[t][hh * Dh:(hh + 1) * Dh], pos0 + t, s.rope_base)
                k[t][hh * Dh:(hh + 1) * Dh] = bf_rope_head(k[t][hh * Dh:(hh + 1) * Dh], pos0 + t, s.rope_base)
        q = [rnd("q", r) for r in q]
        k = [rnd("k", r) for r in k]
        v = [rnd("v", r) for r in v]
        o = [[0.0] * (H * Dh) for _ in range(T)]
        nk = T if key_limit is None else key_limit
        for t in range(T):
            for hh in range(H):
                sc = [sum(q[t][hh * Dh + e] * k[u][hh * Dh + e] for e in range(Dh)) / math.sqrt(Dh)
                      for u in range(nk)]
                m = max(sc)
                ex = [math.exp(x - m) for x in sc]
                z = sum(ex)
                pr = rnd("prob", [x / z for x in ex])
                for e in range(Dh):
                    o[t][hh * Dh + e] = sum(pr[u] * v[u][hh * Dh + e] for u in range(nk))
        for t in range(T):
            proj = bf_matvec(W[p + "wo"], rnd("attn_out", o[t]))
            h[t] = [x + y for x, y in zip(h[t], proj)]
        for t in range(T):
            f = rnd("ffn_norm", bf_norm(h[t], W[p + "ffn_norm_g"], s.rms_eps))
            g = bf_matvec(W[p + "w_gate"], f)
            u = bf_matvec(W[p + "w_up"], f)
            act = rnd("swiglu", [gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)])
            dn = bf_matvec(W[p + "w_down"], act)
            h[t] = [x + y for x, y in zip(h[t], dn)]
    return [bf_matvec(W["lm_head"], rnd("final_norm", bf_norm(h[t], W["final_norm_g"], s.rms_eps))) for t in range(T)]


# ----------------------------------------------------------------- tests
def test_forward_matches_scalar_loops_fp64():
    s = tiny_shape()
    w = tiny_weights(s, 1)
    tokens = [3, 0, 7, 10, 2, 5, 10]
    ref = np.array(bf_forward(s, w, tokens))
    got = O.Model(s, w, np.float64).forward(np.array(tokens))
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)
    sub = O.Model(s, w, np.float64).forward(np.array(tokens), 2, 3)
    np.testing.assert_allclose(sub, ref[2:5], rtol=1e-10, atol=1e-12)


def test_forward_fp32_close_to_fp64():
    s = tiny_shape()
    w = tiny_weights(s, 2)
    tokens = np.array([1, 4, 10, 10, 8])
    a = O.Model(s, w, np.float64).forward(tokens)
    b = O.Model(s, {k: v.astype(np.float32) for k, v in w.items()}, np.float32).forward(tokens)
    assert b.dtype == np.float32
    assert np.max(np.abs(a - b)) / np.max(np.abs(a)) < 1e-5


def test_attention_is_bidirectional_uniform_when_queries_vanish():
    # wq = 0 => all scores 0 => every position's attention output is the plain mean of V over
    # ALL positions (earlier and later): closed form for the non-causal softmax.
    s = tiny_shape(L=1)
    w = tiny_weights(s, 3)
    w["layers.0.wq"] = np.zeros_like(w["layers.0.wq"])
    m = O.Model(s, w, np.float64)
    tokens = np.array([2, 9, 4, 1, 6])
    h = m.embed(tokens)
    q, k, v = m.qkv(0, h, np.arange(5))
    o = O.attention(q, k, v)
    for t in range(5):
        np.testing.assert_allclose(o[t], v.mean(axis=0), rtol=1e-12)
    # and a change of the LAST token changes the logits of the FIRST row
    a = m.forward(tokens, 0, 1)
    tokens2 = tokens.copy()
    tokens2[-1] = 3
    assert np.max(np.abs(a - m.forward(tokens2, 0, 1))) > 1e-6


def test_rope_properties():
    r = np.random.default_rng(0)
    x = r.normal(size=(6, 2, 8))
    pos = np.arange(6)
    y = O.rope(x, pos, 10000.0)
    # position 0 is the identity; norms are preserved
    np.testing.assert_allclose(y[0], x[0], rtol=0, atol=0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    # scalar-loop rotation with the (i, i + Dh/2) pairing
    for t in range(6):
        for h in range(2):
            np.testing.assert_allclose(y[t, h], bf_rope_head(x[t, h].tolist(), t, 10000.0), rtol=1e-12, atol=1e-14)
    # scores depend on relative position only
    q, k = r.normal(size=(6, 2, 8)), r.normal(size=(6, 2, 8))
    s0 = np.einsum("qhd,khd->hqk", O.rope(q, pos, 1e4), O.rope(k, pos, 1e4))
    s1 = np.einsum("qhd,khd->hqk", O.rope(q, pos + 37, 1e4), O.rope(k, pos + 37, 1e4))
    np.testing.assert_allclose(s0, s1, rtol=1e-9, atol=1e-10)


def test_rmsnorm_scale_invariance_and_unit_rms():
    r = np.random.default_rng(1)
    x = r.normal(size=(4, 16))
    g = np.ones(16)
    y = O.rmsnorm(x, g, 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(-1)), 1.0, rtol=1e-12)
    np.testing.assert_allclose(O.rmsnorm(7.5 * x, g, 0.0), y, rtol=1e-12)
    np.testing.assert_allclose(O.rmsnorm(x[0], 2 * g, 1e-5), bf_norm(x[0].tolist(), [2.0] * 16, 1e-5), rtol=1e-12)


def test_zero_projections_reduce_to_embedding_head():
    # wo = 0 and w_down = 0 remove both residual branches: logits = norm(E[x]) . W_lm^T
    s = tiny_shape()
    w = tiny_weights(s, 4)
    for l in range(s.n_layers):
        w[f"layers.{l}.wo"][:] = 0
        w[f"layers.{l}.w_down"][:] = 0
    tokens = np.array([5, 10, 0])
    got = O.Model(s, w, np.float64).forward(tokens)
    for t, tok in enumerate(tokens):
        e = w["tok_emb"][tok]
        n = e / math.sqrt(float((e * e).mean()) + s.rms_eps) * w["final_norm_g"]
        for vtok in range(s.vocab):
            assert got[t, vtok] == pytest.approx(float(np.dot(w["lm_head"][vtok], n)), rel=1e-12, abs=1e-14)


def test_bf16_bit_patterns_widen_exactly():
    vals = np.array([1.0, -2.5, 0.0078125, 3.140625], dtype=np.float32)
    bits = (vals.view(np.uint32) >> 16).astype(np.uint16)
    np.testing.assert_array_equal(O.widen(bits, np.float32), vals)
    np.testing.assert_array_equal(O.widen(bits, np.float64), vals.astype(np.float64))


def test_prefix_cache_one_layer_single_block_equals_full():
    # With one layer, K and V depend on the tokens alone, so a cached step over the last block
    # (nothing after it) equals the full bidirectional forward.
    s = tiny_shape(L=1)
    w = tiny_weights(s, 5)
    m = O.Model(s, w, np.float64)
    X = np.array([1, 2, 3, 4, 10, 10, 10])
    cache = m.prefix_kv(X[:4])
    got = m.forward_block_cached(cache, X[4:], 4)
    np.testing.assert_allclose(got, m.forward(X, 4, 3), rtol=1e-10, atol=1e-12)


def test_prefix_cache_step_matches_scalar_loops():
    # Two layers, block in the middle: cached prefix K/V come from the prefix alone, the block
    # sees prefix + itself and nothing after it.  Brute force: prefix forward restricted to the
    # prefix, then the block rows of a forward over X[0:c+s] whose prefix rows are frozen.
    s = tiny_shape(L=2)
    w = tiny_weights(s, 6)
    m = O.Model(s, w, np.float64)
    X = np.array([1, 2, 3, 10, 10, 7, 10, 10, 10])
    c, n = 3, 3
    cache = m.prefix_kv(X[:c])
    got = m.forward_block_cached(cache, X[c:c + n], c)
    ref = bf_forward_cached(s, w, X[:c].tolist(), X[c:c + n].tolist())
    np.testing.assert_allclose(got, np.array(ref), rtol=1e-10, atol=1e-12)
    # one layer, many blocks: cached step == full forward over the truncated sequence
    s1 = tiny_shape(L=1)
    w1 = tiny_weights(s1, 7)
    m1 = O.Model(s1, w1, np.float64)
    got1 = m1.forward_block_cached(m1.prefix_kv(X[:c]), X[c:c + n], c)
    np.testing.assert_allclose(got1, m1.forward(X[:c + n], c, n), rtol=1e-10, atol=1e-12)


def bf_forward_cached(s, w, prefix, block):
    """Scalar loops: hidden states of the prefix evolve seeing the prefix only; block rows see
    prefix keys/values (from that prefix-only run) and their own."""
    W = {k: np.asarray(v).tolist() for k, v in w.items()}
    H, Dh = s.n_heads, s.head_dim
    c = len(prefix)

    def layer_qkv(l, hrows, pos0):
        p = f"layers.{l}."
        out = []
        for t, hr in enumerate(hrows):
            a = bf_norm(hr, W[p + "attn_norm_g"], s.rms_eps)
            q, k, v = bf_matvec(W[p + "wq"], a), bf_matvec(W[p + "wk"], a), bf_matvec(W[p + "wv"], a)
            for hh in range(H):
                q[hh * Dh:(hh + 1) * Dh] = bf_rope_head(q[hh * Dh:(hh + 1) * Dh], pos0 + t, s.rope_base)
                k[hh * Dh:(hh + 1) * Dh] = bf_rope_head(k[hh * Dh:(hh + 1) * Dh], pos0 + t, s.rope_base)
            out.append((q, k, v))
        return out

    def attend(q, keys, vals):
        o = [0.0] * (H * Dh)
        for hh in range(H):
            sc = [sum(q[hh * Dh + e] * kk[hh * Dh + e] for e in range(Dh)) / math.sqrt(Dh) for kk in keys]
            m = max(sc)
            ex = [math.exp(x - m) for x in sc]
            z = sum(ex)
            for e in range(Dh):
                o[hh * Dh + e] = sum(ex[u] / z * vals[u][hh * Dh + e] for u in range(len(keys)))
        return o

    def finish(l, hr, o):
        p = f"layers.{l}."
        hr = [x + y for x, y in zip(hr, bf_matvec(W[p + "wo"], o))]
        f = bf_norm(hr, W[p + "ffn_norm_g"], s.rms_eps)
        g, u = bf_matvec(W[p + "w_gate"], f), bf_matvec(W[p + "w_up"], f)
        act = [gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)]
        return [x + y for x, y in zip(hr, bf_matvec(W[p + "w_down"], act))]

    hp = [list(W["tok_emb"][t]) for t in prefix]
    hb = [list(W["tok_emb"][t]) for t in block]
    for l in range(s.n_layers):
        qp = layer_qkv(l, hp, 0)
        qb = layer_qkv(l, hb, c)
        pk, pv = [x[1] for x in qp], [x[2] for x in qp]
        bk, bv = [x[1] for x in qb], [x[2] for x in qb]
        hp = [finish(l, hp[t], attend(qp[t][0], pk, pv)) for t in range(len(hp))]
        hb = [finish(l, hb[t], attend(qb[t][0], pk + bk, pv + bv)) for t in range(len(hb))]
    return [bf_matvec(W["lm_head"], bf_norm(hr, W["final_norm_g"], s.rms_eps)) for hr in hb]


# ----------------------------------------------------------------- dual cache (Sec. 4.3, Table 2)
def bf_forward_dual(s, w, x_old, x_new_block, c):
    """Scalar loops: per-layer K/V of every position from a full forward over x_old; then the block
    rows are run again on x_new_block, their own K/V replacing the stored ones at c..c+n-1."""
    W = {k: np.asarray(v).tolist() for k, v in w.items()}
    H, Dh = s.n_heads, s.head_dim
    T, n = len(x_old), len(x_new_block)

    def qkv_row(l, hr, t):
        p = f"layers.{l}."
        a = bf_norm(hr, W[p + "attn_norm_g"], s.rms_eps)
        q, k, v = bf_matvec(W[p + "wq"], a), bf_matvec(W[p + "wk"], a), bf_matvec(W[p + "wv"], a)
        for hh in range(H):
            q[hh * Dh:(hh + 1) * Dh] = bf_rope_head(q[hh * Dh:(hh + 1) * Dh], t, s.rope_base)
            k[hh * Dh:(hh + 1) * Dh] = bf_rope_head(k[hh * Dh:(hh + 1) * Dh], t, s.rope_base)
        return q, k, v

    def attend(q, keys, vals):
        o = [0.0] * (H * Dh)
        for hh in range(H):
            sc = [sum(q[hh * Dh + e] * kk[hh * Dh + e] for e in range(Dh)) / math.sqrt(Dh) for kk in keys]
            m = max(sc)
            ex = [math.exp(x - m) for x in sc]
            z = sum(ex)
            for e in range(Dh):
                o[hh * Dh + e] = sum(ex[u] / z * vals[u][hh * Dh + e] for u in range(len(keys)))
        return o

    def finish(l, hr, o):
        p = f"layers.{l}."
        hr = [x + y for x, y in zip(hr, bf_matvec(W[p + "wo"], o))]
        f = bf_norm(hr, W[p + "ffn_norm_g"], s.rms_eps)
        g, u = bf_matvec(W[p + "w_gate"], f), bf_matvec(W[p + "w_up"], f)
        act = [gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)]
        return [x + y for x, y in zip(hr, bf_matvec(W[p + "w_down"], act))]

    # pass 1: full forward over x_old, remembering every layer's K, V
    h = [list(W["tok_emb"][t]) for t in x_old]
    stored = []
    for l in range(s.n_layers):
        rows = [qkv_row(l, h[t], t) for t in range(T)]
        ks, vs = [r[1] for r in rows], [r[2] for r in rows]
        stored.append((ks, vs))
        h = [finish(l, h[t], attend(rows[t][0], ks, vs)) for t in range(T)]
    # pass 2: the block alone
    hb = [list(W["tok_emb"][t]) for t in x_new_block]
    for l in range(s.n_layers):
        rows = [qkv_row(l, hb[j], c + j) for j in range(n)]
        ks, vs = [list(r) for r in stored[l][0]], [list(r) for r in stored[l][1]]
        for j in range(n):
            ks[c + j], vs[c + j] = rows[j][1], rows[j][2]
        hb = [finish(l, hb[j], attend(rows[j][0], ks, vs)) for j in range(n)]
    return [bf_matvec(W["lm_head"], bf_norm(hr, W["final_norm_g"], s.rms_eps)) for hr in hb]


def test_dual_cache_first_step_equals_full_forward():
    # Right after the refresh nothing is stale: the block's fresh K/V equal the stored ones.
    s = tiny_shape(L=3)
    w = tiny_weights(s, 11)
    m = O.Model(s, w, np.float64)
    X = np.array([1, 2, 3, 10, 7, 10, 10, 10, 10])
    c, n = 3, 3
    got = m.forward_block_dual(m.full_kv(X), X[c:c + n], c)
    np.testing.assert_allclose(got, m.forward(X, c, n), rtol=1e-9, atol=1e-11)


def test_dual_cache_one_layer_is_exact_at_every_step():
    # With one layer K and V of a position depend on its token alone, so stored entries outside
    # the block never go stale: the cached step equals the full forward on the updated sequence.
    s = tiny_shape(L=1)
    w = tiny_weights(s, 12)
    m = O.Model(s, w, np.float64)
    X = np.array([1, 2, 3, 10, 10, 10, 10, 10, 10])
    c, n = 3, 3
    cache = m.full_kv(X)
    X2 = X.copy()
    X2[c:c + n] = [5, 10, 0]
    got = m.forward_block_dual(cache, X2[c:c + n], c)
    np.testing.assert_allclose(got, m.forward(X2, c, n), rtol=1e-10, atol=1e-12)


def test_dual_cache_stale_step_matches_scalar_loops():
    # Two layers, block in the middle, block tokens changed after the refresh: the stored K/V of
    # the other positions are those of the OLD sequence.  Also: the positions after the block are
    # attended to (unlike the prefix cache), and the result is not the full forward's.
    s = tiny_shape(L=2)
    w = tiny_weights(s, 13)
    m = O.Model(s, w, np.float64)
    X = np.array([1, 2, 3, 10, 10, 10, 10, 6, 10])
    c, n = 3, 3
    cache = m.full_kv(X)
    newb = [4, 10, 8]
    got = m.forward_block_dual(cache, np.array(newb), c)
    ref = bf_forward_dual(s, w, X.tolist(), newb, c)
    np.testing.assert_allclose(got, np.array(ref), rtol=1e-10, atol=1e-12)
    X2 = X.copy()
    X2[c:c + n] = newb
    assert np.max(np.abs(got - m.forward(X2, c, n))) > 1e-6          # stale on purpose
    Xs = X.copy()
    Xs[7] = 9                                                          # a token after the block
    other = m.forward_block_dual(m.full_kv(Xs), np.array(newb), c)
    assert np.max(np.abs(other - got)) > 1e-6                         # the suffix is visible


def test_round_bf16_matches_the_library_conversion_and_ties_to_even():
    import torch
    r = np.random.default_rng(3)
    x = np.concatenate([r.normal(size=5000) * 10.0 ** r.integers(-6, 6, 5000), [0.0, -0.0, 1.0, 65504.0]]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(O.round_bf16(x), ref)
    # 1 + 2^-8 is halfway between bf16 neighbours 1 and 1 + 2^-7: ties go to the even mantissa
    assert O.round_bf16(np.array([1.0 + 2.0 ** -8], dtype=np.float32))[0] == 1.0
    assert O.round_bf16(np.array([1.0 + 3 * 2.0 ** -8], dtype=np.float32))[0] == np.float32(1.0 + 2.0 ** -6)
    assert O.round_bf16(np.array([0.5, 2.0], dtype=np.float64)).dtype == np.float64


def test_bf16_gemm_inputs_stay_close_to_full_precision():
    s = tiny_shape()
    w = {k: v.astype(np.float32) for k, v in tiny_weights(s, 8).items()}
    tokens = np.array([1, 4, 10, 10, 8, 2])
    a = O.Model(s, w, np.float32).forward(tokens)
    b = O.Model(s, w, np.float32, gemm_input="bf16").forward(tokens)
    e = np.max(np.abs(a - b)) / np.max(np.abs(a))
    assert 1e-5 < e < 3e-2          # rounding is present, and of the size of bf16's 2^-9 steps


def test_bf16_gemm_inputs_are_rounded_exactly_where_stated():
    """The bf16-input mode against scalar loops that round, one number at a time, at the named points:
    the normalised activations of both half-layers and of the head, the rotated queries and keys, the
    values, the softmax probabilities, the attention output and the SwiGLU output.  Leaving any one of
    them unrounded (or rounding none) must move the result away from the oracle's."""
    s = tiny_shape()
    w = {k: np.asarray([[scalar_bf16(x) for x in row] for row in np.atleast_2d(v)]).reshape(np.shape(v))
         for k, v in tiny_weights(s, 8).items()}                        # bf16-representable weights
    tokens = [1, 4, 10, 10, 8, 2]
    got = O.Model(s, w, np.float64, gemm_input="bf16").forward(np.array(tokens))
    ref = np.array(bf_forward(s, w, tokens, round_at=ROUND_POINTS))
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-12)
    scale = np.max(np.abs(ref))
    for left_out in ROUND_POINTS:
        other = np.array(bf_forward(s, w, tokens, round_at=tuple(p for p in ROUND_POINTS if p != left_out)))
        assert np.max(np.abs(other - got)) > 1e-5 * scale, left_out
    assert np.max(np.abs(np.array(bf_forward(s, w, tokens)) - got)) > 1e-4 * scale


def test_filter_training_in_float32_tracks_float64():
    """The trainer's precision switch: the float32 run starts on the float64 loss curve and stays near it
    on a well-conditioned problem."""
    r = np.random.default_rng(5)
    C = r.uniform(size=(120, 8))
    Y = (r.uniform(size=(120, 8)) < 0.2 + 0.6 * C).astype(np.float64)
    flt = {"w1": r.normal(0, 0.4, (6, 8)), "b1": r.normal(0, 1, 6), "w2": r.normal(0, 0.4, (8, 6)), "b2": r.normal(0, 1, 8)}
    th64, l64 = O.train_filter(flt, C, Y, 50, lr=1e-2)
    th32, l32 = O.train_filter(flt, C, Y, 50, lr=1e-2, dtype=np.float32)
    assert all(v.dtype == np.float32 for v in th32.values()) and all(v.dtype == np.float64 for v in th64.values())
    np.testing.assert_allclose(l32, l64, rtol=1e-4)
    assert abs(l32[0] - l64[0]) < 1e-6 and l64[-1] < l64[0]
