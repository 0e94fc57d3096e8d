"""Pins for the oracle's decode rule: Eq. 3 / Eq. 4 closed forms, the filter, Alg. 2 invariants
and special cases, Alg. 3 (EoTP) stopping, and the values the paper prints."""
import math
import os
import re
import types

import numpy as np
import pytest

from oracle import l2pd_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        m = re.match(r"\s*(\w+)\s*=\s*([-\d.]+)", line)
        if m:
            out[m.group(1)] = float(m.group(2))
    return out


class ScriptedModel:
    """Stands in for M(X): logits depend on the position only (a fixed table)."""

    def __init__(self, table, prompt_len):
        self.table = table          # [gen_len, V]
        self.P = prompt_len
        self.calls = 0

    def forward(self, X, lo, n):
        self.calls += 1
        return self.table[lo - self.P: lo - self.P + n].copy()


def pass_all_filter(s, h=4, z=+50.0):
    return dict(w1=np.zeros((h, s)), b1=np.zeros(h), w2=np.zeros((s, h)), b2=np.full(s, z))


# ----------------------------------------------------------------- Eq. 3 / Eq. 4
def test_conf_uniform_logits_closed_form():
    V, mask = 50, 49
    conf, pre = O.conf_pre(np.zeros((3, V)), mask)
    assert list(pre) == [0, 0, 0]                       # lowest id wins ties
    np.testing.assert_allclose(conf, 1.0 / (V - 1), rtol=1e-14)  # mask id is not a data token


def test_conf_one_raised_logit_closed_form():
    V, mask, beta = 40, 7, 2.5
    z = np.zeros((1, V))
    z[0, 11] = beta
    z[0, mask] = 99.0                                   # must be ignored, however large
    conf, pre = O.conf_pre(z, mask)
    assert pre[0] == 11
    assert conf[0] == pytest.approx(math.exp(beta) / (math.exp(beta) + V - 2), rel=1e-13)


def test_conf_is_max_probability_bruteforce():
    r = np.random.default_rng(0)
    V, mask = 23, 22
    z = r.normal(size=(5, V)) * 3
    conf, pre = O.conf_pre(z, mask)
    for j in range(5):
        ex = [math.exp(z[j, v]) for v in range(V) if v != mask]
        probs = [e / sum(ex) for e in ex]
        assert pre[j] == int(np.argmax(probs))
        assert conf[j] == pytest.approx(max(probs), rel=1e-12)


# ----------------------------------------------------------------- filter
def test_filter_hand_example():
    # c = (0.2, 0.9); W1 = [[1, -1], [2, 0]], b1 = (0.5, -1); hidden pre-act = (-0.2, -0.6) -> relu (0, 0)
    # second example c = (0.9, 0.2): pre-act = (1.2, 0.8) -> W2 = [[1, 1], [-2, 0.5]], b2 = (0, 1)
    #   z = (2.0, -2.4 + 0.4 + 1) = (2.0, -1.0)
    flt = dict(w1=np.array([[1., -1.], [2., 0.]]), b1=np.array([0.5, -1.]),
               w2=np.array([[1., 1.], [-2., 0.5]]), b2=np.array([0., 1.]))
    p = O.filter_prob(np.array([0.2, 0.9]), flt)
    np.testing.assert_allclose(p, [0.5, 1 / (1 + math.exp(-1.0))], rtol=1e-14)
    p = O.filter_prob(np.array([0.9, 0.2]), flt)
    np.testing.assert_allclose(p, [1 / (1 + math.exp(-2.0)), 1 / (1 + math.exp(1.0))], rtol=1e-14)


def test_filter_param_count_matches_paper():
    g = golden()
    assert O.filter_param_count(32, 32) == int(g["filter_params_block32"])
    # the depth variants of Table 3 at the same widths: one 32x32 layer with its bias, and four
    assert O.filter_param_count(32, 32, 1) == 32 * 32 + 32
    assert O.filter_param_count(32, 32, 4) == 2 * int(g["filter_params_block32"])


def deep_filter(s, h, n_layers, seed):
    r = np.random.default_rng(seed)
    dims = [s] + [h] * (n_layers - 1) + [s]
    f = {}
    for k in range(n_layers):
        f[f"w{k + 1}"] = r.normal(size=(dims[k + 1], dims[k]))
        f[f"b{k + 1}"] = r.normal(size=dims[k + 1])
    return f


def test_filter_depth_variants_reduce_to_the_two_layer_filter():
    # confidences are >= 0, so a first layer (I, 0) passes them through its ReLU unchanged: the
    # single-layer filter (W, b) equals the two-layer filter (I, 0, W, b)
    r = np.random.default_rng(61)
    s = 6
    c = r.uniform(size=s)
    one = deep_filter(s, s, 1, 62)
    two = dict(w1=np.eye(s), b1=np.zeros(s), w2=one["w1"], b2=one["b1"])
    np.testing.assert_allclose(O.filter_prob(c, one), O.filter_prob(c, two), rtol=1e-14)
    # hidden activations are >= 0 as well: identity layers in the middle of a four-layer filter
    # leave the two-layer filter around them
    h = 5
    base = deep_filter(s, h, 2, 63)
    four = dict(w1=base["w1"], b1=base["b1"], w2=np.eye(h), b2=np.zeros(h), w3=np.eye(h), b3=np.zeros(h),
                w4=base["w2"], b4=base["b2"])
    np.testing.assert_allclose(O.filter_prob(c, four), O.filter_prob(c, base), rtol=1e-14)
    # and a generic four-layer filter against scalar loops
    f4 = deep_filter(s, h, 4, 64)
    a = list(c)
    for k in (1, 2, 3):
        w, b = f4[f"w{k}"], f4[f"b{k}"]
        a = [max(0.0, b[i] + sum(w[i][j] * a[j] for j in range(len(a)))) for i in range(len(b))]
    z = [f4["b4"][i] + sum(f4["w4"][i][j] * a[j] for j in range(h)) for i in range(s)]
    np.testing.assert_allclose(O.filter_prob(c, f4), [1 / (1 + math.exp(-v)) for v in z], rtol=1e-13)


# ----------------------------------------------------------------- Alg. 2 invariants and special cases
def run(table, P, G, s, flt, tau, mask, eos, **kw):
    m = ScriptedModel(table, P)
    trace = []
    out = O.generate(m, np.arange(P) % 5, G, s, mask, eos, flt, tau, trace=trace, **kw)
    return out, trace, m


def rand_table(G, V, seed):
    return np.random.default_rng(seed).normal(size=(G, V)) * 2.0


def test_tau_ge_one_is_one_token_per_step_in_confidence_order():
    g = golden()
    P, G, s, V = 3, 64, 32, 30
    mask, eos = V - 1, V - 2
    table = rand_table(G, V, 1)
    table[:, eos] = -30.0
    flt = dict(w1=np.random.default_rng(2).normal(size=(8, s)), b1=np.zeros(8),
               w2=np.random.default_rng(3).normal(size=(s, 8)), b2=np.zeros(s))
    (resp, steps, dlen), trace, m = run(table, P, G, s, flt, 1.0, mask, eos)
    assert steps == G == m.calls and dlen == G
    assert steps // (G // s) == int(g["vanilla_decodings_per_block32"])   # 32 decodings per block of 32
    conf, pre = O.conf_pre(table, mask)
    np.testing.assert_array_equal(resp, pre)
    for b in range(G // s):
        order = [int(np.nonzero(t["sel"])[0][0]) for t in trace if t["block"] == b]
        assert all(int(t["sel"].sum()) == 1 for t in trace)
        expect = sorted(range(s), key=lambda j: (-conf[b * s + j], j))
        assert order == expect                       # = one-token-per-step low-confidence remasking


def test_negative_tau_is_one_step_per_block():
    P, G, s, V = 2, 96, 32, 20
    table = rand_table(G, V, 4)
    table[:, V - 2] = -30.0
    flt = dict(w1=np.zeros((4, s)), b1=np.zeros(4), w2=np.zeros((s, 4)), b2=np.zeros(s))
    (resp, steps, dlen), trace, _ = run(table, P, G, s, flt, -0.1, V - 1, V - 2)
    assert steps == G // s
    assert all(t["sel"].all() for t in trace)


def test_strict_threshold_compare():
    # sigmoid(0) = 0.5 exactly; tau = 0.5 must NOT pass (strict >), so only the forced top-1 goes.
    P, G, s, V = 1, 8, 8, 12
    table = rand_table(G, V, 5)
    table[:, V - 2] = -30.0
    flt = dict(w1=np.zeros((2, s)), b1=np.zeros(2), w2=np.zeros((s, 2)), b2=np.zeros(s))
    (_, steps, _), trace, _ = run(table, P, G, s, flt, 0.5, V - 1, V - 2)
    assert np.all(trace[0]["p"] == 0.5)
    assert steps == G
    (_, steps, _), _, _ = run(table, P, G, s, flt, 0.4999, V - 1, V - 2)
    assert steps == 1


def test_never_remask_and_step_bounds():
    P, G, s, V = 4, 64, 16, 25
    mask, eos = V - 1, V - 2
    table = rand_table(G, V, 6) * 2
    table[:, eos] = -30.0
    r = np.random.default_rng(7)
    flt = dict(w1=r.normal(size=(8, s)), b1=r.normal(size=8), w2=r.normal(size=(s, 8)), b2=r.normal(size=s))
    (resp, steps, dlen), trace, _ = run(table, P, G, s, flt, 0.6, mask, eos)
    assert G // s <= steps <= G
    assert not np.any(resp == mask)
    per_block = {}
    for t in trace:
        per_block[t["block"]] = per_block.get(t["block"], 0) + 1
        before = t["X_before"]
        assert t["sel"].sum() >= 1                      # progress every step
        assert np.all(t["masked"][t["sel"]])            # only masked positions are unmasked
    assert max(per_block.values()) <= s
    for a, b in zip(trace[:-1], trace[1:]):
        was = a["X_before"] != mask
        assert np.all(b["X_before"][was] == a["X_before"][was])   # committed tokens never change
    # committed positions feed the filter the constant 1.0: check through a filter that copies its input
    ident = dict(w1=np.eye(s), b1=np.zeros(s), w2=np.eye(s), b2=np.zeros(s))
    (_, _, _), tr2, _ = run(table, P, G, s, ident, 2.0, mask, eos)
    for t in tr2:
        expect = np.where(t["masked"], t["conf"], 1.0)
        np.testing.assert_allclose(t["p"], 1 / (1 + np.exp(-expect)), rtol=1e-12)


def test_identity_filter_is_fixed_confidence_threshold_decoding():
    # W1 = I, W2 = k I: p_j = sigmoid(k c_j) which is monotone in c_j, so p_j > sigmoid(k c*) <=> c_j > c*.
    P, G, s, V = 2, 32, 16, 6
    mask, eos = V - 1, V - 2
    table = rand_table(G, V, 8) * 3
    table[:, eos] = -30.0
    k, cstar = 4.0, 0.55
    flt = dict(w1=np.eye(s), b1=np.zeros(s), w2=k * np.eye(s), b2=np.zeros(s))
    tau = 1 / (1 + math.exp(-k * cstar))
    (_, _, _), trace, _ = run(table, P, G, s, flt, tau, mask, eos)
    saw_parallel = False
    for t in trace:
        want = t["masked"] & (t["conf"] > cstar)
        top = int(np.argmax(np.where(t["masked"], t["conf"], -np.inf)))
        want[top] = True
        np.testing.assert_array_equal(t["sel"], want)
        saw_parallel |= want.sum() > 1
    assert saw_parallel


def test_forced_top1_lowest_index_on_ties():
    P, G, s, V = 1, 4, 4, 5
    table = np.zeros((G, V))                            # every position has the same confidence
    flt = dict(w1=np.zeros((2, s)), b1=np.zeros(2), w2=np.zeros((s, 2)), b2=np.full(s, -50.0))
    (_, steps, _), trace, _ = run(table, P, G, s, flt, 0.5, V - 1, V - 2)
    assert [int(np.nonzero(t["sel"])[0][0]) for t in trace] == [0, 1, 2, 3]


# ----------------------------------------------------------------- Alg. 3 (EoTP)
def test_eotp_stops_after_the_block_that_contains_eos():
    P, G, s, V = 3, 128, 16, 40
    mask, eos = V - 1, V - 2
    table = rand_table(G, V, 9)
    table[:, eos] = -30.0
    g0 = 53
    flt = dict(w1=np.zeros((2, s)), b1=np.zeros(2), w2=np.zeros((s, 2)), b2=np.full(s, -50.0))
    bias = (eos, g0, 60.0)
    (r_on, st_on, dl_on), _, _ = run(table, P, G, s, flt, 1.0, mask, eos, eotp=True, bias=bias)
    (r_off, st_off, dl_off), _, _ = run(table, P, G, s, flt, 1.0, mask, eos, eotp=False, bias=bias)
    nb = g0 // s + 1
    assert st_on == nb * s and dl_on == nb * s
    assert st_off == G and dl_off == G
    np.testing.assert_array_equal(r_on[:dl_on], r_off[:dl_on])
    assert np.all(r_on[dl_on:] == mask)                 # the undecoded tail keeps the mask id
    assert np.all(r_on[g0:dl_on] == eos) and not np.any(r_on[:g0] == eos)
    assert O.tail_all_eos(r_on, eos, dl_on)
    # stopping exactly at the first block whose end is reached with an EOS present
    first = int(np.nonzero(r_off == eos)[0][0])
    assert dl_on == (first // s + 1) * s


def test_eotp_without_eos_equals_off_and_prompt_eos_is_ignored():
    P, G, s, V = 3, 48, 16, 30
    mask, eos = V - 1, V - 2
    table = rand_table(G, V, 10)
    table[:, eos] = -30.0
    flt = pass_all_filter(s)
    m1, m2 = ScriptedModel(table, P), ScriptedModel(table, P)
    prompt = np.array([eos, 1, eos])                    # EOS in the prompt must not stop decoding
    a = O.generate(m1, prompt, G, s, mask, eos, flt, 0.5, eotp=True)
    b = O.generate(m2, prompt, G, s, mask, eos, flt, 0.5, eotp=False)
    np.testing.assert_array_equal(a[0], b[0])
    assert a[1:] == b[1:] == (G // s, G)


def test_bias_hook_positions():
    z = np.zeros((4, 6))
    out = O.apply_bias(z, 10, (2, 12, 5.0))
    assert out[:, 2].tolist() == [0, 0, 5.0, 5.0] and out.sum() == 10.0
    assert O.apply_bias(z, 10, None) is z


def test_untrained_filter_bce_is_ln2():
    # Eq. 6 with sigma(z) = 0.5 for every label is ln 2 ~ 0.69: the level the paper's curve starts at.
    g = golden()
    p = O.sigmoid(np.zeros(8))
    y = np.array([0, 1, 1, 0, 1, 0, 0, 1.0])
    bce = -np.mean(y * np.log(p) + (1 - y) * np.log(1 - p))
    assert bce == pytest.approx(math.log(2), rel=1e-12)
    assert abs(bce - g["bce_initial_loss_approx"]) < 0.02


# ----------------------------------------------------------------- prefix-cache decode on a real (tiny) model
def test_generate_with_prefix_cache_one_layer_equals_truncated_full_recompute():
    from tests.test_oracle_model import tiny_shape, tiny_weights
    s = tiny_shape(L=1, V=13)
    w = tiny_weights(s, 11, scale=1.0)
    m = O.Model(s, w, np.float64)
    r = np.random.default_rng(12)
    flt = dict(w1=r.normal(size=(4, 4)), b1=r.normal(size=4), w2=r.normal(size=(4, 4)), b2=r.normal(size=4))
    prompt = np.array([1, 5, 2])
    trace = []
    resp, steps, dl = O.generate(m, prompt, 8, 4, s.mask_id, s.eos_id, flt, 0.6, prefix_cache=True, trace=trace)
    assert not np.any(resp == s.mask_id) and 2 <= steps <= 8
    for t in trace:
        lo = 3 + t["block"] * 4
        ref = m.forward(t["X_before"][:lo + 4], lo, 4)  # later blocks invisible
        np.testing.assert_allclose(t["logits"], ref, rtol=1e-9, atol=1e-11)


# ----------------------------------------------------------------- dual-cache decode on a real (tiny) model
def test_generate_with_dual_cache_one_layer_equals_full_recompute():
    # One layer: stored K/V never go stale, so the dual-cache trajectory is the full-recompute one.
    from tests.test_oracle_model import tiny_shape, tiny_weights
    s = tiny_shape(L=1, V=13)
    w = tiny_weights(s, 21, scale=1.0)
    m = O.Model(s, w, np.float64)
    r = np.random.default_rng(22)
    flt = dict(w1=r.normal(size=(4, 4)), b1=r.normal(size=4), w2=r.normal(size=(4, 4)), b2=r.normal(size=4))
    prompt = np.array([1, 5, 2])
    full = O.generate(m, prompt, 12, 4, s.mask_id, s.eos_id, flt, 0.6)
    dual = O.generate(m, prompt, 12, 4, s.mask_id, s.eos_id, flt, 0.6, dual_cache=True)
    np.testing.assert_array_equal(full[0], dual[0])
    assert full[1:] == dual[1:]


def test_generate_with_dual_cache_first_step_of_each_block_is_the_full_forward():
    # Several layers: the first step after every refresh sees nothing stale and must reproduce the
    # full bidirectional forward on that state; later steps of a block may not.
    from tests.test_oracle_model import tiny_shape, tiny_weights
    s = tiny_shape(L=3, V=13)
    w = tiny_weights(s, 23, scale=1.0)
    m = O.Model(s, w, np.float64)
    r = np.random.default_rng(24)
    flt = dict(w1=r.normal(size=(4, 4)), b1=r.normal(size=4), w2=r.normal(size=(4, 4)), b2=r.normal(size=4))
    prompt = np.array([3, 0, 7, 4])
    trace = []
    resp, steps, dl = O.generate(m, prompt, 12, 4, s.mask_id, s.eos_id, flt, 2.0, dual_cache=True, trace=trace)
    assert not np.any(resp == s.mask_id) and steps == 12 and dl == 12     # tau > 1: one token per step
    seen, stale = set(), 0
    for t in trace:
        lo = 4 + t["block"] * 4
        ref = m.forward(t["X_before"], lo, 4)
        if t["block"] not in seen:
            seen.add(t["block"])
            np.testing.assert_allclose(t["logits"], ref, rtol=1e-9, atol=1e-11)
        elif np.max(np.abs(t["logits"] - ref)) > 1e-6:
            stale += 1
    assert seen == {0, 1, 2} and stale > 0


# ----------------------------------------------------------------- Sec. 3.3: step-granular EoTP
class LengthRecordingModel(ScriptedModel):
    """ScriptedModel that also records the length of every sequence it is given."""

    def __init__(self, table, prompt_len):
        super().__init__(table, prompt_len)
        self.lengths = []

    def forward(self, X, lo, n):
        self.lengths.append(len(X))
        return super().forward(X, lo, n)


def test_step_eotp_without_eot_equals_plain_decoding():
    P, G, s, V = 3, 48, 16, 30
    mask, eos = V - 1, V - 2
    table = rand_table(G, V, 31)
    table[:, eos] = -30.0
    flt = pass_all_filter(s)
    a = O.generate_eotp_step(ScriptedModel(table, P), np.arange(P), G, s, mask, eos, flt, 0.5)
    b = O.generate(ScriptedModel(table, P), np.arange(P), G, s, mask, eos, flt, 0.5)
    np.testing.assert_array_equal(a[0], b[0])
    assert a[1:] == b[1:]


def test_step_eotp_discards_after_the_first_eot_and_shortens_the_next_input():
    # One token per step in order of confidence (tau = 1, "never" filter).  Block 1 = generation
    # positions 16..31; end-of-text is the greedy token at 21, 24 and 27.  Confidence order inside the
    # block is fixed by the raised logit: position 24 first, then 18, 21, 16, ... so that the
    # truncation happens twice (first at 24, then at 21) with masked positions left before it.
    P, G, s, V = 4, 64, 16, 12
    mask, eos = V - 1, V - 2
    table = np.zeros((G, V))
    for g in range(G):
        table[g, g % 7] = 3.0                       # greedy token, moderate confidence
    order = [24, 18, 21, 16, 17, 19, 20, 22, 23, 25]
    for rank, g in enumerate(order):
        table[g, g % 7] = 0.0
        tok = eos if g in (21, 24, 27) else g % 7
        table[g, tok] = 12.0 - rank                  # decreasing confidence in this order
    table[27, :] = 0.0
    table[27, eos] = 1.0                             # would be end-of-text too, but is discarded first
    never = dict(w1=np.zeros((2, s)), b1=np.zeros(2), w2=np.zeros((s, 2)), b2=np.full(s, -50.0))
    m = LengthRecordingModel(table, P)
    trace = []
    resp, steps, dl = O.generate_eotp_step(m, np.arange(P), G, s, mask, eos, never, 1.0, trace=trace)
    T = P + G
    # block 0: 16 steps on the full length; block 1: step 1 commits 24 (EoT) -> length P+25;
    # step 2 commits 18; step 3 commits 21 (EoT) -> length P+22; then 16, 17, 19, 20 remain: 4 steps
    assert m.lengths[:17] == [T] * 17
    assert m.lengths[17:19] == [P + 25] * 2
    assert m.lengths[19:] == [P + 22] * 4
    assert steps == 16 + 3 + 4 and dl == 22
    assert resp[21] == eos and not np.any(resp[:21] == eos)
    assert np.all(resp[22:] == mask) and not np.any(resp[:22] == mask)
    # the rows predicted shrink with the sequence: 16, then 9 (16..24), then 6 (16..21)
    assert [t["n"] for t in trace[16:]] == [16, 9, 9, 6, 6, 6, 6]
    # block-granular Alg. 3 on the same table decodes the whole block and keeps positions after the EoT
    r3, st3, dl3 = O.generate(ScriptedModel(table, P), np.arange(P), G, s, mask, eos, never, 1.0, eotp=True)
    assert st3 == 32 and dl3 == 32
    np.testing.assert_array_equal(r3[:22], resp[:22])


def test_step_eotp_discarded_positions_feed_the_filter_one():
    # A filter that passes position 0 only if the LAST input is >= 0.99: with the block shortened
    # to one live position (the rest discarded), that input is the constant 1.0 of a discarded slot.
    P, G, s, V = 2, 8, 4, 9
    mask, eos = V - 1, V - 2
    table = np.zeros((G, V))
    table[0, 3] = 0.5                                # low confidence at generation position 0
    table[1, eos] = 9.0                              # end-of-text, unmasked first (highest confidence)
    table[2, 2] = 1.0
    table[3, 1] = 1.0
    flt = dict(w1=np.array([[0.0, 0.0, 0.0, 100.0]]), b1=np.array([-99.0]),
               w2=np.array([[50.0], [0.0], [0.0], [0.0]]), b2=np.array([-25.0, -50.0, -50.0, -50.0]))
    trace = []
    resp, steps, dl = O.generate_eotp_step(ScriptedModel(table, P), np.arange(P), G, s, mask, eos, flt, 0.5,
                                           trace=trace)
    # step 1: input 3 is the confidence of masked position 3 (< 0.99): only the forced top-1 (the EoT at 1) goes
    assert trace[0]["sel"].tolist() == [False, True, False, False]
    # step 2: sequence is P+2 long, positions 2, 3 discarded and enter as 1.0 -> p_0 = sigmoid(25) > tau
    assert trace[1]["n"] == 2 and trace[1]["p"][0] > 0.99
    assert steps == 2 and dl == 2 and resp[1] == eos and resp[0] == 3


# ----------------------------------------------------------------- Alg. 1 (EGP), Eq. 6, AdamW
def test_egp_with_greedy_reference_is_one_step_per_block_all_labels_one():
    P, G, s, V = 3, 32, 8, 20
    mask = V - 1
    table = rand_table(G, V, 41)
    table[:, mask] = -50.0
    ref = np.argmax(table, axis=1)
    C, Y, per_block = O.egp_rollout(ScriptedModel(table, P), np.arange(P), ref, G, s, mask)
    assert per_block == [1] * (G // s) and C.shape == (G // s, s)
    assert np.all(Y == 1.0)
    p = np.exp(table - table.max(1, keepdims=True))
    p[:, mask] = 0.0
    np.testing.assert_allclose(C.reshape(-1), (p / p.sum(1, keepdims=True)).max(1), rtol=1e-12)


def test_egp_mismatching_positions_are_forced_one_at_a_time_with_label_zero():
    # reference differs from the (position-only) greedy prediction at 3 positions of block 0:
    # step 1 unmasks the 5 agreeing ones; the 3 others can never agree, so they are taken one per
    # step in order of confidence, with the reference token and label 0
    P, G, s, V = 2, 8, 8, 12
    mask = V - 1
    table = np.zeros((G, V))
    greedy = [3, 1, 4, 1, 5, 9, 2, 6]
    for g, tok in enumerate(greedy):
        table[g, tok] = 2.0 + 0.1 * g                 # confidence grows with the position
    ref = np.array(greedy)
    ref[[1, 4, 6]] = [0, 0, 0]
    trace = []
    C, Y, per_block = O.egp_rollout(ScriptedModel(table, P), np.arange(P), ref, G, s, mask, trace=trace)
    assert per_block == [4]
    assert Y[0].tolist() == [1, 0, 1, 1, 0, 1, 0, 1]
    assert [t["sel"].nonzero()[0].tolist() for t in trace] == [[0, 2, 3, 5, 7], [6], [4], [1]]
    assert Y[1].tolist() == [1, 0, 1, 1, 0, 1, 0, 1] and Y[3].tolist() == [1, 0, 1, 1, 1, 1, 1, 1]
    assert np.all(C[1][[0, 2, 3, 5, 7]] == 1.0) and C[1][6] < 1.0    # committed positions enter as 1.0


def tiny_filter(s, h, seed):
    r = np.random.default_rng(seed)
    return dict(w1=r.normal(size=(h, s)), b1=r.normal(size=h), w2=r.normal(size=(s, h)), b2=r.normal(size=s))


@pytest.mark.parametrize("n_layers", [1, 2, 4])
def test_bce_gradient_matches_central_differences(n_layers):
    s, h, n = 5, 4, 7
    flt = tiny_filter(s, h, 51) if n_layers == 2 else deep_filter(s, h, n_layers, 51)
    r = np.random.default_rng(52)
    C, Y = r.uniform(size=(n, s)), (r.uniform(size=(n, s)) > 0.4).astype(float)
    loss, g = O.bce_loss_and_grad(flt, C, Y)
    # the definition of Eq. 6 written out entry by entry
    tot = 0.0
    for i in range(n):
        p = O.filter_prob(C[i], flt)
        tot -= np.sum(Y[i] * np.log(p) + (1 - Y[i]) * np.log(1 - p))
    assert abs(loss - tot / (n * s)) < 1e-12
    eps = 1e-6
    for k in flt:
        num = np.zeros_like(flt[k])
        it = np.nditer(flt[k], flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            for sign in (+1, -1):
                f2 = {kk: np.array(vv, copy=True) for kk, vv in flt.items()}
                f2[k][idx] += sign * eps
                num[idx] += sign * O.bce_loss_and_grad(f2, C, Y)[0]
        np.testing.assert_allclose(g[k], num / (2 * eps), rtol=1e-5, atol=1e-8)


def test_single_layer_bce_gradient_is_the_logistic_regression_gradient():
    # one layer: z = W c + b, and the textbook gradient of the mean log loss is (sigma(z) - y) c^T / m
    s, n = 4, 6
    flt = deep_filter(s, s, 1, 57)
    r = np.random.default_rng(58)
    C, Y = r.uniform(size=(n, s)), (r.uniform(size=(n, s)) > 0.5).astype(float)
    _, g = O.bce_loss_and_grad(flt, C, Y)
    gw, gb = np.zeros((s, s)), np.zeros(s)
    for i in range(n):
        for j in range(s):
            z = flt["b1"][j] + sum(flt["w1"][j][t] * C[i][t] for t in range(s))
            e = 1 / (1 + math.exp(-z)) - Y[i][j]
            gb[j] += e / (n * s)
            for t in range(s):
                gw[j][t] += e * C[i][t] / (n * s)
    np.testing.assert_allclose(g["w1"], gw, rtol=1e-12)
    np.testing.assert_allclose(g["b1"], gb, rtol=1e-12)


@pytest.mark.parametrize("n_layers", [1, 4])
def test_training_of_depth_variants_agrees_with_the_library(n_layers):
    import torch
    s, h, n = 6, 5, 9
    flt = deep_filter(s, h, n_layers, 55)
    r = np.random.default_rng(56)
    C, Y = r.uniform(size=(n, s)), (r.uniform(size=(n, s)) > 0.5).astype(float)
    mine, losses = O.train_filter(flt, C, Y, 60, lr=1e-2)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in flt.items()}
    opt = torch.optim.AdamW(list(tp.values()), lr=1e-2, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    Ct, Yt = torch.tensor(C), torch.tensor(Y)
    for _ in range(60):
        opt.zero_grad()
        a = Ct
        for k in range(1, n_layers):
            a = torch.relu(a @ tp[f"w{k}"].T + tp[f"b{k}"])
        z = a @ tp[f"w{n_layers}"].T + tp[f"b{n_layers}"]
        torch.nn.functional.binary_cross_entropy_with_logits(z, Yt).backward()
        opt.step()
    assert set(mine) == set(tp)
    for k in mine:
        np.testing.assert_allclose(mine[k], tp[k].detach().numpy(), rtol=1e-8, atol=1e-10)
    assert losses[-1] < losses[0]


def test_adamw_first_step_closed_form_and_library_agreement():
    # t = 1: m_hat = g, v_hat = g^2, so the step is -lr (g / (|g| + eps) + wd theta)
    th, g = np.array([0.5, -2.0, 3.0]), np.array([0.1, -4.0, 1e-12])
    new, _, _ = O.adamw_step(th, g, np.zeros(3), np.zeros(3), 1, 1e-3)
    np.testing.assert_allclose(new, th - 1e-3 * (g / (np.abs(g) + 1e-8) + 0.01 * th), rtol=1e-12)
    # 60 epochs against the library's optimiser and automatic differentiation
    import torch
    s, h, n = 6, 5, 9
    flt = tiny_filter(s, h, 53)
    r = np.random.default_rng(54)
    C, Y = r.uniform(size=(n, s)), (r.uniform(size=(n, s)) > 0.5).astype(float)
    mine, losses = O.train_filter(flt, C, Y, 60, lr=1e-2)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in flt.items()}
    opt = torch.optim.AdamW(list(tp.values()), lr=1e-2, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    Ct, Yt = torch.tensor(C), torch.tensor(Y)
    for _ in range(60):
        opt.zero_grad()
        z = torch.relu(Ct @ tp["w1"].T + tp["b1"]) @ tp["w2"].T + tp["b2"]
        loss = torch.nn.functional.binary_cross_entropy_with_logits(z, Yt)
        loss.backward()
        opt.step()
    for k in mine:
        np.testing.assert_allclose(mine[k], tp[k].detach().numpy(), rtol=1e-8, atol=1e-10)
    assert losses[-1] < losses[0]
