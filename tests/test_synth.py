"""The seeded input generator: determinism, distribution and shape checks (CPU)."""
import numpy as np
import torch

from paper_2509_25188_amd import synth


def test_normal_is_deterministic_and_normal():
    a = synth.normal(7, "x", (1000, 300), 0.02, torch.float32)
    b = synth.normal(7, "x", (1000, 300), 0.02, torch.float32)
    assert torch.equal(a, b)
    c = synth.normal(8, "x", (1000, 300), 0.02, torch.float32)
    d = synth.normal(7, "y", (1000, 300), 0.02, torch.float32)
    assert not torch.equal(a, c) and not torch.equal(a, d)
    x = a.double().numpy().ravel()
    assert abs(x.mean()) < 2e-4 and abs(x.std() - 0.02) < 2e-4
    assert abs(np.mean(x ** 4) / x.var() ** 2 - 3.0) < 0.05      # kurtosis of a normal
    assert abs(np.corrcoef(x[:-1], x[1:])[0, 1]) < 0.01
    assert abs(np.corrcoef(a.numpy().ravel(), d.numpy().ravel())[0, 1]) < 0.01


def test_chunking_does_not_change_values(monkeypatch):
    a = synth.normal(3, "w", (5000,), 1.0, torch.float32)
    monkeypatch.setattr(synth, "_CHUNK", 777)
    b = synth.normal(3, "w", (5000,), 1.0, torch.float32)
    assert torch.equal(a, b)


def test_prompt_range_and_bf16_bits():
    w = synth.WORKLOADS["8b_g256"]
    p = synth.make_prompt(1, 4, 256, w.prompt_hi)
    assert p.dtype == torch.int32 and p.min() >= 0 and p.max() < w.prompt_hi
    assert p.max() > w.prompt_hi * 0.9
    t = synth.normal(1, "t", (64,), 0.02, torch.bfloat16)
    bits = synth.to_numpy(t)
    assert bits.dtype == np.uint16
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    np.testing.assert_array_equal(back, t.float().numpy())


def test_weight_specs_cover_the_model():
    m = synth.WORKLOADS["tiny"].model
    w = synth.make_weights(m, 1234)
    n = sum(v.numel() for v in w.values())
    d, f, v, L = m.d_model, m.d_ffn, m.vocab, m.n_layers
    assert n == 2 * v * d + d + L * (2 * d + 4 * d * d + 3 * d * f)
    assert torch.all(w["final_norm_g"] == 1)
    assert w["layers.0.w_down"].shape == (d, f) and w["layers.1.w_gate"].shape == (f, d)
    m8 = synth.WORKLOADS["8b_g256"].model
    total = sum(int(np.prod(s)) for _, s, _ in synth.weight_specs(m8))
    assert 7.9e9 < total < 8.2e9


def test_numpy_and_torch_paths_agree():
    for dt in (torch.float32, torch.bfloat16):
        a = synth.normal(5, "k", (333, 1001), 0.3, dt)
        b = synth.normal(5, "k", (333, 1001), 0.3, dt, force_torch=True)
        assert torch.equal(a, b)


def test_threshold_filter_is_a_confidence_threshold():
    # the baseline decoder of bench.py: filter output > 0.5 exactly where the confidence exceeds theta
    import numpy as np
    from oracle import l2pd_oracle as O
    flt = {k: v.numpy() for k, v in synth.threshold_filter(8, 0.9).items()}
    conf = np.array([0.05, 0.5, 0.89, 0.899, 0.901, 0.95, 1.0, 0.0], dtype=np.float32)
    p = O.filter_prob(conf, flt)
    np.testing.assert_array_equal(p > 0.5, conf > 0.9)
