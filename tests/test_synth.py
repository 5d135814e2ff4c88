"""Host-side checks of the seeded input generators (no GPU, no method arithmetic)."""
import numpy as np
import pytest

from paper_2605_08632_amd import synth


def test_bf16_rounding_matches_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(100000) * np.exp(rng.uniform(-20, 20, 100000))).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]      # ties to even
    bits = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = synth.bf16_bits_to_f32(bits)
    assert np.array_equal(synth.f32_to_bf16_bits(back), bits)


def test_head_is_seeded_and_normalised():
    a = synth.make_head(7, 16, 64, 100, "bf16")
    b = synth.make_head(7, 16, 64, 100, "bf16")
    assert np.array_equal(a.H_bits, b.H_bits) and np.array_equal(a.W_bits, b.W_bits)
    c = synth.make_head(7, 16, 64, 100, "fp32")
    np.testing.assert_allclose(np.sqrt((c.H.astype(np.float64) ** 2).mean(axis=1)), 1.0, rtol=1e-6)
    assert abs(c.W.std() * np.sqrt(64) - 4.0) < 0.2


def test_targets_and_padding():
    B, K, V = 200, 8, 1000
    am = np.arange(B * K) % V
    y, agree = synth.make_targets(3, am, B, K, V, 0.5, "zipf")
    assert y.dtype == np.int32 and y.min() >= 0 and y.max() < V
    assert np.all(y[agree] == am[agree]) and 0.4 < agree.mean() < 0.6
    p = synth.agree_probability(("linear", 0.9, 0.3), 2, 4)
    np.testing.assert_allclose(p[:4], [0.9, 0.7, 0.5, 0.3])
    vl = synth.make_valid_len(3, B, K, 0.1)
    assert vl.max() == K and vl.min() >= 1 and 0 < (vl < K).mean() < 0.25
    yp = synth.apply_tail_padding(y, vl, K).reshape(B, K)
    for b in range(B):
        assert np.all(yp[b, vl[b]:] == synth.IGNORE_INDEX) and np.all(yp[b, :vl[b]] >= 0)
    conf = synth.make_external_conf(3, agree)
    assert conf.min() >= 0.05 and conf.max() <= 0.95 and conf[agree].mean() > conf[~agree].mean()
