"""Host-side checks of the seeded input generator (no method arithmetic lives there)."""
import numpy as np
import torch

from paper_2407_20485_amd import synth


def test_budget_integers():
    c = synth.CONFIGS
    assert (c[0].select, c[0].recent, c[0].G) == (32, 32, 4)
    assert (c[1].select, c[1].recent, c[1].G) == (102, 102, 32)
    assert (c[2].select, c[2].recent, c[2].G) == (100, 100, 16384)
    assert (c[3].select, c[3].recent, c[3].G) == (204, 205, 320)
    assert (c[4].select, c[4].recent, c[4].G) == (1638, 1638, 32)
    assert c[4].alphas == (0.1, 0.5, 0.9, 1.0)


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 3
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]        # exact halfway cases
    bits = synth.round_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    assert np.array_equal(synth.bf16_bits_to_f32(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_heads_are_reproducible_and_distinct():
    w = synth.CONFIGS[1]
    a = synth.head_arrays(w, 3)
    b = synth.head_arrays(w, 3)
    c = synth.head_arrays(w, 4)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert not np.array_equal(a[0], c[0])
    assert a[0].shape == (w.n + w.T, w.d)
    # bf16-representable
    assert np.array_equal(synth.bf16_bits_to_f32(synth.round_to_bf16_bits(a[1])), a[1])


def test_generate_layout_matches_head_arrays():
    w = synth.CONFIGS[0]
    out = synth.generate(w, heads=[2, 0], threads=2)
    Q, K, V = synth.head_arrays(w, 2)
    assert np.array_equal(out["q"][0], Q[:w.n]) and np.array_equal(out["vd"][:, 0], V[w.n:])
    w1 = synth.CONFIGS[1]
    out = synth.generate(w1, heads=[5], threads=1)
    Q, K, V = synth.head_arrays(w1, 5)
    assert out["k"].dtype == np.uint16
    assert np.array_equal(synth.bf16_bits_to_f32(out["k"][0]), K[:w1.n])
    assert np.array_equal(synth.bf16_bits_to_f32(out["qd"][:, 0]), Q[w1.n:])


def test_planted_salience_shape():
    w = synth.CONFIGS[0]
    Q, K, V = synth.head_arrays(w, 0)
    # the shared direction shows up as a common mean in Q (unit norm => |mean row| ~ 1)
    u = Q.mean(axis=0)
    assert 0.8 < np.linalg.norm(u) < 1.25
    proj = K @ (u / np.linalg.norm(u))
    assert proj[0] > 1.0                                  # token 0 is always salient
    frac = np.mean(proj > 2.2)
    assert 0.005 < frac < 0.08
