"""The seeded input generator: determinism, statistics, structure, bf16 rounding."""
import numpy as np
import torch

import gen
from gen import cases


def test_mix64_known_values():
    # splitmix64 reference stream for state 0: first outputs of the published generator
    x = np.array([0x9E3779B97F4A7C15, 2 * 0x9E3779B97F4A7C15 & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
    out = gen.mix64(x)
    assert int(out[0]) == 0xE220A8397B1DCDAF
    assert int(out[1]) == 0x6E789E6AA1B965F4


def test_normal12_statistics_and_grid():
    z = gen.normal12(gen.stream_key(1, 1, 0, 0), np.arange(1 << 20))
    assert abs(float(z.mean())) < 5e-3 and abs(float(z.std()) - 1.0) < 5e-3
    assert np.all(z * 1024 == np.round(z * 1024))           # exact multiples of 2^-10
    assert abs(float(np.mean(z ** 4)) - 3.0) < 0.15          # close to Gaussian kurtosis (2.9)
    z2 = gen.normal12(gen.stream_key(1, 1, 0, 1), np.arange(1 << 16))
    assert abs(float(np.corrcoef(z[: 1 << 16], z2)[0, 1])) < 0.02


def test_bf16_rounding_matches_torch():
    x = (np.random.default_rng(0).standard_normal(100000) * 3).astype(np.float32)
    bits = gen.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    np.testing.assert_array_equal(gen.bf16_bits_to_f32(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_case_is_deterministic_and_addressable():
    a, b = gen.make_case(gen.tiny_spec()), gen.make_case(gen.tiny_spec())
    np.testing.assert_array_equal(a.q, b.q)
    K, V = a.kv_group(1, 3)
    rows = np.array([5, 700, 33])
    np.testing.assert_array_equal(a.kv_rows("k", 1, 3, rows)[0], K[rows])
    np.testing.assert_array_equal(b.kv_rows("v", 1, 3, rows)[0], V[rows])
    assert not np.array_equal(K[:50], a.kv_group(0, 3)[0][:50])     # requests are independent
    assert not np.array_equal(K[:50], a.kv_group(1, 2)[0][:50])     # heads are independent
    assert not np.array_equal(K[:50], V[:50])


def test_case_structure():
    spec = gen.tiny_spec(L=2000, T=8)
    c = gen.make_case(spec)
    assert c.q.shape == (9, 2, 32, 128) and c.q.dtype == np.float32
    np.testing.assert_allclose(np.sqrt((c.q.astype(np.float64) ** 2).mean(-1)), 1.0, rtol=1e-6)
    assert c.Lcap == 2008 and c.seq_lens(3).tolist() == [2003, 2003]
    K, _ = c.kv_group(0, 0)
    s = K.astype(np.float64) @ c.q[0, 0, 0].astype(np.float64) / np.sqrt(128)
    hot = c.hot_pos[0, 0]
    plain = np.setdiff1d(np.arange(4, 2000 - 16), hot)
    assert s[:4].min() > 5.0                                   # sinks dominate
    assert s[hot].mean() > 1.2 and s[2000 - 16:].mean() > 2.0  # +2 sigma verticals, +3 recency/appended
    assert abs(s[plain].mean()) < 0.1 and abs(s[plain].std() - 1.0) < 0.1
    # heads of one group look in similar directions; consecutive steps drift slowly
    q = c.q.astype(np.float64)
    assert np.dot(q[0, 0, 0], q[0, 0, 1]) / 128 > 0.85
    assert np.dot(q[0, 0, 0], q[1, 0, 0]) / 128 > 0.98


def test_named_workloads_shapes():
    c5 = gen.make_case(gen.C5)
    assert c5.seq_lens0.min() >= 16384 and c5.seq_lens0.max() <= 65536 and len(set(c5.seq_lens0.tolist())) > 16
    assert np.all(c5.k % 64 == 0) and np.all(np.abs(c5.k - 0.02 * c5.seq_lens0) <= 32)
    c4 = gen.make_case(gen.C4)
    assert c4.kv_bytes() == 2 * 16 * 8 * (131072 + 32) * 128 * 2
    c3 = gen.make_case(gen.C3)
    q = c3.q.astype(np.float64)
    step_cos = [np.dot(q[t, 0, 0], q[t - 1, 0, 0]) / 128 for t in range(1, 33)]
    assert step_cos[15] < 0.93 and step_cos[31] < 0.93 and min(step_cos[:15]) > 0.98   # drift spikes at t = 16, 32


def test_e4m3_rounding_matches_an_independent_implementation():
    """The generator's fp32 -> FP8 E4M3 rounding against torch's own conversion (in range; beyond +-464 the
    generator saturates at 448 where torch returns NaN), and the decode table against torch's decode."""
    import torch
    from gen.cases import E4M3_VALUES, e4m3_bits_to_f32, f32_to_e4m3_bits
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.normal(size=50000).astype(np.float32) * s for s in (1e-3, 0.02, 1.0, 30.0, 300.0)] +
                       [np.array([0, -0.0, 448, 449, 463.9, 464, 480, 1e5, -1e5, 2 ** -6, 2 ** -7, 2 ** -9, 2 ** -10,
                                  1.5 * 2 ** -9, 2.5 * 2 ** -9, 0.5 * 2 ** -9, 0.0625, 0.0615], dtype=np.float32)])
    mine = f32_to_e4m3_bits(x)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    inside = np.abs(x) < 464
    np.testing.assert_array_equal(mine[inside], ref[inside])
    np.testing.assert_array_equal(e4m3_bits_to_f32(mine[~inside]), np.sign(x[~inside]) * 448)
    every = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    np.testing.assert_array_equal(E4M3_VALUES, every)          # NaN patterns compare equal here
    # every stored value survives the trip through bf16 (what the scoring kernel relies on)
    finite = np.isfinite(E4M3_VALUES)
    v = E4M3_VALUES[finite]
    np.testing.assert_array_equal(gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(v)), v)


def test_fp8_key_rows_are_e4m3_values_of_the_bf16_recipe():
    spec = gen.tiny_spec("fp8_rows", k_dtype="fp8")
    case = gen.make_case(spec)
    rows = np.array([0, 3, 5, 100, 700])
    vals, bits = case.kv_rows("k", 1, 2, rows)
    assert bits.dtype == np.uint8 and vals.dtype == np.float32
    np.testing.assert_array_equal(vals, gen.e4m3_bits_to_f32(bits))
    v_vals, v_bits = case.kv_rows("v", 1, 2, rows)
    assert v_bits.dtype == np.uint16                       # values stay bf16
    plain = gen.make_case(gen.tiny_spec("fp8_rows"))       # same seed, bf16 keys: same draws before rounding
    ref, _ = plain.kv_rows("k", 1, 2, rows)
    assert np.abs(vals - ref).max() <= 2.0 ** -4 * np.abs(ref).max()   # half an ulp of 3 mantissa bits


def test_fp16_rows_are_the_half_rounding_of_the_same_draws():
    import torch
    spec = gen.tiny_spec("f16_rows", kv_dtype="f16")
    case = gen.make_case(spec)
    rows = np.array([0, 3, 5, 100, 700])
    plain = gen.make_case(gen.tiny_spec("f16_rows", kv_dtype="f32"))    # same seed: the draws before rounding
    for which in ("k", "v"):
        vals, bits = case.kv_rows(which, 1, 2, rows)
        ref, _ = plain.kv_rows(which, 1, 2, rows)
        assert bits.dtype == np.uint16 and vals.dtype == np.float32
        want = torch.from_numpy(ref).to(torch.float16)                  # an independent round-to-nearest-even
        np.testing.assert_array_equal(bits, want.view(torch.int16).numpy().view(np.uint16))
        np.testing.assert_array_equal(vals, want.float().numpy())
