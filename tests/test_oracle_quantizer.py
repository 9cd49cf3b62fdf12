"""Pins for oracle.quantizer and oracle.hadamard (no GPU)."""
import numpy as np
import pytest

from oracle import hadamard, quantizer


def _golden():
    import os
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_figures.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, val = line.split()[:2]
            out[name] = float(val)
    return out


# ---- Eq. 1 -----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_eq1_round_trip_bound_and_levels(bits):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((64, 128))
    codes, s, z = quantizer.quantize_real(x, bits)
    assert codes.min() == 0 and codes.max() == 2 ** bits - 1
    xq = quantizer.dequantize(codes, s, z)
    # |x - Q(x)| <= s/2 everywhere; the group minimum maps to level 0, the maximum to the top level
    assert np.all(np.abs(x - xq) <= s[:, None] / 2 + 1e-12)
    assert np.all(codes[np.arange(64), x.argmin(1)] == 0)
    assert np.all(codes[np.arange(64), x.argmax(1)] == 2 ** bits - 1)
    np.testing.assert_allclose(xq.min(1), x.min(1), atol=1e-12)
    np.testing.assert_allclose(xq.max(1), x.max(1), atol=1e-12)


def test_eq1_literal_small_case():
    # group [-1, 0, 0.2, 2] at 2 bits: s = 1, z = -1; (x - z)/s = [0, 1, 1.2, 3] -> codes [0, 1, 1, 3]
    codes, s, z = quantizer.quantize_real(np.array([[-1.0, 0.0, 0.2, 2.0]]), 2)
    assert codes.tolist() == [[0, 1, 1, 3]] and s[0] == 1.0 and z[0] == -1.0
    # ties go to the even level: [0, 0.5, 1.5, 2.5, 3] with s = 1 -> [0, 0, 2, 2, 3]
    codes, s, z = quantizer.quantize_real(np.array([[0.0, 0.5, 1.5, 2.5, 3.0]]), 2)
    assert codes.tolist() == [[0, 0, 2, 2, 3]]
    assert quantizer.dequantize(codes, s, z).tolist() == [[0.0, 0.0, 2.0, 2.0, 3.0]]


def test_eq2_error_law_on_uniform_data():
    # Eq. 2: E[(Q(X) - X)^2] = s^2 / 12 when the error is uniform inside a quantization cell
    rng = np.random.default_rng(2)
    x = rng.uniform(-1.0, 1.0, size=(4, 200000))
    for bits in (2, 4):
        codes, s, z = quantizer.quantize_real(x, bits)
        mse = ((quantizer.dequantize(codes, s, z) - x) ** 2).mean(axis=1)
        np.testing.assert_allclose(mse, s ** 2 / 12.0, rtol=0.02)


def test_constant_group_is_all_zero_codes():
    for fn in (lambda a: quantizer.quantize_real(a, 2), quantizer.quantize_exact16, quantizer.quantize_spec32):
        codes, s, z = fn(np.full((3, 128), 1.25, dtype=np.float16))
        assert not codes.any() and not np.asarray(s, dtype=np.float64).any()
        assert np.all(quantizer.dequantize(codes, s, z) == 1.25)


@pytest.mark.parametrize("bits", [2, 4])
def test_spec32_is_eq1_against_stored_scale(bits):
    """The binary32 threshold form must be round-half-even of the REAL quotient (x - z16) / s16, clamped."""
    L = 2 ** bits - 1
    rng = np.random.default_rng(3)
    x16 = (rng.standard_normal((512, 128)) * rng.choice([1e-3, 1.0, 30.0], size=(512, 1))).astype(np.float16)
    x16[:64] = np.round(rng.standard_normal((64, 128)) * 4) / 4  # rows on a coarse grid: many exact ties
    codes, s16, z16 = quantizer.quantize_spec32(x16, bits)
    # rebuild from exact rational arithmetic on the stored patterns (fp16 values are exact in fp64 and so are
    # their differences; the only binary32 rounding in the contract is t = fl32(x - z16))
    t = (x16.astype(np.float32) - z16.astype(np.float32)[:, None]).astype(np.float64)
    s = s16.astype(np.float64)[:, None]
    ref = np.clip(np.rint(t / s), 0, L)  # np.rint is half-to-even; t/s here is only inexact away from ties
    frac = t / s - np.floor(t / s)
    far_from_tie = np.abs(frac - 0.5) > 1e-9
    assert np.all(codes[far_from_tie] == ref[far_from_tie])
    # exact ties, decided in integers: 2t = (2k+1)s  ->  even level
    tie = ~far_from_tie
    if tie.any():
        k = np.floor(t / s)[tie]
        want = np.clip(np.where(k % 2 == 0, k, k + 1), 0, L)
        assert np.all(codes[tie] == want)
    # stored pattern definition
    mn, mx = x16.astype(np.float32).min(1), x16.astype(np.float32).max(1)
    assert np.array_equal(z16.view(np.uint16), mn.astype(np.float16).view(np.uint16))
    assert np.array_equal(s16.view(np.uint16), ((mx - mn) / np.float32(L)).astype(np.float16).view(np.uint16))
    # self-consistent round trip against the stored scale (t >= 0; beyond (L + .5) s can only come from fp16 rounding of s)
    err = np.abs(quantizer.dequantize(codes, s16, z16) - x16.astype(np.float64))
    assert np.all(err <= 0.5 * s + np.abs(mx.astype(np.float64) - mn - L * s[:, 0])[:, None] + 1e-12)


def test_spec32_ties_literal():
    # s16 = 1 exactly: x - z in {0, .5, 1.5, 2.5, 3} -> {0, 0, 2, 2, 3}
    x = np.array([[0.0, 0.5, 1.5, 2.5, 3.0] + [1.0] * 123], dtype=np.float16)
    codes, s16, z16 = quantizer.quantize_spec32(x)
    assert float(s16[0]) == 1.0 and float(z16[0]) == 0.0
    assert codes[0, :5].tolist() == [0, 0, 2, 2, 3]
    # 4 bits, s16 = 1 exactly (range 0..15): every half goes to the even neighbour
    halves = [k + 0.5 for k in range(15)]
    x = np.array([[0.0, 15.0] + halves + [7.0] * 111], dtype=np.float16)
    codes, s16, z16 = quantizer.quantize_spec32(x, 4)
    assert float(s16[0]) == 1.0 and float(z16[0]) == 0.0
    assert codes[0, :2].tolist() == [0, 15]
    assert codes[0, 2:17].tolist() == [0, 2, 2, 4, 4, 6, 6, 8, 8, 10, 10, 12, 12, 14, 14]


def test_spec32_negative_zero_is_canonical():
    x = np.zeros((3, 128), dtype=np.float16)
    x[0, ::2] = -0.0                 # zeros of both signs
    x[1, :] = -0.0                   # only negative zeros: the minimum is -0 whatever the reduction order
    x[2, :] = np.arange(128) / 64.0  # the minimum is a single -0 among positive values
    x[2, 0] = -0.0
    codes, s16, z16 = quantizer.quantize_spec32(x)
    assert not z16.view(np.uint16).any(), "the stored zero-point of a zero minimum is +0"
    assert s16.view(np.uint16)[0] == 0 and s16.view(np.uint16)[1] == 0 and not codes[:2].any()
    assert float(s16[2]) == float(np.float16(np.float32(127 / 64.0) / np.float32(3.0))) and codes[2, 0] == 0


@pytest.mark.parametrize("bits", [2, 4])
def test_spec32_vs_exact16_mismatch_rate_is_tiny(bits):
    rng = np.random.default_rng(4)
    x16 = rng.standard_normal((4096, 128)).astype(np.float16)
    c1, s1, z1 = quantizer.quantize_spec32(x16, bits)
    c2, s2, z2 = quantizer.quantize_exact16(x16, bits)
    assert np.array_equal(z1.view(np.uint16), z2.view(np.uint16))
    assert (s1.view(np.uint16) != s2.view(np.uint16)).mean() < 1e-2  # fl16(fl32(d/3)) double rounding is rare
    same_scale = s1.view(np.uint16) == s2.view(np.uint16)
    assert (c1[same_scale] != c2[same_scale]).mean() < 1e-4


# ---- Hadamard rotation (Sec. 3.1) -----------------------------------------------------------------------

@pytest.mark.parametrize("d", [2, 4, 8, 128])
def test_sylvester_is_hadamard(d):
    H = hadamard.sylvester(d)
    assert set(np.unique(H)) == {-1.0, 1.0}
    assert np.array_equal(H @ H.T, d * np.eye(d))
    assert np.array_equal(H, H.T)
    if d == 4:
        assert H.tolist() == [[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]]


def test_rotation_is_orthogonal_and_self_inverse():
    rng = np.random.default_rng(5)
    v = rng.standard_normal((7, 128))
    r = hadamard.rotate_exact(v)
    np.testing.assert_allclose(np.linalg.norm(r, axis=1), np.linalg.norm(v, axis=1), rtol=1e-13)
    np.testing.assert_allclose(hadamard.rotate_exact(r), v, atol=1e-13)
    # a unit impulse at channel j rotates to row j of H
    e = np.zeros(128)
    e[5] = 1.0
    np.testing.assert_allclose(hadamard.rotate_exact(e), hadamard.sylvester(128)[5] / np.sqrt(128.0), atol=1e-15)


def test_fwht_spec32_equals_dense_product():
    rng = np.random.default_rng(6)
    # small integers: every partial sum is exact in binary32, so the butterfly order cannot matter and the result
    # must equal fp16(fl32(exact_sum * c32)) computed from the dense +-1 matrix
    v = rng.integers(-8, 9, size=(16, 128)).astype(np.float16)
    dense = v.astype(np.float64) @ hadamard.sylvester(128)
    want = (dense.astype(np.float32) * hadamard.INV_SQRT_128_F32).astype(np.float32).astype(np.float16)
    got = hadamard.fwht_spec32(v)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    # generic data: within one fp16 ulp of the fp64 rotation, and mostly identical to its fp16 rounding
    v = rng.standard_normal((256, 128)).astype(np.float16)
    got = hadamard.fwht_spec32(v)
    ref = hadamard.rotate_exact(v)
    assert np.all(np.abs(got.astype(np.float64) - ref) <= np.spacing(np.abs(ref).astype(np.float16)).astype(np.float64))
    assert (got.view(np.uint16) != hadamard.rotate_exact_fp16(v).view(np.uint16)).mean() < 5e-3
    assert abs(float(hadamard.INV_SQRT_128_F32) - 1 / np.sqrt(128.0)) < 2 ** -28


def test_rotation_removes_an_outlier_channel():
    # Sec. 3.1: the rotation spreads an outlier over all channels, so the token-wise range (the scale) drops
    rng = np.random.default_rng(7)
    v = rng.standard_normal((64, 128))
    v[:, 3] *= 20.0
    _, s_raw, _ = quantizer.quantize_real(v, 2)
    _, s_rot, _ = quantizer.quantize_real(hadamard.rotate_exact(v), 2)
    assert s_rot.mean() < 0.5 * s_raw.mean()


# ---- printed accounting (Table 1) -----------------------------------------------------------------------

def test_average_bits_match_table1():
    from oracle import accounting
    g = _golden()
    n = 8192
    kivi = accounting.average_bits(n, bits=2, group=int(g["group_size"]), window=128)
    kvlinc = accounting.average_bits(n, bits=2, group=int(g["group_size"]), window=128, D=int(g["adapter_rank_D"]))
    assert abs(kivi - 2.46484375) < 1e-12 and abs(kvlinc - 2.716796875) < 1e-12
    # the paper prints two decimals (2.7168 appears as 2.71 = 2.46 + 0.25): agree to within one unit of the last digit
    assert abs(kivi - g["kv_bits_kivi_quarot"]) < 0.01
    assert abs(kvlinc - g["kv_bits_kvlinc"]) < 0.01
    # the states are per KV head and counted at 16 bits: per QUERY head (4x) gives 3.47, at 32 bits 2.97
    assert abs(accounting.average_bits(n, D=256, state_bits=32) - g["kv_bits_kvlinc"]) > 0.2
    assert abs(accounting.average_bits(n, D=4 * 256) - g["kv_bits_kvlinc"]) > 0.5
    # without the fp16 window or without scale/zero-point the KIVI figure is missed too
    assert abs(accounting.average_bits(n, window=0) - g["kv_bits_kivi_quarot"]) > 0.2
    gib = accounting.fp16_cache_bytes(layers=32, kv_heads=8, d=128, n=8192, batch=16) / 2 ** 30
    assert gib == g["fp16_cache_gb_llama3_8b_8k_b16"]
