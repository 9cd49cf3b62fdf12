"""Pins for oracle.kvcache and oracle.attention (no GPU)."""
import math
from fractions import Fraction

import numpy as np
import pytest

import kvlinc_synth as synth
from oracle import attention, hadamard, kvcache, quantizer


def _case(n=300, seed=0, d=128):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((n, d)).astype(np.float16)
    K[:, [3, 40]] *= 8
    V = rng.standard_normal((n, d)).astype(np.float16)
    q = rng.standard_normal(d).astype(np.float16)
    Wq = (rng.standard_normal((2, d, d)) / np.sqrt(d)).astype(np.float16)
    Wk = (rng.standard_normal((2, d, d)) / np.sqrt(d)).astype(np.float16)
    return q, K, V, Wq, Wk


def test_window_split_is_the_lazy_block_flush():
    # replay one-token appends: flush 128 tokens only when the window is already full on entry
    nq, nr = 0, 0
    for n in range(1, 700):
        if nr == 128:
            nq, nr = nq + 128, 0
        nr += 1
        assert kvcache.window_split(n) == (nq, nr)
        assert 1 <= nr <= 128 and nq % 128 == 0
    assert kvcache.window_split(8192) == (8064, 128)
    assert kvcache.window_split(1024, keep=32) == (992, 32)
    assert kvcache.window_split(0) == (0, 0)


def test_bits_to_16_converges_to_textbook_attention():
    """Eq. 3 on unquantized operands is the limit of the whole pipeline as the bit width grows."""
    q, K, V, _, _ = _case(n=384)
    ref = attention.softmax_attention(q, K, V)
    errs = []
    for bits in (2, 4, 8, 12, 16):
        c = kvcache.build_cache(K, V, 256, bits=bits, mode="real")
        errs.append(np.abs(attention.decode(q, c) - ref).max())
    assert errs[0] > errs[1] > errs[2] > errs[3] > errs[4]
    assert errs[4] < 1e-5 and errs[2] < 5e-3
    # 4 more bits shrink the step 16x; in the linear regime the error follows (within a generous factor)
    assert 4.0 < errs[2] / errs[3] < 64.0
    # nothing quantized: exact
    c = kvcache.build_cache(K, V, 0, mode="real")
    np.testing.assert_allclose(attention.decode(q, c), ref, atol=1e-13)


def test_rotation_invariance_without_quantization():
    q, K, V, _, _ = _case(n=200)
    a = attention.decode(q, kvcache.build_cache(K, V, 0, mode="real", rotate=True), rotate=True)
    b = attention.decode(q, kvcache.build_cache(K, V, 0, mode="real", rotate=False), rotate=False)
    np.testing.assert_allclose(a, b, atol=1e-12)


def test_the_three_arithmetic_modes_describe_the_same_cache():
    """`spec32` (the GPU contract), `exact16` and `real` differ only in where they round: rotated window values agree
    to an fp16 ulp, almost all codes coincide, and the attention outputs agree far inside the output tolerance."""
    q, K, V, Wq, Wk = _case(n=300, seed=12)
    c32 = kvcache.build_cache(K, V, 256, mode="spec32", Wk=Wk)
    c16 = kvcache.build_cache(K, V, 256, mode="exact16", Wk=Wk)
    cre = kvcache.build_cache(K, V, 256, mode="real", Wk=Wk)
    want = V[256:].astype(np.float64) @ hadamard.orthonormal(128)
    for c in (c32, c16, cre):
        assert np.abs(c["v_res"].astype(np.float64) - want).max() <= 2.0 ** -9 * np.abs(want).max()
    assert (c32["k_codes"] != c16["k_codes"]).mean() < 1e-3 and (c32["v_codes"] != c16["v_codes"]).mean() < 1e-3
    assert (c32["v_codes"] != cre["v_codes"]).mean() < 2e-2
    a, b, r = (attention.decode(q, c, Wq) for c in (c32, c16, cre))
    assert np.abs(a - b).max() < 2e-3 and np.abs(a - r).max() < 2e-2


def test_rotated_value_quantization_beats_raw_on_outlier_values():
    # Obs. 3: token-wise quantization of rotated values has a smaller error than of raw values once a token has
    # an outlier channel
    rng = np.random.default_rng(11)
    V = rng.standard_normal((256, 128))
    V[:, 7] *= 25.0
    V = V.astype(np.float16)
    K = rng.standard_normal((256, 128)).astype(np.float16)
    rot = kvcache.build_cache(K, V, 256, mode="exact16", rotate=True)
    raw = kvcache.build_cache(K, V, 256, mode="exact16", rotate=False)
    err_rot = np.linalg.norm(rot["V_hat"] @ hadamard.orthonormal(128).T - V.astype(np.float64))
    err_raw = np.linalg.norm(raw["V_hat"] - V.astype(np.float64))
    assert err_rot < 0.5 * err_raw


def test_key_axis_choice_matches_observation_2():
    # Obs. 2 / Fig. 4: with channel outliers the channel-wise key scale is far below the token-wise one
    K = synth.keys(2, 0, 0, 512)
    _, s_c, _ = quantizer.quantize_real(K[:128].T.astype(np.float64), 2)
    _, s_t, _ = quantizer.quantize_real(K[:128].astype(np.float64), 2)
    assert np.median(s_c) < 0.5 * np.median(s_t)


@pytest.mark.parametrize("with_correction", [False, True])
def test_block_merge_equals_single_softmax(with_correction):
    """Alg. 1's per-block (Y, m, l) and its merge reproduce the single softmax for ANY block boundaries."""
    q, K, V, Wq, Wk = _case(n=700, seed=2)
    c = kvcache.build_cache(K, V, 640, Wk=Wk)
    W = Wq if with_correction else None
    ref = attention.decode(q, c, W)
    np.testing.assert_allclose(attention.decode_blocks(q, c, W), ref, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(attention.decode_blocks(q, c, W, boundaries=[]), ref, rtol=1e-11, atol=1e-13)
    rng = np.random.default_rng(5)
    cuts = sorted(set(rng.integers(1, 700, size=9).tolist()))
    np.testing.assert_allclose(attention.decode_blocks(q, c, W, boundaries=cuts), ref, rtol=1e-11, atol=1e-13)


def test_zero_states_give_plain_quantized_attention():
    q, K, V, Wq, Wk = _case(n=100, seed=3)
    c = kvcache.build_cache(K, V, 0, Wk=Wk)  # nothing quantized yet -> S = P = 0
    assert not c["S"].any() and not c["P"].any()
    np.testing.assert_allclose(attention.decode(q, c, Wq), attention.decode(q, c, None), atol=1e-14)


def test_zero_weights_closed_form():
    """W = 0 makes both feature maps uniform (1/128 per entry, each half), so f(q, k) = 256 / 128^2 = 1/64 for every
    quantized token: y_rot = (sum e^{s_i} v_i + (1/64) sum_{i<n_q} v_i) / (sum e^{s_i} + n_q / 64)."""
    q, K, V, _, _ = _case(n=300, seed=4)
    Z = np.zeros((2, 128, 128))
    c = kvcache.build_cache(K, V, 256, Wk=Z)
    np.testing.assert_allclose(c["P"], np.full(256, 256 / 128.0), rtol=1e-13)
    keys = np.concatenate([c["K_hat"], c["k_res"].astype(np.float64)])
    vals = np.concatenate([c["V_hat"], c["v_res"].astype(np.float64)])
    w = np.exp(keys @ q.astype(np.float64) / np.sqrt(128.0))
    want = (w @ vals + c["V_hat"].sum(0) / 64.0) / (w.sum() + 256 / 64.0)
    np.testing.assert_allclose(attention.decode(q, c, Z, rotate=False), want, rtol=1e-11)


def test_recurrent_states_equal_quadratic_form_and_literal_eq5():
    q, K, V, Wq, Wk = _case(n=200, seed=6)
    c = kvcache.build_cache(K, V, 128, Wk=Wk)
    a = attention.decode(q, c, Wq)
    np.testing.assert_allclose(attention.decode_quadratic(q, K, c, Wq, Wk), a, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(attention.decode_unshifted(q, c, Wq), a, rtol=1e-10, atol=1e-13)
    # the correction is not a no-op, and Alg. 1's unscaled form differs from Eq. 5 once max score != 0
    assert np.abs(a - attention.decode(q, c, None)).max() > 1e-6
    assert np.abs(a - attention.decode(q, c, Wq, literal_alg1=True)).max() > 1e-6
    # S accumulates group by group (the recurrence of Eq. 5)
    c2 = kvcache.build_cache(K[:128], V[:128], 128, Wk=Wk)
    np.testing.assert_allclose(c2["S"], c["S"], rtol=1e-13)


def test_states_are_additive_over_groups():
    _, K, V, _, Wk = _case(n=384, seed=7)
    full = kvcache.build_cache(K, V, 384, Wk=Wk)
    parts = [kvcache.build_cache(K[a:a + 128], V[a:a + 128], 128, Wk=Wk) for a in (0, 128, 256)]
    np.testing.assert_allclose(sum(p["S"] for p in parts), full["S"], rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(sum(p["P"] for p in parts), full["P"], rtol=1e-12)
    np.testing.assert_allclose(full["P"].sum(), 2 * 384, rtol=1e-12)  # each half of phi sums to one per token


def test_sixteen_bit_state_storage_rounds_at_the_stated_points():
    """state_rounding: one rounding at the end is binary16 of the exact state; a rounding after every group is the
    recurrence S <- fp16(S + phi_k^T V_q of the group) written out here; either stays within the rounding bound of the
    exact state and does round; P is not touched."""
    _, K, V, _, Wk = _case(n=640, seed=17)
    exact = kvcache.build_cache(K, V, 512, Wk=Wk)
    once = kvcache.build_cache(K, V, 512, Wk=Wk, state_rounding=[])
    assert np.array_equal(once["S"], exact["S"].astype(np.float16).astype(np.float64))
    assert np.array_equal(once["P"], exact["P"])
    every = kvcache.build_cache(K, V, 512, Wk=Wk, state_rounding=[128, 256, 384])
    S = np.zeros_like(exact["S"])
    for a in (0, 128, 256, 384):
        part = kvcache.build_cache(K[a:a + 128], V[a:a + 128], 128, Wk=Wk)["S"]
        S = (S + part).astype(np.float16).astype(np.float64)
    assert np.array_equal(every["S"], S)
    assert np.array_equal(every["S"], every["S"].astype(np.float16).astype(np.float64))
    bound = 4 * 2.0 ** -11 * np.abs(exact["S"]).max()  # four roundings, each half a unit in the last place at most
    assert 0 < np.abs(every["S"] - exact["S"]).max() <= bound
    # points that are not crossed do not matter; the state saturates instead of overflowing
    assert np.array_equal(kvcache.build_cache(K, V, 512, Wk=Wk, state_rounding=[512, 640, 1024])["S"], once["S"])
    big = kvcache.build_cache(K, (V.astype(np.float32) * 4096).astype(np.float16), 512, Wk=Wk, state_rounding=[256])
    assert np.isfinite(big["S"]).all() and np.abs(big["S"]).max() <= 65504.0


def test_sliding_value_window_uniform_attention_closed_form():
    """Sec. 4.1 (setup): with a zero query every token weighs the same, so the rotated output is the plain mean of the
    values the mode uses: fp16 values for the newest 128 tokens, dequantized ones for all older tokens -- whatever the key
    window holds (here 44 tokens).  The block mode uses the fp16 values of the 44 window tokens only."""
    _, K, V, _, _ = _case(n=300, seed=11)
    c = kvcache.build_cache(K, V, 256)
    q0 = np.zeros(128, dtype=np.float16)
    vr = c["v_rot"].astype(np.float64)
    want_sliding = (c["V_hat"][:300 - 128].sum(0) + vr[300 - 128:].sum(0)) / 300.0
    want_block = (c["V_hat"].sum(0) + vr[256:].sum(0)) / 300.0
    got_sliding = attention.decode(q0, c, None, rotate=False, value_window="sliding")
    got_block = attention.decode(q0, c, None, rotate=False)
    np.testing.assert_allclose(got_sliding, want_sliding, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(got_block, want_block, rtol=1e-12, atol=1e-14)
    assert np.abs(want_sliding - want_block).max() > 1e-4  # the two modes are told apart by this case


def test_sliding_value_window_equals_block_window_when_the_key_window_is_full():
    """With 128 tokens in the key window the newest 128 tokens are the window tokens: both modes use the same values.
    With fewer than 128 tokens in all nothing is quantized and again nothing differs."""
    q, K, V, Wq, Wk = _case(n=384, seed=12)
    c = kvcache.build_cache(K, V, 256, Wk=Wk)
    np.testing.assert_array_equal(attention.decode(q, c, Wq, value_window="sliding"), attention.decode(q, c, Wq))
    c = kvcache.build_cache(K[:100], V[:100], 0, Wk=Wk)
    np.testing.assert_array_equal(attention.decode(q, c, Wq, value_window="sliding"), attention.decode(q, c, Wq))


def test_sliding_value_window_is_closer_to_unquantized_values():
    """More values in full precision: the error against attention over the quantized keys and exact values shrinks."""
    q, K, V, _, _ = _case(n=300, seed=13)
    c = kvcache.build_cache(K, V, 256)
    exact_v = dict(c)
    exact_v["V_hat"] = c["v_rot"][:256].astype(np.float64)
    ref = attention.decode(q, exact_v, None)
    e_block = np.linalg.norm(attention.decode(q, c, None) - ref)
    e_sliding = np.linalg.norm(attention.decode(q, c, None, value_window="sliding") - ref)
    assert e_sliding < e_block


def test_partial_tail_group_uses_valid_tokens_only():
    _, K, V, _, _ = _case(n=256, seed=8)
    c = kvcache.build_cache(K, V, 224)  # one full group + 96 tokens
    assert c["k_codes"].shape[0] == 2 and not c["k_codes"][1, 96:].any() and not c["v_scale"][1, 96:].any()
    ck, sk, zk = quantizer.quantize_spec32(K[128:224].T)
    assert np.array_equal(c["k_codes"][1, :96], ck.T) and np.array_equal(c["k_scale"][1], sk)
    assert c["k_res"].shape[0] == 32 and np.array_equal(c["k_res"], K[224:])


# ---- brute force in exact rational arithmetic on a hand-sized case (d = G = 4, 2 bits) -------------------------

def _q2_fraction(row):
    """Eq. 1 at 2 bits on a list of Fractions, ties to even, written with integers only."""
    z = min(row)
    s = (max(row) - z) / 3
    codes = []
    for x in row:
        if s == 0:
            codes.append(0)
            continue
        r = (x - z) / s
        k = r.numerator // r.denominator
        frac = r - k
        if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and k % 2 == 1):
            k += 1
        codes.append(min(max(k, 0), 3))
    return codes, s, z


def test_tiny_case_brute_force():
    F = Fraction
    K = [[F(0), F(-3), F(1), F(0)],
         [F(1), F(0), F(1), F(1, 2)],
         [F(2), F(3), F(1), F(3, 2)],
         [F(3), F(6), F(1), F(1, 4)],
         [F(1, 2), F(-1), F(2), F(1)],      # window
         [F(-1), F(1, 2), F(0), F(-1, 2)]]  # window
    V = [[F(1), F(2), F(-1), F(0)],
         [F(0), F(1, 2), F(3), F(-2)],
         [F(4), F(-1), F(1), F(1)],
         [F(-2), F(0), F(0), F(2)],
         [F(1), F(1), F(1), F(1)],
         [F(3), F(-1), F(2), F(0)]]
    q = [F(1), F(-1, 2), F(2), F(1, 4)]
    H4 = [[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]]
    n_q = 4
    # hand-derived key codes per channel over the 4 quantized tokens:
    #   ch0 [0,1,2,3]: s=1 z=0 -> 0,1,2,3 | ch1 [-3,0,3,6]: s=3 z=-3 -> 0,1,2,3 | ch2 constant -> 0,0,0,0
    #   ch3 [0,.5,1.5,.25]: s=.5 z=0 -> 0,1,3,(0.5 -> tie -> 0)
    want_k_codes = [[0, 0, 0, 0], [1, 1, 0, 1], [2, 2, 0, 3], [3, 3, 0, 0]]
    Vr = [[sum(V[t][j] * H4[j][c] for j in range(4)) / 2 for c in range(4)] for t in range(6)]
    k_cols = [_q2_fraction([K[t][c] for t in range(n_q)]) for c in range(4)]
    K_hat = [[k_cols[c][1] * k_cols[c][0][t] + k_cols[c][2] for c in range(4)] for t in range(n_q)]
    v_rows = [_q2_fraction(Vr[t]) for t in range(n_q)]
    V_hat = [[v_rows[t][1] * v_rows[t][0][c] + v_rows[t][2] for c in range(4)] for t in range(n_q)]
    keys = K_hat + K[n_q:]
    vals = V_hat + Vr[n_q:]
    w = [math.exp(float(sum(q[c] * keys[t][c] for c in range(4))) / 2.0) for t in range(6)]
    # adapters: D = 4, W_1, W_2 in R^{4x2}
    Wq = [[[F(1), F(0)], [F(0), F(1)], [F(1, 2), F(-1, 2)], [F(0), F(0)]],
          [[F(0), F(1)], [F(1), F(1)], [F(0), F(0)], [F(-1), F(1, 2)]]]
    Wk = [[[F(2), F(0)], [F(0), F(0)], [F(0), F(1)], [F(0), F(4)]],
          [[F(0), F(0)], [F(1), F(0)], [F(0), F(0)], [F(-4), F(2)]]]

    def phi(x, W):
        out = []
        for half in range(2):
            logits = [float(sum(x[c] * W[half][c][j] for c in range(4))) for j in range(2)]
            e = [math.exp(v) for v in logits]
            out += [v / sum(e) for v in e]
        return out

    pq = phi(q, Wq)
    num = [sum(w[t] * float(vals[t][c]) for t in range(6)) for c in range(4)]
    den = sum(w)
    for t in range(n_q):  # Eq. 4, token by token
        f = sum(a * b for a, b in zip(pq, phi([K[t][c] - K_hat[t][c] for c in range(4)], Wk)))
        num = [num[c] + f * float(V_hat[t][c]) for c in range(4)]
        den += f
    y_rot = [v / den for v in num]
    y = [sum(y_rot[j] * H4[c][j] for j in range(4)) / 2 for c in range(4)]

    tof = lambda a: np.array([[float(x) for x in r] for r in a])
    c = kvcache.build_cache(tof(K), tof(V), n_q, G=4, bits=2, mode="real", Wk=tof2(Wk))
    assert c["k_codes"][0].tolist() == want_k_codes
    assert c["k_codes"][0].tolist() == [[k_cols[ch][0][t] for ch in range(4)] for t in range(4)]
    assert c["v_codes"][0].tolist() == [v_rows[t][0] for t in range(4)]
    assert c["k_scale"][0].tolist() == [1.0, 3.0, 0.0, 0.5] and c["k_zero"][0].tolist() == [0.0, -3.0, 1.0, 0.0]
    np.testing.assert_allclose(c["K_hat"], tof(K_hat), atol=1e-15)
    np.testing.assert_allclose(c["V_hat"], tof(V_hat), atol=1e-15)
    assert float(K[3][3] - K_hat[3][3]) == 0.25  # the one non-zero key error of this case
    got = attention.decode(np.array([float(x) for x in q]), c, tof2(Wq))
    np.testing.assert_allclose(got, y, rtol=1e-12)


def tof2(W):
    return np.array([[[float(x) for x in r] for r in half] for half in W])
