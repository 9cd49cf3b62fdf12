"""Shared helpers of the GPU parity tests: seeded inputs -> GPU cache through the C ABI, and the same inputs ->
oracle, compared field by field."""
import numpy as np

import kvlinc_synth as synth
from oracle import attention as o_attn
from oracle import kvcache as o_cache
from oracle import layout as o_layout

OUT_MAX_ABS = 1e-2   # attention output tolerance (fp16 I/O, fp32 accumulate)
OUT_REL_L2 = 2e-3    # over all compared rows, and for every single row
STATE_REL_L2 = 2e-5  # S, P: fp32 accumulation of up to ~1e5 products against fp64 (measured 1e-6 .. 2e-6)
# Element-wise bounds on the states, relative to the largest magnitude of the tensor.  phi_k is a binary32 softmax of
# binary32 logits whose products are exact (relative error of an entry ~ 1e-6, from the fast exponential), the values
# are exact, and the sums run in binary32 in flush order: an element of S = sum_t phi[t][f] v[t][c] (terms of both
# signs, |S| ~ sqrt(n) |phi v|) is off by at most ~ 1e-6 sum_t |phi v| ~ 1e-6 sqrt(n) |S| if the errors of phi all
# pointed one way, i.e. 4e-4 |S| at n = 131072; they do not: measured 7e-7 .. 3.8e-6 of max |S| for n = 1280 .. 131072.
# P = sum_t phi[t][f] has terms of one sign: the relative error of its terms plus binary32 summation, measured
# 8e-8 .. 4.7e-7 of max |P|.  The bounds leave a factor of 5 to 10 over the worst measured value.
STATE_S_ELEMENT = 2e-5
STATE_P_ELEMENT = 5e-6


def gen_kv(config, B, H_kv, lengths):
    """K, V as [B, H_kv, T, 128] fp16 (rows past a sequence's length are zero), T = max length."""
    T = int(max(lengths))
    K = np.zeros((B, H_kv, T, 128), dtype=np.float16)
    V = np.zeros((B, H_kv, T, 128), dtype=np.float16)
    for b in range(B):
        for g in range(H_kv):
            K[b, g, :lengths[b]] = synth.keys(config, b, g, int(lengths[b]))
            V[b, g, :lengths[b]] = synth.values(config, b, g, int(lengths[b]))
    return K, V


def gen_q(config, B, H_q, step=0):
    return np.stack([synth.queries(config, b, H_q, step) for b in range(B)])


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def u16(a):
    return np.ascontiguousarray(a).view(np.uint16)


def check_counters(cache, lengths, keep=None):
    n_quant = cache.n_quant.cpu().numpy()
    n_res = cache.n_res.cpu().numpy()
    for b in range(cache.B):
        want = o_cache.window_split(int(lengths[b]), keep=keep)
        assert (int(n_quant[b]), int(n_res[b])) == want, (b, n_quant[b], n_res[b], want)
    return n_quant, n_res


def _ordered16(h16):
    """fp16 bit patterns as integers that order like the numbers (for distances in units in the last place)."""
    u = np.ascontiguousarray(h16, dtype=np.float16).view(np.uint16).astype(np.int32)
    return np.where(u & 0x8000, -(u & 0x7FFF), u)


def check_states_against(cache, b, g, S_ref, P_ref, quiet=False):
    """S, P of one (sequence, kv head) against the oracle's (fp64): by norm, element by element, and the binary16 tile
    copy against binary16 of the ORACLE's S -- equal up to one unit in the last place (the rounding of a value that
    differs in its last binary32 bits), or inside the element-wise bound where |S| is small against the tensor's
    largest entries."""
    S = cache.S[b, g].cpu().numpy().astype(np.float64)
    P = cache.P[b, g].cpu().numpy().astype(np.float64)
    for got, want, nm in ((S, S_ref, "S"), (P, P_ref, "P")):
        den = np.linalg.norm(want)
        err = np.linalg.norm(got - want)
        assert err <= STATE_REL_L2 * den + 1e-12, (nm, b, g, err, den)
    s_max, p_max = np.abs(S_ref).max(), np.abs(P_ref).max()
    s_err, p_err = np.abs(S - S_ref).max(), np.abs(P - P_ref).max()
    assert s_err <= STATE_S_ELEMENT * s_max + 1e-12, ("S element", b, g, s_err, s_max)
    assert p_err <= STATE_P_ELEMENT * p_max + 1e-12, ("P element", b, g, p_err, p_max)
    S16 = o_layout.unpack_state_tiles(cache.S16[b, g].cpu().numpy())
    ulps = np.abs(_ordered16(S16) - _ordered16(S_ref.astype(np.float16)))
    near = np.abs(S16.astype(np.float64) - S_ref) <= STATE_S_ELEMENT * s_max
    assert np.isfinite(S16.astype(np.float32)).all()
    assert ((ulps <= 1) | near).all(), ("S16", b, g, int(ulps.max()))
    if not quiet:
        print("  [states] (%d, %d) S elem err %.2e of max, P elem err %.2e of max, S16 != fp16(oracle S) at %d of %d entries"
              % (b, g, s_err / max(s_max, 1e-300), p_err / max(p_max, 1e-300), int((ulps != 0).sum()), ulps.size))
    return s_err / max(s_max, 1e-300), p_err / max(p_max, 1e-300)


def check_pair_against_oracle(cache, b, g, k_rows, v_rows, nq, nr, Wk_g=None, check_states=True):
    """Bit-exact comparison of everything the append path stores for one (sequence, kv head) whose token history is
    k_rows, v_rows [n, 128]; returns the oracle's cache."""
    bits = getattr(cache, "bits", 2)
    pack, unpack = (o_layout.pack_records, o_layout.unpack_records) if bits == 2 else (o_layout.pack_records4, o_layout.unpack_records4)
    ref = o_cache.build_cache(k_rows, v_rows, nq, Wk=Wk_g, bits=bits)
    ng = -(-nq // 128)
    rec = cache.groups[b, g, :ng].cpu().numpy().view(np.uint32)
    if ng:
        # logical fields first (clearer failure), then the physical record bytes
        got = unpack(rec)
        assert np.array_equal(got["k_codes"], ref["k_codes"]), ("k codes", b, g)
        assert np.array_equal(got["v_codes"], ref["v_codes"]), ("v codes", b, g)
        for name in ("k_scale", "k_zero", "v_scale", "v_zero"):
            assert np.array_equal(u16(got[name]), u16(ref[name])), (name, b, g)
        want = pack(ref["k_codes"], ref["v_codes"], ref["k_scale"], ref["k_zero"], ref["v_scale"], ref["v_zero"])
        assert np.array_equal(rec, want), ("records", b, g)
    assert np.array_equal(u16(cache.k_res[b, g, :nr].cpu().numpy()), u16(ref["k_res"])), ("k_res", b, g)
    v_win = o_layout.unpack_value_window(cache.v_res[b, g].cpu().numpy(), nr)
    assert np.array_equal(u16(v_win), u16(ref["v_res"])), ("v_res", b, g)
    if Wk_g is not None and check_states:
        check_states_against(cache, b, g, ref["S"], ref["P"])
    return ref


def check_cache_against_oracle(cache, K, V, lengths, pairs, Wk=None, keep=None, check_states=True):
    """check_pair_against_oracle for the listed (sequence, kv head) pairs of dense K, V [B, H_kv, T, 128]."""
    n_quant, n_res = check_counters(cache, lengths, keep)
    for (b, g) in pairs:
        n = int(lengths[b])
        check_pair_against_oracle(cache, b, g, K[b, g, :n], V[b, g, :n], int(n_quant[b]), int(n_res[b]),
                                  None if Wk is None else Wk[g], check_states)


def oracle_decode(K, V, q, lengths, n_quant, pairs, H_q, H_kv, Wq=None, Wk=None, bits=2):
    """{(b, h): y fp64[128]} for every query head of the listed (sequence, kv head) pairs."""
    gq = H_q // H_kv
    out = {}
    for (b, g) in pairs:
        n = int(lengths[b])
        ref = o_cache.build_cache(K[b, g, :n], V[b, g, :n], int(n_quant[b]), Wk=None if Wk is None else Wk[g], bits=bits)
        for h in range(g * gq, (g + 1) * gq):
            out[(b, h)] = o_attn.decode(q[b, h], ref, None if Wq is None else Wq[h])
    return out


def check_outputs(got, want):
    """got: [B, H_q, 128] array; want: {(b, h): y}.  Max-abs and relative-L2 over all compared rows."""
    g = np.stack([got[b, h].astype(np.float64) for (b, h) in want])
    w = np.stack([want[k] for k in want])
    assert np.isfinite(g).all()
    max_abs = np.abs(g - w).max()
    rel_l2 = np.linalg.norm(g - w) / np.linalg.norm(w)
    worst_row = max(np.linalg.norm(g[i] - w[i]) / np.linalg.norm(w[i]) for i in range(len(w)))
    print("  [parity] rows %d max_abs %.3e rel_l2 %.3e worst_row_rel_l2 %.3e" % (len(w), max_abs, rel_l2, worst_row))
    assert max_abs <= OUT_MAX_ABS, ("max abs", max_abs)
    assert rel_l2 <= OUT_REL_L2, ("rel l2", rel_l2, "worst row", worst_row)
    assert worst_row <= OUT_REL_L2, ("worst row rel l2", worst_row)
    return max_abs, rel_l2, worst_row
