"""Shared helpers of the GPU parity tests: seeded inputs -> GPU cache through the C ABI, and the same inputs ->
oracle, compared field by field."""
import numpy as np

import kvlinc_synth as synth
from oracle import attention as o_attn
from oracle import kvcache as o_cache
from oracle import layout as o_layout

OUT_MAX_ABS = 1e-2   # attention output tolerance (fp16 I/O, fp32 accumulate)
OUT_REL_L2 = 2e-3
STATE_REL_L2 = 1e-4  # S, P: fp32 accumulation of up to ~1e5 products against fp64


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


def check_pair_against_oracle(cache, b, g, k_rows, v_rows, nq, nr, Wk_g=None, check_states=True):
    """Bit-exact comparison of everything the append path stores for one (sequence, kv head) whose token history is
    k_rows, v_rows [n, 128]; returns the oracle's cache."""
    ref = o_cache.build_cache(k_rows, v_rows, nq, Wk=Wk_g)
    ng = -(-nq // 128)
    rec = cache.groups[b, g, :ng].cpu().numpy().view(np.uint32)
    if ng:
        # logical fields first (clearer failure), then the physical record bytes
        got = o_layout.unpack_records(rec)
        assert np.array_equal(got["k_codes"], ref["k_codes"]), ("k codes", b, g)
        assert np.array_equal(got["v_codes"], ref["v_codes"]), ("v codes", b, g)
        for name in ("k_scale", "k_zero", "v_scale", "v_zero"):
            assert np.array_equal(u16(got[name]), u16(ref[name])), (name, b, g)
        want = o_layout.pack_records(ref["k_codes"], ref["v_codes"], ref["k_scale"], ref["k_zero"],
                                     ref["v_scale"], ref["v_zero"])
        assert np.array_equal(rec, want), ("records", b, g)
    assert np.array_equal(u16(cache.k_res[b, g, :nr].cpu().numpy()), u16(ref["k_res"])), ("k_res", b, g)
    v_win = o_layout.unpack_value_window(cache.v_res[b, g].cpu().numpy(), nr)
    assert np.array_equal(u16(v_win), u16(ref["v_res"])), ("v_res", b, g)
    if Wk_g is not None and check_states:
        S = cache.S[b, g].cpu().numpy().astype(np.float64)
        P = cache.P[b, g].cpu().numpy().astype(np.float64)
        for got, want, nm in ((S, ref["S"], "S"), (P, ref["P"], "P")):
            den = np.linalg.norm(want)
            err = np.linalg.norm(got - want)
            assert err <= STATE_REL_L2 * den + 1e-12, (nm, b, g, err, den)
        # the binary16 tile copy the decode step reads: the fp32 state (checked above) rounded to nearest, in the
        # documented tile order
        S16 = o_layout.unpack_state_tiles(cache.S16[b, g].cpu().numpy())
        assert np.array_equal(u16(S16), u16(cache.S[b, g].cpu().numpy().astype(np.float16))), ("S16", b, g)
    return ref


def check_cache_against_oracle(cache, K, V, lengths, pairs, Wk=None, keep=None, check_states=True):
    """check_pair_against_oracle for the listed (sequence, kv head) pairs of dense K, V [B, H_kv, T, 128]."""
    n_quant, n_res = check_counters(cache, lengths, keep)
    for (b, g) in pairs:
        n = int(lengths[b])
        check_pair_against_oracle(cache, b, g, K[b, g, :n], V[b, g, :n], int(n_quant[b]), int(n_res[b]),
                                  None if Wk is None else Wk[g], check_states)


def oracle_decode(K, V, q, lengths, n_quant, pairs, H_q, H_kv, Wq=None, Wk=None):
    """{(b, h): y fp64[128]} for every query head of the listed (sequence, kv head) pairs."""
    gq = H_q // H_kv
    out = {}
    for (b, g) in pairs:
        n = int(lengths[b])
        ref = o_cache.build_cache(K[b, g, :n], V[b, g, :n], int(n_quant[b]), Wk=None if Wk is None else Wk[g])
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
    return max_abs, rel_l2, worst_row
