"""The quantized KV cache of one (sequence, kv head): K_q = Q_C(K), V_q = Q_T(V H) at 2 bits with
group size G (Sec. 3.1, Obs. 3), the G most recent tokens kept in fp16 (Sec. 4.1), and the linear
correction states S_n = sum phi_k(K^e_i)^T V^q_i, P_n = sum phi_k(K^e_i) with K^e = K - K^q
(Sec. 3.2, Eq. 4-5).

Readings taken where the paper leaves room (each is listed with its reason in the design notes):
  * the cache is quantized only after attention has used the new token (Sec. 3.3, last sentence),
    so the window is flushed as one block of G tokens when it is already full at the next append:
    after n appends 1 <= n_res <= G and n_quant is a multiple of G;
  * values are rotated, rounded to fp16, then quantized (in the paper H is folded into the value
    projection, so V H arrives as an fp16 activation); the window keeps the rotated fp16 values;
  * the states sum over quantized tokens only (K^e is undefined for a token that is still fp16) and
    use the dequantized values V^q, as Eq. 4 does.
"""
import numpy as np

from . import hadamard, quantizer


def window_split(n, G=128, keep=None):
    """(n_quant, n_res) after n one-token appends to an empty cache.

    keep=None: the lazy block flush described above.  keep=k: a bulk build that leaves exactly the
    k newest tokens in fp16 and quantizes the rest, the last group possibly partial.
    """
    if n == 0:
        return 0, 0
    n_res = (n - 1) % G + 1 if keep is None else min(keep, n)
    return n - n_res, n_res


def softmax_rows(x):
    x = np.asarray(x, dtype=np.float64)
    m = x.max(axis=-1, keepdims=True)
    e = np.exp(x - m)
    return e / e.sum(axis=-1, keepdims=True)


def feature_map(x, W):
    """phi(X) = [softmax(X W_1), softmax(X W_2)] in R^D (Eq. 6).  W: [2, d, D/2]."""
    x = np.asarray(x, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    return np.concatenate([softmax_rows(x @ W[0]), softmax_rows(x @ W[1])], axis=-1)


def _quantize_rows(x, bits, mode):
    if mode == "spec32":
        return quantizer.quantize_spec32(x, bits)
    if mode == "exact16":
        return quantizer.quantize_exact16(x, bits)
    if mode == "real":
        return quantizer.quantize_real(x, bits)
    raise ValueError(mode)


def build_cache(K, V, n_quant, *, G=128, bits=2, mode="spec32", rotate=True, Wk=None, state_rounding=None):
    """State of the cache holding tokens 0..n-1 (K, V: [n, d] fp16) with the first n_quant quantized.

    Returns a dict with, for the quantized part, per group g (tokens gG .. gG+G-1, the last group
    possibly partial): k_codes, v_codes [n_groups, G, d] (token-in-group, channel; padding codes 0),
    k_scale, k_zero [n_groups, d] per channel, v_scale, v_zero [n_groups, G] per token (padding 0),
    the dequantized K_hat, V_hat [n_quant, d] (fp64); the window k_res (raw) and v_res (rotated)
    [n_res, d]; v_rot, the rotated values of ALL tokens as the window would hold them (for the sliding value window
    of the decode oracle); and S [D, d], P [D] if adapters Wk [2, d, D/2] are given.
    mode: 'spec32' (GPU contract, fp16 storage), 'exact16' (fp64 arithmetic, fp16 storage),
    'real' (Eq. 1 in fp64 throughout, any bit width; for convergence checks only).
    state_rounding: None = S kept exactly (fp64).  Otherwise an iterable of quantized-token counts (multiples of G):
    the state is STORED in 16 bits -- the width the average-bit figures of Table 1 count it at -- and was rounded to
    binary16 each time the quantized part reached one of these counts and at n_quant (the ends of the append calls
    that flushed); between two roundings the sums of Eq. 5 run exactly.  Entries beyond +-65504 saturate.
    """
    K = np.asarray(K)
    V = np.asarray(V)
    n, d = K.shape
    assert V.shape == (n, d) and 0 <= n_quant <= n
    assert d == G, "token-wise value groups span the whole head dimension here (d = G)"
    if not rotate:
        Vr = V
    elif mode == "spec32":
        Vr = hadamard.fwht_spec32(V)
    elif mode == "exact16":
        Vr = hadamard.rotate_exact_fp16(V)
    else:
        Vr = hadamard.rotate_exact(V)
    store = np.float64 if mode == "real" else np.float16
    n_groups = -(-n_quant // G)
    out = {
        "n": n, "n_quant": n_quant, "n_res": n - n_quant, "G": G, "d": d, "bits": bits,
        "k_codes": np.zeros((n_groups, G, d), dtype=np.uint8 if bits <= 8 else np.int64),
        "v_codes": np.zeros((n_groups, G, d), dtype=np.uint8 if bits <= 8 else np.int64),
        "k_scale": np.zeros((n_groups, d), dtype=store), "k_zero": np.zeros((n_groups, d), dtype=store),
        "v_scale": np.zeros((n_groups, G), dtype=store), "v_zero": np.zeros((n_groups, G), dtype=store),
        "K_hat": np.zeros((n_quant, d)), "V_hat": np.zeros((n_quant, d)),
        "k_res": K[n_quant:].copy(), "v_res": Vr[n_quant:].copy(), "v_rot": np.asarray(Vr).copy(),
    }
    for g in range(n_groups):
        t0, t1 = g * G, min((g + 1) * G, n_quant)
        m = t1 - t0
        # keys: channel-wise Q_C -- one group per channel, running over the group's tokens
        ck, sk, zk = _quantize_rows(K[t0:t1].T, bits, mode)
        out["k_codes"][g, :m] = ck.T
        out["k_scale"][g], out["k_zero"][g] = sk, zk
        out["K_hat"][t0:t1] = quantizer.dequantize(ck, sk, zk).T
        # values: token-wise Q_T of the rotated value -- one group per token
        cv, sv, zv = _quantize_rows(Vr[t0:t1], bits, mode)
        out["v_codes"][g, :m] = cv
        out["v_scale"][g, :m], out["v_zero"][g, :m] = sv, zv
        out["V_hat"][t0:t1] = quantizer.dequantize(cv, sv, zv)
    if Wk is not None:
        D = 2 * np.asarray(Wk).shape[-1]
        if n_quant:
            K_err = K[:n_quant].astype(np.float64) - out["K_hat"]
            phi_k = feature_map(K_err, Wk)
            if state_rounding is None:
                out["S"] = phi_k.T @ out["V_hat"]
            else:
                cuts = sorted({int(c) for c in state_rounding if 0 < int(c) < n_quant} | {n_quant})
                assert all(c % G == 0 for c in cuts[:-1])
                S, prev = np.zeros((D, d)), 0
                for cut in cuts:
                    S = S + phi_k[prev:cut].T @ out["V_hat"][prev:cut]
                    S = np.clip(S, -65504.0, 65504.0).astype(np.float16).astype(np.float64)
                    prev = cut
                out["S"] = S
            out["P"] = phi_k.sum(axis=0)
        else:
            out["S"] = np.zeros((D, d))
            out["P"] = np.zeros(D)
    return out
