"""Single-query attention over the quantized cache with the linear correction (Sec. 3.2-3.3).

    Y_hat = ( sum_i exp(q K^q_i / sqrt d) V^q_i + phi_q(q) S ) / ( sum_i exp(q K^q_i / sqrt d) + phi_q(q) P )   (Eq. 5)

where i runs over the quantized tokens AND the fp16 window (whose keys are exact, so they add
plain exp terms and nothing to S, P).  Everything is accumulated in the rotated value basis and
one multiplication by H^T returns to the original basis.

The correction terms are added to the UNSHIFTED exponential sums, as Eq. 5 defines them.  With
M = max_i score_i the same quotient is (num + e^{-M} C_n) / (den + e^{-M} C_d) for the shifted sums
num, den; Alg. 1 prints C_n, C_d added to the shifted sums without that factor, which is kept
here only as the switch ``literal_alg1`` so its distance from Eq. 5 can be reported.

Value window (Sec. 4.1, setup: the most recent tokens stay in full precision).  Keys are quantized per channel over
128 tokens, so they can only leave the window a block at a time; values are quantized per token, so they can leave
one at a time.  ``value_window="block"``: values leave with the keys (the window holds the n_res newest tokens of
both).  ``value_window="sliding"``: the values of the newest ``R`` tokens are always the fp16 ones, those of all older
tokens the quantized ones, whatever the key window holds.  The states S, P are the same in both (they are sums over
the key-quantized tokens of their quantized values).
"""
import numpy as np

from . import hadamard
from .kvcache import feature_map


def _operands(cache, value_window="block", R=128):
    keys = np.concatenate([cache["K_hat"], cache["k_res"].astype(np.float64)], axis=0)
    vals = np.concatenate([cache["V_hat"], cache["v_res"].astype(np.float64)], axis=0)
    if value_window == "sliding":
        n, nq = cache["n"], cache["n_quant"]
        assert n - nq <= R, "the key window is never longer than the value window"
        first = max(0, n - R)  # the values of tokens first .. n-1 are the fp16 ones
        vals[first:] = cache["v_rot"][first:].astype(np.float64)
    else:
        assert value_window == "block"
    return keys, vals


def correction_terms(q, cache, Wq):
    """C_n = phi_q(q) S, C_d = phi_q(q) P (Sec. 3.3)."""
    phi_q = feature_map(np.asarray(q, dtype=np.float64)[None, :], Wq)[0]
    return phi_q @ cache["S"], float(phi_q @ cache["P"])


def decode(q, cache, Wq=None, *, rotate=True, literal_alg1=False, value_window="block"):
    """Eq. 5 for one query row q [d]; returns y [d] in the original basis (fp64).

    Wq: [2, d, D/2] adapters of this query head, or None for plain quantized attention (Eq. 3 on
    the dequantized operands).
    """
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[0]
    keys, vals = _operands(cache, value_window)
    score = keys @ q / np.sqrt(float(d))
    M = score.max()
    e = np.exp(score - M)
    num = e @ vals
    den = e.sum()
    if Wq is not None:
        C_n, C_d = correction_terms(q, cache, Wq)
        if literal_alg1:
            num, den = num + C_n, den + C_d
        else:
            Ms = max(M, 0.0)  # keep both factors <= 1
            num = np.exp(M - Ms) * num + np.exp(-Ms) * C_n
            den = np.exp(M - Ms) * den + np.exp(-Ms) * C_d
    y_rot = num / den
    return y_rot @ hadamard.orthonormal(d).T if rotate else y_rot


def decode_unshifted(q, cache, Wq, *, rotate=True):
    """Eq. 5 typed literally (no max subtraction).  Only safe for moderate scores; used as a pin."""
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[0]
    keys, vals = _operands(cache)
    w = np.exp(keys @ q / np.sqrt(float(d)))
    phi_q = feature_map(q[None, :], Wq)[0]
    y_rot = (w @ vals + phi_q @ cache["S"]) / (w.sum() + phi_q @ cache["P"])
    return y_rot @ hadamard.orthonormal(d).T if rotate else y_rot


def decode_quadratic(q, K16, cache, Wq, Wk, *, rotate=True):
    """Eq. 4: the correction written as sum_i f(q, K^e_i) V^q_i with f = phi_q(q) phi_k(K^e_i)^T,
    summed token by token over the quantized tokens (no states)."""
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[0]
    keys, vals = _operands(cache)
    w = np.exp(keys @ q / np.sqrt(float(d)))
    nq = cache["n_quant"]
    K_err = np.asarray(K16[:nq], dtype=np.float64) - cache["K_hat"]
    phi_q = feature_map(q[None, :], Wq)[0]
    f = np.array([phi_q @ feature_map(K_err[i][None, :], Wk)[0] for i in range(nq)])
    num = w @ vals + (f @ cache["V_hat"] if nq else 0.0)
    den = w.sum() + f.sum()
    y_rot = num / den
    return y_rot @ hadamard.orthonormal(d).T if rotate else y_rot


def decode_blocks(q, cache, Wq=None, *, boundaries=None, rotate=True):
    """Alg. 1: independent blocks of tokens each produce (Y_s^j, m^j, l^j); the merge weighs them by
    w = exp(m - max m), adds the correction (with the Eq. 5 factor) and divides.

    boundaries: increasing token indices that cut [0, n) into blocks; default = one block per
    quantization group plus one for the window.
    """
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[0]
    keys, vals = _operands(cache)
    n = keys.shape[0]
    if boundaries is None:
        G, nq = cache["G"], cache["n_quant"]
        boundaries = list(range(G, nq, G)) + ([nq] if 0 < nq < n else [])
    cuts = [0] + [b for b in boundaries if 0 < b < n] + [n]
    Ys, m, l = [], [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        s = keys[a:b] @ q / np.sqrt(float(d))
        mj = s.max()
        e = np.exp(s - mj)
        Ys.append(e @ vals[a:b])
        m.append(mj)
        l.append(e.sum())
    Ys, m, l = np.array(Ys), np.array(m), np.array(l)
    M = m.max()
    w = np.exp(m - M)
    num = (Ys * w[:, None]).sum(axis=0)
    den = float(l @ w)
    if Wq is not None:
        C_n, C_d = correction_terms(q, cache, Wq)
        num = num + np.exp(-M) * C_n
        den = den + np.exp(-M) * C_d
    y_rot = num / den
    return y_rot @ hadamard.orthonormal(d).T if rotate else y_rot


def softmax_attention(q, K, V):
    """Textbook Eq. 3 for the last row: softmax(q K^T / sqrt d) V on unquantized operands (fp64)."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    s = K @ q / np.sqrt(float(q.shape[0]))
    e = np.exp(s - s.max())
    return (e / e.sum()) @ V
