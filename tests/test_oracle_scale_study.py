"""Oracle-only study of the quantization scale factors on the synthetic keys (Sec. 3.1, Obs. 1-3 and the figure of
layer-wise scale factors): which axis and which placement of the Hadamard matrix give the smaller scale s of Eq. 1 --
and with it, by Eq. 2, the smaller error -- when keys carry a few outlier channels and values carry none.

The paper measures this on Llama / Qwen activations; here the keys are kvlinc_synth's (N(0, 1) with 4 channels per head
scaled by 8), 2-bit, groups of 128.  What is asserted is the ORDER the observations state, on the median scale over all
groups of 8 KV heads; magnitudes are printed.  No GPU."""
import numpy as np

import kvlinc_synth as synth
from oracle import hadamard, quantizer


def _median_scales():
    H = hadamard.orthonormal(128)
    out = {}
    for g in range(8):
        K = synth.keys(2, 0, g, 2048).astype(np.float64).reshape(-1, 128, 128)    # [group, token, channel]
        V = synth.values(2, 0, g, 2048).astype(np.float64).reshape(-1, 128, 128)

        def scale(x, axis):
            rows = x.transpose(0, 2, 1) if axis == "C" else x  # Q_C: one group per channel over the tokens; Q_T: per token
            _, s, _ = quantizer.quantize_real(rows, 2)
            return s.reshape(-1)

        post, pre = K @ H, np.einsum("st,gtc->gsc", H, K)  # K H rotates the channels of a token; H K mixes the tokens
        cases = {"Q_C(K)": scale(K, "C"), "Q_T(K)": scale(K, "T"), "Q_T(KH)": scale(post, "T"), "Q_C(KH)": scale(post, "C"),
                 "Q_T(HK)": scale(pre, "T"), "Q_C(HK)": scale(pre, "C"), "Q_T(V)": scale(V, "T"), "Q_T(VH)": scale(V @ H, "T")}
        for name, s in cases.items():
            out.setdefault(name, []).append(s)
    return {name: float(np.median(np.concatenate(s))) for name, s in out.items()}


def test_scale_factors_follow_observations_1_to_3():
    m = _median_scales()
    print("  [scale study] median scale per configuration:", {k: round(v, 3) for k, v in m.items()})
    # Obs. 2: rotating the keys lowers the token-wise scale, but it stays well above the channel-wise scale of raw keys
    assert m["Q_T(KH)"] < 0.6 * m["Q_T(K)"]
    assert m["Q_T(KH)"] > 1.3 * m["Q_C(K)"]
    assert m["Q_T(K)"] > 2.5 * m["Q_C(K)"]
    # Obs. 3: rotating the keys spreads every outlier channel over all channels and RAISES the channel-wise scale
    assert m["Q_C(KH)"] > 1.4 * m["Q_C(K)"]
    assert m["Q_C(K)"] == min(m[k] for k in ("Q_C(K)", "Q_T(K)", "Q_T(KH)", "Q_C(KH)", "Q_T(HK)"))
    # Obs. 1: pre-multiplication mixes tokens, not channels -- the outlier channels survive it, so token-wise groups
    # keep the large scale that post-multiplication removes (and channel-wise groups gain nothing from it)
    assert abs(m["Q_T(HK)"] - m["Q_T(K)"]) < 0.1 * m["Q_T(K)"]
    assert m["Q_T(HK)"] > 1.6 * m["Q_T(KH)"]
    assert abs(m["Q_C(HK)"] - m["Q_C(K)"]) < 0.1 * m["Q_C(K)"]
    # values have no outliers here: the rotation neither helps nor hurts their token-wise scale
    assert abs(m["Q_T(VH)"] - m["Q_T(V)"]) < 0.05 * m["Q_T(V)"]


def test_pre_multiplication_injects_the_error_of_other_tokens():
    """Obs. 1's explanation: with H K the quantization error of a token's key is a mix of the errors of all tokens of its
    group after the inverse rotation, so the error of one attention logit no longer depends on that token's own
    quantization alone.  Measured as the correlation between |logit error| and the token's own scale: present for K H
    (post), absent for H K (pre)."""
    H = hadamard.orthonormal(128)
    rng = np.random.default_rng(0)
    K = synth.keys(2, 1, 3, 128).astype(np.float64)
    K *= rng.uniform(0.2, 3.0, size=(128, 1))  # tokens of different magnitude: their token-wise scales differ
    q = synth.queries(2, 1, 32)[12].astype(np.float64)

    def logit_error(rotated, back):
        codes, s, z = quantizer.quantize_real(rotated, 2)      # token-wise: one group per row
        return back(quantizer.dequantize(codes, s, z)) @ q - K @ q, s

    e_post, s_post = logit_error(K @ H, lambda x: x @ H.T)
    e_pre, s_pre = logit_error(H @ K, lambda x: H.T @ x)
    own = np.corrcoef(np.abs(e_post), s_post)[0, 1]
    mixed = np.corrcoef(np.abs(e_pre), np.linalg.norm(K, axis=1))[0, 1]
    print("  [scale study] corr(|logit error|, own scale): post %.2f, pre (against the token's own norm) %.2f" % (own, mixed))
    assert own > 0.3 and abs(mixed) < 0.2
