"""Asymmetric N-bit integer quantization with min/max scaling (Sec. 2, Eq. 1).

    X_I = round((X - z) / s),   s = (max X - min X) / (2^N - 1),   z = min X,   Q(X) = s X_I + z

Every routine quantizes along the LAST axis: one row = one group sharing (s, z).  Channel-wise
Q_C of a [tokens, channels] block is ``quantize(block.T)``, token-wise Q_T is ``quantize(block)``
(Sec. 2, Fig. 1).
"""
import numpy as np


def quantize_real(x, bits):
    """Eq. 1 verbatim in fp64: returns (codes int64, s fp64, z fp64).  s == 0 -> codes 0."""
    x = np.asarray(x, dtype=np.float64)
    levels = float(2 ** bits - 1)
    z = x.min(axis=-1)
    s = (x.max(axis=-1) - z) / levels
    safe = np.where(s == 0.0, 1.0, s)
    codes = np.rint((x - z[..., None]) / safe[..., None])  # round half to even
    codes = np.clip(codes, 0.0, levels)
    codes = np.where(s[..., None] == 0.0, 0.0, codes)
    return codes.astype(np.int64), s, z


def quantize_exact16(x16, bits=2):
    """Eq. 1 with the scale and zero-point stored as fp16 (rounded once from fp64).

    Codes are taken against the STORED values so that s16 * code + z16 is what the cache decodes
    to.  Arithmetic is fp64.  Returns (codes int64, s16, z16).
    """
    x = np.asarray(x16, dtype=np.float16).astype(np.float64)
    levels = float(2 ** bits - 1)
    mn = x.min(axis=-1)
    mx = x.max(axis=-1)
    z16 = (mn + 0.0).astype(np.float16)
    z16 = np.where(z16 == 0, np.float16(0.0), z16)
    s16 = ((mx - mn) / levels).astype(np.float16)
    s = s16.astype(np.float64)
    safe = np.where(s == 0.0, 1.0, s)
    codes = np.rint((x - z16.astype(np.float64)[..., None]) / safe[..., None])
    codes = np.clip(codes, 0.0, levels)
    codes = np.where(s[..., None] == 0.0, 0.0, codes)
    return codes.astype(np.int64), s16, z16


def quantize_spec32(x16, bits=2):
    """The quantizer the GPU is held to bit for bit (inputs fp16, one group per row), N = ``bits`` in {2, 4}, L = 2^N - 1:

      mn, mx  = min, max of the group (exact); a zero of either sign counts as +0
      z16     = mn
      d32     = fl32(mx - mn)
      s16     = fp16(fl32(d32 / L))
      t       = fl32(x - z16)
      code    = number of k in 0 .. L-1 with  t > (k + 0.5) s16  (k even)  or  t >= (k + 0.5) s16  (k odd)
                [s16 == 0 -> code 0];  for N = 2:  (t > 0.5 s16) + (t >= 1.5 s16) + (t > 2.5 s16)

    The thresholds (k + 0.5) s16 are exact in binary32 (an 11-bit significand times an odd number below 32), so
    ``code`` is round-half-to-even of the real quotient t / s16 clamped to [0, L]: Eq. 1 against the stored scale,
    without a division.  Returns (codes uint8, s16, z16).
    """
    assert bits in (2, 4)
    L = 2 ** bits - 1
    x16 = np.asarray(x16, dtype=np.float16)
    f32 = np.float32
    x = x16.astype(f32)
    mn = x.min(axis=-1)
    mx = x.max(axis=-1)
    mn = np.where(mn == 0, f32(0.0), mn).astype(f32)
    mx = np.where(mx == 0, f32(0.0), mx).astype(f32)
    z16 = mn.astype(np.float16)  # exact: mn is an fp16 value
    d32 = (mx - mn).astype(f32)
    s16 = (d32 / f32(L)).astype(f32).astype(np.float16)
    s = s16.astype(f32)[..., None]
    t = (x - mn[..., None]).astype(f32)
    code = np.zeros(t.shape, dtype=np.uint8)
    for k in range(L):
        thr = (f32(k + 0.5) * s).astype(f32)
        code += (t >= thr).astype(np.uint8) if k % 2 else (t > thr).astype(np.uint8)
    code = np.where(s == 0, np.uint8(0), code).astype(np.uint8)
    return code, s16, z16


def dequantize(codes, s, z):
    """Q(X) = s X_I + z in fp64 (rows share s, z)."""
    s = np.asarray(s).astype(np.float64)
    z = np.asarray(z).astype(np.float64)
    return s[..., None] * np.asarray(codes, dtype=np.float64) + z[..., None]
