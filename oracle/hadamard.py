"""Hadamard rotation of values: V -> V H with H orthogonal (Sec. 3.1; inverse H^T).

H = H_sylv / sqrt(d), H_sylv[i, j] = (-1)^popcount(i & j) (Sylvester construction, natural
order).  H is symmetric and its own inverse.
"""
import numpy as np

INV_SQRT_128_F32 = np.float32(float.fromhex("0x1.6a09e6p-4"))  # fl32(1/sqrt(128))


def sylvester(d):
    """The +-1 Sylvester-Hadamard matrix of order d (d a power of two), as fp64."""
    assert d > 0 and d & (d - 1) == 0
    i = np.arange(d)
    and_ij = i[:, None] & i[None, :]
    pop = np.zeros((d, d), dtype=np.int64)
    b = and_ij.copy()
    while b.any():
        pop += b & 1
        b >>= 1
    return np.where(pop & 1, -1.0, 1.0)


def orthonormal(d):
    """H = H_sylv / sqrt(d): H H^T = I."""
    return sylvester(d) / np.sqrt(float(d))


def rotate_exact(v):
    """v H in fp64 (v: [..., d])."""
    v = np.asarray(v, dtype=np.float64)
    return v @ orthonormal(v.shape[-1])


def rotate_exact_fp16(v):
    """fp64 rotation rounded once to fp16: what an ideal fp16 producer of V H would store."""
    return rotate_exact(v).astype(np.float16)


def fwht_spec32(v16):
    """The rotated fp16 value the GPU must store, bit for bit.

    Dataflow (binary32, one rounding per add/sub, no fused operations):
      x = float(v);  for h = 1, 2, 4, ..., d/2:  for every i with (i & h) == 0:
          (x[i], x[i+h]) <- (x[i] + x[i+h],  x[i] - x[i+h])
      out = fp16( fl32( x * fl32(1/sqrt(d)) ) )
    Only d = 128 has its scale constant fixed here.
    """
    v16 = np.asarray(v16, dtype=np.float16)
    d = v16.shape[-1]
    assert d == 128, "the binary32 scale constant is fixed for d = 128"
    x = v16.astype(np.float32).copy()
    idx = np.arange(d)
    h = 1
    while h < d:
        lo = idx[(idx & h) == 0]
        a = x[..., lo]
        b = x[..., lo + h]
        s = (a + b).astype(np.float32)
        t = (a - b).astype(np.float32)
        x[..., lo] = s
        x[..., lo + h] = t
        h *= 2
    y = (x * INV_SQRT_128_F32).astype(np.float32)
    return y.astype(np.float16)
