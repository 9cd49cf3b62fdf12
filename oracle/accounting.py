"""Average bits per cached key/value element (Table 1, column "KV Cache").

Counted per (sequence, kv head) at context n: N-bit codes for the quantized tokens, a 16-bit scale
and a 16-bit zero-point per group of G codes, 16 bits per element of the full-precision window of
the `window` most recent tokens (Sec. 4.1), and -- for KVLinC -- the correction states
S in R^{D x d} and P in R^{D} (Sec. 3.2), which do not grow with n.
"""


def bits_per_element_quantized(bits, group):
    return bits + 2.0 * 16.0 / group


def average_bits(n, bits=2, group=128, window=128, d=128, D=0, state_bits=16):
    """Average over the 2*n*d stored elements (keys and values) of one kv head."""
    n_q = max(n - window, 0)
    n_w = n - n_q
    per_tensor = n_q * d * bits_per_element_quantized(bits, group) + n_w * d * 16.0
    total = 2.0 * per_tensor
    if D:
        total += (D * d + D) * float(state_bits)
    return total / (2.0 * n * d)


def fp16_cache_bytes(layers, kv_heads, d, n, batch):
    return layers * 2 * kv_heads * d * n * batch * 2
