"""Seeded synthetic inputs shaped like the paper's workloads (Llama-3-8B / Qwen2.5-7B attention
layers, Sec. 4.1 and 4.4).  Input generation only: none of the method's arithmetic lives here, so
both the CPU reference and the GPU library can be fed from it.

Distributions: q, k, v ~ N(0, 1) rounded to fp16; each KV head has 4 outlier channels (a seeded
choice that depends on the head only) whose keys are multiplied by 8 -- the channel-wise key
outliers the paper describes (Sec. 3.1, Fig. 2); values have none.  Adapter weights ~ N(0, 1/128)
in fp16, W_q per query head and W_k per KV head, each [2, 128, 128] (Eq. 6 with D = 256).

Every (tensor, sequence, head) draws from its own counter-free stream
``default_rng([BASE_SEED, 100 * config + tensor_id, sequence, head])`` so that any slice can be
regenerated on its own.
"""
import numpy as np

BASE_SEED = 20251005
T_Q, T_K, T_V, T_WQ, T_WK, T_LEN, T_OUTLIER = 1, 2, 3, 4, 5, 6, 7
HEAD_DIM = 128
RANK_D = 256
N_OUTLIER = 4
OUTLIER_GAIN = 8.0

# The workloads: B sequences, H_q query heads, H_kv KV heads, context n (tokens already in the
# cache when the query arrives), R window capacity, keep = fp16 tokens a bulk build leaves
# (None = the lazy block flush).
CONFIGS = {
    1: dict(name="c1_b1_ctx1k", B=1, H_q=32, H_kv=8, n=1024, R=32, keep=32),
    2: dict(name="c2_llama3_8b_b16_ctx8k", B=16, H_q=32, H_kv=8, n=8192, R=128, keep=None),
    3: dict(name="c3_b1_ctx128k", B=1, H_q=32, H_kv=8, n=131072, R=128, keep=None),
    4: dict(name="c4_qwen25_7b_b32_ctx32k", B=32, H_q=28, H_kv=4, n=32768, R=128, keep=None),
    5: dict(name="c5_ragged_b64_append", B=64, H_q=32, H_kv=8, n=None, n_min=1024, n_max=16384, steps=256,
            R=128, keep=None),
    # Two shapes of the paper's end-to-end throughput experiment (Sec. 4.4: prompt 256 + 1024 generated tokens):
    # a multi-head model (one query head per KV head) and the grouped-query model at a large batch.
    6: dict(name="c6_llama2_7b_mha_b32_ctx1280", B=32, H_q=32, H_kv=32, n=1280, R=128, keep=None),
    7: dict(name="c7_llama3_8b_b144_ctx1280", B=144, H_q=32, H_kv=8, n=1280, R=128, keep=None),
}


def _rng(config, tensor, seq=0, head=0):
    return np.random.default_rng([BASE_SEED, 100 * config + tensor, seq, head])


def outlier_channels(config, kv_head):
    return np.sort(_rng(config, T_OUTLIER, 0, kv_head).choice(HEAD_DIM, size=N_OUTLIER, replace=False))


def keys(config, seq, kv_head, n):
    """[n, 128] fp16 keys of one (sequence, kv head)."""
    k = _rng(config, T_K, seq, kv_head).standard_normal((n, HEAD_DIM), dtype=np.float32)
    k[:, outlier_channels(config, kv_head)] *= np.float32(OUTLIER_GAIN)
    return k.astype(np.float16)


def values(config, seq, kv_head, n):
    """[n, 128] fp16 values of one (sequence, kv head)."""
    return _rng(config, T_V, seq, kv_head).standard_normal((n, HEAD_DIM), dtype=np.float32).astype(np.float16)


def queries(config, seq, H_q, step=0):
    """[H_q, 128] fp16 queries of one sequence at one decode step."""
    return _rng(config, T_Q, seq, step).standard_normal((H_q, HEAD_DIM), dtype=np.float32).astype(np.float16)


def adapters_q(config, H_q):
    """[H_q, 2, 128, 128] fp16: W_1, W_2 of phi_q for every query head."""
    w = _rng(config, T_WQ).standard_normal((H_q, 2, HEAD_DIM, RANK_D // 2), dtype=np.float32)
    return (w * np.float32(1.0 / np.sqrt(128.0))).astype(np.float16)


def adapters_k(config, H_kv):
    """[H_kv, 2, 128, 128] fp16: W_1, W_2 of phi_k for every KV head."""
    w = _rng(config, T_WK).standard_normal((H_kv, 2, HEAD_DIM, RANK_D // 2), dtype=np.float32)
    return (w * np.float32(1.0 / np.sqrt(128.0))).astype(np.float16)


def ragged_lengths(config, B, n_min, n_max):
    """[B] int32 context lengths, uniform in [n_min, n_max]."""
    return _rng(config, T_LEN).integers(n_min, n_max + 1, size=B).astype(np.int32)
