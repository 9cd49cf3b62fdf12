/*
 * kvlinc.h -- C ABI of the KVLinC 2-bit KV-cache decode path for AMD MI355X (gfx950).
 *
 * The library implements, for one attention layer and one decode step, what Sec. 3 of the paper
 * (arxiv 2510.05373) defines:
 *   - keys quantized per channel, K_q = Q_C(K), values Hadamard-rotated and quantized per token,
 *     V_q = Q_T(V H), both at 2 bits (or at 4: `bits` of the cache descriptor) with group size 128 (Sec. 3.1, Obs. 3; quantizer: Sec. 2, Eq. 1);
 *   - the 128 most recent tokens kept in fp16 and quantized only after attention has used them
 *     (Sec. 4.1 "Setup"; Sec. 3.3, last sentence);
 *   - the linear correction states S, P of the key quantization error (Sec. 3.2, Eq. 4-6);
 *   - single-query attention read directly from the packed cache, split over blocks of tokens and
 *     merged, with the correction added (Sec. 3.3, Alg. 1; Eq. 5).
 *
 * Conventions
 *   - Every pointer inside kvlinc_cache and every tensor argument is a DEVICE pointer owned by the
 *     caller, 16-byte aligned.  The library allocates nothing, keeps no state between calls (but for the address
 *     of its static scratch buffer, see kvlinc_decode_attention_noalloc) and never synchronises: a call validates its
 *     arguments on the host, enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the default stream)
 *     and returns.
 *   - kvlinc_half is the bit pattern of an IEEE binary16 number.
 *   - Return value: 0 = enqueued; negative = rejected before any launch, nothing was touched.
 *   - Faults only the device can see (capacity exhausted, non-finite input, append to a cache whose
 *     last group is partial) set bits in *status and leave that sequence unchanged: its counters, its live group
 *     records and window rows, and its states S, P, S16 (in all KV heads) are bit for bit what they were.  Storage
 *     beyond the counters (group records from n_quant / 128 on, window slots from n_res on -- key slots only when
 *     KVLINC_FLAG_SLIDING_VALUES is set, see flags) is dead and may have been overwritten; a non-finite value is never
 *     stored into the window.
 *   - Magnitudes: the operands of the matrix products carry a block exponent per group and query head, so keys,
 *     queries and values of any finite binary16 magnitude neither overflow nor flush; each operand keeps 2^-12 of
 *     the group's largest one.  A logit is therefore off by up to about 1e-3 of the group's largest |logit|: the
 *     output tolerance holds for logits of a few tens (the paper's workloads) whatever the scale of K, V and q
 *     taken alone, and for any scale of the values; when keys and queries are scaled up together so that logits
 *     reach the hundreds while several tokens stay nearly tied for the maximum, the softmax itself is
 *     ill-conditioned and single rows have come out at 3e-3 relative (tolerance 2e-3).  What can leave its range is
 *     the 16-bit copy of the state: an entry of S beyond +-65504 is stored saturated and reported as
 *     KVLINC_ST_STATE_RANGE (S grows with the context when the rotated values have a common sign).
 *   - Query head h reads KV head h / (H_q / H_kv).  The softmax scale is 1/sqrt(d) (Eq. 3).
 *
 * Cache layout (per sequence b, KV head g; "group" = 128 consecutive tokens from token 0):
 *   groups            [B, H_kv, max_groups, 2304] uint32: one 9216-byte record per group, everything a decode step
 *                     reads of that group, contiguous:
 *                       words    0..1023  key tile,   2-bit codes of the 128x128 block
 *                       words 1024..2047  value tile, 2-bit codes of the 128x128 block of ROTATED values
 *                       words 2048..2111  key scale s of Eq. 1, fp16 per channel 0..127 (channel 2i in the low half)
 *                       words 2112..2175  key zero-point z, fp16 per channel
 *                       words 2176..2303  value (s, z) of token t = 16 n + j in word 2176 + 8 j + n: s in the low half, z in
 *                                         the high
 *                     Logical content of a tile: code(token, channel) in {0..3}.  Both tiles share one word order, made
 *                     for the 16x16x128 matrix-core instruction that consumes them: a tile has 8 blocks n of 16 "rows"
 *                     j, and every row has 128 contraction positions k, cut into 4 quarters g of 32.  The two words
 *                     w = 0, 1 of (n, j, g) sit at word index ((n / 2) * 64 + j + 16 * g) * 4 + 2 * (n % 2) + w.  A word holds
 *                     16 codes p = 0..15, code p at position k = 32 g + 16 w + 8 (p % 2) + p / 2, two codes per nibble:
 *                     code c is stored as the bit pair (hi, lo) = (1,1), (1,0), (0,0), (0,1) for c = 0, 1, 2, 3, with
 *                     hi in bit 4 (p / 2) + 3 - p % 2 and lo in bit 4 (p / 2) + 1 - p % 2.  (With the nibble's other two
 *                     bits forced to 0 and 1, the nibble sign|0|lo|1 is the FP4 E2M1 number c - 1.5.)
 *                     Key tile:   row (n, j) = token 16 n + j, position k = channel k.
 *                     Value tile: row (n, j) = channel 16 n + j, position k = token
 *                                 16 (k % 8) + 4 ((k / 16) % 4) + 2 (k / 64) + (k / 8) % 2.
 *                     A partial last group (bulk build only) has zero codes and zero (s, z) for its missing tokens.
 *                     bits == 4 (Eq. 1 at N = 4, 16 levels): groups is [B, H_kv, max_groups, 4352] uint32, one 17408-byte
 *                     record per group.  A code c = 4 c_hi + c_lo is stored as two 2-bit codes in two 2-bit tiles
 *                     ("planes") of the order and bit pairs above:
 *                       words    0..1023  key tile, high plane (c_hi)      words 1024..2047  key tile, low plane (c_lo)
 *                       words 2048..3071  value tile, high plane           words 3072..4095  value tile, low plane
 *                       words 4096..4159  key scale   words 4160..4223  key zero-point   words 4224..4351  value (s, z),
 *                     the last three fields in the order of the 2-bit record.  (c - 7.5 = 4 (c_hi - 1.5) + (c_lo - 1.5):
 *                     the decode step contracts with the two planes in turn, the high one under a block scale of 4.)
 *   k_res             [B, H_kv, R, 128] fp16: the window's raw keys, slot r = r-th oldest window token.
 *   v_res             [B, H_kv, R/4, 128, 4] fp16: the window's ROTATED values, 4 consecutive slots per channel:
 *                     slot r, channel c at [r/4][c][r%4].
 *   n_quant, n_res    [B] int32: quantized tokens / window tokens of each sequence (context = sum).
 *   S, P              [B, H_kv, D, 128], [B, H_kv, D] fp32 correction states (Eq. 5), rotated value basis.  S is the
 *                     optional fp32 master copy that kvlinc_append_quantize accumulates into; with S == NULL the
 *                     state is STORED in 16 bits only (S16 below, the storage the paper's average-bit figures of
 *                     Table 1 assume): an append that flushes then starts from the binary16 state, accumulates the
 *                     groups of that call in binary32 and rounds once at the end of the call.  P is always fp32.
 *   S16               [B, H_kv, 128, 64, 4] fp16: S in binary16, rewritten by every append that flushes a group and
 *                     read by kvlinc_decode_attention.  Tile t = (f / 64 * 2 + c / 64) * 16 + (f % 64) / 4 holds
 *                     S[f][c] at [t][c % 64][f % 4]  (f = feature 0..255, c = channel 0..127).
 *   Wq, Wk            [H_q, 2, 128, D/2], [H_kv, 2, 128, D/2] fp16: W_1, W_2 of phi_q / phi_k (Eq. 6).
 *                     S16, P, Wq, Wk all NULL (and S NULL) = correction off (plain quantized attention).
 *   flags             KVLINC_FLAG_* bits.  KVLINC_FLAG_ALG1_LITERAL: the merge adds C_n, C_d to the max-shifted sums
 *                     as the last lines of Alg. 1 print them, (num + C_n) / (den + C_d), instead of Eq. 5's
 *                     (num + e^-M C_n) / (den + e^-M C_d) (the two differ by the factor e^-M, M = largest score).
 *                     KVLINC_FLAG_SLIDING_VALUES (Sec. 4.1, setup: the most recent 128 tokens in full precision):
 *                     keys can only leave the fp16 window a group at a time (they are quantized per channel over 128
 *                     tokens), values are quantized per token and leave one at a time: the decode step takes the
 *                     fp16 rotated values of the newest 128 tokens and the quantized values of all older ones,
 *                     whatever n_res is.  The value of token t lives in window slot t % 128: the slots n_res..127 of
 *                     v_res then hold the values of the last 128 - n_res tokens of the newest group and are live (an
 *                     incremental append leaves them there anyway; a bulk append stores them when the flag is set).
 *                     The states and the records are the same with and without the flag.  Needs R = 128 and
 *                     keep_residual = 0; set it when the cache is created and keep it.
 *   status            [1] int32, OR-ed KVLINC_ST_* bits.
 *   split_done        [B, H_kv] int32 scratch counters (arrival counts: of the workgroups of a (sequence, KV head)
 *                     in kvlinc_decode_attention, where the last one merges; of the workgroups of a sequence in
 *                     kvlinc_append_quantize, where the last one updates n_quant / n_res).  Zero them once after
 *                     allocation; every call leaves them at zero.  Two calls on the same cache must not overlap in
 *                     time; calls on different caches (each with a workspace of its own) may, on different streams.
 *   All cache buffers must be zero-initialised before their first use.
 *
 * Quantizer contract (bit exact; Eq. 1 taken against the stored fp16 scale and zero-point):
 *   mn, mx over the group (a zero of either sign counts as +0); z = mn; s = fp16(fl32(fl32(mx - mn) / 3));
 *   t = fl32(x - z); code = (t > 0.5 s) + (t >= 1.5 s) + (t > 2.5 s), code = 0 when s == 0.
 * Rotation contract (bit exact): x = float(v); for h = 1, 2, ..., 64: for i with (i & h) == 0:
 *   (x[i], x[i+h]) <- (x[i] + x[i+h], x[i] - x[i+h]) in binary32; out = fp16(fl32(x * 0x1.6a09e6p-4f)).
 */
#ifndef KVLINC_H
#define KVLINC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t kvlinc_half;

enum {
  KVLINC_OK = 0,
  KVLINC_EINVAL = -1,     /* NULL / misaligned pointer, unsupported shape or parameter */
  KVLINC_EWORKSPACE = -2, /* workspace too small or misaligned */
  KVLINC_EHIP = -3,       /* a HIP call failed (hipGetLastError) */
  KVLINC_ESCRATCH = -4    /* kvlinc_decode_attention_noalloc: the launch needs more scratch than the library's static buffer */
};

enum {
  KVLINC_ST_CAPACITY = 1,  /* a sequence would need more than max_groups groups */
  KVLINC_ST_NONFINITE = 2, /* a key or rotated value that was quantized is Inf or NaN */
  KVLINC_ST_STATIC = 4,    /* append to a sequence whose last group is partial, or an unsupported keep_residual */
  KVLINC_ST_STATE_RANGE = 8 /* an entry of S left the binary16 range: S16 holds +-65504 there, the correction is off */
};

enum {
  KVLINC_FLAG_ALG1_LITERAL = 1,  /* correction added without the e^-M factor (Alg. 1 as printed) */
  KVLINC_FLAG_SLIDING_VALUES = 2 /* values leave the fp16 window one token at a time (Sec. 4.1, setup) */
};

typedef struct kvlinc_cache {
  int32_t B, H_q, H_kv;
  int32_t d;    /* head dimension, must be 128 */
  int32_t G;    /* quantization group size, must be 128 */
  int32_t R;    /* window capacity in tokens, a multiple of 4 in 4..128; one-token appends need R == G */
  int32_t D;    /* rank of the correction feature maps, must be 256 */
  int32_t bits; /* width of the codes: 2 or 4 (the layout of `groups` follows it) */
  int64_t max_groups; /* tile capacity per (sequence, KV head) */
  uint32_t* groups;
  kvlinc_half* k_res;
  kvlinc_half* v_res;
  int32_t* n_quant;
  int32_t* n_res;
  float* S;
  kvlinc_half* S16;
  float* P;
  const kvlinc_half* Wq;
  const kvlinc_half* Wk;
  int32_t* status;
  int32_t* split_done;
  int32_t flags;
} kvlinc_cache;

/* Library version, major*10000 + minor*100 + patch. */
int kvlinc_version(void);

/* Static string for a return code of this library. */
const char* kvlinc_strerror(int code);

/* Host-only check of a cache descriptor (shapes, NULLs, alignment); touches no device memory.
 * Returns KVLINC_OK or KVLINC_EINVAL.  Every other entry point runs it first. */
int kvlinc_cache_validate(const kvlinc_cache* cache);

/*
 * Append new tokens and quantize what leaves the window (Sec. 3.3 last sentence; Sec. 3.1; Eq. 1; Eq. 5 states).
 *
 *   k_new, v_new   [B, H_kv, T, 128] fp16, raw keys and raw (unrotated) values of the new tokens.
 *   n_new          [B] int32 on the device: sequence b appends its first n_new[b] (0..T) rows; NULL = T for all.
 *                  (A value below 0 is read as 0, one above T as T: the kernels never read beyond the T rows.)
 *   T              rows per (sequence, head) in k_new / v_new, >= 1.
 *   keep_residual  0: lazy block flush -- the window is quantized as whole groups of 128 tokens only when a
 *                     token arrives and the window is already full (needs R == 128); after the call
 *                     1 <= n_res <= 128 and n_quant is a multiple of 128.
 *                  k in 1..R: bulk build that leaves exactly the k newest tokens in fp16 and quantizes all
 *                     older ones, the last group possibly partial (its scale/zero-point cover the valid
 *                     tokens only, padding codes are 0).  Such a sequence accepts no further append.
 *
 * Per flushed group: key scale / zero-point / codes per channel, value scale / zero-point / codes per token
 * of the rotated value, S += phi_k(K - K_q)^T V_q and P += sum phi_k(K - K_q) when the adapters are given.
 * New tokens that stay in the window are stored as raw key and rotated fp16 value.  One kernel launch (a bulk
 * append, T > 1, to a cache with more than one KV head or with KVLINC_FLAG_SLIDING_VALUES, or of a long prompt as
 * below, is preceded by a short launch that looks for non-finite input): the workgroup of a sequence that finishes
 * last updates n_quant / n_res, after all of them have read the old values, and only if none of them found a fault.
 *
 * Reproducibility: records, window rows and counters are the same bits in every run.  So are S, P and S16, except
 * after a bulk append of a long prompt to few sequences (T + R >= 64 groups, B * H_kv < 64, and a cache that keeps the
 * fp32 S): its groups are shared out in chunks over the chip, and the chunks' shares of S and P meet in memory by
 * atomic fp32 additions, whose order -- and with it the last bits of S, P -- differs from run to run (the same sums,
 * inside the same tolerance; one 131072-token prompt: 24 ms -> 1.8 ms).
 */
int kvlinc_append_quantize(const kvlinc_cache* cache, const kvlinc_half* k_new, const kvlinc_half* v_new,
                           const int32_t* n_new, int32_t T, int32_t keep_residual, void* stream);

/* Bytes of device scratch kvlinc_decode_attention needs for this cache when no sequence holds more than
 * max_context tokens (<= 0: the cache's full capacity).  0 on an invalid descriptor. */
size_t kvlinc_decode_workspace_bytes(const kvlinc_cache* cache, int32_t max_context);

/*
 * One decode step of corrected attention over the whole cache (Sec. 3.3, Alg. 1, with the correction of Eq. 5).
 *
 *   q            [B, H_q, 128] fp16 query of the current token (its key/value must already be appended).
 *   out          [B, H_q, 128] fp16 attention output in the original (unrotated) value basis.
 *   workspace    device scratch of at least kvlinc_decode_workspace_bytes(cache, max_context) bytes,
 *                16-byte aligned; contents undefined before and after.
 *   max_context  host-side upper bound on n_quant + n_res over the batch (<= 0: capacity).  It only sizes the
 *                launch; results do not depend on it as long as it is an upper bound.
 *
 * out[b, h] = ( sum_i exp(q K_i / sqrt d) V_i + phi_q(q) S ) / ( sum_i exp(q K_i / sqrt d) + phi_q(q) P ) H^T
 * with K_i, V_i the dequantized codes for quantized tokens and the fp16 window entries otherwise.
 * A sequence with no tokens yields zeros.
 *
 * One kernel launch: blocks of groups are processed by separate workgroups that leave (max, sum, numerator) partials
 * in the workspace (Alg. 1, the per-block outputs); the workgroup of a (sequence, KV head) that finishes last, counted
 * in cache->split_done, merges them, adds the correction and writes `out`.  The number of blocks of a sequence follows
 * max_context and the sequence's share of the batch's tokens, so results are deterministic (bit for bit) for a given
 * max_context and given lengths of the sequences of the batch; across different bounds or batch compositions they
 * agree up to the summation order.
 */
int kvlinc_decode_attention(const kvlinc_cache* cache, const kvlinc_half* q, kvlinc_half* out, void* workspace,
                            size_t workspace_bytes, int32_t max_context, void* stream);

/*
 * kvlinc_decode_attention with the kernel's own start and stop time stamps (Sec. 3.3, Alg. 1, as above): start_event
 * and stop_event are hipEvent_t handles (created by the caller with timing enabled, both non-NULL) that the runtime
 * attaches to the dispatch of the decode kernel, so that hipEventElapsedTime(start, stop) after completion is the
 * kernel's execution time without the gaps that separately recorded events add.  For profiling; results are the same.
 */
int kvlinc_decode_attention_timed(const kvlinc_cache* cache, const kvlinc_half* q, kvlinc_half* out, void* workspace,
                                  size_t workspace_bytes, int32_t max_context, void* stream, void* start_event,
                                  void* stop_event);

/*
 * kvlinc_decode_attention for callers that cannot allocate and have no scratch buffer to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus the workspace, same kernels, same
 * results bit for bit.  The split partials go to a buffer of KVLINC_STATIC_SCRATCH_BYTES that is part of the library's
 * device image (every GPU the library runs on holds its own copy until the process ends); the call allocates nothing.
 * A launch that needs more (kvlinc_decode_workspace_bytes(cache, max_context) > KVLINC_STATIC_SCRATCH_BYTES) is
 * rejected with KVLINC_ESCRATCH before anything is enqueued.  All calls on one GPU share that GPU's buffer: two such
 * calls that overlap in time on one GPU (different streams) race, also on different caches.  Nothing in the buffer
 * has to start at zero, and its contents are undefined afterwards.
 */
#define KVLINC_STATIC_SCRATCH_BYTES (16u << 20)
int kvlinc_decode_attention_noalloc(const kvlinc_cache* cache, const kvlinc_half* q, kvlinc_half* out, int32_t max_context,
                                    void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVLINC_H */
