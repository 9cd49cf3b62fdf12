// Decode: single-query attention read directly from the packed 2-bit cache on the CDNA4 matrix cores, with the
// linear correction and the fp16 window (Sec. 3.3, Alg. 1; Sec. 3.2, Eq. 5-6; Sec. 3.1 for the rotated value basis).
//
// decode_main_kernel, one launch per decode step, two kinds of workgroups:
//   streaming workgroups (sequence, kv head, split): the four waves take groups of 128 tokens from a static schedule
//   that is the same for every sequence length; a wave keeps its own (m, l, acc).  The number of splits of a
//   sequence follows its share of the batch's groups, so that sequences of unequal lengths end together.  A group record is fetched in two
//   parts, each requested again for the wave's next group as soon as its contraction has consumed it.  Two waves per
//   (sequence, kv head) also own a 64-token half of the fp16 window, processed as one more block of tokens.  The
//   waves are combined through LDS and the workgroup writes one (m, l, Y_s) per query head (Alg. 1 line 11);
//   correction workgroups (kv head, part of phi, 4 sequences): C_n = phi_q S and C_d = phi_q P, cut into parts over
//   the rows of S, on the matrix cores.
// Every workgroup counts itself in at its (sequence, kv head); the one that arrives last merges, one wave per query
// head: it weighs the splits by 2^(m_j - M), adds the correction as (num + 2^-M C_n) / (den + 2^-M C_d), applies
// H^T and stores fp16 (Alg. 1 lines 13-15 with Eq. 5).  No workgroup waits for another.
//
// The two contractions of a group (Alg. 1 lines 5-10) run on v_mfma_scale_f32_16x16x128_f8f6f4, 16 rows x 16 columns x
// 128 contraction positions per instruction, 8 instructions per contraction and block of 4 query heads:
//   q K^T : columns = 16 tokens, positions = the 128 channels;  E V : columns = 16 channels, positions = the 128 tokens.
// B operand = the codes, read as FP4 (E2M1).  A code c is stored as a bit pair (hi, lo) such that the nibble hi|0|lo|1 is
// the FP4 number c - 1.5; a word keeps the pairs of two codes interleaved in every nibble, so one AND-OR (and one shift
// for the second code of the nibbles) turns 8 codes into a B register.  Codes are never dequantized, and the centred
// codes keep the sums free of a common sign (the matrix cores add with a truncating adder: all-positive products
// would leave a bias that the zero-point term, summed exactly, does not share).
// A operand = the small side, (q * key scale) resp. (p * value scale), as FP8 (E4M3) in three terms per value:
//   x = 2^e (t0 + t1 / 16 + t2 / 256), t_k = fp8 of what the earlier terms left, each term in a row of its own,
//   rows = 4 heads x (3 terms + 1 spare), the factor 2^(e - 4 k) in the row's block scale.
// The terms leave 2^-12 of x at most (better than binary16); e follows the largest |x| of the head in that group, so
// no operand overflows or flushes whatever the magnitude of keys, queries and values.  The three rows of a head are
// summed after the instruction (scores) or once at the end (E V).
// Zero-points never touch the tiles: sum_c q_c (s_c code + z_c) = sum_c (q_c s_c) (code - 1.5) + sum_c q_c (z_c + 1.5 s_c),
// and likewise for the values per token.  Scores live in the log2 domain: x = q.k * log2(e)/sqrt(d).
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include "kvlinc_internal.h"
#include "kvlinc_mfma.h"

namespace kvlinc {
namespace {

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kAlpha = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)

typedef int v8i_t __attribute__((ext_vector_type(8)));
typedef short short2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

// ---- small helpers ----------------------------------------------------------------------------------------------

// Results that one workgroup writes and another reads inside the same launch (split partials, correction parts) go
// through stores and loads that are coherent across the chip's L2 slices: a workgroup-wide cache write-back /
// invalidate (what a device-scope fence costs here) would throw away the streamed records.
__device__ __forceinline__ void st_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}
__device__ __forceinline__ float ld_coherent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

__device__ __forceinline__ float as_f32(uint32_t v) { return __builtin_bit_cast(float, v); }
__device__ __forceinline__ uint32_t as_bits(float v) { return __builtin_bit_cast(uint32_t, v); }

// Reductions with the result in every participating lane.  row: the 16 lanes of a DPP row; quad: 4 adjacent lanes;
// xrow: the 4 lanes l, l ^ 16, l ^ 32, l ^ 48 (row swaps: odd rows of one copy against even rows of the other, then
// the upper 32 lanes of one against the lower 32 of the other).  The *_umax forms take bit patterns of non-negative
// numbers, which order like the numbers themselves (one instruction per step, no NaN handling).
__device__ __forceinline__ float row_allmax(float v) {
  v = fmaxf(v, dpp_f<kRowRor1>(v));
  v = fmaxf(v, dpp_f<kRowRor2>(v));
  v = fmaxf(v, dpp_f<kRowRor4>(v));
  return fmaxf(v, dpp_f<kRowRor8>(v));
}
__device__ __forceinline__ float row_allsum(float v) {
  v += dpp_f<kRowRor1>(v);
  v += dpp_f<kRowRor2>(v);
  v += dpp_f<kRowRor4>(v);
  return v + dpp_f<kRowRor8>(v);
}
__device__ __forceinline__ uint32_t row_umax(uint32_t v) {
  v = max(v, dpp_u<kRowRor1>(v));
  v = max(v, dpp_u<kRowRor2>(v));
  v = max(v, dpp_u<kRowRor4>(v));
  return max(v, dpp_u<kRowRor8>(v));
}
__device__ __forceinline__ uint32_t quad_umax(uint32_t v) {
  v = max(v, dpp_u<kQuadSwap1>(v));
  return max(v, dpp_u<kQuadSwap2>(v));
}
__device__ __forceinline__ float quad_allsum(float v) {
  v += dpp_f<kQuadSwap1>(v);
  return v + dpp_f<kQuadSwap2>(v);
}
__device__ __forceinline__ uint32_t xrow_umax(uint32_t v) {
  auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  v = max(a[0], a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return max(b[0], b[1]);
}
__device__ __forceinline__ float xrow_allsum(float v) {
  auto a = __builtin_amdgcn_permlane16_swap(as_bits(v), as_bits(v), false, false);
  v = as_f32(a[0]) + as_f32(a[1]);
  auto b = __builtin_amdgcn_permlane32_swap(as_bits(v), as_bits(v), false, false);
  return as_f32(b[0]) + as_f32(b[1]);
}

// The compiler may not move LDS traffic of one wave across this point (the hardware keeps a wave's LDS instructions
// in order, which is all a wave needs to hand data from lane to lane through LDS).
__device__ __forceinline__ void lds_order() { asm volatile("" ::: "memory"); }

// ---- operand layouts of v_mfma_scale_f32_16x16x128_f8f6f4 (measured on gfx950) ---------------------------------------
// D:  lane l holds column l % 16, rows 4 (l / 16) + r in its 4 registers.
// B (FP4, 4 registers): lane l holds column l % 16, positions k = 32 (l / 16) + e, nibble e = 0..31 in register order.
// A (FP8, 8 registers): lane l holds row l % 16, byte e = 0..31 in register order at position
//     k = 64 (e / 16) + 16 (l / 16) + e % 16.
// Block scales (E8M0 byte, value 2^(byte - 127)): the scale operand of lane l applies to row / column l % 16 and the
// positions 32 (l / 16) .. 32 (l / 16) + 31.
//
// Roles of a lane.  As a holder of D registers ("row role"): head hd = lane / 16 of the head block, column jd.  As a
// holder of A registers: row 4 ha + ua = (head ha, term ua), quarter ga.  The A registers are built by the lanes in
// 8-byte chunks -- chunk u of (head, quarter g) = bytes 8 u .. 8 u + 7 = positions 64 (u / 2) + 16 g + 8 (u % 2) + 0..7 --
// and handed over through LDS: the builder of (head h, quarter g, chunk u) writes its three terms at
// ex[160 h + 32 term + 2 (4 g + u)], the holder of (head h, term, quarter g) reads 8 words at ex[160 h + 32 term + 8 g].
// Term 3 of every head stays zero.  Word 128 of a head carries the block exponent where builder and holder differ.
constexpr int kExHead = 160;              // words per head in an exchange region (stride 640 B: two heads cover all banks)
constexpr int kExWords = 4 * kExHead;     // one region: 4 heads
constexpr int kExExp = 128;               // word of the block exponent

// B registers from packed words: nibble = hi|0|lo|1 = FP4 (code - 1.5).  One bit-field insert per register: the code bits of the word where `pick` has ones, the constant mantissa bit elsewhere.
// `pick` is 0xAAAAAAAA held in a scalar register (see code_bits_mask) so that the insert is a single instruction.
__device__ __forceinline__ uint32_t centred_nibbles(uint32_t w, uint32_t pick) {
  return 0x11111111u ^ (pick & (w ^ 0x11111111u));  // = (w & pick) | (0x11111111 & ~pick), in the form that selects v_bfi_b32
}
__device__ __forceinline__ uint32_t code_bits_mask() {
  uint32_t m = 0xAAAAAAAAu;
  asm volatile("" : "+s"(m));  // opaque to constant folding, so that the insert stays one instruction
  return m;
}
struct Roles {
  int lane;
  int jd, hd;      // row role
  int ua, ha, ga;  // operand role
  int c0;          // first of the 8 channels whose (q * key scale) this lane builds: chunk ua of (ha, ga)
  int wq;          // where this lane writes its chunk as a builder of q K^T operands (it builds for its own quad)
  int wp;          // ... as a builder of E V operands (it builds from the probabilities it holds in the row role)
  int rd;          // where this lane reads its operand registers
  uint32_t* ex_qk;  // this wave's exchange regions
  uint32_t* ex_pv;
  uint32_t pick;    // code_bits_mask()
};

__device__ __forceinline__ Roles make_roles(int lane, uint32_t* ex_wave) {
  Roles r;
  r.lane = lane;
  r.jd = lane & 15; r.hd = lane >> 4;
  r.ua = lane & 3; r.ha = (lane >> 2) & 3; r.ga = lane >> 4;
  r.c0 = 64 * (r.ua >> 1) + 16 * r.ga + 8 * (r.ua & 1);
  r.wq = kExHead * r.ha + 2 * (4 * r.ga + r.ua);
  r.wp = kExHead * r.hd + 2 * r.jd;
  r.rd = kExHead * r.ha + 32 * r.ua + 8 * r.ga;
  r.ex_qk = ex_wave;
  r.ex_pv = ex_wave + kExWords;
  r.pick = code_bits_mask();
  return r;
}

// x[0..7] as three FP8 terms: with sc = 2^e (sc_bits its binary32 pattern, e chosen so that |x| / sc < 256),
// t_k = fp8((x - what t_0 .. t_{k-1} stand for) / (sc / 16^k)), round to nearest even.  Every residual is exact in
// binary32 (the term agrees with it in its leading bits).  t[k][v] holds values 4 v .. 4 v + 3, lowest byte first.
__device__ __forceinline__ void split_fp8x3(const float (&x)[8], uint32_t sc_bits, uint32_t (&t)[3][2]) {
  float r[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = x[i];
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    const float sc = as_f32(sc_bits - ((uint32_t)(4 * k) << 23));
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      short2_t w = __builtin_bit_cast(short2_t, r[4 * v]);  // any register: both halves are written below
      w = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(w, r[4 * v], r[4 * v + 1], sc, false);
      w = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(w, r[4 * v + 2], r[4 * v + 3], sc, true);
      const uint32_t bits = __builtin_bit_cast(uint32_t, w);
      t[k][v] = bits;
      if (k < 2) {
        const float2_t f0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(bits, sc, false);
        const float2_t f1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(bits, sc, true);
        r[4 * v] -= f0[0]; r[4 * v + 1] -= f0[1];
        r[4 * v + 2] -= f1[0]; r[4 * v + 3] -= f1[1];
      }
    }
  }
}

// Biased binary32 exponent eb of the largest magnitude of a block, from its bit pattern (kept away from the low end of
// the range), for sc = 2^(eb - 127 - 7): |x| / sc < 256, inside FP8's range.  Row `term` then carries the block scale
// byte eb - 7 - 4 term.
__device__ __forceinline__ uint32_t block_exponent(uint32_t mx_bits) { return max(mx_bits, as_bits(0x1p-100f)) >> 23; }
__device__ __forceinline__ uint32_t block_scale_bits(uint32_t eb) { return (eb - 7u) << 23; }

// Builder side of the hand-over: the three terms of this lane's chunk; holder side: the 8 operand registers.
__device__ __forceinline__ void put_terms(uint32_t* ex, int at, const uint32_t (&t)[3][2]) {
#pragma unroll
  for (int k = 0; k < 3; ++k) *reinterpret_cast<u32x2_t*>(ex + at + 32 * k) = u32x2_t{t[k][0], t[k][1]};
}
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v8i_t get_operand(const uint32_t* ex, int at) {
  const u32x4_t a = *reinterpret_cast<const u32x4_t*>(ex + at), b = *reinterpret_cast<const u32x4_t*>(ex + at + 4);
  return v8i_t{(int)a[0], (int)a[1], (int)a[2], (int)a[3], (int)b[0], (int)b[1], (int)b[2], (int)b[3]};
}

// D = A B + C with B = 32 centred codes per lane from two packed words (see centred_nibbles); kScaleB: the block scale
// byte of B (127 = 1, 129 = 4).
template <int kScaleB = 127>
__device__ __forceinline__ float4_t mfma_codes(v8i_t a, uint32_t w0, uint32_t w1, float4_t c, int scale_a, uint32_t pick) {
  const v8i_t b = {(int)centred_nibbles(w0, pick), (int)centred_nibbles(w0 << 1, pick), (int)centred_nibbles(w1, pick),
                   (int)centred_nibbles(w1 << 1, pick), 0, 0, 0, 0};
  return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0 /* A: FP8 E4M3 */, 4 /* B: FP4 E2M1 */, 0, scale_a,
                                                         0, kScaleB);
}
// 4-bit codes: a tile is two planes of 2-bit codes, the base-4 digits of the codes, and
// code - 7.5 = 4 (high digit - 1.5) + (low digit - 1.5): the contraction with the codes is the contraction with the high
// plane under a block scale of 4 plus the contraction with the low plane.
__device__ __forceinline__ float4_t mfma_codes_high(v8i_t a, uint32_t w0, uint32_t w1, float4_t c, int scale_a, uint32_t pick) {
  return mfma_codes<129>(a, w0, w1, c, scale_a, pick);
}

// Register image of one group; BITS / 2 planes per tile.
template <int BITS>
struct KeyRegs {
  uint4 kw[2 * BITS];  // key tile: kw[4 plane + m] = the words of token blocks 2 m (x, y) and 2 m + 1 (z, w) for this lane's (column, quarter)
  uint4 ks, kz;  // key scale / zero-point of the 8 channels c0 .. c0 + 7 this lane builds operands for
};
template <int BITS>
struct ValueRegs {
  uint4 vw[2 * BITS];  // value tile, channel blocks 2 m and 2 m + 1 of every plane
  uint4 sz[2];  // value (scale, zero-point) pairs of tokens 16 n + jd, n = 0..7
};

// A record is fetched in two parts so that each part can be requested again for the next group as soon as its
// contraction has consumed it: the key part flies during E V, the value part during the next q K^T.
// The tiles are read once per launch and by one wave only: non-temporal loads (measured: config 2 23.7 -> 22.2 us,
// config 4 83.7 -> 77.5 us; the short contexts of config 7 lose 2 %).
__device__ __forceinline__ uint4 load_once(const uint4* p) {
  const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(t[0], t[1], t[2], t[3]);
}
template <int BITS>
__device__ __forceinline__ void load_keys(KeyRegs<BITS>& r, const uint32_t* __restrict__ rec, const Roles& lr) {
  const uint4* kt = reinterpret_cast<const uint4*>(rec + Rec<BITS>::kKeyTile);
#pragma unroll
  for (int m = 0; m < 2 * BITS; ++m) r.kw[m] = load_once(kt + m * 64 + lr.lane);  // (the planes follow each other)
  r.ks = *reinterpret_cast<const uint4*>(reinterpret_cast<const half_t*>(rec + Rec<BITS>::kKeyScale) + lr.c0);
  r.kz = *reinterpret_cast<const uint4*>(reinterpret_cast<const half_t*>(rec + Rec<BITS>::kKeyZero) + lr.c0);
}

template <int BITS>
__device__ __forceinline__ void load_values(ValueRegs<BITS>& r, const uint32_t* __restrict__ rec, const Roles& lr) {
  const uint4* vt = reinterpret_cast<const uint4*>(rec + Rec<BITS>::kValueTile);
#pragma unroll
  for (int m = 0; m < 2 * BITS; ++m) r.vw[m] = load_once(vt + m * 64 + lr.lane);
  const uint4* sz = reinterpret_cast<const uint4*>(rec + Rec<BITS>::kValueSZ) + 2 * lr.jd;
  r.sz[0] = sz[0];
  r.sz[1] = sz[1];
}

// NB = head blocks of 4 query heads (1: up to 4 heads per KV head, 2: up to 8).  State of a wave, row role.
template <int NB>
struct WaveState {
  float m[NB];          // reference maximum of this lane's head (equal in the 16 lanes of the row), log2 domain
  float l[NB];          // per-lane partial sum of p
  float pz[NB];         // per-lane partial sum of p * (value zero-point + 1.5 value scale)
  float4_t acc[NB][8];  // E V of channel 16 n + jd: registers 0..2 = the three term rows of the head, register 3 = what
                        // the fp16 window contributed (the matrix cores add the zero term row to it)
};

// q K^T of one group for all heads (Alg. 1 line 7): scores in the log2 domain, sc[nb][n] = head 4 nb + hd, token 16 n + jd.
// qa = this lane's 8 query values (head 4 nb + ha, channels c0 ..) times log2(e) / sqrt(d); qh = the same as binary16 pairs.
template <int NB, int BITS>
__device__ __forceinline__ void qk_phase(const KeyRegs<BITS>& g, int valid, const float (&qa)[NB][8], const uint32_t (&qh)[NB][4],
                                         const Roles& lr, float (&sc)[NB][8]) {
  const uint32_t S[4] = {g.ks.x, g.ks.y, g.ks.z, g.ks.w};
  const uint32_t Z[4] = {g.kz.x, g.kz.y, g.kz.z, g.kz.w};
  v8i_t A[NB];
  int scale_a[NB];
  float4_t c0[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    float x[8], bz = 0.0f, mx = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      x[i] = fmaf(qa[nb][i], (float)as_h2(S[i >> 1])[i & 1], 0.0f);  // (the fused form reads the binary16 operand as it is)
      mx = fmaxf(mx, fabsf(x[i]));
    }
    // sum_c q_c (z_c + 1.5 s_c): what the zero-points and the centring of the codes add to every score of the group.
    // Mid-points and query in binary16 pairs, products summed in binary32: the term is a common offset of the
    // group's scores and small (keys are centred), its rounding (2^-12 of it) is of no account.
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const half2_t mid = as_h2(S[i]) * half2_t{(half_t)Rec<BITS>::kCentre, (half_t)Rec<BITS>::kCentre} + as_h2(Z[i]);
      bz = __builtin_amdgcn_fdot2(as_h2(qh[nb][i]), mid, bz, false);
    }
    const uint32_t eb = block_exponent(xrow_umax(quad_umax(as_bits(mx))));  // over the 128 channels of the head
    bz = xrow_allsum(quad_allsum(bz));
    uint32_t t[3][2];
    split_fp8x3(x, block_scale_bits(eb), t);
    // (two head blocks: the second one goes through the other exchange region, so that one hand-over serves both)
    put_terms(nb == 0 ? lr.ex_qk : lr.ex_pv, lr.wq, t);
    if (NB == 1) {
      lds_order();
      A[nb] = get_operand(lr.ex_qk, lr.rd);
      lds_order();
    }
    scale_a[nb] = (int)eb - 7 - 4 * lr.ua;
    // the head's zero-point term enters as the C operand of its first term row: fetch it from a lane that holds head hd
    // in the operand role (lane 4 hd)
    c0[nb] = float4_t{__builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(16 * lr.hd, __builtin_bit_cast(int, bz))), 0.f,
                      0.f, 0.f};
  }
  if (NB == 2) {
    lds_order();
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) A[nb] = get_operand(nb == 0 ? lr.ex_qk : lr.ex_pv, lr.rd);
    lds_order();
  }
  if constexpr (BITS == 2 && NB == 1) {
    // All eight matrix instructions first, each into registers of its own, then the sums of the term rows: written
    // as one loop the compiler reuses the result registers and every instruction waits for the one before (a dozen
    // idle cycles each; config 3 24.0 -> 22.9 us, config 2 21.5 -> 21.25 us; two head blocks do not gain).
    float4_t dq[8];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const uint32_t w[4] = {g.kw[m].x, g.kw[m].y, g.kw[m].z, g.kw[m].w};
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) dq[2 * m + hf] = mfma_codes(A[0], w[2 * hf], w[2 * hf + 1], c0[0], scale_a[0], lr.pick);
    }
#pragma unroll
    for (int n = 0; n < 8; ++n) sc[0][n] = (dq[n][0] + dq[n][1]) + dq[n][2];
  }
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const uint32_t w[4] = {g.kw[m].x, g.kw[m].y, g.kw[m].z, g.kw[m].w};
    if constexpr (BITS == 2 && NB == 1) {
    } else if constexpr (BITS == 2) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const float4_t d = mfma_codes(A[nb], w[2 * hf], w[2 * hf + 1], c0[nb], scale_a[nb], lr.pick);
          sc[nb][2 * m + hf] = (d[0] + d[1]) + d[2];
        }
    } else {
      const uint32_t wl[4] = {g.kw[4 + m].x, g.kw[4 + m].y, g.kw[4 + m].z, g.kw[4 + m].w};  // low plane
      float4_t d[2][NB];
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) d[hf][nb] = mfma_codes_high(A[nb], w[2 * hf], w[2 * hf + 1], c0[nb], scale_a[nb], lr.pick);
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          d[hf][nb] = mfma_codes(A[nb], wl[2 * hf], wl[2 * hf + 1], d[hf][nb], scale_a[nb], lr.pick);
          sc[nb][2 * m + hf] = (d[hf][nb][0] + d[hf][nb][1]) + d[hf][nb][2];
        }
    }
  }
  if (valid < kGroup) {  // partial last group: tokens >= valid do not exist
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int n = 0; n < 8; ++n)
        if (16 * n + lr.jd >= valid) sc[nb][n] = -INFINITY;
  }
}

// Reference maximum (Alg. 1 line 8).  Any reference m works as long as 2^(x - m) stays moderate, so the reference of a
// head is only raised -- with a maximum over the row and a rescale of the accumulated state -- when some score of the
// group exceeds it by more than `slack`; most groups pay one comparison per register.  (The literal form of Alg. 1's
// last lines adds the correction to sums that are shifted by the TRUE maximum: there the slack is 0, which makes the
// reference the running maximum itself.)
constexpr float kSlack = 5.0f;
template <int NB>
__device__ __forceinline__ void update_reference(const float (&sc)[NB][8], WaveState<NB>& st, float slack) {
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    float mloc = sc[nb][0];
#pragma unroll
    for (int n = 1; n < 8; ++n) mloc = fmaxf(mloc, sc[nb][n]);
    if (__builtin_amdgcn_ballot_w64(mloc > st.m[nb] + slack) != 0) {
      const float mnew = fmaxf(st.m[nb], row_allmax(mloc));
      const float f = mnew == -INFINITY ? 1.0f : exp2f(st.m[nb] - mnew);  // 0 when the old reference is -inf
      st.l[nb] *= f;
      st.pz[nb] *= f;
#pragma unroll
      for (int n = 0; n < 8; ++n) st.acc[nb][n] *= f;
      st.m[nb] = mnew;
    }
  }
}

// p = 2^(x - m), its sums, and E V of one group (Alg. 1 lines 9-10).  MASKED: tokens from `fp16_from` on count in the
// sums of p but not in E V: their values are taken from the fp16 window (pv_window_tail).
template <int NB, int BITS, bool MASKED = false>
__device__ __forceinline__ void pv_phase(const ValueRegs<BITS>& g, const float (&sc)[NB][8], const Roles& lr,
                                         WaveState<NB>& st, int fp16_from = kGroup) {
  const uint32_t SZ[8] = {g.sz[0].x, g.sz[0].y, g.sz[0].z, g.sz[0].w, g.sz[1].x, g.sz[1].y, g.sz[1].z, g.sz[1].w};
  v8i_t A[NB];
  int scale_a[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    float y[8], mx = 0.0f;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const float p = __builtin_amdgcn_exp2f(sc[nb][n] - st.m[nb]);
      const half2_t sz = as_h2(SZ[n]);
      st.l[nb] += p;
      const bool coded = !MASKED || 16 * n + lr.jd < fp16_from;
      y[n] = coded ? fmaf(p, (float)sz[0], 0.0f) : 0.0f;  // p * value scale: the weight of the token's codes
      // sum_t p_t (z_t + 1.5 s_t): the zero-points and the centring of the codes, the same for every channel
      st.pz[nb] = coded ? fmaf(y[n], Rec<BITS>::kCentre, fmaf(p, (float)sz[1], st.pz[nb])) : st.pz[nb];
      mx = fmaxf(mx, y[n]);
    }
    const uint32_t eb = block_exponent(row_umax(as_bits(mx)));  // over the 128 tokens of the head
    uint32_t t[3][2];
    split_fp8x3(y, block_scale_bits(eb), t);
    uint32_t* region = nb == 0 ? lr.ex_pv : lr.ex_qk;
    put_terms(region, lr.wp, t);
    region[kExHead * lr.hd + kExExp] = eb;  // the same value from the 16 lanes of the row
    if (NB == 1) {
      lds_order();
      A[nb] = get_operand(lr.ex_pv, lr.rd);
      scale_a[nb] = (int)lr.ex_pv[kExHead * lr.ha + kExExp] - 7 - 4 * lr.ua;
      lds_order();
    }
  }
  if (NB == 2) {
    lds_order();
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const uint32_t* region = nb == 0 ? lr.ex_pv : lr.ex_qk;
      A[nb] = get_operand(region, lr.rd);
      scale_a[nb] = (int)region[kExHead * lr.ha + kExExp] - 7 - 4 * lr.ua;
    }
    lds_order();
  }
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const uint32_t w[4] = {g.vw[m].x, g.vw[m].y, g.vw[m].z, g.vw[m].w};
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        st.acc[nb][2 * m + hf] = BITS == 2 ? mfma_codes(A[nb], w[2 * hf], w[2 * hf + 1], st.acc[nb][2 * m + hf], scale_a[nb], lr.pick)
                                           : mfma_codes_high(A[nb], w[2 * hf], w[2 * hf + 1], st.acc[nb][2 * m + hf], scale_a[nb], lr.pick);
  }
  if constexpr (BITS == 4) {  // the low plane
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const uint32_t w[4] = {g.vw[4 + m].x, g.vw[4 + m].y, g.vw[4 + m].z, g.vw[4 + m].w};
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          st.acc[nb][2 * m + hf] = mfma_codes(A[nb], w[2 * hf], w[2 * hf + 1], st.acc[nb][2 * m + hf], scale_a[nb], lr.pick);
    }
  }
}

// Sliding value window (Sec. 4.1, setup: the newest 128 tokens in full precision): the tokens j >= from of the newest
// group still have their fp16 rotated values in the window slots j.  Their share of E V is formed here from those values
// by the one wave that has the newest group, on v_mfma_f32_4x4x4_16B_f16 as in window_half: rows = the 4 heads of a head
// block, columns = 64 channels (lane = channel), k = 4 window slots, the probabilities (binary16, through LDS) broadcast
// from one lane quad per block of 4 slots.  The result goes to the spare row of the accumulators through `out`, this
// wave's [NB * 4][128] slice of the combine buffer.
template <int NB>
__device__ __forceinline__ void pv_window_tail(const half_t* __restrict__ v_win, const float (&sc)[NB][8], int from,
                                               const Roles& lr, WaveState<NB>& st, int lane, float (*out)[kHeadDim]) {
  half_t* pb = reinterpret_cast<half_t*>(lr.ex_pv);  // [NB * 4 heads][128 tokens]
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int j = 16 * n + lr.jd;
      pb[(nb * 4 + lr.hd) * kGroup + j] = j >= from ? (half_t)__builtin_amdgcn_exp2f(sc[nb][n] - st.m[nb]) : (half_t)0.0f;
    }
  lds_order();
  const int quad = lane >> 2, hrow = lane & 3;
  half4_t A[NB][2];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) A[nb][hf] = *reinterpret_cast<const half4_t*>(pb + (nb * 4 + hrow) * kGroup + 64 * hf + 4 * quad);
  const uint2* vb = reinterpret_cast<const uint2*>(v_win);  // [slot / 4][channel] -> 4 slots
  const int first = from >> 2;                              // blocks of 4 slots below it hold no such token
  float4_t acc[NB][2];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) acc[nb][0] = acc[nb][1] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int hf = 0; hf < 2; ++hf) {
    uint2 vx[2][16];
#pragma unroll
    for (int bq = 0; bq < 16; ++bq)
#pragma unroll
      for (int ch = 0; ch < 2; ++ch) {
        const int blk = 16 * hf + bq;
        vx[ch][bq] = blk >= first ? vb[(long long)blk * kHeadDim + 64 * ch + lane] : make_uint2(0, 0);
      }
#pragma unroll
    for (int bq = 0; bq < 16; ++bq)
#pragma unroll
      for (int ch = 0; ch < 2; ++ch) {
        const half4_t bop = as_h4(vx[ch][bq].x, vx[ch][bq].y);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb][ch] = mfma_bcast(A[nb][hf], bop, acc[nb][ch], bq);
      }
  }
  // (lane = channel, registers = heads) -> (row = head, lane = channel % 16, channel block n)
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      out[nb * 4 + h][lane] = acc[nb][0][h];
      out[nb * 4 + h][64 + lane] = acc[nb][1][h];
    }
  lds_order();
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int n = 0; n < 8; ++n) st.acc[nb][n][3] += out[nb * 4 + lr.hd][16 * n + lr.jd];
  lds_order();
  // the spare term row of every head of this exchange region reads as zero again
  uint32_t* ex = reinterpret_cast<uint32_t*>(lr.ex_pv);
  for (int i = lane; i < 4 * 32; i += 64) ex[(i >> 5) * kExHead + 96 + (i & 31)] = 0u;
  lds_order();
}

// ---- half of the fp16 window as one more block of 64 tokens of one wave (raw keys, rotated values) ---------------
// On v_mfma_f32_4x4x4_16B_f16 with the A operand broadcast from one lane quad: rows = the 4 heads of a head block.
//   q K^T : columns = 64 tokens (lane = token), k = 4 channels;  E V : columns = 64 channels (lane = channel), k = 4 tokens.
// Runs before the wave's first group, on empty state.

template <int NB>
struct WindowState {
  float m[NB][4];       // maximum per head (wave-uniform), log2 domain
  float l[NB][4];       // per-lane p (lane = token)
  float4_t accw[NB][2];  // E V in true units: [head block][channel half], rows = heads, lane = channel
};

template <int NB>
__device__ __forceinline__ void window_half(const kvlinc_cache& c, const half_t* __restrict__ q, int bh, int b, int g,
                                            int gq, int half, int nr, int lane, WindowState<NB>& st) {
  const int quad = lane >> 2, hrow = lane & 3;
  const uint32_t perm_sel = (lane & 1) ? 0x03020706u : 0x05040100u;
  // 16 x 16 B of this lane's key row now; 32 x 8 B of this lane's two value channels once the keys are consumed
  const int tok = 64 * half + lane;
  const int row = tok < c.R ? tok : c.R - 1;  // rows beyond the capacity do not exist; their scores are masked below
  const uint4* krow = reinterpret_cast<const uint4*>(reinterpret_cast<const half_t*>(c.k_res) +
                                                     ((long long)bh * c.R + row) * kHeadDim);
  uint4 kx[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) kx[i] = krow[i];
  const uint2* vbase = reinterpret_cast<const uint2*>(reinterpret_cast<const half_t*>(c.v_res) +
                                                      (long long)bh * c.R * kHeadDim);
  const int n_blocks = c.R / 4;
  // A operand of q K^T: raw q of this lane's head, channels 8*quad .. 8*quad+7
  half4_t A[NB][2];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int h = nb * 4 + hrow;
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (h < gq) raw = *reinterpret_cast<const uint4*>(q + ((long long)b * c.H_q + g * gq + h) * kHeadDim + 8 * quad);
    A[nb][0] = as_h4(raw.x, raw.y);
    A[nb][1] = as_h4(raw.z, raw.w);
  }
  float4_t acc[NB][2][2];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int a = 0; a < 2; ++a) acc[nb][a][0] = acc[nb][a][1] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const half4_t b0 = as_h4(kx[i].x, kx[i].y), b1 = as_h4(kx[i].z, kx[i].w);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      acc[nb][0][i & 1] = mfma_bcast(A[nb][0], b0, acc[nb][0][i & 1], i);
      acc[nb][1][i & 1] = mfma_bcast(A[nb][1], b1, acc[nb][1][i & 1], i);
    }
  }
  float4_t sc[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    sc[nb] = (acc[nb][0][0] + acc[nb][0][1] + acc[nb][1][0] + acc[nb][1][1]) * kAlpha;
    if (tok >= nr) sc[nb] = float4_t{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  }
  uint2 vx[2][16];
#pragma unroll
  for (int ch = 0; ch < 2; ++ch)
#pragma unroll
    for (int bq = 0; bq < 16; ++bq) {
      const int blk = 16 * half + bq;
      vx[ch][bq] = blk < n_blocks ? vbase[(long long)blk * kHeadDim + 64 * ch + lane] : make_uint2(0, 0);
    }
  half4_t A2[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    float p[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      st.m[nb][h] = wave_allmax(sc[nb][h]);  // finite: the caller passes a half that holds a token
      p[h] = __builtin_amdgcn_exp2f(sc[nb][h] - st.m[nb][h]);
      st.l[nb][h] = p[h];
    }
    const half2_t x01 = {(half_t)p[0], (half_t)p[1]}, x23 = {(half_t)p[2], (half_t)p[3]};
    // 4x4 transpose inside each lane quad: (lane = token, slots = heads) -> (lane = head, slots = tokens)
    A2[nb] = quad_transpose(as_u32(x01), as_u32(x23), perm_sel, lane);
    st.accw[nb][0] = st.accw[nb][1] = float4_t{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int bq = 0; bq < 16; ++bq)
#pragma unroll
    for (int ch = 0; ch < 2; ++ch) {
      const half4_t bop = as_h4(vx[ch][bq].x, vx[ch][bq].y);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) st.accw[nb][ch] = mfma_bcast(A2[nb], bop, st.accw[nb][ch], bq);
    }
}

// ---- correction terms (Sec. 3.3: C_n = phi_q(q) S, C_d = phi_q(q) P; Eq. 6 for phi) -----------------------------------
// The work of a kv head is cut into kCorrParts parts over the rows of S: part r covers the kPartFeat features
// kPartFeat (r % kPartsPerHalf) .. of half hs = r / kPartsPerHalf of phi.  A correction workgroup serves one part
// for up to kCorrSeqs sequences, on the matrix cores:
//   phase 1, wave w = query head w of the block of four: logits[s][f] = sum_c q[s][c] W[c][f] for the sequences s as
//            the 4 rows of the 4x4x4 blocks, block = 4 features (with 32-feature parts blocks 8..15 repeat blocks 0..7), k = 4 channels
//            (32 steps); the W rows are read in their natural order (a lane reads 4 features of one channel) and
//            transposed inside the lane quads;
//   phase 2, wave s = sequence s: e_f = exp(logit_f - m_r) with the part's own maximum m_r,
//            Z_r = sum_f e_f, Cd_r = sum_f e_f P[f], and Cn_r = e S with the 4 heads as rows, block = 4 channels,
//            k = 4 features (kPartSteps steps per channel half), S taken from its binary16 tile copy.
// Output per (query head, part): {Cd_r, m_r, Z_r, -, Cn_r[128]}; the softmax normalisation of each half of phi over
// its parts is left to the merge.

// Workgroup barrier for data exchanged through LDS by ordinary LDS writes.
__device__ __forceinline__ void barrier_lds_only() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

constexpr int kCorrParts = 4;                // 4 or 8
constexpr int kPartFeat = 256 / kCorrParts;  // features per part
constexpr int kPartSteps = kPartFeat / 4;    // feature steps (and distinct feature blocks) per part
constexpr int kPartsPerHalf = kCorrParts / 2;
constexpr int kCorrSeqs = 4;  // sequences served by one correction workgroup (the rows of its matrix products)
// binary16 tile copy of S: tile (part r, channel half hh, feature step fs) holds, for lane = 4 blk + j, the 4 halves
// S[64 r + 4 fs + k][64 hh + lane], k = 0..3: what lane (blk, j) feeds as B operand of that step.
constexpr int kStateTileHalfs = 256;  // halves per tile (64 lanes x 4)
// r64 = 64-feature block of S (0..3), hh = channel half, fs = feature step inside the block (0..15)
__device__ __forceinline__ long long state_tile(int r64, int hh, int fs) { return ((r64 * 2 + hh) * 16 + fs) * kStateTileHalfs; }

__device__ __forceinline__ float quadgroup_allmax(float v) {  // over the 16 lanes that share lane & 3
  v = fmaxf(v, __shfl_xor(v, 4, 64));
  v = fmaxf(v, __shfl_xor(v, 8, 64));
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  v = fmaxf(v, __shfl_xor(v, 32, 64));
  return v;
}
__device__ __forceinline__ float quadgroup_allsum(float v) {
  v += __shfl_xor(v, 4, 64);
  v += __shfl_xor(v, 8, 64);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

// sLogit: [kCorrSeqs][4][kPartFeat] floats of LDS.
// FEW_HEADS: fewer than 4 query heads per kv head (one head block).  The waves whose head does not exist then skip
// phase 1 and leave their logits as they are: phase 2 forms that head's row from them, isolated from the others, and
// stores nothing of it.  (A variant of its own, down to the kernel: with the test in the common code the compiler no
// longer staggers the loads of the two phases, and a second copy of this function in one kernel costs that kernel
// registers; either way the launches with 4 or more heads lose 3 to 4 % of their time.)
template <bool FEW_HEADS>
__device__ __forceinline__ void correction_workgroup(const kvlinc_cache& c, const half_t* __restrict__ q,
                                                     float* __restrict__ corr, int gq, int g, int r, int b_first,
                                                     int n_seq, int n_head_blocks, int lane, int wave, float* sLogit) {
  const int hs = r / kPartsPerHalf, fpart = kPartFeat * (r % kPartsPerHalf);  // features 128 hs + fpart ..
  const int blk = lane >> 2, j = lane & 3, fblk = blk & (kPartSteps - 1);
  const int r64 = (128 * hs + fpart) >> 6, fs0 = (fpart & 63) >> 2;  // position of the part among the state tiles
  const uint32_t perm_sel = (lane & 1) ? 0x03020706u : 0x05040100u;
  const half_t* Wq = reinterpret_cast<const half_t*>(c.Wq);
  const half_t* S16 = reinterpret_cast<const half_t*>(c.S16);
  // everything this wave reads from memory is requested at once: the state tiles and P of its sequence (phase 2),
  // then the W rows and q of its head (phase 1)
  const bool has_seq = wave < n_seq;
  const int b_mine = b_first + (has_seq ? wave : 0), bh_mine = b_mine * c.H_kv + g;
  const half_t* tiles = S16 + (long long)bh_mine * kRank * kHeadDim;
  uint2 sreg[2][kPartSteps];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh)
#pragma unroll
    for (int fs = 0; fs < kPartSteps; ++fs)
      sreg[hh][fs] = *reinterpret_cast<const uint2*>(tiles + state_tile(r64, hh, fs0 + fs) + 4 * lane);
  const float4 p4 = *reinterpret_cast<const float4*>(c.P + (long long)bh_mine * kRank + 128 * hs + fpart + 4 * fblk);
  for (int hb = 0; hb < n_head_blocks; ++hb) {
    // ---- phase 1: this wave's head, all sequences ----
    if (!FEW_HEADS || wave < gq) {
      const int h = hb * 4 + wave;
      const int hc = h < gq ? h : gq - 1;
      const int b_row = b_first + (j < n_seq ? j : n_seq - 1);  // row j of A = sequence j
      const half_t* qrow = q + ((long long)b_row * c.H_q + g * gq + hc) * kHeadDim + 4 * blk;
      const half_t* W0 = Wq + (((long long)g * gq + hc) * 2 + hs) * kHeadDim * (kRank / 2) + (long long)j * (kRank / 2) +
                         fpart + 4 * fblk;
      uint2 w[32];
#pragma unroll
      for (int i = 0; i < 32; ++i) w[i] = *reinterpret_cast<const uint2*>(W0 + (long long)(4 * i) * (kRank / 2));
      const half4_t a0 = __builtin_bit_cast(half4_t, *reinterpret_cast<const uint2*>(qrow));       // channels 4 blk ..
      const half4_t a1 = __builtin_bit_cast(half4_t, *reinterpret_cast<const uint2*>(qrow + 64));  // 64 + 4 blk ..
      float4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        const half4_t bop = quad_transpose(w[i].x, w[i].y, perm_sel, lane);
        d = mfma_bcast(i < 16 ? a0 : a1, bop, d, i & 15);
      }
      if (blk < kPartSteps) {
#pragma unroll
        for (int s = 0; s < kCorrSeqs; ++s) sLogit[(s * 4 + wave) * kPartFeat + lane] = d[s];
      }
    }
    barrier_lds_only();
    // ---- phase 2: this wave's sequence, the four heads of the block; lane = (feature step fs = blk, head j) ----
    if (has_seq) {
      const int b = b_mine;
      // lanes of blocks beyond the part's feature blocks hold no features of their own: their terms are made zero
      const float4 l4 = *reinterpret_cast<const float4*>(sLogit + (wave * 4 + j) * kPartFeat + 4 * fblk);
      const float mx = quadgroup_allmax(fmaxf(fmaxf(l4.x, l4.y), fmaxf(l4.z, l4.w)));
      const float live = blk < kPartSteps ? 1.0f : 0.0f;
      const float e0 = live * __expf(l4.x - mx), e1 = live * __expf(l4.y - mx), e2 = live * __expf(l4.z - mx),
                  e3 = live * __expf(l4.w - mx);
      const float z = quadgroup_allsum((e0 + e1) + (e2 + e3));
      const float cd = quadgroup_allsum(fmaf(e0, p4.x, fmaf(e1, p4.y, fmaf(e2, p4.z, e3 * p4.w))));
      const half4_t aop = {(half_t)e0, (half_t)e1, (half_t)e2, (half_t)e3};
      float4_t acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int fs = 0; fs < kPartSteps; ++fs)
          acc[hh] = mfma_bcast(aop, __builtin_bit_cast(half4_t, sreg[hh][fs]), acc[hh], fs);
      float* out0 = corr + ((long long)b * c.H_q + g * gq + hb * 4) * kCorrParts * kPartStride;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (hb * 4 + i < gq) {
          float* dst = out0 + ((long long)i * kCorrParts + r) * kPartStride;
          st_coherent(dst + 4 + lane, acc[0][i]);
          st_coherent(dst + 4 + 64 + lane, acc[1][i]);
        }
      }
      if (blk == 0 && hb * 4 + j < gq) {
        float* dst = out0 + ((long long)j * kCorrParts + r) * kPartStride;
        st_coherent(dst, cd);
        st_coherent(dst + 1, mx);
        st_coherent(dst + 2, z);
      }
    }
    if (hb + 1 < n_head_blocks) barrier_lds_only();  // the logits buffer is reused
  }
}

// ---- merge the splits of one (sequence, query head), add the correction, rotate back (Alg. 1 lines 13-15; Eq. 5;
// Sec. 3.1).  Run by one wave of the split that arrives last; lane l owns channels 2l and 2l+1. ----------------------

// MB = splits whose partial results are requested together; LOCAL: the partial results are this workgroup's own and
// lie in LDS (plain loads), everything else alike
template <int MB, bool LOCAL = false>
__device__ __forceinline__ void merge_row(const float* __restrict__ p0, const float* __restrict__ corr, int n_splits,
                                          int row, int lane, bool literal, half_t* __restrict__ out) {
  // p0: the row's partial results, n_splits of kPartStride floats
  // correction parts first (their values are needed last): {Cd_r, m_r, Z_r, -, Cn_r[128]}
  float c_cd[kCorrParts], c_m[kCorrParts], c_z[kCorrParts], c_x[kCorrParts], c_y[kCorrParts];
  if (corr != nullptr) {
    const float* cr = corr + (long long)row * kCorrParts * kPartStride;
#pragma unroll
    for (int r = 0; r < kCorrParts; ++r) {
      const float* pr = cr + r * kPartStride;
      c_cd[r] = ld_coherent(pr); c_m[r] = ld_coherent(pr + 1); c_z[r] = ld_coherent(pr + 2);
      c_x[r] = ld_coherent(pr + 4 + 2 * lane); c_y[r] = ld_coherent(pr + 5 + 2 * lane);
    }
  }
  // running merge over batches of splits, every batch requested at once
  float M = -INFINITY, n0 = 0.f, n1 = 0.f, den = 0.f;
  for (int j0 = 0; j0 < n_splits; j0 += MB) {
    float mj[MB], lj[MB], ax[MB], ay[MB];
#pragma unroll
    for (int k = 0; k < MB; ++k) {
      const float* pj = p0 + (long long)(j0 + k < n_splits ? j0 + k : n_splits - 1) * kPartStride;
      if (LOCAL) {
        mj[k] = pj[0]; lj[k] = pj[1];
        ax[k] = pj[4 + 2 * lane]; ay[k] = pj[5 + 2 * lane];
      } else {
        mj[k] = ld_coherent(pj); lj[k] = ld_coherent(pj + 1);
        ax[k] = ld_coherent(pj + 4 + 2 * lane); ay[k] = ld_coherent(pj + 5 + 2 * lane);
      }
    }
    float Mb = M;
#pragma unroll
    for (int k = 0; k < MB; ++k)
      if (j0 + k < n_splits) Mb = fmaxf(Mb, mj[k]);
    if (Mb == -INFINITY) continue;
    const float f = exp2f(M - Mb);  // 0 while nothing has been merged yet
    n0 *= f; n1 *= f; den *= f;
#pragma unroll
    for (int k = 0; k < MB; ++k) {
      if (j0 + k < n_splits && mj[k] != -INFINITY) {
        const float w = exp2f(mj[k] - Mb);
        n0 = fmaf(w, ax[k], n0);
        n1 = fmaf(w, ay[k], n1);
        den = fmaf(w, lj[k], den);
      }
    }
    M = Mb;
  }
  float y0 = 0.f, y1 = 0.f;
  if (M != -INFINITY) {
    float cn0 = 0.f, cn1 = 0.f, cd = 0.f;
    if (corr != nullptr) {
      // the parts of each half of phi share one softmax: phi_f = e_f exp(m_r - M_hs) / Z_hs
#pragma unroll
      for (int hs = 0; hs < 2; ++hs) {
        float zsum = 0.f, Mh = -INFINITY;
#pragma unroll
        for (int i = 0; i < kPartsPerHalf; ++i) {
          zsum += c_z[kPartsPerHalf * hs + i];
          Mh = fmaxf(Mh, c_m[kPartsPerHalf * hs + i]);
        }
        if (zsum > 0.f) {
          float zz = 0.f, xx = 0.f, yy = 0.f, dd = 0.f;
#pragma unroll
          for (int i = 0; i < kPartsPerHalf; ++i) {
            const int rr = kPartsPerHalf * hs + i;
            const float wgt = __expf(c_m[rr] - Mh);
            zz = fmaf(wgt, c_z[rr], zz);
            xx = fmaf(wgt, c_x[rr], xx);
            yy = fmaf(wgt, c_y[rr], yy);
            dd = fmaf(wgt, c_cd[rr], dd);
          }
          const float inv = 1.0f / zz;
          cn0 = fmaf(xx, inv, cn0);
          cn1 = fmaf(yy, inv, cn1);
          cd = fmaf(dd, inv, cd);
        }
      }
    }
    // (num + 2^-M C_n) / (den + 2^-M C_d) with both factors kept <= 1 (M is the log2-domain maximum); the literal
    // form of Alg. 1's last lines leaves the factor 2^-M out
    const float Ms = fmaxf(M, 0.f);
    const float fa = literal ? 1.0f : exp2f(M - Ms), fb = literal ? 1.0f : exp2f(-Ms);
    const float d = fa * den + fb * cd;
    y0 = (fa * n0 + fb * cn0) / d;
    y1 = (fa * n1 + fb * cn1) / d;
  }
  // y = y_rot H^T: butterflies over the 128 channels, two per lane
  {
    const float a = y0 + y1, bb = y0 - y1;
    y0 = a; y1 = bb;
#pragma unroll
    for (int mk = 1; mk < 64; mk <<= 1) {
      const float o0 = __shfl_xor(y0, mk, 64), o1 = __shfl_xor(y1, mk, 64);
      const bool upper = (lane & mk) != 0;
      y0 = upper ? (o0 - y0) : (y0 + o0);
      y1 = upper ? (o1 - y1) : (y1 + o1);
    }
  }
  const half2_t r = {(half_t)(y0 * 0.08838834764831845f), (half_t)(y1 * 0.08838834764831845f)};
  *reinterpret_cast<uint32_t*>(out + (long long)row * kHeadDim + 2 * lane) = as_u32(r);
}

// ---- launch 1 -------------------------------------------------------------------------------------------------------


__device__ __forceinline__ void merge_rows(const float* __restrict__ part, const float* __restrict__ corr,
                                           int max_splits, int n_splits, int row, int lane, bool literal,
                                           half_t* __restrict__ out) {
  const float* p0 = part + (long long)row * max_splits * kPartStride;
  if (n_splits <= 4) merge_row<4>(p0, corr, n_splits, row, lane, literal, out);
  else merge_row<8>(p0, corr, n_splits, row, lane, literal, out);
}

// Splits the groups of a sequence are cut into.  The host fixes the average over the batch (avg_splits) and the most
// one sequence may take (max_splits; grid and workspace are sized for it).  A sequence takes its share of
// B * avg_splits in proportion to its number of groups, rounded up from a quarter on, so that the long and the short
// sequences of a batch end together; a batch of equal lengths gives avg_splits to every sequence.  Integer
// arithmetic only: every wave of the launch that needs the number gets the same one from the same counters.
__device__ __forceinline__ int sequence_splits(const kvlinc_cache& c, int nq_b, int avg_splits, int max_splits,
                                               int lane) {
  if (c.B == 1) return avg_splits;
  int total = 0;
  for (int i = lane; i < c.B; i += 64) total += (c.n_quant[i] + kGroup - 1) / kGroup;
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) total += __shfl_xor(total, m, 64);
  const int count = (nq_b + kGroup - 1) / kGroup;
  int s = avg_splits;
  if (total > 0) {  // ceil(avg count B / total - 1/4)
    const long long num = 4ll * avg_splits * count * c.B - total;
    s = num <= 0 ? 0 : (int)((unsigned long long)(num + 4ll * total - 1) / (unsigned long long)(4ll * total));
  }
  s = min(s, min(max_splits, (count + kWaves - 1) / kWaves));  // at least one group per wave
  return __builtin_amdgcn_readfirstlane(max(s, 1));            // the same in every lane: keep it in a scalar register
}

// Arrival of a workgroup at its (sequence, kv head): every wave first waits until its write-through stores have been
// acknowledged, then one thread counts the workgroup in.  Returns true in the workgroup that completes the count.
__device__ __forceinline__ bool arrive(int* counter, int expected, int* sFlag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) *sFlag = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  __syncthreads();
  return *sFlag == expected - 1;
}

// Grid: B H_kv max_splits streaming workgroups, split-major (workgroup = split * B H_kv + sequence * H_kv + kv head),
// each streaming the groups and the window share of one split of a (sequence, kv head), or leaving at once when its
// sequence uses fewer splits; and, when the correction is on, the correction workgroups: after them (corr_first = 0)
// or leading the first corr_first runs of 256 workgroups (1: all of them first -- they are long chains of dependent
// steps and should start at once).  All of them count themselves in at split_done; the last arrival merges.
// SLIDING: the variant with the sliding value window (KVLINC_FLAG_SLIDING_VALUES) is a kernel of its own, so that the
// default one carries none of its code.
// BITS: so is the one for caches with 4-bit codes (it holds twice the tile words in registers).
// FEW_HEADS: and the one for fewer than 4 query heads per kv head (see correction_workgroup).
template <int NB, bool SLIDING = false, int BITS = 2, bool FEW_HEADS = false>
__global__ __launch_bounds__(kThreads, BITS == 4 ? 2 : (NB == 1 ? 3 : 2)) void decode_main_kernel(kvlinc_cache c, const half_t* __restrict__ q,
                                                                   float* __restrict__ part, float* __restrict__ corr,
                                                                   half_t* __restrict__ out, int max_splits,
                                                                   int avg_splits, int gq, int corr_first) {
  __shared__ __align__(16) float lds[2 * kWaves * NB * 4 + kWaves * NB * 4 * kHeadDim];
  __shared__ __align__(16) uint32_t ex[kWaves][2 * kExWords];  // per wave: operand hand-over of q K^T and of E V
  __shared__ int sFlag;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the schedule in scalar registers
  const int n_corr = corr != nullptr ? c.H_kv * kCorrParts * ((c.B + kCorrSeqs - 1) / kCorrSeqs) : 0;
  const int n_parts = corr != nullptr ? kCorrParts : 0;

  const int n_stream = gridDim.x - n_corr;
  // corr_first = 0: the correction workgroups come last; L >= 1: they lead each of the first L runs of 256
  // workgroups in equal shares.  The dispatcher deals workgroup i to compute unit i mod 256 while places are free, so
  // with L = 2 the correction workgroups pair up on compute units of their own and no streaming workgroup has one
  // as a neighbour.
  bool is_corr;
  int corr_id, stream_id;
  int L = corr_first;  // every run that leads with correction workgroups must lie inside the grid and hold its share
  while (L > 1 && ((int)gridDim.x < 256 * (L - 1) + (n_corr + L - 1) / L || (n_corr + L - 1) / L > 256)) --L;
  if (L == 0 || n_corr == 0) {
    is_corr = (int)blockIdx.x >= n_stream;
    corr_id = blockIdx.x - n_stream;
    stream_id = blockIdx.x;
  } else if (L == 1) {
    is_corr = (int)blockIdx.x < n_corr;
    corr_id = blockIdx.x;
    stream_id = blockIdx.x - n_corr;
  } else {
    const int per = (n_corr + L - 1) / L;
    const int layer = min((int)blockIdx.x / 256, L), pos = layer < L ? (int)blockIdx.x % 256 : 0;
    const int before = min(n_corr, layer * per + min(pos, per));  // correction workgroups ahead of this one
    is_corr = layer < L && pos < per && before < n_corr;
    corr_id = before;
    stream_id = blockIdx.x - before;
  }

  if (is_corr) {
    // ---- one part of the correction (Sec. 3.3: C_n, C_d) for up to kCorrSeqs sequences of one kv head ----
    const int id = corr_id;
    // The workgroups that read the same slice of W (same kv head and part, different sequences) are H_kv * kCorrParts
    // apart in the grid: workgroups are dealt to the 8 XCDs in turn, so with an even H_kv they share one L2.
    const int r = id % kCorrParts, g = (id / kCorrParts) % c.H_kv, sb = id / (kCorrParts * c.H_kv);
    const int b_first = sb * kCorrSeqs;
    const int n_seq = min(kCorrSeqs, c.B - b_first);
    // A sequence without quantized tokens has S = P = 0 (the states only change at a flush), so its parts come out
    // as zero without looking at n_quant.
    correction_workgroup<FEW_HEADS>(c, q, corr, gq, g, r, b_first, n_seq, NB, lane, wave, lds);
    // count this workgroup in at each of its sequences; merge those it completes
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int* sFlags = reinterpret_cast<int*>(lds);
    if (tid < n_seq)
      sFlags[tid] = __hip_atomic_fetch_add(c.split_done + (b_first + tid) * c.H_kv + g, 1, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_SYSTEM);
    __syncthreads();
    for (int s = 0; s < n_seq; ++s) {
      const int b = b_first + s, bh = b * c.H_kv + g;
      const int n_splits = sequence_splits(c, c.n_quant[b], avg_splits, max_splits, lane);
      if (sFlags[s] == n_splits + n_parts - 1) {
        for (int h = wave; h < gq; h += kWaves)
          merge_rows(part, corr, max_splits, n_splits, b * c.H_q + g * gq + h, lane, (c.flags & KVLINC_FLAG_ALG1_LITERAL) != 0, out);
        if (tid == 0) c.split_done[bh] = 0;
      }
    }
    return;
  }

  // ---- one split of the groups and of the window (Alg. 1, the loop over blocks) ----
  const int wg = stream_id;
  // split-major: the splits that only long sequences use come last in the grid, and the workgroups of any one split
  // index are dealt evenly to the XCDs
  const int bh = wg % (c.B * c.H_kv);
  const int sp = wg / (c.B * c.H_kv);
  const int b = bh / c.H_kv;
  const int g = bh % c.H_kv;

  // Static schedule, the same for every sequence length, so that a wave knows its first group before it knows the
  // length.  Time is cut into rounds of 4 n_splits slots, slot(round, wave, split) = 4 n_splits round + n_splits wave
  // + split; the groups 0, 1, 2, ... go to the slots in order, except that the two waves that own a half of the
  // window sit out their first kSkip slots (the window is their work for that time).  Consecutive groups thus go to
  // different workgroups, and every split gets the same share whatever the length.
  constexpr int kSkip = 2;
  int n_splits = avg_splits;  // first guess: right for a batch of equal lengths
  int slots, my_half, off, lead1, rd, idx;
  auto group_of_round = [&](int round) {
    return round * slots + off - min(round, kSkip) - min(round + lead1, kSkip);
  };
  auto plan = [&]() {
    slots = kWaves * n_splits;
    my_half = -1;
    if (n_splits >= 2) {
      if (wave == kWaves - 1 && sp >= n_splits - 2) my_half = n_splits - 1 - sp;
    } else if (wave >= kWaves - 2) {
      my_half = kWaves - 1 - wave;
    }
    // group(round) = slot - (slots skipped before it).  The owners of half 0 and half 1 have the round's last and
    // last but one slot, so the owner of half 0 has skipped min(round, kSkip) slots before a wave's slot and the
    // owner of half 1 one more if it comes earlier in the round.
    const int base1 = n_splits >= 2 ? slots - 2 : kWaves - 2;
    off = wave * n_splits + sp;
    lead1 = off > base1 ? 1 : 0;
    rd = my_half >= 0 ? kSkip : 0;
    idx = group_of_round(rd);
  };
  plan();

  // The first record is requested before the sequence length is known (any group index below the capacity is
  // readable memory); what it holds is used only if the group exists.
  constexpr int kRecordWords = Rec<BITS>::kWords;
  const uint32_t* rec0 = c.groups + (long long)bh * c.max_groups * kRecordWords;
  const Roles lr = make_roles(lane, ex[wave]);
  KeyRegs<BITS> kr;
  ValueRegs<BITS> vr;
  if (sp < avg_splits) {
    const long long first = idx < c.max_groups ? idx : c.max_groups - 1;
    load_keys(kr, rec0 + first * kRecordWords, lr);
    load_values(vr, rec0 + first * kRecordWords, lr);
  }
  const int nq = c.n_quant[b];
  const int nr = c.n_res[b];
  const int count = (nq + kGroup - 1) / kGroup;
  {
    const int mine = sequence_splits(c, nq, avg_splits, max_splits, lane);
    if (sp >= mine) return;  // this sequence uses fewer splits than the grid provides
    if (mine != n_splits) {  // lengths differ within the batch: plan again, request the right first record
      n_splits = mine;
      plan();
      const long long first = idx < c.max_groups ? idx : c.max_groups - 1;
      load_keys(kr, rec0 + first * kRecordWords, lr);
      load_values(vr, rec0 + first * kRecordWords, lr);
    }
  }
  const int expected = n_splits + n_parts;

  // the spare term row of every head reads as zero from here on (this wave's own regions: no barrier needed)
  for (int i = lane; i < 2 * 4 * 32; i += 64) ex[wave][(i >> 7) * kExWords + ((i >> 5) & 3) * kExHead + 96 + (i & 31)] = 0u;
  lds_order();

  float (*sM)[NB * 4] = reinterpret_cast<float (*)[NB * 4]>(lds);                    // [kWaves][NB*4]
  float (*sL)[NB * 4] = reinterpret_cast<float (*)[NB * 4]>(lds + kWaves * NB * 4);  // [kWaves][NB*4]
  float (*sAcc)[NB * 4][kHeadDim] = reinterpret_cast<float (*)[NB * 4][kHeadDim]>(lds + 2 * kWaves * NB * 4);

  WaveState<NB> st;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    st.m[nb] = -INFINITY; st.l[nb] = 0.f; st.pz[nb] = 0.f;
#pragma unroll
    for (int n = 0; n < 8; ++n) st.acc[nb][n] = float4_t{0.f, 0.f, 0.f, 0.f};
  }

  if (my_half >= 0 && nr > 64 * my_half) {
    // this wave's half of the window first, then its results move to the row role: (lane = channel, registers = heads)
    // -> (row = head, lane = channel % 16, register 3 of channel block n), through this wave's part of the combine buffer
    WindowState<NB> ws;
    window_half<NB>(c, q, bh, b, g, gq, my_half, nr, lane, ws);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float lsum[4];
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        lsum[h] = wave_allsum(ws.l[nb][h]);
        sAcc[wave][nb * 4 + h][lane] = ws.accw[nb][0][h];
        sAcc[wave][nb * 4 + h][64 + lane] = ws.accw[nb][1][h];
      }
      lds_order();
#pragma unroll
      for (int n = 0; n < 8; ++n) st.acc[nb][n][3] = sAcc[wave][nb * 4 + lr.hd][16 * n + lr.jd];
      lds_order();
      const float m_mine = lr.hd == 0 ? ws.m[nb][0] : lr.hd == 1 ? ws.m[nb][1] : lr.hd == 2 ? ws.m[nb][2] : ws.m[nb][3];
      const float l_mine = lr.hd == 0 ? lsum[0] : lr.hd == 1 ? lsum[1] : lr.hd == 2 ? lsum[2] : lsum[3];
      st.m[nb] = m_mine;
      st.l[nb] = lr.jd == 0 ? l_mine : 0.f;
    }
  }

  if (idx < count) {
    // q of the head this lane builds operands for (head 4 nb + ha), channels c0 .. c0 + 7, in the log2 domain; heads
    // beyond gq read as 0
    float qa[NB][8];
    uint32_t qh[NB][4];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int h = nb * 4 + lr.ha;
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (h < gq) raw = *reinterpret_cast<const uint4*>(q + ((long long)b * c.H_q + g * gq + h) * kHeadDim + lr.c0);
      const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int i = 0; i < 8; ++i) qa[nb][i] = (float)as_h2(r[i >> 1])[i & 1] * kAlpha;
#pragma unroll
      for (int i = 0; i < 4; ++i) qh[nb][i] = as_u32(half2_t{(half_t)qa[nb][2 * i], (half_t)qa[nb][2 * i + 1]});
    }
    // While a group is consumed the wave's next record is already requested: its key part right after the scores,
    // its value part right after E V.  The wave's last group is a copy of the loop body without requests (a request
    // past the end would be a second trip to memory for a record that the non-temporal loads did not leave in the
    // caches, and the combine would wait for it: config 7 68.8 -> 65.3 us, config 6 53.0 -> 50.2 us).
    // sliding value window: the newest group's tokens from n_res on take their values from the window
    // (the newest group is left to the code below when its last tokens take their values from the window)
    const float slack = (c.flags & KVLINC_FLAG_ALG1_LITERAL) != 0 ? 0.0f : kSlack;
    const bool sliding = SLIDING && nq % kGroup == 0 && nr < kGroup;
    const int count_plain = sliding ? count - 1 : count;
    while (idx < count_plain) {
      const int nxt = group_of_round(++rd);
      if (nxt >= count) break;
      const uint32_t* src = rec0 + (long long)nxt * kRecordWords;
      float sc[NB][8];
      qk_phase<NB, BITS>(kr, min(kGroup, nq - idx * kGroup), qa, qh, lr, sc);
      load_keys(kr, src, lr);
      update_reference<NB>(sc, st, slack);
      pv_phase<NB, BITS>(vr, sc, lr, st);
      load_values(vr, src, lr);
      idx = nxt;
    }
    if (idx < count_plain) {  // the wave's last group: nothing more to request
      float sc[NB][8];
      qk_phase<NB, BITS>(kr, min(kGroup, nq - idx * kGroup), qa, qh, lr, sc);
      update_reference<NB>(sc, st, slack);
      pv_phase<NB, BITS>(vr, sc, lr, st);
      idx = count;
    }
    if (SLIDING && idx < count) {  // sliding value window: the newest group, whose tokens from n_res on have fp16 values
      float sc[NB][8];
      qk_phase<NB, BITS>(kr, kGroup, qa, qh, lr, sc);
      update_reference<NB>(sc, st, slack);
      pv_phase<NB, BITS, true>(vr, sc, lr, st, nr);
      pv_window_tail<NB>(reinterpret_cast<const half_t*>(c.v_res) + (long long)bh * c.R * kHeadDim, sc, nr, lr, st, lane, sAcc[wave]);
    }
  }

  // A sequence with a single split whose correction parts have all arrived has nobody left to wait for: its one
  // workgroup then merges what it holds, without the trip of its partial result through memory.  The look at the
  // counter is taken here so that its latency passes during the combine; a look that comes too early only sends the
  // workgroup down the ordinary way.
  __shared__ int sDirect;
  if (tid == 0) {
    int direct = 0;
    if (n_splits == 1)
      direct = n_parts == 0 ? 1 : (__hip_atomic_load(c.split_done + bh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == n_parts);
    sDirect = direct;
  }
  // combine the four waves (Alg. 1 lines 13-14 restricted to this workgroup) and write (m, l, Y_s)
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const float l = row_allsum(st.l[nb]);
    const float pz = row_allsum(st.pz[nb]);
    const int h = nb * 4 + lr.hd;
    if (lr.jd == 0) { sM[wave][h] = st.m[nb]; sL[wave][h] = l; }
#pragma unroll
    for (int n = 0; n < 8; ++n)
      sAcc[wave][h][16 * n + lr.jd] = ((st.acc[nb][n][0] + st.acc[nb][n][1]) + (st.acc[nb][n][2] + st.acc[nb][n][3])) + pz;
  }
  __syncthreads();
  const bool direct = sDirect != 0;
  float* own = reinterpret_cast<float*>(&ex[0][0]);  // [gq][kPartStride]: the exchange regions are free by now
  for (int i = tid; i < gq * kHeadDim; i += kThreads) {
    const int h = i >> 7, ch = i & 127;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sM[w][h]);
    float a = 0.f, l = 0.f;
    if (M != -INFINITY) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float f = exp2f(sM[w][h] - M);  // 0 for a wave without tokens
        a = fmaf(f, sAcc[w][h][ch], a);
        l = fmaf(f, sL[w][h], l);
      }
    }
    if (direct) {
      float* dst = own + h * kPartStride;
      if (ch == 0) { dst[0] = M; dst[1] = l; }
      dst[4 + ch] = a;
    } else {
      float* dst = part + (((long long)b * c.H_q + g * gq + h) * max_splits + sp) * kPartStride;
      if (ch == 0) { st_coherent(dst, M); st_coherent(dst + 1, l); }
      st_coherent(dst + 4 + ch, a);
    }
  }
  if (direct) {
    __syncthreads();
    for (int h = wave; h < gq; h += kWaves)
      merge_row<4, true>(own + h * kPartStride, corr, 1, b * c.H_q + g * gq + h, lane,
                         (c.flags & KVLINC_FLAG_ALG1_LITERAL) != 0, out);
    if (tid == 0 && n_parts != 0) c.split_done[bh] = 0;  // the arrivals of the correction workgroups
    return;
  }

  // The workgroup that arrives last merges (Alg. 1 lines 13-15): it reads what the others wrote with coherent
  // loads.  No workgroup waits for another.
  if (arrive(c.split_done + bh, expected, &sFlag)) {
    for (int h = wave; h < gq; h += kWaves)
      merge_rows(part, corr, max_splits, n_splits, b * c.H_q + g * gq + h, lane, (c.flags & KVLINC_FLAG_ALG1_LITERAL) != 0, out);
    if (tid == 0) c.split_done[bh] = 0;
  }
}

}  // namespace

// Splits per (sequence, kv head).  Measured on MI355X (256 compute units): the launch is fastest when all its
// workgroups, the correction workgroups included, are resident at once at about two per compute unit -- a second
// generation of workgroups pays the start-up and the merge tail again, and a compute unit that hosts a correction
// workgroup next to two streaming ones finishes late.  The kernel for more than 4 query heads per kv head holds only
// two workgroups per compute unit, and there four splits measured better than three.  At most 32 splits (the merge
// walks the splits serially), at least one group per wave.
DecodeSplits decode_splits(const kvlinc_cache& c, int max_context) {
  constexpr int kTargetWorkgroups = 512, kMaxSplits = 32;
  const long long cap = (long long)c.max_groups * kGroup + c.R;
  const long long ctx = (max_context > 0 && max_context < cap) ? max_context : cap;
  long long groups = (ctx + kGroup - 1) / kGroup;
  if (groups < 1) groups = 1;
  const long long bh = (long long)c.B * c.H_kv;
  const int gq = c.H_q / c.H_kv;
  long long n_corr = 0;
  if (c.S16 != nullptr && gq <= 4) n_corr = (long long)c.H_kv * kCorrParts * ((c.B + kCorrSeqs - 1) / kCorrSeqs);
  long long s = (kTargetWorkgroups - n_corr + bh / 2) / bh;  // rounded to nearest
  if (s > kMaxSplits) s = kMaxSplits;
  const long long most = (groups + kWaves - 1) / kWaves;
  if (s > most) s = most;
  if (s < 1) s = 1;
  // Head room for the longest sequences of a batch of unequal lengths (a single sequence has nobody to differ from).
  long long m = c.B > 1 ? 2 * s : s;
  if (m > kMaxSplits) m = kMaxSplits;
  if (m > most) m = most;
  if (m < s) m = s;
  // The correction workgroups are chains of dependent steps and go first in the grid, except when they alone would
  // fill most of the chip while the streaming workgroups have long contexts ahead of them (many sequences, 16 or
  // more groups per wave): then the streaming workgroups go first, the longest of them decide when the launch ends,
  // and the correction fills the places the short sequences leave.
  const long long all_corr = c.S16 != nullptr ? (long long)c.H_kv * kCorrParts * ((c.B + kCorrSeqs - 1) / kCorrSeqs) : 0;
  const long long resident = 256 * (gq <= 4 ? 3 : 2);
  int corr_first = (2 * all_corr > resident && groups >= 16 * kWaves * s) ? 0 : 1;
  // One or a few long sequences: about one streaming workgroup per compute unit.  The streaming workgroups that
  // would share a compute unit with a correction workgroup finish late (measured 3.6 us at a context of 128k), so
  // the correction workgroups pair up on compute units of their own (two runs of the grid lead with them) and the
  // splits are cut back to leave those compute units free.
  if (all_corr > 0 && bh * s <= 256 && bh * s + all_corr > 256) {
    const long long s2 = (256 - (all_corr + 1) / 2) / bh;
    if (s2 >= 1 && 4 * s2 >= 3 * s) {
      s = s2 < s ? s2 : s;
      if (m > s) m = c.B > 1 ? 2 * s : s;
      if (m > most) m = most;
      if (m < s) m = s;
      corr_first = 2;
    }
  }
  return DecodeSplits{(int)s, (int)m, corr_first};
}

size_t decode_workspace_floats(const kvlinc_cache& c, int n_splits) {
  return (size_t)c.B * c.H_q * (n_splits + kCorrParts) * kPartStride;  // split partials, then the correction parts
}

int launch_decode(const kvlinc_cache& c, const kvlinc_half* q, kvlinc_half* out, float* workspace, DecodeSplits sp,
                  hipStream_t stream, hipEvent_t start, hipEvent_t stop) {
  const int n_splits = sp.most;
  const int gq = c.H_q / c.H_kv;
  const int BH = c.B * c.H_kv;
  const half_t* qq = reinterpret_cast<const half_t*>(q);
  half_t* oo = reinterpret_cast<half_t*>(out);
  float* part = workspace;
  float* corr = c.S16 != nullptr ? workspace + (size_t)c.B * c.H_q * n_splits * kPartStride : nullptr;
  const int n_corr = corr != nullptr ? c.H_kv * kCorrParts * ((c.B + kCorrSeqs - 1) / kCorrSeqs) : 0;
  const dim3 grid(BH * n_splits + n_corr), block(kThreads);
  const int corr_first = sp.corr_first;
  const bool sliding = (c.flags & KVLINC_FLAG_SLIDING_VALUES) != 0;
  void (*kernel)(kvlinc_cache, const half_t*, float*, float*, half_t*, int, int, int, int) =
      c.bits == 4 ? (gq > 4   ? (sliding ? decode_main_kernel<2, true, 4> : decode_main_kernel<2, false, 4>)
                     : gq < 4 ? (sliding ? decode_main_kernel<1, true, 4, true> : decode_main_kernel<1, false, 4, true>)
                              : (sliding ? decode_main_kernel<1, true, 4> : decode_main_kernel<1, false, 4>))
                  : (gq > 4   ? (sliding ? decode_main_kernel<2, true> : decode_main_kernel<2, false>)
                     : gq < 4 ? (sliding ? decode_main_kernel<1, true, 2, true> : decode_main_kernel<1, false, 2, true>)
                              : (sliding ? decode_main_kernel<1, true> : decode_main_kernel<1, false>));
  if (start != nullptr)  // timestamps of the dispatch itself, no extra packets on the stream
    hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, start, stop, 0, c, qq, part, corr, oo, sp.most, sp.avg, gq, corr_first);
  else
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, c, qq, part, corr, oo, sp.most, sp.avg, gq, corr_first);
  return hipGetLastError() == hipSuccess ? KVLINC_OK : KVLINC_EHIP;
}

}  // namespace kvlinc

