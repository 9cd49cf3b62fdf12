// Append / flush path: Hadamard rotation of new values, 2-bit (or 4-bit) quantization of what leaves the fp16 window,
// tile packing, and the update of the linear-correction states (Sec. 3.1, Obs. 3; Sec. 2, Eq. 1; Sec. 3.2, Eq. 5-6;
// Sec. 3.3: the cache is quantized only after attention has used the new token).
//
// This translation unit is compiled with floating-point contraction off: the rotation and the quantizer are
// bit-exact contracts (one binary32 rounding per written operation).
#include <hip/hip_runtime.h>

#include "kvlinc_internal.h"
#include "kvlinc_mfma.h"

#pragma clang fp contract(off)

namespace kvlinc {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kRowH = 136;     // halfs per LDS row of a 128-wide fp16 tile (rows stay 16-byte aligned)
constexpr int kParts = 2;      // workgroups that share the flush of one (sequence, kv head): the two halves of phi
constexpr int kListCap = kThreads;  // items one workgroup looks at per round (one per thread)
constexpr int kPlaneWords = 1024;   // a 128 x 128 tile of 2-bit codes; 4-bit codes take two such planes per tile

struct Lds {
  // raw keys / rotated values [token][channel]; after the quantizer the high / low term of K - K_q; after the logits
  // the high / low term of phi s of the group for this workgroup's 128 features, [feature][token]
  half_t bK[kGroup][kRowH];
  half_t bV[kGroup][kRowH];
  // value codes as the binary16 numbers (code - centre) / f_t (centre = 1.5 at 2 bits, 7.5 at 4; f_t a power of two per
  // token, see vFactor), [token / 4][channel][token % 4]: what the S update multiplies by, and -- sign and magnitude --
  // what the record stores of a code
  half_t cV[kGroup / 4][kHeadDim][4];
  float kScale[kGroup], kZero[kGroup];
  // vScale: the value scale s_t times f_t, the power of two that brings it to [2^13, 2^14) (or as near as the exponent
  // range of the codes' binary16 form allows): phi s_t f_t then fills binary16's range from the top, and the two binary16
  // terms it is carried in leave 2^-38 of the largest entry rather than 2^-25 of one.  vCentre: z + centre s, the value
  // of the centre of the code range.
  float vScale[kGroup], vCentre[kGroup], vFactor[kGroup];
  half_t kmn[kWaves][kGroup], kmx[kWaves][kGroup];  // per-channel key minima / maxima of each wave's tokens
  half_t Wt[kRank / 2][kRowH];  // W_k of the half of phi this workgroup belongs to, [feature][channel]
  float red[kWaves][kRank / 2];
  int light[kListCap], heavy[kListCap];
  int n_light, n_heavy, last_flag;
  // one-token append: the item that thread w looked at is a light one whose new row wave w has read ahead; the
  // sequence's counters as that thread read them
  int ahead[kWaves], ahead_nq[kWaves], ahead_nr[kWaves], ahead_n[kWaves];
};

__device__ inline bool nonfinite_bits(half_t x) {
  return (__builtin_bit_cast(unsigned short, x) & 0x7C00u) == 0x7C00u;
}

// One wave rotates one 128-vector: lane l holds elements 2l and 2l+1.  Stage order h = 1, 2, ..., 64 with
// (x[i], x[i+h]) <- (x[i] + x[i+h], x[i] - x[i+h]) for (i & h) == 0, then the binary32 scale and one rounding to fp16.
__device__ inline void fwht128_wave(float& x0, float& x1, int lane) {
  const float a = x0 + x1;
  const float b = x0 - x1;
  x0 = a;
  x1 = b;
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {  // element stride h = 2m  <->  lane stride m
    const float o0 = __shfl_xor(x0, m, 64);
    const float o1 = __shfl_xor(x1, m, 64);
    const bool upper = (lane & m) != 0;
    x0 = upper ? (o0 - x0) : (x0 + o0);
    x1 = upper ? (o1 - x1) : (x1 + o1);
  }
  const float c = 0x1.6a09e6p-4f;  // fl32(1/sqrt(128))
  x0 = x0 * c;
  x1 = x1 * c;
  // The contract rounds the product to binary32 first and to fp16 afterwards.  Keep the two roundings apart: a
  // fused multiply-and-convert instruction would round the exact product once and differ in rare near-tie cases.
  asm volatile("" : "+v"(x0), "+v"(x1));
}

// The same rotation for NV independent vectors at once (their cross-lane exchanges overlap); per vector the
// operations and their order are those of fwht128_wave.
template <int NV>
__device__ inline void fwht128_wave_multi(float (&x0)[NV], float (&x1)[NV], int lane) {
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const float a = x0[u] + x1[u];
    const float b = x0[u] - x1[u];
    x0[u] = a;
    x1[u] = b;
  }
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    const bool upper = (lane & m) != 0;
    float o0[NV], o1[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      o0[u] = __shfl_xor(x0[u], m, 64);
      o1[u] = __shfl_xor(x1[u], m, 64);
    }
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      x0[u] = upper ? (o0[u] - x0[u]) : (x0[u] + o0[u]);
      x1[u] = upper ? (o1[u] - x1[u]) : (x1[u] + o1[u]);
    }
  }
  const float c = 0x1.6a09e6p-4f;  // fl32(1/sqrt(128))
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    x0[u] = x0[u] * c;
    x1[u] = x1[u] * c;
    asm volatile("" : "+v"(x0[u]), "+v"(x1[u]));  // keep the binary32 rounding apart from the conversion to fp16
  }
}

// Eq. 1 at 2 or 4 bits against the stored fp16 scale / zero-point, decided in binary32 without a division.
struct QP {
  float z;  // value of the stored fp16 zero-point
  float s;  // value of the stored fp16 scale
  half_t z16, s16;
};

template <int BITS>
__device__ inline QP q_params(float mn, float mx) {
  mn = (mn == 0.0f) ? 0.0f : mn;  // a zero of either sign counts as +0
  mx = (mx == 0.0f) ? 0.0f : mx;
  QP r;
  r.z16 = (half_t)mn;  // exact: mn is an fp16 value
  r.z = mn;
  const float d32 = mx - mn;
  const float q32 = d32 / (float)Rec<BITS>::kLevels;  // IEEE-correct binary32 division
  r.s16 = (half_t)q32;
  r.s = (float)r.s16;
  return r;
}

// The code is the number of thresholds (k + 0.5) s, k = 0 .. 2^BITS - 2, that t = x - z lies above -- strictly for even
// k, or on for odd k: round-half-to-even of t / s, clamped.  The thresholds are exact in binary32 (s has 11 significant
// bits, 2 k + 1 at most 5).
template <int BITS>
__device__ inline uint32_t q_code(float x, const QP& p) {
  const float t = x - p.z;
  if constexpr (BITS == 2) {
    const uint32_t c = (uint32_t)(t > 0.5f * p.s) + (uint32_t)(t >= 1.5f * p.s) + (uint32_t)(t > 2.5f * p.s);
    return p.s == 0.0f ? 0u : c;
  } else {
    // An estimate e of the code from an approximate quotient (off by one at most, and only next to a threshold), then
    // the two thresholds around it decide: k = e - 1 (the code is at least e) and k = e (it is e + 1).  t is never
    // negative, so threshold -1 always passes; a code beyond the last level can only come from a scale that was
    // rounded down among the fp16 subnormals, and is clamped like the count of thresholds is.
    constexpr float kTop = (float)Rec<BITS>::kLevels;
    const float e = fminf(fmaxf(__builtin_rintf(t * __builtin_amdgcn_rcpf(p.s)), 0.0f), kTop);
    const bool e_odd = ((int)e & 1) != 0;
    const float lo = (e - 0.5f) * p.s, hi = (e + 0.5f) * p.s;
    const bool at_least_e = e_odd ? t > lo : t >= lo;       // threshold k = e - 1 is even iff e is odd
    const bool above_e = e_odd ? t >= hi : t > hi;
    const float c = fminf(e - 1.0f + (at_least_e ? 1.0f : 0.0f) + (at_least_e && above_e ? 1.0f : 0.0f), kTop);
    return p.s == 0.0f ? 0u : (uint32_t)c;
  }
}

// Every (sequence, kv head) has kParts * n_chunks owners in the grid, fixed by the launch shape alone (n_chunks > 1
// only in a bulk append of few sequences, whose groups are then shared out in chunks).  Each owner reads the sequence's
// counters once and counts itself in at the sequence's first split_done entry when it is done -- with a vote in the
// upper half of the counter if it found a fault; the counters change only in the arrival that completes the count
// (kParts n_chunks H_kv), i.e. after every reader has read them, and only if nobody voted against.  The scan launch
// that precedes a bulk append raises bit 30 of the same entry for a sequence with a non-finite new row: it reads as a
// vote.  The completing arrival leaves the entry at zero, as the decode kernel, which uses the same entries in the
// same way, expects.
constexpr int kFaultVote = 1 << 16;
constexpr int kScanFlag = 1 << 30;
__device__ inline bool arrive(const kvlinc_cache& c, int b, int n_chunks, bool vote, bool* clean) {
  int* counter = c.split_done + (long long)b * c.H_kv;
  const int before = __hip_atomic_fetch_add(counter, vote ? 1 + kFaultVote : 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  *clean = !vote && before < kFaultVote;
  return (before & (kFaultVote - 1)) == kParts * n_chunks * c.H_kv - 1;
}
__device__ inline void finish(const kvlinc_cache& c, int b, int nq, int n, const AppendPlan& plan, bool clean) {
  if (clean && plan.err == 0 && n > 0) {
    c.n_quant[b] = nq + plan.n_flush;
    c.n_res[b] = plan.new_res;
  }
  c.split_done[(long long)b * c.H_kv] = 0;
}
__device__ inline bool scan_flag(const kvlinc_cache& c, int b) {
  return (__hip_atomic_load(c.split_done + (long long)b * c.H_kv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) & kScanFlag) != 0;
}

__device__ inline bool nonfinite_pair(uint32_t w) { return ((w & 0x7C00u) == 0x7C00u) || ((w & 0x7C000000u) == 0x7C000000u); }

// One wave: raw key and rotated value of one new token into its window slot (values live 4 slots per channel: slot u,
// channel ch at [u / 4][ch][u % 4]).  Nothing of a row with a non-finite key or rotated value is stored; returns
// whether the row was such a row.
// (kk, vv: the lane's two elements of the new key and value row)
__device__ inline bool store_window_row(half_t* __restrict__ k_win, half_t* __restrict__ v_win, int slot, uint32_t kk,
                                        uint32_t vv, int lane) {
  const half2_t v2 = as_h2(vv);
  float x0 = (float)v2[0], x1 = (float)v2[1];
  fwht128_wave(x0, x1, lane);
  const half_t r0 = (half_t)x0, r1 = (half_t)x1;
  const bool mine = nonfinite_pair(kk) || nonfinite_bits(r0) || nonfinite_bits(r1);
  if (__builtin_amdgcn_ballot_w64(mine) != 0) return true;
  *reinterpret_cast<uint32_t*>(k_win + (long long)slot * kHeadDim + 2 * lane) = kk;
  v_win[((long long)(slot >> 2) * kHeadDim + 2 * lane) * 4 + (slot & 3)] = r0;
  v_win[((long long)(slot >> 2) * kHeadDim + 2 * lane + 1) * 4 + (slot & 3)] = r1;
  return false;
}
__device__ inline bool store_window_row(half_t* __restrict__ k_win, half_t* __restrict__ v_win, int slot,
                                        const half_t* __restrict__ ks, const half_t* __restrict__ vs, int lane) {
  return store_window_row(k_win, v_win, slot, *reinterpret_cast<const uint32_t*>(ks + 2 * lane),
                          *reinterpret_cast<const uint32_t*>(vs + 2 * lane), lane);
}

// One-token append: is the new row of any kv head of sequence b non-finite (key) or beyond fp16 once rotated (value)?
// The caller's waves share the heads: wave `first` of `stride` takes the heads first, first + stride, ..., eight per
// batch; the verdicts of the waves still have to be combined.  g: a head whose row may be read in place of a missing one.
__device__ inline bool new_rows_of_all_heads_bad(const kvlinc_cache& c, int b, int g, const half_t* __restrict__ k_new,
                                                 const half_t* __restrict__ v_new, int lane, int first, int stride) {
  bool refuse = false;
  for (int g0 = first; g0 < c.H_kv; g0 += stride * 8) {
    uint32_t chk_k[8], chk_v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int g2 = g0 + stride * u;
      const long long row = ((long long)b * c.H_kv + (g2 < c.H_kv ? g2 : g)) * kHeadDim + 2 * lane;
      chk_k[u] = *reinterpret_cast<const uint32_t*>(k_new + row);
      chk_v[u] = *reinterpret_cast<const uint32_t*>(v_new + row);
    }
    // A rotated value is at most sum_i |v_i| / sqrt(128): rows whose sum of magnitudes stays below
    // 65504 sqrt(128) cannot overflow fp16 and need no rotation here (a non-finite v makes the sum non-finite).
    float mag[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      refuse |= nonfinite_pair(chk_k[u]);
      const half2_t h = as_h2(chk_v[u]);
      mag[u] = fabsf((float)h[0]) + fabsf((float)h[1]);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) mag[u] = wave_allsum(mag[u]);
#pragma unroll
    for (int u0 = 0; u0 < 8; u0 += 4) {
      if (mag[u0] < 741000.0f && mag[u0 + 1] < 741000.0f && mag[u0 + 2] < 741000.0f && mag[u0 + 3] < 741000.0f) continue;
      float x0[4], x1[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const half2_t h = as_h2(chk_v[u0 + u]);
        x0[u] = (float)h[0];
        x1[u] = (float)h[1];
      }
      fwht128_wave_multi<4>(x0, x1, lane);
#pragma unroll
      for (int u = 0; u < 4; ++u) refuse |= nonfinite_bits((half_t)x0[u]) || nonfinite_bits((half_t)x1[u]);
    }
  }
  return refuse;
}

struct Counters {
  int nq, nr, n;
  AppendPlan plan;
};
__device__ inline Counters read_counters(const kvlinc_cache& c, int b, const int32_t* __restrict__ n_new, int T, int keep) {
  Counters r;
  r.nq = c.n_quant[b];
  r.nr = c.n_res[b];
  int n = n_new ? n_new[b] : T;
  r.n = n < 0 ? 0 : (n > T ? T : n);
  r.plan = plan_append(r.nq, r.nr, r.n, c.R, keep, c.max_groups);
  return r;
}

// An append that quantizes nothing: one wave stores the new rows of one (sequence, kv head) behind the window's
// tokens.  The slots are dead storage until the counters advance, and they do not advance if any head of the sequence
// votes against.
// known: the sequence's counters as read before, and the lane's elements of the pair's (only) new row, read ahead into
// row_k, row_v (one-token append).
template <bool SLIDING>
__device__ inline void light_item(const kvlinc_cache& c, int p, const half_t* __restrict__ k_new,
                                  const half_t* __restrict__ v_new, const int32_t* __restrict__ n_new, int T, int keep,
                                  int n_chunks, int lane, const Counters* known = nullptr, uint32_t row_k = 0,
                                  uint32_t row_v = 0) {
  const int b = p / c.H_kv;
  const bool have_row = known != nullptr;
  const Counters s = have_row ? *known : read_counters(c, b, n_new, T, keep);
  half_t* k_win = reinterpret_cast<half_t*>(c.k_res) + (long long)p * c.R * kHeadDim;
  half_t* v_win = reinterpret_cast<half_t*>(c.v_res) + (long long)p * c.R * kHeadDim;
  const half_t* k_src = k_new + (long long)p * T * kHeadDim;
  const half_t* v_src = v_new + (long long)p * T * kHeadDim;
  bool row_bad = false;
  // With the sliding value window the value slots behind the key window are live (the values of the newest group's
  // last tokens): nothing may be written there before ALL new rows of ALL kv heads of the sequence have been looked at
  // (several rows: by the scan launch, which precedes every bulk append to such a cache; one row and one kv head: the
  // row is looked at before it is stored anyway).
  if (SLIDING) {
    if (T > 1) row_bad = scan_flag(c, b);
    else if (c.H_kv > 1) row_bad = __builtin_amdgcn_ballot_w64(new_rows_of_all_heads_bad(c, b, p % c.H_kv, k_new, v_new, lane, 0, 1)) != 0;
  }
  if (have_row) {
    if (s.n > 0 && !row_bad) row_bad = store_window_row(k_win, v_win, s.nr, row_k, row_v, lane);
  } else {
    for (int i = 0; i < s.n && !row_bad; ++i)
      row_bad |= store_window_row(k_win, v_win, s.nr + i, k_src + (long long)i * kHeadDim, v_src + (long long)i * kHeadDim, lane);
  }
  if (lane == 0) {
    if (row_bad) atomicOr(c.status, KVLINC_ST_NONFINITE);
    bool clean;
    if (arrive(c, b, n_chunks, row_bad, &clean)) finish(c, b, s.nq, s.n, s.plan, clean);
  }
}

// Non-finite input is refused before anything of the sequence is stored (the window never holds a non-finite value,
// so only the new tokens need a look): a raw key, or a rotated value after its rounding to fp16, that is Inf or NaN.
// One wave, one row: lane l looks at elements 2 l and 2 l + 1.
__device__ inline bool row_is_bad(const half_t* __restrict__ k_row, const half_t* __restrict__ v_row, int lane) {
  const uint32_t kk = *reinterpret_cast<const uint32_t*>(k_row + 2 * lane);
  bool bad = ((kk & 0x7C00u) == 0x7C00u) || ((kk & 0x7C000000u) == 0x7C000000u);
  float x0 = (float)v_row[2 * lane], x1 = (float)v_row[2 * lane + 1];
  fwht128_wave(x0, x1, lane);
  return bad || nonfinite_bits((half_t)x0) || nonfinite_bits((half_t)x1);
}

// Scan launch of a bulk append (T > 1) to a cache with more than one kv head, or whose groups are shared out in
// chunks: every new row of every (sequence, kv head) is looked at once, and a fault raises the sequence's flag (bit 30
// of its first split_done entry) so that ALL the workgroups of that sequence in the append launch that follows refuse
// the append, whichever head or chunk the fault is in.  (With one kv head and one chunk the two workgroups of the
// sequence see all its rows themselves; a one-token append looks at the new rows of all heads itself.)  It also
// precedes every bulk append to a cache with the sliding value window, whose value slots behind the key window are live:
// there not even the rows ahead of a faulty one may be stored.
// Grid: (B H_kv, chunks of kScanRows rows).
constexpr int kScanRows = 256;
__global__ __launch_bounds__(kThreads) void append_scan_kernel(kvlinc_cache c, const half_t* __restrict__ k_new,
                                                                const half_t* __restrict__ v_new,
                                                                const int32_t* __restrict__ n_new, int T) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.x / c.H_kv;
  int n = n_new ? n_new[b] : T;
  n = n < 0 ? 0 : (n > T ? T : n);
  const int first = blockIdx.y * kScanRows, last = min(n, first + kScanRows);
  const half_t* k_src = k_new + (long long)blockIdx.x * T * kHeadDim;
  const half_t* v_src = v_new + (long long)blockIdx.x * T * kHeadDim;
  bool bad = false;
  for (int t = first + wave; t < last; t += kThreads / 64)
    bad |= row_is_bad(k_src + (long long)t * kHeadDim, v_src + (long long)t * kHeadDim, lane);
  if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) atomicOr(c.split_done + (long long)b * c.H_kv, kScanFlag);
}

__device__ inline void unpack8(const uint4& raw, float (&x)[8]) {
  const half2_t a = as_h2(raw.x), b = as_h2(raw.y), c = as_h2(raw.z), d = as_h2(raw.w);
  x[0] = (float)a[0]; x[1] = (float)a[1]; x[2] = (float)b[0]; x[3] = (float)b[1];
  x[4] = (float)c[0]; x[5] = (float)c[1]; x[6] = (float)d[0]; x[7] = (float)d[1];
}
__device__ inline bool nonfinite_any(const uint4& raw) {
  return nonfinite_pair(raw.x) || nonfinite_pair(raw.y) || nonfinite_pair(raw.z) || nonfinite_pair(raw.w);
}

// reductions over the 16 lanes of a row, and over a pair of rows (lanes 0..31 / 32..63), result in every lane
__device__ __forceinline__ float row16_min(float v) {
  v = fminf(v, dpp_f<kRowRor1>(v));
  v = fminf(v, dpp_f<kRowRor2>(v));
  v = fminf(v, dpp_f<kRowRor4>(v));
  return fminf(v, dpp_f<kRowRor8>(v));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_f<kRowRor1>(v));
  v = fmaxf(v, dpp_f<kRowRor2>(v));
  v = fmaxf(v, dpp_f<kRowRor4>(v));
  return fmaxf(v, dpp_f<kRowRor8>(v));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f<kRowRor1>(v);
  v += dpp_f<kRowRor2>(v);
  v += dpp_f<kRowRor4>(v);
  return v + dpp_f<kRowRor8>(v);
}
// The exchange swaps the odd rows of its first operand with the even rows of its second: given the same value twice,
// lane l ends up with its own value and that of lane l ^ 16.  (The second copy is made opaque: this compiler otherwise
// takes the two results of the exchange for equal.)
__device__ __forceinline__ void rowpair_exchange(float v, float& mine_or_other, float& other_or_mine) {
  uint32_t x = __builtin_bit_cast(uint32_t, v), y = x;
  asm volatile("" : "+v"(y));
  const auto a = __builtin_amdgcn_permlane16_swap(x, y, false, false);
  uint32_t a0 = a[0], a1 = a[1];
  asm volatile("" : "+v"(a0), "+v"(a1));
  mine_or_other = __builtin_bit_cast(float, a0);
  other_or_mine = __builtin_bit_cast(float, a1);
}
// reductions over the lanes l, l ^ 16, l ^ 32, l ^ 48 (the four rows of a wave), result in every lane
__device__ __forceinline__ void rows_exchange32(float v, float& p, float& q) {
  uint32_t x = __builtin_bit_cast(uint32_t, v), y = x;
  asm volatile("" : "+v"(y));
  const auto a = __builtin_amdgcn_permlane32_swap(x, y, false, false);
  uint32_t a0 = a[0], a1 = a[1];
  asm volatile("" : "+v"(a0), "+v"(a1));
  p = __builtin_bit_cast(float, a0);
  q = __builtin_bit_cast(float, a1);
}
__device__ __forceinline__ float rows_sum(float v) {
  float p, q;
  rowpair_exchange(v, p, q);
  rows_exchange32(p + q, p, q);
  return p + q;
}
__device__ __forceinline__ float rows_min(float v) {
  float p, q;
  rowpair_exchange(v, p, q);
  rows_exchange32(fminf(p, q), p, q);
  return fminf(p, q);
}
__device__ __forceinline__ float rows_max(float v) {
  float p, q;
  rowpair_exchange(v, p, q);
  rows_exchange32(fmaxf(p, q), p, q);
  return fmaxf(p, q);
}

// bits of the binary16 number (code - 1.5) times a power of two that make the stored bit pair: hi = sign (codes 0, 1),
// lo = magnitude 1.5 rather than 0.5 (codes 0, 3), the leading fraction bit
__device__ __forceinline__ uint32_t hi_of(uint32_t h16) { return (h16 >> 15) & 1u; }
__device__ __forceinline__ uint32_t lo_of(uint32_t h16) { return (h16 >> 9) & 1u; }

// One of the two workgroups that flush the groups of one (sequence, kv head).  Both stage and quantize the whole group
// (the quantizer's outputs feed both halves of the state update); part fp writes half of the record's tile words
// (part 0 also the scales and zero-points) and owns the half fp of phi: the features 128 fp .. 128 fp + 127 of S and P
// (Eq. 6 normalises each half by itself).  The state update runs on the matrix cores (16x16x32, binary16 operands
// whose products are exact: the centred codes are multiples of 0.5, W_k is binary16, the key error and phi s are carried
// as two binary16 terms):
//   logits[t][f] = sum_c (K - K_q)[t][c] W_k[c][f]   for the 128 features of the part's half,
//   phi = softmax over that half (Eq. 6),
//   S[f][c] += sum_t (phi s_t)[t][f] (code[t][c] - ctr) + sum_t phi[t][f] (z_t + ctr s_t),   P[f] += sum_t phi[t][f]   (Eq. 5)
// with V_q[t][c] = z_t + s_t code[t][c] and ctr = (2^BITS - 1) / 2 the centre of the code range.  S stays in registers for all groups of the call.  The matrix instruction lines
// its 32 products and its addend up with the largest of them before it adds, so what it is given is kept small and of
// both signs: the products of every 32 tokens start from a zero addend and are added to S by ordinary binary32
// additions, the codes are centred (the other part is the same for all channels of a row), and of the two terms of the
// key error the small one is contracted first.
template <bool SLIDING, int BITS>
__device__ void flush_item(const kvlinc_cache& c, Lds& L, int item, const half_t* __restrict__ k_new,
                           const half_t* __restrict__ v_new, const int32_t* __restrict__ n_new, int T, int keep,
                           int n_chunks, int tid) {
  using R = Rec<BITS>;
  constexpr float kCentre = R::kCentre;
  const int lane = tid & 63, wave = tid >> 6;
  const int ck = item % n_chunks, fp = (item / n_chunks) % kParts, p = item / (n_chunks * kParts);
  const int b = p / c.H_kv, g = p % c.H_kv;
  const long long bh = p;
  const Counters s = read_counters(c, b, n_new, T, keep);
  const int nq = s.nq, nr = s.nr, n = s.n;
  const AppendPlan plan = s.plan;
  // Chunks (bulk append of few sequences): the groups of the call are shared out evenly among n_chunks owners per
  // part, each of which forms the sum of its groups' contributions to S and P and adds it to the fp32 state in memory
  // with atomic additions (the order of the additions, and with it the last bits of S, then differ from run to run);
  // the arrival that completes the sequence rounds S to its binary16 tiles.  A call with one chunk in use -- every
  // one-token append, every cache without an fp32 state -- keeps S in registers from load to store.
  const int per_chunk = (plan.n_groups + n_chunks - 1) / n_chunks;
  const int j_first = ck * per_chunk, j_last = min(plan.n_groups, j_first + per_chunk);
  const bool chunked = plan.n_groups > per_chunk;  // more than one chunk has groups
  const bool has_work = j_first < j_last;          // (without chunks: the owner of chunk 0 only)

  // (The loads of W_k and of the state are issued before the new rows are looked at: they are wanted in any case but a
  // refusal, and nothing is stored to global memory before the verdict.)
  const half_t* k_res = reinterpret_cast<const half_t*>(c.k_res) + bh * c.R * kHeadDim;
  const half_t* v_res = reinterpret_cast<const half_t*>(c.v_res) + bh * c.R * kHeadDim;
  const half_t* k_src = k_new + bh * (long long)T * kHeadDim;
  const half_t* v_src = v_new + bh * (long long)T * kHeadDim;
  const bool states_live = c.S16 != nullptr;
  const bool have_master = c.S != nullptr;  // fp32 master copy of S; without it the state lives in its binary16 tiles

  // matrix-core roles of a lane: column l16 of a 16-wide tile, rows 4 kq .. 4 kq + 3 of the result, and the eight
  // contraction indices 8 kq .. 8 kq + 7 of each 32-wide step (the same in both operands, so any order of them serves).
  // Logits and softmax: wave w takes the tokens 16 w .. 16 w + 15 and all 128 features of the half (8 tiles), so a
  // token's features sit in the 16 lanes of a row and in the lane's own registers.  S update: wave w holds the rows
  // 16 w .. 16 w + 15 of the half and all 128 channels, eight tiles of 16.
  const int l16 = lane & 15, kq = lane >> 4;
  const int fw = 16 * wave;
  const int frow = (kRank / 2) * fp + fw + 4 * kq;  // first of the 4 rows of S this lane holds in every accumulator
  const int tile0 = ((frow >> 6) * 2) * 16 + ((frow & 63) >> 2);  // binary16 tile of these rows for the channels 0..63
  half_t* tiles = reinterpret_cast<half_t*>(c.S16) + bh * kRank * kHeadDim;

  float4_t acc[8];  // S[frow + r][16 ct + l16]
  float Pacc[8];    // sums of phi[t][16 fo + l16] over the tokens 4 kq .. 4 kq + 3 of this wave's tiles
#pragma unroll
  for (int fo = 0; fo < 8; ++fo) Pacc[fo] = 0.0f;
  float P_old = 0.0f;
  if (states_live && has_work) {
    const half_t* W0 = reinterpret_cast<const half_t*>(c.Wk) + ((long long)g * 2 + fp) * kHeadDim * (kRank / 2);
    {  // transposed into LDS: a lane's B operand (8 channels of one feature) is then one 16-byte read.  Thread: feature
       // tid % 128 (consecutive lanes read consecutive halfs of a row of W), 8 channels per step.
      const int f = tid & 127, c0 = 8 * (tid >> 7);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        half8_t w;
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = W0[(long long)(c0 + 32 * i + e) * (kRank / 2) + f];
        *reinterpret_cast<half8_t*>(&L.Wt[f][c0 + 32 * i]) = w;
      }
    }
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) {
      if (chunked) {
        acc[ct] = float4_t{0.f, 0.f, 0.f, 0.f};
      } else if (have_master) {
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[ct][r] = c.S[(bh * kRank + frow + r) * kHeadDim + 16 * ct + l16];
      } else {
        const half4_t t16 = *reinterpret_cast<const half4_t*>(tiles + ((tile0 + 16 * (ct >> 2)) * 64 + 16 * (ct & 3) + l16) * 4);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[ct][r] = (float)t16[r];
      }
    }
    if (tid < kRank / 2 && !chunked) P_old = c.P[bh * kRank + (kRank / 2) * fp + tid];
  }
  {
    // non-finite new tokens: the verdict has to be the same in all workgroups of the sequence
    bool refuse = false;
    if (T == 1) {
      // A one-token append that flushes the window changes live state (S, P, the window's first slot) in every kv
      // head: the new row of every kv head of this sequence is looked at first, eight heads per wave and batch.
      refuse = new_rows_of_all_heads_bad(c, b, g, k_new, v_new, lane, wave, kWaves);
    } else if (c.H_kv > 1 || n_chunks > 1 || SLIDING) {
      refuse = scan_flag(c, b);  // raised by the scan launch
    } else {
      // bulk append, one kv head: the parts of this (sequence, kv head) are the sequence's only workgroups and see the
      // same rows.  The new rows that will stay in the window (at most R) are looked at here; those that get quantized
      // are looked at when their group is staged, before anything but dead storage has been written.
      const half_t* ks = k_new + (long long)b * T * kHeadDim;
      const half_t* vs = v_new + (long long)b * T * kHeadDim;
      for (int u = max(plan.n_flush, nr) + wave; u < nr + n; u += kWaves)
        refuse |= row_is_bad(ks + (long long)(u - nr) * kHeadDim, vs + (long long)(u - nr) * kHeadDim, lane);
    }
    if (__syncthreads_or(refuse)) {
      if (tid == 0) {
        if (fp == 0) atomicOr(c.status, KVLINC_ST_NONFINITE);
        bool clean;
        if (arrive(c, b, n_chunks, true, &clean)) finish(c, b, nq, n, plan, false);
      }
      return;
    }
  }

  bool bad = false;
  const int sub = tid & 15, tq = tid >> 4;  // quantizer roles: channels 8 sub .. 8 sub + 7; tq = 0 .. 31

  for (int j = j_first; j < j_last; ++j) {
    const int valid = min(kGroup, plan.n_flush - j * kGroup);
    const long long grp = (long long)(nq / kGroup) + j;
    uint32_t* rec = c.groups + (bh * c.max_groups + grp) * R::kWords;
    half_t* rec16 = reinterpret_cast<half_t*>(rec);
    const int ubase = j * kGroup;                    // index of the group's first token in the stream [window, new]
    const int nrg = min(max(nr - ubase, 0), valid);  // tokens of this group that come from the window (only if j == 0)
    // ---- 1. stage the group's raw keys and (raw or already rotated) values in LDS -------------------------
    {
      uint4 kv[4], vv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {  // 16-byte pieces: 16 per token row; token tq + 32 i, piece sub
        const int t = tq + 32 * i, u = ubase + t;
        kv[i] = make_uint4(0, 0, 0, 0);
        vv[i] = make_uint4(0, 0, 0, 0);
        if (t < valid) {
          if (u < nr) {
            kv[i] = *reinterpret_cast<const uint4*>(k_res + (long long)u * kHeadDim + sub * 8);
          } else {
            kv[i] = *reinterpret_cast<const uint4*>(k_src + (long long)(u - nr) * kHeadDim + sub * 8);
            vv[i] = *reinterpret_cast<const uint4*>(v_src + (long long)(u - nr) * kHeadDim + sub * 8);
          }
        }
      }
      // window values live 4 slots per channel: a 16-byte load brings 4 tokens of 2 channels
      uint4 wv[4];
      const int n_wv = ((nrg + 3) >> 2) * 64;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int it = tid + kThreads * i;
        wv[i] = make_uint4(0, 0, 0, 0);
        if (it < n_wv) wv[i] = *reinterpret_cast<const uint4*>(v_res + ((long long)(it >> 6) * kHeadDim + 2 * (it & 63)) * 4);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = tq + 32 * i;
        *reinterpret_cast<uint4*>(&L.bK[t][sub * 8]) = kv[i];
        if (t >= nrg) *reinterpret_cast<uint4*>(&L.bV[t][sub * 8]) = vv[i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int it = tid + kThreads * i, q = it >> 6, cp = it & 63;
        if (it < n_wv) {
          const uint4 w = wv[i];
          const uint32_t lo[4] = {w.x & 0xffffu, w.x >> 16, w.y & 0xffffu, w.y >> 16};
          const uint32_t hi[4] = {w.z & 0xffffu, w.z >> 16, w.w & 0xffffu, w.w >> 16};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (4 * q + e < nrg) *reinterpret_cast<uint32_t*>(&L.bV[4 * q + e][2 * cp]) = lo[e] | (hi[e] << 16);
        }
      }
    }
    __syncthreads();
    // rotate the rows that came from new tokens (window rows are rotated already)
    if (nrg < valid) {
      for (int tb = wave; tb < valid; tb += 4 * kWaves) {  // rows tb, tb + 8, tb + 16, tb + 24 together
        float x0[4], x1[4];
        bool act[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int t = tb + kWaves * u;
          act[u] = t < valid && t >= nrg;
          x0[u] = act[u] ? (float)L.bV[t][2 * lane] : 0.0f;
          x1[u] = act[u] ? (float)L.bV[t][2 * lane + 1] : 0.0f;
        }
        if (!(act[0] || act[1] || act[2] || act[3])) continue;
        fwht128_wave_multi<4>(x0, x1, lane);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (act[u]) {
            const int t = tb + kWaves * u;
            L.bV[t][2 * lane] = (half_t)x0[u];
            L.bV[t][2 * lane + 1] = (half_t)x1[u];
          }
        }
      }
      __syncthreads();
    }
    // ---- 2. Eq. 1: rotated values per token over the channels, keys per channel over the group's tokens ----
    // values: the 16 lanes of a row share the tokens 4 tq .. 4 tq + 3 (8 channels each); rows beyond `valid` are zero
    // and quantize to scale 0, zero-point 0, codes 0
    {
      float x[4][8], mn[4], mx[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint4 raw = *reinterpret_cast<const uint4*>(&L.bV[4 * tq + i][8 * sub]);
        bad |= nonfinite_any(raw);
        unpack8(raw, x[i]);
        mn[i] = fminf(fminf(fminf(x[i][0], x[i][1]), fminf(x[i][2], x[i][3])), fminf(fminf(x[i][4], x[i][5]), fminf(x[i][6], x[i][7])));
        mx[i] = fmaxf(fmaxf(fmaxf(x[i][0], x[i][1]), fmaxf(x[i][2], x[i][3])), fmaxf(fmaxf(x[i][4], x[i][5]), fmaxf(x[i][6], x[i][7])));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        mn[i] = row16_min(mn[i]);
        mx[i] = row16_max(mx[i]);
      }
      QP pv[4];
      float fac[4], inv_fac[4];  // f_t and 1 / f_t: 2^k with k = 13 - (exponent of s_t), kept inside -2 .. 13 so that
                                 // (code - centre) / f_t stays a normal binary16 number (0.5 * 2^-13 .. 7.5 * 4)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pv[i] = q_params<BITS>(mn[i], mx[i]);
        const int e = (int)(__builtin_bit_cast(uint32_t, pv[i].s) >> 23) - 127;
        const int k = pv[i].s == 0.0f ? 0 : min(max(13 - e, -2), 13);
        fac[i] = __builtin_bit_cast(float, (uint32_t)(127 + k) << 23);
        inv_fac[i] = __builtin_bit_cast(float, (uint32_t)(127 - k) << 23);
      }
#pragma unroll
      for (int e = 0; e < 8; e += 2) {  // two channels = 8 halfs = one 16-byte store
        half8_t h;
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // (exact: a multiple of 0.5 times a power of two)
          h[i] = (half_t)(((float)q_code<BITS>(x[i][e], pv[i]) - kCentre) * inv_fac[i]);
          h[4 + i] = (half_t)(((float)q_code<BITS>(x[i][e + 1], pv[i]) - kCentre) * inv_fac[i]);
        }
        *reinterpret_cast<half8_t*>(&L.cV[tq][8 * sub + e][0]) = h;
      }
      if (sub < 4) {  // lane sub of the row writes token 4 tq + sub
        QP mine = pv[0];
        float my_fac = fac[0];
        if (sub == 1) { mine = pv[1]; my_fac = fac[1]; }
        if (sub == 2) { mine = pv[2]; my_fac = fac[2]; }
        if (sub == 3) { mine = pv[3]; my_fac = fac[3]; }
        const int t = 4 * tq + sub;
        L.vScale[t] = mine.s * my_fac;
        L.vFactor[t] = my_fac;
        L.vCentre[t] = mine.z + kCentre * mine.s;
        if (fp == 0) {
          const int sz_word = R::kValueSZ + 8 * (t & 15) + (t >> 4);  // token 16 n + j at word 8 j + n of the field
          rec16[2 * sz_word] = mine.s16;
          rec16[2 * sz_word + 1] = mine.z16;
        }
      }
    }
    // keys: minima / maxima of 8 channels over the tokens tq, tq + 32, ...
    {
      float kmn[8], kmx[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        kmn[e] = INFINITY;
        kmx[e] = -INFINITY;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = tq + 32 * i;
        if (t < valid) {
          const uint4 raw = *reinterpret_cast<const uint4*>(&L.bK[t][8 * sub]);
          bad |= nonfinite_any(raw);
          float x[8];
          unpack8(raw, x);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            kmn[e] = fminf(kmn[e], x[e]);
            kmx[e] = fmaxf(kmx[e], x[e]);
          }
        }
      }
      // over the wave's four rows (token subsets), then one row of each wave leaves its minima / maxima
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        kmn[e] = rows_min(kmn[e]);
        kmx[e] = rows_max(kmx[e]);
      }
      if (kq == 0) {
        half8_t hmn, hmx;  // exact: the values are fp16 values or infinities
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          hmn[e] = (half_t)kmn[e];
          hmx[e] = (half_t)kmx[e];
        }
        *reinterpret_cast<half8_t*>(&L.kmn[wave][8 * sub]) = hmn;
        *reinterpret_cast<half8_t*>(&L.kmx[wave][8 * sub]) = hmx;
      }
    }
    __syncthreads();
    if (tid < kGroup) {
      float mn = (float)L.kmn[0][tid], mx = (float)L.kmx[0][tid];
#pragma unroll
      for (int r = 1; r < kWaves; ++r) {
        mn = fminf(mn, (float)L.kmn[r][tid]);
        mx = fmaxf(mx, (float)L.kmx[r][tid]);
      }
      const QP pk = q_params<BITS>(mn, mx);
      L.kScale[tid] = pk.s;
      L.kZero[tid] = pk.z;
      if (fp == 0) {
        rec16[2 * R::kKeyScale + tid] = pk.s16;
        rec16[2 * R::kKeyZero + tid] = pk.z16;
      }
    }
    __syncthreads();
    // key codes -- this part's half of the key tile goes out from registers -- and K - K_q as two binary16 terms in
    // place of the staged tiles.
    // 2 bits: tile word ((n / 2) * 64 + j + 16 g) * 4 + 2 (n % 2) + w holds, for the row 16 n + j, the positions
    // k = 32 g + 16 w + 8 (p % 2) + p / 2, p = 0..15: code p as the bit pair (hi, lo) = (1,1), (1,0), (0,0), (0,1) for the
    // codes 0..3, hi in bit 4 (p / 2) + 3 - p % 2, lo two below.  Key tile: row = token, position = channel: this
    // thread's 8 channels are the p % 2 = sub % 2 half of the word of (g, w) = (sub / 4, (sub / 2) % 2), its neighbour
    // in the lane pair has the other half.
    // 4 bits: the tile is two such planes of 1024 words, the first of the codes' high base-4 digits, the second of the low.
    {
      QP pk[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pk[e].s = L.kScale[8 * sub + e];
        pk[e].z = L.kZero[8 * sub + e];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = tq + 32 * i;
        const uint4 raw = *reinterpret_cast<const uint4*>(&L.bK[t][8 * sub]);
        float x[8];
        unpack8(raw, x);
        half8_t eh, el;
        uint32_t bits = 0, bits_lo = 0;  // (bits_lo: the low plane of 4-bit codes)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t code = t < valid ? q_code<BITS>(x[e], pk[e]) : 0u;
          float ke = t < valid ? x[e] - (pk[e].s * (float)code + pk[e].z) : 0.0f;
          asm volatile("" : "+v"(ke));  // the binary32 difference first, then its two binary16 terms
          eh[e] = (half_t)ke;
          el[e] = (half_t)(ke - (float)eh[e]);
          // of a 2-bit code (digit) x: hi = not (x / 2), lo = not (x / 2 xor x % 2)
          const uint32_t x = BITS == 2 ? code : code >> 2;
          bits |= (((x >> 1) ^ 1u) << (4 * e + 3 - (sub & 1))) | ((((x >> 1) ^ x ^ 1u) & 1u) << (4 * e + 1 - (sub & 1)));
          if constexpr (BITS == 4) {
            const uint32_t y = code & 3u;
            bits_lo |= (((y >> 1) ^ 1u) << (4 * e + 3 - (sub & 1))) | ((((y >> 1) ^ y ^ 1u) & 1u) << (4 * e + 1 - (sub & 1)));
          }
        }
        *reinterpret_cast<half8_t*>(&L.bK[t][8 * sub]) = eh;
        *reinterpret_cast<half8_t*>(&L.bV[t][8 * sub]) = el;
        bits |= dpp_u<kQuadSwap1>(bits);
        if constexpr (BITS == 4) bits_lo |= dpp_u<kQuadSwap1>(bits_lo);
        if ((i >> 1) == fp && (sub & 1) == 0) {  // this part's half of the key tile: the tokens 64 fp .. 64 fp + 63
          const int nb = t >> 4, jr = t & 15;
          const int word = ((nb >> 1) * 64 + jr + 16 * (sub >> 2)) * 4 + 2 * (nb & 1) + ((sub >> 1) & 1);
          rec[R::kKeyTile + word] = bits;
          if constexpr (BITS == 4) rec[R::kKeyTile + kPlaneWords + word] = bits_lo;
        }
      }
    }
    // ---- 3. this part's half of the value tile: row = channel 16 n + j, position k = token
    // 16 (k % 8) + 4 ((k / 16) % 4) + 2 (k / 64) + (k / 8) % 2, the bit pairs read off the centred codes ----
    {
      // (the centred codes of all tokens were stored before the last barrier)
      const int wi = (kPlaneWords / kParts) * fp + tid;
      const int w = wi & 1, nb = 2 * (wi >> 8) + ((wi >> 1) & 1), l = (wi >> 2) & 63, jr = l & 15, gq4 = l >> 4;
      const int row = 16 * nb + jr, k0 = 32 * gq4 + 16 * w;
      const int tok0 = 4 * ((k0 >> 4) & 3) + 2 * (k0 >> 6);  // token of position k0 + 8 e + i is 16 i + tok0 + e
      uint32_t vw = 0, vw_lo = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int t = 16 * i + tok0;  // even: t and t + 1 share a quad of tokens
        const uint32_t two = *reinterpret_cast<const uint32_t*>(&L.cV[t >> 2][row][t & 3]);
        if constexpr (BITS == 2) {
          const uint32_t h0 = two & 0xffffu, h1 = two >> 16;
          vw |= (hi_of(h0) << (4 * i + 3)) | (lo_of(h0) << (4 * i + 1)) | (hi_of(h1) << (4 * i + 2)) | (lo_of(h1) << (4 * i));
        } else {
          const half2_t h = as_h2(two);
          const float2 f2 = *reinterpret_cast<const float2*>(&L.vFactor[t]);
          const uint32_t c0 = (uint32_t)((float)h[0] * f2.x + kCentre), c1 = (uint32_t)((float)h[1] * f2.y + kCentre);  // exact
          const uint32_t x0 = c0 >> 2, x1 = c1 >> 2, y0 = c0 & 3u, y1 = c1 & 3u;
          vw |= (((x0 >> 1) ^ 1u) << (4 * i + 3)) | ((((x0 >> 1) ^ x0 ^ 1u) & 1u) << (4 * i + 1)) |
                (((x1 >> 1) ^ 1u) << (4 * i + 2)) | ((((x1 >> 1) ^ x1 ^ 1u) & 1u) << (4 * i));
          vw_lo |= (((y0 >> 1) ^ 1u) << (4 * i + 3)) | ((((y0 >> 1) ^ y0 ^ 1u) & 1u) << (4 * i + 1)) |
                   (((y1 >> 1) ^ 1u) << (4 * i + 2)) | ((((y1 >> 1) ^ y1 ^ 1u) & 1u) << (4 * i));
        }
      }
      rec[R::kValueTile + wi] = vw;
      if constexpr (BITS == 4) rec[R::kValueTile + kPlaneWords + wi] = vw_lo;
    }
    __syncthreads();
    // ---- 4. the group's contribution to S and P (Eq. 5, Eq. 6) ----------------------------------------------
    if (states_live) {
      float Zacc[8];  // as Pacc, of phi (z_t + centre s_t)
#pragma unroll
      for (int fo = 0; fo < 8; ++fo) Zacc[fo] = 0.0f;
      // a. logits of this wave's 16 tokens for the 128 features of the half; the small products (low term) first
      float4_t d[8];
#pragma unroll
      for (int ft = 0; ft < 8; ++ft) d[ft] = float4_t{0.f, 0.f, 0.f, 0.f};
      if (16 * wave < valid) {
        const int tr = 16 * wave + l16;
#pragma unroll 1
        for (int kk = 0; kk < 4; ++kk) {
          const half8_t aL = *reinterpret_cast<const half8_t*>(&L.bV[tr][32 * kk + 8 * kq]);
#pragma unroll
          for (int ft = 0; ft < 8; ++ft)
            d[ft] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aL, *reinterpret_cast<const half8_t*>(&L.Wt[16 * ft + l16][32 * kk + 8 * kq]), d[ft], 0, 0, 0);
        }
#pragma unroll 1
        for (int kk = 0; kk < 4; ++kk) {
          const half8_t aH = *reinterpret_cast<const half8_t*>(&L.bK[tr][32 * kk + 8 * kq]);
#pragma unroll
          for (int ft = 0; ft < 8; ++ft)
            d[ft] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aH, *reinterpret_cast<const half8_t*>(&L.Wt[16 * ft + l16][32 * kk + 8 * kq]), d[ft], 0, 0, 0);
        }
      }
      __syncthreads();  // every wave has read its rows of the key error: their place now takes phi s
      half_t(*phH)[kRowH] = L.bK;
      half_t(*phL)[kRowH] = L.bV;
      if (16 * wave < ((valid + 31) & ~31)) {
        // b. softmax over the half: register r of the lane belongs to token 16 wave + 4 kq + r, whose 128 features
        // are the 8 tiles times the 16 lanes of the row.  phi goes on as phi s_t in two binary16 terms, feature-major.
        // (Step c reads tokens in blocks of 32: a wave whose 16 tokens all lie beyond `valid` inside the last such
        // block writes its zeros -- inv = 0 -- over what the key error left there.)
        const int tb = 16 * wave + 4 * kq;
        const float4 sc4 = *reinterpret_cast<const float4*>(&L.vScale[tb]);
        const float4 ce4 = *reinterpret_cast<const float4*>(&L.vCentre[tb]);
        const float sc[4] = {sc4.x, sc4.y, sc4.z, sc4.w}, ce[4] = {ce4.x, ce4.y, ce4.z, ce4.w};
        float m[4], sum[4], inv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
          m[r] = fmaxf(fmaxf(fmaxf(d[0][r], d[1][r]), fmaxf(d[2][r], d[3][r])), fmaxf(fmaxf(d[4][r], d[5][r]), fmaxf(d[6][r], d[7][r])));
#pragma unroll
        for (int r = 0; r < 4; ++r) m[r] = row16_max(m[r]);
#pragma unroll
        for (int ft = 0; ft < 8; ++ft)
#pragma unroll
          for (int r = 0; r < 4; ++r) d[ft][r] = __expf(d[ft][r] - m[r]);
#pragma unroll
        for (int r = 0; r < 4; ++r) sum[r] = ((d[0][r] + d[1][r]) + (d[2][r] + d[3][r])) + ((d[4][r] + d[5][r]) + (d[6][r] + d[7][r]));
#pragma unroll
        for (int r = 0; r < 4; ++r) sum[r] = row16_sum(sum[r]);
#pragma unroll
        for (int r = 0; r < 4; ++r) inv[r] = tb + r < valid ? 1.0f / sum[r] : 0.0f;
#pragma unroll
        for (int fo = 0; fo < 8; ++fo) {
          const float4_t e = d[fo];
          half4_t h4, l4;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float ph = e[r] * inv[r];
            Pacc[fo] += ph;
            Zacc[fo] += ph * ce[r];
            float ws = ph * sc[r];
            // The two terms must add up to the binary32 product: keep its rounding apart from the conversion (a fused
            // multiply-and-convert would round the exact product once, and the low term would then belong to another
            // high term in the rare near-tie cases).
            asm volatile("" : "+v"(ws));
            h4[r] = (half_t)ws;
            l4[r] = (half_t)(ws - (float)h4[r]);
          }
          *reinterpret_cast<half4_t*>(&phH[16 * fo + l16][tb]) = h4;
          *reinterpret_cast<half4_t*>(&phL[16 * fo + l16][tb]) = l4;
        }
      }
      // the term of the code centres is the same for every channel of a row: summed over the wave's tokens here
#pragma unroll
      for (int fo = 0; fo < 8; ++fo) Zacc[fo] = rows_sum(Zacc[fo]);
      if (kq == 0) {
#pragma unroll
        for (int fo = 0; fo < 8; ++fo) L.red[wave][16 * fo + l16] = Zacc[fo];
      }
      __syncthreads();
      // c. S[f][c] += sum_t (phi s)[t][f] (code[t][c] - centre): this wave's 16 features, 8 tiles of 16 channels, 32 tokens
      // per instruction
      for (int t0 = 0; t0 < valid; t0 += 32) {
        const half8_t aH = *reinterpret_cast<const half8_t*>(&phH[fw + l16][t0 + 8 * kq]);
        const half8_t aL = *reinterpret_cast<const half8_t*>(&phL[fw + l16][t0 + 8 * kq]);
        const int q0 = (t0 >> 2) + 2 * kq;  // the lane's 8 tokens are two quads
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) {
          const int ch = 16 * ct + l16;
          const half4_t b0 = *reinterpret_cast<const half4_t*>(&L.cV[q0][ch][0]);
          const half4_t b1 = *reinterpret_cast<const half4_t*>(&L.cV[q0 + 1][ch][0]);
          const half8_t bc = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
          float4_t dd = __builtin_amdgcn_mfma_f32_16x16x32_f16(aH, bc, float4_t{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
          dd = __builtin_amdgcn_mfma_f32_16x16x32_f16(aL, bc, dd, 0, 0, 0);
          acc[ct] += dd;
        }
      }
      {
        float z[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w2 = 0; w2 < kWaves; ++w2) {
          const float4 zz = *reinterpret_cast<const float4*>(&L.red[w2][fw + 4 * kq]);
          z[0] += zz.x; z[1] += zz.y; z[2] += zz.z; z[3] += zz.w;
        }
#pragma unroll
        for (int ct = 0; ct < 8; ++ct)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[ct][r] += z[r];
      }
    }
    __syncthreads();
  }

  // A fault seen only now (one kv head per sequence in a bulk append; every part sees it) leaves states, window and
  // counters as they were; the records written above lie beyond n_quant and are dead storage.
  const bool any_bad = __syncthreads_or(bad) != 0;
  if (!any_bad && states_live && chunked) {
    if (has_work) {
#pragma unroll
      for (int ct = 0; ct < 8; ++ct)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          __hip_atomic_fetch_add(c.S + (bh * kRank + frow + r) * kHeadDim + 16 * ct + l16, acc[ct][r], __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_SYSTEM);
#pragma unroll
      for (int fo = 0; fo < 8; ++fo) Pacc[fo] = rows_sum(Pacc[fo]);
      if (kq == 0) {
#pragma unroll
        for (int fo = 0; fo < 8; ++fo) L.red[wave][16 * fo + l16] = Pacc[fo];
      }
      __syncthreads();
      if (tid < kRank / 2) {
        float add = 0.0f;
#pragma unroll
        for (int w2 = 0; w2 < kWaves; ++w2) add += L.red[w2][tid];
        __hip_atomic_fetch_add(c.P + bh * kRank + (kRank / 2) * fp + tid, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the additions of every wave are done before this owner
    __syncthreads();                                  // counts itself in
  } else if (!any_bad && states_live && has_work) {
    // fp32 master copy (if the cache keeps one), row-major, and the binary16 tiles the decode kernel reads: tile
    // (64-feature block, channel half hh, feature step fb) holds S[64 block + 4 fb + k][64 hh + l] at [l][k].
    // An entry beyond the binary16 range is stored as +-65504 and reported in the status word.
    bool out_of_range = false;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) {
      half4_t t16;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float v = acc[ct][r];
        if (have_master) c.S[(bh * kRank + frow + r) * kHeadDim + 16 * ct + l16] = v;
        out_of_range |= !(fabsf(v) <= 65504.0f);
        t16[r] = (half_t)fminf(fmaxf(v, -65504.0f), 65504.0f);
      }
      *reinterpret_cast<half4_t*>(tiles + ((tile0 + 16 * (ct >> 2)) * 64 + 16 * (ct & 3) + l16) * 4) = t16;
    }
    if (__builtin_amdgcn_ballot_w64(out_of_range) != 0 && lane == 0) atomicOr(c.status, KVLINC_ST_STATE_RANGE);
#pragma unroll
    for (int fo = 0; fo < 8; ++fo) Pacc[fo] = rows_sum(Pacc[fo]);
    if (kq == 0) {
#pragma unroll
      for (int fo = 0; fo < 8; ++fo) L.red[wave][16 * fo + l16] = Pacc[fo];
    }
    __syncthreads();
    if (tid < kRank / 2) {
      float add = 0.0f;
#pragma unroll
      for (int w2 = 0; w2 < kWaves; ++w2) add += L.red[w2][tid];
      c.P[bh * kRank + (kRank / 2) * fp + tid] = P_old + add;
    }
  }

  // count this part in; the arrival that completes the sequence stores the new rows that stay in the window -- raw
  // key, rotated value -- for all its kv heads (only now have all parts staged the window's old rows) and commits.
  // Stream index u >= n_flush goes to slot u - n_flush; old window tokens all left (n_flush >= n_res).
  if (tid == 0) {
    if (any_bad && fp == 0) atomicOr(c.status, KVLINC_ST_NONFINITE);
    bool clean;
    const bool last = arrive(c, b, n_chunks, any_bad, &clean);
    L.last_flag = last ? (clean ? 2 : 1) : 0;
  }
  __syncthreads();
  const int flag = L.last_flag;
  if (flag == 2 && chunked && states_live) {
    // every chunk of every kv head has added its share: S of all kv heads of the sequence goes to the binary16 tiles
    // (tile (64-feature block, channel half hh, feature step fb) holds S[64 block + 4 fb + k][64 hh + l] at [l][k])
    bool out_of_range = false;
    for (int i = tid; i < c.H_kv * 128 * 64; i += kThreads) {
      const int g2 = i >> 13, t = (i >> 6) & 127, l = i & 63;
      const long long bh2 = (long long)b * c.H_kv + g2;
      const int f0 = 64 * (t >> 5) + 4 * (t & 15), ch = 64 * ((t >> 4) & 1) + l;
      half4_t t16;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float v = __hip_atomic_load(c.S + (bh2 * kRank + f0 + k) * kHeadDim + ch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        out_of_range |= !(fabsf(v) <= 65504.0f);
        t16[k] = (half_t)fminf(fmaxf(v, -65504.0f), 65504.0f);
      }
      *reinterpret_cast<half4_t*>(reinterpret_cast<half_t*>(c.S16) + bh2 * kRank * kHeadDim + ((long long)t * 64 + l) * 4) = t16;
    }
    if (__builtin_amdgcn_ballot_w64(out_of_range) != 0 && lane == 0) atomicOr(c.status, KVLINC_ST_STATE_RANGE);
  }
  if (flag == 2) {
    const int first_new = max(plan.n_flush, nr), cnt = nr + n - first_new;
    for (int r = wave; r < cnt * c.H_kv; r += kWaves) {
      const int g2 = r / cnt, u = first_new + r % cnt;
      const long long bh2 = (long long)b * c.H_kv + g2;
      store_window_row(reinterpret_cast<half_t*>(c.k_res) + bh2 * c.R * kHeadDim,
                       reinterpret_cast<half_t*>(c.v_res) + bh2 * c.R * kHeadDim, u - plan.n_flush,
                       k_new + (bh2 * T + (u - nr)) * kHeadDim, v_new + (bh2 * T + (u - nr)) * kHeadDim, lane);
    }
  }
  if (SLIDING && flag == 2 && T > 1) {
    // Sliding value window after a bulk append: the newest 128 tokens keep their fp16 values, the value of stream
    // index u in window slot u % 128 (n_quant is a multiple of 128).  Those among them that were quantized in this
    // call and came in as new tokens are stored here (old window tokens lie in their slots already).
    const int lo = max(nr, nr + n - kGroup), cnt2 = plan.n_flush - lo;
    for (int r = wave; r < cnt2 * c.H_kv; r += kWaves) {
      const int g2 = r / cnt2, u = lo + r % cnt2, slot = u % kGroup;
      const long long bh2 = (long long)b * c.H_kv + g2;
      const half_t* vs = v_new + (bh2 * T + (u - nr)) * kHeadDim;
      half_t* v_win = reinterpret_cast<half_t*>(c.v_res) + bh2 * c.R * kHeadDim;
      float x0 = (float)vs[2 * lane], x1 = (float)vs[2 * lane + 1];
      fwht128_wave(x0, x1, lane);
      v_win[((long long)(slot >> 2) * kHeadDim + 2 * lane) * 4 + (slot & 3)] = (half_t)x0;
      v_win[((long long)(slot >> 2) * kHeadDim + 2 * lane + 1) * 4 + (slot & 3)] = (half_t)x1;
    }
  }
  __syncthreads();
  if (flag != 0 && tid == 0) finish(c, b, nq, n, plan, flag == 2);
}

// One launch serves every sequence: item it of the grid's list is part (it / 8) % kParts of the pair
// (it / (8 kParts)) * 8 + it % 8 of (sequence, kv head), and workgroup x owns the items x, x + G, x + 2 G, ...: the parts of a
// pair sit on one XCD (workgroups are dealt to the 8 XCDs in turn, and G is a multiple of 8), whose L2 then serves
// the rows that all of them stage.
// SLIDING: the variant for caches with the sliding value window (KVLINC_FLAG_SLIDING_VALUES) is a kernel of its own;
// BITS: so is the one for caches with 4-bit codes.
template <bool SLIDING, int BITS>
__global__ __launch_bounds__(kThreads) void append_flush_kernel(kvlinc_cache c, const half_t* __restrict__ k_new,
                                                                 const half_t* __restrict__ v_new,
                                                                 const int32_t* __restrict__ n_new, int T, int keep,
                                                                 int n_chunks) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  Lds& L = *reinterpret_cast<Lds*>(lds_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // (32-bit item arithmetic: at most 2^24 pairs, and more than two owners per pair only below 64 pairs)
  const uint32_t n_pairs = (uint32_t)c.B * (uint32_t)c.H_kv;
  const uint32_t owners = kParts * n_chunks;  // per (sequence, kv head)
  const uint32_t n_items = owners * 8u * ((n_pairs + 7u) / 8u);
  const uint32_t G = gridDim.x;

  for (uint32_t k0 = 0; k0 * G < n_items; k0 += kListCap) {
    if (tid == 0) {
      L.n_light = 0;
      L.n_heavy = 0;
    }
    if (tid < kWaves) L.ahead[tid] = 0;
    __syncthreads();
    // One-token append: wave w requests the new row of the pair of the item that thread w looks at in the first round
    // while the sequence's counters are on their way (most such appends only store that row into the window).  The row
    // goes straight to LDS (this wave's row of the reduction buffer, unused at this point), 4 bytes per lane.  (A
    // one-token append has two owners per pair and at most 2^25 items.)
    int pre_p = -1;
    if (T == 1 && k0 == 0 && (uint32_t)wave * G + blockIdx.x < n_items) {
      const uint32_t it = (uint32_t)wave * G + blockIdx.x;
      const uint32_t p = (it >> 4) * 8u + (it & 7u);
      if (((it >> 3) & 1u) == 0u && p < n_pairs) {
        pre_p = (int)p;
        __builtin_amdgcn_global_load_lds(k_new + (long long)p * kHeadDim + 2 * lane, &L.red[wave][0], 4, 0, 0);
        __builtin_amdgcn_global_load_lds(v_new + (long long)p * kHeadDim + 2 * lane, &L.red[wave][64], 4, 0, 0);
      }
    }
    // every thread looks at one item: what needs a wave or the workgroup is listed, the rest is counted in at once
    const uint32_t it = (k0 + tid) * G + blockIdx.x;
    if (it < n_items) {
      const int own = (int)((it >> 3) % owners);  // (part, chunk): part = own / n_chunks, chunk = own % n_chunks
      const uint32_t p = (it / (8u * owners)) * 8u + (it & 7u);
      if (p < n_pairs) {
        const int b = (int)(p / (uint32_t)c.H_kv);
        const Counters s = read_counters(c, b, n_new, T, keep);
        if (s.plan.err || s.n == 0) {
          if (s.plan.err && own == 0) atomicOr(c.status, s.plan.err);
          bool clean;
          if (arrive(c, b, n_chunks, s.plan.err != 0, &clean)) finish(c, b, s.nq, s.n, s.plan, clean);
        } else if (s.plan.n_groups == 0) {
          if (own == 0) {
            if (T == 1 && k0 == 0 && tid < kWaves) {  // wave `tid` holds the row
              L.ahead[tid] = 1;
              L.ahead_nq[tid] = s.nq;
              L.ahead_nr[tid] = s.nr;
              L.ahead_n[tid] = s.n;
            } else {
              L.light[atomicAdd(&L.n_light, 1)] = (int)p;
            }
          } else {
            bool clean;
            if (arrive(c, b, n_chunks, false, &clean)) finish(c, b, s.nq, s.n, s.plan, clean);
          }
        } else {
          L.heavy[atomicAdd(&L.n_heavy, 1)] = (int)(p * owners) + own;
        }
      }
    }
    __syncthreads();
    const int n_light = L.n_light, n_heavy = L.n_heavy;
    if (L.ahead[wave] != 0) {  // (the barrier has waited for the row)
      Counters s;
      s.nq = L.ahead_nq[wave];
      s.nr = L.ahead_nr[wave];
      s.n = L.ahead_n[wave];
      s.plan = plan_append(s.nq, s.nr, s.n, c.R, keep, c.max_groups);
      light_item<SLIDING>(c, pre_p, k_new, v_new, n_new, T, keep, n_chunks, lane, &s,
                          __builtin_bit_cast(uint32_t, L.red[wave][lane]), __builtin_bit_cast(uint32_t, L.red[wave][64 + lane]));
    }
    for (int i = wave; i < n_light; i += kThreads / 64) light_item<SLIDING>(c, L.light[i], k_new, v_new, n_new, T, keep, n_chunks, lane);
    for (int i = 0; i < n_heavy; ++i) {
      // (the thread index is made opaque here so that none of the flush's address arithmetic is hoisted to the top of
      // the kernel, where every launch -- most of them flush nothing -- would pay for it)
      int tid_here = tid;
      asm volatile("" : "+v"(tid_here));
      flush_item<SLIDING, BITS>(c, L, L.heavy[i], k_new, v_new, n_new, T, keep, n_chunks, tid_here);
      __syncthreads();
    }
    __syncthreads();
  }
}

}  // namespace

int launch_append(const kvlinc_cache& c, const kvlinc_half* k_new, const kvlinc_half* v_new, const int32_t* n_new,
                  int T, int keep, hipStream_t stream) {
  static_assert(sizeof(Lds) <= 160 * 1024, "LDS budget of one CU");
  // per device and cheap: set on every call rather than remembered in process state
  void (*kernel)(kvlinc_cache, const half_t*, const half_t*, const int32_t*, int, int, int) =
      c.bits == 4 ? ((c.flags & KVLINC_FLAG_SLIDING_VALUES) != 0 ? append_flush_kernel<true, 4> : append_flush_kernel<false, 4>)
                  : ((c.flags & KVLINC_FLAG_SLIDING_VALUES) != 0 ? append_flush_kernel<true, 2> : append_flush_kernel<false, 2>);
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)sizeof(Lds)) != hipSuccess)
    return KVLINC_EHIP;
  // A bulk append of few sequences and many groups (a long prompt) would leave most of the chip idle with two
  // workgroups per (sequence, kv head): from 64 groups on, its groups are shared out in chunks of at least 16, about one
  // owner per compute unit.  The chunks add their shares of S and P to the fp32 state with atomic additions -- S and P
  // are then reproducible up to the rounding order only -- so this needs a cache that keeps the fp32 state (or has no
  // correction at all).
  const long long pairs = (long long)c.B * c.H_kv;
  int n_chunks = 1;
  if (T > 1 && pairs * kParts < 128 && (c.S != nullptr || c.S16 == nullptr)) {
    const long long groups_most = ((long long)T + c.R + kGroup - 1) / kGroup;
    long long want = 256 / (pairs * kParts);
    if (want > groups_most / 16) want = groups_most / 16;
    if (want > 64) want = 64;
    if (groups_most >= 64 && want > 1) n_chunks = (int)want;
  }
  if (T > 1 && (c.H_kv > 1 || n_chunks > 1 || (c.flags & KVLINC_FLAG_SLIDING_VALUES) != 0))
    hipLaunchKernelGGL(append_scan_kernel, dim3(c.B * c.H_kv, (T + kScanRows - 1) / kScanRows), dim3(kThreads), 0, stream, c,
                       reinterpret_cast<const half_t*>(k_new), reinterpret_cast<const half_t*>(v_new), n_new, T);
  // one workgroup per compute unit at most (the LDS tiles of a flush fill most of one); items beyond that are taken
  // in further rounds by the same workgroups
  const long long n_items = (long long)kParts * n_chunks * 8 * ((pairs + 7) / 8);
  const int grid = (int)(n_items < 256 ? n_items : 256);
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(kThreads), sizeof(Lds), stream, c,
                     reinterpret_cast<const half_t*>(k_new), reinterpret_cast<const half_t*>(v_new), n_new, T, keep, n_chunks);
  if (hipGetLastError() != hipSuccess) return KVLINC_EHIP;
  return KVLINC_OK;
}

}  // namespace kvlinc
