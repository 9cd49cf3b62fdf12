// Append / flush path: Hadamard rotation of new values, 2-bit quantization of what leaves the fp16 window,
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

constexpr int kThreads = 256;
constexpr int kRowPad = 130;   // halfs per LDS row of a 128-wide fp16 tile (odd number of 32-bit words)
constexpr int kCodePad = 132;  // bytes per LDS row of a 128-wide code tile
constexpr int kChunk = 16;     // tokens per state-update chunk

struct Lds {
  half_t sK[kGroup][kRowPad];
  half_t sV[kGroup][kRowPad];
  uint8_t cK[kGroup][kCodePad];
  uint8_t cV[kGroup][kCodePad];
  float kScale[kGroup], kZero[kGroup], vScale[kGroup], vZero[kGroup];
  float phi[kChunk][kRank];
  // operands of the state update of one chunk of tokens, as binary16 (the key error in two terms hi + lo)
  half_t kErrH[kChunk][kHeadDim + 8];
  half_t kErrL[kChunk][kHeadDim + 8];
  half_t cVh[kChunk][kHeadDim + 8];
  // phi s of the chunk, transposed (feature-major) and in two binary16 terms: the A operands of the S update
  half_t phTH[kRank][kChunk + 4];
  half_t phTL[kRank][kChunk + 4];
  float zs[kRank];
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

// Eq. 1 at 2 bits against the stored fp16 scale / zero-point, decided in binary32 without a division.
struct Q2 {
  float z;  // value of the stored fp16 zero-point
  float s;  // value of the stored fp16 scale
  half_t z16, s16;
};

__device__ inline Q2 q2_params(float mn, float mx) {
  mn = (mn == 0.0f) ? 0.0f : mn;  // a zero of either sign counts as +0
  mx = (mx == 0.0f) ? 0.0f : mx;
  Q2 r;
  r.z16 = (half_t)mn;  // exact: mn is an fp16 value
  r.z = mn;
  const float d32 = mx - mn;
  const float q32 = d32 / 3.0f;  // IEEE-correct binary32 division
  r.s16 = (half_t)q32;
  r.s = (float)r.s16;
  return r;
}

__device__ inline uint32_t q2_code(float x, const Q2& p) {
  const float t = x - p.z;
  const uint32_t c = (uint32_t)(t > 0.5f * p.s) + (uint32_t)(t >= 1.5f * p.s) + (uint32_t)(t > 2.5f * p.s);
  return p.s == 0.0f ? 0u : c;
}

// The counters of a sequence change only after every workgroup of that sequence (one per kv head) has read them:
// each workgroup counts itself in when it is done -- with a vote in the upper half of the counter if it found a
// fault -- and the one that completes the count writes n_quant / n_res unless somebody voted against, and leaves the
// counter (and the sequence's fault flag of the scan launch, see below) at zero.  The counter is the sequence's first
// split_done entry, which the decode kernel uses in the same way and also leaves at zero.
constexpr int kFaultVote = 1 << 16;
__device__ __forceinline__ void commit_sequence(const kvlinc_cache& c, int b, int nq, int n, const AppendPlan& plan, int err) {
  __syncthreads();
  if (threadIdx.x == 0) {
    int* counter = c.split_done + (long long)b * c.H_kv;
    if (err) atomicOr(c.status, err);
    const int before = __hip_atomic_fetch_add(counter, err ? 1 + kFaultVote : 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    if ((before & (kFaultVote - 1)) == c.H_kv - 1) {
      if (err == 0 && before < kFaultVote && n > 0) {
        c.n_quant[b] = nq + plan.n_flush;
        c.n_res[b] = plan.new_res;
      }
      *counter = 0;
      if (c.H_kv > 1) counter[1] = 0;
    }
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

// Scan launch of a bulk append (T > 1) to a cache with more than one kv head: every new row of every (sequence, kv
// head) is looked at once, and a fault raises the sequence's flag -- its second split_done entry -- so that ALL the
// workgroups of that sequence in the append launch that follows refuse the append, whichever head the fault is in.
// (With one kv head per sequence the append workgroup is alone and needs no flag; a one-token append looks at the
// new rows of all heads itself.)  Grid: (B H_kv, chunks of kScanRows rows).
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
  if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) atomicOr(c.split_done + (long long)b * c.H_kv + 1, 1);
}

__global__ __launch_bounds__(kThreads) void append_flush_kernel(kvlinc_cache c, const half_t* __restrict__ k_new,
                                                                 const half_t* __restrict__ v_new,
                                                                 const int32_t* __restrict__ n_new, int T, int keep) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  Lds& L = *reinterpret_cast<Lds*>(lds_raw);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int b = blockIdx.x / c.H_kv;
  const int g = blockIdx.x % c.H_kv;
  const long long bh = (long long)b * c.H_kv + g;

  const int nq = c.n_quant[b];
  const int nr = c.n_res[b];
  int n = n_new ? n_new[b] : T;
  n = n < 0 ? 0 : (n > T ? T : n);
  const AppendPlan plan = plan_append(nq, nr, n, c.R, keep, c.max_groups);
  if (plan.err || n == 0) {
    commit_sequence(c, b, nq, n, plan, plan.err);
    return;
  }
  {
    // non-finite new tokens: the verdict has to be the same in all workgroups of the sequence
    bool refuse = false;
    if (T == 1 && plan.n_flush > 0) {
      // A one-token append that flushes the window changes live state (S, P, the window's first slot) in every kv
      // head: the new row of every kv head of this sequence is looked at first, eight heads per wave and batch.  (One
      // that does not flush only fills a dead window slot: there each workgroup looks at its own row when it stores
      // it, and the counters are not advanced if any of them votes against.)
      for (int g0 = wave; g0 < c.H_kv; g0 += 4 * 8) {
        uint32_t chk_k[8], chk_v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int g2 = g0 + 4 * u;
          const long long row = ((long long)b * c.H_kv + (g2 < c.H_kv ? g2 : g)) * kHeadDim + 2 * lane;
          chk_k[u] = *reinterpret_cast<const uint32_t*>(k_new + row);
          chk_v[u] = *reinterpret_cast<const uint32_t*>(v_new + row);
        }
        // A rotated value is at most sum_i |v_i| / sqrt(128): rows whose sum of magnitudes stays below
        // 65504 sqrt(128) cannot overflow fp16 and need no rotation here (a non-finite v makes the sum non-finite).
        float mag[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          refuse |= ((chk_k[u] & 0x7C00u) == 0x7C00u) || ((chk_k[u] & 0x7C000000u) == 0x7C000000u);
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
    } else if (T > 1 && c.H_kv > 1) {
      refuse = c.split_done[(long long)b * c.H_kv + 1] != 0;  // raised by the scan launch
    } else if (T > 1) {
      // bulk append, one kv head: this workgroup is the sequence's only one.  The new rows that will stay in the
      // window (at most R) are looked at here; those that get quantized are looked at when their group is staged,
      // before anything but dead storage has been written.
      const half_t* ks = k_new + (long long)b * T * kHeadDim;
      const half_t* vs = v_new + (long long)b * T * kHeadDim;
      for (int u = max(plan.n_flush, nr) + wave; u < nr + n; u += kThreads / 64)
        refuse |= row_is_bad(ks + (long long)(u - nr) * kHeadDim, vs + (long long)(u - nr) * kHeadDim, lane);
    }
    if (__syncthreads_or(refuse)) {
      commit_sequence(c, b, nq, n, plan, KVLINC_ST_NONFINITE);
      return;
    }
  }

  const half_t* k_res = reinterpret_cast<const half_t*>(c.k_res) + bh * c.R * kHeadDim;
  const half_t* v_res = reinterpret_cast<const half_t*>(c.v_res) + bh * c.R * kHeadDim;
  const half_t* k_src = k_new + bh * (long long)T * kHeadDim;
  const half_t* v_src = v_new + bh * (long long)T * kHeadDim;
  const bool have_states = c.S16 != nullptr;
  const bool have_master = c.S != nullptr;  // fp32 master copy of S; without it the state lives in its binary16 tiles

  // Correction states of this (sequence, kv head) (Eq. 5).  The update runs on the matrix cores (4x4x4 blocks with a
  // broadcast A operand): wave w owns the features 64 w .. 64 w + 63, i.e. 16 blocks of 4 rows of S, each as two
  // accumulators (channel halves) whose lane 4 b + j holds channel 64 hh + 4 b + j.  Thread f = tid owns P[f].
  const int blk = lane >> 2, jq = lane & 3;
  const uint32_t perm_sel = (lane & 1) ? 0x03020706u : 0x05040100u;
  const int fwave = 64 * wave;
  const bool states_live = have_states && plan.n_groups > 0;
  float4_t sacc[16][2];
  half4_t wop[32];  // W_k of this wave's features as B operands: step cs = channels 4 cs .. 4 cs + 3
  float P_f = 0.0f;
  if (states_live) {
    const half_t* tiles_in = reinterpret_cast<const half_t*>(c.S16) + bh * kRank * kHeadDim;
#pragma unroll
    for (int fb = 0; fb < 16; ++fb)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        if (have_master) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            sacc[fb][hh][i] = c.S[(bh * kRank + fwave + 4 * fb + i) * kHeadDim + 64 * hh + lane];
        } else {  // tile (wave, hh, fb) holds exactly this accumulator
          const half4_t t16 = *reinterpret_cast<const half4_t*>(tiles_in + (((wave * 2 + hh) * 16 + fb) * 64 + lane) * 4);
#pragma unroll
          for (int i = 0; i < 4; ++i) sacc[fb][hh][i] = (float)t16[i];
        }
      }
    P_f = c.P[bh * kRank + tid];
    // a lane reads 4 features of one channel (natural order of W); the lane quad transposes
    const half_t* W0 = reinterpret_cast<const half_t*>(c.Wk) +
                       ((long long)g * 2 + (wave >> 1)) * kHeadDim * (kRank / 2) + (long long)jq * (kRank / 2) +
                       64 * (wave & 1) + 4 * blk;
#pragma unroll
    for (int cs = 0; cs < 32; ++cs) {
      const uint2 w = *reinterpret_cast<const uint2*>(W0 + (long long)(4 * cs) * (kRank / 2));
      wop[cs] = quad_transpose(w.x, w.y, perm_sel, lane);
    }
  }
  bool bad = false;

  for (int j = 0; j < plan.n_groups; ++j) {
    const int valid = min(kGroup, plan.n_flush - j * kGroup);
    const long long grp = (long long)(nq / kGroup) + j;
    // ---- 1. stage the group's raw keys and (raw or already rotated) values in LDS -------------------------
    for (int ch = tid; ch < kGroup * 16; ch += kThreads) {  // 16-byte chunks: 16 per token row
      const int t = ch >> 4, part = ch & 15;
      uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
      if (t < valid) {
        const int u = j * kGroup + t;  // index in the stream [window tokens, new tokens]
        if (u < nr) {
          kv = *reinterpret_cast<const uint4*>(k_res + (long long)u * kHeadDim + part * 8);
          // rotated values live 4 slots per channel: slot u, channel ch at [u/4][ch][u%4]
          half_t tmp[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) tmp[i] = v_res[((long long)(u >> 2) * kHeadDim + part * 8 + i) * 4 + (u & 3)];
          vv = *reinterpret_cast<const uint4*>(tmp);
        } else {
          kv = *reinterpret_cast<const uint4*>(k_src + (long long)(u - nr) * kHeadDim + part * 8);
          vv = *reinterpret_cast<const uint4*>(v_src + (long long)(u - nr) * kHeadDim + part * 8);
        }
      }
      uint32_t* dk = reinterpret_cast<uint32_t*>(&L.sK[t][part * 8]);
      uint32_t* dv = reinterpret_cast<uint32_t*>(&L.sV[t][part * 8]);
      dk[0] = kv.x; dk[1] = kv.y; dk[2] = kv.z; dk[3] = kv.w;
      dv[0] = vv.x; dv[1] = vv.y; dv[2] = vv.z; dv[3] = vv.w;
    }
    __syncthreads();
    // rotate the rows that came from new tokens (window rows are rotated already)
    for (int tb = wave; tb < valid; tb += 4 * (kThreads / 64)) {  // rows tb, tb + 4, tb + 8, tb + 12 together
      float x0[4], x1[4];
      bool act[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = tb + 4 * u;
        act[u] = t < valid && j * kGroup + t >= nr;
        x0[u] = act[u] ? (float)L.sV[t][2 * lane] : 0.0f;
        x1[u] = act[u] ? (float)L.sV[t][2 * lane + 1] : 0.0f;
      }
      if (!(act[0] || act[1] || act[2] || act[3])) continue;
      fwht128_wave_multi<4>(x0, x1, lane);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (act[u]) {
          const int t = tb + 4 * u;
          L.sV[t][2 * lane] = (half_t)x0[u];
          L.sV[t][2 * lane + 1] = (half_t)x1[u];
        }
      }
    }
    __syncthreads();
    // ---- 2. Eq. 1: keys per channel over the group's tokens, rotated values per token over the channels ----
    if (tid < kGroup) {
      const int ch = tid;
      float mn = INFINITY, mx = -INFINITY;
#pragma unroll 8
      for (int t = 0; t < valid; ++t) {
        const half_t h = L.sK[t][ch];
        bad |= nonfinite_bits(h);
        const float x = (float)h;
        mn = fminf(mn, x);
        mx = fmaxf(mx, x);
      }
      const Q2 p = q2_params(mn, mx);
#pragma unroll 8
      for (int t = 0; t < kGroup; ++t) L.cK[t][ch] = t < valid ? (uint8_t)q2_code((float)L.sK[t][ch], p) : 0;
      L.kScale[ch] = p.s;
      L.kZero[ch] = p.z;
      half_t* rec16 = reinterpret_cast<half_t*>(c.groups + (bh * c.max_groups + grp) * kRecordWords);
      rec16[2 * kRecKeyScale + ch] = p.s16;
      rec16[2 * kRecKeyZero + ch] = p.z16;
    } else {
      const int t = tid - kGroup;
      Q2 p;
      p.z = p.s = 0.0f;
      p.z16 = p.s16 = (half_t)0.0f;
      if (t < valid) {
        float mn = INFINITY, mx = -INFINITY;
#pragma unroll 8
        for (int ch = 0; ch < kHeadDim; ++ch) {
          const half_t h = L.sV[t][ch];
          bad |= nonfinite_bits(h);
          const float x = (float)h;
          mn = fminf(mn, x);
          mx = fmaxf(mx, x);
        }
        p = q2_params(mn, mx);
      }
#pragma unroll 8
      for (int ch = 0; ch < kHeadDim; ++ch) L.cV[t][ch] = t < valid ? (uint8_t)q2_code((float)L.sV[t][ch], p) : 0;
      L.vScale[t] = p.s;
      L.vZero[t] = p.z;
      half_t* rec16 = reinterpret_cast<half_t*>(c.groups + (bh * c.max_groups + grp) * kRecordWords);
      const int sz_word = kRecValueSZ + 8 * (t & 15) + (t >> 4);  // token 16 n + j at word 8 j + n of the field
      rec16[2 * sz_word] = p.s16;
      rec16[2 * sz_word + 1] = p.z16;
    }
    __syncthreads();
    // ---- 3. pack the two 4 KB tiles ------------------------------------------------------------------------
    {
      uint32_t* k_tile = c.groups + (bh * c.max_groups + grp) * kRecordWords + kRecKeyTile;
      uint32_t* v_tile = c.groups + (bh * c.max_groups + grp) * kRecordWords + kRecValueTile;
      for (int wi = tid; wi < kTileWords; wi += kThreads) {
        // word wi = ((n / 2) * 64 + j + 16 g) * 4 + 2 (n % 2) + w of both tiles: block n of 16 rows, row j, quarter g of the
        // contraction axis; code p of the word belongs to position k = 32 g + 16 w + 8 (p % 2) + p / 2 and is stored as the
        // bit pair (hi, lo) = (1,1), (1,0), (0,0), (0,1) for the codes 0..3, hi in bit 4 (p / 2) + 3 - p % 2, lo two below.
        // key tile: row = token 16 n + j, position k = channel k;
        // value tile: row = channel 16 n + j, position k = token 16 (k % 8) + 4 ((k / 16) % 4) + 2 (k / 64) + (k / 8) % 2.
        const int w = wi & 1, n = 2 * (wi >> 8) + ((wi >> 1) & 1), l = (wi >> 2) & 63, jr = l & 15, gq4 = l >> 4;
        const int row = 16 * n + jr, k0 = 32 * gq4 + 16 * w;
        const int tok0 = 4 * ((k0 >> 4) & 3) + 2 * (k0 >> 6);  // token of position k0 + 8 e + i is 16 i + tok0 + e
        uint32_t kw = 0, vw = 0;
#pragma unroll
        for (int pp = 0; pp < 16; ++pp) {
          const int e = pp & 1, i = pp >> 1;
          const uint32_t ck = L.cK[row][k0 + 8 * e + i], cv = L.cV[16 * i + tok0 + e][row];
          // hi = not (c / 2), lo = not (c / 2 xor c % 2)
          kw |= (((ck >> 1) ^ 1u) << (4 * i + 3 - e)) | ((((ck >> 1) ^ ck ^ 1u) & 1u) << (4 * i + 1 - e));
          vw |= (((cv >> 1) ^ 1u) << (4 * i + 3 - e)) | ((((cv >> 1) ^ cv ^ 1u) & 1u) << (4 * i + 1 - e));
        }
        k_tile[wi] = kw;
        v_tile[wi] = vw;
      }
    }
    // ---- 4. S += phi_k(K - K_q)^T V_q, P += sum phi_k(K - K_q) over the group's valid tokens (Eq. 5, Eq. 6) ----
    // With V_q[t][c] = z_t + s_t code[t][c]:  S[f][c] += sum_t (phi[t][f] s_t) code[t][c] + sum_t phi[t][f] z_t.
    // Both contractions take binary16 operands whose products are exact: the codes are small integers, W_k is
    // binary16, and the key error and phi s are split into two binary16 terms (hi + lo).
    if (states_live) {
      float Z_f = 0.0f;  // sum_t phi[t][f] z_t of this group, f = tid
      for (int t0 = 0; t0 < valid; t0 += kChunk) {
        __syncthreads();
        for (int i = tid; i < kChunk * kHeadDim; i += kThreads) {
          const int tt = i >> 7, ch = i & 127, t = t0 + tt;
          float ke = 0.0f;
          if (t < valid) ke = (float)L.sK[t][ch] - (L.kScale[ch] * (float)L.cK[t][ch] + L.kZero[ch]);
          const half_t hi = (half_t)ke;
          L.kErrH[tt][ch] = hi;
          L.kErrL[tt][ch] = (half_t)(ke - (float)hi);
          L.cVh[tt][ch] = (half_t)(float)L.cV[t][ch];
        }
        __syncthreads();
        // logits[t][f] = sum_c kErr[t][c] W[c][f]: rows = 4 tokens, block = 4 features, k = 4 channels
        {
          float4_t dH[4], dL[4];
          half4_t aH[4][2], aL[4][2];
#pragma clang loop unroll(full)
          for (int tb = 0; tb < 4; ++tb) {
            dH[tb] = float4_t{0.f, 0.f, 0.f, 0.f};
            dL[tb] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma clang loop unroll(full)
            for (int pr = 0; pr < 2; ++pr) {
              aH[tb][pr] = *reinterpret_cast<const half4_t*>(&L.kErrH[4 * tb + jq][64 * pr + 4 * blk]);
              aL[tb][pr] = *reinterpret_cast<const half4_t*>(&L.kErrL[4 * tb + jq][64 * pr + 4 * blk]);
            }
          }
#pragma clang loop unroll(full)
          for (int cs = 0; cs < 32; ++cs)
#pragma clang loop unroll(full)
            for (int tb = 0; tb < 4; ++tb) {
              dH[tb] = mfma_bcast(aH[tb][cs >> 4], wop[cs], dH[tb], cs & 15);
              dL[tb] = mfma_bcast(aL[tb][cs >> 4], wop[cs], dL[tb], cs & 15);
            }
#pragma clang loop unroll(full)
          for (int tb = 0; tb < 4; ++tb)
#pragma clang loop unroll(full)
            for (int i = 0; i < 4; ++i) L.phi[4 * tb + i][fwave + lane] = dH[tb][i] + dL[tb][i];
        }
        __syncthreads();
        // softmax over each half (128 features) of each token row: 2*kChunk rows, a wave takes two rows at a time so
        // that their cross-lane reductions overlap.  Besides phi (fp32, for P and the zero-point term) it leaves
        // phi s_t as two binary16 terms, feature-major.
        for (int row = 2 * wave; row < 2 * kChunk; row += 2 * (kThreads / 64)) {
          float a0[2], a1[2], m[2], e0[2], e1[2], sum[2];
#pragma clang loop unroll(full)
          for (int u = 0; u < 2; ++u) {
            const float* p = &L.phi[(row + u) >> 1][((row + u) & 1) * 128];
            a0[u] = p[lane];
            a1[u] = p[lane + 64];
            m[u] = fmaxf(a0[u], a1[u]);
          }
#pragma clang loop unroll(full)
          for (int u = 0; u < 2; ++u) m[u] = wave_allmax(m[u]);
#pragma clang loop unroll(full)
          for (int u = 0; u < 2; ++u) {
            e0[u] = __expf(a0[u] - m[u]);
            e1[u] = __expf(a1[u] - m[u]);
            sum[u] = e0[u] + e1[u];
          }
#pragma clang loop unroll(full)
          for (int u = 0; u < 2; ++u) sum[u] = wave_allsum(sum[u]);
#pragma clang loop unroll(full)
          for (int u = 0; u < 2; ++u) {
            const int tt = (row + u) >> 1, hs = (row + u) & 1;
            const bool live = t0 + tt < valid;
            const float inv = live ? 1.0f / sum[u] : 0.0f;
            const float sc_t = live ? L.vScale[t0 + tt] : 0.0f;
            const float p0 = e0[u] * inv, p1 = e1[u] * inv;
            L.phi[tt][hs * 128 + lane] = p0;
            L.phi[tt][hs * 128 + lane + 64] = p1;
            const float w0 = p0 * sc_t, w1 = p1 * sc_t;
            const half_t h0 = (half_t)w0, h1 = (half_t)w1;
            L.phTH[hs * 128 + lane][tt] = h0;
            L.phTH[hs * 128 + lane + 64][tt] = h1;
            L.phTL[hs * 128 + lane][tt] = (half_t)(w0 - (float)h0);
            L.phTL[hs * 128 + lane + 64][tt] = (half_t)(w1 - (float)h1);
          }
        }
        __syncthreads();
#pragma clang loop unroll(full)
        for (int tt = 0; tt < kChunk; ++tt) {
          const float ph = L.phi[tt][tid];
          P_f += ph;
          Z_f += ph * L.vZero[min(t0 + tt, kGroup - 1)];
        }
        // S[f][c] += sum_t (phi s)[t][f] code[t][c]: rows = 4 features, block = 4 channels, k = 4 tokens
        {
          half4_t bop[4][2];
#pragma clang loop unroll(full)
          for (int ts = 0; ts < 4; ++ts)
#pragma clang loop unroll(full)
            for (int hh = 0; hh < 2; ++hh) {
              half4_t v;
#pragma clang loop unroll(full)
              for (int k = 0; k < 4; ++k) v[k] = L.cVh[4 * ts + k][64 * hh + lane];
              bop[ts][hh] = v;
            }
          const int ts_mine = blk & 3;  // the A operand of token step ts is taken from block ts
#pragma clang loop unroll(full)
          for (int fb0 = 0; fb0 < 16; fb0 += 4) {
            half4_t aH[4], aL[4];
#pragma clang loop unroll(full)
            for (int u = 0; u < 4; ++u) {
              const int f = fwave + 4 * (fb0 + u) + jq;
              aH[u] = *reinterpret_cast<const half4_t*>(&L.phTH[f][4 * ts_mine]);
              aL[u] = *reinterpret_cast<const half4_t*>(&L.phTL[f][4 * ts_mine]);
            }
#pragma clang loop unroll(full)
            for (int ts = 0; ts < 4; ++ts)
#pragma clang loop unroll(full)
              for (int hh = 0; hh < 2; ++hh)
#pragma clang loop unroll(full)
                for (int u = 0; u < 4; ++u) {
                  sacc[fb0 + u][hh] = mfma_bcast(aH[u], bop[ts][hh], sacc[fb0 + u][hh], ts);
                  sacc[fb0 + u][hh] = mfma_bcast(aL[u], bop[ts][hh], sacc[fb0 + u][hh], ts);
                }
          }
        }
      }
      // the zero-point term is the same for every channel of a row
      __syncthreads();
      L.zs[tid] = Z_f;
      __syncthreads();
#pragma clang loop unroll(full)
      for (int fb = 0; fb < 16; ++fb) {
        const float4 z4 = *reinterpret_cast<const float4*>(&L.zs[fwave + 4 * fb]);
#pragma clang loop unroll(full)
        for (int hh = 0; hh < 2; ++hh) {
          sacc[fb][hh][0] += z4.x;
          sacc[fb][hh][1] += z4.y;
          sacc[fb][hh][2] += z4.z;
          sacc[fb][hh][3] += z4.w;
        }
      }
    }
    __syncthreads();
  }

  // A fault seen only now (one kv head per sequence in a bulk append: this workgroup is the sequence's only one) leaves
  // states, window and counters as they were; the records written above lie beyond n_quant and are dead storage.
  if (__syncthreads_or(bad)) {
    commit_sequence(c, b, nq, n, plan, KVLINC_ST_NONFINITE);
    return;
  }
  if (states_live) {
    // fp32 master copy (if the cache keeps one), row-major, and the binary16 tiles the decode kernel reads: tile (64-feature block = wave,
    // channel half hh, feature step fb) holds S[64 wave + 4 fb + k][64 hh + l] at [l][k] -- exactly one accumulator.
    // An entry beyond the binary16 range is stored as +-65504 and reported in the status word.
    half_t* tiles = reinterpret_cast<half_t*>(c.S16) + bh * kRank * kHeadDim;
    bool out_of_range = false;
#pragma unroll
    for (int fb = 0; fb < 16; ++fb)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        half4_t t16;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float v = sacc[fb][hh][i];
          if (have_master) c.S[(bh * kRank + fwave + 4 * fb + i) * kHeadDim + 64 * hh + lane] = v;
          out_of_range |= !(fabsf(v) <= 65504.0f);
          t16[i] = (half_t)fminf(fmaxf(v, -65504.0f), 65504.0f);
        }
        *reinterpret_cast<half4_t*>(tiles + (((wave * 2 + hh) * 16 + fb) * 64 + lane) * 4) = t16;
      }
    c.P[bh * kRank + tid] = P_f;
    if (__builtin_amdgcn_ballot_w64(out_of_range) != 0 && lane == 0) atomicOr(c.status, KVLINC_ST_STATE_RANGE);
  }

  // ---- 5. new tokens that stay in the window: raw key, rotated value ----------------------------------------
  // Stream index u >= n_flush goes to slot u - n_flush.  Old window tokens either all left (n_flush >= nr) or
  // none did (n_flush == 0, they keep their slots), so only new tokens are written here.
  half_t* k_win = reinterpret_cast<half_t*>(c.k_res) + bh * c.R * kHeadDim;
  half_t* v_win = reinterpret_cast<half_t*>(c.v_res) + bh * c.R * kHeadDim;
  const int first_new = max(plan.n_flush, nr);
  bool row_bad = false;  // only a one-token append that does not flush can still meet a non-finite row here
  for (int u = first_new + wave; u < nr + n; u += kThreads / 64) {
    const int slot = u - plan.n_flush;
    const half_t* ks = k_src + (long long)(u - nr) * kHeadDim;
    const half_t* vs = v_src + (long long)(u - nr) * kHeadDim;
    const uint32_t kk = *reinterpret_cast<const uint32_t*>(ks + 2 * lane);
    float x0 = (float)vs[2 * lane], x1 = (float)vs[2 * lane + 1];
    fwht128_wave(x0, x1, lane);
    const half_t r0 = (half_t)x0, r1 = (half_t)x1;
    const bool mine = ((kk & 0x7C00u) == 0x7C00u) || ((kk & 0x7C000000u) == 0x7C000000u) || nonfinite_bits(r0) || nonfinite_bits(r1);
    if (__builtin_amdgcn_ballot_w64(mine) != 0) {  // nothing of a faulty row reaches the window
      row_bad = true;
      continue;
    }
    *reinterpret_cast<uint32_t*>(k_win + (long long)slot * kHeadDim + 2 * lane) = kk;
    v_win[((long long)(slot >> 2) * kHeadDim + 2 * lane) * 4 + (slot & 3)] = r0;
    v_win[((long long)(slot >> 2) * kHeadDim + 2 * lane + 1) * 4 + (slot & 3)] = r1;
  }
  commit_sequence(c, b, nq, n, plan, __syncthreads_or(row_bad) ? KVLINC_ST_NONFINITE : 0);
}

}  // namespace

int launch_append(const kvlinc_cache& c, const kvlinc_half* k_new, const kvlinc_half* v_new, const int32_t* n_new,
                  int T, int keep, hipStream_t stream) {
  static_assert(sizeof(Lds) <= 160 * 1024, "LDS budget of one CU");
  // per device and cheap: set on every call rather than remembered in process state
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(append_flush_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)sizeof(Lds)) != hipSuccess)
    return KVLINC_EHIP;
  if (T > 1 && c.H_kv > 1)
    hipLaunchKernelGGL(append_scan_kernel, dim3(c.B * c.H_kv, (T + kScanRows - 1) / kScanRows), dim3(kThreads), 0, stream, c,
                       reinterpret_cast<const half_t*>(k_new), reinterpret_cast<const half_t*>(v_new), n_new, T);
  hipLaunchKernelGGL(append_flush_kernel, dim3(c.B * c.H_kv), dim3(kThreads), sizeof(Lds), stream, c,
                     reinterpret_cast<const half_t*>(k_new), reinterpret_cast<const half_t*>(v_new), n_new, T, keep);
  if (hipGetLastError() != hipSuccess) return KVLINC_EHIP;
  return KVLINC_OK;
}

}  // namespace kvlinc
