// Append / flush path: Hadamard rotation of new values, 2-bit quantization of what leaves the fp16 window,
// tile packing, and the update of the linear-correction states (Sec. 3.1, Obs. 3; Sec. 2, Eq. 1; Sec. 3.2, Eq. 5-6;
// Sec. 3.3: the cache is quantized only after attention has used the new token).
//
// This translation unit is compiled with floating-point contraction off: the rotation and the quantizer are
// bit-exact contracts (one binary32 rounding per written operation).
#include <hip/hip_runtime.h>

#include "kvlinc_internal.h"

#pragma clang fp contract(off)

namespace kvlinc {
namespace {

typedef _Float16 half_t;

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
  float vHat[kChunk][kHeadDim];
  float kErr[kChunk][kHeadDim];
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
// each workgroup counts itself in when it is done, and the one that completes the count writes n_quant / n_res (or
// the error bit) and leaves the counter at zero.  The counter is the sequence's first split_done entry, which the
// decode kernel uses in the same way and also leaves at zero.
__device__ __forceinline__ void commit_sequence(const kvlinc_cache& c, int b, int nq, int n, const AppendPlan& plan) {
  __syncthreads();
  if (threadIdx.x == 0) {
    int* counter = c.split_done + (long long)b * c.H_kv;
    const int before = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    if (before == c.H_kv - 1) {
      if (plan.err) {
        atomicOr(c.status, plan.err);
      } else if (n > 0) {
        c.n_quant[b] = nq + plan.n_flush;
        c.n_res[b] = plan.new_res;
      }
      *counter = 0;
    }
  }
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
    commit_sequence(c, b, nq, n, plan);
    return;
  }

  const half_t* k_res = reinterpret_cast<const half_t*>(c.k_res) + bh * c.R * kHeadDim;
  const half_t* v_res = reinterpret_cast<const half_t*>(c.v_res) + bh * c.R * kHeadDim;
  const half_t* k_src = k_new + bh * (long long)T * kHeadDim;
  const half_t* v_src = v_new + bh * (long long)T * kHeadDim;
  const bool have_states = c.S != nullptr;

  // correction states of this (sequence, kv head): thread f owns row f of S and entry f of P
  float S_row[kHeadDim];
  float P_f = 0.0f;
  float* S_glob = have_states ? c.S + (bh * kRank + tid) * kHeadDim : nullptr;
  if (have_states && plan.n_groups > 0) {
#pragma unroll
    for (int i = 0; i < kHeadDim; i += 4) {
      const float4 v = *reinterpret_cast<const float4*>(S_glob + i);
      S_row[i] = v.x; S_row[i + 1] = v.y; S_row[i + 2] = v.z; S_row[i + 3] = v.w;
    }
    P_f = c.P[bh * kRank + tid];
  }
  const half_t* Wk = have_states ? reinterpret_cast<const half_t*>(c.Wk) + (long long)g * 2 * kHeadDim * (kRank / 2)
                                 : nullptr;
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
    for (int t = wave; t < valid; t += kThreads / 64) {
      if (j * kGroup + t < nr) continue;
      float x0 = (float)L.sV[t][2 * lane], x1 = (float)L.sV[t][2 * lane + 1];
      fwht128_wave(x0, x1, lane);
      L.sV[t][2 * lane] = (half_t)x0;
      L.sV[t][2 * lane + 1] = (half_t)x1;
    }
    __syncthreads();
    // ---- 2. Eq. 1: keys per channel over the group's tokens, rotated values per token over the channels ----
    if (tid < kGroup) {
      const int ch = tid;
      float mn = INFINITY, mx = -INFINITY;
      for (int t = 0; t < valid; ++t) {
        const half_t h = L.sK[t][ch];
        bad |= nonfinite_bits(h);
        const float x = (float)h;
        mn = fminf(mn, x);
        mx = fmaxf(mx, x);
      }
      const Q2 p = q2_params(mn, mx);
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
        for (int ch = 0; ch < kHeadDim; ++ch) {
          const half_t h = L.sV[t][ch];
          bad |= nonfinite_bits(h);
          const float x = (float)h;
          mn = fminf(mn, x);
          mx = fmaxf(mx, x);
        }
        p = q2_params(mn, mx);
      }
      for (int ch = 0; ch < kHeadDim; ++ch) L.cV[t][ch] = t < valid ? (uint8_t)q2_code((float)L.sV[t][ch], p) : 0;
      L.vScale[t] = p.s;
      L.vZero[t] = p.z;
      half_t* rec16 = reinterpret_cast<half_t*>(c.groups + (bh * c.max_groups + grp) * kRecordWords);
      rec16[2 * (kRecValueSZ + t)] = p.s16;
      rec16[2 * (kRecValueSZ + t) + 1] = p.z16;
    }
    __syncthreads();
    // ---- 3. pack the two 4 KB tiles ------------------------------------------------------------------------
    {
      uint32_t* k_tile = c.groups + (bh * c.max_groups + grp) * kRecordWords + kRecKeyTile;
      uint32_t* v_tile = c.groups + (bh * c.max_groups + grp) * kRecordWords + kRecValueTile;
      for (int wi = tid; wi < kTileWords; wi += kThreads) {
        const int w = wi & 3, l = (wi >> 2) & 63, sel = (wi >> 8) & 1, hf = wi >> 9;
        // key tile: token 64*hf + l, word q = 4*sel + w; pair j, element e -> channel 8*(4*w + j/2) + 4*sel + 2*(j%2) + e
        // value tile: channel 64*sel + l, word w of token half hf; pair j, element e -> token 64*hf + 4*(4*w + j/2) + 2*(j%2) + e
        uint32_t kw = 0, vw = 0;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int idx = 4 * (4 * w + jj / 2) + 2 * (jj % 2) + e;  // 0..63
            const int kc = 8 * (4 * w + jj / 2) + 4 * sel + 2 * (jj % 2) + e;
            kw |= (uint32_t)L.cK[64 * hf + l][kc] << (2 * jj + 16 * e);
            vw |= (uint32_t)L.cV[64 * hf + idx][64 * sel + l] << (2 * jj + 16 * e);
          }
        }
        k_tile[wi] = kw;
        v_tile[wi] = vw;
      }
    }
    // ---- 4. S += phi_k(K - K_q)^T V_q, P += sum phi_k(K - K_q) over the group's valid tokens (Eq. 5, Eq. 6) ----
    if (have_states) {
      const int half_sel = tid >> 7, ff = tid & 127;
      const half_t* W = Wk + (long long)half_sel * kHeadDim * (kRank / 2) + ff;
      for (int t0 = 0; t0 < valid; t0 += kChunk) {
        __syncthreads();
        for (int i = tid; i < kChunk * kHeadDim; i += kThreads) {
          const int tt = i >> 7, ch = i & 127, t = t0 + tt;
          float ke = 0.0f, vh = 0.0f;
          if (t < valid) {
            ke = (float)L.sK[t][ch] - (L.kScale[ch] * (float)L.cK[t][ch] + L.kZero[ch]);
            vh = L.vScale[t] * (float)L.cV[t][ch] + L.vZero[t];
          }
          L.kErr[tt][ch] = ke;
          L.vHat[tt][ch] = vh;
        }
        __syncthreads();
        float acc[kChunk];
#pragma unroll
        for (int tt = 0; tt < kChunk; ++tt) acc[tt] = 0.0f;
        for (int ch = 0; ch < kHeadDim; ch += 4) {
          const float w0 = (float)W[(ch + 0) * (kRank / 2)], w1 = (float)W[(ch + 1) * (kRank / 2)];
          const float w2 = (float)W[(ch + 2) * (kRank / 2)], w3 = (float)W[(ch + 3) * (kRank / 2)];
#pragma unroll
          for (int tt = 0; tt < kChunk; ++tt) {
            const float4 e = *reinterpret_cast<const float4*>(&L.kErr[tt][ch]);
            acc[tt] = fmaf(e.x, w0, acc[tt]);
            acc[tt] = fmaf(e.y, w1, acc[tt]);
            acc[tt] = fmaf(e.z, w2, acc[tt]);
            acc[tt] = fmaf(e.w, w3, acc[tt]);
          }
        }
#pragma unroll
        for (int tt = 0; tt < kChunk; ++tt) L.phi[tt][tid] = acc[tt];
        __syncthreads();
        // softmax over each half (128 features) of each token row: 2*kChunk rows, one wave per row at a time
        for (int row = wave; row < 2 * kChunk; row += kThreads / 64) {
          const int tt = row >> 1, hs = row & 1;
          float* p = &L.phi[tt][hs * 128];
          const float a0 = p[lane], a1 = p[lane + 64];
          float m = fmaxf(a0, a1);
#pragma unroll
          for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
          const float e0 = __expf(a0 - m), e1 = __expf(a1 - m);
          float s = e0 + e1;
#pragma unroll
          for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
          const float inv = (t0 + tt < valid) ? 1.0f / s : 0.0f;
          p[lane] = e0 * inv;
          p[lane + 64] = e1 * inv;
        }
        __syncthreads();
#pragma unroll 1
        for (int tt = 0; tt < kChunk; ++tt) {
          const float ph = L.phi[tt][tid];
          P_f += ph;
#pragma unroll
          for (int ch = 0; ch < kHeadDim; ch += 4) {
            const float4 v = *reinterpret_cast<const float4*>(&L.vHat[tt][ch]);
            S_row[ch] = fmaf(ph, v.x, S_row[ch]);
            S_row[ch + 1] = fmaf(ph, v.y, S_row[ch + 1]);
            S_row[ch + 2] = fmaf(ph, v.z, S_row[ch + 2]);
            S_row[ch + 3] = fmaf(ph, v.w, S_row[ch + 3]);
          }
        }
      }
    }
    __syncthreads();
  }

  if (have_states && plan.n_groups > 0) {
#pragma unroll
    for (int i = 0; i < kHeadDim; i += 4)
      *reinterpret_cast<float4*>(S_glob + i) = make_float4(S_row[i], S_row[i + 1], S_row[i + 2], S_row[i + 3]);
    c.P[bh * kRank + tid] = P_f;
    // binary16 tile copy of S for the decode kernel: tile (part r, channel half hh, feature step fs) holds
    // S[64 r + 4 fs + k][64 hh + l] at [l][k]; this thread owns feature f = tid, i.e. (r, fs, k).
    half_t* tiles = reinterpret_cast<half_t*>(c.S16) + bh * kRank * kHeadDim;
    const int r = tid >> 6, fs = (tid & 63) >> 2, k = tid & 3;
#pragma unroll
    for (int ch = 0; ch < kHeadDim; ++ch)
      tiles[(((r * 2 + (ch >> 6)) * 16 + fs) * 64 + (ch & 63)) * 4 + k] = (half_t)S_row[ch];
  }
  if (bad) atomicOr(c.status, KVLINC_ST_NONFINITE);

  // ---- 5. new tokens that stay in the window: raw key, rotated value ----------------------------------------
  // Stream index u >= n_flush goes to slot u - n_flush.  Old window tokens either all left (n_flush >= nr) or
  // none did (n_flush == 0, they keep their slots), so only new tokens are written here.
  half_t* k_win = reinterpret_cast<half_t*>(c.k_res) + bh * c.R * kHeadDim;
  half_t* v_win = reinterpret_cast<half_t*>(c.v_res) + bh * c.R * kHeadDim;
  const int first_new = max(plan.n_flush, nr);
  for (int u = first_new + wave; u < nr + n; u += kThreads / 64) {
    const int slot = u - plan.n_flush;
    const half_t* ks = k_src + (long long)(u - nr) * kHeadDim;
    const half_t* vs = v_src + (long long)(u - nr) * kHeadDim;
    const uint32_t kk = *reinterpret_cast<const uint32_t*>(ks + 2 * lane);
    *reinterpret_cast<uint32_t*>(k_win + (long long)slot * kHeadDim + 2 * lane) = kk;
    float x0 = (float)vs[2 * lane], x1 = (float)vs[2 * lane + 1];
    fwht128_wave(x0, x1, lane);
    v_win[((long long)(slot >> 2) * kHeadDim + 2 * lane) * 4 + (slot & 3)] = (half_t)x0;
    v_win[((long long)(slot >> 2) * kHeadDim + 2 * lane + 1) * 4 + (slot & 3)] = (half_t)x1;
  }
  commit_sequence(c, b, nq, n, plan);
}

}  // namespace

int launch_append(const kvlinc_cache& c, const kvlinc_half* k_new, const kvlinc_half* v_new, const int32_t* n_new,
                  int T, int keep, hipStream_t stream) {
  static_assert(sizeof(Lds) <= 160 * 1024, "LDS budget of one CU");
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(append_flush_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Lds)) != hipSuccess)
      return KVLINC_EHIP;
    attr_set = true;
  }
  hipLaunchKernelGGL(append_flush_kernel, dim3(c.B * c.H_kv), dim3(kThreads), sizeof(Lds), stream, c,
                     reinterpret_cast<const half_t*>(k_new), reinterpret_cast<const half_t*>(v_new), n_new, T, keep);
  if (hipGetLastError() != hipSuccess) return KVLINC_EHIP;
  return KVLINC_OK;
}

}  // namespace kvlinc
