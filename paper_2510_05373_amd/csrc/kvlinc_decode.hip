// Decode path: single-query attention read directly from the packed 2-bit cache, split over blocks of groups,
// merged, corrected and rotated back (Sec. 3.3, Alg. 1; Sec. 3.2, Eq. 5-6; Sec. 3.1 for the rotated value basis).
//
// Launch 1 (decode_split_kernel): one workgroup per (sequence, kv head, block of groups) plus one per
// (sequence, kv head) for the fp16 window.  All query heads of the kv head are processed together, so every
// packed tile is read once.  Scores live in the log2 domain: x = q.k * log2(e)/sqrt(d).  Each workgroup writes
// (m, l, acc[128]) per query head (Alg. 1: m^j, l^j, Y_s^j).
// Launch 2 (decode_merge_kernel): one workgroup per (sequence, kv head): weighs the partial results by
// 2^(m_j - M), computes phi_q(q), C_n = phi_q S, C_d = phi_q P, forms (num + 2^-M C_n) / (den + 2^-M C_d), applies
// H^T and stores fp16.
#include <hip/hip_runtime.h>

#include "kvlinc_internal.h"

namespace kvlinc {
namespace {

typedef _Float16 half_t;

constexpr int kThreads = 128;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kAlpha = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Reductions over the 128 threads (2 waves) of a workgroup for N values at once; `red` is [N][2] floats of LDS.
template <int N, bool IS_MAX>
__device__ inline void block_reduce(float (&v)[N], float* red, int tid) {
#pragma unroll
  for (int h = 0; h < N; ++h) {
    const float r = IS_MAX ? wave_max(v[h]) : wave_sum(v[h]);
    if ((tid & 63) == 0) red[h * 2 + (tid >> 6)] = r;
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < N; ++h) v[h] = IS_MAX ? fmaxf(red[h * 2], red[h * 2 + 1]) : red[h * 2] + red[h * 2 + 1];
  __syncthreads();
}

template <int GQ>
__global__ __launch_bounds__(kThreads) void decode_split_kernel(kvlinc_cache c, const half_t* __restrict__ q,
                                                                 float* __restrict__ part, int n_splits) {
  __shared__ float sQ[GQ][kHeadDim];    // alpha * q
  __shared__ float sQs[GQ][kHeadDim];   // alpha * q * key scale of the current group
  __shared__ float sP[GQ][kGroup];      // 2^(x - m) of the current group
  __shared__ float sVs[kGroup], sVz[kGroup];
  __shared__ float sRed[GQ * 2];

  const int tid = threadIdx.x;
  const int items_per_bh = n_splits + 1;
  const int bh = blockIdx.x / items_per_bh;
  const int sp = blockIdx.x % items_per_bh;
  const int b = bh / c.H_kv;
  const int g = bh % c.H_kv;
  const int nq = c.n_quant[b];
  const int nr = c.n_res[b];

#pragma unroll
  for (int h = 0; h < GQ; ++h)
    sQ[h][tid] = kAlpha * (float)q[((long long)b * c.H_q + g * GQ + h) * kHeadDim + tid];
  __syncthreads();

  float m[GQ], l_loc[GQ], acc[GQ];
#pragma unroll
  for (int h = 0; h < GQ; ++h) { m[h] = -INFINITY; l_loc[h] = 0.0f; acc[h] = 0.0f; }

  if (sp < n_splits) {
    // ---- quantized groups [g0, g1) of this sequence ---------------------------------------------------------
    const int n_groups = (nq + kGroup - 1) / kGroup;
    const int g0 = (int)((long long)n_groups * sp / n_splits);
    const int g1 = (int)((long long)n_groups * (sp + 1) / n_splits);
    for (int grp = g0; grp < g1; ++grp) {
      const int valid = min(kGroup, nq - grp * kGroup);
      const long long gbase = (long long)bh * c.max_groups + grp;
      const float ks = (float)reinterpret_cast<const half_t*>(c.k_scale)[gbase * kGroup + tid];
      const float kz = (float)reinterpret_cast<const half_t*>(c.k_zero)[gbase * kGroup + tid];
      float bias[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        sQs[h][tid] = sQ[h][tid] * ks;
        bias[h] = sQ[h][tid] * kz;
      }
      sVs[tid] = (float)reinterpret_cast<const half_t*>(c.v_scale)[gbase * kGroup + tid];
      sVz[tid] = (float)reinterpret_cast<const half_t*>(c.v_zero)[gbase * kGroup + tid];
      block_reduce<GQ, false>(bias, sRed, tid);  // syncs: sQs, sVs, sVz visible afterwards

      // scores of token tid: x[h] = sum_c (alpha q s)[h][c] * code[tid][c] + sum_c (alpha q z)[h][c]
      float x[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) x[h] = bias[h];
      {
        const uint32_t* tile = c.k_codes + gbase * kTileWords;
        const int hf = tid >> 6, l = tid & 63;
        const uint4 w0 = *reinterpret_cast<const uint4*>(tile + ((hf * 2 + 0) * 64 + l) * 4);
        const uint4 w1 = *reinterpret_cast<const uint4*>(tile + ((hf * 2 + 1) * 64 + l) * 4);
        const uint32_t words[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
        for (int qw = 0; qw < 8; ++qw) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              const int ch = 8 * (4 * (qw % 4) + j / 2) + 4 * (qw / 4) + 2 * (j % 2) + e;
              const float code = (float)((words[qw] >> (2 * j + 16 * e)) & 3u);
#pragma unroll
              for (int h = 0; h < GQ; ++h) x[h] = fmaf(sQs[h][ch], code, x[h]);
            }
          }
        }
      }
      float bm[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        if (tid >= valid) x[h] = -INFINITY;
        bm[h] = x[h];
      }
      block_reduce<GQ, true>(bm, sRed, tid);
      float scale[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        const float mn = fmaxf(m[h], bm[h]);
        scale[h] = exp2f(m[h] - mn);  // 0 on the first group (m = -inf)
        m[h] = mn;
        const float p = exp2f(x[h] - mn);
        l_loc[h] = l_loc[h] * scale[h] + p;
        sP[h][tid] = p;
      }
      __syncthreads();
      // channel tid: acc[h] += sum_t p[h][t] * (s_v[t] * code[t][tid] + z_v[t])
      {
        const uint32_t* tile = c.v_codes + gbase * kTileWords;
        const int chh = tid >> 6, l = tid & 63;
        float a[GQ];
#pragma unroll
        for (int h = 0; h < GQ; ++h) a[h] = 0.0f;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const uint4 wv = *reinterpret_cast<const uint4*>(tile + ((hf * 2 + chh) * 64 + l) * 4);
          const uint32_t words[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
          for (int w = 0; w < 4; ++w) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
#pragma unroll
              for (int e = 0; e < 2; ++e) {
                const int t = 64 * hf + 4 * (4 * w + j / 2) + 2 * (j % 2) + e;
                const float code = (float)((words[w] >> (2 * j + 16 * e)) & 3u);
                const float vh = fmaf(sVs[t], code, sVz[t]);
#pragma unroll
                for (int h = 0; h < GQ; ++h) a[h] = fmaf(sP[h][t], vh, a[h]);
              }
            }
          }
        }
#pragma unroll
        for (int h = 0; h < GQ; ++h) acc[h] = acc[h] * scale[h] + a[h];
      }
      __syncthreads();
    }
  } else if (nr > 0) {
    // ---- the fp16 window: raw keys, rotated values ----------------------------------------------------------
    const half_t* kw = reinterpret_cast<const half_t*>(c.k_res) + (long long)bh * c.R * kHeadDim;
    const half_t* vw = reinterpret_cast<const half_t*>(c.v_res) + (long long)bh * c.R * kHeadDim;
    float x[GQ];
#pragma unroll
    for (int h = 0; h < GQ; ++h) x[h] = 0.0f;
    if (tid < nr) {
      const half_t* row = kw + (long long)tid * kHeadDim;
      for (int ch = 0; ch < kHeadDim; ch += 8) {
        const uint4 raw = *reinterpret_cast<const uint4*>(row + ch);
        const half_t* hv = reinterpret_cast<const half_t*>(&raw);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float kv = (float)hv[i];
#pragma unroll
          for (int h = 0; h < GQ; ++h) x[h] = fmaf(sQ[h][ch + i], kv, x[h]);
        }
      }
    }
    float bm[GQ];
#pragma unroll
    for (int h = 0; h < GQ; ++h) {
      if (tid >= nr) x[h] = -INFINITY;
      bm[h] = x[h];
    }
    block_reduce<GQ, true>(bm, sRed, tid);
#pragma unroll
    for (int h = 0; h < GQ; ++h) {
      m[h] = bm[h];
      const float p = exp2f(x[h] - m[h]);
      l_loc[h] = p;
      sP[h][tid] = p;
    }
    __syncthreads();
    for (int t = 0; t < nr; ++t) {
      const float vv = (float)vw[(long long)t * kHeadDim + tid];
#pragma unroll
      for (int h = 0; h < GQ; ++h) acc[h] = fmaf(sP[h][t], vv, acc[h]);
    }
  }

  block_reduce<GQ, false>(l_loc, sRed, tid);
#pragma unroll
  for (int h = 0; h < GQ; ++h) {
    float* dst = part + (((long long)b * c.H_q + g * GQ + h) * items_per_bh + sp) * kPartStride;
    if (tid == 0) { dst[0] = m[h]; dst[1] = l_loc[h]; }
    dst[4 + tid] = acc[h];
  }
}

template <int GQ>
__global__ __launch_bounds__(kThreads) void decode_merge_kernel(kvlinc_cache c, const half_t* __restrict__ q,
                                                                 const float* __restrict__ part, int n_splits,
                                                                 half_t* __restrict__ out) {
  __shared__ float sQ[GQ][kHeadDim];
  __shared__ float sPhi[GQ][kRank];
  __shared__ float sRed[GQ * 2];
  __shared__ float sY[kHeadDim];

  const int tid = threadIdx.x;
  const int bh = blockIdx.x;
  const int b = bh / c.H_kv;
  const int g = bh % c.H_kv;
  const int items_per_bh = n_splits + 1;
  const bool correct = c.S != nullptr;

  // ---- merge the blocks (Alg. 1: w = exp(m - max m)) ---------------------------------------------------------
  float M[GQ], num[GQ], den[GQ];
#pragma unroll
  for (int h = 0; h < GQ; ++h) {
    const float* p0 = part + ((long long)b * c.H_q + g * GQ + h) * items_per_bh * kPartStride;
    float mm = -INFINITY;
    for (int j = 0; j < items_per_bh; ++j) mm = fmaxf(mm, p0[(long long)j * kPartStride]);
    float n_acc = 0.0f, d_acc = 0.0f;
    for (int j = 0; j < items_per_bh; ++j) {
      const float mj = p0[(long long)j * kPartStride];
      if (mj == -INFINITY) continue;
      const float w = exp2f(mj - mm);
      n_acc = fmaf(w, p0[(long long)j * kPartStride + 4 + tid], n_acc);
      d_acc = fmaf(w, p0[(long long)j * kPartStride + 1], d_acc);
    }
    M[h] = mm; num[h] = n_acc; den[h] = d_acc;
  }

  // ---- correction: phi_q(q) = [softmax(q W_1), softmax(q W_2)], C_n = phi_q S, C_d = phi_q P (Eq. 5, Eq. 6) ----
  float Cn[GQ], Cd[GQ];
#pragma unroll
  for (int h = 0; h < GQ; ++h) { Cn[h] = 0.0f; Cd[h] = 0.0f; }
  if (correct && c.n_quant[b] > 0) {
#pragma unroll
    for (int h = 0; h < GQ; ++h) sQ[h][tid] = (float)q[((long long)b * c.H_q + g * GQ + h) * kHeadDim + tid];
    __syncthreads();
#pragma unroll
    for (int hs = 0; hs < 2; ++hs) {
      float logit[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        const half_t* W = reinterpret_cast<const half_t*>(c.Wq) +
                          ((long long)(g * GQ + h) * 2 + hs) * kHeadDim * (kRank / 2) + tid;
        float a = 0.0f;
        for (int ch = 0; ch < kHeadDim; ++ch) a = fmaf(sQ[h][ch], (float)W[ch * (kRank / 2)], a);
        logit[h] = a;
      }
      float mx[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) mx[h] = logit[h];
      block_reduce<GQ, true>(mx, sRed, tid);
      float e[GQ], s[GQ];
#pragma unroll
      for (int h = 0; h < GQ; ++h) { e[h] = __expf(logit[h] - mx[h]); s[h] = e[h]; }
      block_reduce<GQ, false>(s, sRed, tid);
#pragma unroll
      for (int h = 0; h < GQ; ++h) sPhi[h][hs * 128 + tid] = e[h] / s[h];
    }
    __syncthreads();
    const float* S = c.S + (long long)bh * kRank * kHeadDim + tid;
    const float* P = c.P + (long long)bh * kRank;
    for (int f = 0; f < kRank; ++f) {
      const float sv = S[(long long)f * kHeadDim];
      const float pv = P[f];
#pragma unroll
      for (int h = 0; h < GQ; ++h) {
        Cn[h] = fmaf(sPhi[h][f], sv, Cn[h]);
        Cd[h] = fmaf(sPhi[h][f], pv, Cd[h]);
      }
    }
  }

  // ---- (num + 2^-M C_n) / (den + 2^-M C_d), then y = y_rot H^T, per query head -----------------------------------
  for (int h = 0; h < GQ; ++h) {
    float y = 0.0f;
    if (M[h] != -INFINITY) {
      const float Ms = fmaxf(M[h], 0.0f);
      const float a = exp2f(M[h] - Ms), bf = exp2f(-Ms);
      y = (a * num[h] + bf * Cn[h]) / (a * den[h] + bf * Cd[h]);
    }
    __syncthreads();
    sY[tid] = y;
    for (int hh = 1; hh < kHeadDim; hh <<= 1) {
      __syncthreads();
      const float mine = sY[tid], other = sY[tid ^ hh];
      __syncthreads();
      sY[tid] = (tid & hh) ? (other - mine) : (mine + other);
    }
    __syncthreads();
    out[((long long)b * c.H_q + g * GQ + h) * kHeadDim + tid] = (half_t)(sY[tid] * 0.08838834764831845f);
  }
}

template <int GQ>
int launch_decode_gq(const kvlinc_cache& c, const half_t* q, half_t* out, float* ws, int n_splits,
                     hipStream_t stream) {
  const int bh = c.B * c.H_kv;
  hipLaunchKernelGGL(decode_split_kernel<GQ>, dim3(bh * (n_splits + 1)), dim3(kThreads), 0, stream, c, q, ws,
                     n_splits);
  if (hipGetLastError() != hipSuccess) return KVLINC_EHIP;
  hipLaunchKernelGGL(decode_merge_kernel<GQ>, dim3(bh), dim3(kThreads), 0, stream, c, q, ws, n_splits, out);
  if (hipGetLastError() != hipSuccess) return KVLINC_EHIP;
  return KVLINC_OK;
}

}  // namespace

int decode_splits(const kvlinc_cache& c, int max_context) {
  long long cap = (long long)c.max_groups * kGroup + c.R;
  long long ctx = (max_context > 0 && max_context < cap) ? max_context : cap;
  long long groups = (ctx + kGroup - 1) / kGroup;
  if (groups < 1) groups = 1;
  const long long bh = (long long)c.B * c.H_kv;
  long long target = (4096 + bh - 1) / bh;  // aim at ~16 workgroups per CU
  if (target < 1) target = 1;
  long long s = target < groups ? target : groups;
  if (s > 256) s = 256;
  return (int)s;
}

int launch_decode(const kvlinc_cache& c, const kvlinc_half* q, kvlinc_half* out, float* workspace, int n_splits,
                  hipStream_t stream) {
  const half_t* qq = reinterpret_cast<const half_t*>(q);
  half_t* oo = reinterpret_cast<half_t*>(out);
  switch (c.H_q / c.H_kv) {
    case 1: return launch_decode_gq<1>(c, qq, oo, workspace, n_splits, stream);
    case 2: return launch_decode_gq<2>(c, qq, oo, workspace, n_splits, stream);
    case 3: return launch_decode_gq<3>(c, qq, oo, workspace, n_splits, stream);
    case 4: return launch_decode_gq<4>(c, qq, oo, workspace, n_splits, stream);
    case 5: return launch_decode_gq<5>(c, qq, oo, workspace, n_splits, stream);
    case 6: return launch_decode_gq<6>(c, qq, oo, workspace, n_splits, stream);
    case 7: return launch_decode_gq<7>(c, qq, oo, workspace, n_splits, stream);
    case 8: return launch_decode_gq<8>(c, qq, oo, workspace, n_splits, stream);
    default: return KVLINC_EINVAL;
  }
}

}  // namespace kvlinc
