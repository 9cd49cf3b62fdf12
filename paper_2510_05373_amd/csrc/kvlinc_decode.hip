// Block-split decode over the packed 2-bit cache on the CDNA4 matrix cores (Sec. 3.3, Alg. 1 lines 4-12: unpack,
// q K^T, block max / exp / sum, E V; the dequantization is folded into the small operands instead of being applied
// to the tiles).
//
// One wave owns a group of 128 tokens at a time and keeps its own (m, l, acc); the four waves of a workgroup take
// the groups of the workgroup's range round-robin and are combined through LDS at the end (Alg. 1 line 11 writes
// one (Y_s, m, l) per workgroup and query head).
//
// Both contractions run on v_mfma_f32_4x4x4_16B_f16 with the A operand broadcast from one lane quad (cbsz=4,
// abid=quad): 16 blocks x (4 rows x 4 k) x (4 k x 4 columns).  Rows = the 4 query heads of a head block.
//   q K^T : columns = 64 tokens (lane = token), k = 4 channels; A = q * key scale, held by quad `abid` for its 8 channels.
//   E V   : columns = 64 channels (lane = channel), k = 4 tokens;  A = p * value scale, held by the quad that owns the tokens.
// The B operand is the packed word itself, masked: a 2-bit code left in place inside an fp16 mantissa is the
// subnormal code * 2^(2 pos - 24) (the matrix cores take subnormal inputs exactly), and the factor 2^(-2 pos) is
// folded into the A operand of that k slot.  One AND per two codes, one shift per sixteen.
// Zero-points never touch the tiles: sum_c q_c (s_c code + z_c) = sum_c (q_c s_c) code + sum_c q_c z_c, and likewise
// for the values per token.  The fp16 rounding of (q s) and (p s) is centred: the code is taken as (code - 1.5) and
// 1.5 * rounded operand is added back in binary32, which removes the mean of the rounding error.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "kvlinc_internal.h"

namespace kvlinc {
namespace {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kAlpha = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)
constexpr float kRawScale = 1048576.0f;                  // 2^20: A carries 2^(4 - 2 pos), B carries 2^(2 pos - 24)

// ---- small helpers ----------------------------------------------------------------------------------------------

__device__ __forceinline__ uint32_t as_u32(half2_t v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ half2_t as_h2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ half4_t as_h4(uint32_t a, uint32_t b) {
  u32x2_t v = {a, b};
  return __builtin_bit_cast(half4_t, v);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
constexpr int kQuadSwap1 = 0xB1;   // quad_perm [1,0,3,2]
constexpr int kQuadSwap2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int kRowRor4 = 0x124, kRowRor8 = 0x128, kRowRor1 = 0x121, kRowRor2 = 0x122;

__device__ __forceinline__ float wave_allmax(float v) {
  v = fmaxf(v, dpp_f<kRowRor1>(v));
  v = fmaxf(v, dpp_f<kRowRor2>(v));
  v = fmaxf(v, dpp_f<kRowRor4>(v));
  v = fmaxf(v, dpp_f<kRowRor8>(v));
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  v = fmaxf(v, __shfl_xor(v, 32, 64));
  return v;
}
__device__ __forceinline__ float wave_allsum(float v) {
  v += dpp_f<kRowRor1>(v);
  v += dpp_f<kRowRor2>(v);
  v += dpp_f<kRowRor4>(v);
  v += dpp_f<kRowRor8>(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}
// sum over the 16 lanes that share lane % 4 (one per quad)
__device__ __forceinline__ float quadlane_allsum(float v) {
  v += dpp_f<kRowRor4>(v);
  v += dpp_f<kRowRor8>(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

__device__ __forceinline__ float4_t mfma_bcast(half4_t a, half4_t b, float4_t c, int abid) {
#ifdef KV_EXP_NOMFMA
  c[abid & 3] += (float)b[abid & 3] * (float)a[0];
  return c;
#endif
  switch (abid) {
    case 0: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 0, 0);
    case 1: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 1, 0);
    case 2: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 2, 0);
    case 3: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 3, 0);
    case 4: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 4, 0);
    case 5: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 5, 0);
    case 6: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 6, 0);
    case 7: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 7, 0);
    case 8: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 8, 0);
    case 9: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 9, 0);
    case 10: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 10, 0);
    case 11: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 11, 0);
    case 12: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 12, 0);
    case 13: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 13, 0);
    case 14: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 14, 0);
    default: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, 4, 15, 0);
  }
}

// Position of pair j of a packed word inside the fp16 mantissa after the (optional) shift by 6: the code of pair j
// sits at bits [2 pos + 1 : 2 pos] of its half and reads as code * 2^(2 pos - 24).
__host__ __device__ constexpr int pair_pos(int j) { return j <= 4 ? j : j - 3; }
// The factor the A operand carries for a k slot fed by pair j: 2^(4 - 2 pos).
__device__ __forceinline__ float pair_gain(int j) { return __builtin_ldexpf(1.0f, 4 - 2 * pair_pos(j)); }

// The 8 pairs of a word as fp16x2 subnormals (9 VALU operations for 16 codes).
__device__ __forceinline__ void unpack_word(uint32_t w, uint32_t (&u)[8]) {
#ifdef KV_EXP_NOUNPACK
  for (int j = 0; j < 8; ++j) u[j] = w;
  return;
#endif
  const uint32_t ws = w >> 6;
  u[0] = w & 0x00030003u;
  u[1] = w & 0x000C000Cu;
  u[2] = w & 0x00300030u;
  u[3] = w & 0x00C000C0u;
  u[4] = w & 0x03000300u;
  u[5] = ws & 0x00300030u;
  u[6] = ws & 0x00C000C0u;
  u[7] = ws & 0x03000300u;
}

// Register image of one group, loaded in two parts so that each part can be re-issued for the next group as soon
// as its contraction has consumed it (the loads then fly during the other contraction; no second register set).
struct KeyRegs {
  uint4 kw[2][2];  // key tile: [token half][word quad]
  uint4 ks, kz;    // key scale / zero-point of channels 8*quad .. 8*quad+7
};
struct ValueRegs {
  uint4 vw[2][2];         // value tile: [token half][channel half]
  uint32_t sz[2];         // value (scale, zero-point) fp16 pair of tokens lane, 64 + lane
};

__device__ __forceinline__ void load_keys(KeyRegs& r, const kvlinc_cache& c, long long gbase, int lane) {
  const uint32_t* rec = c.groups + gbase * kRecordWords;
  const uint4* kt = reinterpret_cast<const uint4*>(rec + kRecKeyTile);
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int i = 0; i < 2; ++i) r.kw[hf][i] = kt[(hf * 2 + i) * 64 + lane];
  const int quad = lane >> 2;
  r.ks = reinterpret_cast<const uint4*>(rec + kRecKeyScale)[quad];
  r.kz = reinterpret_cast<const uint4*>(rec + kRecKeyZero)[quad];
}

__device__ __forceinline__ void load_values(ValueRegs& r, const kvlinc_cache& c, long long gbase, int lane) {
  const uint32_t* rec = c.groups + gbase * kRecordWords;
  const uint4* vt = reinterpret_cast<const uint4*>(rec + kRecValueTile);
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int i = 0; i < 2; ++i) r.vw[hf][i] = vt[(hf * 2 + i) * 64 + lane];
  r.sz[0] = rec[kRecValueSZ + lane];
  r.sz[1] = rec[kRecValueSZ + 64 + lane];
}

__device__ __forceinline__ float h2f(uint16_t bits) { return (float)__builtin_bit_cast(half_t, bits); }

// NB = head blocks of 4 query heads (1: up to 4 heads per KV head, 2: up to 8).
template <int NB>
struct WaveState {
  float m[NB][4];       // running maximum per head (wave-uniform), log2 domain
  float l[NB][4];       // per-lane partial sums of p
  float pz[NB][4];      // per-lane partial sums of the zero-point / centring terms of E V
  float4_t acc[NB][2];  // E V in raw matrix-core units: [head block][channel half], rows = heads, lane = channel
};

// Per-lane constants of a wave.
struct LaneConst {
  float inv_gain0, inv_gain1;  // 1 / gain of this quad's k-slot pairs (0,1) and (2,3) in q K^T
  float vgain;                 // gain of this lane's token as a k slot of E V
  uint32_t perm_sel;           // byte selector of the 16-bit exchange inside the 4x4 quad transpose
  int lane;
};

// q K^T of one group for all heads: scores in the log2 domain, [head block][token half], rows = heads, lane = token.
template <int NB>
__device__ __forceinline__ void qk_phase(const KeyRegs& g, int valid, const uint32_t (&Qs)[NB][4], const LaneConst& lc,
                                         float4_t (&sc)[NB][2]) {
  const uint32_t S[4] = {g.ks.x, g.ks.y, g.ks.z, g.ks.w};
  const uint32_t Z[4] = {g.kz.x, g.kz.y, g.kz.z, g.kz.w};
  const half2_t c15 = {(half_t)1.5f, (half_t)1.5f};
  const half2_t m15 = {(half_t)-1.5f, (half_t)-1.5f};
  half4_t A[NB][2];
  float4_t bias[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    uint32_t a[4];
    float t0 = 0.0f, t1 = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[i] = as_u32(as_h2(Qs[nb][i]) * as_h2(S[i]));        // fp16(q gain s), one rounding
      const half2_t mid = as_h2(S[i]) * c15 + as_h2(Z[i]);  // z + 1.5 s
      // gain * [ sum q (z + 1.5 s) ]  -  1.5 * sum rounded(q gain s): the exact compensation of the centring
      if (i & 1) {
        t1 = __builtin_amdgcn_fdot2(as_h2(Qs[nb][i]), mid, t1, false);
        t1 = __builtin_amdgcn_fdot2(as_h2(a[i]), m15, t1, false);
      } else {
        t0 = __builtin_amdgcn_fdot2(as_h2(Qs[nb][i]), mid, t0, false);
        t0 = __builtin_amdgcn_fdot2(as_h2(a[i]), m15, t0, false);
      }
    }
    A[nb][0] = as_h4(a[0], a[1]);
    A[nb][1] = as_h4(a[2], a[3]);
    float b = t0 * lc.inv_gain0 + t1 * lc.inv_gain1;
    b = quadlane_allsum(b) * (1.0f / kRawScale);  // lanes with lane % 4 == h now hold head h's term, in raw units
    bias[nb][0] = dpp_f<0x00>(b);
    bias[nb][1] = dpp_f<0x55>(b);
    bias[nb][2] = dpp_f<0xAA>(b);
    bias[nb][3] = dpp_f<0xFF>(b);
  }
#pragma unroll
  for (int hf = 0; hf < 2; ++hf) {
    float4_t acc0[NB], acc1[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) { acc0[nb] = bias[nb]; acc1[nb] = float4_t{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t words[4] = {g.kw[hf][i].x, g.kw[hf][i].y, g.kw[hf][i].z, g.kw[hf][i].w};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        uint32_t u[8];
        unpack_word(words[w], u);
#pragma unroll
        for (int mstep = 0; mstep < 4; ++mstep) {
          const half4_t bop = as_h4(u[2 * mstep], u[2 * mstep + 1]);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            if (i == 0) acc0[nb] = mfma_bcast(A[nb][0], bop, acc0[nb], 4 * w + mstep);
            else acc1[nb] = mfma_bcast(A[nb][1], bop, acc1[nb], 4 * w + mstep);
          }
        }
      }
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) sc[nb][hf] = (acc0[nb] + acc1[nb]) * (kRawScale * kAlpha);
  }
  if (valid < kGroup) {  // partial last group: tokens >= valid do not exist
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
        if (64 * hf + lc.lane >= valid) sc[nb][hf] = float4_t{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  }
}

// Running maximum (Alg. 1 line 8); the accumulated state is rescaled only when a maximum moved.
template <int NB>
__device__ __forceinline__ void update_max(const float4_t (&sc)[NB][2], WaveState<NB>& st) {
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    float mx[4];
    bool moved = false;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      mx[h] = wave_allmax(fmaxf(sc[nb][0][h], sc[nb][1][h]));
      mx[h] = fmaxf(mx[h], st.m[nb][h]);
      moved |= mx[h] != st.m[nb][h];
    }
    if (__builtin_amdgcn_readfirstlane((int)moved)) {
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const float f = exp2f(st.m[nb][h] - mx[h]);  // 0 when the old maximum is -inf
        st.l[nb][h] *= f;
        st.pz[nb][h] *= f;
        st.acc[nb][0][h] *= f;
        st.acc[nb][1][h] *= f;
        st.m[nb][h] = mx[h];
      }
    }
  }
}

// p = 2^(x - m), its sums, and E V of one group.
template <int NB>
__device__ __forceinline__ void pv_phase(const ValueRegs& g, const float4_t (&sc)[NB][2], const LaneConst& lc,
                                         WaveState<NB>& st) {
#pragma unroll
  for (int hf = 0; hf < 2; ++hf) {
    const float vs = h2f((uint16_t)(g.sz[hf] & 0xFFFFu));
    const float vmid = h2f((uint16_t)(g.sz[hf] >> 16)) + 1.5f * vs;
    const float vsg = vs * lc.vgain;       // value scale with the k-slot gain of this lane's token
    const float comp = -1.5f / lc.vgain;   // exact (power of two times 1.5)
    half4_t A2[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float p[4], ps[4];
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        p[h] = __builtin_amdgcn_exp2f(sc[nb][hf][h] - st.m[nb][h]);
        st.l[nb][h] += p[h];
        ps[h] = p[h] * vsg;
      }
      const half2_t x01 = as_h2(__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(ps[0], ps[1])));
      const half2_t x23 = as_h2(__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(ps[2], ps[3])));
      // sum_t p_t (z_t + 1.5 s_t) - 1.5 sum_t rounded(p_t s_t)
      st.pz[nb][0] = fmaf(p[0], vmid, fmaf((float)x01[0], comp, st.pz[nb][0]));
      st.pz[nb][1] = fmaf(p[1], vmid, fmaf((float)x01[1], comp, st.pz[nb][1]));
      st.pz[nb][2] = fmaf(p[2], vmid, fmaf((float)x23[0], comp, st.pz[nb][2]));
      st.pz[nb][3] = fmaf(p[3], vmid, fmaf((float)x23[1], comp, st.pz[nb][3]));
      // 4x4 transpose inside each lane quad: (lane = token, slots = heads) -> (lane = head, slots = tokens)
      const uint32_t X = as_u32(x01), Y = as_u32(x23);
      const uint32_t TX = dpp_u<kQuadSwap1>(X), TY = dpp_u<kQuadSwap1>(Y);
      const uint32_t X1 = __builtin_amdgcn_perm(TX, X, lc.perm_sel);  // even lane {X.lo, TX.lo}; odd lane {TX.hi, X.hi}
      const uint32_t Y1 = __builtin_amdgcn_perm(TY, Y, lc.perm_sel);
      const uint32_t X2 = dpp_u<kQuadSwap2>(X1), Y2 = dpp_u<kQuadSwap2>(Y1);
      const bool upper = (lc.lane & 2) != 0;
      const uint32_t U = upper ? Y2 : X1;
      const uint32_t W = upper ? Y1 : X2;
      A2[nb] = as_h4(U, W);
    }
#pragma unroll
    for (int ch = 0; ch < 2; ++ch) {
      const uint32_t words[4] = {g.vw[hf][ch].x, g.vw[hf][ch].y, g.vw[hf][ch].z, g.vw[hf][ch].w};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        uint32_t u[8];
        unpack_word(words[w], u);
#pragma unroll
        for (int mstep = 0; mstep < 4; ++mstep) {
          const half4_t bop = as_h4(u[2 * mstep], u[2 * mstep + 1]);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) st.acc[nb][ch] = mfma_bcast(A2[nb], bop, st.acc[nb][ch], 4 * w + mstep);
        }
      }
    }
  }
}

// ---- work item 1: a range of quantized groups of one (sequence, kv head) ----------------------------------------

template <int NB>
__device__ __forceinline__ void group_item(const kvlinc_cache& c, const half_t* __restrict__ q, float* __restrict__ part,
                                           int n_splits, int gq, int bh, int sp, float* lds) {
  float (*sM)[NB * 4] = reinterpret_cast<float (*)[NB * 4]>(lds);                       // [kWaves][NB*4]
  float (*sL)[NB * 4] = reinterpret_cast<float (*)[NB * 4]>(lds + kWaves * NB * 4);     // [kWaves][NB*4]
  float (*sAcc)[NB * 4][kHeadDim] = reinterpret_cast<float (*)[NB * 4][kHeadDim]>(lds + 2 * kWaves * NB * 4);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int b = bh / c.H_kv;
  const int g = bh % c.H_kv;
  const int nq = c.n_quant[b];
  const int n_groups = (nq + kGroup - 1) / kGroup;
  const int g0 = (int)((long long)n_groups * sp / n_splits);
  const int g1 = (int)((long long)n_groups * (sp + 1) / n_splits);
  const int items_per_bh = n_splits + 1;

  const int quad = lane >> 2, hrow = lane & 3;
  const int j0 = 2 * (quad & 3), j1 = j0 + 1;  // pairs feeding this quad's k slots (0,1) and (2,3)
  const float gain0 = pair_gain(j0), gain1 = pair_gain(j1);
  LaneConst lc;
  lc.inv_gain0 = 1.0f / gain0;
  lc.inv_gain1 = 1.0f / gain1;
  lc.vgain = pair_gain(2 * ((lane >> 2) & 3) + ((lane >> 1) & 1));
  lc.perm_sel = (lane & 1) ? 0x03020706u : 0x05040100u;
  lc.lane = lane;

  // q of this lane's head (row hrow of each head block), channels 8*quad .. 8*quad+7, times the k-slot gains;
  // heads beyond gq read as 0
  uint32_t Qs[NB][4];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int h = nb * 4 + hrow;
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (h < gq) raw = *reinterpret_cast<const uint4*>(q + ((long long)b * c.H_q + g * gq + h) * kHeadDim + 8 * quad);
    const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const half_t gn = (half_t)((i & 1) ? gain1 : gain0);
      const half2_t g2 = {gn, gn};
      Qs[nb][i] = as_u32(as_h2(r[i]) * g2);  // exact unless it leaves the fp16 range
    }
  }

  WaveState<NB> st;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
    for (int h = 0; h < 4; ++h) { st.m[nb][h] = -INFINITY; st.l[nb][h] = 0.f; st.pz[nb][h] = 0.f; }
    st.acc[nb][0] = float4_t{0.f, 0.f, 0.f, 0.f};
    st.acc[nb][1] = float4_t{0.f, 0.f, 0.f, 0.f};
  }

  // This wave's groups.  The key part of the next group is requested as soon as q K^T has consumed the current
  // one and flies during E V; the value part likewise flies during the next q K^T.  Past the end the current
  // (cached) group is requested again, so that no branch joins between a load and its first use.
  const long long tile0 = (long long)bh * c.max_groups;
  int grp = g0 + wave;
  if (grp < g1) {
    KeyRegs kr;
    ValueRegs vr;
    load_keys(kr, c, tile0 + grp, lane);
    load_values(vr, c, tile0 + grp, lane);
    while (true) {
      const int nxt = grp + kWaves;
      const bool more = nxt < g1;
      const long long nbase = tile0 + (more ? nxt : grp);
      float4_t sc[NB][2];
      qk_phase<NB>(kr, min(kGroup, nq - grp * kGroup), Qs, lc, sc);
      load_keys(kr, c, nbase, lane);
      update_max<NB>(sc, st);
      pv_phase<NB>(vr, sc, lc, st);
      load_values(vr, c, nbase, lane);
      if (!more) break;
      grp = nxt;
    }
  }

  // combine the four waves (Alg. 1 lines 13-14 restricted to this workgroup) and write (m, l, Y_s)
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const float l = wave_allsum(st.l[nb][h]);
      const float pz = wave_allsum(st.pz[nb][h]);
      if (lane == 0) { sM[wave][nb * 4 + h] = st.m[nb][h]; sL[wave][nb * 4 + h] = l; }
      sAcc[wave][nb * 4 + h][lane] = st.acc[nb][0][h] * kRawScale + pz;
      sAcc[wave][nb * 4 + h][64 + lane] = st.acc[nb][1][h] * kRawScale + pz;
    }
  __syncthreads();
  for (int idx = tid; idx < gq * kHeadDim; idx += kThreads) {
    const int h = idx >> 7, ch = idx & 127;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sM[w][h]);
    float a = 0.f, l = 0.f;
    if (M != -INFINITY) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float f = exp2f(sM[w][h] - M);
        a = fmaf(f, sAcc[w][h][ch], a);
        l = fmaf(f, sL[w][h], l);
      }
    }
    float* dst = part + (((long long)b * c.H_q + g * gq + h) * items_per_bh + sp) * kPartStride;
    if (ch == 0) { dst[0] = M; dst[1] = l; }
    dst[4 + ch] = a;
  }
}

// ---- work item 2: the fp16 window of one (sequence, kv head): raw keys, rotated values ---------------------------
// thread = (token or channel, head half): heads 4*hh .. 4*hh+3

__device__ __forceinline__ void window_item(const kvlinc_cache& c, const half_t* __restrict__ q, float* __restrict__ part,
                                            int n_splits, int gq, int bh, float* lds) {
  float (*sQ)[kHeadDim] = reinterpret_cast<float (*)[kHeadDim]>(lds);            // [8][128] alpha * q
  float (*sP)[kGroup] = reinterpret_cast<float (*)[kGroup]>(lds + 8 * kHeadDim);  // [8][128]
  float* sRed = lds + 16 * kHeadDim;                                             // [8][2]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int tok = tid & 127, hh = tid >> 7;
  const int b = bh / c.H_kv;
  const int g = bh % c.H_kv;
  const int nr = c.n_res[b];
  const int items_per_bh = n_splits + 1;

  for (int i = tid; i < gq * kHeadDim; i += kThreads)
    sQ[i >> 7][i & 127] = kAlpha * (float)q[((long long)b * c.H_q + g * gq) * kHeadDim + i];
  __syncthreads();

  const half_t* kw = reinterpret_cast<const half_t*>(c.k_res) + (long long)bh * c.R * kHeadDim;
  const half_t* vw = reinterpret_cast<const half_t*>(c.v_res) + (long long)bh * c.R * kHeadDim;
  float x[4] = {0.f, 0.f, 0.f, 0.f};
  if (tok < nr && 4 * hh < gq) {
    const half_t* row = kw + (long long)tok * kHeadDim;
#pragma unroll 4
    for (int ch = 0; ch < kHeadDim; ch += 8) {
      const uint4 raw = *reinterpret_cast<const uint4*>(row + ch);
      const half_t* hv = reinterpret_cast<const half_t*>(&raw);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float kv = (float)hv[i];
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = fmaf(sQ[4 * hh + j][ch + i], kv, x[j]);
      }
    }
  }
  float m[4], l[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (tok >= nr) x[j] = -INFINITY;
    const float r = wave_allmax(x[j]);
    if (lane == 0) sRed[(4 * hh + j) * 2 + (wave & 1)] = r;
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    m[j] = fmaxf(sRed[(4 * hh + j) * 2], sRed[(4 * hh + j) * 2 + 1]);
    const float p = (nr > 0) ? exp2f(x[j] - m[j]) : 0.f;
    sP[4 * hh + j][tok] = p;
    l[j] = wave_allsum(p);
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (lane == 0) sRed[(4 * hh + j) * 2 + (wave & 1)] = l[j];
  __syncthreads();
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (4 * hh < gq) {
    for (int t = 0; t < nr; ++t) {
      const float vv = (float)vw[((long long)(t >> 2) * kHeadDim + tok) * 4 + (t & 3)];
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = fmaf(sP[4 * hh + j][t], vv, acc[j]);
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int h = 4 * hh + j;
    if (h >= gq) continue;
    float* dst = part + (((long long)b * c.H_q + g * gq + h) * items_per_bh + n_splits) * kPartStride;
    if (tok == 0) { dst[0] = nr > 0 ? m[j] : -INFINITY; dst[1] = sRed[h * 2] + sRed[h * 2 + 1]; }
    dst[4 + tok] = acc[j];
  }
}

// ---- work item 3: correction terms of one (sequence, kv head): phi_q(q), C_n = phi_q S, C_d = phi_q P -------------
// (Sec. 3.3: computed before the merge; Eq. 6 for phi.)  Output per query head: {C_d, -, -, -, C_n[128]}.
// Both products are laid out so that a wave owns complete output columns (all rows of the contraction), reduces
// with shuffles and needs no cross-wave traffic; loads are issued in batches of eight 16-byte requests per lane.

__device__ __forceinline__ float xor_allsum_16rows(float v) {  // sum over lanes that differ in bits 2..5
  v += dpp_f<kRowRor4>(v);
  v += dpp_f<kRowRor8>(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}
__device__ __forceinline__ float xor_allsum_8rows(float v) {  // sum over lanes that differ in bits 3..5
  v += dpp_f<kRowRor8>(v);
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

__device__ __forceinline__ void correction_item(const kvlinc_cache& c, const half_t* __restrict__ q,
                                                float* __restrict__ corr, int gq, int bh, float* lds) {
  float (*sQ)[kHeadDim] = reinterpret_cast<float (*)[kHeadDim]>(lds);             // [8][128] raw q
  float (*sPhi)[kRank] = reinterpret_cast<float (*)[kRank]>(lds + 8 * kHeadDim);  // [8][256] logits, then phi
  float* sSmall = lds + 8 * kHeadDim + 8 * kRank;                                 // [64]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int b = bh / c.H_kv;
  const int g = bh % c.H_kv;
  float* out0 = corr + ((long long)b * c.H_q + g * gq) * kPartStride;
  if (c.n_quant[b] == 0) {  // states are empty: no correction (and S, P need not be read)
    for (int i = tid; i < gq * kPartStride; i += kThreads) out0[i] = 0.f;
    return;
  }
  for (int i = tid; i < gq * kHeadDim; i += kThreads)
    sQ[i >> 7][i & 127] = (float)q[((long long)b * c.H_q + g * gq) * kHeadDim + i];
  __syncthreads();

  // phase 1: logit[h][hs][f] = sum_c q[h][c] W[h][hs][c][f].  Wave w owns features 32w .. 32w+31 of each half;
  // lane = (chunk of 8 features, group of 8 channels).
  {
    const int chunk = lane & 3, rowgrp = lane >> 2;
    const int f0 = 32 * wave + 8 * chunk;
    const half_t* W0 = reinterpret_cast<const half_t*>(c.Wq) + (long long)g * gq * 2 * kHeadDim * (kRank / 2) +
                       (long long)rowgrp * 8 * (kRank / 2) + f0;
    // batches of eight 16-byte requests per lane, the next batch always in flight while the current one is reduced
    uint4 raw[2][8];
#pragma unroll
    for (int rb = 0; rb < 8; ++rb) raw[0][rb] = *reinterpret_cast<const uint4*>(W0 + rb * (kRank / 2));
    const int n_batches = 2 * gq;  // hb = 2 h + hs
    for (int hb0 = 0; hb0 < n_batches; hb0 += 2) {
#pragma unroll
      for (int par = 0; par < 2; ++par) {
        const int hb = hb0 + par;
        const int nb = hb + 1 < n_batches ? hb + 1 : hb;  // past the end: re-request the current, cached batch
        const half_t* Wn = W0 + (long long)nb * kHeadDim * (kRank / 2);
#pragma unroll
        for (int rb = 0; rb < 8; ++rb) raw[par ^ 1][rb] = *reinterpret_cast<const uint4*>(Wn + rb * (kRank / 2));
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
        for (int rb = 0; rb < 8; ++rb) {
          const float qv = sQ[hb >> 1][rowgrp * 8 + rb];
          const half_t* hv = reinterpret_cast<const half_t*>(&raw[par][rb]);
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[i] = fmaf(qv, (float)hv[i], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = xor_allsum_16rows(acc[i]);
        if (rowgrp == 0) {
          float* dst = &sPhi[hb >> 1][(hb & 1) * 128 + f0];
          *reinterpret_cast<float4*>(dst) = make_float4(acc[0], acc[1], acc[2], acc[3]);
          *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
        }
      }
    }
  }
  __syncthreads();
  // softmax over each half (128 features) of each head: one wave per row at a time
  for (int row = wave; row < 2 * gq; row += kWaves) {
    float* p = &sPhi[row >> 1][(row & 1) * 128];
    const float a0 = p[lane], a1 = p[lane + 64];
    const float mx = wave_allmax(fmaxf(a0, a1));
    const float e0 = __expf(a0 - mx), e1 = __expf(a1 - mx);
    const float inv = 1.0f / wave_allsum(e0 + e1);
    p[lane] = e0 * inv;
    p[lane + 64] = e1 * inv;
  }
  __syncthreads();

  // phase 2: C_n[h][c] = sum_f phi[h][f] S[f][c].  Wave w owns channels 32w .. 32w+31; lane = (chunk of 4
  // channels, group of 32 features).  S is read once for all heads.
  {
    const int chunk = lane & 7, rowgrp = lane >> 3;
    const int c0 = 32 * wave + 4 * chunk;
    const float* S = c.S + (long long)bh * kRank * kHeadDim + (long long)rowgrp * 32 * kHeadDim + c0;
    float acc[kMaxGq][4];
#pragma unroll
    for (int h = 0; h < kMaxGq; ++h)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[h][j] = 0.f;
    float4 s4[2][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) s4[0][i] = *reinterpret_cast<const float4*>(S + (long long)i * kHeadDim);
#pragma unroll
    for (int bt = 0; bt < 4; ++bt) {
      const int i0 = 8 * bt;
      if (bt < 3) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          s4[(bt & 1) ^ 1][i] = *reinterpret_cast<const float4*>(S + (long long)(i0 + 8 + i) * kHeadDim);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float4 sv = s4[bt & 1][i];
#pragma unroll
        for (int h = 0; h < kMaxGq; ++h) {
          if (h < gq) {
            const float ph = sPhi[h][rowgrp * 32 + i0 + i];
            acc[h][0] = fmaf(ph, sv.x, acc[h][0]);
            acc[h][1] = fmaf(ph, sv.y, acc[h][1]);
            acc[h][2] = fmaf(ph, sv.z, acc[h][2]);
            acc[h][3] = fmaf(ph, sv.w, acc[h][3]);
          }
        }
      }
    }
#pragma unroll
    for (int h = 0; h < kMaxGq; ++h) {
      if (h < gq) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[h][j] = xor_allsum_8rows(acc[h][j]);
        if (rowgrp == 0)
          *reinterpret_cast<float4*>(out0 + (long long)h * kPartStride + 4 + c0) =
              make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
      }
    }
    // C_d[h] = sum_f phi[h][f] P[f]
    const float pf = c.P[(long long)bh * kRank + tid];
    for (int h = 0; h < gq; ++h) {
      const float v = wave_allsum(sPhi[h][tid] * pf);
      if (lane == 0) sSmall[h * kWaves + wave] = v;
    }
    __syncthreads();
    if (tid < gq) {
      float cd = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) cd += sSmall[tid * kWaves + w];
      out0[(long long)tid * kPartStride] = cd;
    }
  }
}

constexpr int kLdsFloats = 2 * kWaves * 8 + kWaves * 8 * kHeadDim;  // the group item with two head blocks (largest)

// blockIdx: [0, BH) correction items (only with adapters), then BH window items, then BH * n_splits group items.
template <int NB>
__global__ __launch_bounds__(kThreads, NB == 1 ? 4 : 3) void decode_main_kernel(kvlinc_cache c, const half_t* __restrict__ q,
                                                                float* __restrict__ part, float* __restrict__ corr,
                                                                int n_splits, int gq, int dbg_skip) {
  __shared__ __align__(16) float lds[kLdsFloats];
  static_assert(kLdsFloats >= 2 * kWaves * NB * 4 + kWaves * NB * 4 * kHeadDim, "group item LDS");
  static_assert(kLdsFloats >= 8 * kHeadDim + 8 * kRank + 64, "correction item LDS");
  static_assert(kLdsFloats >= 16 * kHeadDim + 16, "window item LDS");
  const int BH = c.B * c.H_kv;
  int item = blockIdx.x;
  if (corr != nullptr) {
    if (item < BH) { if (!(dbg_skip & 1)) correction_item(c, q, corr, gq, item, lds); return; }
    item -= BH;
  }
  if (item < BH) { if (!(dbg_skip & 2)) window_item(c, q, part, n_splits, gq, item, lds); return; }
  item -= BH;
  if (dbg_skip & 4) return;
  group_item<NB>(c, q, part, n_splits, gq, item / n_splits, item % n_splits, lds);
}

// ---- launch 2: merge the blocks, add the correction, rotate back (Alg. 1 lines 13-15; Eq. 5; Sec. 3.1) ---------------
// one wave per (sequence, query head); lane l owns channels 2l and 2l+1

__global__ __launch_bounds__(kThreads) void decode_merge_kernel(kvlinc_cache c, const float* __restrict__ part,
                                                                 const float* __restrict__ corr, int n_splits,
                                                                 half_t* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * kWaves + (threadIdx.x >> 6);  // b * H_q + h
  if (row >= c.B * c.H_q) return;
  const int items = n_splits + 1;
  const float* p0 = part + (long long)row * items * kPartStride;
  float M = -INFINITY;
  for (int j = lane; j < items; j += 64) M = fmaxf(M, p0[(long long)j * kPartStride]);
  M = wave_allmax(M);
  float n0 = 0.f, n1 = 0.f, den = 0.f;
  for (int j = 0; j < items; ++j) {
    const float mj = p0[(long long)j * kPartStride];
    if (mj == -INFINITY) continue;
    const float w = exp2f(mj - M);
    const float2 a = *reinterpret_cast<const float2*>(p0 + (long long)j * kPartStride + 4 + 2 * lane);
    n0 = fmaf(w, a.x, n0);
    n1 = fmaf(w, a.y, n1);
    den = fmaf(w, p0[(long long)j * kPartStride + 1], den);
  }
  float y0 = 0.f, y1 = 0.f;
  if (M != -INFINITY) {
    float cn0 = 0.f, cn1 = 0.f, cd = 0.f;
    if (corr != nullptr) {
      const float* cr = corr + (long long)row * kPartStride;
      const float2 cn = *reinterpret_cast<const float2*>(cr + 4 + 2 * lane);
      cn0 = cn.x; cn1 = cn.y; cd = cr[0];
    }
    // (num + 2^-M C_n) / (den + 2^-M C_d) with both factors kept <= 1 (M is the log2-domain maximum)
    const float Ms = fmaxf(M, 0.f);
    const float fa = exp2f(M - Ms), fb = exp2f(-Ms);
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

}  // namespace

// Blocks of groups per (sequence, kv head): every wave of a workgroup should own about kGroupsPerWave groups.
int decode_splits(const kvlinc_cache& c, int max_context) {
  constexpr int kGroupsPerWave = 4;
  const long long cap = (long long)c.max_groups * kGroup + c.R;
  const long long ctx = (max_context > 0 && max_context < cap) ? max_context : cap;
  long long groups = (ctx + kGroup - 1) / kGroup;
  if (groups < 1) groups = 1;
  long long s = (groups + kWaves * kGroupsPerWave - 1) / (kWaves * kGroupsPerWave);
  if (const char* e = getenv("KVLINC_SPLITS")) s = atoi(e);
  if (s < 1) s = 1;
  if (s > 1024) s = 1024;
  return (int)s;
}

size_t decode_workspace_floats(const kvlinc_cache& c, int n_splits) {
  return (size_t)c.B * c.H_q * (n_splits + 2) * kPartStride;  // n_splits + window partials, then one correction row
}

int launch_decode(const kvlinc_cache& c, const kvlinc_half* q, kvlinc_half* out, float* workspace, int n_splits,
                  hipStream_t stream) {
  const int gq = c.H_q / c.H_kv;
  const int BH = c.B * c.H_kv;
  const half_t* qq = reinterpret_cast<const half_t*>(q);
  float* part = workspace;
  float* corr = c.S != nullptr ? workspace + (size_t)c.B * c.H_q * (n_splits + 1) * kPartStride : nullptr;
  const dim3 grid(BH * (n_splits + 1 + (corr != nullptr ? 1 : 0))), block(kThreads);
  const char* dbg = getenv("KVLINC_DBG_SKIP");
  const int dbg_skip = dbg ? atoi(dbg) : 0;
  if (gq <= 4) hipLaunchKernelGGL(decode_main_kernel<1>, grid, block, 0, stream, c, qq, part, corr, n_splits, gq, dbg_skip);
  else hipLaunchKernelGGL(decode_main_kernel<2>, grid, block, 0, stream, c, qq, part, corr, n_splits, gq, dbg_skip);
  if (hipGetLastError() != hipSuccess) return KVLINC_EHIP;
  hipLaunchKernelGGL(decode_merge_kernel, dim3((c.B * c.H_q + kWaves - 1) / kWaves), block, 0, stream, c, part, corr,
                     n_splits, reinterpret_cast<half_t*>(out));
  return hipGetLastError() == hipSuccess ? KVLINC_OK : KVLINC_EHIP;
}

}  // namespace kvlinc
