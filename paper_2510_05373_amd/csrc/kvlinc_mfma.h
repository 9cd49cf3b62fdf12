// Device helpers shared by the kernels of libkvlinc: binary16 vector types, lane-quad data movement and the 4x4x4
// matrix-core instruction with a broadcast A operand (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvlinc {
namespace {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));


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

// reductions over the 64 lanes of a wave, result in every lane: rotations inside the rows of 16 lanes, then two
// cross-row exchanges
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

// D = A B + C on the sixteen 4x4 blocks of a wave, k = 4, binary16 operands, binary32 accumulate.  Lane 4 b + i holds
// row i of A_b (4 halves), column i of B_b (4 halves) and column i of D_b (4 floats).  Here every block uses the A
// of block `abid` (broadcast), so one register pair can carry the A operands of 16 successive steps.
__device__ __forceinline__ float4_t mfma_bcast(half4_t a, half4_t b, float4_t c, int abid) {
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


// 4x4 transpose of binary16 elements inside each lane quad: lane t of a quad brings {v[t][0], v[t][1]} in X and
// {v[t][2], v[t][3]} in Y; lane h leaves with {v[0][h], v[1][h], v[2][h], v[3][h]}.
// perm_sel = (lane & 1) ? 0x03020706 : 0x05040100.
__device__ __forceinline__ half4_t quad_transpose(uint32_t X, uint32_t Y, uint32_t perm_sel, int lane) {
  const uint32_t TX = dpp_u<kQuadSwap1>(X), TY = dpp_u<kQuadSwap1>(Y);
  const uint32_t X1 = __builtin_amdgcn_perm(TX, X, perm_sel);  // even lane {X.lo, TX.lo}; odd lane {TX.hi, X.hi}
  const uint32_t Y1 = __builtin_amdgcn_perm(TY, Y, perm_sel);
  const uint32_t X2 = dpp_u<kQuadSwap2>(X1), Y2 = dpp_u<kQuadSwap2>(Y1);
  const bool upper = (lane & 2) != 0;
  return as_h4(upper ? Y2 : X1, upper ? Y1 : X2);
}

}  // namespace
}  // namespace kvlinc
