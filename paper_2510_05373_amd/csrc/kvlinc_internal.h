// Internal declarations shared by the translation units of libkvlinc (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvlinc.h"

namespace kvlinc {

constexpr int kHeadDim = 128;   // d
constexpr int kGroup = 128;     // G: tokens per key group = channels per value group
constexpr int kRank = 256;      // D
// Group record of a cache with BITS-bit codes (words): key tile, value tile, key scale, key zero-point, value
// (scale, zero-point) per token; a tile holds 128 x 128 codes.  kCentre: the middle of the code range, (2^BITS - 1) / 2 --
// the tiles hold the codes as the numbers code - kCentre.
template <int BITS>
struct Rec {
  static_assert(BITS == 2 || BITS == 4, "code widths of the record layout");
  static constexpr int kTile = kGroup * kHeadDim * BITS / 32;
  static constexpr int kKeyTile = 0, kValueTile = kTile, kKeyScale = 2 * kTile, kKeyZero = 2 * kTile + 64,
                       kValueSZ = 2 * kTile + 128, kWords = 2 * kTile + 256;
  static constexpr int kLevels = (1 << BITS) - 1;
  static constexpr float kCentre = 0.5f * kLevels;
};
constexpr int kMaxGq = 8;       // query heads per KV head supported by the decode kernels

// Partial result of one block of tokens for one query head (Alg. 1: m^j, l^j, Y_s^j), log2 domain:
// {m, l, unused, unused, acc[128]}; m = -inf marks an empty block whose other fields are undefined.
constexpr int kPartStride = 132;

// What one append does to one sequence (same arithmetic in the flush kernel and in the counter commit).
struct AppendPlan {
  int n_flush;   // tokens leaving the window / new-token stream into quantized groups
  int n_groups;  // groups written (the last one partial iff n_flush % 128 != 0)
  int new_res;   // window tokens after the append
  int err;       // KVLINC_ST_* bit, 0 = fine; on error the sequence is left unchanged
};

__host__ __device__ inline AppendPlan plan_append(int n_quant, int n_res, int n_new, int R, int keep,
                                                  long long max_groups) {
  AppendPlan p{0, 0, n_res, 0};
  if (n_new <= 0) return p;
  if (n_quant % kGroup != 0) { p.err = KVLINC_ST_STATIC; return p; }
  const int total = n_res + n_new;
  int new_res;
  if (keep == 0) new_res = total <= R ? total : (total - 1) % kGroup + 1;  // lazy block flush (R == G)
  else new_res = keep < total ? keep : total;
  const int n_flush = total - new_res;
  if (n_flush > 0 && n_flush < n_res) { p.err = KVLINC_ST_STATIC; return p; }  // would have to shift the window
  const int n_groups = (n_flush + kGroup - 1) / kGroup;
  if ((long long)(n_quant / kGroup) + n_groups > max_groups) { p.err = KVLINC_ST_CAPACITY; return p; }
  p.n_flush = n_flush;
  p.n_groups = n_groups;
  p.new_res = new_res;
  return p;
}

// Splits of the decode launch (blocks of groups per (sequence, KV head)): the average over the batch, which a batch
// of equal lengths uses for every sequence, and the most one sequence may take; grid and workspace are sized for
// `most`.  corr_first: 0 = the correction workgroups come after the streaming ones in the grid, L >= 1 = they lead
// each of the first L runs of 256 workgroups.
struct DecodeSplits { int avg, most, corr_first; };
DecodeSplits decode_splits(const kvlinc_cache& c, int max_context);

int launch_append(const kvlinc_cache& c, const kvlinc_half* k_new, const kvlinc_half* v_new, const int32_t* n_new,
                  int T, int keep, hipStream_t stream);
size_t decode_workspace_floats(const kvlinc_cache& c, int n_splits);
// start / stop: optional events attached to the kernel's own dispatch (both or neither)
int launch_decode(const kvlinc_cache& c, const kvlinc_half* q, kvlinc_half* out, float* workspace, DecodeSplits splits,
                  hipStream_t stream, hipEvent_t start = nullptr, hipEvent_t stop = nullptr);

}  // namespace kvlinc
