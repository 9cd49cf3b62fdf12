// Measurement aid, not part of the C ABI of libkvlinc: a kernel that only READS the bytes one decode step reads
// (Sec. 3.3, Alg. 1: the packed groups, their scales and zero-points; plus the fp16 window, the 16-bit state, P and
// W_q of this build) and keeps one word per thread, so that the benchmark can put the decode kernel's time next to what
// the memory system delivers for the same bytes in one launch of the same size.  Built into libkvlinc_probe.so.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace {

constexpr int kThreads = 256;
constexpr int kSegments = 8;
constexpr int kUnroll = 4;  // 16-byte loads in flight per thread
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

struct Segments {
  const uint4* ptr[kSegments];   // 16-byte aligned device pointers
  long long n16[kSegments];      // length in 16-byte units
  long long stride16[kSegments]; // for the group records: one run of n16 units every stride16 units, `runs` times
  long long runs[kSegments];
};

// The segments are cut into chunks of kChunk16 16-byte units that never straddle two runs; the workgroups take the
// chunks of every segment in turn.  Inside a chunk consecutive lanes read consecutive 16 bytes (the access shape of the
// decode kernel's record loads), kUnroll rows of the workgroup in flight.
constexpr int kChunk16 = kThreads * kUnroll * 4;  // 64 KiB
__global__ __launch_bounds__(kThreads) void read_only_kernel(Segments s, uint32_t* __restrict__ sink) {
  uint32_t acc = 0;
  for (int k = 0; k < kSegments; ++k) {
    if (s.ptr[k] == nullptr) continue;
    const unsigned per_run = (unsigned)((s.n16[k] + kChunk16 - 1) / kChunk16);
    const unsigned chunks = per_run * (unsigned)s.runs[k];
    for (unsigned q = blockIdx.x; q < chunks; q += gridDim.x) {
      const unsigned run = q / per_run, first = (q % per_run) * kChunk16;
      const uint4* base = s.ptr[k] + (long long)run * s.stride16[k] + first;
      const long long left = s.n16[k] - first;  // units of this run from `first` on
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          const int i = (it * kUnroll + u) * kThreads + threadIdx.x;
          v[u] = make_uint4(0, 0, 0, 0);
          if (i < left) {  // read once: non-temporal, as the decode kernel reads its records
            const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(base + i));
            v[u] = make_uint4(t[0], t[1], t[2], t[3]);
          }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
      }
    }
  }
  sink[(long long)blockIdx.x * kThreads + threadIdx.x] = acc;
}

}  // namespace

// ptr / bytes / stride_bytes / runs: n_segments (<= 8) segments, each `runs` runs of `bytes` bytes (a multiple of 16)
// spaced stride_bytes apart, all device memory, 16-byte aligned.  sink: device buffer of n_workgroups * 256 words.
// start / stop: hipEvent_t attached to the dispatch (both or neither).  Returns 0, or -1 on a bad argument / launch.
extern "C" int kvlinc_probe_read_only(const void* const* ptr, const long long* bytes, const long long* stride_bytes,
                                      const long long* runs, int n_segments, void* sink, int n_workgroups, void* stream,
                                      void* start, void* stop) {
  if (n_segments < 1 || n_segments > kSegments || sink == nullptr || n_workgroups < 1) return -1;
  if ((start == nullptr) != (stop == nullptr)) return -1;
  Segments s{};
  for (int k = 0; k < n_segments; ++k) {
    if (ptr[k] == nullptr || (reinterpret_cast<uintptr_t>(ptr[k]) & 15) || bytes[k] <= 0 || (bytes[k] & 15) ||
        (stride_bytes[k] & 15) || runs[k] < 1 || runs[k] > (1 << 20) || bytes[k] > (1ll << 40) ||
        (runs[k] > 1 && stride_bytes[k] < bytes[k]))
      return -1;
    s.ptr[k] = static_cast<const uint4*>(ptr[k]);
    s.n16[k] = bytes[k] / 16;
    s.stride16[k] = stride_bytes[k] / 16;
    s.runs[k] = runs[k];
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (start != nullptr)
    hipExtLaunchKernelGGL(read_only_kernel, dim3(n_workgroups), dim3(kThreads), 0, st, static_cast<hipEvent_t>(start),
                          static_cast<hipEvent_t>(stop), 0, s, static_cast<uint32_t*>(sink));
  else
    hipLaunchKernelGGL(read_only_kernel, dim3(n_workgroups), dim3(kThreads), 0, st, s, static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? 0 : -1;
}
