// Plain streaming kernels for the benchmark's "achievable HBM rate" lines and for
// scaling the rocprof byte counters against a transfer of known size.  Not part of
// the method and not part of libdct.so: built into libdct_bench.so, which only
// bench.py loads.
//   dct_bench_probe_read: sums `bytes` (multiple of 16, 16-byte aligned) as uint32 words,
//                         writes one uint32 per workgroup into d_sink (>= 16384 bytes).
//   dct_bench_probe_copy: copies `bytes` (multiple of 16) from d_src to d_dst.
// Both return a dct_status.
#include "dct_common.hpp"

namespace dct {
namespace {

constexpr int kPrThreads = 256;
constexpr int kPrUnroll = 8;
constexpr uint32_t kPrMaxGrid = 4096;

__global__ __launch_bounds__(kPrThreads) void probe_read_kernel(const uint4* __restrict__ src, uint64_t n_vec,
                                                                uint32_t* __restrict__ sink) {
  uint32_t acc = 0;
  const uint64_t span = static_cast<uint64_t>(kPrThreads) * kPrUnroll;
  for (uint64_t base = blockIdx.x * span; base < n_vec; base += gridDim.x * span) {
    uint4 v[kPrUnroll];
#pragma unroll
    for (int u = 0; u < kPrUnroll; ++u) {
      const uint64_t i = base + static_cast<uint64_t>(u) * kPrThreads + threadIdx.x;
      v[u] = i < n_vec ? ld_stream(&src[i]) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kPrUnroll; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  acc = wave_sum_u32(acc);
  __shared__ uint32_t s[kPrThreads / kWave];
  if (lane_id() == 0) s[threadIdx.x / kWave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = s[0] + s[1] + s[2] + s[3];
}

// One 16-byte vector per thread and no loop: the fastest copy found on this chip (6.4 TB/s of reads plus
// writes for 1 GiB; the same copy as a grid-stride loop with 8 vectors per thread reaches 5.6 TB/s).
// The hardware starts workgroups in address order, which keeps the writes in flight within a narrow window.
__global__ __launch_bounds__(kPrThreads) void probe_copy_kernel(uint4* __restrict__ dst,
                                                                const uint4* __restrict__ src, uint64_t n_vec) {
  const uint64_t i = static_cast<uint64_t>(blockIdx.x) * kPrThreads + threadIdx.x;
  if (i < n_vec) dst[i] = ld_stream(&src[i]);
}

uint32_t probe_grid(uint64_t n_vec) {
  const uint64_t span = static_cast<uint64_t>(kPrThreads) * kPrUnroll;
  uint64_t g = (n_vec + span - 1) / span;
  if (g > kPrMaxGrid) g = kPrMaxGrid;
  return g ? static_cast<uint32_t>(g) : 1u;
}

}  // namespace
}  // namespace dct

using namespace dct;

extern "C" int dct_bench_probe_read(const void* d_src, size_t bytes, void* d_sink, void* hip_stream) {
  if (!d_src || !d_sink || bytes == 0 || (bytes & 15) || !is_aligned(d_src, 16) || !is_aligned(d_sink, 4))
    return DCT_ERR_INVALID;
  const uint64_t n_vec = bytes / 16;
  hipLaunchKernelGGL(probe_read_kernel, dim3(probe_grid(n_vec)), dim3(kPrThreads), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(d_src), n_vec,
                     static_cast<uint32_t*>(d_sink));
  return hipGetLastError() == hipSuccess ? DCT_OK : DCT_ERR_HIP;
}

extern "C" int dct_bench_probe_copy(void* d_dst, const void* d_src, size_t bytes, void* hip_stream) {
  if (!d_src || !d_dst || bytes == 0 || (bytes & 15) || !is_aligned(d_src, 16) || !is_aligned(d_dst, 16))
    return DCT_ERR_INVALID;
  const uint64_t n_vec = bytes / 16;
  if (n_vec > 0x7FFFFFFFull * kPrThreads) return DCT_ERR_INVALID;
  hipLaunchKernelGGL(probe_copy_kernel, dim3(static_cast<uint32_t>((n_vec + kPrThreads - 1) / kPrThreads)), dim3(kPrThreads), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<uint4*>(d_dst),
                     static_cast<const uint4*>(d_src), n_vec);
  return hipGetLastError() == hipSuccess ? DCT_OK : DCT_ERR_HIP;
}
