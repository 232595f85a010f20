// Plain streaming kernels for the benchmark's "achievable HBM rate" lines and for
// scaling the rocprof byte counters against a transfer of known size.  Not part of
// the method and not part of libdct.so: built into libdct_bench.so, which only
// bench.py loads.
//   dct_bench_probe_read: sums `bytes` (multiple of 16, 16-byte aligned) as uint32 words,
//                         writes one uint32 per workgroup into d_sink (>= 16384 bytes).
//   dct_bench_probe_copy: copies `bytes` (multiple of 16) from d_src to d_dst.
//   dct_bench_probe_rows: the memory traffic of a row kernel and nothing else: `chunks` consecutive chunks of
//                         `chunk_bytes` (1024 * {1, 2, 4, 8, 16}) are read, one wavefront per chunk with the
//                         next chunk in flight, and `out_bytes` (multiple of 16, <= chunk_bytes) are written
//                         per chunk to consecutive places of d_dst.  What a read stream with a small write
//                         stream mixed in can reach on this chip (it is well below a pure read).
// All return a dct_status.
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

// NV 16-byte vectors per lane and chunk; 16 wavefronts per workgroup, one workgroup per CU.
template <int NV>
__global__ __launch_bounds__(1024) void probe_rows_kernel(const uint4* __restrict__ src, uint64_t chunks,
                                                          uint4* __restrict__ dst, uint32_t out_vecs,
                                                          uint32_t* __restrict__ sink) {
  const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
  const uint64_t step = static_cast<uint64_t>(gridDim.x) * 16;
  uint64_t c = static_cast<uint64_t>(blockIdx.x) * 16 + wave;
  uint4 v[NV], w[NV];
  uint32_t acc = 0;
  if (c < chunks) {
#pragma unroll
    for (int j = 0; j < NV; ++j) v[j] = ld_stream(&src[c * (NV * kWave) + j * kWave + lane]);
  }
  for (; c < chunks; c += step) {
    const uint64_t nc = c + step;
    if (nc < chunks) {
#pragma unroll
      for (int j = 0; j < NV; ++j) w[j] = ld_stream(&src[nc * (NV * kWave) + j * kWave + lane]);
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    for (uint32_t q = lane; q < out_vecs; q += kWave) dst[c * out_vecs + q] = make_uint4(acc, acc, acc, acc);
#pragma unroll
    for (int j = 0; j < NV; ++j) v[j] = w[j];
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;  // keeps the loads when nothing is written
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

extern "C" int dct_bench_probe_rows(const void* d_src, uint64_t chunks, uint32_t chunk_bytes, void* d_dst,
                                    uint32_t out_bytes, void* d_sink, void* hip_stream) {
  if (!d_src || !d_dst || !d_sink || chunks == 0 || (out_bytes & 15) || out_bytes > chunk_bytes ||
      !is_aligned(d_src, 16) || !is_aligned(d_dst, 16) || !is_aligned(d_sink, 4))
    return DCT_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const dim3 grid(static_cast<uint32_t>(device_cu_count())), block(1024);
  const auto* src = static_cast<const uint4*>(d_src);
  auto* dst = static_cast<uint4*>(d_dst);
  auto* sink = static_cast<uint32_t*>(d_sink);
  const uint32_t ov = out_bytes / 16;
  switch (chunk_bytes) {
    case 1024: hipLaunchKernelGGL(probe_rows_kernel<1>, grid, block, 0, s, src, chunks, dst, ov, sink); break;
    case 2048: hipLaunchKernelGGL(probe_rows_kernel<2>, grid, block, 0, s, src, chunks, dst, ov, sink); break;
    case 4096: hipLaunchKernelGGL(probe_rows_kernel<4>, grid, block, 0, s, src, chunks, dst, ov, sink); break;
    case 8192: hipLaunchKernelGGL(probe_rows_kernel<8>, grid, block, 0, s, src, chunks, dst, ov, sink); break;
    case 16384: hipLaunchKernelGGL(probe_rows_kernel<16>, grid, block, 0, s, src, chunks, dst, ov, sink); break;
    default: return DCT_ERR_INVALID;
  }
  return hipGetLastError() == hipSuccess ? DCT_OK : DCT_ERR_HIP;
}
