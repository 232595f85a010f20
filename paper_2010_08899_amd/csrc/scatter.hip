// Receiver side of DCT: decompression of what dct_threshold_compact and
// dct_rowtopk_fwd produce (Sec. 2.1 counts compressing and decompressing as
// the overhead of the method; in Algorithm 2 the next worker consumes the masked
// activations, and the parameter server sums the workers' sparse gradients).
//
//   dct_scatter, assign : dense vector = zeros with val[j] at idx[j].  One kernel
//       that writes every output element exactly once: each workgroup owns a
//       contiguous run of 16 KiB tiles, finds where its run starts in the ascending
//       index list (a 256-ary search, three rounds for a million pairs), and then
//       walks the list as it goes: a tile is assembled in LDS (zeros + the few
//       values that fall into it) and written out with full 16-byte stores.
//   dct_scatter, add    : out[idx[j]] += val[j] (fp32), one thread per pair.
//   dct_rowtopk_scatter : dense rows from the per-row lists; one wavefront
//       assembles a row in LDS and writes it with coalesced stores (rows that do not
//       fit: a workgroup zeroes the row in place, then drops the values in).
// The number of valid pairs is read on the device from the count that the
// compaction wrote, so compress -> decompress needs no host round trip.
#include <algorithm>

#include "dct_common.hpp"

namespace dct {
namespace {

constexpr int kScThreads = 256;
constexpr uint32_t kScTileBytes = 16384;
constexpr uint32_t kScMaxGrid = 2048;
// Tiles per workgroup of the assign kernel.  Many short workgroups, started by the hardware in address order,
// keep the stores in flight within a narrow window of the output, which is what writes want on this chip
// (c4: 4 tiles 187 us, 8 tiles 202 us, 16 tiles 214 us); with 2 tiles the search at the start of every
// workgroup costs more than that wins (254 us).
constexpr uint32_t kScTilesPerWg = 4;
constexpr uint32_t kRowLdsBytes = 16384;  // per wavefront in the on-chip row kernel

// Pairs to apply: the survivor count clipped to what the buffers hold; the
// "workspace error" count of a failed compaction means nothing is valid.
__device__ __forceinline__ uint32_t valid_pairs(const uint64_t* count, uint64_t capacity) {
  uint64_t m = capacity;
  if (count) {
    const uint64_t c = *count;
    m = c == DCT_COUNT_WORKSPACE_ERROR ? 0 : (c < capacity ? c : capacity);
  }
  return static_cast<uint32_t>(m);
}

// First position p in the ascending list idx[0, m) with idx[p] >= bound; called by all threads of the
// workgroup.  Invariant: every entry before lo is below the bound, every entry from hi on is not.
__device__ uint32_t lower_bound_wg(const int32_t* __restrict__ idx, uint32_t m, uint32_t bound) {
  uint32_t lo = 0, hi = m;
  while (lo < hi) {
    const uint32_t step = (hi - lo + kScThreads - 1) / kScThreads;
    const uint64_t pos = static_cast<uint64_t>(lo) + static_cast<uint64_t>(threadIdx.x) * step;
    const bool below = pos < hi && static_cast<uint32_t>(idx[pos]) < bound;  // negative indices read as huge
    const uint32_t cnt = __syncthreads_count(below);  // the probes that are below form a prefix
    if (cnt == 0) {
      hi = lo;
    } else {
      const uint64_t next = static_cast<uint64_t>(lo) + static_cast<uint64_t>(cnt) * step;
      lo = lo + (cnt - 1) * step + 1;
      if (next < hi) hi = static_cast<uint32_t>(next);
    }
  }
  return lo;
}

// out (16-byte aligned) = zeros with the pairs dropped in; n elements, tiles of TILE elements.
template <typename W>
__global__ __launch_bounds__(kScThreads) void scatter_assign_kernel(
    const int32_t* __restrict__ idx, const W* __restrict__ val, const uint64_t* __restrict__ count, uint64_t capacity,
    W* __restrict__ out, uint32_t n, uint32_t tiles_per_wg) {
  constexpr uint32_t TILE = kScTileBytes / sizeof(W);
  constexpr uint32_t VPT = kScTileBytes / 16 / kScThreads;  // 16-byte vectors per thread per tile
  constexpr uint32_t EPV = 16 / sizeof(W);
  // two tile buffers, used in turn: a buffer is written into while the barrier since its last clearing
  // is the one of the tile in between, so a tile costs one barrier
  __shared__ uint4 s_tiles[2][kScTileBytes / 16];
  __shared__ uint32_t s_batch_last;

  const uint32_t m = valid_pairs(count, capacity);
  const uint32_t n_tiles = (n + TILE - 1) / TILE;
  const uint32_t tile_lo = blockIdx.x * tiles_per_wg;
  const uint32_t tile_hi = min(tile_lo + tiles_per_wg, n_tiles);
  if (tile_lo >= tile_hi) return;
  uint64_t p = lower_bound_wg(idx, m, tile_lo * TILE);

  // The pairs are taken from the list a batch at a time, one pair per thread, and the batch after it is
  // already on its way: the tiles wait for no load (at c4's density a batch lasts a dozen tiles).
  constexpr uint32_t kNone = 0xFFFFFFFFu;  // never inside a tile: n < 2^31
  auto load_pair = [&](uint64_t first, uint32_t& pi, W& pv) {
    const uint64_t j = first + threadIdx.x;
    pi = j < m ? static_cast<uint32_t>(idx[j]) : kNone;
    pv = j < m ? val[j] : static_cast<W>(0);
  };
  uint32_t bi, ni;
  W bv, nv;
  load_pair(p, bi, bv);
  load_pair(p + kScThreads, ni, nv);
  // index of the batch's last pair (kNone when the list ends inside the batch): once a tile reaches
  // past it, the batch is used up
  if (threadIdx.x == kScThreads - 1) s_batch_last = bi;
  for (uint32_t v = 0; v < VPT; ++v) {
    s_tiles[0][v * kScThreads + threadIdx.x] = make_uint4(0, 0, 0, 0);
    s_tiles[1][v * kScThreads + threadIdx.x] = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();

  for (uint32_t tile = tile_lo; tile < tile_hi; ++tile) {
    const uint32_t t0 = tile * TILE;
    const uint32_t len = min(TILE, n - t0);
    uint4* tile4 = s_tiles[(tile - tile_lo) & 1u];
    W* s_tile = reinterpret_cast<W*>(tile4);
    for (;;) {
      const uint32_t rel = bi - t0;
      if (bi != kNone && rel < len) s_tile[rel] = bv;
      const uint32_t last = s_batch_last;
      if (last == kNone || last - t0 >= len) break;  // uniform; an index below t0 wraps to a huge value:
                                                     // ascending lists never get there, others just stop here
      // the whole batch lies at or before this tile: the prefetched one takes its place
      __syncthreads();  // everybody has read s_batch_last
      p += kScThreads;
      bi = ni;
      bv = nv;
      load_pair(p + kScThreads, ni, nv);
      if (threadIdx.x == kScThreads - 1) s_batch_last = bi;
      __syncthreads();
    }
    __syncthreads();  // the tile's values are in place
    // write the tile and clear what was read (each thread its own vectors)
    uint4* dst = reinterpret_cast<uint4*>(out + t0);
    if (len == TILE) {
#pragma unroll
      for (uint32_t v = 0; v < VPT; ++v) {
        const uint32_t q = v * kScThreads + threadIdx.x;
        dst[q] = tile4[q];
        tile4[q] = make_uint4(0, 0, 0, 0);
      }
    } else {
      for (uint32_t v = 0; v < VPT; ++v) {
        const uint32_t q = v * kScThreads + threadIdx.x;
        for (uint32_t e = 0; e < EPV; ++e) {
          const uint32_t i = q * EPV + e;
          if (i < len) out[t0 + i] = s_tile[i];
        }
        tile4[q] = make_uint4(0, 0, 0, 0);
      }
    }
  }
}

// Element-wise zero fill (outputs that are not 16-byte aligned).
template <typename W>
__global__ void zero_fill_kernel(W* __restrict__ out, uint32_t n) {
  for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n;
       i += static_cast<uint64_t>(gridDim.x) * blockDim.x)
    out[i] = 0;
}

// One thread per pair: out[idx[j]] = val[j], or out[idx[j]] += val[j] (fp32).
template <typename W, bool ADD>
__global__ void scatter_pairs_kernel(const int32_t* __restrict__ idx, const W* __restrict__ val,
                                     const uint64_t* __restrict__ count, uint64_t capacity, W* out, uint32_t n) {
  const uint32_t m = valid_pairs(count, capacity);
  for (uint64_t j = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x; j < m;
       j += static_cast<uint64_t>(gridDim.x) * blockDim.x) {
    const uint32_t i = static_cast<uint32_t>(idx[j]);
    if (i >= n) continue;
    if constexpr (ADD) {
      out[i] = __float_as_uint(__uint_as_float(out[i]) + __uint_as_float(val[j]));
    } else {
      out[i] = val[j];
    }
  }
}

// out[idx[j]] += val[j] (fp32), four pairs per thread and step, a workgroup's 256 threads taking neighbouring
// pairs (pair j0 + 256 u + thread): the four read-modify-writes are independent (a compaction's indices are
// distinct), so their loads are in flight together.
__global__ __launch_bounds__(256) void scatter_add4_kernel(const int32_t* __restrict__ idx,
                                                           const uint32_t* __restrict__ val,
                                                           const uint64_t* __restrict__ count, uint64_t capacity,
                                                           uint32_t* out, uint32_t n) {
  const uint32_t m = valid_pairs(count, capacity);
  for (uint64_t j0 = static_cast<uint64_t>(blockIdx.x) * 1024 + threadIdx.x; j0 < m;
       j0 += static_cast<uint64_t>(gridDim.x) * 1024) {
    uint32_t i[4], v[4], o[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool in = j0 + 256 * u < m;
      i[u] = in ? static_cast<uint32_t>(idx[j0 + 256 * u]) : 0xFFFFFFFFu;  // out of range: skipped below
      v[u] = in ? val[j0 + 256 * u] : 0u;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) o[u] = i[u] < n ? out[i[u]] : 0u;
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i[u] < n) out[i[u]] = __float_as_uint(__uint_as_float(o[u]) + __uint_as_float(v[u]));
  }
}

// Dense rows, one wavefront per row, the row assembled in LDS (D * sizeof(W) <= kRowLdsBytes).
template <typename W, typename I>
__global__ __launch_bounds__(kScThreads) void rowscatter_lds_kernel(
    const I* __restrict__ idx, const W* __restrict__ val, uint32_t B, uint32_t D, uint32_t k,
    W* __restrict__ out, uint64_t out_stride, bool vec_ok) {
  constexpr int kWaves = kScThreads / kWave;
  constexpr uint32_t EPV = 16 / sizeof(W);
  __shared__ uint4 s_rows[kWaves][kRowLdsBytes / 16];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t lane = lane_id();
  uint4* row4 = s_rows[wave];
  W* row = reinterpret_cast<W*>(row4);
  const uint32_t n_vec = (D + EPV - 1) / EPV;  // LDS vectors that cover the row
  for (uint32_t q = lane; q < n_vec; q += kWave) row4[q] = make_uint4(0, 0, 0, 0);
  for (uint64_t b = static_cast<uint64_t>(blockIdx.x) * kWaves + wave; b < B;
       b += static_cast<uint64_t>(gridDim.x) * kWaves) {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    for (uint32_t j = lane; j < k; j += kWave) {
      const uint32_t c = static_cast<uint32_t>(idx[b * k + j]);
      if (c < D) row[c] = val[b * k + j];
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    W* dst = out + b * out_stride;
    if (vec_ok) {  // 16-byte-aligned rows of whole vectors
      uint4* dst4 = reinterpret_cast<uint4*>(dst);
      for (uint32_t q = lane; q < n_vec; q += kWave) {
        const uint4 x = row4[q];
        st_stream(&dst4[q], x.x, x.y, x.z, x.w);
        row4[q] = make_uint4(0, 0, 0, 0);
      }
    } else {
      for (uint32_t c = lane; c < D; c += kWave) dst[c] = row[c];
      __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
      __builtin_amdgcn_wave_barrier();
      for (uint32_t q = lane; q < n_vec; q += kWave) row4[q] = make_uint4(0, 0, 0, 0);
    }
  }
}

// Narrow dense rows (output row stride = D, whole 16-byte vectors): a wavefront assembles R consecutive
// rows at once, R * D * sizeof(W) <= kRowLdsBytes, so that the fixed work per step covers 16 KiB of
// output whatever the row width (one row per step left 512-byte rows at a quarter of the rate).
template <typename W, typename I>
__global__ __launch_bounds__(kScThreads) void rowscatter_block_kernel(
    const I* __restrict__ idx, const W* __restrict__ val, uint32_t B, uint32_t D, uint32_t k,
    W* __restrict__ out, uint32_t R) {
  constexpr int kWaves = kScThreads / kWave;
  constexpr uint32_t EPV = 16 / sizeof(W);
  __shared__ uint4 s_rows[kWaves][kRowLdsBytes / 16];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t lane = lane_id();
  uint4* blk4 = s_rows[wave];
  W* blk = reinterpret_cast<W*>(blk4);
  const uint32_t vpr = D / EPV;  // vectors per row
  for (uint32_t q = lane; q < R * vpr; q += kWave) blk4[q] = make_uint4(0, 0, 0, 0);
  for (uint64_t b0 = (static_cast<uint64_t>(blockIdx.x) * kWaves + wave) * R; b0 < B;
       b0 += static_cast<uint64_t>(gridDim.x) * kWaves * R) {
    const uint32_t rows = static_cast<uint32_t>(min(static_cast<uint64_t>(R), B - b0));
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    const uint32_t n_pairs = rows * k;  // the block's pairs are contiguous in idx / val
    const I* bi = idx + b0 * k;
    const W* bv = val + b0 * k;
    for (uint32_t j = lane; j < n_pairs; j += kWave) {
      const uint32_t r = j / k;
      const uint32_t c = static_cast<uint32_t>(bi[j]);
      if (c < D) blk[r * D + c] = bv[j];
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    uint4* dst4 = reinterpret_cast<uint4*>(out + b0 * D);
    for (uint32_t q = lane; q < rows * vpr; q += kWave) {
      const uint4 x = blk4[q];
      st_stream(&dst4[q], x.x, x.y, x.z, x.w);
      blk4[q] = make_uint4(0, 0, 0, 0);
    }
  }
}

// Dense rows of any width: a workgroup zeroes the row in global memory, waits for those stores, then
// drops the values in.
template <typename W, typename I>
__global__ __launch_bounds__(kScThreads) void rowscatter_global_kernel(
    const I* __restrict__ idx, const W* __restrict__ val, uint32_t B, uint32_t D, uint32_t k, W* out,
    uint64_t out_stride) {
  for (uint64_t b = blockIdx.x; b < B; b += gridDim.x) {
    W* dst = out + b * out_stride;
    for (uint32_t c = threadIdx.x; c < D; c += kScThreads) dst[c] = 0;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the zero stores have landed ...
    __syncthreads();                                  // ... in every wavefront, before a value follows them
    for (uint32_t j = threadIdx.x; j < k; j += kScThreads) {
      const uint32_t c = static_cast<uint32_t>(idx[b * k + j]);
      if (c < D) dst[c] = val[b * k + j];
    }
  }
}

}  // namespace
}  // namespace dct

using namespace dct;

extern "C" int dct_scatter(const int32_t* d_idx, const void* d_val, const uint64_t* d_count, uint64_t capacity, int dt,
                           void* d_out, uint64_t n, int mode, void* hip_stream) {
  if (!d_out || n == 0 || n > 0x7FFFFFFFull) return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  if (mode != DCT_SCATTER_ASSIGN && mode != DCT_SCATTER_ADD) return DCT_ERR_INVALID;
  if (mode == DCT_SCATTER_ADD && dt != DCT_F32) return DCT_ERR_INVALID;
  if (capacity > 0xFFFFFFFFull) capacity = 0xFFFFFFFFull;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (capacity > 0 && (!d_idx || !d_val || !is_aligned(d_idx, 4) || !is_aligned(d_val, es))) return DCT_ERR_INVALID;
  if (!is_aligned(d_out, es) || (d_count && !is_aligned(d_count, 8))) return DCT_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint32_t n32 = static_cast<uint32_t>(n);
  const uint32_t pair_grid = static_cast<uint32_t>(std::min<uint64_t>(kScMaxGrid, (capacity + 255) / 256));

  if (mode == DCT_SCATTER_ADD) {
    if (capacity == 0) return DCT_OK;
    const uint32_t add_grid = static_cast<uint32_t>(std::min<uint64_t>(4u * kScMaxGrid, (capacity + 1023) / 1024));
    hipLaunchKernelGGL(scatter_add4_kernel, dim3(add_grid), dim3(256), 0, s, d_idx,
                       static_cast<const uint32_t*>(d_val), d_count, capacity, static_cast<uint32_t*>(d_out), n32);
    return launch_status();
  }
  if (is_aligned(d_out, 16)) {
    const uint32_t tile = kScTileBytes / static_cast<uint32_t>(es);
    const uint32_t n_tiles = (n32 + tile - 1) / tile;
    const uint32_t tiles_per_wg = kScTilesPerWg;
    const uint32_t grid = (n_tiles + tiles_per_wg - 1) / tiles_per_wg;
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((scatter_assign_kernel<uint32_t>), dim3(grid), dim3(kScThreads), 0, s, d_idx,
                         static_cast<const uint32_t*>(d_val), d_count, capacity, static_cast<uint32_t*>(d_out), n32,
                         tiles_per_wg);
    } else {
      hipLaunchKernelGGL((scatter_assign_kernel<uint16_t>), dim3(grid), dim3(kScThreads), 0, s, d_idx,
                         static_cast<const uint16_t*>(d_val), d_count, capacity, static_cast<uint16_t*>(d_out), n32,
                         tiles_per_wg);
    }
    return launch_status();
  }
  // misaligned output: zero fill, then one thread per pair (stream order keeps the two apart)
  const uint32_t fill_grid = static_cast<uint32_t>(std::min<uint64_t>(kScMaxGrid, (n + 255) / 256));
  if (dt == DCT_F32) {
    hipLaunchKernelGGL((zero_fill_kernel<uint32_t>), dim3(fill_grid), dim3(256), 0, s, static_cast<uint32_t*>(d_out), n32);
    if (capacity)
      hipLaunchKernelGGL((scatter_pairs_kernel<uint32_t, false>), dim3(pair_grid), dim3(256), 0, s, d_idx,
                         static_cast<const uint32_t*>(d_val), d_count, capacity, static_cast<uint32_t*>(d_out), n32);
  } else {
    hipLaunchKernelGGL((zero_fill_kernel<uint16_t>), dim3(fill_grid), dim3(256), 0, s, static_cast<uint16_t*>(d_out), n32);
    if (capacity)
      hipLaunchKernelGGL((scatter_pairs_kernel<uint16_t, false>), dim3(pair_grid), dim3(256), 0, s, d_idx,
                         static_cast<const uint16_t*>(d_val), d_count, capacity, static_cast<uint16_t*>(d_out), n32);
  }
  return launch_status();
}

namespace {

template <typename I>
int launch_rowscatter(const I* d_idx, const void* d_val, int dt, uint32_t B, uint32_t D, uint32_t k, void* d_out,
                      uint64_t out_row_stride_elems, void* hip_stream) {
  if (!d_idx || !d_val || !d_out || B == 0 || D == 0 || k == 0 || k > D || out_row_stride_elems < D)
    return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  if (D > (sizeof(I) == 2 ? 65536u : 0x7FFFFFFFu)) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(d_idx, sizeof(I)) || !is_aligned(d_val, es) || !is_aligned(d_out, es)) return DCT_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint32_t resident = static_cast<uint32_t>(device_cu_count()) * 8u;
  if (static_cast<uint64_t>(D) * es <= kRowLdsBytes) {
    const bool vec_ok = is_aligned(d_out, 16) && (out_row_stride_elems * es) % 16 == 0 && (D * es) % 16 == 0;
    const uint32_t rows_per_step = static_cast<uint32_t>(kRowLdsBytes / (D * es));
    if (vec_ok && out_row_stride_elems == D && rows_per_step >= 8) {  // dense rows of up to 2 KiB: several per step
      const uint32_t steps = ceil_div(B, rows_per_step);
      const uint32_t bgrid = std::min<uint32_t>((steps + 3) / 4, resident);
      if (dt == DCT_F32) {
        hipLaunchKernelGGL((rowscatter_block_kernel<uint32_t, I>), dim3(bgrid), dim3(kScThreads), 0, s, d_idx,
                           static_cast<const uint32_t*>(d_val), B, D, k, static_cast<uint32_t*>(d_out), rows_per_step);
      } else {
        hipLaunchKernelGGL((rowscatter_block_kernel<uint16_t, I>), dim3(bgrid), dim3(kScThreads), 0, s, d_idx,
                           static_cast<const uint16_t*>(d_val), B, D, k, static_cast<uint16_t*>(d_out), rows_per_step);
      }
      return launch_status();
    }
    const uint32_t grid = std::min<uint32_t>(ceil_div(B, 4u), resident);
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((rowscatter_lds_kernel<uint32_t, I>), dim3(grid), dim3(kScThreads), 0, s, d_idx,
                         static_cast<const uint32_t*>(d_val), B, D, k, static_cast<uint32_t*>(d_out),
                         out_row_stride_elems, vec_ok);
    } else {
      hipLaunchKernelGGL((rowscatter_lds_kernel<uint16_t, I>), dim3(grid), dim3(kScThreads), 0, s, d_idx,
                         static_cast<const uint16_t*>(d_val), B, D, k, static_cast<uint16_t*>(d_out),
                         out_row_stride_elems, vec_ok);
    }
  } else {
    const uint32_t grid = std::min<uint32_t>(B, resident * 4u);
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((rowscatter_global_kernel<uint32_t, I>), dim3(grid), dim3(kScThreads), 0, s, d_idx,
                         static_cast<const uint32_t*>(d_val), B, D, k, static_cast<uint32_t*>(d_out),
                         out_row_stride_elems);
    } else {
      hipLaunchKernelGGL((rowscatter_global_kernel<uint16_t, I>), dim3(grid), dim3(kScThreads), 0, s, d_idx,
                         static_cast<const uint16_t*>(d_val), B, D, k, static_cast<uint16_t*>(d_out),
                         out_row_stride_elems);
    }
  }
  return launch_status();
}

}  // namespace

extern "C" int dct_rowtopk_scatter(const int32_t* d_idx, const void* d_val, int dt, uint32_t B, uint32_t D, uint32_t k,
                                   void* d_out, uint64_t out_row_stride_elems, void* hip_stream) {
  return launch_rowscatter(d_idx, d_val, dt, B, D, k, d_out, out_row_stride_elems, hip_stream);
}

extern "C" int dct_rowtopk_scatter_idx16(const uint16_t* d_idx, const void* d_val, int dt, uint32_t B, uint32_t D,
                                         uint32_t k, void* d_out, uint64_t out_row_stride_elems, void* hip_stream) {
  return launch_rowscatter(d_idx, d_val, dt, B, D, k, d_out, out_row_stride_elems, hip_stream);
}
