// dct_rowtopk_fwd / dct_rowtopk_bwd: Algorithm 2.  Forward: per sample (row of
// X_act) the k largest magnitudes, i.e. the mask m_i = I(|X_act,i| >= tau_i)
// made exactly k wide (ties to the lower column), emitted as ascending column
// indices plus the selected values.  Backward: X_grad through the same mask,
// which is a gather of dy at the forward indices (no new selection: Sec. 2.2
// reuses the forward mask in the backward pass).
#include <algorithm>
#include <type_traits>

#include "dct_common.hpp"
#include "rowtopk_fast.hpp"
#include "rowtopk_quad.hpp"

namespace dct {
namespace {

constexpr int kRtThreads = 256;
constexpr int kRtWaves = kRtThreads / kWave;
constexpr int kRtBins = 2048;
constexpr uint32_t kQuadMinRows = 8192;  // below this the one-row-per-wavefront kernel has more wavefronts to offer

// ---------------------------------------------------------------------------
// Generic forward kernel: one wavefront per row, any D, any row stride, rows
// read from memory once per radix pass (digits 11+11+9 for fp32, 8+7 for bf16)
// plus once for the ordered emit.  Wave-synchronous: no workgroup barrier.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
}

// ENC (RowEnc): the row's mask goes out through `idx_out` as 32- or 16-bit column indices or as a
// bitmap of ceil(D/32) words per row.
template <int DT, int ENC>
__global__ __launch_bounds__(kRtThreads) void rowtopk_fwd_generic_kernel(
    const typename Elem<DT>::word_t* __restrict__ x, uint32_t B, uint32_t D, uint64_t stride, uint32_t k,
    void* __restrict__ idx_out, typename Elem<DT>::word_t* __restrict__ val_out,
    typename Elem<DT>::word_t* __restrict__ tau_out) {
  using E = Elem<DT>;
  __shared__ uint32_t s_hist[kRtWaves][kRtBins];
  const int wave = threadIdx.x / kWave;
  const uint32_t lane = lane_id();
  constexpr int kPasses = DT == DCT_F32 ? 3 : 2;
  constexpr int kShift[3] = {DT == DCT_F32 ? 20 : 7, DT == DCT_F32 ? 9 : 0, 0};
  constexpr int kWidth[3] = {DT == DCT_F32 ? 11 : 8, DT == DCT_F32 ? 11 : 7, 9};
  constexpr int kPer = kRtBins / kWave;  // bins per lane in the scan
  uint32_t* h = s_hist[wave];

  for (uint64_t row = static_cast<uint64_t>(blockIdx.x) * kRtWaves + wave; row < B;
       row += static_cast<uint64_t>(gridDim.x) * kRtWaves) {
    const typename E::word_t* xr = x + row * stride;
    uint32_t prefix = 0, k_rem = k, fixed_mask = 0;
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int shift = kShift[p], width = kWidth[p];
      const uint32_t dmask = (1u << width) - 1u;
      for (int i = lane; i < kRtBins; i += kWave) h[i] = 0;
      wave_lds_sync();
      for (uint32_t c0 = 0; c0 < D; c0 += kWave) {
        const uint32_t c = c0 + lane;
        const bool in = c < D;
        const uint32_t key = in ? (static_cast<uint32_t>(xr[c]) & E::kKeyMask) : 0u;
        hist_add(h, in && (key & fixed_mask) == prefix, (key >> shift) & dmask);
      }
      wave_lds_sync();
      // lane L owns bins 2047-32L ... 2047-32L-31 (top down)
      uint32_t sum = 0;
      for (int j = 0; j < kPer; ++j) sum += h[kRtBins - 1 - (lane * kPer + j)];
      uint32_t incl = sum;
#pragma unroll
      for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t t = __shfl_up(incl, d, kWave);
        if (lane >= static_cast<uint32_t>(d)) incl += t;
      }
      uint32_t above = incl - sum;
      const bool mine = above < k_rem && k_rem <= incl;
      uint32_t f_bin = 0, f_above = 0;
      if (mine) {
        bool found = false;
        for (int j = 0; j < kPer; ++j) {
          const uint32_t cj = h[kRtBins - 1 - (lane * kPer + j)];
          if (!found && above < k_rem && k_rem <= above + cj) {
            f_bin = kRtBins - 1 - (lane * kPer + j);
            f_above = above;
            found = true;
          }
          if (!found) above += cj;
        }
      }
      const int src = __builtin_ctzll(ballot64(mine));
      f_bin = __shfl(f_bin, src, kWave);
      f_above = __shfl(f_above, src, kWave);
      prefix |= f_bin << shift;
      k_rem -= f_above;
      fixed_mask |= dmask << shift;
      wave_lds_sync();
    }
    const uint32_t tau = prefix;  // key of the k-th largest magnitude of the row
    const uint32_t quota = k_rem; // ties at tau to keep, lowest columns first

    // ordered emit
    uint32_t out = 0, ties_seen = 0;
    typename E::word_t* vo = val_out + row * k;
    for (uint32_t c0 = 0; c0 < D; c0 += kWave) {
      const uint32_t c = c0 + lane;
      const bool in = c < D;
      const uint32_t raw = in ? static_cast<uint32_t>(xr[c]) : 0u;
      const uint32_t key = raw & E::kKeyMask;
      const bool gt = in && key > tau;
      const bool eq = in && key == tau;
      const uint64_t m_eq = ballot64(eq);
      const bool keep = gt || (eq && ties_seen + lanes_below(m_eq) < quota);
      const uint64_t m_keep = ballot64(keep);
      const uint32_t slot = out + lanes_below(m_keep);
      if (keep && slot < k) {
        put_col<ENC>(idx_out, row * k + slot, c);
        vo[slot] = static_cast<typename E::word_t>(raw);
      }
      if constexpr (ENC == kEncBitmap) {  // the ballot is the mask of these 64 columns
        const uint32_t n_words = (D + 31) / 32;
        uint32_t* mo = static_cast<uint32_t*>(idx_out) + row * n_words;
        const uint32_t w = c0 / 32 + lane;
        if (lane < 2 && w < n_words) mo[w] = static_cast<uint32_t>(m_keep >> (32 * lane));
      }
      out += __popcll(m_keep);
      ties_seen += __popcll(m_eq);
    }
    if (tau_out && lane == 0) tau_out[row] = static_cast<typename E::word_t>(tau);
  }
}

// ---------------------------------------------------------------------------
// Backward: gather through the forward indices.
// ---------------------------------------------------------------------------
template <typename W, typename I>
__global__ __launch_bounds__(256) void rowtopk_bwd_gather_kernel(const W* __restrict__ dy, uint32_t B, uint32_t D,
                                                                uint64_t stride, uint32_t k,
                                                                const I* __restrict__ idx,
                                                                W* __restrict__ dval) {
  const uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= k) return;
  for (uint32_t b = blockIdx.y; b < B; b += gridDim.y) {
    const uint64_t o = static_cast<uint64_t>(b) * k + j;
    const uint32_t c = static_cast<uint32_t>(idx[o]);
    dval[o] = c < D ? dy[static_cast<uint64_t>(b) * stride + c] : static_cast<W>(0);
  }
}

// The same gather with one thread per output element over all rows: for k well below a workgroup's
// 256 threads (narrow rows) the row-per-workgroup grid above leaves most threads idle.
template <typename W, typename I>
__global__ __launch_bounds__(256) void rowtopk_bwd_gather_flat_kernel(const W* __restrict__ dy, uint64_t n_out,
                                                                     uint32_t D, uint64_t stride, uint32_t k,
                                                                     const I* __restrict__ idx,
                                                                     W* __restrict__ dval) {
  const uint64_t o = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (o >= n_out) return;
  const uint32_t b = static_cast<uint32_t>(o / k);  // B < 2^32
  const uint32_t c = static_cast<uint32_t>(idx[o]);
  dval[o] = c < D ? dy[static_cast<uint64_t>(b) * stride + c] : static_cast<W>(0);
}

// The same gather for rows of which the list touches nearly every 64-byte sector anyway (k >= D / 32):
// the whole row is streamed into LDS with coalesced 16-byte loads and the picks are made there.  One
// workgroup of 16 wavefronts per CU; its rows are blocks of 16 consecutive ones, one block in every
// stripe of the grid, taken one at a time from a counter in LDS (a SIMD serves its oldest wavefront
// first: rows dealt out in advance leave the youngest wavefronts behind).  The next row and the first
// 256 entries of its list are on their way while the current row is gathered.  Rows of up to 8 KiB.
constexpr uint32_t kBwdRowBytes = 8192;
constexpr int kBwdWaves = 16;
template <typename W, typename I>
__global__ __launch_bounds__(kBwdWaves * kWave) void rowtopk_bwd_rows_kernel(
    const W* __restrict__ dy, uint32_t B, uint32_t D, uint64_t stride, uint32_t k, const I* __restrict__ idx,
    W* __restrict__ dval) {
  constexpr uint32_t EPV = 16 / sizeof(W);
  constexpr int NV = kBwdRowBytes / 16 / kWave;  // 16-byte vectors per lane: 8
  constexpr int NI = 4;                          // list entries per lane that are fetched ahead
  __shared__ uint4 s_rows[kBwdWaves][kBwdRowBytes / 16];
  __shared__ uint32_t s_taken;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t lane = lane_id();
  uint4* row4 = s_rows[wave];
  const W* row_lds = reinterpret_cast<const W*>(row4);
  const uint32_t n_vec = D / EPV;  // the host guarantees whole vectors and aligned rows
  if (threadIdx.x == 0) s_taken = 0;
  __syncthreads();
  const uint64_t stripe = static_cast<uint64_t>(gridDim.x) * kBwdWaves;
  auto take_row = [&]() -> uint64_t {
    uint32_t n = 0;
    if (lane == 0) n = atomicAdd(&s_taken, 1u);
    n = __builtin_amdgcn_readfirstlane(n);
    return static_cast<uint64_t>(blockIdx.x) * kBwdWaves + (n % kBwdWaves) + static_cast<uint64_t>(n / kBwdWaves) * stripe;
  };
  uint4 nxt[NV];
  uint32_t nidx[NI];
  auto load_row = [&](uint64_t r) {
    const uint4* src = reinterpret_cast<const uint4*>(dy + r * stride) + lane;
#pragma unroll
    for (int j = 0; j < NV; ++j)
      nxt[j] = j * kWave + lane < n_vec ? ld_stream(&src[j * kWave]) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int j = 0; j < NI; ++j)
      nidx[j] = j * kWave + lane < k ? static_cast<uint32_t>(idx[r * k + j * kWave + lane]) : 0u;
  };
  uint64_t row = take_row(), next_row = 0;
  if (row < B) load_row(row);
  for (; row < B; row = next_row) {
    fast::wave_lds_fence();  // the previous row's picks are done
#pragma unroll
    for (int j = 0; j < NV; ++j) row4[j * kWave + lane] = nxt[j];
    uint32_t cur[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) cur[j] = nidx[j];
    fast::wave_lds_fence();
    next_row = take_row();
    if (next_row < B) load_row(next_row);
    W* out = dval + row * k;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const uint32_t o = j * kWave + lane;
      if (o < k) out[o] = cur[j] < D ? row_lds[cur[j]] : static_cast<W>(0);
    }
    for (uint32_t o = NI * kWave + lane; o < k; o += kWave) {
      const uint32_t c = static_cast<uint32_t>(idx[row * k + o]);
      out[o] = c < D ? row_lds[c] : static_cast<W>(0);
    }
  }
}

// ---------------------------------------------------------------------------
// Consumers of the bitmap form, one wavefront per row: column c of a 64-column
// group belongs to lane c % 64; a ballot of the mask bits ranks the kept columns.
// GATHER: dval[b, j] = dy[b, column of the j-th set bit] (slots past the set bits
// are zeroed); otherwise: out[b, :] = zeros with val[b, j] at that column.
// ---------------------------------------------------------------------------
template <typename W, bool GATHER>
__global__ __launch_bounds__(kRtThreads) void rowtopk_bitmask_kernel(const W* __restrict__ src, uint32_t B, uint32_t D,
                                                                     uint64_t stride, uint32_t k,
                                                                     const uint32_t* __restrict__ mask,
                                                                     W* __restrict__ dst, uint64_t dst_stride) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t lane = lane_id();
  const uint32_t n_words = (D + 31) / 32;
  for (uint64_t row = static_cast<uint64_t>(blockIdx.x) * kRtWaves + wave; row < B;
       row += static_cast<uint64_t>(gridDim.x) * kRtWaves) {
    const uint32_t* mr = mask + row * n_words;
    uint32_t base = 0;
    for (uint32_t c0 = 0; c0 < D; c0 += kWave) {
      const uint32_t c = c0 + lane;
      const uint32_t w = c0 / 32 + lane / 32;
      const uint32_t word = w < n_words ? mr[w] : 0u;
      const bool set = c < D && ((word >> (lane % 32)) & 1u);
      const uint64_t m = ballot64(set);
      const uint32_t slot = base + lanes_below(m);
      if constexpr (GATHER) {
        if (set && slot < k) dst[row * k + slot] = src[row * stride + c];
      } else {
        if (c < D) dst[row * dst_stride + c] = (set && slot < k) ? src[row * k + slot] : static_cast<W>(0);
      }
      base += __popcll(m);
    }
    if constexpr (GATHER) {
      for (uint32_t j = base + lane; j < k; j += kWave) dst[row * k + j] = 0;
    }
  }
}

// The same two consumers with lane-contiguous columns: lane l of a wavefront owns columns
// [64 l, 64 l + 64) of a 4096-column pass, i.e. two mask words; one wave scan of the popcounts
// gives every lane its first slot, and the lanes then walk their own set bits, so all the
// gathers of a row are in flight together.  The dense row of the decompression is assembled
// in LDS (zeros + the values at their columns) and written with coalesced stores; it needs
// D * sizeof(W) <= kBmRowBytes.
constexpr uint32_t kBmRowBytes = 16384;
constexpr uint32_t kBmStageElems = 1024;  // columns of a row that are listed in LDS before the gather
constexpr uint32_t kBmWordsList = 512;    // the same for the narrow-row kernel: outputs of one step of a wavefront
template <typename W, bool GATHER>
__global__ __launch_bounds__(kRtThreads) void rowtopk_bitmask_lanes_kernel(
    const W* __restrict__ src, uint32_t B, uint32_t D, uint64_t stride, uint32_t k, const uint32_t* __restrict__ mask,
    W* __restrict__ dst, uint64_t dst_stride, bool vec_ok) {
  constexpr uint32_t EPV = 16 / sizeof(W);
  __shared__ uint4 s_rows[GATHER ? 1 : kRtWaves][GATHER ? 1 : kBmRowBytes / 16];
  __shared__ uint32_t s_cols[GATHER ? kRtWaves : 1][GATHER ? kBmStageElems : 1];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t lane = lane_id();
  const uint32_t n_words = (D + 31) / 32;
  uint4* row4 = s_rows[GATHER ? 0 : wave];
  W* row_lds = reinterpret_cast<W*>(row4);
  uint32_t* list = s_cols[GATHER ? wave : 0];
  // GATHER: the lanes list their columns in LDS at their slots, and lane j then fetches the value of slot
  // j, j + 64, ...: neighbouring lanes ask for neighbouring columns, so one load instruction touches a
  // third as many cache lines as when every lane fetches its own columns (each from a line of its own),
  // and the stores are coalesced.
  const bool staged = GATHER && k <= kBmStageElems;
  const uint32_t n_vec = (D + EPV - 1) / EPV;
  if constexpr (!GATHER) {
    for (uint32_t q = lane; q < n_vec; q += kWave) row4[q] = make_uint4(0, 0, 0, 0);
  }
  // the two mask words of this lane in the pass of 4096 columns that starts at column c0
  auto load_words = [&](uint64_t row, uint32_t c0) -> uint64_t {
    const uint32_t* mr = mask + row * n_words;
    const uint32_t col0 = c0 + lane * 64;
    const uint32_t w0 = col0 / 32;
    uint64_t m = 0;
    if (w0 < n_words) m = mr[w0];
    if (w0 + 1 < n_words) m |= static_cast<uint64_t>(mr[w0 + 1]) << 32;
    if (col0 >= D) m = 0;
    else if (D - col0 < 64) m &= (1ull << (D - col0)) - 1ull;  // bits past the row's end do not count
    return m;
  };
  const uint64_t row_step = static_cast<uint64_t>(gridDim.x) * kRtWaves;
  uint64_t row = static_cast<uint64_t>(blockIdx.x) * kRtWaves + wave;
  uint64_t m_next = row < B ? load_words(row, 0) : 0ull;
  for (; row < B; row += row_step) {
    if constexpr (!GATHER) wave_lds_sync();  // the row buffer is all zeros again
    uint32_t base = 0;
    for (uint32_t c0 = 0; c0 < D; c0 += kWave * 64) {  // passes of 4096 columns
      const uint32_t col0 = c0 + lane * 64;             // this lane's first column
      uint64_t m = c0 == 0 ? m_next : load_words(row, c0);
      if (c0 == 0 && row + row_step < B) m_next = load_words(row + row_step, 0);  // on its way during this row
      const uint32_t pc = __popcll(m);
      const uint32_t incl = wave_prefix_sum(pc);
      uint32_t slot = base + incl - pc;
      {
        // the first eight set bits of every lane without a loop: their loads are independent
        constexpr int kFirst = 8;
        uint32_t cols[kFirst];
        bool ok[kFirst];
        W v[kFirst];
#pragma unroll
        for (int j = 0; j < kFirst; ++j) {
          ok[j] = m != 0 && slot + j < k;
          cols[j] = col0 + (m != 0 ? __builtin_ctzll(m) : 0);
          m &= m - 1;  // stays 0 once it is 0
        }
        if (GATHER && staged) {
#pragma unroll
          for (int j = 0; j < kFirst; ++j)
            if (ok[j]) list[slot + j] = cols[j];
        } else {
#pragma unroll
          for (int j = 0; j < kFirst; ++j) {
            if constexpr (GATHER) v[j] = ok[j] ? src[row * stride + cols[j]] : static_cast<W>(0);
            else v[j] = ok[j] ? src[row * k + slot + j] : static_cast<W>(0);
          }
#pragma unroll
          for (int j = 0; j < kFirst; ++j) {
            if (ok[j]) {
              if constexpr (GATHER) dst[row * k + slot + j] = v[j];
              else row_lds[cols[j]] = v[j];
            }
          }
        }
        slot += min(pc, static_cast<uint32_t>(kFirst));
      }
      while (ballot64(m != 0) != 0) {
        if (m != 0) {
          const uint32_t c = col0 + __builtin_ctzll(m);
          m &= m - 1;
          if (slot < k) {
            if constexpr (GATHER) {
              if (staged) list[slot] = c;
              else dst[row * k + slot] = src[row * stride + c];
            } else {
              row_lds[c] = src[row * k + slot];
            }
          }
          ++slot;
        }
      }
      base += __builtin_amdgcn_readlane(incl, kWave - 1);
    }
    if constexpr (GATHER) {
      if (staged) {
        wave_lds_sync();  // the list is complete
        for (uint32_t j = lane; j < k; j += kWave)
          dst[row * k + j] = j < base ? src[row * stride + list[j]] : static_cast<W>(0);
        wave_lds_sync();  // ... and read, before the next row's columns arrive
      } else {
        for (uint32_t j = base + lane; j < k; j += kWave) dst[row * k + j] = 0;
      }
    } else {
      wave_lds_sync();
      W* out = dst + row * dst_stride;
      if (vec_ok) {
        uint4* out4 = reinterpret_cast<uint4*>(out);
        for (uint32_t q = lane; q < n_vec; q += kWave) {
          const uint4 v = row4[q];
          st_stream(&out4[q], v.x, v.y, v.z, v.w);
          row4[q] = make_uint4(0, 0, 0, 0);
        }
      } else {
        for (uint32_t c = lane; c < D; c += kWave) out[c] = row_lds[c];
        wave_lds_sync();
        for (uint32_t q = lane; q < n_vec; q += kWave) row4[q] = make_uint4(0, 0, 0, 0);
      }
    }
  }
}

// The backward gather through a bitmap for many rows of 4 to 8 KiB with dense masks: as rowtopk_bwd_rows_kernel,
// the row is streamed into LDS; the lanes turn their two mask words (64 columns each) into the ordered list of
// kept columns, also in LDS, and lane j then picks the values of slots j, j + 64, ...  k <= kBwdListCap.
constexpr uint32_t kBwdListCap = 512;
template <typename W>
__global__ __launch_bounds__(kBwdWaves * kWave) void rowtopk_bwd_rows_bitmask_kernel(
    const W* __restrict__ dy, uint32_t B, uint32_t D, uint64_t stride, uint32_t k, const uint32_t* __restrict__ mask,
    W* __restrict__ dval) {
  constexpr uint32_t EPV = 16 / sizeof(W);
  constexpr int NV = kBwdRowBytes / 16 / kWave;
  __shared__ uint4 s_rows[kBwdWaves][kBwdRowBytes / 16];
  __shared__ uint16_t s_list[kBwdWaves][kBwdListCap];
  __shared__ uint32_t s_taken;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t lane = lane_id();
  uint4* row4 = s_rows[wave];
  const W* row_lds = reinterpret_cast<const W*>(row4);
  uint16_t* list = s_list[wave];
  const uint32_t n_vec = D / EPV;            // the host guarantees whole vectors and aligned rows
  const uint32_t n_words = (D + 31) / 32;    // D <= 4096: a lane's two words cover the row
  if (threadIdx.x == 0) s_taken = 0;
  __syncthreads();
  const uint64_t stripe = static_cast<uint64_t>(gridDim.x) * kBwdWaves;
  auto take_row = [&]() -> uint64_t {
    uint32_t n = 0;
    if (lane == 0) n = atomicAdd(&s_taken, 1u);
    n = __builtin_amdgcn_readfirstlane(n);
    return static_cast<uint64_t>(blockIdx.x) * kBwdWaves + (n % kBwdWaves) + static_cast<uint64_t>(n / kBwdWaves) * stripe;
  };
  uint4 nxt[NV];
  uint64_t m_next = 0;
  auto load_row = [&](uint64_t r) {
    const uint4* src = reinterpret_cast<const uint4*>(dy + r * stride) + lane;
#pragma unroll
    for (int j = 0; j < NV; ++j)
      nxt[j] = j * kWave + lane < n_vec ? ld_stream(&src[j * kWave]) : make_uint4(0, 0, 0, 0);
    const uint32_t* mr = mask + r * n_words;
    const uint32_t w0 = lane * 2;
    uint64_t m = 0;
    if (w0 < n_words) m = mr[w0];
    if (w0 + 1 < n_words) m |= static_cast<uint64_t>(mr[w0 + 1]) << 32;
    const uint32_t col0 = lane * 64;
    if (col0 >= D) m = 0;
    else if (D - col0 < 64) m &= (1ull << (D - col0)) - 1ull;  // bits past the row's end do not count
    m_next = m;
  };
  uint64_t row = take_row(), next_row = 0;
  if (row < B) load_row(row);
  for (; row < B; row = next_row) {
    fast::wave_lds_fence();  // the previous row's picks are done
#pragma unroll
    for (int j = 0; j < NV; ++j) row4[j * kWave + lane] = nxt[j];
    uint64_t m = m_next;
    next_row = take_row();
    if (next_row < B) load_row(next_row);
    const uint32_t pc = __popcll(m);
    const uint32_t incl = wave_prefix_sum(pc);
    uint32_t slot = incl - pc;
    const uint32_t base = min(static_cast<uint32_t>(__builtin_amdgcn_readlane(incl, kWave - 1)), k);  // kept columns listed
    while (ballot64(m != 0) != 0) {
      if (m != 0) {
        const uint32_t c = lane * 64 + __builtin_ctzll(m);
        m &= m - 1;
        if (slot < k) list[slot] = static_cast<uint16_t>(c);  // k <= kBwdListCap, c < 4096
        ++slot;
      }
    }
    fast::wave_lds_fence();  // row and list are in place
    W* out = dval + row * k;
    for (uint32_t o = lane; o < k; o += kWave) out[o] = o < base ? row_lds[list[o]] : static_cast<W>(0);
  }
}

// The two consumers for NARROW rows whose mask is a power of two of words, at most 32 (D = 32 ... 1024 in
// powers of two): one lane per mask word, so a wavefront covers 64 / WPR rows at once.  One wave scan of the
// popcounts, less its value at the row's first lane, ranks every word's kept columns within its row.
// GATHER: dval[b, j] = dy[b, column of the j-th set bit]; otherwise the rows are assembled in LDS (2 or 4 KiB of
// dense output per step) and written with coalesced 16-byte stores; that needs dst_stride == D and 16-byte
// aligned output.
template <typename W, bool GATHER>
__global__ __launch_bounds__(kRtThreads) void rowtopk_bitmask_words_kernel(
    const W* __restrict__ src, uint32_t B, uint32_t D, uint64_t stride, uint32_t k, const uint32_t* __restrict__ mask,
    W* __restrict__ dst, uint32_t wpr) {
  constexpr uint32_t EPV = 16 / sizeof(W);
  __shared__ uint4 s_blk[GATHER ? 1 : kRtWaves][GATHER ? 1 : kWave * 32 * sizeof(W) / 16];
  __shared__ uint32_t s_list[GATHER ? kRtWaves : 1][GATHER ? kBmWordsList : 1];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t lane = lane_id();
  const uint32_t rows_per_step = kWave / wpr;
  const uint32_t r_loc = lane / wpr, w = lane % wpr;  // row of the step, word of the row
  uint4* blk4 = s_blk[GATHER ? 0 : wave];
  W* blk = reinterpret_cast<W*>(blk4);
  uint32_t* list = s_list[GATHER ? wave : 0];
  // GATHER: the step's outputs are rows_per_step * k consecutive elements of dval.  The lanes list
  // (row of the step, column) per output in LDS, and lane j then fetches outputs j, j + 64, ...:
  // neighbouring lanes read neighbouring columns and the stores are coalesced.
  const bool staged = GATHER && rows_per_step * k <= kBmWordsList;
  constexpr uint32_t kNoSource = 0xFFFFFFFFu;  // an output beyond the row's set bits: zero
  const uint32_t blk_vecs = kWave * 32 / EPV;  // the step's dense output in 16-byte vectors
  if constexpr (!GATHER) {
    for (uint32_t q = lane; q < blk_vecs; q += kWave) blk4[q] = make_uint4(0, 0, 0, 0);
  }
  const uint64_t n_steps = (static_cast<uint64_t>(B) + rows_per_step - 1) / rows_per_step;
  for (uint64_t step = static_cast<uint64_t>(blockIdx.x) * kRtWaves + wave; step < n_steps;
       step += static_cast<uint64_t>(gridDim.x) * kRtWaves) {
    const uint64_t row = step * rows_per_step + r_loc;
    const bool live = row < B;
    if constexpr (!GATHER) wave_lds_sync();  // the block buffer is all zeros again
    uint32_t m = live ? mask[row * wpr + w] : 0u;  // D = 32 * wpr: every bit of a word is a column
    const uint32_t pc = __popc(m);
    const uint32_t incl = wave_prefix_sum(pc);
    const int first = static_cast<int>(lane - w);  // the row's first lane
    const uint32_t prev = __shfl(incl, first > 0 ? first - 1 : 0, kWave);  // taken by all lanes together
    const uint32_t before_row = first > 0 ? prev : 0u;                      // set bits of the rows in lower lanes
    uint32_t slot = incl - pc - before_row;
    const uint32_t row_bits = __shfl(incl, first + static_cast<int>(wpr) - 1, kWave) - before_row;
    while (ballot64(m != 0) != 0) {
      if (m != 0) {
        const uint32_t c = 32 * w + __builtin_ctz(m);
        m &= m - 1;
        if (slot < k) {
          if constexpr (GATHER) {
            if (staged) list[r_loc * k + slot] = (r_loc << 16) | c;  // c < 1024
            else dst[row * k + slot] = src[row * stride + c];
          } else {
            blk[r_loc * D + c] = src[row * k + slot];
          }
        }
        ++slot;
      }
    }
    if constexpr (GATHER) {
      if (staged) {
        for (uint32_t j = row_bits + w; j < k; j += wpr) list[r_loc * k + j] = kNoSource;  // fewer set bits than k
        wave_lds_sync();  // the list is complete
        const uint64_t row0 = step * rows_per_step;
        const uint32_t rows_here = static_cast<uint32_t>(min(static_cast<uint64_t>(rows_per_step), B - row0));
        for (uint32_t j = lane; j < rows_here * k; j += kWave) {
          const uint32_t e = list[j];
          dst[row0 * k + j] = e != kNoSource ? src[(row0 + (e >> 16)) * stride + (e & 0xFFFFu)] : static_cast<W>(0);
        }
        wave_lds_sync();  // ... and read, before the next step's entries arrive
      } else if (live) {
        for (uint32_t j = row_bits + w; j < k; j += wpr) dst[row * k + j] = 0;  // fewer set bits than k
      }
    } else {
      wave_lds_sync();
      const uint64_t row0 = step * rows_per_step;
      const uint32_t rows_here = static_cast<uint32_t>(min(static_cast<uint64_t>(rows_per_step), B - row0));
      uint4* out4 = reinterpret_cast<uint4*>(dst + row0 * D);
      const uint32_t n_q = rows_here * (D / EPV);
      for (uint32_t q = lane; q < blk_vecs; q += kWave) {
        if (q < n_q) {
          const uint4 v = blk4[q];
          st_stream(&out4[q], v.x, v.y, v.z, v.w);
        }
        blk4[q] = make_uint4(0, 0, 0, 0);
      }
    }
  }
}

}  // namespace
}  // namespace dct

using namespace dct;

namespace {

// idx_or_mask: int32[B*k] or uint16[B*k] column indices, or uint32[B*ceil(D/32)] bitmap words (enc: RowEnc).
int launch_fwd(const void* x, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems, uint32_t k,
               void* idx_or_mask, void* d_val_out, void* d_tau_out, int enc, void* hip_stream) {
  if (!x || !idx_or_mask || !d_val_out || B == 0 || D == 0 || k == 0 || k > D || row_stride_elems < D)
    return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  if (D > (enc == kEncIdx16 ? 65536u : 0x7FFFFFFFu)) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(x, es) || !is_aligned(idx_or_mask, enc == kEncIdx16 ? 2 : 4) || !is_aligned(d_val_out, es) ||
      (d_tau_out && !is_aligned(d_tau_out, es)))
    return DCT_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  void* io = idx_or_mask;
  uint32_t grid = ceil_div(B, kRtWaves);
  if (grid > 65536u * 4) grid = 65536u * 4;
  // rows that fit the on-chip kernel: whole 16-byte vectors, 16-byte-aligned rows, at most 16 KiB
  const uint32_t epv = static_cast<uint32_t>(16 / es);
  // narrow bf16 rows, many of them: four rows per wavefront (the four lists of survivors share 512 staging slots)
  if (dt == DCT_BF16 && D % 8 == 0 && D <= quad::kMaxD && 4 * k <= quad::kStageSlots &&
      B >= kQuadMinRows && is_aligned(x, 16) && row_stride_elems % 8 == 0) {
    const uint32_t vecs = D / 8;
    const uint32_t cus = static_cast<uint32_t>(device_cu_count());
    const auto* xq = static_cast<const uint16_t*>(x);
    auto* vq = static_cast<uint16_t*>(d_val_out);
    auto* tq = static_cast<uint16_t*>(d_tau_out);
    // rows of up to 256 columns, when every wavefront of a full chip gets several groups: eight rows per wavefront
    const uint32_t groups8 = ceil_div(B, quad::kRowsNarrow);
    if (D <= quad::kMaxDNarrow && quad::kRowsNarrow * k <= quad::kStageSlots &&
        groups8 >= 4u * quad::kWavesLarge * cus) {
      const uint32_t nv8 = vecs <= 8 ? 1u : vecs <= 16 ? 2u : 4u;
      const uint32_t qgrid8 = std::min(ceil_div(groups8, static_cast<uint32_t>(quad::kWavesLarge)), cus);
#define DCT_LAUNCH_OCT(NVV, ENCV)                                                                               \
  hipLaunchKernelGGL((quad::rowtopk_fwd_quad_kernel<NVV, ENCV, quad::kWavesLarge, quad::kRowsNarrow>),          \
                     dim3(qgrid8), dim3(quad::kWavesLarge * kWave), 0, s, xq, B, D, row_stride_elems, k, io, vq, tq)
#define DCT_LAUNCH_OCT_NV(ENCV)                  \
  do {                                           \
    if (nv8 == 1) DCT_LAUNCH_OCT(1, ENCV);       \
    else if (nv8 == 2) DCT_LAUNCH_OCT(2, ENCV);  \
    else DCT_LAUNCH_OCT(4, ENCV);                \
  } while (0)
      if (enc == kEncIdx16) DCT_LAUNCH_OCT_NV(kEncIdx16);
      else if (enc == kEncBitmap) DCT_LAUNCH_OCT_NV(kEncBitmap);
      else DCT_LAUNCH_OCT_NV(kEncIdx32);
#undef DCT_LAUNCH_OCT_NV
#undef DCT_LAUNCH_OCT
      return launch_status();
    }
    const uint32_t nv = vecs <= 16 ? 1u : vecs <= 32 ? 2u : vecs <= 64 ? 4u : 8u;
    const uint32_t groups = ceil_div(B, quad::kRows);
    // one large workgroup per CU when each of its wavefronts gets at least four groups, else small workgroups,
    // as many per CU as registers and the LDS row buffers allow
    const bool large = groups >= 4u * quad::kWavesLarge * cus;
    const uint32_t wg_waves = large ? quad::kWavesLarge : quad::kWavesSmall;
    const uint32_t resident = large ? cus : cus * (nv == 8 ? 4u : nv == 4 ? 6u : 8u);
    const uint32_t qgrid = std::min(ceil_div(groups, wg_waves), resident);
#define DCT_LAUNCH_QUAD(NVV, ENCV)                                                                              \
  do {                                                                                                          \
    if (large)                                                                                                  \
      hipLaunchKernelGGL((quad::rowtopk_fwd_quad_kernel<NVV, ENCV, quad::kWavesLarge, quad::kRows>),            \
                         dim3(qgrid), dim3(quad::kWavesLarge * kWave), 0, s, xq, B, D, row_stride_elems, k, io, \
                         vq, tq);                                                                               \
    else                                                                                                        \
      hipLaunchKernelGGL((quad::rowtopk_fwd_quad_kernel<NVV, ENCV, quad::kWavesSmall, quad::kRows>),            \
                         dim3(qgrid), dim3(quad::kWavesSmall * kWave), 0, s, xq, B, D, row_stride_elems, k, io, \
                         vq, tq);                                                                               \
  } while (0)
#define DCT_LAUNCH_QUAD_NV(ENCV)                  \
  do {                                            \
    if (nv == 1) DCT_LAUNCH_QUAD(1, ENCV);        \
    else if (nv == 2) DCT_LAUNCH_QUAD(2, ENCV);   \
    else if (nv == 4) DCT_LAUNCH_QUAD(4, ENCV);   \
    else DCT_LAUNCH_QUAD(8, ENCV);                \
  } while (0)
    if (enc == kEncIdx16) DCT_LAUNCH_QUAD_NV(kEncIdx16);
    else if (enc == kEncBitmap) DCT_LAUNCH_QUAD_NV(kEncBitmap);
    else DCT_LAUNCH_QUAD_NV(kEncIdx32);
#undef DCT_LAUNCH_QUAD_NV
#undef DCT_LAUNCH_QUAD
    return launch_status();
  }
  if (D % epv == 0 && D * es <= 16384u && is_aligned(x, 16) && row_stride_elems % epv == 0) {
    // wavefronts per CU that registers and the LDS row buffers allow (rows of up to 2 / 4 / 8 / 16 KiB); how
    // many of them form a workgroup is the kernel's choice (fast::waves_per_wg)
    const uint32_t row_bytes = D * static_cast<uint32_t>(es);
    const uint32_t waves_per_cu = row_bytes <= 2048u ? 32u : row_bytes <= 4096u ? 24u : row_bytes <= 8192u ? 16u : 8u;
    const uint32_t cus = static_cast<uint32_t>(device_cu_count());
    const uint32_t vecs = D / epv;  // 16-byte vectors per row, spread over 64 lanes
#define DCT_LAUNCH_ONCHIP_W(NVV, MK, F32V, WV)                                                                   \
  do {                                                                                                          \
    using W = std::conditional_t<F32V, uint32_t, uint16_t>;                                                     \
    const dim3 g(std::min(ceil_div(B, static_cast<uint32_t>(WV)), cus * std::max(waves_per_cu / (WV), 1u))),     \
        b((WV) * kWave);                                                                                        \
    hipLaunchKernelGGL((fast::rowtopk_fwd_onchip_kernel<NVV, MK, F32V, WV>), g, b, 0, s, static_cast<const W*>(x), \
                       B, D, row_stride_elems, k, io, static_cast<W*>(d_val_out), static_cast<W*>(d_tau_out));  \
  } while (0)
  // the large workgroup (see fast::waves_per_wg) when each of its wavefronts gets at least four rows
#define DCT_LAUNCH_ONCHIP(NVV, MK, F32V)                                                         \
  do {                                                                                           \
    constexpr uint32_t wl = fast::waves_per_wg<NVV>();                                           \
    if (wl != fast::kWavesSmall && B >= 4u * wl * cus) DCT_LAUNCH_ONCHIP_W(NVV, MK, F32V, wl);   \
    else DCT_LAUNCH_ONCHIP_W(NVV, MK, F32V, fast::kWavesSmall);                                  \
  } while (0)
#define DCT_LAUNCH_ONCHIP_NV(MK, F32V)                       \
  do {                                                       \
    if (vecs <= 64) DCT_LAUNCH_ONCHIP(1, MK, F32V);          \
    else if (vecs <= 128) DCT_LAUNCH_ONCHIP(2, MK, F32V);    \
    else if (vecs <= 256) DCT_LAUNCH_ONCHIP(4, MK, F32V);    \
    else if (vecs <= 512) DCT_LAUNCH_ONCHIP(8, MK, F32V);    \
    else DCT_LAUNCH_ONCHIP(16, MK, F32V);                    \
  } while (0)
#define DCT_LAUNCH_ONCHIP_ENC(F32V)                                        \
  do {                                                                    \
    if (enc == kEncBitmap) DCT_LAUNCH_ONCHIP_NV(kEncBitmap, F32V);        \
    else if (enc == kEncIdx16) DCT_LAUNCH_ONCHIP_NV(kEncIdx16, F32V);     \
    else DCT_LAUNCH_ONCHIP_NV(kEncIdx32, F32V);                           \
  } while (0)
    if (dt == DCT_F32) DCT_LAUNCH_ONCHIP_ENC(true);
    else DCT_LAUNCH_ONCHIP_ENC(false);
#undef DCT_LAUNCH_ONCHIP_ENC
#undef DCT_LAUNCH_ONCHIP_NV
#undef DCT_LAUNCH_ONCHIP
#undef DCT_LAUNCH_ONCHIP_W
    return launch_status();
  }
#define DCT_LAUNCH_GENERIC(DTV, MK)                                                                       \
  hipLaunchKernelGGL((rowtopk_fwd_generic_kernel<DTV, MK>), dim3(grid), dim3(kRtThreads), 0, s,            \
                     static_cast<const Elem<DTV>::word_t*>(x), B, D, row_stride_elems, k, io,              \
                     static_cast<Elem<DTV>::word_t*>(d_val_out), static_cast<Elem<DTV>::word_t*>(d_tau_out))
#define DCT_LAUNCH_GENERIC_ENC(DTV)                                  \
  do {                                                              \
    if (enc == kEncBitmap) DCT_LAUNCH_GENERIC(DTV, kEncBitmap);     \
    else if (enc == kEncIdx16) DCT_LAUNCH_GENERIC(DTV, kEncIdx16);  \
    else DCT_LAUNCH_GENERIC(DTV, kEncIdx32);                        \
  } while (0)
  if (dt == DCT_F32) DCT_LAUNCH_GENERIC_ENC(DCT_F32);
  else DCT_LAUNCH_GENERIC_ENC(DCT_BF16);
#undef DCT_LAUNCH_GENERIC_ENC
#undef DCT_LAUNCH_GENERIC
  return launch_status();
}

}  // namespace

extern "C" int dct_rowtopk_fwd(const void* x, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems,
                               uint32_t k, int32_t* d_idx_out, void* d_val_out, void* d_tau_out,
                               void* hip_stream) {
  return launch_fwd(x, dt, B, D, row_stride_elems, k, d_idx_out, d_val_out, d_tau_out, kEncIdx32, hip_stream);
}

extern "C" int dct_rowtopk_fwd_bitmask(const void* x, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems,
                                       uint32_t k, uint32_t* d_mask_out, void* d_val_out, void* d_tau_out,
                                       void* hip_stream) {
  return launch_fwd(x, dt, B, D, row_stride_elems, k, d_mask_out, d_val_out, d_tau_out, kEncBitmap, hip_stream);
}

extern "C" int dct_rowtopk_bwd_bitmask(const void* dy, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems,
                                       uint32_t k, const uint32_t* d_mask, void* d_dval_out, void* hip_stream) {
  if (!dy || !d_mask || !d_dval_out || B == 0 || D == 0 || k == 0 || k > D || row_stride_elems < D)
    return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  if (D > 0x7FFFFFFFu) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(dy, es) || !is_aligned(d_mask, 4) || !is_aligned(d_dval_out, es)) return DCT_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint32_t cus = static_cast<uint32_t>(device_cu_count());
  const uint32_t resident = cus * 8u;
  // dense masks over many rows of 4 to 8 KiB: stream the rows through LDS
  if (static_cast<uint64_t>(D) * es <= kBwdRowBytes && D * es >= kBwdRowBytes / 2 && D <= 4096u && (D * es) % 16 == 0 &&
      is_aligned(dy, 16) && (row_stride_elems * es) % 16 == 0 && static_cast<uint64_t>(k) * 32 >= D &&
      k <= kBwdListCap && B >= 4u * kBwdWaves * cus) {
    const dim3 rgrid(std::min(ceil_div(B, static_cast<uint32_t>(kBwdWaves)), cus)), rblock(kBwdWaves * kWave);
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((rowtopk_bwd_rows_bitmask_kernel<uint32_t>), rgrid, rblock, 0, s,
                         static_cast<const uint32_t*>(dy), B, D, row_stride_elems, k, d_mask,
                         static_cast<uint32_t*>(d_dval_out));
    } else {
      hipLaunchKernelGGL((rowtopk_bwd_rows_bitmask_kernel<uint16_t>), rgrid, rblock, 0, s,
                         static_cast<const uint16_t*>(dy), B, D, row_stride_elems, k, d_mask,
                         static_cast<uint16_t*>(d_dval_out));
    }
    return launch_status();
  }
  const uint32_t wpr = D / 32;
  if (D % 32 == 0 && wpr <= 32 && (wpr & (wpr - 1)) == 0) {  // narrow rows: several per wavefront, one lane per word
    const uint32_t steps = ceil_div(B, kWave / wpr);
    const uint32_t wgrid = std::min<uint32_t>((steps + kRtWaves - 1) / kRtWaves, resident);
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((rowtopk_bitmask_words_kernel<uint32_t, true>), dim3(wgrid), dim3(kRtThreads), 0, s,
                         static_cast<const uint32_t*>(dy), B, D, row_stride_elems, k, d_mask,
                         static_cast<uint32_t*>(d_dval_out), wpr);
    } else {
      hipLaunchKernelGGL((rowtopk_bitmask_words_kernel<uint16_t, true>), dim3(wgrid), dim3(kRtThreads), 0, s,
                         static_cast<const uint16_t*>(dy), B, D, row_stride_elems, k, d_mask,
                         static_cast<uint16_t*>(d_dval_out), wpr);
    }
    return launch_status();
  }
  const uint32_t grid = std::min<uint32_t>(ceil_div(B, kRtWaves), resident);
  if (dt == DCT_F32) {
    hipLaunchKernelGGL((rowtopk_bitmask_lanes_kernel<uint32_t, true>), dim3(grid), dim3(kRtThreads), 0, s,
                       static_cast<const uint32_t*>(dy), B, D, row_stride_elems, k, d_mask,
                       static_cast<uint32_t*>(d_dval_out), static_cast<uint64_t>(k), false);
  } else {
    hipLaunchKernelGGL((rowtopk_bitmask_lanes_kernel<uint16_t, true>), dim3(grid), dim3(kRtThreads), 0, s,
                       static_cast<const uint16_t*>(dy), B, D, row_stride_elems, k, d_mask,
                       static_cast<uint16_t*>(d_dval_out), static_cast<uint64_t>(k), false);
  }
  return launch_status();
}

extern "C" int dct_rowtopk_scatter_bitmask(const uint32_t* d_mask, const void* d_val, int dt, uint32_t B, uint32_t D,
                                           uint32_t k, void* d_out, uint64_t out_row_stride_elems, void* hip_stream) {
  if (!d_mask || !d_val || !d_out || B == 0 || D == 0 || k == 0 || k > D || out_row_stride_elems < D)
    return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  if (D > 0x7FFFFFFFu) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(d_mask, 4) || !is_aligned(d_val, es) || !is_aligned(d_out, es)) return DCT_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint32_t resident = static_cast<uint32_t>(device_cu_count()) * 8u;
  const uint32_t grid = std::min<uint32_t>(ceil_div(B, kRtWaves), resident);
  const uint32_t wpr = D / 32;
  if (D % 32 == 0 && wpr <= 32 && (wpr & (wpr - 1)) == 0 && out_row_stride_elems == D && is_aligned(d_out, 16)) {
    // narrow dense rows: several per wavefront, one lane per mask word
    const uint32_t steps = ceil_div(B, kWave / wpr);
    const uint32_t wgrid = std::min<uint32_t>((steps + kRtWaves - 1) / kRtWaves, resident);
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((rowtopk_bitmask_words_kernel<uint32_t, false>), dim3(wgrid), dim3(kRtThreads), 0, s,
                         static_cast<const uint32_t*>(d_val), B, D, static_cast<uint64_t>(k), k, d_mask,
                         static_cast<uint32_t*>(d_out), wpr);
    } else {
      hipLaunchKernelGGL((rowtopk_bitmask_words_kernel<uint16_t, false>), dim3(wgrid), dim3(kRtThreads), 0, s,
                         static_cast<const uint16_t*>(d_val), B, D, static_cast<uint64_t>(k), k, d_mask,
                         static_cast<uint16_t*>(d_out), wpr);
    }
    return launch_status();
  }
  if (static_cast<uint64_t>(D) * es <= kBmRowBytes) {  // the row is assembled on chip
    const bool vec_ok = is_aligned(d_out, 16) && (out_row_stride_elems * es) % 16 == 0 && (D * es) % 16 == 0;
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((rowtopk_bitmask_lanes_kernel<uint32_t, false>), dim3(grid), dim3(kRtThreads), 0, s,
                         static_cast<const uint32_t*>(d_val), B, D, static_cast<uint64_t>(k), k, d_mask,
                         static_cast<uint32_t*>(d_out), out_row_stride_elems, vec_ok);
    } else {
      hipLaunchKernelGGL((rowtopk_bitmask_lanes_kernel<uint16_t, false>), dim3(grid), dim3(kRtThreads), 0, s,
                         static_cast<const uint16_t*>(d_val), B, D, static_cast<uint64_t>(k), k, d_mask,
                         static_cast<uint16_t*>(d_out), out_row_stride_elems, vec_ok);
    }
    return launch_status();
  }
  if (dt == DCT_F32) {
    hipLaunchKernelGGL((rowtopk_bitmask_kernel<uint32_t, false>), dim3(grid), dim3(kRtThreads), 0, s,
                       static_cast<const uint32_t*>(d_val), B, D, static_cast<uint64_t>(k), k, d_mask,
                       static_cast<uint32_t*>(d_out), out_row_stride_elems);
  } else {
    hipLaunchKernelGGL((rowtopk_bitmask_kernel<uint16_t, false>), dim3(grid), dim3(kRtThreads), 0, s,
                       static_cast<const uint16_t*>(d_val), B, D, static_cast<uint64_t>(k), k, d_mask,
                       static_cast<uint16_t*>(d_out), out_row_stride_elems);
  }
  return launch_status();
}

namespace {

template <typename I>
int launch_bwd(const void* dy, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems, uint32_t k, const I* d_idx,
               void* d_dval_out, void* hip_stream) {
  if (!dy || !d_idx || !d_dval_out || B == 0 || D == 0 || k == 0 || k > D || row_stride_elems < D)
    return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  if (D > (sizeof(I) == 2 ? 65536u : 0x7FFFFFFFu)) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(dy, es) || !is_aligned(d_idx, sizeof(I)) || !is_aligned(d_dval_out, es)) return DCT_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint64_t n_out = static_cast<uint64_t>(B) * k;
  // dense lists over rows of 4 to 8 KiB, enough rows for every wavefront of the chip: stream the rows through LDS
  const uint32_t cus = static_cast<uint32_t>(device_cu_count());
  if (static_cast<uint64_t>(D) * es <= kBwdRowBytes && D * es >= kBwdRowBytes / 2 && (D * es) % 16 == 0 && is_aligned(dy, 16) &&
      (row_stride_elems * es) % 16 == 0 && static_cast<uint64_t>(k) * 32 >= D && B >= 4u * kBwdWaves * cus) {
    const dim3 rgrid(std::min(ceil_div(B, static_cast<uint32_t>(kBwdWaves)), cus)), rblock(kBwdWaves * kWave);
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((rowtopk_bwd_rows_kernel<uint32_t, I>), rgrid, rblock, 0, s, static_cast<const uint32_t*>(dy),
                         B, D, row_stride_elems, k, d_idx, static_cast<uint32_t*>(d_dval_out));
    } else {
      hipLaunchKernelGGL((rowtopk_bwd_rows_kernel<uint16_t, I>), rgrid, rblock, 0, s, static_cast<const uint16_t*>(dy),
                         B, D, row_stride_elems, k, d_idx, static_cast<uint16_t*>(d_dval_out));
    }
    return launch_status();
  }
  // few outputs per row: one thread per output over all rows (a grid holds fewer than 2^32 threads)
  if (k < 192u && n_out + 255 <= 0xFFFFFFFFull) {
    const dim3 fgrid(static_cast<uint32_t>((n_out + 255) / 256));
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((rowtopk_bwd_gather_flat_kernel<uint32_t, I>), fgrid, dim3(256), 0, s,
                         static_cast<const uint32_t*>(dy), n_out, D, row_stride_elems, k, d_idx,
                         static_cast<uint32_t*>(d_dval_out));
    } else {
      hipLaunchKernelGGL((rowtopk_bwd_gather_flat_kernel<uint16_t, I>), fgrid, dim3(256), 0, s,
                         static_cast<const uint16_t*>(dy), n_out, D, row_stride_elems, k, d_idx,
                         static_cast<uint16_t*>(d_dval_out));
    }
    return launch_status();
  }
  const dim3 grid((k + 255) / 256, B < 65535u ? B : 65535u);
  if (dt == DCT_F32) {
    hipLaunchKernelGGL((rowtopk_bwd_gather_kernel<uint32_t, I>), grid, dim3(256), 0, s,
                       static_cast<const uint32_t*>(dy), B, D, row_stride_elems, k, d_idx,
                       static_cast<uint32_t*>(d_dval_out));
  } else {
    hipLaunchKernelGGL((rowtopk_bwd_gather_kernel<uint16_t, I>), grid, dim3(256), 0, s,
                       static_cast<const uint16_t*>(dy), B, D, row_stride_elems, k, d_idx,
                       static_cast<uint16_t*>(d_dval_out));
  }
  return launch_status();
}

}  // namespace

extern "C" int dct_rowtopk_bwd(const void* dy, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems,
                               uint32_t k, const int32_t* d_idx, void* d_dval_out, void* hip_stream) {
  return launch_bwd(dy, dt, B, D, row_stride_elems, k, d_idx, d_dval_out, hip_stream);
}

extern "C" int dct_rowtopk_fwd_idx16(const void* x, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems,
                                     uint32_t k, uint16_t* d_idx_out, void* d_val_out, void* d_tau_out,
                                     void* hip_stream) {
  return launch_fwd(x, dt, B, D, row_stride_elems, k, d_idx_out, d_val_out, d_tau_out, kEncIdx16, hip_stream);
}

extern "C" int dct_rowtopk_bwd_idx16(const void* dy, int dt, uint32_t B, uint32_t D, uint64_t row_stride_elems,
                                     uint32_t k, const uint16_t* d_idx, void* d_dval_out, void* hip_stream) {
  return launch_bwd(dy, dt, B, D, row_stride_elems, k, d_idx, d_dval_out, hip_stream);
}
