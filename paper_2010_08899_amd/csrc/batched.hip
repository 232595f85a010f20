// Batched DCT-DP: threshold selection and compaction of MANY tensors with a
// fixed number of launches.  The paper compresses layer by layer (Sec. 2.1:
// every layer's gradient gets its own threshold), and most layers of its models
// are small: a tensor of a million elements is a microsecond of memory traffic,
// so one call per layer is pure launch latency.  Here the layers are segments
// of one address range described by a table:
//   select  : table upload (+ workspace clear), one launch per radix digit over
//             all segments (a workgroup histograms 16 Ki elements of one segment
//             into that segment's histogram), one finish launch that writes every
//             segment's threshold record;
//   compact : table upload, a count launch (one workgroup per 8 Ki-element tile:
//             keys above tau, ties at tau), a scan launch (one workgroup per
//             segment: exclusive offsets of its tiles, the segment's count), a write
//             launch (the tile is read again -- these tensors sit in L2 / the
//             memory-side cache -- and the survivors go to their final slots).
// Per segment the results are exactly those of dct_select_threshold and
// dct_threshold_compact on that tensor alone; indices are relative to the segment.
// The table travels as kernel arguments (64 segments per upload launch), so no
// host memory is read after the call returns.
#include <algorithm>
#include <vector>

#include "radix_select.hpp"

namespace dct {
namespace {

constexpr uint32_t kBtMaxSeg = 1024;
constexpr uint32_t kBtUnit = 16384;     // elements per workgroup in a select pass
constexpr uint32_t kBtTile = 8192;      // elements per workgroup in the compaction kernels
constexpr int kBtThreads = kSelThreads;  // 256 (find_bin is instantiated for it)
constexpr uint32_t kBtPerThread = kBtTile / kBtThreads;  // 32
constexpr uint32_t kBtPackSegs = 64;    // segments per upload launch (2.5 KiB of kernel arguments)
constexpr int kBtMaxPasses = 3;

struct BtSeg {
  uint64_t offset;       // first element, from g
  uint64_t out_offset;   // first output slot
  uint32_t n, k, capacity;
  uint32_t unit_start;   // first select workgroup of the segment
  uint32_t tile_start;   // first compaction tile of the segment
  uint32_t pad;
};
static_assert(sizeof(BtSeg) == 40, "BtSeg layout");
struct BtPack {
  BtSeg seg[kBtPackSegs];
};

// Workspace layout, computed the same way on host and device.
struct BtLayout {
  size_t segs, states, hist, counts, offsets, total;
};
__host__ __device__ inline size_t bt_align(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }
__host__ __device__ inline BtLayout bt_layout(uint32_t n_seg, uint64_t total_tiles) {
  BtLayout l;
  size_t o = 0;
  l.segs = o;    o = bt_align(o + static_cast<size_t>(n_seg) * sizeof(BtSeg));
  l.states = o;  o = bt_align(o + static_cast<size_t>(kBtMaxPasses) * n_seg * sizeof(SelState));
  l.hist = o;    o = bt_align(o + static_cast<size_t>(kBtMaxPasses) * n_seg * kSelBins * 4);
  l.counts = o;  o = bt_align(o + static_cast<size_t>(total_tiles) * 8);
  l.offsets = o; o = bt_align(o + static_cast<size_t>(total_tiles) * 8);
  l.total = o;
  return l;
}

// Copies up to 64 table entries from the kernel arguments to the workspace and (select only) clears
// the histograms.
__global__ void bt_upload_kernel(BtPack pack, uint32_t first, uint32_t count, BtSeg* segs, uint32_t* hist,
                                 uint32_t hist_words) {
  if (blockIdx.x == 0 && threadIdx.x < count) segs[first + threadIdx.x] = pack.seg[threadIdx.x];
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < hist_words; i += gridDim.x * blockDim.x) hist[i] = 0;
}

// Segment that owns work item `item` (a select unit or a compaction tile): the last segment whose
// start is <= item.  Called by all threads of the workgroup; `start_of` reads one table entry.
template <typename StartOf>
__device__ uint32_t owner_segment(uint32_t n_seg, uint32_t item, StartOf start_of) {
  bool le = false;
  uint32_t cnt = 0;
  for (uint32_t base = 0; base < n_seg; base += blockDim.x) {  // uniform trip count
    const uint32_t s = base + threadIdx.x;
    le = s < n_seg && start_of(s) <= item;
    cnt += __syncthreads_count(le);
  }
  return cnt - 1;  // segment 0 starts at item 0, so cnt >= 1
}

// ------------------------------------------------------------------ select
// (1024 threads per unit of 16384 elements: a unit's workgroup is often alone on its CU, and with four
// wavefronts nothing hid the latency of its loads and of the LDS updates: 23 us per pass against 11.)
constexpr int kBtPassThreads = 1024;
template <int DT>
__global__ __launch_bounds__(kBtPassThreads) void bt_select_pass_kernel(const typename Elem<DT>::word_t* __restrict__ g,
                                                                    const BtSeg* __restrict__ segs, uint32_t n_seg,
                                                                    SelState* states, uint32_t* hist, int pass) {
  using E = Elem<DT>;
  __shared__ uint32_t h[kSelBins];
  __shared__ uint32_t s_tmp[kBtPassThreads / kWave + 4];
  const uint32_t seg = owner_segment(n_seg, blockIdx.x, [&](uint32_t s) { return segs[s].unit_start; });
  const BtSeg sg = segs[seg];
  const uint32_t unit = blockIdx.x - sg.unit_start;

  SelState st;
  if (pass == 0) {
    st.prefix = 0;
    st.k_rem = sg.k;
    st.n_gt = 0;
    st.from_cand = 0;
    st.n_src = sg.n;
    st.rem_bits = E::kKeyBits;
    st.width = min(kDigitBits, st.rem_bits);
    st.last_count = sg.n;
  } else {
    const uint32_t* prev_hist = hist + (static_cast<size_t>(pass - 1) * n_seg + seg) * kSelBins;
    st = advance_state_with<kBtPassThreads>(states[static_cast<size_t>(pass - 1) * n_seg + seg],
                                            [&](uint32_t b) { return prev_hist[b]; }, s_tmp);
  }
  if (unit == 0 && threadIdx.x == 0) states[static_cast<size_t>(pass) * n_seg + seg] = st;
  if (st.width == 0) return;  // uniform: every digit is fixed already

  const uint32_t shift = st.rem_bits - st.width;
  const uint32_t dmask = (1u << st.width) - 1u;
  const uint32_t fixed_mask = E::kKeyMask & ~((st.rem_bits >= 32u ? 0u : (1u << st.rem_bits)) - 1u);
  const uint32_t prefix = st.prefix;
  for (int i = threadIdx.x; i < kSelBins; i += kBtPassThreads) h[i] = 0;
  __syncthreads();
  const typename E::word_t* src = g + sg.offset;
  const uint32_t lo = unit * kBtUnit;
  const uint32_t hi = min(lo + kBtUnit, sg.n);  // lo < n by construction of the grid
  constexpr int kUnroll = 8;
  for (uint32_t base = lo; base < hi; base += kBtPassThreads * kUnroll) {
    uint32_t key[kUnroll];
    bool in[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t i = base + u * kBtPassThreads + threadIdx.x;
      in[u] = i < hi;
      key[u] = in[u] ? (static_cast<uint32_t>(src[i]) & E::kKeyMask) : 0u;
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) hist_add(h, in[u] && (key[u] & fixed_mask) == prefix, (key[u] >> shift) & dmask);
  }
  __syncthreads();
  uint32_t* gh = hist + (static_cast<size_t>(pass) * n_seg + seg) * kSelBins;
  for (int i = threadIdx.x; i < kSelBins; i += kBtPassThreads) {
    const uint32_t c = h[i];
    if (c) atomicAdd(&gh[i], c);
  }
}

__global__ __launch_bounds__(kBtThreads) void bt_select_finish_kernel(uint32_t n_seg, const SelState* states,
                                                                      const uint32_t* hist, int last,
                                                                      dct_threshold* __restrict__ out) {
  __shared__ uint32_t s_tmp[kSelWaves + 4];
  const uint32_t seg = blockIdx.x;
  const SelState st = advance_state(states[static_cast<size_t>(last) * n_seg + seg],
                                    hist + (static_cast<size_t>(last) * n_seg + seg) * kSelBins, s_tmp);
  if (threadIdx.x == 0) {
    out[seg].tau_key = st.prefix;
    out[seg].n_gt = st.n_gt;
    out[seg].n_eq = st.last_count;
    out[seg].tie_quota = st.k_rem;
  }
}

// ------------------------------------------------------------------ compact
// Flags of the kBtPerThread elements a thread owns in a tile.  A wavefront owns a contiguous quarter
// of the tile, and within it element r * 64 + lane belongs to lane `lane`, round r: index order is
// (wavefront, round, lane).
template <int DT, bool EXACT>
__device__ __forceinline__ void tile_flags(const typename Elem<DT>::word_t* __restrict__ src, uint32_t t0, uint32_t n,
                                           uint32_t tau, uint32_t (&raw)[kBtPerThread], uint32_t& above_bits,
                                           uint32_t& tie_bits) {
  using E = Elem<DT>;
  const uint32_t wave = threadIdx.x / kWave, lane = lane_id();
  above_bits = 0;
  tie_bits = 0;
#pragma unroll
  for (uint32_t r = 0; r < kBtPerThread; ++r) {
    const uint32_t i = t0 + wave * (kBtTile / kSelWaves) + r * kWave + lane;
    const bool in = i < n;
    raw[r] = in ? static_cast<uint32_t>(src[i]) : 0u;
    const uint32_t key = raw[r] & E::kKeyMask;
    const bool tie = EXACT && in && key == tau;
    const bool above = in && key >= tau && !tie;
    above_bits |= above ? (1u << r) : 0u;
    tie_bits |= tie ? (1u << r) : 0u;
  }
}

template <int DT, bool EXACT>
__global__ __launch_bounds__(kBtThreads) void bt_count_kernel(const typename Elem<DT>::word_t* __restrict__ g,
                                                              const BtSeg* __restrict__ segs, uint32_t n_seg,
                                                              const dct_threshold* __restrict__ thr,
                                                              uint64_t* __restrict__ counts) {
  __shared__ uint64_t s_w[kSelWaves];
  const uint32_t seg = owner_segment(n_seg, blockIdx.x, [&](uint32_t s) { return segs[s].tile_start; });
  const BtSeg sg = segs[seg];
  const uint32_t t0 = (blockIdx.x - sg.tile_start) * kBtTile;
  uint32_t raw[kBtPerThread], ab, tb;
  tile_flags<DT, EXACT>(g + sg.offset, t0, sg.n, thr[seg].tau_key, raw, ab, tb);
  const uint64_t mine = (static_cast<uint64_t>(__popc(ab)) << 32) | static_cast<uint64_t>(__popc(tb));
  const uint64_t w = wave_sum_u64(mine);
  if (lane_id() == 0) s_w[threadIdx.x / kWave] = w;
  __syncthreads();
  if (threadIdx.x == 0) counts[blockIdx.x] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

// One workgroup per segment: exclusive prefix of its tiles' counts (both halves of the packed word
// stay below 2^31, so one 64-bit add sums both), and the segment's survivor count.
template <bool EXACT>
__global__ __launch_bounds__(kBtThreads) void bt_scan_kernel(const BtSeg* __restrict__ segs,
                                                             const dct_threshold* __restrict__ thr,
                                                             const uint64_t* __restrict__ counts,
                                                             uint64_t* __restrict__ offsets,
                                                             uint64_t* __restrict__ count_out) {
  __shared__ uint64_t s_w[kSelWaves];
  const uint32_t seg = blockIdx.x;
  const BtSeg sg = segs[seg];
  const uint32_t tiles = (sg.n + kBtTile - 1) / kBtTile;
  const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
  uint64_t carry = 0;
  for (uint32_t base = 0; base < tiles; base += kBtThreads) {  // uniform trip count
    const uint32_t t = base + threadIdx.x;
    const uint64_t v = t < tiles ? counts[sg.tile_start + t] : 0ull;
    uint64_t incl = v;  // inclusive scan within the wavefront
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const uint64_t up = __shfl_up(incl, d, kWave);
      if (lane >= static_cast<uint32_t>(d)) incl += up;
    }
    if (lane == kWave - 1) s_w[wave] = incl;
    __syncthreads();
    uint64_t before = carry;
    for (uint32_t w = 0; w < wave; ++w) before += s_w[w];
    if (t < tiles) offsets[sg.tile_start + t] = before + incl - v;
    carry += s_w[0] + s_w[1] + s_w[2] + s_w[3];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    uint64_t c = carry >> 32;
    if (EXACT) c += min(static_cast<uint32_t>(carry), thr[seg].tie_quota);
    count_out[seg] = c;
  }
}

template <int DT, bool EXACT>
__global__ __launch_bounds__(kBtThreads) void bt_write_kernel(const typename Elem<DT>::word_t* __restrict__ g,
                                                              const BtSeg* __restrict__ segs, uint32_t n_seg,
                                                              const dct_threshold* __restrict__ thr,
                                                              const uint64_t* __restrict__ offsets,
                                                              int32_t* __restrict__ idx_out,
                                                              typename Elem<DT>::word_t* __restrict__ val_out) {
  using word_t = typename Elem<DT>::word_t;
  __shared__ uint32_t s_wa[kSelWaves], s_we[kSelWaves];
  const uint32_t seg = owner_segment(n_seg, blockIdx.x, [&](uint32_t s) { return segs[s].tile_start; });
  const BtSeg sg = segs[seg];
  const uint32_t t0 = (blockIdx.x - sg.tile_start) * kBtTile;
  const uint32_t tau = thr[seg].tau_key;
  const uint32_t quota = EXACT ? thr[seg].tie_quota : 0u;
  uint32_t raw[kBtPerThread], ab, tb;
  tile_flags<DT, EXACT>(g + sg.offset, t0, sg.n, tau, raw, ab, tb);
  const uint32_t wave = threadIdx.x / kWave, lane = lane_id();

  // survivors of each round of this wavefront, then the wavefronts before it
  uint32_t round_a[kBtPerThread], round_e[kBtPerThread];  // exclusive prefixes over the rounds
  uint32_t wa = 0, we = 0;
#pragma unroll
  for (uint32_t r = 0; r < kBtPerThread; ++r) {
    round_a[r] = wa;
    round_e[r] = we;
    wa += __popcll(ballot64((ab >> r) & 1u));
    if (EXACT) we += __popcll(ballot64((tb >> r) & 1u));
  }
  if (lane == 0) {
    s_wa[wave] = wa;
    s_we[wave] = we;
  }
  __syncthreads();
  const uint64_t excl = offsets[blockIdx.x];
  uint32_t a_before = static_cast<uint32_t>(excl >> 32), e_before = static_cast<uint32_t>(excl);
  for (uint32_t w = 0; w < wave; ++w) {
    a_before += s_wa[w];
    e_before += s_we[w];
  }
  int32_t* io = idx_out + sg.out_offset;
  word_t* vo = val_out + sg.out_offset;
#pragma unroll
  for (uint32_t r = 0; r < kBtPerThread; ++r) {
    const bool above = (ab >> r) & 1u, tie = EXACT && ((tb >> r) & 1u);
    const uint64_t m_above = ballot64(above);
    const uint64_t m_tie = EXACT ? ballot64(tie) : 0ull;
    if ((m_above | m_tie) == 0) continue;  // uniform
    // ties before this element in the segment, and how many of them were kept
    const uint32_t ties_before = e_before + round_e[r] + lanes_below(m_tie);
    const uint32_t kept_ties_before = min(ties_before, quota);
    const bool keep = above || (tie && ties_before < quota);
    const uint32_t slot = a_before + round_a[r] + lanes_below(m_above) + kept_ties_before;
    if (keep && slot < sg.capacity) {
      io[slot] = static_cast<int32_t>(t0 + wave * (kBtTile / kSelWaves) + r * kWave + lane);
      vo[slot] = static_cast<word_t>(raw[r]);
    }
  }
}

// Validates the table, clips capacities, assigns work items; returns a status.
int bt_prepare(const dct_segment* h_segs, uint32_t n_seg, bool need_k, std::vector<BtSeg>& out, uint64_t& units,
               uint64_t& tiles) {
  if (!h_segs || n_seg == 0 || n_seg > kBtMaxSeg) return DCT_ERR_INVALID;
  out.resize(n_seg);
  units = 0;
  tiles = 0;
  for (uint32_t s = 0; s < n_seg; ++s) {
    const dct_segment& h = h_segs[s];
    if (h.n == 0 || h.n > 0x7FFFFFFFull) return DCT_ERR_INVALID;
    if (need_k && (h.k == 0 || h.k > h.n)) return DCT_ERR_INVALID;
    BtSeg& b = out[s];
    b.offset = h.offset;
    b.out_offset = h.out_offset;
    b.n = static_cast<uint32_t>(h.n);
    b.k = static_cast<uint32_t>(h.k);
    b.capacity = h.capacity > 0xFFFFFFFFull ? 0xFFFFFFFFu : static_cast<uint32_t>(h.capacity);
    b.unit_start = static_cast<uint32_t>(units);
    b.tile_start = static_cast<uint32_t>(tiles);
    b.pad = 0;
    units += (h.n + kBtUnit - 1) / kBtUnit;
    tiles += (h.n + kBtTile - 1) / kBtTile;
    if (tiles > 0x7FFFFFFFull) return DCT_ERR_INVALID;
  }
  return DCT_OK;
}

void bt_upload(const std::vector<BtSeg>& segs, BtSeg* d_segs, uint32_t* d_hist, uint32_t hist_words, hipStream_t s) {
  const uint32_t n_seg = static_cast<uint32_t>(segs.size());
  for (uint32_t first = 0; first < n_seg; first += kBtPackSegs) {
    BtPack pack;
    const uint32_t count = std::min(kBtPackSegs, n_seg - first);
    for (uint32_t i = 0; i < kBtPackSegs; ++i) pack.seg[i] = segs[first + (i < count ? i : 0)];
    const bool clear = first == 0 && hist_words != 0;
    const uint32_t grid = clear ? std::min<uint32_t>(1024u, (hist_words + 255) / 256) : 1u;
    hipLaunchKernelGGL(bt_upload_kernel, dim3(grid), dim3(256), 0, s, pack, first, count, d_segs, d_hist,
                       clear ? hist_words : 0u);
  }
}

}  // namespace
}  // namespace dct

using namespace dct;

extern "C" size_t dct_batched_workspace_bytes(int dt, const dct_segment* h_segs, uint32_t n_seg) {
  if (dt != DCT_F32 && dt != DCT_BF16) return 0;
  std::vector<BtSeg> segs;
  uint64_t units, tiles;
  if (bt_prepare(h_segs, n_seg, false, segs, units, tiles) != DCT_OK) return 0;
  return bt_layout(n_seg, tiles).total;
}

extern "C" int dct_select_threshold_batched(const void* g, int dt, const dct_segment* h_segs, uint32_t n_seg,
                                            dct_threshold* d_thr_out, void* d_ws, size_t ws_bytes, void* hip_stream) {
  if (!g || !d_thr_out || (dt != DCT_F32 && dt != DCT_BF16)) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(g, es) || !is_aligned(d_thr_out, 16)) return DCT_ERR_INVALID;
  std::vector<BtSeg> segs;
  uint64_t units, tiles;
  const int rc = bt_prepare(h_segs, n_seg, true, segs, units, tiles);
  if (rc != DCT_OK) return rc;
  const BtLayout l = bt_layout(n_seg, tiles);
  if (!d_ws || !is_aligned(d_ws, 256) || ws_bytes < l.total) return DCT_ERR_WORKSPACE;
  char* ws = static_cast<char*>(d_ws);
  auto* d_segs = reinterpret_cast<BtSeg*>(ws + l.segs);
  auto* d_states = reinterpret_cast<SelState*>(ws + l.states);
  auto* d_hist = reinterpret_cast<uint32_t*>(ws + l.hist);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int n_pass = dt == DCT_F32 ? 3 : 2;  // 11 + 11 + 9 key bits, or 11 + 4
  bt_upload(segs, d_segs, d_hist, static_cast<uint32_t>(static_cast<size_t>(n_pass) * n_seg * kSelBins), s);
  for (int p = 0; p < n_pass; ++p) {
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((bt_select_pass_kernel<DCT_F32>), dim3(static_cast<uint32_t>(units)), dim3(kBtPassThreads), 0, s,
                         static_cast<const uint32_t*>(g), d_segs, n_seg, d_states, d_hist, p);
    } else {
      hipLaunchKernelGGL((bt_select_pass_kernel<DCT_BF16>), dim3(static_cast<uint32_t>(units)), dim3(kBtPassThreads), 0,
                         s, static_cast<const uint16_t*>(g), d_segs, n_seg, d_states, d_hist, p);
    }
  }
  hipLaunchKernelGGL(bt_select_finish_kernel, dim3(n_seg), dim3(kBtThreads), 0, s, n_seg, d_states, d_hist,
                     n_pass - 1, d_thr_out);
  return launch_status();
}

extern "C" int dct_threshold_compact_batched(const void* g, int dt, const dct_segment* h_segs, uint32_t n_seg,
                                             const dct_threshold* d_thr, int mode, int32_t* d_idx_out,
                                             void* d_val_out, uint64_t* d_count_out, void* d_ws, size_t ws_bytes,
                                             void* hip_stream) {
  if (!g || !d_thr || !d_count_out || (dt != DCT_F32 && dt != DCT_BF16)) return DCT_ERR_INVALID;
  if (mode != DCT_GE_TAU && mode != DCT_EXACT_K) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(g, es) || !is_aligned(d_thr, 16) || !is_aligned(d_count_out, 8)) return DCT_ERR_INVALID;
  std::vector<BtSeg> segs;
  uint64_t units, tiles;
  const int rc = bt_prepare(h_segs, n_seg, false, segs, units, tiles);
  if (rc != DCT_OK) return rc;
  bool any_capacity = false;
  for (const BtSeg& b : segs) any_capacity = any_capacity || b.capacity != 0;
  if (any_capacity && (!d_idx_out || !d_val_out || !is_aligned(d_idx_out, 4) || !is_aligned(d_val_out, es)))
    return DCT_ERR_INVALID;
  const BtLayout l = bt_layout(n_seg, tiles);
  if (!d_ws || !is_aligned(d_ws, 256) || ws_bytes < l.total) return DCT_ERR_WORKSPACE;
  char* ws = static_cast<char*>(d_ws);
  auto* d_segs = reinterpret_cast<BtSeg*>(ws + l.segs);
  auto* d_counts = reinterpret_cast<uint64_t*>(ws + l.counts);
  auto* d_offsets = reinterpret_cast<uint64_t*>(ws + l.offsets);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  bt_upload(segs, d_segs, nullptr, 0, s);
  const dim3 tgrid(static_cast<uint32_t>(tiles)), block(kBtThreads);

#define DCT_LAUNCH_BATCHED(DTV, EX)                                                                              \
  do {                                                                                                           \
    using W = Elem<DTV>::word_t;                                                                                 \
    hipLaunchKernelGGL((bt_count_kernel<DTV, EX>), tgrid, block, 0, s, static_cast<const W*>(g), d_segs, n_seg,  \
                       d_thr, d_counts);                                                                         \
    hipLaunchKernelGGL((bt_scan_kernel<EX>), dim3(n_seg), block, 0, s, d_segs, d_thr, d_counts,                  \
                       d_offsets, d_count_out);                                                                  \
    hipLaunchKernelGGL((bt_write_kernel<DTV, EX>), tgrid, block, 0, s, static_cast<const W*>(g), d_segs, n_seg,  \
                       d_thr, d_offsets, d_idx_out, static_cast<W*>(d_val_out));                                 \
  } while (0)
  if (dt == DCT_F32) {
    if (mode == DCT_EXACT_K) DCT_LAUNCH_BATCHED(DCT_F32, true); else DCT_LAUNCH_BATCHED(DCT_F32, false);
  } else {
    if (mode == DCT_EXACT_K) DCT_LAUNCH_BATCHED(DCT_BF16, true); else DCT_LAUNCH_BATCHED(DCT_BF16, false);
  }
#undef DCT_LAUNCH_BATCHED
  return launch_status();
}
