// dct_select_threshold: Algorithm 1, "sort |W_grad|; tau = w_floor(N*eta)",
// computed exactly as the k-th largest key WITHOUT sorting or copying the
// gradient (the copy-and-sort routine is what Sec. 3.3 measures as the cost of
// recomputing the threshold every iteration).
//
// The exact part is a radix select over the key bits, most significant digit
// first (11 + 11 + 9 bits for fp32, 8 + 7 for bf16): each pass histograms one
// digit of the keys that match the digits fixed so far (LDS histogram per
// workgroup, merged into one in the workspace), and after a grid barrier every
// workgroup walks the merged histogram from the top bin down to find the bin of the
// k-th largest key.  All passes run in one launch.
//
// For large vectors the radix passes do not run over the vector.  A first kernel
// gathers a stratified sample of 16384 keys, a second one brackets two of its
// order statistics to get bounds lo <= tau <= hi that hold with overwhelming
// probability.  One streaming pass over the vector (coalesced 16-byte loads, one
// workgroup of 16 wavefronts per CU, pieces of 8 KiB taken from a counter in LDS)
// counts the keys above hi and appends the keys in [lo, hi] --
// well under 1 % of the vector -- to a candidate buffer (64 regions, each with its own
// counter) through LDS staging.  The
// radix passes then run over the candidates only, so the vector is read from HBM
// once.  The counts tell exactly whether the bounds held (n_above < k <= n_above
// + n_candidates) and whether the buffer had room.  If it overflowed (ties by the
// million at tau) the radix passes run over the keys of the VECTOR that lie in
// [lo, hi], few distinct values that one pass usually resolves; if the bounds did
// not hold they run over the whole vector.  Either way this is decided on the
// device and the result is always the exact order statistic.  All arithmetic is
// on integers.
//
// With error feedback (Algorithm 1, "W_grad = W_grad + E_grad" precedes the
// sort) the EF variants of the kernels that read the vector read g and the
// residual e together and select on w = g + e, one fp32 addition per element,
// without storing w: dct_ef_threshold_compact forms the same sums again.
#include <algorithm>

#include "dct_common.hpp"
#include "radix_select.hpp"

namespace dct {
namespace {

constexpr int kSelMaxPasses = 3;
constexpr int kSelUnroll = 4;                   // 16-byte loads in flight per lane in the radix passes
constexpr int kTailThreads = 1024;                // the kernel of the radix passes: few, large workgroups
constexpr uint32_t kTailMaxGrid = 256;
constexpr uint32_t kTailWaiters = 64;              // workgroups of a launch that may wait at a grid barrier
constexpr int kTailKeep = 8;                      // 16-byte vectors of candidates per thread kept in registers

constexpr uint64_t kSampleMinN = 1ull << 22;    // below this the radix passes run over the vector itself
constexpr int kSampleThreads = 1024;
constexpr uint32_t kSampleSize = 16384;         // 64 KiB of LDS
constexpr int kGatherThreads = 256;
constexpr int kPartThreads = 1024;              // the partition pass: the CU's 16 wavefronts form one workgroup
constexpr int kPartWaves = kPartThreads / kWave;
constexpr int kPartRowsLarge = 8;               // 16-byte loads per lane per piece (two input streams: half of it each)
constexpr int kPartRowsSmall = 4;               // below 2^26 elements, where a wavefront gets only a few pieces
constexpr uint32_t kPartStage = 1024;           // staged candidate keys per wavefront

// The candidate buffer is cut into kCandRegions regions with a counter each: workgroup w of the
// partition pass appends to region w % kCandRegions.  (All workgroups finish together; their end-of-chunk
// reservations on ONE counter serialised and cost the pass a tenth of its time.)
constexpr uint32_t kCandRegions = 64;
struct alignas(128) RegionCount {
  unsigned long long c;  // keys > hi seen by the region's workgroups (high word), keys in [lo, hi] they appended
                         // (low word; may exceed the region)
  uint32_t pad[30];      // a 128-byte line of its own
};
struct SelWs {
  RegionCount counts[kCandRegions];
  uint32_t lo, hi;     // bounds from the sample
  uint32_t sampled;    // 1 when the sample / partition kernels ran
  uint32_t cand_cap;   // capacity of the whole candidate buffer, a multiple of 4 * kCandRegions keys
  uint32_t bar[kSelMaxPasses];  // workgroups that have merged their histogram of pass p
  uint32_t pad;
  uint32_t hist[kSelMaxPasses][kSelBins];
  uint32_t sample[kSampleSize];       // keys of the stratified sample
  uint32_t cand[4];    // candidate keys follow (cand_cap of them, region r at r * cand_cap / kCandRegions)
};
static_assert(offsetof(SelWs, cand) % 16 == 0, "candidate regions are read as 16-byte vectors");

struct PassDigits {
  int n_pass;
  int shift[kSelMaxPasses];
  int width[kSelMaxPasses];
};
__host__ __device__ inline PassDigits pass_digits(int dt) {
  PassDigits d;
  if (dt == DCT_F32) {
    d.n_pass = 3;
    d.shift[0] = 20; d.shift[1] = 9; d.shift[2] = 0;
    d.width[0] = 11; d.width[1] = 11; d.width[2] = 9;
  } else {
    d.n_pass = 2;
    d.shift[0] = 7; d.shift[1] = 0; d.shift[2] = 0;
    d.width[0] = 8; d.width[1] = 7; d.width[2] = 0;
  }
  return d;
}

// Element i of the vector the selection runs on: g, or g + e with error feedback.
template <int DT, bool EF>
__device__ __forceinline__ uint32_t elem_raw(const typename Elem<DT>::word_t* g, const typename Elem<DT>::word_t* e,
                                             uint64_t i) {
  if constexpr (EF) {
    return __float_as_uint(__uint_as_float(g[i]) + __uint_as_float(e[i]));
  } else {
    return static_cast<uint32_t>(g[i]);
  }
}
// Four fp32 sums (error feedback only).
__device__ __forceinline__ uint4 add4(const uint4& a, const uint4& b) {
  return make_uint4(__float_as_uint(__uint_as_float(a.x) + __uint_as_float(b.x)),
                    __float_as_uint(__uint_as_float(a.y) + __uint_as_float(b.y)),
                    __float_as_uint(__uint_as_float(a.z) + __uint_as_float(b.z)),
                    __float_as_uint(__uint_as_float(a.w) + __uint_as_float(b.w)));
}

// ------------------------------------------------------------------ kernel 1a
// Clears the workspace for the direct (no sample) path.
__global__ void select_init_kernel(SelWs* ws) {
  uint32_t* w = reinterpret_cast<uint32_t*>(ws);
  const uint32_t n_words = offsetof(SelWs, sample) / 4;
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += gridDim.x * blockDim.x) w[i] = 0;
}

// ------------------------------------------------------------------ kernel 1b
// Clear the workspace and gather a stratified sample of the keys: stratum i covers
// [i*n/S, (i+1)*n/S) and contributes one key at a hashed offset.  One key per
// thread, spread over many CUs (a single CU cannot keep enough scattered loads in
// flight).
template <int DT, bool EF>
__global__ __launch_bounds__(kGatherThreads) void select_gather_kernel(
    const typename Elem<DT>::word_t* __restrict__ g, const typename Elem<DT>::word_t* __restrict__ e, uint32_t n,
    SelWs* ws) {
  const uint32_t i = blockIdx.x * kGatherThreads + threadIdx.x;  // the grid has exactly kSampleSize threads
  const uint32_t stratum = n / kSampleSize;                      // >= 256 by the choice of kSampleMinN
  const uint64_t start = static_cast<uint64_t>(i) * n / kSampleSize;
  const uint32_t h = (i * 2654435761u) ^ ((i * 40503u) >> 7);
  const uint32_t raw = elem_raw<DT, EF>(g, e, start + h % stratum);
  uint32_t* w = reinterpret_cast<uint32_t*>(ws);
  const uint32_t n_words = offsetof(SelWs, sample) / 4;
  if (i < n_words) w[i] = 0;
  ws->sample[i] = raw & Elem<DT>::kKeyMask;
}
static_assert(offsetof(SelWs, sample) / 4 <= kSampleSize, "the gather grid also clears the workspace header");

// ------------------------------------------------------------------ kernel 1c
// One workgroup: select two order statistics of the sample as bounds for tau.
template <int DT>
__global__ __launch_bounds__(kSampleThreads) void select_bounds_kernel(uint32_t n, uint32_t k, SelWs* ws,
                                                                       uint32_t cand_cap) {
  using E = Elem<DT>;
  __shared__ uint32_t s_keys[kSampleSize];
  __shared__ uint32_t s_hist[2 * kSelBins];
  __shared__ uint32_t s_tmp[kSampleThreads / kWave + 4];
  const uint32_t t = threadIdx.x;
  {
    const uint4* src = reinterpret_cast<const uint4*>(ws->sample);
    uint4* dst = reinterpret_cast<uint4*>(s_keys);
    for (uint32_t i = t; i < kSampleSize / 4; i += kSampleThreads) dst[i] = src[i];
  }
  __syncthreads();

  // sample ranks (1-based from the top) that bracket rank k of the vector with a
  // margin of five standard deviations of the sample count (binomial: r (S - r) / S), plus slack
  const uint64_t r = static_cast<uint64_t>(k) * kSampleSize / n;
  const uint64_t var = r * (kSampleSize - r) / kSampleSize;
  uint32_t sq = 0;
  while (static_cast<uint64_t>(sq + 1) * (sq + 1) <= var) ++sq;
  const uint64_t delta = 5ull * (sq + 1) + 8;
  const uint64_t rank_hi = r > delta ? r - delta : 0;                     // 0: no upper bound
  const uint64_t rank_lo = r + delta + 1 <= kSampleSize ? r + delta + 1 : 0;  // 0: no lower bound

  // Both order statistics are searched together: while their fixed digits agree
  // (the usual case until the last pass) one histogram serves both.
  // The bounds only have to bracket tau, so the digits below the second pass are not
  // resolved: lo takes zeros there and hi ones (a relative widening of 2^-14 for fp32).
  const PassDigits dg = pass_digits(DT);
  const int n_pass = dg.n_pass < 2 ? dg.n_pass : 2;
  const uint32_t rank[2] = {static_cast<uint32_t>(rank_hi), static_cast<uint32_t>(rank_lo)};
  uint32_t prefix[2] = {0, 0}, k_rem[2] = {rank[0], rank[1]};
  uint32_t fixed_mask = 0;
  for (int p = 0; p < n_pass; ++p) {
    const int shift = dg.shift[p];
    const uint32_t dmask = (1u << dg.width[p]) - 1u;
    const bool shared = rank[0] != 0 && rank[1] != 0 && prefix[0] == prefix[1];  // uniform
    for (uint32_t i = t; i < 2 * kSelBins; i += kSampleThreads) s_hist[i] = 0;
    __syncthreads();
    for (uint32_t i = t; i < kSampleSize; i += kSampleThreads) {
      const uint32_t key = s_keys[i];
      const uint32_t digit = (key >> shift) & dmask;
      if (rank[0] != 0) hist_add(s_hist, (key & fixed_mask) == prefix[0], digit);
      if (rank[1] != 0 && !shared) hist_add(s_hist + kSelBins, (key & fixed_mask) == prefix[1], digit);
    }
    __syncthreads();
    for (int which = 0; which < 2; ++which) {
      if (rank[which] == 0) continue;  // uniform
      const uint32_t* hsel = (which == 1 && !shared) ? s_hist + kSelBins : s_hist;
      const BinHit hit = find_bin<kSampleThreads>([&](uint32_t b) { return hsel[b]; }, k_rem[which], s_tmp);
      prefix[which] |= hit.bin << shift;
      k_rem[which] -= hit.above;
    }
    fixed_mask |= dmask << shift;
  }
  const uint32_t open_bits = E::kKeyMask & ~fixed_mask;
  const uint32_t bound[2] = {rank[0] != 0 ? (prefix[0] | open_bits) : E::kKeyMask,
                             rank[1] != 0 ? prefix[1] : 0u};  // {hi, lo}
  if (t == 0) {
    ws->hi = bound[0];
    ws->lo = bound[1];
    ws->sampled = 1;
    ws->cand_cap = cand_cap;
  }
}

// ------------------------------------------------------------------ kernel 2
// Streaming partition pass: count keys > hi, append keys in [lo, hi] to the
// candidate buffer.  One workgroup per CU.  Its share of the vector are blocks of 16 consecutive
// pieces of 8 KiB, one block in every stripe of the grid, so that the grid as a whole reads one
// moving window; its 16 wavefronts take these pieces one at a time from a counter in LDS.  (A SIMD
// serves its oldest wavefront first.  With the pieces dealt out in advance -- 2048 workgroups of 4
// wavefronts, 8 per CU -- the first workgroup of every CU had finished its share after 60 us and the
// eighth after 150 us, and the last third of the pass ran with too few loads in flight: 170 us
// against 160 us now.)  Candidates are staged in LDS per wavefront and written to the workgroup's
// region of the buffer with one slot reservation per workgroup at the end (and one per wavefront
// whenever its staging area fills up before that).  Their order is irrelevant: only the multiset of
// keys matters.
struct PartGeom {
  uint32_t head, n_vec, tail, grid;
};

template <int DT, bool EF, int PR>
__global__ __launch_bounds__(kPartThreads) void select_partition_kernel(
    const typename Elem<DT>::word_t* __restrict__ g, const typename Elem<DT>::word_t* __restrict__ e, PartGeom geo,
    SelWs* ws) {
  static_assert(!EF || DT == DCT_F32, "error feedback is an fp32 addition");
  using E = Elem<DT>;
  constexpr int V = E::kVec;
  constexpr int ROWS = EF ? PR / 2 : PR;  // rows of 64 vectors per piece
  constexpr uint32_t PIECE = ROWS * kWave;               // vectors per piece
  __shared__ uint32_t s_stage[kPartWaves][kPartStage];
  __shared__ uint32_t s_taken;
  const uint32_t lane = lane_id();
  const int wave = threadIdx.x / kWave;
  const uint32_t wg = blockIdx.x;
  const uint32_t lo = ws->lo, hi = ws->hi;
  const uint32_t region_cap = ws->cand_cap / kCandRegions;
  unsigned long long* region_count = &ws->counts[wg % kCandRegions].c;
  uint32_t* region_keys = ws->cand + static_cast<size_t>(wg % kCandRegions) * region_cap;
  uint32_t* stage = s_stage[wave];
  uint32_t staged = 0, above = 0;
  __shared__ uint32_t s_cnt[kPartWaves], s_abv[kPartWaves], s_base;
  if (threadIdx.x == 0) s_taken = 0;
  __syncthreads();

  // Mid-chunk flush of one wavefront's staging region (only when it fills up).
  auto flush = [&]() {
    if (staged == 0) return;
    uint32_t base = 0;
    if (lane == 0) base = static_cast<uint32_t>(atomicAdd(region_count, static_cast<unsigned long long>(staged)));
    base = __builtin_amdgcn_readfirstlane(base);
    for (uint32_t i = lane; i < staged; i += kWave)
      if (base + i < region_cap) region_keys[base + i] = stage[i];
    staged = 0;
  };
  // NE keys per lane
  auto take = [&](const uint32_t* raw, bool in, auto ne_tag) {
    constexpr int NE = decltype(ne_tag)::value;
    // one compare per element in the common case: keys >= lo are rare (per-lane bitmap)
    uint32_t ge_bits = 0;
#pragma unroll
    for (int e = 0; e < NE; ++e) ge_bits |= (raw[e] & E::kKeyMask) >= lo ? (1u << e) : 0u;
    if (!in) ge_bits = 0;
    const uint64_t m_any = ballot64(ge_bits != 0);
    if (m_any == 0) return;
    uint32_t hi_bits = 0;
#pragma unroll
    for (int e = 0; e < NE; ++e) hi_bits |= (raw[e] & E::kKeyMask) > hi ? (1u << e) : 0u;
    hi_bits &= ge_bits;
    const uint32_t c_bits = ge_bits & ~hi_bits;  // candidates: lo <= key <= hi
    // counts of the row and the candidates in lower lanes: a ballot when no lane holds two
    // keys >= lo (the usual case), else one wave scan of the packed per-lane counts
    uint32_t n_c, before;
    if (ballot64((ge_bits & (ge_bits - 1)) != 0) == 0) {
      const uint64_t m_c = ballot64(c_bits != 0);
      n_c = static_cast<uint32_t>(__popcll(m_c));
      above += static_cast<uint32_t>(__popcll(m_any)) - n_c;
      before = lanes_below(m_c);
    } else {
      const uint32_t mine = __popc(hi_bits) | (__popc(c_bits) << 16);
      const uint32_t incl = wave_prefix_sum(mine);
      const uint32_t total = __builtin_amdgcn_readlane(incl, kWave - 1);
      above += total & 0xFFFFu;
      n_c = total >> 16;
      before = (incl - mine) >> 16;
    }
    if (n_c != 0) {
      if (staged + n_c > kPartStage) flush();  // n_c <= 64 * NE <= 512 <= kPartStage
      if (c_bits != 0) {
        uint32_t slot = staged + before;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
          if ((c_bits >> e) & 1u) stage[slot++] = raw[e] & E::kKeyMask;
        }
      }
      staged += n_c;
    }
  };

  // Pieces of ROWS rows of 64 vectors.  The workgroup's pieces are blocks of 16 consecutive ones, one block
  // in every stripe of gridDim.x blocks (the grid reads one moving window of the vector; order is irrelevant
  // here); its wavefronts take them one at a time from a counter in LDS.
  const uint4* gv = reinterpret_cast<const uint4*>(g + geo.head);
  const uint4* ev = EF ? reinterpret_cast<const uint4*>(e + geo.head) : nullptr;
  const uint32_t pieces = (geo.n_vec + PIECE - 1) / PIECE;
  if (wg == 0 && wave == 0 && geo.head != 0) {
    const bool in = lane < geo.head;
    const uint32_t raw = in ? elem_raw<DT, EF>(g, e, lane) : 0u;
    take(&raw, in, std::integral_constant<int, 1>{});
  }
  if (wg == 0 && wave == 1 && geo.tail != 0) {
    const bool in = lane < geo.tail;
    const uint32_t raw = in ? elem_raw<DT, EF>(g, e, geo.head + geo.n_vec * V + lane) : 0u;
    take(&raw, in, std::integral_constant<int, 1>{});
  }
  constexpr uint32_t kNoPiece = 0xFFFFFFFFu;
  const uint32_t stripe = gridDim.x * kPartWaves;
  auto take_piece = [&]() -> uint32_t {
    uint32_t n = 0;
    if (lane == 0) n = atomicAdd(&s_taken, 1u);
    n = __builtin_amdgcn_readfirstlane(n);
    const uint64_t p = static_cast<uint64_t>(wg) * kPartWaves + (n % kPartWaves) + static_cast<uint64_t>(n / kPartWaves) * stripe;
    return p < pieces ? static_cast<uint32_t>(p) : kNoPiece;  // increasing in n: nothing follows a piece past the end
  };
  // Two register buffers: the next piece's loads are in flight while the current one is processed.
  struct Rows {
    uint4 a[ROWS];
    uint4 b[EF ? ROWS : 1];
  };
  auto load_piece = [&](Rows& buf, uint32_t p) {
    const uint32_t vec0 = p * PIECE + lane;
    if ((p + 1) * PIECE <= geo.n_vec) {  // uniform
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        buf.a[r] = ld_stream(&gv[vec0 + r * kWave]);
        if constexpr (EF) buf.b[r] = ld_stream(&ev[vec0 + r * kWave]);
      }
    } else {
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        const uint32_t vi = vec0 + r * kWave;
        buf.a[r] = vi < geo.n_vec ? gv[vi] : make_uint4(0, 0, 0, 0);
        if constexpr (EF) buf.b[r] = vi < geo.n_vec ? ev[vi] : make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto process_piece = [&](const Rows& buf, uint32_t p) {
    const uint32_t vec0 = p * PIECE + lane;
    const bool full = (p + 1) * PIECE <= geo.n_vec;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
      uint4 v = buf.a[r];
      if constexpr (EF) v = add4(v, buf.b[r]);
      uint32_t raw[V];
#pragma unroll
      for (int i = 0; i < V; ++i) raw[i] = E::raw(v, i);
      take(raw, full || vec0 + r * kWave < geo.n_vec, std::integral_constant<int, V>{});
    }
  };
  {
    Rows va, vb;
    uint32_t p = take_piece();
    if (p != kNoPiece) load_piece(va, p);
    while (p != kNoPiece) {
      uint32_t q = take_piece();
      if (q != kNoPiece) load_piece(vb, q);
      process_piece(va, p);
      if (q == kNoPiece) break;
      p = take_piece();
      if (p != kNoPiece) load_piece(va, p);
      process_piece(vb, q);
    }
  }
  // end of the chunk: one reservation for the whole workgroup (both counts in one 64-bit add)
  if (lane == 0) {
    s_cnt[wave] = staged;
    s_abv[wave] = above;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t c = 0, a = 0;
    for (int w = 0; w < kPartWaves; ++w) {
      c += s_cnt[w];
      a += s_abv[w];
    }
    uint32_t base = 0;
    if (c != 0 || a != 0)
      base = static_cast<uint32_t>(atomicAdd(region_count, (static_cast<unsigned long long>(a) << 32) | c));
    s_base = base;
  }
  __syncthreads();
  uint32_t base = s_base;
  for (int w = 0; w < wave; ++w) base += s_cnt[w];
  for (uint32_t i = lane; i < staged; i += kWave)
    if (base + i < region_cap) region_keys[base + i] = stage[i];
}

// ------------------------------------------------------------------ kernel 3
// Vector vi of a candidate region that holds n_src keys, as the candidate passes use it: key - lo for
// the keys (below 2^31), all ones for the slots past the region's end (they match no prefix).
__device__ __forceinline__ uint4 offset_keys(const uint4& v, uint32_t vi, uint32_t n_src, uint32_t lo_key) {
  const uint32_t n_valid = n_src > vi * 4u ? n_src - vi * 4u : 0u;
  return make_uint4(n_valid > 0u ? v.x - lo_key : 0xFFFFFFFFu, n_valid > 1u ? v.y - lo_key : 0xFFFFFFFFu,
                    n_valid > 2u ? v.z - lo_key : 0xFFFFFFFFu, n_valid > 3u ? v.w - lo_key : 0xFFFFFFFFu);
}

__device__ __forceinline__ uint32_t add_agent(uint32_t* p, uint32_t v) {
  return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The radix passes and the result, in one launch.  Every workgroup derives the search state
// (from the partition counts at first, from the merged histogram after each pass), histograms
// its part of the source in LDS and adds the non-empty bins to the pass's histogram in the
// workspace; a grid barrier (an arrival counter polled with agent-scope loads) separates a pass
// from the search in its histogram, which every workgroup repeats for itself.  The grid is
// small enough to be resident as a whole; a workgroup that waits longer than about a second
// gives up (spin_limit polls) and stores DCT_TAU_KEY_ERROR in the result.
// After the last pass there is no barrier: the workgroup that arrives last finishes alone.
//
// Merging costs more than reading here: after the subtraction of lo the candidates fill most of
// the 2048 bins of the first digit, every workgroup adds most of its bins, and the device
// sustains some 40 G such adds a second (256 workgroups x 2048 bins: 13 us).  The candidate
// passes are therefore left to one workgroup per region (64 of them, 1024 threads each; the
// others leave at once), and what then limits them is one CU's instruction rate: about 27
// keys per thread on c4, held in registers from the first pass on and tested with two
// instructions per key and pass.  On c4 the kernel takes 25 us, against 26 us for the
// three pass kernels and the finishing kernel it replaced, and 43 us less on c3, whose
// larger grids spent their time merging.
template <int DT, bool EF>
__global__ __launch_bounds__(kTailThreads) void select_tail_kernel(
    const typename Elem<DT>::word_t* __restrict__ g_al, const typename Elem<DT>::word_t* __restrict__ e_al,
    uint32_t off, uint32_t n_virt, uint32_t k, SelWs* ws, int n_pass, uint32_t spin_limit,
    dct_threshold* __restrict__ out) {
  static_assert(!EF || DT == DCT_F32, "error feedback is an fp32 addition");
  using E = Elem<DT>;
  constexpr int V = E::kVec;
  __shared__ uint32_t h[kSelBins];
  __shared__ uint32_t s_tmp[kTailThreads / kWave + 4];
  __shared__ uint32_t s_tot[3];
  __shared__ uint32_t s_arrived;
  const uint32_t span = kTailThreads * kSelUnroll;  // vectors per workgroup per iteration
  const uint32_t region_cap = ws->cand_cap / kCandRegions;

  // The head of the candidate region this workgroup will read (if it reads candidates at all) is
  // requested before anything else and stays in registers for all passes: kTailKeep vectors per
  // thread, which is the whole region unless the bounds were wide.  (No partition pass: the
  // counters are zero and nothing is loaded.)
  const uint32_t lo_key = ws->lo;
  uint32_t cnt0 = 0;
  uint4 keep[kTailKeep];
  {
    const uint32_t region0 = blockIdx.x % kCandRegions;
    if (blockIdx.x < kCandRegions) cnt0 = min(static_cast<uint32_t>(ws->counts[region0].c), region_cap);
    const uint4* cv = reinterpret_cast<const uint4*>(ws->cand + static_cast<size_t>(region0) * region_cap);
    const uint32_t vecs0 = (cnt0 + 3) / 4;
#pragma unroll
    for (int u = 0; u < kTailKeep; ++u) {
      const uint32_t vi = u * kTailThreads + threadIdx.x;
      keep[u] = vi < vecs0 ? cv[vi] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kTailKeep; ++u) keep[u] = offset_keys(keep[u], u * kTailThreads + threadIdx.x, cnt0, lo_key);
  }

  // ---- search state before the first pass
  SelState st;
  uint32_t range_lo, range_span;  // the keys that take part: range_lo <= key <= range_lo + range_span
  {
    // totals of the partition pass over the regions (one counter per lane of the first wavefront;
    // all zero when no partition pass ran)
    if (threadIdx.x < kWave) {
      static_assert(kCandRegions == kWave, "one region counter per lane");
      const unsigned long long c = ws->counts[threadIdx.x].c;
      const uint32_t a_sum = wave_sum_u32(static_cast<uint32_t>(c >> 32));
      const uint32_t c_sum = wave_sum_u32(static_cast<uint32_t>(c));  // < 2^31: every key is counted at most once
      const bool over = ballot64(static_cast<uint32_t>(c) > region_cap) != 0;
      if (threadIdx.x == 0) {
        s_tot[0] = a_sum;
        s_tot[1] = c_sum;
        s_tot[2] = over ? 1u : 0u;
      }
    }
    __syncthreads();
    const uint32_t n_above = s_tot[0], n_cand = s_tot[1];  // keys > hi, keys in [lo, hi] (also those that found no room)
    // Three cases.  The bounds held and the candidate buffer has all keys in [lo, hi]: select among the
    // candidates.  The bounds held but the buffer overflowed (ties by the million at tau, as in a mostly
    // zero gradient with k beyond its non-zeros): select among the keys of the VECTOR that lie in
    // [lo, hi], which are few distinct values -- usually one pass.  The bounds failed: select among all keys.
    const bool held = ws->sampled != 0 && n_above < k && k <= n_above + n_cand;
    st.k_rem = held ? k - n_above : k;
    st.n_gt = held ? n_above : 0u;
    st.from_cand = held && s_tot[2] == 0 ? 1u : 0u;
    st.n_src = held ? n_cand : n_virt - off;
    st.last_count = st.n_src;
    // In the first two cases the passes select on key - lo, which lies in [0, hi - lo]: only the bits of that
    // range are left to resolve (the bits in which lo and hi differ can be many more, when a carry separates them).
    range_lo = held ? lo_key : 0u;
    range_span = held ? ws->hi - lo_key : E::kKeyMask;
    st.rem_bits = range_span ? 32u - __builtin_clz(range_span) : 0u;
    st.prefix = 0u;
    st.width = min(kDigitBits, st.rem_bits);
  }
  // Workgroups that take part (the same number in every workgroup's view: it decides the barriers).
  // Only a pass that another pass follows ends in a barrier where workgroups WAIT; at most kTailWaiters
  // workgroups, the first of the grid, ever do, so that several selections at a time (one per hardware
  // queue) still find room for all their waiters.  After the last pass nobody waits: the workgroup that
  // arrives last finishes the job alone.  A single pass over the vector may therefore use the whole grid.
  const uint32_t src_vecs = n_virt / V + 1;
  const uint32_t n_active =
      st.from_cand ? min(gridDim.x, kCandRegions)
                   : min(st.rem_bits <= kDigitBits ? gridDim.x : min(gridDim.x, kTailWaiters), (src_vecs + span - 1) / span);
  if (blockIdx.x >= n_active) return;
  bool finisher = blockIdx.x == 0;  // writes the result

  for (int pass = 0; pass < n_pass && st.width != 0; ++pass) {  // uniform over the grid
    const uint32_t shift = st.rem_bits - st.width;
    const uint32_t dmask = (1u << st.width) - 1u;
    const uint32_t fixed_all = ~((1u << st.rem_bits) - 1u);  // with bit 31: set in no prefix
    const uint32_t prefix = st.prefix;
    for (int i = threadIdx.x; i < kSelBins; i += kTailThreads) h[i] = 0;
    __syncthreads();

    if (st.from_cand) {
      // candidate keys, a region at a time: u32, 16-byte-aligned, as many as the region's counter says
      // One vector of four offset keys per lane (offset_keys() below).  The digits of candidates differ
      // from lane to lane as a rule (plain LDS adds, after one test whether the wavefront has anything
      // to add at all: in the later passes it rarely has); when every key the wavefront adds falls into
      // ONE bin -- ties -- a single add replaces up to 256 that would serialise.
      // (fixed_all has bit 31, which the fillers past a region's end have set)
      auto add_vec = [&](const uint4& v) {
        const uint32_t key[4] = {v.x, v.y, v.z, v.w};
        bool act[4];
        bool any = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          act[e] = (key[e] & fixed_all) == prefix;
          any |= act[e];
        }
        const uint64_t m_any = ballot64(any);
        if (m_any == 0) return;
        // (the empty asm keeps the compiler from computing the digits ahead of the test above, for all the
        // vectors a thread holds: most of a later pass's time went there)
        uint32_t k0 = key[0], k1 = key[1], k2 = key[2], k3 = key[3];
        asm volatile("" : "+v"(k0), "+v"(k1), "+v"(k2), "+v"(k3));
        const uint32_t digit[4] = {(k0 >> shift) & dmask, (k1 >> shift) & dmask, (k2 >> shift) & dmask,
                                   (k3 >> shift) & dmask};
        const uint32_t mine = act[0] ? digit[0] : act[1] ? digit[1] : act[2] ? digit[2] : digit[3];
        const int leader = __builtin_ctzll(m_any);
        const uint32_t d0 = __shfl(mine, leader, kWave);  // a digit that some lane adds
        bool differs = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) differs |= act[e] && digit[e] != d0;
        if (ballot64(differs) == 0) {
          uint32_t total = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) total += static_cast<uint32_t>(__popcll(ballot64(act[e])));
          if (static_cast<int>(lane_id()) == leader) atomicAdd(&h[d0], total);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (act[e]) atomicAdd(&h[digit[e]], 1u);
        }
      };
      for (uint32_t region = blockIdx.x; region < kCandRegions; region += n_active) {
        const uint4* cv = reinterpret_cast<const uint4*>(ws->cand + static_cast<size_t>(region) * region_cap);
        const bool first = region == blockIdx.x;  // its head is in registers
        const uint32_t n_src = first ? cnt0 : static_cast<uint32_t>(ws->counts[region].c);  // <= region_cap here
        const uint32_t reg_vecs = (n_src + 3) / 4;
        if (first) {
#pragma unroll
          for (int u = 0; u < kTailKeep; ++u) add_vec(keep[u]);
        }
        for (uint32_t base = first ? kTailKeep * kTailThreads : 0u; base < reg_vecs; base += span) {
          uint4 v[kSelUnroll];
#pragma unroll
          for (int u = 0; u < kSelUnroll; ++u) {
            const uint32_t vi = base + u * kTailThreads + threadIdx.x;
            v[u] = vi < reg_vecs ? cv[vi] : make_uint4(0, 0, 0, 0);  // a region holds whole vectors
          }
#pragma unroll
          for (int u = 0; u < kSelUnroll; ++u)
            add_vec(offset_keys(v[u], base + u * kTailThreads + threadIdx.x, n_src, lo_key));
        }
      }
    } else {
      // the vector itself.  Vectors [v_lo, v_hi) are entirely inside the data; at most one
      // vector on each side straddles an end and is read element by element by workgroup 0.
      const uint32_t v_lo = off ? 1u : 0u;
      const uint32_t v_hi = n_virt / V;
      const uint4* gv = reinterpret_cast<const uint4*>(g_al);
      const uint4* ev = reinterpret_cast<const uint4*>(e_al);
      for (uint32_t base = v_lo + blockIdx.x * span; base < v_hi; base += n_active * span) {
        uint4 v[kSelUnroll], ve4[EF ? kSelUnroll : 1];
        bool in[kSelUnroll];
#pragma unroll
        for (int u = 0; u < kSelUnroll; ++u) {
          const uint32_t vi = base + u * kTailThreads + threadIdx.x;
          in[u] = vi < v_hi;
          v[u] = in[u] ? gv[vi] : make_uint4(0, 0, 0, 0);
          if constexpr (EF) ve4[u] = in[u] ? ev[vi] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kSelUnroll; ++u) {
          if constexpr (EF) v[u] = add4(v[u], ve4[u]);
#pragma unroll
          for (int e = 0; e < V; ++e) {
            const uint32_t key = (E::raw(v[u], e) & E::kKeyMask) - range_lo;  // below range_lo: wraps past the span
            hist_add(h, in[u] && key <= range_span && (key & fixed_all) == prefix, (key >> shift) & dmask);
          }
        }
      }
      if (blockIdx.x == 0 && threadIdx.x < kWave) {
        // head elements [off, min(V, n_virt)) of a misaligned base, tail elements [v_hi*V, n_virt)
        const uint32_t t = threadIdx.x;
        uint32_t ve = 0xFFFFFFFFu;
        if (t < static_cast<uint32_t>(V)) {
          if (off && t >= off && t < n_virt) ve = t;
        } else if (t < 2u * V) {
          const uint32_t c = v_hi * V + (t - V);
          if (c < n_virt && (c >= static_cast<uint32_t>(V) || !off)) ve = c;
        }
        const bool act = ve != 0xFFFFFFFFu;
        const uint32_t key = (act ? (elem_raw<DT, EF>(g_al, e_al, ve) & E::kKeyMask) : 0u) - range_lo;
        hist_add(h, act && key <= range_span && (key & fixed_all) == prefix, (key >> shift) & dmask);
      }
    }
    __syncthreads();

    // merge, then wait until every workgroup has merged
    uint32_t* gh = ws->hist[pass];
    if (n_active > 1) {
      uint32_t seen = 0;
      for (int i = threadIdx.x; i < kSelBins; i += kTailThreads) {
        const uint32_t c = h[i];
        if (c) seen += add_agent(&gh[i], c);  // the value returned: the addition has been performed
      }
      asm volatile("s_waitcnt vmcnt(0)" ::"v"(seen) : "memory");
      __syncthreads();
      const bool last_pass = st.rem_bits <= st.width;  // uniform over the grid
      if (threadIdx.x == 0) {
        uint32_t arrived = add_agent(&ws->bar[pass], 1u) + 1u;
        if (!last_pass) {
          for (uint32_t spins = 0; arrived < n_active && spins < spin_limit; ++spins) {
            __builtin_amdgcn_s_sleep(2);
            arrived = ld_agent(&ws->bar[pass]);
          }
        }
        s_arrived = arrived;
      }
      __syncthreads();
      if (s_arrived < n_active) {  // uniform
        if (last_pass) return;     // another workgroup arrives last and finishes
        // Somebody never came.  A workgroup that gives up arrives at no later barrier, so no later pass
        // can complete and nobody will write a result: every workgroup that gives up stores the error
        // record itself (the same words from all of them).
        if (threadIdx.x == 0) {
          st_agent(&out->tau_key, DCT_TAU_KEY_ERROR);
          st_agent(&out->n_gt, 0u);
          st_agent(&out->n_eq, 0u);
          st_agent(&out->tie_quota, 0u);
        }
        return;
      }
      if (last_pass) finisher = true;
      st = advance_state_with<kTailThreads>(st, [&](uint32_t b) { return ld_agent(&gh[b]); }, s_tmp);
    } else {
      st = advance_state_with<kTailThreads>(st, [&](uint32_t b) { return h[b]; }, s_tmp);
    }
  }
  if (finisher && threadIdx.x == 0) {
    out->tau_key = st.prefix + range_lo;  // the passes work on key - range_lo
    out->n_gt = st.n_gt;
    out->n_eq = st.last_count;
    out->tie_quota = st.k_rem;
  }
}

// Workgroups of the tail kernel: as many as are resident together (its grid barriers need that), a
// multiple of the region count when there are that many.
template <int DT, bool EF>
uint32_t tail_grid() {
  static const uint32_t per_cu = [] {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, select_tail_kernel<DT, EF>, kTailThreads, 0) != hipSuccess)
      nb = 0;
    return static_cast<uint32_t>(nb > 0 ? nb : 0);
  }();
  const uint64_t resident = static_cast<uint64_t>(per_cu) * static_cast<uint32_t>(device_cu_count());
  uint32_t grid = static_cast<uint32_t>(std::min<uint64_t>(resident, kTailMaxGrid));
  if (grid > kCandRegions) grid -= grid % kCandRegions;
  return grid;
}

// Room for the keys between the sample bounds: about 10 sqrt(p (1 - p) / 16384) of the vector when a
// fraction p is kept, i.e. at most 4 % (p = 1/2).
uint32_t cand_capacity(uint64_t n) {
  return n >= kSampleMinN ? static_cast<uint32_t>(n / 16 + 65536) & ~(4u * kCandRegions - 1u) : 0u;
}

}  // namespace
}  // namespace dct

using namespace dct;

extern "C" size_t dct_select_threshold_workspace_bytes(int dt, uint64_t n) {
  if ((dt != DCT_F32 && dt != DCT_BF16) || n == 0 || n > 0x7FFFFFFFull) return 0;
  return sizeof(SelWs) + static_cast<size_t>(cand_capacity(n)) * 4;
}

namespace {

int launch_select(const void* g, const void* e, int dt, uint64_t n, uint64_t k, dct_threshold* d_thr_out, void* d_ws,
                  size_t ws_bytes, void* hip_stream) {
  const bool ef = e != nullptr;
  if (!g || !d_thr_out || n == 0 || n > 0x7FFFFFFFull || k == 0 || k > n) return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(g, es) || !is_aligned(d_thr_out, 16)) return DCT_ERR_INVALID;
  const uintptr_t addr = reinterpret_cast<uintptr_t>(g);
  const uintptr_t eaddr = reinterpret_cast<uintptr_t>(e);
  // both vectors are walked with the same 16-byte vectors: same offset within 16 bytes
  if (ef && (dt != DCT_F32 || !is_aligned(e, es) || (eaddr & 15) != (addr & 15))) return DCT_ERR_INVALID;
  const uint32_t cand_cap = cand_capacity(n);
  if (!d_ws || !is_aligned(d_ws, 256) || ws_bytes < sizeof(SelWs) + static_cast<size_t>(cand_cap) * 4)
    return DCT_ERR_WORKSPACE;

  const int vec = dt == DCT_F32 ? 4 : 8;
  auto* ws = static_cast<SelWs*>(d_ws);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint32_t n32 = static_cast<uint32_t>(n), k32 = static_cast<uint32_t>(k);
  const auto* g32 = static_cast<const uint32_t*>(g);
  const auto* e32 = static_cast<const uint32_t*>(e);
  const auto* g16 = static_cast<const uint16_t*>(g);

  if (cand_cap != 0) {
    // sample -> bounds, then the streaming partition pass
    PartGeom geo;
    uint64_t head = ((16 - (addr & 15)) & 15) / es;
    if (head > n) head = n;
    geo.head = static_cast<uint32_t>(head);
    geo.n_vec = static_cast<uint32_t>((n - head) / vec);
    geo.tail = static_cast<uint32_t>((n - head) % vec);
    // pieces of 8 KiB, of 4 KiB for vectors of which a wavefront would get only a few of those
    // (2^28 elements: 197 against 206 us; 25 M elements: 53.2 against 50.8 us)
    const bool large = n >= (1ull << 26);
    const uint32_t block_vecs = kWave * (large ? kPartRowsLarge : kPartRowsSmall) * kPartWaves;
    uint32_t blocks = (geo.n_vec + block_vecs - 1) / block_vecs;
    if (blocks == 0) blocks = 1;
    const uint32_t max_grid = static_cast<uint32_t>(device_cu_count());
    geo.grid = blocks < max_grid ? blocks : max_grid;
    const dim3 ggrid(kSampleSize / kGatherThreads), gblock(kGatherThreads), pgrid(geo.grid), pblock(kPartThreads);
    if (ef) {
      hipLaunchKernelGGL((select_gather_kernel<DCT_F32, true>), ggrid, gblock, 0, s, g32, e32, n32, ws);
      hipLaunchKernelGGL((select_bounds_kernel<DCT_F32>), dim3(1), dim3(kSampleThreads), 0, s, n32, k32, ws, cand_cap);
      if (large) hipLaunchKernelGGL((select_partition_kernel<DCT_F32, true, kPartRowsLarge>), pgrid, pblock, 0, s, g32, e32, geo, ws);
      else hipLaunchKernelGGL((select_partition_kernel<DCT_F32, true, kPartRowsSmall>), pgrid, pblock, 0, s, g32, e32, geo, ws);
    } else if (dt == DCT_F32) {
      hipLaunchKernelGGL((select_gather_kernel<DCT_F32, false>), ggrid, gblock, 0, s, g32, nullptr, n32, ws);
      hipLaunchKernelGGL((select_bounds_kernel<DCT_F32>), dim3(1), dim3(kSampleThreads), 0, s, n32, k32, ws, cand_cap);
      if (large) hipLaunchKernelGGL((select_partition_kernel<DCT_F32, false, kPartRowsLarge>), pgrid, pblock, 0, s, g32, nullptr, geo, ws);
      else hipLaunchKernelGGL((select_partition_kernel<DCT_F32, false, kPartRowsSmall>), pgrid, pblock, 0, s, g32, nullptr, geo, ws);
    } else {
      hipLaunchKernelGGL((select_gather_kernel<DCT_BF16, false>), ggrid, gblock, 0, s, g16, nullptr, n32, ws);
      hipLaunchKernelGGL((select_bounds_kernel<DCT_BF16>), dim3(1), dim3(kSampleThreads), 0, s, n32, k32, ws, cand_cap);
      if (large) hipLaunchKernelGGL((select_partition_kernel<DCT_BF16, false, kPartRowsLarge>), pgrid, pblock, 0, s, g16, nullptr, geo, ws);
      else hipLaunchKernelGGL((select_partition_kernel<DCT_BF16, false, kPartRowsSmall>), pgrid, pblock, 0, s, g16, nullptr, geo, ws);
    }
  } else {
    hipLaunchKernelGGL(select_init_kernel, dim3(32), dim3(256), 0, s, ws);
  }
  if (hipGetLastError() != hipSuccess) return DCT_ERR_HIP;

  // radix passes (over the candidates, or over the vector: decided on the device) and the result
  const uint32_t off = static_cast<uint32_t>((addr & 15) / es);
  const uint32_t n_virt = n32 + off;
  const void* g_al = reinterpret_cast<const void*>(addr & ~static_cast<uintptr_t>(15));
  const void* e_al = reinterpret_cast<const void*>(eaddr & ~static_cast<uintptr_t>(15));
  const PassDigits dg = pass_digits(dt);
  const uint32_t spin_limit = wait_limit();  // polls of a grid barrier (by default about a second) before giving up
  const uint32_t tgrid = ef ? tail_grid<DCT_F32, true>()
                            : dt == DCT_F32 ? tail_grid<DCT_F32, false>() : tail_grid<DCT_BF16, false>();
  if (tgrid == 0) return DCT_ERR_HIP;
  if (ef) {
    hipLaunchKernelGGL((select_tail_kernel<DCT_F32, true>), dim3(tgrid), dim3(kTailThreads), 0, s,
                       static_cast<const uint32_t*>(g_al), static_cast<const uint32_t*>(e_al), off, n_virt, k32, ws,
                       dg.n_pass, spin_limit, d_thr_out);
  } else if (dt == DCT_F32) {
    hipLaunchKernelGGL((select_tail_kernel<DCT_F32, false>), dim3(tgrid), dim3(kTailThreads), 0, s,
                       static_cast<const uint32_t*>(g_al), nullptr, off, n_virt, k32, ws, dg.n_pass, spin_limit,
                       d_thr_out);
  } else {
    hipLaunchKernelGGL((select_tail_kernel<DCT_BF16, false>), dim3(tgrid), dim3(kTailThreads), 0, s,
                       static_cast<const uint16_t*>(g_al), nullptr, off, n_virt, k32, ws, dg.n_pass, spin_limit,
                       d_thr_out);
  }
  return launch_status();
}

}  // namespace

extern "C" int dct_select_threshold(const void* g, int dt, uint64_t n, uint64_t k, dct_threshold* d_thr_out,
                                    void* d_ws, size_t ws_bytes, void* hip_stream) {
  return launch_select(g, nullptr, dt, n, k, d_thr_out, d_ws, ws_bytes, hip_stream);
}

extern "C" int dct_ef_select_threshold(const void* g, const void* e, int dt, uint64_t n, uint64_t k,
                                       dct_threshold* d_thr_out, void* d_ws, size_t ws_bytes, void* hip_stream) {
  if (!e) return DCT_ERR_INVALID;
  return launch_select(g, e, dt, n, k, d_thr_out, d_ws, ws_bytes, hip_stream);
}
