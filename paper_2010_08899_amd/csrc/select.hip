// dct_select_threshold: Algorithm 1, the sort of the magnitudes and the element at rank
// floor(N*eta) taken as tau, computed exactly as the k-th largest key WITHOUT sorting or copying the
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
// gathers a stratified sample of 16384 keys (16 workgroups, one key per thread) and
// its first workgroup, as soon as all keys have arrived, brackets two order
// statistics of the sample to get bounds lo <= tau <= hi that hold with overwhelming
// probability.  One streaming pass over the vector (coalesced 16-byte loads, one
// workgroup of 16 wavefronts per CU, pieces of 8 KiB taken from a counter in LDS)
// counts the keys above hi and appends the keys in [lo, hi] --
// well under 1 % of the vector -- to a candidate buffer (64 regions, each with its own
// counter) through LDS staging; on the way it histograms the candidates' top eight
// bits (of key - lo), which is the first radix pass over them for free.  The
// remaining radix passes run over the candidates only, so the vector is read from HBM
// once.  The counts tell exactly whether the bounds held (n_above < k <= n_above
// + n_candidates) and whether the buffer had room.  If it overflowed (ties by the
// million at tau) the radix passes run over the keys of the VECTOR that lie in
// [lo, hi], few distinct values that one pass usually resolves; if the bounds did
// not hold they run over the whole vector.  Either way this is decided on the
// device and the result is always the exact order statistic.  All arithmetic is
// on integers.
//
// With error feedback (Algorithm 1: the residual is added to the gradient before the
// sort) the EF variants of the kernels that read the vector read g and the
// residual e together and select on w = g + e, one fp32 addition per element,
// without storing w: dct_ef_threshold_compact forms the same sums again.
#include <algorithm>
#include <atomic>
#include <chrono>

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
constexpr uint32_t kSampleSize = 16384;         // keys: 16 per thread of the workgroup that brackets them
constexpr uint32_t kCoarseBits = 8;             // the candidates' top bits that the partition pass histograms
constexpr uint32_t kCoarseBins = 1u << kCoarseBits;
constexpr uint32_t kCoarseCopies = 16;
constexpr uint32_t kFinalCap = 16384;           // candidates that one workgroup finishes on its own (16 per thread)
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
  // cleared by the first kernel of every call
  RegionCount counts[kCandRegions];
  uint32_t bar[kSelMaxPasses];  // workgroups that have merged their histogram of pass p
  uint32_t final_count;         // keys appended to final_keys
  uint32_t final_arrived;       // workgroups that have appended theirs
  uint32_t pad0[3];
  // candidates per value of (key - lo) >> coarse_shift, in kCoarseCopies copies (workgroup w adds to copy
  // w % kCoarseCopies: 256 workgroups adding to one word at the end of the pass take microseconds)
  uint32_t coarse[kCoarseCopies][kCoarseBins];
  uint32_t hist[kSelMaxPasses][kSelBins];
  // written by the first kernel of every call
  uint32_t lo, hi;     // bounds from the sample
  uint32_t sampled;    // 1 when the sample / partition kernels ran
  uint32_t cand_cap;   // capacity of the whole candidate buffer, a multiple of 4 * kCandRegions keys
  // The sample: key | call tag << 32.  The tag tells the workgroup that brackets the sample which words are
  // this call's (the workspace is scratch: nothing in it is assumed on entry, so there is no counter to
  // clear); a word that carries the tag by accident only makes the bounds worse, and bounds are verified.
  uint32_t final_keys[kFinalCap];  // the candidates inside the one coarse bin that holds tau (as key - lo)
  uint64_t sample[kSampleSize];
  uint32_t cand[4];    // candidate keys follow (cand_cap of them, region r at r * cand_cap / kCandRegions)
};
constexpr uint32_t kSelClearWords = offsetof(SelWs, lo) / 4;
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
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < kSelClearWords; i += gridDim.x * blockDim.x) w[i] = 0;
  if (blockIdx.x == 0 && threadIdx.x == 0) ws->sampled = 0;
}

// ------------------------------------------------------------------ kernel 1b
// Clear the workspace, gather a stratified sample of the keys and bracket tau.  Stratum i covers
// [i*n/S, (i+1)*n/S) and contributes one key at a hashed offset: one key per thread, 16 workgroups (a
// single CU cannot keep enough scattered loads in flight).  Every thread publishes its key together with
// the call's tag in one 64-bit word; workgroup 0 collects the 16384 words (16 per thread, polling until all
// carry the tag; bounded) and selects two order statistics of the sample as bounds for tau, two radix passes
// over the keys in its registers.  (Letting the sixteen workgroups histogram the first digit of their own
// keys was tried: fetching their histograms costs workgroup 0 more than the pass it saves.)
static_assert(kSelClearWords <= kSampleSize, "the sample grid also clears the workspace header");
template <int DT, bool EF>
__global__ __launch_bounds__(kSampleThreads) void select_sample_kernel(
    const typename Elem<DT>::word_t* __restrict__ g, const typename Elem<DT>::word_t* __restrict__ e, uint32_t n,
    uint32_t rank_hi, uint32_t rank_lo, SelWs* ws, uint32_t cand_cap, uint32_t tag, uint32_t spin_limit) {
  using E = Elem<DT>;
  constexpr int KPT = kSampleSize / kSampleThreads;  // keys per thread of workgroup 0 = workgroups of the grid
  __shared__ uint32_t s_hist[2 * kSelBins];
  __shared__ uint32_t s_tmp[kSampleThreads / kWave + 4], s_scan_b[kSampleThreads / kWave], s_found[4];
  const uint32_t t = threadIdx.x;
  const PassDigits dg = pass_digits(DT);
  const uint64_t tagged = static_cast<uint64_t>(tag) << 32;
  {
    const uint32_t i = blockIdx.x * kSampleThreads + t;  // the grid has exactly kSampleSize threads
    const uint32_t stratum = n / kSampleSize;            // >= 256 by the choice of kSampleMinN
    const uint64_t start = static_cast<uint64_t>(i) * n / kSampleSize;
    const uint32_t h = (i * 2654435761u) ^ ((i * 40503u) >> 7);
    const uint32_t key = elem_raw<DT, EF>(g, e, start + h % stratum) & E::kKeyMask;
    if (i < kSelClearWords) reinterpret_cast<uint32_t*>(ws)[i] = 0;
    st_agent(&ws->sample[i], tagged | key);
  }
  if (blockIdx.x != 0) return;

  // ---- workgroup 0: the whole sample, 16 keys per thread
  uint32_t keys[KPT];
  {
    bool complete = false;  // uniform
    // The other workgroups' words are on their way for as long as this workgroup's own were: a first look at
    // once would find some missing and cost a whole round of 16 loads per thread.
    __builtin_amdgcn_s_sleep(24);
    for (uint32_t spins = 0; !complete && spins <= spin_limit; ++spins) {
      // (tt: the thread's index, opaque to the compiler, which would otherwise keep every address in
      // registers across the iterations of this loop; and all loads first, then their uses: the loads are
      // ordered accesses, and a use between two of them makes the second wait for the first)
      uint32_t tt = t;
      asm volatile("" : "+v"(tt));
      uint64_t w[KPT];
#pragma unroll
      for (int j = 0; j < KPT; ++j) w[j] = ld_agent(&ws->sample[j * kSampleThreads + tt]);
      bool mine = true;
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        keys[j] = static_cast<uint32_t>(w[j]);
        mine = mine && static_cast<uint32_t>(w[j] >> 32) == tag;
      }
      complete = __syncthreads_and(mine) != 0;
      if (!complete) __builtin_amdgcn_s_sleep(2);
    }
    if (!complete) {  // somebody's words never came: no bounds, the radix passes will run over the vector
      if (t == 0) {
        ws->lo = 0;
        ws->hi = E::kKeyMask;
        ws->sampled = 0;
        ws->cand_cap = cand_cap;
      }
      return;
    }
  }

  // rank_hi, rank_lo: the sample ranks (1-based from the top) that bracket rank k of the vector, from the host
  // (sample_ranks); 0 = no bound on that side.

  // Both order statistics are searched together: while their fixed digits agree
  // (the usual case until the last pass) one histogram serves both.
  // The bounds only have to bracket tau, so the digits below the second pass are not
  // resolved: lo takes zeros there and hi ones (a relative widening of 2^-14 for fp32).
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
    const bool one_hist = shared || rank[0] == 0 || rank[1] == 0;  // uniform
    if (p == 0) {
      // first pass: every key takes part, so the lanes that share lane 0's digit (a mostly zero gradient: all of
      // them) are counted with one ballot and one add, without the search for a leader
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const uint32_t digit = (keys[j] >> shift) & dmask;
        const uint32_t d0 = __builtin_amdgcn_readfirstlane(digit);
        const uint64_t m = ballot64(digit == d0);
        if (lane_id() == 0) atomicAdd(&s_hist[d0], static_cast<uint32_t>(__popcll(m)));
        if (digit != d0) atomicAdd(&s_hist[digit], 1u);
        if (!one_hist) {
          if (lane_id() == 0) atomicAdd(&s_hist[kSelBins + d0], static_cast<uint32_t>(__popcll(m)));
          if (digit != d0) atomicAdd(&s_hist[kSelBins + digit], 1u);
        }
      }
    } else {
      // later passes: only the keys of the one or two bins that are followed take part, and most wavefronts hold
      // none: which of a thread's keys do is collected first
      uint32_t act0 = 0, act1 = 0;
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        act0 |= (keys[j] & fixed_mask) == prefix[one_hist && rank[0] == 0 ? 1 : 0] ? (1u << j) : 0u;
        if (!one_hist) act1 |= (keys[j] & fixed_mask) == prefix[1] ? (1u << j) : 0u;
      }
      if (ballot64((act0 | act1) != 0) != 0) {
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
          const uint32_t digit = (keys[j] >> shift) & dmask;
          hist_add(s_hist, (act0 >> j) & 1u, digit);  // (returns at once when no lane takes part)
          if (!one_hist) hist_add(s_hist + kSelBins, (act1 >> j) & 1u, digit);
        }
      }
    }
    __syncthreads();
    {
      // both ranks in one walk from the top bin down (two bins per thread; a rank of 0 finds nothing)
      constexpr int kW = kSampleThreads / kWave;
      const uint32_t* hb = one_hist ? s_hist : s_hist + kSelBins;
      uint32_t ca[2], cb[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        ca[j] = s_hist[kSelBins - 1 - (t * 2 + j)];
        cb[j] = hb[kSelBins - 1 - (t * 2 + j)];
      }
      const uint32_t sa = ca[0] + ca[1], sb = cb[0] + cb[1];
      const uint32_t ia = wave_prefix_sum(sa), ib = one_hist ? ia : wave_prefix_sum(sb);
      if (lane_id() == kWave - 1) {
        s_tmp[t / kWave] = ia;
        s_scan_b[t / kWave] = ib;
      }
      __syncthreads();
      uint32_t above_a = ia - sa, above_b = ib - sb;
      for (uint32_t w = 0; w < t / kWave; ++w) above_a += s_tmp[w];
      if (one_hist) {
        above_b = above_a;
      } else {
        for (uint32_t w = 0; w < t / kWave; ++w) above_b += s_scan_b[w];
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if (rank[0] != 0 && above_a < k_rem[0] && k_rem[0] <= above_a + ca[j]) {
          s_found[0] = kSelBins - 1 - (t * 2 + j);
          s_found[1] = above_a;
        }
        if (rank[1] != 0 && above_b < k_rem[1] && k_rem[1] <= above_b + cb[j]) {
          s_found[2] = kSelBins - 1 - (t * 2 + j);
          s_found[3] = above_b;
        }
        above_a += ca[j];
        above_b += cb[j];
      }
      __syncthreads();
      if (rank[0] != 0) {
        prefix[0] |= s_found[0] << shift;
        k_rem[0] -= s_found[1];
      }
      if (rank[1] != 0) {
        prefix[1] |= s_found[2] << shift;
        k_rem[1] -= s_found[3];
      }
      static_assert(kW + 4 <= kSampleThreads / kWave + 4, "s_tmp holds one word per wavefront");
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

// Shift that maps key - lo, for keys in [lo, hi], onto kCoarseBins values.
__device__ __forceinline__ uint32_t coarse_shift(uint32_t lo, uint32_t hi) {
  const uint32_t span = hi - lo;
  const uint32_t bits = span ? 32u - static_cast<uint32_t>(__builtin_clz(span)) : 0u;
  return bits > kCoarseBits ? bits - kCoarseBits : 0u;
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
  __shared__ uint32_t s_coarse[kCoarseBins];
  __shared__ uint32_t s_taken;
  const uint32_t lane = lane_id();
  const int wave = threadIdx.x / kWave;
  const uint32_t wg = blockIdx.x;
  const uint32_t lo = ws->lo, hi = ws->hi;
  const uint32_t cshift = coarse_shift(lo, hi);
  const uint32_t region_cap = ws->cand_cap / kCandRegions;
  unsigned long long* region_count = &ws->counts[wg % kCandRegions].c;
  uint32_t* region_keys = ws->cand + static_cast<size_t>(wg % kCandRegions) * region_cap;
  uint32_t* stage = s_stage[wave];
  uint32_t staged = 0, above = 0;
  __shared__ uint32_t s_cnt[kPartWaves], s_abv[kPartWaves], s_base;
  if (threadIdx.x == 0) s_taken = 0;
  if (threadIdx.x < kCoarseBins) s_coarse[threadIdx.x] = 0;
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
  auto take = [&](const uint32_t* raw, bool in, auto ne_tag, const uint4* packed = nullptr) {
    constexpr int NE = decltype(ne_tag)::value;
    constexpr bool kPacked = DT == DCT_BF16 && NE == 8;  // whole bf16 vectors: packed compares (`packed`)
    // one compare per element in the common case: keys >= lo are rare (per-lane bitmap)
    uint32_t ge_bits = 0;
    if constexpr (kPacked) {
      ge_bits = bf16x8_ge_bits(*packed, lo);
    } else {
#pragma unroll
      for (int e = 0; e < NE; ++e) ge_bits |= (raw[e] & E::kKeyMask) >= lo ? (1u << e) : 0u;
    }
    if (!in) ge_bits = 0;
    const uint64_t m_any = ballot64(ge_bits != 0);
    if (m_any == 0) return;
    uint32_t hi_bits = 0;
    if constexpr (kPacked) {
      hi_bits = bf16x8_ge_bits(*packed, hi + 1u);  // hi <= 0x7FFF
    } else {
#pragma unroll
      for (int e = 0; e < NE; ++e) hi_bits |= (raw[e] & E::kKeyMask) > hi ? (1u << e) : 0u;
    }
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
          if ((c_bits >> e) & 1u) {
            const uint32_t key = raw[e] & E::kKeyMask;
            stage[slot++] = key;
            atomicAdd(&s_coarse[(key - lo) >> cshift], 1u);  // the candidates' first radix pass, on the way
          }
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
      take(raw, full || vec0 + r * kWave < geo.n_vec, std::integral_constant<int, V>{}, &v);
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
  // (the barriers above have waited for every wavefront's last LDS add)
  if (threadIdx.x < kCoarseBins) {
    const uint32_t c = s_coarse[threadIdx.x];
    if (c != 0)
      __hip_atomic_fetch_add(&ws->coarse[wg % kCoarseCopies][threadIdx.x], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
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
  __shared__ uint32_t s_tot[3], s_cb[3];
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
    if (st.from_cand) {  // uniform
      // The partition pass has histogrammed the top kCoarseBits bits of the candidates (of key - lo): walk
      // that histogram from the top (the first wavefront, four bins per lane) and fix those bits at once.
      const uint32_t cshift = st.rem_bits > kCoarseBits ? st.rem_bits - kCoarseBits : 0u;  // = coarse_shift(lo, hi)
      if (threadIdx.x < kWave) {
        static_assert(kCoarseBins == 4 * kWave, "four bins per lane");
        uint32_t c[4], sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          c[j] = 0;
#pragma unroll
          for (uint32_t q = 0; q < kCoarseCopies; ++q) c[j] += ws->coarse[q][kCoarseBins - 1 - (threadIdx.x * 4 + j)];
          sum += c[j];
        }
        const uint32_t incl = wave_prefix_sum(sum);
        uint32_t above = incl - sum;
        if (above < st.k_rem && st.k_rem <= incl) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (above < st.k_rem && st.k_rem <= above + c[j]) {
              s_cb[0] = kCoarseBins - 1 - (threadIdx.x * 4 + j);
              s_cb[1] = above;
              s_cb[2] = c[j];
              above = 0xFFFFFFFFu;
            } else if (above != 0xFFFFFFFFu) {
              above += c[j];
            }
          }
        }
      }
      __syncthreads();
      st.prefix = s_cb[0] << cshift;
      st.k_rem -= s_cb[1];
      st.n_gt += s_cb[1];
      st.last_count = s_cb[2];
      st.rem_bits = cshift;
    }
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

  // ---- the short way.  The coarse histogram has left one bin of the candidates; when that bin holds few
  // keys (the rule: a few thousand of c4's 1.6 million candidates) every workgroup hands the keys of its
  // region that fall into the bin to a common list, and the workgroup that arrives last selects among them on
  // its own, in LDS, however many bits are left: no grid barrier, no histogram merged through memory.  (Keys
  // and the arrival are returning agent-scope atomics, so a key has been performed before its workgroup's
  // arrival is.)  A bin with more keys than the list holds -- ties, coarse data -- takes the passes below.
  if (st.from_cand && st.rem_bits != 0 && st.last_count <= kFinalCap) {  // uniform over the grid
    const uint32_t fixed_all = ~((1u << st.rem_bits) - 1u);
    const uint32_t prefix = st.prefix;
    const uint32_t low_mask = (1u << st.rem_bits) - 1u;
    constexpr int kFinalPer = kFinalCap / kTailThreads;
    __shared__ uint32_t s_base;
    // this workgroup's keys in the bin: count, place, append
    auto for_each_key = [&](auto&& f) {
      for (uint32_t region = blockIdx.x; region < kCandRegions; region += n_active) {
        const uint4* cv = reinterpret_cast<const uint4*>(ws->cand + static_cast<size_t>(region) * region_cap);
        const bool first = region == blockIdx.x;  // its head is in registers
        const uint32_t n_src = first ? cnt0 : min(static_cast<uint32_t>(ws->counts[region].c), region_cap);
        const uint32_t reg_vecs = (n_src + 3) / 4;
        if (first) {
#pragma unroll
          for (int u = 0; u < kTailKeep; ++u) {
            f(keep[u].x);
            f(keep[u].y);
            f(keep[u].z);
            f(keep[u].w);
          }
        }
        for (uint32_t vi = (first ? kTailKeep * kTailThreads : 0u) + threadIdx.x; vi < reg_vecs; vi += kTailThreads) {
          const uint4 v = offset_keys(cv[vi], vi, n_src, lo_key);
          f(v.x);
          f(v.y);
          f(v.z);
          f(v.w);
        }
      }
    };
    uint32_t mine = 0;
    for_each_key([&](uint32_t key) { mine += (key & fixed_all) == prefix ? 1u : 0u; });
    const uint32_t incl = wave_prefix_sum(mine);
    if (lane_id() == kWave - 1) s_tmp[threadIdx.x / kWave] = incl;
    __syncthreads();
    uint32_t before = incl - mine, total = 0;
    for (uint32_t w = 0; w < kTailThreads / kWave; ++w) {
      const uint32_t c = s_tmp[w];
      before += w < threadIdx.x / kWave ? c : 0u;
      total += c;
    }
    if (threadIdx.x == 0) s_base = total ? add_agent(&ws->final_count, total) : 0u;
    // The keys go out in two steps: into a list in LDS at their ranks, then one key per thread and round from
    // that list to the common list.  (A thread that appends its own matches one after the other waits a
    // memory round trip for each returning atomic: 6 us on c4, where some threads hold four.)
    uint32_t seen = 0;
    for (uint32_t done = 0; done < total; done += kSelBins) {  // uniform; one round unless ties abound
      __syncthreads();  // s_base is set; h is free
      uint32_t rank = before;
      for_each_key([&](uint32_t key) {
        if ((key & fixed_all) == prefix) {
          if (rank >= done && rank < done + kSelBins) h[rank - done] = key & low_mask;
          ++rank;
        }
      });
      __syncthreads();
      const uint32_t chunk = min(total - done, static_cast<uint32_t>(kSelBins));
      for (uint32_t i = threadIdx.x; i < chunk; i += kTailThreads) {
        const uint32_t pos = s_base + done + i;
        if (pos < kFinalCap)
          seen += __hip_atomic_exchange(&ws->final_keys[pos], h[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::"v"(seen) : "memory");
    __syncthreads();
    if (threadIdx.x == 0) s_arrived = add_agent(&ws->final_arrived, 1u) + 1u;
    __syncthreads();
    if (s_arrived < n_active) return;  // uniform: another workgroup arrives last

    // ---- the last workgroup: the k_rem-th largest of the listed keys, radix passes in LDS
    const uint32_t n_final = st.last_count;  // exactly what the coarse histogram counted in the bin
    uint32_t fk[kFinalPer];
#pragma unroll
    for (int j = 0; j < kFinalPer; ++j) {
      const uint32_t i = j * kTailThreads + threadIdx.x;
      fk[j] = i < n_final ? ld_agent(&ws->final_keys[i]) : 0xFFFFFFFFu;  // fillers match no prefix
    }
    uint32_t rem = st.rem_bits, low_prefix = 0, k_rem = st.k_rem, n_gt = st.n_gt, count = n_final;
    while (rem != 0) {  // uniform
      const uint32_t width = min(kDigitBits, rem);
      const uint32_t shift = rem - width;
      const uint32_t fixed = ~((1u << rem) - 1u);
      for (int i = threadIdx.x; i < kSelBins; i += kTailThreads) h[i] = 0;
      __syncthreads();
#pragma unroll
      for (int j = 0; j < kFinalPer; ++j)
        hist_add(h, (fk[j] & fixed) == low_prefix, (fk[j] >> shift) & ((1u << width) - 1u));
      __syncthreads();
      const BinHit hit = find_bin<kTailThreads>([&](uint32_t b) { return h[b]; }, k_rem, s_tmp);
      low_prefix |= hit.bin << shift;
      k_rem -= hit.above;
      n_gt += hit.above;
      count = hit.count;
      rem = shift;
    }
    if (threadIdx.x == 0) {
      out->tau_key = (st.prefix | low_prefix) + range_lo;
      out->n_gt = n_gt;
      out->n_eq = count;
      out->tie_quota = k_rem;
    }
    return;
  }

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

// Room for the keys between the sample bounds.  The bounds are 5 standard deviations of the sample count on
// either side of rank k, so about 10 sqrt(p (1 - p) / 16384) of the vector lies between them when a fraction
// p is kept: at most 4 % (p = 1/2).  cand_capacity(n) serves any k; cand_capacity_for(n, k) is twice the
// expected number for this k plus slack (0.6 % of c4 is expected, 1.4 % + 64 Ki keys are asked for).  A buffer
// that turns out too small costs time, not exactness (the passes then run over the vector).
uint32_t cand_capacity(uint64_t n) {
  return n >= kSampleMinN ? static_cast<uint32_t>(n / 16 + 65536) & ~(4u * kCandRegions - 1u) : 0u;
}
uint32_t cand_capacity_for(uint64_t n, uint64_t k) {
  if (n < kSampleMinN) return 0u;
  const uint64_t r = k * kSampleSize / n;  // the same arithmetic as sample_ranks
  const uint64_t var = r * (kSampleSize - r) / kSampleSize;
  uint64_t sq = 0;
  while ((sq + 1) * (sq + 1) <= var) ++sq;
  const uint64_t window = 2 * (5 * (sq + 1) + 8) + 1;  // sample ranks between the bounds
  const uint64_t want = 2 * (n / kSampleSize + 1) * window + 65536;
  const uint64_t rounded = (want + 4u * kCandRegions - 1u) & ~static_cast<uint64_t>(4u * kCandRegions - 1u);
  return static_cast<uint32_t>(std::min<uint64_t>(rounded, cand_capacity(n)));
}

// Sample ranks (1-based from the top) that bracket rank k of the vector with a margin of five standard
// deviations of the sample count (binomial: r (S - r) / S), plus slack; 0 = no bound on that side.  Where the
// margin reaches past the top of the sample the largest sample key still serves as the upper bound as long as
// about 16 sample keys are expected above tau (none at all: e^-16, the risk the five standard deviations take
// elsewhere); a bound that does not hold is found out and costs time only.
void sample_ranks(uint64_t n, uint64_t k, uint32_t& rank_hi, uint32_t& rank_lo) {
  const uint64_t r = k * kSampleSize / n;
  const uint64_t var = r * (kSampleSize - r) / kSampleSize;
  uint64_t sq = 0;
  while ((sq + 1) * (sq + 1) <= var) ++sq;
  const uint64_t delta = 5ull * (sq + 1) + 8;
  rank_hi = static_cast<uint32_t>(r > delta ? r - delta : (r >= 16 ? 1 : 0));
  rank_lo = static_cast<uint32_t>(r + delta + 1 <= kSampleSize ? r + delta + 1 : 0);
}

// Tag of a call (see SelWs::sample): unique within the process, starting from a value that differs
// from process to process.
uint32_t next_call_tag() {
  static std::atomic<uint32_t> counter{static_cast<uint32_t>(
      std::chrono::steady_clock::now().time_since_epoch().count() * 2654435761ull >> 16)};
  return counter.fetch_add(1, std::memory_order_relaxed);
}

}  // namespace
}  // namespace dct

using namespace dct;

extern "C" size_t dct_select_threshold_workspace_bytes(int dt, uint64_t n) {
  if ((dt != DCT_F32 && dt != DCT_BF16) || n == 0 || n > 0x7FFFFFFFull) return 0;
  return sizeof(SelWs) + static_cast<size_t>(cand_capacity(n)) * 4;
}

extern "C" size_t dct_select_threshold_workspace_bytes_for(int dt, uint64_t n, uint64_t k) {
  if ((dt != DCT_F32 && dt != DCT_BF16) || n == 0 || n > 0x7FFFFFFFull || k == 0 || k > n) return 0;
  return sizeof(SelWs) + static_cast<size_t>(cand_capacity_for(n, k)) * 4;
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
  // the candidate buffer: whatever the workspace offers beyond the fixed part, between what this k needs and
  // what any k needs
  if (!d_ws || !is_aligned(d_ws, 256) || ws_bytes < sizeof(SelWs)) return DCT_ERR_WORKSPACE;
  const uint64_t offered = ((ws_bytes - sizeof(SelWs)) / 4) & ~static_cast<uint64_t>(4u * kCandRegions - 1u);
  if (offered < cand_capacity_for(n, k)) return DCT_ERR_WORKSPACE;
  const uint32_t cand_cap = static_cast<uint32_t>(std::min<uint64_t>(offered, cand_capacity(n)));

  const int vec = dt == DCT_F32 ? 4 : 8;
  const uint32_t spin_limit = wait_limit();  // polls of a device-side wait (by default about a second) before giving up
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
    const dim3 sgrid(kSampleSize / kSampleThreads), sblock(kSampleThreads), pgrid(geo.grid), pblock(kPartThreads);
    const uint32_t tag = next_call_tag();
    uint32_t rank_hi = 0, rank_lo = 0;
    sample_ranks(n, k, rank_hi, rank_lo);
    if (ef) {
      hipLaunchKernelGGL((select_sample_kernel<DCT_F32, true>), sgrid, sblock, 0, s, g32, e32, n32, rank_hi, rank_lo, ws, cand_cap, tag, spin_limit);
      if (large) hipLaunchKernelGGL((select_partition_kernel<DCT_F32, true, kPartRowsLarge>), pgrid, pblock, 0, s, g32, e32, geo, ws);
      else hipLaunchKernelGGL((select_partition_kernel<DCT_F32, true, kPartRowsSmall>), pgrid, pblock, 0, s, g32, e32, geo, ws);
    } else if (dt == DCT_F32) {
      hipLaunchKernelGGL((select_sample_kernel<DCT_F32, false>), sgrid, sblock, 0, s, g32, nullptr, n32, rank_hi, rank_lo, ws, cand_cap, tag, spin_limit);
      if (large) hipLaunchKernelGGL((select_partition_kernel<DCT_F32, false, kPartRowsLarge>), pgrid, pblock, 0, s, g32, nullptr, geo, ws);
      else hipLaunchKernelGGL((select_partition_kernel<DCT_F32, false, kPartRowsSmall>), pgrid, pblock, 0, s, g32, nullptr, geo, ws);
    } else {
      hipLaunchKernelGGL((select_sample_kernel<DCT_BF16, false>), sgrid, sblock, 0, s, g16, nullptr, n32, rank_hi, rank_lo, ws, cand_cap, tag, spin_limit);
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
