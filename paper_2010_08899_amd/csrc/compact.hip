// dct_threshold_compact: Algorithm 1, "M = I(|W_grad| >= tau)" and
// "W_hat = W_grad . M", as ONE pass over the gradient that writes the survivors
// as (ascending index, value) pairs.
//
// Design (gfx950).  The 8 XCDs of the chip have private L2s, so workgroups can
// only talk to each other through the memory-side path (about a microsecond per
// round trip, and polling hammers a few channels).  The kernel therefore keeps
// cross-workgroup traffic to one short exchange at the very end:
//   1. The 16-byte-aligned interior of the vector is split into one contiguous
//      chunk per workgroup (at most 4 workgroups per CU, all resident at once);
//      each of its four wavefronts streams a contiguous quarter with coalesced
//      16-byte loads, 8 KiB per wavefront per iteration.
//   2. Survivors are sparse (<= a few %), so each wavefront appends its
//      (index, value) pairs, in index order, to its own region of LDS (ballot +
//      lane-prefix ranks).  No workgroup waits for another while streaming.
//   3. When a chunk is done the workgroup publishes its two counts (keys above
//      tau, ties at tau) in a 64-bit descriptor.  Descriptors are summed in two
//      levels (members of a group of 64 workgroups, then whole groups), which keeps
//      every poll to one coalesced load of at most 64 descriptors.
//   4. With its exclusive prefix known, the workgroup copies its staged pairs to
//      their final slots; in exactly-k mode a tie is written while fewer than
//      tie_quota ties precede it (ties are staged with a flag bit).
// The survivors of a chunk wait on chip, so the grid as a whole can hold about
// four million of them.  A vector that keeps more (the paper's lower sparsity
// levels) is cut into up to a dozen contiguous slices ("rounds") that are processed
// one after the other by the same workgroups; the (round, workgroup) pairs form one
// sequence for the prefix exchange.  The number of rounds comes from the counts in
// the threshold record.  If a wavefront's LDS region overflows all the same (more
// survivors than the record promised, a tie value that covers much of the vector,
// or more rounds needed than are worth their cost) the workgroup still counts
// everything, and after the scan streams its chunk a second time, writing straight
// to the final slots.
//
// Error feedback (Algorithm 1, "W_grad = W_grad + E_grad" before the mask and
// "E_grad = W_grad - W_hat_grad" after it) rides on the same pass: the EF variant
// streams g and the residual together, forms w = g + e with one fp32 addition per
// element, writes w as the new residual with full 16-byte stores and compacts w.
// The residual of a pair that is actually written out is then overwritten with
// +0 in step 4 (a 4-byte store per survivor), so an entry that finds no room in
// the outputs keeps its value in the residual.  The second-pass fallback re-reads
// w from the new residual, which also makes updating the residual in place safe.
//
// With error feedback the vector is also cut into up to 8 slices when it would not
// have to be: the drains between slices keep the workgroups in step, and a kernel
// that writes a third of what it reads runs faster when its accesses stay within a
// narrow window of the vector (c4: 603 us in 8 slices against 661 us in one).
//
// A workgroup only ever waits for workgroups with a lower index (and, from the
// second round on, for every workgroup's earlier rounds), so the whole grid has to
// be resident: the kernel is compiled for four wavefronts per SIMD and the grid is
// sized from the occupancy the runtime reports.  The waits are bounded all the
// same and a wait that runs out is reported through the count.  The workspace holds two descriptor sets used by alternate
// calls (an epoch word picks the set): every call clears the other set for its
// successor and the last workgroup advances the epoch, so a call is one launch.
#include <algorithm>
#include <type_traits>

#include "dct_common.hpp"

namespace dct {
namespace {

constexpr int kCtThreads = 256;
constexpr int kCtWaves = kCtThreads / kWave;
constexpr int kCtRows = 8;                              // 16-byte loads per lane per iteration
constexpr uint32_t kCtTileVecs = kCtThreads * kCtRows;  // granule of the chunking: 32 KiB
// Workgroups per CU (WG, a template argument of the kernel) and staged pairs per wavefront (each pair 8 bytes of
// LDS; 144 KiB per CU either way).  Three larger workgroups stream better than four (c4 179 -> 174 us; 2^28 dense
// fp32 with 1 % kept: 206 -> 184 us; a CU serves its oldest workgroup first and the youngest sets the kernel's
// time), and on short vectors two do better still (25 M elements: 27.0 -> 26.0 us); with error feedback, which
// writes a third of what it reads, four do (597 against 622 us), and so do bf16 vectors, whose eight elements
// per vector need the wavefronts (2^29 elements, exactly-k: 237 against 251 us).
constexpr int ct_wg_per_cu(bool ef, int dt, uint64_t n) {
  return ef || dt == DCT_BF16 ? 4 : n < (1ull << 26) ? 2 : 3;
}
constexpr uint32_t ct_stage_cap(int wg) { return 4608u / static_cast<uint32_t>(wg); }
constexpr uint32_t kCtMaxGrid = 2048;
constexpr uint32_t kCtGroup = 64;                       // (virtual) workgroups per descriptor group
constexpr uint32_t kCtMaxRounds = 12;                   // slices a dense vector is cut into (at most)
constexpr uint32_t kCtMaxVirtual = kCtMaxGrid * kCtMaxRounds;
constexpr uint32_t kCtMaxGroups = kCtMaxVirtual / kCtGroup;
constexpr uint32_t kCtMagic = 0x44435434u;              // "DCT4"
constexpr uint32_t kCtHeaderBytes = 256;
constexpr uint32_t kCtSpinLimit = 1u << 20;
constexpr uint32_t kTieFlag = 0x80000000u;

// Descriptor: [63:62] status, [61:31] count A (keys above the cut), [30:0] count E (ties).
constexpr uint64_t kStAggregate = 1ull << 62;
constexpr uint64_t kStInclusive = 2ull << 62;
constexpr uint64_t kPayload = (1ull << 62) - 1;

struct CompactHeader {
  uint32_t magic;
  uint32_t epoch;
  uint32_t error;
  uint32_t used[2];  // descriptors of each set that the last call using it wrote (they must be cleared)
  uint32_t pad[59];
};
static_assert(sizeof(CompactHeader) == kCtHeaderBytes, "header size");

struct DescSet {
  uint64_t wg[kCtMaxVirtual];
  uint64_t group[kCtMaxGroups];
};
constexpr size_t kCtWsBytes = kCtHeaderBytes + 2 * sizeof(DescSet);

__device__ __forceinline__ uint64_t pack(uint32_t a, uint32_t e) { return (static_cast<uint64_t>(a) << 31) | e; }
__device__ __forceinline__ uint32_t cnt_a(uint64_t p) { return static_cast<uint32_t>((p & kPayload) >> 31); }
__device__ __forceinline__ uint32_t cnt_e(uint64_t p) { return static_cast<uint32_t>(p & 0x7FFFFFFFu); }

__global__ void compact_ws_init_kernel(uint32_t* ws, uint32_t n_words) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_words) return;
  ws[i] = (i == 0) ? kCtMagic : 0u;
}

// Bounded wait helper: returns false when the spin budget is used up or another
// workgroup has already reported a failure.
__device__ __forceinline__ bool keep_waiting(uint32_t& spins, const uint32_t* error_flag) {
  ++spins;
  if (spins > kCtSpinLimit || ((spins & 255u) == 0 && ld_agent(error_flag) != 0)) return false;
  __builtin_amdgcn_s_sleep(1);
  return true;
}

// Sum of the descriptors of members 0..m-1 of a group (m <= 63), once all are published.
__device__ uint64_t sum_members(const uint64_t* first, uint32_t m, const uint32_t* error_flag, bool& failed) {
  if (m == 0) return 0;
  const uint32_t lane = lane_id();
  uint32_t spins = 0;
  for (;;) {
    const uint64_t d = lane < m ? ld_agent(first + lane) : kStAggregate;
    if (ballot64((d >> 62) == 0) == 0) return wave_sum_u64(d & kPayload);
    if (!keep_waiting(spins, error_flag)) {
      failed = true;
      return 0;
    }
  }
}

// Sum over all groups before group g: nearest groups first, 64 at a time, up to and
// including the first one that carries an inclusive prefix.
__device__ uint64_t group_prefix(const uint64_t* gdesc, uint32_t g, const uint32_t* error_flag, bool& failed) {
  const int lane = lane_id();
  uint64_t sum = 0;
  uint32_t spins = 0;
  int pos = static_cast<int>(g);  // groups [0, pos) are still to be accounted for
  while (pos > 0) {
    const int i = pos - 1 - lane;
    const uint64_t d = i >= 0 ? ld_agent(gdesc + i) : kStInclusive;  // the virtual group -1: inclusive 0
    const uint32_t st = static_cast<uint32_t>(d >> 62);
    const uint64_t invalid = ballot64(st == 0);
    const uint64_t incl = ballot64(st == 2);
    const int f = incl ? __builtin_ctzll(incl) : 63;  // nearest group with an inclusive prefix, if any
    const uint64_t need = (f == 63) ? ~0ull : ((2ull << f) - 1);
    if ((invalid & need) != 0) {
      if (!keep_waiting(spins, error_flag)) {
        failed = true;
        return 0;
      }
      continue;
    }
    sum += wave_sum_u64(lane <= f ? (d & kPayload) : 0ull);
    if (incl) break;
    pos -= kWave;
  }
  return sum;
}

// Work description shared by all workgroups (computed on the host).
struct CompactGeom {
  uint32_t head;         // elements before the first 16-byte-aligned vector (< kVec)
  uint32_t n_vec;        // full 16-byte vectors after the head
  uint32_t tail;         // elements after the last full vector (< kVec)
  uint32_t grid;         // workgroups
  uint32_t tiles;        // granules of kCtTileVecs vectors that cover the full vectors (>= 1)
};

// EF: g is W_grad, e_in the residual E_grad (may be the same buffer as e_out), e_out the new residual.
template <int DT, bool EXACT, bool EF, int WG>
__global__ __launch_bounds__(kCtThreads, WG) void compact_kernel(
    const typename Elem<DT>::word_t* __restrict__ g, const typename Elem<DT>::word_t* e_in,
    typename Elem<DT>::word_t* e_out, CompactGeom geo, const dct_threshold* __restrict__ thr,
    int32_t* __restrict__ idx_out, typename Elem<DT>::word_t* __restrict__ val_out, uint32_t capacity,
    uint64_t* __restrict__ count_out, CompactHeader* hdr) {
  static_assert(!EF || DT == DCT_F32, "error feedback is an fp32 addition");
  using E = Elem<DT>;
  using word_t = typename E::word_t;
  constexpr int V = E::kVec;
  constexpr int ROWS = EF ? kCtRows / 2 : kCtRows;  // two input streams: half the rows per iteration
  constexpr uint32_t kCtStageCap = ct_stage_cap(WG);
  __shared__ uint32_t s_idx[kCtWaves][kCtStageCap];
  __shared__ word_t s_val[kCtWaves][kCtStageCap];
  __shared__ uint32_t s_wave_a[kCtWaves], s_wave_e[kCtWaves];
  __shared__ uint64_t s_excl;

  const uint32_t wg = blockIdx.x;
  const uint32_t lane = lane_id();
  const int wave = threadIdx.x / kWave;

  // ---- workspace: this call's descriptor set; what the previous call wrote into the other set
  // is cleared for the next call
  // (everything the prologue needs from memory is requested before the first wait)
  const uint32_t magic = hdr->magic;
  const uint32_t epoch = hdr->epoch;
  const uint32_t used0 = hdr->used[0], used1 = hdr->used[1];
  const uint32_t tau = thr->tau_key;
  const uint32_t quota = thr->tie_quota;
  const uint32_t thr_gt = thr->n_gt, thr_eq = thr->n_eq;
  if (magic != kCtMagic) {  // never initialised (uniform over the grid)
    if (wg == 0 && threadIdx.x == 0) *count_out = DCT_COUNT_WORKSPACE_ERROR;
    return;
  }
  DescSet* sets = reinterpret_cast<DescSet*>(reinterpret_cast<char*>(hdr) + kCtHeaderBytes);
  DescSet* mine_set = sets + (epoch & 1u);
  {
    DescSet* other = sets + ((epoch & 1u) ^ 1u);
    const uint32_t used = min((epoch & 1u) ? used0 : used1, kCtMaxVirtual);
    for (uint32_t i = wg * kCtThreads + threadIdx.x; i < used; i += geo.grid * kCtThreads) st_agent(&other->wg[i], 0ull);
    const uint32_t used_groups = (used + kCtGroup - 1) / kCtGroup;
    for (uint32_t i = wg * kCtThreads + threadIdx.x; i < used_groups; i += geo.grid * kCtThreads)
      st_agent(&other->group[i], 0ull);
  }

  // ---- rounds.  All survivors of a workgroup's chunk wait in LDS until the chunk's place in the
  // output is known, so a chunk may hold only about 4600 of them.  A vector with more survivors
  // than the whole grid can hold at once is cut into `rounds` contiguous slices that are processed
  // one after the other; the (round, workgroup) pairs form one long sequence of virtual workgroups
  // for the prefix exchange.  The number of rounds is derived from the counts in the threshold
  // record (the same in every workgroup); if it turns out too low, the second-pass fallback of the
  // chunks that overflow keeps the result exact.
  uint32_t rounds;
  {
    // ties are staged too; the record is the same for every lane: keep the arithmetic scalar
    const uint64_t expected = static_cast<uint64_t>(__builtin_amdgcn_readfirstlane(thr_gt)) +
                              __builtin_amdgcn_readfirstlane(thr_eq);
    const uint64_t room = static_cast<uint64_t>(geo.grid) * (kCtWaves * kCtStageCap * 7 / 8);
    // Every round costs a pipeline drain and refill (about 15 us on MI355X); beyond a dozen rounds
    // reading the vector twice (the second-pass fallback) is cheaper.
    rounds = 1;
    while (rounds <= kCtMaxRounds && expected > room * rounds) ++rounds;  // ceil(expected / room), no division
    if (rounds > kCtMaxRounds) rounds = 1;
    if constexpr (EF) {
      // With error feedback the kernel writes as much as a third of what it reads.  The memory system
      // sustains such a mix better when the grid works within a narrow window of the vector, and the
      // slices do just that: 8 slices of >= 128 KiB per workgroup took c4 from 661 to 603 us, their
      // seven drains included (4 slices: 621 us, 16: 649 us).
      uint32_t window_rounds = 1;
      while (window_rounds < 8u && geo.tiles >= 8u * window_rounds * geo.grid) window_rounds *= 2u;
      rounds = max(rounds, window_rounds);
    }
    rounds = min(rounds, geo.tiles);
  }
  const uint32_t n_virtual = rounds * geo.grid;
  const uint32_t tiles_per_round = (geo.tiles + rounds - 1) / rounds;
  // a slice is dealt to the workgroups, and a workgroup's chunk to its wavefronts, in whole rows of 64 vectors
  const uint32_t vecs_per_wg =
      ((tiles_per_round * kCtTileVecs + geo.grid - 1) / geo.grid + kWave - 1) / kWave * kWave;

  // ---- this wavefront's share of the current round: rows of 64 vectors [row_lo, row_hi) of the
  // workgroup's chunk [wg_lo, wg_hi)
  const uint4* gv = reinterpret_cast<const uint4*>(g + geo.head);
  uint32_t wg_lo = 0, wg_hi = 0, row_lo = 0, row_hi = 0;
  uint32_t wave_hi = 0;  // first vector past this wavefront's rows
  bool do_head = false, do_tail = false;
  const uint32_t tail_base = geo.head + geo.n_vec * V;

  // One pass over the wavefront's share.  DIRECT = false: stage survivors (ties
  // flagged) in LDS and count; DIRECT = true: the exclusive counts are known, write
  // to the final slots.  Leaves in wa / we the number of A / E elements seen.
  uint32_t wa = 0, we = 0;
  auto pass = [&](auto direct_tag, uint32_t a_before, uint32_t e_before) {
    constexpr bool DIRECT = decltype(direct_tag)::value;
    uint32_t staged = 0;  // STAGE: pairs appended so far (beyond the region they are only counted)
    uint32_t na = 0, ne = 0;

    // up to NE elements per lane: raw[e], validity, index of element 0
    auto emit = [&](const uint32_t* raw, bool in, uint32_t index0, auto nelem_tag) {
      constexpr int NE = decltype(nelem_tag)::value;
      // Cheap common case first: one compare per element against tau (keys >= tau are the
      // survivors and, in exactly-k mode, the ties), collected in a per-lane bitmap; most groups
      // of rows have none.
      uint32_t ge_bits = 0;
#pragma unroll
      for (int e = 0; e < NE; ++e) ge_bits |= (raw[e] & E::kKeyMask) >= tau ? (1u << e) : 0u;
      if (!in) ge_bits = 0;
      const uint64_t m_any = ballot64(ge_bits != 0);
      if (m_any == 0) return;
      uint32_t e_bits = 0;
      if constexpr (EXACT) {
#pragma unroll
        for (int e = 0; e < NE; ++e) e_bits |= (raw[e] & E::kKeyMask) == tau ? (1u << e) : 0u;
        e_bits &= ge_bits;
      }
      const uint32_t a_bits = ge_bits & ~e_bits;
      uint32_t row_a, row_e;
      {
        if constexpr (!DIRECT) {
          // Index order inside the row is (lane, element), so one wave scan of the per-lane counts
          // (both packed into one word: a lane holds at most 8 elements) places every lane's pairs.
          // When no lane holds two survivors (the usual case) a ballot ranks them.
          uint32_t before;  // pairs of this row in lower lanes
          if (ballot64((ge_bits & (ge_bits - 1)) != 0) == 0) {
            row_e = EXACT ? static_cast<uint32_t>(__popcll(ballot64(e_bits != 0))) : 0u;
            row_a = static_cast<uint32_t>(__popcll(m_any)) - row_e;
            before = lanes_below(m_any);
          } else {
            const uint32_t mine = __popc(a_bits) | (__popc(e_bits) << 16);
            const uint32_t incl = wave_prefix_sum(mine);
            const uint32_t excl = incl - mine;
            const uint32_t total = __builtin_amdgcn_readlane(incl, kWave - 1);
            row_a = total & 0xFFFFu;
            row_e = total >> 16;
            before = (excl & 0xFFFFu) + (excl >> 16);
          }
          if (ge_bits != 0) {
            uint32_t slot = staged + before;
#pragma unroll
            for (int e = 0; e < NE; ++e) {
              if ((ge_bits >> e) & 1u) {
                if (slot < kCtStageCap) {
                  s_idx[wave][slot] = (index0 + e) | (((e_bits >> e) & 1u) ? kTieFlag : 0u);
                  s_val[wave][slot] = static_cast<word_t>(raw[e]);
                }
                ++slot;
              }
            }
          }
          staged += row_a + row_e;
        } else {
          // the exclusive counts are known: one wave scan of the per-lane counts places the row
          const uint32_t mine = __popc(a_bits) | (__popc(e_bits) << 16);
          const uint32_t incl = wave_prefix_sum(mine);
          const uint32_t excl = incl - mine;
          const uint32_t total = __builtin_amdgcn_readlane(incl, kWave - 1);
          row_a = total & 0xFFFFu;
          row_e = total >> 16;
          if (ge_bits != 0) {
            uint32_t a_run = a_before + na + (excl & 0xFFFFu);  // keys above the cut before this lane's
            uint32_t t_run = e_before + ne + (excl >> 16);      // ties before them (both in the whole vector)
#pragma unroll
            for (int e = 0; e < NE; ++e) {
              if ((ge_bits >> e) & 1u) {
                const bool tie = (e_bits >> e) & 1u;
                // a tie survives while fewer than `quota` ties precede it; kept ties before: min(t_run, quota)
                const uint32_t slot = a_run + (EXACT ? min(t_run, quota) : 0u);
                if ((!tie || t_run < quota) && slot < capacity) {
                  idx_out[slot] = static_cast<int32_t>(index0 + e);
                  val_out[slot] = static_cast<word_t>(raw[e]);
                  if constexpr (EF) e_out[index0 + e] = 0;  // delivered: nothing is left behind
                }
                a_run += tie ? 0u : 1u;
                t_run += tie ? 1u : 0u;
              }
            }
          }
        }
      }
      na += row_a;
      ne += row_e;
    };

    // One element of the head or tail: the corrected gradient in the first pass (stored as the
    // new residual), the new residual itself in the second.
    auto edge_element = [&](bool in, uint32_t i) -> uint32_t {
      if (!in) return 0u;
      if constexpr (!EF) {
        return static_cast<uint32_t>(g[i]);
      } else if constexpr (DIRECT) {
        return static_cast<uint32_t>(e_out[i]);
      } else {
        const uint32_t w = __float_as_uint(__uint_as_float(g[i]) + __uint_as_float(e_in[i]));
        e_out[i] = w;
        return w;
      }
    };
    if (do_head) {
      const bool in = lane < geo.head;
      const uint32_t raw = edge_element(in, lane);
      emit(&raw, in, lane, std::integral_constant<int, 1>{});
    }
    // Two register buffers: the loads of the next group of rows are in flight while the current
    // group is processed, so a wavefront always has requests outstanding.
    struct Rows {
      uint4 a[ROWS];               // g (or, in the second pass with error feedback, the new residual)
      uint4 b[EF ? ROWS : 1];      // the residual
    };
    const uint4* av = (EF && DIRECT) ? reinterpret_cast<const uint4*>(e_out + geo.head) : gv;
    const uint4* bv = EF ? reinterpret_cast<const uint4*>(e_in + geo.head) : nullptr;
    uint4* wv = EF ? reinterpret_cast<uint4*>(e_out + geo.head) : nullptr;
    constexpr bool kAdd = EF && !DIRECT;
    auto load_rows = [&](Rows& buf, uint32_t row) {
      const uint32_t vec0 = wg_lo + row * kWave + lane;
      if (wg_lo + (row + ROWS) * kWave <= wave_hi) {  // uniform: all rows inside the wavefront's share
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
          buf.a[r] = ld_stream(&av[vec0 + r * kWave]);
          if constexpr (kAdd) buf.b[r] = ld_stream(&bv[vec0 + r * kWave]);
        }
      } else {
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
          const uint32_t vi = vec0 + r * kWave;
          buf.a[r] = vi < wave_hi ? av[vi] : make_uint4(0, 0, 0, 0);
          if constexpr (kAdd) buf.b[r] = vi < wave_hi ? bv[vi] : make_uint4(0, 0, 0, 0);
        }
      }
    };
    auto process_rows = [&](const Rows& buf, uint32_t row) {
      const uint32_t vec0 = wg_lo + row * kWave + lane;
      const bool full = wg_lo + (row + ROWS) * kWave <= wave_hi;
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        const uint32_t vi = vec0 + r * kWave;
        const bool in = full || vi < wave_hi;
        uint32_t raw[V];
#pragma unroll
        for (int e = 0; e < V; ++e) raw[e] = E::raw(buf.a[r], e);
        if constexpr (kAdd) {
#pragma unroll
          for (int e = 0; e < V; ++e)
            raw[e] = __float_as_uint(__uint_as_float(raw[e]) + __uint_as_float(E::raw(buf.b[r], e)));
          if (in) st_stream(&wv[vi], raw[0], raw[1], raw[2], raw[3]);
        }
        emit(raw, in, geo.head + vi * V, std::integral_constant<int, V>{});
      }
    };
    {
      Rows va, vb;
      uint32_t row = row_lo;
      if (row < row_hi) load_rows(va, row);
      while (row < row_hi) {
        if (row + ROWS < row_hi) load_rows(vb, row + ROWS);
        process_rows(va, row);
        row += ROWS;
        if (row >= row_hi) break;
        if (row + ROWS < row_hi) load_rows(va, row + ROWS);
        process_rows(vb, row);
        row += ROWS;
      }
    }
    if (do_tail) {
      const bool in = lane < geo.tail;
      const uint32_t raw = edge_element(in, tail_base + lane);
      emit(&raw, in, tail_base + lane, std::integral_constant<int, 1>{});
    }
    wa = na;
    we = ne;
    return staged;
  };

  for (uint32_t round = 0; round < rounds; ++round) {
    const uint32_t vwg = round * geo.grid + wg;  // this workgroup's place in the sequence of chunks
    {
      const uint32_t slice_lo = min(round * tiles_per_round * kCtTileVecs, geo.n_vec);
      const uint32_t slice_hi = min(slice_lo + tiles_per_round * kCtTileVecs, geo.n_vec);
      wg_lo = min(slice_lo + wg * vecs_per_wg, slice_hi);
      wg_hi = min(wg_lo + vecs_per_wg, slice_hi);
      const uint32_t rows_total = (wg_hi - wg_lo + kWave - 1) / kWave;
      const uint32_t rows_per_wave = (rows_total + kCtWaves - 1) / kCtWaves;
      row_lo = min(static_cast<uint32_t>(wave) * rows_per_wave, rows_total);
      row_hi = min(row_lo + rows_per_wave, rows_total);
      wave_hi = min(wg_lo + row_hi * kWave, wg_hi);
      do_head = vwg == 0 && wave == 0 && geo.head != 0;
      do_tail = vwg == n_virtual - 1 && wave == kCtWaves - 1 && geo.tail != 0;
    }
    // the previous round's pairs have left the staging area (not in round 0: the barrier would also
    // wait for the descriptor-clearing stores above, a memory round trip before streaming starts)
    if (round != 0) __syncthreads();

    // ---- 1+2: stream the chunk, stage survivors in LDS
    const uint32_t staged = pass(std::false_type{}, 0u, 0u);
    // the residual stores of this pass have landed before anything (the +0 of a delivered pair, the
    // second pass's loads) touches the same addresses again
    if constexpr (EF) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (lane == 0) {
      s_wave_a[wave] = wa;
      s_wave_e[wave] = we | (staged > kCtStageCap ? kTieFlag : 0u);  // top bit: this wavefront's region overflowed
    }
    __syncthreads();

    // ---- 3: wavefront 0 publishes the counts and obtains the exclusive prefix
    if (wave == 0) {
      uint32_t ta = 0, te = 0;
#pragma unroll
      for (int w = 0; w < kCtWaves; ++w) {
        ta += s_wave_a[w];
        te += s_wave_e[w] & ~kTieFlag;
      }
      const uint64_t mine = pack(ta, te);
      const uint32_t grp = vwg / kCtGroup, member = vwg % kCtGroup;
      const bool leader = member == kCtGroup - 1;
      bool failed = false;
      if (lane == 0) st_agent(&mine_set->wg[vwg], kStAggregate | mine);
      const uint64_t before_in_group = sum_members(&mine_set->wg[grp * kCtGroup], member, &hdr->error, failed);
      if (leader && grp != 0 && lane == 0)
        st_agent(&mine_set->group[grp], kStAggregate | ((before_in_group + mine) & kPayload));
      const uint64_t before_groups = group_prefix(mine_set->group, grp, &hdr->error, failed);
      const uint64_t excl = (before_groups + before_in_group) & kPayload;
      if (lane == 0) {
        if (failed) {  // a predecessor never published: report it (the result of this call is void)
          atomicOr(&hdr->error, 1u);
          *count_out = DCT_COUNT_WORKSPACE_ERROR;
          st_agent(&hdr->magic, 0u);
        }
        if (leader) st_agent(&mine_set->group[grp], kStInclusive | ((excl + mine) & kPayload));
        s_excl = excl;
        if (vwg == n_virtual - 1) {  // every other workgroup has read the epoch and published: finish the call
          const uint64_t total = (excl + mine) & kPayload;
          uint64_t c = cnt_a(total);
          if (EXACT) c += min(cnt_e(total), quota);
          const uint32_t err = __builtin_amdgcn_readfirstlane(ld_agent(&hdr->error));
          if (failed || err != 0) {
            *count_out = DCT_COUNT_WORKSPACE_ERROR;
            st_agent(&hdr->magic, 0u);  // force a re-initialisation
          } else {
            *count_out = c;
            st_agent(&hdr->used[epoch & 1u], n_virtual);
            st_agent(&hdr->epoch, epoch + 1u);
          }
        }
      }
    }
    __syncthreads();

    // ---- 4: final slots
    const uint64_t excl = s_excl;
    uint32_t a_before = cnt_a(excl), e_before = cnt_e(excl);
    bool overflow = false;
    for (int w = 0; w < kCtWaves; ++w) {
      const uint32_t ew = s_wave_e[w];
      overflow = overflow || (ew & kTieFlag) != 0;
      if (w < wave) {
        a_before += s_wave_a[w];
        e_before += ew & ~kTieFlag;
      }
    }
    if (overflow) {  // uniform over the workgroup: second pass over the chunk, straight to the outputs
      // With error feedback the second pass reads back what the first one stored (the barriers
      // above have waited for those stores): drop this CU's cached copies of the old lines first.
      if constexpr (EF) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      pass(std::true_type{}, a_before, e_before);
      continue;
    }
    const uint32_t n_staged = wa + we;
    const uint32_t ties_left = EXACT ? (quota > e_before ? quota - e_before : 0u) : 0u;
    uint32_t out = a_before + (EXACT ? min(e_before, quota) : 0u);
    uint32_t ties_seen = 0;
    for (uint32_t j0 = 0; j0 < n_staged; j0 += kWave) {
      const uint32_t j = j0 + lane;
      const bool valid = j < n_staged;
      const uint32_t ent = valid ? s_idx[wave][j] : 0u;
      const bool is_tie = EXACT && (ent & kTieFlag) != 0;
      const uint64_t m_tie = ballot64(is_tie);
      const bool keep = valid && (!is_tie || ties_seen + lanes_below(m_tie) < ties_left);
      const uint64_t m_keep = ballot64(keep);
      const uint32_t slot = out + lanes_below(m_keep);
      if (keep && slot < capacity) {
        idx_out[slot] = static_cast<int32_t>(ent & ~kTieFlag);
        val_out[slot] = s_val[wave][j];
        if constexpr (EF) e_out[ent & ~kTieFlag] = 0;  // delivered: nothing is left behind
      }
      out += __popcll(m_keep);
      ties_seen += __popcll(m_tie);
    }
  }
}

// Head / full vectors / tail split of n elements starting at address `addr`, and the chunking.
CompactGeom make_geom(uintptr_t addr, uint64_t n, int dt, uint32_t wg_per_cu) {
  const uint32_t es = dt == DCT_F32 ? 4 : 2;
  const uint32_t vec = 16 / es;
  CompactGeom geo;
  uint64_t head = ((16 - (addr & 15)) & 15) / es;
  if (head > n) head = n;
  geo.head = static_cast<uint32_t>(head);
  geo.n_vec = static_cast<uint32_t>((n - head) / vec);
  geo.tail = static_cast<uint32_t>((n - head) % vec);
  uint32_t tiles = (geo.n_vec + kCtTileVecs - 1) / kCtTileVecs;
  if (tiles == 0) tiles = 1;
  uint32_t max_grid = static_cast<uint32_t>(device_cu_count()) * wg_per_cu;
  if (max_grid > kCtMaxGrid) max_grid = kCtMaxGrid;
  const uint32_t tiles_per_wg = (tiles + max_grid - 1) / max_grid;
  geo.grid = (tiles + tiles_per_wg - 1) / tiles_per_wg;
  geo.tiles = tiles;
  return geo;
}

// Workgroups of one instantiation that a CU holds at once, at most WG (asked of the runtime once).
// The kernel's waits are on lower-numbered workgroups of the same launch, and with several rounds a
// workgroup also waits on every workgroup's earlier rounds: the whole grid has to be resident.
template <int DT, bool EXACT, bool EF, int WG>
uint32_t resident_per_cu() {
  static const uint32_t cached = [] {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, compact_kernel<DT, EXACT, EF, WG>, kCtThreads, 0) != hipSuccess)
      nb = 0;
    return static_cast<uint32_t>(std::min(std::max(nb, 0), WG));
  }();
  return cached;
}

}  // namespace
}  // namespace dct

using namespace dct;

extern "C" size_t dct_threshold_compact_workspace_bytes(int dt, uint64_t n) {
  if ((dt != DCT_F32 && dt != DCT_BF16) || n == 0 || n > 0x7FFFFFFFull) return 0;
  return kCtWsBytes;
}

extern "C" int dct_threshold_compact_workspace_init(void* d_ws, size_t ws_bytes, void* hip_stream) {
  if (!d_ws || !is_aligned(d_ws, 256) || ws_bytes < kCtWsBytes) return DCT_ERR_WORKSPACE;
  const uint32_t n_words = static_cast<uint32_t>(kCtWsBytes / 4);
  hipLaunchKernelGGL(compact_ws_init_kernel, dim3((n_words + 255) / 256), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<uint32_t*>(d_ws), n_words);
  return launch_status();
}

namespace {

int launch_compact(const void* g, const void* e_in, void* e_out, int dt, uint64_t n, const dct_threshold* d_thr,
                   int mode, int32_t* d_idx_out, void* d_val_out, uint64_t capacity, uint64_t* d_count_out,
                   void* d_ws, size_t ws_bytes, void* hip_stream) {
  const bool ef = e_out != nullptr;
  if (!g || !d_thr || !d_count_out || n == 0 || n > 0x7FFFFFFFull) return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  if (mode != DCT_GE_TAU && mode != DCT_EXACT_K) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(g, es) || !is_aligned(d_thr, 16) || !is_aligned(d_count_out, 8)) return DCT_ERR_INVALID;
  if (capacity > 0 && (!d_idx_out || !d_val_out || !is_aligned(d_idx_out, 4) || !is_aligned(d_val_out, es)))
    return DCT_ERR_INVALID;
  if (ef) {
    if (dt != DCT_F32 || !e_in) return DCT_ERR_INVALID;
    const uintptr_t ga = reinterpret_cast<uintptr_t>(g), ia = reinterpret_cast<uintptr_t>(e_in),
                    oa = reinterpret_cast<uintptr_t>(e_out);
    // the three vectors are walked with the same 16-byte vectors: same offset within 16 bytes
    if (!is_aligned(e_in, es) || (ia & 15) != (ga & 15) || (oa & 15) != (ga & 15)) return DCT_ERR_INVALID;
    const uintptr_t bytes = static_cast<uintptr_t>(n) * es;
    if (ga < oa + bytes && oa < ga + bytes) return DCT_ERR_INVALID;              // g must not overlap e_out
    if (ia != oa && ia < oa + bytes && oa < ia + bytes) return DCT_ERR_INVALID;  // e_in: identical or disjoint
  }
  if (!d_ws || !is_aligned(d_ws, 256) || ws_bytes < kCtWsBytes) return DCT_ERR_WORKSPACE;

  const bool exact = mode == DCT_EXACT_K;
  const uint32_t cap = capacity > 0xFFFFFFFFull ? 0xFFFFFFFFu : static_cast<uint32_t>(capacity);
  auto* hdr = static_cast<CompactHeader*>(d_ws);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

#define DCT_LAUNCH_COMPACT(DTV, EX, EFV, WGV)                                                                   \
  do {                                                                                                          \
    const uint32_t per_cu = resident_per_cu<DTV, EX, EFV, WGV>();                                               \
    if (per_cu == 0) return DCT_ERR_HIP;                                                                        \
    const CompactGeom geo = make_geom(reinterpret_cast<uintptr_t>(g), n, dt, per_cu);                           \
    hipLaunchKernelGGL((compact_kernel<DTV, EX, EFV, WGV>), dim3(geo.grid), dim3(kCtThreads), 0, s,              \
                       static_cast<const Elem<DTV>::word_t*>(g), static_cast<const Elem<DTV>::word_t*>(e_in),   \
                       static_cast<Elem<DTV>::word_t*>(e_out), geo, d_thr, d_idx_out,                           \
                       static_cast<Elem<DTV>::word_t*>(d_val_out), cap, d_count_out, hdr);                      \
  } while (0)
#define DCT_LAUNCH_COMPACT_MODE(DTV, EFV, WGV)                  \
  do {                                                          \
    if (exact) DCT_LAUNCH_COMPACT(DTV, true, EFV, WGV);         \
    else DCT_LAUNCH_COMPACT(DTV, false, EFV, WGV);              \
  } while (0)
  const int wg = ct_wg_per_cu(ef, dt, n);
  if (ef) {
    DCT_LAUNCH_COMPACT_MODE(DCT_F32, true, 4);
  } else if (dt == DCT_BF16) {
    DCT_LAUNCH_COMPACT_MODE(DCT_BF16, false, 4);
  } else if (wg == 2) {
    DCT_LAUNCH_COMPACT_MODE(DCT_F32, false, 2);
  } else {
    DCT_LAUNCH_COMPACT_MODE(DCT_F32, false, 3);
  }
#undef DCT_LAUNCH_COMPACT_MODE
#undef DCT_LAUNCH_COMPACT
  return launch_status();
}

}  // namespace

extern "C" int dct_threshold_compact(const void* g, int dt, uint64_t n, const dct_threshold* d_thr, int mode,
                                     int32_t* d_idx_out, void* d_val_out, uint64_t capacity, uint64_t* d_count_out,
                                     void* d_ws, size_t ws_bytes, void* hip_stream) {
  return launch_compact(g, nullptr, nullptr, dt, n, d_thr, mode, d_idx_out, d_val_out, capacity, d_count_out, d_ws,
                        ws_bytes, hip_stream);
}

extern "C" int dct_ef_threshold_compact(const void* g, const void* e_in, void* e_out, int dt, uint64_t n,
                                        const dct_threshold* d_thr, int mode, int32_t* d_idx_out, void* d_val_out,
                                        uint64_t capacity, uint64_t* d_count_out, void* d_ws, size_t ws_bytes,
                                        void* hip_stream) {
  if (!e_in || !e_out) return DCT_ERR_INVALID;
  return launch_compact(g, e_in, e_out, dt, n, d_thr, mode, d_idx_out, d_val_out, capacity, d_count_out, d_ws,
                        ws_bytes, hip_stream);
}
