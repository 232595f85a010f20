// dct_threshold_compact: Algorithm 1, mask and compressed gradient (the entries
// with |W_grad| >= tau), as ONE pass over the gradient that writes the survivors
// as (ascending index, value) pairs.
//
// Design (gfx950).  The 8 XCDs of the chip have private L2s, so workgroups can
// only talk to each other through the memory-side path (about a microsecond per
// round trip).  The kernel therefore keeps cross-workgroup traffic to one short
// exchange at the very end:
//   1. One workgroup of 16 wavefronts per CU.  The 16-byte-aligned interior of the
//      vector is cut into pieces of 4 KiB and every workgroup owns a contiguous run
//      of pieces.  Its wavefronts take the pieces ("tickets") one at a time from a
//      counter in LDS: a SIMD serves its oldest wavefront first, so work that is
//      dealt out in advance finishes unevenly and the last wavefronts stream with
//      too few loads in flight.  Two register buffers per wavefront keep the next
//      piece's loads in flight while the current piece is compared.
//   2. Survivors are sparse (<= a few %), so each wavefront appends its
//      (index, value) pairs, in the order it meets them, to its own region of LDS
//      (ballot + lane-prefix ranks), and records per ticket how many pairs it holds
//      and where they start.  No workgroup waits for another while streaming.
//   3. When the chunk is done the workgroup publishes its two counts (keys above
//      tau, ties at tau) in one 64-bit descriptor and reads the descriptors of all
//      lower-numbered workgroups in one go (at most 255: four loads per lane of one
//      wavefront, a single round trip when nobody is late).  Meanwhile the other
//      wavefronts turn the per-ticket counts into exclusive offsets.
//   4. With the exclusive prefix known, every staged pair goes to its final slot:
//      prefix of the workgroup + offset of its ticket + rank inside the ticket.  In
//      exactly-k mode ties are staged with a flag bit and written while fewer than
//      tie_quota ties precede them.
// The survivors of a chunk wait on chip, so the grid as a whole can hold about
// four million of them.  A vector that keeps more (the paper's lower sparsity
// levels) is cut into up to a dozen contiguous slices ("rounds") that the same
// workgroups process one after the other; the last workgroup of a round publishes
// the running total for the next round.  The number of rounds comes from the
// counts in the threshold record.  If a wavefront's LDS region overflows all the
// same (more survivors than the record promised, a tie value that covers much of
// the vector, or more rounds needed than are worth their cost) the workgroup still
// counts everything, and after the exchange streams its chunk a second time,
// writing straight to the final slots.
//
// The first piece of every wavefront is requested before anything the kernel reads
// from the workspace or the threshold record is used (under the assumption of a
// single round, which the record then confirms or not): on a 100 MB vector that
// round trip is a twentieth of the kernel.
//
// Error feedback (Algorithm 1: the residual is added before the mask and refreshed
// after it) rides on the same pass: the EF variant streams g and the residual
// together, forms w = g + e with one fp32 addition per element, writes w as the new
// residual with full 16-byte stores and compacts w.  The residual of a pair that is
// actually written out is then overwritten with +0 in step 4 (a 4-byte store per
// survivor), so an entry that finds no room in the outputs keeps its value in the
// residual.  The second-pass fallback re-reads w from the new residual, which also
// makes updating the residual in place safe.  The EF variant never uses rounds (a
// dense vector takes the second pass instead): a workgroup then only ever waits for
// lower-numbered workgroups, which the device started before it.  Because the
// residual is training state, delivery is all or nothing: workgroup 0 waits for all
// descriptors and publishes one decision word; on "commit" everybody delivers, on
// "abort" (its bounded wait ran out) nobody does and the new residual holds w
// everywhere, so nothing is lost.
//
// All waits are bounded.  The workspace holds two descriptor sets used by alternate
// calls (an epoch word picks the set): every call clears the other set for its
// successor and the last workgroup advances the epoch, so a call is one launch.
#include <algorithm>
#include <cstddef>
#include <mutex>
#include <type_traits>

#include "dct_common.hpp"

namespace dct {
namespace {

constexpr int kCtThreads = 1024;
constexpr int kCtWaves = kCtThreads / kWave;
// 16-byte loads per lane and input stream per piece: 4 KiB pieces; with error feedback two streams of 2 KiB
// (four rows of each would not fit the 128 registers a wavefront of a 1024-thread workgroup may use)
constexpr int ct_rows(bool ef) { return ef ? 2 : 4; }
constexpr uint32_t kCtStageCap = 1024;           // staged pairs per wavefront (8 bytes of LDS each)
constexpr uint32_t kCtMaxTickets = 2048;         // tickets of one workgroup per round
constexpr uint32_t kCtMaxGrid = 256;             // one wavefront reads all lower descriptors with four loads per lane
constexpr uint32_t kCtMaxRounds = 12;            // slices a dense vector is cut into (at most)
constexpr uint32_t kCtMaxVirtual = kCtMaxGrid * kCtMaxRounds;
constexpr uint32_t kCtMagic = 0x44435435u;       // "DCT5"
constexpr uint32_t kCtHeaderBytes = 256;
constexpr uint32_t kTieFlag = 0x80000000u;
constexpr uint32_t kNone = 0xFFFFFFFFu;

// Descriptor: [62] published, [61:31] count A (keys above the cut), [30:0] count E (ties).
constexpr uint64_t kStValid = 1ull << 62;
constexpr uint64_t kPayload = (1ull << 62) - 1;
constexpr uint64_t kCommit = 1, kAbort = 2;      // decision word of a call with error feedback

struct CompactHeader {
  uint32_t magic;
  uint32_t epoch;
  uint32_t error;    // a wait ran out: the workspace has to be initialised again
  uint32_t used[2];  // descriptors of each set that the last call using it wrote (they must be cleared)
  uint32_t pad[59];
};
static_assert(sizeof(CompactHeader) == kCtHeaderBytes, "header size");

struct DescSet {
  uint64_t wg[kCtMaxVirtual];
  uint64_t round_total[16];  // [r]: survivors of rounds 0..r, published by the last workgroup of round r
  uint64_t decision;         // error feedback: workgroup 0's commit / abort
  uint64_t pad[15];
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

// Bounded wait helper: returns false when the budget is used up or another
// workgroup has already reported a failure.
__device__ __forceinline__ bool keep_waiting(uint32_t& spins, uint32_t limit, const uint32_t* error_flag) {
  ++spins;
  if (spins > limit || ((spins & 255u) == 0 && ld_agent(error_flag) != 0)) return false;
  __builtin_amdgcn_s_sleep(1);
  return true;
}

// The descriptors of workgroups 0..w-1 of a round, one wavefront, four per lane: valid once all are
// published.  Lanes beyond w hold an empty published descriptor.
struct DescLoad {
  uint64_t d[4];
  __device__ __forceinline__ void load(const uint64_t* round_wg, uint32_t w) {
    const uint32_t lane = lane_id();
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t i = u * kWave + lane;
      d[u] = i < w ? ld_agent(round_wg + i) : kStValid;
    }
  }
  __device__ __forceinline__ bool all_published() const {
    return ballot64(((d[0] & d[1] & d[2] & d[3]) >> 62) == 0) == 0;
  }
  __device__ __forceinline__ uint64_t sum() const {
    return wave_sum_u64((d[0] & kPayload) + (d[1] & kPayload) + (d[2] & kPayload) + (d[3] & kPayload));
  }
};

// A wait has used up its budget: raise the workspace's failure flag, and return only when that has been
// performed.  Whoever waits afterwards polls once more, so that the order is fixed: either the last poll
// already finds everything published (then this workgroup's outputs are right, and the call is merely reported
// as failed), or the workgroup that writes the count, which needs the same descriptors, finds the flag set.
__device__ __forceinline__ void raise_failure(uint32_t* error_flag) {
  if (lane_id() == 0) {
    const uint32_t old = __hip_atomic_fetch_or(error_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::"v"(old) : "memory");
  }
}

// Sum of the descriptors of workgroups 0..w-1 of this round plus the running total of the previous
// round, once all of them are published.  One wavefront; one round trip when nobody is late.
__device__ uint64_t prefix_of(const uint64_t* round_wg, uint32_t w, const uint64_t* prev_total, uint32_t limit,
                              uint32_t* error_flag, bool& failed) {
  uint32_t spins = 0;
  for (bool last = false;; last = true) {
    do {
      DescLoad dl;
      dl.load(round_wg, w);
      const uint64_t pt = prev_total ? ld_agent(prev_total) : kStValid;
      if (dl.all_published() && (pt >> 62) != 0) return dl.sum() + (pt & kPayload);
    } while (!last && keep_waiting(spins, limit, error_flag));
    if (last) break;
    raise_failure(error_flag);
  }
  failed = true;
  return 0;
}

// Error feedback, workgroup 0: all `grid` descriptors published?  (Bounded; a wait that runs out raises the
// failure flag, so that workgroups that start later deliver nothing either.)
__device__ bool all_workgroups_published(const uint64_t* round_wg, uint32_t grid, uint32_t limit, uint32_t* error_flag) {
  uint32_t spins = 0;
  do {
    DescLoad dl;
    dl.load(round_wg, grid);
    if (dl.all_published()) return true;
  } while (keep_waiting(spins, limit, error_flag));
  raise_failure(error_flag);
  return false;
}

// Error feedback, the other workgroups: workgroup 0's decision and, on commit, the exclusive prefix.
__device__ uint64_t decided_prefix(const uint64_t* round_wg, uint32_t w, const uint64_t* decision, uint32_t limit,
                                   uint32_t* error_flag, bool& commit, bool& failed) {
  uint32_t spins = 0;
  for (bool last = false;; last = true) {
    do {
      DescLoad dl;
      dl.load(round_wg, w);
      const uint64_t dec = ld_agent(decision);
      if (dec == kAbort) {
        commit = false;
        return 0;
      }
      if (dec == kCommit && dl.all_published()) {  // (after a commit every descriptor is published)
        commit = true;
        return dl.sum();
      }
    } while (!last && keep_waiting(spins, limit, error_flag));
    if (last) break;
    raise_failure(error_flag);  // workgroup 0 has not decided within four times its own budget
  }
  commit = false;
  failed = true;
  return 0;
}

// Work description shared by all workgroups (computed on the host).
struct CompactGeom {
  uint32_t head;    // elements before the first 16-byte-aligned vector (< kVec)
  uint32_t n_vec;   // full 16-byte vectors after the head
  uint32_t tail;    // elements after the last full vector (< kVec)
  uint32_t grid;    // workgroups (<= kCtMaxGrid)
  uint32_t pieces;  // pieces of ct_rows() * 64 vectors that cover the full vectors (>= 1)
};

// EF: g is W_grad, e_in the residual E_grad (may be the same buffer as e_out), e_out the new residual.
// EARLY: wavefront 0 looks at the lower workgroups' descriptors before the workgroup's barrier (long chunks).
template <int DT, bool EXACT, bool EF, bool EARLY>
__global__ __launch_bounds__(kCtThreads) void compact_kernel(
    const typename Elem<DT>::word_t* __restrict__ g, const typename Elem<DT>::word_t* e_in,
    typename Elem<DT>::word_t* e_out, CompactGeom geo, const dct_threshold* __restrict__ thr,
    int32_t* __restrict__ idx_out, typename Elem<DT>::word_t* __restrict__ val_out, uint32_t capacity,
    uint64_t* __restrict__ count_out, CompactHeader* hdr, uint32_t spin_limit) {
  static_assert(!EF || DT == DCT_F32, "error feedback is an fp32 addition");
  using E = Elem<DT>;
  using word_t = typename E::word_t;
  constexpr int V = E::kVec;
  constexpr int ROWS = ct_rows(EF);
  constexpr uint32_t PIECE = ROWS * kWave;  // vectors per piece
  __shared__ uint32_t s_idx[kCtWaves][kCtStageCap];
  __shared__ word_t s_val[kCtWaves][kCtStageCap];
  // per ticket: keys above the cut (.x) and ties (.y, exactly-k mode only), then their exclusive sums
  using tcount_t = std::conditional_t<EXACT, uint2, uint32_t>;
  __shared__ tcount_t s_tc[kCtMaxTickets];
  auto tc_get = [&](uint32_t t, uint32_t& a, uint32_t& e) {
    if constexpr (EXACT) {
      const uint2 v = s_tc[t];
      a = v.x;
      e = v.y;
    } else {
      a = s_tc[t];
      e = 0;
    }
  };
  auto tc_put = [&](uint32_t t, uint32_t a, uint32_t e) {
    if constexpr (EXACT) s_tc[t] = make_uint2(a, e);
    else s_tc[t] = a;
  };
  __shared__ uint16_t s_tsrc[kCtMaxTickets];            // per ticket: first staged slot in its wavefront's region
  __shared__ uint32_t s_staged[kCtWaves], s_wave_a[kCtWaves], s_wave_e[kCtWaves];
  __shared__ uint32_t s_scan_a[kCtWaves], s_scan_e[kCtWaves];
  __shared__ uint32_t s_taken, s_commit, s_hdr[5];
  __shared__ uint64_t s_excl;

  const uint32_t wg = blockIdx.x;
  const uint32_t lane = lane_id();
  const uint32_t wave = threadIdx.x / kWave;
  // Which chunk of a round this workgroup owns.  A workgroup waits for the counts of all chunks before
  // its own, so the workgroups that finish last should own the last chunks: consecutive workgroups go to
  // different XCDs, and on MI355X those on the odd XCDs are served more slowly while all stream (their
  // workgroups finish about a tenth later), so the even-numbered workgroups take the lower half of the
  // chunks and the odd-numbered the upper half.  (Wrong guesses cost nothing but that microsecond.)
  const uint32_t chunk = wg;

  const uint32_t tau = thr->tau_key;
  const uint32_t quota = thr->tie_quota;
  const uint32_t thr_gt = thr->n_gt, thr_eq = thr->n_eq;

  // ---- geometry.  A round is a contiguous slice of the pieces, a workgroup's chunk a contiguous run of
  // the slice, a ticket 2^tp_shift consecutive pieces of the chunk (one piece unless the chunk has more
  // than kCtMaxTickets of them).
  uint32_t rounds = 1, pieces_per_round = 0, pieces_per_wg = 0, tp_shift = 0;
  uint32_t my_lo = 0, my_hi = 0, tickets = 0;  // this workgroup's pieces [my_lo, my_hi) of the current round
  auto set_rounds = [&](uint32_t r) {
    rounds = r;
    pieces_per_round = (geo.pieces + rounds - 1) / rounds;
    pieces_per_wg = (pieces_per_round + geo.grid - 1) / geo.grid;
    tp_shift = 0;
    while (((pieces_per_wg + (1u << tp_shift) - 1) >> tp_shift) > kCtMaxTickets) ++tp_shift;
  };
  auto set_round = [&](uint32_t round) {
    const uint32_t slice_lo = min(round * pieces_per_round, geo.pieces);
    const uint32_t slice_hi = min(slice_lo + pieces_per_round, geo.pieces);
    my_lo = min(slice_lo + chunk * pieces_per_wg, slice_hi);
    my_hi = min(my_lo + pieces_per_wg, slice_hi);
    tickets = (my_hi - my_lo + (1u << tp_shift) - 1) >> tp_shift;
  };
  const uint4* gv = reinterpret_cast<const uint4*>(g + geo.head);
  const uint32_t tail_base = geo.head + geo.n_vec * V;
  uint32_t a_excl = 0, e_excl = 0;  // survivors before this workgroup's chunk
  auto ticket_of = [&](uint32_t index) -> uint32_t {
    uint32_t vec = index >= geo.head ? (index - geo.head) / V : 0u;
    vec = min(vec, geo.n_vec ? geo.n_vec - 1u : 0u);  // head elements belong to piece 0, tail elements to the last
    return (vec / PIECE - my_lo) >> tp_shift;
  };

  struct Cursor {
    uint32_t t, piece, end;  // ticket, current piece, one past the ticket's last piece (piece == kNone: nothing left)
  };
  auto ticket_cursor = [&](uint32_t n) -> Cursor {
    if (n >= tickets) return Cursor{n, kNone, kNone};
    const uint32_t lo = my_lo + (n << tp_shift);
    const uint32_t hi = min(lo + (1u << tp_shift), my_hi);
    return Cursor{n, lo, hi};
  };
  auto advance = [&](const Cursor& c) -> Cursor {
    if (c.piece + 1 < c.end) return Cursor{c.t, c.piece + 1, c.end};
    uint32_t n = 0;
    if (lane == 0) n = atomicAdd(&s_taken, 1u);
    return ticket_cursor(__builtin_amdgcn_readfirstlane(n));
  };

  // Two register buffers: the loads of the next piece are in flight while the current one is processed.
  struct Rows {
    uint4 a[ROWS];           // g (or, in the second pass with error feedback, the new residual)
    uint4 b[EF ? ROWS : 1];  // the residual
  };
  Rows va, vb;
  const uint4* bv = EF ? reinterpret_cast<const uint4*>(e_in + geo.head) : nullptr;
  uint4* wv = EF ? reinterpret_cast<uint4*>(e_out + geo.head) : nullptr;
  auto load_piece = [&](Rows& buf, uint32_t p, auto direct_tag) {
    constexpr bool DIRECT = decltype(direct_tag)::value;
    const uint4* av = (EF && DIRECT) ? reinterpret_cast<const uint4*>(e_out + geo.head) : gv;
    constexpr bool kAdd = EF && !DIRECT;
    const uint32_t vec0 = p * PIECE + lane;
    if ((p + 1) * PIECE <= geo.n_vec) {  // uniform: the whole piece is inside the vector
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        buf.a[r] = ld_stream(&av[vec0 + r * kWave]);
        if constexpr (kAdd) buf.b[r] = ld_stream(&bv[vec0 + r * kWave]);
      }
    } else {
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        const uint32_t vi = vec0 + r * kWave;
        buf.a[r] = vi < geo.n_vec ? av[vi] : make_uint4(0, 0, 0, 0);
        if constexpr (kAdd) buf.b[r] = vi < geo.n_vec ? bv[vi] : make_uint4(0, 0, 0, 0);
      }
    }
  };

  // ---- the first piece of every wavefront (ticket = wavefront number; the counter in LDS deals the rest),
  // under the assumption of a single round
  set_rounds(1);
  set_round(0);
  Cursor first = ticket_cursor(wave);
  if (first.piece != kNone) load_piece(va, first.piece, std::false_type{});
  if (threadIdx.x == 0) s_taken = kCtWaves;
  lds_barrier();  // (the loads just issued stay in flight)
  // The workspace header is not needed before the workgroup publishes its counts.  ONE thread reads it
  // and leaves it in LDS for the others: a failure flag that is raised while the workgroup starts must not be
  // seen by some of its wavefronts only.  (That wavefront waits a microsecond here; the others stream on.)
  if (threadIdx.x == 0) {
    // (all loads first, then their uses: these are ordered accesses, and a use between two of them makes the
    // second wait for the first -- five round trips instead of one)
    static_assert(offsetof(CompactHeader, magic) == 0 && offsetof(CompactHeader, epoch) == 4 &&
                      offsetof(CompactHeader, error) == 8 && offsetof(CompactHeader, used) == 12,
                  "the header's first five words are read as two 64-bit words and one of 32 bits");
    const uint64_t* h64 = reinterpret_cast<const uint64_t*>(hdr);
    const uint64_t me = ld_agent(h64), eu = ld_agent(h64 + 1);
    const uint32_t u1 = ld_agent(&hdr->used[1]);
    s_hdr[0] = static_cast<uint32_t>(me);
    s_hdr[1] = static_cast<uint32_t>(me >> 32);
    s_hdr[2] = static_cast<uint32_t>(eu);
    s_hdr[3] = static_cast<uint32_t>(eu >> 32);
    s_hdr[4] = u1;
  }

  // ---- rounds.  All survivors of a workgroup's chunk wait in LDS until the chunk's place in the output
  // is known.  A vector with more survivors than the whole grid can hold at once is cut into `rounds`
  // contiguous slices that are processed one after the other.  The number of rounds is derived from the
  // counts in the threshold record (the same in every workgroup); if it turns out too low, the second-pass
  // fallback of the chunks that overflow keeps the result exact.
  {
    const uint64_t expected = static_cast<uint64_t>(__builtin_amdgcn_readfirstlane(thr_gt)) +
                              __builtin_amdgcn_readfirstlane(thr_eq);  // ties are staged too
    const uint64_t room = static_cast<uint64_t>(geo.grid) * (kCtWaves * kCtStageCap / 8);  // an eighth of the staging
    // Every round costs a pipeline drain and refill; beyond a dozen rounds reading the vector twice (the
    // second-pass fallback) is cheaper.  With error feedback there is one round, always.
    uint32_t r = 1;
    if constexpr (!EF) {
      // (5/8 of the staging: tickets taken on demand do not spread evenly over the wavefronts -- regions that
      // are expected to fill beyond two thirds begin to overflow -- and dealing them in turn streams a fifth slower)
      while (r <= kCtMaxRounds && expected > 5 * room * r) ++r;  // ceil(expected / (5/8 of the staging)), no division
      if (r > kCtMaxRounds) r = 1;
      r = min(r, geo.pieces);
    }
    if (r != 1) {  // the assumption did not hold: the piece requested above is not this wavefront's first
      set_rounds(r);
      set_round(0);
      first = ticket_cursor(wave);
      if (first.piece != kNone) load_piece(va, first.piece, std::false_type{});
    }
  }

  // One pass over the workgroup's chunk of the current round, tickets taken on demand.  DIRECT = false:
  // stage survivors (ties flagged) in LDS, count per ticket; DIRECT = true: the exclusive counts are known,
  // write to the final slots.  `loaded`: the wavefront's first piece is already in va.
  uint32_t wave_a = 0, wave_e = 0;  // staging pass: keys above the cut / ties this wavefront met
  auto pass = [&](auto direct_tag, bool loaded) -> uint32_t {
    constexpr bool DIRECT = decltype(direct_tag)::value;
    constexpr bool kAdd = EF && !DIRECT;
    uint32_t staged = 0;                  // STAGE: pairs appended so far (beyond the region they are only counted)
    uint32_t na = 0, ne = 0;              // of the current ticket
    uint32_t a_before = 0, e_before = 0;  // DIRECT: survivors of the whole vector before the current ticket
    uint32_t tk_start = 0;
    wave_a = 0;
    wave_e = 0;

    // up to NE elements per lane: raw[e], validity, index of element 0
    auto emit = [&](const uint32_t* raw, bool in, uint32_t index0, auto nelem_tag, const uint4* packed = nullptr) {
      constexpr int NE = decltype(nelem_tag)::value;
      constexpr bool kPacked = DT == DCT_BF16 && NE == 8;  // whole bf16 vectors: packed compares (`packed`)
      // Cheap common case first: one compare per element against tau (keys >= tau are the
      // survivors and, in exactly-k mode, the ties), collected in a per-lane bitmap; most rows
      // have none.
      uint32_t ge_bits = 0;
      if constexpr (kPacked) {
        ge_bits = bf16x8_ge_bits(*packed, tau);
      } else {
#pragma unroll
        for (int e = 0; e < NE; ++e) ge_bits |= (raw[e] & E::kKeyMask) >= tau ? (1u << e) : 0u;
      }
      if (!in) ge_bits = 0;
      const uint64_t m_any = ballot64(ge_bits != 0);
      if (m_any == 0) return;
      uint32_t e_bits = 0;
      if constexpr (EXACT) {
        if constexpr (kPacked) {
          e_bits = ~bf16x8_ge_bits(*packed, tau + 1u);  // (tau + 1 may be 0x8000: nothing is at or above it)
        } else {
#pragma unroll
          for (int e = 0; e < NE; ++e) e_bits |= (raw[e] & E::kKeyMask) == tau ? (1u << e) : 0u;
        }
        e_bits &= ge_bits;
      }
      const uint32_t a_bits = ge_bits & ~e_bits;
      uint32_t row_a, row_e;
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

    // piece c.piece, its data in buf; `next_t` is the ticket of the piece this wavefront handles next
    auto step = [&](const Rows& buf, const Cursor& c, uint32_t next_t) {
      const uint32_t p = c.piece;
      if (p == my_lo + (c.t << tp_shift)) {  // the first piece of its ticket
        na = 0;
        ne = 0;
        tk_start = staged;
        if constexpr (DIRECT) {
          tc_get(c.t, a_before, e_before);
          a_before += a_excl;
          e_before += e_excl;
        }
      }
      if (p == 0 && geo.head != 0) {
        const bool in = lane < geo.head;
        const uint32_t raw = edge_element(in, lane);
        emit(&raw, in, lane, std::integral_constant<int, 1>{});
      }
      const uint32_t vec0 = p * PIECE + lane;
      const bool full = (p + 1) * PIECE <= geo.n_vec;
#pragma unroll
      for (int r = 0; r < ROWS; ++r) {
        const uint32_t vi = vec0 + r * kWave;
        const bool in = full || vi < geo.n_vec;
        uint32_t raw[V];
#pragma unroll
        for (int e = 0; e < V; ++e) raw[e] = E::raw(buf.a[r], e);
        if constexpr (kAdd) {
#pragma unroll
          for (int e = 0; e < V; ++e)
            raw[e] = __float_as_uint(__uint_as_float(raw[e]) + __uint_as_float(E::raw(buf.b[r], e)));
          if (in) st_stream(&wv[vi], raw[0], raw[1], raw[2], raw[3]);
        }
        emit(raw, in, geo.head + vi * V, std::integral_constant<int, V>{}, &buf.a[r]);
      }
      if (p == geo.pieces - 1 && geo.tail != 0) {
        const bool in = lane < geo.tail;
        const uint32_t raw = edge_element(in, tail_base + lane);
        emit(&raw, in, tail_base + lane, std::integral_constant<int, 1>{});
      }
      if constexpr (!DIRECT) {
        if (next_t != c.t) {  // the ticket is complete
          wave_a += na;
          wave_e += ne;
          if (lane == 0) {
            tc_put(c.t, na, ne);
            s_tsrc[c.t] = static_cast<uint16_t>(min(tk_start, 0xFFFFu));
          }
        }
      }
    };

    Cursor cur = loaded ? first : ticket_cursor(wave);
    if (!loaded && cur.piece != kNone) load_piece(va, cur.piece, direct_tag);
    while (cur.piece != kNone) {
      const Cursor nxt = advance(cur);
      if (nxt.piece != kNone) load_piece(vb, nxt.piece, direct_tag);
      step(va, cur, nxt.t);
      if (nxt.piece == kNone) break;
      cur = advance(nxt);
      if (cur.piece != kNone) load_piece(va, cur.piece, direct_tag);
      step(vb, nxt, cur.t);
    }
    return staged;
  };

  uint32_t epoch = 0;
  DescSet* mine_set = nullptr;

  for (uint32_t round = 0; round < rounds; ++round) {
    const uint32_t vwg = round * geo.grid + chunk;  // this workgroup's place in the sequence of chunks
    if (round != 0) {
      set_round(round);
      __syncthreads();  // the counter in LDS is set again; the previous round's pairs have left the staging area
    }

    // ---- 1+2: stream the chunk, stage survivors in LDS
    const uint32_t staged = pass(std::false_type{}, round == 0);
    // An early look at the descriptors of the lower-numbered workgroups, by wavefront 0 as soon as it has run out
    // of pieces itself (the others may still be streaming): the workgroups that finish last -- and they set the
    // kernel's time -- find everything published and save the round trip after the barrier (1 GiB: 165 -> 162 us).
    [[maybe_unused]] DescLoad early;
    [[maybe_unused]] bool early_ok = false;
    // (An instantiation of its own, chosen by the host for long chunks: on a 100 MB vector, 95 pieces per
    // workgroup, the look gains nothing, and its mere presence in the code cost 0.4 us of 20.8.)
    if constexpr (EARLY) {
      if (round == 0 && wave == 0 && s_hdr[0] == kCtMagic && s_hdr[2] == 0) {
        DescSet* sets = reinterpret_cast<DescSet*>(reinterpret_cast<char*>(hdr) + kCtHeaderBytes);
        early.load(&sets[s_hdr[1] & 1u].wg[0], chunk);
        early_ok = true;
      }
    }
    // the residual stores of this pass have landed before anything (the +0 of a delivered pair, the
    // second pass's loads) touches the same addresses again
    if constexpr (EF) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (lane == 0) {
      s_staged[wave] = staged;
      s_wave_a[wave] = wave_a;
      s_wave_e[wave] = wave_e;
    }
    __syncthreads();
    if (threadIdx.x == 0) s_taken = kCtWaves;  // for the second pass or the next round

    // ---- workspace.  Never initialised, or a wait ran out in an earlier call: nothing is delivered.  (With
    // error feedback the pass above has stored the corrected gradient as the new residual, so nothing is
    // lost either.)
    if (round == 0) {
      const uint32_t magic = s_hdr[0], poisoned = s_hdr[2], used0 = s_hdr[3], used1 = s_hdr[4];
      epoch = s_hdr[1];
      if (magic != kCtMagic || poisoned != 0) {  // uniform over the workgroup
        if (chunk == geo.grid - 1 && threadIdx.x == 0) *count_out = DCT_COUNT_WORKSPACE_ERROR;  // (the count's one writer)
        return;
      }
      DescSet* sets = reinterpret_cast<DescSet*>(reinterpret_cast<char*>(hdr) + kCtHeaderBytes);
      mine_set = sets + (epoch & 1u);
      DescSet* other = sets + ((epoch & 1u) ^ 1u);  // what the previous call wrote there is cleared for the next call
      const uint32_t used = min((epoch & 1u) ? used0 : used1, kCtMaxVirtual);
      for (uint32_t i = wg * kCtThreads + threadIdx.x; i < used; i += geo.grid * kCtThreads) st_agent(&other->wg[i], 0ull);
      if (wg == 0 && threadIdx.x < 17) st_agent(threadIdx.x < 16 ? &other->round_total[threadIdx.x] : &other->decision, 0ull);
    }

    // ---- 3a: wavefront 0 publishes the workgroup's counts at once ...
    uint64_t mine = 0;
    if (wave == 0) {
      uint32_t ta = 0, te = 0;
#pragma unroll
      for (int w = 0; w < kCtWaves; ++w) {
        ta += s_wave_a[w];
        te += s_wave_e[w];
      }
      mine = pack(ta, te);
      if (lane == 0) st_agent(&mine_set->wg[vwg], kStValid | mine);
    }
    // ---- 3b: ... and while that store travels, the per-ticket counts become exclusive sums
    // (two tickets per thread)
    {
      uint32_t my_a[2] = {0, 0}, my_e[2] = {0, 0};
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const uint32_t t = threadIdx.x * 2 + q;
        if (t < tickets) {
          tc_get(t, my_a[q], my_e[q]);
        }
      }
      const uint32_t sum_a = my_a[0] + my_a[1], sum_e = my_e[0] + my_e[1];
      const uint32_t incl_a = wave_prefix_sum(sum_a);
      const uint32_t incl_e = EXACT ? wave_prefix_sum(sum_e) : 0u;
      if (lane == kWave - 1) {
        s_scan_a[wave] = incl_a;
        s_scan_e[wave] = incl_e;
      }
      __syncthreads();
      uint32_t base_a = 0, base_e = 0;
      for (uint32_t w = 0; w < wave; ++w) {
        base_a += s_scan_a[w];
        base_e += s_scan_e[w];
      }
      const uint32_t ex_a = base_a + incl_a - sum_a, ex_e = base_e + incl_e - sum_e;
      const uint32_t t = threadIdx.x * 2;
      if (t < tickets) {
        tc_put(t, ex_a, ex_e);
      }
      if (t + 1 < tickets) {
        tc_put(t + 1, ex_a + my_a[0], ex_e + my_e[0]);
      }
    }

    // ---- 3c: wavefront 0 obtains the exclusive prefix
    if (wave == 0) {
      bool failed = false, commit = true;
      uint64_t excl;
      const uint64_t* round_wg = &mine_set->wg[round * geo.grid];
      if constexpr (EF) {
        // all or nothing: workgroup 0 decides for the whole grid
        if (wg == 0) {
          commit = all_workgroups_published(round_wg, geo.grid, spin_limit, &hdr->error);
          if (lane == 0) st_agent(&mine_set->decision, commit ? kCommit : kAbort);
          excl = 0;
        } else {
          const uint32_t patient = spin_limit > 0x3FFFFFFFu ? 0xFFFFFFFFu : 4u * spin_limit + 1024u;
          excl = decided_prefix(round_wg, chunk, &mine_set->decision, patient, &hdr->error, commit, failed);
        }
      } else {
        if (early_ok && early.all_published())
          excl = early.sum();
        else
          excl = prefix_of(round_wg, chunk, round ? &mine_set->round_total[round - 1] : nullptr, spin_limit,
                           &hdr->error, failed);
      }
      excl &= kPayload;
      if (lane == 0) {
        if (!EF && chunk == geo.grid - 1 && !failed)
          st_agent(&mine_set->round_total[round], kStValid | ((excl + mine) & kPayload));
        s_excl = excl;
        s_commit = commit && !failed ? 1u : 0u;
        // The count has ONE writer, the workgroup of the last chunk: after its last round (every other
        // workgroup has read the epoch and published by then), or when it gives up.
        if (chunk == geo.grid - 1 && (round == rounds - 1 || failed || !commit)) {
          const uint64_t total = (excl + mine) & kPayload;
          uint64_t c = cnt_a(total);
          if (EXACT) c += min(cnt_e(total), quota);
          const uint32_t err = __builtin_amdgcn_readfirstlane(ld_agent(&hdr->error));
          if (failed || !commit || err != 0) {  // a wait ran out somewhere: the workspace refuses from now on
            *count_out = DCT_COUNT_WORKSPACE_ERROR;
          } else {
            *count_out = c;
            st_agent(&hdr->used[epoch & 1u], rounds * geo.grid);
            st_agent(&hdr->epoch, epoch + 1u);
          }
        }
      }
    }
    __syncthreads();

    // ---- 4: final slots
    // A wait ran out, or (error feedback) workgroup 0 decided that nobody delivers: every pair stays where it
    // is -- with error feedback in the residual.  (Uniform over the workgroup.)
    if (s_commit == 0) return;
    a_excl = cnt_a(s_excl);
    e_excl = cnt_e(s_excl);
    bool overflow = false;
    for (int w = 0; w < kCtWaves; ++w) overflow = overflow || s_staged[w] > kCtStageCap;
    if (overflow) {  // uniform over the workgroup: second pass over the chunk, straight to the outputs
      // With error feedback the second pass reads back what the first one stored (the barriers
      // above have waited for those stores): drop this CU's cached copies of the old lines first.
      if constexpr (EF) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      pass(std::true_type{}, false);
      __syncthreads();
      if (threadIdx.x == 0) s_taken = kCtWaves;
      continue;
    }
    const uint32_t n_staged = s_staged[wave];
    if constexpr (!EXACT) {
      for (uint32_t j0 = 0; j0 < n_staged; j0 += kWave) {
        const uint32_t j = j0 + lane;
        if (j < n_staged) {
          const uint32_t index = s_idx[wave][j];
          const uint32_t t = ticket_of(index);
          const uint32_t slot = a_excl + s_tc[t] + (j - s_tsrc[t]);
          if (slot < capacity) {
            idx_out[slot] = static_cast<int32_t>(index);
            val_out[slot] = s_val[wave][j];
            if constexpr (EF) e_out[index] = 0;  // delivered: nothing is left behind
          }
        }
      }
    } else {
      // The entries of a ticket are consecutive in the wavefront's region, in index order.  An entry's
      // place follows from its ticket's offsets and from the keys above the cut / the ties of the same
      // ticket before it: counted with ballots inside the batch of 64 entries, carried from batch to
      // batch while the ticket stays the same.
      uint32_t prev_t = kNone, carry_a = 0, carry_e = 0;
      for (uint32_t j0 = 0; j0 < n_staged; j0 += kWave) {
        const uint32_t j = j0 + lane;
        const bool valid = j < n_staged;
        const uint32_t ent = valid ? s_idx[wave][j] : 0u;
        const bool tie = valid && (ent & kTieFlag) != 0;
        const uint32_t index = ent & ~kTieFlag;
        const uint32_t t = valid ? ticket_of(index) : kNone - 1u;
        uint32_t t_left = __shfl_up(t, 1, kWave);
        if (lane == 0) t_left = prev_t;
        const uint64_t heads = ballot64(t != t_left);  // lanes that start a ticket
        const uint64_t m_tie = ballot64(tie), m_a = ballot64(valid && !tie);
        const uint64_t lt = (1ull << lane) - 1ull;
        const uint64_t my_heads = heads & (lt | (1ull << lane));
        uint64_t seg = lt;  // the lanes below this one that hold entries of the same ticket
        uint32_t ca = carry_a, ce = carry_e;
        if (my_heads != 0) {
          seg = lt & ~((1ull << (63 - __builtin_clzll(my_heads))) - 1ull);
          ca = 0;
          ce = 0;
        }
        uint32_t off_a = 0, off_e = 0;
        if (valid) tc_get(t, off_a, off_e);
        const uint32_t a_run = a_excl + off_a + ca + static_cast<uint32_t>(__popcll(m_a & seg));
        const uint32_t t_run = e_excl + off_e + ce + static_cast<uint32_t>(__popcll(m_tie & seg));
        // a tie survives while fewer than `quota` ties precede it; kept ties before: min(t_run, quota)
        const uint32_t slot = a_run + min(t_run, quota);
        if (valid && (!tie || t_run < quota) && slot < capacity) {
          idx_out[slot] = static_cast<int32_t>(index);
          val_out[slot] = s_val[wave][j];
          if constexpr (EF) e_out[index] = 0;  // delivered: nothing is left behind
        }
        if (heads != 0) {
          const uint64_t last_seg = ~((1ull << (63 - __builtin_clzll(heads))) - 1ull);
          carry_a = static_cast<uint32_t>(__popcll(m_a & last_seg));
          carry_e = static_cast<uint32_t>(__popcll(m_tie & last_seg));
        } else {
          carry_a += static_cast<uint32_t>(__popcll(m_a));
          carry_e += static_cast<uint32_t>(__popcll(m_tie));
        }
        prev_t = __builtin_amdgcn_readlane(t, kWave - 1);
      }
    }
  }
}

// Head / full vectors / tail split of n elements starting at address `addr`, and the pieces.
CompactGeom make_geom(uintptr_t addr, uint64_t n, int dt, bool ef) {
  const uint32_t es = dt == DCT_F32 ? 4 : 2;
  const uint32_t vec = 16 / es;
  CompactGeom geo;
  uint64_t head = ((16 - (addr & 15)) & 15) / es;
  if (head > n) head = n;
  geo.head = static_cast<uint32_t>(head);
  geo.n_vec = static_cast<uint32_t>((n - head) / vec);
  geo.tail = static_cast<uint32_t>((n - head) % vec);
  const uint32_t piece = ct_rows(ef) * kWave;
  geo.pieces = geo.n_vec / piece + (geo.n_vec % piece != 0 ? 1u : 0u);
  if (geo.pieces == 0) geo.pieces = 1;
  uint32_t max_grid = static_cast<uint32_t>(device_cu_count());  // one workgroup per CU: the grid is resident
  if (max_grid > kCtMaxGrid) max_grid = kCtMaxGrid;
  geo.grid = geo.pieces < max_grid ? geo.pieces : max_grid;
  return geo;
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
  const CompactGeom geo = make_geom(reinterpret_cast<uintptr_t>(g), n, dt, ef);
  const uint32_t spin_limit = wait_limit();

  // the early look at the descriptors pays from about 512 pieces per workgroup on (error feedback decides centrally)
  const bool early = !ef && geo.pieces / geo.grid >= 512;
#define DCT_LAUNCH_COMPACT(DTV, EX, EFV, EAV)                                                                   \
  hipLaunchKernelGGL((compact_kernel<DTV, EX, EFV, EAV>), dim3(geo.grid), dim3(kCtThreads), 0, s,               \
                     static_cast<const Elem<DTV>::word_t*>(g), static_cast<const Elem<DTV>::word_t*>(e_in),     \
                     static_cast<Elem<DTV>::word_t*>(e_out), geo, d_thr, d_idx_out,                             \
                     static_cast<Elem<DTV>::word_t*>(d_val_out), cap, d_count_out, hdr, spin_limit)
#define DCT_LAUNCH_COMPACT_MODE(DTV, EFV, EAV)            \
  do {                                                    \
    if (exact) DCT_LAUNCH_COMPACT(DTV, true, EFV, EAV);   \
    else DCT_LAUNCH_COMPACT(DTV, false, EFV, EAV);        \
  } while (0)
  if (ef) {
    DCT_LAUNCH_COMPACT_MODE(DCT_F32, true, false);
  } else if (dt == DCT_BF16) {
    if (early) DCT_LAUNCH_COMPACT_MODE(DCT_BF16, false, true);
    else DCT_LAUNCH_COMPACT_MODE(DCT_BF16, false, false);
  } else {
    if (early) DCT_LAUNCH_COMPACT_MODE(DCT_F32, false, true);
    else DCT_LAUNCH_COMPACT_MODE(DCT_F32, false, false);
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

// ---------------------------------------------------------------------------------------------
// dct_threshold_compact_static: the same call for callers that can hand over no workspace.  The
// descriptor sets live in a file-scope device array; every GPU the library runs on holds its own copy
// until the process ends.  In host code the array's NAME is a stand-in, not a device address: the address
// on the current device comes from hipGetSymbolAddress, once per device, and only that pointer is passed
// to kernels.
static __device__ __align__(256) unsigned char scratch[kCtWsBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (nullptr on failure).
void* scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" size_t dct_threshold_compact_static_scratch_bytes(void) { return kCtWsBytes; }

extern "C" int dct_threshold_compact_static(const void* g, int dt, uint64_t n, const dct_threshold* d_thr, int mode,
                                            int32_t* d_idx_out, void* d_val_out, uint64_t capacity,
                                            uint64_t* d_count_out, void* hip_stream) {
  if (n == 0 || n > 0x7FFFFFFFull) return DCT_ERR_INVALID;  // beyond the int32 index range: no call of this library takes it
  void* ws = scratch_on_current_device();
  if (ws == nullptr) return DCT_ERR_HIP;
  // The array keeps what the last call on this GPU left there -- possibly a refused state after a wait that
  // ran out -- so every call starts from a freshly initialised workspace (a fill kernel ahead of the
  // compaction on the same stream; no memset node, which callers under graph capture could not replay).
  const int rc = dct_threshold_compact_workspace_init(ws, kCtWsBytes, hip_stream);
  if (rc != DCT_OK) return rc;
  return launch_compact(g, nullptr, nullptr, dt, n, d_thr, mode, d_idx_out, d_val_out, capacity, d_count_out, ws,
                        kCtWsBytes, hip_stream);
}
