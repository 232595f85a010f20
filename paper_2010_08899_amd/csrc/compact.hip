// dct_threshold_compact: Algorithm 1, "M = I(|W_grad| >= tau)" and
// "W_hat = W_grad . M", as ONE pass over the gradient that writes the survivors
// as (ascending index, value) pairs.
//
// Design (gfx950): the vector is cut into tiles of 32 KiB.  A workgroup of four
// wavefronts takes the next tile from a ticket counter, loads it with 16-byte
// coalesced loads into registers (8 per lane), counts its survivors with
// wavefront ballots, publishes the tile count in a 64-bit descriptor and finds
// the number of survivors in all earlier tiles by a decoupled look-back over the
// descriptors of its predecessors.  Tickets are handed out in launch order, so
// every tile a workgroup waits for is already running or finished.  Survivors are
// then written straight from registers to their final slots (ballot + lane-prefix
// ranks), so the input is read from HBM exactly once and nothing but the pairs is
// written.  Exactly-k mode carries a second counter (ties seen so far) through the
// same scan: a tie is kept while fewer than tie_quota ties precede it.
//
// The workspace holds the ticket, a completion counter and the descriptors.  The
// workgroup that finishes last writes the survivor count and returns the
// workspace to its initial (all-zero) state, so a call needs a single launch.
#include "dct_common.hpp"

namespace dct {
namespace {

constexpr int kCtThreads = 256;
constexpr int kCtWaves = kCtThreads / kWave;
constexpr int kCtRows = 8;                       // 16-byte loads per lane per tile
constexpr uint32_t kCtTileBytes = kCtThreads * kCtRows * 16;
constexpr uint32_t kCtMagic = 0x44435431u;       // "DCT1"
constexpr uint32_t kCtHeaderBytes = 256;
constexpr uint32_t kCtSpinLimit = 1u << 20;

// Descriptor: [63:62] status, [61:31] count A (keys above the cut), [30:0] count E (ties).
constexpr uint64_t kStAggregate = 1ull << 62;
constexpr uint64_t kStInclusive = 2ull << 62;
constexpr uint64_t kPayload = (1ull << 62) - 1;

struct CompactHeader {
  uint32_t magic;
  uint32_t ticket;
  uint32_t done;
  uint32_t n_desc;
  uint32_t error;
  uint32_t pad[59];
};
static_assert(sizeof(CompactHeader) == kCtHeaderBytes, "header size");

__device__ __forceinline__ uint64_t pack(uint32_t a, uint32_t e) { return (static_cast<uint64_t>(a) << 31) | e; }
__device__ __forceinline__ uint32_t cnt_a(uint64_t p) { return static_cast<uint32_t>((p & kPayload) >> 31); }
__device__ __forceinline__ uint32_t cnt_e(uint64_t p) { return static_cast<uint32_t>(p & 0x7FFFFFFFu); }

__global__ void compact_ws_init_kernel(uint32_t* ws, uint32_t n_words, uint32_t n_desc) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_words) return;
  uint32_t v = 0;
  if (i == 0) v = kCtMagic;
  if (i == 3) v = n_desc;
  ws[i] = v;
}

// Sum of the counts of all tiles before `tile`.  Called by all lanes of one
// wavefront.  `failed` is set when a predecessor never published (only possible
// with a corrupted workspace): the wait is bounded so the kernel always ends.
__device__ uint64_t look_back(const uint64_t* desc, int tile, bool& failed) {
  const int lane = lane_id();
  uint64_t excl = 0;
  int pos = tile - 1;
  uint32_t spins = 0;
  for (;;) {
    const int i = pos - lane;
    const uint64_t d = (i >= 0) ? ld_agent(desc + i) : kStInclusive;
    const uint32_t st = static_cast<uint32_t>(d >> 62);
    const uint64_t invalid = ballot64(st == 0);
    const uint64_t incl = ballot64(st == 2);
    if (incl != 0) {
      const int f = __builtin_ctzll(incl);
      const uint64_t need = (f == 63) ? ~0ull : ((2ull << f) - 1);
      if ((invalid & need) == 0) {
        excl += wave_sum_u64(lane <= f ? (d & kPayload) : 0ull);
        return excl;
      }
    } else if (invalid == 0) {
      excl += wave_sum_u64(d & kPayload);
      pos -= kWave;
      continue;
    }
    if (++spins > kCtSpinLimit) {
      failed = true;
      return excl;
    }
    __builtin_amdgcn_s_sleep(2);
  }
}

template <int DT, bool GUARDED, bool EXACT>
__device__ __forceinline__ void process_tile(const typename Elem<DT>::word_t* __restrict__ g_al, uint32_t off,
                                             uint32_t n_virt, uint32_t tile, uint32_t t_above, uint32_t tau,
                                             uint32_t quota, int32_t* __restrict__ idx_out,
                                             typename Elem<DT>::word_t* __restrict__ val_out, uint32_t capacity,
                                             uint64_t* desc, CompactHeader* hdr, uint32_t* s_wave_a,
                                             uint32_t* s_wave_e, uint64_t* s_excl) {
  using E = Elem<DT>;
  constexpr int V = E::kVec;
  constexpr uint32_t kTileElems = kCtThreads * kCtRows * V;
  const int lane = lane_id();
  const int wave = threadIdx.x / kWave;
  // Virtual element index of this lane's first element in row 0; row r adds r * 64 * V.
  const uint32_t v0 = tile * kTileElems + (wave * kCtRows * kWave + lane) * V;

  uint4 v[kCtRows];
  uint32_t valid[kCtRows];  // per-element validity bits (all ones on the fast path)
#pragma unroll
  for (int r = 0; r < kCtRows; ++r) {
    const uint32_t vi = v0 + r * kWave * V;
    if constexpr (!GUARDED) {
      v[r] = *reinterpret_cast<const uint4*>(g_al + vi);
      valid[r] = (1u << V) - 1;
    } else {
      uint32_t w[4] = {0, 0, 0, 0};
      uint32_t vm = 0;
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const uint32_t ve = vi + e;
        if (ve >= off && ve < n_virt) {
          const uint32_t x = g_al[ve];
          vm |= 1u << e;
          if constexpr (V == 4) w[e] = x; else w[e >> 1] |= x << (16 * (e & 1));
        }
      }
      v[r] = make_uint4(w[0], w[1], w[2], w[3]);
      valid[r] = vm;
    }
  }

  // ---- count survivors of this wavefront's rows
  uint32_t wa = 0, we = 0;
#pragma unroll
  for (int r = 0; r < kCtRows; ++r) {
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const uint32_t key = E::raw(v[r], e) & E::kKeyMask;
      const bool ok = GUARDED ? ((valid[r] >> e) & 1u) != 0 : true;
      wa += __popcll(ballot64(ok && key >= t_above));
      if constexpr (EXACT) we += __popcll(ballot64(ok && key == tau));
    }
  }
  if (lane == 0) {
    s_wave_a[wave] = wa;
    s_wave_e[wave] = we;
  }
  __syncthreads();

  // ---- wavefront 0: publish the tile count, look back for the exclusive prefix
  if (wave == 0) {
    uint32_t ta = 0, te = 0;
#pragma unroll
    for (int w = 0; w < kCtWaves; ++w) {
      ta += s_wave_a[w];
      te += s_wave_e[w];
    }
    const uint64_t mine = pack(ta, te);
    uint64_t excl = 0;
    if (tile == 0) {
      if (lane == 0) st_agent(desc, kStInclusive | mine);
    } else {
      if (lane == 0) st_agent(desc + tile, kStAggregate | mine);
      bool failed = false;
      excl = look_back(desc, static_cast<int>(tile), failed);
      if (lane == 0) {
        if (failed) atomicOr(&hdr->error, 1u);
        st_agent(desc + tile, kStInclusive | ((excl + mine) & kPayload));
      }
    }
    if (lane == 0) *s_excl = excl;
  }
  __syncthreads();

  // ---- write survivors from registers
  const uint64_t excl = *s_excl;
  uint32_t a_before = cnt_a(excl), e_before = cnt_e(excl);
  for (int w = 0; w < wave; ++w) {
    a_before += s_wave_a[w];
    e_before += s_wave_e[w];
  }
#pragma unroll
  for (int r = 0; r < kCtRows; ++r) {
    bool fa[V], fe[V];
    uint64_t ma[V], me[V];
    uint32_t row_a = 0, row_e = 0;
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const uint32_t key = E::raw(v[r], e) & E::kKeyMask;
      const bool ok = GUARDED ? ((valid[r] >> e) & 1u) != 0 : true;
      fa[e] = ok && key >= t_above;
      ma[e] = ballot64(fa[e]);
      row_a += __popcll(ma[e]);
      if constexpr (EXACT) {
        fe[e] = ok && key == tau;
        me[e] = ballot64(fe[e]);
        row_e += __popcll(me[e]);
      } else {
        fe[e] = false;
        me[e] = 0;
      }
    }
    uint32_t out_base = a_before;
    bool keep[V];
    uint64_t mk[V];
    if constexpr (EXACT) {
      out_base += min(e_before, quota);
      if (row_e == 0 || e_before >= quota) {          // no tie of this row survives
#pragma unroll
        for (int e = 0; e < V; ++e) { keep[e] = fa[e]; mk[e] = ma[e]; }
      } else if (e_before + row_e <= quota) {          // every tie of this row survives
#pragma unroll
        for (int e = 0; e < V; ++e) { keep[e] = fa[e] || fe[e]; mk[e] = ma[e] | me[e]; }
      } else {                                         // the quota runs out inside this row
        uint32_t ties_in_lower_lanes = 0;
#pragma unroll
        for (int e = 0; e < V; ++e) ties_in_lower_lanes += lanes_below(me[e]);
        uint32_t tie_rank = e_before + ties_in_lower_lanes;
#pragma unroll
        for (int e = 0; e < V; ++e) {
          keep[e] = fa[e] || (fe[e] && tie_rank < quota);
          tie_rank += fe[e] ? 1u : 0u;
          mk[e] = ballot64(keep[e]);
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < V; ++e) { keep[e] = fa[e]; mk[e] = ma[e]; }
    }
    uint64_t any = 0;
#pragma unroll
    for (int e = 0; e < V; ++e) any |= mk[e];
    if (any != 0) {
      uint32_t slot = out_base;
#pragma unroll
      for (int e = 0; e < V; ++e) slot += lanes_below(mk[e]);
      const uint32_t vi = v0 + r * kWave * V;
#pragma unroll
      for (int e = 0; e < V; ++e) {
        if (keep[e]) {
          if (slot < capacity) {
            idx_out[slot] = static_cast<int32_t>(vi + e - off);
            val_out[slot] = static_cast<typename E::word_t>(E::raw(v[r], e));
          }
          ++slot;
        }
      }
    }
    a_before += row_a;
    e_before += row_e;
  }
}

template <int DT, bool EXACT>
__global__ __launch_bounds__(kCtThreads) void compact_kernel(
    const typename Elem<DT>::word_t* __restrict__ g_al, uint32_t off, uint32_t n_virt, uint32_t num_tiles,
    const dct_threshold* __restrict__ thr, int32_t* __restrict__ idx_out,
    typename Elem<DT>::word_t* __restrict__ val_out, uint32_t capacity, uint64_t* __restrict__ count_out,
    CompactHeader* hdr) {
  __shared__ uint32_t s_tile;
  __shared__ uint32_t s_flag;
  __shared__ uint32_t s_wave_a[kCtWaves], s_wave_e[kCtWaves];
  __shared__ uint64_t s_excl;
  constexpr uint32_t kTileElems = kCtThreads * kCtRows * Elem<DT>::kVec;
  uint64_t* desc = reinterpret_cast<uint64_t*>(reinterpret_cast<char*>(hdr) + kCtHeaderBytes);

  if (threadIdx.x == 0) {
    const bool ok = hdr->magic == kCtMagic && hdr->n_desc >= num_tiles;
    s_flag = ok ? 1u : 0u;
    s_tile = ok ? atomicAdd(&hdr->ticket, 1u) : 0u;
  }
  __syncthreads();
  if (s_flag == 0) {  // workspace was never initialised: report, touch nothing else
    if (blockIdx.x == 0 && threadIdx.x == 0) *count_out = DCT_COUNT_WORKSPACE_ERROR;
    return;
  }
  const uint32_t tile = s_tile;
  if (tile >= num_tiles) {  // ticket counter was not zero on entry: corrupted workspace
    if (threadIdx.x == 0) {
      *count_out = DCT_COUNT_WORKSPACE_ERROR;
      st_agent(&hdr->magic, 0u);
    }
    return;
  }
  const uint32_t tau = thr->tau_key;
  const uint32_t quota = thr->tie_quota;
  const uint32_t t_above = EXACT ? tau + 1u : tau;

  const uint32_t lo = tile * kTileElems;
  const bool full = lo >= off && static_cast<uint64_t>(lo) + kTileElems <= n_virt;
  if (full) {
    process_tile<DT, false, EXACT>(g_al, off, n_virt, tile, t_above, tau, quota, idx_out, val_out, capacity, desc,
                                   hdr, s_wave_a, s_wave_e, &s_excl);
  } else {
    process_tile<DT, true, EXACT>(g_al, off, n_virt, tile, t_above, tau, quota, idx_out, val_out, capacity, desc,
                                  hdr, s_wave_a, s_wave_e, &s_excl);
  }

  // ---- completion: the workgroup that finishes last reports the count and
  // clears the workspace for the next call.
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t prev = __hip_atomic_fetch_add(&hdr->done, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    s_flag = (prev == num_tiles - 1) ? 1u : 0u;
  }
  __syncthreads();
  if (s_flag != 0) {
    const uint64_t total = ld_agent(desc + (num_tiles - 1));
    const bool bad = ld_agent(&hdr->error) != 0 || (total >> 62) != 2;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < num_tiles; i += kCtThreads) st_agent(desc + i, 0ull);
    if (threadIdx.x == 0) {
      uint64_t c = cnt_a(total);
      if (EXACT) c += min(cnt_e(total), quota);
      *count_out = bad ? DCT_COUNT_WORKSPACE_ERROR : c;
      st_agent(&hdr->ticket, 0u);
      st_agent(&hdr->done, 0u);
      st_agent(&hdr->error, 0u);
      if (bad) st_agent(&hdr->magic, 0u);  // force a re-initialisation
    }
  }
}

uint32_t tile_elems(int dt) { return kCtTileBytes / (dt == DCT_F32 ? 4 : 2); }

}  // namespace
}  // namespace dct

using namespace dct;

extern "C" size_t dct_threshold_compact_workspace_bytes(int dt, uint64_t n) {
  if ((dt != DCT_F32 && dt != DCT_BF16) || n == 0 || n > 0x7FFFFFFFull) return 0;
  // One descriptor per tile; +1 tile because a misaligned base shifts the tiling.
  const uint64_t tiles = (n + 8) / tile_elems(dt) + 2;
  return kCtHeaderBytes + tiles * sizeof(uint64_t);
}

extern "C" int dct_threshold_compact_workspace_init(void* d_ws, size_t ws_bytes, void* hip_stream) {
  if (!d_ws || !is_aligned(d_ws, 256) || ws_bytes < kCtHeaderBytes + 8 || ws_bytes > 0xFFFFFFFFull)
    return DCT_ERR_WORKSPACE;
  const uint32_t n_words = static_cast<uint32_t>(ws_bytes / 4);
  const uint32_t n_desc = static_cast<uint32_t>((ws_bytes - kCtHeaderBytes) / 8);
  hipLaunchKernelGGL(compact_ws_init_kernel, dim3((n_words + 255) / 256), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<uint32_t*>(d_ws), n_words, n_desc);
  return launch_status();
}

extern "C" int dct_threshold_compact(const void* g, int dt, uint64_t n, const dct_threshold* d_thr, int mode,
                                     int32_t* d_idx_out, void* d_val_out, uint64_t capacity, uint64_t* d_count_out,
                                     void* d_ws, size_t ws_bytes, void* hip_stream) {
  if (!g || !d_thr || !d_count_out || n == 0 || n > 0x7FFFFFFFull) return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  if (mode != DCT_GE_TAU && mode != DCT_EXACT_K) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(g, es) || !is_aligned(d_thr, 16) || !is_aligned(d_count_out, 8)) return DCT_ERR_INVALID;
  if (capacity > 0 && (!d_idx_out || !d_val_out || !is_aligned(d_idx_out, 4) || !is_aligned(d_val_out, es)))
    return DCT_ERR_INVALID;
  if (!d_ws || !is_aligned(d_ws, 256)) return DCT_ERR_WORKSPACE;

  // Tiles are laid over the 16-byte-aligned address range that covers g: `off`
  // leading virtual elements (and the ones past n) are masked out.
  const uintptr_t addr = reinterpret_cast<uintptr_t>(g);
  const uint32_t off = static_cast<uint32_t>((addr & 15) / es);
  const uint64_t n_virt = n + off;
  const uint32_t te = tile_elems(dt);
  const uint32_t num_tiles = static_cast<uint32_t>((n_virt + te - 1) / te);
  if (ws_bytes < kCtHeaderBytes + static_cast<uint64_t>(num_tiles) * 8) return DCT_ERR_WORKSPACE;
  const void* g_al = reinterpret_cast<const void*>(addr & ~static_cast<uintptr_t>(15));
  const uint32_t cap = capacity > 0xFFFFFFFFull ? 0xFFFFFFFFu : static_cast<uint32_t>(capacity);
  auto* hdr = static_cast<CompactHeader*>(d_ws);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const dim3 grid(num_tiles), block(kCtThreads);

#define DCT_LAUNCH_COMPACT(DTV, EX)                                                                              \
  hipLaunchKernelGGL((compact_kernel<DTV, EX>), grid, block, 0, s,                                               \
                     static_cast<const Elem<DTV>::word_t*>(g_al), off, static_cast<uint32_t>(n_virt), num_tiles, \
                     d_thr, d_idx_out, static_cast<Elem<DTV>::word_t*>(d_val_out), cap, d_count_out, hdr)
  if (dt == DCT_F32) {
    if (mode == DCT_EXACT_K) DCT_LAUNCH_COMPACT(DCT_F32, true); else DCT_LAUNCH_COMPACT(DCT_F32, false);
  } else {
    if (mode == DCT_EXACT_K) DCT_LAUNCH_COMPACT(DCT_BF16, true); else DCT_LAUNCH_COMPACT(DCT_BF16, false);
  }
#undef DCT_LAUNCH_COMPACT
  return launch_status();
}
