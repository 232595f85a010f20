// Forward kernel of dct_rowtopk_fwd (Algorithm 2, forward loop: per row the k largest
// |X_act,i|) for NARROW bf16 rows: up to 1024 columns, four or eight rows per wavefront.
//
// The one-row-per-wavefront kernel (rowtopk_fast.hpp) spends about 250 vector instructions
// per row on work that does not depend on the row's width (wave scans, the walks over the
// window keys and the survivors, the output code), which is what limits it below 2048
// columns.  Here every row of a group of four consecutive rows lives on one DPP row of 16
// lanes -- or, for rows of up to 256 columns when there are very many of them, every row of a
// group of eight on half a DPP row: the per-lane work (packed 16-bit compares, bitmaps, bit
// walks) is the same code, the per-row reductions and scans are DPP operations inside the
// row's lanes, and the fixed work is paid once per group.  What is uniform per row (the
// threshold, the counts, the window) is held per lane, equal within a row.
//
// The search for tau_i is the windowed one of the wide kernel: the row in the same slot of the
// previous group predicts a window of 32 to 128 key values (wider for narrower rows, see
// window_width); two compare sweeps give the bitmaps at its ends, the keys inside it are
// histogrammed (one LDS bin per key value and row, scanned by the row's lanes).  The
// prediction is a running mean of the slot's thresholds (narrow rows vary more from one to
// the next than wide ones); a wavefront's first group predicts from a sample of each row.
// Rows whose window misses gallop away from it and are then bracketed by bisection over the
// window positions, in lock step for the rows of the group.
#pragma once

#include "dct_common.hpp"
#include "rowtopk_fast.hpp"

namespace dct {
namespace quad {

using fast::kSampleRegs;
using fast::pk_add_u16;
using fast::pk_lshr15_u16;
using fast::pk_sub_u16;
using fast::wave_lds_fence;

// Wavefronts per workgroup: 4, or -- when every wavefront of a full chip has several groups to do -- 16, one
// workgroup per CU whose wavefronts take the groups from a counter in LDS (a SIMD serves its oldest wavefront
// first; dealt out in advance, the groups of the last wavefronts set the kernel's time.  512 MiB of rows:
// D = 256 246 -> 233 us, 512 175 -> 157 us, 1024 154 -> 136 us; below 64 k rows the small workgroups, which
// spread over all CUs, are as fast or faster).
constexpr int kWavesSmall = 4;
constexpr int kWavesLarge = 16;
constexpr int kRows = 4;               // rows per wavefront: one DPP row of 16 lanes each ...
constexpr int kRowsNarrow = 8;         // ... or, for rows of up to 256 columns, half a DPP row each
constexpr uint32_t kMaxD = 1024;
constexpr uint32_t kMaxDNarrow = 256;    // (eight rows of 512 columns, 14 wavefronts per CU for the LDS: 152 us against 135)
constexpr uint32_t kStageSlots = kWave * 8;  // survivor columns of a group's rows: rows * k <= kStageSlots
// Width of the prediction window in key values.  The threshold of a narrow row moves more from row to row
// (the standard deviation of the k-th largest of D keys grows like 1/sqrt(D): about 17 key values at D = 256,
// 12 at 512, 8 at 1024 for 5 % of post-ReLU normal values).  A window that misses costs the whole group a
// gallop and a bisection with a count sweep each plus a second pair of bitmaps; a wider window costs more keys
// to histogram.  Lanes with 16 or more key registers first try the NEIGHBOURING window after a miss (one sweep:
// it shares an end with the failed one), which makes a narrow window affordable again.  Measured on 512 MiB of
// rows, four rows per wavefront: D = 256 229 -> 206 us with 128 key values instead of 32 (192 us with the second
// compare sweep in place of the remembered bins); D = 512 153 -> 134 us with 64, 128 us with 32 and the
// neighbour step; D = 1024 (32 key values) 126 -> 117 us with the neighbour step, 150 us with 64 and without.
// Eight rows of 256 columns per wavefront: 156 us with 128 key values, 146 us with 64 and the neighbour step
// (32: the same).
constexpr uint32_t window_width(int row_cols, int regs) {
  if (regs >= 16) return row_cols <= 256 ? 64u : 32u;  // a near miss is cheap there (the neighbouring window)
  return row_cols <= 256 ? 128u : row_cols <= 512 ? 64u : 32u;
}

// The reductions and scans of a row: LANES = 16 (a DPP row) or 8 (half a DPP row) neighbouring lanes.
// Sum over the lanes of a row, delivered to every lane of the row.
template <int LANES>
__device__ __forceinline__ uint32_t row_sum(uint32_t x) {
  uint32_t v = x;
  v += __builtin_amdgcn_update_dpp(0u, v, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0u, v, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0u, v, 0x141, 0xf, 0xf, false);  // row_half_mirror
  if constexpr (LANES == 16) v += __builtin_amdgcn_update_dpp(0u, v, 0x140, 0xf, 0xf, false);  // row_mirror
  return v;
}
// Inclusive prefix sum over the lanes of a row (lower lanes first); s = this lane's number in its row.  The DPP
// shifts run over the 16 lanes of a DPP row: with 8-lane rows a lane drops what comes from the other half.
template <int LANES>
__device__ __forceinline__ uint32_t row_incl_scan(uint32_t x, uint32_t s) {
  uint32_t v = x;
  if constexpr (LANES == 16) {
    v += __builtin_amdgcn_update_dpp(0u, v, 0x111, 0xf, 0xf, false);  // row_shr:1
    v += __builtin_amdgcn_update_dpp(0u, v, 0x112, 0xf, 0xf, false);  // row_shr:2
    v += __builtin_amdgcn_update_dpp(0u, v, 0x114, 0xf, 0xf, false);  // row_shr:4
    v += __builtin_amdgcn_update_dpp(0u, v, 0x118, 0xf, 0xf, false);  // row_shr:8
  } else {
    uint32_t t = __builtin_amdgcn_update_dpp(0u, v, 0x111, 0xf, 0xf, false);
    v += s >= 1u ? t : 0u;
    t = __builtin_amdgcn_update_dpp(0u, v, 0x112, 0xf, 0xf, false);
    v += s >= 2u ? t : 0u;
    t = __builtin_amdgcn_update_dpp(0u, v, 0x114, 0xf, 0xf, false);
    v += s >= 4u ? t : 0u;
  }
  return v;
}
// Inclusive suffix sum over the lanes of a row (this lane and the higher ones).
template <int LANES>
__device__ __forceinline__ uint32_t row_suffix_scan(uint32_t x, uint32_t s) {
  uint32_t v = x;
  if constexpr (LANES == 16) {
    v += __builtin_amdgcn_update_dpp(0u, v, 0x101, 0xf, 0xf, false);  // row_shl:1
    v += __builtin_amdgcn_update_dpp(0u, v, 0x102, 0xf, 0xf, false);  // row_shl:2
    v += __builtin_amdgcn_update_dpp(0u, v, 0x104, 0xf, 0xf, false);  // row_shl:4
    v += __builtin_amdgcn_update_dpp(0u, v, 0x108, 0xf, 0xf, false);  // row_shl:8
  } else {
    uint32_t t = __builtin_amdgcn_update_dpp(0u, v, 0x101, 0xf, 0xf, false);
    v += s < 7u ? t : 0u;
    t = __builtin_amdgcn_update_dpp(0u, v, 0x102, 0xf, 0xf, false);
    v += s < 6u ? t : 0u;
    t = __builtin_amdgcn_update_dpp(0u, v, 0x104, 0xf, 0xf, false);
    v += s < 4u ? t : 0u;
  }
  return v;
}
// The ballot bits of this lane's row.
template <int LANES>
__device__ __forceinline__ uint32_t row_ballot(bool p, uint32_t lane) {
  return static_cast<uint32_t>(ballot64(p) >> (lane & (64u - LANES))) & ((1u << LANES) - 1u);
}

// NV = 16-byte vectors per lane: a lane owns NV * 8 contiguous columns, a row (64 / ROWS) * NV * 8.
// ENC (RowEnc): how the mask is written (32- or 16-bit column indices, or a bitmap of ceil(D/32) words per row).
// ROWS = rows per wavefront, 4 or 8.  The work that does not depend on the row's width (scans, the loops over
// window keys and survivors, the output code) is paid per group: eight rows of 256 columns per wavefront cost
// about what four rows of 512 do (512 MiB of 256-column rows: 192 -> 156 us).
template <int NV, int ENC, int WAVES, int ROWS>
__global__ __launch_bounds__(WAVES * kWave) void rowtopk_fwd_quad_kernel(
    const uint16_t* __restrict__ x, uint32_t B, uint32_t D, uint64_t stride, uint32_t k, void* __restrict__ idx_out,
    uint16_t* __restrict__ val_out, uint16_t* __restrict__ tau_out) {
  constexpr int COLS = NV * 8;                  // columns per lane
  constexpr int REGS = COLS / 2;                // packed key registers per lane (2 columns each)
  constexpr int RPW = REGS < 16 ? REGS : 16;    // registers per bitmap word
  constexpr int WORDS = (REGS + 15) / 16;
  static_assert(WORDS <= 2, "a lane owns at most 64 columns");
  constexpr int CHUNK = (NV + 1) * 16;          // LDS bytes per lane chunk (16 bytes of padding)
  constexpr int kColsPerWord = 2 * RPW;
  constexpr int wB = WORDS - 1;
  constexpr int kWaves = WAVES;
  constexpr int kRows = ROWS;
  constexpr int kLanes = kWave / kRows;  // lanes per row
  static_assert(ROWS == 4 || ROWS == 8, "a row is a DPP row of 16 lanes or half of one");
  constexpr uint32_t kWindow = window_width(NV * 8 * kLanes, REGS);
  constexpr int kBinBits = kWindow == 128 ? 7 : kWindow == 64 ? 6 : 5;
  constexpr int kBinsPerLane = kWindow / kLanes;  // lane s of a row scans bins [s * kBinsPerLane, ...)
  constexpr int kListMax = 32 / kBinBits;         // window keys a stream remembers (bin numbers in one register)
  __shared__ uint4 s_row[kWaves][kWave * (NV + 1)];
  __shared__ __attribute__((aligned(16))) uint32_t s_hist[kWaves][kRows][kWindow];

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t lane = lane_id();
  const uint32_t g = lane / kLanes, s = lane % kLanes;  // row of the group, lane of the row
  char* row_lds = reinterpret_cast<char*>(s_row[wave]);
  uint32_t* hist = s_hist[wave][g];
  const uint32_t n_vec = D / 8;  // the host guarantees whole 16-byte vectors, n_vec <= 16 * NV

  // 16-bit key material of local column lc of this lane
  auto key_at = [&](uint32_t lc) {
    return static_cast<uint32_t>(*reinterpret_cast<const uint16_t*>(row_lds + __umul24(lane, CHUNK) + lc * 2));
  };
  // the stored element of column col of row rg of the group, bit for bit
  auto raw_at = [&](uint32_t rg, uint32_t col) -> uint32_t {
    return *reinterpret_cast<const uint16_t*>(row_lds + __umul24(rg * kLanes + col / COLS, CHUNK) + (col % COLS) * 2);
  };
  // the 16 padding bytes of every lane chunk hold the ordered lists of surviving columns (row rg at rg * k)
  auto stage_at = [&](uint32_t slot) {
    return reinterpret_cast<uint16_t*>(row_lds + __umul24(slot >> 3, CHUNK) + NV * 16 + (slot & 7u) * 2);
  };

  constexpr uint32_t kNone = 0xFFFFFFFFu;
  uint32_t guess = kNone;  // tau of this lane's row slot in the previous group; none yet

  const uint64_t n_groups = (static_cast<uint64_t>(B) + kRows - 1) / kRows;
  const uint64_t group_step = static_cast<uint64_t>(gridDim.x) * kWaves;
  // The workgroup's groups are blocks of kWaves consecutive ones, one block in every stripe of the grid; its
  // wavefronts take them one at a time, in order (the n-th group taken increases with n: a wavefront that is
  // handed a group past the end is done).
  __shared__ uint32_t s_taken;
  if (threadIdx.x == 0) s_taken = 0;
  __syncthreads();
  auto take_group = [&]() -> uint64_t {
    uint32_t n = 0;
    if (lane == 0) n = atomicAdd(&s_taken, 1u);
    n = __builtin_amdgcn_readfirstlane(n);
    return static_cast<uint64_t>(blockIdx.x) * kWaves + (n % kWaves) + static_cast<uint64_t>(n / kWaves) * group_step;
  };
  uint64_t grp = take_group();
  uint4 nxt[NV];
  auto load_group = [&](uint64_t gi) {
    const uint64_t row = gi * kRows + g;
    const uint4* xr = reinterpret_cast<const uint4*>(x + row * stride);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const uint32_t q = j * kLanes + s;
      nxt[j] = (row < B && q < n_vec) ? ld_stream(&xr[q]) : make_uint4(0, 0, 0, 0);
    }
  };
  if (grp < n_groups) load_group(grp);

  uint64_t next_grp = 0;
  for (; grp < n_groups; grp = next_grp) {
    const uint64_t my_row = grp * kRows + g;
    // ---- 1. rows -> LDS (padded) -> registers, lane-contiguous within each row
    wave_lds_fence();  // the previous group's readers are done with the buffer
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const uint32_t q = j * kLanes + s;
      *reinterpret_cast<uint4*>(row_lds + __umul24(g * kLanes + q / NV, CHUNK) + (q % NV) * 16) = nxt[j];
    }
    wave_lds_fence();
    next_grp = take_group();
    if (next_grp < n_groups) load_group(next_grp);
    uint32_t R[4 * NV];
#pragma unroll
    for (int m = 0; m < NV; ++m) {
      const uint4 v = *reinterpret_cast<const uint4*>(row_lds + __umul24(lane, CHUNK) + m * 16);
      R[4 * m + 0] = v.x;
      R[4 * m + 1] = v.y;
      R[4 * m + 2] = v.z;
      R[4 * m + 3] = v.w;
    }
    // K[RPW*w + i] = 16-bit keys of columns (2*RPW*w + i, 2*RPW*w + RPW + i), bit 15 of each half set
    uint32_t K[REGS];
#pragma unroll
    for (int w = 0; w < WORDS; ++w) {
#pragma unroll
      for (int i = 0; i < RPW; ++i) {
        const uint32_t a = R[RPW * w + i / 2], b2 = R[RPW * w + RPW / 2 + i / 2];
        const uint32_t pair = __builtin_amdgcn_perm(b2, a, (i & 1) ? 0x07060302u : 0x05040100u);
        K[RPW * w + i] = (pair & 0x7FFF7FFFu) | 0x80008000u;
      }
    }

    // per-lane bitmap of the keys >= t (t <= 0x8000; t may differ from row to row)
    auto ge_bitmap = [&](uint32_t t, uint32_t* out) {
      const uint32_t t2 = t | (t << 16);
#pragma unroll
      for (int w = 0; w < WORDS; ++w) {
        uint32_t a = 0;
#pragma unroll
        for (int i = 0; i < RPW; ++i)
          a = ((a >> 1) & ~0x80008000u) | (pk_sub_u16(K[RPW * w + i], t2) & 0x80008000u);
        out[w] = RPW == 16 ? a : (((a & 0xFFFFu) >> (16 - RPW)) | ((a >> (32 - 2 * RPW)) & ~((1u << RPW) - 1u)));
      }
    };
    // number of keys >= t in this lane's row
    auto count_ge = [&](uint32_t t) {
      const uint32_t t2 = t | (t << 16);
      uint32_t acc = 0;
#pragma unroll
      for (int i = 0; i < REGS; ++i) acc = pk_add_u16(acc, pk_lshr15_u16(pk_sub_u16(K[i], t2)));
      return row_sum<kLanes>((acc & 0xFFFFu) + (acc >> 16));
    };
    // two independent bit streams per step (see the wide kernel)
    auto pop2 = [&](uint32_t& mA, uint32_t& mB, bool& vA, uint32_t& cA, bool& vB, uint32_t& cB) {
      vA = mA != 0;
      cA = vA ? __builtin_ctz(mA) : 0u;
      mA &= mA - 1;
      if constexpr (WORDS == 2) {
        vB = mB != 0;
        cB = kColsPerWord + (vB ? __builtin_ctz(mB) : 0u);
        mB &= mB - 1;
      } else {
        vB = mA != 0;
        cB = vB ? 31u - __builtin_clz(mA) : 0u;
        mA &= ~(vB ? (1u << cB) : 0u);
      }
    };

    // ---- 2. locate tau of every row
    uint32_t above[WORDS], inwin[WORDS];
    uint32_t wlo = 0, n_above = 0, n_win = 0;
    auto window_at = [&](uint32_t lo_end) {
      wlo = lo_end;
      uint32_t lo_bits[WORDS];
      ge_bitmap(wlo, lo_bits);
      ge_bitmap(wlo + kWindow, above);
      uint32_t ca = 0, cw = 0;
#pragma unroll
      for (int w = 0; w < WORDS; ++w) {
        inwin[w] = lo_bits[w] & ~above[w];
        ca += __popc(above[w]);
        cw += __popc(inwin[w]);
      }
      const uint32_t both = row_sum<kLanes>(ca | (cw << 16));  // each count is at most 1024
      n_above = both & 0xFFFFu;
      n_win = both >> 16;
    };
    if (guess == kNone && REGS > kSampleRegs) {
      // no previous group (uniform): estimate tau as the matching order statistic of a sample of the row
      // (kSampleRegs registers of every lane), by bisection over all 15 key bits
      const uint32_t ks = max(1u, (k * kSampleRegs + REGS - 1) / REGS);
      uint32_t t = 0;
      for (int bit = 14; bit >= 0; --bit) {
        const uint32_t cand = t | (1u << bit);
        const uint32_t t2 = cand | (cand << 16);
        uint32_t acc = 0;
#pragma unroll
        for (int i = 0; i < kSampleRegs; ++i) acc = pk_add_u16(acc, pk_lshr15_u16(pk_sub_u16(K[i], t2)));
        if (row_sum<kLanes>((acc & 0xFFFFu) + (acc >> 16)) >= ks) t = cand;
      }
      guess = t;
    }
    const bool have = guess != kNone;
    {
      uint32_t lo_end = have ? (guess >= kWindow / 2 ? guess - kWindow / 2 : 0u) : 0u;
      lo_end = min(lo_end, 0x8000u - kWindow);
      window_at(lo_end);
    }
    bool hit = have && n_above < k && k <= n_above + n_win;
    if (REGS >= 16 && ballot64(have && !hit) != 0) {
      // Most misses are near misses: try the neighbouring window first.  It shares an end with the failed one, so
      // one compare sweep (at its far end) and one count suffice; rows that hit keep what they have.  (Worth it
      // for long lanes only, where the general path's count sweeps and second pair of bitmaps are expensive.)
      const bool up = n_above >= k;
      const bool can = have && !hit && (up ? wlo + 2u * kWindow <= 0x8000u : wlo >= kWindow);
      uint32_t far[WORDS];
      ge_bitmap(up ? wlo + 2u * kWindow : wlo - kWindow, far);
      uint32_t cf = 0;
#pragma unroll
      for (int w = 0; w < WORDS; ++w) cf += __popc(far[w]);
      const uint32_t n_far = row_sum<kLanes>(cf);  // keys at or above the neighbour's far end
      if (can) {
        if (up) {  // [wlo + W, wlo + 2 W): its lower end is the old upper end
          n_win = n_above - n_far;
          n_above = n_far;
#pragma unroll
          for (int w = 0; w < WORDS; ++w) {
            inwin[w] = above[w] & ~far[w];
            above[w] = far[w];
          }
          wlo += kWindow;
        } else {   // [wlo - W, wlo): its upper end is the old lower end
          const uint32_t n_lo_old = n_above + n_win;
          n_win = n_far - n_lo_old;
          n_above = n_lo_old;
#pragma unroll
          for (int w = 0; w < WORDS; ++w) {
            const uint32_t lo_old = above[w] | inwin[w];
            inwin[w] = far[w] & ~lo_old;
            above[w] = lo_old;
          }
          wlo -= kWindow;
        }
        hit = n_above < k && k <= n_above + n_win;
      }
    }
    if (ballot64(!hit) != 0) {
      // Brackets in units of the window width, per row: count_ge(lo_u * width) >= k > count_ge(hi_u * width).
      // Rows that hit take no part (their bracket is closed from the start).  Every count is taken by all
      // four rows together; a row that does not need it probes a harmless position and ignores the result.
      uint32_t lo_u = 0, hi_u = 0x8000u / kWindow;
      const bool up = n_above >= k;  // tau is at or above the failed window's upper end
      bool gallop = have && !hit;
      if (gallop) {
        if (up) lo_u = (wlo + kWindow) / kWindow;   // rounded down: still has >= k keys at or above it
        else hi_u = (wlo + kWindow - 1) / kWindow;  // rounded up: still has < k keys at or above it
      }
      if (hit) hi_u = lo_u + 1;
      // gallop away from the failed window in the direction the counts point to: most misses are near misses
      for (uint32_t step = 1; ballot64(gallop) != 0; step *= 2) {
        const uint32_t probe = up ? min(lo_u + step, hi_u) : (hi_u > step ? hi_u - step : 0u);
        const uint32_t c = count_ge(probe * kWindow);
        if (gallop) {
          if (up) {
            if (probe == hi_u) gallop = false;
            else if (c >= k) lo_u = probe;
            else { hi_u = probe; gallop = false; }
          } else {
            if (probe == 0u) gallop = false;
            else if (c < k) hi_u = probe;
            else { lo_u = probe; gallop = false; }
          }
        }
      }
      while (ballot64(hi_u - lo_u > 1) != 0) {
        const uint32_t mid = (lo_u + hi_u) / 2;
        const uint32_t c = count_ge(mid * kWindow);  // every lane of the row agrees
        if (hi_u - lo_u > 1) {
          if (c >= k) lo_u = mid; else hi_u = mid;
        }
      }
      window_at(hit ? wlo : lo_u * kWindow);  // a row that had hit gets its window again
    }

    // histogram of the keys inside the window: bin = key - wlo, kWindow bins per row
    {
      uint4* hz = reinterpret_cast<uint4*>(&s_hist[wave][0][0]);  // 16 bytes per lane and step
      constexpr uint32_t kHistVecs = kRows * kWindow / 4;
#pragma unroll
      for (uint32_t i = 0; i < (kHistVecs + kWave - 1) / kWave; ++i)
        if (i * kWave + lane < kHistVecs) hz[i * kWave + lane] = make_uint4(0, 0, 0, 0);
    }
    wave_lds_fence();
    // Lanes with few key registers (rows of up to 256 columns) compare them with tau once more at the end;
    // the others remember the bins of their window keys per stream, so that the second walk needs no LDS reads.
    constexpr bool kSweepAgain = REGS <= 8 || ROWS == 8;
    [[maybe_unused]] uint32_t listA = 0, listB = 0;
    [[maybe_unused]] bool list_full = false;
    [[maybe_unused]] uint32_t n_pops = 0;
    {
      uint32_t mA = inwin[0], mB = WORDS == 2 ? inwin[wB] : 0u;
      uint32_t sh = 0;
      while (ballot64((mA | mB) != 0) != 0) {
        bool vA, vB;
        uint32_t cA, cB;
        pop2(mA, mB, vA, cA, vB, cB);
        const uint32_t bA = (key_at(cA) & 0x7FFFu) - wlo, bB = (key_at(cB) & 0x7FFFu) - wlo;
        if (vA) atomicAdd(&hist[bA], 1u);
        if (vB) atomicAdd(&hist[bB], 1u);
        if constexpr (!kSweepAgain) {
          if (sh < static_cast<uint32_t>(kListMax * kBinBits)) {
            listA |= (vA ? bA : 0u) << sh;
            listB |= (vB ? bB : 0u) << sh;
          } else {
            list_full = true;
          }
          sh += kBinBits;
          ++n_pops;
        }
      }
    }
    wave_lds_fence();
    // lane s of a row scans bins [s * kBinsPerLane, (s + 1) * kBinsPerLane): its own count, the suffix sums over
    // the lanes of the row, and -- were the answer among its bins -- where; the highest lane that reaches k has it
    uint32_t cb[kBinsPerLane];
    {
      const uint32_t* hb = hist + s * kBinsPerLane;
      if constexpr (kBinsPerLane == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(hb);
        cb[0] = v.x;
        cb[1] = v.y;
      } else {
#pragma unroll
        for (int q = 0; q < kBinsPerLane / 4; ++q) {
          const uint4 v = *reinterpret_cast<const uint4*>(hb + 4 * q);
          cb[4 * q + 0] = v.x;
          cb[4 * q + 1] = v.y;
          cb[4 * q + 2] = v.z;
          cb[4 * q + 3] = v.w;
        }
      }
    }
    uint32_t lane_sum = 0;
#pragma unroll
    for (int j = 0; j < kBinsPerLane; ++j) lane_sum += cb[j];
    const uint32_t suf = row_suffix_scan<kLanes>(lane_sum, s);  // window keys in this lane's bins and above
    const uint32_t m_reach = row_ballot<kLanes>(n_above + suf >= k, lane);  // non-empty: lane 0 reaches n_above + n_win >= k
    // walk this lane's bins from the top: the first one at which the count reaches k
    uint32_t acc = n_above + suf - lane_sum, loc = 0;
    bool found = false;
#pragma unroll
    for (int j = kBinsPerLane - 1; j >= 0; --j) {
      acc += cb[j];
      if (!found && acc >= k) {
        found = true;
        loc = (s * kBinsPerLane + j) | (cb[j] << 8) | ((acc - n_above) << 20);  // bin, ties, window keys at or above
      }
    }
    const int src = static_cast<int>((lane & (64u - kLanes)) | (31u - __builtin_clz(m_reach | 1u)));
    loc = __shfl(loc, src, kWave);
    const uint32_t bstar = loc & 0xFFu;
    const uint32_t n_eq = (loc >> 8) & 0xFFFu;
    const uint32_t sfx = loc >> 20;
    const uint32_t tau = wlo + bstar;
    const uint32_t n_gt = n_above + sfx - n_eq;
    const uint32_t quota = k - n_gt;  // ties at tau to keep, lowest columns first
    // the prediction for the next group's row in this slot: a running mean, which varies less than single rows do
    guess = have ? (3u * guess + tau + 2u) / 4u : tau;

    // ---- keep / tie bitmaps: above the window, plus the window keys compared with tau
    uint32_t keep[WORDS], tie[WORDS];
#pragma unroll
    for (int w = 0; w < WORDS; ++w) {
      keep[w] = above[w];
      tie[w] = 0;
    }
    const uint32_t bs = bstar;
    if constexpr (kSweepAgain) {
      uint32_t ge_tau[WORDS];
      ge_bitmap(tau + 1u, keep);  // tau + 1 <= 0x8000
      ge_bitmap(tau, ge_tau);
#pragma unroll
      for (int w = 0; w < WORDS; ++w) tie[w] = ge_tau[w] & ~keep[w];
    } else if (ballot64(list_full) == 0) {
      uint32_t mA = inwin[0], mB = WORDS == 2 ? inwin[wB] : 0u;
      for (uint32_t j = 0; j < n_pops; ++j) {
        const uint32_t bitA = mA & (0u - mA);  // 0 once the stream is exhausted: contributes nothing
        mA ^= bitA;
        uint32_t bitB;
        if constexpr (WORDS == 2) {
          bitB = mB & (0u - mB);
          mB ^= bitB;
        } else {
          bitB = mA != 0 ? 0x80000000u >> __builtin_clz(mA) : 0u;
          mA ^= bitB;
        }
        const uint32_t bA = listA & (kWindow - 1u), bB = listB & (kWindow - 1u);
        listA >>= kBinBits;
        listB >>= kBinBits;
        keep[0] |= bA > bs ? bitA : 0u;
        tie[0] |= bA == bs ? bitA : 0u;
        keep[wB] |= bB > bs ? bitB : 0u;
        tie[wB] |= bB == bs ? bitB : 0u;
      }
    } else {
      uint32_t mA = inwin[0], mB = WORDS == 2 ? inwin[wB] : 0u;
      while (ballot64((mA | mB) != 0) != 0) {
        bool vA, vB;
        uint32_t cA, cB;
        pop2(mA, mB, vA, cA, vB, cB);
        const uint32_t bA = (key_at(cA) & 0x7FFFu) - wlo, bB = (key_at(cB) & 0x7FFFu) - wlo;
        const uint32_t mkA = 1u << cA, mkB = 1u << (cB & 31u);
        keep[0] |= (vA && bA > bs) ? mkA : 0u;
        tie[0] |= (vA && bA == bs) ? mkA : 0u;
        keep[wB] |= (vB && bB > bs) ? mkB : 0u;
        tie[wB] |= (vB && bB == bs) ? mkB : 0u;
      }
    }

    // ---- 3. ties: the `quota` lowest columns among the n_eq ties of a row survive
    {
      uint32_t tc = 0;
#pragma unroll
      for (int w = 0; w < WORDS; ++w) tc += __popc(tie[w]);
      const bool trim = quota < n_eq;  // per row
      if (ballot64(trim) != 0) {
        const uint32_t before = row_incl_scan<kLanes>(tc, s) - tc;               // ties in lower lanes of the row
        const uint32_t allowed = quota > before ? quota - before : 0u;  // ties this lane may keep
        if (trim) {
          // lanes below the boundary keep all their ties, lanes above it none; the one lane on the
          // boundary drops its highest columns until `allowed` ties are left
#pragma unroll
          for (int w = 0; w < WORDS; ++w) tie[w] = allowed != 0 ? tie[w] : 0u;
          if (allowed != 0 && allowed < tc) {
            for (uint32_t drop = tc - allowed; drop != 0; --drop) {
              if (WORDS == 2 && tie[wB] != 0)
                tie[wB] ^= 0x80000000u >> __builtin_clz(tie[wB]);
              else
                tie[0] ^= 0x80000000u >> __builtin_clz(tie[0]);
            }
          }
        }
      }
#pragma unroll
      for (int w = 0; w < WORDS; ++w) keep[w] |= tie[w];
    }

    // ---- 4. write the survivors: slot = survivors in lower lanes of the row + at lower columns of this lane
    uint32_t kc = 0;
#pragma unroll
    for (int w = 0; w < WORDS; ++w) kc += __popc(keep[w]);
    const uint32_t slot = row_incl_scan<kLanes>(kc, s) - kc;
    if constexpr (ENC == kEncBitmap) {
      // the per-lane bitmaps ARE the mask: COLS bits per lane, packed into the row's 32-bit words
      const uint32_t n_words = (D + 31) / 32;
      uint32_t* mo = static_cast<uint32_t*>(idx_out) + my_row * n_words;
      if constexpr (COLS >= 32) {
#pragma unroll
        for (int w = 0; w < WORDS; ++w)
          if (my_row < B && s * WORDS + w < n_words) mo[s * WORDS + w] = keep[w];
      } else {
        constexpr uint32_t kLanesPerWord = 32 / COLS;  // 2 or 4 neighbouring lanes of the row share a word
        uint32_t v = keep[0] << ((s % kLanesPerWord) * COLS);
#pragma unroll
        for (uint32_t d = 1; d < kLanesPerWord; d <<= 1) v |= __shfl_xor(v, d, kWave);
        if (my_row < B && s % kLanesPerWord == 0 && s / kLanesPerWord < n_words) mo[s / kLanesPerWord] = v;
      }
    }
    {
      const uint32_t base = g * k;  // this row's list
      uint32_t mA = keep[0], mB = WORDS == 2 ? keep[wB] : 0u;
      uint32_t slotA = slot, slotB = WORDS == 2 ? slot + __popc(keep[0]) : slot + kc - 1u;
      while (ballot64((mA | mB) != 0) != 0) {
        bool vA, vB;
        uint32_t cA, cB;
        pop2(mA, mB, vA, cA, vB, cB);
        if (vA && slotA < k) *stage_at(base + slotA) = static_cast<uint16_t>(s * COLS + cA);
        if (vB && slotB < k) *stage_at(base + slotB) = static_cast<uint16_t>(s * COLS + cB);
        ++slotA;
        slotB += WORDS == 2 ? 1u : 0xFFFFFFFFu;
      }
    }
    wave_lds_fence();
    // the four rows are consecutive, so their k outputs each form one block of 4 k entries
    {
      const uint64_t row0 = grp * kRows;
      const uint32_t rows_here = static_cast<uint32_t>(min(static_cast<uint64_t>(kRows), B - row0));
      // the lists of the four rows follow one another in the staging slots as their outputs do in memory: entry e
      // of the group belongs to row e / k
      const uint32_t n_out = rows_here * k;
      auto write_groups = [&](auto g_tag) {
        constexpr int G = decltype(g_tag)::value;
        uint32_t col[G], raw[G];
#pragma unroll
        for (int j = 0; j < G; ++j) col[j] = j * kWave + lane < n_out ? *stage_at(j * kWave + lane) : 0u;
#pragma unroll
        for (int j = 0; j < G; ++j) {
          const uint32_t e = j * kWave + lane;
          uint32_t r = 0;
#pragma unroll
          for (uint32_t m = 1; m < static_cast<uint32_t>(kRows); ++m) r += e >= m * k ? 1u : 0u;
          raw[j] = raw_at(r, col[j]);
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
          const uint32_t e = j * kWave + lane;
          if (e < n_out) {
            put_col<ENC>(idx_out, row0 * k + e, col[j]);
            val_out[row0 * k + e] = static_cast<uint16_t>(raw[j]);
          }
        }
      };
      if (n_out <= kWave) {
        write_groups(std::integral_constant<int, 1>{});
      } else if (n_out <= 2 * kWave) {
        write_groups(std::integral_constant<int, 2>{});
      } else if (k <= kWave) {
        // one round per row: the row of an entry is known without comparing
        uint32_t col[kRows], raw[kRows];
#pragma unroll
        for (int r = 0; r < kRows; ++r) col[r] = lane < k ? *stage_at(r * k + lane) : 0u;
#pragma unroll
        for (int r = 0; r < kRows; ++r) raw[r] = raw_at(r, col[r]);
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
          if (static_cast<uint32_t>(r) < rows_here && lane < k) {
            const uint64_t o = (row0 + r) * k + lane;
            put_col<ENC>(idx_out, o, col[r]);
            val_out[o] = static_cast<uint16_t>(raw[r]);
          }
        }
      } else {
        for (uint32_t e = lane; e < n_out; e += kWave) {
          const uint32_t col = *stage_at(e);
          uint32_t r = 0;
#pragma unroll
          for (uint32_t m = 1; m < static_cast<uint32_t>(kRows); ++m) r += e >= m * k ? 1u : 0u;
          put_col<ENC>(idx_out, row0 * k + e, col);
          val_out[row0 * k + e] = static_cast<uint16_t>(raw_at(r, col));
        }
      }
    }
    if (tau_out && s == 0 && my_row < B) tau_out[my_row] = static_cast<uint16_t>(tau);
  }
}

}  // namespace quad
}  // namespace dct
