// On-chip forward kernel of dct_rowtopk_fwd (Algorithm 2, forward loop: per row the
// k largest |X_act,i|) for rows of up to 16 KiB: 8192 bf16 or 4096 fp32 columns.
//
// One wavefront owns one row at a time and keeps it on chip:
//   1. the row is loaded once with coalesced 16-byte loads and written to a
//      padded LDS buffer; every lane then reads back ITS 64 (or fewer) contiguous
//      columns, so that column order is (lane, position in lane);
//   2. keys (sign-cleared bit patterns) stay packed two per register with bit 15
//      of each half set, so that one packed 16-bit subtract compares two keys with
//      a threshold (the borrow lands in bit 15 / 31).  Register i of a group of 16
//      pairs column i with column 16 + i, so that shifting those two bits into an
//      accumulator yields a per-lane bitmap in plain column order;
//   3. tau_i is found exactly.  Rows of one matrix have similar thresholds, so the
//      previous row's tau predicts a window of 32 key values: two packed compare
//      sweeps give the per-lane bitmaps of the keys at or above the window's ends,
//      the few keys inside the window are histogrammed (one LDS bin per lane) and
//      a wave scan over the bins locates the k-th largest key.  The first row of a
//      wavefront takes its prediction from a sample of the row (8 keys per lane);
//      a window that does not contain tau_i is followed by a galloping search from
//      that window in the direction the counts point to, then by bisection;
//   4. ties at tau_i are resolved by column order with one wave scan of per-lane
//      tie counts; the survivors' columns are then listed in order in the padding of
//      the LDS row buffer (slot = survivors in lower lanes + survivors at lower
//      columns of the lane) and written out with coalesced stores.
// fp32 rows run the same search on the UPPER 16 bits of their keys (which have
// exactly the layout of a bf16 key); the k-th largest key then lies among the
// few keys whose upper half equals the result, and a second, small selection on
// their lower halves finishes the job (step 3b in the code).
// Everything is integer work on the key bits; values are copied from the LDS copy
// of the row bit for bit.
#pragma once

#include <type_traits>

#include "dct_common.hpp"

namespace dct {
namespace fast {

// Wavefronts per workgroup: 4, or -- when every wavefront of a full chip has several rows to do -- 16 (8 for
// rows of 16 KiB, all a CU has room for), one workgroup per CU whose wavefronts share a row counter in LDS: a
// SIMD serves its oldest wavefront first, and with the rows dealt out in advance the wavefronts that were
// started first finished their share at 2/3 of the kernel's time and the last ones set it (c5: 76 / 89 / 101 /
// 114 us for the four wavefronts of a SIMD).  Measured per 512 MiB: 8 KiB rows 122 -> 114 us, 16 KiB rows
// 145 -> 139 us, fp32 rows of 2 KiB 173 -> 155 us, of 1 KiB 329 -> 292 us; rows of 4 KiB gain nothing (six small
// workgroups per CU do as well there) and keep the small workgroups, as do small batches, whose few large
// workgroups would leave CUs idle (8 KiB rows: the large workgroup wins from 16 k rows on).
constexpr int kWavesSmall = 4;
template <int NV>
constexpr int waves_per_wg() {
  return NV == 16 ? 8 : NV == 4 ? kWavesSmall : 16;
}
constexpr uint32_t kWindow = 32;
constexpr int kSampleRegs = 4;  // packed registers per lane in the first row's sample (8 keys per lane)

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_sub_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(ushort2_t, a) - __builtin_bit_cast(ushort2_t, b));
}
__device__ __forceinline__ uint32_t pk_add_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(ushort2_t, a) + __builtin_bit_cast(ushort2_t, b));
}
__device__ __forceinline__ uint32_t pk_lshr15_u16(uint32_t a) {
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(ushort2_t, a) >> static_cast<unsigned short>(15));
}

__device__ __forceinline__ uint32_t wave_total(uint32_t x) {
  return __builtin_amdgcn_readlane(wave_prefix_sum(x), 63);
}

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
}

// NV = 16-byte vectors per lane: the lane owns NV*8 (bf16) or NV*4 (fp32) contiguous columns.
// ENC (RowEnc): the row's mask is written through `idx_out` as k ascending column indices of 32 or
// 16 bits, or as a bitmap (ceil(D/32) words per row, bit c%32 of word c/32 = column c kept); the
// values are written either way.
// F32: fp32 rows (the packed 16-bit keys are the upper halves of the fp32 keys).
template <int NV, int ENC, bool F32, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void rowtopk_fwd_onchip_kernel(
    const std::conditional_t<F32, uint32_t, uint16_t>* __restrict__ x, uint32_t B, uint32_t D, uint64_t stride,
    uint32_t k, void* __restrict__ idx_out, std::conditional_t<F32, uint32_t, uint16_t>* __restrict__ val_out,
    std::conditional_t<F32, uint32_t, uint16_t>* __restrict__ tau_out) {
  using word_t = std::conditional_t<F32, uint32_t, uint16_t>;
  constexpr int ES = F32 ? 4 : 2;                   // bytes per element
  constexpr int EPV = 16 / ES;                      // elements per 16-byte vector
  constexpr int COLS = NV * EPV;                    // columns per lane
  constexpr int REGS = COLS / 2;                    // packed key registers per lane (2 columns each)
  constexpr int RPW = REGS < 16 ? REGS : 16;        // registers per bitmap word
  constexpr int WORDS = (REGS + 15) / 16;
  static_assert(WORDS <= 2 || (WORDS == 4 && !F32), "a lane owns at most 64 columns (bf16: 128)");
  constexpr int CHUNK = (NV + 1) * 16;              // LDS bytes per lane chunk (16 bytes of padding)
  constexpr int kWaves = WAVES;
  __shared__ uint4 s_row[kWaves][kWave * (NV + 1)];
  __shared__ uint32_t s_hist[kWaves][kWave];
  __shared__ uint32_t s_fix[F32 ? kWaves : 1][F32 ? kWave * WORDS : 1];  // fp32: decisions handed back to the owner lane

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform: row numbers stay scalar
  const uint32_t lane = lane_id();
  char* row_lds = reinterpret_cast<char*>(s_row[wave]);
  uint32_t* hist = s_hist[wave];
  const uint32_t n_vec = D / EPV;                   // the host guarantees whole 16-byte vectors
  [[maybe_unused]] uint32_t* fix = s_fix[F32 ? wave : 0];
  if constexpr (F32) {
#pragma unroll
    for (int w = 0; w < WORDS; ++w) fix[lane * WORDS + w] = 0;
  }

  // bit q of bitmap word w <-> local column kColsPerWord * w + q of the lane
  constexpr int kColsPerWord = 2 * RPW;
  // 16-bit key material of local column lc (bf16: the element; fp32: its upper half)
  auto key_at = [&](uint32_t lc) {
    return static_cast<uint32_t>(
        *reinterpret_cast<const uint16_t*>(row_lds + lane * CHUNK + lc * ES + (F32 ? 2 : 0)));
  };
  // the stored element of row column col, bit for bit
  auto raw_at_col = [&](uint32_t col) -> uint32_t {
    const char* p = row_lds + (col / COLS) * CHUNK + (col % COLS) * ES;
    if constexpr (F32) return *reinterpret_cast<const uint32_t*>(p);
    else return *reinterpret_cast<const uint16_t*>(p);
  };
  // the 16 padding bytes of every lane chunk hold the ordered list of surviving columns
  constexpr uint32_t kStageSlots = kWave * 8;
  auto stage_at = [&](uint32_t slot) {
    return reinterpret_cast<uint16_t*>(row_lds + (slot >> 3) * CHUNK + NV * 16 + (slot & 7u) * 2);
  };

  uint32_t guess = 0xFFFFFFFFu;  // tau of the previous row of this wavefront; none yet

  // The workgroup's rows are blocks of kWaves consecutive rows, one block in every stripe of gridDim.x blocks
  // (the grid as a whole reads a moving window of the matrix); its wavefronts take them one at a time, in
  // order, from a counter in LDS, so that a wavefront the SIMD favours simply takes more of them.  The n-th
  // row taken is a strictly increasing function of n: a wavefront that is handed a row past the end is done.
  // The next row's loads are issued while the current row is processed.
  const uint64_t row_step = static_cast<uint64_t>(gridDim.x) * kWaves;
  __shared__ uint32_t s_rows_taken;
  if (threadIdx.x == 0) s_rows_taken = 0;
  __syncthreads();
  auto take_row = [&]() -> uint64_t {
    uint32_t n = 0;
    if (lane == 0) n = atomicAdd(&s_rows_taken, 1u);
    n = __builtin_amdgcn_readfirstlane(n);
    return static_cast<uint64_t>(blockIdx.x) * kWaves + (n % kWaves) + static_cast<uint64_t>(n / kWaves) * row_step;
  };
  uint64_t row = take_row();
  uint4 nxt[NV];
  const bool full_width = n_vec == static_cast<uint32_t>(NV * kWave);  // no lane runs past the row's end
  auto load_row = [&](uint64_t r) {
    const uint4* xr = reinterpret_cast<const uint4*>(x + r * stride) + lane;
    if (full_width) {
#pragma unroll
      for (int j = 0; j < NV; ++j) nxt[j] = ld_stream(&xr[j * kWave]);
    } else {
#pragma unroll
      for (int j = 0; j < NV; ++j)
        nxt[j] = j * kWave + lane < n_vec ? ld_stream(&xr[j * kWave]) : make_uint4(0, 0, 0, 0);
    }
  };
  if (row < B) load_row(row);

  uint64_t next_row = 0;
  for (; row < B; row = next_row) {
    // ---- 1. row -> LDS (padded) -> registers, lane-contiguous
    wave_lds_fence();  // the previous row's readers are done with the buffer
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const uint32_t q = j * kWave + lane;
      *reinterpret_cast<uint4*>(row_lds + (q / NV) * CHUNK + (q % NV) * 16) = nxt[j];
    }
    wave_lds_fence();
    next_row = take_row();
    if (next_row < B) load_row(next_row);
    uint32_t R[4 * NV];  // the lane's columns as loaded: two per word (bf16) or one per word (fp32)
#pragma unroll
    for (int m = 0; m < NV; ++m) {
      const uint4 v = *reinterpret_cast<const uint4*>(row_lds + lane * CHUNK + m * 16);
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
        uint32_t pair;
        if constexpr (F32) {
          // the two upper halves: bytes 2,3 of each word
          pair = __builtin_amdgcn_perm(R[2 * RPW * w + RPW + i], R[2 * RPW * w + i], 0x07060302u);
        } else {
          const uint32_t a = R[RPW * w + i / 2], b2 = R[RPW * w + RPW / 2 + i / 2];
          // v_perm_b32 picks bytes from {b2, a}: the two low halves (i even) or the two high halves (i odd)
          pair = __builtin_amdgcn_perm(b2, a, (i & 1) ? 0x07060302u : 0x05040100u);
        }
        K[RPW * w + i] = (pair & 0x7FFF7FFFu) | 0x80008000u;
      }
    }

    // per-lane bitmap of the keys >= t (t <= 0x8000)
    auto ge_bitmap = [&](uint32_t t, uint32_t* out) {
      const uint32_t t2 = t * 0x00010001u;
#pragma unroll
      for (int w = 0; w < WORDS; ++w) {
        uint32_t a = 0;
#pragma unroll
        for (int i = 0; i < RPW; ++i)  // shift the accumulator, insert the two borrow bits (one v_bfi_b32)
          a = ((a >> 1) & ~0x80008000u) | (pk_sub_u16(K[RPW * w + i], t2) & 0x80008000u);
        // flags sit at bits [16-RPW, 16) and [32-RPW, 32): close the gap
        out[w] = RPW == 16 ? a : (((a & 0xFFFFu) >> (16 - RPW)) | ((a >> (32 - 2 * RPW)) & ~((1u << RPW) - 1u)));
      }
    };
    // number of keys >= t in the row
    auto count_ge = [&](uint32_t t) {
      const uint32_t t2 = t * 0x00010001u;
      uint32_t acc = 0;
#pragma unroll
      for (int i = 0; i < REGS; ++i) acc = pk_add_u16(acc, pk_lshr15_u16(pk_sub_u16(K[i], t2)));
      return wave_total((acc & 0xFFFFu) + (acc >> 16));
    };

    // Bit loops run two independent streams per step so that their LDS round trips overlap:
    // with two bitmap words, stream A walks word 0 and stream B word 1 (both upwards); with one
    // word, A takes the lowest and B the highest remaining bit.  c = local column of the bit.
    // The bitmap words of a lane are walked in pairs: stream A takes word 2p, stream B word 2p + 1 (with
    // one word per lane, A takes its lowest and B its highest remaining bit).
    constexpr int PAIRS = (WORDS + 1) / 2;
    auto word_a = [](int p) { return 2 * p; };
    auto word_b = [](int p) { return WORDS == 1 ? 0 : 2 * p + 1; };
    auto pop2 = [&](uint32_t& mA, uint32_t& mB, bool& vA, uint32_t& cA, bool& vB, uint32_t& cB, int p) {
      vA = mA != 0;
      cA = kColsPerWord * word_a(p) + (vA ? __builtin_ctz(mA) : 0u);
      mA &= mA - 1;
      if constexpr (WORDS >= 2) {
        vB = mB != 0;
        cB = kColsPerWord * word_b(p) + (vB ? __builtin_ctz(mB) : 0u);
        mB &= mB - 1;
      } else {
        vB = mA != 0;
        cB = vB ? 31u - __builtin_clz(mA) : 0u;
        mA &= ~(vB ? (1u << cB) : 0u);
      }
    };

    // ---- 3. locate tau
    // window [wlo, wlo + kWindow): bitmaps of the keys at or above its two ends and their counts
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
      const uint32_t both = wave_total(ca | (cw << 16));  // each count is at most 4096
      n_above = both & 0xFFFFu;
      n_win = both >> 16;
    };
    // Brackets in units of the window width: count_ge(lo_u * width) >= k > count_ge(hi_u * width).
    uint32_t lo_u = 0, hi_u = 0x8000u / kWindow;
    const bool had_guess = guess != 0xFFFFFFFFu;  // a previous row of this wavefront (not the sample estimate)
    if (guess == 0xFFFFFFFFu && REGS > kSampleRegs) {
      // no previous row: estimate tau as the matching order statistic of a sample of the row
      // (kSampleRegs registers of every lane), by bisection over all 15 key bits
      const uint32_t ks = max(1u, (k * kSampleRegs + REGS - 1) / REGS);
      uint32_t t = 0;
      for (int bit = 14; bit >= 0; --bit) {
        const uint32_t cand = t | (1u << bit);
        const uint32_t t2 = cand * 0x00010001u;
        uint32_t acc = 0;
#pragma unroll
        for (int i = 0; i < kSampleRegs; ++i) acc = pk_add_u16(acc, pk_lshr15_u16(pk_sub_u16(K[i], t2)));
        if (wave_total((acc & 0xFFFFu) + (acc >> 16)) >= ks) t = cand;
      }
      guess = t;
    }
    bool hit = false;
    if (guess != 0xFFFFFFFFu) {
      uint32_t lo_end = guess >= kWindow / 2 ? guess - kWindow / 2 : 0u;
      lo_end = min(lo_end, 0x8000u - kWindow);
      window_at(lo_end);
      hit = n_above < k && k <= n_above + n_win;
      if (!hit) {
        // gallop away from the failed window in the direction the counts point to
        if (n_above >= k) {  // tau is at or above the window's upper end
          lo_u = (wlo + kWindow) / kWindow;  // rounded down: still has >= k keys at or above it
          for (uint32_t step = 1;; step *= 2) {
            const uint32_t probe = min(lo_u + step, hi_u);
            if (probe == hi_u) break;
            if (count_ge(probe * kWindow) >= k) {
              lo_u = probe;
            } else {
              hi_u = probe;
              break;
            }
          }
        } else {             // fewer than k keys at or above the window's lower end
          hi_u = (wlo + kWindow - 1) / kWindow;  // rounded up: still has < k keys at or above it
          for (uint32_t step = 1;; step *= 2) {
            const uint32_t probe = hi_u > step ? hi_u - step : 0u;
            if (probe == 0u) break;
            if (count_ge(probe * kWindow) < k) {
              hi_u = probe;
            } else {
              lo_u = probe;
              break;
            }
          }
        }
      }
    }
    if (!hit) {
      // bisection between the brackets, in units of the window width
      while (hi_u - lo_u > 1) {
        const uint32_t mid = (lo_u + hi_u) / 2;
        if (count_ge(mid * kWindow) >= k) lo_u = mid; else hi_u = mid;
      }
      window_at(lo_u * kWindow);  // count_ge(wlo) >= k > count_ge(wlo + width): tau is inside
    }

    // histogram of the keys inside the window: bin = key - wlo, one bin per lane
    hist[lane] = 0;
    wave_lds_fence();
    // The bins (key - wlo, 5 bits) of the window keys are also remembered per stream in pop order,
    // six per stream, so that the second walk below needs no LDS reads.
    uint32_t listA[PAIRS], listB[PAIRS], n_pops[PAIRS];  // n_pops: pops of the longest stream (uniform)
    bool list_full = false;
#pragma unroll
    for (int p = 0; p < PAIRS; ++p) {
      listA[p] = listB[p] = n_pops[p] = 0;
      uint32_t mA = inwin[word_a(p)], mB = WORDS >= 2 ? inwin[word_b(p)] : 0u;
      uint32_t sh = 0;
      while (ballot64((mA | mB) != 0) != 0) {
        bool vA, vB;
        uint32_t cA, cB;
        pop2(mA, mB, vA, cA, vB, cB, p);
        const uint32_t bA = (key_at(cA) & 0x7FFFu) - wlo, bB = (key_at(cB) & 0x7FFFu) - wlo;
        if (vA) atomicAdd(&hist[bA], 1u);
        if (vB) atomicAdd(&hist[bB], 1u);
        if (sh < 30u) {
          listA[p] |= (vA ? bA : 0u) << sh;
          listB[p] |= (vB ? bB : 0u) << sh;
        } else {
          list_full = true;
        }
        sh += 5u;
        ++n_pops[p];
      }
    }
    wave_lds_fence();
    const uint32_t c = hist[lane];
    const uint32_t incl = wave_prefix_sum(c);
    const uint32_t suffix = n_win - incl + c;  // keys in bins >= lane
    const uint64_t reach = ballot64(n_above + suffix >= k);  // non-empty: bin 0 reaches n_above + n_win >= k
    const int bstar = 63 - __builtin_clzll(reach);
    const uint32_t tau = wlo + bstar;
    const uint32_t n_eq = __builtin_amdgcn_readlane(c, bstar);
    const uint32_t n_gt = n_above + __builtin_amdgcn_readlane(suffix, bstar) - n_eq;
    const uint32_t quota = k - n_gt;  // ties at tau to keep, lowest columns first
    // the next row's prediction: a running mean of the thresholds seen, which misses less often than the
    // last row's alone (narrow rows vary a lot from one to the next)
    guess = had_guess ? (3u * guess + tau + 2u) / 4u : tau;

    // ---- keep / tie bitmaps: above the window, plus the window keys compared with tau
    uint32_t keep[WORDS], tie[WORDS];
#pragma unroll
    for (int w = 0; w < WORDS; ++w) {
      keep[w] = above[w];
      tie[w] = 0;
    }
    const uint32_t bs = static_cast<uint32_t>(bstar);
    if (!list_full) {
      // every stream popped at most six keys: replay the pops from the remembered bins (no LDS reads)
#pragma unroll
      for (int p = 0; p < PAIRS; ++p) {
        uint32_t mA = inwin[word_a(p)], mB = WORDS >= 2 ? inwin[word_b(p)] : 0u;
        uint32_t la = listA[p], lb = listB[p];
        for (uint32_t j = 0; j < n_pops[p]; ++j) {
          const uint32_t bitA = mA & (0u - mA);  // 0 once the stream is exhausted: contributes nothing
          mA ^= bitA;
          uint32_t bitB;
          if constexpr (WORDS >= 2) {
            bitB = mB & (0u - mB);
            mB ^= bitB;
          } else {
            bitB = mA != 0 ? 0x80000000u >> __builtin_clz(mA) : 0u;
            mA ^= bitB;
          }
          const uint32_t bA = la & 31u, bB = lb & 31u;
          la >>= 5;
          lb >>= 5;
          keep[word_a(p)] |= bA > bs ? bitA : 0u;
          tie[word_a(p)] |= bA == bs ? bitA : 0u;
          keep[word_b(p)] |= bB > bs ? bitB : 0u;
          tie[word_b(p)] |= bB == bs ? bitB : 0u;
        }
      }
    } else {
#pragma unroll
      for (int p = 0; p < PAIRS; ++p) {
        uint32_t mA = inwin[word_a(p)], mB = WORDS >= 2 ? inwin[word_b(p)] : 0u;
        while (ballot64((mA | mB) != 0) != 0) {
          bool vA, vB;
          uint32_t cA, cB;
          pop2(mA, mB, vA, cA, vB, cB, p);
          const uint32_t bA = (key_at(cA) & 0x7FFFu) - wlo, bB = (key_at(cB) & 0x7FFFu) - wlo;
          const uint32_t mkA = 1u << (cA & 31u), mkB = 1u << (cB & 31u);
          keep[word_a(p)] |= (vA && bA > bs) ? mkA : 0u;
          tie[word_a(p)] |= (vA && bA == bs) ? mkA : 0u;
          keep[word_b(p)] |= (vB && bB > bs) ? mkB : 0u;
          tie[word_b(p)] |= (vB && bB == bs) ? mkB : 0u;
        }
      }
    }

    uint32_t tie_quota = quota, tie_n = n_eq;  // ties still to be resolved by column order
    [[maybe_unused]] uint32_t tau_low = 0;
    if constexpr (F32) {
      // ---- 3b. fp32: the search ran on the upper halves of the keys.  The k-th largest key is one of
      // the tie_n keys whose upper half is tau: find t, the tie_quota-th largest LOWER half among them.
      auto low_at = [&](uint32_t lc) {
        return static_cast<uint32_t>(*reinterpret_cast<const uint16_t*>(row_lds + lane * CHUNK + lc * 4));
      };
      uint32_t t = 0;
      if (tie_n <= static_cast<uint32_t>(kWave)) {
        // few of them: list their columns in order, one per lane, and bisect on registers
        uint32_t tc = 0;
#pragma unroll
        for (int w = 0; w < WORDS; ++w) tc += __popc(tie[w]);
        uint32_t ts = wave_prefix_sum(tc) - tc;
#pragma unroll
        for (int w = 0; w < WORDS; ++w) {
          uint32_t m = tie[w];
          while (ballot64(m != 0) != 0) {
            if (m != 0) {
              const uint32_t q = __builtin_ctz(m);
              m &= m - 1;
              *stage_at(ts++) = static_cast<uint16_t>(lane * COLS + kColsPerWord * w + q);
            }
          }
        }
        wave_lds_fence();
        const bool valid = lane < tie_n;
        const uint32_t col = valid ? *stage_at(lane) : 0u;
        const uint32_t low = valid ? (raw_at_col(col) & 0xFFFFu) : 0u;
        for (int bit = 15; bit >= 0; --bit) {
          const uint32_t cand = t | (1u << bit);
          if (static_cast<uint32_t>(__popcll(ballot64(valid && low >= cand))) >= tie_quota) t = cand;
        }
        const bool gt = valid && low > t, eq = valid && low == t;
        const uint64_t m_eq = ballot64(eq);
        const uint32_t left = tie_quota - static_cast<uint32_t>(__popcll(ballot64(gt)));  // >= 1 by the choice of t
        if (gt || (eq && lanes_below(m_eq) < left)) {  // list order is column order
          const uint32_t lc = col % COLS;
          atomicOr(&fix[(col / COLS) * WORDS + lc / kColsPerWord], 1u << (lc % kColsPerWord));
        }
        wave_lds_fence();
#pragma unroll
        for (int w = 0; w < WORDS; ++w) {
          keep[w] |= fix[lane * WORDS + w];
          fix[lane * WORDS + w] = 0;
          tie[w] = 0;
        }
        tie_quota = 0;
        tie_n = 0;
      } else {
        // many keys share the upper half (constant or coarsely quantised rows): every lane walks its own
        // body(bit, lower half) for every set bit of m, a bitmap of local columns col0 ...
        auto walk = [&](uint32_t m, uint32_t col0, auto&& body) {
          while (ballot64(m != 0) != 0) {
            if (m != 0) {
              const uint32_t q = __builtin_ctz(m);
              m &= m - 1;
              body(q, low_at(col0 + q));
            }
          }
        };
        uint32_t mn = 0xFFFFu, mx = 0;
#pragma unroll
        for (int w = 0; w < WORDS; ++w) {
          walk(tie[w], kColsPerWord * w, [&](uint32_t, uint32_t low) {
            mn = min(mn, low);
            mx = max(mx, low);
          });
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
          mn = min(mn, static_cast<uint32_t>(__shfl_xor(mn, d, kWave)));
          mx = max(mx, static_cast<uint32_t>(__shfl_xor(mx, d, kWave)));
        }
        t = mn;  // all lower halves equal (the usual case here): column order alone decides, below
        if (mn != mx) {
          const int top = 31 - __builtin_clz(mn ^ mx);   // bisect on the bits in which they differ
          t = mn & ~((2u << top) - 1u);
          for (int bit = top; bit >= 0; --bit) {
            const uint32_t cand = t | (1u << bit);
            uint32_t cnt = 0;
#pragma unroll
            for (int w = 0; w < WORDS; ++w)
              walk(tie[w], kColsPerWord * w, [&](uint32_t, uint32_t low) { cnt += low >= cand ? 1u : 0u; });
            if (wave_total(cnt) >= tie_quota) t = cand;
          }
          // greater lower halves survive; equal ones are the ties that column order resolves
          uint32_t ng = 0, ne = 0;
#pragma unroll
          for (int w = 0; w < WORDS; ++w) {
            uint32_t up = 0, rest = 0;
            walk(tie[w], kColsPerWord * w, [&](uint32_t q, uint32_t low) {
              const bool greater = low > t, equal = low == t;
              up |= greater ? (1u << q) : 0u;
              rest |= equal ? (1u << q) : 0u;
              ng += greater ? 1u : 0u;
              ne += equal ? 1u : 0u;
            });
            keep[w] |= up;
            tie[w] = rest;
          }
          const uint32_t both = wave_total(ng | (ne << 16));
          tie_quota -= both & 0xFFFFu;
          tie_n = both >> 16;
        }
      }
      tau_low = t;
    }

    // ---- 4. ties: the `tie_quota` lowest columns among the tie_n ties survive
    if (tie_quota >= tie_n) {
#pragma unroll
      for (int w = 0; w < WORDS; ++w) keep[w] |= tie[w];
    } else {
      uint32_t tc = 0;
#pragma unroll
      for (int w = 0; w < WORDS; ++w) tc += __popc(tie[w]);
      const uint32_t before = wave_prefix_sum(tc) - tc;     // ties in lower lanes
      const uint32_t allowed = tie_quota > before ? tie_quota - before : 0u;  // ties this lane may keep
      // lanes below the boundary keep all their ties, lanes above it none; the one lane on the
      // boundary drops its highest columns until `allowed` ties are left
      uint32_t t[WORDS];
#pragma unroll
      for (int w = 0; w < WORDS; ++w) t[w] = allowed != 0 ? tie[w] : 0u;
      if (allowed != 0 && allowed < tc) {
        for (uint32_t drop = tc - allowed; drop != 0; --drop) {
          bool done = false;  // clear the highest remaining tie of the lane
#pragma unroll
          for (int w = WORDS - 1; w >= 0; --w) {
            if (!done && t[w] != 0) {
              t[w] ^= 0x80000000u >> __builtin_clz(t[w]);
              done = true;
            }
          }
        }
      }
#pragma unroll
      for (int w = 0; w < WORDS; ++w) keep[w] |= t[w];
    }

    // ---- write the survivors: slot = survivors in lower lanes + survivors at lower columns of this lane
    uint32_t kc = 0;
#pragma unroll
    for (int w = 0; w < WORDS; ++w) kc += __popc(keep[w]);
    uint32_t slot = wave_prefix_sum(kc) - kc;
    const uint64_t o0 = row * k;  // first output slot of the row
    word_t* vo = val_out + o0;
    if constexpr (ENC == kEncBitmap) {
      // the per-lane bitmaps ARE the mask: COLS bits per lane, packed into 32-bit words
      const uint32_t n_words = (D + 31) / 32;
      uint32_t* mo = static_cast<uint32_t*>(idx_out) + row * n_words;
      if constexpr (COLS >= 32) {
#pragma unroll
        for (int w = 0; w < WORDS; ++w)
          if (lane * WORDS + w < n_words) mo[lane * WORDS + w] = keep[w];
      } else {
        constexpr uint32_t kLanesPerWord = 32 / COLS;  // 2, 4 or 8 neighbouring lanes share a word
        uint32_t v = keep[0] << ((lane % kLanesPerWord) * COLS);
#pragma unroll
        for (uint32_t d = 1; d < kLanesPerWord; d <<= 1) v |= __shfl_xor(v, d, kWave);
        if (lane % kLanesPerWord == 0 && lane / kLanesPerWord < n_words) mo[lane / kLanesPerWord] = v;
      }
    }
    if (k <= kStageSlots) {
      // list the surviving columns in order in LDS, then write idx / val with coalesced stores
      {
        uint32_t first = slot;  // slot of the pair's first survivor
#pragma unroll
        for (int p = 0; p < PAIRS; ++p) {
          uint32_t mA = keep[word_a(p)], mB = WORDS >= 2 ? keep[word_b(p)] : 0u;
          uint32_t slotA = first, slotB = WORDS >= 2 ? first + __popc(mA) : first + kc - 1u;
          first += __popc(mA) + __popc(mB);
          while (ballot64((mA | mB) != 0) != 0) {
            bool vA, vB;
            uint32_t cA, cB;
            pop2(mA, mB, vA, cA, vB, cB, p);
            if (vA && slotA < k) *stage_at(slotA) = static_cast<uint16_t>(lane * COLS + cA);
            if (vB && slotB < k) *stage_at(slotB) = static_cast<uint16_t>(lane * COLS + cB);
            ++slotA;
            slotB += WORDS >= 2 ? 1u : 0xFFFFFFFFu;
          }
        }
      }
      wave_lds_fence();
      // up to G outputs per lane: all list reads first, then all value reads, then the stores
      auto write_groups = [&](auto g_tag) {
        constexpr int G = decltype(g_tag)::value;
        uint32_t col[G], raw[G];
#pragma unroll
        for (int j = 0; j < G; ++j) col[j] = j * kWave + lane < k ? *stage_at(j * kWave + lane) : 0u;
#pragma unroll
        for (int j = 0; j < G; ++j)
          raw[j] = raw_at_col(col[j]);
#pragma unroll
        for (int j = 0; j < G; ++j) {
          const uint32_t o = j * kWave + lane;
          if (o < k) {
            put_col<ENC>(idx_out, o0 + o, col[j]);
            vo[o] = static_cast<word_t>(raw[j]);
          }
        }
      };
      if (k <= kWave) {
        write_groups(std::integral_constant<int, 1>{});
      } else if (k <= 2 * kWave) {
        write_groups(std::integral_constant<int, 2>{});
      } else if (k <= 4 * kWave) {
        write_groups(std::integral_constant<int, 4>{});
      } else {
        for (uint32_t j = lane; j < k; j += kWave) {
          const uint32_t col = *stage_at(j);
          const uint32_t raw = raw_at_col(col);
          put_col<ENC>(idx_out, o0 + j, col);
          vo[j] = static_cast<word_t>(raw);
        }
      }
    } else {
#pragma unroll
      for (int w = 0; w < WORDS; ++w) {
        uint32_t m = keep[w];
        while (ballot64(m != 0) != 0) {
          if (m != 0) {
            const uint32_t q = __builtin_ctz(m);
            m &= m - 1;
            const uint32_t lc = kColsPerWord * w + q;
            if (slot < k) {
              put_col<ENC>(idx_out, o0 + slot, lane * COLS + lc);
              vo[slot] = static_cast<word_t>(raw_at_col(lane * COLS + lc));
            }
            ++slot;
          }
        }
      }
    }
    if (tau_out && lane == 0) tau_out[row] = static_cast<word_t>(F32 ? ((tau << 16) | tau_low) : tau);
  }
}

}  // namespace fast
}  // namespace dct
