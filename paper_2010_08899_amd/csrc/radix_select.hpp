// Radix-select building blocks shared by the single-tensor and the batched
// threshold selection (Algorithm 1, the sorted magnitudes and the element picked as tau,
// without the sort): the per-pass search state and
// the walk over a 2048-bin histogram from the top bin down.
#pragma once

#include "dct_common.hpp"

namespace dct {
namespace {

constexpr int kSelThreads = 256;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelBins = 2048;

struct SelState {
  uint32_t prefix;     // digits fixed so far, in place
  uint32_t k_rem;      // rank still to find among the matching keys (1-based from the top)
  uint32_t n_gt;       // keys known to be above every matching key
  uint32_t from_cand;  // 1: the passes read the candidate buffer, 0: the vector
  uint32_t n_src;      // keys in the source
  uint32_t rem_bits;   // low key bits not fixed yet
  uint32_t width;      // digit width of this pass (0: nothing left to do)
  uint32_t last_count; // keys that match the prefix
};

constexpr uint32_t kDigitBits = 11;


// Walk a 2048-bin histogram from the top bin down and find the bin that holds the
// k_rem-th largest key.  Called by all THREADS threads of a workgroup (THREADS a
// multiple of 64 that divides 2048); s_tmp needs THREADS / 64 + 4 words.  Returns
// {bin, keys in higher bins, keys in the bin} to every thread.
struct BinHit {
  uint32_t bin, above, count;
};
template <int THREADS, typename LoadBin>
__device__ BinHit find_bin(LoadBin load_bin, uint32_t k_rem, uint32_t* s_tmp) {
  constexpr int kPer = kSelBins / THREADS;
  constexpr int kW = THREADS / kWave;
  const uint32_t t = threadIdx.x;
  uint32_t c[kPer];
  uint32_t sum = 0;
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    c[j] = load_bin(kSelBins - 1 - (t * kPer + j));
    sum += c[j];
  }
  const uint32_t incl_w = wave_prefix_sum(sum);
  if (lane_id() == kWave - 1) s_tmp[t / kWave] = incl_w;
  __syncthreads();
  uint32_t before_waves = 0;
  for (uint32_t w = 0; w < t / kWave; ++w) before_waves += s_tmp[w];
  const uint32_t incl = before_waves + incl_w;
  uint32_t above = incl - sum;
  if (above < k_rem && k_rem <= incl) {
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      if (above < k_rem && k_rem <= above + c[j]) {
        s_tmp[kW + 0] = kSelBins - 1 - (t * kPer + j);
        s_tmp[kW + 1] = above;
        s_tmp[kW + 2] = c[j];
        above = 0xFFFFFFFFu;
      } else if (above != 0xFFFFFFFFu) {
        above += c[j];
      }
    }
  }
  __syncthreads();
  BinHit r;
  r.bin = s_tmp[kW + 0];
  r.above = s_tmp[kW + 1];
  r.count = s_tmp[kW + 2];
  __syncthreads();
  return r;
}

// Search state after the pass whose state was `prev` and whose histogram load_bin reads (called by all
// THREADS threads of a workgroup, see find_bin).
template <int THREADS, typename LoadBin>
__device__ SelState advance_state_with(const SelState& prev, LoadBin load_bin, uint32_t* s_tmp) {
  SelState st = prev;
  if (prev.width != 0) {  // uniform
    const BinHit hit = find_bin<THREADS>(load_bin, prev.k_rem, s_tmp);
    st.rem_bits = prev.rem_bits - prev.width;
    st.prefix = prev.prefix | (hit.bin << st.rem_bits);
    st.k_rem = prev.k_rem - hit.above;
    st.n_gt = prev.n_gt + hit.above;
    st.last_count = hit.count;
  }
  st.width = min(kDigitBits, st.rem_bits);
  return st;
}
// The same for a histogram that an earlier kernel completed, by a workgroup of kSelThreads threads.
__device__ SelState advance_state(const SelState& prev, const uint32_t* hist, uint32_t* s_tmp) {
  return advance_state_with<kSelThreads>(prev, [&](uint32_t b) { return hist[b]; }, s_tmp);
}


}  // namespace
}  // namespace dct
