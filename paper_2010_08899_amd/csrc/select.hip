// dct_select_threshold: Algorithm 1, "sort |W_grad|; tau = w_floor(N*eta)",
// computed exactly as the k-th largest key WITHOUT sorting or copying the
// gradient (the copy-and-sort routine is what Sec. 3.3 measures as the cost of
// recomputing the threshold every iteration).
//
// Radix select over the key bits, most significant digit first (11 + 11 + 9 bits
// for fp32, 8 + 7 for bf16).  Each pass streams the vector with 16-byte loads,
// histograms the current digit of the keys that match the digits fixed so far
// into a per-workgroup LDS histogram, and merges it into a global one.  The
// workgroup that finishes a pass last walks the histogram from the top bin down,
// finds the bin that holds the k-th largest key and narrows the search state for
// the next pass; after the last pass it writes the dct_threshold.  All arithmetic
// is on integers.
#include "dct_common.hpp"

namespace dct {
namespace {

constexpr int kSelThreads = 256;
constexpr int kSelBins = 2048;
constexpr int kSelMaxPasses = 3;
constexpr int kSelUnroll = 4;  // 16-byte loads in flight per lane

struct SelState {
  uint32_t prefix;  // digits fixed so far, in place
  uint32_t k_rem;   // rank still to find inside the matching keys (1-based from the top)
  uint32_t n_gt;    // keys known to be above every matching key
  uint32_t pad;
};

struct SelWs {
  SelState state[kSelMaxPasses + 1];
  uint32_t done[kSelMaxPasses];
  uint32_t pad[13];
  uint32_t hist[kSelMaxPasses][kSelBins];
};

__global__ void select_init_kernel(SelWs* ws, uint32_t k) {
  uint32_t* w = reinterpret_cast<uint32_t*>(ws);
  const uint32_t n_words = sizeof(SelWs) / 4;
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += gridDim.x * blockDim.x) w[i] = 0;
  __syncthreads();
  if (blockIdx.x == 0 && threadIdx.x == 0) ws->state[0].k_rem = k;  // block 0 owns word 1 (i < 256)
}

// One histogram update.  Lanes whose digit equals the first active lane's digit
// are counted with one ballot and a single LDS add (skewed data such as a mostly
// zero gradient would otherwise serialise on one bin); the others add directly.
__device__ __forceinline__ void hist_add(uint32_t* h, bool active, uint32_t digit) {
  const uint64_t act = ballot64(active);
  if (act == 0) return;
  const int leader = __builtin_ctzll(act);
  const uint32_t d0 = __shfl(digit, leader, kWave);
  const bool same = active && digit == d0;
  const uint64_t m = ballot64(same);
  if (static_cast<int>(lane_id()) == leader) atomicAdd(&h[d0], static_cast<uint32_t>(__popcll(m)));
  if (active && !same) atomicAdd(&h[digit], 1u);
}

template <int DT>
__global__ __launch_bounds__(kSelThreads) void select_pass_kernel(
    const typename Elem<DT>::word_t* __restrict__ g_al, uint32_t off, uint32_t n_virt, SelWs* ws, int pass,
    int shift, int width, uint32_t fixed_mask, int last_pass, dct_threshold* __restrict__ thr_out) {
  using E = Elem<DT>;
  constexpr int V = E::kVec;
  __shared__ uint32_t h[kSelBins];
  __shared__ uint32_t s_scan[kSelThreads];
  __shared__ uint32_t s_last;
  for (int i = threadIdx.x; i < kSelBins; i += kSelThreads) h[i] = 0;
  const SelState st = ws->state[pass];
  const uint32_t prefix = st.prefix;
  const uint32_t dmask = (1u << width) - 1u;
  __syncthreads();

  // Vectors [v_lo, v_hi) are entirely inside the data; at most one vector on each
  // side straddles an end and is read element by element by workgroup 0.
  const uint32_t v_lo = off ? 1u : 0u;
  const uint32_t v_hi = n_virt / V;
  const uint4* gv = reinterpret_cast<const uint4*>(g_al);
  const uint32_t span = kSelThreads * kSelUnroll;
  for (uint32_t base = v_lo + blockIdx.x * span; base < v_hi; base += gridDim.x * span) {
    uint4 v[kSelUnroll];
    bool in[kSelUnroll];
#pragma unroll
    for (int u = 0; u < kSelUnroll; ++u) {
      const uint32_t vi = base + u * kSelThreads + threadIdx.x;
      in[u] = vi < v_hi;
      v[u] = in[u] ? gv[vi] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kSelUnroll; ++u) {
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const uint32_t key = E::raw(v[u], e) & E::kKeyMask;
        hist_add(h, in[u] && (key & fixed_mask) == prefix, (key >> shift) & dmask);
      }
    }
  }
  if (blockIdx.x == 0) {
    // head elements [off, min(V, n_virt)) when the base is misaligned, tail elements [v_hi*V, n_virt)
    const uint32_t t = threadIdx.x;
    uint32_t ve = 0xFFFFFFFFu;
    if (t < static_cast<uint32_t>(V)) {
      if (off && t >= off && t < n_virt) ve = t;
    } else if (t < 2u * V) {
      const uint32_t c = v_hi * V + (t - V);
      if (c < n_virt && (c >= static_cast<uint32_t>(V) || !off)) ve = c;
    }
    const bool act = ve != 0xFFFFFFFFu;
    const uint32_t key = act ? (static_cast<uint32_t>(g_al[ve]) & E::kKeyMask) : 0u;
    if (t < kWave) hist_add(h, act && (key & fixed_mask) == prefix, (key >> shift) & dmask);
  }
  __syncthreads();

  // merge into the global histogram of this pass
  uint32_t* gh = ws->hist[pass];
  for (int i = threadIdx.x; i < kSelBins; i += kSelThreads) {
    const uint32_t c = h[i];
    if (c) atomicAdd(&gh[i], c);
  }
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t prev = __hip_atomic_fetch_add(&ws->done[pass], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (prev == gridDim.x - 1) ? 1u : 0u;
  }
  __syncthreads();
  if (s_last == 0) return;

  // ---- last workgroup: find the bin of the k_rem-th largest matching key.
  // Thread t owns the 8 bins [2047-8t-7, 2047-8t], walked from the top down.
  constexpr int kPer = kSelBins / kSelThreads;
  uint32_t c[kPer];
  uint32_t sum = 0;
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    c[j] = ld_agent(&gh[kSelBins - 1 - (threadIdx.x * kPer + j)]);
    sum += c[j];
  }
  s_scan[threadIdx.x] = sum;
  __syncthreads();
  // inclusive scan over threads (Hillis-Steele, 256 entries)
  for (int d = 1; d < kSelThreads; d <<= 1) {
    const uint32_t add = threadIdx.x >= static_cast<uint32_t>(d) ? s_scan[threadIdx.x - d] : 0u;
    __syncthreads();
    s_scan[threadIdx.x] += add;
    __syncthreads();
  }
  const uint32_t incl = s_scan[threadIdx.x];
  uint32_t above = incl - sum;  // matching keys in bins above this thread's bins
  const uint32_t k_rem = st.k_rem;
  if (above < k_rem && k_rem <= incl) {
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      if (above < k_rem && k_rem <= above + c[j]) {
        const uint32_t bin = kSelBins - 1 - (threadIdx.x * kPer + j);
        const uint32_t new_prefix = prefix | (bin << shift);
        if (last_pass) {
          thr_out->tau_key = new_prefix;
          thr_out->n_gt = st.n_gt + above;
          thr_out->n_eq = c[j];
          thr_out->tie_quota = k_rem - above;
        } else {
          SelState nx;
          nx.prefix = new_prefix;
          nx.k_rem = k_rem - above;
          nx.n_gt = st.n_gt + above;
          nx.pad = 0;
          ws->state[pass + 1] = nx;
        }
        above = 0xFFFFFFFFu;  // found: stop matching the following bins
      } else if (above != 0xFFFFFFFFu) {
        above += c[j];
      }
    }
  }
}

}  // namespace
}  // namespace dct

using namespace dct;

extern "C" size_t dct_select_threshold_workspace_bytes(int dt, uint64_t n) {
  if ((dt != DCT_F32 && dt != DCT_BF16) || n == 0 || n > 0x7FFFFFFFull) return 0;
  return sizeof(SelWs);
}

extern "C" int dct_select_threshold(const void* g, int dt, uint64_t n, uint64_t k, dct_threshold* d_thr_out,
                                    void* d_ws, size_t ws_bytes, void* hip_stream) {
  if (!g || !d_thr_out || n == 0 || n > 0x7FFFFFFFull || k == 0 || k > n) return DCT_ERR_INVALID;
  if (dt != DCT_F32 && dt != DCT_BF16) return DCT_ERR_INVALID;
  const size_t es = dt == DCT_F32 ? 4 : 2;
  if (!is_aligned(g, es) || !is_aligned(d_thr_out, 16)) return DCT_ERR_INVALID;
  if (!d_ws || !is_aligned(d_ws, 256) || ws_bytes < sizeof(SelWs)) return DCT_ERR_WORKSPACE;

  const uintptr_t addr = reinterpret_cast<uintptr_t>(g);
  const uint32_t off = static_cast<uint32_t>((addr & 15) / es);
  const uint32_t n_virt = static_cast<uint32_t>(n + off);
  const void* g_al = reinterpret_cast<const void*>(addr & ~static_cast<uintptr_t>(15));
  auto* ws = static_cast<SelWs*>(d_ws);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  hipLaunchKernelGGL(select_init_kernel, dim3((sizeof(SelWs) / 4 + 255) / 256), dim3(256), 0, s, ws,
                     static_cast<uint32_t>(k));
  if (hipGetLastError() != hipSuccess) return DCT_ERR_HIP;

  const int vec = dt == DCT_F32 ? 4 : 8;
  const uint32_t n_vec = n_virt / vec + 1;
  const uint32_t span = kSelThreads * kSelUnroll;
  uint32_t grid = (n_vec + span - 1) / span;
  if (grid > 4096) grid = 4096;
  if (grid == 0) grid = 1;

  const int n_pass = dt == DCT_F32 ? 3 : 2;
  const int shifts_f32[3] = {20, 9, 0}, widths_f32[3] = {11, 11, 9};
  const int shifts_bf16[2] = {7, 0}, widths_bf16[2] = {8, 7};
  for (int p = 0; p < n_pass; ++p) {
    const int shift = dt == DCT_F32 ? shifts_f32[p] : shifts_bf16[p];
    const int width = dt == DCT_F32 ? widths_f32[p] : widths_bf16[p];
    const uint32_t key_mask = dt == DCT_F32 ? 0x7FFFFFFFu : 0x7FFFu;
    const uint32_t fixed_mask = key_mask & ~((1u << (shift + width)) - 1u);
    const int last = p == n_pass - 1;
    if (dt == DCT_F32) {
      hipLaunchKernelGGL((select_pass_kernel<DCT_F32>), dim3(grid), dim3(kSelThreads), 0, s,
                         static_cast<const uint32_t*>(g_al), off, n_virt, ws, p, shift, width, fixed_mask, last,
                         d_thr_out);
    } else {
      hipLaunchKernelGGL((select_pass_kernel<DCT_BF16>), dim3(grid), dim3(kSelThreads), 0, s,
                         static_cast<const uint16_t*>(g_al), off, n_virt, ws, p, shift, width, fixed_mask, last,
                         d_thr_out);
    }
    if (hipGetLastError() != hipSuccess) return DCT_ERR_HIP;
  }
  return DCT_OK;
}
