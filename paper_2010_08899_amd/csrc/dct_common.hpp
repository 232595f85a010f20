// Shared device/host helpers of libdct (gfx950 only, wave64).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <stdint.h>

#include "dct.h"

namespace dct {

constexpr int kWave = 64;

// Element traits: storage word, elements per 16-byte vector, key extraction.
// key(x) = bit pattern with the sign bit cleared; unsigned order on keys is the
// magnitude order used by Algorithm 1 (the sort of the magnitudes) and Algorithm 2.
template <int DT>
struct Elem;

template <>
struct Elem<DCT_F32> {
  using word_t = uint32_t;
  static constexpr int kVec = 4;
  static constexpr int kKeyBits = 31;
  static constexpr uint32_t kKeyMask = 0x7FFFFFFFu;
  __device__ static __forceinline__ uint32_t raw(const uint4& v, int e) {
    return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
  }
};

template <>
struct Elem<DCT_BF16> {
  using word_t = uint16_t;
  static constexpr int kVec = 8;
  static constexpr int kKeyBits = 15;
  static constexpr uint32_t kKeyMask = 0x7FFFu;
  __device__ static __forceinline__ uint32_t raw(const uint4& v, int e) {
    const uint32_t w = (e >> 1) == 0 ? v.x : (e >> 1) == 1 ? v.y : (e >> 1) == 2 ? v.z : v.w;
    return (e & 1) ? (w >> 16) : (w & 0xFFFFu);
  }
};

// bf16: which of the eight keys of a 16-byte vector are >= t (t <= 0x8000), as bits in element order.  The keys
// are compared two at a time: with bit 15 of each half set (which also clears the sign), a packed 16-bit subtract
// of t leaves that bit standing exactly where key >= t; the low halves' bits are gathered on even positions, the
// high halves' 15 bits above them.
__device__ __forceinline__ uint32_t bf16x8_ge_bits(const uint4& v, uint32_t t) {
  typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
  const uint32_t t2 = t * 0x00010001u;
  auto flags = [&](uint32_t w) {
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2, w | 0x80008000u) - __builtin_bit_cast(u16x2, t2)) &
           0x80008000u;
  };
  const uint32_t x = (flags(v.x) >> 15) | (flags(v.y) >> 13) | (flags(v.z) >> 11) | (flags(v.w) >> 9);
  return (x | (x >> 15)) & 0xFFu;
}

__device__ __forceinline__ uint32_t lane_id() { return __lane_id(); }

// Number of set bits of `m` in lanes below the calling lane.
__device__ __forceinline__ uint32_t lanes_below(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(m >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(m), 0u));
}

__device__ __forceinline__ uint64_t ballot64(bool p) { return __ballot(p); }

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, kWave);
  return v;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, kWave);
  return v;
}

// Inclusive prefix sum over the 64 lanes (DPP row shifts and row broadcasts); all lanes must be active.
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t x) {
  uint32_t v = x;
  v += __builtin_amdgcn_update_dpp(0u, v, 0x111, 0xf, 0xf, false);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0u, v, 0x112, 0xf, 0xf, false);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0u, v, 0x114, 0xf, 0xf, false);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0u, v, 0x118, 0xf, 0xf, false);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0u, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0u, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
  return v;
}

// One update of a histogram in LDS.  Lanes whose digit equals the first active lane's digit
// are counted with one ballot and a single LDS add (skewed data such as a mostly zero
// gradient, or candidates that share their top digits, would otherwise serialise on one
// bin); the others add directly.
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

// Workgroup barrier that orders LDS accesses only: global loads and stores that are outstanding
// stay in flight (__syncthreads() waits for them as well).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Agent-scope relaxed accesses for words that other workgroups poll or update.
__device__ __forceinline__ uint64_t ld_agent(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint64_t* p, uint64_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16-byte accesses of data that is streamed once: marked non-temporal so that the caches do not
// keep lines nobody will ask for again.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_stream(uint4* p, uint32_t x, uint32_t y, uint32_t z, uint32_t w) {
  const u32x4_t v = {x, y, z, w};
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p));
}

// How a row's mask leaves the row top-k forward kernels: k column indices of 32 or 16 bits, or a
// bitmap of ceil(D/32) words.  `put_col` stores column `col` as entry `pos` of an index list.
enum RowEnc : int { kEncIdx32 = 0, kEncBitmap = 1, kEncIdx16 = 2 };
template <int ENC>
__device__ __forceinline__ void put_col(void* idx_base, uint64_t pos, uint32_t col) {
  if constexpr (ENC == kEncIdx32) static_cast<int32_t*>(idx_base)[pos] = static_cast<int32_t>(col);
  if constexpr (ENC == kEncIdx16) static_cast<uint16_t*>(idx_base)[pos] = static_cast<uint16_t>(col);
}

inline bool is_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// ceil(a / b) for any a: a + b - 1 would wrap for a close to 2^32.
inline uint32_t ceil_div(uint32_t a, uint32_t b) { return a / b + (a % b != 0 ? 1u : 0u); }

// Compute units of the current device.  The only thing the library remembers between calls besides the wait
// limit: a per-device cache of this device attribute (atomic words; two threads racing store the same value).
inline int device_cu_count() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Polls a bounded device-side wait may take before it gives up (process-wide; dct_set_wait_limit).
uint32_t wait_limit();

inline int launch_status() { return hipGetLastError() == hipSuccess ? DCT_OK : DCT_ERR_HIP; }

}  // namespace dct
