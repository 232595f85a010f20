// Status strings and the process-wide bound of the device-side waits.
#include <atomic>

#include "dct_common.hpp"

namespace dct {
namespace {
constexpr uint32_t kDefaultWaitLimit = 1u << 20;  // polls: about a second
std::atomic<uint32_t> g_wait_limit{kDefaultWaitLimit};
}  // namespace

uint32_t wait_limit() { return g_wait_limit.load(std::memory_order_relaxed); }

}  // namespace dct

extern "C" void dct_set_wait_limit(uint32_t polls) {
  dct::g_wait_limit.store(polls ? polls : dct::kDefaultWaitLimit, std::memory_order_relaxed);
}

extern "C" const char* dct_status_string(int status) {
  switch (status) {
    case DCT_OK: return "DCT_OK";
    case DCT_ERR_INVALID: return "DCT_ERR_INVALID: bad argument";
    case DCT_ERR_WORKSPACE: return "DCT_ERR_WORKSPACE: workspace null, misaligned, too small or uninitialised";
    case DCT_ERR_OVERFLOW: return "DCT_ERR_OVERFLOW: more survivors than the output capacity";
    case DCT_ERR_HIP: return "DCT_ERR_HIP: kernel launch failed";
    default: return "unknown dct_status";
  }
}
