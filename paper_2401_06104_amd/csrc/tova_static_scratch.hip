// The library's static device scratch area, for the entry point that must not allocate
// (tova_decode_steps_static): the hand-off scratch of the step kernel -- arrival counters, per-unit
// state words, partial score rows, chunk statistics, PV partials -- lives in a file-scope device
// array instead of a buffer the caller allocated.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends.  In host code the array's name is only a stand-in for the symbol: its device
// address is looked up once per device with hipGetSymbolAddress (that device current) and kept;
// kernels, fills and copies are only ever given that address.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "tova.h"
#include "tova_internal.h"

namespace tova {
namespace {

constexpr int kMaxDevices = 64;

// (`used`: no device code names the array -- kernels receive its address as an argument)
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[TOVA_STATIC_SCRATCH_BYTES];

std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {nullptr};  // device address of `scratch`, per device

}  // namespace

hipError_t static_scratch(void** ptr, size_t* bytes) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255) != 0) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  *bytes = TOVA_STATIC_SCRATCH_BYTES;
  return hipSuccess;
}

}  // namespace tova
