// CPU-only stand-ins for the device side of libtova, so that the host logic of tova_api.cpp
// (validation, buffer layout, launch planning, the launch loops) can be built with
// AddressSanitizer / UndefinedBehaviorSanitizer and run without a GPU or the HIP runtime.
// Every launcher checks the arguments a kernel would rely on and records the launch; nothing
// touches the (fake) device pointers.  Test infrastructure only: never linked into libtova.so.
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cstdlib>

#include "tova_internal.h"

extern "C" const char* hipGetErrorString(hipError_t) { return "stub"; }

namespace tova {

long g_launches = 0;
static unsigned char g_fake_scratch[256] __attribute__((aligned(256)));

static void require(bool ok, const char* what) {
  if (!ok) {
    std::fprintf(stderr, "host_sanitizer stub: launch precondition violated: %s\n", what);
    std::abort();
  }
}

hipError_t launch_step(int, int D, int G, const StepParams& p, const LaunchPlan& lp, hipStream_t) {
  require(D == 32 || D == 64 || D == 128, "head_dim");
  require(G == 1 || G == 2 || G == 4 || G == 8, "group size");
  require(lp.grid >= 1 && lp.block >= 64 && lp.block <= 512 && lp.block % 64 == 0, "launch shape");
  require(lp.lds_bytes > 0 && lp.lds_bytes <= 160 * 1024, "LDS");
  require(p.k >= 1 && p.n >= 0 && p.n <= p.k && p.S >= 1 && p.R >= 1 && (long long)p.S * p.R >= p.k, "chunks cover the slots");
  require(p.n_iter >= 1 && p.H % p.H_kv == 0 && p.pairs % p.H_kv == 0, "heads");
  require(p.q && p.k_new && p.v_new && p.out && p.K && p.V && p.occupancy && p.slot_token, "pointers");
  require(p.unit_mode || (p.sg && p.cnt_pair && p.cnt_unit && p.pstate), "scratch pointers");
  require(p.st_off >= 0 && p.red_off >= 0 && (size_t)(512 + p.st_off) * 4 <= (size_t)lp.lds_bytes, "LDS areas");
  require(!p.unit_mode || lp.grid <= p.pairs / p.H_kv, "a workgroup per unit at most");
  require(p.policy == kPolicyTova || p.unit_mode, "baseline policies need the unit form");
  ++g_launches;
  return hipSuccess;
}
hipError_t launch_prefill(int, int, int G, int C, const PrefillParams& p, const LaunchPlan& lp, hipStream_t) {
  require(C >= 2 && G * C <= 8 && p.n_chunks >= 1 && lp.grid >= 1, "prompt groups");
  require(p.parts >= 1 && p.H_kv % p.parts == 0, "parts divide the KV heads");
  require(p.parts == 1 ? lp.grid <= p.units : lp.grid == p.units * p.parts, "grid of the prompt kernel");
  require(p.parts == 1 || (p.tpart && p.stat && p.gpos && p.cnt_unit && p.pstate && p.error_flag), "hand-over areas");
  require(lp.lds_bytes <= 160 * 1024 && p.uscr != nullptr, "prompt LDS / scratch");
  ++g_launches;
  return hipSuccess;
}
hipError_t launch_repos(int, int, int, const ReposParams& p, const LaunchPlan& lp, hipStream_t) {
  require(p.parts >= 1 && p.H_kv % p.parts == 0 && lp.grid >= 1 && lp.lds_bytes <= 160 * 1024, "repositioned plan");
  ++g_launches;
  return hipSuccess;
}
int repos_resident_blocks(int, int, int, int, int) { return 512; }
int prefill_resident_blocks(int, int, int, int, int, int) { return 768; }
hipError_t launch_policy(const PolicyParams& p, hipStream_t) {
  require(p.units >= 1 && p.w && p.row_bytes % 16 == 0, "policy step");
  ++g_launches;
  return hipSuccess;
}
hipError_t launch_fill_i32(int32_t* dst, int32_t, size_t count, hipStream_t) {
  require(dst != nullptr || count == 0, "fill target");
  ++g_launches;
  return hipSuccess;
}
hipError_t launch_add_i32(int32_t* dst, int32_t, hipStream_t) {
  require(dst != nullptr, "counter to advance");
  ++g_launches;
  return hipSuccess;
}
int stream_is_capturing(hipStream_t) { return 0; }
hipError_t read_i32_sync(const int32_t*, hipStream_t, int32_t* host) {
  *host = 0;
  return hipSuccess;
}
int resident_blocks(int, int, int, int block, int lds_bytes, int) {
  const int by_lds = (160 * 1024) / (lds_bytes > 0 ? lds_bytes : 1);
  const int by_threads = 2048 / block;
  return 256 * (by_lds < by_threads ? by_lds : by_threads);
}
int device_cus() { return 256; }
hipError_t static_scratch(void** ptr, size_t* bytes) {
  *ptr = g_fake_scratch;  // never dereferenced by the stubs
  *bytes = (size_t)32 << 20;
  return hipSuccess;
}

}  // namespace tova
