// The TOVA policy on its own (gfx950 / MI355X): App. B, Alg. 1 as a function of attention weights
// that somebody else has computed.
//
// For callers that keep their own attention kernel: the policy receives the last query's softmax
// weights over the multi-state with the incoming token appended ([heads][k + 1], the incoming
// token last), averages them over the heads of the layer, takes the argmin (lowest index on ties;
// candidates below n_pinned stay out: TOVA+i, App. A) and removes that row -- here by overwriting
// its slot with the incoming key / value rows, or by not storing them if the incoming token itself
// scored lowest (Sec. 4).  While the multi-state has room it only appends (the early return of
// Alg. 1).  A workgroup per (layer, sequence) unit; the weights are read once, coalesced along the
// candidates, heads added in head order (as a sum: the factor 1 / H does not move the argmin).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tova_internal.h"

#include "tova_device.h"

namespace tova {
namespace {

__global__ __launch_bounds__(1024) void tova_policy_kernel(const PolicyParams p) {
  __shared__ float bv[kMaxWaves];
  __shared__ int bi[kMaxWaves];
  const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  const int unit = blockIdx.x;
  const int k = p.k, n = p.n;
  const bool full = (n == k);
  int slot = n;  // below capacity the new rows take slot n
  if (full) {
    const float* w = p.w + (size_t)unit * p.H * (k + 1);
    float best = INFINITY;
    int bj = 0x7fffffff;
    for (int j = tid; j <= k; j += nt) {  // ascending, strict <: the lowest index wins ties
      float s = 0.f;
      constexpr int HB = 16;  // heads whose loads are issued together
      for (int h0 = 0; h0 < p.H; h0 += HB) {
        float v[HB];
#pragma unroll
        for (int u = 0; u < HB; ++u) v[u] = (h0 + u < p.H) ? w[(size_t)(h0 + u) * (k + 1) + j] : 0.f;
#pragma unroll
        for (int u = 0; u < HB; ++u) s += v[u];  // (head order)
      }
      if (j >= p.n_pinned && s < best) {
        best = s;
        bj = j;
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      const float ob = __shfl_xor(best, o);
      const int oj = __shfl_xor(bj, o);
      if (ob < best || (ob == best && oj < bj)) {
        best = ob;
        bj = oj;
      }
    }
    if (lane == 0) {
      bv[wave] = best;
      bi[wave] = bj;
    }
    __syncthreads();
    best = bv[0];
    bj = bi[0];
    for (int x = 1; x < nw; ++x) {
      if (bv[x] < best || (bv[x] == best && bi[x] < bj)) {
        best = bv[x];
        bj = bi[x];
      }
    }
    if (bj > k) bj = k;  // only reachable with non-finite weights
    slot = bj;
  }
  if (slot < k) {  // (slot == k: the incoming token itself is dropped)
    const int row16 = p.row_bytes / 16;  // 16-byte pieces per row
    const V16* kn = reinterpret_cast<const V16*>(static_cast<const char*>(p.k_new) + (size_t)unit * p.H_kv * p.row_bytes);
    const V16* vn = reinterpret_cast<const V16*>(static_cast<const char*>(p.v_new) + (size_t)unit * p.H_kv * p.row_bytes);
    char* Ku = static_cast<char*>(p.K) + ((size_t)unit * p.H_kv * k + slot) * p.row_bytes;
    char* Vu = static_cast<char*>(p.V) + ((size_t)unit * p.H_kv * k + slot) * p.row_bytes;
    for (int x = tid; x < p.H_kv * row16; x += nt) {  // rows of consecutive KV heads are contiguous in k_new
      const int h = x / row16, c = x - h * row16;
      reinterpret_cast<V16*>(Ku + (size_t)h * k * p.row_bytes)[c] = kn[x];
      reinterpret_cast<V16*>(Vu + (size_t)h * k * p.row_bytes)[c] = vn[x];
    }
  }
  if (tid == 0) {
    if (p.evicted) p.evicted[unit] = full ? slot : -1;
    if (slot < k) p.slot_token[(size_t)unit * k + slot] = p.t;
    p.occupancy[unit] = full ? k : n + 1;
  }
}

}  // namespace

hipError_t launch_policy(const PolicyParams& p, hipStream_t stream) {
  // The loads in flight are what streams the weights: with few units a thread per candidate, up to
  // the largest workgroup (256 units, k = 4096: 5.9 TB/s against 4.2 with 256 threads); with many
  // units several small workgroups per CU do better (2048 units, k = 1024: 5.7 against 4.5 TB/s).
  int block = (p.k + 1 + 63) / 64 * 64;
  if (block > 1024) block = 1024;
  if (p.units >= 1024 && block > 256) block = 256;
  hipLaunchKernelGGL(tova_policy_kernel, dim3(p.units), dim3(block), 0, stream, p);
  return hipGetLastError();
}

}  // namespace tova
