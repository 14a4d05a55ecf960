// Shared between the host API (tova_api.cpp) and the device code (tova_kernels.hip, tova_prefill.hip,
// tova_repos.hip).
#ifndef TOVA_INTERNAL_H
#define TOVA_INTERNAL_H

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace tova {



// Which row leaves a full multi-state (tova_config_t.policy).
enum { kPolicyTova = 0, kPolicyWindow = 1, kPolicyH2O = 2 };

// Arguments of one step launch (one token for every unit).
struct StepParams {
  const void* q;       // [units][H][d]
  const void* k_new;   // [units][H_kv][d]
  const void* v_new;   // [units][H_kv][d]
  void* out;           // [units][H][d]
  int32_t* evicted;    // [units] or null
  void* K;             // [units][H_kv][k][d]
  void* V;
  int32_t* occupancy;  // [units]
  int32_t* slot_token; // [units][k]
  float* sg;           // [pairs][kp]        per-KV-head partial of the score vector
  float* escr;         // [pairs][kp][G]     chunk-local exp values   (S > 1 only)
  float* stats;        // [pairs][S][G][2]   chunk-local (max, sum)   (S > 1 only)
  float* accp;         // [2][pairs][S][G][d] chunk-local PV partials, by token parity (S > 1 only)
  int64_t accp_half;   // floats per parity copy
  int32_t* cnt_pair;   // [2][pairs] arrival counters (by token parity), zero between launches
  int32_t* cnt_unit;   // [2][units] (by token parity)
  int32_t* cnt_pub;    // [2][pairs] chunks that have published their softmax statistics (S > 1 only)
  int32_t* slow_flag;  // [pairs][S] chunk left its exp values in escr for the finisher (S > 1 only)
  int32_t st_off;      // float offset, inside the big LDS area, of the chunk-statistics area (S > 1)
  int32_t red_off;     // float offset of the cross-wave PV reduction area: 0 (it reuses the logit area), or
                       // behind the logits when they are still needed after the PV pass (S > 1)
  int32_t spin_limit;  // how often a chunk re-reads the published count before giving up (S > 1)
  int32_t force_slow;  // test hook: no chunk finishes its own scores
  // multi-step launch
  int32_t n_iter;      // decode steps handled by this launch (1 for a per-step launch)
  int32_t persistent;  // blocks keep their (unit, KV head) over n_iter steps and wait for victims
  int32_t unit_mode;   // one block per unit, KV heads in turn: scores and victim stay inside the block
                       // (st_off is then the float offset of the [k + 1] score row in the big LDS area)
  int32_t persist_spin;          // polls of the unit's state word before a block gives up
  int64_t q_stride, kv_stride;   // elements between consecutive steps of q / out and of k_new / v_new
  unsigned long long* pstate;    // [units] (victim << 32) | (token index + 1) of the unit's last finished step
  int32_t* error_flag;           // set when a block gave up waiting
  int32_t pairs;       // units * H_kv
  int32_t H, H_kv, k;
  int32_t n_pinned;    // candidates 0..n_pinned-1 are never the victim
  int32_t policy;      // kPolicyTova / kPolicyWindow / kPolicyH2O (the last two: unit_mode only)
  int32_t h2o_recent;  // H2O: the most recent tokens, the incoming one included, that cannot leave
  float* acc;          // H2O: [units][k] head-summed attention weights aggregated per slot
  int32_t n;           // rows cached before this step, min(t, k)
  int32_t S, R;        // chunks per KV head, slots per chunk
  int32_t kp;          // k + 1 rounded up to 64: stride of sg / escr
  int32_t t;           // index of the incoming token
  const int32_t* t_dev;  // non-null: read the index from there instead (a step recorded into a graph)
  int32_t svc;         // multi-step launch, hand-off form: the block's last wave serves the hand-off instead of streaming V
  float scale;
};

// Arguments of one launch of the multi-token kernel (groups of C tokens of a prompt, one
// workgroup per unit; either the cache is full, or it is filling and has room for every group).
struct PrefillParams {
  const void* q;       // [n_chunks * C][units][H][d]   first token of the launch
  const void* k_new;   // [n_chunks * C][units][H_kv][d]
  const void* v_new;
  void* out;           // like q
  int32_t* evicted;    // [n_chunks * C][units] or null
  void* K;             // [units][H_kv][k][d]
  void* V;
  int32_t* occupancy;  // [units]
  int32_t* slot_token; // [units][k]
  float* uscr;         // [grid][H][C][d] fp32: unmasked PV sums of the unit a workgroup is at
  int32_t filling;     // the multi-state is not full and stays within capacity during this launch:
                       // groups only append their tokens (n0 = rows cached when the launch starts)
  int32_t n0;
  int64_t q_stride, kv_stride;  // elements between consecutive tokens of q / out and of k_new / v_new
  int32_t n_chunks;    // groups of C tokens in this launch
  int32_t units, H, H_kv, k;
  int32_t n_pinned;
  int32_t t;           // index of the first token of the launch
  int32_t e_floats;    // floats of the first big LDS area (logits / reduction / resolution buffers)
  int32_t ncp;         // k + C rounded up to a multiple of 4: stride of the tentative score rows
  int32_t force_exact; // test hook: every token of a full-cache group is computed from scratch (the guard's route)
  float scale;
  // few units: the KV heads of a unit dealt to `parts` workgroups, every workgroup of the grid resident
  int32_t parts;       // 1 = a workgroup owns a unit; else a divisor of H_kv, and the grid is units * parts
  int32_t spin;        // polls of a unit's state word before a workgroup gives up
  float* tpart;        // [units][parts][C][ncp] partial tentative-score rows
  float* stat;         // [units][H][C][2]       (max, sum) per (head, token)
  int32_t* gpos;       // [units][8]             slot every token of the unit's last resolved group ended up in (-1: none)
  int32_t* cnt_unit;   // [units] arrival counters, zero between groups
  unsigned long long* pstate;  // [units] groups of this launch resolved so far
  int32_t* error_flag; // set when a workgroup gave up waiting
};

// Arguments of one launch of the kernel for decode steps with re-assigned positions (tova_repos.hip):
// a workgroup per unit, all steps of the call, fill phase included.
struct ReposParams {
  const void* q;       // [n_iter][units][H][d]   without positional encoding
  const void* k_new;   // [n_iter][units][H_kv][d] without positional encoding
  const void* v_new;
  void* out;           // like q
  int32_t* evicted;    // [n_iter][units] or null
  void* K;             // [units][H_kv][k][d]  keys without positional encoding
  void* V;
  int32_t* occupancy;  // [units]
  int32_t* slot_token; // [units][k]
  int64_t q_stride, kv_stride;  // elements between consecutive steps of q / out and of k_new / v_new
  double log2_base;    // log2 of the rotary base
  int32_t n0;          // rows cached when the launch starts, min(t, k)
  int32_t n_iter;      // decode steps of this launch
  int32_t units, H, H_kv, k;
  int32_t n_pinned;
  int32_t t;           // index of the first incoming token
  int32_t e_floats;    // floats of the first big LDS area (logits / PV reduction / position scratch)
  int32_t persist;     // LDS has room for the token order and the ranks outside that area (kept from step to step)
  float scale;
  // few units: the KV heads of a unit dealt to `parts` workgroups (cache full, all workgroups resident)
  int32_t parts;       // 1 = a workgroup owns a unit; else a divisor of H_kv, and the grid is units * parts
  int32_t spin;        // polls of a unit's state word before a workgroup gives up
  float* sg;           // [units][parts][k + 1 rounded up to 4] partial head sums of a step
  int32_t* cnt_unit;   // [units] arrival counters, zero between steps
  unsigned long long* pstate;  // [units] (victim << 32) | (token index + 1) of the unit's last finished step
  int32_t* error_flag; // set when a workgroup gave up waiting
};

// Arguments of the stand-alone policy kernel (tova_policy.hip): one step, weights given.
struct PolicyParams {
  const float* w;      // [units][H][k + 1] last query's attention weights, the incoming token last
  const void* k_new;   // [units][H_kv][d]
  const void* v_new;
  int32_t* evicted;    // [units] or null
  void* K;             // [units][H_kv][k][d]
  void* V;
  int32_t* occupancy;  // [units]
  int32_t* slot_token; // [units][k]
  int32_t n;           // rows cached before this step, min(t, k)
  int32_t units, H, H_kv, k;
  int32_t n_pinned;
  int32_t t;           // index of the incoming token
  int32_t row_bytes;   // d * sizeof(element)
};

struct LaunchPlan {
  int32_t grid, block, lds_bytes;
};

hipError_t launch_step(int dtype_is_bf16, int D, int G, const StepParams& p, const LaunchPlan& lp,
                       hipStream_t stream);
hipError_t launch_prefill(int dtype_is_bf16, int D, int G, int C, const PrefillParams& p, const LaunchPlan& lp,
                          hipStream_t stream);
hipError_t launch_repos(int dtype_is_bf16, int D, int G, const ReposParams& p, const LaunchPlan& lp, hipStream_t stream);
// how many workgroups of that kernel fit on the current device at once; 0 if the query fails
int repos_resident_blocks(int dtype_is_bf16, int D, int G, int block, int lds_bytes);
int prefill_resident_blocks(int dtype_is_bf16, int D, int G, int C, int block, int lds_bytes);
hipError_t launch_policy(const PolicyParams& p, hipStream_t stream);
hipError_t launch_fill_i32(int32_t* dst, int32_t value, size_t count, hipStream_t stream);
// *dst += add, by a kernel of its own (so that it is ordered behind the kernels that read *dst)
hipError_t launch_add_i32(int32_t* dst, int32_t add, hipStream_t stream);
// nonzero while the stream is being recorded into a graph
int stream_is_capturing(hipStream_t stream);
// waits for the stream, then copies one int32 from device memory to *host
hipError_t read_i32_sync(const int32_t* dev, hipStream_t stream, int32_t* host);
// how many blocks of the step kernel (given instantiation, block size, dynamic LDS) fit on the
// current device at once; 0 if the query fails
int resident_blocks(int dtype_is_bf16, int D, int G, int block, int lds_bytes, int unit_mode);
// compute units of the current device; 0 if the query fails
int device_cus();
// device address and size of the library's static scratch area on the current device
// (tova_static_scratch.hip; looked up once per device, nothing is allocated)
hipError_t static_scratch(void** ptr, size_t* bytes);

}  // namespace tova
#endif
