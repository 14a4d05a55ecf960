// TOVA bounded-KV-cache decode step for gfx950 (MI355X): device code and launchers.
//
// One kernel launch advances every (layer, sequence) unit by one token
// (Sec. 3.2: append the new row, attend; Sec. 4 / App. B Alg. 1: average the
// attention weights over heads, argmin, drop that row).
//
// Work decomposition.  Two forms, chosen by the host:
//  * a workgroup per (unit, KV head, slot chunk): it streams its chunk of K once and its chunk of
//    V once; the head-group partials of the score vector and (with several chunks) the chunks'
//    softmax statistics and PV partials are handed between workgroups through device memory;
//  * a workgroup per unit (many units): it goes through the unit's KV heads in turn and keeps the
//    head-summed scores in LDS, so nothing is handed to anybody.
// In both, rows are read 16 bytes per lane and laid across adjacent lanes so that every wave-level
// load covers whole, contiguous rows, and the G = H / H_kv query heads that share a KV head are
// all served from the same streamed row (grouped-query attention reads K/V once, not G times).
//
//   phase 1  logits   l[i][g] = scale * q_g . K[i]      -> LDS   (vector ALU; matrix cores for bf16
//                                                                 groups of 8 heads, of 4 at d = 128)
//   phase 2  softmax  m_g, e[i][g] = exp(l - m_g), Z_g  (chunk-local), score contributions
//   phase 3  PV       acc_g = sum_i e[i][g] * V[i]               (likewise; see pv_pass_mfma)
//   phase 4  combine  (a) per (unit, KV head): merge the chunks' (m, Z, acc) -> out
//                     (b) per unit: sum the score partials over KV heads in fixed order, argmin
//                         with lowest-index tie break, put the new row into the victim's slot,
//                         log `evicted`.
//
// Hand-offs between workgroups use "the last one to arrive does the merge": results are written
// with agent-scope (write-through) stores, an atomic counter elects the finisher, the finisher
// reads with agent-scope (cache-bypassing) loads.  Per-step launches never wait for another
// workgroup.  The bounded exceptions: a chunk looks a limited number of times for its siblings'
// softmax statistics (and leaves its score rows to the finisher if they are not there), and in a
// multi-step launch a workgroup waits, with a limit and an error flag, for the victim of its own
// unit's previous step.  Every wave reaches its exit whatever the scheduling order.
// In multi-step launches the host may give a workgroup a service wave, which does the hand-off work
// of phases 2 and 4(b) while the other waves are in phase 3 (see SVC in the kernel).
//
// The path is bound by HBM bandwidth (2*k*d*sizeof(elem) bytes per KV head and step against
// 4*G*k*d flops).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tova_internal.h"

#include "tova_device.h"  // element types, cross-lane and cross-workgroup helpers, row geometry

namespace tova {
namespace {


template <typename T, int D, int G, bool MULTI, bool UNIT = false, bool SVC = false>
__global__ __launch_bounds__(512, (G >= 8) ? ((MULTI && !UNIT) ? 2 : 3) : (PvMfma<T, D, G>::OK ? (SVC ? 2 : 3) : ((SVC && G >= 2) ? 3 : 4))) void tova_step_kernel(const StepParams p) {
  static_assert(MULTI || !UNIT, "the one-block-per-unit form is built on the multi-step loop");
  static_assert(!SVC || (MULTI && !UNIT), "the service wave belongs to multi-step launches of the hand-off form");
  using E = Elem<T>;
  using Ge = Geo<T, D, G>;
  constexpr int VEC = Ge::VEC, LV = Ge::LV;
  // V rows per lane and register buffer.  Wide groups in the hand-off form run two 256-thread workgroups per
  // CU (two waves per SIMD): with so few waves the V stream is bound by the loads in flight, so the tiles are
  // twice as deep there (config 5: 59.6 -> 57.1 us per step; a workgroup per unit has more waves and loses
  // with the deeper tiles, 759 -> 839 us, so it keeps the shallow ones; deeper K tiles gave nothing).
  constexpr int UV = (G >= 8 && MULTI && !UNIT) ? 4 : Ge::UV;
  // bf16, d = 128, 8 heads per KV head: the PV pass runs on the matrix cores as well (pv_pass_mfma)
  constexpr bool PVM = PvMfma<T, D, G>::OK;

  extern __shared__ float4 smem4[];
  float* small = reinterpret_cast<float*>(smem4);  // kSmallFloats
  float* big = small + kSmallFloats;
  int* flag_lds = reinterpret_cast<int*>(small + 480);

  const int nt = blockDim.x;
  const int nw = nt >> 6;
  // Service wave (SVC: multi-step launches of the hand-off form, when the host asks for it): the block's last wave
  // takes no part in the PV pass.  While the others stream V it does everything that stands between the
  // softmax and the unit's victim -- the chunk's statistics and score rows, the arrival at the unit's counter
  // and, for the last arrival of the unit, the scan, the argmin and the publication -- so that chain runs
  // beside the V stream instead of behind it.
  constexpr bool svc = SVC;
  const int nws = SVC ? nw - 1 : nw;  // waves of the PV pass

  // Per-step launch (MULTI == false): blockIdx -> (pair = (unit, KV head), chunk); one pass.
  // Consecutive block ids go to consecutive XCDs, so the S chunks of one pair are placed on the
  // same XCD (their partial results then meet in one L2).
  //
  // Multi-step launch (MULTI == true; one chunk per KV head, cache full, every block of the grid
  // resident): block b keeps the pairs b, b + gridDim, ... for all n_iter steps and walks them in
  // (step, pair) order.  There is no grid-wide barrier between steps: units advance independently,
  // and the only wait is a block's wait for the victim of a unit's previous step when it comes
  // back to one of that unit's pairs (every wait is for work that is earlier in the common order,
  // so some block can always make progress).  Each block stores the incoming row of its own pairs
  // itself, so cached rows are only ever written and read by one and the same block.
  //
  // One block per unit (UNIT == true, chosen by the host when there are at least as many units as
  // blocks that fit on the device; always one chunk per KV head): block b keeps the units b,
  // b + gridDim, ... and goes through the KV heads of a unit one after the other.  The head-summed
  // scores then never leave LDS and the victim is found by the block itself: no score rows in
  // device memory, no counters, no waiting for other blocks, and the grid may have any size.
  const int S = p.S, R = p.R, k = p.k, n = p.n;
  const int c_new = min(n / R, S - 1);  // the chunk that also takes the incoming token
  const bool full = (n == k);
  constexpr int ROW16 = D * (int)sizeof(T) / 16;  // 16-byte pieces per row
  // Work items are (pair, chunk) with the chunk index fastest; item li of XCD x is pair
  // (li / S) * 8 + x, so the chunks of a pair, and the pairs of a unit, sit on neighbouring blocks.
  const int xcd = blockIdx.x & 7;
  const int li0 = UNIT ? (int)blockIdx.x : (int)(blockIdx.x >> 3);
  const int li_stride = UNIT ? (int)gridDim.x : MULTI ? (int)(gridDim.x >> 3) : 0x40000000;  // per-step launch: one item per block
  const int li_end = UNIT ? p.pairs / p.H_kv : ((p.pairs + 7) >> 3) * S;
  if (!MULTI) {
    if ((li0 / S) * 8 + xcd >= p.pairs || li0 % S > c_new) return;
  }
  // (without UNIT, an extra pass stores the last step's rows)
  const int n_pass = UNIT ? p.n_iter : MULTI ? p.n_iter + 1 : 1;

  for (int it = 0; it < n_pass; ++it) {
  // (a per-step launch makes exactly one trip through both loops, and the compiler can see that)
  for (int li = li0, trip = 0; MULTI ? (li < li_end) : (trip == 0); li += li_stride, ++trip) {
  const int pair0 = UNIT ? li * p.H_kv : (li / S) * 8 + xcd;  // the item's (first) pair
  const int chunk = UNIT ? 0 : li % S;
  if (MULTI && !UNIT && pair0 >= p.pairs) continue;
  // In a multi-step launch the thread index is re-read through an opaque copy in every pass:
  // otherwise the compiler hoists the lane-dependent address arithmetic of the whole body out of
  // the loops and keeps it in registers across them (+40 VGPRs and spills).
  int tid = threadIdx.x;
  if (MULTI) asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = MULTI ? __builtin_amdgcn_readfirstlane(tid >> 6) : (tid >> 6);
  const int unit = UNIT ? li : pair0 / p.H_kv;
  const int r0 = chunk * R;
  const int r1 = min(r0 + R, n);
  const int ncached = r1 - r0;                 // cached rows of this chunk
  const bool has_new = (chunk == c_new);       // local candidate `ncached` is the incoming token
  const int nloc = ncached + (has_new ? 1 : 0);  // local candidates, >= 1
  // index of the incoming token: the host's count, or (a step recorded into a graph, replayed for token
  // after token) the count kept in state_mem, which a kernel of its own advances after this one
  const int tok = (p.t_dev ? __builtin_amdgcn_readfirstlane(ld_agent_i(p.t_dev)) : p.t) + it;

  if (MULTI && !UNIT && it > 0) {
    const int pair = pair0;
    const T* Kb = reinterpret_cast<const T*>(p.K) + ((size_t)pair * k + r0) * D;
    const T* Vb = reinterpret_cast<const T*>(p.V) + ((size_t)pair * k + r0) * D;
    // Wait (bounded) for the victim of this unit's previous step, then put that step's incoming
    // row of this KV head into the freed slot.  If the wait runs out -- it cannot while all blocks
    // are resident, which the host checks before choosing this launch mode -- the block raises the
    // cache's error flag and leaves; every other block sees the flag in its own wait and leaves too.
    if (tid == 0) {
      unsigned long long w = 0;
      int ok = 0;
      for (int spin = 0;; ++spin) {
        w = ld_agent_u64(p.pstate + unit);
        if ((int)(uint32_t)w == tok) {
          ok = 1;
          break;
        }
        if (spin >= p.persist_spin || ld_agent_i(p.error_flag) != 0) break;
        __builtin_amdgcn_s_sleep(4);
      }
      if (!ok) st_agent_i(p.error_flag, 1);
      flag_lds[2] = ok;
      flag_lds[3] = (int)(w >> 32);
    }
    __syncthreads();
    if (flag_lds[2] == 0) return;  // block-uniform
    const int vic = flag_lds[3];
    // The log entries of that step are written here, by the workgroup that has the unit's first KV head and
    // first chunk: always the same thread, so entries of one slot in successive steps stay in order, and the
    // unit's finisher can publish the victim without waiting for any store of its own.
    if (tid == 0 && chunk == 0 && pair == unit * p.H_kv) {
      if (p.evicted) p.evicted[(size_t)(it - 1) * (p.pairs / p.H_kv) + unit] = vic;
      if (vic < k) p.slot_token[(size_t)unit * k + vic] = tok - 1;
      p.occupancy[unit] = k;
    }
    if (vic >= r0 && vic < r1 && tid < ROW16) {  // (vic == k: the incoming token was dropped) the chunk that owns the slot
      const T* kprev = reinterpret_cast<const T*>(p.k_new) + (size_t)(it - 1) * p.kv_stride + (size_t)pair * D;
      const T* vprev = reinterpret_cast<const T*>(p.v_new) + (size_t)(it - 1) * p.kv_stride + (size_t)pair * D;
      reinterpret_cast<V16*>(const_cast<T*>(Kb) + (size_t)(vic - r0) * D)[tid] = reinterpret_cast<const V16*>(kprev)[tid];
      reinterpret_cast<V16*>(const_cast<T*>(Vb) + (size_t)(vic - r0) * D)[tid] = reinterpret_cast<const V16*>(vprev)[tid];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();  // the row is in place for this block's pass over the pair
    if (it == p.n_iter) continue;
  }

  int32_t* const evp = p.evicted ? p.evicted + (size_t)it * (p.pairs / p.H_kv) : nullptr;

  float* e_lds = big;  // [nloc][G]: logits (log2 domain), then exp values
  float* s_lds = big + p.st_off;  // UNIT: [k + 1] head-summed scores of the unit
  const float scale2 = p.scale * kLog2e;  // softmax is evaluated as 2^(l2 - max l2)

  for (int kv_i = 0; kv_i < (UNIT ? p.H_kv : 1); ++kv_i) {  // UNIT: the KV heads of the unit in turn
  // (UNIT: a fresh opaque copy of the thread index per KV head, for the same reason as above)
  int tid = threadIdx.x;
  if (MULTI) asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = MULTI ? __builtin_amdgcn_readfirstlane(tid >> 6) : (tid >> 6);
  const int pair = pair0 + kv_i;
  const int kvh = pair - unit * p.H_kv;
  const T* Kb = reinterpret_cast<const T*>(p.K) + ((size_t)pair * k + r0) * D;
  const T* Vb = reinterpret_cast<const T*>(p.V) + ((size_t)pair * k + r0) * D;
  const T* knew = reinterpret_cast<const T*>(p.k_new) + (size_t)it * p.kv_stride + (size_t)pair * D;
  const T* vnew = reinterpret_cast<const T*>(p.v_new) + (size_t)it * p.kv_stride + (size_t)pair * D;
  const T* qb = reinterpret_cast<const T*>(p.q) + (size_t)it * p.q_stride +
                ((size_t)unit * p.H + (size_t)kvh * G) * D;

  // ---------------- phase 1: logits ----------------
  // (vector ALUs, or the matrix cores for wide bf16 groups: see logit_pass; the incoming token is
  // candidate `ncached` -- App. B: the last column -- and is taken by the block's last wave)
  float m[G], Z[G];  // chunk-local softmax statistics (log2 domain)
  const bool new_here = has_new && (wave == nw - 1);    // wave-uniform: the incoming token's logits
  const bool new_here_v = has_new && (wave == nws - 1);  // ... and its value row in the PV pass
  // the pair's counters alternate with the token's parity (a block of the unit's next step may already count
  // on one copy while this step's last block still resets the other)
  int32_t* const cnt_pair_p = p.cnt_pair + (size_t)(tok & 1) * p.pairs + pair;
  int32_t* const cnt_unit_p = p.cnt_unit + (size_t)(tok & 1) * (p.pairs / p.H_kv) + unit;  // (likewise the unit's)
  int32_t* const cnt_pub_p = p.cnt_pub + (size_t)(tok & 1) * p.pairs + pair;
  const int rst_tid = svc ? (nw - 1) * 64 : 0;  // who resets counters: with a service wave its first lane, whose
                                                // own wait for its stores precedes the unit's next arrival
  logit_pass<T, D, G>(
      Kb, ncached, 1, new_here, [&](int g) { return qb + g * D; }, [&](int) { return knew; },
      [](int, int) { return false; }, scale2, lane, wave, nw, e_lds, m);

  // The first PV tile is requested now, so that the V stream is already in flight while the
  // block goes through the softmax barriers.
  const int lv = lane % LV;
  const int rv = lane / LV;
  V16 vA[PVM ? 8 : UV];
  if (!SVC || wave < nws) {
    if constexpr (PVM)
      pv_mfma_load<T, D>(vA, Vb, wave * PvMfma<T, D, G>::ROWS, ncached, lane);
    else
      pv_first_tile<T, D, G>(vA, Vb, ncached, lane, wave);
  }

  // ---------------- phase 2: chunk-local softmax ----------------
  // The barrier inside this reduction is also the one that makes the logits visible.
  block_reduce<G, true>(m, small, lane, wave, nw);
#pragma unroll
  for (int g = 0; g < G; ++g) Z[g] = 0.f;
  for (int i = tid; i < nloc; i += nt) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float e = __builtin_amdgcn_exp2f(e_lds[i * G + g] - m[g]);
      e_lds[i * G + g] = e;
      Z[g] += e;
    }
  }
  // ... and the barrier inside this one completes e_lds for the PV pass.
  block_reduce<G, false>(Z, small + kMaxWaves * G, lane, wave, nw);

  // Score contributions leave LDS before the PV pass (each thread re-reads only exp values it
  // wrote itself, so no barrier is needed in front).
  //  * one chunk per KV head: Z is final.
  //  * several chunks: the chunk publishes its (max, sum) now and goes on to its PV pass, which
  //    needs chunk-local values only.  After the pass it looks, a bounded number of times,
  //    whether its siblings have published theirs -- they run on neighbouring CUs at the same
  //    time, so by then they have -- and rescales its exp values, which are kept in LDS through
  //    the pass (the cross-wave reduction area does not reuse that memory in this case), to
  //    final probabilities itself.  If not (a sibling was scheduled much later) it leaves the
  //    exp values in scratch for the pair's finisher.  No wave ever waits without bound.
  const int nact = c_new + 1;         // chunks of this pair that run this step
  float* sl = big + p.st_off;         // [nact][G][2]  all chunks' (max, sum)
  float* wl = sl + 2 * nact * G;      // [nact][G]     2^(m_c - m_g)   (pair finisher)
  float* zl = wl + nact * G;          // [G]           global sum      (pair finisher)
  const float* stp = p.stats + (size_t)pair * S * G * 2;
  bool have_stats = false;            // sl holds the final statistics of every chunk
  int slow = 0;                       // this chunk's score rows are left to the pair finisher
  if (S == 1) {
    if (full || (UNIT && p.policy == kPolicyH2O)) {  // (H2O aggregates the weights of every step, Sec. 4.1)
      float rz[G];
#pragma unroll
      for (int g = 0; g < G; ++g) rz[g] = 1.0f / Z[g];
      float* sg = p.sg + (size_t)pair * p.kp;
      // (a service wave writes the rows itself, see below: its arrival then only waits for its own stores)
      if (!svc) {
        for (int i = tid; i < nloc; i += nt) {
          float a = 0.f;
#pragma unroll
          for (int g = 0; g < G; ++g) a = fmaf(e_lds[i * G + g], rz[g], a);
          if (UNIT)
            s_lds[i] = (kv_i == 0) ? a : s_lds[i] + a;  // (entry i is always this thread's; heads in order)
          else
            st_agent(sg + i, a);
        }
      }
    }
  } else if (!svc) {
    if (wave == 0) {  // wave-uniform: the stores and the counter update are this wave's alone
      if (lane < G) {
        float mg = m[0], zg = Z[0];
#pragma unroll
        for (int g = 1; g < G; ++g) {
          mg = (lane == g) ? m[g] : mg;
          zg = (lane == g) ? Z[g] : zg;
        }
        float* st = p.stats + (((size_t)pair * S + chunk) * G + lane) * 2;
        st_agent(st, mg);
        st_agent(st + 1, zg);
      }
      if (full) {
        // ... and says so on the pair's counter once the stores have completed.  Nobody waits here:
        // the siblings' statistics are only needed after the PV pass (see phase 4a), by which time
        // they have long arrived.
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        if (lane == 0) __hip_atomic_fetch_add(cnt_pub_p, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }

  // The unit's finish by ONE wave (the service wave whose arrival completes the unit's count): head-mean score
  // over the k+1 candidates (as a sum: the factor 1/H does not move the argmin), KV-head partials added in
  // head order, lowest index on ties; then the log entries and the unit's state word.
  auto finish_unit_wave = [&]() {
    // (the reset lands before anyone counts on this copy again, two steps on: this wave waits for its stores
    // before it arrives in the unit's next step)
    if (lane == 0) st_agent_i(cnt_unit_p, 0);
    const float* sgu = p.sg + (size_t)unit * p.H_kv * p.kp;
    float best = INFINITY;
    int bj = 0x7fffffff;
    if (p.H_kv <= 2)
      scan_scores<8, 2>(sgu, p.H_kv, p.kp, k, p.n_pinned, lane, 64, best, bj);
    else if (p.H_kv <= 4)
      scan_scores<8, 4>(sgu, p.H_kv, p.kp, k, p.n_pinned, lane, 64, best, bj);
    else
      scan_scores<4, 8>(sgu, p.H_kv, p.kp, k, p.n_pinned, lane, 64, best, bj);
    wave_argmin(best, bj);
    if (bj > k) bj = k;  // only reachable with non-finite scores
    // (the log entries are written by the unit's first workgroup when it reads this word)
    if (lane == 0) st_agent_u64(p.pstate + unit, ((unsigned long long)(uint32_t)bj << 32) | (uint32_t)(tok + 1));
  };

  // What the service wave does while the other waves are in the PV pass (called in the other branch of
  // that pass, so that the registers of the V tiles are not live here).
  auto service_wave_work = [&]() {
    int ok = full ? 1 : 0;  // (the cache is full in every multi-step launch)
    if (S == 1) {
      if (ok) {
        float rz[G];
#pragma unroll
        for (int g = 0; g < G; ++g) rz[g] = 1.0f / Z[g];
        float* sg = p.sg + (size_t)pair * p.kp;
        for (int i = lane; i < nloc; i += 64) {
          float a = 0.f;
#pragma unroll
          for (int g = 0; g < G; ++g) a = fmaf(e_lds[i * G + g], rz[g], a);
          st_agent(sg + i, a);
        }
      }
    } else {
      // the chunk's statistics, as wave 0 publishes them without a service wave
      if (lane < G) {
        float mg = m[0], zg = Z[0];
#pragma unroll
        for (int g = 1; g < G; ++g) {
          mg = (lane == g) ? m[g] : mg;
          zg = (lane == g) ? Z[g] : zg;
        }
        float* st = p.stats + (((size_t)pair * S + chunk) * G + lane) * 2;
        st_agent(st, mg);
        st_agent(st + 1, zg);
      }
      if (ok) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        if (lane == 0) __hip_atomic_fetch_add(cnt_pub_p, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    if (ok && S > 1) {
      // the siblings' statistics (they run at the same time on neighbouring CUs): a bounded look, else the
      // block takes the route behind its PV pass as it does without a service wave
      int seen = 0;
      if (lane == 0) {
        seen = ld_agent_i(cnt_pub_p);
        for (int sp = 0; sp < p.spin_limit && seen != nact; ++sp) {
          __builtin_amdgcn_s_sleep(16);
          seen = ld_agent_i(cnt_pub_p);
        }
      }
      seen = __builtin_amdgcn_readfirstlane(seen);
      ok = (seen == nact && !p.force_slow) ? 1 : 0;
      if (ok) {
        for (int x = lane; x < nact * G * 2; x += 64) sl[x] = ld_agent(stp + x);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();  // (one wave: its LDS accesses are performed in order)
        float f[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float mg = -INFINITY;
          for (int c = 0; c < nact; ++c) mg = fmaxf(mg, sl[(c * G + g) * 2]);
          float zg = 0.f;
          for (int c = 0; c < nact; ++c)
            zg += sl[(c * G + g) * 2 + 1] * __builtin_amdgcn_exp2f(sl[(c * G + g) * 2] - mg);
          f[g] = __builtin_amdgcn_exp2f(sl[(chunk * G + g) * 2] - mg) / zg;
        }
        float* sg = p.sg + (size_t)pair * p.kp + r0;
        for (int i = lane; i < nloc; i += 64) {
          float a = 0.f;
#pragma unroll
          for (int g = 0; g < G; ++g) a = fmaf(e_lds[i * G + g], f[g], a);
          st_agent(sg + i, a);
        }
      }
    }
    if (ok) {
      // arrival at the unit's counter, once this wave's score rows have completed
      const int expected = p.H_kv * nact;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_s_waitcnt(0);
      int prev = 0;
      if (expected > 1 && lane == 0)
        prev = __hip_atomic_fetch_add(cnt_unit_p, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      prev = __builtin_amdgcn_readfirstlane(prev);
      if (prev + 1 == expected) finish_unit_wave();
    }
    if (lane == 0) flag_lds[4] = ok;
  };

  // ---------------- phase 3: PV ----------------
  float* red = big + p.red_off;  // [nw][G*D]; behind the exp values when they are still needed (S > 1)
  // (the waves of the pass compute, all waves meet at the barrier after which the reduction area may reuse the
  // memory of the exp values -- a service wave gets there when its own work is done --, then the waves of the
  // pass write their sums)
  const bool pv_wave = !SVC || wave < nws;  // wave-uniform
  if constexpr (PVM) {
    // Matrix cores (see pv_pass_mfma; the incoming token's row is added on the vector ALUs).
    float tot[4][4];
    if (pv_wave) {
      f32x4_t pacc[8];
      pv_pass_mfma<T, D, G>(Vb, ncached, e_lds, G, 0, lane, wave, nws, vA, pacc);
      pv_mfma_fold<T, D, G>(pacc, tot, ncached, 1, new_here_v, [&](int) { return vnew; }, e_lds, G, 0, lane);
    } else {
      service_wave_work();
    }
    __syncthreads();
    if (pv_wave) pv_mfma_store<T, D, G>(tot, lane, wave, red);
  } else {
    // combine the RV row groups of the wave, then the waves (in wave order)
    constexpr bool TR = (LV == 16 && (G * VEC) % 4 == 0);
    constexpr int NV = G * VEC;
    float acc[G][VEC];
    float cr[TR ? NV / 4 : 1];
    if (pv_wave) {
      pv_pass<T, D, G>(Vb, ncached, 1, new_here_v, [&](int) { return vnew; }, e_lds, G, 0, lane, wave, nws, vA, acc);
      if constexpr (TR) {
        // Four row groups of 16 lanes.  Transposing reduction: swapping rows between the registers of
        // two different values and adding halves the number of live registers at each of the two
        // stages (odd/even rows, then upper/lower half), and leaves the total of value 4 j + r in row
        // r of register j -- so all 64 lanes, not 16, write the wave's result to LDS.
        float b[NV / 2];
#pragma unroll
        for (int j = 0; j < NV / 2; ++j) {
          unsigned x = __builtin_bit_cast(unsigned, acc[(2 * j) / VEC][(2 * j) % VEC]);
          unsigned y = __builtin_bit_cast(unsigned, acc[(2 * j + 1) / VEC][(2 * j + 1) % VEC]);
          swap_rows16(x, y);  // x: rows 0,2 keep value 2j, rows 1,3 get value 2j+1 of the row below/above
          b[j] = __builtin_bit_cast(float, x) + __builtin_bit_cast(float, y);
        }
#pragma unroll
        for (int j = 0; j < NV / 4; ++j) {
          unsigned x = __builtin_bit_cast(unsigned, b[2 * j]);
          unsigned y = __builtin_bit_cast(unsigned, b[2 * j + 1]);
          swap_rows32(x, y);
          cr[j] = __builtin_bit_cast(float, x) + __builtin_bit_cast(float, y);
        }
      } else {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[g][v] = column_sum<LV>(acc[g][v]);
      }
    } else {
      service_wave_work();
    }
    __syncthreads();  // everyone is done reading e_lds; the reduction area reuses it
    if (pv_wave) {
      if constexpr (TR) {
#pragma unroll
        for (int j = 0; j < NV / 4; ++j) {
          const int idx = 4 * j + rv;  // value index g * VEC + v held by this lane's row
          red[(wave * G + idx / VEC) * D + lv * VEC + idx % VEC] = cr[j];
        }
      } else if (rv == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int v = 0; v < VEC; ++v) red[(wave * G + g) * D + lv * VEC + v] = acc[g][v];
      }
    }
  }
  __syncthreads();
  // (with a service wave: its score rows are written and it has arrived at the unit's counter, unless it did
  // not see the siblings' statistics in time)
  const bool early = svc && flag_lds[4] != 0;  // block-uniform

  T* outb = reinterpret_cast<T*>(p.out) + (size_t)it * p.q_stride + ((size_t)unit * p.H + (size_t)kvh * G) * D;
  bool pair_last = true;  // this block completes its (unit, KV head)
  int unit_add = 1;       // what it contributes to the unit's arrival count (S > 1: per chunk)

  // One chunk per KV head: the block's own PV sums are final.  When the cache is full the stores
  // are issued after the arrival below, so that they do not sit between this block's last read of
  // K/V and the arrival (which waits for the block's outstanding stores).
  auto store_out_single = [&]() {
    for (int x = tid; x < G * D; x += nt) {
      float a = red[x];
      for (int w = 1; w < nws; ++w) a += red[w * G * D + x];
      // Z of head x / D; G is a compile-time constant so this is a select chain
      float zg = Z[0];
#pragma unroll
      for (int g = 1; g < G; ++g) zg = (x / D == g) ? Z[g] : zg;
      E::store(outb + x, a / zg);
    }
  };
  if constexpr (UNIT) {
    store_out_single();
    __syncthreads();  // the reduction area (and with it the exp values) is free for the next KV head
  } else {
  if (S == 1) {
    if (!full) store_out_single();
  } else {
    // ---------------- phase 4a: several chunks per (unit, KV head) ----------------
    // (two copies by token parity: in a multi-step launch the finisher may still be merging step t
    // when a sibling already writes its partial of step t + 1)
    float* ap = p.accp + (size_t)(tok & 1) * p.accp_half + ((size_t)pair * S + chunk) * (G * D);
    for (int x = tid; x < G * D; x += nt) {
      float a = red[x];
      for (int w = 1; w < nws; ++w) a += red[w * G * D + x];
      st_agent(ap + x, a);
    }
    if (early) have_stats = true;  // (sl was filled by the service wave)
    if (full && !early) {
      // the siblings' statistics, and with them this chunk's score rows (see phase 2)
      if (tid == 0) {
        int seen = ld_agent_i(cnt_pub_p);
        for (int sp = 0; sp < p.spin_limit && seen != nact; ++sp) {  // bounded: then the slow route
          __builtin_amdgcn_s_sleep(16);
          seen = ld_agent_i(cnt_pub_p);
        }
        flag_lds[0] = (seen == nact && !p.force_slow) ? 1 : 0;
      }
      __syncthreads();
      have_stats = (flag_lds[0] != 0);
      if (have_stats) {
        for (int x = tid; x < nact * G * 2; x += nt) sl[x] = ld_agent(stp + x);
        __syncthreads();
        float f[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float mg = -INFINITY;
          for (int c = 0; c < nact; ++c) mg = fmaxf(mg, sl[(c * G + g) * 2]);
          float zg = 0.f;
          for (int c = 0; c < nact; ++c)
            zg += sl[(c * G + g) * 2 + 1] * __builtin_amdgcn_exp2f(sl[(c * G + g) * 2] - mg);
          f[g] = __builtin_amdgcn_exp2f(sl[(chunk * G + g) * 2] - mg) / zg;  // (this chunk's own max is in there too)
        }
        float* sg = p.sg + (size_t)pair * p.kp + r0;
        for (int i = tid; i < nloc; i += nt) {
          float a = 0.f;
#pragma unroll
          for (int g = 0; g < G; ++g) a = fmaf(e_lds[i * G + g], f[g], a);
          st_agent(sg + i, a);
        }
      } else {
        slow = 1;
        float* es = p.escr + ((size_t)pair * p.kp + r0) * G;
        for (int i = tid; i < nloc; i += nt) {
#pragma unroll
          for (int g = 0; g < G; ++g) st_agent(es + i * G + g, e_lds[i * G + g]);
        }
        if (tid == 0) st_agent_i(p.slow_flag + (size_t)pair * S + chunk, 1);
      }
    }
    int n_slow = slow;
    if (nact > 1) {
      // arrivals in the low half of the counter, chunks that need the finisher's help in the high half
      const int prev = arrive(cnt_pair_p, 1 + (slow << 16), flag_lds, tid);
      pair_last = ((prev & 0xffff) == nact - 1);
      n_slow += prev >> 16;
    } else {
      __syncthreads();
    }
    unit_add = (slow || early) ? 0 : 1;
    if (pair_last) {
      // ---- pair finisher: global normalisers (log2 domain) m_g = max_c m_c, Z_g = sum_c Z_c 2^(m_c - m_g)
      if (tid == rst_tid) {
        st_agent_i(cnt_pair_p, 0);
        st_agent_i(cnt_pub_p, 0);
      }
      if (!have_stats) {  // (below capacity, or a sibling had not published when this chunk looked)
        for (int x = tid; x < nact * G * 2; x += nt) sl[x] = ld_agent(stp + x);  // all in flight at once
        __syncthreads();
      }
      if (tid < G) {
        float mg = -INFINITY;
        for (int c = 0; c < nact; ++c) mg = fmaxf(mg, sl[(c * G + tid) * 2]);
        float zg = 0.f;
        for (int c = 0; c < nact; ++c) {
          float w = __builtin_amdgcn_exp2f(sl[(c * G + tid) * 2] - mg);
          wl[c * G + tid] = w;
          zg += sl[(c * G + tid) * 2 + 1] * w;
        }
        zl[tid] = zg;
      }
      __syncthreads();
      if (full && n_slow > 0) {
        // score rows of chunks that could not finish their own (rare: flags are read one by one)
        const float* es = p.escr + (size_t)pair * p.kp * G;
        float* sg = p.sg + (size_t)pair * p.kp;
        for (int c = 0; c < nact; ++c) {
          if (ld_agent_i(p.slow_flag + (size_t)pair * S + c) == 0) continue;  // block-uniform
          const int j0 = c * R;
          const int j1 = (c == c_new) ? n + 1 : min(j0 + R, n);
          constexpr int JB = 4;  // rows per thread whose loads are issued together
          for (int jb = j0 + tid; jb < j1; jb += nt * JB) {
            float ev[JB][G];
#pragma unroll
            for (int b = 0; b < JB; ++b) {
              const int j = jb + b * nt;
#pragma unroll
              for (int g = 0; g < G; ++g) ev[b][g] = (j < j1) ? ld_agent(es + (size_t)j * G + g) : 0.f;
            }
#pragma unroll
            for (int b = 0; b < JB; ++b) {
              const int j = jb + b * nt;
              float a = 0.f;
#pragma unroll
              for (int g = 0; g < G; ++g) a = fmaf(ev[b][g], wl[c * G + g] / zl[g], a);
              if (j < j1) st_agent(sg + j, a);
            }
          }
          if (tid == 0) st_agent_i(p.slow_flag + (size_t)pair * S + c, 0);
        }
        unit_add += n_slow;  // ... on whose behalf this block now arrives at the unit's counter
      }
    }
  }

  // ---------------- phase 4b: state update ----------------
  if (!full) {
    // below capacity (App. B: num_kv <= cache_max_size): the new row takes slot n
    if (pair_last) {
      if (tid < ROW16) {
        reinterpret_cast<V16*>(const_cast<T*>(Kb) - (size_t)r0 * D + (size_t)n * D)[tid] =
            reinterpret_cast<const V16*>(knew)[tid];
        reinterpret_cast<V16*>(const_cast<T*>(Vb) - (size_t)r0 * D + (size_t)n * D)[tid] =
            reinterpret_cast<const V16*>(vnew)[tid];
      }
      if (kvh == 0 && tid == 0) {
        if (evp) evp[unit] = -1;
        p.slot_token[(size_t)unit * k + n] = tok;
        p.occupancy[unit] = n + 1;
      }
    }
  } else {
    // The unit's counter collects one arrival per (KV head, chunk); whoever completes the count
    // knows that every score row is written and that nobody reads the unit's K/V any more.
    const int expected = p.H_kv * nact;
    bool unit_last = false;
    if (S == 1 && early) unit_add = 0;
    if (unit_add == 0) {
      // (the service wave has arrived for this block, or the pair's last block will)
    } else if (expected == 1) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      unit_last = true;
    } else {
      const int prev = arrive(cnt_unit_p, unit_add, flag_lds, tid);
      unit_last = (prev + unit_add == expected);
      // (lands before anyone counts on this copy again, two steps on: every wave of this block waits for its
      // stores at the top of the unit's next step, before the block can arrive there)
      if (unit_last) reset_counter(cnt_unit_p, tid);
    }
    if (S == 1) store_out_single();
    if (unit_last) {
      // Head-mean score over the k+1 candidates (as a sum: the factor 1/H does not move the
      // argmin), KV-head partials added in head order; lowest index wins ties.
      const float* sgu = p.sg + (size_t)unit * p.H_kv * p.kp;
      // the incoming row will most likely be stored: fetch this thread's piece of it now, so that
      // its latency overlaps the score loads
      const T* kn = reinterpret_cast<const T*>(p.k_new) + (size_t)it * p.kv_stride + (size_t)unit * p.H_kv * D;
      const T* vn = reinterpret_cast<const T*>(p.v_new) + (size_t)it * p.kv_stride + (size_t)unit * p.H_kv * D;
      V16 pk = V16{{0u, 0u, 0u, 0u}}, pv = V16{{0u, 0u, 0u, 0u}};
      if (!MULTI && tid < p.H_kv * ROW16) {
        pk = reinterpret_cast<const V16*>(kn)[tid];  // rows of consecutive KV heads are contiguous
        pv = reinterpret_cast<const V16*>(vn)[tid];
      }
      float best = INFINITY;
      int bj = 0x7fffffff;
      constexpr int JM = 1;
      if (p.H_kv <= 2)
        scan_scores<8 * JM, 2>(sgu, p.H_kv, p.kp, k, p.n_pinned, tid, nt, best, bj);
      else if (p.H_kv <= 4)
        scan_scores<4 * JM, 4>(sgu, p.H_kv, p.kp, k, p.n_pinned, tid, nt, best, bj);
      else
        scan_scores<2 * JM, 8>(sgu, p.H_kv, p.kp, k, p.n_pinned, tid, nt, best, bj);
      block_argmin(best, bj, small + 256, lane, wave, nw);
      if (bj > k) bj = k;  // only reachable with non-finite scores
      if (bj < k && !MULTI) {
        T* Ku = reinterpret_cast<T*>(p.K) + ((size_t)unit * p.H_kv * k + bj) * D;
        T* Vu = reinterpret_cast<T*>(p.V) + ((size_t)unit * p.H_kv * k + bj) * D;
        for (int x = tid; x < p.H_kv * ROW16; x += nt) {
          const int h = x / ROW16, c = x - h * ROW16;
          if (x >= nt) {  // (only when a unit's new rows have more 16-byte pieces than the block has threads)
            pk = reinterpret_cast<const V16*>(kn)[x];
            pv = reinterpret_cast<const V16*>(vn)[x];
          }
          reinterpret_cast<V16*>(Ku + (size_t)h * k * D)[c] = pk;
          reinterpret_cast<V16*>(Vu + (size_t)h * k * D)[c] = pv;
        }
      }
      if (tid == 0) {
        if (MULTI) {
          // Multi-step launch: publish the victim, at once; every block stores the row of its own KV head
          // when it comes back to the pair, and the unit's first block writes the log entries then.
          st_agent_u64(p.pstate + unit, ((unsigned long long)(uint32_t)bj << 32) | (uint32_t)(tok + 1));
        } else {
          if (evp) evp[unit] = bj;
          if (bj < k) p.slot_token[(size_t)unit * k + bj] = tok;
          p.occupancy[unit] = k;
        }
      }
    }
  }

  // ---------------- the pair finisher merges the chunks' PV partials (off the critical path) ----------------
  if (S > 1 && pair_last) {
    const float* apf = p.accp + (size_t)(tok & 1) * p.accp_half + (size_t)pair * S * (G * D);
    for (int x = tid; x < G * D; x += nt) {
      const int g = x / D;
      float a = 0.f;
      constexpr int CB = 8;  // partials whose loads are issued together
      for (int c0 = 0; c0 < nact; c0 += CB) {
        float pv[CB];
#pragma unroll
        for (int u = 0; u < CB; ++u) pv[u] = (c0 + u < nact) ? ld_agent(apf + (size_t)(c0 + u) * G * D + x) : 0.f;
#pragma unroll
        for (int u = 0; u < CB; ++u) a = (c0 + u < nact) ? fmaf(pv[u], wl[(c0 + u) * G + g], a) : a;
      }
      E::store(outb + x, a / zl[g]);
    }
  }

  }  // !UNIT
  }  // KV heads of the item

  if constexpr (UNIT) {
    // ---------------- the block's own victim and state update (Sec. 4; App. B) ----------------
    const T* kn = reinterpret_cast<const T*>(p.k_new) + (size_t)it * p.kv_stride + (size_t)pair0 * D;
    const T* vn = reinterpret_cast<const T*>(p.v_new) + (size_t)it * p.kv_stride + (size_t)pair0 * D;
    int slot = n;  // below capacity (App. B: num_kv <= cache_max_size) the new row takes slot n
    if (p.policy == kPolicyH2O) {
      // H2O (Sec. 4.1): every row carries the sum of its head-summed weights over all steps since
      // its token came in; this step's weights are added first, then the row with the lowest sum
      // outside the window of the h2o_recent most recent tokens (the incoming one included) leaves.
      // A thread owns the slots j = tid, tid + nt, ...: ascending with a strict <, lowest index on ties.
      float* accu = p.acc + (size_t)unit * k;
      const int32_t* stu = p.slot_token + (size_t)unit * k;
      float best = INFINITY;
      int bj = 0x7fffffff;
      for (int j = tid; j < n; j += nt) {
        const float a = accu[j] + s_lds[j];
        accu[j] = a;
        if (full && stu[j] <= tok - p.h2o_recent && a < best) {
          best = a;
          bj = j;
        }
      }
      if (full) {
        block_argmin(best, bj, small + 256, lane, wave, nw);
        slot = bj < k ? bj : 0;  // (bj >= k is only reachable with non-finite weights)
      }
      // the incoming token starts its own sum -- written by the thread that owns the slot, after its
      // own update of the same entry above
      if (tid == slot % nt) accu[slot] = s_lds[n];
    } else if (full && p.policy == kPolicyWindow) {
      // Window+i (Sec. 4.1): the oldest token that is not one of the first n_pinned leaves; taken from
      // the slot -> token map, so any restored state is handled (tokens are distinct: no ties)
      const int32_t* stu = p.slot_token + (size_t)unit * k;
      int bt = 0x7fffffff, bj = 0x7fffffff;
      for (int j = tid; j < k; j += nt) {
        const int tj = stu[j];
        if (tj >= p.n_pinned && tj < bt) {
          bt = tj;
          bj = j;
        }
      }
      block_argmin(bt, bj, small + 256, lane, wave, nw);
      slot = bj < k ? bj : k - 1;  // (bj >= k is only reachable with a corrupt map)
    } else if (full) {
      // argmin of the head sums (the factor 1/H does not move it): a thread goes through its
      // candidates in ascending order with a strict <, so the lowest index wins ties; candidates
      // below n_pinned are kept out (TOVA+i, App. A)
      float best = INFINITY;
      int bj = 0x7fffffff;
      for (int j = tid; j <= k; j += nt) {
        const float sj = s_lds[j];
        if (j >= p.n_pinned && sj < best) {
          best = sj;
          bj = j;
        }
      }
      block_argmin(best, bj, small + 256, lane, wave, nw);
      if (bj > k) bj = k;  // only reachable with non-finite scores
      slot = bj;
    }
    if (slot < k) {  // (slot == k: the incoming token itself was dropped)
      T* Ku = reinterpret_cast<T*>(p.K) + ((size_t)pair0 * k + slot) * D;
      T* Vu = reinterpret_cast<T*>(p.V) + ((size_t)pair0 * k + slot) * D;
      for (int x = tid; x < p.H_kv * ROW16; x += nt) {  // rows of consecutive KV heads are contiguous in k_new
        const int h = x / ROW16, c = x - h * ROW16;
        reinterpret_cast<V16*>(Ku + (size_t)h * k * D)[c] = reinterpret_cast<const V16*>(kn)[x];
        reinterpret_cast<V16*>(Vu + (size_t)h * k * D)[c] = reinterpret_cast<const V16*>(vn)[x];
      }
    }
    if (tid == 0) {
      if (evp) evp[unit] = full ? slot : -1;
      if (slot < k) p.slot_token[(size_t)unit * k + slot] = tok;
      p.occupancy[unit] = full ? k : n + 1;
    }
    // the rows must have landed before other waves of this block read them in the unit's next step
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
  }
  if (MULTI) __syncthreads();  // LDS is free for the block's next pair
  }  // pairs of this block
  }  // passes
}

// Blocks of the step kernel that can be resident on the device at once.
template <typename T, int D, int G>
int resident_blocks_one(int block, int lds, int form) {  // form: 0 hand-off, 1 workgroup per unit, 2 hand-off with a service wave
  int per_cu = 0, dev = 0, cus = 0;
  const hipError_t e =
      form == 1   ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tova_step_kernel<T, D, G, true, true>, block, (size_t)lds)
      : form == 2 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tova_step_kernel<T, D, G, true, false, true>, block, (size_t)lds)
                  : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tova_step_kernel<T, D, G, true, false>, block, (size_t)lds);
  if (e != hipSuccess)
    return 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  return per_cu * cus;
}
template <typename T, int D>
int resident_blocks_g(int G, int block, int lds, int unit_mode) {
  switch (G) {
    case 1: return resident_blocks_one<T, D, 1>(block, lds, unit_mode);
    case 2: return resident_blocks_one<T, D, 2>(block, lds, unit_mode);
    case 4: return resident_blocks_one<T, D, 4>(block, lds, unit_mode);
    case 8: return resident_blocks_one<T, D, 8>(block, lds, unit_mode);
    default: return 0;
  }
}
template <typename T>
int resident_blocks_d(int D, int G, int block, int lds, int unit_mode) {
  switch (D) {
    case 32: return resident_blocks_g<T, 32>(G, block, lds, unit_mode);
    case 64: return resident_blocks_g<T, 64>(G, block, lds, unit_mode);
    case 128: return resident_blocks_g<T, 128>(G, block, lds, unit_mode);
    default: return 0;
  }
}

__global__ void tova_fill_i32_kernel(int32_t* dst, int32_t value, size_t count) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) dst[i] = value;
}

template <typename T, int D, int G>
hipError_t launch_one(const StepParams& p, const LaunchPlan& lp, hipStream_t stream) {
  if (p.unit_mode) {
    // more dynamic LDS than the default limit: say so (a workgroup per CU), once per size and device
    const hipError_t e = ensure_dynamic_lds<&tova_step_kernel<T, D, G, true, true>>(lp.lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((tova_step_kernel<T, D, G, true, true>), dim3(lp.grid), dim3(lp.block), lp.lds_bytes, stream, p);
  }
  else if (p.persistent && p.svc)
    hipLaunchKernelGGL((tova_step_kernel<T, D, G, true, false, true>), dim3(lp.grid), dim3(lp.block), lp.lds_bytes, stream, p);
  else if (p.persistent)
    hipLaunchKernelGGL((tova_step_kernel<T, D, G, true>), dim3(lp.grid), dim3(lp.block), lp.lds_bytes, stream, p);
  else
    hipLaunchKernelGGL((tova_step_kernel<T, D, G, false>), dim3(lp.grid), dim3(lp.block), lp.lds_bytes, stream, p);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_g(int G, const StepParams& p, const LaunchPlan& lp, hipStream_t s) {
  switch (G) {
    case 1: return launch_one<T, D, 1>(p, lp, s);
    case 2: return launch_one<T, D, 2>(p, lp, s);
    case 4: return launch_one<T, D, 4>(p, lp, s);
    case 8: return launch_one<T, D, 8>(p, lp, s);
    default: return hipErrorInvalidValue;
  }
}

template <typename T>
hipError_t launch_d(int D, int G, const StepParams& p, const LaunchPlan& lp, hipStream_t s) {
  switch (D) {
    case 32: return launch_g<T, 32>(G, p, lp, s);
    case 64: return launch_g<T, 64>(G, p, lp, s);
    case 128: return launch_g<T, 128>(G, p, lp, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t launch_step(int dtype_is_bf16, int D, int G, const StepParams& p, const LaunchPlan& lp,
                       hipStream_t stream) {
  return dtype_is_bf16 ? launch_d<bf16_t>(D, G, p, lp, stream) : launch_d<float>(D, G, p, lp, stream);
}

int resident_blocks(int dtype_is_bf16, int D, int G, int block, int lds_bytes, int unit_mode) {
  return dtype_is_bf16 ? resident_blocks_d<bf16_t>(D, G, block, lds_bytes, unit_mode)
                       : resident_blocks_d<float>(D, G, block, lds_bytes, unit_mode);
}

int device_cus() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  return cus;
}

__global__ void tova_add_i32_kernel(int32_t* dst, int32_t add) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *dst += add;
}

hipError_t launch_add_i32(int32_t* dst, int32_t add, hipStream_t stream) {
  hipLaunchKernelGGL(tova_add_i32_kernel, dim3(1), dim3(64), 0, stream, dst, add);
  return hipGetLastError();
}

int stream_is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
    (void)hipGetLastError();  // (the legacy default stream cannot be asked while another one captures)
    return 0;
  }
  return st == hipStreamCaptureStatusActive;
}

hipError_t read_i32_sync(const int32_t* dev, hipStream_t stream, int32_t* host) {
  hipError_t e = hipStreamSynchronize(stream);
  if (e != hipSuccess) return e;
  return hipMemcpy(host, dev, sizeof(int32_t), hipMemcpyDeviceToHost);
}

hipError_t launch_fill_i32(int32_t* dst, int32_t value, size_t count, hipStream_t stream) {
  if (count == 0) return hipSuccess;
  size_t blocks = (count + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(tova_fill_i32_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, dst, value, count);
  return hipGetLastError();
}

}  // namespace tova
