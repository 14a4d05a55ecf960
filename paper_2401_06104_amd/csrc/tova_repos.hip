// TOVA decode steps with re-assigned positions (gfx950 / MI355X), for decoding beyond the
// training length (Sec. 7.2, "Extrapolation with TOVA").
//
// The multi-state keeps the keys WITHOUT positional encoding.  Before each attention the positions
// of everything the query attends over are re-assigned: between two candidates that are adjacent
// in token order a gap of g tokens counts as ln(ln(g)), gaps of at most 10 as they are; the rotary
// embedding is then applied at those positions, and the rest is the plain TOVA step (softmax, PV,
// head-mean scores, argmin with the lowest index on ties, in-place overwrite: Sec. 4, App. B).
//
// Only differences of positions reach a logit: with D_j the compressed distance from candidate j
// to the incoming token (the sum of the compressed gaps between them),
//     (R(p_q) q) . (R(p_j) k_j) = q . (R(-D_j) k_j),
// R(p) being the rotation of the pair (x_i, x_{i + d/2}) by p * base^(-2i/d).  So the query and
// the incoming key stay as they are and every cached row is turned back by its distance while it
// streams through the logit pass.
//
// A workgroup owns a (layer, sequence) unit, as in the workgroup-per-unit form of the step kernel:
//   0. positions: the unit's slot -> token map (k integers) gives, by counting, every candidate's
//      rank in token order; the compressed gaps are summed from the newest candidate backwards
//      (fp64: distances reach tens of thousands, and the angle D * theta_i is needed to 1e-7
//      of a turn); D_j lands in LDS, one double per candidate; a workgroup that stays with its unit
//      keeps order and ranks in LDS and updates them per step (one candidate leaves, one arrives)
//      instead of reading the map and counting again;
//   1. per KV head: logit pass over the K rows -- a lane holds a 16-byte piece of the first half
//      of a row and the matching piece of the second half, i.e. both elements of VEC rotary pairs;
//      the angle's fraction of a turn is taken in fp64, sine and cosine in fp32 (hardware sin/cos
//      for bf16 data, whose tolerance they meet; the library's sincospi for fp32 data); the rotated
//      row is dotted with the G query heads of the KV head;
//   2. softmax statistics, head-summed scores into an LDS row, PV pass over the V rows (the shared
//      pass of the other kernels: values carry no positions), outputs;
//   3. argmin over the LDS row, the incoming un-rotated key / value rows into the victim's slot.
// Nothing leaves the workgroup except its results, so the grid may have any size, the steps of a
// call run inside one launch, and the fill phase (fewer than k rows cached) runs through the same
// code with the candidates it has.
//
// Few units (the paper runs this experiment at batch 1: 32 layers = 32 units): the KV heads of a unit
// are dealt to P workgroups (parts), cache full, every workgroup of the grid resident.  A head's
// softmax is complete inside its part, so what the parts exchange per step is one row of partial
// head sums each ((k + 1) floats, written past the caches) and an arrival count; the part that
// arrives last adds the rows in part order, picks the victim, updates the map and publishes
// (victim, token index) in the unit's 64-bit state word.  Every part finds the positions itself
// (the map is small), waits -- bounded, with the cache's error flag as the way out -- for that
// word before the unit's next step, and stores the incoming rows of its own KV heads, so a cached
// row is only ever written and read by the same workgroup.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "tova_internal.h"

#include "tova_device.h"

namespace tova {
namespace {

constexpr int kGapKept = 10;  // gaps of up to this many tokens keep their length (Sec. 7.2)

__device__ __forceinline__ double compressed_gap(int g) { return g <= kGapKept ? (double)g : log(log((double)g)); }

template <typename T, int D, int G>
__global__ __launch_bounds__(512, 2) void tova_repos_kernel(const ReposParams p) {
  using E = Elem<T>;
  using Ge = Geo<T, D, G>;
  constexpr int VEC = Ge::VEC, LV = Ge::LV, UV = Ge::UV;
  constexpr int CH = D / VEC;       // 16-byte pieces per row
  constexpr int HC = CH / 2;        // ... per half row = lanes per row in the logit pass
  constexpr int LR = HC, RW = 64 / LR;
  constexpr int U = (G >= 8) ? 2 : 4;  // rows per lane and register buffer (two buffers in flight)
  constexpr int ROW16 = CH;
  static_assert(CH >= 2 && (HC & (HC - 1)) == 0, "a lane holds both halves of its rotary pairs");

  extern __shared__ float4 smem4[];
  float* small = reinterpret_cast<float*>(smem4);  // kSmallFloats
  float* big = small + kSmallFloats;
  const int nt = blockDim.x;
  const int nw = nt >> 6;
  const int k = p.k;
  const int kp = (k + 1 + 3) & ~3;
  float* e_lds = big;                    // [n + 1][G] logits, then exp values; then the PV reduction area
  float* s_lds = big + p.e_floats;       // [k + 1] head-summed scores
  double* dslot = reinterpret_cast<double*>(s_lds + kp);  // [k + 1] compressed distance to the incoming token, by slot
  // position scratch, over the (still unused) logit area
  double* drank = reinterpret_cast<double*>(big);  // [k + 1] the same by rank in token order
  int* tokS = reinterpret_cast<int*>(big + 2 * kp);  // [k + 1] token index by slot; entry n: the incoming token
  int* srt = tokS + kp;                              // [k + 1] token indices in ascending order
  int* rnk = srt + kp;                               // [k + 1] rank by slot
  const float scale2 = p.scale * kLog2e;
  // the rotary frequencies base^(-2i/d), in turns per unit of position, once per workgroup
  double* turns_lds = dslot + kp;  // [d / 2]
  if (p.persist) {
    // room for the order and the ranks outside the logit area: a workgroup that stays with its unit
    // then keeps them from step to step (one candidate leaves and one arrives per step) instead of
    // reading the map and counting again
    srt = reinterpret_cast<int*>(turns_lds + D / 2);
    rnk = srt + kp;
  }
  const bool stays = p.persist && (int)gridDim.x >= p.units * p.parts;  // one item per workgroup
  int last_vic = k;  // what the unit's previous step removed (block-uniform)
  for (int i = threadIdx.x; i < D / 2; i += nt) turns_lds[i] = exp2((double)(-2 * i) / (double)D * p.log2_base) * 0.15915494309189535;  // / (2 pi)
  __syncthreads();

  const int P = p.parts;          // workgroups per unit (1: a workgroup owns the unit)
  const int HP = p.H_kv / P;      // KV heads per part
  int* flag_lds = reinterpret_cast<int*>(small + 480);
  // (with parts, an extra pass stores the last step's rows)
  for (int it = 0; it < p.n_iter + (P > 1 ? 1 : 0); ++it) {
  for (int item = blockIdx.x; item < p.units * P; item += gridDim.x) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // (opaque per pass: keeps the lane arithmetic of the body out of the loops' live ranges)
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int unit = item / P, part = item - unit * P;
  const int n = min(p.n0 + it, k);  // rows cached before this step
  const bool full = (n == k);
  const int nc = n + 1;             // candidates: the cached rows and the incoming token (index n)
  const int tok = p.t + it;
  const int pair0 = unit * p.H_kv;
  const int kv0 = part * HP;        // this workgroup's KV heads: kv0 .. kv0 + HP - 1

  if (P > 1 && it > 0) {
    // Wait (bounded) for the victim of the unit's previous step, then put that step's incoming rows
    // of this part's KV heads into the freed slot.  If the wait runs out -- it cannot while all
    // workgroups are resident, which the host checks -- the workgroup raises the cache's error flag
    // and leaves; every other one sees the flag in its own wait and leaves too.
    if (tid == 0) {
      unsigned long long w = 0;
      int ok = 0;
      for (int spin = 0;; ++spin) {
        w = ld_agent_u64(p.pstate + unit);
        if ((int)(uint32_t)w == tok) {
          ok = 1;
          break;
        }
        if (spin >= p.spin || ld_agent_i(p.error_flag) != 0) break;
        __builtin_amdgcn_s_sleep(4);
      }
      if (!ok) st_agent_i(p.error_flag, 1);
      flag_lds[2] = ok;
      flag_lds[3] = (int)(w >> 32);
    }
    __syncthreads();
    if (flag_lds[2] == 0) return;  // block-uniform
    const int vic = flag_lds[3];
    last_vic = vic;
    if (vic < k) {  // (vic == k: the incoming token was dropped)
      const T* kprev = reinterpret_cast<const T*>(p.k_new) + (size_t)(it - 1) * p.kv_stride + (size_t)(pair0 + kv0) * D;
      const T* vprev = reinterpret_cast<const T*>(p.v_new) + (size_t)(it - 1) * p.kv_stride + (size_t)(pair0 + kv0) * D;
      T* Ku = reinterpret_cast<T*>(p.K) + ((size_t)(pair0 + kv0) * k + vic) * D;
      T* Vu = reinterpret_cast<T*>(p.V) + ((size_t)(pair0 + kv0) * k + vic) * D;
      for (int x = tid; x < HP * ROW16; x += nt) {  // rows of consecutive KV heads are contiguous in k_new
        const int h = x / ROW16, c = x - h * ROW16;
        reinterpret_cast<V16*>(Ku + (size_t)h * k * D)[c] = reinterpret_cast<const V16*>(kprev)[x];
        reinterpret_cast<V16*>(Vu + (size_t)h * k * D)[c] = reinterpret_cast<const V16*>(vprev)[x];
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();  // the rows are in place for this workgroup's passes
    if (it == p.n_iter) continue;
  }

  // ---------------- phase 0: compressed distances (Sec. 7.2) ----------------
  if (stays && it > 0) {
    // the order and the ranks of the previous step are still here
    if (min(p.n0 + it - 1, k) == k && last_vic < k) {
      // that step removed the candidate in slot last_vic, and its incoming token (rank k then) now
      // sits in that slot as the newest cached one
      const int rv = rnk[last_vic];
      __syncthreads();  // everyone has it before the ranks change
      int* tmp = tokS;  // (free)
      for (int r = tid; r < n; r += nt) tmp[r] = (r < rv) ? srt[r] : srt[r + 1];
      for (int j = tid; j < n; j += nt) {
        const int rj = rnk[j];
        rnk[j] = (j == last_vic) ? n - 1 : rj - (rj > rv ? 1 : 0);
      }
      __syncthreads();
      for (int r = tid; r < n; r += nt) srt[r] = tmp[r];
    }
    // (a step that only appended, or dropped its own token, leaves order and ranks as they are)
  } else {
    // (entries from n on hold the largest integer, so that whole 16-byte pieces can be compared)
    for (int j = tid; j < kp; j += nt) tokS[j] = (j < n) ? ld_agent_i(p.slot_token + (size_t)unit * k + j) : 0x7fffffff;
    __syncthreads();
    // Rank in token order by counting (token indices are distinct), up to four cached candidates per
    // thread and trip, four map entries per read (the same address for every lane: a broadcast).  The
    // incoming token is the newest: rank n.
    const int n4 = (n + 3) >> 2;
    auto count_ranks = [&](auto jb_tag) {
      constexpr int JB = decltype(jb_tag)::value;  // candidates per thread and trip
      for (int j0 = tid; j0 < n; j0 += JB * nt) {
        int my[JB], r[JB];
  #pragma unroll
        for (int b = 0; b < JB; ++b) {
          my[b] = tokS[min(j0 + b * nt, kp - 1)];
          r[b] = 0;
        }
  #pragma unroll 4
        for (int i4 = 0; i4 < n4; ++i4) {
          const int4 t4 = reinterpret_cast<const int4*>(tokS)[i4];
  #pragma unroll
          for (int b = 0; b < JB; ++b)
            r[b] += ((t4.x < my[b]) ? 1 : 0) + ((t4.y < my[b]) ? 1 : 0) + ((t4.z < my[b]) ? 1 : 0) + ((t4.w < my[b]) ? 1 : 0);
        }
  #pragma unroll
        for (int b = 0; b < JB; ++b) {
          const int j = j0 + b * nt;
          if (j < n) {
            srt[r[b]] = my[b];
            rnk[j] = r[b];
          }
        }
      }
    };
    if (n <= nt)
      count_ranks(std::integral_constant<int, 1>{});
    else if (n <= 2 * nt)
      count_ranks(std::integral_constant<int, 2>{});
    else
      count_ranks(std::integral_constant<int, 4>{});
  }
  if (tid == 0) {
    srt[n] = tok;
    rnk[n] = n;
  }
  __syncthreads();
  // drank[r] = sum of the compressed gaps between rank r and the newest candidate (rank n, the
  // incoming token).  Thread s sums the gaps of ranks [s * seg, (s + 1) * seg) from the high end,
  // wave 0 turns the segment totals into offsets, every thread adds its segment's offset.
  double* totals = dslot;  // (free until the distances are final)
  const int seg = (n + nt - 1) / nt;
  const int nseg = seg ? (n + seg - 1) / seg : 0;
  {
    const int lo = tid * seg, hi = min(lo + seg, n);
    double run = 0.0;
    for (int r = hi - 1; r >= lo; --r) {
      run += compressed_gap(srt[r + 1] - srt[r]);
      drank[r] = run;
    }
    if (tid < nseg) totals[tid] = run;
    if (tid == 0) drank[n] = 0.0;
  }
  __syncthreads();
  if (wave == 0 && nseg > 0) {
    const int per = (nseg + 63) / 64;
    const int lo = min(lane * per, nseg), hi = min(lo + per, nseg);
    double tot = 0.0;
    for (int s = lo; s < hi; ++s) tot += totals[s];
    double incl = tot;  // after the loop: sum of the totals of this lane and of all later lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double y = __shfl_down(incl, o);
      if (lane + o < 64) incl += y;
    }
    double off = incl - tot;
    for (int s = hi - 1; s >= lo; --s) {
      const double t = totals[s];
      totals[s] = off;
      off += t;
    }
  }
  __syncthreads();
  double seg_off = (tid < nseg) ? totals[tid] : 0.0;
  __syncthreads();  // the totals are read: their memory becomes the distances by slot
  {
    const int lo = tid * seg, hi = min(lo + seg, n);
    for (int r = lo; r < hi; ++r) drank[r] += seg_off;
  }
  __syncthreads();
  for (int j = tid; j < nc; j += nt) dslot[j] = drank[rnk[j]];
  __syncthreads();  // the distances are in place; the position scratch is free for the logits

  // this lane's rotary frequencies, in turns per unit of position
  const int lr = lane % LR, rw = lane / LR;
  double turns[VEC];
#pragma unroll
  for (int u = 0; u < VEC; ++u) turns[u] = turns_lds[lr * VEC + u];

  // ---------------- the unit's victim and state update (Sec. 4; App. B) ----------------
  // (defined here, called below: by a workgroup that owns its unit after the last KV head; with
  // parts, between the last KV head's softmax and its PV pass, so that the summing part's work
  // and the victim's way to the other parts overlap everybody's last PV pass)
  auto victim_and_state = [&]() {
  bool decide = true;  // this workgroup picks the unit's victim
  if (P > 1) {
    // hand the partial head sums over; the part that arrives last adds them up
    float* sgp = p.sg + (size_t)unit * P * kp;
    for (int i = tid; i < nc; i += nt) st_agent(sgp + (size_t)part * kp + i, s_lds[i]);
    const int prev = arrive(p.cnt_unit + unit, 1, flag_lds, tid);
    decide = (prev + 1 == P);
    if (decide) {
      reset_counter(p.cnt_unit + unit, tid);
      for (int j = tid; j < nc; j += nt) {
        float a = 0.f;
        constexpr int PB = 8;  // parts whose loads are issued together
        for (int q0 = 0; q0 < P; q0 += PB) {
          float v[PB];
#pragma unroll
          for (int u = 0; u < PB; ++u) v[u] = (q0 + u < P) ? ld_agent(sgp + (size_t)(q0 + u) * kp + j) : 0.f;
#pragma unroll
          for (int u = 0; u < PB; ++u) a += v[u];  // (part order)
        }
        s_lds[j] = a;  // (entry j is this thread's own)
      }
    }
  }
  int slot = n;  // below capacity the new rows take slot n
  if (full && decide) {
    // argmin of the head sums (the factor 1/H does not move it); a thread takes its candidates in
    // ascending order with a strict <, so the lowest index wins ties; candidates below n_pinned
    // stay out (TOVA+i, App. A)
    float best = INFINITY;
    int bj = 0x7fffffff;
    for (int j = tid; j <= k; j += nt) {
      const float sj = s_lds[j];
      if (j >= p.n_pinned && sj < best) {
        best = sj;
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
    float* bv = small + 256;
    int* bi = reinterpret_cast<int*>(small + 256 + kMaxWaves);
    if (lane == 0) {
      bv[wave] = best;
      bi[wave] = bj;
    }
    __syncthreads();
    best = bv[0];
    bj = bi[0];
    for (int w = 1; w < nw; ++w) {
      const float ob = bv[w];
      const int oj = bi[w];
      if (ob < best || (ob == best && oj < bj)) {
        best = ob;
        bj = oj;
      }
    }
    if (bj > k) bj = k;  // only reachable with non-finite scores
    slot = bj;
  }
  if (P == 1) last_vic = slot;
  if (P == 1 && slot < k) {  // (slot == k: the incoming token itself was dropped)
    const T* kn = reinterpret_cast<const T*>(p.k_new) + (size_t)it * p.kv_stride + (size_t)pair0 * D;
    const T* vn = reinterpret_cast<const T*>(p.v_new) + (size_t)it * p.kv_stride + (size_t)pair0 * D;
    T* Ku = reinterpret_cast<T*>(p.K) + ((size_t)pair0 * k + slot) * D;
    T* Vu = reinterpret_cast<T*>(p.V) + ((size_t)pair0 * k + slot) * D;
    for (int x = tid; x < p.H_kv * ROW16; x += nt) {  // rows of consecutive KV heads are contiguous in k_new
      const int h = x / ROW16, c = x - h * ROW16;
      reinterpret_cast<V16*>(Ku + (size_t)h * k * D)[c] = reinterpret_cast<const V16*>(kn)[x];
      reinterpret_cast<V16*>(Vu + (size_t)h * k * D)[c] = reinterpret_cast<const V16*>(vn)[x];
    }
  }
  if (tid == 0 && decide) {
    int32_t* const evp = p.evicted ? p.evicted + (size_t)it * p.units : nullptr;
    if (evp) st_agent_i(evp + unit, full ? slot : -1);
    if (slot < k) st_agent_i(p.slot_token + (size_t)unit * k + slot, tok);  // (read back, past the caches, in the next step)
    st_agent_i(p.occupancy + unit, full ? k : n + 1);
    if (P > 1) {
      // publish the victim; every part stores the rows of its own KV heads when it comes back to the
      // unit (the counter's reset and the map entry must have landed first)
      __builtin_amdgcn_s_waitcnt(0);
      st_agent_u64(p.pstate + unit, ((unsigned long long)(uint32_t)slot << 32) | (uint32_t)(tok + 1));
    }
  }
  };

  for (int kvh = kv0; kvh < kv0 + HP; ++kvh) {
  const int pair = pair0 + kvh;
  const T* Kb = reinterpret_cast<const T*>(p.K) + (size_t)pair * k * D;
  const T* Vb = reinterpret_cast<const T*>(p.V) + (size_t)pair * k * D;
  const T* knew = reinterpret_cast<const T*>(p.k_new) + (size_t)it * p.kv_stride + (size_t)pair * D;
  const T* vnew = reinterpret_cast<const T*>(p.v_new) + (size_t)it * p.kv_stride + (size_t)pair * D;
  const T* qb = reinterpret_cast<const T*>(p.q) + (size_t)it * p.q_stride + ((size_t)unit * p.H + (size_t)kvh * G) * D;
  const bool new_here = (wave == nw - 1);  // wave-uniform: the block's last wave takes the incoming token

  // ---------------- phase 1: logits of the re-positioned keys ----------------
  float m[G], Z[G];
  {
    float qa[G][VEC], qc[G][VEC];  // the query heads' elements of this lane's pairs: first half, second half
#pragma unroll
    for (int g = 0; g < G; ++g) {
      E::unpack(reinterpret_cast<const V16*>(qb + g * D)[lr], qa[g]);
      E::unpack(reinterpret_cast<const V16*>(qb + g * D)[lr + HC], qc[g]);
      m[g] = -INFINITY;
    }
    auto load_tile = [&](V16(&a)[U], V16(&c)[U], int base) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = base + u * RW + rw;
        a[u] = V16{{0u, 0u, 0u, 0u}};
        c[u] = V16{{0u, 0u, 0u, 0u}};
        if (j < n) {
          a[u] = reinterpret_cast<const V16*>(Kb + (size_t)j * D)[lr];
          c[u] = reinterpret_cast<const V16*>(Kb + (size_t)j * D)[lr + HC];
        }
      }
    };
    // logits of one row held as (first-half piece, second-half piece), dist = its distance; every
    // lane of the row's group calls it; the group's first lane stores
    auto row_logits = [&](const V16& a, const V16& c, double dist, bool rotate, int j, bool live) {
      float x[VEC], y[VEC];
      E::unpack(a, x);
      E::unpack(c, y);
      if (rotate) {
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
          const double rev = dist * turns[u];
          const float f = (float)__builtin_amdgcn_fract(rev);  // the angle as a fraction of a turn, in [0, 1]
          float sn, cs;
          if constexpr (sizeof(T) == 2) {
            sn = __builtin_amdgcn_sinf(f);  // (take turns, not radians)
            cs = __builtin_amdgcn_cosf(f);
          } else {
            sincospif(2.0f * f, &sn, &cs);
          }
          const float xr = fmaf(x[u], cs, y[u] * sn);   // the pair turned back by the angle
          const float yr = fmaf(y[u], cs, -x[u] * sn);
          x[u] = xr;
          y[u] = yr;
        }
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float l = 0.f;
#pragma unroll
        for (int u = 0; u < VEC; ++u) l = fmaf(qa[g][u], x[u], fmaf(qc[g][u], y[u], l));
        l = group_sum<LR>(l) * scale2;
        if (live) {
          m[g] = fmaxf(m[g], l);
          if (lr == 0) e_lds[j * G + g] = l;
        }
      }
    };
    auto compute_tile = [&](const V16(&a)[U], const V16(&c)[U], int base) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = base + u * RW + rw;
        const bool live = (j < n);
        row_logits(a[u], c[u], dslot[live ? j : n], true, j, live);
      }
    };
    constexpr int TILE = RW * U;
    const int stride = nw * TILE;
    V16 a0[U], c0[U], a1[U], c1[U];
    int base = wave * TILE;
    load_tile(a0, c0, base);
    while (base < n) {  // wave-uniform
      load_tile(a1, c1, base + stride);
      compute_tile(a0, c0, base);
      base += stride;
      if (base >= n) break;
      load_tile(a0, c0, base + stride);
      compute_tile(a1, c1, base);
      base += stride;
    }
    if (new_here) {  // the incoming token: distance zero, nothing to turn
      const V16 a = reinterpret_cast<const V16*>(knew)[lr];
      const V16 c = reinterpret_cast<const V16*>(knew)[lr + HC];
      row_logits(a, c, 0.0, false, n, rw == 0);
    }
  }

  // The first PV tile is requested now, so that the V stream is in flight during the softmax barriers.
  const int lv = lane % LV, rv = lane / LV;
  constexpr bool PVM = PvMfma<T, D, G>::OK;  // bf16, d = 128, 8 heads per KV head: PV on the matrix cores
  V16 vA[PVM ? 8 : UV];
  if constexpr (PVM)
    pv_mfma_load<T, D>(vA, Vb, wave * PvMfma<T, D, G>::ROWS, n, lane);
  else
    pv_first_tile<T, D, G>(vA, Vb, n, lane, wave);

  // ---------------- phase 2: softmax statistics, head-summed scores ----------------
  block_reduce<G, true>(m, small, lane, wave, nw);  // (its barrier also makes the logits visible)
#pragma unroll
  for (int g = 0; g < G; ++g) Z[g] = 0.f;
  for (int i = tid; i < nc; i += nt) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float e = __builtin_amdgcn_exp2f(e_lds[i * G + g] - m[g]);
      e_lds[i * G + g] = e;
      Z[g] += e;
    }
  }
  block_reduce<G, false>(Z, small + kMaxWaves * G, lane, wave, nw);  // (... and completes the exp values)
  if (full) {
    float rz[G];
#pragma unroll
    for (int g = 0; g < G; ++g) rz[g] = 1.0f / Z[g];
    for (int i = tid; i < nc; i += nt) {  // (entry i is always this thread's; KV heads in order)
      float a = 0.f;
#pragma unroll
      for (int g = 0; g < G; ++g) a = fmaf(e_lds[i * G + g], rz[g], a);
      s_lds[i] = (kvh == kv0) ? a : s_lds[i] + a;
    }
  }

  if (P > 1 && kvh == kv0 + HP - 1) victim_and_state();  // (block-uniform; the exp values and the first V tile stay as they are)

  // ---------------- phase 3: PV (values carry no positions) ----------------
  float* red = big;  // [nw][G * D]
  if constexpr (PVM) {
    f32x4_t pacc[8];
    pv_pass_mfma<T, D, G>(Vb, n, e_lds, G, 0, lane, wave, nw, vA, pacc);
    pv_mfma_finish<T, D, G>(pacc, n, 1, new_here, [&](int) { return vnew; }, e_lds, G, 0, lane, wave, red);
  } else {
    float acc[G][VEC];
    pv_pass<T, D, G>(Vb, n, 1, new_here, [&](int) { return vnew; }, e_lds, G, 0, lane, wave, nw, vA, acc);
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[g][v] = column_sum<LV>(acc[g][v]);
    __syncthreads();   // everyone is done reading the exp values; the reduction area reuses them
    if (rv == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int v = 0; v < VEC; ++v) red[(wave * G + g) * D + lv * VEC + v] = acc[g][v];
    }
  }
  __syncthreads();
  T* outb = reinterpret_cast<T*>(p.out) + (size_t)it * p.q_stride + ((size_t)unit * p.H + (size_t)kvh * G) * D;
  for (int x = tid; x < G * D; x += nt) {
    float a = red[x];
    for (int w = 1; w < nw; ++w) a += red[w * G * D + x];
    float zg = Z[0];
#pragma unroll
    for (int g = 1; g < G; ++g) zg = (x / D == g) ? Z[g] : zg;
    E::store(outb + x, a / zg);
  }
  __syncthreads();  // the reduction area is free for the next KV head
  }  // KV heads

  if (P == 1) victim_and_state();
  // the rows and the map entry must have landed before the block reads them in the unit's next step
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();  // LDS is free for the block's next unit
  }  // units of this block
  }  // steps
}

template <typename T, int D, int G>
hipError_t launch_repos_one(const ReposParams& p, const LaunchPlan& lp, hipStream_t stream) {
  {  // more dynamic LDS than the default limit: say so, once per size and device
    const hipError_t e = ensure_dynamic_lds<&tova_repos_kernel<T, D, G>>(lp.lds_bytes);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((tova_repos_kernel<T, D, G>), dim3(lp.grid), dim3(lp.block), lp.lds_bytes, stream, p);
  return hipGetLastError();
}
template <typename T, int D>
hipError_t launch_repos_g(int G, const ReposParams& p, const LaunchPlan& lp, hipStream_t s) {
  switch (G) {
    case 1: return launch_repos_one<T, D, 1>(p, lp, s);
    case 2: return launch_repos_one<T, D, 2>(p, lp, s);
    case 4: return launch_repos_one<T, D, 4>(p, lp, s);
    case 8: return launch_repos_one<T, D, 8>(p, lp, s);
    default: return hipErrorInvalidValue;
  }
}
template <typename T>
hipError_t launch_repos_d(int D, int G, const ReposParams& p, const LaunchPlan& lp, hipStream_t s) {
  switch (D) {
    case 32: return launch_repos_g<T, 32>(G, p, lp, s);
    case 64: return launch_repos_g<T, 64>(G, p, lp, s);
    case 128: return launch_repos_g<T, 128>(G, p, lp, s);
    default: return hipErrorInvalidValue;
  }
}

template <typename T, int D>
int repos_resident_g(int G, int block, int lds) {
  int per_cu = 0;
  hipError_t e = hipErrorInvalidValue;
  switch (G) {
    case 1: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tova_repos_kernel<T, D, 1>, block, (size_t)lds); break;
    case 2: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tova_repos_kernel<T, D, 2>, block, (size_t)lds); break;
    case 4: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tova_repos_kernel<T, D, 4>, block, (size_t)lds); break;
    case 8: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tova_repos_kernel<T, D, 8>, block, (size_t)lds); break;
    default: break;
  }
  return e == hipSuccess ? per_cu : 0;
}
template <typename T>
int repos_resident_d(int D, int G, int block, int lds) {
  switch (D) {
    case 32: return repos_resident_g<T, 32>(G, block, lds);
    case 64: return repos_resident_g<T, 64>(G, block, lds);
    case 128: return repos_resident_g<T, 128>(G, block, lds);
    default: return 0;
  }
}

}  // namespace

int repos_resident_blocks(int dtype_is_bf16, int D, int G, int block, int lds_bytes) {
  if (lds_bytes > 64 * 1024) return 0;  // (the split form is only planned with several workgroups per CU)
  const int per_cu = dtype_is_bf16 ? repos_resident_d<bf16_t>(D, G, block, lds_bytes) : repos_resident_d<float>(D, G, block, lds_bytes);
  return per_cu * device_cus();
}

hipError_t launch_repos(int dtype_is_bf16, int D, int G, const ReposParams& p, const LaunchPlan& lp, hipStream_t stream) {
  return dtype_is_bf16 ? launch_repos_d<bf16_t>(D, G, p, lp, stream) : launch_repos_d<float>(D, G, p, lp, stream);
}

}  // namespace tova
