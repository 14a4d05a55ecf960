// Multi-token steps for gfx950 (MI355X): C consecutive tokens of a prompt per pass over the cache.
//
// What it computes is fixed by the single-token step (Sec. 3.2, Sec. 4, App. B Alg. 1): token
// t + i of a group attends over what the bounded multi-state holds after tokens t .. t + i - 1
// have been processed (plus itself), and the policy then removes one row -- the mask formulation
// of the paper's language-modelling runs, where all positions of a text are scored at once with a
// mask derived row by row from the layer's own attention weights.  A prompt is known in advance,
// so the queries of C tokens can share one stream of K and one of V; what one token changes for
// the next is small and is applied as a correction:
//
//   candidates        the k cached rows and the group's own C tokens (candidate k + i); token i
//                     may see candidate k + i' only for i' <= i
//   pass A            per KV head, K and V streamed ONCE for all C tokens: logits, maxima m and
//                     sums Z over all causally allowed candidates, the unmasked PV sums U, and the
//                     "tentative" scores T_i[c] = sum_heads w_i[c] / Z_i   (w = 2^(l - m))
//   resolution        token by token (i = 0 .. C-1), with E_i = candidates removed by tokens < i:
//                     Z'_i = Z_i - sum_{e in E_i} w_i[e]          (a few dot products)
//                     exact score s_i[c] = sum_heads w_i[c] / Z'_i lies in [T_i[c], T_i[c] f_max]
//                     with f = Z / Z' >= 1 per head, so only candidates whose lower bound does not
//                     exceed the smallest upper bound can be the argmin; their scores are
//                     recomputed exactly from their K rows and the argmin is taken among them
//                     (lowest slot index on ties, the token itself last)
//                     out_i = (U_i - sum_{e in E_i} w_i[e] V[e]) / Z'_i
//   guard             Z' = Z - delta and U' = U - ... lose precision when what was removed carries most
//                     of a head's weight for this token (relative error ~ eps * Z / Z').  If for any
//                     head less than kMinKept of Z is left (or nothing: Z' <= 0), the token is not
//                     corrected but computed from scratch over the candidates that are still there
//                     -- the single-token step (logit pass, softmax, PV, head-summed scores, argmin)
//                     inside this kernel; the group's other tokens go on as before.
//   commit            tokens that still hold a slot at the end are stored there.
//
// While the multi-state still has room (App. B: nothing is removed while num_kv <= cache_max_size)
// a group is plain causal attention over the cached rows and its own tokens: pass A, out = U / Z,
// and the tokens take the next free slots.
//
// One workgroup per (layer, sequence) unit, KV heads in turn (the form of the single-token kernel
// for many units): nothing is exchanged between workgroups.  One chunk per KV head.
//
// Few units (the paper scores one text at a time: 32 layers = 32 units): the KV heads of a unit are
// dealt to P workgroups ("parts"), all resident.  Pass A is independent per KV head, so every part
// runs it for its own heads and hands over, through device memory, its partial tentative-score rows,
// its heads' softmax statistics and unmasked PV sums; the part that arrives last adds the rows in
// part order and resolves the group for the whole unit exactly as above, then publishes where every
// token of the group ended up (its slot, or none) and a per-unit group counter.  Every part waits --
// bounded, with the cache's error flag as the way out -- for that counter before its next group and
// stores the rows of its own KV heads itself, written through; the resolving part reads the few rows
// it needs of other parts' heads past the caches.  While the multi-state still has room nothing is
// exchanged at all: every part finishes its own heads.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tova_internal.h"

#include "tova_device.h"

namespace tova {
namespace {

template <typename T>
__device__ __forceinline__ float elem_f32(const T* p, int idx);
template <>
__device__ __forceinline__ float elem_f32<float>(const float* p, int idx) {
  return p[idx];
}
template <>
__device__ __forceinline__ float elem_f32<bf16_t>(const bf16_t* p, int idx) {
  return __uint_as_float((uint32_t)p[idx].x << 16);
}

// element idx of a row that another workgroup of this launch may have written (written through): read
// past the caches, as the aligned 32-bit word that holds it
template <typename T>
__device__ __forceinline__ float elem_f32_agent(const T* p, int idx);
template <>
__device__ __forceinline__ float elem_f32_agent<float>(const float* p, int idx) {
  return ld_agent(p + idx);
}
template <>
__device__ __forceinline__ float elem_f32_agent<bf16_t>(const bf16_t* p, int idx) {
  const uint32_t w = (uint32_t)ld_agent_i(reinterpret_cast<const int32_t*>(p) + (idx >> 1));
  return __uint_as_float((idx & 1) ? (w & 0xffff0000u) : (w << 16));
}
// a 16-byte piece written through (two 64-bit stores)
__device__ __forceinline__ void st_agent_v16(V16* dst, const V16& v) {
  unsigned long long* d = reinterpret_cast<unsigned long long*>(dst);
  st_agent_u64(d, ((unsigned long long)v.w[1] << 32) | v.w[0]);
  st_agent_u64(d + 1, ((unsigned long long)v.w[3] << 32) | v.w[2]);
}

constexpr float kBoundSlack = 1e-4f;  // rounding of the streamed sums against the recomputed ones: ~1e-6
// The corrected sum Z' = Z - (weights of the removed candidates) carries the rounding of Z (a block
// sum of up to k + C fp32 terms: a few 1e-7 relative) magnified by Z / Z'.  With at least an eighth
// of Z left the corrected sums, outputs and scores stay within ~4e-6 relative, inside the 1e-5 bar
// of fp32 data; below that the token is computed from scratch.
constexpr float kMinKept = 0.125f;

template <typename T, int D, int G, int C>
__global__ __launch_bounds__(512, (G * C >= 8 || PvMfma<T, D, G * C>::OK) ? 3 : 4) void tova_prefill_kernel(const PrefillParams p) {
  using E = Elem<T>;
  constexpr int GE = G * C;  // (token, query head) combinations served by one streamed row
  using Ge = Geo<T, D, GE>;
  constexpr int VEC = Ge::VEC, LV = Ge::LV, UV = Ge::UV;
  constexpr int ROW16 = D * (int)sizeof(T) / 16;
  constexpr int EPL = (D + 63) / 64;  // elements of a row per lane in the exact recomputation
  static_assert(GE <= 8 && C <= 8, "register budget of the vector passes");

  extern __shared__ float4 smem4[];
  float* small = reinterpret_cast<float*>(smem4);
  float* big = small + kSmallFloats;
  const int nt = blockDim.x;
  const int nw = nt >> 6;
  const int k = p.k, H = p.H, ncp = p.ncp;
  float* e_lds = big;               // [NC][GE] logits, then exp values; reduction area; resolution buffers
  float* t_lds = big + p.e_floats;  // [C][ncp] tentative scores
  float* mst = t_lds + C * ncp;     // [H][C] maxima (log2 domain)
  float* zst = mst + H * C;         // [H][C] sums over all causally allowed candidates
  float* zcs = zst + H * C;         // [H]    corrected sums of the token being resolved
  float* wev = zcs + H;             // [C][H] that token's weights of the candidates removed before it
  int* pos = reinterpret_cast<int*>(small + 384);  // [C] slot a group token holds (-1: none)
  int* vict = pos + 8;                             // [C] candidate removed at step i
  int* misc = vict + 8;                            // [0] contender count
  const float scale2 = p.scale * kLog2e;
  const int P = p.parts;                 // workgroups per unit (1: a workgroup owns the unit)
  const int HP = p.H_kv / P;             // KV heads per part
  int* flag_lds = reinterpret_cast<int*>(small + 480);
  const bool shared = (P > 1 && !p.filling);  // the parts of a unit hand their results to the one that resolves the group

  // (with parts on a full cache, an extra pass stores the last group's rows)
  for (int ch = 0; ch < p.n_chunks + (shared ? 1 : 0); ++ch) {
  for (int item = blockIdx.x; item < p.units * P; item += gridDim.x) {  // (parts: the grid covers every item)
  const int unit = item / P, part = item - unit * P;
  const int pair0 = unit * p.H_kv;
  const int kv0 = part * HP;             // this workgroup's KV heads: kv0 .. kv0 + HP - 1
  // [H][C][D] unmasked PV sums of the unit at hand: the workgroup's own area, or the unit's when parts share it
  float* const ublk = p.uscr + (size_t)(P > 1 ? unit : (int)blockIdx.x) * H * C * D;
  // rows cached when the group starts: k once the multi-state is full; while it fills (App. B: nothing
  // is removed while num_kv <= cache_max_size) the groups simply append their tokens
  const int n = p.filling ? p.n0 + ch * C : k;
  const int NC = n + C;  // candidates: the cached rows, then the group's own tokens
  const size_t tok_q = (size_t)ch * C * p.q_stride;    // element offset of the group's first token in q / out
  const size_t tok_kv = (size_t)ch * C * p.kv_stride;  // ... in k_new / v_new

  if (shared && ch > 0) {
    // Wait (bounded) until the unit's previous group is resolved, then put that group's rows of this
    // part's KV heads into the slots its tokens ended up in.  If the wait runs out -- it cannot while
    // all workgroups are resident, which the host checks -- the workgroup raises the cache's error flag
    // and leaves; every other one sees the flag in its own wait and leaves too.
    const int tid = threadIdx.x;
    if (tid == 0) {
      int ok = 0;
      for (int spin = 0;; ++spin) {
        if ((int)(uint32_t)ld_agent_u64(p.pstate + unit) == ch) {
          ok = 1;
          break;
        }
        if (spin >= p.spin || ld_agent_i(p.error_flag) != 0) break;
        __builtin_amdgcn_s_sleep(4);
      }
      if (!ok) st_agent_i(p.error_flag, 1);
      flag_lds[2] = ok;
    }
    __syncthreads();
    if (flag_lds[2] == 0) return;  // block-uniform
    if (tid < C) pos[tid] = ld_agent_i(p.gpos + (size_t)unit * 8 + tid);
    __syncthreads();
    const size_t prev_kv = (size_t)(ch - 1) * C * p.kv_stride;
    for (int i = 0; i < C; ++i) {
      const int ps = pos[i];
      if (ps < 0) continue;  // block-uniform
      const T* kn = reinterpret_cast<const T*>(p.k_new) + prev_kv + (size_t)i * p.kv_stride + (size_t)(pair0 + kv0) * D;
      const T* vn = reinterpret_cast<const T*>(p.v_new) + prev_kv + (size_t)i * p.kv_stride + (size_t)(pair0 + kv0) * D;
      T* Ku = reinterpret_cast<T*>(p.K) + ((size_t)(pair0 + kv0) * k + ps) * D;
      T* Vu = reinterpret_cast<T*>(p.V) + ((size_t)(pair0 + kv0) * k + ps) * D;
      for (int x = tid; x < HP * ROW16; x += nt) {  // (written through: the resolving part may read these rows)
        const int h = x / ROW16, c16 = x - h * ROW16;
        st_agent_v16(reinterpret_cast<V16*>(Ku + (size_t)h * k * D) + c16, reinterpret_cast<const V16*>(kn)[x]);
        st_agent_v16(reinterpret_cast<V16*>(Vu + (size_t)h * k * D) + c16, reinterpret_cast<const V16*>(vn)[x]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();  // the rows are in place for this workgroup's passes
    if (ch == p.n_chunks) continue;
  }

  // ================= pass A: one stream of K and V per KV head for all C tokens =================
  for (int kvh = kv0; kvh < kv0 + HP; ++kvh) {
  // (a fresh opaque copy of the thread index per KV head: otherwise the lane arithmetic of the
  // body is hoisted out of the loops and kept in registers across them)
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int pair = pair0 + kvh;
  const T* Kb = reinterpret_cast<const T*>(p.K) + (size_t)pair * k * D;
  const T* Vb = reinterpret_cast<const T*>(p.V) + (size_t)pair * k * D;
  const T* knew0 = reinterpret_cast<const T*>(p.k_new) + tok_kv + (size_t)pair * D;
  const T* vnew0 = reinterpret_cast<const T*>(p.v_new) + tok_kv + (size_t)pair * D;
  const T* qb0 = reinterpret_cast<const T*>(p.q) + tok_q + ((size_t)unit * H + (size_t)kvh * G) * D;

  // ---- logits (log2 domain) of all (token, head) combinations against every candidate: the n
  //      cached rows, then the group's own tokens (a token does not see a later one)
  float m[GE], Z[GE];
  const bool own_here = (wave == nw - 1);  // wave-uniform
  logit_pass<T, D, GE>(
      Kb, n, C, own_here, [&](int ge) { return qb0 + (size_t)(ge / G) * p.q_stride + (ge % G) * D; },
      [&](int r) { return knew0 + (size_t)r * p.kv_stride; }, [&](int ge, int r) { return ge / G < r; }, scale2,
      lane, wave, nw, e_lds, m);

  // the first V tile is requested before the softmax barriers
  const int lv = lane % LV;
  const int rv = lane / LV;
  constexpr bool PVM = PvMfma<T, D, GE>::OK;  // bf16, d = 128, 8 combinations: PV on the matrix cores
  V16 vA[PVM ? 8 : UV];
  if constexpr (PVM)
    pv_mfma_load<T, D>(vA, Vb, wave * PvMfma<T, D, GE>::ROWS, n, lane);
  else
    pv_first_tile<T, D, GE>(vA, Vb, n, lane, wave);

  // ---- maxima, exp values, sums over all causally allowed candidates
  block_reduce<GE, true>(m, small, lane, wave, nw);
#pragma unroll
  for (int ge = 0; ge < GE; ++ge) Z[ge] = 0.f;
  for (int c = tid; c < NC; c += nt) {
#pragma unroll
    for (int ge = 0; ge < GE; ++ge) {
      const float e = __builtin_amdgcn_exp2f(e_lds[c * GE + ge] - m[ge]);  // (masked: 2^-inf = 0)
      e_lds[c * GE + ge] = e;
      Z[ge] += e;
    }
  }
  block_reduce<GE, false>(Z, small + kMaxWaves * GE, lane, wave, nw);

  // ---- tentative scores (heads in order; entry c is always this thread's) and the statistics
  {
    float rz[GE];
#pragma unroll
    for (int ge = 0; ge < GE; ++ge) rz[ge] = 1.0f / Z[ge];
    for (int c = tid; c < NC; c += nt) {
#pragma unroll
      for (int i = 0; i < C; ++i) {
        float a = 0.f;
#pragma unroll
        for (int g = 0; g < G; ++g) a = fmaf(e_lds[c * GE + i * G + g], rz[i * G + g], a);
        if (!p.filling) t_lds[i * ncp + c] = (kvh == kv0) ? a : t_lds[i * ncp + c] + a;
      }
    }
#pragma unroll
    for (int ge = 0; ge < GE; ++ge) {
      if (tid == ge) {
        const int hq = kvh * G + ge % G;
        mst[hq * C + ge / G] = m[ge];
        zst[hq * C + ge / G] = Z[ge];
      }
    }
  }

  // ---- unmasked PV sums: U_(i,g) = sum over allowed candidates of w V
  float* red = big;  // [nw][GE * D]
  if constexpr (PVM) {
    f32x4_t pacc[8];
    pv_pass_mfma<T, D, GE>(Vb, n, e_lds, GE, 0, lane, wave, nw, vA, pacc);
    pv_mfma_finish<T, D, GE>(pacc, n, C, own_here, [&](int r) { return vnew0 + (size_t)r * p.kv_stride; }, e_lds, GE,
                             0, lane, wave, red);
  } else {
    float acc[GE][VEC];
    pv_pass<T, D, GE>(Vb, n, C, own_here, [&](int r) { return vnew0 + (size_t)r * p.kv_stride; }, e_lds, GE, 0, lane,
                      wave, nw, vA, acc);
#pragma unroll
    for (int ge = 0; ge < GE; ++ge)
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[ge][v] = column_sum<LV>(acc[ge][v]);
    __syncthreads();  // everyone is done reading the exp values; the reduction area reuses them
    if (rv == 0) {
#pragma unroll
      for (int ge = 0; ge < GE; ++ge)
#pragma unroll
        for (int v = 0; v < VEC; ++v) red[(wave * GE + ge) * D + lv * VEC + v] = acc[ge][v];
    }
  }
  __syncthreads();
  for (int x = tid; x < GE * D; x += nt) {
    float a = red[x];
    for (int w = 1; w < nw; ++w) a += red[w * GE * D + x];
    const int ge = x / D;
    float* const ud = ublk + ((size_t)(kvh * G + ge % G) * C + ge / G) * D + (x - ge * D);
    if (shared)
      st_agent(ud, a);
    else
      *ud = a;
  }
  __syncthreads();  // the reduction area is free for the next KV head
  }  // KV heads

  // ================= resolution: token by token =================
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);  // the U sums are in memory before other waves read them
  if (shared) {
    // ---- hand over: this part's tentative-score rows and its heads' statistics (the U sums are there
    //      already); whoever arrives last resolves the group for the unit
    float* const tp = p.tpart + ((size_t)unit * P + part) * C * ncp;
    for (int x = tid; x < C * ncp; x += nt) st_agent(tp + x, t_lds[x]);
    float* const sp = p.stat + (size_t)unit * H * C * 2;
    for (int x = tid; x < HP * G * C; x += nt) {
      const int y = kv0 * G * C + x;  // (head, token) entries of this part's heads are contiguous
      st_agent(sp + 2 * y, mst[y]);
      st_agent(sp + 2 * y + 1, zst[y]);
    }
    const int prev = arrive(p.cnt_unit + unit, 1, flag_lds, tid);
    if (prev + 1 != P) continue;  // (block-uniform) not the last: on to the next group, which starts with a wait
    reset_counter(p.cnt_unit + unit, tid);
    for (int x = tid; x < C * ncp; x += nt) {
      float a = 0.f;
      constexpr int PB = 8;  // parts whose loads are issued together
      for (int q0 = 0; q0 < P; q0 += PB) {
        float v[PB];
#pragma unroll
        for (int u = 0; u < PB; ++u) v[u] = (q0 + u < P) ? ld_agent(p.tpart + ((size_t)unit * P + q0 + u) * C * ncp + x) : 0.f;
#pragma unroll
        for (int u = 0; u < PB; ++u) a += v[u];  // (part order)
      }
      t_lds[x] = a;
    }
    for (int x = tid; x < H * C; x += nt) {
      mst[x] = ld_agent(sp + 2 * x);
      zst[x] = ld_agent(sp + 2 * x + 1);
    }
  }
  if (tid < C) pos[tid] = -1;
  __syncthreads();
  float* qs = e_lds;                                       // [H][D] the token's queries in fp32
  int* cont = reinterpret_cast<int*>(e_lds + (size_t)H * D);  // candidates that may be the argmin
  int32_t* const evp = p.evicted ? p.evicted + (size_t)ch * C * p.units : nullptr;

  // w of candidate `cand` for every query head of token i, handed to `sink(hq, w)` by all lanes
  // of the calling wave (a wave per candidate; lanes split the row's elements)
  auto weights_of = [&](int i, int cand, auto&& sink) {
    constexpr int HB = 8;  // KV heads whose rows are requested together (the loads are what takes time here)
    for (int h0 = 0; h0 < p.H_kv; h0 += HB) {
      float kx[HB][EPL];
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) {
        const int h = min(h0 + hb, p.H_kv - 1);
        const T* row = (cand < k) ? reinterpret_cast<const T*>(p.K) + ((size_t)(pair0 + h) * k + cand) * D
                                  : reinterpret_cast<const T*>(p.k_new) + tok_kv + (size_t)(cand - k) * p.kv_stride +
                                        (size_t)(pair0 + h) * D;
        // (with parts a cached row may have been stored by another workgroup of this launch)
#pragma unroll
        for (int e = 0; e < EPL; ++e)
          kx[hb][e] = (lane + 64 * e < D) ? ((shared && cand < k) ? elem_f32_agent<T>(row, lane + 64 * e) : elem_f32<T>(row, lane + 64 * e)) : 0.f;
      }
#pragma unroll
      for (int hb = 0; hb < HB; ++hb) {
        const int h = h0 + hb;
        if (h < p.H_kv) {  // wave-uniform
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const int hq = h * G + g;
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e)
              if (lane + 64 * e < D) part = fmaf(kx[hb][e], qs[hq * D + lane + 64 * e], part);
            const float l2 = group_reduce<64, false>(part) * scale2;
            sink(hq, __builtin_amdgcn_exp2f(l2 - mst[hq * C + i]));
          }
        }
      }
    }
  };
  // slot index a candidate stands for when scores tie (the token at hand counts as index k)
  auto position = [&](int i, int cand) { return cand < k ? cand : (cand == k + i ? k : pos[cand - k]); };

  if (p.filling) {
    // nothing is removed: out = U / Z, the tokens take the next free slots
    const int HO = HP * G;  // query heads of this workgroup's KV heads (all of them without parts)
    for (int x = tid; x < C * HO * D; x += nt) {
      const int i = x / (HO * D), y = kv0 * G * D + (x - i * (HO * D)), hq = y / D;
      T* outi = reinterpret_cast<T*>(p.out) + tok_q + (size_t)i * p.q_stride + (size_t)unit * H * D;
      E::store(outi + y, ublk[((size_t)hq * C + i) * D + (y - hq * D)] / zst[hq * C + i]);
    }
    if (tid < C) {
      pos[tid] = n + tid;
      if (evp && part == 0) evp[(size_t)tid * p.units + unit] = -1;
    }
    if (tid == 0 && part == 0) p.occupancy[unit] = n + C;
    __syncthreads();
  }
  for (int i = 0; i < C && !p.filling; ++i) {
    const T* qi = reinterpret_cast<const T*>(p.q) + tok_q + (size_t)i * p.q_stride + (size_t)unit * H * D;
    for (int x = tid; x < H * D; x += nt) qs[x] = elem_f32<T>(qi, x);
    __syncthreads();
    // (a) what the candidates removed by the group's earlier tokens weigh for this token
    for (int e = wave; e < i; e += nw)
      weights_of(i, vict[e], [&](int hq, float w) {
        if (lane == 0) wev[e * H + hq] = w;
      });
    __syncthreads();
    // (b) corrected sums; f = Z / Z' >= 1 per head, f_max its largest value (1 is used as the lower end)
    float fr[2] = {1.0f, 0.0f};  // [0] f_max, [1] nonzero: some head kept too little of its sum
    for (int hq = tid; hq < H; hq += nt) {
      const float zf = zst[hq * C + i];
      float d = 0.f;
      for (int e = 0; e < i; ++e) d += wev[e * H + hq];
      const float zc = zf - d;
      zcs[hq] = zc;
      fr[0] = fmaxf(fr[0], zf / zc);
      if (!(zc > kMinKept * zf)) fr[1] = 1.0f;  // (also Z' <= 0 and NaN)
    }
    block_reduce<2, true>(fr, small, lane, wave, nw);
    const float f_max = fr[0];
    const bool from_scratch = (fr[1] != 0.0f) || p.force_exact;  // block-uniform
    float* Ti = t_lds + i * ncp;
    auto alive = [&](int c) {
      if (c < p.n_pinned) return false;  // TOVA+i (App. A): the first tokens hold slots 0 .. n_pinned-1
      for (int e = 0; e < i; ++e)
        if (vict[e] == c) return false;
      return true;
    };
    float best = INFINITY;
    int bpos = 0x7fffffff, bcand = k + i;
    if (from_scratch) {
      // ---- the guard's way out: this token as a single-token step over the candidates that are still
      //      there (Sec. 3.2, Sec. 4): per KV head a logit pass over the k cached rows and the group's
      //      tokens up to this one, those that were removed masked out; softmax; scores into the
      //      token's row of t_lds (its tentative scores are no longer needed); PV; outputs
      __syncthreads();  // (everyone has read zcs / the query copy: the big area is rewritten below)
      T* outx = reinterpret_cast<T*>(p.out) + tok_q + (size_t)i * p.q_stride + (size_t)unit * H * D;
      for (int kvh = 0; kvh < p.H_kv; ++kvh) {
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        using Gx = Geo<T, D, G>;
        const int pair = pair0 + kvh;
        const T* Kb = reinterpret_cast<const T*>(p.K) + (size_t)pair * k * D;
        const T* Vb = reinterpret_cast<const T*>(p.V) + (size_t)pair * k * D;
        const T* knew0 = reinterpret_cast<const T*>(p.k_new) + tok_kv + (size_t)pair * D;
        const T* vnew0 = reinterpret_cast<const T*>(p.v_new) + tok_kv + (size_t)pair * D;
        const T* qh = qi + (size_t)kvh * G * D;
        const int n_own = i + 1, ncx = k + n_own;
        const bool own_here = (wave == nw - 1);
        float mx[G], Zx[G];
        // (cached rows are read past the caches on this route: with parts another workgroup of the launch
        // may have stored them, and an earlier trip down this route may have left old copies nearby)
        logit_pass<T, D, G, 2, true>(
            Kb, k, n_own, own_here, [&](int g) { return qh + g * D; },
            [&](int r) { return knew0 + (size_t)r * p.kv_stride; },
            [&](int, int r) { return r < i && pos[r] < 0; },  // an earlier token of the group that holds no slot any more
            scale2, lane, wave, nw, e_lds, mx);
        V16 vX[Gx::UV];
        pv_first_tile<T, D, G, true>(vX, Vb, k, lane, wave);
        __syncthreads();  // the logits are in LDS
        if (tid < i && vict[tid] < k) {  // cached rows that earlier tokens of the group removed
#pragma unroll
          for (int g = 0; g < G; ++g) e_lds[vict[tid] * G + g] = -INFINITY;
        }
        __syncthreads();
#pragma unroll
        for (int g = 0; g < G; ++g) mx[g] = -INFINITY;  // (the pass's running maxima saw the removed rows)
        for (int c = tid; c < ncx; c += nt) {
#pragma unroll
          for (int g = 0; g < G; ++g) mx[g] = fmaxf(mx[g], e_lds[c * G + g]);
        }
        block_reduce<G, true>(mx, small, lane, wave, nw);
#pragma unroll
        for (int g = 0; g < G; ++g) Zx[g] = 0.f;
        for (int c = tid; c < ncx; c += nt) {
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const float e = __builtin_amdgcn_exp2f(e_lds[c * G + g] - mx[g]);
            e_lds[c * G + g] = e;
            Zx[g] += e;
          }
        }
        block_reduce<G, false>(Zx, small + kMaxWaves * G, lane, wave, nw);
        {
          float rz[G];
#pragma unroll
          for (int g = 0; g < G; ++g) rz[g] = 1.0f / Zx[g];
          for (int c = tid; c < ncx; c += nt) {  // (entry c is always this thread's; KV heads in order)
            float a = 0.f;
#pragma unroll
            for (int g = 0; g < G; ++g) a = fmaf(e_lds[c * G + g], rz[g], a);
            Ti[c] = (kvh == 0) ? a : Ti[c] + a;
          }
        }
        float accx[G][Gx::VEC];
        pv_pass<T, D, G, true>(Vb, k, n_own, own_here, [&](int r) { return vnew0 + (size_t)r * p.kv_stride; }, e_lds, G, 0,
                               lane, wave, nw, vX, accx);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int v = 0; v < Gx::VEC; ++v) accx[g][v] = column_sum<Gx::LV>(accx[g][v]);
        float* red = big;  // [nw][G * D]
        __syncthreads();   // everyone is done reading the exp values; the reduction area reuses them
        if (lane / Gx::LV == 0) {
#pragma unroll
          for (int g = 0; g < G; ++g)
#pragma unroll
            for (int v = 0; v < Gx::VEC; ++v) red[(wave * G + g) * D + (lane % Gx::LV) * Gx::VEC + v] = accx[g][v];
        }
        __syncthreads();
        for (int x = tid; x < G * D; x += nt) {
          float a = red[x];
          for (int w = 1; w < nw; ++w) a += red[w * G * D + x];
          float zg = Zx[0];
#pragma unroll
          for (int g = 1; g < G; ++g) zg = (x / D == g) ? Zx[g] : zg;
          E::store(outx + (size_t)kvh * G * D + x, a / zg);
        }
        __syncthreads();  // the reduction area is free for the next KV head
      }
      // the victim among the candidates that are still there, by (score, slot index)
      for (int c = tid; c <= k + i; c += nt) {
        if (!alive(c)) continue;
        const float sc = Ti[c];
        const int pc = position(i, c);
        if (sc < best || (sc == best && pc < bpos)) {
          best = sc;
          bpos = pc;
          bcand = c;
        }
      }
    } else {
    // (c) the smallest upper bound, then the candidates whose lower bound does not exceed it
    float lo[1] = {-INFINITY};  // -(min T)
    for (int c = tid; c <= k + i; c += nt)
      if (alive(c)) lo[0] = fmaxf(lo[0], -Ti[c]);
    if (tid == 0) misc[0] = 0;
    block_reduce<1, true>(lo, small + 64, lane, wave, nw);
    const float bound = -lo[0] * f_max * (1.0f + kBoundSlack);
    for (int c = tid; c <= k + i; c += nt)
      if (alive(c) && Ti[c] * (1.0f - kBoundSlack) <= bound) cont[atomicAdd(&misc[0], 1)] = c;
    __syncthreads();
    const int ncont = misc[0];
    // (d) exact scores of those (a wave per candidate), argmin by (score, slot index)
    for (int x = wave; x < ncont; x += nw) {
      const int cand = cont[x];
      float s = 0.f, a = 0.f;
      weights_of(i, cand, [&](int hq, float w) {
        a = fmaf(w, 1.0f / zcs[hq], a);
        if (hq % G == G - 1) {  // KV-head partials added in head order, as the single-token kernels do
          s += a;
          a = 0.f;
        }
      });
      const int pc = position(i, cand);
      if (s < best || (s == best && pc < bpos)) {
        best = s;
        bpos = pc;
        bcand = cand;
      }
    }
    }  // corrected / from scratch
    // (the lanes of a wave agree already on the corrected route; from scratch each has its own candidates)
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      const float ob = __shfl_xor(best, o);
      const int op = __shfl_xor(bpos, o), oc = __shfl_xor(bcand, o);
      if (ob < best || (ob == best && op < bpos)) {
        best = ob;
        bpos = op;
        bcand = oc;
      }
    }
    float* bv = small + 256;
    int* bi = reinterpret_cast<int*>(small + 256 + kMaxWaves);
    int* bc = bi + kMaxWaves;
    if (lane == 0) {
      bv[wave] = best;
      bi[wave] = bpos;
      bc[wave] = bcand;
    }
    __syncthreads();
    best = bv[0];
    bpos = bi[0];
    bcand = bc[0];
    for (int w = 1; w < nw; ++w) {
      if (bv[w] < best || (bv[w] == best && bi[w] < bpos)) {
        best = bv[w];
        bpos = bi[w];
        bcand = bc[w];
      }
    }
    __syncthreads();  // (everyone has read pos / vict of the earlier tokens)
    // (e) the token takes its victim's slot (or is dropped itself)
    if (tid == 0) {
      vict[i] = bcand;
      if (bcand != k + i) {
        pos[i] = bpos;
        if (bcand >= k) pos[bcand - k] = -1;
      }
      if (evp) evp[(size_t)i * p.units + unit] = bpos;  // (bpos == k: the token itself)
    }
    // (f) the token's output: the removed candidates' share taken out of the unmasked sums
    T* outi = reinterpret_cast<T*>(p.out) + tok_q + (size_t)i * p.q_stride + (size_t)unit * H * D;
    for (int x = tid; x < H * D && !from_scratch; x += nt) {
      const int hq = x / D, dd = x - hq * D;
      const float* up = ublk + ((size_t)hq * C + i) * D + dd;
      float a = shared ? ld_agent(up) : *up;
      for (int e = 0; e < i; ++e) {
        const int cand = vict[e];
        const T* vrow = (cand < k) ? reinterpret_cast<const T*>(p.V) + ((size_t)(pair0 + hq / G) * k + cand) * D
                                   : reinterpret_cast<const T*>(p.v_new) + tok_kv + (size_t)(cand - k) * p.kv_stride +
                                         (size_t)(pair0 + hq / G) * D;
        a = fmaf(-wev[e * H + hq], (shared && cand < k) ? elem_f32_agent<T>(vrow, dd) : elem_f32<T>(vrow, dd), a);
      }
      E::store(outi + x, a / zcs[hq]);
    }
    __syncthreads();
  }

  // ================= commit: the tokens that still hold a slot =================
  if (shared) {
    // the resolving part only says where the tokens ended up; every part stores the rows of its own KV
    // heads when it comes back to the unit (top of the loop)
    if (tid < C) st_agent_i(p.gpos + (size_t)unit * 8 + tid, pos[tid]);
    if (tid == 0) {
      for (int i = 0; i < C; ++i)
        if (pos[i] >= 0) st_agent_i(p.slot_token + (size_t)unit * k + pos[i], p.t + ch * C + i);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);  // (the counter's reset, the slots and the map have landed ...)
    __syncthreads();
    if (tid == 0) st_agent_u64(p.pstate + unit, (unsigned long long)(uint32_t)(ch + 1));  // ... before the group counts as done
    continue;
  }
  for (int i = 0; i < C; ++i) {
    const int ps = pos[i];
    if (ps < 0) continue;  // block-uniform
    const T* kn = reinterpret_cast<const T*>(p.k_new) + tok_kv + (size_t)i * p.kv_stride + (size_t)(pair0 + kv0) * D;
    const T* vn = reinterpret_cast<const T*>(p.v_new) + tok_kv + (size_t)i * p.kv_stride + (size_t)(pair0 + kv0) * D;
    T* Ku = reinterpret_cast<T*>(p.K) + ((size_t)(pair0 + kv0) * k + ps) * D;
    T* Vu = reinterpret_cast<T*>(p.V) + ((size_t)(pair0 + kv0) * k + ps) * D;
    for (int x = tid; x < HP * ROW16; x += nt) {  // (this workgroup's KV heads: all of them without parts)
      const int h = x / ROW16, c16 = x - h * ROW16;
      reinterpret_cast<V16*>(Ku + (size_t)h * k * D)[c16] = reinterpret_cast<const V16*>(kn)[x];
      reinterpret_cast<V16*>(Vu + (size_t)h * k * D)[c16] = reinterpret_cast<const V16*>(vn)[x];
    }
    if (tid == 0 && part == 0) p.slot_token[(size_t)unit * k + ps] = p.t + ch * C + i;
  }
  // the rows must have landed before other waves of this block read them in the unit's next group
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  }  // units (items)
  }  // groups
}

template <typename T, int D>
hipError_t launch_gc(int G, int C, const PrefillParams& p, const LaunchPlan& lp, hipStream_t s) {
#define TOVA_PREFILL_CASE(g, c)                                                                              \
  if (G == g && C == c) {                                                                                    \
    {                                                                                                        \
      const hipError_t e = ensure_dynamic_lds<&tova_prefill_kernel<T, D, g, c>>(lp.lds_bytes);               \
      if (e != hipSuccess) return e;                                                                         \
    }                                                                                                        \
    hipLaunchKernelGGL((tova_prefill_kernel<T, D, g, c>), dim3(lp.grid), dim3(lp.block), lp.lds_bytes, s, p); \
    return hipGetLastError();                                                                                \
  }
  TOVA_PREFILL_CASE(1, 4)
  TOVA_PREFILL_CASE(1, 8)
  TOVA_PREFILL_CASE(2, 2)
  TOVA_PREFILL_CASE(2, 4)
  TOVA_PREFILL_CASE(4, 2)
#undef TOVA_PREFILL_CASE
  return hipErrorInvalidValue;
}

template <typename T, int D>
int resident_gc(int G, int C, int block, int lds) {
  int per_cu = -1;
#define TOVA_PREFILL_CASE(g, c)                                                                                   \
  if (G == g && C == c) {                                                                                         \
    if (ensure_dynamic_lds<&tova_prefill_kernel<T, D, g, c>>(lds) != hipSuccess) return 0;                        \
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tova_prefill_kernel<T, D, g, c>, block, (size_t)lds) != hipSuccess) \
      return 0;                                                                                                   \
  }
  TOVA_PREFILL_CASE(1, 4)
  TOVA_PREFILL_CASE(1, 8)
  TOVA_PREFILL_CASE(2, 2)
  TOVA_PREFILL_CASE(2, 4)
  TOVA_PREFILL_CASE(4, 2)
#undef TOVA_PREFILL_CASE
  if (per_cu < 0) return 0;
  return per_cu * device_cus();
}
template <typename T>
int resident_dgc(int D, int G, int C, int block, int lds) {
  switch (D) {
    case 32: return resident_gc<T, 32>(G, C, block, lds);
    case 64: return resident_gc<T, 64>(G, C, block, lds);
    case 128: return resident_gc<T, 128>(G, C, block, lds);
    default: return 0;
  }
}

template <typename T>
hipError_t launch_dgc(int D, int G, int C, const PrefillParams& p, const LaunchPlan& lp, hipStream_t s) {
  switch (D) {
    case 32: return launch_gc<T, 32>(G, C, p, lp, s);
    case 64: return launch_gc<T, 64>(G, C, p, lp, s);
    case 128: return launch_gc<T, 128>(G, C, p, lp, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

int prefill_resident_blocks(int dtype_is_bf16, int D, int G, int C, int block, int lds_bytes) {
  return dtype_is_bf16 ? resident_dgc<bf16_t>(D, G, C, block, lds_bytes) : resident_dgc<float>(D, G, C, block, lds_bytes);
}

hipError_t launch_prefill(int dtype_is_bf16, int D, int G, int C, const PrefillParams& p, const LaunchPlan& lp,
                          hipStream_t stream) {
  return dtype_is_bf16 ? launch_dgc<bf16_t>(D, G, C, p, lp, stream) : launch_dgc<float>(D, G, C, p, lp, stream);
}

}  // namespace tova
