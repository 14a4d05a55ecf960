// Device-side helpers shared by the kernels of this library (included by the .hip files only):
// element types, cross-lane reductions, block reductions, cross-workgroup hand-off primitives and
// the row geometry of the streaming passes.  Everything lives in an unnamed namespace inside
// tova: each translation unit gets its own copy.
#ifndef TOVA_DEVICE_H
#define TOVA_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace tova {
namespace {

// ---------------------------------------------------------------- elements
struct alignas(16) V16 {
  uint32_t w[4];
};

struct bf16_t {
  uint16_t x;
};
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <typename T>
struct Elem;

template <>
struct Elem<float> {
  static constexpr int VEC = 4;
  static __device__ __forceinline__ void unpack(const V16& p, float (&f)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(p.w[i]);
  }
  // acc + sum of the 4 products of two 16-byte chunks
  static __device__ __forceinline__ float dot(const V16& a, const V16& b, float acc) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc = fmaf(__uint_as_float(a.w[i]), __uint_as_float(b.w[i]), acc);
    return acc;
  }
  static __device__ __forceinline__ void store(float* dst, float v) { *dst = v; }
};

template <>
struct Elem<bf16_t> {
  static constexpr int VEC = 8;
  static __device__ __forceinline__ void unpack(const V16& p, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(p.w[i] << 16);
      f[2 * i + 1] = __uint_as_float(p.w[i] & 0xffff0000u);
    }
  }
  // acc + sum of the 8 products of two 16-byte chunks: v_dot2_f32_bf16 takes the packed
  // pairs as they are (bf16 products are exact in fp32, the accumulation is fp32)
  static __device__ __forceinline__ float dot(const V16& a, const V16& b, float acc) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w[i]),
                                            __builtin_bit_cast(bf16x2_t, b.w[i]), acc, false);
    return acc;
  }
  // round to nearest even, NaN kept quiet
  static __device__ __forceinline__ void store(bf16_t* dst, float v) {
    uint32_t u = __float_as_uint(v);
    uint16_t r;
    if ((u & 0x7fffffffu) > 0x7f800000u) {
      r = 0x7fc0;
    } else {
      u += 0x7fffu + ((u >> 16) & 1u);
      r = (uint16_t)(u >> 16);
    }
    dst->x = r;
  }
};

// ------------------------------------------------------- cross-lane helpers
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Lane l <-> lane l ^ 16 and l ^ 32 exchanges without the LDS crossbar.  The gfx950 permlane
// swaps exchange, between two registers a and b, the odd rows of 16 lanes of a with the even
// rows of b (a' = [a0 b0 a2 b2], b' = [a1 b1 a3 b3]), resp. the upper half of a with the lower
// half of b; swapping a value with a copy of itself therefore leaves both partners of every
// lane in a' and b'.  Written as inline asm with both registers as in/out operands: the
// two-result builtin form returned its first result twice with the ROCm 7.2 compiler.  The
// s_nop pads cover the VALU -> permlane read/write wait states the compiler cannot see.
__device__ __forceinline__ void swap_rows16(unsigned& a, unsigned& b) {
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void swap_rows32(unsigned& a, unsigned& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
template <bool IS_MAX>
__device__ __forceinline__ float combine(float a, float b) {
  return IS_MAX ? fmaxf(a, b) : a + b;
}
template <bool IS_MAX>
__device__ __forceinline__ float fold_rows16(float x) {  // x[l] op x[l ^ 16]
  unsigned a = __builtin_bit_cast(unsigned, x), b = a;
  swap_rows16(a, b);
  return combine<IS_MAX>(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
}
template <bool IS_MAX>
__device__ __forceinline__ float fold_rows32(float x) {  // x[l] op x[l ^ 32]
  unsigned a = __builtin_bit_cast(unsigned, x), b = a;
  swap_rows32(a, b);
  return combine<IS_MAX>(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
}

// Reduction over each group of LPR adjacent lanes whose lanes hold partials of the SAME
// quantity; every lane of the group gets the total.  quad_perm[1,0,3,2], quad_perm[2,3,0,1],
// row_half_mirror, row_mirror (the mirrors are valid because after the first two steps all
// lanes of a quad agree), then the row swaps.
template <int LPR, bool IS_MAX = false>
__device__ __forceinline__ float group_reduce(float x) {
  if (LPR >= 2) x = combine<IS_MAX>(x, dpp_mov<0xB1>(x));
  if (LPR >= 4) x = combine<IS_MAX>(x, dpp_mov<0x4E>(x));
  if (LPR >= 8) x = combine<IS_MAX>(x, dpp_mov<0x141>(x));
  if (LPR >= 16) x = combine<IS_MAX>(x, dpp_mov<0x140>(x));
  if (LPR >= 32) x = fold_rows16<IS_MAX>(x);
  if (LPR >= 64) x = fold_rows32<IS_MAX>(x);
  return x;
}
template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  return group_reduce<LPR, false>(x);
}

// Sum over the 64 / LV lanes that hold the same column chunk (lanes l, l + LV, l + 2 LV, ...),
// for lanes that hold DIFFERENT columns: row rotations inside a row of 16, then the row swaps.
template <int LV>
__device__ __forceinline__ float column_sum(float x) {
  if (LV <= 8) x += dpp_mov<0x128>(x);   // row_ror:8
  if (LV <= 4) x += dpp_mov<0x124>(x);   // row_ror:4
  if (LV <= 16) x = fold_rows16<false>(x);
  if (LV <= 32) x = fold_rows32<false>(x);
  return x;
}

// Small fixed LDS area in front of the big dynamic one (floats).
constexpr int kSmallFloats = 512;
constexpr int kMaxWaves = 16;

// Block-wide max / sum of G per-thread values with ONE barrier: every wave reduces its lanes
// (DPP + row swaps), lane 0 posts the wave's result, and after the barrier every thread
// combines the nw posted values in wave order (so the result does not depend on timing).
// `red` holds kMaxWaves * G floats and must not be in use by a previous reduction.
template <int G, bool IS_MAX>
__device__ __forceinline__ void block_reduce(float (&v)[G], float* red, int lane, int wave, int nw) {
#pragma unroll
  for (int g = 0; g < G; ++g) v[g] = group_reduce<64, IS_MAX>(v[g]);
  if (lane == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) red[wave * G + g] = v[g];
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float a = red[g];
    for (int w = 1; w < nw; ++w) a = combine<IS_MAX>(a, red[w * G + g]);
    v[g] = a;
  }
}

// Block-wide argmin of (value, index) pairs, the lowest index winning ties: every wave reduces its
// lanes by butterfly shuffles, lane 0 posts the wave's pair, and after one barrier every thread
// combines the posted pairs in wave order.  `red` holds 2 * kMaxWaves words and must not be in use.
// (the wave's part: afterwards every lane holds the wave's lowest value and its lowest index)
template <typename V>
__device__ __forceinline__ void wave_argmin(V& best, int& bj) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const V ob = __shfl_xor(best, o);
    const int oj = __shfl_xor(bj, o);
    if (ob < best || (ob == best && oj < bj)) {
      best = ob;
      bj = oj;
    }
  }
}
template <typename V>  // float scores, or int token indices
__device__ __forceinline__ void block_argmin(V& best, int& bj, float* red, int lane, int wave, int nw) {
  static_assert(sizeof(V) == 4, "one word per posted value");
  wave_argmin(best, bj);
  V* bv = reinterpret_cast<V*>(red);
  int* bi = reinterpret_cast<int*>(red + kMaxWaves);
  if (lane == 0) {
    bv[wave] = best;
    bi[wave] = bj;
  }
  __syncthreads();
  best = bv[0];
  bj = bi[0];
  for (int w = 1; w < nw; ++w) {
    const V ob = bv[w];
    const int oj = bi[w];
    if (ob < best || (ob == best && oj < bj)) {
      best = ob;
      bj = oj;
    }
  }
}

// Cross-workgroup hand-off.  A full agent-scope release fence writes back the whole L2 of
// the XCD and an acquire fence invalidates it; issued by every wave of every workgroup that
// costs far more than the step's entire K/V stream.  Instead, everything one workgroup hands
// to another is written with agent-scope (write-through) stores and read with agent-scope
// (cache-bypassing) loads, so no cache maintenance is needed at all: the producer only has
// to wait until its stores have completed before it bumps the arrival counter.
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent_i(int32_t* p, int32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t ld_agent_i(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent_u64(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_agent_u64(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_agent2(const float* p) {  // p is 8-byte aligned
  unsigned long long r = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((uint32_t)r), __uint_as_float((uint32_t)(r >> 32)));
}

// A 16-byte piece of a cached row: an ordinary load, or (COH) past the caches, for rows that another
// workgroup of the same launch may have written through.
template <bool COH>
__device__ __forceinline__ V16 ld_v16(const void* p) {
  if constexpr (COH) {
    const unsigned long long* q = reinterpret_cast<const unsigned long long*>(p);
    const unsigned long long a = ld_agent_u64(q), b = ld_agent_u64(q + 1);
    return V16{{(uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32)}};
  } else {
    return *reinterpret_cast<const V16*>(p);
  }
}

// Arrival on a counter.  All threads of the block call it after writing their results with
// st_agent; it adds `add` to the counter once the block's stores have completed and returns the
// counter's previous value to every thread.  The caller decides from that value whether it is
// the last one, in which case it may read what the others wrote (ld_agent) and must reset the
// counter (reset_counter) for the next step.  Nobody waits for anybody.
__device__ __forceinline__ int arrive(int32_t* counter, int add, int* flag_lds, int tid) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // keep the stores above this point
  __builtin_amdgcn_s_waitcnt(0);                          // ... and wait until they have completed
  __syncthreads();
  if (tid == 0)
    flag_lds[1] = __hip_atomic_fetch_add(counter, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  return flag_lds[1];
}
__device__ __forceinline__ void reset_counter(int32_t* counter, int tid) {
  if (tid == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Unit finisher: per-thread argmin over the head-summed scores of the k+1 candidates.
// sgu[h * kp + j] is KV head h's partial for candidate j.  A thread owns candidate pairs
// (2m, 2m+1), m = tid + i * nt, sums the H_kv partials in head order and keeps the lowest
// (ascending j, strict <, so the lowest index wins ties; candidates below n_pinned are kept out:
// TOVA+i, App. A).  The loads bypass the caches, so
// JB * HB of them are issued before the first is used.
template <int JB, int HB>
__device__ __forceinline__ void scan_scores(const float* sgu, int H_kv, int kp, int k, int n_pinned, int tid,
                                            int nt, float& best, int& bj) {
  const int npair2 = (k + 2) / 2;  // candidate pairs covering 0..k
  for (int m0 = tid; m0 < npair2; m0 += nt * JB) {
    float s0[JB], s1[JB];
#pragma unroll
    for (int b = 0; b < JB; ++b) s0[b] = s1[b] = 0.f;
    for (int h0 = 0; h0 < H_kv; h0 += HB) {
      float2 raw[JB][HB];
#pragma unroll
      for (int b = 0; b < JB; ++b) {
        const int mm = m0 + b * nt;
#pragma unroll
        for (int u = 0; u < HB; ++u) {
          raw[b][u] = make_float2(0.f, 0.f);
          if (mm < npair2 && h0 + u < H_kv) raw[b][u] = ld_agent2(sgu + (size_t)(h0 + u) * kp + 2 * mm);
        }
      }
#pragma unroll
      for (int b = 0; b < JB; ++b)
#pragma unroll
        for (int u = 0; u < HB; ++u) {
          s0[b] += raw[b][u].x;
          s1[b] += raw[b][u].y;
        }
    }
#pragma unroll
    for (int b = 0; b < JB; ++b) {
      const int j0 = 2 * (m0 + b * nt);
      if (j0 >= n_pinned && j0 <= k && s0[b] < best) {
        best = s0[b];
        bj = j0;
      }
      if (j0 + 1 >= n_pinned && j0 + 1 <= k && s1[b] < best) {
        best = s1[b];
        bj = j0 + 1;
      }
    }
  }
}

// ------------------------------------------------------------------ kernel
// Row geometry.  A row of d elements is CH = d / VEC 16-byte chunks.
//  * logit pass: LK = CH / CK adjacent lanes share a row, each holding CK chunks
//    (chunk c * LK + lane), so a wave-level load still covers whole contiguous
//    rows while the cross-lane sum per (row, head) needs only log2(LK) DPP steps;
//  * PV pass: one chunk per lane (LV = CH lanes per row), no cross-lane work in
//    the loop, G * VEC accumulators per lane.
template <typename T, int D, int G>
struct Geo {
  static constexpr int VEC = Elem<T>::VEC;
  static constexpr int CH = D / VEC;
  static constexpr int CK = (CH >= 8) ? 2 : 1;
  static constexpr int LK = CH / CK;
  static constexpr int RK = 64 / LK;  // rows per wave pass, logit pass
  static constexpr int UK = (G >= 8) ? 1 : 2;  // passes per register buffer (two buffers in flight);
                                               // fewer for wide groups, whose q fragments fill the registers
  // Wide bf16 groups run the logit pass on the matrix cores (see the kernel): q.K^T for 16 rows x
  // up to 16 heads per v_mfma_f32_16x16x32_bf16, which takes the register file and the VALU out
  // of the picture (8 heads of q fragments alone are 64 VGPRs on the vector path).  Groups of 4 heads
  // at d = 128 take it as well: three quarters of the instruction's columns are padding then, but the
  // instruction is cheap against the ~25 vector instructions per KB that it replaces (bench workload:
  // 38.3 -> 36.7 us per step together with the PV pass below).
  static constexpr bool MFMA_K =
      (sizeof(T) == 2) && (D % 32 == 0) && ((G >= 8 && G <= 16) || (G == 4 && D == 128));
  static constexpr int LV = CH;
  static constexpr int RV = 64 / LV;  // rows per wave pass, PV pass
  static constexpr int UV = (G >= 8) ? 2 : 4;
  static_assert(D % VEC == 0 && CH <= 64 && (CH & (CH - 1)) == 0, "row geometry");
};

constexpr float kLog2e = 1.4426950408889634f;

// A kernel that wants more dynamic LDS than the 64 KB default has to be told so.  Done once per
// (kernel instantiation, device) for the largest size seen so far, not at every launch.
template <auto Kernel>
inline hipError_t ensure_dynamic_lds(int bytes) {
  constexpr int kDevices = 64;
  static std::atomic<int> granted[kDevices];  // zero-initialised; one array per instantiation
  if (bytes <= 64 * 1024) return hipSuccess;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < kDevices && granted[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && dev >= 0 && dev < kDevices) granted[dev].store(bytes, std::memory_order_release);
  return e;
}

// ------------------------------------------------------------------ streaming passes
// Both kernels stream a KV head's rows twice per token (group): once through the logit pass (K),
// once through the PV pass (V).  A row serves NH "columns": the query heads of the KV head, or
// (token, head) combinations of a group of prompt tokens.  Besides the `nrows` cached rows there
// are `n_own` rows of the caller's own (the incoming token, or the group's tokens), which the
// block's last wave takes (`own_here`, wave-uniform).
//
//   qp(h)        -> const T*  query vector of column h
//   ownp(r)      -> const T*  key (value) row of own candidate r
//   masked(h, r) -> bool      column h must not see own candidate r
//
// logit_pass writes the log2-domain logits l2[j][h] = scale2 * q_h . K[j] to e_lds[j * NH + h]
// (own candidate r is row nrows + r) and leaves per-lane running maxima in m (to be block-reduced).

template <typename T, int D, int NH, int UM = 2, bool COH = false, typename QPtr, typename OwnPtr, typename Mask>
__device__ __forceinline__ void logit_pass(const T* Kb, int nrows, int n_own, bool own_here, QPtr&& qp,
                                           OwnPtr&& ownp, Mask&& masked, float scale2, int lane, int wave,
                                           int nw, float* e_lds, float (&m)[NH]) {
  using E = Elem<T>;
  using Ge = Geo<T, D, NH>;
  constexpr int VEC = Ge::VEC, CK = Ge::CK, LK = Ge::LK, RK = Ge::RK, UK = Ge::UK;
#pragma unroll
  for (int h = 0; h < NH; ++h) m[h] = -INFINITY;
  if constexpr (Ge::MFMA_K) {
    // Matrix cores.  One v_mfma_f32_16x16x32_bf16 contracts 32 elements of d for 16 rows (A: lane l
    // holds row l % 16, eight consecutive elements) against 16 columns (B: lane l holds column
    // l % 16, the same eight elements; columns >= NH are zero); D / 32 of them cover a row.  Which
    // eight elements a lane holds is free as long as A and B agree: MFMA kk takes the 16-byte
    // chunk kk * 4 + l / 16, so the four lanes of a row load 64 contiguous bytes.  Result register
    // r of lane l is the logit of row (l / 16) * 4 + r for column l % 16.
    constexpr int KK = D / 32;  // (UM: 16-row tiles per register buffer)
    const int r16 = lane & 15, c4 = lane >> 4;
    V16 qm[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      qm[kk] = V16{{0u, 0u, 0u, 0u}};
      if (r16 < NH) qm[kk] = *reinterpret_cast<const V16*>(qp(r16) + (kk * 4 + c4) * 8);
    }
    float mh = -INFINITY;  // running maximum of column r16 over the rows this lane sees
    auto load_tile = [&](V16(&dst)[UM][KK], int base) {
#pragma unroll
      for (int u = 0; u < UM; ++u) {
        const int j = base + u * 16 + r16;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) dst[u][kk] = V16{{0u, 0u, 0u, 0u}};
        if (j < nrows) {
          const T* row = Kb + (size_t)j * D;
#pragma unroll
          for (int kk = 0; kk < KK; ++kk) dst[u][kk] = ld_v16<COH>(row + (kk * 4 + c4) * 8);
        }
      }
    };
    // rows row0 .. row0 + 15 of the candidate list; `own`: they are own candidates 0 .. 15
    auto logits16 = [&](const V16(&a)[KK], int row0, int nvalid, bool own) {
      f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a[kk]),
                                                      __builtin_bit_cast(bf16x8_t, qm[kk]), acc, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int j = row0 + c4 * 4 + r;
        float l2 = acc[r] * scale2;
        if (own && masked(r16, c4 * 4 + r)) l2 = -INFINITY;
        if (r16 < NH && j < nvalid) {
          mh = fmaxf(mh, l2);
          e_lds[j * NH + r16] = l2;
        }
      }
    };
    constexpr int TILE = 16 * UM;
    const int stride = nw * TILE;
    int base = wave * TILE;
    V16 bufA[UM][KK], bufB[UM][KK];
    V16 kn[KK];
    if (own_here) {  // the own candidates as rows 0 .. n_own - 1 of an otherwise empty tile
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        kn[kk] = V16{{0u, 0u, 0u, 0u}};
        if (r16 < n_own) kn[kk] = *reinterpret_cast<const V16*>(ownp(r16) + (kk * 4 + c4) * 8);
      }
    }
    load_tile(bufA, base);
    if (own_here) logits16(kn, nrows, nrows + n_own, true);
    while (base < nrows) {  // two register buffers: the next tile is in flight while this one is used
      load_tile(bufB, base + stride);
#pragma unroll
      for (int u = 0; u < UM; ++u) logits16(bufA[u], base + u * 16, nrows, false);
      base += stride;
      if (base >= nrows) break;
      load_tile(bufA, base + stride);
#pragma unroll
      for (int u = 0; u < UM; ++u) logits16(bufB[u], base + u * 16, nrows, false);
      base += stride;
    }
#pragma unroll
    for (int h = 0; h < NH; ++h) m[h] = (h == r16) ? mh : -INFINITY;
  } else {
    // Vector ALUs.  LK adjacent lanes share a row, each holding CK 16-byte chunks of it (chunk
    // c * LK + lane), so a wave-level load covers whole contiguous rows and the cross-lane sum per
    // (row, column) needs log2(LK) DPP steps.
    const int lk = lane % LK;  // position inside the row
    const int rk = lane / LK;  // which of the RK rows of a wave pass
    V16 qf[NH][CK];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const T* qh = qp(h);
#pragma unroll
      for (int c = 0; c < CK; ++c) qf[h][c] = *reinterpret_cast<const V16*>(qh + (c * LK + lk) * VEC);
    }
    auto load_tile = [&](V16(&dst)[UK][CK], int base) {
#pragma unroll
      for (int u = 0; u < UK; ++u) {
        const int j = base + u * RK + rk;
#pragma unroll
        for (int c = 0; c < CK; ++c) dst[u][c] = V16{{0u, 0u, 0u, 0u}};
        if (j < nrows) {
          const T* row = Kb + (size_t)j * D;
#pragma unroll
          for (int c = 0; c < CK; ++c) dst[u][c] = ld_v16<COH>(row + (c * LK + lk) * VEC);
        }
      }
    };
    auto logits_of = [&](const V16(&row)[CK], float(&l2)[NH]) {
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        float a = 0.f;
#pragma unroll
        for (int c = 0; c < CK; ++c) a = E::dot(row[c], qf[h][c], a);
        l2[h] = group_sum<LK>(a) * scale2;
      }
    };
    auto compute_tile = [&](const V16(&src)[UK][CK], int base) {
#pragma unroll
      for (int u = 0; u < UK; ++u) {
        const int j = base + u * RK + rk;
        float l2[NH];
        logits_of(src[u], l2);
        if (j < nrows) {
#pragma unroll
          for (int h = 0; h < NH; ++h) m[h] = fmaxf(m[h], l2[h]);  // running max, per lane
          if (lk == 0) {
#pragma unroll
            for (int h = 0; h < NH; ++h) e_lds[j * NH + h] = l2[h];
          }
        }
      }
    };
    constexpr int TILE = RK * UK;  // rows per wave per buffer
    const int stride = nw * TILE;
    int base = wave * TILE;
    V16 bufA[UK][CK], bufB[UK][CK];
    load_tile(bufA, base);
    if (own_here) {
      for (int r = 0; r < n_own; ++r) {
        V16 kn[CK];
        const T* kr = ownp(r);
#pragma unroll
        for (int c = 0; c < CK; ++c) kn[c] = *reinterpret_cast<const V16*>(kr + (c * LK + lk) * VEC);
        float l2[NH];
        logits_of(kn, l2);
#pragma unroll
        for (int h = 0; h < NH; ++h) {
          if (masked(h, r)) l2[h] = -INFINITY;
          m[h] = fmaxf(m[h], l2[h]);
        }
        if (lane == 0) {
#pragma unroll
          for (int h = 0; h < NH; ++h) e_lds[(nrows + r) * NH + h] = l2[h];
        }
      }
    }
    while (base < nrows) {  // two register buffers: the next tile is in flight while this one is used
      load_tile(bufB, base + stride);
      compute_tile(bufA, base);
      base += stride;
      if (base >= nrows) break;
      load_tile(bufA, base + stride);
      compute_tile(bufB, base);
      base += stride;
    }
  }
}

// PV pass: acc[h][v] += sum_j w[j][col0 + h] * V[j][...] over the cached rows and the own candidates,
// weights read from e_lds (stride NHT columns per candidate).  One 16-byte chunk of a row per lane
// (LV lanes per row, RV rows per wave-level load); the caller requests the first tile early with
// pv_first_tile (so that the V stream is in flight during the softmax barriers) and combines the RV
// row groups and the waves afterwards.
template <typename T, int D, int NH, bool COH = false, int UVN>
__device__ __forceinline__ void pv_first_tile(V16 (&vA)[UVN], const T* Vb, int nrows, int lane, int wave) {
  using Ge = Geo<T, D, NH>;
  constexpr int VEC = Ge::VEC, LV = Ge::LV, RV = Ge::RV, UV = UVN;  // (rows per lane and buffer: the caller's choice)
  const int lv = lane % LV, rv = lane / LV;
  const int base = wave * RV * UV;
#pragma unroll
  for (int u = 0; u < UV; ++u) {
    const int j = base + u * RV + rv;
    vA[u] = V16{{0u, 0u, 0u, 0u}};
    if (j < nrows) vA[u] = ld_v16<COH>(Vb + (size_t)j * D + lv * VEC);
  }
}
template <typename T, int D, int NH, bool COH = false, typename OwnPtr, int UVN, int VECN>
__device__ __forceinline__ void pv_pass(const T* Vb, int nrows, int n_own, bool own_here, OwnPtr&& ownp,
                                        const float* e_lds, int NHT, int col0, int lane, int wave, int nw,
                                        V16 (&vA)[UVN], float (&acc)[NH][VECN]) {
  using E = Elem<T>;
  using Ge = Geo<T, D, NH>;
  constexpr int VEC = Ge::VEC, LV = Ge::LV, RV = Ge::RV, UV = UVN;
  static_assert(VECN == VEC, "tile shape");
  const int lv = lane % LV, rv = lane / LV;
  constexpr int TILEV = RV * UV;
  const int stridev = nw * TILEV;
  auto load_vtile = [&](V16(&dst)[UV], int base) {
#pragma unroll
    for (int u = 0; u < UV; ++u) {
      const int j = base + u * RV + rv;
      dst[u] = V16{{0u, 0u, 0u, 0u}};
      if (j < nrows) dst[u] = ld_v16<COH>(Vb + (size_t)j * D + lv * VEC);
    }
  };
  auto accumulate = [&](const V16& row, const float(&w)[NH]) {
    float vf[VEC];
    E::unpack(row, vf);
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
      for (int v = 0; v < VEC; ++v) acc[h][v] = fmaf(w[h], vf[v], acc[h][v]);
  };
  auto compute_vtile = [&](const V16(&src)[UV], int base) {
#pragma unroll
    for (int u = 0; u < UV; ++u) {
      const int j = base + u * RV + rv;
      float w[NH];
#pragma unroll
      for (int h = 0; h < NH; ++h) w[h] = (j < nrows) ? e_lds[j * NHT + col0 + h] : 0.f;
      accumulate(src[u], w);
    }
  };
#pragma unroll
  for (int h = 0; h < NH; ++h)
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[h][v] = 0.f;
  if (own_here) {  // the own candidates' value rows (first row group of the wave only)
    for (int r = 0; r < n_own; ++r) {
      const V16 vn = *reinterpret_cast<const V16*>(ownp(r) + lv * VEC);
      float w[NH];
#pragma unroll
      for (int h = 0; h < NH; ++h) w[h] = (rv == 0) ? e_lds[(nrows + r) * NHT + col0 + h] : 0.f;
      accumulate(vn, w);
    }
  }
  V16 vB[UV];
  int basev = wave * TILEV;
  while (basev < nrows) {
    load_vtile(vB, basev + stridev);
    compute_vtile(vA, basev);
    basev += stridev;
    if (basev >= nrows) break;
    load_vtile(vA, basev + stridev);
    compute_vtile(vB, basev);
    basev += stridev;
  }
}

// PV pass on the matrix cores (bf16, d = 128, NH = 8 or 4 columns per streamed row; with 4, rows 4 .. 7
// and 12 .. 15 of the weight operand stay zero).  With V stored row by row the
// contraction index (the slot) is not contiguous in memory, but it can be made contiguous in a
// lane's registers without any cross-lane traffic: lane l takes the SAME 16-byte column chunk
// (l % 16) of eight DIFFERENT rows (tile row (l / 16) * 8 + i for load i), so a wave-level load
// still covers four whole contiguous rows and the eight loads of a tile cover 32 adjacent rows.
// Column c of the chunk, taken from the eight loaded registers with four byte permutes, is then
// the B operand (column l % 16, contraction elements (l / 16) * 8 + i) of
// v_mfma_f32_16x16x32_bf16 number c of the tile.  The A operand holds the weights: row m < 8 the
// upper 16 bits of head m's exp value as a bf16, row m + 8 the bf16 of what that leaves (the
// remainder is exact in fp32), so the two halves of the result add up to a product with a 16-bit
// weight mantissa -- the rows that would be zero padding with 8 heads carry the correction instead.
// Result register r of acc[c] in lane l: head (l / 16) * 4 + r (lanes >= 32: its correction), column
// 8 * (l % 16) + c.  The vector version of this pass needs 8 * NH multiply-adds per 16 bytes and
// lane and is bound by them; this one needs four permutes and one matrix instruction.
// (-DTOVA_PV_VECTOR builds the library with this pass on the vector ALUs everywhere: the A/B of the profiles)
template <typename T, int D, int NH>
struct PvMfma {
#ifdef TOVA_PV_VECTOR
  static constexpr bool OK = false;
#else
  static constexpr bool OK = Geo<T, D, NH>::MFMA_K && D == 128 && (NH == 8 || NH == 4);
#endif
  static constexpr int ROWS = 32;  // rows of a wave's tile
};
template <typename T, int D, bool COH = false>
__device__ __forceinline__ void pv_mfma_load(V16 (&vt)[8], const T* Vb, int base, int nrows, int lane) {
  const int n16 = lane & 15, kg = lane >> 4;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int j = base + kg * 8 + i;
    vt[i] = V16{{0u, 0u, 0u, 0u}};
    if (j < nrows) vt[i] = ld_v16<COH>(Vb + (size_t)j * D + n16 * 8);
  }
}
template <typename T, int D, int NH, bool COH = false>
__device__ __forceinline__ void pv_pass_mfma(const T* Vb, int nrows, const float* e_lds, int NHT, int col0,
                                             int lane, int wave, int nw, V16 (&vA)[8], f32x4_t (&acc)[8]) {
  static_assert(PvMfma<T, D, NH>::OK, "shape");
  const int kg = lane >> 4, h = lane & 7;
  const bool corr = (lane & 8) != 0;  // this lane's A row is a correction row
  constexpr int TILE = PvMfma<T, D, NH>::ROWS;
  const int stride = nw * TILE;
  auto compute = [&](const V16(&vt)[8], int base) {
    uint32_t w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int j = base + kg * 8 + i;
      const float e = (j < nrows && h < NH) ? e_lds[j * NHT + col0 + h] : 0.f;  // (NH = 4: half the rows stay zero)
      const uint32_t hi = __float_as_uint(e) & 0xffff0000u;
      w[i] = corr ? __float_as_uint(e - __uint_as_float(hi)) : hi;
    }
    V16 a;
#pragma unroll
    for (int r = 0; r < 4; ++r) a.w[r] = (w[2 * r] >> 16) | (w[2 * r + 1] & 0xffff0000u);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      V16 b;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t x = vt[2 * r].w[c >> 1], y = vt[2 * r + 1].w[c >> 1];
        b.w[r] = (c & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
      }
      acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), acc[c], 0, 0, 0);
    }
  };
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  V16 vB[8];
  int base = wave * TILE;
  while (base < nrows) {
    pv_mfma_load<T, D, COH>(vB, Vb, base + stride, nrows, lane);
    compute(vA, base);
    base += stride;
    if (base >= nrows) break;
    pv_mfma_load<T, D, COH>(vA, Vb, base + stride, nrows, lane);
    compute(vB, base);
    base += stride;
  }
}

// Completes pv_pass_mfma.  Lanes l and l ^ 32 hold the two halves of the same sums: one row swap between
// the registers of columns c and c + 4 and one addition complete both, columns 0 .. 3 in the lower 32
// lanes and 4 .. 7 in the upper ones (pv_mfma_fold).  The own candidates' rows are added on the vector
// ALUs, in fp32, by the wave that has them.  pv_mfma_store then puts the wave's sums at
// red[(wave * NH + head) * D + column]; between the two the caller places the barrier after which the
// reduction area may reuse the memory of the exp values.  pv_mfma_finish is the three in a row, for
// callers all of whose waves take part.
template <typename T, int D, int NH, typename OwnPtr>
__device__ __forceinline__ void pv_mfma_fold(f32x4_t (&pacc)[8], float (&tot)[4][4], int nrows, int n_own, bool own_here,
                                             OwnPtr&& ownp, const float* e_lds, int NHT, int col0, int lane) {
  static_assert(PvMfma<T, D, NH>::OK, "shape");
  // (the row swaps are inline assembly: the compiler does not see that they read the results of matrix
  // instructions, so the wait states between the two are spelled out here, once, on all accumulators)
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3"
               : "+v"(pacc[0]), "+v"(pacc[1]), "+v"(pacc[2]), "+v"(pacc[3]), "+v"(pacc[4]), "+v"(pacc[5]),
                 "+v"(pacc[6]), "+v"(pacc[7]));
  // tot[c % 4][r]: head ((lane >> 4) & 1) * 4 + r, column 8 * (lane & 15) + (lane >> 5) * 4 + c % 4
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float xf = pacc[c][r], yf = pacc[c + 4][r];  // (copies: a bit cast straight from a vector element reads element 0)
      unsigned x = __float_as_uint(xf), y = __float_as_uint(yf);
      swap_rows32(x, y);
      tot[c][r] = __uint_as_float(x) + __uint_as_float(y);
    }
  const int hb = ((lane >> 4) & 1) * 4, cb = (lane & 15) * 8 + (lane >> 5) * 4;
  if (own_here && hb < NH) {  // (NH = 4: lanes 16 .. 31 and 48 .. 63 hold padding)
    for (int o = 0; o < n_own; ++o) {
      const uint2 vn = *reinterpret_cast<const uint2*>(ownp(o) + cb);
      const float vf[4] = {__uint_as_float(vn.x << 16), __uint_as_float(vn.x & 0xffff0000u),
                           __uint_as_float(vn.y << 16), __uint_as_float(vn.y & 0xffff0000u)};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float w = e_lds[(nrows + o) * NHT + col0 + hb + r];
#pragma unroll
        for (int c = 0; c < 4; ++c) tot[c][r] = fmaf(w, vf[c], tot[c][r]);
      }
    }
  }
}
template <typename T, int D, int NH>
__device__ __forceinline__ void pv_mfma_store(const float (&tot)[4][4], int lane, int wave, float* red) {
  const int hb = ((lane >> 4) & 1) * 4, cb = (lane & 15) * 8 + (lane >> 5) * 4;
  if (hb < NH) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
      *reinterpret_cast<float4*>(red + (wave * NH + hb + r) * D + cb) = float4{tot[0][r], tot[1][r], tot[2][r], tot[3][r]};
  }
}
template <typename T, int D, int NH, typename OwnPtr>
__device__ __forceinline__ void pv_mfma_finish(f32x4_t (&pacc)[8], int nrows, int n_own, bool own_here, OwnPtr&& ownp,
                                               const float* e_lds, int NHT, int col0, int lane, int wave, float* red) {
  float tot[4][4];
  pv_mfma_fold<T, D, NH>(pacc, tot, nrows, n_own, own_here, ownp, e_lds, NHT, col0, lane);
  __syncthreads();  // everyone is done reading e_lds; the reduction area may reuse it
  pv_mfma_store<T, D, NH>(tot, lane, wave, red);
}

}  // namespace
}  // namespace tova
#endif  // TOVA_DEVICE_H
