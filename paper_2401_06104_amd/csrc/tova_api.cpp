// Host side of the C ABI declared in include/tova.h: argument validation, buffer layout,
// launch planning and the per-step launch loop.  No device code lives here.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "tova.h"
#include "tova_internal.h"

namespace {

constexpr size_t kAlign = 256;
constexpr int kTargetBlocks = 512;     // two workgroups per CU on 256 CUs
constexpr int kUnitModeUnits = 256;    // from one unit per CU on, a workgroup takes a whole unit
constexpr int kPrefillMinUnits = 256;   // fewest units for which prompt tokens are grouped (see resolve)
constexpr double kPrefillPartsMinBytes = 600e6;  // ... and the K + V bytes a step must stream for that to pay (see resolve)
constexpr int kPrefillMaxParts = 16;    // ... and, with fewer units, the most workgroups a unit's KV heads are dealt to
constexpr int kPrefillMaxGrid = 1024;  // workgroups of the multi-token kernel (each has a scratch area of its own)
constexpr size_t kMinBytesPerSplit = 256 * 1024;  // K+V bytes of a chunk below which splitting only adds
                                                  // hand-offs (each costs ~1 us of memory round trip)
constexpr int kSmallFloats = 512;      // must match the kernel's fixed LDS area
constexpr int kMaxLdsBytes = 64 * 1024;       // per workgroup when several share a CU
constexpr int kMaxLdsBytesUnit = 152 * 1024;  // a workgroup per unit may have a CU's LDS (160 KB) to itself

thread_local char g_hip_msg[256] = {0};

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Resolved {
  int L, B, k, H, H_kv, G, D, esize, bf16;
  int n_pinned, per_head;
  int policy, h2o_recent;  // TOVA_POLICY_*; H2O: tokens of the recent window, the incoming one included
  size_t acc_off;          // in state_mem: H2O's aggregated weights [units][k] (0 bytes for the other policies)
  int units, pairs, S, R, kp, NT, grid, lds, st_off, red_off, spin_limit, force_slow, persist_spin, multi_step, multi_grid, spin_env, svc;
  int unit_mode;  // one workgroup per unit instead of one per (unit, KV head, chunk)
  int pf_C, pf_NT, pf_lds, pf_e_floats, pf_ncp;  // multi-token kernel: tokens per group (0 = not available) and its LDS plan
  int pf_grid;                                   // ... its workgroups (decided in tova_cache_init)
  int pf_parts_max;                              // few units: at most this many workgroups per unit (0: a workgroup per unit only)
  size_t uscr_off, tpart_off, stat_off, gpos_off;
  float scale;
  size_t kv_bytes, state_bytes, scratch_bytes;
  size_t v_off;                                   // in kv_mem
  size_t occ_off, slot_off, err_off, tok_off;     // in state_mem
  size_t cnt_pair_off, cnt_unit_off, cnt_pub_off, slow_off, pstate_off, cnt_bytes;   // in scratch_mem
  size_t sg_off, escr_off, stats_off, accp_off;
};

int resolve(const tova_config_t* c, Resolved* r) {
  if (!c || !r) return TOVA_EINVAL;
  if (c->n_layers <= 0 || c->batch <= 0 || c->capacity_k <= 0 || c->n_q_heads <= 0 ||
      c->n_kv_heads <= 0 || c->head_dim <= 0 || c->n_splits < 0)
    return TOVA_EINVAL;
  if (c->n_q_heads % c->n_kv_heads != 0) return TOVA_EINVAL;
  if (c->dtype != TOVA_F32 && c->dtype != TOVA_BF16) return TOVA_EINVAL;
  if (!(c->softmax_scale == c->softmax_scale)) return TOVA_EINVAL;  // NaN
  if (c->n_pinned < 0 || c->n_pinned >= c->capacity_k) return TOVA_EINVAL;
  if (c->policy != TOVA_POLICY_TOVA && c->policy != TOVA_POLICY_WINDOW && c->policy != TOVA_POLICY_H2O) return TOVA_EINVAL;
  if (c->h2o_heavy < 0 || c->h2o_heavy >= c->capacity_k) return TOVA_EINVAL;
  if (c->policy == TOVA_POLICY_H2O && c->n_pinned != 0) return TOVA_EINVAL;
  if (c->policy != TOVA_POLICY_H2O && c->h2o_heavy != 0) return TOVA_EINVAL;
  const int G = c->n_q_heads / c->n_kv_heads;
  if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) return TOVA_ENOSUP;
  if (G != 1 && G != 2 && G != 4 && G != 8) return TOVA_ENOSUP;
  // index ranges the kernel keeps in 32 bits
  const long long units = (long long)c->n_layers * c->batch;
  const long long pairs = units * c->n_kv_heads;
  if (pairs > (1LL << 28) || c->capacity_k > (1 << 24) || units * c->n_q_heads > (1LL << 30))
    return TOVA_ENOSUP;

  r->L = c->n_layers; r->B = c->batch; r->k = c->capacity_k; r->H = c->n_q_heads;
  r->H_kv = c->n_kv_heads; r->G = G; r->D = c->head_dim;
  r->bf16 = (c->dtype == TOVA_BF16); r->esize = r->bf16 ? 2 : 4;
  r->units = (int)units; r->pairs = (int)pairs;
  r->n_pinned = c->n_pinned;
  r->per_head = (c->per_head != 0);
  r->policy = c->policy;
  // H2O (Sec. 4.1): h rows outside the window ("typically half of the multi-state size"), k - h inside
  r->h2o_recent = c->capacity_k - (c->h2o_heavy > 0 ? c->h2o_heavy : c->capacity_k / 2);
  if (r->per_head) {
    // TOVA-head is the same computation with every KV head as a unit of its own: q [L][B][H][d] is
    // [L*B*H_kv][G][d], K/V [L][B][H_kv][k][d] is [L*B*H_kv][1][k][d]; nothing else changes.
    r->units = (int)pairs;
    r->H = G;
    r->H_kv = 1;
  }
  r->scale = c->softmax_scale > 0.f ? c->softmax_scale : (float)(1.0 / std::sqrt((double)r->D));

  const int k = r->k;
  // groups whose passes run on the matrix cores (8 heads per KV head; 4 at bf16, d = 128): ~160 VGPRs, three
  // waves per SIMD, so workgroups of 256 threads, up to three to a CU
  const bool wide = G >= 8 || (r->bf16 && r->D == 128 && G == 4);
  int nt_env = 0;
  if (const char* e = std::getenv("TOVA_BLOCK_THREADS")) {  // tuning aid: 64..512, multiple of 64
    int v = std::atoi(e);
    if (v >= 64 && v <= 512 && v % 64 == 0) nt_env = v;
  }

  // ---- a workgroup per unit ----
  // With at least one unit per CU a workgroup takes a whole unit and goes through its KV heads one
  // after the other: the head-summed scores stay in LDS (a [k + 1] row behind the big area) and no
  // workgroup ever needs another one's results.  It needs one chunk per KV head, i.e. LDS for the
  // logits of all k + 1 candidates of a KV head's G query heads; for that it may take most of a
  // CU's LDS (one workgroup per CU is enough to stream at full rate in this form).
  r->unit_mode = 0;
  {
    int want = (r->units >= kUnitModeUnits);
    if (const char* e = std::getenv("TOVA_UNIT_MODE")) want = (std::atoi(e) != 0);  // tuning aid / test hook
    // the baseline policies pick their victim inside the workgroup that owns the unit (Window from the
    // slot -> token map, H2O from per-slot sums it alone updates): this form, whatever the unit count
    if (r->policy != TOVA_POLICY_TOVA) want = 1;
    if (want && (c->n_splits <= 1 || r->policy != TOVA_POLICY_TOVA)) {
      const long long e_fl = ((long long)(k + 1) * G + 3) / 4 * 4;
      const long long s_fl = ((long long)k + 1 + 3) / 4 * 4;
      int nt = nt_env ? nt_env : ((k >= 512 && !wide) ? 512 : 256);
      long long red_fl = (long long)(nt / 64) * G * r->D;
      long long st = e_fl > red_fl ? e_fl : red_fl;
      if ((kSmallFloats + st + s_fl) * 4 > kMaxLdsBytes && !nt_env) {  // alone on its CU: all the threads a block may have
        nt = 512;
        red_fl = (long long)(nt / 64) * G * r->D;
        st = e_fl > red_fl ? e_fl : red_fl;
      }
      if ((kSmallFloats + st + s_fl) * 4 <= kMaxLdsBytesUnit) {
        r->unit_mode = 1;
        r->S = 1; r->R = k; r->NT = nt; r->st_off = (int)st; r->red_off = 0;
        r->lds = (int)((kSmallFloats + st + s_fl) * 4);
      }
    }
  }

  if (r->policy != TOVA_POLICY_TOVA && !r->unit_mode) return TOVA_ENOSUP;  // (a KV head's logits do not fit LDS)

  // ---- groups of C prompt tokens per pass over the cache ----
  // C * G (token, head) combinations share a streamed row; the vector passes hold at most 8.  The
  // multi-token kernel has a plan of its own (a workgroup per unit, whatever form the single-token
  // steps take), so it can be used with fewer units than fill the device when it still pays.
  r->pf_C = 0;
  // Measured on MI355X (us per token, tova_decode_steps -> tova_prefill): one query head per KV head
  // (groups of 8 or 4 tokens) wins from 128 units on at k = 512 (x1.28; 192 units x1.89; 64 units x0.69)
  // and from 64 units on at k >= 1024 (x1.4-1.7); grouped heads (groups of 2) only once the units
  // fill the device (200 units x0.89).  Below that the workgroups of this form are too few.
  int pf_min_units = (G == 1) ? (k >= 1024 ? 64 : 128) : kPrefillMinUnits;
  if (const char* e = std::getenv("TOVA_PREFILL_MIN_UNITS")) {  // tuning aid / test hook
    const int v = std::atoi(e);
    if (v >= 1) pf_min_units = v;
  }
  // Fewer units than that: the KV heads of a unit are dealt to several workgroups (see tova_prefill.hip);
  // how many is decided in tova_cache_init, which can ask the device how many fit at once.
  // Measured (us per token, decode steps -> prompt with parts; 32 heads, d = 128, bf16): it pays once a
  // step streams enough for the one workgroup per unit that resolves a group not to be the bottleneck --
  // 32 units at k = 512 / 1024 / 1536 / 2048 / 4096: x0.47 / 0.92 / 1.55 / 1.98 / 2.49; 64 units at
  // k = 512 x1.02; 8 / 16 units at k = 4096 x1.03 / 1.71; 4 heads per KV head, k = 1024, 64 / 128 / 160
  // units: x0.69 / 1.15 / 1.22 -- i.e. from about 600 MB of K and V per step on.
  r->pf_parts_max = 0;
  if (!r->unit_mode && r->units < pf_min_units && r->H_kv >= 2) {
    const double step_bytes = 2.0 * (double)r->pairs * k * r->D * r->esize;
    const char* e = std::getenv("TOVA_PREFILL_PARTS");  // tuning aid / test hook: at most this many (1: never); given, it
    if (step_bytes >= kPrefillPartsMinBytes || e) {     // also lifts the size condition
      r->pf_parts_max = r->H_kv < kPrefillMaxParts ? r->H_kv : kPrefillMaxParts;
      if (e) {
        const int v = std::atoi(e);
        if (v >= 1 && v < r->pf_parts_max) r->pf_parts_max = v;
      }
      if (r->pf_parts_max < 2) r->pf_parts_max = 0;
    }
  }
  if ((r->unit_mode || r->units >= pf_min_units || r->pf_parts_max) && r->policy == TOVA_POLICY_TOVA) {
    const int cands[3] = {8, 4, 2};
    for (int ci = 0; ci < 3 && !r->pf_C; ++ci) {
      const int C = cands[ci], GE = G * C;
      const bool built = (G == 1 && (C == 4 || C == 8)) || (G == 2 && (C == 2 || C == 4)) || (G == 4 && C == 2);
      if (!built) continue;
      // The corrections subtract what the group's earlier tokens removed from sums over everything:
      // that keeps full precision only while the removed candidates carry a small part of the
      // weight, i.e. while a group is small against the multi-state.
      if (k < 8 * C) continue;
      // eight combinations need ~150 VGPRs (three waves per SIMD): workgroups of 256 threads, up to
      // three to a CU (measured better than fewer, larger ones) -- unless the LDS leaves room for
      // one workgroup only, which then has 512 threads
      const long long NC = (long long)k + C, ncp = (NC + 3) / 4 * 4;
      int nt = 0;
      long long e_fl = 0, tot = 0;
      for (int pass = 0; pass < 2; ++pass) {
        nt = nt_env ? nt_env : (GE < 8 ? (k >= 512 ? 512 : 256) : (pass == 0 ? 256 : 512));
        e_fl = NC * GE;
        if ((long long)(nt / 64) * GE * r->D > e_fl) e_fl = (long long)(nt / 64) * GE * r->D;
        if ((long long)r->H * r->D + NC > e_fl) e_fl = (long long)r->H * r->D + NC;
        e_fl = (e_fl + 3) / 4 * 4;
        tot = kSmallFloats + e_fl + C * ncp + 2LL * r->H * C + r->H + (long long)C * r->H;
        if (nt_env || GE < 8 || (160 * 1024) / (tot * 4) >= 2) break;
      }
      if (tot * 4 <= kMaxLdsBytesUnit) {
        r->pf_C = C; r->pf_NT = nt; r->pf_lds = (int)(tot * 4); r->pf_e_floats = (int)e_fl; r->pf_ncp = (int)ncp;
      }
    }
  }

  // ---- split count: enough workgroups to fill 256 CUs, chunks that fit LDS ----
  int S = c->n_splits;
  if (S <= 0) {
    int target = kTargetBlocks;
    if (const char* e = std::getenv("TOVA_TARGET_BLOCKS")) {  // tuning aid
      int v = std::atoi(e);
      if (v >= 1 && v <= (1 << 20)) target = v;
    }
    S = (r->pairs >= target) ? 1 : (target + r->pairs - 1) / r->pairs;
    const size_t pair_bytes = 2 * (size_t)k * r->D * r->esize;  // K + V of one KV head
    int smax = (int)(pair_bytes / kMinBytesPerSplit);
    if (smax < 1) smax = 1;
    if (S > smax) S = smax;
  }
  if (S > k) S = k;
  const int big_cap = kMaxLdsBytes / 4 - kSmallFloats;  // floats available for the big LDS area
  // LDS: logits / exp values of R slots + the new token; the cross-wave reduction area reuses that
  // memory after the PV pass; with several chunks per KV head a small area behind both holds all
  // chunks' softmax statistics and the finisher's merge weights.
  int R = (k + S - 1) / S, NT = 0;
  long long big = 0, st_off = 0, red_off = 0;
  for (; !r->unit_mode;) {
    S = (k + R - 1) / R;  // no dead chunks
    const long long e_fl = ((long long)(R + 1) * G + 3) / 4 * 4;
    bool ok = false;
    // wide groups need ~150 VGPRs: three waves per SIMD, i.e. three 256-thread blocks per CU but only
    // one 512-thread block
    const int cand[2] = {nt_env ? nt_env : ((R >= 512 && !wide) ? 512 : 256), 256};
    for (int ci = 0; ci < 2 && !ok; ++ci) {
      NT = cand[ci];
      const long long red_fl = (long long)(NT / 64) * G * r->D;
      // several chunks per KV head: the exp values are needed again after the PV pass (the chunk's score
      // rows wait for the siblings' statistics until then), so the reduction area sits behind them
      st_off = (S > 1) ? e_fl + red_fl : (e_fl > red_fl ? e_fl : red_fl);
      red_off = (S > 1) ? e_fl : 0;
      big = st_off + (S > 1 ? 3LL * S * G + 2LL * G : 0);
      ok = (big <= big_cap);
    }
    if (ok) break;
    if (R == 1) return TOVA_ENOSUP;
    R -= (R >= 8) ? R / 8 : 1;  // smaller chunks until the chunk fits
  }
  if (!r->unit_mode) {
    r->S = S; r->R = R; r->NT = NT; r->st_off = (int)st_off; r->red_off = (int)red_off;
    r->lds = (int)((kSmallFloats + big) * 4);
  }
  S = r->S;
  r->kp = (int)round_up((size_t)k + 1, 64);
  r->grid = r->unit_mode ? r->units : (r->pairs + 7) / 8 * 8 * S;
  // A chunk looks this many more times (about a microsecond apart) for its siblings' statistics
  // before it leaves its score rows to the pair's finisher.  Only worth it when all workgroups of
  // the grid are resident at once: tova_cache_init asks the device and clears it otherwise.
  r->spin_limit = 24;
  r->spin_env = 0;
  if (const char* e = std::getenv("TOVA_SPIN_LIMIT")) {  // tuning aid / test hook
    int v = std::atoi(e);
    if (v >= 0 && v <= 4096) { r->spin_limit = v; r->spin_env = 1; }
  }
  r->force_slow = 0;
  if (const char* e = std::getenv("TOVA_FORCE_SLOW_MERGE")) r->force_slow = (std::atoi(e) != 0);  // test hook
  // multi-step launches (decided for good in tova_cache_init, which can ask the device)
  r->multi_step = 1;
  if (const char* e = std::getenv("TOVA_MULTI_STEP")) r->multi_step = r->multi_step && (std::atoi(e) != 0);
  // Service wave (multi-step launches of the hand-off form; see the step kernel): the last wave of a workgroup
  // serves the hand-off -- score rows, arrival, and for the unit's last arrival the scan and the victim -- beside
  // the PV pass instead of behind it.  Measured on MI355X (us per step, without -> with): it pays for one chunk
  // per KV head with the 256-thread workgroups of the matrix-core passes while the unit's score rows are small
  // enough for one wave to scan (GQA 32/8: k = 512 20.8 -> 19.7, k = 1024 36.9 -> 35.6, k = 2048 91.0 -> 91.0;
  // 16/4 x 128 sequences 36.6 -> 36.3), and costs where a wave is a larger share of the PV pass's loads in
  // flight or the rows are many (32 heads MHA x 32 layers, k = 512: 42.3 -> 45.6; one layer: 13.0 -> 16.3;
  // GQA 32/16 90.5 -> 92.5; split cache, config 5: 44.6 -> 51.0).  8 heads per KV head: 32/4 x 128 units at
  // k = 256 / 512 / 768 / 1024 17.4 -> 16.6 / 21.7 -> 20.3 / 29.3 -> 26.9 / 36.8 -> 37.3, x 192 units at k = 1024
  // 70.2 -> 63.5, 64/8 x 64 units at k = 512 / 1024 22.2 -> 20.4 / 37.5 -> 36.5: on.
  r->svc = (!r->unit_mode && r->S == 1 && r->bf16 && r->D == 128 && (G == 4 || G == 8) &&
            (long long)r->H_kv * (k + 1) <= 12 * 1024) ? 1 : 0;
  if (const char* e = std::getenv("TOVA_SERVICE_WAVE")) r->svc = (std::atoi(e) != 0);  // tuning aid / test hook
  r->persist_spin = 1 << 22;  // polls of ~0.2 us or more each: seconds, i.e. "something is broken"
  if (const char* e = std::getenv("TOVA_MULTI_STEP_SPIN")) {  // test hook: make the wait run out
    int v = std::atoi(e);
    if (v >= 0) r->persist_spin = v;
  }

  // ---- caller-owned buffers ----
  const size_t kv_one = (size_t)r->pairs * k * r->D * r->esize;
  r->v_off = kv_one;
  r->kv_bytes = 2 * kv_one;
  r->occ_off = 0;
  r->slot_off = round_up((size_t)r->units * 4, kAlign);
  r->err_off = r->slot_off + round_up((size_t)r->units * k * 4, kAlign);
  r->tok_off = r->err_off + 64;  // (same 256-byte block as the error flag)
  r->acc_off = r->err_off + kAlign;
  r->state_bytes = r->acc_off + (r->policy == TOVA_POLICY_H2O ? round_up((size_t)r->units * k * 4, kAlign) : 0);

  size_t off = 0;
  r->cnt_pair_off = off; off += round_up((size_t)r->pairs * 2 * 4, kAlign);  // (two copies, by token parity)
  r->cnt_unit_off = off; off += round_up((size_t)r->units * 2 * 4, kAlign);  // (two copies in the step kernel; the others use the first)
  r->cnt_pub_off = off; off += round_up((size_t)r->pairs * 2 * 4, kAlign);
  r->slow_off = off; off += round_up((size_t)r->pairs * S * 4, kAlign);
  r->pstate_off = off; off += round_up((size_t)r->units * 8, kAlign);
  r->cnt_bytes = off;
  r->sg_off = off;
  if (!r->unit_mode) off += round_up((size_t)r->pairs * r->kp * 4, kAlign);  // (a workgroup per unit keeps the scores in LDS)
  r->escr_off = r->stats_off = r->accp_off = off;
  if (S > 1) {
    r->escr_off = off; off += round_up((size_t)r->pairs * r->kp * G * 4, kAlign);
    r->stats_off = off; off += round_up((size_t)r->pairs * S * G * 2 * 4, kAlign);
    r->accp_off = off; off += 2 * round_up((size_t)r->pairs * S * G * r->D * 4, kAlign);  // two parity copies
  }
  r->uscr_off = off;
  if (r->pf_C) {
    const size_t blocks = (size_t)(r->units < kPrefillMaxGrid ? r->units : kPrefillMaxGrid);
    off += round_up(blocks * r->H * r->pf_C * r->D * 4, kAlign);
  }
  r->tpart_off = r->stat_off = r->gpos_off = off;
  if (r->pf_C && r->pf_parts_max) {  // what the parts of a unit hand to the one that resolves a group
    r->tpart_off = off; off += round_up((size_t)r->units * r->pf_parts_max * r->pf_C * r->pf_ncp * 4, kAlign);
    r->stat_off = off; off += round_up((size_t)r->units * r->H * r->pf_C * 2 * 4, kAlign);
    r->gpos_off = off; off += round_up((size_t)r->units * 8 * 4, kAlign);
  }
  r->scratch_bytes = off;
  return TOVA_OK;
}

int hip_fail(hipError_t e, const char* what) {
  std::snprintf(g_hip_msg, sizeof g_hip_msg, "%s: %s", what, hipGetErrorString(e));
  return TOVA_EHIP;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace

struct tova_cache {
  Resolved r;
  char* kv;
  char* state;
  char* scratch;
  int64_t t;  // tokens seen
  // environment hooks, read once in tova_cache_init
  int prefill_group_off;  // TOVA_PREFILL_GROUP=0: prompts go token by token
  int pf_parts;           // workgroups per unit of the multi-token kernel: 1, or (few units) >= 2; 0: no grouping
  int prefill_exact;      // TOVA_PREFILL_EXACT=1: test hook, every grouped token takes the guard's from-scratch route
  int repos_threads;      // TOVA_REPOS_THREADS (0: the plan's own choice)
  int repos_parts;        // TOVA_REPOS_PARTS (0: no limit given)
};

extern "C" {

int tova_cache_bytes(const tova_config_t* cfg, size_t* kv_bytes, size_t* state_bytes,
                     size_t* scratch_bytes) {
  Resolved r;
  int rc = resolve(cfg, &r);
  if (rc != TOVA_OK) return rc;
  if (kv_bytes) *kv_bytes = r.kv_bytes;
  if (state_bytes) *state_bytes = r.state_bytes;
  if (scratch_bytes) *scratch_bytes = r.scratch_bytes;
  return TOVA_OK;
}

int tova_cache_layout(const tova_config_t* cfg, tova_layout_t* layout) {
  if (!layout) return TOVA_EINVAL;
  Resolved r;
  int rc = resolve(cfg, &r);
  if (rc != TOVA_OK) return rc;
  layout->k_offset = 0;
  layout->v_offset = r.v_off;
  layout->occupancy_offset = r.occ_off;
  layout->slot_token_offset = r.slot_off;
  layout->error_flag_offset = r.err_off;
  layout->n_splits = r.S;
  layout->rows_per_split = r.R;
  layout->block_threads = r.NT;
  layout->grid_blocks = r.grid;
  layout->lds_bytes = r.lds;
  layout->unit_workgroups = r.unit_mode;
  layout->service_wave = (!r.unit_mode && r.svc && r.NT >= 128) ? 1 : 0;
  layout->prefill_group = r.pf_C;
  layout->h2o_acc_offset = r.acc_off;
  layout->tokens_seen_offset = r.tok_off;
  return TOVA_OK;
}

int tova_cache_init(tova_cache_t** out, const tova_config_t* cfg, void* kv_mem, void* state_mem,
                    void* scratch_mem, void* hip_stream) {
  if (!out) return TOVA_EINVAL;
  *out = nullptr;
  Resolved r;
  int rc = resolve(cfg, &r);
  if (rc != TOVA_OK) return rc;
  if (!kv_mem || !state_mem) return TOVA_EINVAL;  // (scratch_mem may be null: see tova_decode_steps_static)
  if (!aligned(kv_mem, kAlign) || !aligned(state_mem, kAlign) || !aligned(scratch_mem, kAlign))
    return TOVA_EINVAL;
  tova_cache* c = new (std::nothrow) tova_cache;
  if (!c) return TOVA_ENOMEM;
  c->r = r;
  c->kv = static_cast<char*>(kv_mem);
  c->state = static_cast<char*>(state_mem);
  c->scratch = static_cast<char*>(scratch_mem);
  c->t = 0;
  c->prefill_group_off = 0;
  if (const char* e = std::getenv("TOVA_PREFILL_GROUP")) c->prefill_group_off = (std::atoi(e) == 0);  // test hook
  c->prefill_exact = 0;
  if (const char* e = std::getenv("TOVA_PREFILL_EXACT")) c->prefill_exact = (std::atoi(e) != 0);  // test hook
  c->repos_threads = 0;
  if (const char* e = std::getenv("TOVA_REPOS_THREADS")) {  // tuning aid
    const int v = std::atoi(e);
    if (v >= 64 && v <= 512 && v % 64 == 0) c->repos_threads = v;
  }
  c->repos_parts = 0;
  if (const char* e = std::getenv("TOVA_REPOS_PARTS")) {  // tuning aid / test hook: at most this many parts
    const int v = std::atoi(e);
    if (v >= 1) c->repos_parts = v;
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // fill kernels, not memsets, so that the call can be recorded into a HIP graph
  hipError_t e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(c->state + r.occ_off), 0,
                                       (size_t)r.units, s);
  if (e == hipSuccess)
    e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(c->state + r.slot_off), -1,
                              (size_t)r.units * r.k, s);
  if (e == hipSuccess && c->scratch)
    e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(c->scratch), 0, r.cnt_bytes / 4, s);
  if (e == hipSuccess)
    e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(c->state + r.err_off), 0, 1, s);
  if (e == hipSuccess)
    e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(c->state + r.tok_off), 0, 1, s);
  if (e == hipSuccess && r.policy == TOVA_POLICY_H2O)  // (0.0f is the all-zero word)
    e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(c->state + r.acc_off), 0, (size_t)r.units * r.k, s);
  // A multi-step launch needs all its blocks resident at once (blocks of a unit wait for each
  // other's results): its grid is capped at what the device can hold, and each block then walks
  // several (unit, KV head) pairs per step.
  c->r.multi_grid = 0;
  const int cap = tova::resident_blocks(r.bf16, r.D, r.G, r.NT, r.lds, r.unit_mode ? 1 : (r.svc && r.NT >= 128 ? 2 : 0)) / 8 * 8;
  if (!r.spin_env && r.grid > cap) c->r.spin_limit = 0;
  if (r.unit_mode) {
    // every launch walks the units with a grid that just fills the device (nothing waits for
    // anything, so this is a matter of efficiency only)
    // Measured on MI355X: with one query head per KV head one workgroup per CU streams best (the
    // fewer concurrent streams, the better for HBM); wider groups have more arithmetic per byte
    // to hide and want two.
    const int cus = tova::device_cus();
    int want = cus > 0 ? cus * (r.G >= 4 ? 2 : 1) : r.grid;
    if (cap >= 8 && want > cap) want = cap;
    c->r.multi_grid = want < r.grid ? want : r.grid;
    if (const char* e = std::getenv("TOVA_UNIT_GRID")) {  // tuning aid
      const int v = std::atoi(e);
      if (v >= 1 && v <= r.grid) c->r.multi_grid = v;
    }
  } else if (c->r.multi_step) {
    int want = r.grid;
    if (const char* ev = std::getenv("TOVA_MULTI_GRID")) {  // tuning aid: fewer workgroups, several items each per step
      const int v = std::atoi(ev) / 8 * 8;
      if (v >= 8 && v < want) want = v;
    }
    c->r.multi_grid = want < cap ? want : cap;   // never more blocks than fit at once
    if (c->r.multi_grid < 8) c->r.multi_step = 0;
  }
  c->r.pf_grid = 0;
  if (r.pf_C) {
    // workgroups of the multi-token kernel: as many per CU as its LDS and registers allow (measured:
    // 256-thread workgroups, three per CU, for eight combinations; else two of 512), never more than
    // have a scratch area
    const int cus = tova::device_cus();
    int per_cu = (160 * 1024) / r.pf_lds;
    const int cap_cu = (r.G * r.pf_C >= 8) ? 3 : 2;
    if (per_cu > cap_cu) per_cu = cap_cu;
    if (per_cu < 1) per_cu = 1;
    int g = cus > 0 ? cus * per_cu : r.units;
    if (const char* ev = std::getenv("TOVA_UNIT_GRID")) {  // tuning aid
      const int v = std::atoi(ev);
      if (v >= 1) g = v;
    }
    if (g > kPrefillMaxGrid) g = kPrefillMaxGrid;
    if (g > r.units) g = r.units;
    c->r.pf_grid = g;
  }
  c->pf_parts = r.pf_C ? 1 : 0;
  if (r.pf_C && r.pf_parts_max) {
    // few units: as many workgroups per unit as divide the KV heads and are all resident (the parts of
    // a unit wait for the one that resolves a group)
    const int cap = tova::prefill_resident_blocks(r.bf16, r.D, r.G, r.pf_C, r.pf_NT, r.pf_lds);
    c->pf_parts = 0;
    for (int pc = r.pf_parts_max; pc >= 2; --pc)
      if (r.H_kv % pc == 0 && (long long)r.units * pc <= cap) {
        c->pf_parts = pc;
        break;
      }
  }
  if (e != hipSuccess) {
    delete c;
    return hip_fail(e, "tova_cache_init");
  }
  *out = c;
  return TOVA_OK;
}

int tova_prefill(tova_cache_t* c, int32_t n_tokens, const void* q, const void* k_new, const void* v_new,
                 void* out, int32_t* evicted, void* hip_stream) {
  if (!c || n_tokens < 0 || !c->scratch) return TOVA_EINVAL;
  if (n_tokens == 0) return TOVA_OK;
  if (!q || !k_new || !v_new || !out) return TOVA_EINVAL;
  if (!aligned(q, 16) || !aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(out, 16) || !aligned(evicted, 4))
    return TOVA_EINVAL;
  const Resolved& r = c->r;
  if (c->t + n_tokens > 0x7fffffffLL) return TOVA_ENOSUP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t q_step = (size_t)r.units * r.H * r.D * r.esize;
  const size_t kv_step = (size_t)r.pairs * r.D * r.esize;
  const int C = (c->prefill_group_off || c->pf_parts == 0) ? 0 : r.pf_C;
  const int parts = c->pf_parts > 1 ? c->pf_parts : 1;
  for (int32_t i = 0; i < n_tokens;) {
    const void* qi = static_cast<const char*>(q) + (size_t)i * q_step;
    const void* ki = static_cast<const char*>(k_new) + (size_t)i * kv_step;
    const void* vi = static_cast<const char*>(v_new) + (size_t)i * kv_step;
    void* oi = static_cast<char*>(out) + (size_t)i * q_step;
    int32_t* ei = evicted ? evicted + (size_t)i * r.units : nullptr;
    int32_t m = n_tokens - i;
    const bool filling = c->t < r.k;
    if (filling && m > r.k - c->t) m = (int32_t)(r.k - c->t);  // (App. B: nothing is removed while there is room)
    if (C >= 2 && m >= C) {
      const int32_t n_chunks = m / C;
      m = n_chunks * C;
      tova::PrefillParams p;
      p.q = qi; p.k_new = ki; p.v_new = vi; p.out = oi; p.evicted = ei;
      p.K = c->kv; p.V = c->kv + r.v_off;
      p.occupancy = reinterpret_cast<int32_t*>(c->state + r.occ_off);
      p.slot_token = reinterpret_cast<int32_t*>(c->state + r.slot_off);
      p.uscr = reinterpret_cast<float*>(c->scratch + r.uscr_off);
      p.filling = filling ? 1 : 0;
      p.n0 = (int32_t)(filling ? c->t : r.k);
      p.q_stride = (int64_t)(q_step / r.esize); p.kv_stride = (int64_t)(kv_step / r.esize);
      p.n_chunks = n_chunks; p.units = r.units; p.H = r.H; p.H_kv = r.H_kv; p.k = r.k;
      p.n_pinned = r.n_pinned; p.t = (int32_t)c->t; p.e_floats = r.pf_e_floats; p.ncp = r.pf_ncp; p.scale = r.scale;
      p.force_exact = c->prefill_exact;
      p.parts = parts;
      p.spin = r.persist_spin;
      p.tpart = reinterpret_cast<float*>(c->scratch + r.tpart_off);
      p.stat = reinterpret_cast<float*>(c->scratch + r.stat_off);
      p.gpos = reinterpret_cast<int32_t*>(c->scratch + r.gpos_off);
      p.cnt_unit = reinterpret_cast<int32_t*>(c->scratch + r.cnt_unit_off);
      p.pstate = reinterpret_cast<unsigned long long*>(c->scratch + r.pstate_off);
      p.error_flag = reinterpret_cast<int32_t*>(c->state + r.err_off);
      const tova::LaunchPlan lp{parts > 1 ? r.units * parts : r.pf_grid, r.pf_NT, r.pf_lds};
      hipError_t e = hipSuccess;
      if (parts > 1 && !filling)  // the units' group counters start from "no group resolved"
        e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(p.pstate), 0, (size_t)r.units * 2, s);
      if (e == hipSuccess) e = tova::launch_prefill(r.bf16, r.D, r.G, C, p, lp, s);
      if (e != hipSuccess) return hip_fail(e, "tova_prefill launch");
      c->t += m;
      i += m;
      continue;
    }
    const int rc = tova_decode_steps(c, m, qi, ki, vi, oi, ei, hip_stream);
    if (rc != TOVA_OK) return rc;
    i += m;
  }
  return TOVA_OK;
}

}  // extern "C"

namespace {

int check_step_args(const tova_cache* c, int32_t n_steps, const void* q, const void* k_new, const void* v_new,
                    const void* out, const int32_t* evicted) {
  if (!c || n_steps < 0) return TOVA_EINVAL;
  if (n_steps == 0) return TOVA_OK;
  if (!q || !k_new || !v_new || !out) return TOVA_EINVAL;
  if (!aligned(q, 16) || !aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(out, 16) ||
      !aligned(evicted, 4))
    return TOVA_EINVAL;
  if (c->t + n_steps > 0x7fffffffLL) return TOVA_ENOSUP;  // token index is kept in 32 bits
  return TOVA_OK;
}

// The launch loop of tova_decode_steps, over a scratch area that is either the caller's
// (scratch_mem of tova_cache_init) or the library's static one (tova_decode_steps_static).
// Arguments have been checked; n_steps >= 1.
int decode_steps_on(tova_cache* c, char* scratch, int32_t n_steps, const void* q, const void* k_new,
                    const void* v_new, void* out, int32_t* evicted, hipStream_t s, bool token_from_device = false) {
  const Resolved& r = c->r;

  const size_t q_step = (size_t)r.units * r.H * r.D * r.esize;
  const size_t kv_step = (size_t)r.pairs * r.D * r.esize;
  tova::StepParams p;
  p.K = c->kv;
  p.V = c->kv + r.v_off;
  p.occupancy = reinterpret_cast<int32_t*>(c->state + r.occ_off);
  p.slot_token = reinterpret_cast<int32_t*>(c->state + r.slot_off);
  p.cnt_pair = reinterpret_cast<int32_t*>(scratch + r.cnt_pair_off);
  p.cnt_unit = reinterpret_cast<int32_t*>(scratch + r.cnt_unit_off);
  p.cnt_pub = reinterpret_cast<int32_t*>(scratch + r.cnt_pub_off);
  p.slow_flag = reinterpret_cast<int32_t*>(scratch + r.slow_off);
  p.st_off = r.st_off; p.red_off = r.red_off; p.spin_limit = r.spin_limit; p.force_slow = r.force_slow;
  p.sg = reinterpret_cast<float*>(scratch + r.sg_off);
  p.escr = reinterpret_cast<float*>(scratch + r.escr_off);
  p.stats = reinterpret_cast<float*>(scratch + r.stats_off);
  p.accp = reinterpret_cast<float*>(scratch + r.accp_off);
  p.accp_half = (int64_t)(round_up((size_t)r.pairs * r.S * r.G * r.D * 4, kAlign) / 4);
  p.pairs = r.pairs; p.H = r.H; p.H_kv = r.H_kv; p.k = r.k; p.n_pinned = r.n_pinned;
  p.policy = r.policy; p.h2o_recent = r.h2o_recent;
  p.acc = reinterpret_cast<float*>(c->state + r.acc_off);
  p.S = r.S; p.R = r.R; p.kp = r.kp; p.scale = r.scale;
  const tova::LaunchPlan lp{r.grid, r.NT, r.lds};

  p.q_stride = (int64_t)(q_step / r.esize);
  p.kv_stride = (int64_t)(kv_step / r.esize);
  p.pstate = reinterpret_cast<unsigned long long*>(scratch + r.pstate_off);
  p.error_flag = reinterpret_cast<int32_t*>(c->state + r.err_off);
  p.persist_spin = r.persist_spin;

  for (int32_t i = 0; i < n_steps;) {
    p.q = static_cast<const char*>(q) + (size_t)i * q_step;
    p.k_new = static_cast<const char*>(k_new) + (size_t)i * kv_step;
    p.v_new = static_cast<const char*>(v_new) + (size_t)i * kv_step;
    p.out = static_cast<char*>(out) + (size_t)i * q_step;
    p.evicted = evicted ? evicted + (size_t)i * r.units : nullptr;
    p.n = (int32_t)(c->t < r.k ? c->t : r.k);
    p.t = token_from_device ? 0 : (int32_t)c->t;
    p.t_dev = token_from_device ? reinterpret_cast<const int32_t*>(c->state + r.tok_off) : nullptr;
    // all remaining steps in one launch once the cache is full (see tova.h)
    const int32_t m = (r.multi_step && c->t >= r.k && n_steps - i >= 2) ? n_steps - i : 1;
    p.n_iter = m;
    p.persistent = (m > 1);
    p.unit_mode = r.unit_mode;
    p.svc = (m > 1 && !r.unit_mode && r.svc && r.NT >= 128) ? 1 : 0;
    hipError_t e = hipSuccess;
    if (m > 1 && !r.unit_mode)  // the units' state words start from "no step finished"
      e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(p.pstate), 0, (size_t)r.units * 2, s);
    const tova::LaunchPlan lpm{r.multi_grid, r.NT, r.lds};
    if (e == hipSuccess) e = tova::launch_step(r.bf16, r.D, r.G, p, (m > 1 || r.unit_mode) ? lpm : lp, s);
    if (e != hipSuccess) return hip_fail(e, "tova_decode_step launch");
    c->t += m;
    i += m;
  }
  return TOVA_OK;
}

}  // namespace

extern "C" {

int tova_decode_steps(tova_cache_t* c, int32_t n_steps, const void* q, const void* k_new,
                      const void* v_new, void* out, int32_t* evicted, void* hip_stream) {
  const int rc = check_step_args(c, n_steps, q, k_new, v_new, out, evicted);
  if (rc != TOVA_OK || n_steps == 0) return rc;
  if (!c->scratch) return TOVA_EINVAL;  // (a cache made for tova_decode_steps_static only)
  return decode_steps_on(c, c->scratch, n_steps, q, k_new, v_new, out, evicted, static_cast<hipStream_t>(hip_stream));
}

int tova_cache_publish_tokens_seen(tova_cache_t* c, void* hip_stream) {
  if (!c) return TOVA_EINVAL;
  const hipError_t e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(c->state + c->r.tok_off), (int32_t)c->t, 1,
                                             static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(e, "tova_cache_publish_tokens_seen");
  return TOVA_OK;
}

int tova_cache_fetch_tokens_seen(tova_cache_t* c, void* hip_stream, int64_t* t) {
  if (!c) return TOVA_EINVAL;
  int32_t v = 0;
  const hipError_t e = tova::read_i32_sync(reinterpret_cast<const int32_t*>(c->state + c->r.tok_off),
                                           static_cast<hipStream_t>(hip_stream), &v);
  if (e != hipSuccess) return hip_fail(e, "tova_cache_fetch_tokens_seen");
  if (v < 0) return TOVA_EINVAL;
  c->t = v;
  if (t) *t = v;
  return TOVA_OK;
}

int tova_decode_step_graph(tova_cache_t* c, const void* q, const void* k_new, const void* v_new, void* out,
                           int32_t* evicted, void* hip_stream) {
  const int rc = check_step_args(c, 1, q, k_new, v_new, out, evicted);
  if (rc != TOVA_OK) return rc;
  if (!c->scratch) return TOVA_EINVAL;
  if (c->t < c->r.k) return TOVA_ENOSUP;  // (the launch shape of a filling step depends on the row count)
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool capturing = tova::stream_is_capturing(s) != 0;
  const int64_t t_before = c->t;
  const int rs = decode_steps_on(c, c->scratch, 1, q, k_new, v_new, out, evicted, s, true);
  if (rs != TOVA_OK) return rs;
  const hipError_t e = tova::launch_add_i32(reinterpret_cast<int32_t*>(c->state + c->r.tok_off), 1, s);
  if (e != hipSuccess) return hip_fail(e, "tova_decode_step_graph: advancing the token count");
  if (capturing) c->t = t_before;  // nothing ran: the replays will, and the count in state_mem follows them
  return TOVA_OK;
}

int tova_decode_steps_static(tova_cache_t* c, int32_t n_steps, const void* q, const void* k_new,
                             const void* v_new, void* out, int32_t* evicted, void* hip_stream) {
  const int rc = check_step_args(c, n_steps, q, k_new, v_new, out, evicted);
  if (rc != TOVA_OK || n_steps == 0) return rc;
  const Resolved& r = c->r;
  // what the decode steps use of the scratch layout: everything in front of the prompt kernel's area
  if (r.uscr_off > TOVA_STATIC_SCRATCH_BYTES) return TOVA_ETOOBIG;
  void* area = nullptr;
  size_t area_bytes = 0;
  hipError_t e = tova::static_scratch(&area, &area_bytes);  // (a look-up; nothing is allocated)
  if (e != hipSuccess) return hip_fail(e, "tova_decode_steps_static: static scratch");
  if (r.uscr_off > area_bytes) return TOVA_ETOOBIG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // The area keeps whatever the previous call on this GPU left, possibly under another cache's
  // layout: the arrival counters, slow-route flags and state words must start at zero (a fill
  // kernel, so that the call can be recorded into a graph).  Everything else in it is written
  // before it is read within a step.
  e = tova::launch_fill_i32(static_cast<int32_t*>(area), 0, r.cnt_bytes / 4, s);
  if (e != hipSuccess) return hip_fail(e, "tova_decode_steps_static: clearing the counters");
  return decode_steps_on(c, static_cast<char*>(area), n_steps, q, k_new, v_new, out, evicted, s);
}

int tova_decode_steps_repositioned(tova_cache_t* c, int32_t n_steps, const void* q, const void* k_new,
                                   const void* v_new, void* out, int32_t* evicted, float rope_base,
                                   void* hip_stream) {
  if (!c || n_steps < 0 || !c->scratch) return TOVA_EINVAL;
  if (!(rope_base == rope_base) || std::isinf(rope_base)) return TOVA_EINVAL;
  if (n_steps == 0) return TOVA_OK;
  if (!q || !k_new || !v_new || !out) return TOVA_EINVAL;
  if (!aligned(q, 16) || !aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(out, 16) ||
      !aligned(evicted, 4))
    return TOVA_EINVAL;
  const Resolved& r = c->r;
  if (r.policy != TOVA_POLICY_TOVA) return TOVA_ENOSUP;
  if (c->t + n_steps > 0x7fffffffLL) return TOVA_ENOSUP;  // token index is kept in 32 bits
  // LDS of a workgroup: logits of the k + 1 candidates of a KV head's G query heads (the position
  // scratch, 20 bytes per candidate, and the PV reduction area share that memory), the head-summed
  // scores, and one double per candidate for the compressed distances
  // Two workgroups of 256 threads per CU when there are units for them and LDS for both: one's
  // logit pass (bound by the rotation arithmetic) then overlaps the other's PV pass (bound by
  // memory); measured 71-74% of peak bandwidth against 61-64% with one workgroup of 512.
  const int cus = tova::device_cus();
  const long long kp = ((long long)r.k + 1 + 3) / 4 * 4;
  // (*persist: room for the token order and the ranks outside the logit area, 8 bytes per candidate, so
  // that a workgroup that stays with its unit keeps them from step to step; taken when it fits)
  auto plan = [&](int nt, long long* e_fl, long long* lds, int* persist) {
    *e_fl = kp * r.G;
    if ((long long)(nt / 64) * r.G * r.D > *e_fl) *e_fl = (long long)(nt / 64) * r.G * r.D;
    if (5 * kp > *e_fl) *e_fl = 5 * kp;
    *lds = (kSmallFloats + *e_fl + kp + 2 * kp + r.D) * 4;  // (+ d / 2 doubles: the rotary frequencies)
    *persist = (*lds + 8 * kp <= kMaxLdsBytesUnit) && (*lds > 80 * 1024 || *lds + 8 * kp <= 80 * 1024);
    if (*persist) *lds += 8 * kp;
  };
  int nt = 0, per_cu = 1, persist = 0;
  long long e_fl = 0, lds = 0;
  for (int pass = 0; pass < 2; ++pass) {
    nt = (pass == 0) ? 256 : ((r.k >= 512) ? 512 : 256);
    if (c->repos_threads) nt = c->repos_threads;
    plan(nt, &e_fl, &lds, &persist);
    per_cu = (int)((160 * 1024) / lds);
    if (per_cu > 2) per_cu = 2;
    if (per_cu < 1) per_cu = 1;
    if (pass == 0 && per_cu == 2 && cus > 0 && r.units >= 2 * cus) break;
  }
  if (lds > kMaxLdsBytesUnit) return TOVA_ENOSUP;

  // Few units: once the cache is full the KV heads of a unit are dealt to `parts` workgroups of 256
  // threads, as many as fill the device twice over at most and are resident together (they wait
  // for each other's results).  It borrows the score rows, counters and state words of the
  // hand-off form of the step kernel, which exist exactly when there are few units.
  int parts = 1;
  long long e_fl_p = 0, lds_p = 0;
  int persist_p = 0;
  if (!r.unit_mode && r.H_kv > 1 && cus > 0 && r.units < cus) {
    plan(256, &e_fl_p, &lds_p, &persist_p);
    const int cap = tova::repos_resident_blocks(r.bf16, r.D, r.G, 256, (int)lds_p);
    int limit = 2 * cus < cap ? 2 * cus : cap;
    if (c->repos_parts && (long long)c->repos_parts * r.units < limit) limit = c->repos_parts * r.units;
    for (int pcand = r.H_kv; pcand >= 2; --pcand)
      if (r.H_kv % pcand == 0 && (long long)r.units * pcand <= limit && (size_t)pcand * kp <= (size_t)r.H_kv * r.kp) {
        parts = pcand;
        break;
      }
  }

  tova::ReposParams p;
  p.K = c->kv;
  p.V = c->kv + r.v_off;
  p.occupancy = reinterpret_cast<int32_t*>(c->state + r.occ_off);
  p.slot_token = reinterpret_cast<int32_t*>(c->state + r.slot_off);
  p.q_stride = (int64_t)r.units * r.H * r.D;
  p.kv_stride = (int64_t)r.pairs * r.D;
  p.log2_base = std::log2(rope_base > 0.f ? (double)rope_base : 10000.0);
  p.units = r.units; p.H = r.H; p.H_kv = r.H_kv; p.k = r.k; p.n_pinned = r.n_pinned;
  p.scale = r.scale;
  p.spin = r.persist_spin;
  p.sg = reinterpret_cast<float*>(c->scratch + r.sg_off);
  p.cnt_unit = reinterpret_cast<int32_t*>(c->scratch + r.cnt_unit_off);
  p.pstate = reinterpret_cast<unsigned long long*>(c->scratch + r.pstate_off);
  p.error_flag = reinterpret_cast<int32_t*>(c->state + r.err_off);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t q_step = (size_t)r.units * r.H * r.D * r.esize;
  const size_t kv_step = (size_t)r.pairs * r.D * r.esize;
  for (int32_t i = 0; i < n_steps;) {
    // with parts: the steps that fill the cache first, a workgroup per unit; then the rest, split
    const bool split = (parts > 1 && c->t >= r.k);
    int32_t m = n_steps - i;
    if (parts > 1 && c->t < r.k && (long long)m > r.k - c->t) m = (int32_t)(r.k - c->t);
    p.q = static_cast<const char*>(q) + (size_t)i * q_step;
    p.k_new = static_cast<const char*>(k_new) + (size_t)i * kv_step;
    p.v_new = static_cast<const char*>(v_new) + (size_t)i * kv_step;
    p.out = static_cast<char*>(out) + (size_t)i * q_step;
    p.evicted = evicted ? evicted + (size_t)i * r.units : nullptr;
    p.n0 = (int32_t)(c->t < r.k ? c->t : r.k);
    p.n_iter = m;
    p.t = (int32_t)c->t;
    p.parts = split ? parts : 1;
    p.e_floats = (int)(split ? e_fl_p : e_fl);
    p.persist = split ? persist_p : persist;
    int grid = cus > 0 ? cus * per_cu : r.units;
    if (grid > r.units) grid = r.units;
    const tova::LaunchPlan lp = split ? tova::LaunchPlan{r.units * parts, 256, (int)lds_p} : tova::LaunchPlan{grid, nt, (int)lds};
    hipError_t e = hipSuccess;
    if (split)  // the units' state words start from "no step finished"
      e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(p.pstate), 0, (size_t)r.units * 2, s);
    if (e == hipSuccess) e = tova::launch_repos(r.bf16, r.D, r.G, p, lp, s);
    if (e != hipSuccess) return hip_fail(e, "tova_decode_steps_repositioned launch");
    c->t += m;
    i += m;
  }
  return TOVA_OK;
}

int tova_policy_step(tova_cache_t* c, const float* attn_weights, const void* k_new, const void* v_new,
                     int32_t* evicted, void* hip_stream) {
  if (!c || !attn_weights || !k_new || !v_new) return TOVA_EINVAL;
  if (!aligned(attn_weights, 4) || !aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(evicted, 4))
    return TOVA_EINVAL;
  const Resolved& r = c->r;
  if (r.policy != TOVA_POLICY_TOVA) return TOVA_ENOSUP;
  if (c->t + 1 > 0x7fffffffLL) return TOVA_ENOSUP;  // token index is kept in 32 bits
  tova::PolicyParams p;
  p.w = attn_weights; p.k_new = k_new; p.v_new = v_new; p.evicted = evicted;
  p.K = c->kv;
  p.V = c->kv + r.v_off;
  p.occupancy = reinterpret_cast<int32_t*>(c->state + r.occ_off);
  p.slot_token = reinterpret_cast<int32_t*>(c->state + r.slot_off);
  p.n = (int32_t)(c->t < r.k ? c->t : r.k);
  p.units = r.units; p.H = r.H; p.H_kv = r.H_kv; p.k = r.k; p.n_pinned = r.n_pinned;
  p.t = (int32_t)c->t;
  p.row_bytes = r.D * r.esize;
  const hipError_t e = tova::launch_policy(p, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return hip_fail(e, "tova_policy_step launch");
  c->t += 1;
  return TOVA_OK;
}

int tova_decode_step(tova_cache_t* c, const void* q, const void* k_new, const void* v_new, void* out,
                     int32_t* evicted, void* hip_stream) {
  return tova_decode_steps(c, 1, q, k_new, v_new, out, evicted, hip_stream);
}

int tova_cache_multi_step_blocks(const tova_cache_t* c, int32_t* blocks) {
  if (!c || !blocks) return TOVA_EINVAL;
  *blocks = c->r.multi_step ? c->r.multi_grid : 0;
  return TOVA_OK;
}

int tova_cache_tokens_seen(const tova_cache_t* c, int64_t* t) {
  if (!c || !t) return TOVA_EINVAL;
  *t = c->t;
  return TOVA_OK;
}

int tova_cache_set_tokens_seen(tova_cache_t* c, int64_t t) {
  if (!c || t < 0) return TOVA_EINVAL;
  if (t > 0x7fffffffLL) return TOVA_ENOSUP;
  c->t = t;
  return TOVA_OK;
}

int tova_cache_status(tova_cache_t* c, void* hip_stream, int32_t* gave_up) {
  if (!c || !gave_up) return TOVA_EINVAL;
  int32_t flag = 0;
  const hipError_t e = tova::read_i32_sync(reinterpret_cast<const int32_t*>(c->state + c->r.err_off),
                                           static_cast<hipStream_t>(hip_stream), &flag);
  if (e != hipSuccess) return hip_fail(e, "tova_cache_status");
  *gave_up = (flag != 0);
  return TOVA_OK;
}

int tova_cache_recover(tova_cache_t* c, int64_t tokens_seen, void* hip_stream) {
  if (!c || tokens_seen < 0) return TOVA_EINVAL;
  if (tokens_seen > 0x7fffffffLL) return TOVA_ENOSUP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(c->state + c->r.err_off), 0, 1, s);
  if (e == hipSuccess && c->scratch)  // arrival counters, slow-route flags, state words: as after tova_cache_init
    e = tova::launch_fill_i32(reinterpret_cast<int32_t*>(c->scratch), 0, c->r.cnt_bytes / 4, s);
  if (e != hipSuccess) return hip_fail(e, "tova_cache_recover");
  c->t = tokens_seen;
  // A launch whose workgroups wait for one another has failed once on this device: from here on
  // this cache steps with one launch per step, where nobody waits for anybody.
  if (!c->r.unit_mode) c->r.multi_step = 0;
  return TOVA_OK;
}

int tova_cache_destroy(tova_cache_t* c) {
  if (!c) return TOVA_EINVAL;
  delete c;
  return TOVA_OK;
}

const char* tova_strerror(int status) {
  switch (status) {
    case TOVA_OK: return "ok";
    case TOVA_EINVAL: return "invalid argument";
    case TOVA_ENOSUP: return "shape not supported by the gfx950 kernels";
    case TOVA_EHIP: return g_hip_msg[0] ? g_hip_msg : "HIP runtime error";
    case TOVA_ENOMEM: return "out of host memory";
    case TOVA_ETOOBIG: return "configuration needs more scratch than the library's static area holds (32 MiB)";
    default: return "unknown status";
  }
}

}  // extern "C"
