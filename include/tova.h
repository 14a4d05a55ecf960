/*
 * tova.h -- C ABI of the TOVA bounded-KV-cache decode step for AMD MI355X (gfx950).
 *
 * The library implements the hot path of the TOVA policy ("Token Omission Via
 * Attention", arXiv 2401.06104): a decoder layer seen as a bounded multi-state
 * RNN whose state is a KV cache of at most k rows (Sec. 3.1-3.3).  One decode
 * step of one (layer, sequence) unit
 *   1. appends the incoming token's k_t, v_t to the multi-state and lets the
 *      query q_t attend over all of it, Softmax(q K^T / sqrt(d)) V per head
 *      (Sec. 3.2, Sec. 2.2) -- the output still sees the row dropped below;
 *   2. if the multi-state now exceeds k rows, averages the attention weights
 *      of q_t over the query heads of the layer, takes the argmin and drops
 *      that row from K and V (Sec. 4; App. B, Alg. 1).  All heads of a layer
 *      share the victim (the "layer" variant that App. A finds best).
 * Rows live in k fixed slots: the victim's slot is overwritten in place by the
 * new token (attention does not depend on row order); if the new token itself
 * scores lowest it is not stored.  Ties go to the lowest candidate index, the
 * new token having the highest (k).
 *
 * Conventions
 *   - every function returns TOVA_OK (0) or a negative tova_status; nothing
 *     throws, aborts or prints.  tova_strerror() describes a code; after
 *     TOVA_EHIP it also carries the HIP runtime's message (thread-local).
 *   - "DEVICE" pointers are HIP device memory on the current device, owned by
 *     the caller, 256-byte aligned, and must outlive every use enqueued on the
 *     stream.  "HOST" pointers are ordinary host memory.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  Calls enqueue work and return; they never synchronise.
 *   - one cache may be used from one host thread at a time.
 *   - inputs must be finite; with NaN scores the victim is unspecified
 *     (but always in range).
 */
#ifndef TOVA_H
#define TOVA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TOVA_OK = 0,
  TOVA_EINVAL = -1, /* null / misaligned pointer, non-positive size, H % H_kv != 0, bad dtype ... */
  TOVA_ENOSUP = -2, /* valid problem, but a shape the kernels do not cover                       */
  TOVA_EHIP = -3,   /* a HIP call (launch) failed                                                  */
  TOVA_ENOMEM = -4, /* host allocation of the descriptor failed                                     */
  TOVA_ETOOBIG = -5 /* tova_decode_steps_static: the configuration needs more scratch than the
                       library's static area holds (TOVA_STATIC_SCRATCH_BYTES)                     */
} tova_status;

enum { TOVA_F32 = 0, TOVA_BF16 = 1 };

/* Which row leaves a full multi-state (Sec. 3.3: the compression policy).  TOVA is the paper's
 * method (Sec. 4); the other two are the baseline policies it is compared with (Sec. 4.1). */
enum {
  TOVA_POLICY_TOVA = 0,   /* the row with the lowest head-averaged attention weight of the current query   */
  TOVA_POLICY_WINDOW = 1, /* Window+i: the oldest token that is not one of the first n_pinned (i = n_pinned; */
                          /* 0 = plain Window, first in first out).  The incoming token is always stored.     */
  TOVA_POLICY_H2O = 2     /* H2O: the h2o_recent most recent tokens (the incoming one included) always stay;  */
                          /* among the others the row whose attention weights, head-averaged and summed over  */
                          /* every step since its token came in (this step included), are lowest.             */
};

typedef struct tova_cache tova_cache_t; /* opaque host-side descriptor */

/* Problem statement, in the paper's terms (App. B: attn_heads, hidden_dim,
 * cache_max_size; batch and layers are independent units). */
typedef struct {
  int32_t n_layers;     /* L                                                          */
  int32_t batch;        /* B independent sequences                                     */
  int32_t capacity_k;   /* k = cache_max_size, the multi-state size (Sec. 3.3)         */
  int32_t n_q_heads;    /* H query heads                                               */
  int32_t n_kv_heads;   /* H_kv, divides H; query head h reads KV head h / (H / H_kv)  */
  int32_t head_dim;     /* d in {32, 64, 128}                                          */
  int32_t dtype;        /* TOVA_F32 or TOVA_BF16: type of q, k, v, K, V and out        */
  float softmax_scale;  /* <= 0 selects 1 / sqrt(d)                                    */
  int32_t n_splits;     /* 0 = automatic; S >= 1 asks for S slot chunks per KV head    */
  /* Variants of the paper's policy ablation (App. A); 0 / 0 is the policy described above.        */
  int32_t n_pinned;     /* TOVA+i: the first i tokens are never dropped, 0 <= i < k (they hold  */
                        /* slots 0..i-1 from the fill phase on and are skipped by the argmin)   */
  int32_t per_head;     /* TOVA-head: nonzero = every KV head (with the H / H_kv query heads it */
                        /* serves, averaged) keeps its own rows and drops its own victim.  Then */
                        /* evicted, occupancy and slot_token have a trailing [H_kv] dimension   */
                        /* after [L][B]: evicted [L][B][H_kv], slot_token [L][B][H_kv][k].      */
  /* Baseline policies (Sec. 4.1); 0 / 0 is TOVA.                                                    */
  int32_t policy;       /* TOVA_POLICY_*.  WINDOW and H2O run in the workgroup-per-unit form for any */
                        /* number of units (TOVA_ENOSUP if a KV head's logits do not fit on-chip     */
                        /* memory) and through tova_decode_step(s) / tova_decode_steps_static /      */
                        /* tova_prefill (token by token) only.  per_head gives the head-wise H2O the */
                        /* paper reports; H2O takes n_pinned = 0.                                     */
  int32_t h2o_heavy;    /* H2O: rows outside the recent window, 0 <= h < k; 0 selects floor(k / 2)   */
                        /* ("typically half of the multi-state size"); the window is k - h tokens.   */
} tova_config_t;

/* Where things live inside the caller's buffers (byte offsets). */
typedef struct {
  size_t k_offset;          /* kv_mem:    K  [L][B][H_kv][k][d]                 */
  size_t v_offset;          /* kv_mem:    V  [L][B][H_kv][k][d]                 */
  size_t occupancy_offset;  /* state_mem: int32 [L][B]    rows in use, min(t,k) */
  size_t slot_token_offset; /* state_mem: int32 [L][B][k] token index held by a slot, -1 = empty */
  size_t error_flag_offset; /* state_mem: int32, 0 = fine; set by a multi-step launch that gave up
                               waiting (see tova_decode_steps); the steps after that were not done */
  int32_t n_splits;         /* resolved split count S                            */
  int32_t rows_per_split;   /* slots per chunk                                   */
  int32_t block_threads;    /* workgroup size the step kernel is launched with   */
  int32_t grid_blocks;      /* workgroups per step                               */
  int32_t lds_bytes;        /* dynamic LDS per workgroup                         */
  int32_t unit_workgroups;  /* nonzero: a workgroup handles a whole (layer, sequence) unit, its KV
                               heads in turn (chosen when L * B alone fills the device); grid_blocks
                               is then L * B, walked by at most a device-filling number of workgroups */
  int32_t prefill_group;    /* tokens of a prompt that share one pass over the cache in tova_prefill
                               (0: it goes token by token)                                         */
  size_t tokens_seen_offset; /* state_mem: int32, the token count as the device sees it; only kept current by
                               the calls below that say so (tova_decode_step_graph and its two helpers)  */
  size_t h2o_acc_offset;    /* state_mem: float [L][B][k] (H2O only; with per_head [L][B][H_kv][k]): per slot,
                               the attention weights summed over the query heads and over all steps
                               since the slot's token came in (divide by H for the head average)   */
  int32_t service_wave;     /* nonzero: in multi-step launches the last wave of a workgroup serves the hand-off
                               between workgroups instead of streaming V (hand-off form only; a tuning
                               decision of the library, reported for the record)                     */
} tova_layout_t;

/* Sizes of the three caller-owned DEVICE buffers.  kv_bytes is exactly
 * 2*L*B*H_kv*k*d*sizeof(elem) (the paper's cache-memory row, Sec. 7.1 table).
 * HOST pointers; any of the three outputs may be NULL. */
int tova_cache_bytes(const tova_config_t* cfg, size_t* kv_bytes, size_t* state_bytes,
                     size_t* scratch_bytes);

/* Offsets and launch plan for a configuration (host only, no GPU needed).  No passage of the
 * paper: library bookkeeping -- where the multi-state H_t = (K_t, V_t) of Sec. 3.2 and the
 * slot -> token map live inside the caller's buffers, and how the step kernel will be launched. */
int tova_cache_layout(const tova_config_t* cfg, tova_layout_t* layout);

/* The empty multi-state H_0 of a bounded multi-state RNN with g(t) = min(t, k) (Sec. 3.1, 3.3):
 * creates a descriptor over caller-owned DEVICE buffers of at least the sizes
 * tova_cache_bytes reports and enqueues kernels that empty the cache
 * (occupancy 0, slot_token -1, scratch counters 0, error flag 0, H2O sums 0).  K/V contents are
 * not touched: empty slots are never read.
 * The environment hooks named in this header (tuning aids and test hooks) are read here and by
 * tova_cache_layout / tova_cache_bytes only, and kept in the descriptor: no stepping call reads
 * the environment. */
int tova_cache_init(tova_cache_t** out, const tova_config_t* cfg, void* kv_mem, void* state_mem,
                    void* scratch_mem, void* hip_stream);

/* One decode step for every (layer, sequence) unit (Sec. 3.2 + Sec. 4).
 *   q      DEVICE [L][B][H][d]      queries of the incoming tokens
 *   k_new  DEVICE [L][B][H_kv][d]   their keys   (post positional encoding)
 *   v_new  DEVICE [L][B][H_kv][d]   their values
 *   out    DEVICE [L][B][H][d]      attention outputs over cached rows + the new row
 *   evicted DEVICE int32 [L][B] or NULL: -1 while the cache is filling,
 *          0..k-1 = slot whose row was dropped and now holds the new token,
 *          k = the new token itself was dropped.
 * Below capacity the new row goes to slot `occupancy` (App. B: no-op branch). */
int tova_decode_step(tova_cache_t* cache, const void* q, const void* k_new, const void* v_new,
                     void* out, int32_t* evicted, void* hip_stream);

/* n_steps consecutive decode steps (Sec. 3.2 + Sec. 4, App. B Alg. 1 once per step: the loop an
 * autoregressive decoder runs over its bounded multi-state) with inputs resident in device memory:
 * the arrays of tova_decode_step with a leading [n_steps] dimension
 * (evicted: [n_steps][L][B], may be NULL).  Same victims and cache contents as n_steps calls; `out`
 * agrees to the rounding of fp32 sums (the rows may be added in another order).
 * Once the cache is full the remaining steps of a call run in ONE launch.
 *  - With L * B >= 256 units and one chunk per KV head (layout: unit_workgroups != 0) a workgroup
 *    owns whole units: it goes through a unit's KV heads in turn, keeps the head-summed scores in
 *    on-chip memory, picks the victim and stores the new rows itself.  Workgroups never wait for
 *    one another; any number of them may run.
 *  - Otherwise a workgroup stays with its (sequence, KV head[, chunk]) items for all steps;
 *    sequences advance independently of one another and the only wait in the kernel is a
 *    workgroup's wait for the victim of its own sequence's previous step.  That wait is bounded;
 *    should it ever run out (it cannot while all workgroups of the launch are resident, which
 *    tova_cache_init checks against an otherwise idle device; another kernel sharing the device
 *    can break that), the kernel sets the int32 at error_flag_offset of state_mem and stops
 *    early.  The units are then at different steps and the cache contents are not usable:
 *    tova_cache_status reports the condition, tova_cache_recover takes the cache back into
 *    service from a snapshot the caller restores (see there).
 * The environment variable TOVA_MULTI_STEP=0 keeps one launch per step; TOVA_UNIT_MODE=0 / 1
 * (read by tova_cache_init / tova_cache_layout) overrides the choice between the two forms,
 * TOVA_SERVICE_WAVE=0 / 1 the use of a service wave (layout: service_wave). */
int tova_decode_steps(tova_cache_t* cache, int32_t n_steps, const void* q, const void* k_new,
                      const void* v_new, void* out, int32_t* evicted, void* hip_stream);

/* A prompt: n_tokens consecutive tokens that are all known in advance (num_q > 1 in the terms of
 * App. B).  Arguments and results are those of tova_decode_steps -- every token attends over what
 * the multi-state holds after the tokens before it, and is followed by the policy, exactly as if
 * it had been given alone; this is the mask formulation the paper uses to score whole texts --
 * but because the queries are known together, groups of 2 to 8 tokens share one pass over the
 * cache (K and V are read once per group instead of once per token).  A later token of a group is
 * corrected for what the earlier ones removed, and the victim is found among the few candidates
 * whose score bounds allow it, from scores recomputed exactly; outputs and victims agree with
 * tova_decode_steps to rounding (different summation order).  While the cache still has room the
 * groups simply append their tokens.  Grouping needs the workgroup-per-unit form (layout:
 * unit_workgroups), 1, 2 or 4 query heads per KV head and a capacity of at least 8 groups (the
 * corrections stay exact to rounding only while what a group removes is a small part of the
 * multi-state); whatever does not meet that (a
 * remainder shorter than a group, the last rows before the cache is full, other shapes) is
 * processed token by token through tova_decode_steps.  TOVA_PREFILL_GROUP=0 in the environment
 * (read by tova_cache_init) turns grouping off. */
int tova_prefill(tova_cache_t* cache, int32_t n_tokens, const void* q, const void* k_new,
                 const void* v_new, void* out, int32_t* evicted, void* hip_stream);

/* Decode steps beyond the training length (Sec. 7.2, "Extrapolation with TOVA").  Arguments and
 * results are those of tova_decode_steps, with one difference in meaning: q, k_new and the cached
 * keys carry NO positional encoding.  Before each attention the positions of everything the query
 * attends over are re-assigned -- between two candidates that are adjacent in token order (the
 * slot -> token map in state_mem gives the order) a gap of g tokens counts as ln(ln(g)), gaps of at
 * most 10 tokens as they are -- and the rotary embedding is applied inside the kernel at those
 * positions: element i of a head vector is paired with element i + d/2, the pair turned by
 * position * rope_base^(-2i/d).  rope_base <= 0 selects 10000; NaN / infinity -> TOVA_EINVAL.
 * Values are not touched; softmax, outputs, scores, victim and the in-place overwrite (of the
 * un-rotated rows) are as in tova_decode_steps, the n_pinned / per_head variants included.
 * The caller keeps one convention per cache: a cache stepped through this entry point holds
 * un-rotated keys and must not be handed to the others, and vice versa.
 * A workgroup owns a (layer, sequence) unit and one launch covers all n_steps, the fill phase
 * included.  With fewer units than compute units (and more than one KV head, and not the
 * unit_workgroups layout) the steps on a full cache instead deal the KV heads of a unit to several
 * workgroups that are all resident; they exchange partial head sums and wait -- bounded -- for the
 * unit's victim before its next step; should such a wait ever run out the kernel sets the int32 at
 * error_flag_offset of state_mem and stops early, as described for tova_decode_steps.
 * Needs on-chip memory for (k + 1) * (4 * max(H / H_kv, 5) + 12) bytes plus 2.5 KiB within 152 KiB,
 * else TOVA_ENOSUP (k = 4096 fits with up to 4 query heads per KV head, k = 2048 with 8).
 * TOVA_REPOS_PARTS=n in the environment (read by tova_cache_init) allows at most n workgroups
 * per unit (1: never split). */
int tova_decode_steps_repositioned(tova_cache_t* cache, int32_t n_steps, const void* q, const void* k_new,
                                   const void* v_new, void* out, int32_t* evicted, float rope_base,
                                   void* hip_stream);

/* The policy on its own (App. B, Alg. 1), for callers that compute attention themselves: one step
 * for every (layer, sequence).  attn_weights: DEVICE fp32 [L][B][H][k+1], the last query's softmax
 * weights over the k slots (in slot order) followed by the incoming token's (index k); with
 * per_head the same memory is read as [L][B][H_kv][H / H_kv][k+1].  While the cache has room the
 * weights are not read and the incoming rows take the next slot (evicted = -1; the early return of
 * Alg. 1).  Otherwise the weights are summed over the heads in head order, the lowest candidate
 * (lowest index on ties, candidates below n_pinned kept out) is the victim: evicted[l][b] = its
 * index, k_new / v_new overwrite its slot, or are not stored if the victim is index k.  k_new,
 * v_new, evicted as in tova_decode_step; the caller's attention must have been taken over exactly
 * the slots as they are, which is what the map in state_mem and K / V show. */
int tova_policy_step(tova_cache_t* cache, const float* attn_weights, const void* k_new,
                     const void* v_new, int32_t* evicted, void* hip_stream);

/* No passage of the paper: library bookkeeping.
 * How tova_decode_steps launches once the cache is full (decided in tova_cache_init, which asks
 * the device how many workgroups fit): *blocks = 0 -> one launch per step; otherwise the number
 * of workgroups of the single launch that runs all remaining steps of a call (with
 * unit_workgroups: of every launch).  HOST out pointer. */
int tova_cache_multi_step_blocks(const tova_cache_t* cache, int32_t* blocks);

/* Number of tokens the cache has seen since tova_cache_init: t of Sec. 3.1-3.3, the cache
 * holds g(t) = min(t, k) rows (HOST out pointer). */
int tova_cache_tokens_seen(const tova_cache_t* cache, int64_t* t);

/* Checkpoint / resume.  The whole state of a cache is the caller's kv_mem and state_mem plus
 * this token count: a caller that has copied those buffers back (e.g. from a snapshot taken
 * after t tokens) tells the library so with this call; the next step then treats the cache as
 * holding min(t, k) rows and numbers the incoming token t.  The occupancy array in state_mem
 * must agree (it does if it was restored together with the rest).  t >= 0. */
int tova_cache_set_tokens_seen(tova_cache_t* cache, int64_t t);

/* For callers that cannot allocate device memory (code under HIP graph capture, serving loops
 * and harnesses that forbid hipMalloc): tova_decode_steps with the hand-off scratch (arrival
 * counters, per-unit state words, partial score rows, chunk statistics, PV partials) taken from
 * a static device array inside the library instead of the cache's scratch_mem.  Arguments and
 * results are those of tova_decode_steps, bit for bit.  The call allocates nothing and frees
 * nothing; what it clears it clears with fill kernels, not memsets.
 *  - The array holds TOVA_STATIC_SCRATCH_BYTES per GPU for the life of the process.  A
 *    configuration whose decode steps need more than that (scratch_bytes of tova_cache_bytes less
 *    the area only tova_prefill uses; the five paper-shaped configurations need at most 22.4 MiB)
 *    -> TOVA_ETOOBIG, nothing is enqueued.
 *  - Every call on a GPU shares that GPU's array, which keeps the previous call's contents: the
 *    call clears the counters it relies on first.  Calls that overlap in time on one GPU (two
 *    streams, two host threads) race on it: keep them in one stream order.  Stepping one cache
 *    alternately through this call and tova_decode_steps is fine.
 *  - tova_cache_init accepts scratch_mem = NULL for a cache that is only ever stepped through this
 *    call (tova_decode_step, tova_decode_steps and tova_prefill then return TOVA_EINVAL). */
#define TOVA_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int tova_decode_steps_static(tova_cache_t* cache, int32_t n_steps, const void* q, const void* k_new,
                             const void* v_new, void* out, int32_t* evicted, void* hip_stream);

/* One decode step that can be recorded into a HIP graph and replayed for token after token (no
 * passage of the paper: it is tova_decode_step, Sec. 3.2 + Sec. 4, for callers that replay launches
 * instead of issuing them).  A launch recorded by the other calls carries the token index as a
 * host-side argument, so replaying it would process "the same token" again; this call's kernels
 * read the index from the int32 at tokens_seen_offset of state_mem and a kernel of its own adds 1
 * to it afterwards.  Arguments and results are those of tova_decode_step; the caller rewrites
 * q / k_new / v_new in place between replays and reads out / evicted after each.
 *  - The cache must be full (tokens seen >= k: the launch shape of a filling step depends on the
 *    row count), else TOVA_ENOSUP.
 *  - tova_cache_publish_tokens_seen enqueues a kernel that writes the host's count into state_mem:
 *    call it once, outside the graph, before the first recording or replay, and again after any
 *    other stepping call or tova_cache_set_tokens_seen.
 *  - Called on a stream that is being captured, the call records its kernels and leaves the
 *    host's count alone (nothing ran); called eagerly it counts one token like any other call.
 *  - After replays the host's count is behind: tova_cache_fetch_tokens_seen waits for the stream,
 *    reads the count back from state_mem (HOST out pointer t, may be NULL) and makes it the
 *    host's; do that before any other call on the cache.
 * Nothing is allocated and no memset is recorded (fill kernels only). */
int tova_decode_step_graph(tova_cache_t* cache, const void* q, const void* k_new, const void* v_new,
                           void* out, int32_t* evicted, void* hip_stream);
int tova_cache_publish_tokens_seen(tova_cache_t* cache, void* hip_stream);
int tova_cache_fetch_tokens_seen(tova_cache_t* cache, void* hip_stream, int64_t* t);

/* Failure handling of the multi-step launches (no passage of the paper: library bookkeeping).
 * tova_cache_status waits for the stream (hipStreamSynchronize) and reads the cache's error flag:
 * *gave_up = 1 if a multi-step launch of tova_decode_steps / tova_decode_steps_static /
 * tova_decode_steps_repositioned ran out of its bounded wait since the flag was last cleared, else
 * 0.  HOST out pointer.  The one call of this library that synchronises. */
int tova_cache_status(tova_cache_t* cache, void* hip_stream, int32_t* gave_up);

/* After tova_cache_status reported 1: the caller copies a snapshot of kv_mem and state_mem taken
 * after `tokens_seen` tokens back into place (the library keeps none), then calls this.  It
 * enqueues kernels that clear the error flag and every hand-off counter in scratch_mem, sets the
 * token count to `tokens_seen`, and makes this cache use one launch per step from now on (the
 * launch mode in which no workgroup waits for another), so the steps can simply be issued again. */
int tova_cache_recover(tova_cache_t* cache, int64_t tokens_seen, void* hip_stream);

/* Frees the host descriptor only; device buffers stay with the caller (no passage of the paper:
 * library bookkeeping). */
int tova_cache_destroy(tova_cache_t* cache);

/* Text for a tova_status (no passage of the paper: library bookkeeping). */
const char* tova_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* TOVA_H */
