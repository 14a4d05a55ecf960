// Drives the host logic of libtova (tova_api.cpp built against stubs.cpp) through the C ABI under
// AddressSanitizer / UndefinedBehaviorSanitizer: a sweep of valid and invalid configurations through
// tova_cache_bytes / tova_cache_layout, and every stepping entry point on descriptors over fake,
// aligned device addresses (the stubs never touch them).  Exits 0 when every return code is the
// expected one; the sanitizers abort the process on any host-side memory error or undefined behaviour.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>

#include "tova.h"

namespace tova { extern long g_launches; }

#define EXPECT(cond)                                                           \
  do {                                                                         \
    if (!(cond)) {                                                             \
      std::fprintf(stderr, "%s:%d: expectation failed: %s\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                            \
    }                                                                          \
  } while (0)

static tova_config_t cfg(int L, int B, int k, int H, int Hkv, int d, int dt, int S = 0, int pinned = 0, int per_head = 0,
                         int policy = 0, int heavy = 0) {
  tova_config_t c;
  std::memset(&c, 0, sizeof c);
  c.n_layers = L; c.batch = B; c.capacity_k = k; c.n_q_heads = H; c.n_kv_heads = Hkv; c.head_dim = d; c.dtype = dt;
  c.n_splits = S; c.n_pinned = pinned; c.per_head = per_head; c.policy = policy; c.h2o_heavy = heavy;
  return c;
}

int main() {
  long configs = 0, valid = 0;
  // ---- the plan over a sweep of shapes: whatever it returns must be self-consistent ----
  const int Ls[] = {1, 2, 32}, Bs[] = {1, 3, 64, 300}, ks[] = {1, 2, 17, 512, 1024, 4096, 70000, 1 << 20};
  const int Hs[] = {1, 4, 32, 64}, Gs[] = {1, 2, 3, 4, 8, 16}, ds[] = {16, 32, 64, 128, 256};
  for (int L : Ls) for (int B : Bs) for (int k : ks) for (int H : Hs) for (int G : Gs) for (int d : ds)
    for (int dt = 0; dt < 2; ++dt) for (int S : {0, 1, 3, 64}) for (int policy = 0; policy < 3; ++policy) {
      if (H % G) continue;
      tova_config_t c = cfg(L, B, k, H, H / G, d, dt, S, 0, 0, policy, 0);
      size_t kv = 0, st = 0, sc = 0;
      tova_layout_t lay;
      const int rc = tova_cache_bytes(&c, &kv, &st, &sc);
      const int rc2 = tova_cache_layout(&c, &lay);
      ++configs;
      EXPECT(rc == rc2);
      EXPECT(rc == TOVA_OK || rc == TOVA_ENOSUP || rc == TOVA_EINVAL);
      if (rc != TOVA_OK) continue;
      ++valid;
      const size_t e = dt ? 2 : 4;
      EXPECT(kv == 2 * (size_t)L * B * (H / G) * k * d * e);
      EXPECT(lay.v_offset == kv / 2 && lay.k_offset == 0);
      EXPECT((long long)lay.n_splits * lay.rows_per_split >= k && (long long)(lay.n_splits - 1) * lay.rows_per_split < k);
      EXPECT(lay.lds_bytes > 0 && lay.lds_bytes <= 160 * 1024 && lay.block_threads % 64 == 0);
      EXPECT(lay.error_flag_offset + 4 <= st && lay.slot_token_offset + 4 * (size_t)L * B * k <= lay.error_flag_offset);
      EXPECT(policy == 0 || lay.unit_workgroups == 1);
      EXPECT(policy != 2 || lay.h2o_acc_offset + 4 * (size_t)L * B * k <= st);
    }
  EXPECT(valid > 1000);
  // ---- invalid arguments ----
  {
    tova_config_t c = cfg(1, 1, 16, 4, 4, 32, TOVA_F32);
    EXPECT(tova_cache_bytes(nullptr, nullptr, nullptr, nullptr) == TOVA_EINVAL);
    EXPECT(tova_cache_layout(&c, nullptr) == TOVA_EINVAL);
    tova_config_t bad = c; bad.n_pinned = 16; EXPECT(tova_cache_bytes(&bad, nullptr, nullptr, nullptr) == TOVA_EINVAL);
    bad = c; bad.policy = 3; EXPECT(tova_cache_bytes(&bad, nullptr, nullptr, nullptr) == TOVA_EINVAL);
    bad = c; bad.policy = TOVA_POLICY_H2O; bad.h2o_heavy = 16; EXPECT(tova_cache_bytes(&bad, nullptr, nullptr, nullptr) == TOVA_EINVAL);
    bad = c; bad.h2o_heavy = 3; EXPECT(tova_cache_bytes(&bad, nullptr, nullptr, nullptr) == TOVA_EINVAL);
    tova_cache_t* h = nullptr;
    EXPECT(tova_cache_init(&h, &c, nullptr, nullptr, nullptr, nullptr) == TOVA_EINVAL && h == nullptr);
    EXPECT(tova_cache_init(&h, &c, (void*)(256 + 8), (void*)512, (void*)768, nullptr) == TOVA_EINVAL);
    EXPECT(tova_cache_status(nullptr, nullptr, nullptr) == TOVA_EINVAL);
    EXPECT(tova_cache_recover(nullptr, 0, nullptr) == TOVA_EINVAL);
    EXPECT(tova_decode_steps_static(nullptr, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == TOVA_EINVAL);
  }
  // ---- the launch loops on fake (aligned, never dereferenced) device addresses ----
  const tova_config_t runs[] = {
      cfg(1, 1, 16, 4, 4, 32, TOVA_F32), cfg(1, 64, 1024, 32, 8, 128, TOVA_BF16), cfg(32, 1, 4096, 32, 4, 128, TOVA_BF16),
      cfg(32, 64, 4096, 32, 32, 128, TOVA_BF16), cfg(1, 1, 512, 32, 32, 128, TOVA_BF16), cfg(2, 3, 300, 8, 2, 128, TOVA_BF16, 3),
      cfg(2, 3, 64, 8, 4, 64, TOVA_BF16, 0, 4, 1), cfg(4, 80, 100, 8, 4, 64, TOVA_BF16, 0, 2, 0, TOVA_POLICY_WINDOW),
      cfg(1, 2, 37, 8, 2, 64, TOVA_F32, 0, 0, 1, TOVA_POLICY_H2O, 5)};
  for (const tova_config_t& c : runs) {
    char* base = reinterpret_cast<char*>((uintptr_t)1 << 40);
    tova_cache_t* h = nullptr;
    EXPECT(tova_cache_init(&h, &c, base, base + ((size_t)1 << 38), base + ((size_t)1 << 39), nullptr) == TOVA_OK && h);
    void* q = base + ((size_t)3 << 38);
    int32_t* ev = reinterpret_cast<int32_t*>(base + ((size_t)5 << 38));
    const long before = tova::g_launches;
    const int k = c.capacity_k;
    EXPECT(tova_decode_steps(h, 0, q, q, q, q, ev, nullptr) == TOVA_OK);
    EXPECT(tova_decode_steps(h, 3, q, q, q, (char*)q + 8, ev, nullptr) == TOVA_EINVAL);      // misaligned
    EXPECT(tova_decode_step(h, q, q, q, q, nullptr, nullptr) == TOVA_OK);
    EXPECT(tova_decode_steps(h, k + 5, q, q, q, q, ev, nullptr) == TOVA_OK);
    EXPECT(tova_prefill(h, 19, q, q, q, q, ev, nullptr) == TOVA_OK);
    const int rs = tova_decode_steps_static(h, 7, q, q, q, q, ev, nullptr);
    EXPECT(rs == TOVA_OK || rs == TOVA_ETOOBIG);
    int64_t t = -1;
    EXPECT(tova_cache_tokens_seen(h, &t) == TOVA_OK && t == 1 + k + 5 + 19 + (rs == TOVA_OK ? 7 : 0));
    if (c.policy == TOVA_POLICY_TOVA) {
      const int rr = tova_decode_steps_repositioned(h, 4, q, q, q, q, ev, 0.f, nullptr);
      EXPECT(rr == TOVA_OK || rr == TOVA_ENOSUP);
      EXPECT(tova_policy_step(h, reinterpret_cast<const float*>(q), q, q, ev, nullptr) == TOVA_OK);
    } else {
      EXPECT(tova_decode_steps_repositioned(h, 4, q, q, q, q, ev, 0.f, nullptr) == TOVA_ENOSUP);
      EXPECT(tova_policy_step(h, reinterpret_cast<const float*>(q), q, q, ev, nullptr) == TOVA_ENOSUP);
    }
    {  // the replayable step: refused while the cache fills, counted like any step when run eagerly
      EXPECT(tova_cache_set_tokens_seen(h, k - 1 > 0 ? k - 1 : 0) == TOVA_OK);
      if (k > 1) EXPECT(tova_decode_step_graph(h, q, q, q, q, ev, nullptr) == TOVA_ENOSUP);
      EXPECT(tova_cache_set_tokens_seen(h, k + 3) == TOVA_OK);
      EXPECT(tova_cache_publish_tokens_seen(h, nullptr) == TOVA_OK);
      EXPECT(tova_decode_step_graph(h, q, q, q, q, ev, nullptr) == TOVA_OK);
      EXPECT(tova_cache_tokens_seen(h, &t) == TOVA_OK && t == k + 4);
      int64_t td = -1;
      EXPECT(tova_cache_fetch_tokens_seen(h, nullptr, &td) == TOVA_OK && td == 0);   // (the stub's device memory reads 0)
      EXPECT(tova_decode_step_graph(nullptr, q, q, q, q, ev, nullptr) == TOVA_EINVAL);
    }
    int32_t gave_up = 7, blocks = -1;
    EXPECT(tova_cache_status(h, nullptr, &gave_up) == TOVA_OK && gave_up == 0);
    EXPECT(tova_cache_recover(h, k, nullptr) == TOVA_OK && tova_cache_tokens_seen(h, &t) == TOVA_OK && t == k);
    EXPECT(tova_cache_multi_step_blocks(h, &blocks) == TOVA_OK && blocks >= 0);
    EXPECT(tova_cache_set_tokens_seen(h, (int64_t)1 << 31) == TOVA_ENOSUP);
    EXPECT(tova_cache_set_tokens_seen(h, 0x7fffffff) == TOVA_OK);
    EXPECT(tova_decode_steps(h, 1, q, q, q, q, ev, nullptr) == TOVA_ENOSUP);                 // the token index would leave 32 bits
    EXPECT(tova::g_launches > before);
    EXPECT(tova_cache_destroy(h) == TOVA_OK);
  }
  EXPECT(std::strcmp(tova_strerror(TOVA_OK), "ok") == 0 && std::strlen(tova_strerror(TOVA_ETOOBIG)) > 10);
  std::printf("host_sanitizer: %ld configurations planned (%ld valid), %ld stub launches, all as expected\n", configs, valid,
              tova::g_launches);
  return 0;
}
