// Host-side sanitizer driver for the C-ABI layer (CPU only, never launches a kernel that could run: the
// library it links is a host-only build without device code, and no device is made visible).
// Drives argument validation, the work plans and the workspace-size arithmetic with extreme sizes under
// AddressSanitizer / UndefinedBehaviorSanitizer (signed and unsigned integer overflow included).
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "msa.h"

static int fails = 0;
#define CHECK(cond)                                              \
  do {                                                           \
    if (!(cond)) {                                               \
      std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); \
      ++fails;                                                   \
    }                                                            \
  } while (0)

static msa_config_t cfg(int32_t N, int32_t G, int32_t P, int32_t Hq, int32_t Hkv, int32_t d) {
  msa_config_t c{};
  c.n_docs = N; c.doc_len = G; c.chunk = P; c.n_q_heads = Hq; c.n_kv_heads = Hkv; c.head_dim = d;
  c.rope_base = 1e6f; c.sim = MSA_SIM_COS; c.select_scope = MSA_SCOPE_GROUP;
  return c;
}

int main() {
  setenv("HIP_VISIBLE_DEVICES", "-1", 1);
  setenv("ROCR_VISIBLE_DEVICES", "", 1);
  void* p = reinterpret_cast<void*>(0x10000);
  const size_t big = ~(size_t)0 >> 1;

  // ---- sizes at the limits: N*C just below 2^31 keys per head, B*M = 2^20 query tokens, k = 64 ----
  const int32_t Ns[] = {1, 2, 15, 17, 97656, (1 << 28) - 1, 0x7fffffff / 16};
  const int32_t BMs[][2] = {{1, 1}, {8, 1}, {33, 1}, {1, 2048}, {1 << 10, 1 << 10}, {1, 1 << 20}, {65535, 1}};
  const int32_t ks[] = {1, 8, 16, 17, 32, 64};
  for (int32_t N : Ns)
    for (int C : {1, 2, 4, 8, 16})
      for (int d : {64, 128})
        for (int scope : {MSA_SCOPE_GROUP, MSA_SCOPE_ALL})
          for (int pool : {0, 1}) {
            if ((int64_t)N * C * 8 > 0x7fffffffLL) continue;  // doc_len = C * P must be an int32
            msa_config_t c = cfg(N, C * 8, 8, 32, 8, d);
            c.select_scope = scope;
            c.token_pool = pool;
            const size_t kr = msa_routing_keys_bytes(&c), in = msa_inv_norm_bytes(&c);
            const unsigned __int128 keys = ((unsigned __int128)N * C + 15) / 16 * 16;
            CHECK((unsigned __int128)kr == keys * 8 * d * 2);
            CHECK((unsigned __int128)in == keys * 8 * 4);
            for (auto& bm : BMs)
              for (int32_t k : ks) {
                const size_t ws = msa_score_topk_workspace_bytes(&c, bm[0], bm[1], k);
                if (k > N) { CHECK(ws == 0); continue; }
                CHECK(ws > 0 && ws % 256 == 0);
                // at least one candidate list of k keys per (selection, query token)
                const unsigned __int128 lo = (unsigned __int128)(scope == MSA_SCOPE_ALL ? 1 : 8) * bm[0] * bm[1] * k * 8;
                CHECK((unsigned __int128)ws >= lo);
                // a valid request reaches the launch stage and fails there (no device code, no device)
                const int rc = msa_score_topk(&c, p, bm[0], bm[1], p, (const float*)p, k, (int32_t*)p, (float*)p, p, big, nullptr);
                CHECK(rc == MSA_ERR_HIP);
                CHECK(msa_score_topk(&c, p, bm[0], bm[1], p, (const float*)p, k, (int32_t*)p, (float*)p, p, ws - 1, nullptr) == MSA_ERR_WORKSPACE);
                const int rn = msa_score_topk_noalloc(&c, p, bm[0], bm[1], p, (const float*)p, k, (int32_t*)p, (float*)p, nullptr);
                CHECK(rn == (ws > msa_noalloc_scratch_bytes() ? MSA_ERR_WORKSPACE : MSA_ERR_HIP));
              }
          }
  // ---- attention plans: long documents, many tokens, the largest local context -------------------
  for (int32_t G : {32, 512, 1 << 20})
    for (int32_t Lloc : {0, 1, 2048, (1 << 24) - 1024})
      for (auto& bm : BMs)
        for (int32_t k : ks)
          for (int pool : {0, 1}) {
            msa_config_t c = cfg(1000, G, 32, 32, 8, 128);
            c.token_pool = pool;
            const size_t ws = msa_sparse_attend_workspace_bytes(&c, bm[0], bm[1], k, Lloc);
            if ((int64_t)bm[0] * bm[1] > 65535) { CHECK(ws == 0); continue; }
            CHECK(ws > 0 && ws % 256 == 0);
            CHECK((unsigned __int128)ws >= (unsigned __int128)bm[0] * bm[1] * 32 * 128 * 4);
            const int rc = msa_sparse_attend(&c, p, bm[0], bm[1], p, p, (const int32_t*)p, k, p, p, Lloc, 512, (const int32_t*)p, p,
                                             (float*)p, p, big, nullptr);
            CHECK(rc == MSA_ERR_HIP);
            CHECK(msa_sparse_attend(&c, p, bm[0], bm[1], p, p, (const int32_t*)p, k, p, p, Lloc, 512, (const int32_t*)p, p,
                                    (float*)p, p, ws - 1, nullptr) == MSA_ERR_WORKSPACE);
          }
  // pooled bank with short stored-rotated documents
  {
    msa_config_t c = cfg(1 << 24, 8, 8, 32, 8, 128);
    c.bank_keys_rotated = 1;
    CHECK(msa_sparse_attend_workspace_bytes(&c, 8, 1, 64, 4096) > 0);
    CHECK(msa_fetch_slots(&c, 1 << 15, 1, 64) == (int64_t)(1 << 15) * 64);
  }
  // ---- index build / pooling over document ranges at the end of a huge bank ---------------------
  {
    msa_config_t c = cfg((1 << 28) - 1, 64, 8, 32, 8, 128);
    CHECK(msa_build_routing_keys(&c, p, (1 << 28) - 2, 1, p, (float*)p, nullptr) == MSA_ERR_HIP);
    CHECK(msa_build_routing_keys(&c, p, (1 << 28) - 2, 2, p, (float*)p, nullptr) == MSA_ERR_INVALID_ARG);
    CHECK(msa_build_routing_keys(&c, p, 0x7fffffff, 0x7fffffff, p, (float*)p, nullptr) == MSA_ERR_INVALID_ARG);
    CHECK(msa_pool_kv(&c, p, p, 0, 1 << 26, p, p, nullptr, nullptr) == MSA_ERR_HIP);
    CHECK(msa_pool_kv(&c, p, p, 0, (1 << 28) - 1, p, p, nullptr, nullptr) == MSA_ERR_UNSUPPORTED);  // > 2^31 workgroups
    CHECK(msa_build_routing_keys(&c, p, 0, (1 << 28) - 1, p, (float*)p, nullptr) == MSA_ERR_UNSUPPORTED);
    CHECK(msa_pool_kv(&c, p, p, 5, 0x7fffffff, p, p, nullptr, nullptr) == MSA_ERR_INVALID_ARG);
  }
  CHECK(msa_pooled_bank_bytes(100ull << 20, 64, 8, 128, 18, 2, 3) == (uint64_t)(168.75 * (1ull << 30)));
  std::printf(fails ? "boundary_sanitize: %d check(s) failed\n" : "boundary_sanitize: ok\n", fails);
  return fails ? 1 : 0;
}
