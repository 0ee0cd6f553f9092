// C-ABI layer: argument validation (host only, before anything is enqueued), work plans, launches.
#include "msa_host.h"

#include <chrono>
#include <mutex>

namespace msa {

static bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// (the mixer multiplies modulo 2^64 on purpose)
__attribute__((no_sanitize("unsigned-integer-overflow"))) unsigned long long launch_nonce48() {
  unsigned long long z = (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count();
  z += 0x9E3779B97F4A7C15ull;  // splitmix64 finaliser
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  z &= 0xFFFFFFFFFFFFull;
  return z ? z : 1ull;
}

// Returns MSA_OK and fills dm, or the status that describes what is wrong with cfg.  The limits on
// the chunking belong to those who read it: routing needs whole 16-byte pieces per chunk and a
// power-of-two C <= 16 (a tile holds whole documents), pooling only the former, attention neither.
enum DimsFor { kForRouting, kForPooling, kForAttend };
static int make_dims(const msa_config_t* cfg, Dims* dm, DimsFor use = kForRouting) {
  if (cfg == nullptr) return MSA_ERR_INVALID_ARG;
  if (cfg->n_docs < 1 || cfg->doc_len < 1 || cfg->chunk < 1 || cfg->n_q_heads < 1 ||
      cfg->n_kv_heads < 1 || cfg->head_dim < 1)
    return MSA_ERR_INVALID_ARG;
  if (cfg->doc_len % cfg->chunk != 0) return MSA_ERR_INVALID_ARG;
  if (cfg->n_q_heads % cfg->n_kv_heads != 0) return MSA_ERR_INVALID_ARG;
  if (cfg->sim != MSA_SIM_DOT && cfg->sim != MSA_SIM_COS) return MSA_ERR_INVALID_ARG;
  if (cfg->select_scope != MSA_SCOPE_GROUP && cfg->select_scope != MSA_SCOPE_ALL)
    return MSA_ERR_INVALID_ARG;
  if (cfg->token_pool != 0 && cfg->token_pool != 1) return MSA_ERR_INVALID_ARG;
  if (cfg->bank_keys_rotated != 0 && cfg->bank_keys_rotated != 1) return MSA_ERR_INVALID_ARG;
  if (!(cfg->rope_base > 1.0f)) return MSA_ERR_INVALID_ARG;
  if ((cfg->profile_start_event == nullptr) != (cfg->profile_stop_event == nullptr)) return MSA_ERR_INVALID_ARG;
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return MSA_ERR_UNSUPPORTED;
  const int C = cfg->doc_len / cfg->chunk;
  if (use != kForAttend && cfg->chunk % 8 != 0) return MSA_ERR_UNSUPPORTED;
  if (use == kForRouting && (!pow2(C) || C > 16)) return MSA_ERR_UNSUPPORTED;
  if (cfg->n_q_heads / cfg->n_kv_heads > 8) return MSA_ERR_UNSUPPORTED;
  if (use == kForRouting && cfg->select_scope == MSA_SCOPE_ALL && cfg->n_kv_heads != 1 &&
      cfg->n_kv_heads != 2 && cfg->n_kv_heads != 4 && cfg->n_kv_heads != 8)
    return MSA_ERR_UNSUPPORTED;
  dm->N = cfg->n_docs;
  dm->G = cfg->doc_len;
  dm->P = cfg->chunk;
  dm->C = C;
  dm->Hq = cfg->n_q_heads;
  dm->Hkv = cfg->n_kv_heads;
  dm->r = cfg->n_q_heads / cfg->n_kv_heads;
  dm->d = cfg->head_dim;
  dm->cos = cfg->sim == MSA_SIM_COS;
  dm->scope_all = cfg->select_scope == MSA_SCOPE_ALL;
  dm->token_pool = cfg->token_pool;
  dm->base = cfg->rope_base;
  dm->lens = cfg->doc_lens;
  dm->prof_start = (hipEvent_t)cfg->profile_start_event;
  dm->prof_stop = (hipEvent_t)cfg->profile_stop_event;
  dm->NC = (int64_t)dm->N * C;
  dm->tiles = (dm->NC + 15) / 16;
  return MSA_OK;
}

// Document lengths the attention kernels read: whole 32-key steps, or (bank keys stored rotated) a
// short power of two so that a step spans whole documents.
static bool attend_doc_len_ok(const msa_config_t* cfg) {
  if (cfg->doc_len % 32 == 0) return true;
  return cfg->bank_keys_rotated == 1 && pow2(cfg->doc_len) && cfg->doc_len <= 16;
}

static bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
static bool misaligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; }

// ---- scratch memory of msa_score_topk_noalloc ---------------------------------------------------
// A file-scope device array takes the place of the caller's workspace for callers that cannot
// allocate.  Every device the library runs on holds its own copy at its own address; in host code the
// array's name is only a handle for hipGetSymbolAddress, never an address to hand to a kernel.
constexpr size_t kNoAllocScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices];  // per device, filled at the first call on that device

// Address of `scratch` on the CURRENT device (looked up once per device, with that device current).
static int scratch_on_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return MSA_ERR_HIP;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return MSA_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MSA_OK;
}

}  // namespace msa

using namespace msa;

extern "C" {

int msa_version(void) { return 105; }

const char* msa_status_string(int status) {
  switch (status) {
    case MSA_OK: return "ok";
    case MSA_ERR_INVALID_ARG: return "invalid argument";
    case MSA_ERR_UNSUPPORTED: return "valid request not supported by this build";
    case MSA_ERR_WORKSPACE: return "workspace too small";
    case MSA_ERR_MISALIGNED: return "pointer not 16-byte aligned";
    case MSA_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}

size_t msa_routing_keys_bytes(const msa_config_t* cfg) {
  Dims dm;
  if (make_dims(cfg, &dm) != MSA_OK) return 0;
  return (size_t)dm.Hkv * (size_t)dm.tiles * 16 * (size_t)dm.d * 2;
}

size_t msa_inv_norm_bytes(const msa_config_t* cfg) {
  Dims dm;
  if (make_dims(cfg, &dm) != MSA_OK) return 0;
  return (size_t)dm.Hkv * (size_t)dm.tiles * 16 * sizeof(float);
}

uint64_t msa_pooled_bank_bytes(uint64_t tokens, uint32_t chunk, uint32_t heads, uint32_t head_dim,
                               uint32_t n_layers, uint32_t bytes_per_elem, uint32_t n_tensors) {
  if (chunk == 0 || tokens % chunk != 0) return 0;
  return (uint64_t)n_tensors * n_layers * (tokens / chunk) * heads * head_dim * bytes_per_elem;
}

size_t msa_score_topk_workspace_bytes(const msa_config_t* cfg, int32_t B, int32_t M, int32_t k) {
  Dims dm;
  if (make_dims(cfg, &dm) != MSA_OK) return 0;
  if (B < 1 || M < 1 || k < 1 || k > MSA_MAX_TOPK || k > dm.N) return 0;
  if ((int64_t)B * M > (1 << 20)) return 0;
  return plan_score(dm, B * M, k).ws_bytes;
}

size_t msa_sparse_attend_workspace_bytes(const msa_config_t* cfg, int32_t B, int32_t M, int32_t k,
                                         int32_t Lloc) {
  Dims dm;
  if (make_dims(cfg, &dm, kForAttend) != MSA_OK) return 0;
  if (B < 1 || M < 1 || k < 1 || k > MSA_MAX_TOPK || Lloc < 0) return 0;
  if ((int64_t)B * M > 65535 || !attend_doc_len_ok(cfg)) return 0;
  return plan_attend(dm, B, M, k, Lloc, cfg->bank_keys_rotated).ws_bytes;
}

int msa_build_routing_keys(const msa_config_t* cfg, const void* K, int32_t doc_begin,
                           int32_t doc_count, void* KR, float* inv_norm, msa_stream_t stream) {
  Dims dm;
  const int rc = make_dims(cfg, &dm);
  if (rc != MSA_OK) return rc;
  if (K == nullptr || KR == nullptr) return MSA_ERR_INVALID_ARG;
  if (inv_norm == nullptr && dm.cos) return MSA_ERR_INVALID_ARG;
  if (doc_begin < 0 || doc_count < 0 || (int64_t)doc_begin + doc_count > dm.N)
    return MSA_ERR_INVALID_ARG;
  if (misaligned(K) || misaligned(KR) || misaligned(inv_norm) || misaligned4(dm.lens))
    return MSA_ERR_MISALIGNED;
  return launch_build(dm, K, doc_begin, doc_count, KR, inv_norm, (hipStream_t)stream);
}

int msa_pool_kv(const msa_config_t* cfg, const void* K, const void* V, int32_t doc_begin,
                int32_t doc_count, void* Kbar, void* Vbar, int32_t* pooled_lens, msa_stream_t stream) {
  Dims dm;
  const int rc = make_dims(cfg, &dm, kForPooling);
  if (rc != MSA_OK) return rc;
  if ((Kbar != nullptr && K == nullptr) || (Vbar != nullptr && V == nullptr)) return MSA_ERR_INVALID_ARG;
  if (doc_begin < 0 || doc_count < 0 || (int64_t)doc_begin + doc_count > dm.N)
    return MSA_ERR_INVALID_ARG;
  if (misaligned(K) || misaligned(V) || misaligned(Kbar) || misaligned(Vbar) || misaligned4(dm.lens) ||
      misaligned4(pooled_lens))
    return MSA_ERR_MISALIGNED;
  return launch_pool_kv(dm, K, V, doc_begin, doc_count, Kbar, Vbar, pooled_lens, (hipStream_t)stream);
}

int64_t msa_fetch_slots(const msa_config_t* cfg, int32_t B, int32_t M, int32_t k) {
  Dims dm;
  if (make_dims(cfg, &dm, kForAttend) != MSA_OK) return 0;
  if (B < 1 || M < 1 || k < 1 || k > MSA_MAX_TOPK) return 0;
  return (int64_t)B * (dm.token_pool ? 1 : M) * k;
}

int msa_fetch_selected(const msa_config_t* cfg, const void* K_host, const void* V_host,
                       const int32_t* idx, int32_t B, int32_t M, int32_t k, void* K_stage,
                       void* V_stage, int32_t* idx_stage, int32_t* lens_stage, msa_stream_t stream) {
  Dims dm;
  const int rc = make_dims(cfg, &dm, kForAttend);
  if (rc != MSA_OK) return rc;
  if (K_host == nullptr || V_host == nullptr || idx == nullptr || K_stage == nullptr ||
      V_stage == nullptr || idx_stage == nullptr)
    return MSA_ERR_INVALID_ARG;
  if (B < 1 || M < 1 || k < 1) return MSA_ERR_INVALID_ARG;
  if (dm.lens != nullptr && lens_stage == nullptr) return MSA_ERR_INVALID_ARG;
  if (k > MSA_MAX_TOPK) return MSA_ERR_UNSUPPORTED;
  if (((int64_t)dm.G * dm.d * 2) % 16 != 0) return MSA_ERR_UNSUPPORTED;
  // a staging slot holds one document per KV head: a length per slot needs them to be the same document
  if (dm.lens != nullptr && !dm.scope_all && dm.Hkv > 1) return MSA_ERR_UNSUPPORTED;
  if (misaligned(K_host) || misaligned(V_host) || misaligned(idx) || misaligned(K_stage) ||
      misaligned(V_stage) || misaligned(idx_stage) || misaligned4(dm.lens) || misaligned4(lens_stage))
    return MSA_ERR_MISALIGNED;
  // the kernel dereferences the host bank: it must be pinned and mapped into the device's address space
  void* Kd = nullptr;
  void* Vd = nullptr;
  {
    hipPointerAttribute_t ka, va;
    const bool k_ok = hipPointerGetAttributes(&ka, K_host) == hipSuccess && ka.type == hipMemoryTypeHost &&
                      ka.devicePointer != nullptr;
    const bool v_ok = k_ok && hipPointerGetAttributes(&va, V_host) == hipSuccess &&
                      va.type == hipMemoryTypeHost && va.devicePointer != nullptr;
    if (!k_ok || !v_ok) {
      (void)hipGetLastError();  // clear the sticky error of a failed query
      return MSA_ERR_INVALID_ARG;
    }
    Kd = ka.devicePointer;
    Vd = va.devicePointer;
  }
  const long long n_rows = (long long)B * (dm.token_pool ? 1 : M);
  return launch_fetch(dm, Kd, Vd, idx, n_rows, k, K_stage, V_stage, idx_stage, lens_stage,
                      (hipStream_t)stream);
}

int msa_score_topk(const msa_config_t* cfg, const void* q_route, int32_t B, int32_t M,
                   const void* KR, const float* inv_norm, int32_t k, int32_t* out_idx,
                   float* out_score, void* workspace, size_t workspace_bytes, msa_stream_t stream) {
  Dims dm;
  const int rc = make_dims(cfg, &dm);
  if (rc != MSA_OK) return rc;
  if (q_route == nullptr || KR == nullptr || out_idx == nullptr || workspace == nullptr)
    return MSA_ERR_INVALID_ARG;
  if (inv_norm == nullptr && dm.cos) return MSA_ERR_INVALID_ARG;
  if (B < 1 || M < 1 || (int64_t)B * M > (1 << 20)) return MSA_ERR_INVALID_ARG;
  if (k < 1 || k > dm.N) return MSA_ERR_INVALID_ARG;
  if (k > MSA_MAX_TOPK) return MSA_ERR_UNSUPPORTED;
  if (misaligned(q_route) || misaligned(KR) || misaligned(inv_norm) || misaligned(out_idx) ||
      misaligned(out_score) || misaligned(workspace))
    return MSA_ERR_MISALIGNED;
  const ScorePlan pl = plan_score(dm, B * M, k);
  if (workspace_bytes < pl.ws_bytes) return MSA_ERR_WORKSPACE;
  return launch_score(dm, pl, q_route, B, M, KR, inv_norm, k, out_idx, out_score, workspace,
                      (hipStream_t)stream);
}

size_t msa_noalloc_scratch_bytes(void) { return kNoAllocScratchBytes; }

int msa_score_topk_noalloc(const msa_config_t* cfg, const void* q_route, int32_t B, int32_t M,
                           const void* KR, const float* inv_norm, int32_t k, int32_t* out_idx,
                           float* out_score, msa_stream_t stream) {
  Dims dm;
  const int rc = make_dims(cfg, &dm);
  if (rc != MSA_OK) return rc;
  if (q_route == nullptr || KR == nullptr || out_idx == nullptr) return MSA_ERR_INVALID_ARG;
  if (inv_norm == nullptr && dm.cos) return MSA_ERR_INVALID_ARG;
  if (B < 1 || M < 1 || (int64_t)B * M > (1 << 20)) return MSA_ERR_INVALID_ARG;
  if (k < 1 || k > dm.N) return MSA_ERR_INVALID_ARG;
  if (k > MSA_MAX_TOPK) return MSA_ERR_UNSUPPORTED;
  if (misaligned(q_route) || misaligned(KR) || misaligned(inv_norm) || misaligned(out_idx) ||
      misaligned(out_score))
    return MSA_ERR_MISALIGNED;
  const ScorePlan pl = plan_score(dm, B * M, k);
  if (pl.ws_bytes > kNoAllocScratchBytes) return MSA_ERR_WORKSPACE;  // beyond the built-in scratch
  void* ws = nullptr;
  const int rs = scratch_on_current_device(&ws);
  if (rs != MSA_OK) return rs;
  // The kernels take the scratch address exactly as they take a caller's workspace; nothing in it has
  // to start at zero (every buffer of the plan is written before it is read within the call).
  return launch_score(dm, pl, q_route, B, M, KR, inv_norm, k, out_idx, out_score, ws,
                      (hipStream_t)stream);
}

int msa_sparse_attend(const msa_config_t* cfg, const void* q, int32_t B, int32_t M, const void* K,
                      const void* V, const int32_t* idx, int32_t k, const void* Kloc,
                      const void* Vloc, int32_t Lloc, int32_t local_pos0, const int32_t* q_pos,
                      void* out, float* lse, void* workspace, size_t workspace_bytes,
                      msa_stream_t stream) {
  Dims dm;
  const int rc = make_dims(cfg, &dm, kForAttend);
  if (rc != MSA_OK) return rc;
  if (q == nullptr || K == nullptr || V == nullptr || idx == nullptr || q_pos == nullptr ||
      out == nullptr || workspace == nullptr)
    return MSA_ERR_INVALID_ARG;
  if (B < 1 || M < 1 || Lloc < 0 || local_pos0 < 0) return MSA_ERR_INVALID_ARG;
  if (Lloc > 0 && (Kloc == nullptr || Vloc == nullptr)) return MSA_ERR_INVALID_ARG;
  if (k < 1) return MSA_ERR_INVALID_ARG;
  if (k > MSA_MAX_TOPK || (int64_t)B * M > 65535 || !attend_doc_len_ok(cfg))
    return MSA_ERR_UNSUPPORTED;
  if ((int64_t)local_pos0 + Lloc > (1 << 24)) return MSA_ERR_UNSUPPORTED;
  if (misaligned(q) || misaligned(K) || misaligned(V) || misaligned(idx) || misaligned(Kloc) ||
      misaligned(Vloc) || misaligned(q_pos) || misaligned(out) || misaligned(lse) ||
      misaligned(workspace) || misaligned4(dm.lens))
    return MSA_ERR_MISALIGNED;
  const AttendPlan pl = plan_attend(dm, B, M, k, Lloc, cfg->bank_keys_rotated);
  if (workspace_bytes < pl.ws_bytes) return MSA_ERR_WORKSPACE;
  return launch_attend(dm, pl, q, B, M, K, V, idx, k, Kloc, Vloc, Lloc, local_pos0, q_pos, out,
                       lse, workspace, cfg->bank_keys_rotated, (hipStream_t)stream);
}

}  // extern "C"
