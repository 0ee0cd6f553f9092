// Host-side declarations shared by the C-ABI layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/msa.h"

namespace msa {

// Validated, derived view of msa_config_t.
struct Dims {
  int N, G, P, C, Hq, Hkv, r, d;
  int cos;        // 1 = cosine, 0 = dot
  int scope_all;  // 1 = head mean over every head, one selection for all KV heads (literal Eq. 2)
  int token_pool; // 1 = document score is the max over the M tokens of a batch row (literal Eq. 2)
  float base;
  const int32_t* lens;  // device [N] document lengths, or null (every document holds G tokens)
  hipEvent_t prof_start, prof_stop;  // the caller's events around the dominant kernel of this call, or null
  int64_t NC;     // N * C routing keys per KV head
  int64_t tiles;  // ceil(NC / 16) tiles of 16 keys per KV head
};

// Work split of the MFMA-bound scoring path for many query tokens (msa_score_gemm.hip).
struct GemmPlan {
  int all_heads;         // 1: head mean over every head (select_scope = ALL): score_gemm_all_kernel
  int n_qblocks;         // blocks of 256 (128: k > 8, or all heads) query tokens
  int n_splits;          // key-range splits per (head, token block)
  int stages_per_split;  // 64-key stages per split (all heads: ranges of stages per split)
  size_t off_lists;      // byte offset of the candidate lists (after the folded fp32 queries)
  // One-pass filter (cosine, d = 128, eight chunks per document, one selection per KV group): the product runs on
  // the bf16 hi parts of the folded queries alone; every document whose one-pass score lies within twice the error
  // bound of the k-th best one-pass score is scored again exactly, and token blocks whose per-lane lists overflow
  // inside that band are redone by the two-pass kernel.
  int filter;            // 1: the filter applies
  int list_len;          // entries per per-lane list (8: k <= 8, 16: k <= 16)
  int tokens_per_wg;     // query tokens per workgroup = per fallback flag
  size_t off_eps;        // fp32 [BM][Hkv]: bound on |one-pass score - exact score| per (token, KV group)
  size_t off_flags;      // int32 [Hkv][n_qblocks]: 1 = this token block is redone by the two-pass kernel
  size_t off_flists;     // 64-bit keys [Hkv][BM][n_splits][2][list_len]: the per-lane lists of the one-pass product
                         // (the two-pass kernel's lists, off_lists, reuse this memory afterwards)
  size_t ws_bytes;
};
constexpr int kFilterMaxCand = 32;
bool gemm_path_applies(const Dims& dm, int BM, int k);
GemmPlan plan_score_gemm(const Dims& dm, int BM, int k);
// Enqueues the scoring kernels.  Without the filter the per-split lists are left for score_merge_kernel.  With it
// the exact winners of every token are written to out_idx / out_score (or out_key: sorted 64-bit keys, token pooling),
// and the lists of the flagged token blocks are left for a merge that is gated by *gate_flags (device int32
// [Hkv][n_qblocks], null without the filter).
int launch_score_gemm_scan(const Dims& dm, const GemmPlan& pl, const void* q_route, int BM,
                           const void* KR, const float* inv_norm, int k, void* ws, hipStream_t st,
                           int32_t* out_idx, float* out_score, unsigned long long* out_key, const int** gate_flags);

// Work split of the routing scan (depends only on the problem size, so the workspace size is a
// pure function of the arguments).
struct ScorePlan {
  int n_splits;          // blocks per KV head
  int q_per_pass;        // queries scored per launch (8 or 16)
  int n_pass;
  int mode;              // scan mode: 0 filter, 1 dense lists, 2 score matrix + row top-k
  int tiles_per_wave;    // mode 2: contiguous tiles per wave
  size_t off_mat;        // mode 2: byte offset of the fp32 score matrix [Hkv][BM][N]
  int exchange;          // 1: waves exchange running maxima to tighten their thresholds
  int it_publish, it_adopt;
  size_t off_gmax;       // byte offset of the exchange buffer inside the workspace
  size_t off_qop;        // byte offset of the prepared query operands
  int n_qtiles;          // 8-query operand tiles (padded to whole passes)
  int all_heads;         // 1: score_scan_all_kernel (scope ALL with more than one KV head)
  int n_sel;             // selections per query token: Hkv, or 1 for scope ALL
  size_t off_tok;        // byte offset of the per-token winner keys (token pooling)
  int merge_parts;       // > 1: two-level merge, first level over merge_lpp lists per block
  int merge_lpp;
  size_t off_part;       // byte offset of the first-level winners
  int use_gemm;          // 1: many query tokens -> the GEMM path below
  GemmPlan gemm;
  size_t ws_bytes;
};
ScorePlan plan_score(const Dims& dm, int BM, int k);

// record the caller's per-call events (msa_config_t.profile_*_event) around the dominant kernel; null = off
inline void profile_mark(const Dims& dm, bool stop, hipStream_t st) {
  hipEvent_t e = stop ? dm.prof_stop : dm.prof_start;
  if (e != nullptr) (void)hipEventRecord(e, st);
}

struct AttendPlan {
  int steps_mem;         // 32-key steps over the selected documents, ceil(k * G / 32)
  int steps_total;       // + ceil(Lloc / 32)
  int steps_per_split;
  int n_splits;
  int prefill;           // 1: shared selection and many tokens -> attend_prefill_kernel
  int split_local;       // 1: per-token selections and many tokens: the selected documents go through the decode
                         //    kernel, the local context (shared by the tokens) through attend_prefill_kernel
  int mem_splits, mem_steps_per_split;  // split_local: decode kernel over the documents
  int loc_splits, loc_steps_per_split;  // split_local: tiled kernel over the local context
  int tpw, n_ttiles;     // prefill: tokens per wave (32 / r), token tiles (4 waves each) per batch row
  size_t off_ml;         // byte offset of the (m, l) pairs inside the workspace
  int fused_merge;       // 1: the decode kernel's last-arriving workgroup of a (query, KV head) merges the splits
  size_t off_tickets;    // byte offset of the arrival counters [B*M][Hkv] (64-bit)
  size_t off_krot;       // tiled kernel: byte offset of the once-rotated keys (0 = none)
  int krot_steps;        // steps per (batch row, KV head) held there
  size_t ws_bytes;
};
AttendPlan plan_attend(const Dims& dm, int B, int M, int k, int Lloc, int bank_keys_rotated);

int launch_build(const Dims& dm, const void* K, int doc_begin, int doc_count, void* KR,
                 float* inv_norm, hipStream_t st);
int launch_score(const Dims& dm, const ScorePlan& pl, const void* q_route, int B, int M, const void* KR,
                 const float* inv_norm, int k, int32_t* out_idx, float* out_score, void* ws,
                 hipStream_t st);
int launch_attend(const Dims& dm, const AttendPlan& pl, const void* q, int B, int M, const void* K,
                  const void* V, const int32_t* idx, int k, const void* Kloc, const void* Vloc,
                  int Lloc, int pos0, const int32_t* q_pos, void* out, float* lse, void* ws,
                  int bank_keys_rotated, hipStream_t st);
int launch_pool_kv(const Dims& dm, const void* K, const void* V, int doc_begin, int doc_count,
                   void* Kbar, void* Vbar, int32_t* pooled_lens, hipStream_t st);

int launch_fetch(const Dims& dm, const void* K_dev_view, const void* V_dev_view, const int32_t* idx,
                 long long n_rows, int k, void* K_stage, void* V_stage, int32_t* idx_stage,
                 int32_t* lens_stage, hipStream_t st);

inline size_t round_up256(size_t x) { return (x + 255) & ~(size_t)255; }

// A 48-bit non-zero value that differs from call to call (clock ticks through a 64-bit mixer): the tag of the
// arrival counters of one launch (arrive_at in msa_device.h).  It only has to differ from whatever the
// caller's workspace happens to hold.
unsigned long long launch_nonce48();

}  // namespace msa
