/*
 * msa.h -- C ABI of the routed-attention hot path of Memory Sparse Attention (MSA) on MI355X (gfx950).
 *
 * Three operations, in the order a query meets them (paper, Section 3.4.1 "Three-Stage Inference"):
 *   msa_build_routing_keys  offline, once per bank version: chunk-wise mean pooling phi(.) of the
 *                           keys (Section 3.2.1, text after Eq. 1) -> routing index
 *   msa_score_topk          online routing: relevance scores (Eq. 2), document score s_i = max_j S_ij,
 *                           top-k documents (Section 3.2.1)
 *   msa_sparse_attend       context assembly (Eq. 3) with document-wise RoPE (Section 3.2.2) and
 *                           attention (Eq. 4) over [selected documents ; local context]
 * and two around them:
 *   msa_pool_kv             offline: the pooled, position-encoded bank K-bar, V-bar of Stage 1 that Eq. 3
 *                           concatenates as printed (attended with bank_keys_rotated = 1)
 *   msa_fetch_selected      the host-DRAM tier of Section 3.4.2: gathers the selected documents from a
 *                           pinned host bank into a device staging bank
 *
 * Notation: N documents, G tokens per document, P chunk size, C = G/P chunks per document,
 * Hq query heads, Hkv key/value heads, r = Hq/Hkv, d head dimension, B sequences, M query tokens per
 * sequence, k selected documents, Lloc local-context tokens.  Query head h uses KV head g = h / r.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers (HIP), 16-byte aligned, dense, row-major in the index
 *     order written next to them (the one exception, the pinned host bank of msa_fetch_selected, says
 *     so); bf16 = bfloat16 bit patterns (uint16_t).  The config struct is a HOST pointer and is read
 *     before the call returns.
 *   - Ownership: the caller owns every buffer, workspace included.  The library allocates nothing,
 *     frees nothing and keeps no state between calls (msa_score_topk_noalloc brings its own fixed
 *     scratch buffer in place of a workspace).
 *   - Asynchrony: work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream); no call synchronises.  Outputs are valid once the stream reaches that point.
 *   - Errors: 0 on success, a negative msa_status otherwise.  Arguments are validated on the host
 *     before anything is enqueued, so an error return (other than MSA_ERR_HIP) means no work was
 *     launched and no GPU is needed to observe it.  No exceptions, no aborts, no printing.
 *   - Inputs are finite by contract.  msa_sparse_attend skips document ids outside [0, N) like -1 pads.
 */
#ifndef MSA_H_
#define MSA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void* msa_stream_t; /* hipStream_t */

typedef enum msa_status {
  MSA_OK = 0,
  MSA_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, k out of range, G % P != 0, ... */
  MSA_ERR_UNSUPPORTED = -2,   /* valid request outside what the kernels implement (see msa_config) */
  MSA_ERR_WORKSPACE = -3,     /* workspace_bytes smaller than the matching *_workspace_bytes()   */
  MSA_ERR_MISALIGNED = -4,    /* a tensor pointer is not 16-byte aligned                         */
  MSA_ERR_HIP = -5            /* a kernel launch failed (hipGetLastError)                        */
} msa_status;

enum { MSA_SIM_DOT = 0, MSA_SIM_COS = 1 };
enum { MSA_SCOPE_GROUP = 0, MSA_SCOPE_ALL = 1 };
enum { MSA_MAX_TOPK = 64 };

typedef struct msa_config {
  int32_t n_docs;       /* N >= 1                                                                  */
  int32_t doc_len;      /* G, tokens per document; G % P == 0; msa_sparse_attend needs G % 32 == 0
                           (or G in {1, 2, 4, 8, 16} with bank_keys_rotated)                       */
  int32_t chunk;        /* P, pooling size (paper: 64); must divide G.  Routing: P % 8 == 0 and C = G/P in
                           {1, 2, 4, 8, 16}; msa_pool_kv: P % 8 == 0; msa_sparse_attend does not read it */
  int32_t n_q_heads;    /* Hq, multiple of Hkv; r = Hq/Hkv <= 8                                    */
  int32_t n_kv_heads;   /* Hkv                                                                     */
  int32_t head_dim;     /* d, 64 or 128                                                            */
  float rope_base;      /* RoPE base (theta_u = base^(-2u/d)), e.g. 1e4 or 1e6                      */
  int32_t sim;          /* MSA_SIM_COS (paper, Eq. 2) or MSA_SIM_DOT                               */
  int32_t select_scope; /* MSA_SCOPE_GROUP: head mean over the r heads of a KV group, one selection
                           per KV head (S = Hkv).  MSA_SCOPE_ALL (literal Eq. 2): head mean over every
                           head, one selection shared by all heads (S = 1); Hkv in {1, 2, 4, 8}        */
  int32_t token_pool;   /* 0: one selection per query token (M' = M).  1 (literal Eq. 2): the document
                           score is the max over the M query tokens of a batch row, one selection per
                           batch row (M' = 1)                                                         */
  int32_t bank_keys_rotated; /* msa_sparse_attend only.  0: the bank holds raw keys, rotated in the gather with
                           positions 0..G-1 (default).  1: the bank's keys already carry their positions
                           (the pooled bank written by msa_pool_kv) and are used as stored; then doc_len
                           may also be 1, 2, 4, 8 or 16                                             */
  const int32_t* doc_lens; /* NULL: every document holds G tokens.  Else DEVICE int32 [N]: document i holds
                           doc_lens[i] tokens, stored in the first rows of its G-row slot of the bank (the
                           paper's G is an average document length, Section 5.1); the kernels clamp each
                           value to [1, G].  Read by msa_build_routing_keys, msa_pool_kv,
                           msa_sparse_attend and msa_fetch_selected; msa_score_topk does not need it (the
                           index already accounts for the lengths)                                    */
  void* profile_start_event; /* Optional per-call timing aid for benchmarks; NULL (both) = off.  A pair of   */
  void* profile_stop_event;  /* the caller's hipEvent_t (timing enabled): msa_score_topk / msa_sparse_attend
                           called with this config record start on the call's stream immediately before their
                           DOMINANT kernel (the scan over the routing index, all passes, or the scoring GEMM;
                           the gather-attention kernel, or the tiled kernel of a shared selection) and stop
                           immediately after it, so that its duration can be told from the small kernels
                           around it.  Nothing is kept after the call returns; other entry points ignore the
                           fields; exactly one of the two being NULL is MSA_ERR_INVALID_ARG                */
} msa_config_t;

/* Library version (major * 100 + minor). */
int msa_version(void);

/* Static, never-NULL description of a status code. */
const char* msa_status_string(int status);

/*
 * Layout of the routing index (output of msa_build_routing_keys, input of msa_score_topk).
 *
 * Keys are numbered c = i*C + j (chunk j of document i) and stored in TILES of 16 keys so that one
 * 64-lane wavefront reads a tile with four (d = 128) fully coalesced 1 KiB loads that are already in
 * MFMA operand order:
 *     KR[g][c / 16][dim / 8][c % 16][dim % 8]          bf16, g < Hkv, tiles = ceil(N*C / 16)
 *     inv_norm[g][c]                                     fp32, padded to tiles*16 entries per head
 * Slots past N*C in the last tile are zero.  A key in plain order [g][c][dim] is recovered by
 * swapping the two middle axes of a tile.
 */

/* Bytes of KR for this config (Hkv * tiles * 16 * d * 2).  0 if cfg is NULL or invalid. */
size_t msa_routing_keys_bytes(const msa_config_t* cfg);
/* Bytes of inv_norm for this config (Hkv * tiles * 16 * 4).  0 if cfg is NULL or invalid. */
size_t msa_inv_norm_bytes(const msa_config_t* cfg);

/*
 * Size of a POOLED bank in the paper's storage estimate (Section 3.4.2, "Tiered Memory Storage
 * Strategy"): n_tensors * n_layers * (tokens / P) * heads * d * bytes_per_elem.  With 100*2^20 tokens,
 * P = 64, 8 heads, d = 128, 18 layers, 2 bytes: 3 tensors -> 168.75 GiB, routing keys alone 56.25 GiB.
 */
uint64_t msa_pooled_bank_bytes(uint64_t tokens, uint32_t chunk, uint32_t heads, uint32_t head_dim,
                               uint32_t n_layers, uint32_t bytes_per_elem, uint32_t n_tensors);

/* Workspace requirements (bytes, multiple of 256).  0 if the arguments are invalid.  The attention workspace
 * holds the split-K partials and, where many query tokens share keys (token_pool = 1 with M >= 8, or the local
 * context with M >= 16), those keys rotated once: B * Hkv * ceil((k*G or 0) + Lloc, 32 rows) * d * 2 bytes more. */
size_t msa_score_topk_workspace_bytes(const msa_config_t* cfg, int32_t B, int32_t M, int32_t k);
size_t msa_sparse_attend_workspace_bytes(const msa_config_t* cfg, int32_t B, int32_t M, int32_t k,
                                         int32_t Lloc);

/*
 * Chunk-wise mean pooling of un-rotated keys into the routing index (Section 3.2.1, phi(.)):
 *     KR(g, i*C + j, :) = bf16_rne( (1/P) * sum_{t in chunk j} K[i][g][t][:] )      fp32 accumulate
 *     inv_norm(g, i*C + j) = 1 / max(||KR(g, i*C + j, :)||, 1e-12)                   of the ROUNDED key
 * for documents i in [doc_begin, doc_begin + doc_count), so a bank can be built or updated in pieces.
 * With cfg->doc_lens a document has ceil(len/P) chunks; its last chunk is the mean over the tokens it holds
 * (phi averages the tokens of a chunk).  The slots of the chunks a document does not have repeat the
 * document's chunk 0, key and norm: the document score is a max over chunks, so a repeated chunk never
 * changes it and msa_score_topk reads the index with no knowledge of the lengths.
 *   K         in   bf16 [N][Hkv][G][d]   (whole bank; only the addressed documents are read)
 *   KR        out  bf16, tiled layout above (whole index; only the addressed keys are written)
 *   inv_norm  out  fp32 [Hkv][tiles*16]; may be NULL iff cfg->sim == MSA_SIM_DOT
 */
int msa_build_routing_keys(const msa_config_t* cfg, const void* K, int32_t doc_begin,
                           int32_t doc_count, void* KR, float* inv_norm, msa_stream_t stream);

/*
 * The paper's own memory bank (Section 3.4.1, Stage 1; Section 3.2.1, Eq. 3): every document is encoded
 * with its own positions 0..G-1 (Section 3.2.2) and then chunk-mean pooled,
 *     Kbar[i][g][j][:] = bf16_rne( (1/P) * sum_{t in chunk j} RoPE(K[i][g][t][:], t) )
 *     Vbar[i][g][j][:] = bf16_rne( (1/P) * sum_{t in chunk j} V[i][g][t][:] )
 * for documents i in [doc_begin, doc_begin + doc_count).  The result is a bank of N documents of C = G/P
 * entries that msa_sparse_attend reads with a config whose doc_len = C and bank_keys_rotated = 1
 * (context length M + k G/P, Section 5.1).  With cfg->doc_lens the last chunk of a document is the mean over
 * the tokens it holds, the rows of chunks it does not have are zero, and pooled_lens receives the number of
 * chunks ceil(len/P) of every addressed document: the doc_lens of the pooled bank's config.
 *   K, V        in   bf16 [N][Hkv][G][d]
 *   Kbar, Vbar  out  bf16 [N][Hkv][C][d]   (either may be NULL to skip it)
 *   pooled_lens out  int32 [N]; may be NULL; written only when cfg->doc_lens is given
 */
int msa_pool_kv(const msa_config_t* cfg, const void* K, const void* V, int32_t doc_begin,
                int32_t doc_count, void* Kbar, void* Vbar, int32_t* pooled_lens, msa_stream_t stream);

/*
 * Routing (Section 3.2.1, Eq. 2 and the text after it), fused so chunk scores never reach memory:
 *     Sc(b,m,g,c) = (1/r) * sum_{h in group g} sim(q_route[b][m][h][:], KR(g,c,:))
 *     s(b,m,g,i)  = max_{j < C} Sc(b,m,g,i*C + j)
 *     out_idx[b][m][g][0..k) = the k documents with the largest s, ordered by (s descending,
 *                               document index ascending); out_score = their s.
 * sim = cosine: x.y / (max(|x|,1e-12) * max(|y|,1e-12)), or the plain dot product.
 * cfg->select_scope == MSA_SCOPE_ALL replaces the group mean by the mean over all Hq heads (each head against
 * the routing keys of its own KV group), giving one selection for all heads: S = 1 instead of S = Hkv.
 * cfg->token_pool == 1 takes, before the document max, the max of Sc over the M query tokens of batch row b,
 * giving one selection per batch row: M' = 1 instead of M' = M.  Both together are Eq. 2 as printed.
 *   q_route   in   bf16 [B][M][Hq][d]
 *   KR, inv_norm   as written by msa_build_routing_keys (inv_norm may be NULL iff sim == DOT)
 *   k              1 <= k <= min(N, MSA_MAX_TOPK)
 *   out_idx   out  int32 [B][M'][S][k]
 *   out_score out  fp32  [B][M'][S][k], may be NULL
 *   workspace      >= msa_score_topk_workspace_bytes(cfg, B, M, k); contents undefined on entry/exit
 * Scores are accumulated in fp32; each query is carried as a bf16 (hi, lo) pair, so a score differs
 * from exact arithmetic by a few 1e-6 relative.  (With many query tokens, cosine, d = 128 and eight chunks per
 * document the matrix product runs on the hi parts alone as a filter, and the reported scores of the winners are
 * recomputed in fp32 from the fp32 folded query: the selection is the same as with exact scores.  The filter's
 * error band assumes |KR row| * inv_norm <= 1.01, which holds for what msa_build_routing_keys writes; an index
 * from elsewhere must keep to it.)
 */
int msa_score_topk(const msa_config_t* cfg, const void* q_route, int32_t B, int32_t M,
                   const void* KR, const float* inv_norm, int32_t k, int32_t* out_idx,
                   float* out_score, void* workspace, size_t workspace_bytes, msa_stream_t stream);

/*
 * msa_score_topk for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical results; the workspace is a buffer of msa_noalloc_scratch_bytes() (32 MiB) built into
 * the library's device code (one copy per GPU, held until the process ends).  The call allocates and
 * frees nothing.  A request whose msa_score_topk_workspace_bytes() exceeds the built-in buffer returns
 * MSA_ERR_WORKSPACE before anything is enqueued (all five benchmark configurations fit).  The stream must
 * belong to the CURRENT device.  Every call on a GPU shares that GPU's buffer: calls that overlap on one GPU
 * (two streams, two threads) race -- serialise them or use msa_score_topk with separate workspaces.
 * The buffer keeps the previous call's contents; nothing in it needs to start at zero.
 */
size_t msa_noalloc_scratch_bytes(void);
int msa_score_topk_noalloc(const msa_config_t* cfg, const void* q_route, int32_t B, int32_t M,
                           const void* KR, const float* inv_norm, int32_t k, int32_t* out_idx,
                           float* out_score, msa_stream_t stream);

/*
 * Sparse attention (Eq. 3-4 with the position scheme of Section 3.2.2).  For query (b,m), head h of
 * KV group g, the keys are, in order:
 *     every token p < G (p < doc_lens[i] when cfg->doc_lens is given) of every document
 *         i = idx[b][m][g][j] >= 0:                                   RoPE(K[i][g][p][:], p)
 *     every local token t < Lloc with local_pos0 + t <= q_pos[b][m]:  RoPE(Kloc[b][g][t][:], local_pos0 + t)
 * with the matching un-rotated value rows, and
 *     out[b][m][h][:] = softmax_j( RoPE(q[b][m][h][:], q_pos[b][m]) . key_j / sqrt(d) ) . value_j
 *     lse[b][m][h]    = log sum_j exp( ... )          (natural log; -inf and out = 0 if no key is visible)
 * RoPE pairs element u with u + d/2, angle p * base^(-2u/d).  Positions restart at 0 in every document
 * (with cfg->bank_keys_rotated the bank keys are taken as stored, un-rotated here);
 * idx == -1 (or any id outside [0, N)) marks "no document"; a document listed twice is attended twice.
 *   q         in   bf16 [B][M][Hq][d]
 *   K, V      in   bf16 [N][Hkv][G][d]
 *   idx       in   int32 [B][M'][S][k], M' and S as msa_score_topk writes them for this cfg (row m' = 0 /
 *                  slot 0 is shared by all query tokens / all KV groups when M' = 1 / S = 1)
 *   Kloc,Vloc in   bf16 [B][Hkv][Lloc][d]; may be NULL iff Lloc == 0
 *   q_pos     in   int32 [B][M]
 *   out       out  bf16 [B][M][Hq][d]
 *   lse       out  fp32 [B][M][Hq], may be NULL
 *   workspace      >= msa_sparse_attend_workspace_bytes(cfg, B, M, k, Lloc)
 * Rotated keys are rounded to bf16 before the fp32-accumulated matrix products; queries and softmax
 * weights are carried as bf16 (hi, lo) pairs.
 */
int msa_sparse_attend(const msa_config_t* cfg, const void* q, int32_t B, int32_t M, const void* K,
                      const void* V, const int32_t* idx, int32_t k, const void* Kloc,
                      const void* Vloc, int32_t Lloc, int32_t local_pos0, const int32_t* q_pos,
                      void* out, float* lse, void* workspace, size_t workspace_bytes,
                      msa_stream_t stream);

/*
 * Tiered bank (Section 3.4.2): the K/V of the whole bank stay in HOST memory and only the selected documents
 * travel to the device, into a staging bank that msa_sparse_attend then reads.
 *   K_host, V_host  in   bf16 [N][Hkv][G][d] in pinned host memory that is mapped into the device's address
 *                        space (hipHostMalloc; anything else is refused with MSA_ERR_INVALID_ARG): one
 *                        kernel reads it directly over the host link
 *   idx             in   DEVICE int32 [B][M'][S][k] as msa_score_topk writes it for cfg
 *   K_stage,V_stage out  DEVICE bf16 [n_slots][Hkv][G][d], n_slots = msa_fetch_slots(cfg, B, M, k) = B*M'*k.
 *                        Entry (b, m', j) owns slot (b*M' + m')*k + j; of a slot only the (slot, g) slabs of
 *                        the KV heads g that select for that entry are written (all Hkv when S = 1)
 *   idx_stage       out  DEVICE int32 [B][M'][S][k]: the slot of every entry, -1 for entries that are -1 or
 *                        outside [0, N)
 *   lens_stage      out  DEVICE int32 [n_slots]: with cfg->doc_lens (then required, and only the rows a document
 *                        holds are copied) the length of the document in every slot, the doc_lens of the staging
 *                        bank's config; else ignored, may be NULL.  Lengths need one document per slot, so
 *                        cfg->doc_lens with S = Hkv > 1 is MSA_ERR_UNSUPPORTED
 * Then call msa_sparse_attend with a config whose n_docs = n_slots and doc_lens = lens_stage (or NULL; everything
 * else as cfg), K = K_stage,
 * V = V_stage, idx = idx_stage: the result is bit-identical to attending the bank in device memory.
 * Asynchronous on `stream`; there is no host synchronisation inside.
 */
int64_t msa_fetch_slots(const msa_config_t* cfg, int32_t B, int32_t M, int32_t k);
int msa_fetch_selected(const msa_config_t* cfg, const void* K_host, const void* V_host, const int32_t* idx,
                       int32_t B, int32_t M, int32_t k, void* K_stage, void* V_stage, int32_t* idx_stage,
                       int32_t* lens_stage, msa_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* MSA_H_ */
