// msa_score_topk: relevance scores (paper, Eq. 2), document max and top-k (Section 3.2.1), fused so
// that chunk scores never leave the chip.  The routing index is streamed from HBM exactly once per
// group of up to 16 queries; this is the O(M L / P) term that dominates online cost (Section 5.1).
//
// Algebra.  With cosine similarity the head mean of Eq. 2 for KV group g is
//     (1/r) sum_h  q_h . key / (|q_h| |key|)  =  ( (1/r) sum_h q_h/|q_h| ) . key * (1/|key|),
// so the r heads of a group fold into ONE fp32 routing query per (token, group) and the scan is a
// thin GEMM  [queries x d] * [d x keys]  followed by a multiply with the stored 1/|key|.
//
// Mapping.  One 16x16x32 bf16 MFMA tile = 16 query rows x 16 keys.  The folded query is carried as
// a bf16 (hi, lo) pair in two adjacent rows (row 2i = hi, row 2i+1 = lo), so one MFMA tile serves 8
// queries at ~16 significant bits and the two halves of a score land in the same lane.  The index is
// stored in tiles of 16 keys already in B-operand order, so a wave reads a tile with d/32 coalesced
// 1 KiB loads and no LDS staging.  Document max = DPP max over the C lanes of a document; top-k =
// per-wave threshold filter + candidate list in LDS, pruned by rank counting on 64-bit
// (score, ~doc) keys, merged per block and then across blocks by a small second kernel.
#include "msa_device.h"
#include "msa_host.h"

namespace msa {

constexpr int kScoreWaves = 4;

struct ScoreArgs {
  const uint16_t* q_route;  // [BM][Hq][D]
  const uint16_t* KR;       // tiled
  const float* inv_norm;    // may be null (dot)
  unsigned long long* ws;   // [Hkv][BM][n_splits][k] candidate keys
  int BM, q0;               // total queries, first query of this pass
  int Hq, Hkv, r;
  int N, C, cos;
  long long tiles;
  int tiles_per_split, n_splits, k;
};

__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ float group_max_rt(float x, int C) {
  if (C >= 2) x = fmaxf(x, dpp_f<kDppXor1>(x));
  if (C >= 4) x = fmaxf(x, dpp_f<kDppXor2>(x));
  if (C >= 8) x = fmaxf(x, dpp_f<kDppHalfMirror>(x));
  if (C >= 16) x = fmaxf(x, dpp_f<kDppMirror>(x));
  return x;
}

// Keep the k largest of the c (<= 128) keys of one candidate list, sorted descending, by rank
// counting (keys are distinct).  Executed by one whole wave.  Returns the new count.
__device__ __forceinline__ int prune_list(volatile unsigned long long* cl, int c, int k, int lane,
                                          volatile float* thr_slot) {
  const unsigned long long ka = (lane < c) ? cl[lane] : 0ull;
  const unsigned long long kb = (lane + 64 < c) ? cl[lane + 64] : 0ull;
  int ra = 0, rb = 0;
  for (int j = 0; j < c; ++j) {
    const unsigned long long x = cl[j];
    ra += (x > ka) ? 1 : 0;
    rb += (x > kb) ? 1 : 0;
  }
  wave_sync();
  if (lane < c && ra < k) cl[ra] = ka;
  if (lane + 64 < c && rb < k) cl[rb] = kb;
  if (c >= k) {
    if (lane < c && ra == k - 1) *thr_slot = key_score(ka);
    if (lane + 64 < c && rb == k - 1) *thr_slot = key_score(kb);
  }
  wave_sync();
  return c < k ? c : k;
}

template <int D, int NQT>
__global__ __launch_bounds__(256) void score_scan_kernel(ScoreArgs a) {
  constexpr int NS = D / 32;              // MFMA k-slices per key
  constexpr int NQ = 8 * NQT;             // queries per pass
  constexpr int CAP = (NQT == 1) ? 128 : 96;
  constexpr int TILE_ELEMS = 16 * D;

  __shared__ float qf[NQ][D];
  __shared__ unsigned long long cand[kScoreWaves][NQ][CAP];
  __shared__ int cnt[kScoreWaves][NQ];
  __shared__ float thr_s[kScoreWaves][NQ];
  __shared__ unsigned long long mbuf[256];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int rr = lane >> 4;  // MFMA k-group / D row-group
  const int n = lane & 15;   // A row / B column / D column
  const int sp = blockIdx.x;
  const int g = blockIdx.y;

  // ---- fold the r heads of this group into one fp32 routing query per token -------------------
  for (int qi = wave; qi < NQ; qi += kScoreWaves) {
    const int qg = a.q0 + qi;
    float f[D / 64];
#pragma unroll
    for (int e = 0; e < D / 64; ++e) f[e] = 0.f;
    if (qg < a.BM) {
      for (int hh = 0; hh < a.r; ++hh) {
        const uint16_t* qp = a.q_route + ((long long)qg * a.Hq + g * a.r + hh) * D;
        float x[D / 64];
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < D / 64; ++e) {
          x[e] = __uint_as_float((uint32_t)qp[lane + 64 * e] << 16);
          ss += x[e] * x[e];
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) ss += __shfl_xor(ss, off, 64);
        const float w = a.cos ? 1.0f / fmaxf(sqrtf(ss), 1e-12f) : 1.0f;
#pragma unroll
        for (int e = 0; e < D / 64; ++e) f[e] += x[e] * w;
      }
    }
#pragma unroll
    for (int e = 0; e < D / 64; ++e) qf[qi][lane + 64 * e] = f[e] / (float)a.r;
  }
  for (int qi = lane; qi < NQ; qi += 64) {
    cnt[wave][qi] = 0;
    thr_s[wave][qi] = (a.q0 + qi < a.BM) ? -INFINITY : INFINITY;
  }
  __syncthreads();

  // ---- A operands: row n of tile t is query 8t + n/2, hi (even n) or lo (odd n) half ----------
  bf16x8_t A[NQT][NS];
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    const int qi = 8 * t + (n >> 1);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      uint32_t w[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        float h0, l0, h1, l1;
        split_bf16(qf[qi][32 * s + 8 * rr + 2 * jj], h0, l0);
        split_bf16(qf[qi][32 * s + 8 * rr + 2 * jj + 1], h1, l1);
        w[jj] = (n & 1) ? pack_bf16(l0, l1) : pack_bf16(h0, h1);
      }
      A[t][s] = as_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
    }
  }
  // per-lane thresholds of the two queries this lane sees per tile: 8t + 2rr and 8t + 2rr + 1
  float thr[NQT][2];
#pragma unroll
  for (int t = 0; t < NQT; ++t) {
    thr[t][0] = thr_s[wave][8 * t + 2 * rr];
    thr[t][1] = thr_s[wave][8 * t + 2 * rr + 1];
  }

  // ---- stream this block's tiles -------------------------------------------------------------
  const long long tb = (long long)sp * a.tiles_per_split;
  long long te = tb + a.tiles_per_split;
  if (te > a.tiles) te = a.tiles;
  const uint16_t* KRg = a.KR + (long long)g * a.tiles * TILE_ELEMS;
  const float* ing = a.inv_norm ? a.inv_norm + (long long)g * a.tiles * 16 : nullptr;
  const int dpt = 16 / a.C;  // documents per tile
  const int ndoc = n / a.C;  // this lane's document inside a tile
  const bool lead_lane = (n & (a.C - 1)) == 0;

  uint4 cur[NS];
  float cinv = 1.0f;
  long long t = tb + wave;
  if (t < te) {
#pragma unroll
    for (int s = 0; s < NS; ++s)
      cur[s] = *reinterpret_cast<const uint4*>(KRg + t * TILE_ELEMS + s * 512 + lane * 8);
    if (ing) cinv = ing[t * 16 + n];
  }
  for (; t < te; t += kScoreWaves) {
    uint4 nxt[NS];
    float ninv = 1.0f;
    const long long tn = t + kScoreWaves;
    if (tn < te) {
#pragma unroll
      for (int s = 0; s < NS; ++s)
        nxt[s] = *reinterpret_cast<const uint4*>(KRg + tn * TILE_ELEMS + s * 512 + lane * 8);
      if (ing) ninv = ing[tn * 16 + n];
    } else {
#pragma unroll
      for (int s = 0; s < NS; ++s) nxt[s] = make_uint4(0, 0, 0, 0);
    }

    const long long doc = t * dpt + ndoc;
    const bool lead = lead_lane && doc < a.N;
    float sc[NQT][2];
    bool hit = false;
#pragma unroll
    for (int tq = 0; tq < NQT; ++tq) {
      f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < NS; ++s) acc = mfma16(A[tq][s], as_bf16x8(cur[s]), acc);
      sc[tq][0] = group_max_rt((acc[0] + acc[1]) * cinv, a.C);
      sc[tq][1] = group_max_rt((acc[2] + acc[3]) * cinv, a.C);
      hit = hit || (lead && (sc[tq][0] >= thr[tq][0] || sc[tq][1] >= thr[tq][1]));
    }
    if (__any(hit)) {
#pragma unroll
      for (int tq = 0; tq < NQT; ++tq) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          if (lead && sc[tq][e] >= thr[tq][e]) {
            const int qi = 8 * tq + 2 * rr + e;
            const int slot = atomicAdd(&cnt[wave][qi], 1);
            cand[wave][qi][slot] = make_key(sc[tq][e], (uint32_t)doc);
          }
        }
      }
      wave_sync();
      for (int qi = 0; qi < NQ; ++qi) {
        const int c = ((volatile int*)cnt[wave])[qi];
        if (c > CAP - 16) {
          const int nc = prune_list(cand[wave][qi], c, a.k, lane, &thr_s[wave][qi]);
          if (lane == 0) cnt[wave][qi] = nc;
        }
      }
      wave_sync();
#pragma unroll
      for (int tq = 0; tq < NQT; ++tq) {
        thr[tq][0] = ((volatile float*)thr_s[wave])[8 * tq + 2 * rr];
        thr[tq][1] = ((volatile float*)thr_s[wave])[8 * tq + 2 * rr + 1];
      }
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) cur[s] = nxt[s];
    cinv = ninv;
  }

  // ---- per-wave lists -> sorted top-k; then merge the four waves per query --------------------
  wave_sync();
  for (int qi = 0; qi < NQ; ++qi) {
    const int c = ((volatile int*)cnt[wave])[qi];
    const int nc = prune_list(cand[wave][qi], c, a.k, lane, &thr_s[wave][qi]);
    if (lane == 0) cnt[wave][qi] = nc;
  }
  __syncthreads();
  for (int qi = 0; qi < NQ; ++qi) {
    const int qg = a.q0 + qi;
    if (qg >= a.BM) break;  // block-uniform
    unsigned long long key = 0ull;
    if (lane < cnt[wave][qi]) key = cand[wave][qi][lane];
    mbuf[tid] = key;
    __syncthreads();
    int rank = 0;
    for (int j = 0; j < 256; ++j) rank += (mbuf[j] > key) ? 1 : 0;
    const int total = __syncthreads_count(key != 0ull);
    unsigned long long* dst = a.ws + (((long long)g * a.BM + qg) * a.n_splits + sp) * a.k;
    if (key != 0ull && rank < a.k) dst[rank] = key;
    if (tid >= total && tid < a.k) dst[tid] = 0ull;
  }
}

// Merge the n_splits sorted lists of one (query, group): bitonic sort of n_splits*k keys in LDS.
__global__ __launch_bounds__(256) void score_merge_kernel(const unsigned long long* __restrict__ ws,
                                                          int32_t* __restrict__ out_idx,
                                                          float* __restrict__ out_score, int BM,
                                                          int Hkv, int n_splits, int k, int n2) {
  extern __shared__ unsigned long long buf[];
  const int tid = threadIdx.x;
  const int qg = blockIdx.x % BM;
  const int g = blockIdx.x / BM;
  const int T = n_splits * k;
  const unsigned long long* src = ws + ((long long)g * BM + qg) * T;
  for (int i = tid; i < n2; i += 256) buf[i] = (i < T) ? src[i] : 0ull;
  for (int size = 2; size <= n2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
      for (int i = tid; i < (n2 >> 1); i += 256) {
        const int pos = 2 * i - (i & (stride - 1));
        const unsigned long long x = buf[pos], y = buf[pos + stride];
        const bool desc = (pos & size) == 0;
        if ((x < y) == desc) {
          buf[pos] = y;
          buf[pos + stride] = x;
        }
      }
    }
  }
  __syncthreads();
  if (tid < k) {
    const unsigned long long key = buf[tid];
    const long long o = ((long long)qg * Hkv + g) * k + tid;
    out_idx[o] = key ? (int32_t)key_doc(key) : -1;
    if (out_score) out_score[o] = key ? key_score(key) : -INFINITY;
  }
}

ScorePlan plan_score(const Dims& dm, int BM, int k) {
  ScorePlan p;
  long long want = 2048 / dm.Hkv;
  if (want < 1) want = 1;
  long long by_tiles = (dm.tiles + 7) / 8;
  long long by_merge = 4096 / k;
  long long ns = want;
  if (ns > by_tiles) ns = by_tiles;
  if (ns > by_merge) ns = by_merge;
  if (ns < 1) ns = 1;
  p.tiles_per_split = (int)((dm.tiles + ns - 1) / ns);
  p.n_splits = (int)((dm.tiles + p.tiles_per_split - 1) / p.tiles_per_split);
  p.q_per_pass = (BM <= 8) ? 8 : 16;
  p.n_pass = (BM + p.q_per_pass - 1) / p.q_per_pass;
  p.ws_bytes = round_up256((size_t)dm.Hkv * BM * p.n_splits * k * sizeof(unsigned long long));
  return p;
}

int launch_score(const Dims& dm, const ScorePlan& pl, const void* q_route, int BM, const void* KR,
                 const float* inv_norm, int k, int32_t* out_idx, float* out_score, void* ws,
                 hipStream_t st) {
  ScoreArgs a;
  a.q_route = (const uint16_t*)q_route;
  a.KR = (const uint16_t*)KR;
  a.inv_norm = dm.cos ? inv_norm : nullptr;
  a.ws = (unsigned long long*)ws;
  a.BM = BM;
  a.Hq = dm.Hq;
  a.Hkv = dm.Hkv;
  a.r = dm.r;
  a.N = dm.N;
  a.C = dm.C;
  a.cos = dm.cos;
  a.tiles = dm.tiles;
  a.tiles_per_split = pl.tiles_per_split;
  a.n_splits = pl.n_splits;
  a.k = k;
  dim3 grid(pl.n_splits, dm.Hkv), block(256);
  for (int pass = 0; pass < pl.n_pass; ++pass) {
    a.q0 = pass * pl.q_per_pass;
    if (dm.d == 128) {
      if (pl.q_per_pass == 8)
        hipLaunchKernelGGL((score_scan_kernel<128, 1>), grid, block, 0, st, a);
      else
        hipLaunchKernelGGL((score_scan_kernel<128, 2>), grid, block, 0, st, a);
    } else {
      if (pl.q_per_pass == 8)
        hipLaunchKernelGGL((score_scan_kernel<64, 1>), grid, block, 0, st, a);
      else
        hipLaunchKernelGGL((score_scan_kernel<64, 2>), grid, block, 0, st, a);
    }
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  }
  int n2 = 2;
  while (n2 < pl.n_splits * k) n2 <<= 1;
  hipLaunchKernelGGL(score_merge_kernel, dim3(BM * dm.Hkv), dim3(256),
                     (size_t)n2 * sizeof(unsigned long long), st, (const unsigned long long*)ws,
                     out_idx, out_score, BM, dm.Hkv, pl.n_splits, k, n2);
  if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  return MSA_OK;
}

}  // namespace msa
