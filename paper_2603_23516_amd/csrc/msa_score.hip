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
// 1 KiB loads and no LDS staging.
//
// Work split.  One wavefront = one stream of tiles of one KV head (wave s of S takes tiles s, s + S, ...),
// with a ring of kPrefetch tiles in flight; a workgroup holds four such streams that never synchronise.  Document max = DPP
// max over the C lanes of a document.  Top-k = threshold filter + per-(wave, query) candidate list in
// LDS: accepted lanes get their slots from a ballot and a population count (no atomics, counters live
// in registers), lists are pruned to the k best by rank counting on 64-bit (score, ~doc) keys, and
// the sorted per-wave lists are combined by a second, small kernel.
#include "msa_device.h"
#include "msa_host.h"

namespace msa {

constexpr int kPrefetch = 4;         // tiles in flight per wave
constexpr int kListBytes = 16384;    // LDS per wave for candidate lists

struct ScoreArgs {
  const uint4* qop;         // [Hkv][n_qtiles][D/32][64] A operands (bf16 hi/lo rows) of 8-query tiles, prepared by
                            // prep_scan_operands_kernel (all-heads scan; per-group scan with the threshold exchange)
  int n_qtiles;
  const uint16_t* q_route;  // [BM][Hq][D] routing queries: a per-group scan without the exchange folds them itself
  const uint16_t* KR;       // tiled
  const float* inv_norm;    // may be null (dot)
  unsigned long long* ws;   // [Hkv][BM][n_splits][k] candidate keys, each list sorted descending
  int BM, q0;               // total queries, first query of this pass
  int Hq, Hkv, r;
  int N, C, cos;
  long long tiles;
  int n_splits, k;
  float* mat;               // MODE 2: document scores [Hkv][BM][N]
  int tiles_per_wave;       // MODE 2: contiguous tiles per wave
  float* gmax;              // [Hkv][BM][n_splits] running per-wave maxima (threshold exchange), or null
  int it_publish, it_adopt; // iterations at which a wave publishes its maxima / adopts the bound
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

// Keep the k largest of the c (<= CAP) distinct keys of one list, sorted descending, by rank
// counting.  Executed by one whole wave.  Returns the new count min(c, k).  UNR candidates are read
// (LDS broadcasts) per round: the final sort of a stream keeps 16 reads in flight (their latency is
// what it waits for: 15.5 -> 9.7 us per wave on the 50M-token bank), the in-stream prunes 4 to keep the
// loop body small.
template <int CAP, int UNR = 4>
__device__ __forceinline__ int prune_list(unsigned long long* cl, int c, int k, int lane) {
  constexpr int PER = CAP / 64;
  unsigned long long key[PER];
  int rank[PER];
#pragma unroll
  for (int p = 0; p < PER; ++p) {
    key[p] = (lane + 64 * p < c) ? cl[lane + 64 * p] : 0ull;
    rank[p] = 0;
  }
  int j = 0;
  for (; j + UNR <= c; j += UNR) {
    unsigned long long x[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) x[u] = cl[j + u];
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      if (64 * p < c) {
#pragma unroll
        for (int u = 0; u < UNR; ++u) rank[p] += (x[u] > key[p]) ? 1 : 0;
      }
    }
  }
  for (; j < c; ++j) {
    const unsigned long long x = cl[j];
#pragma unroll
    for (int p = 0; p < PER; ++p) rank[p] += (x > key[p]) ? 1 : 0;
  }
  wave_sync();
#pragma unroll
  for (int p = 0; p < PER; ++p)
    if (lane + 64 * p < c && rank[p] < k) cl[rank[p]] = key[p];
  wave_sync();
  return c < k ? c : k;
}

// Sum over aligned groups of W consecutive lanes (W a power of two <= 64); every lane gets the sum.
template <int W>
__device__ __forceinline__ float group_sum(float x) {
  if (W >= 2) x += dpp_f<kDppXor1>(x);
  if (W >= 4) x += dpp_f<kDppXor2>(x);
  if (W >= 8) x += dpp_f<kDppHalfMirror>(x);
  if (W >= 16) x += dpp_f<kDppMirror>(x);
  if (W >= 32) x += __shfl_xor(x, 16, 64);
  if (W >= 64) x += __shfl_xor(x, 32, 64);
  return x;
}

// Independent streams (waves) per workgroup: measured 3-5 % faster than single-wave workgroups.
constexpr int kScanWaves = 4;

// One wave folds the r heads of KV group g of the 8 queries of tile qt into one fp32 routing query per token,
//     qf = (1/r) sum_h q_h / max(|q_h|, 1e-12)        (plain mean for the dot product),
// splits it into bf16 hi + lo and leaves the MFMA A operands of the tile in aop[s][lane]: lane 16q + n holds row n
// (query n/2, hi for even n, lo for odd n), dims 32s + 8q .. +8 of slice s.  qf: 8 * D floats of the wave's own LDS.
// Two steps, so that a caller can put other loads between the request for the queries and their use:
// fold_query_load asks for the queries, fold_query_tile folds them.
// Lane = (query lane / LPH, 16-byte piece lane % LPH): a lane loads the same piece of all r heads of
// its query, so the head sum stays in the lane and the norms need only DPP sums over LPH <= 16 lanes.
template <int D>
struct FoldRegs {
  static constexpr int LPH = D / 8, HPL = 64 / LPH, PASSES = 8 / HPL;
  uint4 v[PASSES][8];
};

template <int D>
__device__ __forceinline__ void fold_query_load(const uint16_t* __restrict__ q_route, long long qt, int g, int BM,
                                                int Hq, int r, FoldRegs<D>& fr, int lane) {
  constexpr int LPH = FoldRegs<D>::LPH, HPL = FoldRegs<D>::HPL;
  const int piece = lane % LPH;
  // No branch around a load (rows past the end re-read the last query, heads past r the last head; the fold
  // ignores both): the loads then sit in straight-line code and the wait before the fold can leave the loads
  // that were issued after them in flight.
#pragma unroll
  for (int pass = 0; pass < FoldRegs<D>::PASSES; ++pass) {
    long long qg = qt * 8 + pass * HPL + lane / LPH;
    if (qg > BM - 1) qg = BM - 1;
#pragma unroll
    for (int hh = 0; hh < 8; ++hh) {
      const int hc = hh < r ? hh : r - 1;
      fr.v[pass][hh] = *reinterpret_cast<const uint4*>(q_route + (qg * Hq + g * r + hc) * D + piece * 8);
    }
  }
}

template <int D>
__device__ __forceinline__ void fold_query_tile(const FoldRegs<D>& fr, long long qt, int BM, int r, int cos, float* qf,
                                                uint4 (*aop)[64], int lane) {
  constexpr int NS = D / 32, LPH = FoldRegs<D>::LPH, HPL = FoldRegs<D>::HPL;
  const int piece = lane % LPH;
#pragma unroll
  for (int pass = 0; pass < FoldRegs<D>::PASSES; ++pass) {
    const int qi = pass * HPL + lane / LPH;
    float f[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = 0.f;
#pragma unroll
    for (int hh = 0; hh < 8; ++hh) {
      if (hh < r) {  // wave-uniform
        const uint4 v = fr.v[pass][hh];
        const float x[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                            bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += x[e] * x[e];
        ss = group_sum<LPH>(ss);
        const float w = cos ? 1.0f / fmaxf(sqrtf(ss), 1e-12f) : 1.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] += x[e] * w;
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[qi * D + piece * 8 + e] = (qt * 8 + qi < BM) ? f[e] / (float)r : 0.f;
  }
  wave_sync();
  const int rr = lane >> 4, n = lane & 15;
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    uint32_t w[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      float h0, l0, h1, l1;
      split_bf16(qf[(n >> 1) * D + 32 * s + 8 * rr + 2 * jj], h0, l0);
      split_bf16(qf[(n >> 1) * D + 32 * s + 8 * rr + 2 * jj + 1], h1, l1);
      w[jj] = (n & 1) ? pack_bf16(l0, l1) : pack_bf16(h0, h1);
    }
    aop[s][lane] = make_uint4(w[0], w[1], w[2], w[3]);
  }
  wave_sync();
}

// MODE 0  filter: thresholds, candidate lists, pruning (long streams).
// MODE 1  dense lists: a wave's whole stream holds no more documents than a list has slots, so every
//         document score goes straight to slot (iteration, document-in-tile) of its query's list and
//         the lists are sorted once at the end; no thresholds, ballots or counters in the stream.
// MODE 2  score matrix: like MODE 1 but the wave owns a CONTIGUOUS range of tiles and, instead of
//         sorting, writes the fp32 document scores of every query as one coalesced run of the row
//         mat[g][query][:]; topk_rows_kernel then selects per row.  For short streams (small banks,
//         many queries) the per-wave sorts and the list merge cost more than the stream itself.
// FOLD: the workgroup folds its queries into MFMA operands itself (wave t folds tile t, one workgroup barrier) instead
//       of reading operands that prep_scan_operands_kernel prepared: one launch less, which is what short streams
//       are made of.  Scans with the threshold exchange keep the prepared operands: that launch also resets the
//       exchange buffer, and their waves never synchronise.
template <int D, int NQT, bool COS, int MODE, bool FOLD>
__global__ __launch_bounds__(64 * kScanWaves) __attribute__((amdgpu_waves_per_eu(2)))
void score_scan_kernel(ScoreArgs a) {
  constexpr bool DENSE = MODE != 0;
  constexpr int NS = D / 32;   // MFMA k-slices per key
  constexpr int NQ = 8 * NQT;  // queries per pass
  constexpr int CAP = kListBytes / (8 * NQ);
  constexpr int CAPF = kListBytes / (4 * NQ);  // MODE 2: fp32 scores per query
  constexpr int TILE_ELEMS = 16 * D;

  __shared__ __attribute__((aligned(16))) unsigned char smem[kScanWaves][kListBytes];
  __shared__ int cnt_all[kScanWaves][NQ];
  __shared__ float thr_all[kScanWaves][NQ];
  const int wave = threadIdx.x >> 6;
  unsigned long long* cand = reinterpret_cast<unsigned long long*>(smem[wave]);  // [NQ][CAP]
  float* candf = reinterpret_cast<float*>(smem[wave]);                            // MODE 2: [NQ][CAPF]
  int* cnt_s = cnt_all[wave];
  float* thr_s = thr_all[wave];

  const int lane = threadIdx.x & 63;
  const int rr = lane >> 4;  // MFMA k-group / D row-group
  const int n = lane & 15;   // A row / B column / D column
  const int sp = blockIdx.x * kScanWaves + wave;
  const int g = blockIdx.y;
  // wave-uniform; with FOLD a wave without a stream (the tail of the last workgroup) still takes part in the
  // workgroup barriers of the prologue, otherwise the waves of a workgroup never synchronise
  const bool active = sp < a.n_splits;
  if (!FOLD && !active) return;

  // ---- the queries this wave folds are requested first: a wave's loads return in order, and behind the first tiles
  // of every wave of the grid (tens of MB at once) they would arrive only when that burst has been served ----
  FoldRegs<D> fr;
  bf16x8_t A[NQT][NS];
  if constexpr (FOLD) {
    if (wave < NQT) fold_query_load<D>(a.q_route, a.q0 / 8 + wave, g, a.BM, a.Hq, a.r, fr, lane);
  } else {
    // prepared operands: row n of query tile t is query 8t + n/2, hi (even n) or lo (odd n) half of the folded
    // fp32 routing query
#pragma unroll
    for (int t = 0; t < NQT; ++t) {
      const long long qt = a.q0 / 8 + t;
#pragma unroll
      for (int s = 0; s < NS; ++s)
        A[t][s] = as_bf16x8(a.qop[(((long long)g * a.n_qtiles + qt) * NS + s) * 64 + lane]);
    }
  }

  // ---- start streaming at once: the first kPrefetch tiles are requested before the prologue ----
  // Wave sp takes tiles sp, sp + n_splits, sp + 2 n_splits, ...: at any moment the waves of a head
  // read one contiguous window of the index.  Loads past the end re-read the last tile: they are
  // always issued, so the number of loads in flight is the same on every path.
  const long long S = a.n_splits;
  const long long t0 = (long long)sp * a.tiles_per_wave;  // MODE 2: first tile of this wave
  const long long n_it = !active ? 0
                         : (MODE == 2) ? ((a.tiles - t0 < a.tiles_per_wave) ? a.tiles - t0 : a.tiles_per_wave)
                                       : (a.tiles - sp + S - 1) / S;  // >= 1 by construction of n_splits
  const long long i_last = n_it - 1;
  // MODE 2: the wave walks its range starting rot tiles in and wraps around, so that waves that run in step do
  // not all ask for the same 4 KB position of their 16-tile ranges (the same memory channels) at the same moment
  const long long rot = (MODE == 2 && n_it > 0) ? sp % n_it : 0;
  auto tile_at = [&](long long it) {
    if (MODE != 2) return sp + it * S;
    const long long x = it + rot;
    return t0 + (x >= n_it ? x - n_it : x);
  };
  const uint16_t* KRg = a.KR + (long long)g * a.tiles * TILE_ELEMS + lane * 8;
  const float* ing = COS ? a.inv_norm + (long long)g * a.tiles * 16 + n : nullptr;
  // Long streams (MODE 0) read an index far larger than the caches exactly once: streaming loads.  The short
  // streams of MODE 1 and 2 (an index of at most a few hundred MB) measured faster with plain loads.
  auto load_tile16 = [](const uint16_t* p) {
    return MODE == 0 ? load_stream16(p) : *reinterpret_cast<const uint4*>(p);
  };
  uint4 buf[kPrefetch][NS];
  float binv[kPrefetch];
  {  // a wave without a stream loads tile 0 and drops it: no branch around the loads
#pragma unroll
    for (int u = 0; u < kPrefetch; ++u) {
      const long long t = active ? tile_at((u < n_it) ? u : i_last) : 0;
#pragma unroll
      for (int s = 0; s < NS; ++s)
        buf[u][s] = load_tile16(KRg + t * TILE_ELEMS + s * 512);
      binv[u] = COS ? ing[t * 16] : 1.0f;
    }
  }

  // ---- A operands: row n of query tile t is query 8t + n/2, hi (even n) or lo (odd n) half of the folded fp32
  // routing query ------------------------------------------------------------------------------------------
  if constexpr (FOLD) {
    // wave t folds tile t; the operands pass through the candidate areas, which are free until the stream starts:
    // tile t in the second half of area t, the folding wave's scratch in the first half of its own
    static_assert(NQT <= kScanWaves && 8 * D * 4 <= kListBytes / 2 && NS * 64 * 16 <= kListBytes / 2, "prologue scratch");
    typedef uint4 aop_tile_t[64];
    if (wave < NQT)
      fold_query_tile<D>(fr, a.q0 / 8 + wave, a.BM, a.r, COS ? 1 : 0, reinterpret_cast<float*>(smem[wave]),
                         reinterpret_cast<aop_tile_t*>(smem[wave] + kListBytes / 2), lane);
    lds_barrier();
#pragma unroll
    for (int t = 0; t < NQT; ++t)
#pragma unroll
      for (int s = 0; s < NS; ++s)
        A[t][s] = as_bf16x8(reinterpret_cast<const aop_tile_t*>(smem[t] + kListBytes / 2)[s][lane]);
    lds_barrier();  // every wave has its operands: the candidate areas are the streams' from here on
    if (!active) return;
  } else {
    // The operands were requested ahead of the tiles; they are awaited HERE, ahead of the loop.  A wait that is
    // first needed inside the loop sits in the loop's first block and is paid on every round: there it has to
    // cover the entry from here too, where the operands are the youngest loads, so it would wait for everything,
    // i.e. drain the prefetch at the head of every round.
#pragma unroll
    for (int t = 0; t < NQT; ++t)
#pragma unroll
      for (int s = 0; s < NS; ++s) asm volatile("" : "+v"(A[t][s]));
  }

  // This lane sees queries 8t + 2rr + e (e = 0, 1) of every tile; all 16 lanes of a row keep
  // identical copies of their counters and thresholds.
  float thr[NQT][2];
  int cnt[NQT][2];
#pragma unroll
  for (int t = 0; t < NQT; ++t)
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      thr[t][e] = (a.q0 + 8 * t + 2 * rr + e < a.BM) ? -INFINITY : INFINITY;
      cnt[t][e] = 0;
    }
  int limit = 2 * a.k < 32 ? 32 : 2 * a.k;  // prune a list when it grows past this
  if (limit > CAP - 16) limit = CAP - 16;

  // ---- stream this wave's tiles -----------------------------------------------------------------
  const int dpt = 16 / a.C;  // documents per tile
  const int ndoc = n / a.C;  // this lane's document inside a tile
  const bool lead_lane = (n & (a.C - 1)) == 0;
  const uint32_t below = (1u << n) - 1u;
  float qmax[NQT][2];        // running maximum of this lane's document scores, per query
#pragma unroll
  for (int t = 0; t < NQT; ++t) qmax[t][0] = qmax[t][1] = -INFINITY;
  // One 8-query tile per pass: the published maxima are requested kPrefetch iterations before they
  // are used, all queries at once, so their latency hides behind that many tiles of the stream.
  constexpr bool kEarlyFetch = (NQT == 1);
  constexpr int kFetchLead = 1;  // in groups of kPrefetch iterations
  float exq[kEarlyFetch ? NQ : 1][4];
  {
    for (long long base = 0; base < n_it; base += kPrefetch) {
      // ---- threshold exchange (long streams only): every wave publishes the best score it has
      // seen per query; a little later it adopts theta = the k-th largest of all published maxima.
      // The maxima belong to distinct documents, so at least k documents score >= theta: a valid
      // lower bound on the k-th best score whatever the other waves have written so far.  The maxima
      // are published with device-scope stores and read with device-scope loads: the waves of a head sit on all
      // eight XCDs, each with its own L2, and a plainly stored maximum becomes visible elsewhere only when its
      // line happens to be evicted.  With plain index loads flooding the L2 that happened soon enough; the
      // streaming loads used here leave the L2 alone, and the bound then came from one XCD's maxima only (the
      // k-th largest of 32 instead of 256: scan 272 -> 283 us on the 50M-token index, 256 with these accesses).
      if (!DENSE && kEarlyFetch && a.gmax != nullptr && base == a.it_adopt - kFetchLead * kPrefetch) {
#pragma unroll
        for (int qi = 0; qi < (kEarlyFetch ? NQ : 1); ++qi) {
          const int qg = a.q0 + qi < a.BM ? a.q0 + qi : a.BM - 1;
          const float* src = a.gmax + ((long long)g * a.BM + qg) * a.n_splits;
#pragma unroll
          for (int j = 0; j < 4; ++j)
            exq[qi][j] = (lane + 64 * j < a.n_splits) ? load_dev(src + lane + 64 * j) : -INFINITY;
        }
      }
      if (!DENSE && a.gmax != nullptr && (base == a.it_publish || base == a.it_adopt)) {
        if (base == a.it_publish) {
#pragma unroll
          for (int tq = 0; tq < NQT; ++tq)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              const float mrow = group_max<16>(qmax[tq][e]);
              const int qg = a.q0 + 8 * tq + 2 * rr + e;
              if (n == 0 && qg < a.BM) store_dev(&a.gmax[((long long)g * a.BM + qg) * a.n_splits + sp], mrow);
            }
        } else {
          // theta = k-th largest of the published maxima of one query: bitwise search on the
          // order-preserving integer image, 4 values per lane
          auto kth_largest = [&](const uint32_t (&ord)[4]) -> float {
            uint32_t prefix = 0u;
            for (int bit = 31; bit >= 12; --bit) {
              const uint32_t cnd = prefix | (1u << bit);
              int ge = 0;
#pragma unroll
              for (int j = 0; j < 4; ++j) ge += __popcll(__ballot(ord[j] >= cnd));
              if (ge >= a.k) prefix = cnd;  // wave-uniform
            }
            return prefix ? unorderable(prefix) : -INFINITY;
          };
          if constexpr (kEarlyFetch) {
#pragma unroll
            for (int qi = 0; qi < NQ; ++qi) {
              uint32_t ord[4];
#pragma unroll
              for (int j = 0; j < 4; ++j) ord[j] = orderable(exq[qi][j]);
              const float th = kth_largest(ord);
              if (lane == 0) thr_s[qi] = th;
            }
          } else {
            for (int qi = 0; qi < NQ; ++qi) {
              const int qg = a.q0 + qi;
              if (qg >= a.BM) break;  // wave-uniform
              const float* src = a.gmax + ((long long)g * a.BM + qg) * a.n_splits;
              uint32_t ord[4];
#pragma unroll
              for (int j = 0; j < 4; ++j)
                ord[j] = (lane + 64 * j < a.n_splits) ? orderable(load_dev(src + lane + 64 * j)) : 0u;
              const float th = kth_largest(ord);
              if (lane == 0) thr_s[qi] = th;
            }
          }
          wave_sync();
#pragma unroll
          for (int tq = 0; tq < NQT; ++tq)
#pragma unroll
            for (int e = 0; e < 2; ++e)
              if (a.q0 + 8 * tq + 2 * rr + e < a.BM)
                thr[tq][e] = fmaxf(thr[tq][e], thr_s[8 * tq + 2 * rr + e]);
          wave_sync();
          // Candidates accepted before the bound was known and now below it can never be among the k best: drop
          // them at once.  What is left is a handful of entries per list, so the final sort of the stream (which
          // every wave runs while the memory system idles) has next to nothing to do.
          if (n == 0) {
#pragma unroll
            for (int tq = 0; tq < NQT; ++tq)
#pragma unroll
              for (int e = 0; e < 2; ++e) {
                cnt_s[8 * tq + 2 * rr + e] = cnt[tq][e];
                thr_s[8 * tq + 2 * rr + e] = thr[tq][e];
              }
          }
          wave_sync();
          for (int qi = 0; qi < NQ; ++qi) {
            constexpr int PER = (CAP + 63) / 64;
            const int c = cnt_s[qi];
            const float th = thr_s[qi];
            unsigned long long* cl = cand + qi * CAP;
            unsigned long long x[PER];
            bool kp[PER];
#pragma unroll
            for (int p = 0; p < PER; ++p) {
              const int j = lane + 64 * p;
              x[p] = (j < c) ? cl[j] : 0ull;
              kp[p] = j < c && key_score(x[p]) >= th;
            }
            wave_sync();  // every entry is in a register before the list is rewritten
            int kept = 0;
#pragma unroll
            for (int p = 0; p < PER; ++p) {
              const unsigned long long m = __ballot(kp[p]);
              if (kp[p]) cl[kept + __popcll(m & ((1ull << lane) - 1ull))] = x[p];
              kept += __popcll(m);
            }
            if (lane == 0) cnt_s[qi] = kept;
          }
          wave_sync();
#pragma unroll
          for (int tq = 0; tq < NQT; ++tq) {
            cnt[tq][0] = cnt_s[8 * tq + 2 * rr];
            cnt[tq][1] = cnt_s[8 * tq + 2 * rr + 1];
          }
          wave_sync();
        }
      }
#pragma unroll
      for (int u = 0; u < kPrefetch; ++u) {
        const long long it = base + u;
        const long long t = tile_at(it);
        // The products read the tile (and the scores its reciprocal norms) where they landed, and only then is
        // the next tile of this slot requested into the same registers.  (Requested earlier, while this tile is
        // still needed, the new tile would have to land in other registers; the slots would wander from one round
        // of the loop to the next and be copied back at its end, and a copy of a register with a load in flight
        // waits for that load, i.e. drains the prefetch.)
        float sraw[NQT][2];
#pragma unroll
        for (int tq = 0; tq < NQT; ++tq) {
          f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int s = 0; s < NS; ++s) acc = mfma16(A[tq][s], as_bf16x8(buf[u][s]), acc);
          sraw[tq][0] = (acc[0] + acc[1]) * binv[u];
          sraw[tq][1] = (acc[2] + acc[3]) * binv[u];
          // pinned here: left alone, the compiler sinks one of the two products below the requests (and hoists the
          // requests above them), which keeps the old reciprocal norm alive and sends the new one elsewhere
          asm volatile("" : "+v"(sraw[tq][0]), "+v"(sraw[tq][1])::"memory");
        }
        {
          const long long tn = tile_at((it + kPrefetch < n_it) ? it + kPrefetch : i_last);
#pragma unroll
          for (int s = 0; s < NS; ++s)
            buf[u][s] = load_tile16(KRg + tn * TILE_ELEMS + s * 512);
          binv[u] = COS ? ing[tn * 16] : 1.0f;
        }

        const long long doc = t * dpt + ndoc;
        const bool lead = lead_lane && it < n_it && doc < a.N;
        bool over = false;
        // scores first; the slot arithmetic runs only for tiles in which some lane passes its threshold
        float scv[NQT][2];
        bool any_pred = false;
#pragma unroll
        for (int tq = 0; tq < NQT; ++tq) {
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const float sc = group_max_rt(sraw[tq][e], a.C);
            if (MODE == 2) {
              if (lead) candf[(8 * tq + 2 * rr + e) * CAPF + (int)(t - t0) * dpt + ndoc] = sc;
            } else if (MODE == 1) {
              if (lead) cand[(8 * tq + 2 * rr + e) * CAP + (int)it * dpt + ndoc] = make_key(sc, (uint32_t)doc);
            } else {
              scv[tq][e] = sc;
              if (lead) qmax[tq][e] = fmaxf(qmax[tq][e], sc);
              any_pred = any_pred || (lead && sc >= thr[tq][e]);
            }
          }
        }
        if (!DENSE && __any(any_pred)) {
#pragma unroll
          for (int tq = 0; tq < NQT; ++tq) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              const float sc = scv[tq][e];
              const bool pred = lead && sc >= thr[tq][e];
              const unsigned long long m = __ballot(pred);
              const uint32_t half = (rr & 2) ? (uint32_t)(m >> 32) : (uint32_t)m;
              const uint32_t row = (half >> ((rr & 1) * 16)) & 0xffffu;
              if (pred) {
                const int qi = 8 * tq + 2 * rr + e;
                cand[qi * CAP + cnt[tq][e] + __popc(row & below)] = make_key(sc, (uint32_t)doc);
              }
              cnt[tq][e] += __popc(row);
              over = over || cnt[tq][e] > limit;
            }
          }
        }
        if (__any(over)) {
          // rare path: publish the counters, prune the lists that are too long, reload
          if (n == 0) {
#pragma unroll
            for (int tq = 0; tq < NQT; ++tq) {
              cnt_s[8 * tq + 2 * rr] = cnt[tq][0];
              cnt_s[8 * tq + 2 * rr + 1] = cnt[tq][1];
              thr_s[8 * tq + 2 * rr] = thr[tq][0];
              thr_s[8 * tq + 2 * rr + 1] = thr[tq][1];
            }
          }
          wave_sync();
          for (int qi = 0; qi < NQ; ++qi) {
            const int c = cnt_s[qi];
            if (c > limit) {  // wave-uniform
              unsigned long long* cl = cand + qi * CAP;
              const int nc = prune_list<CAP>(cl, c, a.k, lane);
              if (lane == 0) {
                cnt_s[qi] = nc;
                thr_s[qi] = key_score(cl[a.k - 1]);
              }
            }
          }
          wave_sync();
#pragma unroll
          for (int tq = 0; tq < NQT; ++tq) {
            cnt[tq][0] = cnt_s[8 * tq + 2 * rr];
            cnt[tq][1] = cnt_s[8 * tq + 2 * rr + 1];
            thr[tq][0] = thr_s[8 * tq + 2 * rr];
            thr[tq][1] = thr_s[8 * tq + 2 * rr + 1];
          }
          wave_sync();
        }
      }
    }
  }

  // ---- sort every list and hand the k best to the merge kernel --------------------------------
  if (n == 0) {
#pragma unroll
    for (int tq = 0; tq < NQT; ++tq) {
      cnt_s[8 * tq + 2 * rr] = cnt[tq][0];
      cnt_s[8 * tq + 2 * rr + 1] = cnt[tq][1];
    }
  }
  wave_sync();
  // MODE 1, 2: every list holds the same documents, those of the wave's tiles in order; only the
  // last tile of the index can end early
  int c_dense = 0;
  if (DENSE) {
    const long long left = (long long)a.N - ((MODE == 2) ? t0 + i_last : tile_at(i_last)) * dpt;
    c_dense = (int)i_last * dpt + (int)(left < dpt ? (left < 0 ? 0 : left) : dpt);
  }
  if (MODE == 2) {
    const long long doc0 = t0 * dpt;  // the wave's documents are doc0 .. doc0 + c_dense - 1
    int pw = 1;
    while (pw < c_dense) pw <<= 1;  // wave-uniform
    if (pw <= 64) {
      // 64 / pw queries per wave-wide access (lane = query-in-group * pw + document), eight accesses read from
      // LDS before the first is stored: the runs of one query are short, a loop over single queries would spend
      // its time on one dependent LDS read after the other
      const int qpi = 64 / pw;
      const int j = lane & (pw - 1), qo = lane / pw;
      for (int i0 = 0; i0 < NQ; i0 += 8 * qpi) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int qi = i0 + u * qpi + qo;
          v[u] = (qi < NQ && j < c_dense) ? candf[qi * CAPF + j] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int qi = i0 + u * qpi + qo;
          if (qi < NQ && a.q0 + qi < a.BM && j < c_dense)
            a.mat[((long long)g * a.BM + a.q0 + qi) * a.N + doc0 + j] = v[u];
        }
      }
      return;
    }
    for (int qi = 0; qi < NQ; ++qi) {
      const int qg = a.q0 + qi;
      if (qg >= a.BM) break;  // wave-uniform
      float* row = a.mat + ((long long)g * a.BM + qg) * a.N + doc0;
      for (int j = lane; j < c_dense; j += 64) row[j] = candf[qi * CAPF + j];
    }
    return;
  }
  for (int qi = 0; qi < NQ; ++qi) {
    const int qg = a.q0 + qi;
    if (qg >= a.BM) break;  // wave-uniform
    const int c = DENSE ? c_dense : cnt_s[qi];
    unsigned long long* cl = cand + qi * CAP;
    const int nc = prune_list<CAP, 16>(cl, c, a.k, lane);
    unsigned long long* dst = a.ws + (((long long)g * a.BM + qg) * a.n_splits + sp) * a.k;
    if (lane < a.k) dst[lane] = (lane < nc) ? cl[lane] : 0ull;
  }
}

// Literal Eq. 2 head mean (select_scope = ALL): the chunk score is the mean over EVERY query head of
// the similarity with the routing key of that head's KV group, i.e. the mean over the Hkv groups of
// the per-group scores above, so one selection serves all heads.  A wave's stream interleaves the
// heads: entry e = (tile e / HKV, head e % HKV) through the same ring of kPrefetch loads; the
// per-head partial scores are scaled by that head's 1/|key| and summed, and after the last head the
// document max / threshold / candidate-list logic runs exactly as in score_scan_kernel.  The
// A operands of all HKV heads (8 queries per pass) are too many for registers at two waves per SIMD,
// so a workgroup of four waves (four independent streams) shares one LDS copy of them and every
// wave re-reads the slices of the head at hand.  HKV in {2, 4, 8} (one group: the plain kernel
// already computes this).
constexpr int kAllWaves = 4;

// STREAM: the index is far larger than the caches and read once per pass -> streaming loads (load_stream16); a small
// index that several passes re-read is served partly from the caches and measured faster with plain loads.
template <int D, int HKV, bool COS, bool STREAM>
__global__ __launch_bounds__(64 * kAllWaves) void score_scan_all_kernel(ScoreArgs a) {
  constexpr int NS = D / 32;
  constexpr int NQ = 8;
  constexpr int CAP = 128;  // entries per (wave, query) list: 8 KiB of LDS per wave
  constexpr int TILE_ELEMS = 16 * D;
  constexpr int UT = HKV >= kPrefetch ? 1 : kPrefetch / HKV;  // tiles per unrolled group of entries
  static_assert((UT * HKV) % kPrefetch == 0, "ring slots must be compile-time");

  __shared__ uint4 Aop[HKV][NS][64];
  __shared__ unsigned long long cand_all[kAllWaves][NQ * CAP];
  __shared__ int cnt_all[kAllWaves][NQ];
  __shared__ float thr_all[kAllWaves][NQ];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  unsigned long long* cand = cand_all[wave];
  int* cnt_s = cnt_all[wave];
  float* thr_s = thr_all[wave];
  for (int e = threadIdx.x; e < HKV * NS * 64; e += 64 * kAllWaves) {
    const int h = e / (NS * 64), rest = e % (NS * 64);
    Aop[h][rest / 64][rest % 64] = a.qop[((long long)h * a.n_qtiles + a.q0 / 8) * NS * 64 + rest];
  }
  __syncthreads();
  const int rr = lane >> 4;
  const int n = lane & 15;
  const int sp = blockIdx.x * kAllWaves + wave;
  if (sp >= a.n_splits) return;  // wave-uniform; no block-wide barrier follows
  const long long S = a.n_splits;
  const long long n_it = (a.tiles - sp + S - 1) / S;  // >= 1 because n_splits <= tiles
  const long long i_last = n_it - 1;
  const uint16_t* KRl = a.KR + lane * 8;
  const float* inl = COS ? a.inv_norm + n : nullptr;
  auto tile_of = [&](long long it) { return sp + (it < n_it ? it : i_last) * S; };

  auto load_tile16 = [](const uint16_t* p) {
    return STREAM ? load_stream16(p) : *reinterpret_cast<const uint4*>(p);
  };
  uint4 buf[kPrefetch][NS];
  float binv[kPrefetch];
#pragma unroll
  for (int u = 0; u < kPrefetch; ++u) {
    const int h = u % HKV;
    const long long t = tile_of(u / HKV);
#pragma unroll
    for (int s = 0; s < NS; ++s)
      buf[u][s] = load_tile16(KRl + ((long long)h * a.tiles + t) * TILE_ELEMS + s * 512);
    binv[u] = COS ? inl[((long long)h * a.tiles + t) * 16] : 1.0f;
  }

  float thr[2];
  int cnt[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    thr[e] = (a.q0 + 2 * rr + e < a.BM) ? -INFINITY : INFINITY;
    cnt[e] = 0;
  }
  int limit = 2 * a.k < 32 ? 32 : 2 * a.k;
  if (limit > CAP - 16) limit = CAP - 16;
  const int dpt = 16 / a.C;
  const int ndoc = n / a.C;
  const bool lead_lane = (n & (a.C - 1)) == 0;
  const uint32_t below = (1u << n) - 1u;
  const float inv_heads = 1.0f / (float)HKV;

  for (long long base = 0; base < n_it; base += UT) {
#pragma unroll
    for (int ut = 0; ut < UT; ++ut) {
      const long long it = base + ut;
      const long long t = sp + it * S;
      float tot[2] = {0.f, 0.f};
#pragma unroll
      for (int h = 0; h < HKV; ++h) {
        const int slot = (ut * HKV + h) % kPrefetch;
        uint4 cur[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) cur[s] = buf[slot][s];
        const float cinv = binv[slot];
        {  // the entry kPrefetch ahead of this one takes over the slot (always issued)
          const int en = ut * HKV + h + kPrefetch;
          const int hn = en % HKV;
          const long long tn = tile_of(base + en / HKV);
#pragma unroll
          for (int s = 0; s < NS; ++s)
            buf[slot][s] = load_tile16(KRl + ((long long)hn * a.tiles + tn) * TILE_ELEMS + s * 512);
          binv[slot] = COS ? inl[((long long)hn * a.tiles + tn) * 16] : 1.0f;
        }
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NS; ++s) acc = mfma16(as_bf16x8(Aop[h][s][lane]), as_bf16x8(cur[s]), acc);
        tot[0] += (acc[0] + acc[1]) * cinv;
        tot[1] += (acc[2] + acc[3]) * cinv;
      }
      const long long doc = t * dpt + ndoc;
      const bool lead = lead_lane && it < n_it && doc < a.N;
      bool over = false;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const float sc = group_max_rt(tot[e] * inv_heads, a.C);
        const bool pred = lead && sc >= thr[e];
        const unsigned long long m = __ballot(pred);
        const uint32_t half = (rr & 2) ? (uint32_t)(m >> 32) : (uint32_t)m;
        const uint32_t row = (half >> ((rr & 1) * 16)) & 0xffffu;
        if (pred) cand[(2 * rr + e) * CAP + cnt[e] + __popc(row & below)] = make_key(sc, (uint32_t)doc);
        cnt[e] += __popc(row);
        over = over || cnt[e] > limit;
      }
      if (__any(over)) {
        if (n == 0) {
          cnt_s[2 * rr] = cnt[0];
          cnt_s[2 * rr + 1] = cnt[1];
          thr_s[2 * rr] = thr[0];
          thr_s[2 * rr + 1] = thr[1];
        }
        wave_sync();
        for (int qi = 0; qi < NQ; ++qi) {
          const int c = cnt_s[qi];
          if (c > limit) {  // wave-uniform
            unsigned long long* cl = cand + qi * CAP;
            const int nc = prune_list<CAP>(cl, c, a.k, lane);
            if (lane == 0) {
              cnt_s[qi] = nc;
              thr_s[qi] = key_score(cl[a.k - 1]);
            }
          }
        }
        wave_sync();
        cnt[0] = cnt_s[2 * rr];
        cnt[1] = cnt_s[2 * rr + 1];
        thr[0] = thr_s[2 * rr];
        thr[1] = thr_s[2 * rr + 1];
        wave_sync();
      }
    }
  }

  if (n == 0) {
    cnt_s[2 * rr] = cnt[0];
    cnt_s[2 * rr + 1] = cnt[1];
  }
  wave_sync();
  for (int qi = 0; qi < NQ; ++qi) {
    const int qg = a.q0 + qi;
    if (qg >= a.BM) break;  // wave-uniform
    const int c = cnt_s[qi];
    unsigned long long* cl = cand + qi * CAP;
    const int nc = prune_list<CAP, 16>(cl, c, a.k, lane);
    unsigned long long* dst = a.ws + ((long long)qg * a.n_splits + sp) * a.k;
    if (lane < a.k) dst[lane] = (lane < nc) ? cl[lane] : 0ull;
  }
}

// Literal Eq. 2 token pooling (token_pool = 1): the document score of a question is the max over its
// M query tokens.  The k best documents under that score are all contained in the union of the
// per-token top-k lists: if document D is among them and token m* attains its maximum, every document
// ahead of D in token m*'s ranking is also ahead of D in the pooled ranking, so fewer than k are, and
// D is in m*'s list with exactly its pooled score.  Ranking the union by (best listed score desc,
// index asc) therefore reproduces the pooled top-k exactly.  One block per (batch row, scope slot):
// k rounds of a block-wide arg-max over the M*k listed keys, skipping documents already taken.
constexpr int kPoolSurv = 4096;  // survivors kept in LDS

__global__ __launch_bounds__(256) void pool_tokens_kernel(const unsigned long long* __restrict__ tok_keys,
                                                          int32_t* __restrict__ out_idx,
                                                          float* __restrict__ out_score, int M, int S,
                                                          int k) {
  __shared__ unsigned long long surv[kPoolSurv];
  __shared__ unsigned long long red[4];
  __shared__ uint32_t taken[MSA_MAX_TOPK];
  __shared__ uint32_t floor_s;
  __shared__ int n_surv;
  const int tid = threadIdx.x;
  const int b = blockIdx.x / S;
  const int sl = blockIdx.x % S;
  const long long o_base = ((long long)b * S + sl) * k;
  const int T = M * k;
  auto key_at = [&](int i) {
    const int m = i / k, j = i - m * k;
    return tok_keys[(((long long)b * M + m) * S + sl) * k + j];
  };
  auto block_max = [&](unsigned long long best) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const unsigned long long y = __shfl_xor(best, off, 64);
      best = y > best ? y : best;
    }
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = best;
    __syncthreads();
    best = red[0];
#pragma unroll
    for (int w = 1; w < 4; ++w) best = red[w] > best ? red[w] : best;
    return best;
  };
  // 1. A floor: one token's k listed documents already have pooled scores >= its k-th listed score,
  //    so the pooled k-th best score is at least the largest such k-th score; lower entries drop out.
  unsigned long long fl = 0ull;
  for (int m = tid; m < M; m += 256) {
    const unsigned long long x = tok_keys[(((long long)b * M + m) * S + sl) * k + (k - 1)];
    fl = x > fl ? x : fl;
  }
  fl = block_max(fl);
  if (tid == 0) {
    floor_s = (uint32_t)(fl >> 32);  // score bits only: entries that tie with the floor stay
    n_surv = 0;
  }
  __syncthreads();
  const uint32_t floor_bits = floor_s;
  // 2. Survivors into LDS.
  for (int i = tid; i < T; i += 256) {
    const unsigned long long x = key_at(i);
    if (x != 0ull && (uint32_t)(x >> 32) >= floor_bits) {
      const int slot = atomicAdd(&n_surv, 1);
      if (slot < kPoolSurv) surv[slot] = x;
    }
  }
  __syncthreads();
  const int ns = n_surv;
  if (ns <= kPoolSurv) {
    // 3. k rounds of arg-max over the survivors; the entries of a chosen document are erased.
    for (int round = 0; round < k; ++round) {
      unsigned long long best = 0ull;
      for (int i = tid; i < ns; i += 256) best = surv[i] > best ? surv[i] : best;
      best = block_max(best);
      if (tid == 0) {
        out_idx[o_base + round] = best ? (int32_t)key_doc(best) : -1;
        if (out_score) out_score[o_base + round] = best ? key_score(best) : -INFINITY;
      }
      if (best != 0ull) {
        const uint32_t low = (uint32_t)best;  // ~doc: identical for every entry of that document
        for (int i = tid; i < ns; i += 256)
          if ((uint32_t)surv[i] == low) surv[i] = 0ull;
      }
      __syncthreads();
    }
    return;
  }
  // Fallback (more survivors than LDS holds): rounds over the lists in memory, skipping taken documents.
  unsigned long long prev = ~0ull;
  for (int round = 0; round < k; ++round) {
    unsigned long long best = 0ull;
    for (int i = tid; i < T; i += 256) {
      const unsigned long long x = key_at(i);
      if (x == 0ull || x >= prev || x <= best) continue;  // keys of one document differ in the score bits only
      const uint32_t doc = key_doc(x);
      bool dup = false;
      for (int w = 0; w < round; ++w) dup = dup || taken[w] == doc;
      if (!dup) best = x;
    }
    best = block_max(best);
    if (tid == 0) {
      out_idx[o_base + round] = best ? (int32_t)key_doc(best) : -1;
      if (out_score) out_score[o_base + round] = best ? key_score(best) : -INFINITY;
      taken[round] = best ? key_doc(best) : 0xffffffffu;
    }
    __syncthreads();
    prev = best ? best : 0ull;
  }
}

// Top-k of one row of document scores (MODE 2 of the scan): mat[g][qg][0..N).  One workgroup per row.
//   1. every thread takes the best score of its strided share of the row; every wave finds (a lower bound
//      on) the k-th best of its 64 lane maxima by a bitwise search with ballots, and the largest of the four
//      waves' bounds is a lower bound theta on the k-th best score of the row: some wave holds k distinct
//      documents scoring at least that much;
//   2. every document scoring >= theta goes to LDS (a few k of them) and is ranked by counting on the full
//      key.
// Exact, ties included (keys are (score, ~doc): a total order; theta compares scores only, so equal scores
// survive together).  If more survive than LDS holds (adversarial order), k rounds of a block-wide arg-max
// over the row take over.
constexpr int kRowSurv = 2048;
constexpr int kRowRegs = 32;  // scores a thread keeps in registers between the two passes

__global__ __launch_bounds__(256) void topk_rows_kernel(const float* __restrict__ mat,
                                                        int32_t* __restrict__ out_idx,
                                                        float* __restrict__ out_score,
                                                        unsigned long long* __restrict__ out_key, int BM,
                                                        int n_sel, int N, int k) {
  __shared__ unsigned long long surv[kRowSurv];
  __shared__ unsigned long long red[4];
  __shared__ uint32_t theta_w[4];
  __shared__ int n_surv;
  const int tid = threadIdx.x;
  const int qg = blockIdx.x % BM;
  const int g = blockIdx.x / BM;
  const float* row = mat + ((long long)g * BM + qg) * N;
  const long long o_base = ((long long)qg * n_sel + g) * k;
  float v[kRowRegs];
  unsigned long long best = 0ull;
#pragma unroll
  for (int u = 0; u < kRowRegs; ++u) {
    const int i = u * 256 + tid;
    v[u] = (i < N) ? row[i] : 0.f;
  }
#pragma unroll
  for (int u = 0; u < kRowRegs; ++u) {
    const int i = u * 256 + tid;
    const unsigned long long x = (i < N) ? make_key(v[u], (uint32_t)i) : 0ull;
    best = x > best ? x : best;
  }
  for (int i = kRowRegs * 256 + tid; i < N; i += 256) {  // rows longer than the register share
    const unsigned long long x = make_key(row[i], (uint32_t)i);
    best = x > best ? x : best;
  }
  {
    // the order-preserving image of this lane's best score (0: the lane holds no document); the largest value
    // whose low 12 bits are clear and that at least k lanes of the wave reach, 0 if fewer than k lanes hold one
    const uint32_t ob = (uint32_t)(best >> 32);
    uint32_t prefix = 0u;
    for (int bit = 31; bit >= 12; --bit) {
      const uint32_t cnd = prefix | (1u << bit);
      if (__popcll(__ballot(ob >= cnd)) >= k) prefix = cnd;  // wave-uniform
    }
    if ((tid & 63) == 0) theta_w[tid >> 6] = prefix;
  }
  if (tid == 0) n_surv = 0;
  __syncthreads();
  const uint32_t th01 = theta_w[0] > theta_w[1] ? theta_w[0] : theta_w[1];
  const uint32_t th23 = theta_w[2] > theta_w[3] ? theta_w[2] : theta_w[3];
  const uint32_t theta = th01 > th23 ? th01 : th23;
  auto keep = [&](unsigned long long x) {
    if (x != 0ull && (uint32_t)(x >> 32) >= theta) {
      const int slot = atomicAdd(&n_surv, 1);
      if (slot < kRowSurv) surv[slot] = x;
    }
  };
#pragma unroll
  for (int u = 0; u < kRowRegs; ++u) {
    const int i = u * 256 + tid;
    keep((i < N) ? make_key(v[u], (uint32_t)i) : 0ull);
  }
  for (int i = kRowRegs * 256 + tid; i < N; i += 256) keep(make_key(row[i], (uint32_t)i));
  __syncthreads();
  const int ns = n_surv;
  auto emit = [&](int rank, unsigned long long x) {
    if (out_key) {
      out_key[o_base + rank] = x;
    } else {
      out_idx[o_base + rank] = x ? (int32_t)key_doc(x) : -1;
      if (out_score) out_score[o_base + rank] = x ? key_score(x) : -INFINITY;
    }
  };
  if (ns <= kRowSurv) {
    for (int i = tid; i < ns; i += 256) {
      const unsigned long long x = surv[i];
      int rank = 0;
      for (int j = 0; j < ns; ++j) rank += (surv[j] > x) ? 1 : 0;
      if (rank < k) emit(rank, x);
    }
    for (int i = ns + tid; i < k; i += 256) emit(i, 0ull);  // fewer than k documents (cannot happen for k <= N)
    return;
  }
  unsigned long long prev = ~0ull;
  for (int round = 0; round < k; ++round) {
    unsigned long long bst = 0ull;
    for (int i = tid; i < N; i += 256) {
      const unsigned long long x = make_key(row[i], (uint32_t)i);
      if (x < prev && x > bst) bst = x;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const unsigned long long y = __shfl_xor(bst, off, 64);
      bst = y > bst ? y : bst;
    }
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = bst;
    __syncthreads();
    bst = red[0];
#pragma unroll
    for (int w = 1; w < 4; ++w) bst = red[w] > bst ? red[w] : bst;
    if (tid == 0) emit(round, bst);
    prev = bst ? bst : 0ull;
  }
}

// Combine the n_lists sorted lists (k entries each, zero-padded) of one (query, group).
//   1. A lower bound theta on the k-th best key: the first j+1 entries of every list, with
//      n_lists*(j+1) >= k, are that many distinct candidates, so their k-th largest is one.
//   2. Survivors (key >= theta) are compacted into LDS and ranked by counting.
//   3. If more than kMaxSurv survive (adversarial order), fall back to k rounds of block-wide argmax.
constexpr int kMaxSub = 1152;
constexpr int kMaxSurv = 2048;

// out_key != null: the winners are written as 64-bit keys instead (input of pool_tokens_kernel).
// parts > 1: first level of a two-level merge for very many lists.  Block (g, qg, part) combines
// lists [part * lpp, (part + 1) * lpp) and writes its k winners as a sorted list of keys to
// out_key[g][qg][part][k], the input layout of a second call with n_lists = parts.
__global__ __launch_bounds__(256) void score_merge_kernel(const unsigned long long* __restrict__ ws,
                                                          int32_t* __restrict__ out_idx,
                                                          float* __restrict__ out_score,
                                                          unsigned long long* __restrict__ out_key,
                                                          int BM, int Hkv, int n_lists_total, int k,
                                                          int lpp, int parts, const int* __restrict__ gate,
                                                          int gate_tokens, int gate_blocks) {
  __shared__ unsigned long long sub[kMaxSub];
  __shared__ unsigned long long surv[kMaxSurv];
  __shared__ unsigned long long red[4];
  __shared__ unsigned long long theta_s;
  __shared__ int n_surv;
  const int tid = threadIdx.x;
  const int part = blockIdx.x % parts;
  const int qg = (blockIdx.x / parts) % BM;
  const int g = blockIdx.x / parts / BM;
  // behind the one-pass filter of the scoring GEMM: only the token blocks it flagged have lists to merge
  if (gate != nullptr && gate[g * gate_blocks + qg / gate_tokens] == 0) return;
  const int l0 = part * lpp;
  const int n_lists = (n_lists_total - l0 < lpp) ? n_lists_total - l0 : lpp;
  const int T = n_lists * k;
  const unsigned long long* src = ws + (((long long)g * BM + qg) * n_lists_total + l0) * k;
  const long long o_base =
      (parts > 1) ? (((long long)g * BM + qg) * parts + part) * k : ((long long)qg * Hkv + g) * k;

  const int depth = (k + n_lists - 1) / n_lists;  // entries taken from the head of every list
  // k <= P < k + n_lists; any kMaxSub >= k heads of lists bound the k-th best key just as well
  const int P = (n_lists * depth <= kMaxSub) ? n_lists * depth : kMaxSub;
  for (int i = tid; i < P; i += 256) sub[i] = src[(i / depth) * k + (i % depth)];
  if (tid == 0) {
    n_surv = 0;
    theta_s = 0ull;
  }
  __syncthreads();
  for (int i = tid; i < P; i += 256) {
    const unsigned long long x = sub[i];
    int rank = 0;
    for (int j = 0; j < P; ++j) rank += (sub[j] > x) ? 1 : 0;
    if (rank == k - 1 && x != 0ull) theta_s = x;  // keys are distinct, zeros are padding
  }
  __syncthreads();
  const unsigned long long theta = theta_s;
  if (n_lists * depth <= kMaxSub) {
    // The heads of all lists are in LDS already, and the lists are sorted: a list holds further survivors only if
    // the last entry seen of it is still >= theta, and then only as far as its entries stay >= theta.  After the
    // streams' thresholds have converged that is a handful of entries per (query, head) instead of n_lists * k.
    for (int l = tid; l < n_lists; l += 256) {
      bool more = true;
      for (int j = 0; j < depth; ++j) {
        const unsigned long long x = sub[l * depth + j];
        more = x != 0ull && x >= theta;
        if (!more) break;
        const int slot = atomicAdd(&n_surv, 1);
        if (slot < kMaxSurv) surv[slot] = x;
      }
      for (int j = depth; more && j < k; ++j) {
        const unsigned long long x = src[l * k + j];
        more = x != 0ull && x >= theta;
        if (more) {
          const int slot = atomicAdd(&n_surv, 1);
          if (slot < kMaxSurv) surv[slot] = x;
        }
      }
    }
  } else {
    for (int i0 = 0; i0 < T; i0 += 256 * 8) {  // eight independent loads per thread in flight
      unsigned long long x[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * 256 + tid;
        x[u] = (i < T) ? src[i] : 0ull;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (x[u] != 0ull && x[u] >= theta) {
          const int slot = atomicAdd(&n_surv, 1);
          if (slot < kMaxSurv) surv[slot] = x[u];
        }
      }
    }
  }
  __syncthreads();
  const int S = n_surv;
  if (S <= kMaxSurv) {
    for (int i = tid; i < S; i += 256) {
      const unsigned long long x = surv[i];
      int rank = 0;
      for (int j = 0; j < S; ++j) rank += (surv[j] > x) ? 1 : 0;
      if (rank < k) {
        if (out_key) {
          out_key[o_base + rank] = x;
        } else {
          out_idx[o_base + rank] = (int32_t)key_doc(x);
          if (out_score) out_score[o_base + rank] = key_score(x);
        }
      }
    }
    for (int i = S + tid; i < k; i += 256) {  // fewer than k valid candidates (cannot happen for k <= N)
      if (out_key) {
        out_key[o_base + i] = 0ull;
      } else {
        out_idx[o_base + i] = -1;
        if (out_score) out_score[o_base + i] = -INFINITY;
      }
    }
    return;
  }
  // fallback: k rounds of "largest key below the previous winner"
  unsigned long long prev = ~0ull;
  for (int round = 0; round < k; ++round) {
    unsigned long long best = 0ull;
    for (int i = tid; i < T; i += 256) {
      const unsigned long long x = src[i];
      if (x < prev && x > best) best = x;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const unsigned long long y = __shfl_xor(best, off, 64);
      best = y > best ? y : best;
    }
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = best;
    __syncthreads();
    best = red[0];
#pragma unroll
    for (int w = 1; w < 4; ++w) best = red[w] > best ? red[w] : best;
    if (tid == 0) {
      if (out_key) {
        out_key[o_base + round] = best;
      } else {
        out_idx[o_base + round] = best ? (int32_t)key_doc(best) : -1;
        if (out_score) out_score[o_base + round] = best ? key_score(best) : -INFINITY;
      }
    }
    prev = best ? best : 0ull;
  }
}

// One wave per (tile of 8 queries, KV head): fold the r heads of the group into one fp32 routing
// query per token,  qf = (1/r) sum_h q_h / max(|q_h|, 1e-12)  (plain mean for the dot product), split it
// into bf16 hi + lo and store the MFMA A operands of the tile: lane 16q + n holds row n (query n/2,
// hi for even n, lo for odd n), dims 32s + 8q .. +8 of slice s.  Also resets the threshold-exchange
// buffer of the scan to -inf.
template <int D>
__global__ __launch_bounds__(64) void prep_scan_operands_kernel(const uint16_t* __restrict__ q_route,
                                                                uint4* __restrict__ qop, int BM, int Hq,
                                                                int Hkv, int r, int cos, int n_qtiles,
                                                                float* __restrict__ gmax, long long n_gmax) {
  constexpr int NS = D / 32, LPH = D / 8, HPL = 64 / LPH;
  __shared__ float qf[8][D];
  const int lane = threadIdx.x;
  const int qt = blockIdx.x % n_qtiles;
  const int g = blockIdx.x / n_qtiles;
  if (gmax != nullptr) {
    for (long long i = (long long)blockIdx.x * 64 + lane; i < n_gmax; i += (long long)gridDim.x * 64)
      gmax[i] = -INFINITY;
  }
  // Lane = (query lane / LPH, 16-byte piece lane % LPH): a lane loads the same piece of all r heads of
  // its query, so the head sum stays in the lane and the norms need only DPP sums over LPH <= 16 lanes.
  const int piece = lane % LPH;
#pragma unroll
  for (int pass = 0; pass < 8 / HPL; ++pass) {
    const int qi = pass * HPL + lane / LPH;
    const long long qg = (long long)qt * 8 + qi;
    uint4 v[8];
#pragma unroll
    for (int hh = 0; hh < 8; ++hh) {
      v[hh] = make_uint4(0, 0, 0, 0);
      if (qg < BM && hh < r)
        v[hh] = *reinterpret_cast<const uint4*>(q_route + (qg * Hq + g * r + hh) * D + piece * 8);
    }
    float f[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = 0.f;
#pragma unroll
    for (int hh = 0; hh < 8; ++hh) {
      if (hh < r) {  // wave-uniform
        const float x[8] = {bf16_lo(v[hh].x), bf16_hi(v[hh].x), bf16_lo(v[hh].y), bf16_hi(v[hh].y),
                            bf16_lo(v[hh].z), bf16_hi(v[hh].z), bf16_lo(v[hh].w), bf16_hi(v[hh].w)};
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += x[e] * x[e];
        ss = group_sum<LPH>(ss);
        const float w = cos ? 1.0f / fmaxf(sqrtf(ss), 1e-12f) : 1.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] += x[e] * w;
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[qi][piece * 8 + e] = f[e] / (float)r;
  }
  wave_sync();
  const int rr = lane >> 4, n = lane & 15;
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    uint32_t w[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      float h0, l0, h1, l1;
      split_bf16(qf[n >> 1][32 * s + 8 * rr + 2 * jj], h0, l0);
      split_bf16(qf[n >> 1][32 * s + 8 * rr + 2 * jj + 1], h1, l1);
      w[jj] = (n & 1) ? pack_bf16(l0, l1) : pack_bf16(h0, h1);
    }
    qop[(((long long)g * n_qtiles + qt) * NS + s) * 64 + lane] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Appends the buffers of the merge stage to a finished plan: the first-level winners of a two-level
// merge (very many lists) and the per-token winner keys of the token-pooling pass.
static void add_token_pool(const Dims& dm, int BM, int k, ScorePlan* p) {
  p->merge_lpp = 64;
  p->merge_parts = ((long long)p->n_splits * k > 16384) ? (p->n_splits + p->merge_lpp - 1) / p->merge_lpp : 1;
  p->off_part = p->ws_bytes;
  if (p->merge_parts > 1)
    p->ws_bytes += round_up256((size_t)p->n_sel * BM * p->merge_parts * k * sizeof(unsigned long long));
  p->off_tok = p->ws_bytes;
  if (dm.token_pool)
    p->ws_bytes += round_up256((size_t)BM * p->n_sel * k * sizeof(unsigned long long));
}

ScorePlan plan_score(const Dims& dm, int BM, int k) {
  ScorePlan p;
  // one selection per KV group, or (literal Eq. 2 head mean, more than one group) one for all heads
  p.all_heads = (dm.scope_all && dm.Hkv > 1) ? 1 : 0;
  p.n_sel = dm.scope_all ? 1 : dm.Hkv;
  p.use_gemm = gemm_path_applies(dm, BM, k) ? 1 : 0;
  if (p.use_gemm) {
    p.gemm = plan_score_gemm(dm, BM, k);
    p.n_splits = p.gemm.n_splits;
    p.q_per_pass = BM;
    p.n_pass = 1;
    p.exchange = 0;
    p.mode = 0;
    p.tiles_per_wave = 0;
    p.off_mat = 0;
    p.it_publish = p.it_adopt = 0;
    p.off_gmax = 0;
    p.off_qop = 0;
    p.n_qtiles = 0;
    p.ws_bytes = p.gemm.ws_bytes;
    add_token_pool(dm, BM, k, &p);
    return p;
  }
  p.q_per_pass = (BM <= 8 || p.all_heads) ? 8 : ((BM <= 16 || k > 24) ? 16 : 32);
  p.n_pass = (BM + p.q_per_pass - 1) / p.q_per_pass;
  long long ns = p.all_heads ? 2048 : 2048 / dm.Hkv;  // ~8 waves per CU on 256 CUs
  if (ns < 1) ns = 1;
  // streams of at least kPrefetch tiles; with 32 queries per pass the lists (64 entries each) must
  // also hold every document of the stream without pruning, so streams stay short there
  const long long min_len = kPrefetch;
  const long long by_tiles = (dm.tiles + min_len - 1) / min_len;
  if (ns > by_tiles) ns = by_tiles;
  if (ns > 1024 && !p.all_heads) ns = 1024;
  if (ns < 1) ns = 1;
  const long long tiles_per_split = (dm.tiles + ns - 1) / ns;
  p.n_splits = (int)((dm.tiles + tiles_per_split - 1) / tiles_per_split);
  const size_t list_bytes = round_up256((size_t)p.n_sel * BM * p.n_splits * k * sizeof(unsigned long long));
  // threshold exchange between waves: worth it (and sound) only for long streams with >= k waves per head
  const long long n_it_min = dm.tiles / p.n_splits;
  // Short streams: nothing to filter.  MODE 2 (score matrix + row top-k) when its fp32 rows fit the
  // lists' LDS and the matrix stays small; else MODE 1 (dense lists) when the lists hold the stream.
  p.mode = 0;
  p.tiles_per_wave = 0;
  if (!p.all_heads) {
    const long long dpt = 16 / dm.C;
    const long long n_it_max = (dm.tiles + p.n_splits - 1) / p.n_splits;
    const long long cap = kListBytes / (8 * p.q_per_pass), capf = kListBytes / (4 * p.q_per_pass);
    const size_t mat_bytes = (size_t)dm.Hkv * BM * dm.N * sizeof(float);
    const long long L = n_it_max < kPrefetch ? kPrefetch : n_it_max;
    if (L * dpt <= capf && L <= 64 && mat_bytes <= ((size_t)256 << 20)) {
      p.mode = 2;
      p.tiles_per_wave = (int)L;
      p.n_splits = (int)((dm.tiles + L - 1) / L);
    } else if (n_it_max * dpt <= cap) {
      p.mode = 1;
    }
  }
  p.exchange = (!p.all_heads && p.mode == 0 && n_it_min >= 64 && p.n_splits >= k && p.n_splits <= 256) ? 1 : 0;
  // exchange events sit at the head of a group of kPrefetch iterations
  p.it_publish = (int)(n_it_min / 12) / kPrefetch * kPrefetch;
  p.it_adopt = p.it_publish + 3 * kPrefetch;
  p.off_gmax = list_bytes;
  p.off_qop = list_bytes + (p.exchange ? round_up256((size_t)dm.Hkv * BM * p.n_splits * sizeof(float)) : 0);
  p.n_qtiles = p.n_pass * (p.q_per_pass / 8);
  p.ws_bytes = p.off_qop + round_up256((size_t)dm.Hkv * p.n_qtiles * (dm.d / 32) * 64 * 16);
  p.off_mat = p.ws_bytes;
  if (p.mode == 2) p.ws_bytes += round_up256((size_t)dm.Hkv * BM * dm.N * sizeof(float));
  add_token_pool(dm, BM, k, &p);
  return p;
}

int launch_score(const Dims& dm, const ScorePlan& pl, const void* q_route, int B, int M, const void* KR,
                 const float* inv_norm, int k, int32_t* out_idx, float* out_score, void* ws,
                 hipStream_t st) {
  const int BM = B * M;
  // with token pooling the per-token winners go to the workspace as keys and are pooled at the end
  unsigned long long* tok_keys = dm.token_pool ? (unsigned long long*)((char*)ws + pl.off_tok) : nullptr;
  auto pool_tokens = [&]() -> int {
    if (!dm.token_pool) return MSA_OK;
    hipLaunchKernelGGL(pool_tokens_kernel, dim3(B * pl.n_sel), dim3(256), 0, st,
                       (const unsigned long long*)tok_keys, out_idx, out_score, M, pl.n_sel, k);
    return hipGetLastError() == hipSuccess ? MSA_OK : MSA_ERR_HIP;
  };
  // combine the per-split lists of every (query, selection): one level, or two for very many lists
  const int* gate = nullptr;  // scoring GEMM with its one-pass filter: the token blocks whose lists are to be merged
  const int gate_tokens = pl.use_gemm ? (pl.gemm.tokens_per_wg > 0 ? pl.gemm.tokens_per_wg : 1) : 1;
  const int gate_blocks = pl.use_gemm ? pl.gemm.n_qblocks : 0;
  auto merge = [&](const unsigned long long* lists, int n_lists) -> int {
    if (pl.merge_parts > 1) {
      unsigned long long* part_keys = (unsigned long long*)((char*)ws + pl.off_part);
      hipLaunchKernelGGL(score_merge_kernel, dim3(BM * pl.n_sel * pl.merge_parts), dim3(256), 0, st, lists,
                         (int32_t*)nullptr, (float*)nullptr, part_keys, BM, pl.n_sel, n_lists, k,
                         pl.merge_lpp, pl.merge_parts, gate, gate_tokens, gate_blocks);
      if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
      lists = part_keys;
      n_lists = pl.merge_parts;
    }
    hipLaunchKernelGGL(score_merge_kernel, dim3(BM * pl.n_sel), dim3(256), 0, st, lists, out_idx, out_score,
                       tok_keys, BM, pl.n_sel, n_lists, k, n_lists, 1, gate, gate_tokens, gate_blocks);
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
    return pool_tokens();
  };
  if (pl.use_gemm) {
    const int rc = launch_score_gemm_scan(dm, pl.gemm, q_route, BM, KR, inv_norm, k, ws, st, out_idx, out_score,
                                          tok_keys, &gate);
    if (rc != MSA_OK) return rc;
    return merge((const unsigned long long*)((const char*)ws + pl.gemm.off_lists), pl.gemm.n_splits);
  }
  ScoreArgs a;
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
  a.n_splits = pl.n_splits;
  a.k = k;
  a.gmax = pl.exchange ? (float*)((char*)ws + pl.off_gmax) : nullptr;
  a.it_publish = pl.it_publish;
  a.it_adopt = pl.it_adopt;
  a.qop = (const uint4*)((char*)ws + pl.off_qop);
  a.mat = (pl.mode == 2) ? (float*)((char*)ws + pl.off_mat) : nullptr;
  a.tiles_per_wave = pl.tiles_per_wave;
  a.n_qtiles = pl.n_qtiles;
  a.q_route = (const uint16_t*)q_route;
  const bool fold_in_scan = !pl.all_heads && !pl.exchange;
  if (!fold_in_scan) {
    const long long n_gmax = pl.exchange ? (long long)dm.Hkv * BM * pl.n_splits : 0;
    const unsigned blocks = (unsigned)(pl.n_qtiles * dm.Hkv);
    if (dm.d == 128)
      hipLaunchKernelGGL(prep_scan_operands_kernel<128>, dim3(blocks), dim3(64), 0, st,
                         (const uint16_t*)q_route, (uint4*)((char*)ws + pl.off_qop), BM, dm.Hq, dm.Hkv,
                         dm.r, dm.cos, pl.n_qtiles, a.gmax, n_gmax);
    else
      hipLaunchKernelGGL(prep_scan_operands_kernel<64>, dim3(blocks), dim3(64), 0, st,
                         (const uint16_t*)q_route, (uint4*)((char*)ws + pl.off_qop), BM, dm.Hq, dm.Hkv,
                         dm.r, dm.cos, pl.n_qtiles, a.gmax, n_gmax);
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  }
  // an index of more than 512 MB outgrows the 256 MB of cache behind the L2s even across passes
  const bool stream_index = (size_t)dm.Hkv * dm.tiles * 16 * dm.d * 2 > ((size_t)512 << 20);
  const int wpb = pl.all_heads ? kAllWaves : kScanWaves;
  dim3 grid((pl.n_splits + wpb - 1) / wpb, pl.all_heads ? 1 : dm.Hkv), block(64 * wpb);
  profile_mark(dm, false, st);
  for (int pass = 0; pass < pl.n_pass; ++pass) {
    a.q0 = pass * pl.q_per_pass;
    if (pl.all_heads) {
#define MSA_SCAN_ALL(DD, HH) \
  do { \
    if (dm.cos && stream_index) hipLaunchKernelGGL((score_scan_all_kernel<DD, HH, true, true>), grid, block, 0, st, a); \
    else if (dm.cos) hipLaunchKernelGGL((score_scan_all_kernel<DD, HH, true, false>), grid, block, 0, st, a); \
    else if (stream_index) hipLaunchKernelGGL((score_scan_all_kernel<DD, HH, false, true>), grid, block, 0, st, a); \
    else hipLaunchKernelGGL((score_scan_all_kernel<DD, HH, false, false>), grid, block, 0, st, a); \
  } while (0)
      if (dm.d == 128) {
        if (dm.Hkv == 2) MSA_SCAN_ALL(128, 2); else if (dm.Hkv == 4) MSA_SCAN_ALL(128, 4); else MSA_SCAN_ALL(128, 8);
      } else {
        if (dm.Hkv == 2) MSA_SCAN_ALL(64, 2); else if (dm.Hkv == 4) MSA_SCAN_ALL(64, 4); else MSA_SCAN_ALL(64, 8);
      }
#undef MSA_SCAN_ALL
      if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
      continue;
    }
    const int nqt = pl.q_per_pass / 8;  // 1, 2 or 4
#define MSA_SCAN(DD, QQ, CC) \
  do { \
    if (pl.mode == 2) hipLaunchKernelGGL((score_scan_kernel<DD, QQ, CC, 2, true>), grid, block, 0, st, a); \
    else if (pl.mode == 1) hipLaunchKernelGGL((score_scan_kernel<DD, QQ, CC, 1, true>), grid, block, 0, st, a); \
    else if (fold_in_scan) hipLaunchKernelGGL((score_scan_kernel<DD, QQ, CC, 0, true>), grid, block, 0, st, a); \
    else hipLaunchKernelGGL((score_scan_kernel<DD, QQ, CC, 0, false>), grid, block, 0, st, a); \
  } while (0)
    if (dm.d == 128) {
      if (dm.cos) {
        if (nqt == 1) MSA_SCAN(128, 1, true); else if (nqt == 2) MSA_SCAN(128, 2, true); else MSA_SCAN(128, 4, true);
      } else {
        if (nqt == 1) MSA_SCAN(128, 1, false); else if (nqt == 2) MSA_SCAN(128, 2, false); else MSA_SCAN(128, 4, false);
      }
    } else {
      if (dm.cos) {
        if (nqt == 1) MSA_SCAN(64, 1, true); else if (nqt == 2) MSA_SCAN(64, 2, true); else MSA_SCAN(64, 4, true);
      } else {
        if (nqt == 1) MSA_SCAN(64, 1, false); else if (nqt == 2) MSA_SCAN(64, 2, false); else MSA_SCAN(64, 4, false);
      }
    }
#undef MSA_SCAN
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  }
  profile_mark(dm, true, st);
  if (pl.mode == 2) {
    hipLaunchKernelGGL(topk_rows_kernel, dim3(BM * pl.n_sel), dim3(256), 0, st, (const float*)a.mat, out_idx,
                       out_score, tok_keys, BM, pl.n_sel, dm.N, k);
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
    return pool_tokens();
  }
  return merge((const unsigned long long*)ws, pl.n_splits);
}

}  // namespace msa
