// msa_score_topk for MANY query tokens (prefill routing, B*M >= 64): the relevance scores of Eq. 2
// (paper, Section 3.2.1) as a real GEMM on the matrix cores, with the document max and a per-query
// top-k fused into the epilogue so that scores never reach memory.  This is the one place on the
// path that is MFMA-bound: 2 * (B*M) * Hkv * (N*C) * 2d flops (the factor 2d: the folded fp32 query is
// carried as a bf16 hi part and a bf16 lo part laid side by side along the contraction, so one
// accumulator receives q_hi.key + q_lo.key and a score keeps ~16 significant bits).
//
// Shape of the work
//   fold_queries_kernel : (1/r) sum_h q_h/|q_h| per (token, KV group) in fp32, once.
//   score_gemm_kernel   : a workgroup owns 256 query tokens of one KV head (4 waves x 64 tokens, the
//     queries stay in registers as B operands for the whole kernel) and walks a range of key
//     sub-tiles of 32 keys (= 4 documents at C = 8).  Two sub-tiles (four 16-key index tiles, 16 KiB,
//     contiguous in the tiled index) form a stage that is copied once to LDS (a ring of three
//     buffers, two copies in flight, one workgroup barrier per stage) and read by all four waves as
//     the A operand of v_mfma_f32_32x32x16_bf16: D[key][token].
//     Keys are the ROWS of the product, so the 8 chunks of a document sit in two lanes (l, l ^ 32)
//     as four accumulator registers each: document max = 3 in-lane max + one half-wave swap.
//     Each lane keeps a private sorted top-8 (or top-16) list (score, document) per token block in registers;
//     the lower half of the wave serves documents 0,1 of a sub-tile, the upper half documents 2,3.
//     Lists are merged per token at the end and written as sorted 64-bit keys, the same format the
//     streaming scan writes, so score_merge_kernel combines the key-range splits.
#include "msa_device.h"
#include "msa_host.h"

namespace msa {

typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kGemmMaxK = 16;     // longest per-lane list (k <= 16)
// Two shapes of the kernel: k <= 8 keeps two 32-token blocks per wave (256 tokens per workgroup) with 8-entry
// per-lane lists; 8 < k <= 16 keeps one block per wave (128 tokens per workgroup) with 16-entry lists -- the longer
// lists take the registers of the second block's query operands.

__device__ __forceinline__ f32x16_t mfma32(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  // D(32x32) += A(32x16) * B(16x32).  Lane l: A[l%32][8(l/32)..+8], B[8(l/32)..+8][l%32],
  // D register i: row (i%4) + 8(i/4) + 4(l/32), column l%32.
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Lower half of the wave: max(x[l], x[l + 32]); upper half: max(y[l - 32], y[l]).  One swap serves two values: the
// swap exchanges the upper half of its first operand with the lower half of its second, which leaves {x.lo, y.lo} and
// {x.hi, y.hi}.
__device__ __forceinline__ float max_across_halves_pair(float x, float y) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
  // the maximum as one instruction: fmaxf() first passes both halves of the swap through a canonicalising
  // v_max_f32 x, x, x, because it cannot tell that they are the (already canonical) products of the epilogue
  float m;
  asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(r[0]), "v"(r[1]));
  return m;
}

template <int W>
__device__ __forceinline__ float gsum(float x) {
  if (W >= 2) x += dpp_f<kDppXor1>(x);
  if (W >= 4) x += dpp_f<kDppXor2>(x);
  if (W >= 8) x += dpp_f<kDppHalfMirror>(x);
  if (W >= 16) x += dpp_f<kDppMirror>(x);
  return x;
}

// One wave per (token, KV group): qf[token][g][:] = (1/r) sum_h q_h / max(|q_h|, 1e-12)  (or the plain
// mean for the dot product).
// With eps != null (one-pass filter) it also writes, per (token, KV group), a bound on the difference between the
// score of any document computed from the bf16 hi parts of qf alone and its exact score: for a unit key,
// |(qf - hi(qf)) . key| <= |qf - hi(qf)|, plus the rounding of two fp32 accumulations over d products; and it clears
// the fallback flags of the token blocks.
template <int D>
__global__ __launch_bounds__(64) void fold_queries_kernel(const uint16_t* __restrict__ q_route,
                                                          float* __restrict__ qf, int Hq, int Hkv,
                                                          int r, int cos, float* __restrict__ eps,
                                                          int* __restrict__ flags, int n_flags) {
  constexpr int LPH = D / 8, HPL = 64 / LPH;
  const int lane = threadIdx.x;
  const int g = blockIdx.x % Hkv;
  const long long qg = blockIdx.x / Hkv;
  const int piece = lane % LPH, hs = lane / LPH;
  float f[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = 0.f;
  for (int hp = 0; hp * HPL < r; ++hp) {
    const int hh = hp * HPL + hs;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (hh < r) v = *reinterpret_cast<const uint4*>(q_route + (qg * Hq + g * r + hh) * D + piece * 8);
    const float x[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                        bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += x[e] * x[e];
    ss = gsum<LPH>(ss);
    const float w = cos ? 1.0f / fmaxf(sqrtf(ss), 1e-12f) : 1.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] += x[e] * w;
  }
#pragma unroll
  for (int off = LPH; off < 64; off <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] += __shfl_xor(f[e], off, 64);
  }
  float err2 = 0.f, n2 = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float x = f[e] / (float)r;
    float hi, lo;
    split_bf16(x, hi, lo);
    err2 += lo * lo;
    n2 += x * x;
    f[e] = x;
  }
  if (hs == 0) {
    float* dst = qf + (qg * Hkv + g) * D + piece * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) dst[e] = f[e];
  }
  if (eps != nullptr) {
    err2 = gsum<LPH>(err2);  // lanes 0 .. LPH-1 hold the D elements
    n2 = gsum<LPH>(n2);
    if (lane == 0) eps[qg * Hkv + g] = 1.01f * sqrtf(err2) + 2e-5f * sqrtf(n2) + 1e-7f;
    if (lane == 0 && (int)blockIdx.x < n_flags) flags[blockIdx.x] = 0;
  }
}

struct GemmArgs {
  int C;                    // chunks per document: 4, 8 or 16
  const float* qf;          // [BM][Hkv][D]
  const uint16_t* KR;       // tiled
  const float* inv_norm;    // may be null (dot)
  unsigned long long* ws;   // [Hkv][BM][n_splits][k]   (one-pass filter: [Hkv][BM][n_splits][2][list length])
  const int* flags;         // two-pass kernel behind the filter: [Hkv][n_qblocks], a workgroup runs only if its block's is set
  int BM, Hkv, N, k;
  long long tiles;          // 16-key tiles per head
  int n_qblocks, n_splits, stages_per_split;
};

// C8: eight chunks per document, the benchmark shape, known at compile time (it fills the register file exactly; the
// general epilogue for C = 4 / 16 is a second instantiation).
// HIONLY: the one-pass filter.  Only the bf16 hi parts of the queries are multiplied (half the matrix work, half the
// operand registers); the scores are approximate, within the bound that fold_queries_kernel writes, and both per-lane
// lists of every token are written out whole, for score_filter_select_kernel.
template <int D, int TB, int KL, bool C8, bool HIONLY>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void score_gemm_kernel(GemmArgs a) {
  constexpr int kGemmK = KL;               // per-lane list length
  constexpr int kGemmTokens = 128 * TB;    // tokens per workgroup (4 waves x TB blocks of 32)
  constexpr int NS8 = D / 16;            // 16-wide contraction slices per half (hi / lo)
  constexpr int SUB_BYTES = 32 * D * 2;  // one 32-key sub-tile
  constexpr int STAGE_BYTES = 2 * SUB_BYTES;  // a stage = two sub-tiles = 64 keys, one barrier
  constexpr int TILE_ELEMS = 16 * D;
  constexpr int LOADS = STAGE_BYTES / (256 * 16);  // 16-byte copies per thread per stage (4 at d=128)
  constexpr int MRG_BYTES = 4 * 32 * TB * 2 * kGemmK * 8;
  constexpr int RING_BYTES = 3 * STAGE_BYTES;
  // ring of three stages (two copies in flight while one is multiplied); the end-of-kernel merge of
  // the two half-wave lists reuses the same memory once the ring is drained
  __shared__ __attribute__((aligned(16))) unsigned char smem[RING_BYTES > MRG_BYTES ? RING_BYTES : MRG_BYTES];
  __shared__ __attribute__((aligned(16))) float ibuf[3][64];
  __shared__ __attribute__((aligned(16))) float ones[64];
  unsigned char* const kbuf0 = smem;
  unsigned char* const kbuf1 = smem + STAGE_BYTES;
  unsigned char* const kbuf2 = smem + 2 * STAGE_BYTES;
  typedef unsigned long long mrg_row_t[2 * kGemmK];
  mrg_row_t* const mrg = reinterpret_cast<mrg_row_t*>(smem);  // [4 waves * 32 TB tokens][2 * kGemmK]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = lane >> 5;   // half of the wave
  const int c = lane & 31;   // token column / key row
  const int g = blockIdx.x % a.Hkv;
  const int rest = blockIdx.x / a.Hkv;
  const int qb = rest % a.n_qblocks;
  const int ks = rest / a.n_qblocks;
  if (!HIONLY && a.flags != nullptr && a.flags[g * a.n_qblocks + qb] == 0) return;  // block-uniform, ahead of any barrier
  // Tiles and stages are counted in 32 bits: a head has at most N tiles (C <= 16), N an int.
  const int tiles = (int)a.tiles;
  const int n_stage = (tiles + 3) / 4;
  const int s0 = ks * a.stages_per_split;
  int s1 = s0 + a.stages_per_split;
  if (s1 > n_stage) s1 = n_stage;
  if (tid < 64) ones[tid] = 1.0f;

  // ---- B operands: this wave's 64 tokens, hi and lo halves, resident for the whole kernel -----
  const int tok0 = qb * kGemmTokens + wave * 32 * TB;
  bf16x8_t Bhi[TB][NS8], Blo[HIONLY ? 1 : TB][HIONLY ? 1 : NS8];
#pragma unroll
  for (int cb = 0; cb < TB; ++cb) {
    const int tok = tok0 + 32 * cb + c;
#pragma unroll
    for (int s = 0; s < NS8; ++s) {
      float x[8];
      if (tok < a.BM) {
        const float4* src = reinterpret_cast<const float4*>(a.qf + ((long long)tok * a.Hkv + g) * D + 16 * s + 8 * h);
        const float4 u0 = src[0], u1 = src[1];
        x[0] = u0.x; x[1] = u0.y; x[2] = u0.z; x[3] = u0.w;
        x[4] = u1.x; x[5] = u1.y; x[6] = u1.z; x[7] = u1.w;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = 0.f;
      }
      uint32_t wh[4], wl[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        float h0, l0, h1, l1;
        split_bf16(x[2 * jj], h0, l0);
        split_bf16(x[2 * jj + 1], h1, l1);
        wh[jj] = pack_bf16(h0, h1);
        wl[jj] = pack_bf16(l0, l1);
      }
      Bhi[cb][s] = as_bf16x8(make_uint4(wh[0], wh[1], wh[2], wh[3]));
      if constexpr (!HIONLY) Blo[cb][s] = as_bf16x8(make_uint4(wl[0], wl[1], wl[2], wl[3]));
    }
  }

  // per-lane sorted lists: [token block][rank]
  float lsc[TB][kGemmK];
  int ldoc[TB][kGemmK];
#pragma unroll
  for (int cb = 0; cb < TB; ++cb)
#pragma unroll
    for (int p = 0; p < kGemmK; ++p) {
      lsc[cb][p] = -INFINITY;
      ldoc[cb][p] = -1;
    }

  // Accepted candidates wait in a two-deep per-lane buffer (newest at index 0) and enter the sorted
  // lists only when some lane's buffer is full.  The sorted insertion costs the whole wave ~64 vector
  // instructions however few lanes take part; run for every sub-tile in which ANY of the 64 lanes accepts
  // a document it would run in most of them; run on full buffers it runs far less often (a deeper buffer
  // would help more but does not fit the register budget of two waves per SIMD: three entries spill).  The
  // acceptance test uses the list's last entry as it was at the last flush: a valid (if slightly stale)
  // lower bound, so nothing that belongs in the list is ever turned away.
  constexpr int kPend = HIONLY ? 4 : 2;  // the one-pass kernel has the registers of the lo operands to spare
  float psc[TB][kPend];
  int pdoc[TB][kPend];
  int pcnt[TB];
#pragma unroll
  for (int cb = 0; cb < TB; ++cb) pcnt[cb] = 0;
#pragma unroll
  for (int cb = 0; cb < TB; ++cb)
#pragma unroll
    for (int q = 0; q < kPend; ++q) {
      psc[cb][q] = -INFINITY;
      pdoc[cb][q] = -1;
    }
  // oldest first, so that among equal scores the lower document stays ahead
  auto flush = [&](int cb) __attribute__((always_inline)) {
#pragma unroll
    for (int q = kPend - 1; q >= 0; --q) {
      const float sc = psc[cb][q];
      const int doc = pdoc[cb][q];
      const bool ok = q < pcnt[cb] && sc > lsc[cb][kGemmK - 1];
      // branch-free insertion below every entry with score >= sc
#pragma unroll
      for (int p = kGemmK - 1; p >= 0; --p) {
        const float above = (p > 0) ? lsc[cb][p - 1] : INFINITY;
        const int above_d = (p > 0) ? ldoc[cb][p - 1] : -1;
        const bool shift = ok && sc > above;            // entry p-1 moves down to p
        const bool here = ok && !shift && sc > lsc[cb][p];
        lsc[cb][p] = shift ? above : (here ? sc : lsc[cb][p]);
        ldoc[cb][p] = shift ? above_d : (here ? doc : ldoc[cb][p]);
      }
    }
    pcnt[cb] = 0;
  };
  // One round of the same: every lane that has pending candidates inserts its OLDEST one.  Called when some lane's
  // buffer is full, which makes room in it; the other lanes use the round too.  (Emptying the buffers whenever one
  // of them is full takes kPend rounds for a lane or two that need them: about 1.8 times the rounds in all.)
  auto insert_oldest = [&](int cb) __attribute__((always_inline)) {
    const int pc = pcnt[cb];
    // The oldest pending candidate sits at index pc - 1.  The values pass through empty asm statements so that the
    // chain of selects stays one: as selects between loads of the arrays the compiler turns it into an indexed
    // load, which puts the arrays into scratch memory.
    float sc = psc[cb][0];
    int doc = pdoc[cb][0];
    asm volatile("" : "+v"(sc), "+v"(doc));
#pragma unroll
    for (int q = 1; q < kPend; ++q) {
      float t = psc[cb][q];
      int td = pdoc[cb][q];
      asm volatile("" : "+v"(t), "+v"(td));
      sc = (pc > q) ? t : sc;
      doc = (pc > q) ? td : doc;
    }
    const bool ok = pc > 0 && sc > lsc[cb][kGemmK - 1];
#pragma unroll
    for (int p = kGemmK - 1; p >= 0; --p) {
      const float above = (p > 0) ? lsc[cb][p - 1] : INFINITY;
      const int above_d = (p > 0) ? ldoc[cb][p - 1] : -1;
      const bool shift = ok && sc > above;
      const bool here = ok && !shift && sc > lsc[cb][p];
      lsc[cb][p] = shift ? above : (here ? sc : lsc[cb][p]);
      ldoc[cb][p] = shift ? above_d : (here ? doc : ldoc[cb][p]);
    }
    pcnt[cb] = pc - (pc > 0 ? 1 : 0);
  };

  // ---- staging of key stages: global -> LDS directly (no registers), two stages ahead ---------
  // A 64-lane global_load_lds_dwordx4 lands at LDS base + 16 * lane, and a stage is contiguous in
  // the tiled index, so wave w copies bytes [1024 (4i + w), +1024) of the stage with copy i; the
  // 64 reciprocal norms follow with one dword copy (every wave writes the same 64 floats, so each
  // wave issues exactly LOADS + 1 memory operations per stage and can wait on its own counter).
  const uint16_t* KRg = a.KR + (long long)g * a.tiles * TILE_ELEMS;
  const float* ing = a.inv_norm ? a.inv_norm + (long long)g * a.tiles * 16 : nullptr;
  // Copy i of a thread covers bytes [4096 i, 4096 (i + 1)) of the stage = TPC whole tiles, the same
  // tiles for every thread: the source is a scalar base plus the thread's constant offset.
  constexpr int TILE_BYTES = TILE_ELEMS * 2;
  constexpr int TPC = 4096 / TILE_BYTES;
  const uint32_t goff_full = tid * 16;                 // all TPC tiles of the copy exist
  const uint32_t goff_wrap = (tid * 16) % TILE_BYTES;  // only the first does: the others repeat it (masked)
  auto fetch = [&](int sg, unsigned char* kdst, float* idst) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      int tile = 4 * sg + TPC * i;
      if (tile >= tiles) tile = tiles - 1;             // past the end: repeat the last tile (masked)
      uint32_t goff = goff_full;
      if constexpr (TPC > 1) goff = (tile + TPC <= tiles) ? goff_full : goff_wrap;
      copy16_to_lds_async(reinterpret_cast<const unsigned char*>(KRg) + (long long)tile * TILE_BYTES, goff,
                          kdst + (i * 256 + wave * 64) * 16);
    }
    {
      // dot product: no norms; the copy still runs (from the index itself) to keep the counts equal,
      // and the multiply below reads the constant ones instead
      const int left = tiles - 4 * sg;  // tiles from this stage's first one to the end (>= 1: sg < n_stage)
      const long long key0 = (long long)sg * 64;
      const int room = left >= 4 ? 63 : 16 * left - 1;  // lanes beyond it repeat the last key
      const float* src = ing ? ing + key0 : reinterpret_cast<const float*>(KRg);
      copy4_to_lds_async(src, (uint32_t)((ing && lane > room) ? room : lane) * 4, idst);
    }
  };
  // wait until at most the copies of the newest stage are outstanding
  auto wait_oldest_copy = [&]() __attribute__((always_inline)) {
    if constexpr (LOADS == 4)
      asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
    else
      asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
  };

  // 32 keys x 64 tokens, contraction over [hi | lo], then the epilogue for these four documents
  auto sub_tile = [&](int st, const unsigned char* kcur, const float* icur) __attribute__((always_inline)) {
    f32x16_t acc[TB];
#pragma unroll
    for (int cb = 0; cb < TB; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;
    // A operand: key row c -> tile c/16, slot c%16; dims 16s + 8h .. +8 = piece 2s + h.  All slices
    // are requested before the first product so that LDS latency overlaps the matrix pipeline.
    bf16x8_t av[NS8];
#pragma unroll
    for (int s = 0; s < NS8; ++s)
      av[s] = as_bf16x8(*reinterpret_cast<const uint4*>(
          &kcur[(c >> 4) * (TILE_ELEMS * 2) + ((2 * s + h) * 16 + (c & 15)) * 16]));
#pragma unroll
    for (int s = 0; s < NS8; ++s) {
#pragma unroll
      for (int cb = 0; cb < TB; ++cb) {
        acc[cb] = mfma32(av[s], Bhi[cb][s], acc[cb]);
        if constexpr (!HIONLY) acc[cb] = mfma32(av[s], Blo[cb][s], acc[cb]);
      }
    }
    float inv[16];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float4 v = *reinterpret_cast<const float4*>(&icur[8 * j + 4 * h]);
      inv[4 * j] = v.x;
      inv[4 * j + 1] = v.y;
      inv[4 * j + 2] = v.z;
      inv[4 * j + 3] = v.w;
    }

    // ---- epilogue: document max, insertion into the per-lane lists ------------------------------
#pragma unroll
    for (int cb = 0; cb < TB; ++cb) {
      // a candidate document of this lane: onto the pending buffer (documents arrive in increasing order)
      auto push = [&](float sc, int doc) __attribute__((always_inline)) {
        const bool ok = doc < a.N && sc > lsc[cb][kGemmK - 1];
        if (__any(ok)) {
#pragma unroll
          for (int q = kPend - 1; q > 0; --q) {
            psc[cb][q] = ok ? psc[cb][q - 1] : psc[cb][q];
            pdoc[cb][q] = ok ? pdoc[cb][q - 1] : pdoc[cb][q];
          }
          psc[cb][0] = ok ? sc : psc[cb][0];
          pdoc[cb][0] = ok ? doc : pdoc[cb][0];
          pcnt[cb] += ok ? 1 : 0;
          if (__any(pcnt[cb] == kPend)) insert_oldest(cb);
        }
      };
      // m4[j]: max over the lane's four rows 8j + 4h .. + 3 of the sub-tile
      float m4[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float x0 = acc[cb][4 * j] * inv[4 * j], x1 = acc[cb][4 * j + 1] * inv[4 * j + 1];
        const float x2 = acc[cb][4 * j + 2] * inv[4 * j + 2], x3 = acc[cb][4 * j + 3] * inv[4 * j + 3];
        m4[j] = fmaxf(fmaxf(x0, x1), fmaxf(x2, x3));
      }
      if (C8 || a.C == 8) {
        // a document = rows 8j .. 8j + 7: the lane's four and the other half's four; the lower half of the wave
        // takes documents 0, 1 of the sub-tile, the upper half documents 2, 3
        const int doc0 = st * 4 + 2 * h;
        push(max_across_halves_pair(m4[0], m4[2]), doc0);
        push(max_across_halves_pair(m4[1], m4[3]), doc0 + 1);
      } else if constexpr (!C8) {
        if (a.C == 4) {
          // a document = the lane's four rows: document 2j + h of the sub-tile's eight, no exchange
#pragma unroll
          for (int j = 0; j < 4; ++j) push(m4[j], st * 8 + 2 * j + h);
        } else {
          // C == 16: a document = half of the sub-tile (rows 0..15 / 16..31, both halves of the wave); half h takes
          // document h
          push(max_across_halves_pair(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3])), st * 2 + h);
        }
      }
    }
  };

  auto body = [&](int sg, const unsigned char* kcur, const float* icur, unsigned char* knxt,
                  float* inxt) __attribute__((always_inline)) {
    // always issued (past the end it re-reads the last stage into a buffer nobody reads again)
    fetch((sg + 2 < s1) ? sg + 2 : s1 - 1, knxt, inxt);
    const float* isrc = ing ? icur : ones;
    sub_tile(2 * sg, kcur, isrc);
    sub_tile(2 * sg + 1, kcur + SUB_BYTES, ing ? icur + 32 : ones);
    wait_oldest_copy();  // this wave's part of the next stage has landed ...
    __syncthreads();     // ... and so has everyone's; all waves are done reading kcur
  };

  if (s0 < s1) {
    fetch(s0, kbuf0, ibuf[0]);
    fetch(s0 + 1 < s1 ? s0 + 1 : s1 - 1, kbuf1, ibuf[1]);
    wait_oldest_copy();
  }
  __syncthreads();
  for (int sg = s0; sg < s1; sg += 3) {  // the conditions are block-uniform
    body(sg, kbuf0, ibuf[0], kbuf2, ibuf[2]);
    if (sg + 1 < s1) body(sg + 1, kbuf1, ibuf[1], kbuf0, ibuf[0]);
    if (sg + 2 < s1) body(sg + 2, kbuf2, ibuf[2], kbuf1, ibuf[1]);
  }
  // drain the ring (re-reads issued past the end may still be landing) before its memory is reused
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

#pragma unroll
  for (int cb = 0; cb < TB; ++cb) flush(cb);
  if constexpr (HIONLY) {
    // both lists of every token as they are (sorted, zero = empty slot): [Hkv][BM][n_splits][2][KL]
#pragma unroll
    for (int cb = 0; cb < TB; ++cb) {
      const int tok = tok0 + 32 * cb + c;
      if (tok < a.BM) {
        unsigned long long* dst = a.ws + ((((long long)g * a.BM + tok) * a.n_splits + ks) * 2 + h) * kGemmK;
#pragma unroll
        for (int p = 0; p < kGemmK; ++p)
          dst[p] = (ldoc[cb][p] >= 0) ? make_key(lsc[cb][p], (uint32_t)ldoc[cb][p]) : 0ull;
      }
    }
    return;
  }
  // ---- merge the two half-wave lists of every token, write sorted keys -----------------------
#pragma unroll
  for (int cb = 0; cb < TB; ++cb) {
#pragma unroll
    for (int p = 0; p < kGemmK; ++p)
      mrg[wave * 32 * TB + 32 * cb + c][h * kGemmK + p] =
          (ldoc[cb][p] >= 0) ? make_key(lsc[cb][p], (uint32_t)ldoc[cb][p]) : 0ull;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int cb = 0; cb < TB; ++cb) {
    const int tok = tok0 + 32 * cb + c;
    const unsigned long long* both = mrg[wave * 32 * TB + 32 * cb + c];
#pragma unroll
    for (int p = 0; p < kGemmK; ++p) {
      const unsigned long long key = both[h * kGemmK + p];
      int rank = p;  // entries above it in its own (sorted) list
#pragma unroll
      for (int o = 0; o < kGemmK; ++o) rank += (both[(1 - h) * kGemmK + o] > key) ? 1 : 0;
      if (tok < a.BM && rank < a.k) {
        unsigned long long* dst = a.ws + (((long long)g * a.BM + tok) * a.n_splits + ks) * a.k;
        dst[rank] = key;  // zero keys (empty slots) rank last among themselves: harmless duplicates of 0
      }
    }
  }
}

// ---- Eq. 2 as printed for many query tokens: head mean over EVERY head (select_scope = ALL) -----------
// The chunk score is the mean over the KV groups g of  inv_norm_g(key) * (qf_g(token) . key_g):  every group
// has its own keys and its own reciprocal norms, so the groups' products cannot share one accumulator; each is
// scaled by its group's 1/|key| and added to a running total, and the document max and the top-k run ONCE on the
// total -- eight times the matrix work per selection of the per-group kernel above, and an epilogue that is
// amortised over the groups.
//
// A workgroup owns 128 query tokens (4 waves x 32) and a range of key stages.  The stages are walked in RANGES of
// R stages (R x 64 keys): for each group in turn the wave loads that group's folded queries of its 32 tokens
// (fp32 from the workspace, split into bf16 hi + lo operands in registers) and multiplies them with the group's
// keys of the range, streamed through the same three-buffer ring of asynchronous global -> LDS copies (entry e of
// the stream = range e / (HKV R), group (e / R) % HKV, stage e % R of the range); the totals of the range's
// 2 R sub-tiles stay in registers until the last group has been added.
constexpr int all_range(int KL) { return KL <= 8 ? 3 : 2; }  // stages per range (what the registers hold)

// HIONLY: the one-pass filter, as in score_gemm_kernel (hi parts only, both per-lane lists written out whole:
// [BM][n_splits][2][KL]); the two-pass form behind it runs only for the token blocks flagged in a.flags.
template <int D, int KL, int HKV, bool HIONLY>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void score_gemm_all_kernel(GemmArgs a) {
  constexpr int NS8 = D / 16;
  constexpr int SUB_BYTES = 32 * D * 2;
  constexpr int STAGE_BYTES = 2 * SUB_BYTES;
  constexpr int TILE_ELEMS = 16 * D;
  constexpr int LOADS = STAGE_BYTES / (256 * 16);
  constexpr int R = all_range(KL);
  constexpr int MRG_BYTES = 4 * 32 * 2 * KL * 8;
  constexpr int RING_BYTES = 3 * STAGE_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[RING_BYTES > MRG_BYTES ? RING_BYTES : MRG_BYTES];
  __shared__ __attribute__((aligned(16))) float ibuf[3][64];
  __shared__ __attribute__((aligned(16))) float ones[64];
  typedef unsigned long long mrg_row_t[2 * KL];
  mrg_row_t* const mrg = reinterpret_cast<mrg_row_t*>(smem);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = lane >> 5;
  const int c = lane & 31;
  // Workgroups go to the eight XCDs in turn (blockIdx % 8), each XCD with an L2 of its own: the token blocks of one
  // key split are kept on one XCD, so that XCD streams only its splits' part of the index from memory and the
  // other token blocks find it in the L2.
  int vb = blockIdx.x;
  {
    const int total = a.n_qblocks * a.n_splits;
    if (total % 8 == 0) vb = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
  }
  const int qb = vb % a.n_qblocks;
  const int ks = vb / a.n_qblocks;
  if (!HIONLY && a.flags != nullptr && a.flags[qb] == 0) return;  // block-uniform, ahead of any barrier
  const long long n_sub = (a.tiles + 1) / 2;
  const long long n_stage = (n_sub + 1) / 2;
  const long long n_range = (n_stage + R - 1) / R;
  const long long r0 = (long long)ks * a.stages_per_split;  // ranges per split
  long long r1 = r0 + a.stages_per_split;
  if (r1 > n_range) r1 = n_range;
  if (tid < 64) ones[tid] = 1.0f;
  const int tok = qb * 128 + wave * 32 + c;
  const int n_rg = (r1 > r0) ? (int)(r1 - r0) : 0;  // ranges of this workgroup

  float lsc[KL];
  int ldoc[KL];
#pragma unroll
  for (int p = 0; p < KL; ++p) {
    lsc[p] = -INFINITY;
    ldoc[p] = -1;
  }
  constexpr int kPend = 2;
  float psc[kPend];
  int pdoc[kPend];
  int pcnt = 0;
#pragma unroll
  for (int q = 0; q < kPend; ++q) {
    psc[q] = -INFINITY;
    pdoc[q] = -1;
  }
  auto flush = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int q = kPend - 1; q >= 0; --q) {  // oldest first: among equal scores the lower document stays ahead
      const float sc = psc[q];
      const int doc = pdoc[q];
      const bool ok = q < pcnt && sc > lsc[KL - 1];
#pragma unroll
      for (int p = KL - 1; p >= 0; --p) {
        const float above = (p > 0) ? lsc[p - 1] : INFINITY;
        const int above_d = (p > 0) ? ldoc[p - 1] : -1;
        const bool shift = ok && sc > above;
        const bool here = ok && !shift && sc > lsc[p];
        lsc[p] = shift ? above : (here ? sc : lsc[p]);
        ldoc[p] = shift ? above_d : (here ? doc : ldoc[p]);
      }
    }
    pcnt = 0;
  };

  constexpr int TILE_BYTES = TILE_ELEMS * 2;
  constexpr int TPC = 4096 / TILE_BYTES;
  const uint32_t goff_full = tid * 16;
  const uint32_t goff_wrap = (tid * 16) % TILE_BYTES;
  // The workgroup's stream of stages, in the order it multiplies them: range (local number rl), group, stage of the
  // range.  All of it is kept in small 32-bit counters: no division in the loop (64-bit divisions by HKV * R and a
  // 64-bit modulus per stage were 14 scalar instructions per MFMA).  Past the end the last entry is fetched again.
  auto fetch = [&](int rl, int g, int st, unsigned char* kdst, float* idst) __attribute__((always_inline)) {
    if (rl >= n_rg) {
      rl = n_rg - 1;
      g = HKV - 1;
      st = R - 1;
    }
    const long long sg = (r0 + rl) * R + st;  // may lie past the last stage of the index: fetched clamped, its documents masked
    const unsigned char* KRg = reinterpret_cast<const unsigned char*>(a.KR) + (long long)g * a.tiles * TILE_BYTES;
    const float* ing = a.inv_norm ? a.inv_norm + (long long)g * a.tiles * 16 : nullptr;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      long long tile = 4 * sg + TPC * i;
      if (tile >= a.tiles) tile = a.tiles - 1;
      uint32_t goff = goff_full;
      if constexpr (TPC > 1) goff = (tile + TPC <= a.tiles) ? goff_full : goff_wrap;
      copy16_to_lds_async(KRg + tile * TILE_BYTES, goff, kdst + (i * 256 + wave * 64) * 16);
    }
    {
      long long key0 = sg * 64;
      const long long last = a.tiles * 16 - 1;
      if (key0 > last) key0 = last;
      const int room = (int)(last - key0 < 63 ? last - key0 : 63);
      const float* src = ing ? ing + key0 : reinterpret_cast<const float*>(KRg);
      copy4_to_lds_async(src, (uint32_t)((ing && lane > room) ? room : lane) * 4, idst);
    }
  };
  auto wait_oldest_copy = [&]() __attribute__((always_inline)) {
    if constexpr (LOADS == 4)
      asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
    else
      asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
  };
  // ring slot of a stage: (number of the stage in the stream) mod 3 = (slot of its group's first stage + st) mod 3
  auto mod3 = [](int x) -> int { return x >= 6 ? x - 6 : (x >= 3 ? x - 3 : x); };
  auto ring_k = [&](int slot) -> unsigned char* { return smem + slot * STAGE_BYTES; };
  auto ring_i = [&](int slot) -> float* { return ibuf[slot]; };

  if (n_rg > 0) {
    fetch(0, 0, 0, ring_k(0), ring_i(0));
    fetch(0, 0, 1, ring_k(1), ring_i(1));
    wait_oldest_copy();
  }
  __syncthreads();
  const float inv_groups = 1.0f / (float)HKV;
  int slot0 = 0;  // ring slot of the current group's first stage (always 0 when R == 3)
  for (int rl = 0; rl < n_rg; ++rl) {  // block-uniform
    const long long rg = r0 + rl;
    f32x16_t tot[2 * R];
#pragma unroll
    for (int t = 0; t < 2 * R; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) tot[t][i] = 0.f;
    for (int g = 0; g < HKV; ++g) {
      // this group's folded queries of the wave's 32 tokens: hi and lo operands
      bf16x8_t Bhi[NS8], Blo[HIONLY ? 1 : NS8];
#pragma unroll
      for (int s = 0; s < NS8; ++s) {
        float x[8];
        if (tok < a.BM) {
          const float4* src =
              reinterpret_cast<const float4*>(a.qf + ((long long)tok * HKV + g) * D + 16 * s + 8 * h);
          const float4 u0 = src[0], u1 = src[1];
          x[0] = u0.x; x[1] = u0.y; x[2] = u0.z; x[3] = u0.w;
          x[4] = u1.x; x[5] = u1.y; x[6] = u1.z; x[7] = u1.w;
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i) x[i] = 0.f;
        }
        uint32_t wh[4], wl[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) split_pack_bf16(x[2 * jj], x[2 * jj + 1], wh[jj], wl[jj]);
        Bhi[s] = as_bf16x8(make_uint4(wh[0], wh[1], wh[2], wh[3]));
        if constexpr (!HIONLY) Blo[s] = as_bf16x8(make_uint4(wl[0], wl[1], wl[2], wl[3]));
      }
      // The operands are complete HERE, ahead of the first ring copy of the group.  The compiler waits for its own
      // loads with vmcnt(0) where they are first used; left to itself it places that use (and the wait) behind the
      // copy request of the first stage, and the wait then also covers the copies that were requested a moment ago.
#pragma unroll
      for (int s = 0; s < NS8; ++s) {
        asm volatile("" : "+v"(Bhi[s]));
        if constexpr (!HIONLY) asm volatile("" : "+v"(Blo[s]));
      }
#pragma unroll
      for (int st = 0; st < R; ++st) {
        {  // the stage two ahead in the stream: always issued (past the end: the last entry again)
          constexpr int RR = R;
          const int fst = (st + 2 < RR) ? st + 2 : st + 2 - RR;
          int fg = g, frl = rl;
          if (st + 2 >= RR) {
            fg = g + 1;
            if (fg == HKV) {
              fg = 0;
              frl = rl + 1;
            }
          }
          const int fslot = mod3(slot0 + st + 2);
          fetch(frl, fg, fst, ring_k(fslot), ring_i(fslot));
        }
        const int cslot = mod3(slot0 + st);
        const unsigned char* kcur = ring_k(cslot);
        const float* icur = a.inv_norm ? ring_i(cslot) : ones;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
          const unsigned char* kc = kcur + sub * SUB_BYTES;
          bf16x8_t av[NS8];
#pragma unroll
          for (int s = 0; s < NS8; ++s)
            av[s] = as_bf16x8(*reinterpret_cast<const uint4*>(
                &kc[(c >> 4) * (TILE_ELEMS * 2) + ((2 * s + h) * 16 + (c & 15)) * 16]));
          f32x16_t acc;
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
          for (int s = 0; s < NS8; ++s) {
            acc = mfma32(av[s], Bhi[s], acc);
            if constexpr (!HIONLY) acc = mfma32(av[s], Blo[s], acc);
          }
          const float* ic = a.inv_norm ? icur + 32 * sub : ones;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float4 v = *reinterpret_cast<const float4*>(&ic[8 * j + 4 * h]);
            tot[2 * st + sub][4 * j] += acc[4 * j] * v.x;
            tot[2 * st + sub][4 * j + 1] += acc[4 * j + 1] * v.y;
            tot[2 * st + sub][4 * j + 2] += acc[4 * j + 2] * v.z;
            tot[2 * st + sub][4 * j + 3] += acc[4 * j + 3] * v.w;
          }
        }
        wait_oldest_copy();
        __syncthreads();
      }
      if constexpr (R != 3) slot0 = mod3(slot0 + R);
    }
    // ---- the range's totals are complete: head mean, document max, per-lane lists ----------------------
#pragma unroll
    for (int t = 0; t < 2 * R; ++t) {
      const long long sub_tile = (rg * R + t / 2) * 2 + (t & 1);  // 32 keys
      auto push = [&](float sc, int doc) __attribute__((always_inline)) {
        const bool ok = doc < a.N && sc > lsc[KL - 1];
        if (__any(ok)) {
#pragma unroll
          for (int q = kPend - 1; q > 0; --q) {
            psc[q] = ok ? psc[q - 1] : psc[q];
            pdoc[q] = ok ? pdoc[q - 1] : pdoc[q];
          }
          psc[0] = ok ? sc : psc[0];
          pdoc[0] = ok ? doc : pdoc[0];
          pcnt += ok ? 1 : 0;
          if (__any(pcnt == kPend)) flush();
        }
      };
      float m4[4];  // max over the lane's four rows 8j + 4h .. + 3, head mean applied
#pragma unroll
      for (int j = 0; j < 4; ++j)
        m4[j] = fmaxf(fmaxf(tot[t][4 * j], tot[t][4 * j + 1]), fmaxf(tot[t][4 * j + 2], tot[t][4 * j + 3])) * inv_groups;
      if (a.C == 8) {
        const int doc0 = (int)sub_tile * 4 + 2 * h;
        push(max_across_halves_pair(m4[0], m4[2]), doc0);
        push(max_across_halves_pair(m4[1], m4[3]), doc0 + 1);
      } else if (a.C == 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) push(m4[j], (int)sub_tile * 8 + 2 * j + h);
      } else {  // C == 16
        push(max_across_halves_pair(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3])), (int)sub_tile * 2 + h);
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  flush();
  if constexpr (HIONLY) {
    if (tok < a.BM) {
      unsigned long long* dst = a.ws + (((long long)tok * a.n_splits + ks) * 2 + h) * KL;
#pragma unroll
      for (int p = 0; p < KL; ++p) dst[p] = (ldoc[p] >= 0) ? make_key(lsc[p], (uint32_t)ldoc[p]) : 0ull;
    }
    return;
  }
#pragma unroll
  for (int p = 0; p < KL; ++p)
    mrg[wave * 32 + c][h * KL + p] = (ldoc[p] >= 0) ? make_key(lsc[p], (uint32_t)ldoc[p]) : 0ull;
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  {
    const unsigned long long* both = mrg[wave * 32 + c];
#pragma unroll
    for (int p = 0; p < KL; ++p) {
      const unsigned long long key = both[h * KL + p];
      int rank = p;
#pragma unroll
      for (int o = 0; o < KL; ++o) rank += (both[(1 - h) * KL + o] > key) ? 1 : 0;
      if (tok < a.BM && rank < a.k) {
        unsigned long long* dst = a.ws + ((long long)tok * a.n_splits + ks) * a.k;
        dst[rank] = key;
      }
    }
  }
}

// ---- one-pass filter: candidates, exact scores ----------------------------------------------------------
// One wave per (token, KV group).  Input: the 2 * n_splits per-lane lists of the one-pass product (sorted, KL
// entries each, zero = empty), whose scores s~ differ from the exact scores s by at most eps.  Let t~ be the k-th
// largest s~.  The k documents with the largest s~ all have s >= t~ - eps, so the k-th largest exact score is at
// least t~ - eps, and every document of the exact top-k has s~ >= s - eps >= t~ - 2 eps: the candidates are all
// list entries with s~ >= t~ - 2 eps.  A lane's list holds the KL >= k best documents that lane saw; it can have
// dropped a candidate only if it is full and its last entry is itself inside the band -- then, or with more than
// kFilterMaxCand candidates, the token's block is flagged and redone by the two-pass kernel.
//
constexpr int kFilterMaxEntries = 1024;  // 2 * n_splits * KL

// The exact scores of the candidates follow in the same wave: Eq. 2 in fp32 from the folded fp32 query and the bf16
// routing keys (d = 128, eight chunks per document: eight lanes per chunk, 16 dims per lane), document max, then the k
// best by (score descending, index ascending), written as the final selection (or, for token pooling, as the sorted
// keys of the token).  Four (token, KV group) pairs per workgroup, one per wave; the waves never synchronise.
__global__ __launch_bounds__(256) void score_filter_select_kernel(const unsigned long long* __restrict__ lists,
                                                                  const float* __restrict__ eps,
                                                                  const float* __restrict__ qf,
                                                                  const uint16_t* __restrict__ KR,
                                                                  const float* __restrict__ inv_norm,
                                                                  int* __restrict__ flags, int32_t* __restrict__ out_idx,
                                                                  float* __restrict__ out_score,
                                                                  unsigned long long* __restrict__ out_key, int BM,
                                                                  int Hkv, int n_splits, int KL, int k,
                                                                  int tokens_per_wg, int n_qblocks, long long tiles,
                                                                  int all_heads) {
  constexpr int PER = kFilterMaxEntries / 64;
  constexpr int D = 128, C = 8;
  __shared__ int32_t cand_s[4][kFilterMaxCand];
  __shared__ unsigned long long keys_s[4][kFilterMaxCand];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  // one selection per (token, KV group), or (head mean over every head) per token: then the score of a chunk is the
  // mean over the groups of the groups' scores, and the bound the mean of the groups' bounds
  const int S = all_heads ? 1 : Hkv;    // selections per token
  const int GS = all_heads ? Hkv : 1;   // groups per selection
  const long long pair = (long long)blockIdx.x * 4 + wave;
  if (pair >= (long long)BM * S) return;  // wave-uniform; no workgroup barrier below
  const int g = (int)(pair % S);
  const int tok = (int)(pair / S);
  int32_t* cand = cand_s[wave];
  unsigned long long* keys = keys_s[wave];

  // ---- candidates --------------------------------------------------------------------------------------
  const int T = 2 * n_splits * KL;
  const unsigned long long* src = lists + ((long long)g * BM + tok) * T;
  const int per = (T + 63) / 64;  // wave-uniform: slots of x that hold entries
  unsigned long long x[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int e = lane + 64 * i;
    x[i] = (i < per && e < T) ? src[e] : 0ull;
  }
  // k-th largest one-pass score: bitwise search on the order-preserving image (the high word of a key)
  uint32_t prefix = 0u;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cnd = prefix | (1u << bit);
    int ge = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i)
      if (i < per) ge += __popcll(__ballot((uint32_t)(x[i] >> 32) >= cnd));
    if (ge >= k) prefix = cnd;  // wave-uniform
  }
  // fewer than k entries in all (prefix == 0): every entry is a candidate
  float e_sel = 0.f;
  for (int gg = 0; gg < GS; ++gg) e_sel += eps[(long long)tok * Hkv + g + gg];
  e_sel /= (float)GS;
  const float band = prefix ? unorderable(prefix) - 2.0f * e_sel : -INFINITY;
  int total = 0;
  bool overflow = false;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    if (i < per) {  // wave-uniform
      const int e = lane + 64 * i;
      const bool is = x[i] != 0ull && key_score(x[i]) >= band;
      overflow = overflow || (is && (e % KL) == KL - 1);  // a full list whose last entry is inside the band
      const unsigned long long m = __ballot(is);
      const int slot = total + __popcll(m & ((1ull << lane) - 1ull));
      if (is && slot < kFilterMaxCand) cand[slot] = (int32_t)key_doc(x[i]);
      total += __popcll(m);
    }
  }
  overflow = __any(overflow) || total > kFilterMaxCand;
  if (lane == 0 && overflow) flags[g * n_qblocks + tok / tokens_per_wg] = 1;  // (all heads: g = 0)
  const int n = total < kFilterMaxCand ? total : kFilterMaxCand;
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();

  // ---- exact scores ------------------------------------------------------------------------------------
  const int ch = lane >> 3, part = lane & 7;  // chunk of the document, 16-dim part of the key
  const float inv_gs = 1.0f / (float)GS;
  for (int j0 = 0; j0 < n; j0 += 4) {  // wave-uniform; four candidates at a time, all their loads in flight together
    long long doc[4];
    float tot[4] = {0.f, 0.f, 0.f, 0.f};  // the chunk's score, summed over the groups of the selection
#pragma unroll
    for (int u = 0; u < 4; ++u) doc[u] = cand[j0 + u < n ? j0 + u : n - 1];  // past the end: the last one again
    for (int gg = 0; gg < GS; ++gg) {
      const int gk = g + gg;  // KV group whose keys and folded query are multiplied
      float q[16];
      {
        const float4* qs = reinterpret_cast<const float4*>(qf + ((long long)tok * Hkv + gk) * D + 16 * part);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float4 v = qs[i];
          q[4 * i] = v.x; q[4 * i + 1] = v.y; q[4 * i + 2] = v.z; q[4 * i + 3] = v.w;
        }
      }
      const uint16_t* KRg = KR + (long long)gk * tiles * (16 * D);
      const float* ing = inv_norm + (long long)gk * tiles * 16;
      uint4 a0[4], a1[4];
      float kinv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const long long key = doc[u] * C + ch;       // routing key of this lane's chunk
        const long long tile = key >> 4;
        const int slot = (int)(key & 15);
        // tile layout [d / 8][16 keys][8 dims]: dims 16 part .. + 15 are pieces 2 part and 2 part + 1 of the key
        const uint16_t* kp = KRg + tile * (16 * D) + (2 * part * 16 + slot) * 8;
        a0[u] = *reinterpret_cast<const uint4*>(kp);
        a1[u] = *reinterpret_cast<const uint4*>(kp + 16 * 8);
        kinv[u] = ing[key];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t w[8] = {a0[u].x, a0[u].y, a0[u].z, a0[u].w, a1[u].x, a1[u].y, a1[u].z, a1[u].w};
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          acc = fmaf(q[2 * i], bf16_lo(w[i]), acc);
          acc = fmaf(q[2 * i + 1], bf16_hi(w[i]), acc);
        }
        acc = gsum<8>(acc);                          // the chunk's dot product, in its eight lanes
        tot[u] += acc * kinv[u];
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float sc = tot[u] * inv_gs;
      sc = fmaxf(sc, __shfl_xor(sc, 8, 64));         // document max over the eight chunks
      sc = fmaxf(sc, __shfl_xor(sc, 16, 64));
      sc = fmaxf(sc, __shfl_xor(sc, 32, 64));
      if (lane == 0 && j0 + u < n) keys[j0 + u] = make_key(sc, (uint32_t)doc[u]);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const long long o_base = ((long long)tok * S + g) * k;
  if (lane < n) {
    const unsigned long long mine = keys[lane];
    int rank = 0;
    for (int j = 0; j < n; ++j) rank += (keys[j] > mine) ? 1 : 0;
    if (rank < k) {
      if (out_key) {
        out_key[o_base + rank] = mine;
      } else {
        out_idx[o_base + rank] = (int32_t)key_doc(mine);
        if (out_score) out_score[o_base + rank] = key_score(mine);
      }
    }
  }
  for (int i = n + lane; i < k; i += 64) {  // fewer than k candidates (k > number of documents cannot happen)
    if (out_key) {
      out_key[o_base + i] = 0ull;
    } else {
      out_idx[o_base + i] = -1;
      if (out_score) out_score[o_base + i] = -INFINITY;
    }
  }
}

// ---- host side -----------------------------------------------------------------------------------
bool gemm_path_applies(const Dims& dm, int BM, int k) {
  // (one group with select_scope = ALL is the per-group kernel's case)
  return (dm.C == 4 || dm.C == 8 || dm.C == 16) && k <= kGemmMaxK && BM >= 64;
}

GemmPlan plan_score_gemm(const Dims& dm, int BM, int k) {
  GemmPlan p;
  p.all_heads = (dm.scope_all && dm.Hkv > 1) ? 1 : 0;
  if (p.all_heads) {
    // one workgroup per (128 tokens, range of key stages); the per-token lists are [BM][n_splits][k]
    p.n_qblocks = (BM + 127) / 128;
    const long long n_stage = ((dm.tiles + 1) / 2 + 1) / 2;
    const int R = all_range(k <= 8 ? 8 : 16);
    const long long n_range = (n_stage + R - 1) / R;
    long long want = (2 * 256) / (long long)p.n_qblocks;
    if (want < 1) want = 1;
    long long by_len = (n_range + 3) / 4;                            // at least 4 ranges per split
    long long ns = want < by_len ? want : by_len;
    if (ns < 1) ns = 1;
    if (ns > 64) ns = 64;
    p.stages_per_split = (int)((n_range + ns - 1) / ns);             // RANGES per split on this path
    p.n_splits = (int)((n_range + p.stages_per_split - 1) / p.stages_per_split);
    p.off_lists = round_up256((size_t)BM * dm.Hkv * dm.d * sizeof(float));
    p.ws_bytes = p.off_lists + round_up256((size_t)BM * p.n_splits * k * sizeof(unsigned long long));
    p.list_len = (k <= 8) ? 8 : 16;
    p.tokens_per_wg = 128;
    p.filter = (dm.cos && dm.d == 128 && dm.C == 8 && 2 * p.n_splits * p.list_len <= kFilterMaxEntries) ? 1 : 0;
    p.off_eps = p.off_flags = p.off_flists = 0;
    if (p.filter) {  // as below, with one selection per token
      p.off_flists = p.off_lists;
      size_t end = p.off_flists + round_up256((size_t)BM * p.n_splits * 2 * p.list_len * sizeof(unsigned long long));
      p.off_eps = end;
      end += round_up256((size_t)BM * dm.Hkv * sizeof(float));
      p.off_flags = end;
      end += round_up256((size_t)p.n_qblocks * sizeof(int));
      p.ws_bytes = end;
    }
    return p;
  }
  const int tokens_per_wg = (k <= 8) ? 256 : 128;
  p.n_qblocks = (BM + tokens_per_wg - 1) / tokens_per_wg;
  const long long n_stage = ((dm.tiles + 1) / 2 + 1) / 2;           // stages of 64 keys
  long long want = (2 * 256) / ((long long)dm.Hkv * p.n_qblocks);  // ~2 workgroups per CU
  if (want < 1) want = 1;
  long long by_len = (n_stage + 31) / 32;                          // at least 32 stages per split
  long long ns = want < by_len ? want : by_len;
  if (ns < 1) ns = 1;
  if (ns > 64) ns = 64;
  p.stages_per_split = (int)((n_stage + ns - 1) / ns);
  p.n_splits = (int)((n_stage + p.stages_per_split - 1) / p.stages_per_split);
  p.off_lists = round_up256((size_t)BM * dm.Hkv * dm.d * sizeof(float));
  p.ws_bytes = p.off_lists + round_up256((size_t)dm.Hkv * BM * p.n_splits * k * sizeof(unsigned long long));
  p.list_len = (k <= 8) ? 8 : 16;
  p.tokens_per_wg = tokens_per_wg;
  // The one-pass filter: cosine (the bound needs unit keys), the shape the exact-score kernel is written for, and
  // few enough list entries per token for one wave.
  p.filter = (dm.cos && dm.d == 128 && dm.C == 8 && 2 * p.n_splits * p.list_len <= kFilterMaxEntries) ? 1 : 0;
  p.off_eps = p.off_flags = p.off_flists = 0;
  if (p.filter) {
    // the two-pass kernel's lists (fallback) reuse the memory of the one-pass lists, which are twice as long
    p.off_flists = p.off_lists;
    size_t end = p.off_flists +
                 round_up256((size_t)dm.Hkv * BM * p.n_splits * 2 * p.list_len * sizeof(unsigned long long));
    p.off_eps = end;
    end += round_up256((size_t)BM * dm.Hkv * sizeof(float));
    p.off_flags = end;
    end += round_up256((size_t)dm.Hkv * p.n_qblocks * sizeof(int));
    p.ws_bytes = end;
  }
  return p;
}

int launch_score_gemm_scan(const Dims& dm, const GemmPlan& pl, const void* q_route, int BM, const void* KR,
                           const float* inv_norm, int k, void* ws, hipStream_t st, int32_t* out_idx,
                           float* out_score, unsigned long long* out_key, const int** gate_flags) {
  float* qf = (float*)ws;
  float* eps = pl.filter ? (float*)((char*)ws + pl.off_eps) : nullptr;
  int* flags = pl.filter ? (int*)((char*)ws + pl.off_flags) : nullptr;
  const int n_flags = pl.filter ? (pl.all_heads ? 1 : dm.Hkv) * pl.n_qblocks : 0;
  *gate_flags = flags;
  if (dm.d == 128)
    hipLaunchKernelGGL(fold_queries_kernel<128>, dim3((unsigned)(BM * dm.Hkv)), dim3(64), 0, st,
                       (const uint16_t*)q_route, qf, dm.Hq, dm.Hkv, dm.r, dm.cos, eps, flags, n_flags);
  else
    hipLaunchKernelGGL(fold_queries_kernel<64>, dim3((unsigned)(BM * dm.Hkv)), dim3(64), 0, st,
                       (const uint16_t*)q_route, qf, dm.Hq, dm.Hkv, dm.r, dm.cos, eps, flags, n_flags);
  if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  GemmArgs a;
  a.flags = nullptr;
  a.qf = qf;
  a.KR = (const uint16_t*)KR;
  a.inv_norm = dm.cos ? inv_norm : nullptr;
  a.ws = (unsigned long long*)((char*)ws + pl.off_lists);
  a.BM = BM;
  a.C = dm.C;
  a.Hkv = dm.Hkv;
  a.N = dm.N;
  a.k = k;
  a.tiles = dm.tiles;
  a.n_qblocks = pl.n_qblocks;
  a.n_splits = pl.n_splits;
  a.stages_per_split = pl.stages_per_split;
  if (pl.all_heads) {
    const unsigned nb = (unsigned)(pl.n_qblocks * pl.n_splits);
#define MSA_GEMM_ALL(DD, HH, ONE) \
  do { \
    if (k <= 8) hipLaunchKernelGGL((score_gemm_all_kernel<DD, 8, HH, ONE>), dim3(nb), dim3(256), 0, st, a); \
    else hipLaunchKernelGGL((score_gemm_all_kernel<DD, 16, HH, ONE>), dim3(nb), dim3(256), 0, st, a); \
  } while (0)
#define MSA_GEMM_ALL128(ONE) \
  do { \
    if (dm.Hkv == 2) MSA_GEMM_ALL(128, 2, ONE); else if (dm.Hkv == 4) MSA_GEMM_ALL(128, 4, ONE); \
    else MSA_GEMM_ALL(128, 8, ONE); \
  } while (0)
    if (pl.filter) {  // d = 128: one-pass product -> candidates -> exact scores -> two-pass kernel where flagged
      a.ws = (unsigned long long*)((char*)ws + pl.off_flists);
      profile_mark(dm, false, st);
      MSA_GEMM_ALL128(true);
      profile_mark(dm, true, st);
      if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
      hipLaunchKernelGGL(score_filter_select_kernel, dim3((unsigned)((BM + 3) / 4)), dim3(256), 0, st,
                         (const unsigned long long*)a.ws, (const float*)eps, (const float*)qf, (const uint16_t*)KR,
                         inv_norm, flags, out_idx, out_score, out_key, BM, dm.Hkv, pl.n_splits, pl.list_len, k,
                         pl.tokens_per_wg, pl.n_qblocks, dm.tiles, 1);
      if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
      a.ws = (unsigned long long*)((char*)ws + pl.off_lists);
      a.flags = flags;
      MSA_GEMM_ALL128(false);
      return hipGetLastError() == hipSuccess ? MSA_OK : MSA_ERR_HIP;
    }
    profile_mark(dm, false, st);
    if (dm.d == 128) {
      MSA_GEMM_ALL128(false);
    } else {
      if (dm.Hkv == 2) MSA_GEMM_ALL(64, 2, false); else if (dm.Hkv == 4) MSA_GEMM_ALL(64, 4, false);
      else MSA_GEMM_ALL(64, 8, false);
    }
#undef MSA_GEMM_ALL128
#undef MSA_GEMM_ALL
    profile_mark(dm, true, st);
    return hipGetLastError() == hipSuccess ? MSA_OK : MSA_ERR_HIP;
  }
  const unsigned blocks = (unsigned)(dm.Hkv * pl.n_qblocks * pl.n_splits);
  if (pl.filter) {
    // one-pass product -> candidates -> exact scores; then the two-pass kernel for the flagged token blocks only
    a.ws = (unsigned long long*)((char*)ws + pl.off_flists);
    profile_mark(dm, false, st);
    if (k <= 8) hipLaunchKernelGGL((score_gemm_kernel<128, 2, 8, true, true>), dim3(blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((score_gemm_kernel<128, 1, 16, true, true>), dim3(blocks), dim3(256), 0, st, a);
    profile_mark(dm, true, st);
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
    hipLaunchKernelGGL(score_filter_select_kernel, dim3((unsigned)((BM * dm.Hkv + 3) / 4)), dim3(256), 0, st,
                       (const unsigned long long*)a.ws, (const float*)eps, (const float*)qf, (const uint16_t*)KR,
                       inv_norm, flags, out_idx, out_score, out_key, BM, dm.Hkv, pl.n_splits, pl.list_len, k,
                       pl.tokens_per_wg, pl.n_qblocks, dm.tiles, 0);
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
    a.ws = (unsigned long long*)((char*)ws + pl.off_lists);
    a.flags = flags;
    if (k <= 8) hipLaunchKernelGGL((score_gemm_kernel<128, 2, 8, true, false>), dim3(blocks), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((score_gemm_kernel<128, 1, 16, true, false>), dim3(blocks), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? MSA_OK : MSA_ERR_HIP;
  }
  profile_mark(dm, false, st);
#define MSA_GEMM(DD, TT, KK) \
  do { \
    if (dm.C == 8) hipLaunchKernelGGL((score_gemm_kernel<DD, TT, KK, true, false>), dim3(blocks), dim3(256), 0, st, a); \
    else hipLaunchKernelGGL((score_gemm_kernel<DD, TT, KK, false, false>), dim3(blocks), dim3(256), 0, st, a); \
  } while (0)
  if (k <= 8) {
    if (dm.d == 128) MSA_GEMM(128, 2, 8); else MSA_GEMM(64, 2, 8);
  } else {
    if (dm.d == 128) MSA_GEMM(128, 1, 16); else MSA_GEMM(64, 1, 16);
  }
#undef MSA_GEMM
  profile_mark(dm, true, st);
  if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  return MSA_OK;
}

}  // namespace msa
