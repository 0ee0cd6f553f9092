// msa_sparse_attend for MANY query tokens that SHARE one selection (token_pool = 1: the routing of
// Eq. 2 as printed picks the documents once per question, so all M tokens of a batch row attend the
// same k documents, Eq. 3-4).  Then the gathered keys and values are common to every tile of query
// tokens and attention is a dense contraction on the matrix cores.
//
// Two kernels.
//   rotate_steps_kernel    rotates the keys of every 32-key step ONCE per (batch row, KV head) (Section
//                          3.2.2: positions restart at 0 in every document; the local context continues
//                          at pos0), rounds them to bf16 and stores them in MFMA operand order.
//   attend_prefill_kernel  a workgroup owns a tile of 4 * TPW query tokens of one (batch row, KV head),
//                          TPW = 32 / r tokens per wave, and a contiguous range of steps (split-K as in
//                          the decode path: same partials, same merge kernel; a range that is the only one
//                          writes the final output itself).  Per step:
//     copies     the step's rotated keys and its value rows go global -> LDS asynchronously, 16 bytes per
//                lane, two steps ahead of their use (four stages); value rows land with their 16-byte
//                pieces swizzled so that the transposing reads below are conflict free.  No registers,
//                no vector instructions.
//     scores     S^T[32 keys][32 slots] = K~ Q~^T with v_mfma_f32_32x32x16_bf16; a slot (column) is a
//                (token, head) pair.  The rotated, scaled queries stay in registers as bf16 (hi, lo) pairs
//                laid along the CONTRACTION (two products per slice into one accumulator), so a score
//                exists in exactly one lane and the softmax work is not duplicated.
//     softmax    online, per column (16 keys per lane, the other 16 in lane ^ 32); the weights go back as
//                bf16 hi and lo parts, two B operands of  O^T[dd][slot] += V^T[dd][key] P^T[key][slot]
//                that share one A operand: V^T comes from ds_read_b64_tr_b16 (16 lanes exchange 4 x 4
//                elements on the way out of LDS) in the order of the lane's own score registers.
//   The loop is software pipelined: the score products of step i + 1 are issued next to the softmax
//   arithmetic of step i.  One bare barrier per step.
// Causality: local key t is visible to token m iff pos0 + t <= q_pos[m]; the mask is per column and
// the workgroup stops at the last step any of its tokens can see.
#include "msa_attend.h"

namespace msa {

typedef float f32x16p_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f32x16p_t mfma32p(bf16x8_t a, bf16x8_t b, f32x16p_t c) {
  // D(32x32) += A(32x16) * B(16x32).  Lane l: A[l%32][8(l/32)..+8], B[8(l/32)..+8][l%32],
  // D register i: row (i%4) + 8(i/4) + 4(l/32), column l%32.
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// After the swap of x with itself every lane holds the values of both lanes (l & 31) and (l & 31) + 32.
__device__ __forceinline__ float both_halves_max(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float both_halves_sum(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// The keys of a (batch row, KV head) are the same for every token tile, so they are rotated ONCE, by
// this kernel, and stored step by step in the order the tiled kernel keeps them in LDS
// ([piece][key][8 bf16], 32 keys per step); the tiled kernel then copies a step global -> LDS
// without touching a register or a vector instruction.  One workgroup per (step, KV head, batch row);
// the step numbering and the row clamping are the tiled kernel's (all Lloc local rows are prepared,
// whatever the tokens of a tile can see).  Angles come straight from a double-precision range
// reduction: no recurrence, so these keys are if anything more accurate than in-kernel rotation.
template <int D>
__global__ __launch_bounds__(256) void rotate_steps_kernel(AttendArgs a, RopeTheta th, uint16_t* __restrict__ Krot) {
  constexpr int HALF = D / 2;
  constexpr int PPH = D / 16;
  const int tid = threadIdx.x;
  if (tid >= 32 * PPH) return;
  const int kr = tid / PPH, pc = tid % PPH;
  const int st = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const uint16_t* Kb;
  int rows_valid, p_first;
  if (st < a.steps_mem) {
    const long long idx_row = (a.idx_rows_per_b == 1) ? b : (long long)b * a.M;
    const int32_t* idx_g = a.idx + (idx_row * a.idx_sel + (a.idx_sel == 1 ? 0 : g)) * a.k;
    const int tok = st * 32;
    const int slot = tok / a.G;
    const int pin = tok - slot * a.G;
    const int doc = idx_g[slot];
    if (doc < 0 || doc >= a.N) return;
    int len = a.G;
    if (a.lens != nullptr) {
      len = a.lens[doc];
      len = len < 1 ? 1 : (len > a.G ? a.G : len);
    }
    if (pin >= len) return;
    Kb = a.K + (((long long)doc * a.Hkv + g) * a.G + pin) * D;
    rows_valid = len - pin < 32 ? len - pin : 32;
    p_first = pin;
  } else {
    const int t0 = (st - a.steps_mem) * 32;
    if (t0 >= a.Lloc) return;
    Kb = a.Kloc + (((long long)b * a.Hkv + g) * a.Lloc + t0) * D;
    rows_valid = a.Lloc - t0 < 32 ? a.Lloc - t0 : 32;
    p_first = a.pos0 + t0;
  }
  const int row = kr < rows_valid ? kr : rows_valid - 1;
  const uint16_t* rp = Kb + (long long)row * D + pc * 8;
  const uint4 k1 = *reinterpret_cast<const uint4*>(rp);
  const uint4 k2 = *reinterpret_cast<const uint4*>(rp + HALF);
  const uint32_t w1[4] = {k1.x, k1.y, k1.z, k1.w}, w2[4] = {k2.x, k2.y, k2.z, k2.w};
  uint32_t y1[4], y2[4];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    const float2 c0 = cis_pos(p_first + row, th.th[8 * pc + 2 * jj]);
    const float2 c1 = cis_pos(p_first + row, th.th[8 * pc + 2 * jj + 1]);
    const float p0 = bf16_lo(w1[jj]), p1 = bf16_hi(w1[jj]);
    const float q0 = bf16_lo(w2[jj]), q1 = bf16_hi(w2[jj]);
    y1[jj] = pack_bf16(p0 * c0.x - q0 * c0.y, p1 * c1.x - q1 * c1.y);
    y2[jj] = pack_bf16(q0 * c0.x + p0 * c0.y, q1 * c1.x + p1 * c1.y);
  }
  unsigned char* blk = reinterpret_cast<unsigned char*>(Krot) +
                       (((long long)b * a.Hkv + g) * a.steps_total + st) * (32 * D * 2);
  *reinterpret_cast<uint4*>(&blk[(pc * 32 + kr) * 16]) = make_uint4(y1[0], y1[1], y1[2], y1[3]);
  *reinterpret_cast<uint4*>(&blk[((pc + PPH) * 32 + kr) * 16]) = make_uint4(y2[0], y2[1], y2[2], y2[3]);
}

template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void attend_prefill_kernel(AttendArgs a, RopeTheta th, int tpw,
                                                             int n_ttiles) {
  constexpr int HALF = D / 2;
  constexpr int NP = D / 8;          // 16-byte pieces per row
  constexpr int NS = D / 16;         // 16-wide contraction slices of the score product
  constexpr int NT = D / 32;         // 32-row tiles of the output product
  constexpr int KT_BYTES = 32 * D * 2;
  constexpr int VT_BYTES = 32 * D * 2;
  constexpr int NCP = 32 * NP / 256;  // 16-byte copies per thread, step and operand
  static_assert(NCP >= 1 && NCP * 256 == 32 * NP, "a step is a whole number of 256-thread copies");

  constexpr int NBUF = 4;             // stages in LDS: two in use (values of step i, keys of step i + 1), two on their way
  constexpr int ANG_BYTES = 4 * 16 * HALF * 8;  // prologue only: (cos, sin)(q_pos theta_u), 16 tokens x 4 waves
  constexpr int STAGE_BYTES = NBUF * (KT_BYTES + VT_BYTES);
  __shared__ __attribute__((aligned(16))) unsigned char smem[STAGE_BYTES > ANG_BYTES ? STAGE_BYTES : ANG_BYTES];
  unsigned char* const kt0 = smem;                    // rotated keys [piece][key][8 bf16], NBUF stages
  unsigned char* const vt0 = smem + NBUF * KT_BYTES;  // value rows [key][piece ^ 4 (key & 1)][8 bf16], NBUF stages
  constexpr int kSelCache = MSA_MAX_TOPK;  // a selection has at most this many slots
  __shared__ int sel_doc[kSelCache], sel_len[kSelCache];
  __shared__ int nvis_s[128];      // visible local tokens of each token of the tile (4 waves x 32 / r tokens)

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = lane >> 5;
  const int col = lane & 31;
  const int sp = blockIdx.x;
  const int g = blockIdx.y;
  const int b = blockIdx.z / n_ttiles;
  const int tt = blockIdx.z % n_ttiles;
  const int tile_tok = 4 * tpw;             // tokens per workgroup
  const int m_tile = tt * tile_tok;         // first token of the tile
  const int r = a.r;

  // ---- prologue ---------------------------------------------------------------------------------
  if (tid < 128) {
    int nv = 0;
    const int m = m_tile + tid;
    if (tid < tile_tok && m < a.M) {
      nv = a.q_pos[(long long)b * a.M + m] - a.pos0 + 1;
      nv = nv < 0 ? 0 : (nv > a.Lloc ? a.Lloc : nv);
    }
    nvis_s[tid] = nv;
  }
  __syncthreads();
  int nvis_blk = 0;
  for (int i = 0; i < tile_tok; ++i) nvis_blk = nvis_s[i] > nvis_blk ? nvis_s[i] : nvis_blk;

  // B operands of the score product: column = (token, head) pair; hi and lo parts of the rotated, scaled
  // query are two operands that go into the same accumulator
  const int tl = col / r, hh = col - tl * r;
  const int m_tok = m_tile + wave * tpw + tl;           // this column's query token
  const bool tok_ok = tl < tpw && m_tok < a.M;
  const int nvis_col = tok_ok ? nvis_s[wave * tpw + tl] : 0;
  bf16x8_t bqh[NS], bql[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) bqh[s] = bql[s] = as_bf16x8(make_uint4(0, 0, 0, 0));
  // (cos, sin)(q_pos theta_u) of 16 of this wave's tokens at a time, staged in the wave's own part of
  // the (still unused) key buffer
  float2* ang = reinterpret_cast<float2*>(smem) + wave * (16 * HALF);  // [16][HALF]
  for (int rd = 0; rd * 16 < tpw; ++rd) {
    for (int e = lane; e < 16 * HALF; e += 64) {
      const int t16 = e / HALF, u = e % HALF;
      const int m = m_tile + wave * tpw + rd * 16 + t16;
      const int qp = (rd * 16 + t16 < tpw && m < a.M) ? a.q_pos[(long long)b * a.M + m] : 0;
      ang[e] = cis_pos(qp, th.th[u]);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (tok_ok && (tl >> 4) == rd) {
      const uint16_t* qp = a.q + (((long long)b * a.M + m_tok) * a.Hq + g * r + hh) * D;
#pragma unroll
      for (int s = 0; s < NS / 2; ++s) {
        // dims 16 s + 8 h .. +8 (first half) and their partners + D/2 (slice s + NS/2)
        const uint4 r1 = *reinterpret_cast<const uint4*>(qp + 16 * s + 8 * h);
        const uint4 r2 = *reinterpret_cast<const uint4*>(qp + HALF + 16 * s + 8 * h);
        const uint32_t w1[4] = {r1.x, r1.y, r1.z, r1.w}, w2[4] = {r2.x, r2.y, r2.z, r2.w};
        uint32_t h1w[4], l1w[4], h2w[4], l2w[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          float y1[2], y2[2];
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const float x1 = e ? bf16_hi(w1[jj]) : bf16_lo(w1[jj]);
            const float x2 = e ? bf16_hi(w2[jj]) : bf16_lo(w2[jj]);
            const float2 cs = ang[(tl & 15) * HALF + 16 * s + 8 * h + 2 * jj + e];
            y1[e] = (x1 * cs.x - x2 * cs.y) * a.qscale;
            y2[e] = (x2 * cs.x + x1 * cs.y) * a.qscale;
          }
          float h0, l0, h1, l1;
          split_bf16(y1[0], h0, l0);
          split_bf16(y1[1], h1, l1);
          h1w[jj] = pack_bf16(h0, h1);
          l1w[jj] = pack_bf16(l0, l1);
          split_bf16(y2[0], h0, l0);
          split_bf16(y2[1], h1, l1);
          h2w[jj] = pack_bf16(h0, h1);
          l2w[jj] = pack_bf16(l0, l1);
        }
        bqh[s] = as_bf16x8(make_uint4(h1w[0], h1w[1], h1w[2], h1w[3]));
        bql[s] = as_bf16x8(make_uint4(l1w[0], l1w[1], l1w[2], l1w[3]));
        bqh[s + NS / 2] = as_bf16x8(make_uint4(h2w[0], h2w[1], h2w[2], h2w[3]));
        bql[s + NS / 2] = as_bf16x8(make_uint4(l2w[0], l2w[1], l2w[2], l2w[3]));
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();  // the angle staging area becomes the key buffer

  // ---- this workgroup's steps -----------------------------------------------------------------
  const int sb = sp * a.steps_per_split;
  int se = sb + a.steps_per_split;
  if (se > a.steps_total) se = a.steps_total;
  const long long idx_row = (a.idx_rows_per_b == 1) ? b : (long long)b * a.M;  // shared selection: row of b
  const int32_t* idx_g = a.idx + (idx_row * a.idx_sel + (a.idx_sel == 1 ? 0 : g)) * a.k;

  // The selection of this split's documents, read once: (document, rows that exist) of the slots from the
  // split's first one on; pads and ids outside the bank get 0 rows.
  const int slot0 = (int)(((long long)sb * 32) / a.G);
  {
    const int n_mem_slots = sb < a.steps_mem ? a.k - slot0 : 0;
    if (tid < kSelCache && tid < n_mem_slots) {
      const int doc = idx_g[slot0 + tid];
      int len = 0;
      if (doc >= 0 && doc < a.N) {
        len = a.G;
        if (a.lens != nullptr) {
          len = a.lens[doc];
          len = len < 1 ? 1 : (len > a.G ? a.G : len);
        }
      }
      sel_doc[tid] = doc;
      sel_len[tid] = len;
    }
  }
  __syncthreads();
  auto lookup = [&](int slot, int& doc, int& len) {  // block-uniform; slot < k <= kSelCache
    const int i = slot - slot0;
    doc = __builtin_amdgcn_readfirstlane(sel_doc[i]);
    len = __builtin_amdgcn_readfirstlane(sel_len[i]);
  };

  struct StepSrc {
    const uint16_t* Vb;  // first value row of the step
    int rows_valid, p_first, t0, st, len;
    bool is_mem;
  };
  // first step >= st of this split that holds rows (se if none); block-uniform
  auto locate = [&](int st, StepSrc& ss) -> int {
    while (st < se) {
      if (st < a.steps_mem) {
        const int tok = st * 32;
        const int slot = tok / a.G;
        const int pin = tok - slot * a.G;
        int doc, len;
        lookup(slot, doc, len);
        if (pin >= len) {  // a pad, or past the document's last token: on to the next slot (G % 32 == 0)
          st = (slot + 1) * (a.G / 32);
          continue;
        }
        ss.Vb = a.V + (((long long)doc * a.Hkv + g) * a.G + pin) * D;
        ss.rows_valid = len - pin < 32 ? len - pin : 32;
        ss.p_first = pin;
        ss.t0 = 0;
        ss.len = len;
        ss.is_mem = true;
      } else {
        const int t0 = (st - a.steps_mem) * 32;
        if (t0 >= nvis_blk) return se;
        ss.Vb = a.Vloc + (((long long)b * a.Hkv + g) * a.Lloc + t0) * D;
        ss.rows_valid = nvis_blk - t0 < 32 ? nvis_blk - t0 : 32;
        ss.p_first = a.pos0 + t0;
        ss.t0 = t0;
        ss.len = 0;
        ss.is_mem = false;
      }
      ss.st = st;
      return st;
    }
    return se;
  };
  // the step after ss: inside a document it is the next 32 rows, no lookup
  auto advance = [&](StepSrc& ss) -> int {
    const int st = ss.st + 1;
    if (st >= se) return se;
    if (ss.is_mem && ss.p_first + 32 < ss.len) {
      ss.Vb += 32 * D;
      ss.p_first += 32;
      ss.rows_valid = ss.len - ss.p_first < 32 ? ss.len - ss.p_first : 32;
      ss.st = st;
      return st;
    }
    return locate(st, ss);
  };

  // Global -> LDS copies of a step, 16 bytes per lane: a wave's 64 pieces land side by side.  Keys are
  // stored in operand order already.  Value row `key` keeps its piece c at place c ^ 4 (key & 1): rows
  // that the transposing reads below fetch together then start 64 bytes apart in the banks.
  const unsigned char* const ksrc0 = reinterpret_cast<const unsigned char*>(a.Krot) +
                                     ((long long)b * a.Hkv + g) * a.steps_total * KT_BYTES;
  int vkey[NCP], vcol[NCP];  // this thread's value pieces: row of the step, element of the row
#pragma unroll
  for (int i = 0; i < NCP; ++i) {
    const int x = i * 256 + tid;
    vkey[i] = x / NP;
    vcol[i] = ((x % NP) ^ (4 * (vkey[i] & 1))) * 8;
  }
  auto issue_loads = [&](const StepSrc& ss, int into) {
    const unsigned char* ksrc = ksrc0 + (long long)ss.st * KT_BYTES;
#pragma unroll
    for (int i = 0; i < NCP; ++i)
      copy16_to_lds_async(ksrc, i * 4096 + tid * 16, kt0 + into * KT_BYTES + (i * 256 + wave * 64) * 16);
#pragma unroll
    for (int i = 0; i < NCP; ++i) {
      const int row = vkey[i] < ss.rows_valid ? vkey[i] : ss.rows_valid - 1;
      copy16_to_lds_async(ss.Vb, (row * D + vcol[i]) * 2, vt0 + into * VT_BYTES + (i * 256 + wave * 64) * 16);
    }
  };
  // Transposing 64-bit LDS read (ds_read_b64_tr_b16): among 16 lanes, lane j hands in the address of
  // elements 4 (j % 4) .. + 3 of row j / 4 and receives element j of rows 0 .. 3.  Lane l of the second
  // product needs V[keys 16 sg + 4 h + {0..3, 8..11}][32 t + col]: two such reads per operand.
  const int j16 = lane & 15, q16 = (lane >> 4) & 1;
  const int vrow = 4 * h + (j16 >> 2);                      // + 16 sg + 8 (second read)
  const int vodd = vrow & 1;                                // rows of odd number hold their pieces swapped by 4
  const int vcolb = (16 * q16 + 4 * (j16 & 3)) * 2;          // byte inside the 64-byte group of 32 t
  // byte offset of (vrow, 32 t + ...) for even and for odd t: the swap moves tile t to place t ^ 1
  const int voff_e = vrow * (D * 2) + vcolb + 64 * vodd;
  const int voff_o = vrow * (D * 2) + vcolb - 64 * vodd;

  float m_run = -INFINITY, l_run = 0.f;
  f32x16p_t o[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[t][i] = 0.f;

  // Four stages in LDS.  The loop is software pipelined: iteration i holds the scores of step i (made in
  // iteration i - 1), issues the score products of step i + 1 next to the softmax arithmetic of step i so
  // that matrix and vector units of the wave work at the same time, then the second product of step i;
  // meanwhile the copies of steps i + 2 and i + 3 are under way.
  auto scores = [&](int stage) __attribute__((always_inline)) -> f32x16p_t {
    f32x16p_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const bf16x8_t ak =
          as_bf16x8(*reinterpret_cast<const uint4*>(&kt0[stage * KT_BYTES + ((2 * s + h) * 32 + col) * 16]));
      acc = mfma32p(ak, bqh[s], acc);
      acc = mfma32p(ak, bql[s], acc);
    }
    return acc;
  };
  StepSrc q0 = {}, q1 = {}, q2 = {};  // steps i, i + 1, i + 2
  int s0 = locate(sb, q0), s1 = se, s2 = se;
  if (s0 < se) {
    issue_loads(q0, 0);
    q1 = q0;
    s1 = advance(q1);
    if (s1 < se) {
      issue_loads(q1, 1);
      q2 = q1;
      s2 = advance(q2);
      if (s2 < se) issue_loads(q2, 2);
    }
  }
  f32x16p_t sacc;
#pragma unroll
  for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
  if (s0 < se) {
    if (s2 < se)
      wait_copies_but<4 * NCP>();
    else if (s1 < se)
      wait_copies_but<2 * NCP>();
    else
      wait_copies_but<0>();
    __builtin_amdgcn_s_barrier();  // step s0 is staged for everyone
    sacc = scores(0);
  }
  int buf = 0;
  while (s0 < se) {
    const int rows_valid = q0.rows_valid;
    const int t0 = q0.t0;
    const bool is_mem = q0.is_mem;
    // ---- (a) the keys of step i + 1 have landed (the copies of step i + 2 may be on their way) -----
    if (s2 < se)
      wait_copies_but<2 * NCP>();
    else
      wait_copies_but<0>();
    // (b) step i + 1 is staged for everyone; everyone is done with the stage of step i - 1 (its LDS reads
    // went into matrix products that were issued before this point).  A bare barrier: the fences of
    // __syncthreads would wait for the copies that are meant to stay in flight.
    __builtin_amdgcn_s_barrier();

    // ---- (c) request step i + 3 into the stage that step i - 1 used ---------------------------------
    StepSrc q3 = q2;
    int s3 = se;
    if (s2 < se) {
      s3 = advance(q3);
      if (s3 < se) issue_loads(q3, (buf + 3) & 3);
    }

    // ---- (d) scores of step i: mask, running maximum ------------------------------------------------
    float sc[16];
    float mx = -INFINITY;
    if (is_mem && rows_valid == 32) {  // block-uniform: a whole step of document rows, nothing to mask
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        sc[i] = sacc[i];
        mx = fmaxf(mx, sc[i]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int krow = (i & 3) + 8 * (i >> 2) + 4 * h;
        const float v = sacc[i];
        const bool live = is_mem ? true : (t0 + krow < nvis_col);
        sc[i] = (krow < rows_valid && live) ? v : -INFINITY;
        mx = fmaxf(mx, sc[i]);
      }
    }
    mx = both_halves_max(mx);
    if (mx > m_run) {  // per column; the accumulators of a lane all belong to its column
      const float alpha = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - mx);
      m_run = mx;
      l_run *= alpha;
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[t][i] *= alpha;
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;

    // ---- (e) score products of step i + 1 (after the last step: of a stage nobody waits for, unused)
    // next to the weights of step i ------------------------------------------------------------------
    const f32x16p_t snext = scores((buf + 1) & 3);
    uint32_t pwh[8], pwl[8];
    float psum = 0.f;
#pragma unroll
    for (int i2 = 0; i2 < 8; ++i2) {
      const float p0 = __builtin_amdgcn_exp2f(sc[2 * i2] - m_use);
      const float p1 = __builtin_amdgcn_exp2f(sc[2 * i2 + 1] - m_use);
      psum += p0 + p1;
      split_pack_bf16(p0, p1, pwh[i2], pwl[i2]);
    }
    l_run += psum;

    // ---- (f) second product: O^T[dd][slot] += V^T[dd][key] P^T[key][slot] ---------------------------
    // contraction slot j of slice sg and half h is key 16 sg + (j % 4) + 8 (j / 4) + 4 h: the lane's own
    // score registers 8 sg .. 8 sg + 7
#pragma unroll
    for (int sg = 0; sg < 2; ++sg) {
      const bf16x8_t pbh = as_bf16x8(make_uint4(pwh[4 * sg], pwh[4 * sg + 1], pwh[4 * sg + 2], pwh[4 * sg + 3]));
      const bf16x8_t pbl = as_bf16x8(make_uint4(pwl[4 * sg], pwl[4 * sg + 1], pwl[4 * sg + 2], pwl[4 * sg + 3]));
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const unsigned char* vp = vt0 + buf * VT_BYTES + ((t & 1) ? voff_o : voff_e) + 16 * sg * (D * 2) + 64 * t;
        const s16x4_t v03 = lds_read_tr16(vp);
        const s16x4_t v8b = lds_read_tr16(vp + 8 * (D * 2));
        const bf16x8_t av = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(v03, v8b, 0, 1, 2, 3, 4, 5, 6, 7));
        o[t] = mfma32p(av, pbh, o[t]);
        o[t] = mfma32p(av, pbl, o[t]);
      }
    }
    sacc = snext;
    s0 = s1; q0 = q1;
    s1 = s2; q1 = q2;
    s2 = s3; q2 = q3;
    buf = (buf + 1) & 3;
  }

  // ---- partial results of this split ---------------------------------------------------------------
  const float l_tot = both_halves_sum(l_run);
  if (tok_ok && a.out != nullptr) {
    // the only split of its (token, head): normalise and write the result itself, with the merge
    // kernel's arithmetic for one partial
    const long long qh = ((long long)b * a.M + m_tok) * a.Hq + g * r + hh;
    const float inv_on = l_tot > 0.f ? 1.f : 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = inv_on != 0.f ? o[t][4 * i4 + e] / l_tot : 0.f;
        *reinterpret_cast<uint2*>(&a.out[qh * D + 32 * t + 8 * i4 + 4 * h]) =
            make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
      }
    if (h == 0 && a.lse != nullptr)
      a.lse[qh] = (l_tot > 0.f) ? (m_run + log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
  } else if (tok_ok) {
    const long long ph = (((long long)b * a.M + m_tok) * a.Hq + g * r + hh) * a.ph_splits + a.split0 + sp;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int dd = 32 * t + (i & 3) + 8 * (i >> 2) + 4 * h;
        a.part_o[ph * D + dd] = o[t][i];
      }
    if (h == 0) a.part_ml[ph] = make_float2(m_run, l_tot);
  }
}

int launch_attend_prefill_partial(const Dims& dm, const AttendPlan& pl, const AttendArgs& a,
                                  const RopeTheta& th, int B, hipStream_t st, bool dominant) {
  if (a.Krot == nullptr) return MSA_ERR_INVALID_ARG;  // the plan always reserves the rotated keys
  {
    dim3 rgrid(a.steps_total, dm.Hkv, B);
    if (dm.d == 128)
      hipLaunchKernelGGL(rotate_steps_kernel<128>, rgrid, dim3(256), 0, st, a, th, const_cast<uint16_t*>(a.Krot));
    else
      hipLaunchKernelGGL(rotate_steps_kernel<64>, rgrid, dim3(256), 0, st, a, th, const_cast<uint16_t*>(a.Krot));
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  }
  dim3 grid(pl.n_splits, dm.Hkv, B * pl.n_ttiles), block(256);
  if (dominant) profile_mark(dm, false, st);
  if (dm.d == 128)
    hipLaunchKernelGGL(attend_prefill_kernel<128>, grid, block, 0, st, a, th, pl.tpw, pl.n_ttiles);
  else
    hipLaunchKernelGGL(attend_prefill_kernel<64>, grid, block, 0, st, a, th, pl.tpw, pl.n_ttiles);
  if (dominant) profile_mark(dm, true, st);
  return hipGetLastError() == hipSuccess ? MSA_OK : MSA_ERR_HIP;
}

}  // namespace msa
