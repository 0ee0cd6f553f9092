// msa_sparse_attend: context assembly (paper, Eq. 3) with document-wise RoPE (Section 3.2.2) and
// attention (Eq. 4) over [selected documents ; local context], as a split-K flash-decode with a
// log-sum-exp merge.  HBM-bound: every selected K and V row is read once per (query, KV head) and
// shared by the r query heads of the group.
//
// Key sequence of one (query, KV head): k documents x G tokens, then Lloc local tokens, cut into
// STEPS of 32 keys (G % 32 == 0, so a step never straddles two documents).  A block owns a
// contiguous range of steps, each of its 4 waves a contiguous sub-range, so positions advance by 16
// from one 16-key sub-tile to the next and the rotation angles follow a two-multiply recurrence.
//
// Per sub-tile (S^T = K~ Q~^T on 16x16x32 bf16 MFMA):
//   A = rotated keys: lane (rr, n) loads 16-byte pieces of key row n (dims 32s + 8rr .. +8, s < d/32);
//       element u is paired with u + d/2, which the same lane holds in slice s + d/64.
//       Rotation in fp32 by the lane's running (cos, sin)(p * theta_u), then rounded to bf16.
//   B = the r rotated, pre-scaled queries (log2(e)/sqrt(d) folded in) as bf16 (hi, lo) pairs in
//       columns 2h, 2h+1; the two halves of a score are summed with one DPP exchange.
//   D: lane (rr, n) holds column n (head slot) for keys 4rr .. 4rr+3.
// Online softmax per head slot (exp2 domain), running max shared across the four row groups by
// two shuffles; the weights go back as a bf16 (hi, lo) pair in the same two columns, which is exactly
// the B-operand layout of the second product
//   O^T[dd][slot] += V^T[dd][key] P^T[key][slot]       (8 MFMAs per 32 keys at d = 128)
// whose A operand (V transposed) comes out of an LDS copy of the 32 value rows through transposing reads
// (ds_read_b64_tr_b16); the rows get there by asynchronous global -> LDS copies, two stages per wave.
// Every accumulator of a lane belongs to its own head slot, so the rescale needs no cross-lane data.
// A wave keeps the keys of the next two steps in flight (two register sets, two steps per trip of the loop)
// and the values of the next step (the stage the current step does not use).
//
// MODE selects how the memory bank is read (the local context is always rotated here):
//   0  raw keys, rotated in the gather with positions 0..G-1 (G % 32 == 0);
//   1  keys that already carry their positions (the pooled bank of Section 3.4.1, Stage 1), used as
//      stored, G % 32 == 0;
//   2  the same with short documents, G in {1, 2, 4, 8, 16}: a 32-key step spans 32/G selected
//      documents, so every lane looks up the document of each row it loads and a 32-bit mask
//      records which rows belong to a valid selection.
#include "msa_attend.h"

namespace msa {

template <int D, int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attend_partial_kernel(AttendArgs a, RopeTheta th) {
  constexpr int NS = D / 32;        // MFMA k-slices per key row
  constexpr int HALF = D / 2;
  constexpr int NU = (NS / 2) * 8;  // rotation pairs per lane
  constexpr int NCB = D / 16;       // output column blocks
  constexpr int VBYTES = 32 * D * 2;  // the 32 value rows of a step in LDS
  constexpr int OBYTES = 16 * D * 4;  // one wave's partial output in the merge
  constexpr int STAGE = (2 * VBYTES > OBYTES ? 2 * VBYTES : OBYTES);  // two value stages per wave

  __shared__ float2 base0[16][HALF];  // e^{i n theta_u}: positions 0..15
  __shared__ float2 step16[HALF];     // e^{i 16 theta_u}
  __shared__ float qrot[8][D];        // rotated, scaled queries of this group
  __shared__ __attribute__((aligned(16))) uint16_t stage[kAttWaves][STAGE / 2];
  __shared__ float wm[kAttWaves][16], wl[kAttWaves][16];
  __shared__ float2 estart[kAttWaves][HALF];  // e^{i p theta_u} at a wave's (re)start position
  // theta_u for the restarts inside the stream: read from LDS there, because a global load (which a
  // lane-indexed kernel argument is) could only be awaited together with every prefetch in flight
  __shared__ double theta_s[HALF];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int rr = lane >> 4;
  const int n = lane & 15;
  const int sp = blockIdx.x;
  const int g = blockIdx.y;
  const int bm = blockIdx.z;
  const int b = bm / a.M;
  const int qpos = a.q_pos[bm];
  int n_vis = qpos - a.pos0 + 1;  // visible local tokens
  n_vis = n_vis < 0 ? 0 : (n_vis > a.Lloc ? a.Lloc : n_vis);

  // ---- block prologue: rotation tables and rotated queries ------------------------------------
  // base0[n][u] = e^{i n theta_u}, n < 16, by repeated multiplication with the host's e^{i theta_u}
  // (at most 15 fp32 complex products: error ~1e-6, far below the bf16 rounding of the rotated keys)
  for (int e = tid; e < 4 * HALF; e += 256) {
    const int u = e % HALF, n4 = e / HALF;  // this thread fills positions 4*n4 .. 4*n4 + 3
    const float2 w = th.e1[u];
    const float2 w2 = cmul(w, w);
    const float2 w4 = cmul(w2, w2);
    float2 cur = make_float2(1.f, 0.f);
    for (int i = 0; i < n4; ++i) cur = cmul(cur, w4);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      base0[4 * n4 + i][u] = cur;
      cur = cmul(cur, w);
    }
  }
  if (tid < HALF) {
    step16[tid] = th.e16[tid];
    theta_s[tid] = th.th[tid];
  }
  for (int e = tid; e < a.r * HALF; e += 256) {
    const int hh = e / HALF, u = e % HALF;
    const uint16_t* qp = a.q + ((long long)bm * a.Hq + g * a.r + hh) * D;
    const float x1 = __uint_as_float((uint32_t)qp[u] << 16);
    const float x2 = __uint_as_float((uint32_t)qp[u + HALF] << 16);
    const float2 cs = cis_pos(qpos, th.th[u]);
    qrot[hh][u] = (x1 * cs.x - x2 * cs.y) * a.qscale;
    qrot[hh][u + HALF] = (x2 * cs.x + x1 * cs.y) * a.qscale;
  }
  __syncthreads();

  // B operand of the score product: column n = head slot (head n/2, hi or lo half)
  bf16x8_t bq[NS];
  {
    const int hh = n >> 1;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      uint32_t w[4];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        float x0 = 0.f, x1 = 0.f;
        if (hh < a.r) {
          x0 = qrot[hh][32 * s + 8 * rr + 2 * jj];
          x1 = qrot[hh][32 * s + 8 * rr + 2 * jj + 1];
        }
        float h0, l0, h1, l1;
        split_bf16(x0, h0, l0);
        split_bf16(x1, h1, l1);
        w[jj] = (n & 1) ? pack_bf16(l0, l1) : pack_bf16(h0, h1);
      }
      bq[s] = as_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
    }
  }

  float2 cs[NU];         // (cos, sin)((cur_p + n) * theta_u), u = 32s' + 8rr + j at index 8s' + j
  int cur_p = -1;        // position of key 0 of the sub-tile the state is valid for; -1 = invalid
  float m_run = -INFINITY, l_run = 0.f;
  f32x4_t o[NCB];
#pragma unroll
  for (int c = 0; c < NCB; ++c) o[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  constexpr int NVL = 32 * D * 2 / 1024;  // wave-wide 16-byte copies covering 32 value rows
  constexpr int PPR = D / 8;              // 16-byte pieces per row

  // selected documents of this (query, KV head): lane j holds idx[j] (k <= 64)
  const long long idx_row = (a.idx_rows_per_b == 1) ? b : bm;
  const int my_idx =
      (lane < a.k) ? a.idx[(idx_row * a.idx_sel + (a.idx_sel == 1 ? 0 : g)) * a.k + lane] : -1;
  // ... and the number of rows that document holds
  int my_len = a.G;
  if (a.lens != nullptr && my_idx >= 0 && my_idx < a.N) {
    const int l = a.lens[my_idx];
    my_len = l < 1 ? 1 : (l > a.G ? a.G : l);
  }

  // ---- this wave's steps -----------------------------------------------------------------------
  // With document lengths (MODE 0, 1) the steps are numbered over what is really there -- slot j
  // contributes ceil(len_j / 32) steps, none for a pad, then come the steps of the visible local rows
  // -- so that the split into blocks and waves stays even when documents are short.  pre = inclusive
  // prefix sum of the slots' step counts over the lanes.  Otherwise the host's numbering over whole
  // slots is used as it is.
  const bool compact = MODE != 2 && a.lens != nullptr;  // wave-uniform
  int pre = 0;
  int mem_steps = a.steps_mem, steps_total = a.steps_total, steps_per_split = a.steps_per_split;
  if (compact) {
    pre = (my_idx >= 0 && my_idx < a.N) ? (my_len + 31) >> 5 : 0;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(pre, off, 64);
      if (lane >= off) pre += t;
    }
    mem_steps = __builtin_amdgcn_readlane(pre, 63);
    steps_total = mem_steps + ((n_vis + 31) >> 5);
    steps_per_split = (steps_total + a.n_splits - 1) / a.n_splits;
  }
  const int sb = sp * steps_per_split;
  int se = sb + steps_per_split;
  if (se > steps_total) se = steps_total;
  if (se < sb) se = sb;  // nothing left for this block
  int spw = (se - sb + kAttWaves - 1) / kAttWaves;
  spw = (spw + 1) & ~1;  // the loop takes two steps per trip
  const int wb = sb + wave * spw;
  int we = wb + spw;
  if (we > se) we = se;

  // Where a step's 32 keys live (wave-uniform).  Returns false for a step with nothing to attend.
  struct StepSrc {
    const uint16_t* Kb;
    const uint16_t* Vb;
    int rows_valid, p_first;
    int st;         // step number
    unsigned mask;  // MODE 2, memory steps: bit i set = key row i belongs to a valid selection
    bool is_mem;    // a step over selected documents (else local context)
  };
  // MODE 2: bank element offset of key row `row` (0..31) of memory step st, and whether its document
  // is a valid selection.  Rows of pads, of ids outside the bank and past the k-th document point at
  // document 0 (always present) so that their loads stay inside the bank; their scores are masked.
  auto gather_row = [&](int st, int row, long long& off) -> bool {
    const int tok = st * 32 + row;
    const int slot = tok >> a.gshift;
    const int pin = tok & (a.G - 1);
    const int doc = __shfl(my_idx, slot < a.k ? slot : 0, 64);
    const int len = __shfl(my_len, slot < a.k ? slot : 0, 64);
    const bool ok = slot < a.k && doc >= 0 && doc < a.N && pin < len;
    off = (((long long)(ok ? doc : 0) * a.Hkv + g) * a.G + (ok ? pin : 0)) * D;
    return ok;
  };
  auto locate = [&](int st, StepSrc& ss) -> bool {
    ss.st = st;
    ss.mask = 0xffffffffu;
    ss.is_mem = st < mem_steps;
    if (MODE == 2 && st < mem_steps) {
      long long off;
      const bool ok = gather_row(st, lane & 31, off);
      ss.mask = (unsigned)__ballot(ok);  // lanes 0..31 cover the 32 rows
      ss.Kb = a.K;
      ss.Vb = a.V;
      ss.rows_valid = 32;
      ss.p_first = 0;
      return ss.mask != 0u;
    }
    if (st < mem_steps) {
      int slot, pin;
      if (compact) {
        // the slot whose steps contain st: the first lane whose inclusive prefix exceeds st (pads, ids
        // outside the bank and rows past a document's end own no steps, so they are never reached)
        slot = __popcll(__ballot(pre <= st));
        pin = (st - (slot > 0 ? __builtin_amdgcn_readlane(pre, slot - 1) : 0)) * 32;
      } else {
        const int tok = st * 32;
        slot = tok / a.G;
        pin = tok - slot * a.G;
      }
      const int doc = __builtin_amdgcn_readlane(my_idx, slot);
      if (doc < 0 || doc >= a.N) return false;  // -1 pads, and ids outside the bank, are skipped
      const int len = __builtin_amdgcn_readlane(my_len, slot);
      if (pin >= len) return false;             // past the document's last token
      const long long off = (((long long)doc * a.Hkv + g) * a.G + pin) * D;
      ss.Kb = a.K + off;
      ss.Vb = a.V + off;
      ss.rows_valid = len - pin < 32 ? len - pin : 32;
      ss.p_first = pin;
      return true;
    }
    const int t0 = (st - mem_steps) * 32;
    if (t0 >= n_vis) return false;
    const long long off = (((long long)b * a.Hkv + g) * a.Lloc + t0) * D;
    ss.Kb = a.Kloc + off;
    ss.Vb = a.Vloc + off;
    ss.rows_valid = n_vis - t0 < 32 ? n_vis - t0 : 32;
    ss.p_first = a.pos0 + t0;
    return true;
  };
  auto next_valid = [&](int st, StepSrc& ss) -> int {  // first step >= st with keys, or we
    while (st < we && !locate(st, ss)) ++st;
    return st;
  };
  // Requests of one step.  The step's base addresses are wave-uniform (scalar registers) and every lane adds a
  // 32-bit byte offset, worked out here from an opaque copy of the lane number every time (a few instructions,
  // whereas offsets kept across the loop would cost registers the loop does not have).  One form for full and
  // ragged steps -- a row past the step's last valid row re-reads that row, its score is masked -- so no branch
  // surrounds a request: with the same requests on every path the waits in the loop can name exactly what they
  // need and leave the rest in flight.
  typedef const __attribute__((address_space(1))) char* gptr_t;  // global memory, not generic
  typedef const __attribute__((address_space(1))) u32x4_t* gvec_t;
  // readfirstlane returns a signed int: both halves go through unsigned before widening, or a
  // low word with bit 31 set would sign-extend into the high word
  auto uni64 = [](unsigned long long v) {
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)v);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v >> 32));
    return ((unsigned long long)hi << 32) | (unsigned long long)lo;
  };
  // Keys: 16-byte pieces into registers, lane (rr, n) takes rows n and 16 + n.
  auto issue_keys = [&](const StepSrc& ss, uint4 (&kr)[2][NS]) {
    // Plain loads: a wave-wide key load takes 64 bytes of each of 16 rows, so every 128-byte line is touched by two
    // loads; with the streaming hint the line is not kept for the second one (measured: 112 us per call of the 50M-
    // token decode with the hint on these loads, 101 us without; the value copies below, whole lines, keep it).
    auto ld = [](gvec_t p) { const u32x4_t v = *p; return make_uint4(v.x, v.y, v.z, v.w); };
    gptr_t kb = (gptr_t)uni64((unsigned long long)ss.Kb);
    if (MODE == 2 && ss.is_mem) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        long long off;
        gather_row(ss.st, 16 * h + n, off);
#pragma unroll
        for (int s = 0; s < NS; ++s) kr[h][s] = ld((gvec_t)(kb + (off * 2 + 16 * rr + s * 64)));
      }
    } else {
      const int last = ss.rows_valid - 1;
      int ln = lane;
      asm volatile("" : "+v"(ln));
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        int row = 16 * h + (ln & 15);
        row = row < last ? row : last;
#pragma unroll
        for (int s = 0; s < NS; ++s)
          kr[h][s] = ld((gvec_t)(kb + (unsigned)(row * D * 2 + 16 * (ln >> 4) + s * 64)));
      }
    }
  };
  // Values: copied global -> LDS without passing through registers, into one of the wave's two stages.  The 16-byte
  // slot f = 16 row + c of a stage holds piece c ^ 2 (row & 3) of value row `row`: the transposing reads of the
  // second product (four rows x 32 bytes per 16 lanes) then touch every bank once.  Rows that are masked (past the
  // step's last row, or not a valid selection) hold some existing row: their weights are exactly zero.
  auto issue_values = [&](const StepSrc& ss, int into) {
    int ln = lane, wv = wave;
    asm volatile("" : "+v"(ln), "+v"(wv));
    // the stage's LDS address, in a scalar register (worked out here: see above)
    const uint32_t dst = lds_addr_of(&stage[0][0]) + (uint32_t)__builtin_amdgcn_readfirstlane(wv) * STAGE + into * VBYTES;
    if (MODE == 2 && ss.is_mem) {
#pragma unroll
      for (int i = 0; i < NVL; ++i) {
        const int f = i * 64 + ln;
        const int row = f / PPR;
        const int piece = (f % PPR) ^ (2 * (row & 3));
        long long off;
        gather_row(ss.st, row, off);
        copy16_to_lds_async_stream64(reinterpret_cast<const char*>(a.V) + (off * 2 + piece * 16), dst + i * 1024);
      }
    } else {
      const void* vb = reinterpret_cast<const void*>(uni64((unsigned long long)ss.Vb));
      const int last = ss.rows_valid - 1;
      // slot f = 64 i + lane: row 64 i / PPR + lane / PPR, and the piece (with its swizzle) is the same for every i
      constexpr int RPC = 64 / PPR;  // rows per copy (a multiple of 4)
      const int lrow = (ln & 63) / PPR;
      const int poff = (((ln & 63) % PPR) ^ (2 * (lrow & 3))) * 16;
#pragma unroll
      for (int i = 0; i < NVL; ++i) {
        const int row = i * RPC + lrow;
        const int src_row = row < last ? row : last;
        copy16_to_lds_async_stream(vb, (uint32_t)(src_row * D * 2 + poff), dst + i * 1024);
      }
    }
  };
  // LDS byte of this lane's transposing reads inside a stage: rows 4 rr + (n >> 2) (first read) and 16 more
  // (second read), elements 16 c + 4 (n & 3) .. + 3; column block c is applied with an exclusive or of 32 c
  // (the swizzle above moves piece pair c of row `row` to pair c ^ (row & 3)).
  const int vt_lane = (4 * rr + (n >> 2)) * (D * 2) + (n >> 2) * 32 + ((n >> 1) & 1) * 16 + (n & 1) * 8;

  // The loop keeps three steps in view: s0 is worked on, the keys of s1 are in flight (requested one and a half
  // steps before their use), the values of s1 are requested at the top of s0's turn into the stage that s0 does
  // not use, the keys of s2 in the middle of it into the registers that s0's keys leave.  When there is no further
  // step the requests repeat the last one (results unused), so the number of requests in flight never depends on
  // the path.  Two turns per trip of the loop, so that the two sets of key registers have fixed names.
  StepSrc s0, s1, s2;
  int st0 = next_valid(wb, s0);
  int st1 = we, st2 = we;
  uint4 kA[2][NS], kB[2][NS];
  if (st0 < we) {
    s1 = s0;
    st1 = next_valid(st0 + 1, s1);
    if (st1 >= we) s1 = s0;
    s2 = s1;
    if (st1 < we) st2 = next_valid(st1 + 1, s2);
    if (st2 >= we) s2 = s1;
    issue_keys(s0, kA);
    issue_values(s0, 0);
    issue_keys(s1, kB);
  }

  auto turn = [&](uint4 (&kraw)[2][NS], const int cur_stage) __attribute__((always_inline)) {
    const bool live = st0 < we;  // wave-uniform; false: the spare second turn of the last trip
    const int rows_valid = live ? s0.rows_valid : 0;
    const int p_first = s0.p_first;
    const unsigned cur_mask = s0.mask;
    const bool cur_is_mem = s0.is_mem;
    // The keys of this step are awaited HERE, ahead of the value request below: the compiler's wait names the
    // requests it knows (it leaves the next step's keys, the youngest, in flight); the copies are invisible to it,
    // and issued first they would be the youngest requests and the next step's keys would be awaited too.
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int s = 0; s < NS; ++s) asm volatile("" : "+v"(kraw[h][s].x), "+v"(kraw[h][s].y), "+v"(kraw[h][s].z), "+v"(kraw[h][s].w));
    issue_values(s1, cur_stage ^ 1);

    // ---- rotation state for this step ----------------------------------------------------------
    const bool rot = (MODE == 0) || !cur_is_mem;  // wave-uniform: stored-as-rotated bank keys skip it
    if (live && rot && cur_p != p_first) {
      // The LDS addresses of this rare block are derived here from an opaque copy of the lane number: computed
      // ahead of the loop they would occupy registers across the whole stream, and the spills that follow are
      // reloaded through the vector memory counter, i.e. only together with every prefetch in flight.
      int ln = lane, wv = wave;
      asm volatile("" : "+v"(ln), "+v"(wv));
      const int n_ = ln & 15, rr_ = ln >> 4;
      if (p_first == 0) {
#pragma unroll
        for (int s2i = 0; s2i < NS / 2; ++s2i)
#pragma unroll
          for (int j = 0; j < 8; ++j) cs[8 * s2i + j] = base0[n_][32 * s2i + 8 * rr_ + j];
      } else {
        // wave-cooperative: lane u evaluates e^{i p theta_u} once, everyone combines it with e^{i n theta_u}
        if (ln < HALF) estart[wv][ln] = cis_pos(p_first, theta_s[ln]);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int s2i = 0; s2i < NS / 2; ++s2i)
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int u = 32 * s2i + 8 * rr_ + j;
            cs[8 * s2i + j] = cmul(estart[wv][u], base0[n_][u]);
          }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
      cur_p = p_first;
    }

    // ---- scores of the two 16-key sub-tiles ---------------------------------------------------
    float sc[2][4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t y1[NS / 2][4], y2[NS / 2][4];
#pragma unroll
      for (int s2i = 0; s2i < NS / 2; ++s2i) {
        const uint4 a1 = kraw[h][s2i], a2 = kraw[h][s2i + NS / 2];
        const uint32_t w1[4] = {a1.x, a1.y, a1.z, a1.w};
        const uint32_t w2[4] = {a2.x, a2.y, a2.z, a2.w};
        if (rot) {
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const float2 c0 = cs[8 * s2i + 2 * jj], c1 = cs[8 * s2i + 2 * jj + 1];
            const float p0 = bf16_lo(w1[jj]), p1 = bf16_hi(w1[jj]);
            const float q0 = bf16_lo(w2[jj]), q1 = bf16_hi(w2[jj]);
            y1[s2i][jj] = pack_bf16(p0 * c0.x - q0 * c0.y, p1 * c1.x - q1 * c1.y);
            y2[s2i][jj] = pack_bf16(q0 * c0.x + p0 * c0.y, q1 * c1.x + p1 * c1.y);
          }
        } else {
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            y1[s2i][jj] = w1[jj];
            y2[s2i][jj] = w2[jj];
          }
        }
      }
      f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s2i = 0; s2i < NS / 2; ++s2i) {
        acc = mfma16(as_bf16x8(make_uint4(y1[s2i][0], y1[s2i][1], y1[s2i][2], y1[s2i][3])), bq[s2i], acc);
        acc = mfma16(as_bf16x8(make_uint4(y2[s2i][0], y2[s2i][1], y2[s2i][2], y2[s2i][3])),
                     bq[s2i + NS / 2], acc);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float v = acc[i] + dpp_f<kDppXor1>(acc[i]);  // hi + lo column
        const int row = 16 * h + 4 * rr + i;
        bool live = row < rows_valid;
        if (MODE == 2) live = live && ((cur_mask >> row) & 1u);
        sc[h][i] = live ? v : -INFINITY;
      }
      // advance the rotation state by 16 positions
      if (rot) {
#pragma unroll
        for (int s2i = 0; s2i < NS / 2; ++s2i)
#pragma unroll
          for (int j = 0; j < 8; ++j) cs[8 * s2i + j] = cmul(cs[8 * s2i + j], step16[32 * s2i + 8 * rr + j]);
      }
    }
    if (rot) cur_p += 32;
    issue_keys(s2, kraw);  // the keys of the step after next (this step's are in the scores now)

    // ---- online softmax (exp2 domain) ---------------------------------------------------------
    float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                     fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The accumulator is rescaled only in the steps where some head's running maximum grows
    // (wave-uniform branch); once the maxima have settled most steps skip it.
    const bool bump = mx > m_run;
    if (__any(bump)) {
      const float m_new = bump ? mx : m_run;
      const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int c = 0; c < NCB; ++c) {
        o[c][0] *= alpha;
        o[c][1] *= alpha;
        o[c][2] *= alpha;
        o[c][3] *= alpha;
      }
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
    float psum = 0.f;
    uint32_t pw[4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float pv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = __builtin_amdgcn_exp2f(sc[h][i] - m_use);
        psum += p;
        float hi, lo;
        split_bf16(p, hi, lo);
        pv[i] = (n & 1) ? lo : hi;
      }
      pw[2 * h] = pack_bf16(pv[0], pv[1]);
      pw[2 * h + 1] = pack_bf16(pv[2], pv[3]);
    }
    l_run += psum;
    const bf16x8_t pb = as_bf16x8(make_uint4(pw[0], pw[1], pw[2], pw[3]));

    // ---- second product: V^T straight out of the stage through transposing reads ------------------
    // This step's values were requested in the previous turn, ahead of the keys that the top of this turn left in
    // flight, so they have landed; the wait here states the condition itself (everything but the requests issued
    // since: keys of the next two steps, the next values) and costs nothing when it already holds.
    wait_copies_but<NVL + 4 * NS>();
    {
      const unsigned char* vt = reinterpret_cast<const unsigned char*>(&stage[wave][0]) + cur_stage * VBYTES;
      // (an opaque copy: the eight addresses of a stage, known ahead of the loop, would be kept in registers
      // across it, which the loop does not have)
      int vl = vt_lane;
      asm volatile("" : "+v"(vl));
#pragma unroll
      for (int c = 0; c < NCB; ++c) {
        const unsigned char* vp = vt + (vl ^ (32 * c));
        const s16x4_t v0 = lds_read_tr16(vp);                   // keys 4 rr .. + 3
        const s16x4_t v1 = lds_read_tr16(vp + 16 * (D * 2));    // keys 16 + 4 rr .. + 3
        const bf16x8_t av = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
        o[c] = mfma16(av, pb, o[c]);
      }
    }
    // ---- next turn: s1 becomes the step at hand, a new s2 is located --------------------------------
    st0 = st1;
    s0 = s1;
    st1 = st2;
    s1 = s2;
    if (st2 < we) {
      StepSrc s3 = s2;
      st2 = next_valid(st2 + 1, s3);
      if (st2 < we) s2 = s3;
    }
  };
  // Always two turns per trip: an exit between them would give the loop a second way back to its head (the exit
  // is folded into the latch), on which the keys requested by the first turn are the youngest requests, and the
  // waits of the first turn would be placed for that path, i.e. drain everything.  With an odd number of steps the
  // second turn of the last trip works on a repeat of the last step with every row masked.
  if (st0 < we) {
    do {
      turn(kA, 0);
      turn(kB, 1);
    } while (st0 < we);
  }
  wait_copies_but<0>();  // the repeated requests of the last turns still write into the stages

  // ---- merge the four waves ----------------------------------------------------------------------
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  __syncthreads();  // every wave is done with its value staging area
  {
    float* wo = reinterpret_cast<float*>(&stage[wave][0]);  // [16 slots][D]
#pragma unroll
    for (int c = 0; c < NCB; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) wo[n * D + 16 * c + 4 * rr + i] = o[c][i];
    if (rr == 0) {
      wm[wave][n] = m_run;
      wl[wave][n] = l_run;
    }
  }
  __syncthreads();
  for (int e = tid; e < a.r * D; e += 256) {
    const int hh = e / D, dd = e % D;
    const int s0 = 2 * hh;
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < kAttWaves; ++w) mx = fmaxf(mx, wm[w][s0]);
    float osum = 0.f, lsum = 0.f;
    if (mx != -INFINITY) {
#pragma unroll
      for (int w = 0; w < kAttWaves; ++w) {
        const float mw = wm[w][s0];
        const float f = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mx);
        const float* wo = reinterpret_cast<const float*>(&stage[w][0]);
        osum += f * (wo[s0 * D + dd] + wo[(s0 + 1) * D + dd]);
        lsum += f * wl[w][s0];
      }
    }
    const long long ph = ((long long)bm * a.Hq + g * a.r + hh) * a.ph_splits + a.split0 + sp;
    // device-scope stores: the merging workgroup may run on another XCD
    store_dev(&a.part_o[ph * D + dd], osum);
    if (dd == 0) {
      const float2 mlv = make_float2(mx, lsum);
      store_dev(reinterpret_cast<unsigned long long*>(a.part_ml + ph), __builtin_bit_cast(unsigned long long, mlv));
    }
  }
  if (a.tickets == nullptr) return;  // a separate launch merges the splits

  // ---- the workgroup that arrives last at this (query, KV head) merges its splits -------------------
  // Every workgroup of the launch gets here (one without keys wrote empty partials above).  A thread's partial
  // stores are complete before the workgroup's arrival is counted, so whoever counts the last arrival can read
  // all partials with device-scope loads.
  __shared__ int last_s;
  wait_stores_done();
  __syncthreads();
  if (tid == 0) {
    unsigned long long* word = a.tickets + (long long)bm * a.Hkv + g;
    const uint32_t before = arrive_at(word, a.nonce);
    last_s = (before + 1u == (uint32_t)gridDim.x) ? 1 : 0;
  }
  __syncthreads();
  if (!last_s) return;
  // (m, l) of every (head, split), all loads independent; the staging area is free again (every wave passed the
  // barriers above after its last use)
  const int ns = a.ph_splits;
  float2* mls = reinterpret_cast<float2*>(&stage[0][0]);  // [r][ns]: (max, sum), then (weight, sum)
  for (int t = tid; t < a.r * ns; t += 256) {
    const int hh = t / ns, s = t - hh * ns;
    const long long qh = (long long)bm * a.Hq + g * a.r + hh;
    mls[t] = __builtin_bit_cast(float2, load_dev(reinterpret_cast<const unsigned long long*>(a.part_ml + qh * ns + s)));
  }
  __syncthreads();
  for (int hh = wave; hh < a.r; hh += kAttWaves) {  // one wave per head: maximum, weights, normaliser
    float mx = -INFINITY;
    for (int s = lane; s < ns; s += 64) mx = fmaxf(mx, mls[hh * ns + s].x);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float lsum = 0.f;
    for (int s = lane; s < ns; s += 64) {
      const float2 v = mls[hh * ns + s];
      const float f = (v.x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(v.x - mx);
      mls[hh * ns + s].x = f;
      lsum += f * v.y;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) lsum += __shfl_xor(lsum, off, 64);
    if (lane == 0) {
      wm[0][hh] = mx;
      wl[0][hh] = lsum;
    }
  }
  __syncthreads();
  for (int e = tid; e < a.r * (D / 2); e += 256) {  // a thread owns two adjacent output elements of one head
    const int hh = e / (D / 2), d2 = e % (D / 2);
    const long long qh = (long long)bm * a.Hq + g * a.r + hh;
    const unsigned long long* po = reinterpret_cast<const unsigned long long*>(a.part_o + qh * ns * D) + d2;
    const float2* w = mls + hh * ns;
    float o0 = 0.f, o1 = 0.f;
    int s = 0;
    for (; s + 8 <= ns; s += 8) {
      unsigned long long v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = load_dev(po + (long long)(s + u) * (D / 2));
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float2 x = __builtin_bit_cast(float2, v[u]);
        o0 += w[s + u].x * x.x;
        o1 += w[s + u].x * x.y;
      }
    }
    for (; s < ns; ++s) {
      const float2 x = __builtin_bit_cast(float2, load_dev(po + (long long)s * (D / 2)));
      o0 += w[s].x * x.x;
      o1 += w[s].x * x.y;
    }
    const float lsum = wl[0][hh], mx = wm[0][hh];
    const float r0 = (lsum > 0.f) ? o0 / lsum : 0.f, r1 = (lsum > 0.f) ? o1 / lsum : 0.f;
    reinterpret_cast<uint32_t*>(a.final_out + qh * D)[d2] = pack_bf16(r0, r1);
    if (a.final_lse != nullptr && d2 == 0)
      a.final_lse[qh] = (lsum > 0.f) ? (mx + log2f(lsum)) * 0.6931471805599453f : -INFINITY;
  }
  if (tid == 0) store_dev(a.tickets + (long long)bm * a.Hkv + g, 0ull);  // ready for a replay of this launch
}

// Log-sum-exp merge of the split partials of one (query, head); one thread per output element.
// The (max, sum) pairs are loaded split-parallel and reduced through LDS so that no thread walks a
// chain of dependent loads.
constexpr int kMaxAttSplits = 256;

template <int D>
__global__ __launch_bounds__(D) void attend_merge_kernel(const float* __restrict__ part_o,
                                                         const float2* __restrict__ part_ml,
                                                         uint16_t* __restrict__ out,
                                                         float* __restrict__ lse, int n_splits) {
  __shared__ float wgt[kMaxAttSplits];
  __shared__ float red[4];
  const long long qh = blockIdx.x;
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  constexpr int NW = D / 64;
  float2 ml[kMaxAttSplits / D];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < kMaxAttSplits / D; ++i) {
    const int s = tid + i * D;
    ml[i] = (s < n_splits) ? part_ml[qh * n_splits + s] : make_float2(-INFINITY, 0.f);
    mx = fmaxf(mx, ml[i].x);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  if ((tid & 63) == 0) red[wave] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) mx = fmaxf(mx, red[w]);
  __syncthreads();
  float lsum = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxAttSplits / D; ++i) {
    const int s = tid + i * D;
    const float f = (ml[i].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml[i].x - mx);
    if (s < n_splits) wgt[s] = f;
    lsum += f * ml[i].y;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) lsum += __shfl_xor(lsum, off, 64);
  if ((tid & 63) == 0) red[wave] = lsum;
  __syncthreads();
  lsum = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) lsum += red[w];
  float osum = 0.f;
  const float* po = part_o + qh * n_splits * D + tid;
  int s = 0;
  for (; s + 8 <= n_splits; s += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = po[(long long)(s + u) * D];
#pragma unroll
    for (int u = 0; u < 8; ++u) osum += wgt[s + u] * v[u];
  }
  for (; s < n_splits; ++s) osum += wgt[s] * po[(long long)s * D];
  const float res = (lsum > 0.f) ? osum / lsum : 0.f;
  const uint32_t pk = pack_bf16(res, 0.f);
  out[qh * D + tid] = (uint16_t)(pk & 0xffffu);
  if (lse != nullptr && tid == 0) {
    lse[qh] = (lsum > 0.f) ? (mx + log2f(lsum)) * 0.6931471805599453f : -INFINITY;
  }
}

AttendPlan plan_attend(const Dims& dm, int B, int M, int k, int Lloc, int bank_keys_rotated) {
  AttendPlan p;
  const int BM = B * M;
  p.steps_mem = (int)(((long long)k * dm.G + 31) / 32);
  p.steps_total = p.steps_mem + (Lloc + 31) / 32;
  // many query tokens sharing one selection: the tiled prefill kernel (raw keys, r a power of two)
  p.prefill = (dm.token_pool && M >= 8 && !bank_keys_rotated && dm.G % 32 == 0 &&
               (dm.r == 1 || dm.r == 2 || dm.r == 4 || dm.r == 8)) ? 1 : 0;
  p.tpw = p.prefill ? 32 / dm.r : 0;
  p.n_ttiles = p.prefill ? (M + 4 * p.tpw - 1) / (4 * p.tpw) : 0;
  const long long pairs = p.prefill ? (long long)B * p.n_ttiles * dm.Hkv : (long long)BM * dm.Hkv;
  // aim at <= 512 blocks: two 256-thread blocks are resident per CU (register-limited), so 512 is
  // one full wave of blocks on 256 CUs and nothing waits for a second round
  auto split = [](long long steps, long long prs, long long min_per, int max_splits, int* per_out) -> int {
    long long per = (steps * prs + 511) / 512;
    if (per < min_per) per = min_per;
    const long long per_cap = (steps + max_splits - 1) / max_splits;
    if (per < per_cap) per = per_cap;
    if (per > steps) per = steps;
    if (per < 1) per = 1;
    *per_out = (int)per;
    const long long n = (steps + per - 1) / per;
    return n < 1 ? 1 : (int)n;
  };
  // Many query tokens that the shared-selection kernel above does not take (their own selections, or a
  // bank whose keys are stored rotated): every token gathers its documents (decode kernel), but the local
  // context is the same rows for all tokens of a batch row, so it goes through the tiled kernel once per
  // token tile instead of once per token; the partials of both land in one slot range.
  p.split_local = (!p.prefill && M >= 16 && Lloc >= 32 &&
                   (dm.r == 1 || dm.r == 2 || dm.r == 4 || dm.r == 8)) ? 1 : 0;
  p.mem_splits = p.loc_splits = 0;
  p.mem_steps_per_split = p.loc_steps_per_split = 0;
  if (p.split_local) {
    p.tpw = 32 / dm.r;
    p.n_ttiles = (M + 4 * p.tpw - 1) / (4 * p.tpw);
    p.mem_splits = split(p.steps_mem, (long long)BM * dm.Hkv, kAttWaves, kMaxAttSplits / 2, &p.mem_steps_per_split);
    p.loc_splits = split((Lloc + 31) / 32, (long long)B * p.n_ttiles * dm.Hkv, 1, kMaxAttSplits / 2,
                         &p.loc_steps_per_split);
    p.n_splits = p.mem_splits + p.loc_splits;
    p.steps_per_split = p.mem_steps_per_split;
  } else {
    p.n_splits = split(p.steps_total, pairs, kAttWaves, kMaxAttSplits, &p.steps_per_split);
  }
  const size_t o_bytes = round_up256((size_t)BM * dm.Hq * p.n_splits * dm.d * sizeof(float));
  p.off_ml = o_bytes;
  p.ws_bytes = o_bytes + round_up256((size_t)BM * dm.Hq * p.n_splits * sizeof(float2));
  // decode kernel alone: its last-arriving workgroup per (query, KV head) merges the splits, no merge launch
  // (few splits only: with many, the separate merge launch, one workgroup per head, is the faster way to read them)
  p.fused_merge = (!p.prefill && !p.split_local && p.n_splits <= 16) ? 1 : 0;
  p.off_tickets = p.ws_bytes;
  if (p.fused_merge) p.ws_bytes += round_up256((size_t)BM * dm.Hkv * sizeof(unsigned long long));
  // the tiled kernel reads keys that were rotated once per (batch row, KV head): all steps of a shared
  // selection, or the local steps alone
  p.off_krot = 0;
  p.krot_steps = p.prefill ? p.steps_total : (p.split_local ? (Lloc + 31) / 32 : 0);
  if (p.krot_steps > 0) {
    p.off_krot = p.ws_bytes;
    p.ws_bytes += round_up256((size_t)B * dm.Hkv * p.krot_steps * 32 * dm.d * 2);
  }
  return p;
}

int launch_attend(const Dims& dm, const AttendPlan& pl, const void* q, int B, int M, const void* K,
                  const void* V, const int32_t* idx, int k, const void* Kloc, const void* Vloc,
                  int Lloc, int pos0, const int32_t* q_pos, void* out, float* lse, void* ws,
                  int bank_keys_rotated, hipStream_t st) {
  AttendArgs a;
  a.q = (const uint16_t*)q;
  a.K = (const uint16_t*)K;
  a.V = (const uint16_t*)V;
  a.idx = idx;
  a.Kloc = (const uint16_t*)Kloc;
  a.Vloc = (const uint16_t*)Vloc;
  a.q_pos = q_pos;
  a.lens = dm.lens;
  // a shared selection that is not split: the tiled kernel writes the result itself, no merge
  const bool direct = pl.prefill && pl.n_splits == 1;
  a.out = direct ? (uint16_t*)out : nullptr;
  a.lse = direct ? lse : nullptr;
  a.Krot = pl.krot_steps > 0 ? (const uint16_t*)((char*)ws + pl.off_krot) : nullptr;
  a.part_o = (float*)ws;
  a.part_ml = (float2*)((char*)ws + pl.off_ml);
  a.M = M;
  a.Hq = dm.Hq;
  a.Hkv = dm.Hkv;
  a.r = dm.r;
  a.G = dm.G;
  a.N = dm.N;
  a.idx_sel = dm.scope_all ? 1 : dm.Hkv;
  a.idx_rows_per_b = dm.token_pool ? 1 : M;
  a.gshift = 0;
  while ((1 << a.gshift) < dm.G && a.gshift < 5) ++a.gshift;
  a.k = k;
  a.Lloc = Lloc;
  a.pos0 = pos0;
  a.steps_mem = pl.steps_mem;
  a.steps_total = pl.steps_total;
  a.steps_per_split = pl.steps_per_split;
  a.n_splits = pl.n_splits;
  a.ph_splits = pl.n_splits;
  a.split0 = 0;
  a.qscale = (float)(1.4426950408889634 / sqrt((double)dm.d));
  a.tickets = pl.fused_merge ? (unsigned long long*)((char*)ws + pl.off_tickets) : nullptr;
  a.nonce = launch_nonce48();
  a.final_out = (uint16_t*)out;
  a.final_lse = lse;
  RopeTheta th;
  for (int u = 0; u < kMaxHalf; ++u) {
    th.th[u] = (u < dm.d / 2) ? pow((double)dm.base, -2.0 * (double)u / (double)dm.d) : 0.0;
    th.e1[u] = make_float2((float)cos(th.th[u]), (float)sin(th.th[u]));
    th.e16[u] = make_float2((float)cos(16.0 * th.th[u]), (float)sin(16.0 * th.th[u]));
  }
  const int BM = B * M;
  // how the bank is read (checked before anything is enqueued)
  const int mode = !bank_keys_rotated ? 0 : (dm.G % 32 == 0 ? 1 : 2);
  if (mode != 2 && dm.G % 32 != 0) return MSA_ERR_UNSUPPORTED;
  if (mode == 2 && ((1 << a.gshift) != dm.G || dm.G > 16)) return MSA_ERR_UNSUPPORTED;
  if (pl.split_local) {
    // local context through the tiled kernel (it never touches the bank or the selection: no memory steps) ...
    AttendArgs al = a;
    al.out = nullptr;
    al.steps_mem = 0;
    al.steps_total = (Lloc + 31) / 32;
    al.steps_per_split = pl.loc_steps_per_split;
    al.n_splits = pl.loc_splits;
    al.split0 = pl.mem_splits;
    AttendPlan pll = pl;
    pll.n_splits = pl.loc_splits;
    const int rc = launch_attend_prefill_partial(dm, pll, al, th, B, st, false);
    if (rc != MSA_OK) return rc;
    // ... and the selected documents through the decode kernel below, which sees no local context
    a.Lloc = 0;
    a.steps_total = pl.steps_mem;
    a.steps_per_split = pl.mem_steps_per_split;
    a.n_splits = pl.mem_splits;
  }
  if (pl.prefill) {
    const int rc = launch_attend_prefill_partial(dm, pl, a, th, B, st, true);
    if (rc != MSA_OK) return rc;
  } else {
    profile_mark(dm, false, st);
    dim3 grid(a.n_splits, dm.Hkv, BM), block(256);
#define MSA_LAUNCH_ATTEND(DD, MM) \
  hipLaunchKernelGGL((attend_partial_kernel<DD, MM>), grid, block, 0, st, a, th)
    if (dm.d == 128) {
      if (mode == 0) MSA_LAUNCH_ATTEND(128, 0);
      else if (mode == 1) MSA_LAUNCH_ATTEND(128, 1);
      else MSA_LAUNCH_ATTEND(128, 2);
    } else {
      if (mode == 0) MSA_LAUNCH_ATTEND(64, 0);
      else if (mode == 1) MSA_LAUNCH_ATTEND(64, 1);
      else MSA_LAUNCH_ATTEND(64, 2);
    }
#undef MSA_LAUNCH_ATTEND
    profile_mark(dm, true, st);
  }
  if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  if (direct || pl.fused_merge) return MSA_OK;
  if (dm.d == 128)
    hipLaunchKernelGGL(attend_merge_kernel<128>, dim3(BM * dm.Hq), dim3(128), 0, st,
                       (const float*)a.part_o, (const float2*)a.part_ml, (uint16_t*)out, lse,
                       pl.n_splits);
  else
    hipLaunchKernelGGL(attend_merge_kernel<64>, dim3(BM * dm.Hq), dim3(64), 0, st,
                       (const float*)a.part_o, (const float2*)a.part_ml, (uint16_t*)out, lse,
                       pl.n_splits);
  if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  return MSA_OK;
}

}  // namespace msa
