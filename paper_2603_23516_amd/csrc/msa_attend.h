// Types shared by the attention kernels (decode: msa_attend.hip, shared-selection prefill:
// msa_attend_prefill.hip).
#pragma once
#include "msa_device.h"
#include "msa_host.h"

namespace msa {

constexpr int kAttWaves = 4;
constexpr int kMaxHalf = 64;  // d/2 <= 64

struct RopeTheta {
  double th[kMaxHalf];   // theta_u = base^(-2u/d), computed on the host in double
  float2 e1[kMaxHalf];   // (cos, sin)(theta_u), rounded from double on the host
  float2 e16[kMaxHalf];  // (cos, sin)(16 theta_u)
};

struct AttendArgs {
  const uint16_t* q;     // [BM][Hq][D]
  const uint16_t* K;     // [N][Hkv][G][D]
  const uint16_t* V;
  const int32_t* idx;    // [BM or B][Hkv or 1][k] (see idx_rows_per_b, idx_sel)
  const uint16_t* Kloc;  // [B][Hkv][Lloc][D]
  const uint16_t* Vloc;
  const int32_t* q_pos;  // [BM]
  const int32_t* lens;   // [N] document lengths (rows of a bank slot that exist), or null = G everywhere
  uint16_t* out;         // tiled kernel with a single split: the final output and (or null) log-sum-exp,
  float* lse;            // written directly instead of partials; null = partials
  const uint16_t* Krot;  // tiled kernel: keys of every step, rotated once, [B][Hkv][steps_total][D/8][32][8]; or null
  float* part_o;         // [BM][Hq][n_splits][D]   unnormalised partial outputs
  float2* part_ml;       // [BM][Hq][n_splits]      (running max in log2 units, sum)
  int M, Hq, Hkv, r, G, k, Lloc, pos0, N;
  int gshift;            // log2(G) when G < 32 (MODE 2)
  int idx_sel;           // selections per idx row: Hkv (one per KV group) or 1 (shared by all heads)
  int idx_rows_per_b;    // idx rows per batch row: M (one per query token) or 1 (shared by the M tokens)
  int steps_mem, steps_total, steps_per_split, n_splits;
  int ph_splits, split0;  // partial slots per (query, head) in the workspace, and this launch's first slot
  float qscale;          // log2(e) / sqrt(d)
  unsigned long long* tickets;  // decode kernel: arrival counters [BM][Hkv], or null = a separate merge launch
  unsigned long long nonce;     // this launch's tag of the counters (48 bits, non-zero)
  uint16_t* final_out;          // with tickets: the merged output [BM][Hq][D] and (or null) log-sum-exp
  float* final_lse;
};

// Shared-selection prefill: unnormalised partials of every (token, head, split) in the layout the
// decode path writes, merged by the same attend_merge_kernel.
int launch_attend_prefill_partial(const Dims& dm, const AttendPlan& pl, const AttendArgs& a,
                                  const RopeTheta& th, int B, hipStream_t st, bool dominant);

}  // namespace msa
