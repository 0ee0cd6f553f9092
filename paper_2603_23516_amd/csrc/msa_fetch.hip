// msa_fetch_selected: the tiered bank of the paper's inference engine (Section 3.4.2): the K/V of the
// whole bank stay in host DRAM, only the routing keys live in device memory, and the documents that
// routing selects are fetched on demand.  Here the fetch is ONE kernel that reads pinned, device-mapped
// host memory directly over the host link with the selection still on the device: no host round
// trip for the indices, no per-document copy calls, and it runs on whatever stream the caller gives it
// (so it can overlap the next layer's scoring).  Every selection entry (b, m', j) owns staging slot
// (b M' + m') k + j; the (slot, KV head) slab [G][d] is copied for the head(s) the entry selects for,
// and idx_stage receives the slot number (or -1), ready for msa_sparse_attend over the staging bank.
#include "msa_device.h"
#include "msa_host.h"

namespace msa {

struct FetchArgs {
  const uint4* K_host;   // device-visible address of the pinned host bank [N][Hkv][G][d]
  const uint4* V_host;
  const int32_t* idx;    // [B][M'][S][k]
  uint4* K_stage;        // [n_slots][Hkv][G][d]
  uint4* V_stage;
  int32_t* idx_stage;    // [B][M'][S][k]
  const int32_t* lens;   // [N] document lengths, or null
  int32_t* lens_stage;   // [n_slots] (with lens; then S == 1 or Hkv == 1: one document per slot)
  int N, Hkv, S, k, G;
  long long slab16;      // 16-byte words per (document, head) slab: G * d * 2 / 16
  int row16;             // 16-byte words per token row: d * 2 / 16
};

// One workgroup per (selection entry, head to copy, half = K or V).
__global__ __launch_bounds__(256) void fetch_selected_kernel(FetchArgs a) {
  const int hc = blockIdx.y;           // 0 .. heads_per_entry - 1
  const long long e = blockIdx.x;      // entry ((b M' + m') S + sl) k + j
  const int j = (int)(e % a.k);
  const long long row = e / a.k;       // (b M' + m') S + sl
  const int sl = (int)(row % a.S);
  const long long bm = row / a.S;
  const int doc = a.idx[e];
  const bool ok = doc >= 0 && doc < a.N;
  const long long slot = bm * a.k + j;
  if (hc == 0 && blockIdx.z == 0 && threadIdx.x == 0) a.idx_stage[e] = ok ? (int32_t)slot : -1;
  long long n16 = a.slab16;  // 16-byte words to copy: only the rows the document holds
  if (a.lens != nullptr) {
    int len = ok ? a.lens[doc] : 1;
    len = len < 1 ? 1 : (len > a.G ? a.G : len);
    n16 = (long long)len * a.row16;
    if (hc == 0 && blockIdx.z == 0 && threadIdx.x == 0) a.lens_stage[slot] = len;
  }
  if (!ok) return;  // block-uniform
  const int g = (a.S == 1) ? hc : sl;
  const uint4* src = (blockIdx.z == 0 ? a.K_host : a.V_host) + ((long long)doc * a.Hkv + g) * a.slab16;
  uint4* dst = (blockIdx.z == 0 ? a.K_stage : a.V_stage) + (slot * a.Hkv + g) * a.slab16;
  for (long long i = threadIdx.x; i < n16; i += 256 * 4) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * 256 < n16) v[u] = src[i + u * 256];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * 256 < n16) dst[i + u * 256] = v[u];
  }
}

int launch_fetch(const Dims& dm, const void* K_dev_view, const void* V_dev_view, const int32_t* idx,
                 long long n_rows, int k, void* K_stage, void* V_stage, int32_t* idx_stage,
                 int32_t* lens_stage, hipStream_t st) {
  FetchArgs a;
  a.K_host = (const uint4*)K_dev_view;
  a.V_host = (const uint4*)V_dev_view;
  a.idx = idx;
  a.K_stage = (uint4*)K_stage;
  a.V_stage = (uint4*)V_stage;
  a.idx_stage = idx_stage;
  a.N = dm.N;
  a.Hkv = dm.Hkv;
  a.S = dm.scope_all ? 1 : dm.Hkv;
  a.k = k;
  a.lens = dm.lens;
  a.lens_stage = lens_stage;
  a.G = dm.G;
  a.slab16 = (long long)dm.G * dm.d * 2 / 16;
  a.row16 = dm.d * 2 / 16;
  const long long entries = n_rows * a.S * k;
  if (entries > 0x7fffffffLL) return MSA_ERR_UNSUPPORTED;
  dim3 grid((unsigned)entries, a.S == 1 ? dm.Hkv : 1, 2), block(256);
  hipLaunchKernelGGL(fetch_selected_kernel, grid, block, 0, st, a);
  return hipGetLastError() == hipSuccess ? MSA_OK : MSA_ERR_HIP;
}

}  // namespace msa
