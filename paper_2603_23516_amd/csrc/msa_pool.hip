// msa_pool_kv: the pooled memory bank of the offline encoding stage (paper, Section 3.4.1, Stage 1):
// every document is position-encoded on its own, positions 0..G-1 (Section 3.2.2), and the keys and
// values are chunk-mean pooled (phi of Section 3.2.1) into the K-bar, V-bar that Eq. 3 concatenates.
// A pure HBM stream like the routing-key build: each K and V element is read once, 1/P of it written.
//
// One wavefront owns one chunk of one tensor.  RoPE pairs element u with u + d/2, so a lane loads
// the 16-byte piece `pc` of a row together with piece pc + d/16 (the partner half): d/16 lanes
// cover a row and a wave-wide pair of loads covers 1024/d rows.  The lane's eight angles
// (cos, sin)(p theta_u) start from a double-precision range reduction at the lane's first row and
// advance by the constant row stride with one complex multiply per load pair.
#include "msa_device.h"
#include "msa_host.h"

namespace msa {

struct PoolTheta {
  double th[64];     // theta_u = base^(-2u/d)
  float2 estep[64];  // (cos, sin)(RPL * theta_u), RPL = rows per wave-wide load
};

template <int D, bool ROT>
__global__ __launch_bounds__(256) void pool_chunks_kernel(const uint16_t* __restrict__ X,
                                                          uint16_t* __restrict__ Xbar,
                                                          const int32_t* __restrict__ lens,
                                                          int32_t* __restrict__ pooled_lens, int doc_begin,
                                                          long long n_chunks, int Hkv, int G, int P,
                                                          int C, PoolTheta th) {
  constexpr int LPR = D / 16;    // lanes per row (each holds a piece and its partner half)
  constexpr int RPL = 64 / LPR;  // rows per wave-wide load pair
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const long long cid = (long long)blockIdx.x * 4 + wave;
  if (cid >= n_chunks) return;  // wave-uniform
  const int j = (int)(cid % C);
  const long long t = cid / C;
  const int g = (int)(t % Hkv);
  const long long doc = doc_begin + t / Hkv;
  const uint16_t* src = X + ((doc * Hkv + g) * (long long)G + (long long)j * P) * D;
  const int pc = lane % LPR;
  const int rowoff = lane / LPR;
  // tokens of this chunk (wave-uniform): a tail chunk is short, a chunk past the end has none and pools to zero
  int n_rows = P;
  if (lens != nullptr) {
    int len = lens[doc];
    len = len < 1 ? 1 : (len > G ? G : len);
    n_rows = len - j * P;
    n_rows = n_rows < 0 ? 0 : (n_rows > P ? P : n_rows);
    if (pooled_lens != nullptr && g == 0 && j == 0 && lane == 0) pooled_lens[doc] = (len + P - 1) / P;
  }

  float2 cs[8], stp[8];
  if (ROT) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      cs[e] = cis_pos(j * P + rowoff, th.th[8 * pc + e]);
      stp[e] = th.estep[8 * pc + e];
    }
  }
  float a1[8], a2[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) a1[e] = a2[e] = 0.f;

  const int iters = (P + RPL - 1) / RPL;
  for (int it0 = 0; it0 < iters; it0 += 4) {
    uint4 v1[4], v2[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = (it0 + u) * RPL + rowoff;
      if (row < n_rows) {
        const uint16_t* rp = src + (long long)row * D + pc * 8;
        v1[u] = load_stream16(rp);
        v2[u] = load_stream16(rp + D / 2);
      } else {
        v1[u] = v2[u] = make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t w1[4] = {v1[u].x, v1[u].y, v1[u].z, v1[u].w};
      const uint32_t w2[4] = {v2[u].x, v2[u].y, v2[u].z, v2[u].w};
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const float p0 = bf16_lo(w1[jj]), p1 = bf16_hi(w1[jj]);
        const float q0 = bf16_lo(w2[jj]), q1 = bf16_hi(w2[jj]);
        if (ROT) {
          const float2 c0 = cs[2 * jj], c1 = cs[2 * jj + 1];
          a1[2 * jj] += p0 * c0.x - q0 * c0.y;
          a1[2 * jj + 1] += p1 * c1.x - q1 * c1.y;
          a2[2 * jj] += q0 * c0.x + p0 * c0.y;
          a2[2 * jj + 1] += q1 * c1.x + p1 * c1.y;
        } else {
          a1[2 * jj] += p0;
          a1[2 * jj + 1] += p1;
          a2[2 * jj] += q0;
          a2[2 * jj + 1] += q1;
        }
      }
      if (ROT) {
#pragma unroll
        for (int e = 0; e < 8; ++e) cs[e] = cmul(cs[e], stp[e]);
      }
    }
  }
  // combine the RPL row groups that hold the same columns
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      a1[e] += __shfl_xor(a1[e], off, 64);
      a2[e] += __shfl_xor(a2[e], off, 64);
    }
  }
  if (rowoff == 0) {
    const float fp = (float)(n_rows > 0 ? n_rows : 1);
    uint16_t* dst = Xbar + (((doc * Hkv + g) * (long long)C + j) * D) + pc * 8;
    *reinterpret_cast<uint4*>(dst) =
        make_uint4(pack_bf16(a1[0] / fp, a1[1] / fp), pack_bf16(a1[2] / fp, a1[3] / fp),
                   pack_bf16(a1[4] / fp, a1[5] / fp), pack_bf16(a1[6] / fp, a1[7] / fp));
    *reinterpret_cast<uint4*>(dst + D / 2) =
        make_uint4(pack_bf16(a2[0] / fp, a2[1] / fp), pack_bf16(a2[2] / fp, a2[3] / fp),
                   pack_bf16(a2[4] / fp, a2[5] / fp), pack_bf16(a2[6] / fp, a2[7] / fp));
  }
}

int launch_pool_kv(const Dims& dm, const void* K, const void* V, int doc_begin, int doc_count,
                   void* Kbar, void* Vbar, int32_t* pooled_lens, hipStream_t st) {
  const long long n_chunks = (long long)doc_count * dm.Hkv * dm.C;
  if (n_chunks == 0) return MSA_OK;
  const long long blocks = (n_chunks + 3) / 4;
  if (blocks > 0x7fffffffLL) return MSA_ERR_UNSUPPORTED;
  PoolTheta th;
  const int rpl = 64 / (dm.d / 16);
  for (int u = 0; u < 64; ++u) {
    th.th[u] = (u < dm.d / 2) ? pow((double)dm.base, -2.0 * (double)u / (double)dm.d) : 0.0;
    th.estep[u] = make_float2((float)cos(rpl * th.th[u]), (float)sin(rpl * th.th[u]));
  }
  dim3 grid((unsigned)blocks), block(256);
  if (Kbar != nullptr) {
    if (dm.d == 128)
      hipLaunchKernelGGL((pool_chunks_kernel<128, true>), grid, block, 0, st, (const uint16_t*)K,
                         (uint16_t*)Kbar, dm.lens, pooled_lens, doc_begin, n_chunks, dm.Hkv, dm.G, dm.P, dm.C, th);
    else
      hipLaunchKernelGGL((pool_chunks_kernel<64, true>), grid, block, 0, st, (const uint16_t*)K,
                         (uint16_t*)Kbar, dm.lens, pooled_lens, doc_begin, n_chunks, dm.Hkv, dm.G, dm.P, dm.C, th);
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  }
  if (Vbar != nullptr) {
    if (dm.d == 128)
      hipLaunchKernelGGL((pool_chunks_kernel<128, false>), grid, block, 0, st, (const uint16_t*)V,
                         (uint16_t*)Vbar, dm.lens, Kbar == nullptr ? pooled_lens : nullptr, doc_begin, n_chunks, dm.Hkv, dm.G, dm.P, dm.C, th);
    else
      hipLaunchKernelGGL((pool_chunks_kernel<64, false>), grid, block, 0, st, (const uint16_t*)V,
                         (uint16_t*)Vbar, dm.lens, Kbar == nullptr ? pooled_lens : nullptr, doc_begin, n_chunks, dm.Hkv, dm.G, dm.P, dm.C, th);
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  }
  return MSA_OK;
}

}  // namespace msa
