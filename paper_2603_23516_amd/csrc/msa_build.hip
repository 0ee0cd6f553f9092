// msa_build_routing_keys: chunk-wise mean pooling phi(.) of the keys (paper, Section 3.2.1, text
// after Eq. 1) into the tiled routing index.  A pure HBM stream: every key element is read once,
// 1/P of that volume is written.
//
// One wavefront owns one chunk (P rows of d bf16, contiguous in the bank).  A 64-lane 16-byte load
// covers 1 KiB = 64*8/d rows, so the whole chunk (16 KiB at P=64, d=128) is in flight as P*d/512
// independent loads per wave.  Rows are summed in fp32 per lane, the partial sums of the lanes that
// share a column are combined with cross-lane shuffles, and the d/8 lanes of row-group 0 write the
// 16-byte pieces of the rounded mean straight into the tile slot of this key.
#include "msa_device.h"
#include "msa_host.h"

namespace msa {

template <int D>
__global__ __launch_bounds__(256) void build_routing_keys_kernel(
    const uint16_t* __restrict__ K, uint16_t* __restrict__ KR, float* __restrict__ inv_norm,
    const int32_t* __restrict__ lens, int doc_begin, long long n_chunks, int Hkv, int G, int P, int C,
    long long tiles) {
  constexpr int LPR = D / 8;     // lanes per row (16-byte pieces)
  constexpr int RPL = 64 / LPR;  // rows per wave-wide load
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const long long cid = (long long)blockIdx.x * 4 + wave;
  if (cid >= n_chunks) return;  // wave-uniform
  const int j = (int)(cid % C);
  const long long t = cid / C;
  const int g = (int)(t % Hkv);
  const long long doc = doc_begin + t / Hkv;
  // Tokens of this chunk (wave-uniform).  A chunk past the document's end repeats chunk 0: the
  // document score is a max over chunks, which a repeated chunk cannot change.
  int n_rows = P, jsrc = j;
  if (lens != nullptr) {
    int len = lens[doc];
    len = len < 1 ? 1 : (len > G ? G : len);
    n_rows = len - j * P;
    if (n_rows <= 0) {
      jsrc = 0;
      n_rows = len;
    }
    n_rows = n_rows > P ? P : n_rows;
  }
  const uint16_t* src = K + ((doc * Hkv + g) * (long long)G + (long long)jsrc * P) * D;
  const int piece = lane % LPR;
  const int rowoff = lane / LPR;

  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;

  const int iters = P / RPL;
  for (int it0 = 0; it0 < iters; it0 += 8) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int it = it0 + u;
      if (it < iters && it * RPL + rowoff < n_rows) {
        v[u] = load_stream16(src + (long long)(it * RPL + rowoff) * D + piece * 8);
      } else {
        v[u] = make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      acc[0] += bf16_lo(v[u].x);
      acc[1] += bf16_hi(v[u].x);
      acc[2] += bf16_lo(v[u].y);
      acc[3] += bf16_hi(v[u].y);
      acc[4] += bf16_lo(v[u].z);
      acc[5] += bf16_hi(v[u].z);
      acc[6] += bf16_lo(v[u].w);
      acc[7] += bf16_hi(v[u].w);
    }
  }
  // combine the RPL row groups that hold the same columns
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], off, 64);
  }
  const float fp = (float)n_rows;
  uint4 o;
  o.x = pack_bf16(acc[0] / fp, acc[1] / fp);
  o.y = pack_bf16(acc[2] / fp, acc[3] / fp);
  o.z = pack_bf16(acc[4] / fp, acc[5] / fp);
  o.w = pack_bf16(acc[6] / fp, acc[7] / fp);

  // squared norm of the ROUNDED key
  float ss = 0.f;
  {
    const float r0 = bf16_lo(o.x), r1 = bf16_hi(o.x), r2 = bf16_lo(o.y), r3 = bf16_hi(o.y);
    const float r4 = bf16_lo(o.z), r5 = bf16_hi(o.z), r6 = bf16_lo(o.w), r7 = bf16_hi(o.w);
    ss = r0 * r0 + r1 * r1 + r2 * r2 + r3 * r3 + r4 * r4 + r5 * r5 + r6 * r6 + r7 * r7;
  }
#pragma unroll
  for (int off = 1; off < LPR; off <<= 1) ss += __shfl_xor(ss, off, 64);

  const long long c = doc * C + j;  // key number inside head g
  const long long tile = c >> 4;
  const int n = (int)(c & 15);
  if (rowoff == 0) {
    uint16_t* dst = KR + ((long long)g * tiles + tile) * (16 * D) + (piece * 16 + n) * 8;
    *reinterpret_cast<uint4*>(dst) = o;
  }
  if (lane == 0 && inv_norm != nullptr) {
    inv_norm[(long long)g * tiles * 16 + c] = 1.0f / fmaxf(sqrtf(ss), 1e-12f);
  }
}

// Zero the slots of the last tile that lie past the last key.
template <int D>
__global__ void pad_tail_kernel(uint16_t* __restrict__ KR, float* __restrict__ inv_norm,
                                long long NC, long long tiles, int Hkv) {
  const int n_pad = (int)(tiles * 16 - NC);
  const int per_head = n_pad * (D / 8);
  const int tid = blockIdx.x * blockDim.x + threadIdx.x;
  if (tid >= per_head * Hkv) return;
  const int g = tid / per_head;
  const int e = tid % per_head;
  const int slot = (int)(NC & 15) + e / (D / 8);
  const int piece = e % (D / 8);
  uint16_t* dst = KR + ((long long)g * tiles + (tiles - 1)) * (16 * D) + (piece * 16 + slot) * 8;
  *reinterpret_cast<uint4*>(dst) = make_uint4(0, 0, 0, 0);
  if (piece == 0 && inv_norm != nullptr) inv_norm[(long long)g * tiles * 16 + NC + (slot - (int)(NC & 15))] = 0.f;
}

int launch_build(const Dims& dm, const void* K, int doc_begin, int doc_count, void* KR,
                 float* inv_norm, hipStream_t st) {
  const long long n_chunks = (long long)doc_count * dm.Hkv * dm.C;
  if (n_chunks > 0) {
    const long long blocks = (n_chunks + 3) / 4;
    if (blocks > 0x7fffffffLL) return MSA_ERR_UNSUPPORTED;
    dim3 grid((unsigned)blocks), block(256);
    if (dm.d == 128) {
      hipLaunchKernelGGL(build_routing_keys_kernel<128>, grid, block, 0, st, (const uint16_t*)K,
                         (uint16_t*)KR, inv_norm, dm.lens, doc_begin, n_chunks, dm.Hkv, dm.G, dm.P, dm.C,
                         (long long)dm.tiles);
    } else {
      hipLaunchKernelGGL(build_routing_keys_kernel<64>, grid, block, 0, st, (const uint16_t*)K,
                         (uint16_t*)KR, inv_norm, dm.lens, doc_begin, n_chunks, dm.Hkv, dm.G, dm.P, dm.C,
                         (long long)dm.tiles);
    }
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  }
  const int n_pad = (int)(dm.tiles * 16 - dm.NC);
  if (n_pad > 0 && doc_begin + doc_count == dm.N) {
    const int total = n_pad * (dm.d / 8) * dm.Hkv;
    dim3 grid((total + 255) / 256), block(256);
    if (dm.d == 128) {
      hipLaunchKernelGGL(pad_tail_kernel<128>, grid, block, 0, st, (uint16_t*)KR, inv_norm,
                         (long long)dm.NC, (long long)dm.tiles, dm.Hkv);
    } else {
      hipLaunchKernelGGL(pad_tail_kernel<64>, grid, block, 0, st, (uint16_t*)KR, inv_norm,
                         (long long)dm.NC, (long long)dm.tiles, dm.Hkv);
    }
    if (hipGetLastError() != hipSuccess) return MSA_ERR_HIP;
  }
  return MSA_OK;
}

}  // namespace msa
