// Test-only probes of the device helpers in paper_2603_23516_amd/csrc/msa_device.h: the MFMA operand
// layout, the DPP group maximum, bf16 packing and the ordered selection keys.  One wavefront each.
#include "../../paper_2603_23516_amd/csrc/msa_device.h"

using namespace msa;

// A [16][32], B [32][16] bf16 row-major; D [16][16] fp32 row-major.
__global__ void probe_mfma_kernel(const uint16_t* A, const uint16_t* B, float* D) {
  const int lane = threadIdx.x, rr = lane >> 4, n = lane & 15;
  uint32_t aw[4], bw[4];
  for (int jj = 0; jj < 4; ++jj) {
    const int k0 = 8 * rr + 2 * jj;
    aw[jj] = (uint32_t)A[n * 32 + k0] | ((uint32_t)A[n * 32 + k0 + 1] << 16);
    bw[jj] = (uint32_t)B[k0 * 16 + n] | ((uint32_t)B[(k0 + 1) * 16 + n] << 16);
  }
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  acc = mfma16(as_bf16x8(make_uint4(aw[0], aw[1], aw[2], aw[3])),
               as_bf16x8(make_uint4(bw[0], bw[1], bw[2], bw[3])), acc);
  for (int i = 0; i < 4; ++i) D[(4 * rr + i) * 16 + n] = acc[i];
}

// A [32][16], B [16][32] bf16 row-major; D [32][32] fp32 row-major (v_mfma_f32_32x32x16_bf16 layout).
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
__global__ void probe_mfma32_kernel(const uint16_t* A, const uint16_t* B, float* D, float* swapped) {
  const int lane = threadIdx.x, h = lane >> 5, c = lane & 31;
  uint32_t aw[4], bw[4];
  for (int jj = 0; jj < 4; ++jj) {
    const int k0 = 8 * h + 2 * jj;
    aw[jj] = (uint32_t)A[c * 16 + k0] | ((uint32_t)A[c * 16 + k0 + 1] << 16);
    bw[jj] = (uint32_t)B[k0 * 32 + c] | ((uint32_t)B[(k0 + 1) * 32 + c] << 16);
  }
  probe_f32x16 acc;
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(make_uint4(aw[0], aw[1], aw[2], aw[3])),
                                                as_bf16x8(make_uint4(bw[0], bw[1], bw[2], bw[3])), acc, 0, 0, 0);
  for (int i = 0; i < 16; ++i) D[((i % 4) + 8 * (i / 4) + 4 * h) * 32 + c] = acc[i];
  // half-wave exchange used by the GEMM epilogue: every lane must see max(x[l], x[l ^ 32])
  const float x = (float)((lane * 37) % 101);
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  swapped[lane] = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Direct global -> LDS copy: a 64-lane global_load_lds_dwordx4 must land at LDS base + 16 * lane.
__global__ void probe_load_lds_kernel(const uint4* src, uint4* out) {
  __shared__ __attribute__((aligned(16))) unsigned char buf[4096];
  const int wave = threadIdx.x >> 6;
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + threadIdx.x),
                                   (__attribute__((address_space(3))) void*)(buf + wave * 1024), 16, 0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  out[threadIdx.x] = *reinterpret_cast<const uint4*>(buf + threadIdx.x * 16);
}

__global__ void probe_group_max_kernel(const float* in, float* out, int C) {
  const float x = in[threadIdx.x];
  float y = x;
  if (C == 2) y = group_max<2>(x);
  if (C == 4) y = group_max<4>(x);
  if (C == 8) y = group_max<8>(x);
  if (C == 16) y = group_max<16>(x);
  out[threadIdx.x] = y;
  out[64 + threadIdx.x] = dpp_f<kDppXor1>(x);
}

__global__ void probe_pack_kernel(const float* in, uint16_t* out, float* hi, float* lo, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  out[i] = (uint16_t)(pack_bf16(in[i], 0.f) & 0xffffu);
  float h, l;
  split_bf16(in[i], h, l);
  hi[i] = h;
  lo[i] = l;
}

__global__ void probe_keys_kernel(const float* score, const uint32_t* doc, unsigned long long* key,
                                  float* score_back, uint32_t* doc_back, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const unsigned long long k = make_key(score[i], doc[i]);
  key[i] = k;
  score_back[i] = key_score(k);
  doc_back[i] = key_doc(k);
}

extern "C" void probe_mfma(const void* A, const void* B, void* D) {
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(1), dim3(64), 0, 0, (const uint16_t*)A, (const uint16_t*)B, (float*)D);
}
extern "C" void probe_mfma32(const void* A, const void* B, void* D, void* swapped) {
  hipLaunchKernelGGL(probe_mfma32_kernel, dim3(1), dim3(64), 0, 0, (const uint16_t*)A, (const uint16_t*)B,
                     (float*)D, (float*)swapped);
}
extern "C" void probe_load_lds(const void* src, void* out) {
  hipLaunchKernelGGL(probe_load_lds_kernel, dim3(1), dim3(256), 0, 0, (const uint4*)src, (uint4*)out);
}
extern "C" void probe_group_max(const void* in, void* out, int C) {
  hipLaunchKernelGGL(probe_group_max_kernel, dim3(1), dim3(64), 0, 0, (const float*)in, (float*)out, C);
}
extern "C" void probe_pack(const void* in, void* out, void* hi, void* lo, int n) {
  hipLaunchKernelGGL(probe_pack_kernel, dim3((n + 255) / 256), dim3(256), 0, 0, (const float*)in,
                     (uint16_t*)out, (float*)hi, (float*)lo, n);
}
extern "C" void probe_keys(const void* score, const void* doc, void* key, void* sb, void* db, int n) {
  hipLaunchKernelGGL(probe_keys_kernel, dim3((n + 255) / 256), dim3(256), 0, 0, (const float*)score,
                     (const uint32_t*)doc, (unsigned long long*)key, (float*)sb, (uint32_t*)db, n);
}

// Plain copy of n 16-byte words, grid-stride: the known-size reference for HBM counter calibration.
__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         unsigned long long n) {
  const unsigned long long stride = (unsigned long long)gridDim.x * blockDim.x;
  for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    dst[i] = src[i];
}
extern "C" void probe_copy(const void* src, void* dst, unsigned long long nbytes) {
  hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(256), 0, 0, (const uint4*)src, (uint4*)dst,
                     nbytes / 16);
}

// ---- matrix-pipe ceilings for the GEMM scoring kernel's instruction mix --------------------------
// The inner loop of a 256-thread workgroup (4 waves x 64 tokens, 32 products of 32x32x16 bf16 per
// 32-key sub-tile) with its memory side removed step by step:
//   mode 0  registers only (2 accumulators per wave)
//   mode 1  A operand re-read from LDS for every sub-tile (8 x ds_read_b128), next sub-tile prefetched
//   mode 2  mode 1 + the scale / row-max / half-wave-max epilogue
typedef float probe_f32x16_t __attribute__((ext_vector_type(16)));
template <int MODE>
__global__ __launch_bounds__(256) void probe_mfma_ceiling_kernel(float* out, int iters) {
  __shared__ __attribute__((aligned(16))) unsigned char kbuf[3 * 16384];
  __shared__ float inv_s[64];
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, c = lane & 31;
  for (int i = tid; i < 3 * 16384 / 4; i += 256) reinterpret_cast<uint32_t*>(kbuf)[i] = 0x3f803f80u + i;
  if (tid < 64) inv_s[tid] = 1.0f + tid * 0.001f;
  __syncthreads();
  bf16x8_t Bhi[2][8], Blo[2][8];
  for (int cb = 0; cb < 2; ++cb)
    for (int s = 0; s < 8; ++s)
      for (int e = 0; e < 8; ++e) {
        Bhi[cb][s][e] = (__bf16)(0.01f * (lane + s + e + cb));
        Blo[cb][s][e] = (__bf16)(0.001f * (lane + s - e));
      }
  bf16x8_t av[8], an[8];
  auto load_a = [&](int it, bf16x8_t (&dst)[8]) {
    const unsigned char* kcur = kbuf + (it % 6) * 8192;
#pragma unroll
    for (int s = 0; s < 8; ++s)
      dst[s] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(
                                                &kcur[(c >> 4) * 4096 + ((2 * s + h) * 16 + (c & 15)) * 16]));
  };
  load_a(0, av);
  float best = -1e30f;
  probe_f32x16_t acc[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
    if (MODE >= 1) load_a(it + 1, an);
    if (MODE >= 1) {  // a fresh accumulator per sub-tile; registers-only keeps accumulating
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {  // the two accumulators alternate: no product waits for the one before it
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[s], Bhi[0][s], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[s], Bhi[1][s], acc[1], 0, 0, 0);
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[s], Blo[0][s], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[s], Blo[1][s], acc[1], 0, 0, 0);
    }
    if (MODE == 0) {
      // nothing: the accumulators are consumed after the loop
    } else if (MODE == 1) {
      best = fmaxf(best, acc[0][0] + acc[1][5]);
    } else {
      float inv[16];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float4 v = *reinterpret_cast<const float4*>(&inv_s[8 * j + 4 * h]);
        inv[4 * j] = v.x; inv[4 * j + 1] = v.y; inv[4 * j + 2] = v.z; inv[4 * j + 3] = v.w;
      }
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float x0 = acc[cb][4 * j] * inv[4 * j], x1 = acc[cb][4 * j + 1] * inv[4 * j + 1];
          const float x2 = acc[cb][4 * j + 2] * inv[4 * j + 2], x3 = acc[cb][4 * j + 3] * inv[4 * j + 3];
          float m = fmaxf(fmaxf(x0, x1), fmaxf(x2, x3));
          const uint32_t u = __float_as_uint(m);
          const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
          best = fmaxf(best, fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1])));
        }
    }
    if (MODE >= 1) {
#pragma unroll
      for (int s = 0; s < 8; ++s) av[s] = an[s];
    }
  }
  if (MODE == 0) best = acc[0][3] + acc[1][7];
  if (best == 12345.678f) out[tid] = best;  // keeps the loop alive; never true
}
//   mode 3  mode 2 with two accumulator sets: the products of sub-tile t + 1 are issued before the
//           epilogue of sub-tile t, so a wave overlaps its own matrix and vector work
__global__ __launch_bounds__(256) void probe_mfma_pipelined_kernel(float* out, int iters) {
  __shared__ __attribute__((aligned(16))) unsigned char kbuf[3 * 16384];
  __shared__ float inv_s[64];
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, c = lane & 31;
  for (int i = tid; i < 3 * 16384 / 4; i += 256) reinterpret_cast<uint32_t*>(kbuf)[i] = 0x3f803f80u + i;
  if (tid < 64) inv_s[tid] = 1.0f + tid * 0.001f;
  __syncthreads();
  bf16x8_t Bhi[2][8], Blo[2][8];
  for (int cb = 0; cb < 2; ++cb)
    for (int s = 0; s < 8; ++s)
      for (int e = 0; e < 8; ++e) {
        Bhi[cb][s][e] = (__bf16)(0.01f * (lane + s + e + cb));
        Blo[cb][s][e] = (__bf16)(0.001f * (lane + s - e));
      }
  auto products = [&](int it, probe_f32x16_t (&acc)[2]) __attribute__((always_inline)) {
    const unsigned char* kcur = kbuf + (it % 6) * 8192;
    bf16x8_t av[8];
#pragma unroll
    for (int s = 0; s < 8; ++s)
      av[s] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(
                                               &kcur[(c >> 4) * 4096 + ((2 * s + h) * 16 + (c & 15)) * 16]));
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[cb][i] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[s], Bhi[0][s], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[s], Bhi[1][s], acc[1], 0, 0, 0);
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[s], Blo[0][s], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[s], Blo[1][s], acc[1], 0, 0, 0);
    }
  };
  float best = -1e30f;
  auto epilogue = [&](const probe_f32x16_t (&acc)[2]) __attribute__((always_inline)) {
    float inv[16];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float4 v = *reinterpret_cast<const float4*>(&inv_s[8 * j + 4 * h]);
      inv[4 * j] = v.x; inv[4 * j + 1] = v.y; inv[4 * j + 2] = v.z; inv[4 * j + 3] = v.w;
    }
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float x0 = acc[cb][4 * j] * inv[4 * j], x1 = acc[cb][4 * j + 1] * inv[4 * j + 1];
        const float x2 = acc[cb][4 * j + 2] * inv[4 * j + 2], x3 = acc[cb][4 * j + 3] * inv[4 * j + 3];
        float m = fmaxf(fmaxf(x0, x1), fmaxf(x2, x3));
        const uint32_t u = __float_as_uint(m);
        const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        best = fmaxf(best, fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1])));
      }
  };
  probe_f32x16_t acc0[2], acc1[2];
  products(0, acc0);
  for (int it = 0; it < iters; it += 2) {
    products(it + 1, acc1);
    epilogue(acc0);
    products(it + 2, acc0);
    epilogue(acc1);
  }
  if (best == 12345.678f) out[tid] = best;
}
// Times one launch (after a warm-up launch); returns milliseconds, or -1 on error.  Flops per launch:
// blocks * 4 waves * iters * 32 products * 32768.
extern "C" float probe_mfma_ceiling(int mode, int blocks, int iters, void* scratch) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.f;
  float ms = -1.f;
  for (int rep = 0; rep < 2; ++rep) {
    if (hipEventRecord(e0, 0) != hipSuccess) return -1.f;
    if (mode == 0)
      hipLaunchKernelGGL(probe_mfma_ceiling_kernel<0>, dim3(blocks), dim3(256), 0, 0, (float*)scratch, iters);
    else if (mode == 1)
      hipLaunchKernelGGL(probe_mfma_ceiling_kernel<1>, dim3(blocks), dim3(256), 0, 0, (float*)scratch, iters);
    else if (mode == 2)
      hipLaunchKernelGGL(probe_mfma_ceiling_kernel<2>, dim3(blocks), dim3(256), 0, 0, (float*)scratch, iters);
    else
      hipLaunchKernelGGL(probe_mfma_pipelined_kernel, dim3(blocks), dim3(256), 0, 0, (float*)scratch, iters);
    if (hipEventRecord(e1, 0) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return -1.f;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1.f;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return ms;
}
