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
