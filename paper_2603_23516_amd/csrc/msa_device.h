// Device-side helpers shared by the MSA kernels (gfx950 only, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace msa {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// ---- asynchronous copies global -> LDS ---------------------------------------------------------
// One 64-lane copy of 16 bytes per lane: lane l's 16 bytes from its own global address land at LDS
// byte lds_base + 16 l (lds_base: the same value in every lane; goff < 2^31).  Nothing waits here: the caller counts
// the copy in s_waitcnt vmcnt like any load and orders it against the readers of that LDS itself.
// Written as assembly because for the builtin of the same instruction the compiler, unable to tell
// which LDS bytes a copy fills, waits for EVERY outstanding copy before the next LDS read of any kind,
// which turns a multi-stage pipeline into a synchronous load.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // m0 is reserved: the compiler keeps nothing in it across statements
__device__ __forceinline__ void copy16_to_lds_async(const void* gbase, uint32_t goff, const void* lds_base) {
  // source of lane l: gbase (the same in every lane) + goff (the lane's own byte offset)
  const uint32_t base = __builtin_amdgcn_readfirstlane(
      (uint32_t)(size_t)(const __attribute__((address_space(3))) void*)lds_base);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(goff), "s"(gbase), "s"(base) : "memory", "m0");
}
// The same with 4 bytes per lane: lane l's word lands at lds_base + 4 l.
__device__ __forceinline__ void copy4_to_lds_async(const void* gbase, uint32_t goff, const void* lds_base) {
  const uint32_t base = __builtin_amdgcn_readfirstlane(
      (uint32_t)(size_t)(const __attribute__((address_space(3))) void*)lds_base);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :: "v"(goff), "s"(gbase), "s"(base) : "memory", "m0");
}
// 16 bytes per lane of data that is read once (streaming hint, see load_stream16); the destination is given as an
// LDS byte address in a scalar register (lds_addr_of).  Source: scalar base + lane offset ...
__device__ __forceinline__ void copy16_to_lds_async_stream(const void* gbase, uint32_t goff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
               :: "v"(goff), "s"(gbase), "s"(lds_addr) : "memory", "m0");
}
// ... or a full 64-bit address per lane (rows gathered from anywhere in a large allocation).
__device__ __forceinline__ void copy16_to_lds_async_stream64(const void* gaddr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
               :: "v"(gaddr), "s"(lds_addr) : "memory", "m0");
}
// LDS byte address of a __shared__ object
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(size_t)(const __attribute__((address_space(3))) void*)p;
}
#pragma clang diagnostic pop
template <int N>
__device__ __forceinline__ void wait_copies_but() {  // until at most the N newest loads / copies are outstanding
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// ---- streaming loads ---------------------------------------------------------------------------
// Data that a launch reads exactly once (the routing index of a scan, the rows of a gathered document, the bank
// under the index build) is loaded with the non-temporal hint: the line is not kept in the caches on its way
// through.  A plain streaming read of a large buffer tops out near 6.2 TB/s on this chip; the same loads with the
// hint reach 6.9-7.3 TB/s (measured with loads-only kernels over 1.6 GB and 8 GB, 2 to 16 waves per CU).  Only for
// accesses that take whole 128-byte lines in one instruction: a line that two instructions share is fetched again
// for the second one, and the hint then costs more than it gives.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float load_stream(const float* p) { return __builtin_nontemporal_load(p); }

// ---- transposing LDS read -------------------------------------------------------------------------
// ds_read_b64_tr_b16: among 16 consecutive lanes, lane j hands in the address of elements 4 (j % 4) .. + 3 of row
// j / 4 (four rows of 16 two-byte elements, anywhere in LDS) and receives element j of rows 0 .. 3.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ s16x4_t lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)p);
}

// ---- bf16 <-> fp32 ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Two floats -> packed bf16 pair (a in the low half), round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// x = hi + lo with hi = bf16(x), lo = bf16(x - hi): carries ~16 significant bits through bf16 MFMA.
__device__ __forceinline__ void split_bf16(float x, float& hi, float& lo) {
  hi = bf16_lo(pack_bf16(x, 0.f));
  lo = x - hi;
}

// The same for a pair, straight to packed words: hi_w = (bf16(x0), bf16(x1)), lo_w = (bf16(x0 - hi0), bf16(x1 - hi1)).
__device__ __forceinline__ void split_pack_bf16(float x0, float x1, uint32_t& hi_w, uint32_t& lo_w) {
  hi_w = pack_bf16(x0, x1);
  lo_w = pack_bf16(x0 - bf16_lo(hi_w), x1 - bf16_hi(hi_w));
}

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8_t, v); }

// D(16x16, fp32) += A(16x32, bf16) * B(32x16, bf16).
// Lane l = 16*q + n holds A[n][8q..8q+7], B[8q..8q+7][n], and D[4q..4q+3][n].
__device__ __forceinline__ f32x4_t mfma16(bf16x8_t a, bf16x8_t b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// ---- cross-lane ----------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7 - i inside each group of 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15 - i inside each row of 16

// Max over aligned groups of C consecutive lanes (C in {1,2,4,8,16}); every lane gets the result.
template <int C>
__device__ __forceinline__ float group_max(float x) {
  if (C >= 2) x = fmaxf(x, dpp_f<kDppXor1>(x));
  if (C >= 4) x = fmaxf(x, dpp_f<kDppXor2>(x));
  if (C >= 8) x = fmaxf(x, dpp_f<kDppHalfMirror>(x));
  if (C >= 16) x = fmaxf(x, dpp_f<kDppMirror>(x));
  return x;
}

// ---- rotary position encoding ---------------------------------------------------------------
// (cos, sin)(p * theta): product and range reduction in double, sincos of the reduced angle in fp32.
__device__ __forceinline__ float2 cis_pos(int p, double theta) {
  const double x = (double)p * theta;
  const double kk = rint(x * 0.15915494309189535);
  double red = fma(-kk, 6.283185307179586, x);
  red = fma(-kk, 2.4492935982947064e-16, red);
  float s, c;
  sincosf((float)red, &s, &c);
  return make_float2(c, s);
}

__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}

// ---- ordered 64-bit selection keys ---------------------------------------------------------------
// Larger key = better candidate: score descending, then document index ascending.
__device__ __forceinline__ uint32_t orderable(float s) {
  uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unorderable(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}
__device__ __forceinline__ uint64_t make_key(float score, uint32_t doc) {
  return ((uint64_t)orderable(score) << 32) | (uint64_t)(0xffffffffu - doc);
}
__device__ __forceinline__ uint32_t key_doc(uint64_t key) { return 0xffffffffu - (uint32_t)key; }
__device__ __forceinline__ float key_score(uint64_t key) { return unorderable((uint32_t)(key >> 32)); }

// ---- device-coherent accesses ----------------------------------------------------------------------
// Every XCD has its own L2, so data that one workgroup writes and a workgroup on another XCD reads within the same
// launch must not linger in (or be served from) an L2.  These accesses carry device scope: the store is written
// through to memory, the load is not served from a stale line.  Once a thread's stores are complete
// (wait_stores_done) they are visible to device-scope loads anywhere on the chip; no cache-wide write-back or
// invalidate (which every wave of a launch would have to pay for) is involved.
__device__ __forceinline__ void store_dev(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_dev(unsigned long long* p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_dev(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_dev(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Workgroup barrier for data exchanged through LDS only.  __syncthreads also fences global memory, i.e. waits
// for every global load the wave has in flight; a stream that was started before the barrier should stay in
// flight across it.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// ---- arrival counter that needs no initialisation ------------------------------------------------
// Workgroups that produced parts of one result count themselves in; the one that arrives last combines the
// parts.  The 64-bit word holds (nonce << 16 | arrivals); a word whose upper 48 bits are not this call's nonce
// is a leftover (the caller's workspace has undefined contents) and counts as zero arrivals, so nothing has
// to be cleared before the launch.  The first arrival installs the nonce with a compare-exchange; every later
// one sees the nonce and counts itself with a plain fetch-add (arrivals that come together are then served by
// the memory's atomic unit back to back instead of retrying one after the other).  Returns the number of
// arrivals BEFORE this one.  Every path ends: an exchange fails only because another arrival installed the
// nonce, after which the fetch-add path is taken.  The last arrival stores 0 when it is done, which keeps
// replays of a captured launch (same nonce every time) correct.  nonce48 != 0; fewer than 65536 participants.
__device__ __forceinline__ uint32_t arrive_at(unsigned long long* word, unsigned long long nonce48) {
  unsigned long long old = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if ((old >> 16) != nonce48) {
    const unsigned long long first = (nonce48 << 16) | 1ull;
    if (__hip_atomic_compare_exchange_strong(word, &old, first, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT))
      return 0u;
    if ((old >> 16) != nonce48) {
      // the word changed between the load and the exchange without the nonce appearing: it can only have been
      // a foreign write (the workspace is shared with something else); fall back to the exchange loop
      for (;;) {
        const uint32_t cnt = ((old >> 16) == nonce48) ? (uint32_t)(old & 0xffffull) : 0u;
        if (__hip_atomic_compare_exchange_strong(word, &old, (nonce48 << 16) | (unsigned long long)(cnt + 1u),
                                                 __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
          return cnt;
      }
    }
  }
  old = __hip_atomic_fetch_add(word, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return (uint32_t)(old & 0xffffull);
}

}  // namespace msa
