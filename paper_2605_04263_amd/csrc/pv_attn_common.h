// Device helpers shared by the bf16 MFMA attention kernels (gfx950).
#ifndef PV_ATTN_COMMON_H_
#define PV_ATTN_COMMON_H_

#include <type_traits>

#include "pv_internal.h"

namespace pv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);   // round to nearest even
  return __builtin_bit_cast(unsigned, r);
}
__device__ __forceinline__ float bf16_lo(unsigned u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(unsigned u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

// Value held by the lane 32 away (both halves get the other's value via max/sum of the pair).
__device__ __forceinline__ float pair_max(float x) {
  const unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  const unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16-byte LDS read issued as inline assembly: the compiler neither tracks it nor orders it against
// the global->LDS staging loads (its own LDS reads would wait for every outstanding staging load).
// The caller must execute LDS_WAIT on the destination registers before using them.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
  bf16x8 r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}
// The same read refilling `r` in place: the result is tied to the register that held the operand
// just consumed, so the allocator cannot spread a double-buffered operand over two register sets.
template <int OFF>
__device__ __forceinline__ void lds_refill_b128(bf16x8& r, unsigned addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "+v"(r) : "v"(addr), "n"(OFF));
}
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// (cos, sin) of the rotary angle pos * inv_freq.  Angles reach 1e5 rad, so the product is formed
// in fp64 and reduced there to a fraction of a revolution; the hardware cosine and sine take that
// fraction directly.  Measured against fp64 over the positions and frequencies in use: absolute
// error at most 2.6e-7, four orders below the bf16 rounding of what the result rotates.
__device__ __forceinline__ float2 rotary_cos_sin(int pos, double inv_freq) {
  const double rev = (double)pos * inv_freq * 0.15915494309189535;     // angle / (2 pi)
  const float fr = (float)(rev - floor(rev));
  return make_float2(__builtin_amdgcn_cosf(fr), __builtin_amdgcn_sinf(fr));
}

// s_waitcnt immediate (gfx9 encoding) that waits for vmcnt <= n only.
__host__ __device__ constexpr int vmcnt_imm(int n) { return 0x0f70 | (n & 15) | ((n >> 4) << 14); }

}  // namespace pv
#endif
