// Helpers shared by the MFMA kernel files (gfx950 only): vector types, the per-element-type MFMA
// wrappers, cross-lane reductions over the four row groups of an MFMA tile, the LDS transpose read,
// the two-term split of an fp32 value into element-type operands, and the host-side opt-in for more
// than 64 KB of dynamic LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.h"
#include "lds_optin.h"

namespace aa {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// v_mfma_f32_16x16x32 for the element type, packing / unpacking of element pairs.
// Lane conventions (r = lane % 16, g = lane / 16): an A/B operand holds row/column r and the 8 k-values
// of group g; C/D holds column r and rows 4g..4g+3.
template <class E>
struct Mx;
template <>
struct Mx<ElemBF16> {
  static constexpr uint32_t kOnes2 = 0x3F803F80u;      // two elements of value 1
  static __device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  }
  static __device__ __forceinline__ float bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
  static __device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xFFFF0000u);
  }
  // acc + the two packed elements of w (one v_dot2c against a pair of ones)
  static __device__ __forceinline__ float add_pair(uint32_t w, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, kOnes2), acc, false);
  }
};
template <>
struct Mx<ElemF16> {
  static constexpr uint32_t kOnes2 = 0x3C003C00u;      // two elements of value 1
  static __device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                  0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
  }
  static __device__ __forceinline__ float bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
  static __device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
    const f16x2 h = __builtin_bit_cast(f16x2, w);
    lo = (float)h[0];
    hi = (float)h[1];
  }
  static __device__ __forceinline__ float add_pair(uint32_t w, float acc) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w), __builtin_bit_cast(f16x2, kOnes2), acc, false);
  }
};

// Two-term representation of fp32 values in the element type: hi = rn(v), lo = rn(v - hi).  hi + lo carries
// 16 (bf16) or 22 (fp16) significant bits, so a product against exact 16-bit operands taken as two MFMAs
// (one per term, same accumulator) loses nothing a 16-bit rounding of v would have lost.  Used for the
// pooled agent tokens, which are averages of element-type values and not representable in the type.
template <class E>
__device__ __forceinline__ u32x2 split2(float a, float b) {      // returns {hi pair, lo pair}
  const uint32_t hi = Mx<E>::pack2(a, b);
  float ah, bh;
  Mx<E>::unpack2(hi, ah, bh);
  return u32x2{hi, Mx<E>::pack2(a - ah, b - bh)};
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Reductions over the four lanes r, r+16, r+32, r+48 (same MFMA column, the four row groups) with the
// gfx950 row-swap instructions: permlane32_swap(v, v) yields (lower half twice, upper half twice),
// permlane16_swap(v, v) yields (rows 0,0,2,2) and (rows 1,1,3,3).
__device__ __forceinline__ float xor16_32_max(float v) {
  const uint32_t b = __float_as_uint(v);
  const auto h = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  const uint32_t c = __float_as_uint(fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1])));
  const auto q = __builtin_amdgcn_permlane16_swap(c, c, false, false);
  return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}
__device__ __forceinline__ float xor16_32_sum(float v) {
  const uint32_t b = __float_as_uint(v);
  const auto h = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  const uint32_t c = __float_as_uint(__uint_as_float(h[0]) + __uint_as_float(h[1]));
  const auto q = __builtin_amdgcn_permlane16_swap(c, c, false, false);
  return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// LDS transpose read of 4 x 16 bit (ds_read_b64_tr_b16): within a group of 16 lanes, lane q supplies the
// address of 4 consecutive elements; lane i receives element i%4 of the chunks addressed by lanes
// i/4, 4 + i/4, 8 + i/4 and 12 + i/4.
__device__ __forceinline__ u32x2 lds_read_tr(const uint16_t* p) {
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  return __builtin_bit_cast(u32x2, v);
}

// Kernels whose dynamic LDS may exceed 64 KB need an opt-in per kernel function and device (gfx950 has
// 160 KB per CU).  The registry remembers (function, device) pairs, so the attribute call is made once
// for each kernel instantiation -- instantiations of one template share a pointer type but not an address.
template <class KernelT>
static hipError_t allow_lds(KernelT kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return hipSuccess;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (!lds_optin_registry().needs((const void*)kernel, dev)) return hipSuccess;
  e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess) lds_optin_registry().done((const void*)kernel, dev);
  return e;
}

}  // namespace aa
