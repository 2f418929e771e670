// Device-side helpers for the gfx950 kernels: MFMA fragment types, LDS reads, bf16 packing.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ca {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CA_LDS __attribute__((address_space(3)))

// v_mfma_f32_32x32x16_bf16: C[32x32] += A[32x16] * B[16x32].
//   A: lane l holds A[l%32][8*(l/32) .. +7];  B: lane l holds B[8*(l/32) .. +7][l%32];
//   C: lane l, register i holds C[(i/4)*8 + (l/32)*4 + i%4][l%32].
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// 16-byte LDS read of 8 consecutive bf16.
__device__ __forceinline__ bf16x8 lds_read8(const char *p) { return *reinterpret_cast<const bf16x8 *>(p); }

// ds_read_b64_tr_b16: inside each group of 16 lanes, lane i points at 4 consecutive bf16 and receives
// element (i%4) of the 4 values read by lanes 4j + i/4, j = 0..3.  With lane i pointing at
// tile[r0 + i/4][c0 + 4*(i%4)] the lane gets tile[r0 .. r0+3][c0 + i]: a 4x16 block, transposed.
__device__ __forceinline__ bf16x4 lds_read_tr4(const char *p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CA_LDS bf16x4 *)(p));
}

__device__ __forceinline__ bf16x8 join(bf16x4 lo, bf16x4 hi) {
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ int wave_max(int v) {
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ int wave_min(int v) {
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o));
  return v;
}

}  // namespace ca
