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

// the same reads, addressed by a 32-bit LDS byte address (no generic-pointer arithmetic, and constant parts of
// the address fold into the instruction's offset field)
__device__ __forceinline__ bf16x8 lds_read8_at(uint32_t a) { return *(const CA_LDS bf16x8 *)a; }
__device__ __forceinline__ bf16x4 lds_read_tr4_at(uint32_t a) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((CA_LDS bf16x4 *)a);
}
template <class T>
__device__ __forceinline__ T lds_ld(uint32_t a) {
  return *(const CA_LDS T *)a;
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

// max of a value with the one held by lane l ^ 32 (v_permlane32_swap: no LDS round trip)
__device__ __forceinline__ float xor32_max(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}

__device__ __forceinline__ int wave_max(int v) {
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ int wave_min(int v) {
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o));
  return v;
}

}  // namespace ca

// ---------------------------------------------------------------------------------------------
// LDS tiles of R rows x D bf16 in natural (row-major) layout, rows unpadded, with the 16-byte chunks of
// each row XOR-swizzled by a function of the row.  gfx950's LDS has 64 banks of 4 bytes (256 B/clk).
//   * a 16-byte read (lane <-> row, all lanes the same logical chunk) is served 16 consecutive rows
//     at a time, so sw(r) must take 16 (D=128) distinct values over 16 consecutive rows
//     (for D=64, where two rows share a 256-byte line, 8 distinct values over rows of equal parity);
//   * an 8-byte transposing read is served 4 consecutive rows x two adjacent 32-byte pieces at a time, so
//     bits 2..3 of sw must follow the row's low bits.
// sw(r) below satisfies both, so one tile can feed natural and transposed MFMA operands.
// Because rows are unpadded, a tile can be filled by global_load_lds_dwordx4, which writes
// lane i's 16 bytes at (wave-uniform LDS base) + 16 i: the swizzle is applied by choosing which global
// chunk each lane fetches.
namespace ca {

template <int D>
__device__ __forceinline__ int tile_sw(int r) {
  return D == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
}

// byte offset of logical 16-byte chunk c of row r
template <int D>
__device__ __forceinline__ int tile_off(int r, int c) {
  return r * (2 * D) + ((c ^ tile_sw<D>(r)) << 4);
}

#define CA_GLOBAL __attribute__((address_space(1)))
#define CA_CONST __attribute__((address_space(4)))

// One wave-wide direct load global -> LDS: lane i's 16 (or 4) bytes from `src` land at
// lds_base + 16 i (or 4 i); lds_base must be wave-uniform.  Written as inline assembly on purpose: the
// compiler's wait-count insertion treats every LDS read as possibly aliasing an in-flight direct load
// and would drain the whole prefetch queue (s_waitcnt vmcnt(0)) before it.  Here the kernels pace
// the queue themselves with wait_vmcnt<N>() and a barrier.  Loads the compiler does not know about can
// only make its own vmcnt waits stricter than needed, never weaker: vector loads retire in order.
__device__ __forceinline__ void load_lds16(const void *src, char *lds_base_uniform) {
  const uint32_t base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(CA_LDS char *)lds_base_uniform);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(src), "s"(base)
               : "memory", "m0");
}
// same, addressed as (wave-uniform 64-bit base in SGPRs) + (per-lane unsigned 32-bit byte offset); the LDS
// destination is a byte offset from the start of LDS
__device__ __forceinline__ void load_lds16_sbase(const void *base_uniform, uint32_t lane_off, uint32_t lds_off_uniform) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_off_uniform);
  const uint64_t b = (uint64_t)(uintptr_t)base_uniform;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
  const uint64_t sb = ((uint64_t)hi << 32) | lo;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_off), "s"(sb), "s"(m0v)
               : "memory", "m0");
}
// same, with the LDS destination given as a wave-uniform 32-bit LDS byte address
__device__ __forceinline__ void load_lds16_at(const void *src, uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(src), "s"(lds_addr_uniform)
               : "memory", "m0");
}
__device__ __forceinline__ void load_lds4_at(const void *src, uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :
               : "v"(src), "s"(lds_addr_uniform)
               : "memory", "m0");
}
// the same, read at device scope (past this CU's vector L1): for values other workgroups keep writing
__device__ __forceinline__ void load_lds4_at_fresh(const void *src, uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off sc1"
               :
               : "v"(src), "s"(lds_addr_uniform)
               : "memory", "m0");
}
__device__ __forceinline__ void load_lds4(const void *src, char *lds_base_uniform) {
  const uint32_t base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(CA_LDS char *)lds_base_uniform);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :
               : "v"(src), "s"(base)
               : "memory", "m0");
}

// workgroup barrier without the memory fence of __syncthreads() (which would also drain the direct loads):
// the caller has waited for its own LDS reads (lgkmcnt) and for the direct loads that must be visible
__device__ __forceinline__ void barrier_nofence() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Pins a loaded register value: the load is issued and waited for before this point (the compiler would
// otherwise be free to sink loads from read-only memory to their first use inside a loop, together
// with a vector-memory wait that would drain the direct-load queue on every iteration).
__device__ __forceinline__ void pin(bf16x8 &v) {
  u32x4 w = __builtin_bit_cast(u32x4, v);
  asm volatile("" : "+v"(w));
  v = __builtin_bit_cast(bf16x8, w);
}
// same, but leaves the value in an accumulation register (MFMA A/B operands can be read from either file;
// values only ever consumed by MFMAs need not occupy architectural VGPRs)
__device__ __forceinline__ void pin_acc(bf16x8 &v) {
  u32x4 w = __builtin_bit_cast(u32x4, v);
  asm volatile("" : "+a"(w));
  v = __builtin_bit_cast(bf16x8, w);
}

// MFMA whose result tuple lives in ARCHITECTURAL registers and whose B operand lives in the accumulation file.
// A kernel that runs one wave per SIMD has 256 registers of each kind; once it needs both, the compiler gives
// every MFMA an accumulation-file result, and a result the vector ALU needs next then costs one v_accvgpr_read per
// register.  These forms are for short-lived score tiles that go straight to the vector ALU, with B operands that
// stay resident for the whole kernel and are read by MFMAs only.
// The compiler does not see an MFMA in them, so it inserts none of the wait states the hardware requires between an
// MFMA and a non-MFMA instruction that reads its result: mfma_settle() supplies them (the result of this 8-pass
// MFMA may be read 11 issue slots after it; 12 are waited) and takes the tuples as operands, so no reader can be
// scheduled ahead of it.  Between the first MFMA of a chain and the settle nothing else may touch the tuple.
// Dependent MFMAs on one tuple need no wait.
__device__ __forceinline__ void mfma32_v_first(f32x16 &d, bf16x8 a, bf16x8 b_acc) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0"
               : "=&v"(d)
               : "v"(__builtin_bit_cast(u32x4, a)), "a"(__builtin_bit_cast(u32x4, b_acc)));
}
// d = a b + c, with c another architectural tuple
__device__ __forceinline__ void mfma32_v_first(f32x16 &d, bf16x8 a, bf16x8 b_acc, const f32x16 &c) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3"
               : "=&v"(d)
               : "v"(__builtin_bit_cast(u32x4, a)), "a"(__builtin_bit_cast(u32x4, b_acc)), "v"(c));
}
__device__ __forceinline__ void mfma32_v(f32x16 &d, bf16x8 a, bf16x8 b_acc) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
               : "+v"(d)
               : "v"(__builtin_bit_cast(u32x4, a)), "a"(__builtin_bit_cast(u32x4, b_acc)));
}
__device__ __forceinline__ void mfma_settle(f32x16 &x, f32x16 &y) { asm volatile("s_nop 11" : "+v"(x), "+v"(y)); }
// same; `c` was the C operand of the chain's first MFMA: keeping it an operand here keeps its registers from being
// reused (and overwritten by an LDS read in flight) while that MFMA may still be reading them
__device__ __forceinline__ void mfma_settle(f32x16 &x, f32x16 &y, const f32x16 &c) {
  asm volatile("s_nop 11" : "+v"(x), "+v"(y) : "v"(c));
}
// End of a chain whose first non-MFMA reader is known to be at least a whole phase of MFMAs away (the pipelined loop of
// the dK/dV kernel): no wait states are needed, only the ordering of mfma_settle().  The assembly comment is what
// the static check of the generated instruction stream (isa_check.py, run by the CPU tests) looks for: it verifies that
// nothing but MFMAs touches the tuples for the next 16 issue cycles.
__device__ __forceinline__ void mfma_chain_end(f32x16 &x, f32x16 &y, const f32x16 &c) {
  asm volatile("; chain end" : "+v"(x), "+v"(y) : "v"(c));
}
__device__ __forceinline__ void pin(float &v) { asm volatile("" : "+v"(v)); }
// exp2(x * c - g) as one volatile asm statement: like pin() it stays where it is written in the instruction stream
// (between the MFMAs of its slot), but without the wait state the compiler puts between an empty asm that "defines"
// a register and the first instruction that reads it.  (A multiply-add feeding a transcendental needs no wait state.)
__device__ __forceinline__ uint32_t pack_bf16_pinned(float a, float b) {
  uint32_t r;
  asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// {bf16(p0 * d0), bf16(p1 * d1)} and {bf16(p2 * d2), bf16(p3 * d3)}, pinned likewise
__device__ __forceinline__ void mul_pack_bf16_pinned(float p0, float p1, float p2, float p3, float d0, float d1,
                                                     float d2, float d3, uint32_t &lo, uint32_t &hi) {
  float t0, t1, t2, t3;
  asm volatile(
      "v_mul_f32 %2, %6, %10\n\tv_mul_f32 %3, %7, %11\n\tv_mul_f32 %4, %8, %12\n\tv_mul_f32 %5, %9, %13\n\t"
      "v_cvt_pk_bf16_f32 %0, %2, %3\n\tv_cvt_pk_bf16_f32 %1, %4, %5"
      : "=&v"(lo), "=&v"(hi), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
      : "v"(p0), "v"(p1), "v"(p2), "v"(p3), "v"(d0), "v"(d1), "v"(d2), "v"(d3));
}
__device__ __forceinline__ float exp2_fma_pinned(float x, float c, float g) {
  float r;
  asm volatile("v_fma_f32 %0, %1, %2, -%3\n\tv_exp_f32 %0, %0" : "=v"(r) : "v"(x), "v"(c), "v"(g));
  return r;
}
// x = exp2(x * c - g) in place (the register of x is reused, so a register tuple exponentiated element by element
// stays where it is), pinned likewise
__device__ __forceinline__ void exp2_fma_inplace_pinned(float &x, float c, float g) {
  asm volatile("v_fma_f32 %0, %0, %1, -%2\n\tv_exp_f32 %0, %0" : "+v"(x) : "v"(c), "v"(g));
}
// the same with sum += prev in between.  prev may be the result of the transcendental issued directly before this
// statement: the multiply-add stands between the two.
__device__ __forceinline__ void exp2_fma_add_inplace_pinned(float &x, float c, float g, float &sum, float prev) {
  asm volatile("v_fma_f32 %0, %0, %2, -%3\n\tv_add_f32 %1, %1, %4\n\tv_exp_f32 %0, %0"
               : "+v"(x), "+v"(sum)
               : "v"(c), "v"(g), "v"(prev));
}
// sum += prev where prev may be the result of a transcendental issued directly before (one wait state supplied)
__device__ __forceinline__ void add_after_trans_pinned(float &sum, float prev) {
  asm volatile("s_nop 0\n\tv_add_f32 %0, %0, %1" : "+v"(sum) : "v"(prev));
}
__device__ __forceinline__ void pin(int &v) { asm volatile("" : "+v"(v)); }

// wait until at most n of this wave's vector-memory loads are outstanding (n <= 63)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  // the empty asm statements keep the compiler from moving loads or stores across the wait
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  asm volatile("" ::: "memory");
}


// ---- a wave's 32 x D result tile, stored as whole lines.
// In the accumulator layout of Xt = A B (32x32 MFMAs, 32-row blocks b of the D values) lane (r, g) holds, of row r
// (a key, or a query row), the values 32 b + 8 q4 + 4 g .. + 3 in acc[b][4 q4 ..]: 4 values out of every 8.  Stored
// from there, one instruction touches 32 rows with 16 bytes each, and the 16 D / 32 of them per tile keep a CU's address
// unit busy for microseconds.  Instead the wave passes 64 values per row at a time through an LDS patch of its own
// (PATCH_BYTES at `patch`, an LDS byte address; a wave's LDS instructions execute in order, so nothing synchronises)
// and stores 8 rows x 128 bytes per instruction.  f scales the values (per lane, i.e. per row r); dst_of_row(p)
// returns where row p (0..31) of the tile begins in memory, or nullptr for a row that is not stored.
constexpr int PATCH_ROW_BYTES = 128 + 16;  // 16 bytes off a power of two
constexpr int PATCH_BYTES = 32 * PATCH_ROW_BYTES;
template <int NDB, class F>
__device__ __forceinline__ void store_tile_as_lines(uint32_t patch, const f32x16 (&acc)[NDB], float f, int lane,
                                                    F dst_of_row) {
  const int r = lane & 31, g = lane >> 5, orow = lane >> 3, ocol = lane & 7;
  const uint32_t wr = patch + r * PATCH_ROW_BYTES + 8 * g;  // + 64 (b & 1) + 16 q4
  const uint32_t rd = patch + orow * PATCH_ROW_BYTES + 16 * ocol;  // the lane's row (+ 8 i) and 16-byte piece
  bf16_t *dst[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) dst[i] = dst_of_row(orow + 8 * i);
#pragma unroll
  for (int h = 0; h < NDB / 2; ++h) {
#pragma unroll
    for (int bb = 0; bb < 2; ++bb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x16 &a = acc[2 * h + bb];
        const u32x2 w = {pack_bf16(a[4 * q4] * f, a[4 * q4 + 1] * f), pack_bf16(a[4 * q4 + 2] * f, a[4 * q4 + 3] * f)};
        *(CA_LDS u32x2 *)(wr + 64 * bb + 16 * q4) = w;
      }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32x4 x = *(const CA_LDS u32x4 *)(rd + 8 * i * PATCH_ROW_BYTES);
      if (dst[i]) *reinterpret_cast<u32x4 *>(dst[i] + 64 * h + 8 * ocol) = x;
    }
  }
}

}  // namespace ca
