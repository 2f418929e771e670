// Calibration aid for the matrix-pipe roofline (not a step of the method): a kernel that does nothing but issue
// v_mfma_f32_32x32x16_bf16 back to back from registers, the instruction all three attention kernels are built on.
// Timed over the whole chip it gives the rate the matrix pipes sustain on a given kind of operand data (the chip
// lowers its clock under such load, by an amount that depends on the data), which is what the attention kernels'
// executed flop rates can be held against besides the published peak.
#include <hip/hip_runtime.h>

#include <sstream>

#include "ca_attention.h"
#include "ca_device.h"
#include "ca_internal.h"

namespace ca {

constexpr int CALIB_FRAGS = 8;         // A/B fragment pairs a thread holds
constexpr int CALIB_ROUND = 64;        // MFMAs per loop iteration: every A fragment against every B fragment
constexpr int CALIB_LDS_BYTES = 16384; // side work reads the first 16 KiB of the operands from LDS

// Thread t of every workgroup loads A fragment i from operands[(2 i) * 256 + t] and B fragment i from
// operands[(2 i + 1) * 256 + t] (16 bytes = 8 bf16 each), then runs n_rounds iterations of 64 MFMAs, MFMA (r, j)
// of an iteration being chain[j & 3] += A[j] x B[(j + r) & 7]: four independent accumulation chains, so that no
// MFMA waits for the one before it.  SIDE = 0: nothing else in the loop.  SIDE = 1 / 2: after every MFMA the wave
// also issues the kind of work an attention kernel does per MFMA, results unused: one 16-byte LDS read per lane
// (1 KiB per wave, an MFMA operand's worth), 2 / 4 fp32 multiply-adds and an exponential after every second / after
// every MFMA (about the dK/dV kernel's and the forward kernel's ratio).
template <int SIDE>
__global__ __launch_bounds__(256) void ca_mfma_stream_kernel(const u32x4 *__restrict__ operands, int n_rounds,
                                                             float *__restrict__ sums) {
  extern __shared__ u32x4 calib_lds[];
  u32x4 a[CALIB_FRAGS], b[CALIB_FRAGS];
#pragma unroll
  for (int i = 0; i < CALIB_FRAGS; ++i) {
    a[i] = operands[(2 * i) * 256 + threadIdx.x];
    b[i] = operands[(2 * i + 1) * 256 + threadIdx.x];
  }
  uint32_t lds_addr = 0;
  float v[8], e[4];
  u32x4 t[4];
  if (SIDE > 0) {
#pragma unroll
    for (int i = 0; i < CALIB_LDS_BYTES / 16 / 256; ++i) calib_lds[i * 256 + threadIdx.x] = a[i];
    __syncthreads();
    lds_addr = uint32_t(size_t(&calib_lds[0])) + 16 * threadIdx.x;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = __builtin_bit_cast(float, a[i][0] << 16);  // a bf16 operand value
  }
  f32x16 c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
  for (int it = 0; it < n_rounds; ++it) {
#pragma unroll
    for (int r = 0; r < CALIB_FRAGS; ++r)
#pragma unroll
      for (int j = 0; j < CALIB_FRAGS; ++j) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c[j & 3]) : "v"(a[j]), "v"(b[(j + r) & 7]));
        if (SIDE > 0) {
          // reads stay inside the 16 KiB: 16 * 255 + 3 * 4096 + 16 bytes at most
          asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(t[j & 3]) : "v"(lds_addr), "n"((j & 3) * 4096));
#pragma unroll
          for (int l = 0; l < 2 * SIDE; ++l)
            asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(v[(j + l) & 7]) : "v"(0.75f), "v"(0.25f));
          // its result is not read by the vector instructions that follow it directly
          if (SIDE == 2 || (j & 1)) asm volatile("v_exp_f32 %0, %1" : "=v"(e[j & 3]) : "v"(v[(j + 4) & 7]));
          if ((j & 3) == 3) asm volatile("s_waitcnt lgkmcnt(0)" ::"v"(t[0]), "v"(t[1]), "v"(t[2]), "v"(t[3]));
        }
      }
  }
  // the wait states between the last MFMAs and the first vector instruction that reads their results, tied to the
  // accumulators so that nothing can be scheduled around them
  asm volatile("s_nop 15\n\ts_nop 15" : "+v"(c[0]), "+v"(c[1]), "+v"(c[2]), "+v"(c[3]));
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += (c[0][i] + c[1][i]) + (c[2][i] + c[3][i]);
  sums[size_t(blockIdx.x) * 256 + threadIdx.x] = s;
}

// Which XCD (accelerator complex die; each has its own L2) a workgroup runs on.  The planner's work order relies on
// the workgroups of a launch going to the XCDs round robin in index order; this kernel lets a test see the mapping.
__global__ void ca_xcd_map_kernel(int32_t *__restrict__ out) {
  // hardware register 20 (XCC_ID), bits 3:0
  const uint32_t x = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20) & 15u;
  if (threadIdx.x == 0) out[blockIdx.x] = int32_t(x);
}

// What accumulating dQ with fp32 atomics from a KV-tile-owning backward kernel would cost: every workgroup (four
// waves) runs `steps` steps; in a step every wave issues mfma_per_step MFMAs (four independent chains, operands as in
// the kernel above) and atomics_per_step global_atomic_add_f32 of +1.0 per lane (256 contiguous bytes per wave
// instruction) into the wave's quarter of a 32 KiB tile.  Workgroup i works on region i mod 8 (8 regions of n_tiles
// tiles) and walks the tiles round, a few tiles apart from its neighbours - the access pattern of workgroups that own
// neighbouring KV tiles of one KV head and walk the same query blocks.
__global__ __launch_bounds__(256) void ca_atomic_stream_kernel(const u32x4 *__restrict__ operands, float *tiles,
                                                               int n_tiles, int steps, int mfma_per_step,
                                                               int atomics_per_step, float *__restrict__ sums) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const u32x4 a = operands[threadIdx.x], b = operands[256 + threadIdx.x];
  float *region = tiles + size_t(blockIdx.x % 8) * n_tiles * 8192;
  const int drift = (blockIdx.x / 8) % 8;
  f32x16 c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
  const float one = 1.0f;
  for (int st = 0; st < steps; ++st) {
    float *p = region + size_t((st + drift) % n_tiles) * 8192 + wave * 2048 + lane;
    int issued = 0;
    for (int m = 0; m < mfma_per_step; m += 4) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c[j]) : "v"(a), "v"(b));
        if ((j & 1) && issued < atomics_per_step) {
          asm volatile("global_atomic_add_f32 %0, %1, off" ::"v"(p + 64 * issued), "v"(one) : "memory");
          ++issued;
        }
      }
    }
    for (; issued < atomics_per_step; ++issued)
      asm volatile("global_atomic_add_f32 %0, %1, off" ::"v"(p + 64 * issued), "v"(one) : "memory");
  }
  asm volatile("s_nop 15\n\ts_nop 15" : "+v"(c[0]), "+v"(c[1]), "+v"(c[2]), "+v"(c[3]));
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += (c[0][i] + c[1][i]) + (c[2][i] + c[3][i]);
  sums[size_t(blockIdx.x) * 256 + threadIdx.x] = s;
}

}  // namespace ca

extern "C" int ca_xcd_map(int32_t n_workgroups, int32_t threads_per_workgroup, int32_t *out, void *hip_stream) {
  using namespace ca;
  if (n_workgroups < 0 || n_workgroups > (1 << 24) || threads_per_workgroup < 64 || threads_per_workgroup > 1024 ||
      threads_per_workgroup % 64 != 0) {
    set_error("ca_xcd_map: n_workgroups in 0 .. 2^24, threads_per_workgroup a multiple of 64 in 64 .. 1024");
    return CA_ERR_INVALID_ARG;
  }
  if (n_workgroups == 0) return CA_OK;
  if (!out) {
    set_error("out is null");
    return CA_ERR_INVALID_ARG;
  }
  ca_xcd_map_kernel<<<dim3(unsigned(n_workgroups)), dim3(unsigned(threads_per_workgroup)), 0,
                      static_cast<hipStream_t>(hip_stream)>>>(out);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error(std::string("xcd map launch: ") + hipGetErrorName(e));
    return CA_ERR_HIP;
  }
  return CA_OK;
}

extern "C" int ca_atomic_stream(const void *operands, float *tiles, int32_t n_tiles, int32_t n_workgroups,
                                int32_t steps, int32_t mfma_per_step, int32_t atomics_per_step, float *sums,
                                void *hip_stream) {
  using namespace ca;
  if (n_tiles < 1 || n_tiles > (1 << 16) || n_workgroups < 0 || n_workgroups > (1 << 20) || steps < 0 ||
      steps > (1 << 24) || mfma_per_step < 0 || mfma_per_step > 4096 || mfma_per_step % 4 != 0 ||
      atomics_per_step < 0 || atomics_per_step > 32) {
    set_error("ca_atomic_stream: n_tiles 1 .. 2^16, n_workgroups 0 .. 2^20, steps 0 .. 2^24, mfma_per_step a "
              "multiple of 4 in 0 .. 4096, atomics_per_step 0 .. 32");
    return CA_ERR_INVALID_ARG;
  }
  if (n_workgroups == 0) return CA_OK;
  if (!operands || !tiles || !sums) {
    set_error("operands, tiles or sums is null");
    return CA_ERR_INVALID_ARG;
  }
  ca_atomic_stream_kernel<<<dim3(unsigned(n_workgroups)), 256, 0, static_cast<hipStream_t>(hip_stream)>>>(
      static_cast<const u32x4 *>(operands), tiles, n_tiles, steps, mfma_per_step, atomics_per_step, sums);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error(std::string("atomic stream launch: ") + hipGetErrorName(e));
    return CA_ERR_HIP;
  }
  return CA_OK;
}

extern "C" int ca_mfma_stream(const void *operands, int64_t n_mfma_per_wave, int32_t n_workgroups, int32_t side_work,
                              float *sums, void *hip_stream) {
  using namespace ca;
  std::ostringstream os;
  if (n_mfma_per_wave < 0 || n_mfma_per_wave % CALIB_ROUND != 0 || n_mfma_per_wave / CALIB_ROUND > 0x7fffffff) {
    os << "n_mfma_per_wave " << n_mfma_per_wave << ": must be a non-negative multiple of " << CALIB_ROUND
       << " below 2^37";
    set_error(os.str());
    return CA_ERR_INVALID_ARG;
  }
  if (n_workgroups < 0 || n_workgroups > (1 << 24) || side_work < 0 || side_work > 2) {
    os << "n_workgroups " << n_workgroups << " (0 .. 2^24), side_work " << side_work << " (0, 1 or 2): out of range";
    set_error(os.str());
    return CA_ERR_INVALID_ARG;
  }
  if (n_workgroups == 0) return CA_OK;
  if (!operands || !sums) {
    set_error("operands or sums is null");
    return CA_ERR_INVALID_ARG;
  }
  const dim3 grid{unsigned(n_workgroups)};
  const hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const auto *ops = static_cast<const u32x4 *>(operands);
  const int n_rounds = int(n_mfma_per_wave / CALIB_ROUND);
  if (side_work == 0) ca_mfma_stream_kernel<0><<<grid, 256, 0, st>>>(ops, n_rounds, sums);
  else if (side_work == 1) ca_mfma_stream_kernel<1><<<grid, 256, CALIB_LDS_BYTES, st>>>(ops, n_rounds, sums);
  else ca_mfma_stream_kernel<2><<<grid, 256, CALIB_LDS_BYTES, st>>>(ops, n_rounds, sums);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    os << "mfma stream launch: " << hipGetErrorName(e) << " (" << hipGetErrorString(e) << ")";
    set_error(os.str());
    return CA_ERR_HIP;
  }
  return CA_OK;
}
