// Backward kernels: dQ, dK, dV of L = sum(dO * O) with P recomputed from the saved log-sum-exp
// (Section 2.1: P is not stored in forward, it is recomputed during backward).
//
//   prepass : Delta[h][row] = <dO[row,h,:], O[row,h,:]>
//   main    : one workgroup owns 128 keys of one document for one KV head and walks over every block of 64
//             query slots of that document that can see them, for each query head of the KV head's group:
//               S  = Q K^T, dP = dO V^T            (K, V fragments of the wave's 32 keys stay in registers)
//               P  = exp2(c S - log2e LSE) under the causal mask, dS = P (dP - Delta)
//               dV^T += dO^T P, dK^T += Q^T dS     (Q^T, dO^T through ds_read_b64_tr_b16 from the natural tiles)
//               dS^T -> LDS, then dQ += dS K       (all 128 keys; fp32 atomics into the dQ accumulator)
//             dK and dV are written once, summed over the group's heads and over all tasks of the document.
//   finalize: dQ = scale * accumulator -> bf16
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include <algorithm>

#include "ca_device.h"
#include "ca_internal.h"

namespace ca {

template <int D>
struct BwdSmem {
  static constexpr int TS = D * 2 + 32;          // row stride of the K, Q and dO tiles (bytes)
  static constexpr int DS = BWD_BQ * 2 + 32;     // row stride of dS^T [key][q]
  static constexpr int K_OFF = 0;
  static constexpr int Q_OFF = K_OFF + BWD_BN * TS;
  static constexpr int DO_OFF = Q_OFF + BWD_BQ * TS;
  static constexpr int DS_OFF = DO_OFF + BWD_BQ * TS;
  static constexpr int L2_OFF = DS_OFF + BWD_BN * DS;   // log2e * LSE per slot of the block
  static constexpr int DL_OFF = L2_OFF + BWD_BQ * 4;    // Delta
  static constexpr int POS_OFF = DL_OFF + BWD_BQ * 4;   // document position, -1 for padding
  static constexpr int ROW_OFF = POS_OFF + BWD_BQ * 4;  // packed Q row, -1 for padding
  static constexpr int TOTAL = ROW_OFF + BWD_BQ * 4;
};

__global__ void ca_bwd_delta_kernel(const bf16_t *__restrict__ O, const bf16_t *__restrict__ dO,
                                    float *__restrict__ delta, int64_t total_q, int Hq, int D) {
  // D/8 lanes per (row, head); a wave covers 64 / (D/8) pairs
  const int lanes = D / 8;
  const int64_t idx = (int64_t(blockIdx.x) * blockDim.x + threadIdx.x);
  const int64_t pair = idx / lanes;
  const int c = int(idx % lanes);
  float s = 0.f;
  const bool ok = pair < total_q * Hq;
  if (ok) {
    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(O + pair * D + 8 * c);
    const bf16x8 b = *reinterpret_cast<const bf16x8 *>(dO + pair * D + 8 * c);
#pragma unroll
    for (int i = 0; i < 8; ++i) s += float(a[i]) * float(b[i]);
  }
  for (int o = lanes / 2; o > 0; o >>= 1) s += __shfl_xor(s, o);
  if (ok && c == 0) {
    const int64_t row = pair / Hq;
    const int h = int(pair % Hq);
    delta[int64_t(h) * total_q + row] = s;
  }
}

__global__ void ca_fill_zero_kernel(u32x4 *__restrict__ p, int64_t n16) {
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = u32x4{0, 0, 0, 0};
}

__global__ void ca_bwd_dq_finalize_kernel(const float *__restrict__ acc, bf16_t *__restrict__ dq, int64_t n8,
                                          float scale) {
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n8; i += stride) {
    const f32x4 a = *reinterpret_cast<const f32x4 *>(acc + 8 * i);
    const f32x4 b = *reinterpret_cast<const f32x4 *>(acc + 8 * i + 4);
    u32x4 w = {pack_bf16(a[0] * scale, a[1] * scale), pack_bf16(a[2] * scale, a[3] * scale),
               pack_bf16(b[0] * scale, b[1] * scale), pack_bf16(b[2] * scale, b[3] * scale)};
    *reinterpret_cast<u32x4 *>(dq + 8 * i) = w;
  }
}

template <int D>
__global__ __launch_bounds__(256, 1) void ca_bwd_kernel(const BwdUnit *__restrict__ units,
                                                        const int32_t *__restrict__ slot_row,
                                                        const int32_t *__restrict__ slot_pos,
                                                        const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                        const bf16_t *__restrict__ V, const bf16_t *__restrict__ dO,
                                                        const float *__restrict__ LSE, const float *__restrict__ delta,
                                                        float *__restrict__ dq_acc, bf16_t *__restrict__ dK,
                                                        bf16_t *__restrict__ dV, int Hq, int Hkv, int64_t total_q,
                                                        float scale) {
  using S = BwdSmem<D>;
  constexpr int NS = D / 16, NDB = D / 32, CH = D / 8, RP = 256 / CH, NPQ = BWD_BQ / RP, NPK = BWD_BN / RP;
  constexpr int NDQ = NDB / 2;  // dQ output blocks per wave in the second phase
  constexpr float LOG2E = 1.4426950408889634f;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const BwdUnit u = units[blockIdx.x];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, r = lane & 31;
  const int li = lane & 15, dh = (lane >> 4) & 1;
  const int G = Hq / Hkv, hk = u.kv_head;
  const int kw0 = 32 * wave;
  const float c = scale * LOG2E;
  const size_t kv_stride = size_t(Hkv) * D;

  // resident K, V fragments of the wave's 32 keys (B operands of S = Q K^T and dP = dO V^T)
  bf16x8 kf[NS], vf[NS];
  {
    const bool ok = kw0 + r < u.n_valid;
    const size_t off = (size_t(u.kv_row + kw0 + r) * Hkv + hk) * D + 8 * g;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (ok) {
        kf[s] = *reinterpret_cast<const bf16x8 *>(K + off + 16 * s);
        vf[s] = *reinterpret_cast<const bf16x8 *>(V + off + 16 * s);
      } else {
        kf[s] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
        vf[s] = kf[s];
      }
    }
  }
  // the whole K tile in LDS (B operand of dQ = dS K through transposing reads)
  const int lc = tid % CH, lr = tid / CH;
#pragma unroll
  for (int i = 0; i < NPK; ++i) {
    const int key = lr + RP * i;
    u32x4 w = {0, 0, 0, 0};
    if (key < u.n_valid) w = *reinterpret_cast<const u32x4 *>(K + (size_t(u.kv_row + key) * Hkv + hk) * D + 8 * lc);
    *reinterpret_cast<u32x4 *>(smem + S::K_OFF + key * S::TS + 16 * lc) = w;
  }

  f32x16 acc_dk[NDB], acc_dv[NDB];
#pragma unroll
  for (int b = 0; b < NDB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc_dk[b][i] = 0.f, acc_dv[b][i] = 0.f;

  const int n_blocks = (u.slot_end - u.slot_begin) / BWD_BQ;
  const int n_it = n_blocks * G;
  const int key_pos = u.key_pos0 + kw0 + r;  // document position of this lane's key

  // staging registers for the next (q block, head)
  u32x4 qreg[NPQ], doreg[NPQ];
  float l2reg = 0.f, dlreg = 0.f;
  int posreg = -1, rowreg = -1;
  auto load_block = [&](int it) {
    const int blk = it / G, h = hk * G + it % G;
    const int s0 = u.slot_begin + blk * BWD_BQ;
#pragma unroll
    for (int i = 0; i < NPQ; ++i) {
      const int row = slot_row[s0 + lr + RP * i];
      if (row >= 0) {
        const size_t off = (size_t(row) * Hq + h) * D + 8 * lc;
        qreg[i] = *reinterpret_cast<const u32x4 *>(Q + off);
        doreg[i] = *reinterpret_cast<const u32x4 *>(dO + off);
      } else {
        qreg[i] = u32x4{0, 0, 0, 0};
        doreg[i] = u32x4{0, 0, 0, 0};
      }
    }
    if (tid < BWD_BQ) {
      rowreg = slot_row[s0 + tid];
      posreg = rowreg >= 0 ? slot_pos[s0 + tid] : -1;
      l2reg = rowreg >= 0 ? LSE[size_t(h) * total_q + rowreg] * LOG2E : 0.f;
      dlreg = rowreg >= 0 ? delta[size_t(h) * total_q + rowreg] : 0.f;
    }
  };
  auto store_block = [&]() {
#pragma unroll
    for (int i = 0; i < NPQ; ++i) {
      *reinterpret_cast<u32x4 *>(smem + S::Q_OFF + (lr + RP * i) * S::TS + 16 * lc) = qreg[i];
      *reinterpret_cast<u32x4 *>(smem + S::DO_OFF + (lr + RP * i) * S::TS + 16 * lc) = doreg[i];
    }
    if (tid < BWD_BQ) {
      reinterpret_cast<float *>(smem + S::L2_OFF)[tid] = l2reg;
      reinterpret_cast<float *>(smem + S::DL_OFF)[tid] = dlreg;
      reinterpret_cast<int *>(smem + S::POS_OFF)[tid] = posreg;
      reinterpret_cast<int *>(smem + S::ROW_OFF)[tid] = rowreg;
    }
  };

  if (n_it > 0) load_block(0);
  for (int it = 0; it < n_it; ++it) {
    __syncthreads();  // everyone is done with the previous block's tiles
    store_block();
    __syncthreads();
    if (it + 1 < n_it) load_block(it + 1);
    const int h = hk * G + it % G;

    // ---- phase 1: scores of the wave's 32 keys against the 64 slots
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 sacc, pacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[i] = 0.f, pacc[i] = 0.f;
      const char *qt = smem + S::Q_OFF + (32 * qb + r) * S::TS + 16 * g;
      const char *dot = smem + S::DO_OFF + (32 * qb + r) * S::TS + 16 * g;
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        sacc = mfma32(lds_read8(qt + 32 * s), kf[s], sacc);
        pacc = mfma32(lds_read8(dot + 32 * s), vf[s], pacc);
      }
      uint32_t pw[8], dw[8];
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int qo = (32 * qb + 8 * i4 + 4 * g) * 4;
        const f32x4 l2v = *reinterpret_cast<const f32x4 *>(smem + S::L2_OFF + qo);
        const f32x4 dlv = *reinterpret_cast<const f32x4 *>(smem + S::DL_OFF + qo);
        const int4 pv = *reinterpret_cast<const int4 *>(smem + S::POS_OFF + qo);
        const int pos4[4] = {pv.x, pv.y, pv.z, pv.w};
        float p[4], ds[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * i4 + e;
          p[e] = key_pos <= pos4[e] ? fast_exp2(fmaf(sacc[i], c, -l2v[e])) : 0.f;
          ds[e] = p[e] * (pacc[i] - dlv[e]);
        }
        pw[2 * i4] = pack_bf16(p[0], p[1]);
        pw[2 * i4 + 1] = pack_bf16(p[2], p[3]);
        dw[2 * i4] = pack_bf16(ds[0], ds[1]);
        dw[2 * i4 + 1] = pack_bf16(ds[2], ds[3]);
        *reinterpret_cast<u32x2 *>(smem + S::DS_OFF + (kw0 + r) * S::DS + (32 * qb + 8 * i4 + 4 * g) * 2) =
            u32x2{dw[2 * i4], dw[2 * i4 + 1]};
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pb = __builtin_bit_cast(bf16x8, u32x4{pw[4 * t], pw[4 * t + 1], pw[4 * t + 2], pw[4 * t + 3]});
        const bf16x8 db = __builtin_bit_cast(bf16x8, u32x4{dw[4 * t], dw[4 * t + 1], dw[4 * t + 2], dw[4 * t + 3]});
        const int trow = 32 * qb + 16 * t + 4 * g + (li >> 2);
#pragma unroll
        for (int b = 0; b < NDB; ++b) {
          const int off = trow * S::TS + (32 * b + 16 * dh + 4 * (li & 3)) * 2;
          const bf16x8 dot_t = join(lds_read_tr4(smem + S::DO_OFF + off), lds_read_tr4(smem + S::DO_OFF + off + 8 * S::TS));
          acc_dv[b] = mfma32(dot_t, pb, acc_dv[b]);
          const bf16x8 q_t = join(lds_read_tr4(smem + S::Q_OFF + off), lds_read_tr4(smem + S::Q_OFF + off + 8 * S::TS));
          acc_dk[b] = mfma32(q_t, db, acc_dk[b]);
        }
      }
    }
    __syncthreads();  // dS^T of all 128 keys is in LDS

    // ---- phase 2: dQ of the 64 slots; wave -> (q sub-block wave&1, NDQ column blocks)
    {
      const int qb = wave & 1;
      f32x16 dq[NDQ];
#pragma unroll
      for (int x = 0; x < NDQ; ++x)
#pragma unroll
        for (int i = 0; i < 16; ++i) dq[x][i] = 0.f;
#pragma unroll
      for (int kt = 0; kt < BWD_BN / 16; ++kt) {
        const int krow = 16 * kt + 8 * g + (li >> 2);
        const char *ap = smem + S::DS_OFF + krow * S::DS + (32 * qb + 16 * dh + 4 * (li & 3)) * 2;
        const bf16x8 a = join(lds_read_tr4(ap), lds_read_tr4(ap + 4 * S::DS));
#pragma unroll
        for (int x = 0; x < NDQ; ++x) {
          const int b = (wave >> 1) * NDQ + x;
          const char *bp = smem + S::K_OFF + krow * S::TS + (32 * b + 16 * dh + 4 * (li & 3)) * 2;
          const bf16x8 kb = join(lds_read_tr4(bp), lds_read_tr4(bp + 4 * S::TS));
          dq[x] = mfma32(a, kb, dq[x]);
        }
      }
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int4 rv = *reinterpret_cast<const int4 *>(smem + S::ROW_OFF + (32 * qb + 8 * i4 + 4 * g) * 4);
        const int row4[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (row4[e] < 0) continue;
          float *dst = dq_acc + (size_t(row4[e]) * Hq + h) * D + r;
#pragma unroll
          for (int x = 0; x < NDQ; ++x) unsafeAtomicAdd(dst + 32 * ((wave >> 1) * NDQ + x), dq[x][4 * i4 + e]);
        }
      }
    }
  }

  // ---- write dK (scaled) and dV of the wave's 32 keys
  if (kw0 + r < u.n_valid) {
    const size_t off = (size_t(u.kv_row + kw0 + r) * Hkv + hk) * D + 4 * g;
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        u32x2 wk = {pack_bf16(acc_dk[b][4 * q4] * scale, acc_dk[b][4 * q4 + 1] * scale),
                    pack_bf16(acc_dk[b][4 * q4 + 2] * scale, acc_dk[b][4 * q4 + 3] * scale)};
        u32x2 wv = {pack_bf16(acc_dv[b][4 * q4], acc_dv[b][4 * q4 + 1]),
                    pack_bf16(acc_dv[b][4 * q4 + 2], acc_dv[b][4 * q4 + 3])};
        *reinterpret_cast<u32x2 *>(dK + off + 32 * b + 8 * q4) = wk;
        *reinterpret_cast<u32x2 *>(dV + off + 32 * b + 8 * q4) = wv;
      }
  }
}

static void launch_fill(void *p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return;
  const int64_t n16 = int64_t(bytes / 16);
  const unsigned blocks = unsigned(std::min<int64_t>((n16 + 255) / 256, 256 * 32));
  hipLaunchKernelGGL(ca_fill_zero_kernel, dim3(blocks), dim3(256), 0, st, static_cast<u32x4 *>(p), n16);
}

template <int D>
static hipError_t launch_bwd_t(const ca_plan_t *p, const void *q, const void *k, const void *v, const void *o,
                               const void *d_o, const float *lse, void *dq, void *dk, void *dv, void *ws,
                               hipStream_t st) {
  const size_t q_elems = size_t(p->total_q) * p->hq * D, kv_elems = size_t(p->total_kv) * p->hkv * D;
  float *dq_acc = static_cast<float *>(ws);
  float *delta = reinterpret_cast<float *>(static_cast<char *>(ws) + p->ws_off_delta);
  // every dK/dV row is written: rows no unit owns stay zero
  launch_fill(dk, kv_elems * 2, st);
  launch_fill(dv, kv_elems * 2, st);
  if (q_elems == 0) return hipGetLastError();
  launch_fill(dq_acc, q_elems * 4, st);
  {
    const int64_t threads = int64_t(p->total_q) * p->hq * (D / 8);
    hipLaunchKernelGGL(ca_bwd_delta_kernel, dim3(unsigned((threads + 255) / 256)), dim3(256), 0, st,
                       static_cast<const bf16_t *>(o), static_cast<const bf16_t *>(d_o), delta, p->total_q, p->hq, D);
  }
  if (!p->bwd_units.empty()) {
    auto kern = ca_bwd_kernel<D>;
    static bool attr_done[16] = {};
    if (!attr_done[p->device & 15]) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, BwdSmem<D>::TOTAL);
      if (e != hipSuccess) return e;
      attr_done[p->device & 15] = true;
    }
    hipLaunchKernelGGL(kern, dim3(unsigned(p->bwd_units.size())), dim3(256), BwdSmem<D>::TOTAL, st, p->d_bwd_units,
                       p->d_slot_row, p->d_slot_pos, static_cast<const bf16_t *>(q), static_cast<const bf16_t *>(k),
                       static_cast<const bf16_t *>(v), static_cast<const bf16_t *>(d_o), lse, delta, dq_acc,
                       static_cast<bf16_t *>(dk), static_cast<bf16_t *>(dv), p->hq, p->hkv, p->total_q, p->scale);
  }
  {
    const int64_t n8 = int64_t(q_elems / 8);
    const unsigned blocks = unsigned(std::min<int64_t>((n8 + 255) / 256, 256 * 32));
    hipLaunchKernelGGL(ca_bwd_dq_finalize_kernel, dim3(blocks), dim3(256), 0, st, dq_acc, static_cast<bf16_t *>(dq), n8,
                       p->scale);
  }
  return hipGetLastError();
}

hipError_t launch_bwd(const ca_plan_t *p, const void *q, const void *k, const void *v, const void *o, const void *d_o,
                      const float *lse, void *dq, void *dk, void *dv, void *ws, hipStream_t st) {
  return p->d == 128 ? launch_bwd_t<128>(p, q, k, v, o, d_o, lse, dq, dk, dv, ws, st)
                     : launch_bwd_t<64>(p, q, k, v, o, d_o, lse, dq, dk, dv, ws, st);
}

}  // namespace ca
