// Forward kernel: O = softmax(scale * Q K^T, causal) V and LSE over tiles of query rows
// (core attention, Section 2.1; one fused launch over all CA-tasks, Section 4.1).
//
// One workgroup = one forward unit = 128 query slots of one document x one query head; 4 waves of
// 32 slots.  The wave computes the TRANSPOSED score block S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so
// that a lane owns one query row (column l%32 of the MFMA result) and its 16 registers per block are 16
// different keys: row max and row sum are in-lane work plus one exchange between lanes l and l+32.  The
// bf16 probabilities, still in those registers, are exactly the B operand of O^T += V^T P^T (the key index
// is the contraction index; its order inside a block is the same permutation on both operands).  V^T comes
// out of the natural-layout V tile in LDS through ds_read_b64_tr_b16.  K and V tiles of 64 keys are staged
// through double-buffered LDS; the softmax runs in base 2 with scale*log2(e) folded into one FMA.
#include "ca_device.h"
#include "ca_internal.h"

namespace ca {

template <int D>
struct FwdSmem {
  static constexpr int KSTR = D * 2 + 16;  // K row stride in bytes: odd number of 16-byte chunks
  static constexpr int VSTR = D * 2 + 32;  // V row stride: 4 consecutive rows land in disjoint bank octets
  static constexpr int KBYTES = FWD_BN * KSTR;
  static constexpr int VBYTES = FWD_BN * VSTR;
  static constexpr int STAGE = KBYTES + VBYTES;
  static constexpr int TOTAL = 2 * STAGE;
};

template <int D>
__global__ __launch_bounds__(256, 2) void ca_fwd_kernel(const FwdUnit *__restrict__ units,
                                                        const int32_t *__restrict__ slot_row,
                                                        const int32_t *__restrict__ slot_pos,
                                                        const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                        const bf16_t *__restrict__ V, bf16_t *__restrict__ O,
                                                        float *__restrict__ LSE, int Hq, int Hkv, int64_t total_q,
                                                        float c /* scale * log2(e) */) {
  using S = FwdSmem<D>;
  constexpr int NS = D / 16;   // MFMA k-steps over head_dim
  constexpr int NDB = D / 32;  // 32-row blocks of O^T
  constexpr int CH = D / 8;    // 16-byte chunks per K/V row
  constexpr int RP = 256 / CH; // rows per load pass
  constexpr int NP = FWD_BN / RP;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const FwdUnit u = units[blockIdx.x];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, r = lane & 31;
  const int hk = u.head / (Hq / Hkv);
  const int slot = u.slot0 + wave * 32 + r;
  const int row = slot_row[slot];
  const int pos = slot_pos[slot];
  const int wmax = wave_max(pos), wmin = wave_min(pos);

  // Q fragments: B operand of S^T = K Q^T; lane holds Q[row][16 s + 8 g .. +7]
  bf16x8 qf[NS];
  {
    const bf16_t *qp = Q + (size_t(row < 0 ? 0 : row) * Hq + u.head) * D + 8 * g;
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
  }

  // this thread's share of a K/V tile: chunk lc of rows lr + RP*i
  const int lc = tid % CH, lr = tid / CH;
  const size_t kv_stride = size_t(Hkv) * D;
  const bf16_t *kbase = K + (size_t(u.kv_row0) * Hkv + hk) * D + 8 * lc;
  const bf16_t *vbase = V + (size_t(u.kv_row0) * Hkv + hk) * D + 8 * lc;
  u32x4 kreg[NP], vreg[NP];
  auto load_tile = [&](int j0) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int key = j0 + lr + RP * i;
      if (key < u.n_keys) {
        kreg[i] = *reinterpret_cast<const u32x4 *>(kbase + size_t(key) * kv_stride);
        vreg[i] = *reinterpret_cast<const u32x4 *>(vbase + size_t(key) * kv_stride);
      } else {  // beyond the keys any row of the tile sees: zeros (0 * garbage must stay 0)
        kreg[i] = u32x4{0, 0, 0, 0};
        vreg[i] = u32x4{0, 0, 0, 0};
      }
    }
  };
  auto store_tile = [&](int buf) {
    char *kb = smem + buf * S::STAGE, *vb = kb + S::KBYTES;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      *reinterpret_cast<u32x4 *>(kb + (lr + RP * i) * S::KSTR + 16 * lc) = kreg[i];
      *reinterpret_cast<u32x4 *>(vb + (lr + RP * i) * S::VSTR + 16 * lc) = vreg[i];
    }
  };

  f32x16 acc[NDB];
#pragma unroll
  for (int b = 0; b < NDB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
  float m = -INFINITY, lsum = 0.f;

  const int n_tiles = (u.n_keys + FWD_BN - 1) / FWD_BN;
  load_tile(0);
  store_tile(0);
  __syncthreads();

  // per-lane LDS offsets
  const int k_off = r * S::KSTR + 16 * g;                                         // + 32*s, + 32 rows*KSTR per block
  const int v_off = (4 * g + ((lane & 15) >> 2)) * S::VSTR + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

  for (int j = 0; j < n_tiles; ++j) {
    const int j0 = j * FWD_BN;
    const bool more = j + 1 < n_tiles;
    if (more) load_tile(j0 + FWD_BN);
    if (j0 <= wmax) {
      const char *kb = smem + (j & 1) * S::STAGE, *vb = kb + S::KBYTES;
      f32x16 s0, s1;
#pragma unroll
      for (int i = 0; i < 16; ++i) s0[i] = 0.f, s1[i] = 0.f;
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        bf16x8 a0 = lds_read8(kb + k_off + 32 * s);
        bf16x8 a1 = lds_read8(kb + k_off + 32 * S::KSTR + 32 * s);
        s0 = mfma32(a0, qf[s], s0);
        s1 = mfma32(a1, qf[s], s1);
      }
      if (j0 + FWD_BN - 1 > wmin) {  // some (row, key) of this block is above the diagonal
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = j0 + (i >> 2) * 8 + 4 * g + (i & 3);
          if (key > pos) s0[i] = -INFINITY;
          if (key + 32 > pos) s1[i] = -INFINITY;
        }
      }
      float mx = s0[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s0[i]);
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s1[i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m, mx * c);
      const float alpha = fast_exp2(m - m_new);
      m = m_new;
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        s0[i] = fast_exp2(fmaf(s0[i], c, -m_new));
        s1[i] = fast_exp2(fmaf(s1[i], c, -m_new));
        psum += s0[i] + s1[i];
      }
      lsum = fmaf(lsum, alpha, psum);
#pragma unroll
      for (int b = 0; b < NDB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] *= alpha;
      // P^T as B operands: k-step t of key block kb uses registers 8t .. 8t+7
      bf16x8 pb[4];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        u32x4 w0 = {pack_bf16(s0[8 * t], s0[8 * t + 1]), pack_bf16(s0[8 * t + 2], s0[8 * t + 3]),
                    pack_bf16(s0[8 * t + 4], s0[8 * t + 5]), pack_bf16(s0[8 * t + 6], s0[8 * t + 7])};
        u32x4 w1 = {pack_bf16(s1[8 * t], s1[8 * t + 1]), pack_bf16(s1[8 * t + 2], s1[8 * t + 3]),
                    pack_bf16(s1[8 * t + 4], s1[8 * t + 5]), pack_bf16(s1[8 * t + 6], s1[8 * t + 7])};
        pb[t] = __builtin_bit_cast(bf16x8, w0);
        pb[2 + t] = __builtin_bit_cast(bf16x8, w1);
      }
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) {  // kt = 2*key block + t : keys 16 kt .. 16 kt + 15 of the tile
#pragma unroll
        for (int b = 0; b < NDB; ++b) {
          const char *vp = vb + v_off + (16 * kt) * S::VSTR + 64 * b;
          bf16x8 a = join(lds_read_tr4(vp), lds_read_tr4(vp + 8 * S::VSTR));
          acc[b] = mfma32(a, pb[kt], acc[b]);
        }
      }
    }
    if (more) store_tile((j + 1) & 1);
    __syncthreads();
  }

  // epilogue: O = acc / l (bf16), LSE = ln 2 * (m + log2 l)
  lsum += __shfl_xor(lsum, 32);
  if (row >= 0) {
    const float inv = 1.0f / lsum;
    bf16_t *op = O + (size_t(row) * Hq + u.head) * D + 4 * g;
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        u32x2 w = {pack_bf16(acc[b][4 * q4] * inv, acc[b][4 * q4 + 1] * inv),
                   pack_bf16(acc[b][4 * q4 + 2] * inv, acc[b][4 * q4 + 3] * inv)};
        *reinterpret_cast<u32x2 *>(op + 32 * b + 8 * q4) = w;
      }
    if (g == 0) LSE[size_t(u.head) * total_q + row] = 0.6931471805599453f * (m + fast_log2(lsum));
  }
}

template <int D>
static hipError_t launch_fwd_t(const ca_plan_t *p, const void *q, const void *k, const void *v, void *o, float *lse,
                               hipStream_t st) {
  if (p->fwd_units.empty()) return hipSuccess;
  auto kern = ca_fwd_kernel<D>;
  static bool attr_done[16] = {};
  if (!attr_done[p->device & 15]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       FwdSmem<D>::TOTAL);
    if (e != hipSuccess) return e;
    attr_done[p->device & 15] = true;
  }
  const float c = p->scale * 1.4426950408889634f;
  hipLaunchKernelGGL(kern, dim3(unsigned(p->fwd_units.size())), dim3(256), FwdSmem<D>::TOTAL, st, p->d_fwd_units,
                     p->d_slot_row, p->d_slot_pos, static_cast<const bf16_t *>(q), static_cast<const bf16_t *>(k),
                     static_cast<const bf16_t *>(v), static_cast<bf16_t *>(o), lse, p->hq, p->hkv, p->total_q, c);
  return hipGetLastError();
}

hipError_t launch_fwd(const ca_plan_t *p, const void *q, const void *k, const void *v, void *o, float *lse,
                      hipStream_t st) {
  return p->d == 128 ? launch_fwd_t<128>(p, q, k, v, o, lse, st) : launch_fwd_t<64>(p, q, k, v, o, lse, st);
}

}  // namespace ca
