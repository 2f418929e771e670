// Forward kernel: O = softmax(scale * Q K^T, causal) V and LSE over tiles of query rows
// (core attention, Section 2.1; one fused launch over all CA-tasks, Section 4.1).
//
// One workgroup = one forward unit = 256 query slots of one document x one query head; 8 waves of
// 32 slots, two per SIMD, one workgroup per CU.  The wave computes the TRANSPOSED score block S^T = K Q^T with
// v_mfma_f32_32x32x16_bf16, so that a lane owns one query row (column l%32 of the MFMA result) and its 16
// registers per block are 16 different keys: row max and row sum are in-lane work plus one exchange
// between lanes l and l+32.  The bf16 probabilities, still in those registers, are exactly the B operand of
// O^T += V^T P^T (the key index is the contraction index; its order inside a block is the same permutation
// on both operands).  V^T comes out of the natural-layout V tile in LDS through ds_read_b64_tr_b16.
//
// K and V tiles of 64 keys go from global memory straight into swizzled LDS tiles (global_load_lds), four
// stages each, fetched three tiles ahead.  Per tile a wave does three things: the scores of tile j+1
// (matrix pipe), the softmax of tile j (vector ALU), and P V of tile j (matrix pipe).  Waves 0-3 run them in
// that order, waves 4-7 (their SIMD partners) run softmax, P V, scores: at any moment the two waves of a SIMD
// are in different phases, so the vector work of one hides behind the matrix work of the other.  The softmax
// runs in base 2 with scale*log2(e) folded into one FMA and rescales the accumulators lazily.
#include <type_traits>

#include "ca_device.h"
#include "ca_internal.h"

namespace ca {

template <int D>
struct FwdSmem {
  static constexpr int NST = 4;                // stages of K and of V
  static constexpr int TILE = FWD_BN * 2 * D;  // one K or V tile
  static constexpr int K_OFF = 0;
  static constexpr int V_OFF = NST * TILE;
  static constexpr int TOTAL = 2 * NST * TILE;
};

template <int D>
__global__ __launch_bounds__(512, 2) void ca_fwd_kernel(const FwdUnit *__restrict__ units,
                                                        const int32_t *__restrict__ slot_row,
                                                        const int32_t *__restrict__ slot_pos,
                                                        const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                        const bf16_t *__restrict__ V, bf16_t *__restrict__ O,
                                                        float *__restrict__ LSE, int Hq, int Hkv, int64_t total_q,
                                                        float c /* scale * log2(e) */) {
  using S = FwdSmem<D>;
  constexpr int NS = D / 16;       // MFMA k-steps over head_dim
  constexpr int NDB = D / 32;      // 32-row blocks of O^T
  constexpr int CH = D / 8;        // 16-byte chunks per row
  constexpr int RPI = 64 / CH;     // rows covered by one wave-wide direct load (1 KB)
  constexpr int NLD = FWD_BN / (8 * RPI);  // direct loads per wave per tile
  constexpr int NST = S::NST;
  constexpr int ROWB = 2 * D;
  constexpr float RESCALE_LOG2 = 8.0f;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const FwdUnit u = units[blockIdx.x];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, r = lane & 31;
  const int group = wave >> 2;  // 0: scores first, 1: scores last
  const int li = lane & 15, dh = (lane >> 4) & 1;
  const int hk = u.head / (Hq / Hkv);
  const int slot = u.slot0 + wave * 32 + r;
  const int row = slot_row[slot];
  const int pos = slot_pos[slot];
  const int wmax = wave_max(pos), wmin = wave_min(pos);
  const int n_tiles = (u.n_keys + FWD_BN - 1) / FWD_BN;

  // ---- direct global -> LDS tile loads.  Load n of this wave covers tile rows RPI*(wave + 8n) .. +RPI-1;
  // lane i fills physical chunk i % CH of row i / CH, so it fetches logical chunk (i % CH) ^ sw(row).
  const int ld_rr = lane / CH;
  const int ld_row0 = RPI * wave + ld_rr;  // + 8*RPI*n
  const int ld_chunk = (lane % CH) ^ tile_sw<D>(ld_row0);
  const size_t kv_stride = size_t(Hkv) * D;
  const bf16_t *kg = K + (size_t(u.kv_row0) * Hkv + hk) * D + 8 * ld_chunk;
  const bf16_t *vg = V + (size_t(u.kv_row0) * Hkv + hk) * D + 8 * ld_chunk;
  const int last_key = u.n_keys - 1;
  // Tiles past the end are fetched too (clamped to the last key), so that every iteration issues the same
  // number of loads and the s_waitcnt bookkeeping stays constant.
  auto issue_kv = [&](const bf16_t *src, int area, int tile) {
    char *dst = smem + area + (tile % NST) * S::TILE + 1024 * wave;
#pragma unroll
    for (int n = 0; n < NLD; ++n) {
      const int key = min(tile * FWD_BN + ld_row0 + 8 * RPI * n, last_key);  // rows past the last key are masked later
      load_lds16(src + size_t(key) * kv_stride, dst + 8192 * n);
    }
  };

  issue_kv(kg, S::K_OFF, 0);
  issue_kv(vg, S::V_OFF, 0);
  issue_kv(kg, S::K_OFF, 1);
  issue_kv(vg, S::V_OFF, 1);
  issue_kv(kg, S::K_OFF, 2);
  issue_kv(vg, S::V_OFF, 2);
  issue_kv(kg, S::K_OFF, 3);

  // Q fragments: B operand of S^T = K Q^T; lane holds Q[row][16 s + 8 g .. +7]
  bf16x8 qf[NS];
  {
    const bf16_t *qp = Q + (size_t(row < 0 ? 0 : row) * Hq + u.head) * D + 8 * g;
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
  }

  // per-lane LDS read offsets inside a tile
  int koff[NS];  // K fragment s of key row r (second key block: + 32 rows)
#pragma unroll
  for (int s = 0; s < NS; ++s) koff[s] = tile_off<D>(r, 2 * s + g);
  int voff[2][NDB];  // transposing reads of V: rows 4g + li/4 (+8), 16 head-dim columns of block b
#pragma unroll
  for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
    for (int b = 0; b < NDB; ++b)
      voff[h2][b] = tile_off<D>(4 * g + (li >> 2) + 8 * h2, 4 * b + 2 * dh + ((li >> 1) & 1)) + 8 * (li & 1);

  f32x16 acc[NDB];
#pragma unroll
  for (int b = 0; b < NDB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
  float m = -INFINITY, lsum = 0.f;

  // scores of one tile: two 32-key blocks
  auto scores = [&](const char *kt, f32x16 &s0, f32x16 &s1) {
    bf16x8 ka[NS];
#pragma unroll
    for (int i = 0; i < 16; ++i) s0[i] = 0.f, s1[i] = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s) ka[s] = lds_read8(kt + koff[s]);
#pragma unroll
    for (int s = 0; s < NS; ++s) s0 = mfma32(ka[s], qf[s], s0);
#pragma unroll
    for (int s = 0; s < NS; ++s) ka[s] = lds_read8(kt + koff[s] + 32 * ROWB);
#pragma unroll
    for (int s = 0; s < NS; ++s) s1 = mfma32(ka[s], qf[s], s1);
  };

  f32x16 n0, n1;  // scores of the next tile
  // Everything issued so far has landed, including the Q fragments: from here on the compiler places no
  // vector-memory waits inside the loop (they would drain the direct-load queue every iteration).
  wait_vmcnt<0>();
#pragma unroll
  for (int s = 0; s < NS; ++s) pin(qf[s]);
  barrier_nofence();
  scores(smem + S::K_OFF, n0, n1);

  auto softmax_pv = [&](int j, f32x16 s0, f32x16 s1) {
    const int j0 = j * FWD_BN;
    if (j0 + FWD_BN - 1 > wmin) {  // some (row, key) of this tile is above the diagonal
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
    // Lazy rescaling: the running reference m only moves when some row's maximum has grown by more than
    // 2^RESCALE_LOG2; until then probabilities are taken relative to the stale m (they stay below
    // 2^RESCALE_LOG2, harmless in fp32 and bf16) and the accumulators need no multiply.
    const float m_cand = fmaxf(m, mx * c);
    if (__any(m_cand > m + RESCALE_LOG2)) {
      const float alpha = m == -INFINITY ? 0.f : fast_exp2(m - m_cand);
      m = m_cand;
      lsum *= alpha;
#pragma unroll
      for (int b = 0; b < NDB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] *= alpha;
    }
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      s0[i] = fast_exp2(fmaf(s0[i], c, -m));
      s1[i] = fast_exp2(fmaf(s1[i], c, -m));
      psum += s0[i] + s1[i];
    }
    lsum += psum;
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
    const char *vt = smem + S::V_OFF + (j % NST) * S::TILE;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {  // keys 16 kt .. 16 kt + 15 of the tile
#pragma unroll
      for (int b = 0; b < NDB; ++b) {
        bf16x8 a = join(lds_read_tr4(vt + voff[0][b] + 16 * kt * ROWB), lds_read_tr4(vt + voff[1][b] + 16 * kt * ROWB));
        acc[b] = mfma32(a, pb[kt], acc[b]);
      }
    }
    // The first rows of a document see a handful of keys, their output is as large as a single V row, and
    // the 2^-9 relative rounding of P to bf16 then shows up at the 1e-2 level next to the output's own bf16
    // rounding.  For the waves that hold such rows, the rounding residue of P is fed through the matrix pipe
    // as a second bf16 operand (P = hi + lo), which makes P V as good as fp32 at negligible cost: it
    // happens only in the first tile of the first query rows of each document.
    if (j == 0 && wmin < FWD_BN) {
      bf16x8 pl[4];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        uint32_t l0[4], l1[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t h0 = __builtin_bit_cast(u32x4, pb[t])[e], h1 = __builtin_bit_cast(u32x4, pb[2 + t])[e];
          l0[e] = pack_bf16(s0[8 * t + 2 * e] - __uint_as_float(h0 << 16),
                            s0[8 * t + 2 * e + 1] - __uint_as_float(h0 & 0xffff0000u));
          l1[e] = pack_bf16(s1[8 * t + 2 * e] - __uint_as_float(h1 << 16),
                            s1[8 * t + 2 * e + 1] - __uint_as_float(h1 & 0xffff0000u));
        }
        pl[t] = __builtin_bit_cast(bf16x8, u32x4{l0[0], l0[1], l0[2], l0[3]});
        pl[2 + t] = __builtin_bit_cast(bf16x8, u32x4{l1[0], l1[1], l1[2], l1[3]});
      }
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
        for (int b = 0; b < NDB; ++b) {
          bf16x8 a = join(lds_read_tr4(vt + voff[0][b] + 16 * kt * ROWB), lds_read_tr4(vt + voff[1][b] + 16 * kt * ROWB));
          acc[b] = mfma32(a, pl[kt], acc[b]);
        }
      }
    }
  };

  for (int j = 0; j < n_tiles; ++j) {
    const int j0 = j * FWD_BN;
    const f32x16 s0 = n0, s1 = n1;
    // this wave's parts of K(j+1) and V(j) have landed: only the loads of the last two iterations
    // (tiles j+2, j+3 of V and j+3, j+4 of K) may still be in flight
    wait_vmcnt<4 * NLD>();
    barrier_nofence();  // ... and everybody else's; everybody is done with K(j) and V(j-1)
    issue_kv(vg, S::V_OFF, j + 3);
    issue_kv(kg, S::K_OFF, j + 4);
    const bool next = j + 1 < n_tiles && j0 + FWD_BN <= wmax;
    const char *kn = smem + S::K_OFF + ((j + 1) % NST) * S::TILE;
    if (group == 0) {
      if (next) scores(kn, n0, n1);
      if (j0 <= wmax) softmax_pv(j, s0, s1);
    } else {
      if (j0 <= wmax) softmax_pv(j, s0, s1);
      if (next) scores(kn, n0, n1);
    }
  }
  wait_vmcnt<0>();  // nothing may still be writing LDS when the workgroup ends

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
  hipLaunchKernelGGL(kern, dim3(unsigned(p->fwd_units.size())), dim3(512), FwdSmem<D>::TOTAL, st, p->d_fwd_units,
                     p->d_slot_row, p->d_slot_pos, static_cast<const bf16_t *>(q), static_cast<const bf16_t *>(k),
                     static_cast<const bf16_t *>(v), static_cast<bf16_t *>(o), lse, p->hq, p->hkv, p->total_q, c);
  return hipGetLastError();
}

hipError_t launch_fwd(const ca_plan_t *p, const void *q, const void *k, const void *v, void *o, float *lse,
                      hipStream_t st) {
  return p->d == 128 ? launch_fwd_t<128>(p, q, k, v, o, lse, st) : launch_fwd_t<64>(p, q, k, v, o, lse, st);
}

}  // namespace ca
