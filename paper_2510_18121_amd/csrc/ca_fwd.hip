// Forward kernel: O = softmax(scale * Q K^T, causal) V and LSE over tiles of query rows
// (core attention, Section 2.1; one fused launch over all CA-tasks, Section 4.1).
//
// One workgroup = one forward unit = 256 query slots of one document x one query head, or, for the slots a
// document has left over after its full tiles, 256/hp slots x hp query heads of one KV group (same K/V tiles,
// same loads; only the wave -> (slot group, head) mapping differs); 8 waves of 32 slots, two per SIMD, one
// workgroup per CU.  The wave computes the TRANSPOSED score block S^T = K Q^T
// with v_mfma_f32_32x32x16_bf16, so that a lane owns one query row (column l%32 of the MFMA result) and its
// 16 registers per block are 16 different keys: row max and row sum are in-lane work plus one exchange
// between lanes l and l+32.  The bf16 probabilities, still in those registers, are exactly the B operand of
// O^T += V^T P^T (the key index is the contraction index; its order inside a block is the same permutation
// on both operands).  V^T comes out of the natural-layout V tile in LDS through ds_read_b64_tr_b16.
//
// K and V tiles of 64 keys go from global memory straight into swizzled LDS tiles (global_load_lds), four
// stages each, fetched three tiles ahead.  The loop is software-pipelined inside the wave at the granularity
// of 32-key blocks: a step holds the scores of one block (computed one step earlier) and, in ONE basic block,
// issues the MFMAs of the next block's scores, the exponentials of this block, the MFMAs of this block's P V
// and the row maximum of the next block, so that the vector work sits in the instruction stream between
// independent matrix instructions.  That straight-line form is used for tiles entirely below the diagonal of
// the wave's rows; diagonal tiles take a general path with masking.  The softmax runs in base 2 with
// scale*log2(e) folded into one FMA and rescales the accumulators lazily.
#include <atomic>
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
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void ca_fwd_kernel(const FwdUnit *__restrict__ units,
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
  const uint32_t lds0 = (uint32_t)(uintptr_t)(CA_LDS char *)smem;  // LDS byte address of the dynamic segment

  const FwdUnit u = units[blockIdx.x];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, r = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, dh = (lane >> 4) & 1;
  const int hk = u.head / (Hq / Hkv);
  // wave -> (32-slot group, query head) inside the unit: hp = 1 for a full tile, > 1 for a head-packed unit
  const int hp_lg = __builtin_ctz(u.hp);
  const int head = u.head + (wave & (u.hp - 1));
  const int slot = u.slot0 + (wave >> hp_lg) * 32 + r;
  const int row = slot_row[slot];
  const int pos = slot_pos[slot];
  const int wmax = wave_max(pos), wmin = wave_min(pos);
  const int n_tiles = (u.n_keys + FWD_BN - 1) / FWD_BN;
  // tiles j < n_fast: tile j and the first 32 keys of tile j+1 are entirely visible to every row of this wave
  const int n_fast = max(0, (wmin - 31) / FWD_BN);

  // ---- direct global -> LDS tile loads.  Load n of this wave covers tile rows RPI*(wave + 8n) .. +RPI-1;
  // lane i fills physical chunk i % CH of row i / CH, so it fetches logical chunk (i % CH) ^ sw(row).
  // The address is (scalar tile base) + (per-lane 32-bit offset): advancing to the next tile costs no
  // vector instruction.  Tiles past the end are fetched too (as the last tile, rows clamped to the last key),
  // so that every iteration issues the same number of loads and the s_waitcnt bookkeeping stays constant.
  const uint32_t kv_row_bytes = uint32_t(Hkv) * D * 2;
  const int ld_row0 = RPI * wave + lane / CH;  // + 8*RPI*n
  const uint32_t ld_cbytes = uint32_t((lane % CH) ^ tile_sw<D>(ld_row0)) * 16;
  const int last_tile = n_tiles - 1, last_key_in_tile = u.n_keys - 1 - last_tile * FWD_BN;
  uint32_t ld_off[NLD], ld_off_last[NLD];
#pragma unroll
  for (int n = 0; n < NLD; ++n) {
    ld_off[n] = uint32_t(ld_row0 + 8 * RPI * n) * kv_row_bytes + ld_cbytes;
    ld_off_last[n] = uint32_t(min(ld_row0 + 8 * RPI * n, last_key_in_tile)) * kv_row_bytes + ld_cbytes;
  }
  const char *kg = reinterpret_cast<const char *>(K + (size_t(u.kv_row0) * Hkv + hk) * D);
  const char *vg = reinterpret_cast<const char *>(V + (size_t(u.kv_row0) * Hkv + hk) * D);
  const size_t tile_bytes = size_t(FWD_BN) * kv_row_bytes;
  auto issue_kv = [&](const char *src, int area, int tile) __attribute__((always_inline)) {
    const bool last = tile >= last_tile;
    const char *base = src + size_t(last ? last_tile : tile) * tile_bytes;
    const uint32_t dst = lds0 + uint32_t(area + (tile % NST) * S::TILE + 1024 * wave);
#pragma unroll
    for (int n = 0; n < NLD; ++n) load_lds16_sbase(base, last ? ld_off_last[n] : ld_off[n], dst + 8192 * n);
  };

  issue_kv(kg, S::K_OFF, 0);
  issue_kv(vg, S::V_OFF, 0);
  issue_kv(kg, S::K_OFF, 1);
  issue_kv(vg, S::V_OFF, 1);
  issue_kv(kg, S::K_OFF, 2);
  issue_kv(vg, S::V_OFF, 2);

  // Q fragments: B operand of S^T = K Q^T; lane holds Q[row][16 s + 8 g .. +7]
  bf16x8 qf[NS];
  {
    const bf16_t *qp = Q + (size_t(row < 0 ? 0 : row) * Hq + head) * D + 8 * g;
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
  }

  // per-lane LDS read addresses into the CURRENT stage of K (koff) and of V (voff), advanced once per tile: every
  // LDS read is (loop-carried register) + (immediate block offset)
  uint32_t koff[NS];  // K fragment s of key row r (second key block: + 32 rows)
#pragma unroll
  for (int s = 0; s < NS; ++s) koff[s] = lds0 + uint32_t(S::K_OFF + tile_off<D>(r, 2 * s + g));
  uint32_t voff[2][NDB];  // transposing reads of V: rows 4g + li/4 (+8), 16 head-dim columns of block b
#pragma unroll
  for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
    for (int b = 0; b < NDB; ++b)
      voff[h2][b] = lds0 + uint32_t(S::V_OFF + tile_off<D>(4 * g + (li >> 2) + 8 * h2, 4 * b + 2 * dh + ((li >> 1) & 1)) +
                             8 * (li & 1));

  f32x16 acc[NDB];
#pragma unroll
  for (int b = 0; b < NDB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
  float m = -INFINITY, lsum = 0.f;

  auto advance_k = [&](int j) __attribute__((always_inline)) {
    const int adv = (j % NST) == NST - 1 ? -(NST - 1) * S::TILE : S::TILE;
#pragma unroll
    for (int s = 0; s < NS; ++s) koff[s] += adv;
  };
  auto advance_v = [&](int j) __attribute__((always_inline)) {
    const int adv = (j % NST) == NST - 1 ? -(NST - 1) * S::TILE : S::TILE;
#pragma unroll
    for (int b = 0; b < NDB; ++b) voff[0][b] += adv, voff[1][b] += adv;
  };

  // scores of one 32-key block: kb = byte offset of the block inside the current K stage
  auto scores = [&](uint32_t kb, f32x16 &s) __attribute__((always_inline)) {
    bf16x8 ka[NS];
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int x = 0; x < NS; ++x) ka[x] = lds_read8_at(koff[x] + kb);
#pragma unroll
    for (int x = 0; x < NS; ++x) s = mfma32(ka[x], qf[x], s);
  };
  auto row_max = [&](const f32x16 &s) __attribute__((always_inline)) {
    float a = fmaxf(s[0], s[1]), b = fmaxf(s[8], s[9]);  // two chains
#pragma unroll
    for (int i = 2; i < 8; ++i) a = fmaxf(a, s[i]), b = fmaxf(b, s[8 + i]);
    return xor32_max(fmaxf(a, b));
  };
  // Lazy rescaling: the running reference m only moves when some row's maximum has grown by more than
  // 2^RESCALE_LOG2; until then probabilities are taken relative to the stale m (they stay below
  // 2^RESCALE_LOG2, harmless in fp32 and bf16) and the accumulators need no multiply.
  auto rescale = [&](float mx) __attribute__((always_inline)) {
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
  };
  // exponentials of a block's scores (in place), row-sum update, packing into the two B operands of P V:
  // k-step t uses registers 8t .. 8t+7
  auto exp_pack = [&](f32x16 &s, bf16x8 (&pb)[2]) {
    float p0 = 0.f, p1 = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      s[i] = fast_exp2(fmaf(s[i], c, -m));
      s[8 + i] = fast_exp2(fmaf(s[8 + i], c, -m));
      p0 += s[i];
      p1 += s[8 + i];
    }
    lsum += p0 + p1;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      u32x4 w = {pack_bf16(s[8 * t], s[8 * t + 1]), pack_bf16(s[8 * t + 2], s[8 * t + 3]),
                 pack_bf16(s[8 * t + 4], s[8 * t + 5]), pack_bf16(s[8 * t + 6], s[8 * t + 7])};
      pb[t] = __builtin_bit_cast(bf16x8, w);
    }
  };
  // vb = byte offset of the block inside the current V stage
  auto pv = [&](uint32_t vb, const bf16x8 (&pb)[2]) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {  // keys 16 t .. 16 t + 15 of the block
#pragma unroll
      for (int b = 0; b < NDB; ++b) {
        bf16x8 a = join(lds_read_tr4_at(voff[0][b] + vb + 16 * t * ROWB),
                        lds_read_tr4_at(voff[1][b] + vb + 16 * t * ROWB));
        acc[b] = mfma32(a, pb[t], acc[b]);
      }
    }
  };

  // Everything issued so far has landed, including the Q fragments: from here on the compiler places no
  // vector-memory waits inside the loop (they would drain the direct-load queue every iteration).
  wait_vmcnt<0>();
#pragma unroll
  for (int s = 0; s < NS; ++s) pin(qf[s]);
  barrier_nofence();

  // The pipeline unit is a 32-key block.  cur holds the scores of the block about to be exponentiated
  // (block 0 of tile j at the top of iteration j), nxt receives the following block's.
  f32x16 cur, nxt;
  scores(0, cur);
  float mx_cur = row_max(cur), mx_nxt = 0.f;

  auto top = [&](int j) __attribute__((always_inline)) {
    // this wave's parts of K(j+1) and V(j) have landed: only the loads of tiles j+2 of K and j+1, j+2 of V
    // may still be in flight
    wait_vmcnt<3 * NLD>();
    barrier_nofence();  // ... and everybody else's; everybody is done with K(j-1) and V(j-1)
    issue_kv(kg, S::K_OFF, j + 3);
    issue_kv(vg, S::V_OFF, j + 3);
  };

  // Tile j and block 0 of tile j+1 fully visible: no mask, no skip.  After each (rare) rescale there is one
  // basic block with 8 score MFMAs, 16 exponentials, 8 P V MFMAs and a row maximum, all mutually independent
  // except through the bf16 P operands.
  auto fast = [&](int j) __attribute__((always_inline)) {
    top(j);
    bf16x8 pb[2];
    rescale(mx_cur);
    scores(uint32_t(32 * ROWB), nxt);
    advance_k(j);  // K reads now address tile j+1
    exp_pack(cur, pb);
    pv(0u, pb);
    mx_nxt = row_max(nxt);
    rescale(mx_nxt);
    scores(0u, cur);
    exp_pack(nxt, pb);
    pv(uint32_t(32 * ROWB), pb);
    advance_v(j);
    mx_cur = row_max(cur);
  };

  // general path: diagonal tiles (mask), tiles some waves do not see at all, the first tile of a document
  auto tail_block = [&](int j, int kb, f32x16 &x) __attribute__((always_inline)) {
    const int k0 = j * FWD_BN + 32 * kb;
    if (k0 > wmax) return;
    if (k0 + 31 > wmin) {  // some (row, key) of this block is above the diagonal
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (k0 + (i >> 2) * 8 + 4 * g + (i & 3) > pos) x[i] = -INFINITY;
    }
    rescale(row_max(x));
    bf16x8 pb[2];
    exp_pack(x, pb);
    const uint32_t vb = uint32_t(32 * kb * ROWB);
    pv(vb, pb);
    // The first rows of a document see a handful of keys, their output is as large as a single V row, and
    // the 2^-9 relative rounding of P to bf16 then shows up at the 1e-2 level next to the output's own bf16
    // rounding.  For the waves that hold such rows, the rounding residue of P is fed through the matrix pipe
    // as a second bf16 operand (P = hi + lo), which makes P V as good as fp32 at negligible cost: it
    // happens only in the first tile of the first query rows of each document.
    if (j == 0 && wmin < FWD_BN) {
      bf16x8 pl[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        uint32_t lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t h = __builtin_bit_cast(u32x4, pb[t])[e];
          lo[e] = pack_bf16(x[8 * t + 2 * e] - __uint_as_float(h << 16),
                            x[8 * t + 2 * e + 1] - __uint_as_float(h & 0xffff0000u));
        }
        pl[t] = __builtin_bit_cast(bf16x8, u32x4{lo[0], lo[1], lo[2], lo[3]});
      }
      pv(vb, pl);
    }
  };
  auto tail = [&](int j) __attribute__((always_inline)) {
    const int j0 = j * FWD_BN;
    top(j);
    if (j0 + 32 <= wmax) scores(uint32_t(32 * ROWB), nxt);
    advance_k(j);  // K reads now address tile j+1
    tail_block(j, 0, cur);
    if (j + 1 < n_tiles && j0 + FWD_BN <= wmax) {
      scores(0u, cur);
      mx_cur = row_max(cur);
    }
    tail_block(j, 1, nxt);
    advance_v(j);
  };

  for (int j = 0; j < n_tiles; ++j) {
    if (j < n_fast) {
      fast(j);
    } else {
      tail(j);
    }
  }
  wait_vmcnt<0>();  // nothing may still be writing LDS when the workgroup ends

  // epilogue: O = acc / l (bf16), LSE = ln 2 * (m + log2 l)
  lsum += __shfl_xor(lsum, 32);
  if (row >= 0) {
    const float inv = 1.0f / lsum;
    bf16_t *op = O + (size_t(row) * Hq + head) * D + 4 * g;
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        u32x2 w = {pack_bf16(acc[b][4 * q4] * inv, acc[b][4 * q4 + 1] * inv),
                   pack_bf16(acc[b][4 * q4 + 2] * inv, acc[b][4 * q4 + 3] * inv)};
        *reinterpret_cast<u32x2 *>(op + 32 * b + 8 * q4) = w;
      }
    if (g == 0) LSE[size_t(head) * total_q + row] = 0.6931471805599453f * (m + fast_log2(lsum));
  }
}

template <int D>
static hipError_t launch_fwd_t(const ca_plan_t *p, const void *q, const void *k, const void *v, void *o, float *lse,
                               hipStream_t st) {
  if (p->fwd_units.empty()) return hipSuccess;
  auto kern = ca_fwd_kernel<D>;
  static std::atomic<bool> attr_done[16];  // once per device; a second thread repeating the call is harmless
  if (!attr_done[p->device & 15].load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       FwdSmem<D>::TOTAL);
    if (e != hipSuccess) return e;
    attr_done[p->device & 15].store(true, std::memory_order_release);
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
