// Forward kernel: O = softmax(scale * Q K^T, causal) V and LSE over tiles of query rows
// (core attention, Section 2.1; one fused launch over all CA-tasks, Section 4.1).
//
// One workgroup = one forward unit = 256 query slots of one document x one query head, or, for the slots a
// document has left over after its full tiles, 256/hp slots x hp query heads of one KV group (same K/V tiles,
// same loads; only the (wave, row group) -> (slots, head) mapping differs).  Four waves, one per SIMD, one
// workgroup per CU.  A wave owns TWO groups of 32 slots (64 query rows): every K or V fragment it reads from
// LDS feeds two MFMAs, one per group, which halves the LDS operand traffic per MFMA against a 32-row wave.
//
// Per group the wave computes the TRANSPOSED score block S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so that a lane
// owns one query row (column l%32 of the MFMA result) and its 16 registers per block are 16 different keys: row max
// and row sum are in-lane work plus one exchange between lanes l and l+32.  The bf16 probabilities, still in those
// registers, are exactly the B operand of O^T += V^T P^T (the key index is the contraction index; its order inside a
// block is the same permutation on both operands).  V^T comes out of the natural-layout V tile in LDS through
// ds_read_b64_tr_b16.
//
// K and V tiles of 64 keys go from global memory straight into swizzled LDS tiles (global_load_lds), four stages
// each.  With one wave per SIMD nothing hides a latency except the wave's own instructions, so tiles entirely below
// the diagonal of the wave's rows run a three-stage software pipeline over 32-key blocks, written out slot by slot:
//   step k:  score MFMAs of block k+1  |  exponentials of block k  |  P V MFMAs of block k-1
// every MFMA being followed by its share of the other work (one exponential, a row-sum addition, half a conversion,
// one LDS fragment read for a later MFMA).  The score MFMAs are inline assembly with architectural destination
// registers (the vector ALU reads the scores directly) and the Q fragments in the accumulation file.  The pipeline
// keeps the running maximum it was entered with (see there); diagonal tiles take a general path with masking and
// lazy rescaling of the accumulators.  The softmax runs in base 2 with scale*log2(e) folded into one FMA.
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

constexpr int FWD_WAVES = 4;  // waves per workgroup; each owns two groups of 32 slots

template <int D>
__global__ __launch_bounds__(64 * FWD_WAVES, 1) void ca_fwd_kernel(const FwdUnit *__restrict__ units,
                                                                   const int32_t *__restrict__ slot_row,
                                                                   const int32_t *__restrict__ slot_pos,
                                                                   const bf16_t *__restrict__ Q,
                                                                   const bf16_t *__restrict__ K,
                                                                   const bf16_t *__restrict__ V, bf16_t *__restrict__ O,
                                                                   float *__restrict__ LSE, int Hq, int Hkv,
                                                                   int64_t total_q, float c /* scale * log2(e) */) {
  using S = FwdSmem<D>;
  constexpr int NS = D / 16;       // MFMA k-steps over head_dim
  constexpr int NDB = D / 32;      // 32-row blocks of O^T
  constexpr int CH = D / 8;        // 16-byte chunks per row
  constexpr int RPI = 64 / CH;     // rows covered by one wave-wide direct load (1 KB)
  constexpr int NLD = FWD_BN / (FWD_WAVES * RPI);  // direct loads per wave per tile
  constexpr int NST = S::NST;
  constexpr int ROWB = 2 * D;
  constexpr int BLK = 32 * ROWB;   // bytes of a 32-key block inside a tile
  constexpr float RESCALE_LOG2 = 8.0f;
  static_assert(FWD_BM == 64 * FWD_WAVES, "a workgroup covers one forward unit");
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(CA_LDS char *)smem;  // LDS byte address of the dynamic segment

  const FwdUnit u = units[blockIdx.x];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, r = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, dh = (lane >> 4) & 1;
  const int hk = u.head / (Hq / Hkv);
  // (wave, group x) -> 32-slot group and query head inside the unit: pair 2 wave + x takes slots 32 (pair / hp) ..
  // of head  head + pair % hp  (hp = 1 for a full tile, > 1 for a head-packed unit)
  const int hp_lg = __builtin_ctz(u.hp);
  int head[2], row[2], pos[2];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const int pair = 2 * wave + x;
    head[x] = u.head + (pair & (u.hp - 1));
    const int slot = u.slot0 + (pair >> hp_lg) * 32 + r;
    row[x] = slot_row[slot];
    pos[x] = slot_pos[slot];
  }
  const int wmax = max(wave_max(pos[0]), wave_max(pos[1])), wmin = min(wave_min(pos[0]), wave_min(pos[1]));
  const int n_tiles = (u.n_keys + FWD_BN - 1) / FWD_BN;
  // tiles j < n_fast: tile j and the first 32 keys of tile j+1 are entirely visible to every row of this wave
  const int n_fast = max(0, (wmin - 31) / FWD_BN);

  // ---- direct global -> LDS tile loads.  Load n of this wave covers tile rows RPI*(wave + 4n) .. +RPI-1;
  // lane i fills physical chunk i % CH of row i / CH, so it fetches logical chunk (i % CH) ^ sw(row).
  // The address is (scalar tile base) + (per-lane 32-bit offset): advancing to the next tile costs no
  // vector instruction.  Tiles past the end are fetched too (as the last tile, rows clamped to the last key),
  // so that every iteration issues the same number of loads and the s_waitcnt bookkeeping stays constant.
  const uint32_t kv_row_bytes = uint32_t(Hkv) * D * 2;
  const int ld_row0 = RPI * wave + lane / CH;  // + FWD_WAVES*RPI*n
  const uint32_t ld_cbytes = uint32_t((lane % CH) ^ tile_sw<D>(ld_row0)) * 16;
  const int last_tile = n_tiles - 1, last_key_in_tile = u.n_keys - 1 - last_tile * FWD_BN;
  uint32_t ld_off[NLD], ld_off_last[NLD];
#pragma unroll
  for (int n = 0; n < NLD; ++n) {
    ld_off[n] = uint32_t(ld_row0 + FWD_WAVES * RPI * n) * kv_row_bytes + ld_cbytes;
    ld_off_last[n] = uint32_t(min(ld_row0 + FWD_WAVES * RPI * n, last_key_in_tile)) * kv_row_bytes + ld_cbytes;
  }
  const char *kg = reinterpret_cast<const char *>(K + (size_t(u.kv_row0) * Hkv + hk) * D);
  const char *vg = reinterpret_cast<const char *>(V + (size_t(u.kv_row0) * Hkv + hk) * D);
  const size_t tile_bytes = size_t(FWD_BN) * kv_row_bytes;
  auto issue_kv = [&](const char *src, int area, int tile) __attribute__((always_inline)) {
    const bool last = tile >= last_tile;
    const char *base = src + size_t(last ? last_tile : tile) * tile_bytes;
    const uint32_t dst = lds0 + uint32_t(area + (tile % NST) * S::TILE + 1024 * wave);
#pragma unroll
    for (int n = 0; n < NLD; ++n)
      load_lds16_sbase(base, last ? ld_off_last[n] : ld_off[n], dst + 1024 * FWD_WAVES * n);
  };
  // Issue order K0 V0 K1 V1 K2 | V2 K3 | V3 K4 | ...: K runs three tiles ahead of the tile being multiplied, V two
  // (the pipelined path multiplies P V one block behind the scores, so a V tile is still read while the next K tile
  // is already in use)
  issue_kv(kg, S::K_OFF, 0);
  issue_kv(vg, S::V_OFF, 0);
  issue_kv(kg, S::K_OFF, 1);
  issue_kv(vg, S::V_OFF, 1);
  issue_kv(kg, S::K_OFF, 2);

  // Q fragments: B operand of S^T = K Q^T; lane holds Q[row][16 s + 8 g .. +7].  They live in accumulation registers
  // (read by MFMAs only).
  bf16x8 qf[2][NS];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const bf16_t *qp = Q + (size_t(row[x] < 0 ? 0 : row[x]) * Hq + head[x]) * D + 8 * g;
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[x][s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
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
  int kst = 0, vst = 0;  // stage koff / voff address
  auto advance_k = [&]() __attribute__((always_inline)) {
    const int adv = kst == NST - 1 ? -(NST - 1) * S::TILE : S::TILE;
    kst = kst == NST - 1 ? 0 : kst + 1;
#pragma unroll
    for (int s = 0; s < NS; ++s) koff[s] += adv;
  };
  auto advance_v = [&]() __attribute__((always_inline)) {
    const int adv = vst == NST - 1 ? -(NST - 1) * S::TILE : S::TILE;
    vst = vst == NST - 1 ? 0 : vst + 1;
#pragma unroll
    for (int b = 0; b < NDB; ++b) voff[0][b] += adv, voff[1][b] += adv;
  };

  f32x16 acc[2][NDB];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[x][b][i] = 0.f;
  float m[2] = {-INFINITY, -INFINITY}, lsum[2] = {0.f, 0.f};

  // ------------------------------------------------------------------------------------------ building blocks
  // K fragments of a 32-key block (kb = byte offset of the block inside koff's stage)
  auto read_k = [&](uint32_t kb, bf16x8 (&ka)[NS]) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < NS; ++s) ka[s] = lds_read8_at(koff[s] + kb);
  };
  // V^T fragment (t, b) of a block: keys 16 t .. 16 t + 15, head-dim rows 32 b .. 32 b + 31
  auto read_v = [&](uint32_t vb, int t, int b) __attribute__((always_inline)) {
    return join(lds_read_tr4_at(voff[0][b] + vb + 16 * t * ROWB), lds_read_tr4_at(voff[1][b] + vb + 16 * t * ROWB));
  };
  // scores of both groups for one block, not interleaved with anything (prologue and diagonal tiles)
  auto scores_plain = [&](uint32_t kb, f32x16 &s0, f32x16 &s1) __attribute__((always_inline)) {
    bf16x8 ka[NS];
    read_k(kb, ka);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (s == 0) mfma32_v_first(s0, ka[0], qf[0][0]), mfma32_v_first(s1, ka[0], qf[1][0]);
      else mfma32_v(s0, ka[s], qf[0][s]), mfma32_v(s1, ka[s], qf[1][s]);
    }
    mfma_settle(s0, s1);
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
  auto rescale_to = [&](int x, float m_cand) __attribute__((always_inline)) {
    const float alpha = m[x] == -INFINITY ? 0.f : fast_exp2(m[x] - m_cand);
    m[x] = m_cand;
    lsum[x] *= alpha;
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[x][b][i] *= alpha;
  };
  auto rescale = [&](int x, float mx) __attribute__((always_inline)) {
    const float m_cand = fmaxf(m[x], mx * c);
    if (__any(m_cand > m[x] + RESCALE_LOG2)) rescale_to(x, m_cand);
  };
  // exponentials of a block's scores (in place), row-sum update, packing into the two B operands of P V:
  // k-step t uses registers 8t .. 8t+7
  auto exp_pack = [&](int x, f32x16 &s, uint32_t (&pw)[8]) __attribute__((always_inline)) {
    float p0 = 0.f, p1 = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      s[i] = fast_exp2(fmaf(s[i], c, -m[x]));
      s[8 + i] = fast_exp2(fmaf(s[8 + i], c, -m[x]));
      p0 += s[i];
      p1 += s[8 + i];
    }
    lsum[x] += p0 + p1;
#pragma unroll
    for (int k = 0; k < 8; ++k) pw[k] = pack_bf16(s[2 * k], s[2 * k + 1]);
  };
  auto p_operand = [&](const uint32_t (&pw)[8], int t) __attribute__((always_inline)) {
    return __builtin_bit_cast(bf16x8, u32x4{pw[4 * t], pw[4 * t + 1], pw[4 * t + 2], pw[4 * t + 3]});
  };
  // P V of one block for both groups (or one), not interleaved with anything
  auto pv_plain = [&](uint32_t vb, const uint32_t (&p0)[8], const uint32_t (&p1)[8], bool do0, bool do1)
                      __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int b = 0; b < NDB; ++b) {
        const bf16x8 a = read_v(vb, t, b);
        if (do0) acc[0][b] = mfma32(a, p_operand(p0, t), acc[0][b]);
        if (do1) acc[1][b] = mfma32(a, p_operand(p1, t), acc[1][b]);
      }
  };

  // Everything issued so far has landed, including the Q fragments: from here on the compiler places no
  // vector-memory waits inside the loop (they would drain the direct-load queue every iteration).
  wait_vmcnt<0>();
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int s = 0; s < NS; ++s) pin_acc(qf[x][s]);
  barrier_nofence();

  // this wave's parts of K(j+1) and V(j) have landed: only V(j+1) and K(j+2) may still be in flight
  auto top = [&](int j) __attribute__((always_inline)) {
    wait_vmcnt<2 * NLD>();
    barrier_nofence();  // ... and everybody else's; everybody is done with K(j-1) and V(j-2)
    issue_kv(vg, S::V_OFF, j + 2);
    issue_kv(kg, S::K_OFF, j + 3);
  };

  // ------------------------------------------------------------------------------------------ pipelined path
  // Tiles j < n_fast.  The pipeline exponentiates against the running maximum m as it stood when it was entered (the
  // maximum of the first block): the loop holds no rescaling code, no row maximum and no exit (an exit alone costs the
  // register allocation of the loop dearly).  Probabilities relative to a stale m are merely larger numbers - bf16 and
  // fp32 carry the same exponent range, so neither P nor the accumulators lose accuracy - until one of them overflows;
  // that shows in the row sum.  If the row sum of any row of a workgroup has left the finite range, everything computed
  // here is thrown away and the unit is computed again by the general path alone (below), which rescales block by
  // block.  A later score would have to exceed the first block's maximum by about 2^100 in probability for that (the row sum is
  // checked against 1e30, which leaves the accumulators, |V| times larger at most, well inside fp32).
  int j = 0;
  bool outgrown = false;
  if (n_fast > 0) {
    // tuples: sc[k & 1][x] holds S(k) of group x, then its exponentials; packed P(k) goes to pp[k & 1][x]
    f32x16 sc[2][2];
    uint32_t pp[2][2][8];
    bf16x8 ka[NS];          // K fragments of the block whose scores the next step computes
    bf16x8 va[NS];          // V^T fragments of the block whose P V this step computes (2 NDB = NS of them)

    // One step.  E: tuples holding S(k) (exponentiated here); N: tuples that receive S(k+1).  kn, kb: offsets, from
    // koff's stage, of the keys of S(k+1) (the second half of their fragments is fetched here) and of S(k+2) (the
    // first half, for the next step); vb: block offset of block k-1 in voff's stage.  PV = false leaves block k-1
    // out (first step).  NEXT_TILE: S(k+2) belongs to the tile after S(k+1)'s: koff moves on between the two phases.
    auto step = [&](f32x16 (&E)[2], f32x16 (&N)[2], uint32_t (&PE)[2][8], const uint32_t (&PP)[2][8], uint32_t kn,
                    uint32_t kb, uint32_t vb, const bool PV, const bool NEXT_TILE) __attribute__((always_inline)) {
      constexpr int TS = 2 * NS, TP = 4 * NDB, T = TS + TP;  // MFMA slots: score phase, P V phase
      constexpr int EPS = 32 / T;                            // exponentials per slot
      constexpr int H = NS / 2;
      float pend[2] = {0.f, 0.f};  // exponential of the previous slot, added to the row sum one slot later
      int pend_x = 0;
      // the vector work of slot q: exponential(s) e = q EPS .. of (group e / 16, register e % 16) with the row-sum
      // addition of the one before, and every other exponential the conversion of the pair completed before it
      auto vec_slot = [&](int q) __attribute__((always_inline)) {
#pragma unroll
        for (int e = q * EPS; e < (q + 1) * EPS; ++e) {
          const int x = e >> 4, i = e & 15;
          float v = E[x][i];
          if (e == 0) exp2_fma_inplace_pinned(v, c, m[x]);
          else exp2_fma_add_inplace_pinned(v, c, m[x], lsum[pend_x], pend[(e - 1) & 1]);
          E[x][i] = v;
          pend[e & 1] = v;
          pend_x = x;
          if ((e & 1) == 0 && e >= 2) {
            const int ep = e - 2;  // pair (ep, ep + 1): both exponentials are at least one instruction old
            PE[ep >> 4][(ep & 15) >> 1] = pack_bf16_pinned(E[ep >> 4][ep & 15], E[ep >> 4][(ep & 15) + 1]);
          }
        }
      };
      // Fragments are fetched from LDS H = NS / 2 fragments (2 H slots) ahead of the MFMA pair that uses them, one per
      // odd slot, so that about NS of them are alive at any time rather than 2 NS.
      // ---- score phase: S(k+1); every K fragment feeds group 0's chain, then group 1's
#pragma unroll
      for (int q = 0; q < TS; ++q) {
        const int x = q & 1, s = q >> 1;
        if (s == 0) mfma32_v_first(N[x], ka[0], qf[x][0]);
        else mfma32_v(N[x], ka[s], qf[x][s]);
        if (x == 1) {
          if (s < H) ka[s + H] = lds_read8_at(koff[s + H] + kn);               // later K fragments of S(k+1)
          else if (PV) va[s - H] = read_v(vb, (s - H) / NDB, (s - H) % NDB);   // first V^T fragments of block k-1
        }
        vec_slot(q);
        __builtin_amdgcn_sched_barrier(0);
      }
      mfma_settle(N[0], N[1]);
      if (NEXT_TILE) advance_k();
      // ---- P V phase: block k-1
#pragma unroll
      for (int q = 0; q < TP; ++q) {
        const int f = q >> 1, x = q & 1;  // fragment f = (t, b)
        if (PV) acc[x][f % NDB] = mfma32(va[f], p_operand(PP[x], f / NDB), acc[x][f % NDB]);
        if (x == 1) {
          if (f < H) {
            if (PV) va[f + H] = read_v(vb, (f + H) / NDB, (f + H) % NDB);      // later V^T fragments of block k-1
          } else {
            ka[f - H] = lds_read8_at(koff[f - H] + kb);                        // first K fragments of S(k+2)
          }
        }
        vec_slot(TS + q);
        __builtin_amdgcn_sched_barrier(0);
      }
      add_after_trans_pinned(lsum[pend_x], pend[1]);
      PE[1][7] = pack_bf16_pinned(E[1][14], E[1][15]);
    };

    // prologue: S(0) and its maximum, which becomes m; first K fragments of block 1
    scores_plain(0u, sc[0][0], sc[0][1]);
    m[0] = row_max(sc[0][0]) * c;
    m[1] = row_max(sc[0][1]) * c;
#pragma unroll
    for (int s = 0; s < NS / 2; ++s) ka[s] = lds_read8_at(koff[s] + uint32_t(BLK));
    top(0);  // tile 1 of K has landed: blocks 2 and 3
    step(sc[0], sc[1], pp[0], pp[1], uint32_t(BLK), 0u, uint32_t(BLK), false, true);  // S(1) | exp(0)
    step(sc[1], sc[0], pp[1], pp[0], 0u, uint32_t(BLK), 0u, true, false);             // S(2) | exp(1) | P V(0)
    for (j = 1; j < n_fast; ++j) {
      top(j);
      step(sc[0], sc[1], pp[0], pp[1], uint32_t(BLK), 0u, uint32_t(BLK), true, true);  // S(2j+1) | exp(2j) | P V(2j-1)
      advance_v();                                                                     // voff addresses tile j
      step(sc[1], sc[0], pp[1], pp[0], 0u, uint32_t(BLK), 0u, true, false);            // S(2j+2) | exp(2j+1) | P V(2j)
    }
    // drain: block 2 n_fast - 1 is exponentiated but not multiplied in (voff addresses its tile); the scores computed
    // ahead, S(2 n_fast), are dropped: the general path computes them again, with its mask
    pv_plain(uint32_t(BLK), pp[1][0], pp[1][1], true, true);
    advance_v();
    outgrown = __any(!(lsum[0] < 1.0e30f) || !(lsum[1] < 1.0e30f));  // also true for NaN
  }

  // ------------------------------------------------------------------------------------------ general path
  // diagonal tiles (mask), tiles some rows do not see at all, the first tile of a document
  auto tail_block = [&](int jt, int kb) __attribute__((always_inline)) {
    const int k0 = jt * FWD_BN + 32 * kb;
    if (k0 > wmax) return;
    f32x16 x[2];
    scores_plain(uint32_t(kb * BLK), x[0], x[1]);
    uint32_t pw[2][8];
#pragma unroll
    for (int gx = 0; gx < 2; ++gx) {
      if (k0 + 31 > wmin) {  // some (row, key) of this block may be above the diagonal
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (k0 + (i >> 2) * 8 + 4 * g + (i & 3) > pos[gx]) x[gx][i] = -INFINITY;
      }
      // a row that sees no key of this block keeps m = -inf only if it has seen none at all, which cannot happen:
      // every row sees key 0, and blocks are walked from key 0 on
      rescale(gx, row_max(x[gx]));
      exp_pack(gx, x[gx], pw[gx]);
    }
    const uint32_t vb = uint32_t(kb * BLK);
    pv_plain(vb, pw[0], pw[1], true, true);
    // The first rows of a document see a handful of keys, their output is as large as a single V row, and
    // the 2^-9 relative rounding of P to bf16 then shows up at the 1e-2 level next to the output's own bf16
    // rounding.  For the waves that hold such rows, the rounding residue of P is fed through the matrix pipe
    // as a second bf16 operand (P = hi + lo), which makes P V as good as fp32 at negligible cost: it
    // happens only in the first tile of the first query rows of each document.
    if (jt == 0 && wmin < FWD_BN) {
      uint32_t pl[2][8];
#pragma unroll
      for (int gx = 0; gx < 2; ++gx)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t h = pw[gx][e];
          pl[gx][e] = pack_bf16(x[gx][2 * e] - __uint_as_float(h << 16), x[gx][2 * e + 1] - __uint_as_float(h & 0xffff0000u));
        }
      pv_plain(vb, pl[0], pl[1], true, true);
    }
  };
  for (; j < n_tiles; ++j) {
    top(j);
    tail_block(j, 0);
    tail_block(j, 1);
    advance_k();
    advance_v();
  }
  wait_vmcnt<0>();  // nothing may still be writing LDS
  // Did the pipelined path of any wave of the workgroup meet a maximum beyond its window?  (The tiles are shared, so
  // the workgroup repeats the unit together or not at all.)  Flags go through the first bytes of LDS: every tile read
  // and every direct load of the workgroup is complete after the first barrier.
  barrier_nofence();
  if (lane == 0) *reinterpret_cast<volatile int *>(smem + 4 * wave) = outgrown ? 1 : 0;
  __syncthreads();
  const u32x4 flags = *reinterpret_cast<const u32x4 *>(smem);
  __syncthreads();
  if (__builtin_amdgcn_readfirstlane(flags[0] | flags[1] | flags[2] | flags[3]) != 0) {
    // the whole unit again, every tile through the general path
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      m[x] = -INFINITY;
      lsum[x] = 0.f;
#pragma unroll
      for (int b = 0; b < NDB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[x][b][i] = 0.f;
    }
    while (kst != 0) advance_k();
    while (vst != 0) advance_v();
    issue_kv(kg, S::K_OFF, 0);
    issue_kv(vg, S::V_OFF, 0);
    issue_kv(kg, S::K_OFF, 1);
    issue_kv(vg, S::V_OFF, 1);
    issue_kv(kg, S::K_OFF, 2);
    wait_vmcnt<0>();
    barrier_nofence();
    for (j = 0; j < n_tiles; ++j) {
      top(j);
      tail_block(j, 0);
      tail_block(j, 1);
      advance_k();
      advance_v();
    }
    wait_vmcnt<0>();
    __syncthreads();  // the epilogue writes into the stages
  }

  // epilogue: O = acc / l (bf16), LSE = ln 2 * (m + log2 l).  O leaves as whole lines through a patch of LDS (the
  // stages are free: every wave is past its last tile)
  static_assert(FWD_WAVES * PATCH_BYTES <= S::TOTAL, "patches fit in the stages");
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    float l = lsum[x];
    l += __shfl_xor(l, 32);
    const int rx = row[x], hx = head[x];
    store_tile_as_lines<NDB>(lds0 + wave * PATCH_BYTES, acc[x], 1.0f / l, lane, [&](int p) __attribute__((always_inline)) -> bf16_t * {
      const int rw = __shfl(rx, p);
      return rw >= 0 ? O + (size_t(rw) * Hq + hx) * D : nullptr;
    });
    if (rx >= 0 && g == 0) LSE[size_t(hx) * total_q + rx] = 0.6931471805599453f * (m[x] + fast_log2(l));
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
  hipLaunchKernelGGL(kern, dim3(unsigned(p->fwd_units.size())), dim3(64 * FWD_WAVES), FwdSmem<D>::TOTAL, st,
                     p->d_fwd_units, p->d_slot_row, p->d_slot_pos, static_cast<const bf16_t *>(q),
                     static_cast<const bf16_t *>(k), static_cast<const bf16_t *>(v), static_cast<bf16_t *>(o), lse,
                     p->hq, p->hkv, p->total_q, c);
  return hipGetLastError();
}

hipError_t launch_fwd(const ca_plan_t *p, const void *q, const void *k, const void *v, void *o, float *lse,
                      hipStream_t st) {
  return p->d == 128 ? launch_fwd_t<128>(p, q, k, v, o, lse, st) : launch_fwd_t<64>(p, q, k, v, o, lse, st);
}

}  // namespace ca
