// Backward kernels: dQ, dK, dV of L = sum(dO * O) with P recomputed from the saved log-sum-exp
// (Section 2.1: P is not stored in forward, it is recomputed during backward).
//
//   prep : per (slot, head): -Delta = -<dO, O> and L2 = log2(e) * LSE, stored in SLOT order (the order of the
//          planner's per-document sorted query rows), so that both main kernels read them contiguously.
//          Padding slots get L2 = +huge, which makes their recomputed probabilities exactly 0.
//   dq   : one workgroup = one of the forward's work units (256 query slots x one query head, or 256/hp slots x hp
//          heads of one KV group), walking over the document's keys like the forward does.  Lane <-> query row:
//            S^T = K Q^T, dP^T = V dO^T, P^T = exp2(c S^T - L2), dS^T = P^T (dP^T - Delta),
//            dQ^T += K^T dS^T   (K^T through transposing LDS reads of the same K tile)
//   dkv  : one workgroup = 128 keys of one document x one KV head, walking over every block of 64 query
//          slots that can see them, for each query head of the group.  Lane <-> key:
//            S = Q K^T, dP = dO V^T (K, V fragments of the wave's 32 keys stay in registers),
//            dV^T += dO^T P, dK^T += Q^T dS   (Q^T, dO^T through transposing LDS reads)
//          dK and dV are written once, already summed over the group's heads and all tasks of the document.
//          Workgroups of one KV head that run on one XCD walk the same Q/dO tiles and pace each other through
//          published step counts, so that the tiles are fetched into that XCD's L2 once ("convoy", see the kernel).
// No atomics and no fp32 dQ buffer: the price is that S and dP are computed in both kernels (7 contractions
// instead of the minimal 5).  Results are deterministic.
#include <algorithm>
#include <atomic>

#include "ca_device.h"
#include "ca_internal.h"

namespace ca {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float L2_PADDING = 1.0e30f;  // exp2(x - 1e30) == 0 for every finite score

__global__ void ca_bwd_prep_kernel(const int32_t *__restrict__ slot_row, const int32_t *__restrict__ block_rpk,
                                   const bf16_t *__restrict__ Q, const bf16_t *__restrict__ O,
                                   const bf16_t *__restrict__ dO, const float *__restrict__ LSE,
                                   float *__restrict__ delta_slot, float *__restrict__ l2_slot,
                                   float *__restrict__ delta_kv, float *__restrict__ l2_kv,
                                   bf16_t *__restrict__ q_sorted, bf16_t *__restrict__ do_sorted,
                                   int32_t *__restrict__ progress, int n_progress, int64_t padded, int64_t total_q,
                                   int Hq, int G, int D) {
  // D/8 lanes per (slot, head): -Delta = -<dO, O> and log2(e)*LSE in slot order (for the dQ kernel), and for the
  // dK/dV kernel the slot-ordered copies of Q and dO as [block of 64 slots][head][64][D] - the 64-row tile of a
  // (block, head) is one contiguous run, and the tiles of the heads of a block follow each other - with the same two
  // statistics in the row order of those tiles (padding rows: zeros, with an LSE that makes every probability 0).
  // In a packed block (a document of at most rpk = 16 or 32 rows) tile t of a KV group holds the rows of the group's
  // heads 64/rpk t .. 64/rpk (t + 1) - 1, rpk rows each; the group's remaining tiles are neither written nor read.
  const int lanes = D / 8;
  const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx < n_progress) progress[idx] = 0;  // progress counters of the dK/dV workgroups: nobody has started
  const int64_t pair = idx / lanes;
  const int c = int(idx % lanes);
  const bool ok = pair < padded * Hq;
  const int64_t slot = ok ? pair / Hq : 0;
  const int h = int(pair % Hq);
  const int row = ok ? slot_row[slot] : -1;
  float s = 0.f;
  u32x4 qv = {0, 0, 0, 0}, dv = {0, 0, 0, 0};
  if (row >= 0) {
    const size_t off = (size_t(row) * Hq + h) * D + 8 * c;
    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(O + off);
    const bf16x8 b = *reinterpret_cast<const bf16x8 *>(dO + off);
    qv = *reinterpret_cast<const u32x4 *>(Q + off);
    dv = __builtin_bit_cast(u32x4, b);
#pragma unroll
    for (int i = 0; i < 8; ++i) s += float(a[i]) * float(b[i]);
  }
  for (int o = lanes / 2; o > 0; o >>= 1) s += __shfl_xor(s, o);
  if (ok) {
    const float nd = row >= 0 ? -s : 0.f;  // stored negated: both kernels add it
    const float l2 = row >= 0 && c == 0 ? LSE[int64_t(h) * total_q + row] * LOG2E : L2_PADDING;
    const int64_t blk = slot / BWD_BQ;
    const int rpk = block_rpk[blk];
    int th = h, tr = int(slot % BWD_BQ);  // tile (as a head index) and row of this (slot, head) in the dK/dV tiles
    bool in_tile = true;
    if (rpk != 0) {
      const int hpk = BWD_BQ / rpk, hg = h % G;
      in_tile = tr < rpk;  // the slots beyond are padding of the document
      th = h - hg + hg / hpk;
      tr += (hg % hpk) * rpk;
    }
    if (in_tile) {
      const size_t so = ((size_t(blk) * Hq + th) * BWD_BQ + tr) * D + 8 * c;
      *reinterpret_cast<u32x4 *>(q_sorted + so) = qv;
      *reinterpret_cast<u32x4 *>(do_sorted + so) = dv;
    }
    if (c == 0) {
      delta_slot[int64_t(h) * padded + slot] = nd;
      l2_slot[int64_t(h) * padded + slot] = l2;
      if (in_tile) {
        delta_kv[int64_t(th) * padded + blk * BWD_BQ + tr] = nd;
        l2_kv[int64_t(th) * padded + blk * BWD_BQ + tr] = l2;
      }
    }
  }
}

__global__ void ca_fill_zero_kernel(u32x4 *__restrict__ p, int64_t n16) {
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = u32x4{0, 0, 0, 0};
}

// ------------------------------------------------------------------------------------------------ dQ
template <int D>
struct DqSmem {
  static constexpr int NST = 4;
  static constexpr int TILE = FWD_BN * 2 * D;
  // a stage holds the K tile and then the V tile of one key block: both are reached from one address register
  // through the 16-bit offset field of the LDS instructions
  static constexpr int K_OFF = 0;
  static constexpr int V_OFF = TILE;
  static constexpr int STAGE = 2 * TILE;
  static constexpr int TOTAL = NST * STAGE;
};

template <int D>
__global__ __launch_bounds__(512, 2) void ca_bwd_dq_kernel(const FwdUnit *__restrict__ units,
                                                           const int32_t *__restrict__ slot_row,
                                                           const int32_t *__restrict__ slot_pos,
                                                           const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                           const bf16_t *__restrict__ V, const bf16_t *__restrict__ dO,
                                                           const float *__restrict__ l2_slot,
                                                           const float *__restrict__ delta_slot,
                                                           bf16_t *__restrict__ dQ, int Hq, int Hkv, int64_t padded,
                                                           float scale) {
  using S = DqSmem<D>;
  constexpr int NS = D / 16, NDB = D / 32, CH = D / 8, RPI = 64 / CH, NLD = FWD_BN / (8 * RPI), NST = S::NST;
  constexpr int ROWB = 2 * D;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const uint32_t lds0 = (uint32_t)(uintptr_t)(CA_LDS char *)smem;  // LDS byte address of the dynamic segment
  const FwdUnit u = units[blockIdx.x];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, r = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, dh = (lane >> 4) & 1;
  const int hk = u.head / (Hq / Hkv);
  // wave -> (32-slot group, query head) inside the unit, as in the forward kernel
  const int hp_lg = __builtin_ctz(u.hp);
  const int head = u.head + (wave & (u.hp - 1));
  const int slot = u.slot0 + (wave >> hp_lg) * 32 + r;
  const int row = slot_row[slot];
  const int pos = slot_pos[slot];
  float l2 = l2_slot[int64_t(head) * padded + slot];
  float dl = delta_slot[int64_t(head) * padded + slot];
  const int wmax = wave_max(pos), wmin = wave_min(pos);
  const int n_tiles = (u.n_keys + FWD_BN - 1) / FWD_BN;
  const float c = scale * LOG2E;

  // direct loads addressed as (scalar tile base) + (per-lane 32-bit offset); tiles past the end are fetched as the
  // last tile with rows clamped to the last key (constant number of loads per iteration, see the forward kernel)
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
    const uint32_t dst = lds0 + uint32_t(area + (tile % NST) * S::STAGE + 1024 * wave);
#pragma unroll
    for (int n = 0; n < NLD; ++n) load_lds16_sbase(base, last ? ld_off_last[n] : ld_off[n], dst + 8192 * n);
  };
  issue_kv(kg, S::K_OFF, 0);
  issue_kv(vg, S::V_OFF, 0);
  issue_kv(kg, S::K_OFF, 1);
  issue_kv(vg, S::V_OFF, 1);
  issue_kv(kg, S::K_OFF, 2);
  issue_kv(vg, S::V_OFF, 2);

  // Q and dO fragments (B operands); lane holds row's elements 16 s + 8 g .. +7
  bf16x8 qf[NS], dof[NS];
  {
    const size_t off = (size_t(row < 0 ? 0 : row) * Hq + head) * D + 8 * g;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      qf[s] = *reinterpret_cast<const bf16x8 *>(Q + off + 16 * s);
      dof[s] = *reinterpret_cast<const bf16x8 *>(dO + off + 16 * s);
    }
  }
  int koff[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) koff[s] = lds0 + tile_off<D>(r, 2 * s + g);
  int toff[2][NDB];
#pragma unroll
  for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
    for (int b = 0; b < NDB; ++b)
      toff[h2][b] = lds0 + tile_off<D>(4 * g + (li >> 2) + 8 * h2, 4 * b + 2 * dh + ((li >> 1) & 1)) + 8 * (li & 1);

  f32x16 acc[NDB];
#pragma unroll
  for (int b = 0; b < NDB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;

  // All register loads above are complete from here on, so the compiler places no vector-memory waits
  // inside the loop (they would drain the direct-load queue every iteration).
  wait_vmcnt<0>();
#pragma unroll
  for (int s = 0; s < NS; ++s) pin(qf[s]), pin(dof[s]);
  pin(l2), pin(dl);
  // -Delta enters dP through the matrix pipe: one more k-step whose A fragment is 1 in two k-slots of every key row
  // and whose B fragment holds -Delta of the lane's query row split in two bf16 (hi + lo, 16 bits of mantissa) in
  // the same two slots.  One MFMA per 32 keys instead of 16 vector additions: this kernel is bound by its vector
  // ALU work (the exponentials run at quarter rate), not by the matrix pipe.
  bf16x8 ones_f, dl_f;
  {
    const bf16_t hi = bf16_t(dl), lo = bf16_t(dl - float(hi));
#pragma unroll
    for (int i = 0; i < 8; ++i) ones_f[i] = bf16_t(0.f), dl_f[i] = bf16_t(0.f);
    if (g == 0) ones_f[0] = bf16_t(1.f), ones_f[1] = bf16_t(1.f), dl_f[0] = hi, dl_f[1] = lo;
  }
  pin(ones_f), pin(dl_f);

  for (int j = 0; j < n_tiles; ++j) {
    const int j0 = j * FWD_BN;
    wait_vmcnt<4 * NLD>();  // this wave's parts of K(j), V(j) have landed
    barrier_nofence();      // ... and everybody else's; everybody is done with tile j-1
    issue_kv(kg, S::K_OFF, j + 3);
    issue_kv(vg, S::V_OFF, j + 3);
    const bool seen = j0 <= wmax;  // some row of this wave sees the tile
    constexpr int kt = S::K_OFF, vt = S::V_OFF;  // koff / toff address the current stage
    const bool masked = j0 + FWD_BN - 1 > wmin;
    // one 64-key tile; MASKED is a compile-time constant in each of the two instantiations below
    auto tile = [&](const bool MASKED) __attribute__((always_inline)) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        f32x16 sa, pa;
#pragma unroll
        for (int i = 0; i < 16; ++i) sa[i] = 0.f, pa[i] = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          sa = mfma32(lds_read8_at(kt + koff[s] + 32 * kb * ROWB), qf[s], sa);
          pa = mfma32(lds_read8_at(vt + koff[s] + 32 * kb * ROWB), dof[s], pa);
        }
        pa = mfma32(ones_f, dl_f, pa);  // dP - Delta
        uint32_t dw[8];
        // register i holds key j0 + 32 kb + 4 g + 8 (i / 4) + i % 4: visible iff 8 (i / 4) + i % 4 <= vis
        const int vis = pos - (j0 + 32 * kb + 4 * g);
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          float p0 = fast_exp2(fmaf(sa[i], c, -l2)), p1 = fast_exp2(fmaf(sa[i + 1], c, -l2));
          if (MASKED) {
            p0 = (i >> 2) * 8 + (i & 3) <= vis ? p0 : 0.f;
            p1 = (i >> 2) * 8 + (i & 3) + 1 <= vis ? p1 : 0.f;
          }
          dw[i >> 1] = pack_bf16(p0 * pa[i], p1 * pa[i + 1]);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const bf16x8 db = __builtin_bit_cast(bf16x8, u32x4{dw[4 * t], dw[4 * t + 1], dw[4 * t + 2], dw[4 * t + 3]});
          const int ro = (32 * kb + 16 * t) * ROWB;
#pragma unroll
          for (int b = 0; b < NDB; ++b) {
            const bf16x8 a = join(lds_read_tr4_at(kt + toff[0][b] + ro), lds_read_tr4_at(kt + toff[1][b] + ro));
            acc[b] = mfma32(a, db, acc[b]);
          }
        }
      }
    };
    if (seen) {
      if (masked) tile(true);
      else tile(false);
    }
    {  // the offsets follow the stages round
      const int adv = (j % NST) == NST - 1 ? -(NST - 1) * S::STAGE : S::STAGE;
#pragma unroll
      for (int s = 0; s < NS; ++s) koff[s] += adv;
#pragma unroll
      for (int b = 0; b < NDB; ++b) toff[0][b] += adv, toff[1][b] += adv;
    }
  }
  wait_vmcnt<0>();
  // dQ of the wave's 32 rows, as whole lines through a patch of LDS (the stages are free once every wave is past its
  // last tile)
  __syncthreads();
  static_assert(8 * PATCH_BYTES <= S::TOTAL, "patches fit in the stages");
  store_tile_as_lines<NDB>(lds0 + wave * PATCH_BYTES, acc, scale, lane, [&](int p) __attribute__((always_inline)) -> bf16_t * {
    const int rw = __shfl(row, p);
    return rw >= 0 ? dQ + (size_t(rw) * Hq + head) * D : nullptr;
  });
}

// ------------------------------------------------------------------------------------------------ dK, dV
template <int D>
struct DkvSmem {
  static constexpr int NST = 4;
  static constexpr int TILE = BWD_BQ * 2 * D;       // one Q or dO tile of 64 slots
  static constexpr int Q_OFF = 0;
  static constexpr int DO_OFF = TILE;
  static constexpr int L2_OFF = 2 * TILE;           // 64 floats each: L2, Delta, position, spare
  static constexpr int DL_OFF = L2_OFF + 256;
  static constexpr int POS_OFF = DL_OFF + 256;
  static constexpr int SPARE_OFF = POS_OFF + 256;
  static constexpr int STAGE = 2 * TILE + 1024;
  // behind the stages (which a chain keeps in use from unit to unit): one patch per wave through which it turns its
  // results into whole rows
  static constexpr int OUT_OFF = NST * STAGE;
  static constexpr int TOTAL = OUT_OFF + 4 * PATCH_BYTES;
};

template <int D, bool CHAIN>
__device__ __forceinline__ void dkv_workgroup(const int me, const BwdUnit &first,
                                              const BwdUnit *__restrict__ units, int n_single,
                                              const int32_t *__restrict__ slot_pos, const bf16_t *__restrict__ Qs,
                                              const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
                                              const bf16_t *__restrict__ dOs, const float *__restrict__ l2_slot,
                                              const float *__restrict__ delta_slot, bf16_t *__restrict__ dK,
                                              bf16_t *__restrict__ dV, int32_t *progress, int peer_stride, int Hq,
                                              int Hkv, int64_t padded, float scale) {
  using S = DkvSmem<D>;
  constexpr int NS = D / 16, NDB = D / 32, CH = D / 8, RPI = 64 / CH, NST = S::NST;
  constexpr int NLD = BWD_BQ / (4 * RPI);  // direct loads per wave per Q (or dO) tile
  constexpr int RPW = BWD_BQ / 4;          // tile rows fetched by one wave (contiguous)
  constexpr int ROWB = 2 * D;
  constexpr int PA = NS;                   // k-steps of natural Q/dO fragments held ahead of their MFMAs (all)
  constexpr int PFB = (2 * PA) / (2 * NDB);  // natural fragments fetched per gradient MFMA pair
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const uint32_t lds0 = (uint32_t)(uintptr_t)(CA_LDS char *)smem;  // LDS byte address of the dynamic segment
  // The workgroup's units, one after the other (all of one KV head).  The lane's indices are derived again for every
  // unit (through an opaque copy, so that the compiler does not keep what follows from them in registers across the
  // whole unit loop).  Two things are carried from a unit to the next:
  //  - the Q/dO stream.  Short units that follow each other are mostly the KV tiles of one document under the same
  //    query rows (a shard with a long context): the next unit walks the same (block, head) tiles.  If this unit
  //    ends in the pipelined path, the prefetch cursor wraps round to the first tile instead of stopping at the last,
  //    and the next unit finds its first tiles in the stages, in the state in which the pipelined path expects them:
  //    no drain, no refill (`cont`).
  //  - the next unit's K and V fragments, fetched into registers while this unit computes (`have_kv`).
  int pblk = 0, ph = 0, pst = 0;
  uint32_t pst_addr = lds0;  // LDS address of the stage being filled
  const char *q_tile = nullptr, *do_tile = nullptr, *q_first = nullptr, *do_first = nullptr;
  const float *aux_ptr = nullptr, *aux_first = nullptr;
  int qoff[NS];  // natural fragment s of tile row r (second sub-block: + 32 rows)
  int toff[2][NDB];
  int auxo = 0, auxq = 0, stage = 0, qstage = 0;
  bf16x8 kf[NS], vf[NS], kfn[NS], vfn[NS];
  bool cont = false, have_kv = false;
  // (unit descriptors are fetched two units ahead, so that no unit starts by waiting for its own)
  // Workgroups of one unit and chains are two instances of this function (CHAIN), so that a unit that runs alone pays
  // for none of this.
  BwdUnit u = first;
  const int count = CHAIN ? u.count : 1, follow = u.follow;
  BwdUnit nu = units[count > 1 ? follow : me];
  for (int ui = 0; ui < count; ++ui) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, g = lane >> 5, r = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, dh = (lane >> 4) & 1;
  const int G = Hq / Hkv;
  const int kw0 = 32 * wave;
  const float c = scale * LOG2E;
  const bool has_next = CHAIN && ui + 1 < count;
  const BwdUnit nnu = units[ui + 2 < count ? follow + ui + 1 : me];
  const int hk = u.kv_head;
  const int key_pos = u.key_pos0 + kw0 + r;  // document position of this lane's key
  const int n_blocks = (u.slot_end - u.slot_begin) / BWD_BQ;
  const int Gu = u.heads;  // tiles per block: the heads of the group, or fewer in a block of packed rows
  const int n_it = n_blocks * Gu;
  // Query blocks are walked from the last one backwards (below), so the blocks that lie entirely below the
  // diagonal of this KV tile come first: they take the pipelined path without mask.
  const int n_fast = ((u.slot_end - u.slot_full) / BWD_BQ) * Gu;
  // the stream goes on into the next unit / the next unit's K and V are fetched ahead (the loads go out before the
  // pipelined loop and are waited for, by the compiler, where the fragments change hands at the unit's end; the
  // loop's own waits count loads issued after them, so they can only wait longer.  Issued inside the loop, after its
  // first wait, the loads would have longer to land, but the branch that takes costs every step more than it gains)
  const bool wrap = has_next && n_it > 0 && n_fast == n_it && nu.slot_begin == u.slot_begin && nu.slot_end == u.slot_end;
  const bool fetch_kv = has_next && n_fast >= 1;

  // ---- loads of one (q block, head): this wave fetches tile rows RPW*wave .. +RPW-1 of Q and of dO, plus one
  // 64-float auxiliary array.  Q and dO come from their slot-ordered copies [block][head][64][D], in which the tile
  // of a (block, head) is one contiguous run: a load is (wave-uniform tile address) + (per-lane constant).
  const int ld_rr = lane / CH;  // row inside one direct load
  uint32_t ld_off[NLD];         // byte offset of the lane's chunk from the start of the tile
#pragma unroll
  for (int n = 0; n < NLD; ++n) {
    const int trow = RPW * wave + RPI * n + ld_rr;
    ld_off[n] = uint32_t(trow * ROWB + 16 * ((lane % CH) ^ tile_sw<D>(trow)));
  }
  // Prefetch cursor: (pblk, ph) is the next (query block, head of the group) to fetch.  Query blocks are walked
  // from the document's LAST block backwards: every KV tile of a document then starts at the same block, so the
  // workgroups that run side by side on an XCD (same KV head, neighbouring KV tiles) fetch the same Q/dO tiles
  // at about the same time and share them in that XCD's L2.  Past the last block the cursor stays on it (or wraps,
  // see above): every iteration issues the same number of loads, which keeps the s_waitcnt bookkeeping constant.
  const int64_t head_stride = BWD_BQ * D * 2;            // bytes between the tiles of consecutive heads of a block
  const int64_t block_stride = int64_t(Hq) * head_stride;  // ... of consecutive blocks, same head
  // the wave's auxiliary array: log2e*LSE (wave 0), -Delta (wave 1), slot positions (wave 2); wave 3's load goes to
  // a spare area, so that every wave issues the same number of loads, and brings the peers' progress counters (below)
  const int64_t aux_hstride = wave < 2 ? padded : 0;
  const int aux_bstep = wave == 3 ? 0 : BWD_BQ;
  // Convoy.  The workgroups of one KV head that run on one XCD (units peer_stride apart) walk the same Q/dO tiles
  // from the same last block; as long as they are within an L2's worth of steps of each other only the first
  // of them fetches a tile from beyond the L2.  Each workgroup publishes the number of steps it has taken; wave 3's
  // auxiliary load (a filler otherwise) fetches the counters of up to 32 such peers along with every stage, and a
  // workgroup that finds a peer between CONVOY and CONVOY_REACH steps behind sleeps about 4 microseconds per step
  // until the peer has caught up (peers further behind are left alone; the slowest workgroup never sleeps, so nothing
  // can dead-lock, and results do not depend on any of this).  Counters are published every eighth step: a store per
  // step would sit in the wave's memory queue ahead of the loads its s_waitcnt bookkeeping waits for.
  // Only units that stream at least 64 MB of Q/dO tiles wait for peers: on shorter ones (documents below about 32K
  // rows at four heads per group) the tiles missed in L2 are cheap and the waiting for later-started peers is not
  // (measured: -13 % on batches of 16K-token documents with every unit waiting, nothing gained there).
  constexpr int CONVOY = (1 << 20) / (2 * BWD_BQ * ROWB);  // 1 MB of Q/dO tiles (a quarter of an L2), in steps
  constexpr int CONVOY_REACH = 3 * CONVOY;                 // peers further behind than this are left alone
  constexpr int CONVOY_MIN_STEPS = (64 << 20) / (2 * BWD_BQ * ROWB);
  if (!cont) {
    pblk = n_blocks - 1, ph = 0, pst = 0;
    pst_addr = lds0;
    const int64_t tile0 = (int64_t(u.slot_begin / BWD_BQ + pblk) * Hq + hk * G) * head_stride;
    q_tile = reinterpret_cast<const char *>(Qs) + tile0, do_tile = reinterpret_cast<const char *>(dOs) + tile0;
    aux_ptr = (wave == 0 ? l2_slot + int64_t(hk) * G * padded
               : wave == 1 ? delta_slot + int64_t(hk) * G * padded
                           : reinterpret_cast<const float *>(slot_pos)) +
              u.slot_begin + int64_t(pblk) * BWD_BQ + lane;
    // Only workgroups of a single unit have peers: those come first in the list, and their index is their unit's.
    if (wave == 3) {
      const int grp = 32 * peer_stride;
      const int pu = me - me % grp + me % peer_stride + peer_stride * lane;
      const int32_t *pp = progress + n_single;  // a counter that stays 0: "not running"
      if (!CHAIN && lane < 32 && pu < n_single && pu != me) {
        const BwdUnit o = units[pu];
        if (o.slot_end == u.slot_end && o.kv_head == u.kv_head && o.slot_end > o.slot_begin) pp = progress + pu;
      }
      aux_ptr = reinterpret_cast<const float *>(pp);
    }
    q_first = q_tile, do_first = do_tile, aux_first = aux_ptr;
  }
  int32_t *const my_progress = progress + me;
  auto publish = [&](int steps) __attribute__((always_inline)) {  // call from wave 3 only; chains have no peers
    if (!CHAIN && lane == 0) __hip_atomic_store(my_progress, steps, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  const uint32_t aux_lds = wave == 0 ? S::L2_OFF : wave == 1 ? S::DL_OFF : wave == 2 ? S::POS_OFF : S::SPARE_OFF;
  constexpr int LPI = 2 * NLD + 1;  // loads per wave per iteration
  // The loads of one (block, head) come in LPI pieces, so that the pipelined path can hand them to the memory
  // pipeline a few at a time between its MFMAs (a burst of LPI loads from all four waves at once stalls the
  // issuing waves for hundreds of cycles).  The last piece moves the cursor.
  auto issue_piece = [&](int i) __attribute__((always_inline)) {
    if (i < 2 * NLD) {
      const int n = i >> 1;
      load_lds16_sbase((i & 1) ? do_tile : q_tile, ld_off[n],
                       pst_addr + ((i & 1) ? S::DO_OFF : S::Q_OFF) + (RPW * wave + RPI * n) * ROWB);
      return;
    }
    load_lds4_at_fresh(aux_ptr, pst_addr + aux_lds);  // device scope for all four waves: no branch; the others' arrays are read once anyway
    pst = pst + 1 == NST ? 0 : pst + 1;
    pst_addr = pst == 0 ? lds0 : pst_addr + S::STAGE;
    if (ph + 1 < Gu) {  // next tile of the group, same block
      ++ph;
      q_tile += head_stride, do_tile += head_stride, aux_ptr += aux_hstride;
    } else if (pblk > 0) {  // first head of the group, previous block
      ph = 0;
      --pblk;
      q_tile -= (Gu - 1) * head_stride + block_stride, do_tile -= (Gu - 1) * head_stride + block_stride;
      aux_ptr -= (Gu - 1) * aux_hstride + aux_bstep;
    } else if (wrap) {  // past the end: the next unit's first (block, head), which is this unit's
      ph = 0;
      pblk = n_blocks - 1;
      q_tile = q_first, do_tile = do_first, aux_ptr = aux_first;
    }  // else: past the end, keep re-fetching the final (block, head)
  };
  auto issue_next = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < LPI; ++i) issue_piece(i);
  };
  // Load pieces of the pipelined path go out during its gradient phases (few other instructions there), spread so
  // that the four waves' pieces do not pile up in the memory pipeline (one 1 KB load per 16 cycles per CU): by MFMA
  // slot of the phase, after the barrier in B(2 it + 1), then in B(2 it + 2), then in B(2 it + 3) before its
  // barrier (the cursor piece last).  slot -> piece index, or -1.
  constexpr int NPOST = D == 128 ? 2 : 1, NMID = D == 128 ? 5 : 3, NPRE = LPI - NPOST - NMID;
  static_assert(NPRE >= 1 && NPRE <= 2, "piece schedule");
  auto piece_of = [](int qb, int m) constexpr -> int {
    if (D == 128) {
      if (qb == 1) return m == 10 ? 0 : m == 13 ? 1 : m == 4 ? NPOST + NMID : m == 6 ? NPOST + NMID + 1 : -1;
      return m == 4 ? NPOST : m == 6 ? NPOST + 1 : m == 10 ? NPOST + 2 : m == 12 ? NPOST + 3 : m == 14 ? NPOST + 4 : -1;
    }
    if (qb == 1) return m == 6 ? 0 : m == 2 ? NPOST + NMID : -1;
    return m == 2 ? NPOST : m == 3 ? NPOST + 1 : m == 6 ? NPOST + 2 : -1;
  };
  constexpr int NB1 = NPOST;
  constexpr int LP1 = NB1;  // pieces of the newest block that are issued before the pipelined path takes over

  if (n_it > 0 && !cont) {
    issue_next();  // blocks 0 .. 3: four ahead; the last one is completed further down
    issue_next();
    issue_next();
#pragma unroll
    for (int i = 0; i < LP1; ++i) issue_piece(i);
  }

  // resident K, V fragments of the wave's 32 keys (B operands of S = Q K^T and dP = dO V^T).  Keys past the
  // document's last key are clamped; their positions exceed every query position, so they are masked.
  auto kv_offset = [&](const BwdUnit &x) __attribute__((always_inline)) {
    const int key = min(kw0 + r, x.n_valid - 1);
    return (size_t(x.kv_row + key) * Hkv + hk) * D + 8 * g;
  };
  // (If they were fetched ahead, the previous unit has moved them into place at its end.)  All register loads are
  // complete from here on, so the compiler places no vector-memory waits inside the loops (they would drain the
  // direct-load queue every iteration).
  if (!have_kv) {
    const size_t off = kv_offset(u);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      kf[s] = *reinterpret_cast<const bf16x8 *>(K + off + 16 * s);
      vf[s] = *reinterpret_cast<const bf16x8 *>(V + off + 16 * s);
    }
    wait_vmcnt<0>();
#pragma unroll
    for (int s = 0; s < NS; ++s) pin_acc(kf[s]), pin_acc(vf[s]);
  }
  if (!cont) {
#pragma unroll
    for (int s = 0; s < NS; ++s) qoff[s] = lds0 + tile_off<D>(r, 2 * s + g);
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
      for (int b = 0; b < NDB; ++b)
        toff[h2][b] = lds0 + tile_off<D>(4 * g + (li >> 2) + 8 * h2, 4 * b + 2 * dh + ((li >> 1) & 1)) + 8 * (li & 1);
    // qoff / auxq (natural reads and row statistics of the score chain) and toff / auxo (transposed reads, row
    // statistics of the vector work) are byte offsets into a stage, advanced once per block, so that every LDS read
    // is (loop-carried register) + (immediate).  In the pipelined path the first pair runs one stage ahead of the
    // second for part of the time.
    auxo = lds0 + 16 * g, auxq = auxo;
    stage = 0, qstage = 0;
  }

  f32x16 acc_dk[NDB], acc_dv[NDB];
#pragma unroll
  for (int b = 0; b < NDB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc_dk[b][i] = 0.f, acc_dv[b][i] = 0.f;

  if (!cont) barrier_nofence();

  // ------------------------------------------------------------------------------------------------
  // Pipelined path for blocks entirely below the diagonal.  With one wave per SIMD nothing hides a latency except
  // this wave's own instructions, so the sub-blocks k = 0, 1, .. (two per query block) are software-pipelined and
  // the matrix pipe, the vector ALU, the LDS and the memory pipeline all get their work a little at a time:
  //   phase A(k): the score MFMAs of sub-block k+1 (S and dP - Delta: 2 NS MFMAs into architectural registers; the
  //               dP chain starts from -Delta as its C operand); between them P = exp2(c S - L2) of sub-block k.
  //               Natural Q/dO fragments are held PA k-steps ahead and re-fetched as they are consumed; the first
  //               half of the transposed fragments of sub-block k is fetched meanwhile.
  //   phase B(k): the gradient MFMAs of sub-block k in the order dV, dK (query rows 0..15), dV, dK (rows 16..31);
  //               dS = P (dP - Delta) is formed during the first dV group.  The second half of the transposed
  //               fragments replaces the first as it is consumed; the first natural fragments of sub-block k+2,
  //               L2 of sub-block k+1 and -Delta of sub-block k+2 are fetched meanwhile.
  // sched_barrier fences pin that order.  Block it+1 is read from phase B of block it's first sub-block on, so the
  // workgroup barrier in the middle of the last phase B of block it-1 (after which nobody reads block it-1's stage
  // any more: the rest of the phase works from registers) waits until block it+1 has landed, and the loads of block
  // it+3 into the stage it frees are handed out one at a time over the following phases: four stages, at most
  // two blocks in flight.
  bf16x8 opq[PA], opd[PA];  // natural fragments, k-steps s .. s+PA-1 of the score chain in flight
  bf16x8 opb[2 * NDB];      // transposed fragments: [2b] = dO^T, [2b+1] = Q^T of column block b
  auto advance_q = [&]() __attribute__((always_inline)) {
    const int adv = qstage == NST - 1 ? -(NST - 1) * S::STAGE : S::STAGE;
    qstage = qstage == NST - 1 ? 0 : qstage + 1;
#pragma unroll
    for (int s = 0; s < NS; ++s) qoff[s] += adv;
    auxq += adv;
  };
  auto advance_t = [&]() __attribute__((always_inline)) {
    const int adv = stage == NST - 1 ? -(NST - 1) * S::STAGE : S::STAGE;
    stage = stage == NST - 1 ? 0 : stage + 1;
#pragma unroll
    for (int b = 0; b < NDB; ++b) toff[0][b] += adv, toff[1][b] += adv;
    auxo += adv;
  };
  constexpr int SUB = 32 * ROWB, HALF = 16 * ROWB;
  int it = 0;
  if (n_fast > 0) {
    f32x16 sc[2], dp[2];  // score tiles S and dP - Delta of sub-blocks k (even: [0], odd: [1])
    f32x16 ndt;           // -Delta of the 16 query rows of this lane (C operand layout), for the next dP chain
    f32x4 l2v[4];         // log2e*LSE of the 16 query rows of this lane, sub-block k
    uint32_t pw[8], dw[8];  // P and dS of sub-block k, packed
    float pv[16];           // P of sub-block k
    auto load_l2 = [&](int off) __attribute__((always_inline)) {
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) l2v[i4] = lds_ld<f32x4>(S::L2_OFF + off + 32 * i4);
    };
    auto load_nd = [&](int off) __attribute__((always_inline)) {
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 x = lds_ld<f32x4>(S::DL_OFF + off + 32 * i4);
#pragma unroll
        for (int e = 0; e < 4; ++e) ndt[4 * i4 + e] = x[e];
      }
    };
    // P of query row 4 i4 + e of this lane's 16 (e = 0..3).  The vector work is written as volatile asm statements
    // (exp2_fma_pinned and friends): they stay in the MFMA slot they are written in, which plain arithmetic would not
    // (the instruction selector hoists side-effect-free code across the sched_barrier fences of earlier slots).  A
    // pair of probabilities is packed to bf16 one slot after its second exponential, so that no wait state is
    // needed between the transcendental and the conversion that reads it.
    auto vec_p1 = [&](const f32x16 &sa, int i4, int e) __attribute__((always_inline)) {
      pv[4 * i4 + e] = exp2_fma_pinned(sa[4 * i4 + e], c, l2v[i4][e]);
    };
    auto pack_p = [&](int k) __attribute__((always_inline)) { pw[k] = pack_bf16_pinned(pv[2 * k], pv[2 * k + 1]); };
    auto vec_ds = [&](const f32x16 &da, int i4) __attribute__((always_inline)) {
      mul_pack_bf16_pinned(pv[4 * i4], pv[4 * i4 + 1], pv[4 * i4 + 2], pv[4 * i4 + 3], da[4 * i4], da[4 * i4 + 1],
                           da[4 * i4 + 2], da[4 * i4 + 3], dw[2 * i4], dw[2 * i4 + 1]);
    };
    // Score chain of one sub-block into (sw, dpw); nat = offset of its natural tiles from qoff's stage.  With VEC,
    // P of the first 12 of the lane's 16 rows of (sr) is formed between the MFMAs (the rest follows in phase B: the
    // vector ALU's share of a phase must fit under its MFMAs), and the transposed first-half fragments of the
    // sub-block at offset `tro` of toff's stage are fetched.
    auto phase_a = [&](f32x16 &sw, f32x16 &dpw, const f32x16 &sr, int nat, int tro, bool vec)
                       __attribute__((always_inline)) {
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        // every MFMA is followed by its share of the other work (one transposed fragment half, one exponential),
        // so that the next one finds the matrix pipe free
        const int X = ((s & 1) ? S::Q_OFF : S::DO_OFF) + tro;
        bf16x4 tlo, thi;
        if (s == 0) mfma32_v_first(sw, opq[0], kf[0]);
        else mfma32_v(sw, opq[s % PA], kf[s]);
        if (s + PA < NS) opq[s % PA] = lds_read8_at(S::Q_OFF + nat + qoff[s + PA]);
        if (vec) {
          tlo = lds_read_tr4_at(X + toff[0][s >> 1]);
          if constexpr (NS == 8) {  // pair s in step s (one exponential per MFMA), packed in step s + 1
            if (s >= 1 && s < 7) pack_p(s - 1);
            if (s < 6) vec_p1(sr, s >> 1, 2 * (s & 1));
          } else {  // pairs 2s and 2s+1 in step s (two exponentials per MFMA), each packed one MFMA later
            if (s >= 1) pack_p(2 * s - 1);
            if (s < 3) vec_p1(sr, s, 0), vec_p1(sr, s, 1);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (s == 0) mfma32_v_first(dpw, opd[0], vf[0], ndt);
        else mfma32_v(dpw, opd[s % PA], vf[s]);
        if (s + PA < NS) opd[s % PA] = lds_read8_at(S::DO_OFF + nat + qoff[s + PA]);
        if (vec) {
          thi = lds_read_tr4_at(X + toff[1][s >> 1]);
          opb[s] = join(tlo, thi);
          if constexpr (NS == 8) {
            if (s < 6) vec_p1(sr, s >> 1, 2 * (s & 1) + 1);
          } else {
            if (s < 3) pack_p(2 * s), vec_p1(sr, s, 2), vec_p1(sr, s, 3);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // In the loop the tuples written here are next read by the vector ALU a whole phase B (16 MFMAs) later, and the
      // tuples the following chain overwrites were last read in that phase B: only the first call needs wait states.
      if (vec) mfma_chain_end(sw, dpw, ndt);
      else mfma_settle(sw, dpw, ndt);
    };

    // blocks 0 and 1 have landed (this wave's part); block 2 and the issued part of block 3 may be in flight.
    // (A continued stream is in that state already, for every wave: the previous unit's last barrier saw to it.)
    if (!cont) {
      wait_vmcnt<LPI + LP1>();
      barrier_nofence();
    }
#pragma unroll
    for (int s = 0; s < PA; ++s) {
      opd[s] = lds_read8_at(S::DO_OFF + qoff[s]);
      opq[s] = lds_read8_at(S::Q_OFF + qoff[s]);
    }
    load_nd(auxq);
    phase_a(sc[0], dp[0], sc[0], 0, 0, false);
#pragma unroll
    for (int s = 0; s < PA; ++s) {
      opd[s] = lds_read8_at(S::DO_OFF + SUB + qoff[s]);
      opq[s] = lds_read8_at(S::Q_OFF + SUB + qoff[s]);
    }
    load_l2(auxo);
    load_nd(auxq + 32 * 4);
    if (fetch_kv) {
      const size_t off = kv_offset(nu);
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        kfn[s] = *reinterpret_cast<const bf16x8 *>(K + off + 16 * s);
        vfn[s] = *reinterpret_cast<const bf16x8 *>(V + off + 16 * s);
      }
    }

    for (; it < n_fast; ++it) {
      // wave 3: a peer's counter as of about three steps ago (the other waves read their own filler)
      const int peer_steps = lds_ld<int>(auxo - 16 * g + S::SPARE_OFF + 4 * lane);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        // ---- phase A: scores of the next sub-block (the other half of this block, or the first half of the
        // next block), P of this one
        if (qb == 0) phase_a(sc[1], dp[1], sc[0], SUB, 0, true);
        else phase_a(sc[0], dp[0], sc[1], 0, SUB, true);
        if (qb == 0) advance_q();  // natural reads and chain statistics now address block it+1
        // ---- phase B
        const int QT = S::Q_OFF + qb * SUB, DOT = S::DO_OFF + qb * SUB;  // this sub-block's tiles inside the stage
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          if (qb == 1 && t == 1) {
            // All LDS reads of block it's stage have been issued (the transposed second halves just above).
            // Block it+2 must have landed (this wave's part): only block it+3 may be in flight.
            wait_vmcnt<LPI>();
            barrier_nofence();  // waits for this wave's LDS reads, then for everybody
            advance_t();        // transposed reads and vector statistics now address block it+1
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int w = 0; w < 2; ++w) {  // w = 0: dV group, w = 1: dK group
#pragma unroll
            for (int b = 0; b < NDB; ++b) {
              const int m = (2 * t + w) * NDB + b;  // MFMA number inside the phase
              if (w == 0) {
                const bf16x8 pb =
                    __builtin_bit_cast(bf16x8, u32x4{pw[4 * t], pw[4 * t + 1], pw[4 * t + 2], pw[4 * t + 3]});
                acc_dv[b] = mfma32(opb[2 * b], pb, acc_dv[b]);
                if (t == 0)  // rows 16..31 of this sub-block into the registers just consumed
                  opb[2 * b] = join(lds_read_tr4_at(DOT + HALF + toff[0][b]), lds_read_tr4_at(DOT + HALF + toff[1][b]));
              } else {
                const bf16x8 db =
                    __builtin_bit_cast(bf16x8, u32x4{dw[4 * t], dw[4 * t + 1], dw[4 * t + 2], dw[4 * t + 3]});
                acc_dk[b] = mfma32(opb[2 * b + 1], db, acc_dk[b]);
                if (t == 0)
                  opb[2 * b + 1] = join(lds_read_tr4_at(QT + HALF + toff[0][b]), lds_read_tr4_at(QT + HALF + toff[1][b]));
              }
              // the vector ALU's share of this phase: dS of rows 0..7 before the first dK group, the last quarter
              // of P before the second dV group, dS of rows 8..15 before the second dK group
              if constexpr (NDB == 4) {
                if (m == 0) vec_ds(dp[qb], 0);
                if (m == 1) vec_ds(dp[qb], 1);
                if (m == 2) vec_p1(sc[qb], 3, 0), vec_p1(sc[qb], 3, 1);
                if (m == 3) vec_p1(sc[qb], 3, 2), vec_p1(sc[qb], 3, 3), pack_p(6);  // a pack never directly follows
                if (m == 4) pack_p(7);                                              // the exponentials it reads
                if (m == 8) vec_ds(dp[qb], 2);
                if (m == 9) vec_ds(dp[qb], 3);
              } else {
                if (m == 0) vec_ds(dp[qb], 0), vec_ds(dp[qb], 1);
                if (m == 1) vec_p1(sc[qb], 3, 0), vec_p1(sc[qb], 3, 1);
                if (m == 2) vec_p1(sc[qb], 3, 2), vec_p1(sc[qb], 3, 3), pack_p(6);
                if (m == 3) pack_p(7);
                if (m == 4) vec_ds(dp[qb], 2), vec_ds(dp[qb], 3);
              }
              // first natural fragments of sub-block k+2 (block it+1: first half for qb == 0, second for qb == 1)
#pragma unroll
              for (int o = (2 * PA * m) / (4 * NDB); o < (2 * PA * (m + 1)) / (4 * NDB); ++o) {
                const int sn = o >> 1;
                if (o & 1) opq[sn] = lds_read8_at(S::Q_OFF + qb * SUB + qoff[sn]);
                else opd[sn] = lds_read8_at(S::DO_OFF + qb * SUB + qoff[sn]);
              }
              // load pieces: the block that the barrier has just made room for (qb == 1), the rest of it one
              // phase B later (qb == 0)
              if (piece_of(qb, m) >= 0) issue_piece(piece_of(qb, m));
              __builtin_amdgcn_sched_barrier(0);
            }
          }
          // L2 of sub-block k+1 and -Delta of sub-block k+2 (the chain of sub-block k+1 has consumed its own)
          if (t == 0) {
            load_l2(qb == 0 ? auxo + 32 * 4 : auxq);
            load_nd(qb == 0 ? auxq : auxq + 32 * 4);
          }
        }
      }
      if (wave == 3) {
        if ((it & 7) == 7) publish(it + 1);
        const int lead = it + 1 - peer_steps;
        if (n_it >= CONVOY_MIN_STEPS && __any(peer_steps > 0 && lead > CONVOY && lead <= CONVOY_REACH))
          __builtin_amdgcn_s_sleep(127);
      }
    }
  }

  if (n_it > 0 && !wrap) {  // complete the block whose first pieces were issued last
#pragma unroll
    for (int i = LP1; i < LPI; ++i) issue_piece(i);
  }
  // ------------------------------------------------------------------------------------------------
  // General path: blocks that straddle the diagonal (mask, skip of invisible sub-blocks).  One barrier before
  // and one after the compute, then the refill of this stage.
  for (; it < n_it; ++it) {
    wait_vmcnt<3 * LPI>();  // block `it` has landed (this wave's part); blocks it+1 .. it+3 may be in flight
    barrier_nofence();
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int QT = S::Q_OFF + qb * SUB, DOT = S::DO_OFF + qb * SUB;
      // sub-block entirely above the diagonal for this wave's keys? (slot positions are sorted)
      const int sub_max_pos = lds_ld<int>(lds0 + stage * S::STAGE + S::POS_OFF + (32 * qb + 31) * 4);
      if (sub_max_pos < u.key_pos0 + kw0) continue;
      f32x16 sa, pa;
      f32x4 l2v[4], ndv[4];  // log2e*LSE and -Delta of this lane's 16 query rows
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int qo = (32 * qb + 8 * i4) * 4;
        ndv[i4] = lds_ld<f32x4>(S::DL_OFF + qo + auxo);
        l2v[i4] = lds_ld<f32x4>(S::L2_OFF + qo + auxo);
      }
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const bf16x8 qf = lds_read8_at(QT + qoff[s]), df = lds_read8_at(DOT + qoff[s]);
        if (s == 0) {
          mfma32_v_first(sa, qf, kf[0]);
          mfma32_v_first(pa, df, vf[0]);
        } else {
          mfma32_v(sa, qf, kf[s]);
          mfma32_v(pa, df, vf[s]);
        }
      }
      mfma_settle(sa, pa);
      uint32_t pw[8], dw[8];
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const u32x4 pv = lds_ld<u32x4>(S::POS_OFF + (32 * qb + 8 * i4) * 4 + auxo);
        const int pos4[4] = {int(pv[0]), int(pv[1]), int(pv[2]), int(pv[3])};
        float p[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          p[e] = key_pos <= pos4[e] ? fast_exp2(fmaf(sa[4 * i4 + e], c, -l2v[i4][e])) : 0.f;
        pw[2 * i4] = pack_bf16(p[0], p[1]);
        pw[2 * i4 + 1] = pack_bf16(p[2], p[3]);
        dw[2 * i4] = pack_bf16(p[0] * (pa[4 * i4] + ndv[i4][0]), p[1] * (pa[4 * i4 + 1] + ndv[i4][1]));
        dw[2 * i4 + 1] = pack_bf16(p[2] * (pa[4 * i4 + 2] + ndv[i4][2]), p[3] * (pa[4 * i4 + 3] + ndv[i4][3]));
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pb = __builtin_bit_cast(bf16x8, u32x4{pw[4 * t], pw[4 * t + 1], pw[4 * t + 2], pw[4 * t + 3]});
        const bf16x8 db = __builtin_bit_cast(bf16x8, u32x4{dw[4 * t], dw[4 * t + 1], dw[4 * t + 2], dw[4 * t + 3]});
        const int ro = t * HALF;
#pragma unroll
        for (int b = 0; b < NDB; ++b) {
          const bf16x8 dot_t = join(lds_read_tr4_at(DOT + ro + toff[0][b]), lds_read_tr4_at(DOT + ro + toff[1][b]));
          acc_dv[b] = mfma32(dot_t, pb, acc_dv[b]);
          const bf16x8 q_t = join(lds_read_tr4_at(QT + ro + toff[0][b]), lds_read_tr4_at(QT + ro + toff[1][b]));
          acc_dk[b] = mfma32(q_t, db, acc_dk[b]);
        }
      }
    }
    barrier_nofence();  // everybody is done with this stage
    issue_next();       // block it+4 into it
    advance_q();
    advance_t();
    if (wave == 3) publish(it + 1);
  }
  if (wave == 3) publish(-1);  // finished: peers no longer wait for this workgroup
  if (!wrap) wait_vmcnt<0>();  // nothing may still be writing LDS when the stream ends
  // The next unit's K and V take their place now, before the stores: the wait for them that the compiler puts here
  // waits for everything this wave has in flight, which at this point is a few stream loads issued a step ago.
  if (fetch_kv) {
#pragma unroll
    for (int s = 0; s < NS; ++s) kf[s] = kfn[s], vf[s] = vfn[s];
#pragma unroll
    for (int s = 0; s < NS; ++s) pin_acc(kf[s]), pin_acc(vf[s]);
  }

  // ---- write dK (scaled) and dV of the wave's 32 keys as whole lines through the wave's LDS patch, like
  // store_tile_as_lines (stored straight from the accumulator layout, the 64 instructions per wave kept the CU's
  // address unit busy for longer than a short unit's steps take).  Written out here, with the addresses formed after
  // the LDS reads they wait for: the helper's order costs a chained unit a few tenths of a microsecond more.
  {
    const uint32_t patch = lds0 + S::OUT_OFF + wave * PATCH_BYTES;
    const uint32_t wr = patch + r * PATCH_ROW_BYTES + 8 * g;  // + 64 (b & 1) + 16 q4: values 32 b + 8 q4 + 4 g .. + 3
    const int orow = lane >> 3, ocol = lane & 7;          // the lane's row (+ 8 i) and 16-byte piece of the patch
    const uint32_t rd = patch + orow * PATCH_ROW_BYTES + 16 * ocol;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int h = 0; h < NDB / 2; ++h) {
#pragma unroll
        for (int bb = 0; bb < 2; ++bb)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const f32x16 &a = t == 0 ? acc_dk[2 * h + bb] : acc_dv[2 * h + bb];
            const float f = t == 0 ? scale : 1.0f;
            const u32x2 w = {pack_bf16(a[4 * q4] * f, a[4 * q4 + 1] * f), pack_bf16(a[4 * q4 + 2] * f, a[4 * q4 + 3] * f)};
            *(CA_LDS u32x2 *)(wr + 64 * bb + 16 * q4) = w;
          }
        bf16_t *const out = t == 0 ? dK : dV;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const u32x4 x = *(const CA_LDS u32x4 *)(rd + 8 * i * PATCH_ROW_BYTES);
          const int key = kw0 + orow + 8 * i;
          if (key < u.n_valid)
            *reinterpret_cast<u32x4 *>(out + (size_t(u.kv_row + key) * Hkv + hk) * D + 64 * h + 8 * ocol) = x;
        }
      }
  }
  // every wave is done with the LDS stages before a new stream refills them
  if (has_next && !wrap) __syncthreads();
  cont = wrap, have_kv = fetch_kv;
  u = nu, nu = nnu;
  }
}

// Units that run alone and chains of short units in one launch, so that the dispatcher hands them out longest first
// whatever they are.
template <int D>
__global__ __launch_bounds__(256, 1) void ca_bwd_dkv_kernel(const BwdUnit *__restrict__ units, int n_single,
                                                            const int32_t *__restrict__ slot_pos,
                                                            const bf16_t *__restrict__ Qs, const bf16_t *__restrict__ K,
                                                            const bf16_t *__restrict__ V, const bf16_t *__restrict__ dOs,
                                                            const float *__restrict__ l2_slot,
                                                            const float *__restrict__ delta_slot,
                                                            bf16_t *__restrict__ dK, bf16_t *__restrict__ dV,
                                                            int32_t *progress, int peer_stride, int Hq, int Hkv,
                                                            int64_t padded, float scale) {
  const int me = int(blockIdx.x);  // index of the workgroup = index of its first unit
  const BwdUnit first = units[me];
  if (first.count <= 1)
    dkv_workgroup<D, false>(me, first, units, n_single, slot_pos, Qs, K, V, dOs, l2_slot, delta_slot, dK, dV, progress,
                            peer_stride, Hq, Hkv, padded, scale);
  else
    dkv_workgroup<D, true>(me, first, units, n_single, slot_pos, Qs, K, V, dOs, l2_slot, delta_slot, dK, dV, progress,
                           peer_stride, Hq, Hkv, padded, scale);
}

static void launch_fill(void *p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return;
  const int64_t n16 = int64_t(bytes / 16);
  const unsigned blocks = unsigned(std::min<int64_t>((n16 + 255) / 256, 256 * 32));
  hipLaunchKernelGGL(ca_fill_zero_kernel, dim3(blocks), dim3(256), 0, st, static_cast<u32x4 *>(p), n16);
}

template <class F>
static hipError_t set_smem(F kern, int bytes, int device, std::atomic<bool> *done) {
  // once per device; two threads that meet here both set the same value, which is harmless
  if (!done[device & 15].load(std::memory_order_acquire)) {
    hipError_t e =
        hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    done[device & 15].store(true, std::memory_order_release);
  }
  return hipSuccess;
}

template <int D>
static hipError_t launch_bwd_t(const ca_plan_t *p, const void *q, const void *k, const void *v, const void *o,
                               const void *d_o, const float *lse, void *dq, void *dk, void *dv, void *ws,
                               hipStream_t st, hipEvent_t *ev) {
  if (ev) (void)hipEventRecord(ev[0], st);
  const size_t q_elems = size_t(p->total_q) * p->hq * D, kv_elems = size_t(p->total_kv) * p->hkv * D;
  const int64_t padded = int64_t(p->slot_row.size());
  float *delta_slot = static_cast<float *>(ws);
  float *l2_slot = reinterpret_cast<float *>(static_cast<char *>(ws) + p->ws_off_l2);
  float *delta_kv = reinterpret_cast<float *>(static_cast<char *>(ws) + p->ws_off_delta_kv);
  float *l2_kv = reinterpret_cast<float *>(static_cast<char *>(ws) + p->ws_off_l2_kv);
  bf16_t *q_sorted = reinterpret_cast<bf16_t *>(static_cast<char *>(ws) + p->ws_off_qs);
  bf16_t *do_sorted = reinterpret_cast<bf16_t *>(static_cast<char *>(ws) + p->ws_off_dos);
  int32_t *progress = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + p->ws_off_prog);
  // rows that belong to no work unit (KV outside every scheduled document, Q rows outside every task)
  if (!p->kv_covered) {
    launch_fill(dk, kv_elems * 2, st);
    launch_fill(dv, kv_elems * 2, st);
  }
  if (!p->q_covered) launch_fill(dq, q_elems * 2, st);
  if (padded > 0) {
    const int n_progress = p->bwd_workgroups + 64;
    const int64_t threads = std::max<int64_t>(padded * p->hq * (D / 8), n_progress);
    hipLaunchKernelGGL(ca_bwd_prep_kernel, dim3(unsigned((threads + 255) / 256)), dim3(256), 0, st, p->d_slot_row,
                       p->d_block_rpk, static_cast<const bf16_t *>(q), static_cast<const bf16_t *>(o),
                       static_cast<const bf16_t *>(d_o), lse, delta_slot, l2_slot, delta_kv, l2_kv, q_sorted, do_sorted,
                       progress, n_progress, padded, p->total_q, p->hq, p->hq / p->hkv, D);
  }
  if (ev) (void)hipEventRecord(ev[1], st);
  if (!p->bwd_units.empty()) {
    auto kern = ca_bwd_dkv_kernel<D>;
    static std::atomic<bool> done[16];
    hipError_t e = set_smem(kern, DkvSmem<D>::TOTAL, p->device, done);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(unsigned(p->bwd_workgroups)), dim3(256), DkvSmem<D>::TOTAL, st, p->d_bwd_units,
                       p->bwd_single, p->d_pos_kv, q_sorted, static_cast<const bf16_t *>(k),
                       static_cast<const bf16_t *>(v), do_sorted, l2_kv, delta_kv, static_cast<bf16_t *>(dk),
                       static_cast<bf16_t *>(dv), progress, p->peer_stride, p->hq, p->hkv, padded, p->scale);
  }
  if (ev) (void)hipEventRecord(ev[2], st);
  if (!p->fwd_units.empty()) {
    auto kern = ca_bwd_dq_kernel<D>;
    static std::atomic<bool> done[16];
    hipError_t e = set_smem(kern, DqSmem<D>::TOTAL, p->device, done);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(unsigned(p->fwd_units.size())), dim3(512), DqSmem<D>::TOTAL, st, p->d_fwd_units,
                       p->d_slot_row, p->d_slot_pos, static_cast<const bf16_t *>(q), static_cast<const bf16_t *>(k),
                       static_cast<const bf16_t *>(v), static_cast<const bf16_t *>(d_o), l2_slot, delta_slot,
                       static_cast<bf16_t *>(dq), p->hq, p->hkv, padded, p->scale);
  }
  if (ev) (void)hipEventRecord(ev[3], st);
  return hipGetLastError();
}

hipError_t launch_bwd(const ca_plan_t *p, const void *q, const void *k, const void *v, const void *o, const void *d_o,
                      const float *lse, void *dq, void *dk, void *dv, void *ws, hipStream_t st, hipEvent_t *ev) {
  return p->d == 128 ? launch_bwd_t<128>(p, q, k, v, o, d_o, lse, dq, dk, dv, ws, st, ev)
                     : launch_bwd_t<64>(p, q, k, v, o, d_o, lse, dq, dk, dv, ws, st, ev);
}

}  // namespace ca

