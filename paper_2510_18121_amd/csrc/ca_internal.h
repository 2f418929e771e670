// Internal definitions shared by the host planner, the launchers and the kernels.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "ca_attention.h"

namespace ca {

// Tile geometry.  Every document's sorted query rows occupy a run of "slots" padded to the plan's slot alignment
// (at most SLOT_ALIGN), so that forward tiles and backward q blocks (BWD_BQ slots) both tile the same arrays.
constexpr int SLOT_ALIGN = 256;
constexpr int FWD_BM = 256;  // query rows per forward work unit (8 waves x 32)
constexpr int FWD_BN = 64;   // keys per forward inner step
constexpr int BWD_BN = 128;  // keys owned by one backward work unit (4 waves x 32)
constexpr int BWD_BQ = 64;   // query rows per backward inner step

// One workgroup of the forward / dQ kernels: 8 waves of 32 slots each.  A full tile of a document is 256 slots of
// one query head (hp = 1).  The slots a document has left over after its full tiles are covered by head-packed units
// instead: 256 / hp slots of hp consecutive query heads of one KV group (they read the same K/V), wave w taking
// slots slot0 + 32 (w / hp) .. of head  head + w % hp  - so that short documents keep all 8 waves busy too.
struct FwdUnit {
  int32_t slot0;    // first slot of the unit
  int32_t kv_row0;  // packed KV row of the document's token 0
  int32_t n_keys;   // keys the unit needs: max position + 1
  int32_t head;     // first query head
  int32_t hp;       // query heads per unit: 1, 2, 4 or 8
};

struct BwdUnit {  // one (KV tile, KV head)
  int32_t slot_begin;  // first slot of the first q block that sees this KV tile
  int32_t slot_end;    // end of the document's slots
  int32_t slot_full;   // first q block (slot index) from which every slot sees all keys of the tile
  int32_t kv_row;      // packed KV row of the tile's first key
  int32_t n_valid;     // valid keys in the tile
  int32_t key_pos0;    // document position of the tile's first key
  int32_t kv_head;
  // Chains.  The first n_bwd_workgroups units of the list are one workgroup each; a workgroup goes on with the
  // `count - 1` units stored from index `follow` on (behind the workgroups' own units; same KV head, no longer than
  // its first).  Long units run alone (count 1); short ones are chained, because what a unit costs beyond its steps
  // (filling the pipeline, fetching K and V, draining) can then overlap with the steps of its neighbours.
  int32_t follow;
  int32_t count;  // units of this workgroup including this one; 0 in a unit that follows another
  // (block, head) tiles per query block: the heads of the KV group, or fewer where a document of at most 32 rows has
  // the rows of 2 or 4 heads packed into each 64-row tile (the heads of a group add into the same dK and dV)
  int32_t heads;
};

}  // namespace ca

struct ca_plan {
  // descriptor copy
  int32_t n_docs = 0, n_tasks = 0, hq = 0, hkv = 0, d = 0;
  int64_t total_q = 0, total_kv = 0;
  float scale = 0.f;
  std::vector<int64_t> doc_kv_start, doc_kv_len, task_q_start, task_q_len, task_q_pos, task_kv_len;
  std::vector<int32_t> task_doc;
  // schedule (host)
  std::vector<int32_t> slot_row, slot_pos;
  // for the dK/dV kernel: rows per head in the packed tiles of a 64-slot block (16 or 32; 0 = one head per tile), and
  // the position of every row of its tiles (= slot_pos except in packed blocks)
  std::vector<int32_t> block_rpk, pos_kv;
  std::vector<ca::FwdUnit> fwd_units;
  std::vector<ca::BwdUnit> bwd_units;
  int32_t bwd_workgroups = 0;  // workgroups of the dK/dV kernel: the leading units of bwd_units
  int32_t bwd_single = 0;      // so many leading workgroups are units that run alone (only those pace each other)
  int64_t fwd_steps = 0, bwd_steps = 0;
  // workspace layout for backward: [Delta fp32 hq*padded_slots][log2e*LSE fp32 hq*padded_slots]
  int slot_align = ca::SLOT_ALIGN, heads_packed = 1;  // padding of a document's slots; hp of the packed units
  size_t ws_fwd = 0, ws_bwd = 0, ws_off_l2 = 0, ws_off_qs = 0, ws_off_dos = 0, ws_off_prog = 0;
  size_t ws_off_delta_kv = 0, ws_off_l2_kv = 0;  // the row statistics once more, in the row order of the dK/dV tiles
  int peer_stride = 8;  // distance, in backward units, between units of one KV head that run on one XCD
  bool q_covered = false, kv_covered = false;  // every packed Q row / KV row belongs to some unit
  // device copies
  int device = -1;
  int32_t *d_slot_row = nullptr, *d_slot_pos = nullptr, *d_block_rpk = nullptr, *d_pos_kv = nullptr;
  ca::FwdUnit *d_fwd_units = nullptr;
  ca::BwdUnit *d_bwd_units = nullptr;
  // optional timing events (hipEvent_t, kept as void* so that host-only code needs no HIP header)
  bool profile = false;
  void *ev[7] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  bool ev_fwd = false, ev_bwd = false;
};

namespace ca {
void set_error(const std::string &msg);
int build_plan(const ca_batch_desc *desc, ca_plan_t **out);  // host only
}  // namespace ca
