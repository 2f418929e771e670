// Host-side planner: descriptor validation and the tile schedule.  Pure C++, no HIP calls.
//
// The mask of a query row depends only on its document position p (it sees keys 0..p of its own
// document; Appendix B's shard geometry), not on which CA-task carried it.  So the planner forgets task
// boundaries: per document it lists every query row present in the batch sorted by position and cuts
// that list into tiles.  Rows of different tasks of one document share tiles, which is the paper's
// composability observation (Section 3.2: throughput depends on the aggregate tokens of a fused call,
// not on their document of origin) carried below its 128-token shard granularity.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <sstream>

#include "ca_internal.h"

namespace ca {

static thread_local std::string g_err;
void set_error(const std::string &msg) { g_err = msg; }
const char *last_error() { return g_err.c_str(); }

namespace {
struct Fail {
  int code;
  std::string msg;
};
#define CA_REQUIRE(cond, code, text)        \
  do {                                      \
    if (!(cond)) {                          \
      std::ostringstream os_;               \
      os_ << text;                          \
      throw Fail{code, os_.str()};          \
    }                                       \
  } while (0)

void validate(const ca_batch_desc *d) {
  CA_REQUIRE(d != nullptr, CA_ERR_INVALID_ARG, "descriptor is null");
  CA_REQUIRE(d->n_docs >= 0 && d->n_tasks >= 0, CA_ERR_INVALID_ARG, "negative n_docs or n_tasks");
  CA_REQUIRE(d->n_q_heads >= 1 && d->n_kv_heads >= 1, CA_ERR_INVALID_ARG, "head counts must be >= 1");
  CA_REQUIRE(d->n_q_heads % d->n_kv_heads == 0, CA_ERR_UNSUPPORTED,
             "n_q_heads " << d->n_q_heads << " is not a multiple of n_kv_heads " << d->n_kv_heads);
  CA_REQUIRE(d->head_dim == 64 || d->head_dim == 128, CA_ERR_UNSUPPORTED,
             "head_dim " << d->head_dim << " not supported (64 or 128)");
  CA_REQUIRE(d->total_q >= 0 && d->total_kv >= 0, CA_ERR_INVALID_ARG, "negative total_q or total_kv");
  const int64_t lim = (int64_t(1) << 31) - 4 * SLOT_ALIGN;
  CA_REQUIRE(d->total_q < lim && d->total_kv < lim, CA_ERR_UNSUPPORTED, "total_q / total_kv beyond 2^31 rows");
  CA_REQUIRE(d->total_kv * d->n_kv_heads * d->head_dim < (int64_t(1) << 40), CA_ERR_UNSUPPORTED, "KV buffer too large");
  if (d->n_docs > 0)
    CA_REQUIRE(d->doc_kv_start && d->doc_kv_len, CA_ERR_INVALID_ARG, "document arrays are null");
  if (d->n_tasks > 0) {
    CA_REQUIRE(d->task_doc && d->task_q_start && d->task_q_len && d->task_q_pos && d->task_kv_len,
               CA_ERR_INVALID_ARG, "task arrays are null");
    CA_REQUIRE(d->n_docs > 0, CA_ERR_INVALID_ARG, "tasks given but no documents");
  }
  // documents: in bounds, pairwise disjoint KV ranges
  std::vector<int32_t> order(d->n_docs);
  std::iota(order.begin(), order.end(), 0);
  for (int i = 0; i < d->n_docs; ++i) {
    CA_REQUIRE(d->doc_kv_len[i] >= 1, CA_ERR_INVALID_ARG, "document " << i << " has kv_len " << d->doc_kv_len[i]);
    CA_REQUIRE(d->doc_kv_start[i] >= 0 && d->doc_kv_start[i] <= d->total_kv - d->doc_kv_len[i], CA_ERR_INVALID_ARG,
               "document " << i << " KV range [" << d->doc_kv_start[i] << ", +" << d->doc_kv_len[i]
                           << ") outside the packed KV buffer of " << d->total_kv << " rows");
  }
  std::sort(order.begin(), order.end(), [&](int a, int b) { return d->doc_kv_start[a] < d->doc_kv_start[b]; });
  for (int i = 1; i < d->n_docs; ++i) {
    int a = order[i - 1], b = order[i];
    CA_REQUIRE(d->doc_kv_start[a] + d->doc_kv_len[a] <= d->doc_kv_start[b], CA_ERR_INVALID_ARG,
               "KV ranges of documents " << a << " and " << b << " overlap");
  }
  // tasks: in bounds, causal geometry, pairwise disjoint Q ranges
  std::vector<int32_t> torder(d->n_tasks);
  std::iota(torder.begin(), torder.end(), 0);
  for (int t = 0; t < d->n_tasks; ++t) {
    CA_REQUIRE(d->task_doc[t] >= 0 && d->task_doc[t] < d->n_docs, CA_ERR_INVALID_ARG,
               "task " << t << " names document " << d->task_doc[t]);
    CA_REQUIRE(d->task_q_len[t] >= 1, CA_ERR_INVALID_ARG, "task " << t << " has q_len " << d->task_q_len[t]);
    CA_REQUIRE(d->task_q_start[t] >= 0 && d->task_q_start[t] <= d->total_q - d->task_q_len[t], CA_ERR_INVALID_ARG,
               "task " << t << " query range outside packed Q of " << d->total_q << " rows");
    CA_REQUIRE(d->task_q_pos[t] >= 0, CA_ERR_INVALID_ARG, "task " << t << " has negative q_pos");
    CA_REQUIRE(d->task_kv_len[t] >= 1, CA_ERR_INVALID_ARG,
               "task " << t << " has kv_len " << d->task_kv_len[t] << " (every row must see at least one key)");
    CA_REQUIRE(d->task_kv_len[t] <= d->doc_kv_len[d->task_doc[t]], CA_ERR_INVALID_ARG,
               "task " << t << ": kv_len " << d->task_kv_len[t] << " exceeds its document's resident KV "
                       << d->doc_kv_len[d->task_doc[t]]);
  }
  std::sort(torder.begin(), torder.end(), [&](int a, int b) { return d->task_q_start[a] < d->task_q_start[b]; });
  for (int i = 1; i < d->n_tasks; ++i) {
    int a = torder[i - 1], b = torder[i];
    CA_REQUIRE(d->task_q_start[a] + d->task_q_len[a] <= d->task_q_start[b], CA_ERR_INVALID_ARG,
               "query ranges of tasks " << a << " and " << b << " overlap");
  }
}

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

void schedule(ca_plan_t *p) {
  const int hq = p->hq, hkv = p->hkv, g = hq / hkv;
  // tasks of each document, by position
  std::vector<std::vector<int32_t>> by_doc(p->n_docs);
  for (int t = 0; t < p->n_tasks; ++t) by_doc[p->task_doc[t]].push_back(t);
  // heads packed into the units of partial tiles: the largest of 8, 4, 2, 1 that divides the group size; a document's
  // slots are padded to whole packed units (and to whole backward q blocks)
  const int hp = g % 8 == 0 ? 8 : g % 4 == 0 ? 4 : g % 2 == 0 ? 2 : 1;
  const int sub = FWD_BM / hp;  // slots of a packed unit
  const int align = std::max(sub, BWD_BQ);
  p->heads_packed = hp;
  p->slot_align = align;
  int64_t padded = 0;
  for (auto &v : by_doc) {
    int64_t n = 0;
    for (int t : v) n += p->task_q_len[t];
    padded += round_up(n, align);
  }
  CA_REQUIRE(padded < (int64_t(1) << 31) - SLOT_ALIGN, CA_ERR_UNSUPPORTED, "too many padded query rows");
  p->slot_row.assign(padded, -1);
  p->slot_pos.assign(padded, 0);
  p->block_rpk.assign(padded / BWD_BQ, 0);

  struct TileRef {
    int32_t cost;
    FwdUnit u;
  };
  std::vector<TileRef> ftiles;
  std::vector<BwdUnit> btiles;
  int64_t s = 0, covered_kv = 0, covered_q = 0;
  for (int t = 0; t < p->n_tasks; ++t) covered_q += p->task_q_len[t];
  for (int dd = 0; dd < p->n_docs; ++dd) {
    auto &v = by_doc[dd];
    if (v.empty()) continue;
    std::stable_sort(v.begin(), v.end(), [&](int a, int b) { return p->task_q_pos[a] < p->task_q_pos[b]; });
    // overlapping position ranges of two tasks would interleave; a merge by position keeps slots sorted
    struct Row {
      int32_t pos, row;
    };
    const int64_t s0 = s;
    // a slot's "position" is the last key its row sees: min(document position, kv_len - 1); a task with a prefix
    // shorter than its rows' positions (a shard attending a window of its context) is thereby clipped to the window
    for (int t : v)
      for (int64_t i = 0; i < p->task_q_len[t]; ++i, ++s) {
        p->slot_row[s] = int32_t(p->task_q_start[t] + i);
        p->slot_pos[s] = int32_t(std::min(p->task_q_pos[t] + i, p->task_kv_len[t] - 1));
      }
    const bool sorted = std::is_sorted(p->slot_pos.begin() + s0, p->slot_pos.begin() + s);
    if (!sorted) {  // rare: tasks of one document covering the same positions twice, or clipped below earlier tasks
      std::vector<Row> rows(s - s0);
      for (int64_t i = s0; i < s; ++i) rows[i - s0] = {p->slot_pos[i], p->slot_row[i]};
      std::stable_sort(rows.begin(), rows.end(), [](const Row &a, const Row &b) { return a.pos < b.pos; });
      for (int64_t i = s0; i < s; ++i) p->slot_pos[i] = rows[i - s0].pos, p->slot_row[i] = rows[i - s0].row;
    }
    const int32_t last_pos = p->slot_pos[s - 1];
    // A document that brings at most 32 rows: the dK/dV kernel's 64-row tiles of its one query block take the rows of
    // 4 heads (16 rows each) or 2 heads (32 rows each) of the KV group instead of one head's rows and padding.
    const int64_t n_rows = s - s0;
    const int rpk = n_rows <= 16 && g % 4 == 0 ? 16 : n_rows <= 32 && g % 2 == 0 ? 32 : 0;
    const int32_t tiles_per_block = rpk ? g / (BWD_BQ / rpk) : g;
    if (rpk) p->block_rpk[s0 / BWD_BQ] = rpk;
    const int64_t s1 = round_up(s - s0, align) + s0;
    for (; s < s1; ++s) p->slot_pos[s] = last_pos;  // padding slots: row -1, position of the last real row
    const int32_t kv_row0 = int32_t(p->doc_kv_start[dd]);
    // forward units: full tiles of 256 slots, then head-packed units over the rest
    int64_t a = s0;
    for (; a + FWD_BM <= s1; a += FWD_BM) {
      if (p->slot_row[a] < 0) break;  // pure padding
      int32_t n_keys = p->slot_pos[a + FWD_BM - 1] + 1;
      ftiles.push_back({(n_keys + FWD_BN - 1) / FWD_BN, {int32_t(a), kv_row0, n_keys, 0, 1}});
    }
    for (; a < s1; a += sub) {
      if (p->slot_row[a] < 0) break;  // pure padding
      int32_t n_keys = p->slot_pos[a + sub - 1] + 1;
      ftiles.push_back({(n_keys + FWD_BN - 1) / FWD_BN, {int32_t(a), kv_row0, n_keys, 0, int32_t(hp)}});
    }
    // backward KV tiles: every resident key of the document.  Keys beyond the last query position get a
    // unit without query blocks, which writes their zero gradient.
    const int32_t cover = last_pos + 1;
    const int32_t doc_len = int32_t(p->doc_kv_len[dd]);
    for (int32_t k0 = 0; k0 < doc_len; k0 += BWD_BN) {
      BwdUnit u{int32_t(s1), int32_t(s1), int32_t(s1), kv_row0 + k0, std::min<int32_t>(BWD_BN, doc_len - k0), k0, 0};
      u.heads = tiles_per_block;
      if (k0 < cover) {
        // first slot whose position can see key k0
        const int32_t *b = p->slot_pos.data() + s0, *e = p->slot_pos.data() + s1;
        int64_t first = std::lower_bound(b, e, k0) - b;
        first = first / BWD_BQ * BWD_BQ;
        int64_t end = s1;
        while (end - BWD_BQ >= s0 + first && p->slot_row[end - BWD_BQ] < 0) end -= BWD_BQ;  // drop pure-padding blocks
        u.slot_begin = int32_t(s0 + first);
        u.slot_end = int32_t(end);
        // blocks from here on lie entirely below the diagonal of this tile: no mask needed
        int64_t full = std::lower_bound(b, e, k0 + BWD_BN - 1) - b;
        full = (full + BWD_BQ - 1) / BWD_BQ * BWD_BQ;
        u.slot_full = int32_t(std::min<int64_t>(std::max<int64_t>(s0 + full, u.slot_begin), end));
      }
      btiles.push_back(u);
    }
    covered_kv += doc_len;
  }
  // longest first (the hardware dispatcher hands out workgroups in index order, so this is LPT
  // list scheduling); unit index modulo n_kv_heads equals the KV head, so that with workgroups dealt
  // round-robin to the 8 XCDs each L2 sees the K/V of as few KV heads as possible.
  std::stable_sort(ftiles.begin(), ftiles.end(), [](const TileRef &a, const TileRef &b) { return a.cost > b.cost; });
  p->fwd_units.reserve(ftiles.size() * hq);
  p->fwd_steps = 0;
  for (auto &t : ftiles)
    for (int i = 0; i < hq / t.u.hp; ++i) {  // KV heads fastest; inside a KV head, its groups of hp query heads
      FwdUnit u = t.u;
      u.head = (i % hkv) * g + (i / hkv) * u.hp;
      p->fwd_units.push_back(u);
      p->fwd_steps += t.cost;
    }
  std::stable_sort(btiles.begin(), btiles.end(), [](const BwdUnit &a, const BwdUnit &b) {
    return int64_t(a.slot_end - a.slot_begin) * a.heads > int64_t(b.slot_end - b.slot_begin) * b.heads;
  });
  p->pos_kv = p->slot_pos;
  for (size_t blk = 0; blk < p->block_rpk.size(); ++blk)
    if (const int rpk = p->block_rpk[blk])
      for (int i = 0; i < BWD_BQ; ++i) p->pos_kv[blk * BWD_BQ + i] = p->slot_pos[blk * BWD_BQ + i % rpk];
  p->bwd_steps = 0;
  for (auto &t : btiles) p->bwd_steps += int64_t(t.slot_end - t.slot_begin) / BWD_BQ * t.heads * hkv;
  {
    // Chains of the dK/dV kernel: consecutive KV tiles of the sorted list (equal or similar cost; the tiles of one
    // document under the same query rows are neighbours in it) whose units are short - at most CHAIN_UNIT_STEPS
    // steps each: what chaining saves per unit is a few steps' worth - go to one workgroup per KV head.  A chain
    // takes at most CHAIN_STEPS_MAX steps and CHAIN_UNITS_MAX units, and at most 1/(2 N_CU) of the short units' steps
    // still to be handed out: chains shrink towards the end of the list, so that the last workgroups of the launch
    // are small ones and the CUs finish together.
    constexpr int64_t N_CU = 256, CHAIN_UNIT_STEPS = 16, CHAIN_STEPS_MAX = 256, CHAIN_UNITS_MAX = 32;
    auto cost = [&](const BwdUnit &u) { return int64_t(u.slot_end - u.slot_begin) / BWD_BQ * u.heads; };
    int64_t remaining = 0;  // steps of short units, all KV heads
    for (auto &t : btiles)
      if (cost(t) <= CHAIN_UNIT_STEPS) remaining += cost(t) * hkv;
    struct Chain {
      size_t a, b;  // tiles [a, b) of the sorted list
      int64_t steps;
    };
    std::vector<Chain> chains;
    for (size_t a = 0; a < btiles.size();) {
      size_t b = a + 1;
      int64_t sum = cost(btiles[a]);
      if (sum <= CHAIN_UNIT_STEPS) {
        const int64_t target = std::min<int64_t>(CHAIN_STEPS_MAX, remaining / (2 * N_CU));
        while (b < btiles.size() && sum + cost(btiles[b]) <= target && int64_t(b - a) < CHAIN_UNITS_MAX)
          sum += cost(btiles[b++]);
        remaining -= sum * hkv;
      }
      chains.push_back({a, b, sum});
      a = b;
    }
    // workgroups are handed out in index order: longest first, a chain counting with all its steps
    std::stable_sort(chains.begin(), chains.end(), [](const Chain &x, const Chain &y) { return x.steps > y.steps; });
    size_t first_chain = chains.size();
    for (size_t ci = chains.size(); ci-- > 0;)
      if (chains[ci].b - chains[ci].a > 1) first_chain = ci;
    p->bwd_workgroups = int32_t(chains.size() * hkv);
    p->bwd_units.resize(size_t(p->bwd_workgroups));
    p->bwd_units.reserve(btiles.size() * hkv);
    p->bwd_single = int32_t(first_chain * hkv);
    for (size_t ci = 0; ci < chains.size(); ++ci) {
      const size_t a = chains[ci].a, b = chains[ci].b;
      for (int h = 0; h < hkv; ++h) {
        BwdUnit u = btiles[a];
        u.kv_head = h;
        u.count = int32_t(b - a);
        u.follow = b - a > 1 ? int32_t(p->bwd_units.size()) : 0;
        p->bwd_units[ci * hkv + h] = u;
        for (size_t t = a + 1; t < b; ++t) {
          BwdUnit f = btiles[t];
          f.kv_head = h;
          p->bwd_units.push_back(f);
        }
      }
    }
  }
  p->q_covered = covered_q == p->total_q;
  p->kv_covered = covered_kv == p->total_kv;
  // workspace of backward, all in slot order: per (head, slot) fp32 -Delta and log2(e)*LSE, then bf16 copies of Q
  // and dO as [block of 64 slots][head][64][head_dim] (the dK/dV kernel re-reads their 64-slot tiles once per 128-key tile: in this
  // layout a tile is one contiguous run and needs no row indices)
  const size_t per = (size_t(padded) * hq * sizeof(float) + 255) / 256 * 256;
  const size_t copy = (size_t(padded) * hq * p->d * 2 + 255) / 256 * 256;
  p->ws_off_l2 = per;
  p->ws_off_qs = 2 * per;
  p->ws_off_dos = 2 * per + copy;
  // ... and one progress counter per backward workgroup (plus a block of zeros), by which the dK/dV workgroups that walk
  // the same Q/dO tiles keep within an L2 window of each other.  Workgroups go to the 8 XCDs round robin in index
  // order (workgroup i to XCD (i + c) mod 8) and unit i has KV head i mod n_kv_heads, so units lcm(8, n_kv_heads)
  // apart share both.
  p->ws_off_delta_kv = 2 * per + 2 * copy;
  p->ws_off_l2_kv = 3 * per + 2 * copy;
  p->ws_off_prog = 4 * per + 2 * copy;
  p->peer_stride = int(std::lcm<int64_t>(8, hkv));
  p->ws_bwd = p->ws_off_prog + (size_t(p->bwd_workgroups) + 64) * sizeof(int32_t);
  p->ws_bwd = (p->ws_bwd + 255) / 256 * 256;
  p->ws_fwd = 0;
}
}  // namespace

int build_plan(const ca_batch_desc *desc, ca_plan_t **out) {
  if (!out) {
    set_error("output plan pointer is null");
    return CA_ERR_INVALID_ARG;
  }
  *out = nullptr;
  ca_plan_t *p = nullptr;
  try {
    validate(desc);
    p = new ca_plan_t();
    p->n_docs = desc->n_docs, p->n_tasks = desc->n_tasks;
    p->hq = desc->n_q_heads, p->hkv = desc->n_kv_heads, p->d = desc->head_dim;
    p->total_q = desc->total_q, p->total_kv = desc->total_kv;
    p->scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / std::sqrt(float(desc->head_dim));
    if (desc->n_docs > 0) {
      p->doc_kv_start.assign(desc->doc_kv_start, desc->doc_kv_start + desc->n_docs);
      p->doc_kv_len.assign(desc->doc_kv_len, desc->doc_kv_len + desc->n_docs);
    }
    if (desc->n_tasks > 0) {
      p->task_doc.assign(desc->task_doc, desc->task_doc + desc->n_tasks);
      p->task_q_start.assign(desc->task_q_start, desc->task_q_start + desc->n_tasks);
      p->task_q_len.assign(desc->task_q_len, desc->task_q_len + desc->n_tasks);
      p->task_q_pos.assign(desc->task_q_pos, desc->task_q_pos + desc->n_tasks);
      p->task_kv_len.assign(desc->task_kv_len, desc->task_kv_len + desc->n_tasks);
    }
    schedule(p);
  } catch (const Fail &f) {
    delete p;
    set_error(f.msg);
    return f.code;
  } catch (const std::bad_alloc &) {
    delete p;
    set_error("out of host memory while planning");
    return CA_ERR_INVALID_ARG;
  }
  *out = p;
  return CA_OK;
}

}  // namespace ca

extern "C" {

int ca_plan_host(const ca_batch_desc *desc, ca_plan_t **out) { return ca::build_plan(desc, out); }

const char *ca_last_error(void) { return ca::last_error(); }

const char *ca_error_string(int code) {
  switch (code) {
    case CA_OK: return "ok";
    case CA_ERR_INVALID_ARG: return "invalid argument";
    case CA_ERR_UNSUPPORTED: return "unsupported configuration";
    case CA_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
    case CA_ERR_HIP: return "HIP runtime error";
    case CA_ERR_STATE: return "plan not uploaded to this device";
    default: return "unknown error code";
  }
}

int ca_plan_workspace_bytes(const ca_plan_t *p, size_t *fwd, size_t *bwd) {
  if (!p) {
    ca::set_error("plan is null");
    return CA_ERR_INVALID_ARG;
  }
  if (fwd) *fwd = p->ws_fwd;
  if (bwd) *bwd = p->ws_bwd;
  return CA_OK;
}

int ca_plan_info(const ca_plan_t *p, int64_t *out, int n) {
  if (!p) return 0;
  int64_t full_tiles = 0;
  for (auto &u : p->fwd_units) full_tiles += u.hp == 1 && u.head == 0;
  const int64_t v[13] = {ca::FWD_BM, full_tiles, int64_t(p->fwd_units.size()),
                         ca::BWD_BN, int64_t(p->bwd_units.size()), ca::FWD_BN, int64_t(p->slot_row.size()),
                         p->fwd_steps, p->bwd_steps, ca::BWD_BQ, p->slot_align, p->heads_packed, p->bwd_workgroups};
  for (int i = 0; i < n && i < 13 && out; ++i) out[i] = v[i];
  return 13;
}

int64_t ca_plan_rows(const ca_plan_t *p, int32_t *rows, int32_t *pos) {
  if (!p) return 0;
  if (rows) std::memcpy(rows, p->slot_row.data(), p->slot_row.size() * sizeof(int32_t));
  if (pos) std::memcpy(pos, p->slot_pos.data(), p->slot_pos.size() * sizeof(int32_t));
  return int64_t(p->slot_row.size());
}

int64_t ca_plan_fwd_units(const ca_plan_t *p, int32_t *units) {
  if (!p) return 0;
  if (units) std::memcpy(units, p->fwd_units.data(), p->fwd_units.size() * sizeof(ca::FwdUnit));
  return int64_t(p->fwd_units.size());
}

int64_t ca_plan_bwd_units(const ca_plan_t *p, int32_t *units) {
  if (!p) return 0;
  if (units) std::memcpy(units, p->bwd_units.data(), p->bwd_units.size() * sizeof(ca::BwdUnit));
  return int64_t(p->bwd_units.size());
}

}  // extern "C"
