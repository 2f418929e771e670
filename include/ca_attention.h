/*
 * ca_attention.h - C ABI of the attention-server compute step of core attention disaggregation
 * on one MI355X (gfx950).
 *
 * The operation: causal core attention, P = softmax(scale * Q K^T) with masking, O = P V
 * (Section 2.1, "Context-dependent layers"), forward and backward, over ONE fused launch of many
 * CA-tasks.  A CA-task is a query shard q(t) of one document attending to that document's KV
 * prefix kv(t) = context(q(t)) (Section 4.1, definition of the CA-task); an attention server
 * receives {q(t), kv(t)} for its tasks, runs them all in a single kernel and returns each task's
 * output (Section 4.1, runtime).  Forward keeps only O and one log-sum-exp per (row, head); backward
 * recomputes P from it (Section 2.1: P is never materialised).
 *
 * All tensor pointers are DEVICE pointers owned by the caller; all descriptor arrays are HOST
 * pointers.  No entry point throws; every one returns CA_OK (0) or a negative ca_status, and ca_last_error()
 * then holds a human-readable detail for the calling thread.  The launch calls (ca_forward, ca_backward,
 * ca_merge_partials, ca_sum_partial_dq, ca_mfma_stream) never synchronise the device; ca_plan waits for its own
 * upload and ca_profile_read for the events it reads.  A plan is read-only for the launch calls and may serve several
 * host threads and streams at once, each launch with a workspace of its own (while profiling is enabled on it, one
 * thread and one stream at a time: the timing events belong to the plan).
 *
 * Layouts (row-major, token-major, bf16 unless stated):
 *   Q, O, dO, dQ : [total_q ][n_q_heads ][head_dim]
 *   K, V, dK, dV : [total_kv][n_kv_heads][head_dim]
 *   LSE          : [n_q_heads][total_q] fp32, natural log of the row's sum of exp(scale * score)
 * Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *
 * Semantics: row i of task t sits at document position p = q_pos[t] + i and attends keys
 * j in [0, min(kv_len[t], p + 1)) of its document, i.e. packed KV rows doc_kv_start + j: causal inside
 * the document, diagonal included, nothing across documents (Appendix B's shard geometry,
 * n_q + L_kv - L_q <= n_kv <= L_kv).  Tasks of one document share that document's single KV range;
 * dK/dV are gradients with respect to the packed KV buffer (summed over all tasks and all query heads
 * of a group); KV rows no query attends receive 0.
 *
 * Query shard with a SUB-RANGE of its context (the extension named in the paper's Limitations section): declare
 * the key window [lo, hi) of the context as a "document" (doc_kv_start = row of key lo, doc_kv_len = hi - lo) and
 * the shard as a task on it with q_pos counted from lo and kv_len <= hi - lo.  kv_len may be smaller than
 * q_pos + q_len: rows beyond it see the whole window.  Each (shard, window) task has query rows of its own (copies
 * of the shard's Q and dO).  ca_forward then yields partial O and LSE; ca_merge_partials combines the partial
 * results of a row; ca_backward on the partial tasks, given the MERGED O and LSE in their rows, yields the whole
 * dK, dV of each window and partial dQ that ca_sum_partial_dq adds up.
 */
#ifndef CA_ATTENTION_H
#define CA_ATTENTION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CA_OK = 0,
  CA_ERR_INVALID_ARG = -1, /* null pointer, bad count, range out of bounds, overlapping ranges, kv_len < 1 ... */
  CA_ERR_UNSUPPORTED = -2, /* head_dim not in {64,128}, n_q_heads not a multiple of n_kv_heads, sizes beyond int32 tiles */
  CA_ERR_WORKSPACE = -3,   /* workspace null, too small or not 256-byte aligned */
  CA_ERR_HIP = -4,         /* a HIP runtime call failed; detail string has its name and message */
  CA_ERR_STATE = -5        /* plan not uploaded to a device, or used on a different device */
} ca_status;

typedef struct ca_plan ca_plan_t; /* opaque */

/* One fused batch of CA-tasks (Section 4.1).  All arrays are host memory and are copied by ca_plan. */
typedef struct {
  int32_t n_docs, n_tasks;
  int32_t n_q_heads, n_kv_heads, head_dim; /* n_q_heads % n_kv_heads == 0; head_dim 64 or 128 */
  int64_t total_q, total_kv;               /* rows of packed Q/O/dO/dQ and of packed K/V/dK/dV */
  float softmax_scale;                     /* <= 0 selects 1/sqrt(head_dim) */
  const int64_t *doc_kv_start;             /* [n_docs] packed KV row of the document's token 0 */
  const int64_t *doc_kv_len;               /* [n_docs] resident KV rows of the document (>= 1) */
  const int32_t *task_doc;                 /* [n_tasks] */
  const int64_t *task_q_start;             /* [n_tasks] first row in packed Q */
  const int64_t *task_q_len;               /* [n_tasks] n_q >= 1, any integer */
  const int64_t *task_q_pos;               /* [n_tasks] document position of the first query row */
  const int64_t *task_kv_len;              /* [n_tasks] keys attended: 1 <= kv_len <= doc_kv_len; q_pos + q_len for
                                              the plain causal prefix, less to clip the shard to a key window */
} ca_batch_desc;

/*
 * ca_plan_host: validate the descriptor and build the launch schedule on the host only (no HIP call):
 * per-document sorted query-row lists cut into tiles (rows of different tasks of one document may
 * share a tile; rows of different documents never do), forward work units (tile x head) and backward
 * work units (KV tile x KV head) ordered longest-first.  Usable on a machine without a GPU and from a
 * scheduler thread that prepares the next batch while the GPU runs the current one (Section 4.1: the
 * scheduler works one batch ahead).  The plan owns copies of everything; free with ca_plan_destroy.
 */
int ca_plan_host(const ca_batch_desc *desc, ca_plan_t **out);

/* ca_plan_upload: allocate the plan's small device arrays on the current device and copy the schedule
 * (asynchronously on `hip_stream`, a hipStream_t or NULL for the default stream).  Launches that use the plan must
 * be ordered after that copy: issue them on the same stream, or synchronise it first. */
int ca_plan_upload(ca_plan_t *plan, void *hip_stream);

/* ca_plan = ca_plan_host + ca_plan_upload on the default stream + a wait for the copy: the plan it returns may be
 * used on any stream. */
int ca_plan(const ca_batch_desc *desc, ca_plan_t **out);

/* Bytes of caller-provided device workspace ca_forward / ca_backward need (either pointer may be NULL). */
int ca_plan_workspace_bytes(const ca_plan_t *plan, size_t *fwd_bytes, size_t *bwd_bytes);

/*
 * ca_forward: O and LSE for every query row of every task, one fused launch on `hip_stream`.
 * q,k,v: device bf16 inputs; o: device bf16 output; lse: device fp32 output [n_q_heads][total_q].
 * ws: device workspace of at least fwd_bytes (may be NULL when fwd_bytes is 0), 256-byte aligned.
 * Allocates nothing, never synchronises.
 */
int ca_forward(const ca_plan_t *plan, const void *q, const void *k, const void *v, void *o, float *lse,
               void *ws, size_t ws_bytes, void *hip_stream);

/*
 * ca_backward: dQ, dK, dV of L = sum(dO * O) given the forward's inputs and its saved O and LSE
 * (nothing else is kept between the two calls).  dq like q; dk, dv like k, v (every row written).
 * ws: device workspace of at least bwd_bytes, 256-byte aligned.  It receives, for every (query head, padded row
 * slot), fp32 -<dO, O> and log2(e)*LSE (twice: by head and slot, and in the row order of the dK/dV kernel's tiles), and
 * position-sorted bf16 copies of Q and dO
 * (bwd_bytes is about 4 * n_q_heads * padded_rows * (4 + head_dim) bytes: a little over the size of Q plus dO),
 * and one 4-byte progress counter per workgroup of the dK/dV kernel, through which workgroups that read the same Q/dO
 * tiles pace each other (timing only).  No arithmetic uses atomics: results are bit-reproducible from run to run.  Allocates
 * nothing, never synchronises.  Two calls whose workspaces overlap must not overlap in time on the device.
 */
int ca_backward(const ca_plan_t *plan, const void *q, const void *k, const void *v, const void *o,
                const void *d_o, const float *lse, void *dq, void *dk, void *dv,
                void *ws, size_t ws_bytes, void *hip_stream);

/*
 * ca_backward_static_ws: ca_backward for callers that can neither allocate device memory nor hold a workspace of
 * their own: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and kernels as ca_backward, minus `ws`: the workspace is a device-resident array of
 * CA_STATIC_WS_BYTES inside the library (every GPU the library runs on holds its own copy until the process
 * ends; its address on the current device is looked up on the first call there, with no allocation).
 * A batch whose ca_plan_workspace_bytes() backward figure exceeds CA_STATIC_WS_BYTES is refused with
 * CA_ERR_WORKSPACE before anything is launched (with 32 query heads of 128 that is about 4000 padded query rows).
 * All calls on one GPU share the one array, which keeps the previous call's contents (every launch rewrites
 * what it reads): calls that overlap in time on one GPU - different streams, or threads - race, so issue them on one
 * stream.  Calls no hipMalloc / hipFree, never synchronises.
 */
#define CA_STATIC_WS_BYTES (64u << 20)
int ca_backward_static_ws(const ca_plan_t *plan, const void *q, const void *k, const void *v, const void *o,
                          const void *d_o, const float *lse, void *dq, void *dk, void *dv, void *hip_stream);
size_t ca_static_workspace_bytes(void); /* CA_STATIC_WS_BYTES as the loaded library was built */

void ca_plan_destroy(ca_plan_t *plan);

/*
 * ca_merge_partials: combine partial attention results of query rows over disjoint key sets (Limitations section:
 * a query shard may attend a sub-range of its context; the results over the sub-ranges then have to be merged).
 * With L_i the log-sum-exp and O_i the output of part i:  L = log sum_i exp(L_i),  O = sum_i exp(L_i - L) O_i.
 * part_rows: DEVICE int32 [n_parts][n_rows]; part_rows[i][r] = row of part i of merged row r in the partial buffers,
 *   or -1 (or any value outside [0, total_q_part)) if the row has no such part.  A partial row may belong to one merged
 *   row only.
 * o_part: device bf16 [total_q_part][n_q_heads][head_dim]; lse_part: device fp32 [n_q_heads][total_q_part].
 * o: device bf16 [n_rows][n_q_heads][head_dim]; lse: device fp32 [n_q_heads][n_rows] (merged results; a row without
 *   parts gets O = 0, LSE = -inf).
 * o_back, lse_back: NULL, or buffers shaped like o_part / lse_part that receive the merged O and LSE in every partial
 *   row (what ca_backward needs for the partial tasks); they may be o_part and lse_part themselves (in place).
 * 1 <= n_parts <= 64.  One launch on `hip_stream`; allocates nothing, never synchronises.
 */
int ca_merge_partials(const int32_t *part_rows, int64_t n_rows, int32_t n_parts, const void *o_part,
                      const float *lse_part, int64_t total_q_part, void *o, float *lse, void *o_back,
                      float *lse_back, int32_t n_q_heads, int32_t head_dim, void *hip_stream);

/*
 * ca_sum_partial_dq: dq[r] = sum over the parts i of row r of dq_part[part_rows[i][r]] (fp32 sum of the bf16
 * partial gradients, rounded once): the query gradient of a row whose context was cut into key windows.
 * Arguments as in ca_merge_partials; dq: device bf16 [n_rows][n_q_heads][head_dim]; rows without parts get 0.
 */
int ca_sum_partial_dq(const int32_t *part_rows, int64_t n_rows, int32_t n_parts, const void *dq_part,
                      int64_t total_q_part, void *dq, int32_t n_q_heads, int32_t head_dim, void *hip_stream);

/*
 * Per-kernel timing for profilers and cost models (Section 4.2's profiler benchmarks core attention over
 * a grid of shapes; this is the hook it reads).  After ca_profile_enable(plan, 1) every ca_forward /
 * ca_backward on that plan records HIP events on the caller's stream around its kernels.
 * ca_profile_read blocks until the last recorded events have completed and writes milliseconds to
 * out[0..4): {forward kernel, backward preparation (Delta and log-sum-exp in slot order, zero fills
 * when some rows belong to no task), backward dK/dV kernel, backward dQ kernel}; entries of calls not made since enabling are 0.  Enabling creates events
 * (the only allocation); disabling destroys them.
 */
int ca_profile_enable(ca_plan_t *plan, int on);
int ca_profile_read(ca_plan_t *plan, float *out_ms);

/*
 * ca_mfma_stream: calibration aid for the matrix-pipe roofline, not a step of the method.  Launches n_workgroups
 * workgroups of four waves; every wave issues n_mfma_per_wave v_mfma_f32_32x32x16_bf16 (the instruction the three
 * attention kernels are built on) back to back from registers, with no memory access in the loop.  Timed by the
 * caller over enough workgroups to fill the chip (HIP events on hip_stream around the call), it gives the rate the
 * matrix pipes sustain on this device for this kind of operand data and this many waves per SIMD:
 * n_workgroups * 4 * n_mfma_per_wave * 32768 flops per launch.
 *   operands : device, bf16 [16][256][8] (64 KiB), read only: thread t of every workgroup takes fragment 2i as its
 *              i-th A operand and fragment 2i+1 as its i-th B operand (i = 0..7), 8 values each; MFMA number
 *              64 n + 8 r + j of a wave multiplies A[j] by B[(j + r) mod 8] into accumulation chain j mod 4.
 *   n_mfma_per_wave : a non-negative multiple of 64.
 *   side_work : 0 = MFMAs only.  1 or 2 = every MFMA is followed by the other work an attention kernel issues per
 *              MFMA, results unused: one 16-byte LDS read per lane and 2 (4) fp32 multiply-adds, plus one
 *              exponential per two MFMAs (per MFMA): about the dK/dV (forward) kernel's ratio.  Uses 16 KiB of LDS.
 *   sums     : device, fp32 [n_workgroups][256], written: per thread the sum of its 64 accumulator values (with
 *              all-ones operands exactly 256 * n_mfma_per_wave as long as that is below 2^24), so a caller can
 *              check that the instructions ran.
 * Asynchronous on hip_stream, allocates nothing.  CA_ERR_INVALID_ARG for a bad count or a null pointer.
 */
int ca_mfma_stream(const void *operands, int64_t n_mfma_per_wave, int32_t n_workgroups, int32_t side_work, float *sums,
                   void *hip_stream);

/*
 * ca_xcd_map: which XCD (each of the 8 has an L2 of its own) every workgroup of a launch of n_workgroups workgroups of
 * threads_per_workgroup threads runs on: out[i] = hardware XCC id of workgroup i (device int32 [n_workgroups]).
 * The work order of ca_plan (Section 3.2: throughput should depend on the aggregate tokens of a fused call) puts the
 * units of one KV head on one XCD by assuming that workgroups are dealt to the XCDs round robin in index order
 * (workgroup i to XCD (i + c) mod 8, c depending on where the previous launch stopped); tests read the mapping through this
 * call.  Asynchronous on hip_stream, allocates nothing.
 */
int ca_xcd_map(int32_t n_workgroups, int32_t threads_per_workgroup, int32_t *out, void *hip_stream);

/*
 * ca_atomic_stream: calibration aid, not a step of the method: the cost of summing partial dQ tiles with fp32 atomic
 * adds, which a backward kernel that owns KV tiles and computes S and dP only once (Section 2.1: P is recomputed in
 * backward, once) would have to do.  n_workgroups workgroups of four waves run `steps` steps; per step every wave
 * issues mfma_per_step v_mfma_f32_32x32x16_bf16 (a multiple of 4; fragments 0 and 1 of `operands`, laid out as for
 * ca_mfma_stream) and atomics_per_step (0 .. 32) global_atomic_add_f32 of +1.0 per lane, 256 contiguous bytes per
 * instruction, into its quarter of a 32 KiB tile; workgroup i uses region i mod 8 and tile (step + (i / 8) mod 8) mod
 * n_tiles of it.
 *   tiles : device fp32 [8][n_tiles][8192], read and written (after the launch its sum has grown by
 *           n_workgroups * steps * atomics_per_step * 256);   sums : device fp32 [n_workgroups][256], written.
 * Asynchronous on hip_stream, allocates nothing.  CA_ERR_INVALID_ARG for counts out of range or null pointers.
 */
int ca_atomic_stream(const void *operands, float *tiles, int32_t n_tiles, int32_t n_workgroups, int32_t steps,
                     int32_t mfma_per_step, int32_t atomics_per_step, float *sums, void *hip_stream);

const char *ca_error_string(int code);
const char *ca_last_error(void); /* thread-local detail of the last failing call on this thread */

/*
 * Schedule introspection (host side; for tests, profilers and cost models).
 * ca_plan_info fills `out[0..n)` with, in order: q_tile_rows, n_q_tiles, n_fwd_units, kv_tile_rows,
 * n_bwd_units, fwd_kv_step, padded_rows, sum over forward units of KV steps, sum over backward units of
 * (q blocks x heads) steps, bwd_q_block_rows, slot_align (a document's rows are padded to this many slots),
 * heads_packed (query heads per head-packed forward unit), n_bwd_workgroups (workgroups of the dK/dV kernel: short
 * backward units are chained, see below).  n_q_tiles counts the full 256-slot tiles.
 * Returns the number of values available.
 */
int ca_plan_info(const ca_plan_t *plan, int64_t *out, int n);
/* Copies of the schedule arrays.  Each returns the element count; pass NULL to query it.
 *  rows : [padded_rows] packed Q row of each tile slot, -1 for padding
 *  pos  : [padded_rows] document position of each tile slot
 *  fwd  : [n_fwd_units][5] = {first slot, packed KV row of doc token 0, keys needed (max pos + 1), first head,
 *                             heads per unit hp}: a unit is one workgroup of the forward and dQ kernels and
 *                             covers 256 / hp slots of hp consecutive query heads of one KV group; hp = 1 for the
 *                             full 256-slot tiles of a document, heads_packed for the slots left over
 *  bwd  : [n_bwd_units][10] = {first slot of first q block, slots end, first slot from which every slot sees the
 *                             whole tile, packed KV row of the tile's first key, valid keys in tile, document
 *                             position of the tile's first key, KV head, follow, count, tiles per q block}.  The first
 *                             n_bwd_workgroups units are one workgroup of the dK/dV kernel each (longest first; unit
 *                             index modulo n_kv_heads = KV head); such a unit has count >= 1, and its workgroup goes
 *                             on with the count - 1 units stored from index `follow` on (same KV head, count 0).
 *                             Tiles per q block = the query heads per KV head, or a half or a quarter of that for a
 *                             document of at most 32 / 16 rows, whose 64-row tiles hold the rows of 2 / 4 heads
 */
int64_t ca_plan_rows(const ca_plan_t *plan, int32_t *rows, int32_t *pos);
int64_t ca_plan_fwd_units(const ca_plan_t *plan, int32_t *units);
int64_t ca_plan_bwd_units(const ca_plan_t *plan, int32_t *units);

#ifdef __cplusplus
}
#endif
#endif /* CA_ATTENTION_H */
