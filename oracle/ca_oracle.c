/*
 * CPU oracle for core attention over a fused batch of CA-tasks.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the HIP library; nothing on the product path may call it.
 *
 * What it computes is the plain definition, in fp64, one query row at a time:
 *   - core attention: P = softmax(Q K^T) with a causal mask, O = P V
 *     (Section 2.1, "Context-dependent layers");
 *   - a CA-task t is a query shard q(t) of one document attending to that document's
 *     KV prefix kv(t) = context(q(t)); the results of a document's shards together are the
 *     document's result (Section 4.1, definition of the CA-task);
 *   - the row at document position p sees keys 0..p of its own document, diagonal included;
 *     this is the reading under which a shard's work is proportional to n_q(2 n_kv - n_q)
 *     with n_q + L_kv - L_q <= n_kv <= L_kv (Appendix B);
 *   - a task may name fewer keys than that (kv_len < p + 1): the row then sees keys 0..kv_len-1 only.  With a
 *     "document" that is a window of a longer context this is a query shard attending a sub-range of its
 *     context (the extension named in the Limitations section); ca_oracle_merge combines such partial results;
 *   - the backward is the calculus of that definition for the scalar sum(dO * O), with P
 *     recomputed from the per-row log-sum-exp rather than stored (Section 2.1: P is not
 *     materialised, it is recomputed during backward).
 *
 * No tiling, no online rescaling, no reordering: a two-pass softmax (max, then sum) per row.
 * Query head h reads KV head h / (Hq/Hkv).  All pins of this file live in tests/ (closed
 * forms, a hand-worked example, finite differences, a library attention routine on the
 * whole-document special case, brute force on tiny inputs, invariants).
 *
 * Layouts: Q, O, dO, dQ [total_q][Hq][D]; K, V, dK, dV [total_kv][Hkv][D]; LSE, Delta [Hq][total_q];
 * all double, row-major.  LSE is the natural log of the row's sum of exp(scale * score).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t n_docs, n_tasks, n_q_heads, n_kv_heads, head_dim;
  int64_t total_q, total_kv;
  double scale;
  const int64_t *doc_kv_start;
  const int32_t *task_doc;
  const int64_t *task_q_start, *task_q_len, *task_q_pos, *task_kv_len;
} ca_oracle_batch;

static double dot(const double *a, const double *b, int n) {
  double s = 0.0;
  for (int i = 0; i < n; ++i) s += a[i] * b[i];
  return s;
}

static int64_t visible(const ca_oracle_batch *b, int t, int64_t i) {
  /* number of keys row i of task t sees: min(kv_len, p + 1) */
  int64_t p = b->task_q_pos[t] + i;
  int64_t n = p + 1;
  return n < b->task_kv_len[t] ? n : b->task_kv_len[t];
}

int ca_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Forward: O and LSE for every query row of every task. */
int ca_oracle_forward(const ca_oracle_batch *b, const double *Q, const double *K, const double *V,
                      double *O, double *LSE) {
  const int Hq = b->n_q_heads, Hkv = b->n_kv_heads, D = b->head_dim, G = Hq / Hkv;
  for (int t = 0; t < b->n_tasks; ++t) {
    const int64_t kv0 = b->doc_kv_start[b->task_doc[t]];
    const int64_t nq = b->task_q_len[t];
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int64_t i = 0; i < nq; ++i) {
      for (int h = 0; h < Hq; ++h) {
        const int64_t row = b->task_q_start[t] + i;
        const int64_t n = visible(b, t, i);
        const double *q = Q + (row * Hq + h) * D;
        double *s = (double *)malloc(sizeof(double) * (size_t)n);
        double m = -INFINITY;
        for (int64_t j = 0; j < n; ++j) {
          s[j] = b->scale * dot(q, K + ((kv0 + j) * Hkv + h / G) * D, D);
          if (s[j] > m) m = s[j];
        }
        double l = 0.0;
        for (int64_t j = 0; j < n; ++j) {
          s[j] = exp(s[j] - m);
          l += s[j];
        }
        double *o = O + (row * Hq + h) * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int64_t j = 0; j < n; ++j) {
          const double p = s[j] / l;
          const double *v = V + ((kv0 + j) * Hkv + h / G) * D;
          for (int d = 0; d < D; ++d) o[d] += p * v[d];
        }
        LSE[(int64_t)h * b->total_q + row] = m + log(l);
        free(s);
      }
    }
  }
  return 0;
}

/*
 * Backward of L = sum(dO * O).  Per row: Delta = <dO,O>, dP_j = <dO,V_j>, dS_j = P_j (dP_j - Delta),
 * dQ = scale * sum_j dS_j K_j.  Per key j: dK_j = scale * sum_rows dS_j Q_row, dV_j = sum_rows P_j dO_row,
 * the sums running over every row, every query head of the KV head's group and every task of the
 * document that sees key j.  P_j = exp(scale*score_j - LSE).
 * dK and dV cover the whole packed KV buffer; rows nobody attends come out zero.
 * Any of dQ, dK, dV may be NULL to skip it.
 */
int ca_oracle_backward(const ca_oracle_batch *b, const double *Q, const double *K, const double *V,
                       const double *O, const double *dO, const double *LSE,
                       double *dQ, double *dK, double *dV, double *Delta_out) {
  const int Hq = b->n_q_heads, Hkv = b->n_kv_heads, D = b->head_dim, G = Hq / Hkv;
  double *Delta = (double *)malloc(sizeof(double) * (size_t)(Hq * b->total_q));
  if (!Delta) return -1;
  memset(Delta, 0, sizeof(double) * (size_t)(Hq * b->total_q));
  /* row-owned part: Delta and dQ */
  for (int t = 0; t < b->n_tasks; ++t) {
    const int64_t kv0 = b->doc_kv_start[b->task_doc[t]];
    const int64_t nq = b->task_q_len[t];
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
    for (int64_t i = 0; i < nq; ++i) {
      for (int h = 0; h < Hq; ++h) {
        const int64_t row = b->task_q_start[t] + i;
        const int64_t n = visible(b, t, i);
        const double *q = Q + (row * Hq + h) * D;
        const double *go = dO + (row * Hq + h) * D;
        const double delta = dot(go, O + (row * Hq + h) * D, D);
        const double lse = LSE[(int64_t)h * b->total_q + row];
        Delta[(int64_t)h * b->total_q + row] = delta;
        if (!dQ) continue;
        double *gq = dQ + (row * Hq + h) * D;
        for (int d = 0; d < D; ++d) gq[d] = 0.0;
        for (int64_t j = 0; j < n; ++j) {
          const double *k = K + ((kv0 + j) * Hkv + h / G) * D;
          const double *v = V + ((kv0 + j) * Hkv + h / G) * D;
          const double p = exp(b->scale * dot(q, k, D) - lse);
          const double ds = p * (dot(go, v, D) - delta);
          for (int d = 0; d < D; ++d) gq[d] += b->scale * ds * k[d];
        }
      }
    }
  }
  /* key-owned part: dK and dV */
  if (dK) memset(dK, 0, sizeof(double) * (size_t)(b->total_kv * Hkv * D));
  if (dV) memset(dV, 0, sizeof(double) * (size_t)(b->total_kv * Hkv * D));
  if (dK || dV) {
    for (int t = 0; t < b->n_tasks; ++t) {
      const int64_t kv0 = b->doc_kv_start[b->task_doc[t]];
      const int64_t nq = b->task_q_len[t];
      const int64_t nkeys = visible(b, t, nq - 1); /* keys the task's last row sees */
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
      for (int64_t j = 0; j < nkeys; ++j) {
        for (int hk = 0; hk < Hkv; ++hk) {
          const double *k = K + ((kv0 + j) * Hkv + hk) * D;
          const double *v = V + ((kv0 + j) * Hkv + hk) * D;
          double *gk = dK ? dK + ((kv0 + j) * Hkv + hk) * D : NULL;
          double *gv = dV ? dV + ((kv0 + j) * Hkv + hk) * D : NULL;
          for (int64_t i = 0; i < nq; ++i) {
            if (j >= visible(b, t, i)) continue; /* masked */
            const int64_t row = b->task_q_start[t] + i;
            for (int h = hk * G; h < (hk + 1) * G; ++h) {
              const double *q = Q + (row * Hq + h) * D;
              const double *go = dO + (row * Hq + h) * D;
              const double p = exp(b->scale * dot(q, k, D) - LSE[(int64_t)h * b->total_q + row]);
              const double ds = p * (dot(go, v, D) - Delta[(int64_t)h * b->total_q + row]);
              if (gk) for (int d = 0; d < D; ++d) gk[d] += b->scale * ds * q[d];
              if (gv) for (int d = 0; d < D; ++d) gv[d] += p * go[d];
            }
          }
        }
      }
    }
  }
  if (Delta_out) memcpy(Delta_out, Delta, sizeof(double) * (size_t)(Hq * b->total_q));
  free(Delta);
  return 0;
}

/*
 * Merge of partial results (the Limitations section names a query shard that attends only a sub-range of its
 * context as the extension of the CA-task; the partial outputs of one row over disjoint key sets K_1..K_n then have
 * to be combined).
 * From the definition: with L_i = log sum_{j in K_i} exp(s_j) and O_i = sum_{j in K_i} exp(s_j - L_i) V_j,
 *   L = log sum_i exp(L_i),   O = sum_i exp(L_i - L) O_i
 * is the softmax-weighted sum over the union of the key sets.
 * part_rows[i * n_rows + r] is the row of part i of merged row r in the partial buffers, or -1 if the row has no such
 * part.  O_part [total_q_part][Hq][D], LSE_part [Hq][total_q_part]; O [n_rows][Hq][D], LSE [Hq][n_rows].
 * A row without any part gets O = 0 and LSE = -infinity.
 */
int ca_oracle_merge(int64_t n_rows, int32_t n_parts, const int64_t *part_rows, const double *O_part,
                    const double *LSE_part, int64_t total_q_part, int32_t Hq, int32_t D, double *O, double *LSE) {
  for (int64_t r = 0; r < n_rows; ++r) {
    for (int h = 0; h < Hq; ++h) {
      double m = -INFINITY;
      for (int i = 0; i < n_parts; ++i) {
        const int64_t pr = part_rows[(int64_t)i * n_rows + r];
        if (pr >= 0 && LSE_part[(int64_t)h * total_q_part + pr] > m) m = LSE_part[(int64_t)h * total_q_part + pr];
      }
      double *o = O + (r * Hq + h) * D;
      for (int d = 0; d < D; ++d) o[d] = 0.0;
      if (m == -INFINITY) {
        LSE[(int64_t)h * n_rows + r] = -INFINITY;
        continue;
      }
      double sum = 0.0;
      for (int i = 0; i < n_parts; ++i) {
        const int64_t pr = part_rows[(int64_t)i * n_rows + r];
        if (pr >= 0) sum += exp(LSE_part[(int64_t)h * total_q_part + pr] - m);
      }
      const double l = m + log(sum);
      for (int i = 0; i < n_parts; ++i) {
        const int64_t pr = part_rows[(int64_t)i * n_rows + r];
        if (pr < 0) continue;
        const double w = exp(LSE_part[(int64_t)h * total_q_part + pr] - l);
        const double *op = O_part + (pr * Hq + h) * D;
        for (int d = 0; d < D; ++d) o[d] += w * op[d];
      }
      LSE[(int64_t)h * n_rows + r] = l;
    }
  }
  return 0;
}
