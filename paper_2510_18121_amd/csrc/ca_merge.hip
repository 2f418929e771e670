// Merge of partial attention results over disjoint key windows, and the sum of the partial query gradients
// (the paper's Limitations section: a query shard attending a sub-range of its context).  Both are elementwise over
// (row, head, 8-column chunk) and bound by HBM: per merged (row, head) they read n_parts x (2 D + 4) bytes and
// write (2 D + 4) bytes, plus the same again per part when the merged values are written back.
#include <hip/hip_runtime.h>

#include <sstream>

#include "ca_device.h"
#include "ca_internal.h"

namespace ca {

constexpr int MERGE_THREADS = 256;
constexpr int MERGE_MAX_PARTS = 64;

__device__ __forceinline__ void unpack8(const u32x4 x, float *f) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __builtin_bit_cast(float, x[i] << 16);
    f[2 * i + 1] = __builtin_bit_cast(float, x[i] & 0xffff0000u);
  }
}

// One thread per (row, head, chunk of 8 columns); the D/8 threads of a (row, head) are neighbouring lanes of one
// wave, so every partial log-sum-exp of the row has been read by all of them before any of them writes merged
// values back over the partial buffers (the in-place case).
template <int D, bool SUM_ONLY>
__global__ __launch_bounds__(MERGE_THREADS) void ca_merge_kernel(const int32_t *__restrict__ part_rows, int64_t n_rows,
                                                                 int n_parts, const bf16_t *o_part,
                                                                 const float *lse_part, int64_t total_q_part,
                                                                 bf16_t *__restrict__ o, float *__restrict__ lse,
                                                                 bf16_t *o_back, float *lse_back, int Hq) {
  constexpr int CH = D / 8;
  const int64_t idx = int64_t(blockIdx.x) * MERGE_THREADS + threadIdx.x;
  const int c = int(idx % CH);
  const int h = int((idx / CH) % Hq);
  const int64_t r = idx / (int64_t(CH) * Hq);
  if (r >= n_rows) return;
  auto part = [&](int i) -> int64_t {
    const int64_t pr = part_rows[int64_t(i) * n_rows + r];
    return (pr >= 0 && pr < total_q_part) ? pr : -1;
  };
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  float l = -INFINITY;
  if (SUM_ONLY) {
    for (int i = 0; i < n_parts; ++i) {
      const int64_t pr = part(i);
      if (pr < 0) continue;
      float f[8];
      unpack8(*reinterpret_cast<const u32x4 *>(o_part + (pr * Hq + h) * D + 8 * c), f);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += f[j];
    }
  } else {
    // one pass with a running maximum: sum_i exp(L_i - m) O_i and sum_i exp(L_i - m), rescaled when m grows
    float m = -INFINITY, sum = 0.f;
    for (int i = 0; i < n_parts; ++i) {
      const int64_t pr = part(i);
      if (pr < 0) continue;
      const float li = lse_part[int64_t(h) * total_q_part + pr];
      if (!(li > -INFINITY)) continue;  // a part that saw no key carries no weight
      float f[8];
      unpack8(*reinterpret_cast<const u32x4 *>(o_part + (pr * Hq + h) * D + 8 * c), f);
      if (li > m) {
        const float s = __expf(m - li);  // 0 on the first part (m = -inf)
        sum *= s;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] *= s;
        m = li;
      }
      const float w = __expf(li - m);
      sum += w;
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += w * f[j];
    }
    if (sum > 0.f) {
      l = m + __logf(sum);
      const float inv = 1.f / sum;
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] *= inv;
    }
  }
  u32x4 out;
#pragma unroll
  for (int j = 0; j < 4; ++j) out[j] = pack_bf16(acc[2 * j], acc[2 * j + 1]);
  *reinterpret_cast<u32x4 *>(o + (r * Hq + h) * D + 8 * c) = out;
  if (!SUM_ONLY) {
    if (c == 0) lse[int64_t(h) * n_rows + r] = l;
    if (o_back || lse_back) {
      for (int i = 0; i < n_parts; ++i) {
        const int64_t pr = part(i);
        if (pr < 0) continue;
        if (o_back) *reinterpret_cast<u32x4 *>(o_back + (pr * Hq + h) * D + 8 * c) = out;
        if (lse_back && c == 0) lse_back[int64_t(h) * total_q_part + pr] = l;
      }
    }
  }
}

static int merge_args_ok(const int32_t *part_rows, int64_t n_rows, int32_t n_parts, const void *in, int64_t total_q_part,
                         void *out, int32_t hq, int32_t d) {
  std::ostringstream os;
  if (n_rows < 0 || total_q_part < 0 || n_parts < 1 || n_parts > MERGE_MAX_PARTS || hq < 1) {
    os << "n_rows " << n_rows << ", total_q_part " << total_q_part << ", n_parts " << n_parts << " (1.." << MERGE_MAX_PARTS
       << "), n_q_heads " << hq << ": bad count";
    set_error(os.str());
    return CA_ERR_INVALID_ARG;
  }
  if (d != 64 && d != 128) {
    os << "head_dim " << d << " not supported (64 or 128)";
    set_error(os.str());
    return CA_ERR_UNSUPPORTED;
  }
  const int64_t lim = int64_t(1) << 31;
  if (n_rows >= lim || total_q_part >= lim || n_rows * hq * (d / 8) / MERGE_THREADS >= lim - 1) {
    set_error("n_rows / total_q_part beyond 2^31 rows");
    return CA_ERR_UNSUPPORTED;
  }
  if (n_rows > 0 && (!part_rows || !out || (total_q_part > 0 && !in))) {
    set_error("part_rows, an input or an output pointer is null");
    return CA_ERR_INVALID_ARG;
  }
  return CA_OK;
}

template <bool SUM_ONLY>
static int launch_merge(const int32_t *part_rows, int64_t n_rows, int n_parts, const void *o_part, const float *lse_part,
                        int64_t total_q_part, void *o, float *lse, void *o_back, float *lse_back, int hq, int d,
                        hipStream_t st) {
  if (n_rows == 0) return CA_OK;
  const int64_t threads = n_rows * hq * (d / 8);
  const dim3 grid(unsigned((threads + MERGE_THREADS - 1) / MERGE_THREADS));
  auto *op = static_cast<const bf16_t *>(o_part);
  auto *oo = static_cast<bf16_t *>(o), *ob = static_cast<bf16_t *>(o_back);
  if (d == 128)
    ca_merge_kernel<128, SUM_ONLY><<<grid, MERGE_THREADS, 0, st>>>(part_rows, n_rows, n_parts, op, lse_part,
                                                                  total_q_part, oo, lse, ob, lse_back, hq);
  else
    ca_merge_kernel<64, SUM_ONLY><<<grid, MERGE_THREADS, 0, st>>>(part_rows, n_rows, n_parts, op, lse_part,
                                                                 total_q_part, oo, lse, ob, lse_back, hq);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    std::ostringstream os;
    os << "merge launch: " << hipGetErrorName(e) << " (" << hipGetErrorString(e) << ")";
    set_error(os.str());
    return CA_ERR_HIP;
  }
  return CA_OK;
}

}  // namespace ca

extern "C" {

int ca_merge_partials(const int32_t *part_rows, int64_t n_rows, int32_t n_parts, const void *o_part,
                      const float *lse_part, int64_t total_q_part, void *o, float *lse, void *o_back, float *lse_back,
                      int32_t n_q_heads, int32_t head_dim, void *hip_stream) {
  using namespace ca;
  int rc = merge_args_ok(part_rows, n_rows, n_parts, o_part, total_q_part, o, n_q_heads, head_dim);
  if (rc != CA_OK) return rc;
  if (n_rows > 0 && (!lse || (total_q_part > 0 && !lse_part))) {
    set_error("lse or lse_part is null");
    return CA_ERR_INVALID_ARG;
  }
  return launch_merge<false>(part_rows, n_rows, n_parts, o_part, lse_part, total_q_part, o, lse, o_back, lse_back,
                             n_q_heads, head_dim, static_cast<hipStream_t>(hip_stream));
}

int ca_sum_partial_dq(const int32_t *part_rows, int64_t n_rows, int32_t n_parts, const void *dq_part,
                      int64_t total_q_part, void *dq, int32_t n_q_heads, int32_t head_dim, void *hip_stream) {
  using namespace ca;
  int rc = merge_args_ok(part_rows, n_rows, n_parts, dq_part, total_q_part, dq, n_q_heads, head_dim);
  if (rc != CA_OK) return rc;
  return launch_merge<true>(part_rows, n_rows, n_parts, dq_part, nullptr, total_q_part, dq, nullptr, nullptr, nullptr,
                            n_q_heads, head_dim, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
