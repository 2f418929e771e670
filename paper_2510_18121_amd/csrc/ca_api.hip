// C-ABI entry points that touch the device: plan upload, forward and backward launches.
#include <hip/hip_runtime.h>

#include <mutex>
#include <sstream>

#include "ca_internal.h"

namespace ca {
hipError_t launch_fwd(const ca_plan_t *p, const void *q, const void *k, const void *v, void *o, float *lse,
                      hipStream_t st);
hipError_t launch_bwd(const ca_plan_t *p, const void *q, const void *k, const void *v, const void *o, const void *d_o,
                      const float *lse, void *dq, void *dk, void *dv, void *ws, hipStream_t st, hipEvent_t *ev);

static int hip_fail(const char *what, hipError_t e) {
  std::ostringstream os;
  os << what << ": " << hipGetErrorName(e) << " (" << hipGetErrorString(e) << ")";
  set_error(os.str());
  return CA_ERR_HIP;
}
#define CA_HIP(call)                                  \
  do {                                                \
    hipError_t e_ = (call);                           \
    if (e_ != hipSuccess) return hip_fail(#call, e_); \
  } while (0)

// Device-resident backward workspace for callers that cannot allocate (ca_backward_static_ws).  In host code the
// array's name is only a handle for hipGetSymbolAddress: the address each device holds its copy at is looked up once
// per device and kept in static_ws_ptr; only that pointer is ever handed to kernels.
static __device__ __align__(256) __attribute__((used)) unsigned char static_ws[CA_STATIC_WS_BYTES];
static void *static_ws_ptr[16];
static std::mutex static_ws_mutex;

static int static_ws_on_device(int device, void **out) {
  if (device < 0 || device >= 16) {
    set_error("ca_backward_static_ws supports device ordinals 0..15");
    return CA_ERR_UNSUPPORTED;
  }
  std::lock_guard<std::mutex> lock(static_ws_mutex);
  if (!static_ws_ptr[device]) {  // the calling thread's current device is `device` (checked by the caller)
    void *ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_ws));
    if (e != hipSuccess) return hip_fail("hipGetSymbolAddress(static workspace)", e);
    if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 256 != 0) {
      set_error("static workspace has no usable device address");
      return CA_ERR_HIP;
    }
    static_ws_ptr[device] = ptr;
  }
  *out = static_ws_ptr[device];
  return CA_OK;
}

static void free_device(ca_plan_t *p) {
  if (p->device < 0) return;
  int cur = -1;
  if (hipGetDevice(&cur) == hipSuccess && cur != p->device) (void)hipSetDevice(p->device);
  if (p->d_slot_row) (void)hipFree(p->d_slot_row);
  if (p->d_slot_pos) (void)hipFree(p->d_slot_pos);
  if (p->d_block_rpk) (void)hipFree(p->d_block_rpk);
  if (p->d_pos_kv) (void)hipFree(p->d_pos_kv);
  p->d_block_rpk = p->d_pos_kv = nullptr;
  if (p->d_fwd_units) (void)hipFree(p->d_fwd_units);
  if (p->d_bwd_units) (void)hipFree(p->d_bwd_units);
  p->d_slot_row = p->d_slot_pos = nullptr;
  p->d_fwd_units = nullptr;
  p->d_bwd_units = nullptr;
  if (cur >= 0 && cur != p->device) (void)hipSetDevice(cur);
  p->device = -1;
}

static int check_call(const ca_plan_t *p, void *ws, size_t ws_bytes, size_t need) {
  if (!p) {
    set_error("plan is null");
    return CA_ERR_INVALID_ARG;
  }
  if (p->device < 0) {
    set_error("plan was not uploaded (ca_plan_upload)");
    return CA_ERR_STATE;
  }
  int cur = -1;
  hipError_t e = hipGetDevice(&cur);
  if (e != hipSuccess) return hip_fail("hipGetDevice", e);
  if (cur != p->device) {
    set_error("plan was uploaded to another device than the current one");
    return CA_ERR_STATE;
  }
  if (need > 0) {
    if (!ws || ws_bytes < need) {
      std::ostringstream os;
      os << "workspace of " << ws_bytes << " bytes given, " << need << " needed";
      set_error(os.str());
      return CA_ERR_WORKSPACE;
    }
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) {
      set_error("workspace is not 256-byte aligned");
      return CA_ERR_WORKSPACE;
    }
  }
  return CA_OK;
}
}  // namespace ca

extern "C" {

int ca_plan_upload(ca_plan_t *p, void *hip_stream) {
  using namespace ca;
  if (!p) {
    set_error("plan is null");
    return CA_ERR_INVALID_ARG;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  free_device(p);
  int dev = -1;
  CA_HIP(hipGetDevice(&dev));
  p->device = dev;
  auto up = [&](auto *&dst, const auto &src) -> hipError_t {
    if (src.empty()) return hipSuccess;
    const size_t bytes = src.size() * sizeof(src[0]);
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&dst), bytes);
    if (e != hipSuccess) return e;
    return hipMemcpyAsync(dst, src.data(), bytes, hipMemcpyHostToDevice, st);
  };
  hipError_t e;
  if ((e = up(p->d_slot_row, p->slot_row)) != hipSuccess || (e = up(p->d_slot_pos, p->slot_pos)) != hipSuccess ||
      (e = up(p->d_block_rpk, p->block_rpk)) != hipSuccess || (e = up(p->d_pos_kv, p->pos_kv)) != hipSuccess ||
      (e = up(p->d_fwd_units, p->fwd_units)) != hipSuccess || (e = up(p->d_bwd_units, p->bwd_units)) != hipSuccess) {
    free_device(p);
    return hip_fail("plan upload", e);
  }
  // the host vectors stay alive in the plan, so the asynchronous copies read valid memory
  return CA_OK;
}

int ca_plan(const ca_batch_desc *desc, ca_plan_t **out) {
  int rc = ca_plan_host(desc, out);
  if (rc != CA_OK) return rc;
  rc = ca_plan_upload(*out, nullptr);
  if (rc == CA_OK) {  // callers launch on streams of their own: the schedule must have landed before they do
    const hipError_t e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) rc = ca::hip_fail("plan upload", e);
  }
  if (rc != CA_OK) {
    ca_plan_destroy(*out);
    *out = nullptr;
  }
  return rc;
}

int ca_profile_enable(ca_plan_t *p, int on) {
  using namespace ca;
  if (!p) {
    set_error("plan is null");
    return CA_ERR_INVALID_ARG;
  }
  if (on && !p->profile) {
    for (int i = 0; i < 6; ++i) {
      hipEvent_t e;
      const hipError_t rc = hipEventCreate(&e);
      if (rc != hipSuccess) {  // leave nothing half-made behind
        for (int j = 0; j < i; ++j) (void)hipEventDestroy(static_cast<hipEvent_t>(p->ev[j])), p->ev[j] = nullptr;
        return hip_fail("hipEventCreate", rc);
      }
      p->ev[i] = e;
    }
    p->profile = true;
  } else if (!on && p->profile) {
    for (int i = 0; i < 6; ++i)
      if (p->ev[i]) (void)hipEventDestroy(static_cast<hipEvent_t>(p->ev[i])), p->ev[i] = nullptr;
    p->profile = false;
  }
  p->ev_fwd = p->ev_bwd = false;
  return CA_OK;
}

int ca_profile_read(ca_plan_t *p, float *out) {
  using namespace ca;
  if (!p || !out) {
    set_error("plan or output is null");
    return CA_ERR_INVALID_ARG;
  }
  for (int i = 0; i < 4; ++i) out[i] = 0.f;
  if (!p->profile) {
    set_error("profiling is not enabled on this plan");
    return CA_ERR_STATE;
  }
  auto E = [&](int i) { return static_cast<hipEvent_t>(p->ev[i]); };
  if (p->ev_fwd) {
    CA_HIP(hipEventSynchronize(E(1)));
    CA_HIP(hipEventElapsedTime(&out[0], E(0), E(1)));
  }
  if (p->ev_bwd) {
    CA_HIP(hipEventSynchronize(E(5)));
    CA_HIP(hipEventElapsedTime(&out[1], E(2), E(3)));
    CA_HIP(hipEventElapsedTime(&out[2], E(3), E(4)));
    CA_HIP(hipEventElapsedTime(&out[3], E(4), E(5)));
  }
  return CA_OK;
}

void ca_plan_destroy(ca_plan_t *p) {
  if (!p) return;
  if (p->profile) (void)ca_profile_enable(p, 0);
  ca::free_device(p);
  delete p;
}

int ca_forward(const ca_plan_t *p, const void *q, const void *k, const void *v, void *o, float *lse, void *ws,
               size_t ws_bytes, void *hip_stream) {
  using namespace ca;
  int rc = check_call(p, ws, ws_bytes, p ? p->ws_fwd : 0);
  if (rc != CA_OK) return rc;
  if (p->total_q > 0 && (!q || !o || !lse)) {
    set_error("q, o or lse is null");
    return CA_ERR_INVALID_ARG;
  }
  if (p->total_kv > 0 && (!k || !v)) {
    set_error("k or v is null");
    return CA_ERR_INVALID_ARG;
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  ca_plan_t *mp = const_cast<ca_plan_t *>(p);  // timing state only
  if (p->profile) (void)hipEventRecord(static_cast<hipEvent_t>(mp->ev[0]), st);
  hipError_t e = launch_fwd(p, q, k, v, o, lse, st);
  if (e != hipSuccess) return hip_fail("forward launch", e);
  if (p->profile) {
    (void)hipEventRecord(static_cast<hipEvent_t>(mp->ev[1]), st);
    mp->ev_fwd = true;
  }
  return CA_OK;
}

int ca_backward(const ca_plan_t *p, const void *q, const void *k, const void *v, const void *o, const void *d_o,
                const float *lse, void *dq, void *dk, void *dv, void *ws, size_t ws_bytes, void *hip_stream) {
  using namespace ca;
  int rc = check_call(p, ws, ws_bytes, p ? p->ws_bwd : 0);
  if (rc != CA_OK) return rc;
  if (p->total_q > 0 && (!q || !o || !d_o || !lse || !dq)) {
    set_error("q, o, d_o, lse or dq is null");
    return CA_ERR_INVALID_ARG;
  }
  if (p->total_kv > 0 && (!k || !v || !dk || !dv)) {
    set_error("k, v, dk or dv is null");
    return CA_ERR_INVALID_ARG;
  }
  ca_plan_t *mp = const_cast<ca_plan_t *>(p);  // timing state only
  hipError_t e = launch_bwd(p, q, k, v, o, d_o, lse, dq, dk, dv, ws, static_cast<hipStream_t>(hip_stream),
                            p->profile ? reinterpret_cast<hipEvent_t *>(&mp->ev[2]) : nullptr);
  if (e != hipSuccess) return hip_fail("backward launch", e);
  if (p->profile) mp->ev_bwd = true;
  return CA_OK;
}

int ca_backward_static_ws(const ca_plan_t *p, const void *q, const void *k, const void *v, const void *o,
                          const void *d_o, const float *lse, void *dq, void *dk, void *dv, void *hip_stream) {
  using namespace ca;
  int rc = check_call(p, nullptr, 0, 0);  // plan present, uploaded, and on the current device
  if (rc != CA_OK) return rc;
  if (p->ws_bwd > size_t(CA_STATIC_WS_BYTES)) {
    std::ostringstream os;
    os << "this batch needs a backward workspace of " << p->ws_bwd << " bytes; the static workspace holds "
       << size_t(CA_STATIC_WS_BYTES) << " (use ca_backward with a caller-provided workspace)";
    set_error(os.str());
    return CA_ERR_WORKSPACE;
  }
  void *ws = nullptr;
  rc = static_ws_on_device(p->device, &ws);
  if (rc != CA_OK) return rc;
  return ca_backward(p, q, k, v, o, d_o, lse, dq, dk, dv, ws, size_t(CA_STATIC_WS_BYTES), hip_stream);
}

size_t ca_static_workspace_bytes(void) { return size_t(CA_STATIC_WS_BYTES); }

}  // extern "C"
