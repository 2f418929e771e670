"""Thin Python binding over the C ABI of libca_attention.so (include/ca_attention.h).

Argument marshalling only: every step of the path runs inside the library's HIP kernels.  PyTorch
tensors are used as device memory and streams and nothing else.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libca_attention.so")
_lib = None

CA_OK = 0
CA_ERR_INVALID_ARG, CA_ERR_UNSUPPORTED, CA_ERR_WORKSPACE, CA_ERR_HIP, CA_ERR_STATE = -1, -2, -3, -4, -5


class CaError(RuntimeError):
    """A negative ca_status from the library, with its code and the library's detail string."""

    def __init__(self, code: int, detail: str):
        super().__init__(f"ca_attention error {code}: {detail}")
        self.code = code
        self.detail = detail


class BatchDesc(ctypes.Structure):
    """ca_batch_desc of include/ca_attention.h."""

    _fields_ = [
        ("n_docs", ctypes.c_int32), ("n_tasks", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("total_q", ctypes.c_int64), ("total_kv", ctypes.c_int64), ("softmax_scale", ctypes.c_float),
        ("doc_kv_start", ctypes.c_void_p), ("doc_kv_len", ctypes.c_void_p), ("task_doc", ctypes.c_void_p),
        ("task_q_start", ctypes.c_void_p), ("task_q_len", ctypes.c_void_p), ("task_q_pos", ctypes.c_void_p),
        ("task_kv_len", ctypes.c_void_p),
    ]


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built (python -m paper_2510_18121_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                                    "or python paper_2510_18121_amd/build.py")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.ca_plan_host.argtypes = [ctypes.POINTER(BatchDesc), ctypes.POINTER(vp)]
        L.ca_plan.argtypes = [ctypes.POINTER(BatchDesc), ctypes.POINTER(vp)]
        L.ca_plan_upload.argtypes = [vp, vp]
        L.ca_plan_workspace_bytes.argtypes = [vp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.ca_forward.argtypes = [vp] * 6 + [vp, sz, vp]
        L.ca_backward.argtypes = [vp] * 10 + [vp, sz, vp]
        L.ca_backward_static_ws.argtypes = [vp] * 10 + [vp]
        L.ca_static_workspace_bytes.restype = sz
        L.ca_plan_destroy.argtypes = [vp]
        L.ca_plan_destroy.restype = None
        L.ca_error_string.argtypes = [ctypes.c_int]
        L.ca_error_string.restype = ctypes.c_char_p
        L.ca_last_error.restype = ctypes.c_char_p
        L.ca_profile_enable.argtypes = [vp, ctypes.c_int]
        L.ca_profile_read.argtypes = [vp, vp]
        L.ca_plan_info.argtypes = [vp, vp, ctypes.c_int]
        for f in (L.ca_plan_rows, L.ca_plan_fwd_units, L.ca_plan_bwd_units):
            f.restype = ctypes.c_int64
        L.ca_plan_rows.argtypes = [vp, vp, vp]
        L.ca_plan_fwd_units.argtypes = [vp, vp]
        L.ca_plan_bwd_units.argtypes = [vp, vp]
        i32, i64 = ctypes.c_int32, ctypes.c_int64
        L.ca_merge_partials.argtypes = [vp, i64, i32, vp, vp, i64, vp, vp, vp, vp, i32, i32, vp]
        L.ca_sum_partial_dq.argtypes = [vp, i64, i32, vp, i64, vp, i32, i32, vp]
        L.ca_mfma_stream.argtypes = [vp, i64, i32, i32, vp, vp]
        L.ca_xcd_map.argtypes = [i32, i32, vp, vp]
        L.ca_atomic_stream.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp]
        _lib = L
    return _lib


def _check(rc: int):
    if rc != CA_OK:
        raise CaError(rc, (lib().ca_last_error() or b"").decode())


def make_desc(batch, keep: list) -> BatchDesc:
    """ca_batch_desc from any object with the descriptor's field names (e.g. workloads.Batch)."""
    def arr(x, dt):
        a = np.ascontiguousarray(np.asarray(x), dtype=dt)
        keep.append(a)
        return a.ctypes.data if a.size else None

    d = BatchDesc()
    d.n_docs, d.n_tasks = len(batch.doc_kv_len), len(batch.task_q_len)
    d.n_q_heads, d.n_kv_heads, d.head_dim = batch.n_q_heads, batch.n_kv_heads, batch.head_dim
    d.total_q, d.total_kv, d.softmax_scale = batch.total_q, batch.total_kv, float(batch.softmax_scale)
    d.doc_kv_start = arr(batch.doc_kv_start, np.int64)
    d.doc_kv_len = arr(batch.doc_kv_len, np.int64)
    d.task_doc = arr(batch.task_doc, np.int32)
    d.task_q_start = arr(batch.task_q_start, np.int64)
    d.task_q_len = arr(batch.task_q_len, np.int64)
    d.task_q_pos = arr(batch.task_q_pos, np.int64)
    d.task_kv_len = arr(batch.task_kv_len, np.int64)
    return d


class Plan:
    """Owner of a ca_plan_t*."""

    INFO_KEYS = ("q_tile_rows", "n_q_tiles", "n_fwd_units", "kv_tile_rows", "n_bwd_units", "fwd_kv_step",
                 "padded_rows", "fwd_steps", "bwd_steps", "bwd_q_block_rows", "slot_align", "heads_packed",
                 "n_bwd_workgroups")

    def __init__(self, handle, batch):
        self.handle = ctypes.c_void_p(handle)
        self.batch = batch

    def upload(self, stream=None):
        _check(lib().ca_plan_upload(self.handle, _stream_ptr(stream)))
        return self

    def workspace_bytes(self):
        f, b = ctypes.c_size_t(), ctypes.c_size_t()
        _check(lib().ca_plan_workspace_bytes(self.handle, ctypes.byref(f), ctypes.byref(b)))
        return int(f.value), int(b.value)

    def info(self) -> dict:
        out = np.zeros(len(self.INFO_KEYS), np.int64)
        lib().ca_plan_info(self.handle, out.ctypes.data, len(out))
        return dict(zip(self.INFO_KEYS, out.tolist()))

    def rows(self):
        n = lib().ca_plan_rows(self.handle, None, None)
        r, p = np.zeros(n, np.int32), np.zeros(n, np.int32)
        lib().ca_plan_rows(self.handle, r.ctypes.data, p.ctypes.data)
        return r, p

    def fwd_units(self):
        n = lib().ca_plan_fwd_units(self.handle, None)
        u = np.zeros((n, 5), np.int32)
        lib().ca_plan_fwd_units(self.handle, u.ctypes.data)
        return u

    def bwd_units(self):
        n = lib().ca_plan_bwd_units(self.handle, None)
        u = np.zeros((n, 10), np.int32)
        lib().ca_plan_bwd_units(self.handle, u.ctypes.data)
        return u

    def profile_enable(self, on=True):
        _check(lib().ca_profile_enable(self.handle, 1 if on else 0))

    def profile_read(self) -> dict:
        out = np.zeros(4, np.float32)
        _check(lib().ca_profile_read(self.handle, out.ctypes.data))
        return dict(zip(("fwd_kernel_ms", "bwd_prep_ms", "bwd_dkv_ms", "bwd_dq_ms"), out.tolist()))

    def destroy(self):
        if self.handle:
            lib().ca_plan_destroy(self.handle)
            self.handle = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def ca_plan_host(batch) -> Plan:
    """Validate `batch` and build its launch schedule on the host only (no GPU needed)."""
    keep = []
    d = make_desc(batch, keep)
    h = ctypes.c_void_p()
    _check(lib().ca_plan_host(ctypes.byref(d), ctypes.byref(h)))
    return Plan(h.value, batch)


def ca_plan(batch) -> Plan:
    """ca_plan_host + upload of the schedule to the current device."""
    keep = []
    d = make_desc(batch, keep)
    h = ctypes.c_void_p()
    _check(lib().ca_plan(ctypes.byref(d), ctypes.byref(h)))
    return Plan(h.value, batch)


def _stream_ptr(stream):
    if stream is None:
        import torch
        if torch.cuda.is_available():
            return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        return ctypes.c_void_p(None)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _p(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None and t.numel() > 0 else ctypes.c_void_p(None)


def _expect(t, shape, dtype, name):
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{name}: expected contiguous device tensor {tuple(shape)} {dtype}, got {tuple(t.shape)} {t.dtype}")


def ca_forward(plan: Plan, q, k, v, o, lse, ws=None, stream=None):
    """Launch the fused forward on torch's current stream (or `stream`).  Writes o (bf16) and lse (fp32)."""
    import torch
    b = plan.batch
    _expect(q, (b.total_q, b.n_q_heads, b.head_dim), torch.bfloat16, "q")
    _expect(k, (b.total_kv, b.n_kv_heads, b.head_dim), torch.bfloat16, "k")
    _expect(v, (b.total_kv, b.n_kv_heads, b.head_dim), torch.bfloat16, "v")
    _expect(o, (b.total_q, b.n_q_heads, b.head_dim), torch.bfloat16, "o")
    _expect(lse, (b.n_q_heads, b.total_q), torch.float32, "lse")
    wsb = ws.numel() * ws.element_size() if ws is not None else 0
    _check(lib().ca_forward(plan.handle, _p(q), _p(k), _p(v), _p(o), _p(lse), _p(ws), wsb, _stream_ptr(stream)))


def ca_backward(plan: Plan, q, k, v, o, d_o, lse, dq, dk, dv, ws, stream=None):
    """Launch the backward on torch's current stream (or `stream`).  Writes dq, dk, dv (bf16)."""
    import torch
    b = plan.batch
    qs, ks = (b.total_q, b.n_q_heads, b.head_dim), (b.total_kv, b.n_kv_heads, b.head_dim)
    for t, s, n in ((q, qs, "q"), (o, qs, "o"), (d_o, qs, "d_o"), (dq, qs, "dq"), (k, ks, "k"), (v, ks, "v"),
                    (dk, ks, "dk"), (dv, ks, "dv")):
        _expect(t, s, torch.bfloat16, n)
    _expect(lse, (b.n_q_heads, b.total_q), torch.float32, "lse")
    wsb = ws.numel() * ws.element_size() if ws is not None else 0
    _check(lib().ca_backward(plan.handle, _p(q), _p(k), _p(v), _p(o), _p(d_o), _p(lse), _p(dq), _p(dk), _p(dv),
                             _p(ws), wsb, _stream_ptr(stream)))


def ca_backward_static_ws(plan: Plan, q, k, v, o, d_o, lse, dq, dk, dv, stream=None):
    """ca_backward on the library's own device-resident workspace (for callers that may not allocate)."""
    import torch
    b = plan.batch
    qs, ks = (b.total_q, b.n_q_heads, b.head_dim), (b.total_kv, b.n_kv_heads, b.head_dim)
    for t, s, n in ((q, qs, "q"), (o, qs, "o"), (d_o, qs, "d_o"), (dq, qs, "dq"), (k, ks, "k"), (v, ks, "v"),
                    (dk, ks, "dk"), (dv, ks, "dv")):
        _expect(t, s, torch.bfloat16, n)
    _expect(lse, (b.n_q_heads, b.total_q), torch.float32, "lse")
    _check(lib().ca_backward_static_ws(plan.handle, _p(q), _p(k), _p(v), _p(o), _p(d_o), _p(lse), _p(dq), _p(dk),
                                       _p(dv), _stream_ptr(stream)))


def alloc_workspace(plan: Plan, device="cuda"):
    """A torch uint8 buffer big enough for both calls (torch's allocator returns 256-byte aligned blocks)."""
    import torch
    f, b = plan.workspace_bytes()
    return torch.empty(max(f, b, 256), dtype=torch.uint8, device=device)


def ca_merge_partials(part_rows, o_part, lse_part, o, lse, o_back=None, lse_back=None, stream=None):
    """Merge partial results over disjoint key windows.  part_rows: device int32 [n_parts, n_rows]; o_part bf16
    [total_q_part, Hq, D], lse_part fp32 [Hq, total_q_part]; writes o bf16 [n_rows, Hq, D] and lse fp32 [Hq, n_rows];
    o_back / lse_back (may be o_part / lse_part) receive the merged values in every partial row."""
    import torch
    n_parts, n_rows = part_rows.shape
    tq, hq, d = o_part.shape
    _expect(part_rows, (n_parts, n_rows), torch.int32, "part_rows")
    _expect(o_part, (tq, hq, d), torch.bfloat16, "o_part")
    _expect(lse_part, (hq, tq), torch.float32, "lse_part")
    _expect(o, (n_rows, hq, d), torch.bfloat16, "o")
    _expect(lse, (hq, n_rows), torch.float32, "lse")
    if o_back is not None:
        _expect(o_back, (tq, hq, d), torch.bfloat16, "o_back")
    if lse_back is not None:
        _expect(lse_back, (hq, tq), torch.float32, "lse_back")
    _check(lib().ca_merge_partials(_p(part_rows), n_rows, n_parts, _p(o_part), _p(lse_part), tq, _p(o), _p(lse),
                                   _p(o_back), _p(lse_back), hq, d, _stream_ptr(stream)))


def ca_sum_partial_dq(part_rows, dq_part, dq, stream=None):
    """dq[r] = sum of the partial query gradients of row r (arguments as in ca_merge_partials)."""
    import torch
    n_parts, n_rows = part_rows.shape
    tq, hq, d = dq_part.shape
    _expect(part_rows, (n_parts, n_rows), torch.int32, "part_rows")
    _expect(dq_part, (tq, hq, d), torch.bfloat16, "dq_part")
    _expect(dq, (n_rows, hq, d), torch.bfloat16, "dq")
    _check(lib().ca_sum_partial_dq(_p(part_rows), n_rows, n_parts, _p(dq_part), tq, _p(dq), hq, d, _stream_ptr(stream)))


def ca_mfma_stream(operands, n_mfma_per_wave, sums, side_work=0, stream=None):
    """Back-to-back bf16 MFMAs from registers in sums.shape[0] workgroups (a calibration aid; see the header)."""
    import torch
    _expect(operands, (16, 256, 8), torch.bfloat16, "operands")
    n_wg = sums.shape[0]
    _expect(sums, (n_wg, 256), torch.float32, "sums")
    _check(lib().ca_mfma_stream(_p(operands), int(n_mfma_per_wave), n_wg, int(side_work), _p(sums),
                                _stream_ptr(stream)))


def ca_xcd_map(n_workgroups, threads_per_workgroup=256, device="cuda", stream=None):
    """XCD id of every workgroup of a launch of that shape (int32 tensor on the device)."""
    import torch
    out = torch.full((n_workgroups,), -1, dtype=torch.int32, device=device)
    _check(lib().ca_xcd_map(int(n_workgroups), int(threads_per_workgroup), _p(out), _stream_ptr(stream)))
    return out


def ca_atomic_stream(operands, tiles, n_workgroups, steps, mfma_per_step, atomics_per_step, sums, stream=None):
    """fp32 atomic adds into 32 KiB tiles next to an MFMA stream (a calibration aid; see the header)."""
    import torch
    _expect(operands, (16, 256, 8), torch.bfloat16, "operands")
    n_tiles = tiles.shape[1]
    _expect(tiles, (8, n_tiles, 8192), torch.float32, "tiles")
    _expect(sums, (n_workgroups, 256), torch.float32, "sums")
    _check(lib().ca_atomic_stream(_p(operands), _p(tiles), int(n_tiles), int(n_workgroups), int(steps),
                                  int(mfma_per_step), int(atomics_per_step), _p(sums), _stream_ptr(stream)))
