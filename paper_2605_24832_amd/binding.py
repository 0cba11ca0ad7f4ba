"""ctypes binding of ``liboptimus_attn.so``: argument marshalling only.

Every step of the path (planning, KV append, attention, merge) runs inside the
C-ABI library; this module converts numpy descriptors and torch device tensors
to pointers and checks status codes.  There is no fallback: if the library is
missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboptimus_attn.so")
_lib = None

EXPORTS = (
    "optimus_attn_plan_create", "optimus_attn_plan_update", "optimus_kv_append",
    "optimus_attn_forward", "optimus_attn_forward_pos", "optimus_attn_forward_static", "optimus_attn_static_scratch_bytes",
    "optimus_attn_step",
    "optimus_attn_plan_destroy", "optimus_attn_plan_num_work_items",
    "optimus_attn_plan_num_merge_items", "optimus_attn_plan_get_work_items",
    "optimus_attn_plan_set_tuning", "optimus_attn_set_timing", "optimus_attn_timing_read",
    "optimus_status_string", "optimus_last_hip_error",
    "optimus_kv_write", "optimus_commit_forward", "optimus_reorg_forward",
    "optimus_latency_fit", "optimus_latency_eval", "optimus_select_chunk",
)


class OptimusError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = f"{where}: {status_string(status)} ({status})"
        if status == -11:
            msg += f": {load_library().optimus_last_hip_error().decode()}"
        super().__init__(msg)


class _CParams(ctypes.Structure):
    _fields_ = [
        ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("block_size", ctypes.c_int32), ("mask_mode", ctypes.c_int32),
        ("out_dtype", ctypes.c_int32), ("kv_layout", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("num_pages", ctypes.c_int32),
        ("max_pages_per_req", ctypes.c_int32), ("reserved0", ctypes.c_int32),
        ("k_stride_page", ctypes.c_int64), ("k_stride_head", ctypes.c_int64),
        ("v_stride_page", ctypes.c_int64), ("v_stride_head", ctypes.c_int64),
    ]


class _CCommitParams(ctypes.Structure):
    _fields_ = [
        ("num_tokens", ctypes.c_int32), ("vocab", ctypes.c_int32), ("row_stride", ctypes.c_int64),
        ("threshold", ctypes.c_float), ("batch", ctypes.c_int32), ("min_commit", ctypes.c_int32),
        ("reserved0", ctypes.c_int32),
    ]


class WorkItem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("req", "kv_head", "row_begin", "row_count", "kv_begin", "kv_end", "part_row",
                 "q_token0")]


def library_path() -> str:
    return _LIB_PATH


class LatencyModel(ctypes.Structure):
    """optimus_latency_model_t: three affine regimes over x = batch * chunk."""
    _fields_ = [("x_break", ctypes.c_double * 2), ("beta1", ctypes.c_double * 3),
                ("beta0", ctypes.c_double * 3)]


def load_library():
    """Load the HIP library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2605_24832_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32, i32p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)
        lib.optimus_attn_plan_create.argtypes = [ctypes.POINTER(_CParams), ctypes.c_int,
                                                 ctypes.POINTER(vp)]
        lib.optimus_attn_plan_update.argtypes = [vp, i32, vp, vp, vp, vp,
                                                 ctypes.POINTER(ctypes.c_size_t)]
        lib.optimus_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        lib.optimus_attn_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.optimus_attn_forward_pos.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.optimus_attn_forward_static.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        lib.optimus_attn_step.argtypes = [vp, i32] + [vp] * 13 + [ctypes.c_size_t, vp]
        lib.optimus_attn_static_scratch_bytes.argtypes = []
        lib.optimus_attn_static_scratch_bytes.restype = ctypes.c_size_t
        lib.optimus_attn_plan_destroy.argtypes = [vp]
        lib.optimus_attn_plan_destroy.restype = None
        lib.optimus_attn_plan_num_work_items.argtypes = [vp]
        lib.optimus_attn_plan_num_work_items.restype = i32
        lib.optimus_attn_plan_num_merge_items.argtypes = [vp]
        lib.optimus_attn_plan_num_merge_items.restype = i32
        lib.optimus_attn_plan_get_work_items.argtypes = [vp, ctypes.POINTER(WorkItem), i32]
        lib.optimus_attn_plan_get_work_items.restype = i32
        lib.optimus_attn_plan_set_tuning.argtypes = [vp, i32, i32, i32]
        lib.optimus_attn_set_timing.argtypes = [vp, i32]
        lib.optimus_attn_timing_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float),
                                                 ctypes.POINTER(ctypes.c_int32)]
        lib.optimus_kv_write.argtypes = [ctypes.POINTER(_CParams), ctypes.c_int, vp, vp, vp, vp, vp,
                                         i32, i32, i32, vp]
        lib.optimus_commit_forward.argtypes = [ctypes.POINTER(_CCommitParams), ctypes.c_int, vp, vp,
                                               vp, vp, vp, vp]
        lib.optimus_reorg_forward.argtypes = [ctypes.c_int, i32, i32] + [vp] * 10
        dp = ctypes.POINTER(ctypes.c_double)
        mp = ctypes.POINTER(LatencyModel)
        lib.optimus_latency_fit.argtypes = [i32, dp, dp, mp, dp]
        lib.optimus_latency_eval.argtypes = [mp, ctypes.c_double]
        lib.optimus_latency_eval.restype = ctypes.c_double
        lib.optimus_select_chunk.argtypes = [mp, i32, i32, ctypes.POINTER(i32), dp, ctypes.POINTER(i32), dp]
        lib.optimus_status_string.argtypes = [ctypes.c_int]
        lib.optimus_status_string.restype = ctypes.c_char_p
        lib.optimus_last_hip_error.argtypes = []
        lib.optimus_last_hip_error.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def static_scratch_bytes() -> int:
    return int(load_library().optimus_attn_static_scratch_bytes())


def status_string(status: int) -> str:
    return load_library().optimus_status_string(int(status)).decode()


@dataclass
class AttnParams:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    block_size: int
    num_pages: int
    max_pages_per_req: int
    mask_mode: int = 0
    out_dtype: int = 0          # 0 bf16, 1 fp32
    kv_layout: int = 1
    softmax_scale: float = 0.0  # <= 0 -> 1/sqrt(D)
    k_stride_page: int | None = None
    k_stride_head: int | None = None
    v_stride_page: int | None = None
    v_stride_head: int | None = None

    def to_c(self) -> _CParams:
        tile = self.page_size * self.head_dim
        c = _CParams()
        for f in ("num_q_heads", "num_kv_heads", "head_dim", "page_size", "block_size",
                  "mask_mode", "out_dtype", "kv_layout", "num_pages", "max_pages_per_req"):
            setattr(c, f, int(getattr(self, f)))
        c.softmax_scale = float(self.softmax_scale)
        c.k_stride_head = tile if self.k_stride_head is None else self.k_stride_head
        c.v_stride_head = tile if self.v_stride_head is None else self.v_stride_head
        c.k_stride_page = self.num_kv_heads * tile if self.k_stride_page is None else self.k_stride_page
        c.v_stride_page = self.num_kv_heads * tile if self.v_stride_page is None else self.v_stride_page
        return c


# The marshalling below runs two or three times per decoding iteration, next to kernels of a
# few microseconds: addresses are passed as plain integers (the argtypes are void pointers).

def _ptr(t):
    """Device address of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


def _i32(a):
    """Host int32 array and its address (the array must stay alive during the call)."""
    if not (isinstance(a, np.ndarray) and a.dtype == np.int32 and a.flags.c_contiguous):
        a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.__array_interface__["data"][0]


_raw_stream = None


def _stream_ptr(stream):
    """torch stream -> hipStream_t; None = torch's current stream (the null stream without a GPU)."""
    global _raw_stream
    if stream is not None:
        return stream.cuda_stream
    import torch
    if _raw_stream is None:
        if not torch.cuda.is_available():
            return None
        # the raw-handle query skips building a Stream object on every call
        fast = getattr(torch._C, "_cuda_getCurrentRawStream", None)
        _raw_stream = fast if fast is not None else (lambda dev: torch.cuda.current_stream(dev).cuda_stream)
    return _raw_stream(torch.cuda.current_device())


class HostBatch:
    """The host descriptors of a batch, marshalled once: int32 arrays ``cu_q [batch+1]``,
    ``prefix_len [batch]``, ``block_start [batch]`` and, optionally, ``block_table
    [batch, max_pages_per_req]`` together with their addresses.  A decoding loop keeps one of
    these and rewrites the arrays in place between iterations (the attributes are the arrays
    the library reads), which takes the per-call conversions out of ``Plan.attn_step``."""

    def __init__(self, cu_q, prefix_len, block_start, block_table=None):
        self._cu_q = np.array(cu_q, dtype=np.int32, order="C")
        self._prefix_len = np.array(prefix_len, dtype=np.int32, order="C")
        self._block_start = np.array(block_start, dtype=np.int32, order="C")
        self._block_table = None if block_table is None else np.array(block_table, dtype=np.int32, order="C")
        if len(self._cu_q) != len(self._prefix_len) + 1 or len(self._block_start) != len(self._prefix_len):
            raise ValueError("cu_q must have batch+1 entries, prefix_len and block_start batch")
        self.batch = len(self._prefix_len)
        self._p = (_i32(self._cu_q)[1], _i32(self._prefix_len)[1], _i32(self._block_start)[1],
                   None if self._block_table is None else _i32(self._block_table)[1])

    # read-only attributes: the arrays can be rewritten (``hb.cu_q[:] = ...``), not replaced
    cu_q = property(lambda self: self._cu_q)
    prefix_len = property(lambda self: self._prefix_len)
    block_start = property(lambda self: self._block_start)
    block_table = property(lambda self: self._block_table)


class DeviceBuffers:
    """The device tensors of ``Plan.attn_step`` resolved to addresses once (the tensors are kept
    alive here): for loops that run every iteration on the same buffers."""

    def __init__(self, q, k_new, v_new, k_pool, v_pool, block_table, out, workspace=None, q_pos=None):
        self._keep = (q, k_new, v_new, k_pool, v_pool, block_table, out, workspace, q_pos)
        self._p = (_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                   _ptr(q_pos), _ptr(out), _ptr(workspace))
        self._ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()


class Plan:
    """Owner of one ``optimus_attn_plan_t``; method names follow the C entry points."""

    def __init__(self, params: AttnParams, device: int = 0):
        self._lib = load_library()
        self.params = params
        self.device = device
        self._h = ctypes.c_void_p(0)
        cp = params.to_c()
        rc = self._lib.optimus_attn_plan_create(ctypes.byref(cp), int(device), ctypes.byref(self._h))
        if rc != 0:
            self._h = ctypes.c_void_p(0)
            raise OptimusError(rc, "optimus_attn_plan_create")
        self.workspace_bytes = 0

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.optimus_attn_plan_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def plan_update(self, cu_q, prefix_len, block_start, block_table=None) -> int:
        cu, cu_p = _i32(cu_q)
        pl, pl_p = _i32(prefix_len)
        bs, bs_p = _i32(block_start)
        if block_table is None:
            bt_p = None
        else:
            bt, bt_p = _i32(block_table)
        if len(cu) != len(pl) + 1 or len(bs) != len(pl):
            raise ValueError("cu_q must have batch+1 entries, prefix_len and block_start batch")
        ws = ctypes.c_size_t(0)
        rc = self._lib.optimus_attn_plan_update(self._h, len(pl), cu_p, pl_p, bs_p, bt_p,
                                                ctypes.byref(ws))
        if rc != 0:
            raise OptimusError(rc, "optimus_attn_plan_update")
        self.workspace_bytes = int(ws.value)
        return self.workspace_bytes

    def set_tuning(self, target_items=0, min_split_tokens=0, max_split_tokens=0):
        rc = self._lib.optimus_attn_plan_set_tuning(self._h, target_items, min_split_tokens,
                                                    max_split_tokens)
        if rc != 0:
            raise OptimusError(rc, "optimus_attn_plan_set_tuning")

    def num_work_items(self) -> int:
        return int(self._lib.optimus_attn_plan_num_work_items(self._h))

    def num_merge_items(self) -> int:
        return int(self._lib.optimus_attn_plan_num_merge_items(self._h))

    def work_items(self) -> np.ndarray:
        """Structured array with the fields of ``optimus_work_item_t``."""
        n = self.num_work_items()
        buf = (WorkItem * max(n, 1))()
        got = self._lib.optimus_attn_plan_get_work_items(self._h, buf, n)
        if got < 0:
            raise OptimusError(got, "optimus_attn_plan_get_work_items")
        arr = np.frombuffer(buf, dtype=np.dtype([(f, np.int32) for f, _ in WorkItem._fields_]))
        return arr[:got].copy()

    def kv_append(self, k_pool, v_pool, k_new, v_new, block_table, stream=None) -> None:
        rc = self._lib.optimus_kv_append(self._h, _ptr(k_pool), _ptr(v_pool), _ptr(k_new),
                                         _ptr(v_new), _ptr(block_table), _stream_ptr(stream))
        if rc != 0:
            raise OptimusError(rc, "optimus_kv_append")

    def attn_forward(self, q, k_pool, v_pool, block_table, out, workspace=None, stream=None,
                     q_pos=None) -> None:
        """optimus_attn_forward, or optimus_attn_forward_pos when ``q_pos`` (int32 device tensor) is given."""
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        if q_pos is None:
            rc = self._lib.optimus_attn_forward(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool),
                                                _ptr(block_table), _ptr(out), _ptr(workspace),
                                                ctypes.c_size_t(ws_bytes), _stream_ptr(stream))
        else:
            rc = self._lib.optimus_attn_forward_pos(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool),
                                                    _ptr(block_table), _ptr(q_pos), _ptr(out),
                                                    _ptr(workspace), ctypes.c_size_t(ws_bytes),
                                                    _stream_ptr(stream))
        if rc != 0:
            raise OptimusError(rc, "optimus_attn_forward")

    def attn_step(self, cu_q, prefix_len, block_start, block_table_host, q, k_new, v_new, k_pool, v_pool,
                  block_table, out, workspace=None, stream=None, q_pos=None) -> None:
        """optimus_attn_step: plan_update, kv_append and attn_forward in one call (host descriptors
        as for ``plan_update``; ``workspace`` must be large enough for the new plan)."""
        cu, cu_p = _i32(cu_q)
        pl, pl_p = _i32(prefix_len)
        bs, bs_p = _i32(block_start)
        if block_table_host is None:
            bt_p = None
        else:
            bt, bt_p = _i32(block_table_host)
        if len(cu) != len(pl) + 1 or len(bs) != len(pl):
            raise ValueError("cu_q must have batch+1 entries, prefix_len and block_start batch")
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        rc = self._lib.optimus_attn_step(self._h, len(pl), cu_p, pl_p, bs_p, bt_p, _ptr(q), _ptr(k_new),
                                         _ptr(v_new), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                         _ptr(q_pos), _ptr(out), _ptr(workspace), ws_bytes,
                                         _stream_ptr(stream))
        if rc != 0:
            raise OptimusError(rc, "optimus_attn_step")
        self.workspace_bytes = 0

    def attn_step_bound(self, host: HostBatch, dev: DeviceBuffers, stream=None) -> None:
        """optimus_attn_step on descriptors and buffers marshalled beforehand (same call, same
        checks in the library; only the per-call conversions of ``attn_step`` are gone)."""
        h, d = host._p, dev._p
        rc = self._lib.optimus_attn_step(self._h, host.batch, h[0], h[1], h[2], h[3], d[0], d[1], d[2],
                                         d[3], d[4], d[5], d[6], d[7], d[8], dev._ws_bytes,
                                         _stream_ptr(stream))
        if rc != 0:
            raise OptimusError(rc, "optimus_attn_step")
        self.workspace_bytes = 0

    def attn_forward_static(self, q, k_pool, v_pool, block_table, out, stream=None) -> None:
        """optimus_attn_forward_static: the split-KV partials go to the library's static scratch."""
        rc = self._lib.optimus_attn_forward_static(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool),
                                                   _ptr(block_table), _ptr(out), _stream_ptr(stream))
        if rc != 0:
            raise OptimusError(rc, "optimus_attn_forward_static")

    def set_timing(self, every) -> None:
        """0 / False: off; n (True = 1): time the attention kernel of every n-th forward."""
        rc = self._lib.optimus_attn_set_timing(self._h, int(every))
        if rc != 0:
            raise OptimusError(rc, "optimus_attn_set_timing")

    def timing_read(self):
        """(summed attention-kernel milliseconds, forwards timed) since set_timing."""
        ms = ctypes.c_float(0)
        n = ctypes.c_int32(0)
        rc = self._lib.optimus_attn_timing_read(self._h, ctypes.byref(ms), ctypes.byref(n))
        if rc != 0:
            raise OptimusError(rc, "optimus_attn_timing_read")
        return float(ms.value), int(n.value)


def commit_params(num_tokens, vocab, row_stride, threshold=0.9, batch=0, min_commit=0) -> _CCommitParams:
    c = _CCommitParams()
    c.num_tokens, c.vocab, c.row_stride = int(num_tokens), int(vocab), int(row_stride)
    c.threshold, c.batch, c.min_commit = float(threshold), int(batch), int(min_commit)
    return c


def commit_forward(params: _CCommitParams, logits, cu_q, token_out, conf_out, commit_out,
                   device: int = 0, stream=None) -> None:
    """optimus_commit_forward on torch device tensors (argument marshalling only)."""
    rc = load_library().optimus_commit_forward(
        ctypes.byref(params), int(device), _ptr(logits), _ptr(cu_q), _ptr(token_out), _ptr(conf_out),
        _ptr(commit_out), _stream_ptr(stream))
    if rc != 0:
        raise OptimusError(rc, "optimus_commit_forward")


def kv_write(params: AttnParams, k_pool, v_pool, k_src, v_src, block_table, req: int, first_slot: int,
             device: int = 0, stream=None) -> None:
    """optimus_kv_write: the rows of ``k_src`` / ``v_src`` (bf16 ``[n, Hkv, D]``) go to the logical
    slots ``first_slot ..`` of request ``req`` (argument marshalling only)."""
    cp = params.to_c()
    rc = load_library().optimus_kv_write(
        ctypes.byref(cp), int(device), _ptr(k_pool), _ptr(v_pool), _ptr(k_src), _ptr(v_src),
        _ptr(block_table), int(req), int(first_slot), int(k_src.shape[0]), _stream_ptr(stream))
    if rc != 0:
        raise OptimusError(rc, "optimus_kv_write")


def reorg_forward(decoded, block_start, chunk_req, chunk_out, cu_q_out, prefix_len_out, q_pos_out,
                  kv_slot_out, token_req_out, device: int = 0, stream=None) -> None:
    """optimus_reorg_forward on torch device tensors (argument marshalling only)."""
    batch, block_size = decoded.shape
    rc = load_library().optimus_reorg_forward(
        int(device), int(batch), int(block_size), _ptr(decoded), _ptr(block_start), _ptr(chunk_req),
        _ptr(chunk_out), _ptr(cu_q_out), _ptr(prefix_len_out), _ptr(q_pos_out), _ptr(kv_slot_out),
        _ptr(token_req_out), _stream_ptr(stream))
    if rc != 0:
        raise OptimusError(rc, "optimus_reorg_forward")


def _dbl(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def latency_fit(x, latency):
    """optimus_latency_fit on host arrays: returns ``(LatencyModel, sse)``."""
    xa, xp = _dbl(x)
    ta, tp = _dbl(latency)
    if xa.shape != ta.shape or xa.ndim != 1:
        raise ValueError("x and latency must be 1-d arrays of one length")
    m, sse = LatencyModel(), ctypes.c_double()
    rc = load_library().optimus_latency_fit(len(xa), xp, tp, ctypes.byref(m), ctypes.byref(sse))
    if rc != 0:
        raise OptimusError(rc, "optimus_latency_fit")
    return m, sse.value


def latency_eval(model: LatencyModel, x: float) -> float:
    return float(load_library().optimus_latency_eval(ctypes.byref(model), float(x)))


def select_chunk(model: LatencyModel, batch: int, chunk_sizes, n_commit):
    """optimus_select_chunk: returns ``(best_index, rates float64 [num_candidates])``."""
    cs = np.ascontiguousarray(chunk_sizes, dtype=np.int32)
    na, np_ = _dbl(n_commit)
    if cs.shape != na.shape or cs.ndim != 1:
        raise ValueError("chunk_sizes and n_commit must be 1-d arrays of one length")
    rates = np.zeros(len(cs), dtype=np.float64)
    best = ctypes.c_int32(-1)
    rc = load_library().optimus_select_chunk(
        ctypes.byref(model), int(batch), len(cs), cs.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
        np_, ctypes.byref(best), rates.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise OptimusError(rc, "optimus_select_chunk")
    return int(best.value), rates
