"""ctypes binding of libprism.so (argument marshalling only).

Function names mirror the C ABI in ``include/prism.h``.  Tensors are torch
tensors used purely as device memory; the stream is torch's current stream.
If the library has not been built the loader raises: there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("PRISM_LIB") or os.path.join(_HERE, "libprism.so")
_lib = None

PRISM_OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_HIP, ERR_NO_MEMORY, ERR_TABLE = -1, -2, -3, -4, -5, -6

EXPORTS = (
    "prism_version", "prism_strerror", "prism_last_hip_error", "prism_plan_create",
    "prism_plan_dry_run", "prism_plan_workspace_bytes", "prism_plan_get_info", "prism_plan_forget_workspace",
    "prism_plan_destroy", "prism_kv_append",
    "prism_prefix_attention", "prism_prefix_prefill", "prism_prefix_prefill_static", "prism_validate",
    "prism_plan_profile_enable", "prism_plan_profile_read", "prism_measure_peaks",
)


class PrismError(RuntimeError):
    def __init__(self, code: int, where: str):
        lib = load()
        msg = lib.prism_strerror(code).decode()
        if code == ERR_HIP:
            msg += " (" + lib.prism_last_hip_error().decode() + ")"
        super().__init__(f"{where}: {msg} [{code}]")
        self.code = code


class Shape(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_pages", ctypes.c_int32), ("batch", ctypes.c_int32),
                ("max_blocks_per_req", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class PlanOptions(ctypes.Structure):
    _fields_ = [("tile_rows", ctypes.c_int32), ("split_kv", ctypes.c_int32),
                ("min_split_keys", ctypes.c_int32), ("rows_per_wave", ctypes.c_int32),
                ("reserved", ctypes.c_int32 * 4),
                ("block_table_host", ctypes.c_void_p)]


class PlanInfo(ctypes.Structure):
    _fields_ = [("tile_rows", ctypes.c_int32), ("tile_keys", ctypes.c_int32),
                ("num_items", ctypes.c_int32), ("num_split_items", ctypes.c_int32),
                ("num_reduce_groups", ctypes.c_int32), ("total_suffix", ctypes.c_int32),
                ("rows_per_wave", ctypes.c_int32), ("reserved", ctypes.c_int32 * 1), ("flops", ctypes.c_int64),
                ("kv_bytes_per_request", ctypes.c_int64)]


def load():
    """Load libprism.so; raise if it is missing (build it with build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2605_08581_amd.build` "
                           "(there is no CPU or PyTorch fallback)")
    # PyTorch supplies the device memory and streams, so the library must use
    # the HIP runtime PyTorch ships (same SONAME): make sure that copy is the
    # one already in the process before libprism.so resolves its dependency.
    import torch
    rt = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    if os.path.exists(rt):
        ctypes.CDLL(rt, mode=ctypes.RTLD_GLOBAL)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
    lib.prism_version.restype = ctypes.c_int
    lib.prism_strerror.restype = ctypes.c_char_p
    lib.prism_strerror.argtypes = [ctypes.c_int]
    lib.prism_last_hip_error.restype = ctypes.c_char_p
    lib.prism_plan_create.restype = ctypes.c_int
    lib.prism_plan_create.argtypes = [ctypes.POINTER(Shape), vp, vp, ctypes.POINTER(PlanOptions),
                                      ctypes.POINTER(vp)]
    lib.prism_plan_dry_run.restype = ctypes.c_int
    lib.prism_plan_dry_run.argtypes = [ctypes.POINTER(Shape), vp, vp, ctypes.POINTER(PlanOptions),
                                       ctypes.POINTER(PlanInfo), ctypes.POINTER(ctypes.c_size_t), vp,
                                       ctypes.c_int32]
    lib.prism_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.prism_plan_workspace_bytes.argtypes = [vp]
    lib.prism_plan_get_info.restype = ctypes.c_int
    lib.prism_plan_get_info.argtypes = [vp, ctypes.POINTER(PlanInfo)]
    lib.prism_plan_forget_workspace.restype = ctypes.c_int
    lib.prism_plan_forget_workspace.argtypes = [vp]
    lib.prism_plan_destroy.restype = None
    lib.prism_plan_destroy.argtypes = [vp]
    lib.prism_kv_append.restype = ctypes.c_int
    lib.prism_kv_append.argtypes = [vp] * 7
    lib.prism_prefix_attention.restype = ctypes.c_int
    lib.prism_prefix_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.prism_prefix_prefill.restype = ctypes.c_int
    lib.prism_prefix_prefill.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.prism_prefix_prefill_static.restype = ctypes.c_int
    lib.prism_prefix_prefill_static.argtypes = [vp] * 9
    lib.prism_validate.restype = ctypes.c_int
    lib.prism_validate.argtypes = [ctypes.POINTER(Shape), vp, vp, vp]
    lib.prism_plan_profile_enable.restype = ctypes.c_int
    lib.prism_plan_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.prism_plan_profile_read.restype = ctypes.c_int
    lib.prism_plan_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                            ctypes.POINTER(ctypes.c_double), i32p]
    _ = i32p
    _lib = lib
    return lib


def prism_version() -> int:
    return int(load().prism_version())


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    return ctypes.c_void_p(t.data_ptr())


def _check(name, t, dtype, numel, optional=False):
    """The C ABI takes bare pointers: refuse a tensor that is not what the plan
    was made for (device, dtype, contiguity, element count) before it gets there."""
    import torch
    if t is None:
        if optional or numel == 0:
            return
        raise ValueError(f"{name}: missing")
    if not t.is_cuda:
        raise ValueError(f"{name}: must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    want = {"bf16": torch.bfloat16, "i32": torch.int32, "u8": torch.uint8}[dtype]
    if t.dtype != want:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {want}")
    if t.numel() < numel:
        raise ValueError(f"{name}: {t.numel()} elements, the plan needs {numel}")


def _stream() -> ctypes.c_void_p:
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_shape(num_q_heads, num_kv_heads, head_dim, num_pages, batch, max_blocks_per_req,
               softmax_scale, page_size=16) -> Shape:
    return Shape(num_q_heads, num_kv_heads, head_dim, page_size, num_pages, batch,
                 max_blocks_per_req, softmax_scale)


def prism_validate(shape: Shape, prefix_len, suffix_len, block_table) -> int:
    pl, sl, bt = _host_i32(prefix_len), _host_i32(suffix_len), _host_i32(block_table)
    return int(load().prism_validate(ctypes.byref(shape), pl.ctypes.data, sl.ctypes.data, bt.ctypes.data))


def _options(tile_rows, split_kv, min_split_keys, block_table, rows_per_wave=0):
    """PlanOptions plus the host array it points to (keep both alive during the call)."""
    opt = PlanOptions(tile_rows, split_kv, min_split_keys, rows_per_wave)
    bt = None
    if block_table is not None:
        bt = _host_i32(block_table)
        opt.block_table_host = bt.ctypes.data
    return opt, bt


def prism_plan_dry_run(shape: Shape, prefix_len, suffix_len, tile_rows: int = 0, split_kv: int = 0,
                       min_split_keys: int = 0, block_table=None, rows_per_wave: int = 0):
    """Host-only schedule: returns (PlanInfo, workspace_bytes, items int32 [n, 8])."""
    lib = load()
    pl, sl = _host_i32(prefix_len), _host_i32(suffix_len)
    opt, _bt = _options(tile_rows, split_kv, min_split_keys, block_table, rows_per_wave)
    info, ws = PlanInfo(), ctypes.c_size_t()
    n = lib.prism_plan_dry_run(ctypes.byref(shape), pl.ctypes.data, sl.ctypes.data, ctypes.byref(opt),
                               ctypes.byref(info), ctypes.byref(ws), None, 0)
    if n < 0:
        raise PrismError(n, "prism_plan_dry_run")
    items = np.zeros((n, 8), dtype=np.int32)
    if n:
        lib.prism_plan_dry_run(ctypes.byref(shape), pl.ctypes.data, sl.ctypes.data, ctypes.byref(opt),
                               None, None, items.ctypes.data, n)
    return info, int(ws.value), items


class Plan:
    """Owns a prism_plan_t*.  Methods are the C entry points of the same name."""

    def __init__(self, shape: Shape, prefix_len, suffix_len, tile_rows: int = 0, split_kv: int = 0,
                 min_split_keys: int = 0, block_table=None, rows_per_wave: int = 0):
        lib = load()
        self._lib = lib
        self._h = ctypes.c_void_p()
        self.shape = shape
        pl, sl = _host_i32(prefix_len), _host_i32(suffix_len)
        if pl.shape != (shape.batch,) or sl.shape != (shape.batch,):
            raise ValueError("prefix_len/suffix_len must have `batch` entries")
        if block_table is not None and tuple(np.shape(block_table)) != (shape.batch, shape.max_blocks_per_req):
            raise ValueError("block_table must be [batch, max_blocks_per_req]")
        opt, _bt = _options(tile_rows, split_kv, min_split_keys, block_table, rows_per_wave)
        self._total_suffix = int(sl.sum())
        rc = lib.prism_plan_create(ctypes.byref(shape), pl.ctypes.data, sl.ctypes.data,
                                   ctypes.byref(opt), ctypes.byref(self._h))
        if rc != PRISM_OK:
            self._h = ctypes.c_void_p()
            raise PrismError(rc, "prism_plan_create")

    def close(self):
        h = getattr(self, "_h", None)
        if h is not None and h.value and ctypes is not None:
            self._lib.prism_plan_destroy(h)
            self._h.value = None

    __del__ = close

    def prism_plan_workspace_bytes(self) -> int:
        return int(self._lib.prism_plan_workspace_bytes(self._h))

    def prism_plan_get_info(self) -> PlanInfo:
        info = PlanInfo()
        rc = self._lib.prism_plan_get_info(self._h, ctypes.byref(info))
        if rc != PRISM_OK:
            raise PrismError(rc, "prism_plan_get_info")
        return info

    def prism_plan_forget_workspace(self):
        self._lib.prism_plan_forget_workspace(self._h)

    def _check_call(self, q, k_suffix, v_suffix, k_pool, v_pool, block_table, out, workspace):
        sh, n = self.shape, self._total_suffix
        row_q, row_kv = sh.num_q_heads * sh.head_dim, sh.num_kv_heads * sh.head_dim
        if q is not False:
            _check("q", q, "bf16", n * row_q)
            _check("out", out, "bf16", n * row_q)
            _check("workspace", workspace, "u8", self.prism_plan_workspace_bytes(), optional=True)
        if k_suffix is not False:
            _check("k_suffix", k_suffix, "bf16", n * row_kv)
            _check("v_suffix", v_suffix, "bf16", n * row_kv)
        pool = sh.num_pages * sh.page_size * row_kv
        _check("k_pool", k_pool, "bf16", pool)
        _check("v_pool", v_pool, "bf16", pool)
        _check("block_table", block_table, "i32", sh.batch * sh.max_blocks_per_req)

    def prism_kv_append(self, k_suffix, v_suffix, k_pool, v_pool, block_table):
        self._check_call(False, k_suffix, v_suffix, k_pool, v_pool, block_table, None, None)
        rc = self._lib.prism_kv_append(self._h, _ptr(k_suffix), _ptr(v_suffix), _ptr(k_pool),
                                       _ptr(v_pool), _ptr(block_table), _stream())
        if rc != PRISM_OK:
            raise PrismError(rc, "prism_kv_append")

    def prism_prefix_attention(self, q, k_pool, v_pool, block_table, out, workspace=None):
        if workspace is not None and workspace.numel() >= self.prism_plan_workspace_bytes():
            self._check_call(q, False, False, k_pool, v_pool, block_table, out, workspace)   # size errors come from the library
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        rc = self._lib.prism_prefix_attention(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool),
                                              _ptr(block_table), _ptr(out), _ptr(workspace),
                                              nbytes, _stream())
        if rc != PRISM_OK:
            raise PrismError(rc, "prism_prefix_attention")

    def prism_prefix_prefill(self, q, k_suffix, v_suffix, k_pool, v_pool, block_table, out,
                             workspace=None):
        if workspace is not None and workspace.numel() >= self.prism_plan_workspace_bytes():
            self._check_call(q, k_suffix, v_suffix, k_pool, v_pool, block_table, out, workspace)
        nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        rc = self._lib.prism_prefix_prefill(self._h, _ptr(q), _ptr(k_suffix), _ptr(v_suffix),
                                            _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                            _ptr(out), _ptr(workspace), nbytes, _stream())
        if rc != PRISM_OK:
            raise PrismError(rc, "prism_prefix_prefill")

    def prism_prefix_prefill_static(self, q, k_suffix, v_suffix, k_pool, v_pool, block_table, out):
        self._check_call(q, k_suffix, v_suffix, k_pool, v_pool, block_table, out, None)
        rc = self._lib.prism_prefix_prefill_static(self._h, _ptr(q), _ptr(k_suffix), _ptr(v_suffix),
                                                   _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                                   _ptr(out), _stream())
        if rc != PRISM_OK:
            raise PrismError(rc, "prism_prefix_prefill_static")

    def prism_plan_profile_enable(self, on: bool):
        self._lib.prism_plan_profile_enable(self._h, int(on))

    def prism_plan_profile_read(self):
        a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        n = ctypes.c_int32()
        rc = self._lib.prism_plan_profile_read(self._h, ctypes.byref(a), ctypes.byref(b),
                                               ctypes.byref(c), ctypes.byref(n))
        if rc != PRISM_OK:
            raise PrismError(rc, "prism_plan_profile_read")
        return {"append_ms": a.value, "attention_ms": b.value, "reduce_ms": c.value, "launches": n.value}


def prism_measure_peaks(scratch, repeats: int = 3):
    """(MFMA TFLOP/s, streaming-read GB/s) measured on the current device;
    scratch is a device tensor of at least 1 MiB (1 GiB or more for a
    meaningful read figure)."""
    lib = load()
    m, h = ctypes.c_double(), ctypes.c_double()
    lib.prism_measure_peaks.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32,
                                        ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                        ctypes.c_void_p]
    rc = lib.prism_measure_peaks(_ptr(scratch), scratch.numel() * scratch.element_size(), repeats,
                                 ctypes.byref(m), ctypes.byref(h), _stream())
    if rc != PRISM_OK:
        raise PrismError(rc, "prism_measure_peaks")
    return m.value, h.value


def shape_of(batch) -> Shape:
    """prism_shape_t for a workload.Batch."""
    g = batch.geom
    return make_shape(g.num_q_heads, g.num_kv_heads, g.head_dim, batch.num_pages, batch.batch,
                      batch.max_blocks, batch.softmax_scale, g.page_size)
