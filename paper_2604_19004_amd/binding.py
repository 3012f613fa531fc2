"""Thin ctypes binding of libocean_spgemm.so: argument marshalling only.

Every step of the SpGEMM path runs inside the HIP library; PyTorch is used
for device memory (tensors back every buffer, including the ones the library
asks for through its allocator callback) and for the stream.  There is no CPU
fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

import numpy as np

from . import build as _build

F64, F32 = 0, 1
WF_AUTO, WF_UPPER_BOUND, WF_HLL, WF_SYMBOLIC = 0, 1, 2, 3
SEL_TABLE1, SEL_MI355X = 0, 1
WORKFLOW_NAMES = {WF_AUTO: "auto", WF_UPPER_BOUND: "upper_bound", WF_HLL: "hll", WF_SYMBOLIC: "symbolic"}
MAX_BINS = 12
STAGES = ("analysis", "sketch", "sample", "predict", "binning", "numeric", "retry", "compact")


class ocean_csr(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("nnz", C.c_int64), ("row_ptr", C.c_void_p),
                ("col_idx", C.c_void_p), ("val", C.c_void_p), ("dtype", C.c_int32), ("reserved", C.c_int32)]


ALLOC_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p))
RELEASE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class ocean_allocator(C.Structure):
    _fields_ = [("ctx", C.c_void_p), ("alloc", ALLOC_FN), ("release", RELEASE_FN)]


class ocean_options(C.Structure):
    _fields_ = [("workflow", C.c_int32), ("hll_registers", C.c_int32), ("upper_bound_avg_products", C.c_double),
                ("er_threshold", C.c_double), ("cr_threshold", C.c_double), ("expand_coef", C.c_double),
                ("exact_load_coef", C.c_double), ("sample_ratio", C.c_double), ("sample_min", C.c_int32),
                ("sample_max", C.c_int32), ("sample_seed", C.c_uint32), ("estimate_scale", C.c_double),
                ("validate_inputs", C.c_int32), ("force_hash_kernels", C.c_int32), ("assisted_symbolic", C.c_int32),
                ("assist_sigmas", C.c_double), ("bitmap_query", C.c_int32), ("esc_short_rows", C.c_int32),
                ("bitmap_query_cr", C.c_double), ("selector", C.c_int32), ("compact_in_place", C.c_int32),
                ("tuned_cr_light", C.c_double), ("tuned_cr_heavy", C.c_double), ("tuned_min_products", C.c_double),
                ("tuned_cr_bound", C.c_double), ("bound_load_coef", C.c_double), ("estimate_table_coef", C.c_double), ("dense_range", C.c_int32), ("sort_b_ratio", C.c_double),
                ("allocator", C.POINTER(ocean_allocator))]


class ocean_stats(C.Structure):
    _fields_ = [("products", C.c_int64), ("max_row_products", C.c_int64), ("heavy_products", C.c_int64), ("nnz_c", C.c_int64), ("er", C.c_double),
                ("avg_products", C.c_double), ("sampled_cr", C.c_double), ("cr_mean", C.c_double),
                ("cr_std", C.c_double), ("assist_cr", C.c_double), ("workflow", C.c_int32),
                ("hll_registers", C.c_int32), ("sampled_rows", C.c_int32), ("fell_back", C.c_int32),
                ("rows_per_bin", C.c_int64 * MAX_BINS), ("symbolic_rows_per_bin", C.c_int64 * MAX_BINS),
                ("overflow_rows", C.c_int64), ("symbolic_overflow_rows", C.c_int64), ("temp_slots", C.c_int64), ("peak_bytes", C.c_int64),
                ("compacted_in_place", C.c_int32), ("b_sorted_copy", C.c_int32), ("dense_range_rows", C.c_int32),
                ("stage_ms", C.c_float * 8), ("total_ms", C.c_float), ("bin_ms", C.c_float * MAX_BINS),
                ("bin_products", C.c_int64 * MAX_BINS), ("bin_nnz_a", C.c_int64 * MAX_BINS),
                ("bin_nnz_c", C.c_int64 * MAX_BINS)]

    def as_dict(self) -> dict:
        d = {k: getattr(self, k) for k in ("products", "max_row_products", "heavy_products", "nnz_c", "er", "avg_products", "sampled_cr",
                                           "cr_mean", "cr_std", "assist_cr", "symbolic_overflow_rows", "compacted_in_place", "b_sorted_copy", "dense_range_rows",
                                           "hll_registers", "sampled_rows", "fell_back", "overflow_rows", "temp_slots",
                                           "peak_bytes", "total_ms")}
        d["workflow"] = WORKFLOW_NAMES.get(self.workflow, str(self.workflow))
        d["rows_per_bin"] = list(self.rows_per_bin)
        d["symbolic_rows_per_bin"] = list(self.symbolic_rows_per_bin)
        for k in ("bin_ms", "bin_products", "bin_nnz_a", "bin_nnz_c"):
            d[k] = list(getattr(self, k))
        d["stage_ms"] = {n: float(self.stage_ms[i]) for i, n in enumerate(STAGES)}
        return d


class OceanError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ocean error {code}: {msg}")
        self.code = code


_lib = None


def load():
    """Load the HIP library; raises if it has not been built (python -m paper_2604_19004_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.lib_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with paper_2604_19004_amd.build.build() (no CPU fallback)")
    lib = C.CDLL(path)
    P = C.POINTER
    vp, i64, i32, dbl = C.c_void_p, C.c_int64, C.c_int32, C.c_double
    lib.ocean_default_options.argtypes = [P(ocean_options)]
    lib.ocean_default_options.restype = None
    lib.ocean_spgemm.argtypes = [P(ocean_csr), P(ocean_csr), P(ocean_csr), P(ocean_options), P(ocean_stats), vp]
    lib.ocean_csr_release.argtypes = [P(ocean_csr), P(ocean_allocator)]
    lib.ocean_row_products.argtypes = [P(ocean_csr), P(ocean_csr), vp, P(i64), P(i64), vp]
    lib.ocean_row_products_noalloc.argtypes = [P(ocean_csr), P(ocean_csr), vp, vp, vp]
    lib.ocean_init.argtypes = []
    lib.ocean_finalize.argtypes = []
    lib.ocean_finalize.restype = C.c_int
    lib.ocean_hll_sketch_rows.argtypes = [P(ocean_csr), i32, vp, vp]
    lib.ocean_hll_merge_estimate.argtypes = [P(ocean_csr), vp, i32, vp, i64, vp, vp, i64, vp, vp, vp]
    lib.ocean_symbolic.argtypes = [P(ocean_csr), P(ocean_csr), vp, P(ocean_options), P(ocean_stats), vp]
    lib.ocean_select_workflow.argtypes = [dbl, dbl, dbl, P(ocean_options)]
    lib.ocean_select_workflow.restype = i32
    lib.ocean_select_workflow_tuned.argtypes = [dbl, dbl, dbl, dbl, dbl, P(ocean_options)]
    lib.ocean_select_workflow_tuned.restype = i32
    lib.ocean_hll_register_count.argtypes = [dbl, P(ocean_options)]
    lib.ocean_hll_register_count.restype = i32
    lib.ocean_sample_size.argtypes = [i64, P(ocean_options)]
    lib.ocean_sample_size.restype = i64
    lib.ocean_sample_rows.argtypes = [i64, P(ocean_options), P(i64)]
    lib.ocean_bin_layout.argtypes = [P(i32), P(i32), P(i32), P(i32)]
    lib.ocean_last_error.restype = C.c_char_p
    lib.ocean_version.restype = C.c_int
    for name in ("ocean_spgemm", "ocean_csr_release", "ocean_row_products", "ocean_row_products_noalloc", "ocean_init",
                 "ocean_hll_sketch_rows",
                 "ocean_hll_merge_estimate", "ocean_symbolic", "ocean_sample_rows", "ocean_bin_layout"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise OceanError(rc, load().ocean_last_error().decode())


def default_options(**kw) -> ocean_options:
    o = ocean_options()
    load().ocean_default_options(C.byref(o))
    for k, v in kw.items():
        if not hasattr(o, k):
            raise TypeError(f"unknown option {k}")
        setattr(o, k, v)
    return o


# ---------------------------------------------------------------- host-only helpers
def select_workflow(avg_products: float, er: float, cr: float, opt: ocean_options | None = None) -> int:
    return int(load().ocean_select_workflow(avg_products, er, cr, C.byref(opt) if opt else None))


def select_workflow_tuned(avg_products: float, er: float, cr: float, products: float, heavy_products: float,
                          opt: ocean_options | None = None) -> int:
    return int(load().ocean_select_workflow_tuned(avg_products, er, cr, products, heavy_products,
                                                  C.byref(opt) if opt else None))


def hll_register_count(er: float, opt: ocean_options | None = None) -> int:
    return int(load().ocean_hll_register_count(er, C.byref(opt) if opt else None))


def sample_size(rows: int, opt: ocean_options | None = None) -> int:
    return int(load().ocean_sample_size(rows, C.byref(opt) if opt else None))


def sample_rows(rows: int, opt: ocean_options | None = None) -> np.ndarray:
    n = sample_size(rows, opt)
    out = np.zeros(n, dtype=np.int64)
    _check(load().ocean_sample_rows(rows, C.byref(opt) if opt else None, out.ctypes.data_as(C.POINTER(C.c_int64))))
    return out


def bin_layout():
    num = (C.c_int32 * MAX_BINS)()
    sym = (C.c_int32 * MAX_BINS)()
    nn, ns = C.c_int32(), C.c_int32()
    _check(load().ocean_bin_layout(num, C.byref(nn), sym, C.byref(ns)))
    return list(num)[:nn.value], list(sym)[:ns.value]


# ---------------------------------------------------------------- device side
def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: the Ocean SpGEMM path has no CPU fallback")
    return torch


@dataclass
class DeviceCSR:
    """CSR matrix in device memory, backed by torch tensors."""
    rows: int
    cols: int
    row_ptr: "object"   # torch int64 [rows+1]
    col_idx: "object"   # torch int32 [nnz]
    val: "object"       # torch float64 / float32 [nnz]
    _keep: list = field(default_factory=list, repr=False)

    @property
    def nnz(self) -> int:
        return int(self.col_idx.numel())

    def c_struct(self) -> ocean_csr:
        torch = _torch()
        dt = F64 if self.val.dtype == torch.float64 else F32
        return ocean_csr(self.rows, self.cols, self.nnz, self.row_ptr.data_ptr(),
                         self.col_idx.data_ptr() if self.nnz else None, self.val.data_ptr() if self.nnz else None, dt, 0)


def to_device(m, device="cuda:0") -> DeviceCSR:
    """workloads.CSR (numpy) -> DeviceCSR."""
    torch = _torch()
    return DeviceCSR(m.rows, m.cols, torch.from_numpy(m.row_ptr).to(device), torch.from_numpy(m.col_idx).to(device),
                     torch.from_numpy(m.val).to(device))


class TorchAllocator:
    """ocean_allocator whose memory comes from torch's caching allocator."""

    def __init__(self, device):
        torch = _torch()
        self.device = device
        self.blocks: dict[int, object] = {}

        def _alloc(_ctx, nbytes, out):
            try:
                t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device=self.device)
            except Exception:   # out of memory -> the library reports OCEAN_EALLOC
                return 1
            self.blocks[t.data_ptr()] = t
            out[0] = t.data_ptr()
            return 0

        def _release(_ctx, ptr):
            self.blocks.pop(int(ptr), None)

        self._alloc_cb = ALLOC_FN(_alloc)
        self._release_cb = RELEASE_FN(_release)
        self.struct = ocean_allocator(None, self._alloc_cb, self._release_cb)

    def take(self, ptr: int):
        """Detach the tensor behind a pointer the library handed to the caller."""
        return self.blocks.pop(int(ptr))


def _stream_ptr(stream) -> int:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def spgemm(A: DeviceCSR, B: DeviceCSR, opt: ocean_options | None = None, stream=None, **kw):
    """C = A*B.  Returns (DeviceCSR, stats dict).  Keyword arguments set ocean_options fields."""
    torch = _torch()
    lib = load()
    o = opt if opt is not None else default_options(**kw)
    alloc = TorchAllocator(A.row_ptr.device)
    o.allocator = C.pointer(alloc.struct)
    a, b, c, st = A.c_struct(), B.c_struct(), ocean_csr(), ocean_stats()
    with torch.cuda.device(A.row_ptr.device):
        rc = lib.ocean_spgemm(C.byref(a), C.byref(b), C.byref(c), C.byref(o), C.byref(st), _stream_ptr(stream))
    o.allocator = None
    _check(rc)
    vdt = torch.float64 if c.dtype == F64 else torch.float32
    vsz = 8 if c.dtype == F64 else 4
    rp = alloc.take(c.row_ptr)[: (c.rows + 1) * 8].view(torch.int64)
    if c.nnz > 0:
        col = alloc.take(c.col_idx)[: c.nnz * 4].view(torch.int32)
        val = alloc.take(c.val)[: c.nnz * vsz].view(vdt)
    else:
        if c.col_idx:
            alloc.take(c.col_idx)
        if c.val:
            alloc.take(c.val)
        col = torch.empty(0, dtype=torch.int32, device=rp.device)
        val = torch.empty(0, dtype=vdt, device=rp.device)
    assert not alloc.blocks, "library leaked allocator blocks"
    return DeviceCSR(c.rows, c.cols, rp, col, val), st.as_dict()


def row_products(A: DeviceCSR, B: DeviceCSR, stream=None):
    """(prod tensor int64 [rows], total, max_row)."""
    torch = _torch()
    prod = torch.empty(A.rows, dtype=torch.int64, device=A.row_ptr.device)
    tot, mx = C.c_int64(), C.c_int64()
    a, b = A.c_struct(), B.c_struct()
    with torch.cuda.device(A.row_ptr.device):
        _check(load().ocean_row_products(C.byref(a), C.byref(b), prod.data_ptr(), C.byref(tot), C.byref(mx),
                                         _stream_ptr(stream)))
    return prod, tot.value, mx.value


NOALLOC_MAX_ROWS = 1 << 20


def init():
    """Resolve the library's fixed scratch array on the current device ahead of the first no-alloc call."""
    _torch()
    _check(load().ocean_init())


def finalize():
    """Release the calling thread's pinned read-back buffer and timing events."""
    _check(load().ocean_finalize())


def row_products_noalloc(A: DeviceCSR, B: DeviceCSR, prod, totals, stream=None):
    """ocean_row_products_noalloc: prod (int64 [rows]) and totals (int64 [3]: P, largest row, flags) are
    device tensors of the caller; the call only enqueues work on the stream."""
    torch = _torch()
    a, b = A.c_struct(), B.c_struct()
    with torch.cuda.device(A.row_ptr.device):
        _check(load().ocean_row_products_noalloc(C.byref(a), C.byref(b), prod.data_ptr(), totals.data_ptr(),
                                                 _stream_ptr(stream)))


def hll_sketch_rows(B: DeviceCSR, m: int, stream=None):
    torch = _torch()
    out = torch.empty((B.rows, m), dtype=torch.uint8, device=B.row_ptr.device)
    b = B.c_struct()
    with torch.cuda.device(B.row_ptr.device):
        _check(load().ocean_hll_sketch_rows(C.byref(b), m, out.data_ptr(), _stream_ptr(stream)))
    return out


def hll_merge_estimate(A: DeviceCSR, sketches, m: int, rows=None, prod=None, B: DeviceCSR | None = None,
                       want_merged: bool = False, stream=None):
    """(est float64 [n_rows], merged uint8 [n_rows, m] or None)."""
    torch = _torch()
    dev = A.row_ptr.device
    n_rows = A.rows if rows is None else int(rows.numel())
    est = torch.empty(n_rows, dtype=torch.float64, device=dev)
    merged = torch.empty((n_rows, m), dtype=torch.uint8, device=dev) if want_merged else None
    a = A.c_struct()
    with torch.cuda.device(dev):
        _check(load().ocean_hll_merge_estimate(
            C.byref(a), sketches.data_ptr(), m, rows.data_ptr() if rows is not None else None, n_rows,
            prod.data_ptr() if prod is not None else None, B.row_ptr.data_ptr() if B is not None else None,
            B.cols if B is not None else 0, est.data_ptr(), merged.data_ptr() if want_merged else None,
            _stream_ptr(stream)))
    return est, merged


def symbolic(A: DeviceCSR, B: DeviceCSR, opt: ocean_options | None = None, stream=None):
    """Exact nnz per row of C (int32 tensor) and stats."""
    torch = _torch()
    out = torch.empty(A.rows, dtype=torch.int32, device=A.row_ptr.device)
    o = opt if opt is not None else default_options()
    alloc = TorchAllocator(A.row_ptr.device)
    o.allocator = C.pointer(alloc.struct)
    st = ocean_stats()
    a, b = A.c_struct(), B.c_struct()
    with torch.cuda.device(A.row_ptr.device):
        rc = load().ocean_symbolic(C.byref(a), C.byref(b), out.data_ptr(), C.byref(o), C.byref(st), _stream_ptr(stream))
    o.allocator = None
    _check(rc)
    return out, st.as_dict()
