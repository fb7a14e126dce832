"""ctypes binding of libunisparse_hip.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see include/unisparse.h).
PyTorch supplies device memory (through the allocator callbacks of us_ctx) and the HIP
stream; every step of the computation runs inside the library's kernels.  There is no CPU
fallback: if the shared library is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libunisparse_hip.so")

US_OK = 0
STATUS_NAMES = {0: "US_OK", -1: "US_ERR_NULL", -2: "US_ERR_SHAPE", -3: "US_ERR_INDEX_RANGE",
                -4: "US_ERR_UNSUPPORTED_DESC", -5: "US_ERR_DUPLICATE", -6: "US_ERR_ALLOC",
                -7: "US_ERR_OVERFLOW", -8: "US_ERR_HIP", -9: "US_ERR_FORMAT_MISMATCH", -10: "US_ERR_SCRATCH_LIMIT"}
US_E_AFFINE, US_E_DIV, US_E_MOD, US_E_INDIRECT_ENUM, US_E_INDIRECT_SCHEDULE = 0, 1, 2, 3, 4
(US_F_COO, US_F_CSR, US_F_DCSR, US_F_CSC, US_F_DCSC, US_F_DIA, US_F_DIA_VARIANT, US_F_BCSR, US_F_ELL,
 US_F_BDIA, US_F_CSB, US_F_CISR_PLUS, US_F_BELL) = range(13)
US_P_SUM_GE_ABS, US_P_SUM_GE_FRAC_OF_CAPACITY, US_P_RANK_LT_ABS, US_P_RANK_LT_PERCENTILE = range(4)
US_A_SIZE, US_A_PTR, US_A_IDX, US_A_VAL = range(4)
US_T_NONE, US_T_INT32, US_T_FLOAT32 = range(3)
US_SORT_FINISH_AUTO, US_SORT_FINISH_LDS, US_SORT_FINISH_PASSES = range(3)
US_NOALLOC_SCRATCH_BYTES = 8 << 20

EXPORTS = ["us_convert", "us_convert_formatted", "us_decompose", "us_spmv", "us_spmv_noalloc", "us_spmm", "us_formatted_array",
           "us_formatted_info", "us_free", "us_free_async", "us_status_str", "us_desc_preset", "us_profile_create",
           "us_profile_destroy", "us_profile_reset", "us_profile_collect", "us_profile_entry", "us_profile_set_min_bytes"]


class UnisparseError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)}")
        self.status = status
        self.code = STATUS_NAMES.get(status, str(status))


_ALLOC_T = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
_FREE_T = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class us_ctx(C.Structure):
    _fields_ = [("alloc", _ALLOC_T), ("free", _FREE_T), ("user", C.c_void_p),
                ("hip_stream", C.c_void_p), ("profile", C.c_void_p), ("sort_finish", C.c_int32)]


class us_coo(C.Structure):
    _fields_ = [("nrows", C.c_int64), ("ncols", C.c_int64), ("nnz", C.c_int64),
                ("row", C.c_void_p), ("col", C.c_void_p), ("val", C.c_void_p)]


class us_expr(C.Structure):
    _fields_ = [("kind", C.c_int32), ("c0", C.c_int32), ("c1", C.c_int32), ("c", C.c_int32),
                ("factor", C.c_int32), ("factor2", C.c_int32)]


class us_format_desc(C.Structure):
    _fields_ = [("nlevels", C.c_int32), ("level", us_expr * 5), ("trim_s", C.c_int32),
                ("trim_e", C.c_int32), ("merge_mask", C.c_uint32), ("ell_width", C.c_int64)]


class us_predicate(C.Structure):
    _fields_ = [("group", us_expr * 2), ("ngroup", C.c_int32), ("kind", C.c_int32),
                ("num", C.c_int64), ("den", C.c_int64), ("abs", C.c_int64)]


_lib = None


def lib() -> C.CDLL:
    """Load the HIP library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2403_05802_amd.build` "
                              "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        L.us_status_str.restype = C.c_char_p
        L.us_status_str.argtypes = [C.c_int32]
        L.us_desc_preset.argtypes = [C.c_int32, C.c_int64, C.c_int64, C.POINTER(us_format_desc)]
        L.us_convert.argtypes = [C.POINTER(us_ctx), C.POINTER(us_coo), C.POINTER(us_format_desc),
                                 C.POINTER(C.c_void_p)]
        L.us_convert_formatted.argtypes = [C.POINTER(us_ctx), C.c_void_p, C.POINTER(us_format_desc),
                                           C.POINTER(C.c_void_p)]
        L.us_convert_formatted.restype = C.c_int32
        L.us_decompose.argtypes = [C.POINTER(us_ctx), C.POINTER(us_coo), C.POINTER(us_format_desc),
                                   C.POINTER(us_format_desc), C.POINTER(us_predicate),
                                   C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
        L.us_spmv.argtypes = [C.POINTER(us_ctx), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
        L.us_spmv_noalloc.argtypes = [C.POINTER(us_ctx), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
        L.us_spmm.argtypes = [C.POINTER(us_ctx), C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p,
                              C.c_int64, C.c_int32]
        L.us_formatted_array.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_void_p),
                                         C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        L.us_formatted_info.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                        C.POINTER(C.c_int64), C.POINTER(us_format_desc)]
        L.us_free.restype = None
        L.us_free.argtypes = [C.POINTER(us_ctx), C.c_void_p]
        L.us_free_async.restype = None
        L.us_free_async.argtypes = [C.POINTER(us_ctx), C.c_void_p]
        L.us_profile_create.argtypes = [C.POINTER(C.c_void_p)]
        L.us_profile_destroy.restype = None
        L.us_profile_destroy.argtypes = [C.c_void_p]
        L.us_profile_reset.argtypes = [C.c_void_p]
        L.us_profile_collect.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        L.us_profile_set_min_bytes.argtypes = [C.c_void_p, C.c_double]
        L.us_profile_set_min_bytes.restype = C.c_int32
        L.us_profile_entry.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_int64),
                                       C.POINTER(C.c_double), C.POINTER(C.c_double)]
        for fn in ("us_desc_preset", "us_convert", "us_decompose", "us_spmv", "us_spmv_noalloc", "us_spmm", "us_formatted_array",
                   "us_formatted_info", "us_profile_create", "us_profile_reset", "us_profile_collect",
                   "us_profile_entry"):
            getattr(L, fn).restype = C.c_int32
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != US_OK:
        raise UnisparseError(status, where)


# ----------------------------------------------------------------------------- context
class Context:
    """us_ctx whose allocator hands out torch CUDA(HIP) tensors and whose stream is torch's
    current stream at construction."""

    def __init__(self, device: str = "cuda:0", profile: bool = False):
        lib()
        self.device = torch.device(device)
        self._live: Dict[int, torch.Tensor] = {}
        self.fail_alloc_after: Optional[int] = None  # test hook: allocator returns NULL after n calls
        self._nalloc = 0

        def _alloc(nbytes, _user):
            self._nalloc += 1
            if self.fail_alloc_after is not None and self._nalloc > self.fail_alloc_after:
                return None
            try:
                t = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=self.device)
            except Exception:  # out of memory etc.: report NULL to the library
                return None
            self._live[t.data_ptr()] = t
            return t.data_ptr()

        def _free(ptr, _user):
            self._live.pop(ptr, None)

        self._alloc_cb = _ALLOC_T(_alloc)
        self._free_cb = _FREE_T(_free)
        self.c = us_ctx()
        self.c.alloc = self._alloc_cb
        self.c.free = self._free_cb
        self.c.user = None
        with torch.cuda.device(self.device):
            self.c.hip_stream = torch.cuda.current_stream().cuda_stream
        self.c.profile = None
        self.c.sort_finish = US_SORT_FINISH_AUTO
        self._profile = None
        if profile:
            self.enable_profile()

    def set_sort_lds_finish(self, mode) -> None:
        """us_ctx.sort_finish: True = finish the Sort inside LDS, False = whole-array digit passes only,
        None = chosen by the target tuple (the default)."""
        self.c.sort_finish = US_SORT_FINISH_AUTO if mode is None else (US_SORT_FINISH_LDS if mode else US_SORT_FINISH_PASSES)

    # -- profiling
    def enable_profile(self):
        if self._profile is None:
            p = C.c_void_p()
            _check(lib().us_profile_create(C.byref(p)), "us_profile_create")
            self._profile = p
        self.c.profile = self._profile

    def profile_min_bytes(self, min_bytes: float):
        _check(lib().us_profile_set_min_bytes(self._profile, float(min_bytes)), "us_profile_set_min_bytes")

    def disable_profile(self):
        self.c.profile = None

    def profile_reset(self):
        _check(lib().us_profile_reset(self._profile), "us_profile_reset")

    def profile_report(self) -> List[dict]:
        n = C.c_int32()
        _check(lib().us_profile_collect(self._profile, C.byref(n)), "us_profile_collect")
        out = []
        for i in range(n.value):
            name = C.c_char_p(); k = C.c_int64(); ms = C.c_double(); by = C.c_double()
            _check(lib().us_profile_entry(self._profile, i, C.byref(name), C.byref(k), C.byref(ms), C.byref(by)),
                   "us_profile_entry")
            if k.value:
                out.append({"kernel": name.value.decode(), "launches": k.value, "total_ms": ms.value,
                            "alg_bytes": by.value})
        return out

    def tensor_at(self, ptr: int, count: int, dtype: torch.dtype) -> torch.Tensor:
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        t = self._live.get(ptr)
        if t is None:   # an array inside a larger allocation (a result may keep its arrays in one block)
            for base, blk in self._live.items():
                if base <= ptr and ptr + nbytes <= base + blk.numel():
                    return blk[ptr - base:ptr - base + nbytes].view(dtype)
            raise KeyError(f"device pointer {ptr:#x} does not lie in a live allocation of this context")
        return t[:nbytes].view(dtype)

    def live_bytes(self) -> int:
        return sum(t.numel() for t in self._live.values())

    def __del__(self):
        try:
            if self._profile is not None:
                lib().us_profile_destroy(self._profile)
        except Exception:
            pass


# ----------------------------------------------------------------------------- descriptors
def us_desc_preset(fmt: int, b0: int = 0, b1: int = 0) -> us_format_desc:
    d = us_format_desc()
    _check(lib().us_desc_preset(fmt, b0, b1, C.byref(d)), "us_desc_preset")
    return d


def expr(kind: int, c0: int = 0, c1: int = 0, c: int = 0, factor: int = 1, factor2: int = 1) -> us_expr:
    return us_expr(kind, c0, c1, c, factor, factor2)


def make_desc(levels, trim, merge, ell_width: int = 0) -> us_format_desc:
    d = us_format_desc()
    d.nlevels = len(levels)
    for i, e in enumerate(levels):
        d.level[i] = e
    d.trim_s, d.trim_e = trim if trim is not None else (-1, -1)
    d.merge_mask = sum(1 << l for l in merge)
    d.ell_width = ell_width
    return d


def make_predicate(group, kind: int, num: int = 0, den: int = 1, abs_: int = 0) -> us_predicate:
    p = us_predicate()
    p.ngroup = len(group)
    for i, e in enumerate(group):
        p.group[i] = e
    p.kind, p.num, p.den, p.abs = kind, num, den, abs_
    return p


# ----------------------------------------------------------------------------- formatted tensor
class Formatted:
    def __init__(self, ctx: Context, handle: int):
        self.ctx = ctx
        self.handle = C.c_void_p(handle)
        self._info = None   # (nrows, ncols, nnz, desc), asked for on first use: a conversion loop never needs it

    def _get_info(self):
        if self._info is None:
            nr, nc, nz = C.c_int64(), C.c_int64(), C.c_int64()
            desc = us_format_desc()
            _check(lib().us_formatted_info(self.handle, C.byref(nr), C.byref(nc), C.byref(nz), C.byref(desc)),
                   "us_formatted_info")
            self._info = (nr.value, nc.value, nz.value, desc)
        return self._info

    nrows = property(lambda self: self._get_info()[0])
    ncols = property(lambda self: self._get_info()[1])
    nnz = property(lambda self: self._get_info()[2])
    desc = property(lambda self: self._get_info()[3])

    def us_formatted_array(self, level: int, which: int):
        """(device tensor or None, count).  US_A_SIZE returns (None, extent)."""
        p = C.c_void_p(); n = C.c_int64(); t = C.c_int32()
        _check(lib().us_formatted_array(self.handle, level, which, C.byref(p), C.byref(n), C.byref(t)), "us_formatted_array")
        if which == US_A_SIZE or n.value < 0:
            return None, n.value
        dt = {US_T_INT32: torch.int32, US_T_FLOAT32: torch.float32}[t.value]
        if n.value == 0:
            return torch.empty(0, dtype=dt, device=self.ctx.device), 0
        return self.ctx.tensor_at(p.value, n.value, dt), n.value

    def size(self, level): return self.us_formatted_array(level, US_A_SIZE)[1]
    def ptr(self, level): return self.us_formatted_array(level, US_A_PTR)[0]
    def idx(self, level): return self.us_formatted_array(level, US_A_IDX)[0]
    def val(self): return self.us_formatted_array(0, US_A_VAL)[0]

    def free(self, wait: bool = True):
        """wait=False: us_free_async, which does not wait for the stream.  The tensors behind this context come from
        torch's caching allocator, whose reuse of freed memory is ordered with the stream they were allocated on:
        safe as long as that is the context's stream (the current stream at its construction)."""
        if self.handle:
            (lib().us_free if wait else lib().us_free_async)(C.byref(self.ctx.c), self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _coo_struct(nrows, ncols, row, col, val) -> us_coo:
    assert row.dtype == torch.int32 and col.dtype == torch.int32 and val.dtype == torch.float32
    assert row.is_cuda and col.is_cuda and val.is_cuda
    assert row.is_contiguous() and col.is_contiguous() and val.is_contiguous()
    assert row.numel() == col.numel() == val.numel()
    return us_coo(nrows, ncols, row.numel(), row.data_ptr(), col.data_ptr(), val.data_ptr())


def us_convert(ctx: Context, nrows: int, ncols: int, row, col, val, desc: us_format_desc) -> Formatted:
    coo = _coo_struct(nrows, ncols, row, col, val)
    out = C.c_void_p()
    _check(lib().us_convert(C.byref(ctx.c), C.byref(coo), C.byref(desc), C.byref(out)), "us_convert")
    return Formatted(ctx, out.value)


def us_convert_formatted(ctx: Context, src: Formatted, desc: us_format_desc) -> Formatted:
    out = C.c_void_p()
    _check(lib().us_convert_formatted(C.byref(ctx.c), src.handle, C.byref(desc), C.byref(out)), "us_convert_formatted")
    return Formatted(ctx, out.value)


def us_decompose(ctx: Context, nrows: int, ncols: int, row, col, val, desc_a: us_format_desc,
                 desc_b: us_format_desc, pred: us_predicate) -> Tuple[Formatted, Formatted]:
    coo = _coo_struct(nrows, ncols, row, col, val)
    oa, ob = C.c_void_p(), C.c_void_p()
    _check(lib().us_decompose(C.byref(ctx.c), C.byref(coo), C.byref(desc_a), C.byref(desc_b), C.byref(pred),
                              C.byref(oa), C.byref(ob)), "us_decompose")
    return Formatted(ctx, oa.value), Formatted(ctx, ob.value)


def us_spmv(ctx: Context, A: Formatted, x: torch.Tensor, y: torch.Tensor, accumulate: bool = False) -> torch.Tensor:
    assert x.dtype == torch.float32 and y.dtype == torch.float32 and x.is_cuda and y.is_cuda
    assert x.is_contiguous() and y.is_contiguous() and x.numel() == A.ncols and y.numel() == A.nrows
    _check(lib().us_spmv(C.byref(ctx.c), A.handle, x.data_ptr(), y.data_ptr(), 1 if accumulate else 0), "us_spmv")
    return y


def us_spmv_noalloc(ctx: Context, A: Formatted, x: torch.Tensor, y: torch.Tensor, accumulate: bool = False) -> torch.Tensor:
    assert x.dtype == torch.float32 and y.dtype == torch.float32 and x.is_cuda and y.is_cuda
    assert x.is_contiguous() and y.is_contiguous() and x.numel() == A.ncols and y.numel() == A.nrows
    _check(lib().us_spmv_noalloc(C.byref(ctx.c), A.handle, x.data_ptr(), y.data_ptr(), 1 if accumulate else 0),
           "us_spmv_noalloc")
    return y


def us_spmm(ctx: Context, A: Formatted, X: torch.Tensor, Y: torch.Tensor, accumulate: bool = False) -> torch.Tensor:
    assert X.dtype == torch.float32 and Y.dtype == torch.float32 and X.is_cuda and Y.is_cuda
    assert X.dim() == 2 and Y.dim() == 2 and X.stride(1) == 1 and Y.stride(1) == 1
    assert X.shape[0] == A.ncols and Y.shape[0] == A.nrows and X.shape[1] == Y.shape[1]
    _check(lib().us_spmm(C.byref(ctx.c), A.handle, X.data_ptr(), X.shape[1], X.stride(0), Y.data_ptr(),
                         Y.stride(0), 1 if accumulate else 0), "us_spmm")
    return Y
