"""Python binding of libgp.so: the same calls as include/gp.h, argument
marshalling only.  Every step of the path runs inside the library's HIP
kernels / host C++; there is no Python or CPU fallback, and a missing library is
an error (build it with `python -m paper_2207_12000_amd.build`).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

GP_OK = 0
GP_ERR_INVALID_ARG, GP_ERR_INDEX_RANGE, GP_ERR_OVERFLOW = 1, 2, 3
GP_ERR_OOM_HOST, GP_ERR_OOM_DEVICE, GP_ERR_DEVICE, GP_ERR_UNSUPPORTED = 4, 5, 6, 7
GP_AGG_SYM, GP_AGG_MEAN, GP_AGG_SUM = 0, 1, 2
GP_F32, GP_BF16 = 0, 1
GP_SYMMETRISE, GP_ADD_SELF_LOOPS, GP_PLAN_ON_DEVICE = 1, 2, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgp.so")

# every symbol include/gp.h declares: (restype, argtypes)
_c = ctypes
_SIGNATURES = {
    "gp_plan_blocks": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int64, _c.c_int64, _c.c_uint32,
                                  _c.POINTER(_c.c_void_p)]),
    "gp_plan_destroy": (None, [_c.c_void_p]),
    "gp_plan_num_nodes": (_c.c_int64, [_c.c_void_p]),
    "gp_plan_nnz": (_c.c_int64, [_c.c_void_p]),
    "gp_plan_num_blocks": (_c.c_int32, [_c.c_void_p]),
    "gp_plan_block_offsets": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_block_row_lo": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_block_row_hi": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_rowptr": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_col": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_degree": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_dinv_sqrt": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_dinv": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_num_segments": (_c.c_int64, [_c.c_void_p]),
    "gp_plan_segments": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_segment_offsets": (_c.c_void_p, [_c.c_void_p]),
    "gp_plan_num_partial_rows": (_c.c_int64, [_c.c_void_p]),
    "gp_plan_segment_edges": (_c.c_int64, [_c.c_void_p]),
    "gp_plan_row_clusters": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.POINTER(_c.c_int32), _c.POINTER(_c.c_double),
                                        _c.POINTER(_c.c_double)]),
    "gp_plan_work_lists": (_c.c_int, [_c.c_void_p, _c.c_int32, _c.c_int, _c.c_int32, _c.POINTER(_c.c_int32),
                                      _c.POINTER(_c.c_int32), _c.c_void_p, _c.c_void_p, _c.c_int64]),
    "gp_plan_lds_schedule": (_c.c_int, [_c.c_void_p, _c.c_int32, _c.c_int32, _c.c_void_p]),
    "gp_propagate": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int32, _c.c_int, _c.c_int, _c.c_int32,
                                _c.c_void_p, _c.c_int64, _c.c_void_p]),
    "gp_plan_streamed_shape": (_c.c_int, [_c.c_void_p, _c.POINTER(_c.c_int64), _c.POINTER(_c.c_int64)]),
    "gp_propagate_noalloc": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int32, _c.c_int, _c.c_int, _c.c_int32,
                                        _c.c_void_p, _c.c_int64, _c.c_void_p]),
    "gp_noalloc_partial_row_bytes": (_c.c_int64, []),
    "gp_propagate_combine": (_c.c_int, [_c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_int32, _c.c_int, _c.c_int, _c.c_int32,
                                        _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p]),
    "gp_lc_forward": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int, _c.c_int64, _c.c_int32, _c.c_int32, _c.c_void_p, _c.c_int64,
                                 _c.c_void_p, _c.c_int32, _c.c_void_p, _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p]),
    "gp_lc_forward_branches": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int, _c.c_int64, _c.c_int32, _c.c_int32, _c.c_void_p,
                                          _c.c_int64, _c.c_void_p, _c.c_void_p, _c.c_int, _c.c_int32, _c.c_void_p,
                                          _c.c_void_p, _c.c_void_p, _c.c_int64, _c.c_void_p]),
    "gp_lc_softmax": (_c.c_int, [_c.c_void_p, _c.c_int64, _c.c_int32, _c.c_int64, _c.c_void_p]),
    "gp_solve_normalisation_blocks": (_c.c_int, [_c.c_double] * 7 + [_c.POINTER(_c.c_int64)]),
    "gp_solve_aggregation_blocks": (_c.c_int, [_c.c_double] * 5 + [_c.c_int64, _c.POINTER(_c.c_int64),
                                                                  _c.POINTER(_c.c_int64)]),
    "gp_set_hbm_budget_bytes": (_c.c_int, [_c.c_int64]),
    "gp_set_option": (_c.c_int, [_c.c_char_p, _c.c_int64]),
    "gp_get_option": (_c.c_int64, [_c.c_char_p]),
    "gp_profile_enable": (_c.c_int, [_c.c_int32]),
    "gp_profile_read": (_c.c_int, [_c.c_char_p, _c.POINTER(_c.c_int64), _c.POINTER(_c.c_double)]),
    "gp_status_string": (_c.c_char_p, [_c.c_int]),
    "gp_last_error": (_c.c_char_p, []),
}
EXPORTED_SYMBOLS = tuple(_SIGNATURES)

_lib = None


class GpError(RuntimeError):
    def __init__(self, status: int, where: str):
        l = lib()
        self.status = status
        self.status_name = l.gp_status_string(status).decode()
        super().__init__(f"{where}: {self.status_name}: {l.gp_last_error().decode()}")


def lib():
    """Loads libgp.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2207_12000_amd.build`")
        # PyTorch brings a HIP runtime of its own and loads it for the whole process.  Loaded after this
        # library's, the process holds two runtimes that each open the GPU, and calls through the second
        # fail ("no ROCm-capable device is detected"); loaded before, this library's calls resolve to the
        # runtime that is already there.  So PyTorch goes first wherever it is installed.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def _check(status: int, where: str):
    if status != GP_OK:
        raise GpError(status, where)


def _view(ptr, ctype, count, dtype):
    if not ptr or count == 0:
        return np.empty(0, dtype=dtype)
    return np.ctypeslib.as_array(ctypes.cast(ptr, ctypes.POINTER(ctype)), shape=(count,))


class Plan:
    """Owns a gp_plan*.  The array properties are views of library-owned host
    memory, valid until close()."""

    def __init__(self, handle: int):
        self._h = handle

    @property
    def handle(self) -> int:
        if not self._h:
            raise ValueError("plan is closed")
        return self._h

    def close(self):
        if self._h:
            lib().gp_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    @property
    def n(self) -> int:
        return lib().gp_plan_num_nodes(self.handle)

    @property
    def nnz(self) -> int:
        return lib().gp_plan_nnz(self.handle)

    @property
    def num_blocks(self) -> int:
        return lib().gp_plan_num_blocks(self.handle)

    @property
    def block_off(self):
        return _view(lib().gp_plan_block_offsets(self.handle), ctypes.c_int64, self.num_blocks + 1, np.int64)

    @property
    def block_row_lo(self):
        return _view(lib().gp_plan_block_row_lo(self.handle), ctypes.c_int32, self.num_blocks, np.int32)

    @property
    def block_row_hi(self):
        return _view(lib().gp_plan_block_row_hi(self.handle), ctypes.c_int32, self.num_blocks, np.int32)

    @property
    def rowptr(self):
        return _view(lib().gp_plan_rowptr(self.handle), ctypes.c_int64, self.n + 1, np.int64)

    @property
    def col(self):
        return _view(lib().gp_plan_col(self.handle), ctypes.c_int32, self.nnz, np.int32)

    @property
    def deg(self):
        return _view(lib().gp_plan_degree(self.handle), ctypes.c_int32, self.n, np.int32)

    @property
    def dinv_sqrt(self):
        return _view(lib().gp_plan_dinv_sqrt(self.handle), ctypes.c_float, self.n, np.float32)

    @property
    def dinv(self):
        return _view(lib().gp_plan_dinv(self.handle), ctypes.c_float, self.n, np.float32)


    SEGMENT_DTYPE = np.dtype([("start_lo", "<u4"), ("start_hi", "u1"), ("slice", "u1"), ("len", "<u2"),
                              ("row", "<i4"), ("slot", "<i4")])

    @property
    def segments(self):
        """Structured view of the schedule's 16-byte segment records."""
        cnt = lib().gp_plan_num_segments(self.handle)
        raw = _view(lib().gp_plan_segments(self.handle), ctypes.c_uint8, cnt * 16, np.uint8)
        return raw.view(self.SEGMENT_DTYPE)

    @property
    def segment_off(self):
        return _view(lib().gp_plan_segment_offsets(self.handle), ctypes.c_int64, self.num_blocks + 1, np.int64)

    @property
    def num_partial_rows(self) -> int:
        return lib().gp_plan_num_partial_rows(self.handle)

    @property
    def segment_edges(self) -> int:
        return lib().gp_plan_segment_edges(self.handle)

    def streamed_shape(self):
        """(edge blocks b, column blocks c) of the last streamed gp_propagate on this plan."""
        b, c = ctypes.c_int64(), ctypes.c_int64()
        _check(lib().gp_plan_streamed_shape(self.handle, ctypes.byref(b), ctypes.byref(c)), "gp_plan_streamed_shape")
        return b.value, c.value

    def row_clusters(self):
        """(label[n], num_clusters, inside_fraction, typical_rows) of the cache schedule."""
        label = np.empty(self.n, dtype=np.int32)
        num, inside, typical = ctypes.c_int32(), ctypes.c_double(), ctypes.c_double()
        _check(lib().gp_plan_row_clusters(self.handle, label.ctypes.data, ctypes.byref(num), ctypes.byref(inside),
                                          ctypes.byref(typical)), "gp_plan_row_clusters")
        return label, num.value, inside.value, typical.value

    def work_lists(self, d: int, dtype: int, vec: int):
        """(num_slices, slice_elems, xcd_off[9], records) of the explicit work lists for rows of
        d elements, or num_slices = 0 when the plan keeps the implicit lists."""
        S, elems = ctypes.c_int32(), ctypes.c_int32()
        off = np.zeros(9, dtype=np.int64)
        _check(lib().gp_plan_work_lists(self.handle, d, dtype, vec, ctypes.byref(S), ctypes.byref(elems), off.ctypes.data,
                                        None, 0), "gp_plan_work_lists")
        recs = np.zeros(int(off[8]), dtype=self.SEGMENT_DTYPE)
        if S.value:
            _check(lib().gp_plan_work_lists(self.handle, d, dtype, vec, ctypes.byref(S), ctypes.byref(elems),
                                            off.ctypes.data, recs.ctypes.data, recs.size), "gp_plan_work_lists")
        return S.value, elems.value, off, recs

    def lds_schedule(self, order: int = 0, d: int = 128):
        """The LDS pass's schedule (see gp_plan_lds_schedule in gp.h), or None where it does not
        apply: dict with hot_mode, conflict_free, group_set, group_id_off, group_steps (per
        group), rec_pos (64 per group), ids (uint16 places on the set's list), list_of_set,
        member_off, members, rest (segment records in position order), col (reordered)."""
        v = LdsView()
        _check(lib().gp_plan_lds_schedule(self.handle, d, order, ctypes.byref(v)), "gp_plan_lds_schedule")
        if v.num_groups == 0:
            return None
        G = v.num_groups
        out = {"group_set": np.zeros(G, np.int32), "group_id_off": np.zeros(G, np.int64), "group_steps": np.zeros(G, np.int32),
               "rec_pos": np.zeros(G * 64, np.int32), "ids": np.zeros(v.num_ids, np.uint16),
               "list_of_set": np.zeros(v.num_sets, np.int32), "member_off": np.zeros(v.num_lists + 1, np.int64),
               "members": np.zeros(v.num_members, np.int32), "rest": np.zeros(v.num_positions, self.SEGMENT_DTYPE),
               "col": np.zeros(self.nnz, np.int32)}
        v.group_capacity, v.id_capacity, v.member_capacity = G, v.num_ids, v.num_members
        v.set_capacity = max(v.num_sets, v.num_lists + 1)
        v.position_capacity = max(v.num_positions, self.nnz)
        for k, a in out.items():
            setattr(v, k, a.ctypes.data)
        _check(lib().gp_plan_lds_schedule(self.handle, d, order, ctypes.byref(v)), "gp_plan_lds_schedule")
        out["conflict_free"] = bool(v.conflict_free)
        out["hot_mode"] = int(v.hot_mode)
        return out


class LdsView(ctypes.Structure):
    """gp_lds_view of gp.h."""
    _fields_ = [("num_groups", ctypes.c_int64), ("num_ids", ctypes.c_int64), ("num_members", ctypes.c_int64),
                ("num_positions", ctypes.c_int64),
                ("num_sets", ctypes.c_int32), ("num_lists", ctypes.c_int32), ("conflict_free", ctypes.c_int32),
                ("hot_mode", ctypes.c_int32),
                ("group_capacity", ctypes.c_int64), ("id_capacity", ctypes.c_int64), ("set_capacity", ctypes.c_int64),
                ("member_capacity", ctypes.c_int64), ("position_capacity", ctypes.c_int64),
                ("group_set", ctypes.c_void_p), ("group_id_off", ctypes.c_void_p), ("group_steps", ctypes.c_void_p),
                ("rec_pos", ctypes.c_void_p), ("ids", ctypes.c_void_p),
                ("list_of_set", ctypes.c_void_p), ("member_off", ctypes.c_void_p), ("members", ctypes.c_void_p),
                ("rest", ctypes.c_void_p), ("col", ctypes.c_void_p)]


def gp_plan_blocks(src, dst, n: int, block_budget_edges: int, flags: int) -> Plan:
    """src/dst: int32 host arrays (numpy) of equal length."""
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    if src.shape != dst.shape or src.ndim != 1:
        raise ValueError("src and dst must be 1-D and equally long")
    out = ctypes.c_void_p()
    st = lib().gp_plan_blocks(src.ctypes.data if src.size else None, dst.ctypes.data if dst.size else None,
                              src.size, n, block_budget_edges, flags, ctypes.byref(out))
    _check(st, "gp_plan_blocks")
    return Plan(out.value)


def gp_propagate(plan: Plan, X_ptr: int, ldx: int, d: int, dtype: int, agg: int, K: int, out_ptr: int, ldo: int,
                 stream: Optional[int] = None):
    """Raw-pointer form: X_ptr / out_ptr are device (or pinned host) addresses."""
    st = lib().gp_propagate(plan.handle, X_ptr, ldx, d, dtype, agg, K, out_ptr, ldo, stream or None)
    _check(st, "gp_propagate")


def gp_propagate_noalloc(plan: Plan, X_ptr: int, ldx: int, d: int, dtype: int, agg: int, K: int, out_ptr: int, ldo: int,
                         stream: Optional[int] = None):
    """gp_propagate without any allocation (device operands, plan already on the device)."""
    st = lib().gp_propagate_noalloc(plan.handle, X_ptr, ldx, d, dtype, agg, K, out_ptr, ldo, stream or None)
    _check(st, "gp_propagate_noalloc")


def gp_noalloc_partial_row_bytes() -> int:
    return lib().gp_noalloc_partial_row_bytes()


def gp_propagate_combine(plan: Plan, X_ptr: int, ldx: int, d: int, dtype: int, agg: int, K: int, coeff, out_ptr: int,
                         ldo: int, stream: Optional[int] = None):
    """coeff: K+1 host floats.  X_ptr / out_ptr: device addresses."""
    c = np.ascontiguousarray(coeff, dtype=np.float32)
    if c.shape != (K + 1,):
        raise ValueError("coeff must hold K+1 values")
    st = lib().gp_propagate_combine(plan.handle, X_ptr, ldx, d, dtype, agg, K, c.ctypes.data, out_ptr, ldo, stream or None)
    _check(st, "gp_propagate_combine")


def propagate_tensors(plan: Plan, X, agg: int, K: int, out=None, stream=None):
    """Convenience for torch tensors (memory and streams only): X is an (n, d)
    float32 or bfloat16 tensor on the GPU (or pinned host memory); returns the
    (K+1, n, d) stack.  Enqueued on torch's current stream unless given."""
    import torch
    if X.dim() != 2 or X.stride(1) != 1:
        raise ValueError("X must be 2-D with unit column stride")
    n, d = X.shape
    if n != plan.n:
        raise ValueError("X has the wrong number of rows")
    dtype = {torch.float32: GP_F32, torch.bfloat16: GP_BF16}[X.dtype]
    if out is None:
        out = torch.empty((K + 1, n, d), dtype=X.dtype, device=X.device,
                          pin_memory=(X.device.type == "cpu"))
    if out.shape != (K + 1, n, d) or out.dtype != X.dtype or not out.is_contiguous():
        raise ValueError("out must be a contiguous (K+1, n, d) tensor of X's dtype")
    if stream is None and X.is_cuda:
        stream = torch.cuda.current_stream(X.device).cuda_stream
    gp_propagate(plan, X.data_ptr(), X.stride(0), d, dtype, agg, K, out.data_ptr(), d, stream)
    return out


def gp_lc_forward(stack_ptr: int, ld: int, dtype: int, n: int, d: int, K: int, batch_ptr: Optional[int], B: int, gamma,
                  weight_ptrs, widths, out_ptr: int, ldo: int, stream: Optional[int] = None):
    """Raw-pointer form.  gamma: K+1 host floats; weight_ptrs: T device addresses;
    widths: T output widths; batch_ptr: device address of B int32 row numbers or None."""
    g = np.ascontiguousarray(gamma, dtype=np.float32)
    if g.shape != (K + 1,):
        raise ValueError("gamma must hold K+1 values")
    T = len(weight_ptrs)
    if len(widths) != T:
        raise ValueError("one width per weight matrix")
    W = (ctypes.c_void_p * max(T, 1))(*[int(p) for p in weight_ptrs])
    wd = np.ascontiguousarray(widths, dtype=np.int32)
    st = lib().gp_lc_forward(stack_ptr, ld, dtype, n, d, K, batch_ptr or None, B, g.ctypes.data, T,
                             ctypes.cast(W, ctypes.c_void_p), wd.ctypes.data, out_ptr, ldo, stream or None)
    _check(st, "gp_lc_forward")


GP_COMB_SUM, GP_COMB_CONCAT, GP_COMB_MAX = 0, 1, 2


def gp_lc_softmax(H_ptr: int, B: int, C: int, ld: int, stream: Optional[int] = None):
    """Row softmax in place on a device matrix of B x C floats (rows ld floats apart)."""
    _check(lib().gp_lc_softmax(H_ptr or None, B, C, ld, stream or None), "gp_lc_softmax")


def gp_lc_forward_branches(stack_ptr: int, ld: int, dtype: int, n: int, d: int, K: int, batch_ptr: Optional[int], B: int,
                           gamma, depth, comb: int, weight_ptrs, widths, out_ptr: int, ldo: int,
                           stream: Optional[int] = None):
    """Raw-pointer form.  depth: K+1 host ints (layers branch k applies, 0 = hop left out);
    comb: GP_COMB_SUM / GP_COMB_CONCAT / GP_COMB_MAX; the rest as gp_lc_forward."""
    g = np.ascontiguousarray(gamma, dtype=np.float32)
    dp = np.ascontiguousarray(depth, dtype=np.int32)
    if g.shape != (K + 1,) or dp.shape != (K + 1,):
        raise ValueError("gamma and depth must hold K+1 values")
    T = len(weight_ptrs)
    if len(widths) != T:
        raise ValueError("one width per weight matrix")
    W = (ctypes.c_void_p * max(T, 1))(*[int(p) for p in weight_ptrs])
    wd = np.ascontiguousarray(widths, dtype=np.int32)
    st = lib().gp_lc_forward_branches(stack_ptr, ld, dtype, n, d, K, batch_ptr or None, B, g.ctypes.data, dp.ctypes.data, comb,
                                      T, ctypes.cast(W, ctypes.c_void_p), wd.ctypes.data, out_ptr, ldo, stream or None)
    _check(st, "gp_lc_forward_branches")


def lc_forward_tensors(stack, batch, gamma, weights, out=None, stream=None, depth=None, comb=GP_COMB_SUM):
    """Convenience for torch tensors (memory and streams only): stack is the
    contiguous (K+1, n, d) float32 / bfloat16 GPU tensor gp_propagate filled, batch an
    int32 GPU tensor of row numbers (or None for all rows), weights a list of
    contiguous float32 GPU matrices.  Returns the (B, width) float32 result.  With
    `depth` (K+1 ints) the branch form gp_lc_forward_branches is called."""
    import torch
    if stack.dim() != 3 or not stack.is_contiguous():
        raise ValueError("stack must be a contiguous (K+1, n, d) tensor")
    K1, n, d = stack.shape
    dtype = {torch.float32: GP_F32, torch.bfloat16: GP_BF16}[stack.dtype]
    if batch is not None and (batch.dtype != torch.int32 or batch.dim() != 1 or not batch.is_contiguous()):
        raise ValueError("batch must be a contiguous int32 vector")
    B = n if batch is None else batch.numel()
    inner = d
    for W in weights:
        if W.dtype != torch.float32 or W.dim() != 2 or not W.is_contiguous() or W.shape[0] != inner:
            raise ValueError("weights must be contiguous float32 matrices whose shapes chain from d")
        inner = W.shape[1]
    if depth is not None:
        ends = [weights[dk - 1].shape[1] for dk in depth if dk > 0]
        if not ends:
            raise ValueError("every hop is left out")
        inner = sum(ends) if comb == GP_COMB_CONCAT else ends[0]
    if out is None:
        out = torch.empty((B, inner), dtype=torch.float32, device=stack.device)
    if out.shape != (B, inner) or out.dtype != torch.float32 or out.stride(1) != 1:
        raise ValueError("out must be a (B, width) float32 tensor with unit column stride")
    if stream is None:
        stream = torch.cuda.current_stream(stack.device).cuda_stream
    bp = None if batch is None else batch.data_ptr()
    wp, ww = [W.data_ptr() for W in weights], [W.shape[1] for W in weights]
    if depth is None:
        gp_lc_forward(stack.data_ptr(), d, dtype, n, d, K1 - 1, bp, B, gamma, wp, ww, out.data_ptr(), out.stride(0), stream)
    else:
        gp_lc_forward_branches(stack.data_ptr(), d, dtype, n, d, K1 - 1, bp, B, gamma, depth, comb, wp, ww, out.data_ptr(),
                               out.stride(0), stream)
    return out


def gp_solve_normalisation_blocks(B_A, B_S, B_D, B_GPU, alpha_A=1.0, alpha_S=1.0, alpha_D=1.0) -> int:
    a = ctypes.c_int64()
    _check(lib().gp_solve_normalisation_blocks(B_A, B_S, B_D, B_GPU, alpha_A, alpha_S, alpha_D, ctypes.byref(a)),
           "gp_solve_normalisation_blocks")
    return a.value


def gp_solve_aggregation_blocks(B_S, B_X, B_GPU, beta_S=1.0, beta_X=1.0, max_c=1 << 20):
    b, c = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().gp_solve_aggregation_blocks(B_S, B_X, B_GPU, beta_S, beta_X, max_c, ctypes.byref(b), ctypes.byref(c)),
           "gp_solve_aggregation_blocks")
    return b.value, c.value


def gp_set_hbm_budget_bytes(nbytes: int):
    _check(lib().gp_set_hbm_budget_bytes(nbytes), "gp_set_hbm_budget_bytes")


def gp_set_option(name: str, value: int):
    _check(lib().gp_set_option(name.encode(), value), "gp_set_option")


def gp_get_option(name: str) -> int:
    return lib().gp_get_option(name.encode())


def gp_profile_enable(on: bool):
    _check(lib().gp_profile_enable(1 if on else 0), "gp_profile_enable")


def gp_profile_read(prefix: str = ""):
    n = ctypes.c_int64()
    ms = ctypes.c_double()
    _check(lib().gp_profile_read(prefix.encode(), ctypes.byref(n), ctypes.byref(ms)), "gp_profile_read")
    return n.value, ms.value


def gp_status_string(status: int) -> str:
    return lib().gp_status_string(status).decode()


def gp_last_error() -> str:
    return lib().gp_last_error().decode()
