"""Python face of libaxonn_linear.so: argument marshalling only.

Every function here has the name and the argument order of the C entry point it calls
(include/axonn_linear.h).  Tensors are torch bf16 CUDA tensors used purely as device memory;
no arithmetic happens in Python or in torch.  If the library has not been built the import
of a symbol fails loudly -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch  # noqa: F401  (imported before the library so both share one HIP runtime)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libaxonn_linear.so")

AXONN_NN, AXONN_NT, AXONN_TN = 0, 1, 2
LAYOUTS = {"NN": AXONN_NN, "NT": AXONN_NT, "TN": AXONN_TN}
AXONN_OK, AXONN_ERR_INVALID_ARG, AXONN_ERR_UNSUPPORTED, AXONN_ERR_LAUNCH, AXONN_ERR_WORKSPACE = 0, -1, -2, -3, -4

EXPORTS = (
    "axonn_linear_fwd", "axonn_linear_bwd_data", "axonn_linear_bwd_weight",
    "axonn_linear_gemm_static", "axonn_linear_static_scratch_bytes",
    "axonn_status_string", "axonn_linear_version", "axonn_linear_num_variants",
    "axonn_linear_variant_name", "axonn_linear_variant_supports", "axonn_linear_select_variant",
    "axonn_linear_plan", "axonn_linear_call_plan",
    "axonn_linear_force_variant",
    "axonn_linear_init", "axonn_linear_set_split_k", "axonn_linear_split_k_timeouts",
    "axonn_linear_workspace_bytes", "axonn_linear_set_workspace", "axonn_transpose_bf16",
    "axonn_linear_tune", "axonn_linear_tuned", "axonn_linear_tune_reset", "axonn_linear_tuned_set", "axonn_linear_tuned_call",
    "axonn_comm_group_bandwidths", "axonn_comm_layer_time", "axonn_comm_rank_grids",
)

_lib = None


class PlanPart(ctypes.Structure):
    """axonn_plan_part_t"""
    _fields_ = [("variant", ctypes.c_int), ("m", ctypes.c_int64), ("n", ctypes.c_int64),
                ("row0", ctypes.c_int64), ("col0", ctypes.c_int64)]


class TuneResult(ctypes.Structure):
    """axonn_tune_result_t"""
    _fields_ = [("best_layout", ctypes.c_int), ("best_layout_all_in", ctypes.c_int),
                ("gemm_us", ctypes.c_float * 3), ("restore_first_us", ctypes.c_float * 3),
                ("restore_second_us", ctypes.c_float * 3)]

    def as_dict(self):
        return dict(best_layout=self.best_layout, best_layout_all_in=self.best_layout_all_in,
                    gemm_us=list(self.gemm_us), restore_first_us=list(self.restore_first_us),
                    restore_second_us=list(self.restore_second_us))


OP_INDEX = {"fwd": 0, "bwd_data": 1, "bwd_weight": 2}


class CommLayer(ctypes.Structure):
    """axonn_comm_layer_t"""
    _fields_ = [("m", ctypes.c_int64), ("k", ctypes.c_int64), ("n", ctypes.c_int64), ("transposed", ctypes.c_int)]


class CommGrid(ctypes.Structure):
    """axonn_comm_grid_t"""
    _fields_ = [("gx", ctypes.c_int), ("gy", ctypes.c_int), ("gz", ctypes.c_int), ("gdata", ctypes.c_int),
                ("seconds", ctypes.c_double)]


class AxonnError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


def lib() -> ctypes.CDLL:
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2502_08145_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.axonn_linear_static_scratch_bytes.argtypes = []
        L.axonn_linear_static_scratch_bytes.restype = ctypes.c_size_t
        for name in ("axonn_linear_fwd", "axonn_linear_bwd_data", "axonn_linear_bwd_weight", "axonn_linear_gemm_static"):
            fn = getattr(L, name)
            fn.argtypes = [i64, i64, i64, ci, vp, vp, vp, ci, vp]
            fn.restype = ci
        L.axonn_status_string.argtypes = [ci]
        L.axonn_status_string.restype = ctypes.c_char_p
        L.axonn_linear_version.argtypes = []
        L.axonn_linear_version.restype = ci
        L.axonn_linear_num_variants.argtypes = []
        L.axonn_linear_num_variants.restype = ci
        L.axonn_linear_variant_name.argtypes = [ci]
        L.axonn_linear_variant_name.restype = ctypes.c_char_p
        L.axonn_linear_variant_supports.argtypes = [ci, i64, i64, i64, ci]
        L.axonn_linear_variant_supports.restype = ci
        L.axonn_linear_select_variant.argtypes = [i64, i64, i64, ci]
        L.axonn_linear_select_variant.restype = ci
        L.axonn_linear_plan.argtypes = [i64, i64, i64, ci, ctypes.POINTER(PlanPart)]
        L.axonn_linear_plan.restype = ci
        L.axonn_linear_call_plan.argtypes = [i64, i64, i64, ci, ctypes.POINTER(PlanPart)]
        L.axonn_linear_call_plan.restype = ci
        L.axonn_linear_force_variant.argtypes = [ci]
        L.axonn_linear_force_variant.restype = ci
        L.axonn_linear_workspace_bytes.argtypes = [i64, i64, i64, ci]
        L.axonn_linear_workspace_bytes.restype = ctypes.c_size_t
        L.axonn_linear_set_workspace.argtypes = [vp, ctypes.c_size_t]
        L.axonn_linear_set_workspace.restype = ci
        L.axonn_transpose_bf16.argtypes = [i64, i64, vp, vp, vp]
        L.axonn_transpose_bf16.restype = ci
        L.axonn_linear_tune.argtypes = [ci, i64, i64, i64, vp, vp, vp, vp, ctypes.c_size_t, vp,
                                        ctypes.POINTER(TuneResult)]
        L.axonn_linear_tune.restype = ci
        L.axonn_linear_tuned.argtypes = [ci, i64, i64, i64, ctypes.POINTER(TuneResult)]
        L.axonn_linear_tuned.restype = ci
        L.axonn_linear_tuned_set.argtypes = [ci, i64, i64, i64, ctypes.POINTER(TuneResult)]
        L.axonn_linear_tuned_set.restype = ci
        L.axonn_linear_tuned_call.argtypes = [ci, i64, i64, i64, vp, vp, vp, vp, vp, ctypes.c_size_t, ci, vp,
                                              ctypes.POINTER(ci)]
        L.axonn_linear_tuned_call.restype = ci
        L.axonn_linear_tune_reset.argtypes = []
        L.axonn_linear_tune_reset.restype = None
        dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)
        L.axonn_comm_group_bandwidths.argtypes = [ip, ci, ctypes.c_double, dp, dp]
        L.axonn_comm_group_bandwidths.restype = ci
        L.axonn_comm_layer_time.argtypes = [ctypes.POINTER(CommLayer), ip, dp, ctypes.c_double, dp]
        L.axonn_comm_layer_time.restype = ci
        L.axonn_comm_rank_grids.argtypes = [i64, ctypes.POINTER(CommLayer), ci, ci, ctypes.c_double, dp,
                                            ctypes.c_double, ctypes.POINTER(CommGrid), i64]
        L.axonn_comm_rank_grids.restype = i64
        L.axonn_linear_init.argtypes = []
        L.axonn_linear_init.restype = ci
        L.axonn_linear_set_split_k.argtypes = [ci]
        L.axonn_linear_set_split_k.restype = ci
        L.axonn_linear_split_k_timeouts.argtypes = [ctypes.POINTER(ctypes.c_uint64)]
        L.axonn_linear_split_k_timeouts.restype = ci
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().axonn_status_string(int(status)).decode()


def version() -> int:
    return lib().axonn_linear_version()


def num_variants() -> int:
    return lib().axonn_linear_num_variants()


def variant_name(v: int):
    s = lib().axonn_linear_variant_name(int(v))
    return s.decode() if s is not None else None


def variant_supports(v: int, M: int, N: int, K: int, layout) -> bool:
    return bool(lib().axonn_linear_variant_supports(int(v), M, N, K, _layout(layout)))


MAX_PLAN_PARTS = 4   # AXONN_MAX_PLAN_PARTS


def select_variant(M: int, N: int, K: int, layout) -> int:
    return lib().axonn_linear_select_variant(M, N, K, _layout(layout))


def plan(M: int, N: int, K: int, layout) -> list:
    """The launches behind one product: a list of dicts(variant, m, n, row0, col0), one to four."""
    parts = (PlanPart * MAX_PLAN_PARTS)()
    n = lib().axonn_linear_plan(M, N, K, _layout(layout), parts)
    if n < 0:
        raise AxonnError(n, "axonn_linear_plan")
    return [dict(variant=p.variant, m=p.m, n=p.n, row0=p.row0, col0=p.col0) for p in parts[:n]]


def call_plan(M: int, N: int, K: int, layout) -> list:
    """plan() for a call made now on the current device: without split-K if the registered scratch
    area is missing or too small for it."""
    parts = (PlanPart * MAX_PLAN_PARTS)()
    n = lib().axonn_linear_call_plan(M, N, K, _layout(layout), parts)
    if n < 0:
        raise AxonnError(n, "axonn_linear_call_plan")
    return [dict(variant=p.variant, m=p.m, n=p.n, row0=p.row0, col0=p.col0) for p in parts[:n]]


def plan_name(M: int, N: int, K: int, layout, now: bool = False) -> str:
    """Variant names of the launches of plan() (now=True: of call_plan()), joined by '+'."""
    return "+".join(variant_name(p["variant"]) for p in (call_plan if now else plan)(M, N, K, layout))


def force_variant(v: int) -> None:
    rc = lib().axonn_linear_force_variant(int(v))
    if rc != AXONN_OK:
        raise AxonnError(rc, "axonn_linear_force_variant")


def axonn_linear_init() -> None:
    """Set up the current device (kernel LDS limits) ahead of the first call."""
    rc = lib().axonn_linear_init()
    if rc != 0:
        raise AxonnError(rc, "axonn_linear_init")


def axonn_linear_workspace_bytes(M: int, N: int, K: int, layout) -> int:
    """Split-K scratch bytes the automatically chosen kernel needs for this problem (0: none)."""
    return int(lib().axonn_linear_workspace_bytes(M, N, K, _layout(layout)))


def axonn_linear_set_workspace(buf, check=True) -> int:
    """Register a device buffer (a torch tensor, kept alive by the caller) as the split-K scratch
    area of the current device; None unregisters it."""
    if buf is None:
        rc = lib().axonn_linear_set_workspace(None, 0)
    else:
        if not buf.is_cuda or not buf.is_contiguous():
            raise TypeError("expected a contiguous CUDA tensor")
        rc = lib().axonn_linear_set_workspace(buf.data_ptr(), buf.numel() * buf.element_size())
    if check and rc != 0:
        raise AxonnError(rc, "axonn_linear_set_workspace")
    return rc


WORKSPACE_ALL = 4096 + 256 * 256 * 256 * 4   # flags + 256 slots of one 256 x 256 fp32 tile: enough for every product

_workspace = {}   # device index -> the tensor registered by register_workspace (kept alive here)


def register_workspace(nbytes: int = WORKSPACE_ALL):
    """Allocate `nbytes` of device memory through torch on the current device and register it as that
    device's split-K scratch area (the library itself allocates nothing).  Returns the tensor; it is
    kept alive until unregister_workspace() or the end of the process."""
    dev = torch.cuda.current_device()
    buf = torch.empty((int(nbytes),), dtype=torch.uint8, device=f"cuda:{dev}")
    axonn_linear_set_workspace(buf)
    _workspace[dev] = buf
    return buf


def unregister_workspace() -> None:
    torch.cuda.synchronize()
    axonn_linear_set_workspace(None)
    _workspace.pop(torch.cuda.current_device(), None)


def axonn_linear_set_split_k(enable: bool) -> bool:
    """Allow or forbid the automatic choice of split-K kernels; returns the previous setting."""
    rc = lib().axonn_linear_set_split_k(1 if enable else 0)
    if rc < 0:
        raise AxonnError(rc, "axonn_linear_set_split_k")
    return bool(rc)


def axonn_linear_split_k_timeouts() -> int:
    """Number of split-K waits that were given up on the current device (0 in a healthy run)."""
    n = ctypes.c_uint64(0)
    rc = lib().axonn_linear_split_k_timeouts(ctypes.byref(n))
    if rc != 0:
        raise AxonnError(rc, "axonn_linear_split_k_timeouts")
    return int(n.value)


def _layout(layout) -> int:
    return LAYOUTS[layout] if isinstance(layout, str) else int(layout)


def _ptr(t) -> int:
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous():
        raise TypeError("expected a contiguous bf16 CUDA tensor")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _call(name, M, N, K, layout, a, b, c, fp32_accumulate, stream, check):
    rc = getattr(lib(), name)(int(M), int(N), int(K), _layout(layout), _ptr(a), _ptr(b), _ptr(c),
                              int(fp32_accumulate), _stream(stream))
    if check and rc != AXONN_OK:
        raise AxonnError(rc, name)
    return rc


def axonn_linear_fwd(M, N, K, layout, X, W, Y, fp32_accumulate=1, stream=None, check=True):
    """Y[M,N] = X * W (Algorithm 1 line 3); X, W stored as `layout` says; Y is written."""
    return _call("axonn_linear_fwd", M, N, K, layout, X, W, Y, fp32_accumulate, stream, check)


def axonn_linear_bwd_data(M, N, K, layout, dY, W, dX, fp32_accumulate=1, stream=None, check=True):
    """dX[M,N] = dY * W^T (Algorithm 1 line 11)."""
    return _call("axonn_linear_bwd_data", M, N, K, layout, dY, W, dX, fp32_accumulate, stream, check)


def axonn_linear_bwd_weight(M, N, K, layout, X, dY, dW, fp32_accumulate=1, stream=None, check=True):
    """dW[M,N] = X^T * dY (Algorithm 1 line 13)."""
    return _call("axonn_linear_bwd_weight", M, N, K, layout, X, dY, dW, fp32_accumulate, stream, check)


def axonn_linear_gemm_static(M, N, K, layout, first, second, out, fp32_accumulate=1, stream=None, check=True):
    """out[M,N] = the product, split-K through the library's static scratch array (no allocation anywhere)."""
    return _call("axonn_linear_gemm_static", M, N, K, layout, first, second, out, fp32_accumulate, stream, check)


def axonn_linear_static_scratch_bytes() -> int:
    return int(lib().axonn_linear_static_scratch_bytes())


def axonn_transpose_bf16(rows, cols, src, dst, stream=None, check=True):
    """dst[cols, rows] = transpose of src[rows, cols] (bf16 tensors or raw device addresses)."""
    rc = lib().axonn_transpose_bf16(rows, cols, _ptr(src), _ptr(dst), _stream(stream))
    if check and rc != 0:
        raise AxonnError(rc, "axonn_transpose_bf16")
    return rc


def axonn_linear_tune(op, M, N, K, first, second, out, scratch, stream=None, check=True):
    """Time the product `op` ("fwd", "bwd_data", "bwd_weight") in all three modes; returns a dict
    (see axonn_tune_result_t).  `scratch` is a CUDA tensor for the re-stored operands (or None)."""
    res = TuneResult()
    sp, sb = (0, 0) if scratch is None else (scratch.data_ptr(), scratch.numel() * scratch.element_size())
    rc = lib().axonn_linear_tune(OP_INDEX[op] if isinstance(op, str) else int(op), M, N, K, _ptr(first), _ptr(second),
                                 _ptr(out), sp, sb, _stream(stream), ctypes.byref(res))
    if check and rc != 0:
        raise AxonnError(rc, "axonn_linear_tune")
    return res.as_dict() if rc == 0 else rc


def axonn_linear_tuned(op, M, N, K):
    """The remembered tuning result for this product, or None."""
    res = TuneResult()
    rc = lib().axonn_linear_tuned(OP_INDEX[op] if isinstance(op, str) else int(op), M, N, K, ctypes.byref(res))
    if rc < 0:
        raise AxonnError(rc, "axonn_linear_tuned")
    return res.as_dict() if rc == 1 else None


def axonn_linear_tuned_set(op, M, N, K, best_layout_all_in, best_layout=None) -> None:
    """Remember a tuning result for this product (modes by name or number)."""
    res = TuneResult()
    res.best_layout_all_in = _layout(best_layout_all_in)
    res.best_layout = _layout(best_layout_all_in if best_layout is None else best_layout)
    rc = lib().axonn_linear_tuned_set(OP_INDEX[op] if isinstance(op, str) else int(op), M, N, K, ctypes.byref(res))
    if rc != 0:
        raise AxonnError(rc, "axonn_linear_tuned_set")


def axonn_linear_tuned_call(op, M, N, K, first, second, out, second_restored=None, scratch=None, fp32_accumulate=1,
                            stream=None, check=True):
    """Run the product in its tuned mode; returns the mode that ran (0 NN, 1 NT, 2 TN)."""
    used = ctypes.c_int(-1)
    sp, sb = (0, 0) if scratch is None else (scratch.data_ptr(), scratch.numel() * scratch.element_size())
    rc = lib().axonn_linear_tuned_call(OP_INDEX[op] if isinstance(op, str) else int(op), M, N, K, _ptr(first), _ptr(second),
                                       _ptr(out), _ptr(second_restored), sp, sb, int(fp32_accumulate), _stream(stream),
                                       ctypes.byref(used))
    if check and rc != 0:
        raise AxonnError(rc, "axonn_linear_tuned_call")
    return used.value if rc == 0 else rc


def axonn_linear_tune_reset() -> None:
    lib().axonn_linear_tune_reset()


def _intra_table(g_node, intra_db):
    """{(inner, size): bytes/s} -> the flat (g_node + 1)^2 table the C ABI takes."""
    tab = (ctypes.c_double * ((g_node + 1) * (g_node + 1)))()
    for (inner, size), bw in (intra_db or {}).items():
        if inner <= g_node and size <= g_node:
            tab[inner * (g_node + 1) + size] = float(bw)
    return tab


def axonn_comm_group_bandwidths(grid, g_node, beta_inter, intra_db):
    g = (ctypes.c_int * 4)(*grid)
    out = (ctypes.c_double * 4)()
    rc = lib().axonn_comm_group_bandwidths(g, g_node, float(beta_inter), _intra_table(g_node, intra_db), out)
    if rc != 0:
        raise AxonnError(rc, "axonn_comm_group_bandwidths")
    return tuple(out)


def axonn_comm_layer_time(m, k, n, grid, beta, bytes_per_element=2.0, transposed=False):
    layer = CommLayer(m, k, n, 1 if transposed else 0)
    g = (ctypes.c_int * 4)(*grid)
    b = (ctypes.c_double * 4)(*[float(x) for x in beta])
    out = (ctypes.c_double * 6)()
    rc = lib().axonn_comm_layer_time(ctypes.byref(layer), g, b, float(bytes_per_element), out)
    if rc != 0:
        raise AxonnError(rc, "axonn_comm_layer_time")
    return dict(zip(("ag_z", "rs_z", "ar_y", "ar_x", "ar_data", "total"), out))


def axonn_comm_rank_grids(g_total, layers, g_node, beta_inter, intra_db, bytes_per_element=2.0, top=None):
    """[(seconds, (G_x, G_y, G_z, G_data))], best first; layers = [(m, k, n, transposed)]."""
    arr = (CommLayer * max(1, len(layers)))(*[CommLayer(m, k, n, 1 if t else 0) for m, k, n, t in layers])
    tab = _intra_table(g_node, intra_db)
    count = lib().axonn_comm_rank_grids(g_total, arr, len(layers), g_node, float(beta_inter), tab,
                                        float(bytes_per_element), None, 0)
    if count < 0:
        raise AxonnError(int(count), "axonn_comm_rank_grids")
    n = count if top is None else min(top, count)
    out = (CommGrid * max(1, n))()
    rc = lib().axonn_comm_rank_grids(g_total, arr, len(layers), g_node, float(beta_inter), tab,
                                     float(bytes_per_element), out, n)
    if rc < 0:
        raise AxonnError(int(rc), "axonn_comm_rank_grids")
    return [(out[i].seconds, (out[i].gx, out[i].gy, out[i].gz, out[i].gdata)) for i in range(n)]


OPS = {"fwd": axonn_linear_fwd, "bwd_data": axonn_linear_bwd_data, "bwd_weight": axonn_linear_bwd_weight}
