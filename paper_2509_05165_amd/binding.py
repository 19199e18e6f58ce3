"""ctypes binding with the same names as the C ABI (include/kvc.h).

Device buffers are passed as integer addresses (e.g. ``tensor.data_ptr()``),
streams as the raw hipStream_t value (``torch.cuda.current_stream().cuda_stream``).
Nothing here computes anything: the functions build the C structs, call the
library and raise :class:`KvcError` on a non-zero status.  There is no
fallback: if libkvc.so is missing the import of :func:`lib` fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

KVC_F32, KVC_BF16 = 0, 1
KVC_AGG_MAX, KVC_AGG_MEAN = 0, 1
KVC_ORDER_RANK, KVC_ORDER_POSITION = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def lib_path() -> str:
    return os.path.join(_HERE, "libkvc.so")


class KvcError(RuntimeError):
    def __init__(self, status: int, where: str, message: str):
        self.status = status
        super().__init__(f"{where}: {message}")


class KvcParams(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("layers", C.c_int32), ("hq", C.c_int32), ("hkv", C.c_int32),
        ("head_dim", C.c_int32), ("window", C.c_int32), ("dtype", C.c_int32),
        ("agg_task", C.c_int32), ("agg_group", C.c_int32), ("agg_head", C.c_int32),
        ("add_head_mean", C.c_int32), ("softmax_scale", C.c_float),
        ("value_norm", C.c_int32), ("order", C.c_int32), ("min_per_layer", C.c_int32),
        ("unstructured", C.c_int32), ("causal_tail", C.c_int32),
        ("keep_first", C.c_int32), ("keep_last", C.c_int32),
    ]

    def __init__(self, batch, layers, hq, hkv, head_dim, window, dtype, agg_task=KVC_AGG_MAX,
                 agg_group=KVC_AGG_MEAN, agg_head=KVC_AGG_MEAN, add_head_mean=1,
                 softmax_scale=0.0, value_norm=0, order=KVC_ORDER_RANK, min_per_layer=0,
                 unstructured=0, causal_tail=0, keep_first=0, keep_last=0):
        super().__init__(batch, layers, hq, hkv, head_dim, window, dtype, agg_task, agg_group,
                         agg_head, add_head_mean, softmax_scale, value_norm, order,
                         min_per_layer, unstructured, causal_tail, keep_first, keep_last)


class _Inputs(C.Structure):
    _fields_ = [("q", C.POINTER(C.c_void_p)), ("k", C.POINTER(C.c_void_p)),
                ("v", C.POINTER(C.c_void_p)), ("cu_seqlens", C.POINTER(C.c_int64)),
                ("budget", C.POINTER(C.c_int64))]


class _Outputs(C.Structure):
    _fields_ = [("k_out", C.c_void_p), ("v_out", C.c_void_p), ("lengths", C.c_void_p),
                ("offsets", C.c_void_p), ("scores", C.c_void_p), ("idx", C.c_void_p),
                ("s_sorted", C.c_void_p), ("composite", C.c_void_p), ("tau", C.c_void_p)]


def lib() -> C.CDLL:
    """Load libkvc.so (built in-tree by paper_2509_05165_amd.build)."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} not found: build it with "
                              "`python -m paper_2509_05165_amd.build` (no fallback exists)")
        # PyTorch ships its own copy of the HIP runtime.  If libkvc.so were loaded
        # first it would pull in the system copy, and kernels launched through one
        # copy on memory allocated through the other fail with "no ROCm-capable
        # device is detected": make torch's copy the one this process uses.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(path)
        L.kvc_version.restype = C.c_int
        L.kvc_status_string.restype = C.c_char_p
        L.kvc_status_string.argtypes = [C.c_int]
        L.kvc_last_error.restype = C.c_char_p
        L.kvc_budget.restype = C.c_int64
        L.kvc_budget.argtypes = [C.c_int32, C.c_int32, C.c_int64]
        pp, vp, i64p = C.POINTER(KvcParams), C.c_void_p, C.POINTER(C.c_int64)
        ptab = C.POINTER(C.c_void_p)
        L.kvc_workspace_size.argtypes = [pp, C.c_int64, C.c_int64, C.POINTER(C.c_size_t)]
        L.kvc_score.argtypes = [pp, ptab, ptab, ptab, i64p, vp, vp, C.c_size_t, vp]
        L.kvc_head_rank.argtypes = [pp, vp, i64p, vp, vp, vp, C.c_size_t, vp]
        L.kvc_composite.argtypes = [pp, vp, i64p, vp, vp]
        L.kvc_global_select.argtypes = [pp, vp, i64p, i64p, vp, vp, vp, vp, C.c_size_t, vp]
        L.kvc_global_select_static.argtypes = [pp, vp, i64p, i64p, vp, vp, vp, vp]
        L.kvc_gather.argtypes = [pp, ptab, ptab, vp, vp, vp, i64p, C.c_int64, vp, vp, vp,
                                 C.c_size_t, vp]
        L.kvc_compress.argtypes = [pp, C.POINTER(_Inputs), C.POINTER(_Outputs), vp, C.c_size_t, vp]
        for name in ("kvc_workspace_size", "kvc_score", "kvc_head_rank", "kvc_composite",
                     "kvc_global_select", "kvc_global_select_static", "kvc_gather", "kvc_compress"):
            getattr(L, name).restype = C.c_int
        _LIB = L
    return _LIB


def _check(status: int, where: str):
    if status != 0:
        L = lib()
        name = L.kvc_status_string(status).decode()
        raise KvcError(status, where, f"{name}: {L.kvc_last_error().decode()}")


def _ptr_table(ptrs: Optional[Sequence[int]]):
    if ptrs is None:
        return None
    return (C.c_void_p * len(ptrs))(*[int(p) if p else None for p in ptrs])


def _i64(vals: Optional[Sequence[int]]):
    if vals is None:
        return None
    return (C.c_int64 * len(vals))(*[int(v) for v in vals])


def _vp(x) -> C.c_void_p:
    return C.c_void_p(int(x) if x else None)


def kvc_version() -> int:
    return lib().kvc_version()


def kvc_status_string(status: int) -> str:
    return lib().kvc_status_string(status).decode()


def kvc_last_error() -> str:
    return lib().kvc_last_error().decode()


def kvc_budget(keep_percent: int, layers: int, n: int) -> int:
    return lib().kvc_budget(keep_percent, layers, n)


def kvc_workspace_size(params: KvcParams, total_tokens: int, max_seqlen: int) -> int:
    out = C.c_size_t(0)
    _check(lib().kvc_workspace_size(C.byref(params) if params is not None else None,
                                    total_tokens, max_seqlen, C.byref(out)),
           "kvc_workspace_size")
    return out.value


def kvc_score(params, q, k, cu_seqlens, S, workspace, workspace_bytes, stream=0, v=None):
    _check(lib().kvc_score(C.byref(params), _ptr_table(q), _ptr_table(k), _ptr_table(v),
                           _i64(cu_seqlens), _vp(S), _vp(workspace), workspace_bytes,
                           _vp(stream)), "kvc_score")


def kvc_head_rank(params, S, cu_seqlens, idx, S_sorted, workspace, workspace_bytes, stream=0):
    _check(lib().kvc_head_rank(C.byref(params), _vp(S), _i64(cu_seqlens), _vp(idx),
                               _vp(S_sorted), _vp(workspace), workspace_bytes, _vp(stream)),
           "kvc_head_rank")


def kvc_composite(params, S_sorted, cu_seqlens, I, stream=0):
    _check(lib().kvc_composite(C.byref(params), _vp(S_sorted), _i64(cu_seqlens), _vp(I),
                               _vp(stream)), "kvc_composite")


def kvc_global_select(params, I, cu_seqlens, budget, tau, lengths, offsets, workspace,
                      workspace_bytes, stream=0):
    _check(lib().kvc_global_select(C.byref(params), _vp(I), _i64(cu_seqlens), _i64(budget),
                                   _vp(tau), _vp(lengths), _vp(offsets), _vp(workspace),
                                   workspace_bytes, _vp(stream)), "kvc_global_select")


def kvc_global_select_static(params, I, cu_seqlens, budget, tau, lengths, offsets, stream=0):
    _check(lib().kvc_global_select_static(C.byref(params), _vp(I), _i64(cu_seqlens),
                                          _i64(budget), _vp(tau), _vp(lengths), _vp(offsets),
                                          _vp(stream)), "kvc_global_select_static")


def kvc_gather(params, k, v, idx, lengths, offsets, cu_seqlens, total_budget, k_out, v_out,
               stream=0, workspace=0, workspace_bytes=0):
    _check(lib().kvc_gather(C.byref(params), _ptr_table(k), _ptr_table(v), _vp(idx),
                            _vp(lengths), _vp(offsets), _i64(cu_seqlens), total_budget,
                            _vp(k_out), _vp(v_out), _vp(workspace), workspace_bytes,
                            _vp(stream)), "kvc_gather")


def kvc_compress(params, q, k, v, cu_seqlens, budget, k_out, v_out, lengths, offsets,
                 workspace, workspace_bytes, stream=0, scores=0, idx=0, s_sorted=0, composite=0,
                 tau=0):
    tq, tk, tv = _ptr_table(q), _ptr_table(k), _ptr_table(v)
    cu, bd = _i64(cu_seqlens), _i64(budget)
    inp = _Inputs(C.cast(tq, C.POINTER(C.c_void_p)) if tq is not None else None,
                  C.cast(tk, C.POINTER(C.c_void_p)) if tk is not None else None,
                  C.cast(tv, C.POINTER(C.c_void_p)) if tv is not None else None,
                  C.cast(cu, C.POINTER(C.c_int64)) if cu is not None else None,
                  C.cast(bd, C.POINTER(C.c_int64)) if bd is not None else None)
    out = _Outputs(*[int(x) if x else None
                     for x in (k_out, v_out, lengths, offsets, scores, idx, s_sorted, composite,
                               tau)])
    _check(lib().kvc_compress(C.byref(params), C.byref(inp), C.byref(out), _vp(workspace),
                              workspace_bytes, _vp(stream)), "kvc_compress")


class _ProfileEntry(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int32), ("total_ms", C.c_float)]


def kvc_profile_enable(on: bool) -> None:
    lib().kvc_profile_enable.argtypes = [C.c_int]
    lib().kvc_profile_enable.restype = None
    lib().kvc_profile_enable(1 if on else 0)


def kvc_profile_collect(capacity: int = 64):
    """Returns {kernel name: (launches, total_ms)} for the launches since the
    last collect (HIP events recorded by the library on the launch stream)."""
    fn = lib().kvc_profile_collect
    fn.argtypes = [C.POINTER(_ProfileEntry), C.c_int]
    fn.restype = C.c_int
    buf = (_ProfileEntry * capacity)()
    n = fn(buf, capacity)
    if n < 0:
        raise KvcError(4, "kvc_profile_collect", "HIP event query failed")
    return {buf[i].name.decode(): (buf[i].launches, buf[i].total_ms) for i in range(min(n, capacity))}


def kvc_copy_probe(dst, src, nbytes: int, stream=0) -> None:
    fn = lib().kvc_copy_probe
    fn.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    fn.restype = C.c_int
    _check(fn(_vp(dst), _vp(src), nbytes, _vp(stream)), "kvc_copy_probe")


KVC_MFMA_PROBE_OPERAND_BYTES = 24 * 256 * 16
KVC_MFMA_PROBE_SINK_FLOATS = 512 * 256


def kvc_mfma_probe(operands, iterations: int, mode: int, sink, cycles=0, stream=0) -> float:
    """Enqueues the register-resident MFMA loop; returns the flops it issues."""
    fn = lib().kvc_mfma_probe
    fn.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                   C.POINTER(C.c_double), C.c_void_p]
    fn.restype = C.c_int
    flops = C.c_double(0.0)
    _check(fn(_vp(operands), iterations, mode, _vp(sink), _vp(cycles), C.byref(flops),
              _vp(stream)), "kvc_mfma_probe")
    return flops.value
