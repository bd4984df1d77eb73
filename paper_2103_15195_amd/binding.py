"""Thin ctypes binding of libmergecomp.so (the C ABI in include/mergecomp.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch is used for device memory and streams; tensors are passed by
``data_ptr()``.  There is no CPU fallback: if the library has not been built the
import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MERGECOMP_LIB", os.path.join(_HERE, "libmergecomp.so"))   # override: a build to compare against

MC_ALGO_EFSIGN, MC_ALGO_TOPK, MC_ALGO_DGC, MC_ALGO_QSGD, MC_ALGO_TERNGRAD, MC_ALGO_FP16 = 1, 2, 3, 4, 5, 6
MC_ALGO_SIGNSGD, MC_ALGO_SIGNUM, MC_ALGO_ONEBIT, MC_ALGO_RANDK = 7, 8, 9, 10
ALGO_IDS = {"efsign": 1, "topk": 2, "dgc": 3, "qsgd": 4, "terngrad": 5, "fp16": 6,
            "signsgd": 7, "signum": 8, "onebit": 9, "randk": 10}
MC_PART_EVEN_COUNT, MC_PART_EVEN_ELEMS, MC_PART_USER = 0, 1, 2
MC_SELECT_ABOVE, MC_SELECT_FAST, MC_SELECT_REFILL, MC_SELECT_DENSE = 0, 1, 2, 3
MC_OK, MC_ERR_INVALID_ARG, MC_ERR_RANGE, MC_ERR_ALLOC, MC_ERR_DEVICE, MC_ERR_PAYLOAD = 0, -1, -2, -3, -4, -5

EXPORTS = [
    "mc_partition", "mc_partition_cost", "mc_partition_search", "mc_ctx_create", "mc_ctx_destroy", "mc_group_numel", "mc_group_k", "mc_group_tensors",
    "mc_payload_bytes", "mc_state_bytes", "mc_compress", "mc_compress_static", "mc_static_scratch_bytes", "mc_static_max_elems",
    "mc_decompress_sum", "mc_state_export_residual",
    "mc_state_import_residual", "mc_last_device_status", "mc_last_select_route", "mc_select_stats", "mc_set_barrier_spin_limit", "mc_compress_groups", "mc_decompress_sum_groups", "mc_profile_enable", "mc_profile_select", "mc_profile_reset",
    "mc_profile_kernels", "mc_profile_read", "mc_strerror", "mc_version",
]


class McConfig(C.Structure):
    _fields_ = [("algo", C.c_int32), ("use_ef", C.c_int32), ("ratio_ppm", C.c_uint32), ("qsgd_bits", C.c_int32),
                ("dgc_momentum", C.c_float), ("dgc_sample_ppm", C.c_uint32), ("seed", C.c_uint64)]


class McTimeModel(C.Structure):
    _fields_ = [("fwd_time", C.c_double), ("B_h", C.c_double), ("gamma_h", C.c_double), ("B_g", C.c_double),
                ("gamma_g", C.c_double)]


class McSelectCounts(C.Structure):
    _fields_ = [("calls", C.c_int64 * 4), ("last_bin_keys", C.c_int64), ("last_candidates", C.c_int64),
                ("margin_halvings", C.c_int64), ("margin_cap", C.c_int64)]


class McError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {lib().mc_strerror(status).decode()} ({status})")


_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(or paper_2103_15195_amd/build.py) first")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u32, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64
        L.mc_partition.argtypes = [vp, i32, i32, i32, vp, vp]
        L.mc_partition_cost.argtypes = [vp, vp, i32, C.POINTER(McTimeModel), vp, i32, C.POINTER(C.c_double)]
        L.mc_partition_search.argtypes = [vp, vp, i32, C.POINTER(McTimeModel), i32, C.c_double, vp, C.POINTER(i32),
                                          C.POINTER(C.c_double)]
        L.mc_ctx_create.argtypes = [C.POINTER(vp), C.POINTER(McConfig), vp, i32, vp, i32]
        L.mc_ctx_destroy.argtypes = [vp]
        for f in (L.mc_group_numel, L.mc_group_k):
            f.argtypes = [vp, i32]
            f.restype = i64
        L.mc_group_tensors.argtypes = [vp, i32]
        L.mc_group_tensors.restype = i32
        for f in (L.mc_payload_bytes, L.mc_state_bytes):
            f.argtypes = [vp, i32]
            f.restype = C.c_size_t
        L.mc_compress.argtypes = [vp, i32, u32, u64, vp, vp, vp, vp]
        L.mc_compress_static.argtypes = [vp, i32, u32, u64, vp, vp, vp, vp]
        L.mc_static_scratch_bytes.argtypes = []
        L.mc_static_scratch_bytes.restype = C.c_size_t
        L.mc_static_max_elems.argtypes = []
        L.mc_static_max_elems.restype = i64
        L.mc_decompress_sum.argtypes = [vp, i32, vp, i32, C.c_float, vp, vp]
        L.mc_state_export_residual.argtypes = [vp, i32, vp, vp, vp]
        L.mc_state_import_residual.argtypes = [vp, i32, vp, vp, vp]
        L.mc_last_device_status.argtypes = [vp]
        L.mc_last_select_route.argtypes = [vp]
        L.mc_select_stats.argtypes = [vp, C.POINTER(McSelectCounts), i32]
        L.mc_compress_groups.argtypes = [vp, C.c_uint32, C.c_uint64, vp, vp, vp, vp]
        L.mc_decompress_sum_groups.argtypes = [vp, vp, i32, C.c_float, vp, vp]
        L.mc_set_barrier_spin_limit.argtypes = [vp, C.c_uint32]
        L.mc_profile_enable.argtypes = [vp, i32]
        L.mc_profile_select.argtypes = [vp, u64]
        L.mc_profile_reset.argtypes = [vp]
        L.mc_profile_kernels.argtypes = []
        L.mc_profile_kernels.restype = i32
        L.mc_profile_read.argtypes = [vp, i32, C.POINTER(C.c_char_p), C.POINTER(i64), C.POINTER(C.c_double)]
        L.mc_strerror.argtypes = [C.c_int]
        L.mc_strerror.restype = C.c_char_p
        L.mc_version.restype = C.c_char_p
        _lib = L
    return _lib


def _check(status: int, what: str) -> None:
    if status != MC_OK:
        raise McError(status, what)


def ptr_array(tensors: Sequence) -> C.Array:
    """Host array of device addresses, one per tensor.  Callers in a hot loop build it once and pass it
    in place of the tensor list (the tensors must stay alive and in place)."""
    if isinstance(tensors, C.Array):
        return tensors
    return (C.c_void_p * max(len(tensors), 1))(*[t.data_ptr() if t is not None else None for t in tensors])


_ptr_array = ptr_array


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def mc_partition(numel: Sequence[int], y: int, policy: int = MC_PART_EVEN_ELEMS,
                 user_bounds: Optional[Sequence[int]] = None) -> List[int]:
    """Partition N tensors into y contiguous groups; host-only (needs no GPU)."""
    n = len(numel)
    nm = (C.c_int64 * max(n, 1))(*[int(x) for x in numel])
    ub = None if user_bounds is None else (C.c_int32 * len(user_bounds))(*[int(x) for x in user_bounds])
    out = (C.c_int32 * (max(y, 0) + 1))()
    _check(lib().mc_partition(nm, n, y, policy, ub, out), "mc_partition")
    return list(out)


def mc_partition_cost(numel: Sequence[int], bwd_time: Sequence[float], model: McTimeModel, bounds: Sequence[int]) -> float:
    """F(X_y) of the iteration-time model for a partition; host-only."""
    n = len(numel)
    nm = (C.c_int64 * max(n, 1))(*[int(x) for x in numel])
    bw = (C.c_double * max(n, 1))(*[float(x) for x in bwd_time])
    bd = (C.c_int32 * len(bounds))(*[int(b) for b in bounds])
    F = C.c_double()
    _check(lib().mc_partition_cost(nm, bw, n, C.byref(model), bd, len(bounds) - 1, C.byref(F)), "mc_partition_cost")
    return F.value


def mc_partition_search(numel: Sequence[int], bwd_time: Sequence[float], model: McTimeModel, Y: int, alpha: float):
    """The paper's partition search: returns (boundaries of the partition chosen, its F); host-only."""
    n = len(numel)
    nm = (C.c_int64 * max(n, 1))(*[int(x) for x in numel])
    bw = (C.c_double * max(n, 1))(*[float(x) for x in bwd_time])
    out = (C.c_int32 * (max(min(Y, n), 1) + 1))()
    y, F = C.c_int32(), C.c_double()
    _check(lib().mc_partition_search(nm, bw, n, C.byref(model), Y, alpha, out, C.byref(y), C.byref(F)), "mc_partition_search")
    return list(out)[:y.value + 1], F.value


class Context:
    """One (config, tensor list, partition) on the current device: wraps mc_ctx."""

    def __init__(self, algo, numel: Sequence[int], bounds: Sequence[int], *, use_ef: Optional[int] = None,
                 ratio_ppm: int = 10000, qsgd_bits: int = 8, dgc_momentum: float = 0.9, seed: int = 0,
                 dgc_sample_ppm: int = 0):
        algo = ALGO_IDS.get(algo, algo)
        if use_ef is None:                       # SignSGD remembers nothing; everything else defaults to error feedback
            use_ef = 0 if algo == MC_ALGO_SIGNSGD else 1
        self.algo = int(algo)
        self.numel = [int(x) for x in numel]
        self.bounds = [int(b) for b in bounds]
        self.y = len(self.bounds) - 1
        self.cfg = McConfig(self.algo, use_ef, ratio_ppm, qsgd_bits, dgc_momentum, dgc_sample_ppm, seed)
        nm = (C.c_int64 * max(len(self.numel), 1))(*self.numel)
        bd = (C.c_int32 * len(self.bounds))(*self.bounds)
        self._h = C.c_void_p()
        _check(lib().mc_ctx_create(C.byref(self._h), C.byref(self.cfg), nm, len(self.numel), bd, self.y), "mc_ctx_create")

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().mc_ctx_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # sizes -----------------------------------------------------------------
    def group_numel(self, group: int) -> int:
        return int(lib().mc_group_numel(self._h, group))

    def group_k(self, group: int) -> int:
        return int(lib().mc_group_k(self._h, group))

    def group_tensors(self, group: int) -> range:
        return range(self.bounds[group], self.bounds[group + 1])

    def payload_bytes(self, group: int) -> int:
        return int(lib().mc_payload_bytes(self._h, group))

    def state_bytes(self, group: int) -> int:
        return int(lib().mc_state_bytes(self._h, group))

    # the two hot calls --------------------------------------------------------
    def mc_compress(self, group: int, worker: int, it: int, grads: Sequence, state, payload, stream=None) -> None:
        _check(lib().mc_compress(self._h, group, worker, it, _ptr_array(grads),
                                 None if state is None else state.data_ptr(), payload.data_ptr(),
                                 _stream_handle(stream)), "mc_compress")

    def mc_compress_static(self, group: int, worker: int, it: int, grads: Sequence, state, payload, stream=None) -> None:
        """mc_compress with the reduction partials in the library's static device array (allocates nothing)."""
        _check(lib().mc_compress_static(self._h, group, worker, it, _ptr_array(grads),
                                        None if state is None else state.data_ptr(), payload.data_ptr(),
                                        _stream_handle(stream)), "mc_compress_static")

    def mc_decompress_sum(self, group: int, payloads: Sequence, alpha: float, outs: Sequence, stream=None) -> None:
        W = len(payloads)
        _check(lib().mc_decompress_sum(self._h, group, _ptr_array(payloads), W, alpha, _ptr_array(outs),
                                       _stream_handle(stream)), "mc_decompress_sum")

    # state helpers --------------------------------------------------------------
    def mc_compress_groups(self, worker: int, it: int, grads_all, states, payloads, stream=None) -> None:
        """All groups of one worker in one call; tensor sequences (or ptr_array()s of them): the model's gradients,
        one state and one payload per group."""
        _check(lib().mc_compress_groups(self._h, worker, it, ptr_array(grads_all), None if states is None else ptr_array(states),
                                        ptr_array(payloads), _stream_handle(stream)), "mc_compress_groups")

    def mc_decompress_sum_groups(self, payloads, W: int, alpha: float, outs_all, stream=None) -> None:
        """payloads: W * y entries, worker-major (payloads[w * y + j])."""
        _check(lib().mc_decompress_sum_groups(self._h, ptr_array(payloads), W, alpha, ptr_array(outs_all), _stream_handle(stream)),
               "mc_decompress_sum_groups")

    def mc_state_export_residual(self, group: int, state, e_out, stream=None) -> None:
        _check(lib().mc_state_export_residual(self._h, group, state.data_ptr(), e_out.data_ptr(),
                                              _stream_handle(stream)), "mc_state_export_residual")

    def mc_state_import_residual(self, group: int, e_in, state, stream=None) -> None:
        _check(lib().mc_state_import_residual(self._h, group, e_in.data_ptr(), state.data_ptr(),
                                              _stream_handle(stream)), "mc_state_import_residual")

    def mc_last_device_status(self) -> int:
        return int(lib().mc_last_device_status(self._h))

    def mc_last_select_route(self) -> int:
        r = int(lib().mc_last_select_route(self._h))
        if r < 0:
            raise McError(r, "mc_last_select_route")
        return r

    def mc_set_barrier_spin_limit(self, polls: int) -> None:
        _check(lib().mc_set_barrier_spin_limit(self._h, polls), "mc_set_barrier_spin_limit")

    def mc_select_stats(self, reset: bool = False) -> dict:
        c = McSelectCounts()
        _check(lib().mc_select_stats(self._h, C.byref(c), 1 if reset else 0), "mc_select_stats")
        return {"above": c.calls[0], "fast": c.calls[1], "refill": c.calls[2], "dense": c.calls[3],
                "last_bin_keys": c.last_bin_keys, "last_candidates": c.last_candidates,
                "margin_halvings": c.margin_halvings, "margin_cap": c.margin_cap}

    # profiling ------------------------------------------------------------------
    def profile_enable(self, on: bool, all_kernels: bool = False) -> None:
        if all_kernels:
            _check(lib().mc_profile_select(self._h, (1 << 64) - 1), "mc_profile_select")
        _check(lib().mc_profile_enable(self._h, 1 if on else 0), "mc_profile_enable")

    def profile_enable_only(self, kernel_name: str) -> None:
        """Time only the named kernel slot (keeps event overhead out of a timed region)."""
        for i in range(lib().mc_profile_kernels()):
            name = C.c_char_p()
            _check(lib().mc_profile_read(self._h, i, C.byref(name), None, None), "mc_profile_read")
            if name.value.decode() == kernel_name:
                _check(lib().mc_profile_select(self._h, 1 << i), "mc_profile_select")
                self.profile_enable(True)
                return
        raise KeyError(kernel_name)

    def profile_reset(self) -> None:
        _check(lib().mc_profile_reset(self._h), "mc_profile_reset")

    def profile_read(self) -> dict:
        out = {}
        for i in range(lib().mc_profile_kernels()):
            name, cnt, ms = C.c_char_p(), C.c_int64(), C.c_double()
            _check(lib().mc_profile_read(self._h, i, C.byref(name), C.byref(cnt), C.byref(ms)), "mc_profile_read")
            if cnt.value:
                out[name.value.decode()] = {"launches": cnt.value, "total_ms": ms.value}
        return out
