"""ctypes/numpy front end of the CPU oracle (mc_oracle.c).

TEST INFRASTRUCTURE: imported only by tests/, the smoke check and the
benchmark's cpu_baseline leg.  Nothing here touches the HIP library.

All functions work on ONE merged group given as a flat fp32 numpy vector (the
concatenation of the group's tensors, Section 4.1 of the paper).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mc_oracle.c")
_LIB = os.path.join(_HERE, "libmc_oracle.so")

EFSIGN, TOPK, DGC, QSGD, TERNGRAD, FP16, SIGNSGD, SIGNUM, ONEBIT, RANDK = 1, 2, 3, 4, 5, 6, 7, 8, 9, 10
ALGO_NAMES = {EFSIGN: "efsign", TOPK: "topk", DGC: "dgc", QSGD: "qsgd", TERNGRAD: "terngrad", FP16: "fp16",
              SIGNSGD: "signsgd", SIGNUM: "signum", ONEBIT: "onebit", RANDK: "randk"}
PART_EVEN_COUNT, PART_EVEN_ELEMS, PART_USER = 0, 1, 2
HDR = 128


def build(force: bool = False) -> str:
    """Compile the oracle with gcc: no contraction to FMA, no fast-math."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("algo", C.c_int32), ("use_ef", C.c_int32), ("ratio_ppm", C.c_uint32),
                ("qsgd_bits", C.c_int32), ("dgc_momentum", C.c_float), ("sample_ppm", C.c_uint32), ("seed", C.c_uint64)]


@dataclass
class Config:
    algo: int
    use_ef: int = 1
    ratio_ppm: int = 10000
    qsgd_bits: int = 8
    dgc_momentum: float = 0.9
    seed: int = 0
    dgc_sample_ppm: int = 0

    def c(self) -> _Cfg:
        return _Cfg(self.algo, self.use_ef, self.ratio_ppm, self.qsgd_bits, self.dgc_momentum, self.dgc_sample_ppm, self.seed)


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_philox4x32_10.restype = None
        L.orc_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64]
        L.orc_uniform.restype = C.c_float
        L.orc_randk_key.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64]
        L.orc_randk_key.restype = C.c_uint32
        L.orc_partition.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.orc_partition.restype = C.c_int
        L.orc_partition_cost.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(_TimeModel), C.c_void_p, C.c_int32,
                                         C.POINTER(C.c_double)]
        L.orc_partition_best.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(_TimeModel), C.c_int32, C.c_void_p,
                                         C.POINTER(C.c_double)]
        L.orc_partition_search.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(_TimeModel), C.c_int32, C.c_double,
                                           C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_double)]
        L.orc_topk_count.argtypes = [C.c_int64, C.c_uint32]
        L.orc_topk_count.restype = C.c_int64
        L.orc_sparse_capacity.argtypes = [C.POINTER(_Cfg), C.c_int64]
        L.orc_sparse_capacity.restype = C.c_int64
        L.orc_payload_bytes.argtypes = [C.POINTER(_Cfg), C.c_int64]
        L.orc_payload_bytes.restype = C.c_int64
        L.orc_state_floats.argtypes = [C.POINTER(_Cfg), C.c_int64]
        L.orc_state_floats.restype = C.c_int64
        L.orc_f32_to_f16.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.orc_f16_to_f32.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.orc_compress.argtypes = [C.POINTER(_Cfg), C.c_int64, C.c_uint64, C.c_uint32, C.c_uint64,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_compress.restype = C.c_int
        L.orc_decode.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        L.orc_decode.restype = C.c_int
        L.orc_decompress_sum.argtypes = [C.c_int64, C.c_void_p, C.c_int32, C.c_float, C.c_void_p]
        L.orc_decompress_sum.restype = C.c_int
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> np.ndarray:
    c = np.array(ctr, dtype=np.uint32)
    k = np.array(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def uniform(seed: int, worker: int, it: int, global_index: int) -> float:
    return float(lib().orc_uniform(seed, worker, it, global_index))


def randk_key(seed: int, worker: int, it: int, global_index: int) -> int:
    return int(lib().orc_randk_key(seed, worker, it, global_index))


def partition(numel: Sequence[int], y: int, policy: int = PART_EVEN_ELEMS,
              user_bounds: Optional[Sequence[int]] = None) -> np.ndarray:
    nm = np.ascontiguousarray(numel, dtype=np.int64)
    ub = None if user_bounds is None else np.ascontiguousarray(user_bounds, dtype=np.int32)
    out = np.zeros(max(y, 0) + 1, dtype=np.int32)
    rc = lib().orc_partition(_ptr(nm), len(nm), y, policy, _ptr(ub), _ptr(out))
    if rc:
        raise ValueError(f"orc_partition failed: {rc}")
    return out


class _TimeModel(C.Structure):
    _fields_ = [("fwd", C.c_double), ("B_h", C.c_double), ("gamma_h", C.c_double), ("B_g", C.c_double),
                ("gamma_g", C.c_double)]


@dataclass
class TimeModel:
    """Seconds: forward time, then h(x) = B_h + gamma_h x (compress) and g(x) = B_g + gamma_g x (send), x in elements."""
    fwd: float = 0.0
    B_h: float = 0.0
    gamma_h: float = 0.0
    B_g: float = 0.0
    gamma_g: float = 0.0

    def c(self) -> _TimeModel:
        return _TimeModel(self.fwd, self.B_h, self.gamma_h, self.B_g, self.gamma_g)


def partition_cost(numel: Sequence[int], bwd: Sequence[float], model: TimeModel, bounds: Sequence[int]) -> float:
    """F(X_y) of Section 4.3 for the partition given by its boundaries."""
    nm = np.ascontiguousarray(numel, dtype=np.int64)
    bw = np.ascontiguousarray(bwd, dtype=np.float64)
    bd = np.ascontiguousarray(bounds, dtype=np.int32)
    F = C.c_double()
    m = model.c()
    rc = lib().orc_partition_cost(_ptr(nm), _ptr(bw), len(nm), C.byref(m), _ptr(bd), len(bd) - 1, C.byref(F))
    if rc:
        raise ValueError(f"orc_partition_cost failed: {rc}")
    return F.value


def partition_best(numel: Sequence[int], bwd: Sequence[float], model: TimeModel, y: int) -> Tuple[np.ndarray, float]:
    """Brute force over all partitions into y groups: (boundaries, F_min(y))."""
    nm = np.ascontiguousarray(numel, dtype=np.int64)
    bw = np.ascontiguousarray(bwd, dtype=np.float64)
    out = np.zeros(y + 1, dtype=np.int32)
    F = C.c_double()
    m = model.c()
    rc = lib().orc_partition_best(_ptr(nm), _ptr(bw), len(nm), C.byref(m), y, _ptr(out), C.byref(F))
    if rc:
        raise ValueError(f"orc_partition_best failed: {rc}")
    return out, F.value


def partition_search(numel: Sequence[int], bwd: Sequence[float], model: TimeModel, Y: int,
                     alpha: float) -> Tuple[np.ndarray, float]:
    """Algorithm 2 with a brute-force inner minimisation: (boundaries of the partition returned, its F)."""
    nm = np.ascontiguousarray(numel, dtype=np.int64)
    bw = np.ascontiguousarray(bwd, dtype=np.float64)
    out = np.zeros(min(Y, len(nm)) + 1, dtype=np.int32)
    F, y = C.c_double(), C.c_int32()
    m = model.c()
    rc = lib().orc_partition_search(_ptr(nm), _ptr(bw), len(nm), C.byref(m), Y, alpha, _ptr(out), C.byref(y), C.byref(F))
    if rc:
        raise ValueError(f"orc_partition_search failed: {rc}")
    return out[:y.value + 1].copy(), F.value


def topk_count(n: int, ppm: int) -> int:
    return int(lib().orc_topk_count(n, ppm))


def sparse_capacity(cfg: Config, n: int) -> int:
    c = cfg.c()
    return int(lib().orc_sparse_capacity(C.byref(c), n))


def payload_bytes(cfg: Config, n: int) -> int:
    c = cfg.c()
    return int(lib().orc_payload_bytes(C.byref(c), n))


def state_floats(cfg: Config, n: int) -> int:
    c = cfg.c()
    return int(lib().orc_state_floats(C.byref(c), n))


def new_state(cfg: Config, n: int) -> np.ndarray:
    return np.zeros(state_floats(cfg, n), dtype=np.float32)


def compress(cfg: Config, g: np.ndarray, state: Optional[np.ndarray], *, group_off: int = 0, worker: int = 0,
             it: int = 0, scale_in=None) -> Tuple[np.ndarray, float]:
    """Returns (payload bytes, group scalar computed by the oracle); state is updated in place.
    OneBit has two group scalars: scale_in is then a pair, and the second one computed is header()["scale2"]."""
    g = np.ascontiguousarray(g, dtype=np.float32)
    n = g.size
    if state is not None:
        assert state.dtype == np.float32 and state.flags.c_contiguous and state.size == state_floats(cfg, n)
    payload = np.zeros(payload_bytes(cfg, n), dtype=np.uint8)
    c = cfg.c()
    sin = None if scale_in is None else np.atleast_1d(np.asarray(scale_in, dtype=np.float32)).copy()
    if sin is not None:
        assert sin.size == (2 if cfg.algo == ONEBIT else 1)
    sout = np.zeros(2, dtype=np.float32)
    rc = lib().orc_compress(C.byref(c), n, group_off, worker, it, _ptr(g), _ptr(state), _ptr(payload),
                            _ptr(sin), _ptr(sout))
    if rc:
        raise ValueError(f"orc_compress failed: {rc}")
    return payload, float(sout[0])


def decode(payload: np.ndarray, n: int) -> np.ndarray:
    d = np.zeros(n, dtype=np.float32)
    rc = lib().orc_decode(_ptr(payload), n, _ptr(d))
    if rc:
        raise ValueError(f"orc_decode failed: {rc}")
    return d


def decompress_sum(payloads: List[np.ndarray], n: int, alpha: float = 1.0) -> np.ndarray:
    arr = (C.c_void_p * len(payloads))(*[p.ctypes.data for p in payloads])
    out = np.zeros(n, dtype=np.float32)
    rc = lib().orc_decompress_sum(n, arr, len(payloads), alpha, _ptr(out))
    if rc:
        raise ValueError(f"orc_decompress_sum failed: {rc}")
    return out


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    h = np.zeros(x.size, dtype=np.uint16)
    lib().orc_f32_to_f16(_ptr(x), _ptr(h), x.size)
    return h


def f16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16)
    x = np.zeros(h.size, dtype=np.float32)
    lib().orc_f16_to_f32(_ptr(h), _ptr(x), h.size)
    return x


# ---- payload views (layout: 128-byte header, then the body) -----------------
def header(payload: np.ndarray) -> dict:
    b = payload[:HDR].tobytes()
    return {
        "magic": int(np.frombuffer(b, np.uint32, 1, 0)[0]),
        "algo": int(np.frombuffer(b, np.uint32, 1, 4)[0]),
        "n": int(np.frombuffer(b, np.uint64, 1, 8)[0]),
        "k": int(np.frombuffer(b, np.uint64, 1, 16)[0]),
        "scale": float(np.frombuffer(b, np.float32, 1, 24)[0]),
        "levels": int(np.frombuffer(b, np.uint32, 1, 28)[0]),
        "scale2": float(np.frombuffer(b, np.float32, 1, 32)[0]),       # OneBit: mean of the negative class
    }


DIR_SPAN = 4096


def sparse_directory(payload: np.ndarray) -> np.ndarray:
    """The directory that ends a sparse payload: entry t = kept entries with index below t * DIR_SPAN."""
    h = header(payload)
    cap = h["levels"] or h["k"]
    spans = (h["n"] + DIR_SPAN - 1) // DIR_SPAN
    return payload[HDR + 8 * cap:HDR + 8 * cap + (4 * (spans + 1) if h["n"] else 0)].view(np.uint32)


def with_directory(algo: int, n: int, idx: np.ndarray, val: np.ndarray) -> np.ndarray:
    """A sparse payload (exact-k layout) built from an ascending index list and its values: header, lists, directory."""
    k = int(idx.size)
    spans = (n + DIR_SPAN - 1) // DIR_SPAN
    assert n > 0
    pay = np.zeros(HDR + 8 * k + 4 * (spans + 1), np.uint8)
    pay[0:4] = np.frombuffer(np.uint32(0x3150434D).tobytes(), np.uint8)
    pay[4:8] = np.frombuffer(np.uint32(algo).tobytes(), np.uint8)
    pay[8:16] = np.frombuffer(np.uint64(n).tobytes(), np.uint8)
    pay[16:24] = np.frombuffer(np.uint64(k).tobytes(), np.uint8)
    pay[HDR:HDR + 4 * k] = np.ascontiguousarray(idx, np.uint32).view(np.uint8)
    pay[HDR + 4 * k:HDR + 8 * k] = np.ascontiguousarray(val, np.float32).view(np.uint8)
    pay[HDR + 8 * k:] = np.searchsorted(idx, np.arange(spans + 1, dtype=np.int64) * DIR_SPAN, side="left").astype(np.uint32).view(np.uint8)
    return pay


def sparse_view(payload: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(indices, values) of the kept entries; a payload with a capacity (sampled DGC) holds k <= capacity of them."""
    h = header(payload)
    k, cap = h["k"], h["levels"] or h["k"]
    idx = payload[HDR:HDR + 4 * k].view(np.uint32)
    val = payload[HDR + 4 * cap:HDR + 4 * cap + 4 * k].view(np.float32)
    return idx, val
