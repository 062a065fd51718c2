"""ctypes front end of ``liec_oracle.c``.  TEST INFRASTRUCTURE, NOT THE PRODUCT.

Argument marshalling only: every number comes from the C file, which states
Algorithm 1 (compressed iteration) and Definitions 2 and 4 of the paper as
plain single-threaded loops.  Arrays are numpy float32, C-contiguous.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

IDENTITY, SIGN, TOPK, BLOCKSIGN, RANDK = 0, 1, 2, 3, 4
_NAMES = {"identity": IDENTITY, "sign": SIGN, "topk": TOPK, "blocksign": BLOCKSIGN, "randk": RANDK}

_HERE = os.path.dirname(os.path.abspath(__file__))
# LIEC_ORACLE_SRC / LIEC_ORACLE_LIB point the wrapper at another copy of the C file (the mutation test
# checks that the pins reject copies with a planted mistake); unset, the file next to this one is used.
_SRC = os.environ.get("LIEC_ORACLE_SRC") or os.path.join(_HERE, "liec_oracle.c")
_LIB = os.environ.get("LIEC_ORACLE_LIB") or os.path.join(_HERE, "libliec_oracle.so")
_lib = None


class _CDesc(ctypes.Structure):
    _fields_ = [
        ("scale", ctypes.c_float),
        ("l1", ctypes.c_double),
        ("tau_key", ctypes.c_uint32),
        ("cutoff", ctypes.c_int64),
        ("count_above", ctypes.c_int64),
    ]


@dataclass
class Desc:
    """Non-elementwise part of a compressed message."""

    scale: float = 0.0
    l1: float = 0.0
    tau_key: int = 0
    cutoff: int = 0
    count_above: int = 0


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_LIB_OMP = os.path.splitext(_LIB)[0] + "_omp.so"     # beside whichever build LIEC_ORACLE_LIB names


def build_all_cores(force: bool = False) -> str:
    """The same source with -fopenmp: the independent workers of a step run on several host threads.
    Used only for the bench's labelled "all host cores" timing and by the test that checks its output
    bit for bit against the plain build."""
    if force or not os.path.exists(_LIB_OMP) or os.path.getmtime(_LIB_OMP) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB_OMP, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB_OMP


def step_all_cores(g: np.ndarray, x: np.ndarray, e: np.ndarray, worker_comp, server_comp, lr: float,
                   worker_k: int = 0, server_k: int = 0, rng: Tuple[int, int] = (0, 0)) -> int:
    """`step` through the -fopenmp build; returns the number of threads it may use."""
    global _lib_omp
    if _lib_omp is None:
        build_all_cores()
        _lib_omp = ctypes.CDLL(_LIB_OMP)
        _lib_omp.liec_oracle_threads.restype = ctypes.c_int
    g, x, e = _f32(g), _f32(x, True), _f32(e, True)
    N, d = g.shape
    assert x.shape == (N, d) and e.shape == (d,)
    fn = _lib_omp.liec_oracle_step_rng
    fn.restype = ctypes.c_int
    rc = fn(ctypes.c_int32(N), ctypes.c_int64(d), ctypes.c_int(_comp(worker_comp)), ctypes.c_int64(int(worker_k)),
            ctypes.c_int(_comp(server_comp)), ctypes.c_int64(int(server_k)), ctypes.c_float(lr), _ptr(g), _ptr(x),
            _ptr(e), None, ctypes.c_int32(0), ctypes.c_uint64(int(rng[0])), ctypes.c_uint64(int(rng[1])),
            None, None, None, None, None, None, None)
    if rc != 0:
        raise ValueError(f"liec_oracle_step_rng (all cores) failed with code {rc}")
    return int(_lib_omp.liec_oracle_threads())


_lib_omp = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(_CDesc)
        lib.liec_oracle_compress.restype = ctypes.c_int
        lib.liec_oracle_compress.argtypes = [ctypes.c_int, fp, ctypes.c_int64, ctypes.c_int64, fp, dp]
        lib.liec_oracle_server_average.restype = None
        lib.liec_oracle_server_average.argtypes = [fp, ctypes.c_int32, ctypes.c_int64, fp, fp]
        lib.liec_oracle_error_update.restype = None
        lib.liec_oracle_error_update.argtypes = [fp, fp, ctypes.c_int64, fp]
        lib.liec_oracle_worker_update.restype = None
        lib.liec_oracle_worker_update.argtypes = [fp, fp, fp, ctypes.c_int64, ctypes.c_float, fp]
        lib.liec_oracle_step.restype = ctypes.c_int
        lib.liec_oracle_step.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
                                         ctypes.c_int, ctypes.c_int64, ctypes.c_float, fp, fp, fp,
                                         dp, dp, fp, fp, fp]
        ip = ctypes.POINTER(ctypes.c_int64)
        lib.liec_oracle_compress_ex.restype = ctypes.c_int
        lib.liec_oracle_compress_ex.argtypes = [ctypes.c_int, fp, ctypes.c_int64, ctypes.c_int64, ip, ctypes.c_int32,
                                                fp, dp, fp]
        lib.liec_oracle_step_ex.restype = ctypes.c_int
        lib.liec_oracle_step_ex.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
                                            ctypes.c_int, ctypes.c_int64, ctypes.c_float, fp, fp, fp, ip,
                                            ctypes.c_int32, dp, dp, fp, fp, fp, fp, fp]
        u8p = ctypes.POINTER(ctypes.c_uint8)
        lib.liec_oracle_pack_sign.restype = None
        lib.liec_oracle_pack_sign.argtypes = [fp, ctypes.c_int64, u8p]
        lib.liec_oracle_unpack_sign.restype = None
        lib.liec_oracle_unpack_sign.argtypes = [u8p, ctypes.c_int64, fp, ip, ctypes.c_int32, fp]
        u32p = ctypes.POINTER(ctypes.c_uint32)
        lib.liec_oracle_pack_topk.restype = ctypes.c_int
        lib.liec_oracle_pack_topk.argtypes = [fp, ctypes.c_int64, ctypes.c_int64, u32p, fp]
        lib.liec_oracle_unpack_topk.restype = None
        lib.liec_oracle_unpack_topk.argtypes = [u32p, fp, ctypes.c_int64, ctypes.c_int64, fp]
        lib.liec_oracle_step_sync.restype = ctypes.c_int
        lib.liec_oracle_step_sync.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_float, fp, fp, fp, fp]
        u64, u32 = ctypes.c_uint64, ctypes.c_uint32
        lib.liec_oracle_randk_stream.restype = u64
        lib.liec_oracle_randk_stream.argtypes = [u64, u64, u32]
        lib.liec_oracle_randk_priority.restype = u32
        lib.liec_oracle_randk_priority.argtypes = [u64, u32]
        lib.liec_oracle_randk_priorities.restype = None
        lib.liec_oracle_randk_priorities.argtypes = [u64, u64, u32, ctypes.c_int64, u32p]
        lib.liec_oracle_compress_rng.restype = ctypes.c_int
        lib.liec_oracle_compress_rng.argtypes = [ctypes.c_int, fp, ctypes.c_int64, ctypes.c_int64, ip, ctypes.c_int32,
                                                 u64, u64, u32, fp, dp, fp]
        lib.liec_oracle_step_rng.restype = ctypes.c_int
        lib.liec_oracle_step_rng.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
                                             ctypes.c_int, ctypes.c_int64, ctypes.c_float, fp, fp, fp, ip,
                                             ctypes.c_int32, u64, u64, dp, dp, fp, fp, fp, fp, fp]
        lib.liec_oracle_pack_randk.restype = ctypes.c_int
        lib.liec_oracle_pack_randk.argtypes = [fp, ctypes.c_int64, ctypes.c_int64, u64, u64, u32, u32p, fp]
        lib.liec_oracle_desc_size.restype = ctypes.c_int
        assert lib.liec_oracle_desc_size() == ctypes.sizeof(_CDesc)
        _lib = lib
    return _lib


def _comp(c) -> int:
    return _NAMES[c] if isinstance(c, str) else int(c)


def _f32(a: np.ndarray, writable: bool = False) -> np.ndarray:
    if not (isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags.c_contiguous):
        raise TypeError("oracle arrays must be C-contiguous numpy float32")
    if writable and not a.flags.writeable:
        raise TypeError("oracle output array is read-only")
    return a


def _ptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _desc(c: _CDesc) -> Desc:
    return Desc(float(c.scale), float(c.l1), int(c.tau_key), int(c.cutoff), int(c.count_above))


def compress(comp, v: np.ndarray, k: int = 0, want_p: bool = True,
             rng: Tuple[int, int, int] = (0, 0, 0)) -> Tuple[Optional[np.ndarray], Desc]:
    """p = C(v) (Definition 2, 3 or 4, or identity) and its descriptor.  rng = (seed, draw, row)
    names the random draw of Definition 3."""
    lib = _load()
    v = _f32(v)
    assert v.ndim == 1
    p = np.empty_like(v) if want_p else None
    c = _CDesc()
    rc = lib.liec_oracle_compress_rng(_comp(comp), _ptr(v), v.shape[0], int(k), None, 0, int(rng[0]), int(rng[1]),
                                      int(rng[2]), _ptr(p), ctypes.byref(c), None)
    if rc != 0:
        raise ValueError(f"liec_oracle_compress_rng failed with code {rc}")
    return p, _desc(c)


def randk_priorities(d: int, rng: Tuple[int, int, int]) -> np.ndarray:
    """Priority (31 bits) that the generator of Definition 3's draw gives to each index 0..d-1."""
    lib = _load()
    out = np.empty(d, dtype=np.uint32)
    lib.liec_oracle_randk_priorities(int(rng[0]), int(rng[1]), int(rng[2]), d,
                                     out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)))
    return out


def server_average(P: np.ndarray, e: np.ndarray) -> np.ndarray:
    """v = e + (1/N) sum_i p^i (Algorithm 1, server compensation)."""
    lib = _load()
    P, e = _f32(P), _f32(e)
    N, d = P.shape
    assert e.shape == (d,)
    v = np.empty(d, dtype=np.float32)
    lib.liec_oracle_server_average(_ptr(P), N, d, _ptr(e), _ptr(v))
    return v


def error_update(v: np.ndarray, p: np.ndarray) -> np.ndarray:
    """e_{t+1} = v_t - p_t (Algorithm 1, global error update)."""
    lib = _load()
    v, p = _f32(v), _f32(p)
    out = np.empty_like(v)
    lib.liec_oracle_error_update(_ptr(v), _ptr(p), v.shape[0], _ptr(out))
    return out


def worker_update(g_i: np.ndarray, p_i: np.ndarray, p: np.ndarray, lr: float, x_i: np.ndarray) -> None:
    """x^i <- x^i - eta (p + (g_i - p^i)), in place (Algorithm 1, worker update)."""
    lib = _load()
    g_i, p_i, p, x_i = _f32(g_i), _f32(p_i), _f32(p), _f32(x_i, True)
    d = g_i.shape[0]
    assert p_i.shape == (d,) and p.shape == (d,) and x_i.shape == (d,)
    lib.liec_oracle_worker_update(_ptr(g_i), _ptr(p_i), _ptr(p), d, ctypes.c_float(lr), _ptr(x_i))


@dataclass
class StepTrace:
    worker: List[Desc]
    server: Desc
    v: Optional[np.ndarray]
    p: Optional[np.ndarray]
    P: Optional[np.ndarray]


def step(g: np.ndarray, x: np.ndarray, e: np.ndarray, worker_comp, server_comp, lr: float,
         worker_k: int = 0, server_k: int = 0, trace: bool = False, rng: Tuple[int, int] = (0, 0)) -> StepTrace:
    """One compressed iteration of Algorithm 1; x [N,d] and e [d] are updated in place.
    rng = (seed, draw) names this iteration's draws of Definition 3."""
    lib = _load()
    g, x, e = _f32(g), _f32(x, True), _f32(e, True)
    N, d = g.shape
    assert x.shape == (N, d) and e.shape == (d,)
    wd = (_CDesc * N)()
    sd = _CDesc()
    v = np.empty(d, dtype=np.float32) if trace else None
    p = np.empty(d, dtype=np.float32) if trace else None
    P = np.empty((N, d), dtype=np.float32) if trace else None
    rc = lib.liec_oracle_step_rng(N, d, _comp(worker_comp), int(worker_k), _comp(server_comp), int(server_k),
                                  ctypes.c_float(lr), _ptr(g), _ptr(x), _ptr(e), None, 0, int(rng[0]), int(rng[1]),
                                  wd, ctypes.byref(sd), None, None, _ptr(v), _ptr(p), _ptr(P))
    if rc != 0:
        raise ValueError(f"liec_oracle_step_rng failed with code {rc}")
    return StepTrace([_desc(c) for c in wd], _desc(sd), v, p, P)


def step_sync(g: np.ndarray, x: np.ndarray, e: np.ndarray, lr: float, want_v: bool = False) -> Optional[np.ndarray]:
    """The averaging iteration of Algorithm 1; x [N,d] and e [d] are updated in place."""
    lib = _load()
    g, x, e = _f32(g), _f32(x, True), _f32(e, True)
    N, d = g.shape
    assert x.shape == (N, d) and e.shape == (d,)
    v = np.empty(d, dtype=np.float32) if want_v else None
    rc = lib.liec_oracle_step_sync(N, d, ctypes.c_float(lr), _ptr(g), _ptr(x), _ptr(e), _ptr(v))
    if rc != 0:
        raise ValueError(f"liec_oracle_step_sync failed with code {rc}")
    return v


def _offsets(blocks) -> np.ndarray:
    off = np.ascontiguousarray(np.asarray(blocks, dtype=np.int64))
    assert off.ndim == 1 and off.size >= 2
    return off


def compress_blocksign(v: np.ndarray, blocks) -> Tuple[np.ndarray, np.ndarray]:
    """Definition 5: scaled sign per block; `blocks` are the B+1 block offsets. Returns (p, scales[B])."""
    lib = _load()
    v = _f32(v)
    off = _offsets(blocks)
    B = off.size - 1
    p = np.empty_like(v)
    scales = np.empty(B, dtype=np.float32)
    c = _CDesc()
    rc = lib.liec_oracle_compress_ex(BLOCKSIGN, _ptr(v), v.shape[0], 0, off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                     B, _ptr(p), ctypes.byref(c), _ptr(scales))
    if rc != 0:
        raise ValueError(f"liec_oracle_compress_ex failed with code {rc}")
    return p, scales


@dataclass
class BlockStepTrace:
    worker: List[Desc]
    server: Desc
    worker_scales: np.ndarray
    server_scales: np.ndarray


def step_blocks(g: np.ndarray, x: np.ndarray, e: np.ndarray, worker_comp, server_comp, lr: float, blocks,
                worker_k: int = 0, server_k: int = 0, rng: Tuple[int, int] = (0, 0)) -> BlockStepTrace:
    """One compressed iteration of Algorithm 1 with Definition 5's block table available to both sides
    (and rng = (seed, draw) for Definition 3's draws)."""
    lib = _load()
    g, x, e = _f32(g), _f32(x, True), _f32(e, True)
    N, d = g.shape
    off = _offsets(blocks)
    B = off.size - 1
    wd = (_CDesc * N)()
    sd = _CDesc()
    ws = np.zeros((N, B), dtype=np.float32)
    ss = np.zeros(B, dtype=np.float32)
    rc = lib.liec_oracle_step_rng(N, d, _comp(worker_comp), int(worker_k), _comp(server_comp), int(server_k),
                                  ctypes.c_float(lr), _ptr(g), _ptr(x), _ptr(e),
                                  off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), B, int(rng[0]), int(rng[1]),
                                  wd, ctypes.byref(sd), _ptr(ws), _ptr(ss), None, None, None)
    if rc != 0:
        raise ValueError(f"liec_oracle_step_rng failed with code {rc}")
    return BlockStepTrace([_desc(c) for c in wd], _desc(sd), ws, ss)


def pack_sign(v: np.ndarray) -> np.ndarray:
    """Wire bits of a (blockwise) scaled-sign message: bit j%8 of byte j//8 set when v_j < 0."""
    lib = _load()
    v = _f32(v)
    out = np.empty((v.shape[0] + 7) // 8, dtype=np.uint8)
    lib.liec_oracle_pack_sign(_ptr(v), v.shape[0], out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    return out


def unpack_sign(bits: np.ndarray, d: int, scales, blocks=None) -> np.ndarray:
    """Dense message from wire bits and the scale (one) or per-block scales (with `blocks` offsets)."""
    lib = _load()
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    sc = np.ascontiguousarray(np.atleast_1d(np.asarray(scales, dtype=np.float32)))
    p = np.empty(d, dtype=np.float32)
    if blocks is None:
        offp, B = None, 1
    else:
        off = _offsets(blocks)
        offp, B = off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), off.size - 1
    lib.liec_oracle_unpack_sign(bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), d, _ptr(sc), offp, B, _ptr(p))
    return p


def pack_topk(v: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Wire form of a top-k message: (indices ascending, values), k entries each."""
    lib = _load()
    v = _f32(v)
    idx = np.empty(k, dtype=np.uint32)
    val = np.empty(k, dtype=np.float32)
    rc = lib.liec_oracle_pack_topk(_ptr(v), v.shape[0], k, idx.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), _ptr(val))
    if rc != 0:
        raise ValueError(f"liec_oracle_pack_topk failed with code {rc}")
    return idx, val


def pack_randk(v: np.ndarray, k: int, rng: Tuple[int, int, int]) -> Tuple[np.ndarray, np.ndarray]:
    """Wire form of a random-k message: (indices ascending, values), k entries each."""
    lib = _load()
    v = _f32(v)
    idx = np.empty(k, dtype=np.uint32)
    val = np.empty(k, dtype=np.float32)
    rc = lib.liec_oracle_pack_randk(_ptr(v), v.shape[0], k, int(rng[0]), int(rng[1]), int(rng[2]),
                                    idx.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), _ptr(val))
    if rc != 0:
        raise ValueError(f"liec_oracle_pack_randk failed with code {rc}")
    return idx, val


def unpack_topk(idx: np.ndarray, val: np.ndarray, d: int) -> np.ndarray:
    lib = _load()
    idx = np.ascontiguousarray(idx, dtype=np.uint32)
    val = _f32(np.ascontiguousarray(val, dtype=np.float32))
    p = np.empty(d, dtype=np.float32)
    lib.liec_oracle_unpack_topk(idx.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), _ptr(val), idx.size, d, _ptr(p))
    return p
