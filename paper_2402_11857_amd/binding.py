"""ctypes binding of include/liec.h (same names, argument marshalling only).

torch is imported before the library is loaded so that the HIP runtime torch
ships is the one both sides share; tensors are passed as raw device pointers.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Tuple

import torch

COMP_IDENTITY, COMP_SIGN, COMP_TOPK, COMP_BLOCKSIGN, COMP_RANDK = 0, 1, 2, 3, 4
_COMP_NAMES = {"identity": COMP_IDENTITY, "sign": COMP_SIGN, "topk": COMP_TOPK, "blocksign": COMP_BLOCKSIGN,
               "randk": COMP_RANDK}
OK, EINVAL, ENOMEM, EDEVICE, ENONFINITE = 0, 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libliec.so")
_lib = None


class LiecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().liec_status_string(status).decode() if _lib is not None else str(status)
        super().__init__(f"{where}: {msg} (status {status})")


class LiecInfo(ctypes.Structure):
    _fields_ = [
        ("N", ctypes.c_int32),
        ("d", ctypes.c_int64),
        ("worker_comp", ctypes.c_int32),
        ("server_comp", ctypes.c_int32),
        ("worker_k", ctypes.c_int64),
        ("server_k", ctypes.c_int64),
        ("lr", ctypes.c_float),
        ("steps_done", ctypes.c_int64),
        ("server_scale", ctypes.c_float),
        ("server_l1", ctypes.c_double),
        ("server_tau_key", ctypes.c_uint32),
        ("server_cutoff", ctypes.c_int64),
        ("nonfinite", ctypes.c_int32),
        ("slow_rows", ctypes.c_int32),
        ("band_misses", ctypes.c_int64),
    ]


def library_path() -> str:
    return _LIB_PATH


def lib():
    """Loads libliec.so (built by ``__graft_entry__.build()``); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`. "
                "There is no fallback path.")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
        L.liec_create.restype = ctypes.c_int
        L.liec_create.argtypes = [ctypes.POINTER(vp), i32, i64, ctypes.c_int, i64, f32]
        L.liec_create_ex.restype = ctypes.c_int
        L.liec_create_ex.argtypes = [ctypes.POINTER(vp), i32, i64, ctypes.c_int, i64, ctypes.c_int, i64, f32, vp]
        L.liec_step.restype = ctypes.c_int
        L.liec_step.argtypes = [vp, vp, vp, vp]
        L.liec_step_sync.restype = ctypes.c_int
        L.liec_step_sync.argtypes = [vp, vp, vp, vp]
        L.liec_iteration.restype = ctypes.c_int
        L.liec_iteration.argtypes = [vp, i64, i64, vp, vp, vp]
        L.liec_set_blocks.restype = ctypes.c_int
        L.liec_set_blocks.argtypes = [vp, ctypes.POINTER(i64), i32]
        L.liec_get_block_scales.restype = ctypes.c_int
        L.liec_get_block_scales.argtypes = [vp, ctypes.POINTER(f32), ctypes.POINTER(f32)]
        L.liec_message_bytes.restype = i64
        L.liec_message_bytes.argtypes = [ctypes.c_int, i64, i64, i32]
        L.liec_comm_cost.restype = ctypes.c_int
        L.liec_comm_cost.argtypes = [i32, i64, ctypes.c_int, i64, ctypes.c_int, i64, i32, i32, i32,
                                     ctypes.POINTER(ctypes.c_double)]
        L.liec_pack_sign_bits.restype = ctypes.c_int
        L.liec_pack_sign_bits.argtypes = [vp, i32, vp]
        L.liec_unpack_sign_message.restype = ctypes.c_int
        L.liec_unpack_sign_message.argtypes = [vp, vp, ctypes.POINTER(f32), i32, vp]
        L.liec_pack_topk_message.restype = ctypes.c_int
        L.liec_pack_topk_message.argtypes = [vp, vp, i32, vp, vp]
        L.liec_unpack_topk_message.restype = ctypes.c_int
        L.liec_unpack_topk_message.argtypes = [vp, vp, vp, i64, vp]
        L.liec_set_lr.restype = ctypes.c_int
        L.liec_set_lr.argtypes = [vp, f32]
        L.liec_set_random.restype = ctypes.c_int
        L.liec_set_random.argtypes = [vp, ctypes.c_uint64, ctypes.c_uint64]
        L.liec_get_random.restype = ctypes.c_int
        L.liec_get_random.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]
        L.liec_l2_norm.restype = ctypes.c_int
        L.liec_l2_norm.argtypes = [vp, vp, i64, ctypes.POINTER(ctypes.c_double)]
        L.liec_l2_norm_static.restype = ctypes.c_int
        L.liec_l2_norm_static.argtypes = [vp, i64, vp, vp]
        L.liec_force_search_mode.restype = ctypes.c_int
        L.liec_force_search_mode.argtypes = [vp, i32]
        L.liec_set_search_wait.restype = ctypes.c_int
        L.liec_set_search_wait.argtypes = [vp, i32]
        L.liec_get_search_state.restype = ctypes.c_int
        L.liec_get_search_state.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_uint32)]
        L.liec_set_group_bitmap.restype = ctypes.c_int
        L.liec_set_group_bitmap.argtypes = [vp, i32]
        L.liec_set_gather_batching.restype = ctypes.c_int
        L.liec_set_gather_batching.argtypes = [vp, i32]
        L.liec_get_info.restype = ctypes.c_int
        L.liec_get_info.argtypes = [vp, ctypes.POINTER(LiecInfo)]
        L.liec_get_worker_desc.restype = ctypes.c_int
        L.liec_get_worker_desc.argtypes = [vp, ctypes.POINTER(f32), ctypes.POINTER(ctypes.c_double),
                                           ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(i64)]
        L.liec_profile_begin.restype = ctypes.c_int
        L.liec_profile_begin.argtypes = [vp, i32, i32]
        L.liec_profile_end.restype = ctypes.c_int
        L.liec_profile_end.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_char_p),
                                       ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
        L.liec_destroy.restype = None
        L.liec_destroy.argtypes = [vp]
        L.liec_status_string.restype = ctypes.c_char_p
        L.liec_status_string.argtypes = [ctypes.c_int]
        L.liec_scratch_bytes.restype = i64
        L.liec_scratch_bytes.argtypes = [vp]
        L.liec_device_copy.restype = ctypes.c_int
        L.liec_device_copy.argtypes = [vp, vp, i64, vp]
        _lib = L
    return _lib


def _comp(c) -> int:
    return _COMP_NAMES[c] if isinstance(c, str) else int(c)


def _check(status: int, where: str) -> None:
    if status != OK:
        raise LiecError(status, where)


def _dev_ptr(t: torch.Tensor, shape: Tuple[int, ...], name: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous float32 tensor on the GPU")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t.data_ptr()


# ---- the C entry points, one to one -----------------------------------------------------------
def liec_create(N: int, d: int, compressor, k: int, lr: float) -> int:
    h = ctypes.c_void_p()
    _check(lib().liec_create(ctypes.byref(h), N, d, _comp(compressor), int(k), lr), "liec_create")
    return h.value


def liec_create_ex(N: int, d: int, worker_comp, worker_k: int, server_comp, server_k: int, lr: float,
                   stream: Optional[int] = None) -> int:
    h = ctypes.c_void_p()
    _check(lib().liec_create_ex(ctypes.byref(h), N, d, _comp(worker_comp), int(worker_k), _comp(server_comp),
                                int(server_k), lr, stream), "liec_create_ex")
    return h.value


def liec_step(ctx: int, grads_ptr: int, x_ptr: int, server_err_ptr: int) -> None:
    _check(lib().liec_step(ctx, grads_ptr, x_ptr, server_err_ptr), "liec_step")


def liec_step_sync(ctx: int, grads_ptr: int, x_ptr: int, server_err_ptr: int) -> None:
    _check(lib().liec_step_sync(ctx, grads_ptr, x_ptr, server_err_ptr), "liec_step_sync")


def liec_set_blocks(ctx: int, offsets) -> None:
    off = [int(o) for o in offsets]
    arr = (ctypes.c_int64 * len(off))(*off)
    _check(lib().liec_set_blocks(ctx, arr, len(off) - 1), "liec_set_blocks")


def liec_get_block_scales(ctx: int, N: int, nblocks: int):
    ws = (ctypes.c_float * (N * nblocks))()
    ss = (ctypes.c_float * nblocks)()
    _check(lib().liec_get_block_scales(ctx, ws, ss), "liec_get_block_scales")
    return [list(ws[i * nblocks:(i + 1) * nblocks]) for i in range(N)], list(ss)


def liec_message_bytes(comp, d: int, k: int = 0, nblocks: int = 0) -> int:
    return int(lib().liec_message_bytes(_comp(comp), d, k, nblocks))


def liec_comm_cost(N: int, d: int, worker_comp, worker_k: int, server_comp, server_k: int, nblocks: int = 0,
                   period: int = 0, count_model_exchange: bool = False) -> float:
    out = ctypes.c_double()
    _check(lib().liec_comm_cost(N, d, _comp(worker_comp), worker_k, _comp(server_comp), server_k, nblocks, period,
                                1 if count_model_exchange else 0, ctypes.byref(out)), "liec_comm_cost")
    return out.value


def liec_set_lr(ctx: int, lr: float) -> None:
    _check(lib().liec_set_lr(ctx, lr), "liec_set_lr")


def liec_set_random(ctx: int, seed: int, draw: int) -> None:
    _check(lib().liec_set_random(ctx, seed, draw), "liec_set_random")


def liec_get_random(ctx: int) -> Tuple[int, int]:
    seed, draw = ctypes.c_uint64(), ctypes.c_uint64()
    _check(lib().liec_get_random(ctx, ctypes.byref(seed), ctypes.byref(draw)), "liec_get_random")
    return int(seed.value), int(draw.value)


def liec_get_info(ctx: int) -> Tuple[LiecInfo, int]:
    info = LiecInfo()
    st = lib().liec_get_info(ctx, ctypes.byref(info))
    if st not in (OK, ENONFINITE):
        raise LiecError(st, "liec_get_info")
    return info, st


def liec_get_worker_desc(ctx: int, N: int) -> Dict[str, list]:
    sc = (ctypes.c_float * N)()
    l1 = (ctypes.c_double * N)()
    tau = (ctypes.c_uint32 * N)()
    cut = (ctypes.c_int64 * N)()
    _check(lib().liec_get_worker_desc(ctx, sc, l1, tau, cut), "liec_get_worker_desc")
    return {"scale": list(sc), "l1": list(l1), "tau_key": list(tau), "cutoff": list(cut)}


def liec_destroy(ctx: Optional[int]) -> None:
    if ctx:
        lib().liec_destroy(ctx)


def liec_l2_norm_static(vec: torch.Tensor, out: torch.Tensor, n: Optional[int] = None, stream: Optional[int] = None) -> None:
    """l2 norm of the first n values (default: all) of a contiguous fp32 device tensor into out[0] (a float64
    device tensor), enqueued on `stream` (default: the null stream); nothing is allocated or waited for."""
    if not (vec.is_cuda and vec.dtype == torch.float32 and vec.is_contiguous()):
        raise TypeError("liec_l2_norm_static needs a contiguous fp32 device tensor")
    if not (out.is_cuda and out.dtype == torch.float64 and out.numel() >= 1):
        raise TypeError("liec_l2_norm_static writes to a float64 device tensor")
    count = vec.numel() if n is None else int(n)
    _check(lib().liec_l2_norm_static(vec.data_ptr(), count, out.data_ptr(), stream), "liec_l2_norm_static")


def device_copy(dst: torch.Tensor, src: torch.Tensor, stream: Optional[int] = None) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and dst.is_cuda and src.is_cuda
    _check(lib().liec_device_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream), "liec_device_copy")


# ---- convenience wrapper: owns the handle, checks tensor shapes, nothing else ----------------
class LiecContext:
    """One LIEC-SGD context bound to torch's current stream (or the one given)."""

    def __init__(self, N: int, d: int, worker_comp, server_comp=None, worker_k: int = 0, server_k: int = 0,
                 lr: float = 0.1, stream: Optional[torch.cuda.Stream] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("LiecContext needs a GPU; there is no CPU path")
        server_comp = worker_comp if server_comp is None else server_comp
        self.N, self.d = int(N), int(d)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self._h = None
        self._h = liec_create_ex(self.N, self.d, worker_comp, worker_k, server_comp, server_k, lr,
                                 self.stream.cuda_stream)

    def step(self, grads: torch.Tensor, x: torch.Tensor, server_err: torch.Tensor) -> None:
        liec_step(self._h, _dev_ptr(grads, (self.N, self.d), "grads"), _dev_ptr(x, (self.N, self.d), "x"),
                  _dev_ptr(server_err, (self.d,), "server_err"))

    def step_sync(self, grads: torch.Tensor, x: torch.Tensor, server_err: torch.Tensor) -> None:
        liec_step_sync(self._h, _dev_ptr(grads, (self.N, self.d), "grads"), _dev_ptr(x, (self.N, self.d), "x"),
                       _dev_ptr(server_err, (self.d,), "server_err"))

    def iteration(self, t: int, period: int, grads: torch.Tensor, x: torch.Tensor, server_err: torch.Tensor) -> None:
        """Iteration t of Algorithm 1: averaging iteration when (t + 1) % period == 0, compressed otherwise."""
        _check(lib().liec_iteration(self._h, t, period, _dev_ptr(grads, (self.N, self.d), "grads"),
                                    _dev_ptr(x, (self.N, self.d), "x"), _dev_ptr(server_err, (self.d,), "server_err")),
               "liec_iteration")

    def set_blocks(self, offsets) -> None:
        self._nblocks = len(list(offsets)) - 1
        liec_set_blocks(self._h, offsets)

    def block_scales(self):
        return liec_get_block_scales(self._h, self.N, self._nblocks)

    def pack_sign_bits(self, worker: int, out: torch.Tensor) -> None:
        assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous() and out.numel() == (self.d + 7) // 8
        _check(lib().liec_pack_sign_bits(self._h, worker, out.data_ptr()), "liec_pack_sign_bits")

    def unpack_sign_message(self, bits: torch.Tensor, scales, blockwise: bool, out: torch.Tensor) -> None:
        assert bits.is_cuda and bits.dtype == torch.uint8 and bits.numel() == (self.d + 7) // 8
        _dev_ptr(out, (self.d,), "out")
        sc = [float(v) for v in scales]
        arr = (ctypes.c_float * len(sc))(*sc)
        _check(lib().liec_unpack_sign_message(self._h, bits.data_ptr(), arr, 1 if blockwise else 0, out.data_ptr()),
               "liec_unpack_sign_message")

    def pack_topk_message(self, grads: torch.Tensor, worker: int, idx_out: torch.Tensor, val_out: torch.Tensor) -> None:
        assert idx_out.is_cuda and idx_out.dtype == torch.int32 and idx_out.is_contiguous()
        assert val_out.is_cuda and val_out.dtype == torch.float32 and val_out.numel() == idx_out.numel()
        _check(lib().liec_pack_topk_message(self._h, _dev_ptr(grads, (self.N, self.d), "grads"), worker,
                                            idx_out.data_ptr(), val_out.data_ptr()), "liec_pack_topk_message")

    def unpack_topk_message(self, idx: torch.Tensor, val: torch.Tensor, out: torch.Tensor) -> None:
        assert idx.is_cuda and idx.dtype == torch.int32 and val.dtype == torch.float32 and idx.numel() == val.numel()
        _check(lib().liec_unpack_topk_message(self._h, idx.data_ptr(), val.data_ptr(), idx.numel(),
                                              _dev_ptr(out, (self.d,), "out")), "liec_unpack_topk_message")

    def set_lr(self, lr: float) -> None:
        liec_set_lr(self._h, lr)

    def set_random(self, seed: int, draw: int = 0) -> None:
        liec_set_random(self._h, seed, draw)

    def get_random(self) -> Tuple[int, int]:
        return liec_get_random(self._h)

    def l2_norm(self, vec: torch.Tensor) -> float:
        """l2 norm of a contiguous fp32 device tensor (e.g. the server error), summed in fp64."""
        if not (vec.is_cuda and vec.dtype == torch.float32 and vec.is_contiguous()):
            raise TypeError("l2_norm needs a contiguous fp32 device tensor")
        out = ctypes.c_double()
        _check(lib().liec_l2_norm(self._h, vec.data_ptr(), vec.numel(), ctypes.byref(out)), "liec_l2_norm")
        return float(out.value)

    def force_search_mode(self, mode: int) -> None:
        _check(lib().liec_force_search_mode(self._h, mode), "liec_force_search_mode")

    def set_search_wait(self, polls: int) -> None:
        _check(lib().liec_set_search_wait(self._h, polls), "liec_set_search_wait")

    def search_state(self, row: int) -> Dict[str, int]:
        out = (ctypes.c_uint32 * 8)()
        _check(lib().liec_get_search_state(self._h, row, out), "liec_get_search_state")
        return {"mode": out[0], "lo": out[1], "hi": out[2], "listed": out[3], "misses": out[4], "swing": out[5],
                "general_search": out[6]}

    def set_group_bitmap(self, per_line: int) -> None:
        _check(lib().liec_set_group_bitmap(self._h, per_line), "liec_set_group_bitmap")

    def set_gather_batching(self, on: int) -> None:
        _check(lib().liec_set_gather_batching(self._h, on), "liec_set_gather_batching")

    def info(self) -> LiecInfo:
        return liec_get_info(self._h)[0]

    def info_status(self) -> Tuple[LiecInfo, int]:
        return liec_get_info(self._h)

    def worker_desc(self) -> Dict[str, list]:
        return liec_get_worker_desc(self._h, self.N)

    def scratch_bytes(self) -> int:
        return int(lib().liec_scratch_bytes(self._h))

    def profile_begin(self, max_steps: int, update_only: bool = False) -> None:
        _check(lib().liec_profile_begin(self._h, max_steps, 1 if update_only else 0), "liec_profile_begin")

    def profile_end(self) -> Dict[str, Tuple[float, int]]:
        cap = 32
        n = ctypes.c_int32(cap)
        names = (ctypes.c_char_p * cap)()
        ms = (ctypes.c_double * cap)()
        cnt = (ctypes.c_int64 * cap)()
        _check(lib().liec_profile_end(self._h, ctypes.byref(n), names, ms, cnt), "liec_profile_end")
        return {names[i].decode(): (ms[i], cnt[i]) for i in range(n.value)}

    def close(self) -> None:
        if self._h:
            liec_destroy(self._h)
            self._h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
