"""ctypes binding of libthemis_hip.so: argument marshalling only.

PyTorch is used for device memory and the current HIP stream; every
computation happens in the library's kernels.  Loading fails loudly if the
library has not been built (python paper_2110_04478_amd/csrc/build.py).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libthemis_hip.so")

MAX_DIMS = 4
MAX_CHUNKS = 512

_vp = C.c_void_p


class _Batch(C.Structure):
    _fields_ = [
        ("n", C.c_uint64), ("max_chunks", C.c_uint32), ("threshold_mode", C.c_uint32),
        ("ndims", _vp), ("npus", _vp), ("bw", _vp), ("size_bytes", _vp), ("chunks", _vp),
        ("inter_policy", _vp), ("intra_policy", _vp), ("threshold", _vp),
        ("max_coll", C.c_uint32), ("n_coll", _vp), ("coll_size", _vp), ("release_time", _vp),
        ("fixed_delay", _vp), ("collective_type", _vp),
    ]


_lib = None


def lib():
    """The loaded C ABI library; raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with "
                "`python paper_2110_04478_amd/csrc/build.py` (there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        L.themis_version.restype = C.c_int
        L.themis_status_string.restype = C.c_char_p
        L.themis_status_string.argtypes = [C.c_int]
        L.themis_queue_entry_bytes.restype = C.c_int
        L.themis_queue_entry_bytes.argtypes = [C.c_uint32, C.c_uint32]
        L.themis_workspace_bytes.restype = C.c_size_t
        L.themis_workspace_bytes.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        L.themis_plan_batch.restype = C.c_int
        L.themis_plan_batch.argtypes = [C.POINTER(_Batch), _vp, _vp, _vp]
        L.themis_simulate_batch.restype = C.c_int
        L.themis_simulate_batch.argtypes = [C.POINTER(_Batch), _vp, _vp, _vp, _vp, _vp,
                                            C.c_size_t, _vp]
        L.themis_simulate_batch_noalloc.restype = C.c_int
        L.themis_simulate_batch_noalloc.argtypes = [C.POINTER(_Batch), _vp, _vp, _vp, _vp, _vp]
        L.themis_metrics_batch.restype = C.c_int
        L.themis_metrics_batch.argtypes = [C.POINTER(_Batch), _vp, _vp, _vp, _vp, _vp]
        L.themis_search_workspace_bytes.restype = C.c_size_t
        L.themis_search_workspace_bytes.argtypes = [C.c_uint64, C.c_uint64]
        L.themis_search_batch.restype = C.c_int
        L.themis_search_batch.argtypes = [C.POINTER(_Batch), C.c_uint64, _vp, _vp, _vp,
                                          C.c_size_t, _vp]
        L.themis_beam_workspace_bytes.restype = C.c_size_t
        L.themis_beam_workspace_bytes.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        L.themis_beam_search_batch.restype = C.c_int
        L.themis_beam_search_batch.argtypes = [C.POINTER(_Batch), C.c_uint32, _vp, _vp, _vp,
                                               C.c_size_t, _vp]
        L.themis_classify_batch.restype = C.c_int
        L.themis_classify_batch.argtypes = [C.POINTER(_Batch), _vp, _vp]
        L.themis_sweep_best.restype = C.c_int
        L.themis_sweep_best.argtypes = [C.c_uint64, C.c_int, C.c_int, _vp, C.c_int, _vp, _vp, _vp, _vp]
        L.themis_set_sweep_mapping.restype = C.c_int
        L.themis_set_sweep_mapping.argtypes = [C.c_int]
        L.themis_sweep.restype = C.c_int
        L.themis_sweep.argtypes = [C.POINTER(_Batch), C.c_int, _vp, C.c_int, C.c_uint, _vp,
                                   _vp, C.c_size_t, _vp]
        _lib = L
    return _lib


class ThemisError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"themis: {lib().themis_status_string(status).decode()} ({status})")


def _check(status: int):
    if status != 0:
        raise ThemisError(status)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else _vp(t.data_ptr())


def _stream() -> _vp:
    return _vp(torch.cuda.current_stream().cuda_stream)


@dataclass
class DeviceBatch:
    """A scenario batch resident in HBM (torch tensors own the memory)."""
    n: int
    max_chunks: int
    threshold_mode: int
    ndims: torch.Tensor
    npus: torch.Tensor
    bw: torch.Tensor
    size_bytes: torch.Tensor
    chunks: torch.Tensor
    inter_policy: torch.Tensor
    intra_policy: torch.Tensor
    threshold: torch.Tensor
    max_coll: int = 0
    n_coll: Optional[torch.Tensor] = None
    coll_size: Optional[torch.Tensor] = None
    release_time: Optional[torch.Tensor] = None
    fixed_delay: Optional[torch.Tensor] = None
    collective_type: Optional[torch.Tensor] = None

    @property
    def slots(self) -> int:
        return self.max_chunks * (self.max_coll if self.n_coll is not None else 1)

    @property
    def device(self):
        return self.ndims.device

    def c_struct(self) -> _Batch:
        return _Batch(self.n, self.max_chunks, self.threshold_mode, _ptr(self.ndims),
                      _ptr(self.npus), _ptr(self.bw), _ptr(self.size_bytes), _ptr(self.chunks),
                      _ptr(self.inter_policy), _ptr(self.intra_policy), _ptr(self.threshold),
                      self.max_coll, _ptr(self.n_coll), _ptr(self.coll_size),
                      _ptr(self.release_time), _ptr(self.fixed_delay),
                      _ptr(self.collective_type))


def to_device(b, device="cuda:0") -> DeviceBatch:
    """Copies a host workloads.ScenarioBatch into HBM."""
    def up(a, dt):
        if a is None:
            return None
        a = np.ascontiguousarray(a)
        if not a.flags.writeable:  # broadcast views: torch wants a writable source
            a = a.copy()
        if dt == torch.uint32:  # torch cannot build uint32 from numpy directly everywhere
            return torch.from_numpy(a.view(np.int32)).to(device).view(torch.uint32)
        return torch.from_numpy(a).to(device)
    return DeviceBatch(
        n=int(b.n), max_chunks=int(b.max_chunks), threshold_mode=int(b.threshold_mode),
        ndims=up(b.ndims, torch.uint8), npus=up(b.npus, torch.uint32), bw=up(b.bw, torch.float64),
        size_bytes=up(b.size_bytes, torch.float64), chunks=up(b.chunks, torch.uint32),
        inter_policy=up(b.inter_policy, torch.uint8), intra_policy=up(b.intra_policy, torch.uint8),
        threshold=up(b.threshold, torch.float64), max_coll=int(b.max_coll),
        n_coll=up(b.n_coll, torch.uint32), coll_size=up(b.coll_size, torch.float64),
        release_time=up(b.release_time, torch.float64),
        fixed_delay=up(getattr(b, "fixed_delay", None), torch.float64),
        collective_type=up(getattr(b, "collective_type", None), torch.uint8))


def themis_version() -> int:
    return lib().themis_version()


def themis_queue_entry_bytes(max_chunks: int, max_coll: int = 0) -> int:
    return lib().themis_queue_entry_bytes(max_chunks, max_coll)


def themis_workspace_bytes(n: int, max_chunks: int, max_coll: int = 0) -> int:
    return lib().themis_workspace_bytes(n, max_chunks, max_coll)


def themis_plan_batch(b: DeviceBatch, orders: Optional[torch.Tensor] = None,
                      loads: Optional[torch.Tensor] = None, want_loads: bool = True):
    """Alg. 1 for every scenario -> (orders u8[n, slots], loads f64[4, n] or None)."""
    if orders is None:
        orders = torch.empty((b.n, b.slots), dtype=torch.uint8, device=b.device)
    if loads is None and want_loads:
        loads = torch.empty((MAX_DIMS, b.n), dtype=torch.float64, device=b.device)
    s = b.c_struct()
    _check(lib().themis_plan_batch(C.byref(s), _ptr(orders), _ptr(loads), _stream()))
    return orders, loads


def themis_simulate_batch(b: DeviceBatch, orders: torch.Tensor,
                          t_done: Optional[torch.Tensor] = None,
                          queue_order: Optional[torch.Tensor] = None,
                          busy: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None,
                          want_queue_order: bool = True, want_busy: bool = True):
    """Queue simulation -> (t_done f64[n], queue_order [n,4,2*slots] or None,
    busy f64[4,n] or None)."""
    dev = b.device
    if t_done is None:
        t_done = torch.empty(b.n, dtype=torch.float64, device=dev)
    if queue_order is None and want_queue_order:
        eb = themis_queue_entry_bytes(b.max_chunks, b.max_coll if b.n_coll is not None else 0)
        queue_order = torch.empty((b.n, MAX_DIMS, 2 * b.slots),
                                  dtype=torch.uint8 if eb == 1 else torch.uint16, device=dev)
    if busy is None and want_busy:
        busy = torch.empty((MAX_DIMS, b.n), dtype=torch.float64, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    s = b.c_struct()
    _check(lib().themis_simulate_batch(C.byref(s), _ptr(orders), _ptr(t_done), _ptr(queue_order),
                                       _ptr(busy), _ptr(workspace), ws_bytes, _stream()))
    return t_done, queue_order, busy


STATIC_SCRATCH_BYTES = 32 << 20


def themis_simulate_batch_noalloc(b: DeviceBatch, orders: torch.Tensor, t_done: torch.Tensor,
                                  queue_order: Optional[torch.Tensor],
                                  busy: Optional[torch.Tensor]):
    """themis_simulate_batch on the library's own scratch: every buffer is the
    caller's, nothing is allocated here or in the library."""
    s = b.c_struct()
    _check(lib().themis_simulate_batch_noalloc(C.byref(s), _ptr(orders), _ptr(t_done),
                                               _ptr(queue_order), _ptr(busy), _stream()))
    return t_done, queue_order, busy


def themis_sweep(b: DeviceBatch, thr: torch.Tensor, policy_mask: int,
                 thr_per_scenario: bool = False, t_done: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None):
    """Fused plan + simulate -> t_done f64[n, n_thr, n_pol]."""
    n_thr = int(thr.shape[0])
    n_pol = bin(policy_mask & 7).count("1")
    if t_done is None:
        t_done = torch.empty((b.n, n_thr, n_pol), dtype=torch.float64, device=b.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    s = b.c_struct()
    _check(lib().themis_sweep(C.byref(s), n_thr, _ptr(thr), 1 if thr_per_scenario else 0,
                              policy_mask, _ptr(t_done), _ptr(workspace), ws_bytes, _stream()))
    return t_done


MAPPING_AUTO, MAPPING_LANE, MAPPING_QUAD = 0, 1, 2


def themis_set_sweep_mapping(mapping: int) -> None:
    """Lane mapping of themis_sweep's LDS kernel (MAPPING_AUTO / _LANE / _QUAD), process-wide."""
    _check(lib().themis_set_sweep_mapping(int(mapping)))


def themis_metrics_batch(b: DeviceBatch, t_done: torch.Tensor, transfer: torch.Tensor,
                         utilization: Optional[torch.Tensor] = None,
                         ideal: Optional[torch.Tensor] = None):
    """Average bandwidth utilisation and Ideal time -> (utilization f64[n], ideal f64[n])."""
    if utilization is None:
        utilization = torch.empty(b.n, dtype=torch.float64, device=b.device)
    if ideal is None:
        ideal = torch.empty(b.n, dtype=torch.float64, device=b.device)
    s = b.c_struct()
    _check(lib().themis_metrics_batch(C.byref(s), _ptr(t_done), _ptr(transfer), _ptr(utilization),
                                      _ptr(ideal), _stream()))
    return utilization, ideal


def themis_beam_search_batch(b: DeviceBatch, width: int, workspace: Optional[torch.Tensor] = None):
    """Beam search over per-chunk orders -> (best_t f64[n], best_orders u8[n, max_chunks])."""
    best_t = torch.empty(b.n, dtype=torch.float64, device=b.device)
    best_orders = torch.empty((b.n, b.max_chunks), dtype=torch.uint8, device=b.device)
    if workspace is None:
        workspace = alloc_workspace(lib().themis_beam_workspace_bytes(b.n, b.max_chunks, width),
                                    b.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    s = b.c_struct()
    _check(lib().themis_beam_search_batch(C.byref(s), int(width), _ptr(best_t), _ptr(best_orders),
                                          _ptr(workspace), ws_bytes, _stream()))
    return best_t, best_orders


def themis_search_workspace_bytes(n: int, max_assignments: int) -> int:
    return lib().themis_search_workspace_bytes(n, max_assignments)


def themis_search_batch(b: DeviceBatch, max_assignments: int,
                        workspace: Optional[torch.Tensor] = None):
    """Exhaustive search over per-chunk orders -> (best_t f64[n], best_orders u8[n, max_chunks])."""
    best_t = torch.empty(b.n, dtype=torch.float64, device=b.device)
    best_orders = torch.empty((b.n, b.max_chunks), dtype=torch.uint8, device=b.device)
    if workspace is None:
        workspace = alloc_workspace(themis_search_workspace_bytes(b.n, max_assignments), b.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    s = b.c_struct()
    _check(lib().themis_search_batch(C.byref(s), max_assignments, _ptr(best_t), _ptr(best_orders),
                                     _ptr(workspace), ws_bytes, _stream()))
    return best_t, best_orders


def themis_classify_batch(b: DeviceBatch) -> torch.Tensor:
    """Bandwidth provisioning class of every dimension pair -> u8[6, n]."""
    classes = torch.empty((6, b.n), dtype=torch.uint8, device=b.device)
    s = b.c_struct()
    _check(lib().themis_classify_batch(C.byref(s), _ptr(classes), _stream()))
    return classes


def themis_sweep_best(t_done: torch.Tensor, baseline_col: int = -1):
    """Best threshold per scenario and scheduler of a sweep result f64[n, n_thr, n_pol]
    -> (best_t f64[n, n_pol], best_thr u32[n, n_pol], speedup f64[n, n_pol] or None)."""
    n, n_thr, n_pol = t_done.shape
    assert t_done.dtype == torch.float64 and t_done.is_contiguous()
    best_t = torch.empty((n, n_pol), dtype=torch.float64, device=t_done.device)
    best_thr = torch.empty((n, n_pol), dtype=torch.uint32, device=t_done.device)
    speedup = (torch.empty((n, n_pol), dtype=torch.float64, device=t_done.device)
               if baseline_col >= 0 else None)
    _check(lib().themis_sweep_best(n, n_thr, n_pol, _ptr(t_done), baseline_col, _ptr(best_t),
                                   _ptr(best_thr), _ptr(speedup), _stream()))
    return best_t, best_thr, speedup


def alloc_workspace(nbytes: int, device="cuda:0") -> Optional[torch.Tensor]:
    """Device scratch for the generic path (a plain byte tensor)."""
    if nbytes <= 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)
