"""HIP streams that own part of the device.

Sec. 3.3 of the paper overlaps drafting with verification by giving each a spatial share of the
GPU (there: SM partitions made with Green Contexts).  The MI355X counterpart is a stream created
with a compute-unit mask: kernels enqueued on it are dispatched only to the compute units whose
bits are set.  A persistent-grid kernel such as the verification attention should then be told how
many compute units it will get (``max_workgroups``), so that it launches one workgroup per unit of
its share instead of one per unit of the device.

The mask is an array of 32-bit words, bit i of the concatenation standing for logical compute unit
i; the runtime spreads consecutive logical units over the accelerator dies, so a prefix of the bit
range is an even share of every die.
"""
from __future__ import annotations

import ctypes
from typing import Iterable

import torch

_hip = None


def _runtime():
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")  # the runtime torch has already loaded
        _hip.hipExtStreamCreateWithCUMask.restype = ctypes.c_int
        _hip.hipStreamDestroy.restype = ctypes.c_int
    return _hip


class MaskedStream:
    """A HIP stream restricted to the given logical compute units, usable as a torch stream
    (``with torch.cuda.stream(ms.stream): ...``).  Destroyed with the object."""

    def __init__(self, cu_ids: Iterable[int], device: int = 0):
        ids = sorted(set(int(c) for c in cu_ids))
        n_cus = torch.cuda.get_device_properties(device).multi_processor_count
        if not ids or ids[0] < 0 or ids[-1] >= n_cus:
            raise ValueError(f"compute-unit ids must lie in [0, {n_cus})")
        words = [0] * ((n_cus + 31) // 32)
        for c in ids:
            words[c // 32] |= 1 << (c % 32)
        mask = (ctypes.c_uint32 * len(words))(*words)
        handle = ctypes.c_void_p()
        with torch.cuda.device(device):
            rc = _runtime().hipExtStreamCreateWithCUMask(ctypes.byref(handle), ctypes.c_uint32(len(words)), mask)
        if rc != 0 or not handle.value:
            raise RuntimeError(f"hipExtStreamCreateWithCUMask failed with error {rc}")
        self._handle = handle
        self.n_cus = len(ids)
        self.stream = torch.cuda.ExternalStream(handle.value, device=device)

    def __del__(self):
        h = getattr(self, "_handle", None)
        if h is not None and h.value:
            try:
                self.stream.synchronize()
                _runtime().hipStreamDestroy(h)
            except Exception:  # interpreter shutdown
                pass
            self._handle = None


def split_device(n_first: int, device: int = 0):
    """Two masked streams that partition the device: the first ``n_first`` logical compute units and the rest."""
    n_cus = torch.cuda.get_device_properties(device).multi_processor_count
    if not 0 < n_first < n_cus:
        raise ValueError(f"n_first must lie in (0, {n_cus})")
    return MaskedStream(range(n_first), device), MaskedStream(range(n_first, n_cus), device)
