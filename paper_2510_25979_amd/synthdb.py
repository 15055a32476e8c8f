"""Synthetic map database in the library's storage layout (harness code for bench and tests).

Maps are drawn densely, slice by slice, with :mod:`synth` and converted into the packed layout
on the GPU with ``attncache_pack_maps``, so a 100+ GiB database never exists in dense form.
``dense_entry`` re-draws the slice an entry belongs to (same seed) and returns the entry's dense
maps: that is how tests and the CPU baseline obtain the bytes the database was built from
without reading them back through the packed form.
"""
from __future__ import annotations

import ctypes
import time
from typing import Callable, Optional

import torch

from . import binding as ac
from . import synth


class PinnedBuffer:
    """One hipHostMalloc allocation of exactly `nbytes` (torch's own pinned allocator rounds a
    request up to the next power of two, which matters when the driver's limit on pinned memory
    is what sizes the store), viewed as a torch tensor.  Freed by close() or with the object."""

    def __init__(self, nbytes: int):
        self._hip = ctypes.CDLL("libamdhip64.so")
        self._hip.hipHostMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t, ctypes.c_uint]
        self._hip.hipHostFree.argtypes = [ctypes.c_void_p]
        self.ptr = ctypes.c_void_p()
        rc = self._hip.hipHostMalloc(ctypes.byref(self.ptr), nbytes, 0)
        if rc != 0 or not self.ptr.value:
            self._hip.hipGetLastError()
            self.ptr = ctypes.c_void_p()
            raise MemoryError(f"hipHostMalloc of {nbytes / 2**30:.1f} GiB failed (hipError {rc})")
        self.nbytes = nbytes
        self._raw = (ctypes.c_ubyte * nbytes).from_address(self.ptr.value)

    def tensor(self, dtype, shape) -> torch.Tensor:
        return torch.frombuffer(self._raw, dtype=dtype).view(shape)

    def close(self):
        if self.ptr.value:
            self._raw = None
            self._hip.hipHostFree(self.ptr)
            self.ptr = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class SynthMapStore:
    def __init__(self, w: synth.Workload, device, *, layout: str = "packed", host: bool = False,
                 slice_bytes: int = 8 << 30, log: Optional[Callable[[str], None]] = None):
        self.w = w
        self.device = device
        self.packed = layout == "packed" and w.map_dtype == "bf16"
        L, Hq, S = w.n_layers, w.n_q_heads, w.seq_len
        dt = synth.torch_dtype(w.map_dtype)
        self.tile = ac.packed_tile_elems(S, w.causal) if self.packed else S * S
        shape = (w.n_entries, L, Hq, self.tile) if self.packed else (w.n_entries, L, Hq, S, S)
        self.stored_bytes = w.n_entries * L * Hq * self.tile * (2 if w.map_dtype == "bf16" else 4)
        self.slice_entries = max(1, min(w.n_entries, slice_bytes // w.entry_bytes))
        self._scratch = torch.empty((self.slice_entries, L, Hq, S, S), dtype=dt, device=device)
        self._packed_scratch = None
        self._scratch_slice = -1          # which slice of entries _scratch currently holds
        self._pinned = None
        if host:
            self._pinned = PinnedBuffer(self.stored_bytes)
            self.maps = self._pinned.tensor(dt, shape)
            if self.packed:
                self._packed_scratch = torch.empty((self.slice_entries,) + shape[1:], dtype=dt,
                                                   device=device)
        else:
            self.maps = torch.empty(shape, dtype=dt, device=device)
        t0 = time.time()
        for e0 in range(0, w.n_entries, self.slice_entries):
            e1 = min(w.n_entries, e0 + self.slice_entries)
            n = e1 - e0
            synth.fill_maps(w, self._scratch[:n], first_entry=e0)
            self._scratch_slice = e0
            if self.packed:
                dst = self._packed_scratch[:n] if host else self.maps[e0:e1]
                ac.attncache_pack_maps(self._scratch[:n], dst, causal=w.causal)
                if host:
                    self.maps[e0:e1].copy_(dst)
            else:
                self.maps[e0:e1].copy_(self._scratch[:n])
            torch.cuda.synchronize()
            if log:
                log(f"  maps stored: {e1}/{w.n_entries} ({time.time() - t0:.1f} s)")

    def dense_entry(self, entry: int) -> torch.Tensor:
        """Dense [L,Hq,S,S] maps of one entry, re-drawn from the same seeded slice (on device)."""
        e0 = entry // self.slice_entries * self.slice_entries
        if e0 != self._scratch_slice:
            n = min(self.slice_entries, self.w.n_entries - e0)
            synth.fill_maps(self.w, self._scratch[:n], first_entry=e0)
            self._scratch_slice = e0
        return self._scratch[entry - e0].clone()

    def close(self):
        """Release the pinned host store (the tensor `maps` must not be used afterwards)."""
        if self._pinned is not None:
            self.maps = None
            self._pinned.close()
            self._pinned = None
