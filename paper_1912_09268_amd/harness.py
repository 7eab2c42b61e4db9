"""Device-memory plumbing around the C ABI: allocate the per-layer tensors, the merge arenas and the
pointer tables with torch (ROCm), and hand raw addresses to the binding.  No arithmetic of the
method happens here; torch is used for memory, copies and streams only."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


SENTINEL32 = 0x7FC12345
SENTINEL16 = 0x7FC1


def _torch_dtype(grad_dtype: int):
    return torch.float32 if grad_dtype == B.F32 else torch.int16   # 16-bit gradients travel as raw bit patterns


def _np_view_for_upload(a: np.ndarray) -> np.ndarray:
    return a.view(np.int16) if a.dtype in (np.uint16, np.float16) else a


class DeviceModel:
    """P workers' per-layer gradient tensors, weights, momenta, merge arenas and a reduced arena.

    `misalign` > 0 places every per-layer tensor at an element offset that is not a multiple of
    four inside a slab, to exercise the kernels' under-aligned accesses."""

    def __init__(self, ctx: B.Context, n_elems: Sequence[int], device: str = "cuda:0", misalign: int = 0,
                 fill_arena: bool = False):
        self.ctx = ctx
        self.n_elems = [int(x) for x in n_elems]
        self.L = len(self.n_elems)
        self.P = ctx.P
        self.device = torch.device(device)
        self.gdt = _torch_dtype(ctx.grad_dtype)
        self.misalign = int(misalign)
        self._slabs = []
        self.grads: List[List[torch.Tensor]] = [self._alloc_layers(self.gdt) for _ in range(self.P)]
        self.w = self._alloc_layers(torch.float32)
        self.v = self._alloc_layers(torch.float32)
        arena = max(int(ctx.arena_elems), 1)
        self.merge = [torch.empty(arena, dtype=self.gdt, device=self.device) for _ in range(self.P)]
        self.reduced = torch.empty(arena, dtype=torch.float32, device=self.device)
        if fill_arena:
            self.fill_arenas()
        self.grad_ptrs = self._ptr_table([t for w in self.grads for t in w])
        self.merge_ptrs = self._ptr_table(self.merge)
        self.w_ptrs = self._ptr_table(self.w)
        self.v_ptrs = self._ptr_table(self.v)

    # ---- allocation ------------------------------------------------------------------------
    def _alloc_layers(self, dtype) -> List[torch.Tensor]:
        if self.misalign == 0:
            return [torch.empty(max(n, 0), dtype=dtype, device=self.device) for n in self.n_elems]
        out = []
        for i, n in enumerate(self.n_elems):
            shift = 1 + (i * self.misalign) % 7
            slab = torch.empty(n + 16, dtype=dtype, device=self.device)
            if dtype == torch.float32:
                slab.view(torch.int32).fill_(SENTINEL32)
            else:
                slab.fill_(SENTINEL16)
            self._slabs.append((slab, shift, n))
            out.append(slab[shift:shift + n])
        return out

    def guard_bands_intact(self) -> bool:
        """In misaligned mode every per-layer tensor sits inside a slab with spare elements on both sides,
        pre-filled with a sentinel pattern: True if no call has written there."""
        for slab, shift, n in self._slabs:
            raw = slab.view(torch.int32) if slab.dtype == torch.float32 else slab
            want = SENTINEL32 if slab.dtype == torch.float32 else SENTINEL16
            if not bool((raw[:shift] == want).all()) or not bool((raw[shift + n:] == want).all()):
                return False
        return True

    def _ptr_table(self, tensors: Sequence[torch.Tensor]) -> torch.Tensor:
        addrs = np.asarray([t.data_ptr() for t in tensors] or [0], dtype=np.int64)
        return torch.from_numpy(addrs).to(self.device)

    def fill_arenas(self) -> None:
        """Overwrite the merge and reduced arenas with recognisable NaN bit patterns, so that a test can
        tell which elements a call has written."""
        for m in self.merge:
            if m.dtype == torch.float32:
                m.view(torch.int32).fill_(SENTINEL32)
            else:
                m.fill_(SENTINEL16)
        self.reduced.view(torch.int32).fill_(SENTINEL32)

    # ---- host <-> device -------------------------------------------------------------------
    def _upload_layers(self, layers: List[torch.Tensor], flat: np.ndarray) -> None:
        flat = _np_view_for_upload(np.ascontiguousarray(flat))
        dev = torch.from_numpy(flat).to(self.device)
        pos = 0
        for t, n in zip(layers, self.n_elems):
            if n:
                t.copy_(dev[pos:pos + n])
            pos += n
        del dev

    def upload_grads(self, worker: int, flat: np.ndarray) -> None:
        self._upload_layers(self.grads[worker], flat)

    def upload_weights(self, w_flat: np.ndarray, v_flat: np.ndarray) -> None:
        self._upload_layers(self.w, w_flat)
        self._upload_layers(self.v, v_flat)

    def _download_layers(self, layers: List[torch.Tensor]) -> np.ndarray:
        total = sum(self.n_elems)
        if total == 0:
            return np.zeros(0, np.float32)
        return torch.cat([t.reshape(-1) for t in layers]).cpu().numpy()

    def download_weights(self) -> np.ndarray:
        return self._download_layers(self.w)

    def download_momenta(self) -> np.ndarray:
        return self._download_layers(self.v)

    def download_merge(self, worker: int) -> np.ndarray:
        a = self.merge[worker].cpu().numpy()
        if a.dtype == np.int16:
            return a.view(np.float16) if self.ctx.grad_dtype == B.F16 else a.view(np.uint16)
        return a

    def download_reduced(self) -> np.ndarray:
        return self.reduced.cpu().numpy()

    # ---- the five device calls, on torch's current stream -------------------------------------
    @staticmethod
    def _stream() -> int:
        return int(torch.cuda.current_stream().cuda_stream)

    def pack(self, group: int = -1) -> None:
        self.ctx.pack(group, self.grad_ptrs.data_ptr(), self.merge_ptrs.data_ptr(), self._stream())

    def pack_tensors(self, first_tensor: int, last_tensor: int) -> None:
        self.ctx.pack_tensors(first_tensor, last_tensor, self.grad_ptrs.data_ptr(), self.merge_ptrs.data_ptr(),
                              self._stream())

    def reduce(self, group: int = -1) -> None:
        self.ctx.reduce(group, self.merge_ptrs.data_ptr(), self.reduced.data_ptr(), self._stream())

    def unpack_update(self, lr: float, momentum: float, group: int = -1) -> None:
        self.ctx.unpack_update(group, self.reduced.data_ptr(), self.w_ptrs.data_ptr(), self.v_ptrs.data_ptr(),
                               lr, momentum, self._stream())

    def reduce_update(self, lr: float, momentum: float, group: int = -1) -> None:
        self.ctx.reduce_update(group, self.merge_ptrs.data_ptr(), self.w_ptrs.data_ptr(), self.v_ptrs.data_ptr(),
                               lr, momentum, self._stream())

    def group_pipeline(self, lr: float, momentum: float, group: int = -1, write_reduced: bool = True) -> None:
        self.ctx.group_pipeline(group, self.grad_ptrs.data_ptr(), self.merge_ptrs.data_ptr(),
                                self.reduced.data_ptr() if write_reduced else 0,
                                self.w_ptrs.data_ptr(), self.v_ptrs.data_ptr(), lr, momentum, self._stream())

    def direct_update(self, lr: float, momentum: float, group: int = -1, write_reduced: bool = False) -> None:
        self.ctx.direct_update(group, self.grad_ptrs.data_ptr(), self.reduced.data_ptr() if write_reduced else 0,
                               self.w_ptrs.data_ptr(), self.v_ptrs.data_ptr(), lr, momentum, self._stream())

    def group_pipeline_span(self, lr: float, momentum: float, group_first: int, group_count: int,
                            write_reduced: bool = True) -> None:
        self.ctx.group_pipeline_span(group_first, group_count, self.grad_ptrs.data_ptr(), self.merge_ptrs.data_ptr(),
                                     self.reduced.data_ptr() if write_reduced else 0,
                                     self.w_ptrs.data_ptr(), self.v_ptrs.data_ptr(), lr, momentum, self._stream())

    def group_pipeline_static(self, lr: float, momentum: float, group: int = -1, write_reduced: bool = True) -> None:
        self.ctx.group_pipeline_static(group, self.grad_ptrs.data_ptr(), self.merge_ptrs.data_ptr(),
                                       self.reduced.data_ptr() if write_reduced else 0,
                                       self.w_ptrs.data_ptr(), self.v_ptrs.data_ptr(), lr, momentum, self._stream())

    def handler_replay(self, lr: float, momentum: float, group_ready_s, time_scale: float, streams,
                       write_reduced: bool = False, max_groups_per_launch: int = 0):
        """Blocks until done; `streams` are raw stream handles.  Returns the library's four statistics."""
        return self.ctx.handler_replay(group_ready_s, time_scale, max_groups_per_launch, streams,
                                       self.grad_ptrs.data_ptr(),
                                       self.merge_ptrs.data_ptr(), self.reduced.data_ptr() if write_reduced else 0,
                                       self.w_ptrs.data_ptr(), self.v_ptrs.data_ptr(), lr, momentum)
