"""Activation compression around autograd's saved tensors (phase 4 of the framework, Section 4.4).

The forward pass of a convolutional layer saves its input for the backward pass.  With the hooks
of this module installed, every saved fp32 NCHW activation is replaced by its compressed
container as soon as it is saved (``cmp_arena_push``) and restored when the backward pass asks for
it (``cmp_arena_pop``; data flow of Section 2.1).  The containers live in one device buffer that is
used as a stack: the backward pass consumes activations in the reverse order of the forward pass,
so the memory held at any time is the sum of the containers of the layers not yet differentiated.
Where each container lies is known to the GPU only (it depends on the sizes of those before it),
so neither hook ever waits for the GPU: compression runs behind the forward pass.

Nothing here computes: both hooks marshal arguments for the C ABI.  Parameters, tensors that are
not fp32 4-D CUDA tensors, small tensors and shapes the stack does not take are saved as they are.
"""
from __future__ import annotations

import weakref
from dataclasses import dataclass
from typing import Callable, Iterable, Optional, Union

import torch

from . import binding


class SlotStack:
    """Host mirror of the slot numbering of the device-side stack: slots are numbered in push order,
    and a number is free again once that slot and every slot above it have been released (exact
    for the forward/backward pattern; a release out of order leaves a hole until then)."""

    def __init__(self, capacity: int):
        self.capacity = int(capacity)
        self._live = []

    def push(self) -> int:
        if len(self._live) >= self.capacity:
            raise MemoryError(f"activation stack: more than {self.capacity} tensors held")
        self._live.append(True)
        return len(self._live) - 1

    def release(self, slot: int) -> None:
        if not (0 <= slot < len(self._live)) or not self._live[slot]:
            raise KeyError(slot)
        self._live[slot] = False
        while self._live and not self._live[-1]:
            self._live.pop()

    @property
    def held(self) -> int:
        return len(self._live)


@dataclass
class _Packed:
    """What autograd holds instead of the activation."""
    slot: int
    shape: tuple
    eb: float
    users: int = 1                              # one tensor may be saved by several nodes
    restored: Optional[torch.Tensor] = None     # kept between the first and the last unpack


class ActivationCompressor:
    """saved_tensors_hooks that compress activations.

    eb: the absolute error bound, or a callable ``eb(tensor) -> float`` (the adaptive
        controller of Sections 4.1-4.3 plugs in here).
    arena_bytes: capacity of the container stack on the GPU.
    max_numel: largest activation that will be compressed (sizes the context's scratch).
    min_numel: tensors smaller than this are saved uncompressed.
    slots: most activations held at once.
    """

    def __init__(self, eb: Union[float, Callable[[torch.Tensor], float]], arena_bytes: int, max_numel: int,
                 sub: int = 32, min_numel: int = 1 << 14, device: int = 0, slots: int = 1024):
        self.eb = eb
        self.min_numel = int(min_numel)
        self.max_numel = int(max_numel)
        self.device = torch.device("cuda", device)
        self.ctx = binding.Context(sub=sub, max_numel=self.max_numel, device=device)
        self.capacity = int(arena_bytes) // 256 * 256
        self.buffer = torch.empty(self.capacity, dtype=torch.uint8, device=self.device)
        self.state = torch.empty(binding.cmp_arena_state_bytes(slots), dtype=torch.uint8, device=self.device)
        self.stack = SlotStack(slots)
        rc = binding.cmp_arena_init(self.ctx._h, self.state.data_ptr(), slots, self._stream())
        if rc != binding.CMP_OK:
            raise binding.CmpError(rc, "cmp_arena_init")
        self._skip = set()                      # data pointers never to compress (parameters)
        self._by_tensor = {}                    # (data_ptr, version, shape) -> (weak ref, _Packed), current forward pass
        self.stats = {"packed": 0, "raw_bytes": 0, "passed_through": 0}
        self.on_unpack: Optional[Callable[[_Packed, torch.Tensor], None]] = None    # for tests

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def skip_parameters(self, params: Iterable[torch.Tensor]) -> None:
        for p in params:
            self._skip.add(p.data_ptr())

    # -- hooks -------------------------------------------------------------------------------
    def _wanted(self, t: torch.Tensor) -> bool:
        return (t.is_cuda and t.dtype == torch.float32 and t.dim() == 4 and t.is_contiguous()
                and self.min_numel <= t.numel() <= self.max_numel
                and not isinstance(t, torch.nn.Parameter) and t.data_ptr() not in self._skip
                and binding.cmp_arena_accepts(self.ctx._h, t.shape))

    def pack(self, t: torch.Tensor):
        if not self._wanted(t):
            self.stats["passed_through"] += 1
            return t
        # a tensor saved by several nodes (a ReLU output that is also the next convolution's input)
        # is compressed once; the weak reference tells a live tensor from a recycled address
        key = (t.data_ptr(), t._version, tuple(t.shape))
        hit = self._by_tensor.get(key)
        if hit is not None and hit[0]() is t:
            hit[1].users += 1
            return hit[1]
        eb = float(self.eb(t)) if callable(self.eb) else float(self.eb)
        slot = self.stack.push()
        rc = binding.cmp_arena_push(self.ctx._h, self.buffer.data_ptr(), self.capacity, self.state.data_ptr(), slot,
                                    t.data_ptr(), t.shape, eb, self._stream())        # does not wait
        if rc != binding.CMP_OK:
            self.stack.release(slot)
            raise binding.CmpError(rc, "cmp_arena_push")
        p = _Packed(slot, tuple(t.shape), eb)
        self._by_tensor[key] = (weakref.ref(t), p)
        self.stats["packed"] += 1
        self.stats["raw_bytes"] += 4 * t.numel()
        return p

    def unpack(self, p):
        if not isinstance(p, _Packed):
            return p
        if p.users <= 0:
            # the slot went back when the first saving node took its tensor and the last one
            # dropped it: a second backward over the same graph would read whatever lies there now
            raise RuntimeError("compressed activation already released: a graph whose saved tensors "
                               "were compressed can be walked backward once")
        if p.restored is None:
            out = torch.empty(p.shape, dtype=torch.float32, device=self.device)
            rc = binding.cmp_arena_pop(self.ctx._h, self.buffer.data_ptr(), self.state.data_ptr(), p.slot, p.shape,
                                       p.eb, out.data_ptr(), self._stream())          # decompresses, frees the slot
            if rc != binding.CMP_OK:
                raise binding.CmpError(rc, "cmp_arena_pop")
            self.stack.release(p.slot)
            p.restored = out
            if self.on_unpack is not None:
                self.on_unpack(p, p.restored)
        out = p.restored
        p.users -= 1
        if p.users == 0:
            p.restored = None
        return out

    def hooks(self):
        """Context manager for one forward pass: ``with compressor.hooks(): loss = model(x)``."""
        self._by_tensor = {}
        return torch.autograd.graph.saved_tensors_hooks(self.pack, self.unpack)

    def check(self) -> dict:
        """Waits for the GPU.  Raises if a push did not fit or a pop met a damaged container;
        returns the stack's figures: bytes in use, their peak, slots held, and the status of the
        calls so far (CMP_W_RANGE: some activation lay outside the quantiser's range and was clamped)."""
        rc, top, peak, held, failed = binding.cmp_arena_stats(self.ctx._h, self.state.data_ptr(), self._stream())
        st = self.ctx.last_status()
        if failed:
            raise MemoryError(f"activation stack: {failed} container(s) did not fit into {self.capacity} bytes")
        if st < 0:
            raise binding.CmpError(st, "activation stack")
        return {"top": top, "peak": peak, "held": held, "status": st}
