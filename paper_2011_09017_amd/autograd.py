"""Activation compression around autograd's saved tensors (phase 4 of the framework, Section 4.4).

The forward pass of a convolutional layer saves its input for the backward pass.  With the hooks
of this module installed, every saved fp32 NCHW activation is replaced by its compressed
container (``cmp_compress``) as soon as it is saved and restored (``cmp_decompress``) when the
backward pass asks for it (data flow of Section 2.1).  The containers live in one arena that is
used as a stack: the backward pass consumes activations in the reverse order of the forward pass,
so the memory held at any time is the sum of the containers of the layers not yet differentiated.

Nothing here computes: both hooks marshal arguments for the C ABI.  Parameters, tensors that are
not fp32 4-D CUDA tensors, and small tensors are saved as they are.
"""
from __future__ import annotations

import weakref
from dataclasses import dataclass
from typing import Callable, Iterable, Optional, Union

import torch

from . import binding


class Arena:
    """Stack allocator over one byte range: blocks are released in any order, space comes back
    when the blocks above it have been released too (exact for the forward/backward pattern)."""

    ALIGN = 256

    def __init__(self, capacity: int):
        self.capacity = int(capacity)
        self.top = 0
        self.peak = 0                          # most bytes held by finished blocks
        self.peak_reserved = 0                 # the same, counting a block's worst-case size while it is being filled
        self._blocks = []                      # [offset, size, live]

    def alloc(self, nbytes: int) -> int:
        size = (int(nbytes) + self.ALIGN - 1) // self.ALIGN * self.ALIGN
        if self.top + size > self.capacity:
            raise MemoryError(f"arena: {self.top} + {size} > {self.capacity} bytes")
        off = self.top
        self._blocks.append([off, size, True])
        self.top += size
        self.peak_reserved = max(self.peak_reserved, self.top)
        return off

    def shrink_last(self, nbytes: int) -> None:
        """Give back the unused tail of the block allocated last."""
        blk = self._blocks[-1]
        size = (int(nbytes) + self.ALIGN - 1) // self.ALIGN * self.ALIGN
        assert blk[2] and size <= blk[1]
        self.top -= blk[1] - size
        blk[1] = size
        self.peak = max(self.peak, self.top)

    def free(self, off: int) -> None:
        for blk in reversed(self._blocks):
            if blk[0] == off and blk[2]:
                blk[2] = False
                break
        else:
            raise KeyError(off)
        while self._blocks and not self._blocks[-1][2]:
            off, size, _ = self._blocks.pop()
            self.top = off

    @property
    def live_bytes(self) -> int:
        return sum(b[1] for b in self._blocks if b[2])


@dataclass
class _Packed:
    """What autograd holds instead of the activation."""
    offset: int
    size: int
    shape: tuple
    eb: float
    users: int = 1                              # one tensor may be saved by several nodes
    restored: Optional[torch.Tensor] = None     # kept between the first and the last unpack


class ActivationCompressor:
    """saved_tensors_hooks that compress activations.

    eb: the absolute error bound, or a callable ``eb(tensor) -> float`` (the adaptive
        controller of Sections 4.1-4.3 plugs in here).
    arena_bytes: capacity of the container arena on the GPU.
    max_numel: largest activation that will be compressed (sizes the context's scratch).
    min_numel: tensors smaller than this are saved uncompressed.
    """

    def __init__(self, eb: Union[float, Callable[[torch.Tensor], float]], arena_bytes: int, max_numel: int,
                 sub: int = 32, min_numel: int = 1 << 14, device: int = 0):
        self.eb = eb
        self.min_numel = int(min_numel)
        self.max_numel = int(max_numel)
        self.device = torch.device("cuda", device)
        self.ctx = binding.Context(sub=sub, max_numel=self.max_numel, device=device)
        self.arena = Arena(arena_bytes)
        self.buffer = torch.empty(self.arena.capacity, dtype=torch.uint8, device=self.device)
        self._skip = set()                      # data pointers never to compress (parameters)
        self._by_tensor = {}                    # (data_ptr, version, shape) -> (weak ref, _Packed), current forward pass
        self.stats = {"packed": 0, "raw_bytes": 0, "container_bytes": 0, "passed_through": 0}
        self.on_unpack: Optional[Callable[[_Packed, torch.Tensor], None]] = None    # for tests

    def skip_parameters(self, params: Iterable[torch.Tensor]) -> None:
        for p in params:
            self._skip.add(p.data_ptr())

    # -- hooks -------------------------------------------------------------------------------
    def _wanted(self, t: torch.Tensor) -> bool:
        return (t.is_cuda and t.dtype == torch.float32 and t.dim() == 4 and t.is_contiguous()
                and self.min_numel <= t.numel() <= self.max_numel
                and not isinstance(t, torch.nn.Parameter) and t.data_ptr() not in self._skip)

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
        cap = self.ctx.bound(t.shape)
        off = self.arena.alloc(cap)
        out = self.buffer[off:off + cap]
        _, size, rc = self.ctx.compress(t, eb, out=out, sync=True)      # the size decides where the next one goes
        if rc not in (binding.CMP_OK, binding.CMP_W_RANGE):
            self.arena.free(off)
            raise binding.CmpError(rc, "cmp_compress")
        self.arena.shrink_last(size)
        p = _Packed(off, size, tuple(t.shape), eb)
        self._by_tensor[key] = (weakref.ref(t), p)
        self.stats["packed"] += 1
        self.stats["raw_bytes"] += 4 * t.numel()
        self.stats["container_bytes"] += size
        return p

    def unpack(self, p):
        if not isinstance(p, _Packed):
            return p
        if p.users <= 0:
            # the arena block went back when the last saving node took its tensor: a second
            # backward over the same graph would read whatever was packed there since
            raise RuntimeError("compressed activation already released: a graph whose saved tensors "
                               "were compressed can be walked backward once")
        if p.restored is None:
            buf = self.buffer[p.offset:p.offset + p.size]
            p.restored = self.ctx.decompress(buf, p.size, p.shape, p.eb)
            if self.on_unpack is not None:
                self.on_unpack(p, p.restored)
        out = p.restored
        p.users -= 1
        if p.users == 0:
            p.restored = None
            self.arena.free(p.offset)
        return out

    def hooks(self):
        """Context manager for one forward pass: ``with compressor.hooks(): loss = model(x)``."""
        self._by_tensor = {}
        return torch.autograd.graph.saved_tensors_hooks(self.pack, self.unpack)
