"""ctypes binding of libcmpz.so -- argument marshalling only.

The module-level ``cmp_*`` functions mirror include/cmpz.h one to one (raw device
pointers and sizes).  :class:`Context` is a convenience wrapper that takes torch
tensors for device memory and the current torch stream; every step of the
compression path runs in the library's HIP kernels.  There is no fallback: if
the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcmpz.so")

CMP_OK, CMP_E_ARG, CMP_E_NOSPACE, CMP_E_FORMAT, CMP_E_MISMATCH, CMP_E_HIP, CMP_W_RANGE = 0, -1, -2, -3, -4, -5, 1
CMP_STAGE_QUANT_CODES, CMP_STAGE_HIST, CMP_STAGE_LENS, CMP_STAGE_CODES = 0, 1, 2, 3
CMP_STAGE_OUTLIER_IDX, CMP_STAGE_OUTLIER_VAL = 4, 5
CMP_F_ZERO_BLOCKS = 1

EXPORTS = ["cmp_default_config", "cmp_create", "cmp_destroy", "cmp_bound", "cmp_compress",
           "cmp_compressed_size", "cmp_decompress", "cmp_last_status", "cmp_debug_stage", "cmp_strerror",
           "cmp_profile", "cmp_profile_read", "cmp_default_controller_config", "cmp_estimate_eb",
           "cmp_compress_begin", "cmp_compress_finish", "cmp_compress_batch", "cmp_decompress_batch", "cmp_compress_static",
           "cmp_arena_state_bytes", "cmp_arena_accepts", "cmp_arena_init", "cmp_arena_push", "cmp_arena_pop", "cmp_arena_stats"]


class cmp_controller_config(C.Structure):
    _fields_ = [("sigma_frac", C.c_float), ("a", C.c_float), ("eb_min", C.c_float), ("eb_max", C.c_float)]


class cmp_config(C.Structure):
    _fields_ = [("radius", C.c_uint32), ("chunk", C.c_uint32), ("sub", C.c_uint32),
                ("guard_shift", C.c_uint32), ("max_numel", C.c_uint64), ("flags", C.c_uint32),
                ("reserved", C.c_uint32)]


_lib = None
sync_calls = 0        # calls made through this module that wait for the GPU (for tests of asynchrony)


def lib() -> C.CDLL:
    """Load libcmpz.so (built in-tree by ``python -m paper_2011_09017_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2011_09017_amd.build` "
                "(there is no CPU or PyTorch fallback for the compression path)")
        L = C.CDLL(LIB_PATH)
        vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int
        L.cmp_default_config.argtypes = [vp]; L.cmp_default_config.restype = None
        L.cmp_create.argtypes = [vp, vp, i32]; L.cmp_create.restype = i32
        L.cmp_destroy.argtypes = [vp]; L.cmp_destroy.restype = None
        L.cmp_bound.argtypes = [vp, vp]; L.cmp_bound.restype = sz
        L.cmp_compress.argtypes = [vp, vp, vp, C.c_float, vp, sz, vp, vp]; L.cmp_compress.restype = i32
        L.cmp_compressed_size.argtypes = [vp, vp, vp, vp]; L.cmp_compressed_size.restype = i32
        L.cmp_decompress.argtypes = [vp, vp, sz, vp, C.c_float, vp, vp]; L.cmp_decompress.restype = i32
        L.cmp_last_status.argtypes = [vp, vp]; L.cmp_last_status.restype = i32
        L.cmp_debug_stage.argtypes = [vp, i32, vp, vp]; L.cmp_debug_stage.restype = i32
        L.cmp_strerror.argtypes = [i32]; L.cmp_strerror.restype = C.c_char_p
        L.cmp_compress_batch.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp]; L.cmp_compress_batch.restype = i32
        L.cmp_decompress_batch.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]; L.cmp_decompress_batch.restype = i32
        L.cmp_compress_static.argtypes = [i32, vp, vp, vp, C.c_float, vp, sz, vp]; L.cmp_compress_static.restype = i32
        L.cmp_arena_state_bytes.argtypes = [C.c_uint32]; L.cmp_arena_state_bytes.restype = sz
        L.cmp_arena_accepts.argtypes = [vp, vp]; L.cmp_arena_accepts.restype = i32
        L.cmp_arena_init.argtypes = [vp, vp, C.c_uint32, vp]; L.cmp_arena_init.restype = i32
        L.cmp_arena_push.argtypes = [vp, vp, sz, vp, C.c_uint32, vp, vp, C.c_float, vp]; L.cmp_arena_push.restype = i32
        L.cmp_arena_pop.argtypes = [vp, vp, vp, C.c_uint32, vp, C.c_float, vp, vp]; L.cmp_arena_pop.restype = i32
        L.cmp_arena_stats.argtypes = [vp, vp, vp, vp, vp, vp, vp]; L.cmp_arena_stats.restype = i32
        L.cmp_compress_begin.argtypes = [vp, vp, vp, C.c_float, vp]; L.cmp_compress_begin.restype = i32
        L.cmp_compress_finish.argtypes = [vp, vp, sz, vp, vp]; L.cmp_compress_finish.restype = i32
        L.cmp_default_controller_config.argtypes = [vp]; L.cmp_default_controller_config.restype = None
        L.cmp_estimate_eb.argtypes = [vp, vp, C.c_uint64, vp, C.c_uint64, C.c_uint64, vp, C.c_uint64, vp, vp, vp, vp]
        L.cmp_estimate_eb.restype = i32
        L.cmp_profile.argtypes = [vp, i32]; L.cmp_profile.restype = i32
        L.cmp_profile_read.argtypes = [vp, vp, i32, vp, vp, vp]; L.cmp_profile_read.restype = i32
        _lib = L
    return _lib


def _shape4(shape):
    assert len(shape) == 4
    return (C.c_int64 * 4)(*[int(v) for v in shape])


# --- one-to-one mirrors of the C ABI (raw pointers as ints) -------------------
def cmp_default_config() -> cmp_config:
    cfg = cmp_config()
    lib().cmp_default_config(C.addressof(cfg))
    return cfg


def cmp_create(cfg: cmp_config | None, device: int):
    h = C.c_void_p(0)
    rc = lib().cmp_create(C.addressof(h), C.addressof(cfg) if cfg is not None else None, device)
    return rc, h.value


def cmp_destroy(ctx) -> None:
    lib().cmp_destroy(ctx)


def cmp_bound(ctx, shape) -> int:
    s = _shape4(shape)
    return int(lib().cmp_bound(ctx, C.addressof(s)))


def cmp_compress(ctx, d_x: int, shape, eb: float, d_out: int, out_cap: int, want_size: bool, stream: int):
    global sync_calls
    sync_calls += 1 if want_size else 0
    s = _shape4(shape)
    size = C.c_size_t(0)
    rc = lib().cmp_compress(ctx, d_x, C.addressof(s), C.c_float(eb), d_out, out_cap,
                            C.addressof(size) if want_size else None, stream)
    return rc, int(size.value)


def cmp_compress_batch(ctx, d_xs, shapes, ebs, d_outs, out_caps, want_sizes: bool, stream: int):
    """Lists of raw device pointers / shapes / error bounds / capacities.  Returns (rc, sizes or None)."""
    n = len(d_xs)
    assert len(shapes) == n and len(ebs) == n and len(d_outs) == n and len(out_caps) == n
    xs = (C.c_void_p * n)(*d_xs)
    outs = (C.c_void_p * n)(*d_outs)
    sh = (C.c_int64 * (4 * n))(*[int(v) for s in shapes for v in s])
    eb = (C.c_float * n)(*ebs)
    caps = (C.c_size_t * n)(*out_caps)
    sizes = (C.c_size_t * n)()
    rc = lib().cmp_compress_batch(ctx, n, xs, sh, eb, outs, caps, sizes if want_sizes else None, stream)
    return rc, ([int(v) for v in sizes] if want_sizes else None)


CMP_STATIC_MAX_NUMEL = 1 << 22


def cmp_compress_static(device: int, cfg: "cmp_config | None", d_x: int, shape, eb: float, d_out: int, out_cap: int,
                        stream: int) -> int:
    s = _shape4(shape)
    return lib().cmp_compress_static(device, C.addressof(cfg) if cfg is not None else None, d_x, C.addressof(s),
                                     C.c_float(eb), d_out, out_cap, stream)


def cmp_compressed_size(ctx, d_buf: int, stream: int):
    global sync_calls
    sync_calls += 1
    size = C.c_size_t(0)
    rc = lib().cmp_compressed_size(ctx, d_buf, C.addressof(size), stream)
    return rc, int(size.value)


def cmp_compress_begin(ctx, d_x: int, shape, eb: float, stream: int) -> int:
    s = _shape4(shape)
    return lib().cmp_compress_begin(ctx, d_x, C.addressof(s), C.c_float(eb), stream)


def cmp_compress_finish(ctx, d_out: int, out_cap: int, want_size: bool, stream: int):
    """Returns (rc, size or None)."""
    n = C.c_size_t(0)
    rc = lib().cmp_compress_finish(ctx, d_out, out_cap, C.addressof(n) if want_size else None, stream)
    return rc, (int(n.value) if want_size else None)


def cmp_decompress(ctx, d_buf: int, size: int, shape, eb: float, d_xout: int, stream: int) -> int:
    s = _shape4(shape)
    return lib().cmp_decompress(ctx, d_buf, size, C.addressof(s), C.c_float(eb), d_xout, stream)


def cmp_decompress_batch(ctx, d_bufs, sizes, shapes, ebs, d_xouts, stream: int) -> int:
    n = len(d_bufs)
    assert len(sizes) == n and len(shapes) == n and len(ebs) == n and len(d_xouts) == n
    bufs = (C.c_void_p * n)(*d_bufs)
    outs = (C.c_void_p * n)(*d_xouts)
    sz = (C.c_size_t * n)(*sizes)
    sh = (C.c_int64 * (4 * n))(*[int(v) for s in shapes for v in s])
    eb = (C.c_float * n)(*ebs)
    return lib().cmp_decompress_batch(ctx, n, bufs, sz, sh, eb, outs, stream)


def cmp_arena_state_bytes(slots: int) -> int:
    return int(lib().cmp_arena_state_bytes(slots))


def cmp_arena_accepts(ctx, shape) -> bool:
    s = _shape4(shape)
    return bool(lib().cmp_arena_accepts(ctx, C.addressof(s)))


def cmp_arena_init(ctx, d_state: int, slots: int, stream: int) -> int:
    return lib().cmp_arena_init(ctx, d_state, slots, stream)


def cmp_arena_push(ctx, d_arena: int, arena_cap: int, d_state: int, slot: int, d_x: int, shape, eb: float, stream: int) -> int:
    s = _shape4(shape)
    return lib().cmp_arena_push(ctx, d_arena, arena_cap, d_state, slot, d_x, C.addressof(s), C.c_float(eb), stream)


def cmp_arena_pop(ctx, d_arena: int, d_state: int, slot: int, shape, eb: float, d_xout: int, stream: int) -> int:
    s = _shape4(shape)
    return lib().cmp_arena_pop(ctx, d_arena, d_state, slot, C.addressof(s), C.c_float(eb), d_xout, stream)


def cmp_arena_stats(ctx, d_state: int, stream: int):
    """Waits for the stream.  Returns (rc, top, peak, slots held, pushes failed)."""
    global sync_calls
    sync_calls += 1
    top, peak = C.c_uint64(0), C.c_uint64(0)
    held, failed = C.c_uint32(0), C.c_uint32(0)
    rc = lib().cmp_arena_stats(ctx, d_state, C.addressof(top), C.addressof(peak), C.addressof(held), C.addressof(failed),
                               stream)
    return rc, int(top.value), int(peak.value), int(held.value), int(failed.value)


def cmp_last_status(ctx, stream: int) -> int:
    global sync_calls
    sync_calls += 1
    return lib().cmp_last_status(ctx, stream)


def cmp_debug_stage(ctx, which: int):
    p = C.c_void_p(0)
    n = C.c_size_t(0)
    rc = lib().cmp_debug_stage(ctx, which, C.addressof(p), C.addressof(n))
    return rc, p.value, int(n.value)


def cmp_profile(ctx, enable: bool) -> int:
    return lib().cmp_profile(ctx, 1 if enable else 0)


def cmp_profile_read(ctx, stream: int, cap: int = 32):
    names = (C.c_char_p * cap)()
    ms = (C.c_double * cap)()
    launches = (C.c_uint64 * cap)()
    n = lib().cmp_profile_read(ctx, stream, cap, names, ms, launches)
    if n < 0:
        return n, {}
    return n, {names[k].decode(): (float(ms[k]), int(launches[k])) for k in range(min(n, cap))}


def cmp_estimate_eb(ctx, d_act: int, act_numel: int, d_loss: int, batch_n: int, per_sample: int, d_mom: int,
                    mom_numel: int, cfg: "cmp_controller_config | None", stream: int):
    """Returns (rc, eb, (R, Lbar, Mavg))."""
    eb = C.c_float(0.0)
    stats = (C.c_double * 3)()
    rc = lib().cmp_estimate_eb(ctx, d_act, act_numel, d_loss, batch_n, per_sample, d_mom, mom_numel,
                               C.addressof(cfg) if cfg is not None else None, C.addressof(eb), C.addressof(stats), stream)
    return rc, float(eb.value), (stats[0], stats[1], stats[2])


def cmp_strerror(code: int) -> str:
    return lib().cmp_strerror(code).decode()


class CmpError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {cmp_strerror(code)} ({code})")
        self.code = code


class Context:
    """Owns one cmp_ctx.  Tensors supply device memory; the current torch stream is used."""

    def __init__(self, radius=512, chunk=4096, sub=128, guard_shift=7, max_numel=1 << 28, device=0, zero_blocks=0):
        cfg = cmp_config(radius, chunk, sub, guard_shift, max_numel, CMP_F_ZERO_BLOCKS if zero_blocks else 0, 0)
        rc, self._h = cmp_create(cfg, device)
        if rc != CMP_OK:
            self._h = None
            raise CmpError(rc, "cmp_create")
        self.cfg = cfg
        self.device = torch.device("cuda", device)

    def close(self):
        if getattr(self, "_h", None):
            cmp_destroy(self._h)
            self._h = None

    def __del__(self):
        if cmp_destroy is not None:                  # module globals are gone at interpreter exit
            self.close()

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def bound(self, shape) -> int:
        return cmp_bound(self._h, shape)

    def compress(self, x: torch.Tensor, eb: float, out: torch.Tensor | None = None, sync: bool = True):
        """Returns (container tensor (uint8, full capacity), size or None, rc)."""
        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 4
        if out is None:
            out = torch.empty(self.bound(x.shape), dtype=torch.uint8, device=x.device)
        rc, size = cmp_compress(self._h, x.data_ptr(), x.shape, eb, out.data_ptr(), out.numel(), sync,
                                self._stream())
        if rc < 0 and rc != CMP_E_NOSPACE:
            raise CmpError(rc, "cmp_compress")
        return out, (size if sync else None), rc

    def compress_batch(self, xs, ebs, outs=None, sync: bool = True):
        """Several tensors in one call.  Returns (containers, sizes or None, rc)."""
        for x in xs:
            assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 4
        if outs is None:
            outs = [torch.empty(self.bound(x.shape), dtype=torch.uint8, device=x.device) for x in xs]
        rc, sizes = cmp_compress_batch(self._h, [x.data_ptr() for x in xs], [x.shape for x in xs], list(ebs),
                                       [o.data_ptr() for o in outs], [o.numel() for o in outs], sync, self._stream())
        if rc < 0 and rc != CMP_E_NOSPACE:
            raise CmpError(rc, "cmp_compress_batch")
        return outs, sizes, rc

    def compressed_size(self, buf: torch.Tensor):
        return cmp_compressed_size(self._h, buf.data_ptr(), self._stream())

    def decompress(self, buf: torch.Tensor, size: int, shape, eb: float, out: torch.Tensor | None = None):
        assert buf.is_cuda and buf.dtype == torch.uint8
        if out is None:
            out = torch.empty(tuple(shape), dtype=torch.float32, device=buf.device)
        rc = cmp_decompress(self._h, buf.data_ptr(), size, shape, eb, out.data_ptr(), self._stream())
        if rc != CMP_OK:
            raise CmpError(rc, "cmp_decompress")
        return out

    def decompress_batch(self, bufs, sizes, shapes, ebs, outs=None):
        """Several containers in one call.  Returns the list of reconstructed tensors."""
        if outs is None:
            outs = [torch.empty(tuple(s), dtype=torch.float32, device=b.device) for b, s in zip(bufs, shapes)]
        rc = cmp_decompress_batch(self._h, [b.data_ptr() for b in bufs], list(sizes), list(shapes), list(ebs),
                                  [o.data_ptr() for o in outs], self._stream())
        if rc != CMP_OK:
            raise CmpError(rc, "cmp_decompress_batch")
        return outs

    def estimate_eb(self, act: torch.Tensor, loss: torch.Tensor, mom: torch.Tensor, sigma_frac=0.01, a=0.32,
                    eb_min=1e-6, eb_max=1.0):
        """Sections 4.1-4.3: loss has shape (batch_n, ...).  Returns (rc, eb, (R, Lbar, Mavg))."""
        for t in (act, loss, mom):
            assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
        cfg = cmp_controller_config(sigma_frac, a, eb_min, eb_max)
        batch_n = loss.shape[0]
        rc, eb, stats = cmp_estimate_eb(self._h, act.data_ptr(), act.numel(), loss.data_ptr(), batch_n,
                                        loss.numel() // max(batch_n, 1), mom.data_ptr(), mom.numel(), cfg,
                                        self._stream())
        if rc < 0:
            raise CmpError(rc, "cmp_estimate_eb")
        return rc, eb, stats

    def last_status(self, stream: int | None = None) -> int:
        return cmp_last_status(self._h, self._stream() if stream is None else stream)

    def profile(self, enable: bool) -> None:
        cmp_profile(self._h, enable)

    def profile_read(self, stream: int | None = None) -> dict:
        """{kernel name: (total ms, launches)} since profile(True)."""
        n, d = cmp_profile_read(self._h, self._stream() if stream is None else stream)
        if n < 0:
            raise CmpError(n, "cmp_profile_read")
        return d

    def stage(self, which: int) -> torch.Tensor:
        """Copy of an intermediate result of the last compress (uint8 tensor on the host)."""
        rc, ptr, nbytes = cmp_debug_stage(self._h, which)
        if rc != CMP_OK:
            raise CmpError(rc, "cmp_debug_stage")
        torch.cuda.synchronize(self.device)
        host = torch.empty(nbytes, dtype=torch.uint8)
        if nbytes:
            hip = _hip()
            err = hip.hipMemcpy(C.c_void_p(host.data_ptr()), C.c_void_p(ptr), C.c_size_t(nbytes), 2)
            if err != 0:
                raise RuntimeError(f"hipMemcpy failed: {err}")
        return host


_hiprt = None


def _hip():
    global _hiprt
    if _hiprt is None:
        _hiprt = C.CDLL("libamdhip64.so")
        _hiprt.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        _hiprt.hipMemcpy.restype = C.c_int
    return _hiprt
