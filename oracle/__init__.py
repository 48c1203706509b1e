"""ctypes access to the CPU oracle (``cmpz_oracle.c``).

TEST INFRASTRUCTURE.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product
package never does, and this package never imports the product.

Every function is a thin marshalling layer over one C function; no arithmetic of
the method happens in Python.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cmpz_oracle.c")
_LIB = os.path.join(_HERE, "libcmpz_oracle.so")

OK, E_ARG, E_NOSPACE, E_FORMAT, E_MISMATCH, E_NOMEM, W_RANGE = 0, -1, -2, -3, -4, -6, 1
HEADER_BYTES = 256
QMAX = 16384

# -O2, no contraction, no fast-math: the fp32 operations must round exactly once.
CFLAGS = ["-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
          "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the path of the shared library."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Config(C.Structure):
    _fields_ = [("radius", C.c_uint32), ("chunk", C.c_uint32), ("sub", C.c_uint32),
                ("guard_shift", C.c_uint32), ("zero_blocks", C.c_uint32)]


class _Stages(C.Structure):
    _fields_ = [("q", C.c_void_p), ("delta", C.c_void_p), ("sym", C.c_void_p),
                ("outl_idx", C.c_void_p), ("outl_val", C.c_void_p), ("cnt", C.c_void_p),
                ("lens", C.c_void_p), ("codes", C.c_void_p), ("n_outliers", C.c_uint64),
                ("range_events", C.c_uint64), ("total_bits", C.c_uint64), ("max_len", C.c_uint32)]


@dataclass
class Config:
    radius: int = 512
    chunk: int = 4096
    sub: int = 128
    guard_shift: int = 7
    zero_blocks: int = 0          # 1: sub-blocks of zero residuals are left out of the bit stream (version 2)

    def c(self) -> _Config:
        return _Config(self.radius, self.chunk, self.sub, self.guard_shift, self.zero_blocks)


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, sz, u32, u64, f32 = C.c_void_p, C.c_size_t, C.c_uint32, C.c_uint64, C.c_float
        L.orc_constants.argtypes = [f32, u32, vp, vp, vp]; L.orc_constants.restype = C.c_int
        L.orc_prequant.argtypes = [vp, sz, f32, vp]; L.orc_prequant.restype = u64
        L.orc_lorenzo2d.argtypes = [vp, sz, sz, sz, vp]; L.orc_lorenzo2d.restype = None
        L.orc_prefix2d.argtypes = [vp, sz, sz, sz, vp]; L.orc_prefix2d.restype = None
        L.orc_prefix2d_definition.argtypes = [vp, sz, sz, sz, vp]; L.orc_prefix2d_definition.restype = None
        L.orc_split.argtypes = [vp, sz, u32, vp, vp, vp]; L.orc_split.restype = u64
        L.orc_histogram.argtypes = [vp, sz, u32, vp]; L.orc_histogram.restype = None
        L.orc_codebook_lengths.argtypes = [vp, u32, vp]; L.orc_codebook_lengths.restype = C.c_int
        L.orc_canonical_codes.argtypes = [vp, u32, vp]; L.orc_canonical_codes.restype = C.c_int
        L.orc_zero_blocks.argtypes = [vp, sz, u32, u32, vp]; L.orc_zero_blocks.restype = None
        L.orc_histogram_coded.argtypes = [vp, sz, u32, u32, vp, vp]; L.orc_histogram_coded.restype = None
        L.orc_bound.argtypes = [vp, vp]; L.orc_bound.restype = sz
        L.orc_compress.argtypes = [vp, vp, f32, vp, vp, sz, vp, vp]; L.orc_compress.restype = C.c_int
        L.orc_decompress.argtypes = [vp, sz, vp, f32, vp, vp]; L.orc_decompress.restype = C.c_int
        L.orc_decode_deltas.argtypes = [vp, sz, vp, vp, vp]; L.orc_decode_deltas.restype = C.c_int
        L.orc_dequant.argtypes = [vp, sz, f32, vp]; L.orc_dequant.restype = None
        L.orc_estimate_eb.argtypes = [vp, sz, vp, sz, sz, vp, sz, vp, vp, vp]; L.orc_estimate_eb.restype = C.c_int
        _lib = L
    return _lib


def _p(a: np.ndarray) -> int:
    return a.ctypes.data


def _shape4(shape) -> np.ndarray:
    s = np.asarray(list(shape), dtype=np.int64)
    assert s.shape == (4,)
    return s


def constants(eb: float, guard_shift: int = 7):
    """C0: returns (rc, eb_in, s, r) as numpy float32 scalars."""
    out = np.zeros(3, dtype=np.float32)
    rc = lib().orc_constants(np.float32(eb), guard_shift, _p(out[0:]), _p(out[1:]), _p(out[2:]))
    return rc, out[0], out[1], out[2]


def prequant(x: np.ndarray, r) -> tuple[np.ndarray, int]:
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.size, dtype=np.int32)
    ev = lib().orc_prequant(_p(x), x.size, np.float32(r), _p(q))
    return q.reshape(x.shape), int(ev)


def dequant(q: np.ndarray, s) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int32)
    x = np.empty(q.size, dtype=np.float32)
    lib().orc_dequant(_p(q), q.size, np.float32(s), _p(x))
    return x.reshape(q.shape)


def lorenzo2d(q: np.ndarray) -> np.ndarray:
    """q has shape (planes, H, W)."""
    q = np.ascontiguousarray(q, dtype=np.int32)
    P, H, W = q.shape
    d = np.empty_like(q)
    lib().orc_lorenzo2d(_p(q), P, H, W, _p(d))
    return d


def prefix2d(delta: np.ndarray, definition: bool = False) -> np.ndarray:
    delta = np.ascontiguousarray(delta, dtype=np.int32)
    P, H, W = delta.shape
    q = np.empty_like(delta)
    f = lib().orc_prefix2d_definition if definition else lib().orc_prefix2d
    f(_p(delta), P, H, W, _p(q))
    return q


def split(delta: np.ndarray, radius: int = 512):
    d = np.ascontiguousarray(delta, dtype=np.int32).reshape(-1)
    sym = np.empty(d.size, dtype=np.uint16)
    oi = np.empty(d.size, dtype=np.uint32)
    ov = np.empty(d.size, dtype=np.int32)
    n = int(lib().orc_split(_p(d), d.size, radius, _p(sym), _p(oi), _p(ov)))
    return sym, oi[:n].copy(), ov[:n].copy()


def histogram(sym: np.ndarray, nsym: int = 1024) -> np.ndarray:
    sym = np.ascontiguousarray(sym, dtype=np.uint16).reshape(-1)
    cnt = np.empty(nsym, dtype=np.uint32)
    lib().orc_histogram(_p(sym), sym.size, nsym, _p(cnt))
    return cnt


def zero_blocks(sym: np.ndarray, radius: int = 512, sub: int = 128) -> np.ndarray:
    """C4'/C6': one flag per sub-block of the linear symbol array, 1 = nothing but the zero residual."""
    sym = np.ascontiguousarray(sym, dtype=np.uint16).reshape(-1)
    flags = np.zeros((sym.size + sub - 1) // sub + 1, dtype=np.uint8)
    lib().orc_zero_blocks(_p(sym), sym.size, radius, sub, _p(flags))
    return flags[:(sym.size + sub - 1) // sub]


def histogram_coded(sym: np.ndarray, flags: np.ndarray, nsym: int = 1024, sub: int = 128) -> np.ndarray:
    sym = np.ascontiguousarray(sym, dtype=np.uint16).reshape(-1)
    flags = np.ascontiguousarray(np.concatenate([flags, [0]]), dtype=np.uint8)
    cnt = np.empty(nsym, dtype=np.uint32)
    lib().orc_histogram_coded(_p(sym), sym.size, nsym, sub, _p(flags), _p(cnt))
    return cnt


def codebook_lengths(cnt: np.ndarray) -> tuple[np.ndarray, int]:
    cnt = np.ascontiguousarray(cnt, dtype=np.uint32)
    lens = np.empty(cnt.size, dtype=np.uint8)
    mx = lib().orc_codebook_lengths(_p(cnt), cnt.size, _p(lens))
    return lens, mx


def canonical_codes(lens: np.ndarray) -> tuple[int, np.ndarray]:
    lens = np.ascontiguousarray(lens, dtype=np.uint8)
    codes = np.empty(lens.size, dtype=np.uint64)
    rc = lib().orc_canonical_codes(_p(lens), lens.size, _p(codes))
    return rc, codes


def bound(shape, cfg: Config = Config()) -> int:
    s = _shape4(shape)
    c = cfg.c()
    return int(lib().orc_bound(_p(s), C.addressof(c)))


@dataclass
class Stages:
    q: np.ndarray
    delta: np.ndarray
    sym: np.ndarray
    outl_idx: np.ndarray
    outl_val: np.ndarray
    cnt: np.ndarray
    lens: np.ndarray
    codes: np.ndarray
    n_outliers: int
    range_events: int
    total_bits: int
    max_len: int


def compress(x: np.ndarray, eb: float, cfg: Config = Config(), cap: int | None = None,
             want_stages: bool = False, shape=None):
    """Returns (rc, container bytes as uint8 array (empty unless rc >= 0), needed size, Stages|None)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    s = _shape4(x.shape if shape is None else shape)
    n = int(np.prod(s))
    c = cfg.c()
    if cap is None:
        cap = bound(s, cfg)
    out = np.zeros(max(cap, 1), dtype=np.uint8)
    size = C.c_size_t(0)
    st = None
    stp = None
    if want_stages:
        nsym = 2 * cfg.radius
        arrs = dict(q=np.zeros(n, np.int32), delta=np.zeros(n, np.int32), sym=np.zeros(n, np.uint16),
                    outl_idx=np.zeros(n, np.uint32), outl_val=np.zeros(n, np.int32),
                    cnt=np.zeros(nsym, np.uint32), lens=np.zeros(nsym, np.uint8),
                    codes=np.zeros(nsym, np.uint64))
        st = _Stages(*[_p(arrs[k]) for k in ("q", "delta", "sym", "outl_idx", "outl_val", "cnt", "lens", "codes")],
                     0, 0, 0, 0)
        stp = C.addressof(st)
    rc = lib().orc_compress(_p(x), _p(s), np.float32(eb), C.addressof(c), _p(out), cap,
                            C.addressof(size), stp)
    stages = None
    if want_stages and rc != E_ARG and rc != E_NOMEM:
        k = int(st.n_outliers)
        stages = Stages(arrs["q"], arrs["delta"], arrs["sym"], arrs["outl_idx"][:k].copy(),
                        arrs["outl_val"][:k].copy(), arrs["cnt"], arrs["lens"], arrs["codes"],
                        k, int(st.range_events), int(st.total_bits), int(st.max_len))
    buf = out[: size.value].copy() if rc >= 0 else np.zeros(0, np.uint8)
    return rc, buf, int(size.value), stages


def decompress(buf: np.ndarray, shape, eb: float, cfg: Config = Config(), size: int | None = None):
    """Returns (rc, x' as float32 array of `shape`)."""
    buf = np.ascontiguousarray(buf, dtype=np.uint8)
    s = _shape4(shape)
    c = cfg.c()
    x = np.zeros([int(v) for v in s], dtype=np.float32)
    rc = lib().orc_decompress(_p(buf), buf.size if size is None else size, _p(s), np.float32(eb),
                              C.addressof(c), _p(x))
    return rc, x


def decode_deltas(buf: np.ndarray, cfg: Config = Config()):
    """Returns (rc, sym u16[numel], delta i32[numel]) decoded from a container."""
    buf = np.ascontiguousarray(buf, dtype=np.uint8)
    numel = int(buf[32:40].view("<u8")[0])
    sym = np.zeros(numel, np.uint16)
    delta = np.zeros(numel, np.int32)
    c = cfg.c()
    rc = lib().orc_decode_deltas(_p(buf), buf.size, C.addressof(c), _p(sym), _p(delta))
    return rc, sym, delta


# Byte offsets of the header fields (container layout, written out here on its own).
HDR = dict(magic=0, version=4, status=8, eb_bits=12, shape=16, numel=32, radius=40, chunk=44,
           sub=48, guard_shift=52, nchunks=56, n_outliers=60, range_events=64, max_len=68,
           total_bits=72, off_lens=80, off_chunk_off=88, off_outl_off=96, off_sub_bits=104,
           off_payload=112, off_outl_idx=120, off_outl_val=128, total_size=136)
_U64 = {"numel", "total_bits", "off_lens", "off_chunk_off", "off_outl_off", "off_sub_bits",
        "off_payload", "off_outl_idx", "off_outl_val", "total_size"}


def parse_header(buf: np.ndarray) -> dict:
    """Decode the 256-byte header into a dict (for tests and reports)."""
    b = np.ascontiguousarray(buf[:HEADER_BYTES], dtype=np.uint8)
    out = {}
    for k, o in HDR.items():
        if k == "magic":
            out[k] = bytes(b[0:4])
        elif k == "shape":
            out[k] = [int(v) for v in b[o:o + 16].view("<u4")]
        elif k in _U64:
            out[k] = int(b[o:o + 8].view("<u8")[0])
        else:
            out[k] = int(b[o:o + 4].view("<u4")[0])
    return out


def estimate_eb(act: np.ndarray, loss: np.ndarray, mom: np.ndarray, sigma_frac=0.01, a=0.32, eb_min=1e-6, eb_max=1.0):
    """Sections 4.1-4.3: loss has shape (batch_n, ...).  Returns (rc, eb as float32, (R, Lbar, Mavg))."""
    act = np.ascontiguousarray(act, dtype=np.float32)
    loss = np.ascontiguousarray(loss, dtype=np.float32)
    mom = np.ascontiguousarray(mom, dtype=np.float32)
    batch_n = loss.shape[0]
    per_sample = loss.size // batch_n if batch_n else 0
    cfg = np.array([sigma_frac, a, eb_min, eb_max], dtype=np.float32)
    eb = np.zeros(1, dtype=np.float32)
    stats = np.zeros(3, dtype=np.float64)
    rc = lib().orc_estimate_eb(_p(act), act.size, _p(loss), batch_n, per_sample, _p(mom), mom.size, _p(cfg), _p(eb),
                               _p(stats))
    return rc, eb[0], tuple(stats)
