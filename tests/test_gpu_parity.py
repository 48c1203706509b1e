"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: bit-exact for symbols, histogram, code lengths, codes, the whole container
and the reconstructed fp32 values; |x - x'| <= eb on every element (Section 2.2);
zeros stay zero (Sections 3.2, 4.4).
"""
import numpy as np
import pytest
import torch

from paper_2011_09017_amd.workloads import WORKLOADS, activation

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2011_09017_amd import binding
    binding.lib()
    return binding


def make_ctx(gpu, **kw):
    kw.setdefault("max_numel", 1 << 22)
    return gpu.Context(**kw)


def check_case(gpu, orc, x_host: np.ndarray, eb: float, ctx, ocfg, stages=True, expect_rc=0):
    """Compress on both sides, compare everything, decompress on both sides, compare."""
    shape = x_host.shape
    x = torch.from_numpy(x_host).cuda()
    buf, size, rc = ctx.compress(x, eb)
    assert rc == expect_rc, gpu.cmp_strerror(rc)
    orc_rc, obuf, osize, ost = orc.compress(x_host, eb, ocfg, want_stages=True)
    assert orc_rc == expect_rc
    if stages:
        sym = ctx.stage(gpu.CMP_STAGE_QUANT_CODES).numpy().view(np.uint16)
        assert np.array_equal(sym, ost.sym), "quant codes differ"
        hist = ctx.stage(gpu.CMP_STAGE_HIST).numpy().view(np.uint32)
        assert np.array_equal(hist, ost.cnt), "histogram differs"
        lens = ctx.stage(gpu.CMP_STAGE_LENS).numpy()
        assert np.array_equal(lens, ost.lens), "code lengths differ"
        codes = ctx.stage(gpu.CMP_STAGE_CODES).numpy().view(np.uint64)
        assert np.array_equal(codes & np.uint64((1 << 56) - 1), ost.codes), "codes differ"
        assert np.array_equal((codes >> np.uint64(56)).astype(np.uint8), ost.lens)
    assert size == osize, (size, osize)
    got = buf[:size].cpu().numpy()
    if not np.array_equal(got, obuf):
        bad = np.nonzero(got != obuf)[0]
        h = orc.parse_header(obuf)
        raise AssertionError(f"container differs at {bad.size} bytes, first {bad[:8]}, header {h}")
    # outlier lists sit inside the container; decode them for an explicit comparison
    h = orc.parse_header(got)
    oi = got[h["off_outl_idx"]:h["off_outl_idx"] + 4 * h["n_outliers"]].view("<u4")
    ov = got[h["off_outl_val"]:h["off_outl_val"] + 4 * h["n_outliers"]].view("<i4")
    assert np.array_equal(oi, ost.outl_idx) and np.array_equal(ov, ost.outl_val)
    if stages:
        assert np.array_equal(ctx.stage(gpu.CMP_STAGE_OUTLIER_IDX).numpy().view(np.uint32), ost.outl_idx)
        assert np.array_equal(ctx.stage(gpu.CMP_STAGE_OUTLIER_VAL).numpy().view(np.int32), ost.outl_val)
    # decompress
    y = ctx.decompress(buf, size, shape, eb)
    assert ctx.last_status() in (0, gpu.CMP_W_RANGE)
    orc_rc, oy = orc.decompress(obuf, shape, eb, ocfg)
    assert orc_rc == 0
    yh = y.cpu().numpy()
    assert np.array_equal(yh.view(np.uint32), oy.view(np.uint32)), "reconstruction differs"
    ok = np.isfinite(x_host) if expect_rc else np.ones(shape, bool)
    if expect_rc == 0:
        assert np.abs(yh.astype(np.float64) - x_host.astype(np.float64)).max(initial=0) <= float(np.float32(eb))
    assert np.all(yh[(x_host == 0) & ok].view(np.uint32) == 0)
    return h


SMALL = [
    # shape, k, p_zero, eb
    ((1, 64, 56, 56), 5, 0.5, 1e-2),        # configs[0]
    ((2, 3, 7, 7), 5, 0.5, 1e-2),
    ((3, 5, 55, 55), 5, 0.5, 1e-3),
    ((1, 2, 224, 224), 5, 0.5, 1e-2),
    ((2, 2, 14, 14), 5, 0.85, 1e-2),
    ((1, 1, 1, 4099), 5, 0.5, 1e-2),
    ((1, 1, 4099, 1), 5, 0.5, 1e-2),
    ((1, 1, 1, 2), 5, 0.5, 1e-2),
    ((7, 1, 1, 1), 5, 0.5, 1e-2),
    ((1, 3, 33, 19), 3, 0.6, 5e-3),
    ((2, 8, 28, 28), 5, 0.5, 1e-1),
    ((1, 1, 300, 1000), 5, 0.5, 1e-2),
    ((5, 7, 13, 3), 3, 0.5, 5e-4),
]


@pytest.mark.parametrize("shape,k,p_zero,eb", SMALL)
def test_small_cases_bit_exact(gpu, orc, shape, k, p_zero, eb):
    ctx = make_ctx(gpu)
    x = activation(shape, k, p_zero, seed=sum(shape)).numpy()
    check_case(gpu, orc, x, eb, ctx, orc.Config())


@pytest.mark.parametrize("sub", [32, 64, 128])
@pytest.mark.parametrize("radius", [512, 16, 1])
def test_sub_and_radius_variants(gpu, orc, sub, radius):
    ctx = make_ctx(gpu, sub=sub, radius=radius)
    x = activation((2, 3, 55, 55), 5, 0.5, seed=sub + radius).numpy()
    h = check_case(gpu, orc, x, 1e-3, ctx, orc.Config(radius=radius, sub=sub))
    if radius < 512:
        assert h["n_outliers"] > 0


@pytest.mark.parametrize("sub", [32, 64, 128])
@pytest.mark.parametrize("shape", [(1, 3, 224, 224), (2, 2, 112, 112), (1, 1, 500, 256), (1, 1, 40, 257),
                                   (1, 1, 300, 300), (3, 300, 7, 7), (1, 2, 129, 63)])
def test_band_and_group_shapes(gpu, orc, sub, shape):
    """Planes larger than one band, groups of small planes, and shapes that take the unfused kernels."""
    ctx = make_ctx(gpu, sub=sub)
    x = activation(shape, 5, 0.5, seed=sub + shape[3]).numpy()
    x[0, 0, shape[2] // 2, shape[3] // 3] = 300.0           # one outlier cluster
    check_case(gpu, orc, x, 1e-2, ctx, orc.Config(sub=sub))


@pytest.mark.parametrize("shape,sub", [((23, 230, 45, 47), 32), ((23, 230, 45, 47), 128), ((11, 500, 70, 33), 32)])
def test_many_large_planes(gpu, orc, shape, sub):
    """Planes larger than one band, and more of them than the chip holds waves: every wave walks
    its own planes band by band (with fewer planes, as in the cases above, the four waves of a
    workgroup share a plane).  Odd sizes: the last band of a plane is short."""
    ctx = make_ctx(gpu, sub=sub, max_numel=int(np.prod(shape)))
    x = activation(shape, 5, 0.5, seed=sub + shape[3]).numpy()
    rng = np.random.default_rng(shape[2])
    for _ in range(40):                                      # a few planes with outliers
        x[rng.integers(shape[0]), rng.integers(shape[1]), rng.integers(shape[2]), rng.integers(shape[3])] = 300.0
    h = check_case(gpu, orc, x, 1e-2, ctx, orc.Config(sub=sub))
    assert h["n_outliers"] > 0


@pytest.mark.parametrize("sub", [32, 64])
def test_items_with_and_without_outliers(gpu, orc, sub):
    """The fast decode kernel hands the planes (or groups of small planes) whose chunks hold
    outliers to the second kernel: planes of both kinds side by side, many listed items, none, and
    the same context again afterwards (the list must be empty again)."""
    ctx = make_ctx(gpu, sub=sub)
    ocfg = orc.Config(sub=sub)
    rng = np.random.default_rng(7 + sub)
    for shape in [(4, 8, 56, 56), (6, 40, 14, 14), (3, 5, 120, 100)]:
        x = activation(shape, 5, 0.5, seed=11 * sub + shape[2]).numpy()
        n, c = shape[0], shape[1]
        for _ in range(max(2, n * c // 5)):                  # spikes in about a fifth of the planes
            x[rng.integers(n), rng.integers(c), rng.integers(shape[2]), rng.integers(shape[3])] = 300.0
        h = check_case(gpu, orc, x, 1e-2, ctx, ocfg)
        assert h["n_outliers"] > 0
        y = activation(shape, 5, 0.5, seed=13 * sub + shape[2]).numpy()      # no outliers at all
        h = check_case(gpu, orc, y, 1e-2, ctx, ocfg)
        assert h["n_outliers"] == 0
        x[:] = 300.0 * (rng.random(shape) < 0.02)            # outliers everywhere
        h = check_case(gpu, orc, x.astype(np.float32), 1e-2, ctx, ocfg)
        assert h["n_outliers"] > 0


def test_all_zero_constant_and_single_symbol(gpu, orc):
    ctx = make_ctx(gpu)
    x = np.zeros((2, 2, 30, 30), np.float32)
    h = check_case(gpu, orc, x, 1e-2, ctx, orc.Config())
    assert h["max_len"] == 1
    x[:] = 3.25
    check_case(gpu, orc, x, 1e-2, ctx, orc.Config())


def test_empty_tensor(gpu, orc):
    ctx = make_ctx(gpu)
    for shape in [(0, 3, 5, 5), (2, 3, 0, 5)]:
        x = np.zeros(shape, np.float32)
        check_case(gpu, orc, x, 1e-2, ctx, orc.Config(), stages=False)


def test_adversarial_values(gpu, orc):
    """Quantiser midpoints, +-0, denormals, the edge of the range, every element an outlier."""
    ctx = make_ctx(gpu)
    _, _, s, r = orc.constants(1e-2)
    k = np.arange(0, 16385, dtype=np.float64)
    v = np.concatenate([(k + 0.5) * float(s), k * float(s)]).astype(np.float32)
    v = np.concatenate([v, np.nextafter(v, np.float32(np.inf)), np.nextafter(v, np.float32(-np.inf))])
    v = np.concatenate([v, -v, np.array([0.0, -0.0, 1e-45, -1e-45, 1e-39], np.float32)])
    v = v[np.abs(v * r) <= np.float32(16384.0)]
    rng = np.random.default_rng(0)
    rng.shuffle(v)
    n = (v.size // (4 * 37 * 41)) * (4 * 37 * 41)
    x = v[:n].reshape(4, -1, 37, 41)
    h = check_case(gpu, orc, x, 1e-2, ctx, orc.Config())
    assert h["n_outliers"] > n // 2


@pytest.mark.parametrize("nsym", [30, 36])
def test_long_codewords(gpu, orc, nsym):
    """Residual counts that follow the Fibonacci numbers give a maximally skewed tree: the longest
    codeword has nsym - 1 bits (29: past the short-code packing of the encoder; 35: past 32 bits)."""
    eb = 1e-2
    _, _, s, _ = orc.constants(eb)
    fib = [1, 1]
    while len(fib) < nsym:
        fib.append(fib[-1] + fib[-2])
    vals = np.array([(k + 1) // 2 * (1 if k % 2 else -1) for k in range(nsym)], np.int64)   # 0, 1, -1, 2, -2, ...
    counts = np.array(fib[::-1], np.int64)                   # residual 0 is the most frequent
    n = int(counts.sum())
    pad = (-n) % 64
    counts[0] += pad
    d = np.repeat(vals, counts)
    np.random.default_rng(nsym).shuffle(d)
    q = np.cumsum(d.reshape(-1, 64), axis=1)                 # rows of 64, one row per plane: 1D Lorenzo
    assert np.abs(q).max() < 16384
    x = (q.astype(np.float32) * np.float32(s)).reshape(1, -1, 1, 64)
    ctx = make_ctx(gpu, max_numel=x.size)
    h = check_case(gpu, orc, x, eb, ctx, orc.Config(), stages=True)
    assert h["max_len"] == nsym - 1


def _rows_from_residuals(d, s, width=64):
    """Planes of one row each (1D Lorenzo): the residual sequence d, `width` per plane, as a tensor."""
    q = np.cumsum(d.reshape(-1, width), axis=1)
    assert np.abs(q).max() < 16384
    return (q.astype(np.float32) * np.float32(s)).reshape(1, -1, 1, width)


@pytest.mark.parametrize("sub", [32, 128])
def test_rare_symbols_in_a_row(gpu, orc, sub):
    """Residual counts 1, 1, 2, 4, ..., 2^19: codewords of up to twenty bits, and the rarest residuals
    next to one another, so that four neighbouring codewords exceed the 64 bits the packing kernel
    merges in registers (its two-by-two path) while no codeword exceeds its short-code limit of 27."""
    eb = 1e-2
    _, _, s, _ = orc.constants(eb)
    vals = [0] + [(k + 1) // 2 * (1 if k % 2 else -1) for k in range(1, 21)]       # 0, 1, -1, 2, -2, ...
    counts = [1 << 19] + [1 << (19 - k) for k in range(1, 20)] + [1]              # sums to 2^20
    assert sum(counts) == 1 << 20
    d = np.repeat(np.array(vals, np.int64), counts)
    head = d[-40:].copy()                                        # the rarest residuals, in a row
    rest = d[:-40]
    np.random.default_rng(7).shuffle(rest)
    d = np.concatenate([rest[:1000], head, rest[1000:]])
    x = _rows_from_residuals(d, s)
    ctx = make_ctx(gpu, sub=sub, max_numel=x.size)
    h = check_case(gpu, orc, x, eb, ctx, orc.Config(sub=sub), stages=True)
    assert 19 <= h["max_len"] <= 27


@pytest.mark.parametrize("nsym,reps", [(1023, 4), (600, 7), (2, 4096), (3, 100)])
def test_flat_histograms(gpu, orc, nsym, reps):
    """Every residual equally often: ties at every step of the Huffman construction, so the
    tie-break (a leaf before an internal node, each queue in its order) decides every length."""
    eb = 1e-2
    _, _, s, _ = orc.constants(eb)
    half = nsym // 2
    vals = np.concatenate([np.arange(-half, 0), np.arange(1, nsym - half + 1)]) if nsym > 3 else np.arange(nsym) - 1
    rng = np.random.default_rng(nsym)
    # pairs (v, -v) keep the running sums of a row small; every value and its negative occur `reps` times
    v = np.repeat(vals, reps)
    rng.shuffle(v)
    d = np.stack([v, -v], axis=1).reshape(-1)
    pad = (-d.size) % 64
    d = np.concatenate([d, np.zeros(pad, np.int64)])
    x = _rows_from_residuals(d, s)
    ctx = make_ctx(gpu, sub=32, max_numel=max(x.size, 4096))
    check_case(gpu, orc, x, eb, ctx, orc.Config(sub=32), stages=True)


def test_nan_inf_out_of_range(gpu, orc):
    ctx = make_ctx(gpu)
    x = activation((1, 4, 40, 40), seed=3).numpy()
    x[0, 0, 3, 3] = np.inf; x[0, 1, 7, 0] = -np.inf; x[0, 2, 0, 0] = np.nan; x[0, 3, 39, 39] = 1e30
    h = check_case(gpu, orc, x, 1e-2, ctx, orc.Config(), expect_rc=gpu.CMP_W_RANGE)
    assert h["range_events"] == 4


def test_nospace_and_argument_errors(gpu, orc):
    ctx = make_ctx(gpu)
    x = torch.from_numpy(activation((1, 4, 40, 40), seed=4).numpy()).cuda()
    buf, size, rc = ctx.compress(x, 1e-2)
    assert rc == 0
    small = torch.zeros(size - 16, dtype=torch.uint8, device="cuda")
    guard = torch.full((4096,), 0xAB, dtype=torch.uint8, device="cuda")
    _, need, rc = ctx.compress(x, 1e-2, out=small)
    assert rc == gpu.CMP_E_NOSPACE and need == size
    assert ctx.last_status() == gpu.CMP_E_NOSPACE and ctx.last_status() == 0
    assert bool((guard == 0xAB).all())
    tiny = torch.zeros(64, dtype=torch.uint8, device="cuda")
    _, _, rc = ctx.compress(x, 1e-2, out=tiny)
    assert rc == gpu.CMP_E_NOSPACE
    for bad_eb in [0.0, -1.0, float("nan"), float("inf"), 2.0 ** -61]:
        with pytest.raises(gpu.CmpError):
            ctx.compress(x, bad_eb)
    with pytest.raises(gpu.CmpError):
        gpu.Context(radius=513)
    with pytest.raises(gpu.CmpError):
        gpu.Context(sub=100)
    big = torch.zeros((1, 1, 2048, 4096), device="cuda")
    with pytest.raises(gpu.CmpError):
        make_ctx(gpu, max_numel=1 << 20).compress(big, 1e-2)


def test_corrupted_containers_are_rejected(gpu, orc):
    ctx = make_ctx(gpu)
    shape = (1, 2, 30, 30)
    xh = activation(shape, seed=9).numpy()
    xh[0, 0, 4, 4] = 200.0
    x = torch.from_numpy(xh).cuda()
    buf, size, rc = ctx.compress(x, 1e-2)
    good = buf[:size].clone()
    fields = [k for k in orc.HDR if k not in ("range_events", "total_bits")]
    for name in fields + ["tail"]:
        bad = good.clone()
        o = 255 if name == "tail" else orc.HDR[name]
        bad[o] ^= 1
        ctx.decompress(bad, size, shape, 1e-2)
        st = ctx.last_status()
        host_rc, _ = orc.decompress(bad.cpu().numpy(), shape, 1e-2)
        assert st in (gpu.CMP_E_FORMAT, gpu.CMP_E_MISMATCH), name
        assert st == host_rc, (name, st, host_rc)
    # caller-side mismatches
    ctx.decompress(good, size, shape, 2e-2); assert ctx.last_status() == gpu.CMP_E_MISMATCH
    ctx.decompress(good, size, (1, 2, 30, 31), 1e-2); assert ctx.last_status() in (gpu.CMP_E_MISMATCH, gpu.CMP_E_FORMAT)
    ctx.decompress(good, size - 16, shape, 1e-2); assert ctx.last_status() == gpu.CMP_E_FORMAT
    with pytest.raises(gpu.CmpError):
        ctx.decompress(good, 100, shape, 1e-2)
    # damaged body: must not crash, and a clean call afterwards still works
    rng = np.random.default_rng(1)
    h = orc.parse_header(good.cpu().numpy())
    for sect in ["off_lens", "off_chunk_off", "off_sub_bits", "off_payload", "off_outl_idx"]:
        bad = good.clone()
        bad[h[sect] + int(rng.integers(0, 8))] ^= 0x10
        ctx.decompress(bad, size, shape, 1e-2)
        ctx.last_status()
    # a chunk whose bit stream is empty although it holds codes: header and tables consistent
    # with a payload of zero units
    for sub in (32, 128):
        c2 = make_ctx(gpu, sub=sub)
        b2, s2, _ = c2.compress(x, 1e-2)
        g2 = b2[:s2].cpu().numpy().copy()
        h2 = orc.parse_header(g2)
        assert h2["n_outliers"] > 0 and h2["nchunks"] == 1
        empty = g2[:h2["off_payload"]].copy()
        empty[h2["off_chunk_off"] + 4:h2["off_chunk_off"] + 8] = 0                 # chunk_off[1] = 0
        empty[h2["off_outl_off"] + 4:h2["off_outl_off"] + 8] = 0                   # no outliers either
        empty[h2["off_sub_bits"]:h2["off_payload"]] = 0
        empty[orc.HDR["n_outliers"]:orc.HDR["n_outliers"] + 4] = 0
        for f in ("off_outl_idx", "off_outl_val", "total_size"):
            empty[orc.HDR[f]:orc.HDR[f] + 8] = np.frombuffer(np.uint64(h2["off_payload"]).tobytes(), np.uint8)
        eb2 = torch.from_numpy(np.concatenate([empty, np.zeros(4096, np.uint8)])).cuda()
        c2.decompress(eb2, empty.size, shape, 1e-2)
        assert c2.last_status() == gpu.CMP_E_FORMAT
    y = ctx.decompress(good, size, shape, 1e-2)
    assert ctx.last_status() == 0
    assert np.abs(y.cpu().numpy() - xh).max() <= 1e-2
    # sizes the 32-bit indexing of the kernels cannot take are refused on the host
    assert ctx.bound((1, 1, 65536, 65536)) == 0 and ctx.bound((1, 1, 1, (1 << 32) - 8191)) == 0
    assert ctx.bound((1, 1, 1, (1 << 32) - 8192)) > 0
    with pytest.raises(gpu.CmpError):
        gpu.Context(max_numel=(1 << 32) - 8191)


def test_determinism_and_context_reuse(gpu, orc):
    ctx = make_ctx(gpu)
    a = torch.from_numpy(activation((2, 4, 56, 56), seed=1).numpy()).cuda()
    b = torch.from_numpy(activation((1, 3, 28, 28), seed=2).numpy()).cuda()
    ba, sa, _ = ctx.compress(a, 1e-2)
    ref = ba[:sa].clone()
    for _ in range(3):
        bb, sb, _ = ctx.compress(b, 5e-3)
        ba2, sa2, _ = ctx.compress(a, 1e-2)
        assert sa2 == sa and torch.equal(ba2[:sa2], ref)
    # recompressing the reconstruction reproduces the same codes (quantiser fixed point)
    y = ctx.decompress(ba, sa, a.shape, 1e-2)
    by, sy, _ = ctx.compress(y, 1e-2)
    y2 = ctx.decompress(by, sy, a.shape, 1e-2)
    assert torch.equal(y.view(torch.int32), y2.view(torch.int32))


FULL = [("cfg2_vgg16_conv1_2", 0), ("cfg3_resnet50_bottleneck", 0), ("cfg4_alexnet_conv1", 0)]


def test_compress_in_two_calls_on_two_streams(gpu, orc):
    """cmp_compress_begin on one stream, cmp_compress_finish on another (ordered by an event): the same
    container as the single call; misuse of the pair is refused."""
    ctx = make_ctx(gpu)
    x = activation((3, 8, 40, 24), 5, 0.5, 424242, device="cuda")
    eb = 1e-2
    ref, ref_size, rc = ctx.compress(x, eb)
    assert rc == 0
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    s1.wait_stream(torch.cuda.current_stream())
    out = torch.zeros_like(ref)
    assert gpu.cmp_compress_finish(ctx._h, out.data_ptr(), out.numel(), False, s2.cuda_stream)[0] == gpu.CMP_E_ARG
    assert gpu.cmp_compress_begin(ctx._h, x.data_ptr(), x.shape, eb, s1.cuda_stream) == 0
    assert gpu.cmp_compress_begin(ctx._h, x.data_ptr(), x.shape, eb, s1.cuda_stream) == gpu.CMP_E_ARG
    assert gpu.cmp_compress(ctx._h, x.data_ptr(), x.shape, eb, out.data_ptr(), out.numel(), False,
                            s1.cuda_stream)[0] == gpu.CMP_E_ARG
    ev = torch.cuda.Event()
    ev.record(s1)
    s2.wait_event(ev)
    rc, size = gpu.cmp_compress_finish(ctx._h, out.data_ptr(), out.numel(), True, s2.cuda_stream)
    assert rc == 0 and size == ref_size
    assert torch.equal(out[:size], ref[:size])
    # too small an output: refused, and the context is clean for the next tensor
    assert gpu.cmp_compress_begin(ctx._h, x.data_ptr(), x.shape, eb, s1.cuda_stream) == 0
    s1.synchronize()
    assert gpu.cmp_compress_finish(ctx._h, out.data_ptr(), 64, False, s1.cuda_stream)[0] == gpu.CMP_E_NOSPACE
    s1.synchronize()
    check_case(gpu, orc, x.cpu().numpy(), eb, ctx, orc.Config())


def full_size_case(gpu, orc, ctx, x, eb, sub, label):
    """Whole container and whole reconstruction of one device tensor against the oracle."""
    xh = x.cpu().numpy()
    ocfg = orc.Config(sub=sub)
    print(f"[parity] {label} eb={eb} sub={sub} numel={xh.size}", flush=True)
    buf, size, rc = ctx.compress(x, eb)
    assert rc == 0
    orc_rc, obuf, osize, _ = orc.compress(xh, eb, ocfg)
    assert orc_rc == 0 and size == osize
    assert np.array_equal(buf[:size].cpu().numpy(), obuf)
    y = ctx.decompress(buf, size, x.shape, eb)
    assert ctx.last_status() == 0
    yh = y.cpu().numpy()
    orc_rc, oy = orc.decompress(obuf, xh.shape, eb, ocfg)
    assert orc_rc == 0 and np.array_equal(yh.view(np.uint32), oy.view(np.uint32))
    assert np.abs(yh.astype(np.float64) - xh.astype(np.float64)).max() <= float(np.float32(eb))
    assert np.all(yh[xh == 0].view(np.uint32) == 0)
    print(f"[parity] ok ratio={xh.nbytes / size:.3f}", flush=True)


@pytest.mark.parametrize("sub", [32, 128])
@pytest.mark.parametrize("name,ti", FULL)
def test_full_size_configs_bit_exact(gpu, orc, name, ti, sub):
    """BASELINE configs 2-4 at full size: whole container and whole reconstruction, byte for byte,
    with the sub-block size the benchmark uses (32) and the library default (128)."""
    wl = WORKLOADS[name]
    ctx = make_ctx(gpu, max_numel=wl.numel(), sub=sub)
    x = wl.tensor(ti, device="cuda")
    for eb in wl.ebs:
        full_size_case(gpu, orc, ctx, x, eb, sub, name)


# config 5 (the benchmarked one): one tensor of each of its five distinct shapes, at batch 256
CFG5_DISTINCT = [0, 1, 5, 9, 13]


@pytest.mark.parametrize("ti", CFG5_DISTINCT)
@pytest.mark.parametrize("name", ["cfg5_resnet18_stream", "cfg5_resnet18_stream_sparse"])
def test_config5_shapes_full_size_bit_exact(gpu, orc, name, ti):
    """The ResNet-18 stream at batch 256, 50 % and 85 % zeros, in the launch configuration the
    benchmark times (sub = 32, context sized for the tensor)."""
    wl = WORKLOADS[name]
    shape = wl.shapes[ti]
    n = shape[0] * shape[1] * shape[2] * shape[3]
    ctx = make_ctx(gpu, max_numel=n, sub=32)
    x = wl.tensor(ti, device="cuda")
    full_size_case(gpu, orc, ctx, x, wl.ebs[0], 32, f"{name}[{ti}] {shape}")


def test_batch_equals_single_calls_equals_oracle(gpu, orc):
    """cmp_compress_batch: container i is what cmp_compress gives for tensor i, and what the oracle
    gives; tensors of different shapes, error bounds and outlier content, an empty one, wide rows
    (the untiled first sweep) and more tensors than one launch group holds."""
    sub = 32
    ocfg = orc.Config(sub=sub)
    shapes = [(2, 8, 56, 56), (3, 16, 28, 28), (4, 32, 14, 14), (8, 64, 7, 7), (1, 2, 112, 112), (0, 3, 5, 5),
              (1, 1, 3, 2000), (1, 1, 1, 1), (2, 3, 55, 55)]
    shapes = shapes + [(1, 4, 9 + k, 11 + k) for k in range(20)]          # 29 tensors: two launch groups
    ebs = [1e-2, 5e-3, 1e-2, 1e-1, 1e-3, 1e-2, 1e-2, 1e-2, 1e-3] + [1e-2] * 20
    xs = []
    for k, shape in enumerate(shapes):
        if int(np.prod(shape)) > 1:
            x = activation(shape, 5, 0.5, seed=900 + k).numpy()
        else:
            x = np.full(shape, 0.5, np.float32)
        if k % 3 == 1 and x.size:
            x.reshape(-1)[x.size // 2] = 25000.0 * ebs[k]                 # an outlier cluster, inside the quantiser's range
        xs.append(torch.from_numpy(x).cuda())
    total = sum(x.numel() for x in xs)
    ctx = make_ctx(gpu, sub=sub, max_numel=total)
    single = make_ctx(gpu, sub=sub, max_numel=max(x.numel() for x in xs))
    for rep in range(2):                                                  # the scratch is clean after a call
        outs, sizes, rc = ctx.compress_batch(xs, ebs)
        assert rc == 0
        for x, eb, out, size in zip(xs, ebs, outs, sizes):
            ref, rsize, rrc = single.compress(x, eb)
            assert rrc == 0 and rsize == size
            assert torch.equal(out[:size], ref[:rsize])
            orc_rc, obuf, osize, _ = orc.compress(x.cpu().numpy(), eb, ocfg)
            assert orc_rc == 0 and osize == size
            assert np.array_equal(out[:size].cpu().numpy(), obuf)
            y = single.decompress(out, size, x.shape, eb)
            assert single.last_status() == 0
            orc_rc, oy = orc.decompress(obuf, x.shape, eb, ocfg)
            assert np.array_equal(y.cpu().numpy().view(np.uint32), oy.view(np.uint32))
        # all containers decoded by one call: the same bits as the single calls and the oracle
        ys = ctx.decompress_batch(outs, sizes, [x.shape for x in xs], ebs)
        assert ctx.last_status() == 0
        for x, eb, out, size, y in zip(xs, ebs, outs, sizes, ys):
            y1 = single.decompress(out, size, x.shape, eb)
            assert torch.equal(y.view(torch.int32), y1.view(torch.int32))
    # a damaged container among them is reported, the others still come out
    dam = [o.clone() for o in outs]
    dam[3][0] ^= 1
    ys2 = ctx.decompress_batch(dam, sizes, [x.shape for x in xs], ebs)
    assert ctx.last_status() == gpu.CMP_E_FORMAT
    for k in (0, 4, 8, 28):
        assert torch.equal(ys2[k].view(torch.int32), ys[k].view(torch.int32))
    # a context smaller than the batch works it off in several groups
    small = make_ctx(gpu, sub=sub, max_numel=max(x.numel() for x in xs))
    outs2, sizes2, rc = small.compress_batch(xs, ebs)
    assert rc == 0 and sizes2 == sizes
    for a, b, n in zip(outs, outs2, sizes):
        assert torch.equal(a[:n], b[:n])
    # one container too small: reported, the others are complete; capacity below the fixed sections: refused
    caps = [o.numel() for o in outs]
    tight = [torch.empty(sizes[k] - 16 if k == 4 else caps[k], dtype=torch.uint8, device="cuda") for k in range(len(xs))]
    _, sizes3, rc = ctx.compress_batch(xs, ebs, outs=tight)
    assert rc == gpu.CMP_E_NOSPACE and sizes3 == sizes
    assert ctx.last_status() == gpu.CMP_E_NOSPACE
    for k in (0, 3, 8, 28):
        assert torch.equal(tight[k][:sizes[k]], outs[k][:sizes[k]])
    tight[2] = torch.empty(64, dtype=torch.uint8, device="cuda")
    _, _, rc = ctx.compress_batch(xs, ebs, outs=tight)
    assert rc == gpu.CMP_E_NOSPACE
    outs4, sizes4, rc = ctx.compress_batch(xs, ebs)                         # and the context is still clean
    assert rc == 0 and sizes4 == sizes and torch.equal(outs4[4][:sizes[4]], outs[4][:sizes[4]])


ZB_CASES = [
    # shape, k, p_zero, eb, sub
    ((2, 8, 56, 56), 5, 0.85, 1e-2, 32), ((2, 8, 56, 56), 5, 0.85, 1e-2, 64), ((2, 8, 56, 56), 5, 0.85, 1e-2, 128),
    ((1, 4, 112, 112), 5, 0.5, 1e-2, 32), ((6, 40, 14, 14), 5, 0.85, 1e-2, 32), ((3, 300, 7, 7), 5, 0.85, 1e-2, 32),
    ((2, 3, 55, 55), 5, 0.85, 1e-3, 64), ((1, 1, 40, 257), 5, 0.85, 1e-2, 32), ((1, 1, 3, 2000), 5, 0.85, 1e-2, 128),
    ((1, 1, 1, 4099), 5, 0.85, 1e-2, 32), ((1, 2, 300, 300), 5, 0.85, 1e-2, 32),
]


@pytest.mark.parametrize("shape,k,p_zero,eb,sub", ZB_CASES)
def test_zero_block_variant_bit_exact(gpu, orc, shape, k, p_zero, eb, sub):
    """Container version 2 (sub-blocks of zero residuals are not coded): every stage, the container and
    the reconstruction against the oracle's; planes with outliers; a tensor of zeros and a constant one."""
    ctx = make_ctx(gpu, sub=sub, zero_blocks=1)
    ocfg = orc.Config(sub=sub, zero_blocks=1)
    x = activation(shape, k, p_zero, seed=sub + shape[3]).numpy()
    h = check_case(gpu, orc, x, eb, ctx, ocfg)
    assert h["version"] == 2
    x[0, 0, shape[2] // 2, shape[3] // 3] = 25000.0 * eb              # an outlier among the zeros
    check_case(gpu, orc, x, eb, ctx, ocfg)
    h = check_case(gpu, orc, np.zeros(shape, np.float32), eb, ctx, ocfg)
    assert h["total_bits"] == 0 and h["max_len"] == 0
    check_case(gpu, orc, np.full(shape, 3.25, np.float32), eb, ctx, ocfg)
    # the two variants do not read each other's containers
    plain = make_ctx(gpu, sub=sub)
    buf, size, _ = ctx.compress(torch.from_numpy(x).cuda(), eb)
    plain.decompress(buf, size, shape, eb)
    assert plain.last_status() == gpu.CMP_E_MISMATCH
    buf, size, _ = plain.compress(torch.from_numpy(x).cuda(), eb)
    ctx.decompress(buf, size, shape, eb)
    assert ctx.last_status() == gpu.CMP_E_MISMATCH


@pytest.mark.parametrize("ti", [0, 13])
def test_zero_block_variant_config5_sparse_full_size(gpu, orc, ti):
    wl = WORKLOADS["cfg5_resnet18_stream_sparse"]
    shape = wl.shapes[ti]
    ctx = make_ctx(gpu, max_numel=shape[0] * shape[1] * shape[2] * shape[3], sub=32, zero_blocks=1)
    x = wl.tensor(ti, device="cuda")
    xh = x.cpu().numpy()
    ocfg = orc.Config(sub=32, zero_blocks=1)
    buf, size, rc = ctx.compress(x, 1e-2)
    assert rc == 0
    orc_rc, obuf, osize, _ = orc.compress(xh, 1e-2, ocfg)
    assert orc_rc == 0 and size == osize and np.array_equal(buf[:size].cpu().numpy(), obuf)
    y = ctx.decompress(buf, size, shape, 1e-2)
    assert ctx.last_status() == 0
    orc_rc, oy = orc.decompress(obuf, shape, 1e-2, ocfg)
    assert orc_rc == 0 and np.array_equal(y.cpu().numpy().view(np.uint32), oy.view(np.uint32))
    print(f"[parity] version 2 {shape}: ratio {xh.nbytes / size:.3f}", flush=True)
