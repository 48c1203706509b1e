"""Saved-tensor hooks (phase 4 of the framework, Section 4.4): the slot numbering on the CPU, the
hooks and the device-side stack of containers on the GPU."""
import numpy as np
import pytest
import torch

from paper_2011_09017_amd.autograd import SlotStack


def test_slot_numbers_come_back_in_stack_order():
    s = SlotStack(4)
    a, b, c = s.push(), s.push(), s.push()
    assert (a, b, c) == (0, 1, 2) and s.held == 3
    s.release(b)                    # a hole below the top: its number stays taken
    assert s.held == 3
    s.release(c)                    # top and the hole come back together
    assert s.held == 1 and s.push() == 1
    s.release(1)
    s.release(a)
    assert s.held == 0
    for _ in range(4):
        s.push()
    with pytest.raises(MemoryError):
        s.push()
    with pytest.raises(KeyError):
        s.release(7)
    s.release(2)
    with pytest.raises(KeyError):
        s.release(2)


def _oracle_roundtrip(orc, xh, eb, sub=32):
    rc, buf, size, _ = orc.compress(xh, eb, orc.Config(sub=sub))
    assert rc == 0
    rc, y = orc.decompress(buf, xh.shape, eb, orc.Config(sub=sub))
    assert rc == 0
    return size, y


@pytest.mark.gpu
def test_hooks_compress_conv_inputs_and_restore_the_oracle_reconstruction(orc):
    """A small conv stack: what the backward pass receives is, bit for bit, the oracle's
    reconstruction of what the forward pass saved; the stack is empty afterwards; and the forward
    pass never waits for the GPU."""
    from paper_2011_09017_amd import binding
    from paper_2011_09017_amd.autograd import ActivationCompressor
    torch.manual_seed(2011_09017)
    dev = torch.device("cuda", 0)
    model = torch.nn.Sequential(
        torch.nn.Conv2d(8, 16, 3, padding=1), torch.nn.ReLU(),
        torch.nn.Conv2d(16, 16, 3, padding=1), torch.nn.ReLU(),
        torch.nn.Conv2d(16, 4, 3, padding=1)).to(dev)
    x = torch.randn(4, 8, 32, 32, device=dev)
    eb = 1e-2

    def run(comp):
        model.zero_grad()
        if comp is None:
            loss = model(x).square().mean()
        else:
            before = binding.sync_calls
            with comp.hooks():
                loss = model(x).square().mean()
            assert binding.sync_calls == before, "the forward pass waited for the GPU"
        loss.backward()
        return [p.grad.clone() for p in model.parameters()]

    ref = run(None)
    comp = ActivationCompressor(eb, arena_bytes=8 << 20, max_numel=1 << 20, min_numel=1 << 12)
    comp.skip_parameters(model.parameters())
    seen = []
    comp.on_unpack = lambda p, t: seen.append((p, t.clone()))
    saved = []
    orig_pack = comp.pack

    def spy(t):
        r = orig_pack(t)
        if not isinstance(r, torch.Tensor):
            saved.append((r, t.detach().clone()))
        return r
    comp.pack = spy
    got = run(comp)
    figures = comp.check()

    assert comp.stats["packed"] >= 3                       # the input of every convolution
    assert figures["top"] == 0 and figures["held"] == 0 and comp.stack.held == 0
    originals = {id(p): t for p, t in saved}
    assert len(seen) == len(originals)
    total = 0
    for p, restored in seen:
        xh = originals[id(p)].cpu().numpy()
        size, y = _oracle_roundtrip(orc, xh, eb)
        total += (size + 255) // 256 * 256
        assert np.array_equal(restored.cpu().numpy().view(np.uint32), y.view(np.uint32))
        assert np.abs(y.astype(np.float64) - xh.astype(np.float64)).max() <= float(np.float32(eb))
    # every container was held when the backward pass began: the peak is their sum
    assert figures["peak"] == total and total < comp.stats["raw_bytes"] // 2
    # gradients: finite, and close to those of the uncompressed run (activation error <= eb)
    for g, r in zip(got, ref):
        assert torch.isfinite(g).all()
        assert (g - r).abs().max() <= 0.05 * r.abs().max() + 1e-6


@pytest.mark.gpu
def test_resnet18_shaped_stack_without_host_waits(orc):
    """Seventeen convolutions with the feature-map sizes of the ResNet-18 stream at a small batch:
    no call of the forward pass waits for the GPU, every restored activation is the oracle's
    reconstruction, the stack is empty after the backward pass and its peak is reported."""
    from paper_2011_09017_amd import binding
    from paper_2011_09017_amd.autograd import ActivationCompressor
    torch.manual_seed(17)
    dev = torch.device("cuda", 0)
    layers, cin = [], 3
    plan = [(16, 1)] + [(16, 2)] + [(16, 1)] * 3 + [(32, 2)] + [(32, 1)] * 3 + [(64, 2)] + [(64, 1)] * 3 + [(128, 2)] + [(128, 1)] * 3
    for cout, stride in plan:
        layers += [torch.nn.Conv2d(cin, cout, 3, stride=stride, padding=1), torch.nn.ReLU()]
        cin = cout
    model = torch.nn.Sequential(*layers).to(dev)
    x = torch.randn(2, 3, 224, 224, device=dev)            # 224 -> 112 -> 56 -> 28 -> 14 (-> 7 after the last stride)
    eb = 1e-2
    comp = ActivationCompressor(eb, arena_bytes=64 << 20, max_numel=1 << 22, min_numel=1 << 10)
    comp.skip_parameters(model.parameters())
    pairs = []
    orig_pack = comp.pack

    def spy(t):
        r = orig_pack(t)
        if not isinstance(r, torch.Tensor):
            pairs.append((r, t.detach().clone()))
        return r
    comp.pack = spy
    seen = {}
    comp.on_unpack = lambda p, t: seen.__setitem__(id(p), t.clone())

    before = binding.sync_calls
    with comp.hooks():
        loss = model(x).square().mean()
    assert binding.sync_calls == before, "the forward pass waited for the GPU"
    during = comp.check()
    assert during["held"] == comp.stats["packed"] >= 17 and during["top"] == during["peak"] > 0
    loss.backward()
    after = comp.check()
    assert after["top"] == 0 and after["held"] == 0 and after["peak"] == during["peak"]
    assert after["peak"] < comp.stats["raw_bytes"] // 2
    assert len(seen) == len({id(p) for p, _ in pairs})
    shapes = set()
    for p, t in pairs:
        xh = t.cpu().numpy()
        shapes.add(xh.shape[2])
        _, y = _oracle_roundtrip(orc, xh, eb)
        assert np.array_equal(seen[id(p)].cpu().numpy().view(np.uint32), y.view(np.uint32))
    assert {112, 56, 28, 14} <= shapes
    for prm in model.parameters():
        assert torch.isfinite(prm.grad).all()


@pytest.mark.gpu
def test_stack_overflow_out_of_order_pops_and_second_backward(orc):
    from paper_2011_09017_amd import binding
    from paper_2011_09017_amd.autograd import ActivationCompressor
    from paper_2011_09017_amd.workloads import activation
    dev = torch.device("cuda", 0)
    # raw calls: three pushes, pops out of order, a push that does not fit, an empty slot
    ctx = binding.Context(sub=32, max_numel=1 << 20)
    stream = torch.cuda.current_stream(dev).cuda_stream
    xs = [activation((2, 8, 28, 28), seed=k, device=dev) for k in range(3)]
    _, sizes, _ = ctx.compress_batch(xs, [1e-2] * 3)
    padded = [(s + 255) // 256 * 256 for s in sizes]
    cap = sum(padded) + 512                                  # room for the three, not for a fourth
    arena = torch.zeros(cap, dtype=torch.uint8, device=dev)
    state = torch.zeros(binding.cmp_arena_state_bytes(8), dtype=torch.uint8, device=dev)
    assert binding.cmp_arena_init(ctx._h, state.data_ptr(), 8, stream) == 0
    for k in range(3):
        assert binding.cmp_arena_push(ctx._h, arena.data_ptr(), cap, state.data_ptr(), k, xs[k].data_ptr(), xs[k].shape,
                                      1e-2, stream) == 0
    rc, top, peak, held, failed = binding.cmp_arena_stats(ctx._h, state.data_ptr(), stream)
    assert (rc, top, held, failed) == (0, sum(padded), 3, 0) and peak == top
    assert binding.cmp_arena_push(ctx._h, arena.data_ptr(), cap, state.data_ptr(), 3, xs[0].data_ptr(), xs[0].shape,
                                  1e-2, stream) == 0       # launched; the GPU finds that it does not fit
    rc, top, peak, held, failed = binding.cmp_arena_stats(ctx._h, state.data_ptr(), stream)
    assert rc == binding.CMP_E_NOSPACE and failed == 1 and top == sum(padded)
    assert ctx.last_status() == binding.CMP_E_NOSPACE
    out = torch.empty_like(xs[0])
    # the empty slot pops as a damaged container
    assert binding.cmp_arena_pop(ctx._h, arena.data_ptr(), state.data_ptr(), 3, xs[0].shape, 1e-2, out.data_ptr(), stream) == 0
    assert ctx.last_status() == binding.CMP_E_FORMAT
    # middle first: a hole; then the top: both come back; then the bottom
    for k, want_top in ((1, sum(padded)), (2, padded[0]), (0, 0)):
        assert binding.cmp_arena_pop(ctx._h, arena.data_ptr(), state.data_ptr(), k, xs[k].shape, 1e-2, out.data_ptr(), stream) == 0
        ref = ctx.decompress(ctx.compress(xs[k], 1e-2)[0], sizes[k], xs[k].shape, 1e-2)
        assert torch.equal(out.view(torch.int32), ref.view(torch.int32))
        assert binding.cmp_arena_stats(ctx._h, state.data_ptr(), stream)[1] == want_top
    assert ctx.last_status() == 0
    # shapes the stack does not take
    assert not binding.cmp_arena_accepts(ctx._h, (1, 1, 300, 300)) and binding.cmp_arena_accepts(ctx._h, (1, 1, 300, 256))
    big = torch.zeros((1, 1, 300, 300), device=dev)
    assert binding.cmp_arena_push(ctx._h, arena.data_ptr(), cap, state.data_ptr(), 0, big.data_ptr(), big.shape, 1e-2,
                                  stream) == binding.CMP_E_ARG

    # hooks: a stack too small for the activations is reported by check(); a second backward is refused
    conv = torch.nn.Conv2d(4, 4, 3, padding=1).to(dev)
    x = torch.randn(2, 4, 64, 64, device=dev).relu_()
    comp = ActivationCompressor(1e-2, arena_bytes=4 << 20, max_numel=1 << 20, min_numel=1 << 12)
    comp.skip_parameters(conv.parameters())
    with comp.hooks():
        loss = conv(x).square().mean()
    loss.backward(retain_graph=True)
    assert comp.stats["packed"] >= 1 and comp.check()["top"] == 0
    with pytest.raises(RuntimeError, match="already released"):
        loss.backward()
    tiny = ActivationCompressor(1e-2, arena_bytes=4096, max_numel=1 << 20, min_numel=1 << 12)
    tiny.skip_parameters(conv.parameters())
    with tiny.hooks():
        loss = conv(x).square().mean()
    with pytest.raises(MemoryError):
        tiny.check()
