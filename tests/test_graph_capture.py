"""The batch calls under HIP graph capture (Section 4.4: the same compression runs for every layer in
every iteration, so a framework may record it once and replay it).  The calls allocate nothing,
copy nothing and never wait, so a captured graph holds their kernels only; every replay must give
what the eager calls give on the same inputs, and the oracle's bytes."""
import numpy as np
import pytest
import torch


@pytest.mark.gpu
def test_batch_calls_replay_from_a_graph(orc):
    from paper_2011_09017_amd import binding
    from paper_2011_09017_amd.workloads import activation
    dev = torch.device("cuda", 0)
    shapes = [(4, 16, 56, 56), (4, 32, 28, 28), (4, 64, 14, 14), (4, 128, 7, 7), (2, 3, 33, 65)]
    eb = 1e-2
    ebs = [eb] * len(shapes)
    ctx = binding.Context(sub=32, max_numel=1 << 20)
    inputs = [[activation(s, seed=100 * v + k, device=dev) for k, s in enumerate(shapes)] for v in range(3)]
    xs = [torch.empty_like(t) for t in inputs[0]]                  # the tensors the graph reads
    outs = [torch.zeros(ctx.bound(s), dtype=torch.uint8, device=dev) for s in shapes]
    ys = [torch.empty(s, dtype=torch.float32, device=dev) for s in shapes]
    caps = [o.numel() for o in outs]

    def eager(v):
        """Containers (trimmed) and reconstructions of input set v from plain calls."""
        bufs, sizes, rc = ctx.compress_batch(inputs[v], ebs)
        assert rc == 0
        rec = ctx.decompress_batch(bufs, sizes, shapes, ebs)
        torch.cuda.synchronize(dev)
        return [b[:n].clone() for b, n in zip(bufs, sizes)], [r.clone() for r in rec]

    refs = [eager(v) for v in range(3)]

    side = torch.cuda.Stream(dev)
    for a, src in zip(xs, inputs[0]):
        a.copy_(src)
    side.wait_stream(torch.cuda.current_stream(dev))
    with torch.cuda.stream(side):                                  # once eagerly on the stream that will capture
        ctx.compress_batch(xs, ebs, outs, sync=False)
        ctx.decompress_batch(outs, caps, shapes, ebs, ys)
    torch.cuda.current_stream(dev).wait_stream(side)
    torch.cuda.synchronize(dev)

    before = binding.sync_calls
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ctx.compress_batch(xs, ebs, outs, sync=False)
        # the container sizes are not known to the host: the capacity is what is available there
        ctx.decompress_batch(outs, caps, shapes, ebs, ys)
    assert binding.sync_calls == before

    for v in (1, 2, 0, 1):
        for a, src in zip(xs, inputs[v]):
            a.copy_(src)
        for o in outs:
            o.zero_()                                              # eager work between the replays
        graph.replay()
        torch.cuda.synchronize(dev)
        want_bufs, want_rec = refs[v]
        for k in range(len(shapes)):
            n = want_bufs[k].numel()
            assert torch.equal(outs[k][:n], want_bufs[k]), (v, k)
            assert not outs[k][n:n + 64].any()
            assert torch.equal(ys[k].view(torch.int32), want_rec[k].view(torch.int32)), (v, k)
        assert ctx.last_status() == 0
        # an eager call between two replays must not disturb the next one
        ctx.compress(inputs[(v + 1) % 3][0], eb)

    # and the bytes are the oracle's
    xh = inputs[1][4].cpu().numpy()
    rc, obuf, osize, _ = orc.compress(xh, eb, orc.Config(sub=32))
    assert rc == 0
    assert np.array_equal(refs[1][0][4].cpu().numpy(), obuf[:osize])
