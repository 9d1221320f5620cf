"""The library's calls only launch kernels on the given stream, so a sequence of them can be
captured in a HIP graph.  Each replay, with new contents in the input buffers, must give what
the same calls give when run eagerly (and therefore what the reference gives: the eager calls
are compared with it bit for bit elsewhere)."""
import numpy as np
import pytest

from paper_2409_02423_amd import workloads

pytestmark = pytest.mark.gpu


def test_captured_sequence_replays_like_eager_calls():
    import torch
    from paper_2409_02423_amd import zc
    zc.lib()
    dev = torch.device("cuda:0")
    rows, cols, rate = 256, 1024, 4
    n = rows * cols
    inputs = [torch.from_numpy(workloads.gradient_lowrank(rows, cols, config=5, index=j)).to(dev) for j in range(4)]
    peer = zc.zc_compress(inputs[3], rate)

    x = torch.empty(n, dtype=torch.float32, device=dev)
    c = torch.empty(zc.zc_compressed_size(n, rate), dtype=torch.uint8, device=dev)
    r = torch.empty_like(c)
    y = torch.empty(n, dtype=torch.float32, device=dev)
    c2 = torch.empty(zc.zc2d_compressed_size(rows, cols, 8), dtype=torch.uint8, device=dev)
    y2 = torch.empty(rows, cols, dtype=torch.float32, device=dev)
    cl = torch.empty(zc.zl_max_compressed_size(n), dtype=torch.uint8, device=dev)
    yl = torch.empty(n, dtype=torch.float32, device=dev)

    def sequence(stream):
        zc.zc_compress(x, rate, d_out=c, stream=stream)
        zc.zc_reduce_compressed([peer, c], n, rate, d_out=r, stream=stream)
        zc.zc_decompress(r, n, rate, d_out=y, stream=stream)
        zc.zc2d_compress(x.view(rows, cols), 8, d_out=c2, stream=stream)
        zc.zc2d_decompress(c2, rows, cols, 8, d_out=y2, stream=stream)
        zc.zl_compress(x, d_out=cl, stream=stream)
        zc.zl_decompress(cl, n, d_out=yl, stream=stream)     # the whole capacity as the buffer: the stream is at its start

    outputs = (c, r, y, c2, y2, yl)
    eager = []
    for inp in inputs[:3]:
        x.copy_(inp)
        sequence(None)
        torch.cuda.synchronize()
        size = zc.zl_stream_bytes(cl)
        eager.append([t.clone() for t in outputs] + [cl[:size].clone()])

    for t in outputs + (cl,):
        t.zero_()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    x.copy_(inputs[0])
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        sequence(side)
    for turn in (1, 2, 0, 2):
        print("graph replay with input", turn, flush=True)
        x.copy_(inputs[turn])
        torch.cuda.synchronize()           # eager work and a synchronisation between the replays
        graph.replay()
        torch.cuda.synchronize()
        size = zc.zl_stream_bytes(cl)
        got = [t for t in outputs] + [cl[:size]]
        for g, w, name in zip(got, eager[turn], ("compress", "reduce", "decompress", "4x4 compress", "4x4 decompress",
                                                  "lossless decompress", "lossless stream")):
            assert g.shape == w.shape and torch.equal(g.view(torch.uint8), w.view(torch.uint8)), (name, turn)
        assert torch.equal(yl.view(torch.int32), inputs[turn].view(torch.int32))
