"""The library's calls can be recorded into a HIP graph (after a first eager call has grown the
scratch buffers: nothing allocates or synchronises afterwards) and replayed: every replay, with new
contents in the same input buffers and eager work in between, gives exactly what the eager calls
give -- statistics included, whose partial records a kernel clears (no memset node in the graph)."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


def test_graph_replays_match_eager(fmt):
    dev = torch.device("cuda")
    f = (6, 9, True)
    rng = np.random.default_rng(11)
    n = 3 * 4096 + 77
    M, N, K = 320, 272, 1088                       # large enough for the single-scaled-piece scheme when forced
    x = torch.empty(n, device=dev)
    A = torch.empty((M, K), device=dev)
    B = torch.empty((N, K), device=dev)
    bias = torch.empty(N, device=dev)
    y = torch.empty_like(x)
    codes = torch.empty(n, dtype=torch.int16, device=dev)
    C = torch.empty((M, N), device=dev)
    Y = torch.empty((M, N), device=dev)
    h1, h2 = fmt.new_hist(dev), fmt.new_hist(dev)

    def fill(seed):
        r = np.random.default_rng(seed)
        x.copy_(torch.from_numpy(workloads.log2_normal(n, -14, 6, 0.01, r)))
        A.copy_(torch.from_numpy(r.standard_normal((M, K)).astype(np.float32)))
        B.copy_(torch.from_numpy((r.standard_normal((N, K)) * 0.02).astype(np.float32)))
        bias.copy_(torch.from_numpy(r.standard_normal(N).astype(np.float32)))

    def calls():
        fmt.fmt_quantize(x, f, out=y, hist=h1)
        fmt.fmt_pack16(x, f, out=codes)
        fmt.fmt_gemm(A, B, f, transB=True, out=C)
        fmt.fmt_linear(A, B, bias, f, out=Y, hist=h2)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (y, codes, C, Y, h1, h2)]

    import os
    old = os.environ.get("FMT_GEMM_WINDOW")
    os.environ["FMT_GEMM_WINDOW"] = "1"            # statistics, scaled product, tail and gated kernels all in the graph
    try:
        fill(0)
        calls()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            calls()                                # eager warm-up on the capture stream: scratch is per stream and grown here
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                calls()
        torch.cuda.current_stream().wait_stream(side)
        for seed in (1, 2, 3):
            fill(seed)
            calls()
            want = snapshot()
            for t in (y, codes, C, Y, h1, h2):
                t.zero_()
            (A @ B.t()).sum().item()               # unrelated eager work and a synchronisation between replays
            graph.replay()
            got = snapshot()
            for g, w, name in zip(got, want, ("quantize", "codes", "gemm", "linear", "hist", "linear hist")):
                assert torch.equal(g.view(torch.int32) if g.dtype == torch.float32 else g,
                                   w.view(torch.int32) if w.dtype == torch.float32 else w), (seed, name)
    finally:
        if old is None:
            os.environ.pop("FMT_GEMM_WINDOW", None)
        else:
            os.environ["FMT_GEMM_WINDOW"] = old


def test_overlapping_calls_on_two_streams(fmt):
    """bench.py issues configuration 4's products round-robin on two streams.  Calls on different
    streams use different scratch (workspaces, partial statistics, the device flag of the scaled-piece
    scheme) and may overlap: interleaved on two streams, many times, they must give exactly the
    results of the same calls issued one after the other."""
    dev = torch.device("cuda")
    f = (6, 9, True)
    rng = np.random.default_rng(5)
    shapes = [(512, 384, 1024), (300, 520, 1100), (1024, 256, 2048), (257, 129, 1031)]
    ops = []
    for (M, N, K) in shapes:
        A = torch.from_numpy(rng.standard_normal((M, K)).astype(np.float32)).to(dev)
        B = torch.from_numpy((rng.standard_normal((N, K)) * 0.02).astype(np.float32)).to(dev)
        x = torch.from_numpy(workloads.log2_normal(M * K, -20, 6, 0.01, rng)).to(dev)
        ops.append((A, B, x))
    import os
    old = os.environ.get("FMT_GEMM_WINDOW")
    os.environ["FMT_GEMM_WINDOW"] = "1"
    try:
        serial = []
        for (A, B, x) in ops:
            h = fmt.new_hist(dev)
            serial.append((fmt.fmt_gemm(A, B, f, transB=True), fmt.fmt_quantize(x, f, hist=h), h))
        torch.cuda.synchronize()
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        for s in streams:
            s.wait_stream(torch.cuda.current_stream())
        for rep in range(10):
            outs = []
            for i, (A, B, x) in enumerate(ops):
                s = streams[(i + rep) % 2]
                with torch.cuda.stream(s):
                    h = fmt.new_hist(dev)
                    outs.append((fmt.fmt_gemm(A, B, f, transB=True, stream=s), fmt.fmt_quantize(x, f, hist=h, stream=s), h))
            torch.cuda.synchronize()
            for (c0, y0, h0), (c1, y1, h1) in zip(serial, outs):
                assert torch.equal(c0.view(torch.int32), c1.view(torch.int32)), rep
                assert torch.equal(y0.view(torch.int32), y1.view(torch.int32)), rep
                assert torch.equal(h0, h1), rep
    finally:
        if old is None:
            os.environ.pop("FMT_GEMM_WINDOW", None)
        else:
            os.environ["FMT_GEMM_WINDOW"] = old


def test_growing_scratch_under_capture_is_refused(fmt):
    """A call that would have to grow the library's scratch while its stream is being captured returns
    FMT_ERR_CAPTURE and launches nothing; the same call outside capture succeeds, and can then be
    captured."""
    dev = torch.device("cuda")
    f = (5, 10, True)
    st = torch.cuda.Stream()
    rng = np.random.default_rng(5)
    small = [torch.from_numpy(rng.standard_normal((64, 64)).astype(np.float32)).to(dev) for _ in range(2)]
    big = [torch.from_numpy(rng.standard_normal((1536, 1536)).astype(np.float32)).to(dev) for _ in range(2)]
    Cs, Cb = torch.empty((64, 64), device=dev), torch.empty((1536, 1536), device=dev)
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        fmt.fmt_gemm(small[0], small[1], f, out=Cs)          # this stream's scratch now fits the small product only
        st.synchronize()
        g = torch.cuda.CUDAGraph()
        status = None
        with torch.cuda.graph(g, stream=st):
            fmt.fmt_gemm(small[0], small[1], f, out=Cs)      # fits: recorded
            try:
                fmt.fmt_gemm(big[0], big[1], f, out=Cb)      # would grow: refused, nothing recorded
            except fmt.FmtError as err:
                status = err.status
        assert status == -8
        want = Cs.clone()
        Cs.zero_()
        g.replay()
        st.synchronize()
        assert torch.equal(Cs, want)
        fmt.fmt_gemm(big[0], big[1], f, out=Cb)              # outside capture the same call grows the scratch
        st.synchronize()
    torch.cuda.synchronize()
    ref = big[0].half().float().double() @ big[1].half().float().double()
    assert torch.linalg.norm(Cb.double() - ref) / torch.linalg.norm(ref) < 1e-5


def test_prepare_and_batch_replays_match_eager(fmt):
    """fmt_quantize_prepare_pair_batch (rounded copies and statistics through library scratch), fmt_prepare_pair_batch and
    fmt_gemm_prepared_batch in a graph: the shared prepare launches, the shared product launch (with a member whose k
    runs in parts through library scratch), the sum of its parts and the shared tail launch, replayed three
    times on new tensor contents, bit for bit what the eager calls give."""
    dev = torch.device("cuda")
    f = (6, 9, True)
    shapes = [(1024, 1024, 512)] * 6 + [(64, 96, 6144), (200, 130, 96)]
    X = [torch.empty((M, K), device=dev) for M, N, K in shapes]
    W = [torch.empty((N, K), device=dev) for M, N, K in shapes]
    C = [torch.empty((M, N), device=dev) for M, N, K in shapes]
    Xq = [torch.empty_like(x) for x in X]
    H = [fmt.new_hist() for _ in X]
    bufs = [(torch.empty(fmt.fmt_operand_bytes(M, K, f), dtype=torch.uint8, device=dev),
             torch.empty(fmt.fmt_operand_bytes(K, M, f), dtype=torch.uint8, device=dev),
             torch.empty(fmt.fmt_operand_bytes(N, K, f), dtype=torch.uint8, device=dev),
             torch.empty(fmt.fmt_operand_bytes(K, N, f), dtype=torch.uint8, device=dev)) for M, N, K in shapes]

    def fill(seed):
        r = np.random.default_rng(seed)
        for x, w in zip(X, W):
            x.copy_(torch.from_numpy(workloads.log2_normal(tuple(x.shape), -20, 6, 0.01, r)))
            w.copy_(torch.from_numpy((r.standard_normal(tuple(w.shape)) * 0.02).astype(np.float32)))

    def calls():
        A = [pair[0] for pair in fmt.fmt_quantize_prepare_pair_batch(X, f, Xq, H, outs=[b[0] for b in bufs],
                                                                     outs_t=[b[1] for b in bufs])]
        B = [pair[0] for pair in fmt.fmt_prepare_pair_batch(W, f, outs=[b[2] for b in bufs], outs_t=[b[3] for b in bufs])]
        fmt.fmt_gemm_prepared_batch(A, B, out=C)

    fill(0)
    calls()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        calls()                                    # eager warm-up on the capture stream: its scratch holds the slabs
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            calls()
    torch.cuda.current_stream().wait_stream(side)
    for seed in (1, 2, 3):
        fill(seed)
        calls()
        torch.cuda.synchronize()
        want = [c.clone() for c in C]
        want_q, want_h = [q.clone() for q in Xq], [h.clone() for h in H]
        for c in C + Xq + H:
            c.zero_()
        (X[0] @ W[0].t()).sum().item()             # unrelated eager work and a synchronisation between replays
        graph.replay()
        torch.cuda.synchronize()
        for i, (g, w) in enumerate(zip(C, want)):
            assert torch.equal(g.view(torch.int32), w.view(torch.int32)), (seed, shapes[i])
        for i in range(len(X)):
            assert torch.equal(Xq[i].view(torch.int32), want_q[i].view(torch.int32)), (seed, i)
            assert torch.equal(H[i], want_h[i]), (seed, i)
