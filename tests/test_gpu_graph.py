"""GPU: the library's calls recorded into a HIP graph and replayed.

After dq8.init() no call allocates, frees, synchronises or clears memory with a memset node (the error statistics
clear their sums with a small kernel), so a sequence of calls can be captured on a stream and replayed.  Every
replay, with new contents in the same input buffers and eager work and synchronisations between the replays, is
compared with the oracle bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_1511_04561_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dq8():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (select them with -m gpu on a GPU box)")
    from paper_1511_04561_amd import dq8 as mod
    mod.lib()  # a missing library is an error, not a skip
    mod.init()
    oracle.set_threads(16)
    return mod


def bits(t):
    return t.cpu().numpy().tobytes()


def test_exchange_round_recorded_in_a_graph(dq8):
    """Absmax, encode, decode, K-way average, re-encode, the one-call second round and the error statistics of a
    ragged array with block 4096, recorded once and replayed on three different inputs."""
    kind, block, K = 0, 4096, 3
    n = 37 * 4096 + 1234
    nb = oracle.dq8_oracle.n_blocks(n, block)
    f32 = lambda m: torch.empty(m, dtype=torch.float32, device="cuda")
    u8 = lambda m: torch.empty(m, dtype=torch.uint8, device="cuda")
    x = [f32(n) for _ in range(K)]
    amax, dec, mean = f32(nb), f32(n), f32(n)
    codes, scales = [u8(n) for _ in range(K)], [f32(nb) for _ in range(K)]
    rc, rs, fc, fs = u8(n), f32(nb), u8(n), f32(nb)
    stats = torch.empty((nb, 4), dtype=torch.float64, device="cuda")
    means = torch.empty(2, dtype=torch.float64, device="cuda")
    es = f32(nb)

    def round_of_calls():
        dq8.absmax(x[0], block, scales=amax)
        for k in range(K):
            dq8.encode(kind, x[k], block, scales=scales[k], codes=codes[k])
        dq8.decode(kind, codes[0], scales[0], block, out=dec)
        dq8.decode_accumulate_avg(kind, codes, scales, block, out=mean)
        dq8.encode(kind, mean, block, scales=rs, codes=rc)
        dq8.decode_avg_encode(kind, codes, scales, block, scales=fs, codes=fc)
        dq8.error_stats(kind, x[0], block, scales=es, stats=stats, means=means)

    def load(rep):
        host = [workloads.tensor(5, 4, worker=10 * rep + k, limit=n) for k in range(K)]
        for k in range(K):
            x[k].copy_(torch.from_numpy(host[k]))
        return host

    side = torch.cuda.Stream()
    load(0)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        round_of_calls()  # once outside the graph: whatever a first call sets up is set up
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        round_of_calls()
    for rep in range(1, 4):
        host = load(rep)
        for t in (amax, dec, mean, rs, fs, es):
            t.fill_(-1.0)  # eager work between the replays, and nothing left over from the replay before
        for t in (rc, fc):
            t.fill_(0xEE)
        stats.fill_(-1.0)
        means.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        print("graph replay %d" % rep, flush=True)
        enc = [oracle.encode(kind, h, block) for h in host]
        cl, sl = [e[0] for e in enc], [e[1] for e in enc]
        assert bits(amax) == oracle.absmax(host[0], block).tobytes()
        for k in range(K):
            assert bits(codes[k]) == cl[k].tobytes() and bits(scales[k]) == sl[k].tobytes()
        assert bits(dec) == oracle.decode(kind, cl[0], sl[0], block).tobytes()
        want_mean = oracle.decode_accumulate_avg(kind, cl, sl, block)
        assert bits(mean) == want_mean.tobytes()
        want_rc, want_rs = oracle.encode(kind, want_mean, block)
        assert bits(rc) == want_rc.tobytes() and bits(rs) == want_rs.tobytes()
        assert bits(fc) == want_rc.tobytes() and bits(fs) == want_rs.tobytes()
        want_stats, want_means = oracle.error_stats(kind, host[0], block)
        assert bits(es) == sl[0].tobytes()
        got_stats = stats.cpu().numpy()  # counts and maxima exact; the sums are binary64 sums in an order that is not fixed
        assert np.array_equal(got_stats[:, 2:], want_stats[:, 2:])
        assert np.allclose(got_stats[:, :2], want_stats[:, :2], rtol=1e-12, atol=0)
        assert np.allclose(means.cpu().numpy(), want_means, rtol=1e-12, atol=0)


def test_per_tensor_passes_recorded_in_a_graph(dq8):
    """The small convnet gradient set, one scale per tensor: the ten encode calls and the ten decode calls as one
    graph, replayed on new gradients."""
    shapes = [t.size for _, t in workloads.tensors(2)]
    xs = [torch.empty(m, dtype=torch.float32, device="cuda") for m in shapes]
    cs = [torch.empty(m, dtype=torch.uint8, device="cuda") for m in shapes]
    ss = [torch.empty(1, dtype=torch.float32, device="cuda") for _ in shapes]
    outs = [torch.empty(m, dtype=torch.float32, device="cuda") for m in shapes]

    def passes(kind):
        for x, c, s in zip(xs, cs, ss):
            dq8.encode(kind, x, 0, scales=s, codes=c)
        for c, s, o in zip(cs, ss, outs):
            dq8.decode(kind, c, s, 0, out=o)

    side = torch.cuda.Stream()
    for kind in (0, 1, 2):
        for x in xs:
            x.zero_()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            passes(kind)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            passes(kind)
        for rep in range(1, 3):
            host = [t for _, t in workloads.tensors(2, worker=rep)]
            for x, h in zip(xs, host):
                x.copy_(torch.from_numpy(h))
            for o in outs:
                o.fill_(-1.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for h, c, s, o in zip(host, cs, ss, outs):
                want_c, want_s = oracle.encode(kind, h, 0)
                assert bits(c) == want_c.tobytes() and bits(s) == want_s.tobytes()
                assert bits(o) == oracle.decode(kind, want_c, want_s, 0).tobytes()


def test_segment_calls_recorded_in_a_graph(dq8):
    """The MLP's gradient set as one array with one scale per tensor: compression (zero fill, maxima, codes) and
    decompression recorded once and replayed on new gradients."""
    sizes = [t.size for _, t in workloads.tensors(1)]
    bounds = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n = int(bounds[-1])
    bd = torch.from_numpy(bounds).cuda()
    x = torch.zeros(n, dtype=torch.float32, device="cuda")
    codes = torch.empty(n, dtype=torch.uint8, device="cuda")
    scales = torch.empty(len(sizes), dtype=torch.float32, device="cuda")
    out = torch.empty(n, dtype=torch.float32, device="cuda")

    def calls():
        dq8.encode_segments(0, x, bd, scales=scales, codes=codes)
        dq8.decode_segments(0, codes, scales, bd, out=out)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls()
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        calls()
    for rep in range(1, 4):
        host = np.concatenate([t for _, t in workloads.tensors(1, worker=rep)])
        x.copy_(torch.from_numpy(host))
        scales.fill_(7.0)  # the maxima are merged into zeroed scales: the zero fill has to be part of every replay
        codes.fill_(0xEE)
        out.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_c, want_s = oracle.encode_segments(0, host, bounds)
        assert bits(scales) == want_s.tobytes() and bits(codes) == want_c.tobytes()
        assert bits(out) == oracle.decode_segments(0, want_c, want_s, bounds).tobytes()
