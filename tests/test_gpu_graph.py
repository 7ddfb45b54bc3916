"""The data calls only enqueue kernels (no allocation, no memset node, no synchronisation), so a serving
loop can record them into a HIP graph.  One offload + fetch cycle is captured and replayed several
times, with eager work and synchronisations between the replays; every replay must reproduce the
eager result (descriptor contents through the oracle, decoded pages bit for bit)."""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as o
from paper_2512_11920_amd import kvc

from gpu_util import DEV, check_pool_invariants, compare_pages_with_oracle

pytestmark = pytest.mark.gpu


def _inputs(seed, nb, ppb, N, d):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((nb, ppb, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)
    x[1, 0] = 0  # an all-zero page
    x[2, 1, 3, 7] = np.float16("nan")  # a RAW page
    return x


def test_offload_fetch_cycle_replays_from_a_graph():
    N, d, ppb, nb, n_seq, k = 16, 128, 4, 96, 4, 6
    max_blocks = nb // n_seq
    rng = np.random.default_rng(9)
    table = torch.from_numpy(rng.permutation(nb).astype(np.int32).reshape(n_seq, max_blocks)).to(DEV)
    pred = torch.from_numpy(rng.integers(0, max_blocks, (n_seq, k)).astype(np.int32)).to(DEV)
    c = kvc.Codec(N, d, ppb, kvc.MODE_RLE)
    c.alloc_pool(nb, nb * ppb * N * d * 2 + 64, DEV)
    cache = torch.empty((nb, ppb, N, d), dtype=torch.float16, device=DEV)  # static input buffer of the graph
    out = torch.empty_like(cache)
    got = torch.empty((n_seq * k, ppb, N, d), dtype=torch.float16, device=DEV)

    def cycle(stream=None):
        c.reset_pool(stream=stream)
        c.compress_blocks(cache, stream=stream)
        c.decompress_blocks(out, stream=stream)
        c.gather_decompress(got, table, pred, 1, nb, stream=stream)

    # eager reference for three different inputs
    xs = [_inputs(100 + i, nb, ppb, N, d) for i in range(3)]
    want = []
    for x in xs:
        cache.copy_(torch.from_numpy(x).to(DEV))
        cycle()
        torch.cuda.synchronize()
        want.append((out.cpu().numpy().view(np.uint16).copy(), got.cpu().numpy().view(np.uint16).copy()))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        cycle()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        cycle()

    for rep in range(4):
        x = xs[rep % 3]
        cache.copy_(torch.from_numpy(x).to(DEV))  # eager work between replays
        out.fill_(7.0)
        got.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        st = c.stats()
        assert st["rc"] == 0 and sum(st["pages"]) == nb * ppb and st["pages"][0] == 1, (rep, st)
        desc = c.desc_numpy()
        check_pool_invariants(desc, st["pool_bytes_used"], c.pool.numel())
        compare_pages_with_oracle(x.view(np.uint16).reshape(-1, N, d), desc, c.pool.cpu().numpy(), N, d, kvc.MODE_RLE)
        w_out, w_got = want[rep % 3]
        assert np.array_equal(out.cpu().numpy().view(np.uint16), w_out), rep
        assert np.array_equal(got.cpu().numpy().view(np.uint16), w_got), rep
        # and the gathered blocks are the decoded pool blocks the table names
        tb, pr = table.cpu().numpy(), pred.cpu().numpy()
        for s in range(n_seq):
            for j in range(k):
                assert np.array_equal(w_got[s * k + j], w_out[tb[s, pr[s, j]]]), (s, j)
    od, op = o.compress_pages(xs[0].view(np.uint16).reshape(-1, N, d), N, d, kvc.MODE_RLE)
    assert np.array_equal(want[0][0].reshape(-1, N, d), o.decompress_pages(op, od, N, d)[0])


def test_two_contexts_on_two_streams_do_not_interfere():
    """Contexts own all their state (cursor, status, statistics): two of them driven from two streams at
    the same time give what each gives alone."""
    N, d, ppb, nb = 16, 128, 8, 512
    xs = [_inputs(300 + i, nb, ppb, N, d) for i in range(2)]
    codecs, caches, outs, streams = [], [], [], [torch.cuda.Stream(), torch.cuda.Stream()]
    for i in range(2):
        c = kvc.Codec(N, d, ppb, (kvc.MODE_RLE, kvc.MODE_CHAN)[i])
        c.alloc_pool(nb, nb * ppb * N * d * 2 + 64, DEV)
        codecs.append(c)
        caches.append(torch.from_numpy(xs[i]).to(DEV))
        outs.append(torch.empty_like(caches[i]))
    torch.cuda.synchronize()
    for rep in range(6):  # interleave the enqueues so the kernels of the two contexts overlap
        for i in range(2):
            codecs[i].reset_pool(stream=streams[i])
            codecs[i].compress_blocks(caches[i], stream=streams[i])
        for i in range(2):
            codecs[i].decompress_blocks(outs[i], stream=streams[i])
    torch.cuda.synchronize()
    for i in range(2):
        scheme = (3, 5)[i]
        st = codecs[i].stats()
        assert st["rc"] == 0 and sum(st["pages"]) == nb * ppb, st
        desc = codecs[i].desc_numpy()
        check_pool_invariants(desc, st["pool_bytes_used"], codecs[i].pool.numel())
        od, op = compare_pages_with_oracle(xs[i].view(np.uint16).reshape(-1, N, d), desc, codecs[i].pool.cpu().numpy(), N, d, scheme)
        want, bad = o.decompress_pages(op, od, N, d)
        assert bad == 0 and np.array_equal(outs[i].cpu().numpy().view(np.uint16).reshape(-1, N, d), want)
