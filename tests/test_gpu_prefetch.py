"""GPU parity of the prefetch path (kvc_prefetch_layers) against the plain model of Algorithm 1 plus the
codec oracle: plan arrays bit-exact at every step, buffer contents equal to the oracle's decode wherever
`loc` points, untouched slots untouched."""
import numpy as np
import pytest
import torch

from oracle import kvc_oracle as o
from oracle import prefetch_model as pm
from paper_2512_11920_amd import kvc, synth
from gpu_util import DEV, gpu_compress

pytestmark = pytest.mark.gpu


def _say(m):
    print(m, flush=True)


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("with_l1", [False, True])
def test_prefetch_steps_match_model(with_l1, policy):
    rng = np.random.default_rng(5)
    N, d, ppb, n_layers = 16, 128, 4, 3
    pat = synth.gather_pattern(n_seq=6, k=8, len_lo=48, len_hi=200, seed=11)  # few blocks: many re-predictions
    pbl, n_seq, k = pat.pool_blocks_per_layer, pat.n_seq, pat.k
    x = (rng.standard_normal((n_layers * pbl, ppb, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)
    c, _ = gpu_compress(x, N, d, ppb, 3)
    od, op = o.compress_pages(x.view(np.uint16), N, d, 3, n_threads=8)
    full = o.decompress_pages(op, od, N, d, n_threads=8)[0].reshape(n_layers * pbl, ppb, N, d)
    n_slots = n_layers * n_seq * k
    l2 = torch.full((2 * n_slots, ppb, N, d), 5.0, dtype=torch.float16, device=DEV)
    tags = torch.empty(2 * n_slots, dtype=torch.int32, device=DEV)
    fetch = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    loc = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    c.prefetch_reset(tags, n_seq, k, n_layers)
    c.set_prefetch_policy(policy)
    model_step = pm.prefetch_step_reuse if policy else pm.prefetch_step
    table = torch.from_numpy(pat.block_table).to(DEV)
    l1_np = np.maximum(pat.n_blocks - 2, 0).astype(np.int32) if with_l1 else None
    l1 = torch.from_numpy(l1_np).to(DEV) if with_l1 else None
    m_tags = np.full((2, n_layers, n_seq, k), -1, np.int32)
    m_content = np.full((2 * n_slots, ppb, N, d), np.float16(5.0).view(np.uint16), np.uint16)
    n_fetch = 0
    for step in range(12):
        fill = step % 2
        pred_np = pat.predictions(step).copy()
        if step == 3:
            pred_np[1, 2] = -1
        _say(f"[case] prefetch step {step} fill {fill} l1 {with_l1}")
        # two calls over disjoint layer ranges, as the layer pipeline issues them
        for lo, hi in ((0, 1), (1, n_layers)):
            c.prefetch_layers(l2, tags, fetch, loc, table, torch.from_numpy(pred_np).to(DEV), n_layers, pbl, fill,
                              layer_begin=lo, layer_end=hi, l1_first=l1)
        m_fetch, m_loc, bad = model_step(m_tags, fill, pat.block_table, pred_np, l1_np, n_layers, pbl)
        assert not bad
        assert np.array_equal(tags.cpu().numpy(), m_tags.reshape(-1))
        assert np.array_equal(fetch.cpu().numpy(), m_fetch.reshape(-1))
        assert np.array_equal(loc.cpu().numpy(), m_loc.reshape(-1))
        for slot in np.nonzero(m_fetch.reshape(-1) >= 0)[0]:
            m_content[fill * n_slots + slot] = full[m_fetch.reshape(-1)[slot]]
            n_fetch += 1
        got = l2.cpu().numpy().view(np.uint16)
        assert np.array_equal(got, m_content), "L2 buffer differs from the model"
        # what the consumer reads is the oracle's decode of the predicted block
        for l in range(n_layers):
            for s in range(n_seq):
                for j in range(k):
                    w = m_loc[l, s, j]
                    if w >= 0:
                        assert np.array_equal(got[w], full[l * pbl + pat.block_table[s, pred_np[s, j]]])
    assert 0 < n_fetch < 12 * n_slots
    assert c.stats()["status"] == 0


def test_prefetch_bad_index_sets_status():
    N, d, ppb = 16, 128, 2
    rng = np.random.default_rng(6)
    pat = synth.gather_pattern(n_seq=3, k=4, len_lo=40, len_hi=90, seed=2)
    pbl = pat.pool_blocks_per_layer
    x = rng.standard_normal((pbl, ppb, N, d)).astype(np.float16)
    c, _ = gpu_compress(x, N, d, ppb, 3)
    n_slots = pat.n_seq * pat.k
    l2 = torch.zeros((2 * n_slots, ppb, N, d), dtype=torch.float16, device=DEV)
    tags = torch.empty(2 * n_slots, dtype=torch.int32, device=DEV)
    fetch = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    loc = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    c.prefetch_reset(tags, pat.n_seq, pat.k, 1)
    pred = pat.predictions(0).copy()
    pred[2, 1] = pat.max_blocks + 1
    c.prefetch_layers(l2, tags, fetch, loc, torch.from_numpy(pat.block_table).to(DEV), torch.from_numpy(pred).to(DEV), 1, pbl, 0)
    st = c.stats()
    assert st["status"] & kvc.ST_BAD_INDEX
    assert loc.cpu().numpy().reshape(pat.n_seq, pat.k)[2, 1] == -1
    with pytest.raises(kvc.KvcError):
        c.prefetch_layers(l2, tags, fetch, loc, torch.from_numpy(pat.block_table).to(DEV), torch.from_numpy(pred).to(DEV), 1, pbl, 2)


def _plan_on_gpu(policy, tags_np, fill, table_np, pred_np, n_layers, pbl):
    """One planner + fetch step on small hand-made tables: -> (fetch, loc, tags after, codec)."""
    N, d, ppb = 16, 128, 1
    rng = np.random.default_rng(77)
    x = rng.standard_normal((n_layers * pbl, ppb, N, d)).astype(np.float16)
    c, _ = gpu_compress(x, N, d, ppb, 3)
    c.set_prefetch_policy(policy)
    n_seq, k = pred_np.shape
    n_slots = n_layers * n_seq * k
    l2 = torch.zeros((2 * n_slots, ppb, N, d), dtype=torch.float16, device=DEV)
    tags = torch.from_numpy(np.ascontiguousarray(tags_np, np.int32).reshape(-1)).to(DEV)
    fetch = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    loc = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    c.prefetch_layers(l2, tags, fetch, loc, torch.from_numpy(table_np).to(DEV), torch.from_numpy(pred_np).to(DEV), n_layers, pbl, fill)
    torch.cuda.synchronize()
    return (fetch.cpu().numpy().reshape(n_layers, n_seq, k), loc.cpu().numpy().reshape(n_layers, n_seq, k),
            tags.cpu().numpy().reshape(2, n_layers, n_seq, k), c)


@pytest.mark.parametrize("policy", [0, 1])
def test_hand_counted_plans_boundary_entry(policy):
    """The same hand-counted case as the model's pin: table entries 6 (the last valid block of a 7-block
    layer), 7 and 9; two layers."""
    table = np.array([[6, 7, 9]], np.int32)
    pred = np.array([[0, 1, 2]], np.int32)
    f, l, _, c = _plan_on_gpu(policy, np.full((2, 2, 1, 3), -1), 0, table, pred, 2, 7)
    assert f[:, 0].tolist() == [[6, -1, -1], [13, -1, -1]] and l[:, 0].tolist() == [[0, -1, -1], [3, -1, -1]]
    assert c.stats()["status"] & kvc.ST_BAD_INDEX


@pytest.mark.parametrize("policy", [0, 1])
def test_hand_counted_plan_unmapped_logical_block(policy):
    """The model's hand-counted case: a table entry of -1 is skipped and is no error."""
    f, l, t, c = _plan_on_gpu(policy, np.full((2, 1, 1, 2), -1), 0, np.array([[4, -1]], np.int32), np.array([[0, 1]], np.int32), 1, 8)
    assert f[0, 0].tolist() == [4, -1] and l[0, 0].tolist() == [0, -1] and t[0, 0, 0].tolist() == [4, -1]
    assert c.stats()["status"] == 0


def test_hand_counted_plan_slot_reuse_with_a_block_held_twice():
    """The model's hand-counted cases: the half being filled holds a block twice; only its first copy is kept."""
    table = np.array([[4, 5]], np.int32)
    tags = np.full((2, 1, 1, 2), -1, np.int32)
    tags[0, 0, 0] = [4, 4]
    f, l, t, c = _plan_on_gpu(1, tags, 0, table, np.array([[0, 1]], np.int32), 1, 8)
    assert f[0, 0].tolist() == [-1, 5] and l[0, 0].tolist() == [0, 1] and t[0, 0, 0].tolist() == [4, 5]
    assert c.stats()["status"] == 0
    table = np.array([[4, 5, 6, 7]], np.int32)
    tags = np.full((2, 1, 1, 3), -1, np.int32)
    tags[1, 0, 0] = [4, 4, 6]
    f, l, t, c = _plan_on_gpu(1, tags, 1, table, np.array([[1, 0, 3]], np.int32), 1, 8)
    assert f[0, 0].tolist() == [-1, 5, 7] and l[0, 0].tolist() == [4, 3, 5] and t[1, 0, 0].tolist() == [4, 5, 7]
    assert c.stats()["status"] == 0


def test_hip_graph_replays_match_eager():
    """The codec's launches are capturable: one graph holds reset + compress + decompress + a prefetch step
    on two streams.  It is replayed several times with eager work and synchronisations in between and
    every replay is compared with the eager result (no memset nodes: the library clears with fill kernels)."""
    rng = np.random.default_rng(8)
    N, d, ppb, n_layers = 16, 128, 4, 2
    pat = synth.gather_pattern(n_seq=4, k=4, len_lo=48, len_hi=160, seed=5)
    pbl, n_seq, k = pat.pool_blocks_per_layer, pat.n_seq, pat.k
    nb = n_layers * pbl
    x = torch.from_numpy((rng.standard_normal((nb, ppb, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)).to(DEV)
    c = kvc.Codec(N, d, ppb, 3)
    c.alloc_pool(nb, nb * ppb * N * d + 4096, DEV)
    out = torch.zeros_like(x)
    n_slots = n_layers * n_seq * k
    l2 = torch.zeros((2 * n_slots, ppb, N, d), dtype=torch.float16, device=DEV)
    tags = torch.empty(2 * n_slots, dtype=torch.int32, device=DEV)
    fetch = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    loc = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    table = torch.from_numpy(pat.block_table).to(DEV)
    pred = torch.zeros((n_seq, k), dtype=torch.int32, device=DEV)
    side = torch.cuda.Stream()

    def step(main):
        c.reset_pool(stream=main)
        c.compress_blocks(x, stream=main)
        c.decompress_blocks(out, stream=main)
        c.prefetch_reset(tags, n_seq, k, n_layers, stream=main)
        side.wait_stream(main)
        c.prefetch_layers(l2, tags, fetch, loc, table, pred, n_layers, pbl, 0, layer_begin=0, layer_end=1, stream=main)
        c.prefetch_layers(l2, tags, fetch, loc, table, pred, n_layers, pbl, 0, layer_begin=1, layer_end=2, stream=side)
        main.wait_stream(side)

    def snapshot():
        torch.cuda.synchronize()
        dn = c.desc_numpy()
        return (out.cpu().numpy().view(np.uint16).copy(), dn["mode"].copy(), dn["n16"].copy(), dn["scale"].copy(),
                l2.cpu().numpy().view(np.uint16).copy(), tags.cpu().numpy().copy(), fetch.cpu().numpy().copy(), loc.cpu().numpy().copy())

    pred.copy_(torch.from_numpy(pat.predictions(0)).to(DEV))
    step(torch.cuda.current_stream())
    eager0 = snapshot()
    assert np.array_equal(eager0[0], o.decompress_pages(*o.compress_pages(x.cpu().numpy().view(np.uint16), N, d, 3)[::-1], N, d)[0].reshape(eager0[0].shape))
    cap = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(cap):
        g.capture_begin()
        step(cap)
        g.capture_end()
    for rep in range(5):
        _say(f"[case] graph replay {rep}")
        p = pat.predictions(rep % 3)
        pred.copy_(torch.from_numpy(p).to(DEV))
        out.zero_()
        l2.fill_(3.0)
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        # eager run of the same step for comparison
        out.zero_()
        l2.fill_(3.0)
        step(torch.cuda.current_stream())
        want = snapshot()
        for a, b in zip(got, want):
            assert np.array_equal(a, b)
        assert c.stats()["status"] == 0


# page shape and pages per block; sequences, predictions per sequence, layers, sequence lengths in tokens.  The
# last case issues a few thousand transfers per step, several hundred per layer: queue building over more than
# one chunk of a layer, more engines than 256, engines of the grid that find nothing to do.
@pytest.mark.parametrize("geom", [(16, 128, 4, 5, 8, 4, 48, 200), (16, 64, 3, 5, 8, 4, 48, 200), (8, 32, 2, 5, 8, 4, 48, 200),
                                  (16, 96, 3, 5, 8, 4, 48, 200), (32, 128, 2, 5, 8, 4, 48, 200), (16, 32, 1, 48, 16, 5, 400, 800)])
@pytest.mark.parametrize("omega", [1, 5, 16, 4096])
def test_window_prefetch_matches_unbounded_and_model(omega, geom):
    """Algorithm 1's outstanding-request window: with at most omega blocks in flight the plan arrays and
    the buffer are those of the unbounded call and of the model; the queue the engines worked through
    is the model's issue list (count, per-layer completion), and no more than omega were ever in flight."""
    rng = np.random.default_rng(50 + omega)
    N, d, ppb, n_seq_, k_, n_layers, len_lo, len_hi = geom
    pat = synth.gather_pattern(n_seq=n_seq_, k=k_, len_lo=len_lo, len_hi=len_hi, seed=12)
    pbl, n_seq, k = pat.pool_blocks_per_layer, pat.n_seq, pat.k
    x = (rng.standard_normal((n_layers * pbl, ppb, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)
    c, _ = gpu_compress(x, N, d, ppb, 3)
    n_slots = n_layers * n_seq * k

    def buffers():
        return (torch.full((2 * n_slots, ppb, N, d), 5.0, dtype=torch.float16, device=DEV),
                torch.empty(2 * n_slots, dtype=torch.int32, device=DEV), torch.empty(n_slots, dtype=torch.int32, device=DEV),
                torch.empty(n_slots, dtype=torch.int32, device=DEV))

    l2a, tags_a, fetch_a, loc_a = buffers()  # unbounded
    l2b, tags_b, fetch_b, loc_b = buffers()  # windowed
    c.prefetch_reset(tags_a, n_seq, k, n_layers)
    c.prefetch_reset(tags_b, n_seq, k, n_layers)
    notify = torch.full((n_layers + 4,), -7, dtype=torch.int64, device=DEV)
    work = torch.empty(kvc.window_workspace(n_slots, n_layers), dtype=torch.uint8, device=DEV)
    table = torch.from_numpy(pat.block_table).to(DEV)
    m_tags = np.full((2, n_layers, n_seq, k), -1, np.int32)
    for step in range(6):
        fill = step % 2
        pred_np = pat.predictions(step).copy()
        pred = torch.from_numpy(pred_np).to(DEV)
        lo, hi = (1, 3) if step == 4 else (0, n_layers)
        _say(f"[case] window omega {omega} geometry {geom} step {step} layers [{lo},{hi})")
        c.prefetch_layers(l2a, tags_a, fetch_a, loc_a, table, pred, n_layers, pbl, fill, layer_begin=lo, layer_end=hi)
        c.prefetch_layers_window(l2b, tags_b, fetch_b, loc_b, table, pred, n_layers, pbl, fill, omega, notify, work,
                                 layer_begin=lo, layer_end=hi)
        torch.cuda.synchronize()
        m_fetch, m_loc, bad = pm.prefetch_step(m_tags, fill, pat.block_table, pred_np, None, n_layers, pbl, lo, hi)
        queue, per_layer, batches = pm.window_schedule(m_fetch, omega, lo, hi)
        first = lo * n_seq * k
        sl = slice(first, hi * n_seq * k)
        assert np.array_equal(tags_b.cpu().numpy(), m_tags.reshape(-1)) and torch.equal(tags_a, tags_b)
        assert np.array_equal(fetch_b.cpu().numpy()[sl], m_fetch.reshape(-1)[sl]) and torch.equal(fetch_a[sl], fetch_b[sl])
        assert np.array_equal(loc_b.cpu().numpy()[sl], m_loc.reshape(-1)[sl]) and torch.equal(loc_a[sl], loc_b[sl])
        assert torch.equal(l2a.view(torch.int16), l2b.view(torch.int16)), "windowed buffer differs from the unbounded call's"
        nt = notify.cpu().numpy()
        opened, issued, high, closed = nt[n_layers:]
        assert issued == queue.size and opened > 0 and closed >= opened
        assert (nt[lo:hi] >= opened).all() and (nt[lo:hi] <= closed).all(), "every layer of the call is stamped ready"
        # the queue in the workspace is the model's issue list (relative to the call's first slot)
        hdr = work[:256].view(torch.int32).cpu().numpy()  # n_issued, engines | ticket | done, a cache line each
        engines = min(omega, queue.size)
        if engines > 256:  # many engines only while each has eight transfers
            engines = min(engines, max(256, queue.size // 8))
        assert hdr[0] == queue.size and hdr[1] == engines == high and hdr[32] == queue.size and hdr[16] >= queue.size
        q_off = kvc.window_workspace(0, hi - lo)
        got_q = work[q_off:q_off + 4 * queue.size].view(torch.int32).cpu().numpy()
        assert np.array_equal(got_q + first, queue)
    assert c.stats()["status"] == 0


def test_window_argument_checks():
    N, d, ppb = 16, 128, 2
    pat = synth.gather_pattern(n_seq=3, k=4, len_lo=40, len_hi=90, seed=2)
    pbl = pat.pool_blocks_per_layer
    x = np.random.default_rng(1).standard_normal((pbl, ppb, N, d)).astype(np.float16)
    c, _ = gpu_compress(x, N, d, ppb, 3)
    n_slots = pat.n_seq * pat.k
    l2 = torch.zeros((2 * n_slots, ppb, N, d), dtype=torch.float16, device=DEV)
    tags = torch.full((2 * n_slots,), -1, dtype=torch.int32, device=DEV)
    fetch = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    loc = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    notify = torch.zeros(1 + 4, dtype=torch.int64, device=DEV)
    need = kvc.window_workspace(n_slots, 1)
    assert need == 256 + 256 + 4 * n_slots
    table, pred = torch.from_numpy(pat.block_table).to(DEV), torch.from_numpy(pat.predictions(0)).to(DEV)
    work = torch.empty(need, dtype=torch.uint8, device=DEV)
    for omega, wk in ((0, work), (-1, work), (4, work[: need - 16])):
        with pytest.raises(kvc.KvcError) as e:
            c.prefetch_layers_window(l2, tags, fetch, loc, table, pred, 1, pbl, 0, omega, notify, wk)
        assert e.value.code == kvc.ERR_ARG
    c.prefetch_layers_window(l2, tags, fetch, loc, table, pred, 1, pbl, 0, 4, notify, work)
    torch.cuda.synchronize()
    assert notify.cpu().numpy()[1 + 1] == (fetch.cpu().numpy() >= 0).sum() > 0


def test_prefetch_into_a_strided_buffer():
    """Slots of the L2 buffer follow the cache layout in force: with a padded token-major layout the
    blocks of half 1 and of a layer range that does not start at 0 land block_stride elements apart."""
    rng = np.random.default_rng(9)
    N, d, H, n_layers = 16, 128, 3, 3
    pad = 64
    row, page, block = H * d + pad, d, N * (H * d + pad)
    pat = synth.gather_pattern(n_seq=4, k=4, len_lo=48, len_hi=160, seed=21)
    pbl, n_seq, k = pat.pool_blocks_per_layer, pat.n_seq, pat.k
    x = (rng.standard_normal((n_layers * pbl, H, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)
    c, _ = gpu_compress(x, N, d, H, 3)  # compressed from a dense buffer
    od, op = o.compress_pages(x.view(np.uint16), N, d, 3, n_threads=8)
    full = o.decompress_pages(op, od, N, d, n_threads=8)[0].reshape(n_layers * pbl, H, N, d)
    c.set_cache_layout(block, page, row)
    n_slots = n_layers * n_seq * k
    l2 = torch.full((2 * n_slots * block,), 5.0, dtype=torch.float16, device=DEV)
    tags = torch.empty(2 * n_slots, dtype=torch.int32, device=DEV)
    fetch = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    loc = torch.empty(n_slots, dtype=torch.int32, device=DEV)
    c.prefetch_reset(tags, n_seq, k, n_layers)
    table = torch.from_numpy(pat.block_table).to(DEV)
    m_tags = np.full((2, n_layers, n_seq, k), -1, np.int32)
    want = np.full((2 * n_slots, N, H * d + pad), np.float16(5.0).view(np.uint16), np.uint16)
    for step, (fill, lo, hi) in enumerate(((0, 0, n_layers), (1, 1, n_layers), (0, 2, 3), (1, 0, 2))):
        pred_np = pat.predictions(step)
        _say(f"[case] strided prefetch step {step} fill {fill} layers [{lo},{hi})")
        c.prefetch_layers(l2, tags, fetch, loc, table, torch.from_numpy(pred_np).to(DEV), n_layers, pbl, fill,
                          layer_begin=lo, layer_end=hi)
        m_fetch, m_loc, bad = pm.prefetch_step(m_tags, fill, pat.block_table, pred_np, None, n_layers, pbl, lo, hi)
        assert np.array_equal(tags.cpu().numpy(), m_tags.reshape(-1))
        for slot in np.nonzero(m_fetch.reshape(-1) >= 0)[0]:
            blk = full[m_fetch.reshape(-1)[slot]]  # [H][N][d] -> token-major rows [N][H*d]
            want[fill * n_slots + slot, :, : H * d] = blk.transpose(1, 0, 2).reshape(N, H * d)
        got = l2.cpu().numpy().view(np.uint16).reshape(2 * n_slots, N, H * d + pad)
        assert np.array_equal(got, want), "strided L2 buffer differs from the model (padding must stay untouched)"
    assert c.stats()["status"] == 0
