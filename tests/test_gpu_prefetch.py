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
