"""The entry point that allocates nothing: kvc_prefetch_layers_window_static keeps the window's queue in a
static device array of the library.  Its results must be those of kvc_prefetch_layers_window (which takes
the workspace from the caller), call after call on the shared array -- also when a later call is smaller
than the one before and the array still holds the earlier call's queue."""
import numpy as np
import pytest
import torch

from paper_2512_11920_amd import kvc, synth
from gpu_util import DEV, gpu_compress

pytestmark = pytest.mark.gpu


def _say(m):
    print(m, flush=True)


def test_static_workspace_call_matches_the_workspace_call_twice_in_a_row():
    rng = np.random.default_rng(70)
    N, d, ppb, n_layers, omega = 16, 128, 4, 4, 6
    pat = synth.gather_pattern(n_seq=6, k=8, len_lo=48, len_hi=200, seed=13)
    pbl, n_seq, k = pat.pool_blocks_per_layer, pat.n_seq, pat.k
    x = (rng.standard_normal((n_layers * pbl, ppb, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)
    c, _ = gpu_compress(x, N, d, ppb, 3)
    n_slots = n_layers * n_seq * k

    def buffers():
        tags = torch.empty(2 * n_slots, dtype=torch.int32, device=DEV)
        c.prefetch_reset(tags, n_seq, k, n_layers)
        return (torch.full((2 * n_slots, ppb, N, d), 5.0, dtype=torch.float16, device=DEV), tags,
                torch.full((n_slots,), -9, dtype=torch.int32, device=DEV), torch.full((n_slots,), -9, dtype=torch.int32, device=DEV),
                torch.zeros(n_layers + 4, dtype=torch.int64, device=DEV))

    ref, sta = buffers(), buffers()
    work = torch.empty(kvc.window_workspace(n_slots, n_layers), dtype=torch.uint8, device=DEV)
    table = torch.from_numpy(pat.block_table).to(DEV)
    # first call: all layers (the larger input); second: one layer (smaller: the array still holds the
    # first call's longer queue); third: a middle range into the other half
    for step, (fill, lo, hi) in enumerate(((0, 0, n_layers), (1, 2, 3), (0, 1, 3))):
        pred = torch.from_numpy(pat.predictions(step)).to(DEV)
        _say(f"[case] static window step {step} fill {fill} layers [{lo},{hi})")
        c.prefetch_layers_window(ref[0], ref[1], ref[2], ref[3], table, pred, n_layers, pbl, fill, omega, ref[4], work,
                                 layer_begin=lo, layer_end=hi)
        c.prefetch_layers_window(sta[0], sta[1], sta[2], sta[3], table, pred, n_layers, pbl, fill, omega, sta[4], None,
                                 layer_begin=lo, layer_end=hi)
        torch.cuda.synchronize()
        assert torch.equal(ref[0].view(torch.int16), sta[0].view(torch.int16)), "L2 buffer"
        assert torch.equal(ref[1], sta[1]) and torch.equal(ref[2], sta[2]) and torch.equal(ref[3], sta[3]), "tags / fetch / loc"
        a, b = ref[4].cpu().numpy(), sta[4].cpu().numpy()
        issued = int((ref[2].cpu().numpy()[lo * n_seq * k:hi * n_seq * k] >= 0).sum())
        assert a[n_layers + 1] == b[n_layers + 1] == issued and issued > 0
        assert 1 <= b[n_layers + 2] <= omega and b[n_layers + 3] >= b[n_layers] > 0
        assert (b[lo:hi] >= b[n_layers]).all() and (b[lo:hi] <= b[n_layers + 3]).all()
    assert c.stats()["status"] == 0


def test_static_workspace_call_refuses_what_does_not_fit():
    N, d, ppb = 16, 128, 1
    x = np.zeros((4, ppb, N, d), np.float16)
    c, _ = gpu_compress(x, N, d, ppb, 3)
    n_seq, k = 2049, 32  # 65,568 slots in one layer: 32 more than the static array holds
    dummy = torch.zeros(16, dtype=torch.int32, device=DEV)
    L = kvc.load()
    rc = L.kvc_prefetch_layers_window_static(c._ctx, dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(),
                                             dummy.data_ptr(), 1, dummy.data_ptr(), None, n_seq, k, 1, 0, 1, 4, 0, 4,
                                             dummy.data_ptr(), None)
    assert rc == kvc.ERR_TOO_LARGE and "static workspace" in kvc.strerror(rc)
    rc = L.kvc_prefetch_layers_window_static(c._ctx, dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(),
                                             dummy.data_ptr(), 1, dummy.data_ptr(), None, 1, 1, 2000, 0, 1025, 4, 0, 4,
                                             dummy.data_ptr(), None)
    assert rc == kvc.ERR_TOO_LARGE


def test_static_workspace_call_records_into_a_hip_graph_and_replays():
    """What the entry point is for: under stream capture nothing may allocate.  A graph holding the static
    call is replayed with changing predictions, eager work and synchronisations in between, and every replay
    is compared with an eager run of the workspace call (plan arrays and buffer; the ready stamps are clock
    values and only have to be set)."""
    rng = np.random.default_rng(71)
    N, d, ppb, n_layers, omega = 16, 128, 4, 3, 5
    pat = synth.gather_pattern(n_seq=5, k=8, len_lo=48, len_hi=200, seed=14)
    pbl, n_seq, k = pat.pool_blocks_per_layer, pat.n_seq, pat.k
    x = (rng.standard_normal((n_layers * pbl, ppb, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)
    c, _ = gpu_compress(x, N, d, ppb, 3)
    n_slots = n_layers * n_seq * k

    def buffers():
        return (torch.full((2 * n_slots, ppb, N, d), 5.0, dtype=torch.float16, device=DEV),
                torch.empty(2 * n_slots, dtype=torch.int32, device=DEV), torch.full((n_slots,), -9, dtype=torch.int32, device=DEV),
                torch.full((n_slots,), -9, dtype=torch.int32, device=DEV), torch.zeros(n_layers + 4, dtype=torch.int64, device=DEV))

    g_l2, g_tags, g_fetch, g_loc, g_notify = buffers()   # written by the graph
    e_l2, e_tags, e_fetch, e_loc, e_notify = buffers()   # written eagerly, with a caller-owned workspace
    work = torch.empty(kvc.window_workspace(n_slots, n_layers), dtype=torch.uint8, device=DEV)
    table = torch.from_numpy(pat.block_table).to(DEV)
    pred = torch.zeros((n_seq, k), dtype=torch.int32, device=DEV)  # static input of the graph
    cap = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    c.prefetch_reset(g_tags, n_seq, k, n_layers)
    c.prefetch_reset(e_tags, n_seq, k, n_layers)
    torch.cuda.synchronize()
    with torch.cuda.stream(cap):
        graph.capture_begin()
        c.prefetch_layers_window(g_l2, g_tags, g_fetch, g_loc, table, pred, n_layers, pbl, 0, omega, g_notify, None, stream=cap)
        graph.capture_end()
    c.prefetch_reset(g_tags, n_seq, k, n_layers)  # the capture itself ran nothing
    for rep in range(4):
        _say(f"[case] static window graph replay {rep}")
        pred.copy_(torch.from_numpy(pat.predictions(rep)).to(DEV))
        g_notify.zero_()
        torch.cuda.synchronize()
        graph.replay()
        c.prefetch_layers_window(e_l2, e_tags, e_fetch, e_loc, table, pred, n_layers, pbl, 0, omega, e_notify, work)
        torch.cuda.synchronize()
        assert torch.equal(g_l2.view(torch.int16), e_l2.view(torch.int16)), f"replay {rep}: L2 buffer"
        assert torch.equal(g_tags, e_tags) and torch.equal(g_fetch, e_fetch) and torch.equal(g_loc, e_loc), f"replay {rep}: plan"
        gn, en = g_notify.cpu().numpy(), e_notify.cpu().numpy()
        assert gn[n_layers + 1] == en[n_layers + 1] and (gn[:n_layers] > 0).all() and gn[n_layers + 3] >= gn[n_layers] > 0
    assert c.stats()["status"] == 0
