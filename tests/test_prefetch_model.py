"""Pins for the prefetch model (oracle/prefetch_model.py): the bookkeeping of Algorithm 1 is checked by
carrying the real contents of every L2 slot alongside the tags -- only an issued transfer changes a slot --
and asserting what Algorithm 1 promises: every predicted block can be read where `loc` says, and a block
already in L1 or L2 is never transferred again."""
import numpy as np
import pytest

from oracle import prefetch_model as pm


def _setup(rng, n_layers=3, n_seq=4, k=6, max_blocks=9, pbpl=40):
    table = np.full((n_seq, max_blocks), -1, np.int32)
    perm = rng.permutation(pbpl)
    o = 0
    nb = rng.integers(3, max_blocks + 1, n_seq)
    for s in range(n_seq):
        table[s, : nb[s]] = perm[o:o + nb[s]]
        o += nb[s]
    return table, nb


@pytest.mark.parametrize("reuse", [False, True])
@pytest.mark.parametrize("seed", range(6))
def test_consumer_always_finds_the_predicted_block_and_nothing_resident_is_refetched(seed, reuse):
    rng = np.random.default_rng(seed)
    n_layers, n_seq, k, pbpl = 3, 4, 6, 40
    table, nb = _setup(rng, n_layers, n_seq, k, 9, pbpl)
    n_slots = n_layers * n_seq * k
    tags = np.full((2, n_layers, n_seq, k), -1, np.int32)
    content = np.full(2 * n_slots, -1, np.int64)  # what really sits in each slot
    l1_first = (nb - 1).astype(np.int32) if seed % 2 else None
    total_fetch = total_valid = 0
    for step in range(40):
        fill = step % 2
        pred = (rng.random((n_seq, k)) * nb[:, None]).astype(np.int32)
        pred[rng.random((n_seq, k)) < 0.1] = -1  # some predictions missing
        before = tags.copy()
        step_fn = pm.prefetch_step_reuse if reuse else pm.prefetch_step
        fetch, loc, bad = step_fn(tags, fill, table, pred, l1_first, n_layers, pbpl)
        assert not bad
        # transfers happen, into the slot of the half being filled that `fetch` is indexed by
        for l in range(n_layers):
            for s in range(n_seq):
                base = (l * n_seq + s) * k
                resident_other = set(before[1 - fill, l, s].tolist())
                got = [int(f) for f in fetch[l, s] if f >= 0]
                assert len(got) == len(set(got)), "a block was transferred twice in one step"
                assert not (set(got) & resident_other), "a block resident in the other half was transferred"
                if reuse:  # nothing that was anywhere in the L2 buffer is transferred again
                    assert not (set(got) & set(before[fill, l, s].tolist()))
                for j in range(k):
                    if fetch[l, s, j] >= 0:
                        assert before[fill, l, s, j] != fetch[l, s, j], "transfer into a slot that already held the block"
                        content[fill * n_slots + base + j] = fetch[l, s, j]
        # only issued transfers changed tags, and tags describe contents
        assert np.array_equal(tags.reshape(-1), content.astype(np.int32))
        assert np.array_equal(tags[1 - fill], before[1 - fill])
        # the consumer's view
        for l in range(n_layers):
            for s in range(n_seq):
                for j in range(k):
                    lb = pred[s, j]
                    # (with slot reuse `fetch` is indexed by slot, so slot j may serve another prediction)
                    if lb < 0:
                        assert loc[l, s, j] == pm.NO_BLOCK and (reuse or fetch[l, s, j] == -1)
                    elif l1_first is not None and lb >= l1_first[s]:
                        assert loc[l, s, j] == pm.IN_L1 and (reuse or fetch[l, s, j] == -1)
                    else:
                        total_valid += 1
                        assert content[loc[l, s, j]] == l * pbpl + table[s, lb]
        total_fetch += int((fetch >= 0).sum())
    assert 0 < total_fetch < total_valid  # the residency test does save transfers on this pattern


def test_same_predictions_next_step_transfer_nothing():
    rng = np.random.default_rng(9)
    table, nb = _setup(rng)
    tags = np.full((2, 3, 4, 6), -1, np.int32)
    pred = (rng.random((4, 6)) * nb[:, None]).astype(np.int32)
    f0, _, _ = pm.prefetch_step(tags, 0, table, pred, None, 3, 40)
    assert (f0 >= 0).sum() > 0
    f1, loc1, _ = pm.prefetch_step(tags, 1, table, pred, None, 3, 40)
    assert (f1 >= 0).sum() == 0 and (loc1 >= 0).all() and (loc1 < 3 * 4 * 6).all()  # all found in half 0
    f2, _, _ = pm.prefetch_step(tags, 0, table, pred, None, 3, 40)
    assert (f2 >= 0).sum() == 0


def test_layer_ranges_compose_and_bad_indices_are_flagged():
    rng = np.random.default_rng(10)
    table, nb = _setup(rng)
    pred = (rng.random((4, 6)) * nb[:, None]).astype(np.int32)
    t_all = np.full((2, 3, 4, 6), -1, np.int32)
    f_all, l_all, _ = pm.prefetch_step(t_all, 0, table, pred, None, 3, 40)
    t_parts = np.full((2, 3, 4, 6), -1, np.int32)
    f_parts = np.full((3, 4, 6), -1, np.int32)
    l_parts = np.full((3, 4, 6), -1, np.int32)
    for lo, hi in ((2, 3), (0, 1), (1, 2)):
        f, l, _ = pm.prefetch_step(t_parts, 0, table, pred, None, 3, 40, lo, hi)
        f_parts[lo:hi], l_parts[lo:hi] = f[lo:hi], l[lo:hi]
    assert np.array_equal(t_all, t_parts) and np.array_equal(f_all, f_parts) and np.array_equal(l_all, l_parts)
    pred2 = pred.copy()
    pred2[0, 0] = table.shape[1] + 5
    f, l, bad = pm.prefetch_step(np.full((2, 3, 4, 6), -1, np.int32), 0, table, pred2, None, 3, 40)
    assert bad and (l[:, 0, 0] == -1).all() and (f[:, 0, 0] == -1).all()


@pytest.mark.parametrize("fn", [pm.prefetch_step, pm.prefetch_step_reuse], ids=["positional", "reuse"])
def test_table_entries_at_and_beyond_the_pool_size_are_bad_indices(fn):
    """A layer's pool holds blocks 0 .. pool_blocks_per_layer - 1: an entry equal to that count is the first
    invalid one.  Hand-counted: one sequence, three predictions, table entries 6 (last valid), 7 (= the count)
    and 9; two layers."""
    table = np.array([[6, 7, 9]], np.int32)
    pred = np.array([[0, 1, 2]], np.int32)
    tags = np.full((2, 2, 1, 3), -1, np.int32)
    f, l, bad = fn(tags, 0, table, pred, None, 2, 7)
    assert bad
    assert f[:, 0].tolist() == [[6, -1, -1], [13, -1, -1]]  # layer l's block e is pool block 7 l + e
    assert l[:, 0].tolist() == [[0, -1, -1], [3, -1, -1]]
    f, l, bad = fn(np.full((2, 2, 1, 3), -1, np.int32), 0, table[:, :1], pred[:, :1].repeat(3, 1), None, 2, 7)
    assert not bad  # the last valid entry alone raises no flag


def test_slot_reuse_counts_a_block_held_twice_only_once():
    """The half being filled may hold one block in two slots (the positional policy leaves such states behind).
    Only the first copy is worth keeping: the second slot is free for a new block.  Hand-counted, k = 2: the
    half holds [X, X], the step wants [X, Y] -> Y goes into slot 1, X stays in slot 0, nothing else moves."""
    table = np.array([[4, 5]], np.int32)  # logical block 0 -> X = 4, 1 -> Y = 5
    tags = np.full((2, 1, 1, 2), -1, np.int32)
    tags[0, 0, 0] = [4, 4]
    f, l, bad = pm.prefetch_step_reuse(tags, 0, table, np.array([[0, 1]], np.int32), None, 1, 8)
    assert not bad and f[0, 0].tolist() == [-1, 5] and l[0, 0].tolist() == [0, 1] and tags[0, 0, 0].tolist() == [4, 5]
    # three slots [X, X, Z], wanted [Y, X, W]: slot 0 keeps X, the duplicate in slot 1 takes Y, slot 2 takes W
    table = np.array([[4, 5, 6, 7]], np.int32)
    tags = np.full((2, 1, 1, 3), -1, np.int32)
    tags[1, 0, 0] = [4, 4, 6]
    f, l, bad = pm.prefetch_step_reuse(tags, 1, table, np.array([[1, 0, 3]], np.int32), None, 1, 8)
    assert f[0, 0].tolist() == [-1, 5, 7] and l[0, 0].tolist() == [3 + 1, 3 + 0, 3 + 2] and tags[1, 0, 0].tolist() == [4, 5, 7]


def test_slot_reuse_transfers_one_block_per_new_block_on_a_sliding_window():
    """Predictions pos+1..pos+k with pos advancing one block at a time: after warm-up the reuse policy moves
    exactly one block per sequence per advance, the positional policy k."""
    n_seq, k, nblk = 5, 8, 40
    table = np.arange(n_seq * nblk, dtype=np.int32).reshape(n_seq, nblk)
    counts = {}
    for name, fn in (("positional", pm.prefetch_step), ("reuse", pm.prefetch_step_reuse)):
        tags = np.full((2, 1, n_seq, k), -1, np.int32)
        tot = 0
        for t in range(2 + 3 * 10):
            pos = t // 3
            pred = ((pos + 1 + np.arange(k))[None, :] % nblk).repeat(n_seq, 0).astype(np.int32)
            f, l, _ = fn(tags, t % 2, table, pred, None, 1, n_seq * nblk)
            if t >= 2:
                tot += int((f >= 0).sum())
        counts[name] = tot
    assert counts["reuse"] == n_seq * 10 and counts["positional"] == n_seq * 10 * k


@pytest.mark.parametrize("omega", [1, 3, 16, 64, 0])
@pytest.mark.parametrize("reuse", [False, True])
def test_window_never_exceeds_omega_and_carries_out_every_issued_transfer_once_in_order(omega, reuse):
    """Algorithm 1's WaitCompletion over at most Omega_max concurrent transfers: the batches are pieces of
    the issue list, none longer than omega, their concatenation is exactly the transfers the step issued
    (every one once, in layer / sequence / slot order), and a layer's count is what it issued."""
    rng = np.random.default_rng(100 + omega)
    n_layers, n_seq, k, pbpl = 5, 4, 6, 40
    table, nb = _setup(rng, n_layers, n_seq, k, 9, pbpl)
    tags = np.full((2, n_layers, n_seq, k), -1, np.int32)
    step_fn = pm.prefetch_step_reuse if reuse else pm.prefetch_step
    for step in range(6):
        pred = (rng.random((n_seq, k)) * nb[:, None]).astype(np.int32)
        pred[rng.random((n_seq, k)) < 0.15] = -1
        lo, hi = (1, 4) if step == 3 else (0, n_layers)
        fetch, loc, _ = step_fn(tags, step % 2, table, pred, None, n_layers, pbpl, lo, hi)
        queue, per_layer, batches = pm.window_schedule(fetch, omega, lo, hi)
        flat = fetch.reshape(-1)
        issued = np.nonzero(flat >= 0)[0]  # numpy's flat order is (layer, sequence, slot) order
        assert np.array_equal(queue, issued.astype(np.int32))
        assert all(0 < len(b) <= (omega if omega > 0 else max(1, queue.size)) for b in batches)
        assert np.array_equal(np.concatenate(batches) if batches else np.zeros(0, np.int32), queue)
        assert len(set(queue.tolist())) == queue.size
        assert np.array_equal(per_layer, (fetch >= 0).sum(axis=(1, 2)).astype(np.int32))
        assert per_layer[:lo].sum() == 0 and per_layer[hi:].sum() == 0
        if omega > 0:
            assert len(batches) == -(-queue.size // omega)
            # a full window is kept whenever work remains: only the last batch may be short
            assert all(len(b) == omega for b in batches[:-1])
        until = pm.batches_until_ready(per_layer, omega, lo)
        assert until[-1] == len(batches) and (np.diff(until) >= 0).all()


def test_window_closed_forms():
    """Hand-checked cases: 7 transfers over 3 layers (3, 0, 4) through a window of 2 need 4 batches; the
    first layer is ready after 2, the empty layer with it, the last after 4.  Without a bound: one batch."""
    fetch = np.full((3, 1, 4), -1, np.int32)
    fetch[0, 0, [0, 2, 3]] = [5, 6, 7]
    fetch[2, 0, :] = [20, 21, 22, 23]
    queue, per_layer, batches = pm.window_schedule(fetch, 2)
    assert queue.tolist() == [0, 2, 3, 8, 9, 10, 11] and per_layer.tolist() == [3, 0, 4]
    assert [b.tolist() for b in batches] == [[0, 2], [3, 8], [9, 10], [11]]
    assert pm.batches_until_ready(per_layer, 2).tolist() == [2, 2, 4]
    _, _, one = pm.window_schedule(fetch, 0)
    assert len(one) == 1 and one[0].tolist() == queue.tolist()
    assert pm.batches_until_ready(per_layer, 0).tolist() == [1, 1, 1]
    q0, p0, b0 = pm.window_schedule(np.full((2, 2, 2), -1, np.int32), 4)
    assert q0.size == 0 and p0.tolist() == [0, 0] and b0 == []
    # layers that come before the first transfer wait for nothing: transfers per layer (0, 3, 0, 2)
    per = np.array([0, 3, 0, 2], np.int32)
    assert pm.batches_until_ready(per, 0).tolist() == [0, 1, 1, 1]
    assert pm.batches_until_ready(per, 2).tolist() == [0, 2, 2, 3]


@pytest.mark.parametrize("fn", [pm.prefetch_step, pm.prefetch_step_reuse], ids=["positional", "reuse"])
def test_an_unmapped_logical_block_is_skipped_without_a_flag(fn):
    """A table entry of -1 means the sequence has no such block (tables are padded with it): nothing is
    transferred for it, `loc` says -1, and it is not an error.  Hand-counted: table (4, -1), predictions (0, 1)."""
    tags = np.full((2, 1, 1, 2), -1, np.int32)
    f, l, bad = fn(tags, 0, np.array([[4, -1]], np.int32), np.array([[0, 1]], np.int32), None, 1, 8)
    assert not bad and f[0, 0].tolist() == [4, -1] and l[0, 0].tolist() == [0, -1] and tags[0, 0, 0].tolist() == [4, -1]
