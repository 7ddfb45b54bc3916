"""Plain model of the speculative prefetch step (Algorithm 1 of the paper, without the token
predictor) over a double-buffered L2 prefetch buffer.  TEST INFRASTRUCTURE, like the rest of oracle/.

Algorithm 1, per request s and layer l, for i = 1..k:
    A_virt = (s, l, predicted block i);  A_phys = TranslateAddress(A_virt)        -> block table lookup
    if A_phys not in L1 u L2:  IssueDMA(A_phys, L2[i])                             -> decode into slot i
The paper leaves "in L2" open for a double-buffered L2 (Section 3.3.1).  Reading: a block is in L2
if it sits in any slot of the half filled by the previous step, in a slot of the half being filled
that this step has already passed (it cannot be overwritten any more), or already in slot i itself.
Slots are never cleared, only overwritten (lazy invalidation, Section 3.4.3)."""
from __future__ import annotations

import numpy as np

NO_BLOCK, IN_L1 = -1, -2


def _translate(table, pred, l1_first, l, s, j, pbpl):
    """-> (physical block | NO_BLOCK | IN_L1, bad_index)"""
    lb = int(pred[s, j])
    if lb >= table.shape[1]:
        return NO_BLOCK, True
    if lb < 0:
        return NO_BLOCK, False
    if l1_first is not None and lb >= int(l1_first[s]):
        return IN_L1, False
    e = int(table[s, lb])
    if e >= pbpl:
        return NO_BLOCK, True
    if e < 0:
        return NO_BLOCK, False
    return l * pbpl + e, False


def prefetch_step_reuse(tags: np.ndarray, fill: int, table: np.ndarray, pred: np.ndarray, l1_first, n_layers: int,
                        pool_blocks_per_layer: int, layer_begin: int = 0, layer_end: int | None = None):
    """Slot-reuse variant: the L2 half being filled is treated as a small cache of k slots.  Blocks this
    step wants stay where they are (either half); a wanted block found nowhere is transferred into the
    lowest slot of the fill half whose content is not wanted (or is a duplicate).  fetch is indexed by
    destination slot.  Same return convention as prefetch_step."""
    n_seq, k = pred.shape
    n_slots = n_layers * n_seq * k
    layer_end = n_layers if layer_end is None else layer_end
    fetch = np.full((n_layers, n_seq, k), -1, np.int32)
    loc = np.full((n_layers, n_seq, k), -1, np.int32)
    bad_index = False
    other = 1 - fill
    for l in range(layer_begin, layer_end):
        for s in range(n_seq):
            base = (l * n_seq + s) * k
            want = []
            for j in range(k):
                phys, bad = _translate(table, pred, l1_first, l, s, j, pool_blocks_per_layer)
                bad_index = bad_index or bad
                want.append(phys)
            wanted = {w for w in want if w >= 0}
            keep, seen = [], set()
            for j2 in range(k):
                t = int(tags[fill, l, s, j2])
                keep.append(t in wanted and t not in seen)
                seen.add(t)
            for j in range(k):
                phys = want[j]
                if phys < 0:
                    loc[l, s, j] = phys
                    continue
                where = None
                for j2 in range(k):
                    if tags[other, l, s, j2] == phys:
                        where = other * n_slots + base + j2
                        break
                if where is None:
                    for j2 in range(k):
                        if keep[j2] and tags[fill, l, s, j2] == phys:
                            where = fill * n_slots + base + j2
                            break
                if where is None:
                    j2 = keep.index(False)  # there is always one: at most k distinct blocks are wanted
                    keep[j2] = True
                    tags[fill, l, s, j2] = phys
                    fetch[l, s, j2] = phys
                    where = fill * n_slots + base + j2
                loc[l, s, j] = where
    return fetch, loc, bad_index


def prefetch_step(tags: np.ndarray, fill: int, table: np.ndarray, pred: np.ndarray, l1_first, n_layers: int,
                  pool_blocks_per_layer: int, layer_begin: int = 0, layer_end: int | None = None):
    """tags: int32 [2][n_layers][n_seq][k], updated in place.  Returns (fetch, loc), each int32
    [n_layers][n_seq][k]; entries of layers outside [layer_begin, layer_end) are left at -1 / -1."""
    n_seq, k = pred.shape
    max_blocks = table.shape[1]
    n_slots = n_layers * n_seq * k
    layer_end = n_layers if layer_end is None else layer_end
    fetch = np.full((n_layers, n_seq, k), -1, np.int32)
    loc = np.full((n_layers, n_seq, k), -1, np.int32)
    bad_index = False
    other = 1 - fill
    for l in range(layer_begin, layer_end):
        for s in range(n_seq):
            base = (l * n_seq + s) * k
            for j in range(k):
                lb = int(pred[s, j])
                if lb < 0:
                    continue
                if lb >= max_blocks:
                    bad_index = True
                    continue
                if l1_first is not None and lb >= int(l1_first[s]):
                    loc[l, s, j] = IN_L1
                    continue
                e = int(table[s, lb])
                if e < 0:
                    continue
                if e >= pool_blocks_per_layer:
                    bad_index = True
                    continue
                phys = l * pool_blocks_per_layer + e
                where = None
                for j2 in range(k):  # the half the previous step filled
                    if tags[other, l, s, j2] == phys:
                        where = other * n_slots + base + j2
                        break
                if where is None:
                    for j2 in range(j):  # slots of this half this step is done with
                        if tags[fill, l, s, j2] == phys:
                            where = fill * n_slots + base + j2
                            break
                if where is None:
                    where = fill * n_slots + base + j
                    if tags[fill, l, s, j] != phys:  # not in L1 u L2: issue the transfer into L2[j]
                        tags[fill, l, s, j] = phys
                        fetch[l, s, j] = phys
                loc[l, s, j] = where
    return fetch, loc, bad_index


def window_schedule(fetch: np.ndarray, omega: int, layer_begin: int = 0, layer_end: int | None = None):
    """Outstanding-request window of Algorithm 1 (WaitCompletion over at most Omega_max concurrent
    transfers, Section 3.4.2): the transfers a step issued are carried out in issue order -- layer, then
    sequence, then slot, the order of the loops -- with never more than `omega` of them in flight; the step
    is ready when all have completed.
    fetch: int32 [n_layers][n_seq][k] as returned by prefetch_step / prefetch_step_reuse.
    Returns (queue, per_layer, batches):
      queue      int32 [n_issued]: flat slot index (l*n_seq + s)*k + j of every issued transfer, in issue order;
      per_layer  int32 [n_layers]: transfers issued for each layer (a layer is ready when that many completed);
      batches    list of int32 arrays: the queue cut into consecutive pieces of at most omega entries -- the
                 contents of the window if every transfer takes the same time.  omega <= 0 means no bound
                 (one batch)."""
    n_layers = fetch.shape[0]
    layer_end = n_layers if layer_end is None else layer_end
    queue = []
    per_layer = np.zeros(n_layers, np.int32)
    for l in range(layer_begin, layer_end):
        for s in range(fetch.shape[1]):
            for j in range(fetch.shape[2]):
                if fetch[l, s, j] >= 0:
                    queue.append((l * fetch.shape[1] + s) * fetch.shape[2] + j)
                    per_layer[l] += 1
    queue = np.asarray(queue, np.int32)
    if omega <= 0 or queue.size == 0:
        batches = [queue] if queue.size else []
    else:
        batches = [queue[i:i + omega] for i in range(0, queue.size, omega)]
    return queue, per_layer, batches


def batches_until_ready(per_layer: np.ndarray, omega: int, layer_begin: int = 0):
    """Equal-time model of the window: number of batches after which each layer's transfers have all
    completed (0 for a layer that issued none before any other did)."""
    done = np.cumsum(per_layer)
    if omega <= 0:
        return (done > 0).astype(np.int64)
    return (done + omega - 1) // omega
