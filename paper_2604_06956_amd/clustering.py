"""Key-centric sample clustering for frozen-window micro-batches (Section V-C, "Sample Clustering").

Splitting a batch into N micro-batches makes the keys be deduplicated inside each micro-batch only, so a key whose
samples land in m micro-batches crosses the All2All m times instead of once; the paper answers with a CPU-side
preprocessing step that groups samples which share keys into the same micro-batch.  It gives no algorithm, so the one
below is this build's own (its result cannot be compared with the paper's: parity unpinned).  Whatever the grouping,
Proposition 2 holds: the accumulated gradient of the N micro-batches is the gradient of the whole batch.

The grouping is a balanced label propagation between samples and keys, deterministic (no random numbers, ties go to the
smaller index):

  * only keys that can be gathered into few micro-batches take part: 2 <= multiplicity <= batch/N (a more popular key is
    in every micro-batch whatever is done; a key with one lookup is in one);
  * samples start in the consecutive split; each round every key takes the micro-batch that most of its samples are in,
    every sample scores each micro-batch by the keys labelled with it (a key of multiplicity c weighs 1/c: keeping a rare
    key together saves the same one copy as a frequent one and takes fewer samples), samples are placed in order of
    decreasing best score into their best micro-batch that still has room (all micro-batches hold batch/N samples, give
    or take one).

This is preprocessing on the host, as in the paper; it is not part of the hot path and calls no kernel.  `keys`,
`bag_offsets` follow the library's batch layout (bag b = feature * batch + sample, the lookups of a bag contiguous).
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def sample_of_lookup(bag_offsets: np.ndarray, batch: int) -> np.ndarray:
    """Sample index of every lookup for the feature-major bag order (bag b belongs to sample b mod batch)."""
    lens = np.diff(bag_offsets.astype(np.int64))
    bag_sample = (np.arange(lens.shape[0], dtype=np.int64) % batch).astype(np.int32)
    return np.repeat(bag_sample, lens)


def consecutive_split(batch: int, num_micro: int) -> np.ndarray:
    """Micro-batch i holds samples [batch*i/N, batch*(i+1)/N)."""
    return ((np.arange(batch, dtype=np.int64) * num_micro) // batch).astype(np.int32)


FINE_CLUSTERS = 32   # small N: cluster into about this many groups first, then put whole groups into each micro-batch


def cluster_samples(keys: np.ndarray, bag_offsets: np.ndarray, batch: int, num_micro: int, rounds: int = 8,
                    inverse: Optional[np.ndarray] = None, counts: Optional[np.ndarray] = None) -> np.ndarray:
    """-> assign[batch] int32 in [0, num_micro): the micro-batch of every sample; every micro-batch gets floor or ceil of
    batch/num_micro samples.  `inverse` / `counts` (as np_dedup returns them) may be passed in to skip the host-side
    deduplication of `keys`.

    For num_micro below FINE_CLUSTERS the samples are first clustered into num_micro * f groups (f whole, about
    FINE_CLUSTERS groups in all) and micro-batch m takes groups m*f .. m*f+f-1: a population that falls into more natural
    clusters than there are micro-batches then keeps each of them whole."""
    M = int(num_micro)
    if M <= 1 or batch <= M or keys.shape[0] == 0:
        return consecutive_split(batch, max(M, 1))
    f = 1 if M >= FINE_CLUSTERS else -(-FINE_CLUSTERS // M)
    while f > 1 and batch < M * f * 2:
        f -= 1
    fine_cap = np.full(M * f, batch // (M * f), np.int64)
    fine_cap[: batch % (M * f)] += 1
    fine, shared = _cluster(keys, bag_offsets, batch, fine_cap, rounds, inverse, counts)
    if f == 1:
        return fine
    # fold: a micro-batch is started by the largest group not yet taken (ties: the smaller index) and takes, f - 1 times,
    # the free group that shares the most keys with what it already holds
    G = M * f
    size = np.bincount(fine, minlength=G)
    free = np.ones(G, bool)
    micro_of = np.empty(G, np.int64)
    for m in range(M):
        cand = np.nonzero(free)[0]
        first = cand[np.lexsort((cand, -size[cand]))[0]]
        members = [first]
        free[first] = False
        for _ in range(f - 1):
            cand = np.nonzero(free)[0]
            aff = shared[np.ix_(members, cand)].sum(axis=0)
            nxt = cand[np.lexsort((cand, -aff))[0]]
            members.append(nxt)
            free[nxt] = False
        micro_of[members] = m
    assign = micro_of[fine].astype(np.int32)
    # the folded sizes differ by at most f: move the last samples of the larger micro-batches to the smaller ones
    target = np.full(M, batch // M, np.int64)
    have = np.bincount(assign, minlength=M)
    order_big = np.lexsort((np.arange(M), -have))
    target[order_big[: batch % M]] += 1                   # the larger ones keep the extra sample
    spare = []
    for m in range(M):
        if have[m] > target[m]:
            idx = np.nonzero(assign == m)[0][target[m] - have[m]:]
            spare.extend(idx.tolist())
    spare = np.array(sorted(spare), np.int64)
    at = 0
    for m in range(M):
        need = int(target[m] - have[m])
        if need > 0:
            assign[spare[at:at + need]] = m
            at += need
    return assign


def _cluster(keys: np.ndarray, bag_offsets: np.ndarray, batch: int, cap: np.ndarray, rounds: int,
             inverse: Optional[np.ndarray], counts: Optional[np.ndarray]) -> np.ndarray:
    """Balanced label propagation into len(cap) groups of the given sizes (sum(cap) == batch).  -> (group of every sample,
    shared[g, h] = number of participating keys with samples in both group g and group h)."""
    N = int(cap.shape[0])
    assign = ((np.searchsorted(np.cumsum(cap), np.arange(batch), side="right"))).astype(np.int32)   # nothing to cluster: consecutive
    if inverse is None or counts is None:
        _, inverse, counts = np.unique(keys, return_inverse=True, return_counts=True)
    inverse = np.asarray(inverse).astype(np.int64, copy=False)
    counts = np.asarray(counts).astype(np.int64, copy=False)
    sample = sample_of_lookup(bag_offsets, batch).astype(np.int64)
    cmax = max(2, batch // N)
    eligible_key = (counts >= 2) & (counts <= cmax)
    sel = eligible_key[inverse]
    if not sel.any():
        return assign, np.zeros((N, N))
    # compact ids for the keys that take part
    key_local = np.cumsum(eligible_key) - 1
    lk = key_local[inverse[sel]]
    ls = sample[sel]
    K = int(eligible_key.sum())
    weight = (1.0 / counts[eligible_key])[lk]
    # seeds: every sample is anchored on its most frequent participating key (ties: the smaller key id); the N anchors
    # that hold the most samples start the N micro-batches, all other samples start unplaced
    akey = np.full(batch, -1, np.int64)
    pri = counts[eligible_key][lk] * np.int64(K) + (K - 1 - lk)         # larger = more frequent, then smaller id
    best_pri = np.full(batch, -1, np.int64)
    np.maximum.at(best_pri, ls, pri)
    hit = pri == best_pri[ls]
    akey[ls[hit]] = lk[hit]
    held = np.bincount(akey[akey >= 0], minlength=K)
    seeds = np.lexsort((np.arange(K), -held))[:N]                       # most samples first, ties by key id
    seed_label = np.full(K, -1, np.int64)
    seed_label[seeds] = np.arange(seeds.shape[0])
    assign = np.where(akey >= 0, seed_label[np.maximum(akey, 0)], -1).astype(np.int32)
    for _ in range(rounds):
        # every key takes the micro-batch most of its placed samples are in (ties: the smaller index); a key none of
        # whose samples is placed yet has no label
        placed = assign[ls] >= 0
        votes = np.bincount(lk[placed] * N + assign[ls[placed]], minlength=K * N).reshape(K, N)
        label = votes.argmax(axis=1)
        labelled = votes.max(axis=1) > 0
        use = labelled[lk]
        # every sample scores the micro-batches by the labels of its keys
        score = np.bincount(ls[use] * N + label[lk[use]], weights=weight[use], minlength=batch * N).reshape(batch, N)
        best = score.max(axis=1)
        order = np.lexsort((np.arange(batch), -best))          # decreasing best score, ties by sample index
        pref = np.argsort(-score, axis=1, kind="stable")       # each sample's micro-batches, best first
        new = np.full(batch, -1, np.int32)
        room = cap.copy()
        # placement by preference: all samples whose k-th choice still has room take it, in `order`
        pending = order
        for k in range(N):
            if pending.size == 0:
                break
            want = pref[pending, k]
            srt = np.argsort(want, kind="stable")
            w_sorted = want[srt]
            first = np.searchsorted(w_sorted, np.arange(N))
            rank = np.empty(pending.size, np.int64)
            rank[srt] = np.arange(pending.size) - first[w_sorted]
            ok = rank < room[want]
            new[pending[ok]] = want[ok].astype(np.int32)
            room -= np.bincount(want[ok], minlength=N)
            pending = pending[~ok]
        if np.array_equal(new, assign):
            break
        assign = new
    present = (np.bincount(lk * N + assign[ls], minlength=K * N).reshape(K, N) > 0).astype(np.float32)
    return assign, (present.T @ present).astype(np.float64)


def micro_batch_lookups(bag_offsets: np.ndarray, batch: int, features: int, assign: np.ndarray, micro: int):
    """-> (lookup positions, bag_offsets) of micro-batch `micro`: its samples in ascending order, bags feature-major."""
    samples = np.nonzero(assign == micro)[0].astype(np.int64)
    bags = (np.arange(features, dtype=np.int64)[:, None] * batch + samples[None, :]).ravel()
    off = bag_offsets.astype(np.int64)
    lens = off[bags + 1] - off[bags]
    new_off = np.concatenate([[0], np.cumsum(lens)])
    total = int(new_off[-1])
    # positions: for each selected bag, its contiguous run of lookups
    pos = np.repeat(off[bags] - new_off[:-1], lens) + np.arange(total, dtype=np.int64)
    return pos, new_off.astype(np.int32), bags


def sum_unique(keys: np.ndarray, bag_offsets: np.ndarray, batch: int, features: int, assign: np.ndarray, num_micro: int) -> int:
    """The objective the clustering lowers: sum over micro-batches of their distinct-key counts (host-side count)."""
    total = 0
    for m in range(num_micro):
        pos, _, _ = micro_batch_lookups(bag_offsets, batch, features, assign, m)
        if pos.size:
            total += int(np.unique(keys[pos]).size)
    return total
