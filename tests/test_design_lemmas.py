"""The small arguments the kernels rest on, checked in numpy on random and adversarial inputs (no GPU, no library: these
are models of the index arithmetic, written out so that the argument can be read and broken independently of the HIP code).

 * probes from block maxima: the rows of the blocks whose maximum reaches the nprobe-th largest block maximum contain
   the nprobe best rows under (score descending, id ascending);
 * the bitonic network's pair map (thread t owns (lo, lo | j), lo = t with a zero inserted at bit log2 j) sorts, and for
   j <= 64 the 64 pairs of a wave stay inside one aligned block of 128 keys;
 * inverted lists built from per-(group, centroid) counts and one sequential walker per group come out ascending,
   duplicate-free and equal to the oracle's."""
import numpy as np
import pytest

from oracle import oracle as orc


def _top(scores, ids, n):
    order = np.lexsort((ids, -scores.astype(np.float64)))
    return ids[order][:n]


@pytest.mark.parametrize("seed", range(6))
def test_probes_from_block_maxima(seed):
    rng = np.random.default_rng(seed)
    for C, rows, nprobe in [(1000, 32, 1), (1000, 32, 2), (257, 32, 8), (64, 64, 4), (5, 32, 3), (4096, 32, 7)]:
        col = rng.standard_normal(C).astype(np.float32)
        if seed % 2:                      # heavy ties, also across blocks
            col = np.round(col * 2) / 2
        if seed == 5:
            col[:] = 0.0                  # every block ties
        nblk = (C + rows - 1) // rows
        bmax = np.array([col[b * rows:(b + 1) * rows].max() for b in range(nblk)])
        T = np.sort(bmax)[::-1][nprobe - 1] if nblk >= nprobe else -np.inf
        listed = [b for b in range(nblk) if bmax[b] >= T]
        ids = np.concatenate([np.arange(b * rows, min(C, (b + 1) * rows)) for b in listed])
        assert len(ids) >= min(nprobe, C)
        np.testing.assert_array_equal(_top(col[ids], ids, nprobe), _top(col, np.arange(C), nprobe))


def _bitonic(keys):
    n2 = len(keys)
    s = keys.copy()
    kk = 2
    while kk <= n2:
        j = kk >> 1
        while j > 0:
            t = np.arange(n2 // 2)
            lo = ((t & ~(j - 1)) << 1) | (t & (j - 1))
            hi = lo | j
            if j <= 64:                   # a wave's 64 pairs stay inside its 128 keys
                assert np.array_equal(lo >> 7, t >> 6) and np.array_equal(hi >> 7, t >> 6)
            assert len(np.unique(np.concatenate([lo, hi]))) == n2          # every key in exactly one pair
            up = (lo & kk) == 0
            a, b = s[lo].copy(), s[hi].copy()
            swap = (a > b) == up
            s[lo] = np.where(swap, b, a)
            s[hi] = np.where(swap, a, b)
            j >>= 1
        kk <<= 1
    return s


@pytest.mark.parametrize("n2", [2, 4, 64, 128, 256, 1024, 8192])
def test_bitonic_pair_map_sorts(n2):
    rng = np.random.default_rng(n2)
    keys = rng.integers(0, 2 ** 63, size=n2, dtype=np.uint64)
    keys[rng.integers(0, n2, size=max(1, n2 // 3))] = np.uint64(2 ** 64 - 1)   # padding keys
    np.testing.assert_array_equal(_bitonic(keys), np.sort(keys))


@pytest.mark.parametrize("P,C,G", [(300, 17, 7), (50, 3, 50), (9, 1, 4), (1, 40, 1), (1000, 5, 13)])
def test_grouped_counting_builds_the_inverted_lists(P, C, G):
    rng = np.random.default_rng(P * 31 + C)
    lens = rng.integers(0, 12, size=P)
    doc_offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    codes = rng.integers(0, C, size=int(doc_offsets[-1])).astype(np.int32)
    per = (P + G - 1) // G
    firsts = []                            # (passage, code) for every first occurrence of a code in its passage
    for p in range(P):
        seen = set()
        for c in codes[doc_offsets[p]:doc_offsets[p + 1]]:
            if c not in seen:
                seen.add(c)
                firsts.append((p, int(c)))
    counts = np.zeros((G, C), np.int64)
    for p, c in firsts:
        counts[p // per, c] += 1
    total = counts.sum(axis=0)
    off = np.concatenate([[0], np.cumsum(total)])
    start = np.cumsum(counts, axis=0) - counts                 # position inside list c where group g starts
    pids = np.full(int(off[-1]), -1, np.int64)
    for g in rng.permutation(G):                               # the groups finish in any order ...
        cursor = start[g].copy()
        for p, c in [(p, c) for p, c in firsts if p // per == g]:   # ... each walks its passages in id order
            pids[off[c] + cursor[c]] = p
            cursor[c] += 1
    o_off, o_pids = orc.build_ivf(codes, doc_offsets, C)
    np.testing.assert_array_equal(off, o_off)
    np.testing.assert_array_equal(pids, o_pids)
