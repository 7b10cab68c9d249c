"""The small arguments the kernels rest on, checked in numpy on random and adversarial inputs (no GPU, no library: these
are models of the index arithmetic, written out so that the argument can be read and broken independently of the HIP code).

 * probes from block maxima: the rows of the blocks whose maximum reaches the nprobe-th largest block maximum contain
   the nprobe best rows under (score descending, id ascending);
 * the bitonic network's pair map (thread t owns (lo, lo | j), lo = t with a zero inserted at bit log2 j) sorts, and for
   j <= 64 the 64 pairs of a wave stay inside one aligned block of 128 keys;
 * inverted lists built from per-(group, centroid) counts and one sequential walker per group come out ascending,
   duplicate-free and equal to the oracle's;
 * the probe kernel's list logic, taken step by step: on numbers it emits the exact top-nprobe even when the stored
   scores are only within eps of the exact ones (margin 2 eps, exact re-evaluation of the listed rows); on NaN / +-inf
   every id it emits still lies in [0, C);
 * Eq. 5 decided from approximate scores (sure / open rows, open rows re-evaluated) equals Eq. 5 on the exact scores."""
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


# ----------------------------------------------------------------------------------------------------------------------
# The probe kernel's list logic for one query token, step by step as the kernel takes it (Section 4.1: the nprobe best
# centroids of a token, ties -> smaller id), for exact scores and for approximate ones (every entry within eps of the
# exact one, decisions completed by exact re-evaluation).  What the model must show:
#   * numbers in: the ids it emits are the exact top-nprobe, whatever the approximation does inside its bound, with
#     tie groups longer than either list;
#   * anything in (NaN, +-inf, block maxima that contradict the scores): every emitted id lies in [0, C).
# ----------------------------------------------------------------------------------------------------------------------
TAIL_SEL, TAIL_XCAP, KEY_MAX = 16, 32, (1 << 64) - 1


def _key(score, cid):
    """(score descending, id ascending) as one ascending 64-bit key; the two zeros tie."""
    u = int(np.array([np.float32(score) + np.float32(0.0)], np.float32).view(np.uint32)[0])
    u ^= 0xFFFFFFFF if u >> 31 else 0x80000000
    return ((~u & 0xFFFFFFFF) << 32) | int(cid)


def _insert_desc(top, v):   # keeps the len(top) largest; a NaN never compares greater and never enters
    if v > top[-1]:
        for j in range(len(top) - 1, -1, -1):
            if v > top[j]:
                if j + 1 < len(top):
                    top[j + 1] = top[j]
                top[j] = v


def _insert_key(best, key):
    if key < best[-1]:
        for j in range(len(best) - 1, -1, -1):
            if key < best[j]:
                if j + 1 < len(best):
                    best[j + 1] = best[j]
                best[j] = key


def _tail_model(S, bmax, exact, tile_rows, nprobe, NP, margin):
    """S: the stored scores of one token [C]; bmax: the stored block maxima [nblk]; exact: the exact scores (None: S is
    exact and margin = 0).  Returns the nprobe emitted ids."""
    C, nblk = len(S), len(bmax)
    ninf = np.float32(-np.inf)
    with np.errstate(invalid="ignore"):
        top = [ninf] * NP
        for b in range(nblk):
            _insert_desc(top, bmax[b])
        T = ninf
        for r in range(min(NP, nprobe)):      # "the maximum, its first holder drops it", nprobe times
            T = top[0]
            top = top[1:] + [ninf]
        T = np.float32(T - np.float32(margin))
        sel = [b for b in range(nblk) if bmax[b] >= T]
        blocks = sel if len(sel) <= TAIL_SEL else [b for b in range(nblk) if bmax[b] >= T]   # the long form walks all
        rows = [c for b in blocks for c in range(b * tile_rows, min(C, (b + 1) * tile_rows))]
        best = [KEY_MAX] * NP
        if exact is None:
            for c in rows:
                _insert_key(best, _key(S[c], c))
        else:
            listed = [c for c in rows if S[c] >= T]           # at most one per lane, else evaluated as they are met:
            for c in listed:                                  # either way every such row is ranked by its exact score
                _insert_key(best, _key(exact[c], c))
    return [j if best[j] == KEY_MAX else best[j] & 0xFFFFFFFF for j in range(nprobe)]


def _block_max(col, rows):
    nblk = (len(col) + rows - 1) // rows
    return np.array([np.fmax.reduce(col[b * rows:(b + 1) * rows], initial=np.float32(-np.inf)) for b in range(nblk)],
                    np.float32)


@pytest.mark.parametrize("seed", range(8))
def test_tail_list_logic_matches_the_exact_ranking(seed):
    rng = np.random.default_rng(100 + seed)
    eps = np.float32(2.0 ** -16)
    for C, rows, nprobe in [(700, 32, 1), (700, 32, 2), (2100, 32, 4), (257, 32, 8), (90, 64, 3), (5, 32, 5), (1, 32, 1)]:
        NP = 1 << (nprobe - 1).bit_length()
        exact = (rng.standard_normal(C) * 0.2).astype(np.float32)
        mode = seed % 4
        if mode == 1:                      # many exact ties, across blocks, more than either list holds
            exact = (np.round(exact * 4) / 4).astype(np.float32)
        elif mode == 2:                    # a crowd within a fraction of eps below the best score
            top = exact.max()
            crowd = rng.choice(C, size=min(C, 40), replace=False)
            exact[crowd] = top - (rng.random(len(crowd)) * eps * 0.9).astype(np.float32)
        elif mode == 3:
            exact[:] = np.float32(0.25)    # everything ties: ids decide
        want = _top(exact, np.arange(C), nprobe)
        # exact scores stored
        got = _tail_model(exact, _block_max(exact, rows), None, rows, nprobe, NP, 0.0)
        np.testing.assert_array_equal(got, want[:nprobe] if C >= nprobe else got)
        # approximate scores stored: random errors, and the adversarial one that lifts the losers and sinks the winners
        for adversarial in (False, True):
            err = (rng.uniform(-1, 1, C) * eps).astype(np.float32)
            if adversarial:
                err[:] = eps
                err[want] = -eps
            approx = (exact.astype(np.float64) + err * 0.999).astype(np.float32)
            assert np.all(np.abs(approx.astype(np.float64) - exact) <= eps)
            got = _tail_model(approx, _block_max(approx, rows), exact, rows, nprobe, NP, 2 * eps)
            if C >= nprobe:
                np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("seed", range(6))
def test_tail_list_logic_never_emits_an_id_out_of_range(seed):
    rng = np.random.default_rng(200 + seed)
    special = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 3e38, -3e38], np.float32)
    for C, rows, nprobe in [(300, 32, 1), (300, 32, 2), (300, 32, 8), (70, 64, 4), (8, 32, 8), (1, 32, 1)]:
        NP = 1 << (nprobe - 1).bit_length()
        for trial in range(6):
            S = rng.standard_normal(C).astype(np.float32)
            share = (0.0, 0.02, 0.5, 1.0)[trial % 4]
            hit = rng.random(C) < share
            S[hit] = rng.choice(special, size=int(hit.sum()))
            if trial == 4:
                S[:] = np.nan              # what a query holding a NaN produces: every score is NaN
            bmax = _block_max(S, rows)
            if trial == 5:                 # block maxima that contradict the scores (cannot happen; must still be safe)
                bmax = rng.choice(special, size=len(bmax)).astype(np.float32)
            exact = rng.standard_normal(C).astype(np.float32)
            exact[rng.random(C) < share] = np.nan
            for ex, margin in ((None, 0.0), (exact, 2.0 ** -15)):
                ids = _tail_model(S, bmax, ex, rows, nprobe, NP, margin)
                assert len(ids) == nprobe
                assert all(0 <= int(c) < max(C, nprobe) for c in ids)
                if nprobe <= C:
                    assert all(0 <= int(c) < C for c in ids)


def test_pruning_map_from_approximate_scores_is_the_exact_one():
    """Eq. 5 on approximate scores: a row is kept for sure when an entry reaches t_cs + eps, left open when one reaches
    t_cs - eps, and an open row is decided by the exact values of its entries that reach t_cs - eps."""
    rng = np.random.default_rng(7)
    eps = np.float32(2.0 ** -16)
    for t_cs in (np.float32(0.45), np.float32(0.0), np.float32(-0.3)):
        t_lo = np.nextafter(np.float32(t_cs - eps), np.float32(-np.inf))
        t_hi = np.nextafter(np.float32(t_cs + eps), np.float32(np.inf))
        exact = (rng.standard_normal((4000, 32)) * 0.3).astype(np.float32)
        near = rng.random(exact.shape) < 0.05      # many entries within a few eps of the threshold, on both sides
        exact[near] = (t_cs + rng.uniform(-3, 3, int(near.sum())) * eps).astype(np.float32)
        exact[rng.random(exact.shape) < 0.01] = t_cs   # and exactly on it (Eq. 5 is inclusive)
        for sign in (-1.0, 1.0, 0.0):
            err = (sign if sign else rng.uniform(-1, 1, exact.shape)) * eps * 0.999
            approx = (exact.astype(np.float64) + err).astype(np.float32)
            sure = (approx >= t_hi).any(axis=1)
            maybe = (approx >= t_lo).any(axis=1) & ~sure
            decided = ((approx >= t_lo) & (exact >= t_cs)).any(axis=1)
            keep = sure | (maybe & decided)
            np.testing.assert_array_equal(keep, (exact >= t_cs).any(axis=1))
