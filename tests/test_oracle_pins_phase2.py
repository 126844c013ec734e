"""Pins of the oracle's Phase-2 tail and Phase-3 set operations (Sec. 3.5 "Adaptive Granularity", Sec. 3.6, Alg. 1)
against library routines, closed forms, hand cases and brute force with Python sets."""
import numpy as np
import pytest

from oracle import s3_oracle as orc


def test_smoothing_kernels_closed_forms():
    assert np.array_equal(orc.smoothing_kernel("box", 8), np.full(8, 1 / 8))
    assert np.allclose(orc.smoothing_kernel("triangular", 4), np.array([1, 2, 2, 1]) / 6, rtol=1e-15)
    assert np.allclose(orc.smoothing_kernel("triangular", 5), np.array([1, 2, 3, 2, 1]) / 9, rtol=1e-15)
    for K in (8, 48, 7):
        g = orc.smoothing_kernel("gaussian", K)
        assert g.sum() == pytest.approx(1.0, rel=1e-14) and np.allclose(g, g[::-1], rtol=1e-14)
        # ratio of neighbours: exp(-(u_j^2 - u_{j+1}^2) / 2) with u = (j - (K-1)/2) / (K/6)
        j = np.arange(K - 1)
        u0, u1 = (j - (K - 1) / 2) / (K / 6), (j + 1 - (K - 1) / 2) / (K / 6)
        assert np.allclose(g[:-1] / g[1:], np.exp(-0.5 * (u0 ** 2 - u1 ** 2)), rtol=1e-12)
    with pytest.raises(ValueError):
        orc.smoothing_kernel("box", 0)


@pytest.mark.parametrize("K", [1, 2, 8, 9, 48])
def test_conv1d_matches_numpy_convolve(K):
    rng = np.random.default_rng(K)
    L = 200
    S = rng.random(L) * (rng.random(L) < 0.2)                  # sparse, like a score array
    g = rng.random(K)                                           # asymmetric: a flipped or shifted kernel cannot pass
    full = np.convolve(S, g[::-1], "full")                      # library routine
    want = full[K - 1 - K // 2: K - 1 - K // 2 + L]
    assert np.allclose(orc.conv1d(S, g), want, rtol=1e-13, atol=1e-15)
    # an impulse at t puts tap floor(K / 2) on t
    e = np.zeros(201); e[100] = 1.0
    D = orc.conv1d(e, g)
    assert np.array_equal(D[100 - (K - 1 - K // 2): 100 + K // 2 + 1], g[::-1]) and D.sum() == pytest.approx(g.sum())
    # shorter than the kernel: everything that overlaps is summed
    assert np.allclose(orc.conv1d(np.ones(3), np.ones(K)), [min(3, t + K - K // 2) - max(0, t - K // 2) for t in range(3)])


def test_nms_peaks_hand_cases():
    D = np.array([0, 1, 5, 4, 0, 0, 3, 3, 0, 2.0])
    c, v = orc.nms_peaks(D, 10, 1)
    assert c.tolist() == [2, 6, 9] and v.tolist() == [5, 3, 2]          # 3 is suppressed by 2; tie 6/7 -> 6, which suppresses 7
    c, _ = orc.nms_peaks(D, 2, 1)
    assert c.tolist() == [2, 6]
    c, _ = orc.nms_peaks(D, 10, 0)                                       # radius 0: plain descending order of the positive entries
    assert c.tolist() == [2, 3, 6, 7, 9, 1]
    c, _ = orc.nms_peaks(D, 10, 100)
    assert c.tolist() == [2]
    c, _ = orc.nms_peaks(np.zeros(5), 3, 1)                              # nothing positive: no centre
    assert len(c) == 0


def test_nms_peaks_brute_force():
    rng = np.random.default_rng(3)
    for radius in (0, 2, 7):
        D = rng.random(300) * (rng.random(300) < 0.5)
        c, v = orc.nms_peaks(D, 40, radius)
        alive, want = np.ones(300, bool), []
        for _ in range(40):
            cand = np.where(alive, D, -1.0)
            t = int(np.argmax(cand))                                     # first maximum = smallest position
            if cand[t] <= 0:
                break
            want.append(t)
            alive[max(0, t - radius): t + radius + 1] = False
        assert c.tolist() == want and np.array_equal(v, D[want])
        assert all(abs(a - b) > radius for i, a in enumerate(want) for b in want[:i])


def test_grow_spans_hand_cases():
    D = np.array([0.1, 0.6, 0.9, 1.0, 0.5, 0.49, 0.8, 0.0, 0.0, 2.0])
    lo, hi = orc.grow_spans(D, [3], 0.5, 100)
    assert (lo[0], hi[0]) == (1, 4)                                      # 0.5 >= 0.5 stays, 0.49 stops; 0.1 stops on the left
    lo, hi = orc.grow_spans(D, [3], 0.5, 1)
    assert (lo[0], hi[0]) == (2, 4)                                      # at most one position to either side
    lo, hi = orc.grow_spans(D, [9, 0], 0.0, 3)
    assert (lo[0], hi[0]) == (6, 9) and (lo[1], hi[1]) == (0, 3)         # clipped at the ends of the context
    lo, hi = orc.grow_spans(D, [3], 1.0, 100)
    assert (lo[0], hi[0]) == (3, 3)
    lo, hi = orc.grow_spans(D, [3], 0.5, 0)
    assert (lo[0], hi[0]) == (3, 3)


def test_fuse_is_a_set_union():
    rng = np.random.default_rng(8)
    L = 500
    lo = rng.integers(0, L, 12).astype(np.int32)
    hi = (lo + rng.integers(0, 30, 12)).astype(np.int32)               # some run past the end
    extra = rng.integers(-5, L + 5, 40).astype(np.int32)               # some outside [0, L), some repeated
    for lead, tail in ((0, 0), (16, 7), (600, 0)):
        mask, idx = orc.fuse(L, lo, hi, extra, lead, tail)
        want = set()
        for a, b in zip(lo, hi):
            want |= set(range(int(a), min(int(b), L - 1) + 1))
        want |= {int(e) for e in extra if 0 <= e < L}
        want |= set(range(min(lead, L))) | set(range(max(0, L - tail), L))
        assert idx.tolist() == sorted(want) and np.array_equal(np.flatnonzero(mask), idx) and set(np.unique(mask)) <= {0, 1}
    mask, idx = orc.fuse(10, np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32), 2, 3)
    assert idx.tolist() == [0, 1, 7, 8, 9]


# ------------------------------------------------------------------ compact postings (Sec. 3.4 "CPU Index Size")
def _random_csr(rng, n_feat, L, density):
    lists = [np.flatnonzero(rng.random(L) < density * rng.random()).astype(np.int32) for _ in range(n_feat)]
    lists[3] = np.arange(L, dtype=np.int32)                        # a stop feature: in every token
    lists[5] = np.zeros(0, np.int32)                               # an empty list
    offsets = np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32)
    return lists, offsets, np.concatenate(lists).astype(np.int32)


def test_compact_postings_hand_case():
    # block size 4 (block_log2 = 2), 2 blocks, 3 features: lists [1, 2, 5], [], [0, 4, 6, 7]
    offsets = np.array([0, 3, 3, 7], np.int32)
    positions = np.array([1, 2, 5, 0, 4, 6, 7], np.int32)
    cstart, delta, cfreq = orc.compact_encode(offsets, positions, 2, block_log2=2)
    # block 0: f0 -> 1, 2; f1 -> none; f2 -> 0.  block 1: f0 -> 5 - 4; f2 -> 4 - 4, 6 - 4, 7 - 4
    assert cstart.tolist() == [0, 2, 2, 3, 4, 4, 7] and delta.tolist() == [1, 2, 0, 1, 0, 2, 3] and cfreq.tolist() == [3, 0, 4]
    off2, pos2 = orc.compact_decode(cstart, delta, 3, 2, block_log2=2)
    assert np.array_equal(off2, offsets) and np.array_equal(pos2, positions)
    cstart, delta, cfreq = orc.compact_encode(offsets, positions, 2, block_log2=2, prune_freq=3)    # strict >: the list of 4 goes
    assert cstart.tolist() == [0, 2, 2, 2, 3, 3, 3] and delta.tolist() == [1, 2, 1] and cfreq.tolist() == [3, 0, 0]
    with pytest.raises(ValueError):
        orc.compact_encode(offsets, np.array([2, 1, 5, 0, 4, 6, 7], np.int32), 2, block_log2=2)     # not ascending
    with pytest.raises(ValueError):
        orc.compact_encode(offsets, positions, 1, block_log2=2)                                      # beyond the blocks


def test_compact_postings_round_trip_brute_force():
    rng = np.random.default_rng(17)
    n_feat, L, blk = 40, 1000, 7                                   # blocks of 128 positions, 8 blocks
    lists, offsets, positions = _random_csr(rng, n_feat, L, 0.2)
    nblk = (L + (1 << blk) - 1) >> blk
    for prune in (0, 150):
        cstart, delta, cfreq = orc.compact_encode(offsets, positions, nblk, block_log2=blk, prune_freq=prune)
        kept = [l if not (prune > 0 and len(l) > prune) else l[:0] for l in lists]
        assert cfreq.tolist() == [len(l) for l in kept] and len(delta) == sum(len(l) for l in kept)    # 2 bytes per kept posting
        assert delta.max() < (1 << blk) and np.all(np.diff(cstart) >= 0) and cstart[0] == 0 and cstart[-1] == len(delta)
        # every segment, from the definition: postings of list f that lie in block b, as offsets from the block's start
        for b in range(nblk):
            for f in range(n_feat):
                seg = delta[cstart[b * n_feat + f]: cstart[b * n_feat + f + 1]]
                want = kept[f][(kept[f] >> blk) == b] - (b << blk)
                assert np.array_equal(seg, want)
        off2, pos2 = orc.compact_decode(cstart, delta, n_feat, nblk, block_log2=blk)
        assert np.array_equal(off2, np.concatenate([[0], np.cumsum([len(l) for l in kept])]))
        assert np.array_equal(pos2, np.concatenate(kept))
    assert prune and lists[3].shape[0] > prune                     # the stop feature was really dropped
