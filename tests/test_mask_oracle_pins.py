"""Pins for the mask-generator oracle (Alg. 1, getMask): checked against things other than itself.

* the pooling step against the library routine (torch avg_pool2d, float64) on integer-valued
  scores, where every sum is exact;
* the ranking step against a brute-force rank count written with Python tuples;
* closed forms: a ramp score drops the first pixels; a score that is constant on blocks gives
  masks that are the same picture at every resolution (the propagation property of Sec. 3.1);
* invariants: the exact kept count of Sec. 3.2 (tests/golden/kept_counts.txt), nested masks for
  growing sparsity, ties resolved by pixel index.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import mask_oracle as MO

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def int_score(h, w, seed, hi=1000):
    return np.random.default_rng(seed).integers(0, hi, size=(h, w)).astype(np.float32)


@pytest.mark.parametrize("h,w,ho,wo", [(8, 8, 8, 8), (8, 8, 4, 4), (12, 20, 3, 5), (16, 16, 2, 2),
                                       (9, 9, 4, 4), (15, 10, 7, 3), (7, 7, 1, 1), (224, 224, 7, 7)])
def test_pooling_matches_library_avg_pool(h, w, ho, wo):
    score = int_score(h, w, seed=h * 131 + wo)
    rh, rw = h // ho, w // wo
    want = F.avg_pool2d(torch.from_numpy(score).double()[None, None], (rh, rw), (rh, rw))[0, 0].numpy()
    want = want[:ho, :wo] * (rh * rw)                     # integer scores: the library's mean times the window is the exact sum
    got = MO.layer_score_sums(score, ho, wo)
    assert got.shape == (ho, wo) and got.dtype == np.float64
    assert np.array_equal(got, np.rint(want)) and np.abs(want - np.rint(want)).max() < 1e-6


def brute_force_drop_set(keys, n_drop):
    """Pixel i is dropped when fewer than n_drop pixels come before it in (key, index) order."""
    items = [(float(k), i) for i, k in enumerate(keys.reshape(-1))]
    dropped = set()
    for key_i, i in items:
        before = sum(1 for key_j, j in items if (key_j, j) < (key_i, i))
        if before < n_drop:
            dropped.add(i)
    return dropped


@pytest.mark.parametrize("seed", range(6))
def test_ranking_matches_brute_force_with_many_ties(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 60))
    keys = rng.integers(0, 5, size=n).astype(np.float64)       # few distinct values: ties everywhere
    for n_drop in {0, 1, n // 3, n // 2, n - 1, n}:
        if n_drop < 0:
            continue
        got = set(int(i) for i in MO.rank_pixels(keys, n_drop))
        assert got == brute_force_drop_set(keys, n_drop)


def test_ranking_handles_negative_values_zero_signs_and_infinities():
    keys = np.array([0.0, -0.0, -1.5, np.inf, -np.inf, 2.0, -0.0, 0.0], dtype=np.float64)
    # order: -inf(4), -1.5(2), then the four zeros by index (0, 1, 6, 7), 2.0(5), inf(3)
    assert list(MO.rank_pixels(keys, 8)) == [4, 2, 0, 1, 6, 7, 5, 3]
    assert set(MO.rank_pixels(keys, 3)) == {4, 2, 0}


@pytest.mark.parametrize("h,w,ho,wo", [(8, 8, 8, 8), (8, 8, 4, 4), (12, 18, 4, 6), (9, 9, 4, 4)])
@pytest.mark.parametrize("s", [0.0, 0.25, 0.5, 0.7, 1.0])
def test_ramp_score_drops_the_first_pixels(h, w, ho, wo, s):
    """score[y, x] = y*W + x grows in row-major order, and so does every window sum."""
    score = (np.arange(h * w, dtype=np.float32)).reshape(h, w)
    mask = MO.layer_mask(score, ho, wo, s)
    n = ho * wo
    n_drop = n - MO.kept_pixels(s, n)
    want = np.ones(n, np.uint8)
    want[:n_drop] = 0
    assert mask.dtype == np.uint8 and np.array_equal(mask.reshape(-1), want)


def test_kept_counts_follow_the_golden_table():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "kept_counts.txt")) if l.strip() and not l.startswith("#")]
    assert rows
    for size, s, kept, _kind in rows:
        assert MO.kept_pixels(float(s), int(size)) == int(kept)
    # and the mask really has that many ones
    score = np.random.default_rng(1).random((56, 56), dtype=np.float32)
    for s in (0.0, 0.25, 0.5, 0.7, 0.75):
        m = MO.layer_mask(score, 56, 56, s)
        assert int(m.sum()) == MO.kept_pixels(s, 3136)
    assert int(MO.layer_mask(score, 7, 7, 0.5).sum()) == 25     # 49 * .5 = 24.5 -> 25 kept


def test_masks_are_nested_in_the_sparsity():
    score = np.random.default_rng(5).random((32, 32), dtype=np.float32)
    prev = np.ones((8, 8), np.uint8)
    for s in (0.1, 0.25, 0.5, 0.7, 0.9, 1.0):
        m = MO.layer_mask(score, 8, 8, s)
        assert (m <= prev).all()            # whatever was dropped at a lower sparsity stays dropped
        prev = m
    assert prev.sum() == 0


def test_lowest_scores_are_the_ones_dropped():
    score = np.random.default_rng(9).random((16, 16), dtype=np.float32)
    m = MO.layer_mask(score, 16, 16, 0.5)
    assert score[m == 0].max() < score[m == 1].min()
    # one spot raised above everything survives any sparsity below 1
    score[3, 4] = 10.0
    assert MO.layer_mask(score, 16, 16, 0.99)[3, 4] == 1
    # window sums decide, not single pixels: the 2x2 block holding the big value survives
    assert MO.layer_mask(score, 8, 8, 0.9)[1, 2] == 1


def test_propagated_masks_are_the_same_picture_at_every_resolution():
    """Sec. 3.1: one input-resolution pattern, pooled down, keeps the mask structure across layers.
    With a score that is constant on 4x4 blocks every sum is exact, and the mask of a finer layer is
    the coarser layer's mask blown up."""
    rng = np.random.default_rng(11)
    coarse = rng.permutation(64).astype(np.float32).reshape(8, 8)       # distinct block values
    score = np.kron(coarse, np.ones((4, 4), np.float32))                # 32 x 32 input score
    m8, m16, m32 = MO.get_mask(score, [(8, 8), (16, 16), (32, 32)], 0.25)
    assert np.array_equal(m16, np.kron(m8, np.ones((2, 2), np.uint8)))
    assert np.array_equal(m32, np.kron(m8, np.ones((4, 4), np.uint8)))
    assert int(m8.sum()) == 48 and np.array_equal(m8 == 0, coarse < 16)


def test_get_mask_takes_one_sparsity_per_layer():
    score = np.random.default_rng(3).random((16, 16), dtype=np.float32)
    a, b = MO.get_mask(score, [(16, 16), (8, 8)], [0.5, 0.25])
    assert int(a.sum()) == 128 and int(b.sum()) == 48
    assert np.array_equal(b, MO.layer_mask(score, 8, 8, 0.25))


def test_non_divisible_resolution_uses_the_top_left_corner_of_the_pooled_map():
    score = int_score(9, 9, seed=2)
    sums = MO.layer_score_sums(score, 4, 4)        # ratio 2: pooled map would be 4x4 from the first 8 rows/cols
    assert np.array_equal(sums, score[:8, :8].astype(np.float64).reshape(4, 2, 4, 2).sum(axis=(1, 3)))
    sums = MO.layer_score_sums(score, 5, 5)        # ratio 1: the 5x5 corner of the score itself
    assert np.array_equal(sums, score[:5, :5].astype(np.float64))
