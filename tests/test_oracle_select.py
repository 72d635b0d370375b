"""Pins for the lazy-layer selection oracle (CPU only): the closed form (largest ratios are
lazy) against the priority-queue procedure of the method section, against numpy sorting,
and on ties and edge cases."""
import itertools

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(302303)


def numpy_topk(r, n_lazy):
    order = np.lexsort((np.arange(len(r)), -np.asarray(r, dtype=np.float64)))   # ratio desc, index asc
    mask = np.zeros(len(r), dtype=np.uint8)
    mask[order[:n_lazy]] = 1
    return mask, order


@pytest.mark.parametrize("L", [1, 2, 7, 32, 64])
def test_queue_procedure_equals_top_k(L):
    for trial in range(20):
        r = RNG.random(L)
        if trial % 3 == 0:                      # plant ties
            r = np.round(r * 4) / 4
        for n_lazy in sorted({0, 1, L // 4, L // 2, L - 1, L}):
            if n_lazy < 0 or n_lazy > L:
                continue
            a, order = oracle.select_lazy(r, n_lazy)
            b, pop_step = oracle.select_lazy_queue(r, n_lazy)
            c, np_order = numpy_topk(r, n_lazy)
            np.testing.assert_array_equal(a, b)
            np.testing.assert_array_equal(a, c)
            np.testing.assert_array_equal(order, np_order)
            assert a.sum() == n_lazy
            assert ((pop_step >= 0) == (a == 1)).all()


def test_queue_never_holds_more_than_p_full_layers():
    """A layer is removed at the push that overflows the queue: at step i at most P layers stay full."""
    L, n_lazy = 16, 8
    P = L - n_lazy
    r = RNG.random(L)
    is_lazy, pop_step = oracle.select_lazy_queue(r, n_lazy)
    for i in range(L):
        still_full = sum(1 for j in range(i + 1) if pop_step[j] < 0 or pop_step[j] > i)
        assert still_full <= P
    # the kept layers are exactly the P lowest ratios
    assert set(np.argsort(r)[:P]) == set(np.nonzero(is_lazy == 0)[0])


def test_exhaustive_small_cases_against_definition():
    """All orderings of 5 layers with tied values: lazy set = argmax-k under (ratio desc, index asc)."""
    vals = [0.1, 0.5, 0.5, 0.9, 0.1]
    for perm in itertools.permutations(range(5)):
        r = np.array([vals[i] for i in perm])
        for k in range(6):
            mask, _ = oracle.select_lazy(r, k)
            ranked = sorted(range(5), key=lambda i: (-r[i], i))
            expect = np.zeros(5, dtype=np.uint8)
            expect[ranked[:k]] = 1
            np.testing.assert_array_equal(mask, expect)


def test_select_rejects_bad_arguments():
    with pytest.raises(ValueError):
        oracle.select_lazy(np.array([0.1, np.nan]), 1)
    with pytest.raises(ValueError):
        oracle.select_lazy(np.array([0.1, 0.2]), 3)
    with pytest.raises(ValueError):
        oracle.select_lazy_queue(np.array([0.1, 0.2]), -1)


def test_paper_settings_half_and_quarter(hyperparams):
    L = 32
    r = RNG.random(L)
    half, _ = oracle.select_lazy(r, int(L * hyperparams["lazy_fraction_longbench"]))
    quarter, _ = oracle.select_lazy(r, int(L * hyperparams["lazy_fraction_niah"]))
    assert half.sum() == 16 and quarter.sum() == 8
    assert ((quarter == 1) <= (half == 1)).all()           # nested: the laziest quarter is inside the laziest half
    assert r[half == 1].min() >= r[half == 0].max()


# ---- LightTransfer-Train pre-selection: per-sample sets -> layer frequencies -> most frequent layers ----

def numpy_preselect(sets, n_lazy):
    count = np.asarray(sets, dtype=np.int64).astype(bool).sum(axis=0)
    order = np.lexsort((np.arange(len(count)), -count))                     # frequency desc, index asc
    mask = np.zeros(len(count), dtype=np.uint8)
    mask[order[:n_lazy]] = 1
    return mask, count


@pytest.mark.parametrize("S,L", [(1, 8), (5, 8), (40, 32), (200, 64)])
def test_preselection_counts_and_picks_most_frequent(S, L):
    for n_lazy in sorted({0, 1, L // 2, L - 1, L}):
        sets = (RNG.random((S, L)) < RNG.random(L)).astype(np.uint8)       # layers with different propensities
        mask, count = oracle.preselect_lazy(sets, n_lazy)
        ref_mask, ref_count = numpy_preselect(sets, n_lazy)
        np.testing.assert_array_equal(count, ref_count)
        np.testing.assert_array_equal(mask, ref_mask)
        assert mask.sum() == n_lazy


def test_preselection_special_cases():
    one = np.array([[0, 1, 1, 0, 1, 0]], dtype=np.uint8)
    mask, count = oracle.preselect_lazy(one, 3)                              # one sample: its own set
    np.testing.assert_array_equal(mask, one[0])
    same = np.repeat(one, 7, axis=0)
    mask, count = oracle.preselect_lazy(same, 3)                             # unanimous samples: that set, count = S
    np.testing.assert_array_equal(mask, one[0])
    np.testing.assert_array_equal(count, 7 * one[0])
    tie = np.array([[1, 0, 1, 0], [0, 1, 0, 1]], dtype=np.uint8)             # all frequencies equal: lowest indices
    mask, _ = oracle.preselect_lazy(tie, 2)
    np.testing.assert_array_equal(mask, [1, 1, 0, 0])
    # per-sample sets chosen by ratio, then pre-selected: a layer that is lazy in most samples wins over one
    # that has the single largest ratio once
    ratios = np.array([[0.9, 0.5, 0.1], [0.2, 0.6, 0.1], [0.3, 0.7, 0.1]])
    sets = np.stack([oracle.select_lazy(r, 1)[0] for r in ratios])
    mask, count = oracle.preselect_lazy(sets, 1)
    np.testing.assert_array_equal(count, [1, 2, 0])
    np.testing.assert_array_equal(mask, [0, 1, 0])
