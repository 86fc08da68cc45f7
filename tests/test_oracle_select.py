"""Pins of the oracle's token selection (Section 3.1.2, Algorithm 1 line 3) and pyramid budget (Section 3.1.3
and the appendix paragraph on the pyramid-like allocation) against things other than the oracle itself:
a library sort with explicit tie keys, closed forms for monotone and constant scores, every small case by
exhaustive enumeration, the boundary budgets, and the arithmetic the paper states for the pyramid."""
import itertools

import numpy as np
import pytest

from oracle import ref
from paper_2411_18077_amd import workloads as W


def lexsort_selection(score, k, n_rw):
    """Independent statement of the rule with numpy's lexsort: candidates = all but the last n_rw tokens,
    ordered by (score descending, position ascending); the first k, then the window, by position."""
    L = score.shape[0]
    n_cand = L - n_rw
    pos = np.arange(n_cand)
    order = np.lexsort((pos, -score[:n_cand].astype(np.float64)))
    return np.concatenate([np.sort(order[:k]), np.arange(n_cand, L)]).astype(np.int32)


@pytest.mark.parametrize("kind", ["attention", "ties", "signed"])
@pytest.mark.parametrize("L,k,n_rw", [(1000, 250, 250), (257, 64, 32), (4096, 1024, 1024), (64, 1, 0), (300, 0, 7)])
def test_selection_matches_a_library_sort(kind, L, k, n_rw):
    U = 5
    A = W.make_scores(U, L, seed=11 + L, kind=kind).numpy()
    idx, n_tok = ref.select_hh_rw(A, np.full(U, k), np.full(U, n_rw))
    for u in range(U):
        assert n_tok[u] == k + n_rw
        assert np.array_equal(idx[u, : n_tok[u]], lexsort_selection(A[u], k, n_rw))
        assert (idx[u, n_tok[u]:] == -1).all()              # nothing written beyond the count


def test_ragged_budgets_per_unit():
    U, L = 6, 777
    A = W.make_scores(U, L, seed=5, kind="ties").numpy()
    n_hh = np.array([0, 1, 100, 333, 777, 0], np.int32)
    n_rw = np.array([0, 776, 50, 444, 0, 777], np.int32)
    idx, n_tok = ref.select_hh_rw(A, n_hh, n_rw)
    for u in range(U):
        assert n_tok[u] == n_hh[u] + n_rw[u]
        assert np.array_equal(idx[u, : n_tok[u]], lexsort_selection(A[u], n_hh[u], n_rw[u]))


def test_closed_forms_for_monotone_and_constant_scores():
    L, k, n_rw = 500, 120, 60
    n_cand = L - n_rw
    window = np.arange(n_cand, L)
    inc = np.arange(L, dtype=np.float32)[None]
    idx, n = ref.select_hh_rw(inc, [k], [n_rw])               # largest scores are the latest candidates
    assert np.array_equal(idx[0, : n[0]], np.arange(n_cand - k, L))
    dec = inc[:, ::-1].copy()
    idx, n = ref.select_hh_rw(dec, [k], [n_rw])               # largest scores are the first tokens
    assert np.array_equal(idx[0, : n[0]], np.concatenate([np.arange(k), window]))
    flat = np.full((1, L), 0.25, np.float32)
    idx, n = ref.select_hh_rw(flat, [k], [n_rw])              # all equal: the earliest positions win
    assert np.array_equal(idx[0, : n[0]], np.concatenate([np.arange(k), window]))
    # a huge score inside the recent window must not take a heavy-hitter slot
    a = dec.copy(); a[0, L - 1] = 1e9
    idx, n = ref.select_hh_rw(a, [k], [n_rw])
    assert np.array_equal(idx[0, : n[0]], np.concatenate([np.arange(k), window]))


def test_positive_and_negative_zero_are_equal_scores():
    a = np.array([[-0.0, 0.0, -0.0, 0.0, -1.0, -0.0]], np.float32)
    idx, n = ref.select_hh_rw(a, [3], [0])
    assert idx[0, :3].tolist() == [0, 1, 2]


def test_every_small_case_by_enumeration():
    """All score vectors over {0, 1, 2} of length 1..5 and all budgets: compared with Python's stable sort."""
    for L in range(1, 6):
        vecs = list(itertools.product([0.0, 1.0, 2.0], repeat=L))
        for n_rw in range(L + 1):
            for k in range(L - n_rw + 1):
                A = np.array(vecs, np.float32)
                idx, n = ref.select_hh_rw(A, np.full(len(vecs), k), np.full(len(vecs), n_rw))
                for r, v in enumerate(vecs):
                    cand = sorted(range(L - n_rw), key=lambda i: -v[i])       # stable: ties keep position order
                    want = sorted(cand[:k]) + list(range(L - n_rw, L))
                    assert idx[r, : n[r]].tolist() == want, (v, k, n_rw)


def test_threshold_property():
    """No evicted candidate outranks a kept heavy hitter; equal to the weakest kept one only if later."""
    U, L, k, n_rw = 4, 2048, 512, 256
    A = W.make_scores(U, L, seed=3, kind="ties").numpy()
    idx, n = ref.select_hh_rw(A, np.full(U, k), np.full(U, n_rw))
    for u in range(U):
        kept = idx[u, :k]
        assert (np.diff(idx[u, : n[u]]) > 0).all()
        evicted = np.setdiff1d(np.arange(L - n_rw), kept)
        weakest = A[u, kept].min()
        assert (A[u, evicted] <= weakest).all()
        last_weakest = kept[A[u, kept] == weakest].max()
        assert (evicted[A[u, evicted] == weakest] > last_weakest).all()


def test_heads_of_a_group_are_summed_in_fp32_in_head_order():
    U, rep, L, k, n_rw = 3, 4, 600, 150, 90
    A = W.make_scores(U * rep, L, seed=9, kind="attention").numpy()
    summed = A.reshape(U, rep, L)[:, 0].copy()
    for h in range(1, rep):
        summed = (summed + A.reshape(U, rep, L)[:, h]).astype(np.float32)
    got, n = ref.select_hh_rw(A, np.full(U, k), np.full(U, n_rw), rep=rep)
    want, _ = ref.select_hh_rw(summed, np.full(U, k), np.full(U, n_rw), rep=1)
    assert np.array_equal(got, want)
    # and the sum matters: it differs from selecting on the first head alone
    first, _ = ref.select_hh_rw(A.reshape(U, rep, L)[:, 0].copy(), np.full(U, k), np.full(U, n_rw))
    assert not np.array_equal(got, first)


def test_out_of_range_budgets_give_an_empty_unit_and_leave_the_row_alone():
    L = 50
    A = W.make_scores(6, L, seed=1, kind="attention").numpy()
    n_hh = np.array([-1, 10, 45, 10, 30, 10], np.int32)
    n_rw = np.array([5, -2, 10, 51, 10, 5], np.int32)
    idx, n = ref.select_hh_rw(A, n_hh, n_rw, idx_stride=32)
    assert n.tolist() == [0, 0, 0, 0, 0, 15]                  # unit 4: 40 > idx_stride
    assert (idx[:5] == -1).all()
    assert np.array_equal(idx[5, :15], lexsort_selection(A[5], 10, 5))


def test_empty_prompt_and_no_units():
    idx, n = ref.select_hh_rw(np.zeros((2, 0), np.float32), [0, 0], [0, 0], idx_stride=4)
    assert n.tolist() == [0, 0]
    idx, n = ref.select_hh_rw(np.zeros((0, 8), np.float32), np.zeros(0, np.int32), np.zeros(0, np.int32))
    assert idx.shape == (0, 8)


# ---- pyramid budget ---------------------------------------------------------------------------------

@pytest.mark.parametrize("n_layers,x,d", [(32, 1024.0, 7), (32, 8192.0, 7), (2, 10.0, 7), (40, 333.0, 3), (5, 1.0, 1)])
def test_pyramid_end_points_mean_and_linearity(n_layers, x, d):
    b = ref.pyramid_budget(n_layers, x, d, bottom_heavy=True)
    assert b[0] == pytest.approx(2 * x - x / d, rel=1e-14) and b[-1] == pytest.approx(x / d, rel=1e-14)
    assert b.mean() == pytest.approx(x, rel=1e-13)              # the average heavy budget stays x
    if n_layers > 2:
        assert np.allclose(np.diff(b, 2), 0.0, atol=1e-9 * x)   # linear in the layer index
    assert (np.diff(b) <= 0).all()                              # lower layers hold more
    printed = ref.pyramid_budget(n_layers, x, d, bottom_heavy=False)
    assert np.allclose(printed, b[::-1], rtol=1e-14)            # the appendix formula read literally


def test_pyramid_depth_one_is_uniform_and_single_layer_gets_the_average():
    assert np.allclose(ref.pyramid_budget(12, 100.0, 1), 100.0)
    assert ref.pyramid_budget(1, 77.0, 7).tolist() == [77.0]


def test_pyramid_rejects_bad_arguments():
    for args in [(0, 1.0, 7), (4, -1.0, 7), (4, 1.0, 0)]:
        with pytest.raises(RuntimeError):
            ref.pyramid_budget(*args)
