"""Pins for the oracle's expert correlation table (path length 1, paper Section 6.2).

The paper prints no numbers for its table example (the figure is an image), so nothing here is
compared with values of the paper: the table update is pinned against a library histogram and a
hand count, the prediction against closed forms (a deterministic expert-to-expert map, a single
observed row, uniform rows) and against an exact rational evaluation.
"""
from fractions import Fraction

import numpy as np

from oracle import ref


def rand_idx(rng, N, k, E):
    return np.stack([rng.permutation(E)[:k] for _ in range(N)]).astype(np.int32)


def test_update_matches_histogram2d_and_accumulates():
    rng = np.random.default_rng(0)
    E, k, N = 7, 3, 50
    a, b = rand_idx(rng, N, k, E), rand_idx(rng, N, k, E)
    t = np.zeros((E, E), dtype=np.int64)
    ref.corr_update(t, a, b)
    pairs_p = np.repeat(a, k, axis=1).ravel()          # every (prev slot, cur slot) pair of a token
    pairs_c = np.tile(b, (1, k)).ravel()
    want, _, _ = np.histogram2d(pairs_p, pairs_c, bins=[np.arange(E + 1), np.arange(E + 1)])
    assert np.array_equal(t, want.astype(np.int64))
    assert t.sum() == N * k * k
    assert np.array_equal(t.sum(axis=1), np.bincount(a.ravel(), minlength=E) * k)
    ref.corr_update(t, a, b)                            # a second identical batch group doubles it
    assert np.array_equal(t, 2 * want.astype(np.int64))


def test_update_hand_count():
    # 2 tokens, top-2, 3 experts: token 0 goes {0,1} -> {2,0}, token 1 goes {1,2} -> {1,0}
    t = np.zeros((3, 3), dtype=np.int64)
    ref.corr_update(t, [[0, 1], [1, 2]], [[2, 0], [1, 0]])
    assert t.tolist() == [[1, 0, 1], [2, 1, 1], [1, 1, 0]]


def test_predict_deterministic_map_recovers_permuted_counts():
    """If every token's next experts are a fixed permutation of its previous ones (top-1), the
    score of pi(p) is exactly the number of tokens on p, so the prediction is the true ranking."""
    rng = np.random.default_rng(1)
    E = 16
    pi = rng.permutation(E)
    t = np.zeros((E, E), dtype=np.int64)
    for _ in range(3):                                  # warm-up batch groups
        prev = rng.integers(0, E, size=(200, 1)).astype(np.int32)
        ref.corr_update(t, prev, pi[prev].astype(np.int32))
    counts = np.zeros(E, dtype=np.int32)
    counts[[3, 5, 8, 13]] = [40, 7, 19, 40]            # all four were seen in warm-up? make sure
    seen = t.sum(axis=1) > 0
    assert seen[[3, 5, 8, 13]].all()
    experts, score = ref.corr_predict(t, counts, K=3)
    want_score = np.zeros(E)
    want_score[pi[[3, 5, 8, 13]]] = [40, 7, 19, 40]
    assert np.array_equal(score, want_score)            # frequencies are exactly 1.0
    first_two = sorted([pi[3], pi[13]])                 # equal scores: lower index first
    assert experts.tolist() == [first_two[0], first_two[1], pi[8]]


def test_predict_single_row_and_unseen_rows():
    E = 5
    t = np.zeros((E, E), dtype=np.int64)
    t[2] = [1, 0, 3, 0, 4]                              # only expert 2 was ever observed
    experts, score = ref.corr_predict(t, [9, 9, 8, 9, 9], K=5)
    assert np.array_equal(score, 8 * np.array([1, 0, 3, 0, 4]) / 8.0)
    assert experts.tolist() == [4, 2, 0]                # zero scores are never prefetched
    experts, score = ref.corr_predict(t, [9, 9, 0, 9, 9], K=2)
    assert experts.size == 0 and not score.any()        # nothing known about the active experts


def test_predict_uniform_rows_give_equal_scores_and_index_order():
    E = 6
    t = np.full((E, E), 5, dtype=np.int64)
    experts, score = ref.corr_predict(t, [1, 2, 3, 4, 5, 6], K=4)
    assert np.allclose(score, 21 / 6) and experts.tolist() == [0, 1, 2, 3]


def test_predict_against_exact_rationals():
    rng = np.random.default_rng(2)
    E = 9
    t = rng.integers(0, 50, size=(E, E)).astype(np.int64)
    t[4] = 0
    counts = rng.integers(0, 30, size=E).astype(np.int32)
    experts, score = ref.corr_predict(t, counts, K=E)
    exact = [sum(Fraction(int(counts[p]) * int(t[p, e]), int(t[p].sum()))
                 for p in range(E) if counts[p] > 0 and t[p].sum() > 0) for e in range(E)]
    assert np.allclose(score, [float(x) for x in exact], rtol=1e-14, atol=0)
    order = sorted([e for e in range(E) if exact[e] > 0], key=lambda e: (-exact[e], e))
    # the fp64 ranking may differ from the exact one only where two exact scores nearly coincide
    distinct = all(abs(float(exact[order[i]] - exact[order[i + 1]])) > 1e-9 for i in range(len(order) - 1))
    assert distinct and experts.tolist() == order
    assert abs(float(sum(exact)) - float(sum(int(counts[p]) for p in range(E) if t[p].sum() > 0))) < 1e-9
