"""Pins for the oracle's L1 ranking, kept lists and gathers (Section 3.5 of the paper:
filters are scored by the sum of absolute weights and pruned from the smallest)."""
import numpy as np
import pytest

from paper_2207_01260_amd import synth


def test_scores_closed_form_dyadic(orc):
    # every weight +-2^-m: the score is exactly n * 2^-m
    w = np.empty((5, 4, 3, 3), np.float32)
    sign = np.where(synth.uniform01(3, w[0].size) < 0.5, -1.0, 1.0).reshape(4, 3, 3)
    for j in range(5):
        w[j] = sign * 2.0 ** -(j + 1)
    s = orc.l1_scores(w)
    assert s.tolist() == [36 * 2.0 ** -(j + 1) for j in range(5)]


def test_scores_hand(orc):
    w = np.array([[1, -2, 3], [0, 0, 0], [-0.5, 0.25, -0.125]], np.float32).reshape(3, 3, 1, 1)
    assert orc.l1_scores(w).tolist() == [6.0, 0.0, 0.875]


def test_rank_hand_example(orc):
    scores = np.array([3.0, 9.0, 1.0, 7.0, 5.0])
    order, kept = orc.rank(scores, 3)
    assert order.tolist() == [1, 3, 4, 0, 2]          # descending score
    assert kept.tolist() == [1, 3, 4]                  # ascending index
    order, kept = orc.rank(scores, 4)
    assert kept.tolist() == [0, 1, 3, 4]


def test_rank_ties_lower_index_first(orc):
    scores = np.array([2.0, 5.0, 2.0, 5.0, 2.0, 1.0])
    order, kept = orc.rank(scores, 3)
    assert order.tolist() == [1, 3, 0, 2, 4, 5]
    assert kept.tolist() == [0, 1, 3]
    # duplicated filters: the copy with the lower index survives
    w = synth.tensor_normal((4, 3, 3, 3), 40)
    w2 = np.concatenate([w, w[1:2], w[1:2]])           # filters 4, 5 copy filter 1
    s, order, kept = orc.rank_filters(w2, 1)
    pos = order.tolist()
    assert pos.index(1) < pos.index(4) < pos.index(5)


def test_rank_matches_brute_force_selection(orc):
    for c in (1, 2, 7, 33):
        s = synth.uniform01(41 + c, c)
        s[c // 2] = s[0]                                # plant a tie
        order, _ = orc.rank(s, c)
        left = list(range(c))
        expect = []
        while left:                                     # repeated arg-max, first maximum wins
            best = left[0]
            for j in left[1:]:
                if s[j] > s[best]:
                    best = j
            expect.append(best)
            left.remove(best)
        assert order.tolist() == expect


def test_kept_invariants_and_nesting(orc):
    w = synth.tensor_normal((40, 6, 3, 3), 42)
    s = orc.l1_scores(w)
    prev = set()
    for k in range(1, 41):
        order, kept = orc.rank(s, k)
        assert kept.size == k and np.all(np.diff(kept) > 0)
        pruned = sorted(set(range(40)) - set(kept.tolist()))
        if pruned:
            assert s[kept].min() >= s[pruned].max()
        assert prev <= set(kept.tolist())               # top-k sets are nested
        prev = set(kept.tolist())
    assert sorted(order.tolist()) == list(range(40))


def test_scaling_by_two_keeps_order(orc):
    w = synth.tensor_normal((30, 5, 3, 3), 43)
    _, o1, k1 = orc.rank_filters(w, 11)
    _, o2, k2 = orc.rank_filters(w * np.float32(2.0), 11)
    assert np.array_equal(o1, o2) and np.array_equal(k1, k2)


def test_scores_against_numpy_sum(orc):
    w = synth.tensor_normal((16, 64, 3, 3), 44)
    ref = np.abs(w.astype(np.float64)).reshape(16, -1).sum(axis=1)
    assert np.max(np.abs(orc.l1_scores(w) - ref) / ref) < 1e-13


def test_rank_rejects_bad_keep(orc):
    with pytest.raises(ValueError):
        orc.rank(np.ones(4), 0)
    with pytest.raises(ValueError):
        orc.rank(np.ones(4), 5)


def test_gather_weights_is_fancy_indexing(orc):
    w = synth.tensor_normal((9, 7, 3, 3), 45)
    ko = np.array([0, 3, 4, 8], np.int32)
    ki = np.array([1, 2, 6], np.int32)
    assert np.array_equal(orc.gather_weights(w, ko, ki), w[ko][:, ki])
    assert np.array_equal(orc.gather_weights(w, ko, None), w[ko])
    assert np.array_equal(orc.gather_weights(w, None, ki), w[:, ki])
    assert np.array_equal(orc.gather_weights(w, None, None), w)
    # permutation then inverse permutation is the identity
    perm = np.array([3, 0, 6, 1, 5, 2, 4], np.int32)
    inv = np.argsort(perm).astype(np.int32)
    assert np.array_equal(orc.gather_weights(orc.gather_weights(w, None, perm), None, inv), w)


def test_gather_channels(orc):
    x = synth.tensor_normal((2, 6, 3, 4), 46)
    idx = np.array([0, 2, 5], np.int32)
    assert np.array_equal(orc.gather_channels(x, idx), x[:, idx])


def test_drop_filter_equals_zero_then_slice_single_layer(orc):
    x = synth.tensor_normal((2, 4, 6, 6), 47, 1)
    w = synth.tensor_normal((5, 4, 3, 3), 47, 2)
    full = orc.conv2d_f64(x, w, 1, 1)
    keep = np.array([0, 1, 3, 4], np.int32)
    pruned = orc.conv2d_f64(x, orc.gather_weights(w, keep, None), 1, 1)
    assert np.array_equal(pruned, full[:, keep])


def test_drop_filter_two_layers_bit_exact(orc):
    # zero channel j of layer 1's output and run the full layer 2, versus dropping filter j
    # and gathering layer 2's input channels: identical bits (the zero channel adds exact 0.0
    # and the kept list is ascending, so the surviving terms are summed in the same order)
    x = synth.tensor_normal((1, 3, 6, 6), 48, 1)
    w1 = synth.tensor_normal((6, 3, 3, 3), 48, 2)
    w2 = synth.tensor_normal((4, 6, 3, 3), 48, 3)
    b1 = np.zeros(6, np.float32)
    a1 = orc.conv2d_bias_act(x, w1, b1, 1, 1, 1, synth.ACT_RELU)
    for j in range(6):
        keep = np.array([i for i in range(6) if i != j], np.int32)
        a1z = a1.copy()
        a1z[:, j] = 0.0
        full = orc.conv2d_f64(a1z, w2, 1, 1)
        a1p = orc.conv2d_bias_act(x, orc.gather_weights(w1, keep, None), b1[keep], 1, 1, 1,
                                  synth.ACT_RELU)
        pruned = orc.conv2d_f64(a1p, orc.gather_weights(w2, None, keep), 1, 1)
        assert np.array_equal(full, pruned)


def test_group_scores_are_sums_of_member_norms(orc):
    """A group's channel score is the sum of the members' filter norms; one member alone is the
    plain score; the group ranking can differ from every member's own."""
    a = np.zeros((3, 2, 1, 1), np.float32)
    b = np.zeros((3, 1, 3, 3), np.float32)
    a[0] = 1.0; a[1] = 0.5; a[2] = 0.25          # norms 2, 1, 0.5
    b[0] = 0.0; b[1] = 0.125; b[2] = 1.0         # norms 0, 1.125, 9
    s = orc.group_scores([a, b])
    assert s.tolist() == [2.0, 2.125, 9.5]
    assert np.array_equal(orc.group_scores([a]), orc.l1_scores(a))
    _, kept = orc.rank(s, 2)
    assert kept.tolist() == [1, 2]               # member a alone would keep {0, 1}
    _, _, kept_a = orc.rank_filters(a, 2)
    assert kept_a.tolist() == [0, 1]
    with pytest.raises(ValueError):
        orc.group_scores([a, np.zeros((4, 1, 1, 1), np.float32)])
