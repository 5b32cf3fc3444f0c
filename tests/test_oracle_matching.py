"""Pins for the oracle's bipartite soft matching (Sec. 4.1.2, Appendix A) with the distance of Eq. (5) and
with the plain L2 distance of the benchmark configurations: the distance against the merging error it
is defined to measure (computed through the oracle's own, independent assembly code), brute force on
tiny inputs, cases worked by hand including ties; and the threshold rule of the configurations."""
import numpy as np
import pytest

from oracle import calibrate


def test_distance_is_the_output_error_of_merging(oracle):
    """Eq. (5) is the error Eq. (4) leaves in the layer's output.  Merge one pair with the oracle's
    literal assembly (activations averaged, weight rows summed) and compare ||Y - Y^||_F^2 with
    D(i, j).  Small dyadic values keep every fp32 step exact."""
    rng = np.random.default_rng(3)
    C, N, O = 12, 5, 4
    y = (rng.integers(-8, 9, (N, C)) / 4.0).astype(np.float32)
    W = (rng.integers(-8, 9, (C, O)) / 2.0).astype(np.float32)
    T = np.ones(C, np.int32)
    for a_idx, b_idx in [(0, 0), (2, 5), (5, 1)]:
        i, j = 2 * a_idx, 2 * b_idx + 1                   # channels (positions: nothing is split)
        y_hat = oracle.assemble(oracle.disassemble(y, T), [a_idx], [b_idx])
        W_hat = oracle.reassemble_weight(W, T, [a_idx], [b_idx])
        err = y.astype(np.float64) @ W.astype(np.float64) - y_hat.astype(np.float64) @ W_hat.astype(np.float64)
        assert (err * err).sum() == calibrate.pair_distance(y[:, i], y[:, j], W[i], W[j])


def test_distance_properties():
    rng = np.random.default_rng(4)
    xi, xj, wi, wj = rng.standard_normal(7), rng.standard_normal(7), rng.standard_normal(5), rng.standard_normal(5)
    d = calibrate.pair_distance(xi, xj, wi, wj)
    assert d > 0
    assert np.isclose(d, calibrate.pair_distance(xj, xi, wj, wi), rtol=1e-14)          # symmetric
    assert calibrate.pair_distance(xi, xi, wi, wj) == 0.0                                # same activations: no error
    assert calibrate.pair_distance(xi, xj, wi, wi) == 0.0                                # same weights: no error
    assert np.isclose(calibrate.pair_distance(3 * xi, 3 * xj, wi, wj), 9 * d, rtol=1e-14)
    # the rank-one structure: |u v^T|_F^2 = |u|^2 |v|^2
    assert np.isclose(d, 0.25 * ((xi - xj) ** 2).sum() * ((wi - wj) ** 2).sum(), rtol=1e-13)


def test_nearest_by_eq5_against_brute_force():
    rng = np.random.default_rng(5)
    C, N, O = 31, 6, 5
    y = rng.standard_normal((N, C)).astype(np.float32)
    W = rng.standard_normal((C, O)).astype(np.float32)
    T = np.ones(C, np.int32)
    T[[4, 17]] = [3, 2]                                   # their sub-channels take no part
    best_j, best_d, pos_a, pos_b = calibrate.nearest_by_eq5(y, W, T)
    chan_of = np.repeat(np.arange(C), T)
    assert not np.isin(chan_of[pos_a], [4, 17]).any() and not np.isin(chan_of[pos_b], [4, 17]).any()
    assert pos_a.size + pos_b.size == C - 2 and np.all(pos_a % 2 == 0) and np.all(pos_b % 2 == 1)
    for k, pa in enumerate(pos_a):
        i = chan_of[pa]
        ds = [calibrate.pair_distance(y[:, i], y[:, chan_of[pb]], W[i], W[chan_of[pb]]) for pb in pos_b]
        assert int(np.argmin(ds)) == best_j[k]
        assert np.isclose(best_d[k], min(ds), rtol=1e-12)
    # a subset of rows gives the same answers
    sub_j, sub_d, _, _ = calibrate.nearest_by_eq5(y, W, T, rows=[3, 0, 9])
    assert sub_j.tolist() == best_j[[3, 0, 9]].tolist() and np.array_equal(sub_d, best_d[[3, 0, 9]])


def test_matching_by_hand():
    """Six channels, one token, one output feature: D(i, j) = (x_i - x_j)^2 (w_i - w_j)^2 / 4.
    A = channels 0, 2, 4; B = 1, 3, 5."""
    y = np.array([[1.0, 1.0, 5.0, 4.0, 9.0, 2.0]], np.float32)
    W = np.array([[1.0], [3.0], [2.0], [2.0], [0.0], [7.0]], np.float32)
    T = np.ones(6, np.int32)
    best_j, best_d, pos_a, pos_b = calibrate.nearest_by_eq5(y, W, T)
    # channel 0: to 1: 0; to 3: 9*1/4; to 5: 1*36/4  -> B-member 0, distance 0
    # channel 2: to 1: 16*1/4 = 4; to 3: 1*0/4 = 0; to 5: 9*25/4 -> B-member 1, distance 0
    # channel 4: to 1: 64*9/4 = 144; to 3: 25*4/4 = 25; to 5: 49*49/4 -> B-member 1, distance 25
    assert best_j.tolist() == [0, 1, 1] and best_d.tolist() == [0.0, 0.0, 25.0]
    src_idx, dst_idx = calibrate.select_edges(best_d, best_j, pos_a, pos_b, 2)
    assert src_idx.tolist() == [0, 1] and dst_idx.tolist() == [0, 1]     # the tie of the two zeros: both taken
    src_idx, dst_idx = calibrate.select_edges(best_d, best_j, pos_a, pos_b, 1)
    assert src_idx.tolist() == [0] and dst_idx.tolist() == [0]           # tie: the lower A index
    src_idx, dst_idx = calibrate.match_pairs_eq5(y, W, T, 3)
    assert src_idx.tolist() == [0, 1, 2] and dst_idx.tolist() == [0, 1, 1]   # two sources may share a destination


def test_matching_prefers_pairs_that_cost_nothing():
    """Channels built in identical pairs (same activations, same weights) across the two sets are found
    and merged first, and merging them leaves the layer's output unchanged."""
    rng = np.random.default_rng(6)
    C, N, O = 40, 16, 8
    y = rng.standard_normal((N, C)).astype(np.float32)
    W = rng.standard_normal((C, O)).astype(np.float32)
    twins = [(0, 7), (10, 3), (22, 39)]                   # (even channel, odd channel)
    for a, b_ in twins:
        y[:, b_] = y[:, a]
        W[b_] = W[a]
    T = np.ones(C, np.int32)
    src_idx, dst_idx = calibrate.match_pairs_eq5(y, W, T, 3)
    assert sorted(zip((2 * src_idx).tolist(), (2 * dst_idx + 1).tolist())) == sorted(twins)


def test_theta_grid_is_algorithm_1():
    m = np.array([0.5, 2.0, 8.5, 1.0], np.float32)
    assert calibrate.theta_grid(m, 4) == [2.5, 4.5, 6.5, 8.5]          # min + p/P (max - min)
    assert calibrate.theta_grid(m, 1) == [8.5]                          # p = P: nothing is disassembled


def test_grid_search_prefers_reassembly_when_there_are_outliers(oracle):
    """Algorithm 1 on a small layer with massive outlier channels at 4 bits: the last grid point
    (theta = max: no disassembly, plain quantization) must lose against some smaller theta, and the loss
    reported for a theta is the squared output error of exactly that reassembled, quantized layer."""
    rng = np.random.default_rng(12)
    N, C, O = 48, 96, 40
    x = rng.standard_normal((N, C)).astype(np.float32)
    x[:, [5, 40, 77]] *= np.array([30.0, 55.0, 24.0], np.float32)
    W = (rng.standard_normal((C, O)) / np.sqrt(C)).astype(np.float32)
    theta, thetas, losses = calibrate.grid_search_theta(x, 0, None, None, 0.0, W, 4, 4, 8, n_match_tokens=N)
    assert len(losses) == 8 and theta == thetas[int(np.argmin(losses))]
    assert min(losses) < 0.7 * losses[-1] and theta < thetas[-1]
    # the last grid point is the layer without reassembly
    loss_plain, T, src_idx, dst_idx = calibrate.reassembly_loss(x, 0, None, None, 0.0, W, thetas[-1], 4, 4, N)
    assert np.all(T == 1) and src_idx.size == 0 and loss_plain == losses[-1]
    wq = oracle.quantize_weight(W, 4)
    plain = oracle.reassembled_linear(x, 0, None, None, 0.0, np.ones(C, np.int32), [], [], 4, wq)["y"]
    ref = x.astype(np.float64) @ W.astype(np.float64)
    assert np.isclose(((plain - ref) ** 2).sum(), loss_plain, rtol=1e-12)


# ---------------------------------------------------------------- plain L2 matching (the configurations' "nearest-L2 pairs")

def test_l2_matching_by_hand():
    """Six channels, two tokens.  A = channels 0, 2, 4; B = 1, 3, 5.  Squared distances, token by token:
         channel 0 = (0, 0): to 1 = (3, 4): 25;  to 3 = (0, 5): 25;  to 5 = (1, 1): 2    -> B-member 2, distance 2
         channel 2 = (3, 0): to 1: 0 + 16 = 16;  to 3: 9 + 25 = 34;  to 5: 4 + 1 = 5     -> B-member 2, distance 5
         channel 4 = (0, 1): to 1: 9 + 9 = 18;   to 3: 0 + 16 = 16;  to 5: 1 + 0 = 1     -> B-member 2, distance 1
       and with channel 5 moved to (6, 8): channel 0 sees 25, 25, 100: a tie, which goes to the LOWER member."""
    y = np.array([[0, 3, 3, 0, 0, 1], [0, 4, 0, 5, 1, 1]], np.float32)
    T = np.ones(6, np.int32)
    best_j, best_d, pos_a, pos_b = calibrate.nearest_by_l2(y, T)
    assert best_j.tolist() == [2, 2, 2] and best_d.tolist() == [2.0, 5.0, 1.0]
    assert pos_a.tolist() == [0, 2, 4] and pos_b.tolist() == [1, 3, 5]
    src_idx, dst_idx = calibrate.nearest_pairs(y, T, 2)                 # the two shortest edges: from channels 4 and 0
    assert src_idx.tolist() == [0, 2] and dst_idx.tolist() == [2, 2]
    y[:, 5] = [6, 8]
    best_j, best_d, _, _ = calibrate.nearest_by_l2(y, T)
    # channel 0: 25, 25, 100 -> member 0 (tie);  channel 2: 16, 34, 9 + 64 -> member 0;  channel 4: 18, 16, 36 + 49 -> member 1
    assert best_j.tolist() == [0, 0, 1] and best_d.tolist() == [25.0, 16.0, 16.0]
    src_idx, dst_idx = calibrate.nearest_pairs(y, T, 1)                 # 16 twice: the lower member of A (channel 2) wins
    assert src_idx.tolist() == [1] and dst_idx.tolist() == [0]
    # only the first n_match_tokens tokens count
    best_j, best_d, _, _ = calibrate.nearest_by_l2(y, T, n_match_tokens=1)
    assert best_d.tolist() == [0.0, 0.0, 0.0] and best_j.tolist() == [1, 0, 1]   # token 0 alone: (0, 3, 3, 0, 0, 6)


def test_l2_matching_against_brute_force():
    """Every A x B pair with explicit differences in Python floats; sub-channels of split channels excluded."""
    rng = np.random.default_rng(15)
    C, N = 29, 4
    y = rng.integers(-2, 3, (N, C)).astype(np.float32)          # small integers: distances are exact, ties do occur
    T = np.ones(C, np.int32)
    T[[3, 20]] = [2, 4]
    best_j, best_d, pos_a, pos_b = calibrate.nearest_by_l2(y, T)
    chan_of = np.repeat(np.arange(C), T)
    assert not np.isin(chan_of[pos_a], [3, 20]).any() and not np.isin(chan_of[pos_b], [3, 20]).any()
    ties = 0
    for k, pa in enumerate(pos_a):
        ds = [sum((float(y[n, chan_of[pa]]) - float(y[n, chan_of[pb]])) ** 2 for n in range(N)) for pb in pos_b]
        assert best_d[k] == min(ds) and best_j[k] == ds.index(min(ds))     # list.index: the first minimum
        ties += ds.count(min(ds)) > 1
    assert ties > 0
    r = 6
    src_idx, dst_idx = calibrate.nearest_pairs(y, T, r)
    order = sorted(range(pos_a.size), key=lambda k: (best_d[k], k))[:r]     # shortest edges, ties to the lower A member
    assert src_idx.tolist() == sorted(int(pos_a[k]) // 2 for k in order)
    assert sorted(zip(src_idx.tolist(), dst_idx.tolist())) == sorted((int(pos_a[k]) // 2, (int(pos_b[best_j[k]]) - 1) // 2) for k in order)


def test_expansion_threshold_is_the_largest_that_adds_enough(oracle):
    """("expand", ratio): theta adds at least round(ratio * C) channels and the next float32 above it does not;
    on a hand case the breakpoints are known: m = (1, 2, 12), one added channel needs theta < 12, two need
    theta < 6 (12 -> 3 sub-channels) ... the largest float32 below each breakpoint."""
    m = np.array([1.0, 2.0, 12.0], np.float32)
    below = lambda v: float(np.nextafter(np.float32(v), np.float32(0)))
    for target, edge in [(1, 12.0), (2, 6.0), (3, 4.0), (4, 3.0), (5, 2.4)]:
        th = calibrate.theta_from_rule(m, ("expand", target / 3.0))
        assert calibrate.extra_channels(m, th) >= target
        assert calibrate.extra_channels(m, np.nextafter(np.float32(th), np.float32(np.inf))) < target
        if edge in (12.0, 6.0, 4.0, 3.0):                                   # exact quotients: theta is the float below the edge
            assert th == below(edge)
    rng = np.random.default_rng(16)
    m = np.abs(rng.standard_normal(300)).astype(np.float32)
    m[[7, 90]] *= 40
    for ratio in (0.01, 0.05, 0.3):
        th = calibrate.theta_from_rule(m, ("expand", ratio))
        target = max(1, int(round(ratio * m.size)))
        assert int((oracle.num_split(m, th).astype(np.int64) - 1).sum()) >= target
        assert int((oracle.num_split(m, np.nextafter(np.float32(th), np.float32(np.inf))).astype(np.int64) - 1).sum()) < target


def test_c_routine_agrees_with_the_numpy_form_of_eq5(oracle):
    """oracle_nearest_member with weights against nearest_by_eq5 (numpy): same members, distances to round-off."""
    rng = np.random.default_rng(17)
    C, N, O = 37, 9, 6
    y = rng.standard_normal((N, C)).astype(np.float32)
    W = rng.standard_normal((C, O)).astype(np.float32)
    T = np.ones(C, np.int32)
    T[[8, 30]] = [2, 3]
    ref_j, ref_d, pos_a, pos_b = calibrate.nearest_by_eq5(y, W, T)
    chan_of = np.repeat(np.arange(C), T)
    got_j, got_d = oracle.nearest_member(y, W, chan_of[pos_a], chan_of[pos_b])
    assert np.array_equal(got_j, ref_j) and np.allclose(got_d, ref_d, rtol=1e-13, atol=0)
