"""Pins for channel disassembly (Sec. 4.1.1, Eq. 3), channel assembly (Sec. 4.1.2, Eq. 4) and the
map that composes them.  Invariants, closed forms and an independent fp64 re-statement."""
import numpy as np
import pytest


def random_case(rng, C, n_out, Tmax, r, N=6):
    """Random (y, T, src_idx, dst_idx) with valid merges (no sub-channel takes part)."""
    y = rng.standard_normal((N, C)).astype(np.float32)
    T = np.ones(C, np.int32)
    out = rng.choice(C, size=min(n_out, C), replace=False)
    T[out] = rng.integers(2, Tmax + 1, size=out.size)
    chan_of = np.repeat(np.arange(C), T)
    Cp = chan_of.size
    elig = T[chan_of] == 1
    pa = np.arange(0, Cp, 2)
    pb = np.arange(1, Cp, 2)
    pa, pb = pa[elig[pa]], pb[elig[pb]]
    r = min(r, pa.size) if pb.size else 0
    sp = rng.choice(pa, size=r, replace=False)
    dp = rng.choice(pb, size=r, replace=True)      # several sources may share one destination
    return y, T, (sp // 2).astype(np.int32), ((dp - 1) // 2).astype(np.int32)


def test_T_rule(oracle):
    # T = ceil(m / theta); m <= theta leaves the channel alone; an exact multiple is not rounded up
    m = np.array([0.0, 0.5, 4.0, 4.0000005, 8.0, 11.9, 12.0, 100.0], np.float32)
    assert oracle.num_split(m, 4.0).tolist() == [1, 1, 1, 2, 2, 3, 3, 25]
    assert np.all(oracle.num_split(m, 100.0) == 1)
    assert np.all(oracle.num_split(m, 1e9) == 1)


def test_disassembly_layout_and_count(oracle):
    y = np.arange(1, 6, dtype=np.float32)[None, :] * 8
    T = np.array([1, 4, 1, 2, 1], np.int32)
    d = oracle.disassemble(y, T)
    assert d.shape == (1, 5 + 3 + 1)                      # M + sum(T-1) channels
    assert d[0].tolist() == [8, 4, 4, 4, 4, 24, 16, 16, 40]


@pytest.mark.parametrize("pow2", [True, False])
def test_disassembly_preserves_layer_output(oracle, pow2):
    """Eq. (3) "produces the same output with the original linear layer": exactly when every T is a
    power of two (the scaling is then exact), to fp64 round-off of the fp32 scale otherwise."""
    rng = np.random.default_rng(11)
    C, O = 40, 7
    y = rng.standard_normal((5, C)).astype(np.float32)
    W = rng.standard_normal((C, O)).astype(np.float32)
    T = np.ones(C, np.int32)
    T[[0, 3, 17, 39]] = [2, 8, 4, 2] if pow2 else [3, 7, 5, 6]
    d = oracle.disassemble(y, T)
    What = oracle.reassemble_weight(W, T, [], [])
    assert What.shape == (int(T.sum()), O)
    ref = y.astype(np.float64) @ W.astype(np.float64)
    got = d.astype(np.float64) @ What.astype(np.float64)
    if pow2:
        # same terms, T of them scaled by an exact 1/T: equal up to fp64 summation order
        assert np.allclose(got, ref, rtol=0, atol=1e-12)
        # and the T sub-channels add back to the channel exactly
        assert np.array_equal(d[:, 4:12].sum(1), y[:, 3])
    else:
        assert np.allclose(got, ref, rtol=0, atol=1e-6)   # fl32(1/3) etc. is off by <= 2^-25 relative
        assert not np.allclose(got, ref, rtol=0, atol=1e-12)


def test_theta_above_max_is_identity(oracle):
    rng = np.random.default_rng(1)
    y = rng.standard_normal((4, 30)).astype(np.float32)
    T = oracle.num_split(oracle.channel_absmax(y), float(np.abs(y).max()))
    assert np.all(T == 1)
    row_ptr, src, scale = oracle.build_map(T, [], [])
    assert row_ptr.tolist() == list(range(31)) and src.tolist() == list(range(30)) and np.all(scale == 1)
    assert np.array_equal(oracle.assemble(oracle.disassemble(y, T), [], []), y)
    assert np.array_equal(oracle.apply_map(y, row_ptr, src, scale), y)


def test_merging_identical_channels_is_exact_and_error_closed_form(oracle):
    """Eq. (4): x_i W_i + x_j W_j - (x_i+x_j)/2 (W_i+W_j) = (x_i-x_j)(W_i-W_j)/2, zero when x_i == x_j."""
    rng = np.random.default_rng(2)
    C, O, N = 10, 4, 8
    y = rng.integers(-16, 17, (N, C)).astype(np.float32)   # small integers: every step below is exact
    W = rng.integers(-8, 9, (C, O)).astype(np.float32)
    T = np.ones(C, np.int32)
    src_idx, dst_idx = [2], [3]                            # channel 4 (A) into channel 7 (B)
    i, j = 7, 4
    xh = oracle.assemble(oracle.disassemble(y, T), src_idx, dst_idx)
    What = oracle.reassemble_weight(W, T, src_idx, dst_idx)
    assert xh.shape == (N, C - 1) and What.shape == (C - 1, O)
    full = y.astype(np.float64) @ W.astype(np.float64)
    merged = xh.astype(np.float64) @ What.astype(np.float64)
    err = ((y[:, i] - y[:, j])[:, None] * (W[i] - W[j])[None, :] / 2).astype(np.float64)
    assert np.array_equal(full - merged, err)
    y2 = y.copy()
    y2[:, j] = y2[:, i]
    xh2 = oracle.assemble(oracle.disassemble(y2, T), src_idx, dst_idx)
    assert np.array_equal(xh2.astype(np.float64) @ What.astype(np.float64), y2.astype(np.float64) @ W.astype(np.float64))
    # order of the surviving channels is the original order with channel 4 removed
    assert np.array_equal(np.delete(y2, j, axis=1), xh2)


@pytest.mark.parametrize("seed,C,n_out,Tmax,r", [(0, 16, 2, 4, 3), (1, 33, 5, 8, 9), (2, 64, 0, 2, 20),
                                                 (3, 7, 1, 3, 1), (4, 129, 9, 5, 30), (5, 2, 0, 2, 1)])
def test_assembly_against_independent_fp64_statement(oracle, seed, C, n_out, Tmax, r):
    """Group means and deletions restated with numpy in fp64 on the disassembled matrix."""
    rng = np.random.default_rng(seed)
    y, T, src_idx, dst_idx = random_case(rng, C, n_out, Tmax, r)
    d = oracle.disassemble(y, T)
    Cp = d.shape[1]
    assert Cp == C + int((T - 1).sum())
    xh, keep = oracle.assemble(d, src_idx, dst_idx, return_keep=True)
    assert xh.shape[1] == Cp - len(src_idx)                 # one channel fewer per merged pair
    exp = d.astype(np.float64).copy()
    for dp in np.unique(2 * dst_idx + 1):
        members = [dp] + sorted((2 * src_idx[dst_idx == (dp - 1) // 2]).tolist())
        exp[:, dp] = d[:, members].astype(np.float64).mean(1)
    exp = np.delete(exp, 2 * src_idx, axis=1)
    assert np.array_equal(keep, np.delete(np.arange(Cp), 2 * src_idx))
    assert np.all(np.abs(xh - exp) <= 3e-7 * np.abs(d).max())      # a mean can cancel: absolute bound
    pairs_only = np.array([np.sum(dst_idx == k) for k in dst_idx]) == 1
    if pairs_only.all():                                    # (a+b)/2 is one rounding either way
        assert np.array_equal(xh, exp.astype(np.float32))


@pytest.mark.parametrize("seed,C,n_out,Tmax,r", [(0, 16, 2, 4, 3), (1, 33, 5, 8, 9), (2, 64, 0, 2, 20),
                                                 (3, 7, 1, 3, 1), (4, 129, 9, 5, 30), (6, 257, 20, 8, 60)])
def test_map_form_equals_two_stage_form_bitwise(oracle, seed, C, n_out, Tmax, r):
    rng = np.random.default_rng(100 + seed)
    y, T, src_idx, dst_idx = random_case(rng, C, n_out, Tmax, r)
    two_stage = oracle.assemble(oracle.disassemble(y, T), src_idx, dst_idx)
    row_ptr, src, scale = oracle.build_map(T, src_idx, dst_idx)
    assert row_ptr[0] == 0 and row_ptr[-1] == src.size and np.all(np.diff(row_ptr) >= 1)
    assert np.array_equal(oracle.apply_map(y, row_ptr, src, scale), two_stage)
    # weights: every source channel's row is counted exactly once per unit of activation scale:
    # sum over entries of scale == 1 per source channel when nothing is merged, and the reassembled
    # weight row is the plain sum of the rows the map row names
    W = rng.standard_normal((C, 3)).astype(np.float32)
    What = oracle.reassemble_weight(W, T, src_idx, dst_idx)
    for ch in range(row_ptr.size - 1):
        rows = src[row_ptr[ch]:row_ptr[ch + 1]]
        assert np.allclose(What[ch], W[rows].astype(np.float64).sum(0), rtol=1e-6, atol=1e-7)


def test_outliers_at_the_ends_and_adjacent(oracle):
    y = (np.arange(1, 7, dtype=np.float32) * 6)[None, :]
    T = np.array([3, 1, 1, 2, 2, 3], np.int32)             # first, last and two adjacent channels split
    d = oracle.disassemble(y, T)
    assert d[0].tolist() == [2, 2, 2, 12, 18, 12, 12, 15, 15, 12, 12, 12]
    # positions: channel 1 -> 3 (odd, B member 1), channel 2 -> 4 (even, A member 2): merge them
    xh = oracle.assemble(d, [2], [1])
    assert xh[0].tolist() == [2, 2, 2, 15, 12, 12, 15, 15, 12, 12, 12]
    row_ptr, src, scale = oracle.build_map(T, [2], [1])
    assert np.array_equal(oracle.apply_map(y, row_ptr, src, scale), xh)


def test_sub_channels_cannot_be_merged(oracle):
    T = np.array([2, 1, 1, 1], np.int32)                   # positions 0,1 are sub-channels of channel 0
    with pytest.raises(ValueError):
        oracle.build_map(T, [0], [1])                      # A member 0 = position 0: a sub-channel
    with pytest.raises(ValueError):
        oracle.build_map(T, [1], [0])                      # B member 0 = position 1: a sub-channel
    oracle.build_map(T, [1], [1])                          # positions 2 and 3: fine
    with pytest.raises(ValueError):
        oracle.build_map(np.ones(4, np.int32), [0, 0], [0, 1])   # one A member merged twice
    with pytest.raises(ValueError):
        oracle.build_map(np.ones(4, np.int32), [2], [0])   # index outside set A


def test_calibration_restores_channel_count(oracle):
    from oracle import calibrate
    rng = np.random.default_rng(9)
    y = rng.standard_normal((64, 96)).astype(np.float32)
    y[:, [5, 50, 77]] *= [10, 15, 20]
    cal = calibrate.calibrate(y, ("fixed", 8.0))
    T = cal["T"]
    assert T.max() > 1 and len(cal["src_idx"]) == int((T - 1).sum())
    row_ptr, _, _ = oracle.build_map(T, cal["src_idx"], cal["dst_idx"])
    assert row_ptr.size - 1 == 96                          # merging sum(T-1) pairs restores M channels
    d = oracle.disassemble(y, T)
    assert np.abs(d).max() <= 8.0 * (1 + 1e-6)             # every sub-channel is within the threshold
    th = calibrate.theta_from_rule(cal["absmax"], ("expand", 0.05))
    extra = int((oracle.num_split(cal["absmax"], th) - 1).sum())
    assert extra >= 5 and extra <= 7


# ---------------------------------------------------------------- Appendix B: folded into the preceding layer

def test_fold_worked_example(oracle):
    """Appendix B by hand: channel 1 split in three (columns divided by 3 and repeated), then the
    A-member at disassembled position 0 merged into the B-member at position 5: their mean."""
    Wp = np.array([[2.0, 4.0], [9.0, 3.0], [6.0, 8.0], [1.0, 1.0]])
    bp = np.array([1.0, 6.0, 3.0, 5.0])
    T = np.array([1, 3, 1, 1], np.int32)
    # disassembled axis: [c0, c1/3, c1/3, c1/3, c2, c3]; A = positions 0, 2, 4; B = 1, 3, 5
    W_hat, b_hat = oracle.fold_preceding_linear(Wp, bp, T, [0], [2])
    assert W_hat.tolist() == [[3.0, 1.0], [3.0, 1.0], [3.0, 1.0], [6.0, 8.0], [1.5, 2.5]]
    assert b_hat.tolist() == [2.0, 2.0, 2.0, 3.0, 3.0]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_fold_equals_runtime_reassembly(oracle, seed):
    """What Appendix B claims: reassembling the output of y = x Wp^T + bp at run time (Eq. 3 then
    Eq. 4, the oracle's two literal stages) gives the activations that the folded layer produces
    directly.  The left side runs in the oracle's fp32, so agreement is to fp32 round-off."""
    rng = np.random.default_rng(seed)
    C, Kp, N = 96, 33, 9
    _, T, src_idx, dst_idx = random_case(rng, C, 9, 6, 20)
    Wp = rng.standard_normal((C, Kp))
    bp = rng.standard_normal(C)
    x = rng.standard_normal((N, Kp))
    y = x @ Wp.T + bp
    runtime = oracle.assemble(oracle.disassemble(y.astype(np.float32), T), src_idx, dst_idx).astype(np.float64)
    W_hat, b_hat = oracle.fold_preceding_linear(Wp, bp, T, src_idx, dst_idx)
    folded = x @ W_hat.T + b_hat
    assert folded.shape == runtime.shape
    assert np.abs(folded - runtime).max() <= 2e-6 * np.abs(runtime).max()
    # without a bias, and with nothing to do, the fold is the identity
    W_same, none = oracle.fold_preceding_linear(Wp, None, np.ones(C, np.int32), [], [])
    assert none is None and np.array_equal(W_same, Wp)
