"""Pins for the integer GEMM (Eq. 1 on codes), the dequantising epilogue and the whole path."""
import numpy as np
import pytest


def test_int_gemm_brute_force_python_ints(oracle):
    rng = np.random.default_rng(0)
    a = rng.integers(0, 16, (3, 7), dtype=np.uint8)
    w = rng.integers(0, 16, (4, 7), dtype=np.uint8)
    acc = oracle.int_gemm(a, w)
    for n in range(3):
        for o in range(4):
            assert int(acc[n, o]) == sum(int(a[n, k]) * int(w[o, k]) for k in range(7))


def test_int_gemm_special_operands(oracle):
    rng = np.random.default_rng(1)
    a = rng.integers(0, 64, (5, 33), dtype=np.uint8)
    eye = np.eye(33, dtype=np.uint8)
    assert np.array_equal(oracle.int_gemm(a, eye), a.astype(np.int32))          # one-hot rows pick a code
    ones = np.ones((2, 33), np.uint8)
    assert np.array_equal(oracle.int_gemm(a, ones)[:, 0], a.astype(np.int64).sum(1))   # all-ones: row sums
    # not symmetric in its operands: acc[n,o] pairs activation row n with weight row o
    w = rng.integers(0, 64, (4, 33), dtype=np.uint8)
    assert oracle.int_gemm(a, w).shape == (5, 4)
    assert np.array_equal(oracle.int_gemm(a, w), oracle.int_gemm(w, a).T)


@pytest.mark.parametrize("bits,K", [(4, 300), (6, 257), (8, 128)])
def test_int_gemm_matches_numpy_int64(oracle, bits, K):
    rng = np.random.default_rng(bits)
    a = rng.integers(0, 2 ** bits, (17, K), dtype=np.uint8)
    w = rng.integers(0, 2 ** bits, (23, K), dtype=np.uint8)
    assert np.array_equal(oracle.int_gemm(a, w), a.astype(np.int64) @ w.astype(np.int64).T)


def test_accumulator_bounds_of_the_benchmark_shapes():
    # the largest possible sums stay inside int32
    assert 15 * 15 * 28672 < 2 ** 31 and 63 * 63 * 8192 < 2 ** 31 and 255 * 255 * 28672 < 2 ** 31


def test_epilogue_equals_direct_sum_of_corrected_products(oracle):
    rng = np.random.default_rng(2)
    N, K, O = 6, 50, 5
    a = rng.integers(0, 16, (N, K), dtype=np.uint8)
    w = rng.integers(0, 16, (O, K), dtype=np.uint8)
    ax = rng.uniform(0.01, 1, N).astype(np.float32)
    aw = rng.uniform(0.001, 0.1, O).astype(np.float32)
    bx = rng.integers(-20, 30, N).astype(np.int32)        # zero-points outside [0, qmax] are legal
    bw = rng.integers(0, 16, O).astype(np.int32)
    acc = oracle.int_gemm(a, w)
    y1 = oracle.epilogue(acc, K, ax, bx, a.astype(np.int64).sum(1), aw, bw, w.astype(np.int64).sum(1))
    y2 = oracle.dequant_linear_direct(a, w, ax, bx, aw, bw)
    assert np.array_equal(y1, y2)
    # and against a float64 dequantise-then-multiply
    xa = ax[:, None].astype(np.float64) * (a.astype(np.float64) - bx[:, None])
    xw = aw[:, None].astype(np.float64) * (w.astype(np.float64) - bw[:, None])
    assert np.allclose(y1, xa @ xw.T, rtol=3e-7, atol=1e-9)


def test_whole_path_equals_its_steps(oracle):
    from oracle import calibrate
    rng = np.random.default_rng(3)
    N, C, O = 12, 80, 11
    x = rng.standard_normal((N, C)).astype(np.float32)
    x[:, [7, 40]] *= [25, 60]
    gamma = rng.uniform(0.5, 1.5, C).astype(np.float32)
    W = (rng.standard_normal((C, O)) * 0.02).astype(np.float32)
    y = oracle.norm(x, oracle.NORM_RMS, gamma, None, 1e-5)
    cal = calibrate.calibrate(y, ("fixed", 3.0))
    T, si, di = cal["T"], cal["src_idx"], cal["dst_idx"]
    assert T.max() > 1 and si.size > 0
    What = oracle.reassemble_weight(W, T, si, di)
    wq = oracle.quantize_weight(What, 4)
    out = oracle.reassembled_linear(x, oracle.NORM_RMS, gamma, None, 1e-5, T, si, di, 4, wq)
    xh = oracle.apply_map(y, *oracle.build_map(T, si, di))
    codes, alpha, beta, rowsum = oracle.quantize_rows(xh, 4)
    assert np.array_equal(out["codes"], codes) and np.array_equal(out["alpha"], alpha)
    assert np.array_equal(out["beta"], beta) and np.array_equal(out["rowsum"], rowsum)
    acc = oracle.int_gemm(codes, wq[0])
    assert np.array_equal(out["acc"], acc)
    assert np.array_equal(out["y"], oracle.epilogue(acc, xh.shape[1], alpha, beta, rowsum, wq[1], wq[2], wq[3]))


def test_8bit_path_approximates_the_full_precision_layer(oracle):
    """Sanity on the end result: with 8 bits on both sides, no outliers and an identity map, the
    dequantised output is the fp64 norm->linear up to the two quantizers' step sizes."""
    rng = np.random.default_rng(4)
    N, C, O = 8, 256, 16
    x = rng.standard_normal((N, C)).astype(np.float32)
    gamma = np.ones(C, np.float32)
    W = (rng.standard_normal((C, O)) * 0.02).astype(np.float32)
    T = np.ones(C, np.int32)
    wq = oracle.quantize_weight(W, 8)
    out = oracle.reassembled_linear(x, oracle.NORM_RMS, gamma, None, 1e-5, T, [], [], 8, wq)
    y = x.astype(np.float64) / np.sqrt((x.astype(np.float64) ** 2).mean(1, keepdims=True) + 1e-5)
    ref = y @ W.astype(np.float64)
    # |error| <= sum_k (|y| aw/2 + |w| ax/2 + ax aw/4), a loose per-output bound
    bound = (np.abs(y).sum(1)[:, None] * wq[1][None, :] / 2 + np.abs(W).sum(0)[None, :] * out["alpha"][:, None] / 2
             + C * out["alpha"][:, None] * wq[1][None, :] / 4)
    assert np.all(np.abs(out["y"] - ref) <= bound)
    assert np.abs(out["y"] - ref).max() / np.abs(ref).max() < 0.02


def test_disassembly_helps_the_quantizer(oracle):
    """The point of Sec. 4.1.1: splitting the outlier channel shrinks the per-token range, so the
    4-bit output moves closer to the full-precision one (disassembly itself changes nothing)."""
    rng = np.random.default_rng(5)
    N, C, O = 32, 128, 24
    x = rng.standard_normal((N, C)).astype(np.float32)
    x[:, 17] *= 60
    W = (rng.standard_normal((C, O)) * 0.05).astype(np.float32)
    ref = x.astype(np.float64) @ W.astype(np.float64)

    def run(T):
        What = oracle.reassemble_weight(W, T, [], [])
        out = oracle.reassembled_linear(x, oracle.NORM_NONE, None, None, 0.0, T, [], [], 4,
                                        oracle.quantize_weight(What, 8))
        return np.sqrt(((out["y"] - ref) ** 2).mean())

    T1 = np.ones(C, np.int32)
    T8 = T1.copy()
    T8[17] = 16
    assert run(T8) < 0.5 * run(T1)
