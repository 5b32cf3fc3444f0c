"""Pins for the oracle's uniform quantizer (Preliminaries, Eq. 2) and the storage format."""
from fractions import Fraction

import numpy as np
import pytest
import torch


def rne_fraction(q: Fraction) -> int:
    """Nearest integer, ties to even, on an exact rational."""
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_quantizer_properties(oracle, bits):
    rng = np.random.default_rng(bits)
    x = (rng.standard_normal((40, 97)) * rng.uniform(0.1, 30, (40, 1))).astype(np.float32)
    x[3] = np.abs(x[3]) + 5.0          # all-positive row: zero-point below 0
    x[4] = -np.abs(x[4]) - 5.0         # all-negative row: zero-point above qmax
    codes, alpha, beta, rowsum = oracle.quantize_rows(x, bits)
    qmax = 2 ** bits - 1
    mn, mx = x.min(1), x.max(1)
    # alpha = (max - min) / (2^b - 1)
    assert np.allclose(alpha.astype(np.float64), (mx.astype(np.float64) - mn) / qmax, rtol=3e-7)
    assert codes.min() >= 0 and codes.max() <= qmax
    assert np.array_equal(rowsum, codes.astype(np.int64).sum(1))
    for n in range(x.shape[0]):
        # the minimum always lands on code 0 (beta is minus its rounded quotient) ...
        assert codes[n, x[n].argmin()] == 0
        # ... and the maximum on the top code or one below (two roundings of .5 can cost one step)
        assert codes[n, x[n].argmax()] >= qmax - 1
        # codes are monotone in x
        order = np.argsort(x[n], kind="stable")
        assert np.all(np.diff(codes[n, order].astype(np.int32)) >= 0)
    # beta = -round(min / alpha) to within the rounding of 1/alpha
    assert np.all(np.abs(beta + np.rint(mn.astype(np.float64) / alpha)) <= 1)
    assert beta[3] < 0 and beta[4] > qmax
    # dequantisation alpha*(code - beta) is within alpha/2 of x wherever the clamp did not act
    deq = alpha[:, None].astype(np.float64) * (codes.astype(np.float64) - beta[:, None])
    err = np.abs(deq - x)
    inner = (codes > 0) & (codes < qmax)
    assert np.all(err[inner] <= 0.5 * alpha[:, None].repeat(97, 1)[inner] * (1 + 1e-5))
    assert np.all(err <= 1.0 * alpha[:, None] * (1 + 1e-5))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_quantizer_brute_force_exact_rationals(oracle, bits):
    """Tiny rows, every step re-done in exact rational arithmetic on the fp32 values of alpha and
    1/alpha (numpy float32 scalars), including round-half-even on exact ties."""
    rng = np.random.default_rng(50 + bits)
    qmax = 2 ** bits - 1
    rows = [rng.integers(-12, 13, 7) / 4.0 for _ in range(60)]           # quarter steps: many exact ties
    rows += [rng.standard_normal(7) * 3 for _ in range(60)]
    rows += [np.array([0, qmax, 0.5, 1.5, 2.5, 1.0, 2.0]),              # alpha = 1: ties at every half
             np.array([-1.5, -0.5, 0.5, qmax - 1.5, 0, 1, -1.0])]
    x = np.array(rows, np.float32)
    codes, alpha, beta, rowsum = oracle.quantize_rows(x, bits)
    for n in range(x.shape[0]):
        mn, mx = np.float32(x[n].min()), np.float32(x[n].max())
        a32 = np.float32(np.float32(mx - mn) / np.float32(qmax))
        inv32 = np.float32(np.float32(1.0) / a32)
        assert alpha[n] == a32
        inv = Fraction(float(inv32))
        b = -rne_fraction(Fraction(float(mn)) * inv)
        assert beta[n] == b
        exp = [min(max(rne_fraction(Fraction(float(v)) * inv) + b, 0), qmax) for v in x[n]]
        assert codes[n].tolist() == exp
    # the two hand-made rows: alpha = 1, beta = 0 / 2: ties go to the even integer
    assert alpha[-2] == 1 and codes[-2].tolist() == [0, qmax, 0, 2, 2, 1, 2]
    assert alpha[-1] == 1 and beta[-1] == 2 and codes[-1].tolist()[:3] == [0, 2, 2]


def test_constant_row_and_two_value_row(oracle):
    x = np.array([[3.25] * 6, [0.0] * 6, [-6.0, 9.0, -6.0, 9.0, 9.0, -6.0]], np.float32)
    codes, alpha, beta, rowsum = oracle.quantize_rows(x, 4)
    # max == min: alpha is defined as 1; 3.25 rounds to 3, beta = -3, every code is 0
    assert alpha[0] == 1.0 and beta[0] == -3 and np.all(codes[0] == 0)
    assert alpha[1] == 1.0 and beta[1] == 0 and np.all(codes[1] == 0)
    # two values 15 apart (alpha = 1): they take the two end codes
    assert sorted(set(codes[2].tolist())) == [0, 15]
    deq = alpha[2] * (codes[2].astype(np.float32) - beta[2])
    assert np.allclose(deq, x[2], atol=alpha[2] / 2 * 1.001)


def test_8bit_matches_torch_affine_quantizer(oracle):
    """b = 8: Eq. (2) is the ordinary per-tensor affine uint8 quantizer; torch's implementation
    multiplies by the fp32 reciprocal and rounds the fp32 product, so single codes may differ by one
    where that product rounds across a half."""
    rng = np.random.default_rng(8)
    x = (rng.standard_normal((16, 4096)) * 2).astype(np.float32)
    codes, alpha, beta, _ = oracle.quantize_rows(x, 8)
    n_diff = 0
    for n in range(16):
        assert 0 <= beta[n] <= 255
        tq = torch.quantize_per_tensor(torch.from_numpy(x[n]), float(alpha[n]), int(beta[n]), torch.quint8)
        t = tq.int_repr().numpy().astype(np.int32)
        diff = np.abs(t - codes[n].astype(np.int32))
        assert diff.max() <= 1
        n_diff += int((diff != 0).sum())
    assert n_diff <= 16 * 4096 * 1e-4


def test_per_output_channel_weight_quantization(oracle):
    """Weights: one (alpha, beta) per output channel, ranges taken over the input channels."""
    rng = np.random.default_rng(4)
    K, O = 64, 9
    W = (rng.standard_normal((K, O)) * rng.uniform(0.01, 1, (1, O))).astype(np.float32)
    wcodes, aw, bw, cs = oracle.quantize_weight(W, 4)
    assert wcodes.shape == (O, K)
    c2, a2, b2, s2 = oracle.quantize_rows(np.ascontiguousarray(W.T), 4)    # same quantizer, other axis
    assert np.array_equal(wcodes, c2) and np.array_equal(aw, a2) and np.array_equal(bw, b2) and np.array_equal(cs, s2)
    assert np.allclose(aw, (W.max(0) - W.min(0)) / 15, rtol=3e-7)
    deq = aw[:, None] * (wcodes.astype(np.float32) - bw[:, None])
    assert np.all(np.abs(deq - W.T) <= aw[:, None] * 0.5001 + 1e-9)


def test_packing_layout_by_hand(oracle):
    # 4 bit: even code in the low nibble.  codes 1,2,3 -> 0x21, 0x03
    p = oracle.pack_codes(np.array([[1, 2, 3]], np.uint8), 4, row_bytes=4)
    assert p[0].tolist() == [0x21, 0x03, 0, 0]
    # 6 bit: four codes in 24 little-endian bits.  1 | 2<<6 | 3<<12 | 4<<18 = 0x103081
    p = oracle.pack_codes(np.array([[1, 2, 3, 4, 63]], np.uint8), 6, row_bytes=6)
    assert p[0].tolist() == [0x81, 0x30, 0x10, 63, 0, 0]
    p = oracle.pack_codes(np.array([[7, 255]], np.uint8), 8, row_bytes=3)
    assert p[0].tolist() == [7, 255, 0]
    with pytest.raises(ValueError):
        oracle.pack_codes(np.array([[16]], np.uint8), 4)


@pytest.mark.parametrize("bits", [4, 6, 8])
@pytest.mark.parametrize("K", [1, 5, 64, 131])
def test_pack_roundtrip_and_padding(oracle, bits, K):
    rng = np.random.default_rng(K * bits)
    codes = rng.integers(0, 2 ** bits, (5, K), dtype=np.uint8)
    packed = oracle.pack_codes(codes, bits)
    assert packed.shape[1] % 16 == 0 and packed.shape[1] >= (K * bits + 7) // 8
    assert np.array_equal(oracle.unpack_codes(packed, K, bits), codes)
    # every bit beyond K*bits is zero
    bitsarr = np.unpackbits(packed, axis=1, bitorder="little")
    assert bitsarr[:, K * bits:].sum() == 0
    # cross-check the bit order with numpy's own little-endian bit packing
    ref_bits = ((codes[:, :, None] >> np.arange(bits)[None, None, :]) & 1).reshape(5, K * bits).astype(np.uint8)
    assert np.array_equal(bitsarr[:, :K * bits], ref_bits)
