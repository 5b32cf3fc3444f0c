"""Pins for the oracle's norm step (Sec. 4.3: a normalisation layer precedes the runtime
disassembly/assembly layers).  Checked against torch's own fp64 LayerNorm / RMSNorm, closed forms
and special cases, none of which call the oracle."""
import numpy as np
import pytest
import torch

from paper_2310_08041_amd.workloads import bf16_bits_to_f32, f32_to_bf16_bits


def _ulp_err(got, ref64):
    ref32 = ref64.astype(np.float32)
    ulp = np.spacing(np.abs(ref32)).astype(np.float64)
    return np.abs(got.astype(np.float64) - ref64) / np.maximum(ulp, 1e-45)


@pytest.mark.parametrize("C", [7, 64, 1000])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layernorm_matches_torch_fp64(oracle, C, dtype):
    rng = np.random.default_rng(C)
    x = (rng.standard_normal((9, C)) * 3 + 1.5).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, C).astype(np.float32)
    beta = rng.standard_normal(C).astype(np.float32)
    xin = f32_to_bf16_bits(x) if dtype == "bf16" else x
    xval = bf16_bits_to_f32(xin) if dtype == "bf16" else x
    got = oracle.norm(xin, oracle.NORM_LAYER, gamma, beta, 1e-5)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(xval).double(), (C,), torch.from_numpy(gamma).double(),
                                         torch.from_numpy(beta).double(), 1e-5).numpy()
    # four fp32 roundings (sub, two multiplies, add) plus the rounding of mu and rstd to fp32; the
    # subtraction and the final add can cancel, so measure against the magnitude of the terms
    mu = xval.astype(np.float64).mean(1, keepdims=True)
    rstd = 1.0 / np.sqrt(xval.astype(np.float64).var(1, keepdims=True) + 1e-5)
    scale = np.abs(ref) + np.abs(beta)[None, :] + np.abs(mu) * rstd * np.abs(gamma)[None, :]
    assert np.all(np.abs(got - ref) <= 4 * 6e-8 * scale + 1e-30)


@pytest.mark.parametrize("C", [5, 128, 4096])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rmsnorm_matches_torch_fp64(oracle, C, dtype):
    rng = np.random.default_rng(C + 1)
    x = (rng.standard_normal((5, C)) * 2).astype(np.float32)
    x[:, 3] *= 60
    gamma = rng.uniform(0.5, 1.5, C).astype(np.float32)
    xin = f32_to_bf16_bits(x) if dtype == "bf16" else x
    xval = bf16_bits_to_f32(xin) if dtype == "bf16" else x
    got = oracle.norm(xin, oracle.NORM_RMS, gamma, None, 1e-5)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(xval).double(), (C,), torch.from_numpy(gamma).double(),
                                       1e-5).numpy()
    assert _ulp_err(got, ref).max() <= 2.0   # rstd rounding + two multiplies


def test_layernorm_closed_form_biased_variance(oracle):
    # x = (+1, -1): mean 0, biased variance 1 (the unbiased one would be 2) => y = x*gamma + beta exactly
    x = np.array([[1.0, -1.0], [-1.0, 1.0]], np.float32)
    gamma = np.array([2.0, 4.0], np.float32)
    beta = np.array([0.5, -0.25], np.float32)
    y = oracle.norm(x, oracle.NORM_LAYER, gamma, beta, 0.0)
    assert y.tolist() == [[2.5, -4.25], [-1.5, 3.75]]


def test_layernorm_shift_invariance_and_rms_scale(oracle):
    rng = np.random.default_rng(3)
    x = rng.integers(-8, 9, (4, 32)).astype(np.float32)
    g = np.ones(32, np.float32)
    y0 = oracle.norm(x, oracle.NORM_LAYER, g, None, 0.0)
    y1 = oracle.norm(x + 16.0, oracle.NORM_LAYER, g, None, 0.0)   # integers: the shift is exact
    assert np.array_equal(y0, y1)
    # RMSNorm output has unit mean square when gamma = 1 and eps = 0
    r = oracle.norm(x, oracle.NORM_RMS, g, None, 0.0).astype(np.float64)
    assert np.allclose((r * r).mean(1), 1.0, rtol=1e-6)
    # RMSNorm of a vector of +-4 is +-1 exactly (rstd = 1/4)
    s = np.array([[4.0, -4.0, 4.0, 4.0]], np.float32)
    assert oracle.norm(s, oracle.NORM_RMS, np.ones(4, np.float32), None, 0.0).tolist() == [[1.0, -1.0, 1.0, 1.0]]


def test_eps_enters_under_the_root(oracle):
    # zero row: y = 0 (not NaN) for eps > 0; and a known value: x = (3, 3), eps = 7 => rstd = 1/4
    z = np.zeros((1, 8), np.float32)
    assert np.all(oracle.norm(z, oracle.NORM_RMS, np.ones(8, np.float32), None, 1e-5) == 0)
    assert np.all(oracle.norm(z, oracle.NORM_LAYER, np.ones(8, np.float32), None, 1e-5) == 0)
    x = np.array([[3.0, 3.0]], np.float32)
    assert oracle.norm(x, oracle.NORM_RMS, np.ones(2, np.float32), None, 7.0).tolist() == [[0.75, 0.75]]


def test_norm_none_widens_exactly(oracle):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 17)).astype(np.float32)
    assert np.array_equal(oracle.norm(x, oracle.NORM_NONE), x)
    h = f32_to_bf16_bits(x)
    assert np.array_equal(oracle.norm(h, oracle.NORM_NONE), bf16_bits_to_f32(h))


def test_bf16_rounding_is_nearest_even(oracle):
    # 1 + 2^-8 is the midpoint between bf16 neighbours 1 and 1 + 2^-7 -> even mantissa (1.0);
    # 1 + 3*2^-8 is the midpoint between 1+2^-7 and 1+2^-6 -> even mantissa (1 + 2^-6)
    v = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -3.0], np.float32)
    got = oracle.widen_bf16(oracle.round_to_bf16(v))
    assert got.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -3.0]
    x = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    assert np.array_equal(oracle.round_to_bf16(x), f32_to_bf16_bits(x))
    assert np.array_equal(oracle.round_to_bf16(x), torch.from_numpy(x).bfloat16().view(torch.int16).numpy().view(np.uint16))


def test_channel_absmax(oracle):
    y = np.random.default_rng(2).standard_normal((50, 33)).astype(np.float32)
    assert np.array_equal(oracle.channel_absmax(y), np.abs(y).max(0))
