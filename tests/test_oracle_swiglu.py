"""Pins for the oracle's gated activation x = silu(gate) * up, the producer of a down projection's input in the
models of Sec. 5 (the paper fixes none of its arithmetic; the oracle states its own).  Checked against the
real-number function evaluated in float64, closed forms and special cases, none of which call the oracle."""
import numpy as np

from paper_2310_08041_amd.workloads import bf16_bits_to_f32, f32_to_bf16_bits


def _finite_bf16():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    return bits[np.isfinite(bf16_bits_to_f32(bits))]


def _silu64(g):
    with np.errstate(over="ignore"):
        return g / (1.0 + np.exp(-g))


def _ulps(got32, ref64):
    ulp = np.spacing(np.abs(ref64).astype(np.float32)).astype(np.float64)
    return np.abs(got32.astype(np.float64) - ref64) / ulp


def test_silu_every_finite_bf16_gate_against_float64(oracle):
    """All 65280 finite bfloat16 gates with up = 1: the fp32 value before the last rounding is within 2 ulp of
    g / (1 + e^-g); where that is below 1e-30 in magnitude (gates under -70) the absolute error is below 1e-36."""
    gate = _finite_bf16()
    g = bf16_bits_to_f32(gate).astype(np.float64)
    up = f32_to_bf16_bits(np.ones(gate.size, np.float32))
    x, f = oracle.swiglu(gate[None], up[None], want_f32=True)
    ref = _silu64(g)
    big = np.abs(ref) > 1e-30
    assert _ulps(f[0][big], ref[big]).max() <= 2.0
    assert np.abs(f[0][~big].astype(np.float64) - ref[~big]).max() <= 1e-36
    assert np.array_equal(x[0], f32_to_bf16_bits(f[0]))                      # the output is that value, rounded to nearest even
    # plausible mistakes are far outside that bound: e^+g, the 1 dropped, the division turned round
    sel = big & (np.abs(g) > 0.5) & (np.abs(g) < 20)
    gs = g[sel]
    for wrong in (gs / (1.0 + np.exp(gs)), gs / np.exp(-gs), (1.0 + np.exp(-gs)) / gs):
        assert _ulps(f[0][sel], wrong).max() > 1e3


def test_silu_closed_forms(oracle):
    one = f32_to_bf16_bits(np.ones(1, np.float32))
    zero = f32_to_bf16_bits(np.zeros(1, np.float32))
    assert oracle.swiglu(zero[None], one[None])[0, 0] == 0                   # silu(0) = 0
    # for g >= 20, 1 + e^-g rounds to 1 in fp32: silu(g) = g exactly, so x = bf16(g * up)
    rng = np.random.default_rng(3)
    g = f32_to_bf16_bits(rng.uniform(20, 3e4, 500).astype(np.float32))
    u = f32_to_bf16_bits(rng.standard_normal(500).astype(np.float32))
    x = oracle.swiglu(g[None], u[None])[0]
    assert np.array_equal(x, f32_to_bf16_bits(bf16_bits_to_f32(g) * bf16_bits_to_f32(u)))   # the product of two bf16 is exact in fp32
    # silu(g) - silu(-g) = g
    g = f32_to_bf16_bits(rng.uniform(0.01, 15, 500).astype(np.float32))
    ones = f32_to_bf16_bits(np.ones(500, np.float32))
    _, fp = oracle.swiglu(g[None], ones[None], want_f32=True)
    _, fm = oracle.swiglu((g ^ np.uint16(0x8000))[None], ones[None], want_f32=True)
    gv = bf16_bits_to_f32(g).astype(np.float64)
    assert np.all(np.abs(fp[0].astype(np.float64) - fm[0].astype(np.float64) - gv) <= 4 * np.spacing(gv.astype(np.float32)))
    # far below zero the result is a zero with the sign of -up, not a NaN or an overflow
    g = f32_to_bf16_bits(np.array([-89.0, -1e4, -3e38], np.float32))
    _, f = oracle.swiglu(g[None], f32_to_bf16_bits(np.array([2.0, -3.0, 1.0], np.float32))[None], want_f32=True)
    assert np.all(f[0] == 0) and np.array_equal(np.signbit(f[0]), [True, False, True])


def test_silu_times_up_random_against_float64(oracle):
    """Random gates and ups of activation size: one more rounding (the product) on top of silu's 2 ulp."""
    rng = np.random.default_rng(11)
    gate = f32_to_bf16_bits((rng.standard_normal((64, 512)) * 4).astype(np.float32))
    up = f32_to_bf16_bits((rng.standard_normal((64, 512)) * 2).astype(np.float32))
    x, f = oracle.swiglu(gate, up, want_f32=True)
    ref = _silu64(bf16_bits_to_f32(gate).astype(np.float64)) * bf16_bits_to_f32(up).astype(np.float64)
    assert _ulps(f, ref)[np.abs(ref) > 1e-30].max() <= 2.6
    assert np.array_equal(x, f32_to_bf16_bits(f))
    # monotone where silu is: above its minimum at g = -1.2785 the fp32 values never decrease with the gate
    gate = _finite_bf16()
    g = bf16_bits_to_f32(gate)
    sel = g > -1.27
    order = np.argsort(g[sel], kind="stable")
    _, f = oracle.swiglu(gate[sel][order][None], f32_to_bf16_bits(np.ones(sel.sum(), np.float32))[None], want_f32=True)
    assert np.all(np.diff(f[0].astype(np.float64)) >= 0)
