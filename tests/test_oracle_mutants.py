"""Do the pins have teeth?  Each case plants ONE plausible mistake in the oracle (on the CPU, by
wrapping one of its functions: a dropped term, a wrong sign, a transposed operand, the paper's garbled
listing taken literally, ...) and checks that at least one of the pin tests named next to it fails.
The unmodified oracle passes all of them (they are the ordinary tests of this directory)."""
import numpy as np
import pytest

import test_oracle_gemm as tg
import test_oracle_matching as tm
import test_oracle_golden as tgold
import test_oracle_norm as tn
import test_oracle_quant as tq
import test_oracle_reassembly as tr


class Mutant:
    """The oracle's API with some functions replaced; replacements get the real API as first argument."""

    def __init__(self, base, **planted):
        self._base = base
        self._planted = planted

    def __getattr__(self, name):
        if name in self._planted:
            return lambda *a, **k: self._planted[name](self._base, *a, **k)
        return getattr(self._base, name)


# ---- the planted mistakes -------------------------------------------------------------------

def unbiased_variance(o, x, kind, gamma=None, beta=None, eps=1e-5):
    y = o.norm(x, kind, gamma, beta, eps)
    if kind != o.NORM_LAYER:
        return y
    C = x.shape[1]                      # dividing the variance by C - 1 shrinks every centred value
    b = 0 if beta is None else np.asarray(beta, np.float32)
    return ((y - b) * np.float32(np.sqrt((C - 1) / C)) + b).astype(np.float32)


def rms_subtracts_mean(o, x, kind, gamma=None, beta=None, eps=1e-5):
    if kind != o.NORM_RMS:
        return o.norm(x, kind, gamma, beta, eps)
    xf = o.widen_bf16(x) if x.dtype == np.uint16 else x
    xc = (xf - xf.mean(1, keepdims=True)).astype(np.float32)
    return o.norm(xc, kind, gamma, beta, eps)


def listing_taken_literally(o, y, T):
    d = o.disassemble(y, T)             # "x / (1/T)": sub-channels multiplied by T instead of divided
    Trep = np.repeat(np.asarray(T), np.asarray(T)).astype(np.float32)
    return (d * Trep * Trep).astype(np.float32)


def floor_instead_of_ceil(o, absmax, theta):
    return np.maximum(np.floor(np.asarray(absmax, np.float64) / theta), 1).astype(np.int32)


def merge_sums(o, d, src_idx, dst_idx, return_keep=False):
    out = o.assemble(d, src_idx, dst_idx, return_keep=True)
    xhat, keep = out
    members = np.ones(np.asarray(d).shape[1])
    for s, t in zip(np.asarray(src_idx), np.asarray(dst_idx)):
        members[2 * t + 1] += 1
    xhat = (xhat * members[keep].astype(np.float32)).astype(np.float32)   # a sum where Eq. 4 has a mean
    return (xhat, keep) if return_keep else xhat


def map_forgets_the_scale(o, T, src_idx, dst_idx):
    rp, src, sc = o.build_map(T, src_idx, dst_idx)
    return rp, src, np.where(np.diff(rp)[np.searchsorted(rp, np.arange(src.size), side="right") - 1] > 1, sc, 1.0).astype(np.float32)


def truncating_quantizer(o, x, bits):
    codes, alpha, beta, rowsum = o.quantize_rows(x, bits)
    q = np.floor(np.asarray(x, np.float64) / alpha[:, None].astype(np.float64)) + beta[:, None]
    codes = np.clip(q, 0, 2 ** bits - 1).astype(np.uint8)
    return codes, alpha, beta, codes.sum(1).astype(np.int32)


def symmetric_range(o, x, bits):
    x = np.asarray(x, np.float32)
    m = np.abs(x).max(1, keepdims=True)
    both = np.concatenate([x, m, -m], 1)            # the range forced to be symmetric about zero
    codes, alpha, beta, _ = o.quantize_rows(np.ascontiguousarray(both), bits)
    codes = np.ascontiguousarray(codes[:, :x.shape[1]])
    return codes, alpha, beta, codes.sum(1).astype(np.int32)


def zero_point_sign(o, x, bits):
    codes, alpha, beta, rowsum = o.quantize_rows(x, bits)
    return codes, alpha, -beta, rowsum


def high_nibble_first(o, codes, bits, row_bytes=None):
    p = o.pack_codes(codes, bits, row_bytes)
    return ((p << 4) | (p >> 4)).astype(np.uint8) if bits == 4 else p


def gemm_drops_last_k(o, a, w):
    a = np.array(a, copy=True)
    a[:, -1] = 0
    return o.int_gemm(a, w)


def gemm_wraps_at_16_bits(o, a, w):
    return (o.int_gemm(a, w).astype(np.int64) & 0xFFFF).astype(np.int32)


def epilogue_wrong_sign(o, acc, K, ax, bx, rs, aw, bw, cs):
    good = o.epilogue(acc, K, ax, bx, rs, aw, bw, cs)   # - K bx bw where + K bx bw belongs
    corr = 2.0 * K * np.asarray(bx, np.float64)[:, None] * np.asarray(bw, np.float64)[None, :]
    return (good - corr * np.asarray(ax, np.float64)[:, None] * np.asarray(aw, np.float64)[None, :]).astype(np.float32)


def epilogue_swaps_sums(o, acc, K, ax, bx, rs, aw, bw, cs):
    acc = np.asarray(acc, np.int64)
    bxl, bwl = np.asarray(bx, np.int64)[:, None], np.asarray(bw, np.int64)[None, :]
    br = acc - bxl * np.asarray(rs, np.int64)[:, None] - bwl * np.asarray(cs, np.int64)[None, :] + K * bxl * bwl
    return ((br.astype(np.float32) * np.asarray(ax, np.float32)[:, None]) * np.asarray(aw, np.float32)[None, :]).astype(np.float32)


def weight_rows_averaged(o, W, T, src_idx, dst_idx):
    What = o.reassemble_weight(W, T, src_idx, dst_idx)
    if len(src_idx) == 0:
        return What
    rp, _, sc = o.build_map(np.asarray(T, np.int32), src_idx, dst_idx)
    g = np.diff(rp)
    return (What / np.where(g > 1, g, 1)[:, None]).astype(np.float32)   # averaged like the activations


def weight_quantized_per_tensor(o, What, bits):
    codes, alpha, beta, colsum = o.quantize_weight(What, bits)
    flat = np.asarray(What, np.float32).reshape(1, -1)
    c1, a1, b1, _ = o.quantize_rows(np.ascontiguousarray(flat), bits)
    codes = np.ascontiguousarray(c1.reshape(What.shape).T)
    O = codes.shape[0]
    return codes, np.full(O, a1[0], np.float32), np.full(O, b1[0], np.int32), codes.sum(1).astype(np.int32)


def fold_sums_the_group(o, Wp, bp, T, src_idx, dst_idx):
    W_hat, b_hat = o.fold_preceding_linear(Wp, bp, T, src_idx, dst_idx)
    rp, _, _ = o.build_map(np.asarray(T, np.int32), src_idx, dst_idx)
    members = np.where(np.diff(rp) > 1, np.diff(rp), 1)[:, None].astype(np.float64)
    return W_hat * members, None if b_hat is None else b_hat * members[:, 0]   # (W_i + W_j) where Appendix B has the mean


def fold_forgets_the_division_by_T(o, Wp, bp, T, src_idx, dst_idx):
    W_hat, b_hat = o.fold_preceding_linear(Wp, bp, T, src_idx, dst_idx)
    if len(src_idx) == 0 and np.all(np.asarray(T) == 1):
        return W_hat, b_hat
    rp, src, sc = o.build_map(np.asarray(T, np.int32), src_idx, dst_idx)
    rows = np.diff(rp) == 1
    scale_of_row = np.asarray(sc, np.float64)[rp[:-1]]
    fix = np.where(rows, 1.0 / scale_of_row, 1.0)[:, None]                      # sub-channels copied, not divided by T
    return W_hat * fix, None if b_hat is None else b_hat * fix[:, 0]


CASES = [
    ("LayerNorm divides the variance by C - 1", dict(norm=unbiased_variance),
     [lambda o: tn.test_layernorm_matches_torch_fp64(o, 64, "f32"), tn.test_layernorm_closed_form_biased_variance]),
    ("RMSNorm subtracts the mean", dict(norm=rms_subtracts_mean),
     [lambda o: tn.test_rmsnorm_matches_torch_fp64(o, 128, "f32")]),
    ("sub-channels scaled by T as in the garbled listing", dict(disassemble=listing_taken_literally),
     [tr.test_disassembly_layout_and_count, lambda o: tr.test_disassembly_preserves_layer_output(o, True)]),
    ("T rounded down", dict(num_split=floor_instead_of_ceil), [tr.test_T_rule]),
    ("merged activations summed instead of averaged", dict(assemble=merge_sums),
     [tr.test_merging_identical_channels_is_exact_and_error_closed_form,
      lambda o: tr.test_assembly_against_independent_fp64_statement(o, 1, 33, 5, 8, 9)]),
    ("map loses the 1/T of sub-channels", dict(build_map=map_forgets_the_scale),
     [lambda o: tr.test_map_form_equals_two_stage_form_bitwise(o, 1, 33, 5, 8, 9)]),
    ("quantizer truncates", dict(quantize_rows=truncating_quantizer),
     [lambda o: tq.test_quantizer_properties(o, 4), lambda o: tq.test_quantizer_brute_force_exact_rationals(o, 3)]),
    ("quantizer range symmetric about zero", dict(quantize_rows=symmetric_range),
     [lambda o: tq.test_quantizer_properties(o, 4), tq.test_8bit_matches_torch_affine_quantizer]),
    ("zero-point with the wrong sign", dict(quantize_rows=zero_point_sign),
     [lambda o: tq.test_quantizer_properties(o, 4), tgold.test_hand_worked_example_step_by_step]),
    ("4-bit codes packed high nibble first", dict(pack_codes=high_nibble_first), [tq.test_packing_layout_by_hand]),
    ("GEMM drops the last code of every row", dict(int_gemm=gemm_drops_last_k),
     [tg.test_int_gemm_brute_force_python_ints, tg.test_int_gemm_special_operands]),
    ("GEMM accumulates in 16 bits", dict(int_gemm=gemm_wraps_at_16_bits),
     [lambda o: tg.test_int_gemm_matches_numpy_int64(o, 8, 128)]),
    ("epilogue: K bx bw subtracted", dict(epilogue=epilogue_wrong_sign),
     [tg.test_epilogue_equals_direct_sum_of_corrected_products]),
    ("epilogue: row sums and column sums swapped", dict(epilogue=epilogue_swaps_sums),
     [tg.test_epilogue_equals_direct_sum_of_corrected_products]),
    ("merged weight rows averaged instead of summed", dict(reassemble_weight=weight_rows_averaged),
     [tr.test_merging_identical_channels_is_exact_and_error_closed_form]),
    ("weights quantized per tensor", dict(quantize_weight=weight_quantized_per_tensor),
     [tq.test_per_output_channel_weight_quantization]),
    ("Appendix B: merged columns summed instead of averaged", dict(fold_preceding_linear=fold_sums_the_group),
     [tr.test_fold_worked_example, lambda o: tr.test_fold_equals_runtime_reassembly(o, 0)]),
    ("Appendix B: sub-channel columns not divided by T", dict(fold_preceding_linear=fold_forgets_the_division_by_T),
     [tr.test_fold_worked_example, lambda o: tr.test_fold_equals_runtime_reassembly(o, 1)]),
]


@pytest.mark.parametrize("what,planted,pins", CASES, ids=[c[0] for c in CASES])
def test_a_planted_mistake_fails_a_pin(oracle, what, planted, pins):
    for pin in pins:                       # sanity: the real oracle passes the very same calls
        pin(oracle)
    mutant = Mutant(oracle, **planted)
    caught = 0
    for pin in pins:
        try:
            pin(mutant)
        except AssertionError:
            caught += 1
    assert caught > 0, f"no pin noticed: {what}"


# ---- the same for the offline matching (functions of oracle.calibrate, planted by replacing the
#      module's attribute, so that the functions which call them see the mistake too)

def _distance_second_term_sign(xi, xj, wi, wj):
    xi, xj, wi, wj = (np.asarray(v, np.float64) for v in (xi, xj, wi, wj))
    e = np.outer(xi, wi - wj) / 2.0 + np.outer(xj, wi - wj) / 2.0     # x_j (W_i - W_j): the sign of Eq. (5)'s second term
    return float((e * e).sum())


def _nearest(real, keep_quarter=True, use_weights=True, ties_high=False):
    def planted(y, W, T, n_match_tokens=256, rows=None):
        from oracle import calibrate
        chan_of, pos_a, pos_b = calibrate.matching_sets(T)
        ys, Wd = np.asarray(y[:n_match_tokens], np.float64), np.asarray(W, np.float64)
        rows_ = np.arange(pos_a.size) if rows is None else np.asarray(rows, np.int64)
        best_j, best_d = np.empty(rows_.size, np.int64), np.empty(rows_.size)
        for k, i in enumerate(rows_):
            c = chan_of[pos_a[i]]
            dx = ((ys[:, chan_of[pos_b]].T - ys[:, c][None, :]) ** 2).sum(1)
            dw = ((Wd[chan_of[pos_b]] - Wd[c][None, :]) ** 2).sum(1) if use_weights else 1.0
            d = (0.25 if keep_quarter else 1.0) * dx * dw
            j = int(np.flatnonzero(d == d.min())[-1]) if ties_high else int(d.argmin())
            best_j[k], best_d[k] = j, d[j]
        return best_j, best_d, pos_a, pos_b
    return planted


def _nearest_l2(farthest=False, ties_high=False):
    def planted(y, T, n_match_tokens=256):
        from oracle import calibrate
        chan_of, pos_a, pos_b = calibrate.matching_sets(T)
        ys = np.asarray(y[:n_match_tokens], np.float64)
        best_j, best_d = np.empty(pos_a.size, np.int64), np.empty(pos_a.size)
        for k in range(pos_a.size):
            d = ((ys[:, chan_of[pos_b]].T - ys[:, chan_of[pos_a[k]]][None, :]) ** 2).sum(1)
            want = d.max() if farthest else d.min()
            hits = np.flatnonzero(d == want)
            j = int(hits[-1] if ties_high else hits[0])
            best_j[k], best_d[k] = j, d[j]
        return best_j, best_d, pos_a, pos_b
    return planted


def _theta_one_float_up(absmax, rule):
    from oracle import calibrate
    th = _REAL_THETA_RULE(absmax, rule)
    return float(np.nextafter(np.float32(th), np.float32(np.inf))) if rule[0] == "expand" else th


def _sets_with_sub_channels(T):
    T = np.asarray(T, np.int64)
    chan_of = np.repeat(np.arange(T.size), T)
    return chan_of, np.arange(0, chan_of.size, 2), np.arange(1, chan_of.size, 2)


def _select_longest(best_d, best_j, pos_a, pos_b, r):
    r = min(int(r), pos_a.size)
    pick = np.sort(np.argsort(-np.asarray(best_d), kind="stable")[:r])
    return (pos_a[pick] // 2).astype(np.int32), ((pos_b[np.asarray(best_j)[pick]] - 1) // 2).astype(np.int32)


def _grid_from_zero(absmax, P):
    m = np.asarray(absmax, np.float32).astype(np.float64)
    return [float(np.float32(m.min() + (p / P) * (m.max() - m.min()))) for p in range(0, P)]


from oracle import calibrate as _calibrate_module
_REAL_THETA_RULE = _calibrate_module.theta_from_rule

MATCHING_CASES = [
    ("Eq. (5): second term with the wrong sign", "pair_distance", _distance_second_term_sign,
     [tm.test_distance_is_the_output_error_of_merging, tm.test_distance_properties]),
    ("Eq. (5): the factor 1/4 dropped", "nearest_by_eq5", _nearest(None, keep_quarter=False),
     [tm.test_nearest_by_eq5_against_brute_force, tm.test_matching_by_hand]),
    ("matching on activations only", "nearest_by_eq5", _nearest(None, use_weights=False),
     [tm.test_nearest_by_eq5_against_brute_force, tm.test_matching_by_hand]),
    ("sub-channels of split channels take part", "matching_sets", _sets_with_sub_channels,
     [tm.test_nearest_by_eq5_against_brute_force]),
    ("the r longest edges are merged", "select_edges", _select_longest, [tm.test_matching_by_hand]),
    ("theta grid starts at min(m)", "theta_grid", _grid_from_zero, [tm.test_theta_grid_is_algorithm_1]),
    ("L2 matching: the FARTHEST member of B", "nearest_by_l2", _nearest_l2(farthest=True),
     [tm.test_l2_matching_by_hand, tm.test_l2_matching_against_brute_force]),
    ("L2 matching: ties to the higher member", "nearest_by_l2", _nearest_l2(ties_high=True),
     [tm.test_l2_matching_by_hand, tm.test_l2_matching_against_brute_force]),
    ("expansion threshold one float32 too large", "theta_from_rule", _theta_one_float_up,
     [tm.test_expansion_threshold_is_the_largest_that_adds_enough]),
]


@pytest.mark.parametrize("what,name,planted,pins", MATCHING_CASES, ids=[c[0] for c in MATCHING_CASES])
def test_a_planted_matching_mistake_fails_a_pin(oracle, monkeypatch, what, name, planted, pins):
    import inspect
    from oracle import calibrate

    def run(pin):
        return pin(oracle) if inspect.signature(pin).parameters else pin()

    for pin in pins:
        run(pin)
    monkeypatch.setattr(calibrate, name, planted)
    caught = 0
    for pin in pins:
        try:
            run(pin)
        except AssertionError:
            caught += 1
    assert caught > 0, f"no pin noticed: {what}"
