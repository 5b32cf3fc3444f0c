"""The oracle's side of the comparison of Sec. 4.1.2 (channels dropped instead of merged), pinned to things
other than itself: a map worked out by hand, the whole-path C routine for the merging map, and plain numpy
slicing for what "dropping a channel" means."""
import numpy as np
import pytest

from oracle import api, calibrate
from paper_2310_08041_amd import binding as b
from paper_2310_08041_amd import workloads as wl


def test_pruned_map_worked_by_hand():
    # channels 0..3 with T = 1, 2, 1, 1: the disassembled axis is [0, 1, 1, 2, 3]; set A = positions 0, 2, 4.
    # Dropping A-member 2 (position 4, channel 3) leaves [0, 1, 1, 2] with scales 1, 1/2, 1/2, 1.
    row_ptr, src, scale = calibrate.build_pruned_map([1, 2, 1, 1], [2])
    assert row_ptr.tolist() == [0, 1, 2, 3, 4] and src.tolist() == [0, 1, 1, 2]
    assert scale.tolist() == [1.0, 0.5, 0.5, 1.0]
    # nothing dropped: disassembly alone
    row_ptr, src, scale = calibrate.build_pruned_map([1, 3], [])
    assert src.tolist() == [0, 1, 1, 1] and np.array_equal(scale, np.float32([1, 1 / 3, 1 / 3, 1 / 3]))


def small_layer(seed, N=24, C=96, O=40):
    w = wl.WORKLOADS["tiny"]
    x, _, _ = wl.draw_activations(w, N, C, seed)
    gamma, beta = wl.draw_norm_params(w, C, seed)
    W = wl.draw_weight(w, C, O, seed)
    return w, x, gamma, beta, W


@pytest.mark.parametrize("bits", [4, 8])
def test_map_linear_equals_the_whole_path_routine_for_the_merging_map(bits):
    # map_linear puts the path together from its parts for any map; for the map of Eq. 3 + Eq. 4 the C routine that
    # runs the whole path from (T, src_idx, dst_idx) has to give the same output, bit for bit
    w, x, gamma, beta, W = small_layer(3)
    norm = {"none": 0, "layer": 1, "rms": 2}[w.norm]
    cal = calibrate.calibrate(api.norm(x, norm, gamma, beta, w.eps), ("expand", 0.05), assemble_more=0.1)
    assert cal["src_idx"].size > 0 and cal["T"].max() > 1
    wq = api.quantize_weight(api.reassemble_weight(W, cal["T"], cal["src_idx"], cal["dst_idx"]), bits)
    whole = api.reassembled_linear(x, norm, gamma, beta, w.eps, cal["T"], cal["src_idx"], cal["dst_idx"], bits, wq)["y"]
    parts = calibrate.map_linear(x, norm, gamma, beta, w.eps, *api.build_map(cal["T"], cal["src_idx"], cal["dst_idx"]), W, bits, bits)
    assert np.array_equal(parts.view(np.uint32), whole.view(np.uint32))


def test_dropping_a_channel_is_removing_its_column_and_weight_row():
    # no norm, nothing split: the pruned layer is the plain quantized layer on x and W without those channels
    w, x, _, _, W = small_layer(5)
    x = wl.bf16_bits_to_f32(x) if x.dtype == np.uint16 else x
    C = x.shape[1]
    T = np.ones(C, np.int32)
    src_idx = np.array([0, 3, 4, 11], np.int32)                  # members of set A: channels 0, 6, 8, 22
    kept = np.setdiff1d(np.arange(C), 2 * src_idx)
    got = calibrate.map_linear(x, 0, None, None, 0.0, *calibrate.build_pruned_map(T, src_idx), W, 4, 4)
    codes, alpha, zero, rowsum = api.quantize_rows(np.ascontiguousarray(x[:, kept]), 4)
    wcodes, aw, bw, cs = api.quantize_weight(np.ascontiguousarray(W[kept]), 4)
    want = api.dequant_linear_direct(codes, wcodes, alpha, zero, aw, bw)
    assert np.allclose(got, want, rtol=1e-5, atol=1e-5 * np.abs(want).max())


def test_errors_of_both_maps_and_their_order_on_a_planted_case():
    # two copies of one channel: merging them (Eq. 4) loses nothing before quantization, dropping one loses its
    # whole contribution, so the pruning error has to come out larger
    w, x, gamma, beta, W = small_layer(7, N=32, C=64, O=48)
    x = wl.bf16_bits_to_f32(x) if x.dtype == np.uint16 else x.copy()
    x[:, 1] = x[:, 0]                                           # position 0 is in set A, position 1 in set B
    T = np.ones(64, np.int32)
    errs = calibrate.layer_output_errors(np.ascontiguousarray(x), 0, None, None, 0.0, W, T, [0], [0], 8, 8)
    assert 0.0 <= errs["assembly"] < errs["pruning"]
    direct = np.ascontiguousarray(x).astype(np.float64) @ W.astype(np.float64)
    lost = np.outer(x[:, 0].astype(np.float64), W[0].astype(np.float64))     # what dropping channel 0 removes
    assert abs(errs["pruning"] - (lost ** 2).sum()) < 0.05 * (lost ** 2).sum() + 1e-3 * (direct ** 2).sum()


def test_host_pruned_map_matches_the_oracle():
    w = wl.WORKLOADS["llama7b_qkv"]
    x, _, _ = wl.draw_activations(w, 64, 1000, 9)
    gamma, beta = wl.draw_norm_params(w, 1000, 9)
    cal = calibrate.calibrate(api.norm(x, 2, gamma, beta, w.eps), ("expand", 0.03), assemble_more=0.2)
    want = calibrate.build_pruned_map(cal["T"], cal["src_idx"])
    got = b.qllm_build_pruned_map_host(cal["absmax"], cal["theta"], cal["src_idx"])
    assert np.array_equal(got["num_split"], cal["T"]) and got["C_out"] == want[0].size - 1 == got["nnz"]
    for g, wnt in zip((got["row_ptr"], got["src"], got["scale"]), want):
        assert np.array_equal(g, wnt)
    assert got["plan"] is not None
    # an index outside set A is refused, and so is a member listed twice
    with pytest.raises(b.QllmError):
        b.qllm_build_pruned_map_host(cal["absmax"], cal["theta"], [10 ** 6])
    with pytest.raises(b.QllmError):
        b.qllm_build_pruned_map_host(cal["absmax"], cal["theta"], [int(cal["src_idx"][0])] * 2)
