"""The oracle against a hand-worked example (tests/golden/hand_worked_example.json)."""
import json
import os

import numpy as np

G = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked_example.json")))


def test_hand_worked_example_step_by_step(oracle):
    y = np.array([G["y"]], np.float32)
    T = oracle.num_split(np.abs(y[0]), G["theta"])
    assert T.tolist() == G["T"]
    d = oracle.disassemble(y, T)
    assert d[0].tolist() == G["disassembled"]
    xh = oracle.assemble(d, G["src_idx"], G["dst_idx"])
    assert xh[0].tolist() == G["x_hat"]

    row_ptr, src, scale = oracle.build_map(T, G["src_idx"], G["dst_idx"])
    assert row_ptr.tolist() == G["map_row_ptr"]
    assert src.tolist() == G["map_src"]
    assert scale.tolist() == [float(np.float32(n / dn)) for n, dn in G["map_scale_num_den"]]
    assert oracle.apply_map(y, row_ptr, src, scale)[0].tolist() == G["x_hat"]

    codes, alpha, beta, rowsum = oracle.quantize_rows(xh, G["bits"])
    assert codes[0].tolist() == G["act_codes"]
    assert (alpha[0], beta[0], rowsum[0]) == (G["act_alpha"], G["act_beta"], G["act_rowsum"])

    W = np.array(G["W"], np.float32)
    What = oracle.reassemble_weight(W, T, G["src_idx"], G["dst_idx"])
    assert What.tolist() == G["W_hat"]
    assert (y.astype(np.float64) @ W.astype(np.float64))[0].tolist() == G["y_times_W"]
    assert (xh.astype(np.float64) @ What.astype(np.float64))[0].tolist() == G["x_hat_times_W_hat"]
    assert (np.array(G["y_times_W"]) - np.array(G["x_hat_times_W_hat"])).tolist() == G["merge_error"]

    wcodes, aw, bw, cs = oracle.quantize_weight(What, G["bits"])
    assert wcodes.tolist() == G["w_codes"]
    assert aw.tolist() == G["w_alpha"] and bw.tolist() == G["w_beta"] and cs.tolist() == G["w_colsum"]

    acc = oracle.int_gemm(codes, wcodes)
    assert acc[0].tolist() == G["acc"]
    Y = oracle.epilogue(acc, xh.shape[1], alpha, beta, rowsum, aw, bw, cs)
    assert Y[0].tolist() == G["Y"]
    assert oracle.dequant_linear_direct(codes, wcodes, alpha, beta, aw, bw)[0].tolist() == G["Y"]


def test_hand_worked_example_whole_path(oracle):
    x = np.array([G["y"]], np.float32)
    What = np.array(G["W_hat"], np.float32)
    wq = oracle.quantize_weight(What, G["bits"])
    out = oracle.reassembled_linear(x, oracle.NORM_NONE, None, None, 0.0, G["T"], G["src_idx"], G["dst_idx"],
                                    G["bits"], wq)
    assert out["codes"][0].tolist() == G["act_codes"]
    assert out["acc"][0].tolist() == G["acc"]
    assert out["y"][0].tolist() == G["Y"]
    assert (out["alpha"][0], out["beta"][0], out["rowsum"][0]) == (G["act_alpha"], G["act_beta"], G["act_rowsum"])
