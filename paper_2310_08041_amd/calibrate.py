"""Offline calibration that manufactures a reassembly map for a batch of activations.

This is NOT the hot path: it runs once per layer, before inference (Sec. 4.3: the channel indices are
pre-computed from calibration data).  This module only SEQUENCES library calls; every step is computed
inside libqllm:

  per-channel max |y| after the norm     qllm_norm_channel_absmax        (device; Sec. 4.1.1, vector m of Algorithm 1)
  theta                                  qllm_theta_for_expansion_host / qllm_theta_grid_host  (Sec. 5.2, Algorithm 1)
  T = ceil(m / theta), the map           qllm_build_map_host             (Sec. 4.1.1, Eq. 3 + Eq. 4)
  sets A and B                           qllm_matching_sets_host         (Appendix A step 1)
  nearest member of B for every A        qllm_match_nearest              (device; Eq. (5) with the layer's weights, plain
                                                                          L2 on the activations without: the benchmark's
                                                                          policy for synthetic activations)
  the r shortest edges as (src, dst)     qllm_pairs_host                 (Appendix A step 3)
  score of a theta                       the hot path itself, qllm_linear_f64, qllm_sq_error   (Algorithm 1)

torch allocates the device buffers and moves results to the host.
"""
import numpy as np
import torch

from . import binding as b


def choose_theta(absmax, rule):
    """("fixed", theta) | ("tmax", T_max): theta = max(m) / T_max | ("expand", ratio): the largest theta whose
    disassembly adds at least round(ratio * C) channels (Sec. 5.2 fixes theta through the expansion ratio)."""
    kind, val = rule
    m = np.asarray(absmax, np.float32)
    if kind == "fixed":
        return float(np.float32(val))
    if kind == "tmax":
        return float(np.float32(m.max()) / np.float32(val))
    if kind == "expand":
        return b.qllm_theta_for_expansion_host(m, max(1, int(round(val * m.size))))
    raise ValueError(kind)


def match_pairs(y, num_split, r, W=None):
    """y: [n, C] fp32 device tensor of norm outputs; W: None (plain L2) or the layer's [C, O] fp32 device weights
    (Eq. 5).  Returns (src_idx, dst_idx) int32 numpy arrays and the per-member (best_j, best_d) device tensors."""
    sets = b.qllm_matching_sets_host(num_split)
    nA, nB = sets["chan_a"].size, sets["chan_b"].size
    if r == 0 or nA == 0 or nB == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32), None, None
    chan_a, chan_b = torch.from_numpy(sets["chan_a"]).to(y.device), torch.from_numpy(sets["chan_b"]).to(y.device)
    best_j = torch.empty(nA, dtype=torch.int32, device=y.device)
    best_d = torch.empty(nA, dtype=torch.float64, device=y.device)
    ws = torch.empty(b.qllm_match_workspace_bytes(nA, nB), dtype=torch.uint8, device=y.device)
    b.qllm_match_nearest(y, W, chan_a, chan_b, best_j, best_d, ws)
    src_idx, dst_idx = b.qllm_pairs_host(best_d.cpu().numpy(), best_j.cpu().numpy(), sets["pos_a"], sets["pos_b"], r)
    return src_idx, dst_idx, best_j, best_d


def calibrate(x, norm, gamma, beta, eps, theta_rule, merge=True, n_match=256, W=None, assemble_more=0.0):
    """x: [N, C] device tensor (fp32 / bf16); W: None, or the layer's [C, O] fp32 device weights, which
    switches the pair selection to the distance of Eq. (5).  Returns the dict of qllm_build_map_host plus
    theta, absmax, src_idx, dst_idx."""
    N, C = x.shape
    absmax = torch.zeros(C, dtype=torch.float32, device=x.device)
    y = torch.empty((min(N, n_match), C), dtype=torch.float32, device=x.device)
    b.qllm_norm_channel_absmax(x, norm, gamma, beta, eps, absmax, y)
    m = absmax.cpu().numpy()
    theta = choose_theta(m, theta_rule)
    sizing = b.qllm_build_map_host(m, theta, [], [], with_plan=False)
    r = int(sizing["nnz"] - C) if merge else 0
    r += int(round(assemble_more * C))   # assemble more channels than were disassembled: C^ < C, a shorter GEMM
    src_idx, dst_idx, _, _ = match_pairs(y, sizing["num_split"], r, W)
    out = b.qllm_build_map_host(m, theta, src_idx, dst_idx)
    out.update(theta=theta, absmax=m, src_idx=src_idx, dst_idx=dst_idx)
    return out


def grid_search_theta(x, norm, gamma, beta, eps, W, a_bits, w_bits, P, n_match=256):
    """Algorithm 1 for one linear layer: for every theta of the grid, disassemble, merge the nearest pairs
    under Eq. (5), quantize, run the reassembled layer (the library's hot path) on the calibration batch
    and take the squared error of its output against the full-precision norm -> linear; keep the theta
    with the smallest error.  x: [N, C] device tensor, W: [C, O] fp32 device tensor.
    Returns dict(theta, thetas, losses, map) with `map` the result of `calibrate` at the chosen theta."""
    N, C = x.shape
    O = W.shape[1]
    absmax = torch.zeros(C, dtype=torch.float32, device=x.device)
    y = torch.empty((N, C), dtype=torch.float32, device=x.device)
    b.qllm_norm_channel_absmax(x, norm, gamma, beta, eps, absmax, y)
    ref = torch.empty((N, O), dtype=torch.float64, device=x.device)
    b.qllm_linear_f64(y, W, ref)
    W_host = W.cpu().numpy()
    thetas = b.qllm_theta_grid_host(absmax.cpu().numpy(), P)
    loss = torch.empty(1, dtype=torch.float64, device=x.device)
    err_ws = torch.empty(b.qllm_sq_error_workspace_bytes(N), dtype=torch.uint8, device=x.device)
    losses, maps = [], []
    for theta in thetas:
        cal = calibrate(x, norm, gamma, beta, eps, ("fixed", theta), n_match=n_match, W=W)
        dmap = b.DeviceMap(cal["row_ptr"], cal["src"], cal["scale"], C, cal["plan"])
        q = b.qllm_quantize_weight_host(W_host, cal["row_ptr"], cal["src"], w_bits)
        dw = b.DeviceWeight(q["codes"], q["scale"], q["zero"], q["colsum"], dmap.C_out, w_bits)
        out = torch.empty((N, O), dtype=torch.float32, device=x.device)
        ws = torch.empty(b.qllm_workspace_bytes(N, dmap.C_out, O, a_bits), dtype=torch.uint8, device=x.device)
        b.qllm_reassembled_linear(x, norm, gamma, beta, eps, dmap, a_bits, dw, out, ws)
        b.qllm_sq_error(out, ref, loss, err_ws)
        losses.append(float(loss.cpu().numpy()[0]))
        maps.append(cal)
    best = min(range(len(losses)), key=lambda k: (losses[k], k))
    return dict(theta=thetas[best], thetas=thetas, losses=losses, map=maps[best])
