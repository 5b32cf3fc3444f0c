"""Offline calibration that manufactures a reassembly map for a batch of activations.

This is NOT the hot path: it runs once per layer, before inference (Sec. 4.3: the channel indices are
pre-computed from calibration data).  The per-channel statistic comes from the library's own kernel
(qllm_norm_channel_absmax); T and the CSR map come from qllm_build_map_host.  The pair selection in
between (Appendix A: one edge from every member of set A to its nearest member of set B, keep the r
shortest) comes in two forms: with the layer's weights at hand, the distance of Eq. (5) through the
library's own kernel (qllm_match_nearest, fp64 matrix cores) and qllm_select_edges_host
(`match_pairs_eq5`); without weights -- the benchmark's policy for synthetic activations -- the plain
L2 distance between activation columns over the first `n_match` tokens with torch matrix products
as a library primitive (`match_pairs`).
"""
import numpy as np
import torch

from . import binding as b


def _extra_channels(absmax, theta):
    return b.qllm_build_map_host(absmax, theta, [], [], with_plan=False)["nnz"] - absmax.size


def choose_theta(absmax, rule):
    """("fixed", theta) | ("tmax", T_max): theta = max(m)/T_max | ("expand", ratio): the largest theta
    whose disassembly adds at least ratio*C channels (Sec. 5.2 fixes theta through the expansion ratio)."""
    kind, val = rule
    m = np.asarray(absmax, np.float32)
    if kind == "fixed":
        return float(np.float32(val))
    if kind == "tmax":
        return float(np.float32(m.max()) / np.float32(val))
    if kind == "expand":
        target = max(1, int(round(val * m.size)))
        hi = float(m.max())
        lo = hi / 1e6
        for _ in range(200):
            mid = 0.5 * (lo + hi)
            if _extra_channels(m, float(np.float32(mid))) >= target:
                lo = mid
            else:
                hi = mid
            if hi - lo <= 1e-7 * hi:
                break
        return float(np.float32(lo))
    raise ValueError(kind)


def match_pairs(y, num_split, r, chunk=4096):
    """y: [n, C] fp32 device tensor of norm outputs.  Returns (src_idx, dst_idx) int32 numpy arrays."""
    T = torch.as_tensor(num_split, device=y.device, dtype=torch.int64)
    chan_of = torch.repeat_interleave(torch.arange(T.numel(), device=y.device), T)
    eligible = T[chan_of] == 1
    pos = torch.arange(chan_of.numel(), device=y.device)
    pos_a = pos[(pos % 2 == 0) & eligible]
    pos_b = pos[(pos % 2 == 1) & eligible]
    r = min(r, pos_a.numel())
    if r == 0 or pos_b.numel() == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32)
    yd = y.double()
    cols_b = yd[:, chan_of[pos_b]]
    nb2 = (cols_b * cols_b).sum(0)
    best_d, best_j = [], []
    for s in range(0, pos_a.numel(), chunk):
        a = yd[:, chan_of[pos_a[s:s + chunk]]]
        d2 = (a * a).sum(0)[:, None] + nb2[None, :] - 2.0 * (a.T @ cols_b)
        d, j = d2.min(1)
        best_d.append(d)
        best_j.append(j)
    best_d, best_j = torch.cat(best_d), torch.cat(best_j)
    pick = torch.argsort(best_d, stable=True)[:r].sort().values
    src_idx = (pos_a[pick] // 2).to(torch.int32).cpu().numpy()
    dst_idx = ((pos_b[best_j[pick]] - 1) // 2).to(torch.int32).cpu().numpy()
    return src_idx, dst_idx


def matching_sets(num_split, device):
    """Appendix A step 1 on the disassembled axis: positions of set A (even) and set B (odd), without the
    sub-channels of split channels (Sec. 4.1.2), and the channel of every position."""
    T = torch.as_tensor(num_split, device=device, dtype=torch.int64)
    chan_of = torch.repeat_interleave(torch.arange(T.numel(), device=device), T)
    eligible = T[chan_of] == 1
    pos = torch.arange(chan_of.numel(), device=device)
    return chan_of, pos[(pos % 2 == 0) & eligible], pos[(pos % 2 == 1) & eligible]


def match_pairs_eq5(y, W, num_split, r):
    """y: [n, C] fp32 device tensor of norm outputs, W: [C, O] fp32 device tensor of the layer's weights.
    Returns (src_idx, dst_idx) int32 numpy arrays, and the per-member (best_j, best_d) device tensors."""
    chan_of, pos_a, pos_b = matching_sets(num_split, y.device)
    nA, nB = pos_a.numel(), pos_b.numel()
    if r == 0 or nA == 0 or nB == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32), None, None
    chan_a = chan_of[pos_a].to(torch.int32).contiguous()
    chan_b = chan_of[pos_b].to(torch.int32).contiguous()
    best_j = torch.empty(nA, dtype=torch.int32, device=y.device)
    best_d = torch.empty(nA, dtype=torch.float64, device=y.device)
    ws = torch.empty(b.qllm_match_workspace_bytes(nA, nB), dtype=torch.uint8, device=y.device)
    b.qllm_match_nearest(y, W, chan_a, chan_b, best_j, best_d, ws)
    pick = torch.from_numpy(b.qllm_select_edges_host(best_d.cpu().numpy(), r).astype(np.int64)).to(y.device)
    src_idx = (pos_a[pick] // 2).to(torch.int32).cpu().numpy()
    dst_idx = ((pos_b[best_j[pick].long()] - 1) // 2).to(torch.int32).cpu().numpy()
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
    T = sizing["num_split"]
    r = int(sizing["nnz"] - C) if merge else 0
    r += int(round(assemble_more * C))   # assemble more channels than were disassembled: C^ < C, a shorter GEMM
    if W is None:
        src_idx, dst_idx = match_pairs(y, T, r)
    else:
        src_idx, dst_idx, _, _ = match_pairs_eq5(y, W, T, r)
    out = b.qllm_build_map_host(m, theta, src_idx, dst_idx)
    out.update(theta=theta, absmax=m, src_idx=src_idx, dst_idx=dst_idx)
    return out


def theta_grid(absmax, P):
    """Algorithm 1: theta_p = min(m) + p / P (max(m) - min(m)) for p = 1..P, rounded once to float32."""
    m = np.asarray(absmax, np.float32).astype(np.float64)
    return [float(np.float32(m.min() + (p / P) * (m.max() - m.min()))) for p in range(1, P + 1)]


def grid_search_theta(x, norm, gamma, beta, eps, W, a_bits, w_bits, P, n_match=256):
    """Algorithm 1 for one linear layer: for every theta of the grid, disassemble, merge the nearest pairs
    under Eq. (5), quantize, run the reassembled layer (the library's hot path) on the calibration batch
    and take the squared error of its output against the full-precision norm -> linear; keep the theta
    with the smallest error.  x: [N, C] device tensor, W: [C, O] fp32 device tensor.  The full-precision
    reference is a torch matrix product in float64 (a library primitive).
    Returns dict(theta, thetas, losses, map) with `map` the result of `calibrate` at the chosen theta."""
    N, C = x.shape
    absmax = torch.zeros(C, dtype=torch.float32, device=x.device)
    y = torch.empty((N, C), dtype=torch.float32, device=x.device)
    b.qllm_norm_channel_absmax(x, norm, gamma, beta, eps, absmax, y)
    ref = y.double() @ W.double()
    W_host = W.cpu().numpy()
    thetas = theta_grid(absmax.cpu().numpy(), P)
    losses, maps = [], []
    for theta in thetas:
        cal = calibrate(x, norm, gamma, beta, eps, ("fixed", theta), n_match=n_match, W=W)
        dmap = b.DeviceMap(cal["row_ptr"], cal["src"], cal["scale"], C, cal["plan"])
        q = b.qllm_quantize_weight_host(W_host, cal["row_ptr"], cal["src"], w_bits)
        dw = b.DeviceWeight(q["codes"], q["scale"], q["zero"], q["colsum"], dmap.C_out, w_bits)
        out = torch.empty((N, W.shape[1]), dtype=torch.float32, device=x.device)
        ws = torch.empty(b.qllm_workspace_bytes(N, dmap.C_out, W.shape[1], a_bits), dtype=torch.uint8, device=x.device)
        b.qllm_reassembled_linear(x, norm, gamma, beta, eps, dmap, a_bits, dw, out, ws)
        err = out.double() - ref
        losses.append(float((err * err).sum().item()))
        maps.append(cal)
    best = int(np.argmin(losses))
    return dict(theta=thetas[best], thetas=thetas, losses=losses, map=maps[best])
