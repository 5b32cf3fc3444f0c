"""Oracle-side offline calibration: turns norm outputs into (absmax, theta, T, src_idx, dst_idx).

TEST INFRASTRUCTURE ONLY.  This is the small part of the paper's offline procedure (Sec. 4.1.1,
Sec. 4.1.2, Appendix A, Algorithm 1) needed to manufacture a reassembly map for synthetic inputs:

  m_c   = max over tokens of |y_c|                               (Algorithm 1, "max value of each channel")
  theta = fixed | chosen for an expansion ratio (Sec. 5.2) | max(m)/T_max
  T_c   = ceil(m_c / theta)                                      (Sec. 4.1.1)
  pairs = bipartite soft matching (Appendix A): set A = even, set B = odd positions of the
          disassembled axis; one edge from every A-member to its nearest B-member; the
          r = sum(T_c - 1) shortest edges are merged.  Sub-channels of disassembled channels take
          no part (Sec. 4.1.2).

`pruned_linear` and `layer_output_errors` serve the comparison of Sec. 4.1.2 (channels dropped instead of merged).

Two edge lengths are provided: the plain L2 distance between activation columns over the first
`n_match_tokens` tokens (the benchmark's policy for synthetic data: `nearest_by_l2`, `nearest_pairs`), and
the paper's Eq. (5), which also involves the weights (`pair_distance`, `nearest_by_eq5`, `match_pairs_eq5`).
Every distance is formed from explicit differences in float64, member by member.
"""
import numpy as np

from . import api


def extra_channels(absmax, theta):
    """sum(T_c - 1): how many channels disassembly with this threshold adds (Sec. 4.1.1)."""
    return int((api.num_split(absmax, np.float32(theta)).astype(np.int64) - 1).sum())


def theta_from_rule(absmax, rule):
    """("fixed", theta) | ("tmax", T_max): theta = max(m) / T_max | ("expand", ratio): the LARGEST float32
    threshold whose disassembly adds at least round(ratio * C) channels (Sec. 5.2 fixes theta through the
    expansion ratio).  The number of added channels never grows with theta, so the largest such float32 is
    found by bisection over the float32 values themselves (positive floats order like their bit patterns)."""
    kind, val = rule
    m = np.asarray(absmax, np.float32)
    if kind == "fixed":
        return float(np.float32(val))
    if kind == "tmax":
        return float(np.float32(m.max()) / np.float32(val))
    if kind == "expand":
        target = max(1, int(round(val * m.size)))
        as_f32 = lambda bits: np.array([bits], np.uint32).view(np.float32)[0]
        hi = int(np.array([m.max()], np.float32).view(np.uint32)[0])   # adds nothing: T = 1 everywhere
        lo = int(np.array([m.max() * np.float32(2.0 ** -20)], np.float32).view(np.uint32)[0])  # T up to 2^20: the search floor
        if extra_channels(m, as_f32(lo)) < target:
            raise ValueError("no threshold above max(m) / 2^20 adds that many channels")
        while hi - lo > 1:                                              # invariant: lo adds enough, hi does not
            mid = (lo + hi) // 2
            if extra_channels(m, as_f32(mid)) >= target:
                lo = mid
            else:
                hi = mid
        return float(as_f32(lo))
    raise ValueError(kind)


def nearest_by_l2(y, T, n_match_tokens=256):
    """Appendix A step 2 with the plain squared L2 distance between activation columns,
    D(i, j) = sum over tokens of (y[n, i] - y[n, j])^2: for every member of set A its nearest member of
    set B, the lowest index on ties.  Differences formed explicitly, in float64, by the C routine
    `oracle_nearest_member` (the full-size configurations have 14 000 x 14 000 pairs of 256 tokens).
    Returns (best_j, best_d, pos_a, pos_b) like nearest_by_eq5."""
    chan_of, pos_a, pos_b = matching_sets(T)
    if pos_a.size == 0 or pos_b.size == 0:
        return np.zeros(pos_a.size, np.int64), np.zeros(pos_a.size, np.float64), pos_a, pos_b
    best_j, best_d = api.nearest_member(np.asarray(y[:n_match_tokens], np.float32), None, chan_of[pos_a], chan_of[pos_b])
    return best_j, best_d, pos_a, pos_b


def nearest_pairs(y, T, r, n_match_tokens=256):
    """Appendix A steps 1-3 with the plain L2 distance (the benchmark's policy for synthetic activations,
    which come without trained weights).  Returns (src_idx, dst_idx), int32 [min(r, |A|)], as indices into
    set A / set B."""
    chan_of, pos_a, pos_b = matching_sets(T)
    if r == 0 or pos_a.size == 0 or pos_b.size == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32)
    best_j, best_d, pos_a, pos_b = nearest_by_l2(y, T, n_match_tokens)
    return select_edges(best_d, best_j, pos_a, pos_b, r)


def matching_sets(T):
    """Appendix A step 1 on the disassembled axis: (chan_of, pos_a, pos_b) with set A = even and
    set B = odd positions, sub-channels of disassembled channels left out (Sec. 4.1.2)."""
    T = np.asarray(T, np.int64)
    chan_of = np.repeat(np.arange(T.size), T)
    eligible = T[chan_of] == 1
    pos_a = np.arange(0, chan_of.size, 2)
    pos_b = np.arange(1, chan_of.size, 2)
    return chan_of, pos_a[eligible[pos_a]], pos_b[eligible[pos_b]]


def pair_distance(xi, xj, wi, wj):
    """Eq. (5) as printed: the squared norm of x_i (W_i - W_j) / 2 + x_j (W_j - W_i) / 2, the error
    that merging channels i and j by Eq. (4) leaves in the layer's output.  xi, xj: activation columns
    over the calibration tokens; wi, wj: weight rows over the output features.  float64."""
    xi, xj = np.asarray(xi, np.float64), np.asarray(xj, np.float64)
    wi, wj = np.asarray(wi, np.float64), np.asarray(wj, np.float64)
    e = np.outer(xi, wi - wj) / 2.0 + np.outer(xj, wj - wi) / 2.0
    return float((e * e).sum())


def nearest_by_eq5(y, W, T, n_match_tokens=256, rows=None):
    """Appendix A step 2 with the distance of Eq. (5): for every member of set A (or those listed in
    `rows`, as indices into set A's eligible members) its nearest member of set B, lowest index on
    ties.  The error term of Eq. (5) is the outer product of (x_i - x_j) / 2 and (W_i - W_j), so its
    squared norm is |x_i - x_j|^2 |W_i - W_j|^2 / 4: the differences are formed explicitly, in float64.
    y: [N, C] activations, W: [C, O].  Returns (best_j, best_d): index into set B's eligible members
    and the distance, plus (pos_a, pos_b) for the caller."""
    chan_of, pos_a, pos_b = matching_sets(T)
    ys = np.asarray(y[:n_match_tokens], np.float64)
    Wd = np.asarray(W, np.float64)
    xb = ys[:, chan_of[pos_b]].T                          # [|B|, n]
    wb = Wd[chan_of[pos_b]]                               # [|B|, O]
    rows = np.arange(pos_a.size) if rows is None else np.asarray(rows, np.int64)
    best_j = np.empty(rows.size, np.int64)
    best_d = np.empty(rows.size, np.float64)
    for k, i in enumerate(rows):
        c = chan_of[pos_a[i]]
        dx = xb - ys[:, c][None, :]
        dw = wb - Wd[c][None, :]
        d = 0.25 * (dx * dx).sum(1) * (dw * dw).sum(1)
        j = int(d.argmin())                               # numpy returns the first minimum
        best_j[k], best_d[k] = j, d[j]
    return best_j, best_d, pos_a, pos_b


def select_edges(best_d, best_j, pos_a, pos_b, r):
    """Appendix A step 3: the r shortest edges (ties to the lower A index), as (src_idx, dst_idx) in
    the A / B indexing of the run-time pseudo-code, ascending in src_idx."""
    r = min(int(r), pos_a.size)
    if r == 0 or pos_b.size == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32)
    pick = np.argsort(best_d, kind="stable")[:r]
    pick.sort()
    return (pos_a[pick] // 2).astype(np.int32), ((pos_b[best_j[pick]] - 1) // 2).astype(np.int32)


def match_pairs_eq5(y, W, T, r, n_match_tokens=256):
    """Appendix A steps 1-3 with Eq. (5).  Returns (src_idx, dst_idx)."""
    chan_of, pos_a, pos_b = matching_sets(T)
    if r == 0 or pos_a.size == 0 or pos_b.size == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32)
    best_j, best_d, pos_a, pos_b = nearest_by_eq5(y, W, T, n_match_tokens)
    return select_edges(best_d, best_j, pos_a, pos_b, r)


def calibrate(y, theta_rule, merge=True, n_match_tokens=256, assemble_more=0.0):
    """y: norm output [N, C] float32 (from the oracle).  Returns a dict with absmax, theta, T,
    src_idx, dst_idx.  With merge=True sum(T-1) + assemble_more * C pairs are merged, so C^ == C for
    assemble_more == 0 and C^ < C above it (the speed-up variant of the introduction; fewer only if set A
    has fewer eligible members than that)."""
    absmax = api.channel_absmax(y)
    theta = theta_from_rule(absmax, theta_rule)
    T = api.num_split(absmax, theta)
    r = int((T.astype(np.int64) - 1).sum()) if merge else 0
    r += int(round(assemble_more * T.size))             # "assemble more than disassembled": C^ < C (Sec. 1)
    src_idx, dst_idx = nearest_pairs(y, T, r, n_match_tokens)
    return dict(absmax=absmax, theta=theta, T=T, src_idx=src_idx, dst_idx=dst_idx)


def theta_grid(absmax, P):
    """Algorithm 1: theta_p = min(m) + p / P (max(m) - min(m)), p = 1..P, each rounded once to float32."""
    m = np.asarray(absmax, np.float32).astype(np.float64)
    lo, hi = m.min(), m.max()
    return [float(np.float32(lo + (p / P) * (hi - lo))) for p in range(1, P + 1)]


def reassembly_loss(x, norm_kind, gamma, beta, eps, W, theta, a_bits, w_bits, n_match_tokens=256):
    """Algorithm 1's function ReAssembly(theta) for one linear layer: disassemble with T = ceil(m / theta),
    merge the sum(T - 1) nearest pairs under Eq. (5), quantize reassembled activations and weights, and
    return the squared error of the layer's output against the full-precision norm -> linear.  (The
    paper evaluates Eq. (6) on a whole attention block; one layer has no softmax to go through, so the
    error is taken at the layer's own output.)  Returns (loss, T, src_idx, dst_idx)."""
    y = api.norm(x, norm_kind, gamma, beta, eps)
    absmax = api.channel_absmax(y)
    T = api.num_split(absmax, np.float32(theta))
    r = int((T.astype(np.int64) - 1).sum())
    src_idx, dst_idx = match_pairs_eq5(y, W, T, r, n_match_tokens)
    What = api.reassemble_weight(W, T, src_idx, dst_idx)
    wq = api.quantize_weight(What, w_bits)
    out = api.reassembled_linear(x, norm_kind, gamma, beta, eps, T, src_idx, dst_idx, a_bits, wq, want_acc=False)
    ref = y.astype(np.float64) @ np.asarray(W, np.float64)
    err = out["y"].astype(np.float64) - ref
    return float((err * err).sum()), T, src_idx, dst_idx


def grid_search_theta(x, norm_kind, gamma, beta, eps, W, a_bits, w_bits, P, n_match_tokens=256):
    """Algorithm 1: the theta of the grid with the smallest reassembly error (the first one on ties).
    Returns (theta_star, losses)."""
    y = api.norm(x, norm_kind, gamma, beta, eps)
    thetas = theta_grid(api.channel_absmax(y), P)
    losses = [reassembly_loss(x, norm_kind, gamma, beta, eps, W, t, a_bits, w_bits, n_match_tokens)[0] for t in thetas]
    return thetas[int(np.argmin(losses))], thetas, losses


def build_pruned_map(T, src_idx):
    """The comparison of Sec. 4.1.2 as a map: disassembly (Eq. 3) as in build_map, but the members of set A
    listed in src_idx (A = even positions of the disassembled axis) are dropped instead of merged into a
    member of set B.  Returns (row_ptr, src, scale): one entry per kept position, scale 1/T."""
    T = np.asarray(T, np.int64)
    chan_of = np.repeat(np.arange(T.size), T)
    keep = np.ones(chan_of.size, bool)
    keep[2 * np.asarray(src_idx, np.int64)] = False
    src = chan_of[keep].astype(np.int32)
    scale = (np.float64(1.0) / T[src]).astype(np.float32)
    return np.arange(src.size + 1, dtype=np.int32), src, scale


def map_linear(x, norm_kind, gamma, beta, eps, row_ptr, src, scale, W, a_bits, w_bits):
    """norm -> the map -> per-token quantization (Eq. 2) -> integer GEMM against per-output-channel quantized
    weights -> dequantising epilogue (Eq. 1), for ANY map: a weight row of an output channel is the sum of the
    weight rows of its sources (for one source, that row).  Returns the layer's output [N, O] float32."""
    xhat = api.apply_map(api.norm(x, norm_kind, gamma, beta, eps), row_ptr, src, scale)
    codes, alpha, zero, rowsum = api.quantize_rows(xhat, a_bits)
    W = np.asarray(W, np.float32)
    What = np.empty((row_ptr.size - 1, W.shape[1]), np.float32)
    for ch in range(row_ptr.size - 1):
        acc = W[src[row_ptr[ch]]].copy()
        for e in range(row_ptr[ch] + 1, row_ptr[ch + 1]):
            acc = acc + W[src[e]]                       # float32, entry by entry (Eq. 4: the rows add up)
        What[ch] = acc
    wcodes, aw, bw, cs = api.quantize_weight(What, w_bits)
    return api.epilogue(api.int_gemm(codes, wcodes), codes.shape[1], alpha, zero, rowsum, aw, bw, cs)


def layer_output_errors(x, norm_kind, gamma, beta, eps, W, T, src_idx, dst_idx, a_bits, w_bits):
    """Squared error of the layer's output against the full-precision norm -> linear, for the map that merges the
    listed pairs (Eq. 4) and for the map that drops the same members of set A instead (Sec. 4.1.2's comparison).
    Returns dict(assembly=..., pruning=...)."""
    y = api.norm(x, norm_kind, gamma, beta, eps)
    ref = y.astype(np.float64) @ np.asarray(W, np.float64)
    out = {}
    for name, m in (("assembly", api.build_map(T, src_idx, dst_idx)), ("pruning", build_pruned_map(T, src_idx))):
        err = map_linear(x, norm_kind, gamma, beta, eps, *m, W, a_bits, w_bits).astype(np.float64) - ref
        out[name] = float((err * err).sum())
    return out
