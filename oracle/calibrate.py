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

The edge length here is the plain L2 distance between activation columns over the first
`n_match_tokens` tokens (benchmark policy), not the paper's Eq. (5), which also involves the weights.
"""
import numpy as np

from . import api


def theta_from_rule(absmax, rule):
    kind, val = rule
    m = np.asarray(absmax, np.float32)
    if kind == "fixed":
        return float(np.float32(val))
    if kind == "tmax":
        return float(np.float32(m.max()) / np.float32(val))
    if kind == "expand":
        target = max(1, int(round(val * m.size)))
        lo, hi = 0.0, float(m.max())          # extra(hi) == 0 < target; extra(lo -> 0) -> inf
        lo = hi / 1e6
        for _ in range(200):
            mid = 0.5 * (lo + hi)
            extra = int((api.num_split(m, np.float32(mid)).astype(np.int64) - 1).sum())
            if extra >= target:
                lo = mid
            else:
                hi = mid
            if hi - lo <= 1e-7 * hi:
                break
        return float(np.float32(lo))
    raise ValueError(kind)


def nearest_pairs(y, T, r, n_match_tokens=256, chunk=2048):
    """Bipartite soft matching on the disassembled axis.  Returns (src_idx, dst_idx), int32 [r],
    as indices into set A / set B.  Deterministic: ties go to the lower index."""
    T = np.asarray(T, np.int64)
    if r == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32)
    chan_of = np.repeat(np.arange(T.size), T)           # disassembled position -> source channel
    Cp = chan_of.size
    eligible = T[chan_of] == 1
    pos_a = np.arange(0, Cp, 2)
    pos_b = np.arange(1, Cp, 2)
    pos_a = pos_a[eligible[pos_a]]
    pos_b = pos_b[eligible[pos_b]]
    if pos_a.size == 0 or pos_b.size == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32)
    r = min(r, pos_a.size)                              # tiny layers: merge what can be merged
    ys = np.asarray(y[:n_match_tokens], np.float64)
    cols_a = ys[:, chan_of[pos_a]]                      # [n, |A|]
    cols_b = ys[:, chan_of[pos_b]]                      # [n, |B|]
    nb2 = (cols_b * cols_b).sum(0)
    best_d = np.empty(pos_a.size)
    best_j = np.empty(pos_a.size, np.int64)
    for s in range(0, pos_a.size, chunk):
        a = cols_a[:, s:s + chunk]
        d2 = (a * a).sum(0)[:, None] + nb2[None, :] - 2.0 * (a.T @ cols_b)
        j = d2.argmin(1)
        best_j[s:s + chunk] = j
        best_d[s:s + chunk] = d2[np.arange(j.size), j]
    pick = np.argsort(best_d, kind="stable")[:r]
    pick.sort()
    src_idx = (pos_a[pick] // 2).astype(np.int32)
    dst_idx = ((pos_b[best_j[pick]] - 1) // 2).astype(np.int32)
    return src_idx, dst_idx


def calibrate(y, theta_rule, merge=True, n_match_tokens=256):
    """y: norm output [N, C] float32 (from the oracle).  Returns a dict with absmax, theta, T,
    src_idx, dst_idx.  With merge=True sum(T-1) pairs are merged, so C^ == C (fewer only if set A
    has fewer eligible members than that)."""
    absmax = api.channel_absmax(y)
    theta = theta_from_rule(absmax, theta_rule)
    T = api.num_split(absmax, theta)
    r = int((T.astype(np.int64) - 1).sum()) if merge else 0
    src_idx, dst_idx = nearest_pairs(y, T, r, n_match_tokens)
    return dict(absmax=absmax, theta=theta, T=T, src_idx=src_idx, dst_idx=dst_idx)
