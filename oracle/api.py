"""numpy-facing wrappers over oracle/liboracle.so (ctypes).  TEST INFRASTRUCTURE ONLY.

Every function takes and returns host numpy arrays.  The wrappers of the hot path do no arithmetic of
their own: each sizes the outputs, calls one C routine of qllm_oracle.c and raises on a non-zero status.
The one exception is `fold_preceding_linear` (Appendix B, an offline weight rewrite), which is written
out here in numpy float64.
"""
import ctypes as C
import os

import numpy as np

from .build import LIB, build_oracle

F32, BF16 = 0, 1
NORM_NONE, NORM_LAYER, NORM_RMS = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build_oracle()
        _lib = C.CDLL(LIB)
        _lib.oracle_assembled_count.restype = C.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(rc, name):
    if rc != 0:
        raise ValueError(f"{name} failed with status {rc}")


def _i64(v):
    return C.c_int64(int(v))


def _c(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def round_to_bf16(x):
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    _chk(lib().oracle_round_to_bf16(_p(x), _i64(x.size), _p(out)), "round_to_bf16")
    return out


def widen_bf16(h):
    h = _c(h, np.uint16)
    out = np.empty(h.shape, np.float32)
    _chk(lib().oracle_widen_bf16(_p(h), _i64(h.size), _p(out)), "widen_bf16")
    return out


def norm(x, norm_kind, gamma=None, beta=None, eps=1e-5):
    """x: [N, C] float32, or uint16 holding bfloat16 bits.  Returns y [N, C] float32."""
    assert x.ndim == 2 and x.flags.c_contiguous
    dt = BF16 if x.dtype == np.uint16 else F32
    if dt == F32:
        assert x.dtype == np.float32
    N, Cc = x.shape
    gamma, beta = _c(gamma, np.float32), _c(beta, np.float32)
    y = np.empty((N, Cc), np.float32)
    _chk(lib().oracle_norm(_p(x), dt, _i64(N), _i64(Cc), _i64(Cc), int(norm_kind), _p(gamma), _p(beta),
                           C.c_float(eps), _p(y)), "norm")
    return y


def channel_absmax(y):
    y = _c(y, np.float32)
    out = np.empty(y.shape[1], np.float32)
    _chk(lib().oracle_channel_absmax(_p(y), _i64(y.shape[0]), _i64(y.shape[1]), _p(out)), "channel_absmax")
    return out


def num_split(absmax, theta):
    absmax = _c(absmax, np.float32)
    T = np.empty(absmax.shape[0], np.int32)
    _chk(lib().oracle_num_split(_p(absmax), _i64(absmax.size), C.c_float(theta), _p(T)), "num_split")
    return T


def disassemble(y, T):
    y, T = _c(y, np.float32), _c(T, np.int32)
    N, Cc = y.shape
    Cp = int(T.astype(np.int64).sum())
    d = np.empty((N, Cp), np.float32)
    _chk(lib().oracle_disassemble(_p(y), _i64(N), _i64(Cc), _p(T), _p(d), _i64(Cp)), "disassemble")
    return d


def assemble(d, src_idx, dst_idx, return_keep=False):
    d = _c(d, np.float32)
    src_idx, dst_idx = _c(src_idx, np.int32), _c(dst_idx, np.int32)
    N, Cp = d.shape
    r = src_idx.size
    Chat = Cp - r
    out = np.empty((N, Chat), np.float32)
    keep = np.empty(Chat, np.int32)
    _chk(lib().oracle_assemble(_p(d), _i64(N), _i64(Cp), _p(src_idx), _p(dst_idx), _i64(r), _p(out),
                               _i64(Chat), _p(keep)), "assemble")
    return (out, keep) if return_keep else out


def build_map(T, src_idx, dst_idx):
    """Returns (row_ptr [Chat+1] i32, src [nnz] i32, scale [nnz] f32)."""
    T = _c(T, np.int32)
    src_idx, dst_idx = _c(src_idx, np.int32), _c(dst_idx, np.int32)
    r = src_idx.size
    Cp = int(T.astype(np.int64).sum())
    Chat = Cp - r
    row_ptr = np.empty(Chat + 1, np.int32)
    src = np.empty(Cp, np.int32)
    scale = np.empty(Cp, np.float32)
    co, nz = C.c_int64(0), C.c_int64(0)
    _chk(lib().oracle_build_map(_p(T), _i64(T.size), _p(src_idx), _p(dst_idx), _i64(r), _p(row_ptr), _p(src),
                                _p(scale), C.byref(co), C.byref(nz)), "build_map")
    assert co.value == Chat and nz.value == Cp
    return row_ptr, src, scale


def apply_map(y, row_ptr, src, scale):
    y = _c(y, np.float32)
    row_ptr, src, scale = _c(row_ptr, np.int32), _c(src, np.int32), _c(scale, np.float32)
    N, Cc = y.shape
    Chat = row_ptr.size - 1
    out = np.empty((N, Chat), np.float32)
    _chk(lib().oracle_apply_map(_p(y), _i64(N), _i64(Cc), _p(row_ptr), _p(src), _p(scale), _i64(Chat),
                                _p(out)), "apply_map")
    return out


def quantize_rows(x, bits):
    """Returns (codes [N,K] u8, alpha [N] f32, beta [N] i32, rowsum [N] i32)."""
    x = _c(x, np.float32)
    N, K = x.shape
    codes = np.empty((N, K), np.uint8)
    alpha = np.empty(N, np.float32)
    beta = np.empty(N, np.int32)
    rowsum = np.empty(N, np.int32)
    _chk(lib().oracle_quantize_rows(_p(x), _i64(N), _i64(K), _i64(K), int(bits), _p(codes), _p(alpha), _p(beta),
                                    _p(rowsum)), "quantize_rows")
    return codes, alpha, beta, rowsum


def quantize_weight(What, bits):
    """What: [K, O] (paper layout).  Returns (wcodes [O,K] u8, alpha_w, beta_w, colsum) each [O]."""
    What = _c(What, np.float32)
    K, O = What.shape
    wcodes = np.empty((O, K), np.uint8)
    alpha = np.empty(O, np.float32)
    beta = np.empty(O, np.int32)
    colsum = np.empty(O, np.int32)
    _chk(lib().oracle_quantize_weight(_p(What), _i64(K), _i64(O), int(bits), _p(wcodes), _p(alpha), _p(beta),
                                      _p(colsum)), "quantize_weight")
    return wcodes, alpha, beta, colsum


def packed_row_bytes(K, bits, align=16):
    raw = (K * bits + 7) // 8
    return (raw + align - 1) // align * align


def pack_codes(codes, bits, row_bytes=None):
    codes = _c(codes, np.uint8)
    R, K = codes.shape
    row_bytes = packed_row_bytes(K, bits) if row_bytes is None else row_bytes
    out = np.empty((R, row_bytes), np.uint8)
    _chk(lib().oracle_pack_codes(_p(codes), _i64(R), _i64(K), int(bits), _p(out), _i64(row_bytes)), "pack_codes")
    return out


def unpack_codes(packed, K, bits):
    packed = _c(packed, np.uint8)
    R, row_bytes = packed.shape
    out = np.empty((R, K), np.uint8)
    _chk(lib().oracle_unpack_codes(_p(packed), _i64(R), _i64(K), int(bits), _i64(row_bytes), _p(out)),
         "unpack_codes")
    return out


def reassemble_weight(W, T, src_idx, dst_idx):
    """W: [C, O] float32.  Returns What [Chat, O]."""
    W, T = _c(W, np.float32), _c(T, np.int32)
    src_idx, dst_idx = _c(src_idx, np.int32), _c(dst_idx, np.int32)
    Cc, O = W.shape
    r = src_idx.size
    Chat = int(T.astype(np.int64).sum()) - r
    out = np.empty((Chat, O), np.float32)
    _chk(lib().oracle_reassemble_weight(_p(W), _i64(Cc), _i64(O), _p(T), _p(src_idx), _p(dst_idx), _i64(r),
                                        _p(out), _i64(Chat)), "reassemble_weight")
    return out


def fold_preceding_linear(Wp, bp, T, src_idx, dst_idx):
    """Appendix B in float64: the reassembly moved into the preceding linear layer y = x Wp^T + bp.
    Wp: [C, K_prev] (row c = output channel c of that layer), bp: [C] or None.
    Disassembly: channel c becomes T_c rows Wp[c] / T_c (bias likewise).  Assembly: on the disassembled
    axis, set A = even and set B = odd positions; the A-members src_idx[k] merged into B-member j are
    replaced, together with j, by their mean (for one pair the appendix's (W_i + W_j) / 2); merged
    A-members disappear; the rest keeps its order.  Returns (W^ [C^, K_prev], b^ [C^] or None)."""
    Wp = np.asarray(Wp, np.float64)
    T = np.asarray(T, np.int64)
    src_idx, dst_idx = np.asarray(src_idx, np.int64), np.asarray(dst_idx, np.int64)
    full = Wp if bp is None else np.concatenate([Wp, np.asarray(bp, np.float64)[:, None]], axis=1)
    d = np.repeat(full / T[:, None], T, axis=0)                 # disassembled rows
    total = d.copy()
    count = np.ones(d.shape[0], np.int64)
    gone = np.zeros(d.shape[0], bool)
    for a, j in zip(2 * src_idx, 2 * dst_idx + 1):              # positions on the disassembled axis
        total[j] += d[a]
        count[j] += 1
        gone[a] = True
    out = (total / count[:, None])[~gone]
    return (out, None) if bp is None else (out[:, :-1], out[:, -1])


def int_gemm(a, w):
    """a: [N,K] u8 codes, w: [O,K] u8 codes.  Returns acc [N,O] int32."""
    a, w = _c(a, np.uint8), _c(w, np.uint8)
    N, K = a.shape
    O = w.shape[0]
    assert w.shape[1] == K
    acc = np.empty((N, O), np.int32)
    _chk(lib().oracle_int_gemm(_p(a), _p(w), _i64(N), _i64(K), _i64(O), _p(acc)), "int_gemm")
    return acc


def epilogue(acc, K, alpha_x, beta_x, rowsum_x, alpha_w, beta_w, colsum_w):
    acc = _c(acc, np.int32)
    N, O = acc.shape
    y = np.empty((N, O), np.float32)
    _chk(lib().oracle_epilogue(_p(acc), _i64(N), _i64(O), _i64(K), _p(_c(alpha_x, np.float32)),
                               _p(_c(beta_x, np.int32)), _p(_c(rowsum_x, np.int32)),
                               _p(_c(alpha_w, np.float32)), _p(_c(beta_w, np.int32)),
                               _p(_c(colsum_w, np.int32)), _p(y)), "epilogue")
    return y


def dequant_linear_direct(a, w, alpha_x, beta_x, alpha_w, beta_w):
    a, w = _c(a, np.uint8), _c(w, np.uint8)
    N, K = a.shape
    O = w.shape[0]
    y = np.empty((N, O), np.float32)
    _chk(lib().oracle_dequant_linear_direct(_p(a), _p(w), _i64(N), _i64(K), _i64(O),
                                            _p(_c(alpha_x, np.float32)), _p(_c(beta_x, np.int32)),
                                            _p(_c(alpha_w, np.float32)), _p(_c(beta_w, np.int32)), _p(y)),
         "dequant_linear_direct")
    return y


def reassembled_linear(x, norm_kind, gamma, beta, eps, T, src_idx, dst_idx, a_bits, wq=None, want_acc=True,
                       want_y=True):
    """The whole path.  wq = (wcodes [O,Chat] u8, alpha_w, beta_w, colsum) or None (stop after a4).
    Returns dict(codes, alpha, beta, rowsum[, acc][, y])."""
    assert x.ndim == 2 and x.flags.c_contiguous
    dt = BF16 if x.dtype == np.uint16 else F32
    N, Cc = x.shape
    T = _c(T, np.int32)
    src_idx, dst_idx = _c(src_idx, np.int32), _c(dst_idx, np.int32)
    r = src_idx.size
    Chat = int(T.astype(np.int64).sum()) - r
    gamma, beta = _c(gamma, np.float32), _c(beta, np.float32)
    out = dict(codes=np.empty((N, Chat), np.uint8), alpha=np.empty(N, np.float32), beta=np.empty(N, np.int32),
               rowsum=np.empty(N, np.int32))
    wcodes = aw = bw = cs = None
    O = 0
    if wq is not None:
        wcodes, aw, bw, cs = (_c(wq[0], np.uint8), _c(wq[1], np.float32), _c(wq[2], np.int32),
                              _c(wq[3], np.int32))
        O = wcodes.shape[0]
        assert wcodes.shape[1] == Chat
        if want_acc:
            out["acc"] = np.empty((N, O), np.int32)
        if want_y:
            out["y"] = np.empty((N, O), np.float32)
    _chk(lib().oracle_reassembled_linear(
        _p(x), dt, _i64(N), _i64(Cc), _i64(Cc), int(norm_kind), _p(gamma), _p(beta), C.c_float(eps), _p(T),
        _p(src_idx), _p(dst_idx), _i64(r), int(a_bits), _p(wcodes), _p(aw), _p(bw), _p(cs), _i64(O),
        _p(out["codes"]), _p(out["alpha"]), _p(out["beta"]), _p(out["rowsum"]), _p(out.get("acc")),
        _p(out.get("y"))), "reassembled_linear")
    return out


def nearest_member(y, W, chan_a, chan_b):
    """For every member of set A (its channel in chan_a) the nearest member of set B: plain squared L2 distance
    between the activation columns of y [n, C] (W None), or the distance of Eq. (5) with the weights W [C, O].
    Explicit differences in double; lowest index on ties.  Returns (best_j int64 [nA], best_d float64 [nA])."""
    y = _c(y, np.float32)
    W = _c(W, np.float32)
    chan_a, chan_b = _c(chan_a, np.int32), _c(chan_b, np.int32)
    best_j = np.empty(chan_a.size, np.int64)
    best_d = np.empty(chan_a.size, np.float64)
    O, ldw = (0, 0) if W is None else (W.shape[1], W.shape[1])
    _chk(lib().oracle_nearest_member(_p(y), _i64(y.shape[0]), _i64(y.shape[1]), _p(W), _i64(O), _i64(ldw), _p(chan_a),
                                     _i64(chan_a.size), _p(chan_b), _i64(chan_b.size), _p(best_j), _p(best_d)),
         "nearest_member")
    return best_j, best_d


def swiglu(gate, up, want_f32=False):
    """x = silu(gate) * up for bfloat16 bit patterns gate, up [N, C] (uint16): bfloat16 bits, and on request the fp32
    values before the last rounding."""
    gate, up = _c(gate, np.uint16), _c(up, np.uint16)
    N, Cc = gate.shape
    x = np.empty((N, Cc), np.uint16)
    f = np.empty((N, Cc), np.float32) if want_f32 else None
    _chk(lib().oracle_swiglu(_p(gate), _i64(Cc), _p(up), _i64(Cc), _i64(N), _i64(Cc), _p(x), _i64(Cc), _p(f)), "swiglu")
    return (x, f) if want_f32 else x


def max_threads():
    return int(lib().oracle_max_threads())
