"""ctypes binding of libqllm.so: the same entry points as include/qllm.h, taking torch tensors.

Argument marshalling only.  torch supplies device memory and the current HIP stream; every step of
the layer runs inside the library's kernels.  Importing this module fails loudly if the library has
not been built (run `python __graft_entry__.py` or `paper_2310_08041_amd/_build.py`).
"""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  -- first: libqllm.so must bind to the HIP runtime torch has already loaded;
#                              two HIP runtimes in one process leave the second without a device

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("QLLM_LIB", os.path.join(_HERE, "libqllm.so"))  # override: a library built elsewhere

F32, BF16 = 0, 1
NORM_NONE, NORM_LAYER, NORM_RMS = 0, 1, 2
MAX_CHANNELS, K_PAD, MAP_GROUP, PLAN_HEAD = 32768, 256, 8, 16
QLLM_ERR_MAP = -5

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python __graft_entry__.py)")
_lib = C.CDLL(LIB_PATH)


class QllmError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        detail = f" [{qllm_last_hip_error()}]" if status == -8 else ""
        super().__init__(f"{where}: {status_string(status)} (status {status}){detail}")


class _Map(C.Structure):
    _fields_ = [("C_in", C.c_int64), ("C_out", C.c_int64), ("nnz", C.c_int64), ("row_ptr", C.c_void_p),
                ("src", C.c_void_p), ("scale", C.c_void_p), ("plan", C.c_void_p), ("plan_head", C.c_int32 * PLAN_HEAD)]


class _Weight(C.Structure):
    _fields_ = [("O", C.c_int64), ("K", C.c_int64), ("bits", C.c_int32), ("codes", C.c_void_p),
                ("scale", C.c_void_p), ("zero", C.c_void_p), ("colsum", C.c_void_p), ("tiles6", C.c_void_p),
                ("tiles8", C.c_void_p)]


class _QAct(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scale", C.c_void_p), ("zero", C.c_void_p), ("rowsum", C.c_void_p)]


_i64, _i32, _vp, _f = C.c_int64, C.c_int32, C.c_void_p, C.c_float
_sigs = {
    "qllm_norm_reassemble_quant": (_i32, [_vp, _i32, _i64, _i64, _i64, _i32, _vp, _vp, _f, C.POINTER(_Map), _i32,
                                          C.POINTER(_QAct), _vp]),
    "qllm_int_gemm": (_i32, [C.POINTER(_QAct), _i32, _i64, C.POINTER(_Weight), _vp, _i32, _i64, _vp, _vp, _i64, _vp]),
    "qllm_reassembled_linear": (_i32, [_vp, _i32, _i64, _i64, _i64, _i32, _vp, _vp, _f, C.POINTER(_Map), _i32,
                                       C.POINTER(_Weight), _vp, _i32, _i64, _vp, _i64, _vp]),
    "qllm_reassembled_linear_static": (_i32, [_vp, _i32, _i64, _i64, _i64, _i32, _vp, _vp, _f, C.POINTER(_Map), _i32,
                                              C.POINTER(_Weight), _vp, _i32, _i64, _vp]),
    "qllm_packed_row_bytes": (_i64, [_i64, _i32]),
    "qllm_gemm_workspace_bytes": (_i64, [_i64, _i64, _i64, _i32]),
    "qllm_workspace_bytes": (_i64, [_i64, _i64, _i64, _i32]),
    "qllm_workspace_floor_bytes": (_i64, [_i64, _i64, _i64, _i32]),
    "qllm_gemm_workspace_floor_bytes": (_i64, [_i64, _i64, _i64, _i32]),
    "qllm_tiles6_bytes": (_i64, [_i64, _i64]),
    "qllm_pack_tiles6": (_i32, [_vp, _i64, _i64, _vp, _vp]),
    "qllm_tiles8_bytes": (_i64, [_i64, _i64]),
    "qllm_pack_tiles8": (_i32, [_vp, _i32, _i64, _i64, _vp, _vp]),
    "qllm_swiglu": (_i32, [_vp, _i64, _vp, _i64, _i64, _i64, _vp, _i64, _vp]),
    "qllm_status_string": (C.c_char_p, [_i32]),
    "qllm_last_hip_error": (C.c_char_p, []),
    "qllm_build_map_host": (_i32, [_vp, _i64, _f, _vp, _vp, _i64, _vp, _vp, _vp, C.POINTER(_i64), C.POINTER(_i64),
                                   _vp]),
    "qllm_build_pruned_map_host": (_i32, [_vp, _i64, _f, _vp, _i64, _vp, _vp, _vp, C.POINTER(_i64), C.POINTER(_i64), _vp]),
    "qllm_plan_map_host": (_i32, [_vp, _vp, _vp, _i64, _i64, _vp, C.POINTER(_i64), C.POINTER(_i64)]),
    "qllm_check_map_host": (_i32, [_vp, _vp, _vp, _i64, _i64, _i64]),
    "qllm_quantize_weight_host": (_i32, [_vp, _i64, _i64, _vp, _vp, _i64, _i32, _vp, _vp, _vp, _vp]),
    "qllm_fold_linear_host": (_i32, [_vp, _vp, _i64, _i64, _vp, _vp, _vp, _i64, _vp, _vp]),
    "qllm_pack_codes_host": (_i32, [_vp, _i64, _i64, _i32, _vp]),
    "qllm_unpack_codes_host": (_i32, [_vp, _i64, _i64, _i32, _vp]),
    "qllm_fused_kernel_choice": (_i32, [C.POINTER(_Map), _i32, _i64, _i64, _i32, _i32, _i32]),
    "qllm_norm_channel_absmax": (_i32, [_vp, _i32, _i64, _i64, _i64, _i32, _vp, _vp, _f, _vp, _vp, _i64, _vp]),
    "qllm_match_workspace_bytes": (_i64, [_i64, _i64]),
    "qllm_match_nearest": (_i32, [_vp, _i64, _i64, _vp, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _i64, _vp]),
    "qllm_select_edges_host": (_i64, [_vp, _i64, _i64, _vp]),
    "qllm_matching_sets_host": (_i32, [_vp, _i64, _vp, _vp, C.POINTER(_i64), _vp, _vp, C.POINTER(_i64)]),
    "qllm_pairs_host": (_i64, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp]),
    "qllm_theta_for_expansion_host": (_i32, [_vp, _i64, _i64, C.POINTER(_f)]),
    "qllm_theta_grid_host": (_i32, [_vp, _i64, _i32, _vp]),
    "qllm_linear_f64": (_i32, [_vp, _i64, _i64, _i64, _vp, _i64, _i64, _vp, _i64, _vp]),
    "qllm_sq_error_workspace_bytes": (_i64, [_i64]),
    "qllm_sq_error": (_i32, [_vp, _i32, _i64, _i64, _i64, _vp, _i64, _vp, _vp, _i64, _vp]),
    "qllm_probe_mfma": (_i32, [_i32, _i32, _vp, _vp]),
    "qllm_probe_mfma_fp6": (_i32, [_i32, _i32, _vp, _vp]),
    "qllm_probe_stream": (_i32, [_vp, _vp, _i64, _i32, _vp]),
}
EXPORTS = tuple(_sigs)
for _name, (_res, _args) in _sigs.items():
    _fn = getattr(_lib, _name)           # AttributeError here = the library misses a declared symbol
    _fn.restype, _fn.argtypes = _res, _args


def status_string(status):
    return _lib.qllm_status_string(int(status)).decode()


qllm_status_string = status_string


def qllm_last_hip_error():
    return _lib.qllm_last_hip_error().decode()


def _chk(rc, where):
    if rc != 0:
        raise QllmError(rc, where)


def _np(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _hp(a):
    return None if a is None else a.ctypes.data


def qllm_packed_row_bytes(K, bits):
    v = _lib.qllm_packed_row_bytes(int(K), int(bits))
    _chk(v if v < 0 else 0, "qllm_packed_row_bytes")
    return v


def qllm_workspace_bytes(N, K, O, a_bits):
    v = _lib.qllm_workspace_bytes(int(N), int(K), int(O), int(a_bits))
    _chk(v if v < 0 else 0, "qllm_workspace_bytes")
    return v


def qllm_workspace_floor_bytes(N, K, O, a_bits):
    v = _lib.qllm_workspace_floor_bytes(int(N), int(K), int(O), int(a_bits))
    _chk(v if v < 0 else 0, "qllm_workspace_floor_bytes")
    return int(v)


def qllm_gemm_workspace_floor_bytes(N, K, O, a_bits):
    v = _lib.qllm_gemm_workspace_floor_bytes(int(N), int(K), int(O), int(a_bits))
    _chk(v if v < 0 else 0, "qllm_gemm_workspace_floor_bytes")
    return int(v)


def qllm_tiles6_bytes(rows, K):
    v = _lib.qllm_tiles6_bytes(int(rows), int(K))
    _chk(v if v < 0 else 0, "qllm_tiles6_bytes")
    return int(v)


def qllm_pack_tiles6(codes, rows, K, tiles, stream=None):
    """codes [rows, packed_row_bytes(K, 4)] uint8, tiles [tiles6_bytes(rows, K)] uint8: device tensors."""
    torch = _torch()
    _check_tensor(codes, "codes", (torch.uint8,), numel=int(rows) * qllm_packed_row_bytes(K, 4))
    _check_tensor(tiles, "tiles", (torch.uint8,), numel=qllm_tiles6_bytes(rows, K))
    _check_on_device(codes=codes, tiles=tiles)
    _chk(_lib.qllm_pack_tiles6(_dp(codes), int(rows), int(K), _dp(tiles), _stream(stream)), "qllm_pack_tiles6")


def qllm_tiles8_bytes(rows, K):
    v = _lib.qllm_tiles8_bytes(int(rows), int(K))
    _chk(v if v < 0 else 0, "qllm_tiles8_bytes")
    return int(v)


def qllm_pack_tiles8(codes, bits, rows, K, tiles, stream=None):
    """codes [rows, packed_row_bytes(K, bits)] uint8, tiles [tiles8_bytes(rows, K)] uint8: device tensors."""
    torch = _torch()
    _check_tensor(codes, "codes", (torch.uint8,), numel=int(rows) * qllm_packed_row_bytes(K, bits))
    _check_tensor(tiles, "tiles", (torch.uint8,), numel=qllm_tiles8_bytes(rows, K))
    _check_on_device(codes=codes, tiles=tiles)
    _chk(_lib.qllm_pack_tiles8(_dp(codes), int(bits), int(rows), int(K), _dp(tiles), _stream(stream)), "qllm_pack_tiles8")


def qllm_gemm_workspace_bytes(N, K, O, a_bits):
    v = _lib.qllm_gemm_workspace_bytes(int(N), int(K), int(O), int(a_bits))
    _chk(v if v < 0 else 0, "qllm_gemm_workspace_bytes")
    return v


# ---------------------------------------------------------------- host helpers (numpy in, numpy out)

def qllm_build_map_host(chan_absmax, theta, src_idx, dst_idx, with_plan=True):
    """Returns dict(row_ptr, src, scale, num_split, C_in, C_out, nnz[, plan]) of numpy arrays (plan None
    if the map cannot have one)."""
    m = _np(chan_absmax, np.float32)
    si, di = _np(src_idx, np.int32), _np(dst_idx, np.int32)
    Cc, r = m.size, si.size
    c_out, nnz = _i64(0), _i64(0)
    T = np.empty(Cc, np.int32)
    _chk(_lib.qllm_build_map_host(_hp(m), Cc, theta, _hp(si), _hp(di), r, None, None, None, C.byref(c_out),
                                  C.byref(nnz), _hp(T)), "qllm_build_map_host(size)")
    row_ptr = np.empty(c_out.value + 1, np.int32)
    src = np.empty(nnz.value, np.int32)
    scale = np.empty(nnz.value, np.float32)
    _chk(_lib.qllm_build_map_host(_hp(m), Cc, theta, _hp(si), _hp(di), r, _hp(row_ptr), _hp(src), _hp(scale),
                                  C.byref(c_out), C.byref(nnz), _hp(T)), "qllm_build_map_host")
    out = dict(row_ptr=row_ptr, src=src, scale=scale, num_split=T, C_in=Cc, C_out=c_out.value, nnz=nnz.value)
    if with_plan:
        try:
            out["plan"] = qllm_plan_map_host(row_ptr, src, scale, Cc)[0]
        except QllmError as e:
            if e.status != QLLM_ERR_MAP:
                raise
            # counts that do not fit the plan's fields: no plan, the fused kernel walks the CSR instead
            out["plan"] = None
    return out


def qllm_build_pruned_map_host(chan_absmax, theta, src_idx, with_plan=True):
    """As qllm_build_map_host, with the members of set A listed in src_idx dropped instead of merged (Sec. 4.1.2)."""
    m = _np(chan_absmax, np.float32)
    si = _np(src_idx, np.int32)
    Cc, r = m.size, si.size
    c_out, nnz = _i64(0), _i64(0)
    T = np.empty(Cc, np.int32)
    _chk(_lib.qllm_build_pruned_map_host(_hp(m), Cc, theta, _hp(si), r, None, None, None, C.byref(c_out), C.byref(nnz),
                                         _hp(T)), "qllm_build_pruned_map_host(size)")
    row_ptr = np.empty(c_out.value + 1, np.int32)
    src = np.empty(nnz.value, np.int32)
    scale = np.empty(nnz.value, np.float32)
    _chk(_lib.qllm_build_pruned_map_host(_hp(m), Cc, theta, _hp(si), r, _hp(row_ptr), _hp(src), _hp(scale),
                                         C.byref(c_out), C.byref(nnz), _hp(T)), "qllm_build_pruned_map_host")
    out = dict(row_ptr=row_ptr, src=src, scale=scale, num_split=T, C_in=Cc, C_out=c_out.value, nnz=nnz.value)
    if with_plan:
        out["plan"] = qllm_plan_map_host(row_ptr, src, scale, Cc)[0]
    return out


def qllm_plan_map_host(row_ptr, src, scale, C_in):
    """Returns (plan int32 array, n_general) for a CSR map."""
    row_ptr, src, scale = _np(row_ptr, np.int32), _np(src, np.int32), _np(scale, np.float32)
    c_out = row_ptr.size - 1
    n, g = _i64(0), _i64(0)
    _chk(_lib.qllm_plan_map_host(_hp(row_ptr), _hp(src), _hp(scale), int(C_in), c_out, None, C.byref(n), C.byref(g)),
         "qllm_plan_map_host(size)")
    plan = np.empty(n.value, np.int32)
    _chk(_lib.qllm_plan_map_host(_hp(row_ptr), _hp(src), _hp(scale), int(C_in), c_out, _hp(plan), C.byref(n),
                                 C.byref(g)), "qllm_plan_map_host")
    return plan, g.value


def qllm_check_map_host(row_ptr, src, scale, C_in):
    row_ptr, src, scale = _np(row_ptr, np.int32), _np(src, np.int32), _np(scale, np.float32)
    return _lib.qllm_check_map_host(_hp(row_ptr), _hp(src), _hp(scale), int(C_in), row_ptr.size - 1, src.size)


def qllm_quantize_weight_host(W, row_ptr, src, bits):
    """W [C_in, O] float32 -> dict(codes [O, row_bytes] u8 packed, scale, zero, colsum, O, K, bits)."""
    W = _np(W, np.float32)
    row_ptr, src = _np(row_ptr, np.int32), _np(src, np.int32)
    c_in, O = W.shape
    K = row_ptr.size - 1
    rb = qllm_packed_row_bytes(K, bits)
    codes = np.empty((O, rb), np.uint8)
    scale = np.empty(O, np.float32)
    zero = np.empty(O, np.int32)
    colsum = np.empty(O, np.int32)
    _chk(_lib.qllm_quantize_weight_host(_hp(W), c_in, O, _hp(row_ptr), _hp(src), K, int(bits), _hp(codes),
                                        _hp(scale), _hp(zero), _hp(colsum)), "qllm_quantize_weight_host")
    return dict(codes=codes, scale=scale, zero=zero, colsum=colsum, O=O, K=K, bits=int(bits))


def qllm_fold_linear_host(Wp, bp, row_ptr, src, scale):
    """Wp [C_in, K_prev] float32 (rows = output channels of the preceding layer), bp [C_in] or None ->
    (W_out [C_out, K_prev], b_out [C_out] or None)."""
    Wp = _np(Wp, np.float32)
    row_ptr, src, scale = _np(row_ptr, np.int32), _np(src, np.int32), _np(scale, np.float32)
    c_in, kp = Wp.shape
    c_out = row_ptr.size - 1
    bp = None if bp is None else _np(bp, np.float32)
    W_out = np.empty((c_out, kp), np.float32)
    b_out = None if bp is None else np.empty(c_out, np.float32)
    _chk(_lib.qllm_fold_linear_host(_hp(Wp), None if bp is None else _hp(bp), c_in, kp, _hp(row_ptr), _hp(src),
                                    _hp(scale), c_out, _hp(W_out), None if bp is None else _hp(b_out)),
         "qllm_fold_linear_host")
    return W_out, b_out


def qllm_pack_codes_host(codes, bits):
    codes = _np(codes, np.uint8)
    R, K = codes.shape
    out = np.empty((R, qllm_packed_row_bytes(K, bits)), np.uint8)
    _chk(_lib.qllm_pack_codes_host(_hp(codes), R, K, int(bits), _hp(out)), "qllm_pack_codes_host")
    return out


def qllm_unpack_codes_host(packed, K, bits):
    packed = _np(packed, np.uint8)
    R = packed.shape[0]
    assert packed.shape[1] == qllm_packed_row_bytes(K, bits)
    out = np.empty((R, K), np.uint8)
    _chk(_lib.qllm_unpack_codes_host(_hp(packed), R, int(K), int(bits), _hp(out)), "qllm_unpack_codes_host")
    return out


# ---------------------------------------------------------------- device side (torch tensors)

def _torch():
    return torch


def _dp(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _x_dtype(x):
    torch = _torch()
    if x.dtype == torch.bfloat16:
        return BF16
    if x.dtype == torch.float32:
        return F32
    raise TypeError(f"activations must be float32 or bfloat16, got {x.dtype}")


class DeviceMap:
    """Device copy of a reassembly map (keeps the tensors alive next to the C struct)."""

    def __init__(self, row_ptr, src, scale, C_in, plan=None, device="cuda"):
        torch = _torch()
        self.row_ptr = torch.as_tensor(np.ascontiguousarray(row_ptr, np.int32)).to(device)
        self.src = torch.as_tensor(np.ascontiguousarray(src, np.int32)).to(device)
        self.scale = torch.as_tensor(np.ascontiguousarray(scale, np.float32)).to(device)
        self.plan = None if plan is None else torch.as_tensor(np.ascontiguousarray(plan, np.int32)).to(device)
        head = (C.c_int32 * PLAN_HEAD)()
        if plan is not None:
            head[:] = [int(v) for v in np.asarray(plan).ravel()[:PLAN_HEAD]]
        self.C_in, self.C_out, self.nnz = int(C_in), int(self.row_ptr.numel() - 1), int(self.src.numel())
        self.c = _Map(self.C_in, self.C_out, self.nnz, _dp(self.row_ptr), _dp(self.src), _dp(self.scale),
                      _dp(self.plan), head)


class DeviceWeight:
    """Device copy of packed per-output-channel quantized weights."""

    def __init__(self, codes, scale, zero, colsum, K, bits, device="cuda", tiles6=True, tiles8=None):
        """tiles6: for 4-bit codes also keep the copy laid out for the FP6 matrix-core path (1.5 x the packed size).
        tiles8: also keep the one-byte-per-code copy that the GEMM of 6- and 8-bit activations reads without
        unpacking (None: for 6- and 8-bit codes; 4-bit weights need it only under 8-bit activations, so say True)."""
        torch = _torch()
        self.codes = torch.as_tensor(np.ascontiguousarray(codes, np.uint8)).to(device)
        self.scale = torch.as_tensor(np.ascontiguousarray(scale, np.float32)).to(device)
        self.zero = torch.as_tensor(np.ascontiguousarray(zero, np.int32)).to(device)
        self.colsum = torch.as_tensor(np.ascontiguousarray(colsum, np.int32)).to(device)
        self.O, self.K, self.bits = int(self.codes.shape[0]), int(K), int(bits)
        assert self.codes.shape[1] == qllm_packed_row_bytes(K, bits)
        self.tiles6 = None
        if tiles6 and self.bits == 4:
            self.tiles6 = torch.empty(qllm_tiles6_bytes(self.O, self.K), dtype=torch.uint8, device=device)
            qllm_pack_tiles6(self.codes, self.O, self.K, self.tiles6)
        self.tiles8 = None
        if tiles8 or (tiles8 is None and self.bits != 4):
            self.tiles8 = torch.empty(qllm_tiles8_bytes(self.O, self.K), dtype=torch.uint8, device=device)
            qllm_pack_tiles8(self.codes, self.bits, self.O, self.K, self.tiles8)
        self.c = _Weight(self.O, self.K, self.bits, _dp(self.codes), _dp(self.scale), _dp(self.zero),
                         _dp(self.colsum), _dp(self.tiles6), _dp(self.tiles8))


class DeviceQAct:
    """Caller-owned buffers for the quantized activations of N tokens."""

    def __init__(self, N, K, bits, device="cuda"):
        torch = _torch()
        self.N, self.K, self.bits = int(N), int(K), int(bits)
        self.codes = torch.empty((N, qllm_packed_row_bytes(K, bits)), dtype=torch.uint8, device=device)
        self.scale = torch.empty(N, dtype=torch.float32, device=device)
        self.zero = torch.empty(N, dtype=torch.int32, device=device)
        self.rowsum = torch.empty(N, dtype=torch.int32, device=device)
        self.c = _QAct(_dp(self.codes), _dp(self.scale), _dp(self.zero), _dp(self.rowsum))


def _need(cond, what):
    """The C ABI cannot see how large a device buffer is: whatever it would trust is checked here first."""
    if not cond:
        raise ValueError("libqllm binding: " + what)


def _check_tensor(t, name, dtypes=None, shape=None, numel=None, optional=False):
    """A device tensor whose rows are dense (stride 1 along the last axis)."""
    if t is None:
        _need(optional, f"{name} is required")
        return
    torch = _torch()
    _need(isinstance(t, torch.Tensor), f"{name} must be a torch tensor")
    if dtypes is not None:
        _need(t.dtype in dtypes, f"{name} has dtype {t.dtype}, expected one of {[str(d) for d in dtypes]}")
    if shape is not None:
        _need(tuple(t.shape) == tuple(shape), f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if numel is not None:
        _need(t.numel() == numel and t.is_contiguous(), f"{name} must hold {numel} contiguous elements, has {t.numel()}")
    _need(t.dim() == 0 or t.numel() == 0 or t.stride(-1) == 1, f"{name} must have stride 1 along its last axis")


def _check_on_device(**tensors):
    """Last of a wrapper's checks, so that shapes and dtypes can be tested without a GPU."""
    for name, t in tensors.items():
        _need(t is None or t.is_cuda, f"{name} must be a device (cuda) tensor")


def _check_activation_args(x, norm, gamma, beta, dmap):
    torch = _torch()
    _need(hasattr(x, "dim") and x.dim() == 2, "x must be a 2-d tensor [tokens, channels]")
    N, Cc = x.shape
    _need(int(norm) in (NORM_NONE, NORM_LAYER, NORM_RMS), f"unknown norm kind {norm}")
    if dmap is not None:
        _need(dmap.C_in == Cc, f"the map takes {dmap.C_in} channels, x has {Cc}")
    if int(norm) != NORM_NONE:
        _check_tensor(gamma, "gamma", (torch.float32,), numel=Cc)
    _check_tensor(beta, "beta", (torch.float32,), numel=Cc, optional=True)
    _check_tensor(x, "x", (torch.float32, torch.bfloat16))
    return N, Cc


def _check_qact(out, N, K, bits, name="out"):
    _need(out.N >= N, f"{name} holds {out.N} tokens, {N} needed")
    _need(out.K == K, f"{name} was made for {out.K} channels, the map makes {K}")
    _need(out.bits == int(bits), f"{name} was made for {out.bits}-bit codes, {bits} asked for")


def _check_output(y, N, O, name="y"):
    torch = _torch()
    _check_tensor(y, name, (torch.float32, torch.bfloat16), shape=(N, O))


def qllm_norm_reassemble_quant(x, norm, gamma, beta, eps, dmap, bits, out, stream=None):
    N, Cc = _check_activation_args(x, norm, gamma, beta, dmap)
    _check_qact(out, N, dmap.C_out, bits)
    _check_on_device(x=x, gamma=gamma, beta=beta)
    _chk(_lib.qllm_norm_reassemble_quant(_dp(x), _x_dtype(x), N, Cc, x.stride(0), int(norm), _dp(gamma), _dp(beta),
                                         float(eps), C.byref(dmap.c), int(bits), C.byref(out.c), _stream(stream)),
         "qllm_norm_reassemble_quant")
    return out


FUSED_WALKS_MAP, FUSED_LISTS_IN_LDS, FUSED_LISTS_STREAMED = 0, 1, 2


def qllm_fused_kernel_choice(dmap, x_dtype, N, ldx, norm, has_beta, bits):
    """FUSED_* : the form of the fused kernel qllm_norm_reassemble_quant runs for this map and these arguments.
    x_dtype: F32 / BF16 (or a torch dtype)."""
    if not isinstance(x_dtype, int):
        x_dtype = BF16 if "bfloat16" in str(x_dtype) else F32
    rc = _lib.qllm_fused_kernel_choice(C.byref(dmap.c), int(x_dtype), int(N), int(ldx), int(norm), int(bool(has_beta)), int(bits))
    if rc < 0:
        raise QllmError(rc, "qllm_fused_kernel_choice")
    return rc


def qllm_int_gemm(a, weight, y, acc_dump=None, workspace=None, stream=None):
    torch = _torch()
    _need(a.K == weight.K, f"activations have {a.K} channels, weights {weight.K}")
    _check_output(y, a.N, weight.O)
    _check_tensor(acc_dump, "acc_dump", (torch.int32,), numel=a.N * weight.O, optional=True)
    _check_tensor(workspace, "workspace", (torch.uint8,), optional=True)
    _check_on_device(y=y, acc_dump=acc_dump, workspace=workspace)
    _chk(_lib.qllm_int_gemm(C.byref(a.c), a.bits, a.N, C.byref(weight.c), _dp(y), _x_dtype(y), y.stride(0),
                            _dp(acc_dump), _dp(workspace), 0 if workspace is None else workspace.numel(),
                            _stream(stream)), "qllm_int_gemm")
    return y


def qllm_reassembled_linear(x, norm, gamma, beta, eps, dmap, a_bits, weight, y, workspace, stream=None):
    N, Cc = _check_activation_args(x, norm, gamma, beta, dmap)
    _need(dmap.C_out == weight.K, f"the map makes {dmap.C_out} channels, the weights take {weight.K}")
    _check_output(y, N, weight.O)
    _check_tensor(workspace, "workspace", (_torch().uint8,))
    _check_on_device(y=y, workspace=workspace, x=x, gamma=gamma, beta=beta)
    _chk(_lib.qllm_reassembled_linear(_dp(x), _x_dtype(x), N, Cc, x.stride(0), int(norm), _dp(gamma), _dp(beta),
                                      float(eps), C.byref(dmap.c), int(a_bits), C.byref(weight.c), _dp(y),
                                      _x_dtype(y), y.stride(0), _dp(workspace), workspace.numel(), _stream(stream)),
         "qllm_reassembled_linear")
    return y


STATIC_WORKSPACE_BYTES = 32 << 20


def qllm_reassembled_linear_static(x, norm, gamma, beta, eps, dmap, a_bits, weight, y, stream=None):
    """The layer with the library's built-in workspace: allocates nothing."""
    N, Cc = _check_activation_args(x, norm, gamma, beta, dmap)
    _need(dmap.C_out == weight.K, f"the map makes {dmap.C_out} channels, the weights take {weight.K}")
    _check_output(y, N, weight.O)
    _check_on_device(y=y, x=x, gamma=gamma, beta=beta)
    _chk(_lib.qllm_reassembled_linear_static(_dp(x), _x_dtype(x), N, Cc, x.stride(0), int(norm), _dp(gamma), _dp(beta),
                                             float(eps), C.byref(dmap.c), int(a_bits), C.byref(weight.c), _dp(y),
                                             _x_dtype(y), y.stride(0), _stream(stream)), "qllm_reassembled_linear_static")
    return y


def qllm_norm_channel_absmax(x, norm, gamma, beta, eps, absmax, y_dump=None, stream=None):
    torch = _torch()
    N, Cc = _check_activation_args(x, norm, gamma, beta, None)
    _check_tensor(absmax, "absmax", (torch.float32,), numel=Cc)
    if y_dump is not None:
        _need(y_dump.dim() == 2 and y_dump.shape[1] == Cc and y_dump.shape[0] <= N and y_dump.is_contiguous(),
              f"y_dump must be a contiguous [at most {N}, {Cc}] tensor, is {tuple(y_dump.shape)}")
        _check_tensor(y_dump, "y_dump", (torch.float32,))
    _check_on_device(absmax=absmax, y_dump=y_dump, x=x, gamma=gamma, beta=beta)
    n_dump = 0 if y_dump is None else y_dump.shape[0]
    _chk(_lib.qllm_norm_channel_absmax(_dp(x), _x_dtype(x), N, Cc, x.stride(0), int(norm), _dp(gamma), _dp(beta),
                                       float(eps), _dp(absmax), _dp(y_dump), n_dump, _stream(stream)),
         "qllm_norm_channel_absmax")
    return absmax


def qllm_match_workspace_bytes(nA, nB):
    return int(_lib.qllm_match_workspace_bytes(int(nA), int(nB)))


def qllm_match_nearest(y, W, chan_a, chan_b, best_j, best_d, workspace, stream=None):
    """y [n, C] fp32, W [C, O] fp32 or None (plain L2 on the activations), chan_a / chan_b int32, best_j [nA] int32,
    best_d [nA] float64: device tensors."""
    torch = _torch()
    _need(hasattr(y, "dim") and y.dim() == 2, "y must be a 2-d tensor [tokens, channels]")
    n, Cc = y.shape
    if W is not None:
        _need(W.dim() == 2 and W.shape[0] == Cc, f"W must have one row per channel of y ({Cc}), has shape {tuple(W.shape)}")
    _check_tensor(W, "W", (torch.float32,), optional=True)
    _check_tensor(y, "y", (torch.float32,))
    _check_tensor(chan_a, "chan_a", (torch.int32,), numel=chan_a.numel())
    _check_tensor(chan_b, "chan_b", (torch.int32,), numel=chan_b.numel())
    _check_tensor(best_j, "best_j", (torch.int32,), numel=chan_a.numel())
    _check_tensor(best_d, "best_d", (torch.float64,), numel=chan_a.numel())
    _check_tensor(workspace, "workspace", (torch.uint8,), optional=True)
    _check_on_device(y=y, W=W, chan_a=chan_a, chan_b=chan_b, best_j=best_j, best_d=best_d, workspace=workspace)
    O, ldw = (0, 0) if W is None else (W.shape[1], W.stride(0))
    _chk(_lib.qllm_match_nearest(_dp(y), n, y.stride(0), _dp(W), Cc, O, ldw, _dp(chan_a),
                                 chan_a.numel(), _dp(chan_b), chan_b.numel(), _dp(best_j), _dp(best_d),
                                 _dp(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
                                 _stream(stream)), "qllm_match_nearest")
    return best_j, best_d


def qllm_select_edges_host(best_d, r):
    """best_d [nA] float64 (host) -> the min(r, nA) members of A with the shortest edges, ascending."""
    best_d = _np(best_d, np.float64)
    pick = np.empty(min(int(r), best_d.size), np.int32)
    n = int(_lib.qllm_select_edges_host(_hp(best_d), best_d.size, int(r), _hp(pick)))
    if n < 0:
        _chk(n, "qllm_select_edges_host")
    return pick[:n]


def qllm_matching_sets_host(num_split):
    """num_split [C] int32 (host) -> dict(chan_a, pos_a, chan_b, pos_b) of int32 arrays: Appendix A step 1."""
    T = _np(num_split, np.int32)
    out = [np.empty(T.size, np.int32) for _ in range(4)]
    nA, nB = _i64(0), _i64(0)
    _chk(_lib.qllm_matching_sets_host(_hp(T), T.size, _hp(out[0]), _hp(out[1]), C.byref(nA), _hp(out[2]), _hp(out[3]),
                                      C.byref(nB)), "qllm_matching_sets_host")
    return dict(chan_a=out[0][:nA.value].copy(), pos_a=out[1][:nA.value].copy(), chan_b=out[2][:nB.value].copy(),
                pos_b=out[3][:nB.value].copy())


def qllm_pairs_host(best_d, best_j, pos_a, pos_b, r):
    """Appendix A step 3: (src_idx, dst_idx) int32 arrays of the min(r, |A|) shortest edges."""
    best_d, best_j = _np(best_d, np.float64), _np(best_j, np.int32)
    pos_a, pos_b = _np(pos_a, np.int32), _np(pos_b, np.int32)
    n_max = min(int(r), pos_a.size)
    src_idx, dst_idx = np.empty(max(n_max, 1), np.int32), np.empty(max(n_max, 1), np.int32)
    n = int(_lib.qllm_pairs_host(_hp(best_d), _hp(best_j), _hp(pos_a), _hp(pos_b), pos_a.size, pos_b.size, int(r),
                                 _hp(src_idx), _hp(dst_idx)))
    if n < 0:
        _chk(n, "qllm_pairs_host")
    return src_idx[:n].copy(), dst_idx[:n].copy()


def qllm_theta_for_expansion_host(chan_absmax, extra_target):
    m = _np(chan_absmax, np.float32)
    theta = _f(0.0)
    _chk(_lib.qllm_theta_for_expansion_host(_hp(m), m.size, int(extra_target), C.byref(theta)), "qllm_theta_for_expansion_host")
    return float(theta.value)


def qllm_theta_grid_host(chan_absmax, P):
    m = _np(chan_absmax, np.float32)
    out = np.empty(int(P), np.float32)
    _chk(_lib.qllm_theta_grid_host(_hp(m), m.size, int(P), _hp(out)), "qllm_theta_grid_host")
    return [float(v) for v in out]


def qllm_linear_f64(y, W, out, stream=None):
    """y [N, C] fp32, W [C, O] fp32, out [N, O] float64: device tensors."""
    assert y.is_cuda and W.is_cuda and out.is_cuda and y.dtype == W.dtype == torch.float32 and out.dtype == torch.float64
    assert y.shape[1] == W.shape[0] and out.shape == (y.shape[0], W.shape[1])
    assert y.stride(1) == 1 and W.stride(1) == 1 and out.stride(1) == 1
    _chk(_lib.qllm_linear_f64(_dp(y), y.shape[0], y.shape[1], y.stride(0), _dp(W), W.shape[1], W.stride(0), _dp(out),
                              out.stride(0), _stream(stream)), "qllm_linear_f64")
    return out


def qllm_sq_error_workspace_bytes(N):
    return int(_lib.qllm_sq_error_workspace_bytes(int(N)))


def qllm_sq_error(got, ref, result, workspace, stream=None):
    """got [N, O] fp32 / bf16, ref [N, O] float64, result [1] float64, workspace uint8: device tensors."""
    assert got.is_cuda and ref.is_cuda and result.is_cuda and ref.dtype == result.dtype == torch.float64
    assert got.shape == ref.shape and got.stride(1) == 1 and ref.stride(1) == 1 and result.numel() >= 1
    _chk(_lib.qllm_sq_error(_dp(got), _x_dtype(got), got.shape[0], got.shape[1], got.stride(0), _dp(ref), ref.stride(0),
                            _dp(result), _dp(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
         "qllm_sq_error")
    return result


def qllm_swiglu(gate, up, x, stream=None):
    """x = silu(gate) * up; gate, up, x: [N, C] bfloat16 device tensors (rows may be strided)."""
    torch = _torch()
    _check_tensor(gate, "gate", (torch.bfloat16,))
    _need(gate.dim() == 2, "gate must be [N, C]")
    _check_tensor(up, "up", (torch.bfloat16,), shape=tuple(gate.shape))
    _check_tensor(x, "x", (torch.bfloat16,), shape=tuple(gate.shape))
    _check_on_device(gate=gate, up=up, x=x)
    N, Cc = gate.shape
    ld = lambda t: t.stride(0) if N > 1 else Cc          # the stride of a single row says nothing
    _chk(_lib.qllm_swiglu(_dp(gate), ld(gate), _dp(up), ld(up), int(N), int(Cc), _dp(x), ld(x), _stream(stream)), "qllm_swiglu")
    return x


def qllm_probe_mfma(workgroups, iters, sink, stream=None):
    _chk(_lib.qllm_probe_mfma(int(workgroups), int(iters), _dp(sink), _stream(stream)), "qllm_probe_mfma")


def qllm_probe_mfma_fp6(workgroups, iters, sink, stream=None):
    _chk(_lib.qllm_probe_mfma_fp6(int(workgroups), int(iters), _dp(sink), _stream(stream)), "qllm_probe_mfma_fp6")


def qllm_probe_stream(src, dst, workgroups, stream=None):
    _chk(_lib.qllm_probe_stream(_dp(src), _dp(dst), src.numel() * src.element_size(), int(workgroups), _stream(stream)),
         "qllm_probe_stream")


def raw():
    """The ctypes library handle, for tests that pass deliberately bad arguments."""
    return _lib
