"""Shared case construction for the test-suite: seeded inputs -> oracle-side calibration and
expected values -> (for GPU tests) device-side structs built with the library's own host helpers."""
import numpy as np

from paper_2310_08041_amd import workloads as wl

NORM_ID = {"none": 0, "layer": 1, "rms": 2}


class Case:
    pass


def make_case(oracle, w, N=None, C=None, O=None, seed=None, merge=True, real_weights=True, theta_rule=None,
              assemble_more=0.0):
    """Draws a workload (optionally resized), calibrates it with the oracle and returns a Case with
    inputs (x, gamma, beta), the paper-form map (absmax, theta, T, src_idx, dst_idx), the oracle's
    CSR map and the oracle's weights (one byte per code)."""
    from oracle import calibrate
    c = Case()
    c.w = w
    c.N, c.C, c.O = (w.N if N is None else N), (w.C if C is None else C), (w.O if O is None else O)
    c.norm = NORM_ID[w.norm]
    c.eps = w.eps
    c.x, c.out_ch, c.out_fac = wl.draw_activations(w, c.N, c.C, seed)
    c.gamma, c.beta = wl.draw_norm_params(w, c.C, seed)
    y = oracle.norm(c.x, c.norm, c.gamma, c.beta, c.eps)
    cal = calibrate.calibrate(y, theta_rule or w.theta_rule, merge=merge, assemble_more=assemble_more)
    c.absmax, c.theta, c.T, c.src_idx, c.dst_idx = (cal[k] for k in ("absmax", "theta", "T", "src_idx", "dst_idx"))
    c.row_ptr, c.src, c.scale = oracle.build_map(c.T, c.src_idx, c.dst_idx)
    c.K = c.row_ptr.size - 1
    if real_weights:
        W = wl.draw_weight(w, c.C, c.O, seed)
        c.W = W
        What = oracle.reassemble_weight(W, c.T, c.src_idx, c.dst_idx)
        c.wcodes, c.aw, c.bw, c.cs = oracle.quantize_weight(What, w.w_bits)
    else:
        c.W = None
        c.wcodes, c.aw, c.bw = wl.draw_weight_codes(w, c.K, c.O, seed)
        c.cs = c.wcodes.astype(np.int64).sum(1).astype(np.int32)
    return c


def expected_qact(oracle, c, bits=None):
    """Oracle a1..a4 through the literal two-stage form."""
    return oracle.reassembled_linear(c.x, c.norm, c.gamma, c.beta, c.eps, c.T, c.src_idx, c.dst_idx,
                                     c.w.a_bits if bits is None else bits, None)


def to_torch_x(x, device="cuda"):
    import torch
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(x).to(device)


def rel_err(got, ref):
    """Error relative to max(|ref|, 1e-3 * rms(ref)), so that outputs near zero do not blow it up."""
    ref = ref.astype(np.float64)
    floor = 1e-3 * np.sqrt((ref * ref).mean()) + 1e-30
    return np.abs(got.astype(np.float64) - ref) / np.maximum(np.abs(ref), floor)


def random_csr_map(rng, C_in, C_out, special_every, longest=5):
    """Any CSR map, not only those the paper's reassembly makes: mostly shifted unscaled copies (so that
    plain groups with every misalignment exist), every `special_every`-th row 1..longest entries with arbitrary
    sources (repeats allowed) and arbitrary scales; some inputs are never referenced."""
    row_ptr, src, scale = [0], [], []
    shift = 0
    for ch in range(C_out):
        if ch % special_every == special_every - 1:
            n = int(rng.integers(1, longest + 1))
            src += rng.integers(0, C_in, n).tolist()
            kind = rng.integers(0, 3)
            if kind == 0:
                scale += [1.0] * n                                  # the "sum" convention of a merge
            elif kind == 1:
                scale += [float(np.float32(1.0 / n))] * n
            else:
                scale += rng.uniform(-2.0, 2.0, n).astype(np.float32).tolist()
            shift = int(rng.integers(0, 9))
        else:
            src.append(min(max(ch + shift - 4, 0), C_in - 1))
            scale.append(1.0)
        row_ptr.append(len(src))
    return np.array(row_ptr, np.int32), np.array(src, np.int32), np.array(scale, np.float32)
