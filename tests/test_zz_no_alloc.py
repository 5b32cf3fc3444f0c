"""The entry point that allocates nothing (qllm_reassembled_linear_static) against qllm_reassembled_linear with a
caller's workspace: the same bits, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from helpers import make_case, to_torch_x
from paper_2310_08041_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_static_workspace_entry_point_matches_the_workspace_one(oracle):
    import torch
    from paper_2310_08041_amd import binding as b
    assert torch.cuda.is_available(), "this test needs the MI355X"
    # first a 4-bit shape whose GEMM takes the FP6 path (the activations re-laid into the workspace), then a small-batch
    # 4-bit shape whose GEMM splits K over workgroups (partial accumulators in the workspace), then a smaller
    # decode-sized 6-bit one: stale contents of the shared array must not matter
    for name, N, C, O, y_dtype in [("llama7b_qkv", 300, 4096, 8192, torch.bfloat16), ("llama7b_qkv", 96, 4096, 2048, torch.bfloat16),
                                   ("llama70b_q_decode", 16, 2048, 512, torch.float32)]:
        w = wl.WORKLOADS[name]
        c = make_case(oracle, w, N=N, C=C, O=O)
        r = b.qllm_build_map_host(c.absmax, c.theta, c.src_idx, c.dst_idx)
        dm = b.DeviceMap(r["row_ptr"], r["src"], r["scale"], c.C, r["plan"])
        q = b.qllm_quantize_weight_host(c.W, r["row_ptr"], r["src"], w.w_bits)
        dw = b.DeviceWeight(q["codes"], q["scale"], q["zero"], q["colsum"], c.K, w.w_bits)
        g = torch.from_numpy(c.gamma).cuda()
        x = to_torch_x(c.x)
        need = b.qllm_workspace_bytes(c.N, c.K, c.O, w.a_bits)
        assert 0 < need <= b.STATIC_WORKSPACE_BYTES
        if N == 96:
            assert b.qllm_gemm_workspace_floor_bytes(c.N, c.K, c.O, w.a_bits) > 0      # partial accumulators live there too
        if N == 300:                                                                    # K not split, room for the tiles
            assert b.qllm_gemm_workspace_floor_bytes(c.N, c.K, c.O, w.a_bits) == 0 and dw.tiles6 is not None
            assert need >= b.qllm_workspace_floor_bytes(c.N, c.K, c.O, w.a_bits) + b.qllm_tiles6_bytes(c.N, c.K)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        y_ref = torch.full((c.N, c.O), float("nan"), dtype=y_dtype, device="cuda")
        b.qllm_reassembled_linear(x, c.norm, g, None, c.eps, dm, w.a_bits, dw, y_ref, ws)
        torch.cuda.synchronize()
        y = torch.full((c.N, c.O), float("nan"), dtype=y_dtype, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]                    # allocations so far
        for _ in range(2):
            b.qllm_reassembled_linear_static(x, c.norm, g, None, c.eps, dm, w.a_bits, dw, y)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before              # none through torch either
        assert torch.equal(y.view(torch.int16 if y_dtype == torch.bfloat16 else torch.int32),
                           y_ref.view(torch.int16 if y_dtype == torch.bfloat16 else torch.int32))
        exp = oracle.reassembled_linear(c.x, c.norm, c.gamma, c.beta, c.eps, c.T, c.src_idx, c.dst_idx, w.a_bits,
                                        (c.wcodes, c.aw, c.bw, c.cs))
        got = y.float().cpu().numpy()
        ref = exp["y"] if y_dtype == torch.float32 else oracle.widen_bf16(oracle.round_to_bf16(exp["y"]))
        assert np.array_equal(got, ref)


def test_static_workspace_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2310_08041_amd import binding as b
    # 2048 tokens x 28672 channels at 4 bits need 29 MB for the codes alone plus the parameters: beyond 32 MiB with
    # 8-bit codes; the call must refuse before anything is launched (the pointers are never used)
    N, C, O = 2048, 28672, 64
    assert b.qllm_workspace_bytes(N, C, O, 8) > b.STATIC_WORKSPACE_BYTES
    ident = b.qllm_build_map_host(np.ones(C, np.float32), 2.0, [], [], with_plan=False)
    dm = b.DeviceMap(ident["row_ptr"], ident["src"], ident["scale"], C)
    dw = b.DeviceWeight(np.zeros((O, b.qllm_packed_row_bytes(C, 8)), np.uint8), np.ones(O, np.float32), np.zeros(O, np.int32),
                        np.zeros(O, np.int32), C, 8)
    x = torch.zeros((N, C), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((N, O), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(b.QllmError) as e:
        b.qllm_reassembled_linear_static(x, b.NORM_NONE, None, None, 1e-5, dm, 8, dw, y)
    assert e.value.status == -7
