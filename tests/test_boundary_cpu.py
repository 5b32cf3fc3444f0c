"""The C-ABI library without a GPU: exported symbols, argument validation (every check happens
before a launch), and the host helpers against the oracle."""
import ctypes as C
import types
import json
import os
import re

import numpy as np
import pytest

from helpers import make_case, random_csr_map
from paper_2310_08041_amd import binding as b
from paper_2310_08041_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(qllm_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 14
    lib = C.CDLL(b.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(b.EXPORTS) == names      # the binding wraps exactly what the header declares


def test_status_strings():
    assert b.status_string(0) == "ok"
    seen = {b.status_string(s) for s in range(-8, 1)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert b.status_string(-99) == "unknown status"


def test_packed_row_bytes_and_workspace():
    assert b.qllm_packed_row_bytes(28672, 4) == 14336
    assert b.qllm_packed_row_bytes(1, 4) == 128 and b.qllm_packed_row_bytes(257, 6) == 384
    assert b.qllm_packed_row_bytes(256, 8) == 256
    with pytest.raises(b.QllmError):
        b.qllm_packed_row_bytes(16, 5)
    with pytest.raises(b.QllmError):
        b.qllm_packed_row_bytes(0, 4)
    ws = b.qllm_workspace_bytes(2048, 28672, 8192, 4)
    assert ws >= 2048 * 14336 + 3 * 2048 * 4 and ws % 256 == 0
    # the GEMM must have scratch only where it splits K over workgroups: 4-bit codes, few tiles, a long K
    floor = b.qllm_gemm_workspace_floor_bytes
    assert floor(2048, 28672, 8192, 4) == 0 and floor(16, 8192, 8192, 4) == 0
    assert floor(128, 8192, 8192, 4) == 4 * 128 * 8192 * 4
    assert floor(128, 8192, 8192, 6) == 0 and floor(128, 512, 8192, 4) == 0
    assert b.qllm_workspace_bytes(128, 8192, 8192, 4) >= 128 * 4096 + 4 * 128 * 8192 * 4
    # what serves every path: for 4-bit codes and more than 32 tokens the parts' accumulators where K is split, then
    # room for the activations in the FP6 path's layout (1536 bytes per 16 rows and 128 codes of the padded row)
    assert b.qllm_gemm_workspace_bytes(128, 8192, 8192, 4) == floor(128, 8192, 8192, 4) + b.qllm_tiles6_bytes(128, 8192)
    assert b.qllm_tiles6_bytes(2048, 28672) == 2048 // 16 * (28672 // 128) * 1536
    assert b.qllm_tiles6_bytes(17, 100) == 2 * 2 * 1536                     # rows up to 32, K up to 256
    assert b.qllm_gemm_workspace_bytes(2048, 28672, 8192, 4) == b.qllm_tiles6_bytes(2048, 28672)
    assert b.qllm_gemm_workspace_bytes(16, 8192, 8192, 4) == 0 and b.qllm_gemm_workspace_bytes(16, 8192, 8192, 6) == 0
    # the byte-operand path of 6- and 8-bit activations: one byte per code, rows in blocks of 16, K in tiles of 64
    assert b.qllm_tiles8_bytes(2048, 28672) == 2048 * 28672 and b.qllm_tiles8_bytes(17, 100) == 2 * 2 * 1024
    assert b.qllm_gemm_workspace_bytes(2048, 8192, 8192, 6) == b.qllm_tiles8_bytes(2048, 8192)
    assert b.qllm_gemm_workspace_bytes(40, 100, 8192, 8) == b.qllm_tiles8_bytes(40, 100)
    assert b.qllm_workspace_bytes(2048, 8192, 8192, 6) == b.qllm_workspace_floor_bytes(2048, 8192, 8192, 6) + b.qllm_tiles8_bytes(2048, 8192)
    assert b.qllm_workspace_bytes(2048, 28672, 8192, 4) == b.qllm_workspace_floor_bytes(2048, 28672, 8192, 4) + b.qllm_tiles6_bytes(2048, 28672)
    assert b.qllm_workspace_floor_bytes(2048, 28672, 8192, 4) == 2048 * 14336 + 3 * 2048 * 4


def _structs():
    m = b._Map(64, 64, 64, 0x1000, 0x1000, 0x1000, None)
    q = b._QAct(0x1000, 0x1000, 0x1000, 0x1000)
    w = b._Weight(32, 64, 4, 0x1000, 0x1000, 0x1000, 0x1000, None)
    return m, q, w


def test_fused_entry_point_rejects_bad_arguments_before_launching():
    lib = b.raw()
    m, q, w = _structs()
    f = lib.qllm_norm_reassemble_quant
    X, G = 0x1000, 0x2000     # never dereferenced: every call below fails validation first
    ok = dict(x=X, dt=b.BF16, N=4, C=64, ldx=64, norm=b.NORM_RMS, gamma=G, beta=None, eps=1e-5, bits=4)

    def call(mp=m, qa=q, **kw):
        a = dict(ok, **kw)
        return f(a["x"], a["dt"], a["N"], a["C"], a["ldx"], a["norm"], a["gamma"], a["beta"], a["eps"],
                 C.byref(mp) if mp is not None else None, a["bits"], C.byref(qa) if qa is not None else None, None)

    assert call(x=None) == -1
    assert call(gamma=None) == -1
    assert call(mp=None) == -1 and call(qa=None) == -1
    assert call(dt=7) == -4 and call(norm=3) == -4
    assert call(C=0) == -2 and call(C=b.MAX_CHANNELS + 1, ldx=b.MAX_CHANNELS + 1) == -2
    assert call(ldx=63) == -2 and call(N=-1) == -2
    assert call(bits=5) == -3 and call(bits=2) == -3
    assert call(gamma=G + 4) == -6
    bad_map = b._Map(65, 64, 64, 0x1000, 0x1000, 0x1000, None)      # C_in differs from C
    assert call(mp=bad_map) == -2
    assert call(mp=b._Map(64, 64, 64, None, 0x1000, 0x1000, None)) == -1
    assert call(mp=b._Map(64, 64, 10, 0x1000, 0x1000, 0x1000, None)) == -2
    assert call(qa=b._QAct(0x1008, 0x1000, 0x1000, 0x1000)) == -6
    assert call(qa=b._QAct(0x1000, None, 0x1000, 0x1000)) == -1
    # a plan whose header (host copy) is not that of this map is refused before anything is launched
    head = (C.c_int32 * b.PLAN_HEAD)()
    assert call(mp=b._Map(64, 64, 64, 0x1000, 0x1000, 0x1000, 0x4000, head)) == -5
    head[:] = [0x514C4D50, 5, 64, 64, 32, 0, 8, 0, 0, 16, 48, 56, 56, 56, 0, 56]
    head[2] = 72                                                      # a plan made for another C_in
    assert call(mp=b._Map(64, 64, 64, 0x1000, 0x1000, 0x1000, 0x4000, head)) == -5
    head[2], head[13] = 64, 60                                        # length does not match the parts
    assert call(mp=b._Map(64, 64, 64, 0x1000, 0x1000, 0x1000, 0x4000, head)) == -5
    assert call(mp=b._Map(64, 64, 64, 0x1000, 0x1000, 0x1000, 0x4004, head)) == -6
    assert call(N=0) == 0                                             # empty batch: nothing to do


def test_gemm_entry_point_rejects_bad_arguments_before_launching():
    lib = b.raw()
    m, q, w = _structs()
    f = lib.qllm_int_gemm
    Y = 0x3000

    def call(qa=q, a_bits=4, N=4, wt=w, y=Y, ydt=b.F32, ldy=32, ws_bytes=0):
        return f(C.byref(qa) if qa is not None else None, a_bits, N, C.byref(wt) if wt is not None else None, y,
                 ydt, ldy, None, None, ws_bytes, None)

    assert call(qa=None) == -1 and call(wt=None) == -1 and call(y=None) == -1
    assert call(ydt=5) == -4
    assert call(a_bits=6) == -3                                      # 6-bit activations, 4-bit weights
    assert call(a_bits=4, wt=b._Weight(32, 64, 8, 0x1000, 0x1000, 0x1000, 0x1000)) == -3
    assert call(a_bits=3) == -3
    assert call(ldy=31) == -2 and call(N=-2) == -2
    assert call(wt=b._Weight(0, 64, 4, 0x1000, 0x1000, 0x1000, 0x1000)) == -2
    assert call(a_bits=8, wt=b._Weight(32, 40000, 8, 0x1000, 0x1000, 0x1000, 0x1000)) == -2   # could overflow int32
    assert call(wt=b._Weight(32, 64, 4, 0x1004, 0x1000, 0x1000, 0x1000)) == -6
    assert call(qa=b._QAct(0x1000, 0x1000, None, 0x1000)) == -1
    assert call(N=0) == 0
    # a weight that comes with tiles for the FP6 path, more than 64 tokens, room in the workspace: the tiles' and the
    # workspace's alignment are checked before anything is launched
    big = b._Weight(32, 64, 4, 0x1000, 0x1000, 0x1000, 0x1000, 0x5008)
    assert f(C.byref(q), 4, 128, C.byref(big), Y, b.F32, 32, None, 0x4000, 1 << 20, None) == -6
    good = b._Weight(32, 64, 4, 0x1000, 0x1000, 0x1000, 0x1000, 0x5000)
    assert f(C.byref(q), 4, 128, C.byref(good), Y, b.F32, 32, None, 0x4008, 1 << 20, None) == -6


def test_tiles6_entry_points_reject_bad_arguments_before_launching():
    lib = b.raw()
    f = lib.qllm_pack_tiles6
    assert f(None, 16, 128, 0x2000, None) == -1 and f(0x1000, 16, 128, None, None) == -1
    assert f(0x1000, -1, 128, 0x2000, None) == -2 and f(0x1000, 16, 0, 0x2000, None) == -2
    assert f(0x1008, 16, 128, 0x2000, None) == -6 and f(0x1000, 16, 128, 0x2004, None) == -6
    assert f(0x1000, 0, 128, 0x2000, None) == 0
    assert lib.qllm_tiles6_bytes(-1, 128) == -2 and lib.qllm_tiles6_bytes(16, 0) == -2


def test_tiles8_entry_points_reject_bad_arguments_before_launching():
    lib = b.raw()
    f = lib.qllm_pack_tiles8
    assert f(None, 6, 16, 128, 0x2000, None) == -1 and f(0x1000, 6, 16, 128, None, None) == -1
    assert f(0x1000, 5, 16, 128, 0x2000, None) == -3 and f(0x1000, 0, 16, 128, 0x2000, None) == -3
    assert f(0x1000, 8, -1, 128, 0x2000, None) == -2 and f(0x1000, 8, 16, 0, 0x2000, None) == -2
    assert f(0x1008, 4, 16, 128, 0x2000, None) == -6 and f(0x1000, 4, 16, 128, 0x2004, None) == -6
    assert f(0x1000, 6, 0, 128, 0x2000, None) == 0
    assert lib.qllm_tiles8_bytes(-1, 128) == -2 and lib.qllm_tiles8_bytes(16, 0) == -2
    # a weight's byte copy must be 16-byte aligned, and so must the workspace that receives the activations'
    q = b._QAct(0x1000, 0x1000, 0x1000, 0x1000)
    g = lib.qllm_int_gemm
    bad = b._Weight(32, 64, 6, 0x1000, 0x1000, 0x1000, 0x1000, None, 0x5008)
    assert g(C.byref(q), 6, 64, C.byref(bad), 0x9000, b.F32, 32, None, 0x4000, 1 << 20, None) == -6
    good = b._Weight(32, 64, 6, 0x1000, 0x1000, 0x1000, 0x1000, None, 0x5000)
    assert g(C.byref(q), 6, 64, C.byref(good), 0x9000, b.F32, 32, None, 0x4008, 1 << 20, None) == -6


def test_swiglu_entry_point_rejects_bad_arguments_before_launching():
    f = b.raw().qllm_swiglu
    G, U, X = 0x1000, 0x2000, 0x3000
    assert f(None, 64, U, 64, 4, 64, X, 64, None) == -1 and f(G, 64, None, 64, 4, 64, X, 64, None) == -1
    assert f(G, 64, U, 64, 4, 64, None, 64, None) == -1
    assert f(G, 63, U, 64, 4, 64, X, 64, None) == -2 and f(G, 64, U, 64, 4, 64, X, 10, None) == -2
    assert f(G, 64, U, 64, -1, 64, X, 64, None) == -2 and f(G, 64, U, 64, 4, 0, X, 64, None) == -2
    assert f(G + 1, 64, U, 64, 4, 64, X, 64, None) == -6
    assert f(G, 64, U, 64, 0, 64, X, 64, None) == 0


def test_linear_entry_point_rejects_bad_arguments_before_launching():
    lib = b.raw()
    m, q, w = _structs()
    f = lib.qllm_reassembled_linear

    def call(mp=m, wt=w, N=4, ws=0x4000, ws_bytes=1 << 20):
        return f(0x1000, b.BF16, N, 64, 64, b.NORM_RMS, 0x2000, None, 1e-5, C.byref(mp), 4, C.byref(wt), 0x3000,
                 b.F32, 32, ws, ws_bytes, None)

    assert call(wt=b._Weight(32, 65, 4, 0x1000, 0x1000, 0x1000, 0x1000)) == -2     # K != C_out
    assert call(ws=None) == -7 and call(ws_bytes=16) == -7
    assert call(ws=0x4010) == -6
    assert call(N=0) == 0


# ---------------------------------------------------------------- host helpers against the oracle

def test_build_map_matches_hand_worked_example():
    G = json.load(open(os.path.join(ROOT, "tests", "golden", "hand_worked_example.json")))
    r = b.qllm_build_map_host(np.abs(np.array(G["y"], np.float32)), G["theta"], G["src_idx"], G["dst_idx"])
    assert r["num_split"].tolist() == G["T"]
    assert r["row_ptr"].tolist() == G["map_row_ptr"] and r["src"].tolist() == G["map_src"]
    assert r["scale"].tolist() == [float(np.float32(n / d)) for n, d in G["map_scale_num_den"]]
    assert (r["C_out"], r["nnz"]) == (6, 7)


def check_plan_decodes_to_map(plan, row_ptr, src, scale, C, K):
    """Reads a plan the way its layout is documented in include/qllm.h and rebuilds, for every output channel,
    the list of (source, scale) entries it stands for; that has to be the CSR map the plan was made from."""
    n_groups, n_chunks, n_work = (K + 7) // 8, (C + 7) // 8, (K + 255) // 256 * 32
    magic, version, c_in, c_out, nw, n_comp, nc, n_long, n_pub, n_spec, n_dest, n_segw, off_chunks, plan_len, n_xl, \
        n_xle = plan[:16].tolist()
    assert (magic, version, c_in, c_out, nw, nc) == (0x514C4D50, 8, C, K, n_work, n_chunks)
    r4 = lambda v: (v + 3) // 4 * 4
    off_work = 16
    assert off_chunks == r4(off_work + n_work)
    off_spec = r4(off_chunks + n_chunks)
    off_dest = r4(off_spec + 2 * n_spec)
    off_longs = r4(off_dest + n_dest)
    off_segs = off_longs + 4 * n_long
    off_recs = r4(off_segs + n_segw)
    off_xlrows = off_recs + 8 * n_comp
    off_xlent = off_xlrows + 4 * n_xl
    assert plan_len == plan.size == off_xlent + 2 * n_xle
    work = plan[off_work:off_work + n_work].astype(np.int64) & 0xFFFFFFFF
    kind, grp, field = work >> 30, (work >> 17) & 0x1FFF, work & 0x1FFFF
    assert sorted(grp.tolist()) == list(range(n_work))          # every group exactly once
    assert np.all(np.diff(kind * 8192 + grp) > 0)                # by kind, then by group
    assert np.all(kind[grp >= n_groups] == 2) and np.all(kind[grp < n_groups] < 2) and (kind == 1).sum() == n_comp
    chunks = plan[off_chunks:off_chunks + n_chunks].astype(np.int64) & 0xFFFFFFFF
    passes, slots = chunks & 0xFF, chunks >> 8
    staged = slots != 0xFFFFFF
    assert staged.sum() == n_pub and np.array_equal(slots[staged], np.arange(n_pub))
    chan_of_pos = {int(slots[ch]) * 8 + j: ch * 8 + j for ch in np.nonzero(staged)[0] for j in range(8)}
    zero_at = 8 * n_pub
    spec = plan[off_spec:off_spec + 2 * n_spec].reshape(n_spec, 2)
    dest = plan[off_dest:off_dest + n_dest]
    longs = plan[off_longs:off_segs].reshape(-1, 4).copy()
    segs = plan[off_segs:off_segs + n_segw]
    recs = plan[off_recs:off_xlrows].reshape(n_comp, 8)
    xlrows = plan[off_xlrows:off_xlent].reshape(n_xl, 4)
    xlent = plan[off_xlent:].reshape(n_xle, 2)
    most = longs[:, 3] >> 8                                       # largest position among the 64 entries of a wavefront
    longs[:, 3] &= 0xFF
    for b0 in range(0, n_long, 64):
        assert np.all(most[b0:b0 + 64] == longs[b0:b0 + 64, 3].max())
    as_f = lambda w: np.array([w], np.int32).view(np.float32)[0]
    rebuilt = {}                                                   # output channel -> [(source, scale bits)]
    comp_group = {}
    for kd, g, f in zip(kind, grp, field):
        if kd == 0:                                                # plain: 8 copies of consecutive sources
            assert 0 <= f <= C - 8
            for k in range(8):
                rebuilt[8 * g + k] = [(int(f) + k, np.float32(1.0))]
        elif kd == 1:                                              # composite: masked windows
            hdr = int(segs[f]) & 0xFFFFFFFF
            n_seg, number = hdr & 0xFF, hdr >> 8
            comp_group[number] = int(g)
            first_two = [int(v) for sg in range(min(n_seg, 2)) for v in segs[f + 1 + 3 * sg:f + 3 + 3 * sg]]
            assert recs[number].tolist() == [n_seg | (int(f) << 8)] + first_two + [0] * (4 - len(first_two)) + [int(g), 0, 0]
            seen = 0
            for sg in range(n_seg):
                d, m8, pad = (int(v) for v in segs[f + 1 + 3 * sg:f + 4 + 3 * sg])
                assert pad == 0 and 0 < m8 < 256 and not (seen & m8)
                seen |= m8
                for k in range(8):
                    if m8 >> k & 1:
                        assert 0 <= d + k < C
                        rebuilt[8 * g + k] = [(d + k, np.float32(1.0))]
    assert sorted(comp_group) == list(range(n_comp))
    for i in range(n_spec):                                        # computed channels
        word, sbits = int(spec[i, 0]) & 0xFFFFFFFF, spec[i, 1]
        s0, s1 = word & 0xFFFF, word >> 16
        ch = 8 * comp_group[int(dest[i]) >> 3] + (int(dest[i]) & 7)
        assert ch not in rebuilt
        rebuilt[ch] = [(chan_of_pos[s0], as_f(sbits))] + ([] if s1 == zero_at else [(chan_of_pos[s1], as_f(sbits))])
    at, seen_rows = 0, 0
    while at < n_long:                                             # long rows; padding entries have slot -1 and scale bits 0
        if longs[at, 1] == -1 and longs[at, 3] == 0 and longs[at, 2] == 0 and (at + 1 >= n_long or longs[at + 1, 3] == 0):
            at += 1                                                # padding
            continue
        entries, first = [], at
        while True:
            assert longs[at, 3] == at - first and at // 64 == first // 64   # positions count up inside one wavefront
            entries.append((chan_of_pos[int(longs[at, 0])], as_f(longs[at, 2])))
            at += 1
            if longs[at - 1, 1] >= 0:
                break
        slot = int(longs[at - 1, 1])
        assert n_spec <= slot < n_dest - n_xl
        ch = 8 * comp_group[int(dest[slot]) >> 3] + (int(dest[slot]) & 7)
        assert ch not in rebuilt and 2 <= len(entries) <= 64
        rebuilt[ch] = entries
        seen_rows += 1
    assert seen_rows == n_dest - n_spec - n_xl
    at = 0
    for r in range(n_xl):                                          # rows of more than 64 entries, entries back to back
        first, n, slot, pad = (int(v) for v in xlrows[r])
        assert first == at and n > 64 and slot == n_dest - n_xl + r and pad == 0
        ch = 8 * comp_group[int(dest[slot]) >> 3] + (int(dest[slot]) & 7)
        assert ch not in rebuilt
        rebuilt[ch] = [(chan_of_pos[int(xlent[e, 0])], as_f(xlent[e, 1])) for e in range(first, first + n)]
        at += n
    assert at == n_xle
    assert sorted(rebuilt) == list(range(K))
    expect_pass = np.zeros(n_chunks * 8, bool)
    for ch in range(K):
        e0, e1 = row_ptr[ch], row_ptr[ch + 1]
        want = [(int(src[e]), np.float32(scale[e])) for e in range(e0, e1)]
        assert rebuilt[ch] == want, (ch, rebuilt[ch], want)
        if e1 - e0 == 1 and scale[e0] == 1.0:
            expect_pass[src[e0]] = True
    assert np.array_equal(np.unpackbits(passes.astype(np.uint8), bitorder="little"), expect_pass.astype(np.uint8))
    # staged: the chunks that hold a source of a computed or long channel, or all chunks
    needed = np.zeros(n_chunks, bool)
    for ch in range(K):
        e0, e1 = row_ptr[ch], row_ptr[ch + 1]
        if not (e1 - e0 == 1 and scale[e0] == 1.0):
            needed[src[e0:e1] // 8] = True
    assert np.array_equal(staged, needed) or staged.all()


@pytest.mark.parametrize("C_in,C_out,special_every", [(2048, 2100, 37), (8200, 8000, 61), (1000, 1003, 5), (64, 9, 2)])
@pytest.mark.parametrize("longest", [5, 150])
def test_plan_of_an_arbitrary_map_decodes_to_it(C_in, C_out, special_every, longest):
    # repeated and unreferenced sources, rows of 1..longest entries with any scales, plain groups at every misalignment
    rng = np.random.default_rng(C_in + special_every)
    row_ptr, src, scale = random_csr_map(rng, C_in, C_out, special_every, longest)
    plan, n_comp = b.qllm_plan_map_host(row_ptr, src, scale, C_in)
    assert plan[5] == n_comp
    check_plan_decodes_to_map(plan, row_ptr, src, scale, C_in, C_out)


def host_map(row_ptr, src, scale, C_in, plan):
    """A qllm_map whose pointers are host arrays: enough for the calls that only read sizes and the plan's header."""
    keep = [np.ascontiguousarray(row_ptr, np.int32), np.ascontiguousarray(src, np.int32), np.ascontiguousarray(scale, np.float32)]
    head = (C.c_int32 * b.PLAN_HEAD)()
    plan_ptr = None
    if plan is not None:
        keep.append(np.ascontiguousarray(plan, np.int32))
        head[:] = [int(v) for v in keep[3][:b.PLAN_HEAD]]
        plan_ptr = keep[3].ctypes.data
    m = b._Map(C_in, keep[0].size - 1, keep[1].size, keep[0].ctypes.data, keep[1].ctypes.data, keep[2].ctypes.data, plan_ptr, head)
    m.keep = keep
    return types.SimpleNamespace(c=m)


def test_fused_kernel_choice_follows_what_fits_on_chip():
    rng = np.random.default_rng(5)
    # a benchmark-like map: a few special rows; its lists fit in LDS
    small = random_csr_map(rng, 4096, 4096, 97)
    plan = b.qllm_plan_map_host(*small, 4096)[0]
    m = host_map(*small, 4096, plan)
    assert b.qllm_fused_kernel_choice(m, b.BF16, 2048, 4096, b.NORM_RMS, False, 4) == b.FUSED_LISTS_IN_LDS
    assert b.qllm_fused_kernel_choice(m, b.F32, 1, 4096, b.NORM_LAYER, True, 8) == b.FUSED_LISTS_IN_LDS
    # rows that are not 16-byte aligned, and a map without a plan: the kernel that walks the CSR rows
    assert b.qllm_fused_kernel_choice(m, b.BF16, 2048, 4099, b.NORM_RMS, False, 4) == b.FUSED_WALKS_MAP
    assert b.qllm_fused_kernel_choice(host_map(*small, 4096, None), b.BF16, 2048, 4096, b.NORM_RMS, False, 4) == b.FUSED_WALKS_MAP
    # every other channel computed, on a long row: the lists no longer fit in LDS and are streamed
    big = random_csr_map(rng, 16384, 16000, 2)
    plan = b.qllm_plan_map_host(*big, 16384)[0]
    assert plan[8] == plan[6]                                   # every chunk staged
    m = host_map(*big, 16384, plan)
    for dt in (b.BF16, b.F32):
        for bits in (4, 6, 8):
            assert b.qllm_fused_kernel_choice(m, dt, 64, 16384, b.NORM_LAYER, True, bits) == b.FUSED_LISTS_STREAMED
    # ... unless the row itself does not fit next to its codes (fp32 input of 28 672 channels)
    huge = random_csr_map(rng, 28672, 28672, 4)
    plan = b.qllm_plan_map_host(*huge, 28672)[0]
    m = host_map(*huge, 28672, plan)
    assert b.qllm_fused_kernel_choice(m, b.BF16, 64, 28672, b.NORM_RMS, False, 4) == b.FUSED_LISTS_STREAMED
    assert b.qllm_fused_kernel_choice(m, b.F32, 64, 28672, b.NORM_RMS, False, 4) == b.FUSED_WALKS_MAP
    # arguments the kernel's entry point would reject
    for bad in [dict(x_dtype=7), dict(norm=9), dict(bits=5), dict(N=-1), dict(ldx=100)]:
        args = dict(x_dtype=b.BF16, N=64, ldx=28672, norm=b.NORM_RMS, has_beta=False, bits=4)
        args.update(bad)
        with pytest.raises(b.QllmError):
            b.qllm_fused_kernel_choice(m, **args)


@pytest.mark.parametrize("name,N,C,O", [("tiny", 64, 512, 96), ("llama7b_qkv", 48, 1000, 40),
                                        ("llama70b_down", 32, 2050, 24), ("llama70b_q_decode", 16, 777, 33)])
def test_host_helpers_match_the_oracle(oracle, name, N, C, O):
    w = wl.WORKLOADS[name]
    c = make_case(oracle, w, N=N, C=C, O=O)
    r = b.qllm_build_map_host(c.absmax, c.theta, c.src_idx, c.dst_idx)
    assert np.array_equal(r["num_split"], c.T)
    assert np.array_equal(r["row_ptr"], c.row_ptr) and np.array_equal(r["src"], c.src)
    assert np.array_equal(r["scale"], c.scale)
    assert b.qllm_check_map_host(r["row_ptr"], r["src"], r["scale"], C) == 0
    # the plan decodes back to exactly this map
    check_plan_decodes_to_map(r["plan"], c.row_ptr, c.src, c.scale, C, c.K)



@pytest.mark.parametrize("bits", [4, 6, 8])
def test_pack_helpers_match_the_oracle(oracle, bits):
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 2 ** bits, (7, 300), dtype=np.uint8)
    p = b.qllm_pack_codes_host(codes, bits)
    assert np.array_equal(p, oracle.pack_codes(codes, bits, p.shape[1]))
    assert np.array_equal(b.qllm_unpack_codes_host(p, 300, bits), codes)
    with pytest.raises(b.QllmError):
        b.qllm_pack_codes_host(np.full((1, 4), 2 ** bits if bits < 8 else 0, np.uint8) if bits < 8
                               else np.zeros((1, 0), np.uint8), bits)


def test_build_map_rejects_malformed_merge_lists():
    m = np.array([1, 1, 9, 1, 1, 1], np.float32)        # theta 4: channel 2 splits in 3 -> positions 2,3,4
    with pytest.raises(b.QllmError) as e:
        b.qllm_build_map_host(m, 4.0, [1], [0])         # A member 1 = position 2: a sub-channel
    assert e.value.status == -5
    with pytest.raises(b.QllmError):
        b.qllm_build_map_host(m, 4.0, [0], [1])         # B member 1 = position 3: a sub-channel
    with pytest.raises(b.QllmError):
        b.qllm_build_map_host(m, 4.0, [0, 0], [0, 3])   # A member merged twice
    with pytest.raises(b.QllmError):
        b.qllm_build_map_host(m, 4.0, [4], [0])         # outside set A (8 positions -> 4 members)
    with pytest.raises(b.QllmError):
        b.qllm_build_map_host(m, 0.0, [], [])           # theta must be positive
    ok = b.qllm_build_map_host(m, 4.0, [0, 3], [0, 0])  # positions 0 and 6 both join position 1: group of 3
    assert ok["C_out"] == 6 and np.diff(ok["row_ptr"]).max() == 3
    bad_rp = ok["row_ptr"].copy()
    bad_rp[2] = bad_rp[1]
    assert b.qllm_check_map_host(bad_rp, ok["src"], ok["scale"], 6) == -5
    bad_src = ok["src"].copy()
    bad_src[0] = 6
    assert b.qllm_check_map_host(ok["row_ptr"], bad_src, ok["scale"], 6) == -5


def test_fold_linear_host_matches_the_oracle(oracle):
    """Appendix B through the library's host helper (driven by the CSR map) against the oracle's
    float64 statement of it (driven by T and the index pairs)."""
    rng = np.random.default_rng(5)
    C, Kp = 200, 37
    absmax = np.abs(rng.standard_normal(C)).astype(np.float32) + 0.1
    absmax[[3, 50, 120]] = [9.0, 14.5, 6.1]
    theta = 3.0
    T = oracle.num_split(absmax, theta)
    chan_of = np.repeat(np.arange(C), T)
    elig = T[chan_of] == 1
    pa = np.arange(0, chan_of.size, 2)
    pb = np.arange(1, chan_of.size, 2)
    pa, pb = pa[elig[pa]], pb[elig[pb]]
    sp = rng.choice(pa, size=11, replace=False)
    dp = rng.choice(pb, size=11, replace=True)
    src_idx, dst_idx = (sp // 2).astype(np.int32), ((dp - 1) // 2).astype(np.int32)
    m = b.qllm_build_map_host(absmax, theta, src_idx, dst_idx, with_plan=False)
    Wp = rng.standard_normal((C, Kp)).astype(np.float32)
    bp = rng.standard_normal(C).astype(np.float32)
    W_hat, b_hat = b.qllm_fold_linear_host(Wp, bp, m["row_ptr"], m["src"], m["scale"])
    W_ref, b_ref = oracle.fold_preceding_linear(Wp, bp, T, src_idx, dst_idx)
    assert W_hat.shape == W_ref.shape == (m["row_ptr"].size - 1, Kp)
    assert np.abs(W_hat - W_ref).max() <= 2e-7 * np.abs(W_ref).max()
    assert np.abs(b_hat - b_ref).max() <= 2e-7 * np.abs(b_ref).max()
    W_only, none = b.qllm_fold_linear_host(Wp, None, m["row_ptr"], m["src"], m["scale"])
    assert none is None and np.array_equal(W_only, W_hat)
    # argument checks
    bad = m["src"].copy()
    bad[0] = C
    with pytest.raises(RuntimeError):
        b.qllm_fold_linear_host(Wp, bp, m["row_ptr"], bad, m["scale"])


def test_matching_entry_point_rejects_bad_arguments_before_launching():
    f = b.raw().qllm_match_nearest
    P = 0x1000                # never dereferenced: every call below fails validation first
    ok = dict(y=P, n=16, ldy=64, W=P, C=64, O=32, ldw=32, ca=P, nA=10, cb=P, nB=12, bj=P, bd=P, ws=P, wsb=1 << 20)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["y"], a["n"], a["ldy"], a["W"], a["C"], a["O"], a["ldw"], a["ca"], a["nA"], a["cb"], a["nB"],
                 a["bj"], a["bd"], a["ws"], a["wsb"], None)

    for k in ("y", "ca", "cb", "bj", "bd"):
        assert call(**{k: None}) == -1
    assert call(W=None, O=0, ldw=0, nA=0) == 0                        # no weights: the plain L2 distance (O, ldw ignored)
    assert call(W=None, O=0, ldw=0, ws=None) == -7                    # ... and the same checks after that
    assert call(n=0) == -2 and call(O=0) == -2 and call(ldy=63) == -2 and call(ldw=31) == -2 and call(nA=-1) == -2
    assert call(nB=0) == -2
    assert call(ws=None) == -7 and call(wsb=b.qllm_match_workspace_bytes(10, 12) - 1) == -7
    assert call(ws=P + 4) == -6
    assert call(nA=0) == 0                                            # nothing to match
    assert b.qllm_match_workspace_bytes(10, 12) == 2 * 22 * 8 + 16 * 10 * 12 and b.qllm_match_workspace_bytes(-1, 3) == -2


def test_select_edges_host_matches_the_oracle():
    """Appendix A step 3 with ties: the library's host helper against the oracle's selection."""
    from oracle import calibrate
    rng = np.random.default_rng(8)
    nA = 500
    best_d = rng.integers(0, 40, nA).astype(np.float64)              # many ties
    best_j = rng.integers(0, 300, nA)
    pos_a, pos_b = 2 * np.arange(nA), 2 * np.arange(300) + 1
    for r in (0, 1, 37, 499, 500, 800):
        pick = b.qllm_select_edges_host(best_d, r)
        src_idx, dst_idx = calibrate.select_edges(best_d, best_j, pos_a, pos_b, r)
        assert pick.tolist() == src_idx.tolist()
        assert (dst_idx.tolist() == best_j[pick].tolist())


# ---------------------------------------------------------------- offline host helpers around the channel matching

def test_matching_sets_and_pairs_host_match_the_oracle():
    from oracle import calibrate
    rng = np.random.default_rng(31)
    T = np.ones(41, np.int32)
    T[[0, 13, 40]] = [3, 2, 5]
    sets = b.qllm_matching_sets_host(T)
    chan_of, pos_a, pos_b = calibrate.matching_sets(T)
    assert np.array_equal(sets["pos_a"], pos_a) and np.array_equal(sets["pos_b"], pos_b)
    assert np.array_equal(sets["chan_a"], chan_of[pos_a]) and np.array_equal(sets["chan_b"], chan_of[pos_b])
    best_d = rng.integers(0, 4, pos_a.size).astype(np.float64)               # many ties
    best_j = rng.integers(0, pos_b.size, pos_a.size).astype(np.int32)
    for r in (0, 1, 5, pos_a.size, pos_a.size + 9):
        src_idx, dst_idx = b.qllm_pairs_host(best_d, best_j, pos_a, pos_b, r)
        ref_s, ref_d = calibrate.select_edges(best_d, best_j.astype(np.int64), pos_a, pos_b, r)
        assert np.array_equal(src_idx, ref_s) and np.array_equal(dst_idx, ref_d)
    with pytest.raises(b.QllmError):
        b.qllm_matching_sets_host(np.array([1, 0, 2], np.int32))               # a split count below 1


def test_theta_helpers_match_the_oracle():
    from oracle import calibrate
    rng = np.random.default_rng(32)
    m = np.abs(rng.standard_normal(500)).astype(np.float32)
    m[[3, 77, 300]] *= [40, 90, 25]
    for ratio in (0.002, 0.01, 0.05, 0.1, 0.6):
        target = max(1, int(round(ratio * m.size)))
        assert b.qllm_theta_for_expansion_host(m, target) == calibrate.theta_from_rule(m, ("expand", ratio))
    assert b.qllm_theta_for_expansion_host(np.array([1.0, 2.0, 12.0], np.float32), 2) == float(np.nextafter(np.float32(6), np.float32(0)))
    for P in (1, 4, 7):
        assert b.qllm_theta_grid_host(m, P) == calibrate.theta_grid(m, P)
    assert b.qllm_theta_grid_host(np.array([0.5, 2.0, 8.5, 1.0], np.float32), 4) == [2.5, 4.5, 6.5, 8.5]
    with pytest.raises(b.QllmError):
        b.qllm_theta_for_expansion_host(np.zeros(4, np.float32), 1)


def test_binding_wrappers_reject_mismatched_tensors_before_calling_the_library():
    """The C ABI trusts the sizes it is told; the Python wrappers check what they can see (shape, dtype, dense
    rows, device) and raise before anything reaches the library.  Runs on CPU tensors: every case below fails on a
    shape or dtype check, or at last on "must be a device tensor"."""
    import torch
    N, Cc, K, O = 4, 64, 72, 16
    x = torch.zeros((N, Cc), dtype=torch.float32)
    gamma = torch.ones(Cc)
    dmap = types.SimpleNamespace(C_in=Cc, C_out=K, c=None)
    out = types.SimpleNamespace(N=N, K=K, bits=4, c=None)
    weight = types.SimpleNamespace(O=O, K=K, bits=4, c=None)
    y = torch.zeros((N, O))
    ws = torch.zeros(1024, dtype=torch.uint8)
    fused = lambda **kw: b.qllm_norm_reassemble_quant(**{**dict(x=x, norm=b.NORM_RMS, gamma=gamma, beta=None, eps=1e-5,
                                                                dmap=dmap, bits=4, out=out), **kw})
    cases = [
        (lambda: fused(x=torch.zeros((N, Cc + 8))), "the map takes"),
        (lambda: fused(gamma=torch.ones(Cc - 1)), "gamma must hold"),
        (lambda: fused(gamma=None), "gamma is required"),
        (lambda: fused(beta=torch.ones(Cc, dtype=torch.float64)), "beta has dtype"),
        (lambda: fused(x=torch.zeros((N, 2 * Cc))[:, ::2]), "stride 1"),
        (lambda: fused(x=torch.zeros((N, Cc), dtype=torch.float16)), "x has dtype"),
        (lambda: fused(out=types.SimpleNamespace(N=N - 1, K=K, bits=4)), "holds 3 tokens"),
        (lambda: fused(out=types.SimpleNamespace(N=N, K=K + 8, bits=4)), "channels"),
        (lambda: fused(out=types.SimpleNamespace(N=N, K=K, bits=8)), "8-bit codes"),
        (lambda: fused(norm=7), "unknown norm"),
        (lambda: fused(), "x must be a device"),
        (lambda: b.qllm_int_gemm(out, types.SimpleNamespace(O=O, K=K + 8, bits=4), y), "weights"),
        (lambda: b.qllm_int_gemm(out, weight, torch.zeros((N, O + 1))), "y has shape"),
        (lambda: b.qllm_int_gemm(out, weight, y, acc_dump=torch.zeros(N * O, dtype=torch.int64)), "acc_dump has dtype"),
        (lambda: b.qllm_reassembled_linear(x, b.NORM_NONE, None, None, 0.0, dmap, 4, types.SimpleNamespace(O=O, K=K - 8, bits=4), y, ws),
         "the weights take"),
        (lambda: b.qllm_reassembled_linear(x, b.NORM_NONE, None, None, 0.0, dmap, 4, weight, torch.zeros((N + 1, O)), ws), "y has shape"),
        (lambda: b.qllm_reassembled_linear_static(x, b.NORM_NONE, None, None, 0.0, dmap, 4, weight, y.to(torch.float64)), "y has dtype"),
        (lambda: b.qllm_norm_channel_absmax(x, b.NORM_RMS, gamma, None, 1e-5, torch.zeros(Cc + 1)), "absmax must hold"),
        (lambda: b.qllm_norm_channel_absmax(x, b.NORM_RMS, gamma, None, 1e-5, torch.zeros(Cc), torch.zeros((2, Cc + 1))), "y_dump"),
        (lambda: b.qllm_match_nearest(x, torch.zeros((Cc + 1, O)), *[torch.zeros(3, dtype=torch.int32)] * 3, torch.zeros(3, dtype=torch.float64), ws),
         "one row per channel"),
        (lambda: b.qllm_match_nearest(x, None, torch.zeros(3, dtype=torch.int32), torch.zeros(3, dtype=torch.int32),
                                      torch.zeros(2, dtype=torch.int32), torch.zeros(3, dtype=torch.float64), ws), "best_j must hold"),
    ]
    for call, text in cases:
        with pytest.raises(ValueError, match=text):
            call()
