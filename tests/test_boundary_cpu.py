"""Host-side checks of the C-ABI library that need no GPU: the library loads,
exports what include/agent_attn.h declares, and rejects bad arguments before
launching anything (every call below must fail, so no kernel ever starts)."""
import ctypes
import os
import re

import pytest

from paper_2312_08874_amd import binding
from paper_2312_08874_amd.binding import aa_params, make_desc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # non-null, 256-aligned; never dereferenced because validation fails first


def declared_functions():
    src = open(os.path.join(ROOT, "include", "agent_attn.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(agent_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for nme in names:
        assert getattr(L, nme) is not None


def test_struct_layout_matches_header():
    # int32 x10, float x3, int32, int64 x6, int32 x2 -> 112 bytes; params: 6 ptr, 2 int32, 3 ptr -> 80 bytes
    assert ctypes.sizeof(binding.aa_desc) == 112
    assert binding.aa_desc.image_h.offset == 104 and binding.aa_desc.image_w.offset == 108
    assert ctypes.sizeof(binding.aa_params) == 80


def test_flops_follow_the_cost_model():
    """Eq. (7): agent attention costs 2nNC + 2NnC multiply-adds per image, C = heads*d."""
    for (B, H, N, n, d) in [(1, 1, 196, 49, 32), (64, 3, 196, 49, 64), (1, 8, 16384, 1024, 64)]:
        C = H * d
        macs = 2 * n * N * C + 2 * N * n * C
        assert binding.flops(make_desc(B, H, N, n, d, binding.AA_BF16)) == 2 * macs * B
    assert binding.flops(make_desc(1, 1, 0, 4, 4, binding.AA_F32)) == 0


def test_windows_in_the_descriptor_are_validated_on_the_host():
    """image_h x image_w cut into grid-sized windows: units and workspace scale with the number of windows."""
    one = make_desc(2, 3, 49, 9, 32, binding.AA_BF16, (7, 7), (3, 3))
    win = make_desc(2, 3, 49, 9, 32, binding.AA_BF16, (7, 7), (3, 3), image=(56, 56))
    assert binding.flops(win) == 64 * binding.flops(one)
    assert binding.workspace_bytes(win) > binding.workspace_bytes(one) > 0
    assert "64 windows per image" in binding.plan_str(win)
    same = make_desc(2, 3, 49, 9, 32, binding.AA_BF16, (7, 7), (3, 3), image=(7, 7))      # one window = no windows
    assert binding.workspace_bytes(same) == binding.workspace_bytes(one)
    for image in ((56, 55), (50, 56), (56, 0), (-7, 7), (70000 * 7, 7)):
        assert binding.workspace_bytes(make_desc(2, 3, 49, 9, 32, binding.AA_BF16, (7, 7), (3, 3), image=image)) == 0
    assert binding.workspace_bytes(make_desc(2, 3, 49, 9, 32, binding.AA_BF16, None, None, image=(56, 56))) == 0
    # too many (batch, window, head) units for the launch grid
    assert binding.workspace_bytes(make_desc(64, 8, 49, 9, 32, binding.AA_BF16, (7, 7), (3, 3), image=(112, 112))) == 0


def test_workspace_query():
    d = make_desc(2, 3, 196, 49, 32, binding.AA_BF16, (14, 14), (7, 7))
    w1 = binding.workspace_bytes(d)
    assert w1 > 0 and w1 % 256 == 0
    d2 = make_desc(2, 3, 196, 49, 32, binding.AA_BF16, (14, 14), (7, 7), n_splits=4)
    assert binding.workspace_bytes(d2) >= w1 or binding.workspace_bytes(d2) > 0
    assert binding.workspace_bytes(make_desc(2, 3, 196, 49, 32, 7)) == 0          # bad dtype
    assert binding.workspace_bytes(make_desc(2, 3, 197, 49, 32, 0, (14, 14))) == 0  # N != h*w


def call_fwd(desc, Q=FAKE, K=FAKE * 2, V=FAKE * 3, A=None, params=None, ws=FAKE * 4, ws_bytes=1 << 40,
             out=FAKE * 5 + (1 << 41)):
    L = binding.lib()
    return L.agent_attn_fwd(ctypes.byref(desc), Q, K, V, A, None if params is None else ctypes.byref(params),
                            ws, ws_bytes, out, None)


def test_fwd_rejects_bad_arguments():
    ok = dict(grid=(14, 14), agent_grid=(7, 7))
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 5, **ok)) == -3                      # dtype
    assert call_fwd(make_desc(0, 1, 196, 49, 32, 0, **ok)) == -2                      # batch
    assert call_fwd(make_desc(1, 1, 196, 49, 0, 0, **ok)) == -2                       # d
    assert call_fwd(make_desc(1, 1, 195, 49, 32, 0, **ok)) == -2                      # N != h*w
    assert call_fwd(make_desc(1, 1, 196, 48, 32, 0, **ok)) == -2                      # n != ah*aw
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, grid=(14, 14))) == -4             # pooling without agent grid
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, agent_grid=(7, 7))) == -4         # pooling without token grid
    assert call_fwd(make_desc(1, 1, 196, 400, 32, 0, grid=(14, 14), agent_grid=(20, 20))) == -4
    assert call_fwd(make_desc(1, 1, 196, 49, 512, 0, **ok)) == -7                     # d too large
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, **ok), Q=None) == -1
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, **ok), out=None) == -1
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, **ok), ws=None) == -5
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, **ok), ws=FAKE * 4 + 8) == -5     # misaligned
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, **ok), ws_bytes=64) == -5         # too small
    d = make_desc(1, 1, 196, 49, 32, 0, **ok)
    assert call_fwd(d, out=FAKE) == -6                                                # out aliases Q
    assert call_fwd(d, out=FAKE * 3 + 16) == -6                                       # out overlaps V
    # strides: rows closer than d; some but not all strides of a batched problem; out overlapping a strided input
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, strides=(0, 0, 16), **ok)) == -2
    assert call_fwd(make_desc(2, 3, 196, 49, 32, 0, strides=(0, 0, 96), **ok)) == -2
    assert call_fwd(make_desc(2, 3, 196, 49, 32, 0, strides=(-1, 32, 96), **ok)) == -2
    assert call_fwd(make_desc(2, 3, 196, 49, 32, 0, out_strides=(0, 32, 96), **ok)) == -2
    wide = make_desc(2, 3, 196, 49, 32, 0, strides=(196 * 288, 32, 288), **ok)        # q of a fused [B,N,3,H,d] tensor
    assert call_fwd(wide, out=FAKE + 2 * 196 * 288 * 4 - 64) == -6                    # inside Q's strided extent
    # bias without a token grid; block bias without its size; DWC bias without DWC weights
    p = aa_params()
    p.b1_row = FAKE * 7
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0), A=FAKE * 6, params=p) == -2
    p = aa_params()
    p.b2_blk = FAKE * 7
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, **ok), params=p) == -2
    p = aa_params()
    p.dwc_b = FAKE * 7
    assert call_fwd(make_desc(1, 1, 196, 49, 32, 0, **ok), params=p) == -1


def test_module_entry_point_rejects_bad_arguments():
    """agent_attn_module_fwd validates on the host before it loads the BLAS library or launches anything."""
    L = binding.lib()
    proj = binding.aa_projections(FAKE * 6, None, FAKE * 7, None)
    d = make_desc(2, 3, 196, 49, 64, binding.AA_BF16, (14, 14), (7, 7))
    need = L.agent_attn_module_workspace_bytes(ctypes.byref(d), None)
    plain = binding.workspace_bytes(make_desc(2, 3, 196, 49, 64, binding.AA_BF16, (14, 14), (7, 7),
                                              strides=(196 * 576, 64, 576), out_strides=(196 * 192, 64, 192)))
    assert need >= plain + 4 * 2 * 196 * 192 * 2      # q | k | v and o on top of the attention's workspace

    def call(desc, x=FAKE, p=proj, ws=FAKE * 4, ws_bytes=1 << 40, y=FAKE * 5 + (1 << 41)):
        return L.agent_attn_module_fwd(ctypes.byref(desc), x, None if p is None else ctypes.byref(p), None, ws, ws_bytes,
                                       y, None)

    assert call(d, x=None) == -1 and call(d, p=None) == -1 and call(d, y=None) == -1
    assert call(d, p=binding.aa_projections(None, None, FAKE * 7, None)) == -1
    assert call(d, ws=None) == -5 and call(d, ws_bytes=need - 1) == -5
    assert call(d, y=FAKE + 64) == -6                                                   # y overlaps x
    assert call(make_desc(2, 3, 196, 49, 64, binding.AA_BF16, (14, 14), (7, 7), strides=(196 * 192, 64, 192))) == -2
    assert call(make_desc(2, 3, 196, 49, 64, binding.AA_BF16, None, (7, 7))) == -4      # the module pools: grids needed
    assert call(make_desc(2, 3, 196, 49, 64, 9, (14, 14), (7, 7))) == -3
    assert L.agent_attn_module_workspace_bytes(ctypes.byref(make_desc(2, 3, 195, 49, 64, 2, (14, 14), (7, 7))), None) == 0


def test_stage_entry_points_reject_bad_arguments():
    L = binding.lib()
    d = make_desc(1, 1, 196, 49, 32, 0, (14, 14), (7, 7))
    assert L.agent_pool_fwd(ctypes.byref(d), None, FAKE, None) == -1
    assert L.agent_pool_fwd(ctypes.byref(make_desc(1, 1, 196, 49, 32, 0, (14, 14))), FAKE, FAKE * 9, None) == -4
    assert L.agent_pool_fwd(ctypes.byref(d), FAKE, FAKE + 64, None) == -6
    assert L.agent_aggregate_fwd(ctypes.byref(d), FAKE, FAKE * 2, FAKE * 3, None, None, 0, FAKE * 5, None) == -5
    assert L.agent_aggregate_fwd(ctypes.byref(d), FAKE, None, FAKE * 3, None, FAKE * 4, 1 << 30,
                                 FAKE * 5 + (1 << 41), None) == -1
    assert L.agent_broadcast_fwd(ctypes.byref(d), FAKE, FAKE * 2, FAKE * 3, None, None, None, None) == -1
    d.v_residual_k = 0.5          # k*V requested but V missing
    assert L.agent_broadcast_fwd(ctypes.byref(d), FAKE, FAKE * 2, FAKE * 3, None, None, FAKE * 9 + (1 << 41),
                                 None) == -1
    assert L.agent_attn_fwd(None, FAKE, FAKE, FAKE, None, None, FAKE, 1, FAKE, None) == -1


def test_bias_tables_entry_points_validate_on_the_host():
    L = binding.lib()
    d = make_desc(4, 3, 196, 49, 64, binding.AA_BF16, (14, 14), (7, 7))
    p = aa_params()
    assert L.agent_attn_bias_tables_bytes(ctypes.byref(d), None) == 0
    assert L.agent_attn_bias_tables_bytes(ctypes.byref(d), ctypes.byref(p)) == 0          # no bias component
    p.b1_col = FAKE * 7
    one = L.agent_attn_bias_tables_bytes(ctypes.byref(d), ctypes.byref(p))
    assert one >= 3 * 64 * 196 * 4 and one % 256 == 0                                     # dense B1: H * 64 * N floats
    p.b2_row = FAKE * 8
    both = L.agent_attn_bias_tables_bytes(ctypes.byref(d), ctypes.byref(p))
    assert both > one
    # tables do not depend on the batch; fp32 problems use none
    assert L.agent_attn_bias_tables_bytes(ctypes.byref(make_desc(1, 3, 196, 49, 64, binding.AA_BF16, (14, 14))),
                                          ctypes.byref(p)) == both
    assert L.agent_attn_bias_tables_bytes(ctypes.byref(make_desc(4, 3, 196, 49, 64, binding.AA_F32, (14, 14))),
                                          ctypes.byref(p)) == 0
    # many agents: only the x direction is expanded, far below n * N values per head
    big = make_desc(1, 8, 16384, 1024, 64, binding.AA_BF16, (128, 128), (32, 32))
    p.b1_blk = FAKE * 9
    p.blk_h0 = p.blk_w0 = 7
    half = L.agent_attn_bias_tables_bytes(ctypes.byref(big), ctypes.byref(p))
    assert 0 < half < 8 * 1024 * 16384 * 4 // 8
    # prepared tables shrink the workspace by exactly their size
    w_full = binding.workspace_bytes(d, p)
    q = aa_params.from_buffer_copy(p)
    q.bias_tables = FAKE * 11
    assert w_full - binding.workspace_bytes(d, q) == L.agent_attn_bias_tables_bytes(ctypes.byref(d), ctypes.byref(p))
    # build: NULL params, bad buffer, misaligned prepared tables in a forward call
    assert L.agent_attn_bias_tables(ctypes.byref(d), None, FAKE, 1 << 30, None) == -1
    assert L.agent_attn_bias_tables(ctypes.byref(d), ctypes.byref(p), None, 1 << 30, None) == -5
    assert L.agent_attn_bias_tables(ctypes.byref(d), ctypes.byref(p), FAKE + 8, 1 << 30, None) == -5
    assert L.agent_attn_bias_tables(ctypes.byref(d), ctypes.byref(p), FAKE, 64, None) == -5
    assert L.agent_attn_bias_tables(ctypes.byref(make_desc(4, 3, 196, 49, 64, 2)), ctypes.byref(p), FAKE, 1 << 30,
                                    None) == -2                                           # bias without a grid
    q.bias_tables = FAKE * 11 + 8
    assert call_fwd(d, params=q) == -5


def test_plan_string_is_host_only():
    assert binding.plan_str(make_desc(64, 3, 196, 49, 64, binding.AA_BF16, (14, 14), (7, 7))) == "small_fused"
    assert "small_aggregate" in binding.plan_str(make_desc(32, 3, 3136, 49, 32, binding.AA_BF16, (56, 56), (7, 7)))
    assert binding.plan_str(make_desc(1, 1, 196, 49, 32, binding.AA_F32, (14, 14), (7, 7))) == "fused_f32"
    assert "generic" in binding.plan_str(make_desc(1, 1, 196, 49, 32, binding.AA_F32, (14, 14), (7, 7), n_splits=2))
    assert "generic" in binding.plan_str(make_desc(1, 1, 3136, 49, 32, binding.AA_F32, (56, 56), (7, 7)))
    assert binding.plan_str(make_desc(1, 1, 0, 49, 32, binding.AA_F32)) == ""


def test_status_strings():
    for code in range(-8, 1):
        assert binding.status_str(code) not in ("", "unknown status")
    assert binding.status_str(-99) == "unknown status"


def test_binding_has_no_fallback():
    """The binding must not import the oracle or compute anything itself."""
    src = open(os.path.join(ROOT, "paper_2312_08874_amd", "binding.py")).read()
    assert "oracle" not in src.replace("no CPU or eager fallback", "")


def test_bwd_workspace_of_the_largest_workload():
    """The recomputing backward keeps no attention matrix: for the 16384-token, 1024-agent workload its workspace
    stays below 200 MB, where the path that a module term selects needs the two n x N matrices several times over."""
    L = binding.lib()
    desc = make_desc(1, 8, 16384, 1024, 64, binding.AA_BF16, (128, 128), (32, 32))
    pure = L.agent_attn_bwd_workspace_bytes(ctypes.byref(desc), None)
    p = aa_params()
    p.b1_col = 1 << 42
    with_bias = L.agent_attn_bwd_workspace_bytes(ctypes.byref(desc), ctypes.byref(p))
    assert 0 < pure < 200e6 and with_bias > 2e9
    # fp32 problems take the other path as well
    assert L.agent_attn_bwd_workspace_bytes(ctypes.byref(make_desc(1, 8, 16384, 1024, 64, binding.AA_F32, (128, 128),
                                                                   (32, 32))), None) > 2e9


def test_bwd_rejects_bad_arguments():
    """agent_attn_bwd validates on the host before anything is launched."""
    L = binding.lib()
    G = 1 << 42      # far apart fake addresses: no overlap unless a test makes one
    desc = make_desc(2, 3, 196, 49, 32, binding.AA_BF16, (14, 14), (7, 7))
    need = L.agent_attn_bwd_workspace_bytes(ctypes.byref(desc), None)
    assert need > 0 and need % 256 == 0
    # a pure 16-bit problem keeps no attention matrix in the workspace; with a module term the reference path
    # runs: about 4*n*N + 7*N*d + 4*n*d floats per unit
    assert need < 6 * 4 * (4 * 49 * 196)
    with_bias = aa_params()
    with_bias.b1_col = 12 * G
    need_ref = L.agent_attn_bwd_workspace_bytes(ctypes.byref(desc), ctypes.byref(with_bias))
    assert need_ref >= 6 * 4 * (4 * 49 * 196 + 7 * 196 * 32 + 4 * 49 * 32)
    assert L.agent_attn_bwd_workspace_bytes(ctypes.byref(make_desc(2, 3, 196, 49, 32, 9)), None) == 0

    def call(desc=desc, Q=G, K=2 * G, V=3 * G, A=None, params=None, dO=4 * G, ws=5 * G, ws_bytes=1 << 40, dQ=7 * G,
             dK=8 * G, dV=9 * G, dA=None, grads=None):
        return L.agent_attn_bwd(ctypes.byref(desc), Q, K, V, A, None if params is None else ctypes.byref(params), dO,
                                ws, ws_bytes, dQ, dK, dV, dA, None if grads is None else ctypes.byref(grads), None)

    assert call(dO=None) == -1 and call(dQ=None) == -1 and call(K=None) == -1          # AA_ERR_NULL
    assert call(dA=10 * G) == -1                      # pooled agents: their gradient goes into dQ
    assert call(A=10 * G) == -1                       # given agents: dA is required
    assert call(ws=None) == -5 and call(ws_bytes=need - 1) == -5 and call(ws=5 * G + 8) == -5
    assert call(dQ=G) == -6 and call(dK=7 * G) == -6 and call(dV=4 * G) == -6           # AA_ERR_ALIAS
    assert call(desc=make_desc(2, 3, 196, 49, 32, binding.AA_BF16)) == -4               # no grid to pool on
    g = binding.aa_param_grads()
    g.db1_col = 11 * G
    assert call(grads=g) == -1                        # gradient of a parameter that is not there
    p = aa_params()
    p.b1_col = 12 * G
    assert call(params=p, grads=g, ws_bytes=need - 1) == -5     # accepted up to the workspace check
    # the kernels a pure 16-bit problem runs read 16 bytes at a time; with a module term the other path runs
    assert call(Q=G + 2) == -7 and call(dK=8 * G + 8) == -7                              # AA_ERR_UNSUPPORTED
    assert call(Q=G + 2, params=p, ws_bytes=need - 1) == -5
    # strided tensors are staged through dense copies: seven more [units, N, d] buffers in the workspace
    tm = make_desc(2, 3, 196, 49, 32, binding.AA_BF16, (14, 14), (7, 7), strides=(196 * 96, 32, 96),
                   out_strides=(196 * 96, 32, 96))
    need_tm = L.agent_attn_bwd_workspace_bytes(ctypes.byref(tm), None)
    assert need_tm - need == 7 * 6 * 196 * 32 * 2
    assert call(desc=tm, ws_bytes=need) == -5 and call(desc=tm, dQ=G + 64) == -6
