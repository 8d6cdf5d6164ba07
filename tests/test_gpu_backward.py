"""GPU parity of the backward pass (agent_attn_bwd through the C ABI) against the fp64 oracle's
gradients on the same seeded inputs.

Bar, per gradient tensor g with reference r: fp32 path max-abs <= 1e-4 * max(1, max|r|); fp16 / bf16
paths max-abs <= 1e-2 * max(1, max|r|) and relative L2 <= 5e-3, except bf16 problems with module terms or
the enlarged second scale of Appendix C.1 (see _check): 1e-2 (the former run the kernels that keep the attention matrices in memory, where the probabilities and the
score gradients are stored in bf16 before the products that give dQ, dK, dV, so a gradient chains three
operands of relative error up to 2^-9; five unit roundoffs, as for the parameter gradients below; a near
one-hot broadcast softmax - the SD variant's scale d^-0.15 together with a bias - reaches 7e-3).  Pure
16-bit problems run the kernels that recompute their score tiles and round P and dS once, as operands
of the next product.  fp32 parameter gradients relative L2 <= 1e-4 (fp32 inputs), 5e-3 (fp16 inputs) or 1e-2
(bf16 inputs): the probabilities, V_A and dV_A that feed the MFMA products are rounded to the element
type, each with a relative error of up to one unit roundoff (2^-9 for bf16, 2^-11 for fp16), and a
parameter gradient chains three such operands; the bar is five unit roundoffs for bf16, and a
single small image (no averaging over a batch) reaches 5.4e-3.

With pooled agents the GPU rounds A to the element type as its forward does, and differentiates
through that rounding as if it were the identity.  For the 16-bit types the reference is therefore
assembled from oracle pieces fed with the GPU's pooled A: the gradient for given agents, plus the
pooling gradient of dA.
"""
import dataclasses

import numpy as np
import pytest

from paper_2312_08874_amd import inputs
from tests import util

pytestmark = pytest.mark.gpu
WL = inputs.WORKLOADS


@pytest.fixture(scope="module")
def aa():
    import torch
    assert torch.cuda.is_available()
    from paper_2312_08874_amd import binding
    binding.lib()
    return binding


def _stored(t, dtype, shape):
    import torch
    a = t.reshape(shape).cpu()
    if dtype == "bf16":
        return a.view(torch.int16).numpy().view(np.uint16)
    return a.numpy()


def _check(got, ref, dtype, what, pure=False):
    """pure: a problem without module terms and with the default scales, served by the kernels that keep P and dS
    in fp32 up to the one rounding that makes them matrix operands: the bf16 bar is the forward's 5e-3 there.
    With the enlarged second scale of Appendix C.1 (d^-0.15 instead of d^-0.5: scores four times larger at d = 64)
    the broadcast softmax is peaked, dS2 = P2 o (dP2 - D2) is a small difference of larger terms, and the 2^-9
    roundings behind dP2 = dO V_A^T show (V_A as an operand, P1 as the operand of the product that gives V_A:
    6e-3 .. 7e-3 each in an fp64 emulation with one rounding switched on at a time): dQ reaches 7.4e-3 on seeded
    random problems (two-term dS2 operands did not move it), so those keep the 1e-2 of the problems with module
    terms."""
    scale = max(1.0, float(np.abs(ref).max()))
    util.assert_parity(util.to_host64(got).reshape(ref.shape), ref, dtype, what,
                       max_abs=util.TOL[dtype]["max_abs"] * scale,
                       rel_l2=1e-2 if dtype == "bf16" and not pure else None)


def _check_param(got, ref, dtype, what, floor=0.0):
    """floor: the size a sum of the same terms with random signs would have (root of the summed squares).
    A parameter gradient whose terms cancel exactly (a bias component that is constant along the softmax
    axis, e.g. the column component of a one-column grid) has a reference of 0 and is measured against it."""
    err = float(np.linalg.norm(util.to_host64(got).reshape(ref.shape) - ref))
    rel = err / max(float(np.linalg.norm(ref)), floor, 1e-300)
    assert rel <= {"f32": 1e-4, "f16": 5e-3, "bf16": 1e-2}[dtype], "%s: rel_l2 %.3e" % (what, rel)


def _run_case(aa, oracle, wl, *, given=False, module=False, blk=(3, 2), kw=None, scale_qk=1.0):
    kw = kw or {}
    t = inputs.make_qkv(wl, scale_qk=scale_qk)
    dO = inputs.make_tensor((wl.units, wl.N, wl.d), stream=wl.index * 16 + 12, dtype=wl.dtype)
    shape = (wl.batch, wl.heads, wl.N, wl.d)
    dv = {k: util.to_device(v, wl.dtype, shape) for k, v in t.items()}
    dOd = util.to_device(dO, wl.dtype, shape)
    params = inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, blk=blk, index=wl.index) if module else None
    pd = util.params_to_device(params) if module else None
    A_st = None
    if given:
        A_st = inputs.make_tensor((wl.units, wl.n, wl.d), stream=wl.index * 16 + 11, dtype=wl.dtype)
        Ad = util.to_device(A_st, wl.dtype, (wl.batch, wl.heads, wl.n, wl.d))
        got = aa.agent_attn_bwd(dv["Q"], dv["K"], dv["V"], dOd, Ad, grid=wl.grid if module else None, params=pd, **kw)
    else:
        got = aa.agent_attn_bwd(dv["Q"], dv["K"], dv["V"], dOd, grid=wl.grid, agent_grid=wl.agent_grid, params=pd, **kw)

    f64 = {k: inputs.to_float64(v, wl.dtype) for k, v in t.items()}
    B1 = B2 = None
    okw = dict(heads=wl.heads, grid=wl.grid, scale1=kw.get("scale1") or None, scale2=kw.get("scale2") or None,
               v_residual_k=kw.get("v_residual_k", 0.0))
    if module:
        B1, B2 = util.dense_biases(oracle, params, wl.heads, wl.n, wl.grid)
        okw.update(B1=B1, B2=B2, dwc_w=params["dwc_w"], dwc_b=params["dwc_b"])
    g64 = inputs.to_float64(dO, wl.dtype)
    if given:
        ref = oracle.agent_attn_bwd(f64["Q"], f64["K"], f64["V"], g64, A=inputs.to_float64(A_st, wl.dtype), **okw)
    elif wl.dtype == "f32":
        ref = oracle.agent_attn_bwd(f64["Q"], f64["K"], f64["V"], g64, agent_grid=wl.agent_grid, **okw)
    else:
        A_gpu = aa.agent_pool_fwd(dv["Q"], grid=wl.grid, agent_grid=wl.agent_grid)
        A64 = inputs.to_float64(_stored(A_gpu, wl.dtype, (wl.units, wl.n, wl.d)), wl.dtype)
        ref = oracle.agent_attn_bwd(f64["Q"], f64["K"], f64["V"], g64, A=A64, agent_grid=wl.agent_grid, **okw)
        ref["dQ"] = ref["dQ"] + oracle.pool_bwd(ref.pop("dA"), *wl.grid, *wl.agent_grid)
    for k in ("dQ", "dK", "dV") + (("dA",) if given else ()):
        _check(got[k], ref[k], wl.dtype, "%s %s" % (wl.name, k),
               pure=not module and not kw.get("scale2") and wl.d % 8 == 0 and wl.d <= 128)
    if module:
        h0, w0 = blk
        gh, gw = wl.grid
        for hd in range(wl.heads):
            c1, r1, b1 = oracle.bias1_components_bwd(ref["dB1"][hd], gh, gw, h0, w0)
            c2, r2, b2 = oracle.bias2_components_bwd(ref["dB2"][hd], gh, gw, h0, w0)
            sq = oracle.bias1_components_bwd(ref["dB1"][hd] ** 2, gh, gw, h0, w0) + \
                oracle.bias2_components_bwd(ref["dB2"][hd] ** 2, gh, gw, h0, w0)
            for (key, r), q in zip((("db1_col", c1), ("db1_row", r1), ("db1_blk", b1), ("db2_col", c2), ("db2_row", r2),
                                    ("db2_blk", b2)), sq):
                _check_param(got[key][hd], r, wl.dtype, "%s %s head %d" % (wl.name, key, hd),
                             floor=float(np.sqrt(np.abs(q).sum())))
        _check_param(got["ddwc_w"], ref["ddwc_w"], wl.dtype, wl.name + " ddwc_w")
        _check_param(got["ddwc_b"], ref["ddwc_b"], wl.dtype, wl.name + " ddwc_b")
    return got


def _wl(name, dtype, grid, agrid, d, batch=2, heads=2, index=13):
    return dataclasses.replace(WL["tiny"], name=name, batch=batch, heads=heads, grid=grid, agent_grid=agrid, d=d,
                               dtype=dtype, index=index)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("grid,agrid,d", [((14, 14), (7, 7), 32), ((13, 11), (4, 3), 24), ((1, 1), (1, 1), 8),
                                          ((9, 70), (3, 9), 72), ((20, 20), (5, 5), 64)])
def test_backward_pure_pooled(aa, oracle, grid, agrid, d, dtype):
    _run_case(aa, oracle, _wl("pure", dtype, grid, agrid, d))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_given_agents(aa, oracle, dtype):
    wl = _wl("given", dtype, (10, 13), (1, 20), 40)
    _run_case(aa, oracle, wl, given=True)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("grid,agrid,d", [((12, 10), (3, 5), 32), ((7, 9), (3, 3), 16)])
def test_backward_module_mode(aa, oracle, grid, agrid, d, dtype):
    _run_case(aa, oracle, _wl("module", dtype, grid, agrid, d), module=True)


@pytest.mark.parametrize("agrid,dtype,batch,heads", [((6, 5), "f32", 2, 1), ((6, 5), "bf16", 2, 1),
                                                     ((16, 16), "f16", 1, 2)])
def test_backward_module_mode_many_tokens(aa, oracle, agrid, dtype, batch, heads):
    """Module terms on a 132 x 128 token grid: an agent's row of score gradients takes more than 64 KB of LDS in
    the kernel that sums the bias components (opt-in path), with a batch to add up first (and, for fp32, rows that
    start off the 16-byte grid); with 256 agents a head's broadcast score gradients exceed the size up to which
    that kernel gathers them, so its three components take the one-pass-per-component kernels."""
    _run_case(aa, oracle, _wl("many_tokens", dtype, (132, 128), agrid, 16, batch=batch, heads=heads, index=33),
              module=True, blk=(4, 3))


def test_backward_module_given_agents_and_residual(aa, oracle):
    wl = _wl("module-given", "f32", (8, 8), (2, 8), 24)
    _run_case(aa, oracle, wl, given=True, module=True, kw=dict(v_residual_k=0.075, scale2=24 ** -0.15))


def test_backward_deit_shape(aa, oracle):
    """The DeiT-T shape of the benchmark, two batch elements."""
    wl = dataclasses.replace(WL["deit_t"], batch=2)
    _run_case(aa, oracle, wl)


@pytest.mark.parametrize("name,batch,heads", [("swin_t_s1", 1, 3), ("sd_latent", 1, 2), ("highres", 1, 1)])
def test_backward_workload_shapes(aa, oracle, name, batch, heads):
    """The other benchmark shapes at their real N, n and d (fewer units, so that the oracle's dense n x N matrices
    stay within seconds): every gradient element against the oracle."""
    wl = dataclasses.replace(WL[name], batch=batch, heads=heads)
    _run_case(aa, oracle, wl)


@pytest.mark.parametrize("grid,agrid,d,dtype,given", [((40, 37), (15, 10), 64, "bf16", False),
                                                      ((33, 31), (13, 21), 128, "f16", True),
                                                      ((50, 41), (9, 15), 40, "bf16", True),
                                                      ((26, 20), (14, 19), 104, "f16", False),
                                                      ((64, 48), (3, 2), 16, "bf16", False)])
def test_backward_many_agents_ragged(aa, oracle, grid, agrid, d, dtype, given):
    """Pure 16-bit problems off every tile size of the recomputing kernels: agent counts past one LDS chunk
    (128) with a ragged last chunk and a ragged last block of agents, token counts that end inside a tile
    and are cut into several ranges, head widths 16 .. 128, pooled (ragged windows) and given agents."""
    _run_case(aa, oracle, _wl("ragged", dtype, grid, agrid, d, batch=1, heads=2, index=29), given=given)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("scale_qk,given", [(4.0, True), (4.0, False), (8.0, True)])
def test_backward_peaky_softmaxes(aa, oracle, scale_qk, given, dtype):
    """Q and K four and eight times larger: both softmaxes close to one-hot, weights spread over many orders of
    magnitude, score gradients dominated by a few pairs.  Same bars."""
    _run_case(aa, oracle, _wl("peaky", dtype, (20, 18), (6, 5), 32, batch=1, heads=2, index=37), given=given,
              scale_qk=scale_qk)


@pytest.mark.parametrize("grid,agrid,d", [((12, 12), (4, 4), 32), ((40, 40), (12, 12), 64)])
def test_backward_is_deterministic_and_ignores_workspace(aa, grid, agrid, d):
    import torch
    wl = _wl("det", "bf16", grid, agrid, d)
    t = inputs.make_qkv(wl)
    shape = (wl.batch, wl.heads, wl.N, wl.d)
    dv = {k: util.to_device(v, wl.dtype, shape) for k, v in t.items()}
    dO = util.to_device(inputs.make_tensor((wl.units, wl.N, wl.d), stream=300, dtype=wl.dtype), wl.dtype, shape)
    a = aa.agent_attn_bwd(dv["Q"], dv["K"], dv["V"], dO, grid=wl.grid, agent_grid=wl.agent_grid)
    desc = aa.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, 2, wl.grid, wl.agent_grid)
    import ctypes
    need = int(aa.lib().agent_attn_bwd_workspace_bytes(ctypes.byref(desc), None))
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")
    b = aa.agent_attn_bwd(dv["Q"], dv["K"], dv["V"], dO, grid=wl.grid, agent_grid=wl.agent_grid, workspace=ws)
    for k in ("dQ", "dK", "dV"):
        assert torch.equal(a[k], b[k])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_windows_in_descriptor(aa, dtype):
    """Windows named in the descriptor (Sec. 5.5): the gradients of the image tensors are, bit for bit, those
    of the same windows handed over as a batch (a case the tests above hold against the oracle)."""
    import torch
    batch, heads, image, window, agrid, d = 2, 2, (12, 18), (6, 6), (3, 3), 24 if dtype == "f32" else 32
    (Y, X), (wh, ww) = image, window
    nwin = (Y // wh) * (X // ww)
    params = util.params_to_device(inputs.make_module_params(heads, 9, d, window, blk=(3, 2), index=21))

    def part(x):      # [B,H,Y*X,d] -> [B*windows,H,wh*ww,d]
        v = x.reshape(batch, heads, Y // wh, wh, X // ww, ww, d)
        return v.permute(0, 2, 4, 1, 3, 5, 6).reshape(batch * nwin, heads, wh * ww, d).contiguous()

    def unpart(x):
        v = x.reshape(batch, Y // wh, X // ww, heads, wh, ww, d)
        return v.permute(0, 3, 1, 4, 2, 5, 6).reshape(batch, heads, Y * X, d).contiguous()

    img = [util.to_device(inputs.make_tensor((batch * heads, Y * X, d), stream=700 + i, dtype=dtype), dtype,
                          (batch, heads, Y * X, d)) for i in range(4)]
    a = aa.agent_attn_bwd(*img, grid=image, window=window, agent_grid=agrid, params=params, v_residual_k=0.05)
    b = aa.agent_attn_bwd(*[part(x) for x in img], grid=window, agent_grid=agrid, params=params, v_residual_k=0.05)
    for k in ("dQ", "dK", "dV"):
        assert torch.equal(a[k], unpart(b[k])), k
    for k in a:
        if k not in ("dQ", "dK", "dV"):
            assert torch.equal(a[k], b[k]), k
    assert float(a["dQ"].float().abs().max()) > 0


@pytest.mark.parametrize("seed", range(36))
def test_backward_random_problems(aa, oracle, seed):
    """Seeded random shapes: both product paths (fp32 vector and MFMA, with padded score rows and ragged
    tiles), pooled and given agents, with and without the module terms and the SD-variant scalars."""
    rng = np.random.default_rng(500 + seed)
    dtype = ["f32", "f16", "bf16"][seed % 3]
    module = bool(rng.random() < 0.5)
    gh, gw = int(rng.integers(1, 25)), int(rng.integers(1, 25))
    if module and dtype != "f32":
        # a parameter gradient sums one term per token; the rounding of the 16-bit MFMA operands (relative
        # to the size of P * dP, not of the much smaller dS) only averages out over enough of them
        gh, gw = max(gh, 8), max(gw, 8)
    ah, aw = int(rng.integers(1, min(gh, 10) + 1)), int(rng.integers(1, min(gw, 10) + 1))
    d = int(rng.integers(1, 70)) if (dtype == "f32" and seed % 2) else int(rng.choice([8, 16, 24, 32, 40, 64, 72, 128]))
    wl = _wl("random%d" % seed, dtype, (gh, gw), (ah, aw), d, batch=int(rng.integers(1, 3)),
             heads=int(rng.integers(1, 4)), index=40 + seed)
    kw = dict(v_residual_k=0.075, scale2=float(d) ** -0.15) if rng.random() < 0.3 else None
    _run_case(aa, oracle, wl, given=bool(rng.random() < 0.3), module=module,
              blk=(int(rng.integers(1, 6)), int(rng.integers(1, 6))), kw=kw)


@pytest.mark.parametrize("module", [False, True])
def test_backward_replayed_from_a_graph(aa, module):
    """The backward pass allocates nothing and clears nothing with memsets: captured once, every replay gives the
    bits of the eager call on the inputs of the moment (pure: the recomputing kernels; module terms: the kernels
    that keep the matrices in memory, with their parameter gradients)."""
    import ctypes
    import torch
    wl = _wl("graph", "bf16", (24, 20), (6, 5), 32, batch=2, heads=2, index=41)
    shape = (wl.batch, wl.heads, wl.N, wl.d)
    t = [util.to_device(inputs.make_tensor((wl.units, wl.N, wl.d), stream=900 + i, dtype=wl.dtype), wl.dtype, shape)
         for i in range(4)]
    params = util.params_to_device(inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, blk=(3, 2), index=wl.index)) \
        if module else None
    kw = dict(grid=wl.grid, agent_grid=wl.agent_grid, params=params)
    desc = aa.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, 2, wl.grid, wl.agent_grid)
    need = int(aa.lib().agent_attn_bwd_workspace_bytes(ctypes.byref(desc), aa._pp(aa.make_params(params))))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        aa.agent_attn_bwd(*t, workspace=ws, stream=side, **kw)      # first call outside the capture (one-time set-up)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            got = aa.agent_attn_bwd(*t, workspace=ws, stream=side, **kw)
    torch.cuda.synchronize()
    for rep in range(3):
        for x in t:
            x.copy_(torch.roll(x, shifts=rep + 1, dims=2))
        ws.fill_(rep)
        for v in got.values():
            v.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        eager = aa.agent_attn_bwd(*t, **kw)
        for k in eager:
            assert torch.equal(got[k], eager[k]), "replay %d: %s differs from the eager call" % (rep, k)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", ["token_major", "fused_qkv"])
def test_backward_strided_layouts(aa, dtype, layout):
    """Token-major [B,N,H,d] tensors and the q / k / v slices of a fused projection [B,N,3,H,d]: the
    backward pass stages them through dense copies, so every gradient has the bits of the dense call
    and lands with the strides of its tensor."""
    import torch
    wl = _wl("strided", dtype, (9, 8), (3, 4), 32 if dtype == "bf16" else 20, batch=2, heads=3, index=71)
    t = inputs.make_qkv(wl)
    dO = inputs.make_tensor((wl.units, wl.N, wl.d), stream=wl.index * 16 + 12, dtype=wl.dtype)
    shape = (wl.batch, wl.heads, wl.N, wl.d)
    dense = {k: util.to_device(v, wl.dtype, shape) for k, v in t.items()}
    dense["dO"] = util.to_device(dO, wl.dtype, shape)
    params = util.params_to_device(inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, blk=(3, 2), index=wl.index))
    kw = dict(grid=wl.grid, agent_grid=wl.agent_grid, params=params)
    ref = aa.agent_attn_bwd(dense["Q"], dense["K"], dense["V"], dense["dO"], **kw)
    if layout == "token_major":
        view = {k: v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for k, v in dense.items()}
    else:
        fused = torch.stack([dense[k].permute(0, 2, 1, 3) for k in ("Q", "K", "V")], dim=2).contiguous()   # [B,N,3,H,d]
        view = {k: fused[:, :, i].permute(0, 2, 1, 3) for i, k in enumerate(("Q", "K", "V"))}
        view["dO"] = dense["dO"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not view["Q"].is_contiguous()
    got = aa.agent_attn_bwd(view["Q"], view["K"], view["V"], view["dO"], **kw)
    for k in ("dQ", "dK", "dV"):
        assert got[k].stride() == view["Q"].stride()
        assert torch.equal(got[k], ref[k]), k
    for k in ref:
        if k not in ("dQ", "dK", "dV"):
            assert torch.equal(got[k], ref[k]), k

