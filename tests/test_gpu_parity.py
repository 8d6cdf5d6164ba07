"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle
on the same seeded inputs.  Bar: fp32 max-abs <= 1e-4; bf16/fp16 max-abs <= 1e-2 and
relative L2 <= 5e-3 (fp32 accumulation); index-free, so no bit-exact part except
run-to-run determinism.
"""
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


def dev_qkv(wl, t, units=None):
    u = wl.units if units is None else units
    B = u // wl.heads
    return {k: util.to_device(v[:u], wl.dtype, (B, wl.heads, wl.N, wl.d)) for k, v in t.items()}


def small(wl, batch):
    """Same shape per unit, fewer batch elements (keeps the oracle to seconds)."""
    import dataclasses
    return dataclasses.replace(wl, batch=min(batch, wl.batch))


# --------------------------------------------------------------------------
# a0  pooling
# --------------------------------------------------------------------------
POOL_CASES = [("tiny", (14, 14), (7, 7), 32), ("deit", (14, 14), (7, 7), 64), ("swin", (56, 56), (7, 7), 32),
              ("sd", (64, 64), (16, 16), 40), ("hires", (128, 128), (32, 32), 64),
              ("swin9", (56, 56), (3, 3), 32), ("ragged", (13, 17), (4, 5), 24), ("identity", (6, 5), (6, 5), 8),
              ("one", (9, 9), (1, 1), 72), ("deitb81", (14, 14), (9, 9), 64)]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("name,grid,agrid,d", POOL_CASES, ids=[c[0] for c in POOL_CASES])
def test_pool(aa, oracle, name, grid, agrid, d, dtype):
    units = (2, 3)
    N = grid[0] * grid[1]
    q = inputs.make_tensor((6, N, d), stream=100, dtype=dtype)
    A = aa.agent_pool_fwd(util.to_device(q, dtype, (*units, N, d)), grid=grid, agent_grid=agrid)
    ref = oracle.pool(inputs.to_float64(q, dtype), *grid, *agrid)
    got = util.to_host64(A).reshape(ref.shape)
    half_ulp = {"f32": 2.0 ** -24, "f16": 2.0 ** -11, "bf16": 2.0 ** -8}[dtype]
    win = (-(-grid[0] // agrid[0]) + 1) * (-(-grid[1] // agrid[1]) + 1)      # tokens per window, upper bound
    # one rounding to the storage type plus fp32 accumulation over the window
    bound = np.abs(ref) * half_ulp * 1.01 + win * 4e-7 + (6e-8 if dtype == "f16" else 0.0)
    assert np.all(np.abs(got - ref) <= bound), np.abs(got - ref).max()


# --------------------------------------------------------------------------
# a1 + a1b  aggregation and split merge
# --------------------------------------------------------------------------
AGG_SHAPES = [(196, 49, 32), (196, 49, 64), (3136, 49, 32), (1000, 256, 40), (777, 130, 64), (1, 1, 8),
              (15, 9, 8), (197, 16, 72), (200, 81, 128), (2048, 1024, 64)]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("N,n,d", AGG_SHAPES)
def test_aggregate(aa, oracle, N, n, d, dtype):
    import torch
    units = 2
    a = inputs.make_tensor((units, n, d), stream=110, dtype=dtype, std=0.7)
    k = inputs.make_tensor((units, N, d), stream=111, dtype=dtype)
    v = inputs.make_tensor((units, N, d), stream=112, dtype=dtype)
    ref = np.stack([oracle.softmax_attention(inputs.to_float64(a[u], dtype), inputs.to_float64(k[u], dtype),
                                             inputs.to_float64(v[u], dtype), None, scale=d ** -0.5)
                    for u in range(units)])
    dA, dK, dV = (util.to_device(x, dtype, (1, units, x.shape[1], d)) for x in (a, k, v))
    results = []
    for S in (0, 1, 2, 3, 7):
        if S > N:
            continue
        VA = aa.agent_aggregate_fwd(dA, dK, dV, n_splits=S)
        assert VA.dtype == torch.float32
        got = util.to_host64(VA).reshape(ref.shape)
        util.assert_parity(got, ref, dtype, "aggregate N=%d n=%d d=%d S=%d" % (N, n, d, S))
        results.append(got)


def test_aggregate_peaky_and_offset(aa, oracle):
    """Scores with a large spread (running-max rescale), values with a large mean, a near one-hot row."""
    N, n, d, dtype = 1500, 49, 32, "bf16"
    a = inputs.make_tensor((1, n, d), stream=120, dtype=dtype, std=3.0)
    k = inputs.make_tensor((1, N, d), stream=121, dtype=dtype, std=3.0)
    v = inputs.make_tensor((1, N, d), stream=122, dtype=dtype, mean=10.0)
    k64 = inputs.to_float64(k, dtype)
    k64[0, 1234] = 2.0 * inputs.to_float64(a, dtype)[0, 5]
    k = inputs.to_storage(k64.astype(np.float32), dtype)
    ref = oracle.softmax_attention(inputs.to_float64(a[0], dtype), inputs.to_float64(k[0], dtype),
                                   inputs.to_float64(v[0], dtype), None, scale=d ** -0.5)
    for S in (1, 4, 0):
        VA = aa.agent_aggregate_fwd(*(util.to_device(x, dtype, (1, 1, x.shape[1], d)) for x in (a, k, v)), n_splits=S)
        # values are O(10): the absolute bar scales with them, the relative one does not
        util.assert_parity(util.to_host64(VA)[0, 0], ref, dtype, "peaky S=%d" % S, max_abs=0.1)


# --------------------------------------------------------------------------
# a2  broadcast
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("N,n,d", AGG_SHAPES)
def test_broadcast(aa, oracle, N, n, d, dtype):
    units = 2
    q = inputs.make_tensor((units, N, d), stream=130, dtype=dtype)
    a = inputs.make_tensor((units, n, d), stream=131, dtype=dtype, std=0.7)
    va = inputs.make_tensor((units, n, d), stream=132, dtype="f32")
    ref = np.stack([oracle.softmax_attention(inputs.to_float64(q[u], dtype), inputs.to_float64(a[u], dtype),
                                             va[u].astype(np.float64), None, scale=d ** -0.5) for u in range(units)])
    O = aa.agent_broadcast_fwd(util.to_device(q, dtype, (1, units, N, d)), util.to_device(a, dtype, (1, units, n, d)),
                               util.to_device(va, "f32", (1, units, n, d)))
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "broadcast N=%d n=%d d=%d" % (N, n, d))


# --------------------------------------------------------------------------
# whole path, pure mode: the five evaluation workloads
# --------------------------------------------------------------------------
@pytest.mark.parametrize("name,batch", [("tiny", 1), ("deit_t", 4), ("swin_t_s1", 1), ("sd_latent", 1)])
def test_forward_pure_elementwise(aa, oracle, name, batch):
    """Every output element, at the workload's per-unit shape with a reduced batch."""
    wl = small(WL[name], batch)
    t = inputs.make_qkv(wl)
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid)
    ref = oracle.agent_attn_fwd(*(inputs.to_float64(t[k], wl.dtype) for k in ("Q", "K", "V")), heads=wl.heads,
                                grid=wl.grid, agent_grid=wl.agent_grid)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, wl.dtype, name)


@pytest.mark.parametrize("name,n_units,n_rows", [("deit_t", 24, None), ("swin_t_s1", 6, 512), ("sd_latent", 4, 1024),
                                                 ("highres", 8, 4096)])
def test_forward_pure_full_size_sampled(aa, oracle, name, n_units, n_rows):
    """Full workload on the GPU (the launch configuration bench.py times); oracle on sampled units and rows."""
    wl = WL[name]
    t = inputs.make_qkv(wl)
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid)
    got = util.to_host64(O).reshape(wl.units, wl.N, wl.d)
    assert np.all(np.isfinite(got))
    rng = np.random.default_rng(7)
    unit_ids = sorted(rng.choice(wl.units, size=n_units, replace=False).tolist())
    rows = None if n_rows is None else np.sort(rng.choice(wl.N, size=n_rows, replace=False))
    ref = util.oracle_forward_units(oracle, wl, t, unit_ids, rows=rows)
    sel = got[unit_ids] if rows is None else got[unit_ids][:, rows]
    util.assert_parity(sel, ref, wl.dtype, name + " full size")
    # property that holds at any size (pure mode): outputs are convex combinations of V rows
    v64 = inputs.to_float64(t["V"], wl.dtype)
    slack = {"f32": 1e-5, "f16": 2e-3, "bf16": 1e-2}[wl.dtype]
    assert np.all(got <= v64.max(axis=1, keepdims=True) + slack)
    assert np.all(got >= v64.min(axis=1, keepdims=True) - slack)


def test_forward_is_deterministic(aa):
    import torch
    wl = small(WL["swin_t_s1"], 2)
    dv = dev_qkv(wl, inputs.make_qkv(wl))
    outs = [aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid) for _ in range(3)]
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("grid,agrid,d", [((9, 11), (3, 4), 24), ((14, 14), (7, 7), 32), ((12, 12), (4, 4), 64)])
def test_one_launch_fp32_kernel_is_deterministic(aa, grid, agrid, d):
    """The one-launch fp32 kernel with several MFMA waves per SIMD: same bits on every run, pooled or given agents
    (the softmax shift once depended on when a wave read its score registers)."""
    import dataclasses
    import torch
    wl = dataclasses.replace(WL["tiny"], batch=2, heads=2, grid=grid, agent_grid=agrid, d=d, index=12)
    assert aa.plan_str(aa.make_desc(wl.batch, wl.heads, wl.N, wl.n, d, 0, grid, agrid)) == "fused_f32"
    dv = dev_qkv(wl, inputs.make_qkv(wl))
    A = aa.agent_pool_fwd(dv["Q"], grid=grid, agent_grid=agrid)
    first = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=grid, agent_grid=agrid)
    first_given = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], A)
    for _ in range(12):
        assert torch.equal(first, aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=grid, agent_grid=agrid))
        assert torch.equal(first_given, aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], A))


def test_forward_ignores_workspace_contents(aa):
    import torch
    wl = small(WL["deit_t"], 2)
    dv = dev_qkv(wl, inputs.make_qkv(wl))
    desc = aa.make_desc(wl.batch, wl.heads, wl.N, wl.n, wl.d, aa.AA_BF16, wl.grid, wl.agent_grid)
    nbytes = aa.workspace_bytes(desc)
    ws_nan = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda").view(torch.uint8)
    ws_zero = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    o1 = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid, workspace=ws_nan)
    o2 = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid, workspace=ws_zero)
    assert torch.equal(o1, o2) and bool(torch.isfinite(o1.float()).all())


# --------------------------------------------------------------------------
# explicit agents (learned / external agents, Sec. 4.1)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_with_explicit_agents(aa, oracle, dtype):
    B, H, N, n, d = 2, 2, 300, 20, 48
    q, k, v = (inputs.make_tensor((B * H, N, d), stream=140 + i, dtype=dtype) for i in range(3))
    a = inputs.make_tensor((B * H, n, d), stream=143, dtype=dtype)
    O = aa.agent_attn_fwd(*(util.to_device(x, dtype, (B, H, x.shape[1], d)) for x in (q, k, v, a)))
    ref = oracle.agent_attn_fwd(*(inputs.to_float64(x, dtype) for x in (q, k, v)), heads=H,
                                A=inputs.to_float64(a, dtype))
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "explicit agents")


# --------------------------------------------------------------------------
# a3 + a4  module mode: agent bias (Appendix B) and DWC (Eq. (6)); SD variant (Appendix C.1)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("name,batch,bias_std", [("tiny", 1, 0.5), ("deit_t", 2, 0.5), ("deit_t", 2, 2.0),
                                                 ("swin_t_s1", 1, 0.5), ("sd_latent", 1, 0.5)])
def test_forward_module_mode(aa, oracle, name, batch, bias_std):
    wl = small(WL[name], batch)
    t = inputs.make_qkv(wl)
    params = inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, index=wl.index, bias_std=bias_std)
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid,
                          params=util.params_to_device(params))
    ref = util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), params=params)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, wl.dtype, name + " module")
    pure = util.oracle_forward_units(oracle, wl, t, [0])
    assert np.abs(pure[0] - ref[0]).max() > 0.05      # the module terms do change the result


@pytest.mark.parametrize("dtype,d", [("f32", 24), ("f16", 32), ("bf16", 64), ("f16", 40)])
@pytest.mark.parametrize("which", ["b1_col", "b1_row", "b1_blk", "b2_col", "b2_row", "b2_blk", "dwc_w", "dwc_w+dwc_b"])
def test_module_terms_one_at_a_time(aa, oracle, which, dtype, d):
    """Each module term alone, on every kernel family (fp32 reference kernels, small-agent MFMA with
    d = 32 / 64, large-agent MFMA with a padded head width)."""
    import dataclasses
    wl = dataclasses.replace(WL["deit_t"], batch=1, grid=(12, 10), agent_grid=(3, 5), d=d, dtype=dtype)
    t = inputs.make_qkv(wl)
    full = inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, blk=(4, 3), index=5)
    params = {k: full[k] for k in which.split("+")}
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid,
                          params=util.params_to_device(params))
    # the oracle pools in fp64; the GPU keeps its pooled agents in two element-type terms
    ref = util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), params=params)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, which,
                       max_abs=None if dtype == "f32" else 1e-2 * max(1.0, float(np.abs(ref).max())))


@pytest.mark.parametrize("dtype,d", [("f16", 32), ("bf16", 64), ("bf16", 40)])
@pytest.mark.parametrize("grid,agrid,blk", [((13, 12), (9, 9), (4, 3)), ((20, 16), (10, 13), (7, 7)),
                                            ((9, 24), (5, 13), (1, 1)), ((15, 15), (10, 13), (4, 3)),
                                            ((16, 16), (9, 9), (8, 8)), ((16, 16), (9, 9), (9, 9))])
@pytest.mark.parametrize("which", ["b1_col", "b1_row", "b1_blk", "b2_col", "b2_row", "b2_blk", "all"])
def test_module_terms_many_agents(aa, oracle, which, grid, agrid, blk, dtype, d):
    """Agent bias with more than 64 agents: the kernels read tables of the column and block components
    interpolated along x and interpolate along y themselves (grids whose width is a multiple of four;
    the (15, 15) grid takes the other route).  Token counts off the 64-token tile, agent counts off the
    16-agent tile and beyond the last 64-agent boundary, a 1 x 1 block.  Where the head width pads to 64 and the
    block grid has at most 64 cells, the aggregation takes B1's block component as two more k-steps of its score
    products (fp16 interpolation weights times fp16 block values): an 8 x 8 block fills those k-steps exactly, a
    9 x 9 block does not fit and stays on the tables."""
    import dataclasses
    wl = dataclasses.replace(WL["deit_t"], batch=1, heads=2, grid=grid, agent_grid=agrid, d=d, dtype=dtype)
    t = inputs.make_qkv(wl)
    full = inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, blk=blk, index=6)
    params = full if which == "all" else {which: full[which]}
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid,
                          params=util.params_to_device(params))
    ref = util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), params=params)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, which,
                       max_abs=1e-2 * max(1.0, float(np.abs(ref).max())))


_PREPARED_EXTRA = {"large_dense_many": dict(grid=(15, 15), agent_grid=(10, 13), d=64, dtype="bf16", heads=2),
                   "large_dense_few": dict(grid=(12, 10), agent_grid=(3, 5), d=40, dtype="f16", heads=2)}


@pytest.mark.parametrize("name,batch", [("deit_t", 2), ("swin_t_s1", 1), ("sd_latent", 1), ("large_dense_many", 2),
                                        ("large_dense_few", 2)])
def test_prepared_bias_tables(aa, name, batch):
    """Bias tables built once by agent_attn_bias_tables() and passed in aa_params give the very bits of the
    tables the forward pass builds per call (dense tables on the small-agent kernels, half-expanded ones
    on the large-agent kernels), for another batch size too; the broadcast stage, which has no workspace
    and otherwise evaluates the components per score, reads them as well."""
    import dataclasses
    import torch
    if name in _PREPARED_EXTRA:      # dense tables read by the large-agent kernels
        wl = dataclasses.replace(WL["tiny"], batch=batch, index=31, **_PREPARED_EXTRA[name])
    else:
        wl = small(WL[name], batch)
    t = inputs.make_qkv(wl)
    params = util.params_to_device(inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, index=wl.index))
    dv = dev_qkv(wl, t)
    tables = aa.agent_attn_bias_tables(params, heads=wl.heads, N=wl.N, n=wl.n, d=wl.d, dtype=dv["Q"].dtype,
                                       grid=wl.grid)
    assert tables is not None
    prepared = dict(params, bias_tables=tables)
    kw = dict(grid=wl.grid, agent_grid=wl.agent_grid)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], params=params, **kw)
    O2 = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], params=prepared, **kw)
    assert torch.equal(O, O2)
    one = {k: v[:1].contiguous() for k, v in dv.items()}          # the tables do not depend on the batch
    assert torch.equal(aa.agent_attn_fwd(one["Q"], one["K"], one["V"], params=prepared, **kw), O[:1])
    A = aa.agent_pool_fwd(dv["Q"], **kw)
    VA = aa.agent_aggregate_fwd(A, dv["K"], dv["V"], grid=wl.grid, params=params)
    assert torch.equal(VA, aa.agent_aggregate_fwd(A, dv["K"], dv["V"], grid=wl.grid, params=prepared))
    Oc = aa.agent_broadcast_fwd(dv["Q"], A, VA, dv["V"], grid=wl.grid, params=params).float()
    Ot = aa.agent_broadcast_fwd(dv["Q"], A, VA, dv["V"], grid=wl.grid, params=prepared).float()
    # two evaluation orders of the same bias: at most an output rounding step apart
    assert (Oc - Ot).abs().max().item() <= 2.0 ** -6 * max(1.0, Oc.abs().max().item())
    assert ((Oc - Ot).norm() / Oc.norm()).item() <= 2e-3


def _stored(A, wl):
    """GPU tensor of agents -> numpy array in the storage representation of inputs.to_float64."""
    import torch
    a = A.reshape(wl.units, wl.n, wl.d).cpu()
    if wl.dtype == "bf16":
        return a.view(torch.int16).numpy().view(np.uint16)
    return a.numpy()


@pytest.mark.parametrize("dtype,d", [("f32", 24), ("bf16", 32), ("f16", 40)])
def test_bias_adapted_to_more_agents(aa, oracle, dtype, d):
    """Appendix D.1 / D.2 ("Numbers of agent tokens"): bias parameters of a 7 x 7 = 49-agent model interpolated
    to 14 x 14 = 196 agents on the GPU, against the oracle's interpolation, and the forward pass with the
    adapted bias against the oracle's."""
    import dataclasses
    heads, grid, agrid, agrid2 = 2, (28, 28), (7, 7), (14, 14)
    trained = inputs.make_module_params(heads, agrid[0] * agrid[1], d, grid, blk=(4, 3), index=7)
    dev = util.params_to_device(trained)
    adapted = aa.agent_attn_resize_bias(dev, heads=heads, grid=grid, agent_grid=agrid, new_agent_grid=agrid2)
    ref_params = oracle.resize_bias_agents({k: np.asarray(v, dtype=np.float64) for k, v in trained.items()}, agrid, agrid2)
    for key in ("b1_col", "b1_row", "b1_blk", "b2_col", "b2_row", "b2_blk"):
        got = adapted[key].cpu().numpy().astype(np.float64)
        assert got.shape == ref_params[key].shape
        assert np.abs(got - ref_params[key]).max() <= 1e-6 * max(1.0, np.abs(ref_params[key]).max()), key
    assert adapted["dwc_w"] is dev["dwc_w"]
    wl = dataclasses.replace(WL["deit_t"], batch=1, heads=heads, grid=grid, agent_grid=agrid2, d=d, dtype=dtype, index=7)
    t = inputs.make_qkv(wl)
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=grid, agent_grid=agrid2, params=adapted)
    ref = util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), params=ref_params)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "bias adapted to 196 agents",
                       max_abs=None if dtype == "f32" else 1e-2 * max(1.0, float(np.abs(ref).max())))


def test_highres_module_mode_sampled(aa, oracle):
    wl = WL["highres"]
    t = inputs.make_qkv(wl)
    params = inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, index=wl.index)
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid,
                          params=util.params_to_device(params))
    rows = np.sort(np.random.default_rng(3).choice(wl.N, size=512, replace=False))
    ref = util.oracle_forward_units(oracle, wl, t, [5], rows=rows, params=params)
    util.assert_parity(util.to_host64(O).reshape(wl.units, wl.N, wl.d)[[5]][:, rows], ref, wl.dtype, "highres module")


def test_stable_diffusion_variant(aa, oracle):
    """Appendix C.1: O = sigma(QA^T) sigma(AK^T) V + k V with a larger scale on the second softmax."""
    wl = small(WL["sd_latent"], 1)
    t = inputs.make_qkv(wl)
    dv = dev_qkv(wl, t)
    kw = dict(scale2=wl.d ** -0.15, v_residual_k=0.075)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid, **kw)
    ref = oracle.agent_attn_fwd(*(inputs.to_float64(t[k], wl.dtype) for k in ("Q", "K", "V")), heads=wl.heads,
                                grid=wl.grid, agent_grid=wl.agent_grid, **kw)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, wl.dtype, "sd variant")


# --------------------------------------------------------------------------
# stress distributions and shapes off the tile grid
# --------------------------------------------------------------------------
@pytest.mark.parametrize("scale_qk,v_mean", [(4.0, 0.0), (8.0, 0.0), (1.0, 10.0)])
def test_forward_stress_distributions(aa, oracle, scale_qk, v_mean):
    """Peaky softmaxes / offset values, against the oracle's own fp64 pooling: with scores this large a
    16-bit rounding of the pooled agents alone would move the output by more than the bar, which is why
    the GPU carries them in two element-type terms.  The same problem with the agents handed in (pooled
    by the stage entry point, hence rounded to bf16) is compared with the oracle given those agents."""
    wl = small(WL["swin_t_s1"], 1)
    t = inputs.make_qkv(wl, scale_qk=scale_qk, v_mean=v_mean)
    dv = dev_qkv(wl, t)
    q64, k64, v64 = (inputs.to_float64(t[k], wl.dtype) for k in ("Q", "K", "V"))
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid)
    ref = oracle.agent_attn_fwd(q64, k64, v64, heads=wl.heads, grid=wl.grid, agent_grid=wl.agent_grid)
    # the absolute bar is stated for outputs below 1 in magnitude; a peaky softmax returns single V rows
    # (|O| up to ~4, bf16 half-ulp 2^-7 there), so it is scaled by the largest reference magnitude
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, wl.dtype, "stress x%g mean %g" % (scale_qk, v_mean),
                       max_abs=1e-2 * max(1.0, float(np.abs(ref).max())))
    A = aa.agent_pool_fwd(dv["Q"], grid=wl.grid, agent_grid=wl.agent_grid)
    O2 = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], A)
    ref2 = oracle.agent_attn_fwd(q64, k64, v64, heads=wl.heads, A=util.to_host64(A).reshape(wl.units, wl.n, wl.d))
    util.assert_parity(util.to_host64(O2).reshape(ref2.shape), ref2, wl.dtype, "stress, agents given",
                       max_abs=1e-2 * max(1.0, float(np.abs(ref2).max())))


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("f16", 40), ("bf16", 32)])
@pytest.mark.parametrize("kind", ["scaled x4", "scaled x8", "rising along tokens and agents"])
@pytest.mark.parametrize("units,grid", [((1, 2), (48, 32)), ((3, 12), (64, 32))], ids=["few blocks", "more blocks than CUs"])
def test_large_agent_kernels_growing_maxima(aa, oracle, kind, dtype, d, units, grid):
    """Many agents (the large-agent kernels) with scores that keep outgrowing the running maximum: those kernels
    compute a tile's weights with the old maximum first and fall back to a slow path (scores taken again, maximum
    raised, accumulators rescaled) only when a weight comes out too large.  Peaky inputs and inputs whose scores
    rise along the token axis (aggregation) and along the agent axis (broadcast) take that path again and again.
    The broadcast has two builds of its chunk loop: with more 256-token blocks than the chip has CUs (the second
    shape: 36 units x 8 blocks) it runs the one that fits two blocks on a CU, whose slow path is a pass of its own."""
    import dataclasses
    wl = dataclasses.replace(WL["sd_latent"], batch=units[0], heads=units[1], grid=grid, agent_grid=(16, 16), d=d,
                             dtype=dtype, index=14)
    assert "large_aggregate" in aa.plan_str(aa.make_desc(wl.batch, wl.heads, wl.N, wl.n, d, 1 if dtype == "f16" else 2,
                                                         wl.grid, wl.agent_grid))
    scale = {"scaled x4": 4.0, "scaled x8": 8.0}.get(kind, 1.0)
    t = inputs.make_qkv(wl, scale_qk=scale)
    f = {k: inputs.to_float64(v, dtype) for k, v in t.items()}
    A64 = None
    if kind.startswith("rising"):
        ramp_t = (1.0 + 5.0 * np.arange(wl.N) / wl.N)[None, :, None]
        f["K"] = f["K"] * ramp_t
        f["Q"] = f["Q"] * 2.0
        t = {k: inputs.to_storage(v, dtype) for k, v in f.items()}
        f = {k: inputs.to_float64(v, dtype) for k, v in t.items()}
        # agents handed in, growing with their index: later agent chunks of the broadcast carry the larger scores
        pooled = oracle.pool(f["Q"], *wl.grid, *wl.agent_grid)
        A_st = inputs.to_storage(pooled * (0.5 + 3.0 * np.arange(wl.n) / wl.n)[None, :, None], dtype)
        A64 = inputs.to_float64(A_st, dtype)
    dv = dev_qkv(wl, t)
    if A64 is None:
        O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid)
        ref = oracle.agent_attn_fwd(f["Q"], f["K"], f["V"], heads=wl.heads, grid=wl.grid, agent_grid=wl.agent_grid)
    else:
        O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], util.to_device(A_st, dtype, (wl.batch, wl.heads, wl.n, d)))
        ref = oracle.agent_attn_fwd(f["Q"], f["K"], f["V"], heads=wl.heads, A=A64)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "large agents, " + kind,
                       max_abs=1e-2 * max(1.0, float(np.abs(ref).max())))


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("f16", 40)])
@pytest.mark.parametrize("step", [0.25, 8.0, 40.0], ids=["inside the slack", "around the slack", "past the slack"])
def test_large_broadcast_module_mode_rising_agent_chunks(aa, oracle, step, dtype, d):
    """The broadcast kernel of the paths with module terms walks the agents in chunks of 128 and moves the
    reference of its running softmax only when a chunk's largest score passes it by more than 2^8.  Agents
    handed in whose size grows from chunk to chunk by a small, a middling and a large step take both sides of
    that test (weights above 1 kept as they are; reference raised and the accumulators rescaled)."""
    import dataclasses
    wl = dataclasses.replace(WL["sd_latent"], batch=1, heads=2, grid=(40, 32), agent_grid=(16, 32), d=d, dtype=dtype,
                             index=15)
    t = inputs.make_qkv(wl)
    f = {k: inputs.to_float64(v, dtype) for k, v in t.items()}
    pooled = oracle.pool(f["Q"], *wl.grid, *wl.agent_grid)
    pooled = pooled / np.linalg.norm(pooled, axis=-1, keepdims=True)
    qn = float(np.linalg.norm(f["Q"], axis=-1).mean())
    # the largest base-2 exponent a token sees in chunk c is about 0.4 * (1 + step * c); over the first chunk's
    # it rises by at most 1.2, by 3 to 10 at the median (up to 24), and by 14 to 50 at the median for the three steps
    grow = (1.0 + step * (np.arange(wl.n) // 128)) * np.sqrt(d) / (qn * np.log2(np.e))
    A_st = inputs.to_storage(pooled * grow[None, :, None], dtype)
    full = inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, blk=(5, 4), index=wl.index)
    params = {k: full[k] for k in ("b2_col", "b2_row", "b2_blk", "dwc_w", "dwc_b")}
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], util.to_device(A_st, dtype, (wl.batch, wl.heads, wl.n, d)),
                          grid=wl.grid, params=util.params_to_device(params))
    ref = util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), params=params, A=A_st)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "module broadcast, step %g" % step,
                       max_abs=1e-2 * max(1.0, float(np.abs(ref).max())))


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("f16", 40), ("f16", 24)])
def test_large_broadcast_two_blocks_per_cu_ragged(aa, oracle, dtype, d):
    """The broadcast build that shares a CU between two blocks (more 256-token blocks than CUs: 36 units x 8) on a
    shape off every tile: 2000 tokens (the last block and its last wave are partial), 130 agents (the last chunk
    of 64 holds two agents, the rest is padding that must be masked), ragged pooling windows."""
    import dataclasses
    wl = dataclasses.replace(WL["sd_latent"], batch=3, heads=12, grid=(50, 40), agent_grid=(13, 10), d=d, dtype=dtype,
                             index=21)
    t = inputs.make_qkv(wl)
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid)
    ref = oracle.agent_attn_fwd(*(inputs.to_float64(t[k], wl.dtype) for k in ("Q", "K", "V")), heads=wl.heads,
                                grid=wl.grid, agent_grid=wl.agent_grid)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "ragged, two blocks per CU")


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("grid,agrid,d", [((1, 1), (1, 1), 8), ((3, 5), (3, 3), 8), ((1, 197), (1, 16), 40),
                                          ((10, 20), (9, 9), 72), ((25, 8), (4, 4), 128), ((56, 56), (3, 3), 32),
                                          ((28, 28), (4, 4), 64), ((14, 14), (9, 9), 64)])
def test_forward_odd_shapes(aa, oracle, grid, agrid, d, dtype):
    import dataclasses
    wl = dataclasses.replace(WL["tiny"], batch=1, heads=2, grid=grid, agent_grid=agrid, d=d, dtype=dtype, index=9)
    t = inputs.make_qkv(wl)
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=grid, agent_grid=agrid)
    ref = oracle.agent_attn_fwd(*(inputs.to_float64(t[k], wl.dtype) for k in ("Q", "K", "V")), heads=wl.heads,
                                grid=grid, agent_grid=agrid)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "odd shape %s %s %d" % (grid, agrid, d))


# --------------------------------------------------------------------------
# the one-block-per-unit kernel: every pooling route (window rows fetched by the pooling threads
# themselves for windows of at most four tokens, pooling out of LDS otherwise, ragged windows), every
# agent tile count, given agents, and the module terms
# --------------------------------------------------------------------------
FUSED_SHAPES = [((8, 8), (4, 4), 64), ((16, 12), (8, 6), 32), ((6, 32), (6, 8), 32), ((9, 3), (3, 3), 64),
                ((13, 11), (4, 3), 32), ((18, 14), (6, 7), 64), ((14, 14), (7, 7), 32), ((2, 17), (2, 17), 64),
                ((20, 20), (4, 5), 32)]
_DT = {"f16": 1, "bf16": 2}


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("grid,agrid,d", FUSED_SHAPES)
@pytest.mark.parametrize("module", [False, True])
def test_forward_one_block_per_unit(aa, oracle, grid, agrid, d, dtype, module):
    import dataclasses
    wl = dataclasses.replace(WL["tiny"], batch=2, heads=2, grid=grid, agent_grid=agrid, d=d, dtype=dtype, index=11)
    desc = aa.make_desc(wl.batch, wl.heads, wl.N, wl.n, d, _DT[dtype], grid, agrid)
    assert aa.plan_str(desc) == "small_fused"
    t = inputs.make_qkv(wl)
    dv = dev_qkv(wl, t)
    params = inputs.make_module_params(wl.heads, wl.n, d, grid, blk=(3, 2), index=11) if module else None
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=grid, agent_grid=agrid,
                          params=util.params_to_device(params) if module else None)
    ref = util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), params=params)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "one block per unit %s %s %d" % (grid, agrid, d),
                       max_abs=1e-2 * max(1.0, float(np.abs(ref).max())))
    if not module:      # agents handed in (rounded to the element type by the pooling entry point)
        A = aa.agent_pool_fwd(dv["Q"], grid=grid, agent_grid=agrid)
        O2 = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], A)
        ref2 = util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), A=_stored(A, wl))
        util.assert_parity(util.to_host64(O2).reshape(ref2.shape), ref2, dtype, "agents given",
                           max_abs=1e-2 * max(1.0, float(np.abs(ref2).max())))


# --------------------------------------------------------------------------
# windows in the descriptor (Sec. 5.5, window-size ablation of Agent-Swin): the image tensors are handed over
# as they are; the reference is the oracle on an explicitly partitioned copy, window by window
# --------------------------------------------------------------------------
def _partition(x, heads, image, window):
    """[B*H, Y*X, d] image tensor -> [B*windows*H, wh*ww, d], units ordered (batch, window row-major, head)."""
    (Y, X), (wh, ww) = image, window
    BH, _, d = x.shape
    v = x.reshape(BH // heads, heads, Y // wh, wh, X // ww, ww, d)
    return np.ascontiguousarray(v.transpose(0, 2, 4, 1, 3, 5, 6)).reshape(-1, wh * ww, d)


def _unpartition(o, batch, heads, image, window):
    (Y, X), (wh, ww) = image, window
    v = o.reshape(batch, Y // wh, X // ww, heads, wh, ww, o.shape[-1])
    return np.ascontiguousarray(v.transpose(0, 3, 1, 4, 2, 5, 6)).reshape(batch * heads, Y * X, o.shape[-1])


WINDOW_CASES = [
    # name, image, window, agents, d, dtype, n_splits, token-major layout, kernel family the windows run on
    ("7x7 one block", (56, 56), (7, 7), (3, 3), 32, "bf16", 0, False, "small_fused"),
    ("14x14 one block", (56, 56), (14, 14), (7, 7), 32, "f16", 0, False, "small_fused"),
    ("14x14 one block, token-major", (56, 56), (14, 14), (7, 7), 64, "bf16", 0, True, "small_fused"),
    ("14x14 split", (56, 56), (14, 14), (7, 7), 32, "bf16", 2, False, "small_aggregate"),
    ("28x28 many agents", (56, 56), (28, 28), (9, 9), 32, "f16", 0, False, "large_aggregate"),
    ("28x28 many agents, token-major", (56, 28), (28, 28), (9, 9), 40, "bf16", 0, True, "large_aggregate"),
    ("14x14 fp32", (28, 42), (14, 14), (7, 7), 24, "f32", 0, False, "fused_f32"),
    ("14x14 fp32 split", (28, 42), (14, 14), (7, 7), 24, "f32", 2, False, "generic"),
    ("ragged windows fp32", (15, 20), (5, 4), (2, 3), 20, "f32", 0, True, "fused_f32"),
    ("ragged windows fp32, odd width", (15, 20), (5, 4), (2, 3), 18, "f32", 0, True, "generic"),
    ("whole image as one window", (14, 14), (14, 14), (7, 7), 32, "bf16", 0, False, "small_fused"),
]


@pytest.mark.parametrize("module", [False, True])
@pytest.mark.parametrize("name,image,window,agrid,d,dtype,n_splits,token_major,family", WINDOW_CASES,
                         ids=[c[0] for c in WINDOW_CASES])
def test_forward_windows_in_descriptor(aa, oracle, name, image, window, agrid, d, dtype, n_splits, token_major, family,
                                       module):
    import dataclasses
    import torch
    batch, heads = 2, 3
    (Y, X), (wh, ww) = image, window
    nwin = (Y // wh) * (X // ww)
    wl = dataclasses.replace(WL["tiny"], batch=batch * nwin, heads=heads, grid=window, agent_grid=agrid, d=d, dtype=dtype,
                             index=13)
    desc = aa.make_desc(batch, heads, wl.N, wl.n, d, {"f32": 0, "f16": 1, "bf16": 2}[dtype], window, agrid,
                        n_splits=n_splits, image=image)
    plan = aa.plan_str(desc)
    assert family in plan, plan
    img = {k: inputs.make_tensor((batch * heads, Y * X, d), stream=13 * 16 + 40 + i, dtype=dtype)
           for i, k in enumerate(("Q", "K", "V"))}
    t = {k: _partition(v, heads, image, window) for k, v in img.items()}
    params = inputs.make_module_params(heads, wl.n, d, window, blk=(3, 2), index=13) if module else None
    dev = {}
    for k, v in img.items():
        x = util.to_device(v, dtype, (batch, heads, Y * X, d))
        if token_major:      # [B, Y*X, H, d] in memory, handed over as a [B, H, Y*X, d] view
            x = x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
            assert not x.is_contiguous()
        dev[k] = x
    out = torch.full_like(dev["Q"], float("nan"))
    O = aa.agent_attn_fwd(dev["Q"], dev["K"], dev["V"], grid=image, window=window, agent_grid=agrid, n_splits=n_splits,
                          params=util.params_to_device(params) if module else None, out=out)
    ref = _unpartition(util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), params=params), batch, heads,
                       image, window)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "windows " + name,
                       max_abs=None if dtype == "f32" else 1e-2 * max(1.0, float(np.abs(ref).max())))
    # and what the same library gives for the partitioned copy handed over as a batch of windows (bit for bit
    # where the windows run through the very same kernels)
    part = {k: util.to_device(v, dtype, (batch * nwin, heads, wl.N, d)) for k, v in t.items()}
    O2 = aa.agent_attn_fwd(part["Q"], part["K"], part["V"], grid=window, agent_grid=agrid, n_splits=n_splits,
                           params=util.params_to_device(params) if module else None)
    got2 = _unpartition(util.to_host64(O2).reshape(-1, wl.N, d), batch, heads, image, window)
    got = util.to_host64(O).reshape(got2.shape)
    if family in ("small_fused", "fused_f32"):      # the in-place kernel may cut the tokens into fewer slices: same bar, other rounding
        util.assert_parity(got, got2, dtype, "windows in place against a batch of windows",
                           max_abs=1e-2 * max(1.0, float(np.abs(ref).max())))
    else:
        assert np.array_equal(got, got2)


@pytest.mark.parametrize("window,agrid,n_splits,dtype", [((7, 7), (3, 3), 0, "bf16"), ((14, 14), (7, 7), 2, "f16"),
                                                         ((14, 14), (9, 9), 0, "bf16"), ((7, 7), (2, 2), 0, "f32")])
def test_windows_with_given_agents_and_static_workspace(aa, oracle, window, agrid, n_splits, dtype):
    """Windows with agents handed in per (batch, window, head) -- [B, windows, H, n, d] -- on every kernel family,
    through the ordinary entry point and through the one that allocates nothing."""
    import dataclasses
    import torch
    batch, heads, image, d = 2, 2, (28, 28), 32
    (Y, X), (wh, ww) = image, window
    nwin = (Y // wh) * (X // ww)
    wl = dataclasses.replace(WL["tiny"], batch=batch * nwin, heads=heads, grid=window, agent_grid=agrid, d=d, dtype=dtype,
                             index=16)
    img = {k: inputs.make_tensor((batch * heads, Y * X, d), stream=16 * 16 + 40 + i, dtype=dtype)
           for i, k in enumerate(("Q", "K", "V"))}
    t = {k: _partition(v, heads, image, window) for k, v in img.items()}
    A_st = inputs.make_tensor((wl.units, wl.n, d), stream=16 * 16 + 11, std=0.5, dtype=dtype)      # unit order (b, window, head)
    dev = {k: util.to_device(v, dtype, (batch, heads, Y * X, d)) for k, v in img.items()}
    Ad = util.to_device(A_st, dtype, (batch * nwin, heads, wl.n, d))
    O = aa.agent_attn_fwd(dev["Q"], dev["K"], dev["V"], Ad, grid=image, window=window, n_splits=n_splits)
    ref = _unpartition(util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), A=A_st), batch, heads, image, window)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, dtype, "windows, agents given",
                       max_abs=None if dtype == "f32" else 1e-2 * max(1.0, float(np.abs(ref).max())))
    out = torch.full_like(dev["Q"], float("nan"))
    O2 = aa.agent_attn_fwd_static(dev["Q"], dev["K"], dev["V"], Ad, grid=image, window=window, n_splits=n_splits, out=out)
    assert torch.equal(O, O2)


def test_windows_descriptor_errors(aa):
    import ctypes
    lib = aa.lib()
    ok = aa.make_desc(1, 2, 49, 9, 32, 2, (7, 7), (3, 3), image=(56, 56))
    assert lib.agent_attn_workspace_bytes(ctypes.byref(ok), None) > 0
    for image in ((56, 55), (50, 56), (56, 0), (-7, 7)):      # not a whole number of windows, half given, negative
        bad = aa.make_desc(1, 2, 49, 9, 32, 2, (7, 7), (3, 3), image=image)
        assert lib.agent_attn_workspace_bytes(ctypes.byref(bad), None) == 0
    nogrid = aa.make_desc(1, 2, 49, 9, 32, 2, None, None, image=(56, 56))
    assert lib.agent_attn_workspace_bytes(ctypes.byref(nogrid), None) == 0
    # the stage entry points do not serve windows
    import torch
    Q = torch.zeros(1, 2, 56 * 56, 32, dtype=torch.bfloat16, device="cuda")
    A = torch.zeros(64, 2, 9, 32, dtype=torch.bfloat16, device="cuda")
    assert lib.agent_pool_fwd(ctypes.byref(ok), Q.data_ptr(), A.data_ptr(), None) == -7      # AA_ERR_UNSUPPORTED


# --------------------------------------------------------------------------
# the module with its projections (Sec. 4.2; the 4NC^2 of Eq. (7)): x -> q | k | v -> agent attention -> y
# --------------------------------------------------------------------------
MODULE_CASES = [
    # name, batch, heads, d, grid, window, agent grid, dtype, module terms
    ("deit-like", 2, 3, 64, (14, 14), None, (7, 7), "bf16", True),
    ("swin windows 7x7", 1, 3, 32, (28, 28), (7, 7), (3, 3), "bf16", True),
    ("latent-like, many agents", 1, 4, 40, (32, 32), None, (16, 16), "f16", False),
    ("fp32", 2, 2, 24, (10, 12), None, (5, 4), "f32", True),
    ("fp32 windows, one launch per window", 1, 2, 16, (12, 12), (6, 6), (3, 3), "f32", False),
]


@pytest.mark.parametrize("name,batch,heads,d,grid,window,agrid,dtype,module", MODULE_CASES, ids=[c[0] for c in MODULE_CASES])
def test_module_with_projections(aa, oracle, name, batch, heads, d, grid, window, agrid, dtype, module):
    C, T = heads * d, grid[0] * grid[1]
    n = agrid[0] * agrid[1]
    mk = lambda shape, stream, std: inputs.make_tensor(shape, stream=900 + stream, std=std, dtype=dtype)
    x = mk((batch, T, C), 0, 1.0)
    w_qkv, b_qkv = mk((3 * C, C), 1, C ** -0.5), mk((3 * C,), 2, 0.1)
    w_out, b_out = mk((C, C), 3, C ** -0.5), mk((C,), 4, 0.1)
    params = inputs.make_module_params(heads, n, d, window or grid, blk=(3, 2), index=15) if module else None
    dev = lambda a: util.to_device(a, dtype)
    y = aa.agent_attn_module_fwd(dev(x), dev(w_qkv), dev(b_qkv), dev(w_out), dev(b_out), heads=heads, grid=grid,
                                 agent_grid=agrid, window=window, params=util.params_to_device(params) if module else None)
    ref = util.oracle_module_forward(oracle, x, w_qkv, b_qkv, w_out, b_out, dtype, heads=heads, grid=grid,
                                     agent_grid=agrid, window=window, params=params)
    scale = max(1.0, float(np.abs(ref).max()))
    util.assert_parity(util.to_host64(y).reshape(ref.shape), ref, dtype, "module " + name,
                       max_abs=util.TOL[dtype]["max_abs"] * scale)
    # without the biases of the projections
    y2 = aa.agent_attn_module_fwd(dev(x), dev(w_qkv), None, dev(w_out), None, heads=heads, grid=grid, agent_grid=agrid,
                                  window=window, params=util.params_to_device(params) if module else None)
    ref2 = util.oracle_module_forward(oracle, x, w_qkv, None, w_out, None, dtype, heads=heads, grid=grid,
                                      agent_grid=agrid, window=window, params=params)
    util.assert_parity(util.to_host64(y2).reshape(ref2.shape), ref2, dtype, "module without projection biases " + name,
                       max_abs=util.TOL[dtype]["max_abs"] * max(1.0, float(np.abs(ref2).max())))
    assert np.abs(ref - ref2).max() > 1e-3


def test_binding_rejects_mismatched_tensors(aa):
    """The Python layer refuses tensors whose dtype, device, shape or density differ from what the descriptor
    will say (the C ABI sees only pointers), before anything is launched."""
    import torch
    Q = torch.zeros(1, 2, 64, 32, dtype=torch.bfloat16, device="cuda")
    A = torch.zeros(1, 2, 8, 32, dtype=torch.bfloat16, device="cuda")
    VA = torch.zeros(1, 2, 8, 32, dtype=torch.float32, device="cuda")
    with pytest.raises(AssertionError):
        aa.agent_attn_fwd(Q, Q.float(), Q, A)                                  # K in another dtype
    with pytest.raises(AssertionError):
        aa.agent_attn_fwd(Q, Q, Q, A.float())                                  # A in another dtype
    with pytest.raises(AssertionError):
        aa.agent_attn_fwd(Q, Q, Q, torch.zeros(1, 2, 16, 32, dtype=torch.bfloat16, device="cuda")[:, :, ::2])   # A not dense
    with pytest.raises(AssertionError):
        aa.agent_attn_fwd(Q, Q, Q, A, out=torch.zeros(1, 2, 32, 32, dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(AssertionError):
        aa.agent_broadcast_fwd(Q, A, VA.to(torch.bfloat16))                    # V_A must be fp32
    with pytest.raises(AssertionError):
        aa.agent_attn_bwd(Q, Q, Q, Q.float(), A)                               # dO in another dtype
    # a temporary workspace for a call on a side stream is allocated on that stream
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    O = aa.agent_attn_fwd(Q, Q, Q, A, stream=side)
    side.synchronize()
    assert torch.equal(O, aa.agent_attn_fwd(Q, Q, Q, A))


# --------------------------------------------------------------------------
# strided Q, K, V, out: views of token-major [B,N,H,d] tensors and of a fused [B,N,3,H,d] projection
# output must give exactly the bits of the dense call, on every kernel family
# --------------------------------------------------------------------------
STRIDED_CASES = [
    ("one-block", (14, 14), (7, 7), 64, "bf16", 3),       # one block per unit
    ("split", (40, 40), (7, 7), 32, "f16", 2),            # pool + split aggregate + broadcast
    ("large", (24, 24), (9, 9), 40, "bf16", 2),           # large-agent kernels, padded head width
    ("reference-f32", (9, 11), (3, 4), 24, "f32", 2),     # reference kernels
    ("reference-odd-stride", (9, 11), (3, 4), 20, "bf16", 3),      # strides not a multiple of 8 elements
]


@pytest.mark.parametrize("layout", ["token-major", "fused-qkv"])
@pytest.mark.parametrize("module", [False, True])
@pytest.mark.parametrize("name,grid,agrid,d,dtype,heads", STRIDED_CASES, ids=[c[0] for c in STRIDED_CASES])
def test_forward_strided_layouts(aa, name, grid, agrid, d, dtype, heads, module, layout):
    import dataclasses
    import torch
    wl = dataclasses.replace(WL["tiny"], batch=2, heads=heads, grid=grid, agent_grid=agrid, d=d, dtype=dtype, index=12)
    t = inputs.make_qkv(wl)
    dense = dev_qkv(wl, t)                                  # [B,H,N,d] contiguous
    B, H, N = wl.batch, wl.heads, wl.N
    if layout == "token-major":
        views = {k: v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for k, v in dense.items()}
    else:
        qkv = torch.stack([dense[k].permute(0, 2, 1, 3) for k in ("Q", "K", "V")], dim=2).contiguous()   # [B,N,3,H,d]
        views = {k: qkv[:, :, i].permute(0, 2, 1, 3) for i, k in enumerate(("Q", "K", "V"))}
    for k in views:
        assert not views[k].is_contiguous() and torch.equal(views[k], dense[k])
    params = None
    if module:
        params = util.params_to_device(inputs.make_module_params(H, wl.n, d, grid, blk=(3, 2), index=12))
    kw = dict(grid=grid, agent_grid=agrid, params=params)
    ref = aa.agent_attn_fwd(dense["Q"], dense["K"], dense["V"], **kw)
    # dense output from strided inputs, and a token-major output
    out_dense = torch.empty_like(dense["Q"])
    got = aa.agent_attn_fwd(views["Q"], views["K"], views["V"], out=out_dense, **kw)
    assert torch.equal(got, ref)
    out_tm = torch.full((B, N, H, d), 7.0, dtype=ref.dtype, device="cuda").permute(0, 2, 1, 3)
    got = aa.agent_attn_fwd(views["Q"], views["K"], views["V"], out=out_tm, **kw)
    assert torch.equal(got, ref)
    # stage entry points
    A = aa.agent_pool_fwd(views["Q"], grid=grid, agent_grid=agrid)
    assert torch.equal(A, aa.agent_pool_fwd(dense["Q"], grid=grid, agent_grid=agrid))
    VA = aa.agent_aggregate_fwd(A, views["K"], views["V"], grid=grid, params=params)
    assert torch.equal(VA, aa.agent_aggregate_fwd(A, dense["K"], dense["V"], grid=grid, params=params))
    O = aa.agent_broadcast_fwd(views["Q"], A, VA, views["V"], grid=grid, params=params, out=out_tm)
    assert torch.equal(O, aa.agent_broadcast_fwd(dense["Q"], A, VA, dense["V"], grid=grid, params=params))


# --------------------------------------------------------------------------
# HIP graph capture: the library allocates nothing and clears nothing with memsets, so a forward pass
# can be captured and replayed; every replay must give the bits of the eager call on the current inputs
# --------------------------------------------------------------------------
@pytest.mark.parametrize("name,batch,module", [("deit_t", 4, False), ("deit_t", 4, True), ("swin_t_s1", 2, True),
                                               ("sd_latent", 1, True), ("tiny", 1, True)])
def test_forward_replayed_from_a_graph(aa, name, batch, module):
    import torch
    wl = small(WL[name], batch)
    t = inputs.make_qkv(wl)
    dv = dev_qkv(wl, t)
    params = util.params_to_device(inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, index=wl.index)) \
        if module else None
    kw = dict(grid=wl.grid, agent_grid=wl.agent_grid, params=params)
    out = torch.empty_like(dv["Q"])
    ws = torch.empty(max(256, aa.workspace_bytes(aa._desc_from(dv["Q"], wl.n, wl.grid, wl.agent_grid),
                                                 aa.make_params(params))), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call = aa.prepare_fwd(dv["Q"], dv["K"], dv["V"], out=out, workspace=ws, stream=side, **kw)
        call()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.synchronize()
    for rep in range(4):
        # eager work and a change of the inputs between the replays
        for k in ("Q", "K", "V"):
            dv[k].copy_(torch.roll(dv[k], shifts=rep + 1, dims=2))
        ws.fill_(rep)
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        eager = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], **kw)
        assert torch.equal(out, eager), "replay %d differs from the eager call" % rep


# --------------------------------------------------------------------------
# seeded random problems over the whole admissible range of shapes: every kernel family, ragged pooling
# windows, agent counts off the tile sizes, random subsets of the module terms, the SD-variant scalars
# --------------------------------------------------------------------------
def _random_case(seed):
    import dataclasses
    rng = np.random.default_rng(1000 + seed)
    dtype = ["f32", "f16", "bf16"][seed % 3]
    gh, gw = int(rng.integers(1, 33)), int(rng.integers(1, 33))
    if seed % 4 == 0:
        gw = 4 * max(1, gw // 4)                   # widths the many-agent bias tables accept
    ah, aw = int(rng.integers(1, min(gh, 12) + 1)), int(rng.integers(1, min(gw, 12) + 1))
    if seed % 5 == 0:                              # many agents: more than one 64-agent chunk
        gh, gw = max(gh, 12), 4 * max(3, gw // 4)
        ah, aw = int(rng.integers(8, 13)), int(rng.integers(9, 13))
    if dtype == "f32":
        d = int(rng.integers(1, 80)) if seed % 2 else int(rng.choice([8, 32, 64]))
    else:                                          # half of them the widths of the small-agent kernels
        d = int(rng.choice([32, 64])) if rng.random() < 0.5 else int(rng.choice([8, 16, 24, 40, 72, 96, 128]))
    wl = dataclasses.replace(WL["tiny"], batch=int(rng.integers(1, 3)), heads=int(rng.integers(1, 4)), grid=(gh, gw),
                             agent_grid=(ah, aw), d=d, dtype=dtype, index=20 + seed)
    keys = [k for k in ("b1_col", "b1_row", "b1_blk", "b2_col", "b2_row", "b2_blk", "dwc_w") if rng.random() < 0.4]
    if "dwc_w" in keys and rng.random() < 0.5:
        keys.append("dwc_b")
    blk = (int(rng.integers(1, 8)), int(rng.integers(1, 8)))
    kw = {}
    if rng.random() < 0.3:
        kw = dict(scale2=float(d) ** -0.15, v_residual_k=0.075)
    return wl, keys, blk, kw


@pytest.mark.parametrize("seed", range(90))
def test_forward_random_problems(aa, oracle, seed):
    wl, keys, blk, kw = _random_case(seed)
    t = inputs.make_qkv(wl)
    full = inputs.make_module_params(wl.heads, wl.n, wl.d, wl.grid, blk=blk, index=wl.index)
    params = {k: full[k] for k in keys} or None
    dv = dev_qkv(wl, t)
    O = aa.agent_attn_fwd(dv["Q"], dv["K"], dv["V"], grid=wl.grid, agent_grid=wl.agent_grid,
                          params=util.params_to_device(params) if params else None, **kw)
    ref = util.oracle_forward_units(oracle, wl, t, list(range(wl.units)), params=params, **kw)
    what = "seed %d: grid %s agents %s d %d %s heads %d terms %s %s" % (seed, wl.grid, wl.agent_grid, wl.d, wl.dtype,
                                                                       wl.heads, keys, kw)
    util.assert_parity(util.to_host64(O).reshape(ref.shape), ref, wl.dtype, what,
                       max_abs=None if wl.dtype == "f32" else 1e-2 * max(1.0, float(np.abs(ref).max())))

