"""Pins of the oracle's gradients (CPU only).

The paper prints no gradient; what fixes them is the forward definition (already pinned in
test_oracle_pins.py) and calculus.  Two independent checks: central finite differences of the
forward oracle, and reverse-mode automatic differentiation of the same definition written with
library primitives (torch, fp64: softmax, matmul, adaptive_avg_pool2d, bilinear interpolate,
grouped conv2d).  A dropped term, a wrong sign, a transposed operand or a missing scale in any
gradient fails at least one of them.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

pytestmark = pytest.mark.filterwarnings("ignore")


def _rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------
# one softmax attention: finite differences and row invariants
# --------------------------------------------------------------------------
def test_softmax_attention_bwd_finite_differences(oracle):
    r = _rng(1)
    M, L, d, dv, scale = 4, 5, 3, 2, 0.7
    Qm, Km, Vm = r.normal(size=(M, d)), r.normal(size=(L, d)), r.normal(size=(L, dv))
    bias, g = r.normal(size=(M, L)), r.normal(size=(M, dv))
    dQ, dK, dV, dB = oracle.softmax_attention_bwd(Qm, Km, Vm, g, bias=bias, scale=scale)

    def loss(Qm=Qm, Km=Km, Vm=Vm, bias=bias):
        return float((oracle.softmax_attention(Qm, Km, Vm, bias=bias, scale=scale) * g).sum())

    eps = 1e-6
    for name, x, grad in (("Qm", Qm, dQ), ("Km", Km, dK), ("Vm", Vm, dV), ("bias", bias, dB)):
        num = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            num[idx] = (loss(**{name: xp}) - loss(**{name: xm})) / (2 * eps)
        assert np.abs(num - grad).max() < 1e-8, name


def test_softmax_attention_bwd_row_invariants(oracle):
    """A constant added to a score row changes nothing, so each row of dBias sums to zero; the values
    enter linearly, so dVm = W^T g with the forward's own weights."""
    r = _rng(2)
    M, L, d, dv = 6, 9, 4, 3
    Qm, Km, Vm, g = r.normal(size=(M, d)), r.normal(size=(L, d)), r.normal(size=(L, dv)), r.normal(size=(M, dv))
    _, _, dV, dB = oracle.softmax_attention_bwd(Qm, Km, Vm, g, scale=0.5)
    assert np.abs(dB.sum(axis=1)).max() < 1e-14
    _, W = oracle.softmax_attention(Qm, Km, Vm, scale=0.5, return_weights=True)
    assert np.abs(dV - W.T @ g).max() < 1e-14


# --------------------------------------------------------------------------
# whole operator against reverse-mode automatic differentiation
# --------------------------------------------------------------------------
def _torch_forward(Q, K, V, heads, grid, agent_grid, A, s1, s2, comps, dwc_w, dwc_b, vk):
    """The operator of Sec. 4.1 / 4.2 / Appendix B / C.1 from library primitives.  Tensors fp64."""
    units, N, d = Q.shape
    gh, gw = grid
    if A is None:
        ah, aw = agent_grid
        img = Q.reshape(units, gh, gw, d).permute(0, 3, 1, 2)
        A = F.adaptive_avg_pool2d(img, (ah, aw)).permute(0, 2, 3, 1).reshape(units, ah * aw, d)
    n = A.shape[1]
    hd = torch.arange(units) % heads
    S1 = s1 * A @ K.transpose(1, 2)
    S2 = s2 * Q @ A.transpose(1, 2)
    if comps is not None:
        c1, r1, b1, c2, r2, b2 = comps
        B1 = (c1[:, :, None, :] + r1[:, :, :, None] +
              F.interpolate(b1, size=(gh, gw), mode="bilinear", align_corners=False)).reshape(heads, n, N)
        B2 = (c2[:, None, :, :] + r2[:, :, None, :] +
              F.interpolate(b2.permute(0, 3, 1, 2), size=(gh, gw), mode="bilinear",
                            align_corners=False).permute(0, 2, 3, 1)).reshape(heads, N, n)
        S1 = S1 + B1[hd]
        S2 = S2 + B2[hd]
    VA = torch.softmax(S1, dim=-1) @ V
    O = torch.softmax(S2, dim=-1) @ VA
    if dwc_w is not None:
        img = V.reshape(units // heads, heads, gh, gw, d).permute(0, 1, 4, 2, 3).reshape(units // heads, heads * d, gh, gw)
        conv = F.conv2d(img, dwc_w.reshape(heads * d, 1, 3, 3), dwc_b.reshape(heads * d), padding=1, groups=heads * d)
        O = O + conv.reshape(units // heads, heads, d, gh, gw).permute(0, 1, 3, 4, 2).reshape(units, N, d)
    if vk:
        O = O + vk * V
    return O


CASES = [
    dict(name="pure-pooled", grid=(4, 6), agent_grid=(2, 3), d=5, heads=2, batch=2, module=False, given=False, vk=0.0),
    dict(name="pure-ragged-pool", grid=(5, 7), agent_grid=(2, 3), d=4, heads=1, batch=2, module=False, given=False, vk=0.0),
    dict(name="given-agents", grid=(3, 5), agent_grid=None, d=6, heads=2, batch=1, module=False, given=True, vk=0.0),
    dict(name="module-pooled", grid=(6, 4), agent_grid=(3, 2), d=4, heads=2, batch=2, module=True, given=False, vk=0.0),
    dict(name="module-given-vk", grid=(4, 4), agent_grid=None, d=3, heads=2, batch=2, module=True, given=True, vk=0.075),
    dict(name="sd-variant", grid=(4, 4), agent_grid=(2, 2), d=8, heads=1, batch=2, module=False, given=False, vk=0.075),
]


@pytest.mark.parametrize("case", CASES, ids=[c["name"] for c in CASES])
def test_agent_attn_bwd_matches_autodiff(oracle, case):
    r = _rng(10)
    gh, gw = case["grid"]
    N, d, heads = gh * gw, case["d"], case["heads"]
    units = heads * case["batch"]
    n = 5 if case["given"] else case["agent_grid"][0] * case["agent_grid"][1]
    Q, K, V, dO = (r.normal(size=(units, N, d)) for _ in range(4))
    A = r.normal(size=(units, n, d)) if case["given"] else None
    s1, s2 = d ** -0.5, (d ** -0.15 if case["name"] == "sd-variant" else d ** -0.5)
    h0, w0 = 3, 2
    comps = dwc_w = dwc_b = None
    if case["module"]:
        comps = [r.normal(size=s) * 0.5 for s in ((heads, n, gw), (heads, n, gh), (heads, n, h0, w0),
                                                   (heads, gw, n), (heads, gh, n), (heads, h0, w0, n))]
        dwc_w, dwc_b = r.normal(size=(heads, d, 3, 3)) * 0.3, r.normal(size=(heads, d)) * 0.1

    # oracle
    B1 = B2 = None
    if comps is not None:
        B1 = np.stack([oracle.bias1_dense(comps[0][h], comps[1][h], comps[2][h], n, gh, gw) for h in range(heads)])
        B2 = np.stack([oracle.bias2_dense(comps[3][h], comps[4][h], comps[5][h], n, gh, gw) for h in range(heads)])
    got = oracle.agent_attn_bwd(Q, K, V, dO, heads=heads, grid=case["grid"], agent_grid=case["agent_grid"], A=A,
                                scale1=s1, scale2=s2, B1=B1, B2=B2, dwc_w=dwc_w, dwc_b=dwc_b, v_residual_k=case["vk"])

    # automatic differentiation of the same definition
    tens = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True)
            for k, v in dict(Q=Q, K=K, V=V).items()}
    tA = torch.tensor(A, dtype=torch.float64, requires_grad=True) if A is not None else None
    tcomps = [torch.tensor(c, dtype=torch.float64, requires_grad=True) for c in comps] if comps else None
    tw = torch.tensor(dwc_w, dtype=torch.float64, requires_grad=True) if dwc_w is not None else None
    tb = torch.tensor(dwc_b, dtype=torch.float64, requires_grad=True) if dwc_b is not None else None
    O = _torch_forward(tens["Q"], tens["K"], tens["V"], heads, case["grid"], case["agent_grid"], tA, s1, s2, tcomps,
                       tw, tb, case["vk"])
    ref_fwd = oracle.agent_attn_fwd(Q, K, V, heads=heads, grid=case["grid"], agent_grid=case["agent_grid"], A=A,
                                    scale1=s1, scale2=s2, B1=B1, B2=B2, dwc_w=dwc_w, dwc_b=dwc_b,
                                    v_residual_k=case["vk"])
    assert np.abs(O.detach().numpy() - ref_fwd).max() < 1e-12      # the two forwards are the same function
    (O * torch.tensor(dO)).sum().backward()

    tol = 1e-11
    for k in ("Q", "K", "V"):
        assert np.abs(got["d" + k] - tens[k].grad.numpy()).max() < tol, k
    if A is not None:
        assert np.abs(got["dA"] - tA.grad.numpy()).max() < tol
    if comps is not None:
        for h in range(heads):
            dc1, dr1, db1 = oracle.bias1_components_bwd(got["dB1"][h], gh, gw, h0, w0)
            dc2, dr2, db2 = oracle.bias2_components_bwd(got["dB2"][h], gh, gw, h0, w0)
            for mine, ref in zip((dc1, dr1, db1, dc2, dr2, db2), tcomps):
                assert np.abs(mine - ref.grad.numpy()[h]).max() < tol
        assert np.abs(got["ddwc_w"] - tw.grad.numpy()).max() < tol
        assert np.abs(got["ddwc_b"] - tb.grad.numpy()).max() < tol


def test_agent_attn_bwd_finite_differences_end_to_end(oracle):
    """Directional derivative of the forward oracle itself (no second implementation involved)."""
    r = _rng(20)
    grid, agrid, d, heads, units = (4, 4), (2, 2), 3, 1, 2
    N = 16
    Q, K, V, dO = (r.normal(size=(units, N, d)) for _ in range(4))
    got = oracle.agent_attn_bwd(Q, K, V, dO, heads=heads, grid=grid, agent_grid=agrid, v_residual_k=0.1)
    dirs = {k: r.normal(size=(units, N, d)) for k in "QKV"}
    eps = 1e-6

    def f(t):
        return float((oracle.agent_attn_fwd(Q + t * dirs["Q"], K + t * dirs["K"], V + t * dirs["V"], heads=heads,
                                            grid=grid, agent_grid=agrid, v_residual_k=0.1) * dO).sum())
    num = (f(eps) - f(-eps)) / (2 * eps)
    ana = sum(float((got["d" + k] * dirs[k]).sum()) for k in "QKV")
    assert abs(num - ana) < 1e-7 * max(1.0, abs(ana))


def test_pooled_gradient_is_spread_evenly(oracle):
    """With pooled agents, the part of dQ that comes through A is constant inside each pooling window:
    dQ(pooled) - dQ(broadcast-only) has identical rows within a window."""
    r = _rng(30)
    grid, agrid, d = (4, 6), (2, 3), 4
    N = 24
    Q, K, V, dO = (r.normal(size=(1, N, d)) for _ in range(4))
    pooled = oracle.agent_attn_bwd(Q, K, V, dO, heads=1, grid=grid, agent_grid=agrid)
    A = oracle.pool(Q, *grid, *agrid)
    given = oracle.agent_attn_bwd(Q, K, V, dO, heads=1, grid=grid, agent_grid=agrid, A=A)
    diff = (pooled["dQ"] - given["dQ"]).reshape(4, 6, d)
    for ay in range(2):
        for ax in range(3):
            win = diff[2 * ay:2 * ay + 2, 2 * ax:2 * ax + 2].reshape(4, d)
            assert np.abs(win - win[0]).max() < 1e-14
            assert np.abs(win[0] - given["dA"][0, ay * 3 + ax] / 4.0).max() < 1e-14
