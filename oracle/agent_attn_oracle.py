"""ctypes front end of the fp64 CPU oracle (oracle/agent_attn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  Nothing in the product package imports it,
and it imports nothing from the product package.

All functions take and return float64 numpy arrays.  Inputs that were rounded
to bf16 / fp16 / fp32 must be converted exactly to float64 by the caller.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "agent_attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_dp = ctypes.POINTER(ctypes.c_double)
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def use_library(path: str) -> None:
    """Load a differently built copy of the oracle instead of oracle/liboracle.so.  For the mutation test
    only (tests/test_oracle_mutations.py hands the path to its pytest subprocess with --oracle-lib): it
    checks that the pins notice a mistake planted in a copy of the source."""
    global _lib
    _lib = ctypes.CDLL(path)
    _lib.oracle_num_threads.restype = ctypes.c_int


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def softmax_attention(Qm, Km, Vm, bias=None, scale=1.0, return_weights=False):
    """Sec. 3.1 Eq. (1) with the exp similarity of Sec. 3.2; bias as in Eq. (5)."""
    Qm, Km, Vm, bias = _f64(Qm), _f64(Km), _f64(Vm), _f64(bias)
    M, d = Qm.shape
    L, dv = Vm.shape
    assert Km.shape == (L, d)
    if bias is not None:
        assert bias.shape == (M, L)
    out = np.empty((M, dv), dtype=np.float64)
    w = np.empty((M, L), dtype=np.float64) if return_weights else None
    _load().oracle_softmax_attention(_p(Qm), _p(Km), _p(Vm), _p(bias), ctypes.c_double(scale),
                                     M, L, d, dv, _p(out), _p(w))
    return (out, w) if return_weights else out


def pool(Q, gh, gw, ah, aw):
    """A = Pooling(Q), Sec. 4.2.  Q [units, gh*gw, d] -> [units, ah*aw, d]."""
    Q = _f64(Q)
    units, N, d = Q.shape
    assert N == gh * gw
    A = np.empty((units, ah * aw, d), dtype=np.float64)
    _load().oracle_pool(_p(Q), units, gh, gw, ah, aw, d, _p(A))
    return A


def linear(X, W, b=None):
    """Sec. 4.2 projections: Y = X W^T + b.  X [..., K], W [O, K], b [O] or None -> [..., O]."""
    X, W = _f64(X), _f64(W)
    b = None if b is None else _f64(b)
    K, O = X.shape[-1], W.shape[0]
    assert W.shape[1] == K and (b is None or b.shape == (O,))
    rows = int(np.prod(X.shape[:-1]))
    out = np.empty(X.shape[:-1] + (O,), dtype=np.float64)
    _load().oracle_linear(_p(X), _p(W), _p(b), rows, K, O, _p(out))
    return out


def resize_bilinear(plane, h, w):
    plane = _f64(plane)
    h0, w0 = plane.shape
    out = np.empty((h, w), dtype=np.float64)
    _load().oracle_resize_bilinear(_p(plane), h0, w0, ctypes.c_size_t(1), h, w, _p(out))
    return out


def resize_agent_axis(comp, agent_grid, new_agent_grid, agents_last):
    """Appendix D.1 / D.2 ("Numbers of agent tokens"): one bias component bilinearly interpolated along
    its agent grid.  agents_last False: comp [..., n, inner...] with the agents right after the leading
    (head) axis, e.g. b1_col [H, n, w], b1_blk [H, n, h0, w0]; True: agents on the last axis, e.g.
    b2_col [H, w, n], b2_blk [H, h0, w0, n].  Returns the component for the new agent grid."""
    comp = _f64(comp)
    ah, aw = agent_grid
    ah2, aw2 = new_agent_grid
    if agents_last:
        assert comp.shape[-1] == ah * aw
        outer, inner = int(np.prod(comp.shape[:-1])), 1
        new_shape = comp.shape[:-1] + (ah2 * aw2,)
    else:
        assert comp.shape[1] == ah * aw
        outer, inner = comp.shape[0], int(np.prod(comp.shape[2:]))
        new_shape = (comp.shape[0], ah2 * aw2) + comp.shape[2:]
    out = np.empty(new_shape, dtype=np.float64)
    _load().oracle_resize_agent_axis(_p(comp), outer, ah, aw, inner, ah2, aw2, _p(out))
    return out


def resize_bias_agents(params, agent_grid, new_agent_grid):
    """All bias components of a parameter dict (keys b1_col, b1_row, b1_blk, b2_col, b2_row, b2_blk; each
    [H, ...]) adapted to a new agent grid; other entries are passed through."""
    out = dict(params)
    for key in ("b1_col", "b1_row", "b1_blk"):
        if params.get(key) is not None:
            out[key] = resize_agent_axis(params[key], agent_grid, new_agent_grid, agents_last=False)
    for key in ("b2_col", "b2_row", "b2_blk"):
        if params.get(key) is not None:
            out[key] = resize_agent_axis(params[key], agent_grid, new_agent_grid, agents_last=True)
    return out


def bias1_dense(col1, row1, blk1, n, h, w):
    """Appendix B.  col1 [n,w], row1 [n,h], blk1 [n,h0,w0] (any may be None) -> B1 [n, h*w]."""
    col1, row1, blk1 = _f64(col1), _f64(row1), _f64(blk1)
    h0, w0 = (blk1.shape[1], blk1.shape[2]) if blk1 is not None else (1, 1)
    if col1 is not None:
        assert col1.shape == (n, w)
    if row1 is not None:
        assert row1.shape == (n, h)
    if blk1 is not None:
        assert blk1.shape[0] == n
    B1 = np.empty((n, h * w), dtype=np.float64)
    _load().oracle_bias1_dense(_p(col1), _p(row1), _p(blk1), n, h, w, h0, w0, _p(B1))
    return B1


def bias2_dense(col2, row2, blk2, n, h, w):
    """Appendix B mirrored.  col2 [w,n], row2 [h,n], blk2 [h0,w0,n] -> B2 [h*w, n]."""
    col2, row2, blk2 = _f64(col2), _f64(row2), _f64(blk2)
    h0, w0 = (blk2.shape[0], blk2.shape[1]) if blk2 is not None else (1, 1)
    if col2 is not None:
        assert col2.shape == (w, n)
    if row2 is not None:
        assert row2.shape == (h, n)
    if blk2 is not None:
        assert blk2.shape[2] == n
    B2 = np.empty((h * w, n), dtype=np.float64)
    _load().oracle_bias2_dense(_p(col2), _p(row2), _p(blk2), n, h, w, h0, w0, _p(B2))
    return B2


def dwc(V, wgt, b, gh, gw):
    """DWC(V) of Eq. (6) for one unit.  V [gh*gw, d], wgt [d,3,3], b [d] or None."""
    V, wgt, b = _f64(V), _f64(wgt), _f64(b)
    N, d = V.shape
    assert N == gh * gw and wgt.shape == (d, 3, 3)
    out = np.empty((N, d), dtype=np.float64)
    _load().oracle_dwc(_p(V), _p(wgt), _p(b), gh, gw, d, _p(out))
    return out


def aggregate_partial(A, K, V, B1, scale, t0, t1):
    A, K, V, B1 = _f64(A), _f64(K), _f64(V), _f64(B1)
    n, d = A.shape
    N = K.shape[0]
    m = np.empty(n)
    l = np.empty(n)
    acc = np.empty((n, d))
    _load().oracle_aggregate_partial(_p(A), _p(K), _p(V), _p(B1), ctypes.c_double(scale),
                                     n, N, d, t0, t1, _p(m), _p(l), _p(acc))
    return m, l, acc


def merge_partials(m, l, acc):
    m, l, acc = _f64(m), _f64(l), _f64(acc)
    S, n, d = acc.shape
    VA = np.empty((n, d))
    _load().oracle_merge_partials(_p(m), _p(l), _p(acc), S, n, d, _p(VA))
    return VA


def agent_attn_fwd(Q, K, V, *, heads, grid=None, agent_grid=None, A=None, scale1=None,
                   scale2=None, B1=None, B2=None, dwc_w=None, dwc_b=None, v_residual_k=0.0,
                   return_intermediates=False):
    """Whole forward pass: pooling, aggregation, broadcast and the module terms.

    Q, K, V [units, N, d] with units = batch*heads; A [units, n, d] or None (pool Q);
    B1 [heads, n, N], B2 [heads, N, n] dense or None; dwc_w [heads, d, 3, 3],
    dwc_b [heads, d] or None.  scale defaults to d**-0.5 (Sec. 3.2).
    """
    Q, K, V, A = _f64(Q), _f64(K), _f64(V), _f64(A)
    B1, B2, dwc_w, dwc_b = _f64(B1), _f64(B2), _f64(dwc_w), _f64(dwc_b)
    units, N, d = Q.shape
    assert units % heads == 0
    gh, gw = grid if grid is not None else (1, N)
    assert gh * gw == N
    if A is not None:
        n = A.shape[1]
        ah, aw = agent_grid if agent_grid is not None else (1, n)
    else:
        ah, aw = agent_grid
        n = ah * aw
    if B1 is not None:
        assert B1.shape == (heads, n, N)
    if B2 is not None:
        assert B2.shape == (heads, N, n)
    if dwc_w is not None:
        assert dwc_w.shape == (heads, d, 3, 3)
    s1 = d ** -0.5 if scale1 is None else scale1
    s2 = d ** -0.5 if scale2 is None else scale2
    O = np.empty((units, N, d))
    A_out = np.empty((units, n, d))
    VA_out = np.empty((units, n, d))
    _load().oracle_agent_attn_fwd(_p(Q), _p(K), _p(V), _p(A), units, heads, gh, gw, ah, aw, N, n, d,
                                  ctypes.c_double(s1), ctypes.c_double(s2), _p(B1), _p(B2),
                                  _p(dwc_w), _p(dwc_b), ctypes.c_double(v_residual_k),
                                  _p(O), _p(A_out), _p(VA_out))
    if return_intermediates:
        return O, A_out, VA_out
    return O


# --------------------------------------------------------------------------
# gradients
# --------------------------------------------------------------------------
def softmax_attention_bwd(Qm, Km, Vm, g, bias=None, scale=1.0):
    """Gradient of softmax_attention for upstream g [M, dv]: (dQm, dKm, dVm, dBias)."""
    Qm, Km, Vm, g, bias = _f64(Qm), _f64(Km), _f64(Vm), _f64(g), _f64(bias)
    M, d = Qm.shape
    L, dv = Vm.shape
    dQ, dK, dV = np.empty((M, d)), np.empty((L, d)), np.empty((L, dv))
    dB = np.zeros((M, L))
    _load().oracle_softmax_attention_bwd(_p(Qm), _p(Km), _p(Vm), _p(bias), ctypes.c_double(scale), M, L, d, dv,
                                         _p(g), _p(dQ), _p(dK), _p(dV), _p(dB))
    return dQ, dK, dV, dB


def bias1_components_bwd(dB1, h, w, h0, w0):
    """Dense dB1 [n, N] of one head -> (dcol1 [n,w], drow1 [n,h], dblk1 [n,h0,w0])."""
    dB1 = _f64(dB1)
    n = dB1.shape[0]
    dcol, drow, dblk = np.empty((n, w)), np.empty((n, h)), np.empty((n, h0, w0))
    _load().oracle_bias1_components_bwd(_p(dB1), n, h, w, h0, w0, _p(dcol), _p(drow), _p(dblk))
    return dcol, drow, dblk


def bias2_components_bwd(dB2, h, w, h0, w0):
    """Dense dB2 [N, n] of one head -> (dcol2 [w,n], drow2 [h,n], dblk2 [h0,w0,n])."""
    dB2 = _f64(dB2)
    n = dB2.shape[1]
    dcol, drow, dblk = np.empty((w, n)), np.empty((h, n)), np.empty((h0, w0, n))
    _load().oracle_bias2_components_bwd(_p(dB2), n, h, w, h0, w0, _p(dcol), _p(drow), _p(dblk))
    return dcol, drow, dblk


def agent_attn_bwd(Q, K, V, dO, *, heads, grid=None, agent_grid=None, A=None, scale1=None, scale2=None,
                   B1=None, B2=None, dwc_w=None, dwc_b=None, v_residual_k=0.0):
    """Gradient of agent_attn_fwd for upstream dO [units, N, d].

    Returns a dict: dQ, dK, dV [units,N,d]; dA [units,n,d] when A is given; dB1 [heads,n,N] /
    dB2 [heads,N,n] (dense, summed over the batch) when the bias is given; ddwc_w, ddwc_b when
    dwc_w is given.
    """
    Q, K, V, A, dO = _f64(Q), _f64(K), _f64(V), _f64(A), _f64(dO)
    B1, B2, dwc_w, dwc_b = _f64(B1), _f64(B2), _f64(dwc_w), _f64(dwc_b)
    units, N, d = Q.shape
    gh, gw = grid if grid is not None else (1, N)
    if A is not None:
        n = A.shape[1]
        ah, aw = agent_grid if agent_grid is not None else (1, n)
    else:
        ah, aw = agent_grid
        n = ah * aw
    s1 = d ** -0.5 if scale1 is None else scale1
    s2 = d ** -0.5 if scale2 is None else scale2
    out = {"dQ": np.empty((units, N, d)), "dK": np.empty((units, N, d)), "dV": np.empty((units, N, d))}
    dA = np.empty((units, n, d)) if A is not None else None
    dB1 = np.empty((heads, n, N)) if B1 is not None else None
    dB2 = np.empty((heads, N, n)) if B2 is not None else None
    dw = np.empty((heads, d, 3, 3)) if dwc_w is not None else None
    db = np.empty((heads, d)) if dwc_w is not None else None
    _load().oracle_agent_attn_bwd(_p(Q), _p(K), _p(V), _p(A), units, heads, gh, gw, ah, aw, N, n, d,
                                  ctypes.c_double(s1), ctypes.c_double(s2), _p(B1), _p(B2), _p(dwc_w), _p(dwc_b),
                                  ctypes.c_double(v_residual_k), _p(dO), _p(out["dQ"]), _p(out["dK"]),
                                  _p(out["dV"]), _p(dA), _p(dB1), _p(dB2), _p(dw), _p(db))
    for k, v in (("dA", dA), ("dB1", dB1), ("dB2", dB2), ("ddwc_w", dw), ("ddwc_b", db)):
        if v is not None:
            out[k] = v
    return out


def pool_bwd(dA, gh, gw, ah, aw):
    """Gradient of pool: dA [units, n, d] -> dQ [units, N, d]."""
    dA = _f64(dA)
    units, n, d = dA.shape
    dQ = np.zeros((units, gh * gw, d))
    for u in range(units):
        _load().oracle_pool_bwd(_p(dA[u]), gh, gw, ah, aw, d, _p(dQ[u]))
    return dQ
