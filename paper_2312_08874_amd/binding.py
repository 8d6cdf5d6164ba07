"""Thin Python binding of the C-ABI library (include/agent_attn.h).

Argument marshalling only: every step of the forward pass runs in the HIP
kernels of libagent_attn.so.  torch is used for device memory and streams.
There is no CPU or eager fallback: if the library is missing the import of any
entry point raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libagent_attn.so")

AA_F32, AA_F16, AA_BF16 = 0, 1, 2
AA_OK = 0
STATUS_NAMES = {0: "AA_OK", -1: "AA_ERR_NULL", -2: "AA_ERR_SHAPE", -3: "AA_ERR_DTYPE", -4: "AA_ERR_POOL",
                -5: "AA_ERR_WORKSPACE", -6: "AA_ERR_ALIAS", -7: "AA_ERR_UNSUPPORTED", -8: "AA_ERR_HIP"}


class aa_desc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("N", ctypes.c_int32), ("n", ctypes.c_int32), ("d", ctypes.c_int32),
                ("grid_h", ctypes.c_int32), ("grid_w", ctypes.c_int32),
                ("agent_h", ctypes.c_int32), ("agent_w", ctypes.c_int32),
                ("dtype", ctypes.c_int32),
                ("scale1", ctypes.c_float), ("scale2", ctypes.c_float),
                ("v_residual_k", ctypes.c_float),
                ("n_splits", ctypes.c_int32),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
                ("out_stride_b", ctypes.c_int64), ("out_stride_h", ctypes.c_int64), ("out_stride_n", ctypes.c_int64),
                ("image_h", ctypes.c_int32), ("image_w", ctypes.c_int32)]


class aa_params(ctypes.Structure):
    _fields_ = [("b1_col", ctypes.c_void_p), ("b1_row", ctypes.c_void_p), ("b1_blk", ctypes.c_void_p),
                ("b2_col", ctypes.c_void_p), ("b2_row", ctypes.c_void_p), ("b2_blk", ctypes.c_void_p),
                ("blk_h0", ctypes.c_int32), ("blk_w0", ctypes.c_int32),
                ("dwc_w", ctypes.c_void_p), ("dwc_b", ctypes.c_void_p), ("bias_tables", ctypes.c_void_p)]


class aa_projections(ctypes.Structure):
    _fields_ = [("w_qkv", ctypes.c_void_p), ("b_qkv", ctypes.c_void_p), ("w_out", ctypes.c_void_p),
                ("b_out", ctypes.c_void_p)]


class aa_kernel_time(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("ms", ctypes.c_float)]


class aa_param_grads(ctypes.Structure):
    _fields_ = [("db1_col", ctypes.c_void_p), ("db1_row", ctypes.c_void_p), ("db1_blk", ctypes.c_void_p),
                ("db2_col", ctypes.c_void_p), ("db2_row", ctypes.c_void_p), ("db2_blk", ctypes.c_void_p),
                ("ddwc_w", ctypes.c_void_p), ("ddwc_b", ctypes.c_void_p)]


EXPORTS = ("agent_attn_workspace_bytes", "agent_attn_fwd", "agent_pool_fwd", "agent_aggregate_fwd",
           "agent_broadcast_fwd", "agent_attn_flops", "agent_attn_status_str", "agent_attn_plan_str",
           "agent_attn_bwd_workspace_bytes", "agent_attn_bwd", "agent_attn_bias_tables_bytes",
           "agent_attn_bias_tables", "agent_attn_fwd_static", "agent_attn_static_scratch_bytes",
           "agent_attn_fwd_timed", "agent_attn_resize_bias", "agent_attn_module_workspace_bytes",
           "agent_attn_module_fwd")

_lib = None


class AgentAttnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%s)" % (where, STATUS_NAMES.get(status, status), status_str(status)))


def lib():
    """Load libagent_attn.so (built in-tree by __graft_entry__.build()); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("HIP library %s not built; run `python -c 'import __graft_entry__ as g; g.build()'`"
                              % LIB_PATH)
        # torch ships a HIP runtime of its own: with torch loaded first the library binds to that instance, the one
        # whose allocator hands out the tensors.  Loaded the other way round the process holds two runtimes, and
        # pointers of one mean nothing to the other (every launch fails with AA_ERR_HIP).
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, dp, pp = ctypes.c_void_p, ctypes.POINTER(aa_desc), ctypes.POINTER(aa_params)
        L.agent_attn_workspace_bytes.restype = ctypes.c_size_t
        L.agent_attn_workspace_bytes.argtypes = [dp, pp]
        L.agent_attn_flops.restype = ctypes.c_uint64
        L.agent_attn_flops.argtypes = [dp]
        L.agent_attn_fwd.restype = ctypes.c_int
        L.agent_attn_fwd.argtypes = [dp, vp, vp, vp, vp, pp, vp, ctypes.c_size_t, vp, vp]
        L.agent_attn_fwd_static.restype = ctypes.c_int
        L.agent_attn_fwd_static.argtypes = [dp, vp, vp, vp, vp, pp, vp, vp]
        L.agent_attn_static_scratch_bytes.restype = ctypes.c_size_t
        L.agent_attn_static_scratch_bytes.argtypes = []
        L.agent_attn_fwd_timed.restype = ctypes.c_int
        L.agent_attn_fwd_timed.argtypes = [dp, vp, vp, vp, vp, pp, vp, ctypes.c_size_t, vp, vp,
                                           ctypes.POINTER(aa_kernel_time), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.agent_attn_resize_bias.restype = ctypes.c_int
        L.agent_attn_resize_bias.argtypes = [ctypes.c_int32] * 7 + [pp, pp, vp]
        L.agent_attn_module_workspace_bytes.restype = ctypes.c_size_t
        L.agent_attn_module_workspace_bytes.argtypes = [dp, pp]
        L.agent_attn_module_fwd.restype = ctypes.c_int
        L.agent_attn_module_fwd.argtypes = [dp, vp, ctypes.POINTER(aa_projections), pp, vp, ctypes.c_size_t, vp, vp]
        L.agent_pool_fwd.restype = ctypes.c_int
        L.agent_pool_fwd.argtypes = [dp, vp, vp, vp]
        L.agent_aggregate_fwd.restype = ctypes.c_int
        L.agent_aggregate_fwd.argtypes = [dp, vp, vp, vp, pp, vp, ctypes.c_size_t, vp, vp]
        L.agent_broadcast_fwd.restype = ctypes.c_int
        L.agent_broadcast_fwd.argtypes = [dp, vp, vp, vp, vp, pp, vp, vp]
        L.agent_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.agent_attn_bwd_workspace_bytes.argtypes = [dp, pp]
        L.agent_attn_bwd.restype = ctypes.c_int
        L.agent_attn_bwd.argtypes = [dp, vp, vp, vp, vp, pp, vp, vp, ctypes.c_size_t, vp, vp, vp, vp,
                                     ctypes.POINTER(aa_param_grads), vp]
        L.agent_attn_bias_tables_bytes.restype = ctypes.c_size_t
        L.agent_attn_bias_tables_bytes.argtypes = [dp, pp]
        L.agent_attn_bias_tables.restype = ctypes.c_int
        L.agent_attn_bias_tables.argtypes = [dp, pp, vp, ctypes.c_size_t, vp]
        L.agent_attn_plan_str.restype = ctypes.c_size_t
        L.agent_attn_plan_str.argtypes = [dp, ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
        L.agent_attn_status_str.restype = ctypes.c_char_p
        L.agent_attn_status_str.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().agent_attn_status_str(int(status)).decode()


def _dtype_code(t):
    import torch
    return {torch.float32: AA_F32, torch.float16: AA_F16, torch.bfloat16: AA_BF16}[t.dtype]


def make_desc(batch, heads, N, n, d, dtype, grid=None, agent_grid=None, scale1=0.0, scale2=0.0,
              v_residual_k=0.0, n_splits=0, strides=(0, 0, 0), out_strides=(0, 0, 0), image=None) -> aa_desc:
    """strides / out_strides: (batch, head, token) element strides of Q, K, V / of out; zeros = dense.
    image: (image_h, image_w) when the tensors are images cut into grid-sized windows (N = one window)."""
    gh, gw = grid if grid is not None else (0, 0)
    ah, aw = agent_grid if agent_grid is not None else (0, 0)
    ih, iw = image if image is not None else (0, 0)
    return aa_desc(batch, heads, N, n, d, gh, gw, ah, aw, dtype, scale1, scale2, v_residual_k, n_splits,
                   *[int(x) for x in strides], *[int(x) for x in out_strides], ih, iw)


def make_params(params: dict | None):
    """dict of torch fp32 device tensors (keys as in aa_params; 'bias_tables': the uint8 tensor that
    agent_attn_bias_tables() returned for these components) -> aa_params or None."""
    if not params:
        return None
    p = aa_params()
    if params.get("bias_tables") is not None:
        assert params["bias_tables"].is_cuda and str(params["bias_tables"].dtype) == "torch.uint8"
        p.bias_tables = params["bias_tables"].data_ptr()
    h0 = w0 = 0
    for key in ("b1_col", "b1_row", "b1_blk", "b2_col", "b2_row", "b2_blk", "dwc_w", "dwc_b"):
        t = params.get(key)
        if t is not None:
            assert t.is_cuda and t.is_contiguous() and str(t.dtype) == "torch.float32", key
            setattr(p, key, t.data_ptr())
    if params.get("b1_blk") is not None:
        h0, w0 = params["b1_blk"].shape[-2:]
    if params.get("b2_blk") is not None:
        h0b, w0b = params["b2_blk"].shape[-3:-1]
        assert (h0, w0) in ((0, 0), (h0b, w0b)), "b1_blk and b2_blk must share blk_h0 x blk_w0"
        h0, w0 = h0b, w0b
    p.blk_h0, p.blk_w0 = h0, w0
    return p


def _pp(p):
    return ctypes.byref(p) if p is not None else None


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _check(status, where):
    if status != AA_OK:
        raise AgentAttnError(status, where)


def workspace_bytes(desc: aa_desc, params: aa_params | None = None) -> int:
    return int(lib().agent_attn_workspace_bytes(ctypes.byref(desc), _pp(params)))


def agent_attn_bias_tables(params: dict, *, heads, N, n, d, dtype, grid, out=None, stream=None):
    """Agent-bias tables for problems of this shape (dtype: torch dtype of Q), built once from the bias
    components in `params`; returns a uint8 device tensor to pass on as params['bias_tables'], or None
    when such problems use no tables."""
    import torch
    code = {torch.float32: AA_F32, torch.float16: AA_F16, torch.bfloat16: AA_BF16}[dtype]
    desc = make_desc(1, heads, N, n, d, code, grid)
    p = make_params({k: v for k, v in params.items() if k != "bias_tables"})
    need = int(lib().agent_attn_bias_tables_bytes(ctypes.byref(desc), _pp(p)))
    if need == 0:
        return None
    if out is None:
        out = torch.empty(need, dtype=torch.uint8, device="cuda")
    _check(lib().agent_attn_bias_tables(ctypes.byref(desc), _pp(p), out.data_ptr(), out.numel(), _stream(stream)),
           "agent_attn_bias_tables")
    return out


def plan_str(desc: aa_desc, agents_given: bool = False) -> str:
    buf = ctypes.create_string_buffer(256)
    lib().agent_attn_plan_str(ctypes.byref(desc), int(agents_given), buf, 256)
    return buf.value.decode()


def flops(desc: aa_desc) -> int:
    return int(lib().agent_attn_flops(ctypes.byref(desc)))


def _strides_of(t):
    """(batch, head, token) element strides of a [B,H,N,d] tensor (view); zeros when it is dense."""
    assert t.is_cuda and t.dim() == 4 and (t.stride(3) == 1 or t.shape[3] == 1), "channels must be contiguous"
    return (0, 0, 0) if t.is_contiguous() else (t.stride(0), t.stride(1), t.stride(2))


def _desc_from(Q, n, grid, agent_grid, same=(), out=None, **kw):
    """Descriptor for token tensors shaped like Q.  `same`: further inputs that must share Q's strides
    (K, V); `out`: the output tensor, which may have strides of its own."""
    B, H, N, d = Q.shape
    st = _strides_of(Q)
    for t in same:
        assert t is None or (tuple(t.shape) == tuple(Q.shape) and _strides_of(t) == st), \
            "Q, K, V must share one shape and one set of strides"
        assert t is None or (t.dtype == Q.dtype and t.device == Q.device), "Q, K, V must share one dtype and one device"
    if out is not None:
        assert tuple(out.shape) == tuple(Q.shape) and out.dtype == Q.dtype and out.device == Q.device, \
            "out / dO must have the shape, dtype and device of Q"
    ost = _strides_of(out) if out is not None else (0, 0, 0)
    window = kw.pop("window", None)
    if window is not None:      # Q is the whole image [B,H,grid_h*grid_w,d]; the attention runs per window
        assert grid is not None and grid[0] * grid[1] == N and grid[0] % window[0] == 0 and grid[1] % window[1] == 0
        return make_desc(B, H, window[0] * window[1], n, d, _dtype_code(Q), window, agent_grid, strides=st,
                         out_strides=ost, image=grid, **kw)
    return make_desc(B, H, N, n, d, _dtype_code(Q), grid, agent_grid, strides=st, out_strides=ost, **kw)


def _workspace(desc, params, workspace, stream=None, device=None):
    """The caller's workspace, or a temporary one.  A temporary is allocated on the stream the kernels run on, so
    that the caching allocator does not hand its memory to other work before they are done with it."""
    import torch
    need = workspace_bytes(desc, params)
    if workspace is None:
        workspace = _alloc_bytes(max(need, 256), stream, device)
    else:
        assert workspace.is_cuda and workspace.is_contiguous() and (device is None or workspace.device == device)
    return workspace, need


def _alloc_bytes(nbytes, stream, device):
    import torch
    device = "cuda" if device is None else device
    if stream is None:
        return torch.empty(nbytes, dtype=torch.uint8, device=device)
    with torch.cuda.stream(stream):
        return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _check_agents(A, Q, n, what="A", dtype=None):
    """A / VA: dense [B', H, n, d] (B' = batch, or batch * windows) in Q's dtype (or `dtype`) on Q's device."""
    if A is None:
        return
    assert A.is_cuda and A.device == Q.device and A.dtype == (Q.dtype if dtype is None else dtype), \
        what + " must be on Q's device in the expected dtype"
    assert A.dim() == 4 and A.is_contiguous() and A.shape[1] == Q.shape[1] and A.shape[2] == n and \
        A.shape[3] == Q.shape[3], what + " must be a dense [B,H,n,d] tensor"


def agent_attn_fwd(Q, K, V, A=None, *, grid=None, agent_grid=None, params: dict | None = None, scale1=0.0,
                   scale2=0.0, v_residual_k=0.0, n_splits=0, window=None, out=None, workspace=None, stream=None):
    """O = agent attention of Q, K, V [B,H,N,d] (device tensors).  A None: pool Q onto agent_grid.
    window=(wh, ww): the tensors are grid-sized images and the attention (pooling, bias, DWC included) runs
    inside each wh x ww window on its own; agent_grid and params then describe one window, a given A is
    [B, windows, H, n, d]."""
    import torch
    n = A.shape[2] if A is not None else agent_grid[0] * agent_grid[1]
    if out is None:
        out = torch.empty_like(Q)      # keeps Q's (possibly permuted) layout
    desc = _desc_from(Q, n, grid, agent_grid, same=(K, V), out=out, scale1=scale1, scale2=scale2,
                      v_residual_k=v_residual_k, n_splits=n_splits, window=window)
    p = make_params(params)
    _check_agents(A, Q, n)
    workspace, need = _workspace(desc, p, workspace, stream, Q.device)
    st = lib().agent_attn_fwd(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(A), _pp(p),
                              workspace.data_ptr(), workspace.numel() * workspace.element_size(), out.data_ptr(),
                              _stream(stream))
    _check(st, "agent_attn_fwd")
    return out


def agent_attn_fwd_static(Q, K, V, A=None, *, grid=None, agent_grid=None, params: dict | None = None, scale1=0.0,
                          scale2=0.0, v_residual_k=0.0, n_splits=0, window=None, out, stream=None):
    """agent_attn_fwd on the library's own static workspace: allocates nothing (`out` is the caller's)."""
    n = A.shape[2] if A is not None else agent_grid[0] * agent_grid[1]
    desc = _desc_from(Q, n, grid, agent_grid, same=(K, V), out=out, scale1=scale1, scale2=scale2,
                      v_residual_k=v_residual_k, n_splits=n_splits, window=window)
    p = make_params(params)
    _check_agents(A, Q, n)
    st = lib().agent_attn_fwd_static(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(A), _pp(p),
                                     out.data_ptr(), _stream(stream))
    _check(st, "agent_attn_fwd_static")
    return out


def agent_attn_fwd_timed(Q, K, V, A=None, *, grid=None, agent_grid=None, params: dict | None = None, scale1=0.0,
                         scale2=0.0, v_residual_k=0.0, n_splits=0, window=None, out, workspace, stream=None):
    """agent_attn_fwd with each kernel launch timed by HIP events on the launch stream; blocks until the
    pass is done.  Returns [(launcher name, milliseconds), ...] in launch order."""
    n = A.shape[2] if A is not None else agent_grid[0] * agent_grid[1]
    desc = _desc_from(Q, n, grid, agent_grid, same=(K, V), out=out, scale1=scale1, scale2=scale2,
                      v_residual_k=v_residual_k, n_splits=n_splits, window=window)
    p = make_params(params)
    _check_agents(A, Q, n)
    times = (aa_kernel_time * 16)()
    count = ctypes.c_int(0)
    st = lib().agent_attn_fwd_timed(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(A), _pp(p),
                                    workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                    out.data_ptr(), _stream(stream), times, 16, ctypes.byref(count))
    _check(st, "agent_attn_fwd_timed")
    return [(times[i].name.decode(), float(times[i].ms)) for i in range(count.value)]


def agent_attn_resize_bias(params: dict, *, heads, grid, agent_grid, new_agent_grid, stream=None) -> dict:
    """Bias components of `params` adapted to new_agent_grid (Appendix D.1 / D.2); returns a new dict in which
    they are replaced by freshly allocated tensors and every other entry (DWC) is passed through."""
    import torch
    n2 = new_agent_grid[0] * new_agent_grid[1]
    out = {k: v for k, v in params.items() if k != "bias_tables"}
    for key in ("b1_col", "b1_row", "b1_blk"):
        if params.get(key) is not None:
            t = params[key]
            out[key] = torch.empty((t.shape[0], n2) + tuple(t.shape[2:]), dtype=torch.float32, device=t.device)
    for key in ("b2_col", "b2_row", "b2_blk"):
        if params.get(key) is not None:
            t = params[key]
            out[key] = torch.empty(tuple(t.shape[:-1]) + (n2,), dtype=torch.float32, device=t.device)
    bias_keys = ("b1_col", "b1_row", "b1_blk", "b2_col", "b2_row", "b2_blk")
    src = make_params({k: params[k] for k in bias_keys if params.get(k) is not None})
    dst = make_params({k: out[k] for k in bias_keys if params.get(k) is not None})
    if src is None:
        return out
    st = lib().agent_attn_resize_bias(heads, grid[0], grid[1], agent_grid[0], agent_grid[1], new_agent_grid[0],
                                      new_agent_grid[1], _pp(src), _pp(dst), _stream(stream))
    _check(st, "agent_attn_resize_bias")
    return out


def agent_attn_module_fwd(x, w_qkv, b_qkv, w_out, b_out, *, heads, grid, agent_grid, window=None,
                          params: dict | None = None, scale1=0.0, scale2=0.0, v_residual_k=0.0, n_splits=0, out=None,
                          workspace=None, stream=None):
    """The module with its projections (Sec. 4.2): y = (agent attention of the q, k, v slices of x Wqkv^T + bqkv)
    Wout^T + bout.  x [B, T, C] with C = heads * d and T = grid_h * grid_w tokens; weights [3C, C] and [C, C], biases
    [3C], [C] or None, all in x's dtype on x's device.  window=(wh, ww): attention per window of the grid."""
    import torch
    B, T, C = x.shape
    assert x.is_cuda and x.is_contiguous() and C % heads == 0 and grid[0] * grid[1] == T
    d = C // heads
    for t, shape in ((w_qkv, (3 * C, C)), (b_qkv, (3 * C,)), (w_out, (C, C)), (b_out, (C,))):
        assert t is None or (t.is_cuda and t.device == x.device and t.dtype == x.dtype and t.is_contiguous() and
                             tuple(t.shape) == shape), "projection parameters must be dense, in x's dtype, on x's device"
    assert w_qkv is not None and w_out is not None
    if out is None:
        out = torch.empty_like(x)
    assert tuple(out.shape) == tuple(x.shape) and out.dtype == x.dtype and out.device == x.device and out.is_contiguous()
    n = agent_grid[0] * agent_grid[1]
    if window is not None:
        assert grid[0] % window[0] == 0 and grid[1] % window[1] == 0
        desc = make_desc(B, heads, window[0] * window[1], n, d, _dtype_code(x), window, agent_grid, scale1, scale2,
                         v_residual_k, n_splits, image=grid)
    else:
        desc = make_desc(B, heads, T, n, d, _dtype_code(x), grid, agent_grid, scale1, scale2, v_residual_k, n_splits)
    p = make_params(params)
    need = int(lib().agent_attn_module_workspace_bytes(ctypes.byref(desc), _pp(p)))
    if workspace is None:
        workspace = _alloc_bytes(max(need, 256), stream, x.device)
    proj = aa_projections(w_qkv.data_ptr(), _ptr(b_qkv), w_out.data_ptr(), _ptr(b_out))
    st = lib().agent_attn_module_fwd(ctypes.byref(desc), x.data_ptr(), ctypes.byref(proj), _pp(p), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), out.data_ptr(), _stream(stream))
    _check(st, "agent_attn_module_fwd")
    return out


def static_scratch_bytes() -> int:
    return int(lib().agent_attn_static_scratch_bytes())


def agent_attn_bwd(Q, K, V, dO, A=None, *, grid=None, agent_grid=None, params: dict | None = None, scale1=0.0,
                   scale2=0.0, v_residual_k=0.0, want_param_grads=True, window=None, workspace=None, stream=None):
    """Gradients of agent_attn_fwd for upstream dO.  Returns a dict: dQ, dK, dV (shape and type of Q),
    dA when A is given, and, for every module parameter present in `params` (want_param_grads), its
    fp32 gradient under the parameter's own name prefixed with "d" (db1_col, ..., ddwc_w, ddwc_b)."""
    import torch
    n = A.shape[2] if A is not None else agent_grid[0] * agent_grid[1]
    # Q, K, V (and their gradients) share one set of strides, dO may have its own (the layout of the output)
    desc = _desc_from(Q, n, grid, agent_grid, same=(K, V), out=dO, scale1=scale1, scale2=scale2,
                      v_residual_k=v_residual_k, window=window)
    p = make_params(params)
    need = int(lib().agent_attn_bwd_workspace_bytes(ctypes.byref(desc), _pp(p)))
    _check_agents(A, Q, n)
    if workspace is None:
        workspace = _alloc_bytes(max(need, 256), stream, Q.device)
    out = {k: torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device) for k in ("dQ", "dK", "dV")}
    if A is not None:
        out["dA"] = torch.empty_like(A)
    g = aa_param_grads()
    if params and want_param_grads:
        for key in ("b1_col", "b1_row", "b1_blk", "b2_col", "b2_row", "b2_blk", "dwc_w", "dwc_b"):
            t = params.get(key)
            if t is None and not (key == "dwc_b" and params.get("dwc_w") is not None):
                continue
            shape = t.shape if t is not None else params["dwc_w"].shape[:2]
            gt = torch.empty(tuple(shape), dtype=torch.float32, device="cuda")
            out["d" + key] = gt
            setattr(g, "d" + key, gt.data_ptr())
    st = lib().agent_attn_bwd(ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(A), _pp(p),
                              dO.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                              out["dQ"].data_ptr(), out["dK"].data_ptr(), out["dV"].data_ptr(), _ptr(out.get("dA")),
                              ctypes.byref(g), _stream(stream))
    _check(st, "agent_attn_bwd")
    return out


class PreparedCall:
    """A C-ABI call with its arguments marshalled once; calling it only crosses the ABI.

    Used by callers that issue the same call many times (serving loops, the benchmark): the
    descriptor structs and pointer arguments are built up front, so one invocation costs one
    ctypes call.  Holds references to every tensor involved so the pointers stay valid.
    """

    def __init__(self, fn, name, args, keep):
        self._fn, self._name, self._args, self._keep = fn, name, args, keep

    def __call__(self):
        st = self._fn(*self._args)
        if st != AA_OK:
            raise AgentAttnError(st, self._name)


def prepare_fwd(Q, K, V, A=None, *, grid=None, agent_grid=None, params: dict | None = None, scale1=0.0,
                scale2=0.0, v_residual_k=0.0, n_splits=0, out, workspace=None, stream=None) -> PreparedCall:
    n = A.shape[2] if A is not None else agent_grid[0] * agent_grid[1]
    desc = _desc_from(Q, n, grid, agent_grid, same=(K, V), out=out, scale1=scale1, scale2=scale2,
                      v_residual_k=v_residual_k, n_splits=n_splits)
    p = make_params(params)
    workspace, need = _workspace(desc, p, workspace)
    args = (ctypes.byref(desc), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(A), _pp(p), workspace.data_ptr(),
            workspace.numel() * workspace.element_size(), out.data_ptr(), _stream(stream))
    return PreparedCall(lib().agent_attn_fwd, "agent_attn_fwd", args, (desc, p, Q, K, V, A, params, workspace, out))


def prepare_pool(Q, *, grid, agent_grid, out, stream=None) -> PreparedCall:
    n = agent_grid[0] * agent_grid[1]
    desc = _desc_from(Q, n, grid, agent_grid)
    args = (ctypes.byref(desc), Q.data_ptr(), out.data_ptr(), _stream(stream))
    return PreparedCall(lib().agent_pool_fwd, "agent_pool_fwd", args, (desc, Q, out))


def prepare_aggregate(A, K, V, *, grid=None, params: dict | None = None, scale1=0.0, n_splits=0, out,
                      workspace=None, stream=None) -> PreparedCall:
    desc = _desc_from(K, A.shape[2], grid, None, same=(V,), scale1=scale1, n_splits=n_splits)
    p = make_params(params)
    workspace, need = _workspace(desc, p, workspace)
    args = (ctypes.byref(desc), A.data_ptr(), K.data_ptr(), V.data_ptr(), _pp(p), workspace.data_ptr(),
            workspace.numel() * workspace.element_size(), out.data_ptr(), _stream(stream))
    return PreparedCall(lib().agent_aggregate_fwd, "agent_aggregate_fwd", args,
                        (desc, p, A, K, V, params, workspace, out))


def prepare_broadcast(Q, A, VA, V=None, *, grid=None, params: dict | None = None, scale2=0.0, v_residual_k=0.0,
                      out, stream=None) -> PreparedCall:
    desc = _desc_from(Q, A.shape[2], grid, None, same=(V,), out=out, scale2=scale2, v_residual_k=v_residual_k)
    p = make_params(params)
    args = (ctypes.byref(desc), Q.data_ptr(), A.data_ptr(), VA.data_ptr(), _ptr(V), _pp(p), out.data_ptr(),
            _stream(stream))
    return PreparedCall(lib().agent_broadcast_fwd, "agent_broadcast_fwd", args, (desc, p, Q, A, VA, V, params, out))


def agent_pool_fwd(Q, *, grid, agent_grid, out=None, stream=None):
    import torch
    B, H, N, d = Q.shape
    n = agent_grid[0] * agent_grid[1]
    desc = _desc_from(Q, n, grid, agent_grid)
    if out is None:
        out = torch.empty((B, H, n, d), dtype=Q.dtype, device=Q.device)
    _check_agents(out, Q, n, "A_out")
    _check(lib().agent_pool_fwd(ctypes.byref(desc), Q.data_ptr(), out.data_ptr(), _stream(stream)),
           "agent_pool_fwd")
    return out


def agent_aggregate_fwd(A, K, V, *, grid=None, params: dict | None = None, scale1=0.0, n_splits=0, out=None,
                        workspace=None, stream=None):
    import torch
    B, H, N, d = K.shape
    n = A.shape[2]
    desc = _desc_from(K, n, grid, None, same=(V,), scale1=scale1, n_splits=n_splits)
    p = make_params(params)
    _check_agents(A, K, n)
    workspace, need = _workspace(desc, p, workspace, stream, K.device)
    if out is None:
        out = torch.empty((B, H, n, d), dtype=torch.float32, device=K.device)
    _check_agents(out, K, n, "VA_out", torch.float32)
    st = lib().agent_aggregate_fwd(ctypes.byref(desc), A.data_ptr(), K.data_ptr(), V.data_ptr(), _pp(p),
                                   workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                   out.data_ptr(), _stream(stream))
    _check(st, "agent_aggregate_fwd")
    return out


def agent_broadcast_fwd(Q, A, VA, V=None, *, grid=None, params: dict | None = None, scale2=0.0,
                        v_residual_k=0.0, out=None, stream=None):
    import torch
    n = A.shape[2]
    if out is None:
        out = torch.empty_like(Q)
    desc = _desc_from(Q, n, grid, None, same=(V,), out=out, scale2=scale2, v_residual_k=v_residual_k)
    _check_agents(A, Q, n)
    _check_agents(VA, Q, n, "VA", torch.float32)
    p = make_params(params)
    st = lib().agent_broadcast_fwd(ctypes.byref(desc), Q.data_ptr(), A.data_ptr(), VA.data_ptr(), _ptr(V), _pp(p),
                                   out.data_ptr(), _stream(stream))
    _check(st, "agent_broadcast_fwd")
    return out
