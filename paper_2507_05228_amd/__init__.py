"""Thin Python binding of libcascade (argument marshalling only).

Every step of the path runs in the HIP library; PyTorch supplies device memory and
streams.  The functions carry the names of the C entry points declared in
include/cascade.h.  If the shared library has not been built, loading fails loudly:
there is no CPU fallback.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcascade.so")

OK, EINVAL, ESHAPE, EASSIGN, EUNSUPPORTED, EWORKSPACE, EHIP = range(7)
STATUS_NAMES = ["OK", "EINVAL", "ESHAPE", "EASSIGN", "EUNSUPPORTED", "EWORKSPACE", "EHIP"]
F32, BF16 = 0, 1
MASK_NONE, MASK_CAUSAL = 0, 1
ROWS_ORIGINAL, ROWS_PACKED = 0, 1
U_UNNORMALISED, U_NORMALISED = 0, 1
NORM_NONE, NORM_LAYERNORM, NORM_RMSNORM = 0, 1, 2
ACT_GELU_ERF, ACT_GELU_TANH, ACT_SWIGLU = 0, 1, 2
ATTN_FUSED, ATTN_MATERIALISED = 0, 1
NORM_PRE, NORM_POST = 0, 1
EPI_BIAS, EPI_GELU_ERF, EPI_GELU_TANH, EPI_SWIGLU, EPI_ROPE, EPI_RESIDUAL = 1, 2, 4, 8, 16, 32

EXPORTS = ["cascade_plan_create", "cascade_plan_create_rs", "cascade_plan_maps", "cascade_plan_maps_host",
           "cascade_plan_kv_maps_host", "cascade_cdelta_assignment", "cascade_m_split", "cascade_comm_cost", "cascade_comm_time",
           "cascade_workspace_bytes", "cascade_layer_attention_output", "cascade_plan_destroy",
           "cascade_last_hip_error", "cascade_shard_gemm", "cascade_partial_attn_workspace_bytes",
           "cascade_partial_attn", "cascade_partial_attn_static", "cascade_lse_merge", "cascade_layer_workspace_bytes",
           "cascade_layer_forward", "cascade_layer_forward_staged", "cascade_layer_partials",
           "cascade_layer_stack_workspace_bytes", "cascade_layer_stack_forward",
           "cascade_lm_head_workspace_bytes", "cascade_lm_head", "cascade_greedy_token", "cascade_layer_kv_to_cache", "cascade_norm",
           "cascade_decode_partial_attn", "cascade_mfma_ceiling"]
N_STAGE_EVENTS = 10
STAGE_NAMES = ["gather_norm1", "qkv_gemm", "rope", "attention", "lse_merge", "o_proj", "norm2", "ffn_up", "ffn_down"]


class CascadeError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{where}: CASCADE_{name}")


class GemmDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("rows", C.c_int32), ("k", C.c_int32), ("n_out", C.c_int32),
                ("epilogue", C.c_int32), ("x_rows", C.c_int32), ("y_rows", C.c_int32), ("res_rows", C.c_int32),
                ("rope_cols", C.c_int32), ("head_dim", C.c_int32), ("rope_theta", C.c_float)]


class AttnDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("scale", C.c_float), ("row_layout", C.c_int32), ("u_mode", C.c_int32),
                ("q_stride_b", C.c_int64), ("q_stride_h", C.c_int64), ("q_stride_n", C.c_int64),
                ("kv_stride_b", C.c_int64), ("kv_stride_h", C.c_int64), ("kv_stride_n", C.c_int64)]


class LayerDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ff", C.c_int32), ("norm_kind", C.c_int32), ("norm_eps", C.c_float),
                ("act", C.c_int32), ("rope", C.c_int32), ("rope_theta", C.c_float), ("scale", C.c_float),
                ("attn_mode", C.c_int32), ("io_rows", C.c_int32), ("norm_placement", C.c_int32)]


class LmHeadDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("d_model", C.c_int32), ("vocab", C.c_int32), ("norm_kind", C.c_int32),
                ("norm_eps", C.c_float), ("rows", C.c_int32), ("in_rows", C.c_int32), ("out_rows", C.c_int32)]


LM_ALL_ROWS, LM_LAST_ROW = 0, 1

_WEIGHT_FIELDS = ["wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "bq", "bk", "bv", "bo", "b_up", "b_down",
                  "norm1_g", "norm1_b", "norm2_g", "norm2_b"]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WEIGHT_FIELDS]


_lib = None


def load_library():
    """dlopen libcascade.so and declare the signatures.  Raises if it was not built."""
    global _lib
    if _lib is not None:
        return _lib
    try:
        import torch  # noqa: F401  (its HIP runtime must be the one this process initialises first)
    except ImportError:
        pass
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` (build()) first; "
                           "there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    P, I32, VP = C.POINTER, C.c_int32, C.c_void_p
    lib.cascade_plan_create.argtypes = [P(VP), I32, I32, I32, P(I32), P(I32), I32]
    lib.cascade_plan_create.restype = I32
    lib.cascade_plan_create_rs.argtypes = [P(VP), I32, I32, I32, P(I32), I32, P(I32), P(I32), I32]
    lib.cascade_plan_create_rs.restype = I32
    lib.cascade_plan_kv_maps_host.argtypes = [VP, P(I32), P(P(I32)), P(P(I32)), P(P(I32))]
    lib.cascade_plan_kv_maps_host.restype = I32
    lib.cascade_cdelta_assignment.argtypes = [I32, I32, I32, P(I32), P(I32)]
    lib.cascade_cdelta_assignment.restype = I32
    lib.cascade_m_split.argtypes = [I32, I32, P(I32), I32, P(I32)]
    lib.cascade_m_split.restype = I32
    lib.cascade_comm_cost.argtypes = [I32, I32, I32, I32, I32, I32, I32, C.c_int64, P(C.c_int64), P(C.c_int64), P(C.c_int64)]
    lib.cascade_comm_cost.restype = I32
    F64 = C.c_double
    lib.cascade_comm_time.argtypes = [VP, I32, I32, I32, I32, I32, I32, I32, F64, F64, P(F64), P(F64), P(F64)]
    lib.cascade_comm_time.restype = I32
    lib.cascade_workspace_bytes.argtypes = [VP, VP, I32, I32]
    lib.cascade_workspace_bytes.restype = C.c_size_t
    lib.cascade_layer_attention_output.argtypes = [VP, P(LayerDesc), VP, P(VP)]
    lib.cascade_layer_attention_output.restype = I32
    lib.cascade_plan_maps.argtypes = [VP, P(VP), P(VP), P(VP)]
    lib.cascade_plan_maps.restype = I32
    lib.cascade_plan_maps_host.argtypes = [VP, P(P(I32)), P(P(I32)), P(P(I32))]
    lib.cascade_plan_maps_host.restype = I32
    lib.cascade_plan_destroy.argtypes = [VP]
    lib.cascade_plan_destroy.restype = None
    lib.cascade_last_hip_error.argtypes = []
    lib.cascade_last_hip_error.restype = I32
    lib.cascade_shard_gemm.argtypes = [VP, P(GemmDesc), VP, VP, VP, VP, VP, VP, VP]
    lib.cascade_shard_gemm.restype = I32
    lib.cascade_partial_attn_workspace_bytes.argtypes = [VP, P(AttnDesc)]
    lib.cascade_partial_attn_workspace_bytes.restype = C.c_size_t
    lib.cascade_partial_attn.argtypes = [VP, P(AttnDesc), VP, VP, VP, VP, VP, VP, VP, C.c_size_t, VP]
    lib.cascade_partial_attn.restype = I32
    lib.cascade_partial_attn_static.argtypes = [VP, P(AttnDesc), VP, VP, VP, VP, VP, VP, VP]
    lib.cascade_partial_attn_static.restype = I32
    lib.cascade_lse_merge.argtypes = [VP, P(AttnDesc), VP, VP, VP, VP, VP, VP]
    lib.cascade_lse_merge.restype = I32
    lib.cascade_layer_workspace_bytes.argtypes = [VP, P(LayerDesc)]
    lib.cascade_layer_workspace_bytes.restype = C.c_size_t
    lib.cascade_layer_forward.argtypes = [VP, P(LayerDesc), P(LayerWeights), VP, VP, VP, C.c_size_t, VP]
    lib.cascade_layer_forward.restype = I32
    lib.cascade_layer_forward_staged.argtypes = [VP, P(LayerDesc), P(LayerWeights), VP, VP, VP, C.c_size_t, VP,
                                                 P(VP), I32]
    lib.cascade_layer_forward_staged.restype = I32
    lib.cascade_layer_partials.argtypes = [VP, P(LayerDesc), VP, P(VP), P(VP), P(VP)]
    lib.cascade_layer_partials.restype = I32
    lib.cascade_layer_stack_workspace_bytes.argtypes = [VP, P(LayerDesc), I32]
    lib.cascade_layer_stack_workspace_bytes.restype = C.c_size_t
    lib.cascade_layer_stack_forward.argtypes = [VP, P(LayerDesc), P(LayerWeights), I32, VP, VP, VP, C.c_size_t, VP]
    lib.cascade_layer_stack_forward.restype = I32
    lib.cascade_lm_head_workspace_bytes.argtypes = [VP, P(LmHeadDesc)]
    lib.cascade_lm_head_workspace_bytes.restype = C.c_size_t
    lib.cascade_lm_head.argtypes = [VP, P(LmHeadDesc), VP, VP, VP, VP, VP, VP, C.c_size_t, VP]
    lib.cascade_lm_head.restype = I32
    lib.cascade_greedy_token.argtypes = [VP, I32, I32, I32, VP, VP]
    lib.cascade_greedy_token.restype = I32
    lib.cascade_layer_kv_to_cache.argtypes = [VP, P(LayerDesc), VP, VP, VP, I32, VP, VP]
    lib.cascade_layer_kv_to_cache.restype = I32
    lib.cascade_norm.argtypes = [I32, I32, I32, I32, C.c_float, VP, VP, VP, VP, VP]
    lib.cascade_norm.restype = I32
    lib.cascade_decode_partial_attn.argtypes = [P(AttnDesc), I32, I32, I32, VP, VP, VP, VP, VP, VP, VP, VP]
    lib.cascade_decode_partial_attn.restype = I32
    lib.cascade_mfma_ceiling.argtypes = [I32, I32, P(C.c_float), VP]
    lib.cascade_mfma_ceiling.restype = I32
    _lib = lib
    return lib


def _check(status, where):
    if status != OK:
        raise CascadeError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise CascadeError(EUNSUPPORTED, f"dtype {t.dtype}")


class Plan:
    """Owner of a cascade_plan handle."""

    def __init__(self, handle, batch, seq_len, n_shards, mask_kind, n_kv_shards=None):
        self.handle, self.batch, self.seq_len, self.n_shards, self.mask_kind = handle, batch, seq_len, n_shards, mask_kind
        self.n_kv_shards = n_shards if n_kv_shards is None else n_kv_shards   # partials: one per key/value shard

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.cascade_plan_destroy(self.handle)
            self.handle = None


def cascade_plan_create(batch, seq_len, n_shards, token_to_shard, positions=None, mask_kind=MASK_CAUSAL):
    lib = load_library()
    a = None if token_to_shard is None else np.ascontiguousarray(token_to_shard, dtype=np.int32)
    if a is not None and a.shape != (max(seq_len, 0),):
        raise CascadeError(ESHAPE, "cascade_plan_create: token_to_shard length")
    pos = None if positions is None else np.ascontiguousarray(positions, dtype=np.int32)
    if pos is not None and pos.shape != (seq_len,):
        raise CascadeError(ESHAPE, "cascade_plan_create: positions length")
    h = C.c_void_p()
    I32P = C.POINTER(C.c_int32)
    st = lib.cascade_plan_create(C.byref(h), batch, seq_len, n_shards,
                                 None if a is None else a.ctypes.data_as(I32P),
                                 None if pos is None else pos.ctypes.data_as(I32P), mask_kind)
    _check(st, "cascade_plan_create")
    return Plan(h, batch, seq_len, n_shards, mask_kind)


def cascade_plan_create_rs(batch, seq_len, n_row_shards, token_to_row_shard, n_kv_shards, token_to_kv_shard,
                           positions=None, mask_kind=MASK_CAUSAL):
    lib = load_library()
    I32P = C.POINTER(C.c_int32)
    a = np.ascontiguousarray(token_to_row_shard, dtype=np.int32)
    k = np.ascontiguousarray(token_to_kv_shard, dtype=np.int32)
    if a.shape != (seq_len,) or k.shape != (seq_len,):
        raise CascadeError(ESHAPE, "cascade_plan_create_rs: assignment length")
    pos = None if positions is None else np.ascontiguousarray(positions, dtype=np.int32)
    if pos is not None and pos.shape != (seq_len,):
        raise CascadeError(ESHAPE, "cascade_plan_create_rs: positions length")
    h = C.c_void_p()
    st = lib.cascade_plan_create_rs(C.byref(h), batch, seq_len, n_row_shards, a.ctypes.data_as(I32P), n_kv_shards,
                                    k.ctypes.data_as(I32P), None if pos is None else pos.ctypes.data_as(I32P), mask_kind)
    _check(st, "cascade_plan_create_rs")
    return Plan(h, batch, seq_len, n_row_shards, mask_kind, n_kv_shards)


def cascade_plan_kv_maps_host(plan):
    """(n_kv_shards, kv_perm, kv_offsets, kv_to_row or None) as numpy copies."""
    lib = load_library()
    I32P = C.POINTER(C.c_int32)
    n = C.c_int32()
    p, off, k2r = I32P(), I32P(), I32P()
    _check(lib.cascade_plan_kv_maps_host(plan.handle, C.byref(n), C.byref(p), C.byref(off), C.byref(k2r)),
           "cascade_plan_kv_maps_host")
    return (n.value, np.ctypeslib.as_array(p, (plan.seq_len,)).copy(), np.ctypeslib.as_array(off, (n.value + 1,)).copy(),
            np.ctypeslib.as_array(k2r, (plan.seq_len,)).copy() if k2r else None)


def cascade_cdelta_assignment(seq_len, c, delta):
    """(token_to_shard, n_shards) of the (c, delta)-sharding."""
    lib = load_library()
    out = np.zeros(max(seq_len, 0), dtype=np.int32)
    n = C.c_int32()
    _check(lib.cascade_cdelta_assignment(seq_len, c, delta, out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(n)),
           "cascade_cdelta_assignment")
    return out, n.value


def cascade_m_split(token_to_row_shard, n_row_shards, m):
    """token_to_kv_shard of the m-split of a row sharding (m * n_row_shards key/value shards)."""
    lib = load_library()
    I32P = C.POINTER(C.c_int32)
    a = np.ascontiguousarray(token_to_row_shard, dtype=np.int32)
    out = np.zeros_like(a)
    _check(lib.cascade_m_split(a.shape[0], n_row_shards, a.ctypes.data_as(I32P), m, out.ctypes.data_as(I32P)),
           "cascade_m_split")
    return out


def cascade_comm_cost(n_row_shards, n_kv_shards, bytes_per_value, head_dim, n_heads, n_kv_heads, seq_len,
                      m_split_scheme=False):
    """(stage_a_bytes, stage_b_bytes, rounds) per layer (Equation 1 and the rounds bound)."""
    lib = load_library()
    a, b, r = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib.cascade_comm_cost(n_row_shards, n_kv_shards, int(bool(m_split_scheme)), bytes_per_value, head_dim, n_heads,
                                 n_kv_heads, seq_len, C.byref(a), C.byref(b), C.byref(r)), "cascade_comm_cost")
    return a.value, b.value, r.value


def cascade_comm_time(bytes_per_value, head_dim, n_heads, n_kv_heads, latency_s, bandwidth_bytes_per_s, plan=None,
                      n_kv_shards=0, max_row_shard=0, max_kv_shard=0):
    """(total_s, stage_a_s, stage_b_s) of Equation 2; shard sizes from `plan` or given explicitly."""
    lib = load_library()
    a, b, t = C.c_double(), C.c_double(), C.c_double()
    _check(lib.cascade_comm_time(None if plan is None else plan.handle, n_kv_shards, max_row_shard, max_kv_shard,
                                 bytes_per_value, head_dim, n_heads, n_kv_heads, latency_s, bandwidth_bytes_per_s,
                                 C.byref(a), C.byref(b), C.byref(t)), "cascade_comm_time")
    return t.value, a.value, b.value


OP_SHARD_GEMM, OP_PARTIAL_ATTN, OP_LSE_MERGE, OP_LAYER_FORWARD, OP_LAYER_STACK, OP_LM_HEAD = range(6)


def cascade_workspace_bytes(plan, desc, op, flags=0):
    """Workspace bytes of operation `op` (OP_*) for its descriptor structure."""
    lib = load_library()
    return lib.cascade_workspace_bytes(plan.handle if plan is not None else None,
                                       None if desc is None else C.cast(C.byref(desc), C.c_void_p), op, flags)


def cascade_plan_maps(plan):
    """Device copies of perm, inv_perm, offsets as torch int32 tensors (copied out)."""
    import torch
    lib = load_library()
    p, ip, off = C.c_void_p(), C.c_void_p(), C.c_void_p()
    _check(lib.cascade_plan_maps(plan.handle, C.byref(p), C.byref(ip), C.byref(off)), "cascade_plan_maps")
    out = []
    for ptr, n in ((p, plan.seq_len), (ip, plan.seq_len), (off, plan.n_shards + 1)):
        out.append(torch.as_tensor(_DeviceInt32(ptr.value, n), device="cuda").clone())
    return tuple(out)


class _DeviceInt32:
    """Borrowed view of n int32 values in device memory (for torch.as_tensor)."""

    def __init__(self, ptr, n):
        self.__cuda_array_interface__ = {"shape": (n,), "typestr": "<i4", "data": (ptr, False), "version": 2}


def cascade_plan_maps_host(plan):
    lib = load_library()
    I32P = C.POINTER(C.c_int32)
    p, ip, off = I32P(), I32P(), I32P()
    _check(lib.cascade_plan_maps_host(plan.handle, C.byref(p), C.byref(ip), C.byref(off)), "cascade_plan_maps_host")
    return (np.ctypeslib.as_array(p, (plan.seq_len,)).copy(), np.ctypeslib.as_array(ip, (plan.seq_len,)).copy(),
            np.ctypeslib.as_array(off, (plan.n_shards + 1,)).copy())


def cascade_shard_gemm(plan, X, W, Y, W_up=None, bias=None, residual=None, epilogue=0,
                       x_rows=ROWS_PACKED, y_rows=ROWS_PACKED, res_rows=ROWS_PACKED,
                       rope_cols=0, head_dim=0, rope_theta=0.0, stream=None):
    lib = load_library()
    d = GemmDesc(_dtype_code(X), X.shape[0], X.shape[1], W.shape[0], epilogue, x_rows, y_rows, res_rows,
                 rope_cols, head_dim, rope_theta)
    st = lib.cascade_shard_gemm(plan.handle if plan is not None else None, C.byref(d), _ptr(X), _ptr(W), _ptr(W_up),
                                _ptr(bias), _ptr(residual), _ptr(Y), _stream(stream))
    _check(st, "cascade_shard_gemm")


def _attn_desc(q, n_heads, n_kv_heads, head_dim, scale, row_layout, u_mode, q_strides=None, kv_strides=None):
    d = AttnDesc(_dtype_code(q), n_heads, n_kv_heads, head_dim, scale, row_layout, u_mode, 0, 0, 0, 0, 0, 0)
    if q_strides:
        d.q_stride_b, d.q_stride_h, d.q_stride_n = q_strides
    if kv_strides:
        d.kv_stride_b, d.kv_stride_h, d.kv_stride_n = kv_strides
    return d


def cascade_partial_attn_workspace_bytes(plan, q, n_heads, n_kv_heads, head_dim):
    lib = load_library()
    d = _attn_desc(q, n_heads, n_kv_heads, head_dim, 1.0, ROWS_PACKED, U_UNNORMALISED)
    return lib.cascade_partial_attn_workspace_bytes(plan.handle, C.byref(d))


def cascade_partial_attn(plan, q, k, v, m, e, u, n_heads, n_kv_heads, head_dim, scale,
                         row_layout=ROWS_ORIGINAL, u_mode=U_UNNORMALISED, workspace=None,
                         q_strides=None, kv_strides=None, stream=None):
    lib = load_library()
    d = _attn_desc(q, n_heads, n_kv_heads, head_dim, scale, row_layout, u_mode, q_strides, kv_strides)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.cascade_partial_attn(plan.handle, C.byref(d), _ptr(q), _ptr(k), _ptr(v), _ptr(m), _ptr(e), _ptr(u),
                                  _ptr(workspace), ws_bytes, _stream(stream))
    _check(st, "cascade_partial_attn")


STATIC_SCRATCH_BYTES = 36 << 20


def cascade_partial_attn_static(plan, q, k, v, m, e, u, n_heads, n_kv_heads, head_dim, scale,
                                row_layout=ROWS_ORIGINAL, u_mode=U_UNNORMALISED, q_strides=None, kv_strides=None,
                                stream=None):
    """cascade_partial_attn with the library's static device scratch instead of a workspace."""
    lib = load_library()
    d = _attn_desc(q, n_heads, n_kv_heads, head_dim, scale, row_layout, u_mode, q_strides, kv_strides)
    st = lib.cascade_partial_attn_static(plan.handle, C.byref(d), _ptr(q), _ptr(k), _ptr(v), _ptr(m), _ptr(e), _ptr(u),
                                         _stream(stream))
    _check(st, "cascade_partial_attn_static")


def cascade_lse_merge(plan, m, e, u, o, n_heads, n_kv_heads, head_dim, row_layout=ROWS_PACKED,
                      u_mode=U_UNNORMALISED, lse_out=None, stream=None):
    lib = load_library()
    d = _attn_desc(o, n_heads, n_kv_heads, head_dim, 1.0, row_layout, u_mode)
    st = lib.cascade_lse_merge(plan.handle, C.byref(d), _ptr(m), _ptr(e), _ptr(u), _ptr(o), _ptr(lse_out),
                               _stream(stream))
    _check(st, "cascade_lse_merge")


def make_layer_desc(cfg, attn_mode=ATTN_FUSED, io_rows=ROWS_ORIGINAL, scale=None):
    """LayerDesc from a cascade_inputs.LayerConfig-like object (field copy only)."""
    act = {"gelu": ACT_GELU_ERF, "gelu_tanh": ACT_GELU_TANH, "swiglu": ACT_SWIGLU}[cfg.act]
    nk = {"layernorm": NORM_LAYERNORM, "rmsnorm": NORM_RMSNORM}[cfg.norm]
    return LayerDesc(BF16 if cfg.dtype == "bf16" else F32, cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim,
                     cfg.d_ff, nk, cfg.eps, act, 1 if cfg.rope else 0, cfg.rope_theta,
                     cfg.scale if scale is None else scale, attn_mode, io_rows,
                     NORM_POST if getattr(cfg, "norm_placement", "pre") == "post" else NORM_PRE)


def make_layer_weights(tensors):
    """LayerWeights from a dict of device tensors (absent keys -> NULL).  Keep `tensors` alive."""
    w = LayerWeights()
    for n in _WEIGHT_FIELDS:
        t = tensors.get(n)
        setattr(w, n, None if t is None else t.data_ptr())
    return w


def cascade_layer_workspace_bytes(plan, desc):
    return load_library().cascade_layer_workspace_bytes(plan.handle, C.byref(desc))


def cascade_layer_forward(plan, desc, weights, h_in, h_out, workspace, stream=None):
    lib = load_library()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.cascade_layer_forward(plan.handle, C.byref(desc), C.byref(weights), _ptr(h_in), _ptr(h_out),
                                   _ptr(workspace), ws_bytes, _stream(stream))
    _check(st, "cascade_layer_forward")


def cascade_layer_forward_staged(plan, desc, weights, h_in, h_out, workspace, events, stream=None):
    """events: N_STAGE_EVENTS torch.cuda.Event(enable_timing=True), each recorded once before
    (torch creates the HIP event lazily on its first record)."""
    lib = load_library()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    arr = (C.c_void_p * len(events))(*[ev.cuda_event for ev in events])
    st = lib.cascade_layer_forward_staged(plan.handle, C.byref(desc), C.byref(weights), _ptr(h_in), _ptr(h_out),
                                          _ptr(workspace), ws_bytes, _stream(stream), arr, len(events))
    _check(st, "cascade_layer_forward_staged")


def cascade_layer_stack_workspace_bytes(plan, desc, n_layers):
    return load_library().cascade_layer_stack_workspace_bytes(plan.handle, C.byref(desc), n_layers)


def cascade_layer_stack_forward(plan, desc, weights_list, h_in, h_out, workspace, stream=None):
    """weights_list: one LayerWeights per layer (the tensors behind them must stay alive)."""
    lib = load_library()
    arr = (LayerWeights * len(weights_list))(*weights_list)
    st = lib.cascade_layer_stack_forward(plan.handle, C.byref(desc), arr, len(weights_list), _ptr(h_in), _ptr(h_out),
                                         _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "cascade_layer_stack_forward")


def cascade_norm(x, gain, bias, y, norm_kind, eps, stream=None):
    """x, y [rows, D]."""
    lib = load_library()
    st = lib.cascade_norm(_dtype_code(x), x.shape[0], x.shape[1], norm_kind, eps, _ptr(x), _ptr(gain), _ptr(bias), _ptr(y),
                          _stream(stream))
    _check(st, "cascade_norm")


def cascade_layer_kv_to_cache(plan, desc, workspace, k_cache, v_cache, shard_len, stream=None):
    """k_cache, v_cache [B, Hkv, n_kv_shards, capacity, d]; shard_len int32 [B, n_kv_shards] (device)."""
    lib = load_library()
    st = lib.cascade_layer_kv_to_cache(plan.handle, C.byref(desc), _ptr(workspace), _ptr(k_cache), _ptr(v_cache),
                                       k_cache.shape[3], _ptr(shard_len), _stream(stream))
    _check(st, "cascade_layer_kv_to_cache")


def cascade_lm_head_workspace_bytes(plan, desc):
    return load_library().cascade_lm_head_workspace_bytes(plan.handle, C.byref(desc))


def cascade_lm_head(plan, desc, h_in, norm_gain, norm_bias, w_vocab, logits, workspace, stream=None):
    lib = load_library()
    st = lib.cascade_lm_head(plan.handle, C.byref(desc), _ptr(h_in), _ptr(norm_gain), _ptr(norm_bias), _ptr(w_vocab),
                             _ptr(logits), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "cascade_lm_head")


def cascade_greedy_token(logits, token_out, stream=None):
    """logits [rows, vocab] (bf16 or fp32, contiguous), token_out int32 [rows]."""
    lib = load_library()
    st = lib.cascade_greedy_token(_ptr(logits), _dtype_code(logits), logits.shape[0], logits.shape[1], _ptr(token_out),
                                  _stream(stream))
    _check(st, "cascade_greedy_token")


def cascade_layer_attention_output(plan, desc, workspace, batch, n_heads, head_dim):
    """View [B * N, H * d] (packed rows) of the merged attention output a layer forward left in its workspace."""
    import torch
    lib = load_library()
    o = C.c_void_p()
    _check(lib.cascade_layer_attention_output(plan.handle, C.byref(desc), _ptr(workspace), C.byref(o)),
           "cascade_layer_attention_output")
    es = 2 if desc.dtype == BF16 else 4
    T, W = batch * plan.seq_len, n_heads * head_dim
    off = o.value - workspace.data_ptr()
    flat = workspace.view(torch.uint8)[off:off + T * W * es]
    return flat.view(torch.bfloat16 if desc.dtype == BF16 else torch.float32).view(T, W)


def cascade_layer_partials(plan, desc, workspace, batch, n_heads, head_dim):
    """Views (torch tensors over the workspace) of m, e, u~ after a MATERIALISED layer forward."""
    import torch
    lib = load_library()
    m, e, u = C.c_void_p(), C.c_void_p(), C.c_void_p()
    _check(lib.cascade_layer_partials(plan.handle, C.byref(desc), _ptr(workspace), C.byref(m), C.byref(e), C.byref(u)),
           "cascade_layer_partials")
    base = workspace.data_ptr()
    f = workspace.view(torch.uint8)
    S, N = plan.n_kv_shards, plan.seq_len
    n_me = batch * n_heads * S * N

    def view(ptr, n, shape):
        off = ptr.value - base
        return f[off:off + 4 * n].view(torch.float32).view(*shape)

    return (view(m, n_me, (batch, n_heads, S, N)), view(e, n_me, (batch, n_heads, S, N)),
            view(u, n_me * head_dim, (batch, S, n_heads, N, head_dim)))


# ------------------------------------------------------------------ numpy <-> device marshalling helpers
def to_device(x, dtype_name):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype_name == "bf16" else t


def new_workspace(nbytes):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def cascade_decode_partial_attn(q, k_cache, v_cache, shard_len, m, e, u, scale, u_mode=U_UNNORMALISED, stream=None):
    """q [B,H,d]; k_cache, v_cache [B,Hkv,S,cap,d]; shard_len [B,S] int32 (device); m, e [B,H,S]; u [B,S,H,d]."""
    lib = load_library()
    B, H, d = q.shape
    Hkv, S, cap = k_cache.shape[1], k_cache.shape[2], k_cache.shape[3]
    desc = _attn_desc(q, H, Hkv, d, scale, ROWS_PACKED, u_mode)
    st = lib.cascade_decode_partial_attn(C.byref(desc), B, S, cap, _ptr(shard_len), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                         _ptr(m), _ptr(e), _ptr(u), _stream(stream))
    _check(st, "cascade_decode_partial_attn")


def cascade_mfma_ceiling(lds_operands, iters=200000, stream=None):
    """TFLOP/s sustained by back-to-back bf16 MFMAs with random operands (registers or LDS-fed)."""
    lib = load_library()
    out = C.c_float(0.0)
    _check(lib.cascade_mfma_ceiling(int(bool(lds_operands)), int(iters), C.byref(out), _stream(stream)),
           "cascade_mfma_ceiling")
    return float(out.value)


def layer_forward_numpy(cfg, weights_np, h_np, token_to_shard, positions=None, attn_mode=ATTN_FUSED,
                        io_rows=ROWS_ORIGINAL, mask_kind=MASK_CAUSAL, return_partials=False, token_to_kv_shard=None,
                        fused_qkv=False):
    """Upload numpy inputs, run cascade_layer_forward once, download the output as float64.
    token_to_kv_shard: a second partition for keys / values (row shards != key/value shards).
    fused_qkv: the q, k, v weights (and biases) are uploaded as one [(H + 2 H_KV) d, D] matrix and handed over
    as three views of it (the library then runs the projection as one segment)."""
    import torch
    n_row = int(np.max(token_to_shard)) + 1 if cfg.n_shards is None else cfg.n_shards
    if token_to_kv_shard is None:
        plan = cascade_plan_create(cfg.batch, cfg.seq_len, n_row, token_to_shard, positions, mask_kind)
    else:
        plan = cascade_plan_create_rs(cfg.batch, cfg.seq_len, n_row, token_to_shard, int(np.max(token_to_kv_shard)) + 1,
                                      token_to_kv_shard, positions, mask_kind)
    desc = make_layer_desc(cfg, attn_mode, io_rows)
    tensors = {k: to_device(v, cfg.dtype) for k, v in weights_np.items()}
    if fused_qkv:
        for names in (("wq", "wk", "wv"), ("bq", "bk", "bv")):
            if all(n in tensors for n in names):
                whole = torch.cat([tensors[n] for n in names], dim=0).contiguous()
                row = 0
                for n in names:
                    rows = tensors[n].shape[0]
                    tensors[n] = whole[row:row + rows]
                    row += rows
    w = make_layer_weights(tensors)
    h_in = to_device(h_np, cfg.dtype)
    h_out = torch.empty_like(h_in)
    ws = new_workspace(cascade_layer_workspace_bytes(plan, desc))
    cascade_layer_forward(plan, desc, w, h_in, h_out, ws)
    torch.cuda.synchronize()
    out = h_out.float().cpu().numpy().astype(np.float64)
    if return_partials:
        m, e, u = cascade_layer_partials(plan, desc, ws, cfg.batch, cfg.n_heads, cfg.head_dim)
        return out, tuple(t.cpu().numpy().astype(np.float64) for t in (m, e, u))
    return out
