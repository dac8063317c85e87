"""Thin ctypes binding of libscmoe: one Python function per C entry point, same names.

Only argument marshalling happens here (tensor -> pointer / stride / size); every step of
the layer runs in the HIP kernels.  torch is used for device memory and streams.  There is
no CPU fallback: loading fails loudly when the library has not been built.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libscmoe.so")

F32, BF16 = 0, 1
GELU_ERF, GELU_TANH = 0, 1
CG_NONE, CG_1, CG_2 = 0, 1, 2
MAX_EXPERTS = 64

EXPORTS = ["scmoe_status_string", "scmoe_last_hip_error", "scmoe_set_gemm_variant", "scmoe_padded_ld", "scmoe_capacity",
           "scmoe_gate_top1",
           "scmoe_gate_top2", "scmoe_gate_topk", "scmoe_dispatch_workspace_bytes", "scmoe_dispatch", "scmoe_dispatch_static",
           "scmoe_dispatch_static_max_bytes", "scmoe_expert_ffn",
           "scmoe_expert_ffn_workspace_bytes",
           "scmoe_combine", "scmoe_coef_gate", "scmoe_workspace_bytes", "scmoe_layer_forward",
           "scmoe_offload_pool_bytes", "scmoe_layer_forward_offload", "scmoe_offload_begin", "scmoe_offload_finish", "moe_topk_layer_forward",
           "moe_top2_layer_forward"]


class Desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("T", "d", "F", "E", "k", "capacity", "dtype", "gelu_mode", "normalize", "cg_mode")]


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("W_g", "bias", "W1", "b1", "W2", "b2", "W1s", "b1s", "W2s", "b2s", "W_cg")] + \
               [("ld_w1", C.c_int64), ("ld_w2", C.c_int64)]


class RoutingOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("expert_idx", "gate_w", "counts", "offsets", "dst_row", "src_token")]


class ScmoeError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().scmoe_status_string(status).decode()
        extra = " (hipError %d)" % lib().scmoe_last_hip_error() if status == 5 else ""
        super().__init__("%s: status %d: %s%s" % (where, status, msg, extra))


_lib = None


def lib():
    """The loaded shared library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libscmoe.so is not built: run `python -c 'import __graft_entry__ as g; "
                               "g.build()'` (or paper_2404_05019_amd/build.py) first")
        _lib = C.CDLL(LIB_PATH)
        _lib.scmoe_status_string.restype = C.c_char_p
        _lib.scmoe_status_string.argtypes = [C.c_int]
        i32, i64, vp, sz = C.c_int32, C.c_int64, C.c_void_p, C.c_size_t
        _lib.scmoe_capacity.argtypes = [i32, i32, i32, C.c_double, C.POINTER(i32)]
        _lib.scmoe_padded_ld.argtypes = [i32, i32, C.POINTER(i64)]
        _lib.scmoe_gate_top1.argtypes = [vp, i64, i32, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
        _lib.scmoe_gate_top2.argtypes = _lib.scmoe_gate_top1.argtypes
        _lib.scmoe_gate_topk.argtypes = [vp, i64, i32, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp]
        _lib.scmoe_dispatch_workspace_bytes.argtypes = [i32, i32, i32, C.POINTER(sz)]
        _lib.scmoe_dispatch.argtypes = [vp, i64, i32, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, i64,
                                        vp, sz, vp]
        _lib.scmoe_dispatch_static.argtypes = [vp, i64, i32, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, i64, vp]
        _lib.scmoe_dispatch_static_max_bytes.argtypes = [C.POINTER(sz)]
        _lib.scmoe_expert_ffn.argtypes = [vp, i64, i32, vp, i32, i32, i32, i32, vp, i64, vp, vp, i64, vp, vp, i64,
                                          vp, i64, i32, vp, sz, vp]
        _lib.scmoe_expert_ffn_workspace_bytes.argtypes = [i32, i32, i32, C.POINTER(sz)]
        _lib.scmoe_combine.argtypes = [vp, i64, i32, vp, vp, i32, i32, i32, vp, i64, vp, i64, vp, vp, i64, vp]
        _lib.scmoe_coef_gate.argtypes = [vp, i64, i32, vp, i32, i32, i32, vp, vp]
        _lib.scmoe_workspace_bytes.argtypes = [C.POINTER(Desc), C.POINTER(sz)]
        _lib.scmoe_layer_forward.argtypes = [C.POINTER(Desc), vp, i64, vp, i64, C.POINTER(Weights), vp, i64,
                                             vp, i64, C.POINTER(RoutingOut), vp, sz, vp, vp]
        _lib.scmoe_offload_pool_bytes.argtypes = [C.POINTER(Desc), i32, C.POINTER(sz)]
        _lib.scmoe_layer_forward_offload.argtypes = [C.POINTER(Desc), vp, i64, vp, i64, C.POINTER(Weights), vp, i32,
                                                     i32, vp, vp, i64, vp, sz, vp, vp]
        _lib.scmoe_offload_begin.argtypes = [C.POINTER(Desc), vp, i64, C.POINTER(Weights), vp, i32, i32, vp, vp, sz,
                                             vp, vp]
        _lib.scmoe_offload_finish.argtypes = [C.POINTER(Desc), vp, i64, vp, i64, C.POINTER(Weights), vp, i32, i32, vp,
                                              vp, i64, vp, sz, vp, vp]
        _lib.moe_topk_layer_forward.argtypes = [C.POINTER(Desc), vp, i64, C.POINTER(Weights), vp, i64,
                                                C.POINTER(RoutingOut), vp, sz, vp]
        _lib.moe_top2_layer_forward.argtypes = _lib.moe_topk_layer_forward.argtypes
    return _lib


def _check(status, where):
    if status != 0:
        raise ScmoeError(status, where)


def dtype_code(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("unsupported activation dtype %s" % t.dtype)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _ld(t):
    """Row stride in elements of a 2-D tensor whose last dimension is contiguous."""
    if t is None:
        return 0
    assert t.dim() == 2 and (t.shape[1] == 1 or t.stride(1) == 1), "rows must be contiguous"
    return t.stride(0)


def _ldw(t):
    """Row stride in elements of a weight tensor [E, out, in] or [out, in] whose rows are
    contiguous and whose experts follow each other at out * stride."""
    if t is None:
        return 0
    assert t.stride(-1) == 1, "rows must be contiguous"
    ld = t.stride(-2)
    assert t.dim() == 2 or t.shape[0] == 1 or t.stride(0) == t.shape[1] * ld, "experts must be evenly spaced"
    return ld


def _stream(s):
    if s is None:
        return torch.cuda.current_stream().cuda_stream
    return s.cuda_stream if hasattr(s, "cuda_stream") else int(s)


def scmoe_set_gemm_variant(variant):
    _check(lib().scmoe_set_gemm_variant(int(variant)), "scmoe_set_gemm_variant")


def scmoe_padded_ld(width, dtype):
    out = C.c_int64(0)
    _check(lib().scmoe_padded_ld(width, dtype, C.byref(out)), "scmoe_padded_ld")
    return out.value


def scmoe_capacity(T, E, k, cf):
    out = C.c_int32(0)
    _check(lib().scmoe_capacity(T, E, k, float(cf), C.byref(out)), "scmoe_capacity")
    return out.value


def _gate(fn, name, x, W_g, bias, E, normalize, expert_idx, gate_w, probs, stream):
    T, d = x.shape
    _check(fn(_ptr(x), _ld(x), dtype_code(x), _ptr(W_g), _ptr(bias), T, d, E, normalize,
              _ptr(expert_idx), _ptr(gate_w), _ptr(probs), _stream(stream)), name)


def scmoe_gate_top1(x, W_g, bias, expert_idx, gate_w, probs=None, normalize=0, stream=None):
    _gate(lib().scmoe_gate_top1, "scmoe_gate_top1", x, W_g, bias, W_g.shape[1], normalize, expert_idx,
          gate_w, probs, stream)


def scmoe_gate_top2(x, W_g, bias, expert_idx, gate_w, probs=None, normalize=1, stream=None):
    _gate(lib().scmoe_gate_top2, "scmoe_gate_top2", x, W_g, bias, W_g.shape[1], normalize, expert_idx,
          gate_w, probs, stream)


def scmoe_gate_topk(x, W_g, bias, k, expert_idx, gate_w, probs=None, normalize=1, stream=None):
    T, d = x.shape
    _check(lib().scmoe_gate_topk(_ptr(x), _ld(x), dtype_code(x), _ptr(W_g), _ptr(bias), T, d,
                                 W_g.shape[1], int(k), normalize, _ptr(expert_idx), _ptr(gate_w),
                                 _ptr(probs), _stream(stream)), "scmoe_gate_topk")


def scmoe_dispatch_workspace_bytes(T, E, k):
    out = C.c_size_t(0)
    _check(lib().scmoe_dispatch_workspace_bytes(T, E, k, C.byref(out)), "scmoe_dispatch_workspace_bytes")
    return out.value


def scmoe_dispatch(x, expert_idx, E, k, capacity, counts, offsets, dst_row, src_token, x_perm, workspace,
                   stream=None):
    T, d = x.shape
    _check(lib().scmoe_dispatch(_ptr(x), _ld(x), dtype_code(x), _ptr(expert_idx), T, d, E, k, capacity,
                                _ptr(counts), _ptr(offsets), _ptr(dst_row), _ptr(src_token), _ptr(x_perm),
                                _ld(x_perm), _ptr(workspace),
                                0 if workspace is None else workspace.numel() * workspace.element_size(),
                                _stream(stream)), "scmoe_dispatch")


def scmoe_dispatch_static(x, expert_idx, E, k, capacity, counts, offsets, dst_row, src_token, x_perm, stream=None):
    T, d = x.shape
    _check(lib().scmoe_dispatch_static(_ptr(x), _ld(x), dtype_code(x), _ptr(expert_idx), T, d, E, k, capacity,
                                       _ptr(counts), _ptr(offsets), _ptr(dst_row), _ptr(src_token), _ptr(x_perm),
                                       _ld(x_perm), _stream(stream)), "scmoe_dispatch_static")


def scmoe_dispatch_static_max_bytes():
    out = C.c_size_t(0)
    _check(lib().scmoe_dispatch_static_max_bytes(C.byref(out)), "scmoe_dispatch_static_max_bytes")
    return out.value


def scmoe_expert_ffn_workspace_bytes(dtype, d, F):
    out = C.c_size_t(0)
    _check(lib().scmoe_expert_ffn_workspace_bytes(dtype, d, F, C.byref(out)), "scmoe_expert_ffn_workspace_bytes")
    return out.value


def scmoe_expert_ffn(x_perm, offsets, max_rows, W1, b1, W2, b2, hidden, y_perm, gelu_mode=GELU_ERF,
                     workspace=None, stream=None):
    E, F, d = W1.shape
    _check(lib().scmoe_expert_ffn(_ptr(x_perm), _ld(x_perm), dtype_code(x_perm), _ptr(offsets), max_rows, E,
                                  d, F, _ptr(W1), _ldw(W1), _ptr(b1), _ptr(W2), _ldw(W2), _ptr(b2), _ptr(hidden),
                                  _ld(hidden), _ptr(y_perm), _ld(y_perm), gelu_mode, _ptr(workspace),
                                  0 if workspace is None else workspace.numel() * workspace.element_size(),
                                  _stream(stream)),
           "scmoe_expert_ffn")


def scmoe_combine(y_perm, dst_row, gate_w, k, base, residual, coef, y, stream=None):
    T, d = y.shape
    _check(lib().scmoe_combine(_ptr(y_perm), _ld(y_perm), dtype_code(y), _ptr(dst_row), _ptr(gate_w), T, d, k,
                               _ptr(base), _ld(base), _ptr(residual), _ld(residual), _ptr(coef), _ptr(y),
                               _ld(y), _stream(stream)), "scmoe_combine")


def scmoe_coef_gate(x, W_cg, cg_mode, coef, stream=None):
    T, d = x.shape
    _check(lib().scmoe_coef_gate(_ptr(x), _ld(x), dtype_code(x), _ptr(W_cg), cg_mode, T, d, _ptr(coef),
                                 _stream(stream)), "scmoe_coef_gate")


def make_desc(T, d, F, E, k, capacity, dtype, gelu_mode=GELU_ERF, normalize=0, cg_mode=CG_NONE):
    return Desc(T, d, F, E, k, capacity, dtype, gelu_mode, normalize, cg_mode)


def make_weights(W_g, W1, W2, W1s=None, W2s=None, bias=None, b1=None, b2=None, b1s=None, b2s=None,
                 W_cg=None):
    """Struct of device pointers.  The caller keeps the tensors alive.  W1 / W2 may be views
    with padded rows (see scmoe_padded_ld); the shared expert's weights then use the same
    row strides."""
    ld1, ld2 = _ldw(W1), _ldw(W2)
    assert W1s is None or _ldw(W1s) == ld1, "W1 and W1s must share one row stride"
    assert W2s is None or _ldw(W2s) == ld2, "W2 and W2s must share one row stride"
    return Weights(_ptr(W_g), _ptr(bias), _ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), _ptr(W1s), _ptr(b1s),
                   _ptr(W2s), _ptr(b2s), _ptr(W_cg), ld1, ld2)


def make_routing_out(expert_idx=None, gate_w=None, counts=None, offsets=None, dst_row=None, src_token=None):
    return RoutingOut(_ptr(expert_idx), _ptr(gate_w), _ptr(counts), _ptr(offsets), _ptr(dst_row),
                      _ptr(src_token))


def scmoe_workspace_bytes(desc):
    out = C.c_size_t(0)
    _check(lib().scmoe_workspace_bytes(C.byref(desc), C.byref(out)), "scmoe_workspace_bytes")
    return out.value


def scmoe_layer_forward(desc, x_prev, x_cur, weights, y, workspace, residual=None, routing=None,
                        stream_main=None, stream_aux=None):
    _check(lib().scmoe_layer_forward(
        C.byref(desc), _ptr(x_prev), _ld(x_prev), _ptr(x_cur), _ld(x_cur), C.byref(weights), _ptr(residual),
        _ld(residual), _ptr(y), _ld(y), None if routing is None else C.byref(routing), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream_main),
        None if stream_aux is None else _stream(stream_aux)), "scmoe_layer_forward")


def scmoe_offload_pool_bytes(desc, pool_experts):
    out = C.c_size_t(0)
    _check(lib().scmoe_offload_pool_bytes(C.byref(desc), pool_experts, C.byref(out)), "scmoe_offload_pool_bytes")
    return out.value


def scmoe_layer_forward_offload(desc, x_prev, x_cur, weights, expert_pool, pool_experts, host_plan, y, workspace,
                                async_copy=True, stream_main=None, stream_copy=None):
    """weights: W1 / W2 / b1 / b2 are host tensors (pinned), everything else on the device;
    host_plan: pinned int32 host tensor of 2 * E + 1 entries."""
    assert host_plan.dtype == torch.int32 and not host_plan.is_cuda
    _check(lib().scmoe_layer_forward_offload(
        C.byref(desc), _ptr(x_prev), _ld(x_prev), _ptr(x_cur), _ld(x_cur), C.byref(weights), _ptr(expert_pool),
        pool_experts, 1 if async_copy else 0, _ptr(host_plan), _ptr(y), _ld(y), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream_main),
        None if stream_copy is None else _stream(stream_copy)), "scmoe_layer_forward_offload")


def scmoe_offload_begin(desc, x_prev, weights, expert_pool, pool_experts, host_plan, workspace, async_copy=True,
                        stream_main=None, stream_copy=None):
    assert host_plan.dtype == torch.int32 and not host_plan.is_cuda
    _check(lib().scmoe_offload_begin(
        C.byref(desc), _ptr(x_prev), _ld(x_prev), C.byref(weights), _ptr(expert_pool), pool_experts,
        1 if async_copy else 0, _ptr(host_plan), _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream_main), None if stream_copy is None else _stream(stream_copy)), "scmoe_offload_begin")


def scmoe_offload_finish(desc, x_prev, x_cur, weights, expert_pool, pool_experts, host_plan, y, workspace,
                         async_copy=True, stream_main=None, stream_copy=None):
    assert host_plan.dtype == torch.int32 and not host_plan.is_cuda
    _check(lib().scmoe_offload_finish(
        C.byref(desc), _ptr(x_prev), _ld(x_prev), _ptr(x_cur), _ld(x_cur), C.byref(weights), _ptr(expert_pool),
        pool_experts, 1 if async_copy else 0, _ptr(host_plan), _ptr(y), _ld(y), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream_main),
        None if stream_copy is None else _stream(stream_copy)), "scmoe_offload_finish")


def moe_topk_layer_forward(desc, x, weights, y, workspace, routing=None, stream=None):
    _check(lib().moe_topk_layer_forward(
        C.byref(desc), _ptr(x), _ld(x), C.byref(weights), _ptr(y), _ld(y),
        None if routing is None else C.byref(routing), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)), "moe_topk_layer_forward")


def moe_top2_layer_forward(desc, x, weights, y, workspace, routing=None, stream=None):
    _check(lib().moe_top2_layer_forward(
        C.byref(desc), _ptr(x), _ld(x), C.byref(weights), _ptr(y), _ld(y),
        None if routing is None else C.byref(routing), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)), "moe_top2_layer_forward")
