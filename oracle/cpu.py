"""ctypes front end of the CPU oracle (oracle/scmoe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  It imports nothing from the GPU package.

All arrays are numpy; inputs are float32 (bf16 workloads pass bf16 values widened to
float32), float outputs of the FFN / layer are float64.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("Wg", "bias", "W1", "b1", "W2", "b2", "W1s", "b1s", "W2s", "b2s", "Wcg")]


def lib():
    """Load liboracle.so, compiling it first when it is missing or older than its source."""
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.oracle_gelu.restype = C.c_double
        _lib.oracle_gelu.argtypes = [C.c_double, C.c_int]
        _lib.oracle_round_to_bf16.restype = C.c_double
        _lib.oracle_round_to_bf16.argtypes = [C.c_double]
        _lib.oracle_capacity.restype = C.c_int
        _lib.oracle_capacity.argtypes = [C.c_int, C.c_int, C.c_int, C.c_double]
    return _lib


def _f32(a):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads():
    """Threads the OpenMP loops of the oracle use."""
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))


def gelu(v, mode=0):
    return lib().oracle_gelu(float(v), int(mode))


def round_to_bf16(v):
    """The rounding the "mimic" mode applies where a bf16 pipeline stores a value."""
    return lib().oracle_round_to_bf16(float(v))


def capacity(T, E, k, cf):
    return lib().oracle_capacity(int(T), int(E), int(k), float(cf))


def gate_logits(x, Wg, bias=None):
    """Eq. (4) logits, fp32 ascending-FMA chain.  x [T,d], Wg [d,E] -> [T,E] float32."""
    x, Wg, bias = _f32(x), _f32(Wg), _f32(bias)
    T, d = x.shape
    E = Wg.shape[1]
    assert Wg.shape[0] == d
    out = np.empty((T, E), np.float32)
    lib().oracle_gate_logits(_p(x), C.c_long(d), _p(Wg), _p(bias), T, d, E, _p(out))
    return out


def gate_logits_f64(x, Wg, bias=None):
    x, Wg, bias = _f32(x), _f32(Wg), _f32(bias)
    T, d = x.shape
    E = Wg.shape[1]
    out = np.empty((T, E), np.float64)
    lib().oracle_gate_logits_f64(_p(x), C.c_long(d), _p(Wg), _p(bias), T, d, E, _p(out))
    return out


def gate_topk(logits, k=1, normalize=0):
    """Eq. (2)-(3).  Returns idx [T,k] int32, w [T,k] float32, probs [T,E] float32."""
    logits = _f32(logits)
    T, E = logits.shape
    idx = np.empty((T, k), np.int32)
    w = np.empty((T, k), np.float32)
    probs = np.empty((T, E), np.float32)
    lib().oracle_gate_topk(_p(logits), T, E, k, int(normalize), _p(idx), _p(w), _p(probs))
    return idx, w, probs


def gate(x, Wg, bias=None, k=1, normalize=0):
    return gate_topk(gate_logits(x, Wg, bias), k, normalize)


def dispatch(idx, E, capacity_):
    """Sec. 2.2 input encode.  idx [T,k] -> counts, offsets, dst_row [T,k], src_token [K]."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.ndim == 1:
        idx = idx[:, None]
    T, k = idx.shape
    counts = np.zeros(E, np.int32)
    offsets = np.zeros(E + 1, np.int32)
    dst_row = np.empty((T, k), np.int32)
    src_token = np.full(T * k + 1, -1, np.int32)
    lib().oracle_dispatch(_p(idx), T, E, k, int(capacity_), _p(counts), _p(offsets),
                          _p(dst_row), _p(src_token))
    return counts, offsets, dst_row, src_token[:int(offsets[E])].copy()


def expert_ffn(x_perm, offsets, W1, W2, b1=None, b2=None, gelu_mode=0, mimic=0):
    """Eq. (1) experts over packed segments.  W1 [E,F,d], W2 [E,d,F] -> y_perm [K,d] f64."""
    x_perm, W1, W2, b1, b2 = _f32(x_perm), _f32(W1), _f32(W2), _f32(b1), _f32(b2)
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    E, F, d = W1.shape
    assert W2.shape == (E, d, F) and offsets.shape[0] == E + 1
    K = x_perm.shape[0]
    assert offsets[E] <= K
    y = np.zeros((K, d), np.float64)
    lib().oracle_expert_ffn(_p(x_perm), C.c_long(x_perm.shape[1]), _p(offsets), E, d, F, _p(W1),
                            _p(b1), _p(W2), _p(b2), int(gelu_mode), int(mimic), _p(y))
    return y


def coef_gate(x, Wcg, mode):
    x, Wcg = _f32(x), _f32(Wcg)
    T, d = x.shape
    out = np.empty((T, 2), np.float64)
    lib().oracle_coef_gate(_p(x), C.c_long(d), _p(Wcg), int(mode), T, d, _p(out))
    return out


def combine(y_perm, dst_row, w, base=None, residual=None, coef=None):
    y_perm = np.ascontiguousarray(y_perm, dtype=np.float64)
    dst_row = np.ascontiguousarray(dst_row, dtype=np.int32)
    if dst_row.ndim == 1:
        dst_row = dst_row[:, None]
    T, k = dst_row.shape
    d = y_perm.shape[1]
    w = _f32(w).reshape(T, k)
    f64 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.float64)
    base, residual, coef = f64(base), f64(residual), f64(coef)
    y = np.empty((T, d), np.float64)
    lib().oracle_combine(_p(y_perm), _p(dst_row), _p(w), T, d, k, _p(base), _p(residual),
                         _p(coef), _p(y))
    return y


def _weights(Wd):
    keep = {}
    ws = _Weights()
    for n, _ in _Weights._fields_:
        a = _f32(Wd.get(n))
        keep[n] = a
        setattr(ws, n, None if a is None else a.ctypes.data)
    return ws, keep


def layer_rows(x_prev, x_cur, Wd, routing, tokens, k=1, shared=1, cg_mode=0, gelu_mode=0,
               mimic=0, add_residual=0):
    """Eq. (7) (shared=1) or Eq. (1) (shared=0) for the listed tokens, routing given.

    Wd: dict with keys Wg,bias,W1,b1,W2,b2,W1s,b1s,W2s,b2s,Wcg (missing = None).
    routing: dict with idx, w, dst_row ([T,k]).  Returns [n,d] float64.
    """
    x_cur = _f32(x_cur)
    x_prev = x_cur if x_prev is None else _f32(x_prev)
    ws, keep = _weights(Wd)
    E, F, d = keep["W1"].shape
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    idx = np.ascontiguousarray(routing["idx"], dtype=np.int32)
    w = _f32(routing["w"])
    dst = np.ascontiguousarray(routing["dst_row"], dtype=np.int32)
    y = np.empty((len(tokens), d), np.float64)
    lib().oracle_layer_rows(_p(x_prev), C.c_long(x_prev.shape[1]), _p(x_cur),
                            C.c_long(x_cur.shape[1]), C.byref(ws), d, F, int(k), int(shared),
                            int(cg_mode), int(gelu_mode), int(mimic), int(add_residual),
                            _p(idx), _p(w), _p(dst), _p(tokens), len(tokens), _p(y))
    return y


def route(x_gate, Wd, E, k, C_, normalize=0):
    """Gate + capacity-bounded encode for all tokens.  Returns the routing dict."""
    idx, w, probs = gate(x_gate, Wd["Wg"], Wd.get("bias"), k, normalize)
    counts, offsets, dst_row, src_token = dispatch(idx, E, C_)
    return dict(idx=idx, w=w, probs=probs, counts=counts, offsets=offsets, dst_row=dst_row,
                src_token=src_token)


def layer_forward(x_prev, x_cur, Wd, k=1, capacity_=None, shared=1, normalize=0, cg_mode=0,
                  gelu_mode=0, mimic=0, add_residual=0):
    """The whole block through the single C entry point.  Returns (y [T,d] f64, routing)."""
    x_cur = _f32(x_cur)
    x_prev = x_cur if x_prev is None else _f32(x_prev)
    ws, keep = _weights(Wd)
    E, F, d = keep["W1"].shape
    T = x_cur.shape[0]
    Cc = T * k if capacity_ is None else int(capacity_)
    idx = np.empty((T, k), np.int32)
    w = np.empty((T, k), np.float32)
    counts = np.zeros(E, np.int32)
    offsets = np.zeros(E + 1, np.int32)
    dst_row = np.empty((T, k), np.int32)
    src_token = np.full(T * k + 1, -1, np.int32)
    y = np.empty((T, d), np.float64)
    lib().oracle_layer_forward(_p(x_prev), C.c_long(x_prev.shape[1]), _p(x_cur),
                               C.c_long(x_cur.shape[1]), C.byref(ws), T, d, F, E, int(k), Cc,
                               int(shared), int(normalize), int(cg_mode), int(gelu_mode),
                               int(mimic), int(add_residual), _p(idx), _p(w), _p(counts),
                               _p(offsets), _p(dst_row), _p(src_token), _p(y))
    routing = dict(idx=idx, w=w, counts=counts, offsets=offsets, dst_row=dst_row,
                   src_token=src_token[:int(offsets[E])].copy())
    return y, routing
