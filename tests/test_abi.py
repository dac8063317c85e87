"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and
turns bad arguments into status codes on the host (no kernel is launched by these calls)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2404_05019_amd import binding as B
from paper_2404_05019_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "scmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:int|const char\*)\s+((?:scmoe|moe)_\w+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 14
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_status_strings():
    lib = B.lib()
    assert lib.scmoe_status_string(0) == b"ok"
    seen = {lib.scmoe_status_string(i) for i in range(7)}
    assert len(seen) == 7 and lib.scmoe_status_string(99) == b"unknown status"


def test_capacity_host_function():
    for (T, E, k, cf, C_) in [(256, 4, 1, 1.25, 80), (8192, 8, 1, 1.25, 1280), (16384, 8, 2, 1.25, 5120),
                              (16384, 16, 1, 1.0, 1024), (32768, 16, 1, 1.25, 2560), (10, 3, 1, 1.0, 4),
                              (7, 2, 1, 1.1, 4), (0, 4, 1, 1.25, 0)]:
        assert B.scmoe_capacity(T, E, k, cf) == C_ == inputs.capacity(T, E, k, cf)
    with pytest.raises(B.ScmoeError) as e:
        B.scmoe_capacity(10, 0, 1, 1.0)
    assert e.value.status == 2
    assert B.lib().scmoe_capacity(1, 1, 1, 1.0, None) == 1


def test_padded_ld_host_function():
    assert B.scmoe_padded_ld(2048, B.BF16) == 2112 and B.scmoe_padded_ld(8192, B.BF16) == 8256
    assert B.scmoe_padded_ld(384, B.BF16) == 384 and B.scmoe_padded_ld(64, B.F32) == 64
    assert B.scmoe_padded_ld(128, B.F32) == 160
    out = C.c_int64(0)
    assert B.lib().scmoe_padded_ld(0, B.BF16, C.byref(out)) == 2
    assert B.lib().scmoe_padded_ld(64, 7, C.byref(out)) == 3
    assert B.lib().scmoe_padded_ld(64, B.BF16, None) == 1


def test_workspace_sizes_and_desc_checks():
    assert B.scmoe_expert_ffn_workspace_bytes(B.F32, 64, 256) == 0
    assert B.scmoe_expert_ffn_workspace_bytes(B.BF16, 72, 40) == 0            # not an MFMA shape
    nb = B.scmoe_expert_ffn_workspace_bytes(B.BF16, 2048, 8192)
    assert nb >= 64 << 20 and nb % 16 == 0
    d = B.make_desc(256, 64, 256, 4, 1, 80, B.F32)
    n = B.scmoe_workspace_bytes(d)
    assert n % 256 == 0 and n >= 256 * 256 * 4 * 2
    big = B.make_desc(32768, 2048, 8192, 16, 1, 2560, B.BF16)
    assert B.scmoe_workspace_bytes(big) >= 2 * 32768 * 8192 * 2
    assert B.scmoe_dispatch_workspace_bytes(0, 4, 1) == 0
    assert B.scmoe_dispatch_workspace_bytes(1000, 4, 2) >= 2 * 8 * 4 * 4
    bad = [dict(T=-1), dict(d=0), dict(d=12), dict(F=100), dict(E=0), dict(E=65), dict(capacity=-1),
           dict(dtype=7), dict(k=5), dict(k=0), dict(k=3, E=2), dict(gelu_mode=5), dict(normalize=2), dict(cg_mode=3)]
    base = dict(T=256, d=64, F=256, E=4, k=1, capacity=80, dtype=B.F32)
    for b in bad:
        with pytest.raises(B.ScmoeError):
            B.scmoe_workspace_bytes(B.make_desc(**dict(base, **b)))
    with pytest.raises(B.ScmoeError):                       # top-2 needs two experts
        B.scmoe_workspace_bytes(B.make_desc(**dict(base, E=1, k=2)))


def test_argument_errors_launch_nothing():
    """NULL pointers, bad shapes, misalignment and a short workspace are refused on the host.
    Fake non-NULL addresses are never dereferenced: every call below returns before launch."""
    lib = B.lib()
    P = 0x1000  # aligned fake device address
    st = lib.scmoe_gate_top1(None, 64, B.F32, P, None, 10, 64, 4, 0, P, P, None, None)
    assert st == 1
    assert lib.scmoe_gate_top1(P, 64, 9, P, None, 10, 64, 4, 0, P, P, None, None) == 3
    assert lib.scmoe_gate_top1(P, 64, B.F32, P, None, 10, 60, 4, 0, P, P, None, None) == 2      # d % 8
    assert lib.scmoe_gate_top1(P, 32, B.F32, P, None, 10, 64, 4, 0, P, P, None, None) == 2      # ldx < d
    assert lib.scmoe_gate_top1(P + 4, 64, B.F32, P, None, 10, 64, 4, 0, P, P, None, None) == 2  # alignment
    assert lib.scmoe_gate_top1(P, 64, B.F32, P, None, 10, 64, 65, 0, P, P, None, None) == 2     # E too large
    assert lib.scmoe_gate_top2(P, 64, B.F32, P, None, 10, 64, 1, 0, P, P, None, None) == 2      # k=2, E=1
    assert lib.scmoe_gate_topk(P, 64, B.F32, P, None, 10, 64, 2, 3, 0, P, P, None, None) == 2   # k=3, E=2
    assert lib.scmoe_gate_topk(P, 64, B.F32, P, None, 10, 64, 8, 5, 0, P, P, None, None) == 6   # k too large
    assert lib.scmoe_gate_topk(P, 64, B.F32, P, None, 10, 64, 8, 0, 0, P, P, None, None) == 6
    assert lib.scmoe_gate_topk(None, 64, B.F32, None, None, 0, 64, 4, 3, 0, None, None, None, None) == 0
    assert lib.scmoe_gate_top1(P, 64, B.F32, P, None, 10, 64, 4, 3, P, P, None, None) == 6      # normalize
    assert lib.scmoe_gate_top1(None, 64, B.F32, None, None, 0, 64, 4, 0, None, None, None, None) == 0  # T = 0
    # dispatch: workspace too small, k out of range, NULL outputs
    assert lib.scmoe_dispatch(P, 64, B.F32, P, 1000, 64, 4, 1, 100, P, P, P, P, P, 64, P, 8, None) == 4
    assert lib.scmoe_dispatch(P, 64, B.F32, P, 1000, 64, 4, 5, 100, P, P, P, P, P, 64, P, 1 << 20, None) == 6
    assert lib.scmoe_dispatch(P, 64, B.F32, P, 1000, 64, 4, 1, 100, None, P, P, P, P, 64, P, 1 << 20, None) == 1
    assert lib.scmoe_dispatch(P, 64, B.F32, P, 1000, 64, 4, 1, -1, P, P, P, P, P, 64, P, 1 << 20, None) == 2
    # expert ffn: (x, ld, dtype, offsets, max_rows, E, d, F, W1, ldw1, b1, W2, ldw2, b2, hidden, ldh, y, ldy, gelu,
    #              workspace, ws_bytes, stream)
    ffn = lib.scmoe_expert_ffn
    assert ffn(P, 64, B.BF16, P, 100, 2, 64, 100, P, 64, None, P, 100, None, P, 100, P, 64, 0, None, 0, None) == 2   # F % 8
    assert ffn(P, 64, B.BF16, None, 100, 2, 64, 128, P, 64, None, P, 128, None, P, 128, P, 64, 0, None, 0, None) == 1
    assert ffn(P, 64, B.BF16, P, 100, 2, 64, 128, P, 64, None, P, 128, None, P, 128, P, 64, 4, None, 0, None) == 6
    assert ffn(P, 64, B.BF16, P, 100, 2, 64, 128, P, 56, None, P, 128, None, P, 128, P, 64, 0, None, 0, None) == 2   # ldw1 < d
    assert ffn(P, 64, B.BF16, P, 100, 2, 64, 128, P, 64, None, P, 132, None, P, 128, P, 64, 0, None, 0, None) == 2   # ldw2 % 8
    assert ffn(P, 64, B.BF16, P, 100, 2, 64, 128, P, 64, None, P, 128, None, P, 120, P, 64, 0, None, 0, None) == 2   # ldh < F
    assert ffn(None, 64, B.BF16, None, 0, 2, 64, 128, None, 64, None, None, 128, None, None, 128, None, 64, 0, None, 0, None) == 0
    assert ffn(P, 64, B.BF16, P, 100, 2, 64, 128, P, 64, None, P, 128, None, P, 128, P, 64, 0, P + 8, 1 << 30, None) == 2  # workspace alignment
    # combine / coefficient gate
    assert lib.scmoe_combine(P, 64, B.F32, P, P, 10, 64, 5, None, 0, None, 0, None, P, 64, None) == 6
    assert lib.scmoe_combine(P, 64, B.F32, None, P, 10, 64, 1, None, 0, None, 0, None, P, 64, None) == 1
    assert lib.scmoe_combine(P, 64, B.F32, P, P, 10, 64, 1, P, 8, None, 0, None, P, 64, None) == 2
    assert lib.scmoe_coef_gate(P, 64, B.F32, P, 0, 10, 64, P, None) == 6
    assert lib.scmoe_coef_gate(P, 64, B.F32, None, 1, 10, 64, P, None) == 1
    # layer: short workspace, missing shared weights, k = 2 refused by the ScMoE entry
    desc = B.make_desc(256, 64, 256, 4, 1, 80, B.F32)
    w = B.Weights(P, None, P, None, P, None, P, None, P, None, None, 0, 0)
    need = B.scmoe_workspace_bytes(desc)
    call = lambda d_, w_, ws: lib.scmoe_layer_forward(C.byref(d_), P, 64, P, 64, C.byref(w_), None, 0, P, 64,
                                                      None, P, ws, None, None)
    assert call(desc, w, need - 1) == 4
    assert call(desc, B.Weights(P, None, P, None, P, None, None, None, P, None, None, 0, 0), need) == 1
    assert call(desc, B.Weights(P, None, P, None, P, None, P, None, P, None, None, 60, 0), need) == 2     # ld_w1 < d
    assert call(desc, B.Weights(P, None, P, None, P, None, P, None, P, None, None, 0, 258), need) == 2    # ld_w2 % 4
    assert call(B.make_desc(256, 64, 256, 4, 5, 80, B.F32), w, need * 4) == 6
    assert call(B.make_desc(256, 64, 256, 4, 1, 80, B.F32, cg_mode=1), w, need * 2) == 1      # W_cg missing
    assert lib.moe_top2_layer_forward(C.byref(desc), P, 64, C.byref(w), P, 64, None, P, need, None) == 6
    assert lib.moe_topk_layer_forward(C.byref(desc), P, 64, C.byref(w), P, 64, None, P, 16, None) == 4
    assert lib.scmoe_set_gemm_variant(5) == 6 and lib.scmoe_set_gemm_variant(0) == 0
    # expert offloading: pool size, bad pool / plan arguments (all refused before any GPU call)
    bd = B.make_desc(256, 64, 256, 4, 1, 80, B.BF16)
    assert B.scmoe_offload_pool_bytes(bd, 4) >= 4 * (2 * 64 * 256 * 2 + (256 + 64) * 4)
    assert B.scmoe_offload_pool_bytes(bd, 1) % 256 == 0
    with pytest.raises(B.ScmoeError):
        B.scmoe_offload_pool_bytes(bd, 5)
    needb = B.scmoe_workspace_bytes(bd)
    off = lambda pool, n, asy, plan, w_: lib.scmoe_layer_forward_offload(
        C.byref(bd), P, 64, P, 64, C.byref(w_), pool, n, asy, plan, P, 64, P, needb, None, None)
    assert off(None, 4, 1, P, w) == 1 and off(P, 4, 1, None, w) == 1
    assert off(P, 0, 1, P, w) == 2 and off(P, 5, 1, P, w) == 2
    assert off(P + 16, 4, 1, P, w) == 2                        # pool alignment
    assert off(P, 4, 2, P, w) == 6
    assert off(P, 4, 1, P, B.Weights(P, None, P, None, P, None, P, None, P, None, None, 72, 0)) == 6   # strided host experts


def test_zipf_bias_shapes_the_load():
    """Input recipe of the skewed configuration: the bias gives a Zipf(1.2) top-1 load under
    the generator's own Gaussian model of the logits."""
    E, s = 16, 1.2
    sig = np.full(E, 0.64)
    b = inputs.zipf_bias(sig, s, seed=3)
    rng = np.random.default_rng(0)
    z = rng.standard_normal((200000, E)) * sig
    load = np.bincount(np.argmax(z + b, axis=1), minlength=E) / 200000
    q = np.arange(1, E + 1) ** -s
    q /= q.sum()
    assert np.abs(load - q).max() < 0.01
    assert b.dtype == np.float32 and b.max() == 0.0


def test_stratified_row_sample_covers_every_row_tile(oracle):
    """The row sample of the full-size GPU parity tests (gpu_util.stratified_tokens): on a
    skewed routing with drops, every 128-row block of token order and every 128-row block of
    every expert's packed segment holds a sampled token, and so do each segment's first and
    last row."""
    from gpu_util import stratified_tokens
    T, E, C_ = 5000, 7, 900
    rng = np.random.default_rng(5)
    idx = rng.choice(E, size=(T, 1), p=np.array([.4, .2, .15, .1, .08, .05, .02])).astype(np.int32)
    counts, offsets, dst_row, src_token = oracle.dispatch(idx, E, C_)
    rr = dict(offsets=offsets, src_token=src_token, dst_row=dst_row)
    toks = stratified_tokens(rr, T, E, seed=3)
    assert len(toks) == len(set(toks.tolist())) and toks.min() >= 0 and toks.max() < T
    hit = np.zeros(T, bool)
    hit[toks] = True
    for b0 in range(0, T, 128):
        assert hit[b0:b0 + 128].any()
    assert (dst_row < 0).any() and hit[np.nonzero(dst_row[:, 0] < 0)[0]].any()      # some dropped tokens too
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        assert hit[src_token[lo]] and hit[src_token[hi - 1]]
        for b0 in range(lo, hi, 128):
            assert hit[src_token[b0:min(b0 + 128, hi)]].any()
