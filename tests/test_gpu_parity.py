"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.

Bars: routing indices, counts, offsets and the permutation bit-exact; float outputs within
max|g-r| / max|r| <= 1e-4 (fp32) and 2e-2 (bf16), and at the benchmark sizes also element by
element within tol * (|r| + rms(r)); gate weights within 1e-6.
"""
import numpy as np
import pytest
import torch

from paper_2404_05019_amd import inputs

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2404_05019_amd import binding as B
    from gpu_util import (DEV, TOL, DevLayer, assert_close, assert_routing_equal, relerr, run_layer,
                          stratified_tokens, to_dev, to_host)


def _i32(n, fill=None):
    if fill is None:
        return torch.empty(n, dtype=torch.int32, device=DEV)
    return torch.full((n,), fill, dtype=torch.int32, device=DEV)


# ------------------------------------------------------------------------------------- gate

@pytest.mark.parametrize("T,d,E,dtype,k,use_bias", [
    (256, 64, 4, "f32", 1, False), (1000, 384, 8, "bf16", 1, False), (777, 1024, 16, "bf16", 1, True),
    (130, 72, 3, "f32", 2, True), (513, 264, 64, "bf16", 2, False), (64, 8, 1, "bf16", 1, False),
    (4099, 2048, 16, "bf16", 2, True), (300, 128, 33, "f32", 1, True), (1, 16, 2, "f32", 2, False),
    (1500, 256, 8, "bf16", 3, True), (300, 64, 5, "f32", 4, False), (100, 16, 3, "f32", 3, False),
    (200, 40, 64, "bf16", 4, True),
    (33000, 64, 16, "bf16", 1, True), (32800, 24, 7, "f32", 2, False), (32768, 40, 30, "bf16", 3, True),   # two tokens per lane
    # up to 16 experts (the matrix-core kernel): whole tiles of 256 features plus a rest, with one
    # to eight waves per workgroup, both input types
    (9000, 584, 16, "bf16", 1, True), (5000, 1288, 12, "f32", 2, True), (40000, 520, 16, "bf16", 1, False),
    (2100, 768, 9, "f32", 1, False), (20000, 512, 8, "bf16", 2, False), (17, 2048, 16, "bf16", 1, False),
    (20000, 520, 16, "f32", 1, True), (9000, 264, 5, "f32", 1, False), (6000, 328, 16, "bf16", 1, True),
    # 17 to 64 experts: two or four accumulators per wave, tiles of 128 or 64 features
    (3000, 640, 32, "bf16", 1, True), (40000, 264, 24, "f32", 2, False), (9000, 520, 64, "bf16", 1, False),
    (2000, 1032, 48, "f32", 1, True), (70000, 128, 17, "bf16", 2, False), (20000, 392, 64, "f32", 3, True),
    (5000, 2048, 64, "bf16", 1, False), (12000, 136, 33, "bf16", 4, True),
    # a few tokens with many experts: the one-lane-per-chain kernel
    (100, 72, 40, "f32", 2, True), (60, 520, 64, "bf16", 1, False), (250, 136, 24, "bf16", 3, True)])
@pytest.mark.parametrize("normalize", [0, 1])
def test_gate_parity(oracle, T, d, E, dtype, k, use_bias, normalize):
    rng = np.random.default_rng(T + d + E)
    x = inputs.quantize(rng.standard_normal((T, d)), dtype)
    Wg = (0.02 * rng.standard_normal((d, E))).astype(np.float32)
    bias = (0.3 * rng.standard_normal(E)).astype(np.float32) if use_bias else None
    idx, w, probs = oracle.gate(x, Wg, bias, k, normalize)
    gx, gW, gb = to_dev(x, dtype), to_dev(Wg, "f32"), to_dev(bias, "f32")
    gi, gw = _i32(T * k), torch.empty(T * k, dtype=torch.float32, device=DEV)
    gp = torch.empty((T, E), dtype=torch.float32, device=DEV)
    if k <= 2:
        fn = B.scmoe_gate_top1 if k == 1 else B.scmoe_gate_top2
        fn(gx, gW, gb, gi, gw, gp, normalize=normalize)
        # the general entry point gives the same bits for k = 1 and k = 2
        gi2, gw2 = _i32(T * k), torch.empty(T * k, dtype=torch.float32, device=DEV)
        B.scmoe_gate_topk(gx, gW, gb, k, gi2, gw2, None, normalize=normalize)
        assert torch.equal(gi, gi2) and torch.equal(gw, gw2)
    else:
        B.scmoe_gate_topk(gx, gW, gb, k, gi, gw, gp, normalize=normalize)
    torch.cuda.synchronize()
    assert np.array_equal(gi.cpu().numpy().reshape(T, k), idx)
    assert np.abs(gw.cpu().numpy().reshape(T, k).astype(np.float64) - w).max() <= 1e-6
    assert np.abs(gp.cpu().numpy().astype(np.float64) - probs).max() <= 1e-6


@pytest.mark.parametrize("seed", range(24))
def test_gate_random_shapes(oracle, seed):
    """Seeded sweep of the gate: token counts of every workgroup shape, feature counts that end
    inside a stage, a tile or a step pair, 1 to 64 experts, k up to 4, both input types, strided x."""
    rng = np.random.default_rng(4400 + seed)
    E = int(rng.choice([1, 2, 5, 8, 12, 16, 17, 24, 32, 33, 48, 64]))
    d = 8 * int(rng.integers(1, 140))
    T = int(rng.choice([1, 15, 16, 17, 100, 1000, 4097, 9000, 20001, 40000, 70000]))
    while T * d * E > 3e8:
        T //= 2
    k = int(rng.integers(1, min(E, 4) + 1))
    dtype = "bf16" if rng.integers(0, 2) else "f32"
    normalize = int(rng.integers(0, 2))
    x = inputs.quantize(rng.standard_normal((T, d)), dtype)
    Wg = (0.05 * rng.standard_normal((d, E))).astype(np.float32)
    bias = (0.3 * rng.standard_normal(E)).astype(np.float32) if rng.integers(0, 2) else None
    idx, w, probs = oracle.gate(x, Wg, bias, k, normalize)
    pad = 8 * int(rng.integers(0, 3))                  # x as a view of wider rows
    gfull = torch.zeros((T, d + pad), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device=DEV)
    gfull[:, :d] = to_dev(x, dtype)
    gx = gfull[:, :d]
    gi, gw = _i32(T * k), torch.empty(T * k, dtype=torch.float32, device=DEV)
    gp = torch.empty((T, E), dtype=torch.float32, device=DEV) if rng.integers(0, 2) else None
    B.scmoe_gate_topk(gx, to_dev(Wg, "f32"), to_dev(bias, "f32"), k, gi, gw, gp, normalize=normalize)
    torch.cuda.synchronize()
    assert np.array_equal(gi.cpu().numpy().reshape(T, k), idx)
    assert np.abs(gw.cpu().numpy().reshape(T, k).astype(np.float64) - w).max() <= 1e-6
    if gp is not None:
        assert np.abs(gp.cpu().numpy().astype(np.float64) - probs).max() <= 1e-6


def test_gate_integer_ties_and_strided_view(oracle):
    """Integer inputs: logits exact, many ties, lowest index must win on both sides; x is
    passed as a strided view (ldx > d)."""
    rng = np.random.default_rng(5)
    T, d, E = 700, 16, 6
    x = rng.integers(-2, 3, (T, d)).astype(np.float32)
    Wg = rng.integers(-1, 2, (d, E)).astype(np.float32)
    idx, w, _ = oracle.gate(x, Wg, None, 2, 1)
    big = torch.zeros((T, d + 24), dtype=torch.float32, device=DEV)
    big[:, :d] = torch.from_numpy(x).to(DEV)
    gi, gw = _i32(T * 2), torch.empty(T * 2, dtype=torch.float32, device=DEV)
    B.scmoe_gate_top2(big[:, :d], to_dev(Wg, "f32"), None, gi, gw, None, normalize=1)
    torch.cuda.synchronize()
    assert np.array_equal(gi.cpu().numpy().reshape(T, 2), idx)


@pytest.mark.parametrize("T,d,E,dtype", [(40, 264, 16, "bf16"), (3000, 264, 16, "bf16"), (70000, 72, 8, "f32"),
                                         (600, 136, 40, "bf16"), (40000, 64, 64, "bf16")])
def test_gate_weights_not_16_byte_aligned(oracle, T, d, E, dtype):
    """W_g at an address that is a multiple of 4 but not of 16: the matrix-core kernel copies W_g
    in 16-byte pieces and leaves such calls to the vector-ALU kernels.  Same results."""
    rng = np.random.default_rng(T + E)
    x = inputs.quantize(rng.standard_normal((T, d)), dtype)
    Wg = (0.02 * rng.standard_normal((d, E))).astype(np.float32)
    idx, w, _ = oracle.gate(x, Wg, None, 2, 0)
    buf = torch.zeros(d * E + 1, dtype=torch.float32, device=DEV)
    gW = buf[1:].view(d, E)
    gW.copy_(torch.from_numpy(Wg))
    assert gW.data_ptr() % 16 == 4
    gi, gw = _i32(T * 2), torch.empty(T * 2, dtype=torch.float32, device=DEV)
    B.scmoe_gate_top2(to_dev(x, dtype), gW, None, gi, gw, None, normalize=0)
    torch.cuda.synchronize()
    assert np.array_equal(gi.cpu().numpy().reshape(T, 2), idx)
    assert np.abs(gw.cpu().numpy().reshape(T, 2).astype(np.float64) - w).max() <= 1e-6


def test_gate_nan_rule(oracle):
    """A NaN logit never wins over a number (NaN arrives through the bias)."""
    T, d, E = 64, 8, 4
    x = np.ones((T, d), np.float32)
    Wg = np.tile(np.array([0.1, 0.2, 0.3, 0.25], np.float32), (d, 1))
    bias = np.array([0.0, 0.0, np.nan, 0.0], np.float32)
    idx, _, _ = oracle.gate(x, Wg, bias, 2, 1)
    gi, gw = _i32(T * 2), torch.empty(T * 2, dtype=torch.float32, device=DEV)
    B.scmoe_gate_top2(to_dev(x, "f32"), to_dev(Wg, "f32"), to_dev(bias, "f32"), gi, gw, None)
    torch.cuda.synchronize()
    assert np.array_equal(gi.cpu().numpy().reshape(T, 2), idx)
    assert idx[0].tolist() == [3, 1]


# --------------------------------------------------------------------------------- dispatch

def _run_dispatch(x, idx, E, k, C_, dtype, copy=True):
    T, d = x.shape
    gx = to_dev(x, dtype)
    gi = torch.from_numpy(np.ascontiguousarray(idx, np.int32).reshape(-1)).to(DEV)
    rows = max(min(T * k, E * C_), 1)
    counts, offsets, dst_row = _i32(E), _i32(E + 1), _i32(max(T * k, 1))
    src_token = _i32(rows, -7)
    x_perm = torch.zeros((rows, d), dtype=gx.dtype, device=DEV) if copy else None
    ws = torch.empty(max(B.scmoe_dispatch_workspace_bytes(T, E, k), 16), dtype=torch.uint8, device=DEV)
    B.scmoe_dispatch(gx, gi, E, k, C_, counts, offsets, dst_row, src_token, x_perm, ws)
    torch.cuda.synchronize()
    return (counts.cpu().numpy(), offsets.cpu().numpy(), dst_row.cpu().numpy()[:T * k].reshape(T, k),
            src_token.cpu().numpy(), None if x_perm is None else to_host(x_perm))


@pytest.mark.parametrize("T,E,k,C_,d,dtype", [
    (1, 1, 1, 1, 8, "f32"), (63, 4, 1, 10, 16, "bf16"), (64, 4, 1, 0, 8, "f32"), (257, 4, 1, 257, 24, "bf16"),
    (5000, 8, 1, 700, 64, "bf16"), (5000, 16, 2, 500, 40, "f32"), (1025, 64, 2, 40, 8, "bf16"),
    (4096, 7, 2, 100000, 8, "f32"), (300, 1, 1, 17, 8, "bf16"), (3000, 8, 3, 900, 16, "bf16"),
    (1000, 6, 4, 500, 8, "f32"), (257, 3, 3, 300, 8, "f32"),
    # block boundaries of the one-launch form (blocks of 1024 items): one block, one item past it, two full blocks
    (1024, 8, 1, 100, 8, "f32"), (1025, 5, 1, 300, 8, "f32"), (1024, 16, 2, 90, 8, "bf16"), (683, 9, 3, 200, 8, "f32"),
    # fewer tokens than a wave has lanes with several choices (an item vector spans choices), 64 experts, 33 experts
    (5, 4, 4, 3, 8, "f32"), (40, 6, 3, 100, 8, "bf16"), (4097, 64, 4, 200, 8, "f32"), (9000, 33, 1, 250, 8, "bf16"),
    # the one-launch form's limit of 131072 items: at it, just past it (three kernels with scratch), far past it
    (131072, 16, 1, 9000, 8, "bf16"), (65536, 8, 2, 20000, 8, "f32"), (131073, 16, 1, 9000, 8, "bf16"),
    (43691, 5, 3, 30000, 8, "f32"), (70000, 7, 2, 15000, 8, "bf16"), (400000, 12, 1, 30000, 8, "bf16")])
def test_dispatch_parity(oracle, T, E, k, C_, d, dtype):
    rng = np.random.default_rng(T * 7 + E)
    x = inputs.quantize(rng.standard_normal((T, d)), dtype)
    if k == 1:
        idx = rng.integers(0, E, (T, 1)).astype(np.int32)
    elif k == 2:
        a = rng.integers(0, E, T)
        b = (a + 1 + rng.integers(0, E - 1, T)) % E
        idx = np.stack([a, b], 1).astype(np.int32)
    else:                                             # k distinct experts per token
        idx = np.argsort(rng.random((T, E)), axis=1)[:, :k].astype(np.int32)
    counts, offsets, dst_row, src_token = oracle.dispatch(idx, E, C_)
    gc, go, gd, gs, gxp = _run_dispatch(x, idx, E, k, C_, dtype)
    K = int(offsets[E])
    assert np.array_equal(gc, counts) and np.array_equal(go, offsets)
    assert np.array_equal(gd, dst_row)
    assert np.array_equal(gs[:K], src_token)
    assert (gs[K:] == -7).all()                       # entries past K are left untouched
    assert np.array_equal(gxp[:K], x[src_token])      # raw row copy, bit for bit
    assert (gxp[K:] == 0).all()


def test_dispatch_all_to_one_and_invalid(oracle):
    T, E, C_ = 1000, 5, 300
    x = np.zeros((T, 8), np.float32)
    idx = np.full((T, 1), 3, np.int32)
    idx[5, 0] = -1          # out-of-range entries are dropped, not faults
    idx[6, 0] = E
    counts, offsets, dst_row, src_token = oracle.dispatch(idx, E, C_)
    gc, go, gd, gs, _ = _run_dispatch(x, idx, E, 1, C_, "f32", copy=False)
    assert np.array_equal(gc, counts) and np.array_equal(go, offsets) and np.array_equal(gd, dst_row)
    assert gc.tolist() == [0, 0, 0, 300, 0] and gd[5, 0] == -1 and gd[6, 0] == -1
    assert np.array_equal(gs[:300], src_token)


# ------------------------------------------------------------------------------- expert FFN

def _ffn_case(oracle, E, lens, d, F, dtype, biases, gelu_mode, extra_rows=5, w_scale=0.05, pad=False,
              workspace=False):
    rng = np.random.default_rng(E * 100 + d + F)
    K = int(sum(lens))
    rows = K + extra_rows
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = inputs.quantize(rng.standard_normal((rows, d)), dtype)
    W1 = inputs.quantize(w_scale * rng.standard_normal((E, F, d)), dtype)
    W2 = inputs.quantize(w_scale * rng.standard_normal((E, d, F)), dtype)
    b1 = (0.1 * rng.standard_normal((E, F))).astype(np.float32) if biases else None
    b2 = (0.1 * rng.standard_normal((E, d))).astype(np.float32) if biases else None
    ref = oracle.expert_ffn(x, offsets, W1, W2, b1, b2, gelu_mode=gelu_mode)
    gx = to_dev(x, dtype)
    code = B.BF16 if dtype == "bf16" else B.F32
    # pad: weights and the hidden scratch at the row strides the library recommends
    ld1, ld2 = (B.scmoe_padded_ld(d, code), B.scmoe_padded_ld(F, code)) if pad else (d, F)
    hidden = torch.zeros((rows, ld2), dtype=gx.dtype, device=DEV)[:, :F]
    y = torch.full((rows, d), 7.0, dtype=gx.dtype, device=DEV)
    ws = None
    if workspace:
        ws = torch.full((B.scmoe_expert_ffn_workspace_bytes(code, d, F),), 0x7f, dtype=torch.uint8, device=DEV)
    B.scmoe_expert_ffn(gx, torch.from_numpy(offsets).to(DEV), rows, to_dev(W1, dtype, ld1), to_dev(b1, "f32"),
                       to_dev(W2, dtype, ld2), to_dev(b2, "f32"), hidden, y, gelu_mode=gelu_mode, workspace=ws)
    torch.cuda.synchronize()
    g = to_host(y)
    assert (g[K:] == 7.0).all()                       # rows past offsets[E] are not touched
    if K:
        assert relerr(g[:K], ref[:K]) <= TOL[dtype]
    return g, ref


@pytest.mark.parametrize("E,lens,d,F,dtype,biases,gelu_mode", [
    (4, [64, 60, 70, 62], 64, 256, "f32", False, 0),        # the tiny configuration's shape
    (3, [5, 0, 130], 24, 40, "f32", True, 1),
    (2, [33, 31], 72, 40, "bf16", True, 0),                 # bf16 shape outside the MFMA path
    (1, [300], 64, 64, "bf16", False, 0),
    (3, [300, 0, 517], 128, 320, "bf16", True, 0),          # several tiles, ragged tails, N tail
    (4, [256, 1, 255, 257], 192, 448, "bf16", True, 1),
    (2, [700, 90], 384, 1536, "bf16", False, 0),            # SwinV2-MoE-S stage-3 widths
    (5, [0, 0, 40, 0, 9], 64, 128, "bf16", True, 0)])
def test_expert_ffn_parity(oracle, E, lens, d, F, dtype, biases, gelu_mode):
    _ffn_case(oracle, E, lens, d, F, dtype, biases, gelu_mode)


@pytest.mark.parametrize("E,lens,d,F,dtype", [
    (3, [300, 0, 517], 256, 512, "bf16"),                   # 512- and 1024-byte rows: both get padded
    (2, [130, 70], 128, 384, "f32"),                        # generic kernel with strided weights
    (2, [33, 31], 72, 40, "bf16")])                         # widths the helper leaves dense
def test_expert_ffn_padded_row_strides(oracle, E, lens, d, F, dtype):
    """Weights and hidden scratch stored with padded rows (the padding holds huge values):
    same result as the dense layout."""
    code = B.BF16 if dtype == "bf16" else B.F32
    assert B.scmoe_padded_ld(256, B.BF16) == 320 and B.scmoe_padded_ld(72, B.BF16) == 72
    assert B.scmoe_padded_ld(128, B.F32) == 160 and B.scmoe_padded_ld(2048, B.BF16) == 2112
    g, _ = _ffn_case(oracle, E, lens, d, F, dtype, True, 0, pad=True)
    g0, _ = _ffn_case(oracle, E, lens, d, F, dtype, True, 0, pad=False)
    assert np.array_equal(g, g0)


@pytest.mark.parametrize("E,lens,d,F", [
    (3, [2100, 0, 1900], 128, 4096),      # first GEMM: 17 row tiles x 16 column tiles
    (3, [1900, 2100, 0], 4096, 128),      # second GEMM: the same
    (6, [300, 700, 1, 1500, 256, 1300], 128, 4096)])
@pytest.mark.parametrize("workspace", [False, True])
def test_expert_ffn_many_tiles(oracle, E, lens, d, F, workspace):
    """More than 256 tiles of 256 x 256 in one GEMM, every element compared: the schedule
    then deals chunks of 32 tiles to the 8 XCDs in turn and cuts only the rest into eighths;
    raster groups of several sizes per expert; with a workspace the last round is cut along K."""
    _ffn_case(oracle, E, lens, d, F, "bf16", True, 0, extra_rows=3, workspace=workspace)


@pytest.mark.parametrize("E,lens,d,F,biases,gelu_mode,pad", [
    (4, [3, 0, 7, 1], 128, 256, True, 0, False),
    (1, [32], 64, 64, False, 0, False),
    (8, [1] * 8, 192, 448, True, 1, True),
    (2, [17, 15], 1024, 576, True, 0, False),               # two row subtiles, several k chunks
    (3, [16, 0, 16], 256, 1088, False, 0, True),
    (16, [2, 0, 0, 1, 0, 3, 0, 0, 1, 0, 0, 0, 0, 0, 0, 1], 512, 2048, True, 0, False),
    (16, [100, 3, 0, 0, 17, 64, 1, 0, 0, 0, 0, 0, 0, 0, 0, 40], 256, 576, True, 0, False),   # 64-row blocks
    (8, [0, 65, 0, 0, 16, 33, 0, 14], 128, 320, True, 1, True),
    (64, [5] * 64, 64, 192, False, 0, False),
    (2, [40, 24], 1024, 576, True, 0, False),               # 33-64 rows in all: 64-row blocks, cut along K
    (1, [50], 256, 2048, True, 1, True),
    # the widths of a decode step of the large workload: many parts along K, whose last one to
    # arrive adds them up
    (1, [33], 2048, 8192, True, 0, False), (1, [64], 2048, 8192, False, 0, False), (2, [20, 12], 2048, 4096, True, 0, False)])
@pytest.mark.parametrize("workspace", [False, True])
def test_expert_ffn_few_rows(oracle, E, lens, d, F, biases, gelu_mode, pad, workspace):
    """Calls of at most 64 rows, or of segments averaging at most 16 rows (decode steps), take
    the weight-streaming kernel; with a workspace the small ones are cut along K."""
    _ffn_case(oracle, E, lens, d, F, "bf16", biases, gelu_mode, extra_rows=0, pad=pad, workspace=workspace)


@pytest.mark.parametrize("T,E,k,C_,shared,cg,res", [
    (8, 4, 1, 8, True, 0, False), (20, 8, 1, 3, True, 0, False), (1, 2, 1, 1, True, 0, False),
    (16, 4, 2, 32, False, 0, False), (10, 8, 3, 30, False, 0, False), (32, 16, 1, 32, True, 1, True),
    (12, 4, 2, 5, True, 2, False), (100, 8, 1, 100, True, 0, False), (64, 16, 2, 9, False, 0, False),
    (250, 16, 1, 250, True, 0, False), (48, 8, 1, 48, True, 0, False), (64, 4, 1, 20, True, 1, False)])
def test_layer_decode_batches(oracle, T, E, k, C_, shared, cg, res):
    """Layers of a few tokens (per-token decoding, Sec. 5.3): every GEMM has at most 32 rows."""
    L = inputs.make_layer(T=T, d=256, F=512, E=E, dtype="bf16", seed=300 + T, biases=True, cg_rows=cg,
                          w_scale=0.05)
    _layer_case(oracle, L, "bf16", E, k, C_, shared, normalize=int(k > 1), cg_mode=cg, residual=res)
    if shared:
        _layer_case(oracle, L, "bf16", E, k, C_, shared, normalize=int(k > 1), cg_mode=cg, residual=res,
                    two_streams=True, pad_weights=True)


@pytest.mark.parametrize("seed", range(12))
def test_expert_ffn_random_segments(oracle, seed):
    """Seeded sweep of the MFMA grouped GEMM: 1-10 segments of 0-700 rows (empty ones
    included), widths in multiples of 64, dense or padded strides, with and without the
    split-K workspace, both GELU forms, both tile variants."""
    rng = np.random.default_rng(9000 + seed)
    E = int(rng.integers(1, 11))
    lens = [int(v) for v in rng.integers(0, 701, E) * (rng.random(E) > 0.2)]
    d, F = 64 * int(rng.integers(1, 9)), 64 * int(rng.integers(1, 13))
    B.scmoe_set_gemm_variant(seed % 4)
    try:
        _ffn_case(oracle, E, lens, d, F, "bf16", bool(rng.integers(0, 2)), int(rng.integers(0, 2)),
                  extra_rows=int(rng.integers(0, 9)), pad=bool(rng.integers(0, 2)),
                  workspace=bool(rng.integers(0, 2)))
    finally:
        B.scmoe_set_gemm_variant(0)


def test_expert_ffn_split_k_tail(oracle):
    """Tiles are cut along K from K = 2048 on, when a workspace is given and the last round of
    workgroups is partly filled.  Here both GEMMs have K = 2048 and 296 tiles of 256 x 256 (37
    per XCD on 32 workgroups: 32 whole tiles, then 5 tiles in 6 parts each, added up by finish
    items at the end of the launch); with 128 x 128 tiles 144 per XCD on 128 workgroups.  Every
    element compared with the oracle, for every tile configuration; identical from run to run;
    the workspace may hold anything on entry; and close to the call without a workspace."""
    E, lens, d, F = 3, [4000, 300, 4700], 2048, 2048
    rng = np.random.default_rng(4321)
    K = sum(lens)
    rows = K + 3
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = inputs.quantize(rng.standard_normal((rows, d)), "bf16")
    W1 = inputs.quantize(0.03 * rng.standard_normal((E, F, d)), "bf16")
    W2 = inputs.quantize(0.03 * rng.standard_normal((E, d, F)), "bf16")
    b1 = (0.1 * rng.standard_normal((E, F))).astype(np.float32)
    b2 = (0.1 * rng.standard_normal((E, d))).astype(np.float32)
    ref = oracle.expert_ffn(x, offsets, W1, W2, b1, b2)
    gx, gW1, gW2 = to_dev(x, "bf16"), to_dev(W1, "bf16"), to_dev(W2, "bf16")
    gb1, gb2, goff = to_dev(b1, "f32"), to_dev(b2, "f32"), torch.from_numpy(offsets).to(DEV)

    def run(workspace, fill):
        hidden = torch.zeros((rows, B.scmoe_padded_ld(F, B.BF16)), dtype=torch.bfloat16, device=DEV)[:, :F]
        y = torch.full((rows, d), 7.0, dtype=torch.bfloat16, device=DEV)
        ws = None
        if workspace:
            ws = torch.full((B.scmoe_expert_ffn_workspace_bytes(B.BF16, d, F),), fill, dtype=torch.uint8, device=DEV)
        B.scmoe_expert_ffn(gx, goff, rows, gW1, gb1, gW2, gb2, hidden, y, workspace=ws)
        torch.cuda.synchronize()
        return to_host(y)

    try:
        for variant in (0, 1, 2, 3):
            B.scmoe_set_gemm_variant(variant)
            g1, g2, g0 = run(True, 0x7f), run(True, 0xc3), run(False, 0)
            for g in (g1, g0):
                assert (g[K:] == 7.0).all()
                assert_close(g[:K], ref[:K], "bf16")
            assert np.array_equal(g1, g2)
            assert relerr(g1, g0) <= 1e-2
    finally:
        B.scmoe_set_gemm_variant(0)


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
def test_expert_ffn_tile_variants(oracle, variant):
    """Every tile configuration of the MFMA grouped GEMM meets the same bar."""
    B.scmoe_set_gemm_variant(variant)
    try:
        _ffn_case(oracle, 3, [300, 77, 517], 256, 384, "bf16", True, 0)
        _ffn_case(oracle, 1, [1000], 128, 512, "bf16", False, 0)
    finally:
        B.scmoe_set_gemm_variant(0)


# --------------------------------------------------------------------------- combine / CG

@pytest.mark.parametrize("T,d,k,dtype,use_base,use_res,use_coef", [
    (300, 64, 1, "f32", True, False, False), (257, 384, 1, "bf16", True, True, True),
    (100, 8, 2, "f32", False, False, False), (1000, 1024, 2, "bf16", True, False, True),
    (64, 2048, 1, "bf16", False, True, False), (200, 128, 3, "bf16", True, False, False),
    (90, 64, 4, "f32", True, True, True)])
def test_combine_parity(oracle, T, d, k, dtype, use_base, use_res, use_coef):
    rng = np.random.default_rng(T + d)
    K = T * k // 2 + 1
    yp = inputs.quantize(rng.standard_normal((K, d)), dtype)
    slots = rng.permutation(T * k)
    dst = -np.ones(T * k, np.int32)
    dst[slots[:K]] = rng.permutation(K).astype(np.int32)
    dst = dst.reshape(T, k)
    w = rng.random((T, k)).astype(np.float32)
    base = inputs.quantize(rng.standard_normal((T, d)), dtype) if use_base else None
    res = inputs.quantize(rng.standard_normal((T, d)), dtype) if use_res else None
    coef = rng.random((T, 2)).astype(np.float32) if use_coef else None
    ref = oracle.combine(yp, dst, w, base, res, coef)
    y = torch.empty((T, d), dtype=to_dev(yp, dtype).dtype, device=DEV)
    B.scmoe_combine(to_dev(yp, dtype), torch.from_numpy(dst.reshape(-1)).to(DEV), to_dev(w.reshape(-1), "f32"),
                    k, to_dev(base, dtype), to_dev(res, dtype), to_dev(coef, "f32"), y)
    torch.cuda.synchronize()
    assert relerr(to_host(y), ref) <= (1e-6 if dtype == "f32" else 4e-3)


@pytest.mark.parametrize("mode,dtype,d", [(1, "f32", 64), (2, "bf16", 384), (1, "bf16", 2048), (2, "f32", 72)])
def test_coef_gate_parity(oracle, mode, dtype, d):
    rng = np.random.default_rng(d + mode)
    T = 333
    x = inputs.quantize(rng.standard_normal((T, d)), dtype)
    Wcg = (0.05 * rng.standard_normal((mode, d))).astype(np.float32)
    ref = oracle.coef_gate(x, Wcg, mode)
    coef = torch.empty((T, 2), dtype=torch.float32, device=DEV)
    B.scmoe_coef_gate(to_dev(x, dtype), to_dev(Wcg, "f32"), mode, coef)
    torch.cuda.synchronize()
    assert np.abs(coef.cpu().numpy() - ref).max() <= 1e-5


# -------------------------------------------------------------------------------- the layer

def _layer_case(oracle, L, dtype, E, k, C_, shared, normalize=0, cg_mode=0, gelu_mode=0, residual=False,
                two_streams=False, pad_weights=False):
    D = DevLayer(L, dtype, pad_weights)
    y, r = run_layer(D, k, C_, shared, normalize, cg_mode, gelu_mode, residual, two_streams)
    ref, rr = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=k, capacity_=C_, shared=int(shared),
                                   normalize=normalize, cg_mode=cg_mode, gelu_mode=gelu_mode,
                                   add_residual=int(residual))
    assert_routing_equal(r, rr)
    assert relerr(y, ref) <= TOL[dtype]
    return y, r, ref, rr


@pytest.mark.parametrize("two_streams", [False, True])
def test_layer_tiny_config(oracle, two_streams):
    """BASELINE configuration 1: T=256, d=64, F=256, E=4, fp32, cf 1.25 (C=80)."""
    L, cfg = inputs.make_config("tiny")
    y, r, ref, rr = _layer_case(oracle, L, "f32", cfg["E"], 1, cfg["C"], True, two_streams=two_streams)
    assert cfg["C"] == 80 and int(r["offsets"][-1]) == int((r["dst_row"] >= 0).sum())


@pytest.mark.parametrize("k,shared,C_,normalize,cg,res,gelu", [
    (1, True, 200, 0, 0, False, 0), (1, True, 100000, 0, 1, True, 0), (1, True, 150, 0, 2, False, 1),
    (2, False, 300, 1, 0, False, 0), (2, False, 100000, 0, 0, False, 0), (1, False, 0, 0, 0, False, 0),
    (1, True, 0, 1, 0, False, 0), (3, False, 450, 1, 0, False, 0), (3, False, 100000, 0, 0, False, 1),
    (4, False, 600, 1, 0, False, 0), (3, True, 450, 1, 1, False, 0)])
def test_layer_bf16_mfma_path(oracle, k, shared, C_, normalize, cg, res, gelu):
    """bf16 layer on the MFMA path with gather-on-load: ragged T, binding capacity, drops."""
    L = inputs.make_layer(T=700, d=128, F=256, E=4, dtype="bf16", seed=11 + k, biases=True, cg_rows=cg,
                          w_scale=0.05)
    y, r, ref, rr = _layer_case(oracle, L, "bf16", 4, k, C_, shared, normalize, cg, gelu, res, two_streams=shared,
                                pad_weights=(C_ == 200 or C_ == 300))
    if shared and cg == 0 and not res:
        # dropped tokens: the expert term is exactly zero, so y equals the shared output
        dropped = r["dst_row"][:, 0] < 0
        D = DevLayer(dict(L, W2=np.zeros_like(L["W2"]), b2=np.zeros_like(L["b2"])), "bf16")
        s, _ = run_layer(D, 1, C_, True, normalize)
        assert np.array_equal(y[dropped], s[dropped])


@pytest.mark.parametrize("k,shared,C_,cg,res,two_streams", [
    (1, True, 160, 0, False, False),      # routed second GEMM decodes (scatter, gate weight, add) in finish items
    (1, True, 150, 2, True, False),       # ... and so does the shared expert's (its coefficient, the residual)
    (1, True, 100000, 1, False, True),    # two streams
    (1, False, 150, 0, False, False),     # standard top-1 layer: decode with nothing below
    (2, True, 300, 0, False, False)])     # two routed items per token: plain second GEMMs, combine kernel
def test_layer_tiles_cut_along_k(oracle, k, shared, C_, cg, res, two_streams):
    """A layer whose second GEMMs have K = F = 2048 and only a handful of tiles, so that every
    tile is cut along K and written by finish items: the fused output decodes (scatter and gate
    weight of the routed rows, coefficient and residual of the shared expert's rows) in that
    path.  Every row compared with the oracle."""
    L = inputs.make_layer(T=700, d=256, F=2048, E=4, dtype="bf16", seed=31 + k + cg, biases=True, cg_rows=cg,
                          w_scale=0.03)
    y, r, ref, rr = _layer_case(oracle, L, "bf16", 4, k, C_, shared, 0 if k == 1 else 1, cg, 0, res,
                                two_streams=two_streams)
    assert_close(y, ref, "bf16")
    if C_ < 700:
        assert (r["dst_row"] < 0).any()


def test_scmoe2_two_routed_experts_plus_shared(oracle):
    """ScMoE-2: top-2 routing on x_prev with the shared expert on x_cur."""
    L = inputs.make_layer(T=600, d=128, F=256, E=8, dtype="bf16", seed=51, biases=True, w_scale=0.05)
    _layer_case(oracle, L, "bf16", 8, 2, 120, True, normalize=1)
    _layer_case(oracle, L, "bf16", 8, 2, 100000, True, normalize=0, two_streams=True, pad_weights=True)


def test_layer_f32_generic_path_with_options(oracle):
    L = inputs.make_layer(T=333, d=40, F=72, E=5, dtype="f32", seed=21, biases=True, cg_rows=1, w_scale=0.1)
    _layer_case(oracle, L, "f32", 5, 1, 50, True, cg_mode=1, residual=True)
    _layer_case(oracle, L, "f32", 5, 2, 90, False, normalize=1)


def test_shared_expert_moe_is_scmoe_with_equal_inputs(oracle):
    """Eq. (6) is Eq. (7) with x_prev == x_cur."""
    L = inputs.make_layer(T=500, d=64, F=128, E=4, dtype="bf16", seed=31, w_scale=0.05)
    L["x_prev"] = L["x_cur"]
    _layer_case(oracle, L, "bf16", 4, 1, 200, True)


def test_layer_in_place_output(oracle):
    """y may be the same buffer as x_cur: the layer then must not write y before it has read
    its inputs (the fused decode is skipped for overlapping buffers)."""
    L = inputs.make_layer(T=900, d=128, F=256, E=4, dtype="bf16", seed=61, biases=True, w_scale=0.05)
    D = DevLayer(L, "bf16")
    ref, rr = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=1, capacity_=300, shared=1)
    desc = B.make_desc(D.T, D.d, D.F, D.E, 1, 300, D.code)
    ws = torch.empty(B.scmoe_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    y = D.x_cur.clone()
    B.scmoe_layer_forward(desc, D.x_prev, y, D.weights, y, ws)
    torch.cuda.synchronize()
    assert relerr(to_host(y), ref) <= TOL["bf16"]
    y2 = torch.empty_like(y)
    B.scmoe_layer_forward(desc, D.x_prev, D.x_cur, D.weights, y2, ws)      # separate buffers: fused decode
    torch.cuda.synchronize()
    assert relerr(to_host(y2), ref) <= TOL["bf16"]
    assert relerr(to_host(y2), to_host(y)) <= 1e-2


@pytest.mark.parametrize("cg", [0, 1, 2])
def test_layer_output_in_place_of_the_residual(oracle, cg):
    """y may be the residual's buffer (y = layer(x) + y): the fused decode of the residual and
    coefficient-gate forms is skipped then; with a buffer of its own it runs, same result."""
    L = inputs.make_layer(T=900, d=128, F=256, E=4, dtype="bf16", seed=62 + cg, biases=True, cg_rows=cg, w_scale=0.05)
    D = DevLayer(L, "bf16")
    ref, rr = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=1, capacity_=300, shared=1, cg_mode=cg,
                                   add_residual=1)
    desc = B.make_desc(D.T, D.d, D.F, D.E, 1, 300, D.code, 0, 0, cg)
    ws = torch.empty(B.scmoe_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    y = D.x_cur.clone()
    B.scmoe_layer_forward(desc, D.x_prev, D.x_cur, D.weights, y, ws, residual=y)
    torch.cuda.synchronize()
    assert relerr(to_host(y), ref) <= TOL["bf16"]
    y2 = torch.empty_like(y)
    B.scmoe_layer_forward(desc, D.x_prev, D.x_cur, D.weights, y2, ws, residual=D.x_cur.clone())
    torch.cuda.synchronize()
    assert relerr(to_host(y2), ref) <= TOL["bf16"]
    assert relerr(to_host(y2), to_host(y)) <= 1e-2


@pytest.mark.parametrize("seed", range(24))
def test_layer_random_configurations(oracle, seed):
    """Seeded sweep over shapes and options: widths on and off the MFMA path (multiples of 64
    or not), 1 to 12 experts, k up to 4, binding and loose capacities, both dtypes, both layer
    kinds, every merge mode."""
    rng = np.random.default_rng(7000 + seed)
    dtype = "bf16" if seed % 3 else "f32"
    mfma = dtype == "bf16" and seed % 2 == 0
    step = 64 if mfma else 8
    d = step * int(rng.integers(1, 7 if mfma else 20))
    F = step * int(rng.integers(1, 9 if mfma else 24))
    T = int(rng.integers(1, 900))
    E = int(rng.integers(1, 13))
    k = int(rng.integers(1, min(E, 4) + 1))
    shared = bool(rng.integers(0, 2))
    cg = int(rng.integers(0, 3)) if shared else 0
    C_ = int(rng.choice([0, 1, max(1, T * k // (2 * E)), -(-T * k // E), T * k]))
    L = inputs.make_layer(T=T, d=d, F=F, E=E, dtype=dtype, seed=7100 + seed, biases=bool(rng.integers(0, 2)),
                          cg_rows=cg, w_scale=0.05 if dtype == "bf16" else 0.1,
                          zipf=1.2 if seed % 5 == 0 else None)
    _layer_case(oracle, L, dtype, E, k, C_, shared, normalize=int(rng.integers(0, 2)), cg_mode=cg,
                gelu_mode=int(rng.integers(0, 2)), residual=shared and bool(rng.integers(0, 2)),
                two_streams=shared and bool(rng.integers(0, 2)), pad_weights=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("seed", range(20))
def test_layer_random_small_batches(oracle, seed):
    """Seeded sweep over decode-size calls on the MFMA widths: 1 to 300 tokens, 1 to 64 experts,
    k up to 4: the few-row GEMM in its three forms (32-row and 64-row blocks, cut along K or
    not), the per-chain gate, the tiled GEMM with 128-row tiles and forced split-K."""
    rng = np.random.default_rng(8000 + seed)
    T = int(rng.choice([1, 2, 7, 16, 31, 32, 33, 48, 64, 65, 100, 129, 200, 300]))
    E = int(rng.choice([1, 2, 3, 8, 16, 40, 64]))
    k = int(rng.integers(1, min(E, 4) + 1))
    d, F = 64 * int(rng.integers(1, 6)), 64 * int(rng.integers(1, 10))
    shared = bool(rng.integers(0, 2))
    cg = int(rng.integers(0, 3)) if shared else 0
    C_ = int(rng.choice([1, max(1, T * k // (2 * E)), -(-T * k // E), T * k]))
    L = inputs.make_layer(T=T, d=d, F=F, E=E, dtype="bf16", seed=8100 + seed, biases=bool(rng.integers(0, 2)),
                          cg_rows=cg, w_scale=0.05)
    _layer_case(oracle, L, "bf16", E, k, C_, shared, normalize=int(rng.integers(0, 2)), cg_mode=cg,
                gelu_mode=int(rng.integers(0, 2)), residual=shared and bool(rng.integers(0, 2)),
                two_streams=shared and bool(rng.integers(0, 2)), pad_weights=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("two_streams", [False, True])
def test_layer_in_a_hip_graph(oracle, two_streams):
    """The layer call makes no host synchronisation, allocates nothing and clears its
    counters with a kernel, so a caller can capture it in a HIP graph.  The graph is replayed
    on changing inputs with eager work and synchronisations in between; every replay must give
    the bits of the eager call on the same inputs."""
    L = inputs.make_layer(T=700, d=128, F=256, E=4, dtype="bf16", seed=77, biases=True, w_scale=0.05)
    D = DevLayer(L, "bf16")
    desc = B.make_desc(D.T, D.d, D.F, D.E, 1, 200, D.code)
    ws = torch.empty(B.scmoe_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    ws_eager = torch.empty_like(ws)
    xp, xc = D.x_prev.clone(), D.x_cur.clone()
    y = torch.empty((D.T, D.d), dtype=D.tdtype, device=DEV)
    y_eager = torch.empty_like(y)
    aux = torch.cuda.Stream() if two_streams else None
    B.scmoe_layer_forward(desc, xp, xc, D.weights, y, ws, stream_aux=aux)     # first call: one-time set-up
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.scmoe_layer_forward(desc, xp, xc, D.weights, y, ws, stream_aux=aux)
    ref, _ = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=1, capacity_=200, shared=1)
    for rep in range(4):
        if rep:
            xp.copy_(torch.roll(D.x_prev, rep, 0))
            xc.copy_(torch.roll(D.x_cur, 2 * rep, 0))
        y.fill_(3.0)
        g.replay()
        torch.cuda.synchronize()
        B.scmoe_layer_forward(desc, xp, xc, D.weights, y_eager, ws_eager, stream_aux=aux)
        torch.cuda.synchronize()
        assert torch.equal(y, y_eager), "replay %d differs from the eager call" % rep
        if rep == 0:
            assert relerr(to_host(y), ref) <= TOL["bf16"]


def test_layer_is_deterministic(oracle):
    """The same call gives the same bits every time.  One- and two-stream mode launch the
    GEMMs differently (which tiles end up in a split-K tail differs), so across the modes the
    routing is identical and the output equal up to that rounding."""
    L = inputs.make_layer(T=3000, d=128, F=256, E=8, dtype="bf16", seed=41, w_scale=0.05)
    D = DevLayer(L, "bf16")
    outs = [run_layer(D, 1, 300, True, two_streams=(i % 2 == 1)) for i in range(4)]
    for i, (y, r) in enumerate(outs[1:], 1):
        if i % 2 == 0:
            assert np.array_equal(y, outs[0][0])
        else:
            assert np.array_equal(y, outs[1][0]) and relerr(y, outs[0][0]) <= 1e-2
        for key in ("idx", "counts", "offsets", "dst_row", "src_token", "w"):
            assert np.array_equal(r[key], outs[0][1][key])


# ------------------------------------------------------------------ expert offloading

def _offload_case(oracle, T, E, k, C_, pool_experts, async_copy, seed):
    """Routed experts in pinned host memory, migrated on demand: the same from call to call,
    the resident layer's numbers up to the rounding of a different tile schedule (which tiles
    of a GEMM fall into the split-K tail depends on what shares the launch), and within the
    bar of the oracle."""
    L = inputs.make_layer(T=T, d=128, F=256, E=E, dtype="bf16", seed=seed, biases=True, w_scale=0.05)
    D = DevLayer(L, "bf16")
    desc = B.make_desc(T, D.d, D.F, E, k, C_, D.code)
    ws = torch.empty(B.scmoe_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    # resident reference through the combine path (y in place of a copy of x_cur: no fused decode)
    y_res = D.x_cur.clone()
    B.scmoe_layer_forward(desc, D.x_prev, y_res, D.weights, y_res, ws)
    torch.cuda.synchronize()
    host = lambda t: None if t is None else t.cpu().pin_memory()
    hW1, hW2, hb1, hb2 = host(D.W1), host(D.W2), host(D.b1), host(D.b2)
    wts = B.make_weights(D.Wg, hW1, hW2, D.W1s, D.W2s, D.bias, hb1, hb2, D.b1s, D.b2s, D.Wcg)
    pool = torch.full((B.scmoe_offload_pool_bytes(desc, pool_experts),), 0x7f, dtype=torch.uint8, device=DEV)
    plan = torch.zeros(2 * E + 1, dtype=torch.int32).pin_memory()
    y = torch.empty((T, D.d), dtype=D.tdtype, device=DEV)
    copy_stream = torch.cuda.Stream()
    first = None
    for _ in range(2):                                   # the pool is reused from call to call
        B.scmoe_layer_forward_offload(desc, D.x_prev, D.x_cur, wts, pool, pool_experts, plan, y, ws,
                                      async_copy=async_copy, stream_copy=copy_stream)
        torch.cuda.synchronize()
        assert relerr(to_host(y), to_host(y_res)) <= 1e-2
        assert first is None or torch.equal(y, first)
        first = y.clone()
    ref, rr = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=k, capacity_=C_, shared=1,
                                   normalize=0)
    assert relerr(to_host(y), ref) <= TOL["bf16"]
    assert np.array_equal(plan[:E].numpy(), rr["counts"])
    # The two halves as calls of their own, with work of the caller on the main stream in between
    # (the window the migration hides in): the same bits as the single call.
    y2 = torch.full_like(y, float("nan"))
    filler_a = torch.randn((512, 512), device=DEV)
    pool.fill_(0x7f)
    B.scmoe_offload_begin(desc, D.x_prev, wts, pool, pool_experts, plan, ws, async_copy=async_copy,
                          stream_copy=copy_stream)
    filler_b = filler_a @ filler_a
    B.scmoe_offload_finish(desc, D.x_prev, D.x_cur, wts, pool, pool_experts, plan, y2, ws, async_copy=async_copy,
                           stream_copy=copy_stream)
    torch.cuda.synchronize()
    assert torch.equal(y2, first) and bool(torch.isfinite(filler_b).all())
    return plan[:E].numpy()


@pytest.mark.parametrize("async_copy", [True, False])
def test_offload_matches_resident_layer(oracle, async_copy):
    _offload_case(oracle, 700, 4, 1, 300, 4, async_copy, seed=71)
    _offload_case(oracle, 600, 8, 2, 200, 8, async_copy, seed=72)          # ScMoE-2 routing


def test_offload_decode_step_migrates_only_selected_experts(oracle):
    """A decode-like step: 3 tokens select at most 3 of 8 experts, and a pool of 3 is enough."""
    counts = _offload_case(oracle, 3, 8, 1, 3, 3, True, seed=73)
    assert (counts > 0).sum() <= 3 and counts.sum() == 3


def test_offload_pool_too_small_is_an_error(oracle):
    L = inputs.make_layer(T=500, d=128, F=256, E=8, dtype="bf16", seed=74, w_scale=0.05)
    D = DevLayer(L, "bf16")
    desc = B.make_desc(500, D.d, D.F, 8, 1, 500, D.code)
    ws = torch.empty(B.scmoe_workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    host = lambda t: None if t is None else t.cpu().pin_memory()
    wts = B.make_weights(D.Wg, host(D.W1), host(D.W2), D.W1s, D.W2s, D.bias, None, None, D.b1s, D.b2s, None)
    pool = torch.empty(B.scmoe_offload_pool_bytes(desc, 2), dtype=torch.uint8, device=DEV)
    plan = torch.zeros(17, dtype=torch.int32).pin_memory()
    y = torch.empty((500, D.d), dtype=D.tdtype, device=DEV)
    with pytest.raises(B.ScmoeError) as e:                # 500 tokens select more than 2 of 8 experts
        B.scmoe_layer_forward_offload(desc, D.x_prev, D.x_cur, wts, pool, 2, plan, y, ws)
    assert e.value.status == 4
    with pytest.raises(B.ScmoeError) as e:
        B.scmoe_offload_begin(desc, D.x_prev, wts, pool, 2, plan, ws)
    assert e.value.status == 4 and int(plan[:8].sum()) == 500     # (the counts are on the host by then)
    with pytest.raises(B.ScmoeError) as e:                # and a finish on such a plan refuses too
        B.scmoe_offload_finish(desc, D.x_prev, D.x_cur, wts, pool, 2, plan, y, ws)
    assert e.value.status == 4
    torch.cuda.synchronize()


# --------------------------------------------------- full benchmark sizes

def _full_size(oracle, name, dense=False, k=1, shared=True, normalize=0, pad_weights=False, two_streams=False,
               cg_mode=0, residual=False):
    """Routing compared for every token.  Output rows: all of them (dense), or a seeded sample
    that takes a row from every row tile of both chains (gpu_util.stratified_tokens); both readings
    of the parity bar are asserted.  One stream is what bench.py times."""
    L, cfg = inputs.make_config(name)
    T, E = cfg["T"], cfg["E"]
    if cg_mode:
        L["Wcg"] = (0.02 * np.random.default_rng(77).standard_normal((2, L["x_cur"].shape[1]))).astype(np.float32)
    C_ = inputs.capacity(T, E, k, cfg["cf"])
    D = DevLayer(L, cfg["dtype"], pad_weights)
    y, r = run_layer(D, k, C_, shared, normalize, cg_mode=cg_mode, residual=residual,
                     two_streams=two_streams and shared)
    xg = L["x_prev"] if shared else L["x_cur"]
    rr = oracle.route(xg, L, E, k, C_, normalize)
    assert_routing_equal(r, rr)
    assert (r["counts"] <= C_).all() and r["counts"].sum() == (r["dst_row"] >= 0).sum()
    tokens = np.arange(T, dtype=np.int32) if dense else stratified_tokens(rr, T, E, seed=1234)
    ref = oracle.layer_rows(L["x_prev"], L["x_cur"], L, rr, tokens, k=k, shared=int(shared), cg_mode=cg_mode,
                            add_residual=int(residual))
    assert_close(y[tokens], ref, cfg["dtype"])
    return cfg, r


def test_full_size_small(oracle):
    cfg, r = _full_size(oracle, "small", dense=True)
    assert cfg["C"] == 1280 and int(r["offsets"][-1]) == cfg["T"]      # near-uniform: no drops


def test_full_size_medium_and_top2_baseline(oracle):
    cfg, r = _full_size(oracle, "medium", dense=True)
    assert cfg["C"] == 2560
    cfg2, r2 = _full_size(oracle, "medium", k=2, shared=False, normalize=1)
    assert int(r2["offsets"][-1]) <= 2 * cfg["T"]


def test_full_size_medium_top3_and_scmoe2(oracle):
    """The two layers of equal compute volume that Table 4 sets side by side: the standard
    top-3 layer and ScMoE-2 (two routed experts on x_prev plus the shared expert)."""
    cfg3, r3 = _full_size(oracle, "medium", k=3, shared=False, normalize=1)
    assert int(r3["offsets"][-1]) <= 3 * cfg3["T"]
    assert (np.sort(r3["idx"], axis=1)[:, 1:] != np.sort(r3["idx"], axis=1)[:, :-1]).all()   # distinct experts
    _full_size(oracle, "medium", k=2, shared=True, normalize=1)


def test_full_size_skewed(oracle):
    """Zipf(1.2) expert load with capacity factor 1.0: a large share of tokens is dropped."""
    cfg, r = _full_size(oracle, "skewed", two_streams=True)
    kept = int(r["offsets"][-1])
    assert cfg["C"] == 1024 and 0.4 * cfg["T"] < kept < 0.75 * cfg["T"]
    assert (r["counts"][:3] == 1024).all()


def test_full_size_skewed_other_fused_forms(oracle):
    """The skewed load (nearly half of the tokens dropped) through the other layers whose
    decode is fused into the second GEMM: coefficient gate CG-2 with a residual (the shared
    expert's rows are scaled and added to in place, the routed rows carry the routed
    coefficient), and the standard top-1 layer (dropped tokens' rows are zeroed)."""
    _full_size(oracle, "skewed", cg_mode=2, residual=True)
    _full_size(oracle, "skewed", cg_mode=1)
    cfg, r = _full_size(oracle, "skewed", shared=False)
    assert int(r["offsets"][-1]) < 0.75 * cfg["T"]


@pytest.mark.parametrize("pad_weights", [True, False])
def test_full_size_large(oracle, pad_weights):
    """The benchmark workload: dense weight rows on one stream (the configuration bench.py times),
    and padded rows with the shared expert on a second stream."""
    cfg, r = _full_size(oracle, "large", pad_weights=pad_weights, two_streams=pad_weights)
    assert cfg["C"] == 2560
