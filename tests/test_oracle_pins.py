"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test ties one part of oracle/scmoe_oracle.c to a closed form, a textbook value, a
library routine, an invariant of the paper's equations, or a brute force written
independently in Python.  Citations name the passage of the ScMoE paper the pinned
function follows.
"""
import math
import os

import numpy as np
import pytest
import torch

from paper_2404_05019_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _phi_table():
    tab = {}
    with open(os.path.join(GOLDEN, "normal_cdf.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            v, p = line.split()
            tab[float(v)] = float(p)
    return tab


# ----------------------------------------------------------------------------- gate (Eq. 2-4)

def test_gate_zero_matrix_uniform(oracle):
    """W_g = 0: all logits equal, so expert 0 wins (lowest index) and p = 1/E exactly."""
    rng = np.random.default_rng(0)
    x = rng.standard_normal((37, 24)).astype(np.float32)
    for E in (1, 2, 5, 16):
        idx, w, probs = oracle.gate(x, np.zeros((24, E), np.float32))
        assert (idx == 0).all()
        assert np.array_equal(probs, np.full((37, E), np.float32(1.0 / E)))
        assert np.array_equal(w[:, 0], probs[:, 0])


def test_gate_one_hot_column(oracle):
    """Only column e* non-zero and positive, x > 0: every token goes to e*."""
    rng = np.random.default_rng(1)
    x = np.abs(rng.standard_normal((50, 16))).astype(np.float32) + 0.1
    for estar in (0, 3, 6):
        Wg = np.zeros((16, 7), np.float32)
        Wg[:, estar] = 0.5
        idx, w, probs = oracle.gate(x, Wg)
        assert (idx[:, 0] == estar).all()
        assert np.allclose(probs.sum(1), 1.0, atol=1e-6)


def test_gate_integer_inputs_exact_with_ties(oracle):
    """Small-integer x and W_g make every partial sum exact in fp32, so the logits must equal
    an integer matmul and the choice must be the first maximum, ties included (Eq. (3))."""
    rng = np.random.default_rng(2)
    T, d, E = 300, 12, 6
    x = rng.integers(-2, 3, (T, d))
    Wg = rng.integers(-1, 2, (d, E))
    bias = rng.integers(-1, 2, E)
    ref = x @ Wg + bias[None, :]
    logits = oracle.gate_logits(x.astype(np.float32), Wg.astype(np.float32), bias.astype(np.float32))
    assert np.array_equal(logits.astype(np.int64), ref)
    n_ties = int((np.sort(ref, 1)[:, -1] == np.sort(ref, 1)[:, -2]).sum())
    assert n_ties > 10  # the case really contains ties
    idx, w, _ = oracle.gate_topk(logits, k=2)
    # brute force: first choice = first maximum; second = first maximum of the rest
    for t in range(T):
        row = list(ref[t])
        e1 = row.index(max(row))
        rest = [(v, e) for e, v in enumerate(row) if e != e1]
        m2 = max(v for v, _ in rest)
        e2 = min(e for v, e in rest if v == m2)
        assert idx[t, 0] == e1 and idx[t, 1] == e2
    idx1, _, _ = oracle.gate_topk(logits, k=1)
    assert np.array_equal(idx1[:, 0], np.argmax(ref, axis=1))


def test_gate_logit_chain_order_and_fma(oracle):
    """The logit is an ascending single-FMA chain in fp32 (a stated reading of Eq. (4)).
    Case 1: 2^24 + 1 - 2^24 is 0 in ascending order (1 is absorbed), 1 in any order that
    cancels first.  Case 2: a product whose low bits survive only under a fused
    multiply-add: (1+2^-12)^2 - (1+2^-11) = 2^-24."""
    x = np.array([[2.0 ** 24, 1.0, -(2.0 ** 24)]], np.float32)
    Wg = np.ones((3, 1), np.float32)
    assert oracle.gate_logits(x, Wg)[0, 0] == 0.0
    x2 = np.array([[1.0, -1.0, 2.0 ** 24]], np.float32)[:, ::-1].copy()  # 2^24, -1... reversed
    assert oracle.gate_logits(x2, Wg)[0, 0] == np.float32(2.0 ** 24 - 1.0) + np.float32(1.0)
    a = np.float32(1.0 + 2.0 ** -12)
    x3 = np.array([[-(1.0 + 2.0 ** -11), a]], np.float32)
    W3 = np.array([[1.0], [a]], np.float32)
    assert oracle.gate_logits(x3, W3)[0, 0] == np.float32(2.0 ** -24)
    # bias is added last with one rounding
    b = np.array([2.0 ** -30], np.float32)
    assert oracle.gate_logits(x3, W3, b)[0, 0] == np.float32(2.0 ** -24) + np.float32(2.0 ** -30)


def test_gate_random_vs_fp64_matmul(oracle):
    """Random inputs: fp32 chain logits are within rounding of numpy's fp64 matmul, and
    the arg max agrees wherever the fp64 margin is not tiny (non-fragile tokens)."""
    rng = np.random.default_rng(3)
    T, d, E = 2000, 96, 8
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (0.02 * rng.standard_normal((d, E))).astype(np.float32)
    bias = (0.1 * rng.standard_normal(E)).astype(np.float32)
    ref = x.astype(np.float64) @ Wg.astype(np.float64) + bias.astype(np.float64)
    logits = oracle.gate_logits(x, Wg, bias)
    scale = np.abs(x.astype(np.float64)) @ np.abs(Wg.astype(np.float64)) + 1.0
    assert (np.abs(logits - ref) <= d * 2.0 ** -24 * scale).all()
    assert np.allclose(oracle.gate_logits_f64(x, Wg, bias), ref, rtol=0, atol=1e-12)
    idx, w, probs = oracle.gate_topk(logits, k=1)
    srt = np.sort(ref, axis=1)
    margin = srt[:, -1] - srt[:, -2]
    safe = margin > 2.0 ** -20 * scale.max(axis=1)
    assert safe.sum() > 0.95 * T
    assert np.array_equal(idx[safe, 0], np.argmax(ref, axis=1)[safe])


def test_gate_probs_against_torch_softmax(oracle):
    """Eq. (2) with k = E is a plain softmax: check against torch's fp64 softmax; the
    top-1 weight is the largest probability."""
    rng = np.random.default_rng(4)
    logits = (3.0 * rng.standard_normal((500, 11))).astype(np.float32)
    idx, w, probs = oracle.gate_topk(logits, k=1)
    ref = torch.softmax(torch.from_numpy(logits).double(), dim=1).numpy()
    assert np.allclose(probs, ref, rtol=0, atol=1e-7)
    assert np.allclose(probs.sum(1), 1.0, atol=1e-6)
    assert np.allclose(w[:, 0], ref.max(1), atol=1e-7)
    assert np.array_equal(idx[:, 0], ref.argmax(1))


def test_gate_top2_weights_closed_form(oracle):
    """Eq. (2) with k = 2: softmax over the two selected logits == p_j / (p_1 + p_2);
    normalize=0 returns the raw full-softmax entries; k=1 normalize=1 gives weight 1."""
    rng = np.random.default_rng(5)
    logits = (2.0 * rng.standard_normal((400, 9))).astype(np.float32)
    idx, w, probs = oracle.gate_topk(logits, k=2, normalize=1)
    p = torch.softmax(torch.from_numpy(logits).double(), dim=1).numpy()
    order = np.argsort(-logits, axis=1, kind="stable")
    assert np.array_equal(idx, order[:, :2])
    p1 = np.take_along_axis(p, idx[:, :1], 1)[:, 0]
    p2 = np.take_along_axis(p, idx[:, 1:2], 1)[:, 0]
    assert np.allclose(w[:, 0], p1 / (p1 + p2), atol=1e-7)
    assert np.allclose(w[:, 1], p2 / (p1 + p2), atol=1e-7)
    assert np.allclose(w.sum(1), 1.0, atol=1e-6)
    _, w0, _ = oracle.gate_topk(logits, k=2, normalize=0)
    assert np.allclose(w0[:, 0], p1, atol=1e-7) and np.allclose(w0[:, 1], p2, atol=1e-7)
    _, w1, _ = oracle.gate_topk(logits, k=1, normalize=1)
    assert (w1 == 1.0).all()


@pytest.mark.parametrize("k", [3, 4, 7])
def test_gate_topk_general(oracle, k):
    """Eq. (2)-(3) for k > 2 (the top-3 baseline of Table 4): the selection is the k largest
    logits in descending order (a stable sort gives the lowest index among equals), the
    normalised weights are p_j / sum of the selected p, the raw ones the softmax entries."""
    rng = np.random.default_rng(50 + k)
    logits = (2.0 * rng.standard_normal((300, 7))).astype(np.float32)
    logits[::5] = np.round(logits[::5])                       # rows with ties
    idx, w, probs = oracle.gate_topk(logits, k=k, normalize=1)
    order = np.argsort(-logits, axis=1, kind="stable")[:, :k]
    assert np.array_equal(idx, order)
    p = torch.softmax(torch.from_numpy(logits).double(), dim=1).numpy()
    ps = np.take_along_axis(p, order, 1)
    assert np.allclose(w, ps / ps.sum(1, keepdims=True), atol=1e-7)
    _, w0, _ = oracle.gate_topk(logits, k=k, normalize=0)
    assert np.allclose(w0, ps, atol=1e-7)
    if k == 7:                                                # k = E: the plain softmax, sorted
        assert np.allclose(w, ps, atol=1e-7)
        assert (np.sort(idx, axis=1) == np.arange(7)).all()


def test_gate_nan_never_wins(oracle):
    nan = np.float32("nan")
    logits = np.array([[nan, 1.0, 2.0], [0.5, nan, 0.5], [nan, nan, nan], [nan, -5.0, nan]], np.float32)
    idx, _, _ = oracle.gate_topk(logits, k=2)
    assert idx.tolist() == [[2, 1], [0, 2], [0, 1], [1, 0]]
    idx, _, _ = oracle.gate_topk(logits, k=3)
    assert idx.tolist() == [[2, 1, 0], [0, 2, 1], [0, 1, 2], [1, 0, 2]]


# ------------------------------------------------------------------ dispatch (Sec. 2.2 encode)

def _dispatch_bruteforce(idx, E, C):
    """O(n^2) statement of the drop rule: an item is kept iff fewer than C earlier items
    (first choices before second choices, then token order) chose the same expert."""
    T, k = idx.shape
    items = [(j, t) for j in range(k) for t in range(T)]
    slot = {}
    for n, (j, t) in enumerate(items):
        e = idx[t, j]
        earlier = sum(1 for (jj, tt) in items[:n] if idx[tt, jj] == e)
        slot[(t, j)] = earlier
    counts = [min(sum(1 for it in items if idx[it[1], it[0]] == e), C) for e in range(E)]
    offsets = [0]
    for c in counts:
        offsets.append(offsets[-1] + c)
    dst = -np.ones((T, k), np.int64)
    for (t, j), s in slot.items():
        if s < C:
            dst[t, j] = offsets[idx[t, j]] + s
    return np.array(counts), np.array(offsets), dst


@pytest.mark.parametrize("T,E,k,C", [(1, 1, 1, 1), (70, 4, 1, 10), (70, 4, 1, 0), (70, 4, 1, 70),
                                     (65, 3, 2, 20), (130, 5, 2, 1000), (64, 1, 1, 17),
                                     (65, 5, 3, 20), (40, 6, 4, 9)])
def test_dispatch_bruteforce(oracle, T, E, k, C):
    rng = np.random.default_rng(T * 31 + E)
    if k == 1:
        idx = rng.integers(0, E, (T, 1)).astype(np.int32)
    else:
        idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    counts, offsets, dst_row, src_token = oracle.dispatch(idx, E, C)
    bc, bo, bd = _dispatch_bruteforce(idx, E, C)
    assert np.array_equal(counts, bc) and np.array_equal(offsets, bo) and np.array_equal(dst_row, bd)
    # invariants
    K = int(offsets[E])
    assert K == int((dst_row >= 0).sum()) == int(counts.sum()) == len(src_token)
    assert (counts <= C).all()
    kept = dst_row[dst_row >= 0]
    assert sorted(kept.tolist()) == list(range(K))            # a permutation of the packed rows
    for t in range(T):
        for j in range(k):
            if dst_row[t, j] >= 0:
                assert src_token[dst_row[t, j]] == t
    if k == 1:
        for e in range(E):                                    # stability: token order inside a segment
            seg = src_token[offsets[e]:offsets[e + 1]]
            assert (np.diff(seg) > 0).all()
            assert (idx[seg, 0] == e).all()


def test_dispatch_all_to_one_expert(oracle):
    T, E, C = 100, 4, 30
    idx = np.full((T, 1), 2, np.int32)
    counts, offsets, dst_row, src_token = oracle.dispatch(idx, E, C)
    assert counts.tolist() == [0, 0, 30, 0] and offsets.tolist() == [0, 0, 0, 30, 30]
    assert dst_row[:30, 0].tolist() == list(range(30)) and (dst_row[30:] == -1).all()
    assert src_token.tolist() == list(range(30))


def test_dispatch_top2_first_choices_fill_first(oracle):
    """A saturated expert takes no second choices: with C first choices already there,
    every second choice for it is dropped even from early tokens."""
    T, E, C = 8, 2, 8
    idx = np.array([[0, 1]] * 8, np.int32)
    counts, offsets, dst_row, _ = oracle.dispatch(idx, E, C)
    assert counts.tolist() == [8, 8]
    idx[:, 1] = 0  # (degenerate) both choices expert 0: second choices all dropped
    counts, offsets, dst_row, _ = oracle.dispatch(idx, E, C)
    assert counts.tolist() == [8, 0] and (dst_row[:, 1] == -1).all() and (dst_row[:, 0] >= 0).all()


def test_capacity_formula(oracle):
    """C = ceil(cf*k*T/E); the five benchmark shapes give exact integers."""
    cases = [(256, 4, 1, 1.25, 80), (8192, 8, 1, 1.25, 1280), (16384, 8, 1, 1.25, 2560),
             (16384, 8, 2, 1.25, 5120), (16384, 16, 1, 1.0, 1024), (32768, 16, 1, 1.25, 2560),
             (10, 3, 1, 1.0, 4), (7, 2, 1, 1.1, 4), (100, 8, 2, 2.0, 50)]
    for T, E, k, cf, C in cases:
        assert oracle.capacity(T, E, k, cf) == C
        assert inputs.capacity(T, E, k, cf) == C
        assert C == math.ceil(round(cf * 100) * k * T / (100 * E) - 1e-12)


# ------------------------------------------------------------------ experts (Eq. 1, Sec. 2.1)

def test_gelu_textbook_values(oracle):
    """Exact GELU is v*Phi(v): textbook normal-CDF values (tests/golden/normal_cdf.txt)."""
    for v, phi in _phi_table().items():
        assert abs(oracle.gelu(v, 0) - v * phi) < 2e-15
    for v in (0.1, 0.7, 2.5, 6.0):
        assert abs((oracle.gelu(v, 0) - oracle.gelu(-v, 0)) - v) < 1e-15   # odd-part identity
    assert oracle.gelu(0.0, 0) == 0.0 and oracle.gelu(0.0, 1) == 0.0
    assert abs(oracle.gelu(40.0, 0) - 40.0) < 1e-12 and abs(oracle.gelu(-40.0, 0)) < 1e-12
    t = torch.tensor([-3.0, -0.5, 0.3, 1.7, 4.0], dtype=torch.float64)
    ref = torch.nn.functional.gelu(t, approximate="tanh")
    for v, r in zip(t.tolist(), ref.tolist()):
        assert abs(oracle.gelu(v, 1) - r) < 1e-14


@pytest.mark.parametrize("gelu_mode,approx", [(0, "none"), (1, "tanh")])
def test_expert_ffn_matches_torch_fp64(oracle, gelu_mode, approx):
    """Segments through experts == torch fp64 linear -> gelu -> linear per segment.  d != F
    and random biases, so a transposed operand or a dropped bias fails.  E = 1 with one
    segment is the dense MLP / shared expert."""
    rng = np.random.default_rng(7)
    for E, d, F, lens in [(1, 24, 40, [33]), (3, 16, 56, [5, 0, 12]), (4, 8, 8, [1, 2, 3, 4])]:
        K = sum(lens)
        offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        x = rng.standard_normal((K + 3, d)).astype(np.float32)       # 3 rows past offsets[E]
        W1 = (0.3 * rng.standard_normal((E, F, d))).astype(np.float32)
        W2 = (0.3 * rng.standard_normal((E, d, F))).astype(np.float32)
        b1 = (0.3 * rng.standard_normal((E, F))).astype(np.float32)
        b2 = (0.3 * rng.standard_normal((E, d))).astype(np.float32)
        y = oracle.expert_ffn(x, offsets, W1, W2, b1, b2, gelu_mode=gelu_mode)
        assert (y[K:] == 0).all()
        tx = torch.from_numpy(x).double()
        for e in range(E):
            seg = slice(offsets[e], offsets[e + 1])
            h = torch.nn.functional.gelu(
                torch.nn.functional.linear(tx[seg], torch.from_numpy(W1[e]).double(), torch.from_numpy(b1[e]).double()),
                approximate=approx)
            ref = torch.nn.functional.linear(h, torch.from_numpy(W2[e]).double(), torch.from_numpy(b2[e]).double())
            assert np.allclose(y[seg], ref.numpy(), rtol=1e-12, atol=1e-13)
        y0 = oracle.expert_ffn(x, offsets, W1, W2, None, None, gelu_mode=gelu_mode)
        h = torch.nn.functional.gelu(tx[:lens[0]] @ torch.from_numpy(W1[0]).double().T, approximate=approx)
        assert np.allclose(y0[:lens[0]], (h @ torch.from_numpy(W2[0]).double().T).numpy(), rtol=1e-12, atol=1e-13)


def test_mimic_mode_rounds_to_bf16(oracle):
    """mimic=1 output values are bf16-representable and close to the unrounded ones."""
    rng = np.random.default_rng(8)
    x = inputs.quantize(rng.standard_normal((9, 16)), "bf16")
    W1 = inputs.quantize(0.2 * rng.standard_normal((1, 32, 16)), "bf16")
    W2 = inputs.quantize(0.2 * rng.standard_normal((1, 16, 32)), "bf16")
    off = np.array([0, 9], np.int32)
    y = oracle.expert_ffn(x, off, W1, W2)
    ym = oracle.expert_ffn(x, off, W1, W2, mimic=1)
    ym32 = ym.astype(np.float32)
    assert np.array_equal(inputs.quantize(ym32, "bf16"), ym32)
    assert np.abs(ym - y).max() <= 2.0 ** -7 * np.abs(y).max()
    # and bf16 rounding itself agrees with torch's conversion (ties to even)
    a = rng.standard_normal(10000).astype(np.float32)
    assert np.array_equal(inputs.quantize(a, "bf16"),
                          torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_round_to_bf16_tie_rule_and_direction(oracle):
    """The C helper behind mimic mode, bit for bit against torch's fp32 -> bf16 conversion
    (round to nearest, ties to even) on the cases a wrong rule gets wrong: exact ties with an
    even and with an odd kept mantissa (truncation, round-half-up and round-half-away all
    fail one of them), one fp32 ulp above and below a tie, negatives, the carry into the
    exponent, subnormals, signed zeros, and values already representable."""
    def f32(bits):
        return np.array(bits, dtype=np.uint32).view(np.float32)
    bits = []
    for hi in (0x3F80, 0x3F81, 0x4049, 0x40FF, 0x7F7E, 0x0001, 0x0000, 0x007F, 0x0080, 0x00FF):
        for lo in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000):
            for sign in (0, 0x80000000):
                bits.append(sign | (hi << 16) | lo)
    bits.append(0x7F7F7FFF)                         # largest value that still rounds to a finite bf16
    bits.append(0x3FFF8000)                         # tie with an all-ones kept mantissa: carries into the exponent
    rng = np.random.default_rng(81)
    bits.extend(int(b) for b in rng.integers(0, 0x7F000000, 4000, dtype=np.int64))
    bits.extend(int(b) | 0x80000000 for b in rng.integers(0, 0x7F000000, 4000, dtype=np.int64))
    a = f32(bits)
    want = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    got = np.array([oracle.round_to_bf16(float(v)) for v in a], dtype=np.float64)
    assert np.isfinite(want).all()
    assert np.array_equal(got.astype(np.float32).view(np.uint32), want.view(np.uint32))
    assert np.array_equal(got, want.astype(np.float64))          # and exactly those values as doubles
    # hand-checked ties: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7 -> the even one (1);
    # 1 + 3 * 2^-8 lies halfway between 1 + 2^-7 and 1 + 2^-6 -> the even one (1 + 2^-6)
    assert oracle.round_to_bf16(1.0 + 2.0 ** -8) == 1.0
    assert oracle.round_to_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert oracle.round_to_bf16(-(1.0 + 2.0 ** -8)) == -1.0
    assert oracle.round_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -23) == 1.0 + 2.0 ** -7
    assert math.isinf(oracle.round_to_bf16(float("inf"))) and math.isnan(oracle.round_to_bf16(float("nan")))


# ------------------------------------------------------------------ layer (Eq. 6, 7, 14-17)

def _layer_bruteforce(L, E, k, C, shared, normalize=0, cg_mode=0, residual=False):
    """Eq. (7) token by token in numpy fp64, written independently of the C code:
    gating by fp64 matmul (inputs are chosen so that no arg max is fragile)."""
    erf = np.vectorize(math.erf)
    g = lambda v: 0.5 * v * (1.0 + erf(v / math.sqrt(2.0)))
    xp, xc = L["x_prev"].astype(np.float64), L["x_cur"].astype(np.float64)
    xg = xp if shared else xc
    T, d = xc.shape
    logits = xg @ L["Wg"].astype(np.float64)
    if L.get("bias") is not None:
        logits = logits + L["bias"].astype(np.float64)
    p = np.exp(logits - logits.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    order = np.argsort(-logits, axis=1, kind="stable")[:, :k]
    seen = np.zeros(E, int)
    kept = np.zeros((T, k), bool)
    for j in range(k):
        for t in range(T):
            e = order[t, j]
            kept[t, j] = seen[e] < C
            seen[e] += 1
    y = np.zeros((T, d))
    for t in range(T):
        sel = order[t]
        if normalize:
            ww = p[t, sel] / p[t, sel].sum()
        else:
            ww = p[t, sel]
        routed = np.zeros(d)
        for j in range(k):
            if not kept[t, j]:
                continue
            e = sel[j]
            h = L["W1"][e].astype(np.float64) @ xg[t]
            if L.get("b1") is not None:
                h = h + L["b1"][e]
            o = L["W2"][e].astype(np.float64) @ g(h)
            if L.get("b2") is not None:
                o = o + L["b2"][e]
            routed += ww[j] * o
        c0 = c1 = 1.0
        if cg_mode == 1:
            c0 = 1.0 / (1.0 + math.exp(-float(L["Wcg"][0].astype(np.float64) @ xc[t])))
        elif cg_mode == 2:
            a = L["Wcg"].astype(np.float64) @ xc[t]
            ea = np.exp(a - a.max())
            c0, c1 = ea / ea.sum()
        y[t] = c1 * routed
        if shared:
            h = L["W1s"].astype(np.float64) @ xc[t]
            if L.get("b1s") is not None:
                h = h + L["b1s"]
            s = L["W2s"].astype(np.float64) @ g(h)
            if L.get("b2s") is not None:
                s = s + L["b2s"]
            y[t] += c0 * s
        if residual:
            y[t] += xc[t]
    return y, order, kept


def _tiny(seed, T=48, d=12, F=20, E=4, biases=True, cg_rows=0, w_scale=0.3):
    return inputs.make_layer(T=T, d=d, F=F, E=E, dtype="f32", seed=seed, biases=biases,
                             cg_rows=cg_rows, w_scale=w_scale)


@pytest.mark.parametrize("k,shared,C,normalize,cg,res", [
    (1, 1, 1000, 0, 0, False), (1, 1, 9, 0, 0, True), (2, 0, 1000, 1, 0, False),
    (2, 0, 14, 1, 0, False), (2, 0, 14, 0, 0, False), (1, 1, 9, 0, 1, False),
    (1, 1, 1000, 0, 2, True), (1, 0, 9, 0, 0, False), (1, 1, 0, 0, 0, False),
    (2, 1, 14, 1, 0, False), (2, 1, 1000, 0, 1, True), (3, 0, 1000, 1, 0, False),
    (3, 0, 20, 1, 0, True), (3, 0, 20, 0, 0, False), (3, 1, 20, 1, 2, False),
    (4, 0, 30, 1, 0, False)])
def test_layer_bruteforce(oracle, k, shared, C, normalize, cg, res):
    L = _tiny(11 + k + C % 7, cg_rows=cg)
    E = L["Wg"].shape[1]
    ref, order, kept = _layer_bruteforce(L, E, k, C, shared, normalize, cg, res)
    y, r = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=k, capacity_=C, shared=shared,
                                normalize=normalize, cg_mode=cg, add_residual=int(res))
    assert np.array_equal(r["idx"], order)
    assert np.array_equal(r["dst_row"] >= 0, kept)
    assert np.allclose(y, ref, rtol=1e-6, atol=1e-6)   # the oracle's gate weights are fp32 outputs


def test_worked_example_by_hand(oracle):
    """A 3-token layer small enough to evaluate by hand from Eq. (7) and the normal-CDF
    table: gate logits (ln 3, 0) give p = 3/4; capacity 1 drops the third token."""
    phi = _phi_table()
    ln3 = math.log(3.0)
    L = dict(
        x_prev=np.array([[1, 0], [0, 1], [1, 0]], np.float32),
        x_cur=np.array([[0.5, 0.5], [1, 1], [1.5, 0]], np.float32),
        Wg=np.array([[ln3, 0], [0, ln3]], np.float32),
        W1=np.array([[[1, 0], [2, 0]], [[0, 3], [0, 0.5]]], np.float32),
        W2=np.array([[[1, 1], [1, -1]], [[2, 0], [0, 2]]], np.float32),
        W1s=np.array([[1, 1], [0, 0]], np.float32),
        W2s=np.array([[1, 0], [0, 1]], np.float32))
    y, r = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=1, capacity_=1)
    assert r["idx"][:, 0].tolist() == [0, 1, 0]
    assert r["dst_row"][:, 0].tolist() == [0, 1, -1]
    assert np.allclose(r["w"][:, 0], 0.75, atol=1e-7)
    g1, g2, g3, g05, g15 = phi[1.0], 2 * phi[2.0], 3 * phi[3.0], 0.5 * phi[0.5], 1.5 * phi[1.5]
    expect = np.array([[g1 + 0.75 * (g1 + g2), 0.75 * (g1 - g2)],
                       [g2 + 0.75 * 2 * g3, 0.75 * 2 * g05],
                       [g15, 0.0]])
    w = r["w"][:, 0].astype(np.float64)
    assert np.allclose(y, expect, rtol=0, atol=1e-6)
    # with the oracle's own (fp32-rounded ln 3) weights the match is to fp64 rounding
    expect_w = np.array([[g1 + w[0] * (g1 + g2), w[0] * (g1 - g2)],
                         [g2 + w[1] * 2 * g3, w[1] * 2 * g05], [g15, 0.0]])
    assert np.allclose(y, expect_w, rtol=0, atol=1e-14)


def test_layer_invariants(oracle):
    L = _tiny(21, T=60, biases=False)
    E = 4
    y, r = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=1, capacity_=11)
    dropped = r["dst_row"][:, 0] < 0
    assert dropped.any() and (~dropped).any()
    # the shared expert alone (dense MLP): zero routed weights
    Lz = dict(L, W2=np.zeros_like(L["W2"]))
    s, _ = oracle.layer_forward(L["x_prev"], L["x_cur"], Lz, k=1, capacity_=11)
    dense = torch.nn.functional.linear(
        torch.nn.functional.gelu(torch.from_numpy(L["x_cur"]).double() @ torch.from_numpy(L["W1s"]).double().T),
        torch.from_numpy(L["W2s"]).double()).numpy()
    assert np.allclose(s, dense, rtol=1e-12, atol=1e-13)
    # dropped tokens: expert term exactly zero -> y == s bit for bit
    assert np.array_equal(y[dropped], s[dropped])
    assert not np.allclose(y[~dropped], s[~dropped])
    # zero shared weights -> y[t] = w[t] * E_idx(x_prev[t])
    Ls = dict(L, W2s=np.zeros_like(L["W2s"]))
    yr, _ = oracle.layer_forward(L["x_prev"], L["x_cur"], Ls, k=1, capacity_=11)
    assert np.allclose(yr + s, y, rtol=1e-12, atol=1e-13)
    xp = torch.from_numpy(L["x_prev"]).double()
    for t in np.nonzero(~dropped)[0][:10]:
        e = r["idx"][t, 0]
        o = torch.nn.functional.gelu(xp[t] @ torch.from_numpy(L["W1"][e]).double().T) @ torch.from_numpy(L["W2"][e]).double().T
        assert np.allclose(yr[t], float(r["w"][t, 0]) * o.numpy(), rtol=1e-12, atol=1e-13)
    # counts / capacity invariants (combine weight == selected gate probability)
    logits = oracle.gate_logits(L["x_prev"], L["Wg"])
    _, _, probs = oracle.gate_topk(logits)
    assert np.array_equal(r["w"][:, 0], probs[np.arange(60), r["idx"][:, 0]])
    assert r["counts"].sum() == (~dropped).sum() and (r["counts"] <= 11).all()
    # x_prev == x_cur is the shared-expert MoE of Eq. (6)
    y6, r6 = oracle.layer_forward(None, L["x_cur"], L, k=1, capacity_=1000)
    ref6, _, _ = _layer_bruteforce(dict(L, x_prev=L["x_cur"]), E, 1, 1000, 1)
    assert np.allclose(y6, ref6, rtol=1e-6, atol=1e-6)


def test_layer_permutation_equivariance(oracle):
    """Without drops the layer acts on tokens independently: permuting the rows of x_prev
    and x_cur permutes the rows of y.  With a binding capacity the drop set depends on
    token order (the stated reading), so equivariance must fail there."""
    L = _tiny(23, T=64, biases=True)
    perm = np.random.default_rng(5).permutation(64)
    y, _ = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=1, capacity_=64)
    Lp = dict(L, x_prev=L["x_prev"][perm], x_cur=L["x_cur"][perm])
    yp, _ = oracle.layer_forward(Lp["x_prev"], Lp["x_cur"], Lp, k=1, capacity_=64)
    assert np.array_equal(yp, y[perm])
    yc, _ = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=1, capacity_=8)
    ycp, _ = oracle.layer_forward(Lp["x_prev"], Lp["x_cur"], Lp, k=1, capacity_=8)
    assert not np.array_equal(ycp, yc[perm])


def test_identical_experts_make_routing_irrelevant(oracle):
    """All experts equal, no drops, weights normalised over the selected experts (Eq. (2)
    literally): the routed term is E_0(x) whatever the gate picks; E = 1 is a dense MLP."""
    L = _tiny(29, T=40, E=4, biases=True)
    for key in ("W1", "W2", "b1", "b2"):
        L[key] = np.repeat(L[key][:1], 4, axis=0)
    for k in (1, 2):
        y, _ = oracle.layer_forward(None, L["x_cur"], L, k=k, shared=0, normalize=1)
        one = dict(L, W1=L["W1"][:1], W2=L["W2"][:1], b1=L["b1"][:1], b2=L["b2"][:1], Wg=L["Wg"][:, :1])
        y1, r1 = oracle.layer_forward(None, L["x_cur"], one, k=1, shared=0, normalize=0)
        assert (r1["w"] == 1.0).all()
        assert np.allclose(y, y1, rtol=1e-6, atol=1e-6)   # k=2 weights sum to 1 only within fp32


def test_two_experts_top2_is_full_mixture(oracle):
    """E = 2, k = 2, no capacity: Eq. (1) with the full softmax over both experts."""
    L = _tiny(31, T=30, E=2, biases=False)
    y, r = oracle.layer_forward(None, L["x_cur"], L, k=2, shared=0, normalize=1)
    x = torch.from_numpy(L["x_cur"]).double()
    p = torch.softmax(x @ torch.from_numpy(L["Wg"]).double(), dim=1)
    outs = [torch.nn.functional.gelu(x @ torch.from_numpy(L["W1"][e]).double().T) @ torch.from_numpy(L["W2"][e]).double().T
            for e in range(2)]
    ref = p[:, :1] * outs[0] + p[:, 1:] * outs[1]
    assert np.allclose(y, ref.numpy(), rtol=1e-6, atol=1e-7)   # gate weights are stored in fp32


def test_three_experts_top3_is_full_mixture(oracle):
    """E = 3, k = 3, no capacity: every expert runs on every token, weighted by the full
    softmax (Eq. (1) without sparsity), whatever order the selection lists them in."""
    L = _tiny(33, T=26, E=3, biases=False)
    y, r = oracle.layer_forward(None, L["x_cur"], L, k=3, shared=0, normalize=1)
    x = torch.from_numpy(L["x_cur"]).double()
    p = torch.softmax(x @ torch.from_numpy(L["Wg"]).double(), dim=1)
    ref = sum(p[:, e:e + 1] * (torch.nn.functional.gelu(x @ torch.from_numpy(L["W1"][e]).double().T)
                              @ torch.from_numpy(L["W2"][e]).double().T) for e in range(3))
    assert np.allclose(y, ref.numpy(), rtol=1e-6, atol=1e-7)


def test_coefficient_gates(oracle):
    """Eq. (14)-(17): W_cg = 0 gives coef 0.5 (CG-1: sigmoid(0); CG-2: softmax of equal
    scores), and random W_cg matches torch's sigmoid / softmax."""
    L = _tiny(37, T=20, cg_rows=2)
    z = np.zeros_like(L["Wcg"])
    y, _ = oracle.layer_forward(L["x_prev"], L["x_cur"], L, capacity_=1000)
    s, _ = oracle.layer_forward(L["x_prev"], L["x_cur"], dict(L, W2=np.zeros_like(L["W2"]), b2=np.zeros_like(L["b2"])), capacity_=1000)
    y1, _ = oracle.layer_forward(L["x_prev"], L["x_cur"], dict(L, Wcg=z), capacity_=1000, cg_mode=1)
    y2, _ = oracle.layer_forward(L["x_prev"], L["x_cur"], dict(L, Wcg=z), capacity_=1000, cg_mode=2)
    assert np.allclose(y1, 0.5 * s + (y - s), rtol=1e-12, atol=1e-13)
    assert np.allclose(y2, 0.5 * y, rtol=1e-12, atol=1e-13)
    xc = torch.from_numpy(L["x_cur"]).double()
    W = torch.from_numpy(L["Wcg"]).double()
    c1 = oracle.coef_gate(L["x_cur"], L["Wcg"][:1], 1)
    assert np.allclose(c1[:, 0], torch.sigmoid(xc @ W[0]).numpy(), atol=1e-14) and (c1[:, 1] == 1).all()
    c2 = oracle.coef_gate(L["x_cur"], L["Wcg"], 2)
    assert np.allclose(c2, torch.softmax(xc @ W.T, dim=1).numpy(), atol=1e-14)


def test_combine_is_linear_in_gate_weight(oracle):
    rng = np.random.default_rng(41)
    yp = rng.standard_normal((10, 6))
    dst = np.array([[3], [-1], [0], [9], [-1], [5]], np.int32)
    w = rng.random((6, 1)).astype(np.float32)
    base = rng.standard_normal((6, 6))
    res = rng.standard_normal((6, 6))
    y = oracle.combine(yp, dst, w, base, res)
    y2 = oracle.combine(yp, dst, 2 * w, base, res)
    for t in range(6):
        r = dst[t, 0]
        exp_t = base[t] + res[t] + (float(w[t, 0]) * yp[r] if r >= 0 else 0.0)
        assert np.allclose(y[t], exp_t, rtol=1e-14, atol=1e-15)
    assert np.allclose(y2 - y, y - base - res, rtol=1e-12, atol=1e-13)


def test_layer_rows_equals_full_layer(oracle):
    """Sampled rows (the form used for parity at full benchmark sizes) equal the rows of
    the full-layer call."""
    L = _tiny(43, T=50, biases=True)
    y, r = oracle.layer_forward(L["x_prev"], L["x_cur"], L, k=1, capacity_=10)
    rows = np.array([0, 7, 49, 23], np.int32)
    yr = oracle.layer_rows(L["x_prev"], L["x_cur"], L, r, rows, k=1, shared=1)
    assert np.array_equal(yr, y[rows])
    rt = oracle.route(L["x_prev"], L, 4, 1, 10)
    for key in ("idx", "w", "counts", "offsets", "dst_row", "src_token"):
        assert np.array_equal(rt[key], r[key])


def test_equal_compute_of_top2_and_scmoe():
    """Sec. 4.1: a top-2 layer and ScMoE (one shared + one routed expert) have the same
    computational volume when nothing is dropped: 4*d*F per (token, expert) pair."""
    T, d, F = 16384, 1024, 4096
    top2 = 4 * d * F * (2 * T)
    scmoe = 4 * d * F * T + 4 * d * F * T
    assert top2 == scmoe == 549755813888
