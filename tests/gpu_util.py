"""Helpers of the GPU parity tests: the error metrics of the parity bar and the routing comparison."""
import numpy as np

from paper_2404_05019_amd.devlayer import DEV, DevLayer, run_layer, to_dev, to_host  # noqa: F401 (re-exported)


def relerr(g, r):
    """max |g - r| / max |r|: the error metric of the parity bar."""
    g = np.asarray(g, np.float64)
    r = np.asarray(r, np.float64)
    den = np.abs(r).max()
    return float(np.abs(g - r).max() / (den if den > 0 else 1.0))


TOL = {"f32": 1e-4, "bf16": 2e-2}


def pass_rate(g, r, tol):
    """Share of elements with |g - r| <= tol * (|r| + rms(r)): the element-wise reading of the
    same bar.  Unlike relerr it is not dominated by the largest elements, so a systematic error
    in the small ones shows."""
    g = np.asarray(g, np.float64)
    r = np.asarray(r, np.float64)
    if r.size == 0:
        return 1.0
    rms = float(np.sqrt(np.mean(r * r)))
    return float(np.mean(np.abs(g - r) <= tol * (np.abs(r) + rms)))


def assert_close(g, r, dtype):
    """Both readings of the parity bar: max-abs error over max-abs reference within the
    tolerance, and every element within tol * (|r| + rms(r)).  Returns (relerr, pass rate)."""
    err, rate = relerr(g, r), pass_rate(g, r, TOL[dtype])
    assert err <= TOL[dtype], err
    assert rate == 1.0, rate
    return err, rate


def assert_routing_equal(g, r, w_tol=1e-6):
    """Integer routing state must match bit for bit; gate weights are floats."""
    for key in ("idx", "counts", "offsets", "dst_row", "src_token"):
        assert np.array_equal(g[key], r[key]), "routing array %s differs" % key
    assert np.abs(g["w"].astype(np.float64) - r["w"].astype(np.float64)).max() <= w_tol


def stratified_tokens(rr, T, E, seed, block=128):
    """Tokens chosen so that every tile of both GEMM chains is compared: one seeded row out of
    every `block` consecutive token rows (the shared expert's row tiles) and out of every
    `block` consecutive packed rows of every expert segment (the routed experts' row tiles,
    counted from the segment start as the kernels do), plus the first and the last packed row
    of every segment (the ragged last tile) and some dropped tokens.  A compared row spans all
    column tiles, so the tiles of the split-K tail are among them whichever they are; 128 is
    the smallest row tile any kernel variant uses."""
    rng = np.random.default_rng(seed)
    toks = [0, T - 1]
    for b0 in range(0, T, block):
        toks.append(int(rng.integers(b0, min(b0 + block, T))))
    offs, src = rr["offsets"], rr["src_token"]
    for e in range(E):
        lo, hi = int(offs[e]), int(offs[e + 1])
        if hi > lo:
            toks += [int(src[lo]), int(src[hi - 1])]
        for b0 in range(lo, hi, block):
            toks.append(int(src[int(rng.integers(b0, min(b0 + block, hi)))]))
    dropped = np.nonzero((rr["dst_row"] < 0).any(axis=1))[0]
    if len(dropped):
        toks += [int(t) for t in dropped[rng.integers(0, len(dropped), 16)]]
    return np.unique(np.asarray(toks, dtype=np.int32))
