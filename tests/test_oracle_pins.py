"""Pins for the CPU oracle (no GPU).

The oracle is what the HIP path is judged against, so it is pinned here to
things other than itself: a hand-worked example, brute force over codes and
over fine grids, closed forms, exact on-grid cases, metamorphic relations and
the invariants Section 3.1/3.4/3.5 of the paper fix.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_1902_06822_amd import synth

SIGNED = (-8, 7)
UNSIGNED = (0, 15)


# ------------------------------------------------------------------ helpers
def np_def_sse(x, alpha, qmin, qmax):
    """Eq. 8 in numpy fp64 (np.rint = ties to even)."""
    x = np.asarray(x, np.float64)
    q = np.clip(np.rint(x / alpha), qmin, qmax)
    return float(np.sum((x - alpha * q) ** 2))


def read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = v
    return out


# ------------------------------------------------------------------ hand example
def test_hand_worked_example(golden_dir):
    g = read_golden(os.path.join(golden_dir, "hand_example.txt"))
    alpha = float(g["alpha"][0])
    x = np.array([float(v) for v in g["x"]], np.float32)
    for tag, (lo, hi), signed in (("signed", SIGNED, True), ("unsigned", UNSIGNED, False)):
        codes = np.array([int(v) for v in g[f"{tag}_codes"]], np.int32)
        sse = float(g[f"{tag}_sse"][0])
        packed = np.array([int(v, 16) for v in g[f"{tag}_packed_hex"]], np.uint8)
        assert oracle.def_sse(x, alpha, lo, hi) == sse
        assert oracle.can_sse(x, alpha, lo, hi) == sse           # all values exact in fp32
        got = oracle.can_codes(x, [alpha], lo, hi).ravel()
        np.testing.assert_array_equal(got, codes)
        np.testing.assert_array_equal(oracle.can_pack_int4(codes), packed)
        np.testing.assert_array_equal(oracle.can_quantize_pack_int4(x, [alpha], lo, hi), packed)
        np.testing.assert_array_equal(oracle.can_unpack_int4(packed, codes.size, signed), codes)


# ------------------------------------------------------------------ fixed-alpha optimality of [x/alpha]
@pytest.mark.parametrize("rng_seed", [0, 1, 2])
@pytest.mark.parametrize("qr", [SIGNED, UNSIGNED])
def test_rounding_is_optimal_code_joint_bruteforce(rng_seed, qr):
    """Section 3.4: for fixed alpha no code assignment beats [T/alpha] (all 16^3 assignments)."""
    rng = np.random.default_rng(rng_seed)
    x = (rng.normal(0, 0.5, 3)).astype(np.float32)
    if qr == UNSIGNED:
        x = np.abs(x)
    for alpha in (0.03, 0.11, 0.4):
        best = min(oracle.def_sse_codes(x, list(c), alpha)
                   for c in itertools.product(range(qr[0], qr[1] + 1), repeat=3))
        got = oracle.def_sse(x, alpha, *qr)
        assert got <= best * (1 + 1e-12) + 1e-300
        assert got >= best * (1 - 1e-12)


@pytest.mark.parametrize("qr", [SIGNED, UNSIGNED])
def test_def_sse_separable_bruteforce(qr):
    """Per-element brute force over the 16 codes on a longer vector."""
    rng = np.random.default_rng(7)
    x = rng.standard_t(4, 300).astype(np.float32) * 0.1
    codes = np.arange(qr[0], qr[1] + 1, dtype=np.float64)
    for alpha in (0.004, 0.02, 0.07, 0.5):
        per = ((x.astype(np.float64)[:, None] - alpha * codes[None, :]) ** 2).min(axis=1)
        assert oracle.def_sse(x, alpha, *qr) == pytest.approx(per.sum(), rel=1e-12)


# ------------------------------------------------------------------ canonical vs definition
@pytest.mark.parametrize("n", [1, 9, 63, 64, 65, 147, 576, 4608, 25088, 70001])
@pytest.mark.parametrize("qr", [SIGNED, UNSIGNED])
def test_canonical_close_to_definition(n, qr):
    rng = np.random.default_rng(n)
    x = rng.laplace(0, 0.02, n).astype(np.float32)
    if qr == UNSIGNED:
        x = np.maximum(x, 0)
    a = float(np.abs(x).max())
    if a == 0:
        return
    for frac in (0.1, 0.37, 0.8, 1.0):
        alpha = np.float32(a / qr[1] * frac)
        c = oracle.can_sse(x, alpha, *qr)
        d = oracle.def_sse(x, float(alpha), *qr)
        assert c == pytest.approx(d, rel=1e-5, abs=1e-30)
        assert d == pytest.approx(np_def_sse(x, float(alpha), *qr), rel=1e-12)


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 127, 128, 129, 191, 640, 4096, 4097, 12345])
def test_canonical_sum_exact_when_terms_are_exact(n):
    """x = alpha0*(k + 1/4): every residual is alpha0/4 exactly, so f = n*alpha0^2/16 exactly.
    A dropped, repeated or misplaced chunk (tail handling, pairwise tree) changes the count."""
    alpha0 = 2.0 ** -5
    rng = np.random.default_rng(n)
    k = rng.integers(-7, 7, n)
    x = ((k + 0.25) * alpha0).astype(np.float32)
    assert oracle.can_sse(x, alpha0, *SIGNED) == n * alpha0 ** 2 / 16
    assert oracle.def_sse(x, alpha0, *SIGNED) == n * alpha0 ** 2 / 16


def test_uniform_quantiser_noise_closed_form():
    """Textbook: without clipping the error of a uniform quantiser is ~ n*alpha^2/12."""
    rng = np.random.default_rng(3)
    n = 200000
    x = rng.uniform(-1, 1, n).astype(np.float32)
    alpha = 1.0 / 7.0            # max-abs scale: no clipping beyond +-7.5*alpha
    for f in (oracle.def_sse, oracle.can_sse):
        assert f(x, alpha, *SIGNED) == pytest.approx(n * alpha ** 2 / 12, rel=0.02)


# ------------------------------------------------------------------ grid, argmin
def test_grid_definition():
    """Linear grid over (0, absmax/qmax], last point = max-abs scale of Section 3.1."""
    for a, qmax, G in ((0.7, 7, 128), (3.3, 15, 50), (1e-3, 7, 500), (2.0, 7, 1)):
        g = oracle.can_grid(a, qmax, G)
        smax = np.float32(a) / np.float32(qmax)
        assert g[-1] == smax
        assert np.all(np.diff(g) > 0) and g[0] > 0
        np.testing.assert_allclose(g, smax * (np.arange(1, G + 1) / G), rtol=3e-7)


@pytest.mark.parametrize("seed", range(6))
def test_grid_argmin_bruteforce_and_fine_grid(seed):
    rng = np.random.default_rng(seed)
    n, G = int(rng.integers(2, 17)), int(rng.integers(2, 33))
    x = rng.normal(0, 1, n).astype(np.float32)
    r = oracle.can_search(x, *SIGNED, G, 0, want_grid=True)
    e = r["grid_sse"]
    j = r["idx"]
    assert np.all(e[j] <= e)
    assert j == int(np.flatnonzero(e == e.min())[0])           # lowest index among ties
    grid = oracle.can_grid(np.abs(x).max(), 7, G)
    assert r["scale"] == grid[j] and r["sse"] == e[j]
    # the grid values themselves follow the definition
    for jj in range(G):
        assert e[jj] == pytest.approx(np_def_sse(x, float(grid[jj]), *SIGNED), rel=1e-5, abs=1e-30)
    # a 1e5-point fine grid in fp64 can only do better than (or as well as) the coarse argmin
    fine = np.linspace(float(grid[-1]) / 1e5, float(grid[-1]), 100000)
    xd = x.astype(np.float64)
    ef = np.sum((xd[None, :] - fine[:, None] * np.clip(np.rint(xd[None, :] / fine[:, None]), -8, 7)) ** 2,
                axis=1)
    assert ef.min() <= e[j] * (1 + 1e-5)
    # and every coarse grid value is matched by the nearest fine point up to the local slope
    assert ef.min() >= 0.0


def test_argmin_tie_break_lowest_index():
    """x = {-7, 0} * 2^-2 in the signed range: the max-abs scale 2^-2 (code -7) and 7/8 of it
    (code -8) both give zero error, and both are grid points when 8 divides G.  Every tied
    scale is optimal; the contract returns the lowest index."""
    x = np.array([-7, 0, -7, 0, 0], np.float32) * 0.25
    for G in (8, 16, 64):
        r = oracle.can_search(x, *SIGNED, G, 0, want_grid=True)
        e = r["grid_sse"]
        zeros = np.flatnonzero(e == 0.0)
        np.testing.assert_array_equal(zeros, [7 * G // 8 - 1, G - 1])
        assert r["idx"] == 7 * G // 8 - 1 and r["sse"] == 0.0
        assert r["scale"] == np.float32(0.25 * 0.875)
        np.testing.assert_array_equal(oracle.can_codes(x, [r["scale"]], *SIGNED).ravel(), [-8, 0, -8, 0, 0])


# ------------------------------------------------------------------ exact cases
@pytest.mark.parametrize("qr,qlo", [(SIGNED, -7), (UNSIGNED, 0)])
@pytest.mark.parametrize("G", [128, 256, 500, 50])
def test_on_grid_inputs_give_zero_error(qr, qlo, G):
    alpha0 = 2.0 ** -6
    w, q = synth.on_grid_tensor(5, 200, 11, alpha0, qlo, qr[1])
    scale, idx, sse = oracle.can_search_kernelwise(w, *qr, G, 20)
    assert np.all(idx == G - 1)
    assert np.all(scale == np.float32(alpha0))
    assert np.all(sse == 0.0)
    np.testing.assert_array_equal(oracle.can_codes(w, scale, *qr), q)


def test_all_zero_and_tiny_tensors():
    z = np.zeros(100, np.float32)
    r = oracle.can_search(z, *SIGNED, 64, 20, want_grid=True)
    assert (r["scale"], r["idx"], r["sse"], r["rc"]) == (1.0, 0, 0.0, 0)
    assert np.all(oracle.can_codes(z, [r["scale"]], *SIGNED) == 0)
    t = np.full(10, 1e-20, np.float32)
    r = oracle.can_search(t, *SIGNED, 64, 20)
    assert r["scale"] == 1.0 and r["idx"] == 0
    assert r["sse"] == pytest.approx(10 * 1e-40, rel=1e-3)


def test_rejected_inputs():
    for bad in (np.inf, np.nan, 1e30):
        x = np.array([0.1, bad, -0.2], np.float32)
        r = oracle.can_search(x, *SIGNED, 16, 5)
        assert r["rc"] == -1 and r["idx"] == -1 and np.isnan(r["scale"]) and np.isnan(r["sse"])


def test_constant_unsigned_tensor():
    x = np.full(77, 0.9375, np.float32)          # 15 * 2^-4
    r = oracle.can_search(x, *UNSIGNED, 128, 20)
    assert r["idx"] == 127 and r["scale"] == np.float32(0.0625) and r["sse"] == 0.0
    assert np.all(oracle.can_codes(x, [r["scale"]], *UNSIGNED) == 15)


def test_single_element():
    for v in (0.37, -0.37):
        x = np.array([v], np.float32)
        r = oracle.can_search(x, *SIGNED, 32, 20)
        assert r["sse"] <= oracle.can_sse(x, np.float32(abs(v)) / np.float32(7), *SIGNED)
        assert r["sse"] < 1e-12


def test_negative_inputs_saturate_to_zero_in_unsigned_range():
    x = np.array([-1.0, -0.1, 0.6, 1.0], np.float32)
    codes = oracle.can_codes(x, [1.0 / 15], *UNSIGNED).ravel()
    np.testing.assert_array_equal(codes, [0, 0, 9, 15])


# ------------------------------------------------------------------ invariants
@pytest.mark.parametrize("kind", ["laplace", "normal", "outliers", "student"])
def test_invariant_chain(kind):
    """E_final <= E_grid(j*) <= E(max-abs scale) (Section 3.1 scale is the last grid point)."""
    w = synth.small_weights(16, 147, 5, kind)
    for k in range(w.shape[0]):
        g = oracle.can_search(w[k], *SIGNED, 64, 0, want_grid=True)
        r = oracle.can_search(w[k], *SIGNED, 64, 20)
        assert r["idx"] == g["idx"]
        assert r["sse"] <= g["sse"] <= g["grid_sse"][-1]
        assert r["sse"] == oracle.can_sse(w[k], r["scale"], *SIGNED)
        assert g["grid_sse"][-1] == oracle.can_sse(w[k], oracle.can_absmax(w[k]) / np.float32(7), *SIGNED)


@pytest.mark.parametrize("m", [-9, -3, 4, 11])
def test_power_of_two_scaling_is_exact(m):
    w = synth.small_weights(6, 321, 9, "laplace")
    s0, i0, e0 = oracle.can_search_kernelwise(w, *SIGNED, 100, 20)
    w2 = (w * np.float32(2.0 ** m)).astype(np.float32)
    s1, i1, e1 = oracle.can_search_kernelwise(w2, *SIGNED, 100, 20)
    np.testing.assert_array_equal(i0, i1)
    np.testing.assert_array_equal(s0 * np.float32(2.0 ** m), s1)
    np.testing.assert_array_equal(e0 * 4.0 ** m, e1)
    np.testing.assert_array_equal(oracle.can_codes(w, s0, *SIGNED), oracle.can_codes(w2, s1, *SIGNED))


def test_kernelwise_rows_are_independent_problems():
    """Section 3.3: each kernel gets its own scale; row k of [K][n] is problem k."""
    w = synth.small_weights(7, 130, 21, "normal")
    s, i, e = oracle.can_search_kernelwise(w, *SIGNED, 48, 20)
    for k in range(7):
        r = oracle.can_search(w[k].copy(), *SIGNED, 48, 20)
        assert (r["scale"], r["idx"], r["sse"]) == (s[k], i[k], e[k])
    assert len(set(s.tolist())) == 7


# ------------------------------------------------------------------ refinement
@pytest.mark.parametrize("seed", range(4))
def test_refinement_structure(seed):
    rng = np.random.default_rng(seed)
    x = rng.laplace(0, 0.05, 500).astype(np.float32)
    G, iters = 40, 20
    r = oracle.can_search(x, *SIGNED, G, iters, want_grid=True, want_probes=True)
    grid = oracle.can_grid(np.abs(x).max(), 7, G)
    j = r["idx"]
    lo = 0.0 if j == 0 else grid[j - 1]
    hi = grid[j] if j == G - 1 else grid[j + 1]
    p = r["probes"]
    assert p.size == 2 + iters
    assert np.all(p > lo) and np.all(p < hi)
    # probes: every value is a real evaluation; the best one (or the grid point) is returned
    ev = np.array([oracle.can_sse(x, a, *SIGNED) for a in p])
    best = min(ev.min(), r["grid_sse"][j])
    assert r["sse"] == best
    assert r["scale"] in set(p.tolist()) | {grid[j]}
    # interval shrinks by the golden ratio each iteration: late probes cluster
    phi = 0.6180339887
    assert abs(float(p[-1]) - float(p[-2])) <= (hi - lo) * phi ** (iters - 2)
    # first two probes are the golden points of the bracket
    w = np.float32(hi) - np.float32(lo)
    assert p[0] == pytest.approx(hi - phi * w, rel=1e-6)
    assert p[1] == pytest.approx(lo + phi * w, rel=1e-6)


def test_refinement_converges_to_the_vertex_where_f_is_a_parabola():
    """With a fine grid and few elements the codes do not change across the bracket, so
    f(alpha) = sum (x - alpha*q)^2 is an exact parabola there with vertex sum(xq)/sum(q^2):
    a golden-section search must close in on it (this pins which half is kept)."""
    G, iters, used = 2048, 30, 0
    for seed in range(40):
        rng = np.random.default_rng(1000 + seed)
        x = rng.normal(0, 1, 6).astype(np.float32)
        r = oracle.can_search(x, *SIGNED, G, iters, want_probes=True)
        grid = oracle.can_grid(np.abs(x).max(), 7, G)
        j = r["idx"]
        if j == 0 or j == G - 1:
            continue
        lo, hi = grid[j - 1], grid[j + 1]
        q_lo = oracle.can_codes(x, [lo], *SIGNED).ravel()
        q_hi = oracle.can_codes(x, [hi], *SIGNED).ravel()
        if not np.array_equal(q_lo, q_hi):
            continue                                    # a code flips inside the bracket: not a parabola
        q = q_lo.astype(np.float64)
        vertex = float(np.dot(x.astype(np.float64), q) / np.dot(q, q))
        target = min(max(vertex, float(lo)), float(hi))
        w0 = float(hi) - float(lo)
        # near the vertex f is flat to within fp32 rounding of the sums, so the search cannot resolve
        # alpha much better than sqrt(eps); a search that kept the wrong half ends >= 0.38*w0 away
        assert abs(float(r["probes"][-1]) - target) <= 0.05 * w0
        assert abs(float(r["scale"]) - target) <= 0.05 * w0
        used += 1
    assert used >= 10


def test_refine_iters_zero_returns_grid_point():
    x = synth.small_weights(1, 300, 2, "student")[0]
    r = oracle.can_search(x, *SIGNED, 77, 0)
    assert r["scale"] == oracle.can_grid(np.abs(x).max(), 7, 77)[r["idx"]]


# ------------------------------------------------------------------ codes and packing
@pytest.mark.parametrize("K,n", [(1, 1), (3, 9), (5, 27), (2, 147), (1, 2), (4, 64)])
def test_pack_roundtrip_and_error_from_packed(K, n):
    w = synth.small_weights(K, n, 100 + K * n, "outliers")
    s, i, e = oracle.can_search_kernelwise(w, *SIGNED, 64, 20)
    packed = oracle.can_quantize_pack_int4(w, s, *SIGNED)
    assert packed.size == (K * n + 1) // 2                     # CR 0.125 (Table 3 caption)
    q = oracle.can_unpack_int4(packed, K * n, True).reshape(K, n)
    np.testing.assert_array_equal(q, oracle.can_codes(w, s, *SIGNED))
    assert q.min() >= -8 and q.max() <= 7
    for k in range(K):
        d = float(np.sum((w[k].astype(np.float64) - float(s[k]) * q[k]) ** 2))
        assert d == pytest.approx(e[k], rel=1e-5, abs=1e-30)
    if (K * n) % 2:
        assert packed[-1] >> 4 == 0


def test_codes_match_definition_away_from_ties():
    rng = np.random.default_rng(5)
    x = rng.normal(0, 1, 5000).astype(np.float32)
    alpha = np.float32(0.2137)
    t = x.astype(np.float64) / float(alpha)
    away = np.abs(t - np.floor(t) - 0.5) > 1e-5
    ref = np.clip(np.rint(t), -8, 7).astype(np.int32)
    got = oracle.can_codes(x, [alpha], *SIGNED).ravel()
    np.testing.assert_array_equal(got[away], ref[away])


# ------------------------------------------------------------------ residual (second tensor)
@pytest.mark.parametrize("kind", ["laplace", "student"])
def test_residual_reduces_error_and_reconstructs(kind):
    w = synth.small_weights(8, 200, 77, kind)
    G = 64
    s1, i1, e1 = oracle.can_search_kernelwise(w, *SIGNED, G, 20)
    s2, i2, e2, p2 = oracle.can_residual_quantize(w, s1, *SIGNED, G, 20)
    assert np.all(e2 <= e1)                                     # Algorithm 1 never increases the objective
    q1 = oracle.can_codes(w, s1, *SIGNED)
    q2 = oracle.can_unpack_int4(p2, w.size, True).reshape(w.shape)
    R = oracle.can_residual(w, s1, *SIGNED)
    np.testing.assert_allclose(R, w.astype(np.float64) - s1[:, None].astype(np.float64) * q1,
                               rtol=0, atol=1e-7)
    for k in range(w.shape[0]):
        d = oracle.def_sse_dual(w[k], q1[k], q2[k], float(s1[k]), float(s2[k]))
        assert d == pytest.approx(e2[k], rel=2e-5, abs=1e-30)
    # the residual search is the plain search applied to R
    s2b, i2b, e2b = oracle.can_search_kernelwise(R, *SIGNED, G, 20)
    np.testing.assert_array_equal(s2, s2b)
    np.testing.assert_array_equal(i2, i2b)
    np.testing.assert_array_equal(e2, e2b)


def test_residual_on_grid_gives_zero():
    """T = a1*Q1 + a2*Q2 with a1 = 2^-2, a2 = 2^-6 (so |a2*Q2| < a1/2): second error is 0."""
    rng = np.random.default_rng(1)
    K, n = 3, 90
    q1 = rng.integers(-7, 8, (K, n))
    q2 = rng.integers(-7, 8, (K, n))
    q2[:, 0] = 7
    w = (q1 * 2.0 ** -2 + q2 * 2.0 ** -6).astype(np.float32)
    s1 = np.full(K, 2.0 ** -2, np.float32)
    s2, i2, e2, p2 = oracle.can_residual_quantize(w, s1, *SIGNED, 32, 20)
    assert np.all(e2 == 0.0) and np.all(s2 == np.float32(2.0 ** -6)) and np.all(i2 == 31)
    np.testing.assert_array_equal(oracle.can_unpack_int4(p2, K * n, True).reshape(K, n), q2)


# ------------------------------------------------------------------ Algorithm 1 iterated (two tensors)
def _fma32(t, a, q):
    """fp32 fused multiply-add t - a*q via exact fp64 arithmetic and one rounding."""
    return (t.astype(np.float64) - np.float64(a) * q.astype(np.float64)).astype(np.float32)


def test_alternating_first_sweep_is_the_residual_fit():
    w = synth.small_weights(6, 147, 12, "student")
    G = 64
    o = oracle.can_dual_alternating(w, *SIGNED, G, 20, 1e-3, 1)
    s1, _, _ = oracle.can_search_kernelwise(w, *SIGNED, G, 20)
    s2, _, e2, p2 = oracle.can_residual_quantize(w, s1, *SIGNED, G, 20)
    np.testing.assert_array_equal(o["scale1"], s1)
    np.testing.assert_array_equal(o["scale2"], s2)
    np.testing.assert_array_equal(o["sse"], e2)
    np.testing.assert_array_equal(o["packed2"], p2)
    np.testing.assert_array_equal(o["packed1"], oracle.can_quantize_pack_int4(w, s1, *SIGNED))
    assert np.all(o["sweeps"] == 1)


def test_alternating_lowers_the_error_and_reports_it_truthfully():
    K, n, G = 10, 576, 128
    w = synth.small_weights(K, n, 3, "laplace")
    prev = None
    for max_sweeps in (1, 2, 3, 6):
        o = oracle.can_dual_alternating(w, *SIGNED, G, 20, 0.0, max_sweeps)
        assert np.all(o["sweeps"] >= 1) and np.all(o["sweeps"] <= max_sweeps)
        q1 = oracle.can_unpack_int4(o["packed1"], K * n, True).reshape(K, n)
        q2 = oracle.can_unpack_int4(o["packed2"], K * n, True).reshape(K, n)
        for k in range(K):
            d = oracle.def_sse_dual(w[k], q1[k], q2[k], float(o["scale1"][k]), float(o["scale2"][k]))
            assert d == pytest.approx(o["sse"][k], rel=3e-5)
            # the kept state is a fixed point of the second half-step: (a2,Q2) = phi(T - a1*Q1)
            r = _fma32(w[k], o["scale1"][k], q1[k])
            f = oracle.can_search(r, *SIGNED, G, 20)
            assert f["scale"] == o["scale2"][k] and f["sse"] == o["sse"][k]
            np.testing.assert_array_equal(oracle.can_codes(r, [f["scale"]], *SIGNED).ravel(), q2[k])
        if prev is not None:
            assert np.all(o["sse"] <= prev)                   # more sweeps never hurt (worse sweeps are discarded)
        prev = o["sse"]
    one = oracle.can_dual_alternating(w, *SIGNED, G, 20, 0.0, 1)["sse"]
    # on these kernels alternating does help: a sweep that fitted the wrong residual would be discarded
    assert np.all(prev < one) and np.mean(prev / one) < 0.95


def test_alternating_second_sweep_refits_the_first_tensor_against_the_second():
    """Algorithm 1, j = 1 of the second sweep: (a1,Q1) = phi(T - a2*Q2) with the second tensor of the
    first sweep (not the other way round)."""
    K, n, G = 8, 321, 64
    w = synth.small_weights(K, n, 33, "laplace")
    o1 = oracle.can_dual_alternating(w, *SIGNED, G, 20, 0.0, 1)
    o2 = oracle.can_dual_alternating(w, *SIGNED, G, 20, 0.0, 2)
    q2_first = oracle.can_unpack_int4(o1["packed2"], K * n, True).reshape(K, n)
    q1_second = oracle.can_unpack_int4(o2["packed1"], K * n, True).reshape(K, n)
    checked = 0
    for k in range(K):
        if o2["sweeps"][k] != 2:
            continue
        r = _fma32(w[k], o1["scale2"][k], q2_first[k])
        f = oracle.can_search(r, *SIGNED, G, 20)
        assert f["scale"] == o2["scale1"][k]
        np.testing.assert_array_equal(oracle.can_codes(r, [f["scale"]], *SIGNED).ravel(), q1_second[k])
        checked += 1
    assert checked >= K // 2


def test_alternating_never_keeps_a_worse_sweep():
    """phi is a grid heuristic: with a coarse grid a sweep can raise the error; such a sweep is discarded,
    so the reported error is non-increasing in the number of sweeps allowed."""
    for seed, (K, n, G, kind) in enumerate(((6, 27, 8, "normal"), (6, 9, 8, "outliers"), (4, 64, 16, "laplace"),
                                            (4, 147, 6, "student"))):
        w = synth.small_weights(K, n, seed * 7 + n, kind)
        prev = None
        for m in range(1, 8):
            e = oracle.can_dual_alternating(w, *SIGNED, G, 3, 0.0, m)["sse"]
            if prev is not None:
                assert np.all(e <= prev)
            prev = e


def test_alternating_stopping_rule():
    w = synth.small_weights(8, 300, 21, "laplace")
    big = oracle.can_dual_alternating(w, *SIGNED, 64, 20, 1.0, 10)       # any gain counts as converged
    assert np.all(big["sweeps"] <= 2)
    tight = oracle.can_dual_alternating(w, *SIGNED, 64, 20, 0.0, 10)
    assert np.all(tight["sweeps"] >= big["sweeps"]) and np.all(tight["sse"] <= big["sse"])
    mid = oracle.can_dual_alternating(w, *SIGNED, 64, 20, 0.02, 10)
    assert np.all(mid["sweeps"] <= tight["sweeps"])


def test_alternating_on_a_tensor_that_is_two_grids():
    rng = np.random.default_rng(4)
    K, n = 3, 64
    q1 = rng.integers(-7, 8, (K, n))
    q2 = rng.integers(-7, 8, (K, n))
    q1[:, 0] = 7
    q2[:, 1] = 7
    w = (q1 * 2.0 ** -2 + q2 * 2.0 ** -6).astype(np.float32)
    w[:, 0] = 7 * 2.0 ** -2 + 0 * 2.0 ** -6          # the max-abs element is exactly 7*a1
    q2[:, 0] = 0
    o = oracle.can_dual_alternating(w, *SIGNED, 32, 20, 1e-3, 10)
    # the first fit need not recover a1 = 2^-2 (MMSE shrinks the scale), but the pair must reproduce T
    # at least as well as the construction when it does; in any case the error is tiny and sweeps stop
    assert np.all(o["sse"] <= 1e-3 * np.sum(w.astype(np.float64) ** 2, axis=1))
    assert np.all(o["sweeps"] <= 10)


def test_alternating_rejects_non_finite_kernels():
    w = synth.small_weights(3, 50, 2, "normal")
    w[1, 7] = np.inf
    o = oracle.can_dual_alternating(w, *SIGNED, 32, 5, 1e-3, 4)
    assert np.isnan(o["scale1"][1]) and np.isnan(o["scale2"][1]) and np.isnan(o["sse"][1]) and o["sweeps"][1] == 0
    assert np.all(np.isfinite(o["sse"][[0, 2]]))
    z = np.zeros((2, 40), np.float32)
    o = oracle.can_dual_alternating(z, *SIGNED, 32, 5, 1e-3, 4)
    assert np.all(o["sse"] == 0) and np.all(o["sweeps"] == 1) and np.all(o["packed1"] == 0)


# ------------------------------------------------------------------ dual line search (Eq. 12)
def test_dual_objective_is_the_best_of_all_code_pairs():
    """Eq. 12: for fixed scales the per-element optimum over all 16 x 16 code pairs equals the
    enumeration over the first code with the second one rounded (brute force, fp64)."""
    rng = np.random.default_rng(0)
    x = rng.normal(0, 0.3, 40).astype(np.float32)
    codes = np.arange(-8, 8, dtype=np.float64)
    for a1, a2 in ((0.11, 0.013), (0.05, 0.05), (0.3, 0.002), (0.02, 0.015)):
        rec = a1 * codes[:, None] + a2 * codes[None, :]
        best = ((x.astype(np.float64)[:, None, None] - rec[None]) ** 2).reshape(x.size, -1).min(axis=1)
        assert oracle.def_dual_sse(x, a1, a2, *SIGNED) == pytest.approx(best.sum(), rel=1e-12)
        assert oracle.can_dual_sse(x, a1, a2, *SIGNED) == pytest.approx(best.sum(), rel=2e-5)


def test_dual_objective_never_worse_than_quantizing_the_residual():
    """The enumeration includes t = [T/a1], so with the same scales it cannot lose to the residual fit."""
    w = synth.small_weights(6, 200, 17, "student")
    s1, _, _ = oracle.can_search_kernelwise(w, *SIGNED, 64, 20)
    s2, _, e2, _ = oracle.can_residual_quantize(w, s1, *SIGNED, 64, 20)
    for k in range(6):
        assert oracle.can_dual_sse(w[k], s1[k], s2[k], *SIGNED) <= e2[k] * (1 + 1e-6)


def test_dual_linesearch_grid_argmin_codes_and_error():
    K, n, G1, G2 = 4, 150, 12, 10
    w = synth.small_weights(K, n, 23, "laplace")
    kw = oracle.can_dual_linesearch_kernelwise(w, *SIGNED, G1, G2)
    for k in range(K):
        r = oracle.can_dual_linesearch(w[k], *SIGNED, G1, G2, want_grid=True)
        g = r["grid"]
        flat = int(np.argmin(g))                                   # first minimum in row-major order
        assert (r["idx1"], r["idx2"]) == (flat // G2, flat % G2) and r["sse"] == g.min()
        a1 = oracle.can_grid(np.abs(w[k]).max(), 7, G1)[r["idx1"]]
        assert r["scale1"] == a1 and r["scale2"] == oracle.can_dual_alpha2(a1, G2, r["idx2"])
        assert r["scale2"] == np.float32(a1) * (np.float32(r["idx2"] + 1) / np.float32(G2))
        for (ja, jb) in ((0, 0), (3, 7), (G1 - 1, G2 - 1)):
            aa = oracle.can_grid(np.abs(w[k]).max(), 7, G1)[ja]
            assert g[ja, jb] == oracle.can_dual_sse(w[k], aa, oracle.can_dual_alpha2(aa, G2, jb), *SIGNED)
        d = oracle.def_sse_dual(w[k], r["q1"], r["q2"], float(r["scale1"]), float(r["scale2"]))
        assert d == pytest.approx(r["sse"], rel=3e-5)
        assert r["q1"].min() >= -8 and r["q1"].max() <= 7 and r["q2"].min() >= -8 and r["q2"].max() <= 7
        assert (kw["scale1"][k], kw["scale2"][k], kw["idx1"][k], kw["idx2"][k], kw["sse"][k]) == \
               (r["scale1"], r["scale2"], r["idx1"], r["idx2"], r["sse"])
    q1 = oracle.can_unpack_int4(kw["packed1"], K * n, True).reshape(K, n)
    np.testing.assert_array_equal(q1[2], oracle.can_dual_linesearch(w[2], *SIGNED, G1, G2)["q1"])


def test_dual_linesearch_finds_an_exact_two_grid_tensor():
    """T = a1*Q1 + a2*Q2 with a1 the max-abs scale and a2 = a1/4 on the grid: error 0 is reachable."""
    rng = np.random.default_rng(3)
    n, G1, G2 = 64, 8, 8
    a1, a2 = 2.0 ** -3, 2.0 ** -5
    q1 = rng.integers(-6, 7, n)
    q2 = rng.integers(-1, 2, n)
    q1[0], q2[0] = 7, 0
    x = (q1 * a1 + q2 * a2).astype(np.float32)
    x[0] = 7 * a1
    r = oracle.can_dual_linesearch(x, *SIGNED, G1, G2, want_grid=True)
    assert r["sse"] == 0.0 and r["grid"][G1 - 1, G2 // 4 - 1] == 0.0
    zeros = np.argwhere(r["grid"] == 0.0)
    assert len(zeros) >= 2                                   # a2 = a1/8 reproduces T as well (codes 2*Q2)
    assert (r["idx1"], r["idx2"]) == tuple(zeros[0])         # first of the equal minima in row-major order
    rec = float(r["scale1"]) * r["q1"] + float(r["scale2"]) * r["q2"]
    np.testing.assert_array_equal(rec.astype(np.float32), x)


def test_dual_codes_tie_rule():
    """2.25*a1 = 2*a1 + 2*a2 = 3*a1 - 6*a2 for a2 = a1/8: both code pairs are exact; the first code tried
    (the lowest) is kept.  Either pair is a correct answer; the rule only makes the output unique."""
    a1, a2 = 2.0 ** -3, 2.0 ** -6
    q1, q2 = oracle.can_dual_codes(np.array([2.25 * a1, 0.0, -2.25 * a1], np.float32), a1, a2, *SIGNED)
    np.testing.assert_array_equal(q1, [2, 0, -3])
    np.testing.assert_array_equal(q2, [2, 0, 6])


def test_dual_linesearch_beats_the_residual_fit_and_scales_exactly():
    w = synth.small_weights(5, 576, 3, "laplace")
    one = oracle.can_dual_alternating(w, *SIGNED, 256, 20, 0.0, 1)["sse"]
    o = oracle.can_dual_linesearch_kernelwise(w, *SIGNED, 24, 24)
    assert np.all(o["sse"] < 0.5 * one)            # the paper reports a 5x lower error on average
    o2 = oracle.can_dual_linesearch_kernelwise((w * np.float32(8)).astype(np.float32), *SIGNED, 24, 24)
    np.testing.assert_array_equal(o["idx1"], o2["idx1"])
    np.testing.assert_array_equal(o["idx2"], o2["idx2"])
    np.testing.assert_array_equal(o["packed1"], o2["packed1"])
    np.testing.assert_array_equal(o["packed2"], o2["packed2"])
    np.testing.assert_array_equal(o["sse"] * 64.0, o2["sse"])
    np.testing.assert_array_equal(o["scale2"] * np.float32(8), o2["scale2"])


def test_dual_linesearch_degenerate_inputs():
    z = np.zeros(30, np.float32)
    r = oracle.can_dual_linesearch(z, *SIGNED, 4, 4)
    assert (r["scale1"], r["scale2"], r["idx1"], r["idx2"], r["sse"], r["rc"]) == (1.0, 1.0, 0, 0, 0.0, 0)
    assert not r["q1"].any() and not r["q2"].any()
    z[3] = np.nan
    r = oracle.can_dual_linesearch(z, *SIGNED, 4, 4)
    assert r["rc"] == -1 and np.isnan(r["scale1"]) and r["idx1"] == -1 and np.isnan(r["sse"])


# ------------------------------------------------------------------ activation variants (Eq. 16, Eq. 2)
def test_activation_second_tensor_closed_form():
    """x = m + f/16 with first scale 1: the residual is f/16, f in -7..7, which a signed second tensor
    represents exactly with scale 1/16 = the last grid point, and with no smaller one."""
    rng = np.random.default_rng(11)
    m = rng.integers(0, 16, 300)
    f = rng.integers(-7, 8, 300)
    f[:2] = (-7, 7)
    m[f < 0] = np.maximum(m[f < 0], 1)                      # keep x >= 0
    x = (m + f / 16.0).astype(np.float32)
    for G in (8, 100):
        r = oracle.can_act_residual_quantize(x, 1.0, UNSIGNED, SIGNED, G, 20)
        assert (r["scale"], r["idx"], r["sse"]) == (np.float32(1 / 16), G - 1, 0.0)
        np.testing.assert_array_equal(oracle.can_unpack_int4(r["packed"], x.size, True), f)
    # an unsigned second range cannot code the negative residuals: their squares stay
    ru = oracle.can_act_residual_quantize(x, 1.0, UNSIGNED, UNSIGNED, 8, 0)
    assert ru["sse"] >= float(np.sum((f[f < 0] / 16.0) ** 2)) > 0


@pytest.mark.parametrize("seed", range(3))
def test_activation_second_tensor_error_is_the_reconstruction_error(seed):
    x = synth.acts_relu_normal(30000, seed)
    first = oracle.can_search(x, *UNSIGNED, 128, 20)
    b1 = first["scale"]
    for q2 in (SIGNED, UNSIGNED):
        r = oracle.can_act_residual_quantize(x, b1, UNSIGNED, q2, 128, 20)
        q1 = np.clip(np.rint(x.astype(np.float64) / float(b1)), *UNSIGNED)
        q2c = oracle.can_unpack_int4(r["packed"], x.size, q2[0] < 0).astype(np.float64)
        assert q2c.min() >= q2[0] and q2c.max() <= q2[1]
        rec = float(b1) * q1 + float(r["scale"]) * q2c                       # Eq. 16, in fp64
        err = float(np.sum((x.astype(np.float64) - rec) ** 2))
        assert abs(err - r["sse"]) <= 2e-5 * err
        assert r["sse"] < first["sse"]
    # the signed second range is the better choice for the (two-sided) residual
    assert oracle.can_act_residual_quantize(x, b1, UNSIGNED, SIGNED, 128, 20)["sse"] < \
        oracle.can_act_residual_quantize(x, b1, UNSIGNED, UNSIGNED, 128, 20)["sse"]


def test_activation_second_tensor_reduces_to_the_weight_residual_for_equal_ranges():
    w = synth.small_weights(1, 700, 9, "laplace")
    s1 = oracle.can_search(w[0], *SIGNED, 64, 10)["scale"]
    s2, j2, e2, p2 = oracle.can_residual_quantize(w, [s1], *SIGNED, 64, 10)
    r = oracle.can_act_residual_quantize(w[0], s1, SIGNED, SIGNED, 64, 10)
    assert (r["scale"], r["idx"], r["sse"]) == (s2[0], j2[0], e2[0])
    np.testing.assert_array_equal(r["packed"], p2)


def test_activation_second_tensor_of_an_exact_first_tensor_is_zero():
    x = (np.float32(0.375) * np.random.default_rng(2).integers(0, 16, 500)).astype(np.float32)
    r = oracle.can_act_residual_quantize(x, 0.375, UNSIGNED, SIGNED, 32, 5)
    assert (r["scale"], r["idx"], r["sse"], r["rc"]) == (1.0, 0, 0.0, 0) and not r["packed"].any()
    r = oracle.can_act_residual_quantize(x, np.nan, UNSIGNED, SIGNED, 32, 5)
    assert r["rc"] == -1 and np.isnan(r["scale"]) and r["idx"] == -1


def test_offset_form_hand_example():
    """T = {-1, 0, 1, 2}, 2 bits: delta = -1, shifted tensor {0,1,2,3}; scale 1 is exact, scale 1/2
    saturates 2 -> 1.5 and 3 -> 1.5: error 0.25 + 2.25."""
    x = np.array([1, -1, 0, 2], np.float32)
    o = oracle.can_offset_search(x, 3, 2, 0)
    assert (o["delta"], o["scale"], o["idx"], o["sse"]) == (-1.0, 1.0, 1, 0.0)
    np.testing.assert_array_equal(oracle.can_unpack_int4(o["packed"], 4, False), [2, 0, 1, 3])
    assert oracle.def_offset_sse(x, -1.0, 0.5, 3) == 2.5
    assert oracle.def_offset_sse(x, -1.0, 1.0, 3) == 0.0
    assert oracle.can_min(x) == -1.0


@pytest.mark.parametrize("seed", range(3))
def test_offset_form_last_grid_point_is_the_uniform_quantizer_of_eq2(seed):
    rng = np.random.default_rng(seed)
    x = rng.normal(1.5, 1.0, 4000).astype(np.float32)
    delta = np.float32(x.min())
    alpha_u = np.float32(np.float32(x.max() - delta) / np.float32(15))        # Eq. 2
    y = (x - delta).astype(np.float32)
    assert oracle.can_grid(oracle.can_absmax(y), 15, 37)[-1] == alpha_u
    # Eq. 2 evaluated directly in numpy fp64
    xd = x.astype(np.float64)
    that = float(alpha_u) * np.clip(np.rint((xd - float(delta)) / float(alpha_u)), 0, 15) + float(delta)
    e_u = float(np.sum((xd - that) ** 2))
    assert abs(oracle.def_offset_sse(x, delta, alpha_u, 15) - e_u) <= 1e-12 * e_u
    o = oracle.can_offset_search(x, 15, 37, 20)
    assert o["delta"] == delta and o["sse"] <= e_u * (1 + 1e-5)
    # the canonical error is that of the reconstruction alpha*codes + delta
    codes = oracle.can_unpack_int4(o["packed"], x.size, False).astype(np.float64)
    err = float(np.sum((xd - (float(o["scale"]) * codes + float(delta))) ** 2))
    assert abs(err - o["sse"]) <= 2e-5 * err
    assert abs(oracle.def_offset_sse(x, delta, o["scale"], 15) - o["sse"]) <= 2e-5 * err


def test_offset_form_is_shift_invariant_and_equals_the_unsigned_search_at_min_zero():
    rng = np.random.default_rng(4)
    x = (rng.integers(0, 4096, 3000) / 256.0).astype(np.float32)              # multiples of 2^-8 below 16
    x[0] = 0.0
    a = oracle.can_offset_search(x, 15, 64, 20)
    plain = oracle.can_search(x, *UNSIGNED, 64, 20)
    assert (a["delta"], a["scale"], a["idx"], a["sse"]) == (0.0, plain["scale"], plain["idx"], plain["sse"])
    np.testing.assert_array_equal(a["packed"], oracle.can_quantize_pack_int4(x, [plain["scale"]], *UNSIGNED))
    for c in (-8.0, 32.0, -1024.0):                                             # exact shifts
        b = oracle.can_offset_search((x + np.float32(c)).astype(np.float32), 15, 64, 20)
        assert (b["delta"], b["scale"], b["idx"], b["sse"]) == (c, a["scale"], a["idx"], a["sse"])
        np.testing.assert_array_equal(b["packed"], a["packed"])


def test_offset_form_beats_the_signed_form_on_asymmetric_data():
    x = np.random.default_rng(8).normal(3.0, 1.0, 6000).astype(np.float32)
    assert oracle.can_offset_search(x, 15, 128, 20)["sse"] < 0.5 * oracle.can_search(x, *SIGNED, 128, 20)["sse"]


def test_offset_form_degenerate_inputs():
    c = np.full(100, 2.5, np.float32)
    o = oracle.can_offset_search(c, 15, 16, 4)
    assert (o["delta"], o["scale"], o["idx"], o["sse"], o["rc"]) == (2.5, 1.0, 0, 0.0, 0) and not o["packed"].any()
    for bad in (np.nan, np.inf, -np.inf):
        c[7] = bad
        o = oracle.can_offset_search(c, 15, 16, 4)
        assert o["rc"] == -1 and np.isnan(o["delta"]) and np.isnan(o["scale"]) and o["idx"] == -1
        assert np.isnan(oracle.can_min(c))
    wide = np.array([2.0 ** 61, 0.0, 1.0], np.float32)       # finite, but the shifted range exceeds the accepted one
    o = oracle.can_offset_search(wide, 15, 16, 4)
    assert o["rc"] == -1 and np.isnan(o["delta"]) and np.isnan(o["scale"]) and not o["packed"].any()


# ------------------------------------------------------------------ comparison optimisers (Section 3.4, Table 2)
def np_ls_scale(x, alpha, qmin, qmax):
    """One alternating update in numpy fp64: codes for alpha, then the least-squares scale for those codes."""
    x = np.asarray(x, np.float64)
    q = np.clip(np.rint(x * float(np.float32(1.0) / np.float32(alpha))), qmin, qmax)
    return float(np.sum(x * q) / np.sum(q * q)), q


@pytest.mark.parametrize("kind", ["normal", "laplace", "outliers"])
def test_uniform_mode_is_the_max_abs_quantizer(kind):
    """One grid point and no refinement is Section 3.1's quantizer without offset."""
    w = synth.small_weights(6, 300, 12, kind)
    s, j, e = oracle.can_search_kernelwise(w, *SIGNED, 1, 0)
    for k in range(6):
        smax = np.float32(np.abs(w[k]).max()) / np.float32(7)
        assert s[k] == smax and j[k] == 0
        assert abs(e[k] - np_def_sse(w[k], smax, *SIGNED)) <= 1e-5 * e[k]


def test_golden_mode_searches_the_whole_range():
    """One grid point plus refinement is a golden-section search over (0, max-abs scale]."""
    x = synth.small_weights(1, 700, 5, "laplace")[0]
    smax = np.float32(np.abs(x).max()) / np.float32(7)
    o = oracle.can_search(x, *SIGNED, 1, 24, want_probes=True)
    pr = o["probes"]
    phi = np.float32(0.6180339887)
    assert abs(pr[0] - smax * (1 - phi)) <= 1e-6 * smax and abs(pr[1] - smax * phi) <= 1e-6 * smax
    assert np.all(pr > 0) and np.all(pr <= smax) and len(pr) == 26
    assert o["sse"] <= oracle.can_sse(x, smax, *SIGNED)
    # 24 iterations shrink the bracket to phi^24 of the range: the result is a local minimum at that resolution
    width = float(smax) * float(phi) ** 24
    for d in (-4 * width, 4 * width):
        assert o["sse"] <= oracle.can_sse(x, np.float32(o["scale"] + d), *SIGNED) * (1 + 1e-6)


@pytest.mark.parametrize("q", [SIGNED, UNSIGNED, (-1, 1)])
def test_alternating_first_update_is_the_least_squares_scale(q):
    x = synth.small_weights(1, 500, 21, "normal")[0]
    if q[0] == 0:
        x = np.abs(x)
    smax = np.float32(np.abs(x).max()) / np.float32(q[1])
    o = oracle.can_alternating_scale(x, *q, 1)
    ls, codes = np_ls_scale(x, smax, *q)
    assert o["updates"] == 1 and abs(float(o["scale"]) - ls) <= 1e-7 * ls
    # least squares: no other scale is better for these codes
    for f in (0.99, 1.01):
        assert oracle.def_sse_codes(x, codes.astype(np.int32), ls) < oracle.def_sse_codes(x, codes.astype(np.int32), ls * f)
    if q == (-1, 1):
        # ternary closed form: the mean magnitude of the elements beyond half the scale
        big = np.abs(x.astype(np.float64)) * float(np.float32(1) / smax) > 0.5
        assert abs(ls - np.abs(x.astype(np.float64))[big].mean()) <= 1e-12 * ls


def test_alternating_follows_the_update_rule_and_descends():
    x = synth.small_weights(1, 800, 33, "student")[0]
    alpha = np.float32(np.abs(x).max()) / np.float32(7)
    prev = oracle.can_sse(x, alpha, *SIGNED)
    for it in range(1, 12):
        o = oracle.can_alternating_scale(x, *SIGNED, it)
        ls, _ = np_ls_scale(x, alpha, *SIGNED)
        if np.float32(ls) == alpha:
            assert o["updates"] < it and o["scale"] == alpha
            break
        assert o["updates"] == it and abs(float(o["scale"]) - ls) <= 2e-7 * ls
        assert o["sse"] <= prev * (1 + 1e-6)                    # each half-step is optimal for its variable
        assert abs(o["sse"] - np_def_sse(x, o["scale"], *SIGNED)) <= 1e-5 * o["sse"]
        alpha, prev = o["scale"], o["sse"]


def test_alternating_closed_form_and_degenerate_inputs():
    x = (np.float32(0.25) * np.random.default_rng(3).integers(-7, 8, 400)).astype(np.float32)
    x[:2] = (-1.75, 1.75)
    o = oracle.can_alternating_scale(x, *SIGNED, 10)
    assert (o["scale"], o["sse"], o["updates"], o["rc"]) == (0.25, 0.0, 0, 0)        # the max-abs scale is already exact
    y = x.copy()
    y[0] = 4.0                                                 # one outlier: max-abs scale 4/7, optimum back at 0.25-ish
    o = oracle.can_alternating_scale(y, *SIGNED, 50)
    assert o["updates"] >= 1 and o["sse"] < oracle.can_sse(y, np.float32(4.0) / np.float32(7), *SIGNED)
    z = np.zeros(100, np.float32)
    o = oracle.can_alternating_scale(z, *SIGNED, 10)
    assert (o["scale"], o["sse"], o["updates"], o["rc"]) == (1.0, 0.0, 0, 0)
    z[5] = np.inf
    o = oracle.can_alternating_scale(z, *SIGNED, 10)
    assert o["rc"] == -1 and np.isnan(o["scale"]) and np.isnan(o["sse"])


def test_comparison_modes_order_as_in_table_2():
    """Uniform is the start of both iterative methods, so neither can be worse than it; the grid search with
    refinement is the best of the four on aggregate (the paper's accuracy ordering, here in MSE)."""
    for kind in ("normal", "laplace", "student"):
        w = synth.small_weights(48, 576, 17, kind)
        e_uni = oracle.can_search_kernelwise(w, *SIGNED, 1, 0)[2]
        e_gold = oracle.can_search_kernelwise(w, *SIGNED, 1, 20)[2]
        e_omse = oracle.can_search_kernelwise(w, *SIGNED, 256, 20)[2]
        a_alt, e_alt, _ = oracle.can_alternating_scale_kernelwise(w, *SIGNED, 50)
        assert np.all(e_alt <= e_uni * (1 + 1e-6)) and np.all(e_gold <= e_uni) and np.all(e_omse <= e_uni)
        assert e_omse.sum() < e_gold.sum() < e_uni.sum() and e_omse.sum() < e_alt.sum() < e_uni.sum()
        for k in (0, 47):
            one = oracle.can_alternating_scale(w[k], *SIGNED, 50)
            assert (one["scale"], one["sse"]) == (a_alt[k], e_alt[k])


# ------------------------------------------------------------------ workloads
def test_workload_shapes_match_architectures():
    c = [synth.config(i) for i in range(1, 6)]
    assert c[0].weight_elements == 36864 and c[0].act_elements == 524288
    assert c[1].weight_elements == 11678912 and len(c[1].weight_shapes) == 21
    assert c[2].weight_elements == 3469760 and len(c[2].weight_shapes) == 53
    assert sum(s.K for s in c[2].weight_shapes if s.n == 9) == 7136
    assert c[3].weight_elements == 25502912 and len(c[3].weight_shapes) == 54
    assert c[3].act_elements == 341262336
    assert c[4].weight_elements == 138344128 and len(c[4].weight_shapes) == 16
    assert c[4].act_elements == 145842176
    w0 = c[1].weight_tensor(0)
    assert w0.dtype == np.float32 and w0.shape == (64, 147)
    np.testing.assert_array_equal(w0, c[1].weight_tensor(0))    # seeded
