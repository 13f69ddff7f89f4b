"""GPU parity of the dual line search (Section 3.5, Eq. 12) against the oracle: scales, grid indices,
errors and both code tensors bit for bit."""
import sys

import numpy as np
import pytest

import oracle
from paper_1902_06822_amd import synth

pytestmark = pytest.mark.gpu
SIGNED = (-8, 7)


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1902_06822_amd import binding
    binding.load_library()
    return binding


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def compare(B, w, q, G1, G2, tag, want_grid=False):
    import torch
    r = B.dual_line_search(torch.from_numpy(w).cuda(), q[0], q[1], G1, G2, want_grid=want_grid)
    torch.cuda.synchronize()
    o = oracle.can_dual_linesearch_kernelwise(w, q[0], q[1], G1, G2)
    np.testing.assert_array_equal(r.idx1.cpu().numpy(), o["idx1"], err_msg=f"idx1 {tag}")
    np.testing.assert_array_equal(r.idx2.cpu().numpy(), o["idx2"], err_msg=f"idx2 {tag}")
    for name, got, ref, tol in (("scale1", r.scale1, o["scale1"], 1e-6), ("scale2", r.scale2, o["scale2"], 1e-6),
                                ("sse", r.sse, o["sse"], 1e-4)):
        g = got.cpu().numpy()
        np.testing.assert_allclose(g, ref, rtol=tol, atol=0, err_msg=f"{name} {tag}")
        np.testing.assert_array_equal(g, ref, err_msg=f"{name} bits {tag}")
    np.testing.assert_array_equal(r.packed1.cpu().numpy(), o["packed1"], err_msg=f"codes1 {tag}")
    np.testing.assert_array_equal(r.packed2.cpu().numpy(), o["packed2"], err_msg=f"codes2 {tag}")
    return r, o


@pytest.mark.parametrize("K,n,kind,G1,G2", [
    (40, 9, "outliers", 16, 16), (12, 27, "normal", 32, 32), (9, 147, "laplace", 20, 70),
    (8, 576, "laplace", 24, 64), (3, 1152, "student", 16, 24), (2, 4608, "laplace", 8, 12),
    (5, 64, "normal", 32, 16), (7, 130, "laplace", 5, 130), (1, 8192, "normal", 4, 6),
    (600, 9, "normal", 12, 8), (3, 7, "outliers", 1, 1), (4, 63, "student", 64, 1), (4, 65, "student", 1, 64),
    (2, 64, "normal", 1024, 3), (2, 70, "laplace", 3, 1024), (16, 9, "normal", 1024, 1024)])   # the largest grids
def test_dual_line_search_matches_oracle(B, K, n, kind, G1, G2):
    say(f"dual line search K={K} n={n} {kind} G1={G1} G2={G2}")
    w = synth.small_weights(K, n, 9100 + K + n, kind)
    compare(B, w, SIGNED, G1, G2, f"K={K} n={n}")


def test_dual_line_search_full_grid_of_errors(B):
    say("dual line search: every grid error")
    w = synth.small_weights(6, 200, 31, "laplace")
    G1, G2 = 12, 70
    r, _ = compare(B, w, SIGNED, G1, G2, "grid", want_grid=True)
    g = r.grid.cpu().numpy().reshape(6, G1, G2)
    for k in range(6):
        o = oracle.can_dual_linesearch(w[k], *SIGNED, G1, G2, want_grid=True)
        np.testing.assert_array_equal(g[k], o["grid"], err_msg=f"grid row {k}")


def test_dual_line_search_narrow_ranges(B):
    say("dual line search: ternary and unsigned ranges")
    w = synth.small_weights(10, 100, 77, "normal")
    compare(B, w, (-1, 1), 16, 16, "ternary")
    compare(B, w, (-2, 1), 16, 16, "int2")
    compare(B, np.abs(w), (0, 15), 16, 16, "unsigned")


def test_dual_line_search_degenerate_kernels(B):
    say("dual line search: zero, tiny, huge, inf and NaN kernels among ordinary ones")
    w = synth.small_weights(8, 90, 5, "normal")
    w[1] = 0.0
    w[2] = np.float32(2.0 ** -70)
    w[3, 4] = np.float32(2.0 ** 61)
    w[4, 0] = np.inf
    w[5, 89] = np.nan
    import torch
    r = B.dual_line_search(torch.from_numpy(w).cuda(), *SIGNED, 16, 16, want_grid=True)
    torch.cuda.synchronize()
    o = oracle.can_dual_linesearch_kernelwise(w, *SIGNED, 16, 16)
    for name in ("scale1", "scale2", "idx1", "idx2", "sse", "packed1", "packed2"):
        np.testing.assert_array_equal(getattr(r, name).cpu().numpy(), o[name], err_msg=name)
    assert np.all(np.isnan(r.scale1.cpu().numpy()[3:6])) and np.all(r.idx1.cpu().numpy()[3:6] == -1)
    assert r.scale1.cpu().numpy()[1] == 1.0 and r.sse.cpu().numpy()[1] == 0.0
    g = r.grid.cpu().numpy()
    assert np.all(np.isnan(g[3:6])) and np.all(g[1] == 0.0)


def test_dual_line_search_beats_alternating_start(B):
    """The exhaustive pair is never worse than the one-shot residual fit restricted to the same grids'
    corner (a1 = max-abs scale, a2 = a1): a property that holds at any size."""
    import torch
    say("dual line search: property check on a full layer")
    c = synth.config(1)
    w = c.weight_tensor(0)
    K, n = w.shape
    r = B.dual_line_search(torch.from_numpy(w).cuda(), *SIGNED, 16, 16, want_grid=True)
    torch.cuda.synchronize()
    g = r.grid.cpu().numpy()
    sse = r.sse.cpu().numpy()
    np.testing.assert_array_equal(sse, g.min(axis=1))
    flat = r.idx1.cpu().numpy() * 16 + r.idx2.cpu().numpy()
    np.testing.assert_array_equal(flat, g.argmin(axis=1))
    rows = [0, K // 2, K - 1]
    o = oracle.can_dual_linesearch_kernelwise(np.ascontiguousarray(w[rows]), *SIGNED, 16, 16)
    np.testing.assert_array_equal(sse[rows], o["sse"])
    np.testing.assert_array_equal(r.scale2.cpu().numpy()[rows], o["scale2"])


def test_dual_line_search_rejects_bad_arguments(B):
    import torch
    w = torch.zeros((2, 8193), dtype=torch.float32, device="cuda")
    with pytest.raises(RuntimeError):
        B.dual_line_search(w, *SIGNED, 8, 8)
    w = torch.zeros((2, 16), dtype=torch.float32, device="cuda")
    for bad in ((0, 8), (8, 0), (1025, 8), (8, 1025)):
        with pytest.raises(RuntimeError):
            B.dual_line_search(w, *SIGNED, *bad)
    with pytest.raises(RuntimeError):
        B.dual_line_search(w, 1, 7, 8, 8)
