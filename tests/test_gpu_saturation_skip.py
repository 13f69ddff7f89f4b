"""The sweeps leave the saturation out for chunks whose largest magnitude stays inside the integer range at the
smallest scale of a wave.  These cases put chunk maxima right at, just below and just above that limit for every
wave, in both signs and in signed and unsigned ranges, and compare every grid error with the oracle bit for bit."""
import sys

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


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


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def boundary_tensor(K, nchunks, tail, q, G, seed):
    """Kernels whose chunks have their extreme element at (limit + 1/2) times the first scale of each block of 64
    candidates, and one float above and below it; small noise elsewhere; a ragged tail."""
    qmin, qmax = q
    rng = np.random.default_rng(seed)
    n = 64 * nchunks + tail
    w = (rng.standard_normal((K, n)) * 0.01).astype(np.float32)
    if qmin == 0:
        w = np.abs(w)
    for k in range(K):
        a = np.float32(1.0 + 0.37 * k)
        w[k, 3] = a                                     # the kernel's abs-max, in chunk 0
        smax = np.float32(a / np.float32(qmax))
        for c in range(1, nchunks):
            block = (c * 7 + k) % max(1, (G + 63) // 64)
            alpha = np.float32(smax * (np.float32(64 * block + 1) / np.float32(G)))
            limit = qmax if (c + k) % 3 else (-qmin if qmin < 0 else qmax)
            v = np.float32(alpha * np.float32(limit + 0.5))
            v = [v, np.nextafter(v, np.float32(0)), np.nextafter(v, np.float32(np.inf))][(c + 2 * k) % 3]
            sign = -1.0 if (qmin < 0 and (c + k) % 2) else 1.0
            if abs(v) < a:
                w[k, 64 * c + (c * 5) % 64] = np.float32(sign * v)
        if qmin == 0 and nchunks > 2:
            w[k, 64 * 2 + 9] = np.float32(-0.004)       # a negative element in an unsigned range: never skipped
    return w


@pytest.mark.parametrize("q", [(-8, 7), (0, 15), (-2, 1), (0, 3)])
@pytest.mark.parametrize("G,cpl", [(256, 0), (512, 0), (500, 2), (128, 1), (1024, 0)])
def test_kernelwise_grid_at_the_skip_limit(B, q, G, cpl):
    for nchunks, tail in ((9, 0), (72, 17), (130, 5), (200, 0)):      # one tile, two masks, streaming tiles
        w = boundary_tensor(5, nchunks, tail, q, G, 77 + nchunks)
        say(f"skip limit kernelwise q={q} G={G} cpl={cpl} n={w.shape[1]}")
        absmax, grid = B.mmse_grid_sse_kernelwise(dev(w), B.params(*q, G, 0, cpl))
        grid = grid.cpu().numpy()
        for k in range(w.shape[0]):
            r = oracle.can_search(w[k], *q, G, 0, want_grid=True)
            np.testing.assert_array_equal(grid[k], r["grid_sse"], err_msg=f"k={k} n={w.shape[1]}")


@pytest.mark.parametrize("q", [(0, 15), (-8, 7)])
@pytest.mark.parametrize("G", [256, 512, 128])
def test_activation_grid_at_the_skip_limit(B, q, G):
    w = boundary_tensor(1, 150, 31, q, G, 5)[0]          # three blocks, the last one ragged
    say(f"skip limit activation q={q} G={G} N={w.size}")
    absmax, grid = B.mmse_grid_sse_activation(dev(w), B.params(*q, G, 0))
    r = oracle.can_search(w, *q, G, 0, want_grid=True)
    np.testing.assert_array_equal(grid.cpu().numpy().reshape(-1), r["grid_sse"])


@pytest.mark.parametrize("q", [(-8, 7), (0, 15)])
def test_whole_search_at_the_skip_limit(B, q):
    w = boundary_tensor(40, 72, 0, q, 256, 11)
    say(f"skip limit search q={q}")
    r = B.mmse_scale_search_batched([dev(w), dev(w[:, :1100])], B.params(*q, 256, 20), want_packed=True)
    for x, got in zip((w, w[:, :1100]), r):
        s, j, e = oracle.can_search_kernelwise(np.ascontiguousarray(x), *q, 256, 20)
        np.testing.assert_array_equal(got.idx.cpu().numpy(), j)
        np.testing.assert_array_equal(got.scale.cpu().numpy(), s)
        np.testing.assert_array_equal(got.sse.cpu().numpy(), e)
        np.testing.assert_array_equal(got.packed.cpu().numpy(),
                                      oracle.can_quantize_pack_int4(np.ascontiguousarray(x), s, *q))
