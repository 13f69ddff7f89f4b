"""The activation sweep stages every 64-element chunk compacted to its non-zero elements (a zero adds nothing to a
chunk's sum at any scale).  These cases give chunks every interesting number of non-zero elements (none, one, around
the multiples of eight the compacted chunk is padded to, all), zeros of both signs, tiny values that are not zero,
whole blocks of zeros and a ragged tail, and compare grid errors, scale, error and codes with the oracle bit for
bit."""
import sys

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

COUNTS = (0, 1, 2, 7, 8, 9, 15, 16, 17, 31, 32, 33, 55, 56, 57, 62, 63, 64)


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


def sparse_tensor(nchunks, tail, signed, seed, zero_blocks=()):
    """Chunk c holds COUNTS[(c + seed) % len] non-zero elements at random places; every third zero is -0.0; some of
    the non-zero elements are the smallest subnormal; the blocks of 4096 listed in zero_blocks are all zero."""
    rng = np.random.default_rng(seed)
    n = 64 * nchunks + tail
    x = np.zeros(n, np.float32)
    for c in range((n + 63) // 64):
        m = min(64, n - 64 * c)
        cnt = min(COUNTS[(c + seed) % len(COUNTS)], m)
        where = rng.choice(m, cnt, replace=False)
        v = np.abs(rng.standard_normal(cnt)).astype(np.float32) * np.float32(0.5 + (c % 5))
        if signed:
            v *= rng.choice(np.array([-1.0, 1.0], np.float32), cnt)
        if cnt > 2:
            v[0] = np.float32(1e-45) if not signed or c % 2 else np.float32(-1e-45)
        x[64 * c + where] = v
    for b in zero_blocks:
        x[4096 * b:4096 * (b + 1)] = 0.0
    z = np.flatnonzero(x == 0.0)
    x[z[::3]] = np.float32(-0.0)
    return x


@pytest.mark.parametrize("q", [(0, 15), (-8, 7), (0, 3)])
@pytest.mark.parametrize("G", [512, 256, 100, 2048])          # two candidates per lane, two sets of waves, one, four
def test_grid_errors_of_sparse_chunks(B, q, G):
    for nchunks, tail, zb in ((64, 0, ()), (150, 31, ()), (200, 5, (1,)), (3, 1, ()), (0, 7, ())):
        x = sparse_tensor(nchunks, tail, q[0] < 0, 3 + nchunks, zb)
        say(f"zero compaction grid q={q} G={G} N={x.size} zero blocks={zb}")
        absmax, grid = B.mmse_grid_sse_activation(dev(x), B.params(*q, G, 0))
        r = oracle.can_search(x, *q, G, 0, want_grid=True)
        np.testing.assert_array_equal(grid.cpu().numpy().reshape(-1), r["grid_sse"], err_msg=f"N={x.size}")


@pytest.mark.parametrize("q", [(0, 15), (-8, 7)])
@pytest.mark.parametrize("G", [512, 200, 64, 1500])
def test_search_and_codes_of_sparse_tensors(B, q, G):
    xs = [sparse_tensor(130, 9, q[0] < 0, 21, (0,)), sparse_tensor(64, 0, q[0] < 0, 22),
          sparse_tensor(1, 3, q[0] < 0, 23), sparse_tensor(700, 63, q[0] < 0, 24, (3, 9))]
    say(f"zero compaction search q={q} G={G} sizes={[x.size for x in xs]}")
    got = B.mmse_scale_search_activation_batched([dev(x) for x in xs], B.params(*q, G, 20), want_packed=True)
    for i, (x, g) in enumerate(zip(xs, got)):
        o = oracle.can_search(x, *q, G, 20)
        assert int(g.idx[0]) == o["idx"], f"idx of tensor {i}"
        np.testing.assert_array_equal(g.scale.cpu().numpy(), np.array([o["scale"]], np.float32), err_msg=f"scale {i}")
        np.testing.assert_array_equal(g.sse.cpu().numpy(), np.array([o["sse"]]), err_msg=f"sse {i}")
        np.testing.assert_array_equal(g.packed.cpu().numpy(), oracle.can_quantize_pack_int4(x, [o["scale"]], *q),
                                      err_msg=f"codes {i}")


def test_one_nonzero_element_in_a_large_tensor(B):
    x = np.zeros(3 * 4096 + 17, np.float32)
    x[2 * 4096 + 1234] = np.float32(3.25)
    say("zero compaction: one non-zero element")
    absmax, grid = B.mmse_grid_sse_activation(dev(x), B.params(0, 15, 512, 0))
    r = oracle.can_search(x, 0, 15, 512, 0, want_grid=True)
    np.testing.assert_array_equal(grid.cpu().numpy().reshape(-1), r["grid_sse"])


def test_a_workspace_that_held_another_tensor(B):
    """The compacted copy and its chunk words live in the caller's workspace: a second search in the same workspace
    must not see what the first one left there (a larger, denser tensor, then smaller and sparser ones)."""
    p = B.params(0, 15, 512, 20)
    big = np.abs(np.random.default_rng(3).normal(0, 1, 4096 * 9 + 77)).astype(np.float32) + np.float32(0.01)   # no zeros
    ws = B.alloc_workspace(B.mmse_workspace_bytes_activation(big.size, p))
    say("zero compaction: one workspace, several tensors in a row")
    for x in (big, sparse_tensor(300, 11, False, 5, (2,)), sparse_tensor(40, 0, False, 6), big[:4096 * 2 + 5] * (big[:4096 * 2 + 5] > 1.0)):
        x = np.ascontiguousarray(x, np.float32)
        got = B.mmse_scale_search_activation(dev(x), p, ws)
        o = oracle.can_search(x, 0, 15, 512, 20)
        assert int(got.idx[0]) == o["idx"]
        np.testing.assert_array_equal(got.scale.cpu().numpy(), np.array([o["scale"]], np.float32))
        np.testing.assert_array_equal(got.sse.cpu().numpy(), np.array([o["sse"]]))
