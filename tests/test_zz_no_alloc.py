"""The entry point for callers that cannot allocate (mmse_scale_search_kernelwise_noalloc: the per-kernel
abs-max lives in a fixed device array inside the library) against mmse_scale_search_kernelwise, through the
raw C ABI, on two calls in a row, the second with a smaller input; then the same against the oracle."""
import ctypes as C
import sys

import numpy as np
import pytest

import oracle
from paper_1902_06822_amd import synth

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


def run_both(B, w, G, iters):
    import torch
    lib = B.load_library()
    K, n = w.shape
    wd = torch.from_numpy(w).cuda()
    p = B.params(-8, 7, G, iters)
    stream = torch.cuda.current_stream().cuda_stream

    def outputs():
        return (torch.full((K,), -1.0, dtype=torch.float32, device="cuda"),
                torch.full((K,), -7, dtype=torch.int32, device="cuda"),
                torch.full((K,), -1.0, dtype=torch.float64, device="cuda"))

    s0, j0, e0 = outputs()
    ws = B.alloc_workspace(B.mmse_workspace_bytes_kernelwise(K, n, p))
    rc = lib.mmse_scale_search_kernelwise(wd.data_ptr(), K, n, C.byref(p), s0.data_ptr(), j0.data_ptr(), e0.data_ptr(),
                                          ws.data_ptr(), ws.numel(), stream)
    assert rc == 0
    s1, j1, e1 = outputs()
    rc = lib.mmse_scale_search_kernelwise_noalloc(wd.data_ptr(), K, n, C.byref(p), s1.data_ptr(), j1.data_ptr(),
                                                  e1.data_ptr(), stream)
    assert rc == 0, B.status_string(rc)
    torch.cuda.synchronize()
    got = (s1.cpu().numpy(), j1.cpu().numpy(), e1.cpu().numpy())
    ref = (s0.cpu().numpy(), j0.cpu().numpy(), e0.cpu().numpy())
    for g, r, name in zip(got, ref, ("scale", "idx", "sse")):
        np.testing.assert_array_equal(g, r, err_msg=f"{name} K={K} n={n}")
    return got


def test_noalloc_entry_point_matches_the_workspace_one(B):
    G, iters = 256, 20
    # first call: 3000 kernels of 576 weights (several workgroups of the refinement, a ragged last one)
    say("no-alloc entry point: K=3000 n=576")
    w_big = synth.small_weights(3000, 576, seed=71, kind="laplace")
    got_big = run_both(B, w_big, G, iters)
    # second call, smaller, on the same scratch array: 37 kernels of 147 weights (odd n, partial chunk)
    say("no-alloc entry point: K=37 n=147")
    w_small = synth.small_weights(37, 147, seed=72, kind="student")
    got_small = run_both(B, w_small, G, iters)
    for w, got in ((w_big, got_big), (w_small, got_small)):
        s, j, e = oracle.can_search_kernelwise(w, -8, 7, G, iters)
        np.testing.assert_array_equal(got[1], j)
        np.testing.assert_allclose(got[0], s, rtol=1e-6, atol=0)
        np.testing.assert_allclose(got[2], e, rtol=1e-4, atol=0)


def test_noalloc_entry_point_rejects_what_it_cannot_hold(B):
    lib = B.load_library()
    p = B.params(-8, 7, 256, 20)
    a = 0x10000                      # never dereferenced: the call fails in validation
    assert lib.mmse_scale_search_kernelwise_noalloc(a, 262145, 8, C.byref(p), a, a, a, None) == -2
    assert lib.mmse_scale_search_kernelwise_noalloc(None, 8, 8, C.byref(p), a, a, a, None) == -1
    assert lib.mmse_scale_search_kernelwise_noalloc(a, 8, 8, None, a, a, a, None) == -1
