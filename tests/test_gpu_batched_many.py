"""Batched weight search over more tensors than one launch holds (59; 36 for the calls whose tensors use stored
codes of another tensor): mixed kernel sizes, tiny kernels (at most 64 elements) sharing the sweep launch with
ordinary ones, long kernels that stream through LDS.  Everything equal to the oracle."""
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


def make_tensors(G, longk):
    rng = np.random.default_rng(190206822 + G)
    shapes = []
    for i in range(57):
        n = int(rng.choice([1, 8, 9, 27, 63, 64, 65, 147, 576, 1152, 2304]))
        shapes.append((int(rng.integers(1, 12)), n))
    shapes += [(3000, 9), (70, 64), (5, 4608)]
    if longk:
        shapes += [(2, 25088), (1, 9000)]
    ws = [synth.small_weights(K, n, 7000 + 31 * i, ("laplace", "normal", "student", "outliers")[i % 4])
          for i, (K, n) in enumerate(shapes)]
    return shapes, ws


@pytest.mark.parametrize("G,iters,longk", [(256, 20, False), (512, 7, False), (96, 3, True), (640, 2, False), (320, 0, False)])
def test_more_tensors_than_one_launch_holds(B, G, iters, longk):
    import torch
    shapes, ws_host = make_tensors(G, longk)
    say(f"{len(shapes)} tensors, G={G}, iters={iters}, long kernels: {longk}")
    dev = [torch.from_numpy(w).cuda() for w in ws_host]
    p = B.params(-8, 7, G, iters)
    got = B.mmse_scale_search_batched(dev, p, want_packed=True)
    torch.cuda.synchronize()
    for i, w in enumerate(ws_host):
        s, j, e = oracle.can_search_kernelwise(w, -8, 7, G, iters)
        pk = oracle.can_quantize_pack_int4(w, s, -8, 7)
        np.testing.assert_array_equal(got[i].idx.cpu().numpy(), j, err_msg=f"idx tensor {i} {shapes[i]}")
        np.testing.assert_array_equal(got[i].scale.cpu().numpy(), s, err_msg=f"scale tensor {i} {shapes[i]}")
        np.testing.assert_array_equal(got[i].sse.cpu().numpy(), e, err_msg=f"sse tensor {i} {shapes[i]}")
        np.testing.assert_array_equal(got[i].packed.cpu().numpy(), pk, err_msg=f"codes tensor {i} {shapes[i]}")
    if G == 256:
        # second tensor on the residual of all of them
        got2 = B.mmse_scale_search_batched(dev, p, want_packed=True, scale1=[r.scale for r in got])
        torch.cuda.synchronize()
        for i, w in enumerate(ws_host):
            s2, j2, e2, p2 = oracle.can_residual_quantize(w, got[i].scale.cpu().numpy(), -8, 7, G, iters)
            np.testing.assert_array_equal(got2[i].idx.cpu().numpy(), j2, err_msg=f"idx2 tensor {i}")
            np.testing.assert_array_equal(got2[i].scale.cpu().numpy(), s2, err_msg=f"scale2 tensor {i}")
            np.testing.assert_array_equal(got2[i].packed.cpu().numpy(), p2, err_msg=f"codes2 tensor {i}")


def test_alternating_two_tensor_fit_over_more_layers_than_one_launch_holds(B):
    """Algorithm 1 iterated, batched over 45 layers: its later sweeps read stored codes (the extension fields of
    the descriptor table, 36 tensors per launch)."""
    import torch
    rng = np.random.default_rng(190206822 + 77)
    shapes = [(int(rng.integers(1, 6)), int(rng.choice([9, 27, 64, 130, 576]))) for _ in range(45)]
    ws_host = [synth.small_weights(K, n, 9100 + i, ("laplace", "student")[i % 2]) for i, (K, n) in enumerate(shapes)]
    say(f"dual alternating, {len(shapes)} layers")
    dev = [torch.from_numpy(w).cuda() for w in ws_host]
    p = B.params(-8, 7, 64, 6)
    got = B.dual_quantize_alternating_batched(dev, p, 1e-3, 4)
    torch.cuda.synchronize()
    for i, w in enumerate(ws_host):
        ref = oracle.can_dual_alternating(w, -8, 7, 64, 6, 1e-3, 4)
        np.testing.assert_array_equal(got[i].sweeps.cpu().numpy(), ref["sweeps"], err_msg=f"sweeps layer {i}")
        np.testing.assert_array_equal(got[i].scale1.cpu().numpy(), ref["scale1"], err_msg=f"scale1 layer {i}")
        np.testing.assert_array_equal(got[i].scale2.cpu().numpy(), ref["scale2"], err_msg=f"scale2 layer {i}")
        np.testing.assert_array_equal(got[i].packed1.cpu().numpy(), ref["packed1"], err_msg=f"codes1 layer {i}")
        np.testing.assert_array_equal(got[i].packed2.cpu().numpy(), ref["packed2"], err_msg=f"codes2 layer {i}")
