"""GPU parity at the full sizes of the benchmark's configurations 4 and 5, in the launch
configuration ``bench.py`` times (the batched whole-net entry point; the per-layer activation
entry point).  The comparisons are complete: every kernel and every tensor of both
configurations, first and second tensor, all codes."""
import sys

import numpy as np
import pytest

import oracle
from paper_1902_06822_amd import select, synth

pytestmark = pytest.mark.gpu
SIGNED = (-8, 7)
UNSIGNED = (0, 15)


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


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_equal(r, s, i, e, tag):
    np.testing.assert_array_equal(r.idx.cpu().numpy(), i, err_msg=f"idx {tag}")
    np.testing.assert_allclose(r.scale.cpu().numpy(), s, rtol=1e-6, atol=0, err_msg=f"scale {tag}")
    np.testing.assert_allclose(r.sse.cpu().numpy(), e, rtol=1e-4, atol=0, err_msg=f"sse {tag}")
    np.testing.assert_array_equal(r.scale.cpu().numpy(), s, err_msg=f"scale bits {tag}")
    np.testing.assert_array_equal(r.sse.cpu().numpy(), e, err_msg=f"sse bits {tag}")


def test_config4_weights_with_selected_residual_layers(B):
    import torch
    c = synth.config(4)
    say("config 4: 54 weight tensors, batched")
    ws = [c.weight_tensor(i) for i in range(len(c.weight_shapes))]
    dev = [to_dev(w) for w in ws]
    p = B.params(*SIGNED, c.grid_points, c.refine_iters)
    res = B.mmse_scale_search_batched(dev, p, want_packed=True)
    torch.cuda.synchronize()
    ref = []
    for i, (w, r) in enumerate(zip(ws, res)):
        s, j, e = oracle.can_search_kernelwise(w, *SIGNED, c.grid_points, c.refine_iters)
        ref.append((s, j, e))
        check_equal(r, s, j, e, f"cfg4 tensor {i}")
        np.testing.assert_array_equal(r.packed.cpu().numpy(), oracle.can_quantize_pack_int4(w, s, *SIGNED))
    # key layers: top 10 % by normalised error (host rule), second tensor on those only
    energy = [float(np.sum(w.astype(np.float64) ** 2)) for w in ws]
    layer_sse = B.mmse_layer_error_sums([r.sse for r in res]).cpu().numpy()
    np.testing.assert_allclose(layer_sse, [e.sum() for (_, _, e) in ref], rtol=1e-13, atol=0)
    nmse = select.normalized_mse(list(layer_sse), energy)
    key = select.select_top_fraction(nmse, 0.10)
    assert len(key) == 5
    say(f"config 4: residual on layers {key}")
    res2 = B.mmse_scale_search_batched([dev[i] for i in key], p, want_packed=True,
                                       scale1=[res[i].scale for i in key])
    torch.cuda.synchronize()
    for i, r2 in zip(key, res2):
        s2, j2, e2, p2 = oracle.can_residual_quantize(ws[i], ref[i][0], *SIGNED, c.grid_points, c.refine_iters)
        check_equal(r2, s2, j2, e2, f"cfg4 residual layer {i}")
        np.testing.assert_array_equal(r2.packed.cpu().numpy(), p2)
        assert np.all(r2.sse.cpu().numpy() <= res[i].sse.cpu().numpy())


@pytest.mark.parametrize("cfg,which", [(4, "largest"), (4, "first"), (4, "last"), (5, "largest"), (5, "last")])
def test_full_size_activation_tensors(B, cfg, which):
    import torch
    c = synth.config(cfg)
    sizes = [a.per_image for a in c.act_shapes]
    li = {"largest": int(np.argmax(sizes)), "first": 0, "last": len(sizes) - 1}[which]
    N = c.act_shapes[li].numel(c.act_batch)
    say(f"config {cfg}: activation tensor {c.act_shapes[li].name} N={N} G={c.grid_points}")
    x = c.act_tensor(li)
    xd = to_dev(x)
    p = B.params(*UNSIGNED, c.grid_points, c.refine_iters)
    r = B.mmse_scale_search_activation(xd, p)
    packed = B.quantize_pack_int4(xd, r.scale, *UNSIGNED)
    torch.cuda.synchronize()
    o = oracle.can_search(x, *UNSIGNED, c.grid_points, c.refine_iters)
    check_equal(r, np.array([o["scale"]], np.float32), np.array([o["idx"]], np.int32), np.array([o["sse"]]),
                f"cfg{cfg} act {li}")
    np.testing.assert_array_equal(packed.cpu().numpy(), oracle.can_quantize_pack_int4(x, [o["scale"]], *UNSIGNED))
    if which == "largest":       # every grid error of the full-size tensor
        amax, grid = B.mmse_grid_sse_activation(xd, B.params(*UNSIGNED, c.grid_points, 0))
        torch.cuda.synchronize()
        og = oracle.can_search(x, *UNSIGNED, c.grid_points, 0, want_grid=True)
        np.testing.assert_array_equal(grid.cpu().numpy(), og["grid_sse"], err_msg=f"cfg{cfg} act {li} grid errors")
        assert float(amax[0]) == float(x.max())
    # invariant that holds at any size: the result is no worse than the max-abs scale
    assert float(r.sse[0]) <= oracle.can_sse(x, np.float32(x.max()) / np.float32(15), *UNSIGNED)


@pytest.mark.parametrize("cfg", [4, 5])
def test_full_size_activation_second_tensor_and_offset_form(B, cfg):
    """Eq. 16 and Eq. 2 on the largest calibration tensor of the configuration, complete comparison."""
    import torch
    c = synth.config(cfg)
    li = int(np.argmax([a.per_image for a in c.act_shapes]))
    x = c.act_tensor(li)
    say(f"config {cfg}: second tensor and offset form of {c.act_shapes[li].name} N={x.size}")
    xd = to_dev(x)
    G, it = c.grid_points, c.refine_iters
    first = B.mmse_scale_search_activation(xd, B.params(*UNSIGNED, G, it))
    r2 = B.activation_residual_quantize(xd, first.scale, *UNSIGNED, B.params(*SIGNED, G, it))
    torch.cuda.synchronize()
    o1 = oracle.can_search(x, *UNSIGNED, G, it)
    o2 = oracle.can_act_residual_quantize(x, o1["scale"], UNSIGNED, SIGNED, G, it)
    assert float(first.scale[0]) == o1["scale"]
    check_equal(r2, np.array([o2["scale"]], np.float32), np.array([o2["idx"]], np.int32), np.array([o2["sse"]]),
                f"cfg{cfg} second tensor")
    np.testing.assert_array_equal(r2.packed.cpu().numpy(), o2["packed"])
    assert float(r2.sse[0]) < o1["sse"]
    del r2
    y = x - np.float32(0.75)                       # a pre-activation-like tensor with a negative floor
    yd = to_dev(y)
    ro = B.mmse_scale_search_offset(yd, B.params(*UNSIGNED, G, it))
    torch.cuda.synchronize()
    oo = oracle.can_offset_search(y, 15, G, it)
    assert float(ro.delta[0]) == oo["delta"] == -0.75
    check_equal(ro, np.array([oo["scale"]], np.float32), np.array([oo["idx"]], np.int32), np.array([oo["sse"]]),
                f"cfg{cfg} offset")
    np.testing.assert_array_equal(ro.packed.cpu().numpy(), oo["packed"])


@pytest.mark.parametrize("cfg", [4, 5])
def test_all_activation_tensors_of_a_network_batched(B, cfg):
    """Every calibration tensor of configurations 4 (54 tensors, 341 M elements) and 5 (16 tensors, 146 M
    elements, G = 512) through the batched entry point, in the launch configuration `bench.py --part whole`
    times, against the oracle tensor by tensor."""
    import torch
    c = synth.config(cfg)
    G, it = c.grid_points, c.refine_iters
    say(f"config {cfg}: {len(c.act_shapes)} activation tensors, batched")
    order = sorted(range(len(c.act_shapes)), key=lambda i: -c.act_shapes[i].per_image)
    dev = [to_dev(c.act_tensor(i)) for i in order]
    res = B.mmse_scale_search_activation_batched(dev, B.params(*UNSIGNED, G, it))
    torch.cuda.synchronize()
    got = [(float(r.scale[0]), int(r.idx[0]), float(r.sse[0])) for r in res]
    del dev
    for n_, i in enumerate(order):
        x = c.act_tensor(i)
        o = oracle.can_search(x, *UNSIGNED, G, it)
        assert got[n_] == (float(o["scale"]), o["idx"], o["sse"]), f"cfg{cfg} activation tensor {i} ({c.act_shapes[i].name})"
        np.testing.assert_array_equal(res[n_].packed.cpu().numpy(),
                                      oracle.can_quantize_pack_int4(x, [o["scale"]], *UNSIGNED),
                                      err_msg=f"cfg{cfg} activation codes {i}")
        res[n_].packed = None


def test_config5_weights_and_second_tensor_complete(B):
    """Every one of the 13 416 kernels of configuration 5 (138 M weights, G = 512), in the launch configuration
    `bench.py` times (batched, second tensor on all 16 layers): scales, indices, errors and all packed codes of
    the first search and of the second tensor against the oracle."""
    import torch
    c = synth.config(5)
    G, it = c.grid_points, c.refine_iters
    say("config 5: 16 weight tensors (138 M weights), batched, second tensor on all layers, complete comparison")
    ws = [c.weight_tensor(i) for i in range(len(c.weight_shapes))]
    dev = [to_dev(w) for w in ws]
    p = B.params(*SIGNED, G, it)
    res = B.mmse_scale_search_batched(dev, p, want_packed=True)
    res2 = B.mmse_scale_search_batched(dev, p, want_packed=True, scale1=[r.scale for r in res])
    torch.cuda.synchronize()
    for i, (w, r, r2) in enumerate(zip(ws, res, res2)):
        K, n = w.shape
        say(f"config 5: tensor {i} ({K} x {n})")
        s, j, e = oracle.can_search_kernelwise(w, *SIGNED, G, it)
        check_equal(r, s, j, e, f"cfg5 tensor {i}")
        np.testing.assert_array_equal(r.packed.cpu().numpy(), oracle.can_quantize_pack_int4(w, s, *SIGNED),
                                      err_msg=f"cfg5 tensor {i} codes")
        s2, j2, e2, p2 = oracle.can_residual_quantize(w, s, *SIGNED, G, it)
        check_equal(r2, s2, j2, e2, f"cfg5 second tensor {i}")
        np.testing.assert_array_equal(r2.packed.cpu().numpy(), p2, err_msg=f"cfg5 second tensor {i} codes")
        # properties that hold for every kernel at any size
        assert np.all(r2.sse.cpu().numpy() <= r.sse.cpu().numpy())
        assert np.all(np.isfinite(r.scale.cpu().numpy())) and np.all(r.idx.cpu().numpy() >= 0)
        assert np.all(r.idx.cpu().numpy() < G)
        assert r.packed.numel() == (K * n + 1) // 2
