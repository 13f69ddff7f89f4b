"""GPU parity at the largest sizes the C ABI accepts (MMSE_MAX_TENSOR_ELEMS elements in one activation
tensor; K * n just below it with the longest kernel, MMSE_MAX_KERNEL_ELEMS): every index past 2^31 bytes and
every block number near 2^19 is exercised.  Scales, indices and errors are compared completely; the codes on
windows at the start, around the middle and at the ragged end (a window is coded exactly as in a full run)."""
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


def test_activation_tensor_of_maximum_size(B):
    import torch
    N = 2 ** 31 - 1
    G, iters = 32, 2
    say(f"activation tensor of {N} elements, G={G}, {iters} refinement iterations")
    x = synth.tiled_normal(N, 190206822 + 9001, relu=True)
    x[N - 3] = np.float32(9.5)                       # the abs-max sits in the last, partial block
    xd = torch.from_numpy(x).cuda()
    p = B.params(0, 15, G, iters)
    r = B.mmse_scale_search_activation(xd, p)
    packed = B.quantize_pack_int4(xd, r.scale, 0, 15)
    torch.cuda.synchronize()
    say("oracle")
    o = oracle.can_search(x, 0, 15, G, iters)
    assert int(r.idx.cpu()[0]) == o["idx"]
    assert float(r.scale.cpu()[0]) == float(o["scale"])
    assert float(r.sse.cpu()[0]) == o["sse"]
    assert packed.numel() == (N + 1) // 2
    s = np.array([o["scale"]], np.float32)
    for start, length in ((0, 70000), (2 ** 30 - 5000, 10000), (2 ** 31 - 2 ** 24 - 2, 12346), (N - 65537, 65537)):
        assert start % 2 == 0
        ref = oracle.can_quantize_pack_int4(x[start:start + length].reshape(1, -1), s, 0, 15)
        got = packed[start // 2:start // 2 + ref.size].cpu().numpy()
        np.testing.assert_array_equal(got, ref, err_msg=f"codes from element {start}")
    del xd, packed
    torch.cuda.empty_cache()


def test_weight_tensor_of_maximum_size(B):
    import torch
    K, n = 32767, 65536                              # K * n = 2 147 418 112, the longest kernel the ABI takes
    G, iters = 16, 1
    say(f"weight tensor {K} x {n}, G={G}, {iters} refinement iteration")
    w = synth.tiled_normal(K * n, 190206822 + 9002).reshape(K, n)
    w *= np.float32(0.05)
    wd = torch.from_numpy(w).cuda()
    p = B.params(-8, 7, G, iters)
    res = B.mmse_scale_search_batched([wd], p, want_packed=True)[0]
    torch.cuda.synchronize()
    say("oracle")
    s, j, e = oracle.can_search_kernelwise(w, -8, 7, G, iters)
    np.testing.assert_array_equal(res.idx.cpu().numpy(), j)
    np.testing.assert_array_equal(res.scale.cpu().numpy(), s)
    np.testing.assert_array_equal(res.sse.cpu().numpy(), e)
    assert res.packed.numel() == K * n // 2
    for k0 in (0, K // 2, 16384, K - 2):             # row 16384 starts at byte 2^29, element 2^30
        ref = oracle.can_quantize_pack_int4(w[k0:k0 + 2], s[k0:k0 + 2], -8, 7)
        got = res.packed[k0 * n // 2:(k0 + 2) * n // 2].cpu().numpy()
        np.testing.assert_array_equal(got, ref, err_msg=f"codes of kernels {k0}, {k0 + 1}")
    del wd, res
    torch.cuda.empty_cache()


def test_batched_calls_with_the_most_tensors(B):
    """4096 weight tensors and 1024 activation tensors in one call each: the largest descriptor tables
    (103 and 16 launch groups)."""
    import torch
    say("batched weights: 4096 tensors")
    rng = np.random.default_rng(190206822 + 9003)
    ws = []
    for i in range(4096):
        K, n = int(rng.integers(1, 4)), int(rng.choice([1, 9, 27, 64, 65, 130, 576]))
        ws.append(synth.small_weights(K, n, 40000 + i, ("laplace", "normal", "student", "outliers")[i % 4]))
    p = B.params(-8, 7, 40, 6)
    res = B.mmse_scale_search_batched([torch.from_numpy(w).cuda() for w in ws], p, want_packed=True)
    torch.cuda.synchronize()
    for i, (w, r) in enumerate(zip(ws, res)):
        s, j, e = oracle.can_search_kernelwise(w, -8, 7, 40, 6)
        np.testing.assert_array_equal(r.idx.cpu().numpy(), j, err_msg=f"idx of tensor {i}")
        np.testing.assert_array_equal(r.scale.cpu().numpy(), s, err_msg=f"scale of tensor {i}")
        np.testing.assert_array_equal(r.sse.cpu().numpy(), e, err_msg=f"sse of tensor {i}")
        np.testing.assert_array_equal(r.packed.cpu().numpy(), oracle.can_quantize_pack_int4(w, s, -8, 7),
                                      err_msg=f"codes of tensor {i}")
    say("batched activations: 1024 tensors")
    xs = [synth.acts_relu_normal(int(rng.integers(1, 9000)), 50000 + i) for i in range(1024)]
    pa = B.params(0, 15, 48, 5)
    res = B.mmse_scale_search_activation_batched([torch.from_numpy(x).cuda() for x in xs], pa)
    torch.cuda.synchronize()
    for i, (x, r) in enumerate(zip(xs, res)):
        o = oracle.can_search(x, 0, 15, 48, 5)
        assert int(r.idx.cpu()[0]) == o["idx"] and float(r.scale.cpu()[0]) == float(o["scale"]), i
        assert float(r.sse.cpu()[0]) == o["sse"], i
        np.testing.assert_array_equal(r.packed.cpu().numpy(),
                                      oracle.can_quantize_pack_int4(x, np.array([o["scale"]], np.float32), 0, 15),
                                      err_msg=f"codes of activation tensor {i}")


def test_batched_activations_with_more_than_65535_block_groups(B):
    """64 tensors of about 65 536 blocks each in one launch group: 4.2 M blocks (the most one group takes),
    65 536 rows after the first tree stage (more than a grid's y axis holds).  Then the same with one tensor
    two blocks longer, which no longer fits the group and is searched by a second set of launches.  The
    tensors are views of one buffer with five different lengths, so the oracle has five problems to solve."""
    import torch
    base_n = 2 ** 28
    say(f"64 activation tensors of about {base_n} elements in one batched call")
    x = synth.tiled_normal(base_n + 8192, 190206822 + 9004, relu=True)
    lengths = [base_n, base_n - 1, base_n - 4097, base_n - 60000]
    assert sum(((n + 4095) // 4096 + 63) // 64 for n in lengths) * 16 == 65536      # rows after one tree stage
    xd = torch.from_numpy(x).cuda()
    G, iters = 4, 1
    p = B.params(0, 15, G, iters)
    res = B.mmse_scale_search_activation_batched([xd[:lengths[i % 4]] for i in range(64)], p, want_packed=False)
    torch.cuda.synchronize()
    say("oracle")
    ref = [oracle.can_search(x[:n], 0, 15, G, iters) for n in lengths]

    def same(r, o, tag):
        assert int(r.idx.cpu()[0]) == o["idx"], tag
        assert float(r.scale.cpu()[0]) == float(o["scale"]), tag
        assert float(r.sse.cpu()[0]) == o["sse"], tag

    for i, r in enumerate(res):
        same(r, ref[i % 4], i)
    say("one tensor longer: two launch groups")
    sizes = [base_n + 8192] + [base_n] * 63
    assert sum((n + 4095) // 4096 for n in sizes) == 2 ** 22 + 2
    res = B.mmse_scale_search_activation_batched([xd[:n] for n in sizes], p, want_packed=False)
    torch.cuda.synchronize()
    same(res[0], oracle.can_search(x, 0, 15, G, iters), "longer tensor")
    for i in range(1, 64):
        same(res[i], ref[0], i)
    del xd, res
    torch.cuda.empty_cache()


def check_sampled_kernels(w, r, qr, G, iters, seed, tag):
    """Oracle on a sample of whole kernels (the ends, the middle, random ones): kernels are independent
    problems, so a sampled kernel is checked exactly as in a complete run."""
    K, n = w.shape
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([np.arange(0, 2000), np.arange(K // 2 - 1000, K // 2 + 1000),
                                     np.arange(K - 2000, K), rng.integers(0, K, 20000)]))
    s, j, e = oracle.can_search_kernelwise(w[rows], *qr, G, iters)
    np.testing.assert_array_equal(r.idx.cpu().numpy()[rows], j, err_msg=f"idx {tag}")
    np.testing.assert_array_equal(r.scale.cpu().numpy()[rows], s, err_msg=f"scale {tag}")
    np.testing.assert_array_equal(r.sse.cpu().numpy()[rows], e, err_msg=f"sse {tag}")
    codes = oracle.can_codes(w[rows], s, *qr)
    flat = (rows[:, None].astype(np.int64) * n + np.arange(n)[None, :]).ravel()
    packed = r.packed.cpu().numpy()
    got = ((packed[flat // 2] >> ((flat % 2) * 4)) & 0xF).astype(np.int32)
    got = np.where(got >= 8, got - 16, got) if qr[0] < 0 else got
    np.testing.assert_array_equal(got, codes.ravel(), err_msg=f"codes {tag}")


def test_weight_launches_are_cut_at_the_work_item_limit(B):
    """Tensors with the most kernels the ABI takes (2^22 each): a launch holds one of them on the
    general path (one workgroup per kernel) and four on the short-kernel path (four kernels per workgroup)."""
    import torch
    K = 2 ** 22
    say("short-kernel path: five tensors of 2^22 one-element kernels")
    ws = [synth.tiled_normal(K, 190206822 + 9010 + i).reshape(K, 1) for i in range(5)]
    p = B.params(-8, 7, 40, 2)
    res = B.mmse_scale_search_batched([torch.from_numpy(w).cuda() for w in ws], p, want_packed=True)
    torch.cuda.synchronize()
    for i, (w, r) in enumerate(zip(ws, res)):
        check_sampled_kernels(w, r, (-8, 7), 40, 2, 70 + i, f"short kernels, tensor {i}")
    say("general path: two tensors of 2^22 two-element kernels, G = 520")
    ws = [synth.tiled_normal(2 * K, 190206822 + 9020 + i).reshape(K, 2) for i in range(2)]
    p = B.params(-8, 7, 520, 0)
    res = B.mmse_scale_search_batched([torch.from_numpy(w).cuda() for w in ws], p, want_packed=True)
    torch.cuda.synchronize()
    for i, (w, r) in enumerate(zip(ws, res)):
        check_sampled_kernels(w, r, (-8, 7), 520, 0, 80 + i, f"general path, tensor {i}")


def test_dual_alternating_over_more_than_2_31_weights_in_one_call(B):
    """Three layers of 10 923 kernels of 65 536 weights through the batched Algorithm 1: together just over
    2^31 weights in one call (tentative and kept codes of 1 GB each).  Sampled kernels are compared with the
    oracle; every kernel must report a sweep count in range."""
    import torch
    K, n = 10923, 65536
    assert 3 * K * n > 2 ** 31
    say(f"Algorithm 1, three layers of {K} x {n}")
    G, iters, eps, max_sweeps = 32, 4, 0.0, 3
    p = B.params(-8, 7, G, iters)
    ws = [synth.tiled_normal(K * n, 190206822 + 9030 + i).reshape(K, n) for i in range(3)]
    res = B.dual_quantize_alternating_batched([torch.from_numpy(w).cuda() for w in ws], p, eps, max_sweeps)
    torch.cuda.synchronize()
    say("oracle on sampled kernels")
    rows = np.array([0, 1, 4095, 4096, K // 2, K - 2, K - 1])
    for i, (w, r) in enumerate(zip(ws, res)):
        o = oracle.can_dual_alternating(np.ascontiguousarray(w[rows]), -8, 7, G, iters, eps, max_sweeps)
        sw = r.sweeps.cpu().numpy()
        assert sw.min() >= 1 and sw.max() <= max_sweeps
        np.testing.assert_array_equal(sw[rows], o["sweeps"], err_msg=f"sweeps {i}")
        np.testing.assert_array_equal(r.scale1.cpu().numpy()[rows], o["scale1"], err_msg=f"scale1 {i}")
        np.testing.assert_array_equal(r.scale2.cpu().numpy()[rows], o["scale2"], err_msg=f"scale2 {i}")
        np.testing.assert_array_equal(r.sse.cpu().numpy()[rows], o["sse"], err_msg=f"sse {i}")
        for name in ("packed1", "packed2"):
            got = torch.stack([getattr(r, name)[k * (n // 2):(k + 1) * (n // 2)] for k in rows]).cpu().numpy().ravel()
            np.testing.assert_array_equal(got, o[name], err_msg=f"{name} {i}")
    del res
    torch.cuda.empty_cache()
