"""Seeded random shapes, grids, ranges and distributions through the main entry points, GPU against
oracle bit for bit.  The fixed cases elsewhere are chosen by hand; these are not."""
import sys

import numpy as np
import pytest

import oracle
from paper_1902_06822_amd import synth

pytestmark = pytest.mark.gpu
RANGES = [(-8, 7), (0, 15), (-1, 1), (-2, 1), (0, 3), (-4, 3)]
KINDS = ["laplace", "normal", "outliers", "student"]


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


def random_weight_case(rng):
    n = int(rng.choice([rng.integers(1, 70), rng.integers(60, 700), rng.integers(600, 5000), rng.integers(8000, 9000)]))
    K = int(max(1, min(rng.integers(1, 400), 200000 // n)))
    G = int(rng.choice([1, 2, 37, 64, 65, 128, 256, 500, 512, 513, 1024, 2048]))
    iters = int(rng.choice([0, 1, 2, 3, 20, 33]))
    q = RANGES[int(rng.integers(len(RANGES)))]
    kind = KINDS[int(rng.integers(len(KINDS)))]
    return K, n, G, iters, q, kind


def run_weight_cases(B, seed, count):
    import torch
    rng = np.random.default_rng(seed)
    for c in range(count):
        K, n, G, iters, q, kind = random_weight_case(rng)
        w = synth.small_weights(K, n, int(rng.integers(1 << 30)), kind)
        if q[0] == 0:
            w = np.abs(w)
        tag = f"seed={seed} case={c} K={K} n={n} G={G} iters={iters} q={q} {kind}"
        say(tag)
        wd = dev(w)
        p = B.params(*q, G, iters)
        r = B.mmse_scale_search_batched([wd], p, want_packed=True)[0]
        r2 = B.mmse_scale_search_batched([wd], p, want_packed=True, scale1=[r.scale])[0]
        torch.cuda.synchronize()
        s, j, e = oracle.can_search_kernelwise(w, *q, G, iters)
        np.testing.assert_array_equal(r.idx.cpu().numpy(), j, err_msg=tag)
        np.testing.assert_array_equal(r.scale.cpu().numpy(), s, err_msg=tag)
        np.testing.assert_array_equal(r.sse.cpu().numpy(), e, err_msg=tag)
        np.testing.assert_array_equal(r.packed.cpu().numpy(), oracle.can_quantize_pack_int4(w, s, *q), err_msg=tag)
        s2, j2, e2, p2 = oracle.can_residual_quantize(w, s, *q, G, iters)
        np.testing.assert_array_equal(r2.idx.cpu().numpy(), j2, err_msg=tag)
        np.testing.assert_array_equal(r2.scale.cpu().numpy(), s2, err_msg=tag)
        np.testing.assert_array_equal(r2.sse.cpu().numpy(), e2, err_msg=tag)
        np.testing.assert_array_equal(r2.packed.cpu().numpy(), p2, err_msg=tag)


def run_activation_cases(B, seed, count):
    import torch
    rng = np.random.default_rng(seed)
    for c in range(count):
        sizes = [int(rng.choice([rng.integers(1, 5000), rng.integers(4000, 70000), rng.integers(60000, 600000)]))
                 for _ in range(int(rng.integers(1, 6)))]
        G = int(rng.choice([1, 50, 64, 128, 256, 500, 512, 1024]))
        iters = int(rng.choice([0, 1, 2, 5, 20, 21]))
        q = RANGES[int(rng.integers(len(RANGES)))]
        tag = f"seed={seed} case={c} sizes={sizes} G={G} iters={iters} q={q}"
        say(tag)
        xs = []
        for n in sizes:
            x = synth.acts_relu_student_t(n, int(rng.integers(1 << 30))) if rng.integers(2) else \
                synth.acts_relu_normal(n, int(rng.integers(1 << 30)))
            if q[0] < 0:
                x = (x - np.float32(0.6)).astype(np.float32)
            if rng.integers(3) == 0:                  # any share of zeros, in runs and scattered, also among signed data
                keep = float(rng.choice([0.02, 0.3, 0.9]))
                mask = rng.random(n) < keep
                if rng.integers(2):
                    mask &= (np.arange(n) // int(rng.integers(40, 9000))) % 2 == 0
                x = np.where(mask, x, np.float32(0.0)).astype(np.float32)
            xs.append(x)
        res = B.mmse_scale_search_activation_batched([dev(x) for x in xs], B.params(*q, G, iters))
        torch.cuda.synchronize()
        for x, r in zip(xs, res):
            o = oracle.can_search(x, *q, G, iters)
            assert (float(r.scale[0]), int(r.idx[0]), float(r.sse[0])) == (float(o["scale"]), o["idx"], o["sse"]), tag
            np.testing.assert_array_equal(r.packed.cpu().numpy(), oracle.can_quantize_pack_int4(x, [o["scale"]], *q),
                                          err_msg=tag)


def run_multi_tensor_case(B, seed):
    """Several random tensors in one batched call: tiny, short, ordinary and streaming kernels share the launches."""
    import torch
    rng = np.random.default_rng(seed)
    G = int(rng.choice([64, 128, 256, 500, 512, 1024]))
    iters = int(rng.choice([0, 3, 20]))
    q = RANGES[int(rng.integers(len(RANGES)))]
    ws = []
    for _ in range(int(rng.integers(2, 9))):
        n = int(rng.choice([rng.integers(1, 17), rng.integers(1, 70), rng.integers(60, 700), rng.integers(600, 5000),
                            rng.integers(8000, 12000)]))
        K = int(max(1, min(rng.integers(1, 3000), 400000 // n)))
        w = synth.small_weights(K, n, int(rng.integers(1 << 30)), KINDS[int(rng.integers(len(KINDS)))])
        ws.append(np.abs(w) if q[0] == 0 else w)
    tag = f"multi seed={seed} G={G} iters={iters} q={q} shapes={[w.shape for w in ws]}"
    say(tag)
    res = B.mmse_scale_search_batched([dev(w) for w in ws], B.params(*q, G, iters), want_packed=True)
    torch.cuda.synchronize()
    for w, r in zip(ws, res):
        s, j, e = oracle.can_search_kernelwise(w, *q, G, iters)
        np.testing.assert_array_equal(r.idx.cpu().numpy(), j, err_msg=tag)
        np.testing.assert_array_equal(r.scale.cpu().numpy(), s, err_msg=tag)
        np.testing.assert_array_equal(r.sse.cpu().numpy(), e, err_msg=tag)
        np.testing.assert_array_equal(r.packed.cpu().numpy(), oracle.can_quantize_pack_int4(w, s, *q), err_msg=tag)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_weight_cases(B, seed):
    run_weight_cases(B, seed, 14)


@pytest.mark.parametrize("seed", [21, 22])
def test_random_activation_cases(B, seed):
    run_activation_cases(B, seed, 10)


@pytest.mark.parametrize("seed", [31, 32, 33, 34])
def test_random_multi_tensor_calls(B, seed):
    run_multi_tensor_case(B, seed)
