"""GPU parity of the activation variants against the oracle: the second tensor from the residual
(Section 3.7, Eq. 16) and the offset form (Section 3.1, Eq. 2), bit for bit."""
import sys

import numpy as np
import pytest

import oracle
from paper_1902_06822_amd import synth

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


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def same(got, ref, name):
    g = got.cpu().numpy()
    np.testing.assert_array_equal(g, np.asarray(ref, g.dtype).reshape(g.shape), err_msg=name)


def check_residual(B, x, q1, q2, G, iters, tag):
    import torch
    xd = dev(x)
    first = B.mmse_scale_search_activation(xd, B.params(*q1, G, iters))
    r = B.activation_residual_quantize(xd, first.scale, *q1, B.params(*q2, G, iters))
    torch.cuda.synchronize()
    o1 = oracle.can_search(x, *q1, G, iters)
    same(first.scale, [o1["scale"]], f"first scale {tag}")
    o = oracle.can_act_residual_quantize(x, o1["scale"], q1, q2, G, iters)
    same(r.idx, [o["idx"]], f"idx {tag}")
    np.testing.assert_allclose(r.scale.cpu().numpy(), [o["scale"]], rtol=1e-6, atol=0, err_msg=f"scale {tag}")
    np.testing.assert_allclose(r.sse.cpu().numpy(), [o["sse"]], rtol=1e-4, atol=0, err_msg=f"sse {tag}")
    same(r.scale, [o["scale"]], f"scale bits {tag}")
    same(r.sse, [o["sse"]], f"sse bits {tag}")
    same(r.packed, o["packed"], f"codes {tag}")
    return r, o, o1


@pytest.mark.parametrize("N", [1, 63, 4096, 4097, 100001, 1000003])
@pytest.mark.parametrize("q2", [SIGNED, UNSIGNED])
def test_activation_residual_matches_oracle(B, N, q2):
    say(f"activation residual N={N} second range {q2}")
    x = synth.acts_relu_normal(N, 40 + N % 97)
    check_residual(B, x, UNSIGNED, q2, 128, 20, f"N={N}")


@pytest.mark.parametrize("G,iters", [(512, 0), (1024, 7), (37, 64)])
def test_activation_residual_grids_and_heavy_tails(B, G, iters):
    say(f"activation residual student-t G={G} iters={iters}")
    x = synth.acts_relu_student_t(300000, 5)
    r, o, o1 = check_residual(B, x, UNSIGNED, SIGNED, G, iters, f"G={G}")
    assert float(r.sse[0]) < o1["sse"]


def test_activation_residual_signed_first_tensor(B):
    say("activation residual: signed first tensor (network input)")
    x = np.random.default_rng(6).normal(0, 1, 70001).astype(np.float32)
    check_residual(B, x, SIGNED, SIGNED, 256, 20, "signed input")


def test_activation_residual_degenerate(B):
    import torch
    say("activation residual: exact first tensor, NaN first scale, non-finite input")
    x = (np.float32(0.375) * np.random.default_rng(2).integers(0, 16, 5000)).astype(np.float32)
    p = B.params(*SIGNED, 32, 5)
    s1 = dev(np.array([0.375], np.float32))
    r = B.activation_residual_quantize(dev(x), s1, *UNSIGNED, p)
    torch.cuda.synchronize()
    o = oracle.can_act_residual_quantize(x, 0.375, UNSIGNED, SIGNED, 32, 5)
    assert (float(r.scale[0]), int(r.idx[0]), float(r.sse[0])) == (o["scale"], o["idx"], o["sse"]) == (1.0, 0, 0.0)
    same(r.packed, o["packed"], "codes")
    r = B.activation_residual_quantize(dev(x), dev(np.array([np.nan], np.float32)), *UNSIGNED, p)
    torch.cuda.synchronize()
    assert np.isnan(float(r.scale[0])) and int(r.idx[0]) == -1 and np.isnan(float(r.sse[0]))
    assert not r.packed.cpu().numpy().any()
    x[77] = np.inf
    r = B.activation_residual_quantize(dev(x), s1, *UNSIGNED, p)
    torch.cuda.synchronize()
    o = oracle.can_act_residual_quantize(x, 0.375, UNSIGNED, SIGNED, 32, 5)
    assert o["rc"] == -1 and np.isnan(float(r.scale[0])) and int(r.idx[0]) == -1
    same(r.packed, o["packed"], "codes of a rejected tensor")


def check_offset(B, x, qmax, G, iters, tag):
    import torch
    r = B.mmse_scale_search_offset(dev(x), B.params(0, qmax, G, iters))
    torch.cuda.synchronize()
    o = oracle.can_offset_search(x, qmax, G, iters)
    same(r.idx, [o["idx"]], f"idx {tag}")
    same(r.delta, [o["delta"]], f"delta {tag}")
    np.testing.assert_allclose(r.scale.cpu().numpy(), [o["scale"]], rtol=1e-6, atol=0, err_msg=f"scale {tag}")
    np.testing.assert_allclose(r.sse.cpu().numpy(), [o["sse"]], rtol=1e-4, atol=0, err_msg=f"sse {tag}")
    same(r.scale, [o["scale"]], f"scale bits {tag}")
    same(r.sse, [o["sse"]], f"sse bits {tag}")
    same(r.packed, o["packed"], f"codes {tag}")
    return r, o


@pytest.mark.parametrize("N", [1, 2, 65, 4095, 8193, 250007, 2000001])
def test_offset_search_matches_oracle(B, N):
    say(f"offset form N={N}")
    x = np.random.default_rng(N).normal(1.5, 1.0, N).astype(np.float32)
    check_offset(B, x, 15, 128, 20, f"N={N}")


@pytest.mark.parametrize("G,iters,qmax", [(512, 0, 15), (2048, 3, 15), (50, 20, 3), (16, 64, 1)])
def test_offset_search_grids_ranges_and_distributions(B, G, iters, qmax):
    say(f"offset form G={G} iters={iters} qmax={qmax}")
    x = (-synth.acts_relu_student_t(150001, 3) + np.float32(0.25)).astype(np.float32)    # long negative tail
    check_offset(B, x, qmax, G, iters, f"G={G}")
    check_offset(B, synth.acts_relu_normal(150001, 3), qmax, G, iters, f"relu G={G}")   # delta = 0


def test_offset_search_degenerate(B):
    say("offset form: constant, signed zeros, NaN, infinities, too wide a range")
    c = np.full(10000, 2.5, np.float32)
    r, o = check_offset(B, c, 15, 16, 4, "constant")
    assert float(r.delta[0]) == 2.5 and float(r.scale[0]) == 1.0 and float(r.sse[0]) == 0.0
    z = np.zeros(5000, np.float32)
    z[::2] = -0.0
    z[17] = 3.0
    check_offset(B, z, 15, 16, 4, "signed zeros")
    for bad, where in ((np.nan, 7), (-np.nan, 4099), (np.inf, 0), (-np.inf, 9999)):
        c2 = c.copy()
        c2[where] = bad
        r, o = check_offset(B, c2, 15, 16, 4, f"{bad}")
        assert np.isnan(float(r.delta[0])) and np.isnan(float(r.scale[0])) and int(r.idx[0]) == -1
    wide = np.array([2.0 ** 61, 0.0, 1.0] * 100, np.float32)
    r, o = check_offset(B, wide, 15, 16, 4, "wide")
    assert np.isnan(float(r.delta[0]))


def test_offset_search_rejects_signed_range(B):
    x = dev(np.ones(16, np.float32))
    with pytest.raises(RuntimeError):
        B.mmse_scale_search_offset(x, B.params(-8, 7, 16, 4))
    with pytest.raises(RuntimeError):
        B.activation_residual_quantize(x, x[:1], 1, 7, B.params(-8, 7, 16, 4))
