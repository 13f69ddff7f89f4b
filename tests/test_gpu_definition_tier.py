"""The errors the GPU returns against the plain definition of the objective (Section 3.4, Eq. 7-8):
f(alpha) = sum_i (T_i - alpha*[T_i/alpha])^2 evaluated in fp64 with a true division (the oracle's
definition tier, which knows nothing of chunks, trees or reciprocals), at the scale the GPU returned,
for every kernel and every activation tensor of the five configurations.  Bar: 1e-4 relative."""
import sys

import numpy as np
import pytest

import oracle
from paper_1902_06822_amd import select, synth

pytestmark = pytest.mark.gpu
SIGNED = (-8, 7)
UNSIGNED = (0, 15)
RTOL = 1e-4


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


def check_rows(w, scale, sse, rng, tag):
    """|sse_gpu - f_def(w_k, scale_k)| <= RTOL * f_def for every row k."""
    K = w.shape[0]
    ref = np.array([oracle.def_sse(w[k], float(scale[k]), *rng) for k in range(K)])
    bad = np.abs(sse - ref) > RTOL * ref
    assert not bad.any(), (tag, int(bad.sum()), np.flatnonzero(bad)[:5], sse[bad][:5], ref[bad][:5])


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_returned_errors_match_the_definition(B, cfg):
    import torch
    c = synth.config(cfg)
    G, it = c.grid_points, c.refine_iters
    say(f"config {cfg}: definition-tier check of every returned error")
    ws = [c.weight_tensor(i) for i in range(len(c.weight_shapes))]
    dev = [to_dev(w) for w in ws]
    p = B.params(*SIGNED, G, it)
    res = B.mmse_scale_search_batched(dev, p, want_packed=False)
    torch.cuda.synchronize()
    for i, (w, r) in enumerate(zip(ws, res)):
        check_rows(w, r.scale.cpu().numpy(), r.sse.cpu().numpy(), SIGNED, f"cfg{cfg} tensor {i}")
    # second tensor (Section 3.5): on every layer (configuration 5) or on the selected ones (configuration 4)
    key = []
    if c.residual == "all":
        key = list(range(len(ws)))
    elif c.residual == "top10pct":
        energy = [float(np.sum(w.astype(np.float64) ** 2)) for w in ws]
        sums = B.mmse_layer_error_sums([r.sse for r in res]).cpu().numpy()
        key = select.select_top_fraction(select.normalized_mse(list(sums), energy), 0.10)
    if key:
        res2 = B.mmse_scale_search_batched([dev[i] for i in key], p, want_packed=False,
                                           scale1=[res[i].scale for i in key])
        torch.cuda.synchronize()
        for i, r2 in zip(key, res2):
            # what the first tensor leaves (one fused multiply-add per element, as the method forms it), then the
            # plain definition on it
            R = oracle.can_residual(ws[i], res[i].scale.cpu().numpy(), *SIGNED)
            check_rows(R, r2.scale.cpu().numpy(), r2.sse.cpu().numpy(), SIGNED, f"cfg{cfg} second tensor {i}")
    del dev, res
    if not c.act_shapes:
        return
    order = sorted(range(len(c.act_shapes)), key=lambda i: -c.act_shapes[i].per_image)
    xs = [to_dev(c.act_tensor(i)) for i in order]
    ra = B.mmse_scale_search_activation_batched(xs, B.params(*UNSIGNED, G, it), want_packed=False)
    torch.cuda.synchronize()
    got = [(float(r.scale[0]), float(r.sse[0])) for r in ra]
    del xs
    for n_, i in enumerate(order):
        x = c.act_tensor(i)
        ref = oracle.def_sse(x, got[n_][0], *UNSIGNED)
        assert abs(got[n_][1] - ref) <= RTOL * ref, (f"cfg{cfg} activation {c.act_shapes[i].name}", got[n_], ref)
