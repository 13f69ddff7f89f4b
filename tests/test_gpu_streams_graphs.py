"""Stream and graph behaviour of the library on the GPU: everything is enqueued on the caller's
stream, nothing synchronises or allocates, so a call can run on a side stream and can be captured
into a HIP graph and replayed; results are identical to the eager ones every time."""
import sys

import numpy as np
import pytest

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


def snapshot(results):
    return [(r.scale.cpu().numpy().copy(), r.idx.cpu().numpy().copy(), r.sse.cpu().numpy().copy(),
             None if r.packed is None else r.packed.cpu().numpy().copy()) for r in results]


def assert_same(a, b):
    for x, y in zip(a, b):
        for u, v in zip(x, y):
            if u is None:
                assert v is None
            else:
                np.testing.assert_array_equal(u, v)


def test_side_stream_gives_the_same_results(B):
    import torch
    say("side stream")
    ws = [synth.small_weights(K, n, 40 + i, "laplace") for i, (K, n) in enumerate([(64, 576), (32, 147), (100, 9)])]
    dev = [torch.from_numpy(w).cuda() for w in ws]
    p = B.params(*SIGNED, 128, 20)
    plan = B.BatchedPlan(dev, p, want_packed=True)
    ref = snapshot(plan.run())
    side = torch.cuda.Stream()
    for r in plan.results:
        r.scale.zero_(); r.idx.zero_(); r.sse.zero_(); r.packed.zero_()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        plan.run()
    side.synchronize()
    assert_same(ref, snapshot(plan.results))


def test_graph_capture_and_replay_of_the_whole_weight_path(B):
    import torch
    say("graph replay: batched weights")
    c = synth.config(1)
    ws = [c.weight_tensor(0), synth.small_weights(48, 1152, 7, "student"), synth.small_weights(33, 27, 8, "normal")]
    dev = [torch.from_numpy(w).cuda() for w in ws]
    p = B.params(*SIGNED, 256, 20)
    plan = B.BatchedPlan(dev, p, want_packed=True)
    ref = snapshot(plan.run())
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        plan.run()                      # warm-up on the capture stream
    s.synchronize()
    with torch.cuda.graph(g, stream=s):
        plan.run()
    for rep in range(4):
        for r in plan.results:
            r.scale.fill_(-1.0); r.idx.fill_(-7); r.sse.fill_(-1.0); r.packed.fill_(0xAB)
        junk = torch.randn(1 << 20, device="cuda").sum()     # unrelated eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_same(ref, snapshot(plan.results))
        assert torch.isfinite(junk)


def test_graph_capture_and_replay_of_the_activation_path(B):
    import torch
    say("graph replay: activation search")
    x = synth.acts_relu_normal(300007, 99)
    xd = torch.from_numpy(x).cuda()
    p = B.params(*UNSIGNED, 128, 20)
    ws = B.alloc_workspace(B.mmse_workspace_bytes_activation(x.size, p))
    out = B.mmse_scale_search_activation(xd, p, ws)
    packed = B.quantize_pack_int4(xd, out.scale, *UNSIGNED)
    torch.cuda.synchronize()
    ref = (out.scale.item(), out.idx.item(), out.sse.item(), packed.cpu().numpy().copy())
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        B.mmse_scale_search_activation(xd, p, ws, out)
        B.quantize_pack_int4(xd, out.scale, *UNSIGNED, packed)
    s.synchronize()
    with torch.cuda.graph(g, stream=s):
        B.mmse_scale_search_activation(xd, p, ws, out)
        B.quantize_pack_int4(xd, out.scale, *UNSIGNED, packed)
    for rep in range(4):
        out.scale.fill_(-1.0); out.idx.fill_(-7); out.sse.fill_(-1.0); packed.fill_(0xAB)
        ws.fill_(0xCD)                  # the workspace holds nothing a call relies on
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert (out.scale.item(), out.idx.item(), out.sse.item()) == ref[:3]
        np.testing.assert_array_equal(packed.cpu().numpy(), ref[3])


def test_graph_capture_and_replay_of_the_later_entry_points(B):
    """Dual line search, the activation variants and the alternating comparison mode under capture: every
    replay, with the outputs and the workspaces scribbled over in between, gives the eager result."""
    import torch
    say("graph replay: dual line search, activation variants, alternating mode")
    w = torch.from_numpy(synth.small_weights(70, 147, 5, "laplace")).cuda()
    x = torch.from_numpy(synth.acts_relu_normal(123457, 98) - np.float32(0.5)).cuda()
    pu, ps = B.params(*UNSIGNED, 64, 10), B.params(*SIGNED, 64, 10)
    ws_d = B.alloc_workspace(B.mmse_workspace_bytes_dual_linesearch(70, 147, 16, 20))
    ws_a = B.alloc_workspace(B.mmse_workspace_bytes_activation(x.numel(), pu))
    ws_b = B.alloc_workspace(B.mmse_workspace_bytes_activation(x.numel(), pu))
    ws_c = B.alloc_workspace(B.mmse_workspace_bytes_activation(x.numel(), pu))
    d = B.dual_line_search(w, *SIGNED, 16, 20, ws=ws_d)
    first = B.mmse_scale_search_activation(x, pu, ws_a)
    second = B.activation_residual_quantize(x, first.scale, *UNSIGNED, ps, ws_b)
    off = B.mmse_scale_search_offset(x, pu, ws_c)
    torch.cuda.synchronize()
    alt = B.mmse_scale_alternating_kernelwise(w, *SIGNED, 20)
    torch.cuda.synchronize()
    outs = [d.scale1, d.scale2, d.idx1, d.idx2, d.sse, d.packed1, d.packed2, first.scale, second.scale, second.idx,
            second.sse, second.packed, off.delta, off.scale, off.idx, off.sse, off.packed]
    ref = [t.cpu().numpy().copy() for t in outs]
    ref_alt = [t.cpu().numpy().copy() for t in alt]

    def work():
        B.dual_line_search(w, *SIGNED, 16, 20, ws=ws_d, out=d)
        B.mmse_scale_search_activation(x, pu, ws_a, first)
        B.activation_residual_quantize(x, first.scale, *UNSIGNED, ps, ws_b, second)
        B.mmse_scale_search_offset(x, pu, ws_c, off)

    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        work()
    s.synchronize()
    with torch.cuda.graph(g, stream=s):
        work()
    for rep in range(3):
        for t in outs:
            t.fill_(3)
        for t in (ws_d, ws_a, ws_b, ws_c):
            t.fill_(0xCD)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for t, r in zip(outs, ref):
            np.testing.assert_array_equal(t.cpu().numpy(), r)
        again = B.mmse_scale_alternating_kernelwise(w, *SIGNED, 20)
        torch.cuda.synchronize()
        for t, r in zip(again, ref_alt):
            np.testing.assert_array_equal(t.cpu().numpy(), r)
