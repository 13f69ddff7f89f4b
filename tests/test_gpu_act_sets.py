"""A call of few activation blocks sweeps every block with several sets of waves that take one aligned part of it
each (eight chunks at the least) and add their sums pairwise; the sums and their order are those of one set.  These
cases walk the grid sizes that give eight, four, two and one set, with ragged blocks whose last parts are short,
missing or empty, and compare every grid error, then scale, error and codes, with the oracle bit for bit; the same
tensors are also searched inside a call large enough to be swept with the fewest sets."""
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


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


SIZES = [1, 64 * 7 + 3, 64 * 8, 64 * 9 + 1, 64 * 16, 64 * 17 - 5, 64 * 33, 4096, 4096 + 64 * 8 + 1,
         4096 * 3 + 64 * 47 + 9, 4096 * 20]


@pytest.mark.parametrize("G", [64, 100, 128, 200, 256, 384, 512, 1024])
@pytest.mark.parametrize("q", [(0, 15), (-8, 7)])
def test_grid_errors_with_every_number_of_sets(B, G, q):
    for i, n in enumerate(SIZES):
        x = synth.acts_relu_normal(n, 900 + i) if q[0] == 0 else \
            np.random.default_rng(900 + i).normal(0, 1, n).astype(np.float32)
        say(f"sets: grid q={q} G={G} N={n}")
        absmax, grid = B.mmse_grid_sse_activation(dev(x), B.params(*q, G, 0))
        r = oracle.can_search(x, *q, G, 0, want_grid=True)
        np.testing.assert_array_equal(grid.cpu().numpy().reshape(-1), r["grid_sse"], err_msg=f"N={n}")


@pytest.mark.parametrize("G", [64, 128, 256, 512])
def test_small_and_large_calls_agree_with_the_oracle(B, G):
    xs = [synth.acts_relu_student_t(n, 40 + i) for i, n in enumerate(SIZES)]
    filler = synth.acts_relu_normal(4096 * 600, 7)                   # pushes the second call past the few-blocks limit
    say(f"sets: small call and large call G={G}")
    p = B.params(0, 15, G, 20)
    small = B.mmse_scale_search_activation_batched([dev(x) for x in xs], p, want_packed=True)
    large = B.mmse_scale_search_activation_batched([dev(x) for x in xs] + [dev(filler)], p, want_packed=True)
    for i, x in enumerate(xs):
        o = oracle.can_search(x, 0, 15, G, 20)
        codes = oracle.can_quantize_pack_int4(x, [o["scale"]], 0, 15)
        for name, got in (("small", small[i]), ("large", large[i])):
            assert int(got.idx[0]) == o["idx"], f"idx {name} {i}"
            np.testing.assert_array_equal(got.scale.cpu().numpy(), np.array([o["scale"]], np.float32), err_msg=f"scale {name} {i}")
            np.testing.assert_array_equal(got.sse.cpu().numpy(), np.array([o["sse"]]), err_msg=f"sse {name} {i}")
            np.testing.assert_array_equal(got.packed.cpu().numpy(), codes, err_msg=f"codes {name} {i}")
