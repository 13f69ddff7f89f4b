"""CPU-side checks of the C ABI: the library loads, exports what include/mmse.h declares,
and rejects bad arguments before touching the GPU (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_1902_06822_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_1902_06822_amd import build
        build.build()
    binding.load_library()
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mmse.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*\s*|int\s+|void\s+)(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_symbols_are_exported(B):
    names = declared_functions()
    assert set(names) == set(B.EXPORTS) | set(B.VOID_EXPORTS), (names, B.EXPORTS)
    lib = B.load_library()
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layouts_match_header(B):
    assert C.sizeof(B.MmseParams) == 20
    assert C.sizeof(B.MmseTensorDesc) == 64
    assert B.MmseTensorDesc.K.offset == 8 and B.MmseTensorDesc.packed_dev.offset == 56
    assert C.sizeof(B.MmseDualDesc) == 72 and B.MmseDualDesc.sweeps_dev.offset == 64
    assert C.sizeof(B.MmseActDesc) == 48 and B.MmseActDesc.N.offset == 8 and B.MmseActDesc.packed_dev.offset == 40


def test_status_strings(B):
    assert B.status_string(0) == "ok"
    for rc in range(-7, 0):
        assert B.status_string(rc) not in ("ok", "unknown status")
    assert B.status_string(-99) == "unknown status"


def test_workspace_queries(B):
    p = B.params(-8, 7, 256, 20)
    assert B.mmse_workspace_bytes_kernelwise(5800, 576, p) == 23296          # 5800 floats, rounded to 256
    n0 = B.mmse_workspace_bytes_activation(4096, B.params(-8, 7, 256, 0))
    n1 = B.mmse_workspace_bytes_activation(4096, p)
    n2 = B.mmse_workspace_bytes_activation(51380224, B.params(0, 15, 512, 20))
    assert 256 < n0 < 16384
    assert n1 == n0 + 4096 * 4 + 256          # with a refinement: the block's compacted copy and its 64 chunk words
    assert n2 > 12544 * 512 * 8 + 12544 * (4096 * 4 + 256)
    with pytest.raises(RuntimeError):
        B.mmse_workspace_bytes_kernelwise(0, 5, p)
    with pytest.raises(RuntimeError):
        B.mmse_workspace_bytes_activation(-1, p)


@pytest.mark.parametrize("bad", [dict(qmin=1), dict(qmax=0), dict(qmin=-9, qmax=7), dict(grid_points=0),
                                 dict(grid_points=2049), dict(refine_iters=-1), dict(refine_iters=65),
                                 dict(cands_per_lane=3), dict(grid_points=1024, cands_per_lane=1)])
def test_bad_parameters_are_rejected(B, bad):
    kw = dict(qmin=-8, qmax=7, grid_points=256, refine_iters=20, cands_per_lane=0)
    kw.update(bad)
    p = B.params(**kw)
    out = C.c_size_t(0)
    assert B.load_library().mmse_workspace_bytes_kernelwise(8, 8, C.byref(p), C.byref(out)) == -3


def test_entry_points_validate_before_enqueue(B):
    """Fake (never dereferenced) addresses: every call must fail in validation, on the host."""
    lib = B.load_library()
    p = B.params(-8, 7, 256, 20)
    a = 0x10000            # 64 KiB: aligned to everything, never touched
    # NULL pointers
    assert lib.mmse_scale_search_kernelwise(None, 4, 4, C.byref(p), a, a, a, a, 4096, None) == -1
    assert lib.mmse_scale_search_kernelwise(a, 4, 4, C.byref(p), None, a, a, a, 4096, None) == -1
    assert lib.mmse_scale_search_kernelwise(a, 4, 4, None, a, a, a, a, 4096, None) == -1
    assert lib.mmse_scale_search_activation(None, 4, C.byref(p), a, a, a, a, 1 << 20, None) == -1
    assert lib.quantize_pack_int4(a, 4, 4, None, -8, 7, a, None) == -1
    assert lib.residual_quantize(a, 4, 4, None, C.byref(p), a, a, a, a, a, 4096, None) == -1
    assert lib.mmse_scale_search_batched(None, 1, C.byref(p), a, 4096, None) == -1
    assert lib.mmse_grid_sse_kernelwise(a, 4, 4, C.byref(p), None, a, None) == -1
    assert lib.mmse_scale_search_kernelwise(a, (1 << 22) + 1, 4, C.byref(p), a, a, a, a, 1 << 30, None) == -2   # more kernels than a launch holds
    assert lib.mmse_scale_alternating_kernelwise(a, (1 << 22) + 1, 4, -8, 7, 10, a, a, a, None) == -2
    big = (B.MmseTensorDesc * 2)(B.MmseTensorDesc(a, 4, 4, None, a, a, a, None), B.MmseTensorDesc(a, (1 << 22) + 1, 1, None, a, a, a, None))
    assert lib.mmse_scale_search_batched(big, 2, C.byref(p), a, 1 << 40, None) == -2          # second tensor: too many kernels
    bigd = (B.MmseDualDesc * 2)(B.MmseDualDesc(a, 4, 4, a, a, a, a, a, a), B.MmseDualDesc(a, (1 << 22) + 1, 1, a, a, a, a, a, a))
    assert lib.dual_quantize_alternating_batched(bigd, 2, C.byref(p), 1e-3, 4, a, 1 << 44, None) == -2
    assert lib.dual_quantize_alternating(a, 4, 4, C.byref(p), 1e-3, 4, a, a, None, a, a, a, a, 1 << 20, None) == -1
    assert lib.dual_quantize_alternating(a, 4, 4, C.byref(p), -1.0, 4, a, a, a, a, a, a, a, 1 << 20, None) == -3
    assert lib.dual_quantize_alternating(a, 4, 4, C.byref(p), 1e-3, 0, a, a, a, a, a, a, a, 1 << 20, None) == -3
    assert lib.dual_quantize_alternating(a, 4, 4, C.byref(p), 1e-3, 4, a, a, a, a, a, a, a, 256, None) == -4
    assert lib.dual_quantize_alternating_batched(None, 1, C.byref(p), 1e-3, 4, a, 1 << 20, None) == -1
    dls = lambda **kw: lib.dual_line_search(*[kw.get(k, d) for k, d in (
        ("w", a), ("K", 4), ("n", 4), ("qmin", -8), ("qmax", 7), ("G1", 8), ("G2", 8), ("s1", a), ("s2", a), ("i1", a),
        ("i2", a), ("sse", a), ("p1", a), ("p2", a), ("grid", None), ("ws", a), ("ws_bytes", 1 << 20), ("stream", None))])
    assert dls(w=None) == -1 and dls(p2=None) == -1 and dls(sse=None) == -1
    assert dls(n=8193) == -2 and dls(K=0) == -2
    assert dls(G1=0) == -3 and dls(G2=1025) == -3 and dls(qmin=1) == -3 and dls(qmin=-9) == -3
    assert dls(ws=None) == -4 and dls(ws_bytes=16) == -4 and dls(ws=a + 8) == -4
    assert dls(sse=a + 4) == -6 and dls(grid=a + 4) == -6
    pu = B.params(0, 15, 256, 20)
    assert lib.activation_residual_quantize(a, 64, None, 0, 15, C.byref(p), a, a, a, a, a, 1 << 20, None) == -1
    assert lib.activation_residual_quantize(a, 64, a, 1, 15, C.byref(p), a, a, a, a, a, 1 << 20, None) == -3
    assert lib.activation_residual_quantize(a, 64, a, 0, 16, C.byref(p), a, a, a, a, a, 1 << 20, None) == -3
    assert lib.activation_residual_quantize(a, 0, a, 0, 15, C.byref(p), a, a, a, a, a, 1 << 20, None) == -2
    assert lib.activation_residual_quantize(a, 64, a, 0, 15, C.byref(p), a, a, a, a, a, 16, None) == -4
    assert lib.mmse_scale_search_offset(a, 64, C.byref(pu), None, a, a, a, a, a, 1 << 20, None) == -1
    assert lib.mmse_scale_search_offset(a, 64, C.byref(p), a, a, a, a, a, a, 1 << 20, None) == -3      # signed range
    assert lib.mmse_scale_search_offset(None, 64, C.byref(pu), a, a, a, a, a, a, 1 << 20, None) == -1
    assert lib.mmse_scale_search_offset(a, 64, C.byref(pu), a + 2, a, a, a, a, a, 1 << 20, None) == -6
    assert lib.mmse_scale_search_offset(a, 64, C.byref(pu), a, a, a, a, a, None, 0, None) == -4
    assert lib.mmse_scale_alternating_kernelwise(a, 4, 4, -8, 7, 10, None, a, a, None) == -1
    assert lib.mmse_scale_alternating_kernelwise(a, 4, 65537, -8, 7, 10, a, a, a, None) == -2
    assert lib.mmse_scale_alternating_kernelwise(a, 4, 4, -8, 7, 1001, a, a, a, None) == -3
    assert lib.mmse_scale_alternating_kernelwise(a, 4, 4, -8, 7, 10, a, a + 4, a, None) == -6
    d1 = (B.MmseActDesc * 2)(B.MmseActDesc(a, 64, a, a, a, None), B.MmseActDesc(a, 4097, a, a, a, a))
    assert lib.mmse_scale_search_activation_batched(d1, 2, C.byref(pu), a, 16, None) == -4
    assert lib.mmse_scale_search_activation_batched(None, 2, C.byref(pu), a, 1 << 24, None) == -1
    assert lib.mmse_scale_search_activation_batched(d1, 0, C.byref(pu), a, 1 << 24, None) == -2
    assert lib.mmse_scale_search_activation_batched(d1, 1025, C.byref(pu), a, 1 << 24, None) == -2
    d2 = (B.MmseActDesc * 1)(B.MmseActDesc(a, 0, a, a, a, None))
    assert lib.mmse_scale_search_activation_batched(d2, 1, C.byref(pu), a, 1 << 24, None) == -2
    d3 = (B.MmseActDesc * 1)(B.MmseActDesc(a, 8, None, a, a, None))
    assert lib.mmse_scale_search_activation_batched(d3, 1, C.byref(pu), a, 1 << 24, None) == -1
    sizes = (C.c_int64 * 2)(64, 4097)
    need2, need1a, need1b = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    assert lib.mmse_workspace_bytes_activation_batched(sizes, 2, C.byref(pu), C.byref(need2)) == 0
    assert lib.mmse_workspace_bytes_activation(64, C.byref(pu), C.byref(need1a)) == 0
    assert lib.mmse_workspace_bytes_activation(4097, C.byref(pu), C.byref(need1b)) == 0
    assert max(need1a.value, need1b.value) <= need2.value <= 2 * (need1a.value + need1b.value)
    ptrs, ks = (C.c_void_p * 2)(a, a), (C.c_int64 * 2)(5, 7)
    assert lib.mmse_layer_error_sums(ptrs, ks, 2, None, None) == -1
    assert lib.mmse_layer_error_sums(None, ks, 2, a, None) == -1
    assert lib.mmse_layer_error_sums(ptrs, ks, 0, a, None) == -2
    assert lib.mmse_layer_error_sums(ptrs, (C.c_int64 * 2)(5, 0), 2, a, None) == -2
    assert lib.mmse_layer_error_sums((C.c_void_p * 2)(a, a + 4), ks, 2, a, None) == -6
    assert lib.mmse_layer_error_sums((C.c_void_p * 2)(a, None), ks, 2, a, None) == -1
    assert lib.mmse_grid_sse_activation(a, 64, C.byref(pu), None, a, a, 1 << 20, None) == -1
    assert lib.mmse_grid_sse_activation(a, 64, C.byref(pu), a, a + 4, a, 1 << 20, None) == -6
    assert lib.mmse_grid_sse_activation(a, 0, C.byref(pu), a, a, a, 1 << 20, None) == -2
    assert lib.mmse_grid_sse_activation(a, 64, C.byref(pu), a, a, a, 64, None) == -4
    # sizes
    assert lib.mmse_scale_search_kernelwise(a, 0, 4, C.byref(p), a, a, a, a, 4096, None) == -2
    assert lib.mmse_scale_search_kernelwise(a, 4, 65537, C.byref(p), a, a, a, a, 4096, None) == -2
    assert lib.mmse_scale_search_kernelwise(a, 1 << 20, 4096, C.byref(p), a, a, a, a, 1 << 30, None) == -2
    assert lib.mmse_scale_search_activation(a, 0, C.byref(p), a, a, a, a, 1 << 20, None) == -2
    assert lib.mmse_scale_search_activation(a, 1 << 31, C.byref(p), a, a, a, a, 1 << 20, None) == -2
    assert lib.quantize_pack_int4(a, 4, -1, a, -8, 7, a, None) == -2
    # parameters
    assert lib.quantize_pack_int4(a, 4, 4, a, 1, 7, a, None) == -3
    # workspace: missing, misaligned, too small
    assert lib.mmse_scale_search_kernelwise(a, 4, 4, C.byref(p), a, a, a, None, 4096, None) == -4
    assert lib.mmse_scale_search_kernelwise(a, 4, 4, C.byref(p), a, a, a, a + 64, 4096, None) == -4
    assert lib.mmse_scale_search_kernelwise(a, 400, 4, C.byref(p), a, a, a, a, 1024, None) == -4
    assert lib.mmse_scale_search_activation(a, 1 << 20, C.byref(p), a, a, a, a, 4096, None) == -4
    # alignment of typed outputs
    assert lib.mmse_scale_search_kernelwise(a + 2, 4, 4, C.byref(p), a, a, a, a, 4096, None) == -6
    assert lib.mmse_scale_search_kernelwise(a, 4, 4, C.byref(p), a, a, a + 4, a, 4096, None) == -6
    assert lib.mmse_scale_search_activation(a, 64, C.byref(p), a, a + 2, a, a, 1 << 20, None) == -6


def test_binding_refuses_host_tensors(B):
    import torch
    with pytest.raises(ValueError):
        B.mmse_scale_search_kernelwise(torch.zeros(4, 4), B.params(-8, 7, 16, 0))


def test_missing_library_is_an_error(B, monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", os.path.join(ROOT, "does_not_exist.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.load_library()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_product_path_does_not_touch_the_oracle():
    """Only tests, smoke() and bench.py's cpu_baseline leg may use oracle/."""
    pkg = os.path.join(ROOT, "paper_1902_06822_amd")
    pat = re.compile(r"^\s*(import\s+oracle|from\s+oracle)|libmmse_oracle|mmse_oracle\.c|oracle/", re.M)
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not pat.search(text), f
    assert not pat.search(open(os.path.join(ROOT, "include", "mmse.h")).read())


def test_kernels_spill_nothing():
    """Register arrays of the hot kernels (tree partials, staged temporaries, chunk data) must stay in
    VGPRs: the compiler's resource report may show no scratch for them."""
    import shutil
    import subprocess
    from paper_1902_06822_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    r = subprocess.run([hipcc, *flags, "--cuda-device-only", "-c", *build.SRC, "-o", os.devnull,
                        "-Rpass-analysis=kernel-resource-usage"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    name, seen = None, {}
    for line in r.stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and name:
            seen[name] = int(m.group(1))
    for must in ("k_sweep_kernelwise", "k_refine_kernelwise", "k_pack_int4", "k_act_sweep", "k_act_probe",
                 "k_act_absmax", "k_act_reduce64", "k_act_argmin", "k_act_finish", "k_dual_ls", "k_alt_kernelwise"):
        assert any(must in k for k in seen), (must, sorted(seen))
    assert len(seen) >= 30
    for k, scratch in seen.items():              # every kernel of the library, not only the hot ones
        assert scratch == 0, (k, scratch)
