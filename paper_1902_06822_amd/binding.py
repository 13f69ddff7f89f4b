"""Thin ctypes binding of ``libmmse_hip.so`` (see ``include/mmse.h``).

Argument marshalling only: every step of the search runs in the HIP kernels.
PyTorch supplies device memory and the current stream.  There is no CPU
fallback: if the library is missing, or a call fails, a RuntimeError is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch  # loaded first so that the HIP runtime torch ships is the one the library binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmmse_hip.so")

EXPORTS = (
    "mmse_workspace_bytes_kernelwise", "mmse_workspace_bytes_activation",
    "mmse_scale_search_kernelwise", "mmse_scale_search_activation", "mmse_scale_search_kernelwise_noalloc",
    "quantize_pack_int4", "residual_quantize", "mmse_scale_search_batched",
    "mmse_grid_sse_kernelwise", "mmse_workspace_bytes_dual", "dual_quantize_alternating",
    "mmse_workspace_bytes_dual_batched", "dual_quantize_alternating_batched",
    "mmse_workspace_bytes_dual_linesearch", "dual_line_search",
    "activation_residual_quantize", "mmse_scale_search_offset", "mmse_scale_alternating_kernelwise",
    "mmse_workspace_bytes_activation_batched", "mmse_scale_search_activation_batched", "mmse_layer_error_sums",
    "mmse_grid_sse_activation",
    "mmse_trace_create", "mmse_trace_read", "mmse_scale_search_batched_traced",
    "mmse_scale_search_activation_batched_traced",
    "mmse_status_string",
)
VOID_EXPORTS = ("mmse_trace_destroy",)

# MMSE_STAGE_* of include/mmse.h: the kernel a traced launch ran
STAGE_NAMES = {1: "k_sweep_kernelwise", 3: "k_refine_kernelwise<64>", 4: "k_refine_kernelwise<16>",
               5: "k_pack_int4", 6: "k_sweep_kernelwise (fused search)", 10: "k_act_init", 11: "k_act_absmax", 12: "k_act_sweep", 13: "k_act_reduce64 (grid sums)",
               14: "k_act_argmin", 15: "k_act_probe", 16: "k_act_reduce64 (probe sums)", 17: "k_act_finish",
               18: "k_act_pack"}


class MmseParams(C.Structure):
    _fields_ = [("qmin", C.c_int32), ("qmax", C.c_int32), ("grid_points", C.c_int32),
                ("refine_iters", C.c_int32), ("cands_per_lane", C.c_int32)]


class MmseTensorDesc(C.Structure):
    _fields_ = [("w_dev", C.c_void_p), ("K", C.c_int64), ("n", C.c_int64),
                ("scale1_dev", C.c_void_p), ("scale_dev", C.c_void_p), ("idx_dev", C.c_void_p),
                ("sse_dev", C.c_void_p), ("packed_dev", C.c_void_p)]


class MmseActDesc(C.Structure):
    _fields_ = [("x_dev", C.c_void_p), ("N", C.c_int64), ("scale_dev", C.c_void_p), ("idx_dev", C.c_void_p),
                ("sse_dev", C.c_void_p), ("packed_dev", C.c_void_p)]


class MmseDualDesc(C.Structure):
    _fields_ = [("w_dev", C.c_void_p), ("K", C.c_int64), ("n", C.c_int64),
                ("scale1_dev", C.c_void_p), ("scale2_dev", C.c_void_p), ("packed1_dev", C.c_void_p),
                ("packed2_dev", C.c_void_p), ("sse_dev", C.c_void_p), ("sweeps_dev", C.c_void_p)]


_lib = None


def load_library() -> C.CDLL:
    """Load the HIP library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1902_06822_amd.build` "
            "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i64, i32, szp = C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_size_t)
    pp = C.POINTER(MmseParams)
    lib.mmse_workspace_bytes_kernelwise.argtypes = [i64, i64, pp, szp]
    lib.mmse_workspace_bytes_activation.argtypes = [i64, pp, szp]
    lib.mmse_scale_search_kernelwise.argtypes = [vp, i64, i64, pp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.mmse_scale_search_activation.argtypes = [vp, i64, pp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.mmse_scale_search_kernelwise_noalloc.argtypes = [vp, i64, i64, pp, vp, vp, vp, vp]
    lib.quantize_pack_int4.argtypes = [vp, i64, i64, vp, i32, i32, vp, vp]
    lib.residual_quantize.argtypes = [vp, i64, i64, vp, pp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.mmse_scale_search_batched.argtypes = [C.POINTER(MmseTensorDesc), i32, pp, vp, C.c_size_t, vp]
    lib.mmse_grid_sse_kernelwise.argtypes = [vp, i64, i64, pp, vp, vp, vp]
    lib.mmse_workspace_bytes_dual.argtypes = [i64, i64, pp, szp]
    lib.dual_quantize_alternating.argtypes = [vp, i64, i64, pp, C.c_double, i32, vp, vp, vp, vp, vp, vp, vp,
                                              C.c_size_t, vp]
    lib.mmse_workspace_bytes_dual_batched.argtypes = [C.POINTER(MmseDualDesc), i32, pp, szp]
    lib.dual_quantize_alternating_batched.argtypes = [C.POINTER(MmseDualDesc), i32, pp, C.c_double, i32, vp,
                                                      C.c_size_t, vp]
    lib.mmse_workspace_bytes_dual_linesearch.argtypes = [i64, i64, i32, i32, szp]
    lib.dual_line_search.argtypes = [vp, i64, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                     C.c_size_t, vp]
    lib.activation_residual_quantize.argtypes = [vp, i64, vp, i32, i32, C.POINTER(MmseParams), vp, vp, vp, vp, vp,
                                                 C.c_size_t, vp]
    lib.mmse_scale_search_offset.argtypes = [vp, i64, C.POINTER(MmseParams), vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.mmse_scale_alternating_kernelwise.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
    lib.mmse_workspace_bytes_activation_batched.argtypes = [C.POINTER(C.c_int64), i32, C.POINTER(MmseParams), szp]
    lib.mmse_scale_search_activation_batched.argtypes = [C.POINTER(MmseActDesc), i32, C.POINTER(MmseParams), vp,
                                                         C.c_size_t, vp]
    lib.mmse_layer_error_sums.argtypes = [C.POINTER(C.c_void_p), C.POINTER(C.c_int64), i32, vp, vp]
    lib.mmse_grid_sse_activation.argtypes = [vp, i64, pp, vp, vp, vp, C.c_size_t, vp]
    lib.mmse_trace_create.argtypes = [i32, C.POINTER(vp)]
    lib.mmse_trace_destroy.argtypes = [vp]
    lib.mmse_trace_destroy.restype = None
    lib.mmse_trace_read.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_float)]
    lib.mmse_scale_search_batched_traced.argtypes = [C.POINTER(MmseTensorDesc), i32, pp, vp, C.c_size_t, vp, vp]
    lib.mmse_scale_search_activation_batched_traced.argtypes = [C.POINTER(MmseActDesc), i32, pp, vp, C.c_size_t, vp, vp]
    lib.mmse_status_string.argtypes = [C.c_int]
    lib.mmse_status_string.restype = C.c_char_p
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def status_string(rc: int) -> str:
    return load_library().mmse_status_string(rc).decode()


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{what} failed: {status_string(rc)} ({rc})")


def params(qmin: int, qmax: int, grid_points: int, refine_iters: int, cands_per_lane: int = 0) -> MmseParams:
    return MmseParams(qmin, qmax, grid_points, refine_iters, cands_per_lane)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class StageTrace:
    """Per-kernel durations of a traced batched call (``mmse_trace_*``): HIP events on the launch stream."""

    def __init__(self, capacity: int = 256):
        self.capacity = capacity
        self._h = C.c_void_p(None)
        _check(load_library().mmse_trace_create(capacity, C.byref(self._h)), "mmse_trace_create")

    @property
    def handle(self):
        return self._h

    def read(self):
        """[(stage id, milliseconds)] per kernel launch, in launch order (waits for the last kernel)."""
        n = C.c_int32(0)
        stages = (C.c_int32 * self.capacity)()
        ms = (C.c_float * self.capacity)()
        _check(load_library().mmse_trace_read(self._h, self.capacity, C.byref(n), stages, ms), "mmse_trace_read")
        return [(int(stages[i]), float(ms[i])) for i in range(n.value)]

    def close(self):
        if self._h:
            load_library().mmse_trace_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"expected a contiguous {dtype} device tensor, got {t.dtype} on {t.device}")
    return t


def mmse_workspace_bytes_kernelwise(K: int, n: int, p: MmseParams) -> int:
    out = C.c_size_t(0)
    _check(load_library().mmse_workspace_bytes_kernelwise(K, n, C.byref(p), C.byref(out)),
           "mmse_workspace_bytes_kernelwise")
    return out.value


def mmse_workspace_bytes_activation(N: int, p: MmseParams) -> int:
    out = C.c_size_t(0)
    _check(load_library().mmse_workspace_bytes_activation(N, C.byref(p), C.byref(out)),
           "mmse_workspace_bytes_activation")
    return out.value


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


@dataclass
class SearchResult:
    scale: torch.Tensor     # fp32 [K]
    idx: torch.Tensor       # int32 [K]
    sse: torch.Tensor       # fp64 [K]
    packed: Optional[torch.Tensor] = None   # uint8 [ceil(K*n/2)]


def _outputs(K: int, device) -> SearchResult:
    return SearchResult(torch.empty(K, dtype=torch.float32, device=device),
                        torch.empty(K, dtype=torch.int32, device=device),
                        torch.empty(K, dtype=torch.float64, device=device))


def mmse_scale_search_kernelwise(w: torch.Tensor, p: MmseParams, ws: Optional[torch.Tensor] = None,
                                 out: Optional[SearchResult] = None) -> SearchResult:
    _dev(w, torch.float32)
    K, n = w.shape
    if ws is None:
        ws = alloc_workspace(mmse_workspace_bytes_kernelwise(K, n, p), w.device)
    if out is None:
        out = _outputs(K, w.device)
    _check(load_library().mmse_scale_search_kernelwise(
        w.data_ptr(), K, n, C.byref(p), out.scale.data_ptr(), out.idx.data_ptr(), out.sse.data_ptr(),
        ws.data_ptr(), ws.numel(), _stream()), "mmse_scale_search_kernelwise")
    return out


def mmse_scale_search_kernelwise_noalloc(w: torch.Tensor, p: MmseParams, out: SearchResult) -> SearchResult:
    """The kernel-wise search without a workspace (a fixed array inside the library); `out` must exist."""
    _dev(w, torch.float32)
    K, n = w.shape
    _check(load_library().mmse_scale_search_kernelwise_noalloc(
        w.data_ptr(), K, n, C.byref(p), out.scale.data_ptr(), out.idx.data_ptr(), out.sse.data_ptr(), _stream()),
        "mmse_scale_search_kernelwise_noalloc")
    return out


def mmse_scale_search_activation(x: torch.Tensor, p: MmseParams, ws: Optional[torch.Tensor] = None,
                                 out: Optional[SearchResult] = None) -> SearchResult:
    _dev(x, torch.float32)
    N = x.numel()
    if ws is None:
        ws = alloc_workspace(mmse_workspace_bytes_activation(N, p), x.device)
    if out is None:
        out = _outputs(1, x.device)
    _check(load_library().mmse_scale_search_activation(
        x.data_ptr(), N, C.byref(p), out.scale.data_ptr(), out.idx.data_ptr(), out.sse.data_ptr(),
        ws.data_ptr(), ws.numel(), _stream()), "mmse_scale_search_activation")
    return out


def quantize_pack_int4(x: torch.Tensor, scale: torch.Tensor, qmin: int, qmax: int,
                       packed: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(x, torch.float32)
    _dev(scale, torch.float32)
    if x.dim() == 1:
        K, n = 1, x.numel()
    else:
        K, n = x.shape
    if scale.numel() != K:
        raise ValueError("one scale per row expected")
    if packed is None:
        packed = torch.empty((K * n + 1) // 2, dtype=torch.uint8, device=x.device)
    _check(load_library().quantize_pack_int4(x.data_ptr(), K, n, scale.data_ptr(), qmin, qmax,
                                             packed.data_ptr(), _stream()), "quantize_pack_int4")
    return packed


def residual_quantize(w: torch.Tensor, scale1: torch.Tensor, p: MmseParams,
                      ws: Optional[torch.Tensor] = None, want_packed: bool = True) -> SearchResult:
    _dev(w, torch.float32)
    _dev(scale1, torch.float32)
    K, n = w.shape
    if ws is None:
        ws = alloc_workspace(mmse_workspace_bytes_kernelwise(K, n, p), w.device)
    out = _outputs(K, w.device)
    if want_packed:
        out.packed = torch.empty((K * n + 1) // 2, dtype=torch.uint8, device=w.device)
    _check(load_library().residual_quantize(
        w.data_ptr(), K, n, scale1.data_ptr(), C.byref(p), out.scale.data_ptr(), out.idx.data_ptr(),
        out.sse.data_ptr(), _ptr(out.packed), ws.data_ptr(), ws.numel(), _stream()), "residual_quantize")
    return out


class BatchedPlan:
    """Host-side descriptor table for ``mmse_scale_search_batched`` (buffers allocated once)."""

    def __init__(self, weights: Sequence[torch.Tensor], p: MmseParams, want_packed: bool = True,
                 scale1: Optional[Sequence[Optional[torch.Tensor]]] = None):
        self.p = p
        self.weights = list(weights)
        self.results: List[SearchResult] = []
        descs = (MmseTensorDesc * len(self.weights))()
        sumK = 0
        for i, w in enumerate(self.weights):
            _dev(w, torch.float32)
            K, n = w.shape
            r = _outputs(K, w.device)
            if want_packed:
                r.packed = torch.empty((K * n + 1) // 2, dtype=torch.uint8, device=w.device)
            self.results.append(r)
            s1 = None if scale1 is None else scale1[i]
            descs[i] = MmseTensorDesc(w.data_ptr(), K, n, _ptr(s1), r.scale.data_ptr(), r.idx.data_ptr(),
                                      r.sse.data_ptr(), _ptr(r.packed))
            sumK += K
        self._scale1 = scale1
        self.descs = descs
        self.ws = alloc_workspace(mmse_workspace_bytes_kernelwise(sumK, 1, p), self.weights[0].device)

    def run(self) -> List[SearchResult]:
        _check(load_library().mmse_scale_search_batched(self.descs, len(self.weights), C.byref(self.p),
                                                        self.ws.data_ptr(), self.ws.numel(), _stream()),
               "mmse_scale_search_batched")
        return self.results

    def run_subset(self, indices: Sequence[int]) -> List[SearchResult]:
        """One batched call over some of the plan's tensors (their buffers exist already; only the host-side
        descriptor table of the call is built here)."""
        sub = (MmseTensorDesc * len(indices))(*[self.descs[i] for i in indices])
        _check(load_library().mmse_scale_search_batched(sub, len(indices), C.byref(self.p), self.ws.data_ptr(),
                                                        self.ws.numel(), _stream()), "mmse_scale_search_batched")
        return [self.results[i] for i in indices]

    def run_traced(self, trace: StageTrace) -> List[SearchResult]:
        _check(load_library().mmse_scale_search_batched_traced(self.descs, len(self.weights), C.byref(self.p),
                                                               self.ws.data_ptr(), self.ws.numel(), _stream(),
                                                               trace.handle), "mmse_scale_search_batched_traced")
        return self.results


def mmse_scale_search_batched(weights: Sequence[torch.Tensor], p: MmseParams, want_packed: bool = True,
                              scale1: Optional[Sequence[Optional[torch.Tensor]]] = None) -> List[SearchResult]:
    return BatchedPlan(weights, p, want_packed, scale1).run()


def mmse_grid_sse_kernelwise(w: torch.Tensor, p: MmseParams):
    _dev(w, torch.float32)
    K, n = w.shape
    absmax = torch.empty(K, dtype=torch.float32, device=w.device)
    grid = torch.empty((K, p.grid_points), dtype=torch.float64, device=w.device)
    _check(load_library().mmse_grid_sse_kernelwise(w.data_ptr(), K, n, C.byref(p), absmax.data_ptr(),
                                                   grid.data_ptr(), _stream()), "mmse_grid_sse_kernelwise")
    return absmax, grid


@dataclass
class DualResult:
    scale1: torch.Tensor    # fp32 [K]
    scale2: torch.Tensor    # fp32 [K]
    packed1: torch.Tensor   # uint8 [ceil(K*n/2)]
    packed2: torch.Tensor
    sse: torch.Tensor       # fp64 [K]
    sweeps: torch.Tensor    # int32 [K]


def mmse_workspace_bytes_dual(K: int, n: int, p: MmseParams) -> int:
    out = C.c_size_t(0)
    _check(load_library().mmse_workspace_bytes_dual(K, n, C.byref(p), C.byref(out)), "mmse_workspace_bytes_dual")
    return out.value


def dual_quantize_alternating(w: torch.Tensor, p: MmseParams, eps: float, max_sweeps: int,
                              ws: Optional[torch.Tensor] = None, out: Optional[DualResult] = None) -> DualResult:
    _dev(w, torch.float32)
    K, n = w.shape
    if ws is None:
        ws = alloc_workspace(mmse_workspace_bytes_dual(K, n, p), w.device)
    if out is None:
        nb = (K * n + 1) // 2
        out = DualResult(torch.empty(K, dtype=torch.float32, device=w.device),
                         torch.empty(K, dtype=torch.float32, device=w.device),
                         torch.empty(nb, dtype=torch.uint8, device=w.device),
                         torch.empty(nb, dtype=torch.uint8, device=w.device),
                         torch.empty(K, dtype=torch.float64, device=w.device),
                         torch.empty(K, dtype=torch.int32, device=w.device))
    _check(load_library().dual_quantize_alternating(
        w.data_ptr(), K, n, C.byref(p), float(eps), int(max_sweeps), out.scale1.data_ptr(), out.scale2.data_ptr(),
        out.packed1.data_ptr(), out.packed2.data_ptr(), out.sse.data_ptr(), out.sweeps.data_ptr(),
        ws.data_ptr(), ws.numel(), _stream()), "dual_quantize_alternating")
    return out


def _dual_outputs(K: int, n: int, device) -> DualResult:
    nb = (K * n + 1) // 2
    return DualResult(torch.empty(K, dtype=torch.float32, device=device),
                      torch.empty(K, dtype=torch.float32, device=device),
                      torch.empty(nb, dtype=torch.uint8, device=device),
                      torch.empty(nb, dtype=torch.uint8, device=device),
                      torch.empty(K, dtype=torch.float64, device=device),
                      torch.empty(K, dtype=torch.int32, device=device))


class DualBatchedPlan:
    """Host-side descriptor table for ``dual_quantize_alternating_batched`` (buffers allocated once)."""

    def __init__(self, weights: Sequence[torch.Tensor], p: MmseParams, eps: float, max_sweeps: int):
        self.p, self.eps, self.max_sweeps = p, float(eps), int(max_sweeps)
        self.weights = list(weights)
        self.results: List[DualResult] = []
        self.descs = (MmseDualDesc * len(self.weights))()
        for i, w in enumerate(self.weights):
            _dev(w, torch.float32)
            K, n = w.shape
            r = _dual_outputs(K, n, w.device)
            self.results.append(r)
            self.descs[i] = MmseDualDesc(w.data_ptr(), K, n, r.scale1.data_ptr(), r.scale2.data_ptr(),
                                         r.packed1.data_ptr(), r.packed2.data_ptr(), r.sse.data_ptr(),
                                         r.sweeps.data_ptr())
        need = C.c_size_t(0)
        _check(load_library().mmse_workspace_bytes_dual_batched(self.descs, len(self.weights), C.byref(p),
                                                                C.byref(need)), "mmse_workspace_bytes_dual_batched")
        self.ws = alloc_workspace(need.value, self.weights[0].device)

    def run(self) -> List[DualResult]:
        _check(load_library().dual_quantize_alternating_batched(
            self.descs, len(self.weights), C.byref(self.p), self.eps, self.max_sweeps,
            self.ws.data_ptr(), self.ws.numel(), _stream()), "dual_quantize_alternating_batched")
        return self.results


def dual_quantize_alternating_batched(weights: Sequence[torch.Tensor], p: MmseParams, eps: float,
                                      max_sweeps: int) -> List[DualResult]:
    return DualBatchedPlan(weights, p, eps, max_sweeps).run()


@dataclass
class DualLineSearchResult:
    scale1: torch.Tensor
    scale2: torch.Tensor
    idx1: torch.Tensor
    idx2: torch.Tensor
    sse: torch.Tensor
    packed1: torch.Tensor
    packed2: torch.Tensor
    grid: Optional[torch.Tensor] = None


def mmse_workspace_bytes_dual_linesearch(K: int, n: int, G1: int, G2: int) -> int:
    out = C.c_size_t(0)
    _check(load_library().mmse_workspace_bytes_dual_linesearch(K, n, G1, G2, C.byref(out)),
           "mmse_workspace_bytes_dual_linesearch")
    return out.value


def dual_line_search(w: torch.Tensor, qmin: int, qmax: int, G1: int, G2: int, want_grid: bool = False,
                     ws: Optional[torch.Tensor] = None, out: Optional[DualLineSearchResult] = None
                     ) -> DualLineSearchResult:
    _dev(w, torch.float32)
    K, n = w.shape
    if ws is None:
        ws = alloc_workspace(mmse_workspace_bytes_dual_linesearch(K, n, G1, G2), w.device)
    if out is None:
        nb = (K * n + 1) // 2
        f32 = lambda: torch.empty(K, dtype=torch.float32, device=w.device)
        i32t = lambda: torch.empty(K, dtype=torch.int32, device=w.device)
        out = DualLineSearchResult(f32(), f32(), i32t(), i32t(), torch.empty(K, dtype=torch.float64, device=w.device),
                                   torch.empty(nb, dtype=torch.uint8, device=w.device),
                                   torch.empty(nb, dtype=torch.uint8, device=w.device),
                                   torch.empty((K, G1 * G2), dtype=torch.float64, device=w.device) if want_grid else None)
    _check(load_library().dual_line_search(
        w.data_ptr(), K, n, qmin, qmax, G1, G2, out.scale1.data_ptr(), out.scale2.data_ptr(), out.idx1.data_ptr(),
        out.idx2.data_ptr(), out.sse.data_ptr(), out.packed1.data_ptr(), out.packed2.data_ptr(), _ptr(out.grid),
        ws.data_ptr(), ws.numel(), _stream()), "dual_line_search")
    return out


def activation_residual_quantize(x: torch.Tensor, scale1: torch.Tensor, qmin1: int, qmax1: int, p: MmseParams,
                                 ws: Optional[torch.Tensor] = None, out: Optional[SearchResult] = None,
                                 want_packed: bool = True) -> SearchResult:
    """Eq. 16: search (and codes) of the residual of the first tensor; p describes the second tensor."""
    _dev(x, torch.float32)
    _dev(scale1, torch.float32)
    N = x.numel()
    if ws is None:
        ws = alloc_workspace(mmse_workspace_bytes_activation(N, p), x.device)
    if out is None:
        out = SearchResult(torch.empty(1, dtype=torch.float32, device=x.device),
                           torch.empty(1, dtype=torch.int32, device=x.device),
                           torch.empty(1, dtype=torch.float64, device=x.device),
                           torch.empty((N + 1) // 2, dtype=torch.uint8, device=x.device) if want_packed else None)
    _check(load_library().activation_residual_quantize(
        x.data_ptr(), N, scale1.data_ptr(), qmin1, qmax1, C.byref(p), out.scale.data_ptr(), out.idx.data_ptr(),
        out.sse.data_ptr(), _ptr(out.packed), ws.data_ptr(), ws.numel(), _stream()), "activation_residual_quantize")
    return out


@dataclass
class OffsetResult:
    delta: torch.Tensor
    scale: torch.Tensor
    idx: torch.Tensor
    sse: torch.Tensor
    packed: Optional[torch.Tensor] = None


def mmse_scale_search_offset(x: torch.Tensor, p: MmseParams, ws: Optional[torch.Tensor] = None,
                             out: Optional[OffsetResult] = None, want_packed: bool = True) -> OffsetResult:
    """Eq. 2 with the MMSE scale: delta = min x, unsigned codes of x - delta."""
    _dev(x, torch.float32)
    N = x.numel()
    if ws is None:
        ws = alloc_workspace(mmse_workspace_bytes_activation(N, p), x.device)
    if out is None:
        out = OffsetResult(torch.empty(1, dtype=torch.float32, device=x.device),
                           torch.empty(1, dtype=torch.float32, device=x.device),
                           torch.empty(1, dtype=torch.int32, device=x.device),
                           torch.empty(1, dtype=torch.float64, device=x.device),
                           torch.empty((N + 1) // 2, dtype=torch.uint8, device=x.device) if want_packed else None)
    _check(load_library().mmse_scale_search_offset(
        x.data_ptr(), N, C.byref(p), out.delta.data_ptr(), out.scale.data_ptr(), out.idx.data_ptr(),
        out.sse.data_ptr(), _ptr(out.packed), ws.data_ptr(), ws.numel(), _stream()), "mmse_scale_search_offset")
    return out


def mmse_scale_alternating_kernelwise(w: torch.Tensor, qmin: int, qmax: int, max_iters: int):
    """Alternating optimisation of Section 3.4's comparison: (scale [K], sse [K], updates [K])."""
    _dev(w, torch.float32)
    K, n = w.shape
    scale = torch.empty(K, dtype=torch.float32, device=w.device)
    sse = torch.empty(K, dtype=torch.float64, device=w.device)
    upd = torch.empty(K, dtype=torch.int32, device=w.device)
    _check(load_library().mmse_scale_alternating_kernelwise(
        w.data_ptr(), K, n, qmin, qmax, max_iters, scale.data_ptr(), sse.data_ptr(), upd.data_ptr(), _stream()),
        "mmse_scale_alternating_kernelwise")
    return scale, sse, upd


class ActBatchedPlan:
    """Host-side descriptor table for ``mmse_scale_search_activation_batched`` (buffers allocated once)."""

    def __init__(self, tensors: Sequence[torch.Tensor], p: MmseParams, want_packed: bool = True):
        self.p = p
        self.tensors = list(tensors)
        self.results: List[SearchResult] = []
        descs = (MmseActDesc * len(self.tensors))()
        sizes = (C.c_int64 * len(self.tensors))()
        for i, x in enumerate(self.tensors):
            _dev(x, torch.float32)
            N = x.numel()
            r = _outputs(1, x.device)
            if want_packed:
                r.packed = torch.empty((N + 1) // 2, dtype=torch.uint8, device=x.device)
            self.results.append(r)
            descs[i] = MmseActDesc(x.data_ptr(), N, r.scale.data_ptr(), r.idx.data_ptr(), r.sse.data_ptr(), _ptr(r.packed))
            sizes[i] = N
        self.descs = descs
        need = C.c_size_t(0)
        _check(load_library().mmse_workspace_bytes_activation_batched(sizes, len(self.tensors), C.byref(p), C.byref(need)),
               "mmse_workspace_bytes_activation_batched")
        self.ws = alloc_workspace(need.value, self.tensors[0].device)

    def run(self) -> List[SearchResult]:
        _check(load_library().mmse_scale_search_activation_batched(self.descs, len(self.tensors), C.byref(self.p),
                                                                   self.ws.data_ptr(), self.ws.numel(), _stream()),
               "mmse_scale_search_activation_batched")
        return self.results

    def run_traced(self, trace: StageTrace) -> List[SearchResult]:
        _check(load_library().mmse_scale_search_activation_batched_traced(
            self.descs, len(self.tensors), C.byref(self.p), self.ws.data_ptr(), self.ws.numel(), _stream(),
            trace.handle), "mmse_scale_search_activation_batched_traced")
        return self.results


def mmse_scale_search_activation_batched(tensors: Sequence[torch.Tensor], p: MmseParams,
                                         want_packed: bool = True) -> List[SearchResult]:
    return ActBatchedPlan(tensors, p, want_packed).run()


class LayerSumsPlan:
    """Per-layer totals of per-kernel errors (``mmse_layer_error_sums``); buffers and tables built once."""

    def __init__(self, sse_tensors: Sequence[torch.Tensor]):
        self.tensors = list(sse_tensors)
        n = len(self.tensors)
        self.ptrs = (C.c_void_p * n)(*[_dev(t, torch.float64).data_ptr() for t in self.tensors])
        self.sizes = (C.c_int64 * n)(*[t.numel() for t in self.tensors])
        self.out = torch.empty(n, dtype=torch.float64, device=self.tensors[0].device)

    def run(self) -> torch.Tensor:
        _check(load_library().mmse_layer_error_sums(self.ptrs, self.sizes, len(self.tensors), self.out.data_ptr(),
                                                    _stream()), "mmse_layer_error_sums")
        return self.out


def mmse_layer_error_sums(sse_tensors: Sequence[torch.Tensor]) -> torch.Tensor:
    return LayerSumsPlan(sse_tensors).run()


def mmse_grid_sse_activation(x: torch.Tensor, p: MmseParams):
    """(absmax [1], f(alpha_j) [G]) of an activation tensor: the candidate sweep alone."""
    _dev(x, torch.float32)
    N = x.numel()
    ws = alloc_workspace(mmse_workspace_bytes_activation(N, p), x.device)
    absmax = torch.empty(1, dtype=torch.float32, device=x.device)
    grid = torch.empty(p.grid_points, dtype=torch.float64, device=x.device)
    _check(load_library().mmse_grid_sse_activation(x.data_ptr(), N, C.byref(p), absmax.data_ptr(), grid.data_ptr(),
                                                   ws.data_ptr(), ws.numel(), _stream()), "mmse_grid_sse_activation")
    return absmax, grid
