// mmse_kernels.hip -- gfx950 (MI355X) kernels and C ABI of the MMSE INT4 scale search.
//
// Method: arXiv 1902.06822.  For a tensor T and integer range Z_p the scale alpha
// minimises f(alpha) = sum_i (T_i - alpha*[T_i/alpha]_Zp)^2 (Section 3.4, Eq. 7-8),
// found by evaluating f on a grid of G candidates in parallel and taking the argmin;
// weights are searched per output-channel kernel (Section 3.3), activations per
// layer (Section 3.7, Eq. 15); the residual of a first fit can be fitted again
// (Section 3.5, Algorithm 1; Eq. 16).
//
// Arithmetic contract (what every kernel below computes, bit for bit):
//   inv = 1.0f/alpha;  q = clamp(rint(x*inv), qmin, qmax);  r = fma(-alpha, q, x);
//   s   = fma(r, r, s) sequentially over a chunk of 64 consecutive elements (fp32);
//   f   = pairwise fp64 sum of the chunk sums (adjacent pairs, level by level; a value
//         without a partner is carried up unchanged).
// Chunk sums are >= +0, so padding a chunk with zeros or a tree level with 0.0 never
// changes a bit; the kernels use that freely.  Nothing is ever accumulated with
// floating-point atomics: every result is independent of scheduling.
//
// Files: this translation unit holds the host side (validation, launch plans) and the C ABI; the kernels are in
//   mmse_common.h      constants, element arithmetic, summation tree, the LDS-fed sweep core
//   mmse_weights.h     k_sweep_kernelwise (with sweep_small_wave and the fused search), k_refine_kernelwise, k_pack_int4
//   mmse_dual.h        Algorithm 1 iterated (bookkeeping kernels) and the dual line search of Eq. 12
//   mmse_compare.h     the alternating optimiser of the paper's comparison
//   mmse_activation.h  k_act_*: per-layer activation path, batched over tensors, with its variants
//
// Kernel map
//   k_sweep_kernelwise   one workgroup per weight kernel: slice staged in LDS (abs-max
//                        and the optional residual transform fused into the staging),
//                        waves split the grid, lanes own candidates, elements are
//                        broadcast from LDS; binary-counter tree of fp64 partials in
//                        registers; argmin with lowest-index tie-break.
//   k_refine_kernelwise  golden-section refinement, lane = (kernel, 64-element chunk)
//                        packed densely so that 9-element depthwise kernels use one
//                        lane each; chunk held in registers across the 22 probes.
//   k_pack_int4          fused quantize + INT4 pack, 8 elements per thread.
//   k_act_*              one activation tensor spread over the whole GPU.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>
#include <atomic>
#include <new>

#include "mmse.h"

#include "mmse_common.h"
#include "mmse_weights.h"
#include "mmse_dual.h"
#include "mmse_compare.h"
#include "mmse_activation.h"

namespace {

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

// Measurement aid: HIP events recorded on the launch stream after every kernel of a traced call.
struct mmse_trace {
    int capacity;
    int used;
    hipEvent_t* ev;
    int* stage;
};

namespace {

thread_local mmse_trace* t_trace = nullptr;     // set for the duration of a *_traced call on this host thread

inline void trace_mark(hipStream_t s, int stage)
{
    mmse_trace* T = t_trace;
    if (!T || T->used >= T->capacity) return;
    if (hipEventRecord(T->ev[T->used], s) != hipSuccess) return;
    T->stage[T->used++] = stage;
}

// A launch holds at most 2^32 - 1 work-items.  Workgroups have up to 512 threads where their count follows the
// number of kernels or blocks (1024 only for kernels of more than 32768 elements, of which a tensor has fewer
// than 65536), so launches are cut at this many workgroups.
constexpr long long kMaxLaunchWG = 1LL << 22;
constexpr int kFewBlocks = 512;         // activation blocks in a call up to which the chip's 256 CUs are not all busy twice over
constexpr long long kFusedMaxKernels = 1024;      // calls of at most this many kernels and elements take the single-launch
constexpr long long kFusedMaxElements = 1 << 20;  // search: beyond, the separate refinement kernel packs its lanes better
static_assert(kMaxLaunchWG == MMSE_MAX_KERNELS, "one workgroup per kernel");

int check_params(const mmse_params_t* p)
{
    if (!p) return MMSE_ERR_NULL;
    if (!(p->qmin <= 0 && p->qmax > 0 && p->qmax - p->qmin <= 15)) return MMSE_ERR_PARAMS;
    if (p->grid_points < 1 || p->grid_points > MMSE_MAX_GRID_POINTS) return MMSE_ERR_PARAMS;
    if (p->refine_iters < 0 || p->refine_iters > MMSE_MAX_REFINE_ITERS) return MMSE_ERR_PARAMS;
    const int c = p->cands_per_lane;
    if (!(c == 0 || c == 1 || c == 2 || c == 4)) return MMSE_ERR_PARAMS;
    if (c != 0 && (p->grid_points + 64 * c - 1) / (64 * c) > 8) return MMSE_ERR_PARAMS;
    return MMSE_OK;
}

int pick_cands(const mmse_params_t* p)
{
    if (p->cands_per_lane) return p->cands_per_lane;
    // Two candidates per lane halve the LDS reads per evaluation (0.81-0.82 of the VALU peak instead of 0.77-0.78)
    // but also the waves per workgroup, and a workgroup's LDS slice then allows fewer waves per SIMD: it pays
    // from four waves per workgroup on, i.e. above 384 grid points.
    const int G = p->grid_points;
    if (G <= 384) return 1;
    if (G <= 1024) return 2;
    return 4;
}

bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_tensor(const mmse_tensor_desc_t& d, bool need_outputs)
{
    if (!d.w_dev) return MMSE_ERR_NULL;
    if (need_outputs && (!d.scale_dev || !d.idx_dev || !d.sse_dev)) return MMSE_ERR_NULL;
    if (d.K <= 0 || d.n <= 0 || d.n > MMSE_MAX_KERNEL_ELEMS) return MMSE_ERR_SIZE;
    if (d.K > MMSE_MAX_TENSOR_ELEMS / d.n || d.K > MMSE_MAX_KERNELS) return MMSE_ERR_SIZE;
    if (!aligned_to(d.w_dev, 4) || !aligned_to(d.scale_dev, 4) || !aligned_to(d.idx_dev, 4) ||
        !aligned_to(d.sse_dev, 8) || !aligned_to(d.scale1_dev, 4))
        return MMSE_ERR_ALIGN;
    return MMSE_OK;
}

void fill_common(Batch& B, const mmse_params_t* p)
{
    B.G = p->grid_points;
    B.qmax = p->qmax;
    B.iters = p->refine_iters;
    B.lo = (float)p->qmin;
    B.hi = (float)p->qmax;
}

// ---- the weight path: which workgroups every tensor gets in every launch ----------------------------------
// Launches of one call: the sweep (ordinary kernels and, in the same launch, tiny ones), the refinement by
// class of lanes per kernel, the code pass for what the refinement did not code.
enum { ST_SWEEP = 0, ST_REF0, ST_REF1, ST_REF2, ST_REF3, ST_PACK, ST_COUNT };

struct WeightShape {        // launch shape of the call: the same for host and device
    int waves;              // waves of a sweep workgroup
    int CS;                 // candidates per lane of the one-wave-per-kernel path (0: not used)
    int do_search;
    int iters;
    int fused;              // the sweep launch also refines and codes (small calls)
};

__host__ __device__ inline int refine_class(int n)
{
    const int m = (n + kChunk - 1) / kChunk;
    return n <= 16 ? 0 : (m <= 256 ? 1 : (m <= 512 ? 2 : 3));
}
__host__ __device__ inline int refine_threads(int cls) { return cls == 3 ? 1024 : (cls == 2 ? 512 : 256); }

// Workgroups tensor (K, n) gets in launch `stage` (0: none).
__host__ __device__ inline long long stage_wgs(int stage, long long K, int n, bool has_packed, const WeightShape& sh)
{
    if (stage == ST_SWEEP) {
        if (!sh.do_search) return 0;
        return (sh.CS > 0 && n <= kChunk) ? (K + sh.waves - 1) / sh.waves : K;
    }
    if (stage >= ST_REF0 && stage <= ST_REF3) {
        const int cls = stage - ST_REF0;
        if (!sh.do_search || sh.iters <= 0 || sh.fused || refine_class(n) != cls) return 0;
        const int lanes = cls == 0 ? 1 : (n + kChunk - 1) / kChunk;
        const int cpw = refine_threads(cls) / lanes;
        return (K + cpw - 1) / cpw;
    }
    // codes: everything without a search; with one, what the refinement kernel did not code itself (odd n, or no refinement)
    if (!has_packed) return 0;
    if (sh.do_search && (sh.iters > 0 || sh.fused) && (n & 1) == 0) return 0;
    const long long per_wg = (long long)kPackThreads * kPackPerThread;
    return (K * n + per_wg - 1) / per_wg;
}

// Candidates per lane of the one-wave-per-kernel path for a sweep with C candidates per lane in the ordinary
// path, or 0 when that combination is not compiled (explicit tuning values, grids above 512 points).
int small_cs(int C, int G)
{
    if (C == 1 && G <= 64) return 1;
    if (C == 1 && G <= 128) return 2;
    if (C == 1 && G <= 256) return 4;
    if (C == 1 && G <= 384) return 8;
    if (C == 2 && G > 384 && G <= 512) return 8;
    return 0;
}

template <int C, int CS>
void launch_sweep_lv(const Batch& B, dim3 grid, dim3 block, size_t lds, int chunks, hipStream_t s)
{
    // binary-counter levels for the longest kernel of the launch: each level is two registers per candidate
    if constexpr (CS > 0) {
        hipLaunchKernelGGL((k_sweep_kernelwise<C, kLevelsKWSmall, CS, false>), grid, block, lds, s, B);
    } else {
        if (chunks <= 128) hipLaunchKernelGGL((k_sweep_kernelwise<C, kLevelsKWSmall, 0, false>), grid, block, lds, s, B);
        else if (chunks < 512) hipLaunchKernelGGL((k_sweep_kernelwise<C, 9, 0, false>), grid, block, lds, s, B);
        else if (chunks < 1024) hipLaunchKernelGGL((k_sweep_kernelwise<C, 10, 0, false>), grid, block, lds, s, B);
        else hipLaunchKernelGGL((k_sweep_kernelwise<C, kLevelsKW, 0, false>), grid, block, lds, s, B);
    }
}

// CS > 0 and fused only together with kernels of at most 128 chunks (the caller checks)
int launch_sweep(int C, int CS, bool fused, const Batch& B, int nwg, int waves, size_t lds, int chunks, hipStream_t s)
{
    const dim3 grid(nwg), block(64 * waves);
    if (fused) {
        if (C == 1) hipLaunchKernelGGL((k_sweep_kernelwise<1, kLevelsKWSmall, 0, true>), grid, block, lds, s, B);
        else if (C == 2) hipLaunchKernelGGL((k_sweep_kernelwise<2, kLevelsKWSmall, 0, true>), grid, block, lds, s, B);
        else hipLaunchKernelGGL((k_sweep_kernelwise<4, kLevelsKWSmall, 0, true>), grid, block, lds, s, B);
        trace_mark(s, MMSE_STAGE_W_FUSED);
        return hipGetLastError() == hipSuccess ? MMSE_OK : MMSE_ERR_LAUNCH;
    }
    if (C == 1 && CS == 0) launch_sweep_lv<1, 0>(B, grid, block, lds, chunks, s);
    else if (C == 1 && CS == 1) launch_sweep_lv<1, 1>(B, grid, block, lds, chunks, s);
    else if (C == 1 && CS == 2) launch_sweep_lv<1, 2>(B, grid, block, lds, chunks, s);
    else if (C == 1 && CS == 4) launch_sweep_lv<1, 4>(B, grid, block, lds, chunks, s);
    else if (C == 1 && CS == 8) launch_sweep_lv<1, 8>(B, grid, block, lds, chunks, s);
    else if (C == 2 && CS == 0) launch_sweep_lv<2, 0>(B, grid, block, lds, chunks, s);
    else if (C == 2 && CS == 8) launch_sweep_lv<2, 8>(B, grid, block, lds, chunks, s);
    else if (C == 4 && CS == 0) launch_sweep_lv<4, 0>(B, grid, block, lds, chunks, s);
    else return MMSE_ERR_PARAMS;
    trace_mark(s, MMSE_STAGE_W_SWEEP);
    return hipGetLastError() == hipSuccess ? MMSE_OK : MMSE_ERR_LAUNCH;
}

struct Item {              // one tensor of a batched call, host side
    TensorArgs a;
    int order;
};

// One launch of `stage` for the tensors in B (kernel-argument table or device-resident table), nwg workgroups.
// lds_floats / chunks: LDS of the sweep and the longest kernel of the launch in chunks; xf: some member is
// searched through a transform.
int launch_stage(int stage, const Batch& B, int nwg, int C, const WeightShape& sh, int lds_floats, int chunks, bool xf,
                 hipStream_t s)
{
    if (nwg <= 0) return MMSE_OK;
    if (stage == ST_SWEEP)   // fused: the reduction buffers of the refinement (two doubles per thread) follow the slice
        return launch_sweep(C, sh.CS, sh.fused != 0, B, nwg, sh.waves,
                            (size_t)lds_floats * sizeof(float) + (sh.fused ? (size_t)sh.waves * 64 * 2 * sizeof(double) : 0),
                            chunks, s);
    if (stage == ST_PACK) {
        hipLaunchKernelGGL(k_pack_int4, dim3(nwg), dim3(kPackThreads), 0, s, B);
        trace_mark(s, MMSE_STAGE_W_PACK);
        return hipGetLastError() == hipSuccess ? MMSE_OK : MMSE_ERR_LAUNCH;
    }
    const int cls = stage - ST_REF0;
    const int threads = refine_threads(cls);
    // LDS: combine buffer (2 doubles per thread) + one transpose tile per wave
    const int tile_chunks = cls == 0 ? 0 : 32 * 256 / threads;
    const size_t lds = (size_t)threads * 2 * sizeof(double) + (size_t)(threads / 64) * tile_chunks * kTileStride * sizeof(float);
    if (cls == 0) {
        if (xf) hipLaunchKernelGGL((k_refine_kernelwise<16, true>), dim3(nwg), dim3(threads), lds, s, B, tile_chunks);
        else hipLaunchKernelGGL((k_refine_kernelwise<16, false>), dim3(nwg), dim3(threads), lds, s, B, tile_chunks);
    } else {
        if (xf) hipLaunchKernelGGL((k_refine_kernelwise<kChunk, true>), dim3(nwg), dim3(threads), lds, s, B, tile_chunks);
        else hipLaunchKernelGGL((k_refine_kernelwise<kChunk, false>), dim3(nwg), dim3(threads), lds, s, B, tile_chunks);
    }
    trace_mark(s, cls == 0 ? MMSE_STAGE_W_REFINE_SMALL : MMSE_STAGE_W_REFINE);
    return hipGetLastError() == hipSuccess ? MMSE_OK : MMSE_ERR_LAUNCH;
}

// The stages for a list of tensors (already validated): sweep, refinement, codes; one launch per stage for up to
// kMaxBatch tensors (kMaxBatchExt when the call uses the extension fields), groups of that many beyond.
int run_weight_tensors(Item* items, int count, const mmse_params_t* p, bool do_search, hipStream_t s)
{
    const int G = p->grid_points;
    const int C = pick_cands(p);
    // largest kernels first: the hardware dispatcher hands out workgroups in order, so the
    // long ones start early and the short ones fill the tail.
    for (int i = 1; i < count; ++i) {
        Item it = items[i];
        int j = i - 1;
        while (j >= 0 && items[j].a.n < it.a.n) { items[j + 1] = items[j]; --j; }
        items[j + 1] = it;
    }
    int max_n = 0;
    bool any_small = false, xf = false;
    for (int i = 0; i < count; ++i) {
        max_n = items[i].a.n > max_n ? items[i].a.n : max_n;
        any_small = any_small || items[i].a.n <= kChunk;
        xf = xf || items[i].a.scale1 != nullptr || items[i].a.sub_packed != nullptr;
    }
    WeightShape sh{};
    sh.waves = (G + 64 * C - 1) / (64 * C);
    sh.do_search = do_search ? 1 : 0;
    sh.iters = p->refine_iters;
    // A call of few kernels is a chain of dependent launches that mostly wait for each other; then one launch does
    // the whole search (k_sweep_kernelwise, FUSED): every kernel must fit one LDS tile and have at most as many
    // chunks as a sweep workgroup has lanes.
    long long sumK = 0, sumKn = 0;
    for (int i = 0; i < count; ++i) { sumK += items[i].a.K; sumKn += (long long)items[i].a.K * items[i].a.n; }
    sh.fused = (do_search && sumK <= kFusedMaxKernels && sumKn <= kFusedMaxElements && max_n <= kTile &&
                (max_n + kChunk - 1) / kChunk <= 64 * sh.waves) ? 1 : 0;
    // tiny kernels take the one-wave-per-kernel path inside the sweep launch, when that variant is compiled for this
    // grid and no kernel of the call needs more than the short binary counter
    sh.CS = (!sh.fused && any_small && max_n <= kTile) ? small_cs(C, G) : 0;

    // sweep launch: LDS for the longest kernel that is staged whole (chunks padded apart in the fused search), or
    // the streaming tile of the longer ones
    auto sweep_lds = [&](const TensorArgs& a) -> int {
        if (sh.CS > 0 && a.n <= kChunk) return 0;
        const int npad = (a.n + kChunk - 1) & ~(kChunk - 1);
        if (sh.fused) return npad / kChunk * (kChunk + 4);
        return npad <= kTile ? npad : kTileStream;
    };

    long long totals[ST_COUNT] = {};
    for (int st = 0; st < ST_COUNT; ++st)
        for (int i = 0; i < count; ++i)
            totals[st] += stage_wgs(st, items[i].a.K, items[i].a.n, items[i].a.packed != nullptr, sh);
    bool has_ext = false;
    for (int i = 0; i < count; ++i) {
        const TensorArgs& a = items[i].a;
        has_ext = has_ext || a.grid_sse || a.sub_packed || a.sub_scale || a.active;
    }
    const int cap = has_ext ? kMaxBatchExt : kMaxBatch;
    for (int st = 0; st < ST_COUNT; ++st) {
        if (totals[st] == 0) continue;
        Batch B{};
        fill_common(B, p);
        B.has_ext = has_ext ? 1 : 0;
        int nb = 0, wg = 0, lds_floats = 0, gmax_n = 0;
        bool gxf = false;
        auto flush = [&]() -> int {
            if (nb == 0) return MMSE_OK;
            B.start[nb] = wg;
            B.count = nb;
            B.fused_part_off = lds_floats;
            WeightShape gsh = sh;
            const int chunks = ((gmax_n + kChunk - 1) & ~(kChunk - 1)) / kChunk;
            const int rc = launch_stage(st, B, wg, C, gsh, lds_floats, chunks, gxf, s);
            nb = 0; wg = 0; lds_floats = 0; gmax_n = 0; gxf = false;
            return rc;
        };
        for (int i = 0; i < count; ++i) {
            const TensorArgs& a = items[i].a;
            const long long add = stage_wgs(st, a.K, a.n, a.packed != nullptr, sh);
            if (add == 0) continue;
            if (nb > 0 && wg + add > kMaxLaunchWG) { const int rc = flush(); if (rc) return rc; }
            B.t[nb] = TensorCore{a.w, a.scale1, a.scale, a.idx, a.sse, a.absmax, a.packed, a.K, a.n};
            if (has_ext) B.e[nb] = TensorExt{a.grid_sse, a.sub_packed, a.sub_scale, a.active};
            B.start[nb] = wg;
            wg += (int)add;
            const int l = sweep_lds(a);
            lds_floats = l > lds_floats ? l : lds_floats;
            gmax_n = a.n > gmax_n ? a.n : gmax_n;
            gxf = gxf || a.scale1 != nullptr || a.sub_packed != nullptr;
            if (++nb == cap) { const int rc = flush(); if (rc) return rc; }
        }
        const int rc = flush();
        if (rc) return rc;
    }
    return MMSE_OK;
}

struct ActPlan {
    int count;
    int start[kMaxActBatch + 1];   // first block of each tensor in the concatenated numbering
    int levels;             // reduce64 stages of the grid sums until every tensor has <= 64 rows
    int plevels;            // reduce64 stages of the probe sums until every tensor has <= 4096 rows
    int total_rows[8];      // rows of all tensors together at each level
    size_t off_part[8];     // byte offsets of the grid-sum levels ([rows][G] doubles)
    size_t off_probe[8];    // byte offsets of the probe levels ([rows][kMaxProbes] doubles); only the columns below a
                            // tensor's nprobe are written in a pass, and only those are read
    size_t off_compact;     // with a refinement: every block as k_act_sweep staged it, 4096 floats each, and
    size_t off_meta;        // 64 words each that say where its chunks are (k_act_probe reads these)
    size_t bytes;
};

// Workspace of one launch group: the states, then the levels of the grid sums, then those of the probe sums, then
// (when the search refines: iters > 0) the compacted copy of the tensors for the refinement passes.
ActPlan plan_activation(const long long* N, int count, int G, int iters)
{
    ActPlan P{};
    P.count = count;
    int maxnb = 1;
    for (int t = 0; t < count; ++t) {
        const int nb = (int)((N[t] + kBlockElems - 1) / kBlockElems);
        P.start[t + 1] = P.start[t] + nb;
        maxnb = nb > maxnb ? nb : maxnb;
    }
    while (act_rows(maxnb, P.levels) > 64) ++P.levels;          // k_act_argmin takes the last <= 64 rows itself
    while (act_rows(maxnb, P.plevels) > 4096) ++P.plevels;      // k_act_finish takes the last <= 4096 rows itself
    for (int l = 0; l <= P.levels; ++l) {
        int r = 0;
        for (int t = 0; t < count; ++t) r += act_rows(P.start[t + 1] - P.start[t], l);
        P.total_rows[l] = r;
    }
    size_t off = round256(sizeof(ActState) * (size_t)count);
    for (int l = 0; l <= P.levels; ++l) { P.off_part[l] = off; off += round256((size_t)P.total_rows[l] * G * sizeof(double)); }
    for (int l = 0; l <= P.plevels; ++l) { P.off_probe[l] = off; off += round256((size_t)P.total_rows[l] * kMaxProbes * sizeof(double)); }
    if (iters > 0) {
        P.off_compact = off; off += (size_t)P.start[count] * kBlockElems * sizeof(float);
        P.off_meta = off; off += round256((size_t)P.start[count] * kBlockChunks * sizeof(unsigned));
    }
    P.bytes = off;
    return P;
}

// passes over the tensor that the refinement needs: the first settles 4 evaluations, each later one 3
int refine_passes(int iters)
{
    if (iters <= 0) return 0;
    return 1 + (iters > 2 ? (iters - 2 + 2) / 3 : 0);
}

// The tensors of a batched activation call are searched in launch groups: at most kMaxActBatch tensors and at
// most kMaxLaunchWG blocks each (one tensor alone has at most 2^19 blocks).  Returns how many tensors the group
// that starts at tensor `first` takes; N_of(i) is the size of tensor i.
template <class SizeOf>
int act_group_size(int first, int count, SizeOf N_of)
{
    int m = 0;
    long long blocks = 0;
    while (first + m < count && m < kMaxActBatch) {
        const long long nb = ((long long)N_of(first + m) + kBlockElems - 1) / kBlockElems;
        if (m > 0 && blocks + nb > kMaxLaunchWG) break;
        blocks += nb;
        ++m;
    }
    return m;
}

// Scratch of mmse_scale_search_kernelwise_noalloc: one abs-max per kernel.  Every GPU the library runs on holds
// its own copy of the array, at its own address, until the process ends.
static __device__ __align__(256) float scratch[MMSE_NOALLOC_MAX_KERNELS];

constexpr int kMaxDevices = 64;
std::atomic<float*> scratch_ptr[kMaxDevices];       // per device: the array's address there, once known

int scratch_address(float** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MMSE_ERR_LAUNCH;
    float* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        void* sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return MMSE_ERR_LAUNCH;
        ptr = static_cast<float*>(sym);
        scratch_ptr[dev].store(ptr, std::memory_order_release);    // two threads racing here store the same value
    }
    *out = ptr;
    return MMSE_OK;
}

struct DualPlan {           // workspace of dual_quantize_alternating, byte offsets
    size_t absmax, idx, ts1, ts2, tsse1, tsse, active, accepted, tp1, tp2, bytes;
};

DualPlan plan_dual(long long K, long long n)
{
    DualPlan P{};
    const size_t nb = (size_t)((K * n + 1) / 2);
    size_t off = 0;
    P.absmax = off; off += round256((size_t)K * sizeof(float));
    P.idx = off; off += round256((size_t)K * sizeof(int32_t));
    P.ts1 = off; off += round256((size_t)K * sizeof(float));
    P.ts2 = off; off += round256((size_t)K * sizeof(float));
    P.tsse1 = off; off += round256((size_t)K * sizeof(double));
    P.tsse = off; off += round256((size_t)K * sizeof(double));
    P.active = off; off += round256((size_t)K);
    P.accepted = off; off += round256((size_t)K);
    P.tp1 = off; off += round256(nb);
    P.tp2 = off; off += round256(nb);
    P.bytes = off;
    return P;
}

}  // namespace


// ---------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------
extern "C" {

const char* mmse_status_string(int status)
{
    switch (status) {
        case MMSE_OK: return "ok";
        case MMSE_ERR_NULL: return "a required pointer is NULL";
        case MMSE_ERR_SIZE: return "tensor size is not positive or exceeds the documented limits";
        case MMSE_ERR_PARAMS: return "bad quantization range, grid size, refinement count or tuning value";
        case MMSE_ERR_WORKSPACE: return "workspace is NULL, misaligned or too small";
        case MMSE_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
        case MMSE_ERR_ALIGN: return "a device pointer is not aligned to its element type";
        case MMSE_ERR_HOST_MEMORY: return "host memory for the call's descriptor tables could not be allocated";
        default: return "unknown status";
    }
}

int mmse_workspace_bytes_kernelwise(int64_t K, int64_t n, const mmse_params_t* p, size_t* bytes_out)
{
    if (!bytes_out) return MMSE_ERR_NULL;
    const int rc = check_params(p);
    if (rc) return rc;
    if (K <= 0 || n <= 0 || K > MMSE_MAX_TENSOR_ELEMS) return MMSE_ERR_SIZE;
    *bytes_out = round256((size_t)K * sizeof(float));
    return MMSE_OK;
}

int mmse_workspace_bytes_activation(int64_t N, const mmse_params_t* p, size_t* bytes_out)
{
    if (!bytes_out) return MMSE_ERR_NULL;
    const int rc = check_params(p);
    if (rc) return rc;
    if (N <= 0 || N > MMSE_MAX_TENSOR_ELEMS) return MMSE_ERR_SIZE;
    const long long n1 = N;
    *bytes_out = plan_activation(&n1, 1, p->grid_points, p->refine_iters).bytes;
    return MMSE_OK;
}

int mmse_workspace_bytes_activation_batched(const int64_t* N_host, int32_t count, const mmse_params_t* p, size_t* bytes_out)
{
    if (!bytes_out || !N_host) return MMSE_ERR_NULL;
    const int rc = check_params(p);
    if (rc) return rc;
    if (count <= 0 || count > MMSE_MAX_BATCH_TENSORS) return MMSE_ERR_SIZE;
    for (int i = 0; i < count; ++i)
        if (N_host[i] <= 0 || N_host[i] > MMSE_MAX_TENSOR_ELEMS) return MMSE_ERR_SIZE;
    size_t total = 0;
    for (int g0 = 0; g0 < count;) {
        const int m = act_group_size(g0, count, [&](int i) { return N_host[i]; });
        long long n[kMaxActBatch];
        for (int i = 0; i < m; ++i) n[i] = N_host[g0 + i];
        total += plan_activation(n, m, p->grid_points, p->refine_iters).bytes;
        g0 += m;
    }
    *bytes_out = total;
    return MMSE_OK;
}

int mmse_scale_search_batched(const mmse_tensor_desc_t* descs_host, int32_t count, const mmse_params_t* p,
                              void* ws_dev, size_t ws_bytes, void* stream)
{
    int rc = check_params(p);
    if (rc) return rc;
    if (!descs_host) return MMSE_ERR_NULL;
    if (count <= 0 || count > 4096) return MMSE_ERR_SIZE;
    long long sumK = 0;
    for (int i = 0; i < count; ++i) {
        rc = check_tensor(descs_host[i], true);
        if (rc) return rc;
        sumK += descs_host[i].K;
    }
    const size_t absmax_bytes = round256((size_t)sumK * sizeof(float));
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < absmax_bytes) return MMSE_ERR_WORKSPACE;
    // the host-side table: on the stack for up to kStackItems tensors, else temporary host memory
    constexpr int kStackItems = 64;
    Item stack_items[kStackItems] = {};
    Item* items = stack_items;
    if (count > kStackItems) {
        items = new (std::nothrow) Item[count]();       // value-initialised: every optional pointer starts as nullptr
        if (!items) return MMSE_ERR_HOST_MEMORY;
    }
    float* ws = static_cast<float*>(ws_dev);
    long long off = 0;
    for (int i = 0; i < count; ++i) {
        const mmse_tensor_desc_t& d = descs_host[i];
        TensorArgs& a = items[i].a;
        a.w = d.w_dev; a.scale1 = d.scale1_dev; a.scale = d.scale_dev; a.idx = d.idx_dev; a.sse = d.sse_dev;
        a.absmax = ws + off; a.grid_sse = nullptr; a.packed = d.packed_dev;
        a.sub_packed = nullptr; a.sub_scale = nullptr; a.active = nullptr;
        a.K = (int)d.K; a.n = (int)d.n;
        items[i].order = i;
        off += d.K;
    }
    rc = run_weight_tensors(items, count, p, true, static_cast<hipStream_t>(stream));
    if (items != stack_items) delete[] items;
    return rc;
}

int mmse_scale_search_kernelwise(const float* w_dev, int64_t K, int64_t n, const mmse_params_t* p,
                                 float* scale_dev, int32_t* idx_dev, double* sse_dev,
                                 void* ws_dev, size_t ws_bytes, void* stream)
{
    mmse_tensor_desc_t d{};
    d.w_dev = w_dev; d.K = K; d.n = n; d.scale1_dev = nullptr;
    d.scale_dev = scale_dev; d.idx_dev = idx_dev; d.sse_dev = sse_dev; d.packed_dev = nullptr;
    return mmse_scale_search_batched(&d, 1, p, ws_dev, ws_bytes, stream);
}

// For callers that cannot allocate: the per-kernel abs-max that the sweep hands to the refinement lives in the
// file-scope device array `scratch` instead of a caller's workspace.  Host code never uses the array's name as
// an address: scratch_address() asks the runtime for the array's address on the current device, once per device.
int mmse_scale_search_kernelwise_noalloc(const float* w_dev, int64_t K, int64_t n, const mmse_params_t* p,
                                         float* scale_dev, int32_t* idx_dev, double* sse_dev, void* stream)
{
    // every argument check of the plain entry point first, so that a bad call fails the same way without a GPU
    int rc = check_params(p);
    if (rc) return rc;
    mmse_tensor_desc_t d{};
    d.w_dev = w_dev; d.K = K; d.n = n; d.scale_dev = scale_dev; d.idx_dev = idx_dev; d.sse_dev = sse_dev;
    rc = check_tensor(d, true);
    if (rc) return rc;
    if (K > MMSE_NOALLOC_MAX_KERNELS) return MMSE_ERR_SIZE;
    float* ptr = nullptr;
    rc = scratch_address(&ptr);
    if (rc) return rc;
    return mmse_scale_search_kernelwise(w_dev, K, n, p, scale_dev, idx_dev, sse_dev, ptr,
                                        sizeof(float) * (size_t)MMSE_NOALLOC_MAX_KERNELS, stream);
}

int residual_quantize(const float* w_dev, int64_t K, int64_t n, const float* scale1_dev,
                      const mmse_params_t* p, float* scale2_dev, int32_t* idx2_dev, double* sse2_dev,
                      uint8_t* packed2_dev, void* ws_dev, size_t ws_bytes, void* stream)
{
    if (!scale1_dev) return MMSE_ERR_NULL;
    mmse_tensor_desc_t d{};
    d.w_dev = w_dev; d.K = K; d.n = n; d.scale1_dev = scale1_dev;
    d.scale_dev = scale2_dev; d.idx_dev = idx2_dev; d.sse_dev = sse2_dev; d.packed_dev = packed2_dev;
    return mmse_scale_search_batched(&d, 1, p, ws_dev, ws_bytes, stream);
}

int quantize_pack_int4(const float* x_dev, int64_t K, int64_t n, const float* scale_dev,
                       int32_t qmin, int32_t qmax, uint8_t* packed_dev, void* stream)
{
    if (!x_dev || !scale_dev || !packed_dev) return MMSE_ERR_NULL;
    if (K <= 0 || n <= 0 || K > MMSE_MAX_TENSOR_ELEMS / n) return MMSE_ERR_SIZE;
    if (!(qmin <= 0 && qmax > 0 && qmax - qmin <= 15)) return MMSE_ERR_PARAMS;
    if (!aligned_to(x_dev, 4) || !aligned_to(scale_dev, 4)) return MMSE_ERR_ALIGN;
    mmse_params_t p{qmin, qmax, 1, 0, 0};
    Item it{};
    it.a.w = x_dev; it.a.scale = const_cast<float*>(scale_dev); it.a.packed = packed_dev;
    it.a.K = (int)K; it.a.n = (int)n;
    // the pack kernel indexes by flat element, so any n is fine here (one activation tensor is K = 1)
    return run_weight_tensors(&it, 1, &p, false, static_cast<hipStream_t>(stream));
}

int mmse_grid_sse_kernelwise(const float* w_dev, int64_t K, int64_t n, const mmse_params_t* p,
                             float* absmax_dev, double* grid_sse_dev, void* stream)
{
    int rc = check_params(p);
    if (rc) return rc;
    if (!w_dev || !absmax_dev || !grid_sse_dev) return MMSE_ERR_NULL;
    mmse_tensor_desc_t d{};
    d.w_dev = w_dev; d.K = K; d.n = n;
    rc = check_tensor(d, false);
    if (rc) return rc;
    if (!aligned_to(absmax_dev, 4) || !aligned_to(grid_sse_dev, 8)) return MMSE_ERR_ALIGN;
    mmse_params_t q = *p;
    q.refine_iters = 0;
    Item it{};
    it.a.w = w_dev; it.a.absmax = absmax_dev; it.a.grid_sse = grid_sse_dev;
    it.a.K = (int)K; it.a.n = (int)n;
    return run_weight_tensors(&it, 1, &q, true, static_cast<hipStream_t>(stream));
}

int mmse_workspace_bytes_dual(int64_t K, int64_t n, const mmse_params_t* p, size_t* bytes_out)
{
    if (!bytes_out) return MMSE_ERR_NULL;
    const int rc = check_params(p);
    if (rc) return rc;
    if (K <= 0 || n <= 0 || n > MMSE_MAX_KERNEL_ELEMS || K > MMSE_MAX_TENSOR_ELEMS / n || K > MMSE_MAX_KERNELS) return MMSE_ERR_SIZE;
    *bytes_out = plan_dual(K, n).bytes;
    return MMSE_OK;
}

int dual_quantize_alternating_batched(const mmse_dual_desc_t* descs_host, int32_t count, const mmse_params_t* p,
                                      double eps, int32_t max_sweeps, void* ws_dev, size_t ws_bytes, void* stream)
{
    int rc = check_params(p);
    if (rc) return rc;
    if (!descs_host) return MMSE_ERR_NULL;
    if (count <= 0 || count > 4096) return MMSE_ERR_SIZE;
    if (!(eps >= 0.0) || max_sweeps < 1 || max_sweeps > 64) return MMSE_ERR_PARAMS;
    size_t need = 0;
    for (int i = 0; i < count; ++i) {
        const mmse_dual_desc_t& d = descs_host[i];
        if (!d.w_dev || !d.scale1_dev || !d.scale2_dev || !d.packed1_dev || !d.packed2_dev || !d.sse_dev || !d.sweeps_dev)
            return MMSE_ERR_NULL;
        if (d.K <= 0 || d.n <= 0 || d.n > MMSE_MAX_KERNEL_ELEMS || d.K > MMSE_MAX_TENSOR_ELEMS / d.n || d.K > MMSE_MAX_KERNELS) return MMSE_ERR_SIZE;
        if (!aligned_to(d.w_dev, 4) || !aligned_to(d.scale1_dev, 4) || !aligned_to(d.scale2_dev, 4) ||
            !aligned_to(d.sse_dev, 8) || !aligned_to(d.sweeps_dev, 4))
            return MMSE_ERR_ALIGN;
        need += plan_dual(d.K, d.n).bytes;
    }
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < need) return MMSE_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    struct W { float* absmax; int32_t* idx; float *ts1, *ts2; double *tsse1, *tsse; uint8_t *active, *accepted, *tp1, *tp2; };
    W* wk = new (std::nothrow) W[count]();
    Item* items = new (std::nothrow) Item[count]();
    if (!wk || !items) { delete[] wk; delete[] items; return MMSE_ERR_HOST_MEMORY; }
    {
        char* ws = static_cast<char*>(ws_dev);
        for (int i = 0; i < count; ++i) {
            const DualPlan P = plan_dual(descs_host[i].K, descs_host[i].n);
            wk[i].absmax = reinterpret_cast<float*>(ws + P.absmax);
            wk[i].idx = reinterpret_cast<int32_t*>(ws + P.idx);
            wk[i].ts1 = reinterpret_cast<float*>(ws + P.ts1);
            wk[i].ts2 = reinterpret_cast<float*>(ws + P.ts2);
            wk[i].tsse1 = reinterpret_cast<double*>(ws + P.tsse1);
            wk[i].tsse = reinterpret_cast<double*>(ws + P.tsse);
            wk[i].active = reinterpret_cast<uint8_t*>(ws + P.active);
            wk[i].accepted = reinterpret_cast<uint8_t*>(ws + P.accepted);
            wk[i].tp1 = reinterpret_cast<uint8_t*>(ws + P.tp1);
            wk[i].tp2 = reinterpret_cast<uint8_t*>(ws + P.tp2);
            ws += P.bytes;
        }
    }
    // one phi for every tensor: which = 0 first sweep j=1, 1 first sweep j=2, 2 later sweep j=1, 3 later sweep j=2
    auto fit = [&](int which) -> int {
        for (int i = 0; i < count; ++i) {
            const mmse_dual_desc_t& d = descs_host[i];
            TensorArgs a{};
            a.w = d.w_dev; a.idx = wk[i].idx; a.absmax = wk[i].absmax; a.K = (int)d.K; a.n = (int)d.n;
            if (which == 0) { a.scale = d.scale1_dev; a.sse = wk[i].tsse1; a.packed = d.packed1_dev; }
            if (which == 1) { a.sub_packed = d.packed1_dev; a.sub_scale = d.scale1_dev;
                              a.scale = d.scale2_dev; a.sse = d.sse_dev; a.packed = d.packed2_dev; }
            if (which == 2) { a.sub_packed = d.packed2_dev; a.sub_scale = d.scale2_dev; a.active = wk[i].active;
                              a.scale = wk[i].ts1; a.sse = wk[i].tsse1; a.packed = wk[i].tp1; }
            if (which == 3) { a.sub_packed = wk[i].tp1; a.sub_scale = wk[i].ts1; a.active = wk[i].active;
                              a.scale = wk[i].ts2; a.sse = wk[i].tsse; a.packed = wk[i].tp2; }
            items[i].a = a;
            items[i].order = i;
        }
        return run_weight_tensors(items, count, p, true, s);
    };
    // bookkeeping kernels over all tensors: kind 0 init, 1 accept, 2 copy codes
    auto book = [&](int kind) -> int {
        int b0 = 0;
        while (b0 < count) {
            DualBatch D{};
            D.eps = eps;
            int nb = 0;
            long long wg = 0;
            while (b0 + nb < count && nb < kMaxDualBatch) {
                const mmse_dual_desc_t& d = descs_host[b0 + nb];
                const long long units = kind == 2 ? (((long long)d.K * d.n + 1) / 2 + 15) / 16 : d.K;   // 16 bytes of codes, or one kernel, per thread
                const long long add = (units + 255) / 256;
                if (nb > 0 && wg + add > kMaxLaunchWG) break;          // the rest goes into the next launch
                const W& w = wk[b0 + nb];
                DualTensor& T = D.t[nb];
                T.sse = d.sse_dev; T.tsse = w.tsse; T.s1 = d.scale1_dev; T.ts1 = w.ts1; T.s2 = d.scale2_dev; T.ts2 = w.ts2;
                T.sweeps = d.sweeps_dev; T.active = w.active; T.accepted = w.accepted;
                T.tp1 = w.tp1; T.p1 = d.packed1_dev; T.tp2 = w.tp2; T.p2 = d.packed2_dev;
                T.K = (int)d.K; T.n = (int)d.n;
                D.start[nb] = (int)wg;
                wg += add;
                ++nb;
            }
            D.start[nb] = (int)wg;
            D.count = nb;
            if (kind == 0) hipLaunchKernelGGL(k_dual_init, dim3((unsigned)wg), dim3(256), 0, s, D);
            else if (kind == 1) hipLaunchKernelGGL(k_dual_accept, dim3((unsigned)wg), dim3(256), 0, s, D);
            else hipLaunchKernelGGL(k_dual_copy_codes, dim3((unsigned)wg), dim3(256), 0, s, D);
            if (hipGetLastError() != hipSuccess) return MMSE_ERR_LAUNCH;
            b0 += nb;
        }
        return MMSE_OK;
    };

    // first sweep, from an empty second tensor: the plain fit, then the fit of what it leaves
    rc = fit(0);
    if (!rc) rc = fit(1);
    if (!rc) rc = book(0);
    for (int sweep = 1; sweep < max_sweeps && !rc; ++sweep) {
        rc = fit(2);                    // j = 1: T - a2*Q2
        if (!rc) rc = fit(3);           // j = 2: T - a1*Q1
        if (!rc) rc = book(1);
        if (!rc) rc = book(2);
    }
    delete[] items;
    delete[] wk;
    return rc;
}

int mmse_workspace_bytes_dual_batched(const mmse_dual_desc_t* descs_host, int32_t count, const mmse_params_t* p,
                                      size_t* bytes_out)
{
    if (!bytes_out || !descs_host) return MMSE_ERR_NULL;
    const int rc = check_params(p);
    if (rc) return rc;
    if (count <= 0 || count > 4096) return MMSE_ERR_SIZE;
    size_t need = 0;
    for (int i = 0; i < count; ++i) {
        const mmse_dual_desc_t& d = descs_host[i];
        if (d.K <= 0 || d.n <= 0 || d.n > MMSE_MAX_KERNEL_ELEMS || d.K > MMSE_MAX_TENSOR_ELEMS / d.n || d.K > MMSE_MAX_KERNELS) return MMSE_ERR_SIZE;
        need += plan_dual(d.K, d.n).bytes;
    }
    *bytes_out = need;
    return MMSE_OK;
}

int dual_quantize_alternating(const float* w_dev, int64_t K, int64_t n, const mmse_params_t* p,
                              double eps, int32_t max_sweeps,
                              float* scale1_dev, float* scale2_dev, uint8_t* packed1_dev, uint8_t* packed2_dev,
                              double* sse_dev, int32_t* sweeps_dev, void* ws_dev, size_t ws_bytes, void* stream)
{
    mmse_dual_desc_t d{};
    d.w_dev = w_dev; d.K = K; d.n = n; d.scale1_dev = scale1_dev; d.scale2_dev = scale2_dev;
    d.packed1_dev = packed1_dev; d.packed2_dev = packed2_dev; d.sse_dev = sse_dev; d.sweeps_dev = sweeps_dev;
    return dual_quantize_alternating_batched(&d, 1, p, eps, max_sweeps, ws_dev, ws_bytes, stream);
}

static int dual_ls_waves(int G1, int G2)
{
    const int units = (G1 * G2 + 63) / 64;
    return units < 8 ? units : 8;
}

static int dual_ls_splits(int64_t K, int G1, int G2)
{
    // enough workgroups to give every SIMD about four waves, but never more splits than units per wave
    const int units = (G1 * G2 + 63) / 64, nw = dual_ls_waves(G1, G2);
    long long want = (4096 + K * nw - 1) / (K * nw);
    const int cap = (units + nw - 1) / nw;
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    return (int)want;
}

int mmse_layer_error_sums(const double* const* sse_dev_ptrs_host, const int64_t* K_host, int32_t count,
                          double* sums_dev, void* stream)
{
    if (!sse_dev_ptrs_host || !K_host || !sums_dev) return MMSE_ERR_NULL;
    if (count <= 0 || count > MMSE_MAX_BATCH_TENSORS) return MMSE_ERR_SIZE;
    if (!aligned_to(sums_dev, 8)) return MMSE_ERR_ALIGN;
    for (int i = 0; i < count; ++i) {
        if (!sse_dev_ptrs_host[i]) return MMSE_ERR_NULL;
        if (K_host[i] <= 0 || K_host[i] > MMSE_MAX_TENSOR_ELEMS) return MMSE_ERR_SIZE;
        if (!aligned_to(sse_dev_ptrs_host[i], 8)) return MMSE_ERR_ALIGN;
    }
    for (int g0 = 0; g0 < count; g0 += kMaxSumBatch) {
        SumBatch B{};
        const int m = (count - g0) < kMaxSumBatch ? (count - g0) : kMaxSumBatch;
        for (int i = 0; i < m; ++i) { B.v[i] = sse_dev_ptrs_host[g0 + i]; B.n[i] = (int)K_host[g0 + i]; }
        hipLaunchKernelGGL(k_layer_sums, dim3(m), dim3(256), 0, static_cast<hipStream_t>(stream), B, sums_dev + g0);
        if (hipGetLastError() != hipSuccess) return MMSE_ERR_LAUNCH;
    }
    return MMSE_OK;
}

int mmse_scale_alternating_kernelwise(const float* w_dev, int64_t K, int64_t n, int32_t qmin, int32_t qmax,
                                      int32_t max_iters, float* scale_dev, double* sse_dev, int32_t* updates_dev,
                                      void* stream)
{
    if (!w_dev || !scale_dev || !sse_dev || !updates_dev) return MMSE_ERR_NULL;
    if (K <= 0 || n <= 0 || n > MMSE_MAX_KERNEL_ELEMS || K > MMSE_MAX_TENSOR_ELEMS / n || K > MMSE_MAX_KERNELS) return MMSE_ERR_SIZE;
    if (!(qmin <= 0 && qmax > 0 && qmax - qmin <= 15) || max_iters < 0 || max_iters > 1000) return MMSE_ERR_PARAMS;
    if (!aligned_to(w_dev, 4) || !aligned_to(scale_dev, 4) || !aligned_to(sse_dev, 8) || !aligned_to(updates_dev, 4))
        return MMSE_ERR_ALIGN;
    const int nchunks = (int)((n + kChunk - 1) / kChunk);
    const unsigned nthr = nchunks <= 64 ? 64u : 256u;
    hipLaunchKernelGGL(k_alt_kernelwise, dim3((unsigned)K), dim3(nthr), 0, static_cast<hipStream_t>(stream),
                       w_dev, (int)n, qmax, (float)qmin, (float)qmax, max_iters, scale_dev, sse_dev, updates_dev);
    if (hipGetLastError() != hipSuccess) return MMSE_ERR_LAUNCH;
    return MMSE_OK;
}

int mmse_workspace_bytes_dual_linesearch(int64_t K, int64_t n, int32_t G1, int32_t G2, size_t* bytes_out)
{
    if (!bytes_out) return MMSE_ERR_NULL;
    if (K <= 0 || n <= 0 || n > kTile || K > MMSE_MAX_TENSOR_ELEMS / n || K > MMSE_MAX_KERNELS) return MMSE_ERR_SIZE;
    if (G1 < 1 || G2 < 1 || G1 > 1024 || G2 > 1024) return MMSE_ERR_PARAMS;
    const int sp = dual_ls_splits(K, G1, G2);
    *bytes_out = round256((size_t)K * sizeof(float)) + round256((size_t)K * sp * sizeof(double)) +
                 round256((size_t)K * sp * sizeof(int));
    return MMSE_OK;
}

int dual_line_search(const float* w_dev, int64_t K, int64_t n, int32_t qmin, int32_t qmax, int32_t G1, int32_t G2,
                     float* scale1_dev, float* scale2_dev, int32_t* idx1_dev, int32_t* idx2_dev, double* sse_dev,
                     uint8_t* packed1_dev, uint8_t* packed2_dev, double* grid_dev,
                     void* ws_dev, size_t ws_bytes, void* stream)
{
    if (!w_dev || !scale1_dev || !scale2_dev || !idx1_dev || !idx2_dev || !sse_dev || !packed1_dev || !packed2_dev)
        return MMSE_ERR_NULL;
    if (K <= 0 || n <= 0 || n > kTile || K > MMSE_MAX_TENSOR_ELEMS / n || K > MMSE_MAX_KERNELS) return MMSE_ERR_SIZE;
    if (!(qmin <= 0 && qmax > 0 && qmax - qmin <= 15)) return MMSE_ERR_PARAMS;
    if (G1 < 1 || G2 < 1 || G1 > 1024 || G2 > 1024) return MMSE_ERR_PARAMS;
    if (!aligned_to(w_dev, 4) || !aligned_to(scale1_dev, 4) || !aligned_to(scale2_dev, 4) || !aligned_to(idx1_dev, 4) ||
        !aligned_to(idx2_dev, 4) || !aligned_to(sse_dev, 8) || !aligned_to(grid_dev, 8))
        return MMSE_ERR_ALIGN;
    size_t need = 0;
    mmse_workspace_bytes_dual_linesearch(K, n, G1, G2, &need);
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < need) return MMSE_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    DualLsArgs A{};
    A.w = w_dev; A.K = (int)K; A.n = (int)n; A.G1 = G1; A.G2 = G2; A.splits = dual_ls_splits(K, G1, G2);
    A.qmin = qmin; A.qmax = qmax; A.lo = (float)qmin; A.hi = (float)qmax;
    char* ws = static_cast<char*>(ws_dev);
    A.absmax = reinterpret_cast<float*>(ws);
    ws += round256((size_t)K * sizeof(float));
    A.part_e = reinterpret_cast<double*>(ws);
    ws += round256((size_t)K * A.splits * sizeof(double));
    A.part_idx = reinterpret_cast<int*>(ws);
    A.grid = grid_dev;
    A.scale1 = scale1_dev; A.scale2 = scale2_dev; A.idx1 = idx1_dev; A.idx2 = idx2_dev; A.sse = sse_dev;
    A.packed1 = packed1_dev; A.packed2 = packed2_dev;
    const int npad = (int)((n + kChunk - 1) & ~(int64_t)(kChunk - 1));
    const size_t lds = (size_t)npad * sizeof(float);
    const unsigned nwg = (unsigned)(K * A.splits);
    const unsigned nthr = 64u * (unsigned)dual_ls_waves(G1, G2);
    if (qmax - qmin == 15) hipLaunchKernelGGL(k_dual_ls<true>, dim3(nwg), dim3(nthr), lds, s, A);
    else hipLaunchKernelGGL(k_dual_ls<false>, dim3(nwg), dim3(nthr), lds, s, A);
    if (hipGetLastError() != hipSuccess) return MMSE_ERR_LAUNCH;
    hipLaunchKernelGGL(k_dual_ls_pick, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, s, A);
    if (hipGetLastError() != hipSuccess) return MMSE_ERR_LAUNCH;
    const long long total = (long long)K * n, per_wg = (long long)kPackThreads * kPackPerThread;
    hipLaunchKernelGGL(k_dual_ls_codes, dim3((unsigned)((total + per_wg - 1) / per_wg)), dim3(kPackThreads), 0, s, A);
    if (hipGetLastError() != hipSuccess) return MMSE_ERR_LAUNCH;
    return MMSE_OK;
}

// The per-layer search for a group of at most kMaxActBatch tensors in one set of launches (arguments already
// validated).  pre_mode selects what is searched (the tensor, the residual of a first tensor, the tensor
// shifted by its minimum; the last two for a single tensor only); packed != nullptr also writes the codes.
struct ActItem { const float* x; long long N; float* scale; int32_t* idx; double* sse; uint8_t* packed; };

static int run_activation_group(const ActItem* items, int count, const mmse_params_t* p, int pre_mode,
                                const float* scale1_dev, int qmin1, int qmax1, float* delta_dev,
                                char* ws, const ActPlan& P, hipStream_t s,
                                float* absmax_out = nullptr, double* grid_out = nullptr)
{
    const int G = p->grid_points;
    ActBatch B{};
    ActOut O{};
    bool any_packed = false;
    long long maxN = 0, sumN = 0;
    for (int t = 0; t < count; ++t) {
        B.x[t] = items[t].x; B.N[t] = items[t].N; B.start[t] = P.start[t];
        O.scale[t] = items[t].scale; O.idx[t] = items[t].idx; O.sse[t] = items[t].sse; O.packed[t] = items[t].packed;
        any_packed = any_packed || items[t].packed != nullptr;
        maxN = items[t].N > maxN ? items[t].N : maxN;
        sumN += items[t].N;
    }
    B.start[count] = P.start[count];
    B.count = count;
    B.S = reinterpret_cast<ActState*>(ws);
    ActState* S = B.S;
    const int total = P.start[count];
    const float lo = (float)p->qmin, hi = (float)p->qmax;
    ActPre pre{};
    pre.mode = pre_mode;
    pre.s = pre_mode == 1 ? scale1_dev : (pre_mode == 2 ? &S->delta : nullptr);
    pre.lo1 = (float)qmin1; pre.hi1 = (float)qmax1;
#define MMSE_CHECK_LAUNCH(stage) do { if (hipGetLastError() != hipSuccess) return MMSE_ERR_LAUNCH; trace_mark(s, stage); } while (0)

    hipLaunchKernelGGL(k_act_init, dim3(1), dim3(64), 0, s, S, count);
    MMSE_CHECK_LAUNCH(MMSE_STAGE_A_INIT);
    {
        // 24 waves per CU over all tensors of the batch (each tensor in proportion to its size), eight non-temporal
        // 16-byte loads in flight per thread: measured fastest on MI355X for sets of tensors much larger than
        // the caches (6.9-7.0 TB/s on 0.58 and 1.4 GB; a third of the waves: 3.8, plain loads: 6.2)
        constexpr int U = 8;
        const long long per_wg = 4LL * kAbsmaxThreads * U;             // elements per workgroup and trip
        long long want = (maxN + per_wg - 1) / per_wg;
        long long cap = (384 * maxN + sumN - 1) / sumN;
        if (cap > 384) cap = 384;
        if (want > cap) want = cap;
        const int grid = (int)(want < 1 ? 1 : want);
        const dim3 g(grid, count);
        if (pre_mode == 0) hipLaunchKernelGGL((k_act_absmax<U, 0>), g, dim3(kAbsmaxThreads), 0, s, B, pre);
        else if (pre_mode == 1) hipLaunchKernelGGL((k_act_absmax<U, 1>), g, dim3(kAbsmaxThreads), 0, s, B, pre);
        else hipLaunchKernelGGL((k_act_absmax<U, 2>), g, dim3(kAbsmaxThreads), 0, s, B, pre);
        MMSE_CHECK_LAUNCH(MMSE_STAGE_A_ABSMAX);
        if (pre_mode == 2) {
            hipLaunchKernelGGL(k_act_offset_setup, dim3(1), dim3(64), 0, s, S, delta_dev);
            MMSE_CHECK_LAUNCH(MMSE_STAGE_A_ABSMAX);
        }
    }
    {
        // 129 ... 384 grid points, tuning left to the library: two candidates per lane and two sets of waves that
        // take half a block each (see k_act_sweep)
        const bool split = p->cands_per_lane == 0 && G > 128 && G <= kMaxSplitCands;
        const int C = split ? 2 : pick_cands(p);
        const int wps = (G + 64 * C - 1) / (64 * C);                  // waves that cover the grid once
        int sets = split ? 2 : 1;
        // a call of few blocks leaves most of the machine idle while every wave walks its whole block: more sets
        // of waves per block, each with a smaller part of it (up to eight waves a workgroup; same sums, same order)
        if (total <= kFewBlocks)
            while (sets < 8 && wps * sets * 2 <= 8 && sets * 2 * wps * 64 * C <= kMaxExchange) sets *= 2;
        const int waves = sets * wps;
        double* part0 = reinterpret_cast<double*>(ws + P.off_part[0]);
        float* compact = p->refine_iters > 0 ? reinterpret_cast<float*>(ws + P.off_compact) : nullptr;
        unsigned* meta = p->refine_iters > 0 ? reinterpret_cast<unsigned*>(ws + P.off_meta) : nullptr;
        if (C == 1) hipLaunchKernelGGL(k_act_sweep<1>, dim3(total), dim3(64 * waves), 0, s, B, G, p->qmax, lo, hi, part0, pre, sets, compact, meta);
        else if (C == 2) hipLaunchKernelGGL(k_act_sweep<2>, dim3(total), dim3(64 * waves), 0, s, B, G, p->qmax, lo, hi, part0, pre, sets, compact, meta);
        else hipLaunchKernelGGL(k_act_sweep<4>, dim3(total), dim3(64 * waves), 0, s, B, G, p->qmax, lo, hi, part0, pre, sets, compact, meta);
        MMSE_CHECK_LAUNCH(MMSE_STAGE_A_SWEEP);
    }
    for (int l = 0; l < P.levels; ++l) {
        hipLaunchKernelGGL(k_act_reduce64, dim3(P.total_rows[l + 1], (G + 255) / 256), dim3(256), 0, s, B, l + 1,
                           reinterpret_cast<const double*>(ws + P.off_part[l]), G,
                           reinterpret_cast<double*>(ws + P.off_part[l + 1]), 0);
        MMSE_CHECK_LAUNCH(MMSE_STAGE_A_REDUCE);
    }
    {
        int threads = ((G + 63) / 64) * 64;
        if (threads > 256) threads = 256;
        hipLaunchKernelGGL(k_act_argmin, dim3(count), dim3(threads), 0, s, B, P.levels,
                           reinterpret_cast<const double*>(ws + P.off_part[P.levels]), G, p->qmax, p->refine_iters, O,
                           absmax_out, grid_out);
        MMSE_CHECK_LAUNCH(MMSE_STAGE_A_ARGMIN);
    }
    for (int pass = 0; pass < refine_passes(p->refine_iters); ++pass) {
        hipLaunchKernelGGL(k_act_probe, dim3(total), dim3(256), 0, s, B, lo, hi,
                           reinterpret_cast<double*>(ws + P.off_probe[0]),
                           reinterpret_cast<const float*>(ws + P.off_compact),
                           reinterpret_cast<const unsigned*>(ws + P.off_meta));
        MMSE_CHECK_LAUNCH(MMSE_STAGE_A_PROBE);
        for (int l = 0; l < P.plevels; ++l) {
            hipLaunchKernelGGL(k_act_reduce64, dim3(P.total_rows[l + 1], 1), dim3(64), 0, s, B, l + 1,
                               reinterpret_cast<const double*>(ws + P.off_probe[l]), kMaxProbes,
                               reinterpret_cast<double*>(ws + P.off_probe[l + 1]), 1);
            MMSE_CHECK_LAUNCH(MMSE_STAGE_A_PROBE_REDUCE);
        }
        hipLaunchKernelGGL(k_act_finish, dim3(count), dim3(512), 0, s, B, P.plevels,
                           reinterpret_cast<const double*>(ws + P.off_probe[P.plevels]), p->refine_iters, O);
        MMSE_CHECK_LAUNCH(MMSE_STAGE_A_FINISH);
    }
    if (any_packed) {
        hipLaunchKernelGGL(k_act_pack, dim3(total), dim3(kPackThreads), 0, s, B, pre, O, lo, hi);
        MMSE_CHECK_LAUNCH(MMSE_STAGE_A_PACK);
    }
#undef MMSE_CHECK_LAUNCH
    return MMSE_OK;
}

static int run_activation(const float* x_dev, int64_t N, const mmse_params_t* p, int pre_mode,
                          const float* scale1_dev, int qmin1, int qmax1, float* delta_dev,
                          float* scale_dev, int32_t* idx_dev, double* sse_dev, uint8_t* packed_dev,
                          void* ws_dev, size_t ws_bytes, void* stream)
{
    int rc = check_params(p);
    if (rc) return rc;
    if (!x_dev || !scale_dev || !idx_dev || !sse_dev) return MMSE_ERR_NULL;
    if (N <= 0 || N > MMSE_MAX_TENSOR_ELEMS) return MMSE_ERR_SIZE;
    if (!aligned_to(x_dev, 4) || !aligned_to(scale_dev, 4) || !aligned_to(idx_dev, 4) || !aligned_to(sse_dev, 8))
        return MMSE_ERR_ALIGN;
    const long long n1 = N;
    const ActPlan P = plan_activation(&n1, 1, p->grid_points, p->refine_iters);
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < P.bytes) return MMSE_ERR_WORKSPACE;
    const ActItem item{x_dev, n1, scale_dev, idx_dev, sse_dev, packed_dev};
    return run_activation_group(&item, 1, p, pre_mode, scale1_dev, qmin1, qmax1, delta_dev,
                                static_cast<char*>(ws_dev), P, static_cast<hipStream_t>(stream));
}

int mmse_grid_sse_activation(const float* x_dev, int64_t N, const mmse_params_t* p, float* absmax_dev,
                             double* grid_sse_dev, void* ws_dev, size_t ws_bytes, void* stream)
{
    int rc = check_params(p);
    if (rc) return rc;
    if (!x_dev || !absmax_dev || !grid_sse_dev) return MMSE_ERR_NULL;
    if (N <= 0 || N > MMSE_MAX_TENSOR_ELEMS) return MMSE_ERR_SIZE;
    if (!aligned_to(x_dev, 4) || !aligned_to(absmax_dev, 4) || !aligned_to(grid_sse_dev, 8)) return MMSE_ERR_ALIGN;
    const long long n1 = N;
    mmse_params_t q = *p;
    q.refine_iters = 0;
    const ActPlan P = plan_activation(&n1, 1, q.grid_points, q.refine_iters);
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < P.bytes) return MMSE_ERR_WORKSPACE;
    ActState* S = reinterpret_cast<ActState*>(ws_dev);
    const ActItem item{x_dev, n1, &S->out_scale, &S->out_idx, &S->out_sse, nullptr};   // the search results stay in the workspace
    return run_activation_group(&item, 1, &q, 0, nullptr, 0, 0, nullptr, static_cast<char*>(ws_dev), P,
                                static_cast<hipStream_t>(stream), absmax_dev, grid_sse_dev);
}

int mmse_scale_search_activation_batched(const mmse_act_desc_t* descs_host, int32_t count, const mmse_params_t* p,
                                         void* ws_dev, size_t ws_bytes, void* stream)
{
    int rc = check_params(p);
    if (rc) return rc;
    if (!descs_host) return MMSE_ERR_NULL;
    if (count <= 0 || count > MMSE_MAX_BATCH_TENSORS) return MMSE_ERR_SIZE;
    for (int i = 0; i < count; ++i) {
        const mmse_act_desc_t& d = descs_host[i];
        if (!d.x_dev || !d.scale_dev || !d.idx_dev || !d.sse_dev) return MMSE_ERR_NULL;
        if (d.N <= 0 || d.N > MMSE_MAX_TENSOR_ELEMS) return MMSE_ERR_SIZE;
        if (!aligned_to(d.x_dev, 4) || !aligned_to(d.scale_dev, 4) || !aligned_to(d.idx_dev, 4) || !aligned_to(d.sse_dev, 8))
            return MMSE_ERR_ALIGN;
    }
    // launch groups, each with its own slice of the workspace: sized first, then run
    size_t need = 0;
    for (int g0 = 0; g0 < count;) {
        const int m = act_group_size(g0, count, [&](int i) { return descs_host[i].N; });
        long long n[kMaxActBatch];
        for (int i = 0; i < m; ++i) n[i] = descs_host[g0 + i].N;
        need += plan_activation(n, m, p->grid_points, p->refine_iters).bytes;
        g0 += m;
    }
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < need) return MMSE_ERR_WORKSPACE;
    char* ws = static_cast<char*>(ws_dev);
    for (int g0 = 0; g0 < count;) {
        const int m = act_group_size(g0, count, [&](int i) { return descs_host[i].N; });
        long long n[kMaxActBatch];
        ActItem items[kMaxActBatch];
        for (int i = 0; i < m; ++i) {
            const mmse_act_desc_t& d = descs_host[g0 + i];
            n[i] = d.N;
            items[i] = ActItem{d.x_dev, (long long)d.N, d.scale_dev, d.idx_dev, d.sse_dev, d.packed_dev};
        }
        const ActPlan P = plan_activation(n, m, p->grid_points, p->refine_iters);
        rc = run_activation_group(items, m, p, 0, nullptr, 0, 0, nullptr, ws, P, static_cast<hipStream_t>(stream));
        if (rc) return rc;
        ws += P.bytes;
        g0 += m;
    }
    return MMSE_OK;
}

// ---- measurement aid: per-kernel durations of a batched call from HIP events on its stream ----
int mmse_trace_create(int32_t capacity, mmse_trace_t** trace_out)
{
    if (!trace_out) return MMSE_ERR_NULL;
    *trace_out = nullptr;
    if (capacity < 2 || capacity > 4096) return MMSE_ERR_SIZE;
    mmse_trace* T = new (std::nothrow) mmse_trace{};
    if (!T) return MMSE_ERR_HOST_MEMORY;
    T->ev = new (std::nothrow) hipEvent_t[capacity]();
    T->stage = new (std::nothrow) int[capacity]();
    if (!T->ev || !T->stage) { delete[] T->ev; delete[] T->stage; delete T; return MMSE_ERR_HOST_MEMORY; }
    for (int i = 0; i < capacity; ++i) {
        if (hipEventCreate(&T->ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(T->ev[j]);
            delete[] T->ev; delete[] T->stage; delete T;
            return MMSE_ERR_LAUNCH;
        }
    }
    T->capacity = capacity;
    T->used = 0;
    *trace_out = T;
    return MMSE_OK;
}

void mmse_trace_destroy(mmse_trace_t* T)
{
    if (!T) return;
    for (int i = 0; i < T->capacity; ++i) (void)hipEventDestroy(T->ev[i]);
    delete[] T->ev;
    delete[] T->stage;
    delete T;
}

int mmse_trace_read(mmse_trace_t* T, int32_t capacity, int32_t* count_out, int32_t* stage_out, float* ms_out)
{
    if (!T || !count_out || !stage_out || !ms_out) return MMSE_ERR_NULL;
    const int n = T->used > 0 ? T->used - 1 : 0;          // event 0 precedes the first kernel
    if (capacity < n) return MMSE_ERR_SIZE;
    if (T->used > 0 && hipEventSynchronize(T->ev[T->used - 1]) != hipSuccess) return MMSE_ERR_LAUNCH;
    for (int i = 0; i < n; ++i) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, T->ev[i], T->ev[i + 1]) != hipSuccess) return MMSE_ERR_LAUNCH;
        stage_out[i] = T->stage[i + 1];
        ms_out[i] = ms;
    }
    *count_out = n;
    return MMSE_OK;
}

int mmse_scale_search_batched_traced(const mmse_tensor_desc_t* descs_host, int32_t count, const mmse_params_t* p,
                                     void* ws_dev, size_t ws_bytes, void* stream, mmse_trace_t* trace)
{
    if (!trace) return MMSE_ERR_NULL;
    trace->used = 0;
    t_trace = trace;
    trace_mark(static_cast<hipStream_t>(stream), MMSE_STAGE_START);
    const int rc = mmse_scale_search_batched(descs_host, count, p, ws_dev, ws_bytes, stream);
    t_trace = nullptr;
    return rc;
}

int mmse_scale_search_activation_batched_traced(const mmse_act_desc_t* descs_host, int32_t count, const mmse_params_t* p,
                                                void* ws_dev, size_t ws_bytes, void* stream, mmse_trace_t* trace)
{
    if (!trace) return MMSE_ERR_NULL;
    trace->used = 0;
    t_trace = trace;
    trace_mark(static_cast<hipStream_t>(stream), MMSE_STAGE_START);
    const int rc = mmse_scale_search_activation_batched(descs_host, count, p, ws_dev, ws_bytes, stream);
    t_trace = nullptr;
    return rc;
}

int mmse_scale_search_activation(const float* x_dev, int64_t N, const mmse_params_t* p,
                                 float* scale_dev, int32_t* idx_dev, double* sse_dev,
                                 void* ws_dev, size_t ws_bytes, void* stream)
{
    return run_activation(x_dev, N, p, 0, nullptr, 0, 0, nullptr, scale_dev, idx_dev, sse_dev, nullptr,
                          ws_dev, ws_bytes, stream);
}

int activation_residual_quantize(const float* x_dev, int64_t N, const float* scale1_dev, int32_t qmin1, int32_t qmax1,
                                 const mmse_params_t* p, float* scale2_dev, int32_t* idx2_dev, double* sse2_dev,
                                 uint8_t* packed2_dev, void* ws_dev, size_t ws_bytes, void* stream)
{
    if (!scale1_dev) return MMSE_ERR_NULL;
    if (!(qmin1 <= 0 && qmax1 > 0 && qmax1 - qmin1 <= 15)) return MMSE_ERR_PARAMS;
    if (!aligned_to(scale1_dev, 4)) return MMSE_ERR_ALIGN;
    return run_activation(x_dev, N, p, 1, scale1_dev, qmin1, qmax1, nullptr, scale2_dev, idx2_dev, sse2_dev,
                          packed2_dev, ws_dev, ws_bytes, stream);
}

int mmse_scale_search_offset(const float* x_dev, int64_t N, const mmse_params_t* p, float* delta_dev,
                             float* scale_dev, int32_t* idx_dev, double* sse_dev, uint8_t* packed_dev,
                             void* ws_dev, size_t ws_bytes, void* stream)
{
    if (!delta_dev) return MMSE_ERR_NULL;
    if (p && p->qmin != 0) return MMSE_ERR_PARAMS;           // Eq. 2 is stated for the unsigned range
    if (!aligned_to(delta_dev, 4)) return MMSE_ERR_ALIGN;
    return run_activation(x_dev, N, p, 2, nullptr, 0, 0, delta_dev, scale_dev, idx_dev, sse_dev, packed_dev,
                          ws_dev, ws_bytes, stream);
}

}  // extern "C"
