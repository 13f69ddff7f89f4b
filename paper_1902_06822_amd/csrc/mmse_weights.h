// mmse_weights.h -- kernel-wise weight path: grid sweep (general and one-wave-per-kernel), golden-section refinement, INT4 packing.
#ifndef MMSE_WEIGHTS_H_
#define MMSE_WEIGHTS_H_
#include "mmse_common.h"

namespace {

// ---------------------------------------------------------------------------------
// k_sweep_kernelwise: abs-max + grid sweep + argmin, one workgroup per weight kernel
// ---------------------------------------------------------------------------------
template <int CS> __device__ __forceinline__ void sweep_small_wave(const Batch& B, const TensorArgs& A, int k, int lane);

// LV: binary-counter levels, enough for the longest kernel of the launch.  CS > 0: kernels of at most 64
// elements take the one-wave-per-kernel path (sweep_small_wave with CS candidates per lane), as many per
// workgroup as it has waves; the host counts their workgroups accordingly.
// FUSED: the whole search of a kernel in this one launch, for calls so small that the chain of dependent
// launches, not the arithmetic, is what takes the time: after the argmin the workgroup refines the scale from the
// slice it still holds in LDS (chunks padded apart by four floats so that lanes reading different chunks hit
// different banks; lane = (scale, chunk), the scales of a round being the one the golden section waits for and
// those its next iterations could ask for, as many as the workgroup has lanes for) and writes the codes.  The
// host only picks this variant when every kernel fits one LDS tile and has at most as many chunks as the
// workgroup has lanes.  Same arithmetic, same order, same bits as the separate kernels.
template <int C, int LV, int CS, bool FUSED>
__global__ void __launch_bounds__(512) k_sweep_kernelwise(const Batch B)
{
    extern __shared__ float4 smem4[];
    float* slice = reinterpret_cast<float*>(smem4);
    __shared__ unsigned s_amax[16];
    __shared__ double s_bestE[16];
    __shared__ int s_bestJ[16];
    __shared__ unsigned s_bounds[kTile / kChunk];         // largest bound_key of every staged chunk

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthreads = blockDim.x, nwaves = nthreads >> 6;
    int k;
    const int t = find_tensor(B, blockIdx.x, k);
    const TensorArgs A = tensor_of(B, t);
    const int n = A.n;
    if constexpr (CS > 0) {
        if (n <= kChunk) {                                    // uniform over the workgroup; no barrier on this path
            const int ks = k * nwaves + wave;
            if (ks < A.K) sweep_small_wave<CS>(B, A, ks, lane);
            return;
        }
    }
    const float* __restrict__ src = A.w + (size_t)k * n;
    const float lo = B.lo, hi = B.hi;
    if (A.active != nullptr && A.active[k] == 0) return;      // uniform: the whole workgroup leaves
    const Xform X = make_xform(A, k, lo, true);
    const long long flat0 = (long long)k * n;

    const int npad = (n + kChunk - 1) & ~(kChunk - 1);
    const bool single = FUSED || npad <= kTile;
    constexpr int CSTRIDE = FUSED ? kChunk + 4 : kChunk;      // floats between chunk starts in LDS

    // ---- pass 1: abs-max (and, when the kernel fits one tile, the LDS staging)
    unsigned amax = 0;
    if (single) {
        for (int i = tid; i < npad; i += nthreads) {       // a wave stages one whole chunk per turn
            const float v = i < n ? xform_apply(X, src[i], flat0 + i, lo, hi) : 0.0f;
            slice[FUSED ? i + 4 * (i >> 6) : i] = v;
            const unsigned b = abs_bits(v);
            amax = b > amax ? b : amax;
            if constexpr (!FUSED) {
                const unsigned kb = wave_max_u32(bound_key(v, lo));
                if (lane == 0) s_bounds[i >> 6] = kb;
            }
        }
    } else {
        for (int i = tid; i < n; i += nthreads) {
            const unsigned b = abs_bits(xform_apply(X, src[i], flat0 + i, lo, hi));
            amax = b > amax ? b : amax;
        }
    }
    amax = wave_max_u32(amax);
    if (lane == 0) s_amax[wave] = amax;
    __syncthreads();
    unsigned am = 0;
    for (int w = 0; w < nwaves; ++w) am = s_amax[w] > am ? s_amax[w] : am;
    const float a = __uint_as_float(am);      // bit pattern order == value order for |x|; inf/NaN sort last

    const int G = B.G;
    if (!(a <= kHuge)) {                      // inf, NaN or too large: rejected
        if (tid == 0) {
            const float nanf_ = __uint_as_float(0x7fc00000u);
            if (A.absmax) A.absmax[k] = a;
            if (A.scale) A.scale[k] = nanf_;
            if (A.idx) A.idx[k] = -1;
            if (A.sse) A.sse[k] = (double)nanf_;
        }
        if (A.grid_sse)
            for (int j = tid; j < G; j += nthreads) A.grid_sse[(size_t)k * G + j] = (double)__uint_as_float(0x7fc00000u);
        if constexpr (FUSED) {                // a rejected kernel is coded as zeros
            if (A.packed != nullptr && (n & 1) == 0) {
                uint8_t* dst = A.packed + (((size_t)k * n) >> 1);
                for (int i = tid; i < (n >> 1); i += nthreads) dst[i] = 0;
            }
        }
        return;
    }
    const bool tiny = a < kTiny;              // coded as all-zero with scale 1
    const float qmaxf = (float)B.qmax, Gf = (float)G;

    // ---- candidates of this lane: j = wave*64*C + u*64 + lane
    float alpha[C], inv[C];
    int jcand[C];
#pragma unroll
    for (int u = 0; u < C; ++u) {
        const int j = (wave * C + u) * 64 + lane;
        jcand[u] = j;
        const int jj = j < G ? j : G - 1;
        alpha[u] = tiny ? 1.0f : grid_alpha(a, qmaxf, Gf, jj);
        inv[u] = 1.0f / alpha[u];
    }

    // ---- pass 2: sweep
    double st[C][LV];
#pragma unroll
    for (int u = 0; u < C; ++u)
#pragma unroll
        for (int l = 0; l < LV; ++l) st[u][l] = 0.0;
    unsigned ci = 0;
    if (single) {
        unsigned long long in0 = 0, in1 = 0;
        if constexpr (!FUSED) {
            const float inv_min = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(inv[0])));   // lane 0: the wave's smallest scale
            const int nfull = n / kChunk;
            in0 = chunks_inside_range(s_bounds, nfull < 64 ? nfull : 64, inv_min, lo, hi, lane);
            if (nfull > 64) in1 = chunks_inside_range(s_bounds + 64, nfull - 64, inv_min, lo, hi, lane);
        }
        sweep_slice<C, LV, CSTRIDE>(slice, (n + 7) & ~7, ci, alpha, inv, lo, hi, st, in0, in1);
    } else {
        for (int t0 = 0; t0 < npad; t0 += kTileStream) {
            const int tlen = (npad - t0) < kTileStream ? (npad - t0) : kTileStream;
            __syncthreads();
            for (int i = tid; i < tlen; i += nthreads) {
                const int gi = t0 + i;
                const float v = gi < n ? xform_apply(X, src[gi], flat0 + gi, lo, hi) : 0.0f;
                slice[i] = v;
                const unsigned kb = wave_max_u32(bound_key(v, lo));
                if (lane == 0) s_bounds[i >> 6] = kb;
            }
            __syncthreads();
            const int valid = ((n + 7) & ~7) - t0;       // the last tile may end in a partial chunk
            const int nvalid = valid < tlen ? valid : tlen;
            const float inv_min = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(inv[0])));
            const unsigned long long in0 = chunks_inside_range(s_bounds, nvalid / kChunk, inv_min, lo, hi, lane);
            sweep_slice<C, LV>(slice, nvalid, ci, alpha, inv, lo, hi, st, in0);
        }
    }
    double E[C];
    tree_fold<C, LV>(st, ci, E);

    if (A.grid_sse) {
#pragma unroll
        for (int u = 0; u < C; ++u)
            if (jcand[u] < G) A.grid_sse[(size_t)k * G + jcand[u]] = E[u];
    }

    // ---- argmin, lowest index among equal minima
    double bE = __longlong_as_double(0x7ff0000000000000LL);
    int bJ = INT_MAX;
#pragma unroll
    for (int u = 0; u < C; ++u)
        if (jcand[u] < G && E[u] < bE) { bE = E[u]; bJ = jcand[u]; }
    wave_argmin(bE, bJ);
    if (lane == 0) { s_bestE[wave] = bE; s_bestJ[wave] = bJ; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < nwaves; ++w) {
            const double oe = s_bestE[w];
            const int oj = s_bestJ[w];
            if (oe < bE || (oe == bE && oj < bJ)) { bE = oe; bJ = oj; }
        }
        if (bJ == INT_MAX) bJ = 0;            // only if every f overflowed to inf
        if (A.absmax) A.absmax[k] = a;
        if (A.idx) A.idx[k] = bJ;
        if constexpr (!FUSED) {
            if (A.sse) A.sse[k] = bE;
            if (A.scale) A.scale[k] = tiny ? 1.0f : grid_alpha(a, qmaxf, Gf, bJ);
        }
    }
    if constexpr (FUSED) {
        // ---- refinement between the grid neighbours of the argmin, from the slice in LDS.  Every thread keeps the
        // state of the search in registers and does the same bookkeeping (it is a few dozen instructions; one thread
        // doing it for all would cost a barrier and a trip through LDS per round).
        __shared__ double vals2[2][kMaxProbes];   // f at the scales of a round; rounds alternate between the halves, so
                                                  // that a round's values are never written while the last one's are read
        __shared__ double s_argE;
        __shared__ int s_argJ;
        double* part = reinterpret_cast<double*>(slice + B.fused_part_off);      // two buffers of nthreads doubles
        const int m = npad / kChunk;                          // chunks = lanes per scale (host: m <= nthreads)
        const int S = nthreads / m;                           // scales evaluated at a time
        const int max_depth = S >= 8 ? 2 : (S >= 4 ? 1 : 0);
        const int iters = B.iters;
        if (tid == 0) { s_argE = bE; s_argJ = bJ; }
        __syncthreads();
        const int j = s_argJ;
        const float aj = tiny ? 1.0f : grid_alpha(a, qmaxf, Gf, j);
        GsRegs R;
        R.it = 0; R.best = s_argE; R.best_a = aj; R.done = 1; R.have_c = R.have_d = 0;
        R.lo_a = R.hi_a = R.pc = R.pd = 1.0f; R.ec = R.ed = 0.0;
        if (!tiny && iters > 0) {
            R.lo_a = j == 0 ? 0.0f : grid_alpha(a, qmaxf, Gf, j - 1);
            R.hi_a = j == G - 1 ? aj : grid_alpha(a, qmaxf, Gf, j + 1);
            const float w = R.hi_a - R.lo_a;
            R.pc = __builtin_fmaf(-kPhi, w, R.hi_a);
            R.pd = __builtin_fmaf(kPhi, w, R.lo_a);
            R.done = 0;
        }
        float pr[kMaxProbes];
        int np = gs_plan_list(R, iters, max_depth, pr);
        const int slot = tid / m, c = tid - slot * m;
        const float4* my4 = reinterpret_cast<const float4*>(slice + c * CSTRIDE);
        int par = 0;
        while (!R.done) {                                     // uniform: every thread holds the same state
            double* vals = vals2[par];
            par ^= 1;
            for (int base = 0; base < np; base += S) {
                const int pi = base + slot;
                const bool on = slot < S && pi < np;
                double v = 0.0;
                if (on) {
                    float al[1] = {1.0f};
#pragma unroll
                    for (int i = 0; i < kMaxProbes; ++i) al[0] = (i == pi) ? pr[i] : al[0];
                    const float iv[1] = {1.0f / al[0]};
                    float sum[1] = {0.0f};
                    // the chunk comes from LDS two 8-element groups ahead of its use
                    float4 q[4] = {my4[0], my4[1], my4[2], my4[3]};
#pragma unroll
                    for (int e = 0; e < kChunk / 8; ++e) {
                        const float4 p0 = q[(2 * e) & 3], p1 = q[(2 * e + 1) & 3];
                        const float xs[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
                        if (e + 2 < kChunk / 8) { q[(2 * e) & 3] = my4[2 * e + 4]; q[(2 * e + 1) & 3] = my4[2 * e + 5]; }
                        __builtin_amdgcn_sched_barrier(0);
                        eval_stage<8, 1>(xs, al, iv, lo, hi, sum);
                    }
                    v = (double)sum[0];
                }
                // pairwise tree over the m chunk sums of every scale: aligned groups of sixteen per step; the step
                // that leaves one value writes it to vals
                double* cur = part;
                double* nxt = part + nthreads;
                if (m == 1) { if (on) vals[pi] = v; } else cur[tid] = v;
                __syncthreads();
                int cnt = m;
                while (cnt > 1) {
                    const int ncnt = (cnt + 15) >> 4;
                    if (on && c < ncnt) {
                        double e16[16];
#pragma unroll
                        for (int i = 0; i < 16; ++i) e16[i] = (16 * c + i < cnt) ? cur[slot * m + 16 * c + i] : 0.0;
#pragma unroll
                        for (int w = 1; w < 16; w <<= 1)
#pragma unroll
                            for (int i = 0; i < 16; i += 2 * w) e16[i] = e16[i] + e16[i + w];
                        if (ncnt == 1) vals[pi] = e16[0]; else nxt[slot * m + c] = e16[0];
                    }
                    __syncthreads();
                    double* tmp = cur; cur = nxt; nxt = tmp;
                    cnt = ncnt;
                }
            }
            double v8[kMaxProbes];
#pragma unroll
            for (int i = 0; i < kMaxProbes; ++i) v8[i] = vals[i];
            gs_advance(R, pr, v8, np, iters);
            np = gs_plan_list(R, iters, max_depth, pr);
        }
        const float best_a = R.best_a;
        if (tid == 0) {
            if (A.scale) A.scale[k] = best_a;
            if (A.sse) A.sse[k] = R.best;
        }
        // ---- codes, for even n (bytes of a kernel with odd n straddle its neighbours: k_pack_int4 does those)
        if (A.packed != nullptr && (n & 1) == 0) {
            const float invb = 1.0f / best_a;
            uint8_t* dst = A.packed + (((size_t)k * n) >> 1);
            const bool word_ok = (reinterpret_cast<uintptr_t>(dst) & 3u) == 0;
            for (int e0 = tid * 8; e0 < n; e0 += nthreads * 8) {
                const float4* p4 = reinterpret_cast<const float4*>(slice + e0 + 4 * (e0 >> 6));
                const float4 p0 = p4[0], p1 = p4[1];
                const float xs[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
                unsigned word = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) word |= ((unsigned)(int)code_of(xs[i], invb, lo, hi) & 0xFu) << (4 * i);
                const int len = (n - e0) < 8 ? (n - e0) : 8;         // even
                if (len == 8 && word_ok) {
                    *reinterpret_cast<unsigned*>(dst + (e0 >> 1)) = word;
                } else {
                    for (int b = 0; b < (len >> 1); ++b) dst[(e0 >> 1) + b] = (uint8_t)(word >> (8 * b));
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// sweep_small_wave: the same for kernels of at most 64 elements (depthwise 3x3, first layers,
// narrow pointwise layers): one WAVE per kernel, as many kernels per workgroup as it has waves, no LDS and no
// barrier; part of k_sweep_kernelwise, so that a network's tiny and ordinary kernels share one launch.  Lane i
// holds element i; an element reaches all lanes as a scalar operand (v_readlane), lanes own C >= ceil(G/64)
// candidates each; a single chunk needs no tree.
// ---------------------------------------------------------------------------------
template <int C>
__device__ __forceinline__ void sweep_small_wave(const Batch& B, const TensorArgs& A, int k, int lane)
{
    if (A.active != nullptr && A.active[k] == 0) return;
    const int n = A.n;                                        // <= 64
    const float lo = B.lo, hi = B.hi;
    const Xform X = make_xform(A, k, lo, true);
    const long long flat0 = (long long)k * n;
    const float x = lane < n ? xform_apply(X, A.w[flat0 + lane], flat0 + lane, lo, hi) : 0.0f;
    const float a = __uint_as_float(wave_max_u32(abs_bits(x)));

    const int G = B.G;
    if (!(a <= kHuge)) {
        const float nanf_ = __uint_as_float(0x7fc00000u);
        if (lane == 0) {
            if (A.absmax) A.absmax[k] = a;
            if (A.scale) A.scale[k] = nanf_;
            if (A.idx) A.idx[k] = -1;
            if (A.sse) A.sse[k] = (double)nanf_;
        }
        if (A.grid_sse)
            for (int j = lane; j < G; j += 64) A.grid_sse[(size_t)k * G + j] = (double)nanf_;
        return;
    }
    const bool tiny = a < kTiny;
    const float qmaxf = (float)B.qmax, Gf = (float)G;
    float alpha[C], inv[C], s[C];
    int jcand[C];
#pragma unroll
    for (int u = 0; u < C; ++u) {
        const int j = u * 64 + lane;
        jcand[u] = j;
        const int jj = j < G ? j : G - 1;
        alpha[u] = tiny ? 1.0f : grid_alpha(a, qmaxf, Gf, jj);
        inv[u] = 1.0f / alpha[u];
        s[u] = 0.0f;
    }
    constexpr int NE = (C >= 4) ? 4 : 8;
    const int xb = __float_as_int(x);
    for (int e0 = 0; e0 < n; e0 += NE) {                      // lanes >= n hold 0: exact no-ops
        float xs[NE];
#pragma unroll
        for (int i = 0; i < NE; ++i) xs[i] = __int_as_float(__builtin_amdgcn_readlane(xb, (e0 + i) & 63));
        eval_stage<NE, C>(xs, alpha, inv, lo, hi, s);
    }
    double E[C];
#pragma unroll
    for (int u = 0; u < C; ++u) E[u] = (double)s[u];
    if (A.grid_sse) {
#pragma unroll
        for (int u = 0; u < C; ++u)
            if (jcand[u] < G) A.grid_sse[(size_t)k * G + jcand[u]] = E[u];
    }
    double bE = __longlong_as_double(0x7ff0000000000000LL);
    int bJ = INT_MAX;
#pragma unroll
    for (int u = 0; u < C; ++u)
        if (jcand[u] < G && E[u] < bE) { bE = E[u]; bJ = jcand[u]; }
    wave_argmin(bE, bJ);
    if (lane == 0) {
        if (bJ == INT_MAX) bJ = 0;
        if (A.absmax) A.absmax[k] = a;
        if (A.idx) A.idx[k] = bJ;
        if (A.sse) A.sse[k] = bE;
        if (A.scale) A.scale[k] = tiny ? 1.0f : grid_alpha(a, qmaxf, Gf, bJ);
    }
}

// ---------------------------------------------------------------------------------
// k_refine_kernelwise: golden-section refinement between the grid neighbours of j*
// ---------------------------------------------------------------------------------
// Pairwise sum across the m lanes (chunks) of one kernel.  v: this lane's chunk sum; c: chunk number;
// the kernel's first lane is a multiple of m.  While m is even the lowest tree levels pair neighbouring
// lanes of one 16-lane row, so they are DPP shifts (no LDS, no barrier): d = min(4, trailing zeros of m)
// levels leave m >> d partial sums, which go through LDS three tree levels per barrier.
// All lanes of the workgroup call it together.  cur / nxt: this kernel's slices of the two halves of the
// combine buffer; they alternate so that a call never overwrites what a slower lane is still reading.
__device__ __forceinline__ double tree_combine(double v, int c, int m, bool active,
                                               double*& cur, double*& nxt)
{
    if (m == 1) return v;                     // m is uniform over the workgroup
    int d = 0;
    if ((m & 1) == 0) { v = v + dpp_row_shl<1>(v); d = 1; }
    if ((m & 3) == 0) { v = v + dpp_row_shl<2>(v); d = 2; }
    if ((m & 7) == 0) { v = v + dpp_row_shl<4>(v); d = 3; }
    if ((m & 15) == 0) { v = v + dpp_row_shl<8>(v); d = 4; }
    int cnt = m >> d;
    if (active && (c & ((1 << d) - 1)) == 0) cur[c >> d] = v;
    __syncthreads();
    while (cnt > 1) {
        const int ncnt = (cnt + 7) >> 3;
        if (active && c < ncnt) {
            double e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = (8 * c + i < cnt) ? cur[8 * c + i] : 0.0;
            nxt[c] = ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
        }
        __syncthreads();
        double* t = cur; cur = nxt; nxt = t;
        cnt = ncnt;
    }
    const double r = active ? cur[0] : 0.0;
    // the next call starts in the other half, so it cannot overwrite what a slower lane still reads
    double* t = cur; cur = nxt; nxt = t;
    return r;
}

constexpr int kTileStride = 68;   // floats between chunks in the transpose tile (64 + 4: keeps 16-byte alignment)

// CL: element slots per lane, 64 (general) or 16 (kernels of <= 16 elements).  XF: some tensor of the launch is
// searched through a transform (the residual of a first tensor); without it that code is left out altogether.
template <int CL, bool XF>
__global__ void __launch_bounds__(1024) k_refine_kernelwise(const Batch B, int tile_chunks)
{
    // dynamic LDS: [combine buffer: 2 x blockDim doubles][per-wave transpose tiles]
    extern __shared__ double smem_d[];
    double* buf = smem_d;
    float* tiles = reinterpret_cast<float*>(smem_d + 2 * blockDim.x);

    const int tid = threadIdx.x;
    int g;
    const int t = find_tensor(B, blockIdx.x, g);
    const TensorArgs A = tensor_of(B, t);
    const int n = A.n;
    const int m = (CL == kChunk) ? (n + kChunk - 1) / kChunk : 1;
    const int cpw = blockDim.x / m;           // kernels per workgroup (host guarantees m <= blockDim)
    const int ch = tid / m, c = tid - ch * m;
    const int k = g * cpw + ch;
    const float lo = B.lo, hi = B.hi;
    const bool in_range = (ch < cpw) && (k < A.K) && (A.active == nullptr || A.active[k < A.K ? k : 0] != 0);
    bool active = in_range;

    float a = 0.0f;
    int j = 0;
    double Ej = 0.0;
    if (active) { a = A.absmax[k]; j = A.idx[k]; Ej = A.sse[k]; }
    if (!(a <= kHuge) || a < kTiny) active = false;       // rejected or all-zero: nothing to refine

    // this lane's chunk, kept in registers for all probes (zeros beyond the end are exact no-ops)
    float x[CL];
    const Xform X = make_xform(A, k, lo, active);
    const bool coalesced = (CL == kChunk) && (n % kChunk == 0) &&
                           ((reinterpret_cast<uintptr_t>(A.w) & 15u) == 0) && tile_chunks > 0;
    if (coalesced) {
        // The workgroup's lanes map to consecutive 64-element chunks of memory.  Each wave reads
        // its own 64 chunks with fully coalesced 16-byte loads, tile_chunks chunks at a time,
        // and hands every lane its chunk through a wave-private LDS tile.
        const int lane = tid & 63, wave = tid >> 6;
        const int left = A.K - g * cpw;
        const int nvalid = (left < cpw ? left : cpw) * m;              // chunks this workgroup owns
        const float4* __restrict__ src4 =
            reinterpret_cast<const float4*>(A.w + (size_t)g * cpw * n) + (size_t)wave * 64 * (kChunk / 4);
        float* tile = tiles + (size_t)wave * tile_chunks * kTileStride;
        const int per_lane = tile_chunks / 4;                          // float4 loads per lane and pass
#pragma unroll
        for (int i = 0; i < CL; ++i) x[i] = 0.0f;
        for (int p0 = 0; p0 < 64; p0 += tile_chunks) {
            for (int r = 0; r < per_lane; ++r) {
                const int f = r * 64 + lane;                           // float4 number inside this pass
                const int cj = f >> 4;                                 // chunk inside this pass
                if (wave * 64 + p0 + cj < nvalid) {
                    const float4 v = src4[(size_t)p0 * (kChunk / 4) + f];
                    *reinterpret_cast<float4*>(tile + cj * kTileStride + (f & 15) * 4) = v;
                }
            }
            __syncthreads();
            if (lane >= p0 && lane < p0 + tile_chunks && in_range) {
                const float4* t4 = reinterpret_cast<const float4*>(tile + (lane - p0) * kTileStride);
#pragma unroll
                for (int i = 0; i < CL / 4; ++i) {
                    const float4 v = t4[i];
                    x[4 * i + 0] = v.x; x[4 * i + 1] = v.y; x[4 * i + 2] = v.z; x[4 * i + 3] = v.w;
                }
            }
            __syncthreads();
        }
        if (!active) {
#pragma unroll
            for (int i = 0; i < CL; ++i) x[i] = 0.0f;
        }
    } else {
        const int e0 = c * kChunk;
        const int len = active ? ((n - e0) < CL ? (n - e0) : CL) : 0;
        const float* __restrict__ src = A.w + ((size_t)(active ? k : 0) * n + (active ? e0 : 0));
        const bool vec = ((reinterpret_cast<uintptr_t>(src) & 15u) == 0) && (len == CL);
        if (vec) {
            const float4* s4 = reinterpret_cast<const float4*>(src);
#pragma unroll
            for (int i = 0; i < CL / 4; ++i) {
                const float4 v = s4[i];
                x[4 * i + 0] = v.x; x[4 * i + 1] = v.y; x[4 * i + 2] = v.z; x[4 * i + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < CL; ++i) x[i] = (i < len) ? src[i] : 0.0f;
        }
    }
    if (XF && X.mode != 0 && active) {
        const int e0x = c * kChunk;
        const int lenx = (n - e0x) < CL ? (n - e0x) : CL;
        const long long f0 = (long long)k * n + e0x;
        const uint8_t* codes = X.mode == 2 ? X.sub + (f0 >> 1) : nullptr;
        if (X.mode == 2 && CL >= 32 && lenx == CL && (f0 & 1) == 0 && (reinterpret_cast<uintptr_t>(codes) & 15u) == 0) {
            // the stored codes of a whole chunk: CL / 2 bytes in 16-byte loads, unpacked from registers
#pragma unroll
            for (int v = 0; v < CL / 32; ++v) {
                const uint4 q4 = reinterpret_cast<const uint4*>(codes)[v];
                const unsigned words[4] = {q4.x, q4.y, q4.z, q4.w};
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    const unsigned wd = words[i >> 3];
                    const int q = X.sub_signed ? __builtin_amdgcn_sbfe((int)wd, 4 * (i & 7), 4)
                                               : (int)__builtin_amdgcn_ubfe(wd, 4 * (i & 7), 4);
                    x[32 * v + i] = __builtin_fmaf(-X.s1, (float)q, x[32 * v + i]);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < CL; ++i)
                if (i < lenx) x[i] = xform_apply(X, x[i], f0 + i, lo, hi);
        }
    }

    const int G = B.G;
    const float qmaxf = (float)B.qmax, Gf = (float)G;
    double* cur = buf + (tid - c);
    double* nxt = buf + blockDim.x + (tid - c);

    auto eval = [&](float alpha) -> double {
        const float inv = 1.0f / alpha;
        float s[1] = {0.0f};
        const float al[1] = {alpha}, iv[1] = {inv};
#pragma unroll
        for (int i = 0; i < CL; i += 8) {
            const float xs[8] = {x[i], x[i + 1], x[i + 2], x[i + 3], x[i + 4], x[i + 5], x[i + 6], x[i + 7]};
            eval_stage<8, 1>(xs, al, iv, lo, hi, s);
        }
        return tree_combine((double)s[0], c, m, active, cur, nxt);
    };

    const float aj = active ? grid_alpha(a, qmaxf, Gf, j) : 1.0f;
    float best_a = aj;
    double best = Ej;
    if (B.iters > 0) {
        float lo_a = (!active || j == 0) ? 0.0f : grid_alpha(a, qmaxf, Gf, j - 1);
        float hi_a = (!active || j == G - 1) ? aj : grid_alpha(a, qmaxf, Gf, j + 1);
        float w = hi_a - lo_a;
        float pc = __builtin_fmaf(-kPhi, w, hi_a);
        float pd = __builtin_fmaf(kPhi, w, lo_a);
        if (!active) { pc = 1.0f; pd = 1.0f; }
        double ec = eval(pc);
        double ed = eval(pd);
        if (ec < best) { best = ec; best_a = pc; }
        if (ed < best) { best = ed; best_a = pd; }
        for (int it = 0; it < B.iters; ++it) {
            const bool left = ec <= ed;       // keep [lo, d]: the new probe is a new c
            float probe;
            if (left) {
                hi_a = pd; pd = pc; ed = ec;
                w = hi_a - lo_a;
                pc = __builtin_fmaf(-kPhi, w, hi_a);
                probe = pc;
            } else {
                lo_a = pc; pc = pd; ec = ed;
                w = hi_a - lo_a;
                pd = __builtin_fmaf(kPhi, w, lo_a);
                probe = pd;
            }
            if (!active) probe = 1.0f;
            const double e = eval(probe);
            if (left) ec = e; else ed = e;
            if (e < best) { best = e; best_a = probe; }
        }
    }
    if (active && c == 0) {
        A.scale[k] = best_a;
        A.sse[k] = best;
    }

    // Fused INT4 codes, when n is even, so that every chunk starts and ends on a byte boundary (tensors with
    // odd n are coded by k_pack_int4): the chunk is still in registers, the scale is final.
    if (A.packed != nullptr && (n & 1) == 0 && in_range) {
        const float inv = 1.0f / (active ? best_a : 1.0f);      // all-zero / rejected kernels: x is 0 here, codes 0
        const int e0 = c * kChunk;
        const int len = (n - e0) < CL ? (n - e0) : CL;
        unsigned words[CL / 8];
#pragma unroll
        for (int w = 0; w < CL / 8; ++w) {
            unsigned word = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                word |= ((unsigned)(int)code_of(x[8 * w + i], inv, lo, hi) & 0xFu) << (4 * i);
            words[w] = word;
        }
        uint8_t* dst = A.packed + (((size_t)k * n + e0) >> 1);
        if (len == CL && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
            if constexpr (CL == kChunk) {
                reinterpret_cast<uint4*>(dst)[0] = make_uint4(words[0], words[1], words[2], words[3]);
                reinterpret_cast<uint4*>(dst)[1] = make_uint4(words[4], words[5], words[6], words[7]);
            } else {
                reinterpret_cast<uint2*>(dst)[0] = make_uint2(words[0], words[1]);
            }
        } else {
            const int nbytes = len >> 1;
#pragma unroll
            for (int b = 0; b < CL / 2; ++b)
                if (b < nbytes) dst[b] = (uint8_t)(words[b >> 2] >> (8 * (b & 3)));
        }
    }
}

// ---------------------------------------------------------------------------------
// k_pack_int4: codes [x/scale]_Zp, two per byte in memory order over the whole tensor
// ---------------------------------------------------------------------------------
__global__ void __launch_bounds__(kPackThreads) k_pack_int4(const Batch B)
{
    int g;
    const int t = find_tensor(B, blockIdx.x, g);
    const TensorArgs A = tensor_of(B, t);
    const int n = A.n;
    const long long total = (long long)A.K * n;
    const long long e0 = ((long long)g * kPackThreads + threadIdx.x) * kPackPerThread;
    if (e0 >= total) return;
    const float lo = B.lo, hi = B.hi;
    const float* __restrict__ src = A.w;
    const float* __restrict__ scale = A.scale;

    const int cnt = (total - e0) < kPackPerThread ? (int)(total - e0) : kPackPerThread;
    float v[kPackPerThread];
    if (cnt == kPackPerThread && (reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
        const float4 p0 = reinterpret_cast<const float4*>(src + e0)[0];
        const float4 p1 = reinterpret_cast<const float4*>(src + e0)[1];
        v[0] = p0.x; v[1] = p0.y; v[2] = p0.z; v[3] = p0.w;
        v[4] = p1.x; v[5] = p1.y; v[6] = p1.z; v[7] = p1.w;
    } else {
#pragma unroll
        for (int i = 0; i < kPackPerThread; ++i) v[i] = (i < cnt) ? src[e0 + i] : 0.0f;
    }

    int k = (int)((unsigned)e0 / (unsigned)n);          // K*n < 2^31: 32-bit division is enough
    int r = (int)((unsigned)e0 - (unsigned)k * (unsigned)n);   // position inside kernel k
    float sc = scale[k];
    float inv = 1.0f / sc;
    Xform X = make_xform(A, k, lo, true);
    unsigned word = 0;
#pragma unroll
    for (int i = 0; i < kPackPerThread; ++i) {
        if (i < cnt) {
            if (r == n) {                     // crossed into the next kernel
                r = 0; ++k;
                sc = scale[k];
                inv = 1.0f / sc;
                X = make_xform(A, k, lo, true);
            }
            const float x = xform_apply(X, v[i], e0 + i, lo, hi);
            // a rejected kernel (scale NaN) is coded as zeros
            const int q = (sc == sc) ? (int)code_of(x, inv, lo, hi) : 0;
            word |= ((unsigned)q & 0xFu) << (4 * i);
            ++r;
        }
    }
    uint8_t* dst = A.packed + (e0 >> 1);
    if (cnt == kPackPerThread && (reinterpret_cast<uintptr_t>(A.packed) & 3u) == 0) {
        *reinterpret_cast<unsigned*>(dst) = word;
    } else {
        const int nbytes = (cnt + 1) >> 1;
        for (int b = 0; b < nbytes; ++b) dst[b] = (uint8_t)(word >> (8 * b));
    }
}

// ---------------------------------------------------------------------------------
// k_layer_sums: per-layer total of the per-kernel errors (the layer MSE that picks the key layers,
// Section 3.5), one workgroup per layer; fixed order: thread-strided fp64 partials, then a tree in LDS.
// ---------------------------------------------------------------------------------
constexpr int kMaxSumBatch = 64;
struct SumBatch {
    const double* v[kMaxSumBatch];
    int n[kMaxSumBatch];
};

__global__ void __launch_bounds__(256) k_layer_sums(const SumBatch B, double* __restrict__ out)
{
    __shared__ double part[256];
    const double* __restrict__ v = B.v[blockIdx.x];
    const int n = B.n[blockIdx.x];
    double acc = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) acc = acc + v[i];
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] = part[threadIdx.x] + part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[blockIdx.x] = part[0];
}

}  // namespace

#endif  // MMSE_WEIGHTS_H_
