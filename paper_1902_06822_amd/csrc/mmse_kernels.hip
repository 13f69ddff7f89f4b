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

#include "mmse.h"

namespace {

constexpr int kChunk = 64;             // elements per sequential fp32 chunk
constexpr int kMaxBatch = 32;          // tensors per launch (descriptor table lives in kernarg)
constexpr int kTile = 8192;            // floats of one kernel staged in LDS at a time
constexpr int kLevelsKW = 11;          // binary-counter levels for <= 1024 chunks (65536 elements)
constexpr int kLevelsKWSmall = 8;      // ... for <= 128 chunks (8192 elements: one LDS tile)
constexpr int kBlockChunks = 64;       // activation block = 64 chunks = 4096 elements
constexpr int kBlockElems = kBlockChunks * kChunk;
constexpr int kLevelsBlk = 7;          // levels for 64 chunks
constexpr float kTiny = 0x1p-60f;
constexpr float kHuge = 0x1p+60f;
constexpr float kPhi = 0.6180339887f;
constexpr int kPackPerThread = 8;
constexpr int kPackThreads = 256;

struct TensorArgs {
    const float* w;
    const float* scale1;     // nullptr, or first-tensor scales (search/pack the residual)
    float* scale;
    int32_t* idx;
    double* sse;
    float* absmax;           // workspace [K]
    double* grid_sse;        // optional [K][G]
    uint8_t* packed;
    const uint8_t* sub_packed;   // nullptr, or stored codes Q of another tensor: search/pack w - sub_scale*Q
    const float* sub_scale;      // [K], with sub_packed
    const uint8_t* active;       // nullptr, or [K]: kernels with 0 are skipped by the search
    int K;
    int n;
};

struct Batch {
    TensorArgs t[kMaxBatch];
    int start[kMaxBatch + 1];   // prefix sum of workgroups per tensor
    int count;
    int G;
    int qmax;
    int iters;
    float lo, hi;               // (float)qmin, (float)qmax
};

// ---------------------------------------------------------------------------------
// element arithmetic
// ---------------------------------------------------------------------------------
__device__ __forceinline__ float code_of(float x, float inv, float lo, float hi)
{
    return __builtin_amdgcn_fmed3f(__builtin_rintf(x * inv), lo, hi);
}

__device__ __forceinline__ float sq_err_acc(float x, float alpha, float inv, float lo, float hi, float s)
{
    const float q = code_of(x, inv, lo, hi);
    const float r = __builtin_fmaf(-alpha, q, x);
    return __builtin_fmaf(r, r, s);
}

// Grid candidate j: (absmax/qmax) * ((j+1)/G), three correctly rounded fp32 operations.
__device__ __forceinline__ float grid_alpha(float absmax, float qmaxf, float Gf, int j)
{
    const float smax = absmax / qmaxf;
    const float frac = (float)(j + 1) / Gf;
    return smax * frac;
}

// What a search reads: the weights themselves, or what another INT4 tensor leaves of them
// (Section 3.5: T - sum_{i != j} alpha_i*Q_i), formed with one fused multiply-add per element and
// never stored.  mode 1 recomputes Q = [w/alpha] from alpha; mode 2 reads Q from packed codes.
struct Xform {
    int mode;                // 0 none, 1 subtract alpha*[w/alpha], 2 subtract alpha*stored code
    float s1, inv1;
    const uint8_t* sub;
    bool sub_signed;
};

__device__ __forceinline__ Xform make_xform(const TensorArgs& A, int k, float lo, bool valid)
{
    Xform X;
    X.mode = A.sub_packed != nullptr ? 2 : (A.scale1 != nullptr ? 1 : 0);
    X.s1 = 1.0f; X.inv1 = 1.0f; X.sub = A.sub_packed; X.sub_signed = lo < 0.0f;
    if (valid) {
        if (X.mode == 1) { X.s1 = A.scale1[k]; X.inv1 = 1.0f / X.s1; }
        if (X.mode == 2) X.s1 = A.sub_scale[k];
    }
    return X;
}

// v: element number `flat` of the tensor (row-major over [K][n]).
__device__ __forceinline__ float xform_apply(const Xform& X, float v, long long flat, float lo, float hi)
{
    if (X.mode == 1) {
        v = __builtin_fmaf(-X.s1, code_of(v, X.inv1, lo, hi), v);
    } else if (X.mode == 2) {
        int q = (X.sub[flat >> 1] >> ((flat & 1) * 4)) & 0xF;
        if (X.sub_signed && q >= 8) q -= 16;
        v = __builtin_fmaf(-X.s1, (float)q, v);
    }
    return v;
}

// Ordering point for an LDS tile that only one wave touches: the LDS unit executes a wave's
// instructions in order, so a read issued after a write of the same wave sees it; the fences keep the
// compiler from moving LDS accesses across this point.  No workgroup barrier: the waves stay independent.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Lane i receives lane i + N of its row of 16 lanes (zero beyond the row).
template <int N>
__device__ __forceinline__ double dpp_row_shl(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, 0x100 + N, 0xf, 0xf, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, 0x100 + N, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double readlane_f64(double v, int l)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), l);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), l);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ unsigned abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }

__device__ __forceinline__ unsigned wave_max_u32(unsigned v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned o = (unsigned)__shfl_xor((int)v, off, 64);
        v = o > v ? o : v;
    }
    return v;
}

// (value, index) minimum over a wave; the lower index wins among equal values.
__device__ __forceinline__ void wave_argmin(double& e, int& j)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double oe = __shfl_xor(e, off, 64);
        const int oj = __shfl_xor(j, off, 64);
        if (oe < e || (oe == e && oj < j)) { e = oe; j = oj; }
    }
}

// Binary-counter form of the pairwise sum: after chunk number ci has been pushed,
// st[.][l] holds the sum of a complete aligned group of 2^l chunks whenever bit l of
// (ci+1) is set.  ci is wave-uniform, so the ladder is scalar control flow.
template <int C, int L, int l>
__device__ __forceinline__ void tree_push_level(double (&st)[C][L], double (&t)[C], unsigned ci)
{
    if constexpr (l < L) {
        if ((ci >> l) & 1u) {
#pragma unroll
            for (int u = 0; u < C; ++u) t[u] = st[u][l] + t[u];
            tree_push_level<C, L, l + 1>(st, t, ci);
        } else {
#pragma unroll
            for (int u = 0; u < C; ++u) st[u][l] = t[u];
        }
    }
}

template <int C, int L>
__device__ __forceinline__ void tree_push(double (&st)[C][L], double (&t)[C], unsigned ci)
{
    tree_push_level<C, L, 0>(st, t, ci);
}

// Sum of the m chunks pushed so far (carries the unpaired partial groups upward).
template <int C, int L>
__device__ __forceinline__ void tree_fold(const double (&st)[C][L], unsigned m, double (&out)[C])
{
#pragma unroll
    for (int u = 0; u < C; ++u) out[u] = 0.0;
#pragma unroll
    for (int l = 0; l < L; ++l) {
        if ((m >> l) & 1u) {
#pragma unroll
            for (int u = 0; u < C; ++u) out[u] = st[u][l] + out[u];
        }
    }
}

// Squared errors of NE elements against C candidates, accumulated into s[C] in element
// order.  The five operations of an evaluation form a dependent chain, so they are issued
// stage by stage over all NE*C evaluations: consecutive instructions are independent and
// the VALU pipeline latency is covered inside one wave.  (Order of the accumulation, the
// only thing that affects the result, is unchanged: element by element per candidate.)
// Scheduling fences keep the compiler from re-serialising the stages; LDS/VMEM/SALU
// instructions may still move across them.
#define MMSE_STAGE_FENCE() __builtin_amdgcn_sched_barrier(0x94)
template <int NE, int C>
__device__ __forceinline__ void eval_stage(const float (&x)[NE], const float (&alpha)[C], const float (&inv)[C],
                                           float lo, float hi, float (&s)[C])
{
    float t[NE][C];
#pragma unroll
    for (int i = 0; i < NE; ++i)
#pragma unroll
        for (int u = 0; u < C; ++u) t[i][u] = x[i] * inv[u];
    MMSE_STAGE_FENCE();
#pragma unroll
    for (int i = 0; i < NE; ++i)
#pragma unroll
        for (int u = 0; u < C; ++u) t[i][u] = __builtin_rintf(t[i][u]);
    MMSE_STAGE_FENCE();
#pragma unroll
    for (int i = 0; i < NE; ++i)
#pragma unroll
        for (int u = 0; u < C; ++u) t[i][u] = __builtin_amdgcn_fmed3f(t[i][u], lo, hi);
    MMSE_STAGE_FENCE();
#pragma unroll
    for (int i = 0; i < NE; ++i)
#pragma unroll
        for (int u = 0; u < C; ++u) t[i][u] = __builtin_fmaf(-alpha[u], t[i][u], x[i]);
    MMSE_STAGE_FENCE();
#pragma unroll
    for (int i = 0; i < NE; ++i) {
#pragma unroll
        for (int u = 0; u < C; ++u) s[u] = __builtin_fmaf(t[i][u], t[i][u], s[u]);
        MMSE_STAGE_FENCE();
    }
}

// Sweep the `nelem` elements (a multiple of 8; zero padded) that sit in LDS at `slice` for the C
// candidates of this lane: whole 64-element chunks, then a last shorter chunk that only walks the
// 8-element groups it has (padding zeros would be exact no-ops, so skipping them changes nothing).
template <int C, int L>
__device__ __forceinline__ void sweep_slice(const float* slice, int nelem, unsigned& ci,
                                            const float (&alpha)[C], const float (&inv)[C],
                                            float lo, float hi, double (&st)[C][L])
{
    const float4* s4 = reinterpret_cast<const float4*>(slice);
    constexpr int NE = (C >= 4) ? 4 : 8;            // elements per stage group
    const int nfull = nelem / kChunk;
    const int tail = nelem - nfull * kChunk;        // 0, 8, ..., 56 elements of a last partial chunk
    const int ntotal = nfull + (tail > 0 ? 1 : 0);
    for (int c = 0; c < ntotal; ++c, ++ci) {
        float s[C];
#pragma unroll
        for (int u = 0; u < C; ++u) s[u] = 0.0f;
        if (c < nfull) {
            // elements come from LDS one group ahead of their use (same address in every lane: broadcast)
            float4 nxt[NE / 4];
#pragma unroll
            for (int q = 0; q < NE / 4; ++q) nxt[q] = s4[c * (kChunk / 4) + q];
#pragma unroll
            for (int e = 0; e < kChunk / NE; ++e) {
                float x[NE];
#pragma unroll
                for (int q = 0; q < NE / 4; ++q) {
                    x[4 * q + 0] = nxt[q].x; x[4 * q + 1] = nxt[q].y; x[4 * q + 2] = nxt[q].z; x[4 * q + 3] = nxt[q].w;
                }
                if (e + 1 < kChunk / NE) {
#pragma unroll
                    for (int q = 0; q < NE / 4; ++q) nxt[q] = s4[c * (kChunk / 4) + (e + 1) * (NE / 4) + q];
                }
                __builtin_amdgcn_sched_barrier(0);       // the prefetch is issued before this group's arithmetic
                eval_stage<NE, C>(x, alpha, inv, lo, hi, s);
            }
        } else {
            for (int e = 0; e < tail / NE; ++e) {
                float x[NE];
#pragma unroll
                for (int q = 0; q < NE / 4; ++q) {
                    const float4 v = s4[c * (kChunk / 4) + e * (NE / 4) + q];
                    x[4 * q + 0] = v.x; x[4 * q + 1] = v.y; x[4 * q + 2] = v.z; x[4 * q + 3] = v.w;
                }
                eval_stage<NE, C>(x, alpha, inv, lo, hi, s);
            }
        }
        double t[C];
#pragma unroll
        for (int u = 0; u < C; ++u) t[u] = (double)s[u];
        tree_push<C, L>(st, t, ci);
    }
}

__device__ __forceinline__ int find_tensor(const Batch& B, int bid)
{
    int t = 0;
    while (t + 1 < B.count && bid >= B.start[t + 1]) ++t;
    return t;
}

// ---------------------------------------------------------------------------------
// k_sweep_kernelwise: abs-max + grid sweep + argmin, one workgroup per weight kernel
// ---------------------------------------------------------------------------------
template <int C, int LV>   // LV: binary-counter levels, enough for the longest kernel of the launch
__global__ void __launch_bounds__(512) k_sweep_kernelwise(const Batch B)
{
    extern __shared__ float4 smem4[];
    float* slice = reinterpret_cast<float*>(smem4);
    __shared__ unsigned s_amax[16];
    __shared__ double s_bestE[16];
    __shared__ int s_bestJ[16];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthreads = blockDim.x, nwaves = nthreads >> 6;
    const int t = find_tensor(B, blockIdx.x);
    const TensorArgs& A = B.t[t];
    const int k = blockIdx.x - B.start[t];
    const int n = A.n;
    const float* __restrict__ src = A.w + (size_t)k * n;
    const float lo = B.lo, hi = B.hi;
    if (A.active != nullptr && A.active[k] == 0) return;      // uniform: the whole workgroup leaves
    const Xform X = make_xform(A, k, lo, true);
    const long long flat0 = (long long)k * n;

    const int npad = (n + kChunk - 1) & ~(kChunk - 1);
    const bool single = npad <= kTile;

    // ---- pass 1: abs-max (and, when the kernel fits one tile, the LDS staging)
    unsigned amax = 0;
    if (single) {
        for (int i = tid; i < npad; i += nthreads) {
            const float v = i < n ? xform_apply(X, src[i], flat0 + i, lo, hi) : 0.0f;
            slice[i] = v;
            const unsigned b = abs_bits(v);
            amax = b > amax ? b : amax;
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
        sweep_slice<C, LV>(slice, (n + 7) & ~7, ci, alpha, inv, lo, hi, st);
    } else {
        for (int t0 = 0; t0 < npad; t0 += kTile) {
            const int tlen = (npad - t0) < kTile ? (npad - t0) : kTile;
            __syncthreads();
            for (int i = tid; i < tlen; i += nthreads) {
                const int gi = t0 + i;
                slice[i] = gi < n ? xform_apply(X, src[gi], flat0 + gi, lo, hi) : 0.0f;
            }
            __syncthreads();
            const int valid = ((n + 7) & ~7) - t0;       // the last tile may end in a partial chunk
            sweep_slice<C, LV>(slice, valid < tlen ? valid : tlen, ci, alpha, inv, lo, hi, st);
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
        if (A.sse) A.sse[k] = bE;
        if (A.scale) A.scale[k] = tiny ? 1.0f : grid_alpha(a, qmaxf, Gf, bJ);
    }
}

// ---------------------------------------------------------------------------------
// k_sweep_small: the same for kernels of at most 64 elements (depthwise 3x3, first layers,
// narrow pointwise layers): one WAVE per kernel, four kernels per workgroup, no LDS and no
// barrier.  Lane i holds element i; an element reaches all lanes as a scalar operand
// (v_readlane), lanes own C = ceil(G/64) candidates each; a single chunk needs no tree.
// ---------------------------------------------------------------------------------
template <int C>
__global__ void __launch_bounds__(256) k_sweep_small(const Batch B)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = find_tensor(B, blockIdx.x);
    const TensorArgs& A = B.t[t];
    const int k = (blockIdx.x - B.start[t]) * 4 + wave;
    if (k >= A.K) return;                                     // waves are independent: no barrier below
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
// Pairwise sum across the m lanes (chunks) of one kernel through LDS, three tree levels
// per barrier.  v: this lane's chunk sum; c: chunk number; l0: first lane of the kernel.
// All lanes of the workgroup call it together.  `par` alternates the buffer so that
// a call never overwrites what a slower lane is still reading from the previous call.
__device__ __forceinline__ double tree_combine(double v, int c, int m, bool active,
                                               double*& cur, double*& nxt)
{
    // cur / nxt: this kernel's slice of the two halves of the combine buffer (lane c at [c]).
    if (m == 1) return v;                     // m is uniform over the workgroup
    if (active) cur[c] = v;
    __syncthreads();
    int cnt = m;
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

template <int CL>   // element slots per lane: 64 (general) or 16 (kernels of <= 16 elements)
__global__ void __launch_bounds__(1024) k_refine_kernelwise(const Batch B, int tile_chunks)
{
    // dynamic LDS: [combine buffer: 2 x blockDim doubles][per-wave transpose tiles]
    extern __shared__ double smem_d[];
    double* buf = smem_d;
    float* tiles = reinterpret_cast<float*>(smem_d + 2 * blockDim.x);

    const int tid = threadIdx.x;
    const int t = find_tensor(B, blockIdx.x);
    const TensorArgs& A = B.t[t];
    const int g = blockIdx.x - B.start[t];
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
    if (X.mode != 0 && active) {
        const int e0x = c * kChunk;
        const int lenx = (n - e0x) < CL ? (n - e0x) : CL;
        const long long f0 = (long long)k * n + e0x;
#pragma unroll
        for (int i = 0; i < CL; ++i)
            if (i < lenx) x[i] = xform_apply(X, x[i], f0 + i, lo, hi);
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

    // Fused INT4 codes (the host passes `packed` here only when n is even, so that every chunk
    // starts and ends on a byte boundary): the chunk is still in registers, the scale is final.
    if (A.packed != nullptr && in_range) {
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
    const int t = find_tensor(B, blockIdx.x);
    const TensorArgs& A = B.t[t];
    const int g = blockIdx.x - B.start[t];
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
// Algorithm 1 iterated (Section 3.5): bookkeeping between alternating sweeps, per kernel
// ---------------------------------------------------------------------------------
constexpr int kMaxDualBatch = 24;

struct DualTensor {
    double* sse;             // kept error per kernel
    const double* tsse;      // error of the tentative sweep
    float* s1; const float* ts1;
    float* s2; const float* ts2;
    int32_t* sweeps;
    uint8_t* active;
    uint8_t* accepted;
    const uint8_t* tp1; uint8_t* p1;     // tentative / kept codes of the first tensor
    const uint8_t* tp2; uint8_t* p2;
    int K;
    int n;
};

struct DualBatch {
    DualTensor t[kMaxDualBatch];
    int start[kMaxDualBatch + 1];        // prefix sum of workgroups per tensor
    int count;
    double eps;
};

__device__ __forceinline__ int find_dual_tensor(const DualBatch& D, int bid)
{
    int t = 0;
    while (t + 1 < D.count && bid >= D.start[t + 1]) ++t;
    return t;
}

// After the first sweep: a kernel goes on iterating unless it was rejected or is already exact.
__global__ void __launch_bounds__(256) k_dual_init(const DualBatch D)
{
    const int t = find_dual_tensor(D, blockIdx.x);
    const DualTensor& T = D.t[t];
    const int k = (blockIdx.x - D.start[t]) * blockDim.x + threadIdx.x;
    if (k >= T.K) return;
    const double e = T.sse[k];
    const bool ok = e == e;
    T.sweeps[k] = ok ? 1 : 0;
    T.active[k] = (ok && e > 0.0) ? 1 : 0;
}

// After a later sweep: keep it if it lowered the error; stop when the relative gain is <= eps,
// when the error reached 0, or when the sweep was no better (then it is discarded).
__global__ void __launch_bounds__(256) k_dual_accept(const DualBatch D)
{
    const int t = find_dual_tensor(D, blockIdx.x);
    const DualTensor& T = D.t[t];
    const int k = (blockIdx.x - D.start[t]) * blockDim.x + threadIdx.x;
    if (k >= T.K) return;
    uint8_t acc = 0;
    if (T.active[k]) {
        const double e = T.sse[k], te = T.tsse[k];
        if (te < e) {
            acc = 1;
            const bool conv = (e - te) <= D.eps * e;
            T.s1[k] = T.ts1[k]; T.s2[k] = T.ts2[k]; T.sse[k] = te; T.sweeps[k] += 1;
            if (conv || !(te > 0.0)) T.active[k] = 0;
        } else {
            T.active[k] = 0;
        }
    }
    T.accepted[k] = acc;
}

// Codes of the kernels whose sweep was kept move from the tentative to the kept buffers, nibble by
// nibble (a byte can hold codes of two kernels when n is odd).
__global__ void __launch_bounds__(256) k_dual_copy_codes(const DualBatch D)
{
    const int t = find_dual_tensor(D, blockIdx.x);
    const DualTensor& T = D.t[t];
    const long long total = (long long)T.K * T.n;
    const long long b = (long long)(blockIdx.x - D.start[t]) * blockDim.x + threadIdx.x;
    if (2 * b >= total) return;
    const unsigned e0 = (unsigned)(2 * b);
    const bool a0 = T.accepted[e0 / (unsigned)T.n] != 0;
    const bool a1 = (long long)e0 + 1 < total && T.accepted[(e0 + 1) / (unsigned)T.n] != 0;
    if (!a0 && !a1) return;
    const unsigned mask = (a0 ? 0x0Fu : 0u) | (a1 ? 0xF0u : 0u);
    T.p1[b] = (uint8_t)((T.p1[b] & ~mask) | (T.tp1[b] & mask));
    T.p2[b] = (uint8_t)((T.p2[b] & ~mask) | (T.tp2[b] & mask));
}

// ---------------------------------------------------------------------------------
// Dual line search (Section 3.5, Eq. 12): exhaustive G1 x G2 grid over (a1, a2), per element the
// best of the 2^p first codes with the second code rounded
// ---------------------------------------------------------------------------------
struct DualLsArgs {
    const float* w;
    int K, n, G1, G2, splits;
    int qmin, qmax;
    float lo, hi;
    float* absmax;           // workspace [K]
    double* part_e;          // workspace [K][splits]: best error found by one workgroup
    int* part_idx;           // workspace [K][splits]: its flat grid index a*G2 + b
    double* grid;            // optional [K][G1*G2]
    float* scale1; float* scale2; int32_t* idx1; int32_t* idx2; double* sse;
    uint8_t* packed1; uint8_t* packed2;
};

// Error of one element for the pair (a1, a2): min over the first code t of
// (x - a1*t - a2*[(x - a1*t)/a2])^2.  The minimum is taken over |d| and squared once: rounding is
// monotonic, so fl(min|d| ^2) is the minimum of the fl(d^2) bit for bit.  6 VALU instructions per code
// (fma, mul, rndne, med3, fma, min with |.| as a source modifier).
template <bool FULL16>
__device__ __forceinline__ float dual_elem_err(float x, float a1, float a2, float inv2, float lo, float hi,
                                               int qmin, int qmax)
{
    float best = __uint_as_float(0x7f800000u);
    if constexpr (FULL16) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float r = __builtin_fmaf(-a1, (float)(qmin + i), x);
            const float d = __builtin_fmaf(-a2, code_of(r, inv2, lo, hi), r);
            best = __builtin_fminf(best, __builtin_fabsf(d));
        }
    } else {
        for (int t = qmin; t <= qmax; ++t) {
            const float r = __builtin_fmaf(-a1, (float)t, x);
            const float d = __builtin_fmaf(-a2, code_of(r, inv2, lo, hi), r);
            best = __builtin_fminf(best, __builtin_fabsf(d));
        }
    }
    return best * best;
}

// One workgroup per (kernel, split): the kernel's slice sits in LDS; a wave takes units of 64
// consecutive pairs in row-major (a, b) order, lane = pair; every unit is a full sweep of the
// slice.  The best (error, flat index) of the workgroup goes to the workspace; k_dual_ls_pick
// takes the minimum over the splits.  The splits exist so that a layer with few kernels still
// fills the GPU.
template <bool FULL16>
__global__ void __launch_bounds__(512) k_dual_ls(const DualLsArgs A)
{
    extern __shared__ float4 smem4[];
    float* slice = reinterpret_cast<float*>(smem4);
    __shared__ unsigned s_amax[8];
    __shared__ double s_bestE[8];
    __shared__ int s_bestI[8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthreads = blockDim.x, nwaves = nthreads >> 6;
    const int k = blockIdx.x / A.splits, sp = blockIdx.x - k * A.splits;
    const int n = A.n;
    const float* __restrict__ src = A.w + (size_t)k * n;
    const float lo = A.lo, hi = A.hi;
    const int npad = (n + kChunk - 1) & ~(kChunk - 1);
    unsigned amax = 0;
    for (int i = tid; i < npad; i += nthreads) {
        const float v = i < n ? src[i] : 0.0f;
        slice[i] = v;
        const unsigned b = abs_bits(v);
        amax = b > amax ? b : amax;
    }
    amax = wave_max_u32(amax);
    if (lane == 0) s_amax[wave] = amax;
    __syncthreads();
    unsigned am = 0;
    for (int w = 0; w < nwaves; ++w) am = s_amax[w] > am ? s_amax[w] : am;
    const float a = __uint_as_float(am);
    const size_t pslot = (size_t)k * A.splits + sp;
    const double inf = __longlong_as_double(0x7ff0000000000000LL);
    if (sp == 0 && tid == 0) A.absmax[k] = a;
    if (!(a <= kHuge)) {                                      // rejected: k_dual_ls_pick writes the NaNs
        if (tid == 0) { A.part_e[pslot] = inf; A.part_idx[pslot] = INT_MAX; }
        if (A.grid && sp == 0)
            for (int j = tid; j < A.G1 * A.G2; j += nthreads)
                A.grid[(size_t)k * A.G1 * A.G2 + j] = (double)__uint_as_float(0x7fc00000u);
        return;
    }
    const int n8 = (n + 7) & ~7;
    if (a < kTiny) {                                          // all-zero kernel: scales 1, codes 0, error = sum x^2
        double E = inf;
        if (sp == 0 && wave == 0) {
            const float one[1] = {1.0f};
            double st[1][kLevelsKWSmall];
#pragma unroll
            for (int l = 0; l < kLevelsKWSmall; ++l) st[0][l] = 0.0;
            unsigned ci = 0;
            sweep_slice<1, kLevelsKWSmall>(slice, n8, ci, one, one, lo, hi, st);
            double e1[1];
            tree_fold<1, kLevelsKWSmall>(st, ci, e1);
            E = e1[0];
        }
        if (tid == 0) { A.part_e[pslot] = E; A.part_idx[pslot] = sp == 0 ? 0 : INT_MAX; }
        if (A.grid && sp == 0 && wave == 0)
            for (int j = lane; j < A.G1 * A.G2; j += 64) A.grid[(size_t)k * A.G1 * A.G2 + j] = E;
        return;
    }

    const float qmaxf = (float)A.qmax, G1f = (float)A.G1, G2f = (float)A.G2;
    const int pairs = A.G1 * A.G2;
    const int units = (pairs + 63) >> 6;
    const float4* s4 = reinterpret_cast<const float4*>(slice);
    double bE = inf;
    int bI = INT_MAX;
    for (int u = sp * nwaves + wave; u < units; u += A.splits * nwaves) {
        const bool valid = u * 64 + lane < pairs;
        const int flat = valid ? u * 64 + lane : pairs - 1;
        const int ja = flat / A.G2, jb = flat - ja * A.G2;
        const float a1 = grid_alpha(a, qmaxf, G1f, ja);
        const float a2 = a1 * ((float)(jb + 1) / G2f);
        const float inv2 = 1.0f / a2;
        double st[1][kLevelsKWSmall];
#pragma unroll
        for (int l = 0; l < kLevelsKWSmall; ++l) st[0][l] = 0.0;
        unsigned ci = 0;
        for (int c0 = 0; c0 < n8; c0 += kChunk, ++ci) {
            const int len = (n8 - c0) < kChunk ? (n8 - c0) : kChunk;   // multiple of 8; zeros pad to 8: exact no-ops
            float sum = 0.0f;
            for (int e = 0; e < len; e += 4) {
                const float4 v = s4[(c0 + e) >> 2];
                sum = sum + dual_elem_err<FULL16>(v.x, a1, a2, inv2, lo, hi, A.qmin, A.qmax);
                sum = sum + dual_elem_err<FULL16>(v.y, a1, a2, inv2, lo, hi, A.qmin, A.qmax);
                sum = sum + dual_elem_err<FULL16>(v.z, a1, a2, inv2, lo, hi, A.qmin, A.qmax);
                sum = sum + dual_elem_err<FULL16>(v.w, a1, a2, inv2, lo, hi, A.qmin, A.qmax);
            }
            double t[1] = {(double)sum};
            tree_push<1, kLevelsKWSmall>(st, t, ci);
        }
        double E1[1];
        tree_fold<1, kLevelsKWSmall>(st, ci, E1);
        const double E = E1[0];
        if (valid) {
            if (A.grid) A.grid[(size_t)k * A.G1 * A.G2 + flat] = E;
            if (E < bE || (E == bE && flat < bI)) { bE = E; bI = flat; }
        }
    }
    wave_argmin(bE, bI);
    if (lane == 0) { s_bestE[wave] = bE; s_bestI[wave] = bI; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < nwaves; ++w) {
            const double oe = s_bestE[w];
            const int oi = s_bestI[w];
            if (oe < bE || (oe == bE && oi < bI)) { bE = oe; bI = oi; }
        }
        A.part_e[pslot] = bE;
        A.part_idx[pslot] = bI;
    }
}

// Minimum over the splits of every kernel (first flat index among equal errors) and the outputs.
__global__ void __launch_bounds__(256) k_dual_ls_pick(const DualLsArgs A)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= A.K) return;
    const float a = A.absmax[k];
    if (!(a <= kHuge)) {
        const float nanf_ = __uint_as_float(0x7fc00000u);
        A.scale1[k] = nanf_; A.scale2[k] = nanf_; A.idx1[k] = -1; A.idx2[k] = -1; A.sse[k] = (double)nanf_;
        return;
    }
    double bE = A.part_e[(size_t)k * A.splits];
    int bI = A.part_idx[(size_t)k * A.splits];
    for (int sp = 1; sp < A.splits; ++sp) {
        const double oe = A.part_e[(size_t)k * A.splits + sp];
        const int oi = A.part_idx[(size_t)k * A.splits + sp];
        if (oe < bE || (oe == bE && oi < bI)) { bE = oe; bI = oi; }
    }
    if (bI == INT_MAX) bI = 0;
    A.sse[k] = bE;
    if (a < kTiny) {
        A.scale1[k] = 1.0f; A.scale2[k] = 1.0f; A.idx1[k] = 0; A.idx2[k] = 0;
        return;
    }
    const int ja = bI / A.G2, jb = bI - ja * A.G2;
    const float a1 = grid_alpha(a, (float)A.qmax, (float)A.G1, ja);
    A.scale1[k] = a1;
    A.scale2[k] = a1 * ((float)(jb + 1) / (float)A.G2);
    A.idx1[k] = ja;
    A.idx2[k] = jb;
}

// Both code tensors for the chosen scales, 8 elements per thread; the first of equally good first
// codes is kept.  All-zero and rejected kernels are coded as zeros.
__global__ void __launch_bounds__(kPackThreads) k_dual_ls_codes(const DualLsArgs A)
{
    const int n = A.n;
    const long long total = (long long)A.K * n;
    const long long e0 = ((long long)blockIdx.x * kPackThreads + threadIdx.x) * kPackPerThread;
    if (e0 >= total) return;
    const float lo = A.lo, hi = A.hi;
    const int cnt = (total - e0) < kPackPerThread ? (int)(total - e0) : kPackPerThread;
    int k = (int)((unsigned)e0 / (unsigned)n);
    int r = (int)((unsigned)e0 - (unsigned)k * (unsigned)n);
    unsigned w1 = 0, w2 = 0;
    for (int i = 0; i < cnt; ++i) {
        if (r == n) { r = 0; ++k; }
        const float am = A.absmax[k];
        int t1 = 0, t2 = 0;
        if (am <= kHuge && !(am < kTiny)) {
            const float x = A.w[e0 + i], a1 = A.scale1[k], a2 = A.scale2[k], inv2 = 1.0f / a2;
            float best = __uint_as_float(0x7f800000u);
            for (int t = A.qmin; t <= A.qmax; ++t) {
                const float rr = __builtin_fmaf(-a1, (float)t, x);
                const float q = code_of(rr, inv2, lo, hi);
                const float d = __builtin_fmaf(-a2, q, rr);
                const float e = d * d;
                if (e < best) { best = e; t1 = t; t2 = (int)q; }
            }
        }
        w1 |= ((unsigned)t1 & 0xFu) << (4 * i);
        w2 |= ((unsigned)t2 & 0xFu) << (4 * i);
        ++r;
    }
    const int nbytes = (cnt + 1) >> 1;
    uint8_t* d1 = A.packed1 + (e0 >> 1);
    uint8_t* d2 = A.packed2 + (e0 >> 1);
    for (int b = 0; b < nbytes; ++b) { d1[b] = (uint8_t)(w1 >> (8 * b)); d2[b] = (uint8_t)(w2 >> (8 * b)); }
}

// ---------------------------------------------------------------------------------
// Comparison optimiser of Section 3.4 (Table 2, "Altern."): from the max-abs scale, alternate
// codes Q = [w/alpha] and the least-squares scale alpha = sum w*Q / sum Q^2 until the scale repeats.
// One workgroup per kernel; a thread owns chunks of 64 elements (fp64 sum of the exact products inside a
// chunk, pairwise tree over the chunks in LDS, integer sum of squares): not a hot path, kept plain.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ double block_tree_sum(double (*buf)[1024], int m, int tid, int nthreads)
{
    int cur = 0;
    __syncthreads();
    while (m > 1) {
        const int h = m >> 1;
        for (int i = tid; i < h; i += nthreads) buf[cur ^ 1][i] = buf[cur][2 * i] + buf[cur][2 * i + 1];
        if ((m & 1) && tid == 0) buf[cur ^ 1][h] = buf[cur][m - 1];
        m = h + (m & 1);
        cur ^= 1;
        __syncthreads();
    }
    const double r = buf[cur][0];
    __syncthreads();                       // the buffers are free again
    return r;
}

__global__ void __launch_bounds__(256) k_alt_kernelwise(const float* __restrict__ w, int n, int qmax, float lo, float hi,
                                                        int max_iters, float* scale, double* sse, int32_t* updates)
{
    __shared__ double buf[2][1024];
    __shared__ unsigned s_amax[4];
    __shared__ int s_den[4];
    __shared__ float s_alpha;
    __shared__ int s_stop;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthreads = blockDim.x, nwaves = nthreads >> 6;
    const int k = blockIdx.x;
    const float* __restrict__ src = w + (size_t)k * n;
    const int nchunks = (n + kChunk - 1) / kChunk;

    unsigned amax = 0;
    for (int i = tid; i < n; i += nthreads) {
        const unsigned b = abs_bits(src[i]);
        amax = b > amax ? b : amax;
    }
    amax = wave_max_u32(amax);
    if (lane == 0) s_amax[wave] = amax;
    __syncthreads();
    unsigned am = 0;
    for (int v = 0; v < nwaves; ++v) am = s_amax[v] > am ? s_amax[v] : am;
    const float a = __uint_as_float(am);
    if (!(a <= kHuge)) {
        if (tid == 0) {
            const float nanf_ = __uint_as_float(0x7fc00000u);
            scale[k] = nanf_; sse[k] = (double)nanf_; updates[k] = 0;
        }
        return;
    }
    float alpha = a < kTiny ? 1.0f : a / (float)qmax;
    int upd = 0;
    const int iters = a < kTiny ? 0 : max_iters;
    for (int it = 0; it < iters; ++it) {
        const float inv = 1.0f / alpha;
        int den = 0;
        for (int c = tid; c < nchunks; c += nthreads) {
            const int s0 = c * kChunk;
            const int len = (n - s0) < kChunk ? (n - s0) : kChunk;
            double num = 0.0;
            for (int i = 0; i < len; ++i) {
                const float x = src[s0 + i];
                const float q = code_of(x, inv, lo, hi);
                num = __builtin_fma((double)x, (double)q, num);
                den += (int)q * (int)q;
            }
            buf[0][c] = num;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) den += __shfl_xor(den, off, 64);
        if (lane == 0) s_den[wave] = den;
        const double num = block_tree_sum(buf, nchunks, tid, nthreads);      // its first barrier also covers s_den
        if (tid == 0) {
            int d = 0;
            for (int v = 0; v < nwaves; ++v) d += s_den[v];
            int stop = 1;
            if (d != 0) {
                const float next = (float)(num / (double)d);
                if (next != alpha) { s_alpha = next; stop = 0; }
            }
            s_stop = stop;
        }
        __syncthreads();
        const int stop = s_stop;
        if (!stop) { alpha = s_alpha; upd = it + 1; }
        __syncthreads();                   // s_stop, s_alpha and s_den are rewritten in the next round
        if (stop) break;
    }
    {
        const float inv = 1.0f / alpha;
        for (int c = tid; c < nchunks; c += nthreads) {
            const int s0 = c * kChunk;
            const int len = (n - s0) < kChunk ? (n - s0) : kChunk;
            float sum = 0.0f;
            for (int i = 0; i < len; ++i) {
                const float x = src[s0 + i];
                const float r = __builtin_fmaf(-alpha, code_of(x, inv, lo, hi), x);
                sum = __builtin_fmaf(r, r, sum);
            }
            buf[0][c] = (double)sum;
        }
        const double e = block_tree_sum(buf, nchunks, tid, nthreads);
        if (tid == 0) { scale[k] = alpha; sse[k] = e; updates[k] = upd; }
    }
}

// ---------------------------------------------------------------------------------
// activation tensor: one problem of N elements over the whole GPU
// ---------------------------------------------------------------------------------
// Workspace layout (all offsets multiples of 256 bytes):
//   ActState                              scalars of the search
//   part0[nb][G] doubles                  per-block tree sums of the grid sweep
//   part1[ceil(nb/64)][G], part2, ...     upper tree levels, 64 blocks at a time
//   probe0[nb], probe1[...], ...          same hierarchy for one refinement probe
constexpr int kMaxProbes = 8;          // scales evaluated in one pass over an activation tensor

struct ActState {
    unsigned absmax_bits;
    int status;              // 0 normal, 1 all-zero (scale 1), 2 rejected
    int j;                   // grid argmin
    int it;                  // golden-section iterations decided so far
    int done;                // refinement finished
    int have_c, have_d;      // f(pc), f(pd) known
    int nprobe;              // scales to evaluate in the next pass
    float absmax;
    float lo_a, hi_a, pc, pd, best_a;
    float probes[kMaxProbes];
    double ec, ed, best;
    unsigned min_key, max_key;   // offset form: order-preserving keys of min and max
    float delta;                 // offset form: min of the tensor
};

// What the activation kernels search instead of the stored tensor (never written to memory):
//   mode 1: the residual of a first tensor, x - s*[x/s] saturated to [lo1, hi1]   (Section 3.7, Eq. 16)
//   mode 2: the shifted tensor x - delta, delta = min x                            (Section 3.1, Eq. 2)
struct ActPre {
    int mode;
    const float* s;              // device: the first scale (mode 1) or delta (mode 2)
    float lo1, hi1;
};
struct ActPreV { int mode; float s, inv, lo1, hi1; };

__device__ __forceinline__ ActPreV act_pre_load(const ActPre& P)
{
    ActPreV V;
    V.mode = P.mode; V.lo1 = P.lo1; V.hi1 = P.hi1;
    V.s = P.mode != 0 ? *P.s : 0.0f;
    V.inv = P.mode == 1 ? 1.0f / V.s : 0.0f;
    return V;
}

__device__ __forceinline__ float act_pre(const ActPreV& V, float v)
{
    if (V.mode == 1) return __builtin_fmaf(-V.s, code_of(v, V.inv, V.lo1, V.hi1), v);
    if (V.mode == 2) return v - V.s;
    return v;
}

// Order-preserving map of fp32 bit patterns to unsigned integers (-NaN < -inf < ... < +inf < +NaN).
__device__ __forceinline__ unsigned order_key(float v)
{
    const unsigned b = __float_as_uint(v);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float order_unkey(unsigned k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Several activation tensors searched by the same launches: the 4096-element blocks of all tensors
// are numbered consecutively (start[t] = first block of tensor t); every tensor has its own state.
constexpr int kMaxActBatch = 64;
struct ActBatch {
    const float* x[kMaxActBatch];
    long long N[kMaxActBatch];
    int start[kMaxActBatch + 1];
    int count;
    ActState* S;                 // [count]
};
struct ActOut {
    float* scale[kMaxActBatch];
    int32_t* idx[kMaxActBatch];
    double* sse[kMaxActBatch];
    uint8_t* packed[kMaxActBatch];
};

// tensor that owns block b: the largest t with start[t] <= b
__device__ __forceinline__ int act_find(const ActBatch& B, int b)
{
    int lo = 0, hi = B.count - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (B.start[mid] <= b) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// rows a tensor of nb blocks has after l tree stages of 64
__host__ __device__ inline int act_rows(int nb, int l)
{
    for (int i = 0; i < l; ++i) nb = (nb + 63) / 64;
    return nb;
}

// At tree level l the rows of all tensors are again stored one tensor after the other.  Finds the
// tensor that owns row r of that level; returns its first row there (first) and at the level below (below).
__device__ __forceinline__ int act_find_level(const ActBatch& B, int l, int r, int& first, int& below)
{
    int acc = 0, accb = 0, t = 0;
    for (; t < B.count; ++t) {
        const int nb = B.start[t + 1] - B.start[t];
        const int rows = act_rows(nb, l);
        if (r < acc + rows || t == B.count - 1) break;
        acc += rows;
        accb += act_rows(nb, l - 1);
    }
    first = acc; below = accb;
    return t;
}

__global__ void k_act_init(ActState* Sall, int count)
{
    if (blockIdx.x == 0 && (int)threadIdx.x < count) {
        ActState* S = Sall + threadIdx.x;
        S->absmax_bits = 0; S->status = 0; S->j = 0; S->it = 0; S->done = 1;
        S->have_c = S->have_d = 0; S->nprobe = 0; S->absmax = 0.0f;
        S->lo_a = S->hi_a = S->pc = S->pd = S->best_a = 1.0f;
        for (int i = 0; i < kMaxProbes; ++i) S->probes[i] = 1.0f;
        S->ec = S->ed = S->best = 0.0;
        S->min_key = 0xffffffffu; S->max_key = 0u; S->delta = 0.0f;
    }
}

// ---- golden-section bookkeeping (one thread) ---------------------------------------
// The search is sequential: each iteration needs f at one new scale.  One pass over a big
// tensor costs a full read of it, so a pass evaluates the scale(s) the search is waiting
// for *and* every scale the next two iterations could ask for (both outcomes of each
// comparison: 1 + 2 + 4, or 2 + 2 + 4 at the start).  act_advance then replays the plain
// sequential algorithm, looking values up by scale; it stops when a value is missing.
// The probes are produced by the same fp32 expressions on both paths, so a lookup is an
// exact match.  Nothing about the result depends on how much was evaluated ahead.
template <int DEPTH>
__device__ void act_enumerate(float lo_a, float hi_a, float pc, float pd, int depth, float* list, int& n)
{
    if constexpr (DEPTH > 0) {
        if (depth == 0) return;
        {   // f(pc) <= f(pd): keep [lo, pd]
            const float nh = pd, npd = pc;
            const float npc = __builtin_fmaf(-kPhi, nh - lo_a, nh);
            if (n < kMaxProbes) list[n++] = npc;
            act_enumerate<DEPTH - 1>(lo_a, nh, npc, npd, depth - 1, list, n);
        }
        {   // otherwise: keep [pc, hi]
            const float nl = pc, npc = pd;
            const float npd = __builtin_fmaf(kPhi, hi_a - nl, nl);
            if (n < kMaxProbes) list[n++] = npd;
            act_enumerate<DEPTH - 1>(nl, hi_a, npc, npd, depth - 1, list, n);
        }
    }
}

__device__ void act_plan(ActState* S, int iters)
{
    int n = 0;
    float list[kMaxProbes];
    if (!S->done) {
        if (!S->have_c) list[n++] = S->pc;
        if (!S->have_d) list[n++] = S->pd;
        int depth = iters - S->it;
        if (depth > 2) depth = 2;
        act_enumerate<2>(S->lo_a, S->hi_a, S->pc, S->pd, depth, list, n);
    }
    S->nprobe = n;
    for (int i = 0; i < kMaxProbes; ++i) S->probes[i] = i < n ? list[i] : 1.0f;
}

__device__ bool act_lookup(const float* probes, const double* vals, int n, float a, double& out)
{
    for (int i = 0; i < n; ++i)
        if (probes[i] == a) { out = vals[i]; return true; }
    return false;
}

__device__ void act_advance(ActState* S, const double* vals, int iters)
{
    float lo_a = S->lo_a, hi_a = S->hi_a, pc = S->pc, pd = S->pd, best_a = S->best_a;
    double ec = S->ec, ed = S->ed, best = S->best;
    int have_c = S->have_c, have_d = S->have_d, it = S->it, done = S->done;
    const int n = S->nprobe;
    while (!done) {
        if (!have_c) {
            if (!act_lookup(S->probes, vals, n, pc, ec)) break;
            have_c = 1;
            if (ec < best) { best = ec; best_a = pc; }
        }
        if (!have_d) {
            if (!act_lookup(S->probes, vals, n, pd, ed)) break;
            have_d = 1;
            if (ed < best) { best = ed; best_a = pd; }
        }
        if (it == iters) { done = 1; break; }
        if (ec <= ed) {
            hi_a = pd; pd = pc; ed = ec;
            pc = __builtin_fmaf(-kPhi, hi_a - lo_a, hi_a);
            have_c = 0;
        } else {
            lo_a = pc; pc = pd; ec = ed;
            pd = __builtin_fmaf(kPhi, hi_a - lo_a, lo_a);
            have_d = 0;
        }
        ++it;
    }
    S->lo_a = lo_a; S->hi_a = hi_a; S->pc = pc; S->pd = pd; S->best_a = best_a;
    S->ec = ec; S->ed = ed; S->best = best;
    S->have_c = have_c; S->have_d = have_d; S->it = it; S->done = done;
}

// MODE 0: max |x| (integer max of the bit patterns); 1: max |residual of the first tensor|;
// 2: min and max of x as order-preserving keys (offset form).
template <int U, int MODE>
__global__ void __launch_bounds__(256) k_act_absmax(const ActBatch B, const ActPre pre)
{
    const float* __restrict__ x = B.x[blockIdx.y];
    const long long N = B.N[blockIdx.y];
    ActState* S = B.S + blockIdx.y;
    if ((long long)blockIdx.x * blockDim.x * 4 * U >= N) return;       // nothing of this tensor for this workgroup
    __shared__ unsigned s_amax[4];
    __shared__ unsigned s_amin[4];
    unsigned amax = 0, amin = 0xffffffffu;
    ActPreV V{};
    if constexpr (MODE == 1) V = act_pre_load(pre);
    auto take = [&](float v) {
        if constexpr (MODE == 2) {
            const unsigned k = order_key(v);
            amax = k > amax ? k : amax;
            amin = k < amin ? k : amin;
        } else {
            if constexpr (MODE == 1) v = act_pre(V, v);
            const unsigned b = abs_bits(v);
            amax = b > amax ? b : amax;
        }
    };
    const bool aligned = (reinterpret_cast<uintptr_t>(x) & 15u) == 0;
    // U independent 16-byte loads per thread and trip: enough bytes in flight to fill HBM
    const long long tile = (long long)blockDim.x * 4 * U;                 // elements per workgroup and trip
    const long long stride = (long long)gridDim.x * tile;
    for (long long base = (long long)blockIdx.x * tile; base < N; base += stride) {
        if (aligned && base + tile <= N) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                v[u] = *reinterpret_cast<const float4*>(x + base + ((long long)u * blockDim.x + threadIdx.x) * 4);
#pragma unroll
            for (int u = 0; u < U; ++u) { take(v[u].x); take(v[u].y); take(v[u].z); take(v[u].w); }
        } else {
            for (long long i = base + threadIdx.x; i < base + tile && i < N; i += blockDim.x) take(x[i]);
        }
    }
    amax = wave_max_u32(amax);
    if constexpr (MODE == 2) amin = ~wave_max_u32(~amin);
    if ((threadIdx.x & 63) == 0) { s_amax[threadIdx.x >> 6] = amax; s_amin[threadIdx.x >> 6] = amin; }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned am = s_amax[0], an = s_amin[0];
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w) {
            am = s_amax[w] > am ? s_amax[w] : am;
            an = s_amin[w] < an ? s_amin[w] : an;
        }
        if constexpr (MODE == 2) {
            atomicMax(&S->max_key, am);
            atomicMin(&S->min_key, an);
        } else {
            atomicMax(&S->absmax_bits, am);       // integer max: exact and order-free
        }
    }
}

// Offset form: delta = min x; the search range is that of x - delta, whose largest element is
// fl(max - delta) because rounding is monotonic.  Anything not finite rejects the tensor.
__global__ void k_act_offset_setup(ActState* S, float* delta_out)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const float mn = order_unkey(S->min_key), mx = order_unkey(S->max_key);
    const float nanf_ = __uint_as_float(0x7fc00000u);
    const bool finite = (abs_bits(mn) < 0x7f800000u) && (abs_bits(mx) < 0x7f800000u);
    const float range = finite ? mx - mn : nanf_;
    S->delta = mn;
    S->absmax_bits = abs_bits(range);
    *delta_out = (range <= kHuge) ? mn : nanf_;
}

// Grid sweep of one 4096-element block per workgroup; waves split the candidates.
template <int C>
__global__ void __launch_bounds__(512) k_act_sweep(const ActBatch B, int G, int qmax,
                                                    float lo, float hi, double* part0, const ActPre pre)
{
    __shared__ float4 slice4[kBlockElems / 4];
    float* slice = reinterpret_cast<float*>(slice4);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthreads = blockDim.x;
    const int t = act_find(B, blockIdx.x);
    const float* __restrict__ x = B.x[t];
    const long long N = B.N[t];
    const ActState* S = B.S + t;
    const float a = __uint_as_float(S->absmax_bits);
    if (!(a <= kHuge)) return;                // rejected: k_act_argmin reports it
    const bool tiny = a < kTiny;
    const long long base = (long long)(blockIdx.x - B.start[t]) * kBlockElems;
    const int len = (N - base) < kBlockElems ? (int)(N - base) : kBlockElems;
    const int npad = (len + kChunk - 1) & ~(kChunk - 1);
    const ActPreV V = act_pre_load(pre);
    for (int i = tid; i < npad; i += nthreads) slice[i] = i < len ? act_pre(V, x[base + i]) : 0.0f;
    __syncthreads();

    const float qmaxf = (float)qmax, Gf = (float)G;
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
    double st[C][kLevelsBlk];
#pragma unroll
    for (int u = 0; u < C; ++u)
#pragma unroll
        for (int l = 0; l < kLevelsBlk; ++l) st[u][l] = 0.0;
    unsigned ci = 0;
    sweep_slice<C, kLevelsBlk>(slice, (len + 7) & ~7, ci, alpha, inv, lo, hi, st);
    double E[C];
    tree_fold<C, kLevelsBlk>(st, ci, E);
#pragma unroll
    for (int u = 0; u < C; ++u)
        if (jcand[u] < G) part0[(size_t)blockIdx.x * G + jcand[u]] = E[u];
}

// One tree stage over blocks: out[g][j] = pairwise sum of in[64g .. 64g+63][j].
// When a stage leaves a single row and fin != nullptr the caller continues with it.
// Output row blockIdx.y of level `level` belongs to one tensor; its inputs are that tensor's rows of level - 1.
__global__ void __launch_bounds__(256) k_act_reduce64(const ActBatch B, int level, const double* __restrict__ in, int G,
                                                      double* __restrict__ out)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    int first, below;
    const int t = act_find_level(B, level, blockIdx.y, first, below);
    const int g = blockIdx.y - first;                                   // group of 64 input rows inside the tensor
    const int rows = act_rows(B.start[t + 1] - B.start[t], level - 1);
    if (j >= G) return;
    in += (size_t)below * G;
    double v[64];
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        const int r = g * 64 + i;
        v[i] = r < rows ? in[(size_t)r * G + j] : 0.0;
    }
#pragma unroll
    for (int w = 1; w < 64; w <<= 1)
#pragma unroll
        for (int i = 0; i < 64; i += 2 * w) v[i] = v[i] + v[i + w];
    out[(size_t)blockIdx.y * G + j] = v[0];
}

// Argmin over the G grid sums (one workgroup) and set-up of the refinement state.
__global__ void __launch_bounds__(1024) k_act_argmin(const ActBatch B, const double* __restrict__ tot, int G, int qmax,
                                                     int iters, const ActOut O)
{
    __shared__ double s_bestE[16];
    __shared__ int s_bestJ[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    ActState* S = B.S + blockIdx.x;
    float* scale = O.scale[blockIdx.x];
    int32_t* idx = O.idx[blockIdx.x];
    double* sse = O.sse[blockIdx.x];
    tot += (size_t)blockIdx.x * G;                 // the last level holds one row per tensor
    const float a = __uint_as_float(S->absmax_bits);
    if (!(a <= kHuge)) {
        if (tid == 0) {
            const float nanf_ = __uint_as_float(0x7fc00000u);
            S->status = 2; S->absmax = a;
            *scale = nanf_; *idx = -1; *sse = (double)nanf_;
        }
        return;
    }
    double bE = __longlong_as_double(0x7ff0000000000000LL);
    int bJ = INT_MAX;
    for (int j = tid; j < G; j += blockDim.x) {
        const double e = tot[j];
        if (e < bE) { bE = e; bJ = j; }       // ascending j per thread: strict < keeps the lowest
    }
    wave_argmin(bE, bJ);
    if (lane == 0) { s_bestE[wave] = bE; s_bestJ[wave] = bJ; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < nwaves; ++w) {
            const double oe = s_bestE[w];
            const int oj = s_bestJ[w];
            if (oe < bE || (oe == bE && oj < bJ)) { bE = oe; bJ = oj; }
        }
        if (bJ == INT_MAX) bJ = 0;
        const bool tiny = a < kTiny;
        const float qmaxf = (float)qmax, Gf = (float)G;
        const float aj = tiny ? 1.0f : grid_alpha(a, qmaxf, Gf, bJ);
        S->absmax = a; S->j = bJ; S->status = tiny ? 1 : 0; S->it = 0;
        S->best = bE; S->best_a = aj;
        S->done = 1; S->have_c = S->have_d = 0;
        *idx = bJ; *scale = aj; *sse = bE;
        if (!tiny && iters > 0) {
            const float lo_a = bJ == 0 ? 0.0f : grid_alpha(a, qmaxf, Gf, bJ - 1);
            const float hi_a = bJ == G - 1 ? aj : grid_alpha(a, qmaxf, Gf, bJ + 1);
            const float w = hi_a - lo_a;
            S->lo_a = lo_a; S->hi_a = hi_a;
            S->pc = __builtin_fmaf(-kPhi, w, hi_a);
            S->pd = __builtin_fmaf(kPhi, w, lo_a);
            S->done = 0;
        }
        act_plan(S, iters);
    }
}

// One refinement pass: f at up to kMaxProbes scales for every block of 64 chunks.
// lane = chunk, wave = block.  A block is handled as two halves by element: elements 0..31 of every
// chunk, then elements 32..63 (the fp32 chunk sums simply continue, so the order of additions is
// unchanged).  All 16 coalesced 16-byte loads of the wave are issued up front; the first half goes
// through a wave-private LDS tile to become half a chunk per lane and is evaluated for all scales
// while the loads of the second half are still in flight.  Tree over the 64 chunk sums by DPP.
constexpr int kHalfStride = 36;        // floats between chunks in the half-chunk tile (32 + 4: keeps 16-byte alignment)

__device__ __forceinline__ void probe_fetch(const float* __restrict__ x, long long N, long long base, int h, int lane,
                                            bool aligned, float4 (&stg)[8])
{
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int f = r * 64 + lane;                         // float4 number inside the half: chunk f / 8, position f % 8
        const long long e = base + (long long)(f >> 3) * kChunk + h * 32 + (f & 7) * 4;
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (aligned && e + 4 <= N) {
            v = *reinterpret_cast<const float4*>(x + e);
        } else if (e < N) {
            v.x = x[e];
            if (e + 1 < N) v.y = x[e + 1];
            if (e + 2 < N) v.z = x[e + 2];
            if (e + 3 < N) v.w = x[e + 3];
        }
        stg[r] = v;
    }
}

__device__ __forceinline__ void probe_stage(float* tile, const ActPreV& V, long long N, long long base, int h, int lane,
                                            const float4 (&stg)[8], float (&xr)[32])
{
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int f = r * 64 + lane;
        float4 v = stg[r];
        if (V.mode != 0) {                                   // padding stays exactly zero
            const long long e = base + (long long)(f >> 3) * kChunk + h * 32 + (f & 7) * 4;
            if (e < N) v.x = act_pre(V, v.x);
            if (e + 1 < N) v.y = act_pre(V, v.y);
            if (e + 2 < N) v.z = act_pre(V, v.z);
            if (e + 3 < N) v.w = act_pre(V, v.w);
        }
        *reinterpret_cast<float4*>(tile + (f >> 3) * kHalfStride + (f & 7) * 4) = v;
    }
    wave_lds_sync();
    const float4* t4 = reinterpret_cast<const float4*>(tile + lane * kHalfStride);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float4 v = t4[i];
        xr[4 * i + 0] = v.x; xr[4 * i + 1] = v.y; xr[4 * i + 2] = v.z; xr[4 * i + 3] = v.w;
    }
    wave_lds_sync();
}

__device__ __forceinline__ void probe_eval(const float (&xr)[32], int np, const float (&pr)[kMaxProbes],
                                           const float (&pinv)[kMaxProbes], float lo, float hi, float (&s)[kMaxProbes])
{
#pragma unroll
    for (int pi = 0; pi < kMaxProbes; ++pi) {
        if (pi < np) {
            float sp[1] = {s[pi]};
            const float al[1] = {pr[pi]}, iv[1] = {pinv[pi]};
#pragma unroll
            for (int i = 0; i < 32; i += 8) {
                const float xs[8] = {xr[i], xr[i + 1], xr[i + 2], xr[i + 3], xr[i + 4], xr[i + 5], xr[i + 6], xr[i + 7]};
                eval_stage<8, 1>(xs, al, iv, lo, hi, sp);
            }
            s[pi] = sp[0];
        }
    }
}

__global__ void __launch_bounds__(256) k_act_probe(const ActBatch B, float lo, float hi, double* probe0, const ActPre pre)
{
    __shared__ float4 tile4[4][64 * kHalfStride / 4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int blk = blockIdx.x * 4 + wave;                    // block in the concatenated numbering
    const int total = B.start[B.count];
    if (blk >= total) return;                                 // the waves of a workgroup are independent: no barriers below
    const int t = act_find(B, blk);
    const ActState* S = B.S + t;
    if (S->status != 0 || S->done) return;
    const float* __restrict__ x = B.x[t];
    const long long N = B.N[t];
    const ActPreV V = act_pre_load(pre);
    const int np = S->nprobe;
    const long long base = (long long)(blk - B.start[t]) * kBlockElems;   // first element of this wave's block
    float* tile = reinterpret_cast<float*>(tile4[wave]);
    const bool aligned = (reinterpret_cast<uintptr_t>(x) & 15u) == 0;

    float4 stg0[8], stg1[8];
    probe_fetch(x, N, base, 0, lane, aligned, stg0);
    probe_fetch(x, N, base, 1, lane, aligned, stg1);
    // the scales of this pass (unused slots hold 1.0)
    float pr[kMaxProbes], pinv[kMaxProbes], s[kMaxProbes];
#pragma unroll
    for (int i = 0; i < kMaxProbes; ++i) pr[i] = S->probes[i];
#pragma unroll
    for (int i = 0; i < kMaxProbes; ++i) { pinv[i] = 1.0f / pr[i]; s[i] = 0.0f; }

    float xr[32];
    probe_stage(tile, V, N, base, 0, lane, stg0, xr);
    probe_eval(xr, np, pr, pinv, lo, hi, s);
    probe_stage(tile, V, N, base, 1, lane, stg1, xr);
    probe_eval(xr, np, pr, pinv, lo, hi, s);

    // pairwise tree over the 64 chunk sums: lane i (a multiple of 2w) adds lane i + w; four levels inside
    // rows of 16 lanes by DPP shifts, the last two on the four row heads as scalar operands
#pragma unroll
    for (int pi = 0; pi < kMaxProbes; ++pi) {
        if (pi < np) {
            double v = (double)s[pi];
            v = v + dpp_row_shl<1>(v);
            v = v + dpp_row_shl<2>(v);
            v = v + dpp_row_shl<4>(v);
            v = v + dpp_row_shl<8>(v);
            const double r0 = readlane_f64(v, 0), r1 = readlane_f64(v, 16), r2 = readlane_f64(v, 32), r3 = readlane_f64(v, 48);
            const double tot = (r0 + r1) + (r2 + r3);
            if (lane == 0) probe0[(size_t)blk * kMaxProbes + pi] = tot;
        }
    }
}

// Last tree level(s) over <= 64 rows of per-scale sums, then the golden-section bookkeeping.
__global__ void __launch_bounds__(64) k_act_finish(const ActBatch B, int level, const double* __restrict__ part, int iters,
                                                   const ActOut O)
{
    __shared__ double vals[kMaxProbes];
    ActState* S = B.S + blockIdx.x;
    if (S->status != 0 || S->done) return;
    float* scale = O.scale[blockIdx.x];
    double* sse = O.sse[blockIdx.x];
    int first = 0;
    for (int u = 0; u < (int)blockIdx.x; ++u) first += act_rows(B.start[u + 1] - B.start[u], level);
    const int rows = act_rows(B.start[blockIdx.x + 1] - B.start[blockIdx.x], level);
    part += (size_t)first * kMaxProbes;
    const int t = threadIdx.x;
    if (t < kMaxProbes) {
        double v[64];
#pragma unroll
        for (int i = 0; i < 64; ++i) v[i] = (i < rows && t < S->nprobe) ? part[(size_t)i * kMaxProbes + t] : 0.0;
#pragma unroll
        for (int w = 1; w < 64; w <<= 1)
#pragma unroll
            for (int i = 0; i < 64; i += 2 * w) v[i] = v[i] + v[i + w];
        vals[t] = v[0];
    }
    __syncthreads();
    if (t == 0) {
        act_advance(S, vals, iters);
        act_plan(S, iters);
        *scale = S->best_a;
        *sse = S->best;
    }
}

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

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
    const int G = p->grid_points;
    if (G <= 512) return 1;     // one candidate per lane: most waves per SIMD, which the dual-issue VALU needs
    if (G <= 1024) return 2;
    return 4;
}

bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_tensor(const mmse_tensor_desc_t& d, bool need_outputs)
{
    if (!d.w_dev) return MMSE_ERR_NULL;
    if (need_outputs && (!d.scale_dev || !d.idx_dev || !d.sse_dev)) return MMSE_ERR_NULL;
    if (d.K <= 0 || d.n <= 0 || d.n > MMSE_MAX_KERNEL_ELEMS) return MMSE_ERR_SIZE;
    if (d.K > MMSE_MAX_TENSOR_ELEMS / d.n) return MMSE_ERR_SIZE;
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

template <int C>
int launch_sweep(const Batch& B, int nwg, int G, int max_npad, hipStream_t s)
{
    const int waves = (G + 64 * C - 1) / (64 * C);
    const size_t lds = (size_t)(max_npad < kTile ? max_npad : kTile) * sizeof(float);
    if (max_npad <= kTile)
        hipLaunchKernelGGL((k_sweep_kernelwise<C, kLevelsKWSmall>), dim3(nwg), dim3(64 * waves), lds, s, B);
    else
        hipLaunchKernelGGL((k_sweep_kernelwise<C, kLevelsKW>), dim3(nwg), dim3(64 * waves), lds, s, B);
    return hipGetLastError() == hipSuccess ? MMSE_OK : MMSE_ERR_LAUNCH;
}

int launch_sweep_any(int C, const Batch& B, int nwg, int G, int max_npad, hipStream_t s)
{
    if (C == 1) return launch_sweep<1>(B, nwg, G, max_npad, s);
    if (C == 2) return launch_sweep<2>(B, nwg, G, max_npad, s);
    return launch_sweep<4>(B, nwg, G, max_npad, s);
}

struct Item {              // one tensor of a batched call, host side
    TensorArgs a;
    int order;
};

// The three stages for a list of tensors (already validated): sweep, refine, pack.
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
    if (do_search) {
        // kernels of <= 64 elements go to the one-wave-per-kernel path (when the grid fits 8 candidates a lane)
        // ... and when there are enough of them to pay for a launch of their own
        long long small_rows = 0;
        for (int i = 0; i < count; ++i)
            if (items[i].a.n <= kChunk) small_rows += items[i].a.K;
        const bool small_ok = G <= 512 && small_rows >= 2048;
        for (int pass = 0; pass < 2; ++pass) {                 // 0: general kernels, 1: small ones
            Batch B{};
            fill_common(B, p);
            int nb = 0, wg = 0, max_npad = 0;
            auto flush = [&]() -> int {
                if (nb == 0) return MMSE_OK;
                B.start[nb] = wg;
                B.count = nb;
                int rc = MMSE_OK;
                if (pass == 0) {
                    rc = launch_sweep_any(C, B, wg, G, max_npad, s);
                } else {
                    const int cs = (G + 63) / 64;
                    if (cs <= 1) hipLaunchKernelGGL(k_sweep_small<1>, dim3(wg), dim3(256), 0, s, B);
                    else if (cs <= 2) hipLaunchKernelGGL(k_sweep_small<2>, dim3(wg), dim3(256), 0, s, B);
                    else if (cs <= 4) hipLaunchKernelGGL(k_sweep_small<4>, dim3(wg), dim3(256), 0, s, B);
                    else hipLaunchKernelGGL(k_sweep_small<8>, dim3(wg), dim3(256), 0, s, B);
                    rc = hipGetLastError() == hipSuccess ? MMSE_OK : MMSE_ERR_LAUNCH;
                }
                nb = 0; wg = 0; max_npad = 0;
                return rc;
            };
            for (int i = 0; i < count; ++i) {
                const TensorArgs& a = items[i].a;
                const bool small = small_ok && a.n <= kChunk;
                if (small != (pass == 1)) continue;
                B.t[nb] = a;
                B.start[nb] = wg;
                wg += pass == 0 ? a.K : (a.K + 3) / 4;
                const int npad = (a.n + kChunk - 1) & ~(kChunk - 1);
                max_npad = npad > max_npad ? npad : max_npad;
                if (++nb == kMaxBatch) { const int rc = flush(); if (rc) return rc; }
            }
            const int rc = flush();
            if (rc) return rc;
        }
        if (p->refine_iters > 0) {
            // classes: kernels of <= 16 elements (one lane each, 16 slots), then by lanes per kernel
            for (int cls = 0; cls < 4; ++cls) {
                const int threads = cls == 3 ? 1024 : (cls == 2 ? 512 : 256);
                Batch B{};
                fill_common(B, p);
                int nb = 0, wg = 0;
                auto flush = [&]() -> int {
                    if (nb == 0) return MMSE_OK;
                    B.start[nb] = wg;
                    B.count = nb;
                    // LDS: combine buffer (2 doubles per thread) + one transpose tile per wave
                    const int tile_chunks = cls == 0 ? 0 : 32 * 256 / threads;
                    const size_t lds = (size_t)threads * 2 * sizeof(double) +
                                       (size_t)(threads / 64) * tile_chunks * kTileStride * sizeof(float);
                    if (cls == 0) hipLaunchKernelGGL(k_refine_kernelwise<16>, dim3(wg), dim3(threads), lds, s, B, tile_chunks);
                    else hipLaunchKernelGGL(k_refine_kernelwise<kChunk>, dim3(wg), dim3(threads), lds, s, B, tile_chunks);
                    nb = 0; wg = 0;
                    return hipGetLastError() == hipSuccess ? MMSE_OK : MMSE_ERR_LAUNCH;
                };
                for (int i = 0; i < count; ++i) {
                    const TensorArgs& a = items[i].a;
                    const int m = (a.n + kChunk - 1) / kChunk;
                    const int c = a.n <= 16 ? 0 : (m <= 256 ? 1 : (m <= 512 ? 2 : 3));
                    if (c != cls) continue;
                    const int lanes = cls == 0 ? 1 : m;
                    const int cpw = threads / lanes;
                    B.t[nb] = a;
                    if (a.n & 1) B.t[nb].packed = nullptr;     // odd n: bytes straddle kernels, k_pack_int4 does those
                    B.start[nb] = wg;
                    wg += (a.K + cpw - 1) / cpw;
                    if (++nb == kMaxBatch) { const int rc = flush(); if (rc) return rc; }
                }
                const int rc = flush();
                if (rc) return rc;
            }
        }
    }
    // pack
    {
        Batch B{};
        fill_common(B, p);
        int nb = 0, wg = 0;
        auto flush = [&]() -> int {
            if (nb == 0) return MMSE_OK;
            B.start[nb] = wg;
            B.count = nb;
            hipLaunchKernelGGL(k_pack_int4, dim3(wg), dim3(kPackThreads), 0, s, B);
            nb = 0; wg = 0;
            return hipGetLastError() == hipSuccess ? MMSE_OK : MMSE_ERR_LAUNCH;
        };
        for (int i = 0; i < count; ++i) {
            const TensorArgs& a = items[i].a;
            if (!a.packed) continue;
            if (do_search && p->refine_iters > 0 && (a.n & 1) == 0) continue;   // coded by the refinement kernel
            const long long total = (long long)a.K * a.n;
            const long long per_wg = (long long)kPackThreads * kPackPerThread;
            B.t[nb] = a;
            B.start[nb] = wg;
            wg += (int)((total + per_wg - 1) / per_wg);
            if (++nb == kMaxBatch) { const int rc = flush(); if (rc) return rc; }
        }
        const int rc = flush();
        if (rc) return rc;
    }
    return MMSE_OK;
}

// Codes of the searched tensors (input, residual or shifted input) for their final scales: one
// workgroup per 4096-element block, 8 elements -> one 32-bit store, two such groups per thread;
// a rejected tensor (scale NaN) is coded as zeros.
__global__ void __launch_bounds__(kPackThreads) k_act_pack(const ActBatch B, const ActPre pre, const ActOut O,
                                                           float lo, float hi)
{
    const int t = act_find(B, blockIdx.x);
    const float* __restrict__ x = B.x[t];
    const long long N = B.N[t];
    uint8_t* __restrict__ packed = O.packed[t];
    if (!packed) return;
    const ActPreV V = act_pre_load(pre);
    const float sc = *O.scale[t], inv = 1.0f / sc;
    const long long blk0 = (long long)(blockIdx.x - B.start[t]) * kBlockElems;
#pragma unroll
    for (int h = 0; h < kBlockElems / (kPackThreads * kPackPerThread); ++h) {
        const long long e0 = blk0 + ((long long)h * kPackThreads + threadIdx.x) * kPackPerThread;
        if (e0 >= N) continue;
        const int cnt = (N - e0) < kPackPerThread ? (int)(N - e0) : kPackPerThread;
        float v[kPackPerThread];
        if (cnt == kPackPerThread && (reinterpret_cast<uintptr_t>(x) & 15u) == 0) {
            const float4 p0 = reinterpret_cast<const float4*>(x + e0)[0];
            const float4 p1 = reinterpret_cast<const float4*>(x + e0)[1];
            v[0] = p0.x; v[1] = p0.y; v[2] = p0.z; v[3] = p0.w;
            v[4] = p1.x; v[5] = p1.y; v[6] = p1.z; v[7] = p1.w;
        } else {
#pragma unroll
            for (int i = 0; i < kPackPerThread; ++i) v[i] = (i < cnt) ? x[e0 + i] : 0.0f;
        }
        unsigned word = 0;
#pragma unroll
        for (int i = 0; i < kPackPerThread; ++i) {
            if (i < cnt) {
                const int q = (sc == sc) ? (int)code_of(act_pre(V, v[i]), inv, lo, hi) : 0;
                word |= ((unsigned)q & 0xFu) << (4 * i);
            }
        }
        uint8_t* dst = packed + (e0 >> 1);
        if (cnt == kPackPerThread && (reinterpret_cast<uintptr_t>(packed) & 3u) == 0) {
            *reinterpret_cast<unsigned*>(dst) = word;
        } else {
            const int nbytes = (cnt + 1) >> 1;
            for (int b = 0; b < nbytes; ++b) dst[b] = (uint8_t)(word >> (8 * b));
        }
    }
}

struct ActPlan {
    int count;
    int start[kMaxActBatch + 1];   // first block of each tensor in the concatenated numbering
    int levels;             // reduce64 stages of the grid sums until every tensor has one row
    int plevels;            // reduce64 stages of the probe sums until every tensor has <= 64 rows
    int total_rows[8];      // rows of all tensors together at each level
    size_t off_part[8];     // byte offsets of the grid-sum levels ([rows][G] doubles)
    size_t off_probe[8];    // byte offsets of the probe levels ([rows][kMaxProbes] doubles)
    size_t bytes;
};

// Workspace of one launch group: the states, then the levels of the grid sums, then those of the probe sums.
ActPlan plan_activation(const long long* N, int count, int G)
{
    ActPlan P{};
    P.count = count;
    int maxnb = 1;
    for (int t = 0; t < count; ++t) {
        const int nb = (int)((N[t] + kBlockElems - 1) / kBlockElems);
        P.start[t + 1] = P.start[t] + nb;
        maxnb = nb > maxnb ? nb : maxnb;
    }
    while (act_rows(maxnb, P.levels) > 1) ++P.levels;
    while (act_rows(maxnb, P.plevels) > 64) ++P.plevels;
    for (int l = 0; l <= P.levels; ++l) {
        int r = 0;
        for (int t = 0; t < count; ++t) r += act_rows(P.start[t + 1] - P.start[t], l);
        P.total_rows[l] = r;
    }
    size_t off = round256(sizeof(ActState) * (size_t)count);
    for (int l = 0; l <= P.levels; ++l) { P.off_part[l] = off; off += round256((size_t)P.total_rows[l] * G * sizeof(double)); }
    for (int l = 0; l <= P.plevels; ++l) { P.off_probe[l] = off; off += round256((size_t)P.total_rows[l] * kMaxProbes * sizeof(double)); }
    P.bytes = off;
    return P;
}

// passes over the tensor that the refinement needs: the first settles 4 evaluations, each later one 3
int refine_passes(int iters)
{
    if (iters <= 0) return 0;
    return 1 + (iters > 2 ? (iters - 2 + 2) / 3 : 0);
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
    *bytes_out = plan_activation(&n1, 1, p->grid_points).bytes;
    return MMSE_OK;
}

int mmse_workspace_bytes_activation_batched(const int64_t* N_host, int32_t count, const mmse_params_t* p, size_t* bytes_out)
{
    if (!bytes_out || !N_host) return MMSE_ERR_NULL;
    const int rc = check_params(p);
    if (rc) return rc;
    if (count <= 0 || count > MMSE_MAX_BATCH_TENSORS) return MMSE_ERR_SIZE;
    size_t total = 0;
    for (int g0 = 0; g0 < count; g0 += kMaxActBatch) {
        long long n[kMaxActBatch];
        const int m = (count - g0) < kMaxActBatch ? (count - g0) : kMaxActBatch;
        for (int i = 0; i < m; ++i) {
            if (N_host[g0 + i] <= 0 || N_host[g0 + i] > MMSE_MAX_TENSOR_ELEMS) return MMSE_ERR_SIZE;
            n[i] = N_host[g0 + i];
        }
        total += plan_activation(n, m, p->grid_points).bytes;
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
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < round256((size_t)sumK * sizeof(float)))
        return MMSE_ERR_WORKSPACE;
    Item* items = new Item[count]();       // value-initialised: every optional pointer starts as nullptr
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
    delete[] items;
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
    if (K <= 0 || n <= 0 || n > MMSE_MAX_KERNEL_ELEMS || K > MMSE_MAX_TENSOR_ELEMS / n) return MMSE_ERR_SIZE;
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
        if (d.K <= 0 || d.n <= 0 || d.n > MMSE_MAX_KERNEL_ELEMS || d.K > MMSE_MAX_TENSOR_ELEMS / d.n) return MMSE_ERR_SIZE;
        if (!aligned_to(d.w_dev, 4) || !aligned_to(d.scale1_dev, 4) || !aligned_to(d.scale2_dev, 4) ||
            !aligned_to(d.sse_dev, 8) || !aligned_to(d.sweeps_dev, 4))
            return MMSE_ERR_ALIGN;
        need += plan_dual(d.K, d.n).bytes;
    }
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < need) return MMSE_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    struct W { float* absmax; int32_t* idx; float *ts1, *ts2; double *tsse1, *tsse; uint8_t *active, *accepted, *tp1, *tp2; };
    W* wk = new W[count]();
    Item* items = new Item[count]();
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
        for (int b0 = 0; b0 < count; b0 += kMaxDualBatch) {
            DualBatch D{};
            D.eps = eps;
            const int nb = (count - b0) < kMaxDualBatch ? (count - b0) : kMaxDualBatch;
            int wg = 0;
            for (int j = 0; j < nb; ++j) {
                const mmse_dual_desc_t& d = descs_host[b0 + j];
                const W& w = wk[b0 + j];
                DualTensor& T = D.t[j];
                T.sse = d.sse_dev; T.tsse = w.tsse; T.s1 = d.scale1_dev; T.ts1 = w.ts1; T.s2 = d.scale2_dev; T.ts2 = w.ts2;
                T.sweeps = d.sweeps_dev; T.active = w.active; T.accepted = w.accepted;
                T.tp1 = w.tp1; T.p1 = d.packed1_dev; T.tp2 = w.tp2; T.p2 = d.packed2_dev;
                T.K = (int)d.K; T.n = (int)d.n;
                D.start[j] = wg;
                const long long units = kind == 2 ? ((long long)d.K * d.n + 1) / 2 : d.K;
                wg += (int)((units + 255) / 256);
            }
            D.start[nb] = wg;
            D.count = nb;
            if (kind == 0) hipLaunchKernelGGL(k_dual_init, dim3(wg), dim3(256), 0, s, D);
            else if (kind == 1) hipLaunchKernelGGL(k_dual_accept, dim3(wg), dim3(256), 0, s, D);
            else hipLaunchKernelGGL(k_dual_copy_codes, dim3(wg), dim3(256), 0, s, D);
            if (hipGetLastError() != hipSuccess) return MMSE_ERR_LAUNCH;
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
        if (d.K <= 0 || d.n <= 0 || d.n > MMSE_MAX_KERNEL_ELEMS || d.K > MMSE_MAX_TENSOR_ELEMS / d.n) return MMSE_ERR_SIZE;
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

int mmse_scale_alternating_kernelwise(const float* w_dev, int64_t K, int64_t n, int32_t qmin, int32_t qmax,
                                      int32_t max_iters, float* scale_dev, double* sse_dev, int32_t* updates_dev,
                                      void* stream)
{
    if (!w_dev || !scale_dev || !sse_dev || !updates_dev) return MMSE_ERR_NULL;
    if (K <= 0 || n <= 0 || n > MMSE_MAX_KERNEL_ELEMS || K > MMSE_MAX_TENSOR_ELEMS / n) return MMSE_ERR_SIZE;
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
    if (K <= 0 || n <= 0 || n > kTile || K > MMSE_MAX_TENSOR_ELEMS / n) return MMSE_ERR_SIZE;
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
    if (K <= 0 || n <= 0 || n > kTile || K > MMSE_MAX_TENSOR_ELEMS / n) return MMSE_ERR_SIZE;
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
                                char* ws, const ActPlan& P, hipStream_t s)
{
    const int G = p->grid_points;
    ActBatch B{};
    ActOut O{};
    bool any_packed = false;
    long long maxN = 0;
    for (int t = 0; t < count; ++t) {
        B.x[t] = items[t].x; B.N[t] = items[t].N; B.start[t] = P.start[t];
        O.scale[t] = items[t].scale; O.idx[t] = items[t].idx; O.sse[t] = items[t].sse; O.packed[t] = items[t].packed;
        any_packed = any_packed || items[t].packed != nullptr;
        maxN = items[t].N > maxN ? items[t].N : maxN;
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
#define MMSE_CHECK_LAUNCH() do { if (hipGetLastError() != hipSuccess) return MMSE_ERR_LAUNCH; } while (0)

    hipLaunchKernelGGL(k_act_init, dim3(1), dim3(64), 0, s, S, count);
    MMSE_CHECK_LAUNCH();
    {
        // per tensor at most one workgroup per CU, eight 16-byte loads in flight per thread: measured fastest
        // on MI355X (6.9 TB/s on a 205 MB tensor; more, smaller workgroups lose up to 2x)
        constexpr int U = 8;
        long long want = (maxN + 1024 * U - 1) / (1024 * U);
        const int grid = (int)(want < 256 ? (want < 1 ? 1 : want) : 256);
        const dim3 g(grid, count);
        if (pre_mode == 0) hipLaunchKernelGGL((k_act_absmax<U, 0>), g, dim3(256), 0, s, B, pre);
        else if (pre_mode == 1) hipLaunchKernelGGL((k_act_absmax<U, 1>), g, dim3(256), 0, s, B, pre);
        else hipLaunchKernelGGL((k_act_absmax<U, 2>), g, dim3(256), 0, s, B, pre);
        MMSE_CHECK_LAUNCH();
        if (pre_mode == 2) {
            hipLaunchKernelGGL(k_act_offset_setup, dim3(1), dim3(64), 0, s, S, delta_dev);
            MMSE_CHECK_LAUNCH();
        }
    }
    {
        const int C = pick_cands(p);
        const int waves = (G + 64 * C - 1) / (64 * C);
        double* part0 = reinterpret_cast<double*>(ws + P.off_part[0]);
        if (C == 1) hipLaunchKernelGGL(k_act_sweep<1>, dim3(total), dim3(64 * waves), 0, s, B, G, p->qmax, lo, hi, part0, pre);
        else if (C == 2) hipLaunchKernelGGL(k_act_sweep<2>, dim3(total), dim3(64 * waves), 0, s, B, G, p->qmax, lo, hi, part0, pre);
        else hipLaunchKernelGGL(k_act_sweep<4>, dim3(total), dim3(64 * waves), 0, s, B, G, p->qmax, lo, hi, part0, pre);
        MMSE_CHECK_LAUNCH();
    }
    for (int l = 0; l < P.levels; ++l) {
        hipLaunchKernelGGL(k_act_reduce64, dim3((G + 255) / 256, P.total_rows[l + 1]), dim3(256), 0, s, B, l + 1,
                           reinterpret_cast<const double*>(ws + P.off_part[l]), G,
                           reinterpret_cast<double*>(ws + P.off_part[l + 1]));
        MMSE_CHECK_LAUNCH();
    }
    {
        int threads = ((G + 63) / 64) * 64;
        if (threads > 1024) threads = 1024;
        hipLaunchKernelGGL(k_act_argmin, dim3(count), dim3(threads), 0, s, B,
                           reinterpret_cast<const double*>(ws + P.off_part[P.levels]), G, p->qmax, p->refine_iters, O);
        MMSE_CHECK_LAUNCH();
    }
    for (int pass = 0; pass < refine_passes(p->refine_iters); ++pass) {
        hipLaunchKernelGGL(k_act_probe, dim3((total + 3) / 4), dim3(256), 0, s, B, lo, hi,
                           reinterpret_cast<double*>(ws + P.off_probe[0]), pre);
        MMSE_CHECK_LAUNCH();
        for (int l = 0; l < P.plevels; ++l) {
            hipLaunchKernelGGL(k_act_reduce64, dim3(1, P.total_rows[l + 1]), dim3(64), 0, s, B, l + 1,
                               reinterpret_cast<const double*>(ws + P.off_probe[l]), kMaxProbes,
                               reinterpret_cast<double*>(ws + P.off_probe[l + 1]));
            MMSE_CHECK_LAUNCH();
        }
        hipLaunchKernelGGL(k_act_finish, dim3(count), dim3(64), 0, s, B, P.plevels,
                           reinterpret_cast<const double*>(ws + P.off_probe[P.plevels]), p->refine_iters, O);
        MMSE_CHECK_LAUNCH();
    }
    if (any_packed) {
        hipLaunchKernelGGL(k_act_pack, dim3(total), dim3(kPackThreads), 0, s, B, pre, O, lo, hi);
        MMSE_CHECK_LAUNCH();
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
    const ActPlan P = plan_activation(&n1, 1, p->grid_points);
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < P.bytes) return MMSE_ERR_WORKSPACE;
    const ActItem item{x_dev, n1, scale_dev, idx_dev, sse_dev, packed_dev};
    return run_activation_group(&item, 1, p, pre_mode, scale1_dev, qmin1, qmax1, delta_dev,
                                static_cast<char*>(ws_dev), P, static_cast<hipStream_t>(stream));
}

int mmse_scale_search_activation_batched(const mmse_act_desc_t* descs_host, int32_t count, const mmse_params_t* p,
                                         void* ws_dev, size_t ws_bytes, void* stream)
{
    int rc = check_params(p);
    if (rc) return rc;
    if (!descs_host) return MMSE_ERR_NULL;
    if (count <= 0 || count > MMSE_MAX_BATCH_TENSORS) return MMSE_ERR_SIZE;
    size_t need = 0;
    for (int i = 0; i < count; ++i) {
        const mmse_act_desc_t& d = descs_host[i];
        if (!d.x_dev || !d.scale_dev || !d.idx_dev || !d.sse_dev) return MMSE_ERR_NULL;
        if (d.N <= 0 || d.N > MMSE_MAX_TENSOR_ELEMS) return MMSE_ERR_SIZE;
        if (!aligned_to(d.x_dev, 4) || !aligned_to(d.scale_dev, 4) || !aligned_to(d.idx_dev, 4) || !aligned_to(d.sse_dev, 8))
            return MMSE_ERR_ALIGN;
    }
    // groups of at most kMaxActBatch tensors, each with its own slice of the workspace
    ActPlan plans[(MMSE_MAX_BATCH_TENSORS + kMaxActBatch - 1) / kMaxActBatch];
    int ngroups = 0;
    for (int g0 = 0; g0 < count; g0 += kMaxActBatch, ++ngroups) {
        long long n[kMaxActBatch];
        const int m = (count - g0) < kMaxActBatch ? (count - g0) : kMaxActBatch;
        for (int i = 0; i < m; ++i) n[i] = descs_host[g0 + i].N;
        plans[ngroups] = plan_activation(n, m, p->grid_points);
        need += plans[ngroups].bytes;
    }
    if (!ws_dev || !aligned_to(ws_dev, 256) || ws_bytes < need) return MMSE_ERR_WORKSPACE;
    char* ws = static_cast<char*>(ws_dev);
    for (int g = 0; g < ngroups; ++g) {
        ActItem items[kMaxActBatch];
        const int g0 = g * kMaxActBatch;
        const int m = plans[g].count;
        for (int i = 0; i < m; ++i) {
            const mmse_act_desc_t& d = descs_host[g0 + i];
            items[i] = ActItem{d.x_dev, (long long)d.N, d.scale_dev, d.idx_dev, d.sse_dev, d.packed_dev};
        }
        rc = run_activation_group(items, m, p, 0, nullptr, 0, 0, nullptr, ws, plans[g], static_cast<hipStream_t>(stream));
        if (rc) return rc;
        ws += plans[g].bytes;
    }
    return MMSE_OK;
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
