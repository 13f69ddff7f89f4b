// mmse_dual.h -- two INT4 tensors per kernel: bookkeeping of Algorithm 1 iterated, and the dual line search of Eq. 12.
#ifndef MMSE_DUAL_H_
#define MMSE_DUAL_H_
#include "mmse_common.h"

namespace {

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

// Codes of the kernels whose sweep was kept move from the tentative to the kept buffers: 16 bytes (32 codes)
// per thread in one piece where they belong to one kernel, else nibble by nibble (a byte can hold codes of
// two kernels when n is odd).
__global__ void __launch_bounds__(256) k_dual_copy_codes(const DualBatch D)
{
    const int t = find_dual_tensor(D, blockIdx.x);
    const DualTensor& T = D.t[t];
    const long long total = (long long)T.K * T.n;
    const long long nbytes = (total + 1) >> 1;
    const long long b0 = ((long long)(blockIdx.x - D.start[t]) * blockDim.x + threadIdx.x) * 16;
    if (b0 >= nbytes) return;
    const unsigned n = (unsigned)T.n;
    const long long elast = (2 * b0 + 31 < total) ? 2 * b0 + 31 : total - 1;
    const unsigned k0 = (unsigned)(2 * b0) / n, k1 = (unsigned)elast / n;       // K * n < 2^31
    const uintptr_t al = reinterpret_cast<uintptr_t>(T.p1) | reinterpret_cast<uintptr_t>(T.tp1) |
                         reinterpret_cast<uintptr_t>(T.p2) | reinterpret_cast<uintptr_t>(T.tp2);
    if (k0 == k1 && b0 + 16 <= nbytes && (al & 15u) == 0) {
        if (T.accepted[k0] != 0) {
            *reinterpret_cast<uint4*>(T.p1 + b0) = *reinterpret_cast<const uint4*>(T.tp1 + b0);
            *reinterpret_cast<uint4*>(T.p2 + b0) = *reinterpret_cast<const uint4*>(T.tp2 + b0);
        }
        return;
    }
    for (int j = 0; j < 16; ++j) {
        const long long b = b0 + j;
        if (b >= nbytes) break;
        const unsigned e0 = (unsigned)(2 * b);
        const bool a0 = T.accepted[e0 / n] != 0;
        const bool a1 = (long long)e0 + 1 < total && T.accepted[(e0 + 1) / n] != 0;
        if (!a0 && !a1) continue;
        const unsigned mask = (a0 ? 0x0Fu : 0u) | (a1 ? 0xF0u : 0u);
        T.p1[b] = (uint8_t)((T.p1[b] & ~mask) | (T.tp1[b] & mask));
        T.p2[b] = (uint8_t)((T.p2[b] & ~mask) | (T.tp2[b] & mask));
    }
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

}  // namespace

#endif  // MMSE_DUAL_H_
