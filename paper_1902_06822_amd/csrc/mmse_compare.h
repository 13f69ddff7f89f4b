// mmse_compare.h -- the alternating optimiser the paper compares against (Section 3.4, Table 2).
#ifndef MMSE_COMPARE_H_
#define MMSE_COMPARE_H_
#include "mmse_common.h"

namespace {

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
        __syncthreads();                   // s_stop, s_alpha and s_den are rewritten by the next iteration
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

}  // namespace

#endif  // MMSE_COMPARE_H_
