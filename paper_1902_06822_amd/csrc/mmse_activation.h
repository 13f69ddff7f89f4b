// mmse_activation.h -- per-layer activation path: one or many tensors spread over the whole GPU (Section 3.7), with the residual and offset variants.
#ifndef MMSE_ACTIVATION_H_
#define MMSE_ACTIVATION_H_
#include "mmse_common.h"

namespace {

// ---------------------------------------------------------------------------------
// activation tensor: one problem of N elements over the whole GPU
// ---------------------------------------------------------------------------------
// Workspace layout (all offsets multiples of 256 bytes):
//   ActState                              scalars of the search
//   part0[nb][G] doubles                  per-block tree sums of the grid sweep
//   part1[ceil(nb/64)][G], part2, ...     upper tree levels, 64 blocks at a time
//   probe0[nb], probe1[...], ...          same hierarchy for one refinement probe
// What the activation kernels search instead of the stored tensor (formed as the tensor is read; the grid sweep leaves
// its non-zero values in the workspace for the refinement passes, see k_act_sweep):
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
        for (int i = 0; i < kMaxProbes; ++i) { S->probes[i] = 1.0f; S->probe_inv[i] = 1.0f; }
        S->ec = S->ed = S->best = 0.0;
        S->min_key = 0xffffffffu; S->max_key = 0u; S->delta = 0.0f;
    }
}

// MODE 0: max |x| (integer max of the bit patterns); 1: max |residual of the first tensor|;
// 2: min and max of x as order-preserving keys (offset form).
// Large workgroups: the pass needs some 50 MB of loads in flight to fill HBM, and every workgroup ends with one
// atomic on its tensor's state word; atomics on one address retire one after the other (about 9 ns each on
// MI355X), and all workgroups finish together, so there should be few of them.
constexpr int kAbsmaxThreads = 1024;
template <int U, int MODE>
__global__ void __launch_bounds__(kAbsmaxThreads) k_act_absmax(const ActBatch B, const ActPre pre)
{
    const float* __restrict__ x = B.x[blockIdx.y];
    const long long N = B.N[blockIdx.y];
    ActState* S = B.S + blockIdx.y;
    if ((long long)blockIdx.x * blockDim.x * 4 * U >= N) return;       // nothing of this tensor for this workgroup
    __shared__ unsigned s_amax[kAbsmaxThreads / 64];
    __shared__ unsigned s_amin[kAbsmaxThreads / 64];
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
                v[u] = load_stream_f4(x + base + ((long long)u * blockDim.x + threadIdx.x) * 4);
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

// Where a chunk of a block's compacted copy starts (floats from the start of the block's 4096-float slot, a multiple
// of 8, at most 4096 - its length) and how many elements it has there (a multiple of 8, at most 64), as one word.
__device__ __forceinline__ unsigned compact_meta(int off, int len) { return (unsigned)off | ((unsigned)len << 16); }
__device__ __forceinline__ int compact_off(unsigned m) { return (int)(m & 0xffffu); }
__device__ __forceinline__ int compact_len(unsigned m) { return (int)(m >> 16); }

// Grid sweep of one 4096-element block per workgroup; waves split the candidates.  With sets > 1 (2, 4 or 8) the
// waves form that many sets that each cover all candidates and take one aligned part of the block (32, 16 or 8
// chunks) each: the parts are the subtrees at one level of the block's pairwise tree, so set 0 adds their sums
// pairwise at the end (one exchange through LDS; a part that lies beyond a ragged block contributes an exact 0).
// Two sets keep four waves per workgroup, and with them eight waves per SIMD within the LDS of a CU, for grids that
// two candidates per lane would otherwise cover with two waves; four and eight sets are for calls of so few blocks
// that the machine is not full, where they shorten the one sweep every wave has to get through.
constexpr int kMaxSplitCands = 384;
constexpr int kMaxExchange = kBlockElems / 2;           // doubles that fit the slice once it has been swept

template <int C>
__global__ void __launch_bounds__(512) k_act_sweep(const ActBatch B, int G, int qmax,
                                                    float lo, float hi, double* part0, const ActPre pre, int sets,
                                                    float* compact, unsigned* meta)
{
    __shared__ float4 slice4[kBlockElems / 4];
    __shared__ unsigned s_bounds[kBlockChunks];             // largest bound_key of every chunk of the block
    __shared__ int s_len[kBlockChunks];                     // its length once compacted to its non-zero elements (low
                                                            // byte; above it, where its copy in the workspace starts)
    float* slice = reinterpret_cast<float*>(slice4);
    const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x;
    const int wps = (nthreads >> 6) / sets;                             // waves per set
    const int set = (tid >> 6) / wps, wave = (tid >> 6) - set * wps;     // wave: its number inside the set
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
    // A wave stages one whole chunk per turn, compacted to its non-zero elements (in their order) and zero-filled up
    // to a whole stage group of the sweep: a zero leaves its chunk's sum unchanged at every scale, and post-ReLU data
    // is half zeros.
    for (int i = tid; i < npad; i += nthreads) {
        const float v = i < len ? act_pre(V, x[base + i]) : 0.0f;
        const bool nz = v != 0.0f;
        const unsigned long long m = __ballot(nz);
        const int cnt = __popcll(m);
        const int pos = __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
        const int c0 = i & ~63;
        const int padded = (cnt + kPartGranule<C> - 1) & ~(kPartGranule<C> - 1);
        if (nz) slice[c0 + pos] = v;
        if (lane < padded - cnt) slice[c0 + cnt + lane] = 0.0f;
        const unsigned kb = wave_max_u32(bound_key(v, lo));
        if (lane == 0) { s_bounds[i >> 6] = kb; s_len[i >> 6] = padded; }
    }
    __syncthreads();

    // For the refinement passes: the block as staged (the variant's operation applied, zeros dropped) goes to the
    // workspace, chunk after chunk without gaps, each zero-filled up to a multiple of eight elements, with where
    // every chunk starts and how long it is (compact_meta); k_act_probe reads that instead of the tensor.
    if (compact != nullptr) {
        if (tid < kBlockChunks) {
            const int l4 = tid < npad / kChunk ? s_len[tid] : 0;
            const int l8 = (l4 + 7) & ~7;
            int end = l8;                                        // inclusive prefix sum over the 64 chunks
#pragma unroll
            for (int d = 1; d < kBlockChunks; d <<= 1) {
                const int up = __shfl_up(end, d, 64);
                if (lane >= d) end += up;
            }
            s_len[tid] = l4 | ((end - l8) << 8);
            meta[(size_t)blockIdx.x * kBlockChunks + tid] = compact_meta(end - l8, l8);
        }
        __syncthreads();
        float* out = compact + (size_t)blockIdx.x * kBlockElems;
        for (int c = tid >> 6; c < npad / kChunk; c += nthreads >> 6) {
            const int w = s_len[c], l4 = w & 0xff;
            if (lane < ((l4 + 7) & ~7)) out[(w >> 8) + lane] = lane < l4 ? slice[c * kChunk + lane] : 0.0f;
        }
    }

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
    const int part = kBlockElems / sets;
    const int e0 = set * part;
    int nel = npad - e0;                                       // whole chunks: the staging has compacted a ragged one too
    nel = nel < 0 ? 0 : (nel < part ? nel : part);
    if (nel > 0) {
        const float inv_min = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(inv[0])));   // lane 0: the wave's smallest scale
        const unsigned long long in0 = chunks_inside_range(s_bounds + e0 / kChunk, nel / kChunk, inv_min, lo, hi, lane);
        const int lengths = lane < nel / kChunk ? s_len[e0 / kChunk + lane] & 0xff : 0;
        sweep_slice<C, kLevelsBlk, kChunk, true>(slice + e0, nel, ci, alpha, inv, lo, hi, st, in0, 0ull, lengths);
    }
    double E[C];
    tree_fold<C, kLevelsBlk>(st, ci, E);                    // 0.0 when this set has no chunk
    if (sets > 1) {
        // the sums of sets 1 ... meet those of set 0 in the slice, which nobody reads any more after the first barrier
        double* exch = reinterpret_cast<double*>(slice4);
        const int ncand = wps * 64 * C;                      // candidates a set covers (>= G); sets * ncand <= kMaxExchange
        __syncthreads();
        if (set != 0) {
#pragma unroll
            for (int u = 0; u < C; ++u) exch[set * ncand + jcand[u]] = E[u];
        }
        __syncthreads();
        if (set == 0) {
#pragma unroll
            for (int u = 0; u < C; ++u) {
                const double* v = exch + jcand[u];
                if (sets == 2) E[u] = E[u] + v[ncand];
                else if (sets == 4) E[u] = (E[u] + v[ncand]) + (v[2 * ncand] + v[3 * ncand]);
                else E[u] = ((E[u] + v[ncand]) + (v[2 * ncand] + v[3 * ncand]))
                          + ((v[4 * ncand] + v[5 * ncand]) + (v[6 * ncand] + v[7 * ncand]));
            }
        }
    }
    if (set == 0) {
#pragma unroll
        for (int u = 0; u < C; ++u)
            if (jcand[u] < G) part0[(size_t)blockIdx.x * G + jcand[u]] = E[u];
    }
}

// One tree stage over blocks: out[g][j] = pairwise sum of in[64g .. 64g+63][j].
// When a stage leaves a single row and fin != nullptr the caller continues with it.
// Output row blockIdx.x of level `level` belongs to one tensor; its inputs are that tensor's rows of level - 1.
// (Rows on the x axis of the grid: a batch of large tensors has more than 65535 of them.)
// probe_cols != 0: the columns are the scales of a refinement pass; only those the tensor's state asks for were
// written by k_act_probe (none for a tensor that is finished, all-zero or rejected), the rest is skipped here
// as it is in k_act_finish.
__global__ void __launch_bounds__(256) k_act_reduce64(const ActBatch B, int level, const double* __restrict__ in, int G,
                                                      double* __restrict__ out, int probe_cols)
{
    const int j = blockIdx.y * blockDim.x + threadIdx.x;
    int first, below;
    const int t = act_find_level(B, level, blockIdx.x, first, below);
    if (probe_cols) {
        const ActState* S = B.S + t;
        if (S->status != 0 || S->done || j >= S->nprobe) return;
    }
    const int g = blockIdx.x - first;                                   // group of 64 input rows inside the tensor
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
    out[(size_t)blockIdx.x * G + j] = v[0];
}

// Pairwise tree over `rows` (<= 64) values v[0], v[stride], ... as a 64-wide tree padded with zeros
// (adding +0.0 to a sum changes nothing, so these are the bits of "a value without a partner is carried
// up").  Four groups of 16 values, each loaded in one go so that the loads are in flight together.
__device__ __forceinline__ double tree_rows64(const double* __restrict__ v, int rows, size_t stride)
{
    double g[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        double e[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) e[i] = (16 * q + i < rows) ? v[(size_t)(16 * q + i) * stride] : 0.0;
#pragma unroll
        for (int w = 1; w < 16; w <<= 1)
#pragma unroll
            for (int i = 0; i < 16; i += 2 * w) e[i] = e[i] + e[i + w];
        g[q] = e[0];
        if (16 * (q + 1) >= rows) {            // nothing but zeros beyond this group
#pragma unroll
            for (int r = 0; r < 4; ++r) if (r > q) g[r] = 0.0;
            break;
        }
    }
    return (g[0] + g[1]) + (g[2] + g[3]);
}

// Argmin over the G grid sums (one workgroup) and set-up of the refinement state.
__global__ void __launch_bounds__(256) k_act_argmin(const ActBatch B, int level, const double* __restrict__ tot, int G,
                                                     int qmax, int iters, const ActOut O,
                                                     float* absmax_out, double* grid_out)   // optional: [count], [count][G]
{
    __shared__ double s_bestE[16];
    __shared__ int s_bestJ[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    ActState* S = B.S + blockIdx.x;
    float* scale = O.scale[blockIdx.x];
    int32_t* idx = O.idx[blockIdx.x];
    double* sse = O.sse[blockIdx.x];
    // the level handed over holds at most 64 rows per tensor: the last tree levels are taken here
    int first = 0;
    for (int u = 0; u < (int)blockIdx.x; ++u) first += act_rows(B.start[u + 1] - B.start[u], level);
    const int rows = act_rows(B.start[blockIdx.x + 1] - B.start[blockIdx.x], level);
    tot += (size_t)first * G;
    const float a = __uint_as_float(S->absmax_bits);
    if (tid == 0 && absmax_out) absmax_out[blockIdx.x] = a;
    if (!(a <= kHuge)) {
        if (tid == 0) {
            const float nanf_ = __uint_as_float(0x7fc00000u);
            S->status = 2; S->absmax = a;
            *scale = nanf_; *idx = -1; *sse = (double)nanf_;
        }
        if (grid_out)
            for (int j = tid; j < G; j += blockDim.x) grid_out[(size_t)blockIdx.x * G + j] = (double)__uint_as_float(0x7fc00000u);
        return;
    }
    double bE = __longlong_as_double(0x7ff0000000000000LL);
    int bJ = INT_MAX;
    for (int j = tid; j < G; j += blockDim.x) {
        const double e = tree_rows64(tot + j, rows, (size_t)G);
        if (grid_out) grid_out[(size_t)blockIdx.x * G + j] = e;
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

// One refinement pass: f at up to kMaxProbes scales for every block of 64 chunks, one workgroup of four waves
// per block.  It reads the compacted copy that k_act_sweep left in the workspace (half the bytes and half the
// evaluations on post-ReLU data; a zero changes no sum): coalesced non-temporal 16-byte loads into LDS, the first
// half of the slot without waiting for the block's length.  lane = (scale, pair of chunks): the eight lanes of a
// scale-group read the same element (a broadcast), the eight groups of a wave walk eight different chunks, each
// as far as it goes, and the wave takes as many turns as its longest chunk.  The chunk sums of a scale are then 32
// level-1 nodes of the block's pairwise tree; the first wave adds them up.
__global__ void __launch_bounds__(256) k_act_probe(const ActBatch B, float lo, float hi, double* probe0,
                                                   const float* __restrict__ compact, const unsigned* __restrict__ meta)
{
    __shared__ float4 tile4[kBlockElems / 4];
    __shared__ unsigned s_meta[kBlockChunks];
    __shared__ double node[kBlockChunks / 2][kMaxProbes];
    const int tid = threadIdx.x;
    const int t = act_find(B, blockIdx.x);
    const ActState* S = B.S + t;
    if (S->status != 0 || S->done) return;                    // uniform over the workgroup
    const int np = S->nprobe;
    const float* src = compact + (size_t)blockIdx.x * kBlockElems;
    const unsigned* mb = meta + (size_t)blockIdx.x * kBlockChunks;
    constexpr int R = kBlockElems / 4 / 256;                  // 16-byte pieces per thread for a whole slot
    float4 v[R];
#pragma unroll
    for (int r = 0; r < R / 2; ++r) v[r] = load_stream_f4(src + (size_t)(r * 256 + tid) * 4);
    const unsigned last = mb[kBlockChunks - 1];
    const int total = compact_off(last) + compact_len(last);  // floats of the block's copy
    if (tid < kBlockChunks) s_meta[tid] = mb[tid];
#pragma unroll
    for (int r = R / 2; r < R; ++r) {
        v[r] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if ((r * 256 + tid) * 4 < total) v[r] = load_stream_f4(src + (size_t)(r * 256 + tid) * 4);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) tile4[r * 256 + tid] = v[r];
    __syncthreads();

    const int p = tid & 7, g = tid >> 3;                      // scale, pair of chunks (2g, 2g + 1)
    const float alpha[1] = {S->probes[p]};
    const float inv[1] = {S->probe_inv[p]};
    double st[1][2] = {{0.0, 0.0}};
    unsigned ci = 0;
#pragma unroll 1
    for (int slot = 0; slot < 2; ++slot, ++ci) {
        const unsigned m = s_meta[2 * g + slot];
        const int turns = compact_len(m) >> 3;                // of eight elements
        const int most = __builtin_amdgcn_readfirstlane((int)wave_max_u32((unsigned)turns));
        const float4* p4 = tile4 + (compact_off(m) >> 2);
        float s[1] = {0.0f};
#pragma unroll 1
        for (int k = 0; k < most; ++k) {
            if (k < turns) {
                const float4 a = p4[2 * k], b = p4[2 * k + 1];
                const float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                eval_stage<8, 1>(x, alpha, inv, lo, hi, s);
            }
        }
        double ts[1] = {(double)s[0]};
        tree_push<1, 2>(st, ts, ci);
    }
    double E[1];
    tree_fold<1, 2>(st, ci, E);
    node[g][p] = E[0];
    __syncthreads();
    if (tid < 64) {
        // the upper five tree levels of a scale: lane (p, k) adds the eight nodes 8k .. 8k + 7 pairwise, the four
        // results are combined as (k0 + k1) + (k2 + k3) through shuffles (the whole first wave takes part)
        const int k = (tid >> 3) & 3;
        double v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = node[8 * k + i][p];
        double r = ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
        r = r + __shfl_down(r, 8, 64);
        r = r + __shfl_down(r, 16, 64);
        if (tid < np) probe0[(size_t)blockIdx.x * kMaxProbes + tid] = r;
    }
}

// Last tree levels over <= 4096 rows of per-scale sums (groups of 64 rows, then the groups), then the
// golden-section bookkeeping.  One workgroup per tensor; thread (g, p) owns group g of scale p.
__global__ void __launch_bounds__(512) k_act_finish(const ActBatch B, int level, const double* __restrict__ part, int iters,
                                                    const ActOut O)
{
    __shared__ double grp[64][kMaxProbes];
    __shared__ double vals[kMaxProbes];
    ActState* S = B.S + blockIdx.x;
    if (S->status != 0 || S->done) return;
    float* scale = O.scale[blockIdx.x];
    double* sse = O.sse[blockIdx.x];
    int first = 0;
    for (int u = 0; u < (int)blockIdx.x; ++u) first += act_rows(B.start[u + 1] - B.start[u], level);
    const int rows = act_rows(B.start[blockIdx.x + 1] - B.start[blockIdx.x], level);
    part += (size_t)first * kMaxProbes;
    const int t = threadIdx.x, g = t >> 3, pr = t & 7;
    const int ngroups = (rows + 63) >> 6;
    {
        const int r0 = g * 64;
        const int cnt = (g < ngroups && pr < S->nprobe) ? ((rows - r0) < 64 ? (rows - r0) : 64) : 0;
        grp[g][pr] = tree_rows64(part + (size_t)r0 * kMaxProbes + pr, cnt, kMaxProbes);
    }
    __syncthreads();
    if (t < kMaxProbes) vals[t] = tree_rows64(&grp[0][t], ngroups, kMaxProbes);
    __syncthreads();
    if (t == 0) {
        act_advance_plan(S, vals, iters);
        *scale = S->best_a;
        *sse = S->best;
    }
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
            const float4 p0 = reinterpret_cast<const float4*>(x + e0)[0];     // plain loads and stores: the streaming hints
            const float4 p1 = reinterpret_cast<const float4*>(x + e0)[1];     // gain nothing on a read + write pass
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

}  // namespace

#endif  // MMSE_ACTIVATION_H_
