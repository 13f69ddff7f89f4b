// mmse_common.h -- constants, element arithmetic, the canonical summation tree and the LDS-fed sweep core shared by all kernels (gfx950).
#ifndef MMSE_COMMON_H_
#define MMSE_COMMON_H_
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>

namespace {


constexpr int kChunk = 64;             // elements per sequential fp32 chunk
constexpr int kMaxBatch = 59;          // tensors per launch: the descriptor table lives in kernarg (4 KB at most)
constexpr int kMaxBatchExt = 36;       // ... when some tensor of the launch uses the fields of TensorExt
constexpr int kTile = 8192;            // floats of one kernel staged in LDS at a time
constexpr int kTileStream = 4096;      // ... for longer kernels, which stream through LDS tile by tile
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

// The tensors of one launch travel in the kernel argument buffer (no host-to-device copy, no allocation): 64
// bytes per tensor, so that a network of up to kMaxBatch layers is one launch per stage; the fields only the
// two-tensor methods and the grid-error output use are a second, shorter array that overlays the end of the first.
struct TensorCore {
    const float* w;
    const float* scale1;
    float* scale;
    int32_t* idx;
    double* sse;
    float* absmax;
    uint8_t* packed;
    int K;
    int n;
};
struct TensorExt {
    double* grid_sse;
    const uint8_t* sub_packed;
    const float* sub_scale;
    const uint8_t* active;
};
struct Batch {
    union {
        TensorCore t[kMaxBatch];
        struct {
            TensorCore t_with_ext[kMaxBatchExt];
            TensorExt e[kMaxBatchExt];          // has_ext != 0: count <= kMaxBatchExt
        };
    };
    int start[kMaxBatch + 1];   // prefix sum of the workgroups each tensor gets in this launch
    int count;
    int G;
    int qmax;
    int iters;
    float lo, hi;               // (float)qmin, (float)qmax
    int has_ext;
    int fused_part_off;         // fused search: floats from the start of the LDS slice to its reduction buffers
};
static_assert(sizeof(TensorCore) == 64 && sizeof(TensorExt) == 32, "descriptor sizes");
static_assert(sizeof(Batch) <= 4096, "the descriptor table must fit the kernel argument buffer");

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

// 16-byte load for data that is streamed through once (a whole activation tensor per read-only pass): the
// non-temporal hint keeps such lines from displacing what the caches hold for others, which on MI355X is worth
// about a tenth of the read bandwidth of a pass over a tensor much larger than the caches (6.9 against 6.2 TB/s);
// a pass that also writes (the code passes) gains nothing from it and loses when the tensor fits the caches.
typedef float mmse_vf4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream_f4(const float* p)
{
    const mmse_vf4 v = __builtin_nontemporal_load(reinterpret_cast<const mmse_vf4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ unsigned abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// Cross-lane exchange inside rows of 16 lanes without LDS: the partner of lane i is i ^ 1, i ^ 2, then 7 - i inside
// its group of eight and 15 - i inside its row; for a reduction whose operation is symmetric, after the four
// steps every lane of a row holds the row's result.  The four row results then meet as scalar operands.
constexpr int kDppXor1 = 0xB1;          // quad_perm [1, 0, 3, 2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2, 3, 0, 1]
constexpr int kDppHalfMirror = 0x141;   // row_half_mirror
constexpr int kDppMirror = 0x140;       // row_mirror
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) { return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false); }
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v)
{
    return __hiloint2double(dpp_i32<CTRL>(__double2hiint(v)), dpp_i32<CTRL>(__double2loint(v)));
}

__device__ __forceinline__ unsigned wave_max_u32(unsigned v)
{
    unsigned o;
    o = (unsigned)dpp_i32<kDppXor1>((int)v); v = o > v ? o : v;
    o = (unsigned)dpp_i32<kDppXor2>((int)v); v = o > v ? o : v;
    o = (unsigned)dpp_i32<kDppHalfMirror>((int)v); v = o > v ? o : v;
    o = (unsigned)dpp_i32<kDppMirror>((int)v); v = o > v ? o : v;
    const unsigned r0 = (unsigned)__builtin_amdgcn_readlane((int)v, 0), r1 = (unsigned)__builtin_amdgcn_readlane((int)v, 16);
    const unsigned r2 = (unsigned)__builtin_amdgcn_readlane((int)v, 32), r3 = (unsigned)__builtin_amdgcn_readlane((int)v, 48);
    const unsigned a = r0 > r1 ? r0 : r1, b = r2 > r3 ? r2 : r3;
    return a > b ? a : b;
}

// (value, index) minimum over a wave; the lower index wins among equal values.  Every lane returns the result.
template <int CTRL>
__device__ __forceinline__ void argmin_step(double& e, int& j)
{
    const double oe = dpp_f64<CTRL>(e);
    const int oj = dpp_i32<CTRL>(j);
    if (oe < e || (oe == e && oj < j)) { e = oe; j = oj; }
}

__device__ __forceinline__ void wave_argmin(double& e, int& j)
{
    argmin_step<kDppXor1>(e, j);
    argmin_step<kDppXor2>(e, j);
    argmin_step<kDppHalfMirror>(e, j);
    argmin_step<kDppMirror>(e, j);
    double be = readlane_f64(e, 0);
    int bj = __builtin_amdgcn_readlane(j, 0);
#pragma unroll
    for (int r = 16; r < 64; r += 16) {
        const double oe = readlane_f64(e, r);
        const int oj = __builtin_amdgcn_readlane(j, r);
        if (oe < be || (oe == be && oj < bj)) { be = oe; bj = oj; }
    }
    e = be; j = bj;
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
// CLAMP = false leaves the saturation out: for callers that have shown it to be the identity for every one of
// these evaluations (sweep_slice), where it then is four instructions per evaluation instead of five.
template <int NE, int C, bool CLAMP = true>
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
    if constexpr (CLAMP) {
#pragma unroll
        for (int i = 0; i < NE; ++i)
#pragma unroll
            for (int u = 0; u < C; ++u) t[i][u] = __builtin_amdgcn_fmed3f(t[i][u], lo, hi);
        MMSE_STAGE_FENCE();
    }
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

// What a chunk's elements contribute to its entry of the bounds array (the entry is the largest key of the chunk):
// |x| as a bit pattern, or +inf for a negative element of an unsigned range, which no scale brings into the range.
__device__ __forceinline__ unsigned bound_key(float v, float lo)
{
    return (lo == 0.0f && v < 0.0f) ? 0x7f800000u : abs_bits(v);
}

// Which of up to 64 chunks a wave may evaluate without the saturation (bit c: chunk c): those whose largest
// magnitude (bounds[c], a bound_key, in LDS; zero counts as an element) rounds to a code inside the range at
// inv_min = 1 / the smallest scale any lane of the wave sweeps.  x*inv, the rounding and the reciprocal are
// monotonic, so no code of such a chunk at any scale of the wave has a larger magnitude than that one; the
// saturation would return its argument, and the bits are the same without it.  (Sufficient, not necessary: the
// magnitude is tested against the smaller of the two ends of a signed range.)  One chunk per lane, then a vote.
__device__ __forceinline__ unsigned long long chunks_inside_range(const unsigned* bounds, int nchunks, float inv_min,
                                                                   float lo, float hi, int lane)
{
    const float limit = (lo == 0.0f || hi < -lo) ? hi : -lo;
    bool in = false;
    if (lane < nchunks) in = __builtin_rintf(__uint_as_float(bounds[lane]) * inv_min) <= limit;
    return __ballot(in);
}

// The elements of one whole chunk at s4 against the C candidates of this lane, fetched from LDS one group ahead of
// their use (same address in every lane: broadcast).
template <int C, bool CLAMP>
__device__ __forceinline__ void sweep_chunk(const float4* s4, const float (&alpha)[C], const float (&inv)[C],
                                            float lo, float hi, float (&s)[C])
{
    constexpr int NE = (C >= 2) ? 4 : 8;            // elements per stage group (8 temporaries either way with C <= 2)
    float4 nxt[NE / 4];
#pragma unroll
    for (int q = 0; q < NE / 4; ++q) nxt[q] = s4[q];
#pragma unroll
    for (int e = 0; e < kChunk / NE; ++e) {
        float x[NE];
#pragma unroll
        for (int q = 0; q < NE / 4; ++q) {
            x[4 * q + 0] = nxt[q].x; x[4 * q + 1] = nxt[q].y; x[4 * q + 2] = nxt[q].z; x[4 * q + 3] = nxt[q].w;
        }
        if (e + 1 < kChunk / NE) {
#pragma unroll
            for (int q = 0; q < NE / 4; ++q) nxt[q] = s4[(e + 1) * (NE / 4) + q];
        }
        __builtin_amdgcn_sched_barrier(0);       // the prefetch is issued before this group's arithmetic
        eval_stage<NE, C, CLAMP>(x, alpha, inv, lo, hi, s);
    }
}

// The same for the first `nelem` elements of a chunk (a multiple of the stage group: 4 with two or more candidates
// per lane, else 8; fewer than 64; may be 0): the first 32 unrolled like a whole chunk when there are that many
// (post-ReLU chunks have 32 non-zero elements on average), then a loop of eight elements a turn and one last group of
// four: for chunks that have been compacted to their non-zero elements (sweep_slice).  In the loop, fetching a turn
// ahead (in one buffer handed on, or in two named ones) was measured no faster (other waves cover the LDS latency);
// single elements at the end instead of zero-filling the last group gained 1 %.
template <int C>
constexpr int kPartGranule = (C >= 2) ? 4 : 8;

template <int C, bool CLAMP>
__device__ __forceinline__ void sweep_chunk_part(const float4* s4, int nelem, const float (&alpha)[C], const float (&inv)[C],
                                                 float lo, float hi, float (&s)[C])
{
    constexpr int NE = (C >= 2) ? 4 : 8;
    const float4* p4 = s4;
    int turns = nelem >> 3;
    if (turns >= 4) {                                         // the first 32 elements unrolled, fetched a group ahead
        float4 nxt[NE / 4];
#pragma unroll
        for (int q = 0; q < NE / 4; ++q) nxt[q] = s4[q];
#pragma unroll
        for (int e = 0; e < 32 / NE; ++e) {
            float x[NE];
#pragma unroll
            for (int q = 0; q < NE / 4; ++q) {
                x[4 * q + 0] = nxt[q].x; x[4 * q + 1] = nxt[q].y; x[4 * q + 2] = nxt[q].z; x[4 * q + 3] = nxt[q].w;
            }
            if (e + 1 < 32 / NE) {
#pragma unroll
                for (int q = 0; q < NE / 4; ++q) nxt[q] = s4[(e + 1) * (NE / 4) + q];
            }
            __builtin_amdgcn_sched_barrier(0);
            eval_stage<NE, C, CLAMP>(x, alpha, inv, lo, hi, s);
        }
        turns -= 4;
        p4 += 8;
    }
#pragma unroll 1
    for (int t = turns; t > 0; --t, p4 += 2) {                // nelem is uniform: the count lives in a scalar register
        const float4 a = p4[0], b = p4[1];
        const float xs[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int g = 0; g < 8 / NE; ++g) {
            float x[NE];
#pragma unroll
            for (int i = 0; i < NE; ++i) x[i] = xs[g * NE + i];
            eval_stage<NE, C, CLAMP>(x, alpha, inv, lo, hi, s);
        }
    }
    if constexpr (NE == 4) {
        if (nelem & 4) {
            const float4 a = p4[0];
            const float x[4] = {a.x, a.y, a.z, a.w};
            eval_stage<4, C, CLAMP>(x, alpha, inv, lo, hi, s);
        }
    }
}

// Sweep the `nelem` elements (a multiple of 8; zero padded) that sit in LDS at `slice` for the C
// candidates of this lane: whole 64-element chunks, then a last shorter chunk that only walks the
// 8-element groups it has (padding zeros would be exact no-ops, so skipping them changes nothing).
// CS: floats between the starts of consecutive chunks in LDS (kChunk, or more when the chunks are padded apart
// so that lanes reading different chunks at the same time hit different banks).
// inside0 / inside1: bit c set (chunks 0-63 / 64-127 of this slice): the caller has shown with chunks_inside_range
// that the saturation is the identity for chunk c at every scale of this wave; such a chunk takes four instructions
// per evaluation instead of five.
// SPARSE: every chunk of the slice (at most 64 of them, all of them whole) has been compacted to its non-zero
// elements, zero-filled up to a multiple of kPartGranule<C>; lane c holds the resulting length of chunk c in `lengths`.  An
// element that is zero leaves the sum of its chunk unchanged at every scale (its code is zero, its residual is zero,
// and s + 0 = s exactly), so walking only the others, in their order, gives the same bits; post-ReLU activations are
// half zeros.
template <int C, int L, int CS = kChunk, bool SPARSE = false>
__device__ __forceinline__ void sweep_slice(const float* slice, int nelem, unsigned& ci,
                                            const float (&alpha)[C], const float (&inv)[C],
                                            float lo, float hi, double (&st)[C][L],
                                            unsigned long long inside0 = 0, unsigned long long inside1 = 0, int lengths = 0)
{
    const float4* s4 = reinterpret_cast<const float4*>(slice);
    constexpr int NE = (C >= 2) ? 4 : 8;
    const int nfull = nelem / kChunk;
    const int tail = nelem - nfull * kChunk;        // 0, 8, ..., 56 elements of a last partial chunk
    const int ntotal = nfull + (tail > 0 ? 1 : 0);
#pragma unroll 1
    for (int c = 0; c < ntotal; ++c, ++ci) {
        float s[C];
#pragma unroll
        for (int u = 0; u < C; ++u) s[u] = 0.0f;
        if (c < nfull) {
            const bool inside = (((c < 64 ? inside0 : inside1) >> (c & 63)) & 1ull) != 0;       // scalar: c is uniform
            // (the empty statements hide from the compiler that both branches start at the same address: it would
            // merge their first fetches ahead of the branch, at the price of registers the sweep needs for its waves)
            int cc = c;
            int len = kChunk;
            if constexpr (SPARSE) len = __builtin_amdgcn_readlane(lengths, c);
            if (len < kChunk) {
                if (inside) {
                    asm volatile("" : "+s"(cc));
                    sweep_chunk_part<C, false>(s4 + cc * (CS / 4), len, alpha, inv, lo, hi, s);
                } else {
                    asm volatile("" : "+s"(cc));
                    sweep_chunk_part<C, true>(s4 + cc * (CS / 4), len, alpha, inv, lo, hi, s);
                }
            } else if (inside) {
                asm volatile("" : "+s"(cc));
                sweep_chunk<C, false>(s4 + cc * (CS / 4), alpha, inv, lo, hi, s);
            } else {
                asm volatile("" : "+s"(cc));
                sweep_chunk<C, true>(s4 + cc * (CS / 4), alpha, inv, lo, hi, s);
            }
        } else {
            for (int e = 0; e < tail / NE; ++e) {
                float x[NE];
#pragma unroll
                for (int q = 0; q < NE / 4; ++q) {
                    const float4 v = s4[c * (CS / 4) + e * (NE / 4) + q];
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

constexpr int kMaxProbes = 8;          // scales evaluated in one pass over an activation tensor

// State of one golden-section refinement with look-ahead (per activation tensor in device memory; per kernel in
// LDS in the fused weight search).
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
    float probe_inv[kMaxProbes];     // 1 / probes[i], for the kernels that evaluate them
    double ec, ed, best;
    unsigned min_key, max_key;   // offset form: order-preserving keys of min and max
    float out_scale; int out_idx; double out_sse;    // result slots for calls that only want the grid errors
    float delta;                 // offset form: min of the tensor
};

// ---- golden-section bookkeeping (one thread) ---------------------------------------
// The search is sequential: each iteration needs f at one new scale.  One pass over a big
// tensor costs a full read of it, so a pass evaluates the scale(s) the search is waiting
// for *and* every scale the next two iterations could ask for (both outcomes of each
// comparison: 1 + 2 + 4, or 2 + 2 + 4 at the start).  gs_advance then replays the plain
// sequential algorithm, looking values up by scale; it stops when a value is missing.
// The probes are produced by the same fp32 expressions on both paths, so a lookup is an
// exact match.  Nothing about the result depends on how much was evaluated ahead.
// The search state in registers (one thread does the bookkeeping; memory is read once and written once).
struct GsRegs {
    float lo_a, hi_a, pc, pd, best_a;
    double ec, ed, best;
    int have_c, have_d, it, done;
};

__device__ __forceinline__ GsRegs gs_load(const ActState* S)
{
    GsRegs R;
    R.lo_a = S->lo_a; R.hi_a = S->hi_a; R.pc = S->pc; R.pd = S->pd; R.best_a = S->best_a;
    R.ec = S->ec; R.ed = S->ed; R.best = S->best;
    R.have_c = S->have_c; R.have_d = S->have_d; R.it = S->it; R.done = S->done;
    return R;
}

__device__ __forceinline__ void gs_store(ActState* S, const GsRegs& R)
{
    S->lo_a = R.lo_a; S->hi_a = R.hi_a; S->pc = R.pc; S->pd = R.pd; S->best_a = R.best_a;
    S->ec = R.ec; S->ed = R.ed; S->best = R.best;
    S->have_c = R.have_c; S->have_d = R.have_d; S->it = R.it; S->done = R.done;
}

// f at scale a among the n values of the last pass (the first match, as the list may hold a scale twice)
__device__ __forceinline__ bool gs_lookup(const float (&pr)[kMaxProbes], const double (&v)[kMaxProbes], int n, float a, double& out)
{
    bool hit = false;
#pragma unroll
    for (int i = 0; i < kMaxProbes; ++i)
        if (!hit && i < n && pr[i] == a) { out = v[i]; hit = true; }
    return hit;
}

// Replays the sequential golden section with the values of the last pass until one is missing.
__device__ __forceinline__ void gs_advance(GsRegs& R, const float (&pr)[kMaxProbes], const double (&v)[kMaxProbes], int n, int iters)
{
    while (!R.done) {
        if (!R.have_c) {
            if (!gs_lookup(pr, v, n, R.pc, R.ec)) break;
            R.have_c = 1;
            if (R.ec < R.best) { R.best = R.ec; R.best_a = R.pc; }
        }
        if (!R.have_d) {
            if (!gs_lookup(pr, v, n, R.pd, R.ed)) break;
            R.have_d = 1;
            if (R.ed < R.best) { R.best = R.ed; R.best_a = R.pd; }
        }
        if (R.it == iters) { R.done = 1; break; }
        if (R.ec <= R.ed) {
            R.hi_a = R.pd; R.pd = R.pc; R.ed = R.ec;
            R.pc = __builtin_fmaf(-kPhi, R.hi_a - R.lo_a, R.hi_a);
            R.have_c = 0;
        } else {
            R.lo_a = R.pc; R.pc = R.pd; R.ec = R.ed;
            R.pd = __builtin_fmaf(kPhi, R.hi_a - R.lo_a, R.lo_a);
            R.have_d = 0;
        }
        ++R.it;
    }
}

// The scales of the next pass.  max_depth: iterations to look ahead (0: only the scale(s) the search waits for;
// 2: up to 1 + 2 + 4 scales).  with_inv: also store their reciprocals.
// The scales of the next pass: the one(s) the search waits for, then what its next one or two iterations could
// ask for -- after "keep [lo, pd]" (L) or "keep [pc, hi]" (R), and after each of those again (LL, LR, RL, RR) --
// by the same fp32 expressions gs_advance uses.  Every index below is a constant (no array in scratch memory).
__device__ __forceinline__ int gs_plan_list(const GsRegs& R, int iters, int max_depth, float (&list)[kMaxProbes])
{
    int depth = iters - R.it;
    if (depth > max_depth) depth = max_depth;
    if (R.done) depth = 0;
    const float L = __builtin_fmaf(-kPhi, R.pd - R.lo_a, R.pd);
    const float Rr = __builtin_fmaf(kPhi, R.hi_a - R.pc, R.pc);
    const float LL = __builtin_fmaf(-kPhi, R.pc - R.lo_a, R.pc);
    const float LR = __builtin_fmaf(kPhi, R.pd - L, L);
    const float RL = __builtin_fmaf(-kPhi, Rr - R.pc, Rr);
    const float RR = __builtin_fmaf(kPhi, R.hi_a - R.pd, R.pd);
    const int ncand = depth <= 0 ? 0 : (depth == 1 ? 2 : 6);
    float cand[6] = {L, Rr, LL, LR, RL, RR};
#pragma unroll
    for (int i = 0; i < 6; ++i) cand[i] = i < ncand ? cand[i] : 1.0f;
    const int npend = R.done ? 0 : (R.have_c ? 0 : 1) + (R.have_d ? 0 : 1);
    const float p0 = !R.have_c ? R.pc : R.pd;         // first pending scale (when there is one)
    // list = [pending..., cand...], padded with 1.0
    const float a0[kMaxProbes] = {cand[0], cand[1], cand[2], cand[3], cand[4], cand[5], 1.0f, 1.0f};
    const float a1[kMaxProbes] = {p0, cand[0], cand[1], cand[2], cand[3], cand[4], cand[5], 1.0f};
    const float a2[kMaxProbes] = {R.pc, R.pd, cand[0], cand[1], cand[2], cand[3], cand[4], cand[5]};
#pragma unroll
    for (int i = 0; i < kMaxProbes; ++i) list[i] = npend == 0 ? a0[i] : (npend == 1 ? a1[i] : a2[i]);
    return npend + ncand;
}

__device__ __forceinline__ void gs_plan(ActState* S, const GsRegs& R, int iters, int max_depth, bool with_inv)
{
    float list[kMaxProbes];
    const int n = gs_plan_list(R, iters, max_depth, list);
    S->nprobe = n;
#pragma unroll
    for (int i = 0; i < kMaxProbes; ++i) {
        const float a = i < n ? list[i] : 1.0f;
        S->probes[i] = a;
        if (with_inv) S->probe_inv[i] = 1.0f / a;
    }
}

__device__ void act_plan(ActState* S, int iters, int max_depth = 2, bool with_inv = true)
{
    const GsRegs R = gs_load(S);
    gs_plan(S, R, iters, max_depth, with_inv);
}

// advance with the values of the last pass, then plan the next one
__device__ void act_advance_plan(ActState* S, const double* vals, int iters, int max_depth = 2, bool with_inv = true)
{
    GsRegs R = gs_load(S);
    const int n = S->nprobe;
    float pr[kMaxProbes];
    double v[kMaxProbes];
#pragma unroll
    for (int i = 0; i < kMaxProbes; ++i) { pr[i] = S->probes[i]; v[i] = vals[i]; }
    gs_advance(R, pr, v, n, iters);
    gs_store(S, R);
    gs_plan(S, R, iters, max_depth, with_inv);
}

// Tensor that owns workgroup bid, and that workgroup's number inside the tensor.
__device__ __forceinline__ int find_tensor(const Batch& B, int bid, int& local)
{
    int t = 0;
    while (t + 1 < B.count && bid >= B.start[t + 1]) ++t;
    local = bid - B.start[t];
    return t;
}

__device__ __forceinline__ TensorArgs tensor_of(const Batch& B, int t)
{
    const TensorCore& c = B.t[t];
    TensorArgs A;
    A.w = c.w; A.scale1 = c.scale1; A.scale = c.scale; A.idx = c.idx; A.sse = c.sse; A.absmax = c.absmax;
    A.packed = c.packed; A.K = c.K; A.n = c.n;
    A.grid_sse = nullptr; A.sub_packed = nullptr; A.sub_scale = nullptr; A.active = nullptr;
    if (B.has_ext) {
        const TensorExt& e = B.e[t];
        A.grid_sse = e.grid_sse; A.sub_packed = e.sub_packed; A.sub_scale = e.sub_scale; A.active = e.active;
    }
    return A;
}

}  // namespace

#endif  // MMSE_COMMON_H_
