/*
 * mmse.h -- C ABI of the MI355X (gfx950) MMSE INT4 scale-search library.
 *
 * Method: "Low-bit Quantization of Neural Networks for Efficient Inference"
 * (arXiv 1902.06822).  A tensor T is approximated linearly as alpha * Q with Q
 * integer in Z_p (Section 3.1, Eq. 1); alpha minimises the constrained squared
 * error ||T - alpha*[T/alpha]_Zp||^2 (Section 3.4, Eq. 7-8) by an exact line
 * search over a grid of a few hundred points; weights get one alpha per
 * output-channel kernel (Section 3.3), activations one per layer (Section 3.7,
 * Eq. 15); badly approximated layers get a second INT4 tensor fitted to the
 * residual (Section 3.5, Algorithm 1, first sweep; Eq. 16).
 *
 * General conventions
 *   - every *_dev pointer is DEVICE memory owned by the caller; the library
 *     allocates no device memory (a batched call of more than 64 tensors builds
 *     its descriptor table in temporary host memory), keeps no state between
 *     calls and never synchronises:
 *     all work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and results are valid once the stream has drained.
 *   - weight tensors are fp32, row-major [K][n]: K kernels of n elements
 *     (n = c*w*h of Section 3.1).  Activation tensors are flat fp32 [N].
 *   - return value: MMSE_OK or a negative mmse_status_t.  All argument checks
 *     happen before anything is enqueued, so a failed call has no side effect.
 *   - inputs must be finite.  A problem whose max |T| is below 2^-60 is coded
 *     as all-zero (scale 1, idx 0, sse = sum T^2); one whose max |T| exceeds
 *     2^60 or holds inf/NaN is rejected on the device: scale = NaN, idx = -1,
 *     sse = NaN for that problem, its codes are written as zeros.
 *   - "sse" is the SUM of squared errors (the paper omits the mean factor,
 *     Section 3.2), accumulated as documented in csrc/mmse_kernels.hip.
 */
#ifndef MMSE_H_
#define MMSE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mmse_status_t {
    MMSE_OK = 0,
    MMSE_ERR_NULL = -1,        /* a required pointer is NULL                           */
    MMSE_ERR_SIZE = -2,        /* K, n or N <= 0, or beyond the limits below           */
    MMSE_ERR_PARAMS = -3,      /* bad quantization range, grid size or refine count    */
    MMSE_ERR_WORKSPACE = -4,   /* ws_dev NULL / misaligned / ws_bytes too small        */
    MMSE_ERR_LAUNCH = -5,      /* the HIP runtime refused a launch                     */
    MMSE_ERR_ALIGN = -6,       /* a device pointer is not aligned to its element type  */
    MMSE_ERR_HOST_MEMORY = -7  /* host memory for a batched call's tables ran out      */
} mmse_status_t;

/* Limits (checked; MMSE_ERR_SIZE / MMSE_ERR_PARAMS otherwise). */
#define MMSE_MAX_KERNEL_ELEMS 65536      /* n of one weight kernel                     */
#define MMSE_MAX_GRID_POINTS 2048        /* G                                           */
#define MMSE_MAX_REFINE_ITERS 64
#define MMSE_MAX_TENSOR_ELEMS 2147483647 /* K*n and N                                   */
#define MMSE_MAX_KERNELS 4194304         /* K of one weight tensor (quantize_pack_int4: any K) */
#define MMSE_MAX_BATCH_TENSORS 1024      /* activation tensors of one batched call      */

/* Search parameters.
 *   qmin,qmax     integer range Z_p of Section 3.1: -8,7 (signed INT4) or 0,15
 *                 (unsigned, no offset term); any qmin <= 0 < qmax with
 *                 qmax - qmin <= 15 is accepted.
 *   grid_points   G >= 1 candidates alpha_j = (max|T|/qmax) * (j+1)/G, j = 0..G-1;
 *                 the last one is the max-abs scale of Section 3.1.
 *   refine_iters  golden-section iterations applied between the grid neighbours
 *                 of the argmin (0 = return the grid point).
 *   cands_per_lane  tuning only, never changes a result: grid candidates each
 *                 lane of the sweep kernel carries (0 = automatic; 1, 2 or 4). */
typedef struct mmse_params_t {
    int32_t qmin, qmax;
    int32_t grid_points;
    int32_t refine_iters;
    int32_t cands_per_lane;
} mmse_params_t;

/* One weight tensor of a batched call.  Outputs as in mmse_scale_search_kernelwise;
 * scale1_dev and packed_dev are optional (NULL):
 *   scale1_dev != NULL  search the residual w - scale1*[w/scale1] (second tensor of
 *                       Section 3.5) instead of w itself;
 *   packed_dev != NULL  also emit the packed INT4 codes of the searched tensor. */
typedef struct mmse_tensor_desc_t {
    const float *w_dev;        /* [K][n]                                   */
    int64_t K, n;
    const float *scale1_dev;   /* [K] or NULL                              */
    float *scale_dev;          /* [K]                                      */
    int32_t *idx_dev;          /* [K]                                      */
    double *sse_dev;           /* [K]                                      */
    uint8_t *packed_dev;       /* ceil(K*n/2) bytes or NULL                */
} mmse_tensor_desc_t;

/* Workspace sizes (bytes; host call, nothing enqueued).  ws_dev must be aligned
 * to 256 bytes.  For a batched call pass the sum of K over all tensors as K and
 * any n.  With refine_iters > 0 the activation workspace includes 4 bytes per
 * element (in whole blocks of 4096 elements, plus 256 bytes per block): the grid
 * sweep leaves the searched values there with the zeros dropped, and the
 * refinement passes read that copy instead of the tensor. */
int mmse_workspace_bytes_kernelwise(int64_t K, int64_t n, const mmse_params_t *p, size_t *bytes_out);
int mmse_workspace_bytes_activation(int64_t N, const mmse_params_t *p, size_t *bytes_out);

/* Kernel-wise search (Sections 3.3-3.4): for every row k of w_dev,
 *   scale_dev[k]  the chosen alpha_k
 *   idx_dev[k]    grid argmin j*_k (lowest index among equal minima)
 *   sse_dev[k]    sum_i (w_ki - alpha_k*[w_ki/alpha_k])^2 at the returned scale. */
int mmse_scale_search_kernelwise(const float *w_dev, int64_t K, int64_t n, const mmse_params_t *p,
                                 float *scale_dev, int32_t *idx_dev, double *sse_dev,
                                 void *ws_dev, size_t ws_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): mmse_scale_search_kernelwise with the workspace replaced by a fixed
 * array inside the library (4 bytes per kernel, MMSE_NOALLOC_MAX_KERNELS kernels = 1 MiB per GPU, held
 * until the process ends).  Same arguments otherwise, same results.  K above the limit is MMSE_ERR_SIZE.
 * The call allocates nothing on the device or the host.  All calls on one GPU share that GPU's array:
 * two calls that overlap on one GPU (different streams, or different host threads) race and give wrong
 * results; calls on one stream, or ordered by events, are fine.  Nothing in the array needs clearing
 * between calls: the sweep writes every entry that the refinement of the same call reads. */
#define MMSE_NOALLOC_MAX_KERNELS 262144
int mmse_scale_search_kernelwise_noalloc(const float *w_dev, int64_t K, int64_t n, const mmse_params_t *p,
                                         float *scale_dev, int32_t *idx_dev, double *sse_dev, void *stream);

/* Per-layer search for calibration activations (Section 3.7, Eq. 15): one problem
 * of N elements; scale_dev, idx_dev, sse_dev hold one element each. */
int mmse_scale_search_activation(const float *x_dev, int64_t N, const mmse_params_t *p,
                                 float *scale_dev, int32_t *idx_dev, double *sse_dev,
                                 void *ws_dev, size_t ws_bytes, void *stream);

/* Second tensor of an activation (Section 3.7, Eq. 16): X ~ beta1*[X/beta1] + beta2*[(X - beta1*X1)/beta2].
 * scale1_dev holds beta1 (one float, device; normally the output of mmse_scale_search_activation), the
 * first codes X1 = [X/beta1] saturate to [qmin1, qmax1]; the residual X - beta1*X1 (one fused
 * multiply-add per element, formed as the tensor is read) is searched in p's range with p's grid and refinement
 * ("one iteration only" of Algorithm 1).  The residual of unsigned first codes has both signs, so the
 * second range is independent of the first: p->qmin..p->qmax, e.g. -8..7.  Outputs as in
 * mmse_scale_search_activation, plus the residual's codes in packed2_dev (ceil(N/2) bytes, layout of
 * quantize_pack_int4) when it is not NULL.  A NaN or rejected beta1 rejects the residual too.
 * Workspace: mmse_workspace_bytes_activation(N, p). */
int activation_residual_quantize(const float *x_dev, int64_t N, const float *scale1_dev, int32_t qmin1, int32_t qmax1,
                                 const mmse_params_t *p, float *scale2_dev, int32_t *idx2_dev, double *sse2_dev,
                                 uint8_t *packed2_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* Offset form (Section 3.1, Eq. 2) with the scale found by the MMSE search: delta = min_i x_i, the shifted
 * tensor x - delta (one fp32 subtraction per element, formed as the tensor is read) is searched in the unsigned range
 * 0..p->qmax (p->qmin must be 0); the last grid point is Eq. 2's own scale (max - delta)/qmax.
 * x ~ scale*codes + delta.  delta_dev: one float out (NaN when the tensor is rejected: a non-finite element,
 * or max - min above 2^60); sse_dev is the error of the shifted tensor; packed_dev (optional) its codes.
 * Workspace: mmse_workspace_bytes_activation(N, p). */
int mmse_scale_search_offset(const float *x_dev, int64_t N, const mmse_params_t *p, float *delta_dev,
                             float *scale_dev, int32_t *idx_dev, double *sse_dev, uint8_t *packed_dev,
                             void *ws_dev, size_t ws_bytes, void *stream);

/* Q = [x/scale]_Zp (Section 3.4) for a [K][n] tensor with one scale per row, packed
 * two codes per byte in memory order over the whole tensor: element 2m in the low
 * nibble of byte m, element 2m+1 in the high nibble, two's-complement nibbles, a
 * missing last element leaves the high nibble 0.  packed_dev: ceil(K*n/2) bytes.
 * (The paper defines no storage layout; this one is this library's.) */
int quantize_pack_int4(const float *x_dev, int64_t K, int64_t n, const float *scale_dev,
                       int32_t qmin, int32_t qmax, uint8_t *packed_dev, void *stream);

/* Second tensor for a key layer (Section 3.5, Algorithm 1 with j = 2 after j = 1;
 * same mechanism as Eq. 16): R = w - scale1*[w/scale1] is formed on the fly, then
 * searched and coded exactly like a weight tensor.  packed2_dev may be NULL. */
int residual_quantize(const float *w_dev, int64_t K, int64_t n, const float *scale1_dev,
                      const mmse_params_t *p, float *scale2_dev, int32_t *idx2_dev, double *sse2_dev,
                      uint8_t *packed2_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* Algorithm 1 of Section 3.5 iterated for two INT4 tensors, every kernel of a [K][n] layer on its own:
 *   sweep:  (a1,Q1) = phi(w - a2*Q2);  (a2,Q2) = phi(w - a1*Q1)      phi = search + codes of Section 3.4
 * starting from Q2 = 0 (so max_sweeps = 1 is mmse_scale_search_kernelwise + residual_quantize).  The paper
 * does not define its "convergence rate > epsilon"; here a kernel stops after a sweep whose relative gain
 * (E_prev - E)/E_prev is <= eps, when E reaches 0, after max_sweeps (1..64) sweeps, or when a sweep did not
 * lower E (that sweep is discarded: phi is a grid heuristic).  Outputs per kernel k: scale1_dev[k],
 * scale2_dev[k], sse_dev[k] = ||w_k - a1*Q1 - a2*Q2||^2, sweeps_dev[k] = sweeps kept (0 for a rejected
 * kernel); packed1_dev / packed2_dev: codes of the two tensors, ceil(K*n/2) bytes each, layout as in
 * quantize_pack_int4.  All max_sweeps sweeps are enqueued at once; kernels that have stopped are skipped
 * on the device.  Workspace: mmse_workspace_bytes_dual. */
typedef struct mmse_dual_desc_t {
    const float *w_dev;        /* [K][n]                      */
    int64_t K, n;
    float *scale1_dev;         /* [K]                         */
    float *scale2_dev;         /* [K]                         */
    uint8_t *packed1_dev;      /* ceil(K*n/2) bytes           */
    uint8_t *packed2_dev;      /* ceil(K*n/2) bytes           */
    double *sse_dev;           /* [K]                         */
    int32_t *sweeps_dev;       /* [K]                         */
} mmse_dual_desc_t;

int mmse_workspace_bytes_dual(int64_t K, int64_t n, const mmse_params_t *p, size_t *bytes_out);
int dual_quantize_alternating(const float *w_dev, int64_t K, int64_t n, const mmse_params_t *p,
                              double eps, int32_t max_sweeps,
                              float *scale1_dev, float *scale2_dev, uint8_t *packed1_dev, uint8_t *packed2_dev,
                              double *sse_dev, int32_t *sweeps_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* The same for `count` layers described in HOST memory; every phi runs as one batched launch over
 * all layers.  Workspace: mmse_workspace_bytes_dual_batched (the sum of the per-layer sizes).  count in
 * 1..4096, else MMSE_ERR_SIZE. */
int mmse_workspace_bytes_dual_batched(const mmse_dual_desc_t *descs_host, int32_t count,
                                      const mmse_params_t *p, size_t *bytes_out);
int dual_quantize_alternating_batched(const mmse_dual_desc_t *descs_host, int32_t count, const mmse_params_t *p,
                                      double eps, int32_t max_sweeps, void *ws_dev, size_t ws_bytes, void *stream);

/* Dual line search (Section 3.5, Eq. 12) for every kernel of a [K][n] layer, n <= 8192 ("reserved to small
 * tensors (convolutional kernels)"): exhaustive search of a G1 x G2 grid of scale pairs,
 *   a1_a = (max|w_k|/qmax)*(a+1)/G1,   a2_b = a1_a*(b+1)/G2        (the paper gives no grid for a2; this
 *   one covers (0, a1]: the two tensors play symmetric roles),
 * where the error of a pair is sum_i min_t (w_i - a1*t - a2*[(w_i - a1*t)/a2])^2 over all first codes t in
 * [qmin, qmax].  The first of equal minima in row-major (a, b) order is returned:
 *   scale1_dev[k], scale2_dev[k], idx1_dev[k] = a, idx2_dev[k] = b, sse_dev[k], and the two code tensors
 *   (layout of quantize_pack_int4; among equally good first codes the lowest is kept).
 * grid_dev is optional: [K][G1*G2] errors of every pair.  G1, G2 in 1..1024. */
int mmse_workspace_bytes_dual_linesearch(int64_t K, int64_t n, int32_t G1, int32_t G2, size_t *bytes_out);
int dual_line_search(const float *w_dev, int64_t K, int64_t n, int32_t qmin, int32_t qmax, int32_t G1, int32_t G2,
                     float *scale1_dev, float *scale2_dev, int32_t *idx1_dev, int32_t *idx2_dev, double *sse_dev,
                     uint8_t *packed1_dev, uint8_t *packed2_dev, double *grid_dev,
                     void *ws_dev, size_t ws_bytes, void *stream);

/* Comparison optimisers of Section 3.4 (Table 2), error only.  Two of them are grid modes of the search
 * entry points above: grid_points = 1, refine_iters = 0 is the max-abs "Uniform" quantizer of Section 3.1;
 * grid_points = 1, refine_iters = N is a golden-section search over (0, max-abs scale] ("Golden").  The third,
 * alternating optimisation ("Altern."), is this entry point: for every row of a [K][n] tensor start from the
 * max-abs scale and repeat  Q = [w/alpha]_Zp,  alpha = sum_i w_i*Q_i / sum_i Q_i^2  until the scale repeats
 * or max_iters (0..1000) updates were made.  scale_dev[k]: the last scale; sse_dev[k]: the error at it;
 * updates_dev[k]: updates made.  All-zero and rejected rows as in the search entry points.  No workspace. */
int mmse_scale_alternating_kernelwise(const float *w_dev, int64_t K, int64_t n, int32_t qmin, int32_t qmax,
                                      int32_t max_iters, float *scale_dev, double *sse_dev, int32_t *updates_dev,
                                      void *stream);

/* Whole network in a handful of launches: `count` weight tensors described in HOST
 * memory (the descriptors are consumed before the call returns).  Semantics per
 * tensor are those of mmse_scale_search_kernelwise / residual_quantize /
 * quantize_pack_int4.  Workspace: mmse_workspace_bytes_kernelwise(sum K, ...).  count in 1..4096, else
 * MMSE_ERR_SIZE.  Up to 59 tensors are one launch per stage (sweep, refinement by kernel-size class, codes);
 * longer lists run in groups of 59, each with its own launches. */
int mmse_scale_search_batched(const mmse_tensor_desc_t *descs_host, int32_t count,
                              const mmse_params_t *p, void *ws_dev, size_t ws_bytes, void *stream);

/* One activation tensor of a batched call; outputs as in mmse_scale_search_activation (one element each),
 * packed_dev (ceil(N/2) bytes, layout of quantize_pack_int4) optional. */
typedef struct mmse_act_desc_t {
    const float *x_dev;        /* [N]                                      */
    int64_t N;
    float *scale_dev;          /* [1]                                      */
    int32_t *idx_dev;          /* [1]                                      */
    double *sse_dev;           /* [1]                                      */
    uint8_t *packed_dev;       /* ceil(N/2) bytes or NULL                  */
} mmse_act_desc_t;

/* The calibration activations of a whole network (Section 3.7, Eq. 15: one scale per layer input) in one set
 * of launches instead of one per tensor: `count` tensors (1..MMSE_MAX_BATCH_TENSORS) described in HOST memory
 * (consumed before the call returns), every tensor searched exactly as by mmse_scale_search_activation, with
 * the same results; a per-layer search is some thirty dependent launches, most of them tiny, so for a
 * network of many layers sharing them is what keeps the GPU busy.  N_host: the `count` element counts. */
int mmse_workspace_bytes_activation_batched(const int64_t *N_host, int32_t count, const mmse_params_t *p,
                                            size_t *bytes_out);
int mmse_scale_search_activation_batched(const mmse_act_desc_t *descs_host, int32_t count, const mmse_params_t *p,
                                         void *ws_dev, size_t ws_bytes, void *stream);

/* Layer errors for the choice of key layers (Section 3.5: the layers whose MSE is above a threshold get a
 * second tensor): sums_dev[l] = sum_k sse_l[k] for `count` layers (1..MMSE_MAX_BATCH_TENSORS); the pointers
 * sse_dev_ptrs_host[l] (device arrays of K_host[l] doubles, outputs of the searches above) and K_host are read
 * on the host before the call returns.  Fixed summation order, fp64.  The ranking itself is host logic. */
int mmse_layer_error_sums(const double *const *sse_dev_ptrs_host, const int64_t *K_host, int32_t count,
                          double *sums_dev, void *stream);

/* The grid evaluation alone (the f(alpha_j) of Eq. 8 for every candidate):
 * absmax_dev[k] = max_i |w_ki|, grid_sse_dev[k*G + j] = f_k(alpha_kj).  Used to
 * check and to time the candidate sweep by itself. */
int mmse_grid_sse_kernelwise(const float *w_dev, int64_t K, int64_t n, const mmse_params_t *p,
                             float *absmax_dev, double *grid_sse_dev, void *stream);

/* The same for an activation tensor: absmax_dev[0] = max_i |x_i|, grid_sse_dev[j] = f(alpha_j), j < G, summed over
 * the whole tensor in the library's fixed order.  Workspace: mmse_workspace_bytes_activation(N, p). */
int mmse_grid_sse_activation(const float *x_dev, int64_t N, const mmse_params_t *p, float *absmax_dev,
                             double *grid_sse_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* Measurement aid (no part of the method): the two batched searches with a HIP event recorded on `stream`
 * before the first and after every kernel launch, so that a harness can read how long each kernel of a call
 * took without a profiler.  A trace object owns `capacity` (2..4096) events; a traced call overwrites what the
 * trace held.  mmse_trace_read waits for the last event and returns, for each kernel launch i in launch order,
 * stage_out[i] = MMSE_STAGE_* of the kernel and ms_out[i] = time from the previous event to the event after it
 * (kernel duration plus the launch gap, a few microseconds); launches beyond the trace's capacity are not
 * recorded.  Results of a traced call are those of the plain call. */
typedef struct mmse_trace mmse_trace_t;
enum {
    MMSE_STAGE_START = 0,
    MMSE_STAGE_W_SWEEP = 1,         /* k_sweep_kernelwise: abs-max, grid sweep, argmin (Section 3.4);
                                       kernels of <= 64 elements one wave each in the same launch      */
    /* 2: not used */
    MMSE_STAGE_W_REFINE = 3,        /* k_refine_kernelwise<64>: refinement (+ codes when n is even)      */
    MMSE_STAGE_W_REFINE_SMALL = 4,  /* k_refine_kernelwise<16>                                           */
    MMSE_STAGE_W_PACK = 5,          /* k_pack_int4                                                       */
    MMSE_STAGE_W_FUSED = 6,         /* k_sweep_kernelwise, whole search in one launch (small calls)      */
    MMSE_STAGE_A_INIT = 10,
    MMSE_STAGE_A_ABSMAX = 11,       /* k_act_absmax                                                      */
    MMSE_STAGE_A_SWEEP = 12,        /* k_act_sweep (Section 3.7, Eq. 15)                                 */
    MMSE_STAGE_A_REDUCE = 13,       /* k_act_reduce64 over the grid sums                                 */
    MMSE_STAGE_A_ARGMIN = 14,
    MMSE_STAGE_A_PROBE = 15,        /* k_act_probe: one refinement pass over the tensors                 */
    MMSE_STAGE_A_PROBE_REDUCE = 16,
    MMSE_STAGE_A_FINISH = 17,
    MMSE_STAGE_A_PACK = 18          /* k_act_pack                                                        */
};
int mmse_trace_create(int32_t capacity, mmse_trace_t **trace_out);
void mmse_trace_destroy(mmse_trace_t *trace);
int mmse_trace_read(mmse_trace_t *trace, int32_t capacity, int32_t *count_out, int32_t *stage_out, float *ms_out);
int mmse_scale_search_batched_traced(const mmse_tensor_desc_t *descs_host, int32_t count, const mmse_params_t *p,
                                     void *ws_dev, size_t ws_bytes, void *stream, mmse_trace_t *trace);
int mmse_scale_search_activation_batched_traced(const mmse_act_desc_t *descs_host, int32_t count,
                                                const mmse_params_t *p, void *ws_dev, size_t ws_bytes,
                                                void *stream, mmse_trace_t *trace);

const char *mmse_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MMSE_H_ */
