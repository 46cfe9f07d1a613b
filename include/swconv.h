/*
 * swconv - sparse Winograd convolution forward pass for AMD MI355X (gfx950).
 *
 * C ABI.  Plain pointers and sizes only; every pointer argument is marked HOST or DEVICE.
 *
 * The library computes the "Winograd layer" of arxiv 1702.08597, Section 3, Eq. 4:
 *
 *     O~(k,tau,:,:) = A^T [ sum_c W_F(k,c,:,:) (.) ( B^T I~(c,tau,:,:) B ) ] A
 *
 * with W_F a free, natively pruned (sparse) K x C x t x t parameter tensor, t = m + r - 1,
 * in the three steps Section 5 names:
 *   (1) input transform   V[p][c][tau] = (B^T d B)[i][j],  d = the t x t input tile of (c,tau)
 *   (2) per-position sparse x dense product   M[p] = W_F[p] * V[p]   (K x C times C x T),
 *       one for each of the P = t*t Winograd positions p = i*t + j  (remark after Eq. 4's
 *       intermediate variables; Section 5 calls it SpMDM and the bulk of the computation)
 *   (3) output transform  Y = A^T m^ A,  m^[i][j] = M[i*t+j][k][tau], scattered to the output.
 *
 * Conventions (where the paper is silent, these readings are part of the contract):
 *   - fp32 data, int32 indices.  Unit stride and dilation, square r x r kernel, square m x m
 *     output tile (Section 3 assumes unit stride/dilation; A1=A2, B1=B2 when r=s, m=n).
 *   - Supported F(m x m, r x r): (m,r) = (2,3), (4,3) and, for the 5x5 layers of Section 6
 *     (Table 1), (2,5) and (4,5).  A, B are the standard minimal-filtering matrices for points
 *     {0,1,-1,inf}, {0,1,-1,2,-2,inf} and {0,1,-1,2,-2,1/2,-1/2,inf} (the paper defers to Lavin &
 *     Gray for the 3x3 values and names no 5x5 ones):
 *       F(2,3): B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1],  A^T = [1 1 1 0; 0 1 -1 -1]
 *       F(4,3): B^T = [4 0 -5 0 1 0; 0 -4 -4 1 1 0; 0 4 -4 -1 1 0; 0 -2 -1 2 1 0;
 *                      0 2 -1 -2 1 0; 0 4 0 -5 0 1]
 *               A^T = [1 1 1 1 1 0; 0 1 -1 2 -2 0; 0 1 1 4 4 0; 0 1 -1 8 -8 1]
 *       F(2,5): B^T as F(4,3) (same six points),  A^T = [1 1 1 1 1 0; 0 1 -1 2 -2 1]
 *               (for reference, the matching 6 x 5 filter transform has rows
 *                [1/4 0 0 0 0], -1/6 [1 1 1 1 1], -1/6 [1 -1 1 -1 1], 1/24 [1 2 4 8 16],
 *                1/24 [1 -2 4 -8 16], [0 0 0 0 1]; the library itself never applies it: W_F is
 *                given in the Winograd domain)
 *       F(4,5): t = 8.  Row i of B^T = coefficients, ascending powers, of prod_{k != i} (x - p_k)
 *               over the seven finite points p = (0, 1, -1, 2, -2, 1/2, -1/2), last row those of
 *               prod_k (x - p_k):
 *               B^T = [-1 0 21/4 0 -21/4 0 1 0; 0 1 1 -17/4 -17/4 1 1 0; 0 -1 1 17/4 -17/4 -1 1 0;
 *                      0 1/2 1/4 -5/2 -5/4 2 1 0; 0 -1/2 1/4 5/2 -5/4 -2 1 0; 0 2 4 -5/2 -5 1/2 1 0;
 *                      0 -2 4 5/2 -5 -1/2 1 0; 0 -1 0 21/4 0 -21/4 0 1]
 *               A^T = [1 1 1 1 1 1 1 0; 0 1 -1 2 -2 1/2 -1/2 0; 0 1 1 4 4 1/4 1/4 0;
 *                      0 1 -1 8 -8 1/8 -1/8 1]
 *               (matching filter transform: G[i][j] = p_i^j / prod_{k != i} (p_i - p_k), last row e_4)
 *   - Ho = H + 2*pad - r + 1, Wo likewise; th = ceil(Ho/m), tw = ceil(Wo/m); T = N*th*tw.
 *     Tile tau = (n*th + ty)*tw + tx reads input rows ty*m - pad ... ty*m - pad + t - 1 (zero
 *     outside the image: this covers both the convolution padding and a ragged last tile, per
 *     the footnote to the divisibility assumption in Section 3) and owns output rows
 *     ty*m ... ty*m + m - 1; outputs outside Ho x Wo are computed and dropped.
 *   - Inputs must be finite: a structural zero of W_F is skipped, not multiplied.
 *
 * Every function returns a swconv_status (0 = success); nothing throws or aborts across the
 * ABI; output arguments are untouched on failure unless stated otherwise.
 */
#ifndef SWCONV_H
#define SWCONV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct swconv_plan swconv_plan; /* opaque, owned by the library */

typedef enum {
  SWCONV_OK = 0,
  SWCONV_EINVAL = 1,       /* bad shape, null pointer, malformed CSR                 */
  SWCONV_EUNSUPPORTED = 2, /* an F(m,r) that is not built; sizes beyond the kernels   */
  SWCONV_ENOMEM = 3,       /* host or device allocation failed                       */
  SWCONV_EHIP = 4,         /* HIP runtime error (no device, launch failure, ...)     */
  SWCONV_ESTATE = 5        /* forward before weights were set                        */
} swconv_status;

/* Human-readable name of a status code; never NULL; static storage. */
const char* swconv_status_string(int status);

/*
 * Create a plan for one layer shape (Eq. 1/Eq. 4 dimensions: N images, C input channels of
 * H x W, K output channels; F(m x m, r x r); zero padding `pad` on all four sides).
 * Touches no device: device buffers (V, M workspaces, packed weights) are allocated by the
 * first swconv_set_weights / swconv_set_weights_dense on the then-current HIP device.
 * Errors: EINVAL for non-positive sizes, pad < 0, Ho or Wo < 1 or index ranges beyond int32;
 * EUNSUPPORTED for an unsupported (m,r) or a shape whose panels do not fit the kernels' LDS
 * budget (C > 638).  On success *out owns the plan; release with swconv_plan_destroy.
 */
int swconv_plan_create(swconv_plan** out, int N, int C, int H, int W, int K, int m, int r, int pad);

/* Frees the plan and every host and device buffer it owns.  NULL is allowed. */
void swconv_plan_destroy(swconv_plan* plan);

/*
 * Set the pruned Winograd-domain weights as per-position CSR (Section 2 names CSR as the
 * general sparse format; Section 5: one sparse K x C matrix per position).
 *   rowptr  HOST, P*K + 1 entries, rowptr[0] = 0, non-decreasing, global offsets: row (p,k)
 *           is [rowptr[p*K + k], rowptr[p*K + k + 1]).
 *   colidx  HOST, nnz = rowptr[P*K] entries, 0 <= c < C, strictly ascending within a row.
 *   vals    HOST, nnz entries; vals[q] = W_F[k][c][i][j] with p = i*t + j.  Stored zeros are
 *           legal and are treated as non-zeros.  nnz = 0 is legal (colidx/vals may be NULL).
 * The arrays are validated, re-packed into the kernels' sliced layout (rows of a position
 * sorted by length, grouped four at a time, padded with zero weights) together with a
 * static, cost-balanced schedule for the persistent workgroups of the sparse product, and copied
 * to the device before the call returns; the caller keeps ownership of its arrays.  May be called
 * again with a new pattern; what the workspaces hold then counts as stale (swconv_debug_copy_V / _M and a
 * swconv_backward with in_dev = NULL return ESTATE until the next forward pass).  Blocks the host.
 * Errors: EINVAL on any CSR violation (the plan keeps its previous weights); ENOMEM; EHIP when
 * no device is usable - the host-side packed copy is still kept in that case, so
 * swconv_debug_export_weights works without a GPU.
 */
int swconv_set_weights(swconv_plan* plan, const int32_t* rowptr, const int32_t* colidx, const float* vals);

/*
 * Forward pass of Eq. 4 with the sparse weights: three kernels (Section 5's steps 1-3)
 * enqueued on `hip_stream` (a hipStream_t; NULL = the default stream).  Asynchronous: returns
 * after enqueueing, does not synchronise.  For m = 2 layers with at most 128 input channels
 * whose rows have at most 32 stored entries (the 5x5 layer of Section 6) steps 2 and 3 run as
 * ONE kernel that keeps the per-position products on chip (Section 5: a core that owns its
 * tiles through all steps can fuse the second and third); the environment variable
 * SWCONV_FUSE_OUTPUT=0, read by swconv_plan_create, keeps such a plan on three kernels.
 * SWCONV_FUSE_OUTPUT=2 also runs F(4x4,3x3) layers with C a multiple of 4, C <= 256 and rows of
 * at most 224 stored entries through a fused kernel of their own (measured slower than the two
 * kernels on the layers tried, hence not the default).
 *   in_dev   DEVICE, N x C x H x W fp32, contiguous (W fastest), read-only.
 *   out_dev  DEVICE, N x K x Ho x Wo fp32, contiguous; every element is overwritten.
 * The two must not alias and must live on the device the weights were set on.  The plan owns
 * the V and M workspaces, so one plan must not run on two streams at once.  The call allocates
 * nothing and enqueues kernels only: after one eager call (which sets kernel attributes once per
 * process) it may be recorded into a HIP graph; the same holds for swconv_backward once one eager
 * backward pass has packed the transposed weights.
 * Errors: EINVAL (null), ESTATE (no weights), EHIP (launch failure).
 */
int swconv_forward(swconv_plan* plan, void* hip_stream, const float* in_dev, float* out_dev);

/*
 * swconv_forward for callers that cannot allocate device memory and do not want every plan to hold
 * workspaces of its own: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The same kernels as swconv_forward, with the two intermediates (V, then M on the
 * next 256-byte boundary) in a static device array of SWCONV_STATIC_SCRATCH_BYTES (64 MiB) that
 * the library's code object carries: every GPU the library runs on holds one copy until the
 * process ends, and all plans share it.  The call allocates and frees nothing and calls no
 * allocating routine; the array's device address is looked up once per device (by the first
 * swconv_set_weights on that device, else by the first call here).  Arguments, asynchrony and
 * results as for swconv_forward: the output is bit-identical to it.
 * Limits: 4*P*(C+K)*Tp bytes (Tp = T rounded up to 128), rounded as above, must fit the array -
 * e.g. the N = 32, 256 -> 384, 13 x 13, F(4x4,3x3) layer (47.2 MB) does, N = 64 does not:
 * SWCONV_EUNSUPPORTED, nothing is launched.  Calls on one GPU share the array, whatever their
 * plans or streams: two calls that overlap in time race; order them on one stream or with events.
 * The array keeps the last call's contents, and nothing in it has to start at zero (step 1
 * writes every column of V and step 2 every row of M that a later step reads).  The plan's own
 * workspaces are untouched, so swconv_debug_copy_V / _M and a swconv_backward with in_dev = NULL
 * return ESTATE until a swconv_forward has run.
 * Errors: EINVAL (null), ESTATE (no weights), EUNSUPPORTED (too large; more than 64 devices),
 * EHIP (symbol lookup or launch failure).
 */
#define SWCONV_STATIC_SCRATCH_BYTES (64u << 20)
int swconv_forward_noalloc(swconv_plan* plan, void* hip_stream, const float* in_dev, float* out_dev);

/*
 * The 0 %-sparsity comparison: the same layer with a dense W_F, computed with the same
 * transforms and a dense batched fp32 MFMA product for step 2.  Not the paper's method - the
 * paper has no dense Winograd implementation and projects one (Section 6.2); this is the
 * in-house baseline the sparse path is compared with.
 *   wf  HOST, [P][K][C] fp32, wf[p][k][c] = W_F[k][c][i][j].
 * Errors as for swconv_set_weights / swconv_forward.
 */
int swconv_set_weights_dense(swconv_plan* plan, const float* wf);
int swconv_forward_dense(swconv_plan* plan, void* hip_stream, const float* in_dev, float* out_dev);

/*
 * Backward pass of the layer (Section 3, Eq. 5 and Eq. 6) for L a scalar loss: from dL/dO to
 *   dL/dZ(k,tau) = A dL/dO~(k,tau) A^T,          dL/dO~ = dL/dO read through psi^-1 (zero where a tile
 *                                                reaches past Ho x Wo: those outputs were dropped)
 *   dL/dW_F(:,:,p) = dL/dZ(:,:,p) I_F(:,:,p)^T,  at the stored entries of the pruned W_F only
 *   dL/dI_F(:,:,p) = W_F(:,:,p)^T dL/dZ(:,:,p),  dL/dI~ = B dL/dI_F B^T,  dL/dI = overlap-add through phi
 * enqueued on `hip_stream`.
 *   in_dev     DEVICE, N x C x H x W, the input of the forward pass (I_F is recomputed from it); or NULL:
 *              I_F is taken from the plan's workspace, where the last swconv_forward on this plan left it
 *              (ESTATE if a backward pass or no forward pass came after swconv_set_weights; only needed
 *              for dL/dW_F)
 *   dout_dev   DEVICE, N x K x Ho x Wo, dL/dO
 *   din_dev    DEVICE, N x C x H x W or NULL: dL/dI, every element overwritten
 *   dvals_dev  DEVICE, nnz floats or NULL: dL/dW_F at the stored entries, in the order of the CSR
 *              arrays given to swconv_set_weights
 * The first call after swconv_set_weights also packs the transposed weights on the host and blocks.
 * Overwrites the plan's workspaces (swconv_debug_copy_V / _M then see backward data).
 * Errors: EINVAL, ESTATE (no weights), EUNSUPPORTED (K > 638: the panels of dL/dZ do not fit LDS; or
 * N*C*(H+m)*(W+m) >= 2^31), ENOMEM, EHIP.
 */
int swconv_backward(swconv_plan* plan, void* hip_stream, const float* in_dev, const float* dout_dev, float* din_dev,
                    float* dvals_dev);

/*
 * One pruning step on the stored entries of W_F (Section 4.2): the SGD step of Eq. 9 on L + lambda |w|_1
 * (Eq. 7; the subgradient of |w| at 0 is taken as 0), then the thresholding function of Eq. 8,
 *     w' = w - eta (dL/dw + lambda sign w),   T(w') = 0 if |w'| (|dL/dw| + beta) < eps, else w'
 * with dL/dw the gradient the step was taken with (e.g. the dvals of swconv_backward), and the per-position
 * CSR of the entries that survive.  The paper recommends eps = 1e-4, beta = 0.1.  fp32, one rounding per
 * operation (sum, fused multiply-add, sum, product), so the keep/drop decision is reproducible.
 * Enqueued on `hip_stream` (three small kernels); independent of any plan.
 *   rows            P*K, the CSR rows
 *   rowptr_dev      DEVICE, rows + 1 entries; colidx_dev, vals_dev, grad_dev DEVICE, nnz entries, CSR order
 *   updated_dev     DEVICE, nnz floats: T(w') in the OLD pattern (0 where dropped); must not alias vals_dev
 *                   (the last kernel takes the decisions again from vals_dev)
 *   rowptr_out_dev  DEVICE, rows + 1 entries; colidx_out_dev, vals_out_dev DEVICE, capacity nnz: the new CSR;
 *                   its entry count is rowptr_out_dev[rows]
 * Errors: EINVAL (null pointers, rows < 1, a negative or NaN hyper-parameter), EHIP.
 */
int swconv_prune_step(int64_t rows, const int32_t* rowptr_dev, const int32_t* colidx_dev, const float* vals_dev,
                      const float* grad_dev, float eta, float lambda, float eps, float beta, void* hip_stream,
                      float* updated_dev, int32_t* rowptr_out_dev, int32_t* colidx_out_dev, float* vals_out_dev);

/*
 * swconv_set_weights for CSR arrays that live on the device (e.g. the output of swconv_prune_step): waits
 * for `hip_stream`, copies the arrays to the host (the re-packing is host code) and proceeds as
 * swconv_set_weights.  Blocks the host.  Errors as for swconv_set_weights, EHIP for a failed copy.
 */
int swconv_set_weights_device(swconv_plan* plan, void* hip_stream, const int32_t* rowptr_dev,
                              const int32_t* colidx_dev, const float* vals_dev);

/*
 * Fine-tuning with the sparsity pattern fixed (Section 4.3): new values for the weights set last,
 * same rowptr and colidx.  Nothing is re-packed and nothing crosses to the host: one small kernel
 * per packed copy of W_F (the forward stream, the fused kernel's packages, the transposed stream of
 * the backward pass if it exists) writes the values in place, enqueued on `hip_stream`.
 *   vals_dev  DEVICE, nnz floats in the order of the colidx passed to swconv_set_weights.
 * Passes enqueued later on the same stream see the new values; a pass on another stream needs
 * the caller's own ordering.  Errors: ESTATE (no weights), EINVAL (null), EHIP.
 */
int swconv_update_values(swconv_plan* plan, void* hip_stream, const float* vals_dev);

/*
 * Measurement helper for the backward pass: `iters` passes with every kernel launched with its own
 * pair of HIP events (as swconv_profile_forward); mean milliseconds per kernel, in launch order:
 *   stage_ms  HOST, 7 floats: dL/dZ transform, input transform (I_F again), sampled products,
 *             reduction to CSR order, transposed sparse product, patch transform, gather;
 *             0 for kernels the call does not run (din_dev or dvals_dev NULL).  Where the image
 *             planes fit LDS (3x3 filters) the last two run as one kernel that keeps no patch
 *             buffer: the sixth value is its time and the seventh is 0 (the environment
 *             variable SWCONV_FUSE_INPUT_GRAD=0, read by swconv_plan_create, keeps two kernels).
 * Blocks the host.  Errors as for swconv_backward; EINVAL for iters < 1.
 */
int swconv_profile_backward(swconv_plan* plan, void* hip_stream, const float* in_dev, const float* dout_dev,
                            float* din_dev, float* dvals_dev, int iters, float* stage_ms);

/* Test hooks: intermediates of the last backward pass, canonical layouts.
 *   dZ_host  HOST, [P][K][T] (dL/dZ)      dV_host  HOST, [P][C][T] (dL/dI_F)
 * Errors: ESTATE when no backward pass has run; EHIP. */
int swconv_debug_copy_dZ(swconv_plan* plan, float* dZ_host);
int swconv_debug_copy_dV(swconv_plan* plan, float* dV_host);

/*
 * Measurement helper: run `iters` sparse forward passes on `hip_stream`, every kernel launched
 * with a pair of HIP events that take the kernel's own start and end time stamps on that stream
 * (no extra packets between the kernels), synchronise, and return the mean duration of each
 * step in milliseconds.
 *   stage_ms  HOST, 3 floats: input transform, sparse product, output transform; when steps
 *             2 and 3 run fused, the second is that kernel's time and the third is 0.
 * Blocks the host.  Errors as for swconv_forward; EINVAL for iters < 1.
 */
int swconv_profile_forward(swconv_plan* plan, void* hip_stream, const float* in_dev, float* out_dev, int iters,
                           float* stage_ms);

/*
 * Test hooks (not on the timed path).  They synchronise the device and copy the intermediates
 * of the last forward into caller buffers in the canonical layouts of the definition above.
 *   V_host  HOST, [P][C][T] fp32        M_host  HOST, [P][K][T] fp32
 * After a forward pass with steps 2 and 3 fused M was never stored: swconv_debug_copy_M then runs
 * step 2 alone on the V of that pass (default stream) before copying.
 * Errors: ESTATE when no forward has run; EHIP.
 */
int swconv_debug_copy_V(swconv_plan* plan, float* V_host);
int swconv_debug_copy_M(swconv_plan* plan, float* M_host);

/*
 * Round trip of the re-packed sparse weights: unpacks the host-side copy of the sliced layout
 * back to per-position CSR (padding dropped, rows back in their original order).
 *   rowptr HOST P*K + 1 entries; colidx, vals HOST nnz entries each (nnz as passed to
 *   swconv_set_weights).  The result equals that call's arrays bit for bit.
 * Errors: ESTATE when no sparse weights were set.
 */
int swconv_debug_export_weights(swconv_plan* plan, int32_t* rowptr, int32_t* colidx, float* vals);

/*
 * Verifies the static schedule of the sparse product on the host: every (position, tile block,
 * slice) unit is assigned to exactly one persistent workgroup, no launched workgroup is idle and
 * no work item has more slices than the kernel stages descriptors for.
 * Returns SWCONV_OK, or SWCONV_EINVAL when the schedule is not a partition; ESTATE when no sparse
 * weights were set.  Needs no GPU.
 */
int swconv_debug_check_schedule(const swconv_plan* plan);

/*
 * Channel groups (the grouped 5x5 and 3x3 layers of AlexNet, Section 6): a plan made for the C
 * input and K output channels of ONE group can work inside the tensors of the whole layer.  The
 * strides are the distances, in floats, between consecutive images of the input / dL/dI tensor
 * (in_stride >= C*H*W) and of the output / dL/dO tensor (out_stride >= K*Ho*Wo); 0 restores the
 * dense default.  The caller then passes pointers to the group's first channel of image 0, e.g.
 * in + g*C*H*W with in_stride = G*C*H*W.  Applies to every later forward and backward call;
 * channels outside the group are neither read nor written.  Errors: EINVAL for a stride below
 * the dense one or so large that the last image's offset leaves 2^40 floats.
 */
int swconv_plan_set_image_strides(swconv_plan* plan, int64_t in_stride, int64_t out_stride);

/*
 * Sizes derived by the plan (any pointer may be NULL): positions P, tiles T, Ho, Wo.
 */
int swconv_plan_sizes(const swconv_plan* plan, int* P, int64_t* T, int* Ho, int* Wo);

/*
 * Statistics of the packed weights and the work list built by swconv_set_weights:
 *   nnz          stored entries as passed in
 *   padded_nnz   entries after padding to the sliced layout (what the kernel multiplies)
 *   work_items   entries of the statically scheduled work list
 *   max_item     padded entries multiplied by the heaviest persistent workgroup
 * Errors: ESTATE when no sparse weights were set.
 */
int swconv_plan_weight_stats(const swconv_plan* plan, int64_t* nnz, int64_t* padded_nnz, int* work_items,
                             int64_t* max_item);

#ifdef __cplusplus
}
#endif
#endif /* SWCONV_H */
