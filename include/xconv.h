/*
 * xconv.h -- C ABI of the MI355X (gfx950) XConv weight-gradient library.
 *
 * The library implements the low-memory stochastic weight gradient of a 2-D
 * convolutional layer (Algorithm 1 of the paper) with probing vectors that act
 * on the channel axis:
 *
 *   forward   Xt[b,j,y,x] = sum_n Z[n,j] X[b,n,y,x]                 (Alg. 1 fwd step 3; Eq. (6) step (i))
 *   backward  G[m,j,ky,kx] = sum_{b,oy,ox} dY[b,m,oy,ox] Xt[b,j,oy*sh+ky-ph, ox*sw+kx-pw]
 *                                                                    (Alg. 1 bwd step 3 and the shift of step 4)
 *             dW[m,n,ky,kx] = (1/r) sum_j Z[n,j] G[m,j,ky,kx]        (Alg. 1 bwd step 4; Eq. (6) step (iii))
 *   exact     dW[m,n,ky,kx] = sum_{b,oy,ox} dY[b,m,oy,ox] X[b,n,oy*sh+ky-ph, ox*sw+kx-pw]
 *                                                                    (Eq. (2) / Eq. (5))
 *
 * Z is [C_in, r] with i.i.d. unit-variance entries (E[z z^T] = I, Eq. (3)); taps
 * outside the image contribute zero (zero padding, cross-correlation, dilation
 * 1, groups 1).  H' = floor((H + 2*pad_h - kH)/stride_h) + 1, W' likewise.
 *
 * Conventions for every entry point
 *   - "_dev" pointers are device (HBM) addresses on the current HIP device,
 *     "_host" pointers are host addresses.  All buffers are owned and allocated
 *     by the caller; the library allocates no device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Device work is enqueued on it and the call returns without waiting.
 *     A call issues kernel launches only (no allocation, no memset, no copy, no
 *     synchronisation), so it may be recorded into a HIP graph by stream capture;
 *     the first call for a kernel sets that kernel's LDS attribute and is best
 *     made once outside a capture.
 *   - Return value: an xconv_status.  Arguments are validated on the host before
 *     anything is enqueued; on a non-zero status nothing was launched (except
 *     XCONV_EHIP, which reports a failed launch).  Nothing aborts or throws.
 *   - dW is overwritten, never accumulated into.
 */
#ifndef XCONV_H
#define XCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    XCONV_OK = 0,
    XCONV_EINVAL = 1,       /* null pointer, non-positive extent, empty output, bad enum   */
    XCONV_EUNSUPPORTED = 2, /* valid but not implemented (see xconv_check_desc)             */
    XCONV_EWORKSPACE = 3,   /* ws_bytes smaller than xconv_workspace_bytes()                */
    XCONV_EHIP = 4          /* the HIP runtime reported an error while enqueuing            */
} xconv_status;

typedef enum { XCONV_F32 = 0, XCONV_BF16 = 1, XCONV_F16 = 2 } xconv_dtype;   /* storage of X, dY, Xt; sums and dW are fp32 */
typedef enum { XCONV_NCHW = 0, XCONV_NHWC = 1 } xconv_layout;                /* of X and dY ([B,C,H,W] or [B,H,W,C]); dW is always [C_out,C_in,kH,kW] */
typedef enum { XCONV_RADEMACHER = 0, XCONV_GAUSSIAN = 1, XCONV_USER_Z = 2 } xconv_probe;
typedef enum { XCONV_OP_PROBE = 0, XCONV_OP_ESTIMATE = 1, XCONV_OP_EXACT = 2 } xconv_op;

/* Problem statement of one layer (Algorithm 1: X, dY, the seed s and r; the
 * layer arguments in/out channels, kernel, stride, padding). */
typedef struct xconv_desc {
    int32_t B, C_in, C_out, H, W;            /* input extent                                         */
    int32_t kH, kW;                          /* kernel extent                                        */
    int32_t stride_h, stride_w, pad_h, pad_w;
    int32_t r;                               /* number of probing vectors, >= 1                      */
    int32_t dtype;                           /* xconv_dtype                                          */
    int32_t layout;                          /* xconv_layout                                         */
    int32_t probe;                           /* xconv_probe: how Z is obtained when no Z is passed   */
    int32_t keep_q15;                        /* 0: dense probes, scaled by 1/r (Eq. (3), (6)).
                                              * 1..32767: block-sparse probes (Eq. (7)): every entry
                                              * Z[n,j] is kept with probability keep_q15/32768 and is
                                              * zero otherwise (one probability for all n), and the
                                              * estimate of input channel n is scaled by 1/nnz(Z_n),
                                              * the number of non-zero entries of row n of Z (Eq. (8));
                                              * a row without any gives zeros.  With a caller's Z
                                              * any non-zero value selects that scaling.              */
    uint64_t seed;                           /* Algorithm 1's s: same value in forward and backward  */
} xconv_desc;

/* Host-only validation.  XCONV_EINVAL: null desc, an extent < 1, stride < 1,
 * pad < 0, r < 1, H' or W' < 1, unknown enum, keep_q15 outside 0..32767.
 * XCONV_EUNSUPPORTED: r > 1024; C_in or C_out > 65536; kH*kW > 49;
 * an extent whose tensors exceed 2^31-1 elements per image plane. */
xconv_status xconv_check_desc(const xconv_desc *desc);

/* Bytes of the stored probe output Xt.  Its layout is the library's own
 * ([B, H, W, r rounded up to 16] in the storage dtype); callers treat it as
 * opaque and keep it between forward and backward.  0 for an invalid desc. */
size_t xconv_xt_bytes(const xconv_desc *desc);

/* Bytes of device scratch the given op (xconv_op) needs in `ws_dev`.  The
 * scratch holds Z (fp32, and for the probe in matrix-core operand order) when
 * it is regenerated from the seed, the split partial sums
 * of the correlation, a repacked copy of dY when H'*W' is not a whole number of
 * 16-byte vectors or dY is channels-last (the correlation reads dY as planes; the
 * copy costs one extra read and write of dY) and, for the exact gradient, a
 * channels-last copy of X (not needed for an NHWC X whose C_in is a multiple of 16).
 * 0 for an invalid desc. */
size_t xconv_workspace_bytes(const xconv_desc *desc, int op);

/* Z[s] on the host: fills Z_host[C_in*r] (row-major [C_in][r], fp32) with the
 * probing matrix that `desc->probe` and `desc->seed` define (Alg. 1 fwd step 2
 * / bwd step 2).  Rademacher: +1/-1 from the top bit of word c*r+j of the
 * SplitMix64 stream of the seed.  Gaussian: Box-Muller in double on words
 * 2(c*r+j), 2(c*r+j)+1, rounded to fp32.  keep_q15 != 0: entry c*r+j is then
 * zeroed unless the top 15 bits of word c*r+j of the stream of
 * (seed xor 0x5851F42D4C957F2D) are below keep_q15.  XCONV_EINVAL for XCONV_USER_Z. */
xconv_status xconv_probe_matrix(const xconv_desc *desc, float *Z_host);

/* The same matrix generated on the device into Z_dev[C_in*r] (fp32). */
xconv_status xconv_probe_matrix_dev(const xconv_desc *desc, float *Z_dev, void *stream);

/* Forward probe (Alg. 1 fwd step 3).  X_dev: [B,C_in,H,W] (or [B,H,W,C_in] for
 * XCONV_NHWC, read directly) in desc->dtype.
 * Xt_dev: xconv_xt_bytes() bytes, written once.  Z_dev: [C_in,r] fp32 or NULL;
 * NULL draws Z from (probe, seed) into the workspace (XCONV_USER_Z then is
 * XCONV_EINVAL).  Sums are fp32; Xt is rounded once (nearest even) to
 * desc->dtype.  ws_dev may be NULL when Z_dev is given; with a workspace Z is
 * first laid out once in the matrix-core operand order, without one every
 * workgroup gathers its operands from Z_dev (same result, slower).  A non-NULL
 * ws_dev smaller than xconv_workspace_bytes(XCONV_OP_PROBE) is
 * XCONV_EWORKSPACE. */
xconv_status xconv_probe_fwd(const xconv_desc *desc, const void *X_dev, void *Xt_dev,
                             const float *Z_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* Backward estimate (Alg. 1 bwd steps 1-4).  dY_dev: [B,C_out,H',W'] (or
 * [B,H',W',C_out] for XCONV_NHWC) in desc->dtype, 16-byte aligned.  Xt_dev: as written by xconv_probe_fwd for the same desc.
 * Z_dev: as above (must be the Z used in the forward).  dW_dev:
 * [C_out,C_in,kH,kW] fp32, overwritten.  The result is deterministic for given
 * inputs (fixed-order two-pass reduction, no atomics). */
xconv_status xconv_dw_estimate(const xconv_desc *desc, const void *dY_dev, const void *Xt_dev,
                               const float *Z_dev, float *dW_dev,
                               void *ws_dev, size_t ws_bytes, void *stream);

/* xconv_dw_estimate for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): no workspace argument.
 * The scratch is a device array inside the library, XCONV_STATIC_SCRATCH_BYTES per GPU the
 * library runs on, held until the process ends; its address is looked up once per device, on
 * the first call with that device current.  The call allocates and frees nothing.  Arguments,
 * result and status as xconv_dw_estimate; XCONV_EWORKSPACE when
 * xconv_workspace_bytes(desc, XCONV_OP_ESTIMATE) exceeds XCONV_STATIC_SCRATCH_BYTES (nothing is
 * launched then), XCONV_EHIP when the runtime does not give the array's address.  All calls on
 * one GPU share the one array: calls that overlap in time on a GPU (two streams, two threads)
 * race on it, so issue them on one stream or order them with events. */
#define XCONV_STATIC_SCRATCH_BYTES (40u * 1024u * 1024u)
size_t xconv_static_scratch_bytes(void);
xconv_status xconv_dw_estimate_static(const xconv_desc *desc, const void *dY_dev, const void *Xt_dev,
                                      const float *Z_dev, float *dW_dev, void *stream);

/* Exact weight gradient (Eq. (2)/(5)), for comparison with the estimate: same
 * correlation kernel with the C_in real channels in place of the r probed
 * ones.  X_dev: [B,C_in,H,W] (XCONV_NHWC: X and dY channels-last); dY_dev 16-byte aligned; dW_dev: [C_out,C_in,kH,kW] fp32, overwritten.
 * desc->r, probe and seed are ignored (r must still be >= 1). */
xconv_status xconv_dw_exact(const xconv_desc *desc, const void *dY_dev, const void *X_dev,
                            float *dW_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* The rest of the layer (Sec. 2: the forward pass and the backpropagation through the layer
 * stay exact, only the weight gradient is estimated; Alg. 1 forward step 1), so that a layer can
 * run on this library alone:
 *
 *   xconv_conv_fwd   Y[b,m,oy,ox]  = sum_{n,ky,kx} W[m,n,ky,kx] X[b,n, oy*sh+ky-ph, ox*sw+kx-pw]
 *   xconv_dx_exact   dX[b,n,iy,ix] = sum_{m,ky,kx} W[m,n,ky,kx] dY[b,m,oy,ox]
 *                                    over the (oy, ox) with oy*sh+ky-ph = iy, ox*sw+kx-pw = ix
 *
 * (zero padding, cross-correlation, no bias).  X, Y, dY, dX in desc->dtype and desc->layout
 * ([B,C,H,W] or [B,H,W,C]); W_dev: [C_out,C_in,kH,kW] in desc->dtype, row-major, for both layouts.
 * Sums are fp32, the output is rounded once (nearest even) and overwritten.  No scratch; one
 * kernel launch each; desc->r, probe and seed are ignored.  Pointers aligned to the element size.
 * XCONV_EUNSUPPORTED when an image of X or Y has more than 2^31-1 elements. */
xconv_status xconv_conv_fwd(const xconv_desc *desc, const void *X_dev, const void *W_dev, void *Y_dev, void *stream);
xconv_status xconv_dx_exact(const xconv_desc *desc, const void *dY_dev, const void *W_dev, void *dX_dev, void *stream);

/* Launch plan of the correlation kernel for op XCONV_OP_ESTIMATE or
 * XCONV_OP_EXACT, for reports and tests (host only).  Fills out[0..15] with
 * K-splits S, steps NS, rows per step RB, columns per step CW, waves along
 * output channels WM, along probe columns WJ, along the k-steps WK, workgroup
 * tile M_WG, J_WG, LDS bytes, tiles NTM, NTJ, offset groups NOG, column stride
 * CS, dY vector chunks per row NCHR, 0. */
xconv_status xconv_plan_info(const xconv_desc *desc, int op, int32_t *out);

/* Test helper: writes the stored Xt as plain fp32 [B,r,H,W] into out_dev. */
xconv_status xconv_xt_unpack(const xconv_desc *desc, const void *Xt_dev, float *out_dev, void *stream);

/* ---- volumetric layers (3-D convolution) --------------------------------------
 * The paper's implementations cover 2-D and 3-D convolutional layers (appendix
 * "Implementation and code"; the experiment "Volumetric segmentation under
 * finetuning" uses 3x3x3 kernels on 96^3 patches).  The estimator of Algorithm 1
 * is the same with one more spatial axis:
 *
 *   Xt[b,j,z,y,x]     = sum_n Z[n,j] X[b,n,z,y,x]
 *   G[m,j,kz,ky,kx]   = sum_{b,oz,oy,ox} dY[b,m,oz,oy,ox] Xt[b,j,oz*sd+kz-pad_d, oy*sh+ky-ph, ox*sw+kx-pw]
 *   dW[m,n,kz,ky,kx]  = (1/r) sum_j Z[n,j] G[m,j,kz,ky,kx]
 *
 * `l` states the layer in the plane (B, channels, H, W, kH, kW, strides, pads, r,
 * dtype, probe, keep_q15, seed) exactly as for a 2-D layer; D, kD, stride_d (sd above)
 * and pad_d add the depth axis, D' = floor((D + 2*pad_d - kD)/stride_d) + 1.  Supported:
 * pad_d <= kD-1 and kD <= 7; anything else is XCONV_EUNSUPPORTED.  l.layout ==
 * XCONV_NCHW means X [B,C_in,D,H,W] and dY [B,C_out,D',H',W'], XCONV_NHWC the
 * channels-last forms [B,D,H,W,C_in] and [B,D',H',W',C_out] (X is then read in place
 * by the probe, dY always through the slice-major copy).
 * dW is [C_out,C_in,kD,kH,kW] fp32.
 * The conventions of the 2-D entry points (pointers, stream, status, alignment,
 * determinism, Z_dev / seed handling) hold unchanged. */
typedef struct xconv3d_desc {
    xconv_desc l;
    int32_t D, kD, stride_d, pad_d;
} xconv3d_desc;

/* Host-only validation: `l` as xconv_check_desc; XCONV_EINVAL for D, kD or stride_d
 * < 1, pad_d < 0 or D' < 1; XCONV_EUNSUPPORTED as stated above and for volumes of more
 * than 2^28 voxels per channel. */
xconv_status xconv3d_check_desc(const xconv3d_desc *desc);

/* Bytes of the stored probe output (opaque layout: depth slices [H,W,r rounded up
 * to 16], zero slices between images, one run of slices per residue of the depth
 * index modulo stride_d) and of the scratch of an op
 * (xconv_op); 0 for an invalid desc.  The scratch of the two gradient ops
 * includes room for a slice-major copy of dY, which is made (one extra read and
 * write of dY) unless the correlation kernel can read dY in place: a layer the
 * producer/consumer kernels take (fp32 with W' a multiple of 4; 16-bit storage with
 * W' even and r a multiple of 32; kernels larger than 1x1), dY 16-byte aligned and
 * smaller than 1 GiB. */
size_t xconv3d_xt_bytes(const xconv3d_desc *desc);
size_t xconv3d_workspace_bytes(const xconv3d_desc *desc, int op);

/* Forward probe of a volumetric layer; arguments as xconv_probe_fwd. */
xconv_status xconv3d_probe_fwd(const xconv3d_desc *desc, const void *X_dev, void *Xt_dev,
                               const float *Z_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* Backward estimate of a volumetric layer; arguments as xconv_dw_estimate, ws_dev
 * required.  Runs the 2-D correlation once per kernel-depth offset on the depth
 * slices of all images, then one expansion over the kD*kH*kW offsets. */
xconv_status xconv3d_dw_estimate(const xconv3d_desc *desc, const void *dY_dev, const void *Xt_dev,
                                 const float *Z_dev, float *dW_dev,
                                 void *ws_dev, size_t ws_bytes, void *stream);

/* Exact weight gradient of a volumetric layer (Eq. (2)/(5) over kD*kH*kW offsets), for
 * comparison with the estimate; arguments as xconv_dw_exact with X_dev [B,C_in,D,H,W].
 * The scratch holds a channels-last copy of X in depth slices. */
xconv_status xconv3d_dw_exact(const xconv3d_desc *desc, const void *dY_dev, const void *X_dev,
                              float *dW_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* Test helper: writes the stored Xt as plain fp32 [B,r,D,H,W] into out_dev. */
xconv_status xconv3d_xt_unpack(const xconv3d_desc *desc, const void *Xt_dev, float *out_dev, void *stream);

/* ---- probing vectors over pixels and channels ----------------------------------
 * The estimator as the paper states it (Sec. 3 multi-channel case, Eq. (6); Algorithm
 * 1): r probing vectors of length K = C_in*H*W, Z [K, r] with row (n, y, x) =
 * (n*H + y)*W + x, drawn from (probe, seed) and never handed over; entry (k, j) is
 * word k*r + j of the generator xconv_probe_matrix documents, rounded to desc->dtype.
 *
 *   forward   Xbar[b,j] = sum_{n,y,x} Z[(n,y,x),j] X[b,n,y,x]                 (Alg. 1 fwd step 3)
 *   backward  L[j,m,oy,ox] = (1/r) sum_b Xbar[b,j] dY[b,m,oy,ox], rounded once to desc->dtype
 *                                                                              (Alg. 1 bwd step 3)
 *             dW[m,n,ky,kx] = sum_j sum_{oy,ox} L[j,m,oy,ox] Z[(n, oy*sh+ky-ph, ox*sw+kx-pw), j]
 *                                                                              (Alg. 1 bwd step 4)
 *
 * The stored state is Xbar, B*r floats: C_in*H*W/r times smaller than X in fp32.  Z is
 * regenerated in scratch in each pass (r*K values of desc->dtype).  keep_q15 != 0
 * selects block-sparse probing vectors (Eq. (7)): block (n, j), the H*W entries of
 * vector j on channel n, is zero unless the top 15 bits of word n*r + j of the mask
 * stream (see xconv_probe_matrix) are below keep_q15, and the estimate of input channel
 * n is scaled by 1/nnz(Z_n), the number of kept blocks of channel n, instead of 1/r
 * (Eq. (8)); a channel without any gives zeros.  Supported: both layouts (Z is indexed
 * by (n, y, x) as above whatever the order X keeps its values in), Rademacher or
 * Gaussian probes from the seed (XCONV_USER_Z is XCONV_EUNSUPPORTED), C_in*H*W and
 * C_out*H'*W' up to 2^28, B up to 65536.  All
 * other conventions as above; X_dev and dY_dev 16-byte aligned, ws_dev required. */
size_t xconv_pixel_xbar_bytes(const xconv_desc *desc);
size_t xconv_pixel_workspace_bytes(const xconv_desc *desc, int op);    /* XCONV_OP_PROBE or XCONV_OP_ESTIMATE */
xconv_status xconv_pixel_probe_fwd(const xconv_desc *desc, const void *X_dev, float *Xbar_dev,
                                   void *ws_dev, size_t ws_bytes, void *stream);
xconv_status xconv_pixel_dw_estimate(const xconv_desc *desc, const void *dY_dev, const float *Xbar_dev,
                                     float *dW_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* Independent probing (Sec. 3: trace estimation applied to every input/output channel
 * pair on its own, the alternative that the multi-channel case of Eq. (6) is set
 * against; the experiments' "Indep." curves): input channel n has r probing vectors of
 * its own, Z_n [H*W, r] = the rows of channel n of the Z above (same generator words),
 *
 *   forward   Xbar[b,n,j] = sum_{y,x} Z_n[(y,x),j] X[b,n,y,x]
 *   backward  L_n[j,m,oy,ox] = (1/r) sum_b Xbar[b,n,j] dY[b,m,oy,ox], rounded once to desc->dtype
 *             dW[m,n,ky,kx] = sum_j sum_{oy,ox} L_n[j,m,oy,ox] Z_n[(oy*sh+ky-ph, ox*sw+kx-pw), j]
 *
 * so no term mixes two input channels (no crosstalk), at C_in times the stored state:
 * Xbar is [B, C_in, r] floats, H*W/r times smaller than X in fp32.  The backward pass
 * runs in groups of input channels (16 or more), each as the multi-channel estimator with
 * block-diagonal probing vectors over the group; limits as above and C_in*r <= 65536,
 * keep_q15 == 0 (else XCONV_EUNSUPPORTED). */
size_t xconv_pixel_indep_xbar_bytes(const xconv_desc *desc);
size_t xconv_pixel_indep_workspace_bytes(const xconv_desc *desc, int op);
xconv_status xconv_pixel_indep_probe_fwd(const xconv_desc *desc, const void *X_dev, float *Xbar_dev,
                                         void *ws_dev, size_t ws_bytes, void *stream);
xconv_status xconv_pixel_indep_dw_estimate(const xconv_desc *desc, const void *dY_dev, const float *Xbar_dev,
                                           float *dW_dev, void *ws_dev, size_t ws_bytes, void *stream);

/* ---- ReLU that keeps signs only --------------------------------------------------
 * A ReLU in front of a convolution used to find its output stored by that convolution;
 * with the entry points above, the convolution keeps the probe output instead, so the ReLU
 * keeps one bit per element (Sec. 5, "Overall effective memory savings").
 *
 *   forward   Y[i] = max(X[i], 0);  bit i%64 of the 64-bit word i/64 of mask = (X[i] > 0)
 *   backward  dX[i] = that bit ? dY[i] : 0
 *
 * n elements of `dtype` (an xconv_dtype) in any shape, taken in memory order.  mask_dev:
 * xconv_relu_mask_bytes(n) bytes, 8-byte aligned, owned by the caller; X_dev, Y_dev,
 * dY_dev, dX_dev 16-byte aligned.  Y_dev may equal X_dev and dX_dev may equal dY_dev
 * (in place).  A NaN stays a NaN in Y and counts as not positive.  n == 0 is a no-op;
 * XCONV_EINVAL for a bad dtype, n < 0, a null or misaligned pointer; n above 2^40 is
 * XCONV_EUNSUPPORTED. */
size_t xconv_relu_mask_bytes(long long n);
xconv_status xconv_relu_fwd(int dtype, const void *X_dev, void *Y_dev, void *mask_dev, long long n, void *stream);
xconv_status xconv_relu_bwd(int dtype, const void *dY_dev, const void *mask_dev, void *dX_dev, long long n, void *stream);

/* Reference measurement for the roofline figures (not part of the method): enqueues a loop of `iters` x 4
 * independent 32x32 matrix instructions per wave (32x32x16 for the 16-bit types, 32x32x2 for fp32) on every
 * SIMD of the device, with operands of random bits, and stores the number of floating-point operations of
 * the launch in *flops (host; may be null).  Timed by the caller (xconv_prof_* or its own events), flops /
 * time is the matrix-core rate the chip sustains at the clock it holds.  out_dev: device scratch of at least
 * XCONV_DIAG_OUT_BYTES, 4-byte aligned, caller-owned (one float per wave is written; the values mean
 * nothing).  XCONV_EINVAL for a bad dtype, iters outside 1 .. 2^24 or a null or misaligned pointer,
 * XCONV_EWORKSPACE for too small a buffer. */
#define XCONV_DIAG_OUT_BYTES 8192
xconv_status xconv_diag_mfma_rate(int dtype, int iters, float *out_dev, size_t out_bytes, double *flops, void *stream);

/* Per-kernel timing with HIP events recorded on the launch stream.  While
 * enabled, every kernel the library enqueues is bracketed by two events.
 * xconv_prof_collect synchronises those events, writes up to `max` records
 * (kernel id, milliseconds) in launch order, returns how many it wrote and
 * clears the list.  Kernel ids: see xconv_prof_kernel_name.  Not thread safe;
 * meant for the benchmark, off by default. */
void xconv_prof_enable(int on);
int xconv_prof_collect(int32_t *kernel_ids, float *ms, int max);
const char *xconv_prof_kernel_name(int kernel_id);

const char *xconv_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* XCONV_H */
