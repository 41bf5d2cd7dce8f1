/*
 * mi355conv -- fp32 NCHW 2-D convolution layer (forward, backward-data,
 * backward-weight) for AMD Instinct MI355X (gfx950).  Plain C ABI.
 *
 * The paper's analysis (Sec. 4.1) singles out the convolution layers as where
 * convnet training time goes, and its Sec. 4.4 proposes that a framework call a
 * single hardware-specific `conv` entry point loaded at run time.  This header is
 * that entry point for one piece of hardware.  The algorithms behind it are the
 * two the paper recommends in Sec. 4.2: "implicitgemm" (the lowered matrix exists
 * only on chip) and "winograd" (minimal filtering, for 3x3 stride-1 filters).
 *
 * Operation (cross-correlation, zero padding; the element-wise reading of the
 * Sec. 4.2 "im2col" statement that one image convolved with the weights is one
 * matrix product W[K x CRS] * lowered(x)[CRS x PQ]):
 *
 *   P = floor((H + 2*pad_h - R) / stride_h) + 1,  Q likewise
 *   y [n,k,p,q] = bias[k] + sum_{c,r,s} x[n,c,p*stride_h-pad_h+r,q*stride_w-pad_w+s] * w[k,c,r,s]
 *   dx[n,c,h,v] = sum of dy[n,k,p,q] * w[k,c,r,s] over every (k,p,q,r,s) whose tap
 *                 lands on (h,v)                              (transpose of the above)
 *   dw[k,c,r,s] = scale * sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*stride_h-pad_h+r,q*stride_w-pad_w+s]
 *   db[k]       = scale * sum_{n,p,q} dy[n,k,p,q]
 *
 * Layout: every tensor is dense, contiguous fp32 in DEVICE memory:
 *   x, dx : [N][C][H][W]     w, dw : [K][C][R][S]     y, dy : [N][K][P][Q]
 *   bias, dbias : [K]
 * Pointers need 4-byte alignment (16-byte alignment of the tensors' bases lets
 * the library use wider accesses).  Inputs and outputs must not alias.  Each
 * tensor must have fewer than 2^31 elements.  Dilation 1, one group.
 *
 * Ownership: the caller owns every buffer, including the workspace.  The library
 * allocates no device memory and keeps no state between calls; it only enqueues
 * kernels on the caller's stream and returns without synchronising.  Concurrent
 * calls from several threads on different streams are safe if their buffers (and
 * workspaces) differ (one-time kernel attribute set-up is guarded).
 *
 * Errors: every function returns CONV2D_OK (0) or a negative code.  On an argument,
 * algorithm or workspace error nothing has been enqueued; CONV2D_ERR_LAUNCH (HIP refused a
 * launch) may follow earlier launches of the same call.  No exceptions cross this boundary.
 */
#ifndef MI355CONV_H
#define MI355CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t N, C, H, W;          /* input batch, channels, height, width          */
    int32_t K, R, S;             /* filters, filter height, filter width          */
    int32_t stride_h, stride_w;  /* >= 1                                          */
    int32_t pad_h, pad_w;        /* >= 0, zeros, applied on both sides            */
} conv2d_desc;

typedef enum {
    CONV2D_ALGO_AUTO = 0,        /* library picks (see conv2d_pick_algo)          */
    CONV2D_ALGO_IGEMM = 1,       /* implicit GEMM on fp32 MFMA, any geometry      */
    CONV2D_ALGO_WINOGRAD = 2,    /* F(2x2,3x3), stride 1: 3x3 filters, and filters up
                                  * to 6x6 as sums of 3x3 sub-filters of shifted
                                  * inputs; stride 2..4 (both directions equal) with a
                                  * filter spanning exactly 3 x 3 strides (11x11/4,
                                  * 5x5/2, ...): as the stride-1 3x3 layer over the
                                  * space-to-depth rearrangement of the input, which
                                  * the workspace then holds a copy of              */
    CONV2D_ALGO_WINOGRAD4 = 3,   /* F(4x4,3x3), stride-1 filters of 3x3 up to 6x6 (the
                                  * larger ones as sums of 3x3 sub-filters): filter,
                                  * input and output transforms as separate kernels
                                  * around 36 batched GEMMs; the workspace holds the
                                  * transformed input and the products (2.25 x the
                                  * layer's input and output each).  All three passes */
    CONV2D_ALGO_FFT = 4          /* product of spectra (Sec. 4.2 "fft": the choice for
                                  * large filters): stride 1, any filter size, padded
                                  * input at most 32 x 32 (one tile per image);
                                  * 544 complex GEMMs between transform kernels, the
                                  * workspace holds the spectra of filters, images and
                                  * products.  All three passes                        */
} conv2d_algo;

typedef enum {
    CONV2D_FWD = 0,
    CONV2D_BWD_DATA = 1,
    CONV2D_BWD_WEIGHT = 2
} conv2d_op;

enum {
    CONV2D_OK = 0,
    CONV2D_ERR_NULL = -1,        /* null descriptor or required pointer           */
    CONV2D_ERR_GEOMETRY = -2,    /* non-positive size, stride < 1, pad < 0,
                                    H+2*pad_h < R (or W), tensor >= 2^31 elements */
    CONV2D_ERR_ALGO = -3,        /* algorithm cannot do this geometry / unknown   */
    CONV2D_ERR_WORKSPACE = -4,   /* workspace null or smaller than required       */
    CONV2D_ERR_LAUNCH = -5,      /* HIP reported a launch error                   */
    CONV2D_ERR_STATIC_LIMIT = -6 /* conv2d_fwd_static: the layer needs more workspace
                                    than CONV2D_STATIC_SCRATCH_BYTES              */
};

/* Size of the library-owned scratch area conv2d_fwd_static works in (per GPU). */
#define CONV2D_STATIC_SCRATCH_BYTES (64u << 20)

/* Output height P and width Q (Sec. 4.2 lowering: one column per output pixel).
 * Host-only, touches no device. */
int conv2d_output_dims(const conv2d_desc *d, int32_t *P, int32_t *Q);

/* The algorithm AUTO resolves to for this op and geometry.  Returns a
 * conv2d_algo value, or a negative error code. */
int conv2d_pick_algo(const conv2d_desc *d, conv2d_op op);

/* Bytes of device workspace `op` needs with `algo` (AUTO = whatever AUTO picks).
 * Returns 0 for an invalid descriptor or unsupported algo.  Host-only.
 * The workspace holds the re-laid-out filter matrix and gather table of the
 * implicit GEMM, transformed filters/tiles for Winograd, and the partial sums of
 * the weight-gradient reduction over the batch. */
size_t conv2d_workspace_bytes(const conv2d_desc *d, conv2d_op op, conv2d_algo algo);

/* Forward (Torch's updateOutput; Sec. 4.1/4.2).  Overwrites all of y.
 * bias may be NULL (no bias); it is added in the kernel's epilogue, before the
 * only store of y (Sec. 4.2 "Neon": transforms and epilogue belong in the product's kernel).
 * ws: device pointer to >= conv2d_workspace_bytes(d, CONV2D_FWD, algo) bytes,
 * 256-byte aligned (checked: CONV2D_ERR_WORKSPACE otherwise); contents are scratch.  hip_stream: a hipStream_t (NULL = the
 * default stream). */
int conv2d_fwd(const conv2d_desc *d, const float *x, const float *w, const float *bias,
               float *y, void *ws, size_t ws_bytes, conv2d_algo algo, void *hip_stream);

/* conv2d_fwd for callers that cannot allocate or own device memory beyond their
 * tensors: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same result as conv2d_fwd(d, x, w, bias, y, ws, ..., algo, hip_stream)
 * (same kernels, same summation order), but the workspace is a library-owned static
 * device array of CONV2D_STATIC_SCRATCH_BYTES (64 MiB) that every GPU the library runs
 * on holds from the load of its code until the process ends; the call itself allocates
 * and frees nothing.  A layer with conv2d_workspace_bytes(d, CONV2D_FWD, algo) above that
 * size is refused with CONV2D_ERR_STATIC_LIMIT and nothing is enqueued (every layer of the
 * AlexNet, VGG-16 and inception configurations fits; filter banks beyond about 512 x 512
 * of 3x3 do not).  With CONV2D_ALGO_AUTO, a layer for which AUTO's choice is the unfused
 * F(4x4,3x3) path or the frequency-domain path (whose workspaces hold whole transformed
 * tensors) and does not fit is computed by the fused F(2x2,3x3) kernels instead; the result then differs from
 * conv2d_fwd's by rounding only.  All calls on one GPU share that one area, which keeps the previous
 * call's contents (nothing in it needs to start at zero): calls that overlap on one GPU,
 * i.e. on different streams without ordering between them, race.  Calls on one stream
 * are ordered and safe.  The current device must be the one the tensors live on. */
int conv2d_fwd_static(const conv2d_desc *d, const float *x, const float *w, const float *bias,
                      float *y, conv2d_algo algo, void *hip_stream);

/* Forward followed by the rectifier of the layer after it, in the same epilogue:
 * y = max(0, conv(x, w) + bias), stored once.  (Sec. 4.1 lists the RELU layers as the
 * small remainder of the per-layer time next to the convolutions; fusing them is the
 * fusion item of Sec. 4.2 "Neon" taken one step further: the separate
 * layer would read and write y once more.)  Same arguments, workspace, algorithm choice
 * and errors as conv2d_fwd; the sum is the one conv2d_fwd forms, max(., 0) is applied to
 * it in fp32 (a NaN sum gives 0). */
int conv2d_fwd_relu(const conv2d_desc *d, const float *x, const float *w, const float *bias,
                    float *y, void *ws, size_t ws_bytes, conv2d_algo algo, void *hip_stream);

/* The same followed by 2x2 / stride-2 max pooling (the pooling layers Sec. 4.1 lists next
 * to RELU; in the VGG stack one follows the last convolution of every block):
 * y_pooled[n,k,i,j] = max over a, b in {0,1} of max(0, conv(x,w)[n,k,2i+a,2j+b] + bias[k]),
 * a device tensor N x K x P/2 x Q/2, overwritten; the unpooled y is never stored.  Only for
 * layers the Winograd path takes (its 2x2 output blocks are the pooling windows) with even
 * P and Q: otherwise CONV2D_ERR_ALGO.  Workspace:
 * conv2d_workspace_bytes(d, CONV2D_FWD, CONV2D_ALGO_WINOGRAD).  Other arguments and errors
 * as conv2d_fwd. */
int conv2d_fwd_relu_pool2(const conv2d_desc *d, const float *x, const float *w, const float *bias,
                          float *y_pooled, void *ws, size_t ws_bytes, void *hip_stream);

/* Several 1x1, stride-1, unpadded convolutions of the SAME input in one pass over it
 * (Sec. 4.2 singles out GoogLeNet's 1x1 layers; its inception module applies three of
 * them to one input, and they are bound by reading that input).  Group g has K[g]
 * filters w[g] (K[g] x C, device), an optional bias[g] (K[g], device; bias or bias[g]
 * may be NULL) and its own output y[g] (N x K[g] x H x W, device), overwritten.
 * d describes the stacked layer: R = S = 1, stride 1, pad 0 and d->K = sum of K[g];
 * 1 <= ngroup <= 4.  K, w, bias and y are HOST arrays (of counts / device pointers)
 * read before the call returns.  Workspace: conv2d_workspace_bytes(d, CONV2D_FWD,
 * CONV2D_ALGO_IGEMM).  Every output element equals what conv2d_fwd computes for its
 * group alone (same summation order).  Errors: CONV2D_ERR_ALGO if d is not a 1x1
 * stride-1 unpadded layer, CONV2D_ERR_GEOMETRY for a bad group list. */
int conv2d_fwd_1x1_group(const conv2d_desc *d, const float *x, int32_t ngroup, const int32_t *K,
                         const float *const *w, const float *const *bias, float *const *y,
                         void *ws, size_t ws_bytes, void *hip_stream);

/* Backward w.r.t. the input (Torch's updateGradInput; the benchmarks of Sec. 3.4
 * time forward plus backward).  Overwrites all of dx, including pixels no
 * output window covers (they get 0). */
int conv2d_bwd_data(const conv2d_desc *d, const float *dy, const float *w, float *dx,
                    void *ws, size_t ws_bytes, conv2d_algo algo, void *hip_stream);

/* Backward w.r.t. the weights (Torch's accGradParameters), including the
 * reduction over the batch (Sec. 4.2 "im2col": per-image products are small;
 * lowering many images into one product is what makes them efficient).
 * accumulate == 0: dw = scale*grad, dbias = scale*grad_b.
 * accumulate != 0: dw += scale*grad, dbias += scale*grad_b.
 * dbias may be NULL (bias gradient not computed).  The result is deterministic:
 * partial sums are combined in a fixed order, never with atomics. */
int conv2d_bwd_weight(const conv2d_desc *d, const float *x, const float *dy,
                      float *dw, float *dbias, float scale, int accumulate,
                      void *ws, size_t ws_bytes, conv2d_algo algo, void *hip_stream);

/* Per-element operation of the experiment of Sec. 3.3 (bandwidth of per-element
 * kernels against the number of floats per launch; the paper does not name the
 * operation): y[i] = fl(fl(a * x[i]) + b) for i < n, the two operations rounded to
 * fp32 separately (no fused multiply-add).  x and y are device pointers to n floats
 * (4-byte aligned; 16-byte alignment of both selects the vector path); y may equal
 * x.  n == 0 is a no-op; n < 0 returns CONV2D_ERR_GEOMETRY.  Enqueues on hip_stream
 * and returns. */
int apply_mul_add(const float *x, float *y, int64_t n, float a, float b, void *hip_stream);

/* ---- measurement helpers (not part of the convolution path) ------------------------
 * Opt-in timing of the library's main kernels, for roofline figures: between
 * conv2d_profile_begin(capacity) and conv2d_profile_end() every launch of a main kernel
 * (the GEMM / Winograd / streaming kernels and the transform kernels of the unfused
 * Winograd and frequency-domain paths; not the small preparation and reduction kernels) is bracketed by two HIP
 * events on its stream, up to `capacity` launches.  begin creates the host-side event
 * objects (kept for reuse until the library is unloaded) and returns CONV2D_OK or an
 * error; end returns the number of launches recorded.  After the caller has synchronised
 * the streams, conv2d_profile_record(i, ...) returns launch i's kernel id, the algorithmic
 * flops and minimal HBM bytes the launcher stated for it, and its duration in ms.
 * Process-wide host state, not thread-safe: one measuring thread at a time. */
int conv2d_profile_begin(int capacity);
int conv2d_profile_end(void);
int conv2d_profile_record(int i, int32_t *kernel, double *flops, double *bytes, float *ms);
const char *conv2d_profile_kernel_name(int kernel);

/* What the chip sustains, for calibrating roofline fractions (Sec. 3.3 measures the
 * bandwidth of trivial kernels in the same spirit).  conv2d_probe_mfma_f32 enqueues a
 * kernel that does nothing but v_mfma_f32_32x32x2_f32 (512 workgroups x 4 waves x iters x
 * 32 instructions) and stores the flops it executes in *flops (host); sink: 4 bytes of
 * device memory, never written.  conv2d_probe_copy enqueues a 16-byte-vector copy of n
 * floats from src to dst (device, 16-byte aligned, n % 4 == 0), or a fill of dst when src
 * is NULL.  The caller times them with events. */
int conv2d_probe_mfma_f32(float *sink, int32_t iters, double *flops, void *hip_stream);
int conv2d_probe_copy(const float *src, float *dst, int64_t n, void *hip_stream);

/* Static, never-NULL description of a status code. */
const char *conv2d_status_string(int status);

/* Library version string (static). */
const char *conv2d_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MI355CONV_H */
