/*
 * conv1d.h - C ABI of the MI355X (gfx950) 1D dilated convolution layer.
 *
 * The layer is the one defined in Section 2 (Eq. 2) of "Efficient and Generic
 * 1D Dilated Convolution Layer for Deep Learning": stride 1, one group, no bias
 * (Section 3, first paragraph: bias is left to the framework), zero padding at
 * the edges.  Eq. 2 is read the way Algorithms 1 and 2 index it (input column
 * q + s*d contributes to output column q through tap s, i.e. cross-correlation).
 *
 * Geometry shared by every entry point
 *   N        batch size
 *   C        input channels
 *   K        filters (output channels)
 *   W        input width, NOT including padding
 *   S        filter width (taps)
 *   dilation d >= 1, distance between taps along the width
 *   padding  P >= 0 zeros assumed on each side of the width axis; they are
 *            implicit and never materialised
 *   Q        output width = W + 2*P - (S-1)*d   (conv1d_out_width)
 *
 * Tensor layouts (all row-major, contiguous, innermost index last)
 *   x  [N][C][W]   layer input                 dtype
 *   w  [K][C][S]   filter weights              dtype
 *   y  [N][K][Q]   layer output                float
 *   dy [N][K][Q]   gradient w.r.t. the output  dtype
 *   dx [N][C][W]   gradient w.r.t. the input   float
 *   dw [K][C][S]   gradient w.r.t. the weights float
 * `dtype` is CONV1D_FP32 (IEEE binary32) or CONV1D_BF16 (bfloat16, 2 bytes);
 * products are accumulated in FP32 and outputs are FP32, never rounded back to
 * bfloat16, except where a caller of the _ex entry points asks for bfloat16
 * storage.  C, K and W may be odd for either dtype.
 *
 * Pointers, ownership, execution
 *   Every tensor pointer is a DEVICE pointer owned by the caller and must stay
 *   valid until the work queued on `stream` has finished.  `stream` is a
 *   hipStream_t passed as void* (NULL = the default stream).  Calls only
 *   enqueue kernels: they do not allocate, free or synchronise, and they
 *   OVERWRITE their output (beta = 0 in the notation of Eq. 3).  Inputs and
 *   outputs must not alias.  float tensors must be 4-byte aligned, bfloat16
 *   tensors 2-byte aligned; 16-byte alignment (any torch allocation) enables
 *   the fast kernels.  A bfloat16 weight tensor is read in 4-byte words: if
 *   it holds an odd number of elements, the 2 bytes behind its last element
 *   are read too (and ignored), so its allocation must extend to the next
 *   4-byte boundary, as any device allocation does.  Calls are thread-safe
 *   and re-entrant across streams as long as their outputs and workspaces
 *   are distinct.
 *
 * Non-finite inputs
 *   Inputs are expected to be finite.  The kernels pad taps and channels up to
 *   the sizes of their matrix tiles with zero weights (or zero-filled columns)
 *   that multiply real input values, and 0 * Inf = NaN.  An Inf or NaN input
 *   element can therefore (a) turn an output that the definition makes +-Inf
 *   into NaN, and (b) turn outputs into NaN that the definition says do not
 *   depend on it, but only these:
 *     conv1d_fwd, conv1d_bwd_data: outputs of the SAME sample within 64*d
 *       columns of the columns the element contributes to;
 *     conv1d_bwd_weight: dw[.][c][.] for a non-finite x[n][c][i], and
 *       dw[k][.][.] for a non-finite dy[n][k][q].
 *   Every other output is computed as if the input were finite, and every
 *   output that the definition makes non-finite is non-finite.
 *
 * Errors
 *   Every int-returning entry point returns CONV1D_OK (0) or a negative
 *   conv1d_status_t; nothing is thrown and errno is untouched.  Argument errors
 *   (CONV1D_EINVAL, CONV1D_EUNSUPPORTED, CONV1D_EWORKSPACE) are detected before
 *   anything is launched.  CONV1D_EHIP reports that the HIP runtime refused a
 *   launch; a pass that consists of several launches (FP32 layers with more
 *   than 16 channels whose weights do not fit in LDS; the second stage of
 *   conv1d_bwd_weight) may have enqueued its earlier kernels by then, so the
 *   output is unspecified after CONV1D_EHIP.
 */
#ifndef CONV1D_MI355X_H
#define CONV1D_MI355X_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { CONV1D_FP32 = 0, CONV1D_BF16 = 1 } conv1d_dtype_t;

typedef enum {
    CONV1D_OK = 0,
    CONV1D_EINVAL = -1,       /* null pointer, non-positive size, d < 1, P < 0, Q <= 0, bad dtype, misaligned pointer */
    CONV1D_EUNSUPPORTED = -2, /* a forced kernel variant cannot run this geometry, or sizes overflow 32-bit tile indices */
    CONV1D_EWORKSPACE = -3,   /* workspace missing or smaller than conv1d_bwd_weight_workspace_bytes() */
    CONV1D_EHIP = -4,         /* the HIP runtime refused a launch */
    CONV1D_ESCRATCH = -5      /* conv1d_bwd_weight_noalloc: the geometry needs more than CONV1D_NOALLOC_SCRATCH_BYTES */
} conv1d_status_t;

/* Kernel families.  AUTO lets the library choose from the geometry; the others
 * force one family (experiments and tests) and fail with CONV1D_EUNSUPPORTED
 * when that family cannot run the geometry. */
typedef enum {
    CONV1D_VARIANT_AUTO = 0,
    CONV1D_VARIANT_GENERIC = 1, /* plain FMA, any geometry */
    CONV1D_VARIANT_SMALLC = 2,  /* MFMA, C and K <= 16, taps held in registers */
    CONV1D_VARIANT_IGEMM = 3    /* MFMA, any C and K in blocks of 16 channels x 16 filters (implicit GEMM over channel blocks and taps) */
} conv1d_variant_t;

typedef enum { CONV1D_PASS_FWD = 0, CONV1D_PASS_BWD_DATA = 1, CONV1D_PASS_BWD_WEIGHT = 2 } conv1d_pass_t;

/* Output width Q = W + 2*padding - (S-1)*dilation (Section 2; Fig. 1 has
 * W=17, S=3, d=3, P=3 -> Q=17).  Returns a value <= 0 when the geometry is
 * invalid (any non-positive size, dilation < 1, padding < 0, or no output column). */
int conv1d_out_width(int W, int S, int dilation, int padding);

/* Forward pass (Eq. 2; Algorithms 1 and 2):
 *   y[n][k][q] = sum_{c<C} sum_{s<S} x[n][c][q + s*d - P] * w[k][c][s],  x = 0 outside [0,W).
 * x: device, dtype, N*C*W elements (read).  w: device, dtype, K*C*S elements (read).
 * y: device, float, N*K*Q elements (overwritten). */
int conv1d_fwd(const void* x, const void* w, float* y,
               int N, int C, int K, int W, int S, int dilation, int padding,
               int dtype, void* stream);

/* Forward pass with a fused epilogue:
 *   z = conv1d_fwd(x, w)[n][k][q] + bias[k]      bias: device, float, K elements, or NULL for none
 *                                                 (Section 3 leaves the bias to the framework: this is where it goes)
 *   z = max(z, 0)                                 with CONV1D_EPI_RELU (Section 4.4: the ReLU that follows the layer)
 *   y = z as float, or as bfloat16 (nearest, ties to even) with CONV1D_EPI_OUT_BF16, which needs dtype ==
 *       CONV1D_BF16 (Section 4.4: activations stay in BF16, no conversion pass).
 * y: device, N*K*Q elements of float (4-byte aligned) or bfloat16 (2-byte aligned), overwritten.
 * flags = 0 and bias = NULL is conv1d_fwd.  Unknown flag bits: CONV1D_EINVAL. */
#define CONV1D_EPI_RELU 1
#define CONV1D_EPI_OUT_BF16 2
int conv1d_fwd_ex(const void* x, const void* w, const float* bias, void* y,
                  int N, int C, int K, int W, int S, int dilation, int padding,
                  int dtype, int flags, void* stream);

/* Backward-data pass (Section 3.2, Algorithm 3: the adjoint of the forward map in x):
 *   dx[n][c][i] = sum_{k<K} sum_{s<S} w[k][c][s] * dy[n][k][i + P - s*d],  dy = 0 outside [0,Q).
 * dy: device, dtype, N*K*Q elements (read).  w: device, dtype, K*C*S (read).
 * dx: device, float, N*C*W elements (overwritten). */
int conv1d_bwd_data(const void* dy, const void* w, float* dx,
                    int N, int C, int K, int W, int S, int dilation, int padding,
                    int dtype, void* stream);

/* Backward-data pass whose result is stored as bfloat16 with CONV1D_EPI_OUT_BF16 (Section 4.4: in BF16 training
 * the gradients that flow to the previous layer stay in BF16); needs dtype == CONV1D_BF16.  dx: device, N*C*W
 * elements of float or bfloat16, overwritten.  No other flag is valid here; flags = 0 is conv1d_bwd_data. */
int conv1d_bwd_data_ex(const void* dy, const void* w, void* dx,
                       int N, int C, int K, int W, int S, int dilation, int padding,
                       int dtype, int flags, void* stream);

/* Bytes of device scratch conv1d_bwd_weight needs for this geometry (partial
 * sums of the first reduction stage).  Returns 0 for an invalid geometry.
 * The size covers every kernel variant, so a forced variant never needs more. */
size_t conv1d_bwd_weight_workspace_bytes(int N, int C, int K, int W, int S, int dilation, int padding,
                                         int dtype);

/* Backward-weight pass (Section 3.3, Algorithm 4: the adjoint of the forward map in w):
 *   dw[k][c][s] = sum_{n<N} sum_{q<Q} x[n][c][q + s*d - P] * dy[n][k][q].
 * The sum over (n, q) is split over workgroups; their partial sums go to
 * `workspace` and a second kernel adds them in a fixed order, so results are
 * bit-identical from run to run (no floating-point atomics).
 * x: device, dtype, N*C*W (read).  dy: device, dtype, N*K*Q (read).
 * dw: device, float, K*C*S (overwritten).
 * workspace: device, 256-byte aligned, at least workspace_bytes >=
 * conv1d_bwd_weight_workspace_bytes(...); contents on entry are ignored and
 * on exit unspecified.  Two calls in flight must not share a workspace.
 * Sizes: one partial tile of the workgroup's share of dw per workgroup, e.g.
 * 13.4 MB for N=16, C=K=15, W=60000, S=51, d=8; 27.3 MB for N=8, C=K=64,
 * W=20000, S=51; 37.7 MB for N=32, C=K=256, W=8192, S=9, d=4. */
int conv1d_bwd_weight(const void* x, const void* dy, float* dw,
                      void* workspace, size_t workspace_bytes,
                      int N, int C, int K, int W, int S, int dilation, int padding,
                      int dtype, void* stream);

/* Both backward passes of a layer in one call, as a framework's backward step asks for them (Section 4.3 times
 * forward() and backward() of the layer; backward is Sections 3.2 and 3.3 together):
 *   dx = conv1d_bwd_data(dy, w)   and   dw = conv1d_bwd_weight(x, dy),   results bit-identical to those calls.
 * The kernels of the two passes are queued back to back; for bfloat16 layers with C, K <= 16 and d = 8 the
 * second stage of the weight gradient is not a launch of its own: the backward-data kernel adds up the partial
 * sums while it waits for its first inputs.  Workspace as for conv1d_bwd_weight
 * (conv1d_bwd_workspace_bytes returns the same size).  dx and dw must not alias each other or an input. */
size_t conv1d_bwd_workspace_bytes(int N, int C, int K, int W, int S, int dilation, int padding, int dtype);
int conv1d_bwd(const void* x, const void* dy, const void* w, float* dx, float* dw,
               void* workspace, size_t workspace_bytes,
               int N, int C, int K, int W, int S, int dilation, int padding,
               int dtype, void* stream);

/* conv1d_bwd_weight for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same result, bit for bit, as conv1d_bwd_weight on the same
 * inputs.  The partial sums go to a buffer of CONV1D_NOALLOC_SCRATCH_BYTES that
 * is part of the library's device image (one copy per GPU, held until the
 * process ends); the call allocates and frees nothing (its first call on a GPU
 * looks the buffer's address up, with that GPU current; `stream` must belong
 * to the current GPU).  Returns CONV1D_ESCRATCH, having launched nothing, when
 * conv1d_bwd_weight_workspace_bytes(...) exceeds the buffer.  All calls on one
 * GPU share the buffer: two calls that overlap in time on the same GPU (on
 * different streams or from different threads) race and give wrong results;
 * calls queued on one stream are safe.  The buffer keeps the last call's
 * partial sums; nothing in it has to be cleared, every kernel writes the
 * partial sums it later reads.
 * x, dy, dw and the geometry as for conv1d_bwd_weight. */
#define CONV1D_NOALLOC_SCRATCH_BYTES (64u << 20)
int conv1d_bwd_weight_noalloc(const void* x, const void* dy, float* dw,
                              int N, int C, int K, int W, int S, int dilation, int padding,
                              int dtype, void* stream);

/* Force a kernel family for all later calls of this process (CONV1D_VARIANT_*).
 * Returns CONV1D_EINVAL for an unknown value.  The setting is one process-wide
 * atomic: changing it while other threads are inside the library changes the
 * family of their later launches too.  For experiments and tests only. */
int conv1d_set_variant(int variant);

/* Name of the kernel the current variant setting selects for a pass
 * (conv1d_pass_t) and geometry, e.g. "smallc_mfma_bf16"; "invalid" for a bad
 * geometry, "unsupported" when a forced variant cannot run it.  The string is
 * static storage. */
const char* conv1d_kernel_name(int pass, int N, int C, int K, int W, int S, int dilation, int padding,
                               int dtype);

/* Human-readable text for a conv1d_status_t (static storage). */
const char* conv1d_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CONV1D_MI355X_H */
