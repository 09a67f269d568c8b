/*
 * cct.h - C ABI of libcct.so: the lowering-based convolutional layer of
 * "Caffe con Troll" (arXiv 1504.04343) as hand-written HIP for gfx950 (MI355X).
 *
 * The layer is computed in the paper's three phases (Sec. 2.1): LOWER the batch of
 * input tensors into one matrix D^ (all images of a chunk side by side, Sec. 2.2),
 * MULTIPLY it with the lowered kernels K^ on the matrix cores, LIFT the product R^
 * back to a tensor and add the bias.  Three lowering layouts exist (Sec. 2.1,
 * Type 1 "expensive lowering", Type 2 "balanced", Type 3 "expensive lifting") and
 * an automatic optimizer picks one from the ratio of input to output channels
 * (Sec. 1, Appendix A).  The paper states the forward pass only; the two backward
 * passes are the adjoints of the same three phases run in reverse order.
 *
 * Problem statement (Sec. 2): a batch of b data tensors with d channels and o kernels
 * of size k x k x d.  Here: x is N x C x H x W (NCHW, contiguous fp32), w is
 * O x (C/groups) x K x K (contiguous fp32), y is N x O x Hout x Wout with
 * Hout = floor((H + 2*pad - K)/stride) + 1 (same for W).  Semantics (stride, zero
 * padding on all four sides, channel groups, bias, no kernel flip) are Caffe's, which
 * the paper's system reproduces layer by layer (Sec. 1, Sec. 3.2):
 *
 *   y[n,o,r,c] = bias[o] + sum_{ci,i,j} x[n, (o/Og)*Cg+ci, r*stride+i-pad, c*stride+j-pad] * w[o,ci,i,j]
 *
 * General rules for every entry point
 *  - All tensor pointers are DEVICE pointers (HIP global memory) unless stated
 *    otherwise; descriptors and scalar outputs are HOST pointers.
 *  - The caller owns every buffer including the workspace.  The library never
 *    allocates or frees device memory, never synchronises, and enqueues work only on
 *    the given HIP stream (`hip_stream` is a hipStream_t passed as void*; NULL = the
 *    default stream).  Calls return as soon as the work is enqueued.
 *  - Outputs are overwritten (beta = 0), never accumulated.  Inputs, outputs and
 *    workspace must not overlap.
 *  - Return value: CCT_OK (0) or a negative CCT_E* code.  On error nothing has been
 *    enqueued for that call (except CCT_EHIP, which reports a failed launch).
 *  - The workspace must be 256-byte aligned.  Its size decides how many images are
 *    lowered and multiplied together (Sec. 2.2 recommends the largest batch that memory
 *    allows): the library processes the batch in chunks of the largest number of
 *    images whose buffers fit the workspace it was given.
 */
#ifndef CCT_H_
#define CCT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Lowering layout, Sec. 2.1.  AUTO lets cct_pick_lowering decide (it may also pick FUSED). */
typedef enum {
  CCT_LOWER_AUTO = 0,
  CCT_LOWER_TYPE1 = 1, /* D^ rows = output positions, cols = (ci,i,j); trivial lifting      */
  CCT_LOWER_TYPE2 = 2, /* D^ rows = (input row, output col), cols = (ci,j); lift sums K rows */
  CCT_LOWER_TYPE3 = 3, /* D^ rows = input positions, cols = ci; lift sums K*K entries        */
  CCT_LOWER_FUSED = 4  /* the fusion of Sec. 2.1 ("Fusion"): lowering, multiply and lifting in
                          one kernel, D^ (Type-1 layout) is never materialised: the GEMM gathers
                          its operand tiles from x (through LDS when they fit).  fp32 only;
                          forward pass; backward-data pass of stride-1 layers with pad <= K-1
                          (computed as the convolution of dy with the flipped kernels);
                          backward-weights pass when the input rows that 32 positions touch fit
                          in LDS (K >= 2), or when the layer is unpadded (the split-K GEMM then
                          gathers the lowered rows from x).  Anything else returns
                          CCT_EUNSUPPORTED when FUSED is requested explicitly (AUTO never picks
                          an unsupported layout). */
} cct_lowering_t;

typedef enum {
  CCT_PREC_F32 = 0,            /* fp32 operands, fp32 MFMA accumulate                        */
  CCT_PREC_BF16_IN_F32_ACC = 1 /* operands rounded to bf16 (nearest-even) while lowering,
                                  bf16 MFMA with fp32 accumulate, fp32 outputs               */
} cct_precision_t;

typedef enum {
  CCT_PASS_FORWARD = 0,
  CCT_PASS_BACKWARD_DATA = 1,
  CCT_PASS_BACKWARD_WEIGHTS = 2
} cct_pass_t;

enum {
  CCT_OK = 0,
  CCT_EINVAL = -1,       /* null required pointer, non-positive dim, C or O not divisible by
                            groups, stride < 1, pad < 0, kernel larger than the padded input,
                            unknown enum value, misaligned workspace                         */
  CCT_EWORKSPACE = -2,   /* workspace smaller than what one image needs                      */
  CCT_EUNSUPPORTED = -3, /* explicitly requested combination the library does not run, or
                            sizes beyond its 31-bit row/column limits                        */
  CCT_EHIP = -4,         /* a HIP call failed; see cct_last_hip_error                        */
  CCT_ESCRATCH = -5      /* cct_conv_forward_static: the buffers of one image exceed
                            CCT_STATIC_SCRATCH_BYTES                                         */
};

/* Host struct.  `lowering` holds a cct_lowering_t, `precision` a cct_precision_t. */
typedef struct {
  int32_t N, C, H, W;          /* input x: N x C x H x W                                    */
  int32_t O, K;                /* kernels w: O x (C/groups) x K x K; bias: O floats or NULL */
  int32_t stride, pad, groups;
  int32_t lowering;
  int32_t precision;
} cct_conv_desc_t;

/* Human-readable text for a return code (host, static storage). */
const char* cct_strerror(int code);
/* The hipError_t (as int) of the last failed launch on this thread, 0 if none. */
int cct_last_hip_error(void);

/* Output size, m = n - k + 1 generalised to stride and pad (Sec. 2, below eq. (1)).  Host only. */
int cct_conv_output_dims(const cct_conv_desc_t* desc, int32_t* Hout, int32_t* Wout);

/*
 * Shapes of the lowered matrices per channel group, in the paper's orientation
 * (Sec. 2.1): D^ is rows x cols, K^ is cols x rcols, R^ = D^ K^ is rows x rcols.
 * rows counts all N images (Sec. 2.2: the batched matrix is b times larger).
 *   Type 1: rows = N*Hout*Wout, cols = Cg*K*K, rcols = Og
 *   Type 2: rows = N*H*Wout,    cols = Cg*K,   rcols = Og*K
 *   Type 3: rows = N*H*W,       cols = Cg,     rcols = Og*K*K
 * `lowering` must be TYPE1..TYPE3 (FUSED has no materialised matrices).  Host only.
 */
int cct_lowered_shape(const cct_conv_desc_t* desc, cct_lowering_t lowering, int64_t* rows,
                      int64_t* cols, int64_t* rcols);

/*
 * The automatic lowering optimizer (Sec. 1; Appendix A: which layout is fastest depends
 * on how the number of input channels compares with the number of output channels).
 * Host only, no device work.  Evaluates a cost model
 * (bytes moved by lowering and lifting at the measured HBM rate + GEMM flops at the
 * measured MFMA rate, both calibrated on MI355X) for each layout that the library can
 * run for `pass` on this shape and returns the cheapest.  Never returns a layout that
 * cct_conv_* would reject for the same descriptor; for K == 1, stride == 1, pad == 0 all
 * three layouts coincide and TYPE1 is returned, as it is for a fully connected layer
 * (K == H == W, pad 0, one group, fp32), where every lowering is a reshape.  desc->lowering is
 * ignored.
 */
int cct_pick_lowering(const cct_conv_desc_t* desc, cct_pass_t pass, cct_lowering_t* picked);

/* The optimizer's cost estimate (seconds) for one layout; CCT_EUNSUPPORTED if the layout
 * cannot run for this shape/pass.  Host only. */
int cct_lowering_cost(const cct_conv_desc_t* desc, cct_pass_t pass, cct_lowering_t lowering,
                      double* seconds);

/*
 * Workspace size.  cct_conv_workspace_bytes gives the recommended size (chunks sized by
 * the library's tuned default); cct_conv_workspace_bytes_for_chunk gives the size needed
 * to process `images_per_chunk` images (1..N) at a time.  Any workspace at least as large
 * as the 1-image size is accepted by cct_conv_*; a larger one means larger chunks, up to
 * the whole batch.  desc->lowering == AUTO is resolved with cct_pick_lowering.  Host only.
 *
 * Fully connected layers (K == H == W, pad 0, groups 1, fp32, lowering AUTO or TYPE1: one output
 * pixel per image, the m = 1 case of Sec. 2.1 where every lowering is a reshape of x) run as plain
 * matrix products on x, w and dy in place, never chunked: the recommended workspace holds the
 * split partial products of the forward pass (a few times N*O floats), or a packed copy of dy
 * (about N*O floats) and, for the backward-data pass, its split partial products (a few times
 * N*C*K*K floats).  With a smaller workspace these two passes use fewer splits, and a workspace
 * too small for the unsplit product (forward: N*O floats; backward: the packed dy) sends the layer
 * through the general, chunked path.  The forward
 * pass of such a layer with C*K*K a multiple of 32 reads w with 16-byte loads: w must be 16-byte
 * aligned (CCT_EINVAL otherwise; force another lowering for a misaligned tensor).
 */
int cct_conv_workspace_bytes(const cct_conv_desc_t* desc, cct_pass_t pass, size_t* bytes);
int cct_conv_workspace_bytes_for_chunk(const cct_conv_desc_t* desc, cct_pass_t pass,
                                       int32_t images_per_chunk, size_t* bytes);

/*
 * Forward pass (Sec. 2.1: lowering phase, multiply phase, lifting phase; batched over
 * the chunk, Sec. 2.2).  x, w: device, read.  bias: device, O floats, may be NULL.
 * y: device, written (N*O*Hout*Wout floats).
 */
int cct_conv_forward(const cct_conv_desc_t* desc, const float* x, const float* w,
                     const float* bias, float* y, void* workspace, size_t workspace_bytes,
                     void* hip_stream);

/*
 * Forward pass for callers that cannot allocate or pass device memory of their own beyond the
 * tensors: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same computation, same kernels and same results as cct_conv_forward with a workspace of
 * CCT_STATIC_SCRATCH_BYTES bytes, but the workspace is a fixed array of that size inside the
 * library's device image (every GPU the library is used on holds its own copy until the process
 * ends).  The call allocates and
 * frees nothing, on the host side it only looks up that array's device address the first time it
 * runs on a device.  The batch is processed in chunks of as many images as fit the array;
 * CCT_ESCRATCH (nothing enqueued) if the buffers of a single image do not fit, which can only
 * happen with a materialised layout (the fused layout AUTO prefers needs the packed kernels only).
 * All calls on one GPU share the array, which keeps the previous call's contents (every kernel
 * writes what it later reads, nothing needs to start at zero): calls that may overlap in time on
 * the same GPU, e.g. on two streams, race and must be serialised by the caller.
 * The current device must be the one that owns x, w, bias, y and the stream.
 */
#define CCT_STATIC_SCRATCH_BYTES (32u << 20)
int cct_conv_forward_static(const cct_conv_desc_t* desc, const float* x, const float* w,
                            const float* bias, float* y, void* hip_stream);

/*
 * Backward pass w.r.t. the data: dx = adjoint of the forward map in x applied to dy,
 *   dx[n,q*Cg+ci,h,w] = sum_{o in group q} sum_{i,j} dy[n,o,r,c] * w[o,ci,i,j]
 *   over (i,j) with h = r*stride+i-pad, w = c*stride+j-pad for a valid output position (r,c).
 * Computed as the three phases reversed: inverse lifting of dy, multiply with K^ transposed,
 * inverse lowering (a gather, no atomics).  A phase that is a reshape or a plain gather is done
 * inside the multiply kernel instead of through a matrix in the workspace (Type 1: dy is read
 * in place; Type 2 at stride 1: dy is gathered; Type 3 and 1x1 kernels: dx is written in place).
 * w, dy: device, read.  dx: device, written.
 */
int cct_conv_backward_data(const cct_conv_desc_t* desc, const float* w, const float* dy,
                           float* dx, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * Backward pass w.r.t. the kernels and bias:
 *   dw[o,ci,i,j] = sum_{n,r,c} dy[n,o,r,c] * x[n,q*Cg+ci,r*stride+i-pad,c*stride+j-pad]
 *   dbias[o]     = sum_{n,r,c} dy[n,o,r,c]
 * Computed as D^ transposed times the inverse-lifted dy, reduced over all rows of the
 * batched lowered matrix in fixed order (bit-reproducible run to run).
 * x, dy: device, read.  dw: device, written.  dbias: device, O floats, may be NULL.
 */
int cct_conv_backward_weights(const cct_conv_desc_t* desc, const float* x, const float* dy,
                              float* dw, float* dbias, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/*
 * Test/debug export of the lowering phase alone (Sec. 2.1), whole batch, fp32.
 * The library stores the lowered data matrix TRANSPOSED ("K-major"): for group q,
 * entry (row, col) of the paper's D^ lives at
 *     dhat[(q*cols + col) * ld + row],   ld = cct_lowered_ld(desc, lowering)
 * with row/col numbered as
 *   Type 1: row = (n*Hout + r)*Wout + c,  col = (ci*K + i)*K + j   -> x[n,q*Cg+ci,r*s+i-p,c*s+j-p]
 *   Type 2: row = (n*H + h)*Wout + c,     col = ci*K + j           -> x[n,q*Cg+ci,h,c*s+j-p]
 *   Type 3: row = (n*H + h)*W + w,        col = ci                 -> x[n,q*Cg+ci,h,w]
 * and +0.0f where the source lies in the padding.  Entries with row in [rows, ld) are padding
 * and receive zeros.
 * dhat: device, groups*cols*ld floats.  A pure copy: bit-exact by construction.
 */
int cct_lowered_ld(const cct_conv_desc_t* desc, cct_lowering_t lowering, int64_t* ld);
int cct_lower(const cct_conv_desc_t* desc, cct_lowering_t lowering, const float* x, float* dhat,
              void* hip_stream);

/*
 * The other layers of CaffeNet (Sec. 1: the system optimises all layers
 * with the same techniques and matches Caffe's output layer by layer; Sec. 2.2: whole-batch
 * processing applies to every layer).  The paper does not define them; the semantics are Caffe's.
 * All pointers are device pointers; outputs are overwritten; nothing is allocated.
 *
 * ReLU: y[i] = max(x[i], 0) for i < n.  Backward: dx[i] = dy[i] where x[i] > 0, else 0 (x may be
 * the layer's input or its output: the test agrees).  y may alias x and dx may alias dy.
 */
int cct_relu_forward(const float* x, float* y, int64_t n, void* hip_stream);
int cct_relu_backward(const float* x, const float* dy, float* dx, int64_t n, void* hip_stream);

/*
 * Max pooling over K x K windows with stride `stride` and zero-excluded padding `pad` (< K) of an
 * N x C x H x W tensor.  Output size per axis: ceil((in + 2*pad - K)/stride) + 1, minus one if the
 * last window would start beyond the image (Caffe's rule; CaffeNet: 55 -> 27, 27 -> 13 with K = 3,
 * stride 2).  Windows are clipped to the image; y[n,c,r,q] is the maximum of its window and
 * argmax[n,c,r,q] (N*C*Hout*Wout int32, may be NULL in the forward call) the plane index h*W + w of
 * the FIRST maximum in row-major order of the window.  Backward: dx[n,c,h,w] = sum of dy over the
 * windows whose argmax is (h,w); computed as a gather, bit-reproducible.
 */
typedef struct {
  int32_t N, C, H, W;
  int32_t K, stride, pad;
} cct_pool_desc_t;
int cct_pool_output_dims(const cct_pool_desc_t* desc, int32_t* Hout, int32_t* Wout);
int cct_maxpool_forward(const cct_pool_desc_t* desc, const float* x, float* y, int32_t* argmax,
                        void* hip_stream);
int cct_maxpool_backward(const cct_pool_desc_t* desc, const float* dy, const int32_t* argmax,
                         float* dx, void* hip_stream);

/*
 * Local response normalisation across channels, the layer CaffeNet puts after its first two
 * pooling layers (Sec. 1 names the non-convolutional layers only collectively; the definition is
 * Caffe's):  scale[n,c,h,w] = k + (alpha/size) * sum of x[n,c',h,w]^2 over the `size` channels
 * centred on c (size odd; channels outside [0,C) contribute nothing),  y = x * scale^(-beta).
 * Backward is the exact derivative, computed from x and dy (scale is recomputed, nothing is kept
 * from the forward pass).  x, y, dy, dx: device, contiguous NCHW fp32, N*C*H*W elements; y / dx
 * are overwritten and must not alias x.  size must be 1, 3, 5, 7 or 9 (CCT_EUNSUPPORTED
 * otherwise), k > 0, alpha >= 0 (CCT_EINVAL otherwise).  CaffeNet: size 5, alpha 1e-4, beta 0.75,
 * k 1.  Arithmetic is fp32 (powf).
 */
typedef struct {
  int32_t N, C, H, W;
  int32_t size;
  float alpha, beta, k;
} cct_lrn_desc_t;
int cct_lrn_forward(const cct_lrn_desc_t* desc, const float* x, float* y, void* hip_stream);
int cct_lrn_backward(const cct_lrn_desc_t* desc, const float* x, const float* dy, float* dx,
                     void* hip_stream);

/*
 * Dropout, the layer CaffeNet puts after fc6 and fc7 while training (semantics are Caffe's):
 * y[i] = x[i] * scale where mask[i] != 0, else 0, with scale = 1 / (1 - ratio); the backward pass is
 * the same map applied to dy.  The random draw is the caller's: mask is an input (device, one byte
 * per element), so the library holds no generator state.  y may alias x.  scale > 0 (CCT_EINVAL).
 */
int cct_dropout_forward(const float* x, const uint8_t* mask, float scale, float* y, int64_t n,
                        void* hip_stream);
int cct_dropout_backward(const float* dy, const uint8_t* mask, float scale, float* dx, int64_t n,
                         void* hip_stream);

/*
 * Softmax with multinomial logistic loss, CaffeNet's last layer, on N x C scores (contiguous):
 *   prob[n,c] = exp(x[n,c] - max_c x[n,:]) / sum_c exp(x[n,c] - max_c x[n,:]),
 *   image_loss[n] = -(x[n,l] - max - log(sum)) with l = label[n],  loss[0] = mean of image_loss.
 * Backward: dx[n,c] = (prob[n,c] - [c == label[n]]) / N.  All pointers are device pointers;
 * prob (N*C), image_loss (N), loss (1) and dx (N*C) are overwritten; label holds N int32 values.
 * A label outside [0, C) makes image_loss[n] and loss NaN and contributes no one-hot term; nothing
 * is read out of bounds.  Sums run in a fixed order (bit-reproducible).  N*C < 2^31.
 */
int cct_softmax_loss_forward(int32_t N, int32_t C, const float* x, const int32_t* label, float* prob,
                             float* image_loss, float* loss, void* hip_stream);
int cct_softmax_loss_backward(int32_t N, int32_t C, const float* prob, const int32_t* label,
                              float* dx, void* hip_stream);

/*
 * Measurement aid (used by bench.py for the per-kernel roofline figures).  While enabled,
 * every kernel launch of the library is bracketed by two HIP events on the launching stream.
 * This is the one place where the library creates HIP objects (events, host side only); it
 * still allocates no device memory.  cct_profile_enable(1) clears earlier records and starts
 * recording, cct_profile_enable(0) stops.  cct_profile_read waits (host) for the recorded
 * events and returns one entry per kernel name: number of launches, summed event time, and
 * the summed ALGORITHMIC flops and bytes of those launches (GEMM: 2*M*N*K of the true sizes;
 * index-map kernels: bytes of the tensor read once + the matrix written once, or vice versa).
 * entries: host array of max_entries; *n receives the number written.
 */
typedef struct {
  char name[96];
  int64_t launches;
  double total_ms;
  double flops;
  double bytes;
} cct_profile_entry_t;
int cct_profile_enable(int on);
int cct_profile_read(cct_profile_entry_t* entries, int32_t max_entries, int32_t* n);

/*
 * Measurement aid: a plain device-to-device copy of `bytes` bytes (multiple of 16, both
 * pointers 16-byte aligned, device memory, must not overlap) done by one kernel
 * ("calibration_copy_kernel") that reads every byte once and writes every byte once.  A
 * profiler run that includes it gives the scale between a hardware counter (FETCH_SIZE,
 * WRITE_SIZE) and real bytes.
 */
int cct_calibration_copy(const void* src, void* dst, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CCT_H_ */
