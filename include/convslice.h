/*
 * convslice.h -- C ABI of libconvslice.so (AMD Instinct MI355X, gfx950 only).
 *
 * One device's share of a convolutional layer as defined by arXiv 1712.02546,
 * Section 4.1.2 and Algorithms 1-2: every device receives the same input maps
 * and a contiguous block [k0,k1) of the layer's kernels, convolves all inputs
 * with its own kernels and returns its own output maps, which the master puts
 * side by side.  The abstract counts the backward convolutions in the same
 * distributed work, so the library has three entry points: forward, input
 * gradient, weight gradient.
 *
 * Conventions (the paper prints no formula; these are the textbook ones):
 *   cross-correlation, zero padding, no bias, no activation,
 *   P = floor((H + 2*pad_h - R) / stride_h) + 1, Q likewise,
 *   row-major tensors, innermost index last:
 *     x, dx : [N][C][H][W]        w, dw : [K][C][R][S]        y, dy : [N][K][P][Q]
 *
 * Slice addressing.  w, dw, y and dy always point at FULL-layer tensors with K
 * channels; a call reads and writes only channels k0 <= k < k1 and never
 * touches the others, so calls on disjoint slices that share y (or dw)
 * assemble the whole layer in place.  dx receives the partial sum over the
 * slice's kernels; with accumulate = 1 it is added to what dx holds, so the
 * slices of a partition can be summed by consecutive calls on one stream.  A
 * device that holds only its own kernels and maps in memory uses K = k1-k0,
 * k0 = 0 on its packed buffers.
 *
 * Pointers.  x, w, y, dy, dx, dw and ws are DEVICE pointers (hipMalloc'ed or
 * equivalent, e.g. a PyTorch-ROCm tensor's data_ptr()), owned by the caller,
 * 16-byte aligned.  desc is a HOST pointer, read before the call returns.
 * Inputs are never written.  ws is scratch the caller provides: at least
 * conv_workspace_bytes(desc, pass) bytes, 256-byte aligned, contents
 * undefined before and after.  Calls that overlap in time must not share ws.
 * The size never grows when the slice shrinks: a workspace sized for
 * [k0,k1) serves every call of the same layer and pass on a part of it.
 *
 * Execution.  Work is enqueued on hip_stream (a hipStream_t passed as void*,
 * NULL = default stream) and the call returns without synchronising.  The
 * library allocates no device memory and keeps no state between calls apart
 * from one-time kernel attribute set-up and the one-shot timing probe below.
 * A call enqueues kernel launches only (no copies, no memsets, no events unless
 * the probe is armed), so after one ordinary call of the same layer and pass
 * on the device (which does the attribute set-up) the calls can be recorded
 * into a HIP graph by stream capture and replayed.
 *
 * Errors.  Every entry point returns CONV_OK (0) or a negative conv_status_t.
 * All argument checks happen before the first launch; on an argument error
 * nothing is enqueued.  k0 == k1 is valid: forward and weight gradient do
 * nothing, input gradient zero-fills dx unless accumulate = 1.
 *
 * Precision.  CONV_F32: fp32 tensors, fp32 matrix-core (MFMA) products and
 * accumulation.  CONV_BF16: x, w, y, dy, dx are bfloat16 (upper 16 bits of an
 * fp32, round-to-nearest-even on output), accumulation is fp32, dw is fp32.
 * bf16 products run on the bf16 matrix-core instructions, with one
 * exception that converts its operands to fp32 copies and runs the fp32
 * kernels: forward pass and input gradient of layers with fewer than 8
 * input channels that the few-channel path does not take (C*R*S > 480 or
 * P*Q < 32).  conv_pass_path() names the kernel and arithmetic of a pass.
 *
 * Limits.  Each tensor (and each internal transposed copy, whose batch extent
 * is rounded up to a multiple of 32) must have fewer than 2^30 - 4096 elements
 * (the kernels address their work copies with 32-bit byte offsets);
 * R*S <= 1024.  Otherwise CONV_ERR_SHAPE.
 */
#ifndef CONVSLICE_H
#define CONVSLICE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CONV_OK = 0,
  CONV_ERR_NULL = -1,      /* a required pointer is NULL                         */
  CONV_ERR_SHAPE = -2,     /* non-positive extent, P < 1 or Q < 1, limit exceeded */
  CONV_ERR_SLICE = -3,     /* not 0 <= k0 <= k1 <= K                             */
  CONV_ERR_DTYPE = -4,     /* dtype is not a conv_dtype_t                        */
  CONV_ERR_WORKSPACE = -5, /* ws_bytes too small, or ws missing / misaligned     */
  CONV_ERR_LAUNCH = -6,    /* the HIP runtime refused a launch                   */
  CONV_ERR_ALIGN = -7,     /* a tensor pointer is not 16-byte aligned            */
  CONV_ERR_PASS = -8,      /* pass is not a conv_pass_t                          */
  CONV_ERR_PARTITION = -9  /* convlayer.h: bad times, device count or k-bounds   */
} conv_status_t;

typedef enum { CONV_F32 = 0, CONV_BF16 = 1 } conv_dtype_t;

typedef enum { CONV_PASS_FWD = 0, CONV_PASS_BWD_DATA = 1, CONV_PASS_BWD_WEIGHT = 2 } conv_pass_t;

typedef struct {
  int32_t N, C, H, W;      /* input extents                                  */
  int32_t K, R, S;         /* FULL layer: K kernels of C x R x S             */
  int32_t stride_h, stride_w;
  int32_t pad_h, pad_w;
  int32_t k0, k1;          /* this device's kernels, 0 <= k0 <= k1 <= K      */
  int32_t dtype;           /* conv_dtype_t of x, w, y, dy, dx (dw is fp32)   */
  int32_t accumulate;      /* conv_bwd_data only: 0 -> dx = ..., 1 -> dx += ... */
} conv_desc_t;

/* Output extents P and Q of the layer.  Returns CONV_OK or CONV_ERR_*. */
int conv_output_dims(const conv_desc_t *desc, int32_t *P, int32_t *Q);

/* Scratch bytes the given pass needs for this descriptor (0 on invalid input).  Host arithmetic,
 * except that the first call asks the HIP runtime for the compute-unit count of the current
 * device (512 workgroup slots are assumed when no device is visible): sizes are valid for
 * that device. */
size_t conv_workspace_bytes(const conv_desc_t *desc, int pass);

/*
 * Forward pass of the slice (Algorithm 2's loop over the device's own maps):
 *   y[n,k,p,q] = sum_{c,r,s} x[n,c,p*stride_h-pad_h+r,q*stride_w-pad_w+s] * w[k,c,r,s]
 * for k0 <= k < k1.  Reads x (all C channels) and w[k0:k1]; writes y[:,k0:k1].
 */
int conv_fwd(const conv_desc_t *desc, const void *x, const void *w, void *y,
             void *ws, size_t ws_bytes, void *hip_stream);

/*
 * conv_fwd for callers that cannot allocate device memory or hand over a
 * workspace (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the same kernels, with the workspace taken from a device
 * array of CONV_NOALLOC_MAX_WORKSPACE bytes that is part of the library's code
 * object (each GPU the library runs on holds its own copy until the process
 * ends).  The call itself allocates nothing.  Arguments and errors as for
 * conv_fwd; a layer whose conv_workspace_bytes(desc, CONV_PASS_FWD) exceeds
 * CONV_NOALLOC_MAX_WORKSPACE is refused with CONV_ERR_WORKSPACE before any
 * launch.  All calls on one GPU share that GPU's array: calls that overlap in
 * time on one GPU (different streams or host threads) race and must be
 * serialised by the caller; calls on one stream are safe.  The array keeps the
 * last call's contents; the kernels write every part they read, so no call
 * depends on them.
 */
#define CONV_NOALLOC_MAX_WORKSPACE (96u << 20)
int conv_fwd_noalloc(const conv_desc_t *desc, const void *x, const void *w, void *y,
                     void *hip_stream);

/*
 * Input gradient of the slice (backward convolution, abstract):
 *   dx[n,c,h,v] (+)= sum_{k0<=k<k1} sum_{r,s} dy[n,k,p,q] * w[k,c,r,s]
 * over the (p,q) with p*stride_h-pad_h+r = h and q*stride_w-pad_w+s = v.
 * Reads dy[:,k0:k1] and w[k0:k1]; writes (accumulate=0) or adds to
 * (accumulate=1) the whole of dx.  Pixels no window covers receive 0.
 */
int conv_bwd_data(const conv_desc_t *desc, const void *dy, const void *w, void *dx,
                  void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Weight gradient of the slice (backward convolution, abstract):
 *   dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*stride_h-pad_h+r,q*stride_w-pad_w+s]
 * for k0 <= k < k1.  Reads x and dy[:,k0:k1]; writes dw[k0:k1] (always fp32).
 */
int conv_bwd_weight(const conv_desc_t *desc, const void *x, const void *dy, void *dw,
                    void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Measurement aid, not part of the method: arms a one-shot probe for the NEXT
 * conv_fwd / conv_bwd_data / conv_bwd_weight call made by the calling host
 * thread.  That call records start_event (a hipEvent_t passed as void*) on its
 * stream right before its matrix-core kernel and stop_event right after it, so
 * the kernel's duration can be read with hipEventElapsedTime once the stream
 * has drained; the layout kernels around it are outside the bracket (a pass
 * that runs its matrix-core kernel once per group of images -- the input
 * gradient of a few-channel layer whose intermediate exceeds 160 MiB -- is
 * bracketed from the first group's kernel to the last one's, with the sums
 * over taps of the groups in between).  The probe
 * is consumed by that call (also when it fails or has nothing to launch).
 * Passing NULL for either event disarms it.  Always returns CONV_OK.
 */
int conv_probe_next_call(void *start_event, void *stop_event);

/*
 * Measurement aid: which kernel family serves the given pass of this layer, as
 * "<matrix-core kernel>: <arithmetic>, <layout>" (static string; host logic only, the
 * same decision the pass itself takes).  "invalid descriptor" / "unknown pass" otherwise.
 */
const char *conv_pass_path(const conv_desc_t *desc, int pass);

/* Static, never-NULL description of a status code. */
const char *conv_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CONVSLICE_H */
