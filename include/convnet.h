/*
 * convnet.h -- the layers of the paper's network other than the convolutions
 * (arXiv 1712.02546, Section 4.1: "Normalization layer", "Pooling layer, with stride 2",
 * "Fully connected layer", "Loss layer, with softmax loss"), so that the share of a training
 * step that is not convolution (the paper's "Comp. time", Section 4.2) can be measured on the
 * same GPU.  Part of libconvslice.so.  The paper only names these layers; the definitions
 * below are this library's reading of them.
 *
 * All tensors are fp32 DEVICE buffers owned by the caller, row-major (NCHW for maps), 4-byte
 * aligned; labels are int32 device buffers.  Calls enqueue on hip_stream (hipStream_t as
 * void*, NULL = default stream) and return without synchronising; they allocate nothing and
 * use no atomics, so results are the same on every run.  Return values are conv_status_t
 * (convslice.h): CONV_ERR_NULL for a missing pointer, CONV_ERR_SHAPE for a non-positive or
 * inconsistent extent (window larger than the map, even or non-positive normalisation size,
 * more than 2^31-1 elements per tensor), CONV_ERR_LAUNCH if the runtime refuses a launch.
 */
#ifndef CONVNET_H
#define CONVNET_H

#include "convslice.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Local response normalisation across channels (maps [N][C][HW]):
 *   scale[n,c,i] = kappa + alpha * sum_{c' in W(c)} x[n,c',i]^2,   y = x * scale^(-beta),
 * W(c) = the `size` channels centred on c (size odd), clipped at 0 and C.  scale is written for
 * the backward pass (same shape as x), which also takes y.  N at most 65535.  Backward:
 *   dx[c] = dy[c]*scale[c]^(-beta) - 2*alpha*beta*x[c] * sum_{c' in W(c)} dy[c']*x[c']*scale[c']^(-beta-1).
 */
int net_norm_fwd(const float *x, float *y, float *scale, int32_t N, int32_t C, int32_t HW, int32_t size,
                 float kappa, float alpha, float beta, void *hip_stream);
int net_norm_bwd(const float *x, const float *y, const float *scale, const float *dy, float *dx, int32_t N,
                 int32_t C, int32_t HW, int32_t size, float kappa, float alpha, float beta, void *hip_stream);

/*
 * Max pooling of NC maps of H x W over win x win windows with the given stride, no padding:
 * y is [NC][P][Q], P = floor((H - win)/stride) + 1.  Backward: dx[NC][H][W] receives, for every
 * window, dy at the window's first maximum in row-major order; inputs outside every window get 0.
 */
int net_pool_fwd(const float *x, float *y, int32_t NC, int32_t H, int32_t W, int32_t win, int32_t stride,
                 void *hip_stream);
int net_pool_bwd(const float *x, const float *dy, float *dx, int32_t NC, int32_t H, int32_t W, int32_t win,
                 int32_t stride, void *hip_stream);

/*
 * Fully connected layer: y[n,o] = sum_i x[n,i]*W[o,i] + b[o]   (x [N][I], W [O][I], b [O], y [N][O]).
 * Backward: dx[n,i] = sum_o dy[n,o]*W[o,i];  dW[o,i] = sum_n dy[n,o]*x[n,i];  db[o] = sum_n dy[n,o].
 * Any of dx, dW, db may be NULL (not computed).
 */
int net_fc_fwd(const float *x, const float *W, const float *b, float *y, int32_t N, int32_t I, int32_t O,
               void *hip_stream);
int net_fc_bwd(const float *x, const float *W, const float *dy, float *dx, float *dW, float *db, int32_t N,
               int32_t I, int32_t O, void *hip_stream);

/*
 * Softmax loss over logits z [N][O] and labels [N] (0 <= label < O, not checked on the device):
 * *loss (one device float) = mean_n -log softmax(z[n])[labels[n]];  dz = (softmax(z) - onehot) / N.
 */
int net_softmax_loss_fwd(const float *z, const int32_t *labels, float *loss, int32_t N, int32_t O,
                         void *hip_stream);
int net_softmax_loss_bwd(const float *z, const int32_t *labels, float *dz, int32_t N, int32_t O,
                         void *hip_stream);

/* Plain gradient step w -= lr * dw over count floats (the paper states no momentum or decay). */
int net_sgd_update(float *w, const float *dw, float lr, int64_t count, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CONVNET_H */
