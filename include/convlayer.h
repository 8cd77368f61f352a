/*
 * convlayer.h -- the master's side of arXiv 1712.02546 on one GPU: the workload
 * partition of Section 3.1.1 (calibration probe, Eq. (1)) and a driver that runs
 * all slices of a partitioned layer through the per-device entry points of
 * convslice.h and assembles the layer's outputs in place (Algorithm 1 without
 * the sockets: inputs broadcast, kernels split, the returned maps put side by
 * side).
 *
 * Same conventions as convslice.h: conv_status_t return codes, device pointers
 * for tensors and workspaces, host pointers for descriptors, times, shares and
 * bounds.  The k0/k1 fields of a layer descriptor are ignored by the conv_layer_*
 * and conv_calibrate calls (the slices come from `bounds`, the probe runs the
 * slice given to it, see below).
 */
#ifndef CONVLAYER_H
#define CONVLAYER_H

#include "convslice.h"

#ifdef __cplusplus
extern "C" {
#endif

/* CONV_ERR_PARTITION: n < 1 or n > CONV_MAX_DEVICES, a time that is not finite and positive,
 * K < 0, or bounds that are not 0 = b[0] <= b[1] <= ... <= b[n] = K. */
#define CONV_MAX_DEVICES 64 /* most devices / slices one partition may have */

/*
 * Eq. (1) of Section 3.1.1.  t[i] > 0 is the time device i needed for the common
 * probe workload (any unit); host arrays.
 *   shares[i] = (max(t)/t[i]) / sum_j (max(t)/t[j])                 (n doubles, may be NULL)
 *   bounds[0] = 0 <= ... <= bounds[n] = K, device i owns kernels [bounds[i], bounds[i+1])
 *                                                                    (n+1 ints, may be NULL)
 * The paper does not say how fractional kernel counts are rounded.  Here: largest
 * remainder -- floor(shares[i]*K) each, the kernels left over go one each to the
 * largest fractional parts, equal parts (within K * 2^-40) to the lower device index.
 * Arithmetic is IEEE double.  Returns CONV_OK, CONV_ERR_NULL (t) or CONV_ERR_PARTITION.
 */
int conv_partition(const double *t, int32_t n, int32_t K, double *shares, int32_t *bounds);

/*
 * The estimate the worked example of Section 3.1.1 makes: device i needs
 * t[i]*shares[i] for its share; *finish is the largest of these, *speedup is
 * min(t) / *finish (the fastest device alone against the partitioned run, no
 * communication).  Either output may be NULL.
 */
int conv_partition_estimate(const double *t, const double *shares, int32_t n, double *finish,
                            double *speedup);

/*
 * Calibration probe of Section 3.1.1: times a convolution with the layer's image
 * and kernel sizes on random values.  pass_mask is a bit set of (1 << conv_pass_t)
 * (0 means forward only, the paper's probe); the slice [k0,k1) of desc is what is
 * timed, so a probe can "simulate part of the layer".  The call fills its operands
 * (carved from ws) with a fixed pseudo-random pattern in (-1,1), runs one untimed
 * and `reps` timed repetitions of the selected passes on hip_stream, WAITS for
 * them, and returns the mean seconds per repetition in *seconds.  It creates and
 * destroys two HIP events; it allocates no device memory.
 * ws must hold conv_calibrate_workspace_bytes(desc, pass_mask) bytes.
 */
size_t conv_calibrate_workspace_bytes(const conv_desc_t *desc, int pass_mask);
int conv_calibrate(const conv_desc_t *desc, int pass_mask, int reps, void *ws, size_t ws_bytes,
                   void *hip_stream, double *seconds);

/*
 * Partitioned layer (Algorithm 1, lines "all slaves receive same inputs but
 * different kernels" ... "master node receives all feature maps").  bounds is a
 * host array of n_slices+1 ints as produced by conv_partition; slice i is kernels
 * [bounds[i], bounds[i+1]).  Tensor arguments are those of the matching conv_*
 * call on the full layer.
 *
 *   conv_layer_fwd / conv_layer_bwd_weight: the slices write disjoint channel
 *     blocks of y / dw.  Slices that are too small to fill the GPU (< 2e10 FLOP per
 *     pass) are enqueued on up to four internal streams (default priority, created
 *     on first use and kept for the life of the process) that fork from and join
 *     back into hip_stream with events, so they share the GPU; if every slice is
 *     large they run one after the other on hip_stream.  Either way, work enqueued
 *     on hip_stream after the call sees all of y / dw.
 *   conv_layer_bwd_data: dx is the sum of the slices' partial gradients, added in
 *     slice order on hip_stream itself (slice 0 honours desc->accumulate, the
 *     others accumulate), so the result does not depend on timing.
 *
 * ws must hold conv_layer_workspace_bytes(...) bytes: every slice gets a region
 * of its own (for bwd_data one region reused in turn).  Empty slices are skipped.
 * The calls return without synchronising.  Host threads may call concurrently:
 * the fork / enqueue / join sequence on the device's internal streams is taken
 * under a lock, so calls that use them are enqueued one after the other (and
 * their slices serialise on those streams).  As for every entry point, calls
 * that overlap in time must not share ws.  Workspace sizes are valid for the
 * device that is current when they are queried.
 */
size_t conv_layer_workspace_bytes(const conv_desc_t *desc, const int32_t *bounds, int32_t n_slices,
                                  int pass);
int conv_layer_fwd(const conv_desc_t *desc, const int32_t *bounds, int32_t n_slices, const void *x,
                   const void *w, void *y, void *ws, size_t ws_bytes, void *hip_stream);
int conv_layer_bwd_data(const conv_desc_t *desc, const int32_t *bounds, int32_t n_slices,
                        const void *dy, const void *w, void *dx, void *ws, size_t ws_bytes,
                        void *hip_stream);
int conv_layer_bwd_weight(const conv_desc_t *desc, const int32_t *bounds, int32_t n_slices,
                          const void *x, const void *dy, void *dw, void *ws, size_t ws_bytes,
                          void *hip_stream);

/*
 * Scalability model of Section 4.2.  All host code.
 *
 * conv_comm_elements: Eq. (2) -- elements the master exchanges with the slaves for one
 *   batch, summed over the distributed layers: in^2*inCh*batch (input maps) +
 *   k^2*numK*inCh (kernels) + out^2*numK*batch (output maps) per layer.
 * conv_comm_elements_partition: the same count for one layer split at `bounds` among
 *   n_devices when device `master` keeps its own block at home.  The paper does not
 *   spell this case out; here every other device receives all input maps and its own
 *   kernels and returns its own maps (one slave holding every kernel gives Eq. (2)).
 * conv_scaling_estimate: time of one batch = t_comm + max_i(shares[i]*t_conv[i]) + t_comp
 *   ("Comm. time", "Conv. time" of the slowest node, "Comp. time" of the other layers),
 *   with t_comm = elements * bytes_per_element * 8 / bits_per_second (the paper:
 *   doubles at about 5 Mbps); *speedup compares with device `master` doing all
 *   convolutions alone without communication; *amdahl is the bound
 *   1 / (1 - conv fraction of that single-device time).  Outputs may be NULL.
 * Counts are returned as doubles (exact below 2^53).  Errors: CONV_ERR_NULL,
 * CONV_ERR_SHAPE (negative extents or batch), CONV_ERR_PARTITION (bounds, times,
 * shares, master index, non-positive bandwidth).
 */
typedef struct {
  int32_t in;    /* input width = height  */
  int32_t inCh;  /* input channels        */
  int32_t k;     /* kernel width = height */
  int32_t numK;  /* kernels               */
  int32_t out;   /* output width = height */
} conv_comm_layer_t;

int conv_comm_elements(const conv_comm_layer_t *layers, int32_t n_layers, int64_t batch, double *elements);
int conv_comm_elements_partition(const conv_comm_layer_t *layer, int64_t batch, const int32_t *bounds,
                                 int32_t n_devices, int32_t master, double *elements);
int conv_scaling_estimate(const double *t_conv, const double *shares, int32_t n_devices, int32_t master,
                          double t_comp, double elements, double bytes_per_element, double bits_per_second,
                          double *batch_seconds, double *speedup, double *amdahl);

#ifdef __cplusplus
}
#endif
#endif /* CONVLAYER_H */
