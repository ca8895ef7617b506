/*
 * rocket.h -- C ABI of the MI355X (gfx950) ROCKET transform library.
 *
 * The library computes the hot path of "Making the 'exceptionally fast' ROCKET
 * model faster": K random dilated, padded, biased 1-D convolution kernels are
 * applied to every (multivariate) series and each kernel output is pooled
 * (paper section 3, parts (1) and (2)), with the backward pass that the soft
 * pooling allows.  Around it: the input prologue for raw 8-bit samples
 * (sections 4.1, 4.3), the ridge regressor on the features (part (3), section
 * 3.3), inference in one call, a training step on the kernels (section 6), and
 * a MINIROCKET-style variant (sections 2 and 6: predetermined two-valued
 * kernels, biases from the data, PPV only).
 *
 * Notation.  Kernel k has length len in {7,9,11}, dilation d >= 1, padding
 * p in {0, (len-1)d/2}, a bias, a list of n_ch distinct channels and one weight
 * row of len floats per listed channel.  For a series x (C rows of L floats)
 *
 *     y[t] = bias + sum_c sum_j w[c][j] * x[channel[c]][t + j*d - p],   x = 0 outside [0,L)
 *     t = 0 .. n-1,   n = L + 2p - (len-1)d      (cross-correlation, no flip)
 *
 * Features (section 3.2):
 *     ROCKET_F_MAX      max_t y[t]
 *     ROCKET_F_PPV      (1/n) #{t : y[t] > 0}                       Eq. 1-2
 *     ROCKET_F_SOFTPPV  (1/n) sum_t 1/(1+exp(-(lambda*y[t]+shift)))  Eq. 3-4
 * The prose under Eq. 3 fixes shift = -3; the printed formula is shift = +3.
 *
 * Conventions.  Every function returns ROCKET_OK (0) or a negative error code
 * and never throws or aborts; rocket_last_error() gives the message of the
 * last failure on the calling thread.  "host" / "device" below says where a
 * pointer must live.  All arrays are contiguous.  Device work is enqueued on
 * the given HIP stream (a hipStream_t passed as void*, NULL = default stream)
 * and is not synchronised: the caller synchronises the stream before reading
 * results.  Outputs are overwritten, never accumulated into.  Inputs must be
 * finite.  A handle may be used from one thread at a time.
 */
#ifndef ROCKET_MI355X_H
#define ROCKET_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ROCKET_OK = 0,
    ROCKET_EINVAL = -1,      /* bad argument value (null pointer, size < 1, bad mask, non-finite scalar) */
    ROCKET_ENOMEM = -2,      /* host or device allocation failed */
    ROCKET_EHIP = -3,        /* a HIP runtime call or kernel launch failed */
    ROCKET_ESHAPE = -4,      /* kernel parameters inconsistent with (C, L) */
    ROCKET_EWORKSPACE = -5   /* workspace missing or smaller than rocket_workspace_bytes() */
};

/* feature mask bits; output planes appear in bit order */
enum { ROCKET_F_MAX = 1, ROCKET_F_PPV = 2, ROCKET_F_SOFTPPV = 4 };

/* opaque, library-owned set of K kernels for series of shape C x L */
typedef struct rocket_kernels rocket_kernels;

/* Borrowed host pointers into a handle; valid until the handle is freed.
 * weights of kernel k start at weights[w_off[k]] and are channel-major
 * (n_ch[k] rows of length[k]); its channel list starts at channels[ch_off[k]]. */
typedef struct rocket_kernels_view {
    int32_t K, C, L;
    int64_t total_channels;   /* sum of n_ch          */
    int64_t total_weights;    /* sum of n_ch * length */
    const int32_t *length, *dilation, *padding, *n_ch;   /* [K] */
    const float *bias;                                   /* [K] */
    const int64_t *ch_off, *w_off;                       /* [K+1] */
    const int32_t *channels;                             /* [total_channels] */
    const float *weights;                                /* [total_weights] */
} rocket_kernels_view;

/*
 * Random kernel initialisation (section 3.1): length uniform on {7,9,11};
 * N(0,1) weights, mean-centred per (kernel, channel) row; bias uniform on
 * [-1,1); dilation floor(2^(u*log2((L-1)/(len-1)))); a fair coin between
 * "same" padding and none; a random subset of floor(2^(u*log2(min(C,9)+1)))
 * channels.  Kernel k is drawn from its own SplitMix64 stream of (seed, k), so
 * the result is a pure function of (seed, K, C, L).  Host only: no GPU needed.
 * Requires K, C >= 1 and L >= 11.  *out receives a new handle (free it with
 * rocket_free_kernels).
 */
int rocket_make_kernels(uint64_t seed, int32_t K, int32_t C, int32_t L, rocket_kernels **out);

/*
 * Builds a handle from kernels generated elsewhere (the paper loads externally
 * generated kernels into its model, section 3.1).  All pointers are host
 * arrays that are copied: length, dilation, padding, n_ch, bias have K entries;
 * channels has sum(n_ch) entries; weights has sum(n_ch*length) entries, kernel
 * after kernel, channel-major.  Checks: length in {7,9,11}; d >= 1;
 * padding is 0 or (len-1)d/2; n = L + 2p - (len-1)d >= 1; 1 <= n_ch <= C;
 * channels distinct and in [0,C); weights and biases finite.  Violations give
 * ROCKET_ESHAPE.
 */
int rocket_kernels_import(int32_t K, int32_t C, int32_t L,
                          const int32_t *length, const int32_t *dilation, const int32_t *padding,
                          const float *bias, const int32_t *n_ch, const int32_t *channels,
                          const float *weights, rocket_kernels **out);

/* Fills *view with borrowed host pointers to the handle's arrays. */
int rocket_kernels_view_get(const rocket_kernels *kernels, rocket_kernels_view *view);

/* Replaces all weights and/or all biases (host arrays in the handle's layout;
 * either may be NULL = keep).  For training loops and finite differences. */
int rocket_kernels_set_params(rocket_kernels *kernels, const float *weights, const float *bias);

/* Number of output planes of a feature mask (its population count), 0 if invalid. */
int32_t rocket_num_features(uint32_t feature_mask);

/*
 * Bytes of device workspace that rocket_transform (backward = 0) or
 * rocket_soft_ppv_backward (backward = 1) needs for a batch of B series.
 * Returns 0 on invalid arguments.  The workspace holds a zero-padded copy of
 * the batch (so that dilated reads never leave a row) and partial results: for
 * the transform the pooled values of every (series, time tile of a kernel), for
 * the backward pass the partial gradients of every (series, time tile of a
 * kernel); and 16 bytes per (series, channel) row for the statistics of the
 * 8-bit entry points.  Its contents are scratch.
 */
size_t rocket_workspace_bytes(const rocket_kernels *kernels, int32_t B, uint32_t feature_mask, int backward);

/*
 * The transform, parts (1) and (2) of section 3 fused: x_dev is device memory,
 * B x C x L float32 (row-major, L contiguous) with C, L those of the handle;
 * out_dev is device memory, B x (F*K) float32 with F = rocket_num_features(mask):
 * out[b*F*K + f*K + k] is feature plane f (bit order of the mask) of kernel k
 * in the handle's kernel order.  workspace_dev: device memory of at least
 * rocket_workspace_bytes(kernels, B, mask, 0) bytes, 256-byte aligned.
 * lambda and shift are used by ROCKET_F_SOFTPPV only (the paper's reading is
 * shift = -3).  On first use the handle uploads its parameters to the current
 * device (one hipMalloc); later calls allocate nothing, copy nothing and never
 * synchronise: they only launch kernels on hip_stream, so they can be recorded
 * by a stream capture (while rocket_profile_enable is off).
 */
int rocket_transform(rocket_kernels *kernels, const float *x_dev, int32_t B, uint32_t feature_mask,
                     float lambda, float shift, float *out_dev,
                     void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/*
 * rocket_transform for callers that cannot allocate device memory or hand over a workspace
 * (a serving loop that transforms one reading after another, a harness that forbids
 * allocation): same inputs, same outputs, bit for bit, but the workspace is a 64 MiB array
 * that lives in the library's device image (each GPU the library runs on holds it until the
 * process ends).  The call allocates and frees nothing and creates no events; it only
 * launches kernels on hip_stream.  Requirements: rocket_workspace_bytes(kernels, B, mask, 0)
 * must not exceed 64 MiB (ROCKET_EWORKSPACE otherwise; 64 MiB hold e.g. 8 series of
 * 20 x 50,000 samples with 10,000 kernels, or 256 x 1 x 1,000 with 10,000 kernels), and the
 * handle's parameters must already be on the current device (ROCKET_EINVAL otherwise): one
 * earlier rocket_transform call on the handle uploads them, and so does any other compute
 * call; after rocket_kernels_set_params they have to be uploaded again the same way.
 * All calls on one GPU share the one array: two calls that overlap in time on the same GPU
 * (different streams, different threads) race and give wrong results; calls on one stream
 * are ordered by the stream.  Nothing in the array needs clearing between calls: every word a
 * call reads it has written before.  rocket_profile_enable is ignored by this entry point.
 */
int rocket_transform_noalloc(rocket_kernels *kernels, const float *x_dev, int32_t B, uint32_t feature_mask,
                             float lambda, float shift, float *out_dev, void *hip_stream);

/*
 * Backward pass through the pooling (the gradient flow that softPPV allows,
 * section 3.2): given grad_out_dev (device, same layout as the transform's
 * output for feature_mask, which must contain ROCKET_F_SOFTPPV), computes the
 * gradient of sum(grad_out * features) with respect to the stored weights and
 * biases, summed over the batch:
 *     s_t = 1/(1+exp(-(lambda*y_t+shift))),  q_t = g_soft[b,k]*(lambda/n)*s_t*(1-s_t)
 *     grad_b[k]       = sum_b sum_t q_t
 *     grad_w[k][c][j] = sum_b sum_t q_t * x_b[channel[c]][t + j*d - p]
 * If include_max != 0 (mask must contain ROCKET_F_MAX) the max plane adds its
 * sub-gradient at the first position attaining the maximum.  The PPV plane has
 * zero gradient and is ignored.  grad_w_dev: device, total_weights floats in
 * the layout of `weights`; grad_b_dev: device, K floats.  No gradient with
 * respect to x.  workspace: rocket_workspace_bytes(kernels, B, mask, 1) bytes.
 * Kernels with more than 9 channels (possible only through rocket_kernels_import)
 * are rejected with ROCKET_ESHAPE.  Every sum (over positions, over the batch) is taken
 * in a fixed order without atomics, so two runs on the same inputs agree bit for bit.
 */
int rocket_soft_ppv_backward(rocket_kernels *kernels, const float *x_dev, int32_t B, uint32_t feature_mask,
                             const float *grad_out_dev, float lambda, float shift, int include_max,
                             float *grad_w_dev, float *grad_b_dev,
                             void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/*
 * The same two calls for raw 8-bit samples with the input prologue fused in.  The paper's
 * examples are integer light intensities and every channel of every example is
 * z-normalised before the transform (sections 4.1 and 4.3).  x_u8_dev is device memory,
 * B x C x L uint8; each (series, channel) row is replaced by (x - mean) / std with its own
 * mean and population standard deviation (divide by L; exact integer sums, then fp64,
 * rounded once to fp32), a row of zero variance by zeros, and the result is transformed
 * exactly as the float32 entry points do.  The normalised values exist only in the padded
 * workspace copy: the batch is read as one byte per sample and no fp32 batch is stored.
 * All other arguments, the workspace size and the error behaviour are those of
 * rocket_transform and rocket_soft_ppv_backward.
 */
int rocket_transform_u8(rocket_kernels *kernels, const uint8_t *x_u8_dev, int32_t B, uint32_t feature_mask,
                        float lambda, float shift, float *out_dev,
                        void *workspace_dev, size_t workspace_bytes, void *hip_stream);
int rocket_soft_ppv_backward_u8(rocket_kernels *kernels, const uint8_t *x_u8_dev, int32_t B, uint32_t feature_mask,
                                const float *grad_out_dev, float lambda, float shift, int include_max,
                                float *grad_w_dev, float *grad_b_dev,
                                void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/*
 * The work decomposition, for inspection and tests.  The outputs of kernel k are viewed as
 * rows of d consecutive positions (position t = row*d + column); its n / d full rows are cut
 * into jobs (time tiles), one workgroup per (series, job) in both passes.  Job j covers rows
 * [row0[j], row1[j]) of kernel kernel[j]; bit 0 of flags[j] says that it also owns the partial
 * last row (the n mod d positions after the full rows), bit 1 that it is the only job of its
 * kernel.  Jobs are listed in launch order.  The pointers are borrowed from the handle
 * (host memory, *count entries each, stride_bytes apart: they point into an array of records).
 */
int rocket_jobs_view_get(const rocket_kernels *kernels, int32_t *count, const int32_t **kernel,
                         const int32_t **row0, const int32_t **row1, const int32_t **flags,
                         int32_t *stride_bytes);

/* Algorithmic work of one call, for roofline accounting: *conv_fma receives
 * sum_k n_k*n_ch_k*len_k (fused multiply-adds per series of the forward conv),
 * *outputs receives sum_k n_k (pooled positions per series). */
int rocket_work_per_series(const rocket_kernels *kernels, double *conv_fma, double *outputs);

/*
 * Timing of the dominant kernel, for roofline measurement.  While enabled, every
 * rocket_transform / rocket_soft_ppv_backward call on this handle records a HIP
 * event pair on its stream around its main kernel (the conv + pooling kernel;
 * the padding copy and the small reduction kernels are outside the pair).
 * rocket_profile_read waits for the recorded events, returns the number of
 * launches and their summed duration in milliseconds since the last read, and
 * clears the list.  Disabled by default; enabling allocates events per call.
 */
int rocket_profile_enable(rocket_kernels *kernels, int enable);
int rocket_profile_read(rocket_kernels *kernels, int32_t *launches, double *total_ms);

/*
 * Measured ceiling for the roofline figure: runs a kernel that issues nothing but plain
 * (one per lane) FP32 fused multiply-adds from every vector ALU of the current device, waits
 * for it, and returns its rate in *tflops (host pointer).  The transform's arithmetic is made
 * of the same instruction; the data-sheet FP32 vector peak assumes the packed form and is
 * twice this.  Takes a few milliseconds; allocates and frees a few bytes and two events.
 */
int rocket_calibrate_fma(double *tflops, void *hip_stream);

/*
 * Measured rates of the other units that can bound the transform's kernels on the current device, one
 * micro-kernel per unit, for the roofline discussion (which unit stops a kernel).  out (host, at least
 * ROCKET_CAL_COUNT doubles) receives, by index:
 *   ROCKET_CAL_LOAD_B32_L1       GB/s of 4-byte buffer loads into registers, every CU re-reading 4 KB (L1 hits)
 *   ROCKET_CAL_LOAD_B32_L2       the same from 64 regions of 1 MB (L1 misses, L2 hits)
 *   ROCKET_CAL_LOAD_B128_L1/_L2  the two as 16-byte loads
 *   ROCKET_CAL_LOAD_B128_TO_LDS  GB/s of 16-byte buffer loads that write LDS directly (L2 hits)
 *   ROCKET_CAL_LDS_READ_B32      GB/s of 4-byte LDS reads without bank conflicts
 *   ROCKET_CAL_MFMA_F32_4X4X1    TFLOP/s of the 4x4x1 FP32 matrix instruction (all its multiply-adds counted)
 *   ROCKET_CAL_MFMA_VALU_SERIAL  time of matrix wavefronts and vector-FMA wavefronts run together, divided by
 *                                the sum of their times run alone: 1 = the two pipes do not overlap, 0.5 = fully
 *   ROCKET_CAL_STRIP_VALU        TFLOP/s (useful multiply-adds) of the conv strip as the forward kernel forms it
 *                                (32 rows x 64 columns per wavefront, length 9, four channels, max + PPV pooling)
 *   ROCKET_CAL_STRIP_MFMA        the same strip with the multiply-adds as 4x4x1 matrix instructions in Toeplitz
 *                                form (bit-identical outputs): whether the matrix cores would speed the conv up
 * All rates are whole-device.  Takes some tens of milliseconds; allocates and frees 70 MB of device memory and
 * synchronises the stream.  ROCKET_EHIP if the two forms of the strip disagree in any output.
 */
enum {
    ROCKET_CAL_LOAD_B32_L1 = 0, ROCKET_CAL_LOAD_B32_L2 = 1, ROCKET_CAL_LOAD_B128_L1 = 2, ROCKET_CAL_LOAD_B128_L2 = 3,
    ROCKET_CAL_LOAD_B128_TO_LDS = 4, ROCKET_CAL_LDS_READ_B32 = 5, ROCKET_CAL_MFMA_F32_4X4X1 = 6,
    ROCKET_CAL_MFMA_VALU_SERIAL = 7, ROCKET_CAL_STRIP_VALU = 8, ROCKET_CAL_STRIP_MFMA = 9, ROCKET_CAL_COUNT = 10
};
int rocket_calibrate_units(double *out, int32_t count, void *hip_stream);

/*
 * Ridge regressor on the pooled features (paper section 3 part (3), section 3.3):
 * minimises ||y - X w - b||^2 + alpha ||w||^2 over (w, b), the intercept b unpenalised.
 * features_dev: device, n x p float32 row-major (the transform's output for n series);
 * targets_dev: device, n float32; alpha > 0.  coef_dev (device, p doubles) and
 * intercept_dev (device, 1 double) receive w and b.  All arithmetic is fp64 and every sum
 * has a fixed order: a fit is reproducible bit for bit.  The fit solves the n x n dual
 * system (the paper has 677 training examples and p = 20,000), stored densely in the
 * workspace: n <= 32768, ROCKET_EINVAL beyond.  workspace_dev:
 * rocket_ridge_workspace_bytes(n, p) bytes of device memory (0 for sizes the fit rejects),
 * 256-byte aligned.  Asynchronous on hip_stream like the other calls.
 */
size_t rocket_ridge_workspace_bytes(int32_t n, int32_t p);
int rocket_ridge_fit(const float *features_dev, const float *targets_dev, int32_t n, int32_t p, double alpha,
                     double *coef_dev, double *intercept_dev, void *workspace_dev, size_t workspace_bytes,
                     void *hip_stream);

/* Predictions pred_dev[i] = b + features_dev[i] . w for m rows (device pointers; fp64 out). */
int rocket_ridge_predict(const float *features_dev, int32_t m, int32_t p, const double *coef_dev,
                         const double *intercept_dev, double *pred_dev, void *hip_stream);

/*
 * Inference in one call, the use the paper builds the model for (section 4.1: one surface-
 * roughness value per example at line speed; section 3 parts (1)-(3)): transforms a batch and
 * applies a fitted ridge regressor, pred[b] = intercept + sum_i features[b][i] * coef[i].
 * x_dev: device, B x C x L float32 (x_is_u8 = 0) or raw uint8 normalised as in
 * rocket_transform_u8 (x_is_u8 = 1).  coef_dev (F*K doubles) and intercept_dev (1 double) are
 * those of rocket_ridge_fit for the same kernels and feature mask.  features_dev (device,
 * B x F*K float32) receives the features exactly as rocket_transform writes them; pred_dev
 * (device, B doubles) the predictions, exactly as rocket_ridge_predict computes them from
 * those features.  Workspace and errors as for rocket_transform.
 */
int rocket_infer(rocket_kernels *kernels, const void *x_dev, int x_is_u8, int32_t B, uint32_t feature_mask,
                 float lambda, float shift, const double *coef_dev, const double *intercept_dev,
                 float *features_dev, double *pred_dev,
                 void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/*
 * Training the kernel weights through softPPV.  Section 3.2 replaces the step function by a
 * sigmoid so that gradients can flow, and section 6 names training the weights as the thing
 * to try next; these calls are one plain instance of it: the features feed a fixed linear
 * head (coef, intercept, e.g. from rocket_ridge_fit), the loss is the mean squared error of
 * its predictions, and weights and biases move one gradient-descent step.
 *
 * rocket_mse_grad: pred_dev (device, B doubles), targets_dev (device, B float32), coef_dev
 * (device, p doubles) -> grad_out_dev[b*p + i] = (2/B) (pred[b] - y[b]) coef[i] (device,
 * B x p float32, the layout rocket_soft_ppv_backward takes) and, if loss_dev is not NULL,
 * *loss_dev = (1/B) sum_b (pred[b] - y[b])^2 (device, 1 double).  B <= 65535.
 *
 * rocket_sgd_update: w <- w - lr*grad_w, b <- b - lr*grad_b on the handle's device copy of
 * the parameters (grad_w_dev: total_weights float32, grad_b_dev: K float32, as written by
 * rocket_soft_ppv_backward); with recentre != 0 every (kernel, channel) row of weights then has
 * its mean subtracted, which keeps the sampler's invariant of section 3.1.  Nothing is copied
 * to the host: later transforms on the handle use the new parameters, and the next
 * rocket_kernels_view_get (or rocket_kernels_set_params, rocket_kernels_subset) first waits for
 * the device to finish and downloads them.  Updates and transforms of one handle are ordered
 * by the stream they share; an update on a different stream than the previous one first waits
 * for the device.
 *
 * rocket_train_step: transform (feature_mask must contain ROCKET_F_SOFTPPV; the max plane, when
 * present, sends its sub-gradient to its first arg-max, the PPV plane none), prediction, loss
 * gradient, backward pass and update, enqueued on one stream.  x_dev is float32 (x_is_u8 = 0) or
 * raw uint8 (x_is_u8 = 1, normalised as in rocket_transform_u8).  *loss_dev (may be NULL)
 * receives the loss before the update.  workspace_dev: rocket_train_workspace_bytes(kernels, B,
 * mask) bytes, 256-byte aligned.
 */
int rocket_mse_grad(const double *pred_dev, const float *targets_dev, const double *coef_dev, int32_t B, int32_t p,
                    float *grad_out_dev, double *loss_dev, void *hip_stream);
int rocket_sgd_update(rocket_kernels *kernels, const float *grad_w_dev, const float *grad_b_dev, float lr,
                      int recentre, void *hip_stream);
size_t rocket_train_workspace_bytes(const rocket_kernels *kernels, int32_t B, uint32_t feature_mask);
int rocket_train_step(rocket_kernels *kernels, const void *x_dev, int x_is_u8, int32_t B, uint32_t feature_mask,
                      float lambda, float shift, const double *coef_dev, const double *intercept_dev,
                      const float *targets_dev, float lr, int recentre, double *loss_dev,
                      void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/*
 * MINIROCKET-style variant.  The paper describes MINIROCKET in its related-work section only (section 2) and
 * names it as the extension to build next (section 6): two-valued kernels, so that the convolution needs
 * additions only; weights from a predetermined set; biases sampled from the input data; PPV as the only
 * pooled feature.  Everything the paragraph leaves open is this build's reading (parity with the original
 * model is not claimed):
 *
 * rocket_minirocket_kernels: `groups` groups of 84 kernels of length 9.  The 84 are all weight rows with
 * three weights of 2 and six of -1 (zero sum, like the mean-centred weights of section 3.1), in lexicographic
 * order of the positions of the 2s; the same row applies to every channel of the kernel.  A group shares
 * dilation, padding and channel subset, drawn by the laws of section 3.1 from the stream of (seed, group).
 * Biases start at 0.  Host only.  Requires groups, C >= 1 and L >= 9.  K = 84 * groups.
 *
 * rocket_minirocket_fit_bias: kernel k draws, from the stream of (seed + 1, k), one of the B series of x_dev
 * (device, B x C x L float32) and a level q in [0, 1); its bias becomes minus the order statistic of rank
 * floor(q (n - 1)) (0-based, ascending) of its bias-free output on that series, so that on that series
 * PPV = (n - 1 - rank) / n when the outputs are distinct.  Works on any handle.  The biases are written into
 * the handle's device copy; the host copy follows on the next rocket_kernels_view_get (as after
 * rocket_sgd_update).  workspace_dev: rocket_minirocket_fit_workspace_bytes(kernels, B) bytes, 256-byte
 * aligned.  One-time set-up work, not tuned for speed; it synchronises hip_stream once.
 *
 * The features are one PPV per kernel (Eq. 1-2): rocket_transform with feature_mask = ROCKET_F_PPV computes
 * them like those of any other kernels, and
 *
 * rocket_minirocket_transform computes the same features with a kernel made for the predetermined set: the
 * 84 kernels of a group share their channel-summed input and the nine tap values of every position, so that
 * one kernel's output costs one addition and one comparison ("convolution by additions", section 2).
 * x_dev: device, B x C x L float32; out_dev: device, B x K float32, out[b * K + k] = PPV of kernel k.  It
 * evaluates 3 y = U_a + U_b + U_c with U_j = 9 T_j - (T_0 + ... + T_8) in fp32, a different rounding order
 * from rocket_transform's multiply-adds: the two agree except at outputs within rounding of zero.
 * workspace_dev: rocket_minirocket_workspace_bytes(kernels, B) bytes, 256-byte aligned.  Only for handles of
 * rocket_minirocket_kernels whose weights have not been changed since (biases may be: rocket_minirocket_fit_bias,
 * rocket_kernels_set_params with weights = NULL); ROCKET_EINVAL otherwise, and the workspace size is 0.
 * Allocates a few KB of device memory at its first call on a handle.  Asynchronous on hip_stream.
 * rocket_minirocket_transform_u8 is the same from raw 8-bit samples (device, B x C x L uint8), every
 * (series, channel) row z-normalised on the way as in rocket_transform_u8 (sections 4.1, 4.3).
 */
int rocket_minirocket_kernels(uint64_t seed, int32_t groups, int32_t C, int32_t L, rocket_kernels **out);
size_t rocket_minirocket_fit_workspace_bytes(const rocket_kernels *kernels, int32_t B);
int rocket_minirocket_fit_bias(rocket_kernels *kernels, const float *x_dev, int32_t B, uint64_t seed,
                               void *workspace_dev, size_t workspace_bytes, void *hip_stream);
size_t rocket_minirocket_workspace_bytes(const rocket_kernels *kernels, int32_t B);
int rocket_minirocket_transform(rocket_kernels *kernels, const float *x_dev, int32_t B, float *out_dev,
                                void *workspace_dev, size_t workspace_bytes, void *hip_stream);
int rocket_minirocket_transform_u8(rocket_kernels *kernels, const uint8_t *x_u8_dev, int32_t B, float *out_dev,
                                   void *workspace_dev, size_t workspace_bytes, void *hip_stream);
/*
 * The work items of rocket_minirocket_transform, for tests of its plan (host only).  *items points at *count
 * records of 8 int32 {group, mode, first, count, col0, width, rows, 0}, valid while the handle lives.
 * mode 0: output positions [first, first + count) of the group; it stages count + 8 d channel-summed samples.
 * mode 1: rows [first, first + rows) x columns [col0, col0 + width) of the group's output viewed as rows of d
 * positions (position = row * d + column; columns beyond d and positions beyond the output are skipped); it
 * stages (rows + 8) * width samples.  No item stages more than 6,144 samples; width is a multiple of 64.
 * ROCKET_EINVAL if the handle does not hold the predetermined set.
 */
int rocket_minirocket_jobs_view_get(const rocket_kernels *kernels, int32_t *count, const int32_t **items);

/*
 * Pruning (section 6: many of the random kernels are of little use to a given problem and can
 * be dropped by the regressor's feature importance).  Creates a new handle that holds kernels
 * index[0..count) of `kernels` (host array; any order, repeats allowed) with their current
 * parameters.  The choice of which kernels to keep is the caller's.
 */
int rocket_kernels_subset(const rocket_kernels *kernels, const int32_t *index, int32_t count, rocket_kernels **out);

/* Frees a handle and its device mirror; NULL is allowed. */
void rocket_free_kernels(rocket_kernels *kernels);

/* Message of the last error on this thread ("" if none); static storage. */
const char *rocket_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ROCKET_MI355X_H */
