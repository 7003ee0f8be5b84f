/*
 * synk.h - C ABI of libsynk: the data-parallel hot path of Synkhronos
 * (arXiv 1710.04162) as hand-written HIP kernels for AMD MI355X (gfx950).
 *
 * One synchronous-SGD step of the paper (Sec. 3.3) on one GPU, with the N
 * workers of Sec. 3.1-3.2 emulated as N device buffers:
 *
 *   synk_gather_rows        input indexing (Sec. 5.2) + scatter of the index
 *                           list over workers (Sec. 3.2 step 1)
 *   synk_gather_slice, synk_scatter_rows, synk_gather_resident
 *                           the same with a slice for a list, the scatter of an
 *                           array over the workers (Sec. 4.2), and indexing of
 *                           shares that already live on the workers (Sec. 5.2)
 *   synk_sliced_grad, synk_sliced_grad_indexed, synk_sliced_grad_conv,
 *   synk_sliced_grad_conv_indexed
 *                           the gradient function run over every worker's
 *                           share in slices, slice results aggregated on the
 *                           GPU (Sec. 5.1), one flat gradient per worker
 *                           (Sec. 3.3 step 1)
 *   synk_sliced_eval        a function with six outputs, one reduce/gather op
 *                           each (Sec. 3.1), evaluated in slices (Sec. 5.1)
 *   synk_reduce_buffers     reduce/gather of N worker results (Sec. 3.2 step
 *                           3, Sec. 3.3 step 2)
 *   synk_broadcast, synk_all_reduce, synk_all_gather
 *                           the collectives over the N worker copies of a
 *                           variable (Sec. 3.2), incl. the parameter average
 *   synk_sgd_update         momentum update on the flat array (Sec. 3.3 step 3)
 *   synk_reduce_sgd_update  the last two fused into one pass over memory
 *   synk_reduce_update      the same pass with the other update rules of
 *                           Sec. 3.3 (Nesterov momentum, RMSProp, Adam)
 *
 * Conventions common to every call
 * --------------------------------
 * - Returns SYNK_OK (0) or a negative SYNK_ERR_* code; never throws and may be
 *   called from several host threads.  The only state kept between calls is
 *   the pending event pair of synk_profile_next_launch, one per host thread.
 * - All argument checks run on the host BEFORE the first HIP call, so a call
 *   with invalid arguments returns its error code without touching a device.
 * - "device" pointers are device memory owned by the caller and stay owned by
 *   the caller.  "host" pointers (pointer tables, small descriptor arrays) are
 *   read during the call and may be freed when it returns.
 * - The library allocates nothing.  Scratch memory is a caller-provided
 *   workspace (ws, ws_bytes), sized by the matching *_workspace_bytes call,
 *   256-byte aligned; its contents are undefined between calls.  (One entry
 *   point, synk_sliced_eval_static, uses a fixed array of its own instead.)
 * - Kernels are launched asynchronously on `stream` (a hipStream_t passed as
 *   void*; NULL = the default stream).  No call synchronises except
 *   synk_poll_error.  Calls on one stream execute in call order.
 * - At most SYNK_MAX_WORKERS workers / buffers per call.
 * - Splitting `count` data points over `parts` workers or slices always uses
 *   the same rule (Sec. 3.2 asks for shares as equal as they can be and names
 *   no remainder rule): contiguous runs, share i has
 *   count/parts + (i < count%parts ? 1 : 0) points; shares may be empty.
 * - Float results are run-to-run reproducible: no floating-point atomics.
 */
#ifndef SYNK_H
#define SYNK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SYNK_VERSION 100
#define SYNK_MAX_WORKERS 64
#define SYNK_MAX_LAYERS 8
#define SYNK_MAX_CHANNELS 16

/* status codes */
#define SYNK_OK 0
#define SYNK_ERR_NULL (-1)        /* a required pointer is NULL */
#define SYNK_ERR_SHAPE (-2)       /* a size/count is negative, zero where it may not be, or inconsistent */
#define SYNK_ERR_DTYPE (-3)       /* dtype code unknown or not supported by this call */
#define SYNK_ERR_OP (-4)          /* op code unknown or not defined for the dtype */
#define SYNK_ERR_ALIGN (-5)       /* a device pointer is not aligned as documented */
#define SYNK_ERR_WORKSPACE (-6)   /* ws is NULL/misaligned or ws_bytes too small */
#define SYNK_ERR_INDEX (-7)       /* an index was out of range (synk_poll_error) */
#define SYNK_ERR_HIP (-8)         /* a HIP runtime call failed */
#define SYNK_ERR_UNSUPPORTED (-9) /* valid request outside what is implemented */

/* element types */
#define SYNK_U8 0
#define SYNK_I32 1
#define SYNK_F32 2
#define SYNK_BF16 3

/* reduce / gather ops (Sec. 3.1: one per function output) */
#define SYNK_SUM 0
#define SYNK_MEAN 1
#define SYNK_MAX 2
#define SYNK_MIN 3
#define SYNK_PROD 4
#define SYNK_CONCAT 5

/* flags */
#define SYNK_FLAG_CHECK_INDEX 1u /* record out-of-range indexes in ws (see synk_poll_error) */

int synk_version(void);
const char* synk_status_string(int status);

/* For callers that time one kernel: the next launch, on this host thread, of
 * the selected kernel carries the two events (hipEvent_t created with timing
 * enabled, passed as void*): start_event takes the dispatch's begin timestamp
 * and stop_event its end timestamp, so hipEventElapsedTime between them is the
 * kernel's duration without the gaps around it.  Other launches leave the pair
 * pending (also past the end of a call that never launches the selected
 * kernel).  Both NULL cancels a pending pair; exactly one NULL -> ERR_NULL.
 *
 * SYNK_KERNEL_MAIN selects a call's main kernel: the gather kernel of the
 * gather calls, the fused reduce+update kernels, the reduce and collective
 * kernels, stage 1 of synk_sliced_eval, the forward convolution of
 * synk_sliced_grad_conv, the first layer's forward product of
 * synk_sliced_grad.  The other ids select kernels of synk_sliced_grad:
 * the forward product of layer l (1-based), the last layer's kernel (fused
 * head or softmax), the launch that holds dW_L, dW_{L-1} and dZ_{L-2} together
 * (when the shapes allow that grouping), and the weight-gradient or
 * input-gradient product of layer l when it is launched on its own.
 * synk_profile_next_launch(a, b) = synk_profile_next_launch_of(SYNK_KERNEL_MAIN, a, b). */
#define SYNK_KERNEL_MAIN 0
#define SYNK_KERNEL_MLP_HEAD 1
#define SYNK_KERNEL_MLP_BACKWARD_GROUP 2
#define SYNK_KERNEL_MLP_FORWARD(l) (16 + (l))
#define SYNK_KERNEL_MLP_DW(l) (32 + (l))
#define SYNK_KERNEL_MLP_DX(l) (48 + (l))
int synk_profile_next_launch(void* start_event, void* stop_event);
int synk_profile_next_launch_of(int kernel, void* start_event, void* stop_event);
/* 1 while a pair handed in on this host thread has not been attached to a launch yet, else 0. */
int synk_profile_pending(void);

/* Measured peaks for the rooflines a caller reports (timing kernels only; nothing of
 * the method).  Launches one probe on `stream`; *work receives what the launch
 * does (flops or bytes), to be divided by the launch's duration, e.g. taken with
 * synk_profile_next_launch.
 *   SYNK_PROBE_MFMA_BF16  512 workgroups of 8 wavefronts, each iters x 4 32x32x16
 *                         bf16 MFMAs on registers; buf: >= 4 bytes (never written
 *                         in practice)
 *   SYNK_PROBE_FILL       buf_bytes of 16-byte stores, one per thread, in address
 *                         order
 *   SYNK_PROBE_LDS_FETCH  256 workgroups, each bringing iters (<= 48) tiles of 128
 *                         rows x 128 bytes (row pitch 6 KB) from buf straight into
 *                         LDS; buf_bytes >= 768 KB, read only
 *   SYNK_PROBE_READ       floor(buf_bytes / 32 KB) workgroups, each loading 32 KB in
 *                         address order with 16-byte loads (eight per thread, all
 *                         issued before the first use); buf: read only unless the
 *                         XOR of a workgroup's words is 0x9e3779b9 (fill it with
 *                         one repeated value); iters ignored
 *   SYNK_PROBE_MFMA_BESIDE_VALU + n (n = 0, 1, 2, 4, 6, 8, 12) and
 *   SYNK_PROBE_MFMA_BESIDE_LDS + n (n = 1, 2, 4)
 *                         256 workgroups of 4 wavefronts (one per SIMD), each doing
 *                         2 * iters bf16 32x32x16 MFMAs (two independent sums) with n
 *                         vector-ALU additions, or n 4-byte LDS reads, after every
 *                         MFMA: launch time / (2 * iters) is the time per MFMA with
 *                         that much other work of the same wavefront beside it;
 *                         buf_bytes >= 4, never written in practice; other n ->
 *                         ERR_UNSUPPORTED
 * buf: device, 16-byte aligned.  Errors: NULL -> ERR_NULL; iters < 1, alignment ->
 * ERR_SHAPE; buffer too small -> ERR_WORKSPACE; unknown probe -> ERR_UNSUPPORTED. */
#define SYNK_PROBE_MFMA_BF16 0
#define SYNK_PROBE_FILL 1
#define SYNK_PROBE_LDS_FETCH 2
#define SYNK_PROBE_READ 3
#define SYNK_PROBE_MFMA_BESIDE_VALU 16
#define SYNK_PROBE_MFMA_BESIDE_LDS 32
int synk_probe_launch(int probe, void* buf, size_t buf_bytes, int iters, double* work, void* stream);

/* Host-side helper: the split rule above.  Writes parts+1 offsets
 * (start[0] = 0, start[parts] = count) into `start` (host). */
int synk_split(int64_t count, int parts, int64_t* start);

/* ------------------------------------------------------------------ gather
 * Input indexing, Sec. 5.2: the minibatch is data[idx[0..n_idx)], duplicates
 * allowed; Sec. 3.2 step 1: the index list is split over n_workers by the
 * split rule and worker w receives its rows, in list order, densely packed in
 * dst[w] ([share_w x row_elems], row-major).
 *
 *   data        device, [n_rows x row_elems] of src_dtype, row-major, dense
 *   idx         device, int32[n_idx], each in [0, n_rows)
 *   dst         host array[n_workers] of device pointers, each large enough
 *               for its share; dst[w] may be NULL only if share w is empty
 *   dst_dtype   == src_dtype: bit-exact copy (any dtype);
 *               SYNK_BF16 from SYNK_F32: round-to-nearest-even;
 *               SYNK_F32 from SYNK_U8: out = lut[c*256 + x] with channel
 *               c = element_index / (row_elems/channels): needs `lut`
 *               (device float[channels*256], see synk_build_norm_lut) and
 *               row_elems % channels == 0, channels <= SYNK_MAX_CHANNELS
 *   labels      device int32[n_rows] or NULL; if given, dst_labels is a host
 *               array[n_workers] of device int32 buffers receiving
 *               labels[idx[j]] in the same order
 *   flags       SYNK_FLAG_CHECK_INDEX: needs ws of
 *               synk_gather_workspace_bytes(); whether this call met an
 *               out-of-range index is recorded there.  With or without the flag a row whose index
 *               is out of range is skipped (its destination is left
 *               untouched) rather than read out of bounds.
 * Alignment: none required; 16-byte aligned data/dst and a row pitch that is
 * a multiple of 16 bytes select the widest copy path.
 * Errors: NULL -> ERR_NULL; n_rows<0, row_elems<=0, n_idx<0, n_workers out of
 * [1,SYNK_MAX_WORKERS], row_elems%channels -> ERR_SHAPE; dtype pair not
 * listed -> ERR_DTYPE; flag set with no/small ws -> ERR_WORKSPACE.
 * n_idx == 0 is a no-op.
 */
size_t synk_gather_workspace_bytes(void);
int synk_gather_rows(const void* data, int64_t n_rows, int64_t row_elems, int src_dtype,
                     const int32_t* idx, int64_t n_idx,
                     void* const* dst, int n_workers, int dst_dtype,
                     const float* lut, int channels,
                     const int32_t* labels, int32_t* const* dst_labels,
                     uint32_t flags, void* ws, size_t ws_bytes, void* stream);

/* The same gather with the index list given as a slice (Sec. 5.2 allows
 * either form of indexes): row j of the minibatch is
 * data[start + j*step], j < ceil((stop-start)/step), step >= 1,
 * 0 <= start <= stop <= n_rows; the list is split over the workers as above.
 * Errors as synk_gather_rows; step < 1 -> ERR_SHAPE; start/stop outside the
 * stated range -> ERR_INDEX (nothing is launched). */
int synk_gather_slice(const void* data, int64_t n_rows, int64_t row_elems, int src_dtype,
                      int64_t start, int64_t stop, int64_t step,
                      void* const* dst, int n_workers, int dst_dtype,
                      const float* lut, int channels,
                      const int32_t* labels, int32_t* const* dst_labels, void* stream);

/* The "scatter" collective (Sec. 4.2): an array is divided over the workers'
 * memories by its first dimension, shares as equal as possible, in order:
 * dst[w] receives rows [start_w, start_w + size_w) of data (split rule),
 * bit-exact, and dst_labels[w] the matching labels when labels != NULL.
 * Equals synk_gather_slice(0, n_rows, 1) with dst_dtype == dtype. */
int synk_scatter_rows(const void* data, int64_t n_rows, int64_t row_elems, int dtype,
                      void* const* dst, int n_workers,
                      const int32_t* labels, int32_t* const* dst_labels, void* stream);

/* Input indexing of data that already lives on the workers (Sec. 5.2: every
 * device may be given its own index list, or all of them the same one):
 * worker w excerpts rows idx[w][0..n_idx[w]) of its own
 * share shares[w] ([share_rows[w] x row_elems]) into dst[w], in list order.
 * shares, share_rows, idx, n_idx, dst, labels, dst_labels: host arrays of
 * n_workers entries (idx[w], shares[w], labels[w] device pointers; pass the
 * same idx pointer n times to apply one list everywhere).  A worker with
 * n_idx[w] == 0 is skipped and may have NULL pointers.  dtype pairs, lut,
 * flags/ws and out-of-range handling as in synk_gather_rows; the error word
 * collects over all workers.  One launch for all workers; a share holds
 * fewer than 2^31 rows. */
int synk_gather_resident(const void* const* shares, const int64_t* share_rows, int64_t row_elems,
                         int src_dtype, const int32_t* const* idx, const int64_t* n_idx,
                         void* const* dst, int n_workers, int dst_dtype,
                         const float* lut, int channels,
                         const int32_t* const* labels, int32_t* const* dst_labels,
                         uint32_t flags, void* ws, size_t ws_bytes, void* stream);

/* Builds on the device the table used by the U8->F32 gather:
 * lut[c*256 + x] = (float)(((double)x - (double)mean[c]) / (double)std[c]),
 * i.e. the float64 quotient rounded once to float32.  mean, std: host
 * float[channels] on the 0..255 scale, std != 0; lut: device
 * float[channels*256]. */
int synk_build_norm_lut(const float* mean, const float* std, int channels, float* lut, void* stream);

/* Synchronises `stream`, reads and clears the error word the most recent call
 * with SYNK_FLAG_CHECK_INDEX left in ws.  Returns SYNK_OK, SYNK_ERR_INDEX, or
 * SYNK_ERR_HIP. */
int synk_poll_error(void* ws, void* stream);

/* ------------------------------------------------------------- sliced grad
 * The gradient function of synchronous SGD (Sec. 3.3 step 1) for a ReLU MLP
 * with softmax cross-entropy, called the way Sec. 3.2 and 5.1 describe: every
 * worker runs it on its own rows, cut into n_slices slices by the split rule;
 * all slices see the same parameter values (Sec. 5.1: updates are applied
 * once, afterwards); a worker's slice results are aggregated on the GPU with
 * grad_op and land in that worker's own flat gradient array and loss.
 *
 * Function on a row set R: h_0 = X_R; h_l = relu(h_{l-1} W_l + b_l) for
 * l < L; logits = h_{L-1} W_L + b_L; l_i = logsumexp(logits_i) -
 * logits_i[y_i]; outputs loss_R = mean_i l_i and g_R = d loss_R / d params.
 * relu'(0) = 0.  Aggregation over a worker's slices s with |R_s| rows:
 *   SYNK_MEAN  sum_s (|R_s|/|R_w|) out_s  (= the unsliced call on the share)
 *   SYNK_SUM   sum_s out_s
 *
 *   m.dims          host int64[n_layers+1]: d_0 (features) .. d_L (classes)
 *   m.compute_dtype SYNK_F32: fp32 GEMM operands; SYNK_BF16: X, W_l, hidden
 *                   activations and dZ_l are rounded (nearest-even) to bf16
 *                   where they enter a GEMM, products accumulate in fp32,
 *                   everything else is fp32
 *   params          device float[P], P = sum_l d_{l-1} d_l + d_l, layout
 *                   W_1, b_1, W_2, b_2, ...; W_l is [d_{l-1} x d_l] row-major
 *   params_lp       device bf16[P], the same array rounded to bf16 (as
 *                   written by synk_sgd_update / synk_cast_bf16); required
 *                   for SYNK_BF16, ignored for SYNK_F32
 *   x               host array[n_workers] of device [rows[w] x d_0] buffers
 *                   in compute_dtype (as written by synk_gather_rows)
 *   y               host array[n_workers] of device int32[rows[w]], each in
 *                   [0, d_L); a label outside that range contributes as if no
 *                   class were the target (never reads out of bounds)
 *   rows            host int64[n_workers], >= 0, not all zero; rows and layer
 *                   widths are limited to 2^21 each
 *   grad            host array[n_workers] of device float[P]; fully
 *                   overwritten (a worker with no rows gets zeros)
 *   loss            device float[n_workers]
 *   ws              synk_sliced_grad_workspace_bytes(m, rows, n_workers, &b).
 *                   All slices are evaluated in one pass, every row carrying
 *                   the weight its slice has under grad_op, so the workspace
 *                   holds the activations of ALL rows of all workers:
 *                   n_slices changes the aggregation (and, for SYNK_SUM, the
 *                   weights), not the workspace size; the memory-bounding
 *                   effect slicing has in Sec. 5.1 is not reproduced.
 * Errors: NULL -> ERR_NULL; n_layers out of [1,SYNK_MAX_LAYERS], dims <= 0,
 * rows < 0, all rows zero, n_workers out of range, n_slices <= 0 -> ERR_SHAPE;
 * compute_dtype -> ERR_DTYPE; grad_op not SUM/MEAN -> ERR_OP; params, x[w] or
 * grad[w] not 4-byte (F32) / 2-byte (BF16) aligned -> ERR_ALIGN; ws ->
 * ERR_WORKSPACE.  16-byte aligned x[w], grad[w], params, params_lp and layer
 * widths that are multiples of 8 select the vector load paths.
 */
typedef struct {
  int n_layers;
  const int64_t* dims;
  int compute_dtype;
} synk_mlp_desc;

int synk_mlp_param_count(const synk_mlp_desc* m, int64_t* count);
int synk_sliced_grad_workspace_bytes(const synk_mlp_desc* m, const int64_t* rows, int n_workers,
                                     size_t* bytes);
int synk_sliced_grad(const synk_mlp_desc* m, const float* params, const void* params_lp,
                     const void* const* x, const int32_t* const* y, const int64_t* rows,
                     int n_workers, int n_slices, int grad_op,
                     float* const* grad, float* loss,
                     void* ws, size_t ws_bytes, void* stream);

/* synk_sliced_grad with the input indexing folded in (Sec. 5.2: the data lives on
 * the device and a call names the rows it uses; Sec. 3.2 step 1; Sec. 3.3 step 1):
 * the minibatch is data[idx[0..n_idx)], split over n_workers by the split rule
 * exactly as synk_gather_rows splits it, and the result equals
 * synk_gather_rows(data, idx -> x, labels -> y) followed by synk_sliced_grad on
 * those x, y and shares, bit for bit.  The workers' rows and labels are kept in the
 * workspace.  Where the first forward product's kernel can read its rows through
 * the index (bf16: shares that are whole 64-row tiles, d0 a multiple of 64, widths
 * multiples of 64, 16-byte aligned data; fp32: the small-batch kernel) no gather
 * launch takes place: that kernel also leaves the rows behind for the weight
 * gradient; otherwise the call runs the gather itself first.
 *   data      device, [n_data x d0] in compute_dtype (for SYNK_BF16 the dataset is
 *             held in bf16: cast it once with synk_cast_bf16), row-major, dense
 *   labels    device int32[n_data]
 *   idx       device int32[n_idx], each in [0, n_data); an index outside the
 *             range never reads out of bounds (the fused kernels read row 0 for
 *             it, the gather launch leaves the row's previous workspace contents);
 *             validate lists with synk_gather_rows + SYNK_FLAG_CHECK_INDEX
 *   ws        synk_sliced_grad_indexed_workspace_bytes(m, n_idx, n_workers, &b)
 * params, params_lp, n_slices, grad_op, grad, loss: as synk_sliced_grad.
 * SYNK_KERNEL_MAIN selects the first forward product (never the gather launch).
 * Errors: as synk_sliced_grad; n_idx < 1, n_data < 1 -> ERR_SHAPE. */
int synk_sliced_grad_indexed_workspace_bytes(const synk_mlp_desc* m, int64_t n_idx, int n_workers,
                                             size_t* bytes);
int synk_sliced_grad_indexed(const synk_mlp_desc* m, const float* params, const void* params_lp,
                             const void* data, const int32_t* labels, int64_t n_data,
                             const int32_t* idx, int64_t n_idx,
                             int n_workers, int n_slices, int grad_op,
                             float* const* grad, float* loss,
                             void* ws, size_t ws_bytes, void* stream);

/* A second function for the same sliced call (Sec. 3.2, 5.1; Sec. 3.3 step 1):
 * one block of the network family the scaling study trains (Sec. 6), a 3x3
 * convolution + batch normalisation + ReLU, closed the way that network ends
 * (global average pool, one affine layer, softmax cross-entropy).
 *
 * Function on an image set R (n images, each H x W x C_in, channels last, i.e.
 * a row of H*W*C_in values as synk_gather_rows writes it):
 *   z = conv3x3(X, Wc), stride 1, zero padding 1, no bias;
 *   mu_c, var_c = mean and biased variance of z[..., c] over all n*H*W positions
 *   of R;  xhat = (z - mu) / sqrt(var + eps);  a = relu(gamma * xhat + beta);
 *   p_i = mean of a_i over its H*W positions;  logits = p Wf + bf;
 *   l_i = logsumexp(logits_i) - logits_i[y_i];  loss_R = mean_i l_i;
 *   g_R = d loss_R / d params.  relu'(0) = 0.
 * Every slice is one call of the function (Sec. 5.1), so mu and var are those
 * of the slice; aggregation over a worker's slices as in synk_sliced_grad
 * (SYNK_MEAN: weights |R_s|/|R_w|; SYNK_SUM).  All slices see the same
 * parameter values.
 *
 *   d.compute_dtype SYNK_F32: fp32 throughout; SYNK_BF16: X, Wc and dz are
 *                   rounded (nearest-even) to bf16 where they enter a
 *                   contraction, products accumulate in fp32, and the
 *                   convolution's output z is stored in bf16 (statistics and
 *                   normalisation read the rounded z); the arithmetic of the
 *                   statistics, normalisation, pooling, the affine layer and
 *                   the loss is fp32 in both modes
 *   params          device float[P]: Wc [3 x 3 x C_in x C_out] (tap-major: the
 *                   [9 C_in x C_out] matrix of the convolution written as a
 *                   product), gamma [C_out], beta [C_out], Wf [C_out x
 *                   classes] row-major, bf [classes]; 16-byte aligned
 *   x               host array[n_workers] of device [rows[w] x H*W*C_in]
 *                   buffers in compute_dtype, 16-byte aligned
 *   y               host array[n_workers] of device int32[rows[w]]; a label
 *                   outside [0, classes) contributes as if no class were the
 *                   target (never reads out of bounds)
 *   rows            host int64[n_workers] images per worker, >= 0, not all 0
 *   grad            host array[n_workers] of device float[P], 16-byte aligned;
 *                   fully overwritten (a worker with no images gets zeros)
 *   loss            device float[n_workers]
 *   ws              synk_sliced_grad_conv_workspace_bytes(...)
 * Limits: C_in and C_out multiples of 8, C_out <= 512, classes <= 4096, H, W,
 * C_in <= 4096, n_workers * n_slices <= 65535, total pixels (images * H * W)
 * below 2^29.
 * Errors: NULL -> ERR_NULL; limits, rows < 0, all rows zero, n_workers out of
 * range, n_slices <= 0, eps < 0 -> ERR_SHAPE; compute_dtype -> ERR_DTYPE;
 * grad_op not SUM/MEAN -> ERR_OP; alignment -> ERR_ALIGN; ws -> ERR_WORKSPACE.
 */
typedef struct {
  int height, width, c_in, c_out, classes;
  int compute_dtype;
  float eps;
} synk_convblock_desc;

int synk_convblock_param_count(const synk_convblock_desc* d, int64_t* count);
int synk_sliced_grad_conv_workspace_bytes(const synk_convblock_desc* d, const int64_t* rows,
                                          int n_workers, int n_slices, size_t* bytes);
int synk_sliced_grad_conv(const synk_convblock_desc* d, const float* params,
                          const void* const* x, const int32_t* const* y, const int64_t* rows,
                          int n_workers, int n_slices, int grad_op,
                          float* const* grad, float* loss,
                          void* ws, size_t ws_bytes, void* stream);

/* synk_sliced_grad_conv with the input indexing folded in, as synk_sliced_grad_indexed is
 * for the MLP (Sec. 5.2; Sec. 3.2 step 1): the minibatch is data[idx[0..n_idx)], split over
 * n_workers by the split rule, and the result equals synk_gather_rows followed by
 * synk_sliced_grad_conv bit for bit.  Where both convolution kernels can read an image
 * through the index list (compute_dtype SYNK_BF16, C_in a multiple of 64, 31 <= W <= 61) no
 * gather takes place and no copy of the images is made; otherwise the call gathers into its
 * workspace first.
 *   data    device, [n_data x H*W*C_in] in compute_dtype, channels last, 16-byte aligned
 *   labels  device int32[n_data];  idx: device int32[n_idx], each in [0, n_data) (an index
 *           outside reads row 0 in the kernels that read through the list)
 *   ws      synk_sliced_grad_conv_indexed_workspace_bytes(d, n_idx, n_workers, n_slices, &b)
 * Other arguments, limits and errors as synk_sliced_grad_conv; n_idx < 1, n_data < 1 ->
 * ERR_SHAPE. */
int synk_sliced_grad_conv_indexed_workspace_bytes(const synk_convblock_desc* d, int64_t n_idx,
                                                  int n_workers, int n_slices, size_t* bytes);
int synk_sliced_grad_conv_indexed(const synk_convblock_desc* d, const float* params,
                                  const void* data, const int32_t* labels, int64_t n_data,
                                  const int32_t* idx, int64_t n_idx,
                                  int n_workers, int n_slices, int grad_op,
                                  float* const* grad, float* loss,
                                  void* ws, size_t ws_bytes, void* stream);

/* out[i] = bf16(in[i]), round-to-nearest-even; device float[len] -> device
 * bf16[len].  Makes the params_lp array for a first step. */
int synk_cast_bf16(const float* in, void* out, int64_t len, void* stream);

/* ------------------------------------------------------------- sliced eval
 * A function with six outputs, each with its own reduce/gather op (Sec. 3.1),
 * evaluated over n_slices contiguous slices of the rows (split rule) whose
 * results are aggregated on the GPU (Sec. 5.1).  With a_i = argmax_c
 * logits[i,c] (lowest c on ties):
 *   ce_sum       float[1]      sum_i logsumexp(logits_i) - logits_i[y_i]  SUM
 *   class_counts int32[classes] #{i : a_i = c}                            SUM
 *   max_logit    float[1]      max over all entries                       MAX
 *   min_logit    float[1]      min over all entries                       MIN
 *   n_correct    int32[1]      #{i : a_i = y_i}                           SUM
 *   argmax       int32[rows]   a_i                                        CONCAT
 * logits: device float[rows x classes] row-major; labels: device int32[rows]
 * (a label outside [0,classes) adds only the logsumexp term and never counts
 * as correct).  Inputs must be finite (other input never faults: a row of
 * -inf only counts as class 0, a row of NaN as some class in range).  All
 * outputs are device pointers and are fully overwritten.  rows >= 1, classes in [1, 4096], n_slices >= 1.
 */
int synk_sliced_eval_workspace_bytes(int64_t rows, int64_t classes, int n_slices, size_t* bytes);
int synk_sliced_eval(const float* logits, const int32_t* labels, int64_t rows, int64_t classes,
                     int n_slices,
                     float* ce_sum, int32_t* class_counts, float* max_logit, float* min_logit,
                     int32_t* n_correct, int32_t* argmax,
                     void* ws, size_t ws_bytes, void* stream);

/* synk_sliced_eval for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid it): the same
 * computation, kernels and results, with the per-(slice, chunk) partial results
 * kept in a fixed array inside the library's device image instead of a
 * caller's workspace.  The call allocates and frees nothing and calls no
 * allocating routine; the caller still passes inputs and outputs.
 *   Limit: synk_sliced_eval_workspace_bytes(rows, classes, n_slices) must not
 *   exceed SYNK_SLICED_EVAL_STATIC_BYTES (1 MiB: e.g. 65,536 rows in 64 slices
 *   takes 128 KiB; about 520,000 rows fit); beyond it -> ERR_WORKSPACE and
 *   nothing is launched.  Each GPU the library runs on holds its own copy of
 *   the array until the process ends.
 *   Sharing: every call on a GPU uses that GPU's one array, which keeps the last
 *   call's contents (nothing needs clearing: stage 1 rewrites every entry
 *   stage 2 reads).  Calls that overlap in time on one GPU (different streams
 *   or host threads) race on it: serialise them, or use synk_sliced_eval with
 *   separate workspaces.
 *   synk_static_scratch_init resolves the array's address for the CURRENT device
 *   (once per device; the entry point does the same on its first call on a
 *   device).  Call it before capturing the entry point into a graph.
 * Other arguments, outputs and errors as synk_sliced_eval. */
#define SYNK_SLICED_EVAL_STATIC_BYTES (1u << 20)
int synk_static_scratch_init(void);
int synk_sliced_eval_static(const float* logits, const int32_t* labels, int64_t rows, int64_t classes,
                            int n_slices,
                            float* ce_sum, int32_t* class_counts, float* max_logit, float* min_logit,
                            int32_t* n_correct, int32_t* argmax, void* stream);

/* ------------------------------------------------------------------ reduce
 * Reduce or gather N equally long worker results (Sec. 3.2 step 3; Sec. 3.3
 * step 2 for the flat gradient): out[i] = op_w bufs[w][i].
 *   bufs     host array[n] of device buffers of `dtype` (F32 or I32)
 *   op       SUM, MAX, MIN, PROD: folded in buffer order;
 *            MEAN (F32 only): sum_w weights[w]*bufs[w][i], weights = 1/n when
 *            NULL (host float[n] otherwise);
 *            CONCAT: out = bufs[0] ++ bufs[1] ++ ..., buffer w having lens[w]
 *            elements (host int64[n]; `len` is ignored)
 *   out      device, len elements (CONCAT: sum of lens); may alias bufs[0]
 *            except for CONCAT
 * Errors: MEAN on I32 -> ERR_OP; weights with an op other than MEAN ->
 * ERR_OP; CONCAT without lens -> ERR_NULL; n out of [1,SYNK_MAX_WORKERS],
 * len < 0 -> ERR_SHAPE.  len == 0 is a no-op.
 */
int synk_reduce_buffers(const void* const* bufs, int n, int64_t len, int dtype, int op,
                        const float* weights, const int64_t* lens, void* out, void* stream);

/* ------------------------------------------------------------- collectives
 * The collectives over the N worker copies of a variable (Sec. 3.2, the
 * part on shared variables, which lists broadcast and all-reduce among its
 * collectives; App. A: averaging the parameters over the workers).  Reduce-
 * to-one and gather-to-one are synk_reduce_buffers.  Elements are 4 bytes
 * (SYNK_F32 or SYNK_I32); pointer tables, lens and weights are host arrays
 * read during the call, the buffers device memory, 4-byte aligned (16-byte
 * alignment of every buffer selects the vector path).
 *
 * synk_broadcast: dsts[w][i] = src[i], i < len, for each of the n workers.
 *   src must not overlap a destination (src == dsts[w] itself is allowed).
 * synk_all_reduce: in place; every bufs[w][i] becomes the fold, in worker
 *   order, of bufs[0..n)[i] under op (SUM, MEAN, MAX, MIN, PROD; MEAN takes
 *   optional weights, default 1/n, and is the parameter / gradient average).
 *   The n buffers must be distinct and must not overlap.
 * synk_all_gather: every dsts[w] (length sum of lens) receives the
 *   concatenation of srcs[0..n) in worker order; srcs[w] has lens[w] >= 0
 *   elements.  A source may be the matching segment of its own destination.
 * Errors: NULL -> ERR_NULL; n out of [1,SYNK_MAX_WORKERS], negative length,
 * repeated buffer in all_reduce -> ERR_SHAPE; dtype -> ERR_DTYPE; op (CONCAT,
 * MEAN on I32, weights without MEAN) -> ERR_OP; alignment -> ERR_ALIGN.  A
 * call with nothing to move returns SYNK_OK without a launch.
 */
int synk_broadcast(const void* src, void* const* dsts, int n, int64_t len, int dtype, void* stream);
int synk_all_reduce(void* const* bufs, int n, int64_t len, int dtype, int op, const float* weights,
                    void* stream);
int synk_all_gather(const void* const* srcs, const int64_t* lens, int n, int dtype, void* const* dsts,
                    void* stream);

/* ------------------------------------------------------------------ update
 * Momentum update with the combined gradient (Sec. 3.3 step 3; the paper
 * names the rule, the formula is this library's reading):
 *   g = G[i] + weight_decay * p[i];  v[i] = momentum * v[i] - lr * g;
 *   p[i] = p[i] + v[i];  if p_lp: p_lp[i] = bf16(p[i]) (nearest-even)
 * p, v: device float[len], updated in place; g: device float[len];
 * p_lp: device bf16[len] or NULL.
 */
int synk_sgd_update(float* p, float* v, const float* g, int64_t len,
                    float lr, float momentum, float weight_decay, void* p_lp, void* stream);

/* Sec. 3.3 steps 2 and 3 in one pass: G[i] = sum_w weights[w]*grads[w][i]
 * (weights NULL = 1/n), then the update above; G is never written to memory.
 * Optionally also the mean of the per-worker scalar losses (Sec. 3.2 step 3):
 * loss_out[0] = sum_w weights[w]*loss_in[w] (both device; both NULL to skip).
 * Same results as synk_reduce_buffers(MEAN) followed by synk_sgd_update. */
int synk_reduce_sgd_update(const float* const* grads, int n, int64_t len, const float* weights,
                           float* p, float* v, float lr, float momentum, float weight_decay,
                           void* p_lp, const float* loss_in, float* loss_out, void* stream);

/* The other update rules the paper lists for its synchronous-SGD helpers
 * (Sec. 3.3: momentum, Nesterov momentum, RMSProp, Adam), fused with the
 * N-buffer average exactly like synk_reduce_sgd_update.  The paper gives no
 * formulas; these are the published forms, with g = G[i] + weight_decay*p[i]:
 *   SYNK_RULE_MOMENTUM  s1 = momentum*s1 - lr*g;  p += s1
 *   SYNK_RULE_NESTEROV  s1 = momentum*s1 - lr*g;  p += momentum*s1 - lr*g
 *   SYNK_RULE_RMSPROP   s1 = rho*s1 + (1-rho)*g*g;  p -= lr*g / sqrt(s1 + eps)
 *   SYNK_RULE_ADAM      s1 = beta1*s1 + (1-beta1)*g;  s2 = beta2*s2 + (1-beta2)*g*g;
 *                       p -= lr*sqrt(1-beta2^step)/(1-beta1^step) * s1 / (sqrt(s2) + eps)
 * u: host; `step` is the number of this update (1 for the first; ADAM only).
 * p, s1, s2: device float[len], updated in place, 16-byte aligned; s2 is
 * required for ADAM and ignored otherwise.  grads, weights, p_lp, loss_in,
 * loss_out as in synk_reduce_sgd_update.  All arithmetic in fp32; the ADAM
 * step size is formed on the host in double and rounded once.
 * Errors: NULL -> ERR_NULL; unknown rule -> ERR_OP; n or len out of range,
 * ADAM with step < 1 or a beta outside [0,1) -> ERR_SHAPE; alignment ->
 * ERR_ALIGN. */
#define SYNK_RULE_MOMENTUM 0
#define SYNK_RULE_NESTEROV 1
#define SYNK_RULE_RMSPROP 2
#define SYNK_RULE_ADAM 3
typedef struct {
  int rule;
  float lr;
  float momentum;     /* MOMENTUM, NESTEROV */
  float rho;          /* RMSPROP */
  float beta1, beta2; /* ADAM */
  float eps;          /* RMSPROP, ADAM */
  float weight_decay;
  int64_t step;       /* ADAM: 1, 2, ... */
} synk_update_desc;
int synk_reduce_update(const synk_update_desc* u, const float* const* grads, int n, int64_t len,
                       const float* weights, float* p, float* s1, float* s2, void* p_lp,
                       const float* loss_in, float* loss_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SYNK_H */
