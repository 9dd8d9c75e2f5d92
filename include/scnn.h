/*
 * scnn.h -- C ABI of the MI355X (gfx950) forward sparse convolution layer with
 * attention, after Hackel et al., "Inference, Learning and Attention Mechanisms
 * that Exploit and Preserve Sparsity in CNNs".
 *
 * Data model (Sec. 3 of the paper: a sparse tensor is a coordinate list plus
 * values, sorted so that memory access coalesces).  This library stores one row
 * per occupied site with a channel vector:
 *
 *   coords  int32 [rows, 1+ndim]   (b, c_1 .. c_ndim); rows unique and sorted
 *                                  ascending by (b, lin); lin is the row-major
 *                                  site index, last coordinate fastest
 *   feats   fp32  [rows, C]        row-major; exact 0.0f means "entry absent"
 *   filter  fp32  [T, C_in, C_out] T = prod(ksize); tap t is row-major over
 *                                  (delta_1..delta_ndim) + h, h = (ksize-1)/2;
 *                                  exact 0.0f means "weight pruned"
 *
 * Pointers.  `extent` and `ksize` are HOST pointers (ndim int32 each).  Every
 * other array pointer is a DEVICE pointer owned by the caller.  The library
 * allocates no device memory: scratch comes from the caller's `workspace`
 * (device, 256-byte aligned), sized by the matching *_workspace() query.
 *
 * Execution.  All work is enqueued on `hip_stream` (a hipStream_t passed as
 * void*; NULL = the default stream).  No call synchronises with the host.
 *
 * Result counters.  `nnz_out` points to SCNN_NNZ_LEN device int64 values:
 *   [0] rows produced (the true count, even when it exceeds out_capacity;
 *       rows beyond out_capacity are not written)
 *   [1] number of candidate output sites examined (conv) / input rows (others)
 *   [2] status bits, see SCNN_FLAG_*; 0 = fine
 *   [3] notes, not errors: 1 = the attention step found some column's k-th
 *       strongest response outside the bracket it had estimated from a sample
 *       of the column and settled that column from the whole column instead
 *       (same result, more time); else 0
 * The caller reads them after its own synchronisation.
 *
 * Return value: SCNN_OK or a negative SCNN_E* code; scnn_last_error() gives a
 * host string for the calling thread's last failure.  No exception crosses
 * this boundary.  Preconditions that are not checked on the host (sorted,
 * unique, in-range coordinates; finite values) are reported through the
 * status bits where the kernels can see them cheaply.  With
 * SCNN_FLAG_BAD_COORD or SCNN_FLAG_UNSORTED set the results of the call are
 * undefined (a row with an out-of-range coordinate is never used as an
 * address, but the rows that share its 64-site bitmap word are then looked up
 * one row off); every access stays inside the caller's arrays.
 */
#ifndef SCNN_H_
#define SCNN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SCNN_OK 0
#define SCNN_EINVAL (-1)     /* null pointer, ndim not 2/3, even or zero filter size, C <= 0, rho_up not in [0,1], ... */
#define SCNN_ECAPACITY (-2)  /* a size does not fit the library's 31-bit row / site indices */
#define SCNN_EWORKSPACE (-3) /* workspace_bytes smaller than the query's answer, or workspace misaligned */
#define SCNN_EUNSORTED (-4)  /* only from scnn_validate_rows */
#define SCNN_EHIP (-5)       /* a HIP call or kernel launch failed */

#define SCNN_NNZ_LEN 4
#define SCNN_FLAG_CAND_OVERFLOW 1u /* more candidate sites than cand_capacity: output is empty */
#define SCNN_FLAG_OUT_OVERFLOW 2u  /* more output rows than out_capacity: output truncated */
#define SCNN_FLAG_BAD_COORD 4u     /* an input row had a coordinate outside the grid: row skipped */
#define SCNN_FLAG_UNSORTED 8u      /* input rows not strictly ascending by (b, lin): result undefined */
#define SCNN_FLAG_INTERNAL 16u     /* a bounded device-side wait ran out: result invalid (should never happen) */

#define SCNN_TOPK_ABS 0    /* keep the k responses of largest magnitude (Sec. 3.2, second variant) */
#define SCNN_TOPK_SIGNED 1 /* keep the k largest raw responses       (Sec. 3.2, first variant)  */

#define SCNN_FUSE_RELU 1u     /* sparse ReLU after the selection */
#define SCNN_FUSE_MAXPOOL2 2u /* then sparse max-pooling, window = stride = 2 (Sec. 3.3) */

const char* scnn_last_error(void);
int scnn_version(void);

/* k of the k-selection from the density bound rho_up (Sec. 1, Sec. 3.2: at
 * most rho_up of the n_sites sites of one channel of one sample stay non-zero).
 * floor(rho_up * n_sites), except that a product within 1e-9 (relative) of an
 * integer counts as that integer; clamped to [0, n_sites].  Host only. */
int64_t scnn_k_from_rho(double rho_up, int64_t n_sites);

/* Upper bound on the number of candidate output sites of a convolution:
 * min(batch * prod(extent), nnz_in * prod(ksize)).  Host only; < 0 on error. */
int64_t sparse_conv_fwd_max_rows(int ndim, const int32_t* extent, int batch, int64_t nnz_in, const int32_t* ksize);

/* Bytes of workspace sparse_conv_fwd needs for these sizes.  cand_capacity <= 0
 * means the bound above.  Host only; 0 on error. */
size_t sparse_conv_fwd_workspace(int ndim, const int32_t* extent, int batch, int64_t nnz_in, int c_in, int c_out,
                                 const int32_t* ksize, unsigned fuse, int64_t cand_capacity);

/* Forward direct sparse convolution with attention (Algorithm 1), optionally
 * followed by sparse ReLU and sparse 2^ndim max-pooling.
 *
 *   out[b, p, oc] = sum over taps delta, channels ic of
 *                   w[tap(delta), ic, oc] * in[b, p + delta, ic]
 * (stride 1, zero "same" padding: an input at q updates p = q - delta, updates
 * leaving the grid are dropped -- Alg. 1 steps 5-9).  Inputs, weights and
 * responses are fp32.  The vector kernels sum each response in fp64 and round
 * to fp32 once.  The matrix-core kernels first add the at most 32 products of
 * one tap and 32-channel chunk in fp32; the quad kernel then adds these partial
 * sums in fp32 where a response has at most 32 of them (filters of up to 32
 * taps on up to 32 input channels, 16 taps on 64: the r = 128 layer's 27 x 1),
 * in fp64 otherwise; the pair-list kernel always adds them in fp64.  All stay
 * within 1e-5 relative + 1e-6 absolute of the exact sum on the workloads this
 * library is tested on.  In general the error of a matrix-core response follows
 * the magnitudes it is summed from, not its own: about 2e-8 * A, A = the sum of
 * |w * in| over its products (fp32 roundings of partial sums of that size),
 * which the stated tolerance covers while A stays below about 50 (the r = 128
 * workload: A around 20); scnn_set_conv_path(1) sums everything in fp64 for
 * data beyond that.  The vector kernels and the quad kernel add in an order
 * fixed by the data alone and are reproducible bit for bit; the pair-list
 * kernel adds its per-tap partial sums with LDS atomics in no fixed order, so a
 * run can differ from another in the last bits of the fp64 sum, which survives
 * the rounding to fp32 for about one response in 10^8.  Responses that are
 * exactly 0 are not entries (step 13).  bias (nullable, device, [c_out]) is added to the
 * entries (step 14); an entry whose biased value is exactly 0 stops being one.
 * Per (sample b, output channel oc) only the k = scnn_k_from_rho(rho_up, N)
 * entries with the largest score survive (step 15; score = |v| or v by
 * topk_mode); ties at the k-th score go to the lower lin.  Fewer than k entries:
 * all survive.  Then, by `fuse`: entries with v <= 0 are dropped; then entries
 * are max-pooled over the present members of each 2^ndim block, the output grid
 * being ceil(extent/2).  Output rows = sites with at least one surviving entry,
 * ascending by (b, lin), absent entries stored as 0.0f (steps 16-17).
 *
 * out_coords int32 [out_capacity, 1+ndim], out_feats fp32 [out_capacity, c_out].
 * cand_capacity: as given to the workspace query (<= 0: the default bound). */
int sparse_conv_fwd(int ndim, const int32_t* extent, int batch, const int32_t* in_coords, const float* in_feats,
                    int64_t nnz_in, int c_in, const int32_t* ksize, const float* w, const float* bias, int c_out,
                    double rho_up, int topk_mode, unsigned fuse, int32_t* out_coords, float* out_feats,
                    int64_t out_capacity, int64_t cand_capacity, int64_t* nnz_out, void* workspace,
                    size_t workspace_bytes, void* hip_stream);

/* sparse_conv_fwd for a layer that follows another one on the same stream
 * without a host read in between: the number of input rows is taken on the
 * device from nnz_in_dev[0] (for instance the previous call's nnz_out), clamped
 * to in_capacity, the row capacity of in_coords / in_feats that also sizes the
 * workspace (sparse_conv_fwd_workspace with nnz_in = in_capacity).  Rows past
 * the device count are never read.  Everything else as sparse_conv_fwd.  A
 * chain of such calls contains no allocation, host synchronisation or memset
 * node, so it can be captured in a HIP graph (per-stage timing must be off). */
int sparse_conv_fwd_chained(int ndim, const int32_t* extent, int batch, const int32_t* in_coords,
                            const float* in_feats, int64_t in_capacity, const int64_t* nnz_in_dev, int c_in,
                            const int32_t* ksize, const float* w, const float* bias, int c_out, double rho_up,
                            int topk_mode, unsigned fuse, int32_t* out_coords, float* out_feats, int64_t out_capacity,
                            int64_t cand_capacity, int64_t* nnz_out, void* workspace, size_t workspace_bytes,
                            void* hip_stream);

/* The attention step alone (Sec. 3.2; Alg. 1 steps 13, 15-17): k-selection per
 * (sample, channel) over the non-zero entries of a site-major response matrix
 * resp[rows, channels] whose rows are given by `coords`.  k is the integer
 * count per (sample, channel).  Same tie rule and output format as above. */
size_t attention_topk_workspace(int ndim, const int32_t* extent, int batch, int64_t rows, int channels);
int attention_topk(int ndim, const int32_t* extent, int batch, const int32_t* coords, const float* resp,
                   int64_t rows, int channels, int64_t k, int topk_mode, int32_t* out_coords, float* out_feats,
                   int64_t out_capacity, int64_t* nnz_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Sparse ReLU (listed among the paper's layers, Sec. 1): entries with v > 0
 * survive, rows left without an entry are removed. */
size_t sparse_relu_workspace(int64_t rows, int channels);
int sparse_relu(int ndim, const int32_t* coords, const float* feats, int64_t rows, int channels,
                int32_t* out_coords, float* out_feats, int64_t out_capacity, int64_t* nnz_out, void* workspace,
                size_t workspace_bytes, void* hip_stream);

/* sparse_relu for callers that cannot allocate device memory or hold a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation.  Same kernels and same results as sparse_relu; the scratch
 * (counters, one flag and one offset per row, scan sums: about 8 MiB) is a
 * device array inside the library image, held by every GPU the library runs on
 * until the process ends.  At most sparse_relu_static_max_rows() (2^20) rows:
 * more returns SCNN_ECAPACITY and does nothing.  The call allocates and frees
 * nothing, issues no memset node and does not synchronise.  All calls on one
 * GPU share that GPU's array: calls that overlap on one GPU (different streams
 * or host threads) race -- serialise them.  Inputs and outputs are the caller's
 * device arrays as for sparse_relu. */
int64_t sparse_relu_static_max_rows(void);
int sparse_relu_static(int ndim, const int32_t* coords, const float* feats, int64_t rows, int channels,
                       int32_t* out_coords, float* out_feats, int64_t out_capacity, int64_t* nnz_out,
                       void* hip_stream);

/* Sparse max-pooling (Sec. 3.3): output site = floor(p / window), output extent
 * = ceil(extent / window), maximum over the present entries of each cluster,
 * per channel.  window == stride; only window = 2 is implemented. */
size_t sparse_maxpool_workspace(int ndim, const int32_t* extent, int batch, int64_t rows, int channels);
int sparse_maxpool(int ndim, const int32_t* extent, int batch, int window, const int32_t* coords, const float* feats,
                   int64_t rows, int channels, int32_t* out_coords, float* out_feats, int64_t out_capacity,
                   int64_t* nnz_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* sparseToDense (the layer that closes the sparse part of the paper's networks,
 * appendix table of architectures): dense fp32 [batch, channels, extent...]
 * (channel-major, last spatial axis fastest) with dense[b, c, site(r)] =
 * feats[r, c] for every row r and 0 everywhere else.  dense: device pointer,
 * 16-byte aligned, overwritten entirely.  Rows outside the grid are skipped.
 * rows_dev (nullable, device): the row count is read from there, capped by
 * rows, so that the call can end a chain without a host read. */
int sparse_to_dense(int ndim, const int32_t* extent, int batch, const int32_t* coords, const float* feats,
                    int64_t rows, const int64_t* rows_dev, int channels, float* dense, void* hip_stream);

/* Adaptive density regularisation (Sec. 3.5, Eq. 4).  The density of a layer's
 * output, rho = (non-zero entries of out_feats[0 .. rows)) / (n_sites_total *
 * channels) with n_sites_total = batch * prod(extent), sets the bias of the L2
 * regulariser sum (w + b)^2:
 *     b = o + b1 * (rho - rho_up)   if rho > rho_up,    b = -b2 * (rho_up - rho)   otherwise.
 * result (device, double[4]) = {rho, b, lambda * sum over un-pruned weights of
 * (w + b)^2, non-zero entries}; grad_w (device, fp32 [n_w], nullable) =
 * 2 * lambda * (w + b) on un-pruned weights and 0 on pruned ones (exact 0.0f:
 * Eq. 3 gives a removed weight no gradient).  rows_dev (nullable, device): the
 * row count is read from there (capped by rows) so that the call can follow
 * sparse_conv_fwd without a host read.  Sums in fp64 in a fixed order.
 * workspace: density_regulariser_workspace() bytes, 256-byte aligned. */
size_t density_regulariser_workspace(void);
int density_regulariser(const float* out_feats, int64_t rows, const int64_t* rows_dev, int channels, int64_t n_sites_total,
                        double rho_up, double o, double b1, double b2, double lambda, const float* w, int64_t n_w,
                        float* grad_w, double* result, void* workspace, size_t workspace_bytes, void* hip_stream);

/* One-warning-shot pruning (Sec. 3.6), called once per epoch: a non-zero weight
 * with |w| < eps that already carried a warning from the previous call is set
 * to exactly 0 (and stays 0 under sparse_conv_bwd); one that is small for the
 * first time only receives the warning; any other weight loses its warning.
 * w (device, fp32 [n_w]) and warned (device, one byte per weight, 0/1; all 0
 * before the first epoch) are updated in place.  counts (device, int64[2]) =
 * {weights removed by this call, non-zero weights left}. */
int prune_weights(float* w, unsigned char* warned, int64_t n_w, float eps, int64_t* counts, void* hip_stream);

/* Optional precondition check of a coordinate list (synchronises the stream):
 * SCNN_OK, SCNN_EINVAL (coordinate outside the grid) or SCNN_EUNSORTED (rows
 * not strictly ascending by (b, lin)).  workspace: at least 256 bytes. */
int scnn_validate_rows(int ndim, const int32_t* extent, int batch, const int32_t* coords, int64_t rows,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* Back-propagation through the convolution (Algorithm 2) with the masks of
 * Eq. 3: gradients reach only non-zero input values and non-zero (un-pruned)
 * filter weights, so both results have the fixed shapes of the forward
 * operands (Sec. 3.4, first advantage).
 *
 *   bp_data[r, ic]       = sum over taps t, channels oc of
 *                          w[t, ic, oc] * g[b(r), site(r) - delta_t, oc]   if in_feats[r, ic] != 0, else 0
 *   bp_filter[t, ic, oc] = sum over input rows r of
 *                          in_feats[r, ic] * g[b(r), site(r) - delta_t, oc] if w[t, ic, oc] != 0, else 0
 *
 * with the forward pass's get_update_id (an input at q seen through tap delta
 * belongs to output site q - delta; sites outside the grid contribute
 * nothing).  g is the gradient of the loss with respect to the convolution's
 * output, given as sparse rows on the output grid (same extent, stride 1):
 * g_coords int32 [g_rows, 1+ndim] strictly ascending by (b, lin), g_feats fp32
 * [g_rows, c_out]; sites without a row and zero entries carry no gradient (the
 * caller zeroes the entries that the forward selection / ReLU dropped).
 * in_coords / in_feats / w are the forward operands.  bp_data fp32
 * [nnz_in, c_in] and bp_filter fp32 [prod(ksize), c_in, c_out] are overwritten
 * entirely.  Sums are carried in fp64 and rounded to fp32 once, except that the
 * matrix-core kernels (C_out = 16 or a multiple of 32 up to 128, C_in a multiple
 * of 16 up to 64, 16-byte aligned value arrays) first add up to 32 products (bp_data)
 * or the at most 128 products of one tap within one 128-row tile (bp_filter) in
 * fp32.  Error bound of the matrix-core kernels: with A the sum of the
 * magnitudes of the products behind an element, |result - exact| <=
 * 1e-5 |exact| + 1e-6 + c A with c = 2e-8 for bp_data and 1e-7 for bp_filter
 * (a third of, resp. 1.7 times, the fp32 unit roundoff 2^-24: the fp32 chains
 * leave an error proportional to A, not to the cancelling result); the vector
 * kernels meet 1e-5 |exact| + 1e-6 alone.  bp_filter adds its partial sums in
 * a fixed order: repeated calls give identical bits.  info (device, int64[SCNN_NNZ_LEN]) receives {nnz_in, g_rows,
 * SCNN_FLAG_* bits, 0}; with SCNN_FLAG_BAD_COORD or SCNN_FLAG_UNSORTED set the
 * results are undefined (all accesses stay in bounds).  All array arguments are
 * device pointers; extent and ksize are host pointers.  Asynchronous on
 * hip_stream; scnn_set_conv_path(1) forces the vector kernels here too. */
size_t sparse_conv_bwd_workspace(int ndim, const int32_t* extent, int batch, int64_t nnz_in, int c_in, int c_out,
                                 const int32_t* ksize, int64_t g_rows);
int sparse_conv_bwd(int ndim, const int32_t* extent, int batch, const int32_t* in_coords, const float* in_feats,
                    int64_t nnz_in, int c_in, const int32_t* ksize, const float* w, int c_out,
                    const int32_t* g_coords, const float* g_feats, int64_t g_rows, float* bp_data, float* bp_filter,
                    int64_t* info, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Kernel choice for the convolution step of sparse_conv_fwd (and, for 1, of
 * sparse_conv_bwd), for the calling thread:
 * 0 = by shape and size.  Wide layers (C_in >= 32, or C_in = 8, 16 or 24 on
 *     layers whose workspace holds at least 1024 tiles of 128 candidate
 *     sites - 128 tiles when C_in is 16 or 24 and C_out at least 24 - with
 *     C_in * C_out >= 256 and C_out >= 24, or C_in * C_out >= 384)
 *     take the quad matrix-core kernel where C_in is 8, 16, 24, 32, 40, 48 or
 *     64 (or 96 or 128 with a C_out the pair-list kernel does not take), C_out
 *     at most 128, the filter has at most 32 taps and in_feats is 16-byte
 *     aligned; else the pair-list matrix-core
 *     kernel where C_in is 16 or a multiple of 32 up to 128 (any number of
 *     taps) and C_out a multiple of 16 up to 64.  Everything else takes the
 *     vector kernels;
 * 1 = always the vector kernels;
 * 2 = a matrix-core kernel whenever one takes the shape, whatever the size:
 *     the quad kernel wherever it takes the shape (also 96 and 128 input
 *     channels, and 8, 16, 24 on small layers);
 * 3 = the pair-list matrix-core kernel where it takes the shape (C_in = 16 or
 *     a multiple of 32 up to 128, C_out a multiple of 16 up to 64).
 * All compute the same sums to the same rounding rule; the switch exists so
 * that tests and measurements can reach each.  The setting enters the
 * workspace size: query the workspace under the setting the call will run with.
 * scnn_last_conv_kernel() names the kernel family the calling thread's last
 * sparse_conv_fwd call launched ("k_conv_quad", "k_conv_mfma", "k_conv_valu";
 * "" before the first call). */
const char* scnn_last_conv_kernel(void);
int scnn_set_conv_path(int path);

/* Measurement support (not part of the method): when enabled on the calling
 * thread, every sparse_conv_fwd call records HIP events on its stream at the
 * boundaries of its stages (workspace clear + filter preparation + index build,
 * candidate sites, pair lists, convolution, k-selection, compaction + write,
 * pooling), and every sparse_conv_bwd call at the boundaries of its own
 * (filter preparation + index of the gradient rows, pair lists, adjoint
 * convolution, bp_data write, bp_filter).  scnn_profile_collect waits for
 * the recorded calls, adds their per-stage milliseconds into stage_ms
 * [scnn_profile_stage_count()] and the number of calls into *calls, then
 * forgets them.  on = 1: every boundary; on = 2: only the two events around
 * the convolution stage of sparse_conv_fwd (the other stages read 0), for
 * timing the dominant kernel inside a throughput measurement at little
 * cost; on = 3: those two events on every fourth sparse_conv_fwd call after
 * this one, the first included (the events of a call cost about 0.01 ms of
 * stream time; *calls then counts the calls that were timed); on = 0: none.
 * Host pointers. */
int scnn_profile_enable(int on);
int scnn_profile_stage_count(void);
const char* scnn_profile_stage_name(int stage);
int scnn_profile_collect(double* stage_ms, int64_t* calls);

/* A plain device-to-device streaming copy (bytes a multiple of 16, device
 * pointers): the kernel of known traffic against which hardware memory
 * counters are scaled when the library's kernels are profiled. */
int scnn_calibration_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SCNN_H_ */
