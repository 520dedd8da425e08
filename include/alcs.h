/*
 * alcs.h - C ABI of the MI355X (gfx950) SIMD-structured sparse convolution library.
 *
 * The operation is the inference kernel of "Architecture Aware Latency Constrained
 * Sparse Neural Networks on Mobile Devices" (arXiv 2109.00170), Section 3.2:
 * every group of V adjacent output channels keeps or drops the weights at one
 * filter position (c, r, s) as a unit (Section 3.2.1), the kept V-vectors are
 * stored per group in a grouped CSR format (Section 3.2.2, "Storage format"), and
 * the convolution is the product of that block-sparse matrix with the (virtual)
 * patch matrix of the input (Section 3.2.2, "Overview" / "Efficient multiplication
 * computation").
 *
 * Conventions shared by all entry points
 *   - fp32 data, int32 indices, NCHW tensors, row-major, densely packed.
 *   - kernel is 1 or 3 (square); pad = (kernel-1)/2 zeros on every side;
 *     Ho = (H + 2*pad - kernel)/stride + 1, likewise Wo; cross-correlation (the
 *     filter is not flipped), as in the paper's convolution equation.
 *   - G = ceil(Cout / V) groups; group g owns output channels [g*V, g*V+V).
 *     The flattened column index of filter position (c, r, s) is
 *     col = (c*kernel + r)*kernel + s, K = Cin*kernel*kernel columns per group.
 *   - Pointers named *_host point to host memory, *_dev to memory of the current
 *     HIP device.  The caller owns every buffer it passes in.  Device buffers must
 *     be 16-byte aligned (anything hipMalloc or PyTorch returns is).
 *   - Every function returns ALCS_OK (0) or a negative alcs_status; nothing throws
 *     across the boundary.  Launches are asynchronous on `stream` (a hipStream_t
 *     passed as void*, NULL = the default stream); the library never synchronises
 *     and never allocates inside alcs_sparse_conv / alcs_dense_conv.
 *   - Y is overwritten completely and must not alias X, bias or the weights.
 *   - Inputs are expected to be finite; with Inf/NaN in X the result is
 *     unspecified (as it is for the defining sum once 0*Inf terms appear).
 */
#ifndef ALCS_H
#define ALCS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum alcs_status {
    ALCS_OK = 0,
    ALCS_E_INVALID_ARG = -1, /* null pointer, non-positive size, shape mismatch with the handle */
    ALCS_E_UNSUPPORTED = -2, /* kernel not in {1,3}, V not in {1,2,4,8,16}, stride not in {1,2}, size limits */
    ALCS_E_ALLOC = -3,       /* host or device allocation failed */
    ALCS_E_HIP = -4,         /* a HIP runtime call failed (see alcs_last_hip_error) */
    ALCS_E_NO_DEVICE = -5    /* the handle has no device copy (packed without a GPU) */
} alcs_status;

/* Opaque packed weight tensor; created by alcs_pack_weights, owned by the library
 * until alcs_packed_free.  Immutable after creation (but for alcs_packed_set_options and
 * alcs_packed_add_bf16_weights, neither of which may run while another thread uses the handle);
 * may be used from several streams at once.  The library keeps no state outside
 * handles except two per-thread diagnostics (alcs_last_hip_error, alcs_last_launch),
 * the device array of alcs_topn_mask_static and the compute-unit / XCD counts of each
 * device, read from its properties once. */
typedef struct alcs_packed alcs_packed_t;

/* Human-readable name of a status code (static string, never NULL). */
const char *alcs_strerror(int status);

/* hipError_t value of the last failing HIP call made by this thread's library
 * calls (0 if none), for diagnostics after ALCS_E_HIP. */
int alcs_last_hip_error(void);

/* Library version, encoded major*10000 + minor*100 + patch. */
int alcs_version(void);

/*
 * Offline re-organisation of the pruned weights (Section 3.2.2, "Storage format":
 * "number of non-zero columns", "column offsets", "non-zero values" per filter
 * group; done once before inference).
 *
 *   W_host    [Cout, Cin, kernel, kernel] fp32.
 *   mask_host [G, Cin, kernel, kernel] uint8, non-zero = block kept; NULL keeps all
 *             blocks.  The mask rules: a kept block is stored even if its values
 *             are zero, a dropped block contributes nothing whatever W holds there.
 *   V         group size, one of 1, 2, 4, 8, 16.  If Cout is not a multiple of V
 *             the last group is ragged: its missing rows are stored as +0.0f and
 *             never written to Y.
 *   out       receives the handle.
 *
 * Builds (a) the canonical grouped CSR on the host (see alcs_packed_export) and
 * (b) a device-side layout tuned for the kernels, uploaded to the current HIP
 * device with blocking copies.  Without a usable HIP device (b) is skipped, the
 * call still succeeds, and alcs_sparse_conv on that handle returns
 * ALCS_E_NO_DEVICE.  Errors: ALCS_E_INVALID_ARG (null W/out, sizes <= 0),
 * ALCS_E_UNSUPPORTED (kernel, V, or Cin*kernel^2 / Cout beyond 2^24),
 * ALCS_E_ALLOC, ALCS_E_HIP.
 */
int alcs_pack_weights(const float *W_host, const uint8_t *mask_host, int Cout, int Cin, int kernel,
                      int V, alcs_packed_t **out);

/* Shape of a packed tensor: number of groups G, columns per group K, and the total
 * number of kept blocks nnzb.  Any output pointer may be NULL. */
int alcs_packed_info(const alcs_packed_t *p, int *G, int *K, int64_t *nnzb);

/* 1 if the handle has a device copy, else 0 (negative status on a NULL handle). */
int alcs_packed_on_device(const alcs_packed_t *p);

/*
 * Canonical grouped CSR of Section 3.2.2, for bit-exact comparison:
 *   row_ptr_host [G+1]     running total of the per-group kept-column counts
 *                          (count_g = row_ptr[g+1]-row_ptr[g], row_ptr[0] = 0);
 *   col_idx_host [nnzb]    column offset of each kept column = its absolute
 *                          0-based position col in the flattened filter,
 *                          ascending inside a group;
 *   vals_host    [nnzb*V]  the V weights of each kept column, top row first.
 * Caller-allocated host arrays of exactly these sizes.
 */
int alcs_packed_export(const alcs_packed_t *p, int32_t *row_ptr_host, int32_t *col_idx_host,
                       float *vals_host);

/* Host-side consistency check of the tuned layout: re-derives the canonical arrays
 * from the padded/segmented arrays the kernels read and compares bit for bit, and
 * checks every padded slot (zero weight, offset of the all-zero row) and every
 * stored offset against the LDS tile bounds the kernels assume.  Needs no GPU.
 * Returns ALCS_OK or ALCS_E_INVALID_ARG on the first inconsistency. */
int alcs_packed_selfcheck(const alcs_packed_t *p);

/* A 64-bit hash (FNV-1a) of the layout the kernels read - its tile parameters, group order, work
 * records, weight planes and selector tables - into *hash_out (host).  Two handles whose layouts
 * are the same bytes have the same hash: the check that a handle built on the device
 * (alcs_pack_from_csr_device) equals the one alcs_pack_weights builds on the host.  For a
 * handle built on the device this, like alcs_packed_export and alcs_packed_selfcheck, fetches the
 * arrays to the host first (blocking copies; ALCS_E_HIP if they fail). */
int alcs_packed_layout_hash(const alcs_packed_t *p, unsigned long long *hash_out);

/* Releases host and device memory of a handle (NULL is ignored).  The caller must
 * make sure no launch that reads it is still in flight. */
void alcs_packed_free(alcs_packed_t *p);

/*
 * The sparse convolution (Section 3.2.2, "Efficient multiplication computation"):
 *   Y[n, g*V+v, ho, wo] = bias[g*V+v]
 *       + sum over the group's kept columns j of
 *         vals[g][j][v] * Xpad[n, c_j, ho*stride + r_j - pad, wo*stride + s_j - pad]
 *
 *   Wp        handle from alcs_pack_weights with a device copy on the current device.
 *   X_dev     [N, Cin, H, W] fp32.
 *   bias_dev  [Cout] fp32 or NULL (= zeros).
 *   Y_dev     [N, Cout, Ho, Wo] fp32, fully overwritten.
 *   Cin, Cout, kernel must equal the values the handle was packed with
 *   (ALCS_E_INVALID_ARG otherwise - checked on the host before anything is
 *   launched); stride is 1 or 2.  Size limits (ALCS_E_UNSUPPORTED beyond): the
 *   flattened output pixel axis N*Ho*Wo at most 2^31 - 1025, H*W and Ho*Wo below
 *   2^31 each (tensors of more than 2^31 elements are fine: element offsets are
 *   64-bit), at most 2^30 workgroups.  N == 0 is a no-op that returns ALCS_OK.
 *   The accumulation order inside a sum is unspecified (fp32 results agree with the
 *   definition to rounding, not bit for bit).
 */
int alcs_sparse_conv(const alcs_packed_t *Wp, const float *X_dev, const float *bias_dev,
                     float *Y_dev, int N, int Cin, int Cout, int H, int W, int kernel, int stride,
                     void *stream);

/*
 * alcs_sparse_conv with the kernel's own begin and end time stamps recorded on two
 * caller-created hipEvent_t (passed as void*, either may be NULL): the pair measures
 * the launch itself (hipEventElapsedTime after synchronising on stop_event), without
 * the gaps that event packets put on a stream around a short kernel.  For benchmarks;
 * arguments, results and errors are those of alcs_sparse_conv (Section 3.2.2,
 * "Efficient multiplication computation").
 */
int alcs_sparse_conv_timed(const alcs_packed_t *Wp, const float *X_dev, const float *bias_dev,
                           float *Y_dev, int N, int Cin, int Cout, int H, int W, int kernel,
                           int stride, void *stream, void *start_event, void *stop_event);

/* Activations of alcs_sparse_conv_fused. */
typedef enum alcs_activation {
    ALCS_ACT_NONE = 0,  /* identity */
    ALCS_ACT_RELU = 1,  /* max(v, 0) */
    ALCS_ACT_RELU6 = 2  /* min(max(v, 0), 6) */
} alcs_activation;

/*
 * alcs_sparse_conv with the element-wise layers that follow the convolution folded into
 * its epilogue, so that they cost no pass of their own over Y (they are the "other layers
 * (e.g. ReLU layers ...)" whose latency Section 3.3, Eq. (2) books as the constant tau):
 *   Y = act(sparse_conv(X) + bias + residual)
 *   residual_dev  [N, Cout, Ho, Wo] fp32 (a shortcut connection) or NULL; it may be Y_dev
 *                 itself (every element is read and then written by the same thread),
 *                 but must not overlap Y in any other way; 16-byte aligned like the others.
 *   activation    an alcs_activation value (ALCS_E_INVALID_ARG otherwise).
 * With residual_dev = NULL and ALCS_ACT_NONE this is alcs_sparse_conv.  Other arguments,
 * results and errors as there.  NaN inputs to ReLU/ReLU6 give 0 (fmax semantics).
 */
int alcs_sparse_conv_fused(const alcs_packed_t *Wp, const float *X_dev, const float *bias_dev,
                           const float *residual_dev, float *Y_dev, int N, int Cin, int Cout, int H,
                           int W, int kernel, int stride, int activation, void *stream);

/*
 * alcs_sparse_conv_fused (Section 3.2.2, "Efficient multiplication computation") on tensors stored
 * as bfloat16: X_dev, residual_dev and Y_dev hold the upper 16 bits of a float per element (NCHW,
 * same shapes); the packed weights, the bias and every sum stay float32, and Y is rounded to
 * nearest even once, after bias, residual and activation.  The layers this library runs at the
 * HBM roofline move half the bytes.  1x1 handles whose input channels fit one on-chip tile only
 * (at most 2558 input channels, 639 for V < 4; ALCS_E_UNSUPPORTED otherwise); X_dev, Y_dev and
 * residual_dev 8-byte aligned; everything else as alcs_sparse_conv_fused.
 */
int alcs_sparse_conv_bf16(const alcs_packed_t *Wp, const uint16_t *X_dev, const float *bias_dev,
                          const uint16_t *residual_dev, uint16_t *Y_dev, int N, int Cin, int Cout,
                          int H, int W, int kernel, int stride, int activation, void *stream);

/*
 * The same layer in 16-bit arithmetic (Section 3.2.1: the group size follows the width of the
 * machine's vector unit over the element width - here the 16-bit matrix instruction, which takes
 * four kept columns of four output channels at a time; groups of V = 8 and 16 are two and four
 * such instructions on one input operand): X_dev, residual_dev and Y_dev bfloat16 as for
 * alcs_sparse_conv_bf16, and the packed WEIGHTS rounded to bfloat16 (nearest even) as well;
 * products are exact, sums float32, the bias float32, Y rounded once at the end.  The result is
 * the definition evaluated on the rounded weights and inputs, up to float32 summation error.
 *
 * alcs_packed_add_bf16_weights: gives a handle the rounded copy of its weights in the
 *   instruction's layout (device memory of the handle, freed with it; a kernel on `stream`, no
 *   wait: use the handle on that stream, or synchronise first).  Once per handle; a second call
 *   does nothing.  Handles it takes: kernel 1, V in {4, 8, 16}, all input channels in one
 *   on-chip tile: at most 1278 input channels (1279 for handles with one group per wavefront;
 *   up to 638 the tile has 128 pixels and a lane two of them, beyond that 64 and one); handles
 *   that alcs_pack_weights built with several groups per wavefront are taken as they are (every
 *   group gets a segment of its own in the 16-bit arrays).  Others ALCS_E_UNSUPPORTED.
 *   ALCS_E_NO_DEVICE
 *   for a handle without a device copy; the handle's device must be current.
 * alcs_sparse_conv_bf16_mfma: arguments and errors as alcs_sparse_conv_bf16, the three tensors
 *   16-byte aligned; ALCS_E_INVALID_ARG for a handle without the rounded weights.
 */
int alcs_packed_add_bf16_weights(alcs_packed_t *p, void *stream);
int alcs_sparse_conv_bf16_mfma(const alcs_packed_t *Wp, const uint16_t *X_dev, const float *bias_dev,
                               const uint16_t *residual_dev, uint16_t *Y_dev, int N, int Cin, int Cout,
                               int H, int W, int kernel, int stride, int activation, void *stream);

/*
 * Depthwise 3x3 layer and the MobileNet block (the network pruned in Section 4 of the paper:
 * every pointwise convolution is preceded by a depthwise 3x3 layer with its own bias and
 * activation; they are among the layers behind the constant tau of Section 3.3, Eq. (2)).
 *
 * alcs_depthwise_conv:  Z[n,c,ho,wo] = act(bias[c] + sum_{r,s} D[c,r,s] *
 *     X[n, c, ho*stride + r - 1, wo*stride + s - 1]),  zero outside the image, no kernel flip;
 *     Ho = (H-1)/stride + 1, Wo = (W-1)/stride + 1.  dw_weights_dev is [C,3,3], X_dev [N,C,H,W],
 *     Y_dev [N,C,Ho,Wo], bias_dev [C] or NULL: device memory, caller-owned, no aliasing.
 *
 * alcs_dw_sparse_conv_fused:  Y = act(conv1x1(Wp; Z) + bias + residual) with Z the depthwise
 *     layer above applied to X_dev (dw_weights_dev, dw_bias_dev, dw_stride, dw_activation), in
 *     one kernel: Z is produced tile by tile in on-chip memory and never written out.  Wp must
 *     be a 1x1 handle with Cin inputs; X_dev is [N,Cin,H,W]; Y_dev and residual_dev (NULL or a
 *     tensor of Y's shape, may be Y_dev itself) are [N,Cout,Ho,Wo].  workspace_dev is NULL or
 *     [N,Cin,Ho,Wo] floats of scratch.  With a workspace the library runs the two layers one
 *     after the other through it (same result to rounding; the workspace's contents afterwards
 *     are unspecified) where that is the faster or the only way: small layers whose output
 *     groups are split over several workgroups per pixel tile (each would evaluate the
 *     depthwise layer again), handles whose input channels do not fit one on-chip tile (more
 *     than 2558 input channels, or V < 4 with more than 639), inputs of more than about 10^9
 *     elements per image.  Without a workspace the first kind still runs as one kernel and
 *     the other two return ALCS_E_UNSUPPORTED.
 *
 * Both: stride in {1, 2} (else ALCS_E_UNSUPPORTED); activations are alcs_activation values
 * (else ALCS_E_INVALID_ARG); X_dev / Y_dev / residual_dev 16-byte aligned for the fused call;
 * asynchronous on `stream`, nothing allocated, N = 0 is a no-op.
 */
int alcs_depthwise_conv(const float *dw_weights_dev, const float *X_dev, const float *bias_dev,
                        float *Y_dev, int N, int C, int H, int W, int stride, int activation,
                        void *stream);
int alcs_dw_sparse_conv_fused(const alcs_packed_t *Wp, const float *dw_weights_dev,
                              const float *dw_bias_dev, int dw_stride, int dw_activation,
                              const float *X_dev, const float *bias_dev, const float *residual_dev,
                              float *Y_dev, float *workspace_dev, int N, int Cin, int Cout, int H,
                              int W, int activation, void *stream);

/*
 * Dense convolution with the same conventions: the sparsity-0 case of the
 * operation above and the same-GPU baseline (the role the dense models play in the
 * paper's Section 4.1 timing protocol).
 *   W_dev [Cout, Cin, kernel, kernel] fp32 on the device; other arguments as above.
 */
int alcs_dense_conv(const float *W_dev, const float *X_dev, const float *bias_dev, float *Y_dev,
                    int N, int Cin, int Cout, int H, int W, int kernel, int stride, void *stream);

/*
 * Options of a packed tensor: the shape of its device layout and of the launches that use it.
 * They belong to the handle (the library keeps no process-wide state); every field is an int,
 * 0 = the automatic choice, negative values are ALCS_E_INVALID_ARG.  Results never depend on
 * them beyond floating-point summation order.  For tests, benchmarks and callers who know
 * their shapes; the defaults come from sweeps on MI355X.
 *
 *   read when the handle is packed (they shape the device layout; alcs_packed_set_options
 *   leaves them as they were):
 *     chunk_channels   input channels per on-chip chunk (forces the kernels that stream the
 *                      input channels through LDS in chunks)
 *     group_slots      output-channel groups multiplied per wavefront by the 1x1 kernels: 1, 2
 *                      or 4 (automatic: 1 below 512 input channels or for V < 4; from 512
 *                      channels on 4 for V = 4 or 8 when no group keeps more than twice the mean
 *                      number of columns, else 2; 4 from 1280 channels on)
 *   read at every launch:
 *     pixels_per_lane  1x1 kernels: 1, 2 or 4 (1 or 2 with several groups per wavefront);
 *                      3x3 kernel: 1 or 2 (2: tiles of twice the height, stride 1, V = 4 or 8)
 *     waves            wavefronts per workgroup
 *     group_tiles      number of workgroups that share one pixel tile
 *     path             1 = plain-FMA inner loop where it exists (V = 4), 2 = MFMA inner loop,
 *                      4 = persistent double-buffered 1x1 kernel with the weights in LDS where
 *                      applicable, 5 = pipelined persistent 1x1 kernel (four groups per
 *                      wavefront, at most 512 input channels and 64 kept columns per group)
 *                      wherever it applies, 6 = never that kernel and, for 3x3 handles whose
 *                      pattern is shared by the nine taps, the column-by-column walk instead
 *                      of the walk over channel records; 7 = that record walk wherever it
 *                      exists (V = 4 or 8; the default takes it with pixels_per_lane 2 only)
 *     tile_width       output-tile width of the 3x3 kernel: 8, 16 or 32 (tile height 64/width)
 *     groups_per_wave  groups whose accumulators a wavefront of the chunked 1x1 kernel and of
 *                      the 3x3 kernel holds: 2 or 4 (automatic: 4, or 2 when the layer has few
 *                      groups, for V >= 8, or where halving lets two workgroups share a
 *                      compute unit)
 *     dw_own_taps      alcs_dw_sparse_conv_fused: every lane loads all nine taps of its pixel
 *                      instead of sharing them with its neighbours
 *     dw_one_kernel    alcs_dw_sparse_conv_fused: stay in one kernel even where the call would
 *                      run the two layers through its workspace for speed
 *     full_tiles       1x1 kernels: keep full pixel tiles where the launch would give every
 *                      workgroup fewer pixels so as to occupy all compute units
 *     measure_skip     must be 0.  (A measurement build of the library, compiled with
 *                      -DALCS_MEASURE=1 and never shipped as libalcs.so, skips phases of the
 *                      kernels by these bits - 1 input staging, 2 multiply, 4 output stores,
 *                      8 everything - to time the others; results are then meaningless.)
 *     reserved         must be 0
 */
typedef struct alcs_options {
    int pixels_per_lane, waves, group_tiles, path, tile_width, groups_per_wave;
    int chunk_channels, group_slots;
    int dw_own_taps, dw_one_kernel, full_tiles;
    int measure_skip;
    int reserved[4];
} alcs_options;

/* alcs_pack_weights with options (NULL = all automatic, i.e. alcs_pack_weights itself); the
 * offline re-organisation of Section 3.2.2, "Storage format".  ALCS_E_INVALID_ARG for a
 * negative field, a non-zero reserved field or measure_skip. */
int alcs_pack_weights_opt(const float *W_host, const uint8_t *mask_host, int Cout, int Cin, int kernel,
                          int V, const alcs_options *options, alcs_packed_t **out);

/* Replaces the launch options of a handle (the two layout fields keep their pack-time
 * values) / reads the handle's options back.  Setting options is the one way a handle changes
 * after it is packed (besides alcs_packed_add_bf16_weights, which only adds): it must not run
 * while another thread launches with that handle. */
int alcs_packed_set_options(alcs_packed_t *p, const alcs_options *options);
int alcs_packed_get_options(const alcs_packed_t *p, alcs_options *options);

/* Latency model (Section 3.3 of the paper).  A layer is timed at n numbers of non-zero weights
 * k[0] < k[1] < ... < k[n-1] (the paper uses 0, 0.1 N, ..., N: eleven runs of
 * alcs_sparse_conv_timed per layer), giving run times t[0..n-1] in any unit.
 *
 * alcs_latency_estimate: Eqs. (4)-(6) - the estimate for a layer with s non-zero weights,
 *   t[0] plus, for every interval that s has reached, the interval's slope
 *   (t[i+1]-t[i]) / (k[i+1]-k[i]) times the part of it below s: the piecewise-linear
 *   interpolant of the measured points, t[0] for s <= k[0] and t[n-1] for s >= k[n-1].
 * alcs_network_latency: Eq. (2) - tau (the run time of all layers that are not pruned, a
 *   constant) plus the estimates of L layers.  Layer l owns the n_host[l] knots that start at
 *   index n_host[0] + ... + n_host[l-1] of k_host / t_host and has s_host[l] non-zero weights.
 *
 * All pointers are host memory, read during the call only; results are written to
 * *estimate_out / *latency_out.  ALCS_E_INVALID_ARG: null pointers, fewer than two knots,
 * knots not strictly increasing, non-finite table entries or tau, NaN s.  No GPU is used. */
int alcs_latency_estimate(const double *k_host, const double *t_host, int n, double s,
                          double *estimate_out);
int alcs_network_latency(double tau, const double *k_host, const double *t_host, const int *n_host,
                         int L, const double *s_host, double *latency_out);

/*
 * Projection onto the latency constraint (Section 3.4, Algorithm 1 of the paper) on the GPU.
 *
 * alcs_block_scores (steps 1-2): scores_dev[g*K + col] = squared L2 norm of the block of V weights
 *   W[g*V .. g*V+V-1][col] (K = Cin*kernel*kernel columns of the stretched filter, G = ceil(Cout/V)
 *   groups; rows beyond Cout count as zero).  The score decides an order, so its arithmetic is
 *   fixed: float32, sum = 0, then sum = sum + w_v*w_v for v = 0 .. V-1 with product and sum
 *   rounded separately.  W_dev [Cout,Cin,kernel,kernel] and scores_dev [G*K] are device memory.
 *
 * alcs_topn_mask (step 7): mask_dev[i] = 1 for the N blocks with the largest score among
 *   scores_dev[0 .. n_blocks), 0 for the others; larger score first (compared through the bit
 *   pattern: scores are non-negative, NaN ranks above infinity), lower index first among equal
 *   scores.  seg_starts_host [n_segments + 1] (ascending, first 0, last n_blocks; NULL = one
 *   segment) splits the array into layers; seg_counts_host [n_segments] (or NULL) receives the
 *   number of kept blocks per segment.  mask_dev may be NULL (counts only).  n_blocks < 2^32.
 *   The call returns after the stream has finished when counts are asked for.
 *
 * alcs_project_latency: the whole of Algorithm 1.  scores_dev holds the scores of n_layers layers
 *   back to back (layer l = [seg_starts_host[l], seg_starts_host[l+1])), V_host[l] is the layer's
 *   group size (a kept block is V non-zero weights), (tau, k_host, t_host, n_host) are the latency
 *   tables in the layout of alcs_network_latency.  N0 = 0, N1 = n_blocks, t0 / t1 = latency with
 *   nothing / everything kept; while t1 - t0 > eps: N = (N0+N1)/2, t = latency of the network
 *   that keeps the N largest blocks; t < budget moves (t0, N0) up, else (t1, N1) down; the
 *   result keeps the (N0+N1)/2 largest blocks.  Halves are integer divisions and the loop also
 *   ends when N1 - N0 <= 1.  Outputs: mask_dev [n_blocks] (device, may be NULL), *N_out,
 *   *t0_out, *t1_out (host, may be NULL).  Synchronises `stream` once per bisection step.
 *
 * workspace_dev: device memory of at least alcs_select_workspace_bytes(n_segments) bytes, 8-byte
 * aligned, owned by the caller, overwritten by the call; calls that share a workspace must not
 * overlap.  Errors: ALCS_E_INVALID_ARG (null pointers, N outside [0, n_blocks], bad segment
 * table, negative eps), ALCS_E_UNSUPPORTED (V, kernel, 2^32 blocks or more), ALCS_E_HIP.
 */
int alcs_block_scores(const float *W_dev, int Cout, int Cin, int kernel, int V, float *scores_dev,
                      void *stream);
size_t alcs_select_workspace_bytes(int n_segments);
int alcs_topn_mask(const float *scores_dev, long long n_blocks, long long N,
                   const long long *seg_starts_host, int n_segments, uint8_t *mask_dev,
                   long long *seg_counts_host, void *workspace_dev, void *stream);
int alcs_project_latency(const float *scores_dev, const long long *seg_starts_host, const int *V_host,
                         int n_layers, double tau, const double *k_host, const double *t_host,
                         const int *n_host, double budget, double eps, uint8_t *mask_dev,
                         long long *N_out, double *t0_out, double *t1_out, void *workspace_dev,
                         void *stream);

/*
 * alcs_topn_mask for callers that cannot allocate device memory or bring a workspace (code that
 * runs where hipMalloc is forbidden: tight serving loops, harnesses that rule it out): the same
 * selection, same arguments minus workspace_dev, same results bit for bit, with the selection
 * state in a device array that is part of the library image.  The call allocates nothing, on the
 * host or on the device.
 *   - At most ALCS_TOPN_STATIC_MAX_SEGMENTS segments (ALCS_E_UNSUPPORTED beyond; n_blocks is
 *     limited only as in alcs_topn_mask: the state's size depends on the segments alone).
 *   - Every GPU the library is used on holds one copy of the array (about 33 KB) until the
 *     process ends; its address is looked up on the first call on that device.
 *   - All calls on one GPU share that array, whatever their stream: calls that overlap on one GPU
 *     race, the caller serialises them.  The array keeps the previous call's contents; each call
 *     clears what it needs itself.
 */
#define ALCS_TOPN_STATIC_MAX_SEGMENTS 1024
int alcs_topn_mask_static(const float *scores_dev, long long n_blocks, long long N,
                          const long long *seg_starts_host, int n_segments, uint8_t *mask_dev,
                          long long *seg_counts_host, void *stream);

/*
 * The storage format of Section 3.2.2 ("Storage format") built on the device, and a handle made
 * from the format's arrays.
 *
 * alcs_pack_csr_device: the canonical arrays of alcs_packed_export - row_ptr_dev [G+1],
 *   col_idx_dev [nnzb], vals_dev [nnzb*V] - from W_dev [Cout,Cin,kernel,kernel] and mask_dev
 *   [G,Cin,kernel,kernel] (NULL keeps every block), all device memory owned by the caller; bit for
 *   bit what alcs_pack_weights builds on the host.  The call synchronises `stream` once to learn
 *   nnzb, which it stores in *nnzb_out (host, may be NULL).  With col_idx_dev = vals_dev = NULL
 *   only row_ptr_dev is filled (a counting pass to size the other two); otherwise
 *   capacity_blocks (the number of blocks col_idx_dev / vals_dev have room for) must be at least
 *   nnzb, else ALCS_E_INVALID_ARG and nothing but row_ptr_dev is written.
 *
 * alcs_pack_from_csr: a handle like alcs_pack_weights' from canonical arrays in host memory
 *   (copied; columns must ascend inside every group and lie below K, counts must add up:
 *   ALCS_E_INVALID_ARG otherwise).  Together: device flags -> device arrays -> one copy of the
 *   kept values to the host -> handle, without the dense weights leaving the device.
 *
 * alcs_pack_from_csr_device: the same handle from canonical arrays in device memory (caller's;
 *   copied into the handle's own allocation), with the layout the kernels read built by kernels
 *   on `stream`: the host reads back a few scalars (block count, longest group, padded length)
 *   and neither the arrays nor the layout cross the bus.  The arrays are checked on the device
 *   like alcs_pack_from_csr checks them on the host (ALCS_E_INVALID_ARG).  `options` as for
 *   alcs_pack_weights_opt (NULL = automatic).  The call returns with the handle complete (it
 *   synchronises `stream`); alcs_packed_export and alcs_packed_selfcheck fetch the arrays to the
 *   host on first use.  With more than 16384 groups (an FC layer of more than 16384 * V outputs) the
 *   arrays are copied to the host once and the layout is built there, as alcs_pack_from_csr does.
 *
 * alcs_pack_weights_device: W_dev and mask_dev as for alcs_pack_csr_device -> handle, i.e. the
 *   two calls above in one with the intermediate arrays in a temporary of the library (sized for
 *   every block kept, freed before the call returns).  This is the re-packing step of a pruning
 *   loop (Section 3.4, Algorithm 1) whose weights and flags live on the device.
 *
 * alcs_pack_network_device: the same for n_layers layers in one call - every step is enqueued for
 *   all layers before the host waits for its scalars, so a network costs three waits on `stream`
 *   instead of three a layer.  layers[i] names layer i (device pointers as for
 *   alcs_pack_csr_device; options may be NULL); out [n_layers] receives the handles - all of them,
 *   or none (every entry NULL) when the call fails.  workspace_dev: device memory of at least
 *   alcs_pack_workspace_bytes(layers, n_layers) bytes, 256-byte aligned, the caller's, free for
 *   other use when the call returns; NULL (workspace_bytes ignored) lets the call allocate and
 *   free it itself.  alcs_pack_workspace_bytes depends on the layers' shapes and options only
 *   (it sizes for every block kept) and returns a negative status for shapes the packer refuses;
 *   layers of more than 16384 groups are not taken here (ALCS_E_UNSUPPORTED: pack them one by one).
 */
typedef struct alcs_layer_desc {
    const float *W_dev;       /* [Cout, Cin, kernel, kernel] */
    const uint8_t *mask_dev;  /* [G, Cin, kernel, kernel] keep flags, NULL keeps every block */
    int Cout, Cin, kernel, V;
    const alcs_options *options; /* host pointer, NULL = automatic */
} alcs_layer_desc;
long long alcs_pack_workspace_bytes(const alcs_layer_desc *layers, int n_layers);
int alcs_pack_network_device(const alcs_layer_desc *layers, int n_layers, void *workspace_dev,
                             long long workspace_bytes, void *stream, alcs_packed_t **out);
int alcs_pack_csr_device(const float *W_dev, const uint8_t *mask_dev, int Cout, int Cin, int kernel,
                         int V, int32_t *row_ptr_dev, int32_t *col_idx_dev, float *vals_dev,
                         long long capacity_blocks, long long *nnzb_out, void *stream);
int alcs_pack_from_csr(const int32_t *row_ptr_host, const int32_t *col_idx_host, const float *vals_host,
                       int Cout, int Cin, int kernel, int V, alcs_packed_t **out);
int alcs_pack_from_csr_device(const int32_t *row_ptr_dev, const int32_t *col_idx_dev, const float *vals_dev,
                              int Cout, int Cin, int kernel, int V, const alcs_options *options, void *stream,
                              alcs_packed_t **out);
int alcs_pack_weights_device(const float *W_dev, const uint8_t *mask_dev, int Cout, int Cin, int kernel, int V,
                             const alcs_options *options, void *stream, alcs_packed_t **out);

/* What the last alcs_sparse_conv call of this thread launched: fills up to `cap`
 * ints {mode (1 = all input channels resident in LDS, 2 = chunked, 3 = 3x3,
 * 4 = persistent double-buffered with the weights in LDS, 5 = pipelined persistent,
 * 6 = the 16-bit kernel of alcs_sparse_conv_bf16_mfma, whose path reads 3,
 * 7 = 3x3 walking channel records (handles whose pattern is shared by the nine taps)),
 * pv, waves, workgroups, lds_bytes, group_tiles,
 * chunk_channels, path, group_slots, tile_width (3x3 only, else 0)} and returns how many were
 * written.  For tests and benchmarks. */
int alcs_last_launch(int *out, int cap);

#ifdef __cplusplus
}
#endif
#endif /* ALCS_H */
