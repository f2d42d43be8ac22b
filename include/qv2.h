/*
 * qv2 -- the per-layer local-metric sensitivity pass of QuantuneV2
 * (arXiv 2501.07161) for AMD MI355X (gfx950).  C ABI.
 *
 * The pass follows the paper's execution process (Sec. 4, steps 1-4):
 *   1. calibration: min / max and tensor statistics of every weight and
 *      activation tensor                                   -> qv2_calibrate
 *   2. scale / zero-point and uniform int8 quantization of all layers
 *      (Sec. 2.1 Eq. 1-3, Sec. 4 Eq. 4-5)                   -> qv2_calibrate,
 *                                                              qv2_fakequant_metrics
 *   3. local metrics SQNR and MSE per layer (Sec. 6.1 Eq. 6-7), for a tensor
 *      against its own dequantized form                     -> qv2_fakequant_metrics
 *      and for a layer's output in the fp32 inference against the same output
 *      in the quantized inference (Algorithm 2, D[i] vs Q[i]) -> qv2_pair_metrics
 *   4. SQNR delta (Sec. 6.4 Eq. 16) and the sensitivity list
 *      (Algorithm 2, RankLayersBySensitivity)               -> qv2_rank
 * Steps 1-3 are also available as one call that visits every tensor as few
 * times as the method allows       -> qv2_calibrate_fakequant_pair_metrics
 * and steps 1-4 as one host call   -> qv2_sensitivity_pass
 *
 * Conventions
 *  - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  Every
 *    device buffer (tensors, codes, params, sums, workspace) is allocated and
 *    freed by the caller.  The library owns only the opaque qv2_plan (host
 *    tables plus a device copy of them - qv2_plan_device_bytes() says how large - released
 *    by qv2_plan_destroy).
 *  - Device calls only enqueue work on `hip_stream` (a hipStream_t passed as
 *    void*; NULL = the default stream) and never synchronise it, except that
 *    the first device call on a plan uploads the plan's tables with a blocking
 *    copy.  Outputs are valid once the caller has synchronised the stream.
 *    The tables stay on the device that was current at that first call; a later
 *    call with another device current returns QV2_ERR_HIP.  A stream capture
 *    (HIP graph) may record any device call after the first one on its plan.
 *  - A plan serves one thread at a time (the first device call uploads its tables
 *    and the optional timing events belong to it); different plans are independent,
 *    and calls on one plan that may overlap on the GPU need separate workspaces.
 *  - Every call returns a qv2_status.  Arguments are validated on the host
 *    before anything is launched; nothing aborts or throws across the ABI.
 *  - Identical inputs give bit-identical outputs (no floating-point atomics;
 *    every reduction has a fixed order).
 *  - Inputs must be finite.  NaNs are ignored by min / max but poison sums.
 *
 * Quantizer (fixed by this library; fp32 arithmetic, one rounding per step):
 *   asymmetric (Eq. 2, N = 256, range widened to contain 0):
 *      lo = min(min,0)  hi = max(max,0)  scale = (hi-lo)/255
 *      inv_scale = 1/scale     zp = clamp(rne(-128 - lo*inv_scale), -128, 127)
 *   symmetric (Eq. 4, b = 8):  scale = max(|min|,|max|)/127, inv_scale = 1/scale, zp = 0
 *   degenerate (scale below the smallest normal float): scale = inv_scale = 1, zp = 0
 *   code  = clamp(rne(x*inv_scale) + zp, -128, 127)       (round half to even)
 *   xhat  = (code - zp) * scale
 */
#ifndef QV2_H
#define QV2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  QV2_OK = 0,
  QV2_ERR_NULL = -1,       /* a required pointer is NULL                         */
  QV2_ERR_SHAPE = -2,      /* bad numel / channels / count / layer positions     */
  QV2_ERR_SCHEME = -3,     /* unknown qv2_scheme                                 */
  QV2_ERR_WORKSPACE = -4,  /* workspace smaller than qv2_workspace_bytes()       */
  QV2_ERR_NONFINITE = -5,  /* NaN / Inf where a finite value is required         */
  QV2_ERR_HIP = -6,        /* a HIP runtime call or kernel launch failed         */
  QV2_ERR_ALIGN = -7,      /* a device pointer is not aligned as required        */
  QV2_ERR_IO = -8,         /* a file could not be created or written             */
  QV2_ERR_NOMEM = -9,      /* host memory for the plan or a work list ran out    */
  QV2_ERR_STATE = -10      /* the plan is not in the state the call needs (its tables not on
                              the device yet; no pass begun in that slot)          */
} qv2_status;

typedef enum {
  QV2_ASYM_TENSOR = 0,     /* Sec. 2.1 Eq. 1-3 over the whole tensor             */
  QV2_SYM_TENSOR = 1,      /* Sec. 4 Eq. 4-5 over the whole tensor               */
  QV2_SYM_CHANNEL = 2      /* Sec. 4 Eq. 4-5 per slice of dim 0 (output channel) */
} qv2_scheme;

/* One row of the layer table (host memory, caller-owned, copied by the plan). */
typedef struct {
  const float* x;      /* DEVICE, contiguous fp32, 4-byte aligned (16-byte: fast path) */
  const float* qrun;   /* DEVICE or NULL: the same tensor taken from the quantized
                          inference (Algorithm 2's Q[i]); enables pair metrics      */
  int8_t* codes;       /* DEVICE or NULL: receives numel int8 codes.  NULL = metrics
                          only: the quantize sweep then stores nothing (4 B/element) */
  int64_t numel;       /* > 0                                                       */
  int32_t channels;    /* QV2_SYM_CHANNEL: number of dim-0 slices, must divide
                          numel; other schemes: must be 1                           */
  int32_t scheme;      /* qv2_scheme                                                */
  int32_t kind;        /* 0 weight, 1 activation; used by qv2_rank_tensors only     */
  int32_t layer;       /* layer index this tensor belongs to; qv2_rank_tensors only */
} qv2_tensor;

/* Per segment (a whole tensor, or one output channel).  This array is the
 * calibration cache of Sec. 5: it may be saved and handed back to
 * qv2_fakequant_metrics without recalibrating. */
typedef struct {
  float min, max;          /* -0.0 is reported as +0.0                            */
  float scale, inv_scale;
  int32_t zp;
  int32_t _pad;
} qv2_qparams;

/* Per segment.  qv2_calibrate writes sum_x, sum_x2, n and clears sum_e2;
 * qv2_fakequant_metrics writes sum_e2 and rewrites sum_x2 and n from the data
 * it quantized (so SQNR is consistent when cached params are used). */
typedef struct {
  double sum_x, sum_x2, sum_e2;
  int64_t n;
} qv2_sums;

/* Per tensor of the plan (entries of tensors without qrun are zero). */
typedef struct {
  double sum_ref2;         /* sum x^2          (signal energy, Eq. 6)             */
  double sum_d2;           /* sum (x - qrun)^2 (noise energy, Eq. 6-7)            */
  int64_t n;
  int64_t _pad;
} qv2_pair_sums;

/* Per tensor: the per-segment records of a tensor folded on the device, so that a caller who
 * only needs per-tensor metrics copies a few KB to the host instead of every segment. */
typedef struct {
  double sum_x, sum_x2, sum_e2;
  int64_t n;
  float min, max;
  int32_t _pad[2];
} qv2_tensor_sums;

/* Per tensor, host, fp64. */
typedef struct {
  double mse;              /* Eq. 7: sum_e2 / numel                               */
  double sqnr_db;          /* Eq. 6: 10 log10(sum_x2 / sum_e2); +inf if sum_e2==0 */
  double mean, var;        /* population variance                                 */
  float absmax, min, max;
  int32_t _pad;
} qv2_metrics;

/* Constants of the ranking.  The paper says only that the weight SQNR delta
 * gets more gain than the activation one; 0.6 / 0.4 are this library's defaults. */
typedef struct {
  double alpha_w;          /* default 0.6                                         */
  double alpha_a;          /* default 0.4                                         */
  double mse_factor;       /* default 5 (Algorithm 2: MSE > 5 x mean MSE)         */
  double sqnr_cap_db;      /* default 200: |SQNR| is clamped before differencing  */
  int32_t mse_source;      /* 0 activation-pair MSE (default), 1 weight MSE,
                              2 either, each against its own mean                 */
  int32_t _pad;
} qv2_rank_config;

typedef struct qv2_plan qv2_plan;

/* ---- plan (host only; needs no GPU) ------------------------------------- */

/* Validates the layer table and cuts it into tiles: one flat tile table over all
 * tensors, so that one launch covers every layer whatever its size.
 * Errors: NULL table or out -> ERR_NULL; n_tensors <= 0, numel <= 0 or > 2^36, channels
 * not dividing numel (or != 1 for per-tensor schemes), more than 2^31-1 segments, or more tiles
 * than one launch can take (a sweep is one launch of at most 2^32-1 threads: 2^24-1 quantize
 * tiles of 2048 elements over all tensors with a code buffer, i.e. just under 2^35 elements of
 * them; 2^23-1 read tiles of 32768 elements) -> ERR_SHAPE; unknown scheme -> ERR_SCHEME; x (or qrun) not
 * 4-byte aligned -> ERR_ALIGN; x NULL -> ERR_NULL; no host memory for the tile
 * tables -> ERR_NOMEM (the host functions below that build work lists - qv2_rank,
 * qv2_rank_tensors, qv2_bops_select, qv2_regroup_for_fusion - return it too). */
/* Test hooks, not part of the interface: the environment variables QV2_TILE_ELEMS (read-only
 * sweeps) and QV2_QUANT_TILE_ELEMS (quantize sweeps), read here, override the tile lengths so that
 * tests can force many tiles onto small tensors and tuning runs can sweep them.  The defaults are
 * the measured best; production callers leave both unset. */
qv2_status qv2_plan_create(const qv2_tensor* h_tensors, int32_t n_tensors, qv2_plan** out);
void qv2_plan_destroy(qv2_plan* plan);

int32_t qv2_plan_num_tensors(const qv2_plan* plan);
/* Total segments; params / sums arrays have this many entries, tensor after
 * tensor in table order, channel after channel. */
int64_t qv2_plan_num_segments(const qv2_plan* plan);
/* Index of the first segment of tensor `t` (-1 if out of range). */
int64_t qv2_plan_segment_begin(const qv2_plan* plan, int32_t t);
/* Tile counts, for diagnostics and tests: tiles of the calibration pass, of the
 * quantize passes (shorter stream tiles) and of the pair pass. */
int64_t qv2_plan_num_tiles(const qv2_plan* plan);
int64_t qv2_plan_num_quant_tiles(const qv2_plan* plan);
int64_t qv2_plan_num_pair_tiles(const qv2_plan* plan);
/* Elements of the tensors that qv2_calibrate_fakequant_pair_metrics reads from HBM once (their
 * channels are short enough to be held on chip, see there); for byte accounting. */
int64_t qv2_plan_num_single_read_elements(const qv2_plan* plan);
/* Bytes of device workspace any device call on this plan needs (256-byte
 * aligned base).  Calls that may overlap in time need separate workspaces. */
size_t qv2_workspace_bytes(const qv2_plan* plan);

/* Puts the plan's tables on the current device now: one device allocation of
 * qv2_plan_device_bytes(plan) bytes and host-to-device copies on hip_stream, which is waited for
 * before the call returns.  Optional - every device call does the same on first use (on the
 * default stream) - except for qv2_calibrate_fakequant_pair_metrics_noalloc, which never
 * allocates and so needs the tables in place.  A plan that is already on the current device is
 * left alone; one that sits on another device gives ERR_HIP. */
qv2_status qv2_plan_upload(qv2_plan* plan, void* hip_stream);
/* Size of that device allocation in bytes (0 for a NULL plan); needs no GPU. */
size_t qv2_plan_device_bytes(const qv2_plan* plan);

/* Optional timing of the tile kernels (for benchmarks).  When enabled, every
 * launch of a tile kernel is bracketed by two HIP events on the call's stream;
 * after the stream has been synchronised qv2_plan_kernel_ms returns the duration
 * of the most recent launch of that kernel (0 if it has not run).  Enabling
 * creates the events (the only allocation outside the first-use table upload). */
typedef enum {
  QV2_K_STATS_STREAM = 0, QV2_K_STATS_ROWS = 1, QV2_K_QUANT_STREAM = 2, QV2_K_QUANT_ROWS = 3,
  QV2_K_PAIR_STREAM = 4, QV2_K_QUANTPAIR_STREAM = 5, QV2_K_QUANTPAIR_ROWS = 6, QV2_K_HIST = 7,
  QV2_K_SINGLE_READ_ROWS = 8, QV2_K_STATSPAIR_STREAM = 9,
  QV2_K_COUNT = 10
} qv2_kernel_id;
qv2_status qv2_plan_set_timing(qv2_plan* plan, int32_t enable);
/* Restricts the bracketing to one kernel (a qv2_kernel_id; -1 = all again): every pair of events
 * between two dependent launches costs a few microseconds of device time, which matters on small
 * tensor sets.  Forgets the durations recorded so far. */
qv2_status qv2_plan_time_only(qv2_plan* plan, int32_t kernel);
qv2_status qv2_plan_kernel_ms(const qv2_plan* plan, int32_t kernel, float* ms_out);
/* All QV2_K_COUNT durations in one call: ms_out[QV2_K_COUNT], HOST, written. */
qv2_status qv2_plan_kernels_ms(const qv2_plan* plan, float* ms_out);

/* ---- device passes ------------------------------------------------------- */

/* Step 1-2 (Sec. 4; Sec. 5 calibration stage; Eq. 2, Eq. 4): per segment
 * min, max, sum x, sum x^2, then scale / inv_scale / zero-point.
 * d_params[num_segments], d_sums[num_segments]: DEVICE, written. */
qv2_status qv2_calibrate(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums,
                         void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Step 2-3 (Eq. 1, 3, 5; Eq. 6-7): quantize every element with its segment's
 * parameters, write the int8 code (where codes != NULL), dequantize and
 * accumulate sum x^2 and sum (x - xhat)^2 per segment.
 * d_params: DEVICE, read.  d_sums: DEVICE, sum_e2 / sum_x2 / n written. */
qv2_status qv2_fakequant_metrics(qv2_plan* plan, const qv2_qparams* d_params, qv2_sums* d_sums,
                                 void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Step 3 on the two-inference protocol (Algorithm 2, CalculateSQNR /
 * CalculateMSE on D[i], Q[i]): for every tensor with qrun != NULL the energies
 * sum x^2 and sum (x - qrun)^2.  d_pair_sums[num_tensors]: DEVICE, written. */
qv2_status qv2_pair_metrics(qv2_plan* plan, qv2_pair_sums* d_pair_sums,
                            void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Steps 2-3 in one sweep: the result of qv2_fakequant_metrics followed by
 * qv2_pair_metrics, with every tensor read from HBM once instead of twice
 * (per element 4 B x + 4 B qrun read, 1 B code written, instead of 5 + 8 B).
 * Both comparisons of step 3 (tensor vs its dequantized form, Eq. 6-7; fp32-run
 * vs quantized-run output, Algorithm 2) are taken in the same visit of x.
 * Arguments as in the two separate calls.  Codes, sum_x2 and sum_e2 are
 * bit-identical to qv2_fakequant_metrics; the pair sums equal those of
 * qv2_pair_metrics up to fp64 summation order (the two passes cut tensors into
 * tiles of different length). */
qv2_status qv2_fakequant_pair_metrics(qv2_plan* plan, const qv2_qparams* d_params,
                                      qv2_sums* d_sums, qv2_pair_sums* d_pair_sums,
                                      void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Steps 1-3 in one call (Sec. 4 steps 1-3; Eq. 1-5; Algorithm 2's D[i] / Q[i]): the
 * results of qv2_calibrate followed by qv2_fakequant_pair_metrics (parameters, codes, sum_x
 * and sum_e2 bit for bit; sum_x2, which stays the calibration sweep's instead of being summed
 * again, and the pair sums up to fp64 summation order), with every tensor
 * made of short segments (per-output-channel tensors whose channel has at most 8192
 * elements - at most 32768 when the channels are whole 16-byte vectors on 16-byte boundaries
 * and the code buffer is 4-byte aligned) read from HBM ONCE: a group of whole channels is held
 * in registers (or staged in LDS), and range, parameters, codes and energies of each channel
 * are taken from that copy.  Longer
 * segments still need two reads (their scale depends on the global range); the comparison
 * with qrun rides on the first, read-only one, the second writes the codes.
 * d_params, d_sums: DEVICE, written.  d_pair_sums[num_tensors]: DEVICE, written; NULL
 * skips the comparison with qrun (the results are then those of qv2_calibrate followed
 * by qv2_fakequant_metrics).  Workspace, stream and errors as in the separate calls. */
qv2_status qv2_calibrate_fakequant_pair_metrics(qv2_plan* plan, qv2_qparams* d_params,
                                                qv2_sums* d_sums, qv2_pair_sums* d_pair_sums,
                                                void* d_workspace, size_t workspace_bytes,
                                                void* hip_stream);

/* For callers that cannot allocate - code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: qv2_calibrate_fakequant_pair_metrics without a workspace
 * argument and without any allocation, by this library or a library it calls.  The partial
 * records go to a fixed array in device memory that belongs to the library (QV2_STATIC_SCRATCH_BYTES,
 * one copy per GPU, held until the process ends); outputs and results are those of
 * qv2_calibrate_fakequant_pair_metrics, bit for bit.
 * The plan must already be on the current device (qv2_plan_upload, or any earlier device call
 * on it): otherwise ERR_STATE.  A plan whose qv2_workspace_bytes() exceeds
 * QV2_STATIC_SCRATCH_BYTES is refused with ERR_WORKSPACE.  Every call on a GPU shares that GPU's
 * array: calls that may overlap in time on one GPU (two streams, two threads, two plans) race
 * and must use the entry point with a workspace argument instead.  Nothing in the array has to
 * be cleared between calls (each call writes every record it later reads).
 * Other errors: ERR_NULL, ERR_ALIGN, ERR_HIP (another device current than the plan's; the
 * array's address could not be obtained; a launch failed). */
#define QV2_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
qv2_status qv2_calibrate_fakequant_pair_metrics_noalloc(qv2_plan* plan, qv2_qparams* d_params,
                                                        qv2_sums* d_sums, qv2_pair_sums* d_pair_sums,
                                                        void* hip_stream);

/* qv2_calibrate_fakequant_pair_metrics that also accumulates the cross terms of the cosine
 * similarity (Sec. 6.1 Eq. 8): d_seg_xxhat[num_segments] and d_pair_xq[num_tensors] as in
 * qv2_fakequant_pair_metrics_cos (DEVICE, written, 8-byte aligned; all three of d_pair_sums,
 * d_seg_xxhat and d_pair_xq are required).  sum x * qrun is taken in the read-only calibration
 * sweep and sum x * xhat in the quantize sweep, so the cosine costs no extra pass over memory. */
qv2_status qv2_calibrate_fakequant_pair_metrics_cos(qv2_plan* plan, qv2_qparams* d_params,
                                                    qv2_sums* d_sums, qv2_pair_sums* d_pair_sums,
                                                    double* d_seg_xxhat, double* d_pair_xq,
                                                    void* d_workspace, size_t workspace_bytes,
                                                    void* hip_stream);

/* qv2_fakequant_pair_metrics that also accumulates the cross terms of the cosine
 * similarity (Sec. 6.1 Eq. 8, one of the paper's four candidate local metrics):
 *   d_seg_xxhat[num_segments] : sum x * xhat per segment (tensor vs its dequantized form)
 *   d_pair_xq[num_tensors]    : sum x * qrun per tensor (0 for tensors without qrun)
 * Both DEVICE, written, 8-byte aligned.  All other outputs as qv2_fakequant_pair_metrics
 * (codes, sum_x2, sum_e2 bit-identical to it).  The norms of xhat and qrun follow from
 * the energies already kept: sum b^2 = sum (a-b)^2 - sum a^2 + 2 sum a*b. */
qv2_status qv2_fakequant_pair_metrics_cos(qv2_plan* plan, const qv2_qparams* d_params,
                                          qv2_sums* d_sums, qv2_pair_sums* d_pair_sums,
                                          double* d_seg_xxhat, double* d_pair_xq,
                                          void* d_workspace, size_t workspace_bytes,
                                          void* hip_stream);

/* Calibration histograms (Sec. 5, calibration stage): for every tensor the counts of x,
 * and of qrun where present, over nbins equal bins of the tensor's calibrated range
 * [min, max] (taken from d_params; for a per-channel tensor the range over its channels).
 * The paper gives no binning rule; this library's, in fp32 with one rounding per step:
 *   inv_w = nbins / (max - min)   (0 when max - min is not positive and finite)
 *   bin   = clamp(floor((v - min) * inv_w), 0, nbins - 1)
 * so values of qrun outside x's range fall into the edge bins.
 * nbins: 2 .. 4096.  d_hist_x, d_hist_q: DEVICE, num_tensors * nbins uint64 counts each,
 * written; d_hist_q may be NULL; rows of tensors without qrun are zero.
 * d_workspace: at least qv2_histogram_workspace_bytes(plan, nbins) bytes (that function
 * returns 0 for a bad nbins).  Per element 4 B read per stream.
 * Errors: ERR_NULL, ERR_SHAPE (nbins), ERR_WORKSPACE, ERR_ALIGN, ERR_HIP. */
size_t qv2_histogram_workspace_bytes(const qv2_plan* plan, int32_t nbins);
qv2_status qv2_histogram(qv2_plan* plan, const qv2_qparams* d_params, int32_t nbins,
                         uint64_t* d_hist_x, uint64_t* d_hist_q, void* d_workspace,
                         size_t workspace_bytes, void* hip_stream);

/* Conv + BN folding (Sec. 6.3 Eq. 10-12), the weights of the fused graph IR: per output
 * channel c, f_c = gamma_c / sqrt(var_c) (no epsilon, as printed), w_out = f_c * w,
 * bias_out_c = f_c * (bias_c - mean_c) + beta_c; fp32, one rounding per operation.
 * All pointers DEVICE.  d_w, d_w_out: channels * inner floats (may alias); the per-channel
 * vectors have `channels` entries.  d_bias may be NULL (taken as 0); d_bias_out may be NULL
 * (then d_mean and d_beta are not needed).  channels: 1 .. 65535.
 * Errors: ERR_NULL, ERR_SHAPE, ERR_HIP. */
qv2_status qv2_bn_fold(const float* d_w, int32_t channels, int64_t inner, const float* d_gamma,
                       const float* d_var, const float* d_bias, const float* d_mean,
                       const float* d_beta, float* d_w_out, float* d_bias_out, void* hip_stream);

/* Folds the per-segment params / sums of every tensor into one record per tensor (sums of
 * the channels' sums, min / max over channels) in a fixed order.
 * d_params, d_sums: DEVICE, read; d_tensor_sums[num_tensors]: DEVICE, written. */
qv2_status qv2_tensor_sums_fold(qv2_plan* plan, const qv2_qparams* d_params, const qv2_sums* d_sums,
                                qv2_tensor_sums* d_tensor_sums, void* hip_stream);

/* ---- host finalize and ranking (need no GPU) ----------------------------- */

/* Eq. 6-7 and the tensor statistics from host copies of params and sums; a
 * per-channel tensor's metrics come from the sums of its channels' sums.
 * h_out[num_tensors].  ERR_NONFINITE if any sum is NaN / Inf (outputs still
 * written). */
qv2_status qv2_finalize(const qv2_plan* plan, const qv2_qparams* h_params,
                        const qv2_sums* h_sums, qv2_metrics* h_out);

/* qv2_finalize from host copies of per-tensor records (qv2_tensor_sums_fold). */
qv2_status qv2_finalize_tensors(const qv2_tensor_sums* h_tensor_sums, int32_t n_tensors,
                                qv2_metrics* h_out);

/* MSE and SQNR (dB) of n pair-sum records; entries with n == 0 give 0 and +inf. */
qv2_status qv2_pair_finalize(const qv2_pair_sums* h_pair, int32_t n,
                             double* h_mse, double* h_sqnr_db);

/* Eq. 8 per tensor from host copies of the sums and cross terms:
 * h_cos_quant[num_tensors] = cos(x, xhat) (a per-channel tensor as one vector),
 * h_cos_pair[num_tensors] = cos(x, qrun), NaN for tensors without qrun.
 * A zero vector: 1 when both vectors are zero, else 0 (the paper is silent).
 * ERR_NONFINITE if any input sum is NaN / Inf (outputs still written). */
qv2_status qv2_cosine_finalize(const qv2_plan* plan, const qv2_sums* h_sums,
                               const double* h_seg_xxhat, const qv2_pair_sums* h_pair,
                               const double* h_pair_xq, double* h_cos_quant, double* h_cos_pair);

/* Sec. 6.1 Eq. 9: KL(P || Q) = sum_i P_i ln(P_i / Q_i) between two histograms over the same
 * bins (P: original layer output, Q: quantized layer output), with
 * P_i = (count_i + eps) / (total + eps * nbins).  eps = 0 is the plain definition: empty P
 * bins contribute 0, an empty Q bin under a non-empty P bin gives +inf.  The paper names no
 * smoothing constant; eps is the caller's choice.
 * Errors: ERR_NULL, ERR_SHAPE (nbins <= 0, an empty histogram), ERR_NONFINITE (eps < 0 / NaN). */
qv2_status qv2_kl_divergence(const uint64_t* h_hist_p, const uint64_t* h_hist_q, int32_t nbins,
                             double eps, double* kl_out);

void qv2_rank_config_default(qv2_rank_config* cfg);

/* Step 4 (Eq. 16; Algorithm 2).  Per layer i (0..n_layers-1, in graph order):
 *   delta_i = (SQNR_i - SQNR_{i-1}) / (L_i - L_{i-1}), delta_0 = 0, for the weight
 *   and the activation series; score_i = alpha_w*delta^w_i + alpha_a*delta^a_i;
 *   layers whose MSE exceeds mse_factor x the mean MSE come first, largest MSE
 *   first; the rest follow in ascending score; equal keys keep layer order.
 * w_sqnr_db / a_sqnr_db: either may be NULL (its deltas count as 0), not both.
 * w_mse / a_mse: the one(s) cfg->mse_source selects must be non-NULL, finite, >= 0.
 * layer_pos: graph positions L_i, strictly increasing; NULL = 0..n-1.
 * order_out[n_layers]: layer indices, most sensitive (keep in fp32) first.
 * score_out[n_layers] (may be NULL): the scores, indexed by layer.
 * Errors: ERR_NULL, ERR_SHAPE (n_layers <= 0, positions not increasing,
 * mse_source out of range), ERR_NONFINITE (NaN SQNR, non-finite or negative MSE). */
qv2_status qv2_rank(const double* w_sqnr_db, const double* a_sqnr_db,
                    const double* w_mse, const double* a_mse,
                    const int32_t* layer_pos, int32_t n_layers,
                    const qv2_rank_config* cfg, int32_t* order_out, double* score_out);

/* Step 4 straight from the per-tensor records of a plan (qv2_tensor_sums_fold and the pair
 * sums): the layer table's `kind` and `layer` fields route every tensor to its layer's series -
 * a weight (kind 0) gives the layer's weight SQNR / MSE (Eq. 6-7 against its own dequantized
 * form), an activation (kind 1) with qrun gives the activation SQNR / MSE (fp32 run against
 * quantized run); activations without qrun are ignored - and qv2_rank does the rest.
 * A series must have an entry for every layer 0..n_layers-1 or for none (then it is left out,
 * as a NULL series of qv2_rank; cfg->mse_source must then name the other one).
 * h_tensor_sums[num_tensors], h_pair_sums[num_tensors] (may be NULL when no tensor has qrun).
 * Errors: as qv2_rank, plus ERR_SHAPE for a layer index outside 0..n_layers-1, two tensors
 * of one kind in a layer, or a series with gaps. */
qv2_status qv2_rank_tensors(const qv2_plan* plan, const qv2_tensor_sums* h_tensor_sums,
                            const qv2_pair_sums* h_pair_sums, const int32_t* layer_pos,
                            int32_t n_layers, const qv2_rank_config* cfg, int32_t* order_out,
                            double* score_out);

/* Steps 1-4 in one host call: the device work of qv2_calibrate_fakequant_pair_metrics, whose
 * last fold here also makes the per-tensor records of qv2_tensor_sums_fold (same bits), then
 * Eq. 6-7 for every tensor and pair and qv2_rank_tensors on the host.  Unlike the device calls
 * above it waits for hip_stream (the ranking needs the records), so it returns with every
 * output valid.
 * d_records / h_records: num_tensors qv2_tensor_sums followed by num_tensors qv2_pair_sums
 *   (80 bytes per tensor), DEVICE and HOST, 8-byte aligned; both are written.  When h_records
 *   is pinned host memory that the device can address (hipHostMalloc), the fold kernels write
 *   every record there as well and no copy follows; otherwise one copy brings them over.
 * d_params / d_sums / d_workspace / hip_stream: as in qv2_calibrate_fakequant_pair_metrics.
 * layer_pos / n_layers / cfg / order_out / score_out: as in qv2_rank_tensors.
 * h_metrics[num_tensors], h_pair_mse[num_tensors], h_pair_sqnr_db[num_tensors]: each may be
 *   NULL; entries of tensors without qrun hold MSE 0 and SQNR +inf.
 * Errors: those of the calls it makes.  Non-finite sums (a NaN or Inf among the inputs) are
 * reported as ERR_NONFINITE only after every output has been written: the metrics of every
 * tensor (those of the tensors without such values are unaffected), and the list - which is the
 * true list when the affected tensors are not part of a series the ranking uses, and otherwise
 * (the ranking cannot order a NaN) layer order 0..n_layers-1 with NaN scores. */
qv2_status qv2_sensitivity_pass(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums,
                                void* d_records, void* h_records, void* d_workspace,
                                size_t workspace_bytes, void* hip_stream,
                                const int32_t* layer_pos, int32_t n_layers,
                                const qv2_rank_config* cfg, qv2_metrics* h_metrics,
                                double* h_pair_mse, double* h_pair_sqnr_db, int32_t* order_out,
                                double* score_out);

/* qv2_sensitivity_pass in two halves, so that a caller who runs pass after pass (a calibration
 * service; a sweep over rank configurations) can overlap the host half of one pass with the device
 * half of the next.  _begin enqueues the device work (and the copy of the records, where
 * h_records is not pinned) on hip_stream and marks its end with one of the plan's two
 * completion events (slot 0 or 1; created on first use); it does not wait.  _end waits for that mark, then finalizes and ranks as
 * qv2_sensitivity_pass does, from the same h_records.  Two passes may be in flight on one plan
 * when they use different slots and different h_records (which should be pinned, or the copy
 * blocks); they share the device buffers, which is safe on one stream.  Arguments and errors as
 * in qv2_sensitivity_pass; slot outside 0..1 -> ERR_SHAPE; _end on a slot that never began ->
 * ERR_STATE. */
qv2_status qv2_sensitivity_pass_begin(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums,
                                      void* d_records, void* h_records, void* d_workspace,
                                      size_t workspace_bytes, void* hip_stream, int32_t slot);
qv2_status qv2_sensitivity_pass_end(qv2_plan* plan, const void* h_records, int32_t slot,
                                    const int32_t* layer_pos, int32_t n_layers,
                                    const qv2_rank_config* cfg, qv2_metrics* h_metrics,
                                    double* h_pair_mse, double* h_pair_sqnr_db, int32_t* order_out,
                                    double* score_out);

/* ---- after the ranking: baselines and the BOPs cut (Sec. 7; need no GPU) ---- */

/* Sensitivity lists of the paper's two compile-time baselines, in this library's
 * convention (index 0 = the layer kept in fp32 first).
 *  QV2_ORDER_INORDER: quantization proceeds from the first layer on, so the layers
 *    still in fp32 at any budget are the last ones: n-1, ..., 0 (w_sqnr_db unused).
 *  QV2_ORDER_WEIGHT_SQNR: ascending weight SQNR, equal values keep layer order.
 * Errors: ERR_NULL, ERR_SHAPE (n_layers <= 0), ERR_SCHEME (unknown kind),
 * ERR_NONFINITE (NaN SQNR). */
typedef enum { QV2_ORDER_INORDER = 0, QV2_ORDER_WEIGHT_SQNR = 1 } qv2_baseline;
qv2_status qv2_baseline_order(int32_t kind, const double* w_sqnr_db, int32_t n_layers,
                              int32_t* order_out);

/* Eq. 17: BOPs reduction rate (%) = (1 - sum bits_i*MAC_i / sum 32*MAC_i) * 100 with
 * bits_i = 32 where keep_fp32[i] != 0, else 8.  macs: finite, >= 0, not all zero
 * (else ERR_NONFINITE). */
qv2_status qv2_bops_reduction_pct(const double* macs, const uint8_t* keep_fp32, int32_t n_layers,
                                  double* pct_out);

/* Cuts a sensitivity list for a target BOPs reduction rate: layers are taken from the
 * head of `order` and kept in fp32 while the rate stays >= target_pct; the walk stops
 * at the first layer that would push it below (a prefix of the list is kept).
 * keep_fp32_out[n_layers] by layer index; n_keep_out / achieved_pct_out may be NULL.
 * Errors: ERR_NULL, ERR_SHAPE (n_layers <= 0, order not a permutation),
 * ERR_NONFINITE (bad macs or NaN target). */
qv2_status qv2_bops_select(const int32_t* order, const double* macs, int32_t n_layers,
                           double target_pct, uint8_t* keep_fp32_out, int32_t* n_keep_out,
                           double* achieved_pct_out);

/* Step 5 (Sec. 4): writes the configuration that states every layer's bit-width - 32 for the
 * layers kept in fp32 (keep_fp32[i] != 0, e.g. from qv2_bops_select), 8 for the others - as a
 * text table in layer order: a header line "layer,name,bits", then "<index>,<name>,<32|8>".
 * The paper hands this file to its compiler and prints no format; this one is the library's.
 * path: HOST file name, created or truncated.  layer_names: n_layers NUL-terminated names
 * without commas or line breaks, or NULL (then "layer<index>").
 * Errors: ERR_NULL, ERR_SHAPE (n_layers <= 0, a name with a comma or line break), ERR_IO. */
qv2_status qv2_write_config(const char* path, const uint8_t* keep_fp32,
                            const char* const* layer_names, int32_t n_layers);

/* Fusion-aware adjustment of a sensitivity list (Sec. 6.5 only allows the positions of
 * fusion-capable operators to change and gives no rule; this is the reading taken): layers with the
 * same group_id (a convolution and the BN / Add / ReLU neighbours it fuses with) keep one
 * precision, so each group moves as a block to the position of its most sensitive member;
 * list order is kept inside a block and between blocks.  order_out may not alias order.
 * Errors: ERR_NULL, ERR_SHAPE (n_layers <= 0, order not a permutation). */
qv2_status qv2_regroup_for_fusion(const int32_t* order, const int32_t* group_id, int32_t n_layers,
                                  int32_t* order_out);

const char* qv2_status_string(qv2_status s);

#ifdef __cplusplus
}
#endif
#endif /* QV2_H */
