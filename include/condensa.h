/*
 * condensa.h -- C ABI of the compression step of Condensa's L-C optimizer on MI355X (gfx950).
 *
 * The library applies the paper's per-layer compression operators (Section 3.1: quantize /
 * dequantize, prune, filter_prune, blockprune) in their whole-model "scheme" form (Table 1:
 * Quantize, Prune, FilterPrune, BlockPrune, Compose) to a list of weight tensors, and the
 * compression (C) step of the L-C algorithm with its multiplier update (Section 3.3).  A target
 * sparsity s (Introduction: proportion of zero-valued parameters) is passed as the density
 * d = 1 - s; the library turns it into an exact kept count and a magnitude threshold
 * (Section 3.1: the schemes derive the magnitude threshold from the sparsity).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Pointers named *_dev and every pointer stored inside a table are DEVICE pointers.  The
 *    tables themselves (arrays of condensa_tensor, arrays of pointers, arrays of densities) are
 *    HOST memory; they are consumed before the call returns and may be freed right after.
 *  - The caller owns all memory, including the workspace.  The library allocates no device
 *    memory and frees none.  (It keeps a small pinned host staging ring for the tables.)
 *  - All device work is enqueued on `stream` (a hipStream_t, NULL = the default stream) and the
 *    call returns without waiting.  Results, including condensa_select records, are in device
 *    memory once the stream has reached that point.
 *  - Return value: CONDENSA_OK or a negative error code.  Argument errors are found before
 *    anything is enqueued, so a failing call has no side effect.
 *  - Tensors are fp32, row-major, contiguous.  16-byte aligned pointers get 128-bit accesses,
 *    any other alignment is accepted and takes a scalar path.
 *  - The flat index of an element is its position in the concatenation of the call's tensors in
 *    table order.  Tensors with zero elements and calls with zero tensors are valid.  A call may
 *    carry at most 3 * 2^32 (12 884 901 888) elements in total (CONDENSA_ERR_SIZE beyond that).
 *  - kept count  k = llround(density * N) (binary64 product, halves away from zero), clamped to
 *    [0, N]; density must lie in [0, 1].
 *  - Ordering key of a value x is the bit pattern of |x|: -0 equals +0, infinities rank above
 *    every finite value and NaN patterns above infinity.  Among equal keys the lowest index is
 *    kept first.  Pruned positions are written as +0.0; kept values are copied bit for bit.
 *  - Masks are one byte per element, 1 = kept, 0 = pruned.
 *  - Calls that share a workspace must be ordered on one stream.
 *  - Buffers of one call must not overlap in memory (byte ranges are compared, not just start
 *    addresses): every output, the workspace included, against every input and against every other
 *    output; CONDENSA_ERR_ARG otherwise.  The only exception is the exact in-place form that an entry
 *    point documents (theta == w, lambda updated in place).
 *  - Every entry point that takes a workspace also takes `config`, the tuning knobs of THIS call
 *    (condensa_config below); NULL means the process-wide defaults.  Two callers with different
 *    settings therefore never interfere.
 */
#ifndef CONDENSA_H
#define CONDENSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t condensa_status;

enum {
    CONDENSA_OK            = 0,
    CONDENSA_ERR_NULL      = -1,  /* a required pointer is NULL                                  */
    CONDENSA_ERR_SIZE      = -2,  /* negative count, too many tensors/densities, size overflow   */
    CONDENSA_ERR_DENSITY   = -3,  /* density outside [0,1] or NaN; mu not finite and positive    */
    CONDENSA_ERR_SHAPE     = -4,  /* ndim/shape not valid for the operator, block does not divide */
    CONDENSA_ERR_WORKSPACE = -5,  /* workspace NULL, misaligned (256 B) or too small             */
    CONDENSA_ERR_ARG       = -6,  /* bad scope / option / aliasing                               */
    CONDENSA_ERR_HIP       = -7   /* a HIP runtime call failed (see condensa_last_hip_error)     */
};

enum { CONDENSA_SCOPE_GLOBAL = 0,       /* one ranking over all tensors of the call              */
       CONDENSA_SCOPE_PER_TENSOR = 1 }; /* every tensor ranked on its own                         */

enum { CONDENSA_OP_PRUNE = 0,        /* condensa_prune                                               */
       CONDENSA_OP_FILTER_PRUNE = 1, /* condensa_filter_prune, _neuron_prune, _structure_prune        */
       CONDENSA_OP_BLOCK_PRUNE = 2,  /* condensa_block_prune, _block_prune_nd                         */
       CONDENSA_OP_QUANTIZE = 3,
       CONDENSA_OP_LC_STEP = 4,      /* condensa_lc_step, _lc_step_pq                                 */
       CONDENSA_OP_COUNT_NONZERO = 5,
       CONDENSA_OP_LC_SGD_STEP = 6 };

#define CONDENSA_MAX_DENSITIES 16
#define CONDENSA_MAX_TENSORS   65536

/* One weight tensor (Section 3.1: operators are applied per layer; schemes walk all layers). */
typedef struct {
    const float* w;        /* device, fp32 row-major contiguous; may be NULL iff it has 0 elements */
    int64_t      shape[4]; /* conv [Cout,Cin,kh,kw]; matrix [R,C]; vector [n]; unused dims ignored */
    int32_t      ndim;     /* 1..4                                                                 */
    int32_t      reserved; /* must be 0                                                            */
} condensa_tensor;

/*
 * Outcome of one ranking (one per density, and per tensor under PER_TENSOR scope).  Element
 * pruning ranks the 31-bit |x| patterns, structure pruning the binary64 patterns of the
 * structures' sums of squares.  An element/structure with key K and index i (flat index for
 * GLOBAL scope, index inside the tensor for PER_TENSOR) is kept iff
 *      K > threshold_key  ||  (K == threshold_key && i < tie_end).
 */
typedef struct {
    uint64_t n;             /* population size                                                     */
    uint64_t k;             /* kept count                                                          */
    uint64_t n_gt;          /* keys strictly above the threshold                                   */
    uint64_t n_tie_kept;    /* keys equal to the threshold that are kept ( = k - n_gt )            */
    uint64_t n_tie;         /* keys equal to the threshold                                         */
    uint64_t threshold_key; /* the k-th largest key; UINT64_MAX when k == 0                        */
    uint64_t tie_end;       /* n when all ties are kept, else 1 + index of the last kept tie; 0 if k == 0 */
    uint64_t path;          /* diagnostic: 1 = radix levels over the data, 2 = sampled window,
                               3 = sampled window missed, radix levels as fallback                 */
} condensa_select;

/*
 * Tuning / test knobs of one call.  They choose between forms of the computation that give the same
 * results; normal use passes NULL.  condensa_config_init fills a struct with the process-wide defaults
 * (what NULL stands for), after which single fields can be changed.  Invalid values: CONDENSA_ERR_ARG.
 */
typedef struct {
    int32_t select_path;    /* 0 auto, 1 radix levels over the data only (structure calls: one launch per
                               level), 2 sampled window even for small N (8x8 block pruning: aggregation
                               and apply in one sweep whatever the number of blocks, where shapes allow) */
    int32_t sample_log2;    /* log2 of the sample size of the window path (10..26); 0 = auto           */
    int32_t window_margin;  /* half-width of the sampled window in 1/16 standard deviations of the sample
                               rank; default 80 (= 5 sigma of a sample whose units of 4 neighbours are
                               fully correlated, i.e. 10 sigma of independent draws); 0 makes windows miss */
    int32_t cand_shift;     /* candidate capacity = N >> value (1..30); 0 = auto                        */
    int32_t profile;        /* bit p set: bracket phase p of the call with HIP events on its stream     */
    int32_t apply_threads;  /* workgroup size of the two-sweep L-C apply: 0 (default = 64), 64, 128, 256 */
    int32_t fused_sweep;    /* window path with one density: 0 = selection and apply share one sweep when
                               the outputs do not alias the inputs, 1 = always two sweeps               */
    int32_t reserved;       /* must be 0                                                               */
} condensa_config;
condensa_status condensa_config_init(condensa_config* config);

/*
 * Bytes of workspace (256-byte aligned device memory) the operator needs for the given problem:
 * total_elems = sum of tensor sizes, n_structures = number of filters/blocks (0 for element
 * operators).  The size depends on sample_log2 and cand_shift of `config`: size the workspace with the
 * config the call will get.  Returns 0 for invalid arguments.  CONDENSA_OP_QUANTIZE needs none (returns 0).
 */
size_t condensa_workspace_bytes(int op, uint64_t total_elems, uint64_t n_structures,
                                int n_tensors, int n_densities, int scope, const condensa_config* config);

/*
 * Prune() scheme / prune operator: unstructured magnitude pruning (Background: magnitude
 * thresholding; Section 3.3: Theta is made sparse by dropping the weights of lowest magnitude;
 * Table 1).  Serves n_densities target densities from one sweep over the weights, which is what a
 * sparsity search with up to 10 samples per search (Results) asks of the same reference weights.
 * Optionally fuses Quantize(float16) (Evaluation, Objective 1: Compose([Prune(), Quantize(float16)])).
 *
 *  tensors, n_tensors     host table of the weight tensors
 *  densities, n_densities host array, 1..CONDENSA_MAX_DENSITIES values in [0,1]
 *  scope                  GLOBAL: one threshold for the whole call; PER_TENSOR: one per tensor
 *  theta                  NULL, or host table [n_densities * n_tensors] (entry j*n_tensors + t) of
 *                         device fp32 outputs shaped like tensor t; entries may be NULL (skipped).
 *                         theta may alias w only when n_densities == 1.
 *  theta_f16              same layout, binary16 bit patterns of round-to-nearest-even(theta)
 *  mask                   same layout, bytes
 *  results_dev            device array: [n_densities] for GLOBAL, [n_densities * n_tensors] for
 *                         PER_TENSOR (entry j*n_tensors + t)
 *  workspace_dev/bytes    see condensa_workspace_bytes(CONDENSA_OP_PRUNE, ...)
 * With theta, theta_f16 and mask all NULL only the thresholds are computed.
 * One density, GLOBAL scope, large tensors and theta not aliasing w: the selection and the outputs come
 * from ONE sweep over the weights (see condensa_config.fused_sweep); results are the same either way.
 */
condensa_status condensa_prune(const condensa_tensor* tensors, int n_tensors,
                               const double* densities, int n_densities, int scope,
                               float* const* theta, uint16_t* const* theta_f16, uint8_t* const* mask,
                               condensa_select* results_dev,
                               void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/*
 * condensa_prune for callers that cannot allocate device memory or provide a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  GLOBAL scope, same outputs and
 * records as condensa_prune (bit for bit).  The call allocates nothing, on the device or through the
 * runtime: its workspace is a 2 MiB array that is part of the library's device code (every GPU the
 * library runs on holds its own copy until the process ends), the host tables live on the caller's
 * stack and reach the device as kernel arguments, and no timing events are created.  Limits
 * (CONDENSA_ERR_SIZE beyond them): at most CONDENSA_STATIC_MAX_ELEMS elements in total, at most
 * CONDENSA_STATIC_MAX_TENSORS tensors and CONDENSA_STATIC_MAX_DENSITIES densities.  The selection always
 * runs the radix levels over the weights (the form condensa_prune picks by itself below 2^26 elements).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race; order them on one stream.  The first call on a device looks up the array's address.
 */
#define CONDENSA_STATIC_MAX_ELEMS     (1ull << 26)
#define CONDENSA_STATIC_MAX_TENSORS   128
#define CONDENSA_STATIC_MAX_DENSITIES 4
condensa_status condensa_prune_static(const condensa_tensor* tensors, int n_tensors,
                                      const double* densities, int n_densities,
                                      float* const* theta, uint16_t* const* theta_f16, uint8_t* const* mask,
                                      condensa_select* results_dev, void* stream);

/*
 * FilterPrune scheme / filter_prune operator (Table 1, FilterPrune row: whole filters, i.e. the 3-D
 * slices of a convolution weight, are scored and removed; Section 3.1: filter aggregation).  Every tensor must have ndim == 4; filter f of a
 * tensor is the contiguous run of Cin*kh*kw weights of output channel f.  Aggregate: sum of
 * squares in binary64, added in memory order (the ranking of L2 norms); `density` counts filters.
 * Structure ids run over all filters of the call in table order.
 *
 *  theta, mask        NULL or host tables [n_tensors] of device outputs (entries may be NULL)
 *  sumsq_dev          NULL or device double [F]: the aggregates (the ranking keys)
 *  norms_dev          NULL or device float  [F]: (float)sqrt(sumsq)
 *  keep_idx_dev       NULL or device int32  [F]: ids of kept filters, ascending; entries past the
 *                     kept count are not written
 *  structure_mask_dev NULL or device bytes  [F]
 *  results_dev        device: 1 record (GLOBAL) or n_tensors records (PER_TENSOR)
 */
condensa_status condensa_filter_prune(const condensa_tensor* tensors, int n_tensors,
                                      double density, int scope,
                                      float* const* theta, uint8_t* const* mask,
                                      double* sumsq_dev, float* norms_dev, int32_t* keep_idx_dev,
                                      uint8_t* structure_mask_dev, condensa_select* results_dev,
                                      void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/*
 * BlockPrune scheme / blockprune operator for 2-D blocks (Table 1, BlockPrune row: blocks of a given
 * size are scored and removed).  Every tensor must have ndim == 2 with block_h | R and block_w | C
 * (CONDENSA_ERR_SHAPE otherwise).  Block ids are row-major over the block grid of a matrix,
 * matrices in table order; inside a block the squares are added in row-major order.
 * Other arguments as for condensa_filter_prune.
 */
condensa_status condensa_block_prune(const condensa_tensor* tensors, int n_tensors,
                                     int block_h, int block_w, double density, int scope,
                                     float* const* theta, uint8_t* const* mask,
                                     double* sumsq_dev, float* norms_dev, int32_t* keep_idx_dev,
                                     uint8_t* structure_mask_dev, condensa_select* results_dev,
                                     void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/*
 * NeuronPrune scheme / neuron_prune operator (Table 1: neurons, seen as 1-D blocks, are aggregated and pruned).
 * Every tensor must have ndim == 2, [out, in]; neuron r is row r (the weights into output unit r).
 * Aggregate, ranking and arguments as for condensa_filter_prune.
 */
condensa_status condensa_neuron_prune(const condensa_tensor* tensors, int n_tensors,
                                      double density, int scope,
                                      float* const* theta, uint8_t* const* mask,
                                      double* sumsq_dev, float* norms_dev, int32_t* keep_idx_dev,
                                      uint8_t* structure_mask_dev, condensa_select* results_dev,
                                      void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/*
 * StructurePrune scheme (Table 1: neuron and filter pruning together): tensors with ndim == 2
 * contribute their neurons, tensors with ndim == 4 their filters, to one list of structures (ids in
 * table order) that is ranked globally or per tensor.  Arguments as for condensa_filter_prune.
 */
condensa_status condensa_structure_prune(const condensa_tensor* tensors, int n_tensors,
                                         double density, int scope,
                                         float* const* theta, uint8_t* const* mask,
                                         double* sumsq_dev, float* norms_dev, int32_t* keep_idx_dev,
                                         uint8_t* structure_mask_dev, condensa_select* results_dev,
                                         void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/*
 * BlockPrune with n-D blocks and ragged edges (Table 1: blocks of any dimensionality and a given size; the evaluation
 * prunes blocks of size 5 in LSTM matrices).  block_shape has block_ndim (1..4) positive entries and
 * every tensor must have ndim == block_ndim.  The block grid has ceil(dim / block) cells per
 * dimension; cells on the far edge of a dimension that the block does not divide are smaller.
 * Block ids are row-major over the grid of a tensor, tensors in table order; inside a block the
 * squares are added in row-major order.  1-D blocks along the rows of a matrix are block_shape
 * {1, bs}.  Other arguments as for condensa_filter_prune.
 */
condensa_status condensa_block_prune_nd(const condensa_tensor* tensors, int n_tensors,
                                        const int32_t* block_shape, int block_ndim,
                                        double density, int scope,
                                        float* const* theta, uint8_t* const* mask,
                                        double* sumsq_dev, float* norms_dev, int32_t* keep_idx_dev,
                                        uint8_t* structure_mask_dev, condensa_select* results_dev,
                                        void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/*
 * Quantize(float16) scheme / quantize + dequantize operators (Section 3.1; Background:
 * low-precision approximation = quantisation with a fixed codebook).  q = binary16 bits of x
 * rounded to nearest even (overflow to infinity, gradual underflow, NaN -> quiet NaN keeping the
 * sign and the top ten payload bits); dq = exact widening of q.  q_dev or dq_dev may be NULL (not
 * both).  n may be 0.  x_dev may alias dq_dev.
 */
condensa_status condensa_quantize(const float* x_dev, uint64_t n, uint16_t* q_dev, float* dq_dev,
                                  void* stream);

/* dequantize operator alone: dq = exact widening of the binary16 bit patterns q. */
condensa_status condensa_dequantize(const uint16_t* q_dev, uint64_t n, float* dq_dev, void* stream);

/*
 * Quantize(dtype) for the other common 16-bit floating-point type, bfloat16 (Table 1: Quantize(dtype);
 * Conclusions: data types for quantization as an extension).  q = upper half of the binary32 pattern
 * after rounding to nearest even on the 16 dropped bits (a carry runs into the exponent: values above the
 * largest finite bfloat16 become infinity; subnormals are kept); NaN -> quiet NaN keeping the sign and
 * the upper payload bits.  dq = exact widening.  Arguments and aliasing as for condensa_quantize /
 * condensa_dequantize.
 */
condensa_status condensa_quantize_bf16(const float* x_dev, uint64_t n, uint16_t* q_dev, float* dq_dev,
                                       void* stream);
condensa_status condensa_dequantize_bf16(const uint16_t* q_dev, uint64_t n, float* dq_dev, void* stream);

/*
 * Quantize(dtype) for the two 8-bit floating-point formats of the OCP 8-bit floating point specification
 * (Table 1: Quantize(dtype); Background: low-precision approximation is quantization with a fixed
 * codebook).  format: CONDENSA_FP8_E4M3 (4 exponent bits, bias 7, 3 fraction bits, no infinity, S.1111.111
 * is NaN, largest finite value 448) or CONDENSA_FP8_E5M2 (5 exponent bits, bias 15, 2 fraction bits,
 * IEEE-like infinities and NaNs, largest finite value 57344); anything else is CONDENSA_ERR_ARG.
 * q = the nearest finite value of the format, ties to the even fraction, subnormals kept.  Finite inputs
 * beyond the largest finite value saturate to it; infinite inputs stay infinite in E5M2 and saturate in
 * E4M3; NaN gives the format's NaN (E5M2: S.11111.10) with the sign kept.  dq = exact widening (NaN codes
 * widen to the binary32 quiet NaN S.0x7FC00000).  q_dev holds one byte per element; q_dev or dq_dev may be
 * NULL (not both); dq_dev may alias x_dev.  4-byte aligned q_dev and 16-byte aligned x_dev / dq_dev get
 * vector accesses.
 */
enum { CONDENSA_FP8_E4M3 = 0, CONDENSA_FP8_E5M2 = 1 };
condensa_status condensa_quantize_fp8(const float* x_dev, uint64_t n, int format, uint8_t* q_dev, float* dq_dev,
                                      void* stream);
condensa_status condensa_dequantize_fp8(const uint8_t* q_dev, uint64_t n, int format, float* dq_dev, void* stream);

/*
 * One compression step of the L-C algorithm with the augmented-Lagrangian updates (Section 3.3;
 * mu_j = mu_0 a^j is the caller's schedule, L-C Optimizer Settings).  Per element, in binary32
 * with one rounding per operation and no fused multiply-add:
 *      t = lambda / mu;  v = w - t;
 *      theta = prune(v) at `density`, one global ranking over all tensors of the call;
 *      e = w - theta;  p = mu * e;  lambda' = lambda - p;  g = p - lambda'.
 * theta is C(w - lambda/mu), lambda' the new multiplier estimate and g = mu (w - theta) - lambda'
 * the gradient of the penalty that the next learning step adds to the loss gradient.
 *
 *  lambda      host table [n_tensors] of device fp32 multipliers shaped like the weights
 *  lambda_out  NULL (update lambda in place) or host table of device outputs; with separate outputs and
 *              large tensors the whole step reads w and lambda once (condensa_config.fused_sweep), in place
 *              it reads them twice
 *  theta, grad, mask  NULL or host tables [n_tensors]; entries may be NULL (skipped).  None of
 *              them may alias w or lambda.
 *  result_dev  device, one record
 */
condensa_status condensa_lc_step(const condensa_tensor* tensors, int n_tensors,
                                 float* const* lambda, float* const* lambda_out,
                                 float mu, double density,
                                 float* const* theta, float* const* grad, uint8_t* const* mask,
                                 condensa_select* result_dev,
                                 void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/*
 * The L-C compression step for the composed scheme Compose([Prune(), Quantize(float16)]) (Evaluation,
 * Objective 1: P+Q).  As condensa_lc_step, except that the pruned v is rounded to binary16
 * (theta_f16: NULL or host table of device outputs holding the bit patterns) and the updates use the
 * decompression D(theta) = exact widening of those patterns (Section 3.3: w = D(Theta)):
 *      theta = widen(binary16(prune(v)));  e = w - theta;  p = mu * e;  lambda' = lambda - p;  g = p - lambda'.
 * `theta`, if given, receives D(theta) in fp32.  The mask still marks the k selected positions, also
 * where a kept value underflows to zero in binary16.
 *  nnz_dev    NULL, or device uint64: receives the memory-footprint objective of the compressed model
 *             (Evaluation, Objective 1) as the number of stored binary16 codes other than +0 and -0, i.e. k
 *             less the kept values that underflow.  It is counted inside the sweeps that write theta: no extra
 *             pass over the model and no host round trip; footprint in bytes = 2 * nnz.
 */
condensa_status condensa_lc_step_pq(const condensa_tensor* tensors, int n_tensors,
                                    float* const* lambda, float* const* lambda_out,
                                    float mu, double density,
                                    float* const* theta, uint16_t* const* theta_f16,
                                    float* const* grad, uint8_t* const* mask, uint64_t* nnz_dev,
                                    condensa_select* result_dev,
                                    void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/*
 * Memory-footprint objective (Evaluation, Objective 1: the bytes taken by the model's non-zero
 * parameters): writes to *count_dev the number of non-zero elements over all tensors; the
 * footprint is that count times the element size.  kind = CONDENSA_COUNT_F32: tensors hold fp32
 * values; CONDENSA_COUNT_CODES16: `w` of every tensor points to 16-bit floating-point codes (binary16 as
 * written to theta_f16, or bfloat16) and shape counts those; CONDENSA_COUNT_CODES8: to 8-bit
 * floating-point codes (condensa_quantize_fp8).  +0 and -0 are zeros.  Workspace:
 * condensa_workspace_bytes(CONDENSA_OP_COUNT_NONZERO, ...).
 */
enum { CONDENSA_COUNT_F32 = 0, CONDENSA_COUNT_CODES16 = 1, CONDENSA_COUNT_CODES8 = 2 };
condensa_status condensa_count_nonzero(const condensa_tensor* tensors, int n_tensors, int kind,
                                       uint64_t* count_dev,
                                       void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/*
 * One SGD-with-momentum update of the learning (L) step with the L-C penalty folded in (Section 3.3:
 * the L step trains the uncompressed model with an added quadratic penalty; L-C Optimizer Settings:
 * SGD, momentum 0.9).  The gradient of L(w) + mu/2 ||w - theta - lambda/mu||^2 is
 * grad L + mu (w - theta) - lambda, so the separate penalty-gradient buffer of condensa_lc_step is not
 * needed.  Per element, binary32, one rounding per operation, no fused multiply-add:
 *      g = (grad_loss + mu * (w - theta)) - lambda;   buf = momentum * buf + g;   w = w - lr * buf.
 * `w` of every tensor in the table and momentum_buf are UPDATED IN PLACE; grad_loss, theta, lambda are
 * host tables [n_tensors] of device inputs shaped like the weights.  The five buffers of a tensor
 * must be distinct.  Workspace: condensa_workspace_bytes(CONDENSA_OP_LC_SGD_STEP, ...).
 */
condensa_status condensa_lc_sgd_step(const condensa_tensor* tensors, int n_tensors,
                                     const float* const* grad_loss, const float* const* theta,
                                     const float* const* lambda, float* const* momentum_buf,
                                     float mu, float lr, float momentum,
                                     void* workspace_dev, size_t workspace_bytes, void* stream,
    const condensa_config* config);

/* mu_j = mu_0 * a^j (L-C Optimizer Settings: mu_0 = 1e-3, a = 1.1), evaluated in binary64 (host). */
float condensa_mu_schedule(double mu0, double a, int j);

/*
 * Network thinning, final phase (Section 3.4): physically remove the zero structures that structure
 * pruning left, given the lists of what to keep.  The tensor [Cout, Cin, ...] (ndim 2..4, `shape` is a
 * HOST array) is gathered into the dense [n_out, n_in, ...] tensor
 *      out[o, i, ...] = w[keep_out[o] - keep_out_offset, keep_in[i] - keep_in_offset, ...].
 * keep_out_dev / keep_in_dev are DEVICE arrays of ids (for example slices of the keep_idx output of
 * the structure-pruning calls, whose ids run over the whole call: pass the tensor's first id as the
 * offset); a NULL list keeps the whole dimension.  The dependency analysis that decides which
 * successor loses which input channels is the caller's (the paper's graph phases are not part of this
 * library).  An id that falls outside the tensor yields zeros, never an out-of-bounds read.
 * out_dev must hold n_out * n_in * prod(shape[2:]) floats and must not alias w_dev.
 */
condensa_status condensa_thin(const float* w_dev, const int64_t* shape, int ndim,
                              const int32_t* keep_out_dev, int64_t n_keep_out, int64_t keep_out_offset,
                              const int32_t* keep_in_dev, int64_t n_keep_in, int64_t keep_in_offset,
                              float* out_dev, void* stream);

/* ---- process-wide DEFAULTS of the knobs above: what a NULL config stands for ---------------------- */
enum {
    CONDENSA_OPT_SELECT_PATH   = 0, /* condensa_config.select_path   */
    CONDENSA_OPT_SAMPLE_LOG2   = 1, /* condensa_config.sample_log2   */
    CONDENSA_OPT_WINDOW_MARGIN = 2, /* condensa_config.window_margin */
    CONDENSA_OPT_CAND_SHIFT    = 3, /* condensa_config.cand_shift    */
    CONDENSA_OPT_PROFILE       = 4, /* condensa_config.profile       */
    CONDENSA_OPT_APPLY_THREADS = 5, /* condensa_config.apply_threads */
    CONDENSA_OPT_FUSED_SWEEP   = 6, /* condensa_config.fused_sweep   */
    CONDENSA_OPT_COUNT         = 7
};
condensa_status condensa_set_option(int option, int64_t value);
int64_t         condensa_get_option(int option);

/*
 * Phase timing (benchmarks).  For every phase whose bit (1 << phase) is set in the call's
 * condensa_config.profile, the entry point records a pair of timing events on the caller's stream around that phase.  condensa_profile_read waits
 * for the recorded events, adds the elapsed milliseconds of all finished intervals of `phase` to
 * its running totals and returns those totals; condensa_profile_reset drops totals and events.
 */
enum {
    CONDENSA_PHASE_SAMPLE    = 0,  /* sampling and the ranking of the sample                        */
    CONDENSA_PHASE_SWEEP     = 1,  /* full sweeps over the weights that feed the selection (the one-sweep
                                      form also writes the outputs here)                          */
    CONDENSA_PHASE_RESOLVE   = 2,  /* ranking of candidates / aggregates, tie search, records       */
    CONDENSA_PHASE_APPLY     = 3,  /* the mask / theta / L-C update kernel, or the fix-up pass after the
                                      one-sweep form                                              */
    CONDENSA_PHASE_AGGREGATE = 4,  /* per-structure sums of squares                                 */
    CONDENSA_PHASE_COUNT     = 5
};
condensa_status condensa_profile_read(int phase, double* total_ms, uint64_t* intervals);
condensa_status condensa_profile_reset(void);

const char* condensa_status_string(condensa_status s);
int         condensa_last_hip_error(void);   /* hipError_t of the last failing runtime call, 0 if none */
/* Diagnostic: kernels the library has enqueued since it was loaded (all threads, all streams); the
   difference around a call is that call's number of launches. */
uint64_t    condensa_launch_count(void);
int         condensa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CONDENSA_H */
