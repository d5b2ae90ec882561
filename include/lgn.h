/*
 * lgn.h -- C interface of the MI355X (gfx950) library for on-the-fly compression of neural
 * gradients after "Neural gradients are near-lognormal: improved quantized and sparse training"
 * (Chmiel et al., ICLR 2021).
 *
 * The path, per gradient tensor g (contiguous, 1-D view, fp32, bf16 or fp16):
 *
 *   lgn_stats      lognormal parameters: mean and standard deviation of ln|g| over the non-zero
 *                  entries, plus counts and extrema                      (Section 3)
 *   lgn_threshold  stochastic-pruning threshold alpha for a target sparsity, from the closed form
 *                  S(alpha)                                              (Section 5.1-5.2)
 *   lgn_fp_params  exponent/mantissa split that minimises the expected relative error, and the
 *                  per-tensor power-of-two gradient scale                (Section 4.2-4.4, Alg. 1)
 *   lgn_prune      stochastic pruning T_{alpha,eps}                      (Section 5, first equation)
 *   lgn_fp_quantize  FP(1,e,m) quantization with scale 2^s               (Section 4.1, Alg. 1)
 *   lgn_prune_quantize_fused   the two operators in one pass
 *   lgn_stats_solve            the first three steps in one launch
 *   lgn_batch_stats_solve, lgn_batch_prune_quantize_fused
 *                              those two launches for many tensors at once (all layers of a network)
 *   lgn_stats_solve_static     lgn_stats_solve for callers that cannot allocate a workspace
 *
 * Beyond that path: the prefix code of a pruned tensor (lgn_prefix_encode / lgn_prefix_decode,
 * appendix "Encoding"), statistics of one mode of a bi-modal gradient (lgn_stats_masked), the
 * stochastic-underflow threshold (lgn_threshold_floor) and heterogeneous per-layer sparsity
 * (lgn_log_histogram, lgn_sparsity_allocate).
 *
 * General rules
 *   - Every pointer argument is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or keeps device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call only
 *     enqueues kernels on that stream and returns; nothing synchronises with the host, and the
 *     parameter structs are read and written on the device, so a whole chain
 *     stats -> threshold -> fp_params -> fused runs without a host round trip.
 *   - n is a 64-bit element count; n = 0 is allowed everywhere.
 *   - Tensor pointers must be 16-byte aligned; CODE8 / PACKED outputs 4-byte aligned.
 *   - Return value: LGN_OK or a negative LGN_ERR_* code; lgn_last_error() gives the text of the
 *     last error on the calling thread.  Conditions that depend on the data (empty tensor, zero
 *     spread, nothing to prune, ...) cannot be reported synchronously and are written to the
 *     `status` bit field of the device structs.
 *   - Random words: Philox4x32-10 keyed by `seed`.  Global element j = elem_offset + i draws word
 *     (j & 3) of the block with counter (lo32(j>>2), hi32(j>>2), 0, 0).  The upper 16 bits of that
 *     word are the element's pruning variable, the lower 16 bits its rounding variable, so
 *     lgn_prune followed by lgn_fp_quantize with the same seed and offset draws what
 *     lgn_prune_quantize_fused draws.  Because the counter is the global index, processing a
 *     tensor in several calls with the matching elem_offset gives the same bits as one call.
 */
#ifndef LGN_H
#define LGN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LGN_VERSION 100

/* return codes */
#define LGN_OK 0
#define LGN_ERR_INVALID_ARG (-1) /* null pointer, misaligned pointer, value out of range */
#define LGN_ERR_UNSUPPORTED (-2) /* unknown dtype / enum                                 */
#define LGN_ERR_WORKSPACE (-3)   /* workspace missing or too small                       */
#define LGN_ERR_DEVICE (-4)      /* the HIP runtime refused a launch                     */

/* element types */
#define LGN_F32 0
#define LGN_BF16 1
#define LGN_F16 2 /* IEEE half precision */

/* rounding of the mantissa */
#define LGN_ROUND_NEAREST_EVEN 0 /* ties to the even FP-n code          */
#define LGN_ROUND_STOCHASTIC 1   /* up with probability (cut-off part)/(spacing), on a 2^-16 grid */

/* what a quantizing call writes */
#define LGN_OUT_VALUE 0  /* n elements of the input dtype holding 2^s * q, rounded to        */
                         /* nearest-even where the dtype cannot hold it (bf16 and fp16      */
                         /* mantissas, subnormal results at very small scales)              */
#define LGN_OUT_CODE8 1  /* n bytes, the N-bit code in the low bits                           */
#define LGN_OUT_PACKED 2 /* little-endian bit stream, code i at bits [i*N, (i+1)*N),          */
                         /* lgn_packed_bytes(n, N) bytes, last byte zero padded               */

/* scale rule (Alg. 1 and Appendix "Neural gradients lognormal distributions are truncated") */
#define LGN_SCALE_QUANTILE 0 /* top binade holds the scale_arg-quantile of the fitted lognormal */
#define LGN_SCALE_MAX 1      /* top binade holds max|g| (Alg. 1 as printed)                    */
#define LGN_SCALE_CENTER 2   /* 2^s is the geometric mean: s = round(mu / ln 2)                */

/* how sigma enters the expected relative error (Section 4.2) */
#define LGN_SIGMA_PAPER_LITERAL 0 /* natural-log sigma used as printed; reproduces Table 2 */
#define LGN_SIGMA_BASE2 1         /* sigma / ln 2, the spread of log2|g|                   */

/* status bits written to the device structs */
#define LGN_ST_EMPTY 1u            /* no finite non-zero element: mu, sigma are NaN, alpha = 0 */
#define LGN_ST_SIGMA0 2u           /* all finite non-zero magnitudes are equal                 */
#define LGN_ST_NOTHING_TO_PRUNE 4u /* existing zeros already reach the target: alpha = 0       */
#define LGN_ST_NOT_CONVERGED 8u    /* the threshold solve hit its iteration limit              */
#define LGN_ST_ALPHA_BELOW_FP_RANGE 16u /* pruning params only: 0 < alpha < 2^(E_min + s), the smallest
                                           magnitude of the format the threshold is used with, so the
                                           quantizer flushes every +-alpha pruning produces.  Set by
                                           lgn_stats_solve (it computes both) and by
                                           lgn_threshold_floor (which then raises alpha); lgn_threshold
                                           alone does not know the format and never sets it          */
#define LGN_ST_HAS_NONFINITE 32u   /* Inf / NaN entries were seen (and skipped by the statistics);
                                      copied from the statistics into both parameter structs, so it
                                      travels with the codes: a NaN has no code of its own and
                                      comes out as the largest code of its sign                  */

/* Result of lgn_stats (device memory, 72 bytes, 8-byte aligned). */
typedef struct lgn_stats_t {
    uint64_t n;           /* elements scanned                                             */
    uint64_t nnz;         /* finite non-zero elements                                     */
    uint64_t n_nonfinite; /* Inf or NaN elements (skipped)                                */
    double mean_log2;     /* mean of log2|g| over the nnz elements                        */
    double m2_log2;       /* sum of squared deviations of log2|g| from that mean          */
    double mu;            /* mean_log2 * ln 2                                             */
    double sigma;         /* sqrt(m2_log2 / nnz) * ln 2   (population standard deviation) */
    float max_abs;        /* largest finite |g|, 0 if nnz = 0                             */
    float min_abs_nz;     /* smallest non-zero finite |g|, 0 if nnz = 0                   */
    uint32_t status;
    uint32_t reserved;
} lgn_stats_t;

/* Result of lgn_threshold (device memory, 24 bytes). */
typedef struct lgn_prune_params_t {
    float alpha;     /* threshold, rounded to the tensor dtype; 0 = prune nothing        */
    uint32_t status;
    double s_eff;    /* S' = (S n - (n - nnz)) / nnz, sparsity asked of the non-zero part */
    double s_pred;   /* closed-form sparsity of the non-zero part at the rounded alpha    */
} lgn_prune_params_t;

/* Result of lgn_fp_params (device memory, 32 bytes). */
typedef struct lgn_fp_params_t {
    int32_t n_bits;    /* N = 1 + e_bits + m_bits                                */
    int32_t e_bits;    /* exponent bits (the paper's n2)                         */
    int32_t m_bits;    /* mantissa bits (the paper's n1)                         */
    int32_t scale_exp; /* s: the tensor is quantized as 2^s * Q(g / 2^s)         */
    double eta;        /* expected relative error of the split                   */
    uint32_t status;
    uint32_t reserved;
} lgn_fp_params_t;

/*
 * FP(1,e,m) word (Section 4.1, with the encoding choices needed to fit N bits):
 *   code = sign << (e+m) | c << m | k,   c in [1, 2^e - 1],  value = (1 + k/2^m) 2^(c - 2^(e-1) + s)
 *   c = 0 encodes zero (whatever k and sign are).  No subnormal, Inf or NaN codes.
 *   |g| >= 2^(2^(e-1) + s) saturates to the largest code; |g| < 2^(1 - 2^(e-1) + s) flushes to
 *   zero, decided before rounding.  Zero gives code 0; Inf and NaN give the largest code of their
 *   sign (with VALUE output NaN stays NaN).
 */

/*
 * Tuning knobs.  They change how the work is laid out on the device, never a result.  Process-wide;
 * read at every launch; value < 0 restores the default.  Not part of the method: timing
 * experiments and the tests of the cache-reuse boundary use them.
 *   LGN_TUNE_STATS_KEEP_MB         how much of a tensor's tail the statistics pass reads with
 *                                  ordinary (cache-allocating) loads, so that the pass that
 *                                  follows finds it in the memory-side cache; 0 = all streaming
 *                                  (default 224, range 0..4096)
 *   LGN_TUNE_STATS_BLOCKS_PER_CU   workgroups per compute unit of the statistics pass; 0 = by
 *                                  element type (2 for fp32, 6 for 16-bit types) (range 0..8)
 *   LGN_TUNE_STREAM_PAIRS_PER_WAVE tile pairs (512 elements) a wave of a streaming kernel walks;
 *                                  0 = by element type (6 for fp32, 24 for 16-bit types)
 *                                  (default 0, range 0..4096)
 *   LGN_TUNE_STREAM_BLOCKS_PER_CU  upper limit of the streaming grid in workgroups per compute
 *                                  unit (default 1024, range 1..1024)
 *   LGN_TUNE_STATS_STRICT_PUBLISH  how a workgroup of the one-launch statistics forms makes its
 *                                  record visible before it takes its ticket.  0 (default): it
 *                                  writes the record with device-scope write-through stores and
 *                                  waits for them to complete, which makes them visible device-wide
 *                                  on this hardware but is no promise of the memory model.  1: it
 *                                  also issues the device-scope release fence the model asks for;
 *                                  that writes back everything dirty in its L2 (what the pass
 *                                  before left there included) and costs 4 us on an 822 MB tensor
 *                                  when the statistics run alone, 11 us behind a fused pass, 55 us
 *                                  on 10^9 bf16 elements.  Results are identical; the setting is
 *                                  there so that a suspected stale read can be ruled out.
 * lgn_set_tuning returns LGN_ERR_INVALID_ARG for an unknown knob or a value out of range.
 */
#define LGN_TUNE_STATS_KEEP_MB 0
#define LGN_TUNE_STATS_BLOCKS_PER_CU 1
#define LGN_TUNE_STREAM_PAIRS_PER_WAVE 2
#define LGN_TUNE_STREAM_BLOCKS_PER_CU 3
#define LGN_TUNE_STATS_STRICT_PUBLISH 4
int lgn_set_tuning(int knob, long value);
long lgn_get_tuning(int knob); /* -1 for an unknown knob */

/* Bytes of workspace lgn_stats and lgn_stats_solve need for n elements (a few tens of KiB,
 * independent of n).  Host function, no device work. */
size_t lgn_workspace_bytes(uint64_t n, int dtype);

/* Prepares a workspace for lgn_stats_solve: clears the 64-byte ticket area at its end with a
 * small fill kernel on `stream`.  Needed once per workspace (every lgn_stats_solve leaves the
 * ticket cleared again); lgn_stats does not need it. */
int lgn_workspace_init(void *ws, size_t ws_bytes, void *stream);

/* Bytes of a PACKED output: ceil(n * n_bits / 8). Host function. */
size_t lgn_packed_bytes(uint64_t n, int n_bits);

/*
 * Lognormal statistics of g (Section 3: the fit is made on |g| excluding zero-valued entries;
 * Appendix "Stochastic pruning complexity": mean and standard deviation, O(n)).
 *   g        device, n elements of `dtype`, read once
 *   out      device, one lgn_stats_t, written
 *   ws       device workspace of at least lgn_workspace_bytes(n, dtype) bytes, 8-byte aligned;
 *            the per-block records at its start are overwritten, the ticket area at its end is
 *            not touched
 * Two launches: per-block partial moments, then a one-block combine.  log2|g| is taken in fp32
 * (one hardware instruction, relative error about 1e-7) and accumulated in fp64 as deviations
 * from a per-wave pivot; partial results are merged pairwise as (count, mean, M2), so the result
 * does not suffer from cancellation.
 * Errors: INVALID_ARG (null/misaligned), UNSUPPORTED (dtype), WORKSPACE, DEVICE.
 */
int lgn_stats(const void *g, uint64_t n, int dtype, lgn_stats_t *out, void *ws, size_t ws_bytes,
              void *stream);

/*
 * Statistics of the right mode of a bi-modal gradient (appendix "Algorithm for bi-Modal lognormal
 * pruning", steps 1 and 3): as lgn_stats, but only the entries of g whose entry in `mask` is
 * non-zero enter the fit (the mask is the gradient on the other side of the batch-norm, whose
 * zeros mark the left mode).
 *   mask       device, n entries, 16-byte aligned, read once
 *   mask_kind  LGN_MASK_SAME_DTYPE: a tensor of g's dtype, an entry counts unless it is +0 or -0;
 *              LGN_MASK_U8: one byte per element, counts unless 0; LGN_MASK_NONE: mask ignored
 * out->n is the size of the whole tensor and out->nnz the number of entries in the fit, so the zero
 * credit of lgn_threshold, S' = (S n - (n - nnz)) / nnz, is step 2's S' = (S - l) / (1 - l); the
 * threshold is then applied to the whole tensor with lgn_prune (step 4).  max_abs, min_abs_nz and
 * n_nonfinite refer to the entries in the fit.
 */
#define LGN_MASK_NONE 0
#define LGN_MASK_SAME_DTYPE 1
#define LGN_MASK_U8 2
int lgn_stats_masked(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                     lgn_stats_t *out, void *ws, size_t ws_bytes, void *stream);

/*
 * lgn_stats, lgn_threshold and lgn_fp_params in ONE launch (same passages as those three): the
 * workgroup that finishes last combines the per-block records and runs both solvers, so the two
 * parameter structs are ready when the statistics pass ends.  Results are identical to the three
 * separate calls, except that this call also sets LGN_ST_ALPHA_BELOW_FP_RANGE in p_out->status
 * when both a threshold and a format are asked for and the threshold lies below the format's range.
 *   target_sparsity  in [0, 1), or negative to skip the threshold (p_out may then be null)
 *   n_bits           in [2, 8], or 0 to skip the format (f_out may then be null)
 *   mask, mask_kind  as in lgn_stats_masked (null and LGN_MASK_NONE for a plain tensor)
 *   other arguments  as in lgn_stats / lgn_threshold / lgn_fp_params
 *   ws               as for lgn_stats, and prepared once with lgn_workspace_init: the kernel
 *                    counts finished workgroups in the ticket area, which must be zero on entry
 *                    and is zero again on exit.  Calls that overlap in time need separate
 *                    workspaces.
 */
int lgn_stats_solve(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                    double target_sparsity, int alpha_dtype, int n_bits, int e_bits, int scale_mode,
                    double scale_arg, int sigma_units, lgn_stats_t *st_out,
                    lgn_prune_params_t *p_out, lgn_fp_params_t *f_out, void *ws, size_t ws_bytes,
                    void *stream);

/*
 * lgn_stats_solve for callers that cannot allocate device memory and so have no workspace to pass:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (without ws) and the same results, bit for bit.  The per-block records and the ticket
 * live in an array of lgn_static_scratch_bytes() = 82 176 bytes inside the library's device image
 * (one copy per GPU, held until the process ends); it serves any n up to LGN_STATIC_MAX_ELEMENTS, a
 * larger n is refused with LGN_ERR_INVALID_ARG.  The call allocates nothing and launches one
 * 64-thread fill kernel (the ticket) and the statistics kernel on `stream`.  Every call on a GPU
 * uses that GPU's one array: calls that overlap in time on one GPU (different streams, several host
 * threads) race and must use lgn_stats_solve with workspaces of their own instead.
 */
#define LGN_STATIC_MAX_ELEMENTS (1ull << 40)
int lgn_stats_solve_static(const void *g, const void *mask, int mask_kind, uint64_t n, int dtype,
                           double target_sparsity, int alpha_dtype, int n_bits, int e_bits,
                           int scale_mode, double scale_arg, int sigma_units, lgn_stats_t *st_out,
                           lgn_prune_params_t *p_out, lgn_fp_params_t *f_out, void *stream);
size_t lgn_static_scratch_bytes(void);

/*
 * Threshold alpha such that stochastic pruning leaves a fraction `target_sparsity` of the WHOLE
 * tensor at zero (Section 5.1 poses the problem: the alpha that induces a given sparsity; closed
 * form of Section 5.2; existing zeros are credited as in Appendix "Algorithm for bi-Modal lognormal
 * pruning", step 2).
 *   st              device, read
 *   target_sparsity in [0, 1)
 *   alpha_dtype     LGN_F32, LGN_BF16 or LGN_F16: alpha is rounded to this type (it is compared with,
 *                   and stored into, tensors of this type)
 *   out             device, written
 * One single-wave launch: safeguarded Newton iteration on ln(alpha) in fp64.
 */
int lgn_threshold(const lgn_stats_t *st, double target_sparsity, int alpha_dtype,
                  lgn_prune_params_t *out, void *stream);

/*
 * Stochastic underflow: raises a pruning threshold to the smallest magnitude the format *f can
 * represent, alpha_out = max(alpha_in, 2^(E_min + s)), E_min = 1 - 2^(e-1) (Section 4.1).  With it
 * the fused pass sends |g| below the format's range to 0 or +-alpha_out with the mean kept (the
 * pruning operator of Section 5) instead of flushing it to zero.
 *   f     device, read
 *   in    device or null (null: alpha_in = 0, no pruning besides the underflow rule)
 *   out   device, written; may equal in.  LGN_ST_ALPHA_BELOW_FP_RANGE is set if the threshold was
 *         raised.  A floor outside the fp32 normal range is not applied.
 */
int lgn_threshold_floor(const lgn_fp_params_t *f, const lgn_prune_params_t *in, lgn_prune_params_t *out,
                        void *stream);

/*
 * FP-n format and scale (Section 4.3: minimise the expected relative error over the splits with
 * e + m = n_bits - 1; Section 4.4 and Alg. 1: per-tensor power-of-two scale).
 *   n_bits      total bits N in [2, 8]
 *   e_bits      exponent bits in [1, N-1], or -1 to take the minimiser
 *   scale_mode  LGN_SCALE_*;  scale_arg is the quantile (0,1) for LGN_SCALE_QUANTILE (the paper's
 *               example is 0.997), ignored otherwise; its standard normal quantile is evaluated
 *               on the host before the launch (it does not depend on the tensor)
 *   sigma_units LGN_SIGMA_*
 * One single-wave launch.
 */
int lgn_fp_params(const lgn_stats_t *st, int n_bits, int e_bits, int scale_mode, double scale_arg,
                  int sigma_units, lgn_fp_params_t *out, void *stream);

/*
 * Stochastic pruning (Section 5): out_i = g_i if |g_i| > alpha; else sign(g_i) alpha if
 * |g_i| >= fl32(alpha * u_i); else 0, with u_i = ((word >> 16) + 1/2) / 2^16 in (0, 1).  Zeros stay
 * (+)zero; NaN and Inf pass through.  alpha is read from *p on the device (alpha = 0 keeps every
 * non-zero element).
 *   out   device, n elements of `dtype`; may equal g (in place)
 */
int lgn_prune(const void *g, uint64_t n, int dtype, const lgn_prune_params_t *p, uint64_t seed,
              uint64_t elem_offset, void *out, void *stream);

/*
 * FP(1,e,m) quantization with scale 2^s (Section 4.1; Alg. 1 last line).  (N, e, m, s) are read
 * from *f on the device; the caller sizes a PACKED output with the N it asked lgn_fp_params for.
 *   rounding  LGN_ROUND_*; stochastic rounding goes up iff the cut-off fraction of a spacing plus
 *             (r + 1/2) / 2^16 reaches one, r the lower 16 bits of the element's word
 *   out       device; layout per out_kind (VALUE may be in place)
 */
int lgn_fp_quantize(const void *g, uint64_t n, int dtype, const lgn_fp_params_t *f, int rounding,
                    uint64_t seed, uint64_t elem_offset, void *out, int out_kind, void *stream);

/* Prune, then quantize what pruning returned, in one pass over g; bit-identical to
 * lgn_fp_quantize(lgn_prune(g)) with the same seed and offset. */
int lgn_prune_quantize_fused(const void *g, uint64_t n, int dtype, const lgn_prune_params_t *p,
                             const lgn_fp_params_t *f, int rounding, uint64_t seed,
                             uint64_t elem_offset, void *out, int out_kind, void *stream);

/*
 * Many tensors, two launches (per-layer thresholds and formats for all layers of a network:
 * Section 5.2 last paragraph, appendix "Stochastic pruning complexity" -- the parameters are per
 * layer, so a backward pass holds one small problem per layer; one pair of launches per layer
 * leaves the device idle between them).  lgn_batch_stats_solve is lgn_stats_solve for every item,
 * lgn_batch_prune_quantize_fused is lgn_prune_quantize_fused (elem_offset 0) for every item; the
 * statistics may differ from the one-tensor call in the last bits (another summation order), the
 * parameters follow from them as in the one-tensor call, and the codes are those of the one-tensor
 * call for the same parameters.
 *   items   HOST array of `count` descriptors (read during the call only); all device pointers in
 *           it are the caller's, as in the one-tensor calls.  All tensors share `dtype`.
 *   count   any number >= 0; the tables travel in the kernel arguments, 32 tensors per launch, so
 *           up to 32 tensors take one launch per call and nothing is uploaded or allocated
 *   ws      as for lgn_stats_solve (prepared with lgn_workspace_init)
 * An item with n = 0 is allowed (its statistics report an empty tensor).  Errors: as the
 * one-tensor calls, for the first offending item.
 */
typedef struct lgn_batch_item_t {
    const void *g;          /* device, n elements, 16-byte aligned                                 */
    void *out;              /* device, output of the fused pass (layout per out_kind)             */
    uint64_t n;
    uint64_t seed;          /* key of this tensor's random words                                  */
    double target_sparsity; /* in [0, 1), or negative: no threshold (p not written)               */
    int32_t n_bits;         /* in [2, 8], or 0: no format (f not written)                         */
    int32_t e_bits;         /* in [1, n_bits - 1], or -1 for the minimiser                        */
    lgn_stats_t *st;        /* device, written by lgn_batch_stats_solve                           */
    lgn_prune_params_t *p;  /* device, written by lgn_batch_stats_solve, read by the fused pass   */
    lgn_fp_params_t *f;     /* device, likewise                                                   */
} lgn_batch_item_t;

int lgn_batch_stats_solve(const lgn_batch_item_t *items, int count, int dtype, int alpha_dtype,
                          int scale_mode, double scale_arg, int sigma_units, void *ws, size_t ws_bytes,
                          void *stream);
int lgn_batch_prune_quantize_fused(const lgn_batch_item_t *items, int count, int dtype, int rounding,
                                   int out_kind, void *stream);

/* Decode CODE8 or PACKED codes back to values 2^s * q of type `dtype`. */
int lgn_dequantize(const void *codes, uint64_t n, int in_kind, const lgn_fp_params_t *f, int dtype,
                   void *out, void *stream);

/*
 * Prefix code of a pruned tensor (appendix "Encoding", table of codewords): 0 -> "0",
 * +alpha -> "100", -alpha -> "101", any other value -> "11" followed by the value itself.
 *   in        device, n elements: LGN_OUT_VALUE = values of `dtype` as lgn_prune writes them (the
 *             value after "11" is the 32- or 16-bit pattern), LGN_OUT_CODE8 = one FP-n code per
 *             byte as lgn_fp_quantize / lgn_prune_quantize_fused write them (the value is the
 *             N-bit code, N read from *f); 16-byte aligned
 *   p         device; alpha marks the special class.  VALUE: an element is +-alpha if its
 *             magnitude pattern equals alpha's (rounded to `dtype`).  CODE8: if its magnitude code
 *             equals the code alpha takes with nearest rounding in the format *f.  May be null
 *             (then, and for alpha = 0, there is no special class).
 *   f         device, needed for CODE8 (ignored for VALUE)
 *   out       device, the bit stream: stream bit k is bit (k & 7) of byte k >> 3; codewords first
 *             symbol first, the value after "11" least significant bit first.  Only the all-zero
 *             pattern takes the codeword "0", so decoding returns the input exactly.
 *   table     device, lgn_prefix_table_bytes(n) bytes: ceil(n / 4096) + 2 entries of 64 bits,
 *             then LGN_PREFIX_MAX_BLOCKS entries of scratch for the encoder, then 16 numbers of
 *             16 bits per chunk.  Elements are coded in chunks of LGN_PREFIX_CHUNK, every chunk
 *             starts on a 32-bit boundary (padding bits are zero); table[c] = index of the first
 *             32-bit word of chunk c, table[nchunks] = number of words of the whole stream,
 *             table[nchunks + 1] = 0, or 1 if out_capacity was too small (the chunks that did not
 *             fit are then not written).  The 16-bit numbers are the lengths in bits of each
 *             chunk's sixteen sub-blocks of LGN_PREFIX_SUB elements (0 past the end of the tensor):
 *             sub-block j of chunk c begins at stream bit 32 table[c] + the lengths of the
 *             sub-blocks before it, which is where the decoder starts its parsers.
 *   out_capacity  bytes available at out; lgn_prefix_bound_bytes(n, width) always suffices
 *             (width = 32, 16 or N)
 * Three launches (words per chunk, scan of per-workgroup sums, emit); `in` is read twice.
 */
#define LGN_PREFIX_CHUNK 4096
#define LGN_PREFIX_SUB 256
#define LGN_PREFIX_MAX_BLOCKS 2048 /* entries of scratch the encoder keeps behind the table */
size_t lgn_prefix_table_bytes(uint64_t n);
size_t lgn_prefix_bound_bytes(uint64_t n, int width);
int lgn_prefix_encode(const void *in, uint64_t n, int in_kind, int dtype, const lgn_prune_params_t *p,
                      const lgn_fp_params_t *f, void *out, size_t out_capacity, uint64_t *table,
                      void *stream);

/* Inverse of lgn_prefix_encode: writes n elements (values of `dtype`, or one code per byte) to
 * out.  in_kind, dtype, *p and *f must be those of the encoding call.  One thread per sub-block of
 * LGN_PREFIX_SUB elements.  `in` must hold at least table[nchunks] words and `table` must be the
 * whole table of that stream as the encoder left it (entries ascending, table[c + 1] <=
 * table[nchunks], sub-block lengths behind it): the call has no size of `in` to check the entries
 * against, and reads words of [table[c], table[c + 1]) only for every chunk.  Bits of the stream
 * itself are not trusted: whatever they are, exactly n elements are written. */
int lgn_prefix_decode(const void *in, const uint64_t *table, uint64_t n, int in_kind, int dtype,
                      const lgn_prune_params_t *p, const lgn_fp_params_t *f, void *out, void *stream);

/*
 * Histogram of the finite non-zero magnitudes of g on a logarithmic grid with eight bins per
 * binade (LGN_HIST_BINS = 2048 bins: bin = top eleven bits of the fp32 magnitude pattern, i.e.
 * exponent and three mantissa bits).  A high quantile of ln|g| read off it serves as the
 * truncation point of the lognormal model (section "Neural gradients lognormal distributions are
 * truncated": the sample maximum is too noisy, a quantile such as 0.997 is taken).
 *   hist   device, LGN_HIST_BINS counts of 64 bits, overwritten (cleared by a small kernel first)
 */
#define LGN_HIST_BINS 2048
int lgn_log_histogram(const void *g, uint64_t n, int dtype, uint64_t *hist, void *stream);

/* Per-layer result of lgn_sparsity_allocate (device memory, 32 bytes). */
typedef struct lgn_alloc_t {
    double sparsity;  /* zero fraction of the whole tensor predicted at the layer's threshold      */
    double cosine;    /* closed-form cosine similarity between the layer and its pruned version   */
    double k;         /* truncation point of the lognormal model in units of sigma                */
    uint32_t status;  /* LGN_ALLOC_* bits */
    uint32_t reserved;
} lgn_alloc_t;
#define LGN_ALLOC_LOWERED 1u /* threshold lowered to keep the layer's minimum cosine similarity */
#define LGN_ALLOC_CAPPED 2u  /* the compensating sparsity was limited by max_sparsity           */

/*
 * Heterogeneous stochastic pruning (appendix "Cosine similarity and heterogeneous stochastic
 * pruning", "Heterogeneous algorithm"), one launch for all layers of a network.
 *   stats          device, n_layers structs in the order of the backward pass (deepest layer first)
 *   hists          device, n_layers x LGN_HIST_BINS counts from lgn_log_histogram, or null: then the
 *                  truncation point is the `quantile` of the fitted normal itself
 *   overall_sparsity  the element-weighted mean sparsity wanted over all layers
 *   n_deep, min_cosine  the first n_deep layers each have a minimum cosine similarity
 *                  (device, n_deep doubles): where the threshold for overall_sparsity would give
 *                  less, the threshold is lowered until the closed form meets the minimum
 *   max_sparsity   cap on the sparsity the remaining layers get to make up the difference
 *                  (the paper suggests 0.96 to 0.98)
 *   quantile       of ln|g| that defines the truncation point (the paper's example: 0.997)
 *   p_out          device, n_layers lgn_prune_params_t, ready for lgn_prune / the fused pass
 *   a_out          device, n_layers lgn_alloc_t
 * The cosine similarity uses the truncated-lognormal closed forms of the appendix with the cut-off
 * k sigma taken in the log domain.
 */
int lgn_sparsity_allocate(const lgn_stats_t *stats, const uint64_t *hists, int n_layers,
                          double overall_sparsity, int n_deep, const double *min_cosine,
                          double max_sparsity, double quantile, int alpha_dtype,
                          lgn_prune_params_t *p_out, lgn_alloc_t *a_out, void *stream);

const char *lgn_last_error(void);
int lgn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LGN_H */
