/*
 * libcast: the per-step optimizer hot path of CAST (arXiv 2509.25996) for AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer marked DEVICE is an address in the memory of the current HIP device;
 * pointers marked HOST are ordinary process memory.  The caller owns every buffer: the
 * library allocates nothing, keeps no state between calls and frees nothing (one exception,
 * described where it is declared: cast_adams_step_multi_noalloc works in a device buffer that
 * is part of the library's image, and remembers that buffer's address per device).
 *
 * Execution: each call validates its arguments on the host, then enqueues its kernels on the
 * HIP stream passed as `stream` (a hipStream_t cast to void*; NULL = the default stream) and
 * returns without waiting.  Validation failures return a negative status and enqueue nothing.
 *
 * Tensors are row-major [rows, cols]; rows = out_features, cols = in_features of a linear
 * layer.  Groups of M consecutive entries run along a row (Sec. 3, Eq. 3).  The weights w and
 * the two moments m, v share one row stride `ld` (in entries, ld >= cols; ld == cols for dense
 * arrays): a caller may interleave the three arrays row by row in one allocation ([rows][3][cols],
 * ld = 3*cols), which keeps their streams close together in HBM and is measurably faster.
 * Every other buffer (gradient, mask bits, scale, packed outputs) is dense.  Empty tensors
 * (rows == 0 or cols == 0) are accepted and do nothing.
 *
 * Shapes accepted: M in {2, 4, 8}, 1 <= N < M, cols % M == 0.  With weight scaling in n
 * segments: cols % n == 0 and (cols / n) % M == 0, so that no group lies in two segments.
 * All fp32 buffers must be 16-byte aligned, bf16 buffers 8-byte aligned, word buffers 4-byte.
 * The fast kernels need rows (and scale segments) that are multiples of 32 entries and ld % 4 == 0;
 * any other accepted shape runs on slower scalar kernels with identical results.
 *
 * Mask storage (one bit per parameter; Remark at the end of Sec. 4.1): uint32 words, each row
 * padded to whole words; M[r, c] is bit (c % 32) of word [r * ceil(cols/32) + c / 32].
 * Padding bits are written as zero.
 *
 * Tie rule for Eq. 6 (the paper's ">= xi" keeps more than N entries when magnitudes tie,
 * against Eq. 4): exactly N entries are kept and among equal magnitudes the lower column
 * index is kept.  Magnitude is the IEEE-754 bit pattern with the sign bit cleared, compared
 * as an unsigned integer (-0 equals +0, denormals keep their order, NaN ranks above inf).
 */
#ifndef CAST_H
#define CAST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t cast_status;
enum {
    CAST_OK = 0,
    CAST_ERR_NULL = -1,   /* a required pointer is NULL                                   */
    CAST_ERR_SHAPE = -2,  /* rows/cols/N/M/n violate the rules above                      */
    CAST_ERR_ALIGN = -3,  /* a buffer is not aligned as required                          */
    CAST_ERR_DTYPE = -4,  /* unknown dtype code                                           */
    CAST_ERR_CONFIG = -5, /* a scalar of cast_adams_config is out of range (e.g. bias_corr <= 0) */
    CAST_ERR_LAUNCH = -6, /* the HIP runtime refused the launch (hipGetLastError != success) */
    CAST_ERR_SCRATCH = -7 /* cast_adams_step_multi_noalloc only: the list exceeds its fixed limits  */
};

enum { CAST_F32 = 0, CAST_BF16 = 1 };

/* Second moment from g^2 instead of mu~^2 (Eq. 9's form; not the paper's method).  With alpha = 0
 * this makes the step textbook Adam: what the tests pin against a library optimizer, and a way to
 * step dense parameters such as the scale factors A of Eq. 12 with this library. */
#define CAST_FLAG_V_FROM_GRAD 1u
/* (flag value 2 is not in use: CAST_ERR_CONFIG) */
/* Storage variant outside the paper (Algorithm 1 does not say how the moments are kept): the first
 * moment is kept in bf16.  `m` then points to bf16 values (uint16_t), 16-byte aligned, whose row
 * stride in bf16 entries is cols when ld == cols and 2 * ld otherwise (the byte pitch of w and v,
 * as when the rows of the three arrays are interleaved in one allocation).  The new mu is rounded
 * to nearest even when stored; mu~, v and the update of the same iteration use the unrounded
 * value.  22.125 instead of 26.125 bytes per parameter.  Only with CAST_RULE_ADAMS and
 * CAST_RULE_ADDITIVE (else CAST_ERR_CONFIG); the compute copy can be written along (24.125 bytes
 * per parameter) and refresh statistics gathered. */
#define CAST_FLAG_MU_BF16 4u
/* Both moments in bf16 (only together with CAST_FLAG_MU_BF16; same rules and exclusions): `v`
 * points to bf16 values laid out like `m`.  With beta_2 = 0.999 one iteration changes v by a
 * thousandth, less than half a bf16 unit in the last place, so rounded to nearest a stored v would
 * never move: the new v is rounded STOCHASTICALLY when stored (away from zero with probability
 * (discarded 16 bits) / 65536, so the expectation is the fp32 value; infinities and NaN go through
 * round-to-nearest); the update of the same iteration uses the unrounded value.  The 16 random
 * bits of the entry with index i = row * cols + col are the upper half of
 *   mix(((uint32)i ^ mix(sr_seed + 0x9e3779b9)) + (uint32)(i >> 32) * 0x9e3779b9),
 *   mix(x): x ^= x >> 16; x *= 0x7feb352d; x ^= x >> 15; x *= 0x846ca68b; x ^= x >> 16   (uint32)
 * a counter-based generator: the result depends on (sr_seed, i) only, whatever the launch shape.
 * The caller passes another cfg->sr_seed every iteration (a step counter will do).
 * 18.125 bytes per parameter, 20.125 with the compute copy. */
#define CAST_FLAG_V_BF16 8u

/* Update rules.  CAST_RULE_ADAMS is the paper's method (Algorithm 1, Eq. 8); the others are the
 * rules it is set against, for ablations.  In all of them the decay acts only on entries whose
 * mask bit is 0 and has strength alpha * lambda, like the second term of Eq. 7 (Eq. 9 and 10 are
 * printed for one always-decayed parameter with strength lambda: alpha = 1 gives that form).
 *   ADAMW_L1       Eq. 9:  mu, v from g and g^2;  w -= lr * (mu^/(sqrt(v^)+eps) + alpha*lambda*Sign(w))
 *   ADAM_L1        Eq. 10: g~ = g + alpha*lambda*Sign(w);  mu, v from g~ and g~^2
 *   ADDITIVE       Eq. 8 with mu~ = mu + alpha*lambda*Sign(w): the decay is added to the momentum
 *                  instead of being traded against it (the additive decay of Sec. 4.1.2)
 *   MASKED_FROZEN  sparsity-aware fine-tuning (Sec. 6.7): entries with mask bit 0 keep w, mu, v;
 *                  the others follow Eq. 8 with mu~ = mu */
enum {
    CAST_RULE_ADAMS = 0,
    CAST_RULE_ADAMW_L1 = 1,
    CAST_RULE_ADAM_L1 = 2,
    CAST_RULE_ADDITIVE = 3,
    CAST_RULE_MASKED_FROZEN = 4
};

/* Inputs of one AdamS iteration (Algorithm 1).  All scalars are used as given, in fp32. */
typedef struct {
    int32_t  n_keep;         /* N                                                            */
    int32_t  m_group;        /* M                                                            */
    float    lr;             /* gamma_t                                        Algorithm 1   */
    float    beta1, beta2;   /* beta_1, beta_2 (the paper prints no values)                  */
    float    eps;            /* epsilon                                                      */
    float    lambda;         /* regularization strength lambda                 Eq. 7         */
    float    alpha;          /* alpha_t = t / T, in [0, 1]                     Eq. 7         */
    float    bias_corr1;     /* 1 - beta_1^s, s >= 1, computed by the caller   Eq. 8         */
    float    bias_corr2;     /* 1 - beta_2^s                                                 */
    int32_t  refresh_mask;   /* 1 on iterations with t mod T_1 == 0: take the mask from the  */
                             /* incoming weights (Eq. 6) and store it; 0: read mask_bits     */
    int32_t  scale_segments; /* n of Eq. 12; 0 = no weight scaling                           */
    int32_t  grad_dtype;     /* CAST_F32 or CAST_BF16                                        */
    uint32_t flags;          /* 0, or an OR of CAST_FLAG_*                                   */
    int32_t  rule;           /* CAST_RULE_*; 0 = AdamS                                       */
    uint32_t sr_seed;        /* seed of the rounding bits under CAST_FLAG_V_BF16, else unused */
} cast_adams_config;

const char *cast_status_str(cast_status s);

/* Bytes of the mask, of the packed values and of the packed metadata for a shape (HOST
 * outputs; any of the three may be NULL).  value_dtype sizes the values buffer. */
cast_status cast_sizes(int64_t rows, int64_t cols, int n_keep, int m_group, int value_dtype,
                       size_t *mask_bytes, size_t *values_bytes, size_t *meta_bytes);

/*
 * Magnitude mask, Eq. 6 (Sec. 4.1) under the N-per-group constraint of Eq. 4.
 *   w          DEVICE in   fp32 [rows, cols], row stride ld
 *   mask_bits  DEVICE out  uint32 [rows, ceil(cols/32)]
 */
cast_status cast_nm_select(const float *w, int64_t rows, int64_t cols, int64_t ld, int n_keep,
                           int m_group, uint32_t *mask_bits, void *stream);

/*
 * One matrix of a list for the once-per-run entry points below (cast_nm_select_multi,
 * cast_weight_scale_multi, cast_nm_project_compress_multi): the arguments of the single-matrix call
 * of the same name.  Matrices of one shape share kernel launches.
 */
typedef struct {
    const float *w;        /* DEVICE in   fp32 [rows, cols], row stride ld                                      */
    int64_t rows, cols, ld;
    const float *scale;    /* DEVICE in   A, fp32 [rows, n_segments]; weight_scale: required; project_compress:  */
                           /*             or NULL; select: unused                                               */
    uint32_t *mask_bits;   /* DEVICE      select: out; project_compress: in, or NULL (Eq. 6 on w);               */
                           /*             weight_scale: unused                                                  */
    void *out;             /* DEVICE out  weight_scale: out; project_compress: values; select: unused           */
    uint32_t *meta;        /* DEVICE out  project_compress only                                                 */
    uint32_t *mask_status; /* DEVICE i/o  project_compress with a stored mask only, or NULL: the number of groups     */
                           /*             whose stored bits are not exactly N ones is ADDED to this word (clear it   */
                           /*             before the call; 0 afterwards = the mask is a valid N:M mask).  Such        */
                           /*             groups are still packed, with meaningless values and positions.            */
} cast_matrix;

/* cast_nm_select over a list (validated as a whole before anything is launched). */
cast_status cast_nm_select_multi(const cast_matrix *matrices /* HOST */, int count, int n_keep, int m_group,
                                 void *stream);

/*
 * One AdamS iteration over one weight matrix: the body of Algorithm 1's loop (Eq. 8), with
 * the proportional decay of Eq. 7 on the entries whose mask bit is 0.
 *
 *   w, m, v     DEVICE in/out  fp32 [rows, cols], row stride ld: theta, first moment mu, second moment v
 *                              (m, or m and v, bf16 under CAST_FLAG_MU_BF16 / CAST_FLAG_V_BF16, see there).
 *   grad        DEVICE in      [rows, cols] of cfg->grad_dtype.  With scale == NULL it is dL/dW;
 *                              with scale != NULL it is dL/dW_scale and the chain rule of Eq. 12
 *                              (dL/dW = A[r, s] * grad) is applied inside.
 *   mask_bits   DEVICE         written when cfg->refresh_mask (from w as it comes in), else read.
 *   scale       DEVICE in      A, fp32 [rows, n], or NULL iff cfg->scale_segments == 0.
 *   scale_grad  DEVICE out     dL/dA, fp32 [rows, n] = sum over each row segment of grad * w (w as it
 *                              comes in), or NULL to skip it.  Summed in fp32 in a fixed order, so it is
 *                              reproducible but differs from a double sum by rounding.
 *
 * Per entry, in fp32, one rounding per operation, no fused multiply-add:
 *   g = grad (* A);  mu = b1*mu + (1-b1)*g;  mu~ = keep ? mu : (1-alpha)*mu + (alpha*lambda)*Sign(w)
 *   v = b2*v + (1-b2)*mu~^2;  w = w - lr * ((mu~/bias_corr1) / (sqrt(v/bias_corr2) + eps))
 * mu (not mu~) and v are stored.  Sign(+-0) = Sign(NaN) = 0.
 */
cast_status cast_adams_step(float *w, const void *grad, float *m, float *v, uint32_t *mask_bits,
                            const float *scale, float *scale_grad, int64_t rows, int64_t cols,
                            int64_t ld, const cast_adams_config *cfg /* HOST */, void *stream);

/*
 * The same iteration, which in the same pass also writes the weights the next forward pass
 * multiplies with (Algorithm 2 applies the weight scaling of Eq. 12 before every forward pass):
 *   compute_copy  DEVICE out  bf16 dense [rows, cols], 16-byte aligned:
 *                             round-to-nearest-even of copy_scale[r, s] * w_new (one fp32 multiply),
 *                             or of w_new itself when copy_scale is NULL
 *   copy_scale    DEVICE in   fp32 [rows, n] with n = cfg->scale_segments, or NULL (required NULL
 *                             when n = 0).  It may be `scale` itself.  dL/dA of this iteration is
 *                             only produced by this very launch, so the A folded here cannot have
 *                             seen it yet: the copy is exact for a frozen A or for an A whose update
 *                             lags one iteration; otherwise call cast_weight_scale after updating A.
 * Costs 2 more bytes per parameter (28.125 with bf16 gradients) instead of a separate pass that
 * reads w again (6 bytes per parameter).
 */
cast_status cast_adams_step_emit(float *w, const void *grad, float *m, float *v, uint32_t *mask_bits,
                                 const float *scale, float *scale_grad, const float *copy_scale,
                                 void *compute_copy, int64_t rows, int64_t cols, int64_t ld,
                                 const cast_adams_config *cfg /* HOST */, void *stream);

/*
 * The same iteration over a list of matrices that share one configuration (all linear weights
 * of a model in one call): validated as a whole before anything is launched, then stepped one
 * launch per matrix, small matrices of one shape several to a launch.  w, m, v and mask_bits come
 * out as from cast_adams_step on each matrix, bit for bit; so does scale_grad, except for row
 * segments of more than 2048 entries other than 4096, which the list call steps in pieces of 512,
 * 1024 or 2048 entries: their sums are added in another, equally fixed order (per piece, then the
 * pieces left to right).
 *   tensors    HOST in   `count` descriptors; the device buffers they name follow the rules of
 *                        cast_adams_step (scale / scale_grad NULL or not for all alike, per cfg).
 *                        No two descriptors may name overlapping buffers: the matrices are stepped
 *                        in an order of the library's choosing, several of them by one launch.
 *   workspace  DEVICE    at least cast_adams_multi_workspace_bytes(tensors, count, cfg) bytes (it
 *                        depends on shapes, row strides, scale_grad and refresh_stats being NULL or
 *                        not and cfg->scale_segments only; it holds the dL/dA sums of the pieces and
 *                        the per-workgroup refresh statistics until follow-up launches of the same
 *                        call have added them up), 16-byte aligned, owned by the caller; it is
 *                        overwritten by every call and used by the kernels of that call, so it must
 *                        not be shared between streams (too small: CAST_ERR_SHAPE; may be NULL when
 *                        0 bytes are needed)
 * The call enqueues kernel launches only (no copies, no memsets, nothing allocated on the device), so
 * it can be recorded while the stream is being captured into a HIP graph.
 */
/* Mask-learning statistics of one matrix gathered by a refresh step itself (appendix "Mask
 * Learning"; the numerators of the flip rate r_t and the initial flip rate i_t, and both terms of
 * the sparse weight ratio S_t), from the weights as they come in:
 *   flips_prev = ||M_new - M_stored||_0   against the mask mask_bits held when the call began
 *   flips_init = ||M_new - M_initial||_0  against initial_mask_bits (0 when that is NULL)
 *   l1_kept    = ||W (.) M_new||_1,  l1_all = ||W||_1
 * Counts are exact; the norms are summed in a fixed order (fp32 within a workgroup, double across
 * workgroups), so they are reproducible and within 1e-6 relative of a double sum. */
typedef struct {
    uint64_t flips_prev;
    uint64_t flips_init;
    double   l1_kept;
    double   l1_all;
} cast_refresh_stats;

typedef struct {
    float *w;
    const void *grad;
    float *m;
    float *v;
    uint32_t *mask_bits;
    const float *scale;
    float *scale_grad;
    int64_t rows, cols, ld;
    void *compute_copy;         /* as in cast_adams_step_emit, or NULL */
    const float *copy_scale;    /* as in cast_adams_step_emit, or NULL */
    const uint32_t *initial_mask_bits;   /* DEVICE in, or NULL: see cast_refresh_stats */
    cast_refresh_stats *refresh_stats;   /* DEVICE out, or NULL: overwritten by calls with          */
                                         /* cfg->refresh_mask = 1, left alone by the others         */
} cast_tensor;

size_t cast_adams_multi_workspace_bytes(const cast_tensor *tensors /* HOST */, int count,
                                        const cast_adams_config *cfg /* HOST */);

cast_status cast_adams_step_multi(const cast_tensor *tensors, int count, const cast_adams_config *cfg,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * cast_adams_step_multi for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, serving loops and harnesses that forbid allocation.  Same arguments, same
 * validation, same kernels and therefore the same results bit for bit (dL/dA included); the workspace
 * is a buffer of CAST_NOALLOC_SCRATCH_BYTES bytes built into the library, one per GPU, held from the
 * moment the library's code is loaded on that GPU until the process ends.  The call allocates nothing
 * on the host or the device and frees nothing; it enqueues kernel launches only.
 *   - A list that needs more (cast_adams_multi_workspace_bytes(tensors, count, cfg) >
 *     CAST_NOALLOC_SCRATCH_BYTES) or has more than CAST_NOALLOC_MAX_TENSORS matrices is rejected with
 *     CAST_ERR_SCRATCH and nothing is launched.  (The LLaMA2-7B-shaped set with n = 2 needs 3 MiB,
 *     the 13B-shaped one 44 MiB; refresh statistics add 16 bytes per workgroup.)
 *   - All calls on one GPU share that GPU's buffer.  Every byte a call reads from it was written by
 *     the same call before, so nothing needs clearing between calls; but two calls whose kernels can
 *     overlap (different streams, or graphs replayed concurrently) race on it: keep all calls of this
 *     entry point on one GPU in one stream order.
 *   - The first call on a GPU looks the buffer's address up (hipGetSymbolAddress); make that call
 *     outside of stream capture.
 */
#define CAST_NOALLOC_SCRATCH_BYTES (64u << 20)
#define CAST_NOALLOC_MAX_TENSORS 4096
cast_status cast_adams_step_multi_noalloc(const cast_tensor *tensors /* HOST */, int count,
                                          const cast_adams_config *cfg /* HOST */, void *stream);

/* How many kernel launches cast_adams_step_multi makes for this list (HOST only, nothing is
 * enqueued; assumes a workspace of the size cast_adams_multi_workspace_bytes returns):
 * step_launches = launches of the step kernel (one launch may step several matrices),
 * other_launches = the rest (dL/dA reductions of odd shapes, sums of split row segments).
 * For accounting (time per launch = time per call / launches); either pointer may be NULL. */
cast_status cast_adams_multi_launches(const cast_tensor *tensors /* HOST */, int count,
                                      const cast_adams_config *cfg /* HOST */,
                                      int32_t *step_launches /* HOST out */,
                                      int32_t *other_launches /* HOST out */);

/*
 * Weight scaling forward / fold, Eq. 12 (Eq. 11 when n_segments == 1):
 *   out[r, c] = scale[r, c / (cols / n_segments)] * w[r, c]      (one fp32 multiply)
 *   w DEVICE in fp32 [rows, cols], row stride ld; scale DEVICE in fp32 [rows, n_segments];
 *   out DEVICE out dense [rows, cols] of out_dtype (bf16 = round to nearest even of the fp32 product);
 *   out may be w itself when out_dtype is CAST_F32 and ld == cols.
 */
cast_status cast_weight_scale(const float *w, const float *scale, int64_t rows, int64_t cols,
                              int64_t ld, int n_segments, void *out, int out_dtype, void *stream);

/* cast_weight_scale over a list: the scaled weights of the whole model before a forward pass
 * (Algorithm 2 applies Eq. 12 before every forward pass). */
cast_status cast_weight_scale_multi(const cast_matrix *matrices /* HOST */, int count, int n_segments,
                                    int out_dtype, void *stream);

/*
 * Gradient of the scale alone, for callers that do not take it from cast_adams_step:
 *   scale_grad[r, s] = sum over c in segment s of grad_scaled[r, c] * w[r, c]
 * (the derivative of Eq. 12 with respect to A).  Same summation order as cast_adams_step.
 */
cast_status cast_weight_scale_grad(const float *w, const void *grad_scaled, int grad_dtype,
                                   int64_t rows, int64_t cols, int64_t ld, int n_segments,
                                   float *scale_grad, void *stream);

/* One matrix of a list for cast_weight_scale_grad_multi (Eq. 12, derivative with respect to A). */
typedef struct {
    const float *w;             /* DEVICE in: fp32 [rows, cols], row stride ld, 16-byte aligned        */
    const void *grad_scaled;    /* DEVICE in: dL/dW_scale, dense [rows, cols] of the call's grad_dtype */
    int64_t rows, cols, ld;
    float *scale_grad;          /* DEVICE out: fp32 [rows, n_segments]                                 */
} cast_scale_grad_matrix;

/* cast_weight_scale_grad over a list (HOST array): matrices of one shape share launches; same
 * results, matrix by matrix, as the single call.  All or nothing: an invalid matrix, or an unknown
 * grad_dtype, returns its error before anything is launched.  count == 0 is CAST_OK. */
cast_status cast_weight_scale_grad_multi(const cast_scale_grad_matrix *matrices /* HOST */, int count,
                                         int grad_dtype, int n_segments, void *stream);

/*
 * Final hard prune (last loop of Algorithm 1 / Algorithm 2), fold of the scale (Sec. 4.2)
 * and packing into values + index metadata.  The paper gives no packed layout; this one is
 * the library's own:
 *
 *   mask_bits == NULL: the mask is Eq. 6 on w (projection onto the N:M set);
 *   mask_bits != NULL: the stored mask is applied as is (Algorithm 1 literally); it must hold
 *                      exactly N ones per group.  This call does not check that; the list call
 *                      cast_nm_project_compress_multi does when given a mask_status word.
 *   values  DEVICE out [rows, cols*N/M] of value_dtype: for each group its kept entries in
 *           ascending column order, each multiplied by scale[r, s] if scale != NULL (one fp32
 *           multiply; bf16 = round to nearest even of that; any NaN becomes 0x7FC0).
 *   meta    DEVICE out uint32 [rows, ceil((cols/M) * f / 32)]: each kept entry's position in its
 *           group in b = ceil(log2 M) bits; the N positions of a group concatenated ascending,
 *           first in the least significant bits; group field padded to f = next power of two
 *           >= N*b bits (2:4 -> 4, 4:8 -> 16, 1:2 -> 1); group i of a row at bit
 *           (i % (32/f)) * f of word i / (32/f); unused bits zero.
 */
cast_status cast_nm_project_compress(const float *w, const float *scale, int n_segments,
                                     const uint32_t *mask_bits, int64_t rows, int64_t cols,
                                     int64_t ld, int n_keep, int m_group, void *values,
                                     int value_dtype, uint32_t *meta, void *stream);

/* cast_nm_project_compress over a list: the last loop of Algorithm 1 over the whole model.
 * n_segments applies to the matrices whose scale is not NULL. */
cast_status cast_nm_project_compress_multi(const cast_matrix *matrices /* HOST */, int count, int n_segments,
                                           int n_keep, int m_group, int value_dtype, void *stream);

/*
 * Mask-learning statistics of one matrix (appendix "Mask Learning"): the numerators of the
 * flip rate r_t / initial flip rate i_t and both terms of the sparse weight ratio S_t.
 *   mask_bits, other_bits  DEVICE in  masks to compare (other_bits may be NULL: flips = 0)
 *   flips     DEVICE in/out uint64[1]: += ||M - M_other||_0
 *   l1        DEVICE in/out double[2]: [0] += ||W (.) M||_1, [1] += ||W||_1
 * The outputs are accumulated into (clear them before the first matrix), so one pair of
 * buffers can be summed over all matrices of a model as the appendix's definitions do.
 * The double additions are atomic and their order is not fixed: l1 is reproducible only to rounding.
 */
cast_status cast_mask_stats(const float *w, const uint32_t *mask_bits, const uint32_t *other_bits,
                            int64_t rows, int64_t cols, int64_t ld, unsigned long long *flips,
                            double *l1, void *stream);

/*
 * The same statistics for a list of matrices, each into a record of its own, without atomics: every workgroup
 * leaves its counts and fp32 partial norms in the workspace and a second launch adds them up per matrix in a
 * fixed order (counts exactly, norms in double), so the results are reproducible and within 1e-6 relative of
 * a double sum.  Matrices of one shape share launches.
 *   stats  DEVICE out  OVERWRITTEN: flips_prev = ||M - M_other||_0 (0 when other_bits is NULL), flips_init = 0,
 *                      l1_kept = ||W (.) M||_1, l1_all = ||W||_1
 *   workspace  DEVICE  at least cast_mask_stats_multi_workspace_bytes(matrices, count) bytes, 16-byte aligned
 */
typedef struct {
    const float *w;               /* DEVICE in  fp32 [rows, cols], row stride ld */
    int64_t rows, cols, ld;
    const uint32_t *mask_bits;    /* DEVICE in  M */
    const uint32_t *other_bits;   /* DEVICE in  the mask flips are counted against, or NULL */
    cast_refresh_stats *stats;    /* DEVICE out */
} cast_stats_matrix;

size_t cast_mask_stats_multi_workspace_bytes(const cast_stats_matrix *matrices /* HOST */, int count);

cast_status cast_mask_stats_multi(const cast_stats_matrix *matrices /* HOST */, int count, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * Measurement aid, not part of the method: a plain device-to-device copy kernel of `bytes`
 * bytes (a multiple of 16; both pointers 16-byte aligned), used to calibrate the HBM byte
 * counters and to measure the achievable copy bandwidth beside the optimizer kernels.
 */
cast_status cast_hbm_copy_probe(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Measurement aid, not part of the method: the launches cast_adams_step_multi would make for this list
 * of 2:4 matrices on a non-refresh iteration (same plans, same shared launches, same loads,
 * prefetches and stores of w, m, v, grad and mask_bits, same dL/dA sums), with the arithmetic of
 * the iteration replaced by three multiply-adds per entry (bf16 moments are stored by truncation).
 * Its duration is what the memory system gives this access pattern: the ceiling the real step can
 * be held against.  grad_dtype: CAST_BF16 or CAST_F32; moment_flags: 0 (fp32 moments),
 * CAST_FLAG_MU_BF16 or CAST_FLAG_MU_BF16 | CAST_FLAG_V_BF16, the latter two with bf16 gradients
 * only (anything else: CAST_ERR_CONFIG), with m and v laid out as those flags lay them out for
 * the step.  w, m, v and scale_grad are OVERWRITTEN with meaningless values.  Descriptors as for
 * cast_adams_step_multi (no compute_copy, no refresh_stats; shapes the fast kernels take only, else
 * CAST_ERR_SHAPE); workspace as for that call with the same scale_segments.
 */
cast_status cast_hbm_stream_probe(const cast_tensor *tensors /* HOST */, int count, int scale_segments,
                                  int grad_dtype, uint32_t moment_flags,
                                  void *workspace /* DEVICE */, size_t workspace_bytes, void *stream);

/*
 * Diagnostic, runs on the HOST (both pointers HOST): out[i] = x[i] / y computed by the very
 * routine the kernels use for the two bias-correction divisions of Eq. 8 (a short FMA sequence
 * with a precomputed reciprocal inside a checked range, the IEEE division outside it).  It
 * exists so that the claim "identical to the correctly rounded quotient" can be tested on any
 * machine.
 */
cast_status cast_debug_div_by_uniform(const float *x, float y, float *out, int64_t n);

/*
 * Diagnostic, runs on the HOST: how the step kernels would cover a [rows, cols] matrix with row
 * stride ld and n_segments scaling segments (allow_split = 1: as in a list call with a workspace;
 * allow_split = 2 or 3 with n_segments = 0: how the selection, scaling and pack kernels cover it instead,
 * with 4 or 8 entries per thread and load: `wave` then counts the wavefronts of a workgroup's first piece,
 * then those of its second, ..., each with a span of its own of 256 or 512 entries, plan[2] says how
 * many, plan[3] = plan[4] = 1; other values: CAST_ERR_SHAPE), and
 * where wavefront `wave` of workgroup `block` would work, computed by the very functions the
 * kernels use.  It exists so that "every entry is covered exactly once and nothing outside the
 * matrix is touched" can be tested for any shape without a GPU.
 *   plan[0] = 1 if the vector kernels apply (else the scalar kernels run and the rest is unused)
 *   plan[1] = workgroups, plan[2] = wavefronts per workgroup, plan[3] = cooperating wavefronts per span,
 *   plan[4] = pieces per row segment (1 = not split)
 *   span[0] = first entry in w/m/v (with row stride), span[1] = first entry in dense numbering,
 *   span[2] = entries (0: this wavefront has nothing to do), span[3] = index into scale / scale_grad
 *             (split plans: piece number), span[4] = its place among the cooperating wavefronts
 */
cast_status cast_debug_plan(int64_t rows, int64_t cols, int64_t ld, int n_segments, int allow_split,
                            int64_t block, int wave, int64_t plan[5] /* HOST out */,
                            int64_t span[5] /* HOST out */);

#ifdef __cplusplus
}
#endif
#endif /* CAST_H */
