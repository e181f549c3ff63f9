/*
 * CPU oracle for the AdamS / N:M hot path of CAST (arXiv 2509.25996).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
 * check and the benchmark's CPU-baseline leg may build, load or call it.  It is a
 * plain, slow, loop-per-element restatement of what the paper defines, written to
 * be checked against the paper by eye; it shares no code with the GPU library.
 *
 * What it follows:
 *   - groups and the N-per-group constraint ........ Sec. 3, Eq. 3 and Eq. 4
 *   - magnitude mask ................................ Sec. 4.1, Eq. 6
 *   - AdamS update .................................. Sec. 4.1, Algorithm 1 and Eq. 8
 *   - proportional decay ............................ Sec. 4.1.2, Eq. 7
 *   - weight scaling (forward, fold) ................ Sec. 4.2, Eq. 11 and Eq. 12
 *   - final hard prune .............................. Algorithm 1 (last loop), Algorithm 2 (last loop)
 *   - mask-learning statistics ...................... Appendix "Mask Learning"
 *
 * Readings taken where the paper is silent (each also listed in the design notes):
 *   - Eq. 6 keeps more than N entries on magnitude ties, contradicting Eq. 4; here exactly
 *     N are kept and among equal magnitudes the lower column index wins.
 *   - "magnitude" is the IEEE-754 bit pattern with the sign bit cleared, compared as an
 *     unsigned integer: -0 == +0, denormals are ordered exactly, inf > finite, NaN > inf.
 *   - Sign(+-0) = 0 and Sign(NaN) = 0.
 *   - the mask of a refresh step is taken from the weights before that step's update,
 *     and from the unscaled weights when weight scaling is in use.
 *   - the gradient of the scale A is not printed in the paper; it is the derivative of
 *     Eq. 12:  dL/dW = a * dL/dW_scale,  dL/da = sum over the row segment of dL/dW_scale * W.
 *   - the packed (values + index metadata) layout is not in the paper; see oracle_project_compress.
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py except the
 * packed metadata LAYOUT itself, which is this project's own definition ("parity unpinned"
 * by the paper; pinned only by an independent decoder and its invariants), and the choice of
 * generator behind the stochastically rounded bf16 second moment (oracle_sr_bits: which mixer,
 * which constants, which 16 of its 32 bits are this project's definition, "parity unpinned";
 * what a rounding needs of it, uniform bits without structure along index and seed, is pinned,
 * and the rounding itself is pinned exactly).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

typedef struct {
    int32_t n_keep;         /* N                                                        */
    int32_t m_group;        /* M                                                        */
    float   lr;             /* gamma_t                              Algorithm 1         */
    float   beta1, beta2;   /* beta_1, beta_2                       Algorithm 1 inputs  */
    float   eps;            /* epsilon                                                   */
    float   lambda;         /* regularization strength lambda       Eq. 7               */
    float   alpha;          /* alpha_t = t / T                      Eq. 7               */
    float   bias_corr1;     /* 1 - beta_1^t  (given by the caller)  Eq. 8               */
    float   bias_corr2;     /* 1 - beta_2^t                                             */
    int32_t refresh_mask;   /* 1: recompute the mask from the incoming weights (Eq. 6)  */
    int32_t scale_segments; /* n of Eq. 12; 0 = gradient is already w.r.t. W            */
    int32_t v_from_grad;    /* 1: second moment from g^2 (Eq. 9 form, test pin only)    */
    int32_t rule;           /* which update rule; 0 = AdamS (Eq. 8), see RULE_* below   */
    int32_t mu_bf16;        /* 1: the first moment is KEPT in bf16 between iterations (a
                             * storage variant outside the paper): what is stored is the new
                             * mu rounded to nearest-even bf16; everything computed in the
                             * same iteration (mu~, v, the update) uses the unrounded value  */
    int32_t v_bf16;         /* 1: the second moment is kept in bf16 too, rounded STOCHASTICALLY
                             * when stored (with beta_2 = 0.999 a step changes v by a thousandth,
                             * less than half a bf16 unit in the last place: rounded to nearest it
                             * would never move).  Outside the paper like mu_bf16; the update of
                             * the same iteration uses the unrounded value.  See
                             * oracle_bf16_stochastic and oracle_sr_bits.                     */
    uint32_t sr_seed;       /* seed of the rounding bits; the caller changes it every iteration */
} oracle_adams_cfg;

uint16_t oracle_bf16_rne(float x);

uint16_t oracle_bf16_stochastic(float x, uint32_t r16);
uint32_t oracle_sr_bits(uint32_t seed, uint64_t index);

/* the value a stochastically rounded bf16 store of x reads back as; index = row * cols + col */
static float through_bf16_sr(float x, uint32_t seed, int64_t index)
{
    uint32_t bits = (uint32_t)oracle_bf16_stochastic(x, oracle_sr_bits(seed, (uint64_t)index)) << 16;
    float y;
    memcpy(&y, &bits, sizeof y);
    return y;
}

/* the value a bf16 store of x reads back as */
static float through_bf16(float x)
{
    uint32_t bits = (uint32_t)oracle_bf16_rne(x) << 16;
    float y;
    memcpy(&y, &bits, sizeof y);
    return y;
}

/* The update rules the paper sets AdamS against (Sec. 4.1.2, 4.1.3, 5.7).  In all of them the
 * decay acts only where the mask bit is 0 and has strength alpha*lambda, like Eq. 7's second
 * term (Eq. 9 and 10 are printed for a single always-decayed parameter with strength lambda:
 * alpha = 1 and mask bit 0 give exactly the printed forms). */
enum {
    RULE_ADAMS = 0,          /* Eq. 8                                                         */
    RULE_ADAMW_L1 = 1,       /* Eq. 9: decay added to the update, outside the moments          */
    RULE_ADAM_L1 = 2,        /* Eq. 10: decay added to the gradient, inside both moments       */
    RULE_ADDITIVE = 3,       /* Eq. 8 with mu~ = mu + alpha*lambda*Sign: decay added to, not   */
                             /* traded against, the momentum (the "additive decay" of Fig. 3) */
    RULE_MASKED_FROZEN = 4   /* sparsity-aware fine-tuning (Sec. 6.7): entries with mask bit 0 */
                             /* are not updated at all; the others follow Eq. 8 (mu~ = mu)     */
};

/* ------------------------------------------------------------------------------------ */
/* Eq. 6 with the tie rule above.                                                        */

static uint32_t magnitude_key(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, sizeof bits);
    return bits & 0x7fffffffu;
}

/* keep[j] = 1 iff fewer than N entries of the group precede entry j in the order
 * "larger magnitude first, then lower index first". */
static void select_group(const float *w, int M, int N, uint8_t *keep)
{
    for (int j = 0; j < M; ++j) {
        int rank = 0;
        uint32_t kj = magnitude_key(w[j]);
        for (int k = 0; k < M; ++k) {
            uint32_t kk = magnitude_key(w[k]);
            if (kk > kj || (kk == kj && k < j)) ++rank;
        }
        keep[j] = (uint8_t)(rank < N);
    }
}

int oracle_nm_select(const float *w, int64_t rows, int64_t cols, int n_keep, int m_group,
                     uint8_t *keep /* [rows*cols], 0 or 1 */)
{
    if (m_group < 2 || n_keep < 1 || n_keep >= m_group || cols % m_group) return -1;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t i = 0; i < cols / m_group; ++i)
            select_group(w + r * cols + i * m_group, m_group, n_keep, keep + r * cols + i * m_group);
    return 0;
}

/* Mask storage used by the library: one bit per parameter, each row padded to whole
 * 32-bit words; bit (c % 32) of word [r * ceil(cols/32) + c / 32] is M[r, c]. */
void oracle_pack_mask_bits(const uint8_t *keep, int64_t rows, int64_t cols, uint32_t *words)
{
    int64_t wpr = (cols + 31) / 32;
    for (int64_t k = 0; k < rows * wpr; ++k) words[k] = 0u;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c)
            if (keep[r * cols + c]) words[r * wpr + c / 32] |= (uint32_t)1 << (c % 32);
}

void oracle_unpack_mask_bits(const uint32_t *words, int64_t rows, int64_t cols, uint8_t *keep)
{
    int64_t wpr = (cols + 31) / 32;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c)
            keep[r * cols + c] = (uint8_t)((words[r * wpr + c / 32] >> (c % 32)) & 1u);
}

/* ------------------------------------------------------------------------------------ */
/* One parameter, one iteration of Algorithm 1 (body of its inner loop), real arithmetic
 * carried in double.                                                                    */

typedef struct {
    double lr, beta1, beta2, eps, lambda, alpha, bias_corr1, bias_corr2;
    int v_from_grad;
    int rule;
} adams_params_f64;

static double sign_f64(double x) { return (double)(x > 0.0) - (double)(x < 0.0); }

/* Eq. 9 (decay after the adaptive step) and Eq. 10 (decay inside the gradient), real arithmetic. */
static void adamw_l1_element_f64(double theta_prev, double g, double mu_prev, double v_prev, int m_bit,
                                 const adams_params_f64 *p, double *theta, double *mu, double *v)
{
    double mu_t = p->beta1 * mu_prev + (1.0 - p->beta1) * g;
    double v_t = p->beta2 * v_prev + (1.0 - p->beta2) * g * g;
    double mu_hat = mu_t / p->bias_corr1;
    double v_hat = v_t / p->bias_corr2;
    double update = mu_hat / (sqrt(v_hat) + p->eps);
    if (m_bit == 0) update += p->alpha * p->lambda * sign_f64(theta_prev);
    *theta = theta_prev - p->lr * update;
    *mu = mu_t;
    *v = v_t;
}

static void adam_l1_element_f64(double theta_prev, double g, double mu_prev, double v_prev, int m_bit,
                                const adams_params_f64 *p, double *theta, double *mu, double *v)
{
    double g_tilde = g;
    if (m_bit == 0) g_tilde += p->alpha * p->lambda * sign_f64(theta_prev);
    double mu_t = p->beta1 * mu_prev + (1.0 - p->beta1) * g_tilde;
    double v_t = p->beta2 * v_prev + (1.0 - p->beta2) * g_tilde * g_tilde;
    double mu_hat = mu_t / p->bias_corr1;
    double v_hat = v_t / p->bias_corr2;
    *theta = theta_prev - p->lr * (mu_hat / (sqrt(v_hat) + p->eps));
    *mu = mu_t;
    *v = v_t;
}

static void adams_element_f64(double theta_prev, double g, double mu_prev, double v_prev, int m_bit,
                              const adams_params_f64 *p, double *theta, double *mu, double *v)
{
    if (p->rule == RULE_ADAMW_L1) { adamw_l1_element_f64(theta_prev, g, mu_prev, v_prev, m_bit, p, theta, mu, v); return; }
    if (p->rule == RULE_ADAM_L1) { adam_l1_element_f64(theta_prev, g, mu_prev, v_prev, m_bit, p, theta, mu, v); return; }
    if (p->rule == RULE_MASKED_FROZEN && m_bit == 0) { *theta = theta_prev; *mu = mu_prev; *v = v_prev; return; }
    double mu_t = p->beta1 * mu_prev + (1.0 - p->beta1) * g;
    double mu_tilde;
    if (m_bit == 0 && p->rule == RULE_ADDITIVE)
        mu_tilde = mu_t + p->alpha * p->lambda * sign_f64(theta_prev);
    else if (m_bit == 0)
        mu_tilde = (1.0 - p->alpha) * mu_t + p->alpha * p->lambda * sign_f64(theta_prev);
    else
        mu_tilde = mu_t;
    double second = p->v_from_grad ? g * g : mu_tilde * mu_tilde;
    double v_t = p->beta2 * v_prev + (1.0 - p->beta2) * second;
    double mu_hat = mu_tilde / p->bias_corr1;
    double v_hat = v_t / p->bias_corr2;
    *theta = theta_prev - p->lr * (mu_hat / (sqrt(v_hat) + p->eps));
    *mu = mu_t; /* the stored first moment is the undecayed one */
    *v = v_t;
}

/* The same body with every operation rounded to fp32 once, in the order written, with no
 * fused multiply-add: the arithmetic a GPU kernel that keeps its state in fp32 performs.
 * It exists so that decisions an integer depends on (the next mask refresh) are taken in
 * the precision the state is held in. */
typedef struct {
    float lr, beta1, one_minus_beta1, beta2, one_minus_beta2, eps;
    float one_minus_alpha, alpha_lambda, bias_corr1, bias_corr2;
    int v_from_grad;
    int rule;
} adams_params_f32;

static float sign_f32(float x) { return (float)(x > 0.0f) - (float)(x < 0.0f); }

/* Eq. 9 and Eq. 10, one fp32 rounding per operation in the order written. */
static void adamw_l1_element_f32(float theta_prev, float g, float mu_prev, float v_prev, int m_bit,
                                 const adams_params_f32 *p, float *theta, float *mu, float *v)
{
    float t0 = p->beta1 * mu_prev;
    float t1 = p->one_minus_beta1 * g;
    float mu_t = t0 + t1;
    float second = g * g;
    float s0 = p->beta2 * v_prev;
    float s1 = p->one_minus_beta2 * second;
    float v_t = s0 + s1;
    float mu_hat = mu_t / p->bias_corr1;
    float v_hat = v_t / p->bias_corr2;
    float denom = sqrtf(v_hat) + p->eps;
    float update = mu_hat / denom;
    if (m_bit == 0) {
        float decay = p->alpha_lambda * sign_f32(theta_prev);
        update = update + decay;
    }
    float step = p->lr * update;
    *theta = theta_prev - step;
    *mu = mu_t;
    *v = v_t;
}

static void adam_l1_element_f32(float theta_prev, float g, float mu_prev, float v_prev, int m_bit,
                                const adams_params_f32 *p, float *theta, float *mu, float *v)
{
    float g_tilde = g;
    if (m_bit == 0) {
        float decay = p->alpha_lambda * sign_f32(theta_prev);
        g_tilde = g + decay;
    }
    float t0 = p->beta1 * mu_prev;
    float t1 = p->one_minus_beta1 * g_tilde;
    float mu_t = t0 + t1;
    float second = g_tilde * g_tilde;
    float s0 = p->beta2 * v_prev;
    float s1 = p->one_minus_beta2 * second;
    float v_t = s0 + s1;
    float mu_hat = mu_t / p->bias_corr1;
    float v_hat = v_t / p->bias_corr2;
    float denom = sqrtf(v_hat) + p->eps;
    float q = mu_hat / denom;
    float step = p->lr * q;
    *theta = theta_prev - step;
    *mu = mu_t;
    *v = v_t;
}

static void adams_element_f32(float theta_prev, float g, float mu_prev, float v_prev, int m_bit,
                              const adams_params_f32 *p, float *theta, float *mu, float *v)
{
    if (p->rule == RULE_ADAMW_L1) { adamw_l1_element_f32(theta_prev, g, mu_prev, v_prev, m_bit, p, theta, mu, v); return; }
    if (p->rule == RULE_ADAM_L1) { adam_l1_element_f32(theta_prev, g, mu_prev, v_prev, m_bit, p, theta, mu, v); return; }
    if (p->rule == RULE_MASKED_FROZEN && m_bit == 0) { *theta = theta_prev; *mu = mu_prev; *v = v_prev; return; }
    float t0 = p->beta1 * mu_prev;
    float t1 = p->one_minus_beta1 * g;
    float mu_t = t0 + t1;
    float mu_tilde;
    if (m_bit == 0 && p->rule == RULE_ADDITIVE) {
        float d1 = p->alpha_lambda * sign_f32(theta_prev);
        mu_tilde = mu_t + d1;
    } else if (m_bit == 0) {
        float sgn = (float)(theta_prev > 0.0f) - (float)(theta_prev < 0.0f);
        float d0 = p->one_minus_alpha * mu_t;
        float d1 = p->alpha_lambda * sgn;
        mu_tilde = d0 + d1;
    } else {
        mu_tilde = mu_t;
    }
    float second = p->v_from_grad ? g * g : mu_tilde * mu_tilde;
    float s0 = p->beta2 * v_prev;
    float s1 = p->one_minus_beta2 * second;
    float v_t = s0 + s1;
    float mu_hat = mu_tilde / p->bias_corr1;
    float v_hat = v_t / p->bias_corr2;
    float denom = sqrtf(v_hat) + p->eps;
    float q = mu_hat / denom;
    float step = p->lr * q;
    *theta = theta_prev - step;
    *mu = mu_t;
    *v = v_t;
}

static int check_step_shape(int64_t rows, int64_t cols, const oracle_adams_cfg *c)
{
    if (rows < 0 || cols < 0) return -1;
    if (c->rule < RULE_ADAMS || c->rule > RULE_MASKED_FROZEN) return -1;
    if (c->m_group < 2 || c->n_keep < 1 || c->n_keep >= c->m_group) return -1;
    if (cols % c->m_group) return -1;
    if (c->scale_segments < 0) return -1;
    if (c->scale_segments > 0) {
        if (cols % c->scale_segments) return -1;
        if ((cols / c->scale_segments) % c->m_group) return -1; /* no group straddles two segments */
    }
    return 0;
}

/*
 * One AdamS iteration over one weight matrix, state stored in fp32, arithmetic in double.
 *   w, mu, v  [rows, cols] fp32, updated in place
 *   grad      [rows, cols] fp32 (a bf16 gradient is widened, exactly, by the caller);
 *             dL/dW when A == NULL, dL/dW_scale when A != NULL
 *   keep      [rows, cols] bytes; written when cfg->refresh_mask, read otherwise
 *   A         [rows, n] scale factors of Eq. 12, or NULL
 *   gA        [rows, n] out: dL/dA, or NULL
 */
int oracle_adams_step_f64(float *w, const float *grad, float *mu, float *v, uint8_t *keep,
                          const float *A, double *gA, int64_t rows, int64_t cols,
                          const oracle_adams_cfg *cfg, int nthreads)
{
    if (check_step_shape(rows, cols, cfg)) return -1;
    const int M = cfg->m_group, N = cfg->n_keep, n = cfg->scale_segments;
    if ((A != NULL) != (n > 0)) return -1;
    adams_params_f64 p = { cfg->lr, cfg->beta1, cfg->beta2, cfg->eps, cfg->lambda, cfg->alpha,
                           cfg->bias_corr1, cfg->bias_corr2, cfg->v_from_grad, cfg->rule };
    (void)nthreads;
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        if (gA) for (int s = 0; s < n; ++s) gA[r * n + s] = 0.0;
        for (int64_t i = 0; i < cols / M; ++i) {
            int64_t base = r * cols + i * M;
            if (cfg->refresh_mask) select_group(w + base, M, N, keep + base);
            for (int j = 0; j < M; ++j) {
                int64_t c = i * M + j, idx = base + j;
                double g = grad[idx];
                if (A) {
                    int64_t s = c / (cols / n);
                    if (gA) gA[r * n + s] += (double)grad[idx] * (double)w[idx];
                    g = (double)A[r * n + s] * (double)grad[idx];
                }
                double th, m1, v1;
                adams_element_f64(w[idx], g, mu[idx], v[idx], keep[idx], &p, &th, &m1, &v1);
                w[idx] = (float)th;
                mu[idx] = cfg->mu_bf16 ? through_bf16((float)m1) : (float)m1;
                v[idx] = cfg->v_bf16 ? through_bf16_sr((float)v1, cfg->sr_seed, idx) : (float)v1;
            }
        }
    }
    return 0;
}

/* As above with the per-operation fp32 arithmetic.  gA is still summed in double. */
int oracle_adams_step_f32(float *w, const float *grad, float *mu, float *v, uint8_t *keep,
                          const float *A, double *gA, int64_t rows, int64_t cols,
                          const oracle_adams_cfg *cfg, int nthreads)
{
    if (check_step_shape(rows, cols, cfg)) return -1;
    const int M = cfg->m_group, N = cfg->n_keep, n = cfg->scale_segments;
    if ((A != NULL) != (n > 0)) return -1;
    adams_params_f32 p;
    p.lr = cfg->lr;
    p.beta1 = cfg->beta1;
    p.one_minus_beta1 = 1.0f - cfg->beta1;
    p.beta2 = cfg->beta2;
    p.one_minus_beta2 = 1.0f - cfg->beta2;
    p.eps = cfg->eps;
    p.one_minus_alpha = 1.0f - cfg->alpha;
    p.alpha_lambda = cfg->alpha * cfg->lambda;
    p.bias_corr1 = cfg->bias_corr1;
    p.bias_corr2 = cfg->bias_corr2;
    p.v_from_grad = cfg->v_from_grad;
    p.rule = cfg->rule;
    (void)nthreads;
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        if (gA) for (int s = 0; s < n; ++s) gA[r * n + s] = 0.0;
        for (int64_t i = 0; i < cols / M; ++i) {
            int64_t base = r * cols + i * M;
            if (cfg->refresh_mask) select_group(w + base, M, N, keep + base);
            for (int j = 0; j < M; ++j) {
                int64_t c = i * M + j, idx = base + j;
                float g = grad[idx];
                if (A) {
                    int64_t s = c / (cols / n);
                    if (gA) gA[r * n + s] += (double)grad[idx] * (double)w[idx];
                    g = A[r * n + s] * grad[idx];
                }
                float th, m1, v1;
                adams_element_f32(w[idx], g, mu[idx], v[idx], keep[idx], &p, &th, &m1, &v1);
                w[idx] = th;
                mu[idx] = cfg->mu_bf16 ? through_bf16(m1) : m1;
                v[idx] = cfg->v_bf16 ? through_bf16_sr(v1, cfg->sr_seed, idx) : v1;
            }
        }
    }
    return 0;
}

/* Algorithm 1's inner loop on a flat array with the whole state in double and the mask
 * given.  Used only to pin the arithmetic against closed forms and a library Adam to
 * double-precision tolerances. */
int oracle_adams_elements_state64(double *theta, const double *grad, double *mu, double *v,
                                  const uint8_t *m_bits, int64_t count, double lr, double beta1,
                                  double beta2, double eps, double lambda, double alpha,
                                  double bias_corr1, double bias_corr2, int v_from_grad, int rule)
{
    adams_params_f64 p = { lr, beta1, beta2, eps, lambda, alpha, bias_corr1, bias_corr2, v_from_grad, rule };
    for (int64_t i = 0; i < count; ++i)
        adams_element_f64(theta[i], grad[i], mu[i], v[i], m_bits[i], &p, &theta[i], &mu[i], &v[i]);
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Eq. 12: row-major reshape (R x C) -> (R*n x C/n); segment s of row r is scaled by A[r, s]. */

int oracle_weight_scale(const float *w, const float *A, int64_t rows, int64_t cols, int n, float *out)
{
    if (n < 1 || cols % n) return -1;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c)
            out[r * cols + c] = A[r * n + c / (cols / n)] * w[r * cols + c];
    return 0;
}

/* dL/dA[r, s] = sum over the columns of segment s of dL/dW_scale[r, c] * W[r, c]. */
int oracle_weight_scale_grad(const float *w, const float *grad_scaled, int64_t rows, int64_t cols,
                             int n, double *gA)
{
    if (n < 1 || cols % n) return -1;
    for (int64_t r = 0; r < rows; ++r)
        for (int s = 0; s < n; ++s) {
            double acc = 0.0;
            for (int64_t c = s * (cols / n); c < (s + 1) * (cols / n); ++c)
                acc += (double)grad_scaled[r * cols + c] * (double)w[r * cols + c];
            gA[r * n + s] = acc;
        }
    return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Final hard prune, fold of the scale, and packing.
 *
 * keep == NULL : true projection, the mask is Eq. 6 on the given weights
 * keep != NULL : Algorithm 1 as printed, the last refreshed mask is applied
 *
 * values [rows, cols*N/M]: for each group, its kept entries in ascending column order,
 *        each multiplied once (fp32) by A[r, s] when A != NULL.
 * meta:  each kept entry's position inside its group in b = ceil(log2 M) bits; a group's N
 *        positions are concatenated in ascending order, the first in the least significant
 *        bits; the group field is padded to f = the next power of two >= N*b bits; 32/f
 *        groups share a word, group i of a row sits at bit (i % (32/f)) * f of word
 *        [r * ceil((cols/M) * f / 32) + i / (32/f)]; unused bits are zero.
 */
static int ceil_log2(int x) { int b = 0; while ((1 << b) < x) ++b; return b; }

int oracle_meta_field_bits(int n_keep, int m_group)
{
    int raw = n_keep * ceil_log2(m_group), f = 1;
    while (f < raw) f <<= 1;
    return f;
}

int oracle_project_compress(const float *w, const float *A, int n, const uint8_t *keep_in,
                            int64_t rows, int64_t cols, int n_keep, int m_group,
                            float *values, uint32_t *meta)
{
    if (m_group < 2 || n_keep < 1 || n_keep >= m_group || cols % m_group) return -1;
    if (A && (n < 1 || cols % n || (cols / n) % m_group)) return -1;
    const int b = ceil_log2(m_group), f = oracle_meta_field_bits(n_keep, m_group);
    if (f > 32) return -1;
    const int64_t groups = cols / m_group, gpw = 32 / f, mwpr = (groups + gpw - 1) / gpw;
    for (int64_t k = 0; k < rows * mwpr; ++k) meta[k] = 0u;
    uint8_t keep[64];
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t i = 0; i < groups; ++i) {
            const float *wg = w + r * cols + i * m_group;
            if (keep_in) memcpy(keep, keep_in + r * cols + i * m_group, (size_t)m_group);
            else select_group(wg, m_group, n_keep, keep);
            uint32_t field = 0u;
            int q = 0;
            for (int j = 0; j < m_group; ++j) {
                if (!keep[j]) continue;
                if (q >= n_keep) return -2; /* a given mask with more than N ones in a group */
                float val = wg[j];
                if (A) val = A[r * n + (i * m_group + j) / (cols / n)] * val;
                values[r * groups * n_keep + i * n_keep + q] = val;
                field |= (uint32_t)j << (q * b);
                ++q;
            }
            if (q != n_keep) return -2;
            meta[r * mwpr + i / gpw] |= field << ((i % gpw) * f);
        }
    return 0;
}

/* fp32 -> bf16, round to nearest, ties to even; any NaN becomes the quiet NaN 0x7FC0. */
uint16_t oracle_bf16_rne(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, sizeof bits);
    if ((bits & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    uint32_t lsb = (bits >> 16) & 1u;
    bits += 0x7fffu + lsb;
    return (uint16_t)(bits >> 16);
}

/* Stochastic rounding of a fp32 value to bf16 with 16 given random bits r16 (0 .. 65535): the
 * value is rounded away from zero with probability (discarded low bits) / 65536, towards zero
 * otherwise, so the expectation over uniform r16 is the value itself; a value that is a bf16
 * number already is never changed.  Done on the bit pattern: adding r16 to the 32 bits carries
 * into bit 16 exactly when low16 + r16 >= 65536 (a carry out of the mantissa moves to the next
 * binade, the largest finite values can reach infinity).  Infinities and NaN go through the
 * round-to-nearest conversion. */
uint16_t oracle_bf16_stochastic(float x, uint32_t r16)
{
    uint32_t bits;
    memcpy(&bits, &x, sizeof bits);
    if ((bits & 0x7f800000u) == 0x7f800000u) return oracle_bf16_rne(x);
    return (uint16_t)((bits + (r16 & 0xffffu)) >> 16);
}

/* The integer finalizer published as "lowbias32" (C. Wellons, "Prospecting for hash functions",
 * 2018): xor-shift 16, multiply 0x7feb352d, xor-shift 15, multiply 0x846ca68b, xor-shift 16. */
static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

/* The 16 rounding bits of one matrix entry: a counter-based generator (nothing is carried from
 * entry to entry or step to step), this project's own definition.  The seed is mixed into a key
 * first (so that seeds that differ in a few low bits, a step counter say, do not hand an entry
 * the bits its neighbour had a step earlier), the key is folded with the 64-bit entry index into
 * 32 bits, those are mixed, and the upper 16 bits are used. */
uint32_t oracle_sr_bits(uint32_t seed, uint64_t index)
{
    uint32_t key = mix32(seed + 0x9e3779b9u);
    uint32_t x = (uint32_t)index ^ key;
    x += (uint32_t)(index >> 32) * 0x9e3779b9u;
    return mix32(x) >> 16;
}

void oracle_bf16_rne_array(const float *x, int64_t count, uint16_t *out)
{
    for (int64_t i = 0; i < count; ++i) out[i] = oracle_bf16_rne(x[i]);
}

/* ------------------------------------------------------------------------------------ */
/* Appendix "Mask Learning": numerators and denominators of r_t / i_t (mask changes against
 * another mask) and of S_t (kept L1 mass over total L1 mass), for one matrix. */
int oracle_mask_stats(const float *w, const uint8_t *keep, const uint8_t *keep_other,
                      int64_t count, int64_t *flips, double *l1_kept, double *l1_total)
{
    int64_t f = 0;
    double a = 0.0, b = 0.0;
    for (int64_t i = 0; i < count; ++i) {
        if (keep_other && keep[i] != keep_other[i]) ++f;
        double mag = fabs((double)w[i]);
        b += mag;
        if (keep[i]) a += mag;
    }
    *flips = f;
    *l1_kept = a;
    *l1_total = b;
    return 0;
}
