// The C ABI of libcast: argument validation on the host, then dispatch to the kernels.
// Nothing here touches the device except the kernel launches themselves.
#include <math.h>

#include <vector>

#include "cast_internal.h"

using namespace cast;

namespace {

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

cast_status check_nm(int n_keep, int m_group)
{
    if (m_group != 2 && m_group != 4 && m_group != 8) return CAST_ERR_SHAPE;
    if (n_keep < 1 || n_keep >= m_group) return CAST_ERR_SHAPE;
    return CAST_OK;
}

cast_status check_ld(int64_t cols, int64_t ld) { return ld >= cols ? CAST_OK : CAST_ERR_SHAPE; }

cast_status check_matrix(int64_t rows, int64_t cols, int m_group)
{
    if (rows < 0 || cols < 0) return CAST_ERR_SHAPE;
    if (cols % m_group) return CAST_ERR_SHAPE;
    if (rows > 0 && cols > 0 && rows > INT64_MAX / cols) return CAST_ERR_SHAPE;
    // one launch covers at most 2^31-1 workgroups of 4 spans of >= 256 entries
    if (rows > 0 && cols > 0 && rows * cols > ((int64_t)1 << 40)) return CAST_ERR_SHAPE;
    return CAST_OK;
}

cast_status check_segments(int64_t cols, int n_segments, int m_group)
{
    if (n_segments < 1) return CAST_ERR_SHAPE;
    if (cols % n_segments) return CAST_ERR_SHAPE;
    if ((cols / n_segments) % m_group) return CAST_ERR_SHAPE;   // no group in two segments
    return CAST_OK;
}

// one wavefront per row segment, 4 per workgroup, at most 2^31-1 workgroups per launch
bool too_many_segments(int64_t rows, int n_segments) { return rows > (((int64_t)1 << 31) / n_segments); }

bool dtype_ok(int d) { return d == CAST_F32 || d == CAST_BF16; }
size_t dtype_align(int d) { return d == CAST_BF16 ? 8 : 16; }

}  // namespace

extern "C" {

const char *cast_status_str(cast_status s)
{
    switch (s) {
    case CAST_OK: return "ok";
    case CAST_ERR_NULL: return "a required pointer is NULL";
    case CAST_ERR_SHAPE: return "shape, N:M or segment count not accepted";
    case CAST_ERR_ALIGN: return "a buffer is not aligned as required";
    case CAST_ERR_DTYPE: return "unknown dtype code";
    case CAST_ERR_CONFIG: return "a configuration scalar is out of range";
    case CAST_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case CAST_ERR_SCRATCH: return "the list needs more workspace, or has more matrices, than the entry point that allocates nothing holds";
    default: return "unknown status";
    }
}

cast_status cast_sizes(int64_t rows, int64_t cols, int n_keep, int m_group, int value_dtype,
                       size_t *mask_bytes, size_t *values_bytes, size_t *meta_bytes)
{
    cast_status rc = check_nm(n_keep, m_group);
    if (rc != CAST_OK) return rc;
    rc = check_matrix(rows, cols, m_group);
    if (rc != CAST_OK) return rc;
    if (!dtype_ok(value_dtype)) return CAST_ERR_DTYPE;
    const int f = meta_field_bits(n_keep, m_group);
    const int64_t groups = cols / m_group, gpw = 32 / f;
    if (mask_bytes) *mask_bytes = (size_t)(rows * ((cols + 31) / 32)) * 4;
    if (values_bytes) *values_bytes = (size_t)(rows * groups * n_keep) * (value_dtype == CAST_BF16 ? 2 : 4);
    if (meta_bytes) *meta_bytes = (size_t)(rows * ((groups + gpw - 1) / gpw)) * 4;
    return CAST_OK;
}

static cast_status validate_select(const cast_matrix &t, int n_keep, int m_group)
{
    cast_status rc = check_nm(n_keep, m_group);
    if (rc != CAST_OK) return rc;
    rc = check_matrix(t.rows, t.cols, m_group);
    if (rc != CAST_OK) return rc;
    if (check_ld(t.cols, t.ld) != CAST_OK) return CAST_ERR_SHAPE;
    if (t.rows == 0 || t.cols == 0) return CAST_OK;
    if (!t.w || !t.mask_bits) return CAST_ERR_NULL;
    if (!aligned(t.w, 16) || !aligned(t.mask_bits, 4)) return CAST_ERR_ALIGN;
    return CAST_OK;
}

cast_status cast_nm_select_multi(const cast_matrix *matrices, int count, int n_keep, int m_group, void *stream)
{
    if (count < 0) return CAST_ERR_SHAPE;
    if (count == 0) return CAST_OK;
    if (!matrices) return CAST_ERR_NULL;
    for (int i = 0; i < count; ++i) {      // all or nothing
        const cast_status rc = validate_select(matrices[i], n_keep, m_group);
        if (rc != CAST_OK) return rc;
    }
    return launch_nm_select_list(matrices, count, n_keep, m_group, static_cast<hipStream_t>(stream));
}

cast_status cast_nm_select(const float *w, int64_t rows, int64_t cols, int64_t ld, int n_keep,
                           int m_group, uint32_t *mask_bits, void *stream)
{
    const cast_matrix t{w, rows, cols, ld, nullptr, mask_bits, nullptr, nullptr, nullptr};
    return cast_nm_select_multi(&t, 1, n_keep, m_group, stream);
}

// everything cast_adams_step checks before launching
static cast_status validate_step(const float *w, const void *grad, const float *m, const float *v,
                                 const uint32_t *mask_bits, const float *scale, const float *scale_grad,
                                 int64_t rows, int64_t cols, int64_t ld, const cast_adams_config *cfg,
                                 const void *compute_copy = nullptr, const float *copy_scale = nullptr)
{
    if (!cfg) return CAST_ERR_NULL;
    cast_status rc = check_nm(cfg->n_keep, cfg->m_group);
    if (rc != CAST_OK) return rc;
    rc = check_matrix(rows, cols, cfg->m_group);
    if (rc != CAST_OK) return rc;
    if (check_ld(cols, ld) != CAST_OK) return CAST_ERR_SHAPE;
    if (!dtype_ok(cfg->grad_dtype)) return CAST_ERR_DTYPE;
    if (cfg->scale_segments < 0) return CAST_ERR_SHAPE;
    if (cfg->flags & ~(CAST_FLAG_V_FROM_GRAD | CAST_FLAG_MU_BF16 | CAST_FLAG_V_BF16)) return CAST_ERR_CONFIG;
    if ((cfg->flags & CAST_FLAG_V_BF16) && !(cfg->flags & CAST_FLAG_MU_BF16)) return CAST_ERR_CONFIG;      // both moments or the first alone
    if (cfg->rule < CAST_RULE_ADAMS || cfg->rule > CAST_RULE_MASKED_FROZEN) return CAST_ERR_CONFIG;
    if ((cfg->flags & CAST_FLAG_MU_BF16) && cfg->rule != CAST_RULE_ADAMS && cfg->rule != CAST_RULE_ADDITIVE) return CAST_ERR_CONFIG;
    // the bias corrections divide: they must be positive finite numbers (1 - beta^s with s >= 1)
    if (!(cfg->bias_corr1 > 0.0f) || !(cfg->bias_corr2 > 0.0f) || isinf(cfg->bias_corr1) || isinf(cfg->bias_corr2))
        return CAST_ERR_CONFIG;
    if (rows == 0 || cols == 0) return CAST_OK;      // nothing to do: buffers may be NULL
    if ((cfg->scale_segments > 0) != (scale != nullptr)) return scale ? CAST_ERR_SHAPE : CAST_ERR_NULL;
    if (scale_grad && !scale) return CAST_ERR_NULL;
    if (copy_scale && (!compute_copy || cfg->scale_segments == 0)) return compute_copy ? CAST_ERR_SHAPE : CAST_ERR_NULL;
    if (cfg->scale_segments > 0 && cols > 0) {
        rc = check_segments(cols, cfg->scale_segments, cfg->m_group);
        if (rc != CAST_OK) return rc;
        if (too_many_segments(rows, cfg->scale_segments)) return CAST_ERR_SHAPE;
    }
    if (!w || !grad || !m || !v || !mask_bits) return CAST_ERR_NULL;
    if (!aligned(w, 16) || !aligned(m, 16) || !aligned(v, 16) || !aligned(grad, dtype_align(cfg->grad_dtype)) ||
        !aligned(mask_bits, 4) || !aligned(scale, 4) || !aligned(scale_grad, 4) || !aligned(compute_copy, 16) ||
        !aligned(copy_scale, 4))
        return CAST_ERR_ALIGN;
    return CAST_OK;
}

cast_status cast_adams_step_emit(float *w, const void *grad, float *m, float *v, uint32_t *mask_bits,
                                 const float *scale, float *scale_grad, const float *copy_scale,
                                 void *compute_copy, int64_t rows, int64_t cols, int64_t ld,
                                 const cast_adams_config *cfg, void *stream)
{
    const cast_status rc = validate_step(w, grad, m, v, mask_bits, scale, scale_grad, rows, cols, ld, cfg, compute_copy, copy_scale);
    if (rc != CAST_OK) return rc;
    if (rows > 0 && cols > 0 && !compute_copy) return CAST_ERR_NULL;
    StepExtras x;
    x.compute_copy = compute_copy;
    x.copy_scale = copy_scale;
    return launch_adams_step(w, grad, m, v, mask_bits, scale, scale_grad, rows, cols, ld, cfg, x, static_cast<hipStream_t>(stream));
}

cast_status cast_adams_step(float *w, const void *grad, float *m, float *v, uint32_t *mask_bits,
                            const float *scale, float *scale_grad, int64_t rows, int64_t cols,
                            int64_t ld, const cast_adams_config *cfg, void *stream)
{
    const cast_status rc = validate_step(w, grad, m, v, mask_bits, scale, scale_grad, rows, cols, ld, cfg);
    if (rc != CAST_OK) return rc;
    return launch_adams_step(w, grad, m, v, mask_bits, scale, scale_grad, rows, cols, ld, cfg, StepExtras{},
                             static_cast<hipStream_t>(stream));
}

size_t cast_adams_multi_workspace_bytes(const cast_tensor *tensors, int count, const cast_adams_config *cfg)
{
    return multi_workspace_bytes(tensors, count, cfg);
}

cast_status cast_adams_step_multi(const cast_tensor *tensors, int count, const cast_adams_config *cfg,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (count < 0) return CAST_ERR_SHAPE;
    if (!cfg) return CAST_ERR_NULL;
    if (count == 0) return CAST_OK;
    if (!tensors) return CAST_ERR_NULL;
    if (!aligned(workspace, 16)) return CAST_ERR_ALIGN;
    for (int i = 0; i < count; ++i) {    // all or nothing: nothing is launched if any matrix is rejected
        const cast_tensor &t = tensors[i];
        const cast_status rc = validate_step(t.w, t.grad, t.m, t.v, t.mask_bits, t.scale, t.scale_grad, t.rows, t.cols, t.ld, cfg,
                                             t.compute_copy, t.copy_scale);
        if (rc != CAST_OK) return rc;
    }
    for (int i = 0; i < count; ++i)
        if (!aligned(tensors[i].initial_mask_bits, 4) || !aligned(tensors[i].refresh_stats, 8)) return CAST_ERR_ALIGN;
    const size_t need = multi_workspace_bytes(tensors, count, cfg);
    if (need > 0 && !workspace) return CAST_ERR_NULL;
    if (workspace_bytes < need) return CAST_ERR_SHAPE;
    std::vector<char> taken((size_t)count);
    return launch_adams_step_multi(tensors, count, cfg, workspace, taken.data(), static_cast<hipStream_t>(stream));
}

cast_status cast_adams_step_multi_noalloc(const cast_tensor *tensors, int count, const cast_adams_config *cfg, void *stream)
{
    if (count < 0) return CAST_ERR_SHAPE;
    if (!cfg) return CAST_ERR_NULL;
    if (count == 0) return CAST_OK;
    if (!tensors) return CAST_ERR_NULL;
    if (count > CAST_NOALLOC_MAX_TENSORS) return CAST_ERR_SCRATCH;
    for (int i = 0; i < count; ++i) {
        const cast_tensor &t = tensors[i];
        const cast_status rc = validate_step(t.w, t.grad, t.m, t.v, t.mask_bits, t.scale, t.scale_grad, t.rows, t.cols, t.ld, cfg,
                                             t.compute_copy, t.copy_scale);
        if (rc != CAST_OK) return rc;
    }
    for (int i = 0; i < count; ++i)
        if (!aligned(tensors[i].initial_mask_bits, 4) || !aligned(tensors[i].refresh_stats, 8)) return CAST_ERR_ALIGN;
    if (multi_workspace_bytes(tensors, count, cfg) > (size_t)CAST_NOALLOC_SCRATCH_BYTES) return CAST_ERR_SCRATCH;
    void *workspace = nullptr;
    const cast_status rc = builtin_workspace(&workspace);
    if (rc != CAST_OK) return rc;
    char taken[CAST_NOALLOC_MAX_TENSORS];      // host scratch on the stack: nothing is allocated anywhere
    return launch_adams_step_multi(tensors, count, cfg, workspace, taken, static_cast<hipStream_t>(stream));
}

cast_status cast_adams_multi_launches(const cast_tensor *tensors, int count, const cast_adams_config *cfg,
                                      int32_t *step_launches, int32_t *other_launches)
{
    if (count < 0) return CAST_ERR_SHAPE;
    if (!cfg || (count > 0 && !tensors)) return CAST_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const cast_tensor &t = tensors[i];
        const cast_status rc = validate_step(t.w, t.grad, t.m, t.v, t.mask_bits, t.scale, t.scale_grad, t.rows, t.cols, t.ld, cfg,
                                             t.compute_copy, t.copy_scale);
        if (rc != CAST_OK) return rc;
    }
    MultiTally tally{0, 0};
    std::vector<char> taken((size_t)count);
    const cast_status rc = launch_adams_step_multi(tensors, count, cfg, nullptr, taken.data(), nullptr, &tally);
    if (step_launches) *step_launches = tally.step_launches;
    if (other_launches) *other_launches = tally.other_launches;
    return rc;
}

static cast_status validate_scale(const cast_matrix &t, int n_segments, int out_dtype)
{
    if (t.rows < 0 || t.cols < 0 || n_segments < 1 || (t.cols % n_segments) || t.ld < t.cols) return CAST_ERR_SHAPE;
    if (t.rows > 0 && t.cols > 0 && t.rows > (((int64_t)1 << 40) / t.cols)) return CAST_ERR_SHAPE;
    if (!dtype_ok(out_dtype)) return CAST_ERR_DTYPE;
    if (t.rows == 0 || t.cols == 0) return CAST_OK;
    if (!t.w || !t.scale || !t.out) return CAST_ERR_NULL;
    if (!aligned(t.w, 16) || !aligned(t.out, dtype_align(out_dtype)) || !aligned(t.scale, 4)) return CAST_ERR_ALIGN;
    return CAST_OK;
}

cast_status cast_weight_scale_multi(const cast_matrix *matrices, int count, int n_segments, int out_dtype, void *stream)
{
    if (count < 0) return CAST_ERR_SHAPE;
    if (count == 0) return CAST_OK;
    if (!matrices) return CAST_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const cast_status rc = validate_scale(matrices[i], n_segments, out_dtype);
        if (rc != CAST_OK) return rc;
    }
    return launch_weight_scale_list(matrices, count, n_segments, out_dtype, static_cast<hipStream_t>(stream));
}

cast_status cast_weight_scale(const float *w, const float *scale, int64_t rows, int64_t cols,
                              int64_t ld, int n_segments, void *out, int out_dtype, void *stream)
{
    const cast_matrix t{w, rows, cols, ld, scale, nullptr, out, nullptr, nullptr};
    return cast_weight_scale_multi(&t, 1, n_segments, out_dtype, stream);
}

static cast_status validate_scale_grad(const cast_scale_grad_matrix &t, int grad_dtype, int n_segments)
{
    if (t.rows < 0 || t.cols < 0 || n_segments < 1 || (t.cols % n_segments) || t.ld < t.cols) return CAST_ERR_SHAPE;
    if (t.rows > 0 && t.cols > 0 && t.rows > (((int64_t)1 << 40) / t.cols)) return CAST_ERR_SHAPE;
    if (!dtype_ok(grad_dtype)) return CAST_ERR_DTYPE;
    if (too_many_segments(t.rows, n_segments)) return CAST_ERR_SHAPE;
    if (t.rows == 0 || t.cols == 0) return CAST_OK;
    if (!t.w || !t.grad_scaled || !t.scale_grad) return CAST_ERR_NULL;
    if (!aligned(t.w, 16) || !aligned(t.grad_scaled, dtype_align(grad_dtype)) || !aligned(t.scale_grad, 4)) return CAST_ERR_ALIGN;
    return CAST_OK;
}

cast_status cast_weight_scale_grad_multi(const cast_scale_grad_matrix *matrices, int count, int grad_dtype,
                                         int n_segments, void *stream)
{
    if (count < 0) return CAST_ERR_SHAPE;
    if (!dtype_ok(grad_dtype)) return CAST_ERR_DTYPE;
    if (count == 0) return CAST_OK;
    if (!matrices) return CAST_ERR_NULL;
    for (int i = 0; i < count; ++i) {      // all or nothing
        const cast_status rc = validate_scale_grad(matrices[i], grad_dtype, n_segments);
        if (rc != CAST_OK) return rc;
    }
    return launch_scale_grad_list(matrices, count, grad_dtype, n_segments, static_cast<hipStream_t>(stream));
}

cast_status cast_weight_scale_grad(const float *w, const void *grad_scaled, int grad_dtype,
                                   int64_t rows, int64_t cols, int64_t ld, int n_segments,
                                   float *scale_grad, void *stream)
{
    const cast_scale_grad_matrix t{w, grad_scaled, rows, cols, ld, scale_grad};
    return cast_weight_scale_grad_multi(&t, 1, grad_dtype, n_segments, stream);
}

static cast_status validate_pack(const cast_matrix &t, int n_segments, int n_keep, int m_group, int value_dtype)
{
    cast_status rc = check_nm(n_keep, m_group);
    if (rc != CAST_OK) return rc;
    rc = check_matrix(t.rows, t.cols, m_group);
    if (rc != CAST_OK) return rc;
    if (check_ld(t.cols, t.ld) != CAST_OK) return CAST_ERR_SHAPE;
    if (!dtype_ok(value_dtype)) return CAST_ERR_DTYPE;
    if (t.scale && t.cols > 0) {
        rc = check_segments(t.cols, n_segments, m_group);
        if (rc != CAST_OK) return rc;
    }
    if (t.rows == 0 || t.cols == 0) return CAST_OK;
    if (!t.w || !t.out || !t.meta) return CAST_ERR_NULL;
    if (!aligned(t.w, 16) || !aligned(t.out, 8) || !aligned(t.meta, 4) || !aligned(t.mask_bits, 4) || !aligned(t.scale, 4) ||
        !aligned(t.mask_status, 4))
        return CAST_ERR_ALIGN;
    return CAST_OK;
}

cast_status cast_nm_project_compress_multi(const cast_matrix *matrices, int count, int n_segments, int n_keep, int m_group,
                                           int value_dtype, void *stream)
{
    if (count < 0) return CAST_ERR_SHAPE;
    if (count == 0) return CAST_OK;
    if (!matrices) return CAST_ERR_NULL;
    for (int i = 0; i < count; ++i) {
        const cast_status rc = validate_pack(matrices[i], n_segments, n_keep, m_group, value_dtype);
        if (rc != CAST_OK) return rc;
    }
    return launch_project_compress_list(matrices, count, n_segments, n_keep, m_group, value_dtype, static_cast<hipStream_t>(stream));
}

cast_status cast_nm_project_compress(const float *w, const float *scale, int n_segments,
                                     const uint32_t *mask_bits, int64_t rows, int64_t cols,
                                     int64_t ld, int n_keep, int m_group, void *values,
                                     int value_dtype, uint32_t *meta, void *stream)
{
    const cast_matrix t{w, rows, cols, ld, scale, const_cast<uint32_t *>(mask_bits), values, meta, nullptr};
    return cast_nm_project_compress_multi(&t, 1, n_segments, n_keep, m_group, value_dtype, stream);
}

cast_status cast_mask_stats(const float *w, const uint32_t *mask_bits, const uint32_t *other_bits,
                            int64_t rows, int64_t cols, int64_t ld, unsigned long long *flips,
                            double *l1, void *stream)
{
    if (rows < 0 || cols < 0 || ld < cols) return CAST_ERR_SHAPE;
    if (rows > 0 && cols > 0 && rows > (((int64_t)1 << 40) / cols)) return CAST_ERR_SHAPE;
    if (rows == 0 || cols == 0) return CAST_OK;
    if (!w || !mask_bits || !flips || !l1) return CAST_ERR_NULL;
    if (!aligned(w, 4) || !aligned(mask_bits, 4) || !aligned(other_bits, 4) || !aligned(flips, 8) || !aligned(l1, 8))
        return CAST_ERR_ALIGN;
    return launch_mask_stats(w, mask_bits, other_bits, rows, cols, ld, flips, l1, static_cast<hipStream_t>(stream));
}

size_t cast_mask_stats_multi_workspace_bytes(const cast_stats_matrix *matrices, int count)
{
    return matrices && count > 0 ? mask_stats_list_workspace_bytes(matrices, count) : 0;
}

cast_status cast_mask_stats_multi(const cast_stats_matrix *matrices, int count, void *workspace, size_t workspace_bytes,
                                  void *stream)
{
    if (count < 0) return CAST_ERR_SHAPE;
    if (count == 0) return CAST_OK;
    if (!matrices) return CAST_ERR_NULL;
    for (int i = 0; i < count; ++i) {      // all or nothing
        const cast_stats_matrix &t = matrices[i];
        if (t.rows < 0 || t.cols < 0 || t.ld < t.cols) return CAST_ERR_SHAPE;
        if (t.rows > 0 && t.cols > 0 && t.rows > (((int64_t)1 << 40) / t.cols)) return CAST_ERR_SHAPE;
        if (!t.stats) return CAST_ERR_NULL;
        if (!aligned(t.stats, 8)) return CAST_ERR_ALIGN;
        if (t.rows == 0 || t.cols == 0) continue;
        if (!t.w || !t.mask_bits) return CAST_ERR_NULL;
        if (!aligned(t.w, 4) || !aligned(t.mask_bits, 4) || !aligned(t.other_bits, 4)) return CAST_ERR_ALIGN;
    }
    const size_t need = mask_stats_list_workspace_bytes(matrices, count);
    if (need > 0 && !workspace) return CAST_ERR_NULL;
    if (!aligned(workspace, 16)) return CAST_ERR_ALIGN;
    if (workspace_bytes < need) return CAST_ERR_SHAPE;
    return launch_mask_stats_list(matrices, count, workspace, static_cast<hipStream_t>(stream));
}

cast_status cast_hbm_copy_probe(void *dst, const void *src, size_t bytes, void *stream)
{
    if (bytes == 0) return CAST_OK;
    if (!dst || !src) return CAST_ERR_NULL;
    if (bytes % 16) return CAST_ERR_SHAPE;
    if (!aligned(dst, 16) || !aligned(src, 16)) return CAST_ERR_ALIGN;
    return launch_copy_probe(dst, src, bytes, static_cast<hipStream_t>(stream));
}

cast_status cast_hbm_stream_probe(const cast_tensor *tensors, int count, int scale_segments, int grad_dtype,
                                  uint32_t moment_flags, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!dtype_ok(grad_dtype)) return CAST_ERR_DTYPE;
    if (moment_flags != 0 && moment_flags != CAST_FLAG_MU_BF16 && moment_flags != (CAST_FLAG_MU_BF16 | CAST_FLAG_V_BF16)) return CAST_ERR_CONFIG;
    if (moment_flags != 0 && grad_dtype != CAST_BF16) return CAST_ERR_CONFIG;
    cast_adams_config cfg{};
    cfg.n_keep = 2;
    cfg.m_group = 4;
    cfg.beta1 = 0.5f;
    cfg.beta2 = 0.5f;
    cfg.bias_corr1 = 1.0f;
    cfg.bias_corr2 = 1.0f;
    cfg.refresh_mask = 0;
    cfg.scale_segments = scale_segments;
    cfg.grad_dtype = grad_dtype;
    cfg.flags = moment_flags;
    if (count < 0) return CAST_ERR_SHAPE;
    if (count == 0) return CAST_OK;
    if (!tensors) return CAST_ERR_NULL;
    if (!aligned(workspace, 16)) return CAST_ERR_ALIGN;
    for (int i = 0; i < count; ++i) {
        const cast_tensor &t = tensors[i];
        const cast_status rc = validate_step(t.w, t.grad, t.m, t.v, t.mask_bits, t.scale, t.scale_grad, t.rows, t.cols, t.ld, &cfg);
        if (rc != CAST_OK) return rc;
        if (t.compute_copy || t.refresh_stats) return CAST_ERR_CONFIG;
        // only shapes the vector kernels take: the others would run the real step
        if (t.rows > 0 && t.cols > 0 && !plan_spans(t.rows, t.cols, t.ld, scale_segments, false).vec) return CAST_ERR_SHAPE;
    }
    const size_t need = multi_workspace_bytes(tensors, count, &cfg);
    if (need > 0 && !workspace) return CAST_ERR_NULL;
    if (workspace_bytes < need) return CAST_ERR_SHAPE;
    cfg.flags |= kInternalFlagStreamProbe;
    std::vector<char> taken((size_t)count);
    return launch_adams_step_multi(tensors, count, &cfg, workspace, taken.data(), static_cast<hipStream_t>(stream));
}

cast_status cast_debug_plan(int64_t rows, int64_t cols, int64_t ld, int n_segments, int allow_split,
                            int64_t block, int wave, int64_t plan[5], int64_t span[5])
{
    if (!plan || !span) return CAST_ERR_NULL;
    if (rows <= 0 || cols <= 0 || ld < cols || n_segments < 0 || block < 0 || wave < 0) return CAST_ERR_SHAPE;
    if (n_segments > 0 && cols % n_segments) return CAST_ERR_SHAPE;
    // allow_split: 0, 1 = the step kernels' plan without / with split plans; 2, 3 = the plan of the selection and
    // pack kernels with spans starting on 32 / 64 columns
    if (allow_split < 0 || allow_split > 3 || (allow_split >= 2 && n_segments != 0)) return CAST_ERR_SHAPE;
    if (allow_split >= 2) {      // the selection, scaling and pack kernels: 4 or 8 entries per thread and load
        const RowsPlan r = plan_rows(rows, cols, ld, allow_split == 2 ? 4 : 8);
        const int slots = kBlockWaves * r.geom.loads;
        plan[0] = r.vec ? 1 : 0;
        plan[1] = r.grid;
        plan[2] = slots;
        plan[3] = 1;
        plan[4] = 1;
        for (int k = 0; k < 5; ++k) span[k] = 0;
        if (!r.vec || block >= (int64_t)r.grid || wave >= slots) return CAST_OK;
        const RowsPiece piece = r.same_row ? rows_piece<true>(r.geom, (uint32_t)block, wave % kBlockWaves, wave / kBlockWaves)
                                           : rows_piece<false>(r.geom, (uint32_t)block, wave % kBlockWaves, wave / kBlockWaves);
        const int64_t col = piece.col;
        if (col >= cols) return CAST_OK;
        const int64_t len = kWave * r.geom.lane_entries;
        span[0] = (int64_t)piece.row * ld + col;
        span[1] = (int64_t)piece.row * cols + col;
        span[2] = col + len <= cols ? len : cols - col;
        span[3] = block * slots + wave;      // a span of its own for every wavefront and piece
        span[4] = 0;
        return CAST_OK;
    }
    const SpanPlan p = plan_spans(rows, cols, ld, n_segments, allow_split != 0);
    const int block_waves = p.block_threads / kWave;
    plan[0] = p.vec ? 1 : 0;
    plan[1] = p.grid;
    plan[2] = block_waves;
    plan[3] = p.geom.waves_per_span;
    plan[4] = p.geom.pieces_per_segment;
    for (int k = 0; k < 5; ++k) span[k] = 0;
    if (!p.vec || block >= (int64_t)p.grid || wave >= block_waves) return CAST_OK;
    const SpanSlot slot = span_slot(p.geom, block, wave, block_waves);
    int64_t segment = slot.span;
    const SpanOrigin o = p.geom.pieces_per_segment > 1 ? piece_origin(p.geom, slot.span, segment) : span_origin(p.geom, slot.span);
    span[0] = o.state_begin;
    span[1] = o.dense_begin;
    span[2] = o.len;
    span[3] = slot.span;
    span[4] = slot.sub;
    return CAST_OK;
}

cast_status cast_debug_div_by_uniform(const float *x, float y, float *out, int64_t n)
{
    if (n < 0) return CAST_ERR_SHAPE;
    if (n == 0) return CAST_OK;
    if (!x || !out) return CAST_ERR_NULL;
    return debug_div_by_uniform(x, y, out, n);
}

}  // extern "C"
