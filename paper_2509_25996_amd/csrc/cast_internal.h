// Host-side declarations shared by the translation units of libcast (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/cast.h"
#include "cast_device.h"

namespace cast {

// How one launch covers a matrix.  With weight scaling a span is one row segment of Eq. 12, so
// its scale factor is a wave-uniform scalar and dL/dA of that segment is reduced inside the
// workgroup, written once, without atomics.  Without scaling a dense matrix is treated as one
// flat array cut into short spans; a matrix with strided rows is cut into equal pieces of its rows.
struct SpanPlan {
    bool vec;            // the vector kernels apply (spans start on mask-word boundaries)
    SpanGeom geom;
    int block_threads;   // a multiple of 64, from 256 to 1024
    unsigned grid;       // workgroups
    int64_t segments;    // split plans: row segments of the matrix (rows * n), else 0
};

// Not part of the ABI (cast_adams_config::flags with this bit is refused): set by cast_hbm_stream_probe on its own
// copy of the configuration to make the list call run the probe flavour of the step kernel.
constexpr uint32_t kInternalFlagStreamProbe = 0x80000000u;

// allow_split: row segments of more than 16 chunks of 256 entries may be cut into pieces with a
// workgroup each; the caller then supplies a PieceArea for the pieces' dL/dA sums.
SpanPlan plan_spans(int64_t rows, int64_t cols, int64_t ld, int n_segments, bool allow_split = false);
// How the selection, scaling and pack kernels cover a matrix (see RowsGeom): `lane_entries` consecutive entries
// per thread and load.  vec = false: the shape goes to the scalar kernels.
struct RowsPlan {
    bool vec;
    bool same_row;       // rows are whole numbers of workgroups
    RowsGeom geom;
    unsigned grid;       // workgroups per matrix
};
RowsPlan plan_rows(int64_t rows, int64_t cols, int64_t ld, int lane_entries);
constexpr int kMaxListed = 16;      // matrices of equal shape that one launch of these kernels can take (gridDim.y)

// Device memory for the piece sums of split plans: what is left of it, and who collects the
// second halves (adding the pieces up) of the matrices that took a part.
struct PieceArea {
    float *base;
    uint64_t floats;
    void *jobs;
};

struct StatsPartial;

// Device memory for the per-workgroup refresh statistics: what is left of it, and who collects
// the jobs that add the slots of a matrix up.
struct StatsArea {
    StatsPartial *base;
    uint64_t slots;
    void *jobs;
};

// What a step may do beyond Algorithm 1's loop body.
struct StepExtras {
    void *compute_copy = nullptr;              // bf16 copy of the new weights for the next forward pass
    const float *copy_scale = nullptr;         // the A folded into it
    const uint32_t *initial_mask = nullptr;    // refresh statistics: the mask flips_init counts against
    cast_refresh_stats *refresh_stats = nullptr;
    PieceArea *area = nullptr;                 // list calls: room for split plans
    StatsArea *stats_area = nullptr;           // list calls: room for refresh statistics
};

cast_status launch_adams_step(float *w, const void *grad, float *m, float *v, uint32_t *mask_bits,
                              const float *scale, float *scale_grad, int64_t rows, int64_t cols,
                              int64_t ld, const cast_adams_config *cfg, const StepExtras &extras,
                              hipStream_t stream);
cast_status launch_scale_grad(const float *w, const void *grad, int grad_dtype, int64_t rows,
                              int64_t cols, int64_t ld, int n_segments, float *scale_grad,
                              hipStream_t stream);
cast_status launch_scale_grad_list(const cast_scale_grad_matrix *m, int count, int grad_dtype, int n_segments,
                                   hipStream_t stream);
// Matrices of one shape (and, for `alike`, the same optional buffers) go several to a launch: up to
// kMaxListed of them and about 72 M entries, the rule of the step kernels (a short launch pays some 2.6 us
// of ramp, a very long one lets the compute units drift apart).  Collects into `group` the indices, from
// `first` on, of matrices not yet taken that are like matrix `first`, and marks them taken.
template <typename Matrix, typename Alike>
inline int take_group(const Matrix *m, int count, std::vector<char> &taken, int first, Alike alike, int (&group)[kMaxListed])
{
    const Matrix &t = m[first];
    int most = kMaxListed;
    const int64_t entries = t.rows * t.cols;
    const int64_t launch_entries = (int64_t)72 << 20;
    if (entries > 0 && launch_entries / entries < most) most = (int)(launch_entries / entries);
    if (most < 1) most = 1;
    int n = 0;
    group[n++] = first;
    taken[first] = 1;
    for (int j = first + 1; j < count && n < most; ++j)
        if (!taken[j] && m[j].rows == t.rows && m[j].cols == t.cols && m[j].ld == t.ld && alike(m[j], t)) {
            group[n++] = j;
            taken[j] = 1;
        }
    return n;
}

// Lists of matrices (already validated): matrices of one shape share launches.
cast_status launch_nm_select_list(const cast_matrix *m, int count, int n_keep, int m_group, hipStream_t stream);
cast_status launch_weight_scale_list(const cast_matrix *m, int count, int n_segments, int out_dtype, hipStream_t stream);
cast_status launch_project_compress_list(const cast_matrix *m, int count, int n_segments, int n_keep, int m_group,
                                         int value_dtype, hipStream_t stream);
size_t mask_stats_list_workspace_bytes(const cast_stats_matrix *m, int count);
cast_status launch_mask_stats_list(const cast_stats_matrix *m, int count, void *workspace, hipStream_t stream);
cast_status launch_mask_stats(const float *w, const uint32_t *mask_bits, const uint32_t *other_bits,
                              int64_t rows, int64_t cols, int64_t ld, unsigned long long *flips,
                              double *l1, hipStream_t stream);
cast_status launch_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t stream);
size_t multi_workspace_bytes(const cast_tensor *tensors, int count, const cast_adams_config *cfg);
struct MultiTally {
    int step_launches;     // launches of the step kernels (a launch may step several matrices)
    int other_launches;    // dL/dA reductions of odd shapes, sums of split plans and of refresh statistics
    int split_matrices = 0;
};
// taken: `count` bytes of host scratch
cast_status launch_adams_step_multi(const cast_tensor *tensors, int count, const cast_adams_config *cfg,
                                    void *workspace, char *taken, hipStream_t stream, MultiTally *tally = nullptr);
// Device address, on the current GPU, of the library's built-in workspace of CAST_NOALLOC_SCRATCH_BYTES bytes.
cast_status builtin_workspace(void **out);
cast_status debug_div_by_uniform(const float *x, float y, float *out, int64_t n);

inline cast_status launch_status()
{
    return hipGetLastError() == hipSuccess ? CAST_OK : CAST_ERR_LAUNCH;
}

inline int meta_index_bits(int m_group) { return m_group == 2 ? 1 : (m_group == 4 ? 2 : 3); }
inline int meta_field_bits(int n_keep, int m_group)
{
    int raw = n_keep * meta_index_bits(m_group), f = 1;
    while (f < raw) f <<= 1;
    return f;
}

}  // namespace cast
