// Host side of the AdamS step: how a launch covers a matrix (plan_spans), which kernel
// instantiation runs, and how a list of matrices becomes launches.  The kernels are in
// adams_step_kernels.h.
#include <stdlib.h>

#include <mutex>
#include <vector>

#include "adams_step_kernels.h"

#pragma clang fp contract(off)

namespace cast {

// Collects the second halves of the split plans of a list call and launches them in batches.
struct PieceJobQueue {
    PieceJobs pending;
    int count = 0;
    int64_t most_segments = 0;

    cast_status flush(hipStream_t st)
    {
        if (count == 0) return CAST_OK;
        const unsigned grid = (unsigned)((most_segments + kBlockThreads - 1) / kBlockThreads);
        hipLaunchKernelGGL(sum_piece_sums, dim3(grid, (unsigned)count), dim3(kBlockThreads), 0, st, pending);
        count = 0;
        most_segments = 0;
        return launch_status();
    }

    bool full() const { return count == kMaxPieceJobs; }

    void add(const PieceJob &j)      // not when full()
    {
        pending.job[count++] = j;
        if (j.segments > most_segments) most_segments = j.segments;
    }
};

// Collects the jobs that add up the refresh statistics of a list call and launches them in batches.
struct StatsJobQueue {
    StatsJobs pending;
    int count = 0;

    cast_status flush(hipStream_t st)
    {
        if (count == 0) return CAST_OK;
        hipLaunchKernelGGL(sum_refresh_stats, dim3((unsigned)count), dim3(kMaxBlockThreads), 0, st, pending);
        count = 0;
        return launch_status();
    }
    bool full() const { return count == kMaxStatsJobs; }
    void add(const StatsJob &j) { pending.job[count++] = j; }      // not when full()
};


// The comparison rule as the kernel flavour carries it: those with code of their own, else none.
static int flavour_rule(int rule)
{
    return rule == CAST_RULE_ADAMW_L1 ? kRuleAdamwL1 : rule == CAST_RULE_ADAM_L1 ? kRuleAdamL1 : rule == CAST_RULE_MASKED_FROZEN ? kRuleMaskedFrozen : 0;
}

// The kernel flavour for one matrix: how the moments are stored comes first (the API has seen to it that bf16
// moments do not come with the rules that have code of their own), then the rule and what else the kernel has to do.
static int step_flavour(const cast_adams_config *cfg, bool copy, bool stats)
{
    if (cfg->flags & kInternalFlagStreamProbe)
        return (cfg->flags & CAST_FLAG_V_BF16) ? kStreamProbeBothBf16 : (cfg->flags & CAST_FLAG_MU_BF16) ? kStreamProbeMuBf16 : kStreamProbe;
    if (cfg->flags & CAST_FLAG_V_BF16) return (copy || stats) ? kBothBf16Emit : kBothBf16;
    if (cfg->flags & CAST_FLAG_MU_BF16) return (copy || stats) ? kMuBf16Emit : kMuBf16;
    const int rule = flavour_rule(cfg->rule);
    if (rule != 0) return with_rule((copy || stats) ? kEmitAndCount : 0, rule);
    return copy ? kEmitAndCount : (stats ? kStatsOnly : 0);
}

// Launch-plan parameters.  The shipped library uses the measured-best constants; a build with
// -DCAST_TUNING (never the one build.py makes) reads them from the environment once per process,
// for sweeps.  They decide the span and piece plan, hence the summation order of dL/dA and the
// launch counts, which is why the product build does not let the environment near them.
#ifdef CAST_TUNING
static int knob(const char *name, int fallback, int lo, int hi)
{
    const char *e = getenv(name);
    if (!e || !*e) return fallback;
    const int x = atoi(e);
    return x < lo || x > hi ? fallback : x;
}
#else
static constexpr int knob(const char *, int fallback, int, int) { return fallback; }
#endif

SpanPlan plan_spans(int64_t rows, int64_t cols, int64_t ld, int n_segments, bool allow_split)
{
    // HBM rewards a narrow window of addresses in flight: wavefronts are kept short-lived (about
    // one chunk of 256 entries each) and the spans of one workgroup are contiguous, so that the
    // workgroups the dispatcher has resident at any time cover a compact range of every array.
    // CAST_SPAN_LEN forces the flat span length (a multiple of 256, at most 64 chunks: a wavefront's flip
    // counts and offsets stay far below 32 bits), CAST_WAVES_PER_SPAN the number of cooperating
    // wavefronts, CAST_BLOCK_WAVES the workgroup size in wavefronts; 0 = chosen by the plan.
    static const int forced_len = knob("CAST_SPAN_LEN", 0, 0, 64 * kChunk);
    static const int forced_p = knob("CAST_WAVES_PER_SPAN", 0, 0, kMaxBlockWaves);
    static const int forced_bw = knob("CAST_BLOCK_WAVES", 0, 0, kMaxBlockWaves);
    static const int piece_len = knob("CAST_PIECE_LEN", 1024, 32, 1 << 20);
    SpanPlan p{};
    SpanGeom &g = p.geom;
    g.total = rows * cols;
    g.cols = cols;
    g.row_gap = ld - cols;
    g.m_row_gap = g.row_gap;
    g.waves_per_span = 1;
    g.div_spans_per_row = make_fast_div(1);
    g.pieces_per_segment = 1;
    g.div_pieces = make_fast_div(1);
    static const int split_min_chunks = knob("CAST_SPLIT_MIN_CHUNKS", kPieceChunks + 1, 2, 1 << 20);
    static const int piece_chunks_knob = knob("CAST_PIECE_CHUNKS", 0, 0, kPieceChunks);      // 0: chosen per segment length
    int block_waves = kBlockWaves;
    int per_row = n_segments;
    if (per_row == 0 && ld != cols) {
        // strided rows, no scaling: cut every row into equal pieces that start on mask words
        for (int k = 1; k <= 64 && per_row == 0; ++k)
            if (cols % k == 0 && (cols / k) % 32 == 0 && cols / k <= piece_len) per_row = k;
        if (per_row == 0 && cols % 32 == 0 && cols < ((int64_t)1 << 28)) per_row = 1;
    }
    if (per_row > 0) {
        g.spans_per_row = per_row;
        g.div_spans_per_row = make_fast_div((uint32_t)per_row);
        g.span_len = cols / per_row;
        g.num_spans = rows * per_row;
        p.vec = cols % per_row == 0 && g.span_len % 32 == 0 && g.span_len < ((int64_t)1 << 28) && ld % 4 == 0 &&
                g.num_spans < ((int64_t)1 << 31);
        const int64_t chunks = (g.span_len + kChunk - 1) / kChunk;
        // Pieces of 8, 4 or 2 chunks: the largest size that leaves at most 11 % of the wavefronts of a
        // segment's workgroups without a chunk (21.5 chunks: 8, 8, 5.5; 28 chunks: seven fours; 10 chunks:
        // five twos).  Measured on the benchmark shapes: smaller pieces than needed are no faster.
        int piece_chunks = 2;
        for (int c = kPieceChunks; c > 2; c /= 2) {
            const int64_t slots = (chunks + c - 1) / c * c * kChunk;      // entries the wavefronts could take
            if ((slots - g.span_len) * 100 <= slots * 11) { piece_chunks = c; break; }
        }
        if (piece_chunks_knob == 1 || piece_chunks_knob == 2 || piece_chunks_knob == 4 || piece_chunks_knob == 8) piece_chunks = piece_chunks_knob;
        const int64_t pieces = (chunks + piece_chunks - 1) / piece_chunks;
        g.segment_len = g.span_len;
        // 8 and 16 chunks fill one workgroup of 8 or 16 wavefronts exactly and stay whole
        if (allow_split && p.vec && n_segments > 0 && chunks >= split_min_chunks && chunks != kMaxBlockWaves && pieces > 1 &&
            g.num_spans * pieces < ((int64_t)1 << 31) && pieces * per_row < ((int64_t)1 << 24)) {
            // More chunks than a workgroup has wavefronts, or a number of them that leaves wavefront slots
            // of the compute units empty (10-wavefront workgroups fill 30 of 32): with several chunks per
            // wavefront the workgroups are few, large and long-lived, and the compute units run half empty.
            // Cut the segment into pieces, one chunk per wavefront, workgroups of 8 wavefronts.
            g.pieces_per_segment = (int)pieces;
            g.div_pieces = make_fast_div((uint32_t)pieces);
            g.span_len = (int64_t)piece_chunks * kChunk;
            g.spans_per_row = per_row * (int)pieces;
            g.div_spans_per_row = make_fast_div((uint32_t)g.spans_per_row);
            p.segments = g.num_spans;
            g.num_spans *= pieces;
            g.waves_per_span = piece_chunks;
            block_waves = kPieceChunks;
        } else {
            if (chunks <= kBlockWaves) {
                while (chunks > g.waves_per_span) g.waves_per_span *= 2;     // 1, 2 or 4: several spans per workgroup
            } else {
                // one span per workgroup: a wavefront per chunk, or all 16 with one or more chunks each
                g.waves_per_span = chunks < kMaxBlockWaves ? (int)chunks : kMaxBlockWaves;
                block_waves = g.waves_per_span;
            }
        }
    } else {
        g.spans_per_row = 0;   // flat: the matrix is one contiguous array
        p.vec = cols % 32 == 0 && ld == cols;
        int64_t len = 2 * kChunk;
        if (forced_len >= kChunk && forced_len % kChunk == 0) len = forced_len;
        g.span_len = len;
        g.num_spans = (g.total + len - 1) / len;
    }
    if (g.pieces_per_segment == 1) {
        if (forced_p == 1 || forced_p == 2 || forced_p == 4 || forced_p == 8 || forced_p == 16) g.waves_per_span = forced_p;
        if (forced_bw == 4 || forced_bw == 8 || forced_bw == 16) block_waves = forced_bw;
    }
    if (block_waves < g.waves_per_span) block_waves = g.waves_per_span;
    if (block_waves % g.waves_per_span) block_waves = g.waves_per_span;
    p.block_threads = block_waves * kWave;
    const int64_t spans_per_block = block_waves / g.waves_per_span;
    p.grid = (unsigned)((g.num_spans + spans_per_block - 1) / spans_per_block);
    return p;
}

static StepScalars make_scalars(const cast_adams_config *cfg)
{
    StepScalars s;
    s.lr = cfg->lr;
    s.beta1 = cfg->beta1;
    s.one_minus_beta1 = 1.0f - cfg->beta1;
    s.beta2 = cfg->beta2;
    s.one_minus_beta2 = 1.0f - cfg->beta2;
    s.eps = cfg->eps;
    s.one_minus_alpha = 1.0f - cfg->alpha;
    s.alpha_lambda = cfg->alpha * cfg->lambda;
    s.bias_corr1 = make_divisor(cfg->bias_corr1);
    s.bias_corr2 = make_divisor(cfg->bias_corr2);
    s.decay_pos = s.alpha_lambda * 1.0f;
    s.decay_neg = s.alpha_lambda * -1.0f;
    s.decay_zero = s.alpha_lambda * 0.0f;       // keeps the sign a product with +0 has
    s.n_keep = cfg->n_keep;
    s.v_from_grad = (cfg->flags & CAST_FLAG_V_FROM_GRAD) ? 1 : 0;
    s.rule = cfg->rule;
    s.sr_key = sr_key_of(cfg->sr_seed);
    if (cfg->rule == CAST_RULE_ADDITIVE) s.one_minus_alpha = 1.0f;                              // mu~ = mu + alpha*lambda*Sign
    if (cfg->rule == CAST_RULE_ADAMW_L1 || cfg->rule == CAST_RULE_ADAM_L1) s.v_from_grad = 1;   // Eq. 9, Eq. 10
    // the short forms need both bias corrections in [2^-12, 2] and a small non-negative epsilon
    s.short_forms = (s.bias_corr1.fast && s.bias_corr2.fast && cfg->eps >= 0.0f && cfg->eps <= 0x1p20f) ? 1 : 0;
    return s;
}

// the shape of a vector launch
struct VecLaunch {
    unsigned grid_x, grid_y;
    int block_threads;
    bool split;
    int extra;       // the kernel flavour (EXTRA of adams_step_vec)
};

template <int M, bool BF16, bool REFRESH, bool SCALED, int EXTRA>
static void launch_vec_flavour(const VecLaunch &l, const SpanArgs &a, dim3 grid, dim3 block, hipStream_t st)
{
    if constexpr (SCALED) {
        if (l.split) {
            hipLaunchKernelGGL((adams_step_vec<M, BF16, REFRESH, true, true, EXTRA>), grid, block, 0, st, a);
            return;
        }
    }
    hipLaunchKernelGGL((adams_step_vec<M, BF16, REFRESH, SCALED, false, EXTRA>), grid, block, 0, st, a);
}

// The rules combine with the plain kernel and with the one that can write the compute copy and gather
// statistics; the other abilities exist for AdamS (and additive decay, which is AdamS to the kernels) only.
template <int M, bool BF16, bool REFRESH, bool SCALED, int RULE>
static void launch_vec_abilities(const VecLaunch &l, const SpanArgs &a, dim3 grid, dim3 block, hipStream_t st)
{
    if constexpr (RULE != 0) {
        if (abilities(l.extra) != 0) launch_vec_flavour<M, BF16, REFRESH, SCALED, with_rule(kEmitAndCount, RULE)>(l, a, grid, block, st);
        else launch_vec_flavour<M, BF16, REFRESH, SCALED, with_rule(0, RULE)>(l, a, grid, block, st);
    } else {
        switch (abilities(l.extra)) {
        case kEmitAndCount: launch_vec_flavour<M, BF16, REFRESH, SCALED, kEmitAndCount>(l, a, grid, block, st); break;
        case kMuBf16: launch_vec_flavour<M, BF16, REFRESH, SCALED, kMuBf16>(l, a, grid, block, st); break;
        case kMuBf16Emit: launch_vec_flavour<M, BF16, REFRESH, SCALED, kMuBf16Emit>(l, a, grid, block, st); break;
        case kBothBf16: launch_vec_flavour<M, BF16, REFRESH, SCALED, kBothBf16>(l, a, grid, block, st); break;
        case kBothBf16Emit: launch_vec_flavour<M, BF16, REFRESH, SCALED, kBothBf16Emit>(l, a, grid, block, st); break;
        // the bandwidth probes exist for 2:4 with a stored mask only; with bf16 moments for bf16 gradients only
        case kStreamProbe:
            if constexpr (M == 4 && !REFRESH) {
                launch_vec_flavour<4, BF16, false, SCALED, kStreamProbe>(l, a, grid, block, st);
                break;
            }
            [[fallthrough]];
        case kStreamProbeMuBf16:
            if constexpr (M == 4 && BF16 && !REFRESH) {
                if (abilities(l.extra) == kStreamProbeMuBf16) {
                    launch_vec_flavour<4, true, false, SCALED, kStreamProbeMuBf16>(l, a, grid, block, st);
                    break;
                }
            }
            [[fallthrough]];
        case kStreamProbeBothBf16:
            if constexpr (M == 4 && BF16 && !REFRESH) {
                if (abilities(l.extra) == kStreamProbeBothBf16) {
                    launch_vec_flavour<4, true, false, SCALED, kStreamProbeBothBf16>(l, a, grid, block, st);
                    break;
                }
            }
            [[fallthrough]];
        case kStatsOnly:      // refresh statistics without a compute copy: a flavour of the refresh kernels only
            if constexpr (REFRESH) {
                launch_vec_flavour<M, BF16, true, SCALED, kStatsOnly>(l, a, grid, block, st);
                break;
            }
            [[fallthrough]];
        default: launch_vec_flavour<M, BF16, REFRESH, SCALED, 0>(l, a, grid, block, st); break;
        }
    }
}

template <int M, bool BF16, bool REFRESH, bool SCALED>
static void launch_vec_kernel(const VecLaunch &l, const SpanArgs &a, hipStream_t st)
{
    const dim3 grid(l.grid_x, l.grid_y), block(l.block_threads);
    switch (rule_of(l.extra)) {
    case kRuleAdamwL1: launch_vec_abilities<M, BF16, REFRESH, SCALED, kRuleAdamwL1>(l, a, grid, block, st); break;
    case kRuleAdamL1: launch_vec_abilities<M, BF16, REFRESH, SCALED, kRuleAdamL1>(l, a, grid, block, st); break;
    case kRuleMaskedFrozen: launch_vec_abilities<M, BF16, REFRESH, SCALED, kRuleMaskedFrozen>(l, a, grid, block, st); break;
    default: launch_vec_abilities<M, BF16, REFRESH, SCALED, 0>(l, a, grid, block, st); break;
    }
}

template <int M, bool BF16>
static void launch_vec_flags(bool refresh, bool scaled, const VecLaunch &l, const SpanArgs &a, hipStream_t st)
{
    if (refresh) { if (scaled) launch_vec_kernel<M, BF16, true, true>(l, a, st); else launch_vec_kernel<M, BF16, true, false>(l, a, st); }
    else { if (scaled) launch_vec_kernel<M, BF16, false, true>(l, a, st); else launch_vec_kernel<M, BF16, false, false>(l, a, st); }
}

static void launch_vec_any(int m_group, bool bf16, bool refresh, bool scaled, const VecLaunch &l, const SpanArgs &a,
                           hipStream_t st)
{
    switch (m_group) {
    case 2: if (bf16) launch_vec_flags<2, true>(refresh, scaled, l, a, st); else launch_vec_flags<2, false>(refresh, scaled, l, a, st); break;
    case 4: if (bf16) launch_vec_flags<4, true>(refresh, scaled, l, a, st); else launch_vec_flags<4, false>(refresh, scaled, l, a, st); break;
    default: if (bf16) launch_vec_flags<8, true>(refresh, scaled, l, a, st); else launch_vec_flags<8, false>(refresh, scaled, l, a, st); break;
    }
}

template <int M>
static void launch_unit_dtype(bool bf16, unsigned grid, const UnitArgs &a, hipStream_t st)
{
    if (bf16) hipLaunchKernelGGL((adams_step_unit<M, true>), dim3(grid), dim3(kBlockThreads), 0, st, a);
    else hipLaunchKernelGGL((adams_step_unit<M, false>), dim3(grid), dim3(kBlockThreads), 0, st, a);
}

// dL/dA of a list (already validated): matrices of one shape and row stride share launches of the span kernel.
cast_status launch_scale_grad_list(const cast_scale_grad_matrix *m, int count, int grad_dtype, int n_segments, hipStream_t st)
{
    static_assert(kMaxListed <= kMaxFused, "a group of a list must fit the kernel's argument sets");
    const bool bf16 = grad_dtype == CAST_BF16;
    std::vector<char> taken((size_t)count, 0);
    for (int i = 0; i < count; ++i) {
        if (taken[i] || m[i].rows == 0 || m[i].cols == 0) continue;
        int group[kMaxListed];
        const int n = take_group(m, count, taken, i, [](const cast_scale_grad_matrix &, const cast_scale_grad_matrix &) { return true; }, group);
        const cast_scale_grad_matrix &t0 = m[i];
        const SpanPlan p = plan_spans(t0.rows, t0.cols, t0.ld, n_segments, false);
        if (p.vec) {
            ScaleGradArgs a{{}, p.geom};
            for (int k = 0; k < n; ++k) a.set[k] = ScaleGradSet{m[group[k]].w, m[group[k]].grad_scaled, m[group[k]].scale_grad};
            const dim3 grid(p.grid, (unsigned)n), block(p.block_threads);
            if (bf16) hipLaunchKernelGGL(scale_grad_vec<true>, grid, block, 0, st, a);
            else hipLaunchKernelGGL(scale_grad_vec<false>, grid, block, 0, st, a);
            if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
            continue;
        }
        for (int k = 0; k < n; ++k) {
            const cast_scale_grad_matrix &t = m[group[k]];
            const unsigned grid = (unsigned)((t.rows * n_segments + kBlockWaves - 1) / kBlockWaves);
            if (bf16) hipLaunchKernelGGL(scale_grad_rows<true>, dim3(grid), dim3(kBlockThreads), 0, st, t.w, t.grad_scaled, t.scale_grad, t.rows, t.cols, t.ld, n_segments);
            else hipLaunchKernelGGL(scale_grad_rows<false>, dim3(grid), dim3(kBlockThreads), 0, st, t.w, t.grad_scaled, t.scale_grad, t.rows, t.cols, t.ld, n_segments);
            if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
        }
    }
    return CAST_OK;
}

cast_status launch_scale_grad(const float *w, const void *grad, int grad_dtype, int64_t rows,
                              int64_t cols, int64_t ld, int n_segments, float *scale_grad, hipStream_t st)
{
    const cast_scale_grad_matrix t{w, grad, rows, cols, ld, scale_grad};
    return launch_scale_grad_list(&t, 1, grad_dtype, n_segments, st);
}

// Row stride, in its own entries, of a first moment kept in bf16: dense when w and v are, else the
// same byte pitch as theirs (the three arrays interleaved row by row in one allocation).
static int64_t mu_bf16_ld(int64_t cols, int64_t ld) { return ld == cols ? cols : 2 * ld; }

// Takes `slots` partial-sum slots out of the statistics area of a list call and queues the job
// that adds them up into `out` (the caller has checked that the area has the room).
static StatsPartial *take_stats_slots(StatsArea *area, uint64_t slots, cast_refresh_stats *out, const uint32_t *initial_mask)
{
    StatsPartial *base = area->base;
    area->base += slots;
    area->slots -= slots;
    static_cast<StatsJobQueue *>(area->jobs)->add(StatsJob{base, (int64_t)slots, out, initial_mask != nullptr});
    return base;
}

cast_status launch_adams_step(float *w, const void *grad, float *m, float *v, uint32_t *mask_bits,
                              const float *scale, float *scale_grad, int64_t rows, int64_t cols,
                              int64_t ld, const cast_adams_config *cfg, const StepExtras &x, hipStream_t st)
{
    if (rows == 0 || cols == 0) return CAST_OK;
    const bool bf16 = cfg->grad_dtype == CAST_BF16;
    const bool refresh = cfg->refresh_mask != 0;
    const bool scaled = scale != nullptr;
    PieceArea *area = x.area;
    SpanPlan p = plan_spans(rows, cols, ld, cfg->scale_segments, area != nullptr && scale_grad != nullptr);
    if (p.geom.pieces_per_segment > 1 && (uint64_t)p.geom.num_spans > area->floats)
        p = plan_spans(rows, cols, ld, cfg->scale_segments, false);       // no room for the pieces' sums
    const bool split = p.geom.pieces_per_segment > 1;
    // refresh statistics: one slot per workgroup in the caller's workspace, added up afterwards
    const int64_t unit_grid = (rows * ((cols + 63) / 64) + kBlockThreads - 1) / kBlockThreads;
    const uint64_t stats_slots = p.vec ? p.grid : (uint64_t)unit_grid;
    const bool stats = refresh && x.refresh_stats != nullptr && x.stats_area != nullptr && stats_slots <= x.stats_area->slots;
    if (refresh && x.refresh_stats != nullptr && !stats) return CAST_ERR_SHAPE;      // workspace too small (not reachable through the API)
    StatsPartial *stats_partials = stats ? take_stats_slots(x.stats_area, stats_slots, x.refresh_stats, x.initial_mask) : nullptr;
    const uint32_t *stats_initial = stats ? x.initial_mask : nullptr;
    const bool mu16 = (cfg->flags & CAST_FLAG_MU_BF16) != 0, v16 = (cfg->flags & CAST_FLAG_V_BF16) != 0;
    const int extra = step_flavour(cfg, x.compute_copy != nullptr, stats);
    p.geom.m_row_gap = mu_bf16_ld(cols, ld) - cols;
    if (p.vec) {
        SpanArgs a{{{w, grad, m, v, mask_bits, scale, scale_grad, split ? area->base : nullptr, stats_partials, stats_initial,
                     static_cast<uint16_t *>(x.compute_copy), x.copy_scale}},
                   p.geom, make_scalars(cfg)};
        launch_vec_any(cfg->m_group, bf16, refresh, scaled, VecLaunch{p.grid, 1, p.block_threads, split, extra}, a, st);
        if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
        if (split) {      // this matrix's part of the area is now in use until the pieces have been added up
            const PieceJob job{area->base, scale_grad, p.segments, p.geom.pieces_per_segment};
            const uint64_t used = ((uint64_t)p.geom.num_spans + 3) & ~(uint64_t)3;
            area->base += used;
            area->floats -= used < area->floats ? used : area->floats;
            static_cast<PieceJobQueue *>(area->jobs)->add(job);
        }
        return CAST_OK;
    }
    // odd shapes: refresh statistics and dL/dA first (they need the stored mask and the incoming weights), then the element pass
    if (stats) {
        const dim3 grid((unsigned)unit_grid), block(kBlockThreads);
        switch (cfg->m_group) {
        case 2: hipLaunchKernelGGL(refresh_stats_unit<2>, grid, block, 0, st, w, mask_bits, stats_initial, rows, cols, ld, cfg->n_keep, stats_partials); break;
        case 4: hipLaunchKernelGGL(refresh_stats_unit<4>, grid, block, 0, st, w, mask_bits, stats_initial, rows, cols, ld, cfg->n_keep, stats_partials); break;
        default: hipLaunchKernelGGL(refresh_stats_unit<8>, grid, block, 0, st, w, mask_bits, stats_initial, rows, cols, ld, cfg->n_keep, stats_partials); break;
        }
        if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
    }
    if (scaled && scale_grad) {
        cast_status rc = launch_scale_grad(w, grad, cfg->grad_dtype, rows, cols, ld, cfg->scale_segments, scale_grad, st);
        if (rc != CAST_OK) return rc;
    }
    UnitArgs a{w, grad, m, v, mask_bits, scale, rows, cols, ld, cfg->scale_segments, refresh ? 1 : 0, make_scalars(cfg),
               static_cast<uint16_t *>(x.compute_copy), x.copy_scale, mu16 ? mu_bf16_ld(cols, ld) : 0, v16 ? 1 : 0};
    const unsigned grid = (unsigned)unit_grid;
    switch (cfg->m_group) {
    case 2: launch_unit_dtype<2>(bf16, grid, a, st); break;
    case 4: launch_unit_dtype<4>(bf16, grid, a, st); break;
    default: launch_unit_dtype<8>(bf16, grid, a, st); break;
    }
    return launch_status();
}

// Up to kMaxFused matrices of one shape in one launch (no split plan): the ramp-up and ramp-down of a launch cost about 2.6 us, which is 4 % of the 70 us a
// 4096 x 4096 matrix takes.  `flavour`: the kernel flavour all of them need; each matrix its own buffers.
static cast_status launch_adams_step_fused(const cast_tensor *const *ts, int n, const SpanPlan &p, const cast_adams_config *cfg,
                                           int flavour, StatsArea *stats_area, hipStream_t st)
{
    SpanArgs a{{}, p.geom, make_scalars(cfg)};
    const bool refresh = cfg->refresh_mask != 0;
    a.geom.m_row_gap = mu_bf16_ld(ts[0]->cols, ts[0]->ld) - ts[0]->cols;
    for (int k = 0; k < n; ++k) {
        const cast_tensor &t = *ts[k];
        StatsPartial *partials = nullptr;
        if (can_count(flavour) && refresh && t.refresh_stats) {
            if (stats_area == nullptr || p.grid > stats_area->slots) return CAST_ERR_SHAPE;      // (not reachable through the API)
            partials = take_stats_slots(stats_area, p.grid, t.refresh_stats, t.initial_mask_bits);
        }
        a.set[k] = TensorPtrs{t.w, t.grad, t.m, t.v, t.mask_bits, t.scale, t.scale_grad, nullptr, partials,
                              partials ? t.initial_mask_bits : nullptr,
                              can_emit(flavour) ? static_cast<uint16_t *>(t.compute_copy) : nullptr, can_emit(flavour) ? t.copy_scale : nullptr};
    }
    launch_vec_any(cfg->m_group, cfg->grad_dtype == CAST_BF16, refresh, cfg->scale_segments > 0,
                   VecLaunch{p.grid, (unsigned)n, p.block_threads, false, flavour}, a, st);
    return launch_status();
}

// Workspace of a list call: room for the piece sums of every matrix with a split plan, then one
// slot per workgroup for every matrix that wants refresh statistics.
struct MultiLayout {
    uint64_t piece_floats;
    uint64_t stats_slots;
    size_t total() const { return (size_t)piece_floats * sizeof(float) + (size_t)stats_slots * sizeof(StatsPartial); }
};

static MultiLayout multi_layout(const cast_tensor *ts, int count, const cast_adams_config *cfg)
{
    const size_t n = (size_t)(count > 0 ? count : 0);
    MultiLayout l{0, 0};
    for (size_t i = 0; ts && cfg && i < n; ++i) {      // a slot per workgroup for every matrix that wants refresh statistics
        if (ts[i].rows <= 0 || ts[i].cols <= 0 || !ts[i].refresh_stats) continue;
        const bool may_split = cfg->scale_segments > 0 && ts[i].scale_grad;
        const SpanPlan p = plan_spans(ts[i].rows, ts[i].cols, ts[i].ld, cfg->scale_segments, may_split);
        const int64_t unit_grid = (ts[i].rows * ((ts[i].cols + 63) / 64) + kBlockThreads - 1) / kBlockThreads;
        l.stats_slots += p.vec ? p.grid : (uint64_t)unit_grid;
    }
    if (ts && cfg && cfg->scale_segments > 0)
        for (size_t i = 0; i < n; ++i) {
            if (ts[i].rows <= 0 || ts[i].cols <= 0 || !ts[i].scale_grad) continue;
            const SpanPlan p = plan_spans(ts[i].rows, ts[i].cols, ts[i].ld, cfg->scale_segments, true);
            if (p.geom.pieces_per_segment > 1) l.piece_floats += ((uint64_t)p.geom.num_spans + 3) & ~(uint64_t)3;
        }
    return l;
}

size_t multi_workspace_bytes(const cast_tensor *ts, int count, const cast_adams_config *cfg)
{
    return multi_layout(ts, count, cfg).total();
}

// A list of matrices that share one configuration: one launch per matrix, small matrices of one
// shape and one kernel flavour several to a launch, long row segments as split plans whose pieces'
// sums (and the refresh statistics' partial sums) go through the workspace and are added up by
// follow-up launches.  Kernel launches only: nothing is copied, cleared or allocated on the device.
// `taken`: `count` bytes of host scratch from the caller (which matrices have been stepped).
// With `tally` the call only counts the launches it would make (nothing is enqueued).
cast_status launch_adams_step_multi(const cast_tensor *ts, int count, const cast_adams_config *cfg,
                                    void *workspace, char *taken, hipStream_t st, MultiTally *tally)
{
    const bool dry = tally != nullptr;
    if (dry) *tally = MultiTally{0, 0};
    const bool want_stats = cfg->refresh_mask != 0;
    const MultiLayout layout = multi_layout(ts, count, cfg);
    PieceJobQueue jobs;
    // the workspace: piece sums, then statistics slots (a dry run has none)
    float *const piece_base = static_cast<float *>(workspace);
    StatsPartial *const stats_base = workspace ? reinterpret_cast<StatsPartial *>(piece_base + layout.piece_floats) : nullptr;
    PieceArea area{piece_base, layout.piece_floats, &jobs};
    for (int i = 0; i < count; ++i) taken[i] = 0;
    StatsJobQueue stats_jobs;
    StatsArea stats_area{stats_base, layout.stats_slots, &stats_jobs};
    // Small matrices of one shape and one kernel flavour share a launch (they need not follow each
    // other in the list: the matrices are independent).  A launch is kept below about 72 M entries: q, k, v, o of a
    // LLaMA2-7B layer go together, 16 of the 768 x 768 matrices of a 125M model; longer launches
    // lose to the drift between compute units what they gain on ramps.
    static const int fuse_limit = knob("CAST_FUSE", kMaxFused, 1, kMaxFused);            // matrices per launch (1 = never fuse)
    static const int64_t fuse_max_params = (int64_t)knob("CAST_FUSE_MAX_MPARAMS", 24, 1, 1024) << 20;
    static const int64_t fuse_launch_params = (int64_t)knob("CAST_FUSE_LAUNCH_MPARAMS", 72, 1, 1024) << 20;
    int dry_stats = 0;      // dry run: statistics jobs waiting for their launch
    auto stats_room = [&](int n) -> cast_status {      // room for n more statistics jobs before their launch is enqueued
        if (dry) {
            if (dry_stats + n > kMaxStatsJobs) {
                if (dry_stats > 0) ++tally->other_launches;
                dry_stats = 0;
            }
            return CAST_OK;
        }
        return stats_jobs.count + n > kMaxStatsJobs ? stats_jobs.flush(st) : CAST_OK;
    };
    auto flavour_of = [&](const cast_tensor &t) {      // of the kernels a matrix needs
        return step_flavour(cfg, t.compute_copy != nullptr, want_stats && t.refresh_stats != nullptr);
    };
    for (int i = 0; i < count; ++i) {
        if (taken[i]) continue;
        const cast_tensor &t = ts[i];
        const bool with_stats = want_stats && t.refresh_stats != nullptr;
        if (fuse_limit > 1 && t.rows > 0 && t.cols > 0 && t.rows * t.cols <= fuse_max_params) {
            int most = (int)(fuse_launch_params / (t.rows * t.cols));
            if (most > fuse_limit) most = fuse_limit;
            if (most > kMaxFused) most = kMaxFused;
            const int flavour = flavour_of(t);
            const cast_tensor *same[kMaxFused] = {&t};
            int where[kMaxFused] = {i};
            int n = 1, n_stats = with_stats ? 1 : 0;
            for (int j = i + 1; j < count && n < most; ++j)
                if (!taken[j] && flavour_of(ts[j]) == flavour && ts[j].rows == t.rows && ts[j].cols == t.cols && ts[j].ld == t.ld &&
                    (ts[j].scale_grad == nullptr) == (t.scale_grad == nullptr)) {
                    same[n] = &ts[j];
                    where[n] = j;
                    ++n;
                    if (want_stats && ts[j].refresh_stats) ++n_stats;
                }
            if (n > 1) {
                const SpanPlan p = plan_spans(t.rows, t.cols, t.ld, cfg->scale_segments, true);
                if (p.vec && p.geom.pieces_per_segment == 1) {
                    if (stats_room(n_stats) != CAST_OK) return CAST_ERR_LAUNCH;
                    if (dry) {
                        ++tally->step_launches;
                        dry_stats += n_stats;
                    } else {
                        const cast_status rc = launch_adams_step_fused(same, n, p, cfg, flavour, layout.stats_slots ? &stats_area : nullptr, st);
                        if (rc != CAST_OK) return rc;
                    }
                    for (int k = 0; k < n; ++k) taken[where[k]] = 1;
                    continue;
                }
            }
        }
        if (t.rows == 0 || t.cols == 0) continue;
        if (with_stats && stats_room(1) != CAST_OK) return CAST_ERR_LAUNCH;
        if (dry) {       // one step launch; odd shapes with dL/dA take a reduction launch first; split plans a sum at the end
            const SpanPlan p = plan_spans(t.rows, t.cols, t.ld, cfg->scale_segments, layout.piece_floats > 0 && t.scale_grad);
            ++tally->step_launches;
            if (!p.vec && t.scale && t.scale_grad) ++tally->other_launches;
            if (p.geom.pieces_per_segment > 1 && ++tally->split_matrices % kMaxPieceJobs == 1) ++tally->other_launches;
            if (with_stats) {
                if (!p.vec) ++tally->other_launches;
                ++dry_stats;
            }
            continue;
        }
        if (jobs.full() && jobs.flush(st) != CAST_OK) return CAST_ERR_LAUNCH;     // make room
        StepExtras x;
        x.compute_copy = t.compute_copy;
        x.copy_scale = t.copy_scale;
        x.initial_mask = t.initial_mask_bits;
        x.refresh_stats = t.refresh_stats;
        x.area = layout.piece_floats ? &area : nullptr;
        x.stats_area = layout.stats_slots ? &stats_area : nullptr;
        cast_status rc = launch_adams_step(t.w, t.grad, t.m, t.v, t.mask_bits, t.scale, t.scale_grad, t.rows, t.cols, t.ld, cfg, x, st);
        if (rc != CAST_OK) return rc;
    }
    if (dry) {
        if (dry_stats > 0) ++tally->other_launches;
        return CAST_OK;
    }
    if (jobs.flush(st) != CAST_OK) return CAST_ERR_LAUNCH;
    return stats_jobs.flush(st);
}

}  // namespace cast

// Built-in workspace of cast_adams_step_multi_noalloc: device memory the library itself holds, one
// copy per GPU from the moment the code object is loaded there until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; the device address it yields (a different
// one on every GPU) is what launches receive.  (No `used` attribute here: with it the compiler keeps
// the device symbol local and at default alignment, and the runtime cannot find it by name.)
static __device__ __align__(256) unsigned char scratch[CAST_NOALLOC_SCRATCH_BYTES];

namespace cast {

cast_status builtin_workspace(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static void *address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CAST_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(guard);
    if (address[dev] == nullptr) {      // first call with this device current
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return CAST_ERR_LAUNCH;
        }
        address[dev] = p;
    }
    *out = address[dev];
    return CAST_OK;
}

// ---- statistics of given masks over a list ------------------------------------------------------------------
static uint64_t mask_stats_slots(const cast_stats_matrix &t)
{
    if (t.rows <= 0 || t.cols <= 0) return 0;
    const RowsPlan p = plan_rows(t.rows, t.cols, t.ld, 4);
    if (p.vec) return p.grid;
    const int64_t words = t.rows * ((t.cols + 31) / 32);
    return (uint64_t)((words + kBlockThreads - 1) / kBlockThreads);
}

size_t mask_stats_list_workspace_bytes(const cast_stats_matrix *m, int count)
{
    uint64_t slots = 0;
    for (int i = 0; i < count; ++i) slots += mask_stats_slots(m[i]);
    return (size_t)slots * sizeof(StatsPartial);
}

cast_status launch_mask_stats_list(const cast_stats_matrix *m, int count, void *workspace, hipStream_t st)
{
    StatsPartial *next = static_cast<StatsPartial *>(workspace);
    StatsJobQueue jobs;
    std::vector<char> taken((size_t)count, 0);
    for (int i = 0; i < count; ++i) {
        if (taken[i]) continue;
        if (m[i].rows == 0 || m[i].cols == 0) {      // an empty matrix: zeros, from a job without slots
            if (jobs.full() && jobs.flush(st) != CAST_OK) return CAST_ERR_LAUNCH;
            jobs.add(StatsJob{next, 0, m[i].stats, 0});
            taken[i] = 1;
            continue;
        }
        int group[kMaxListed];
        const int n = take_group(m, count, taken, i, [](const cast_stats_matrix &x, const cast_stats_matrix &y) { return (x.other_bits == nullptr) == (y.other_bits == nullptr); }, group);
        const RowsPlan p = plan_rows(m[i].rows, m[i].cols, m[i].ld, 4);
        const uint64_t slots = mask_stats_slots(m[i]);
        MaskStatsArgs a{{}, p.geom};
        // room for the whole group's jobs first: a flush in between would add up slots nobody has written yet
        if (jobs.count + n > kMaxStatsJobs && jobs.flush(st) != CAST_OK) return CAST_ERR_LAUNCH;
        for (int k = 0; k < n; ++k) {
            const cast_stats_matrix &t = m[group[k]];
            jobs.add(StatsJob{next, (int64_t)slots, t.stats, 0});
            if (p.vec && (reinterpret_cast<uintptr_t>(t.w) & 15) == 0) {
                a.set[k] = MaskStatsSet{t.w, t.mask_bits, t.other_bits, next};
            } else {
                hipLaunchKernelGGL(mask_stats_words, dim3((unsigned)slots), dim3(kBlockThreads), 0, st, t.w, t.mask_bits, t.other_bits,
                                   t.rows, t.cols, t.ld, next);
                if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
                a.set[k] = MaskStatsSet{nullptr, nullptr, nullptr, nullptr};
            }
            next += slots;
        }
        if (p.vec) {      // the matrices of the group whose weights are 16-byte aligned, in one launch
            int dense = 0;
            for (int k = 0; k < n; ++k)
                if (a.set[k].w) a.set[dense++] = a.set[k];
            if (dense > 0) {
                if (p.same_row) hipLaunchKernelGGL(mask_stats_rows<true>, dim3(p.grid, (unsigned)dense), dim3(kBlockThreads), 0, st, a);
                else hipLaunchKernelGGL(mask_stats_rows<false>, dim3(p.grid, (unsigned)dense), dim3(kBlockThreads), 0, st, a);
                if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
            }
        }
    }
    return jobs.flush(st);
}

cast_status debug_div_by_uniform(const float *x, float y, float *out, int64_t n)
{
    const UniformDivisor d = make_divisor(y);
    for (int64_t i = 0; i < n; ++i) out[i] = div_by_uniform(x[i], d);
    return CAST_OK;
}

}  // namespace cast
