// Mask selection alone (Eq. 6), weight scaling forward/fold (Eq. 12), the final hard prune
// with packing into values + index metadata, the mask-learning statistics of the appendix
// "Mask Learning", and a plain copy kernel used to calibrate bandwidth measurements.
#include "cast_device.h"
#include "cast_internal.h"

#pragma clang fp contract(off)

namespace cast {

__device__ __forceinline__ void ld4(const float *p, int64_t idx, float (&x)[4])
{
    const float4 t = *reinterpret_cast<const float4 *>(p + idx);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
}

// ---- Eq. 6 ----------------------------------------------------------------------------------
// Flat walk, 256 entries per wavefront per chunk; requires cols % 32 == 0 so that flat mask
// words coincide with the row-padded layout.
template <int M>
__global__ __launch_bounds__(kBlockThreads) void nm_select_vec(const float *w, uint32_t *mask,
                                                               int64_t total, int64_t span_len,
                                                               int n_keep)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t span = (int64_t)blockIdx.x * kBlockWaves + threadIdx.x / kWave;
    const int64_t begin = span * span_len;
    int64_t len = total - begin;
    if (len > span_len) len = span_len;
    for (int64_t base = 0; base < len; base += kChunk) {   // len <= 0 for spans past the end
        const int64_t off = base + lane * kLaneElems;
        const bool act = off < len;
        float x[4] = {0, 0, 0, 0};
        if (act) ld4(w, begin + off, x);
        const uint32_t nib = keep_nibble<M>(x, n_keep, lane);
        const uint32_t word = or_reduce_8lanes(nib << ((lane & 7) * 4));
        if (act && (lane & 7) == 0) mask[(begin + off) >> 5] = word;
    }
}

// Any shape with cols % M == 0: one thread per mask word (32 consecutive columns of a row).
template <int M>
__global__ __launch_bounds__(kBlockThreads) void nm_select_unit(const float *w, uint32_t *mask,
                                                                int64_t rows, int64_t cols, int n_keep)
{
    const int64_t words_per_row = (cols + 31) / 32;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= rows * words_per_row) return;
    const int64_t r = tid / words_per_row, cb = (tid % words_per_row) * 32;
    const int64_t ce = (cb + 32 < cols) ? cb + 32 : cols;
    uint32_t word = 0;
    for (int64_t c = cb; c < ce; c += M) {
        float x[M];
#pragma unroll
        for (int j = 0; j < M; ++j) x[j] = w[r * cols + c + j];
        word |= keep_bits_group<M>(x, n_keep) << (unsigned)(c - cb);
    }
    mask[tid] = word;
}

cast_status launch_nm_select(const float *w, int64_t rows, int64_t cols, int n_keep, int m_group,
                             uint32_t *mask_bits, hipStream_t st)
{
    if (rows == 0 || cols == 0) return CAST_OK;
    SpanPlan p = plan_spans(rows, cols, 0);
    p.span_len = 2 * kChunk;
    p.num_spans = (p.total + p.span_len - 1) / p.span_len;
    if (p.vec) {
        const unsigned grid = (unsigned)((p.num_spans + kBlockWaves - 1) / kBlockWaves);
        switch (m_group) {
        case 2: hipLaunchKernelGGL(nm_select_vec<2>, dim3(grid), dim3(kBlockThreads), 0, st, w, mask_bits, p.total, p.span_len, n_keep); break;
        case 4: hipLaunchKernelGGL(nm_select_vec<4>, dim3(grid), dim3(kBlockThreads), 0, st, w, mask_bits, p.total, p.span_len, n_keep); break;
        default: hipLaunchKernelGGL(nm_select_vec<8>, dim3(grid), dim3(kBlockThreads), 0, st, w, mask_bits, p.total, p.span_len, n_keep); break;
        }
    } else {
        const int64_t words = rows * ((cols + 31) / 32);
        const unsigned grid = (unsigned)((words + kBlockThreads - 1) / kBlockThreads);
        switch (m_group) {
        case 2: hipLaunchKernelGGL(nm_select_unit<2>, dim3(grid), dim3(kBlockThreads), 0, st, w, mask_bits, rows, cols, n_keep); break;
        case 4: hipLaunchKernelGGL(nm_select_unit<4>, dim3(grid), dim3(kBlockThreads), 0, st, w, mask_bits, rows, cols, n_keep); break;
        default: hipLaunchKernelGGL(nm_select_unit<8>, dim3(grid), dim3(kBlockThreads), 0, st, w, mask_bits, rows, cols, n_keep); break;
        }
    }
    return launch_status();
}

// ---- Eq. 12 forward / fold --------------------------------------------------------------------
template <bool BF16OUT>
__global__ __launch_bounds__(kBlockThreads) void weight_scale_vec(const float *w, const float *scale,
                                                                  void *out, int64_t total,
                                                                  int64_t seg_len)
{
    // one thread per 4 consecutive entries; a segment boundary never falls inside them
    const int64_t idx = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (idx >= total) return;
    float x[4];
    ld4(w, idx, x);
    const float A = scale[idx / seg_len];   // flat segment index = r * n + s
#pragma unroll
    for (int j = 0; j < 4; ++j) x[j] = A * x[j];
    if constexpr (BF16OUT) {
        uint2 o;
        o.x = f32_to_bf16_rne(x[0]) | (f32_to_bf16_rne(x[1]) << 16);
        o.y = f32_to_bf16_rne(x[2]) | (f32_to_bf16_rne(x[3]) << 16);
        *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(out) + idx) = o;
    } else {
        *reinterpret_cast<float4 *>(static_cast<float *>(out) + idx) = make_float4(x[0], x[1], x[2], x[3]);
    }
}

template <bool BF16OUT>
__global__ __launch_bounds__(kBlockThreads) void weight_scale_scalar(const float *w, const float *scale,
                                                                     void *out, int64_t total,
                                                                     int64_t seg_len)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const float y = scale[idx / seg_len] * w[idx];
    if constexpr (BF16OUT) static_cast<uint16_t *>(out)[idx] = (uint16_t)f32_to_bf16_rne(y);
    else static_cast<float *>(out)[idx] = y;
}

cast_status launch_weight_scale(const float *w, const float *scale, int64_t rows, int64_t cols,
                                int n_segments, void *out, int out_dtype, hipStream_t st)
{
    if (rows == 0 || cols == 0) return CAST_OK;
    const int64_t total = rows * cols, seg_len = cols / n_segments;
    const bool bf16 = out_dtype == CAST_BF16;
    if (seg_len % 4 == 0) {
        const unsigned grid = (unsigned)((total / 4 + kBlockThreads - 1) / kBlockThreads);
        if (bf16) hipLaunchKernelGGL(weight_scale_vec<true>, dim3(grid), dim3(kBlockThreads), 0, st, w, scale, out, total, seg_len);
        else hipLaunchKernelGGL(weight_scale_vec<false>, dim3(grid), dim3(kBlockThreads), 0, st, w, scale, out, total, seg_len);
    } else {
        const unsigned grid = (unsigned)((total + kBlockThreads - 1) / kBlockThreads);
        if (bf16) hipLaunchKernelGGL(weight_scale_scalar<true>, dim3(grid), dim3(kBlockThreads), 0, st, w, scale, out, total, seg_len);
        else hipLaunchKernelGGL(weight_scale_scalar<false>, dim3(grid), dim3(kBlockThreads), 0, st, w, scale, out, total, seg_len);
    }
    return launch_status();
}

// ---- hard prune + fold + pack ---------------------------------------------------------------
// 2:4, the paper's pattern: a lane holds one group; its two kept values leave as one 8-byte
// (fp32) or 4-byte (bf16) store and the 4-bit index fields of 8 adjacent lanes form one
// metadata word, exactly like the mask words.
template <bool BF16OUT>
__global__ __launch_bounds__(kBlockThreads) void project_compress_2of4_vec(
    const float *w, const float *scale, const uint32_t *mask, void *values, uint32_t *meta,
    int64_t total, int64_t span_len, int64_t seg_len)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t span = (int64_t)blockIdx.x * kBlockWaves + threadIdx.x / kWave;
    const int64_t begin = span * span_len;
    int64_t len = total - begin;
    if (len > span_len) len = span_len;
    for (int64_t base = 0; base < len; base += kChunk) {
        const int64_t off = base + lane * kLaneElems;
        const bool act = off < len;
        const int64_t idx = begin + off;
        float x[4] = {0, 0, 0, 0};
        uint32_t nib = 0x3u;
        float A = 1.0f;
        if (act) {
            ld4(w, idx, x);
            if (mask) nib = (mask[idx >> 5] >> (unsigned)(idx & 31)) & 0xFu;
            if (scale) A = scale[idx / seg_len];
        }
        if (!mask) nib = keep_nibble<4>(x, 2, lane);
        // positions of the two kept entries, ascending
        const uint32_t first = (uint32_t)__builtin_ctz(nib | 0x10u);
        const uint32_t rest = nib & (nib - 1u);
        const uint32_t second = (uint32_t)__builtin_ctz(rest | 0x10u) & 3u;
        float a = first == 0 ? x[0] : (first == 1 ? x[1] : x[2]);
        float b = second == 1 ? x[1] : (second == 2 ? x[2] : x[3]);
        if (scale) { a = A * a; b = A * b; }
        const uint32_t field = (first & 3u) | (second << 2);
        const uint32_t word = or_reduce_8lanes(field << ((lane & 7) * 4));
        if (act) {
            const int64_t o = (idx >> 2) * 2;   // two values per group
            if constexpr (BF16OUT)
                static_cast<uint32_t *>(values)[o >> 1] = f32_to_bf16_rne(a) | (f32_to_bf16_rne(b) << 16);
            else
                *reinterpret_cast<float2 *>(static_cast<float *>(values) + o) = make_float2(a, b);
            if ((lane & 7) == 0) meta[idx >> 5] = word;
        }
    }
}

// Any N:M and any shape with cols % M == 0: one thread per 64 consecutive columns of a row,
// which always holds a whole number of metadata words.
template <int M, bool BF16OUT>
__global__ __launch_bounds__(kBlockThreads) void project_compress_unit(
    const float *w, const float *scale, const uint32_t *mask, void *values, uint32_t *meta,
    int64_t rows, int64_t cols, int n_keep, int n_segments)
{
    constexpr int B = M == 2 ? 1 : (M == 4 ? 2 : 3);
    int f = 1;
    while (f < n_keep * B) f <<= 1;
    const int groups_per_word = 32 / f;
    const int64_t units_per_row = (cols + 63) / 64;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= rows * units_per_row) return;
    const int64_t r = tid / units_per_row, c0 = (tid % units_per_row) * 64;
    const int64_t ce = (c0 + 64 < cols) ? c0 + 64 : cols;
    const int64_t groups = cols / M;
    const int64_t mask_wpr = (cols + 31) / 32;
    const int64_t meta_wpr = (groups + groups_per_word - 1) / groups_per_word;
    const int64_t seg_len = n_segments > 0 ? cols / n_segments : cols;
    uint32_t word = 0;
    for (int64_t c = c0; c < ce; c += M) {
        const int64_t gi = c / M;
        float x[M];
#pragma unroll
        for (int j = 0; j < M; ++j) x[j] = w[r * cols + c + j];
        uint32_t bits;
        if (mask) bits = (mask[r * mask_wpr + c / 32] >> (unsigned)(c % 32)) & ((1u << M) - 1u);
        else bits = keep_bits_group<M>(x, n_keep);
        const float A = scale ? scale[r * n_segments + c / seg_len] : 1.0f;
        uint32_t field = 0;
        int q = 0;
#pragma unroll
        for (int j = 0; j < M; ++j) {
            if (((bits >> j) & 1u) && q < n_keep) {
                float y = x[j];
                if (scale) y = A * y;
                const int64_t o = (r * groups + gi) * n_keep + q;
                if constexpr (BF16OUT) static_cast<uint16_t *>(values)[o] = (uint16_t)f32_to_bf16_rne(y);
                else static_cast<float *>(values)[o] = y;
                field |= (uint32_t)j << (q * B);
                ++q;
            }
        }
        const int slot = (int)(gi % groups_per_word);
        word |= field << (slot * f);
        if (slot == groups_per_word - 1 || c + M >= ce) {
            meta[r * meta_wpr + gi / groups_per_word] = word;
            word = 0;
        }
    }
}

template <int M>
static void launch_pack_unit(bool bf16, unsigned grid, hipStream_t st, const float *w, const float *scale,
                             const uint32_t *mask, void *values, uint32_t *meta, int64_t rows,
                             int64_t cols, int n_keep, int n_segments)
{
    if (bf16) hipLaunchKernelGGL((project_compress_unit<M, true>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, mask, values, meta, rows, cols, n_keep, n_segments);
    else hipLaunchKernelGGL((project_compress_unit<M, false>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, mask, values, meta, rows, cols, n_keep, n_segments);
}

cast_status launch_project_compress(const float *w, const float *scale, int n_segments,
                                    const uint32_t *mask_bits, int64_t rows, int64_t cols,
                                    int n_keep, int m_group, void *values, int value_dtype,
                                    uint32_t *meta, hipStream_t st)
{
    if (rows == 0 || cols == 0) return CAST_OK;
    const bool bf16 = value_dtype == CAST_BF16;
    const int64_t seg_len = scale ? cols / n_segments : cols;
    if (n_keep == 2 && m_group == 4 && cols % 32 == 0 && seg_len % 4 == 0) {
        SpanPlan p = plan_spans(rows, cols, 0);
        p.span_len = 2 * kChunk;
        p.num_spans = (p.total + p.span_len - 1) / p.span_len;
        const unsigned grid = (unsigned)((p.num_spans + kBlockWaves - 1) / kBlockWaves);
        if (bf16) hipLaunchKernelGGL(project_compress_2of4_vec<true>, dim3(grid), dim3(kBlockThreads), 0, st, w, scale, mask_bits, values, meta, p.total, p.span_len, seg_len);
        else hipLaunchKernelGGL(project_compress_2of4_vec<false>, dim3(grid), dim3(kBlockThreads), 0, st, w, scale, mask_bits, values, meta, p.total, p.span_len, seg_len);
        return launch_status();
    }
    const int64_t units = rows * ((cols + 63) / 64);
    const unsigned grid = (unsigned)((units + kBlockThreads - 1) / kBlockThreads);
    switch (m_group) {
    case 2: launch_pack_unit<2>(bf16, grid, st, w, scale, mask_bits, values, meta, rows, cols, n_keep, n_segments); break;
    case 4: launch_pack_unit<4>(bf16, grid, st, w, scale, mask_bits, values, meta, rows, cols, n_keep, n_segments); break;
    default: launch_pack_unit<8>(bf16, grid, st, w, scale, mask_bits, values, meta, rows, cols, n_keep, n_segments); break;
    }
    return launch_status();
}

// ---- appendix "Mask Learning" ---------------------------------------------------------------
// One thread per mask word; exact integer flip count, L1 sums in double; one atomic of each
// kind per workgroup.
__global__ __launch_bounds__(kBlockThreads) void mask_stats_kernel(
    const float *w, const uint32_t *mask, const uint32_t *other, int64_t rows, int64_t cols,
    unsigned long long *flips, double *l1)
{
    __shared__ double sh_kept[kBlockWaves], sh_total[kBlockWaves];
    __shared__ unsigned long long sh_flips[kBlockWaves];
    const int64_t words_per_row = (cols + 31) / 32;
    const int64_t n_words = rows * words_per_row;
    double kept = 0.0, total = 0.0;
    unsigned long long nf = 0;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n_words;
         t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = t / words_per_row, cb = (t % words_per_row) * 32;
        const int64_t ce = (cb + 32 < cols) ? cb + 32 : cols;
        const uint32_t word = mask[t];
        if (other) nf += (unsigned long long)__popc(word ^ other[t]);
        for (int64_t c = cb; c < ce; ++c) {
            const double mag = fabs((double)w[r * cols + c]);
            total += mag;
            if ((word >> (unsigned)(c - cb)) & 1u) kept += mag;
        }
    }
    for (int d = 1; d < kWave; d <<= 1) {
        kept += __shfl_xor(kept, d, kWave);
        total += __shfl_xor(total, d, kWave);
        nf += __shfl_xor(nf, d, kWave);
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) { sh_kept[wave] = kept; sh_total[wave] = total; sh_flips[wave] = nf; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < kBlockWaves; ++k) { kept += sh_kept[k]; total += sh_total[k]; nf += sh_flips[k]; }
        atomicAdd(&l1[0], kept);
        atomicAdd(&l1[1], total);
        if (other) atomicAdd(flips, nf);
    }
}

cast_status launch_mask_stats(const float *w, const uint32_t *mask_bits, const uint32_t *other_bits,
                              int64_t rows, int64_t cols, unsigned long long *flips, double *l1,
                              hipStream_t st)
{
    if (rows == 0 || cols == 0) return CAST_OK;
    const int64_t n_words = rows * ((cols + 31) / 32);
    int64_t grid = (n_words + kBlockThreads - 1) / kBlockThreads;
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(mask_stats_kernel, dim3((unsigned)grid), dim3(kBlockThreads), 0, st, w, mask_bits, other_bits, rows, cols, flips, l1);
    return launch_status();
}

// ---- measurement aid ------------------------------------------------------------------------
__global__ __launch_bounds__(kBlockThreads) void copy_probe_kernel(float4 *dst, const float4 *src, int64_t n16)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

cast_status launch_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t st)
{
    if (bytes == 0) return CAST_OK;
    const int64_t n16 = (int64_t)(bytes / 16);
    const unsigned grid = (unsigned)((n16 + kBlockThreads - 1) / kBlockThreads);
    hipLaunchKernelGGL(copy_probe_kernel, dim3(grid), dim3(kBlockThreads), 0, st, static_cast<float4 *>(dst), static_cast<const float4 *>(src), n16);
    return launch_status();
}

}  // namespace cast
