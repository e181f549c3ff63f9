// Mask selection alone (Eq. 6), weight scaling forward/fold (Eq. 12), the final hard prune
// with packing into values + index metadata, the mask-learning statistics of the appendix
// "Mask Learning", and a plain copy kernel used to calibrate bandwidth measurements.
//
// w may have a row stride ld >= cols; masks, packed values, metadata and scaled outputs are dense.
#include "cast_device.h"
#include "cast_internal.h"

#pragma clang fp contract(off)

namespace cast {

__device__ __forceinline__ void unpack4u(const vu4_t &x, float (&f)[4])
{
    f[0] = __uint_as_float(x.x); f[1] = __uint_as_float(x.y); f[2] = __uint_as_float(x.z); f[3] = __uint_as_float(x.w);
}

// These kernels do little arithmetic per byte, so what counts is memory requests in flight: a
// wavefront takes up to kBatch chunks of its span and asks for all of them before it works on the
// first.  The plan: dense matrices are cut into spans of kBatch chunks, one wavefront each; rows
// with a stride are cut into the fewest equal pieces of at most 16 * kBatch chunks that start on
// `align` columns, and as many wavefronts share a piece as it has kBatch chunks (a power of two).
constexpr int kBatch = 4;

SpanPlan plan_batched(int64_t rows, int64_t cols, int64_t ld, int align)
{
    int per_row = 0;
    if (ld != cols)
        for (int k = 1; k <= 64 && per_row == 0; ++k)
            if (cols % k == 0 && (cols / k) % align == 0 && cols / k <= (int64_t)kMaxBlockWaves * kBatch * kChunk) per_row = k;
    SpanPlan p = plan_spans(rows, cols, ld, per_row);
    if (!p.vec) return p;
    SpanGeom &g = p.geom;
    if (g.spans_per_row == 0) {
        g.span_len = (int64_t)kBatch * kChunk;
        g.num_spans = (g.total + g.span_len - 1) / g.span_len;
    }
    const int64_t chunks = (g.span_len + kChunk - 1) / kChunk;
    int P = 1;
    while ((int64_t)P * kBatch < chunks && P < kMaxBlockWaves) P *= 2;
    g.waves_per_span = P;
    const int block_waves = P > kBlockWaves ? P : kBlockWaves;
    p.block_threads = block_waves * kWave;
    const int64_t spans_per_block = block_waves / P;
    p.grid = (unsigned)((g.num_spans + spans_per_block - 1) / spans_per_block);
    return p;
}

// ---- Eq. 6 ----------------------------------------------------------------------------------
// Spans start on mask words; a wavefront's chunks of a span are sub, sub + P, sub + 2P, ...
template <int M>
__global__ __launch_bounds__(kMaxBlockThreads) void nm_select_vec(const float *w, uint32_t *mask,
                                                                  const SpanGeom geom, int n_keep)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int stride = geom.waves_per_span * kChunk;
    const SpanSlot slot = span_slot(geom, blockIdx.x, wave, blockDim.x / kWave);
    const int64_t span = slot.span;
    const int sub = slot.sub;
    const SpanOrigin o = span_origin(geom, span);
    const int len = o.len;
    const __amdgpu_buffer_rsrc_t rw = span_resource(w + o.state_begin, len * 4);
    const __amdgpu_buffer_rsrc_t rmask = span_resource(mask + (o.dense_begin >> 5), len / 8);
    for (int base = sub * kChunk; base < len; base += kBatch * stride) {
        vu4_t raw[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k)      // past the end of the span: zeros
            raw[k] = __builtin_amdgcn_raw_buffer_load_b128(rw, (base + k * stride + lane * kLaneElems) * 4, 0, kAuxLoad);
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            if (base + k * stride >= len) break;      // wave-uniform
            const int off = base + k * stride + lane * kLaneElems;
            float x[4];
            unpack4u(raw[k], x);
            const uint32_t nib = keep_nibble<M>(x, n_keep, lane);
            const uint32_t word = or_reduce_8lanes(nib << ((lane & 7) * 4));
            if ((lane & 7) == 0) __builtin_amdgcn_raw_buffer_store_b32(word, rmask, (off >> 5) * 4, 0, kAuxStore);
        }
    }
}

// M = 8 with a whole group per lane (8 consecutive entries, two 16-byte loads): the ranking needs no
// exchange between lanes, and the bytes of four adjacent lanes form a mask word.  Units of 512 entries
// per wavefront, two of them requested before the first is worked on.
__global__ __launch_bounds__(kMaxBlockThreads) void nm_select_8_vec(const float *w, uint32_t *mask, const SpanGeom geom, int n_keep)
{
    constexpr int kUnit = 2 * kChunk;
    constexpr int kUnitsInFlight = 2;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int stride = geom.waves_per_span * kUnit;
    const SpanSlot slot = span_slot(geom, blockIdx.x, wave, blockDim.x / kWave);
    const int sub = slot.sub;
    const SpanOrigin o = span_origin(geom, slot.span);
    const int len = o.len;
    const __amdgpu_buffer_rsrc_t rw = span_resource(w + o.state_begin, len * 4);
    const __amdgpu_buffer_rsrc_t rmask = span_resource(mask + (o.dense_begin >> 5), len / 8);
    for (int base = sub * kUnit; base < len; base += kUnitsInFlight * stride) {
        vu4_t lo[kUnitsInFlight], hi[kUnitsInFlight];
#pragma unroll
        for (int k = 0; k < kUnitsInFlight; ++k) {      // past the end of the span: zeros
            const int off = base + k * stride + lane * 8;
            lo[k] = __builtin_amdgcn_raw_buffer_load_b128(rw, off * 4, 0, kAuxLoad);
            hi[k] = __builtin_amdgcn_raw_buffer_load_b128(rw, off * 4 + 16, 0, kAuxLoad);
        }
#pragma unroll
        for (int k = 0; k < kUnitsInFlight; ++k) {
            if (base + k * stride >= len) break;      // wave-uniform
            const int off = base + k * stride + lane * 8;
            const float x[8] = {__uint_as_float(lo[k].x), __uint_as_float(lo[k].y), __uint_as_float(lo[k].z), __uint_as_float(lo[k].w),
                                __uint_as_float(hi[k].x), __uint_as_float(hi[k].y), __uint_as_float(hi[k].z), __uint_as_float(hi[k].w)};
            uint32_t word = keep_bits_group<8>(x, n_keep) << ((lane & 3) * 8);
            word |= dpp_u32<kDppQuadXor1>(word);
            word |= dpp_u32<kDppQuadXor2>(word);
            if ((lane & 3) == 0) __builtin_amdgcn_raw_buffer_store_b32(word, rmask, (off >> 5) * 4, 0, kAuxStore);
        }
    }
}

// Any shape with cols % M == 0: one thread per mask word (32 consecutive columns of a row).
template <int M>
__global__ __launch_bounds__(kBlockThreads) void nm_select_unit(const float *w, uint32_t *mask,
                                                                int64_t rows, int64_t cols, int64_t ld,
                                                                int n_keep)
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
        for (int j = 0; j < M; ++j) x[j] = w[r * ld + c + j];
        word |= keep_bits_group<M>(x, n_keep) << (unsigned)(c - cb);
    }
    mask[tid] = word;
}

cast_status launch_nm_select(const float *w, int64_t rows, int64_t cols, int64_t ld, int n_keep,
                             int m_group, uint32_t *mask_bits, hipStream_t st)
{
    if (rows == 0 || cols == 0) return CAST_OK;
    const SpanPlan p = plan_batched(rows, cols, ld, 32);
    if (p.vec) {
        switch (m_group) {
        case 2: hipLaunchKernelGGL(nm_select_vec<2>, dim3(p.grid), dim3(p.block_threads), 0, st, w, mask_bits, p.geom, n_keep); break;
        case 4: hipLaunchKernelGGL(nm_select_vec<4>, dim3(p.grid), dim3(p.block_threads), 0, st, w, mask_bits, p.geom, n_keep); break;
        default: hipLaunchKernelGGL(nm_select_8_vec, dim3(p.grid), dim3(p.block_threads), 0, st, w, mask_bits, p.geom, n_keep); break;
        }
    } else {
        const int64_t words = rows * ((cols + 31) / 32);
        const unsigned grid = (unsigned)((words + kBlockThreads - 1) / kBlockThreads);
        switch (m_group) {
        case 2: hipLaunchKernelGGL(nm_select_unit<2>, dim3(grid), dim3(kBlockThreads), 0, st, w, mask_bits, rows, cols, ld, n_keep); break;
        case 4: hipLaunchKernelGGL(nm_select_unit<4>, dim3(grid), dim3(kBlockThreads), 0, st, w, mask_bits, rows, cols, ld, n_keep); break;
        default: hipLaunchKernelGGL(nm_select_unit<8>, dim3(grid), dim3(kBlockThreads), 0, st, w, mask_bits, rows, cols, ld, n_keep); break;
        }
    }
    return launch_status();
}

// ---- Eq. 12 forward / fold --------------------------------------------------------------------
// One thread per W consecutive entries of a row (W = 4: 16-byte accesses; W = 1 for odd shapes).
template <bool BF16OUT, int W>
__global__ __launch_bounds__(kBlockThreads) void weight_scale_kernel(const float *w, const float *scale,
                                                                     void *out, int64_t rows, int64_t cols,
                                                                     int64_t ld, int64_t seg_len)
{
    const int64_t idx = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * W;     // dense index
    if (idx >= rows * cols) return;
    const int64_t r = idx / cols, c = idx - r * cols;
    const float A = scale[idx / seg_len];      // dense segment index = r * n + s
    float x[W];
    if constexpr (W == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(w + r * ld + c);
        x[0] = A * t.x; x[1] = A * t.y; x[2] = A * t.z; x[3] = A * t.w;
    } else {
        x[0] = A * w[r * ld + c];
    }
    if constexpr (BF16OUT) {
        uint16_t *o = static_cast<uint16_t *>(out) + idx;
        if constexpr (W == 4) {
            uint2 q;
            q.x = f32x2_to_bf16_rne(x[0], x[1]);
            q.y = f32x2_to_bf16_rne(x[2], x[3]);
            *reinterpret_cast<uint2 *>(o) = q;
        } else {
            o[0] = (uint16_t)f32_to_bf16_rne(x[0]);
        }
    } else {
        float *o = static_cast<float *>(out) + idx;
        if constexpr (W == 4) *reinterpret_cast<float4 *>(o) = make_float4(x[0], x[1], x[2], x[3]);
        else o[0] = x[0];
    }
}

cast_status launch_weight_scale(const float *w, const float *scale, int64_t rows, int64_t cols,
                                int64_t ld, int n_segments, void *out, int out_dtype, hipStream_t st)
{
    if (rows == 0 || cols == 0) return CAST_OK;
    const int64_t total = rows * cols, seg_len = cols / n_segments;
    const bool bf16 = out_dtype == CAST_BF16;
    if (seg_len % 4 == 0 && ld % 4 == 0) {
        const unsigned grid = (unsigned)((total / 4 + kBlockThreads - 1) / kBlockThreads);
        if (bf16) hipLaunchKernelGGL((weight_scale_kernel<true, 4>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, out, rows, cols, ld, seg_len);
        else hipLaunchKernelGGL((weight_scale_kernel<false, 4>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, out, rows, cols, ld, seg_len);
    } else {
        const unsigned grid = (unsigned)((total + kBlockThreads - 1) / kBlockThreads);
        if (bf16) hipLaunchKernelGGL((weight_scale_kernel<true, 1>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, out, rows, cols, ld, seg_len);
        else hipLaunchKernelGGL((weight_scale_kernel<false, 1>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, out, rows, cols, ld, seg_len);
    }
    return launch_status();
}

// ---- hard prune + fold + pack ---------------------------------------------------------------
// The half-density patterns 2:4 (the paper's) and 1:2 (4:8 has a kernel of its own below).  A lane holds 4
// consecutive entries and always ends up with exactly two kept values, which leave as one 8-byte (fp32) or
// 4-byte (bf16) store at values[off / 2]:
//   2:4  the lane is one group; the 4-bit index fields of 8 adjacent lanes form one metadata word;
//   1:2  the lane is two groups with one kept entry each; 16 lanes' bit pairs form one word.
template <int M, bool BF16OUT>
__global__ __launch_bounds__(kMaxBlockThreads) void project_compress_half_vec(
    const float *w, const float *scale, const uint32_t *mask, void *values, uint32_t *meta,
    const SpanGeom geom, uint32_t seg_len, FastDivU32 div_seg_len)
{
    static_assert(M == 4 || M == 2, "2:4 and 1:2 only");
    constexpr int kEntriesPerWord = M == 4 ? 32 : 64;      // columns one metadata word describes
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int stride = geom.waves_per_span * kChunk;
    const SpanSlot slot = span_slot(geom, blockIdx.x, wave, blockDim.x / kWave);
    const int64_t span = slot.span;
    const int sub = slot.sub;
    const SpanOrigin o = span_origin(geom, span);
    const int len = o.len;
    const __amdgpu_buffer_rsrc_t rw = span_resource(w + o.state_begin, len * 4);
    const __amdgpu_buffer_rsrc_t rmask = span_resource(mask ? mask + (o.dense_begin >> 5) : nullptr, mask ? len / 8 : 0);
    const __amdgpu_buffer_rsrc_t rmeta = span_resource(meta + o.dense_begin / kEntriesPerWord, len / kEntriesPerWord * 4);
    // half of the entries are kept: the values of a span start at dense_begin / 2
    const int vbytes = BF16OUT ? 2 : 4;
    const __amdgpu_buffer_rsrc_t rval = span_resource(static_cast<char *>(values) + (o.dense_begin >> 1) * vbytes, (len >> 1) * vbytes);
    // Eq. 12: the scale factor of an entry is that of its segment, dense index / seg_len.  One
    // 64-bit division per span, then 32-bit ones relative to the span's first segment.
    int64_t first_seg = 0;
    uint32_t first_seg_off = 0;
    if (scale) {
        first_seg = o.dense_begin / (int64_t)seg_len;
        first_seg_off = (uint32_t)(o.dense_begin - first_seg * (int64_t)seg_len);
    }
    for (int base = sub * kChunk; base < len; base += kBatch * stride) {
        vu4_t raw[kBatch];
        uint32_t bits[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {      // past the end of the span: zeros
            const int off = base + k * stride + lane * kLaneElems;
            raw[k] = __builtin_amdgcn_raw_buffer_load_b128(rw, off * 4, 0, kAuxLoad);
            bits[k] = mask ? __builtin_amdgcn_raw_buffer_load_b32(rmask, (off >> 5) * 4, 0, kAuxLoad) : 0u;
        }
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            if (base + k * stride >= len) break;      // wave-uniform
            const int off = base + k * stride + lane * kLaneElems;
            float x[4];
            unpack4u(raw[k], x);
            uint32_t nib;
            if (mask) nib = (bits[k] >> (off & 31)) & 0xFu;
            else nib = keep_nibble<M>(x, M / 2, lane);
            float A = 1.0f;
            if (scale && off < len) A = scale[first_seg + fast_div(first_seg_off + (uint32_t)off, div_seg_len)];
            float a, b;          // the two values this lane stores
            uint32_t word;       // the metadata word its run of lanes forms
            if constexpr (M == 4) {
                const uint32_t first = (uint32_t)__builtin_ctz(nib | 0x10u);      // positions of the two kept entries, ascending
                const uint32_t rest = nib & (nib - 1u);
                const uint32_t second = (uint32_t)__builtin_ctz(rest | 0x10u) & 3u;
                a = first == 0 ? x[0] : (first == 1 ? x[1] : x[2]);
                b = second == 1 ? x[1] : (second == 2 ? x[2] : x[3]);
                const uint32_t field = (first & 3u) | (second << 2);
                word = or_reduce_8lanes(field << ((lane & 7) * 4));
            } else if constexpr (M == 2) {
                const uint32_t ia = (nib & 1u) ? 0u : 1u, ib = (nib & 4u) ? 0u : 1u;   // which entry of each pair is kept
                a = ia ? x[1] : x[0];
                b = ib ? x[3] : x[2];
                word = or_reduce_16lanes((ia | (ib << 1)) << ((lane & 15) * 2));
            }
            if (scale) { a = A * a; b = A * b; }
            if constexpr (BF16OUT) {
                __builtin_amdgcn_raw_buffer_store_b32(f32x2_to_bf16_rne(a, b), rval, (off >> 1) * 2, 0, kAuxStore);
            } else {
                const vu2_t pair = {__float_as_uint(a), __float_as_uint(b)};
                __builtin_amdgcn_raw_buffer_store_b64(pair, rval, (off >> 1) * 4, 0, kAuxStore);
            }
            constexpr int kLanesPerWord = kEntriesPerWord / kLaneElems;
            if ((lane & (kLanesPerWord - 1)) == 0)
                __builtin_amdgcn_raw_buffer_store_b32(word, rmeta, (off / kEntriesPerWord) * 4, 0, kAuxStore);
        }
    }
}

// 4:8 with a whole group per lane: 8 consecutive entries (two 16-byte loads), so the four kept values
// are picked inside the lane (the k-th kept entry can only be one of entries k .. k + 4) and leave as
// one 16-byte (fp32) or 8-byte (bf16) store; two adjacent lanes' 12-bit index fields form a metadata
// word.  A wavefront takes units of 512 entries, two of them requested before the first is worked on.
// The exchange between lane pairs that the 4-entries-per-lane form needs made it ALU-bound.
template <bool BF16OUT>
__global__ __launch_bounds__(kMaxBlockThreads) void project_compress_4of8_vec(
    const float *w, const float *scale, const uint32_t *mask, void *values, uint32_t *meta,
    const SpanGeom geom, uint32_t seg_len, FastDivU32 div_seg_len)
{
    constexpr int kUnit = 2 * kChunk;          // entries a wavefront handles at a time: 8 per lane
    constexpr int kUnitsInFlight = 2;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int stride = geom.waves_per_span * kUnit;
    const SpanSlot slot = span_slot(geom, blockIdx.x, wave, blockDim.x / kWave);
    const int sub = slot.sub;
    const SpanOrigin o = span_origin(geom, slot.span);
    const int len = o.len;
    const __amdgpu_buffer_rsrc_t rw = span_resource(w + o.state_begin, len * 4);
    const __amdgpu_buffer_rsrc_t rmask = span_resource(mask ? mask + (o.dense_begin >> 5) : nullptr, mask ? len / 8 : 0);
    const __amdgpu_buffer_rsrc_t rmeta = span_resource(meta + o.dense_begin / 16, len / 16 * 4);
    const int vbytes = BF16OUT ? 2 : 4;
    const __amdgpu_buffer_rsrc_t rval = span_resource(static_cast<char *>(values) + (o.dense_begin >> 1) * vbytes, (len >> 1) * vbytes);
    int64_t first_seg = 0;
    uint32_t first_seg_off = 0;
    if (scale) {
        first_seg = o.dense_begin / (int64_t)seg_len;
        first_seg_off = (uint32_t)(o.dense_begin - first_seg * (int64_t)seg_len);
    }
    for (int base = sub * kUnit; base < len; base += kUnitsInFlight * stride) {
        vu4_t lo[kUnitsInFlight], hi[kUnitsInFlight];
        uint32_t bits[kUnitsInFlight];
#pragma unroll
        for (int k = 0; k < kUnitsInFlight; ++k) {      // past the end of the span: zeros
            const int off = base + k * stride + lane * 8;
            lo[k] = __builtin_amdgcn_raw_buffer_load_b128(rw, off * 4, 0, kAuxLoad);
            hi[k] = __builtin_amdgcn_raw_buffer_load_b128(rw, off * 4 + 16, 0, kAuxLoad);
            bits[k] = mask ? __builtin_amdgcn_raw_buffer_load_b32(rmask, (off >> 5) * 4, 0, kAuxLoad) : 0u;
        }
#pragma unroll
        for (int k = 0; k < kUnitsInFlight; ++k) {
            if (base + k * stride >= len) break;      // wave-uniform
            const int off = base + k * stride + lane * 8;
            const float x[8] = {__uint_as_float(lo[k].x), __uint_as_float(lo[k].y), __uint_as_float(lo[k].z), __uint_as_float(lo[k].w),
                                __uint_as_float(hi[k].x), __uint_as_float(hi[k].y), __uint_as_float(hi[k].z), __uint_as_float(hi[k].w)};
            const uint32_t kept = mask ? (bits[k] >> (off & 31)) & 0xFFu : keep_bits_group<8>(x, 4);
            // positions of the four kept entries, ascending (a given mask with fewer bits: the guard bit keeps them in range)
            const uint32_t r1 = kept & (kept - 1u), r2 = r1 & (r1 - 1u), r3 = r2 & (r2 - 1u);
            const uint32_t p0 = (uint32_t)__builtin_ctz(kept | 0x100u) & 7u, p1 = (uint32_t)__builtin_ctz(r1 | 0x100u) & 7u;
            const uint32_t p2 = (uint32_t)__builtin_ctz(r2 | 0x100u) & 7u, p3 = (uint32_t)__builtin_ctz(r3 | 0x100u) & 7u;
            float v0 = p0 == 0 ? x[0] : (p0 == 1 ? x[1] : (p0 == 2 ? x[2] : (p0 == 3 ? x[3] : x[4])));
            float v1 = p1 == 1 ? x[1] : (p1 == 2 ? x[2] : (p1 == 3 ? x[3] : (p1 == 4 ? x[4] : x[5])));
            float v2 = p2 == 2 ? x[2] : (p2 == 3 ? x[3] : (p2 == 4 ? x[4] : (p2 == 5 ? x[5] : x[6])));
            float v3 = p3 == 3 ? x[3] : (p3 == 4 ? x[4] : (p3 == 5 ? x[5] : (p3 == 6 ? x[6] : x[7])));
            if (scale) {
                float A = 1.0f;
                if (off < len) A = scale[first_seg + fast_div(first_seg_off + (uint32_t)off, div_seg_len)];
                v0 = A * v0; v1 = A * v1; v2 = A * v2; v3 = A * v3;
            }
            if constexpr (BF16OUT) {
                const vu2_t h = {f32x2_to_bf16_rne(v0, v1), f32x2_to_bf16_rne(v2, v3)};
                __builtin_amdgcn_raw_buffer_store_b64(h, rval, off, 0, kAuxStore);            // (off / 2) values of 2 bytes
            } else {
                const vu4_t q = {__float_as_uint(v0), __float_as_uint(v1), __float_as_uint(v2), __float_as_uint(v3)};
                __builtin_amdgcn_raw_buffer_store_b128(q, rval, off * 2, 0, kAuxStore);       // (off / 2) values of 4 bytes
            }
            const uint32_t field = p0 | (p1 << 3) | (p2 << 6) | (p3 << 9);
            const uint32_t word = field | (dpp_u32<kDppQuadXor1>(field) << 16);           // even lane: its group, then the odd lane's
            if ((lane & 1) == 0) __builtin_amdgcn_raw_buffer_store_b32(word, rmeta, (off >> 4) * 4, 0, kAuxStore);
        }
    }
}

// Any N:M and any shape with cols % M == 0: one thread per 64 consecutive columns of a row,
// which always holds a whole number of metadata words.
template <int M, bool BF16OUT>
__global__ __launch_bounds__(kBlockThreads) void project_compress_unit(
    const float *w, const float *scale, const uint32_t *mask, void *values, uint32_t *meta,
    int64_t rows, int64_t cols, int64_t ld, int n_keep, int n_segments)
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
        for (int j = 0; j < M; ++j) x[j] = w[r * ld + c + j];
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
                             int64_t cols, int64_t ld, int n_keep, int n_segments)
{
    if (bf16) hipLaunchKernelGGL((project_compress_unit<M, true>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, mask, values, meta, rows, cols, ld, n_keep, n_segments);
    else hipLaunchKernelGGL((project_compress_unit<M, false>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, mask, values, meta, rows, cols, ld, n_keep, n_segments);
}

cast_status launch_project_compress(const float *w, const float *scale, int n_segments,
                                    const uint32_t *mask_bits, int64_t rows, int64_t cols,
                                    int64_t ld, int n_keep, int m_group, void *values,
                                    int value_dtype, uint32_t *meta, hipStream_t st)
{
    if (rows == 0 || cols == 0) return CAST_OK;
    const bool bf16 = value_dtype == CAST_BF16;
    const int64_t seg_len64 = scale ? cols / n_segments : cols;
    // the vector kernel: half-density patterns, spans and rows that are whole metadata words
    // (32 columns for 2:4, 16 for 4:8, 64 for 1:2), scale segments that are whole groups
    const int word_cols = m_group == 4 ? 32 : (m_group == 8 ? 16 : 64);
    const SpanPlan p = plan_batched(rows, cols, ld, word_cols < 32 ? 32 : word_cols);
    if (2 * n_keep == m_group && p.vec && seg_len64 % m_group == 0 && cols % word_cols == 0 && p.geom.span_len % word_cols == 0 &&
        seg_len64 < ((int64_t)1 << 31)) {
        const uint32_t seg_len = (uint32_t)seg_len64;
        const FastDivU32 div_seg_len = make_fast_div(seg_len);
        const dim3 grid(p.grid), block(p.block_threads);
        switch (m_group) {
        case 4:
            if (bf16) hipLaunchKernelGGL((project_compress_half_vec<4, true>), grid, block, 0, st, w, scale, mask_bits, values, meta, p.geom, seg_len, div_seg_len);
            else hipLaunchKernelGGL((project_compress_half_vec<4, false>), grid, block, 0, st, w, scale, mask_bits, values, meta, p.geom, seg_len, div_seg_len);
            break;
        case 8:
            if (bf16) hipLaunchKernelGGL(project_compress_4of8_vec<true>, grid, block, 0, st, w, scale, mask_bits, values, meta, p.geom, seg_len, div_seg_len);
            else hipLaunchKernelGGL(project_compress_4of8_vec<false>, grid, block, 0, st, w, scale, mask_bits, values, meta, p.geom, seg_len, div_seg_len);
            break;
        default:
            if (bf16) hipLaunchKernelGGL((project_compress_half_vec<2, true>), grid, block, 0, st, w, scale, mask_bits, values, meta, p.geom, seg_len, div_seg_len);
            else hipLaunchKernelGGL((project_compress_half_vec<2, false>), grid, block, 0, st, w, scale, mask_bits, values, meta, p.geom, seg_len, div_seg_len);
            break;
        }
        return launch_status();
    }
    const int64_t units = rows * ((cols + 63) / 64);
    const unsigned grid = (unsigned)((units + kBlockThreads - 1) / kBlockThreads);
    switch (m_group) {
    case 2: launch_pack_unit<2>(bf16, grid, st, w, scale, mask_bits, values, meta, rows, cols, ld, n_keep, n_segments); break;
    case 4: launch_pack_unit<4>(bf16, grid, st, w, scale, mask_bits, values, meta, rows, cols, ld, n_keep, n_segments); break;
    default: launch_pack_unit<8>(bf16, grid, st, w, scale, mask_bits, values, meta, rows, cols, ld, n_keep, n_segments); break;
    }
    return launch_status();
}

// ---- appendix "Mask Learning" ---------------------------------------------------------------
// One thread per mask word; exact integer flip count, L1 sums in double; one atomic of each
// kind per workgroup.
__global__ __launch_bounds__(kBlockThreads) void mask_stats_kernel(
    const float *w, const uint32_t *mask, const uint32_t *other, int64_t rows, int64_t cols,
    int64_t ld, unsigned long long *flips, double *l1)
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
            const double mag = fabs((double)w[r * ld + c]);
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

// The same for rows that are whole mask words (cols % 32 == 0) with 16-byte aligned row starts:
// 8 adjacent lanes share a mask word and read its 32 weights as 8 consecutive 16-byte loads, so a
// wavefront reads 1 KiB of contiguous weights per step (4.25 bytes per parameter in all, one
// pass).  Atomics on one address retire at about 60 million a second, so the matrix is walked by
// few, large workgroups (256 of 1024 threads, one per compute unit, four loads in flight per lane):
// with 4096 workgroups the three atomics per workgroup took five times as long as the reading.
__global__ __launch_bounds__(kMaxBlockThreads) void mask_stats_vec(
    const float *w, const uint32_t *mask, const uint32_t *other, int64_t n_words, FastDivU32 div_words_per_row,
    uint32_t words_per_row, int64_t ld, unsigned long long *flips, double *l1)
{
    __shared__ double sh_kept[kMaxBlockWaves], sh_total[kMaxBlockWaves];
    __shared__ unsigned long long sh_flips[kMaxBlockWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int part = lane & 7;                       // which 4 of the word's 32 entries
    double kept = 0.0, total = 0.0;
    unsigned long long nf = 0;
    const int64_t words_per_round = (int64_t)gridDim.x * (kMaxBlockThreads / 8);
    constexpr int kInFlight = 4;                     // independent loads per lane and loop iteration
    for (int64_t t0 = ((int64_t)blockIdx.x * kMaxBlockThreads + threadIdx.x) / 8; t0 < n_words; t0 += kInFlight * words_per_round) {
        uint32_t word[kInFlight], diff[kInFlight];
        vf4_t x[kInFlight];
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
            const int64_t t = t0 + k * words_per_round;
            word[k] = 0;
            diff[k] = 0;
            x[k] = vf4_t{0.0f, 0.0f, 0.0f, 0.0f};
            if (t < n_words) {
                const uint32_t r = fast_div((uint32_t)t, div_words_per_row);
                const uint32_t word_in_row = (uint32_t)t - r * words_per_row;
                word[k] = __builtin_nontemporal_load(mask + t);
                if (other) diff[k] = __builtin_nontemporal_load(other + t);
                x[k] = __builtin_nontemporal_load(
                    reinterpret_cast<const vf4_t *>(w + (int64_t)r * ld + (int64_t)word_in_row * 32 + part * 4));
            }
        }
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
            if (other && part == 0) nf += (unsigned long long)__popc(word[k] ^ diff[k]);     // past the end: 0 ^ 0
            const uint32_t nib = (word[k] >> (part * 4)) & 0xFu;
            const float xs[4] = {x[k].x, x[k].y, x[k].z, x[k].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double mag = (double)__builtin_fabsf(xs[j]);
                total += mag;
                kept += ((nib >> j) & 1u) ? mag : 0.0;
            }
        }
    }
    for (int d = 1; d < kWave; d <<= 1) {
        kept += __shfl_xor(kept, d, kWave);
        total += __shfl_xor(total, d, kWave);
        nf += __shfl_xor(nf, d, kWave);
    }
    if (lane == 0) { sh_kept[wave] = kept; sh_total[wave] = total; sh_flips[wave] = nf; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < kMaxBlockWaves; ++k) { kept += sh_kept[k]; total += sh_total[k]; nf += sh_flips[k]; }
        atomicAdd(&l1[0], kept);
        atomicAdd(&l1[1], total);
        if (other) atomicAdd(flips, nf);
    }
}

cast_status launch_mask_stats(const float *w, const uint32_t *mask_bits, const uint32_t *other_bits,
                              int64_t rows, int64_t cols, int64_t ld, unsigned long long *flips,
                              double *l1, hipStream_t st)
{
    if (rows == 0 || cols == 0) return CAST_OK;
    if (cols % 32 == 0 && ld % 4 == 0 && (reinterpret_cast<uintptr_t>(w) & 15) == 0 && rows * (cols / 32) < ((int64_t)1 << 31)) {
        const int64_t n_words = rows * (cols / 32);
        int64_t grid = (n_words * 8 + kMaxBlockThreads - 1) / kMaxBlockThreads;
        if (grid > 256) grid = 256;
        hipLaunchKernelGGL(mask_stats_vec, dim3((unsigned)grid), dim3(kMaxBlockThreads), 0, st, w, mask_bits, other_bits, n_words,
                           make_fast_div((uint32_t)(cols / 32)), (uint32_t)(cols / 32), ld, flips, l1);
        return launch_status();
    }
    const int64_t n_words = rows * ((cols + 31) / 32);
    int64_t grid = (n_words + kBlockThreads - 1) / kBlockThreads;
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(mask_stats_kernel, dim3((unsigned)grid), dim3(kBlockThreads), 0, st, w, mask_bits, other_bits, rows, cols, ld, flips, l1);
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
