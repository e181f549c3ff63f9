// Mask selection alone (Eq. 6), weight scaling forward/fold (Eq. 12), the final hard prune
// with packing into values + index metadata, the mask-learning statistics of the appendix
// "Mask Learning", and a plain copy kernel used to calibrate bandwidth measurements.
//
// w may have a row stride ld >= cols; masks, packed values, metadata and scaled outputs are dense.
#include <vector>

#include "cast_device.h"
#include "cast_internal.h"

#pragma clang fp contract(off)

namespace cast {

// Cache policies of this file's kernels (0 = default, 2 = non-temporal), as measured over the
// LLaMA2-7B-shaped set with every matrix writing to buffers of its own: weights and masks, read once,
// and the outputs that every lane writes (packed values, scaled weights: whole cache lines per
// wavefront) with the non-temporal hint (default policy: pack and Eq. 12 into bf16 10 % slower; it only
// looks faster when all matrices write into one small buffer that stays in the last-level cache).
#ifndef CAST_AUX_ONCE_LOAD
#define CAST_AUX_ONCE_LOAD 2
#endif
#ifndef CAST_AUX_FULL_STORE
#define CAST_AUX_FULL_STORE 2
#endif
constexpr int kAuxOnceLoad = CAST_AUX_ONCE_LOAD;      // weights (and masks) read once
constexpr int kAuxFullStore = CAST_AUX_FULL_STORE;    // packed values, scaled weights: every lane stores, whole lines

template <typename T>
__device__ __forceinline__ T load_once(const T *p)
{
    if constexpr ((kAuxOnceLoad & 2) != 0) return __builtin_nontemporal_load(p);
    else return *p;
}

template <typename T>
__device__ __forceinline__ void store_full(T *p, const T &x)
{
    if constexpr ((kAuxFullStore & 2) != 0) __builtin_nontemporal_store(x, p);
    else *p = x;
}

// ---- how these kernels cover a matrix ----------------------------------------------------------
// They do little arithmetic per byte and read every weight once, so what counts is plain, wide,
// independent loads: a thread owns kLoads pieces of E consecutive entries (E = 4: one 16-byte load;
// E = 8 for the 4:8 pack: two), a wavefront kLoads consecutive chunks of 64 * E entries of a row, a
// workgroup of 256 threads 4 * kLoads consecutive chunks (see RowsGeom), and all loads of a thread
// are requested before the first is used.  Rows are whole mask words (cols % 32 == 0), so every run
// of 8 lanes (E = 4) holds one mask word.  blockIdx.y picks one of up to kMaxListed matrices of equal
// shape whose buffers travel in the kernel arguments (list calls).
// Measured over the LLaMA2-7B-shaped set (weights row-interleaved with the moments): two loads per
// thread beat one (-15 %), three (-9 %) and four (-2 %); mask and metadata words, which fill a cache
// line only together with their neighbours', are stored with the default policy so that the L2 merges
// them (non-temporal: 7 % slower).  A form in which wavefronts walked spans through buffer resources
// with four chunks in flight, like the step kernels, ran at 5.2 TB/s where this one runs at 6.3.
RowsPlan plan_rows(int64_t rows, int64_t cols, int64_t ld, int lane_entries)
{
    RowsPlan p{};
    const int64_t chunk = (int64_t)kWave * lane_entries;
    p.vec = rows > 0 && cols > 0 && cols % 32 == 0 && ld % 4 == 0 && cols <= ((int64_t)1 << 30);
    if (!p.vec) return p;
    const int64_t chunks_per_row = (cols + chunk - 1) / chunk;
    if (rows * chunks_per_row >= ((int64_t)1 << 31)) { p.vec = false; return p; }
    p.geom.cols = (int)cols;
    p.geom.ld = ld;
    p.geom.lane_entries = lane_entries;
    p.geom.loads = kLoads;
    p.geom.chunks_per_row = (uint32_t)chunks_per_row;
    p.geom.num_chunks = (uint32_t)(rows * chunks_per_row);
    p.geom.div_chunks_per_row = make_fast_div((uint32_t)chunks_per_row);
    const int64_t per_block = (int64_t)kBlockWaves * kLoads;
    p.same_row = chunks_per_row % per_block == 0 && cols % chunk == 0;
    p.grid = (unsigned)((rows * chunks_per_row + per_block - 1) / per_block);
    return p;
}

// ---- Eq. 6 ----------------------------------------------------------------------------------
struct SelectSet {
    const float *w;
    uint32_t *mask;
};

struct SelectArgs {
    SelectSet set[kMaxListed];
    RowsGeom geom;
    int n_keep;
};

template <int M, bool SAME_ROW>
__global__ __launch_bounds__(kBlockThreads) void nm_select_rows(const SelectArgs a)
{
    const SelectSet t = a.set[blockIdx.y];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int cols = a.geom.cols;
    vf4_t raw[kLoads];
    int col[kLoads];
    uint32_t *dst[kLoads];
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const RowsPiece piece = rows_piece<SAME_ROW>(a.geom, blockIdx.x, wave, k);
        col[k] = piece.col + lane * 4;
        dst[k] = t.mask + (int64_t)piece.row * (cols >> 5);
        raw[k] = vf4_t{0.0f, 0.0f, 0.0f, 0.0f};      // past the end of the row: zeros, nothing stored
        if (col[k] < cols) raw[k] = load_once(reinterpret_cast<const vf4_t *>(t.w + (int64_t)piece.row * a.geom.ld + col[k]));
    }
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const float x[4] = {raw[k].x, raw[k].y, raw[k].z, raw[k].w};
        const uint32_t nib = keep_nibble<M>(x, a.n_keep, lane);      // all 64 lanes take part
        const uint32_t word = or_reduce_8lanes(nib << ((lane & 7) * 4));
        if ((lane & 7) == 0 && col[k] < cols) dst[k][col[k] >> 5] = word;
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

cast_status launch_nm_select_list(const cast_matrix *m, int count, int n_keep, int m_group, hipStream_t st)
{
    std::vector<char> taken((size_t)count, 0);
    for (int i = 0; i < count; ++i) {
        if (taken[i] || m[i].rows == 0 || m[i].cols == 0) continue;
        int group[kMaxListed];
        const int n = take_group(m, count, taken, i, [](const cast_matrix &, const cast_matrix &) { return true; }, group);
        const RowsPlan p = plan_rows(m[i].rows, m[i].cols, m[i].ld, 4);
        if (p.vec) {
            SelectArgs a{{}, p.geom, n_keep};
            for (int k = 0; k < n; ++k) a.set[k] = SelectSet{m[group[k]].w, m[group[k]].mask_bits};
            const dim3 grid(p.grid, (unsigned)n), block(kBlockThreads);
            switch (m_group * 2 + (p.same_row ? 1 : 0)) {
            case 4: hipLaunchKernelGGL((nm_select_rows<2, false>), grid, block, 0, st, a); break;
            case 5: hipLaunchKernelGGL((nm_select_rows<2, true>), grid, block, 0, st, a); break;
            case 8: hipLaunchKernelGGL((nm_select_rows<4, false>), grid, block, 0, st, a); break;
            case 9: hipLaunchKernelGGL((nm_select_rows<4, true>), grid, block, 0, st, a); break;
            case 16: hipLaunchKernelGGL((nm_select_rows<8, false>), grid, block, 0, st, a); break;
            default: hipLaunchKernelGGL((nm_select_rows<8, true>), grid, block, 0, st, a); break;
            }
            if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
            continue;
        }
        for (int k = 0; k < n; ++k) {      // other shapes: one thread per mask word, one launch per matrix
            const cast_matrix &t = m[group[k]];
            const int64_t words = t.rows * ((t.cols + 31) / 32);
            const unsigned grid = (unsigned)((words + kBlockThreads - 1) / kBlockThreads);
            switch (m_group) {
            case 2: hipLaunchKernelGGL(nm_select_unit<2>, dim3(grid), dim3(kBlockThreads), 0, st, t.w, t.mask_bits, t.rows, t.cols, t.ld, n_keep); break;
            case 4: hipLaunchKernelGGL(nm_select_unit<4>, dim3(grid), dim3(kBlockThreads), 0, st, t.w, t.mask_bits, t.rows, t.cols, t.ld, n_keep); break;
            default: hipLaunchKernelGGL(nm_select_unit<8>, dim3(grid), dim3(kBlockThreads), 0, st, t.w, t.mask_bits, t.rows, t.cols, t.ld, n_keep); break;
            }
            if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
        }
    }
    return CAST_OK;
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
        const vf4_t t = load_once(reinterpret_cast<const vf4_t *>(w + r * ld + c));
        x[0] = A * t.x; x[1] = A * t.y; x[2] = A * t.z; x[3] = A * t.w;
    } else {
        x[0] = A * w[r * ld + c];
    }
    if constexpr (BF16OUT) {
        uint16_t *o = static_cast<uint16_t *>(out) + idx;
        if constexpr (W == 4) {
            const vu2_t q = {f32x2_to_bf16_rne(x[0], x[1]), f32x2_to_bf16_rne(x[2], x[3])};
            store_full(reinterpret_cast<vu2_t *>(o), q);
        } else {
            o[0] = (uint16_t)f32_to_bf16_rne(x[0]);
        }
    } else {
        float *o = static_cast<float *>(out) + idx;
        if constexpr (W == 4) store_full(reinterpret_cast<vf4_t *>(o), vf4_t{x[0], x[1], x[2], x[3]});
        else o[0] = x[0];
    }
}

// The same for rows that are whole mask words (the benchmark shapes): the row-block form of this file.
struct ScaleSet {
    const float *w;
    const float *scale;
    void *out;
};

struct ScaleArgs {
    ScaleSet set[kMaxListed];
    RowsGeom geom;
    FastDivU32 div_seg_len;
    int n_segments;
};

template <bool BF16OUT, bool SAME_ROW>
__global__ __launch_bounds__(kBlockThreads) void weight_scale_rows(const ScaleArgs a)
{
    const ScaleSet t = a.set[blockIdx.y];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int cols = a.geom.cols;
    vf4_t raw[kLoads];
    float A[kLoads];
    int64_t at[kLoads];      // dense index of the thread's first entry, -1: nothing to do
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const RowsPiece piece = rows_piece<SAME_ROW>(a.geom, blockIdx.x, wave, k);
        const int c = piece.col + lane * 4;
        at[k] = -1;
        raw[k] = vf4_t{0.0f, 0.0f, 0.0f, 0.0f};
        A[k] = 0.0f;
        if (c < cols) {
            at[k] = (int64_t)piece.row * cols + c;
            raw[k] = load_once(reinterpret_cast<const vf4_t *>(t.w + (int64_t)piece.row * a.geom.ld + c));
            A[k] = t.scale[(int64_t)piece.row * a.n_segments + fast_div((uint32_t)c, a.div_seg_len)];
        }
    }
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        if (at[k] < 0) continue;
        const float x0 = A[k] * raw[k].x, x1 = A[k] * raw[k].y, x2 = A[k] * raw[k].z, x3 = A[k] * raw[k].w;      // Eq. 12
        if constexpr (BF16OUT) {
            const vu2_t q = {f32x2_to_bf16_rne(x0, x1), f32x2_to_bf16_rne(x2, x3)};
            store_full(reinterpret_cast<vu2_t *>(static_cast<uint16_t *>(t.out) + at[k]), q);
        } else {
            store_full(reinterpret_cast<vf4_t *>(static_cast<float *>(t.out) + at[k]), vf4_t{x0, x1, x2, x3});
        }
    }
}

cast_status launch_weight_scale_list(const cast_matrix *m, int count, int n_segments, int out_dtype, hipStream_t st)
{
    const bool bf16 = out_dtype == CAST_BF16;
    std::vector<char> taken((size_t)count, 0);
    for (int i = 0; i < count; ++i) {
        if (taken[i] || m[i].rows == 0 || m[i].cols == 0) continue;
        int group[kMaxListed];
        const int n = take_group(m, count, taken, i, [](const cast_matrix &, const cast_matrix &) { return true; }, group);
        const cast_matrix &t0 = m[i];
        const int64_t seg_len = t0.cols / n_segments;
        const RowsPlan p = plan_rows(t0.rows, t0.cols, t0.ld, 4);
        if (p.vec && seg_len % 4 == 0) {
            ScaleArgs a{{}, p.geom, make_fast_div((uint32_t)seg_len), n_segments};
            for (int k = 0; k < n; ++k) a.set[k] = ScaleSet{m[group[k]].w, m[group[k]].scale, m[group[k]].out};
            const dim3 grid(p.grid, (unsigned)n), block(kBlockThreads);
            if (p.same_row) {
                if (bf16) hipLaunchKernelGGL((weight_scale_rows<true, true>), grid, block, 0, st, a);
                else hipLaunchKernelGGL((weight_scale_rows<false, true>), grid, block, 0, st, a);
            } else {
                if (bf16) hipLaunchKernelGGL((weight_scale_rows<true, false>), grid, block, 0, st, a);
                else hipLaunchKernelGGL((weight_scale_rows<false, false>), grid, block, 0, st, a);
            }
            if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
            continue;
        }
        for (int k = 0; k < n; ++k) {
            const cast_matrix &t = m[group[k]];
            const int64_t total = t.rows * t.cols;
            if (seg_len % 4 == 0 && t.ld % 4 == 0) {
                const unsigned grid = (unsigned)((total / 4 + kBlockThreads - 1) / kBlockThreads);
                if (bf16) hipLaunchKernelGGL((weight_scale_kernel<true, 4>), dim3(grid), dim3(kBlockThreads), 0, st, t.w, t.scale, t.out, t.rows, t.cols, t.ld, seg_len);
                else hipLaunchKernelGGL((weight_scale_kernel<false, 4>), dim3(grid), dim3(kBlockThreads), 0, st, t.w, t.scale, t.out, t.rows, t.cols, t.ld, seg_len);
            } else {
                const unsigned grid = (unsigned)((total + kBlockThreads - 1) / kBlockThreads);
                if (bf16) hipLaunchKernelGGL((weight_scale_kernel<true, 1>), dim3(grid), dim3(kBlockThreads), 0, st, t.w, t.scale, t.out, t.rows, t.cols, t.ld, seg_len);
                else hipLaunchKernelGGL((weight_scale_kernel<false, 1>), dim3(grid), dim3(kBlockThreads), 0, st, t.w, t.scale, t.out, t.rows, t.cols, t.ld, seg_len);
            }
            if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
        }
    }
    return CAST_OK;
}

// ---- hard prune + fold + pack ---------------------------------------------------------------
struct PackSet {
    const float *w;
    const float *scale;       // or NULL
    const uint32_t *mask;     // or NULL: Eq. 6 on w
    void *values;
    uint32_t *meta;
    uint32_t *status;         // or NULL: where the number of stored-mask groups without exactly N ones is added
};

// Adds the wavefront's count of invalid groups to *status with one atomic, and only if there are any: a valid
// mask costs no atomics at all.
__device__ __forceinline__ void report_bad_groups(uint32_t *status, uint32_t bad_in_lane)
{
    const uint32_t total = wave_sum_u32(bad_in_lane);
    if (total != 0 && (threadIdx.x & (kWave - 1)) == 0) atomicAdd(status, total);
}

struct PackArgs {
    PackSet set[kMaxListed];
    RowsGeom geom;
    FastDivU32 div_seg_len;
    int n_segments;
};

// The half-density patterns 2:4 (the paper's) and 1:2 (4:8 has a kernel of its own below).  A lane holds 4
// consecutive entries and always ends up with exactly two kept values, which leave as one 8-byte (fp32) or
// 4-byte (bf16) store at values[dense index / 2]:
//   2:4  the lane is one group; the 4-bit index fields of 8 adjacent lanes form one metadata word;
//   1:2  the lane is two groups with one kept entry each; 16 lanes' bit pairs form one word.
template <int M, bool BF16OUT, bool SAME_ROW>
__global__ __launch_bounds__(kBlockThreads) void project_compress_half_rows(const PackArgs a)
{
    static_assert(M == 4 || M == 2, "2:4 and 1:2 only");
    constexpr int kEntriesPerWord = M == 4 ? 32 : 64;      // columns one metadata word describes
    const PackSet t = a.set[blockIdx.y];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int cols = a.geom.cols;
    vf4_t raw[kLoads];
    uint32_t bits[kLoads];
    float A[kLoads];
    int col[kLoads];
    int64_t dense_row[kLoads];      // dense index of the first entry of the chunk's row
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const RowsPiece piece = rows_piece<SAME_ROW>(a.geom, blockIdx.x, wave, k);
        const uint32_t row = piece.row;
        dense_row[k] = (int64_t)row * cols;
        col[k] = piece.col + lane * 4;
        raw[k] = vf4_t{0.0f, 0.0f, 0.0f, 0.0f};
        bits[k] = 0;
        A[k] = 1.0f;
        if (col[k] < cols) {
            raw[k] = load_once(reinterpret_cast<const vf4_t *>(t.w + (int64_t)row * a.geom.ld + col[k]));
            if (t.mask) bits[k] = load_once(t.mask + (int64_t)row * (cols >> 5) + (col[k] >> 5));
            if (t.scale) A[k] = t.scale[(int64_t)row * a.n_segments + fast_div((uint32_t)col[k], a.div_seg_len)];      // Eq. 12
        }
    }
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const float x[4] = {raw[k].x, raw[k].y, raw[k].z, raw[k].w};
        uint32_t nib;
        if (t.mask) nib = (bits[k] >> (col[k] & 31)) & 0xFu;
        else nib = keep_nibble<M>(x, M / 2, lane);
        float va, vb;        // the two values this lane stores
        uint32_t word;       // the metadata word its run of lanes forms
        if constexpr (M == 4) {
            const uint32_t first = (uint32_t)__builtin_ctz(nib | 0x10u);      // positions of the two kept entries, ascending
            const uint32_t rest = nib & (nib - 1u);
            const uint32_t second = (uint32_t)__builtin_ctz(rest | 0x10u) & 3u;
            va = first == 0 ? x[0] : (first == 1 ? x[1] : x[2]);
            vb = second == 1 ? x[1] : (second == 2 ? x[2] : x[3]);
            const uint32_t field = (first & 3u) | (second << 2);
            word = or_reduce_8lanes(field << ((lane & 7) * 4));
        } else {
            const uint32_t ia = (nib & 1u) ? 0u : 1u, ib = (nib & 4u) ? 0u : 1u;   // which entry of each pair is kept
            va = ia ? x[1] : x[0];
            vb = ib ? x[3] : x[2];
            word = or_reduce_16lanes((ia | (ib << 1)) << ((lane & 15) * 2));
        }
        if (t.mask && t.status) {      // uniform over the workgroup
            uint32_t bad = 0;
            if (col[k] < cols) bad = M == 4 ? (uint32_t)(__popc(nib) != 2) : (uint32_t)(__popc(nib & 3u) != 1) + (uint32_t)(__popc(nib >> 2) != 1);
            report_bad_groups(t.status, bad);
        }
        if (col[k] >= cols) continue;      // (after the cross-lane steps, which all 64 lanes take)
        if (t.scale) { va = A[k] * va; vb = A[k] * vb; }
        const int64_t at = (dense_row[k] + col[k]) >> 1;      // half of the entries are kept
        if constexpr (BF16OUT) {
            store_full(static_cast<uint32_t *>(t.values) + (at >> 1), f32x2_to_bf16_rne(va, vb));
        } else {
            store_full(reinterpret_cast<vu2_t *>(static_cast<float *>(t.values) + at), vu2_t{__float_as_uint(va), __float_as_uint(vb)});
        }
        constexpr int kLanesPerWord = kEntriesPerWord / kLaneElems;
        if ((lane & (kLanesPerWord - 1)) == 0) t.meta[(dense_row[k] + col[k]) / kEntriesPerWord] = word;
    }
}

// 4:8 with a whole group per lane: 8 consecutive entries (two 16-byte loads), so the four kept values
// are picked inside the lane (the k-th kept entry can only be one of entries k .. k + 4) and leave as
// one 16-byte (fp32) or 8-byte (bf16) store; two adjacent lanes' 12-bit index fields form a metadata
// word.  The exchange between lane pairs that a 4-entries-per-lane form needs made it ALU-bound.
template <bool BF16OUT, bool SAME_ROW>
__global__ __launch_bounds__(kBlockThreads) void project_compress_4of8_rows(const PackArgs a)
{
    const PackSet t = a.set[blockIdx.y];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int cols = a.geom.cols;
    vf4_t lo[kLoads], hi[kLoads];
    uint32_t bits[kLoads];
    float A[kLoads];
    int col[kLoads];
    int64_t dense_row[kLoads];
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const RowsPiece piece = rows_piece<SAME_ROW>(a.geom, blockIdx.x, wave, k);
        const uint32_t row = piece.row;
        dense_row[k] = (int64_t)row * cols;
        col[k] = piece.col + lane * 8;
        lo[k] = hi[k] = vf4_t{0.0f, 0.0f, 0.0f, 0.0f};
        bits[k] = 0;
        A[k] = 1.0f;
        if (col[k] < cols) {
            const vf4_t *src = reinterpret_cast<const vf4_t *>(t.w + (int64_t)row * a.geom.ld + col[k]);
            lo[k] = load_once(src);
            hi[k] = load_once(src + 1);
            if (t.mask) bits[k] = load_once(t.mask + (int64_t)row * (cols >> 5) + (col[k] >> 5));
            if (t.scale) A[k] = t.scale[(int64_t)row * a.n_segments + fast_div((uint32_t)col[k], a.div_seg_len)];
        }
    }
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const float x[8] = {lo[k].x, lo[k].y, lo[k].z, lo[k].w, hi[k].x, hi[k].y, hi[k].z, hi[k].w};
        const uint32_t kept = t.mask ? (bits[k] >> (col[k] & 31)) & 0xFFu : keep_bits_group<8>(x, 4);
        // positions of the four kept entries, ascending (a given mask with fewer bits: the guard bit keeps them in range)
        const uint32_t r1 = kept & (kept - 1u), r2 = r1 & (r1 - 1u), r3 = r2 & (r2 - 1u);
        const uint32_t p0 = (uint32_t)__builtin_ctz(kept | 0x100u) & 7u, p1 = (uint32_t)__builtin_ctz(r1 | 0x100u) & 7u;
        const uint32_t p2 = (uint32_t)__builtin_ctz(r2 | 0x100u) & 7u, p3 = (uint32_t)__builtin_ctz(r3 | 0x100u) & 7u;
        float v0 = p0 == 0 ? x[0] : (p0 == 1 ? x[1] : (p0 == 2 ? x[2] : (p0 == 3 ? x[3] : x[4])));
        float v1 = p1 == 1 ? x[1] : (p1 == 2 ? x[2] : (p1 == 3 ? x[3] : (p1 == 4 ? x[4] : x[5])));
        float v2 = p2 == 2 ? x[2] : (p2 == 3 ? x[3] : (p2 == 4 ? x[4] : (p2 == 5 ? x[5] : x[6])));
        float v3 = p3 == 3 ? x[3] : (p3 == 4 ? x[4] : (p3 == 5 ? x[5] : (p3 == 6 ? x[6] : x[7])));
        const uint32_t field = p0 | (p1 << 3) | (p2 << 6) | (p3 << 9);
        const uint32_t word = field | (dpp_u32<kDppQuadXor1>(field) << 16);           // even lane: its group, then the odd lane's
        if (t.mask && t.status) report_bad_groups(t.status, (uint32_t)(col[k] < cols && __popc(kept) != 4));
        if (col[k] >= cols) continue;
        if (t.scale) { v0 = A[k] * v0; v1 = A[k] * v1; v2 = A[k] * v2; v3 = A[k] * v3; }
        const int64_t at = (dense_row[k] + col[k]) >> 1;
        if constexpr (BF16OUT) {
            const vu2_t h = {f32x2_to_bf16_rne(v0, v1), f32x2_to_bf16_rne(v2, v3)};
            store_full(reinterpret_cast<vu2_t *>(static_cast<uint16_t *>(t.values) + at), h);
        } else {
            store_full(reinterpret_cast<vf4_t *>(static_cast<float *>(t.values) + at), vf4_t{v0, v1, v2, v3});
        }
        if ((lane & 1) == 0) t.meta[(dense_row[k] + col[k]) >> 4] = word;
    }
}

// Any N:M and any shape with cols % M == 0: one thread per 64 consecutive columns of a row,
// which always holds a whole number of metadata words.
template <int M, bool BF16OUT>
__global__ __launch_bounds__(kBlockThreads) void project_compress_unit(
    const float *w, const float *scale, const uint32_t *mask, void *values, uint32_t *meta,
    int64_t rows, int64_t cols, int64_t ld, int n_keep, int n_segments, uint32_t *status)
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
    uint32_t word = 0, bad = 0;
    for (int64_t c = c0; c < ce; c += M) {
        const int64_t gi = c / M;
        float x[M];
#pragma unroll
        for (int j = 0; j < M; ++j) x[j] = w[r * ld + c + j];
        uint32_t bits;
        if (mask) bits = (mask[r * mask_wpr + c / 32] >> (unsigned)(c % 32)) & ((1u << M) - 1u);
        else bits = keep_bits_group<M>(x, n_keep);
        if (mask && status && (int)__popc(bits) != n_keep) ++bad;
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
    if (bad != 0) atomicAdd(status, bad);      // invalid stored masks only
}

template <int M>
static void launch_pack_unit(bool bf16, unsigned grid, hipStream_t st, const float *w, const float *scale,
                             const uint32_t *mask, void *values, uint32_t *meta, int64_t rows,
                             int64_t cols, int64_t ld, int n_keep, int n_segments, uint32_t *status)
{
    if (bf16) hipLaunchKernelGGL((project_compress_unit<M, true>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, mask, values, meta, rows, cols, ld, n_keep, n_segments, status);
    else hipLaunchKernelGGL((project_compress_unit<M, false>), dim3(grid), dim3(kBlockThreads), 0, st, w, scale, mask, values, meta, rows, cols, ld, n_keep, n_segments, status);
}

template <bool BF16OUT, bool SAME_ROW>
static void launch_pack_rows_as(int m_group, dim3 grid, dim3 block, hipStream_t st, const PackArgs &a)
{
    switch (m_group) {
    case 4: hipLaunchKernelGGL((project_compress_half_rows<4, BF16OUT, SAME_ROW>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((project_compress_4of8_rows<BF16OUT, SAME_ROW>), grid, block, 0, st, a); break;
    default: hipLaunchKernelGGL((project_compress_half_rows<2, BF16OUT, SAME_ROW>), grid, block, 0, st, a); break;
    }
}

static void launch_pack_rows(int m_group, bool bf16, bool same_row, dim3 grid, dim3 block, hipStream_t st, const PackArgs &a)
{
    if (bf16) { if (same_row) launch_pack_rows_as<true, true>(m_group, grid, block, st, a); else launch_pack_rows_as<true, false>(m_group, grid, block, st, a); }
    else { if (same_row) launch_pack_rows_as<false, true>(m_group, grid, block, st, a); else launch_pack_rows_as<false, false>(m_group, grid, block, st, a); }
}

cast_status launch_project_compress_list(const cast_matrix *m, int count, int n_segments, int n_keep, int m_group,
                                         int value_dtype, hipStream_t st)
{
    const bool bf16 = value_dtype == CAST_BF16;
    std::vector<char> taken((size_t)count, 0);
    auto alike = [](const cast_matrix &x, const cast_matrix &y) { return (x.scale == nullptr) == (y.scale == nullptr) && (x.mask_bits == nullptr) == (y.mask_bits == nullptr); };
    for (int i = 0; i < count; ++i) {
        if (taken[i] || m[i].rows == 0 || m[i].cols == 0) continue;
        int group[kMaxListed];
        const int n = take_group(m, count, taken, i, alike, group);
        const cast_matrix &t0 = m[i];
        const int segs = t0.scale ? n_segments : 0;
        const int64_t seg_len = segs ? t0.cols / segs : t0.cols;
        // the vector kernels: half-density patterns, rows that are whole mask words and whole metadata words
        // (32 columns for 2:4, 16 for 4:8, 64 for 1:2), scale segments that are whole lanes (4 entries, 8 for 4:8:
        // with 1:2 a lane holds two groups, which must not lie in two segments)
        const int word_cols = m_group == 4 ? 32 : (m_group == 8 ? 16 : 64);
        const RowsPlan p = plan_rows(t0.rows, t0.cols, t0.ld, m_group == 8 ? 8 : 4);
        const int lane_entries = m_group == 8 ? 8 : 4;      // a lane's entries share one scale factor
        if (2 * n_keep == m_group && p.vec && t0.cols % word_cols == 0 && seg_len % lane_entries == 0) {
            PackArgs a{{}, p.geom, make_fast_div((uint32_t)seg_len), segs};
            for (int k = 0; k < n; ++k) {
                const cast_matrix &t = m[group[k]];
                a.set[k] = PackSet{t.w, t.scale, t.mask_bits, t.out, t.meta, t.mask_bits ? t.mask_status : nullptr};
            }
            const dim3 grid(p.grid, (unsigned)n), block(kBlockThreads);
            launch_pack_rows(m_group, bf16, p.same_row, grid, block, st, a);
            if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
            continue;
        }
        for (int k = 0; k < n; ++k) {
            const cast_matrix &t = m[group[k]];
            const int64_t units = t.rows * ((t.cols + 63) / 64);
            const unsigned grid = (unsigned)((units + kBlockThreads - 1) / kBlockThreads);
            switch (m_group) {
            case 2: launch_pack_unit<2>(bf16, grid, st, t.w, t.scale, t.mask_bits, t.out, t.meta, t.rows, t.cols, t.ld, n_keep, segs, t.mask_bits ? t.mask_status : nullptr); break;
            case 4: launch_pack_unit<4>(bf16, grid, st, t.w, t.scale, t.mask_bits, t.out, t.meta, t.rows, t.cols, t.ld, n_keep, segs, t.mask_bits ? t.mask_status : nullptr); break;
            default: launch_pack_unit<8>(bf16, grid, st, t.w, t.scale, t.mask_bits, t.out, t.meta, t.rows, t.cols, t.ld, n_keep, segs, t.mask_bits ? t.mask_status : nullptr); break;
            }
            if (launch_status() != CAST_OK) return CAST_ERR_LAUNCH;
        }
    }
    return CAST_OK;
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
                word[k] = load_once(mask + t);
                if (other) diff[k] = load_once(other + t);
                x[k] = load_once(reinterpret_cast<const vf4_t *>(w + (int64_t)r * ld + (int64_t)word_in_row * 32 + part * 4));
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
