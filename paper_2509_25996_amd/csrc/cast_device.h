// Device-side building blocks shared by the gfx950 kernels of libcast.
//
// Wavefronts are 64 lanes.  In the vector kernels every lane owns 4 consecutive fp32
// entries of a row (one 16-byte load per array), so a wavefront covers 256 consecutive
// entries per step and every load/store instruction touches one contiguous 1 KiB block.
// A group of M entries (Eq. 3) therefore lives in a quarter lane pair (M = 2: two groups per
// lane), in one lane (M = 4) or in two adjacent lanes (M = 8), and the mask bits of 8
// adjacent lanes form one 32-bit mask word.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

namespace cast {

constexpr int kWave = 64;
constexpr int kLaneElems = 4;                    // fp32 entries per lane per chunk
constexpr int kChunk = kWave * kLaneElems;       // 256 entries per wavefront per chunk
constexpr int kBlockThreads = 256;
constexpr int kBlockWaves = kBlockThreads / kWave;
constexpr int kMaxBlockWaves = 16;               // the step kernels run with 4 to 16 wavefronts per workgroup
constexpr int kMaxBlockThreads = kMaxBlockWaves * kWave;
constexpr int kPieceChunks = 8;                  // split plans: chunks (= wavefronts) per piece of a row segment

// ---- how a matrix is cut into spans ---------------------------------------------------------
// A span is the unit of work of one wavefront (or of 2..16 cooperating wavefronts of one
// workgroup): a run of consecutive entries inside one row that starts and ends on a mask word.
// w, mu and v may have a row stride ld > cols (e.g. the three arrays interleaved row by row in
// one allocation, which keeps their streams close together in HBM); the gradient, the mask
// bits and the packed outputs are always dense.
struct FastDivU32 {           // n / d for 32-bit n by multiply-high and shifts (d >= 1)
    uint32_t mul, shift, is_one;
};

inline FastDivU32 make_fast_div(uint32_t d)
{
    FastDivU32 f{0, 0, 1};
    if (d <= 1) return f;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;                                  // l = ceil(log2 d)
    f.mul = (uint32_t)((((1ull << l) - d) << 32) / d + 1);        // floor(2^32 (2^l - d) / d) + 1
    f.shift = l - 1;
    f.is_one = 0;
    return f;
}

__host__ __device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDivU32 &f)
{
    if (f.is_one) return n;
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t t = __umulhi(f.mul, n);
#else
    const uint32_t t = (uint32_t)(((uint64_t)f.mul * n) >> 32);
#endif
    return (t + ((n - t) >> 1)) >> f.shift;
}

struct SpanGeom {
    int64_t total;          // rows * cols
    int64_t cols;
    int64_t row_gap;        // ld - cols: entries skipped between the rows of w, mu, v
    int64_t m_row_gap;      // the same for a first moment kept in bf16, in its own entries (else = row_gap)
    int64_t span_len;       // entries per span (the last span of a flat plan may be shorter)
    int64_t num_spans;
    int spans_per_row;      // 0: flat plan (the matrix is one contiguous array, spans ignore rows)
    int waves_per_span;     // 1, 2 or 4 (several spans per workgroup), or 5..16 = the workgroup's wavefronts
    FastDivU32 div_spans_per_row;
    // Split plan (pieces_per_segment > 1): a row segment of segment_len entries is cut into pieces of
    // span_len entries (the last one shorter), one span each; spans_per_row then counts pieces.
    int pieces_per_segment;
    int64_t segment_len;
    FastDivU32 div_pieces;
};

// Which span a wavefront works on and its place among the cooperating wavefronts.  Either the
// whole workgroup shares one span, or the number of cooperating wavefronts is a power of two, so
// this is shifts and masks on scalar registers (a runtime division would be carried out, and
// leave its result, in vector registers).
struct SpanSlot {
    int64_t span;
    int sub;
};

__host__ __device__ __forceinline__ SpanSlot span_slot(const SpanGeom &g, int64_t block, int wave, int block_waves)
{
    SpanSlot s;
    if (g.waves_per_span == block_waves) {     // one span per workgroup: any number of wavefronts
        s.span = block;
        s.sub = wave;
        return s;
    }
    const int shift = __builtin_ctz((unsigned)g.waves_per_span);
    s.span = block * (block_waves >> shift) + (wave >> shift);
    s.sub = wave & (g.waves_per_span - 1);
    return s;
}

struct SpanOrigin {
    int64_t state_begin;    // first entry of the span in w, mu, v
    int64_t dense_begin;    // first entry of the span in dense [rows, cols] numbering
    int64_t m_begin;        // first entry of the span in a first moment kept in bf16
    int len;                // entries (0 for spans past the end)
};

__host__ __device__ __forceinline__ SpanOrigin span_origin(const SpanGeom &g, int64_t span)
{
    SpanOrigin o{0, 0, 0, 0};
    if (span >= g.num_spans) return o;
    o.dense_begin = span * g.span_len;
    o.state_begin = o.dense_begin;
    o.m_begin = o.dense_begin;
    if (g.spans_per_row == 0) {
        const int64_t rem = g.total - o.dense_begin;
        o.len = (int)(rem < g.span_len ? rem : g.span_len);
    } else {
        o.len = (int)g.span_len;
        if (g.row_gap != 0) {
            const int64_t row = (int64_t)fast_div((uint32_t)span, g.div_spans_per_row);
            o.state_begin += row * g.row_gap;
            o.m_begin += row * g.m_row_gap;
        }
    }
    return o;
}

// Split plan: span = piece number; `segment` tells which row segment (scale factor) it belongs to.
__host__ __device__ __forceinline__ SpanOrigin piece_origin(const SpanGeom &g, int64_t span, int64_t &segment)
{
    SpanOrigin o{0, 0, 0, 0};
    segment = 0;
    if (span >= g.num_spans) return o;
    const uint32_t seg = fast_div((uint32_t)span, g.div_pieces);
    const int64_t done = (int64_t)((uint32_t)span - seg * (uint32_t)g.pieces_per_segment) * g.span_len;
    const int64_t rem = g.segment_len - done;
    segment = seg;
    o.len = (int)(rem < g.span_len ? rem : g.span_len);
    o.dense_begin = (int64_t)seg * g.segment_len + done;
    o.state_begin = o.dense_begin;
    o.m_begin = o.dense_begin;
    if (g.row_gap != 0) {
        const int64_t row = (int64_t)fast_div((uint32_t)span, g.div_spans_per_row);
        o.state_begin += row * g.row_gap;
        o.m_begin += row * g.m_row_gap;
    }
    return o;
}

// ---- how the selection, scaling and pack kernels cut a matrix ---------------------------------
// A row is cut into chunks of 64 * lane_entries consecutive entries, one wavefront's load (the last
// chunk of a row may be shorter); the chunks of the whole matrix are numbered row after row, and
// wavefront w of workgroup b takes chunks 4 * loads * b + w, + 4, + 8, ...: a workgroup covers
// 4 * loads consecutive chunks (its k-th load instruction the k-th run of four, as in a plain
// one-thread-per-16-bytes walk; giving a wavefront adjacent chunks instead measured 3 % slower in
// the selection), which may run from the end of one row into the next, so that only the
// last workgroup of a matrix can be partly idle (rows of 11008 entries are 43 chunks: cutting every row
// into workgroups of its own left one of six workgroups 37.5 % full and cost 10 % on such matrices).
#ifndef CAST_ROWS_LOADS
#define CAST_ROWS_LOADS 2
#endif
constexpr int kLoads = CAST_ROWS_LOADS;      // pieces per workgroup = loads in flight per thread (measured: 2 beats 1, 3 and 4)

struct RowsGeom {
    int cols;                 // entries per row (at most 2^30)
    int64_t ld;               // row stride of w
    int lane_entries;         // 4, or 8 for the 4:8 pack
    int loads;                // chunks per wavefront
    uint32_t chunks_per_row;
    uint32_t num_chunks;      // rows * chunks_per_row
    FastDivU32 div_chunks_per_row;
};

struct RowsPiece {
    uint32_t row;
    int col;                  // first column of the wavefront's chunk; cols for chunks past the end of the matrix
};

// The k-th chunk of wavefront `wave` of workgroup `block` (all wave-uniform).  SAME_ROW: the caller knows
// that rows are whole numbers of workgroups (chunks_per_row is a multiple of 4 * loads); the row then depends
// on the workgroup alone and is worked out once for all of a wavefront's chunks, which counts in kernels whose
// wavefronts live for two loads.
template <bool SAME_ROW = false>
__host__ __device__ __forceinline__ RowsPiece rows_piece(const RowsGeom &g, uint32_t block, int wave, int k)
{
    RowsPiece p;
    if constexpr (SAME_ROW) {
        const uint32_t first = block * (uint32_t)(g.loads * kBlockWaves);
        p.row = fast_div(first, g.div_chunks_per_row);
        p.col = (int)((first - p.row * g.chunks_per_row + (uint32_t)(k * kBlockWaves + wave)) * (uint32_t)(kWave * g.lane_entries));
        return p;
    }
    const uint32_t chunk = (block * (uint32_t)g.loads + (uint32_t)k) * (uint32_t)kBlockWaves + (uint32_t)wave;
    if (chunk >= g.num_chunks) {
        p.row = 0;
        p.col = g.cols;
        return p;
    }
    p.row = fast_div(chunk, g.div_chunks_per_row);
    p.col = (int)((chunk - p.row * g.chunks_per_row) * (uint32_t)(kWave * g.lane_entries));
    return p;
}

// ---- cross-lane moves inside a row of 16 lanes (DPP: no LDS traffic) -------------------
// quad_perm selectors: lane i of each quad reads lane perm[i] of the same quad.
constexpr int kDppQuadXor1 = 0xB1;       // [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141; // lane i of each 8 reads lane 7-i
constexpr int kDppRowMirror = 0x140;     // lane i of each 16 reads lane 15-i

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}

// A 64-bit value that is the same in every lane, moved to scalar registers.
__device__ __forceinline__ unsigned long long uniform_u64(unsigned long long x)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((unsigned long long)hi << 32) | lo;
}

// OR of a value over each aligned run of 8 lanes; every lane of the run gets the result.
__device__ __forceinline__ uint32_t or_reduce_8lanes(uint32_t x)
{
    x |= dpp_u32<kDppQuadXor1>(x);
    x |= dpp_u32<kDppQuadXor2>(x);
    x |= dpp_u32<kDppRowHalfMirror>(x);
    return x;
}

// OR over each aligned run of 16 lanes (a DPP row).
__device__ __forceinline__ uint32_t or_reduce_16lanes(uint32_t x)
{
    x = or_reduce_8lanes(x);
    x |= dpp_u32<kDppRowMirror>(x);
    return x;
}

// Sum over the 64 lanes in a fixed order, the same in every lane of the result: a butterfly inside
// each row of 16 lanes with four DPP moves (partner lane ^1, lane ^2, mirror within 8, mirror
// within 16: no LDS traffic), then the four row sums added in row order from scalar registers.
__device__ __forceinline__ float wave_sum_fixed_order(float x)
{
    x = x + __uint_as_float(dpp_u32<kDppQuadXor1>(__float_as_uint(x)));
    x = x + __uint_as_float(dpp_u32<kDppQuadXor2>(__float_as_uint(x)));
    x = x + __uint_as_float(dpp_u32<kDppRowHalfMirror>(__float_as_uint(x)));
    x = x + __uint_as_float(dpp_u32<kDppRowMirror>(__float_as_uint(x)));
    const float r0 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), 0));
    const float r1 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), 16));
    const float r2 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), 32));
    const float r3 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), 48));
    return ((r0 + r1) + r2) + r3;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x)
{
    x += dpp_u32<kDppQuadXor1>(x);
    x += dpp_u32<kDppQuadXor2>(x);
    x += dpp_u32<kDppRowHalfMirror>(x);
    x += dpp_u32<kDppRowMirror>(x);
    return __builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16) + __builtin_amdgcn_readlane(x, 32) +
           __builtin_amdgcn_readlane(x, 48);
}

// ---- Eq. 6: which of a lane's 4 entries are kept -----------------------------------------
// Magnitude key: the bit pattern with the sign cleared, ordered as an unsigned integer.
__device__ __forceinline__ uint32_t magnitude_key(float x) { return __float_as_uint(x) & 0x7fffffffu; }

// Returns a 4-bit field, bit j set iff entry j of the lane is among the N largest
// magnitudes of its group, ties going to the lower column.  The rank of an entry is the
// number of entries of its group that precede it in that order; it is kept iff rank < N.
// Must be called by all 64 lanes together (M = 8 exchanges keys with the neighbouring lane).
template <int M>
__device__ __forceinline__ uint32_t keep_nibble(const float (&w)[4], int n_keep, int lane)
{
    const uint32_t k0 = magnitude_key(w[0]), k1 = magnitude_key(w[1]);
    const uint32_t k2 = magnitude_key(w[2]), k3 = magnitude_key(w[3]);
    if constexpr (M == 2) {
        // two groups per lane, N = 1: the first entry wins a tie
        const uint32_t a = k0 >= k1, b = k2 >= k3;
        return a | ((a ^ 1u) << 1) | (b << 2) | ((b ^ 1u) << 3);
    } else {
        // "x precedes y" for columns x < y  <=>  key_x >= key_y
        const int c01 = k0 >= k1, c02 = k0 >= k2, c03 = k0 >= k3;
        const int c12 = k1 >= k2, c13 = k1 >= k3, c23 = k2 >= k3;
        int r0 = (1 - c01) + (1 - c02) + (1 - c03);
        int r1 = c01 + (1 - c12) + (1 - c13);
        int r2 = c02 + c12 + (1 - c23);
        int r3 = c03 + c13 + c23;
        if constexpr (M == 8) {
            // the other half of the group sits in lane ^ 1.  For the even lane (lower columns)
            // a neighbour entry precedes only if strictly larger; for the odd lane also if equal.
            const uint32_t odd = (uint32_t)lane & 1u;
            const uint32_t p0 = dpp_u32<kDppQuadXor1>(k0) + odd, p1 = dpp_u32<kDppQuadXor1>(k1) + odd;
            const uint32_t p2 = dpp_u32<kDppQuadXor1>(k2) + odd, p3 = dpp_u32<kDppQuadXor1>(k3) + odd;
            // keys are < 2^31, so key + 1 cannot wrap
            r0 += (p0 > k0) + (p1 > k0) + (p2 > k0) + (p3 > k0);
            r1 += (p0 > k1) + (p1 > k1) + (p2 > k1) + (p3 > k1);
            r2 += (p0 > k2) + (p1 > k2) + (p2 > k2) + (p3 > k2);
            r3 += (p0 > k3) + (p1 > k3) + (p2 > k3) + (p3 > k3);
        }
        return (uint32_t)(r0 < n_keep) | ((uint32_t)(r1 < n_keep) << 1) |
               ((uint32_t)(r2 < n_keep) << 2) | ((uint32_t)(r3 < n_keep) << 3);
    }
}

// Same rule for one whole group held by one thread (scalar kernels for odd shapes).
template <int M>
__device__ __forceinline__ uint32_t keep_bits_group(const float (&w)[M], int n_keep)
{
    uint32_t key[M];
#pragma unroll
    for (int j = 0; j < M; ++j) key[j] = magnitude_key(w[j]);
    // rank[j] = entries that come before entry j in the order "larger magnitude first, then lower index":
    // one comparison per pair decides for both of its entries
    int rank[M];
#pragma unroll
    for (int j = 0; j < M; ++j) rank[j] = j;           // as if every lower index came first ...
#pragma unroll
    for (int j = 0; j < M; ++j) {
#pragma unroll
        for (int k = j + 1; k < M; ++k) {
            const int later_wins = key[k] > key[j];     // ... unless the higher index has the strictly larger magnitude
            rank[j] += later_wins;
            rank[k] -= later_wins;
        }
    }
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < M; ++j) bits |= (uint32_t)(rank[j] < n_keep) << j;
    return bits;
}

// ---- bf16 <-> fp32 ----------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// round to nearest, ties to even; any NaN -> 0x7FC0
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x)
{
    uint32_t b = __float_as_uint(x);
    if ((b & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    b += 0x7fffu + ((b >> 16) & 1u);
    return b >> 16;
}

// Two values at once with the hardware's packed conversion (round to nearest even; gfx950 has it):
// lo -> bits 0..15, hi -> bits 16..31.  NaNs are made the canonical quiet NaN first, so that the
// result is 0x7FC0 like the scalar form's whatever the conversion does with signs and payloads.
__device__ __forceinline__ uint32_t f32x2_to_bf16_rne(float lo, float hi)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const float qnan = __uint_as_float(0x7fc00000u);
    const f32x2 v = {lo != lo ? qnan : lo, hi != hi ? qnan : hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// ---- streaming accesses through buffer resources ------------------------------------------
// Every byte of the optimizer state is touched once per step, so nothing is worth keeping in
// the caches: loads and stores carry the non-temporal hint.  The vector kernels address each
// span through a buffer resource (base pointer + byte length in scalar registers, 32-bit
// offsets in vector registers): the hardware range check returns zeros for loads past the end
// of the span and drops stores there, so ragged tails need no branches and no 64-bit address
// arithmetic per lane.
typedef float vf4_t __attribute__((ext_vector_type(4)));
typedef uint32_t vu4_t __attribute__((ext_vector_type(4)));
typedef uint32_t vu2_t __attribute__((ext_vector_type(2)));

// cache-policy bits of buffer instructions: 2 = nt (streaming), 16 = sc1
#ifndef CAST_AUX_LOAD
#define CAST_AUX_LOAD 2
#endif
#ifndef CAST_AUX_STORE
#define CAST_AUX_STORE 2
#endif
constexpr int kAuxLoad = CAST_AUX_LOAD;
constexpr int kAuxStore = CAST_AUX_STORE;
constexpr int kRsrcWord3 = 0x00020000;        // raw buffer, 32-bit data format (gfx9 family)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t span_resource(const void *base, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, kRsrcWord3);
}

// ---- correctly rounded division by a divisor that is the same for every entry ---------------
// The two bias corrections divide every entry by the same number.  With r = RN(1/y) from the
// host, two Newton corrections carried by exact FMA residuals give RN(x/y) itself (Markstein's
// theorem: a faithful quotient corrected once with the correctly rounded reciprocal is the
// correctly rounded quotient) as long as nothing under- or overflows on the way.  That is
// guaranteed by range checks: the host enables the short path only for 2^-12 <= y <= 2, and
// an entry may take it only if 2^-63 <= |x| < 2^66; zeros, denormals, huge values, inf and NaN
// take the full IEEE division.  The FMAs here are the division algorithm, not a contraction of
// the update's own multiply-adds.
struct UniformDivisor {
    float y;      // the divisor
    float r;      // RN(1 / y)
    int fast;     // 1 if y is in the range where the short path is valid
};

inline UniformDivisor make_divisor(float y)
{
    UniformDivisor d;
    d.y = y;
    d.r = 1.0f / y;                                   // correctly rounded on the host
    d.fast = (y >= 0x1p-12f && y <= 2.0f) ? 1 : 0;
    return d;
}

__host__ __device__ __forceinline__ bool in_short_division_range(float x)
{
    uint32_t bits;
    __builtin_memcpy(&bits, &x, 4);
    return (((bits >> 23) & 0xffu) - 64u) < 129u;      // biased exponent in [64, 192]
}

__host__ __device__ __forceinline__ float div_short(float x, const UniformDivisor &d)
{
    const float q0 = x * d.r;
    const float e0 = __builtin_fmaf(-d.y, q0, x);
    const float q1 = __builtin_fmaf(e0, d.r, q0);      // faithful
    const float e1 = __builtin_fmaf(-d.y, q1, x);      // exact residual
    return __builtin_fmaf(e1, d.r, q1);                // correctly rounded
}

__host__ __device__ __forceinline__ float div_by_uniform(float x, const UniformDivisor &d)
{
    if (d.fast && in_short_division_range(x)) return div_short(x, d);
    return x / d.y;
}

// ---- stochastic rounding to bf16 (CAST_FLAG_V_BF16) -----------------------------------------
// The integer mixer of the rounding bits as include/cast.h defines them.
__host__ __device__ __forceinline__ uint32_t sr_mix(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

__host__ __device__ __forceinline__ uint32_t sr_key_of(uint32_t seed) { return sr_mix(seed + 0x9e3779b9u); }

// 16 rounding bits of the entry whose 64-bit index has the low half index_lo and the high half
// folded into hi_term = high * 0x9e3779b9.
__host__ __device__ __forceinline__ uint32_t sr_bits(uint32_t key, uint32_t index_lo, uint32_t hi_term)
{
    return sr_mix((index_lo ^ key) + hi_term) >> 16;
}

// x to bf16, away from zero with probability (discarded bits) / 65536 given 16 uniform bits r16;
// infinities and NaN as round-to-nearest converts them.
__device__ __forceinline__ uint32_t f32_to_bf16_sr(float x, uint32_t r16)
{
    const uint32_t bits = __float_as_uint(x);
    const uint32_t rounded = (bits + r16) >> 16;
    return (bits & 0x7f800000u) == 0x7f800000u ? f32_to_bf16_rne(x) : rounded;
}

// ---- Algorithm 1 --------------------------------------------------------------------------
// Scalars of one iteration, prepared on the host in fp32 (one rounding each).
struct StepScalars {
    float lr, beta1, one_minus_beta1, beta2, one_minus_beta2, eps;
    float one_minus_alpha, alpha_lambda;
    float decay_pos, decay_neg, decay_zero;   // alpha_lambda * Sign(w) for w > 0, w < 0, otherwise
    UniformDivisor bias_corr1, bias_corr2;
    int n_keep;
    int v_from_grad;
    int short_forms;       // 1 if the uniform scalars allow the short division / square-root forms
    uint32_t sr_key;       // CAST_FLAG_V_BF16: the mixed seed of the rounding bits
    int rule;              // CAST_RULE_*; read by the one-entry code (adams_entry); the vector kernels have it as a template argument
};

// The comparison rules (Eq. 9, Eq. 10, Sec. 6.7) as the kernels see them.  Additive decay needs no
// code of its own: the host passes one_minus_alpha = 1 (1 * mu is mu, exactly).  For Eq. 9 and 10
// the host also sets v_from_grad, and the kernels treat every entry as kept inside the moments.
constexpr int kRuleAdamwL1 = 1, kRuleAdamL1 = 2, kRuleMaskedFrozen = 4;

// alpha*lambda*Sign(w) with Sign(+-0) = Sign(NaN) = 0: the three possible products come from the host
__device__ __forceinline__ float decay_term(float w, const StepScalars &s)
{
    // the three values are read before the choice: read inside its arms, the compiler merges the reads into
    // one per-lane load from the kernel arguments at a chosen address, a vector memory access per entry
    const float pos = s.decay_pos, neg = s.decay_neg, zero = s.decay_zero;
    return w > 0.0f ? pos : (w < 0.0f ? neg : zero);
}

// Every line below is one correctly rounded fp32 operation: the library is compiled with
// -ffp-contract=off (no fused multiply-add) and -fhip-fp32-correctly-rounded-divide-sqrt, and
// fp32 denormals are not flushed on gfx9, so the result is the same on any IEEE-754 machine.

// First half of the body of Algorithm 1's loop: the moments.
__device__ __forceinline__ void adams_moments(float w, float g, float &mu, float v, bool keep,
                                              const StepScalars &s, float &mu_tilde, float &v_t)
{
    const float t0 = s.beta1 * mu;
    const float t1 = s.one_minus_beta1 * g;
    const float mu_t = t0 + t1;                                   // Eq. 8, first line
    const float d1 = decay_term(w, s);
    const float d0 = s.one_minus_alpha * mu_t;
    const float decayed = d0 + d1;                                // Eq. 7 on the momentum
    mu_tilde = keep ? mu_t : decayed;                             // Algorithm 1: only where m = 0
    const float squared = s.v_from_grad ? g : mu_tilde;
    const float second = squared * squared;
    const float s0 = s.beta2 * v;
    const float s1 = s.one_minus_beta2 * second;
    v_t = s0 + s1;                                                // v from the decayed momentum
    mu = mu_t;                                                    // the undecayed moment is stored
}

// Second half: bias-corrected moments (already divided) to the adaptive step mu^ / (sqrt(v^) + eps)
// and to the new weight.
__device__ __forceinline__ float adams_quotient(float mu_hat, float v_hat, const StepScalars &s)
{
    const float denom = __builtin_sqrtf(v_hat) + s.eps;           // IEEE square root
    return mu_hat / denom;                                        // IEEE division
}

__device__ __forceinline__ float adams_update(float w, float mu_hat, float v_hat, const StepScalars &s)
{
    const float step = s.lr * adams_quotient(mu_hat, v_hat, s);
    return w - step;
}

// One entry, start to end, any rule (scalar kernels).
__device__ __forceinline__ void adams_entry(float &w, float g, float &mu, float &v, bool keep,
                                            const StepScalars &s)
{
    if (s.rule == kRuleMaskedFrozen && !keep) return;             // Sec. 6.7: not updated at all
    const bool no_momentum_decay = s.rule == kRuleAdamwL1 || s.rule == kRuleAdamL1;
    const float d = decay_term(w, s);
    if (s.rule == kRuleAdamL1 && !keep) g = g + d;                // Eq. 10: decay inside the gradient
    float mu_tilde, v_t;
    adams_moments(w, g, mu, v, keep || no_momentum_decay, s, mu_tilde, v_t);
    float q = adams_quotient(div_by_uniform(mu_tilde, s.bias_corr1), div_by_uniform(v_t, s.bias_corr2), s);
    if (s.rule == kRuleAdamwL1 && !keep) q = q + d;               // Eq. 9: decay beside the adaptive step
    const float step = s.lr * q;
    w = w - step;
    v = v_t;
}

// Correctly rounded square root of a normal number well inside the exponent range: the hardware
// approximation is within one unit in the last place, so the answer is that value or one of its
// two neighbours; exact FMA residuals against the neighbours decide (the range and special-value
// handling a general sqrtf needs is left out).
__device__ __forceinline__ float sqrt_short(float x)
{
    const float s = __builtin_amdgcn_sqrtf(x);
    const float s_dn = __uint_as_float(__float_as_uint(s) - 1u);
    const float s_up = __uint_as_float(__float_as_uint(s) + 1u);
    const float r_dn = __builtin_fmaf(-s_dn, s, x);               // x - s_dn * s
    const float r_up = __builtin_fmaf(-s_up, s, x);               // x - s_up * s
    float y = r_dn <= 0.0f ? s_dn : s;
    y = r_up > 0.0f ? s_up : y;
    return y;
}

// Correctly rounded x / d for operands well inside the exponent range: the refinement sequence
// of the IEEE division without its range scaling and special-value fix-up.
__device__ __forceinline__ float div_short_any(float x, float d)
{
    const float r0 = __builtin_amdgcn_rcpf(d);
    const float e = __builtin_fmaf(-d, r0, 1.0f);
    const float r = __builtin_fmaf(e, r0, r0);
    const float q0 = x * r;
    const float e0 = __builtin_fmaf(-d, q0, x);
    const float q1 = __builtin_fmaf(e0, r, q0);
    const float e1 = __builtin_fmaf(-d, q1, x);
    return __builtin_fmaf(e1, r, q1);
}

// The 4 entries of a lane.  The division by the bias corrections, the square root and the
// final division each have a short form that gives the same correctly rounded result when
// every operand is a normal number far from the ends of the exponent range.  Whether that holds
// is decided once per wavefront (a scalar branch) from the smallest and the largest magnitude
// among the 8 dividends of the live lanes: 2^-63 <= |mu~|, v < 2^66 (so zeros, denormals, inf
// take the long forms; a NaN goes through either form as a NaN).  `live` is false for lanes
// past the end of the span, whose zeros must not force the long forms.
// RULE: 0 is Algorithm 1 alone, else the comparison rule to apply (Eq. 9, Eq. 10, frozen masked entries).  Nothing of the incoming state is set aside for the
// rules (registers decide how many wavefronts a compute unit holds): what a rule needs of the
// old values is used before they are overwritten.
// ONE_LOOP only chooses between two spellings of the same arithmetic (the short/long decision
// inside or outside the loop over the four entries); which one the compiler schedules better was
// measured per kernel flavour: outside for the plain step, inside when the compute copy is written
// (6 % on that step).
template <int RULE = 0, bool ONE_LOOP = false>
__device__ __forceinline__ void adams_entries4(float (&w)[4], float (&g)[4], float (&mu)[4],
                                               float (&v)[4], uint32_t nib, bool live,
                                               const StepScalars &s)
{
    float mt[4], vt[4];
    // what the rule changes; which entries it touches is read off nib where needed
    bool l1_in_grad = false, keep_all_in_moments = false, l1_beside_step = false, frozen = false;
    if constexpr (RULE != 0) {
        l1_in_grad = RULE == kRuleAdamL1;                                            // Eq. 10
        keep_all_in_moments = RULE == kRuleAdamwL1 || RULE == kRuleAdamL1;           // no decay on the momentum
        l1_beside_step = RULE == kRuleAdamwL1;                                       // Eq. 9
        frozen = RULE == kRuleMaskedFrozen;                                          // Sec. 6.7
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool kept = (nib >> j) & 1u;
        if constexpr (RULE != 0) {
            if (l1_in_grad) {
                const float decayed = g[j] + decay_term(w[j], s);
                g[j] = kept ? g[j] : decayed;
            }
        }
        float mu_new = mu[j];
        adams_moments(w[j], g[j], mu_new, v[j], kept || keep_all_in_moments, s, mt[j], vt[j]);
        if constexpr (RULE != 0) {
            mu[j] = (frozen && !kept) ? mu[j] : mu_new;           // a frozen entry keeps its moments
        } else {
            mu[j] = mu_new;
        }
    }
    float lo = __builtin_fminf(__builtin_fabsf(mt[0]), __builtin_fabsf(mt[1]));
    float hi = __builtin_fmaxf(__builtin_fabsf(mt[0]), __builtin_fabsf(mt[1]));
#pragma unroll
    for (int j = 2; j < 4; ++j) { lo = __builtin_fminf(lo, __builtin_fabsf(mt[j])); hi = __builtin_fmaxf(hi, __builtin_fabsf(mt[j])); }
#pragma unroll
    for (int j = 0; j < 4; ++j) { lo = __builtin_fminf(lo, vt[j]); hi = __builtin_fmaxf(hi, vt[j]); }
    const bool out_of_range = !(lo >= 0x1p-63f) || !(hi < 0x1p66f);
    if constexpr (RULE != 0) {
        // a frozen entry: its old v takes the place of the new one from here on (the quotient computed from
        // it is not used; the choice of forms above has seen the new one), so that the old state need not
        // stay in registers through the divisions
#pragma unroll
        for (int j = 0; j < 4; ++j) vt[j] = (frozen && !((nib >> j) & 1u)) ? v[j] : vt[j];
    }
    // what the rules change after the adaptive step q = mu^ / (sqrt(v^) + eps) is known
    auto finish = [&](int j, float q) {
        if constexpr (RULE != 0) {
            const bool kept = (nib >> j) & 1u;
            if (l1_beside_step) {
                const float decayed = q + decay_term(w[j], s);
                q = kept ? q : decayed;
            }
            const float step = s.lr * q;
            const float stepped = w[j] - step;
            w[j] = (frozen && !kept) ? w[j] : stepped;
        } else {
            const float step = s.lr * q;
            w[j] = w[j] - step;
        }
        v[j] = vt[j];
    };
    const bool short_forms = s.short_forms && !__any(out_of_range && live);      // wave-uniform
    if constexpr (ONE_LOOP) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (short_forms) {
                const float mu_hat = div_short(mt[j], s.bias_corr1);
                const float v_hat = div_short(vt[j], s.bias_corr2);
                const float denom = sqrt_short(v_hat) + s.eps;
                finish(j, div_short_any(mu_hat, denom));
            } else {
                finish(j, adams_quotient(mt[j] / s.bias_corr1.y, vt[j] / s.bias_corr2.y, s));
            }
        }
    } else if (short_forms) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float mu_hat = div_short(mt[j], s.bias_corr1);
            const float v_hat = div_short(vt[j], s.bias_corr2);
            const float denom = sqrt_short(v_hat) + s.eps;
            finish(j, div_short_any(mu_hat, denom));
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) finish(j, adams_quotient(mt[j] / s.bias_corr1.y, vt[j] / s.bias_corr2.y, s));
    }
}

}  // namespace cast
