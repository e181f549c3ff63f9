// Device side of the fused AdamS iteration (Algorithm 1 / Eq. 8 with the decay of Eq. 7 and the mask
// of Eq. 6) and of the reduction that yields dL/dA for the weight scaling of Eq. 12: the kernels and
// what they pass around.  Host-side planning and launching is in adams_step.hip.
//
// The work is a single streaming read-modify-write over w, mu, v (fp32), the gradient (bf16
// or fp32) and one mask bit per entry: 26.125 bytes per parameter with bf16 gradients (22.125
// with the first moment kept in bf16 as well) and nothing is read twice.  There is no contraction, so no MFMA; the kernel is bound by HBM.
#pragma once
#include "cast_device.h"
#include "cast_internal.h"

#pragma clang fp contract(off)

namespace cast {

// The buffers of one matrix.  A launch carries up to kMaxFused sets in its arguments
// (workgroups with blockIdx.y = k step matrix k).
struct TensorPtrs {
    float *w;
    const void *grad;
    float *m;             // bf16 values instead when the first moment is kept in bf16 (flavour 3)
    float *v;
    uint32_t *mask;
    const float *scale;
    float *scale_grad;
    float *piece_sums;    // split plans: one partial dL/dA sum per piece, else unused
    // Flavours that gather refresh statistics only:
    struct StatsPartial *stats_partials;   // one slot per workgroup of the launch, or NULL
    const uint32_t *initial_mask;          // the mask flips_init counts against, or NULL
    // Flavours that can write the bf16 copy of the updated weights for the next forward pass
    // (Eq. 12 applied: copy_scale[r, s] * w_new, or w_new itself when copy_scale is NULL), or NULL:
    uint16_t *compute_copy;
    const float *copy_scale;
};

// What one workgroup contributes to the mask-learning statistics of a refresh step
// (appendix "Mask Learning"): changed mask bits against the stored and the initial mask, and
// the L1 norms of the kept and of all incoming weights.
struct StatsPartial {
    uint32_t flips_prev, flips_init;
    float l1_kept, l1_all;
};

constexpr int kMaxFused = 16;     // matrices of equal shape that one launch can step (gridDim.y)

struct SpanArgs {
    TensorPtrs set[kMaxFused];   // the buffer sets of the launch: matrix blockIdx.y
    SpanGeom geom;
    StepScalars s;
};

// Kernel flavours (template argument EXTRA) = what the kernel can do besides Algorithm 1, in the low four bits,
// plus the comparison rule it applies (Eq. 9, Eq. 10, frozen masked entries; 0: none), fixed at compile time,
// shifted left by four.  The low bits: 0 plain; 1 can also write the bf16 compute copy and gather refresh
// statistics; 3 plain with the first moment kept in bf16 (CAST_FLAG_MU_BF16); 4 plain that can gather refresh
// statistics (refresh steps only: without the code for the compute copy it runs close to flavour 0); 5 the
// first moment in bf16, with the abilities of 1; 6 both moments in bf16, the second one rounded stochastically
// (CAST_FLAG_V_BF16); 7 the same with the abilities of 1.  The rules combine with 0 and 1.
// 8, 9, 10 are not the method: the walk, the loads, the prefetch and the stores of flavour 0 (9: of flavour 3,
// 10: of flavour 6) around a few multiply-adds instead of Algorithm 1's arithmetic, bf16 moments stored by
// truncation (cast_hbm_stream_probe: what the memory system gives these access patterns).
constexpr int kEmitAndCount = 1;
constexpr int kMuBf16 = 3;
constexpr int kStatsOnly = 4;
constexpr int kMuBf16Emit = 5;
constexpr int kBothBf16 = 6;
constexpr int kBothBf16Emit = 7;
constexpr int kStreamProbe = 8;
constexpr int kStreamProbeMuBf16 = 9;
constexpr int kStreamProbeBothBf16 = 10;
constexpr int abilities(int extra) { return extra & 15; }
constexpr int rule_of(int extra) { return extra >> 4; }      // kRuleAdamwL1, kRuleAdamL1, kRuleMaskedFrozen or 0
constexpr int with_rule(int extra, int rule) { return extra | (rule << 4); }
constexpr bool can_emit(int extra) { return abilities(extra) == kEmitAndCount || abilities(extra) == kMuBf16Emit || abilities(extra) == kBothBf16Emit; }
constexpr bool can_count(int extra) { return can_emit(extra) || abilities(extra) == kStatsOnly; }
constexpr bool is_probe(int extra) { return abilities(extra) >= kStreamProbe && abilities(extra) <= kStreamProbeBothBf16; }
constexpr bool v_is_bf16(int extra) { return abilities(extra) == kBothBf16 || abilities(extra) == kBothBf16Emit || abilities(extra) == kStreamProbeBothBf16; }
constexpr bool mu_is_bf16(int extra) { return abilities(extra) == kMuBf16 || abilities(extra) == kMuBf16Emit || abilities(extra) == kStreamProbeMuBf16 || v_is_bf16(extra); }

// Registers of one chunk as loaded: 4 consecutive entries of each array per lane.
template <bool BF16>
struct Chunk {
    vu4_t w, m, v;    // a bf16 moment: the first 2 dwords of m (of v) hold 4 values
    vu4_t g;          // fp32 gradient: 4 dwords; bf16: the first 2 dwords hold 4 values
    uint32_t word;    // the mask word that holds this lane's 4 bits (non-refresh steps)
    uint32_t initial; // the same word of the initial mask (refresh steps that gather statistics)
};

// The five streams of one span, each behind a buffer resource whose length is the span's own,
// so that any access past the end of the span is void (loads give 0, stores are dropped).
struct SpanBuffers {
    __amdgpu_buffer_rsrc_t w, m, v, g, mask;
    __amdgpu_buffer_rsrc_t initial_mask;      // flavours with refresh statistics only
};

// WORD: whether the stored mask word is wanted (non-refresh steps; refresh steps that count flips);
// INITIAL: whether the initial mask's word is (the latter only)
template <bool BF16, bool WORD, bool INITIAL = false, bool MU16 = false, bool V16 = false>
__device__ __forceinline__ void chunk_load(Chunk<BF16> &c, const SpanBuffers &b, int off)
{
    c.w = __builtin_amdgcn_raw_buffer_load_b128(b.w, off * 4, 0, kAuxLoad);
    if constexpr (BF16) {
        const vu2_t t = __builtin_amdgcn_raw_buffer_load_b64(b.g, off * 2, 0, kAuxLoad);
        c.g.x = t.x; c.g.y = t.y; c.g.z = 0; c.g.w = 0;
    } else {
        c.g = __builtin_amdgcn_raw_buffer_load_b128(b.g, off * 4, 0, kAuxLoad);
    }
    if constexpr (MU16) {
        const vu2_t t = __builtin_amdgcn_raw_buffer_load_b64(b.m, off * 2, 0, kAuxLoad);
        c.m.x = t.x; c.m.y = t.y; c.m.z = 0; c.m.w = 0;
    } else {
        c.m = __builtin_amdgcn_raw_buffer_load_b128(b.m, off * 4, 0, kAuxLoad);
    }
    if constexpr (V16) {
        const vu2_t t = __builtin_amdgcn_raw_buffer_load_b64(b.v, off * 2, 0, kAuxLoad);
        c.v.x = t.x; c.v.y = t.y; c.v.z = 0; c.v.w = 0;
    } else {
        c.v = __builtin_amdgcn_raw_buffer_load_b128(b.v, off * 4, 0, kAuxLoad);
    }
    if constexpr (WORD) c.word = __builtin_amdgcn_raw_buffer_load_b32(b.mask, (off >> 5) * 4, 0, kAuxLoad);
    else c.word = 0;
    if constexpr (INITIAL) c.initial = __builtin_amdgcn_raw_buffer_load_b32(b.initial_mask, (off >> 5) * 4, 0, kAuxLoad);
    else c.initial = 0;
}

__device__ __forceinline__ void unpack4(const vu4_t &x, float (&f)[4])
{
    f[0] = __uint_as_float(x.x); f[1] = __uint_as_float(x.y); f[2] = __uint_as_float(x.z); f[3] = __uint_as_float(x.w);
}

__device__ __forceinline__ vu4_t pack4(const float (&f)[4])
{
    vu4_t x = {__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3])};
    return x;
}

// What a wavefront needs to know about the span it works on; everything here is wave-uniform
// and lives in scalar registers.
struct SpanCtx {
    SpanBuffers b;
    float *scale_grad;   // where dL/dA of this matrix goes, or NULL
    int64_t span;        // index of the span in the matrix (= index into scale / scale_grad; split plans: piece number)
    int64_t segment;     // split plans: the row segment the piece belongs to (index into scale)
    float A;             // its scale factor
    int len;             // entries; 0 for spans past the end of the matrix
    int sub;             // which of the waves_per_span cooperating wavefronts this one is
    __amdgpu_buffer_rsrc_t copy;   // EXTRA: the span's part of the bf16 compute copy
    float copy_A;                  // EXTRA: the factor folded into it
    bool emit;                     // EXTRA: whether there is a compute copy to write
    StatsPartial *stats_slot;      // EXTRA: where this workgroup leaves its refresh statistics, or NULL
    int64_t dense_begin;           // EXTRA (a bf16 second moment): index row * cols + col of the span's first entry
};

// `matrix` selects the buffer set, `block` the workgroup's share of that matrix:
// block_waves / waves_per_span consecutive spans.
template <bool BF16, bool SCALED, bool SPLIT = false, int EXTRA = 0>
__device__ __forceinline__ void span_open(const SpanArgs &a, uint32_t matrix, int64_t block, int wave, SpanCtx &c)
{
    const TensorPtrs t = a.set[matrix];     // a scalar load from the kernel arguments at a wave-uniform offset
    const SpanSlot slot = span_slot(a.geom, block, wave, blockDim.x / kWave);
    c.span = (int64_t)uniform_u64((unsigned long long)slot.span);
    c.sub = slot.sub;
    // 64-bit products are cheapest on the vector ALU, so the compiler may leave these wave-uniform
    // numbers in vector registers; buffer resources need them in scalar registers
    SpanOrigin o;
    c.segment = c.span;
    if constexpr (SPLIT) {
        o = piece_origin(a.geom, c.span, c.segment);
        c.segment = (int64_t)uniform_u64((unsigned long long)c.segment);
    } else {
        o = span_origin(a.geom, c.span);
    }
    o.state_begin = (int64_t)uniform_u64((unsigned long long)o.state_begin);
    o.dense_begin = (int64_t)uniform_u64((unsigned long long)o.dense_begin);
    o.len = __builtin_amdgcn_readfirstlane(o.len);
    c.len = o.len;
    c.b.w = span_resource(t.w + o.state_begin, c.len * 4);
    if constexpr (mu_is_bf16(EXTRA)) c.b.m = span_resource(reinterpret_cast<uint16_t *>(t.m) + (int64_t)uniform_u64((unsigned long long)o.m_begin), c.len * 2);
    else c.b.m = span_resource(t.m + o.state_begin, c.len * 4);
    if constexpr (v_is_bf16(EXTRA)) c.b.v = span_resource(reinterpret_cast<uint16_t *>(t.v) + (int64_t)uniform_u64((unsigned long long)o.m_begin), c.len * 2);
    else c.b.v = span_resource(t.v + o.state_begin, c.len * 4);
    c.dense_begin = v_is_bf16(EXTRA) ? (int64_t)uniform_u64((unsigned long long)o.dense_begin) : 0;
    if constexpr (BF16) c.b.g = span_resource(static_cast<const uint16_t *>(t.grad) + o.dense_begin, c.len * 2);
    else c.b.g = span_resource(static_cast<const float *>(t.grad) + o.dense_begin, c.len * 4);
    c.b.mask = span_resource(t.mask + (o.dense_begin >> 5), c.len / 8);    // spans start and end on mask words
    c.A = 1.0f;
    c.scale_grad = nullptr;
    if constexpr (SCALED) {
        if (c.len > 0) c.A = t.scale[c.segment];
        c.scale_grad = SPLIT ? t.piece_sums : t.scale_grad;     // split plans: the pieces' sums are added up afterwards
    }
    c.emit = false;
    c.copy_A = 1.0f;
    if constexpr (can_emit(EXTRA)) {
        c.emit = t.compute_copy != nullptr;
        // without a copy the resource is empty: every store through it would be void anyway
        c.copy = span_resource(t.compute_copy + (c.emit ? o.dense_begin : 0), c.emit ? c.len * 2 : 0);
        if (c.emit && t.copy_scale && c.len > 0) c.copy_A = t.copy_scale[c.segment];
    }
    if constexpr (can_count(EXTRA)) {
        c.stats_slot = t.stats_partials ? t.stats_partials + block : nullptr;
        const bool initial = t.stats_partials && t.initial_mask;
        c.b.initial_mask = span_resource(t.initial_mask + (initial ? (o.dense_begin >> 5) : 0), initial ? c.len / 8 : 0);
    } else {
        c.stats_slot = nullptr;
    }
}

__device__ __forceinline__ int first_offset(const SpanCtx &c, int lane) { return c.sub * kChunk + lane * kLaneElems; }

// One wavefront (or waves_per_span cooperating ones) walks one span in chunks of 256 entries;
// `cur` holds the first chunk, already requested by the caller, and every further chunk is
// requested before the current one is worked on, so that memory requests stay in flight during
// the arithmetic (flavours with both moments in bf16: after it, see kPrefetch).  Control flow is uniform across the wavefront: lanes past the end of the span
// carry zeros through the arithmetic and the buffer range check voids their stores, so the
// cross-lane steps (M = 8 key exchange, mask word assembly, the dL/dA butterfly) always see
// all 64 lanes.
// LDS through which the wavefronts of a workgroup combine their refresh statistics.
struct StatsShared {
    uint32_t flips_prev[kMaxBlockWaves], flips_init[kMaxBlockWaves];
    float l1_kept[kMaxBlockWaves], l1_all[kMaxBlockWaves];
};

template <int M, bool BF16, bool REFRESH, bool SCALED, int EXTRA = 0>
__device__ __forceinline__ void span_run(const SpanArgs &a, const SpanCtx &c, Chunk<BF16> cur, int lane, int wave,
                                         float *partial, StatsShared *stats_shared = nullptr)
{
    constexpr bool kStats = REFRESH && can_count(EXTRA);      // refresh statistics are gathered if c.stats_slot says so
    constexpr bool kMu16 = mu_is_bf16(EXTRA);
    constexpr bool kV16 = v_is_bf16(EXTRA);
    // Whether the next chunk is requested before the current one is worked on.  The launch plans give nearly every
    // wavefront exactly one chunk, so the request is usually void (past the end of the span); measured over the
    // LLaMA2-7B shapes it still pays to issue it with fp32 moments (+4 %) and with the first moment in bf16 (+2 %),
    // and costs 2 % with both moments in bf16, whose wavefronts then fetch a further chunk only when there is one.
    constexpr bool kPrefetch = !kV16;
    uint32_t flips_prev = 0, flips_init = 0;
    float l1_kept = 0.0f, l1_all = 0.0f;
    const int P = a.geom.waves_per_span;
    const int len = c.len;
    const SpanBuffers &b = c.b;
    const float A = c.A;
    const bool want_gA = SCALED && c.scale_grad != nullptr;
    float acc = 0.0f;
    const int stride = P * kChunk;
    int off = first_offset(c, lane);      // this lane's first entry, relative to the span
    for (int base = c.sub * kChunk; base < len; base += stride) {
        [[maybe_unused]] Chunk<BF16> nxt;
        if constexpr (kPrefetch)
            chunk_load<BF16, (!REFRESH || can_count(EXTRA)), kStats, kMu16, kV16>(nxt, b, off + stride);     // past the end: all zeros, never used

        float w[4], g[4], mu[4], v[4];
        unpack4(cur.w, w);
        if constexpr (kMu16) {
            mu[0] = bf16_lo(cur.m.x); mu[1] = bf16_hi(cur.m.x); mu[2] = bf16_lo(cur.m.y); mu[3] = bf16_hi(cur.m.y);
        } else {
            unpack4(cur.m, mu);
        }
        if constexpr (kV16) {
            v[0] = bf16_lo(cur.v.x); v[1] = bf16_hi(cur.v.x); v[2] = bf16_lo(cur.v.y); v[3] = bf16_hi(cur.v.y);
        } else {
            unpack4(cur.v, v);
        }
        if constexpr (BF16) {
            g[0] = bf16_lo(cur.g.x); g[1] = bf16_hi(cur.g.x); g[2] = bf16_lo(cur.g.y); g[3] = bf16_hi(cur.g.y);
        } else {
            unpack4(cur.g, g);
        }
        uint32_t nib;
        if constexpr (REFRESH) {
            nib = keep_nibble<M>(w, a.s.n_keep, lane);                   // from the incoming weights
            if constexpr (kStats) {
                if (c.stats_slot) {      // appendix "Mask Learning": L1 norms here, flips below where the new word is whole
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float mag = __builtin_fabsf(w[j]);
                        l1_all = l1_all + mag;
                        l1_kept = l1_kept + (((nib >> j) & 1u) ? mag : 0.0f);
                    }
                }
            }
            const uint32_t word = or_reduce_8lanes(nib << ((lane & 7) * 4));
            if ((lane & 7) == 0) __builtin_amdgcn_raw_buffer_store_b32(word, b.mask, (off >> 5) * 4, 0, kAuxStore);
            if constexpr (kStats) {
                // spans are whole mask words, so the first lane of a word inside the span sees all 32 of its entries
                // (lanes past the end hold zeros, of which the first N of a group would count as kept)
                if (c.stats_slot && (lane & 7) == 0 && off < len) {
                    flips_prev += __popc(word ^ cur.word);
                    flips_init += __popc(word ^ cur.initial);
                }
            }
        } else {
            nib = (cur.word >> (off & 31)) & 0xFu;
        }
        if constexpr (SCALED) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (want_gA) acc = __builtin_fmaf(g[j], w[j], acc);     // dL/dA term, incoming w
                g[j] = A * g[j];                                         // chain rule of Eq. 12
            }
        }
        if constexpr (is_probe(EXTRA)) {
            // bandwidth probe: every loaded value is used and every stream rewritten, with next to no arithmetic
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                mu[j] = 0.5f * mu[j] + g[j];
                v[j] = 0.5f * v[j] + (((nib >> j) & 1u) ? g[j] : mu[j]);
                w[j] = 0.5f * w[j] + v[j];
            }
        } else {
            adams_entries4<rule_of(EXTRA), can_emit(EXTRA)>(w, g, mu, v, nib, off < len, a.s);
        }
        __builtin_amdgcn_raw_buffer_store_b128(pack4(w), b.w, off * 4, 0, kAuxStore);
        if constexpr (kMu16 && is_probe(EXTRA)) {
            const vu2_t h = {(__float_as_uint(mu[0]) >> 16) | (__float_as_uint(mu[1]) & 0xffff0000u),
                             (__float_as_uint(mu[2]) >> 16) | (__float_as_uint(mu[3]) & 0xffff0000u)};
            __builtin_amdgcn_raw_buffer_store_b64(h, b.m, off * 2, 0, kAuxStore);
        } else if constexpr (kMu16) {       // rounded to nearest even for the store only: v and w above used the unrounded value
            const vu2_t h = {f32x2_to_bf16_rne(mu[0], mu[1]), f32x2_to_bf16_rne(mu[2], mu[3])};
            __builtin_amdgcn_raw_buffer_store_b64(h, b.m, off * 2, 0, kAuxStore);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(pack4(mu), b.m, off * 4, 0, kAuxStore);
        }
        if constexpr (kV16 && is_probe(EXTRA)) {
            const vu2_t h = {(__float_as_uint(v[0]) >> 16) | (__float_as_uint(v[1]) & 0xffff0000u),
                             (__float_as_uint(v[2]) >> 16) | (__float_as_uint(v[3]) & 0xffff0000u)};
            __builtin_amdgcn_raw_buffer_store_b64(h, b.v, off * 2, 0, kAuxStore);
        } else if constexpr (kV16) {
            // rounded stochastically for the store only, with the bits of index row * cols + col: spans begin on
            // multiples of 32 entries and off is a multiple of 4, so adding the entry number to the low half carries nothing
            const uint64_t first = (uint64_t)c.dense_begin + (uint32_t)off;
            const uint32_t lo = (uint32_t)first, hi_term = (uint32_t)(first >> 32) * 0x9e3779b9u;
            uint32_t h[4], r16[4];
            bool finite = true;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                r16[j] = sr_bits(a.s.sr_key, lo + (uint32_t)j, hi_term);
                finite = finite && __builtin_fabsf(v[j]) < __builtin_inff();
            }
            // Infinities and NaN go through round-to-nearest; whether a wavefront holds any is decided once (a second
            // moment is finite unless the step has already overflowed), which keeps that conversion out of the usual path.
            if (__any(!finite)) {
#pragma unroll
                for (int j = 0; j < 4; ++j) h[j] = f32_to_bf16_sr(v[j], r16[j]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) h[j] = (__float_as_uint(v[j]) + r16[j]) >> 16;
            }
            const vu2_t packed = {h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
            __builtin_amdgcn_raw_buffer_store_b64(packed, b.v, off * 2, 0, kAuxStore);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(pack4(v), b.v, off * 4, 0, kAuxStore);
        }
        if constexpr (can_emit(EXTRA)) {
            if (c.emit) {      // the weights the next forward pass multiplies with: bf16(A * w_new), Eq. 12
                vu2_t h;
                h.x = f32x2_to_bf16_rne(c.copy_A * w[0], c.copy_A * w[1]);
                h.y = f32x2_to_bf16_rne(c.copy_A * w[2], c.copy_A * w[3]);
                __builtin_amdgcn_raw_buffer_store_b64(h, c.copy, off * 2, 0, kAuxStore);
            }
        }

        off += stride;
        if constexpr (kPrefetch) {
            cur = nxt;
        } else {
            if (base + stride >= len) break;      // uniform: the usual case, one chunk per wavefront
            chunk_load<BF16, (!REFRESH || can_count(EXTRA)), kStats, kMu16, kV16>(cur, b, off);
        }
    }

    bool synced = false;      // whether a workgroup barrier has been passed since the statistics went to LDS
    if constexpr (kStats) {
        if (c.stats_slot) {      // uniform over the workgroup: every wavefront leaves its sums in LDS
            // 32-bit counts cannot overflow: all the spans of a workgroup together hold fewer than 2^28 entries
            flips_prev = wave_sum_u32(flips_prev);
            flips_init = wave_sum_u32(flips_init);
            l1_kept = wave_sum_fixed_order(l1_kept);
            l1_all = wave_sum_fixed_order(l1_all);
            if (lane == 0) {
                stats_shared->flips_prev[wave] = flips_prev;
                stats_shared->flips_init[wave] = flips_init;
                stats_shared->l1_kept[wave] = l1_kept;
                stats_shared->l1_all[wave] = l1_all;
            }
        }
    }
    if constexpr (SCALED) {
        if (want_gA) {   // uniform over the workgroup
            const float wave_total = wave_sum_fixed_order(acc);
            if (P == 1) {
                if (lane == 0 && len > 0) c.scale_grad[c.span] = wave_total;
            } else {
                if (lane == 0) partial[wave] = wave_total;
                __syncthreads();
                synced = true;
                if (lane == 0 && c.sub == 0 && len > 0) {
                    float sum = partial[wave];
                    for (int p = 1; p < P; ++p) sum = sum + partial[wave + p];
                    c.scale_grad[c.span] = sum;
                }
            }
        }
    }
    if constexpr (kStats) {
        if (c.stats_slot) {      // one slot per workgroup, the wavefronts' sums added in wavefront order
            if (!synced) __syncthreads();
            if (threadIdx.x == 0) {
                StatsPartial out{0, 0, 0.0f, 0.0f};
                for (int k = 0; k < (int)(blockDim.x / kWave); ++k) {
                    out.flips_prev += stats_shared->flips_prev[k];
                    out.flips_init += stats_shared->flips_init[k];
                    out.l1_kept = k == 0 ? stats_shared->l1_kept[0] : out.l1_kept + stats_shared->l1_kept[k];
                    out.l1_all = k == 0 ? stats_shared->l1_all[0] : out.l1_all + stats_shared->l1_all[k];
                }
                *c.stats_slot = out;
            }
        }
    }
}

// One workgroup per share of a matrix.  SPLIT: the spans are
// pieces of row segments (Eq. 12) too long for one workgroup of short-lived wavefronts; each
// workgroup leaves the dL/dA sum of its piece in a[.].piece_sums and sum_piece_sums adds them up.
// EXTRA: the kernel flavour (above); the plain ones (0) carry no code but Algorithm 1's.
template <int M, bool BF16, bool REFRESH, bool SCALED, bool SPLIT = false, int EXTRA = 0>
__global__ __launch_bounds__(kMaxBlockThreads) void adams_step_vec(const SpanArgs a)
{
    __shared__ float partial[kMaxBlockWaves];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);   // wave-uniform, in a scalar register
    SpanCtx c;
    span_open<BF16, SCALED, SPLIT, EXTRA>(a, blockIdx.y, blockIdx.x, wave, c);
    Chunk<BF16> first;
    chunk_load<BF16, (!REFRESH || can_count(EXTRA)), (REFRESH && can_count(EXTRA)), mu_is_bf16(EXTRA), v_is_bf16(EXTRA)>(first, c.b, first_offset(c, lane));
    if constexpr (REFRESH && can_count(EXTRA)) {
        __shared__ StatsShared stats_shared;
        span_run<M, BF16, REFRESH, SCALED, EXTRA>(a, c, first, lane, wave, partial, &stats_shared);
    } else {
        span_run<M, BF16, REFRESH, SCALED, EXTRA>(a, c, first, lane, wave, partial);
    }
}

// Second half of a split plan: dL/dA of a row segment = its pieces' sums, added in column order.
// One launch serves up to kMaxPieceJobs matrices (blockIdx.y), their descriptors passed by value.
struct PieceJob {
    const float *piece_sums;
    float *scale_grad;
    int64_t segments;
    int pieces_per_segment;
};

constexpr int kMaxPieceJobs = 32;

struct PieceJobs {
    PieceJob job[kMaxPieceJobs];
};

__global__ __launch_bounds__(kBlockThreads) void sum_piece_sums(const PieceJobs jobs)
{
    const PieceJob &j = jobs.job[blockIdx.y];
    const int64_t seg = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (seg >= j.segments) return;
    const float *p = j.piece_sums + seg * j.pieces_per_segment;
    float total = p[0];
    for (int k = 1; k < j.pieces_per_segment; ++k) total = total + p[k];
    j.scale_grad[seg] = total;
}

// dL/dA alone, with exactly the traversal and summation order of adams_step_vec; like it, a launch
// covers up to kMaxFused matrices of one shape (matrix blockIdx.y).
struct ScaleGradSet {
    const float *w;
    const void *grad;
    float *scale_grad;
};
struct ScaleGradArgs {
    ScaleGradSet set[kMaxFused];
    SpanGeom geom;
};

template <bool BF16>
__global__ __launch_bounds__(kMaxBlockThreads) void scale_grad_vec(const ScaleGradArgs a)
{
    __shared__ float partial[kMaxBlockWaves];
    const SpanGeom &geom = a.geom;
    const float *w = a.set[blockIdx.y].w;
    const void *grad = a.set[blockIdx.y].grad;
    float *scale_grad = a.set[blockIdx.y].scale_grad;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int P = geom.waves_per_span;
    const SpanSlot slot = span_slot(geom, blockIdx.x, wave, blockDim.x / kWave);
    const int64_t span = slot.span;
    const int sub = slot.sub;
    const SpanOrigin o = span_origin(geom, span);
    const int len = o.len;
    __amdgpu_buffer_rsrc_t rw = span_resource(w + o.state_begin, len * 4), rg;
    if constexpr (BF16) rg = span_resource(static_cast<const uint16_t *>(grad) + o.dense_begin, len * 2);
    else rg = span_resource(static_cast<const float *>(grad) + o.dense_begin, len * 4);
    float acc = 0.0f;
    for (int base = sub * kChunk; base < len; base += P * kChunk) {
        const int off = base + lane * kLaneElems;
        float wv[4], g[4];
        unpack4(__builtin_amdgcn_raw_buffer_load_b128(rw, off * 4, 0, kAuxLoad), wv);
        if constexpr (BF16) {
            const vu2_t t = __builtin_amdgcn_raw_buffer_load_b64(rg, off * 2, 0, kAuxLoad);
            g[0] = bf16_lo(t.x); g[1] = bf16_hi(t.x); g[2] = bf16_lo(t.y); g[3] = bf16_hi(t.y);
        } else {
            unpack4(__builtin_amdgcn_raw_buffer_load_b128(rg, off * 4, 0, kAuxLoad), g);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = __builtin_fmaf(g[j], wv[j], acc);
    }
    const float wave_total = wave_sum_fixed_order(acc);
    if (P == 1) {
        if (lane == 0 && len > 0) scale_grad[span] = wave_total;
    } else {
        if (lane == 0) partial[wave] = wave_total;
        __syncthreads();
        if (lane == 0 && sub == 0 && len > 0) {
            float t = partial[wave];
            for (int p = 1; p < P; ++p) t = t + partial[wave + p];
            scale_grad[span] = t;
        }
    }
}

// ---- any shape with cols % M == 0: one thread per 64 consecutive columns of a row -----------
struct UnitArgs {
    float *w;
    const void *grad;
    float *m;
    float *v;
    uint32_t *mask;
    const float *scale;
    int64_t rows, cols, ld;
    int n_segments;
    int refresh;
    StepScalars s;
    uint16_t *compute_copy;     // bf16 [rows, cols] or NULL
    const float *copy_scale;    // [rows, n_segments] or NULL
    int64_t m_ld;               // > 0: m is bf16 with this row stride (in its own entries); 0: fp32 like w and v
    int v_bf16;                 // 1: v is bf16 too, laid out like m, stored with stochastic rounding
};

template <bool BF16>
__device__ __forceinline__ float load_grad1(const void *grad, int64_t idx)
{
    if constexpr (BF16) return bf16_to_f32(static_cast<const uint16_t *>(grad)[idx]);
    else return static_cast<const float *>(grad)[idx];
}

template <int M, bool BF16>
__global__ __launch_bounds__(kBlockThreads) void adams_step_unit(const UnitArgs a)
{
    const int64_t units_per_row = (a.cols + 63) / 64;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= a.rows * units_per_row) return;
    const int64_t r = tid / units_per_row, c0 = (tid % units_per_row) * 64;
    const int64_t words_per_row = (a.cols + 31) / 32;
    const int64_t seg_len = a.n_segments > 0 ? a.cols / a.n_segments : a.cols;
    for (int half = 0; half < 2; ++half) {
        const int64_t cb = c0 + half * 32;
        if (cb >= a.cols) break;
        const int64_t ce = (cb + 32 < a.cols) ? cb + 32 : a.cols;
        uint32_t *word_ptr = a.mask + r * words_per_row + cb / 32;
        uint32_t word = a.refresh ? 0u : *word_ptr;
        for (int64_t c = cb; c < ce; c += M) {
            const int64_t idx = r * a.ld + c;          // in w, mu, v
            const int64_t gidx = r * a.cols + c;       // in the gradient
            float wv[M];
#pragma unroll
            for (int j = 0; j < M; ++j) wv[j] = a.w[idx + j];
            uint32_t bits;
            if (a.refresh) {
                bits = keep_bits_group<M>(wv, a.s.n_keep);
                word |= bits << (unsigned)(c - cb);
            } else {
                bits = (word >> (unsigned)(c - cb)) & ((1u << M) - 1u);
            }
            float A = 1.0f, copy_A = 1.0f;
            if (a.scale) A = a.scale[r * a.n_segments + c / seg_len];
            if (a.copy_scale) copy_A = a.copy_scale[r * a.n_segments + c / seg_len];
#pragma unroll
            for (int j = 0; j < M; ++j) {
                float g = load_grad1<BF16>(a.grad, gidx + j);
                if (a.scale) g = A * g;
                uint16_t *m16 = reinterpret_cast<uint16_t *>(a.m) + r * a.m_ld + c + j;
                uint16_t *v16 = reinterpret_cast<uint16_t *>(a.v) + r * a.m_ld + c + j;
                float mu = a.m_ld > 0 ? bf16_to_f32(*m16) : a.m[idx + j];
                float vv = a.v_bf16 ? bf16_to_f32(*v16) : a.v[idx + j];
                adams_entry(wv[j], g, mu, vv, (bits >> j) & 1u, a.s);
                a.w[idx + j] = wv[j];
                if (a.m_ld > 0) *m16 = (uint16_t)f32_to_bf16_rne(mu);
                else a.m[idx + j] = mu;
                if (a.v_bf16) {
                    const uint64_t entry = (uint64_t)(gidx + j);
                    *v16 = (uint16_t)f32_to_bf16_sr(vv, sr_bits(a.s.sr_key, (uint32_t)entry, (uint32_t)(entry >> 32) * 0x9e3779b9u));
                } else {
                    a.v[idx + j] = vv;
                }
                if (a.compute_copy) a.compute_copy[gidx + j] = (uint16_t)f32_to_bf16_rne(copy_A * wv[j]);
            }
        }
        if (a.refresh) *word_ptr = word;
    }
}

// dL/dA for any shape: one wavefront per row segment, lanes stride over its entries.
template <bool BF16>
__global__ __launch_bounds__(kBlockThreads) void scale_grad_rows(const float *w, const void *grad,
                                                                 float *scale_grad, int64_t rows,
                                                                 int64_t cols, int64_t ld, int n_segments)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t seg = (int64_t)blockIdx.x * kBlockWaves + threadIdx.x / kWave;
    const int64_t seg_len = cols / n_segments;
    const bool live = seg < rows * n_segments;
    float acc = 0.0f;
    if (live) {
        const int64_t r = seg / n_segments, c0 = (seg % n_segments) * seg_len;
        for (int64_t i = lane; i < seg_len; i += kWave)
            acc = __builtin_fmaf(load_grad1<BF16>(grad, r * cols + c0 + i), w[r * ld + c0 + i], acc);
    }
    const float t = wave_sum_fixed_order(acc);
    if (lane == 0 && live) scale_grad[seg] = t;
}

// Refresh statistics for shapes the vector kernels do not take: one thread per 64 columns of a row,
// run before the step (it needs the stored mask and the incoming weights); the new mask is
// worked out here a second time.  One slot per workgroup, like the vector kernels.
template <int M>
__global__ __launch_bounds__(kBlockThreads) void refresh_stats_unit(const float *w, const uint32_t *mask,
                                                                    const uint32_t *initial_mask, int64_t rows, int64_t cols,
                                                                    int64_t ld, int n_keep, StatsPartial *partials)
{
    __shared__ StatsShared sh;
    const int64_t units_per_row = (cols + 63) / 64;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t flips_prev = 0, flips_init = 0;
    float l1_kept = 0.0f, l1_all = 0.0f;
    if (tid < rows * units_per_row) {
        const int64_t r = tid / units_per_row, c0 = (tid % units_per_row) * 64;
        const int64_t words_per_row = (cols + 31) / 32;
        for (int half = 0; half < 2; ++half) {
            const int64_t cb = c0 + half * 32;
            if (cb >= cols) break;
            const int64_t ce = (cb + 32 < cols) ? cb + 32 : cols;
            const int64_t word_index = r * words_per_row + cb / 32;
            uint32_t fresh = 0;
            for (int64_t c = cb; c < ce; c += M) {
                float wv[M];
#pragma unroll
                for (int j = 0; j < M; ++j) wv[j] = w[r * ld + c + j];
                const uint32_t bits = keep_bits_group<M>(wv, n_keep);
                fresh |= bits << (unsigned)(c - cb);
#pragma unroll
                for (int j = 0; j < M; ++j) {
                    const float mag = __builtin_fabsf(wv[j]);
                    l1_all = l1_all + mag;
                    l1_kept = l1_kept + (((bits >> j) & 1u) ? mag : 0.0f);
                }
            }
            flips_prev += __popc(fresh ^ mask[word_index]);
            if (initial_mask) flips_init += __popc(fresh ^ initial_mask[word_index]);
        }
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    flips_prev = wave_sum_u32(flips_prev);
    flips_init = wave_sum_u32(flips_init);
    l1_kept = wave_sum_fixed_order(l1_kept);
    l1_all = wave_sum_fixed_order(l1_all);
    if (lane == 0) { sh.flips_prev[wave] = flips_prev; sh.flips_init[wave] = flips_init; sh.l1_kept[wave] = l1_kept; sh.l1_all[wave] = l1_all; }
    __syncthreads();
    if (threadIdx.x == 0) {
        StatsPartial out{flips_prev, flips_init, l1_kept, l1_all};
        for (int k = 1; k < kBlockWaves; ++k) {
            out.flips_prev += sh.flips_prev[k];
            out.flips_init += sh.flips_init[k];
            out.l1_kept = out.l1_kept + sh.l1_kept[k];
            out.l1_all = out.l1_all + sh.l1_all[k];
        }
        partials[blockIdx.x] = out;
    }
}

// The statistics of given masks (no step): the row-block form of the selection and pack kernels, one slot per
// workgroup.  w with the non-temporal hint; a mask word is read by the 8 lanes that hold its 32 entries.
struct MaskStatsSet {
    const float *w;
    const uint32_t *mask;
    const uint32_t *other;      // or NULL
    StatsPartial *partials;     // one slot per workgroup of this matrix
};

struct MaskStatsArgs {
    MaskStatsSet set[kMaxListed];
    RowsGeom geom;
};

__device__ __forceinline__ void stats_block_sum(StatsShared &sh, uint32_t flips, float l1_kept, float l1_all, StatsPartial *slot)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    flips = wave_sum_u32(flips);
    l1_kept = wave_sum_fixed_order(l1_kept);
    l1_all = wave_sum_fixed_order(l1_all);
    if (lane == 0) { sh.flips_prev[wave] = flips; sh.l1_kept[wave] = l1_kept; sh.l1_all[wave] = l1_all; }
    __syncthreads();
    if (threadIdx.x == 0) {
        StatsPartial out{flips, 0u, l1_kept, l1_all};
        for (int k = 1; k < (int)(blockDim.x / kWave); ++k) {
            out.flips_prev += sh.flips_prev[k];
            out.l1_kept = out.l1_kept + sh.l1_kept[k];
            out.l1_all = out.l1_all + sh.l1_all[k];
        }
        *slot = out;
    }
}

template <bool SAME_ROW>
__global__ __launch_bounds__(kBlockThreads) void mask_stats_rows(const MaskStatsArgs a)
{
    __shared__ StatsShared sh;
    const MaskStatsSet t = a.set[blockIdx.y];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int cols = a.geom.cols;
    vf4_t raw[kLoads];
    uint32_t word[kLoads], diff[kLoads];
    int col[kLoads];
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const RowsPiece piece = rows_piece<SAME_ROW>(a.geom, blockIdx.x, wave, k);
        col[k] = piece.col + lane * 4;
        raw[k] = vf4_t{0.0f, 0.0f, 0.0f, 0.0f};
        word[k] = diff[k] = 0;
        if (col[k] < cols) {
            const int64_t at = (int64_t)piece.row * (cols >> 5) + (col[k] >> 5);
            raw[k] = __builtin_nontemporal_load(reinterpret_cast<const vf4_t *>(t.w + (int64_t)piece.row * a.geom.ld + col[k]));
            word[k] = __builtin_nontemporal_load(t.mask + at);
            if (t.other) diff[k] = word[k] ^ __builtin_nontemporal_load(t.other + at);
        }
    }
    uint32_t flips = 0;
    float l1_kept = 0.0f, l1_all = 0.0f;
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const uint32_t nib = (word[k] >> (col[k] & 31)) & 0xFu;      // lanes past the end: zeros, nothing counted
        const float x[4] = {raw[k].x, raw[k].y, raw[k].z, raw[k].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float mag = __builtin_fabsf(x[j]);
            l1_all = l1_all + mag;
            l1_kept = l1_kept + (((nib >> j) & 1u) ? mag : 0.0f);
        }
        if ((lane & 7) == 0) flips += __popc(diff[k]);      // one lane per mask word
    }
    stats_block_sum(sh, flips, l1_kept, l1_all, t.partials + blockIdx.x);
}

// Any shape: one thread per mask word, the row padded to whole words.
__global__ __launch_bounds__(kBlockThreads) void mask_stats_words(const float *w, const uint32_t *mask, const uint32_t *other,
                                                                  int64_t rows, int64_t cols, int64_t ld, StatsPartial *partials)
{
    __shared__ StatsShared sh;
    const int64_t words_per_row = (cols + 31) / 32;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t flips = 0;
    float l1_kept = 0.0f, l1_all = 0.0f;
    if (t < rows * words_per_row) {
        const int64_t r = t / words_per_row, cb = (t % words_per_row) * 32;
        const int64_t ce = (cb + 32 < cols) ? cb + 32 : cols;
        const uint32_t word = mask[t];
        if (other) flips = __popc(word ^ other[t]);
        for (int64_t c = cb; c < ce; ++c) {
            const float mag = __builtin_fabsf(w[r * ld + c]);
            l1_all = l1_all + mag;
            l1_kept = l1_kept + (((word >> (unsigned)(c - cb)) & 1u) ? mag : 0.0f);
        }
    }
    stats_block_sum(sh, flips, l1_kept, l1_all, partials + blockIdx.x);
}

// Second half of the refresh statistics: the slots of a matrix added up, counts exactly, norms in
// double, always in the same order (each thread a strided share, then a tree), so the result is
// reproducible.  One workgroup per matrix, up to kMaxStatsJobs matrices per launch.
struct StatsJob {
    const StatsPartial *partials;
    int64_t slots;
    cast_refresh_stats *out;
    int has_initial;
};

constexpr int kMaxStatsJobs = 32;

struct StatsJobs {
    StatsJob job[kMaxStatsJobs];
};

__global__ __launch_bounds__(kMaxBlockThreads) void sum_refresh_stats(const StatsJobs jobs)
{
    __shared__ unsigned long long sh_prev[kMaxBlockThreads], sh_init[kMaxBlockThreads];
    __shared__ double sh_kept[kMaxBlockThreads], sh_all[kMaxBlockThreads];
    const StatsJob &j = jobs.job[blockIdx.x];
    unsigned long long prev = 0, init = 0;
    double kept = 0.0, all = 0.0;
    for (int64_t i = threadIdx.x; i < j.slots; i += kMaxBlockThreads) {
        const StatsPartial p = j.partials[i];
        prev += p.flips_prev;
        init += p.flips_init;
        kept += (double)p.l1_kept;
        all += (double)p.l1_all;
    }
    sh_prev[threadIdx.x] = prev; sh_init[threadIdx.x] = init; sh_kept[threadIdx.x] = kept; sh_all[threadIdx.x] = all;
    __syncthreads();
    for (int half = kMaxBlockThreads / 2; half > 0; half >>= 1) {
        if ((int)threadIdx.x < half) {
            sh_prev[threadIdx.x] += sh_prev[threadIdx.x + half];
            sh_init[threadIdx.x] += sh_init[threadIdx.x + half];
            sh_kept[threadIdx.x] += sh_kept[threadIdx.x + half];
            sh_all[threadIdx.x] += sh_all[threadIdx.x + half];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        j.out->flips_prev = sh_prev[0];
        j.out->flips_init = j.has_initial ? sh_init[0] : 0ull;
        j.out->l1_kept = sh_kept[0];
        j.out->l1_all = sh_all[0];
    }
}

}  // namespace cast
