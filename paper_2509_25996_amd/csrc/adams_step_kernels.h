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

// The buffers of one matrix.  A dispatcher-dealt launch carries up to kMaxFused sets in its
// arguments (workgroups with blockIdx.y = k step matrix k); the work queue reads the set of a
// matrix from a table in device memory.
struct TensorPtrs {
    float *w;
    const void *grad;
    float *m;             // bf16 values instead when the first moment is kept in bf16 (flavour 3)
    float *v;
    uint32_t *mask;
    const float *scale;
    float *scale_grad;
    float *piece_sums;    // split plans: one partial dL/dA sum per piece, else unused
    // Flavours that gather refresh statistics only (never read by the work queue):
    struct StatsPartial *stats_partials;   // one slot per workgroup of the launch, or NULL
    const uint32_t *initial_mask;          // the mask flips_init counts against, or NULL
    // Flavours that can write the bf16 copy of the updated weights for the next forward pass
    // (Eq. 12 applied: copy_scale[r, s] * w_new, or w_new itself when copy_scale is NULL), or NULL:
    uint16_t *compute_copy;
    const float *copy_scale;
};                        // 96 bytes per entry; the work queue reads the first 64

// What one workgroup contributes to the mask-learning statistics of a refresh step
// (appendix "Mask Learning"): changed mask bits against the stored and the initial mask, and
// the L1 norms of the kept and of all incoming weights.
struct StatsPartial {
    uint32_t flips_prev, flips_init;
    float l1_kept, l1_all;
};

// The table is addressed through the constant address space: its entries do not change while a
// kernel runs, and only then are they read with scalar loads, straight into the scalar registers
// where buffer resources have to live.
typedef const TensorPtrs __attribute__((address_space(4))) *ConstTable;

constexpr int kMaxFused = 16;     // matrices of equal shape that one dispatcher-dealt launch can step (gridDim.y)

struct SpanArgs {
    TensorPtrs set[kMaxFused];   // the buffer sets of a dispatcher-dealt launch: matrix blockIdx.y
    ConstTable table;     // the buffer sets of a list launch (work queue)
    SpanGeom geom;
    StepScalars s;
};

static ConstTable as_const_table(const void *device_ptr)
{
    return (ConstTable)(uintptr_t)device_ptr;
}

// Kernel flavours (template argument EXTRA) = what the kernel can do besides Algorithm 1, in the low four bits,
// plus the comparison rule it applies (Eq. 9, Eq. 10, frozen masked entries; 0: none), fixed at compile time,
// shifted left by four.  The low bits: 0 plain; 1 can also write the bf16 compute copy and gather refresh
// statistics; 3 plain with the first moment kept in bf16 (CAST_FLAG_MU_BF16); 4 plain that can gather refresh
// statistics (refresh steps only: without the code for the compute copy it runs close to flavour 0); 5 the
// first moment in bf16, with the abilities of 1; 6 both moments in bf16, the second one rounded stochastically
// (CAST_FLAG_V_BF16); 7 the same with the abilities of 1.  The rules combine with 0 and 1.
constexpr int kEmitAndCount = 1;
constexpr int kMuBf16 = 3;
constexpr int kStatsOnly = 4;
constexpr int kMuBf16Emit = 5;
constexpr int kBothBf16 = 6;
constexpr int kBothBf16Emit = 7;
constexpr int abilities(int extra) { return extra & 15; }
constexpr int rule_of(int extra) { return extra >> 4; }      // kRuleAdamwL1, kRuleAdamL1, kRuleMaskedFrozen or 0
constexpr int with_rule(int extra, int rule) { return extra | (rule << 4); }
constexpr bool can_emit(int extra) { return abilities(extra) == kEmitAndCount || abilities(extra) == kMuBf16Emit || abilities(extra) == kBothBf16Emit; }
constexpr bool can_count(int extra) { return can_emit(extra) || abilities(extra) == kStatsOnly; }
constexpr bool v_is_bf16(int extra) { return abilities(extra) == kBothBf16 || abilities(extra) == kBothBf16Emit; }
constexpr bool mu_is_bf16(int extra) { return abilities(extra) == kMuBf16 || abilities(extra) == kMuBf16Emit || v_is_bf16(extra); }

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

// `matrix` selects the buffer set (entry of the table of a list call), `block` the workgroup's
// share of that matrix: block_waves / waves_per_span consecutive spans.
template <bool BF16, bool SCALED, bool FROM_TABLE, bool SPLIT = false, int EXTRA = 0>
__device__ __forceinline__ void span_open(const SpanArgs &a, uint32_t matrix, int64_t block, int wave, SpanCtx &c)
{
    // The buffer set of this launch, or of one matrix of a list.  The table is read through the
    // constant address space so that the (wave-uniform) loads are scalar loads and the pointers
    // arrive in scalar registers, where buffer resources have to live.
    TensorPtrs t;
    if constexpr (FROM_TABLE) {
        // explicit scalar loads of the first 64 bytes of the entry (two 8-dword reads)
        typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
        const uint64_t entry = uniform_u64((uint64_t)(uintptr_t)a.table + (uint64_t)matrix * sizeof(TensorPtrs));
        u32x8 lo, hi;
        asm volatile("s_load_dwordx8 %0, %2, 0x0\n\ts_load_dwordx8 %1, %2, 0x20\n\ts_waitcnt lgkmcnt(0)"
                     : "=&s"(lo), "=&s"(hi) : "s"(entry) : "memory");
        auto ptr = [](uint32_t l, uint32_t h) { return (uintptr_t)(((uint64_t)h << 32) | l); };
        t.w = (float *)ptr(lo[0], lo[1]);
        t.grad = (const void *)ptr(lo[2], lo[3]);
        t.m = (float *)ptr(lo[4], lo[5]);
        t.v = (float *)ptr(lo[6], lo[7]);
        t.mask = (uint32_t *)ptr(hi[0], hi[1]);
        t.scale = (const float *)ptr(hi[2], hi[3]);
        t.scale_grad = (float *)ptr(hi[4], hi[5]);
        t.piece_sums = (float *)ptr(hi[6], hi[7]);
        t.stats_partials = nullptr;
        t.initial_mask = nullptr;
        t.compute_copy = nullptr;
        t.copy_scale = nullptr;
    } else {
        t = a.set[matrix];     // a scalar load from the kernel arguments at a wave-uniform offset
    }
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
// the arithmetic.  Control flow is uniform across the wavefront: lanes past the end of the span
// carry zeros through the arithmetic and the buffer range check voids their stores, so the
// cross-lane steps (M = 8 key exchange, mask word assembly, the dL/dA butterfly) always see
// all 64 lanes.
// LDS through which the wavefronts of a workgroup combine their refresh statistics.
struct StatsShared {
    uint32_t flips[kMaxBlockWaves];       // flips against the stored mask | flips against the initial mask << 16
    float l1_kept[kMaxBlockWaves], l1_all[kMaxBlockWaves];
};

template <int M, bool BF16, bool REFRESH, bool SCALED, int EXTRA = 0>
__device__ __forceinline__ void span_run(const SpanArgs &a, const SpanCtx &c, Chunk<BF16> cur, int lane, int wave,
                                         float *partial, StatsShared *stats_shared = nullptr)
{
    constexpr bool kStats = REFRESH && can_count(EXTRA);      // refresh statistics are gathered if c.stats_slot says so
    constexpr bool kMu16 = mu_is_bf16(EXTRA);
    constexpr bool kV16 = v_is_bf16(EXTRA);
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
        Chunk<BF16> nxt;
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
        adams_entries4<rule_of(EXTRA), can_emit(EXTRA)>(w, g, mu, v, nib, off < len, a.s);
        __builtin_amdgcn_raw_buffer_store_b128(pack4(w), b.w, off * 4, 0, kAuxStore);
        if constexpr (kMu16) {       // rounded to nearest even for the store only: v and w above used the unrounded value
            const vu2_t h = {f32x2_to_bf16_rne(mu[0], mu[1]), f32x2_to_bf16_rne(mu[2], mu[3])};
            __builtin_amdgcn_raw_buffer_store_b64(h, b.m, off * 2, 0, kAuxStore);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(pack4(mu), b.m, off * 4, 0, kAuxStore);
        }
        if constexpr (kV16) {
            // rounded stochastically for the store only, with the bits of index row * cols + col: spans begin on
            // multiples of 32 entries and off is a multiple of 4, so adding the entry number to the low half carries nothing
            const uint64_t first = (uint64_t)c.dense_begin + (uint32_t)off;
            const uint32_t lo = (uint32_t)first, hi_term = (uint32_t)(first >> 32) * 0x9e3779b9u;
            uint32_t h[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) h[j] = f32_to_bf16_sr(v[j], sr_bits(a.s.sr_key, lo + (uint32_t)j, hi_term));
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

        cur = nxt;
        off += stride;
    }

    bool synced = false;      // whether a workgroup barrier has been passed since the statistics went to LDS
    if constexpr (kStats) {
        if (c.stats_slot) {      // uniform over the workgroup: every wavefront leaves its sums in LDS
            const uint32_t flips = wave_sum_u32(flips_prev | (flips_init << 16));     // at most 64 * 4 * 64 each
            l1_kept = wave_sum_fixed_order(l1_kept);
            l1_all = wave_sum_fixed_order(l1_all);
            if (lane == 0) {
                stats_shared->flips[wave] = flips;
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
                uint32_t flips = 0;
                StatsPartial out{0, 0, 0.0f, 0.0f};
                for (int k = 0; k < (int)(blockDim.x / kWave); ++k) {
                    flips = stats_shared->flips[k];
                    out.flips_prev += flips & 0xFFFFu;
                    out.flips_init += flips >> 16;
                    out.l1_kept = k == 0 ? stats_shared->l1_kept[0] : out.l1_kept + stats_shared->l1_kept[k];
                    out.l1_all = k == 0 ? stats_shared->l1_all[0] : out.l1_all + stats_shared->l1_all[k];
                }
                *c.stats_slot = out;
            }
        }
    }
}

// One matrix, one workgroup per share, dealt by the hardware dispatcher.  SPLIT: the spans are
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
    span_open<BF16, SCALED, false, SPLIT, EXTRA>(a, blockIdx.y, blockIdx.x, wave, c);
    Chunk<BF16> first;
    chunk_load<BF16, (!REFRESH || can_count(EXTRA)), (REFRESH && can_count(EXTRA)), mu_is_bf16(EXTRA), v_is_bf16(EXTRA)>(first, c.b, first_offset(c, lane));
    if constexpr (REFRESH && can_count(EXTRA)) {
        __shared__ StatsShared stats_shared;
        span_run<M, BF16, REFRESH, SCALED, EXTRA>(a, c, first, lane, wave, partial, &stats_shared);
    } else {
        span_run<M, BF16, REFRESH, SCALED, EXTRA>(a, c, first, lane, wave, partial);
    }
}

// Work queue: a fixed set of resident workgroups draws runs of consecutive shares, in order, from
// a ticket counter in device memory (zero at launch).  Whatever the relative speed of the compute
// units and of the 8 XCDs, the shares in flight are always the most recently drawn ones, so every
// array is walked front to back through one narrow, steadily advancing window, which is what HBM
// serves fastest, and no wavefront is launched after the first.  One counter serves about 60
// million tickets a second, so a ticket stands for 2^log2_run shares.  The loop is
// software-pipelined: while a workgroup works on one share, the first chunk of its next share is
// already on its way and the ticket after the current one has been asked for.  Every workgroup
// leaves when its next share lies past the end; nobody waits for anybody.
struct QueueArgs {
    unsigned long long *ticket_counter;
    uint32_t tasks;                  // shares in this launch (all matrices)
    uint32_t blocks_per_matrix;
    FastDivU32 div_blocks_per_matrix;
    int log2_run;                    // shares per ticket = 1 << log2_run
};

// One chunk of 256 entries of the plain flavour (no compute copy, no statistics, AdamS rule family):
// what span_run does per iteration, for the work queue, which runs its own pipeline.
template <int M, bool BF16, bool REFRESH, bool SCALED>
__device__ __forceinline__ void chunk_step(const SpanArgs &a, const SpanCtx &c, const Chunk<BF16> &cur, int lane, int off,
                                           bool want_gA, float &acc)
{
    const SpanBuffers &b = c.b;
    float w[4], g[4], mu[4], v[4];
    unpack4(cur.w, w);
    unpack4(cur.m, mu);
    unpack4(cur.v, v);
    if constexpr (BF16) {
        g[0] = bf16_lo(cur.g.x); g[1] = bf16_hi(cur.g.x); g[2] = bf16_lo(cur.g.y); g[3] = bf16_hi(cur.g.y);
    } else {
        unpack4(cur.g, g);
    }
    uint32_t nib;
    if constexpr (REFRESH) {
        nib = keep_nibble<M>(w, a.s.n_keep, lane);
        const uint32_t word = or_reduce_8lanes(nib << ((lane & 7) * 4));
        if ((lane & 7) == 0) __builtin_amdgcn_raw_buffer_store_b32(word, b.mask, (off >> 5) * 4, 0, kAuxStore);
    } else {
        nib = (cur.word >> (off & 31)) & 0xFu;
    }
    if constexpr (SCALED) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (want_gA) acc = __builtin_fmaf(g[j], w[j], acc);
            g[j] = c.A * g[j];
        }
    }
    adams_entries4<0, false>(w, g, mu, v, nib, off < c.len, a.s);
    __builtin_amdgcn_raw_buffer_store_b128(pack4(w), b.w, off * 4, 0, kAuxStore);
    __builtin_amdgcn_raw_buffer_store_b128(pack4(mu), b.m, off * 4, 0, kAuxStore);
    __builtin_amdgcn_raw_buffer_store_b128(pack4(v), b.v, off * 4, 0, kAuxStore);
}

// Every wavefront has one chunk of a share (the host sends only such plans here): while it works on
// it, its chunk of the next share is on its way.  One barrier per share publishes the ticket and
// hands the wavefronts' dL/dA sums of the share before to the wavefront that adds them up (two sets
// of LDS slots, used in turn).  SPLIT: as in adams_step_vec.
template <int M, bool BF16, bool REFRESH, bool SCALED, bool SPLIT = false>
__global__ __launch_bounds__(kMaxBlockThreads) void adams_step_vec_queue(const SpanArgs a, const QueueArgs q)
{
    __shared__ float partial[2][kMaxBlockWaves];
    __shared__ unsigned long long drawn[2];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t run_mask = (1u << q.log2_run) - 1u;
    const int P = a.geom.waves_per_span;
    unsigned long long pending = 0;

    if (threadIdx.x == 0) drawn[0] = atomicAdd(q.ticket_counter, 1ull);
    __syncthreads();
    const unsigned long long first_ticket = uniform_u64(drawn[0]);
    if ((first_ticket << q.log2_run) >= q.tasks) return;
    uint32_t share = (uint32_t)first_ticket << q.log2_run;      // wave-uniform
    Chunk<BF16> cur;
    {
        const uint32_t matrix = fast_div(share, q.div_blocks_per_matrix);
        SpanCtx c;
        span_open<BF16, SCALED, true, SPLIT>(a, matrix, (int64_t)(share - matrix * q.blocks_per_matrix), wave, c);
        chunk_load<BF16, !REFRESH>(cur, c.b, first_offset(c, lane));
    }
    if (threadIdx.x == 0) pending = atomicAdd(q.ticket_counter, 1ull);
    float *sum_to = nullptr;      // where this wavefront puts the dL/dA of the share before, if it is the one to add it up

    uint32_t seq = 0;             // shares this workgroup has finished
    for (;; ++seq) {
        const bool last_of_run = (seq & run_mask) == run_mask;          // wave-uniform
        const int slot = ((seq >> q.log2_run) + 1) & 1;
        if (last_of_run && threadIdx.x == 0) drawn[slot] = pending;
        __syncthreads();
        if constexpr (SCALED) {
            if (sum_to != nullptr && lane == 0) {
                const float *from = partial[(seq + 1) & 1] + wave;
                float sum = from[0];
                for (int p = 1; p < P; ++p) sum = sum + from[p];
                *sum_to = sum;
            }
        }
        unsigned long long next = (unsigned long long)share + 1;
        if (last_of_run) next = uniform_u64(drawn[slot]) << q.log2_run;
        const bool has_next = next < q.tasks;
        const uint32_t next_share = __builtin_amdgcn_readfirstlane((uint32_t)next);
        if (has_next && last_of_run && threadIdx.x == 0) pending = atomicAdd(q.ticket_counter, 1ull);
        // Scalar registers hold one span context at a time: the next share's is built only to request
        // its first chunk, and the current share's after that.
        Chunk<BF16> nxt;
        if (has_next) {
            const uint32_t matrix = fast_div(next_share, q.div_blocks_per_matrix);
            SpanCtx ahead;
            span_open<BF16, SCALED, true, SPLIT>(a, matrix, (int64_t)(next_share - matrix * q.blocks_per_matrix), wave, ahead);
            chunk_load<BF16, !REFRESH>(nxt, ahead.b, first_offset(ahead, lane));
        }
        const uint32_t matrix = fast_div(share, q.div_blocks_per_matrix);
        SpanCtx c;
        span_open<BF16, SCALED, true, SPLIT>(a, matrix, (int64_t)(share - matrix * q.blocks_per_matrix), wave, c);
        const bool want_gA = SCALED && c.scale_grad != nullptr;
        float acc = 0.0f;
        chunk_step<M, BF16, REFRESH, SCALED>(a, c, cur, lane, first_offset(c, lane), want_gA, acc);
        if constexpr (SCALED) {
            sum_to = nullptr;
            if (want_gA) {
                const float wave_total = wave_sum_fixed_order(acc);
                if (P == 1) {
                    if (lane == 0 && c.len > 0) c.scale_grad[c.span] = wave_total;
                } else {
                    if (lane == 0) partial[seq & 1][wave] = wave_total;
                    if (c.sub == 0 && c.len > 0) sum_to = c.scale_grad + c.span;
                }
            }
        }
        if (!has_next) break;
        share = next_share;
        cur = nxt;
    }
    if constexpr (SCALED) {
        __syncthreads();
        if (sum_to != nullptr && lane == 0) {      // the last share's sums
            const float *from = partial[seq & 1] + wave;
            float sum = from[0];
            for (int p = 1; p < P; ++p) sum = sum + from[p];
            *sum_to = sum;
        }
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

// dL/dA alone, with exactly the traversal and summation order of adams_step_vec.
template <bool BF16>
__global__ __launch_bounds__(kMaxBlockThreads) void scale_grad_vec(const float *w, const void *grad,
                                                                   float *scale_grad, const SpanGeom geom)
{
    __shared__ float partial[kMaxBlockWaves];
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
    __shared__ uint32_t sh_init[kBlockWaves];
    if (lane == 0) { sh.flips[wave] = flips_prev; sh_init[wave] = flips_init; sh.l1_kept[wave] = l1_kept; sh.l1_all[wave] = l1_all; }
    __syncthreads();
    if (threadIdx.x == 0) {
        StatsPartial out{flips_prev, flips_init, l1_kept, l1_all};
        for (int k = 1; k < kBlockWaves; ++k) {
            out.flips_prev += sh.flips[k];
            out.flips_init += sh_init[k];
            out.l1_kept = out.l1_kept + sh.l1_kept[k];
            out.l1_all = out.l1_all + sh.l1_all[k];
        }
        partials[blockIdx.x] = out;
    }
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
