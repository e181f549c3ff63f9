// Stand-alone measurement aid (not part of libcast, not part of the method): what the memory system of the GPU
// gives the access pattern of the AdamS step when almost nothing else happens.  Every kernel here reads and
// rewrites the streams of one step (weights, two moments, gradient, one mask bit per entry) around three
// multiply-adds per entry, in the plainest forms there are, so that the library's kernels and its own probe
// (cast_hbm_stream_probe) can be held against them.  16 matrices are visited in rotation, so that the
// 256 MB last-level cache never holds what a launch reads.
//
//   stream_skeleton [rows [cols [matrices]]]        (default 11008 4096 16; cols a multiple of 256)
//
// One line per variant: microseconds per launch and algorithmic GB/s (bytes per entry as stated in the line).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

typedef float vf4 __attribute__((ext_vector_type(4)));
typedef uint32_t vu2 __attribute__((ext_vector_type(2)));
typedef uint32_t vu4 __attribute__((ext_vector_type(4)));

template <bool NT, typename T> __device__ __forceinline__ T load(const T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename T> __device__ __forceinline__ void store(T *p, T x)
{
    if constexpr (NT) __builtin_nontemporal_store(x, p);
    else *p = x;
}

__device__ __forceinline__ vf4 widen(vu2 h)
{
    return vf4{__uint_as_float(h.x << 16), __uint_as_float(h.x & 0xffff0000u), __uint_as_float(h.y << 16), __uint_as_float(h.y & 0xffff0000u)};
}
__device__ __forceinline__ vu2 truncate(vf4 x)
{
    return vu2{(__float_as_uint(x.x) >> 16) | (__float_as_uint(x.y) & 0xffff0000u), (__float_as_uint(x.z) >> 16) | (__float_as_uint(x.w) & 0xffff0000u)};
}

// every loaded value is used and every stream rewritten
__device__ __forceinline__ void touch(vf4 &w, vf4 &m, vf4 &v, vf4 g, uint32_t nibble)
{
    float *wf = (float *)&w, *mf = (float *)&m, *vf = (float *)&v, *gf = (float *)&g;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        mf[j] = 0.5f * mf[j] + gf[j];
        vf[j] = 0.5f * vf[j] + (((nibble >> j) & 1u) ? gf[j] : mf[j]);
        wf[j] = 0.5f * wf[j] + vf[j];
    }
}

// fp32 state in rows of [cols w][cols m][cols v]; a thread owns K pieces of 4 entries, BT * 4 entries apart; a
// workgroup covers K * BT * 4 consecutive entries of one row.  GRAD32: fp32 gradients instead of bf16.
template <int K, int BT, bool NT_LOAD, bool NT_STORE, bool GRAD32>
__global__ __launch_bounds__(BT) void rmw_plain(float *state, const void *grad, const uint32_t *mask, int cols, int blocks_per_row)
{
    const int64_t row = blockIdx.x / blocks_per_row;
    const int first = (blockIdx.x % blocks_per_row) * (K * BT * 4);
    float *r = state + row * 3 * cols;
    const uint32_t *rmask = mask + row * (cols / 32);
    vf4 w[K], m[K], v[K], g[K];
    uint32_t word[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int c = first + k * BT * 4 + threadIdx.x * 4;
        if (c < cols) {
            w[k] = load<NT_LOAD>((const vf4 *)(r + c));
            m[k] = load<NT_LOAD>((const vf4 *)(r + cols + c));
            v[k] = load<NT_LOAD>((const vf4 *)(r + 2 * cols + c));
            if constexpr (GRAD32) g[k] = load<NT_LOAD>((const vf4 *)((const float *)grad + row * cols + c));
            else g[k] = widen(load<NT_LOAD>((const vu2 *)((const uint16_t *)grad + row * cols + c)));
            word[k] = load<NT_LOAD>(rmask + (c >> 5));
        }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int c = first + k * BT * 4 + threadIdx.x * 4;
        if (c < cols) {
            touch(w[k], m[k], v[k], g[k], (word[k] >> (c & 31)) & 15u);
            store<NT_STORE>((vf4 *)(r + c), w[k]);
            store<NT_STORE>((vf4 *)(r + cols + c), m[k]);
            store<NT_STORE>((vf4 *)(r + 2 * cols + c), v[k]);
        }
    }
}

// the same bytes with w, m, v interleaved in tiles of TILE entries inside a row instead of whole sub-rows
template <int TILE>
__global__ __launch_bounds__(256) void rmw_tiled(float *state, const uint16_t *grad, const uint32_t *mask, int cols, int blocks_per_row)
{
    const int64_t row = blockIdx.x / blocks_per_row;
    const int c = (blockIdx.x % blocks_per_row) * 1024 + threadIdx.x * 4;
    if (c >= cols) return;
    float *p = state + row * 3 * cols + (int64_t)(c / TILE) * (3 * TILE) + (c % TILE);
    vf4 w = load<true>((const vf4 *)p), m = load<true>((const vf4 *)(p + TILE)), v = load<true>((const vf4 *)(p + 2 * TILE));
    const vf4 g = widen(load<true>((const vu2 *)(grad + row * cols + c)));
    const uint32_t word = load<true>(mask + row * (cols / 32) + (c >> 5));
    touch(w, m, v, g, (word >> (c & 31)) & 15u);
    store<true>((vf4 *)p, w);
    store<true>((vf4 *)(p + TILE), m);
    store<true>((vf4 *)(p + 2 * TILE), v);
}

// bf16 moments: rows of [cols fp32 w][cols bf16 m][cols bf16 v] (V16, 8 * cols bytes) or [cols fp32 w][cols bf16 m]
// [cols fp32 v] (10 * cols bytes); one wavefront per 256 entries.  Options that rebuild the library's structure step
// by step: REDUCE, a sum of g * w over the workgroup through LDS (the dL/dA of Eq. 12); BUFFER, the accesses
// through buffer resources whose range is the wavefront's 256 entries; VOIDED (with BUFFER), a second set of loads
// just past that range, which the range check answers with zeros (the request for a next chunk that does not exist).
template <bool V16, int BT, bool REDUCE, bool BUFFER, bool VOIDED>
__global__ __launch_bounds__(BT) void rmw_bf16(uint8_t *state, const uint16_t *grad, const uint32_t *mask, float *sums, int cols, int blocks_per_row)
{
    __shared__ float partial[BT / 64];
    const int64_t row = blockIdx.x / blocks_per_row;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x & 63;      // wave: in a scalar register
    const int first = (blockIdx.x % blocks_per_row) * (BT * 4) + wave * 256;     // the wavefront's 256 entries
    const int len = min(256, cols - first);
    uint8_t *r = state + row * (int64_t)(V16 ? 8 : 10) * cols;
    uint8_t *pw = r + 4 * (int64_t)first, *pm = r + 4 * (int64_t)cols + 2 * (int64_t)first;
    uint8_t *pv = r + 6 * (int64_t)cols + (V16 ? 2 : 4) * (int64_t)first;
    const uint16_t *pg = grad + row * cols + first;
    const uint32_t *pk = mask + row * (cols / 32) + first / 32;
    float acc = 0.0f;
    if (len > 0) {      // uniform over the wavefront
        const int off = lane * 4;
        vf4 w, m, v, g;
        uint32_t word;
        if constexpr (BUFFER) {
            constexpr int kRaw32 = 0x00020000;
            __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(pw, 0, len * 4, kRaw32);
            __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(pm, 0, len * 2, kRaw32);
            __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(pv, 0, len * (V16 ? 2 : 4), kRaw32);
            __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(pg), 0, len * 2, kRaw32);
            __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(pk), 0, len / 8, kRaw32);
            constexpr int kNt = 2;
            const vu4 wb = __builtin_amdgcn_raw_buffer_load_b128(rw, off * 4, 0, kNt);
            m = widen(__builtin_amdgcn_raw_buffer_load_b64(rm, off * 2, 0, kNt));
            if constexpr (V16) {
                v = widen(__builtin_amdgcn_raw_buffer_load_b64(rv, off * 2, 0, kNt));
            } else {
                const vu4 vb = __builtin_amdgcn_raw_buffer_load_b128(rv, off * 4, 0, kNt);
                v = vf4{__uint_as_float(vb.x), __uint_as_float(vb.y), __uint_as_float(vb.z), __uint_as_float(vb.w)};
            }
            g = widen(__builtin_amdgcn_raw_buffer_load_b64(rg, off * 2, 0, kNt));
            word = __builtin_amdgcn_raw_buffer_load_b32(rk, (off >> 5) * 4, 0, kNt);
            uint32_t nothing = 0;
            if constexpr (VOIDED) {
                const int past = off + 256;      // beyond the resources' ranges: zeros come back, no memory is touched
                const vu4 a = __builtin_amdgcn_raw_buffer_load_b128(rw, past * 4, 0, kNt);
                const vu2 b = __builtin_amdgcn_raw_buffer_load_b64(rm, past * 2, 0, kNt);
                const vu2 c = __builtin_amdgcn_raw_buffer_load_b64(rv, past * (V16 ? 2 : 4), 0, kNt);
                const vu2 d = __builtin_amdgcn_raw_buffer_load_b64(rg, past * 2, 0, kNt);
                const uint32_t e = __builtin_amdgcn_raw_buffer_load_b32(rk, (past >> 5) * 4, 0, kNt);
                nothing = a.x | b.x | c.x | d.x | e;
            }
            w = vf4{__uint_as_float(wb.x), __uint_as_float(wb.y), __uint_as_float(wb.z), __uint_as_float(wb.w)};
            if constexpr (REDUCE) acc = g.x * w.x + g.y * w.y + g.z * w.z + g.w * w.w;
            touch(w, m, v, g, (word >> (off & 31)) & 15u);
            w.x += __uint_as_float(nothing);      // keeps the voided loads alive
            const vu4 wo = {__float_as_uint(w.x), __float_as_uint(w.y), __float_as_uint(w.z), __float_as_uint(w.w)};
            __builtin_amdgcn_raw_buffer_store_b128(wo, rw, off * 4, 0, kNt);
            __builtin_amdgcn_raw_buffer_store_b64(truncate(m), rm, off * 2, 0, kNt);
            if constexpr (V16) {
                __builtin_amdgcn_raw_buffer_store_b64(truncate(v), rv, off * 2, 0, kNt);
            } else {
                const vu4 vo = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
                __builtin_amdgcn_raw_buffer_store_b128(vo, rv, off * 4, 0, kNt);
            }
        } else if (off < len) {
            w = load<true>((const vf4 *)pw + lane);
            m = widen(load<true>((const vu2 *)pm + lane));
            if constexpr (V16) v = widen(load<true>((const vu2 *)pv + lane));
            else v = load<true>((const vf4 *)pv + lane);
            g = widen(load<true>((const vu2 *)pg + lane));
            word = load<true>(pk + (off >> 5));
            if constexpr (REDUCE) acc = g.x * w.x + g.y * w.y + g.z * w.z + g.w * w.w;
            touch(w, m, v, g, (word >> (off & 31)) & 15u);
            store<true>((vf4 *)pw + lane, w);
            store<true>((vu2 *)pm + lane, truncate(m));
            if constexpr (V16) store<true>((vu2 *)pv + lane, truncate(v));
            else store<true>((vf4 *)pv + lane, v);
        }
    }
    if constexpr (REDUCE) {      // every thread of the workgroup arrives here
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (lane == 0) partial[wave] = acc;
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.0f;
            for (int k = 0; k < BT / 64; ++k) t += partial[k];
            sums[blockIdx.x] = t;
        }
    }
}

// a pure streaming read of `count` 16-byte pieces (the sum keeps the loads alive; one float per workgroup is written)
__global__ __launch_bounds__(256) void read_only(const vf4 *data, int64_t count, float *sums)
{
    __shared__ float partial[4];
    const int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    float acc = 0.0f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t at = i + k * 256;
        if (at < count) {
            const vf4 x = load<true>(data + at);
            acc += x.x + x.y + x.z + x.w;
        }
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if ((threadIdx.x & 63) == 0) partial[threadIdx.x / 64] = acc;
    __syncthreads();
    if (threadIdx.x == 0) sums[blockIdx.x] = partial[0] + partial[1] + partial[2] + partial[3];
}

template <typename F>
static float microseconds(F launch, int reps = 32)
{
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    launch();
    launch();
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(a));
    for (int i = 0; i < reps; ++i) launch();
    CHECK(hipEventRecord(b));
    CHECK(hipEventSynchronize(b));
    float ms = 0.0f;
    CHECK(hipEventElapsedTime(&ms, a, b));
    CHECK(hipGetLastError());
    CHECK(hipEventDestroy(a));
    CHECK(hipEventDestroy(b));
    return ms * 1e3f / reps;
}

static void report(const char *what, double bytes_per_entry, int64_t entries, float us)
{
    printf("%-58s %6.3f B/entry %8.2f us %8.1f GB/s\n", what, bytes_per_entry, us, bytes_per_entry * entries / (us * 1e-6) / 1e9);
    fflush(stdout);
}

int main(int argc, char **argv)
{
    const int64_t rows = argc > 1 ? atoll(argv[1]) : 11008;
    const int cols = argc > 2 ? atoi(argv[2]) : 4096;
    const int matrices = argc > 3 ? atoi(argv[3]) : 16;
    if (rows < 1 || cols < 256 || cols % 256 || matrices < 1 || matrices > 64 || rows * cols > ((int64_t)1 << 28)) {
        printf("usage: stream_skeleton [rows [cols [matrices]]]: cols a multiple of 256, rows * cols <= 2^28, 1..64 matrices\n");
        return 2;
    }
    const int64_t n = rows * cols;
    float *state, *sums;
    void *grad;
    uint32_t *mask;
    // the largest of the layouts decides the sizes: 12 bytes of state and 4 bytes of gradient per entry
    CHECK(hipMalloc(&state, (size_t)matrices * n * 12));
    CHECK(hipMalloc(&grad, (size_t)matrices * n * 4));
    CHECK(hipMalloc(&mask, (size_t)matrices * n / 8));
    CHECK(hipMalloc(&sums, (size_t)64 << 20));
    CHECK(hipMemset(state, 0, (size_t)matrices * n * 12));
    CHECK(hipMemset(grad, 0, (size_t)matrices * n * 4));
    CHECK(hipMemset(mask, 0x55, (size_t)matrices * n / 8));
    printf("%lld x %d, %d matrices in rotation\n", (long long)rows, cols, matrices);
    int turn = 0;
    auto next = [&] { return turn++ % matrices; };

#define PLAIN(label, K, BT, NTL, NTS, G32) { \
        const int per = (K) * (BT) * 4, bpr = (cols + per - 1) / per; \
        const float us = microseconds([&] { const int64_t k = next(); \
            hipLaunchKernelGGL((rmw_plain<K, BT, NTL, NTS, G32>), dim3((unsigned)(rows * bpr)), dim3(BT), 0, 0, state + k * n * 3, \
                               (const void *)((const char *)grad + k * n * ((G32) ? 4 : 2)), mask + k * n / 32, cols, bpr); }); \
        report(label, (G32) ? 28.125 : 26.125, n, us); }
#define TILED(label, TILE) if (cols % (TILE) == 0) { \
        const int bpr = (cols + 1023) / 1024; \
        const float us = microseconds([&] { const int64_t k = next(); \
            hipLaunchKernelGGL((rmw_tiled<TILE>), dim3((unsigned)(rows * bpr)), dim3(256), 0, 0, state + k * n * 3, (const uint16_t *)grad + k * n, \
                               mask + k * n / 32, cols, bpr); }); \
        report(label, 26.125, n, us); }
#define BF16(label, V16, BT, RED, BUF, VO) { \
        const int bpr = (cols + (BT) * 4 - 1) / ((BT) * 4); \
        const float us = microseconds([&] { const int64_t k = next(); \
            hipLaunchKernelGGL((rmw_bf16<V16, BT, RED, BUF, VO>), dim3((unsigned)(rows * bpr)), dim3(BT), 0, 0, (uint8_t *)state + k * n * ((V16) ? 8 : 10), \
                               (const uint16_t *)grad + k * n, mask + k * n / 32, sums, cols, bpr); }); \
        report(label, (V16) ? 18.125 : 22.125, n, us); }

    for (int pass = 0; pass < 2; ++pass) {
        printf("-- pass %d\n", pass + 1);
        PLAIN("fp32 state, 1 piece per thread, 256 threads, nt/nt", 1, 256, true, true, false)
        PLAIN("fp32 state, 1 piece per thread, 512 threads", 1, 512, true, true, false)
        PLAIN("fp32 state, 1 piece per thread, 1024 threads", 1, 1024, true, true, false)
        PLAIN("fp32 state, 2 pieces per thread, 256 threads", 2, 256, true, true, false)
        PLAIN("fp32 state, 4 pieces per thread, 256 threads", 4, 256, true, true, false)
        PLAIN("fp32 state, 1 piece, 256 threads, default loads, nt stores", 1, 256, false, true, false)
        PLAIN("fp32 state, 1 piece, 256 threads, nt loads, default stores", 1, 256, true, false, false)
        PLAIN("fp32 state, fp32 gradients, 1 piece, 256 threads", 1, 256, true, true, true)
        TILED("fp32 state in tiles of 256 entries (1 KiB) per array", 256)
        TILED("fp32 state in tiles of 1024 entries (4 KiB) per array", 1024)
        BF16("first moment bf16, 256 threads", false, 256, false, false, false)
        BF16("both moments bf16, 256 threads", true, 256, false, false, false)
        BF16("both moments bf16, 512 threads", true, 512, false, false, false)
        BF16("both moments bf16, 512 threads, dL/dA sum", true, 512, true, false, false)
        BF16("both moments bf16, 512 threads, buffer resources", true, 512, false, true, false)
        BF16("both moments bf16, 512 threads, buffers, dL/dA sum", true, 512, true, true, false)
        BF16("both moments bf16, 512 threads, buffers, sum, voided loads", true, 512, true, true, true)
        {
            const int64_t pieces = n * 12 / 16;      // the fp32 state of one matrix
            const float us = microseconds([&] { const int64_t k = next();
                hipLaunchKernelGGL(read_only, dim3((unsigned)((pieces + 1023) / 1024)), dim3(256), 0, 0, (const vf4 *)(state + k * n * 3), pieces, sums); });
            report("pure read of the fp32 state", 12.0, n, us);
        }
    }
    CHECK(hipFree(state));
    CHECK(hipFree(grad));
    CHECK(hipFree(mask));
    CHECK(hipFree(sums));
    return 0;
}
