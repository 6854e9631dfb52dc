// Device code of the sharded optimizer step for gfx950 (CDNA4, wave64).
//
// The step is a pure stream: per element it reads N gradient contributions and
// three FP32 state words, and writes three FP32 state words and one 16-bit
// parameter (bf16 or binary16), each byte exactly once.  There is no reuse and no contraction, so
// nothing here uses MFMA, and LDS only serves the sum-of-squares tree.  What
// decides the speed is how the request stream looks to the HBM controllers.
// Measured on MI355X, in this order of importance:
//   - one wavefront per workgroup, one 256-element tile per workgroup, and a
//     grid with one workgroup per tile: the dispatcher hands tiles out in
//     address order, so the whole device sweeps each of the 12-15 streams as
//     one narrow moving window (persistent grid-stride grids lose ~10 %);
//   - only about eight such waves resident per CU (the launch asks for dynamic
//     LDS it never touches, purely to cap residency): more waves in flight
//     widen the window and cost another ~8 %;
//   - the non-temporal hint on every load and store (nothing is reused);
//   - every wave-level access one contiguous 1 KiB (FP32, 16 B per lane) or
//     512 B (bf16, 8 B per lane) span, so each store instruction fills whole
//     128-byte lines by itself;
//   - outside the kernel's control: where the operands lie physically.  A launch whose
//     streams are spread over a working set of hundreds of GB runs 5 % slower than one
//     whose streams lie within a few GiB of one another (ps_arena.cpp lays flat buffers
//     out accordingly).
// In this mix a byte read costs about 0.12 ps and a byte written about 0.22 ps (the same
// kernel with its contributions served from L2: 1.23 ms per 2^28 elements, from HBM: 1.75;
// read-only scans reach 7.0-7.3 TB/s, the 12 B read + 14 B written of the state alone 5.7),
// so with a third of its bytes written the step ends at 0.81-0.83 of the 8 TB/s peak.
//
// Work decomposition.  A tile is 256 consecutive elements; lane t owns
// elements 4t..4t+3.  All loads of a tile are issued before the first
// arithmetic instruction.  Elements past the last whole tile are handled by a
// bounds-checked one-element-per-lane kernel.
//
// Arithmetic.  Every line of step_element() is one correctly rounded binary32
// operation (the translation unit is compiled with contraction off and with
// IEEE division and square root), so results do not depend on launch shape or
// on which kernel (tile or tail) handles an element.
#ifndef PS_KERNEL_TEMPLATES_H
#define PS_KERNEL_TEMPLATES_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ps_internal.h"

namespace ps {

constexpr int kWave = 64;               // threads per workgroup of the streaming kernels
constexpr int kTileElems = kWave * 4;    // elements per tile
constexpr int kThreads = 256;            // threads per workgroup of the small helper kernels

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool NT, typename T>
__device__ __forceinline__ T load_vec(const T *p)
{
    if constexpr (NT)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}

template <bool NT, typename T>
__device__ __forceinline__ void store_vec(T *p, T x)
{
    if constexpr (NT)
        __builtin_nontemporal_store(x, p);
    else
        *p = x;
}

// Element types of the 16-bit buffers: uint16_t stands for bf16 bit patterns,
// f16_bits for IEEE binary16 (the FP16 of the paper's Table 1); float is float.
struct f16_bits {
    uint16_t v;
};

// bf16 -> binary32 is a 16-bit shift of the pattern (exact).
__device__ __forceinline__ float widen_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float widen_hi(uint32_t pair)
{
    return __uint_as_float(pair & 0xffff0000u);
}

// binary16 -> binary32 (exact, subnormals included: the conversion instruction
// does not flush them).
__device__ __forceinline__ float widen_f16(uint32_t bits16)
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
}

// The two 16-bit values packed in one 32-bit word, widened according to G.
template <typename G>
__device__ __forceinline__ float widen16_lo(uint32_t pair)
{
    if constexpr (sizeof(G) == 2 && !__is_same(G, uint16_t))
        return widen_f16(pair & 0xffffu);
    else
        return widen_lo(pair);
}
template <typename G>
__device__ __forceinline__ float widen16_hi(uint32_t pair)
{
    if constexpr (sizeof(G) == 2 && !__is_same(G, uint16_t))
        return widen_f16(pair >> 16);
    else
        return widen_hi(pair);
}

// binary32 -> bf16, round to nearest, ties to even; NaN -> quiet NaN, sign kept.
__device__ __forceinline__ uint32_t narrow_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = ((u >> 16) & 0x8000u) | 0x7fc0u;
    return (u & 0x7fffffffu) > 0x7f800000u ? nan : r;
}

// binary32 -> binary16, round to nearest, ties to even (the conversion
// instruction under the default rounding mode; overflow goes to infinity, small
// magnitudes to subnormals); NaN -> quiet NaN 0x7E00, sign kept.
__device__ __forceinline__ uint32_t narrow_f16(float x)
{
    const uint32_t u = __float_as_uint(x);
    const uint32_t nan = ((u >> 16) & 0x8000u) | 0x7e00u;
    const uint32_t r = __builtin_bit_cast(uint16_t, (_Float16)x);
    return (u & 0x7fffffffu) > 0x7f800000u ? nan : r;
}

// The 16-bit image of a new master weight in the parameters' format.
__device__ __forceinline__ uint32_t narrow16(float x, uint32_t out_f16)
{
    return out_f16 ? narrow_f16(x) : narrow_bf16(x);
}

// The per-element update.  acc is the fixed-order sum of the N per-device
// contributions (the Reduce-Scatter result of Section 2.3 for this element; one
// data type and one order for all of them, Theorem 4).  acc * gs is the
// global-batch mean that gradient integrity requires (Theorem 3, Eq. 15; the
// division by N of the proof of Theorem 5).  m, v and th are the FP32 Adam moments
// and master weight of Table 1; the paper prints no Adam formula, the textbook
// bias-corrected form with decoupled decay is used in this exact operation order.
__device__ __forceinline__ void step_element(float acc, float &th, float &m, float &v,
                                             const StepScalars &s)
{
    float g = acc * s.gs;
    g = g * s.cc;
    float m1 = __builtin_fmaf(s.b1, m, s.omb1 * g);
    float v1 = __builtin_fmaf(s.b2, v, (s.omb2 * g) * g);
    float den = __builtin_fmaf(__builtin_sqrtf(v1), s.isb2, s.ep);
    float u = m1 / den;
    float t0 = __builtin_fmaf(-s.lw, th, th);
    th = __builtin_fmaf(-s.step, u, t0);
    m = m1;
    v = v1;
}

// Four independent elements at once (ext-vector lanes cannot bind to references).
__device__ __forceinline__ void step_element4(const f32x4 acc, f32x4 &th, f32x4 &m, f32x4 &v,
                                              const StepScalars &s)
{
    float t[4] = {th.x, th.y, th.z, th.w};
    float mm[4] = {m.x, m.y, m.z, m.w};
    float vv[4] = {v.x, v.y, v.z, v.w};
    const float ac[4] = {acc.x, acc.y, acc.z, acc.w};
#pragma unroll
    for (int i = 0; i < 4; ++i)
        step_element(ac[i], t[i], mm[i], vv[i], s);
    th = f32x4{t[0], t[1], t[2], t[3]};
    m = f32x4{mm[0], mm[1], mm[2], mm[3]};
    v = f32x4{vv[0], vv[1], vv[2], vv[3]};
}

// One contribution's four consecutive elements, widened to binary32.
template <typename G, bool NT>
__device__ __forceinline__ f32x4 load_contrib4(const void *base, uint64_t elem)
{
    if constexpr (sizeof(G) == 2) {
        u32x2 w = load_vec<NT>(reinterpret_cast<const u32x2 *>(
            reinterpret_cast<const uint16_t *>(base) + elem));
        f32x4 r;
        r.x = widen16_lo<G>(w.x);
        r.y = widen16_hi<G>(w.x);
        r.z = widen16_lo<G>(w.y);
        r.w = widen16_hi<G>(w.y);
        return r;
    } else {
        return load_vec<NT>(
            reinterpret_cast<const f32x4 *>(reinterpret_cast<const float *>(base) + elem));
    }
}

template <typename G>
__device__ __forceinline__ float load_contrib1(const void *base, uint64_t elem)
{
    if constexpr (sizeof(G) == 2)
        return widen16_lo<G>(reinterpret_cast<const uint16_t *>(base)[elem]);
    else
        return reinterpret_cast<const float *>(base)[elem];
}

// The clip coefficient of a launch: the host's value, or what the device holds at
// clip_coef_device by now.  Returns false when that is NaN: the step is skipped.
__device__ __forceinline__ bool resolve_clip(StepScalars &s)
{
    if (s.cc_device) {
        const float c = *s.cc_device;
        if (!(c == c))
            return false;
        s.cc = c;
    }
    return true;
}

// Clip coefficient from the sums of squares (one lane), the host formula in binary64.
__global__ void clip_coef_kernel(const double *sumsq_local, const double *sumsq_others,
                                 double max_norm, float *coef_out)
{
    const double a = *sumsq_local, b = sumsq_others ? *sumsq_others : 0.0;
    const double total = a + b;
    double coef;
    if (!(total - total == 0.0) || a < 0.0 || b < 0.0 || !(max_norm > 0.0)) {
        coef = __builtin_nan("");
    } else {
        coef = max_norm / (__builtin_sqrt(total) + 1e-6);
        coef = coef < 1.0 ? coef : 1.0;
    }
    *coef_out = (float)coef;
}

struct UpdateArgs {
    ContribPtrs g;
    const float *accum; // sum of earlier micro-batches, added to this one's; or NULL
    float *master, *m, *v;
    uint16_t *out;
    uint64_t n_tiles; // whole tiles (tile kernel) or element count (tail kernel)
    uint32_t n_contrib;
    StepScalars s;
};

// Fused reduce + AdamW + bf16 cast over whole tiles, one wave per tile.  Each
// device runs this on its own shard only (proof of Corollary 1, part 1); the bf16
// image it writes is the persistent S* shard that the next All-Gather reads
// (Definition 1, Eq. 3), or this shard's slice of the replicated parameters.
//   N : contribution count known at compile time, 0 = read it from args
//   G : uint16_t (bf16 bits), f16_bits (binary16) or float
//   A : a.accum is added to the contributions' sum (the last micro-batch of an
//       accumulated step: what accumulate_tiles would store is used straight away)
// The loop only repeats when there are more tiles than the grid can hold.
template <int N, typename G, bool A>
__global__ __launch_bounds__(kWave) void update_tiles(const UpdateArgs a)
{
    const uint32_t n = N ? N : a.n_contrib;
    StepScalars s = a.s;
    if (!resolve_clip(s))
        return;
    for (uint64_t tile = blockIdx.x; tile < a.n_tiles; tile += gridDim.x) {
        const uint64_t e = tile * kTileElems + (uint64_t)threadIdx.x * 4;
        f32x4 acc, run, th, mm, vv;
        if constexpr (N != 0) {
            f32x4 gr[N];
#pragma unroll
            for (int r = 0; r < N; ++r)
                gr[r] = load_contrib4<G, true>(a.g.p[r], e);
            if constexpr (A)
                run = load_vec<true>(reinterpret_cast<const f32x4 *>(a.accum + e));
            th = load_vec<true>(reinterpret_cast<const f32x4 *>(a.master + e));
            mm = load_vec<true>(reinterpret_cast<const f32x4 *>(a.m + e));
            vv = load_vec<true>(reinterpret_cast<const f32x4 *>(a.v + e));
            acc = gr[0];
#pragma unroll
            for (int r = 1; r < N; ++r)
                acc = acc + gr[r];
        } else {
            if constexpr (A)
                run = load_vec<true>(reinterpret_cast<const f32x4 *>(a.accum + e));
            th = load_vec<true>(reinterpret_cast<const f32x4 *>(a.master + e));
            mm = load_vec<true>(reinterpret_cast<const f32x4 *>(a.m + e));
            vv = load_vec<true>(reinterpret_cast<const f32x4 *>(a.v + e));
            acc = load_contrib4<G, true>(a.g.p[0], e);
            for (uint32_t r = 1; r < n; ++r)
                acc = acc + load_contrib4<G, true>(a.g.p[r], e);
        }
        if constexpr (A)
            acc = run + acc;
        step_element4(acc, th, mm, vv, s);
        u32x2 pk;
        pk.x = narrow16(th.x, s.out_f16) | (narrow16(th.y, s.out_f16) << 16);
        pk.y = narrow16(th.z, s.out_f16) | (narrow16(th.w, s.out_f16) << 16);
        store_vec<true>(reinterpret_cast<f32x4 *>(a.master + e), th);
        store_vec<true>(reinterpret_cast<f32x4 *>(a.m + e), mm);
        store_vec<true>(reinterpret_cast<f32x4 *>(a.v + e), vv);
        store_vec<true>(reinterpret_cast<u32x2 *>(a.out + e), pk);
    }
}

// Same update, one element per lane with a bounds check; a.n_tiles is the
// element count here.  Used for what is left after the last whole tile.
template <typename G>
__global__ __launch_bounds__(kWave) void update_tail(const UpdateArgs a)
{
    const uint64_t e = (uint64_t)blockIdx.x * kWave + threadIdx.x;
    StepScalars s = a.s;
    if (e >= a.n_tiles || !resolve_clip(s))
        return;
    float acc = load_contrib1<G>(a.g.p[0], e);
    for (uint32_t r = 1; r < a.n_contrib; ++r)
        acc = acc + load_contrib1<G>(a.g.p[r], e);
    if (a.accum)
        acc = a.accum[e] + acc;
    float th = a.master[e], m = a.m[e], v = a.v[e];
    step_element(acc, th, m, v, s);
    a.master[e] = th;
    a.m[e] = m;
    a.v[e] = v;
    a.out[e] = (uint16_t)narrow16(th, s.out_f16);
}

struct AccumArgs {
    ContribPtrs g;
    float *accum;
    uint64_t n_tiles; // whole tiles (tile kernel) or element count (tail kernel)
    uint32_t n_contrib;
    uint32_t overwrite; // first micro-batch: store the sum instead of adding it
};

// Gradient accumulation: accum (+)= fixed-order sum of one micro-batch's
// contributions.  Same launch shape as the update.
template <int N, typename G, bool OVERWRITE>
__global__ __launch_bounds__(kWave) void accumulate_tiles(const AccumArgs a)
{
    const uint32_t n = N ? N : a.n_contrib;
    for (uint64_t tile = blockIdx.x; tile < a.n_tiles; tile += gridDim.x) {
        const uint64_t e = tile * kTileElems + (uint64_t)threadIdx.x * 4;
        f32x4 acc, run;
        if constexpr (N != 0) {
            f32x4 gr[N];
#pragma unroll
            for (int r = 0; r < N; ++r)
                gr[r] = load_contrib4<G, true>(a.g.p[r], e);
            if constexpr (!OVERWRITE)
                run = load_vec<true>(reinterpret_cast<const f32x4 *>(a.accum + e));
            acc = gr[0];
#pragma unroll
            for (int r = 1; r < N; ++r)
                acc = acc + gr[r];
        } else {
            if constexpr (!OVERWRITE)
                run = load_vec<true>(reinterpret_cast<const f32x4 *>(a.accum + e));
            acc = load_contrib4<G, true>(a.g.p[0], e);
            for (uint32_t r = 1; r < n; ++r)
                acc = acc + load_contrib4<G, true>(a.g.p[r], e);
        }
        if constexpr (!OVERWRITE)
            acc = run + acc;
        store_vec<true>(reinterpret_cast<f32x4 *>(a.accum + e), acc);
    }
}

template <typename G>
__global__ __launch_bounds__(kWave) void accumulate_tail(const AccumArgs a)
{
    const uint64_t e = (uint64_t)blockIdx.x * kWave + threadIdx.x;
    if (e >= a.n_tiles)
        return;
    float acc = load_contrib1<G>(a.g.p[0], e);
    for (uint32_t r = 1; r < a.n_contrib; ++r)
        acc = acc + load_contrib1<G>(a.g.p[r], e);
    a.accum[e] = a.overwrite ? acc : a.accum[e] + acc;
}

// ---- sum of squares: the only place that needs cross-lane traffic ----
// No atomics anywhere: the paper's determinism assumption (Theorem 5, assumption 1)
// names atomics in reductions as what breaks it (Remark 3).  Every tree below has a
// shape that depends only on the element count.

// Butterfly over the 64 lanes; every lane ends with the same bits.
template <typename T>
__device__ __forceinline__ T wave_sum(T x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        x += __shfl_xor(x, off, 64);
    return x;
}

// Fixed-shape tree for a workgroup of THREADS lanes: butterfly inside each wave,
// then the wave sums through LDS, added in wave order.  Every lane must call it.
template <typename T, int THREADS>
__device__ __forceinline__ T block_sum_n(T x)
{
    __shared__ T partial[THREADS / 64];
    x = wave_sum(x);
    if ((threadIdx.x & 63) == 0)
        partial[threadIdx.x >> 6] = x;
    __syncthreads();
    T t = partial[0];
#pragma unroll
    for (int w = 1; w < THREADS / 64; ++w)
        t += partial[w];
    __syncthreads();
    return t;
}

template <typename T>
__device__ __forceinline__ T block_sum(T x)
{
    return block_sum_n<T, kThreads>(x);
}

// The same tree for Q values at once with a single barrier; its LDS is not
// protected against reuse, so a kernel calls it once, as its last collective.
template <typename T, int THREADS, int Q>
__device__ __forceinline__ void block_sum_once(T (&x)[Q])
{
    __shared__ T partial[Q][THREADS / 64];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        x[q] = wave_sum(x[q]);
        if ((threadIdx.x & 63) == 0)
            partial[q][threadIdx.x >> 6] = x[q];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        T t = partial[q][0];
#pragma unroll
        for (int w = 1; w < THREADS / 64; ++w)
            t += partial[q][w];
        x[q] = t;
    }
}

// Tiles each workgroup of the reduce pass walks, one after the other.
constexpr uint32_t kReduceTilesPerGroup = 4;

struct ReduceArgs {
    ContribPtrs g;
    float *reduced; // may be null
    double *partials;
    uint64_t n_tiles; // whole tiles (tile kernel) or element count (tail kernel)
    uint64_t first_group; // tile kernel: group handled by workgroup 0 of this launch
    uint32_t n_contrib;
    uint32_t partial_slot; // tail kernel: where its single partial goes
    float gs;
};

// Reduce the contributions, scale to the mean, optionally store it, and leave
// one binary64 partial sum of squares per group of four tiles in partials[group].
// Group b owns tiles [4b, 4b+4); a launch covers the groups from first_group on
// (a long range goes out as several launches, which changes nothing in the
// result: the partials land where one launch would put them).
template <int N, typename G>
__global__ __launch_bounds__(kWave) void reduce_sumsq_tiles(const ReduceArgs a)
{
    const uint32_t n = N ? N : a.n_contrib;
    double ss = 0.0;
    const uint64_t group = a.first_group + blockIdx.x;
    const uint64_t t0 = group * kReduceTilesPerGroup;
    const uint64_t t1 = t0 + kReduceTilesPerGroup < a.n_tiles ? t0 + kReduceTilesPerGroup : a.n_tiles;
    for (uint64_t tile = t0; tile < t1; ++tile) {
        const uint64_t e = tile * kTileElems + (uint64_t)threadIdx.x * 4;
        f32x4 acc;
        if constexpr (N != 0) {
            f32x4 gr[N];
#pragma unroll
            for (int r = 0; r < N; ++r)
                gr[r] = load_contrib4<G, true>(a.g.p[r], e);
            acc = gr[0];
#pragma unroll
            for (int r = 1; r < N; ++r)
                acc = acc + gr[r];
        } else {
            acc = load_contrib4<G, true>(a.g.p[0], e);
            for (uint32_t r = 1; r < n; ++r)
                acc = acc + load_contrib4<G, true>(a.g.p[r], e);
        }
        const f32x4 g = acc * a.gs;
        ss += (double)g.x * (double)g.x;
        ss += (double)g.y * (double)g.y;
        ss += (double)g.z * (double)g.z;
        ss += (double)g.w * (double)g.w;
        if (a.reduced)
            store_vec<true>(reinterpret_cast<f32x4 *>(a.reduced + e), g);
    }
    const double t = wave_sum(ss);
    if (threadIdx.x == 0)
        a.partials[group] = t;
}

// Tail: a single wave strides over the leftover elements (fewer than one tile).
template <typename G>
__global__ __launch_bounds__(kWave) void reduce_sumsq_tail(const ReduceArgs a)
{
    double ss = 0.0;
    for (uint64_t e = threadIdx.x; e < a.n_tiles; e += kWave) {
        float acc = load_contrib1<G>(a.g.p[0], e);
        for (uint32_t r = 1; r < a.n_contrib; ++r)
            acc = acc + load_contrib1<G>(a.g.p[r], e);
        const float g = acc * a.gs;
        ss += (double)g * (double)g;
        if (a.reduced)
            a.reduced[e] = g;
    }
    const double t = wave_sum(ss);
    if (threadIdx.x == 0)
        a.partials[a.partial_slot] = t;
}

// First stage of the final sum: workgroup b adds the contiguous slice
// [b*per, min((b+1)*per, n)) of `in` in a fixed order into out[b].
template <typename T>
__global__ __launch_bounds__(kThreads) void fold_partials(const T *in, uint64_t n, uint64_t per,
                                                          T *out)
{
    const uint64_t lo = (uint64_t)blockIdx.x * per;
    const uint64_t hi = lo + per < n ? lo + per : n;
    T ss = 0;
    for (uint64_t i = lo + threadIdx.x; i < hi; i += kThreads)
        ss += in[i];
    const T t = block_sum(ss);
    if (threadIdx.x == 0)
        out[blockIdx.x] = t;
}

// Last stage: sum partials[0 .. n) in a fixed order (lane-strided, then the
// block tree) and store the total, or add it to what *out already holds.
template <typename T>
__global__ __launch_bounds__(kThreads) void finalize_sum(const T *partials, uint32_t n, T *out,
                                                        int accumulate)
{
    T ss = 0;
    for (uint32_t i = threadIdx.x; i < n; i += kThreads)
        ss += partials[i];
    const T t = block_sum(ss);
    if (threadIdx.x == 0)
        *out = accumulate ? *out + t : t;
}

// ---- verification protocol: read-only scans ----

struct ScanArgs {
    const void *a;
    const void *b;
    void *partials0; // per-workgroup partial sums (first quantity)
    void *partials1; // second quantity, where there is one
    uint64_t n_tiles; // finishing kernels: leftover units; group kernels take their extent from the grid
    uint64_t first_index;
};

// The scans only read, and a read-only stream is fastest on this part with large
// workgroups that keep four 16-byte loads per lane in flight: 1024 lanes, 64 KiB
// per workgroup (7.0-7.3 TB/s; single-wave workgroups as in the update kernel
// stay at 6.1-6.6).  A launch covers whole groups; what is left, and the groups' partial
// sums, go to one finishing workgroup.
constexpr int kScanThreads = 1024;
constexpr int kDiffVecs = 2;     // 16-byte vectors per lane and buffer: a group is 32 KiB of each
constexpr int kChecksumVecs = 4; // 16-byte vectors per lane: a group is 64 KiB = 8192 words

// Sums of (a-b)^2 and a^2 in binary64.  Every lane takes 16 bytes per load
// whatever the element type.  Fixed order: per lane by vector and element, then
// the block tree, one pair of partials per workgroup.
template <typename G>
__global__ __launch_bounds__(kScanThreads) void diff_sumsq_tiles(const ScanArgs s)
{
    constexpr int K = kDiffVecs;
    double sd = 0.0, sa = 0.0;
    const uint64_t v0 = (uint64_t)blockIdx.x * (kScanThreads * K) + threadIdx.x;
    u32x4 x[K], y[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        x[k] = load_vec<true>(reinterpret_cast<const u32x4 *>(s.a) + v0 + (uint64_t)k * kScanThreads);
        y[k] = load_vec<true>(reinterpret_cast<const u32x4 *>(s.b) + v0 + (uint64_t)k * kScanThreads);
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t xw[4] = {x[k].x, x[k].y, x[k].z, x[k].w}, yw[4] = {y[k].x, y[k].y, y[k].z, y[k].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (sizeof(G) == 2) {
                const double xl = (double)widen16_lo<G>(xw[i]), xh = (double)widen16_hi<G>(xw[i]);
                const double dl = xl - (double)widen16_lo<G>(yw[i]);
                const double dh = xh - (double)widen16_hi<G>(yw[i]);
                sd += dl * dl;
                sa += xl * xl;
                sd += dh * dh;
                sa += xh * xh;
            } else {
                const double xv = (double)__uint_as_float(xw[i]);
                const double d = xv - (double)__uint_as_float(yw[i]);
                sd += d * d;
                sa += xv * xv;
            }
        }
    }
    double both[2] = {sd, sa};
    block_sum_once<double, kScanThreads, 2>(both);
    if (threadIdx.x == 0) {
        reinterpret_cast<double *>(s.partials0)[blockIdx.x] = both[0];
        reinterpret_cast<double *>(s.partials1)[blockIdx.x] = both[1];
    }
}

// Last stage of the difference scan, one workgroup: adds the n_partials pairs the groups
// left (lane-strided, fixed order), then the elements past the last whole group (fewer
// than one group's worth; s.a and s.b point at the first of them), runs the block tree
// once and stores the two totals, or adds them to what out2 holds.
template <typename G>
__global__ __launch_bounds__(kScanThreads) void diff_sumsq_finish(const ScanArgs s, uint64_t n_partials,
                                                                  double *out2, int accumulate)
{
    double both[2] = {0.0, 0.0};
    const double *p0 = reinterpret_cast<const double *>(s.partials0);
    const double *p1 = reinterpret_cast<const double *>(s.partials1);
    // four lane-strided rows at a time, all eight loads in flight; the order is fixed
    uint64_t i = threadIdx.x;
    for (; i + 3 * kScanThreads < n_partials; i += 4 * kScanThreads) {
        const double a0 = p0[i], a1 = p0[i + kScanThreads], a2 = p0[i + 2 * kScanThreads],
                     a3 = p0[i + 3 * kScanThreads];
        const double b0 = p1[i], b1 = p1[i + kScanThreads], b2 = p1[i + 2 * kScanThreads],
                     b3 = p1[i + 3 * kScanThreads];
        both[0] += (a0 + a1) + (a2 + a3);
        both[1] += (b0 + b1) + (b2 + b3);
    }
    for (; i < n_partials; i += kScanThreads) {
        both[0] += p0[i];
        both[1] += p1[i];
    }
    for (uint64_t e = threadIdx.x; e < s.n_tiles; e += kScanThreads) {
        const double x = (double)load_contrib1<G>(s.a, e), y = (double)load_contrib1<G>(s.b, e);
        const double d = x - y;
        both[0] += d * d;
        both[1] += x * x;
    }
    block_sum_once<double, kScanThreads, 2>(both);
    if (threadIdx.x == 0) {
        out2[0] = accumulate ? out2[0] + both[0] : both[0];
        out2[1] = accumulate ? out2[1] + both[1] : both[1];
    }
}

// Intermediate stage for very long buffers: workgroup (b, q) adds the contiguous slice
// [b*per, min((b+1)*per, n)) of quantity q's partials into its second-level slot b.
struct FoldArgs {
    const void *in[2];
    void *out[2];
};

template <typename T>
__global__ __launch_bounds__(kThreads) void fold_partials_q(const FoldArgs f, uint64_t n, uint64_t per)
{
    const T *in = reinterpret_cast<const T *>(f.in[blockIdx.y]);
    T *out = reinterpret_cast<T *>(f.out[blockIdx.y]);
    const uint64_t lo = (uint64_t)blockIdx.x * per;
    const uint64_t hi = lo + per < n ? lo + per : n;
    T ss = 0;
    for (uint64_t i = lo + threadIdx.x; i < hi; i += kThreads)
        ss += in[i];
    const T t = block_sum(ss);
    if (threadIdx.x == 0)
        out[blockIdx.x] = t;
}

// One word's contribution to the checksum: the splitmix64 output function of
// w + (index + 1) * golden-ratio increment.  The product is passed in (`ramp`)
// so that callers walking consecutive indices can form it by addition.
constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

__device__ __forceinline__ uint64_t checksum_mix(uint64_t w, uint64_t ramp)
{
    uint64_t z = w + ramp;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ uint64_t checksum_term(uint64_t w, uint64_t index)
{
    return checksum_mix(w, (index + 1) * kGolden);
}

// Checksum over whole groups of 8192 words; lane t owns words 2t, 2t+1 of each of
// the group's four 16-KiB rows, all loaded before the arithmetic.  One 64-bit
// multiply per lane forms (index + 1) * increment for its first word; the
// others follow by adding multiples of the increment (arithmetic modulo 2^64).
__global__ __launch_bounds__(kScanThreads) void checksum_tiles(const ScanArgs s)
{
    constexpr int K = kChecksumVecs;
    uint64_t c = 0;
    const uint64_t v0 = (uint64_t)blockIdx.x * (kScanThreads * K) + threadIdx.x;
    u32x4 v[K];
#pragma unroll
    for (int k = 0; k < K; ++k)
        v[k] = load_vec<true>(reinterpret_cast<const u32x4 *>(s.a) + v0 + (uint64_t)k * kScanThreads);
    uint64_t ramp = (s.first_index + v0 * 2 + 1) * kGolden; // this lane's first word in the buffer
#pragma unroll
    for (int k = 0; k < K; ++k) {
        c += checksum_mix((uint64_t)v[k].x | ((uint64_t)v[k].y << 32), ramp);
        c += checksum_mix((uint64_t)v[k].z | ((uint64_t)v[k].w << 32), ramp + kGolden);
        ramp += (uint64_t)(kScanThreads * 2) * kGolden; // next row: 2048 words further on
    }
    uint64_t one[1] = {c};
    block_sum_once<uint64_t, kScanThreads, 1>(one);
    if (threadIdx.x == 0)
        reinterpret_cast<uint64_t *>(s.partials0)[blockIdx.x] = one[0];
}

// Last stage of the checksum, one workgroup: the groups' partials, then the words past the
// last whole group (s.a points at the first of them, s.first_index is its index), all
// modulo 2^64, stored or added to *out.
__global__ __launch_bounds__(kScanThreads) void checksum_finish(const ScanArgs s, uint64_t n_partials,
                                                                uint64_t *out, int accumulate)
{
    uint64_t one[1] = {0};
    const uint64_t *p0 = reinterpret_cast<const uint64_t *>(s.partials0);
    uint64_t i = threadIdx.x;
    for (; i + 3 * kScanThreads < n_partials; i += 4 * kScanThreads)
        one[0] += (p0[i] + p0[i + kScanThreads]) + (p0[i + 2 * kScanThreads] + p0[i + 3 * kScanThreads]);
    for (; i < n_partials; i += kScanThreads)
        one[0] += p0[i];
    for (i = threadIdx.x; i < s.n_tiles; i += kScanThreads)
        one[0] += checksum_term(reinterpret_cast<const uint64_t *>(s.a)[i], s.first_index + i);
    block_sum_once<uint64_t, kScanThreads, 1>(one);
    if (threadIdx.x == 0)
        *out = accumulate ? *out + one[0] : one[0];
}

// Plain copy with the update kernel's access shape: one wave per 1 KiB, 16 B
// per lane; what is left beyond whole KiB goes 16 B per lane in group 0.
__global__ __launch_bounds__(kWave) void copy_tiles(u32x4 *dst, const u32x4 *src,
                                                    uint64_t n_tiles, uint64_t n_vec)
{
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint64_t i = tile * kWave + threadIdx.x;
        store_vec<true>(dst + i, load_vec<true>(src + i));
    }
    if (blockIdx.x == 0)
        for (uint64_t i = n_tiles * kWave + threadIdx.x; i < n_vec; i += kWave)
            dst[i] = src[i];
}

struct StageArgs {
    ContribPtrs src;
    char *dst;
    uint64_t slot_stride_bytes;
    uint64_t first_vec;  // position of the bucket's first vector in the periodic source
    uint64_t period_vec; // source length in 16-byte vectors
    uint64_t n_vec;      // vectors per contribution in this bucket
    uint32_t wrap_once;  // period_vec >= vectors per trip: at most one wrap inside a trip
};

// Bucket staging: blockIdx.y selects the contribution, each wave moves U KiB per
// trip and strides over the bucket by the grid width.  The source repeats with
// period_vec (a multiple of 64 U is not required: the wrap is found per lane,
// from one wave-uniform remainder per trip).
template <int U>
__global__ __launch_bounds__(kWave) void stage_bucket(const StageArgs a)
{
    const u32x4 *src = reinterpret_cast<const u32x4 *>(a.src.p[blockIdx.y]);
    u32x4 *dst = reinterpret_cast<u32x4 *>(a.dst + (uint64_t)blockIdx.y * a.slot_stride_bytes);
    for (uint64_t base = (uint64_t)blockIdx.x * (kWave * U); base < a.n_vec;
         base += (uint64_t)gridDim.x * (kWave * U)) {
        // position of this trip's first vector in the source, same for all lanes
        const uint64_t s0 = (a.first_vec + base) % a.period_vec;
        u32x4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t i = base + (uint64_t)u * kWave + threadIdx.x;
            uint64_t s = s0 + (uint64_t)u * kWave + threadIdx.x;
            if (s >= a.period_vec)
                s = a.wrap_once ? s - a.period_vec : s % a.period_vec;
            if (i < a.n_vec)
                x[u] = load_vec<false>(src + s); // plain load: a short source stays in L2
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t i = base + (uint64_t)u * kWave + threadIdx.x;
            if (i < a.n_vec)
                store_vec<true>(dst + i, x[u]);
        }
    }
}

} // namespace ps

#endif
