// Kernel instantiations and launch shapes for gfx950.  The launch shapes are
// constants of the library, never queried from the device, so that the
// reduction tree of the sum of squares is the same on every run.
#include "ps_kernel_templates.h"

#include <atomic>
#include <mutex>

namespace ps {

// Dynamic LDS requested by the streaming launches.  The kernels never touch it:
// with 160 KiB of LDS per CU it caps how many single-wave workgroups are
// resident per CU, which is what keeps the HBM request stream narrow.  The best
// cap depends on how many bytes one wave keeps in flight; measured on MI355X:
//   update, 8 bf16 contributions (7 KiB per wave)        8 waves per CU  6.6 TB/s
//   update, 2..4 bf16 contributions (4-5 KiB)            8-10 waves      6.6 TB/s
//   update, one contribution (3.5-4 KiB)                 10-12 waves     6.6 TB/s
//   accumulate (4.5-5 KiB, one store)                    12 waves        6.5-6.7 TB/s
//   reduce + sum of squares, four tiles per workgroup    6 waves (fp32), 8 (bf16)
// Two waves fewer or four more than the best cost 5-10 %.
constexpr uint32_t lds_for_waves(uint32_t waves_per_cu)
{
    return (163840u / waves_per_cu) & ~255u;
}

// Measurement aid: a residency cap for the update kernel that replaces the choice below
// (0 = none; 3..32 waves per CU; above 32 = no cap at all).
static std::atomic<uint32_t> update_residency_override{0};

void set_update_residency(uint32_t waves_per_cu) { update_residency_override.store(waves_per_cu); }

static uint32_t update_lds(uint32_t n_contrib, int dtype, bool with_accum)
{
    const uint32_t forced = update_residency_override.load();
    if (forced)
        return forced > 32 ? 0u : lds_for_waves(forced < 3 ? 3 : forced);
    if (n_contrib == 1 && !with_accum)
        return lds_for_waves(dtype == PS_BF16 ? 12 : 10);
    const uint32_t in_flight = n_contrib * (dtype == PS_BF16 ? 512u : 1024u) + 3072u +
                               (with_accum ? 1024u : 0u);
    return lds_for_waves(in_flight <= 4608u ? 10 : 8);
}

constexpr uint32_t kAccumLdsBytes = lds_for_waves(12);

static uint32_t reduce_lds(int dtype) { return lds_for_waves(dtype == PS_BF16 ? 8 : 6); }

// The staging copy, when it has the device to itself, runs best with the same cap
// (8 waves of 4 KiB in flight per CU: 6.8 TB/s of writes from an L2-resident
// source).  When it shares the device with the update kernel it asks for no LDS,
// so that it never waits behind the update's own LDS reservations.
constexpr uint32_t kStageAloneLdsBytes = lds_for_waves(8);
// Largest grid used; beyond it the kernels loop (never reached below 5e11 elements).
constexpr uint64_t kMaxGrid = 0x7fffffffull;
// Second level of the sum-of-squares tree.
constexpr uint32_t kFoldBlocks = 1024;
// groups of four tiles per launch of the reduce kernel: 2^27 elements
constexpr uint64_t kReduceLaunchGroups = (1ull << 27) / (kTileElems * kReduceTilesPerGroup);

static uint32_t grid_for(uint64_t n)
{
    return (uint32_t)(n < kMaxGrid ? n : kMaxGrid);
}

template <typename G>
static const void *advance(const void *p, uint64_t elems)
{
    return reinterpret_cast<const G *>(p) + elems;
}

template <int N, typename G>
static void launch_update_n(const UpdateArgs &a, uint32_t grid, hipStream_t st)
{
    const uint32_t lds = update_lds(a.n_contrib, sizeof(G) == 2 ? PS_BF16 : PS_F32, a.accum != nullptr);
    if (a.accum)
        hipLaunchKernelGGL((update_tiles<N, G, true>), dim3(grid), dim3(kWave), lds, st, a);
    else
        hipLaunchKernelGGL((update_tiles<N, G, false>), dim3(grid), dim3(kWave), lds, st, a);
}

template <typename G>
static int launch_update_t(uint32_t n_contrib, const ContribPtrs &g, const float *accum,
                           float *master, float *m, float *v, uint16_t *out, uint64_t count,
                           const StepScalars &s, hipStream_t st)
{
    const uint64_t n_tiles = count / kTileElems;
    const uint64_t body = n_tiles * kTileElems;
    UpdateArgs a;
    a.g = g;
    a.accum = accum;
    a.master = master;
    a.m = m;
    a.v = v;
    a.out = out;
    a.n_contrib = n_contrib;
    a.s = s;
    if (n_tiles) {
        a.n_tiles = n_tiles;
        const uint32_t grid = grid_for(n_tiles);
        switch (n_contrib) {
        case 1: launch_update_n<1, G>(a, grid, st); break;
        case 2: launch_update_n<2, G>(a, grid, st); break;
        case 3: launch_update_n<3, G>(a, grid, st); break;
        case 4: launch_update_n<4, G>(a, grid, st); break;
        case 5: launch_update_n<5, G>(a, grid, st); break;
        case 6: launch_update_n<6, G>(a, grid, st); break;
        case 7: launch_update_n<7, G>(a, grid, st); break;
        case 8: launch_update_n<8, G>(a, grid, st); break;
        default: launch_update_n<0, G>(a, grid, st); break; // 9..16: contribution loop not unrolled
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return (int)e;
    }
    if (count > body) {
        const uint64_t rest = count - body;
        for (uint32_t r = 0; r < n_contrib; ++r)
            a.g.p[r] = advance<G>(g.p[r], body);
        a.accum = accum ? accum + body : nullptr;
        a.master = master + body;
        a.m = m + body;
        a.v = v + body;
        a.out = out + body;
        a.n_tiles = rest;
        const uint32_t grid = (uint32_t)((rest + kWave - 1) / kWave);
        hipLaunchKernelGGL((update_tail<G>), dim3(grid), dim3(kWave), 0, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return (int)e;
    }
    return 0;
}

int launch_update(int dtype, uint32_t n_contrib, const ContribPtrs &g, const float *accum,
                  float *master, float *m, float *v, uint16_t *out, uint64_t count,
                  const StepScalars &s, void *stream)
{
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (dtype == PS_BF16)
        return launch_update_t<uint16_t>(n_contrib, g, accum, master, m, v, out, count, s, st);
    if (dtype == PS_F16)
        return launch_update_t<f16_bits>(n_contrib, g, accum, master, m, v, out, count, s, st);
    return launch_update_t<float>(n_contrib, g, accum, master, m, v, out, count, s, st);
}

template <int N, typename G>
static void launch_accum_n(const AccumArgs &a, uint32_t grid, hipStream_t st)
{
    if (a.overwrite)
        hipLaunchKernelGGL((accumulate_tiles<N, G, true>), dim3(grid), dim3(kWave), kAccumLdsBytes, st, a);
    else
        hipLaunchKernelGGL((accumulate_tiles<N, G, false>), dim3(grid), dim3(kWave), kAccumLdsBytes, st, a);
}

template <typename G>
static int launch_accum_t(uint32_t n_contrib, const ContribPtrs &g, float *accum, int overwrite,
                          uint64_t count, hipStream_t st)
{
    const uint64_t n_tiles = count / kTileElems;
    const uint64_t body = n_tiles * kTileElems;
    AccumArgs a;
    a.g = g;
    a.accum = accum;
    a.n_contrib = n_contrib;
    a.overwrite = overwrite ? 1u : 0u;
    if (n_tiles) {
        a.n_tiles = n_tiles;
        const uint32_t grid = grid_for(n_tiles);
        switch (n_contrib) {
        case 1: launch_accum_n<1, G>(a, grid, st); break;
        case 2: launch_accum_n<2, G>(a, grid, st); break;
        case 3: launch_accum_n<3, G>(a, grid, st); break;
        case 4: launch_accum_n<4, G>(a, grid, st); break;
        case 5: launch_accum_n<5, G>(a, grid, st); break;
        case 6: launch_accum_n<6, G>(a, grid, st); break;
        case 7: launch_accum_n<7, G>(a, grid, st); break;
        case 8: launch_accum_n<8, G>(a, grid, st); break;
        default: launch_accum_n<0, G>(a, grid, st); break; // 9..16: contribution loop not unrolled
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return (int)e;
    }
    if (count > body) {
        const uint64_t rest = count - body;
        for (uint32_t r = 0; r < n_contrib; ++r)
            a.g.p[r] = advance<G>(g.p[r], body);
        a.accum = accum + body;
        a.n_tiles = rest;
        hipLaunchKernelGGL((accumulate_tail<G>), dim3((uint32_t)((rest + kWave - 1) / kWave)),
                           dim3(kWave), 0, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return (int)e;
    }
    return 0;
}

int launch_accumulate(int dtype, uint32_t n_contrib, const ContribPtrs &g, float *accum,
                      int overwrite, uint64_t count, void *stream)
{
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (dtype == PS_BF16)
        return launch_accum_t<uint16_t>(n_contrib, g, accum, overwrite, count, st);
    if (dtype == PS_F16)
        return launch_accum_t<f16_bits>(n_contrib, g, accum, overwrite, count, st);
    return launch_accum_t<float>(n_contrib, g, accum, overwrite, count, st);
}

static uint64_t reduce_groups(uint64_t count)
{
    const uint64_t n_tiles = count / kTileElems;
    return (n_tiles + kReduceTilesPerGroup - 1) / kReduceTilesPerGroup;
}

uint64_t reduce_workspace_doubles(uint64_t count)
{
    return kFoldBlocks + reduce_groups(count) + 1; // second level, groups, tail
}

// Fold n first-level partials into at most kFoldBlocks sums (scratch `level2`),
// then into *out.  The slicing depends only on n.
template <typename T>
static int fold_to_one(const T *level1, T *level2, uint64_t n, T *out, int accumulate,
                       hipStream_t st)
{
    const T *last = level1;
    uint32_t n_last = (uint32_t)n;
    if (n > kFoldBlocks) {
        const uint64_t per = (n + kFoldBlocks - 1) / kFoldBlocks;
        const uint32_t blocks = (uint32_t)((n + per - 1) / per);
        hipLaunchKernelGGL((fold_partials<T>), dim3(blocks), dim3(kThreads), 0, st, level1, n, per,
                           level2);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return (int)e;
        last = level2;
        n_last = blocks;
    }
    hipLaunchKernelGGL((finalize_sum<T>), dim3(1), dim3(kThreads), 0, st, last, n_last, out,
                       accumulate);
    return (int)hipGetLastError();
}

template <int N, typename G>
static void launch_reduce_n(const ReduceArgs &a, uint32_t grid, hipStream_t st)
{
    hipLaunchKernelGGL((reduce_sumsq_tiles<N, G>), dim3(grid), dim3(kWave),
                       reduce_lds(sizeof(G) == 2 ? PS_BF16 : PS_F32), st, a);
}

template <typename G>
static int launch_reduce_t(uint32_t n_contrib, const ContribPtrs &g, float gs, float *reduced,
                           uint64_t count, double *workspace, double *sumsq_out, int accumulate,
                           hipStream_t st)
{
    const uint64_t n_tiles = count / kTileElems;
    const uint64_t body = n_tiles * kTileElems;
    const uint64_t groups = reduce_groups(count);
    if (groups >= UINT32_MAX) // the tail's partial slot is a 32-bit index
        return (int)hipErrorInvalidConfiguration;
    double *level2 = workspace;
    double *level1 = workspace + kFoldBlocks;
    uint64_t n_partials = 0;
    ReduceArgs a;
    a.g = g;
    a.reduced = reduced;
    a.partials = level1;
    a.n_contrib = n_contrib;
    a.partial_slot = 0;
    a.gs = gs;
    a.n_tiles = n_tiles;
    // Several launches of 2^27 elements each: over a long range the groups of
    // one launch drift apart and the request stream widens (6.4 against 6.7
    // TB/s over 2.2e9 elements); each launch boundary pulls them together again.
    for (uint64_t g0 = 0; g0 < groups; g0 += kReduceLaunchGroups) {
        a.first_group = g0;
        const uint32_t grid = (uint32_t)(groups - g0 < kReduceLaunchGroups ? groups - g0
                                                                          : kReduceLaunchGroups);
        switch (n_contrib) {
        case 1: launch_reduce_n<1, G>(a, grid, st); break;
        case 2: launch_reduce_n<2, G>(a, grid, st); break;
        case 3: launch_reduce_n<3, G>(a, grid, st); break;
        case 4: launch_reduce_n<4, G>(a, grid, st); break;
        case 5: launch_reduce_n<5, G>(a, grid, st); break;
        case 6: launch_reduce_n<6, G>(a, grid, st); break;
        case 7: launch_reduce_n<7, G>(a, grid, st); break;
        case 8: launch_reduce_n<8, G>(a, grid, st); break;
        default: launch_reduce_n<0, G>(a, grid, st); break; // 9..16: contribution loop not unrolled
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return (int)e;
    }
    n_partials = groups;
    a.first_group = 0;
    if (count > body) {
        for (uint32_t r = 0; r < n_contrib; ++r)
            a.g.p[r] = advance<G>(g.p[r], body);
        a.reduced = reduced ? reduced + body : nullptr;
        a.n_tiles = count - body;
        a.partial_slot = (uint32_t)n_partials;
        hipLaunchKernelGGL((reduce_sumsq_tail<G>), dim3(1), dim3(kWave), 0, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return (int)e;
        n_partials += 1;
    }
    return fold_to_one(level1, level2, n_partials, sumsq_out, accumulate, st);
}

int launch_reduce_sumsq(int dtype, uint32_t n_contrib, const ContribPtrs &g, float gs,
                        float *reduced_out, uint64_t count, double *partials, double *sumsq_out,
                        int accumulate, void *stream)
{
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (dtype == PS_BF16)
        return launch_reduce_t<uint16_t>(n_contrib, g, gs, reduced_out, count, partials,
                                         sumsq_out, accumulate, st);
    if (dtype == PS_F16)
        return launch_reduce_t<f16_bits>(n_contrib, g, gs, reduced_out, count, partials,
                                         sumsq_out, accumulate, st);
    return launch_reduce_t<float>(n_contrib, g, gs, reduced_out, count, partials, sumsq_out,
                                  accumulate, st);
}

// ---- partial sums for callers that cannot allocate ----
// The workspace of one reduce pass over PS_STATIC_MAX_ELEMS elements, held by every
// device the library runs on until the process ends (8 MiB + 8 KiB).  Host code never
// uses the array's name as an address: it asks the runtime once per device, with that
// device current, and passes the pointer it got to the kernels like any workspace.
constexpr uint64_t kScratchDoubles =
    kFoldBlocks + PS_STATIC_MAX_ELEMS / ((uint64_t)kTileElems * kReduceTilesPerGroup) + 1;
static __device__ __align__(256) double scratch[kScratchDoubles];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static double *scratch_ptr[kMaxDevices]; // per device: where its copy of `scratch` lives

int static_reduce_scratch(double **out, uint64_t *doubles)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return (int)e;
    if (dev < 0 || dev >= kMaxDevices)
        return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        double *p = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return (int)e;
        if (!p)
            return (int)hipErrorInvalidSymbol;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    *doubles = kScratchDoubles;
    return 0;
}

int launch_clip_coef(const double *sumsq_local, const double *sumsq_others, double max_norm,
                     float *coef_out, void *stream)
{
    hipLaunchKernelGGL(clip_coef_kernel, dim3(1), dim3(1), 0, reinterpret_cast<hipStream_t>(stream),
                       sumsq_local, sumsq_others, max_norm, coef_out);
    return (int)hipGetLastError();
}

// Workspace of the verification scans, in 8-byte slots, for a buffer of `bytes` bytes:
// two partial arrays (one partial per 32 KiB at most), each with its own second level.
uint64_t verify_workspace_slots(uint64_t bytes)
{
    const uint64_t group_bytes = (uint64_t)kScanThreads * kDiffVecs * 16;
    return 2 * (kFoldBlocks + bytes / group_bytes + 2);
}

// The single finishing workgroup adds up to kFinishDirect partials by itself (a few
// microseconds).  More than that go through one folding launch first: slices of at least
// kFoldSlice partials, at most kFoldBlocks of them, each added by its own workgroup (both
// quantities of the difference scan in the same launch).  The slicing depends only on the
// number of partials, so the tree is the same on every run.
constexpr uint64_t kFinishDirect = 4096;
constexpr uint64_t kFoldSlice = 2048;

template <typename T>
static int fold_for_finish(ScanArgs &s, void *l2a, void *l2b, uint64_t &n_partials, int quantities,
                           hipStream_t st)
{
    if (n_partials <= kFinishDirect)
        return 0;
    uint64_t per = (n_partials + kFoldBlocks - 1) / kFoldBlocks;
    if (per < kFoldSlice)
        per = kFoldSlice;
    const uint32_t blocks = (uint32_t)((n_partials + per - 1) / per);
    FoldArgs f;
    f.in[0] = s.partials0;
    f.in[1] = s.partials1;
    f.out[0] = l2a;
    f.out[1] = l2b;
    hipLaunchKernelGGL((fold_partials_q<T>), dim3(blocks, quantities), dim3(kThreads), 0, st, f,
                       n_partials, per);
    s.partials0 = l2a;
    s.partials1 = l2b;
    n_partials = blocks;
    return (int)hipGetLastError();
}

template <typename G>
static int launch_diff_t(const void *a, const void *b, uint64_t count, double *out2,
                         int accumulate, uint64_t *workspace, uint64_t slots, hipStream_t st)
{
    constexpr uint64_t kGroupElems = (uint64_t)kScanThreads * kDiffVecs * (16 / sizeof(G));
    const uint64_t groups = count / kGroupElems; // whole groups; the finishing workgroup takes the rest
    const uint64_t body = groups * kGroupElems;
    if (groups > kMaxGrid)
        return (int)hipErrorInvalidConfiguration;
    const uint64_t half = slots / 2;
    double *l2a = reinterpret_cast<double *>(workspace), *l1a = l2a + kFoldBlocks;
    double *l2b = l2a + half, *l1b = l2b + kFoldBlocks;
    ScanArgs s;
    s.a = a;
    s.b = b;
    s.partials0 = l1a;
    s.partials1 = l1b;
    s.first_index = 0;
    s.n_tiles = groups;
    uint64_t n_partials = groups;
    if (groups) {
        hipLaunchKernelGGL((diff_sumsq_tiles<G>), dim3((uint32_t)groups), dim3(kScanThreads), 0,
                           st, s);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return (int)e;
    }
    int fe = fold_for_finish<double>(s, l2a, l2b, n_partials, 2, st);
    if (fe != 0)
        return fe;
    s.a = advance<G>(a, body);
    s.b = advance<G>(b, body);
    s.n_tiles = count - body;
    hipLaunchKernelGGL((diff_sumsq_finish<G>), dim3(1), dim3(kScanThreads), 0, st, s, n_partials,
                       out2, accumulate);
    return (int)hipGetLastError();
}

int launch_diff_sumsq(int dtype, const void *a, const void *b, uint64_t count, double *out2,
                      int accumulate, void *workspace, uint64_t slots, void *stream)
{
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    uint64_t *ws = reinterpret_cast<uint64_t *>(workspace);
    if (dtype == PS_BF16)
        return launch_diff_t<uint16_t>(a, b, count, out2, accumulate, ws, slots, st);
    if (dtype == PS_F16)
        return launch_diff_t<f16_bits>(a, b, count, out2, accumulate, ws, slots, st);
    return launch_diff_t<float>(a, b, count, out2, accumulate, ws, slots, st);
}

int launch_checksum(const void *buf, uint64_t n_words, uint64_t first_index, uint64_t *out,
                    int accumulate, void *workspace, void *stream)
{
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    constexpr uint64_t kGroupWords = (uint64_t)kScanThreads * kChecksumVecs * 2;
    const uint64_t groups = n_words / kGroupWords; // whole groups; the finishing workgroup takes the rest
    const uint64_t body = groups * kGroupWords;
    if (groups > kMaxGrid)
        return (int)hipErrorInvalidConfiguration;
    uint64_t *l2 = reinterpret_cast<uint64_t *>(workspace), *l1 = l2 + kFoldBlocks;
    ScanArgs s;
    s.a = buf;
    s.b = nullptr;
    s.partials0 = l1;
    s.partials1 = nullptr;
    s.first_index = first_index;
    s.n_tiles = groups;
    uint64_t n_partials = groups;
    if (groups) {
        hipLaunchKernelGGL(checksum_tiles, dim3((uint32_t)groups), dim3(kScanThreads), 0, st, s);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return (int)e;
    }
    int fe = fold_for_finish<uint64_t>(s, l2, nullptr, n_partials, 1, st);
    if (fe != 0)
        return fe;
    s.a = reinterpret_cast<const uint64_t *>(buf) + body;
    s.first_index = first_index + body;
    s.n_tiles = n_words - body;
    hipLaunchKernelGGL(checksum_finish, dim3(1), dim3(kScanThreads), 0, st, s, n_partials, out,
                       accumulate);
    return (int)hipGetLastError();
}

int launch_copy(void *dst, const void *src, uint64_t bytes, void *stream)
{
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const uint64_t n_vec = bytes / 16;
    const uint64_t n_tiles = n_vec / kWave;
    uint32_t grid = grid_for(n_tiles);
    if (grid == 0)
        grid = 1;
    // one 16-B access per lane in flight: leave residency uncapped
    hipLaunchKernelGGL(copy_tiles, dim3(grid), dim3(kWave), 0, st,
                       reinterpret_cast<u32x4 *>(dst), reinterpret_cast<const u32x4 *>(src),
                       n_tiles, n_vec);
    return (int)hipGetLastError();
}

int launch_stage(uint32_t n_contrib, const ContribPtrs &src, void *dst, uint64_t slot_stride_bytes,
                 uint64_t first_vec, uint64_t period_vec, uint64_t n_vec, bool alone, void *stream)
{
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    constexpr int U = 4;
    const uint64_t groups = (n_vec + kWave * U - 1) / (kWave * U);
    if (groups == 0)
        return 0;
    if (groups > kMaxGrid)
        return (int)hipErrorInvalidConfiguration;
    StageArgs a;
    a.src = src;
    a.dst = reinterpret_cast<char *>(dst);
    a.slot_stride_bytes = slot_stride_bytes;
    a.first_vec = first_vec % period_vec;
    a.period_vec = period_vec;
    a.n_vec = n_vec;
    a.wrap_once = period_vec >= (uint64_t)kWave * U;
    hipLaunchKernelGGL((stage_bucket<U>), dim3((uint32_t)groups, n_contrib), dim3(kWave),
                       alone ? kStageAloneLdsBytes : 0u, st, a);
    return (int)hipGetLastError();
}

} // namespace ps
