// Stand-alone check of the C ABI without Python: hipMalloc'd buffers, ps_step_update and
// ps_step_reduce_sumsq through include/ps_step.h, then a second step on arena buffers with
// the allocation-free reduce and the bucket loop that reads in place, all compared bit for
// bit with the C oracle (oracle/step.c, linked in as an object).  Test infrastructure,
// built by build().
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ps_step.h"

extern "C" {
typedef struct { float gs, cc, b1, omb1, b2, omb2, ep, step, isb2, lw; } oracle_scalars;
void oracle_derive_scalars(double, double, double, double, double, uint64_t, uint32_t, double, double,
                           oracle_scalars *);
void oracle_step_f32(const void *const *, uint32_t, int, const oracle_scalars *, float *, float *,
                     float *, uint16_t *, int, uint64_t, uint64_t);
double oracle_mean_sumsq(const void *const *, uint32_t, int, float, float *, uint64_t, uint64_t);
uint16_t oracle_bf16_rne(float);
}

#define HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define PS(x) do { ps_status_t s_ = (x); if (s_ != PS_OK) { std::printf("ps error %d (%s) at line %d\n", (int)s_, ps_last_error(), __LINE__); return 3; } } while (0)

// seeded inputs: a 64-bit LCG and sums of uniforms (bell-shaped, exact values do not matter)
static uint64_t g_state = 20260102;
static double uni() { g_state = g_state * 6364136223846793005ull + 1442695040888963407ull; return (double)(g_state >> 11) / 9007199254740992.0; }
static float bell(double sd) { double s = 0; for (int i = 0; i < 6; ++i) s += uni(); return (float)((s - 3.0) * 1.4142 * sd); }

template <typename T> static T *upload(const std::vector<T> &h)
{
    T *d = nullptr;
    if (hipMalloc((void **)&d, h.size() * sizeof(T)) != hipSuccess) return nullptr;
    if (hipMemcpy(d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
    return d;
}

int main()
{
    std::setvbuf(stdout, nullptr, _IONBF, 0);
    const uint32_t N = 6;
    const uint64_t n = 7 * 2048 + 250 + 3, valid = n - 5;
    std::printf("abi parity: n=%llu valid=%llu N=%u fp32 contributions\n", (unsigned long long)n, (unsigned long long)valid, N);
    ps_spec_t spec;
    PS(ps_spec_preset("zero3", N, 2, n * N, &spec));
    ps_cost_t cost;
    PS(ps_cost_eval(&spec, &cost));
    if (cost.shard_len != n) { std::printf("geometry\n"); return 1; }

    std::vector<std::vector<float>> g(N, std::vector<float>(n));
    for (auto &v : g) for (auto &x : v) x = bell(1e-3);
    std::vector<float> th(n), m(n), v(n);
    for (uint64_t e = 0; e < n; ++e) { th[e] = bell(0.02); m[e] = std::fabs(bell(1e-3)); float t = bell(1e-3); v[e] = t * t; }
    std::vector<uint16_t> p(n, 0xBEEF);

    // oracle
    std::vector<float> oth = th, om = m, ov = v;
    std::vector<uint16_t> op = p;
    const void *gp[N];
    for (uint32_t r = 0; r < N; ++r) gp[r] = g[r].data();
    oracle_scalars s;
    oracle_derive_scalars(3e-4, 0.9, 0.999, 1e-8, 0.1, 1000, N, 0.0, 0.0, &s);
    oracle_step_f32(gp, N, 1, &s, oth.data(), om.data(), ov.data(), op.data(), 0, 0, valid);
    std::vector<float> omean(n, -1.0f);
    const double oss = oracle_mean_sumsq(gp, N, 1, s.gs, omean.data(), 0, valid);

    // device
    void *dg[N];
    for (uint32_t r = 0; r < N; ++r) if (!(dg[r] = upload(g[r]))) return 2;
    float *dth = upload(th), *dm = upload(m), *dv = upload(v);
    uint16_t *dp = upload(p);
    std::vector<float> red_init(n, -1.0f);
    float *dred = upload(red_init);
    double *dss = nullptr;
    void *ws = nullptr;
    HIP(hipMalloc((void **)&dss, 8));
    HIP(hipMalloc(&ws, ps_workspace_bytes(n)));
    if (!dth || !dm || !dv || !dp || !dred) return 2;
    hipStream_t st;
    HIP(hipStreamCreate(&st));
    ps_adamw_t hp = {3e-4, 0.9, 0.999, 1e-8, 0.1, 1000, 0.0, 0.0};
    ps_shard_t sh = {dth, dm, dv, dp, n, valid};
    ps_grads_t gr = {(const void *const *)dg, N, PS_F32};
    PS(ps_step_reduce_sumsq(&spec, &gr, 0.0, dred, dss, 0, ws, ps_workspace_bytes(n), 0, n, valid, st));
    PS(ps_step_update(&spec, &hp, &sh, &gr, 0, n, st));
    HIP(hipStreamSynchronize(st));
    std::vector<float> rth(n), rm(n), rv(n), rred(n);
    std::vector<uint16_t> rp(n);
    double rss = 0;
    HIP(hipMemcpy(rth.data(), dth, n * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(rm.data(), dm, n * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(rv.data(), dv, n * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(rp.data(), dp, n * 2, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(rred.data(), dred, n * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(&rss, dss, 8, hipMemcpyDeviceToHost));

    int bad = 0;
    bad += std::memcmp(rth.data(), oth.data(), n * 4) != 0;
    bad += std::memcmp(rm.data(), om.data(), n * 4) != 0;
    bad += std::memcmp(rv.data(), ov.data(), n * 4) != 0;
    bad += std::memcmp(rp.data(), op.data(), n * 2) != 0;
    bad += std::memcmp(rred.data(), omean.data(), n * 4) != 0;          // pad (-1) included
    bad += !(std::fabs(rss - oss) <= 1e-12 * oss);
    for (uint64_t e = valid; e < n; ++e) bad += rp[e] != 0xBEEF;
    // ---- second step (t = 1001): arena buffers, allocation-free reduce, bucket loop in place ----
    oracle_scalars s2;
    oracle_derive_scalars(3e-4, 0.9, 0.999, 1e-8, 0.1, 1001, N, 0.0, 0.0, &s2);
    oracle_step_f32(gp, N, 1, &s2, oth.data(), om.data(), ov.data(), op.data(), 0, 0, valid);
    const uint32_t eb[N + 4] = {4, 4, 4, 4, 4, 4, 4, 4, 4, 2};        // six contributions, master, m, v, parameters
    ps_arena_t *arena = nullptr;
    PS(ps_arena_create(n, 1u << 20, eb, N + 4, &arena));
    void *ab[N + 4];
    for (uint32_t k = 0; k < N + 4; ++k) {
        ab[k] = ps_arena_buffer(arena, k);
        bad += ab[k] == nullptr || ((uintptr_t)ab[k] & ((2u << 20) - 1)) != 0;
    }
    bad += ps_arena_buffer(arena, N + 4) != nullptr;
    for (uint32_t r = 0; r < N; ++r) HIP(hipMemcpy(ab[r], dg[r], n * 4, hipMemcpyDeviceToDevice));
    HIP(hipMemcpy(ab[N], dth, n * 4, hipMemcpyDeviceToDevice));
    HIP(hipMemcpy(ab[N + 1], dm, n * 4, hipMemcpyDeviceToDevice));
    HIP(hipMemcpy(ab[N + 2], dv, n * 4, hipMemcpyDeviceToDevice));
    HIP(hipMemcpy(ab[N + 3], dp, n * 2, hipMemcpyDeviceToDevice));
    ps_grads_t gr2 = {(const void *const *)ab, N, PS_F32};
    PS(ps_step_reduce_sumsq_static(&spec, &gr2, 0.0, nullptr, dss, 0, 0, n, valid, st));
    ps_adamw_t hp2 = hp;
    hp2.step = 1001;
    ps_shard_t sh2 = {(float *)ab[N], (float *)ab[N + 1], (float *)ab[N + 2], ab[N + 3], n, valid};
    ps_bucket_plan_t plan;
    std::memset(&plan, 0, sizeof plan);
    plan.source = (const void *const *)ab;
    plan.n_contrib = N;
    plan.dtype = PS_F32;
    plan.bucket_elems = 4096;
    plan.source_elems = (n + 511) / 512 * 512;     // the arena rounds every buffer up to whole 2 MiB pages
    plan.compute_stream = st;
    plan.copy_engine = PS_COPY_NONE;
    PS(ps_step_update_bucketed(&spec, &hp2, &sh2, &plan));
    HIP(hipStreamSynchronize(st));
    double rss2 = 0;
    HIP(hipMemcpy(rth.data(), ab[N], n * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(rm.data(), ab[N + 1], n * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(rv.data(), ab[N + 2], n * 4, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(rp.data(), ab[N + 3], n * 2, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(&rss2, dss, 8, hipMemcpyDeviceToHost));
    bad += std::memcmp(rth.data(), oth.data(), n * 4) != 0;
    bad += std::memcmp(rm.data(), om.data(), n * 4) != 0;
    bad += std::memcmp(rv.data(), ov.data(), n * 4) != 0;
    bad += std::memcmp(rp.data(), op.data(), n * 2) != 0;
    bad += rss2 != rss;                                                 // same kernels, same tree, same bits
    PS(ps_arena_destroy(arena));
    // error path through the C ABI
    ps_grads_t missing = {(const void *const *)dg, N - 1, PS_F32};
    bad += ps_step_update(&spec, &hp, &sh, &missing, 0, n, st) != PS_EINVAL;
    bad += std::strlen(ps_last_error()) == 0;
    std::printf(bad ? "abi parity FAILED (%d)\n" : "abi parity ok\n", bad);
    return bad ? 1 : 0;
}
