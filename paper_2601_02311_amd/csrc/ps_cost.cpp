// Host-only part of the library: status text, Table 2 presets, and the
// derivation rules that turn a placement specification into bytes per device,
// bytes communicated per step and the shard's index range.  No HIP calls here.
#include <cmath>
#include <cstdio>
#include <cstring>

#include "ps_internal.h"

namespace ps {

static thread_local char g_last_error[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
    va_end(ap);
}

void clear_error() { g_last_error[0] = '\0'; }

static bool mode_ok(int32_t m) { return m >= PS_R && m <= PS_O; }

ps_status_t check_spec(const ps_spec_t *s)
{
    if (!s) {
        set_error("spec is NULL");
        return PS_EINVAL;
    }
    if (!mode_ok(s->theta) || !mode_ok(s->omega) || !mode_ok(s->grad) || !mode_ok(s->act)) {
        set_error("placement mode outside {R,S,S*,M,O}");
        return PS_EINVAL;
    }
    if (s->reserved != 0) {
        set_error("spec.reserved must be 0");
        return PS_EINVAL;
    }
    if (s->n_devices == 0) {
        set_error("n_devices must be >= 1");
        return PS_EINVAL;
    }
    if (s->shard_index >= s->n_devices) {
        set_error("shard_index %u not below n_devices %u", s->shard_index, s->n_devices);
        return PS_ERANGE;
    }
    return PS_OK;
}

// Eq. 2 with the padding rule: psi_padded = ceil(psi / (N*a)) * N*a, shard i is
// [i*n, (i+1)*n) with n = psi_padded / N; what lies beyond psi is padding.
ps_status_t shard_geometry(const ps_spec_t *s, uint64_t *psi_padded, uint64_t *offset,
                           uint64_t *len, uint64_t *valid)
{
    const uint64_t N = s->n_devices;
    const uint64_t a = s->align_elems > 1 ? s->align_elems : 1;
    const uint64_t unit = N * a; // both below 2^32
    if (a == 1 && s->psi % N != 0) {
        set_error("n_devices %llu does not divide psi %llu (set align_elems to pad)",
                  (unsigned long long)N, (unsigned long long)s->psi);
        return PS_ERANGE;
    }
    const uint64_t q = s->psi / unit + (s->psi % unit != 0);
    if (q != 0 && unit > UINT64_MAX / q) {
        set_error("padded psi overflows 64 bits");
        return PS_ERANGE;
    }
    const uint64_t padded = q * unit;
    const uint64_t n = padded / N;
    const uint64_t off = (uint64_t)s->shard_index * n;
    uint64_t val = 0;
    if (s->psi > off)
        val = s->psi - off < n ? s->psi - off : n;
    *psi_padded = padded;
    *offset = off;
    *len = n;
    *valid = val;
    return PS_OK;
}

// mu(pi, s) of Theorem 1 split into its persistent part and the s_unit part.
static ps_status_t mu(int32_t mode, uint64_t s, uint64_t N, uint64_t s_unit,
                      uint64_t *persistent, uint64_t *transient)
{
    *persistent = 0;
    *transient = 0;
    switch (mode) {
    case PS_R:
        *persistent = s;
        return PS_OK;
    case PS_S:
    case PS_SG:
        if (s % N != 0) {
            set_error("state of %llu bytes is not divisible by N=%llu",
                      (unsigned long long)s, (unsigned long long)N);
            return PS_ERANGE;
        }
        *persistent = s / N;
        if (mode == PS_SG)
            *transient = s_unit;
        return PS_OK;
    case PS_M:
        *transient = s_unit;
        return PS_OK;
    case PS_O:
        return PS_OK;
    }
    return PS_EINVAL;
}

static bool add_ok(uint64_t a, uint64_t b, uint64_t *out)
{
    if (a > UINT64_MAX - b)
        return false;
    *out = a + b;
    return true;
}

static bool mul_ok(uint64_t a, uint64_t b, uint64_t *out)
{
    if (a != 0 && b > UINT64_MAX / a)
        return false;
    *out = a * b;
    return true;
}

} // namespace ps

using namespace ps;

extern "C" {

uint32_t ps_abi_version(void) { return PS_ABI_VERSION; }

const char *ps_status_string(ps_status_t st)
{
    switch (st) {
    case PS_OK: return "ok";
    case PS_EINVAL: return "invalid argument";
    case PS_EUNSUPPORTED: return "placement not executed by this path";
    case PS_EALIGN: return "pointer or offset not 16-byte aligned";
    case PS_ERANGE: return "size or index out of range";
    case PS_ENODEVICE: return "no HIP device";
    case PS_EHIP: return "HIP call failed";
    }
    return "unknown status";
}

const char *ps_last_error(void) { return g_last_error; }

ps_status_t ps_spec_preset(const char *name, uint32_t n_devices, uint32_t shard_index,
                           uint64_t psi, ps_spec_t *spec)
{
    clear_error();
    if (!name || !spec) {
        set_error("name or spec is NULL");
        return PS_EINVAL;
    }
    // Table 2: (pi_Theta, pi_Omega, pi_G, pi_A)
    static const struct {
        const char *name;
        int32_t th, om, g, a;
    } rows[] = {
        {"dp", PS_R, PS_R, PS_R, PS_R},
        {"zero1", PS_R, PS_S, PS_R, PS_R},
        {"zero2", PS_R, PS_S, PS_S, PS_R},
        {"zero3", PS_SG, PS_S, PS_S, PS_R},
        {"fsdp", PS_SG, PS_S, PS_S, PS_R},
        {"zero_offload", PS_O, PS_O, PS_S, PS_R},
        {"tp", PS_S, PS_S, PS_S, PS_S},
        {"pp", PS_S, PS_S, PS_S, PS_R},
    };
    for (const auto &r : rows) {
        if (std::strcmp(name, r.name) == 0) {
            std::memset(spec, 0, sizeof *spec);
            spec->theta = r.th;
            spec->omega = r.om;
            spec->grad = r.g;
            spec->act = r.a;
            spec->n_devices = n_devices;
            spec->shard_index = shard_index;
            spec->psi = psi;
            return PS_OK;
        }
    }
    set_error("unknown strategy '%s'", name);
    return PS_EINVAL;
}

double ps_clip_coef(double sumsq_local, double sumsq_others, double max_norm)
{
    const double total = sumsq_local + sumsq_others;
    if (!std::isfinite(total) || sumsq_local < 0.0 || sumsq_others < 0.0 || !(max_norm > 0.0))
        return std::nan("");
    const double coef = max_norm / (std::sqrt(total) + 1e-6);
    return coef < 1.0 ? coef : 1.0;
}

ps_status_t ps_select_strategy(uint64_t psi, uint64_t device_mem_bytes, uint32_t n_devices,
                               uint64_t layer_bytes, int32_t fast_interconnect, ps_spec_t *spec,
                               int32_t *fits, int32_t *add_tp)
{
    clear_error();
    if (!spec || !fits || !add_tp) {
        set_error("spec, fits or add_tp is NULL");
        return PS_EINVAL;
    }
    if (n_devices == 0) {
        set_error("n_devices must be >= 1");
        return PS_EINVAL;
    }
    // 16 psi < 0.7 M  <=>  160 psi < 7 M, in 128-bit integers
    const unsigned __int128 model10 = (unsigned __int128)psi * 160u;
    const unsigned __int128 cap7 = (unsigned __int128)device_mem_bytes * 7u;
    *add_tp = 0;
    if (model10 < cap7) {
        *fits = 1;
        return ps_spec_preset("dp", n_devices, 0, psi, spec);
    }
    // 16 psi / N < 0.7 M  <=>  160 psi < 7 M N
    *fits = model10 < cap7 * n_devices ? 1 : 0;
    if (!*fits && fast_interconnect &&
        (unsigned __int128)layer_bytes * 10u > (unsigned __int128)device_mem_bytes * 3u)
        *add_tp = 1;
    return ps_spec_preset("zero3", n_devices, 0, psi, spec);
}

ps_status_t ps_compose_index(uint32_t inner, uint32_t outer, uint32_t device,
                             uint32_t *inner_group, uint32_t *inner_rank,
                             uint32_t *outer_group, uint32_t *outer_rank)
{
    clear_error();
    if (!inner_group || !inner_rank || !outer_group || !outer_rank) {
        set_error("an output pointer is NULL");
        return PS_EINVAL;
    }
    if (inner == 0 || outer == 0) {
        set_error("group sizes must be >= 1");
        return PS_EINVAL;
    }
    if ((uint64_t)inner * outer > UINT32_MAX || device >= (uint64_t)inner * outer) {
        set_error("device %u not below inner * outer = %llu", device,
                  (unsigned long long)inner * outer);
        return PS_ERANGE;
    }
    *inner_group = device / inner;
    *inner_rank = device % inner;
    *outer_group = *inner_rank;
    *outer_rank = *inner_group;
    return PS_OK;
}

ps_status_t ps_compose_cost(const ps_spec_t *outer, uint32_t inner, ps_cost_t *cost)
{
    clear_error();
    if (!outer || !cost) {
        set_error("outer or cost is NULL");
        return PS_EINVAL;
    }
    if (inner == 0) {
        set_error("inner degree must be >= 1");
        return PS_EINVAL;
    }
    if (outer->psi % inner != 0) {
        set_error("inner degree %u does not divide psi = %llu", inner,
                  (unsigned long long)outer->psi);
        return PS_ERANGE;
    }
    // Each device of the outer group holds the same 1/inner of every state; the
    // outer rules then act on that share among the group's devices.
    ps_spec_t local = *outer;
    local.psi = outer->psi / inner;
    return ps_cost_eval(&local, cost);
}

ps_status_t ps_cost_eval(const ps_spec_t *spec, ps_cost_t *cost)
{
    clear_error();
    if (!cost) {
        set_error("cost is NULL");
        return PS_EINVAL;
    }
    ps_status_t st = check_spec(spec);
    if (st != PS_OK)
        return st;
    std::memset(cost, 0, sizeof *cost);
    const uint64_t N = spec->n_devices;

    // Shard geometry first: byte sizes are taken on the padded length, which is
    // what the flat buffers hold (equal to psi whenever N divides psi).
    st = shard_geometry(spec, &cost->psi_padded, &cost->shard_offset, &cost->shard_len,
                        &cost->valid_len);
    if (st != PS_OK)
        return st;

    // Remark 1: |Theta| = 2P, |G| = 2P, |Omega| = 12P bytes.
    uint64_t theta, omega, grad;
    if (!mul_ok(cost->psi_padded, 2, &theta) || !mul_ok(cost->psi_padded, 12, &omega)) {
        set_error("12*psi overflows 64 bits");
        return PS_ERANGE;
    }
    grad = theta;

    uint64_t tr[4];
    if ((st = mu(spec->theta, theta, N, spec->s_unit_bytes, &cost->theta_bytes, &tr[0])) ||
        (st = mu(spec->omega, omega, N, spec->s_unit_bytes, &cost->omega_bytes, &tr[1])) ||
        (st = mu(spec->grad, grad, N, spec->s_unit_bytes, &cost->grad_bytes, &tr[2])) ||
        (st = mu(spec->act, spec->act_bytes, N, spec->s_unit_bytes, &cost->act_bytes, &tr[3])))
        return st;
    uint64_t t = 0, p = 0;
    bool ok = add_ok(tr[0], tr[1], &t) && add_ok(t, tr[2], &t) && add_ok(t, tr[3], &t) &&
              add_ok(cost->theta_bytes, cost->omega_bytes, &p) &&
              add_ok(p, cost->grad_bytes, &p) && add_ok(p, cost->act_bytes, &p);
    cost->transient_bytes = t;
    cost->persistent_total = p;
    ok = ok && add_ok(p, t, &cost->peak_total);

    // Theorem 2 with the ring costs: All-Reduce 2(N-1)/N |T|, Reduce-Scatter and
    // All-Gather (N-1)/N |T|; kept multiplied by N.
    uint64_t g_x = 0, th_x = 0;
    ok = ok && mul_ok(grad, N - 1, &g_x) && mul_ok(theta, N - 1, &th_x);
    if (spec->grad == PS_R)
        ok = ok && mul_ok(g_x, 2, &cost->comm_grad_sync_xN);
    else if (spec->grad == PS_S)
        cost->comm_grad_sync_xN = g_x;
    if (spec->theta == PS_SG)
        ok = ok && mul_ok(th_x, 2, &cost->comm_param_gather_xN);
    if (!ok) {
        set_error("cost overflows 64 bits");
        return PS_ERANGE;
    }
    cost->comm_total_bytes =
        ((double)cost->comm_grad_sync_xN + (double)cost->comm_param_gather_xN) / (double)N;
    if (spec->theta == PS_R && (spec->omega == PS_S || spec->omega == PS_SG))
        cost->implied_update_gather_xN = th_x;

    return PS_OK;
}

} // extern "C"
