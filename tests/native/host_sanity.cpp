// Host-only driver for the sanitizer test: exercises the placement evaluator and the
// strategy/composition helpers (no HIP calls) under AddressSanitizer and UBSan.
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "ps_step.h"

#define CHECK(cond)                                                                               \
    do {                                                                                          \
        if (!(cond)) {                                                                            \
            std::printf("FAILED %s:%d: %s (%s)\n", __FILE__, __LINE__, #cond, ps_last_error());   \
            return 1;                                                                             \
        }                                                                                         \
    } while (0)

int main()
{
    const char *names[] = {"dp", "zero1", "zero2", "zero3", "fsdp", "zero_offload", "tp", "pp"};
    const uint64_t P = 70000000000ull;
    for (const char *name : names) {
        ps_spec_t spec;
        ps_cost_t cost;
        CHECK(ps_spec_preset(name, 8, 3, P, &spec) == PS_OK);
        CHECK(ps_cost_eval(&spec, &cost) == PS_OK);
        CHECK(cost.persistent_total + cost.transient_bytes == cost.peak_total);
        CHECK(cost.shard_len * 8 == cost.psi_padded && cost.valid_len == cost.shard_len);
    }
    ps_spec_t spec;
    ps_cost_t cost;
    CHECK(ps_spec_preset("zero3", 8, 0, P, &spec) == PS_OK && ps_cost_eval(&spec, &cost) == PS_OK);
    CHECK(cost.peak_total == 140000000000ull);
    CHECK(cost.comm_total_bytes == 367.5e9);
    // every error path, including overflow and NULLs
    CHECK(ps_cost_eval(nullptr, &cost) == PS_EINVAL);
    CHECK(ps_cost_eval(&spec, nullptr) == PS_EINVAL);
    CHECK(ps_spec_preset(nullptr, 8, 0, P, &spec) == PS_EINVAL);
    CHECK(ps_spec_preset("nope", 8, 0, P, &spec) == PS_EINVAL);
    CHECK(std::strlen(ps_last_error()) > 0);
    CHECK(ps_spec_preset("dp", 4, 0, ~0ull, &spec) == PS_OK && ps_cost_eval(&spec, &cost) == PS_ERANGE);
    CHECK(ps_spec_preset("zero3", 6, 5, 13015864320ull - 1001, &spec) == PS_OK);
    spec.align_elems = 256;
    CHECK(ps_cost_eval(&spec, &cost) == PS_OK && cost.valid_len == cost.shard_len - 1001);
    spec.align_elems = 0xffffffffu; // N * align near 2^35: padded psi must not wrap
    CHECK(ps_cost_eval(&spec, &cost) == PS_OK || ps_cost_eval(&spec, &cost) == PS_ERANGE);
    int32_t fits = 0, tp = 0;
    CHECK(ps_select_strategy(P, 80000000000ull, 8, 30000000000ull, 1, &spec, &fits, &tp) == PS_OK);
    CHECK(!fits && tp && spec.theta == PS_SG);
    CHECK(ps_select_strategy(~0ull, ~0ull, 0xffffffffu, ~0ull, 1, &spec, &fits, &tp) == PS_OK);
    uint32_t a, b, c, d;
    CHECK(ps_compose_index(4, 2, 6, &a, &b, &c, &d) == PS_OK && a == 1 && b == 2 && c == 2 && d == 1);
    CHECK(ps_compose_index(65536, 65536, 0, &a, &b, &c, &d) == PS_ERANGE);
    CHECK(ps_spec_preset("dp", 2, 0, P, &spec) == PS_OK && ps_compose_cost(&spec, 4, &cost) == PS_OK);
    CHECK(cost.peak_total == 280000000000ull && cost.comm_total_bytes == 35e9);
    CHECK(ps_compose_cost(&spec, 0, &cost) == PS_EINVAL && ps_compose_cost(&spec, 3, &cost) == PS_ERANGE);
    CHECK(ps_compose_cost(nullptr, 4, &cost) == PS_EINVAL && ps_compose_cost(&spec, 4, nullptr) == PS_EINVAL);
    CHECK(ps_clip_coef(4.0, 12.0, 1.0) < 1.0 && ps_clip_coef(-1.0, 0.0, 1.0) != ps_clip_coef(-1.0, 0.0, 1.0));
    for (int st = 0; st < 9; ++st)
        CHECK(ps_status_string((ps_status_t)st) != nullptr);
    std::printf("host sanity ok\n");
    return 0;
}
