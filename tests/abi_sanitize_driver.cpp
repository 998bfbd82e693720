// Host-side calls through the C ABI for a build of the library whose host code carries the
// compiler's address and undefined-behaviour sanitizers (tests/test_abi_sanitized.py builds both
// and runs this).  Every call here ends in the library's own argument and state checks, before
// any device work, so it runs on a machine without a GPU; pointers named `junk` are never
// dereferenced on these paths.  A wrong status ends the run with a message; a sanitizer report
// ends it by itself.
#include "../include/sja.h"

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

static int failures = 0;
#define EXPECT(call, want)                                                                     \
    do {                                                                                       \
        const long long got__ = (long long)(call);                                             \
        if (got__ != (long long)(want)) {                                                      \
            std::printf("line %d: %s gave %lld, expected %lld\n", __LINE__, #call, got__,    \
                        (long long)(want));                                                    \
            ++failures;                                                                        \
        }                                                                                      \
    } while (0)

int main()
{
    void *junk = reinterpret_cast<void *>(uintptr_t(256));
    const int32_t *ji = static_cast<const int32_t *>(junk);
    int32_t *jo = static_cast<int32_t *>(junk);
    const int64_t *jl = static_cast<const int64_t *>(junk);
    const uint8_t *jb = static_cast<const uint8_t *>(junk);
    int64_t *jlo = static_cast<int64_t *>(junk);

    for (int s = 0; s >= -9; --s) EXPECT(std::strlen(sja_status_string(s)) > 0, 1);
    EXPECT(sja_workspace_bytes(-1, 4, 4), 0);
    EXPECT(sja_workspace_bytes(4, 4, 16) > 0, 1);
    EXPECT(sja_workspace_bytes(SJA_MAX_GAPS, SJA_MAX_JOBS, SJA_MAX_SEGMENTS) >= 0, 1);

    sja_ctx *h = nullptr;
    EXPECT(sja_create(nullptr, 0), SJA_ERR_NULL);
    EXPECT(sja_create(&h, -1), SJA_ERR_SIZE);
    EXPECT(sja_create(&h, 0), SJA_OK);
    EXPECT(std::strlen(sja_last_error(nullptr)) > 0, 1);

    sja_params par;
    std::memset(&par, 0, sizeof par);
    par.policy = SJA_POLICY_MIXED;
    par.wait_scale = 1000;
    par.sla_weight[0] = 4; par.sla_weight[1] = 2; par.sla_weight[2] = 1;

    // calls out of sequence
    EXPECT(sja_fit(h, nullptr, 4, ji, ji, jo, nullptr), SJA_ERR_STATE);
    EXPECT(sja_fit_select(h, nullptr, 4, ji, ji, &par, ji, jb, nullptr, nullptr, jo, jo, jlo), SJA_ERR_STATE);
    EXPECT(sja_select(h, nullptr, &par, ji, jb, nullptr, nullptr, jo, jo, jlo), SJA_ERR_STATE);
    EXPECT(sja_resolve(h, nullptr, &par, ji, jb, jo, jo, jlo, jo, jo), SJA_ERR_STATE);
    EXPECT(sja_advance(h, nullptr, 4, ji, ji, ji, ji, ji, jo, jo, 1, jlo), SJA_ERR_STATE);
    EXPECT(sja_cover(h, nullptr, 4, ji, ji, ji, 2, ji, jo, jo), SJA_ERR_STATE);
    float ms = 0.f;
    EXPECT(sja_last_fit_kernel_ms(h, &ms), SJA_ERR_STATE);
    EXPECT(sja_last_fit_kernel_ms(h, nullptr), SJA_ERR_NULL);

    // prepare: sizes, nulls, workspace
    EXPECT(sja_prepare_profiles(h, nullptr, -1, 10, jl, ji, ji, jb, ji, jo, jo, jo), SJA_ERR_SIZE);
    EXPECT(sja_prepare_profiles(h, nullptr, 4, -1, jl, ji, ji, jb, ji, jo, jo, jo), SJA_ERR_SIZE);
    EXPECT(sja_prepare_profiles(h, nullptr, 4, 10, nullptr, ji, ji, jb, ji, jo, jo, jo), SJA_ERR_NULL);
    EXPECT(sja_prepare_profiles(h, nullptr, 4, 10, jl, ji, ji, jb, ji, jo, jo, nullptr), SJA_ERR_NULL);
    EXPECT(sja_prepare_profiles(h, nullptr, 4, 10, jl, ji, ji, jb, ji, jo, jo, jo), SJA_ERR_WORKSPACE);
    EXPECT(std::strstr(sja_last_error(h), "workspace") != nullptr, 1);
    EXPECT(sja_set_workspace(h, reinterpret_cast<void *>(uintptr_t(257)), 1 << 20), SJA_ERR_WORKSPACE);
    EXPECT(sja_set_workspace(h, nullptr, 1 << 20), SJA_ERR_NULL);
    EXPECT(sja_set_workspace(h, reinterpret_cast<void *>(uintptr_t(512)), 16), SJA_OK);
    EXPECT(sja_prepare_profiles(h, nullptr, 4, 10, jl, ji, ji, jb, ji, jo, jo, jo), SJA_ERR_WORKSPACE);
    EXPECT(sja_prepare_profiles_static(h, nullptr, 32768, int64_t(1) << 25, jl, ji, ji, jb, ji, jo, jo, jo), SJA_ERR_SIZE);
    EXPECT(std::strstr(sja_last_error(h), "built-in scratch") != nullptr, 1);
    EXPECT(sja_prepare_profiles_static(h, nullptr, 4, 64, nullptr, ji, ji, jb, ji, jo, jo, jo), SJA_ERR_NULL);

    // validate: sizes, nulls, policy
    uint32_t *jw = static_cast<uint32_t *>(junk);
    EXPECT(sja_validate(h, nullptr, -1, 0, jl, nullptr, nullptr, ji, nullptr, nullptr, nullptr, jw), SJA_ERR_SIZE);
    EXPECT(sja_validate(h, nullptr, 4, 8, nullptr, ji, ji, ji, nullptr, nullptr, nullptr, jw), SJA_ERR_NULL);
    EXPECT(sja_validate(h, nullptr, 4, 8, jl, ji, ji, ji, nullptr, nullptr, nullptr, nullptr), SJA_ERR_NULL);
    sja_params bad = par;
    bad.policy = 7;
    EXPECT(sja_validate(h, nullptr, 4, 8, jl, ji, ji, ji, &bad, ji, jb, jw), SJA_ERR_POLICY);

    // switches that are host bookkeeping only
    EXPECT(sja_set_resolve_mode(h, SJA_RESOLVE_LISTS), SJA_OK);
    EXPECT(sja_set_resolve_mode(h, SJA_RESOLVE_MATRIX), SJA_OK);
    EXPECT(sja_set_resolve_mode(h, 7), SJA_ERR_SIZE);
    EXPECT(sja_set_resolve_mode(h, SJA_RESOLVE_LISTS), SJA_OK);
    EXPECT(sja_set_score(h, SJA_SCORE_AREA), SJA_OK);
    EXPECT(sja_set_score(h, 5), SJA_ERR_SIZE);
    EXPECT(sja_set_score(h, SJA_SCORE_RECTANGLE), SJA_OK);
    EXPECT(sja_enable_timing(h, 1), SJA_OK);
    EXPECT(sja_enable_timing(h, 0), SJA_OK);

    sja_limits lim;
    lim.tau_min = 3; lim.tau_max = 9; lim.power_cap = 5; lim.now = 1;
    EXPECT(sja_set_limits(h, &lim, ji, ji), SJA_OK);
    lim.tau_min = -1;
    EXPECT(sja_set_limits(h, &lim, nullptr, nullptr), SJA_ERR_SIZE);
    lim.tau_min = 0; lim.tau_max = -1;
    EXPECT(sja_set_limits(h, &lim, nullptr, nullptr), SJA_ERR_SIZE);
    EXPECT(sja_set_limits(h, nullptr, nullptr, nullptr), SJA_OK);
    EXPECT(sja_set_limits(nullptr, nullptr, nullptr, nullptr), SJA_ERR_NULL);

    // hysteresis: the set is copied, exactly SJA_MAX_CAPS entries fit
    int32_t *caps = static_cast<int32_t *>(std::malloc(sizeof(int32_t) * SJA_MAX_CAPS));   // exact size: reads past it are reported
    for (int i = 0; i < SJA_MAX_CAPS; ++i) caps[i] = 10 * (i + 1);
    EXPECT(sja_set_hysteresis(h, SJA_MAX_CAPS, caps, 10), SJA_OK);
    EXPECT(sja_set_hysteresis(h, SJA_MAX_CAPS + 1, caps, 10), SJA_ERR_SIZE);
    EXPECT(sja_set_hysteresis(h, 3, caps, 0), SJA_ERR_SIZE);
    EXPECT(sja_set_hysteresis(h, -1, caps, 1), SJA_ERR_SIZE);
    EXPECT(sja_set_hysteresis(h, 2, nullptr, 1), SJA_ERR_NULL);
    caps[1] = 5;
    EXPECT(sja_set_hysteresis(h, 3, caps, 1), SJA_ERR_SIZE);
    EXPECT(sja_set_hysteresis(h, 0, nullptr, 0), SJA_OK);
    std::free(caps);

    // null contexts everywhere
    EXPECT(sja_fit(nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr), SJA_ERR_NULL);
    EXPECT(sja_resolve(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr), SJA_ERR_NULL);
    EXPECT(sja_advance(nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr), SJA_ERR_NULL);
    EXPECT(sja_cover(nullptr, nullptr, 0, nullptr, nullptr, nullptr, 0, nullptr, nullptr, nullptr), SJA_ERR_NULL);
    EXPECT(sja_set_hysteresis(nullptr, 0, nullptr, 0), SJA_ERR_NULL);

    EXPECT(sja_destroy(h), SJA_OK);
    EXPECT(sja_destroy(nullptr), SJA_ERR_NULL);
    if (failures) {
        std::printf("%d unexpected results\n", failures);
        return 1;
    }
    std::printf("host ABI checks passed\n");
    return 0;
}
