// Optional per-kernel timing with HIP events, for benchmarks.  Off by default; when on, every
// kernel launch of the selected level is bracketed by two events recorded on the launch stream.
#include "common.h"

#include <vector>

namespace relibra {

struct ProfState {
    int level = 0;
    std::vector<hipEvent_t> pool;     // 2 events per record
    std::vector<int> ids;
    size_t used = 0;
};
static ProfState g_prof;

static inline int prof_level_of(int id) { return (id >= RELIBRA_K_FWD_GATE_UP && id <= RELIBRA_K_WGRAD_GATE_UP) ? 1 : 2; }

bool prof_before(int id, hipStream_t s)
{
    ProfState &p = g_prof;
    if (p.level < prof_level_of(id) || p.used >= p.ids.size()) return false;
    return hipEventRecord(p.pool[2 * p.used], s) == hipSuccess;
}

void prof_after(int id, hipStream_t s)
{
    ProfState &p = g_prof;
    if (hipEventRecord(p.pool[2 * p.used + 1], s) == hipSuccess) p.ids[p.used++] = id;
}

}  // namespace relibra

using namespace relibra;

extern "C" int relibra_prof_start(int level, int max_records)
{
    ProfState &p = g_prof;
    if (level < 0 || level > 2 || max_records < 0) return RELIBRA_EINVAL;
    p.level = 0;
    p.used = 0;
    while (p.pool.size() < 2 * (size_t)max_records) {
        hipEvent_t e;
        RELIBRA_HIP_TRY(hipEventCreate(&e));
        p.pool.push_back(e);
    }
    p.ids.assign((size_t)max_records, -1);
    p.level = level;
    return RELIBRA_OK;
}

extern "C" int relibra_prof_stop(double *ms_by_kernel, int64_t *launches_by_kernel)
{
    ProfState &p = g_prof;
    p.level = 0;
    if (!ms_by_kernel || !launches_by_kernel) return RELIBRA_EINVAL;
    for (int i = 0; i < RELIBRA_K_COUNT; ++i) { ms_by_kernel[i] = 0.0; launches_by_kernel[i] = 0; }
    for (size_t r = 0; r < p.used; ++r) {
        RELIBRA_HIP_TRY(hipEventSynchronize(p.pool[2 * r + 1]));
        float ms = 0.0f;
        RELIBRA_HIP_TRY(hipEventElapsedTime(&ms, p.pool[2 * r], p.pool[2 * r + 1]));
        ms_by_kernel[p.ids[r]] += ms;
        launches_by_kernel[p.ids[r]] += 1;
    }
    p.used = 0;
    return RELIBRA_OK;
}
