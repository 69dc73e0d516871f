// Step kernel for several out-peers per node or caller-supplied mixing rows (Alg. 1 / Alg. 3 with a
// general sparse P^(k)): every work-item gathers its column of local steps into a private LDS column
// and forms the rows' sums from there; optionally with the consensus statistics.
#include "internal.h"

#pragma clang fp contract(off)

using namespace sgp_detail;

namespace {
#include "device_common.inc"
#include "stats_tail.inc"
#include "step_gather.inc"

template <int V, int OPT, bool ZOUT, bool STATS>
void launch_gather_as(const StepArgs &a, size_t col0, long ncols, const int *tab, const float *tabw, int S,
                      float *partial, hipEvent_t fin)
{
    const size_t lds = gather_lds_bytes(a.n, V);
    dim3 grid(grid_for(ncols, kGatherBlock)), block(kGatherBlock);
    auto go = [&](auto kernel) {
        // more than 64 KiB of dynamic LDS has to be asked for per kernel (a failure shows up as the
        // launch error that the caller checks)
        if (lds > 64 * 1024)
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        launch_step(kernel, grid, block, lds, a.stream, fin, a.x, a.u, a.g, a.z, a.wop, a.n, a.ld, col0, ncols,
                    tab, tabw, S, a.p, a.hp, partial);
    };
    if (tabw) go(k_step_gather<V, OPT, ZOUT, true, STATS>);
    else go(k_step_gather<V, OPT, ZOUT, false, STATS>);
    *a.name = STATS ? "k_step_gather_stats" : "k_step_gather";
}

template <int V, int OPT>
void launch_gather_opt(const StepArgs &a, bool zout, bool stats, size_t col0, long ncols, const int *tab,
                       const float *tabw, int S, float *partial, hipEvent_t fin)
{
    if constexpr (V == 4 && OPT != kOptAdam) {
        if (stats) {
            launch_gather_as<4, OPT, true, true>(a, col0, ncols, tab, tabw, S, partial, fin);
            return;
        }
    }
    if (zout) launch_gather_as<V, OPT, true, false>(a, col0, ncols, tab, tabw, S, nullptr, nullptr);
    else launch_gather_as<V, OPT, false, false>(a, col0, ncols, tab, tabw, S, nullptr, nullptr);
}
}  // namespace

namespace sgp_detail {

void launch_gather(const StepArgs &a, int V, int opt, bool zout, bool stats, size_t col0, long ncols, const int *tab,
                   const float *tabw, int S, float *partial, hipEvent_t fin)
{
    auto with_v = [&]<int VV>() {
        if (opt == kOptAdam) launch_gather_opt<VV, kOptAdam>(a, zout, stats, col0, ncols, tab, tabw, S, partial, fin);
        else if (opt == kOptNesterov)
            launch_gather_opt<VV, kOptNesterov>(a, zout, stats, col0, ncols, tab, tabw, S, partial, fin);
        else launch_gather_opt<VV, kOptSgd>(a, zout, stats, col0, ncols, tab, tabw, S, partial, fin);
    };
    if (V == 4) with_v.template operator()<4>();
    else with_v.template operator()<1>();
}

}  // namespace sgp_detail
