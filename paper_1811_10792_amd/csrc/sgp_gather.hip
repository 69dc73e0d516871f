// Step kernel for several out-peers per node or caller-supplied mixing rows (Alg. 1 / Alg. 3 with a
// general sparse P^(k)): every work-item gathers its column of local steps into a private LDS column
// and forms the rows' sums from there; optionally with the consensus statistics.
// Compiled twice, side by side: as is for the plain kernels (launch_gather), and with
// -DSGP_GATHER_STATS=1 for the kernels with statistics (launch_gather_stats).
#include "internal.h"

#ifndef SGP_GATHER_STATS
#define SGP_GATHER_STATS 0
#endif

#pragma clang fp contract(off)

using namespace sgp_detail;

namespace {
#include "device_common.inc"
#include "stats_tail.inc"
#include "step_gather.inc"

template <int V, int OPT, bool ZOUT, bool STATS, int NB, bool MANY>
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
    if (tabw) go(k_step_gather<V, OPT, ZOUT, true, STATS, NB, MANY>);
    else go(k_step_gather<V, OPT, ZOUT, false, STATS, NB, MANY>);
    *a.name = STATS ? "k_step_gather_stats" : "k_step_gather";
}

}  // namespace

namespace sgp_detail {

#if SGP_GATHER_STATS

void launch_gather_stats(const StepArgs &a, int opt, long ncols, const int *tab, const float *tabw, int S,
                         float *partial, hipEvent_t fin)
{
    auto with_opt = [&]<int OPT>() {     // one kernel per range of node counts
        if (a.n <= 8) launch_gather_as<4, OPT, true, true, 8, false>(a, 0, ncols, tab, tabw, S, partial, fin);
        else if (a.n <= 16) launch_gather_as<4, OPT, true, true, 16, false>(a, 0, ncols, tab, tabw, S, partial, fin);
        else launch_gather_as<4, OPT, true, true, 32, true>(a, 0, ncols, tab, tabw, S, partial, fin);
    };
    if (opt == kOptNesterov) with_opt.template operator()<kOptNesterov>();
    else with_opt.template operator()<kOptSgd>();
}

#else

void launch_gather(const StepArgs &a, int V, int opt, bool zout, size_t col0, long ncols, const int *tab,
                   const float *tabw, int S)
{
    auto with = [&]<int VV, int OPT>() {
        auto with_z = [&]<bool ZOUT>() {
            // the deeper pipeline for many nodes exists for the 128-bit layout only
            if constexpr (VV == 4) {
                if (a.n > 16) {
                    launch_gather_as<VV, OPT, ZOUT, false, kStatsCache, true>(a, col0, ncols, tab, tabw, S, nullptr,
                                                                               nullptr);
                    return;
                }
            }
            launch_gather_as<VV, OPT, ZOUT, false, kStatsCache, false>(a, col0, ncols, tab, tabw, S, nullptr, nullptr);
        };
        if (zout) with_z.template operator()<true>();
        else with_z.template operator()<false>();
    };
    auto with_v = [&]<int VV>() {
        if (opt == kOptAdam) with.template operator()<VV, kOptAdam>();
        else if (opt == kOptNesterov) with.template operator()<VV, kOptNesterov>();
        else with.template operator()<VV, kOptSgd>();
    };
    if (V == 4) with_v.template operator()<4>();
    else with_v.template operator()<1>();
}

#endif

}  // namespace sgp_detail
