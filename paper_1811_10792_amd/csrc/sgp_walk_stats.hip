// One-peer walk with the consensus statistics taken from registers (Alg. 1 / Alg. 3, and Alg. 2 with
// tau = 1 and two out-peers).  The unrolled bodies of one variant of the kernel take about half a
// minute to compile, so this file is compiled once per variant, side by side, with
//   -DSGP_WALK_NEST=0|1    local optimiser: gradient step / Nesterov momentum
//   -DSGP_WALK_CACHED=0|1  streaming / ordinary loads and stores
//   -DSGP_WALK_MSG=0|1|2   one iteration of delay with one / two out-peers (never together with CACHED)
// and each object defines the launcher of its variant.
#include "internal.h"

#pragma clang fp contract(off)

#ifndef SGP_WALK_NEST
#define SGP_WALK_NEST 1
#endif
#ifndef SGP_WALK_CACHED
#define SGP_WALK_CACHED 0
#endif
#ifndef SGP_WALK_MSG
#define SGP_WALK_MSG 0
#endif

using namespace sgp_detail;

namespace {
#include "device_common.inc"
#include "stats_tail.inc"
#include "step_walk_stats.inc"
}  // namespace

namespace sgp_detail {

template <>
void launch_walk_stats_variant<(SGP_WALK_NEST != 0), (SGP_WALK_CACHED != 0), SGP_WALK_MSG>(
    const StepArgs &a, long cols4, int h, int len, float *partial, hipEvent_t fin, const float *msg_prev,
    float *msg_cur, int ha, int hb)
{
    auto go = [&]<int NB>() {
        launch_step(k_step_one_peer_stats<(SGP_WALK_NEST != 0), (SGP_WALK_CACHED != 0), SGP_WALK_MSG, NB>,
                    dim3(grid_for(cols4, kStatsStepBlock)), dim3(kStatsStepBlock), weight_lds_bytes(a.n), a.stream,
                    fin, a.x, a.u, a.g, a.z, a.wop, a.n, a.ld, cols4, h, len, a.p, a.hp, partial, msg_prev, msg_cur,
                    ha, hb);
    };
    switch ((a.n + 3) / 4) {     // one kernel per group of four node counts
    case 0:
    case 1: go.template operator()<4>(); break;
    case 2: go.template operator()<8>(); break;
    case 3: go.template operator()<12>(); break;
    case 4: go.template operator()<16>(); break;
    case 5: go.template operator()<20>(); break;
    case 6: go.template operator()<24>(); break;
    case 7: go.template operator()<28>(); break;
    default: go.template operator()<32>(); break;
    }
}

}  // namespace sgp_detail
