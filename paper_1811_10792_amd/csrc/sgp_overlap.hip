// Step kernels of tau-overlap SGP (Alg. 2) at a communication round: every node keeps its own share
// and adds the messages that were sent one round earlier.
#include "internal.h"

#pragma clang fp contract(off)

using namespace sgp_detail;

namespace {
#include "device_common.inc"
#include "step_overlap.inc"

template <int V, int OPT, bool ZOUT>
void launch_delay_as(const StepArgs &a, size_t col0, long ncols, const float *msg_prev, float *msg_cur,
                     const int *tab_prev, int S, int ha, int hb)
{
    dim3 grid(grid_for(ncols, kDelayBlock * kDelayCols)), block(kDelayBlock);
    const size_t lds = weight_lds_bytes(a.n);
    const int nm = tab_prev ? S - 1 : 0;
    if (nm == 2 && SGP_DELAY_WINDOW) {   // two messages: each message row is loaded once
        const int stride = ((hb - ha) % a.n + a.n) % a.n;
        const int len = a.n / gcd_int(a.n, stride);
        hipLaunchKernelGGL((k_step_delay2<V, OPT, ZOUT>), grid, block, lds, a.stream, a.x, a.u, a.g, a.z,
                           a.wop, msg_prev, msg_cur, a.n, a.ld, col0, ncols, ha, hb, stride, len,
                           a.p, a.hp);
        *a.name = "k_step_delay2";
        return;
    }
    *a.name = "k_step_delay";
    if (nm == 0)
        hipLaunchKernelGGL((k_step_delay<V, OPT, ZOUT, 0>), grid, block, lds, a.stream, a.x, a.u, a.g,
                           a.z, a.wop, msg_prev, msg_cur, a.n, a.ld, col0, ncols, tab_prev, S,
                           a.p, a.hp);
    else if (nm == 1)
        hipLaunchKernelGGL((k_step_delay<V, OPT, ZOUT, 1>), grid, block, lds, a.stream, a.x, a.u, a.g,
                           a.z, a.wop, msg_prev, msg_cur, a.n, a.ld, col0, ncols, tab_prev, S,
                           a.p, a.hp);
#if !SGP_DELAY_WINDOW
    else if (nm == 2)
        hipLaunchKernelGGL((k_step_delay<V, OPT, ZOUT, 2>), grid, block, lds, a.stream, a.x, a.u, a.g,
                           a.z, a.wop, msg_prev, msg_cur, a.n, a.ld, col0, ncols, tab_prev, S,
                           a.p, a.hp);
#endif
    else
        hipLaunchKernelGGL((k_step_delay<V, OPT, ZOUT, -1>), grid, block, lds, a.stream, a.x, a.u, a.g,
                           a.z, a.wop, msg_prev, msg_cur, a.n, a.ld, col0, ncols, tab_prev, S,
                           a.p, a.hp);
}

template <int V, int OPT>
void launch_delay_opt(const StepArgs &a, bool zout, size_t col0, long ncols, const float *msg_prev, float *msg_cur,
                      const int *tab_prev, int S, int ha, int hb)
{
    if (zout) launch_delay_as<V, OPT, true>(a, col0, ncols, msg_prev, msg_cur, tab_prev, S, ha, hb);
    else launch_delay_as<V, OPT, false>(a, col0, ncols, msg_prev, msg_cur, tab_prev, S, ha, hb);
}
}  // namespace

namespace sgp_detail {

void launch_delay(const StepArgs &a, int V, int opt, bool zout, size_t col0, long ncols, const float *msg_prev,
                  float *msg_cur, const int *tab_prev, int S, int ha, int hb)
{
    auto with_v = [&]<int VV>() {
        if (opt == kOptAdam) launch_delay_opt<VV, kOptAdam>(a, zout, col0, ncols, msg_prev, msg_cur, tab_prev, S, ha, hb);
        else if (opt == kOptNesterov)
            launch_delay_opt<VV, kOptNesterov>(a, zout, col0, ncols, msg_prev, msg_cur, tab_prev, S, ha, hb);
        else launch_delay_opt<VV, kOptSgd>(a, zout, col0, ncols, msg_prev, msg_cur, tab_prev, S, ha, hb);
    };
    if (V == 4) with_v.template operator()<4>();
    else with_v.template operator()<1>();
}

}  // namespace sgp_detail
