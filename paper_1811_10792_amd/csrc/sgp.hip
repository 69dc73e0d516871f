// SGP update for n simulated nodes resident in one MI355X's HBM: host-side peer scheduler, HIP
// kernels for gfx950 and the C ABI declared in include/sgp.h.
//
// Kernel design.  The PushSum mix couples nodes but never coordinates (x <- P x acts on the
// n-vector of one coordinate), so a work-item owns a 128-bit group of four coordinates for ALL
// n nodes.  It reads x, u, g of every node once, writes u, x, z once, and the "messages" of
// Alg. 1's send/receive step never leave registers (or LDS): 24 bytes of HBM traffic per node-parameter, the
// algorithmic minimum, and the in-place update is race-free because no other work-item touches
// those coordinates.  Everything is a stream (about 0.4 flop per byte), so there is no MFMA
// here; what matters is 128-bit coalesced accesses and enough loads in flight per CU.
//
// All floating-point code here is compiled without multiply-add contraction, so each operation
// rounds separately, in the order written.
//
// Layout of the sources.  Several translation units, so that the kernel families compile side by side;
// each includes internal.h and then the .inc files it needs inside an anonymous namespace:
//   sgp.hip                       handle, host peer scheduler, C ABI, and the kernels of
//     schedule.inc                  host peer scheduler of the directed exponential graph
//     device_common.inc             128-bit access helpers, push-sum weight update inside the step
//                                   kernels, local optimiser step (included by every unit)
//     stats_tail.inc                end of every step kernel with fused statistics (every unit with one)
//     step_one_peer.inc             one out-peer: walk over the cycles of the shift
//     step_complete.inc             complete graph
//     debias_copy.inc               stand-alone de-bias, reference copy
//     stats.inc                     stand-alone consensus statistics and the final reductions
//   sgp_walk_stats.hip            the one-peer walk with the consensus statistics taken from registers
//                                 (step_walk_stats.inc); compiled once per variant of the kernel
//   sgp_gather.hip                several out-peers / caller-supplied rows: private LDS columns (step_gather.inc);
//                                 compiled twice, without and with the statistics
//   sgp_overlap.hip               tau-overlap SGP: own share now, messages of the previous round (step_overlap.inc)
//   internal.h                    constants, kernel argument structures, launchers across the units
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "sgp.h"
#include "internal.h"

#pragma clang fp contract(off)

using namespace sgp_detail;

namespace {

#include "schedule.inc"
#include "device_common.inc"
#include "stats_tail.inc"
#include "step_one_peer.inc"
#include "step_complete.inc"
#include "debias_copy.inc"
#include "stats.inc"

}  // namespace

// ------------------------------------------------------------------------------------------
// Handle
// ------------------------------------------------------------------------------------------
namespace {
constexpr int kStatsGridMax = 2048;
constexpr int kResultSlots = 3;   // statistics results: one synchronous, two in flight
constexpr size_t kCachedStateBytes = (size_t)160 << 20;   // x, u, g, z together: below this, cached accesses
constexpr int kStepCounters = (1 + kCountLines) * kCountStride;   // the step kernels' counters of finished blocks
}  // namespace

struct sgp_handle {
    int n;
    int64_t d, ld;
    int topology, peers, delay;
    int L;          // length of the peer list
    int distinct;   // distinct out-peers per iteration (the same for every k)
    int S;          // sources per receiver = distinct + 1

    bool dev_ready;
    bool biased;        // z = x instead of x / w (ablation without the push-sum weight)
    int *d_tab;         // [max(L,1)][n][S] sorted source lists, one table per k mod L
    int cS;             // caller-supplied mixing rows (SGP_TOPO_CUSTOM): entries per row, 0 = not set
    int *d_cidx;        // [n][cS] senders, -1 = padding
    float *d_cw;        // [n][cS] weights
    unsigned *d_done;   // counters of finished blocks: the step kernels' (kStepCounters), then one per result slot
    float wd;           // weight decay coefficient, 0 = off
    bool wd_on_x;       // decay acts on the numerator instead of the de-biased parameters
    float *d_partial;   // [(n+1)][G] partial sums of the stand-alone statistics
    int G;
    double *d_sums;     // [n+1] per-node sums of squares (+ the average's) of the stand-alone statistics
    // the fused step+statistics kernel, per result slot: its partial table [33][Gf], the block sums
    // of the reduction [kSlotSumBlocks][33] and a copy of the weights the step produced
    float *d_partial_f[kResultSlots];
    double *d_sums_f[kResultSlots];
    float *d_w_snap[kResultSlots];
    bool fused_ready;
    hipStream_t side;       // the reduction of the fused statistics runs here, beside the next step
    hipEvent_t ev_step[kResultSlots];   // step kernel of the slot finished (recorded on the caller's stream)
    double *h_result;   // [kResultSlots][8 + n], pinned host memory that the last statistics kernel writes
                        // directly (no copy behind it): slot 0 for the synchronous calls, 1.. for begin/end
    double *h_result_dev;   // the same memory as the device addresses it
    hipEvent_t ev_res[kResultSlots];    // result of the slot copied to the host
    bool ev_made;
    int pend_head, pend_count;   // ring of outstanding begin/end results (slots 1 + index)
    float *d_msg[2];    // overlap mode: pre-weighted messages p*xh_j, [n][ld] each
    bool msg_external;  // d_msg points into caller-owned memory
    float *d_msgw[2];   // overlap mode: pre-weighted weights p*w_j, [n] each
    int cur;            // buffer that the NEXT step writes
    bool have_msgs;
    int64_t last_k;
    int last_hip;
    const char *last_kernel;              // name of the step kernel of the latest successful step

    bool timing;                          // bracket the step kernel with events
    hipEvent_t ev[SGP_TIMING_RING][2];
    bool ev_timing_made;
    int64_t ev_head;                      // timed steps recorded so far
    int64_t ev_read;                      // timed steps already reported
};

namespace {

// Device allocation of the library.  Tests can make the next allocations fail (sgp_debug_fail_alloc)
// to exercise the out-of-memory paths without exhausting the device.
std::atomic<int> g_allocs_until_failure{-1};   // -1: off; k >= 0: k more allocations succeed, then one fails

template <typename T>
hipError_t dev_malloc(T **out, size_t bytes)
{
    int left = g_allocs_until_failure.load();
    while (left >= 0) {
        if (g_allocs_until_failure.compare_exchange_weak(left, left - 1)) {
            if (left == 0) {
                *out = nullptr;
                return hipErrorOutOfMemory;
            }
            break;
        }
    }
    return hipMalloc(reinterpret_cast<void **>(out), bytes);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

int hip_fail(sgp_handle *h, hipError_t e)
{
    if (h) h->last_hip = (int)e;
    return e == hipErrorOutOfMemory ? SGP_ERR_NOMEM : SGP_ERR_HIP;
}

#define SGP_HIP_TRY(h, expr)                           \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return hip_fail((h), e_); \
    } while (0)

// Sorted source lists of every receiver for each of the L distinct schedules.
void build_tables(const sgp_handle *h, int *tab)
{
    const int n = h->n, S = h->S, tables = h->L > 0 ? h->L : 1;
    for (int t = 0; t < tables; ++t) {
        Schedule s = make_schedule(n, h->peers, t);
        for (int i = 0; i < n; ++i) {
            int *row = tab + ((size_t)t * n + i) * S;
            int cnt = 0;
            row[cnt++] = i;
            for (int q = 0; q < s.distinct; ++q) row[cnt++] = (i - s.uniq[q] % n + n) % n;
            for (int a = 1; a < cnt; ++a) {          // insertion sort, ascending
                int v = row[a], b = a - 1;
                while (b >= 0 && row[b] > v) { row[b + 1] = row[b]; --b; }
                row[b + 1] = v;
            }
        }
    }
}

// (Re)builds the source tables of the directed exponential graph for the handle's current peers.
// The new table is complete before the old one is released, so a failure leaves the handle as it was.
int upload_tables(sgp_handle *h)
{
    const int n = h->n, S = h->S, tables = h->L > 0 ? h->L : 1;
    size_t tab_elems = (size_t)tables * n * S;
    int *host_tab = static_cast<int *>(std::malloc(tab_elems * sizeof(int)));
    if (!host_tab) return SGP_ERR_NOMEM;
    build_tables(h, host_tab);
    int *fresh = nullptr;
    hipError_t e = dev_malloc(&fresh, tab_elems * sizeof(int));
    if (e == hipSuccess) e = hipMemcpy(fresh, host_tab, tab_elems * sizeof(int), hipMemcpyHostToDevice);
    std::free(host_tab);
    if (e != hipSuccess) {
        if (fresh) (void)hipFree(fresh);
        return hip_fail(h, e);
    }
    if (h->d_tab) (void)hipFree(h->d_tab);   // waits for the kernels that still read it
    h->d_tab = fresh;
    return SGP_OK;
}

// Device resources every launching call needs.  Each pointer is allocated once: a call that failed
// half way is picked up where it stopped.
int ensure_device(sgp_handle *h)
{
    if (h->dev_ready) return SGP_OK;
    const int n = h->n;
    if (!h->d_tab) {
        int rc = upload_tables(h);
        if (rc != SGP_OK) return rc;
    }
    h->G = kStatsGridMax;
    const size_t res_bytes = (size_t)kResultSlots * (8 + n) * sizeof(double);
    if (!h->d_done) {
        SGP_HIP_TRY(h, dev_malloc(&h->d_done, (kStepCounters + kResultSlots) * sizeof(unsigned)));
        SGP_HIP_TRY(h, hipMemset(h->d_done, 0, (kStepCounters + kResultSlots) * sizeof(unsigned)));
    }
    if (!h->d_partial) SGP_HIP_TRY(h, dev_malloc(&h->d_partial, (size_t)(n + 1) * h->G * sizeof(float)));
    if (!h->d_sums) SGP_HIP_TRY(h, dev_malloc(&h->d_sums, (size_t)(n + 1) * sizeof(double)));
    if (!h->h_result) {
        SGP_HIP_TRY(h, hipHostMalloc(reinterpret_cast<void **>(&h->h_result), res_bytes, hipHostMallocMapped));
        SGP_HIP_TRY(h, hipHostGetDevicePointer(reinterpret_cast<void **>(&h->h_result_dev), h->h_result, 0));
    }
    if (h->delay) {
        size_t bytes = (size_t)n * (size_t)h->ld * sizeof(float);
        for (int b = 0; b < 2; ++b) {
            if (!h->msg_external && !h->d_msg[b]) SGP_HIP_TRY(h, dev_malloc(&h->d_msg[b], bytes));
            if (!h->d_msgw[b]) SGP_HIP_TRY(h, dev_malloc(&h->d_msgw[b], (size_t)n * sizeof(float)));
        }
    }
    h->dev_ready = true;
    return SGP_OK;
}

// Whether a step with statistics can take them inside the step kernel (conditions common to every
// kernel family; overlap mode additionally needs exactly two messages per receiver).
bool fused_stats_applies(const sgp_handle *h, bool adam, bool vec, long tail)
{
    return !adam && h->n <= kStatsCache && vec && tail == 0;
}

// Resources of the fused step+statistics path: a stream of its own for the reduction, events, and
// per result slot the partial table, the block sums and the weight copy.  Allocated once, before
// anything of the step that needs them is launched.
int ensure_fused(sgp_handle *h)
{
    if (h->fused_ready) return SGP_OK;
    const unsigned Gf = grid_for((long)(h->d / 4), kStatsStepBlock);
    if (!h->side) SGP_HIP_TRY(h, hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking));
    for (int s = 0; s < kResultSlots; ++s) {
        if (!h->d_partial_f[s])
            SGP_HIP_TRY(h, dev_malloc(&h->d_partial_f[s], (size_t)(kStatsCache + 1) * Gf * sizeof(float)));
        if (!h->d_sums_f[s])
            SGP_HIP_TRY(h, dev_malloc(&h->d_sums_f[s], (size_t)kSlotSumBlocks * (kStatsCache + 1) * sizeof(double)));
        if (!h->d_w_snap[s]) SGP_HIP_TRY(h, dev_malloc(&h->d_w_snap[s], (size_t)h->n * sizeof(float)));
    }
    h->fused_ready = true;
    return SGP_OK;
}

int ensure_result_events(sgp_handle *h)
{
    if (h->ev_made) return SGP_OK;
    for (int s = 0; s < kResultSlots; ++s) {
        if (!h->ev_step[s]) SGP_HIP_TRY(h, hipEventCreate(&h->ev_step[s]));
        if (!h->ev_res[s]) SGP_HIP_TRY(h, hipEventCreateWithFlags(&h->ev_res[s], hipEventDisableTiming));
    }
    h->ev_made = true;
    return SGP_OK;
}

void release_device(sgp_handle *h)
{
    if (h->ev_timing_made)
        for (int i = 0; i < SGP_TIMING_RING; ++i) {
            if (h->ev[i][0]) (void)hipEventDestroy(h->ev[i][0]);
            if (h->ev[i][1]) (void)hipEventDestroy(h->ev[i][1]);
        }
    for (int s = 0; s < kResultSlots; ++s) {
        if (h->ev_step[s]) (void)hipEventDestroy(h->ev_step[s]);
        if (h->ev_res[s]) (void)hipEventDestroy(h->ev_res[s]);
        if (h->d_partial_f[s]) (void)hipFree(h->d_partial_f[s]);
        if (h->d_sums_f[s]) (void)hipFree(h->d_sums_f[s]);
        if (h->d_w_snap[s]) (void)hipFree(h->d_w_snap[s]);
    }
    if (h->side) (void)hipStreamDestroy(h->side);
    if (h->d_tab) (void)hipFree(h->d_tab);
    if (h->d_cidx) (void)hipFree(h->d_cidx);
    if (h->d_cw) (void)hipFree(h->d_cw);
    if (h->d_done) (void)hipFree(h->d_done);
    if (h->d_partial) (void)hipFree(h->d_partial);
    if (h->d_sums) (void)hipFree(h->d_sums);
    if (h->h_result) (void)hipHostFree(h->h_result);
    for (int b = 0; b < 2; ++b) {
        if (h->d_msg[b] && !h->msg_external) (void)hipFree(h->d_msg[b]);
        if (h->d_msgw[b]) (void)hipFree(h->d_msgw[b]);
    }
}

template <int V, int OPT, bool ZOUT>
void launch_one_peer(const StepArgs &a, size_t col0, long ncols, int h, int len)
{
    if (a.cached)
        hipLaunchKernelGGL((k_step_one_peer<V, OPT, ZOUT, true>), dim3(grid_for(ncols, kOpBlock * kOpCols)),
                           dim3(kOpBlock), weight_lds_bytes(a.n), a.stream, a.x, a.u, a.g, a.z, a.wop, a.n, a.ld,
                           col0, ncols, h, len, a.p, a.hp);
    else
        hipLaunchKernelGGL((k_step_one_peer<V, OPT, ZOUT, false>), dim3(grid_for(ncols, kOpBlock * kOpCols)),
                           dim3(kOpBlock), weight_lds_bytes(a.n), a.stream, a.x, a.u, a.g, a.z, a.wop, a.n, a.ld,
                           col0, ncols, h, len, a.p, a.hp);
    *a.name = "k_step_one_peer";
}

template <int V, int OPT, bool ZOUT, bool STATS = false>
void launch_complete(const StepArgs &a, size_t col0, long ncols, float *partial = nullptr, hipEvent_t fin = nullptr)
{
    launch_step(k_step_complete<V, OPT, ZOUT, STATS>, dim3(grid_for(ncols, kOpBlock)), dim3(kOpBlock),
                weight_lds_bytes(a.n), a.stream, fin, a.x, a.u, a.g, a.z, a.wop, a.n, a.ld, col0, ncols, a.p, a.hp,
                partial);
    *a.name = STATS ? "k_step_complete_stats" : "k_step_complete";
}

// The unrolled walk with the statistics taken from registers: one out-peer (or none) without delay
// (msgs = 0), or one iteration of delay with msgs = 1 or 2 messages per receiver.
void launch_walk_stats(const StepArgs &a, int opt, long cols4, int h, int len, float *partial, hipEvent_t fin,
                       int msgs = 0, const float *msg_prev = nullptr, float *msg_cur = nullptr, int ha = 0, int hb = 0)
{
    const bool nest = opt == kOptNesterov;
    auto go = [&]<bool CACHED, int MSG>() {
        if (nest) launch_walk_stats_variant<true, CACHED, MSG>(a, cols4, h, len, partial, fin, msg_prev, msg_cur, ha, hb);
        else launch_walk_stats_variant<false, CACHED, MSG>(a, cols4, h, len, partial, fin, msg_prev, msg_cur, ha, hb);
    };
    if (msgs == 2) {
        go.template operator()<false, 2>();
        *a.name = "k_step_delay2_stats";
    } else if (msgs == 1) {
        go.template operator()<false, 1>();
        *a.name = "k_step_delay1_stats";
    } else {
        if (a.cached) go.template operator()<true, 0>();
        else go.template operator()<false, 0>();
        *a.name = "k_step_one_peer_stats";
    }
}

// Calls f.template operator()<OPT, ZOUT>() for the run-time optimiser and z flag.
template <typename F>
void dispatch_flags(int opt, bool zout, F &&f)
{
    if (opt == kOptAdam) {
        if (zout) f.template operator()<kOptAdam, true>();
        else f.template operator()<kOptAdam, false>();
    } else if (opt == kOptNesterov) {
        if (zout) f.template operator()<kOptNesterov, true>();
        else f.template operator()<kOptNesterov, false>();
    } else {
        if (zout) f.template operator()<kOptSgd, true>();
        else f.template operator()<kOptSgd, false>();
    }
}

}  // namespace

// ------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------
extern "C" {

const char *sgp_status_string(int status)
{
    switch (status) {
        case SGP_OK: return "SGP_OK";
        case SGP_ERR_INVALID_ARG: return "SGP_ERR_INVALID_ARG";
        case SGP_ERR_UNSUPPORTED: return "SGP_ERR_UNSUPPORTED";
        case SGP_ERR_ALIGNMENT: return "SGP_ERR_ALIGNMENT";
        case SGP_ERR_SEQUENCE: return "SGP_ERR_SEQUENCE";
        case SGP_ERR_HIP: return "SGP_ERR_HIP";
        case SGP_ERR_NOMEM: return "SGP_ERR_NOMEM";
        default: return "SGP_ERR_UNKNOWN";
    }
}

int sgp_create(sgp_handle **out, int32_t n, int64_t d, int64_t ld, int32_t topology, int32_t peers,
               int32_t delay)
{
    if (!out) return SGP_ERR_INVALID_ARG;
    *out = nullptr;
    if (n < 1 || n > SGP_MAX_NODES || d < 1 || ld < d || peers < 1 || peers > SGP_MAX_PEERS ||
        delay < 0 || delay > SGP_MAX_DELAY)
        return SGP_ERR_INVALID_ARG;
    if (topology != SGP_TOPO_DIRECTED_EXP && topology != SGP_TOPO_COMPLETE && topology != SGP_TOPO_CUSTOM)
        return SGP_ERR_UNSUPPORTED;
    if (topology != SGP_TOPO_DIRECTED_EXP && delay != 0) return SGP_ERR_UNSUPPORTED;
    sgp_handle *h = new (std::nothrow) sgp_handle();
    if (!h) return SGP_ERR_NOMEM;
    std::memset(h, 0, sizeof(*h));
    h->n = n;
    h->d = d;
    h->ld = ld;
    h->topology = topology;
    h->peers = peers;
    h->delay = delay;
    Schedule s = make_schedule(n, peers, 0);
    h->L = s.L;
    h->distinct = s.distinct;
    h->S = s.distinct + 1;
    h->last_k = -1;
    h->last_kernel = "";
    *out = h;
    return SGP_OK;
}

int sgp_destroy(sgp_handle *h)
{
    if (!h) return SGP_OK;
    int rc = SGP_OK;
    // also after a set-up that failed half way, or mixing rows set on a handle that never stepped:
    // every pointer is checked on its own
    if (h->dev_ready || h->side || h->d_tab || h->d_cidx) {
        hipError_t e = hipDeviceSynchronize();
        if (e != hipSuccess) rc = SGP_ERR_HIP;
    }
    release_device(h);
    delete h;
    return rc;
}

int sgp_reset(sgp_handle *h)
{
    if (!h) return SGP_ERR_INVALID_ARG;
    h->have_msgs = false;
    h->last_k = -1;
    return SGP_OK;
}

int sgp_set_topology(sgp_handle *h, int32_t topology, int32_t peers)
{
    if (!h || peers < 1 || peers > SGP_MAX_PEERS) return SGP_ERR_INVALID_ARG;
    if (topology != SGP_TOPO_DIRECTED_EXP && topology != SGP_TOPO_COMPLETE && topology != SGP_TOPO_CUSTOM)
        return SGP_ERR_UNSUPPORTED;
    if (h->delay != 0) return SGP_ERR_UNSUPPORTED;
    const int old_topology = h->topology, old_peers = h->peers;
    h->topology = topology;
    h->peers = peers;
    Schedule s = make_schedule(h->n, peers, 0);
    h->L = s.L;
    h->distinct = s.distinct;
    h->S = s.distinct + 1;
    if (h->d_tab && peers != old_peers) {   // tables exist: rebuild them now, not inside a step
        int rc = upload_tables(h);
        if (rc != SGP_OK) {                 // the old tables are still in place: keep the old setting
            h->topology = old_topology;
            h->peers = old_peers;
            s = make_schedule(h->n, old_peers, 0);
            h->L = s.L;
            h->distinct = s.distinct;
            h->S = s.distinct + 1;
            return rc;
        }
    }
    return SGP_OK;
}

int sgp_set_mixing(sgp_handle *h, const int32_t *in_idx, const float *in_weight, int32_t entries)
{
    if (!h || !in_idx || !in_weight || entries < 1 || entries > h->n) return SGP_ERR_INVALID_ARG;
    const size_t cnt = (size_t)h->n * entries;
    for (size_t q = 0; q < cnt; ++q)
        if (in_idx[q] < -1 || in_idx[q] >= h->n) return SGP_ERR_INVALID_ARG;
    // the new rows are complete before the old ones are released
    int *idx = nullptr;
    float *wts = nullptr;
    hipError_t e = dev_malloc(&idx, cnt * sizeof(int));
    if (e == hipSuccess) e = dev_malloc(&wts, cnt * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(idx, in_idx, cnt * sizeof(int), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(wts, in_weight, cnt * sizeof(float), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (idx) (void)hipFree(idx);
        if (wts) (void)hipFree(wts);
        return hip_fail(h, e);
    }
    if (h->d_cidx) (void)hipFree(h->d_cidx);   // hipFree waits for the kernels that still read the old rows
    if (h->d_cw) (void)hipFree(h->d_cw);
    h->d_cidx = idx;
    h->d_cw = wts;
    h->cS = entries;
    return SGP_OK;
}

int sgp_set_weight_decay(sgp_handle *h, float weight_decay, int on_numerator)
{
    if (!h || !(weight_decay >= 0.0f)) return SGP_ERR_INVALID_ARG;
    h->wd = weight_decay;
    h->wd_on_x = on_numerator != 0;
    return SGP_OK;
}

int sgp_set_biased(sgp_handle *h, int biased)
{
    if (!h) return SGP_ERR_INVALID_ARG;
    h->biased = biased != 0;
    return SGP_OK;
}

int sgp_set_message_buffers(sgp_handle *h, float *buf0, float *buf1)
{
    if (!h || !buf0 || !buf1 || buf0 == buf1 || !h->delay || !aligned16(buf0) || !aligned16(buf1))
        return SGP_ERR_INVALID_ARG;
    if (h->dev_ready || (h->d_msg[0] && !h->msg_external)) return SGP_ERR_SEQUENCE;
    h->d_msg[0] = buf0;
    h->d_msg[1] = buf1;
    h->msg_external = true;
    h->have_msgs = false;
    h->last_k = -1;
    return SGP_OK;
}

int sgp_last_hip_error(const sgp_handle *h) { return h ? h->last_hip : 0; }

int sgp_debug_fail_alloc(int32_t succeed_first)
{
    g_allocs_until_failure.store(succeed_first < 0 ? -1 : succeed_first);
    return SGP_OK;
}

const char *sgp_last_step_kernel(const sgp_handle *h) { return h ? h->last_kernel : ""; }

int sgp_schedule(int32_t n, int32_t peers, int64_t k, int32_t *out_peers, int32_t *in_peers,
                 float *weight)
{
    if (n < 1 || n > SGP_MAX_NODES || peers < 1 || peers > SGP_MAX_PEERS || k < 0)
        return SGP_ERR_INVALID_ARG;
    Schedule s = make_schedule(n, peers, k);
    for (int i = 0; i < n; ++i)
        for (int r = 0; r < peers; ++r) {
            int hop = s.hop[r];
            if (out_peers) out_peers[(size_t)i * peers + r] = hop < 0 ? -1 : (i + hop) % n;
            if (in_peers) in_peers[(size_t)i * peers + r] = hop < 0 ? -1 : ((i - hop) % n + n) % n;
        }
    if (weight) *weight = s.p;
    return SGP_OK;
}

int sgp_peer_schedule(const sgp_handle *h, int64_t k, int32_t *out_peers, int32_t *in_peers,
                      float *weight)
{
    if (!h || k < 0) return SGP_ERR_INVALID_ARG;
    if (h->topology != SGP_TOPO_DIRECTED_EXP) return SGP_ERR_UNSUPPORTED;
    if (h->delay > 1) {
        if (k % h->delay != 0) {   // no communication at this iteration: every node keeps everything
            const size_t cnt = (size_t)h->n * h->peers;
            for (size_t q = 0; q < cnt; ++q) {
                if (out_peers) out_peers[q] = -1;
                if (in_peers) in_peers[q] = -1;
            }
            if (weight) *weight = 1.0f;
            return SGP_OK;
        }
        k /= h->delay;
    }
    return sgp_schedule(h->n, h->peers, k, out_peers, in_peers, weight);
}

// What step_impl did about the statistics: G > 0 means the fused kernel ran and left its partial
// table (G blocks) in the slot's table for a walk with this hop and cycle length.
struct FusedStats {
    int slot = 0;   // in: result slot whose table and weight copy the fused kernel may use
    bool in_order = false;   // in: the caller waits for the result right away: the reduction goes onto the
                             // caller's stream behind the step kernel, no event and no second stream between
    int G = 0, hop = 0, len = 1;
};

// Adam's scalars as sgp_step_adam hands them over (NULL: SGD / Nesterov).
struct AdamArgs {
    float *v2;
    float beta1, beta2, eps;
    int64_t t;
};

// One iteration; with fused != NULL the caller wants the statistics of z^(k+1) as well: when the
// fused kernel applies, it is used and *fused describes the partial table it left, otherwise
// fused->G stays 0 and the caller runs the stand-alone statistics pass.
// Order: every check, then every allocation, then the launches, then (only when the launches were
// accepted) the bookkeeping of overlap mode: a call that fails has not touched x, u, w, z.
static int step_impl(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out,
                     float gamma, float momentum, int64_t k, void *stream, FusedStats *fused,
                     const AdamArgs *adam = nullptr)
{
    if (!h || !x || !w || !g || k < 0) return SGP_ERR_INVALID_ARG;
    const int opt = adam ? kOptAdam : momentum != 0.0f ? kOptNesterov : kOptSgd;
    const bool nest = opt != kOptSgd;          // the momentum / first-moment array is in use
    if (nest && !m) return SGP_ERR_INVALID_ARG;
    if (adam && (!adam->v2 || adam->t < 1 || !(adam->beta1 >= 0.0f && adam->beta1 < 1.0f) ||
                 !(adam->beta2 >= 0.0f && adam->beta2 < 1.0f) || !(adam->eps >= 0.0f)))
        return SGP_ERR_INVALID_ARG;
    if (!aligned4(x) || !aligned4(w) || !aligned4(g) || (nest && !aligned4(m)) ||
        (adam && !aligned4(adam->v2)) || (z_out && !aligned4(z_out)))
        return SGP_ERR_ALIGNMENT;
    if (z_out && (z_out == x || z_out == g || (nest && z_out == m) || (adam && z_out == adam->v2)))
        return SGP_ERR_INVALID_ARG;
    if (adam && (adam->v2 == x || adam->v2 == m || adam->v2 == g)) return SGP_ERR_INVALID_ARG;
    if (h->delay && h->last_k >= 0 && k != h->last_k + 1) return SGP_ERR_SEQUENCE;

    // tau >= 2: nodes communicate at the iterations with k mod tau == 0 only, and the schedule
    // advances once per communication round
    const int tau = h->delay;
    const bool sending = tau <= 1 || (k % tau) == 0;
    const int64_t round = tau > 1 ? k / tau : k;
    const int n = h->n, S = h->S;
    const Schedule s = make_schedule(n, h->peers, round);
    const int kmod = h->L > 0 ? (int)(round % h->L) : 0;
    const bool complete = h->topology == SGP_TOPO_COMPLETE;
    const bool custom = h->topology == SGP_TOPO_CUSTOM;
    if (custom && h->cS == 0) return SGP_ERR_SEQUENCE;         // sgp_set_mixing has not been called
    const bool gather = sending && (custom || (h->delay == 0 && !complete && s.distinct > 1));

    bool vec = (h->ld % 4 == 0) && aligned16(x) && aligned16(g) && (!nest || aligned16(m)) &&
               (!adam || aligned16(adam->v2)) && (!z_out || aligned16(z_out));
    if (gather && n > kGatherVecMaxNodes) vec = false;   // the private columns must fit the LDS
    if (gather && n > SGP_MAX_NODES_GATHER) return SGP_ERR_UNSUPPORTED;
    const long cols4 = vec ? (long)(h->d / 4) : 0;             // full 128-bit groups
    const size_t tail0 = (size_t)cols4 * 4;
    const long tail = (long)(h->d - (int64_t)tail0);           // scalar columns after them
    // overlap mode: the fused walk exists for one and for two messages per receiver (one or two
    // distinct out-peers, and something has been sent already)
    const bool two_msgs = h->delay != 0 && sending && h->have_msgs && h->L > 0 && S == 3;
    const bool one_msg = h->delay != 0 && sending && h->have_msgs && h->L > 0 && S == 2;
    // a problem whose arrays (x, u, g, z) all stay in the 256 MB last-level cache from one iteration to
    // the next is better served by ordinary loads and stores than by streaming ones
    const bool cached = (size_t)n * (size_t)h->ld * sizeof(float) * 4 <= kCachedStateBytes;
    const bool use_fused = fused && z_out && fused_stats_applies(h, adam != nullptr, cols4 > 0, tail) &&
                           (h->delay == 0 || !sending || two_msgs || one_msg);

    int rc = ensure_device(h);
    if (rc != SGP_OK) return rc;
    if (use_fused && ((rc = ensure_fused(h)) != SGP_OK || (rc = ensure_result_events(h)) != SGP_OK)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);

    const bool decay = h->wd != 0.0f;
    Hyper hp{};
    hp.gamma = gamma;
    hp.mom = momentum;
    hp.wd = h->wd;
    hp.wd_mode = !decay ? 0 : (h->wd_on_x || h->biased) ? 1 : 2;
    if (adam) {   // bias corrections in double, rounded once
        hp.v2 = adam->v2;
        hp.beta1 = adam->beta1;
        hp.c1 = 1.0f - adam->beta1;
        hp.beta2 = adam->beta2;
        hp.c2 = 1.0f - adam->beta2;
        hp.bc1 = (float)(1.0 - std::pow((double)adam->beta1, (double)adam->t));
        hp.bc2 = (float)(1.0 - std::pow((double)adam->beta2, (double)adam->t));
        hp.eps = adam->eps;
    }
    // the push-sum weight update, carried out by the step kernel itself
    WeightOp wop{};
    wop.w = w;
    wop.p = s.p;
    wop.biased = (int)h->biased;
    wop.done = h->d_done;
    wop.hop = -1;
    const char *kname = "";
    StepArgs a{x, m, z_out, g, wop, n, (size_t)h->ld, s.p, hp, st, &kname, cached};
    const int *tab_k = h->d_tab + (size_t)kmod * n * S;
    // a step is one launch over the 128-bit groups plus, for d % 4 != 0 or unaligned arrays, one over
    // the remaining scalar columns; the last of them writes the new weights back
    auto two_launches = [&](auto &&launch4, auto &&launch1) {
        if (cols4 > 0) {
            a.wop.publish = tail > 0 ? 0 : 1;
            launch4();
        }
        if (tail > 0) {
            a.wop.publish = 1;
            launch1();
        }
    };

    hipEvent_t *tev = nullptr;
    if (h->timing) {
        tev = h->ev[h->ev_head % SGP_TIMING_RING];
        SGP_HIP_TRY(h, hipEventRecord(tev[0], st));
    }

    // with fused statistics: the slot's table and weight copy, and the slot's event attached to the
    // kernel itself as its completion event (no marker of its own on the caller's stream); the
    // reduction on the library's stream waits for it
    float *partial = nullptr;
    hipEvent_t fin = nullptr;
    if (use_fused) {
        partial = h->d_partial_f[fused->slot];
        fin = fused->in_order ? nullptr : h->ev_step[fused->slot];
        a.wop.publish = 1;
        a.wop.w_snap = h->d_w_snap[fused->slot];
        fused->G = (int)grid_for(cols4, kStatsStepBlock);
        fused->hop = 0;                  // slot s holds node s unless a walk says otherwise
        fused->len = 1;
    }

    if (!sending) {
        // between two communication rounds: a local step, x <- xh, w unchanged (Alg. 2, else branch
        // of the send test), which is the one-peer walk with n cycles of length 1 and weight 1
        a.wop.kind = kWKeep;
        a.p = 1.0f;
        if (use_fused) launch_walk_stats(a, opt, cols4, 0, 1, partial, fin);
        else
        dispatch_flags(opt, z_out != nullptr, [&]<int OPT, bool ZOUT>() {
            two_launches([&] { launch_one_peer<4, OPT, ZOUT>(a, 0, cols4, 0, 1); },
                         [&] { launch_one_peer<1, OPT, ZOUT>(a, tail0, tail, 0, 1); });
        });
    } else if (complete) {
        a.p = 1.0f / (float)n;
        a.wop.kind = kWComplete;
        a.wop.p = a.p;
        if (use_fused) {
            if (opt == kOptNesterov) launch_complete<4, kOptNesterov, true, true>(a, 0, cols4, partial, fin);
            else launch_complete<4, kOptSgd, true, true>(a, 0, cols4, partial, fin);
        } else
        dispatch_flags(opt, z_out != nullptr, [&]<int OPT, bool ZOUT>() {
            two_launches([&] { launch_complete<4, OPT, ZOUT>(a, 0, cols4); },
                         [&] { launch_complete<1, OPT, ZOUT>(a, tail0, tail); });
        });
    } else if (custom || gather) {
        const int *tab = custom ? h->d_cidx : tab_k;
        const float *tabw = custom ? h->d_cw : nullptr;
        const int entries = custom ? h->cS : S;
        a.wop.kind = custom ? kWCustom : kWTable;
        a.wop.tab = tab;
        a.wop.tabw = tabw;
        a.wop.S = entries;
        const bool zo = z_out != nullptr;
        if (use_fused) launch_gather_stats(a, opt, cols4, tab, tabw, entries, partial, fin);
        else
            two_launches([&] { launch_gather(a, 4, opt, zo, 0, cols4, tab, tabw, entries); },
                         [&] { launch_gather(a, 1, opt, zo, tail0, tail, tab, tabw, entries); });
    } else if (h->delay == 0) {
        const int hop = s.distinct ? s.uniq[0] % n : 0;
        const int ncyc = s.distinct ? gcd_int(n, hop) : n;   // no peer: n cycles of length 1
        const int len = n / ncyc;
        a.wop.kind = kWOnePeer;
        a.wop.hop = s.distinct ? hop : -1;
        if (use_fused) {
            launch_walk_stats(a, opt, cols4, hop, len, partial, fin);
            fused->hop = hop;
            fused->len = len;
        } else
        dispatch_flags(opt, z_out != nullptr, [&]<int OPT, bool ZOUT>() {
            two_launches([&] { launch_one_peer<4, OPT, ZOUT>(a, 0, cols4, hop, len); },
                         [&] { launch_one_peer<1, OPT, ZOUT>(a, tail0, tail, hop, len); });
        });
    } else {
        const int *tab_prev = nullptr;
        int ha = 0, hb = 0;          // the previous round's hops, when there are exactly two
        if (h->have_msgs && h->L > 0 && (S == 3 || S == 2)) {
            const Schedule sp = make_schedule(n, h->peers, round - 1);
            ha = sp.uniq[0] % n;
            if (S == 3) hb = sp.uniq[1] % n;
        }
        if (h->have_msgs && h->L > 0) {
            const int kprev = (int)((round - 1) % h->L);
            tab_prev = h->d_tab + (size_t)kprev * n * S;
        }
        const int cur = h->cur, prv = cur ^ 1;
        a.wop.kind = kWDelay;
        a.wop.tab = tab_prev;
        a.wop.S = S;
        a.wop.msgw_prev = h->d_msgw[prv];
        a.wop.msgw_cur = h->d_msgw[cur];
        if (use_fused && one_msg) {  // one message per receiver: rows are independent, cycles of one node
            launch_walk_stats(a, opt, cols4, 0, 1, partial, fin, 1, h->d_msg[prv], h->d_msg[cur], ha, 0);
            fused->hop = 0;
            fused->len = 1;
        } else if (use_fused) {      // two messages per receiver: the stride walk of k_step_delay2
            const int stride = ((hb - ha) % n + n) % n;
            const int len = n / gcd_int(n, stride);
            launch_walk_stats(a, opt, cols4, stride, len, partial, fin, 2, h->d_msg[prv], h->d_msg[cur], ha, hb);
            fused->hop = stride;
            fused->len = len;
        } else {
            const bool zo = z_out != nullptr;
            two_launches(
                [&] { launch_delay(a, 4, opt, zo, 0, cols4, h->d_msg[prv], h->d_msg[cur], tab_prev, S, ha, hb); },
                [&] { launch_delay(a, 1, opt, zo, tail0, tail, h->d_msg[prv], h->d_msg[cur], tab_prev, S, ha, hb); });
        }
    }
    SGP_HIP_TRY(h, hipGetLastError());
    if (tev) {
        SGP_HIP_TRY(h, hipEventRecord(tev[1], st));
        ++h->ev_head;
    }
    // the launches were accepted: advance the overlap-mode sequence
    if (h->delay) {
        if (sending) {
            h->cur ^= 1;
            h->have_msgs = true;
        }
        h->last_k = k;
    }
    h->last_kernel = kname;
    return SGP_OK;
}

int sgp_step(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out, float gamma,
             float momentum, int64_t k, void *stream)
{
    return step_impl(h, x, w, m, g, z_out, gamma, momentum, k, stream, nullptr);
}

int sgp_step_adam(sgp_handle *h, float *x, float *w, float *m1, float *m2, const float *g, float *z_out,
                  float gamma, float beta1, float beta2, float eps, int64_t t, int64_t k, void *stream)
{
    const AdamArgs adam{m2, beta1, beta2, eps, t};
    return step_impl(h, x, w, m1, g, z_out, gamma, 0.0f, k, stream, nullptr, &adam);
}

int sgp_step_bf16(sgp_handle *h, float *x, float *w, void *m, const void *g16, void *z16, float gamma,
                  float momentum, int64_t k, int32_t storage, void *stream)
{
    if (!h || !x || !w || !m || !g16 || !z16 || k < 0) return SGP_ERR_INVALID_ARG;
    if (storage != SGP_STORE_BF16_GZ && storage != (SGP_STORE_BF16_GZ | SGP_STORE_BF16_U)) return SGP_ERR_INVALID_ARG;
    if (z16 == g16 || z16 == m || g16 == m || (void *)x == m) return SGP_ERR_INVALID_ARG;
    const bool u16 = (storage & SGP_STORE_BF16_U) != 0;
    auto aligned2 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 1u) == 0; };
    if (!aligned4(x) || !aligned4(w) || !aligned2(g16) || !aligned2(z16) || !(u16 ? aligned2(m) : aligned4(m)))
        return SGP_ERR_ALIGNMENT;
    const int n = h->n;
    const Schedule s = make_schedule(n, h->peers, k);
    // the experiment covers the blocking one-peer step with Nesterov momentum (Alg. 3)
    if (h->delay != 0 || h->topology != SGP_TOPO_DIRECTED_EXP || s.distinct > 1 || momentum == 0.0f)
        return SGP_ERR_UNSUPPORTED;
    int rc = ensure_device(h);
    if (rc != SGP_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);

    auto aligned8 = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 7u) == 0; };
    const bool vec = (h->ld % 4 == 0) && aligned16(x) && (u16 ? aligned8(m) : aligned16(m)) && aligned8(g16) &&
                     aligned8(z16);
    const long cols4 = vec ? (long)(h->d / 4) : 0;      // groups of four coordinates
    const size_t tail0 = (size_t)cols4 * 4;
    const long tail = (long)(h->d - (int64_t)tail0);    // scalar columns after them
    Hyper hp{};
    hp.gamma = gamma;
    hp.mom = momentum;
    hp.wd = h->wd;
    hp.wd_mode = h->wd == 0.0f ? 0 : (h->wd_on_x || h->biased) ? 1 : 2;
    const int hop = s.distinct ? s.uniq[0] % n : 0;
    const int len = s.distinct ? n / gcd_int(n, hop) : 1;
    WeightOp wop{};
    wop.w = w;
    wop.kind = kWOnePeer;
    wop.hop = s.distinct ? hop : -1;
    wop.p = s.p;
    wop.biased = (int)h->biased;
    wop.done = h->d_done;

    hipEvent_t *tev = nullptr;
    if (h->timing) {
        tev = h->ev[h->ev_head % SGP_TIMING_RING];
        SGP_HIP_TRY(h, hipEventRecord(tev[0], st));
    }
    auto launch = [&](auto kernel, int cols_per_item, size_t col0, long ncols, int publish) {
        wop.publish = publish;
        hipLaunchKernelGGL(kernel, dim3(grid_for(ncols, kOpBlock * cols_per_item)), dim3(kOpBlock),
                           weight_lds_bytes(n), st, x, m, g16, z16, wop, n, (size_t)h->ld, col0, ncols, hop, len,
                           s.p, hp);
    };
    if (cols4 > 0) {
        if (u16) launch(k_step_one_peer_h16<4, 3>, kH16Cols, 0, cols4, tail > 0 ? 0 : 1);
        else launch(k_step_one_peer_h16<4, 1>, kH16Cols, 0, cols4, tail > 0 ? 0 : 1);
    }
    if (tail > 0) {
        if (u16) launch(k_step_one_peer_h16<1, 3>, kH16Cols, tail0, tail, 1);
        else launch(k_step_one_peer_h16<1, 1>, kH16Cols, tail0, tail, 1);
    }
    SGP_HIP_TRY(h, hipGetLastError());
    if (tev) {
        SGP_HIP_TRY(h, hipEventRecord(tev[1], st));
        ++h->ev_head;
    }
    h->last_kernel = "k_step_one_peer_h16";
    return SGP_OK;
}

// Enqueues the reduction of a partial table to the statistics, which the last kernel writes straight
// into result slot `slot` of the pinned host buffer (8 + n doubles: no copy engine, no further
// call), and records ev_res[slot] behind it.
// fused == NULL: the stand-alone kernels' table [(n+1)][G], reduced on the caller's stream.
// Otherwise the fused step kernel's table of that slot, reduced on the library's own stream behind
// an event, so that the caller's stream is free for the next iteration at once; the weights are then
// taken from the copy the step kernel made (the caller's array may be overwritten by the next step
// before the reduction has read it).
static int enqueue_stats(sgp_handle *h, const FusedStats *fused, const float *w, int slot, hipStream_t st)
{
    const int n = h->n;
    int rc = ensure_result_events(h);
    if (rc != SGP_OK) return rc;
    double *d_res = h->h_result_dev + (size_t)slot * (8 + n);   // 8 + n doubles, written once, over the bus
    hipStream_t rs = st;
    if (fused) {
        if (!fused->in_order) {
            rs = h->side;
            SGP_HIP_TRY(h, hipStreamWaitEvent(rs, h->ev_step[slot], 0));   // recorded by the step kernel's launch
        }
        const int B = std::min(kSlotSumBlocks, fused->G);
        hipLaunchKernelGGL(k_stats_reduce_slots, dim3(B), dim3(kSlotSumBlock), 0, rs, h->d_partial_f[slot], fused->G,
                           h->d_sums_f[slot], h->d_done + kStepCounters + slot, n, fused->hop, fused->len, h->d_w_snap[slot],
                           d_res);
    } else {
        hipLaunchKernelGGL(k_stats_rowsum, dim3(n + 1), dim3(kRowSumBlock), 0, rs, h->d_partial, h->G, h->d_sums);
        hipLaunchKernelGGL(k_stats_final, dim3(1), dim3(64), 0, rs, h->d_sums, n, w, d_res);
    }
    SGP_HIP_TRY(h, hipGetLastError());
    SGP_HIP_TRY(h, hipEventRecord(h->ev_res[slot], rs));
    return SGP_OK;
}

static void read_stats(const sgp_handle *h, int slot, sgp_stats *host_out, double *per_node_dist_host)
{
    const int n = h->n;
    const double *r = h->h_result + (size_t)slot * (8 + n);
    host_out->dist_max = r[0];
    host_out->dist_mean = r[1];
    host_out->dist_min = r[2];
    host_out->w_sum = r[3];
    host_out->zbar_norm = r[4];
    host_out->argmax = (int32_t)r[5];
    host_out->argmin = (int32_t)r[6];
    if (per_node_dist_host)
        for (int i = 0; i < n; ++i) per_node_dist_host[i] = r[8 + i];
}

// Reduces a partial table to the statistics (slot 0, in host memory) and waits: for the result and
// for everything enqueued on the caller's stream before it.
static int finish_stats(sgp_handle *h, const FusedStats *fused, const float *w, sgp_stats *host_out,
                        double *per_node_dist_host, hipStream_t st)
{
    int rc = enqueue_stats(h, fused, w, 0, st);
    if (rc != SGP_OK) return rc;
    SGP_HIP_TRY(h, hipEventSynchronize(h->ev_res[0]));
    SGP_HIP_TRY(h, hipStreamSynchronize(st));
    read_stats(h, 0, host_out, per_node_dist_host);
    return SGP_OK;
}

static int run_stats(sgp_handle *h, const float *z, const StatSource &src, int mode, bool vec, const float *w,
                     sgp_stats *host_out, double *per_node_dist_host, hipStream_t st, int slot);

int sgp_step_stats(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out,
                   float gamma, float momentum, int64_t k, sgp_stats *host_out,
                   double *per_node_dist_host, void *stream)
{
    if (!z_out || !host_out) return SGP_ERR_INVALID_ARG;
    FusedStats fused;
    fused.in_order = true;
    int rc = step_impl(h, x, w, m, g, z_out, gamma, momentum, k, stream, &fused);
    if (rc != SGP_OK) return rc;
    if (fused.G > 0)
        return finish_stats(h, &fused, w, host_out, per_node_dist_host, static_cast<hipStream_t>(stream));
    return sgp_consensus_stats(h, z_out, w, host_out, per_node_dist_host, stream);
}

int sgp_step_stats_begin(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out,
                         float gamma, float momentum, int64_t k, void *stream)
{
    if (!h || !z_out) return SGP_ERR_INVALID_ARG;
    if (h->pend_count >= 2) return SGP_ERR_SEQUENCE;   // fetch a result with sgp_step_stats_end first
    int rc = ensure_result_events(h);                  // before anything is launched
    if (rc != SGP_OK) return rc;
    const int idx = (h->pend_head + h->pend_count) % 2;
    FusedStats fused;
    fused.slot = 1 + idx;
    rc = step_impl(h, x, w, m, g, z_out, gamma, momentum, k, stream, &fused);
    if (rc != SGP_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (fused.G > 0) {
        rc = enqueue_stats(h, &fused, w, 1 + idx, st);
    } else {
        const bool vec = (h->ld % 4 == 0) && aligned16(z_out);
        rc = run_stats(h, z_out, StatSource{}, 0, vec, w, nullptr, nullptr, st, 1 + idx);
    }
    if (rc != SGP_OK) return rc;
    ++h->pend_count;
    return SGP_OK;
}

int sgp_step_stats_end(sgp_handle *h, sgp_stats *host_out, double *per_node_dist_host)
{
    if (!h || !host_out) return SGP_ERR_INVALID_ARG;
    if (h->pend_count == 0) return SGP_ERR_SEQUENCE;
    const int idx = h->pend_head;
    SGP_HIP_TRY(h, hipEventSynchronize(h->ev_res[1 + idx]));
    read_stats(h, 1 + idx, host_out, per_node_dist_host);
    h->pend_head = (idx + 1) % 2;
    --h->pend_count;
    return SGP_OK;
}

int sgp_set_kernel_timing(sgp_handle *h, int enable)
{
    if (!h) return SGP_ERR_INVALID_ARG;
    if (enable && !h->ev_timing_made) {   // here, not inside a step: a step allocates nothing after its first launch
        h->ev_timing_made = true;         // release_device destroys whatever was created
        for (int i = 0; i < SGP_TIMING_RING; ++i) {
            SGP_HIP_TRY(h, hipEventCreate(&h->ev[i][0]));
            SGP_HIP_TRY(h, hipEventCreate(&h->ev[i][1]));
        }
    }
    h->timing = enable != 0;
    h->ev_read = h->ev_head;
    return SGP_OK;
}

int sgp_step_kernel_times(sgp_handle *h, float *ms_out, int32_t max, int32_t *count)
{
    if (!h || !ms_out || !count || max < 0) return SGP_ERR_INVALID_ARG;
    *count = 0;
    int64_t first = h->ev_read;
    if (h->ev_head - first > SGP_TIMING_RING) first = h->ev_head - SGP_TIMING_RING;
    if (h->ev_head - first > max) first = h->ev_head - max;
    if (h->ev_head == first) return SGP_OK;
    SGP_HIP_TRY(h, hipEventSynchronize(h->ev[(h->ev_head - 1) % SGP_TIMING_RING][1]));
    for (int64_t i = first; i < h->ev_head; ++i) {
        hipEvent_t *e = h->ev[i % SGP_TIMING_RING];
        SGP_HIP_TRY(h, hipEventElapsedTime(&ms_out[(*count)++], e[0], e[1]));
    }
    h->ev_read = h->ev_head;
    return SGP_OK;
}

int sgp_debias(sgp_handle *h, const float *x, const float *w, float *z, void *stream)
{
    if (!h || !x || !w || !z) return SGP_ERR_INVALID_ARG;
    if (!aligned4(x) || !aligned4(w) || !aligned4(z)) return SGP_ERR_ALIGNMENT;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool vec = (h->ld % 4 == 0) && aligned16(x) && aligned16(z);
    const long cols4 = vec ? (long)(h->d / 4) : 0;
    const size_t tail0 = (size_t)cols4 * 4;
    const long tail = (long)(h->d - (int64_t)tail0);
    if (cols4 > 0)
        hipLaunchKernelGGL(k_debias<4>, dim3(grid_for(cols4, kBlock), h->n), dim3(kBlock), 0, st, x, w,
                           z, (size_t)h->ld, (size_t)0, cols4);
    if (tail > 0)
        hipLaunchKernelGGL(k_debias<1>, dim3(grid_for(tail, kBlock), h->n), dim3(kBlock), 0, st, x, w,
                           z, (size_t)h->ld, tail0, tail);
    SGP_HIP_TRY(h, hipGetLastError());
    return SGP_OK;
}

// Launches the stand-alone statistics kernels over z (mode 0) or over the on-the-fly half step
// (mode 1, 2): every block writes its column of the partial table [(n+1)][G]; blocks beyond the tile
// count write 0, so the table needs no clearing.
static void launch_stats_passes(int n, int64_t d, int64_t ld, const float *z, const StatSource &src, int mode,
                                bool vec, float *partial, int G, hipStream_t st)
{
    const long cols4 = vec ? (long)(d / 4) : 0;
    const size_t tail0 = (size_t)cols4 * 4;
    const long tail = (long)(d - (int64_t)tail0);
    const size_t lds_large = (size_t)(kBlock / 64) * (n + 1) * sizeof(float);

    bool first = true;
    auto run = [&](auto vtag, auto mtag, size_t col0, long ncols) {
        constexpr int V = decltype(vtag)::value;
        constexpr int MODE = decltype(mtag)::value;
        long ntiles = (ncols + kBlock - 1) / kBlock;
        int acc = first ? 0 : 1;
        if (n <= kStatsCache)
            hipLaunchKernelGGL((k_stats_small<V, MODE>), dim3(G), dim3(kBlock), 0, st, z, src, n,
                               (size_t)ld, col0, ncols, ntiles, partial, G, acc);
        else
            hipLaunchKernelGGL((k_stats_large<V, MODE>), dim3(G), dim3(kBlock), lds_large, st, z, src, n,
                               (size_t)ld, col0, ncols, ntiles, partial, G, acc);
        first = false;
    };
    auto both = [&](auto mtag) {
        if (cols4 > 0) run(std::integral_constant<int, 4>{}, mtag, 0, cols4);
        if (tail > 0) run(std::integral_constant<int, 1>{}, mtag, tail0, tail);
    };
    if (mode == 0) both(std::integral_constant<int, 0>{});
    else if (mode == 1) both(std::integral_constant<int, 1>{});
    else both(std::integral_constant<int, 2>{});
}

// The stand-alone statistics on a handle: the passes above, then the final reduction, into result
// slot `slot` (0: copy to the host and wait; else enqueue only).
static int run_stats(sgp_handle *h, const float *z, const StatSource &src, int mode, bool vec, const float *w,
                     sgp_stats *host_out, double *per_node_dist_host, hipStream_t st, int slot)
{
    launch_stats_passes(h->n, h->d, h->ld, z, src, mode, vec, h->d_partial, h->G, st);
    SGP_HIP_TRY(h, hipGetLastError());
    if (slot != 0) return enqueue_stats(h, nullptr, w, slot, st);
    return finish_stats(h, nullptr, w, host_out, per_node_dist_host, st);
}

int sgp_consensus_stats(sgp_handle *h, const float *z, const float *w, sgp_stats *host_out,
                        double *per_node_dist_host, void *stream)
{
    if (!h || !z || !w || !host_out) return SGP_ERR_INVALID_ARG;
    if (!aligned4(z) || !aligned4(w)) return SGP_ERR_ALIGNMENT;
    int rc = ensure_device(h);
    if (rc != SGP_OK) return rc;
    const bool vec = (h->ld % 4 == 0) && aligned16(z);
    return run_stats(h, z, StatSource{}, 0, vec, w, host_out, per_node_dist_host,
                     static_cast<hipStream_t>(stream), 0);
}

int sgp_pregossip_stats(sgp_handle *h, const float *x, const float *w, const float *m, const float *g,
                        float gamma, float momentum, sgp_stats *host_out, double *per_node_dist_host,
                        void *stream)
{
    if (!h || !x || !w || !g || !host_out) return SGP_ERR_INVALID_ARG;
    const bool nest = momentum != 0.0f;
    if (nest && !m) return SGP_ERR_INVALID_ARG;
    if (!aligned4(x) || !aligned4(w) || !aligned4(g) || (nest && !aligned4(m))) return SGP_ERR_ALIGNMENT;
    int rc = ensure_device(h);
    if (rc != SGP_OK) return rc;
    StatSource src{};
    src.x = x;
    src.u = m;
    src.g = g;
    src.w = h->biased ? nullptr : w;
    src.hp.gamma = gamma;
    src.hp.mom = momentum;
    src.hp.wd = h->wd;
    src.hp.wd_mode = h->wd == 0.0f ? 0 : (h->wd_on_x || h->biased) ? 1 : 2;
    const bool vec = (h->ld % 4 == 0) && aligned16(x) && aligned16(g) && (!nest || aligned16(m));
    return run_stats(h, nullptr, src, nest ? 2 : 1, vec, w, host_out, per_node_dist_host,
                     static_cast<hipStream_t>(stream), 0);
}

}  // extern "C"

// ------------------------------------------------------------------------------------------
// Statistics without any allocation: the partial table and the row sums live in a file-scope
// device array.  Every GPU holds its own copy of the array at its own address; the address is
// looked up once per device and used from then on (the array's name is not a device address in
// host code).
// ------------------------------------------------------------------------------------------
namespace {

constexpr int kNoAllocGrid = kStatsGridMax;
constexpr size_t kNoAllocPartialBytes = (size_t)(SGP_NOALLOC_MAX_NODES + 1) * kNoAllocGrid * sizeof(float);
constexpr size_t kNoAllocSumsBytes = ((size_t)(SGP_NOALLOC_MAX_NODES + 1) * sizeof(double) + 255) / 256 * 256;
constexpr size_t kNoAllocScratchBytes = kNoAllocPartialBytes + kNoAllocSumsBytes;
static_assert(kNoAllocPartialBytes % 256 == 0, "the row sums start on a 256-byte boundary");

constexpr int kNoAllocMaxDevices = 64;
std::mutex g_noalloc_mutex;
void *g_noalloc_ptr[kNoAllocMaxDevices];   // device address of this device's copy, once looked up

}  // namespace

static __device__ __align__(256) unsigned char sgp_noalloc_scratch[kNoAllocScratchBytes];

extern "C" {

int sgp_consensus_stats_noalloc(int32_t n, int64_t d, int64_t ld, const float *z, const float *w,
                                double *out_device, void *stream)
{
    if (n < 1 || d < 1 || ld < d || !z || !w || !out_device) return SGP_ERR_INVALID_ARG;
    if (n > SGP_NOALLOC_MAX_NODES) return SGP_ERR_UNSUPPORTED;   // beyond the fixed scratch array
    if (!aligned4(z) || !aligned4(w) || (reinterpret_cast<uintptr_t>(out_device) & 7u)) return SGP_ERR_ALIGNMENT;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SGP_ERR_HIP;
    if (dev < 0 || dev >= kNoAllocMaxDevices) return SGP_ERR_UNSUPPORTED;
    void *base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_noalloc_mutex);
        if (!g_noalloc_ptr[dev]) {
            void *p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(sgp_noalloc_scratch)) != hipSuccess || !p) return SGP_ERR_HIP;
            g_noalloc_ptr[dev] = p;
        }
        base = g_noalloc_ptr[dev];
    }
    float *partial = static_cast<float *>(base);
    double *sums = reinterpret_cast<double *>(static_cast<unsigned char *>(base) + kNoAllocPartialBytes);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool vec = (ld % 4 == 0) && aligned16(z);
    // every block of every pass writes its whole column of the table (zeros where it has no
    // tile), and k_stats_rowsum writes every sum: nothing of the previous call is read
    launch_stats_passes(n, d, ld, z, StatSource{}, 0, vec, partial, kNoAllocGrid, st);
    hipLaunchKernelGGL(k_stats_rowsum, dim3(n + 1), dim3(kRowSumBlock), 0, st, partial, kNoAllocGrid, sums);
    hipLaunchKernelGGL(k_stats_final, dim3(1), dim3(64), 0, st, sums, n, w, out_device);
    if (hipGetLastError() != hipSuccess) return SGP_ERR_HIP;
    return SGP_OK;
}

int sgp_smooth_region_classes(int32_t *class_of_granule, int32_t count)
{
    if (count < 0 || (count > 0 && !class_of_granule)) return SGP_ERR_INVALID_ARG;
    int32_t *cls = class_of_granule;
    // regions are contiguous address ranges: a single granule whose two neighbours agree with each
    // other but not with it is a timing outlier and takes their class
    for (int i = 1; i + 1 < count; ++i)
        if (cls[i - 1] == cls[i + 1] && cls[i] != cls[i - 1]) cls[i] = cls[i - 1];
    // classes renumbered in order of first appearance
    std::vector<int32_t> order;
    for (int i = 0; i < count; ++i) {
        int pos = -1;
        for (size_t q = 0; q < order.size(); ++q)
            if (order[q] == cls[i]) pos = (int)q;
        if (pos < 0) {
            order.push_back(cls[i]);
            pos = (int)order.size() - 1;
        }
        cls[i] = pos;
    }
    return SGP_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------
// Carving arrays out of a probed arena (host-only integer logic).
// ------------------------------------------------------------------------------------------
struct sgp_placer {
    int64_t granule;
    std::vector<int32_t> classes;
    // free byte ranges [start, end) per class, in the order they are tried
    std::vector<std::vector<std::pair<int64_t, int64_t>>> free_ranges;
    std::vector<int32_t> order;   // classes by capacity, largest first
};

namespace {

void placer_fill(sgp_placer *p)
{
    const int count = (int)p->classes.size();
    int ncls = 0;
    for (int32_t c : p->classes) ncls = std::max(ncls, c + 1);
    const int64_t g = p->granule;
    p->free_ranges.assign((size_t)ncls, {});
    std::vector<int64_t> capacity((size_t)ncls, 0);
    for (int c = 0; c < ncls; ++c) {
        std::vector<std::pair<int, int>> runs;   // (first granule, length) of the maximal runs of class c
        for (int i = 0; i < count;) {
            if (p->classes[i] != c) { ++i; continue; }
            int j = i;
            while (j < count && p->classes[j] == c) ++j;
            runs.push_back({i, j - i});
            capacity[c] += (int64_t)(j - i) * g;
            i = j;
        }
        std::stable_sort(runs.begin(), runs.end(),
                         [](const std::pair<int, int> &a, const std::pair<int, int> &b) { return a.second > b.second; });
        // the interiors of the long runs first, longest first (a granule at the edge of a run may
        // straddle a region boundary, and a short run may be a timing outlier), then what was
        // trimmed off, then the short runs
        std::vector<std::pair<int64_t, int64_t>> inner, edges, shorts;
        for (const auto &r : runs) {
            const int64_t s0 = r.first, k = r.second;
            if (k >= 4) {
                inner.push_back({(s0 + 1) * g, (s0 + k - 1) * g});
                edges.push_back({s0 * g, (s0 + 1) * g});
                edges.push_back({(s0 + k - 1) * g, (s0 + k) * g});
            } else {
                shorts.push_back({s0 * g, (s0 + k) * g});
            }
        }
        auto &dst = p->free_ranges[c];
        dst.insert(dst.end(), inner.begin(), inner.end());
        dst.insert(dst.end(), edges.begin(), edges.end());
        dst.insert(dst.end(), shorts.begin(), shorts.end());
    }
    p->order.resize((size_t)ncls);
    for (int c = 0; c < ncls; ++c) p->order[c] = c;
    std::stable_sort(p->order.begin(), p->order.end(),
                     [&](int32_t a, int32_t b) { return capacity[a] > capacity[b]; });
}

}  // namespace

extern "C" {

int sgp_placer_create(sgp_placer **out, const int32_t *class_of_granule, int32_t count, int64_t granule_bytes)
{
    if (!out) return SGP_ERR_INVALID_ARG;
    *out = nullptr;
    if (!class_of_granule || count < 1 || granule_bytes < 4096 || (granule_bytes & 4095)) return SGP_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i)
        if (class_of_granule[i] < 0 || class_of_granule[i] > 1024) return SGP_ERR_INVALID_ARG;
    sgp_placer *p = new (std::nothrow) sgp_placer();
    if (!p) return SGP_ERR_NOMEM;
    p->granule = granule_bytes;
    p->classes.assign(class_of_granule, class_of_granule + count);
    placer_fill(p);
    *out = p;
    return SGP_OK;
}

int sgp_placer_destroy(sgp_placer *p)
{
    delete p;
    return SGP_OK;
}

int sgp_placer_reset(sgp_placer *p)
{
    if (!p) return SGP_ERR_INVALID_ARG;
    placer_fill(p);
    return SGP_OK;
}

int sgp_placer_take(sgp_placer *p, int32_t role, int64_t nbytes, int64_t *offset_out, int32_t *class_out)
{
    // which of the regions (ranked by capacity) a role prefers: the written streams x, u, z go to
    // three different ones; g is read-only and shares the region of x; both message buffers of
    // overlap mode go with u (one written into the region of z measured 2.5 % slower); Adam's second
    // moment goes with x.  Measured over all 3^7 assignments of x, u, v, g, z and the two message
    // buffers to the regions (n = 16, d = 53 M, two peers, one iteration of delay): with Adam this map
    // is within 0.3 % of the best one (and 2.2 % faster than v with z and the second message buffer
    // with x), without Adam within 0.4 %.
    static const int kWant[SGP_ROLE_COUNT] = {0, 0, 1, 2, 1, 1, 0};
    if (!p || !offset_out || role < 0 || role >= SGP_ROLE_COUNT || nbytes < 1) return SGP_ERR_INVALID_ARG;
    const int64_t need = (nbytes + 4095) / 4096 * 4096;
    const int ncls = (int)p->order.size();
    for (int j = 0; j < ncls; ++j) {          // the preferred region, then any other with room
        const int32_t cls = p->order[(size_t)((kWant[role] + j) % ncls)];
        for (auto &run : p->free_ranges[(size_t)cls])
            if (run.second - run.first >= need) {
                *offset_out = run.first;
                run.first += need;
                if (class_out) *class_out = cls;
                return SGP_OK;
            }
    }
    return SGP_ERR_NOMEM;
}

// Times the probe problem with its state arrays in granule `ref` and z in granule `cand`: median
// step-kernel duration of the last four of six iterations.
static int probe_time(sgp_handle *h, unsigned char *arena, int64_t granule, size_t arr, int ref, int cand,
                      float *w_dev, hipStream_t st, float *ms_out)
{
    const int n = h->n;
    float *x = reinterpret_cast<float *>(arena + (size_t)ref * granule);
    float *u = reinterpret_cast<float *>(arena + (size_t)ref * granule + arr);
    float *g = reinterpret_cast<float *>(arena + (size_t)ref * granule + 2 * arr);
    float *z = reinterpret_cast<float *>(arena + (size_t)cand * granule + (cand == ref ? 3 * arr : 0));
    float ones[32];
    for (int i = 0; i < n; ++i) ones[i] = 1.0f;
    SGP_HIP_TRY(h, hipMemsetAsync(x, 0, 3 * arr, st));
    SGP_HIP_TRY(h, hipMemcpyAsync(w_dev, ones, (size_t)n * sizeof(float), hipMemcpyHostToDevice, st));
    SGP_HIP_TRY(h, hipStreamSynchronize(st));      // `ones` is on this stack frame
    for (int k = 0; k < 6; ++k) {
        int rc = sgp_step(h, x, w_dev, u, g, z, 0.1f, 0.9f, k, st);
        if (rc != SGP_OK) return rc;
    }
    float ms[8];
    int32_t cnt = 0;
    int rc = sgp_step_kernel_times(h, ms, 8, &cnt);
    if (rc != SGP_OK) return rc;
    if (cnt != 6) return SGP_ERR_HIP;
    std::sort(ms + 2, ms + 6);
    *ms_out = ms[4];
    return SGP_OK;
}

int sgp_probe_regions(void *arena, int64_t arena_bytes, int64_t granule_bytes, int32_t max_classes,
                      int32_t *class_of_granule, float *probe_ms, int32_t *structured, void *stream)
{
    constexpr int kProbeNodes = 32;
    constexpr int64_t kProbeD = (int64_t)1 << 22;
    if (!arena || !class_of_granule || !structured || granule_bytes < 4096 || (granule_bytes & 4095) ||
        arena_bytes < granule_bytes || max_classes < 1 || !aligned16(arena))
        return SGP_ERR_INVALID_ARG;
    const int64_t count64 = arena_bytes / granule_bytes;
    if (count64 > (1 << 20)) return SGP_ERR_INVALID_ARG;
    const int count = (int)count64;
    const size_t arr = (size_t)kProbeNodes * kProbeD * sizeof(float);
    *structured = 0;
    for (int i = 0; i < count; ++i) {
        class_of_granule[i] = 0;
        if (probe_ms) probe_ms[i] = 0.0f;
    }
    if (count < 2 || (int64_t)(4 * arr) > granule_bytes) return SGP_OK;   // nothing to tell apart

    sgp_handle *h = nullptr;
    int rc = sgp_create(&h, kProbeNodes, kProbeD, kProbeD, SGP_TOPO_DIRECTED_EXP, 1, 0);
    if (rc != SGP_OK) return rc;
    float *w_dev = nullptr;
    std::vector<int> cls((size_t)count, -1);
    std::vector<float> times((size_t)count, 0.0f);
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char *base = static_cast<unsigned char *>(arena);
    rc = sgp_set_kernel_timing(h, 1);
    if (rc == SGP_OK && dev_malloc(&w_dev, kProbeNodes * sizeof(float)) != hipSuccess) rc = SGP_ERR_NOMEM;
    for (int c = 0; c < max_classes && rc == SGP_OK; ++c) {
        int ref = -1;
        for (int i = 0; i < count && ref < 0; ++i)
            if (cls[i] < 0) ref = i;
        if (ref < 0) break;
        float lo = 0.0f, hi = 0.0f;
        bool first = true;
        for (int i = 0; i < count && rc == SGP_OK; ++i) {
            if (cls[i] >= 0) continue;
            rc = probe_time(h, base, granule_bytes, arr, ref, i, w_dev, st, &times[i]);
            if (c == 0 && probe_ms) probe_ms[i] = times[i];
            lo = first ? times[i] : std::min(lo, times[i]);
            hi = first ? times[i] : std::max(hi, times[i]);
            first = false;
        }
        if (rc != SGP_OK) break;
        if (hi < 1.08f * lo) {          // no contrast: everything left behaves like the reference
            for (int i = 0; i < count; ++i)
                if (cls[i] < 0) cls[i] = c;
            break;
        }
        *structured = 1;
        const float mid = 0.5f * (lo + hi);
        for (int i = 0; i < count; ++i)
            if (cls[i] < 0 && times[i] > mid) cls[i] = c;   // slow with the reference: same region
        cls[ref] = c;
    }
    if (w_dev) (void)hipFree(w_dev);
    (void)sgp_destroy(h);
    if (rc != SGP_OK) return rc;
    for (int i = 0; i < count; ++i)
        if (cls[i] < 0) cls[i] = max_classes - 1;
    for (int i = 0; i < count; ++i) class_of_granule[i] = cls[i];
    return sgp_smooth_region_classes(class_of_granule, count);
}

int sgp_copy(void *dst, const void *src, int64_t nbytes, void *stream)
{
    if (!dst || !src || nbytes < 0 || (nbytes & 15) || !aligned16(dst) || !aligned16(src))
        return SGP_ERR_INVALID_ARG;
    if (nbytes == 0) return SGP_OK;
    size_t count = (size_t)nbytes / 16;
    size_t blocks = (count + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffffu) return SGP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_copy, dim3((unsigned)blocks), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                       static_cast<floatx4 *>(dst), static_cast<const floatx4 *>(src), count);
    if (hipGetLastError() != hipSuccess) return SGP_ERR_HIP;
    return SGP_OK;
}

int sgp_stream_pattern(const void *const *reads, int32_t n_reads, void *const *writes, int32_t n_writes,
                       int64_t nbytes, void *stream)
{
    if (n_reads < 0 || n_reads > kPatternMax || n_writes < 0 || n_writes > kPatternMax || n_reads + n_writes == 0 ||
        nbytes < 0 || (nbytes & 15) || (n_reads && !reads) || (n_writes && !writes))
        return SGP_ERR_INVALID_ARG;
    PatternPtrs p{};
    for (int j = 0; j < n_reads; ++j) {
        if (!reads[j] || !aligned16(reads[j])) return SGP_ERR_INVALID_ARG;
        p.r[j] = static_cast<const floatx4 *>(reads[j]);
    }
    for (int j = 0; j < n_writes; ++j) {
        if (!writes[j] || !aligned16(writes[j])) return SGP_ERR_INVALID_ARG;
        p.w[j] = static_cast<floatx4 *>(writes[j]);
    }
    // arrays may coincide (a written array that is also read: in place) but not overlap otherwise
    auto overlap_ok = [&](const void *a, const void *b) {
        const char *ca = static_cast<const char *>(a), *cb = static_cast<const char *>(b);
        return ca == cb || ca + nbytes <= cb || cb + nbytes <= ca;
    };
    for (int j = 0; j < n_writes; ++j) {
        for (int q = 0; q < n_reads; ++q)
            if (!overlap_ok(writes[j], reads[q])) return SGP_ERR_INVALID_ARG;
        for (int q = 0; q < j; ++q)
            if (writes[q] == writes[j] || !overlap_ok(writes[j], writes[q])) return SGP_ERR_INVALID_ARG;
    }
    if (nbytes == 0) return SGP_OK;
    const size_t count = (size_t)nbytes / 16;
    const size_t blocks = (count + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffffu) return SGP_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_stream_pattern, dim3((unsigned)blocks), dim3(kBlock), 0, static_cast<hipStream_t>(stream), p,
                       n_reads, n_writes, count);
    if (hipGetLastError() != hipSuccess) return SGP_ERR_HIP;
    return SGP_OK;
}

}  // extern "C"
