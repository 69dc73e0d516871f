// Shared by the translation units of the library (not part of the public interface): tuning
// knobs, launch constants, the argument structures that host code hands to the kernels, and the
// launchers that one translation unit defines for the others.  The kernels are spread over several
// translation units only so that they compile side by side; every unit includes this header first
// and keeps its kernels in an anonymous namespace.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstddef>
#include <cstdint>

// Tuning knobs (overridable at build time for tuning runs; the same value in every unit).
// One-peer step kernel: single-wave blocks, one 128-bit column group per work-item measured best
// (n = 32, d = 25.6 M: 3.05 ms; 256 x 4: 3.07 ms; 256 x 2: 3.17 ms).
#ifndef SGP_OP_BLOCK
#define SGP_OP_BLOCK 64
#endif
#ifndef SGP_OP_COLS
#define SGP_OP_COLS 1
#endif
#ifndef SGP_DELAY_BLOCK
#define SGP_DELAY_BLOCK 256
#endif
#ifndef SGP_DELAY_COLS
#define SGP_DELAY_COLS 2
#endif
#ifndef SGP_DELAY_WINDOW
#define SGP_DELAY_WINDOW 1   // two-peer overlap: walk with the stride of the two hops (0: table walk)
#endif
#ifndef SGP_NT_LOAD
#define SGP_NT_LOAD 1
#endif
#ifndef SGP_NT_STORE
#define SGP_NT_STORE 1
#endif
#ifndef SGP_STATS_BLOCK
#define SGP_STATS_BLOCK 64
#endif
#ifndef SGP_STATS_DEPTH
#define SGP_STATS_DEPTH 4
#endif
#ifndef SGP_STATS_EXACT
#define SGP_STATS_EXACT 1    // walk with statistics: bodies with the node count known exactly for 4, 8, 16, 32
#endif
#ifndef SGP_H16_COLS
#define SGP_H16_COLS 1
#endif
#ifndef SGP_XCD_REMAP
#define SGP_XCD_REMAP 1
#endif

namespace sgp_detail {

// Local optimiser of the step kernels (template parameter OPT).
constexpr int kOptSgd = 0;        // Alg. 1, gradient step
constexpr int kOptNesterov = 1;   // Alg. 3, momentum and gradient steps
constexpr int kOptAdam = 2;       // Adam as published, on the numerator (hyperparameter appendix)

// Hyperparameters of the local optimiser step, as the kernels take them.
struct Hyper {
    float gamma;          // step size
    float mom;            // Nesterov coefficient
    float wd;             // weight decay coefficient
    int wd_mode;          // 0: none; 1: decay acts on the numerator x; 2: on the de-biased x / w^(k)
    // Adam only: second-moment array [n][ld] (the first moment lives in the momentum array), the
    // decay rates with their complements, the bias corrections 1 - beta^t and epsilon
    float *v2;
    float beta1, c1, beta2, c2, bc1, bc2, eps;
};

// ------------------------------------------------------------------------------------------
// Push-sum weights (Alg. 1, weight update: w_i <- sum_j p_ij w_j) inside the step kernels.
// n floats are nothing next to the n x d state, so every block forms all n new weights itself at
// its start, from the caller's array, which keeps the OLD weights for as long as the kernel runs:
// the block that finishes last (counters in device memory tell) writes the new ones back, and only
// if they differ from the old ones at all.  A step is then one kernel launch, with no one-block
// weight kernel in front of it.
// ------------------------------------------------------------------------------------------
constexpr int kWKeep = 0;       // no communication at this iteration: w stays
constexpr int kWOnePeer = 1;    // p w_i + p w_{(i - hop) mod n}; hop < 0: no peer, p w_i
constexpr int kWTable = 2;      // sum over the sorted source list tab[i][0..S), uniform weight p
constexpr int kWComplete = 3;   // sum_j p w_j, ascending j
constexpr int kWCustom = 4;     // caller-supplied rows: sum over the used entries of tabw * w_j, in order
constexpr int kWDelay = 5;      // own share p w_i plus the pre-weighted weights in flight of the
                                // senders in tab[i][0..S) other than i; the share is also sent on

struct WeightOp {
    float *w;                  // [n] caller's weights: w^(k) while the kernel runs, w^(k+1) afterwards
    int kind;
    int hop;                   // kWOnePeer
    const int *tab;            // kWTable, kWDelay (NULL: nothing in flight), kWCustom (-1 = unused entry)
    const float *tabw;         // kWCustom
    int S;
    float p;                   // uniform mixing weight
    const float *msgw_prev;    // kWDelay: [n] pre-weighted weights sent at the previous round
    float *msgw_cur;           //          [n] the ones sent now
    int biased;                // ablation without the push-sum weight: never divide, z = x
    int publish;               // this launch is the last one of its step: its last block writes w
    float *w_snap;             // nullable: a second copy of w^(k+1), written by the launch's first block, for a
                               // statistics reduction that may still be running when the next step overwrites w
    unsigned *done;            // counters of finished blocks (layout at publish_weights); zero between launches
};

// Counters of finished blocks: two levels, so that a hundred thousand blocks do not queue up at one
// address (see publish_weights).
constexpr int kCountLines = 64;     // first-level counters
constexpr int kCountStride = 32;    // unsigned per 128-byte line; counter j lives at done[j * kCountStride],
                                    // j = 0: top level, j = 1 .. kCountLines: first level

// LDS bytes a step kernel needs for the two weight arrays.
__host__ __device__ constexpr size_t weight_lds_bytes(int n) { return ((size_t)2 * n * sizeof(float) + 15) / 16 * 16; }

constexpr int kBlock = 256;     // work-items per block of the streaming kernels
constexpr int kGatherBlock = 64;
constexpr int kGatherVecMaxNodes = 150;   // private LDS columns of 128-bit values: 150 KiB + weights per block
                                          // (a workgroup can address 160 KiB on gfx950)
constexpr int kBatch = 4;       // nodes whose loads are issued back to back before any use

constexpr int kOpBlock = SGP_OP_BLOCK;   // one-peer walk: work-items per block
constexpr int kOpCols = SGP_OP_COLS;     //                128-bit column groups per work-item
constexpr int kH16Cols = SGP_H16_COLS;   // 16-bit storage walk: column groups (of V coordinates) per work-item
constexpr int kDelayBlock = SGP_DELAY_BLOCK;   // overlap kernels: work-items per block
constexpr int kDelayCols = SGP_DELAY_COLS;     //                  128-bit column groups per work-item

constexpr int kStatsCache = 32;   // nodes whose z the fused and the small-n statistics kernels keep in registers
constexpr int kStatsStepBlock = SGP_STATS_BLOCK;   // work-items per block of the walk with fused statistics
constexpr int kStatsDepth = SGP_STATS_DEPTH;       // rows whose loads are in flight per work-item there

static_assert(kStatsStepBlock == kGatherBlock && kStatsStepBlock == kOpBlock,
              "every kernel with fused statistics writes one line of partial sums per 64 column groups");

// What every step launcher needs besides its own arguments.
struct StepArgs {
    float *x, *u, *z;
    const float *g;
    WeightOp wop;
    int n;
    size_t ld;
    float p;
    Hyper hp;
    hipStream_t stream;
    const char **name;    // receives the name of the kernel launched
    bool cached;          // small problem: ordinary loads and stores instead of streaming ones
};

inline unsigned grid_for(long ncols, int block) { return (unsigned)((ncols + block - 1) / block); }

inline int gcd_int(int a, int b)
{
    while (b) { int t = a % b; a = b; b = t; }
    return a;
}

// LDS of the gather kernel: the two weight arrays, then one private column of n values per work-item.
inline size_t gather_lds_bytes(int n, int V) { return weight_lds_bytes(n) + (size_t)n * kGatherBlock * V * sizeof(float); }

// fin != NULL: the launch carries the statistics and `fin` is attached to the kernel as its
// completion event.
template <typename K, typename... Args>
void launch_step(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, hipEvent_t fin, Args... args)
{
    if (fin) hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, nullptr, fin, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
}

// ------------------------------------------------------------------------------------------
// Launchers defined in one translation unit and called from sgp.hip.  None of them checks its
// arguments or the launch: the caller has validated shapes and reads hipGetLastError afterwards.
// V is 4 (128-bit column groups, ncols of them starting at group-aligned column col0) or 1.
// ------------------------------------------------------------------------------------------

// sgp_walk_stats.hip, compiled once per variant: the unrolled walk with the statistics taken from
// registers, for any n <= kStatsCache: one out-peer (or none) without delay (MSG = 0), or one
// iteration of delay with MSG = 1 or 2 out-peers (msg_prev, msg_cur, the previous round's hops ha
// and, MSG = 2, hb; otherwise unused).  The variants that exist are declared here; MSG != 0 has no
// CACHED form.
template <bool NEST, bool CACHED, int MSG>
void launch_walk_stats_variant(const StepArgs &a, long cols4, int h, int len, float *partial, hipEvent_t fin,
                               const float *msg_prev, float *msg_cur, int ha, int hb);
#define SGP_DECLARE_WALK_STATS(NEST, CACHED, MSG)                                                              \
    template <>                                                                                                \
    void launch_walk_stats_variant<NEST, CACHED, MSG>(const StepArgs &a, long cols4, int h, int len,          \
                                                      float *partial, hipEvent_t fin, const float *msg_prev,  \
                                                      float *msg_cur, int ha, int hb);
SGP_DECLARE_WALK_STATS(false, false, 0)
SGP_DECLARE_WALK_STATS(true, false, 0)
SGP_DECLARE_WALK_STATS(false, true, 0)
SGP_DECLARE_WALK_STATS(true, true, 0)
SGP_DECLARE_WALK_STATS(false, false, 1)
SGP_DECLARE_WALK_STATS(true, false, 1)
SGP_DECLARE_WALK_STATS(false, false, 2)
SGP_DECLARE_WALK_STATS(true, false, 2)
#undef SGP_DECLARE_WALK_STATS

// sgp_gather.hip (compiled twice, without and with the statistics): several out-peers or
// caller-supplied rows (tabw != NULL), through private LDS columns.  With statistics: Alg. 1 or
// Alg. 3 only, 128-bit layout from column 0, z written, n <= kStatsCache.
void launch_gather(const StepArgs &a, int V, int opt, bool zout, size_t col0, long ncols, const int *tab,
                   const float *tabw, int S);
void launch_gather_stats(const StepArgs &a, int opt, long ncols, const int *tab, const float *tabw, int S,
                         float *partial, hipEvent_t fin);

// sgp_overlap.hip: one iteration of delay; tab_prev == NULL: nothing in flight yet.
void launch_delay(const StepArgs &a, int V, int opt, bool zout, size_t col0, long ncols, const float *msg_prev,
                  float *msg_cur, const int *tab_prev, int S, int ha, int hb);

}  // namespace sgp_detail
