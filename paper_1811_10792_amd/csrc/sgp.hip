// SGP update for n simulated nodes resident in one MI355X's HBM: host-side peer scheduler, HIP
// kernels for gfx950 and the C ABI declared in include/sgp.h.
//
// Kernel design.  The PushSum mix couples nodes but never coordinates (x <- P x acts on the
// n-vector of one coordinate), so a work-item owns a 128-bit group of four coordinates for ALL
// n nodes.  It reads x, u, g of every node once, writes u, x, z once, and the "messages" of
// Alg. 1 line 5 never leave registers (or LDS): 24 bytes of HBM traffic per node-parameter, the
// algorithmic minimum, and the in-place update is race-free because no other work-item touches
// those coordinates.  Everything is a stream (about 0.4 flop per byte), so there is no MFMA
// here; what matters is 128-bit coalesced accesses and enough loads in flight per CU.
//
// All floating-point code in this file is compiled without multiply-add contraction, so each
// operation rounds separately, in the order written.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>

#include "sgp.h"

#pragma clang fp contract(off)

// Tuning knobs (overridable at build time for tuning runs).
// One-peer step kernel: single-wave blocks, one 128-bit column group per work-item measured best
// (n = 32, d = 25.6 M: 3.05 ms; 256 x 4: 3.07 ms; 256 x 2: 3.17 ms).
#ifndef SGP_OP_BLOCK
#define SGP_OP_BLOCK 64
#endif
#ifndef SGP_OP_DYNLDS
#define SGP_OP_DYNLDS 0   // unused dynamic LDS per block: an occupancy limiter for experiments
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

namespace {

// ------------------------------------------------------------------------------------------
// Peer scheduler (host, integers only).  Appendix A: the peer list holds the hop distances
// 2^0 .. 2^floor(log2(n-1)), L = floor(log2(n-1)) + 1 entries; at iteration k a node sends to
// `peers` consecutive entries starting at entry k mod L (wrapping), i.e. to (i + hop) mod n.
// ------------------------------------------------------------------------------------------
struct Schedule {
    int L;                        // entries in the peer list (0 when n == 1)
    int distinct;                 // distinct hop distances used at this iteration
    int hop[SGP_MAX_PEERS];       // hop per requested peer slot, -1 where it repeats an earlier one
    int uniq[SGP_MAX_PEERS];      // the distinct hops, in slot order
    float p;                      // uniform weight 1 / (1 + distinct)
};

int peer_list_length(int n)
{
    int L = 0;
    for (int t = n - 1; t > 0; t >>= 1) ++L;   // bit length of n-1
    return L;
}

Schedule make_schedule(int n, int peers, int64_t k)
{
    Schedule s;
    s.L = peer_list_length(n);
    s.distinct = 0;
    for (int r = 0; r < peers; ++r) {
        s.hop[r] = -1;
        if (s.L == 0) continue;
        int hop = 1 << (int)((k + r) % s.L);
        bool seen = false;
        for (int q = 0; q < s.distinct; ++q) seen = seen || (s.uniq[q] == hop);
        if (!seen) {
            s.hop[r] = hop;
            s.uniq[s.distinct++] = hop;
        }
    }
    s.p = 1.0f / (float)(1 + s.distinct);
    return s;
}

int gcd_int(int a, int b)
{
    while (b) { int t = a % b; a = b; b = t; }
    return a;
}

// ------------------------------------------------------------------------------------------
// Device helpers
// ------------------------------------------------------------------------------------------
typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int V> struct vec_of;
template <> struct vec_of<4> { typedef floatx4 type; };
template <> struct vec_of<1> { typedef float type; };

// The state arrays are 13-110 GB per step and are touched once: stream them past the caches.
template <int V>
__device__ __forceinline__ typename vec_of<V>::type ld_stream(const float *p)
{
#if SGP_NT_LOAD
    return __builtin_nontemporal_load(reinterpret_cast<const typename vec_of<V>::type *>(p));
#else
    return *reinterpret_cast<const typename vec_of<V>::type *>(p);
#endif
}
template <int V>
__device__ __forceinline__ void st_stream(float *p, typename vec_of<V>::type v)
{
#if SGP_NT_STORE
    __builtin_nontemporal_store(v, reinterpret_cast<typename vec_of<V>::type *>(p));
#else
    *reinterpret_cast<typename vec_of<V>::type *>(p) = v;
#endif
}
template <int V>
__device__ __forceinline__ typename vec_of<V>::type ld_cached(const float *p)
{
    return *reinterpret_cast<const typename vec_of<V>::type *>(p);
}

__device__ __forceinline__ float hsum(floatx4 v) { return (v.x + v.y) + (v.z + v.w); }
__device__ __forceinline__ float hsum(float v) { return v; }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
    return v;
}

// Step size, momentum and weight decay of the local optimiser step, as the kernels take them.
struct Hyper {
    float gamma;          // step size
    float mom;            // Nesterov coefficient
    float wd;             // weight decay coefficient
    int wd_mode;          // 0: none; 1: decay acts on the numerator x; 2: on the de-biased x / w^(k)
    const float *w_old;   // [n] weights before this iteration's update (read when wd_mode == 2)
};

// Local optimiser step on the numerator.  Alg. 3 lines 4-5: u <- m u + g; xh = x - gamma (m u + g)
// with the NEW u.  Alg. 1 line 4: xh = x - gamma g.  With weight decay g is replaced by
// g + wd * theta, theta = x or x / w_old (the hyperparameter appendix names a weight decay of 1e-4
// without saying which copy of the parameters it acts on; both are offered).
template <int V, bool NEST>
__device__ __forceinline__ typename vec_of<V>::type half_step(typename vec_of<V>::type xv,
                                                             typename vec_of<V>::type uv,
                                                             typename vec_of<V>::type gv,
                                                             const Hyper &hp, float *u_dst,
                                                             float w_old)
{
    typedef typename vec_of<V>::type T;
    if (hp.wd_mode != 0) {   // uniform over the grid
        T th = xv;
        if (hp.wd_mode == 2) th = xv / w_old;
        T dec = hp.wd * th;
        gv = gv + dec;
    }
    if (NEST) {
        T mu = hp.mom * uv;
        T un = mu + gv;
        st_stream<V>(u_dst, un);
        T mun = hp.mom * un;
        T dir = mun + gv;
        T stp = hp.gamma * dir;
        return xv - stp;
    } else {
        T stp = hp.gamma * gv;
        return xv - stp;
    }
}

// z = x / w, IEEE division.  When every weight is exactly 1 (any doubly-stochastic schedule
// started from w = 1, i.e. every non-delayed regular graph) the division is the identity bit for
// bit; the weight kernel records that in a device flag and the step kernels then run a copy of
// their loop without the division (DIV = false).
template <int V, bool DIV>
__device__ __forceinline__ typename vec_of<V>::type debias_val(typename vec_of<V>::type xn, float wi)
{
    if (DIV) return xn / wi;
    return xn;
}

constexpr int kBlock = 256;     // work-items per block of the streaming kernels
constexpr int kGatherBlock = 64;
constexpr int kBatch = 4;       // nodes whose loads are issued back to back before any use

constexpr int kOpBlock = SGP_OP_BLOCK;   // work-items per block
constexpr int kOpCols = SGP_OP_COLS;     // 128-bit column groups per work-item

// ------------------------------------------------------------------------------------------
// Fused step, one out-peer (or none, n == 1).  The in-neighbour of node i is (i - h) mod n, so
// walking a cycle c, c+h, c+2h, ... of the shift needs only the previous and the first xh of the
// cycle in registers, for any n and any run-time h.  There are gcd(n, h) cycles of n/gcd nodes.
//   x_new[i] = p*xh[i] + p*xh[(i-h) mod n]   (two exactly-rounded products; their sum does not
//                                             depend on the order of the two terms)
// ------------------------------------------------------------------------------------------
// The walk is software-pipelined.  On gfx9-family parts loads and stores share one in-order
// completion counter, so a wave that waits for freshly issued loads also waits for the write
// acknowledgements of every store issued before them.  Issuing the NEXT node's loads before the
// current node's stores keeps the stores out of that wait.  The walk over all cycles is
// flattened so that the pipeline never drains at a cycle boundary (hop n/2 has n/2 cycles of 2).
template <int V, bool NEST, int C>
struct RowRegs {
    typename vec_of<V>::type x[C], u[C], g[C];
    float w;    // new weight of the node (de-bias)
    float wo;   // its weight before this iteration (weight decay on the de-biased parameters)
    int node;
};

struct WalkPos {
    int cyc, pos, node;
    __device__ __forceinline__ void advance(int n, int h, int len)
    {
        if (++pos == len) {
            pos = 0;
            node = ++cyc;
        } else {
            node += h;
            if (node >= n) node -= n;
        }
    }
};

// What keeps the pipeline alive is that the compiler can count, at every wait, how many memory
// operations were issued after the loads it waits for.  It can only do that when every path through
// the code issues the same number, so:
//  - every row of the walk issues the same stores: its own u, and x and z of exactly ONE node.  A
//    node that opens a cycle cannot be finished before the cycle closes; its result is then parked
//    and written by the next row (which opens the next cycle and has nothing of its own to write);
//    the last parked node is written after the walk;
//  - full blocks run an instantiation without per-lane predicates (MASKED = false);
//  - the first row and the last one or two are peeled off, so that inside the loop the prefetch of
//    the next row is unconditional.
template <int V, bool NEST, bool ZOUT, bool DIV, bool MASKED>
__device__ __forceinline__ void one_peer_body(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, int n, size_t ld, size_t col0,
    long ncols, int h, int len, float p, Hyper hp)
{
    typedef typename vec_of<V>::type T;
    constexpr int C = kOpCols;
    const long cbase = (long)blockIdx.x * (kOpBlock * C) + threadIdx.x;
    size_t off[C];
    bool live[C];
#pragma unroll
    for (int j = 0; j < C; ++j) {
        long c = cbase + (long)j * kOpBlock;
        live[j] = !MASKED || c < ncols;
        off[j] = col0 + (size_t)(live[j] ? c : 0) * V;
    }
    if (MASKED && !live[0]) return;

    auto load_row = [&](RowRegs<V, NEST, C> &r, int node) {
        r.node = node;
        r.w = (ZOUT && DIV) ? w[node] : 1.0f;
        r.wo = hp.wd_mode == 2 ? hp.w_old[node] : 1.0f;
        const size_t row = (size_t)node * ld;
#pragma unroll
        for (int j = 0; j < C; ++j)
            if (live[j]) {
                r.x[j] = ld_stream<V>(x + row + off[j]);
                if (NEST) r.u[j] = ld_stream<V>(u + row + off[j]);
                r.g[j] = ld_stream<V>(g + row + off[j]);
            }
    };

    T first[C], prev[C], parked[C];
#pragma unroll
    for (int j = 0; j < C; ++j) first[j] = prev[j] = parked[j] = T(0);
    int first_node = 0, parked_node = 0;
    float first_w = 1.0f, parked_w = 1.0f;
    int ppos = 0;   // position of the node being processed within its cycle

    auto emit = [&](int node, float wi, const T (&xn)[C]) {
        const size_t row = (size_t)node * ld;
#pragma unroll
        for (int j = 0; j < C; ++j)
            if (live[j]) {
                st_stream<V>(x + row + off[j], xn[j]);
                if (ZOUT) st_stream<V>(z + row + off[j], debias_val<V, DIV>(xn[j], wi));
            }
    };

    // EMIT = false only for the very first row, which opens the first cycle with nothing parked.
    auto process_row = [&]<bool EMIT>(const RowRegs<V, NEST, C> &r) {
        const size_t row = (size_t)r.node * ld;
        const bool opens = (ppos == 0), closes = (ppos == len - 1);
        T xn[C];
#pragma unroll
        for (int j = 0; j < C; ++j) {
            T xh = T(0);
            if (live[j])
                xh = half_step<V, NEST>(r.x[j], NEST ? r.u[j] : r.x[j], r.g[j], hp,
                                        u + row + off[j], r.wo);
            if (opens) {
                xn[j] = parked[j];
                first[j] = xh;
            } else {
                T a0 = p * xh;
                T a1 = p * prev[j];
                xn[j] = a0 + a1;
            }
            prev[j] = xh;
        }
        const int out_node = opens ? parked_node : r.node;
        const float out_w = opens ? parked_w : r.w;
        if (opens) {
            first_node = r.node;
            first_w = r.w;
        }
        if (closes) {   // the first node of the cycle hears from the last one visited
#pragma unroll
            for (int j = 0; j < C; ++j) {
                T pk = p * first[j];
                if (len > 1) {
                    T a1 = p * prev[j];
                    pk = pk + a1;
                }
                parked[j] = pk;
            }
            parked_node = first_node;
            parked_w = first_w;
            ppos = 0;
        } else {
            ++ppos;
        }
        if (EMIT) emit(out_node, out_w, xn);
    };

    WalkPos lp{0, 0, 0};
    RowRegs<V, NEST, C> ra, rb;
    load_row(ra, lp.node);
    lp.advance(n, h, len);
    if (n > 1) {
        load_row(rb, lp.node);
        lp.advance(n, h, len);
    }
    process_row.template operator()<false>(ra);
    int t = 1;                      // rb holds row t (if t < n); later rows are not loaded yet
    for (; t + 2 < n; t += 2) {
        load_row(ra, lp.node);
        lp.advance(n, h, len);
        process_row.template operator()<true>(rb);
        load_row(rb, lp.node);
        lp.advance(n, h, len);
        process_row.template operator()<true>(ra);
    }
    if (t + 1 < n) {
        load_row(ra, lp.node);
        process_row.template operator()<true>(rb);
        process_row.template operator()<true>(ra);
    } else if (t < n) {
        process_row.template operator()<true>(rb);
    }
    emit(parked_node, parked_w, parked);
}

template <int V, bool NEST, bool ZOUT>
__global__ __launch_bounds__(kOpBlock) void k_step_one_peer(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, const int *__restrict__ unit_w, int n,
    size_t ld, size_t col0, long ncols, int h, int len, float p, Hyper hp)
{
    const bool full = ((long)blockIdx.x + 1) * (kOpBlock * kOpCols) <= ncols;
#define SGP_OP_CALL(DIV, MASKED) \
    one_peer_body<V, NEST, ZOUT, DIV, MASKED>(x, u, g, z, w, n, ld, col0, ncols, h, len, p, hp)
    if (ZOUT && *unit_w == 0) {
        if (full) SGP_OP_CALL(true, false);
        else SGP_OP_CALL(true, true);
    } else {
        if (full) SGP_OP_CALL(false, false);
        else SGP_OP_CALL(false, true);
    }
#undef SGP_OP_CALL
}

// ------------------------------------------------------------------------------------------
// Fused step, any number of out-peers: every xh of the work-item's coordinates is parked in a
// private LDS column (no barrier: a work-item only reads what it wrote), then each receiver sums
// its sources.  tab[i*S + q], q < S, lists node i's sources (itself included) in ascending index.
// ------------------------------------------------------------------------------------------
template <int V, bool NEST, bool ZOUT, bool DIV, bool WEIGHTED>
__device__ __forceinline__ void gather_body(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, int n, size_t ld, size_t col0,
    long ncols, const int *__restrict__ tab, const float *__restrict__ tabw, int S, float p,
    Hyper hp)
{
    typedef typename vec_of<V>::type T;
    extern __shared__ __align__(16) unsigned char smem[];
    T *stash = reinterpret_cast<T *>(smem) + threadIdx.x;   // node i lives at stash[i * kGatherBlock]
    long c = (long)blockIdx.x * kGatherBlock + threadIdx.x;
    if (c >= ncols) return;
    const size_t off = col0 + (size_t)c * V;

    for (int i0 = 0; i0 < n; i0 += kBatch) {
        T xv[kBatch], uv[kBatch], gv[kBatch];
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            if (i0 + q < n) {
                size_t a = (size_t)(i0 + q) * ld + off;
                xv[q] = ld_stream<V>(x + a);
                if (NEST) uv[q] = ld_stream<V>(u + a);
                gv[q] = ld_stream<V>(g + a);
            }
        }
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            if (i0 + q < n) {
                size_t a = (size_t)(i0 + q) * ld + off;
                stash[(i0 + q) * kGatherBlock] =
                    half_step<V, NEST>(xv[q], NEST ? uv[q] : xv[q], gv[q], hp, u + a,
                                       hp.wd_mode == 2 ? hp.w_old[i0 + q] : 1.0f);
            }
        }
    }
    for (int i = 0; i < n; ++i) {
        const int *src = tab + (size_t)i * S;
        T acc = T(0);
        if (!WEIGHTED) {
            acc = p * stash[src[0] * kGatherBlock];
            for (int q = 1; q < S; ++q) {
                T term = p * stash[src[q] * kGatherBlock];
                acc = acc + term;
            }
        } else {   // own weight per entry; entries < 0 are padding; the first term opens the sum
            const float *wq = tabw + (size_t)i * S;
            bool any = false;
            for (int q = 0; q < S; ++q) {
                const int j = src[q];
                if (j < 0) continue;
                T term = wq[q] * stash[j * kGatherBlock];
                acc = any ? acc + term : term;
                any = true;
            }
        }
        size_t a = (size_t)i * ld + off;
        st_stream<V>(x + a, acc);
        if (ZOUT) st_stream<V>(z + a, debias_val<V, DIV>(acc, DIV ? w[i] : 1.0f));
    }
}

template <int V, bool NEST, bool ZOUT, bool WEIGHTED>
__global__ __launch_bounds__(kGatherBlock) void k_step_gather(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, const int *__restrict__ unit_w, int n,
    size_t ld, size_t col0, long ncols, const int *__restrict__ tab, const float *__restrict__ tabw,
    int S, float p, Hyper hp)
{
    if (ZOUT && *unit_w == 0)
        gather_body<V, NEST, ZOUT, true, WEIGHTED>(x, u, g, z, w, n, ld, col0, ncols, tab, tabw, S, p,
                                                   hp);
    else
        gather_body<V, NEST, ZOUT, false, WEIGHTED>(x, u, g, z, w, n, ld, col0, ncols, tab, tabw, S, p,
                                                    hp);
}

// ------------------------------------------------------------------------------------------
// Fused step on the complete graph, every entry of P equal to 1/n (the setting in which SGP
// coincides with parallel SGD over AllReduce, section 3).  All receivers get the same sum
// sum_j fl(xh_j / n), ascending j, so a work-item adds it up once while it streams the rows
// (pass 1, pipelined like the one-peer walk) and then writes it to every node (pass 2).
// ------------------------------------------------------------------------------------------
template <int V, bool NEST, bool ZOUT, bool DIV, bool MASKED>
__device__ __forceinline__ void complete_body(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, int n, size_t ld, size_t col0,
    long ncols, float p, Hyper hp)
{
    typedef typename vec_of<V>::type T;
    const long c = (long)blockIdx.x * kOpBlock + threadIdx.x;
    if (MASKED && c >= ncols) return;
    const size_t off = col0 + (size_t)c * V;
    struct Row {
        T x, u, g;
    } ra, rb;
    auto load_row = [&](Row &r, int node) {
        const size_t a = (size_t)node * ld + off;
        r.x = ld_stream<V>(x + a);
        if (NEST) r.u = ld_stream<V>(u + a);
        r.g = ld_stream<V>(g + a);
    };
    T acc = T(0);
    auto process_row = [&](const Row &r, int node) {
        T xh = half_step<V, NEST>(r.x, NEST ? r.u : r.x, r.g, hp, u + (size_t)node * ld + off,
                                  hp.wd_mode == 2 ? hp.w_old[node] : 1.0f);
        T term = p * xh;
        acc = acc + term;
    };
    load_row(ra, 0);
    int t = 0;                      // ra holds row t; later rows are not loaded yet
    for (; t + 2 < n; t += 2) {
        load_row(rb, t + 1);
        process_row(ra, t);
        load_row(ra, t + 2);
        process_row(rb, t + 1);
    }
    if (t + 1 < n) {
        load_row(rb, t + 1);
        process_row(ra, t);
        process_row(rb, t + 1);
    } else {
        process_row(ra, t);
    }
    for (int i = 0; i < n; ++i) {
        const size_t a = (size_t)i * ld + off;
        st_stream<V>(x + a, acc);
        if (ZOUT) st_stream<V>(z + a, debias_val<V, DIV>(acc, DIV ? w[i] : 1.0f));
    }
}

template <int V, bool NEST, bool ZOUT>
__global__ __launch_bounds__(kOpBlock) void k_step_complete(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, const int *__restrict__ unit_w, int n,
    size_t ld, size_t col0, long ncols, float p, Hyper hp)
{
    const bool full = ((long)blockIdx.x + 1) * kOpBlock <= ncols;
#define SGP_COMPLETE_CALL(DIV, MASKED) \
    complete_body<V, NEST, ZOUT, DIV, MASKED>(x, u, g, z, w, n, ld, col0, ncols, p, hp)
    if (ZOUT && *unit_w == 0) {
        if (full) SGP_COMPLETE_CALL(true, false);
        else SGP_COMPLETE_CALL(true, true);
    } else {
        if (full) SGP_COMPLETE_CALL(false, false);
        else SGP_COMPLETE_CALL(false, true);
    }
#undef SGP_COMPLETE_CALL
}

// ------------------------------------------------------------------------------------------
// Fused step of 1-overlap SGP (Alg. 2, tau = 1).  Node i keeps its own share p*xh_i (which is
// also the message it sends: uniform weights), and then adds the messages that its in-neighbours
// of the PREVIOUS iteration sent, in ascending sender index.  msg_prev/msg_cur are [n][ld]
// buffers of pre-weighted messages p*xh_j.  tab_prev lists the previous iteration's sources of
// every node, sorted, the node itself included exactly once (skipped here); NULL when nothing
// has been sent yet.  There is no dependency between nodes inside an iteration, so the nodes are
// simply visited in order, software-pipelined like the one-peer walk.
// NM = messages per node known at compile time (0, 1, 2), or -1: read S at run time and fetch the
// messages while summing.
// ------------------------------------------------------------------------------------------
constexpr int kDelayBlock = SGP_DELAY_BLOCK;   // work-items per block
constexpr int kDelayCols = SGP_DELAY_COLS;     // 128-bit column groups per work-item

template <int V, bool NEST, int C, int M>
struct DelayRegs {
    typename vec_of<V>::type x[C], u[C], g[C], m[M > 0 ? M : 1][C];
    float w, wo;
    int node;
};

template <int V, bool NEST, bool ZOUT, int NM, bool DIV, bool MASKED>
__device__ __forceinline__ void delay_body(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, const float *__restrict__ msg_prev,
    float *__restrict__ msg_cur, int n, size_t ld, size_t col0, long ncols,
    const int *__restrict__ tab_prev, int S, float p, Hyper hp)
{
    typedef typename vec_of<V>::type T;
    constexpr int C = kDelayCols;
    constexpr int M = NM > 0 ? NM : 0;
    const long cbase = (long)blockIdx.x * (kDelayBlock * C) + threadIdx.x;
    size_t off[C];
    bool live[C];
#pragma unroll
    for (int j = 0; j < C; ++j) {
        long c = cbase + (long)j * kDelayBlock;
        live[j] = !MASKED || c < ncols;
        off[j] = col0 + (size_t)(live[j] ? c : 0) * V;
    }
    if (MASKED && !live[0]) return;

    auto load_row = [&](DelayRegs<V, NEST, C, M> &r, int node) {
        r.node = node;
        r.w = (ZOUT && DIV) ? w[node] : 1.0f;
        r.wo = hp.wd_mode == 2 ? hp.w_old[node] : 1.0f;
        const size_t row = (size_t)node * ld;
#pragma unroll
        for (int j = 0; j < C; ++j)
            if (live[j]) {
                r.x[j] = ld_stream<V>(x + row + off[j]);
                if (NEST) r.u[j] = ld_stream<V>(u + row + off[j]);
                r.g[j] = ld_stream<V>(g + row + off[j]);
            }
        if (M > 0) {
            // the sorted list holds `node` once, at position ps; message s is entry s + (s >= ps)
            const int *src = tab_prev + (size_t)node * (M + 1);
            int ps = 0;
#pragma unroll
            for (int e = 0; e < M + 1; ++e) ps += (src[e] < node) ? 1 : 0;
#pragma unroll
            for (int sidx = 0; sidx < M; ++sidx) {
                const int sender = src[sidx + (sidx >= ps ? 1 : 0)];
                const size_t mrow = (size_t)sender * ld;
#pragma unroll
                for (int j = 0; j < C; ++j)
                    if (live[j]) r.m[sidx][j] = ld_cached<V>(msg_prev + mrow + off[j]);
            }
        }
    };

    auto process_row = [&](const DelayRegs<V, NEST, C, M> &r) {
        const size_t row = (size_t)r.node * ld;
#pragma unroll
        for (int j = 0; j < C; ++j)
            if (live[j]) {
                const size_t a = row + off[j];
                T xh = half_step<V, NEST>(r.x[j], NEST ? r.u[j] : r.x[j], r.g[j], hp, u + a, r.wo);
                T own = p * xh;
                st_stream<V>(msg_cur + a, own);
                T acc = own;
                if (NM > 0) {
#pragma unroll
                    for (int sidx = 0; sidx < M; ++sidx) acc = acc + r.m[sidx][j];
                } else if (NM < 0) {
                    const int *src = tab_prev + (size_t)r.node * S;
                    for (int e = 0; e < S; ++e) {
                        const int sender = src[e];
                        if (sender != r.node)
                            acc = acc + ld_cached<V>(msg_prev + (size_t)sender * ld + off[j]);
                    }
                }
                st_stream<V>(x + a, acc);
                if (ZOUT) st_stream<V>(z + a, debias_val<V, DIV>(acc, r.w));
            }
    };

    DelayRegs<V, NEST, C, M> ra, rb;
    // every row issues the same memory operations, the prefetch inside the loop is unconditional
    // and full blocks carry no predicates: the compiler can then wait for exactly the loads it needs
    load_row(ra, 0);
    int t = 0;                      // ra holds row t; later rows are not loaded yet
    for (; t + 2 < n; t += 2) {
        load_row(rb, t + 1);
        process_row(ra);
        load_row(ra, t + 2);
        process_row(rb);
    }
    if (t + 1 < n) {
        load_row(rb, t + 1);
        process_row(ra);
        process_row(rb);
    } else {
        process_row(ra);
    }
}

template <int V, bool NEST, bool ZOUT, int NM>
__global__ __launch_bounds__(kDelayBlock) void k_step_delay(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, const int *__restrict__ unit_w,
    const float *__restrict__ msg_prev, float *__restrict__ msg_cur, int n, size_t ld, size_t col0,
    long ncols, const int *__restrict__ tab_prev, int S, float p, Hyper hp)
{
    const bool full = ((long)blockIdx.x + 1) * (kDelayBlock * kDelayCols) <= ncols;
#define SGP_DELAY_CALL(DIV, MASKED)                                                                   \
    delay_body<V, NEST, ZOUT, NM, DIV, MASKED>(x, u, g, z, w, msg_prev, msg_cur, n, ld, col0, ncols, \
                                               tab_prev, S, p, hp)
    if (ZOUT && *unit_w == 0) {
        if (full) SGP_DELAY_CALL(true, false);
        else SGP_DELAY_CALL(true, true);
    } else {
        if (full) SGP_DELAY_CALL(false, false);
        else SGP_DELAY_CALL(false, true);
    }
#undef SGP_DELAY_CALL
}

// ------------------------------------------------------------------------------------------
// Overlap step with exactly two messages per receiver (two out-peers): receiver i hears from
// ja = i - ha and jb = i - hb (mod n), the previous round's hops.  Walking the receivers with the
// stride hb - ha makes jb of one row equal to ja of the row before, so each message row is loaded
// once and handed on in registers, instead of being fetched by both of its receivers (the table
// driven kernel above fetched 2-24 % more than the algorithmic bytes, depending on how far apart
// in the ascending walk the two receivers of a message are).  The row that opens a cycle of the
// stride lacks its second message until the cycle closes; it is parked like the cycle-opening
// node of the one-peer walk, so that every row issues the same loads and stores.
// The sum keeps the order of the dense row: own share, then the two messages in ascending sender.
// ------------------------------------------------------------------------------------------
template <int V, bool NEST, bool ZOUT, bool DIV, bool MASKED>
__device__ __forceinline__ void delay2_body(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, const float *__restrict__ msg_prev,
    float *__restrict__ msg_cur, int n, size_t ld, size_t col0, long ncols, int ha, int hb,
    int stride, int len, float p, Hyper hp)
{
    typedef typename vec_of<V>::type T;
    constexpr int C = kDelayCols;
    const long cbase = (long)blockIdx.x * (kDelayBlock * C) + threadIdx.x;
    size_t off[C];
    bool live[C];
#pragma unroll
    for (int j = 0; j < C; ++j) {
        long c = cbase + (long)j * kDelayBlock;
        live[j] = !MASKED || c < ncols;
        off[j] = col0 + (size_t)(live[j] ? c : 0) * V;
    }
    if (MASKED && !live[0]) return;

    auto load_row = [&](DelayRegs<V, NEST, C, 1> &r, int node) {
        r.node = node;
        r.w = (ZOUT && DIV) ? w[node] : 1.0f;
        r.wo = hp.wd_mode == 2 ? hp.w_old[node] : 1.0f;
        const size_t row = (size_t)node * ld;
        int ja = node - ha;
        if (ja < 0) ja += n;
        const size_t mrow = (size_t)ja * ld;
#pragma unroll
        for (int j = 0; j < C; ++j)
            if (live[j]) {
                r.x[j] = ld_stream<V>(x + row + off[j]);
                if (NEST) r.u[j] = ld_stream<V>(u + row + off[j]);
                r.g[j] = ld_stream<V>(g + row + off[j]);
                r.m[0][j] = ld_stream<V>(msg_prev + mrow + off[j]);
            }
    };

    T prev_ma[C], first_own[C], first_ma[C], parked[C];
#pragma unroll
    for (int j = 0; j < C; ++j) prev_ma[j] = first_own[j] = first_ma[j] = parked[j] = T(0);
    int first_node = 0, parked_node = 0;
    float first_w = 1.0f, parked_w = 1.0f;
    int ppos = 0;

    auto emit = [&](int node, float wi, const T (&xn)[C]) {
        const size_t row = (size_t)node * ld;
#pragma unroll
        for (int j = 0; j < C; ++j)
            if (live[j]) {
                st_stream<V>(x + row + off[j], xn[j]);
                if (ZOUT) st_stream<V>(z + row + off[j], debias_val<V, DIV>(xn[j], wi));
            }
    };
    // own + the two messages, lower sender index first; sender of ma is node - ha, of mb node - hb
    auto total = [&](int node, T own, T ma, T mb) {
        int ja = node - ha, jb = node - hb;
        if (ja < 0) ja += n;
        if (jb < 0) jb += n;
        const bool a_first = ja < jb;
        T s1 = own + (a_first ? ma : mb);
        return s1 + (a_first ? mb : ma);
    };

    auto process_row = [&]<bool EMIT>(const DelayRegs<V, NEST, C, 1> &r) {
        const size_t row = (size_t)r.node * ld;
        const bool opens = (ppos == 0), closes = (ppos == len - 1);
        T xn[C];
#pragma unroll
        for (int j = 0; j < C; ++j) {
            T own = T(0);
            if (live[j]) {
                T xh = half_step<V, NEST>(r.x[j], NEST ? r.u[j] : r.x[j], r.g[j], hp, u + row + off[j], r.wo);
                own = p * xh;
                st_stream<V>(msg_cur + row + off[j], own);
            }
            if (opens) {
                xn[j] = parked[j];
                first_own[j] = own;
                first_ma[j] = r.m[0][j];
            } else {
                xn[j] = total(r.node, own, r.m[0][j], prev_ma[j]);
            }
            prev_ma[j] = r.m[0][j];
        }
        const int out_node = opens ? parked_node : r.node;
        const float out_w = opens ? parked_w : r.w;
        if (opens) {
            first_node = r.node;
            first_w = r.w;
        }
        if (closes) {   // the opening row's second message is this row's first one
#pragma unroll
            for (int j = 0; j < C; ++j) parked[j] = total(first_node, first_own[j], first_ma[j], prev_ma[j]);
            parked_node = first_node;
            parked_w = first_w;
            ppos = 0;
        } else {
            ++ppos;
        }
        if (EMIT) emit(out_node, out_w, xn);
    };

    WalkPos lp{0, 0, 0};
    DelayRegs<V, NEST, C, 1> ra, rb;
    load_row(ra, lp.node);
    lp.advance(n, stride, len);
    load_row(rb, lp.node);          // n >= 3 here: two distinct peers
    lp.advance(n, stride, len);
    process_row.template operator()<false>(ra);
    int t = 1;                      // rb holds row t; later rows are not loaded yet
    for (; t + 2 < n; t += 2) {
        load_row(ra, lp.node);
        lp.advance(n, stride, len);
        process_row.template operator()<true>(rb);
        load_row(rb, lp.node);
        lp.advance(n, stride, len);
        process_row.template operator()<true>(ra);
    }
    if (t + 1 < n) {
        load_row(ra, lp.node);
        process_row.template operator()<true>(rb);
        process_row.template operator()<true>(ra);
    } else {
        process_row.template operator()<true>(rb);
    }
    emit(parked_node, parked_w, parked);
}

template <int V, bool NEST, bool ZOUT>
__global__ __launch_bounds__(kDelayBlock) void k_step_delay2(
    float *__restrict__ x, float *__restrict__ u, const float *__restrict__ g,
    float *__restrict__ z, const float *__restrict__ w, const int *__restrict__ unit_w,
    const float *__restrict__ msg_prev, float *__restrict__ msg_cur, int n, size_t ld, size_t col0,
    long ncols, int ha, int hb, int stride, int len, float p, Hyper hp)
{
    const bool full = ((long)blockIdx.x + 1) * (kDelayBlock * kDelayCols) <= ncols;
#define SGP_DELAY2_CALL(DIV, MASKED)                                                                  \
    delay2_body<V, NEST, ZOUT, DIV, MASKED>(x, u, g, z, w, msg_prev, msg_cur, n, ld, col0, ncols, ha, \
                                            hb, stride, len, p, hp)
    if (ZOUT && *unit_w == 0) {
        if (full) SGP_DELAY2_CALL(true, false);
        else SGP_DELAY2_CALL(true, true);
    } else {
        if (full) SGP_DELAY2_CALL(false, false);
        else SGP_DELAY2_CALL(false, true);
    }
#undef SGP_DELAY2_CALL
}

// Push-sum weights, blocking form (Alg. 1 line 7): w_i <- sum over sources, ascending, of p*w_j.
// One block; every work-item reads before anyone writes.
__global__ void k_w_mix(float *w, int n, const int *__restrict__ tab, int S, float p,
                        int *__restrict__ unit_w, int biased, float *__restrict__ w_old)
{
    int i = threadIdx.x;
    float acc = 0.0f;
    if (i < n) {
        w_old[i] = w[i];
        const int *src = tab + (size_t)i * S;
        acc = p * w[src[0]];
        for (int q = 1; q < S; ++q) {
            float term = p * w[src[q]];
            acc = acc + term;
        }
    }
    const int all_one = __syncthreads_and(i >= n || acc == 1.0f);
    if (i < n) w[i] = acc;
    if (i == 0) *unit_w = all_one | biased;   // biased ablation: z = x, never divide
}

// Complete graph: every node ends with the same weight sum_j fl(p * w_j), ascending j.
__global__ void k_w_complete(float *w, int n, float p, int *__restrict__ unit_w, int biased,
                             float *__restrict__ w_old)
{
    int i = threadIdx.x;
    float acc = 0.0f;
    if (i < n) {
        w_old[i] = w[i];
        for (int j = 0; j < n; ++j) {
            float term = p * w[j];
            acc = acc + term;
        }
    }
    const int all_one = __syncthreads_and(i >= n || acc == 1.0f);
    if (i < n) w[i] = acc;
    if (i == 0) *unit_w = all_one | biased;
}

// Caller-supplied sparse rows: w_i <- sum over the row's entries, in the order given, of weight * w_j.
__global__ void k_w_custom(float *w, int n, const int *__restrict__ tab, const float *__restrict__ tabw,
                           int S, int *__restrict__ unit_w, int biased, float *__restrict__ w_old)
{
    int i = threadIdx.x;
    float acc = 0.0f;
    if (i < n) {
        w_old[i] = w[i];
        bool any = false;
        for (int q = 0; q < S; ++q) {
            const int j = tab[(size_t)i * S + q];
            if (j < 0) continue;
            float term = tabw[(size_t)i * S + q] * w[j];
            acc = any ? acc + term : term;
            any = true;
        }
    }
    const int all_one = __syncthreads_and(i >= n || acc == 1.0f);
    if (i < n) w[i] = acc;
    if (i == 0) *unit_w = all_one | biased;
}

// Iteration without communication: the weights stay, only the flag is refreshed.
__global__ void k_w_keep(const float *__restrict__ w, int n, int *__restrict__ unit_w, int biased,
                         float *__restrict__ w_old)
{
    int i = threadIdx.x;
    if (i < n) w_old[i] = w[i];
    const int all_one = __syncthreads_and(i >= n || w[i] == 1.0f);
    if (i == 0) *unit_w = all_one | biased;
}

// Push-sum weights under one iteration of delay: own share now, the previous iteration's
// messages (pre-weighted p*w_j) in ascending sender index; the share is also the new message.
__global__ void k_w_delay(float *w, const float *__restrict__ msgw_prev, float *__restrict__ msgw_cur,
                          int n, const int *__restrict__ tab_prev, int S, float p,
                          int *__restrict__ unit_w, int biased, float *__restrict__ w_old)
{
    int i = threadIdx.x;
    float own = 0.0f, acc = 0.0f;
    if (i < n) {
        w_old[i] = w[i];
        own = p * w[i];
        acc = own;
        if (tab_prev) {
            const int *src = tab_prev + (size_t)i * S;
            for (int q = 0; q < S; ++q) {
                int j = src[q];
                if (j != i) acc = acc + msgw_prev[j];
            }
        }
    }
    const int all_one = __syncthreads_and(i >= n || acc == 1.0f);
    if (i < n) {
        w[i] = acc;
        msgw_cur[i] = own;
    }
    if (i == 0) *unit_w = all_one | biased;   // biased ablation: z = x, never divide
}

// z = x / w (Alg. 1 line 8) as a stand-alone pass; blockIdx.y = node.
template <int V>
__global__ __launch_bounds__(kBlock) void k_debias(const float *__restrict__ x,
                                                  const float *__restrict__ w,
                                                  float *__restrict__ z, size_t ld, size_t col0,
                                                  long ncols)
{
    long c = (long)blockIdx.x * kBlock + threadIdx.x;
    if (c >= ncols) return;
    int i = blockIdx.y;
    size_t a = (size_t)i * ld + col0 + (size_t)c * V;
    const float wi = w[i];
    typename vec_of<V>::type xv = ld_stream<V>(x + a);
    st_stream<V>(z + a, wi == 1.0f ? xv : xv / wi);
}

// ------------------------------------------------------------------------------------------
// Consensus statistics: per node sum_e (z_i[e] - zbar[e])^2 with zbar the node-wise average.
// |z_i - zbar| is typically orders of magnitude below |z_i|, so the differences are formed
// against a reference row first: a_i = z_i - z_0 (exact or nearly so), abar = mean_i a_i, and the
// squared terms are (a_i - abar)^2; every rounding error is then relative to the deviation
// itself.  Partial sums: float per work-item and block, double from there on.
// partial is [(n+1)][G]; row n carries sum_e zbar[e]^2.
// ------------------------------------------------------------------------------------------
constexpr int kStatsCache = 32;   // nodes whose z the small-n kernel keeps in registers

#include "step_stats_kernel.inc"

template <int V>
__global__ __launch_bounds__(kBlock) void k_stats_small(const float *__restrict__ z, int n,
                                                       size_t ld, size_t col0, long ncols,
                                                       long ntiles, float *__restrict__ partial,
                                                       int G, int accumulate)
{
    typedef typename vec_of<V>::type T;
    float acc[kStatsCache + 1];
#pragma unroll
    for (int i = 0; i <= kStatsCache; ++i) acc[i] = 0.0f;
    const float inv_n = 1.0f / (float)n;

    for (long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        long c = tile * kBlock + threadIdx.x;
        if (c < ncols) {
            const size_t off = col0 + (size_t)c * V;
            T a[kStatsCache];
#pragma unroll
            for (int i = 0; i < kStatsCache; ++i)
                if (i < n) a[i] = ld_stream<V>(z + (size_t)i * ld + off);
            T ref = a[0];
            T asum = T(0);
#pragma unroll
            for (int i = 0; i < kStatsCache; ++i)
                if (i < n) {
                    a[i] = a[i] - ref;
                    asum = asum + a[i];
                }
            T abar = asum * inv_n;
#pragma unroll
            for (int i = 0; i < kStatsCache; ++i)
                if (i < n) {
                    T t = a[i] - abar;
                    acc[i] += hsum(t * t);
                }
            T zb = ref + abar;
            acc[kStatsCache] += hsum(zb * zb);
        }
    }

    __shared__ float red[kBlock / 64][kStatsCache + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i <= kStatsCache; ++i) {
        if (i < n || i == kStatsCache) {
            float v = wave_sum(acc[i]);
            if (lane == 0) red[wave][i] = v;
        }
    }
    __syncthreads();
    int i = threadIdx.x;
    if (i <= kStatsCache && (i < n || i == kStatsCache)) {
        float v = (red[0][i] + red[1][i]) + (red[2][i] + red[3][i]);
        size_t row = (i == kStatsCache) ? (size_t)n : (size_t)i;
        float *dst = partial + row * G + blockIdx.x;
        *dst = accumulate ? *dst + v : v;
    }
}

// Any n: two sweeps over the nodes (average first, then squared differences, re-reading z).
template <int V>
__global__ __launch_bounds__(kBlock) void k_stats_large(const float *__restrict__ z, int n,
                                                       size_t ld, size_t col0, long ncols,
                                                       long ntiles, float *__restrict__ partial,
                                                       int G, int accumulate)
{
    typedef typename vec_of<V>::type T;
    extern __shared__ __align__(16) unsigned char smem[];
    float *red = reinterpret_cast<float *>(smem);          // [kBlock/64][n+1]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < (kBlock / 64) * (n + 1); i += kBlock) red[i] = 0.0f;
    __syncthreads();
    const float inv_n = 1.0f / (float)n;

    for (long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        long c = tile * kBlock + threadIdx.x;
        const bool active = c < ncols;
        const size_t off = col0 + (size_t)(active ? c : 0) * V;
        T ref = ld_cached<V>(z + off);
        T asum = T(0);
        for (int i = 1; i < n; ++i) {
            T ai = ld_cached<V>(z + (size_t)i * ld + off) - ref;
            asum = asum + ai;
        }
        T abar = asum * inv_n;
        for (int i = 0; i < n; ++i) {
            T ai = ld_cached<V>(z + (size_t)i * ld + off) - ref;
            T t = ai - abar;
            float v = wave_sum(active ? hsum(t * t) : 0.0f);
            if (lane == 0) red[wave * (n + 1) + i] += v;
        }
        T zb = ref + abar;
        float v = wave_sum(active ? hsum(zb * zb) : 0.0f);
        if (lane == 0) red[wave * (n + 1) + n] += v;
    }
    __syncthreads();
    for (int i = threadIdx.x; i <= n; i += kBlock) {
        float v = 0.0f;
        for (int wv = 0; wv < kBlock / 64; ++wv) v += red[wv * (n + 1) + i];
        float *dst = partial + (size_t)i * G + blockIdx.x;
        *dst = accumulate ? *dst + v : v;
    }
}

// Final reduction, step 1: block r adds up row r of the partial table in double.
constexpr int kRowSumBlock = 1024;
__global__ __launch_bounds__(kRowSumBlock) void k_stats_rowsum(const float *__restrict__ partial, int G,
                                                              double *__restrict__ sums)
{
    const float *row = partial + (size_t)blockIdx.x * G;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;   // independent chains: loads overlap
    int b = threadIdx.x;
    for (; b + 3 * kRowSumBlock < G; b += 4 * kRowSumBlock) {
        const float v0 = row[b], v1 = row[b + kRowSumBlock], v2 = row[b + 2 * kRowSumBlock],
                    v3 = row[b + 3 * kRowSumBlock];
        s0 += (double)v0; s1 += (double)v1; s2 += (double)v2; s3 += (double)v3;
    }
    for (; b < G; b += kRowSumBlock) s0 += (double)row[b];
    double s = wave_sum((s0 + s1) + (s2 + s3));
    __shared__ double red[kRowSumBlock / 64];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot = 0.0;
        for (int i = 0; i < kRowSumBlock / 64; ++i) tot += red[i];
        sums[blockIdx.x] = tot;
    }
}

// Step 2: out[0..6] = max, mean, min, sum w, ||zbar||, argmax, argmin; out[8+i] = dist_i.
__device__ __forceinline__ void stats_final_body(const double *sums, int n, const float *__restrict__ w,
                                                 double *__restrict__ out)
{
    __shared__ double dist[SGP_MAX_NODES];
    __shared__ float wgt[SGP_MAX_NODES];
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        const double di = sqrt(sums[i]);
        dist[i] = di;
        wgt[i] = w[i];
        out[8 + i] = di;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double dmax = 0.0, dmin = 0.0, dsum = 0.0, wsum = 0.0;
        int amax = 0, amin = 0;
        for (int i = 0; i < n; ++i) {
            const double di = dist[i];
            if (i == 0 || di > dmax) { dmax = di; amax = i; }
            if (i == 0 || di < dmin) { dmin = di; amin = i; }
            dsum += di;
            wsum += (double)wgt[i];
        }
        out[0] = dmax;
        out[1] = dsum / (double)n;
        out[2] = dmin;
        out[3] = wsum;
        out[4] = sqrt(sums[n]);
        out[5] = (double)amax;
        out[6] = (double)amin;
        out[7] = 0.0;
    }
}

__global__ void k_stats_final(const double *__restrict__ sums, int n, const float *__restrict__ w,
                              double *__restrict__ out)
{
    stats_final_body(sums, n, w, out);
}

// Step 2 after the fused kernel: adds the B block sums of k_stats_slotsum in block order and moves
// every slot's sum to the node that the walk emitted into that slot.
constexpr int kFinalSlotsBlock = 256;
__global__ __launch_bounds__(kFinalSlotsBlock) void k_stats_final_slots(
    const double *__restrict__ sums2, int B, int n, int hop, int len, const float *__restrict__ w,
    double *__restrict__ out)
{
    __shared__ double all[kSlotSumBlocks * (kStatsCache + 1)];
    __shared__ double sums[kStatsCache + 1];
    for (int i = threadIdx.x; i < B * (kStatsCache + 1); i += kFinalSlotsBlock) all[i] = sums2[i];
    __syncthreads();
    const int s = threadIdx.x;
    if (s < n || s == kStatsCache) {
        double tot = 0.0;
        for (int b = 0; b < B; ++b) tot += all[b * (kStatsCache + 1) + s];
        sums[s == kStatsCache ? n : stats_slot_node(s, n, hop, len)] = tot;
    }
    __syncthreads();
    stats_final_body(sums, n, w, out);
}

__global__ __launch_bounds__(kBlock) void k_copy(floatx4 *__restrict__ dst,
                                                const floatx4 *__restrict__ src, size_t count)
{
    size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < count) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Handle
// ------------------------------------------------------------------------------------------
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
    bool tab_stale;     // topology or peer count changed: rebuild d_tab before the next step
    int cS;             // caller-supplied mixing rows (SGP_TOPO_CUSTOM): entries per row, 0 = not set
    int *d_cidx;        // [n][cS] senders, -1 = padding
    float *d_cw;        // [n][cS] weights
    int *d_unit_w;      // 1 if every push-sum weight equals 1 after the latest weight update
    float *d_w_old;     // [n] the weights before the latest update (weight decay on x / w)
    float wd;           // weight decay coefficient, 0 = off
    bool wd_on_x;       // decay acts on the numerator instead of the de-biased parameters
    float *d_partial;   // [(n+1)][G] partial sums of the statistics
    float *d_partial_f; // [(n+1)][Gf] partial sums written by the fused step+statistics kernel
    size_t partial_f_elems;
    int G;
    double *d_sums;     // [n+1] per-node sums of squares (+ the average's), or the fused kernel's
                        // [kSlotSumBlocks][33] block sums
    double *d_result;   // [8 + n]
    double *h_result;   // pinned mirror
    float *d_msg[2];    // overlap mode: pre-weighted messages p*xh_j, [n][ld] each
    bool msg_external;  // d_msg points into caller-owned memory
    float *d_msgw[2];   // overlap mode: pre-weighted weights p*w_j, [n] each
    int cur;            // buffer that the NEXT step writes
    bool have_msgs;
    int64_t last_k;
    int last_hip;

    bool timing;                          // bracket the step kernel with events
    hipEvent_t ev[SGP_TIMING_RING][2];
    bool ev_made;
    int64_t ev_head;                      // timed steps recorded so far
    int64_t ev_read;                      // timed steps already reported
};

namespace {

constexpr int kStatsGridMax = 2048;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

int hip_fail(sgp_handle *h, hipError_t e)
{
    if (h) h->last_hip = (int)e;
    return SGP_ERR_HIP;
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
int upload_tables(sgp_handle *h)
{
    if (h->d_tab) {
        (void)hipFree(h->d_tab);   // waits for the kernels that still read it
        h->d_tab = nullptr;
    }
    const int n = h->n, S = h->S, tables = h->L > 0 ? h->L : 1;
    size_t tab_elems = (size_t)tables * n * S;
    int *host_tab = static_cast<int *>(std::malloc(tab_elems * sizeof(int)));
    if (!host_tab) return SGP_ERR_NOMEM;
    build_tables(h, host_tab);
    hipError_t e = hipMalloc(&h->d_tab, tab_elems * sizeof(int));
    if (e == hipSuccess)
        e = hipMemcpy(h->d_tab, host_tab, tab_elems * sizeof(int), hipMemcpyHostToDevice);
    std::free(host_tab);
    if (e != hipSuccess) return e == hipErrorOutOfMemory ? SGP_ERR_NOMEM : hip_fail(h, e);
    h->tab_stale = false;
    return SGP_OK;
}

int ensure_device(sgp_handle *h)
{
    if (h->dev_ready) return h->tab_stale ? upload_tables(h) : SGP_OK;
    const int n = h->n;
    int rc = upload_tables(h);
    if (rc != SGP_OK) return rc;
    hipError_t e;

    h->G = kStatsGridMax;
    e = hipMalloc(&h->d_unit_w, sizeof(int));
    if (e == hipSuccess) e = hipMalloc(&h->d_w_old, (size_t)n * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(&h->d_partial, (size_t)(n + 1) * h->G * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(&h->d_sums,
                                       (size_t)std::max(n + 1, kSlotSumBlocks * (kStatsCache + 1)) * sizeof(double));
    if (e == hipSuccess) e = hipMalloc(&h->d_result, (size_t)(8 + n) * sizeof(double));
    if (e == hipSuccess)
        e = hipHostMalloc(reinterpret_cast<void **>(&h->h_result), (size_t)(8 + n) * sizeof(double),
                          hipHostMallocDefault);
    if (e == hipSuccess && h->delay) {
        size_t bytes = (size_t)n * (size_t)h->ld * sizeof(float);
        for (int b = 0; b < 2 && e == hipSuccess; ++b) {
            if (!h->msg_external) e = hipMalloc(&h->d_msg[b], bytes);
            if (e == hipSuccess) e = hipMalloc(&h->d_msgw[b], (size_t)n * sizeof(float));
        }
    }
    if (e != hipSuccess) return e == hipErrorOutOfMemory ? SGP_ERR_NOMEM : hip_fail(h, e);
    h->dev_ready = true;
    return SGP_OK;
}

void release_device(sgp_handle *h)
{
    if (h->ev_made)
        for (int i = 0; i < SGP_TIMING_RING; ++i) {
            (void)hipEventDestroy(h->ev[i][0]);
            (void)hipEventDestroy(h->ev[i][1]);
        }
    if (h->d_tab) (void)hipFree(h->d_tab);
    if (h->d_cidx) (void)hipFree(h->d_cidx);
    if (h->d_cw) (void)hipFree(h->d_cw);
    if (h->d_unit_w) (void)hipFree(h->d_unit_w);
    if (h->d_w_old) (void)hipFree(h->d_w_old);
    if (h->d_partial) (void)hipFree(h->d_partial);
    if (h->d_partial_f) (void)hipFree(h->d_partial_f);
    if (h->d_sums) (void)hipFree(h->d_sums);
    if (h->d_result) (void)hipFree(h->d_result);
    if (h->h_result) (void)hipHostFree(h->h_result);
    for (int b = 0; b < 2; ++b) {
        if (h->d_msg[b] && !h->msg_external) (void)hipFree(h->d_msg[b]);
        if (h->d_msgw[b]) (void)hipFree(h->d_msgw[b]);
    }
}

unsigned grid_for(long ncols, int block) { return (unsigned)((ncols + block - 1) / block); }

struct StepArgs {
    float *x, *u, *z;
    const float *g, *w;
    const int *unit_w;
    int n;
    size_t ld;
    float p;
    Hyper hp;
    hipStream_t stream;
};

template <int V, bool NEST, bool ZOUT>
void launch_one_peer(const StepArgs &a, size_t col0, long ncols, int h, int len)
{
    hipLaunchKernelGGL((k_step_one_peer<V, NEST, ZOUT>), dim3(grid_for(ncols, kOpBlock * kOpCols)),
                       dim3(kOpBlock), SGP_OP_DYNLDS,
                       a.stream, a.x, a.u, a.g, a.z, a.w, a.unit_w, a.n, a.ld, col0, ncols, h,
                       len, a.p, a.hp);
}

template <int V, bool NEST, bool ZOUT>
void launch_gather(const StepArgs &a, size_t col0, long ncols, const int *tab, const float *tabw, int S)
{
    size_t lds = (size_t)a.n * kGatherBlock * V * sizeof(float);
    dim3 grid(grid_for(ncols, kGatherBlock)), block(kGatherBlock);
    if (tabw)
        hipLaunchKernelGGL((k_step_gather<V, NEST, ZOUT, true>), grid, block, lds, a.stream, a.x, a.u, a.g,
                           a.z, a.w, a.unit_w, a.n, a.ld, col0, ncols, tab, tabw, S, a.p, a.hp);
    else
        hipLaunchKernelGGL((k_step_gather<V, NEST, ZOUT, false>), grid, block, lds, a.stream, a.x, a.u, a.g,
                           a.z, a.w, a.unit_w, a.n, a.ld, col0, ncols, tab, tabw, S, a.p, a.hp);
}

template <int V, bool NEST, bool ZOUT>
void launch_complete(const StepArgs &a, size_t col0, long ncols)
{
    hipLaunchKernelGGL((k_step_complete<V, NEST, ZOUT>), dim3(grid_for(ncols, kOpBlock)), dim3(kOpBlock),
                       0, a.stream, a.x, a.u, a.g, a.z, a.w, a.unit_w, a.n, a.ld, col0, ncols, a.p,
                       a.hp);
}

template <int V, bool NEST, bool ZOUT>
void launch_delay(const StepArgs &a, size_t col0, long ncols, const float *msg_prev, float *msg_cur,
                  const int *tab_prev, int S, int ha, int hb)
{
    dim3 grid(grid_for(ncols, kDelayBlock * kDelayCols)), block(kDelayBlock);
    const int nm = tab_prev ? S - 1 : 0;
    if (nm == 2 && SGP_DELAY_WINDOW) {   // two messages: each message row is loaded once
        const int stride = ((hb - ha) % a.n + a.n) % a.n;
        const int len = a.n / gcd_int(a.n, stride);
        hipLaunchKernelGGL((k_step_delay2<V, NEST, ZOUT>), grid, block, 0, a.stream, a.x, a.u, a.g, a.z,
                           a.w, a.unit_w, msg_prev, msg_cur, a.n, a.ld, col0, ncols, ha, hb, stride, len,
                           a.p, a.hp);
        return;
    }
    if (nm == 0)
        hipLaunchKernelGGL((k_step_delay<V, NEST, ZOUT, 0>), grid, block, 0, a.stream, a.x, a.u, a.g,
                           a.z, a.w, a.unit_w, msg_prev, msg_cur, a.n, a.ld, col0, ncols, tab_prev, S,
                           a.p, a.hp);
    else if (nm == 1)
        hipLaunchKernelGGL((k_step_delay<V, NEST, ZOUT, 1>), grid, block, 0, a.stream, a.x, a.u, a.g,
                           a.z, a.w, a.unit_w, msg_prev, msg_cur, a.n, a.ld, col0, ncols, tab_prev, S,
                           a.p, a.hp);
    else if (nm == 2)
        hipLaunchKernelGGL((k_step_delay<V, NEST, ZOUT, 2>), grid, block, 0, a.stream, a.x, a.u, a.g,
                           a.z, a.w, a.unit_w, msg_prev, msg_cur, a.n, a.ld, col0, ncols, tab_prev, S,
                           a.p, a.hp);
    else
        hipLaunchKernelGGL((k_step_delay<V, NEST, ZOUT, -1>), grid, block, 0, a.stream, a.x, a.u, a.g,
                           a.z, a.w, a.unit_w, msg_prev, msg_cur, a.n, a.ld, col0, ncols, tab_prev, S,
                           a.p, a.hp);
}

// Calls f.template operator()<NEST, ZOUT>() for the run-time pair of flags.
template <typename F>
void dispatch_flags(bool nest, bool zout, F &&f)
{
    if (nest) {
        if (zout) f.template operator()<true, true>();
        else f.template operator()<true, false>();
    } else {
        if (zout) f.template operator()<false, true>();
        else f.template operator()<false, false>();
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
    *out = h;
    return SGP_OK;
}

int sgp_destroy(sgp_handle *h)
{
    if (!h) return SGP_OK;
    int rc = SGP_OK;
    if (h->dev_ready) {
        hipError_t e = hipDeviceSynchronize();
        if (e != hipSuccess) rc = SGP_ERR_HIP;
        release_device(h);
    }
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
    h->topology = topology;
    h->peers = peers;
    Schedule s = make_schedule(h->n, peers, 0);
    h->L = s.L;
    h->distinct = s.distinct;
    h->S = s.distinct + 1;
    h->tab_stale = true;
    return SGP_OK;
}

int sgp_set_mixing(sgp_handle *h, const int32_t *in_idx, const float *in_weight, int32_t entries)
{
    if (!h || !in_idx || !in_weight || entries < 1 || entries > h->n) return SGP_ERR_INVALID_ARG;
    const size_t cnt = (size_t)h->n * entries;
    for (size_t q = 0; q < cnt; ++q)
        if (in_idx[q] < -1 || in_idx[q] >= h->n) return SGP_ERR_INVALID_ARG;
    if (h->d_cidx) {   // hipFree waits for the kernels that still read the old rows
        (void)hipFree(h->d_cidx);
        h->d_cidx = nullptr;
    }
    if (h->d_cw) {
        (void)hipFree(h->d_cw);
        h->d_cw = nullptr;
    }
    h->cS = 0;
    hipError_t e = hipMalloc(&h->d_cidx, cnt * sizeof(int));
    if (e == hipSuccess) e = hipMalloc(&h->d_cw, cnt * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(h->d_cidx, in_idx, cnt * sizeof(int), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(h->d_cw, in_weight, cnt * sizeof(float), hipMemcpyHostToDevice);
    if (e != hipSuccess) return e == hipErrorOutOfMemory ? SGP_ERR_NOMEM : hip_fail(h, e);
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
    if (h->dev_ready) return SGP_ERR_SEQUENCE;
    h->d_msg[0] = buf0;
    h->d_msg[1] = buf1;
    h->msg_external = true;
    h->have_msgs = false;
    h->last_k = -1;
    return SGP_OK;
}

int sgp_last_hip_error(const sgp_handle *h) { return h ? h->last_hip : 0; }

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
// table (G blocks) in h->d_partial_f for a walk with this hop and cycle length.
struct FusedStats {
    int G = 0, hop = 0, len = 1;
};

// One iteration; with fused != NULL the caller wants the statistics of z^(k+1) as well: when the
// fused kernel applies, it is used and *fused describes the partial table it left in
// h->d_partial_f, otherwise fused->G stays 0 and the caller runs the stand-alone statistics pass.
static int step_impl(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out,
                     float gamma, float momentum, int64_t k, void *stream, FusedStats *fused)
{
    if (!h || !x || !w || !g || k < 0) return SGP_ERR_INVALID_ARG;
    const bool nest = momentum != 0.0f;
    if (nest && !m) return SGP_ERR_INVALID_ARG;
    if (!aligned4(x) || !aligned4(w) || !aligned4(g) || (nest && !aligned4(m)) ||
        (z_out && !aligned4(z_out)))
        return SGP_ERR_ALIGNMENT;
    if (z_out && (z_out == x || z_out == g || (nest && z_out == m))) return SGP_ERR_INVALID_ARG;
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
    const bool gather = custom || (h->delay == 0 && !complete && s.distinct > 1);
    if (gather && n > 256) return SGP_ERR_UNSUPPORTED;

    int rc = ensure_device(h);
    if (rc != SGP_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);

    bool vec = (h->ld % 4 == 0) && aligned16(x) && aligned16(g) && (!nest || aligned16(m)) &&
               (!z_out || aligned16(z_out));
    if (gather && n > 64) vec = false;   // keep the LDS stash within 64 KiB
    const long cols4 = vec ? (long)(h->d / 4) : 0;             // full 128-bit groups
    const size_t tail0 = (size_t)cols4 * 4;
    const long tail = (long)(h->d - (int64_t)tail0);           // scalar columns after them

    const bool decay = h->wd != 0.0f;
    const Hyper hp{gamma, momentum, h->wd, !decay ? 0 : (h->wd_on_x || h->biased) ? 1 : 2, h->d_w_old};
    StepArgs a{x, m, z_out, g, w, h->d_unit_w, n, (size_t)h->ld, s.p, hp, st};
    const int *tab_k = h->d_tab + (size_t)kmod * n * S;
    const unsigned wblock = (unsigned)((n + 63) / 64 * 64);

    hipEvent_t *tev = nullptr;
    if (h->timing) {
        if (!h->ev_made) {
            for (int i = 0; i < SGP_TIMING_RING; ++i) {
                SGP_HIP_TRY(h, hipEventCreate(&h->ev[i][0]));
                SGP_HIP_TRY(h, hipEventCreate(&h->ev[i][1]));
            }
            h->ev_made = true;
        }
        tev = h->ev[h->ev_head % SGP_TIMING_RING];
    }

    if (!sending) {
        // between two communication rounds: a local step, x <- xh, w unchanged (Alg. 2, else branch
        // of the send test), which is the one-peer walk with n cycles of length 1 and weight 1
        hipLaunchKernelGGL(k_w_keep, dim3(1), dim3(wblock), 0, st, w, n, h->d_unit_w, (int)h->biased, h->d_w_old);
        if (tev) SGP_HIP_TRY(h, hipEventRecord(tev[0], st));
        StepArgs al = a;
        al.p = 1.0f;
        dispatch_flags(nest, z_out != nullptr, [&]<bool NEST, bool ZOUT>() {
            if (cols4 > 0) launch_one_peer<4, NEST, ZOUT>(al, 0, cols4, 0, 1);
            if (tail > 0) launch_one_peer<1, NEST, ZOUT>(al, tail0, tail, 0, 1);
        });
        h->last_k = k;
    } else if (complete) {
        StepArgs ac = a;
        ac.p = 1.0f / (float)n;
        hipLaunchKernelGGL(k_w_complete, dim3(1), dim3(wblock), 0, st, w, n, ac.p, h->d_unit_w,
                           (int)h->biased, h->d_w_old);
        if (tev) SGP_HIP_TRY(h, hipEventRecord(tev[0], st));
        dispatch_flags(nest, z_out != nullptr, [&]<bool NEST, bool ZOUT>() {
            if (cols4 > 0) launch_complete<4, NEST, ZOUT>(ac, 0, cols4);
            if (tail > 0) launch_complete<1, NEST, ZOUT>(ac, tail0, tail);
        });
    } else if (custom) {
        hipLaunchKernelGGL(k_w_custom, dim3(1), dim3(wblock), 0, st, w, n, h->d_cidx, h->d_cw, h->cS,
                           h->d_unit_w, (int)h->biased, h->d_w_old);
        if (tev) SGP_HIP_TRY(h, hipEventRecord(tev[0], st));
        dispatch_flags(nest, z_out != nullptr, [&]<bool NEST, bool ZOUT>() {
            if (cols4 > 0) launch_gather<4, NEST, ZOUT>(a, 0, cols4, h->d_cidx, h->d_cw, h->cS);
            if (tail > 0) launch_gather<1, NEST, ZOUT>(a, tail0, tail, h->d_cidx, h->d_cw, h->cS);
        });
    } else if (h->delay == 0) {
        // w first: the fused kernel de-biases with the NEW weights and never needs the old ones
        hipLaunchKernelGGL(k_w_mix, dim3(1), dim3(wblock), 0, st, w, n, tab_k, S, s.p, h->d_unit_w,
                           (int)h->biased, h->d_w_old);
        if (tev) SGP_HIP_TRY(h, hipEventRecord(tev[0], st));
        if (!gather) {
            const int hop = s.distinct ? s.uniq[0] % n : 0;
            const int ncyc = s.distinct ? gcd_int(n, hop) : n;   // no peer: n cycles of length 1
            const int len = n / ncyc;
            if (fused && z_out && n <= kStatsCache && cols4 > 0 && tail == 0) {
                const unsigned Gf = grid_for(cols4, kStatsStepBlock);
                const size_t need = (size_t)(kStatsCache + 1) * Gf;
                if (need > h->partial_f_elems) {
                    if (h->d_partial_f) (void)hipFree(h->d_partial_f);
                    h->d_partial_f = nullptr;
                    h->partial_f_elems = 0;
                    hipError_t e = hipMalloc(&h->d_partial_f, need * sizeof(float));
                    if (e != hipSuccess) return e == hipErrorOutOfMemory ? SGP_ERR_NOMEM : hip_fail(h, e);
                    h->partial_f_elems = need;
                }
                if (nest)
                    hipLaunchKernelGGL(k_step_one_peer_stats<true>, dim3(Gf), dim3(kStatsStepBlock), 0, st, x, m, g,
                                       z_out, w, h->d_unit_w, n, (size_t)h->ld, cols4, hop, len, s.p, hp,
                                       h->d_partial_f);
                else
                    hipLaunchKernelGGL(k_step_one_peer_stats<false>, dim3(Gf), dim3(kStatsStepBlock), 0, st, x, m, g,
                                       z_out, w, h->d_unit_w, n, (size_t)h->ld, cols4, hop, len, s.p, hp,
                                       h->d_partial_f);
                fused->G = (int)Gf;
                fused->hop = hop;
                fused->len = len;
            } else
            dispatch_flags(nest, z_out != nullptr, [&]<bool NEST, bool ZOUT>() {
                if (cols4 > 0) launch_one_peer<4, NEST, ZOUT>(a, 0, cols4, hop, len);
                if (tail > 0) launch_one_peer<1, NEST, ZOUT>(a, tail0, tail, hop, len);
            });
        } else {
            dispatch_flags(nest, z_out != nullptr, [&]<bool NEST, bool ZOUT>() {
                if (cols4 > 0) launch_gather<4, NEST, ZOUT>(a, 0, cols4, tab_k, nullptr, S);
                if (tail > 0) launch_gather<1, NEST, ZOUT>(a, tail0, tail, tab_k, nullptr, S);
            });
        }
    } else {
        const int *tab_prev = nullptr;
        int ha = 0, hb = 0;          // the previous round's hops, when there are exactly two
        if (h->have_msgs && h->L > 0 && S == 3) {
            const Schedule sp = make_schedule(n, h->peers, round - 1);
            ha = sp.uniq[0] % n;
            hb = sp.uniq[1] % n;
        }
        if (h->have_msgs && h->L > 0) {
            const int kprev = (int)((round - 1) % h->L);
            tab_prev = h->d_tab + (size_t)kprev * n * S;
        }
        const int cur = h->cur, prv = cur ^ 1;
        hipLaunchKernelGGL(k_w_delay, dim3(1), dim3(wblock), 0, st, w, h->d_msgw[prv], h->d_msgw[cur],
                           n, tab_prev, S, s.p, h->d_unit_w, (int)h->biased, h->d_w_old);
        if (tev) SGP_HIP_TRY(h, hipEventRecord(tev[0], st));
        dispatch_flags(nest, z_out != nullptr, [&]<bool NEST, bool ZOUT>() {
            if (cols4 > 0)
                launch_delay<4, NEST, ZOUT>(a, 0, cols4, h->d_msg[prv], h->d_msg[cur], tab_prev, S, ha, hb);
            if (tail > 0)
                launch_delay<1, NEST, ZOUT>(a, tail0, tail, h->d_msg[prv], h->d_msg[cur], tab_prev, S, ha,
                                            hb);
        });
        h->cur = prv;
        h->have_msgs = true;
        h->last_k = k;
    }
    if (tev) {
        SGP_HIP_TRY(h, hipEventRecord(tev[1], st));
        ++h->ev_head;
    }
    SGP_HIP_TRY(h, hipGetLastError());
    return SGP_OK;
}

int sgp_step(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out, float gamma,
             float momentum, int64_t k, void *stream)
{
    return step_impl(h, x, w, m, g, z_out, gamma, momentum, k, stream, nullptr);
}

// Reduces a partial table to the statistics, copies them to the host and waits.  fused == NULL:
// the stand-alone kernels' table [(n+1)][G]; else the fused kernel's.
static int finish_stats(sgp_handle *h, const float *partial, int G, const FusedStats *fused, const float *w,
                        sgp_stats *host_out, double *per_node_dist_host, hipStream_t st)
{
    const int n = h->n;
    if (fused) {
        const int B = std::min(kSlotSumBlocks, G);
        hipLaunchKernelGGL(k_stats_slotsum, dim3(B), dim3(kSlotSumBlock), 0, st, partial, G, h->d_sums);
        hipLaunchKernelGGL(k_stats_final_slots, dim3(1), dim3(kFinalSlotsBlock), 0, st, h->d_sums, B, n, fused->hop,
                           fused->len, w, h->d_result);
    } else {
        hipLaunchKernelGGL(k_stats_rowsum, dim3(n + 1), dim3(kRowSumBlock), 0, st, partial, G, h->d_sums);
        hipLaunchKernelGGL(k_stats_final, dim3(1), dim3(64), 0, st, h->d_sums, n, w, h->d_result);
    }
    SGP_HIP_TRY(h, hipGetLastError());
    SGP_HIP_TRY(h, hipMemcpyAsync(h->h_result, h->d_result, (size_t)(8 + n) * sizeof(double),
                                  hipMemcpyDeviceToHost, st));
    SGP_HIP_TRY(h, hipStreamSynchronize(st));
    host_out->dist_max = h->h_result[0];
    host_out->dist_mean = h->h_result[1];
    host_out->dist_min = h->h_result[2];
    host_out->w_sum = h->h_result[3];
    host_out->zbar_norm = h->h_result[4];
    host_out->argmax = (int32_t)h->h_result[5];
    host_out->argmin = (int32_t)h->h_result[6];
    if (per_node_dist_host)
        for (int i = 0; i < n; ++i) per_node_dist_host[i] = h->h_result[8 + i];
    return SGP_OK;
}

int sgp_step_stats(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out,
                   float gamma, float momentum, int64_t k, sgp_stats *host_out,
                   double *per_node_dist_host, void *stream)
{
    if (!z_out || !host_out) return SGP_ERR_INVALID_ARG;
    FusedStats fused;
    int rc = step_impl(h, x, w, m, g, z_out, gamma, momentum, k, stream, &fused);
    if (rc != SGP_OK) return rc;
    if (fused.G > 0)
        return finish_stats(h, h->d_partial_f, fused.G, &fused, w, host_out, per_node_dist_host,
                            static_cast<hipStream_t>(stream));
    return sgp_consensus_stats(h, z_out, w, host_out, per_node_dist_host, stream);
}

int sgp_set_kernel_timing(sgp_handle *h, int enable)
{
    if (!h) return SGP_ERR_INVALID_ARG;
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

int sgp_consensus_stats(sgp_handle *h, const float *z, const float *w, sgp_stats *host_out,
                        double *per_node_dist_host, void *stream)
{
    if (!h || !z || !w || !host_out) return SGP_ERR_INVALID_ARG;
    if (!aligned4(z) || !aligned4(w)) return SGP_ERR_ALIGNMENT;
    int rc = ensure_device(h);
    if (rc != SGP_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int n = h->n;
    const bool vec = (h->ld % 4 == 0) && aligned16(z);
    const long cols4 = vec ? (long)(h->d / 4) : 0;
    const size_t tail0 = (size_t)cols4 * 4;
    const long tail = (long)(h->d - (int64_t)tail0);
    const int G = h->G;
    const size_t lds_large = (size_t)(kBlock / 64) * (n + 1) * sizeof(float);

    // every block writes its column of the partial table; blocks beyond the tile count write 0
    bool first = true;
    auto run = [&](auto vtag, size_t col0, long ncols) {
        constexpr int V = decltype(vtag)::value;
        long ntiles = (ncols + kBlock - 1) / kBlock;
        int acc = first ? 0 : 1;
        if (n <= kStatsCache)
            hipLaunchKernelGGL(k_stats_small<V>, dim3(G), dim3(kBlock), 0, st, z, n, (size_t)h->ld,
                               col0, ncols, ntiles, h->d_partial, G, acc);
        else
            hipLaunchKernelGGL(k_stats_large<V>, dim3(G), dim3(kBlock), lds_large, st, z, n,
                               (size_t)h->ld, col0, ncols, ntiles, h->d_partial, G, acc);
        first = false;
    };
    if (cols4 > 0) run(std::integral_constant<int, 4>{}, 0, cols4);
    if (tail > 0) run(std::integral_constant<int, 1>{}, tail0, tail);
    SGP_HIP_TRY(h, hipGetLastError());
    return finish_stats(h, h->d_partial, G, nullptr, w, host_out, per_node_dist_host, st);
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

}  // extern "C"
