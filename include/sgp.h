/*
 * sgp.h -- C ABI of the MI355X (gfx950) library for the per-iteration update of Stochastic
 * Gradient Push (SGP, arXiv 1811.10792) over n simulated nodes whose states all live in one
 * GPU's memory.
 *
 * One iteration at node i (Alg. 1; with Nesterov momentum, Alg. 3):
 *     u_i  <- momentum * u_i + g_i                                  (Alg. 3 only)
 *     xh_i  = x_i - gamma * (momentum * u_i + g_i)                  (Alg. 1: x_i - gamma * g_i)
 *     x_i  <- sum_j p_ij^(k) xh_j ,   w_i <- sum_j p_ij^(k) w_j     (PushSum mix)
 *     z_i   = x_i / w_i                                             (de-bias)
 * with P^(k) the column-stochastic mixing matrix of the time-varying directed exponential
 * graph with uniform weights (Appendix A "Definition of P^(k)", Appendix C).  The exchange of
 * messages between nodes is an on-device gather; no inter-GPU communication is involved.
 *
 * Data layout (all device memory is CALLER-OWNED, float32):
 *     x, m (the paper's momentum buffer u), g, z : [n][ld] row-major, one row per node, row
 *         stride ld >= d elements; only the first d elements of a row are read or written.
 *     w : [n].
 * The fast path needs ld % 4 == 0 and 16-byte aligned base pointers (128-bit accesses);
 * otherwise a scalar path is used.  For full bandwidth choose ld as a multiple of 256 elements so
 * that every row starts on a 1 KiB boundary: rows that start off a 128-byte boundary split each
 * wavefront's 1 KiB access over an extra cache line and cost about 15 % of the achieved HBM
 * bandwidth (measured on MI355X).  Where the arrays sit matters as well: the 288 GiB of HBM behave as
 * three 96 GiB regions, and arrays that are written at the same time (x, m, z) slow each other down
 * when they share one; with x (and g), m and z in three different regions the step kernels reach
 * 80 % of the HBM peak, with back-to-back allocations 64 %.  The library takes the pointers as they
 * come; sgp_probe_regions (below) finds the regions of a caller's arena by timing, so that the caller
 * can carve x, m and z out of three different ones (the Python package's placement module does that).
 * State arrays are streamed past the caches (non-temporal accesses), except for problems whose four
 * arrays together stay below 160 MiB and can live in the last-level cache from one iteration to the
 * next: those are accessed with ordinary loads and stores (chosen at launch time).
 * Arithmetic is IEEE binary32, round to nearest even, every
 * operation rounded separately (no fused multiply-add), correctly rounded division, subnormals
 * kept.  Sums over senders are taken in ascending sender index.
 *
 * Every function returns an int status: SGP_OK or a negative SGP_ERR_* code; nothing throws or
 * aborts.  Device work is enqueued on the given HIP stream (hipStream_t passed as void*, NULL =
 * default stream) and is asynchronous with respect to the host unless stated otherwise.  A
 * handle must not be used from two host threads at once, and all calls on one handle must be
 * enqueued on streams that are ordered with respect to each other.
 */
#ifndef SGP_H_
#define SGP_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SGP_OK 0
#define SGP_ERR_INVALID_ARG (-1) /* null pointer, size or parameter out of range */
#define SGP_ERR_UNSUPPORTED (-2) /* valid request the library has no kernel for */
#define SGP_ERR_ALIGNMENT (-3)   /* a float pointer that is not 4-byte aligned */
#define SGP_ERR_SEQUENCE (-4)    /* overlap mode: k is not the previous call's k plus one */
#define SGP_ERR_HIP (-5)         /* a HIP call failed; see sgp_last_hip_error */
#define SGP_ERR_NOMEM (-6)       /* host or device allocation failed */

#define SGP_TOPO_DIRECTED_EXP 0 /* time-varying directed exponential graph (Appendix A) */
#define SGP_TOPO_COMPLETE 1     /* every entry of P equal to 1/n: SGP then coincides with parallel
                                   SGD over AllReduce (section 3) */
#define SGP_TOPO_CUSTOM 2       /* caller-supplied sparse rows of P, see sgp_set_mixing */

#define SGP_MAX_NODES 1024 /* largest n accepted by sgp_create */
#define SGP_MAX_NODES_GATHER 600 /* largest n for more than one peer without delay and for custom rows
                                    (128-bit accesses up to n = 150, scalar ones beyond) */
#define SGP_MAX_PEERS 16   /* largest peers accepted by sgp_create */
#define SGP_MAX_DELAY 64   /* largest delay (tau) accepted by sgp_create */

typedef struct sgp_handle sgp_handle;

/* Result of sgp_consensus_stats ("Parameter deviations": Euclidean distance between each node's
 * parameters and the node-wise average, summarised by mean, max and min over nodes). */
typedef struct sgp_stats {
    double dist_max;  /* max_i || z_i - zbar ||_2 ,  zbar = (1/n) sum_i z_i */
    double dist_mean; /* (1/n) sum_i || z_i - zbar ||_2 */
    double dist_min;  /* min_i || z_i - zbar ||_2 */
    double w_sum;     /* sum_i w_i (equals n, minus weight in transit in overlap mode) */
    double zbar_norm; /* || zbar ||_2 */
    int32_t argmax;   /* node attaining dist_max (lowest index on ties) */
    int32_t argmin;   /* node attaining dist_min (lowest index on ties) */
} sgp_stats;

/*
 * Creates a handle for n nodes of d parameters with row stride ld (elements).
 *   topology : SGP_TOPO_DIRECTED_EXP, or (delay == 0 only) SGP_TOPO_COMPLETE / SGP_TOPO_CUSTOM,
 *              for which peers is ignored (pass 1).
 *   peers    : out-peers per iteration, 1..SGP_MAX_PEERS (the paper uses 1 and 2).  At iteration
 *              k a node sends to the peers 2^((k+r) mod L) hops ahead, r = 0..peers-1, where
 *              L = floor(log2(n-1)) + 1 is the length of the peer list 2^0 .. 2^floor(log2(n-1));
 *              a peer reached twice counts once, and each out-neighbour (the node itself
 *              included) gets weight 1/|N_out|.
 *   delay    : tau of Alg. 2, 0..SGP_MAX_DELAY.  0 = blocking SGP (Alg. 1/3).  1 = 1-overlap SGP:
 *              the mix at iteration k uses the node's own share of iteration k and the messages
 *              that were sent at iteration k-1.  tau >= 2: nodes send only at the iterations with
 *              k mod tau == 0 (communication round c = k / tau uses the peers of schedule entry c)
 *              and keep x_i <- xh_i, w_i unchanged at the others; every message is received tau
 *              iterations after it was sent, i.e. at the next sending iteration.  For delay >= 1
 *              the library owns two [n][ld] message buffers.
 * Host-only: no device memory is touched until the first call that launches work.
 * Errors: SGP_ERR_INVALID_ARG (out == NULL, n < 1, n > SGP_MAX_NODES, d < 1, ld < d, peers or
 * delay out of range), SGP_ERR_UNSUPPORTED (unknown topology, or a topology other than the
 * exponential graph with delay > 0); *out is NULL on error.
 */
int sgp_create(sgp_handle **out, int32_t n, int64_t d, int64_t ld, int32_t topology,
               int32_t peers, int32_t delay);

/* Frees the handle and the device memory the library allocated for it (never caller memory).
 * Synchronises the device first.  NULL is accepted. */
int sgp_destroy(sgp_handle *h);

/* Overlap mode: makes the library keep its two message buffers in caller-owned device memory
 * (each [n][ld] floats, 16-byte aligned, distinct, not overlapping any state array) instead of
 * allocating them, e.g. so that the caller controls where in HBM they live.  Must be called
 * before the first sgp_step on the handle; also drops messages in flight like sgp_reset.
 * Errors: SGP_ERR_INVALID_ARG (null, equal or misaligned pointers, delay == 0),
 * SGP_ERR_SEQUENCE (device resources already set up). */
int sgp_set_message_buffers(sgp_handle *h, float *buf0, float *buf1);

/*
 * Changes the communication topology (and, for the exponential graph, the number of out-peers) from
 * the next sgp_step on, for schedules that communicate more at the start of training (the hybrid
 * AR/1P and 2P/1P schemes of the experiments: complete graph or two peers first, one peer later).
 * The iteration index k keeps counting.  Blocking mode only: SGP_ERR_UNSUPPORTED if delay > 0.
 * Synchronises the device when the handle has already launched work.
 */
int sgp_set_topology(sgp_handle *h, int32_t topology, int32_t peers);

/*
 * SGP_TOPO_CUSTOM: sets the mixing matrix used by the following steps as sparse rows, so that any
 * column-stochastic P with positive diagonal (section 3; non-uniform weights, irregular graphs)
 * can be run, e.g. the 4-node example of the appendix on message delays.
 *   in_idx    [n][entries] host : in_idx[i*entries + q] = a node that receiver i hears from (its own
 *                                 index included if it keeps a share), or -1 for an unused entry
 *   in_weight [n][entries] host : p_{i,j} of that entry
 * Receiver i computes sum_q fl(in_weight * xh_j) over its used entries in the order given (list
 * senders in ascending index to reproduce a dense row-times-vector product).  The arrays are copied;
 * may be called again between steps (time-varying P).  n <= SGP_MAX_NODES_GATHER.
 * Errors: SGP_ERR_INVALID_ARG (null, entries < 1 or > n, index out of range), SGP_ERR_NOMEM,
 * SGP_ERR_HIP.  sgp_step on a custom handle without mixing rows returns SGP_ERR_SEQUENCE.
 */
int sgp_set_mixing(sgp_handle *h, const int32_t *in_idx, const float *in_weight, int32_t entries);

/*
 * Weight decay fused into the local step (the hyperparameter appendix: the ImageNet runs use
 * weight decay 1e-4 with Nesterov momentum): from the next sgp_step on, g_i is replaced by
 * g_i + weight_decay * theta_i before the local step of Alg. 1 / Alg. 3, where theta_i is the
 * de-biased z_i^(k) = x_i^(k) / w_i^(k) (on_numerator == 0; the gradient of the L2 term at the
 * point where g_i was evaluated) or the numerator x_i^(k) (on_numerator != 0; what an optimizer
 * that steps on the biased parameters applies).  The paper does not say which; they coincide
 * whenever w = 1, i.e. for blocking SGP on the exponential graph.  With sgp_set_biased the
 * numerator is used.  weight_decay = 0 switches it off.  Costs no extra memory traffic (x is
 * read anyway).  Errors: SGP_ERR_INVALID_ARG (null handle, negative or NaN coefficient).
 */
int sgp_set_weight_decay(sgp_handle *h, float weight_decay, int on_numerator);

/* Ablation without the push-sum weight ("biased" overlap SGP in the paper's comparison of 1-OSGP
 * with its biased implementation): with biased != 0 every later step writes z_i = x_i instead of
 * x_i / w_i.  w is still updated and reported.  Any delay; takes effect at the next sgp_step. */
int sgp_set_biased(sgp_handle *h, int biased);

/* Overlap mode: drops the messages in flight, so that the next sgp_step receives nothing (as
 * the first iteration of Alg. 2 does) and may start at any k.  No-op for delay == 0. */
int sgp_reset(sgp_handle *h);

/*
 * One SGP iteration k for all nodes (the loop body of Alg. 1 / Alg. 3; overlap mode: Alg. 2
 * with tau = 1), in place.
 *   x        [n][ld] device, in/out : push-sum numerators x^(k) -> x^(k+1)
 *   w        [n]     device, in/out : push-sum weights   w^(k) -> w^(k+1)
 *   m        [n][ld] device, in/out : momentum buffers u^(k) -> u^(k+1); may be NULL when
 *                                     momentum == 0 (then Alg. 1 is run and m is not touched)
 *   g        [n][ld] device, in     : stochastic gradients evaluated by the caller at z^(k)
 *   z_out    [n][ld] device, out    : de-biased z^(k+1) = x^(k+1)/w^(k+1); NULL = not wanted;
 *                                     must not overlap x, m or g
 *   gamma, momentum : step size and Nesterov coefficient
 *   k        >= 0   : iteration index; selects P^(k) (the schedule is a pure function of k)
 * Overlap mode (delay >= 1): the first call after sgp_create/sgp_reset receives nothing and may
 * start at any k; every later call must pass the previous k plus one (else SGP_ERR_SEQUENCE and
 * nothing is launched).  Messages sent at the last sending iteration stay in the library's
 * buffers.
 * Errors: SGP_ERR_INVALID_ARG, SGP_ERR_ALIGNMENT, SGP_ERR_SEQUENCE, SGP_ERR_UNSUPPORTED (more
 * than one peer without delay, or caller-supplied rows, and n > SGP_MAX_NODES_GATHER: those modes
 * keep one LDS column of n values per work-item), SGP_ERR_NOMEM, SGP_ERR_HIP.  A call that returns
 * an error has not modified x, w, m or z_out.
 * The push-sum weights are updated by the step kernel itself: w holds w^(k) until the kernel's last
 * block has finished and w^(k+1) afterwards; one call is one kernel launch (two when d % 4 != 0 or
 * an array is not 16-byte aligned).  w is read at every call, so the caller may overwrite it between
 * steps.
 * HIP graphs: after the first call on a handle (which allocates the library's small tables) sgp_step
 * allocates nothing, records no memset and only launches kernels on `stream`, so a run of iterations
 * can be captured into a graph and replayed.  Measured on MI355X this no longer pays: since a step
 * became one launch, replaying a captured cycle of the schedule was no faster than eager calls
 * (31.8 against 30.2 us per iteration at n = 8, d = 2^20; 9.5 against 9.1 us at n = 4, d = 1024).
 */
int sgp_step(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out,
             float gamma, float momentum, int64_t k, void *stream);

/*
 * One SGP iteration with Adam as the local optimiser (the machine-translation runs combine SGP with
 * the Adam preconditioner; the paper prints no formulas, so Adam is taken as published by Kingma
 * and Ba and applied to the numerator with the gradient evaluated at z):
 *     m1_i <- beta1 m1_i + (1 - beta1) g_i ,   m2_i <- beta2 m2_i + (1 - beta2) g_i^2
 *     xh_i  = x_i - gamma * (m1_i / (1 - beta1^t)) / (sqrt(m2_i / (1 - beta2^t)) + eps)
 * followed by the same mix, weight update and de-bias as sgp_step, for every topology and delay.
 *   m1, m2 [n][ld] device, in/out : first and second moment (start at zero); m2 must not overlap
 *                                   any other array
 *   t >= 1                        : Adam's step count (bias corrections are formed in double and
 *                                   rounded once to float)
 * Other arguments, layout, overlap-mode sequencing and errors as for sgp_step; weight decay set by
 * sgp_set_weight_decay is added to g_i first (L2 form).  32 bytes of HBM traffic per node-parameter
 * (40 in overlap mode).
 */
int sgp_step_adam(sgp_handle *h, float *x, float *w, float *m1, float *m2, const float *g, float *z_out,
                  float gamma, float beta1, float beta2, float eps, int64_t t, int64_t k, void *stream);

/*
 * Bandwidth experiment, NOT part of the paper's method: sgp_step with some arrays stored as bfloat16
 * (the upper 16 bits of a binary32: 8 exponent bits, 7 fraction bits).  Arithmetic is unchanged
 * (binary32, operation by operation as in sgp_step); a stored value is widened exactly when it is
 * loaded and rounded to nearest, ties to even, when it is stored (NaN stays NaN).  In particular the
 * local step uses the new momentum as computed, not as stored.
 *   storage = SGP_STORE_BF16_GZ                    : g and z_out are bfloat16 [n][ld]; 20 bytes of HBM
 *                                                    traffic per node-parameter instead of 24
 *   storage = SGP_STORE_BF16_GZ | SGP_STORE_BF16_U : m is bfloat16 [n][ld] as well; 16 bytes
 * x [n][ld] and w [n] stay float.  Blocking mode (delay 0) on the exponential graph with one
 * distinct out-peer and momentum != 0 only: anything else is SGP_ERR_UNSUPPORTED.  The fast path
 * needs ld % 4 == 0, 16-byte aligned float arrays and 8-byte aligned bfloat16 arrays.
 * Other arguments, errors and weight handling as for sgp_step.
 */
#define SGP_STORE_BF16_GZ 1
#define SGP_STORE_BF16_U 2
int sgp_step_bf16(sgp_handle *h, float *x, float *w, void *m, const void *g16, void *z16, float gamma,
                  float momentum, int64_t k, int32_t storage, void *stream);

/* z_i = x_i / w_i for all nodes (last line of Alg. 1); x [n][ld], w [n], z [n][ld] device.
 * Used for z^(0) and whenever sgp_step was called with z_out == NULL. */
int sgp_debias(sgp_handle *h, const float *x, const float *w, float *z, void *stream);

/*
 * Consensus statistics of z [n][ld] (device) and w [n] (device): per-node distance to the
 * node-wise average and its max / mean / min, sum of weights, norm of the average.
 *   host_out           : host, written on return
 *   per_node_dist_host : host [n] doubles, or NULL
 * Enqueues the reduction kernels on `stream`, copies the result back and SYNCHRONISES the
 * stream before returning.
 */
int sgp_consensus_stats(sgp_handle *h, const float *z, const float *w, sgp_stats *host_out,
                        double *per_node_dist_host, void *stream);

/*
 * The same statistics at the measurement point of the figure on parameter deviations: after the
 * local step and before communication (the gradient step of Alg. 1 done, nothing sent yet).  Takes the state BEFORE
 * iteration k and the gradient of iteration k, forms xh_i as sgp_step would (gradient step of Alg. 1, or
 * momentum and gradient steps of Alg. 3 when momentum != 0, weight decay included) and reports the deviations of
 * xh_i / w_i from their node-wise average.  Nothing is modified: call it before the sgp_step that
 * consumes the same g.  Reads x, g (and m) once (twice for n > 32).  SYNCHRONISES the stream.
 */
int sgp_pregossip_stats(sgp_handle *h, const float *x, const float *w, const float *m, const float *g,
                        float gamma, float momentum, sgp_stats *host_out, double *per_node_dist_host,
                        void *stream);

/*
 * sgp_step followed by sgp_consensus_stats of the z^(k+1) it wrote, in one call (Alg. 1 / Alg. 3
 * plus the "Parameter deviations" statistics).  Arguments as in those two calls; z_out and
 * host_out are required.  With n <= 32, d % 4 == 0, the 128-bit layout and SGD or Nesterov as the
 * local step, the statistics are accumulated inside the step kernel while z is still in registers
 * (z is not read back from HBM), for every topology without delay, for the iterations between two
 * communication rounds of tau-overlap SGP, and for overlap iterations that receive one or two
 * messages per node (one or two out-peers; the very first iteration, which receives nothing, does
 * not qualify); otherwise the two kernels run one after the other.  The state written is identical to
 * sgp_step's; the statistics agree with sgp_consensus_stats to rounding (a different reference row
 * is subtracted before squaring).  The reduction of the fused kernel's partial sums follows the step
 * kernel on the caller's stream.  SYNCHRONISES the stream.
 */
int sgp_step_stats(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out,
                   float gamma, float momentum, int64_t k, sgp_stats *host_out,
                   double *per_node_dist_host, void *stream);

/*
 * The same work as sgp_step_stats without draining the stream every iteration.
 * sgp_step_stats_begin enqueues iteration k, the statistics of the z it writes and their copy to
 * the host, and returns at once; sgp_step_stats_end hands out the oldest result not yet fetched,
 * waiting (for that result only) if it is not there yet.  At most two results may be outstanding:
 * a third begin returns SGP_ERR_SEQUENCE, as does an end with nothing outstanding.  Typical loop:
 * begin(k); if (k > 0) end(result of k-1); ... ; end(last).  The GPU then never waits for the host.
 * The reduction of a fused kernel's partial sums runs on a stream that the library owns, behind the
 * step kernel (its last block writes the result into pinned host memory), so that the caller's
 * stream carries the step kernels and nothing else.
 * All begin calls between two ends must use streams that are ordered with respect to each other.
 */
int sgp_step_stats_begin(sgp_handle *h, float *x, float *w, float *m, const float *g, float *z_out,
                         float gamma, float momentum, int64_t k, void *stream);
int sgp_step_stats_end(sgp_handle *h, sgp_stats *host_out, double *per_node_dist_host);

/*
 * sgp_consensus_stats for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Handle-free; calls no hipMalloc / hipFree / hipHostMalloc
 * and does not synchronise.  Its scratch (the [(n+1)][2048] float table of partial sums and n+1
 * doubles) is a fixed device array inside the library, about 1.06 MB, which every GPU the library
 * runs on holds until the process ends; n is therefore limited to SGP_NOALLOC_MAX_NODES.
 *   z [n][ld] device, w [n] device : as for sgp_consensus_stats
 *   out_device [8 + n] doubles, device, 8-byte aligned, written by the last kernel enqueued:
 *       out[0] dist_max, [1] dist_mean, [2] dist_min, [3] sum_i w_i, [4] ||zbar||_2, [5] argmax,
 *       [6] argmin (both as doubles), [7] 0, out[8 + i] = || z_i - zbar ||_2
 * Runs the same kernels as sgp_consensus_stats, so the values are identical to that call's.
 * All calls on one GPU share that GPU's scratch array: calls whose kernels overlap in time on one
 * GPU (different streams, or different host threads) race; order them.  Nothing in the array has to
 * be cleared between calls (every entry that is read has been written by the same call).
 * Errors: SGP_ERR_INVALID_ARG (null pointer, n < 1, d < 1, ld < d), SGP_ERR_UNSUPPORTED
 * (n > SGP_NOALLOC_MAX_NODES), SGP_ERR_ALIGNMENT, SGP_ERR_HIP.
 */
#define SGP_NOALLOC_MAX_NODES 128
int sgp_consensus_stats_noalloc(int32_t n, int64_t d, int64_t ld, const float *z, const float *w,
                                double *out_device, void *stream);

/*
 * Peer schedule of iteration k (host-only, integer arithmetic; Appendix A).  Exponential graph only
 * (SGP_ERR_UNSUPPORTED otherwise).
 *   out_peers [n][peers] : out_peers[i*peers + r] = node that i sends to over its r-th hop,
 *                          (i + 2^((k+r) mod L)) mod n, or -1 if that peer repeats an earlier one
 *                          (or n == 1)
 *   in_peers  [n][peers] : in_peers[i*peers + r] = node that i receives from over the r-th hop,
 *                          (i - 2^((k+r) mod L)) mod n, or -1 likewise
 *   weight               : the uniform mixing weight 1/|N_out| of that iteration
 * Any output pointer may be NULL.  In overlap mode the messages RECEIVED at iteration k are
 * those of sgp_peer_schedule(k - delay).  With delay >= 2 an iteration that is not a multiple of
 * delay has no peers (all entries -1, weight 1), and iteration k = c * delay uses schedule entry c.
 */
int sgp_peer_schedule(const sgp_handle *h, int64_t k, int32_t *out_peers, int32_t *in_peers,
                      float *weight);

/* Same as sgp_peer_schedule without a handle. */
int sgp_schedule(int32_t n, int32_t peers, int64_t k, int32_t *out_peers, int32_t *in_peers,
                 float *weight);

/* Static, human-readable name of a status code. */
const char *sgp_status_string(int status);

/* hipError_t value of the last failed HIP call on this handle (0 if none). */
int sgp_last_hip_error(const sgp_handle *h);

/* Test hook: the library's next `succeed_first` device allocations (process-wide) succeed, the one
 * after them fails as if the device were out of memory, later ones succeed again; a negative value
 * switches the hook off.  Lets a test drive the SGP_ERR_NOMEM paths: a step that fails this way has
 * launched nothing, and a repeated call picks the set-up up where it stopped. */
int sgp_debug_fail_alloc(int32_t succeed_first);

/* Measurement utility: static name of the step kernel that the latest successful step on this
 * handle launched ("k_step_one_peer", "k_step_gather", "k_step_complete", "k_step_delay",
 * "k_step_delay2", "k_step_one_peer_h16", and with fused statistics "k_step_one_peer_stats",
 * "k_step_gather_stats", "k_step_complete_stats", "k_step_delay1_stats", "k_step_delay2_stats";
 * "" before the first step), so that a benchmark can report what ran instead of re-deriving the library's dispatch. */
const char *sgp_last_step_kernel(const sgp_handle *h);

/*
 * Measurement utility.  With timing enabled, sgp_step brackets its fused step kernel (not the
 * single-block weight kernel in front of it) with HIP events recorded on the stream the kernel is
 * launched on; the library keeps the last SGP_TIMING_RING pairs.
 * sgp_step_kernel_times waits for the most recent timed kernel, writes the durations (ms, oldest
 * first) of the timed steps since the previous call into ms_out[0 .. max-1] and their number into
 * *count (at most min(max, SGP_TIMING_RING); older ones are dropped).
 */
#define SGP_TIMING_RING 64
int sgp_set_kernel_timing(sgp_handle *h, int enable);
int sgp_step_kernel_times(sgp_handle *h, float *ms_out, int32_t max, int32_t *count);

/*
 * Measurement utility: finds which parts of a caller-owned device arena interfere with each other
 * as concurrent HBM streams.  On MI355X, arrays that are written at the same time slow each other
 * down when they lie in the same one of (measured) three 96 GiB regions of the 288 GiB, and user
 * space cannot see physical addresses; so nothing is assumed and the arena is classified by timing.
 * The arena is cut into granules of granule_bytes.  A small SGP problem (32 nodes, 2^22 coordinates,
 * one peer, Nesterov) is stepped with x, m, g inside a reference granule and z inside the granule
 * under test; the granule belongs to the reference's region when that step is slow (above the
 * midpoint between the fastest and the slowest candidate; less than 8 % contrast = one region).
 * Repeats with a new reference until every granule has a class or max_classes is reached; a single
 * granule that disagrees with two agreeing neighbours is treated as a timing outlier.
 *   arena, arena_bytes      : device memory, 16-byte aligned; its CONTENTS ARE DESTROYED
 *   granule_bytes           : multiple of 4096; at least 2 GiB for the probe problem to fit (smaller
 *                             granules, or fewer than two of them, are reported as one class)
 *   class_of_granule [arena_bytes / granule_bytes] host, out : classes numbered from 0 in order of
 *                             first appearance; equal class = same region
 *   probe_ms [same length]  host, out, nullable : the step-kernel time (ms) of the first pass, i.e.
 *                             with the first granule as reference (0 where not measured)
 *   structured              host, out : 1 if more than one region was told apart
 * Allocates a few hundred bytes of device memory, launches a few hundred small kernels on `stream`
 * and SYNCHRONISES it; takes of the order of a second per pass.
 * Errors: SGP_ERR_INVALID_ARG, SGP_ERR_NOMEM, SGP_ERR_HIP.
 */
int sgp_probe_regions(void *arena, int64_t arena_bytes, int64_t granule_bytes, int32_t max_classes,
                      int32_t *class_of_granule, float *probe_ms, int32_t *structured, void *stream);

/* Host-only: the clean-up that sgp_probe_regions applies to its raw classes, in place: a single
 * granule whose two neighbours agree with each other but not with it takes their class (regions are
 * contiguous address ranges, so such a granule is a timing outlier), then the classes are renumbered
 * from 0 in order of first appearance.  Errors: SGP_ERR_INVALID_ARG (null with count > 0, count < 0). */
int sgp_smooth_region_classes(int32_t *class_of_granule, int32_t count);

/*
 * Host-only: carves arrays out of an arena whose granules sgp_probe_regions has classified, so that
 * arrays which are written at the same time land in different regions.  No device call is made; the
 * offsets are relative to the arena's start and multiples of 4096.
 *   sgp_placer_create : class_of_granule [count] as sgp_probe_regions wrote it, granule_bytes as given there
 *   sgp_placer_take   : a fresh range of nbytes for an array in the given role.  Roles: x, u (the
 *                       array `m` of sgp_step) and z are the three written streams and go to three
 *                       different regions, the largest regions first; g is read-only and shares the
 *                       region of x; the two message buffers of overlap mode go with u;
 *                       Adam's second moment with x.  Inside a region the interiors of long runs of
 *                       granules are used before their edge granules (which may straddle a region
 *                       boundary) and before short runs.  When the preferred region is full, any
 *                       other with room is taken; *class_out (nullable) tells which region it was.
 *                       SGP_ERR_NOMEM when nothing fits.
 *   sgp_placer_reset  : forgets every range handed out.
 * Errors: SGP_ERR_INVALID_ARG, SGP_ERR_NOMEM.
 */
typedef struct sgp_placer sgp_placer;
#define SGP_ROLE_X 0
#define SGP_ROLE_G 1
#define SGP_ROLE_U 2
#define SGP_ROLE_Z 3
#define SGP_ROLE_MSG0 4
#define SGP_ROLE_MSG1 5
#define SGP_ROLE_V 6
#define SGP_ROLE_COUNT 7
int sgp_placer_create(sgp_placer **out, const int32_t *class_of_granule, int32_t count, int64_t granule_bytes);
int sgp_placer_destroy(sgp_placer *p);
int sgp_placer_reset(sgp_placer *p);
int sgp_placer_take(sgp_placer *p, int32_t role, int64_t nbytes, int64_t *offset_out, int32_t *class_out);

/* Measurement utility: plain 128-bit streaming copy of nbytes (multiple of 16, both pointers
 * 16-byte aligned, device memory) on `stream`.  Serves as the known-size reference when
 * hardware traffic counters are scaled, and as the practical bandwidth ceiling of the part. */
int sgp_copy(void *dst, const void *src, int64_t nbytes, void *stream);

/* Measurement utility: one launch, on `stream`, of a structure-free kernel that reads each of
 * n_reads arrays and writes each of n_writes arrays of nbytes once, with 128-bit streaming
 * accesses: the traffic of a step kernel (3 reads and 3 writes per node-parameter) without its walk,
 * for any choice of where the arrays lie and of which are updated in place.  Every written element
 * is the float sum of the elements read at its offset (zero without reads).
 * reads, writes: HOST arrays of n_reads / n_writes DEVICE pointers, 16-byte aligned; 0..4 of each
 * and at least one in total; nbytes a multiple of 16.  A written array may coincide with a read
 * array (in place); apart from that no two arrays may overlap (SGP_ERR_INVALID_ARG).  Nothing is
 * allocated; the caller times the launch. */
int sgp_stream_pattern(const void *const *reads, int32_t n_reads, void *const *writes, int32_t n_writes,
                       int64_t nbytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SGP_H_ */
