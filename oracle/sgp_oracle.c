/*
 * CPU oracle for the per-iteration update of Stochastic Gradient Push (SGP).
 *
 * TEST INFRASTRUCTURE ONLY: a plain, slow, dense reference that the GPU library is checked
 * against.  It shares no code with the GPU path and must never be linked into it; only the
 * tests, the smoke check and the benchmark's CPU-baseline leg load it.
 *
 * What it computes, and where the paper defines it:
 *   sgpo_mixing_matrix_*   dense P^(k) of the directed exponential graph with uniform weights
 *                          (Appendix A "Definition of P^(k)", Appendix C mixing weights)
 *   sgpo_step_*            one SGP iteration, Alg. 1 / Alg. 3, as the dense product of
 *                          eq. "UpdateRule" applied per coordinate; optionally with weight
 *                          decay, or with Adam as the local step (hyperparameter appendix)
 *   sgpo_step_delay1_*     one iteration of 1-overlap SGP, Alg. 2 with tau = 1
 *   sgpo_step_osgp_*       one iteration of tau-overlap SGP, Alg. 2 with tau >= 1, and the
 *                          biased ablation that skips the de-bias
 *   sgpo_debias_*          z = x / w
 *   sgpo_consensus_stats   distance of every node's de-biased parameters to the node-wise
 *                          average (the "parameter deviations" paragraph and figure)
 *   sgpo_step_bf16         (not in the paper: storage experiment) sgpo_step_f32 with g, z and
 *                          optionally u held in memory as bfloat16; pinned by reduction to
 *                          sgpo_step_f32 on the widened inputs and to torch's bfloat16 rounding
 *
 * Pins (tests/test_oracle_pins.py): printed 4-node mixing matrix and its four update equations,
 * printed 8-node neighbour list, exact averaging after one cycle for n = 32 in 5 iterations,
 * column-stochastic conservation, consensus fixed point, all-reduce special case, brute-force
 * dense products written in numpy, the augmented virtual-node matrix for the delayed form,
 * closed-form weight recursions under delay.  sgpo_consensus_stats is pinned by closed forms
 * on constructed inputs and a numpy one-liner.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC (see oracle/sgp_oracle.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define CAT2_(a, b) a##b
#define CAT2(a, b) CAT2_(a, b)
#define FN(name) CAT2(name, SFX)

#define REAL double
#define SFX _f64
#define SQRT sqrt
#include "sgp_oracle_impl.inc"
#undef REAL
#undef SFX
#undef SQRT

#define REAL float
#define SFX _f32
#define SQRT sqrtf
#include "sgp_oracle_impl.inc"
#undef REAL
#undef SFX
#undef SQRT

/* Threads used by the coordinate loops (results do not depend on it). */
void sgpo_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

int sgpo_get_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Consensus statistics of z [n][d] (double):
 *   zbar[e]  = (1/n) sum_i z_i[e]                       node-wise average
 *   dist[i]  = || z_i - zbar ||_2                        Euclidean distance to it
 *   out[0..4] = max_i dist, mean_i dist, min_i dist, sum_i w_i, ||zbar||_2
 * ("Parameter deviations": distance between the parameters at individual nodes and the
 *  node-wise average, reported as mean with max and min over nodes.)
 */
void sgpo_consensus_stats(int n, int64_t d, const double *z, const double *w, double *dist,
                          double *out)
{
    double *zbar = (double *)malloc(sizeof(double) * (size_t)d);
    for (int64_t e = 0; e < d; e++) {
        double s = 0.0;
        for (int i = 0; i < n; i++) s += z[(size_t)i * (size_t)d + (size_t)e];
        zbar[e] = s / (double)n;
    }
    double dmax = 0.0, dmin = 0.0, dsum = 0.0;
    for (int i = 0; i < n; i++) {
        double s = 0.0;
        for (int64_t e = 0; e < d; e++) {
            double t = z[(size_t)i * (size_t)d + (size_t)e] - zbar[e];
            s += t * t;
        }
        dist[i] = sqrt(s);
        if (i == 0 || dist[i] > dmax) dmax = dist[i];
        if (i == 0 || dist[i] < dmin) dmin = dist[i];
        dsum += dist[i];
    }
    double wsum = 0.0;
    for (int i = 0; i < n; i++) wsum += w[i];
    double zn = 0.0;
    for (int64_t e = 0; e < d; e++) zn += zbar[e] * zbar[e];
    out[0] = dmax;
    out[1] = dsum / (double)n;
    out[2] = dmin;
    out[3] = wsum;
    out[4] = sqrt(zn);
    free(zbar);
}

/* ------------------------------------------------------------------------------------------
 * Storage experiment (not part of the paper's method): the binary32 iteration of sgpo_step_f32
 * with some arrays held in memory as bfloat16, i.e. the upper 16 bits of a binary32 (1 sign, 8
 * exponent, 7 fraction bits).  Loading widens exactly (append 16 zero bits).  Storing rounds to
 * the nearest bfloat16, ties to the one with an even last bit; a value beyond the largest finite
 * bfloat16 by half a step or more becomes infinity; NaN stays NaN.
 * ------------------------------------------------------------------------------------------ */
float sgpo_bf16_to_float(uint16_t h)
{
    uint32_t b = (uint32_t)h << 16;
    float f;
    memcpy(&f, &b, sizeof f);
    return f;
}

uint16_t sgpo_float_to_bf16(float f)
{
    uint32_t b;
    memcpy(&b, &f, sizeof b);
    uint32_t keep = b >> 16, drop = b & 0xffffu;
    if ((b & 0x7f800000u) == 0x7f800000u && (b & 0x007fffffu) != 0u) return (uint16_t)(keep | 0x0040u);
    if (drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) keep += 1u;   /* a carry runs into the exponent */
    return (uint16_t)keep;
}

/*
 * One SGP iteration (Alg. 3, Nesterov momentum) with g given and z returned as bfloat16, and the
 * momentum buffer held as bfloat16 when u_is_bf16 != 0 (then u points to uint16_t [n][d], else to
 * float [n][d]).  Everything between load and store is sgpo_step_f32's arithmetic: the local step
 * uses the new momentum as computed, the stored copy is its rounding.
 */
int sgpo_step_bf16(int n, int64_t d, const float *P, float *x, float *w, void *u, const uint16_t *g16,
                   uint16_t *z16, float gamma, float m, int u_is_bf16)
{
    float *w_new = (float *)malloc(sizeof(float) * (size_t)n);
    if (!w_new) return -1;
    for (int i = 0; i < n; i++) {
        float acc = 0.0f;
        for (int j = 0; j < n; j++) {
            float term = P[(size_t)i * n + j] * w[j];
            acc = acc + term;
        }
        w_new[i] = acc;
    }
#pragma omp parallel
    {
        float *xh = (float *)malloc(sizeof(float) * (size_t)n);
#pragma omp for schedule(static)
        for (int64_t e = 0; e < d; e++) {
            for (int i = 0; i < n; i++) {
                size_t a = (size_t)i * (size_t)d + (size_t)e;
                float ui = u_is_bf16 ? sgpo_bf16_to_float(((uint16_t *)u)[a]) : ((float *)u)[a];
                float gi = sgpo_bf16_to_float(g16[a]);
                xh[i] = sgpo_local_step_f32(x[a], 0.0f, &ui, NULL, gi, gamma, m, 1, 0.0f, NULL);
                if (u_is_bf16) ((uint16_t *)u)[a] = sgpo_float_to_bf16(ui);
                else ((float *)u)[a] = ui;
            }
            for (int i = 0; i < n; i++) {
                float acc = 0.0f;
                for (int j = 0; j < n; j++) {
                    float term = P[(size_t)i * n + j] * xh[j];
                    acc = acc + term;
                }
                size_t a = (size_t)i * (size_t)d + (size_t)e;
                x[a] = acc;
                z16[a] = sgpo_float_to_bf16(acc / w_new[i]);
            }
        }
        free(xh);
    }
    for (int i = 0; i < n; i++) w[i] = w_new[i];
    free(w_new);
    return 0;
}
