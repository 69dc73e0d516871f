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
