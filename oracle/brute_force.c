/* Scalar triple-loop attention, forward and gradients, for tiny shapes.
 *
 * TEST INFRASTRUCTURE ONLY: an independent pin for the numpy oracle.  Every sum of the
 * textbook definition (see attention_ref.py for the formulas and the passages of the
 * paper they follow) is written out as a scalar loop; nothing is vectorised, tiled or
 * reordered.  One (batch, head) slice per call; all arrays are fp64, row-major [S, D].
 */
#include <math.h>
#include <stdlib.h>

int brute_attn_fwd(const double* q, const double* k, const double* v, double* o, double* lse,
                   int S, int D, double scale, int causal) {
    for (int i = 0; i < S; i++) {
        int last = causal ? i : S - 1;
        double m = -INFINITY;
        for (int j = 0; j <= last; j++) {
            double s = 0.0;
            for (int d = 0; d < D; d++) s += q[i * D + d] * k[j * D + d];
            s *= scale;
            if (s > m) m = s;
        }
        double z = 0.0;
        for (int j = 0; j <= last; j++) {
            double s = 0.0;
            for (int d = 0; d < D; d++) s += q[i * D + d] * k[j * D + d];
            z += exp(s * scale - m);
        }
        lse[i] = m + log(z);
        for (int d = 0; d < D; d++) o[i * D + d] = 0.0;
        for (int j = 0; j <= last; j++) {
            double s = 0.0;
            for (int d = 0; d < D; d++) s += q[i * D + d] * k[j * D + d];
            double p = exp(s * scale - lse[i]);
            for (int d = 0; d < D; d++) o[i * D + d] += p * v[j * D + d];
        }
    }
    return 0;
}

int brute_attn_bwd(const double* q, const double* k, const double* v, const double* g,
                   double* dq, double* dk, double* dv, int S, int D, double scale, int causal) {
    double* o = (double*)malloc(sizeof(double) * S * D);
    double* lse = (double*)malloc(sizeof(double) * S);
    if (!o || !lse) { free(o); free(lse); return 1; }
    brute_attn_fwd(q, k, v, o, lse, S, D, scale, causal);
    for (int n = 0; n < S * D; n++) { dq[n] = 0.0; dk[n] = 0.0; dv[n] = 0.0; }
    for (int i = 0; i < S; i++) {
        int last = causal ? i : S - 1;
        /* delta_i = sum_j p_ij dp_ij */
        double delta = 0.0;
        for (int j = 0; j <= last; j++) {
            double s = 0.0, dp = 0.0;
            for (int d = 0; d < D; d++) { s += q[i * D + d] * k[j * D + d]; dp += g[i * D + d] * v[j * D + d]; }
            delta += exp(s * scale - lse[i]) * dp;
        }
        for (int j = 0; j <= last; j++) {
            double s = 0.0, dp = 0.0;
            for (int d = 0; d < D; d++) { s += q[i * D + d] * k[j * D + d]; dp += g[i * D + d] * v[j * D + d]; }
            double p = exp(s * scale - lse[i]);
            double ds = p * (dp - delta);
            for (int d = 0; d < D; d++) {
                dv[j * D + d] += p * g[i * D + d];
                dq[i * D + d] += scale * ds * k[j * D + d];
                dk[j * D + d] += scale * ds * q[i * D + d];
            }
        }
    }
    free(o); free(lse);
    return 0;
}
