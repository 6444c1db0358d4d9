/* Plain C twin of the MoE block oracle: scalar loops in double, nothing else.
 * Test infrastructure only; shares nothing with the HIP path.
 *
 * Block as in Sec. 2.3 of the paper: a router sends each token to its top-k of E
 * experts, each expert is a two-layer MLP (here gate/up projections, SiLU(gate)*up,
 * down projection), and the k outputs are summed with the renormalised router
 * weights.  Selection is on the logits, descending, first index wins among equals.
 *
 * Layouts (row-major doubles): x[T][H], wr[E][H], b[E], wg[E][I][H], wu[E][I][H],
 * wd[E][H][I].  Outputs: idx[T][k], w[T][k], counts[E], perm[T*k], inv_perm[T*k],
 * out[T][H].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

void brute_moe_layer(int T, int H, int E, int k, int I, const double *x, const double *wr,
                     const double *b, const double *wg, const double *wu, const double *wd,
                     int32_t *idx, double *w, int32_t *counts, int32_t *perm, int32_t *inv_perm,
                     double *out)
{
    double *l = malloc(sizeof(double) * E);
    double *p = malloc(sizeof(double) * E);
    char *taken = malloc(E);
    double *a = malloc(sizeof(double) * I);
    for (int t = 0; t < T; ++t) {
        const double *xt = x + (size_t)t * H;
        for (int e = 0; e < E; ++e) {
            double s = 0.0;
            for (int h = 0; h < H; ++h) s += xt[h] * wr[(size_t)e * H + h];
            l[e] = s + b[e];
            taken[e] = 0;
        }
        double m = l[0];
        for (int e = 1; e < E; ++e) if (l[e] > m) m = l[e];
        double z = 0.0;
        for (int e = 0; e < E; ++e) { p[e] = exp(l[e] - m); z += p[e]; }
        for (int e = 0; e < E; ++e) p[e] /= z;
        double zs = 0.0;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e;
            }
            taken[best] = 1;
            idx[t * k + j] = best;
            zs += p[best];
        }
        for (int j = 0; j < k; ++j) w[t * k + j] = p[idx[t * k + j]] / zs;
        for (int h = 0; h < H; ++h) out[(size_t)t * H + h] = 0.0;
        for (int j = 0; j < k; ++j) {
            int e = idx[t * k + j];
            const double *g_w = wg + (size_t)e * I * H;
            const double *u_w = wu + (size_t)e * I * H;
            const double *d_w = wd + (size_t)e * H * I;
            for (int i = 0; i < I; ++i) {
                double g = 0.0, u = 0.0;
                for (int h = 0; h < H; ++h) {
                    g += g_w[(size_t)i * H + h] * xt[h];
                    u += u_w[(size_t)i * H + h] * xt[h];
                }
                a[i] = g / (1.0 + exp(-g)) * u;
            }
            for (int h = 0; h < H; ++h) {
                double y = 0.0;
                for (int i = 0; i < I; ++i) y += d_w[(size_t)h * I + i] * a[i];
                out[(size_t)t * H + h] += w[t * k + j] * y;
            }
        }
    }
    /* counting sort of the flat ids by expert, in flat-id order (stable) */
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int f = 0; f < T * k; ++f) counts[idx[f]]++;
    int32_t *cur = malloc(sizeof(int32_t) * E);
    int32_t run = 0;
    for (int e = 0; e < E; ++e) { cur[e] = run; run += counts[e]; }
    for (int f = 0; f < T * k; ++f) {
        int e = idx[f];
        perm[cur[e]] = f;
        inv_perm[f] = cur[e];
        cur[e]++;
    }
    free(cur); free(l); free(p); free(taken); free(a);
}
