/* Driver for the host-sanitizer build of the C oracle: small forward and backward problems for the
 * three solver branches (sort-based alpha = 1.5 and 2, bisection otherwise), causal and not.  The
 * sanitizers abort on any invalid access or undefined operation; the driver itself only checks
 * that every row of P sums to one. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_entmax_attn_fwd(const double* Q, const double* K, const double* V, int B, int H, int N, int d, double alpha,
                           int causal, int tile, double* O, double* tau, double* margin, double* P);
int oracle_entmax_attn_bwd(const double* Q, const double* K, const double* V, const double* dO, int B, int H, int N, int d,
                           double alpha, int causal, double* dQ, double* dK, double* dV, double* delta);

static double rnd(unsigned* s) { *s = *s * 1664525u + 1013904223u; return ((*s >> 8) / 16777216.0) * 4.0 - 2.0; }

int main(void) {
    const int B = 1, H = 2, N = 128, d = 16, tile = 64, T = N / tile;
    const size_t n = (size_t)B * H * N * d;
    double *Q = malloc(n * 8), *K = malloc(n * 8), *V = malloc(n * 8), *G = malloc(n * 8), *O = malloc(n * 8);
    double *dQ = malloc(n * 8), *dK = malloc(n * 8), *dV = malloc(n * 8);
    double *tau = malloc((size_t)B * H * N * 8), *delta = malloc((size_t)B * H * N * 8);
    double *margin = malloc((size_t)B * H * T * T * 8), *P = malloc((size_t)B * H * N * N * 8);
    unsigned s = 12345u;
    for (size_t i = 0; i < n; ++i) { Q[i] = rnd(&s); K[i] = rnd(&s); V[i] = rnd(&s); G[i] = rnd(&s); }
    const double alphas[3] = {1.5, 2.0, 1.25};
    for (int a = 0; a < 3; ++a)
        for (int causal = 0; causal < 2; ++causal) {
            if (oracle_entmax_attn_fwd(Q, K, V, B, H, N, d, alphas[a], causal, tile, O, tau, margin, P)) return 2;
            if (oracle_entmax_attn_bwd(Q, K, V, G, B, H, N, d, alphas[a], causal, dQ, dK, dV, delta)) return 3;
            for (int r = 0; r < B * H * N; ++r) {
                double sum = 0;
                for (int j = 0; j < N; ++j) sum += P[(size_t)r * N + j];
                if (fabs(sum - 1.0) > 1e-9) { printf("row %d sums to %.12f\n", r, sum); return 4; }
            }
        }
    free(Q); free(K); free(V); free(G); free(O); free(dQ); free(dK); free(dV); free(tau); free(delta); free(margin); free(P);
    printf("ok\n");
    return 0;
}
