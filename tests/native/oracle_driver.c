/* Test driver: the fp64 convolution oracle (conv_oracle.c) as a plain executable, so that it can
 * be built with -fsanitize=address,undefined.  Reads "N C H W K R S sh sw ph pw nidx" and the path
 * of a raw file of doubles (x, w, dy, then nidx int64 indices for each of the three sampled forms)
 * from argv, runs the three operations in full and at the sampled indices, and writes the results
 * (y, dx, dw, y_at, dx_at, dw_at) to the output path as raw doubles. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct { int64_t N, C, H, W, K, R, S, sh, sw, ph, pw; } oc_layer;
void oc_conv_fwd(const oc_layer *L, const double *x, const double *w, double *y);
void oc_conv_bwd_data(const oc_layer *L, const double *dy, const double *w, double *dx);
void oc_conv_bwd_filter(const oc_layer *L, const double *x, const double *dy, double beta, double *dw);
void oc_conv_fwd_at(const oc_layer *L, const double *x, const double *w, const int64_t *idx, int64_t n, double *out);
void oc_conv_bwd_data_at(const oc_layer *L, const double *dy, const double *w, const int64_t *idx, int64_t n, double *out);
void oc_conv_bwd_filter_at(const oc_layer *L, const double *x, const double *dy, const int64_t *idx, int64_t n, double *out);

int main(int argc, char **argv)
{
    if (argc != 15) return 2;
    oc_layer L;
    int64_t *f = (int64_t *)&L;
    for (int i = 0; i < 11; ++i) f[i] = atoll(argv[1 + i]);
    const int64_t nidx = atoll(argv[12]);
    const int64_t P = (L.H + 2 * L.ph - L.R) / L.sh + 1, Q = (L.W + 2 * L.pw - L.S) / L.sw + 1;
    const int64_t nx = L.N * L.C * L.H * L.W, nw = L.K * L.C * L.R * L.S, ny = L.N * L.K * P * Q;
    double *x = malloc(sizeof(double) * nx), *w = malloc(sizeof(double) * nw), *dy = malloc(sizeof(double) * ny);
    int64_t *idx = malloc(sizeof(int64_t) * 3 * nidx);
    double *y = malloc(sizeof(double) * ny), *dx = malloc(sizeof(double) * nx), *dw = calloc(nw, sizeof(double));
    double *at = malloc(sizeof(double) * 3 * nidx);
    FILE *in = fopen(argv[13], "rb");
    if (!in || !x || !w || !dy || !idx || !y || !dx || !dw || !at) return 3;
    if (fread(x, sizeof(double), nx, in) != (size_t)nx || fread(w, sizeof(double), nw, in) != (size_t)nw ||
        fread(dy, sizeof(double), ny, in) != (size_t)ny || fread(idx, sizeof(int64_t), 3 * nidx, in) != (size_t)(3 * nidx))
        return 4;
    fclose(in);
    oc_conv_fwd(&L, x, w, y);
    oc_conv_bwd_data(&L, dy, w, dx);
    oc_conv_bwd_filter(&L, x, dy, 0.0, dw);
    oc_conv_fwd_at(&L, x, w, idx, nidx, at);
    oc_conv_bwd_data_at(&L, dy, w, idx + nidx, nidx, at + nidx);
    oc_conv_bwd_filter_at(&L, x, dy, idx + 2 * nidx, nidx, at + 2 * nidx);
    FILE *out = fopen(argv[14], "wb");
    if (!out) return 5;
    fwrite(y, sizeof(double), ny, out);
    fwrite(dx, sizeof(double), nx, out);
    fwrite(dw, sizeof(double), nw, out);
    fwrite(at, sizeof(double), 3 * nidx, out);
    fclose(out);
    free(x); free(w); free(dy); free(idx); free(y); free(dx); free(dw); free(at);
    return 0;
}
