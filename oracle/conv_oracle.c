/*
 * TEST INFRASTRUCTURE ONLY.  fp64 CPU oracle for the convolution layer of the
 * micro-batched convolution method (arXiv 1804.04806).  Nothing in the product
 * path may call into this file; it shares no code with the HIP kernels.
 *
 * What it computes is the plain definition:
 *   Forward        : the seven-loop 2-D convolution of Algorithm 1 (Section 2),
 *                    read as cross-correlation (no filter flip) with zero
 *                    padding and a general stride; the listing itself has
 *                    neither stride nor padding.
 *   BackwardData   : the adjoint of Forward with respect to X ("neuron errors",
 *                    Section 2).
 *   BackwardFilter : the parameter-gradient sum over samples of Section 2's
 *                    gradient equation, WITHOUT the 1/N factor (that belongs to
 *                    the loss), added onto beta * dW so that micro-batches can
 *                    accumulate with output scale 1 (Section 2, last paragraph).
 *
 * Layouts: X (N,C,H,W), W (K,C,R,S) with R the filter height and S its width,
 * Y (N,K,P,Q), all dense row-major, P = floor((H+2*ph-R)/sh)+1, Q likewise.
 * Everything is double; callers widen the fp32 bits the GPU gets.
 * Loops are threaded over independent output slices only (OpenMP); every output
 * element is one sequential fp64 sum in the loop order of Algorithm 1.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t N, C, H, W, K, R, S, sh, sw, ph, pw;
} oc_layer;

int64_t oc_out_h(const oc_layer *L) { return (L->H + 2 * L->ph - L->R) / L->sh + 1; }
int64_t oc_out_w(const oc_layer *L) { return (L->W + 2 * L->pw - L->S) / L->sw + 1; }

int oc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* one output element of Forward: sum over c, r, s (Algorithm 1, inner three loops) */
static double fwd_elem(const oc_layer *L, const double *x, const double *w,
                       int64_t n, int64_t k, int64_t p, int64_t q)
{
    double acc = 0.0;
    for (int64_t c = 0; c < L->C; ++c)
        for (int64_t r = 0; r < L->R; ++r)
            for (int64_t s = 0; s < L->S; ++s) {
                int64_t h = p * L->sh - L->ph + r;
                int64_t v = q * L->sw - L->pw + s;
                if (h < 0 || h >= L->H || v < 0 || v >= L->W) continue; /* zero padding */
                acc += w[((k * L->C + c) * L->R + r) * L->S + s] *
                       x[((n * L->C + c) * L->H + h) * L->W + v];
            }
    return acc;
}

/* one element of BackwardData: every (k, r, s) whose tap lands on input pixel (h, v) */
static double bwd_data_elem(const oc_layer *L, const double *dy, const double *w,
                            int64_t n, int64_t c, int64_t h, int64_t v)
{
    const int64_t P = oc_out_h(L), Q = oc_out_w(L);
    double acc = 0.0;
    for (int64_t k = 0; k < L->K; ++k)
        for (int64_t r = 0; r < L->R; ++r)
            for (int64_t s = 0; s < L->S; ++s) {
                int64_t hp = h + L->ph - r, vq = v + L->pw - s;
                if (hp < 0 || vq < 0 || hp % L->sh != 0 || vq % L->sw != 0) continue;
                int64_t p = hp / L->sh, q = vq / L->sw;
                if (p >= P || q >= Q) continue;
                acc += dy[((n * L->K + k) * P + p) * Q + q] *
                       w[((k * L->C + c) * L->R + r) * L->S + s];
            }
    return acc;
}

/* one element of the BackwardFilter sum over n, p, q (no beta term) */
static double bwd_filter_elem(const oc_layer *L, const double *x, const double *dy,
                              int64_t k, int64_t c, int64_t r, int64_t s)
{
    const int64_t P = oc_out_h(L), Q = oc_out_w(L);
    double acc = 0.0;
    for (int64_t n = 0; n < L->N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q) {
                int64_t h = p * L->sh - L->ph + r;
                int64_t v = q * L->sw - L->pw + s;
                if (h < 0 || h >= L->H || v < 0 || v >= L->W) continue;
                acc += dy[((n * L->K + k) * P + p) * Q + q] *
                       x[((n * L->C + c) * L->H + h) * L->W + v];
            }
    return acc;
}

void oc_conv_fwd(const oc_layer *L, const double *x, const double *w, double *y)
{
    const int64_t P = oc_out_h(L), Q = oc_out_w(L);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < L->N; ++n)
        for (int64_t k = 0; k < L->K; ++k)
            for (int64_t p = 0; p < P; ++p)
                for (int64_t q = 0; q < Q; ++q)
                    y[((n * L->K + k) * P + p) * Q + q] = fwd_elem(L, x, w, n, k, p, q);
}

void oc_conv_bwd_data(const oc_layer *L, const double *dy, const double *w, double *dx)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < L->N; ++n)
        for (int64_t c = 0; c < L->C; ++c)
            for (int64_t h = 0; h < L->H; ++h)
                for (int64_t v = 0; v < L->W; ++v)
                    dx[((n * L->C + c) * L->H + h) * L->W + v] = bwd_data_elem(L, dy, w, n, c, h, v);
}

void oc_conv_bwd_filter(const oc_layer *L, const double *x, const double *dy, double beta, double *dw)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t k = 0; k < L->K; ++k)
        for (int64_t c = 0; c < L->C; ++c)
            for (int64_t r = 0; r < L->R; ++r)
                for (int64_t s = 0; s < L->S; ++s) {
                    int64_t i = ((k * L->C + c) * L->R + r) * L->S + s;
                    double old = (beta == 0.0) ? 0.0 : beta * dw[i]; /* beta 0 ignores old contents */
                    dw[i] = old + bwd_filter_elem(L, x, dy, k, c, r, s);
                }
}

/*
 * Sampled forms for layers too large to run whole: out[i] is the full, exact
 * reduction for the output element with flat index idx[i].
 */
void oc_conv_fwd_at(const oc_layer *L, const double *x, const double *w,
                    const int64_t *idx, int64_t n_idx, double *out)
{
    const int64_t P = oc_out_h(L), Q = oc_out_w(L);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t t = idx[i];
        int64_t q = t % Q; t /= Q;
        int64_t p = t % P; t /= P;
        int64_t k = t % L->K; t /= L->K;
        out[i] = fwd_elem(L, x, w, t, k, p, q);
    }
}

void oc_conv_bwd_data_at(const oc_layer *L, const double *dy, const double *w,
                         const int64_t *idx, int64_t n_idx, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t t = idx[i];
        int64_t v = t % L->W; t /= L->W;
        int64_t h = t % L->H; t /= L->H;
        int64_t c = t % L->C; t /= L->C;
        out[i] = bwd_data_elem(L, dy, w, t, c, h, v);
    }
}

void oc_conv_bwd_filter_at(const oc_layer *L, const double *x, const double *dy,
                           const int64_t *idx, int64_t n_idx, double *out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t t = idx[i];
        int64_t s = t % L->S; t /= L->S;
        int64_t r = t % L->R; t /= L->R;
        int64_t c = t % L->C; t /= L->C;
        out[i] = bwd_filter_elem(L, x, dy, t, c, r, s);
    }
}
