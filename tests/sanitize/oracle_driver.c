/* Driver for the sanitizer build of the oracle (tests/test_oracle_sanitized.py): runs every entry point of
 * oracle/conv_oracle.c on heap buffers of exactly the required sizes - ragged shapes, strides with a floor
 * remainder, padding larger than the filter - so that AddressSanitizer sees any index past a tensor and
 * UndefinedBehaviorSanitizer any overflow, and cross-checks the scatter nests against the gather evaluators
 * and the printed hand example.  Exit status 0 = clean and consistent. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef int64_t i64;
int orc_out_dim(int in, int filt, int stride, int pad);
void orc_conv2d_fwd(int, int, int, int, int, int, int, int, int, const float *, const float *, double *);
void orc_conv2d_bwd_data(int, int, int, int, int, int, int, int, int, const float *, const float *, double *);
void orc_conv2d_bwd_weight(int, int, int, int, int, int, int, int, int, const float *, const float *, double *);
void orc_conv2d_fwd_at(int, int, int, int, int, int, int, int, int, const float *, const float *, i64, const i64 *, double *, double *);
void orc_conv2d_bwd_data_at(int, int, int, int, int, int, int, int, int, const float *, const float *, i64, const i64 *, double *, double *);
void orc_conv2d_bwd_weight_at(int, int, int, int, int, int, int, int, int, const float *, const float *, i64, const i64 *, double *, double *);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static float rnd(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (float)((double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static float *filled(size_t n)
{
    float *p = malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}

static int check_all(i64 n, const double *full, const double *val, const double *den, const char *what)
{
    for (i64 i = 0; i < n; ++i) {
        if (fabs(full[i] - val[i]) > 1e-12 * (den[i] + 1e-300) || fabs(val[i]) > den[i] * (1 + 1e-12)) {
            fprintf(stderr, "%s mismatch at %lld: %g vs %g (D %g)\n", what, (long long)i, full[i], val[i], den[i]);
            return 1;
        }
    }
    return 0;
}

static int one_case(int N, int C, int H, int W, int K, int R, int S, int stride, int pad)
{
    const int P = orc_out_dim(H, R, stride, pad), Q = orc_out_dim(W, S, stride, pad);
    const size_t nx = (size_t)N * C * H * W, nw = (size_t)K * C * R * S, ny = (size_t)N * K * P * Q;
    float *x = filled(nx), *w = filled(nw), *dy = filled(ny);
    double *y = malloc(ny * sizeof(double)), *dx = malloc(nx * sizeof(double)), *dw = malloc(nw * sizeof(double));
    const size_t nmax = nx > ny ? (nx > nw ? nx : nw) : (ny > nw ? ny : nw);
    i64 *idx = malloc(nmax * sizeof(i64));
    double *val = malloc(nmax * sizeof(double)), *den = malloc(nmax * sizeof(double));
    for (size_t i = 0; i < nmax; ++i) idx[i] = (i64)i;
    int bad = 0;
    orc_conv2d_fwd(N, C, H, W, K, R, S, stride, pad, x, w, y);
    orc_conv2d_fwd_at(N, C, H, W, K, R, S, stride, pad, x, w, (i64)ny, idx, val, den);
    bad |= check_all((i64)ny, y, val, den, "fwd");
    orc_conv2d_bwd_data(N, C, H, W, K, R, S, stride, pad, dy, w, dx);
    orc_conv2d_bwd_data_at(N, C, H, W, K, R, S, stride, pad, dy, w, (i64)nx, idx, val, den);
    bad |= check_all((i64)nx, dx, val, den, "bwd_data");
    orc_conv2d_bwd_weight(N, C, H, W, K, R, S, stride, pad, x, dy, dw);
    orc_conv2d_bwd_weight_at(N, C, H, W, K, R, S, stride, pad, x, dy, (i64)nw, idx, val, den);
    bad |= check_all((i64)nw, dw, val, den, "bwd_weight");
    /* adjoint identity <fwd(x,w),dy> = <x,bwd_data(dy,w)> = <w,bwd_weight(x,dy)> */
    double a = 0, b = 0, c = 0;
    for (size_t i = 0; i < ny; ++i) a += y[i] * dy[i];
    for (size_t i = 0; i < nx; ++i) b += dx[i] * x[i];
    for (size_t i = 0; i < nw; ++i) c += dw[i] * w[i];
    if (fabs(a - b) > 1e-9 * (fabs(a) + 1) || fabs(a - c) > 1e-9 * (fabs(a) + 1)) {
        fprintf(stderr, "adjoint identity fails: %g %g %g\n", a, b, c);
        bad = 1;
    }
    free(x); free(w); free(dy); free(y); free(dx); free(dw); free(idx); free(val); free(den);
    return bad;
}

int main(void)
{
    int bad = 0;
    /* the hand example: x = 1..9 (3x3), w = [[1,0],[0,-1]] -> y = -4 everywhere */
    {
        const float x[9] = {1, 2, 3, 4, 5, 6, 7, 8, 9}, w[4] = {1, 0, 0, -1};
        double y[4];
        orc_conv2d_fwd(1, 1, 3, 3, 1, 2, 2, 1, 0, x, w, y);
        for (int i = 0; i < 4; ++i) bad |= y[i] != -4.0;
    }
    bad |= one_case(2, 3, 9, 7, 5, 3, 3, 1, 1);
    bad |= one_case(1, 3, 35, 33, 4, 11, 11, 4, 2);   /* floor remainder */
    bad |= one_case(2, 4, 9, 9, 6, 1, 1, 2, 0);       /* positions no tap reaches */
    bad |= one_case(1, 2, 4, 5, 3, 1, 1, 1, 2);       /* pad beyond the filter */
    bad |= one_case(1, 1, 1, 1, 1, 1, 1, 1, 0);
    bad |= one_case(3, 5, 8, 6, 7, 3, 2, 3, 1);       /* R != S, stride 3 */
    if (!bad) puts("oracle sanitizer run: clean and consistent");
    return bad;
}
