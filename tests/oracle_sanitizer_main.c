/*
 * Sanitizer driver for the CPU oracle (test infrastructure).  Built together
 * with oracle/conv_oracle.c under -fsanitize=address,undefined: every tensor is
 * a heap block of exactly its size, so an access outside a tensor, a signed
 * overflow in the index arithmetic or a misaligned access stops the run.  The
 * checks themselves are closed forms and identities of the definitions (they
 * repeat, in C, a few of the pins of tests/test_oracle_pins.py so that the
 * sanitised code is known to compute the same thing).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_conv_fwd(const double *, const double *, double *, int, int, int, int, int, int, int, int, int);
void oracle_conv_bwd_data(const double *, const double *, double *, int, int, int, int, int, int, int, int, int);
void oracle_conv_bwd_filter(const double *, const double *, double *, int, int, int, int, int, int, int, int, int);
void oracle_conv_fwd_at(const double *, const double *, int, int, int, int, int, int, int, int, int,
                        const int64_t *, int64_t, double *);
void oracle_conv_bwd_data_at(const double *, const double *, int, int, int, int, int, int, int, int, int,
                             const int64_t *, int64_t, double *);
void oracle_conv_bwd_filter_at(const double *, const double *, int, int, int, int, int, int, int, int, int,
                               const int64_t *, int64_t, double *);
void oracle_relu_fwd(const double *, double *, int64_t);
void oracle_relu_bwd(const double *, const double *, double *, int64_t);
void oracle_maxpool3x3s2_fwd(const double *, double *, int32_t *, int64_t, int, int);
void oracle_maxpool3x3s2_bwd(const double *, const double *, double *, int64_t, int, int);
void oracle_round_bf16(const uint32_t *, uint16_t *, int64_t);
int oracle_out_extent(int, int, int, int);
int oracle_pool_extent(int);

static int fails = 0;
#define CHECK(c) do { if (!(c)) { printf("FAIL line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

static double *alloc(size_t n) { double *p = malloc(n * sizeof(double)); if (!p) abort(); return p; }

/* small integers from a linear congruential sequence: every sum below is exact in double */
static uint32_t lcg_state = 12345u;
static double small_int(void)
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (double)((int)((lcg_state >> 16) % 9u) - 4);
}

static void fill(double *p, size_t n) { for (size_t i = 0; i < n; ++i) p[i] = small_int(); }

static double dot(const double *a, const double *b, size_t n)
{
    double s = 0.0;
    for (size_t i = 0; i < n; ++i) s += a[i] * b[i];
    return s;
}

/* <conv(x,w),g> = <x,dgrad(g,w)> = <w,wgrad(x,g)>, the element-wise entry points against the full ones */
static void identities(int N, int C, int H, int W, int K, int R, int S, int st, int pad)
{
    const int P = oracle_out_extent(H, R, st, pad), Q = oracle_out_extent(W, S, st, pad);
    CHECK(P > 0 && Q > 0);
    const size_t nx = (size_t)N * C * H * W, nw = (size_t)K * C * R * S, ny = (size_t)N * K * P * Q;
    double *x = alloc(nx), *w = alloc(nw), *g = alloc(ny), *y = alloc(ny), *dx = alloc(nx), *dw = alloc(nw);
    fill(x, nx); fill(w, nw); fill(g, ny);
    oracle_conv_fwd(x, w, y, N, C, H, W, K, R, S, st, pad);
    oracle_conv_bwd_data(g, w, dx, N, C, H, W, K, R, S, st, pad);
    oracle_conv_bwd_filter(x, g, dw, N, C, H, W, K, R, S, st, pad);
    const double a = dot(y, g, ny);
    CHECK(a == dot(x, dx, nx));
    CHECK(a == dot(w, dw, nw));
    size_t nmax = nx > ny ? nx : ny;
    if (nw > nmax) nmax = nw;
    int64_t *idx = malloc(nmax * sizeof(int64_t));
    double *out = alloc(nmax);
    for (size_t i = 0; i < nmax; ++i) idx[i] = (int64_t)i;
    oracle_conv_fwd_at(x, w, N, C, H, W, K, R, S, st, pad, idx, (int64_t)ny, out);
    for (size_t i = 0; i < ny; ++i) CHECK(out[i] == y[i]);
    oracle_conv_bwd_data_at(g, w, N, C, H, W, K, R, S, st, pad, idx, (int64_t)nx, out);
    for (size_t i = 0; i < nx; ++i) CHECK(out[i] == dx[i]);
    oracle_conv_bwd_filter_at(x, g, N, C, H, W, K, R, S, st, pad, idx, (int64_t)nw, out);
    for (size_t i = 0; i < nw; ++i) CHECK(out[i] == dw[i]);
    free(x); free(w); free(g); free(y); free(dx); free(dw); free(idx); free(out);
}

/* all-ones input and filter: every output counts the taps that fall inside the input */
static void all_ones(int N, int C, int H, int W, int K, int R, int S, int st, int pad)
{
    const int P = oracle_out_extent(H, R, st, pad), Q = oracle_out_extent(W, S, st, pad);
    const size_t nx = (size_t)N * C * H * W, nw = (size_t)K * C * R * S, ny = (size_t)N * K * P * Q;
    double *x = alloc(nx), *w = alloc(nw), *y = alloc(ny);
    for (size_t i = 0; i < nx; ++i) x[i] = 1.0;
    for (size_t i = 0; i < nw; ++i) w[i] = 1.0;
    oracle_conv_fwd(x, w, y, N, C, H, W, K, R, S, st, pad);
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    int rows = 0, cols = 0;
                    for (int r = 0; r < R; ++r) rows += (p * st - pad + r >= 0 && p * st - pad + r < H);
                    for (int s = 0; s < S; ++s) cols += (q * st - pad + s >= 0 && q * st - pad + s < W);
                    CHECK(y[(((size_t)n * K + k) * P + p) * Q + q] == (double)(C * rows * cols));
                }
    free(x); free(w); free(y);
}

int main(void)
{
    /* the hand-worked 3x3 example (tests/golden): stride 1 without padding, stride 2 with padding 1 */
    {
        const double x[9] = {1, 2, 3, 4, 5, 6, 7, 8, 9}, w[4] = {1, 2, 3, 4}, dy[4] = {1, 2, 3, 4};
        double *xh = alloc(9), *wh = alloc(4), *gh = alloc(4), *y = alloc(4), *dx = alloc(9), *dw = alloc(4);
        for (int i = 0; i < 9; ++i) xh[i] = x[i];
        for (int i = 0; i < 4; ++i) { wh[i] = w[i]; gh[i] = dy[i]; }
        oracle_conv_fwd(xh, wh, y, 1, 1, 3, 3, 1, 2, 2, 1, 0);
        CHECK(y[0] == 37 && y[1] == 47 && y[2] == 67 && y[3] == 77);
        oracle_conv_bwd_data(gh, wh, dx, 1, 1, 3, 3, 1, 2, 2, 1, 0);
        const double dx_want[9] = {1, 4, 4, 6, 20, 16, 9, 24, 16};
        for (int i = 0; i < 9; ++i) CHECK(dx[i] == dx_want[i]);
        oracle_conv_bwd_filter(xh, gh, dw, 1, 1, 3, 3, 1, 2, 2, 1, 0);
        CHECK(dw[0] == 37 && dw[1] == 47 && dw[2] == 67 && dw[3] == 77);
        CHECK(oracle_out_extent(3, 2, 2, 1) == 2);
        oracle_conv_fwd(xh, wh, y, 1, 1, 3, 3, 1, 2, 2, 2, 1);
        CHECK(y[0] == 4 && y[1] == 18 && y[2] == 36 && y[3] == 77);
        free(xh); free(wh); free(gh); free(y); free(dx); free(dw);
    }
    CHECK(oracle_out_extent(224, 11, 4, 2) == 55 && oracle_out_extent(27, 5, 1, 2) == 27);
    CHECK(oracle_out_extent(2, 5, 1, 1) == 0);
    /* shapes with padding beyond the filter, strides that leave input rows unread, 1x1 outputs, thin planes */
    identities(2, 3, 7, 9, 4, 3, 3, 1, 1);
    identities(1, 2, 12, 11, 3, 5, 5, 2, 2);
    identities(2, 1, 23, 25, 2, 11, 11, 4, 2);
    identities(1, 2, 9, 9, 2, 9, 9, 1, 0);
    identities(2, 2, 8, 10, 3, 3, 3, 1, 5);
    identities(1, 2, 30, 5, 2, 4, 1, 4, 0);
    identities(3, 1, 1, 1, 2, 1, 1, 1, 0);
    all_ones(1, 3, 9, 7, 2, 3, 5, 2, 2);
    all_ones(2, 1, 13, 13, 1, 11, 11, 4, 2);
    /* glue: ReLU, pooling on the smallest plane and on a plane whose last row / column no window covers */
    {
        const int HW[3][2] = {{3, 3}, {8, 5}, {13, 13}};
        for (int t = 0; t < 3; ++t) {
            const int H = HW[t][0], W = HW[t][1], planes = 3;
            const int PH = oracle_pool_extent(H), PW = oracle_pool_extent(W);
            CHECK(PH == (H - 3) / 2 + 1 && PW == (W - 3) / 2 + 1);
            const size_t nx = (size_t)planes * H * W, ny = (size_t)planes * PH * PW;
            double *x = alloc(nx), *y = alloc(ny), *g = alloc(ny), *dx = alloc(nx), *r = alloc(nx);
            int32_t *arg = malloc(ny * sizeof(int32_t));
            fill(x, nx); fill(g, ny);
            oracle_maxpool3x3s2_fwd(x, y, arg, planes, H, W);
            oracle_maxpool3x3s2_bwd(x, g, dx, planes, H, W);
            double sg = 0.0, sdx = 0.0;
            for (size_t i = 0; i < ny; ++i) {
                const size_t pl = i / ((size_t)PH * PW);
                CHECK(arg[i] >= 0 && arg[i] < H * W && x[pl * H * W + arg[i]] == y[i]);
                sg += g[i];
            }
            for (size_t i = 0; i < nx; ++i) sdx += dx[i];
            CHECK(sg == sdx);                      /* every gradient lands on exactly one element */
            oracle_relu_fwd(x, r, (int64_t)nx);
            for (size_t i = 0; i < nx; ++i) CHECK(r[i] == (x[i] > 0 ? x[i] : 0.0));
            oracle_relu_bwd(x, x, r, (int64_t)nx);
            for (size_t i = 0; i < nx; ++i) CHECK(r[i] == (x[i] > 0 ? x[i] : 0.0));
            free(x); free(y); free(g); free(dx); free(r); free(arg);
        }
    }
    /* bfloat16 rounding: ties both ways, carry into the exponent, overflow, NaN */
    {
        const uint32_t in[8] = {0x3F800000u, 0x3F808000u, 0x3F818000u, 0x3FFFFFFFu, 0x7F7FFFFFu, 0x80000000u,
                                0x7F800001u, 0x00008001u};
        const uint16_t want[8] = {0x3F80, 0x3F80, 0x3F82, 0x4000, 0x7F80, 0x8000, 0x7FC0, 0x0001};
        uint32_t *b = malloc(sizeof(in));
        uint16_t *o = malloc(sizeof(want));
        for (int i = 0; i < 8; ++i) b[i] = in[i];
        oracle_round_bf16(b, o, 8);
        for (int i = 0; i < 8; ++i) CHECK(o[i] == want[i]);
        free(b); free(o);
    }
    printf("oracle sanitizer run: %d failures\n", fails);
    return fails ? 1 : 0;
}
