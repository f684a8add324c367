/*
 * CPU oracle for the convolutional hot path of synchronous-SGD ConvNet training
 * ("Multi-GPU Training of ConvNets", arXiv 1312.5853).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a slow, literal,
 * direct-loop evaluation of what a convolutional layer computes, kept
 * deliberately free of blocking, fusion or reordering so that it can be
 * checked against the definitions by eye.  It shares no source, header,
 * helper or constant with the HIP library; only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.
 *
 * The paper itself prints no formula: it speaks of a convolutional layer
 * whose filters are applied to the layer input by convolution
 * (model-parallelism paragraph, where a layer's filters are split into two
 * halves) and of training by ordinary supervised back-propagation, each GPU
 * computing the gradients of every model parameter on its samples
 * (optimisation and data-parallelism paragraphs).  The definitions below are
 * the standard ones those statements denote, in the NCHW / KCRS layout with
 * one stride and one symmetric zero padding for both axes:
 *
 *   P = floor((H + 2*pad - R) / stride) + 1,   Q likewise from W and S
 *
 *   forward          y[n,k,p,q]  = sum_{c,r,s} x[n,c,p*st-pad+r,q*st-pad+s] * w[k,c,r,s]
 *   backward-data    dx[n,c,h,w] = sum over (k,p,q,r,s) with p*st-pad+r = h and
 *                                  q*st-pad+s = w of dy[n,k,p,q] * w[k,c,r,s]
 *   backward-filter  dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*st-pad+r,q*st-pad+s]
 *
 * with x read as zero outside 0 <= h < H, 0 <= w < W, and no filter flip
 * (cross-correlation).  All arithmetic is IEEE double; callers widen fp32 or
 * bf16 test data to double exactly before the call.
 *
 * Parity pins (tests/test_oracle_pins.py): all-ones closed form, delta
 * filter / delta input, brute force in a different loop order on small
 * integers, the three-way adjoint identity, exact finite differences of the
 * bilinear form, reduction to a matrix product (1x1) and to a dot product
 * (R=H,S=W), stride-s == subsampled stride-1, linearity, the batch- and
 * filter-split decompositions the paper's two schemes rely on, and a
 * hand-worked fixture.  The paper prints no worked numeric example, so
 * paper-value parity is unpinned; every function here is pinned by the
 * mathematics above.
 *
 * bfloat16 storage (the reduced-precision variant keeps tensors as the upper
 * 16 bits of an IEEE binary32 value): oracle_round_bf16 rounds binary32 to the
 * nearest such value, ties to the even 16-bit pattern.  Pinned by hand-written
 * bit patterns (exact values, both tie directions, carry into the exponent,
 * overflow to infinity, signed zeros, NaN) and against torch's CPU conversion.
 *
 * Glue layers of the five-layer stack (not in the paper's text; they come
 * with the Krizhevsky architecture it trains): ReLU and 3x3 stride-2 max
 * pooling without padding, floor output size, first maximum in row-major
 * window order wins.
 */
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

static int out_extent(int in, int filt, int stride, int pad)
{
    int span = in + 2 * pad - filt;
    if (span < 0) return 0;
    return span / stride + 1;
}

int oracle_out_extent(int in, int filt, int stride, int pad)
{
    return out_extent(in, filt, stride, pad);
}

/* forward: one accumulator per output element, taps in (c, r, s) order */
void oracle_conv_fwd(const double *x, const double *w, double *y,
                     int N, int C, int H, int W, int K, int R, int S,
                     int stride, int pad)
{
    const int P = out_extent(H, R, stride, pad);
    const int Q = out_extent(W, S, stride, pad);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h = p * stride - pad + r;
                                int v = q * stride - pad + s;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                acc += x[(((size_t)n * C + c) * H + h) * W + v] *
                                       w[(((size_t)k * C + c) * R + r) * S + s];
                            }
                    y[(((size_t)n * K + k) * P + p) * Q + q] = acc;
                }
}

/* backward-data in scatter form: every (output position, tap) pair adds its
 * product to the input position it read in the forward pass. */
void oracle_conv_bwd_data(const double *dy, const double *w, double *dx,
                          int N, int C, int H, int W, int K, int R, int S,
                          int stride, int pad)
{
    const int P = out_extent(H, R, stride, pad);
    const int Q = out_extent(W, S, stride, pad);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double *dxn = dx + (size_t)n * C * H * W;
        for (size_t i = 0; i < (size_t)C * H * W; ++i) dxn[i] = 0.0;
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double g = dy[(((size_t)n * K + k) * P + p) * Q + q];
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h = p * stride - pad + r;
                                int v = q * stride - pad + s;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                dxn[((size_t)c * H + h) * W + v] +=
                                    g * w[(((size_t)k * C + c) * R + r) * S + s];
                            }
                }
    }
}

/* backward-filter: one accumulator per filter tap, samples in (n, p, q) order */
void oracle_conv_bwd_filter(const double *x, const double *dy, double *dw,
                            int N, int C, int H, int W, int K, int R, int S,
                            int stride, int pad)
{
    const int P = out_extent(H, R, stride, pad);
    const int Q = out_extent(W, S, stride, pad);
#pragma omp parallel for schedule(static)
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int p = 0; p < P; ++p)
                            for (int q = 0; q < Q; ++q) {
                                int h = p * stride - pad + r;
                                int v = q * stride - pad + s;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                acc += dy[(((size_t)n * K + k) * P + p) * Q + q] *
                                       x[(((size_t)n * C + c) * H + h) * W + v];
                            }
                    dw[(((size_t)k * C + c) * R + r) * S + s] = acc;
                }
}

/*
 * Element-wise entry points: the same three definitions evaluated only at the
 * listed flat output indices, for parity checks on tensors too large to
 * evaluate in full.  idx[i] is a flat index into the respective output
 * tensor (y: NKPQ, dx: NCHW, dw: KCRS); out[i] receives that element.
 */
void oracle_conv_fwd_at(const double *x, const double *w,
                        int N, int C, int H, int W, int K, int R, int S,
                        int stride, int pad,
                        const int64_t *idx, int64_t nidx, double *out)
{
    const int P = out_extent(H, R, stride, pad);
    const int Q = out_extent(W, S, stride, pad);
    (void)N;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < nidx; ++i) {
        int64_t t = idx[i];
        int q = (int)(t % Q); t /= Q;
        int p = (int)(t % P); t /= P;
        int k = (int)(t % K); t /= K;
        int n = (int)t;
        double acc = 0.0;
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    int h = p * stride - pad + r;
                    int v = q * stride - pad + s;
                    if (h < 0 || h >= H || v < 0 || v >= W) continue;
                    acc += x[(((size_t)n * C + c) * H + h) * W + v] *
                           w[(((size_t)k * C + c) * R + r) * S + s];
                }
        out[i] = acc;
    }
}

/* One dx element: every (k, p, q, r, s) is visited and kept only when its
 * window position lands on (h, w) -- the definition's constraint, literally. */
void oracle_conv_bwd_data_at(const double *dy, const double *w,
                             int N, int C, int H, int W, int K, int R, int S,
                             int stride, int pad,
                             const int64_t *idx, int64_t nidx, double *out)
{
    const int P = out_extent(H, R, stride, pad);
    const int Q = out_extent(W, S, stride, pad);
    (void)N;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < nidx; ++i) {
        int64_t t = idx[i];
        int v0 = (int)(t % W); t /= W;
        int h0 = (int)(t % H); t /= H;
        int c = (int)(t % C); t /= C;
        int n = (int)t;
        double acc = 0.0;
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int r = 0; r < R; ++r) {
                    if (p * stride - pad + r != h0) continue;
                    for (int q = 0; q < Q; ++q)
                        for (int s = 0; s < S; ++s) {
                            if (q * stride - pad + s != v0) continue;
                            acc += dy[(((size_t)n * K + k) * P + p) * Q + q] *
                                   w[(((size_t)k * C + c) * R + r) * S + s];
                        }
                }
        out[i] = acc;
    }
}

void oracle_conv_bwd_filter_at(const double *x, const double *dy,
                               int N, int C, int H, int W, int K, int R, int S,
                               int stride, int pad,
                               const int64_t *idx, int64_t nidx, double *out)
{
    const int P = out_extent(H, R, stride, pad);
    const int Q = out_extent(W, S, stride, pad);
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < nidx; ++i) {
        int64_t t = idx[i];
        int s = (int)(t % S); t /= S;
        int r = (int)(t % R); t /= R;
        int c = (int)(t % C); t /= C;
        int k = (int)t;
        double acc = 0.0;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    int h = p * stride - pad + r;
                    int v = q * stride - pad + s;
                    if (h < 0 || h >= H || v < 0 || v >= W) continue;
                    acc += dy[(((size_t)n * K + k) * P + p) * Q + q] *
                           x[(((size_t)n * C + c) * H + h) * W + v];
                }
        out[i] = acc;
    }
}

/* ---- glue layers of the conv stack --------------------------------------- */

void oracle_relu_fwd(const double *x, double *y, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}

/* derivative taken as 0 at x == 0 (strict mask) */
void oracle_relu_bwd(const double *x, const double *dy, double *dx, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) dx[i] = x[i] > 0.0 ? dy[i] : 0.0;
}

static int pool_extent(int in) { return in < 3 ? 0 : (in - 3) / 2 + 1; }

int oracle_pool_extent(int in) { return pool_extent(in); }

/* 3x3 window, stride 2, no padding; planes = N*C.  arg (may be NULL) receives
 * the flat in-plane index (h*W + w) of the chosen element. */
void oracle_maxpool3x3s2_fwd(const double *x, double *y, int32_t *arg,
                             int64_t planes, int H, int W)
{
    const int PH = pool_extent(H), PW = pool_extent(W);
#pragma omp parallel for schedule(static)
    for (int64_t pl = 0; pl < planes; ++pl) {
        const double *xp = x + (size_t)pl * H * W;
        for (int i = 0; i < PH; ++i)
            for (int j = 0; j < PW; ++j) {
                int best = (2 * i) * W + 2 * j;
                double m = xp[best];
                for (int r = 0; r < 3; ++r)
                    for (int s = 0; s < 3; ++s) {
                        int at = (2 * i + r) * W + (2 * j + s);
                        if (xp[at] > m) { m = xp[at]; best = at; }
                    }
                y[((size_t)pl * PH + i) * PW + j] = m;
                if (arg) arg[((size_t)pl * PH + i) * PW + j] = best;
            }
    }
}

/* routes each output gradient to the element the forward pass chose */
void oracle_maxpool3x3s2_bwd(const double *x, const double *dy, double *dx,
                             int64_t planes, int H, int W)
{
    const int PH = pool_extent(H), PW = pool_extent(W);
#pragma omp parallel for schedule(static)
    for (int64_t pl = 0; pl < planes; ++pl) {
        const double *xp = x + (size_t)pl * H * W;
        double *dxp = dx + (size_t)pl * H * W;
        for (int i = 0; i < H * W; ++i) dxp[i] = 0.0;
        for (int i = 0; i < PH; ++i)
            for (int j = 0; j < PW; ++j) {
                int best = (2 * i) * W + 2 * j;
                double m = xp[best];
                for (int r = 0; r < 3; ++r)
                    for (int s = 0; s < 3; ++s) {
                        int at = (2 * i + r) * W + (2 * j + s);
                        if (xp[at] > m) { m = xp[at]; best = at; }
                    }
                dxp[best] += dy[((size_t)pl * PH + i) * PW + j];
            }
    }
}

/* ---- bfloat16 storage ------------------------------------------------------ */

/*
 * Round IEEE binary32 bit patterns to bfloat16 (sign, 8 exponent bits, 7
 * fraction bits = the upper half of the binary32 pattern), nearest value, ties
 * to the pattern whose last kept bit is 0.  For finite values the binary32
 * patterns of one sign are ordered like the magnitudes they encode, so the two
 * bfloat16 neighbours of a value are its upper half `keep` and `keep + 1`; the
 * dropped half `rest` says which is nearer (0x8000 = exactly half way).  A
 * carry out of the fraction moves into the exponent, and past the largest
 * finite value into the pattern of infinity, as rounding to nearest requires.
 * NaN stays NaN (quiet bit set so that a payload in the dropped half cannot
 * turn it into infinity); infinities and zeros have rest == 0 and pass.
 */
void oracle_round_bf16(const uint32_t *bits, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        const uint32_t b = bits[i];
        const uint32_t magnitude = b & 0x7FFFFFFFu;
        uint32_t keep = b >> 16;
        const uint32_t rest = b & 0xFFFFu;
        if (magnitude > 0x7F800000u) {          /* NaN */
            out[i] = (uint16_t)(keep | 0x0040u);
            continue;
        }
        if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
        out[i] = (uint16_t)keep;
    }
}
