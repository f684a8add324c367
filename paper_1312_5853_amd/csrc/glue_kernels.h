// ReLU, bias and 3x3 / stride-2 max-pooling kernels.
// Part of convnet_hotpath.hip: included there, inside its anonymous namespace, after the common
// definitions (kThreads, kPitch, vector types); not a stand-alone header.
// ---------------------------------------------------------------------------
// Glue layers
// ---------------------------------------------------------------------------
// four elements per thread where the pointers allow it, scalar tail otherwise
// 16-byte groups of the element-wise kernels: 4 floats, or 8 bfloat16 widened to float
__device__ __forceinline__ void ld_vec16(const float *p, int64_t g, float (&v)[4])
{
    const f32x4 q = reinterpret_cast<const f32x4 *>(p)[g];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = q[k];
}
__device__ __forceinline__ void ld_vec16(const unsigned short *p, int64_t g, float (&v)[8])
{
    const u32x4 q = reinterpret_cast<const u32x4 *>(p)[g];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        v[2 * k] = __uint_as_float(q[k] << 16);
        v[2 * k + 1] = __uint_as_float(q[k] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ void st_vec16(float *p, int64_t g, const float (&v)[4])
{
    reinterpret_cast<f32x4 *>(p)[g] = f32x4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ void st_vec16(unsigned short *p, int64_t g, const float (&v)[8])
{
    u32x4 q;
#pragma unroll
    for (int k = 0; k < 4; ++k) q[k] = (unsigned)bf16_round(v[2 * k]) | ((unsigned)bf16_round(v[2 * k + 1]) << 16);
    reinterpret_cast<u32x4 *>(p)[g] = q;
}

// One thread handles a 16-byte group (4 floats or 8 bfloat16) when `vec` (pointers 16-byte aligned), else one
// element; the last few threads of the vector form take the tail elements one each.
template <typename T>
__global__ void relu_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t n, int vec)
{
    constexpr int V = 16 / (int)sizeof(T);
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (vec) {
        const int64_t nv = n / V;
        if (i < nv) {
            float v[V];
            ld_vec16(x, i, v);
#pragma unroll
            for (int k = 0; k < V; ++k) v[k] = v[k] > 0.f ? v[k] : 0.f;
            st_vec16(y, i, v);
        }
        const int64_t t = nv * V + i;
        if (i < n - nv * V) { const float v = ld_elem(x, t); st_elem(y, t, v > 0.f ? v : 0.f); }
    } else if (i < n) {
        const float v = ld_elem(x, i);
        st_elem(y, i, v > 0.f ? v : 0.f);
    }
}

template <typename T>
__global__ void relu_bwd_kernel(const T *__restrict__ x, const T *__restrict__ dy, T *__restrict__ dx, int64_t n,
                                int vec)
{
    constexpr int V = 16 / (int)sizeof(T);
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (vec) {
        const int64_t nv = n / V;
        if (i < nv) {
            float a[V], g[V];
            ld_vec16(x, i, a);
            ld_vec16(dy, i, g);
#pragma unroll
            for (int k = 0; k < V; ++k) g[k] = a[k] > 0.f ? g[k] : 0.f;
            st_vec16(dx, i, g);
        }
        const int64_t t = nv * V + i;
        if (i < n - nv * V) st_elem(dx, t, ld_elem(x, t) > 0.f ? ld_elem(dy, t) : 0.f);
    } else if (i < n) {
        st_elem(dx, i, ld_elem(x, i) > 0.f ? ld_elem(dy, i) : 0.f);
    }
}

// y[n][k][:] += b[k], in place; one thread per element (bf16 tensors: fp32 add, result rounded once)
template <typename T>
__global__ void bias_fwd_kernel(T *__restrict__ y, const float *__restrict__ b, int64_t total, int K, FastDiv div_pq,
                                FastDiv div_k)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const uint32_t plane = fastdiv((uint32_t)i, div_pq);             // n * K + k
    const uint32_t k = plane - fastdiv(plane, div_k) * (uint32_t)K;
    st_elem(y, i, ld_elem(y, i) + b[k]);
}

// Bias gradient, first stage: work-group (k, s) adds dy[n][k][:] over the samples n = s, s + nsplit, ... in a
// fixed order (thread t takes positions t, t + 256, ...; then a tree over the 256 thread sums) -> part[k][s]
template <typename T>
__global__ __launch_bounds__(256) void bias_bwd_partial(const T *__restrict__ dy, float *__restrict__ part, int N,
                                                         int K, int PQ, int nsplit)
{
    __shared__ float red[256];
    const int k = blockIdx.x, sidx = blockIdx.y, tid = threadIdx.x;
    float acc = 0.f;
    for (int n = sidx; n < N; n += nsplit) {
        const T *row = dy + ((int64_t)n * K + k) * PQ;
        for (int e = tid; e < PQ; e += 256) acc += ld_elem(row, e);
    }
    red[tid] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (tid < w) red[tid] += red[tid + w];
        __syncthreads();
    }
    if (tid == 0) part[k * nsplit + sidx] = red[0];
}

// Bias gradient of one-position planes (a fully connected layer's [N][K] output gradient): thread k adds column k
// over the samples in order; neighbouring threads read neighbouring addresses.
template <typename T>
__global__ void bias_bwd_columns(const T *__restrict__ dy, float *__restrict__ db, int N, int K)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    float acc = 0.f;
#pragma unroll 8
    for (int n = 0; n < N; ++n) acc += ld_elem(dy, (int64_t)n * K + k);
    db[k] = acc;
}

// second stage: db[k] = part[k][0] + part[k][1] + ...
__global__ void bias_bwd_finish(const float *__restrict__ part, float *__restrict__ db, int K, int nsplit)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    float s = 0.f;
    for (int t = 0; t < nsplit; ++t) s += part[k * nsplit + t];
    db[k] = s;
}

// index (within the plane) of the first maximum of the 3x3 window at (2i, 2j)
template <typename T>
__device__ __forceinline__ int pool_argmax(const T *__restrict__ xp, int W, int i, int j, float &m)
{
    int best = (2 * i) * W + 2 * j;
    m = ld_elem(xp, best);
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            int at = (2 * i + r) * W + (2 * j + s);
            float v = ld_elem(xp, at);
            if (v > m) { m = v; best = at; }
        }
    return best;
}

template <bool RELU, typename T>
__global__ void maxpool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t total,
                                   int H, int W, int PH, int PW, FastDiv dPW, FastDiv dPH)
{
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    int i, j;
    int64_t pl;
    if (total < ((int64_t)1 << 31)) {                // the usual case: two multiplies instead of 64-bit divisions
        const uint32_t u = fastdiv((uint32_t)t, dPW);
        j = (int)((uint32_t)t - u * (uint32_t)PW);
        const uint32_t q = fastdiv(u, dPH);
        i = (int)(u - q * (uint32_t)PH);
        pl = q;
    } else {
        j = (int)(t % PW);
        const int64_t u = t / PW;
        i = (int)(u % PH);
        pl = u / PH;
    }
    float m;
    pool_argmax(x + pl * H * W, W, i, j, m);
    st_elem(y, t, RELU ? (m > 0.f ? m : 0.f) : m);
}

// Backward of the pooling (optionally of ReLU followed by pooling).  A
// work-group stages a group of whole planes in LDS and finds every window's first
// maximum once.  The gradients are then added into an LDS plane in four phases,
// one per parity class (i % 2, j % 2) of the windows: windows of one class do not
// overlap, so a phase needs no atomics, and an element always receives its (at
// most four) gradients in the same order.
// With RELU the input x is the pre-activation: the window maximum of relu(x)
// sits where the maximum of x sits whenever it is positive, and a non-positive
// maximum passes no gradient, so dx = [x > 0] * (pooled gradient routed by x).
//
// The pass is HBM-bound (read x and dy, write dx once each), so the loop is
// built to keep loads in flight: a thread holds NR elements of the next group
// of planes (and its NR/4 gradients) in registers, fetched while the current
// group is being worked on in LDS.
// group * H*W <= 256 * NR; windows are fewer than a quarter of the elements.
// A thread's unit of global access in the tiled pooling backward: one float, or two adjacent bfloat16 as
// one aligned 32-bit access.  Indices outside [0, limit) do not exist (the pair grid is shifted by
// align_shift() so that pairs are 4-byte aligned even where a plane group starts on an odd element).
__device__ __forceinline__ int align_shift(const float *) { return 0; }
__device__ __forceinline__ int align_shift(const unsigned short *p)
{
    return (int)((reinterpret_cast<uintptr_t>(p) >> 1) & 1);
}
__device__ __forceinline__ void ld_group(const float *p, int e, int limit, float (&v)[1])
{
    v[0] = e < limit ? p[e] : 0.f;
}
__device__ __forceinline__ void ld_group(const unsigned short *p, int e, int limit, float (&v)[2])
{
    if (e >= 0 && e + 1 < limit) {
        const unsigned u = *reinterpret_cast<const unsigned *>(p + e);
        v[0] = __uint_as_float(u << 16);
        v[1] = __uint_as_float(u & 0xFFFF0000u);
    } else {
        v[0] = (e >= 0 && e < limit) ? ld_elem(p, e) : 0.f;
        v[1] = (e + 1 >= 0 && e + 1 < limit) ? ld_elem(p, e + 1) : 0.f;
    }
}
__device__ __forceinline__ void st_group(float *p, int e, int limit, const float (&v)[1])
{
    if (e < limit) p[e] = v[0];
}
__device__ __forceinline__ void st_group(unsigned short *p, int e, int limit, const float (&v)[2])
{
    if (e >= 0 && e + 1 < limit) {
        *reinterpret_cast<unsigned *>(p + e) = (unsigned)bf16_round(v[0]) | ((unsigned)bf16_round(v[1]) << 16);
    } else {
        if (e >= 0 && e < limit) p[e] = bf16_round(v[0]);
        if (e + 1 >= 0 && e + 1 < limit) p[e + 1] = bf16_round(v[1]);
    }
}

template <bool RELU, int NR, typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_tiled(const T *__restrict__ x, const T *__restrict__ dy,
                                                          T *__restrict__ dx, int64_t planes, int H, int W,
                                                          int PH, int PW, int group, FastDiv dPP, FastDiv dPW)
{
    constexpr int NG = NR / 4;
    constexpr int EV = 4 / (int)sizeof(T);          // adjacent elements per access: 1 float or 2 bfloat16
    static_assert(NR % EV == 0 && NG % EV == 0, "whole access groups per thread");
    // groups per thread; with pairs one more, since the pair grid may start one element early
    constexpr int KX = NR / EV + (EV > 1), KG = NG / EV + (EV > 1);
    extern __shared__ float pool_lds[];
    const int HW = H * W, PP = PH * PW;
    // Element e of the staged group sits at index e + (shift of its pair grid): a bfloat16 pair then is two
    // adjacent floats at an 8-byte aligned LDS address, one store / one load instead of two with a two-way bank
    // conflict.  Both arrays have room for that one extra element.
    float *sx = pool_lds;                            // group * HW inputs
    float *sacc = pool_lds + ((group * HW + 2) & ~1);    // group * HW routed gradients
    const int tid = threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * group;
    float xr[KX][EV], gr[KG][EV];
    int xs = 0, gs = 0;                              // shifts of the pair grids of the fetched x and dy groups

    auto fetch = [&](int64_t pl0) {
        const int np = (int)min((int64_t)group, planes - pl0);
        const T *xg = x + pl0 * HW;
        const T *gg = dy + pl0 * PP;
        xs = align_shift(xg);
        gs = align_shift(gg);
#pragma unroll
        for (int k = 0; k < KX; ++k) ld_group(xg, EV * (tid + 256 * k) - xs, np * HW, xr[k]);
#pragma unroll
        for (int k = 0; k < KG; ++k) ld_group(gg, EV * (tid + 256 * k) - gs, np * PP, gr[k]);
    };

    int64_t pl0 = (int64_t)blockIdx.x * group;
    if (pl0 < planes) fetch(pl0);
    for (; pl0 < planes; pl0 += stride) {
        const int np = (int)min((int64_t)group, planes - pl0);
        T *og = dx + pl0 * HW;
        const int os = align_shift(og);
        const int xc = xs;                           // (xs moves on with the prefetch below)
        float *const sxe = sx + xc, *const sae = sacc + xc;
        typedef float f32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int k = 0; k < KX; ++k) {
            const int e0 = EV * (tid + 256 * k) - xc;
            if (EV == 2 && e0 >= 0 && e0 + 1 < np * HW) {
                *reinterpret_cast<f32x2 *>(sxe + e0) = f32x2{xr[k][0], xr[k][EV - 1]};
                *reinterpret_cast<f32x2 *>(sae + e0) = f32x2{0.f, 0.f};
            } else {
#pragma unroll
                for (int u = 0; u < EV; ++u) {
                    const int e = e0 + u;
                    if (e >= 0 && e < np * HW) { sxe[e] = xr[k][u]; sae[e] = 0.f; }
                }
            }
        }
        __syncthreads();
        // every window's first maximum, once; cls = parity class (i % 2, j % 2) of the window, -1 = no window
        int best[KG][EV], cls[KG][EV];
        float g[KG][EV];
#pragma unroll
        for (int k = 0; k < KG; ++k)
#pragma unroll
            for (int u = 0; u < EV; ++u) {
                const int o = EV * (tid + 256 * k) - gs + u;
                best[k][u] = 0; cls[k][u] = -1; g[k][u] = gr[k][u];
                if (o >= 0 && o < np * PP) {
                    const int pl = (int)fastdiv((uint32_t)o, dPP), rem = o - pl * PP;
                    const int i = (int)fastdiv((uint32_t)rem, dPW), j = rem - i * PW;
                    float m;
                    best[k][u] = pl * HW + pool_argmax(sxe + pl * HW, W, i, j, m);
                    cls[k][u] = (i & 1) * 2 + (j & 1);
                }
            }
        if (pl0 + stride < planes) fetch(pl0 + stride);
        // windows of one parity class are disjoint (stride 2, extent 3), so within a phase every accumulator has at
        // most one writer; an element receives its up to four gradients in phase order
#pragma unroll
        for (int c = 0; c < 4; ++c) {
#pragma unroll
            for (int k = 0; k < KG; ++k)
#pragma unroll
                for (int u = 0; u < EV; ++u)
                    if (cls[k][u] == c) sae[best[k][u]] += g[k][u];
            __syncthreads();
        }
#pragma unroll
        for (int k = 0; k < KX; ++k) {
            float res[EV];
            const int e0 = EV * (tid + 256 * k) - os;
            if (EV == 2 && os == xc && e0 >= 0 && e0 + 1 < np * HW) {
                const f32x2 a = *reinterpret_cast<const f32x2 *>(sae + e0);
                const f32x2 v = *reinterpret_cast<const f32x2 *>(sxe + e0);
                res[0] = (RELU && !(v[0] > 0.f)) ? 0.f : a[0];
                res[EV - 1] = (RELU && !(v[1] > 0.f)) ? 0.f : a[1];
            } else {
#pragma unroll
                for (int u = 0; u < EV; ++u) {
                    const int e = e0 + u;
                    float sum = 0.f;
                    if (e >= 0 && e < np * HW) {
                        sum = sae[e];
                        if (RELU && !(sxe[e] > 0.f)) sum = 0.f;
                    }
                    res[u] = sum;
                }
            }
            st_group(og, e0, np * HW, res);
        }
        __syncthreads();
    }
}

// Fallback for planes too large to stage: one thread per input element
// recomputes the windows that contain it.
template <bool RELU, typename T>
__global__ void maxpool_bwd_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                   T *__restrict__ dx, int64_t total, int H, int W, int PH, int PW)
{
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    int w = (int)(t % W);
    int64_t u = t / W;
    int h = (int)(u % H);
    int64_t pl = u / H;
    const T *xp = x + pl * H * W;
    const T *gp = dy + pl * PH * PW;
    const int self = h * W + w;
    int i_lo = h >= 2 ? (h - 1) / 2 : 0, i_hi = h / 2;
    int j_lo = w >= 2 ? (w - 1) / 2 : 0, j_hi = w / 2;
    if (i_hi > PH - 1) i_hi = PH - 1;
    if (j_hi > PW - 1) j_hi = PW - 1;
    float s = 0.f;
    for (int i = i_lo; i <= i_hi; ++i)
        for (int j = j_lo; j <= j_hi; ++j) {
            float m;
            if (pool_argmax(xp, W, i, j, m) == self) s += ld_elem(gp, i * PW + j);
        }
    if (RELU && !(ld_elem(xp, self) > 0.f)) s = 0.f;
    st_elem(dx, t, s);
}
