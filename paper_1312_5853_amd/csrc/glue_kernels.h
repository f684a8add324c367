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

// Backward of the pooling (optionally of ReLU followed by pooling): every window's gradient goes to the window's
// first maximum.  With RELU the input x is the pre-activation: the window maximum of relu(x) sits where the maximum
// of x sits whenever it is positive, and a non-positive maximum passes no gradient, so
// dx = [x > 0] * (pooled gradient routed by x).  The pass is HBM-bound: read x and dy, write dx, once each.
//
// ---- pooling by walking down the plane: no LDS, no barriers -------------------------------------------------------
// A lane owns two adjacent columns (2j, 2j + 1) of one plane and walks down its rows; lanes 0 .. PW - 1 of a plane's
// segment also own window column j, lane PW only the last column(s).  The window's third column comes from the next
// lane, and the gradient routed to it goes back to that lane, by a lane shift; the window's third row is carried to
// the next window row in registers.  An element's up to four gradients are added in a fixed order (the lane's own two
// window rows first, then the neighbour's sum).  So every element is read once and written once, as adjacent pairs (4 or 8 bytes,
// element-aligned only: planes of odd extent start on odd elements), and a wave keeps D window rows of loads in flight.
// seg = PW + 1 lanes per plane, ppw = 64 / seg planes per wave.
typedef float pool_pair_f32 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ pool_pair_f32 ld_pair_raw(const float *p)
{
    pool_pair_f32 r;
    __builtin_memcpy(&r, p, 8);
    return r;
}
__device__ __forceinline__ unsigned ld_pair_raw(const unsigned short *p)
{
    unsigned r;
    __builtin_memcpy(&r, p, 4);
    return r;
}
__device__ __forceinline__ float pair_lo(pool_pair_f32 r) { return r[0]; }
__device__ __forceinline__ float pair_hi(pool_pair_f32 r) { return r[1]; }
__device__ __forceinline__ float pair_lo(unsigned r) { return __uint_as_float(r << 16); }
__device__ __forceinline__ float pair_hi(unsigned r) { return __uint_as_float(r & 0xFFFF0000u); }
__device__ __forceinline__ void st_pair(float *p, float a, float b)
{
    const pool_pair_f32 r = {a, b};
    __builtin_memcpy(p, &r, 8);
}
__device__ __forceinline__ void st_pair(unsigned short *p, float a, float b)
{
    // rounded to nearest even by v_cvt_pk_bf16_f32: one instruction instead of about fourteen (these kernels' bf16
    // form is bound by its vector instructions, not by bytes)
    typedef float pool_f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 pool_bf16x2 __attribute__((ext_vector_type(2)));
    const pool_f32x2 v = {a, b};
    const pool_bf16x2 r = __builtin_convertvector(v, pool_bf16x2);
    __builtin_memcpy(p, &r, 4);
}
__device__ __forceinline__ void st_one(float *p, float v) { *p = v; }
__device__ __forceinline__ void st_one(unsigned short *p, float v)
{
    const __bf16 r = (__bf16)v;
    __builtin_memcpy(p, &r, 2);
}
__device__ __forceinline__ float raw_elem(float v) { return v; }
__device__ __forceinline__ float raw_elem(unsigned short v) { return __uint_as_float((unsigned)v << 16); }

// what a lane of the walking kernels knows about its place
struct PoolWalkLane {
    int j;              // column pair (2j, 2j + 1); window column j where j < PW
    bool live;          // the lane has a plane
    bool has1;          // column 2j + 1 exists
    int64_t plane;      // its plane (a valid one also for idle lanes, which load but never store)
    int lim;            // largest pair offset within the plane whose second element is still inside the tensor
};
__device__ __forceinline__ bool pool_walk_lane(PoolWalkLane &L, int64_t planes, int HW, int W, int seg, int ppw,
                                               FastDiv dseg)
{
    const int lane = threadIdx.x & 63;
    const int64_t first = ((int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * ppw;
    if (first >= planes) return false;                           // the whole wave is past the end
    const int sub = (int)fastdiv((uint32_t)lane, dseg);
    L.j = lane - sub * seg;
    L.live = sub < ppw && first + sub < planes;
    L.plane = L.live ? first + sub : first;
    L.has1 = 2 * L.j + 1 < W;
    L.lim = L.plane == planes - 1 ? HW - 2 : HW - 1;
    return true;
}

template <bool RELU, typename T, int D>
__global__ __launch_bounds__(256) void maxpool_bwd_walk(const T *__restrict__ x, const T *__restrict__ dy,
                                                         T *__restrict__ dx, int64_t planes, int H, int W, int PH,
                                                         int PW, int seg, int ppw, FastDiv dseg)
{
    PoolWalkLane L;
    if (!pool_walk_lane(L, planes, H * W, W, seg, ppw, dseg)) return;
    const int j = L.j, c0 = 2 * j;
    const bool win = L.live && j < PW;
    const T *xp = x + L.plane * (H * W);
    const T *gp = dy + L.plane * (PH * PW) + (j < PW ? j : PW - 1);
    T *op = dx + L.plane * (H * W);
    typedef decltype(ld_pair_raw(xp)) Raw;

    // the pair of row h, read from a clamped offset (only the last pair of the tensor is ever clamped, by one element:
    // first_of() then takes the pair's second value as the lane's first column)
    auto pair_off = [&](int h) { const int o = h * W + c0; return o < L.lim ? o : L.lim; };
    auto first_of = [&](Raw r, int h) { return h * W + c0 > L.lim ? pair_hi(r) : pair_lo(r); };
    auto store_row = [&](int h, float d0, float d1) {
        if (!L.live) return;
        if (L.has1) st_pair(op + h * W + c0, d0, d1);
        else st_one(op + h * W + c0, d0);
    };

    Raw r1[D], r2[D];
    T gr[D];
    auto issue = [&](int slot, int i) {
        const int ic = i < PH ? i : PH - 1;
        r1[slot] = ld_pair_raw(xp + pair_off(2 * ic + 1));
        r2[slot] = ld_pair_raw(xp + pair_off(2 * ic + 2));
        gr[slot] = gp[ic * PW];
    };
    const Raw r0 = ld_pair_raw(xp + pair_off(0));
#pragma unroll
    for (int d = 0; d < D; ++d) issue(d, d);

    float a00 = first_of(r0, 0), a01 = pair_hi(r0), a02 = __shfl_down(a00, 1);
    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f;                    // gradients routed so far to row 2i of (2j, 2j+1, 2j+2)
    auto finish_row = [&](int h, float e0, float e1, float e2, float v0, float v1) {
        const float t = __shfl_up(e2, 1);
        float d0 = j > 0 ? e0 + t : e0, d1 = e1;
        if (RELU && !(v0 > 0.f)) d0 = 0.f;
        if (RELU && !(v1 > 0.f)) d1 = 0.f;
        store_row(h, d0, d1);
    };
    auto step = [&](int d, int i) {                              // window row i from slot d; refill the slot
        const float a10 = first_of(r1[d], 2 * i + 1), a11 = pair_hi(r1[d]);
        const float a20 = first_of(r2[d], 2 * i + 2), a21 = pair_hi(r2[d]);
        const float g = win ? raw_elem(gr[d]) : 0.f;
        issue(d, i + D);
        const float a12 = __shfl_down(a10, 1), a22 = __shfl_down(a20, 1);
        int best = 0;
        float m = a00;
        if (a01 > m) { m = a01; best = 1; }
        if (a02 > m) { m = a02; best = 2; }
        if (a10 > m) { m = a10; best = 3; }
        if (a11 > m) { m = a11; best = 4; }
        if (a12 > m) { m = a12; best = 5; }
        if (a20 > m) { m = a20; best = 6; }
        if (a21 > m) { m = a21; best = 7; }
        if (a22 > m) { m = a22; best = 8; }
        finish_row(2 * i, acc0 + (best == 0 ? g : 0.f), acc1 + (best == 1 ? g : 0.f), acc2 + (best == 2 ? g : 0.f),
                   a00, a01);
        finish_row(2 * i + 1, best == 3 ? g : 0.f, best == 4 ? g : 0.f, best == 5 ? g : 0.f, a10, a11);
        acc0 = best == 6 ? g : 0.f; acc1 = best == 7 ? g : 0.f; acc2 = best == 8 ? g : 0.f;
        a00 = a20; a01 = a21; a02 = a22;
    };
    // whole groups of D window rows without a branch between them (a branch would make the compiler wait for every
    // load in flight), then the rest
    int i0 = 0;
    for (; i0 + D <= PH; i0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) step(d, i0 + d);
    }
#pragma unroll
    for (int d = 0; d < D - 1; ++d)
        if (i0 + d < PH) step(d, i0 + d);
    finish_row(2 * PH, acc0, acc1, acc2, a00, a01);
    for (int h = 2 * PH + 1; h < H; ++h) store_row(h, 0.f, 0.f);      // a last row that no window reaches
}

template <bool RELU, typename T, int D>
__global__ __launch_bounds__(256) void maxpool_fwd_walk(const T *__restrict__ x, T *__restrict__ y, int64_t planes,
                                                         int H, int W, int PH, int PW, int seg, int ppw, FastDiv dseg)
{
    PoolWalkLane L;
    if (!pool_walk_lane(L, planes, H * W, W, seg, ppw, dseg)) return;
    const int j = L.j, c0 = 2 * j;
    const bool win = L.live && j < PW;
    const T *xp = x + L.plane * (H * W);
    T *yp = y + L.plane * (PH * PW) + j;
    typedef decltype(ld_pair_raw(xp)) Raw;
    auto pair_off = [&](int h) { const int o = h * W + c0; return o < L.lim ? o : L.lim; };
    auto first_of = [&](Raw r, int h) { return h * W + c0 > L.lim ? pair_hi(r) : pair_lo(r); };

    Raw r1[D], r2[D];
    auto issue = [&](int slot, int i) {
        const int ic = i < PH ? i : PH - 1;
        r1[slot] = ld_pair_raw(xp + pair_off(2 * ic + 1));
        r2[slot] = ld_pair_raw(xp + pair_off(2 * ic + 2));
    };
    const Raw r0 = ld_pair_raw(xp + pair_off(0));
#pragma unroll
    for (int d = 0; d < D; ++d) issue(d, d);
    float a00 = first_of(r0, 0), a01 = pair_hi(r0), a02 = __shfl_down(a00, 1);
    auto step = [&](int d, int i) {
        const float a10 = first_of(r1[d], 2 * i + 1), a11 = pair_hi(r1[d]);
        const float a20 = first_of(r2[d], 2 * i + 2), a21 = pair_hi(r2[d]);
        issue(d, i + D);
        const float a12 = __shfl_down(a10, 1), a22 = __shfl_down(a20, 1);
        float m = a00;                                           // the same scan as pool_argmax
        if (a01 > m) m = a01;
        if (a02 > m) m = a02;
        if (a10 > m) m = a10;
        if (a11 > m) m = a11;
        if (a12 > m) m = a12;
        if (a20 > m) m = a20;
        if (a21 > m) m = a21;
        if (a22 > m) m = a22;
        if (win) st_one(yp + i * PW, RELU ? (m > 0.f ? m : 0.f) : m);      // (an input value or zero: the rounding is exact)
        a00 = a20; a01 = a21; a02 = a22;
    };
    int i0 = 0;
    for (; i0 + D <= PH; i0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) step(d, i0 + d);
    }
#pragma unroll
    for (int d = 0; d < D - 1; ++d)
        if (i0 + d < PH) step(d, i0 + d);
}

// Planes wider than a wavefront's column pairs: one thread per input element recomputes the windows that contain it.
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
