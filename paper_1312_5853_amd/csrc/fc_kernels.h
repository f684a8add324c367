// Fully connected GEMM kernel, its split-sum kernel and the SGD update kernel.
// Part of convnet_hotpath.hip: included there, inside its anonymous namespace, after the common
// definitions (kThreads, kPitch, vector types); not a stand-alone header.
// ---------------------------------------------------------------------------
// Fully connected layers: D[M x Nc] = sum_k A(m, k) * B(k, n) on 128 x 128 tiles
// ---------------------------------------------------------------------------
//
// x [N][I], w [O][I], y [N][O], all row-major.  The three passes as GEMMs whose
// output has its columns contiguous in memory (so a wave's stores are 128-byte
// runs):
//   forward          y [N x O]  rows n, cols o, k = i:  A = x  (k contiguous),  B = w  (k contiguous)
//   backward-data    dx[N x I]  rows n, cols i, k = o:  A = dy (k contiguous),  B = w  (cols contiguous)
//   backward-filter  dw[O x I]  rows o, cols i, k = n:  A = dy (rows contiguous), B = x (cols contiguous)
// An operand with k contiguous ("k-major") is staged in LDS as [row][16] (pitch
// 20 floats) and read with b128 like the convolution tiles.  An operand whose
// rows / columns are contiguous ("transposed") is staged as [k][128] (pitch 132
// floats: 16-byte global loads become b128 LDS writes) and each lane reads its
// eight reduction elements with ds_read_b32: lanes 0..31 take consecutive
// floats, lanes 32..63 sit 8 * 132 floats further = 32 banks further, so both
// the writes and the reads are conflict-free.  Both operands feed reduction
// element 8 * (lane / 32) + t to the t-th matrix instruction of a step.
// Register sets, LDS double buffer and load / store slots between the matrix
// instructions work as in colgemm_fast_kernel.  The reduction is cut into
// ksplit ranges (grid = tiles * ksplit); with ksplit > 1 the kernel writes
// partial sums [ksplit][M][Nc] and fc_reduce_kernel adds them in a fixed order.
struct FcArgs {
    const float *A, *B;
    float *D;              // ksplit == 1: the result (row pitch ldd); else unused
    float *part;           // ksplit > 1: partial sums [ksplit][M][Nc]
    int M, Nc, K;
    int lda, ldb, ldd;
    int mtiles, ntiles, ksplit, steps_per_split;
    const float *bias;     // forward: one value per column (output neuron), or null
    int relu;
};

template <bool AT, bool BT>
__global__ __launch_bounds__(kThreads, 2) void fc_gemm_kernel(const FcArgs p)
{
    constexpr int TM = 2, TN = 2, BM = 128, BN = 128, KC = 16;
    constexpr int PK = KC + 4;                // [row][16] pitch
    constexpr int PT = 128 + 4;               // [k][128] pitch
    constexpr int ASZ = AT ? KC * PT : BM * PK, BSZ = BT ? KC * PT : BN * PK;
    __shared__ __attribute__((aligned(16))) float As0[2 * ASZ];
    __shared__ __attribute__((aligned(16))) float Bs0[2 * BSZ];

    const int ntile = p.mtiles * p.ntiles;
    const int unit = blockIdx.x;
    const int ks = unit / ntile;
    const int tile = unit - ks * ntile;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;
    const int k_begin = ks * p.steps_per_split * KC;
    const int k_end = min(p.K, k_begin + p.steps_per_split * KC);
    const int nsteps = (k_end - k_begin + KC - 1) / KC;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // Two 16-byte pieces per thread, operand and step.  k-major: piece q = tid + 256 * i covers row q / 4,
    // reduction elements 4 * (q % 4)..; transposed: reduction element q / 32, rows (columns) 4 * (q % 32)...
    // A piece outside the matrix or past the end of the reduction range reads the matrix base and stores zeros.
    const float *aptr[2], *bptr[2];
    int alds[2], blds[2], akoff[2], bkoff[2];
    bool arow[2], brow[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = tid + i * kThreads;
        if (AT) {
            const int k = q >> 5, c = (q & 31) * 4;
            arow[i] = m0 + c < p.M;
            akoff[i] = k;
            alds[i] = k * PT + c;
            aptr[i] = p.A + (size_t)(k_begin + k) * p.lda + (arow[i] ? m0 + c : 0);
        } else {
            const int row = q >> 2, kq = (q & 3) * 4;
            arow[i] = m0 + row < p.M;
            akoff[i] = kq;
            alds[i] = row * PK + kq;
            aptr[i] = p.A + (size_t)(arow[i] ? m0 + row : 0) * p.lda + k_begin + kq;
        }
        if (BT) {
            const int k = q >> 5, c = (q & 31) * 4;
            brow[i] = n0 + c < p.Nc;
            bkoff[i] = k;
            blds[i] = k * PT + c;
            bptr[i] = p.B + (size_t)(k_begin + k) * p.ldb + (brow[i] ? n0 + c : 0);
        } else {
            const int row = q >> 2, kq = (q & 3) * 4;
            brow[i] = n0 + row < p.Nc;
            bkoff[i] = kq;
            blds[i] = row * PK + kq;
            bptr[i] = p.B + (size_t)(brow[i] ? n0 + row : 0) * p.ldb + k_begin + kq;
        }
    }
    const size_t a_adv = AT ? (size_t)KC * p.lda : KC, b_adv = BT ? (size_t)KC * p.ldb : KC;

    f32x4 areg[2][2], breg[2][2];
    bool aok[2][2], bok[2][2];
    int kload = k_begin;                      // first reduction element of the next step to load
    auto slot_load = [&](int set, int q) {    // q = 0, 1: A pieces; 2, 3: B pieces (3 also advances the step)
        if (q < 2) {
            aok[set][q] = arow[q] && kload + akoff[q] < k_end;
            areg[set][q] = *reinterpret_cast<const f32x4 *>(aok[set][q] ? aptr[q] : p.A);
            aptr[q] += a_adv;
        } else {
            const int i = q - 2;
            bok[set][i] = brow[i] && kload + bkoff[i] < k_end;
            breg[set][i] = *reinterpret_cast<const f32x4 *>(bok[set][i] ? bptr[i] : p.B);
            bptr[i] += b_adv;
            if (i == 1) kload += KC;
        }
    };
    auto slot_store = [&](int set, int q) {   // the same pieces into LDS buffer `set`
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        if (q < 2) *reinterpret_cast<f32x4 *>(&As0[set * ASZ + alds[q]]) = aok[set][q] ? areg[set][q] : zero;
        else *reinterpret_cast<f32x4 *>(&Bs0[set * BSZ + blds[q - 2]]) = bok[set][q - 2] ? breg[set][q - 2] : zero;
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    const int a_frag = AT ? half * 8 * PT + wm * 64 + l32 : (wm * 64 + l32) * PK + half * 8;
    const int b_frag = BT ? half * 8 * PT + wn * 64 + l32 : (wn * 64 + l32) * PK + half * 8;
    constexpr int NMMA = 8 * TM * TN;

    if (nsteps > 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) slot_load(0, q);
#pragma unroll
        for (int q = 0; q < 4; ++q) slot_store(0, q);
        if (nsteps > 1) {
#pragma unroll
            for (int q = 0; q < 4; ++q) slot_load(1, q);
        }
    }
    __syncthreads();

    // par / mode as in colgemm_fast_kernel: mode 2 = loads of step + 2 and stores of step + 1, 1 = stores only
    auto do_step = [&](auto par_c, auto mode_c) {
        constexpr int par = decltype(par_c)::value, mode = decltype(mode_c)::value;
        const float *As = As0 + par * ASZ, *Bs = Bs0 + par * BSZ;
        float fa[TM][8], fb[TN][8];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (AT) {
#pragma unroll
                for (int t = 0; t < 8; ++t) fa[i][t] = As[a_frag + t * PT + i * 32];
            } else {
                const f32x4 *q = reinterpret_cast<const f32x4 *>(&As[a_frag + i * 32 * PK]);
                const f32x4 lo = q[0], hi = q[1];
#pragma unroll
                for (int t = 0; t < 4; ++t) { fa[i][t] = lo[t]; fa[i][4 + t] = hi[t]; }
            }
        }
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) {
            if (BT) {
#pragma unroll
                for (int t = 0; t < 8; ++t) fb[jn][t] = Bs[b_frag + t * PT + jn * 32];
            } else {
                const f32x4 *q = reinterpret_cast<const f32x4 *>(&Bs[b_frag + jn * 32 * PK]);
                const f32x4 lo = q[0], hi = q[1];
#pragma unroll
                for (int t = 0; t < 4; ++t) { fb[jn][t] = lo[t]; fb[jn][4 + t] = hi[t]; }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
            acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t], fb[jn][t], acc[i][jn], 0, 0, 0);
            if (mode > 0 && m < 8) {          // one slot after each of the first eight matrix instructions
                __builtin_amdgcn_sched_barrier(0);
                if (m < 4) {
                    if (mode == 2) slot_load(par, m);
                } else {
                    slot_store(par ^ 1, m - 4);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (mode > 0) __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    int step = 0;
    for (; step + 3 < nsteps; step += 2) {
        do_step(P0{}, M2{});
        do_step(P1{}, M2{});
    }
    const int rest = nsteps - step;
    if (rest == 3) {
        do_step(P0{}, M2{});
        do_step(P1{}, P1{});
        do_step(P0{}, P0{});
    } else if (rest == 2) {
        do_step(P0{}, P1{});
        do_step(P1{}, P0{});
    } else if (rest == 1) {
        do_step(P0{}, P0{});
    }

    // accumulator value v of block (i, jn): row 32 * i + 8 * (v / 4) + 4 * (lane / 32) + v % 4, column lane % 32
    const bool final_sums = p.ksplit == 1;
    float *out = final_sums ? p.D : p.part + (size_t)ks * p.M * p.Nc;
    const int ldo = final_sums ? p.ldd : p.Nc;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 32 + l32;
        if (col >= p.Nc) continue;
        // The wait for the bias load must sit here, once: left to the compiler it lands in front of every
        // conditional store below, as a wait for ALL outstanding memory operations, the stores before it included,
        // so that the 64 stores of a tile went out one round trip at a time.
        float bv = final_sums && p.bias ? p.bias[col] : 0.f;
        asm volatile("" : "+v"(bv));          // the loaded value is complete from here on
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (v >> 2) * 8 + (v & 3);
                float r = acc[i][jn][v] + bv;
                if (final_sums && p.relu) r = r > 0.f ? r : 0.f;
                if (row < p.M) out[(size_t)row * ldo + col] = r;
            }
        }
    }
}

// D[m][n] = part[0][m][n] + part[1][m][n] + ... (fixed order), then bias per column and ReLU
__global__ void fc_reduce_kernel(const float *__restrict__ part, float *__restrict__ D, int nsplit, int M, int Nc,
                                 int ldd, const float *__restrict__ bias, int relu)
{
    const int64_t total = (int64_t)M * Nc;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        float v = part[i];
        for (int k = 1; k < nsplit; ++k) v += part[(size_t)k * total + i];
        const int m = (int)(i / Nc), n = (int)(i - (int64_t)m * Nc);
        if (bias) v += bias[n];
        if (relu) v = v > 0.f ? v : 0.f;
        D[(size_t)m * ldd + n] = v;
    }
}

// The same update for up to kSgdMaxTensors parameter tensors in ONE launch: tensor t owns the blocks
// [first_block[t], first_block[t + 1]) of 256 threads x 4 parameters (16-byte aligned tensors) or x 1 parameter.
constexpr int kSgdMaxTensors = 24;
struct SgdMultiArgs {
    float *w[kSgdMaxTensors];
    const float *dw[kSgdMaxTensors];
    float *vel[kSgdMaxTensors];
    int64_t count[kSgdMaxTensors];
    unsigned first_block[kSgdMaxTensors + 1];
    int vec[kSgdMaxTensors];
    int n;
    float lr, momentum, weight_decay, grad_scale;
};

__device__ __forceinline__ void sgd_update_elems(float *__restrict__ w, const float *__restrict__ dw,
                                                 float *__restrict__ vel, int64_t count, int64_t i, float lr,
                                                 float momentum, float weight_decay, float grad_scale, int vec);

__global__ void sgd_update_multi_kernel(const SgdMultiArgs a)
{
    int t = 0;
    while (t + 1 < a.n && blockIdx.x >= a.first_block[t + 1]) ++t;          // uniform: at most 23 steps
    const int64_t i = (int64_t)(blockIdx.x - a.first_block[t]) * blockDim.x + threadIdx.x;
    sgd_update_elems(a.w[t], a.dw[t], a.vel[t], a.count[t], i, a.lr, a.momentum, a.weight_decay, a.grad_scale, a.vec[t]);
}

// SGD with momentum and weight decay, one thread per four parameters:
//   v = momentum * v - lr * (weight_decay * w + grad_scale * dw);  w += v
__device__ __forceinline__ void sgd_update_elems(float *__restrict__ w, const float *__restrict__ dw,
                                                 float *__restrict__ vel, int64_t count, int64_t i, float lr,
                                                 float momentum, float weight_decay, float grad_scale, int vec)
{
    if (vec) {
        const int64_t n4 = count >> 2;
        if (i < n4) {
            f32x4 wv = reinterpret_cast<f32x4 *>(w)[i];
            const f32x4 g = reinterpret_cast<const f32x4 *>(dw)[i];
            f32x4 v = reinterpret_cast<f32x4 *>(vel)[i];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = momentum * v[e] - lr * (weight_decay * wv[e] + grad_scale * g[e]);
                wv[e] += v[e];
            }
            reinterpret_cast<f32x4 *>(vel)[i] = v;
            reinterpret_cast<f32x4 *>(w)[i] = wv;
        }
        const int64_t t = (n4 << 2) + i;      // scalar tail
        if (i < (count & 3)) {
            const float v = momentum * vel[t] - lr * (weight_decay * w[t] + grad_scale * dw[t]);
            vel[t] = v;
            w[t] += v;
        }
    } else if (i < count) {
        const float v = momentum * vel[i] - lr * (weight_decay * w[i] + grad_scale * dw[i]);
        vel[i] = v;
        w[i] += v;
    }
}

__global__ void sgd_update_kernel(float *__restrict__ w, const float *__restrict__ dw, float *__restrict__ vel,
                                  int64_t count, float lr, float momentum, float weight_decay, float grad_scale,
                                  int vec)
{
    sgd_update_elems(w, dw, vel, count, (int64_t)blockIdx.x * blockDim.x + threadIdx.x, lr, momentum, weight_decay,
                     grad_scale, vec);
}
