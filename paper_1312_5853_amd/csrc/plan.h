// Host-side planning for the convolution passes: argument checks, derived
// extents, tile-shape choice, split count of the backward-filter reduction and
// the workspace layout.  Plain C++ with no HIP dependency, so the same header
// compiles into a CPU-only self-test.
#ifndef CONVNET_PLAN_H
#define CONVNET_PLAN_H

#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <algorithm>

#include "fastdiv.h"

namespace convnet {

constexpr int kStatusOk = 0;
constexpr int kErrInvalidArg = -1;
constexpr int kErrTooLarge = -2;
constexpr int kErrBadDtype = -3;
constexpr int kErrWorkspace = -4;
constexpr int kErrMisaligned = -5;
constexpr int kErrHip = -6;
constexpr int kErrScratchLimit = -7;

constexpr int kOpFwd = 0, kOpBwdData = 1, kOpBwdFilter = 2;
constexpr int kDtypeF32 = 0, kDtypeBf16 = 1, kDtypeBf16OutBf16 = 2;

constexpr int kChunk = 16;            // reduction elements staged in LDS per step
constexpr int kTapTablePad = 256;     // tap table length is rounded up to this
constexpr int64_t kMaxSpanBytes = (int64_t)1 << 31;
constexpr int kTargetGroups = 512;    // work-groups wanted in flight: 2 per CU on 256 CUs

struct Problem {
    int N, C, H, W, K, R, S, stride, pad;
    int P, Q;
    int64_t x_bs, y_bs;               // batch strides in elements
    int dtype;                        // of the inputs: kDtypeF32 or kDtypeBf16
    bool out_bf16;                    // forward / backward-data write bf16 (caller passed kDtypeBf16OutBf16)
    // Grouped (multi-column) layer: C and K above are the PER-COLUMN counts, the batch strides those of the
    // full tensors; column g starts g * x_gs / y_gs / w_gs elements into x / y / the filters.
    int groups;
    int64_t x_gs, y_gs, w_gs;
};

// Tile shape of one work-group (4 waves): each wave owns TM x TN MFMA tiles of
// 32 x 32; waves are laid out WM x WN.
struct TileShape {
    int TM, TN, WM, WN;
    int mfma;                          // edge of the square matrix-instruction block: 32, or 16 for the 48-row tile
    int bm() const { return TM * WM * mfma; }
    int bn() const { return TN * WN * mfma; }
};

constexpr TileShape kTile128x128 = {2, 2, 2, 2, 32};
constexpr TileShape kTile96x128 = {3, 1, 1, 4, 32};
constexpr TileShape kTile64x128 = {2, 1, 1, 4, 32};
constexpr TileShape kTile32x256 = {1, 2, 1, 4, 32};
constexpr TileShape kTile48x256 = {3, 4, 1, 4, 16};   // fp32 forward / backward-data fast path only
constexpr TileShape kTile128x256 = {2, 4, 2, 2, 32};  // bf16 direct-to-LDS kernel only

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline int64_t round_up64(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Row-tile choice: the block height that pads M (rows of the GEMM view) least;
// ties go to the taller block (more reuse of the gathered operand).
inline TileShape pick_tile(int M)
{
    const TileShape cand[4] = {kTile128x128, kTile96x128, kTile64x128, kTile32x256};
    TileShape best = cand[0];
    int best_cost = round_up(M, best.bm());
    for (int i = 1; i < 4; ++i) {
        int cost = round_up(M, cand[i].bm());
        if (cost < best_cost) { best = cand[i]; best_cost = cost; }
    }
    return best;
}

inline int out_extent(int in, int filt, int stride, int pad)
{
    int span = in + 2 * pad - filt;
    return span < 0 ? 0 : span / stride + 1;
}

// Fills P, Q and checks everything that can be checked without touching the GPU.
inline int make_problem(Problem &pb, int N, int C, int H, int W, int K, int R, int S,
                        int stride, int pad, int64_t x_bs, int64_t y_bs, int dtype)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0) return kErrInvalidArg;
    if (stride <= 0 || pad < 0) return kErrInvalidArg;
    if (dtype != kDtypeF32 && dtype != kDtypeBf16 && dtype != kDtypeBf16OutBf16) return kErrBadDtype;
    pb.out_bf16 = dtype == kDtypeBf16OutBf16;
    if (pb.out_bf16) dtype = kDtypeBf16;
    // keep every intermediate below 2^31 before multiplying extents together
    if (pad > (1 << 20) || stride > (1 << 20)) return kErrTooLarge;
    if ((int64_t)H + 2 * (int64_t)pad < R || (int64_t)W + 2 * (int64_t)pad < S) return kErrInvalidArg;
    pb.N = N; pb.C = C; pb.H = H; pb.W = W; pb.K = K; pb.R = R; pb.S = S;
    pb.stride = stride; pb.pad = pad; pb.dtype = dtype;
    pb.groups = 1; pb.x_gs = 0; pb.y_gs = 0; pb.w_gs = 0;
    pb.P = out_extent(H, R, stride, pad);
    pb.Q = out_extent(W, S, stride, pad);
    if (pb.P <= 0 || pb.Q <= 0) return kErrInvalidArg;
    const int64_t x_sample = (int64_t)C * H * W, y_sample = (int64_t)K * pb.P * pb.Q;
    const int64_t w_elems = (int64_t)K * C * R * S;
    if (x_bs == 0) x_bs = x_sample;
    if (y_bs == 0) y_bs = y_sample;
    if (x_bs < x_sample || y_bs < y_sample) return kErrInvalidArg;
    pb.x_bs = x_bs; pb.y_bs = y_bs;
    const int64_t fat = 4;   // widest element the kernels index with 32-bit offsets
    if (x_sample >= kMaxSpanBytes / fat || y_sample >= kMaxSpanBytes / fat) return kErrTooLarge;
    if (x_bs >= kMaxSpanBytes / fat || y_bs >= kMaxSpanBytes / fat) return kErrTooLarge;
    if ((int64_t)N * x_bs * fat >= kMaxSpanBytes) return kErrTooLarge;
    if ((int64_t)N * y_bs * fat >= kMaxSpanBytes) return kErrTooLarge;
    if (w_elems * fat >= kMaxSpanBytes) return kErrTooLarge;
    if ((int64_t)C * R * S >= (1 << 28) || (int64_t)K * R * S >= (1 << 28)) return kErrTooLarge;
    return kStatusOk;
}

// What one pass needs in the workspace, in bytes from its 256-aligned base.
struct Plan {
    int op;
    TileShape tile;
    int M;            // rows of the GEMM view: K (fwd, wgrad) or C (dgrad)
    int Mpad;
    int Kg;           // fwd: C*R*S, dgrad: K*R*S, wgrad: C*R*S (columns of dw)
    int Kgpad;        // Kg rounded up to kChunk
    int tab_len;      // tap table entries
    int kc;           // reduction depth of one step (16, or 32 where the fast path allows)
    int nsplit;       // wgrad: partial sums over the (n, p, q) reduction
    int chunks_per_split;
    size_t tab_off, tab_bytes;
    size_t wt_off, wt_bytes;          // re-laid-out filters (fwd, dgrad)
    size_t part_off, part_bytes;      // wgrad partials
    bool widen;                       // bf16 activation-side inputs are widened to dense fp32 copies first
    bool widen_w;                     // bf16 filters are widened to fp32 first (forward, backward-data)
    // forward with few channels: the input rows of a 128-position tile are staged once in LDS (patch kernel),
    // row tile of patch_tm * 32 filters, patch_nr rows of pitch patch_wp per channel, patch_lds bytes of LDS
    bool patch;
    int patch_tm, patch_nr, patch_wp, patch_lds;
    size_t cvt_off[2], cvt_bytes[2];  // bf16 -> fp32 staging of the two inputs
    size_t blk_off, blk_bytes;        // channel-blocked copy of the gathered bf16 tensor (forward, backward-data)
    size_t stage_off, stage_bytes;    // dense fp32 result of forward / backward-data before it is rounded to bf16
    // bf16 backward-filter of a stride-1 layer whose output has the input's extent: packed copies in which a
    // filter tap is a linear shift (row pitch lin_wq, lin_jy / lin_jx elements per image), 64 positions per step
    bool lin;
    int lin_wq, lin_jy, lin_jx, lin_steps;
    size_t lin_dy_off, lin_dy_bytes, lin_x_off, lin_x_bytes;
    // columns of a grouped layer run in ONE launch (fp32 kernels of the fast paths): the filter and partial-sum
    // regions then hold `groups` consecutive copies; otherwise the host runs the columns one after the other
    bool fused_groups;
    // bf16 forward / stride-1 backward-data on the direct-to-LDS kernel: channel-blocked, zero-padded copy of the
    // gathered tensor (dma_hp x dma_wp positions per plane, dma_ph rows / dma_pw columns of zeros before the data),
    // dma_kc channels per step, dma_occ work-groups per CU
    bool dma;
    int dma_kc, dma_occ, dma_hp, dma_wp, dma_ph, dma_pw;
    size_t xb_off, xb_bytes;
    // bf16 backward-filter of a stride-4, pad-2 layer with at most four input channels on the bf16 matrix
    // instruction (input rows staged as shifted copies in LDS): rows_splits output-row ranges per image,
    // rows_wgs work-groups with one partial result each, rows_lds bytes of LDS
    bool rows;
    int rows_splits, rows_wgs, rows_lds;
    // the same decomposition for fp32 tensors (any stride up to 4): rows_wp = LDS pitch of a staged input row
    bool rows_f32;
    int rows_wp;
    size_t total;
};

constexpr TileShape kTile128x192 = {2, 3, 2, 2, 32};  // bf16 direct-to-LDS kernel only

// Tile width, step depth and work-groups per CU of the direct-to-LDS bf16 kernel (128 rows per tile).  Width: the
// one that needs the least time on 256 CUs, rounds of tiles x columns per tile (a wider tile moves less through the
// memory path per matrix instruction, so ties go to it).  One round: 64-channel steps, one work-group per CU (three
// LDS buffers of up to 48 KB).  More rounds: 32-channel steps so that two work-groups share a CU and hide each
// other's barriers and epilogues.
inline void pick_dma_tile(int channels, int mtiles, int64_t ncols, TileShape &tile, int &kc, int &occ)
{
    const TileShape cand[3] = {kTile128x256, kTile128x192, kTile128x128};
    int64_t best = -1, best_rounds = 1;
    for (int i = 0; i < 3; ++i) {
        const int64_t tiles = mtiles * ((ncols + cand[i].bn() - 1) / cand[i].bn());
        const int64_t rounds = (tiles + 255) / 256;
        const int64_t cost = rounds * cand[i].bn();
        if (best < 0 || cost < best) { best = cost; tile = cand[i]; best_rounds = rounds; }
    }
    if (best_rounds > 1 || channels % 64 != 0) { kc = 32; occ = 2; }
    else { kc = 64; occ = 1; }
}

inline Plan make_plan(int op, const Problem &pb)
{
    Plan pl = {};
    pl.op = op;
    const int G = pb.groups > 1 ? pb.groups : 1;
    const int RS = pb.R * pb.S;
    if (op == kOpFwd) { pl.M = pb.K; pl.Kg = pb.C * RS; }
    else if (op == kOpBwdData) { pl.M = pb.C; pl.Kg = pb.K * RS; }
    else { pl.M = pb.K; pl.Kg = pb.C * RS; }
    pl.tile = pick_tile(pl.M);
    {
        // bf16 inputs, at least 97 GEMM rows, gathered channel count a multiple of 32: the direct-to-LDS kernel
        const bool fwd = op == kOpFwd;
        const int Cg = fwd ? pb.C : pb.K;
        if (pb.dtype == kDtypeBf16 && G == 1 && (fwd || (op == kOpBwdData && pb.stride == 1)) && Cg % 32 == 0 &&
            pl.M > 96) {
            const int OH = fwd ? pb.P : pb.H, OW = fwd ? pb.Q : pb.W, mul = fwd ? pb.stride : 1;
            const int ph = fwd ? pb.pad : pb.R - 1 - pb.pad, pw = fwd ? pb.pad : pb.S - 1 - pb.pad;
            const int64_t hp = (int64_t)(OH - 1) * mul + pb.R, wp = (int64_t)(OW - 1) * mul + pb.S;
            const int64_t bytes = (int64_t)pb.N * (Cg / 16) * hp * wp * 32;
            if (ph >= 0 && pw >= 0 && bytes < kMaxSpanBytes) {
                pl.dma = true;
                pl.dma_hp = (int)hp; pl.dma_wp = (int)wp; pl.dma_ph = ph; pl.dma_pw = pw;
                const int64_t ncols = (int64_t)pb.N * OH * OW;
                pick_dma_tile(Cg, ceil_div(pl.M, 128), ncols, pl.tile, pl.dma_kc, pl.dma_occ);
                pl.xb_bytes = (size_t)bytes;
            }
        }
    }
    if (!pl.dma) {
        // 33..48 rows on the fp32 fast path: 16 x 16 matrix blocks instead of padding to 64 rows
        const int Cg = op == kOpFwd ? pb.C : pb.K;
        if (pb.dtype == kDtypeF32 && pl.M > 32 && pl.M <= 48 && Cg % kChunk == 0 &&
            (op == kOpFwd || (op == kOpBwdData && pb.stride == 1)))
            pl.tile = kTile48x256;
    }
    pl.Mpad = round_up(pl.M, pl.tile.bm());
    pl.Kgpad = round_up(pl.Kg, kChunk);
    pl.tab_len = round_up(pl.Kg + 2 * kChunk, kTapTablePad);   // two steps of slack for the prefetch
    pl.kc = kChunk;
    pl.nsplit = 1;
    pl.chunks_per_split = 0;
    size_t off = 0;
    pl.tab_off = off; pl.tab_bytes = (size_t)pl.tab_len * 16; off += round_up64(pl.tab_bytes, 256);
    if (op == kOpBwdFilter) {
        const int64_t J = (int64_t)pb.N * pb.P * pb.Q;
        const int jchunks = (int)((J + kChunk - 1) / kChunk);
        pl.fused_groups = G > 1 && pb.dtype == kDtypeF32 && pb.C % kChunk == 0;
        const int tiles = (pl.Mpad / pl.tile.bm()) * ceil_div(pl.Kg, pl.tile.bn()) * (pl.fused_groups ? G : 1);
        // as many splits as fill two work-groups per CU without exceeding them
        int want = kTargetGroups / tiles;
        int most = jchunks / 8 > 0 ? jchunks / 8 : 1;     // at least 8 chunks of work per split
        int nsplit = want < most ? want : most;
        if (nsplit < 1) nsplit = 1;
        pl.chunks_per_split = ceil_div(jchunks, nsplit);
        pl.nsplit = ceil_div(jchunks, pl.chunks_per_split);
        if (pb.dtype == kDtypeBf16 && pb.C % kChunk == 0 && pl.tile.bn() == 128 && pb.stride == 1 &&
            pb.P == pb.H && pb.Q == pb.W && pb.R - 1 == 2 * pb.pad && pb.S - 1 == 2 * pb.pad) {
            const int wq = pb.W + pb.pad;
            const int jy = round_up(pb.P * wq, 8);
            const int jx = round_up(jy + (pb.R - 1) * wq + pb.S, 8);
            const int64_t steps = ((int64_t)pb.N * jy + 63) / 64;
            // (x is packed twice: the second copy, moved up by one element, serves the taps with an odd shift)
            // (dy is packed step-major with its rows padded to whole 128-row tiles: the direct-to-LDS kernel, one
            // work-group of 128 x 256 per CU)
            const int kpad = round_up(pb.K, 128);
            const int64_t dy_bytes = (int64_t)kpad * steps * 64 * 2, x_bytes = (int64_t)2 * pb.C * pb.N * jx * 2;
            if (jy >= 64 && dy_bytes < kMaxSpanBytes && x_bytes < kMaxSpanBytes) {
                pl.lin = true;
                pl.lin_wq = wq; pl.lin_jy = jy; pl.lin_jx = jx; pl.lin_steps = (int)steps;
                want = 256 / ((kpad / 128) * ceil_div(pl.Kg, 256));
                int ns = want < (int)(steps / 4) ? want : (int)(steps / 4);     // at least 4 steps per split
                if (ns < 1) ns = 1;
                pl.chunks_per_split = ceil_div((int)steps, ns);
                pl.nsplit = ceil_div((int)steps, pl.chunks_per_split);
                pl.lin_dy_off = off; pl.lin_dy_bytes = (size_t)dy_bytes; off += round_up64(pl.lin_dy_bytes, 256);
                pl.lin_x_off = off; pl.lin_x_bytes = (size_t)x_bytes; off += round_up64(pl.lin_x_bytes, 256);
            }
        }
        pl.part_off = off;
        const bool staged = pb.C % kChunk == 0;          // fast path always goes through the partials
        pl.part_bytes = (pl.nsplit > 1 || staged) ? (size_t)pl.nsplit * pb.K * pb.C * RS * 4 : 0;
        if (pb.dtype == kDtypeBf16 && G == 1 && pb.stride == 4 && pb.pad == 2 && pb.S <= 11 && pb.R <= 12 &&
            pb.C <= 4 && pl.Kg <= 384 && pb.K <= 96 && pb.Q <= 64 && pb.W % 8 == 0 && pb.x_bs % 8 == 0) {
            const int lds = 2 * 96 * 144 + pb.C * 16 * pb.S * 144 + (255 * 16 + 10 * 144 + 16);   // + trash area
            if (lds <= 150 * 1024) {
                pl.rows = true;
                pl.rows_lds = lds;
                int splits = ceil_div(256, pb.N);
                if (splits > pb.P) splits = pb.P;
                pl.rows_splits = splits;
                const int64_t units = (int64_t)pb.N * splits;
                pl.rows_wgs = units < 256 ? (int)units : 256;
                const size_t need = (size_t)pl.rows_wgs * pb.K * pl.Kg * 4;
                if (need > pl.part_bytes) pl.part_bytes = need;     // the table path stays available at run time
            }
        }
        if (pb.dtype == kDtypeF32 && G == 1 && pb.C <= 4 && pb.K > 48 && pb.K <= 96 && pl.Kg > 128 && pl.Kg <= 384 &&
            pb.Q <= 57 && pb.R + pb.stride <= 16 && pb.stride <= 4 && pb.W <= 256) {
            int wp = pb.W + 2 * pb.pad;                      // pitch = 48 mod 64: taps of up to four filter rows
            wp += (48 - wp % 64 + 64) % 64;                  // read by one wave fall into different banks
            const int64_t lds = ((int64_t)2 * 96 * 58 + (int64_t)pb.C * 16 * wp + 64) * 4;   // + slack
            if (lds <= 150 * 1024) {
                pl.rows_f32 = true;
                pl.rows_lds = (int)lds;
                pl.rows_wp = wp;
                int splits = ceil_div(256, pb.N);
                if (splits > pb.P) splits = pb.P;
                pl.rows_splits = splits;
                const int64_t units = (int64_t)pb.N * splits;
                pl.rows_wgs = units < 256 ? (int)units : 256;
                pl.part_bytes = (size_t)pl.rows_wgs * pb.K * pl.Kg * 4;
            }
        }
        off += round_up64(pl.part_bytes * (pl.fused_groups ? G : 1), 256);
    } else {
        const int Cr_ = op == kOpFwd ? pb.C : pb.K;
        // (fp32 kernels, and the bf16 kernel that stages through registers: neither widens nor takes the direct-to-LDS path)
        pl.fused_groups = G > 1 && (pb.dtype == kDtypeF32 || pb.dtype == kDtypeBf16) && Cr_ % kChunk == 0 &&
                          (op == kOpFwd || pb.stride == 1) && !pl.dma;
        const int GF = pl.fused_groups ? G : 1;
        pl.wt_off = off;
        pl.wt_bytes = (size_t)pl.Mpad * pl.Kgpad * 4;
        off += round_up64(pl.wt_bytes * GF, 256);
        // Fast path (channel count of the gathered tensor a multiple of 16, unit-stride gather rows):
        // the reduction may be cut into ranges when that balances the CUs better.  Model: a CU
        // holding c work-groups runs them at eff(c) of its MFMA rate; the launch lasts as long
        // as its fullest CU; the partial outputs cost one extra pass over memory per range.
        const int Cr = op == kOpFwd ? pb.C : pb.K;
        const int OH = op == kOpFwd ? pb.P : pb.H, OW = op == kOpFwd ? pb.Q : pb.W;
        if (Cr % kChunk == 0 && (op == kOpFwd || pb.stride == 1) && !pl.dma) {
            const int64_t ncols = (int64_t)pb.N * OH * OW;
            const int tiles = (pl.Mpad / pl.tile.bm()) * (int)((ncols + pl.tile.bn() - 1) / pl.tile.bn()) * GF;
            const double out_mb = (double)ncols * pl.M * 4.0 * GF / 1e6;
            // measured fraction of the MFMA rate a CU reaches with c resident work-groups
            const double eff16[5] = {1.0, 0.71, 0.83, 0.87, 0.88};
            // (32-deep steps were measured too: no faster at two work-groups per CU, so steps stay 16 deep)
            double best = 1e30;
            for (int kc = kChunk; kc <= kChunk; kc *= 2) {
                const int steps = (Cr / kc) * RS;
                const double step_us = pl.tile.bm() * pl.tile.bn() * 2.0 * kc / 64.0 / 4.0 / 2100.0;   // MFMA time
                for (int ks = 1; ks <= 4; ++ks) {
                    if (steps * kc / ks < 256) break;
                    const int sps = ceil_div(steps, ks);
                    const int units = tiles * ceil_div(steps, sps);
                    const int per_cu = ceil_div(ceil_div(units, 8), 32);
                    const int resident = per_cu < 4 ? per_cu : 4;
                    double us = per_cu * sps * step_us / eff16[resident];
                    if (ks > 1) us += 5.0 + (ks + 1) * out_mb / 4.5;      // launch + partial traffic at ~4.5 MB/us
                    if (us < best * 0.97) {
                        best = us; pl.kc = kc; pl.nsplit = ceil_div(steps, sps); pl.chunks_per_split = sps;
                    }
                }
            }
            if (pl.nsplit > 1) {
                pl.part_off = off;
                pl.part_bytes = (size_t)pl.nsplit * ncols * pl.M * 4;
                off += round_up64(pl.part_bytes * GF, 256);
            }
        }
        if (pl.chunks_per_split == 0) pl.chunks_per_split = pl.Kgpad / kChunk;
    }
    // bf16 inputs go straight to the bf16 MFMA kernels where the gathered channel count is a multiple of 16
    // (backward-filter: 128-column tiles only).  The few-channel kernels (patch forward, table backward-filter)
    // read bf16 tensors themselves and only want fp32 filters; every other shape is widened to dense fp32
    // copies, batch strides dropped, and takes the fp32 kernels.
    const int Cr = op == kOpBwdData ? pb.K : pb.C;
    const bool bf16_kernel = Cr % kChunk == 0 &&
        (op == kOpFwd || (op == kOpBwdData && pb.stride == 1) || (op == kOpBwdFilter && pl.tile.bn() == 128));
    if (op == kOpFwd && !(pb.C % kChunk == 0)) {
        const int tm = pl.M <= 32 ? 1 : pl.M <= 64 ? 2 : pl.M <= 96 ? 3 : 4;
        const int bm = tm * 32, mpad = round_up(pl.M, bm);
        int span = (pb.Q + 126) / pb.Q;                 // output rows a 128-position tile can straddle, minus one
        if (span > pb.P - 1) span = pb.P - 1;
        const int nr = span * pb.stride + pb.R;
        const int need_w = pb.W + 2 * pb.pad > (pb.Q - 1) * pb.stride + pb.S ? pb.W + 2 * pb.pad
                                                                              : (pb.Q - 1) * pb.stride + pb.S;
        const int wp = round_up(need_w, 4);
        const int64_t lds64 = ((int64_t)2 * bm * 20 + pl.Kgpad + (int64_t)pb.C * nr * wp) * 4;
        if (lds64 <= 80 * 1024 && (int64_t)mpad * pl.Kgpad * 4 <= (int64_t)pl.wt_bytes) {
            pl.patch = true;
            pl.patch_tm = tm; pl.patch_nr = nr; pl.patch_wp = wp; pl.patch_lds = (int)lds64;
        }
    }
    const bool bf16_in = pb.dtype == kDtypeBf16;
    const bool direct = pl.patch || (op == kOpBwdFilter && pb.C % kChunk != 0);   // kernels that read bf16 themselves
    pl.widen = bf16_in && !bf16_kernel && !direct;
    pl.widen_w = bf16_in && !bf16_kernel && op != kOpBwdFilter;
    if (pl.dma) {
        pl.xb_off = off;
        off += round_up64(pl.xb_bytes, 256);
    } else if (pb.dtype == kDtypeBf16 && bf16_kernel && op != kOpBwdFilter) {
        pl.blk_off = off;
        pl.blk_bytes = (size_t)pb.N * Cr * (pl.fused_groups ? G : 1) * (op == kOpFwd ? pb.H * pb.W : pb.P * pb.Q) * 2;
        off += round_up64(pl.blk_bytes, 256);
    }
    if (pb.out_bf16 && op != kOpBwdFilter && !bf16_kernel && !pl.patch) {
        pl.stage_off = off;
        pl.stage_bytes = (size_t)pb.N * (op == kOpFwd ? (size_t)pb.K * pb.P * pb.Q : (size_t)pb.C * pb.H * pb.W) * 4;
        off += round_up64(pl.stage_bytes, 256);
    }
    if (pl.widen || pl.widen_w) {
        const int64_t x_e = (int64_t)pb.N * pb.C * pb.H * pb.W, y_e = (int64_t)pb.N * pb.K * pb.P * pb.Q;
        const int64_t w_e = (int64_t)pb.K * pb.C * RS;
        // slot 0: the activation-side input; slot 1: the filters (forward, backward-data) or dy (backward-filter)
        const int64_t a = op == kOpBwdData ? y_e : x_e;
        const int64_t b = op == kOpBwdFilter ? y_e : w_e;
        const bool need0 = pl.widen, need1 = op == kOpBwdFilter ? pl.widen : pl.widen_w;
        pl.cvt_off[0] = off; pl.cvt_bytes[0] = need0 ? (size_t)a * 4 : 0; off += round_up64(pl.cvt_bytes[0], 256);
        pl.cvt_off[1] = off; pl.cvt_bytes[1] = need1 ? (size_t)b * 4 : 0; off += round_up64(pl.cvt_bytes[1], 256);
    }
    pl.total = off;
    return pl;
}

// ---------------------------------------------------------------------------
// Fully connected layers: x [N][I], w [O][I], y [N][O].  GEMM extents, operand
// orientation and the split of the reduction for fc_gemm_kernel (128 x 128
// tiles, 16 reduction elements per step).
// ---------------------------------------------------------------------------
struct FcPlan {
    int M, Nc, K;                 // output rows, output columns, reduction length
    int lda, ldb, ldd;
    bool at, bt;                  // operand A / B has its rows (columns) contiguous rather than k
    int mtiles, ntiles, ksplit, steps_per_split;
    size_t part_bytes;            // ksplit > 1: partial sums [ksplit][M][Nc], the whole workspace
};

inline int make_fc_plan(FcPlan &pl, int op, int N, int I, int O, int dtype)
{
    if (N <= 0 || I <= 0 || O <= 0) return kErrInvalidArg;
    if (op != kOpFwd && op != kOpBwdData && op != kOpBwdFilter) return kErrInvalidArg;
    if (I % 4 != 0 || O % 4 != 0) return kErrInvalidArg;      // 16-byte pieces along I and O
    if (dtype != kDtypeF32) return kErrBadDtype;
    const int64_t lim = (int64_t)1 << 31;
    if ((int64_t)N * I >= lim || (int64_t)N * O >= lim || (int64_t)O * I >= lim) return kErrTooLarge;
    if (op == kOpFwd) { pl.M = N; pl.Nc = O; pl.K = I; pl.lda = I; pl.ldb = I; pl.ldd = O; pl.at = false; pl.bt = false; }
    else if (op == kOpBwdData) { pl.M = N; pl.Nc = I; pl.K = O; pl.lda = O; pl.ldb = I; pl.ldd = I; pl.at = false; pl.bt = true; }
    else { pl.M = O; pl.Nc = I; pl.K = N; pl.lda = O; pl.ldb = I; pl.ldd = I; pl.at = true; pl.bt = true; }
    pl.mtiles = ceil_div(pl.M, 128);
    pl.ntiles = ceil_div(pl.Nc, 128);
    // aim at two work-groups per compute unit, with at least eight steps per range
    const int64_t tiles = (int64_t)pl.mtiles * pl.ntiles;
    const int steps = ceil_div(pl.K, kChunk);
    int ks = (int)std::min<int64_t>(std::max<int64_t>(1, 512 / tiles), std::max(1, steps / 8));
    ks = std::min(ks, 32);
    pl.steps_per_split = ceil_div(steps, ks);
    pl.ksplit = ceil_div(steps, pl.steps_per_split);
    pl.part_bytes = pl.ksplit > 1 ? (size_t)pl.ksplit * pl.M * pl.Nc * 4 : 0;
    if (tiles * pl.ksplit >= lim) return kErrTooLarge;
    return kStatusOk;
}

}  // namespace convnet
#endif
