// CPU-only self-test of the host-side planning code (no HIP): the magic-number
// division against the / operator, the tile choice and the workspace plan.
#include <cstdio>
#include <cstdlib>

#include "../paper_1312_5853_amd/csrc/plan.h"

using namespace convnet;

static int fails = 0;
#define CHECK(c) do { if (!(c)) { std::printf("FAIL line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

int main()
{
    // fastdiv: every divisor up to 4096 plus large ones, numerators dense at the ends and around multiples
    const unsigned big[] = {4097, 65535, 65536, 65537, 1000003, 43264, 387200, 93312, (1u << 30) + 1, (1u << 31) - 1};
    unsigned long long checked = 0;
    for (unsigned d = 1; d <= 4096 + sizeof(big) / sizeof(big[0]); ++d) {
        const unsigned dd = d <= 4096 ? d : big[d - 4097];
        const FastDiv f = make_fastdiv(dd);
        for (unsigned n = 0; n < 70000; ++n) { CHECK(fastdiv(n, f) == n / dd); ++checked; }
        for (unsigned k = 1; k < 64; ++k) {
            const unsigned long long m = (unsigned long long)dd * k * 33554467ull % (1ull << 31);
            for (long long delta = -2; delta <= 2; ++delta) {
                long long n = (long long)m + delta;
                if (n < 0 || n >= (1ll << 31)) continue;
                CHECK(fastdiv((unsigned)n, f) == (unsigned)n / dd);
                ++checked;
            }
        }
        const unsigned top = (1u << 31) - 1;
        for (unsigned n = top; n > top - 1000; --n) { CHECK(fastdiv(n, f) == n / dd); ++checked; }
    }
    // tile choice pads the row count least
    CHECK(pick_tile(384).bm() == 128 && pick_tile(256).bm() == 128 && pick_tile(128).bm() == 128);
    CHECK(pick_tile(96).bm() == 96 && pick_tile(48).bm() == 64 && pick_tile(16).bm() == 32 && pick_tile(3).bm() == 32);
    CHECK(pick_tile(100).bm() == 128 && pick_tile(192).bm() == 96);
    // problems
    Problem pb;
    CHECK(make_problem(pb, 128, 3, 224, 224, 96, 11, 11, 4, 2, 0, 0, 0) == kStatusOk && pb.P == 55 && pb.Q == 55);
    CHECK(make_problem(pb, 128, 48, 27, 27, 128, 5, 5, 1, 2, 0, 0, 0) == kStatusOk && pb.P == 27);
    CHECK(make_problem(pb, 1, 1, 2, 2, 1, 3, 3, 1, 0, 0, 0, 0) == kErrInvalidArg);      // filter larger than padded input
    CHECK(make_problem(pb, 0, 1, 2, 2, 1, 1, 1, 1, 0, 0, 0, 0) == kErrInvalidArg);
    CHECK(make_problem(pb, 1, 1, 2, 2, 1, 1, 1, 0, 0, 0, 0, 0) == kErrInvalidArg);
    CHECK(make_problem(pb, 1, 1, 2, 2, 1, 1, 1, 1, -1, 0, 0, 0) == kErrInvalidArg);
    CHECK(make_problem(pb, 1, 1, 2, 2, 1, 1, 1, 1, 0, 0, 0, 7) == kErrBadDtype);
    CHECK(make_problem(pb, 1, 1, 2, 2, 1, 1, 1, 1, 0, 3, 0, 0) == kErrInvalidArg);      // batch stride below one sample
    CHECK(make_problem(pb, 4096, 64, 64, 64, 64, 3, 3, 1, 1, 0, 0, 0) == kErrTooLarge); // 2^30 elements = 2^32 bytes
    CHECK(make_problem(pb, 2047, 64, 64, 64, 64, 3, 3, 1, 1, 0, 0, 0) == kStatusOk);    // just under 2^31 bytes
    CHECK(make_problem(pb, 2048, 64, 64, 64, 64, 3, 3, 1, 1, 0, 0, 0) == kErrTooLarge);
    // plans: split count keeps the launch within two work-groups per CU and covers the reduction exactly
    CHECK(make_problem(pb, 128, 256, 13, 13, 384, 3, 3, 1, 1, 0, 0, 0) == kStatusOk);
    Plan pl = make_plan(kOpBwdFilter, pb);
    const int jchunks = (128 * 169 + 15) / 16;
    CHECK(pl.nsplit * (pl.Mpad / pl.tile.bm()) * ((pl.Kg + pl.tile.bn() - 1) / pl.tile.bn()) <= kTargetGroups);
    CHECK(pl.nsplit * pl.chunks_per_split >= jchunks && (pl.nsplit - 1) * pl.chunks_per_split < jchunks);
    CHECK(pl.total >= pl.part_off + pl.part_bytes && pl.part_bytes == (size_t)pl.nsplit * 384 * 2304 * 4);
    pl = make_plan(kOpFwd, pb);
    CHECK(pl.M == 384 && pl.Kg == 2304 && pl.Kgpad == 2304 && pl.wt_bytes == (size_t)384 * 2304 * 4);
    pl = make_plan(kOpBwdData, pb);
    CHECK(pl.M == 256 && pl.Kg == 3456);
    // the workspace need does not depend on the batch strides, for either dtype and for widened shapes too
    for (int dt = 0; dt < 2; ++dt)
        for (int op = kOpFwd; op <= kOpBwdFilter; ++op) {
            Problem dense, wide;
            CHECK(make_problem(dense, 5, 21, 27, 27, 33, 5, 5, 1, 2, 0, 0, dt) == kStatusOk);
            CHECK(make_problem(wide, 5, 21, 27, 27, 33, 5, 5, 1, 2, 96 * 729, 256 * 729, dt) == kStatusOk);
            CHECK(make_plan(op, dense).total == make_plan(op, wide).total);
            // 21 channels, 33 filters: only backward-data has to widen its activation-side input (the few-channel
            // forward and backward-filter kernels read bf16 themselves); the filters are widened wherever they are read
            CHECK(make_plan(op, dense).widen == (dt == 1 && op == kOpBwdData));
            CHECK(make_plan(op, dense).widen_w == (dt == 1 && op != kOpBwdFilter));
            CHECK(make_plan(op, dense).patch == (op == kOpFwd));
            CHECK(make_problem(dense, 5, 48, 27, 27, 128, 5, 5, 1, 2, 0, 0, dt) == kStatusOk);
            CHECK(make_problem(wide, 5, 48, 27, 27, 128, 5, 5, 1, 2, 96 * 729, 256 * 729, dt) == kStatusOk);
            CHECK(make_plan(op, dense).total == make_plan(op, wide).total);
            CHECK(!make_plan(op, dense).widen && !make_plan(op, dense).widen_w && !make_plan(op, dense).patch);
        }
    // fully connected plans: GEMM views, ranges that cover the reduction exactly, argument checks
    FcPlan fp;
    CHECK(make_fc_plan(fp, kOpFwd, 128, 9216, 4096, 0) == kStatusOk);
    CHECK(fp.M == 128 && fp.Nc == 4096 && fp.K == 9216 && !fp.at && !fp.bt && fp.ldd == 4096);
    CHECK(fp.ksplit == 16 && fp.steps_per_split == 36 && fp.part_bytes == (size_t)16 * 128 * 4096 * 4);
    CHECK(make_fc_plan(fp, kOpBwdData, 128, 9216, 4096, 0) == kStatusOk);
    CHECK(fp.M == 128 && fp.Nc == 9216 && fp.K == 4096 && !fp.at && fp.bt && fp.lda == 4096 && fp.ldb == 9216);
    CHECK(fp.ksplit * fp.steps_per_split >= 256 && (fp.ksplit - 1) * fp.steps_per_split < 256);
    CHECK(make_fc_plan(fp, kOpBwdFilter, 128, 9216, 4096, 0) == kStatusOk);
    CHECK(fp.M == 4096 && fp.Nc == 9216 && fp.K == 128 && fp.at && fp.bt && fp.ksplit == 1 && fp.part_bytes == 0);
    for (int K : {1, 15, 16, 17, 100, 1000, 4096, 9216})
        for (int op : {kOpFwd, kOpBwdData, kOpBwdFilter}) {
            const int N = op == kOpBwdFilter ? K : 8, I = op == kOpFwd ? 4 * K : 12, O = op == kOpBwdData ? 4 * K : 20;
            CHECK(make_fc_plan(fp, op, N, I, O, 0) == kStatusOk);
            const int steps = (fp.K + 15) / 16;
            CHECK(fp.ksplit >= 1 && fp.ksplit * fp.steps_per_split >= steps && (fp.ksplit - 1) * fp.steps_per_split < steps);
        }
    CHECK(make_fc_plan(fp, kOpFwd, 0, 16, 16, 0) == kErrInvalidArg);
    CHECK(make_fc_plan(fp, kOpFwd, 4, 18, 16, 0) == kErrInvalidArg);       // I not a multiple of 4
    CHECK(make_fc_plan(fp, kOpFwd, 4, 16, 18, 0) == kErrInvalidArg);
    CHECK(make_fc_plan(fp, 3, 4, 16, 16, 0) == kErrInvalidArg);
    CHECK(make_fc_plan(fp, kOpFwd, 4, 16, 16, 1) == kErrBadDtype);
    CHECK(make_fc_plan(fp, kOpFwd, 4, 1 << 16, 1 << 15, 0) == kErrTooLarge);
    std::printf("%llu divisions checked, %d failures\n", checked, fails);
    return fails ? 1 : 0;
}
