// Launch plan of the tiled FP4 GEMM: host-only, plain C++ (no HIP types), so that it can be
// compiled and exercised on its own (tests build it with the address and undefined-behaviour
// sanitizers).  Which tile shape, how many workgroups per launch, which sub-rectangles.
#ifndef NVFP4_GEMM_PLAN_H
#define NVFP4_GEMM_PLAN_H

#include <algorithm>
#include <cstdint>

namespace nvfp4 {

constexpr int kPlanBK = 64;            // K elements per pipeline step of the tiled kernels

// Tile choice.  Cost of a launch in units of "one 64-k step of a 256x256 tile":
// waves of workgroups over the 256 CUs times (steps per tile * relative step cost +
// a fixed per-tile overhead worth about 8 steps), plus about 4 for the launch itself.
enum TileKind { kTile128 = 0, kTile256x256 = 1, kTile256x192 = 2, kTile64 = 3 };
struct TileShape { int bm, bn; double step_cost; };
static const TileShape kShapes[4] = {{128, 128, 0.30}, {256, 256, 1.0}, {256, 192, 0.80}, {64, 64, 0.16}};
constexpr int kCUs = 256;

static double tile_cost(int64_t M, int64_t N, int64_t K, const TileShape &t)
{
    const int64_t tiles = ((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
    const double waves = (double)((tiles + kCUs - 1) / kCUs);
    return waves * ((double)(K / kPlanBK) * t.step_cost + 8.0) + 4.0;
}

// big_only: only the 256-row tile shapes (the kernels that can carry the LoRA phase)
static TileKind choose_tile(int64_t M, int64_t N, int64_t K, double *cost = nullptr, bool big_only = false)
{
    // order of preference on ties: the larger tile
    static const TileKind order[4] = {kTile256x256, kTile256x192, kTile128, kTile64};
    TileKind best = kTile256x256;
    double cbest = 1e300;
    for (int i = 0; i < (big_only ? 2 : 4); ++i) {
        const double c = tile_cost(M, N, K, kShapes[order[i]]);
        if (c < cbest) {
            cbest = c;
            best = order[i];
        }
    }
    if (cost) *cost = cbest;
    return best;
}

// A launch plan: the main launch runs whole waves of tiles (in row-major tile
// order) with one tile shape; what is left of the tile grid -- the tail of one row
// of tiles and the rows below it -- goes to up to two more launches on the
// corresponding sub-rectangles of the output, each with the tile shape that suits
// it, when the cost model says that beats one more, mostly idle, wave.
struct SubLaunch { int64_t m_lo, m_hi, n_lo, n_hi; TileKind kind; int64_t tiles; };   // tiles: how many of its grid to run (prefix)
struct LaunchPlan { int n; SubLaunch part[3]; };

static LaunchPlan plan_gemm(int64_t M, int64_t N, int64_t K, bool big_only = false)
{
    LaunchPlan p{};
    double whole;
    const TileKind kind = choose_tile(M, N, K, &whole, big_only);
    const TileShape &t = kShapes[kind];
    const int64_t tm = (M + t.bm - 1) / t.bm, tn = (N + t.bn - 1) / t.bn, tiles = tm * tn;
    p.n = 1;
    p.part[0] = {0, M, 0, N, kind, tiles};
    const int64_t main_tiles = tiles / kCUs * kCUs, rest = tiles - main_tiles;
    if (main_tiles == 0 || rest == 0) return p;
    // the remainder in tile order: tail of tile row q (from tile column c) and tile rows q+1 .. tm-1
    const int64_t q = main_tiles / tn, c = main_tiles % tn;
    double split = (double)(main_tiles / kCUs) * ((double)(K / kPlanBK) * t.step_cost + 8.0) + 4.0;
    SubLaunch extra[2];
    int ne = 0;
    if (c != 0) {
        const int64_t m_lo = q * t.bm, m_hi = std::min<int64_t>(M, (q + 1) * t.bm);
        extra[ne++] = {m_lo, m_hi, c * t.bn, N, kTile128, 0};
    }
    const int64_t full_from = c == 0 ? q : q + 1;
    if (full_from < tm) extra[ne++] = {full_from * t.bm, M, 0, N, kTile128, 0};
    for (int i = 0; i < ne; ++i) {
        double ci;
        extra[i].kind = choose_tile(extra[i].m_hi - extra[i].m_lo, extra[i].n_hi - extra[i].n_lo, K, &ci, big_only);
        const TileShape &ts = kShapes[extra[i].kind];
        extra[i].tiles = ((extra[i].m_hi - extra[i].m_lo + ts.bm - 1) / ts.bm) * ((extra[i].n_hi - extra[i].n_lo + ts.bn - 1) / ts.bn);
        split += ci;
    }
    // alternative when the main launch would end inside a tile row: end it at the last whole tile row
    // instead, so that the leftover is one rectangle (one more launch instead of two)
    if (c != 0 && q > 0) {
        SubLaunch below = {q * t.bm, M, 0, N, kTile128, 0};
        double cb;
        below.kind = choose_tile(M - below.m_lo, N, K, &cb, big_only);
        const TileShape &ts = kShapes[below.kind];
        below.tiles = ((M - below.m_lo + ts.bm - 1) / ts.bm) * ((N + ts.bn - 1) / ts.bn);
        const int64_t rows_tiles = q * tn;
        const double by_rows = (double)((rows_tiles + kCUs - 1) / kCUs) * ((double)(K / kPlanBK) * t.step_cost + 8.0) + 4.0 + cb;
        if (by_rows < whole && by_rows < split) {
            p.part[0].tiles = rows_tiles;
            p.part[p.n++] = below;
            return p;
        }
    }
    if (split < whole) {
        p.part[0].tiles = main_tiles;
        for (int i = 0; i < ne; ++i) p.part[p.n++] = extra[i];
    }
    return p;
}

// The tiled kernels address an operand through a 32-bit buffer offset and rely on the range
// check to zero-fill rows past its end, so one launch sees at most max_operand_rows(K) rows of
// A and of W; larger problems are cut into chunks of that many rows (pointer offsets only).
static int64_t max_operand_rows(int64_t K) { return ((0x7FF00000LL - 1) / (K >> 1)) / 256 * 256; }

static bool tiled_ok(int64_t M, int64_t N, int64_t K)
{
    (void)M;
    return K % kPlanBK == 0 && N % 8 == 0 && max_operand_rows(K) >= 256;
}

// f(m_lo, m_hi, n_lo, n_hi, plan) for every chunk of the problem, in launch order
template <class F>
static void for_each_chunk(int64_t M, int64_t N, int64_t K, bool big_only, F &&f)
{
    const int64_t step = max_operand_rows(K);
    for (int64_t m_lo = 0; m_lo < M; m_lo += step)
        for (int64_t n_lo = 0; n_lo < N; n_lo += step) {
            const int64_t m_hi = std::min(M, m_lo + step), n_hi = std::min(N, n_lo + step);
            f(m_lo, m_hi, n_lo, n_hi, plan_gemm(m_hi - m_lo, n_hi - n_lo, K, big_only));
        }
}

}  // namespace nvfp4
#endif  // NVFP4_GEMM_PLAN_H
