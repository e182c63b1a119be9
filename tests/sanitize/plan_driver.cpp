// Exercises the GEMM launch planner (csrc/nvfp4_gemm_plan.h, host-only) under the address and
// undefined-behaviour sanitizers and checks its one invariant: over all chunks and launches of a
// problem every output element is covered by exactly one tile.  Prints "ok" on success.
#include "../../paper_2605_18739_amd/csrc/nvfp4_gemm_plan.h"

#include <cstdio>
#include <cstdlib>
#include <vector>

using namespace nvfp4;

static long check(int64_t M, int64_t N, int64_t K, bool big_only)
{
    std::vector<unsigned char> hit((size_t)(M * N), 0);
    long launches = 0;
    for_each_chunk(M, N, K, big_only, [&](int64_t cm, int64_t cm_hi, int64_t cn, int64_t cn_hi, const LaunchPlan &p) {
        if (p.n < 1 || p.n > 3) std::abort();
        for (int i = 0; i < p.n; ++i) {
            const SubLaunch &s = p.part[i];
            const TileShape &t = kShapes[s.kind];
            if (big_only && t.bm < 256) std::abort();
            const int64_t m_lo = cm + s.m_lo, m_hi = cm + s.m_hi, n_lo = cn + s.n_lo, n_hi = cn + s.n_hi;
            if (m_lo < cm || m_hi > cm_hi || n_lo < cn || n_hi > cn_hi || m_lo >= m_hi || n_lo >= n_hi) std::abort();
            const int64_t tn = (n_hi - n_lo + t.bn - 1) / t.bn, tm = (m_hi - m_lo + t.bm - 1) / t.bm;
            if (s.tiles < 1 || s.tiles > tm * tn) std::abort();
            for (int64_t tile = 0; tile < s.tiles; ++tile) {          // a prefix of the row-major tile grid
                const int64_t r0 = m_lo + tile / tn * t.bm, c0 = n_lo + tile % tn * t.bn;
                for (int64_t r = r0; r < std::min<int64_t>(r0 + t.bm, m_hi); ++r)
                    for (int64_t c = c0; c < std::min<int64_t>(c0 + t.bn, n_hi); ++c)
                        if (hit[(size_t)(r * N + c)]++) { std::printf("double cover %lld %lld\n", (long long)r, (long long)c); std::abort(); }
            }
            ++launches;
        }
    });
    for (size_t i = 0; i < hit.size(); ++i)
        if (hit[i] != 1) { std::printf("hole at %zu of %lldx%lldx%lld\n", i, (long long)M, (long long)N, (long long)K); std::abort(); }
    return launches;
}

int main()
{
    const int64_t shapes[][3] = {{1, 8, 64}, {63, 72, 64}, {128, 256, 256}, {3520, 3072, 3072}, {3520, 14336, 3072},
                                 {3520, 3072, 14336}, {4400, 8192, 640}, {4100, 8200, 128}, {700, 1544, 64},
                                 {17600, 3072, 14336}, {14336, 3072, 17600}, {257, 4104, 192}, {5000, 520, 320}};
    long total = 0;
    for (const auto &s : shapes) {
        if (!tiled_ok(s[0], s[1], s[2])) std::abort();
        total += check(s[0], s[1], s[2], false);
        total += check(s[0], s[1], s[2], true);
    }
    // a pseudo-random sweep of small and medium shapes
    uint32_t st = 7u;
    for (int i = 0; i < 300; ++i) {
        st = st * 1664525u + 1013904223u;
        const int64_t M = 1 + (st >> 8) % 2600;
        st = st * 1664525u + 1013904223u;
        const int64_t N = 8 * (1 + (st >> 8) % 330);
        st = st * 1664525u + 1013904223u;
        const int64_t K = 64 * (1 + (st >> 8) % 40);
        total += check(M, N, K, (i & 3) == 0);
    }
    if (tiled_ok(64, 64, 48) || tiled_ok(64, 12, 64)) std::abort();   // shapes only the untiled kernel takes
    if (max_operand_rows(1 << 20) < 256) std::abort();
    std::printf("ok %ld launches\n", total);
    return 0;
}
