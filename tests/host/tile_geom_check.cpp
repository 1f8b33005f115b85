// Host-side brute-force check of the tile geometry used by the convolution kernels
// (paper_1810_09868_amd/csrc/common.h): for every tile of every listed shape, every tile row
// must be a distinct output pixel, every pixel must be covered exactly once, and the halo row
// that each of the nine taps reads must hold exactly the neighbouring input pixel, or be a
// zero row when the neighbour lies outside the image.  Prints "ok <count>" or the first error.
#include <cstdio>
#include <vector>

#include "../../paper_1810_09868_amd/csrc/common.h"

using namespace vgg;

static long check(int N, int H, int W, int rows)
{
    const TileGeom g = make_tile_geom(N, H, W, rows);
    std::vector<int> seen((size_t)g.M, 0);
    long taps = 0;
    for (int t = 0; t < g.ntiles; ++t) {
        const TileOrigin o = tile_origin(g, t);
        for (int j = 0; j < rows; ++j) {
            int m, hrow;
            tile_row(g, o, j, m, hrow);
            if (m != tile_pixel(g, o, j)) { printf("tile_pixel mismatch N%d H%d W%d rows%d tile%d j%d\n", N, H, W, rows, t, j); return -1; }
            if (m < 0) continue;
            if (m >= g.M || seen[m]++) { printf("pixel %d bad/duplicate N%d H%d W%d rows%d\n", m, N, H, W, rows); return -1; }
            const int n = m / (H * W), h = (m / W) % H, w = m % W;
            for (int kh = 0; kh < 3; ++kh)
                for (int kw = 0; kw < 3; ++kw) {
                    const int i = hrow + kh * g.pitch + kw;
                    if (i < 0 || i >= g.S) { printf("halo row %d outside [0,%d) N%d H%d W%d rows%d tile%d j%d\n", i, g.S, N, H, W, rows, t, j); return -1; }
                    const int hh = h + kh - 1, ww = w + kw - 1;
                    const int want = (hh < 0 || hh >= H || ww < 0 || ww >= W) ? -1 : (n * H + hh) * W + ww;
                    const int got = halo_pixel(g, o, i);
                    if (got != want) { printf("tap (%d,%d) of pixel %d reads %d, wants %d (N%d H%d W%d rows%d)\n", kh, kw, m, got, want, N, H, W, rows); return -1; }
                    ++taps;
                }
        }
    }
    for (int m = 0; m < g.M; ++m)
        if (!seen[m]) { printf("pixel %d not covered N%d H%d W%d rows%d\n", m, N, H, W, rows); return -1; }
    return taps;
}

// fast_div against the division it replaces: every small divisor, a few large ones, numerators
// around every multiple of the divisor they can reach plus the top of the 31-bit range.
static bool check_fast_div()
{
    std::vector<int> ds;
    for (int d = 1; d <= 3000; ++d) ds.push_back(d);
    for (int d : {50176, 50177, 65535, 65536, 65537, 1000003, (1 << 30) - 1, 1 << 30, (1 << 30) + 1, 2147483647}) ds.push_back(d);
    for (int d : ds) {
        const FastDiv f = make_fast_div(d);
        auto ok = [&](long long n) {
            if (n < 0 || n > 2147483647ll) return true;
            if (fast_div((int)n, f) != (int)(n / d)) { printf("fast_div(%lld, %d) = %d\n", n, d, fast_div((int)n, f)); return false; }
            return true;
        };
        for (long long n = 0; n < 4096; ++n) if (!ok(n)) return false;
        for (long long k = 1; k <= 2147483647ll / d; k += 1 + k / 7)
            for (int e = -1; e <= 1; ++e) if (!ok(k * d + e)) return false;
        const long long top = 2147483647ll / d * d;
        for (int e = -2; e <= 2; ++e) if (!ok(top + e)) return false;
        for (long long n = 2147483647ll - 64; n <= 2147483647ll; ++n) if (!ok(n)) return false;
    }
    return true;
}

int main()
{
    if (!check_fast_div()) return 1;
    const int shapes[][3] = {{2, 224, 224}, {3, 112, 112}, {5, 56, 56}, {7, 28, 28}, {100, 14, 14}, {9, 14, 14}, {3, 5, 7},
                             {1, 2, 2}, {4, 1, 1}, {2, 3, 300}, {2, 300, 3}, {5, 16, 48}, {1, 32, 32}, {2, 17, 16}, {1, 8, 16},
                             {3, 24, 16}};
    long total = 0;
    for (auto &s : shapes)
        for (int rows : {128, 256}) {
            const long c = check(s[0], s[1], s[2], rows);
            if (c < 0) return 1;
            total += c;
        }
    printf("ok %ld\n", total);
    return 0;
}
