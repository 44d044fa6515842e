// Host-side check of the device index map (paper_2605_28691_amd/csrc/index_map.h): src_token() with its multiply-high
// divisions must equal the plain integer formulas of Algorithm 1 for every position of a grid, and src_token_padded() (the
// any-resolution map, Sec. 3.2) the plain pad-then-index formulas on grids that are not multiples of s*s.  Built and run by
// tests/test_host_logic.py with hipcc (host pass only); exits non-zero on the first mismatch.
#include <cstdio>
#include <cstdlib>

#include "../paper_2605_28691_amd/csrc/index_map.h"

using namespace skiparse;

int main() {
    const int shapes[][4] = {{2, 8, 8, 2}, {3, 8, 12, 2}, {21, 48, 80, 2}, {2, 9, 18, 3}, {1, 16, 32, 4}, {5, 2, 2, 2}, {3, 4, 4, 2}, {1, 25, 50, 5}, {21, 30, 52, 2}};
    long checked = 0;
    for (auto& sh : shapes) {
        const int T = sh[0], H = sh[1], W = sh[2], s = sh[3];
        for (int group = 0; group < 2; group++) {
            if (group && (H % (s * s) || W % (s * s))) continue;
            const GridMap g = make_gridmap(T, H, W, s, group != 0);
            const int Hs = H / s, Ws = W / s;
            for (int p = 0; p < s; p++)
                for (int q = 0; q < s; q++)
                    for (int j = 0; j < g.n_sub; j++) {
                        const int ws = j % Ws, hs = (j / Ws) % Hs, t = j / (Ws * Hs);
                        const int h = group ? (hs / s) * s * s + p * s + hs % s : hs * s + p;
                        const int w = group ? (ws / s) * s * s + q * s + ws % s : ws * s + q;
                        const uint32_t want = (uint32_t)((t * H + h) * W + w);
                        const uint32_t got = src_token(g, (uint32_t)p, (uint32_t)q, (uint32_t)j);
                        if (got != want) {
                            printf("mismatch T%d H%d W%d s%d group%d p%d q%d j%d: got %u want %u\n", T, H, W, s, group, p, q, j, got, want);
                            return 1;
                        }
                        checked++;
                    }
        }
    }
    // any-resolution mode (Sec. 3.2): pad the END of H and W to multiples of s*s, index the padded grid with Algorithm 1's
    // formulas, and call a position real when it lies inside the unpadded grid; its token number is then counted on the
    // unpadded grid.  Every real token must be met exactly once over all classes.
    const int pad_shapes[][4] = {{2, 7, 9, 2}, {3, 5, 6, 2}, {1, 10, 11, 3}, {2, 3, 3, 2}, {1, 17, 13, 4}, {4, 8, 10, 2}, {2, 9, 9, 3}, {21, 45, 80, 2}, {3, 8, 8, 2}};
    for (auto& sh : pad_shapes) {
        const int T = sh[0], H = sh[1], W = sh[2], s = sh[3];
        const int Hp = (H + s * s - 1) / (s * s) * (s * s), Wp = (W + s * s - 1) / (s * s) * (s * s);
        for (int group = 0; group < 2; group++) {
            const GridMap g = make_gridmap(T, H, W, s, group != 0, true);
            if (g.n_sub != T * Hp * Wp / (s * s) || g.n_tok != T * H * W) { printf("padded sizes wrong\n"); return 1; }
            const int Hs = Hp / s, Ws = Wp / s;
            long n_real = 0;
            unsigned char* seen = (unsigned char*)calloc((size_t)T * H * W, 1);
            for (int p = 0; p < s; p++)
                for (int q = 0; q < s; q++)
                    for (int j = 0; j < g.n_sub; j++) {
                        const int ws = j % Ws, hs = (j / Ws) % Hs, t = j / (Ws * Hs);
                        const int h = group ? (hs / s) * s * s + p * s + hs % s : hs * s + p;
                        const int w = group ? (ws / s) * s * s + q * s + ws % s : ws * s + q;
                        const bool want_real = h < H && w < W;
                        bool real = false;
                        const uint32_t got = src_token_padded(g, (uint32_t)p, (uint32_t)q, (uint32_t)j, &real);
                        if (real != want_real || (want_real && got != (uint32_t)((t * H + h) * W + w))) {
                            printf("padded mismatch T%d H%d W%d s%d group%d p%d q%d j%d: got %u real %d, want real %d\n", T, H, W, s, group, p, q, j, got, (int)real, (int)want_real);
                            return 1;
                        }
                        if (real) {
                            if (seen[got]++) { printf("padded map meets token %u twice\n", got); return 1; }
                            n_real++;
                        }
                        checked++;
                    }
            free(seen);
            if (n_real != (long)T * H * W) { printf("padded map: %ld real positions, want %d\n", n_real, T * H * W); return 1; }
        }
    }
    // the multiply-high division over its whole admissible range for a few divisors: n * d < 2^32
    for (uint32_t d : {1u, 2u, 3u, 7u, 40u, 641u, 65535u}) {
        const FastDiv f = make_fastdiv(d);
        const uint64_t limit = (1ull << 32) / d;
        for (uint64_t n = 0; n < limit; n += (limit > 5000000 ? limit / 4999999 : 1)) {
            if (f.div((uint32_t)n) != (uint32_t)(n / d)) { printf("fastdiv %u fails at %llu\n", d, (unsigned long long)n); return 1; }
            checked++;
        }
        const uint32_t last = (uint32_t)(limit - 1);
        if (f.div(last) != last / d) { printf("fastdiv %u fails at the top of its range\n", d); return 1; }
    }
    printf("ok %ld checks\n", checked);
    return 0;
}
