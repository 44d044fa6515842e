// Host-side check of the device index map (paper_2605_28691_amd/csrc/index_map.h): src_token() with its multiply-high
// divisions must equal the plain integer formulas of Algorithm 1 for every position of a grid.  Built and run by
// tests/test_host_logic.py with hipcc (host pass only); exits non-zero on the first mismatch.
#include <cstdio>
#include <cstdlib>

#include "../paper_2605_28691_amd/csrc/index_map.h"

using namespace skiparse;

static GridMap make(int T, int H, int W, int s, int group) {
    GridMap g;
    g.mode = group ? MODE_GROUP : MODE_TOKEN;
    g.s = s;
    g.W = W;
    g.n_tok = T * H * W;
    g.n_sub = g.n_tok / (s * s);
    g.a = group ? 1u : (uint32_t)s;
    g.b = group ? (uint32_t)(s * s - s) : 0u;
    g.cmul = group ? (uint32_t)s : 1u;
    g.ws = make_fastdiv((uint32_t)(W / s));
    g.sdiv = make_fastdiv((uint32_t)s);
    return g;
}

int main() {
    const int shapes[][4] = {{2, 8, 8, 2}, {3, 8, 12, 2}, {21, 48, 80, 2}, {2, 9, 18, 3}, {1, 16, 32, 4}, {5, 2, 2, 2}, {3, 4, 4, 2}, {1, 25, 50, 5}, {21, 30, 52, 2}};
    long checked = 0;
    for (auto& sh : shapes) {
        const int T = sh[0], H = sh[1], W = sh[2], s = sh[3];
        for (int group = 0; group < 2; group++) {
            if (group && (H % (s * s) || W % (s * s))) continue;
            const GridMap g = make(T, H, W, s, group);
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
