// Host-side check of the swizzled LDS tile layout (paper_2605_28691_amd/csrc/lds_layout.h), for head_dim 64 and 128:
//   1. the direct-to-LDS staging (lane l of instruction ii fetches chunk (l % CH) ^ swz(row) of row ii*RPI + l/CH and lands at
//      byte ii*1024 + 16*l) puts every (row, chunk) exactly once at row*RB + ((chunk ^ swz(row)) * 16);
//   2. the fragment read addresses and the transposing read addresses the kernels use point at the chunks they mean;
//   3. both kinds of read are free of bank conflicts (64 banks of 4 bytes; a 16-byte read is served 16 lanes at a time, an
//      8-byte transposing read 32 lanes at a time).
// Built and run by tests/test_host_logic.py with hipcc (host pass only); prints "ok" or the first failure.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <utility>
#include <vector>

#include <hip/hip_runtime.h>

#include "../paper_2605_28691_amd/csrc/lds_layout.h"

using namespace skiparse;

template <int D>
static int check() {
    constexpr int RB = 2 * D, CH = D / 8, NW = 8, RPI = 64 / CH, IPW = CH / NW, KS = D / 16, MT = D / 32;
    std::map<std::pair<int, int>, int> loc;  // (row, chunk) -> byte address in the tile
    for (int wave = 0; wave < NW; wave++)
        for (int i = 0; i < IPW; i++)
            for (int lane = 0; lane < 64; lane++) {
                const int ii = wave * IPW + i, row = ii * RPI + lane / CH;
                const int c = (lane % CH) ^ (int)lds_swizzle<D>(row);
                if (loc.count({row, c})) return printf("D=%d: (row %d, chunk %d) fetched twice\n", D, row, c), 1;
                loc[{row, c}] = ii * 1024 + lane * 16;
            }
    if ((int)loc.size() != 64 * CH) return printf("D=%d: %zu chunks staged, want %d\n", D, loc.size(), 64 * CH), 1;
    for (auto& kv : loc)
        if (kv.second != kv.first.first * RB + ((kv.first.second ^ (int)lds_swizzle<D>(kv.first.first)) * 16))
            return printf("D=%d: row %d chunk %d lands at %d\n", D, kv.first.first, kv.first.second, kv.second), 1;
    auto conflicts = [](const std::vector<int>& addrs, int bytes, int lanes_per_pass) {
        int worst = 0;
        for (size_t g = 0; g < addrs.size(); g += lanes_per_pass) {
            int hits[64] = {0};
            for (int l = 0; l < lanes_per_pass; l++)
                for (int b = 0; b < bytes / 4; b++) worst = std::max(worst, ++hits[(addrs[g + l] / 4 + b) % 64]);
        }
        return worst;
    };
    // fragment reads: lane (lq, h) of MFMA step ks reads chunk 2*ks + h of row 32*half + lq
    for (int half = 0; half < 2; half++)
        for (int ks = 0; ks < KS; ks++) {
            std::vector<int> addrs;
            for (int lane = 0; lane < 64; lane++) {
                const int lq = lane & 31, h = lane >> 5;
                const int a = ((lq * RB + ((h ^ (int)lds_swizzle<D>(lq)) * 16)) ^ (ks * 32)) + half * 32 * RB;  // the XOR form
                const int b = lq * RB + (((2 * ks + h) ^ (int)lds_swizzle<D>(lq)) * 16) + half * 32 * RB;       // the table form
                if (a != b || a != loc[{half * 32 + lq, 2 * ks + h}]) return printf("D=%d: fragment address ks=%d lane=%d\n", D, ks, lane), 1;
                addrs.push_back(a);
            }
            if (conflicts(addrs, 16, 16) != 1) return printf("D=%d: fragment read ks=%d has bank conflicts\n", D, ks), 1;
        }
    // transposing reads: lane i of a 16-lane group addresses row i/4 (+4h, +8*sec, +16*m2, +32*half), channels 4*(i%4).. of the
    // 16-channel group lgrp of channel block mt
    for (int half = 0; half < 2; half++)
        for (int m2 = 0; m2 < 2; m2++)
            for (int mt = 0; mt < MT; mt++)
                for (int sec = 0; sec < 2; sec++) {
                    std::vector<int> addrs;
                    for (int lane = 0; lane < 64; lane++) {
                        const int h = lane >> 5, li = lane & 15, lgrp = (lane >> 4) & 1;
                        const int row = 4 * h + (li >> 2) + 8 * sec, ch = mt * 4 + lgrp * 2 + ((li & 3) >> 1);
                        const int a = row * RB + ((ch ^ (int)lds_swizzle<D>(row)) * 16) + 8 * (li & 1) + (half * 32 + m2 * 16) * RB;
                        const int full_row = row + half * 32 + m2 * 16, col0 = mt * 32 + lgrp * 16 + 4 * (li & 3);
                        if (a != loc[{full_row, col0 / 8}] + (col0 % 8) * 2) return printf("D=%d: transposing address lane=%d\n", D, lane), 1;
                        addrs.push_back(a);
                    }
                    if (conflicts(addrs, 8, 32) != 1) return printf("D=%d: transposing read has bank conflicts\n", D), 1;
                }
    return 0;
}

// The 8-bit tile of the fp8 kernel: rows of D bytes, 4 staging wavefronts, K fragments of 2 x 16 bytes per lane (row lq + 32*kt, chunks
// 4j + 2h and 4j + 2h + 1), transposing byte reads (lane i of a 16-lane group: row i/2 (+8h, +16*g16), 8 bytes at 8*(i%2) of chunk
// 2*mt + lgrp).
template <int D>
static int check8() {
    constexpr int RB = D, CH = D / 16, NW = 4, RPI = 64 / CH, IPW = CH / NW, NJ = D / 64, MT = D / 32;
    std::map<std::pair<int, int>, int> loc;
    for (int wave = 0; wave < NW; wave++)
        for (int i = 0; i < IPW; i++)
            for (int lane = 0; lane < 64; lane++) {
                const int ii = wave * IPW + i, row = ii * RPI + lane / CH;
                const int c = (lane % CH) ^ (int)lds_swizzle8<D>(row);
                if (loc.count({row, c})) return printf("fp8 D=%d: (row %d, chunk %d) fetched twice\n", D, row, c), 1;
                loc[{row, c}] = ii * 1024 + lane * 16;
            }
    if ((int)loc.size() != 64 * CH) return printf("fp8 D=%d: %zu chunks staged, want %d\n", D, loc.size(), 64 * CH), 1;
    for (auto& kv : loc)
        if (kv.second != kv.first.first * RB + ((kv.first.second ^ (int)lds_swizzle8<D>(kv.first.first)) * 16))
            return printf("fp8 D=%d: row %d chunk %d lands at %d\n", D, kv.first.first, kv.first.second, kv.second), 1;
    auto conflicts = [](const std::vector<int>& addrs, int bytes, int lanes_per_pass) {
        int worst = 0;
        for (size_t g = 0; g < addrs.size(); g += lanes_per_pass) {
            int hits[64] = {0};
            for (int l = 0; l < lanes_per_pass; l++)
                for (int b = 0; b < bytes / 4; b++) worst = std::max(worst, ++hits[(addrs[g + l] / 4 + b) % 64]);
        }
        return worst;
    };
    for (int kt = 0; kt < 2; kt++)
        for (int j = 0; j < NJ; j++)
            for (int e = 0; e < 2; e++) {
                std::vector<int> addrs;
                for (int lane = 0; lane < 64; lane++) {
                    const int lq = lane & 31, h = lane >> 5;
                    const int k_rd0 = lq * RB + (((2 * h) ^ (int)lds_swizzle8<D>(lq)) * 16);
                    const int a = (k_rd0 ^ ((4 * j + e) * 16)) + kt * 32 * RB;  // the kernel's XOR form
                    if (a != loc[{kt * 32 + lq, 4 * j + 2 * h + e}]) return printf("fp8 D=%d: fragment address j=%d e=%d lane=%d\n", D, j, e, lane), 1;
                    addrs.push_back(a);
                }
                if (conflicts(addrs, 16, 16) != 1) return printf("fp8 D=%d: fragment read j=%d has bank conflicts\n", D, j), 1;
            }
    for (int g16 = 0; g16 < 4; g16++)
        for (int mt = 0; mt < MT; mt++) {
            std::vector<int> addrs;
            for (int lane = 0; lane < 64; lane++) {
                const int h = lane >> 5, li = lane & 15, lgrp = (lane >> 4) & 1;
                const int v_row = 8 * h + (li >> 1);
                const int v_rd0 = v_row * RB + ((lgrp ^ (int)lds_swizzle8<D>(v_row)) * 16) + 8 * (li & 1);
                const int a = (v_rd0 ^ (mt * 32)) + g16 * 16 * RB;  // the kernel's XOR form
                const int full_row = v_row + 16 * g16, byte0 = mt * 32 + lgrp * 16 + 8 * (li & 1);
                if (a != loc[{full_row, byte0 / 16}] + byte0 % 16) return printf("fp8 D=%d: transposing address lane=%d\n", D, lane), 1;
                addrs.push_back(a);
            }
            if (conflicts(addrs, 8, 32) != 1) return printf("fp8 D=%d: transposing read has bank conflicts\n", D), 1;
        }
    return 0;
}

int main() {
    if (check<128>() || check<64>() || check8<128>() || check8<64>()) return 1;
    printf("ok\n");
    return 0;
}
