// Skiparse index maps for device code (Algorithm 1, "Skiparse Rearrange").
//
// A subsequence is named by its spatial class (p, q) and a batch element b; position j inside it enumerates
// (t, hs, ws) row-major over the reduced grid (T, H/s, W/s).  src_token() returns the token number
// n = (t*H + h)*W + w that sits at position j.  Because t*H + h and hs only ever appear combined, the map needs a
// single division of j by W/s:
//     r = j / Ws (= t*Hs + hs),  ws = j % Ws
//     token-wise: t*H + h = r*s + p                      w = ws*s + q
//     group-wise: t*H + h = (r/s)*s*s + p*s + r%s        w = (ws/s)*s*s + q*s + ws%s     (needs Hs % s == 0)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace skiparse {

enum Mode : int { MODE_DENSE = 0, MODE_TOKEN = 1, MODE_GROUP = 2 };

// Division of a 32-bit n by a run-time constant d through one multiply-high; exact while n * d < 2^32
// (mul = floor(2^32 / d) + 1, so mul * d = 2^32 + e with 1 <= e <= d and the error term n * e / 2^32 stays below 1).
struct FastDiv {
    uint32_t d;
    uint32_t mul;
    __host__ __device__ inline uint32_t div(uint32_t n) const {
#if defined(__HIP_DEVICE_COMPILE__)
        return d == 1u ? n : __umulhi(n, mul);
#else
        return d == 1u ? n : (uint32_t)(((uint64_t)n * mul) >> 32);
#endif
    }
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    f.mul = d <= 1u ? 0u : (uint32_t)((1ull << 32) / d) + 1u;
    return f;
}

struct GridMap {
    int mode;     // MODE_DENSE: position j is token j
    int s;        // sparse ratio
    int W;        // original row length
    int n_tok;    // tokens per batch element in the original layout (T*H*W)
    int n_sub;    // tokens per subsequence
    FastDiv ws;   // division by W/s
    FastDiv sdiv; // division by s
};

__device__ inline uint32_t src_token(const GridMap& g, uint32_t p, uint32_t q, uint32_t j) {
    if (g.mode == MODE_DENSE) return j;
    uint32_t r = g.ws.div(j);
    uint32_t ws = j - r * g.ws.d;
    uint32_t row, w;
    uint32_t s = (uint32_t)g.s;
    if (g.mode == MODE_TOKEN) {
        row = r * s + p;
        w = ws * s + q;
    } else {
        uint32_t ro = g.sdiv.div(r), wo = g.sdiv.div(ws);
        row = ro * s * s + p * s + (r - ro * s);
        w = wo * s * s + q * s + (ws - wo * s);
    }
    return row * (uint32_t)g.W + w;
}

}  // namespace skiparse
