// Skiparse index maps for device code (Algorithm 1, "Skiparse Rearrange").
//
// A subsequence is named by its spatial class (p, q) and a batch element b; position j inside it enumerates
// (t, hs, ws) row-major over the reduced grid (T, H/s, W/s).  src_token() returns the token number
// n = (t*H + h)*W + w that sits at position j.  Because t*H + h and hs only ever appear combined, the map needs a
// single division of j by W/s:
//     r = j / Ws (= t*Hs + hs),  ws = j % Ws
//     token-wise: t*H + h = r*s + p                      w = ws*s + q
//     group-wise: t*H + h = (r/s)*s*s + p*s + r%s        w = (ws/s)*s*s + q*s + ws%s     (needs Hs % s == 0)
// Both are instances of one branch-free form  f(x) = x*a + (x/s)*b + c  with (a, b) = (s, 0) for token-wise and
// (1, s*s - s) for group-wise, c = p (or q) for token-wise and p*s (or q*s) for group-wise.  The dense case (position j is
// token j) uses a = 1, b = 0, c = 0 and a divisor of 2^31 so that r is always 0.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace skiparse {

enum Mode : int { MODE_DENSE = 0, MODE_TOKEN = 1, MODE_GROUP = 2 };

// Division of a 32-bit n by a run-time constant d through one multiply-high; exact while n * d < 2^32
// (mul = floor(2^32 / d) + 1, so mul * d = 2^32 + e with 1 <= e <= d and the error term n * e / 2^32 stays below 1).
// d = 1 would need a multiplier of 2^32: it is expressed as mul = 0 plus `one` = 1 (quotient = n * one).
struct FastDiv {
    uint32_t d;
    uint32_t mul;
    uint32_t one;
    __host__ __device__ inline uint32_t div(uint32_t n) const {
#if defined(__HIP_DEVICE_COMPILE__)
        return __umulhi(n, mul) + n * one;
#else
        return (uint32_t)(((uint64_t)n * mul) >> 32) + n * one;
#endif
    }
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    f.mul = d <= 1u ? 0u : (uint32_t)((1ull << 32) / d) + 1u;
    f.one = d <= 1u ? 1u : 0u;
    return f;
}

struct GridMap {
    int mode;      // MODE_DENSE: position j is token j
    int s;         // sparse ratio
    int W;         // original row length
    int n_tok;     // tokens per batch element in the original layout (T*H*W)
    int n_sub;     // tokens per subsequence
    uint32_t a;    // f(x) = x*a + (x/s)*b + c, see above
    uint32_t b;
    uint32_t cmul; // c = p*cmul (rows) or q*cmul (columns)
    FastDiv ws;    // division by W/s
    FastDiv sdiv;  // division by s
    // Any-resolution mode (Sec. 3.2): positions enumerate the grid padded at the end of H and W to multiples of s*s;
    // H_real rows of every H_pad are real, and columns below W (the real row length above) are real.
    int H_real;
    FastDiv hpad;  // division by the padded H
};

__host__ __device__ inline uint32_t src_token(const GridMap& g, uint32_t p, uint32_t q, uint32_t j) {
    const uint32_t r = g.ws.div(j);
    const uint32_t ws = j - r * g.ws.d;
    const uint32_t row = r * g.a + g.sdiv.div(r) * g.b + p * g.cmul;
    const uint32_t w = ws * g.a + g.sdiv.div(ws) * g.b + q * g.cmul;
    return row * (uint32_t)g.W + w;
}

// Any-resolution mode: position j of class (p, q) on the padded grid -> token number in the UNPADDED tensor and whether the
// position is a real token.  g.ws divides by W_pad/s, g.hpad by H_pad; rows and columns of the padded grid come out of the
// same affine forms as in src_token().
__host__ __device__ inline uint32_t src_token_padded(const GridMap& g, uint32_t p, uint32_t q, uint32_t j, bool* real) {
    const uint32_t r = g.ws.div(j);
    const uint32_t ws = j - r * g.ws.d;
    const uint32_t row = r * g.a + g.sdiv.div(r) * g.b + p * g.cmul;  // t * H_pad + h
    const uint32_t w = ws * g.a + g.sdiv.div(ws) * g.b + q * g.cmul;
    const uint32_t t = g.hpad.div(row);
    const uint32_t h = row - t * g.hpad.d;
    *real = h < (uint32_t)g.H_real && w < (uint32_t)g.W;
    return (t * (uint32_t)g.H_real + h) * (uint32_t)g.W + w;
}

// Host side: the map of a grid.  `group` selects the group-wise pattern; `pad` the any-resolution mode, in which the
// subsequences are those of the grid padded at the end of H and W to the next multiples of s*s.
inline GridMap make_dense_gridmap(size_t n) {
    GridMap g;
    g.mode = MODE_DENSE;
    g.s = 1;
    g.W = 0;
    g.n_tok = (int)n;
    g.n_sub = (int)n;
    g.a = 1;
    g.b = 0;
    g.cmul = 0;
    g.ws = make_fastdiv(0xffffffffu);  // multiplier 2: the quotient is 0 for every position below 2^31
    g.H_real = 1;
    g.hpad = make_fastdiv(1);
    g.sdiv = make_fastdiv(1);
    return g;
}

inline GridMap make_gridmap(int T, int H, int W, int s, bool group, bool pad = false) {
    const int n_tok = T * H * W;
    if (s == 1) return make_dense_gridmap((size_t)n_tok);
    const int Hp = pad ? (H + s * s - 1) / (s * s) * (s * s) : H;
    const int Wp = pad ? (W + s * s - 1) / (s * s) * (s * s) : W;
    GridMap g;
    g.mode = group ? MODE_GROUP : MODE_TOKEN;
    g.s = s;
    g.W = W;
    g.n_tok = n_tok;
    g.n_sub = T * Hp * Wp / (s * s);
    g.a = group ? 1u : (uint32_t)s;
    g.b = group ? (uint32_t)(s * s - s) : 0u;
    g.cmul = group ? (uint32_t)s : 1u;
    g.ws = make_fastdiv((uint32_t)(Wp / s));
    g.sdiv = make_fastdiv((uint32_t)s);
    g.H_real = H;
    g.hpad = make_fastdiv((uint32_t)Hp);
    return g;
}

}  // namespace skiparse
