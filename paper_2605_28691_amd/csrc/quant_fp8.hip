// bf16 -> FP8 E4M3 block quantisation fused with the Skiparse rearrangement (8-bit variant of the attention path).
//
// One workgroup handles one (subsequence, head, block of 128 consecutive positions): it gathers the block's rows from
// the original layout (Algorithm 1 index map), takes max |x| over the block, and writes
//     code = e4m3( clamp( x * (448 / amax), -448, 448 ) )     scale = amax / 448      (1 and 1 if amax = 0)
// in the sparse layout.  All decisions are taken in float32.  Bound by HBM bandwidth: 2 bytes read and 1 byte written
// per element, every row segment (head_dim bf16 values) read as whole 16-byte chunks.
#include "kernels.h"

namespace skiparse {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int QBLOCK = 128;  // positions per scale block

// PAD: any-resolution mode (Sec. 3.2): positions run over the grid padded to multiples of s*s; a padding position is a row of zero
// codes and does not enter the block's maximum.
template <int D, bool PAD>
__global__ __launch_bounds__(256) void quantize_fp8_kernel(const unsigned short* __restrict__ x, unsigned char* __restrict__ x8,
                                                           float* __restrict__ scales, int B, int heads, GridMap g, uint32_t n_blk) {
    constexpr int CH = D / 8;                    // 16-byte chunks per row segment
    constexpr int ROWS_PER_PASS = 256 / CH;      // rows covered by the workgroup at once
    constexpr int PASSES = QBLOCK / ROWS_PER_PASS;
    __shared__ float wave_max[4];
    const uint32_t tid = threadIdx.x;
    const uint32_t blk = blockIdx.x % n_blk, uh = blockIdx.x / n_blk;  // uh = sb * heads + head
    const uint32_t head = uh % (uint32_t)heads, sb = uh / (uint32_t)heads;
    const uint32_t pq = sb / (uint32_t)B, b = sb - pq * (uint32_t)B;
    const uint32_t p = g.mode == MODE_DENSE ? 0u : pq / (uint32_t)g.s, q = g.mode == MODE_DENSE ? 0u : pq - p * (uint32_t)g.s;
    const uint32_t n_sub = (uint32_t)g.n_sub;
    const size_t C = (size_t)heads * D;
    const uint32_t c = tid % CH, r0 = tid / CH;

    u32x4 v[PASSES];
    float amax = 0.f;
#pragma unroll
    for (int ps = 0; ps < PASSES; ps++) {
        const uint32_t j = blk * QBLOCK + r0 + ps * ROWS_PER_PASS;
        v[ps] = u32x4{0u, 0u, 0u, 0u};
        if (j < n_sub) {
            bool real = true;
            const uint32_t tok = PAD ? src_token_padded(g, p, q, j, &real) : src_token(g, p, q, j);
            if (real) {
                const size_t row = (size_t)b * (uint32_t)g.n_tok + tok;
                v[ps] = __builtin_nontemporal_load((const u32x4*)(x + row * C + (size_t)head * D) + c);
            }
        }
#pragma unroll
        for (int e = 0; e < 4; e++) {
            amax = fmaxf(amax, fabsf(__uint_as_float(v[ps][e] << 16)));          // low bf16 of the dword
            amax = fmaxf(amax, fabsf(__uint_as_float(v[ps][e] & 0xffff0000u)));  // high bf16
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    if ((tid & 63u) == 0) wave_max[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
    const float inv = amax > 0.f ? 448.0f / amax : 1.0f;
    if (tid == 0) scales[(size_t)uh * n_blk + blk] = amax > 0.f ? amax / 448.0f : 1.0f;

#pragma unroll
    for (int ps = 0; ps < PASSES; ps++) {
        const uint32_t j = blk * QBLOCK + r0 + ps * ROWS_PER_PASS;
        if (j >= n_sub) continue;
        u32x2 out;
#pragma unroll
        for (int e = 0; e < 4; e += 2) {  // dwords e, e+1 hold elements 2e..2e+3 -> four codes = one output dword
            const float x0 = fminf(fmaxf(__uint_as_float(v[ps][e] << 16) * inv, -448.0f), 448.0f);
            const float x1 = fminf(fmaxf(__uint_as_float(v[ps][e] & 0xffff0000u) * inv, -448.0f), 448.0f);
            const float x2 = fminf(fmaxf(__uint_as_float(v[ps][e + 1] << 16) * inv, -448.0f), 448.0f);
            const float x3 = fminf(fmaxf(__uint_as_float(v[ps][e + 1] & 0xffff0000u) * inv, -448.0f), 448.0f);
            int pk = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, 0, false);  // codes of x0, x1 into the low half
            pk = __builtin_amdgcn_cvt_pk_fp8_f32(x2, x3, pk, true);      // codes of x2, x3 into the high half
            out[e >> 1] = (uint32_t)pk;
        }
        unsigned char* dst = x8 + ((size_t)sb * n_sub + j) * C + (size_t)head * D + c * 8;
        __builtin_nontemporal_store(out, (u32x2*)dst);
    }
}

hipError_t launch_quantize_fp8(const void* x, void* x8, float* scales, int B, int heads, int head_dim, const GridMap& g, bool pad,
                               hipStream_t stream) {
    const uint32_t s2 = g.mode == MODE_DENSE ? 1u : (uint32_t)(g.s * g.s);
    const uint32_t n_blk = ((uint32_t)g.n_sub + QBLOCK - 1) / QBLOCK;
    const uint64_t blocks = (uint64_t)B * s2 * (uint32_t)heads * n_blk;
    if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
    const unsigned short* xs = (const unsigned short*)x;
    unsigned char* x8c = (unsigned char*)x8;
    if (head_dim == 128 && pad)
        quantize_fp8_kernel<128, true><<<(uint32_t)blocks, 256, 0, stream>>>(xs, x8c, scales, B, heads, g, n_blk);
    else if (head_dim == 128)
        quantize_fp8_kernel<128, false><<<(uint32_t)blocks, 256, 0, stream>>>(xs, x8c, scales, B, heads, g, n_blk);
    else if (head_dim == 64 && pad)
        quantize_fp8_kernel<64, true><<<(uint32_t)blocks, 256, 0, stream>>>(xs, x8c, scales, B, heads, g, n_blk);
    else if (head_dim == 64)
        quantize_fp8_kernel<64, false><<<(uint32_t)blocks, 256, 0, stream>>>(xs, x8c, scales, B, heads, g, n_blk);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace skiparse
