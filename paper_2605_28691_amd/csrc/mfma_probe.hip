// Measurement aid: a loop of nothing but matrix-core instructions on caller-supplied operands.  It shows what the matrix pipe
// of this chip sustains by itself under the board's power management (on random operands the clock drops well below nominal),
// which is the ceiling the attention kernels are judged against besides the nominal peak.
//
// Built into a library of its own (libskiparse_probe.so, declared in include/skiparse_probe.h): the benchmark and one GPU test load
// it; the attention library does not contain it.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/skiparse_probe.h"
#include "lds_layout.h"

namespace skiparse_probe {

constexpr int MFMA_PROBE_OPERAND_BYTES = 4 * 2 * 64 * 32;  // what the kernels read of the caller's operand buffer

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int PROBE_THREADS = 256;  // 4 wavefronts, one per SIMD; 512 workgroups put two wavefronts on every SIMD of 256 compute units
constexpr int PROBE_FRAGS = 4;      // operand pairs cycled through, so that consecutive MFMAs see different data

// operands: at least PROBE_FRAGS * 2 * 64 * 32 bytes of arbitrary (e.g. random bf16 / e4m3) data
template <bool FP8>
__global__ __launch_bounds__(PROBE_THREADS) void mfma_probe_kernel(const char* __restrict__ operands, float* __restrict__ sink, int iters) {
    const uint32_t lane = threadIdx.x & 63u;
    i32x8 a[PROBE_FRAGS], b[PROBE_FRAGS];  // 32 bytes per lane each; the bf16 instruction uses the first 16
#pragma unroll
    for (int f = 0; f < PROBE_FRAGS; f++) {
        a[f] = *(const i32x8*)(operands + ((size_t)(2 * f) * 64 + lane) * 32);
        b[f] = *(const i32x8*)(operands + ((size_t)(2 * f + 1) * 64 + lane) * 32);
    }
    f32x16 acc[PROBE_FRAGS];
#pragma unroll
    for (int f = 0; f < PROBE_FRAGS; f++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[f][r] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int f = 0; f < PROBE_FRAGS; f++) {
            if (FP8) {
                acc[f] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[f], b[(f + 1) % PROBE_FRAGS], acc[f], 0, 0, 0, 0, 0, 0);
            } else {
                const bf16x8 av = __builtin_bit_cast(bf16x8, __builtin_shufflevector(a[f], a[f], 0, 1, 2, 3));
                const bf16x8 bv = __builtin_bit_cast(bf16x8, __builtin_shufflevector(b[(f + 1) % PROBE_FRAGS], b[(f + 1) % PROBE_FRAGS], 0, 1, 2, 3));
                acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[f], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int f = 0; f < PROBE_FRAGS; f++)
#pragma unroll
        for (int r = 0; r < 16; r++) s += acc[f][r];
    sink[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

// The bf16 loop with CHAIN consecutive MFMAs on the SAME accumulator before moving to the next of the four (CHAIN = 1 is
// mfma_probe_kernel's round robin): shows whether keeping an accumulator in the matrix pipe for several instructions in a row changes
// what the pipe sustains under the power limit (register-file traffic of the accumulators) and how dependent issue behaves.
template <int CHAIN>
__global__ __launch_bounds__(PROBE_THREADS) void mfma_chain_probe_kernel(const char* __restrict__ operands, float* __restrict__ sink, int iters) {
    const uint32_t lane = threadIdx.x & 63u;
    bf16x8 a[PROBE_FRAGS], b[PROBE_FRAGS];
#pragma unroll
    for (int f = 0; f < PROBE_FRAGS; f++) {
        a[f] = *(const bf16x8*)(operands + ((size_t)(2 * f) * 64 + lane) * 32);
        b[f] = *(const bf16x8*)(operands + ((size_t)(2 * f + 1) * 64 + lane) * 32);
    }
    f32x16 acc[PROBE_FRAGS];
#pragma unroll
    for (int f = 0; f < PROBE_FRAGS; f++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[f][r] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int f = 0; f < PROBE_FRAGS; f++)
#pragma unroll
            for (int c = 0; c < CHAIN; c++)
                acc[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(f + c) % PROBE_FRAGS], b[(f + c + 1) % PROBE_FRAGS], acc[f], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    float s = 0.f;
#pragma unroll
    for (int f = 0; f < PROBE_FRAGS; f++)
#pragma unroll
        for (int r = 0; r < 16; r++) s += acc[f][r];
    sink[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

static hipError_t launch_mfma_chain_probe(const void* operands, float* sink, int chain, int blocks, int iters, hipStream_t stream) {
    const char* ops = (const char*)operands;
    switch (chain) {
        case 1: mfma_chain_probe_kernel<1><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 2: mfma_chain_probe_kernel<2><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 4: mfma_chain_probe_kernel<4><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 8: mfma_chain_probe_kernel<8><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Second probe: the same bf16 MFMA loop with NV independent v_fma_f32 per MFMA in between (fences keep the order).  Shows how much
// vector-ALU work the matrix pipe hides: on this chip a 32x32x16 MFMA keeps the vector issue port busy for about 20 of its 32
// clocks, so only about three full-rate vector instructions per MFMA are free.
template <int NV>
__global__ __launch_bounds__(PROBE_THREADS) void mfma_valu_probe_kernel(const char* __restrict__ operands, float* __restrict__ sink, int iters) {
    const uint32_t lane = threadIdx.x & 63u;
    const i32x8 a8 = *(const i32x8*)(operands + (size_t)lane * 32), b8 = *(const i32x8*)(operands + ((size_t)64 + lane) * 32);
    const bf16x8 av = __builtin_bit_cast(bf16x8, __builtin_shufflevector(a8, a8, 0, 1, 2, 3));
    const bf16x8 bv = __builtin_bit_cast(bf16x8, __builtin_shufflevector(b8, b8, 0, 1, 2, 3));
    f32x16 acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; r++) {
        acc0[r] = 0.f;
        acc1[r] = 0.f;
    }
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = (float)(lane + i) * 1e-3f;
    const float c = 0.999f;
    for (int it = 0; it < iters; it++) {
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < NV; i++) v[i % 16] = fmaf(v[i % 16], c, c);
        __builtin_amdgcn_sched_barrier(0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv, av, acc1, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < NV; i++) v[(i + 8) % 16] = fmaf(v[(i + 8) % 16], c, c);
        __builtin_amdgcn_sched_barrier(0);
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r++) s += acc0[r] + acc1[r] + v[r];
    sink[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

// The same for the 8-bit matrix instruction (32x32x64, 64 clocks): NV independent v_fma_f32 after every MFMA.
template <int NV>
__global__ __launch_bounds__(PROBE_THREADS) void mfma8_valu_probe_kernel(const char* __restrict__ operands, float* __restrict__ sink, int iters) {
    const uint32_t lane = threadIdx.x & 63u;
    const i32x8 av = *(const i32x8*)(operands + (size_t)lane * 32), bv = *(const i32x8*)(operands + ((size_t)64 + lane) * 32);
    f32x16 acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; r++) {
        acc0[r] = 0.f;
        acc1[r] = 0.f;
    }
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; i++) v[i] = (float)(lane + i) * 1e-3f;
    const float c = 0.999f;
    for (int it = 0; it < iters; it++) {
        acc0 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc0, 0, 0, 0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < NV; i++) v[i % 16] = fmaf(v[i % 16], c, c);
        __builtin_amdgcn_sched_barrier(0);
        acc1 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bv, av, acc1, 0, 0, 0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < NV; i++) v[(i + 8) % 16] = fmaf(v[(i + 8) % 16], c, c);
        __builtin_amdgcn_sched_barrier(0);
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r++) s += acc0[r] + acc1[r] + v[r];
    sink[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

static hipError_t launch_mfma8_valu_probe(const void* operands, float* sink, int valu_per_mfma, int blocks, int iters, hipStream_t stream) {
    const char* ops = (const char*)operands;
    switch (valu_per_mfma) {
        case 0: mfma8_valu_probe_kernel<0><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 4: mfma8_valu_probe_kernel<4><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 8: mfma8_valu_probe_kernel<8><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 12: mfma8_valu_probe_kernel<12><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 16: mfma8_valu_probe_kernel<16><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Third probe: the bf16 MFMA loop with the A operand of EVERY MFMA read from LDS (ds_read_b128, 32 KiB of the caller's operands walked
// in 8 KiB steps), as an attention kernel has to feed its matrix products; B operands cycle through 8 register fragments.
__global__ __launch_bounds__(PROBE_THREADS) void mfma_lds_probe_kernel(const char* __restrict__ operands, float* __restrict__ sink, int iters) {
    __shared__ __attribute__((aligned(16))) char lds[32768];
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    for (uint32_t i = tid; i < 32768u / 16u; i += PROBE_THREADS) ((i32x4*)lds)[i] = *(const i32x4*)(operands + (i * 16u) % MFMA_PROBE_OPERAND_BYTES);
    __syncthreads();
    bf16x8 b[8];
#pragma unroll
    for (int f = 0; f < 8; f++) b[f] = *(const bf16x8*)(operands + ((size_t)f * 64 + lane) * 16);
    f32x16 acc[PROBE_FRAGS];
#pragma unroll
    for (int f = 0; f < PROBE_FRAGS; f++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[f][r] = 0.f;
    const char* base = lds + lane * 16u;
    for (int it = 0; it < iters; it++) {
        const char* p = base + (it & 3) * 8192;
        bf16x8 a[8];
#pragma unroll
        for (int f = 0; f < 8; f++) a[f] = *(const bf16x8*)(p + f * 1024);
#pragma unroll
        for (int f = 0; f < 8; f++) acc[f % PROBE_FRAGS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], b[f], acc[f % PROBE_FRAGS], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int f = 0; f < PROBE_FRAGS; f++)
#pragma unroll
        for (int r = 0; r < 16; r++) s += acc[f][r];
    sink[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

// Fourth probe: LDS read instructions only, addressed exactly as the attention kernels address a staged tile of 64 rows of 128 bf16
// (packed rows, XOR-swizzled chunk positions): KIND 0 = the 16-byte fragment reads of K (ds_read_b128, 1 KiB per wavefront
// instruction), KIND 1 = the transposing reads of V^T (ds_read_b64_tr_b16, 512 bytes per wavefront instruction), KIND 2 = plain
// 8-byte reads at the transposing reads' addresses.  16 reads per iteration, all independent; the values are folded into one word
// per thread so that nothing is optimised away.  Timed by the benchmark: bytes per clock and compute unit that each kind of read
// sustains, which bounds how fast an LDS-fed matrix product can be supplied.
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
#define PROBE_LDS_PTR(T) __attribute__((address_space(3))) T*

template <int KIND>
__global__ __launch_bounds__(512) void lds_read_probe_kernel(const char* __restrict__ operands, float* __restrict__ sink, int iters) {
    constexpr int RB = 256;  // row bytes of a 128-channel bf16 tile
    __shared__ __attribute__((aligned(1024))) char tile[2][64 * RB];
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    for (uint32_t i = tid; i < 2u * 64u * RB / 16u; i += 512u) ((i32x4*)&tile[0][0])[i] = *(const i32x4*)(operands + (i * 16u) % MFMA_PROBE_OPERAND_BYTES);
    __syncthreads();
    const uint32_t lq = lane & 31u, h = lane >> 5, li = lane & 15u, lgrp = (lane >> 4) & 1u;
    uint32_t k_rd[8], v_rd[2][4];
#pragma unroll
    for (int ks = 0; ks < 8; ks++) k_rd[ks] = lq * RB + (((uint32_t)(2 * ks) + h) ^ skiparse::lds_swizzle<128>(lq)) * 16u;
#pragma unroll
    for (int sec = 0; sec < 2; sec++)
#pragma unroll
        for (int mt = 0; mt < 4; mt++) {
            const uint32_t row = 4 * h + (li >> 2) + 8 * sec;
            const uint32_t ch = (uint32_t)(mt * 4) + lgrp * 2 + ((li & 3u) >> 1);
            v_rd[sec][mt] = row * RB + ((ch ^ skiparse::lds_swizzle<128>(row)) * 16u) + 8 * (li & 1u);
        }
    int fold = 0;
    for (int it = 0; it < iters; it++) {
        const char* t = &tile[it & 1][0] + ((it >> 1) & 1) * 32 * RB;  // the two 32-row halves of the two tiles in turn
        if (KIND == 0) {
            i32x4 f[16];
#pragma unroll
            for (int g = 0; g < 16; g++) f[g] = *(const i32x4*)(&tile[it & 1][0] + k_rd[g & 7] + (g >> 3) * 32 * RB);
#pragma unroll
            for (int g = 0; g < 16; g++) fold ^= f[g][0] ^ f[g][3];
        } else if (KIND == 1) {
            bf16x4 f[16];
#pragma unroll
            for (int g = 0; g < 16; g++)
                f[g] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((PROBE_LDS_PTR(bf16x4))(PROBE_LDS_PTR(char))(t + v_rd[g & 1][(g >> 1) & 3] + (g >> 3) * 16 * RB));
#pragma unroll
            for (int g = 0; g < 16; g++) fold ^= __builtin_bit_cast(i32x2, f[g])[0] ^ __builtin_bit_cast(i32x2, f[g])[1];
        } else {
            i32x2 f[16];
#pragma unroll
            for (int g = 0; g < 16; g++) f[g] = *(const i32x2*)(t + v_rd[g & 1][(g >> 1) & 3] + (g >> 3) * 16 * RB);
#pragma unroll
            for (int g = 0; g < 16; g++) fold ^= f[g][0] ^ f[g][1];
        }
        asm volatile("" : "+v"(fold)::"memory");  // the reads of the next iteration may not be merged with these
    }
    sink[(size_t)blockIdx.x * 512 + tid] = (float)(fold & 0xffff);
}

static hipError_t launch_lds_read_probe(const void* operands, float* sink, int kind, int blocks, int iters, hipStream_t stream) {
    const char* ops = (const char*)operands;
    switch (kind) {
        case 0: lds_read_probe_kernel<0><<<blocks, 512, 0, stream>>>(ops, sink, iters); break;
        case 1: lds_read_probe_kernel<1><<<blocks, 512, 0, stream>>>(ops, sink, iters); break;
        case 2: lds_read_probe_kernel<2><<<blocks, 512, 0, stream>>>(ops, sink, iters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

static hipError_t launch_mfma_lds_probe(const void* operands, float* sink, int blocks, int iters, hipStream_t stream) {
    mfma_lds_probe_kernel<<<blocks, PROBE_THREADS, 0, stream>>>((const char*)operands, sink, iters);
    return hipGetLastError();
}

static hipError_t launch_mfma_valu_probe(const void* operands, float* sink, int valu_per_mfma, int blocks, int iters, hipStream_t stream) {
    const char* ops = (const char*)operands;
    switch (valu_per_mfma) {
        case 0: mfma_valu_probe_kernel<0><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 2: mfma_valu_probe_kernel<2><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 4: mfma_valu_probe_kernel<4><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 6: mfma_valu_probe_kernel<6><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        case 8: mfma_valu_probe_kernel<8><<<blocks, PROBE_THREADS, 0, stream>>>(ops, sink, iters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

static hipError_t launch_mfma_probe(const void* operands, float* sink, int fp8, int blocks, int iters, hipStream_t stream) {
    if (fp8)
        mfma_probe_kernel<true><<<blocks, PROBE_THREADS, 0, stream>>>((const char*)operands, sink, iters);
    else
        mfma_probe_kernel<false><<<blocks, PROBE_THREADS, 0, stream>>>((const char*)operands, sink, iters);
    return hipGetLastError();
}

thread_local int g_last_hip_error = 0;

static int finish(hipError_t e) {
    if (e == hipSuccess) return SKIPARSE_OK;
    g_last_hip_error = (int)e;
    return SKIPARSE_EHIP;
}

static bool bad_buffers(const void* operands, const float* sink) {
    return !operands || !sink || (reinterpret_cast<uintptr_t>(operands) & 15u) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3u) != 0;
}

}  // namespace skiparse_probe

using namespace skiparse_probe;

extern "C" {

int skiparse_mfma_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int dtype, int blocks, int iters,
                        double* flop, void* stream) {
    if (bad_buffers(operands, sink)) return SKIPARSE_EINVAL;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return SKIPARSE_EINVAL;
    if (dtype != SKIPARSE_BF16 && dtype != SKIPARSE_FP8_E4M3) return SKIPARSE_EUNSUPPORTED;
    if (operand_bytes < (size_t)MFMA_PROBE_OPERAND_BYTES || sink_bytes < (size_t)blocks * 256 * sizeof(float)) return SKIPARSE_EWORKSPACE;
    const double per_mfma = dtype == SKIPARSE_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 64;
    if (flop) *flop = per_mfma * 4.0 /* per iteration */ * iters * 4.0 /* wavefronts */ * blocks;
    return finish(launch_mfma_probe(operands, sink, dtype == SKIPARSE_FP8_E4M3, blocks, iters, (hipStream_t)stream));
}

int skiparse_mfma_lds_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int blocks, int iters, double* flop,
                            void* stream) {
    if (bad_buffers(operands, sink)) return SKIPARSE_EINVAL;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return SKIPARSE_EINVAL;
    if (operand_bytes < (size_t)MFMA_PROBE_OPERAND_BYTES || sink_bytes < (size_t)blocks * 256 * sizeof(float)) return SKIPARSE_EWORKSPACE;
    if (flop) *flop = 2.0 * 32 * 32 * 16 * 8.0 /* MFMAs per iteration */ * iters * 4.0 /* wavefronts */ * blocks;
    return finish(launch_mfma_lds_probe(operands, sink, blocks, iters, (hipStream_t)stream));
}

int skiparse_mfma_valu_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int valu_per_mfma, int blocks,
                             int iters, double* flop, void* stream) {
    if (bad_buffers(operands, sink)) return SKIPARSE_EINVAL;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return SKIPARSE_EINVAL;
    if (valu_per_mfma < 0 || valu_per_mfma > 8 || (valu_per_mfma & 1)) return SKIPARSE_EUNSUPPORTED;
    if (operand_bytes < (size_t)MFMA_PROBE_OPERAND_BYTES || sink_bytes < (size_t)blocks * 256 * sizeof(float)) return SKIPARSE_EWORKSPACE;
    if (flop) *flop = 2.0 * 32 * 32 * 16 * 2.0 /* MFMAs per iteration */ * iters * 4.0 /* wavefronts */ * blocks;
    return finish(launch_mfma_valu_probe(operands, sink, valu_per_mfma, blocks, iters, (hipStream_t)stream));
}

int skiparse_mfma8_valu_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int valu_per_mfma, int blocks,
                              int iters, double* flop, void* stream) {
    if (bad_buffers(operands, sink)) return SKIPARSE_EINVAL;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return SKIPARSE_EINVAL;
    if (valu_per_mfma < 0 || valu_per_mfma > 16 || (valu_per_mfma & 3)) return SKIPARSE_EUNSUPPORTED;
    if (operand_bytes < (size_t)MFMA_PROBE_OPERAND_BYTES || sink_bytes < (size_t)blocks * 256 * sizeof(float)) return SKIPARSE_EWORKSPACE;
    if (flop) *flop = 2.0 * 32 * 32 * 64 * 2.0 /* MFMAs per iteration */ * iters * 4.0 /* wavefronts */ * blocks;
    return finish(launch_mfma8_valu_probe(operands, sink, valu_per_mfma, blocks, iters, (hipStream_t)stream));
}

int skiparse_mfma_chain_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int chain, int blocks, int iters,
                              double* flop, void* stream) {
    if (bad_buffers(operands, sink)) return SKIPARSE_EINVAL;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return SKIPARSE_EINVAL;
    if (chain != 1 && chain != 2 && chain != 4 && chain != 8) return SKIPARSE_EUNSUPPORTED;
    if (operand_bytes < (size_t)MFMA_PROBE_OPERAND_BYTES || sink_bytes < (size_t)blocks * 256 * sizeof(float)) return SKIPARSE_EWORKSPACE;
    if (flop) *flop = 2.0 * 32 * 32 * 16 * 4.0 * chain /* MFMAs per iteration */ * iters * 4.0 /* wavefronts */ * blocks;
    return finish(launch_mfma_chain_probe(operands, sink, chain, blocks, iters, (hipStream_t)stream));
}

int skiparse_lds_read_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int kind, int blocks, int iters,
                            double* bytes, void* stream) {
    if (bad_buffers(operands, sink)) return SKIPARSE_EINVAL;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return SKIPARSE_EINVAL;
    if (kind < 0 || kind > 2) return SKIPARSE_EUNSUPPORTED;
    if (operand_bytes < (size_t)MFMA_PROBE_OPERAND_BYTES || sink_bytes < (size_t)blocks * 512 * sizeof(float)) return SKIPARSE_EWORKSPACE;
    if (bytes) *bytes = (kind == 0 ? 1024.0 : 512.0) * 16.0 /* reads per iteration */ * iters * 8.0 /* wavefronts */ * blocks;
    return finish(launch_lds_read_probe(operands, sink, kind, blocks, iters, (hipStream_t)stream));
}

int skiparse_probe_device_info(int device, int* compute_units, int* clock_khz) {
    if (device < 0 || !compute_units || !clock_khz) return SKIPARSE_EINVAL;
    hipError_t e = hipDeviceGetAttribute(compute_units, hipDeviceAttributeMultiprocessorCount, device);
    if (e == hipSuccess) e = hipDeviceGetAttribute(clock_khz, hipDeviceAttributeClockRate, device);
    return finish(e);
}

int skiparse_probe_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
