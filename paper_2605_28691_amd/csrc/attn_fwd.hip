// bf16 flash-attention forward for gfx950, with the Skiparse row addressing folded in.
//
// Computes, for every attention unit (a subsequence or batch element, and a head),
//     O = softmax(Q K^T * scale) V                      (Sec. 3.1: attention inside each subsequence)
// without ever forming the N x N matrix: keys are walked in tiles of 64 with a running row maximum and row sum.
//
// Mapping onto the hardware
//   * One workgroup = 4 wavefronts; each wavefront owns QT tiles of 32 query rows for the whole key walk.
//   * The products are formed transposed, S^T = K Q^T and O^T = V^T P^T, with v_mfma_f32_32x32x16_bf16.  In the
//     32x32 accumulator layout lane l holds column l%32, so every lane owns ONE query: its 16 registers per 32-key
//     block are 16 keys of that query, the row maximum and sum are in-lane loops plus one exchange with lane l^32,
//     and the exponentiated accumulator registers, rounded to bf16, ARE the B operand of the second product -- the
//     probabilities never leave registers.
//   * K and V tiles are staged through LDS (global -> registers -> LDS, double buffered, one barrier per tile).
//     K is read back as the A operand with 16-byte reads; V^T is read with ds_read_b64_tr_b16, the gfx950
//     transposing LDS read, so V stays row-major in LDS.
//   * The key order inside a 16-key MFMA step is whatever the accumulator layout gives (keys 4h..4h+3 and
//     8+4h..8+4h+3 for lane half h); V^T is fetched in the same order, so no shuffle is needed.
//   * Row addresses come from src_token(): in the dense mode position j is row j, in the sparse modes it is the
//     token the Skiparse rearrangement (Algorithm 1) would have put at position j, so q, k, v are read and out is
//     written in the original layout and no permuted copy exists.
//   * Workgroups are numbered so that all query tiles of one unit run on the same XCD (workgroup id mod 8 selects
//     the XCD under round-robin dispatch) and walk K/V in step: the per-XCD L2 then serves the re-reads.
#include "kernels.h"

namespace skiparse {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

#define LDS_PTR(T) __attribute__((address_space(3))) T*

constexpr int KT = 64;          // keys per tile
constexpr int NTHREADS = 256;   // 4 wavefronts
constexpr float RESCALE_LOG2 = 8.0f;  // the running maximum is only raised when it grew by more than 2^8

template <int D>
struct Tile {
    static constexpr int CHUNKS = D / 8;                 // 16-byte chunks per row
    static constexpr int ROWS_PER_PASS = NTHREADS / CHUNKS;
    static constexpr int PASSES = KT / ROWS_PER_PASS;
    static constexpr int K_STRIDE = D * 2 + 16;          // bytes; +16 spreads the 16-byte reads of 16 rows over all banks
    static constexpr int V_STRIDE = D * 2 + 64;          // bytes; +64 keeps the 4 rows of a transposing read on distinct banks
    static constexpr int K_BYTES = KT * K_STRIDE;
    static constexpr int V_BYTES = KT * V_STRIDE;
    static constexpr int BUF_BYTES = K_BYTES + V_BYTES;
};

// Exchange between lanes l and l^32 (the two halves of one query's keys) with v_permlane32_swap: afterwards `lo` is
// the value of the pair's lower lane and `hi` that of its upper lane, in both lanes.  The two results are copied into
// scalars before any cast: a bit-cast applied directly to an element of the returned vector reads element 0 twice.
__device__ inline void lane_pair(float x, float& lo, float& hi) {
    const unsigned a = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    lo = __uint_as_float(r0);
    hi = __uint_as_float(r1);
}
__device__ inline float lane_pair_max(float x) {
    float lo, hi;
    lane_pair(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ inline float lane_pair_sum(float x) {
    float lo, hi;
    lane_pair(x, lo, hi);
    return lo + hi;
}

template <int D, int QT>
__global__ __launch_bounds__(NTHREADS, (QT == 1 ? 2 : 1)) void attn_fwd_bf16_kernel(AttnArgs a, uint32_t q_tiles,
                                                                                    uint32_t n_units) {
    using TL = Tile<D>;
    constexpr int KS = D / 16;   // MFMA steps along head_dim for S^T = K Q^T
    constexpr int MT = D / 32;   // 32-row blocks of O^T
    constexpr int BR = 128 * QT; // query rows per workgroup
    __shared__ __attribute__((aligned(16))) char lds[2 * TL::BUF_BYTES];

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t lq = lane & 31u, h = lane >> 5;

    // workgroup -> (unit, query tile): id%8 is the XCD, each XCD owns units xcd, xcd+8, ...
    const uint32_t xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
    const uint32_t ul = idx / q_tiles, qt = idx - ul * q_tiles;
    const uint32_t unit = ul * 8u + xcd;
    if (unit >= n_units) return;
    const uint32_t bb = unit / (uint32_t)a.heads, head = unit - bb * (uint32_t)a.heads;
    uint32_t p = 0, q = 0, b = bb;
    if (a.g.mode != MODE_DENSE) {
        const uint32_t pq = bb / (uint32_t)a.B;
        b = bb - pq * (uint32_t)a.B;
        p = pq / (uint32_t)a.g.s;
        q = pq - p * (uint32_t)a.g.s;
    }
    const uint32_t n_seq = (uint32_t)a.g.n_sub;
    const size_t C = (size_t)a.heads * D;
    const size_t unit_off = (size_t)b * (uint32_t)a.g.n_tok * C + (size_t)head * D;  // elements
    const __bf16* Qg = (const __bf16*)a.q + unit_off;
    const __bf16* Kg = (const __bf16*)a.k + unit_off;
    const __bf16* Vg = (const __bf16*)a.v + unit_off;
    __bf16* Og = (__bf16*)a.out + unit_off;

    // ---- Q fragments (B operand of S^T = K Q^T): lane = query lq, 8 consecutive channels starting at 16*ks + 8*h
    bf16x8 qf[QT][KS];
    size_t q_row_off[QT];
    bool q_valid[QT];
#pragma unroll
    for (int qi = 0; qi < QT; qi++) {
        const uint32_t j = qt * BR + (wave * QT + qi) * 32u + lq;
        q_valid[qi] = j < n_seq;
        q_row_off[qi] = (size_t)src_token(a.g, p, q, q_valid[qi] ? j : n_seq - 1u) * C;
#pragma unroll
        for (int ks = 0; ks < KS; ks++)
            qf[qi][ks] = *(const bf16x8*)(Qg + q_row_off[qi] + ks * 16 + 8 * h);
    }

    // ---- staging: thread -> (row r0 + pass*ROWS_PER_PASS, 16-byte chunk c) of a K/V tile
    const uint32_t st_c = tid % TL::CHUNKS, st_r = tid / TL::CHUNKS;
    u32x4 kreg[TL::PASSES], vreg[TL::PASSES];
    auto load_tile = [&](uint32_t t) {
#pragma unroll
        for (int ps = 0; ps < TL::PASSES; ps++) {
            uint32_t j = t * KT + st_r + ps * TL::ROWS_PER_PASS;
            j = j < n_seq ? j : n_seq - 1u;  // rows past the end are masked later; read a valid row instead
            const size_t off = (size_t)src_token(a.g, p, q, j) * C + st_c * 8;
            kreg[ps] = *(const u32x4*)(Kg + off);
            vreg[ps] = *(const u32x4*)(Vg + off);
        }
    };
    auto store_tile = [&](uint32_t buf) {
        char* base = lds + buf * TL::BUF_BYTES;
#pragma unroll
        for (int ps = 0; ps < TL::PASSES; ps++) {
            const uint32_t r = st_r + ps * TL::ROWS_PER_PASS;
            *(u32x4*)(base + r * TL::K_STRIDE + st_c * 16) = kreg[ps];
            *(u32x4*)(base + TL::K_BYTES + r * TL::V_STRIDE + st_c * 16) = vreg[ps];
        }
    };

    // ---- running state: every lane tracks its own query (pairs l, l^32 hold the same values)
    f32x16 oacc[QT][MT];
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int qi = 0; qi < QT; qi++) {
        m_run[qi] = -INFINITY;
        l_run[qi] = 0.f;
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int r = 0; r < 16; r++) oacc[qi][mt][r] = 0.f;
    }
    const float c = a.scale * 1.4426950408889634f;  // logits are kept raw; exp(x*scale) = exp2(x*c)

    // LDS read offsets that do not depend on the tile
    const uint32_t k_rd = lq * TL::K_STRIDE + h * 16;  // + kt*32*K_STRIDE + ks*32
    // transposing V read: 16-lane group covers 4 keys x 16 channels; lane i of the group addresses key i/4, channels 4*(i%4)..
    const uint32_t li = lane & 15u, lgrp = (lane >> 4) & 1u;
    const uint32_t v_rd = (4 * h + (li >> 2)) * TL::V_STRIDE + (lgrp * 16 + 4 * (li & 3u)) * 2;  // + g16*16*V_STRIDE (+8 rows) + mt*64

    const uint32_t n_kt = (n_seq + KT - 1) / KT;
    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (uint32_t t = 0; t < n_kt; t++) {
        const bool more = t + 1 < n_kt;
        if (more) load_tile(t + 1);
        const char* kb = lds + (t & 1u) * TL::BUF_BYTES;
        const char* vb = kb + TL::K_BYTES;

        // S^T = K Q^T for two blocks of 32 keys
        f32x16 sacc[QT][2];
#pragma unroll
        for (int qi = 0; qi < QT; qi++)
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int r = 0; r < 16; r++) sacc[qi][kt][r] = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; kt++)
#pragma unroll
            for (int ks = 0; ks < KS; ks++) {
                const bf16x8 kf = *(const bf16x8*)(kb + k_rd + kt * 32 * TL::K_STRIDE + ks * 32);
#pragma unroll
                for (int qi = 0; qi < QT; qi++)
                    sacc[qi][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qi][ks], sacc[qi][kt], 0, 0, 0);
            }

        // keys past the end of the sequence (last tile only) get a logit of -inf
        if (!more && (n_seq % KT) != 0) {
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const uint32_t key = t * KT + kt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                    if (key >= n_seq) {
#pragma unroll
                        for (int qi = 0; qi < QT; qi++) sacc[qi][kt][r] = -INFINITY;
                    }
                }
        }

        // online softmax; probabilities become the B operand of O^T += V^T P^T
        bf16x8 pf[QT][4];
#pragma unroll
        for (int qi = 0; qi < QT; qi++) {
            float mx = sacc[qi][0][0];
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int r = 0; r < 16; r++) mx = fmaxf(mx, sacc[qi][kt][r]);
            mx = lane_pair_max(mx);
            const float m_cand = fmaxf(m_run[qi], mx);
            const bool grow = (m_cand - m_run[qi]) * c > RESCALE_LOG2;
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float alpha = __builtin_amdgcn_exp2f((m_run[qi] - m_cand) * c);
                l_run[qi] *= alpha;
#pragma unroll
                for (int mt = 0; mt < MT; mt++)
#pragma unroll
                    for (int r = 0; r < 16; r++) oacc[qi][mt][r] *= alpha;
                m_run[qi] = m_cand;
            }
            const float mc = m_run[qi] * c;
            float lsum = 0.f;
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int g = 0; g < 2; g++) {
                    bf16x8 pk;
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        const float pe = __builtin_amdgcn_exp2f(fmaf(sacc[qi][kt][g * 8 + e], c, -mc));
                        lsum += pe;
                        pk[e] = (__bf16)pe;
                    }
                    pf[qi][kt * 2 + g] = pk;
                }
            l_run[qi] += lsum;
        }

        // O^T += V^T P^T: 4 steps of 16 keys, MT blocks of 32 channels
#pragma unroll
        for (int g16 = 0; g16 < 4; g16++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const char* va = vb + v_rd + g16 * 16 * TL::V_STRIDE + mt * 64;
                const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(LDS_PTR(char))va);
                const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(LDS_PTR(char))(va + 8 * TL::V_STRIDE));
                const bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int qi = 0; qi < QT; qi++)
                    oacc[qi][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qi][g16], oacc[qi][mt], 0, 0, 0);
            }

        if (more) store_tile((t + 1) & 1u);
        __syncthreads();
    }

    // ---- epilogue: O = O^T / l, rounded to bf16; lane owns query lq, register r of block mt is channel 32*mt + 8*(r/4) + 4*h + r%4
#pragma unroll
    for (int qi = 0; qi < QT; qi++) {
        const float inv = 1.0f / lane_pair_sum(l_run[qi]);
        if (q_valid[qi]) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; e++) o[e] = (__bf16)(oacc[qi][mt][g * 4 + e] * inv);
                    *(bf16x4*)(Og + q_row_off[qi] + mt * 32 + g * 8 + 4 * h) = o;
                }
        }
    }
}

template <int D, int QT>
static hipError_t launch_t(const AttnArgs& a, hipStream_t stream) {
    const uint32_t s2 = a.g.mode == MODE_DENSE ? 1u : (uint32_t)(a.g.s * a.g.s);
    const uint32_t n_units = (uint32_t)a.B * s2 * (uint32_t)a.heads;
    const uint32_t q_tiles = ((uint32_t)a.g.n_sub + 128 * QT - 1) / (128 * QT);
    const uint32_t units_padded = (n_units + 7u) / 8u * 8u;
    const uint64_t blocks = (uint64_t)units_padded * q_tiles;
    if (blocks > 0x7fffffffull) return hipErrorInvalidConfiguration;
    attn_fwd_bf16_kernel<D, QT><<<(uint32_t)blocks, NTHREADS, 0, stream>>>(a, q_tiles, n_units);
    return hipGetLastError();
}

hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t stream) {
    if (a.head_dim == 128) return launch_t<128, 1>(a, stream);
    if (a.head_dim == 64) return launch_t<64, 1>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace skiparse
