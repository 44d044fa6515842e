// FP8 (E4M3) flash-attention forward for gfx950: the 8-bit variant of the Skiparse attention path.
//
// Inputs are the quantised tensors in the sparse layout (one row of head_dim bytes per position and head) with one
// float32 scale per (subsequence, head, block of 128 positions); the output is bf16 in the original layout.
//     S = (q8 k8^T) * sq * sk * scale          logits, fp32
//     P = exp(S - m)                           fp32; the reference m is only raised when the scaled probabilities of a tile
//                                              would not fit E4M3 (row-sum guard, see below)
//     P8 = e4m3(P * sv / sv_max * 16)          the key block's V scale is folded into the probabilities
//     O  = (P8 v8) * sv_max / 16 / sum(P)      fp32 accumulation, bf16 result
// Both products use v_mfma_f32_32x32x64_f8f6f4 (64-deep contraction, twice the bf16 rate), transposed as in the bf16
// kernel (S^T = K Q^T, O^T = V^T P^T) so that each lane owns one query.  A workgroup is 4 wavefronts x 32 queries; a
// wavefront's queries lie inside one 128-position scale block; keys are walked in tiles of 64, which never straddle one.
//   * The probabilities leave the accumulators as 16 values per 32-key block in the accumulator's key order (4h..4h+3,
//     8+4h..); packed to bytes, one v_permlane32_swap per 16 keys turns that into 8 consecutive keys per lane half,
//     which is the order ds_read_b64_tr_b8 (transposing LDS read for bytes) delivers V^T in.
//   * K/V tiles of 64 keys go from global memory straight into LDS (global_load_lds_dwordx4: no staging registers, no LDS
//     stores), double buffered.  Rows are packed (head_dim bytes); the position of a row's 16-byte chunk is XOR-swizzled with
//     the row number (lds_swizzle8) so that the 16-byte fragment reads of K (16 consecutive rows) and the transposing byte
//     reads of V^T (8 rows x 32 bytes per phase) both touch every bank once.
#include <type_traits>

#include "kernels.h"
#include "lds_layout.h"

namespace skiparse {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define LDS_PTR(T) __attribute__((address_space(3))) T*

constexpr int KT8 = 64;            // keys per tile = contraction depth of one PV MFMA
constexpr int NW8 = 4;             // wavefronts per workgroup: 128 queries (one scale block) share each K/V tile
constexpr int WAVES_PER_SIMD8 = 3; // three workgroups per compute unit: the kernel is not software-pipelined, the overlap of one
                                   // wavefront's exponentials with another's MFMAs comes from occupancy (needs <= 168 VGPRs)
constexpr int NT8 = 64 * NW8;
constexpr float P_GAIN = 16.0f;    // probabilities are multiplied by (sv / sv_max) * 16 before the E4M3 cast

__device__ inline void lane_pair_f(float x, float& lo, float& hi) {
    const unsigned a = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];  // copy out before casting (see the bf16 kernel)
    lo = __uint_as_float(r0);
    hi = __uint_as_float(r1);
}

// PAD: any-resolution mode (Sec. 3.2): positions run over the grid padded to multiples of s*s (the quantiser has put zero codes at the
// padding positions); a padding position is a masked key (a -inf bias per staged row, formed a tile ahead by one wavefront and added
// to the logits) and a skipped query.
template <int D, bool PAD>
__attribute__((amdgpu_waves_per_eu(WAVES_PER_SIMD8, WAVES_PER_SIMD8)))
__global__ __launch_bounds__(NT8) void attn_fwd_fp8_kernel(Fp8AttnArgs a, uint32_t q_tiles, uint32_t total, uint32_t per_xcd) {
    constexpr int NJ = D / 64;         // 64-channel MFMA steps of S^T = K Q^T
    constexpr int MT = D / 32;         // 32-channel blocks of O^T
    constexpr int RB = D;              // row bytes in LDS (packed rows, swizzled chunk positions)
    constexpr int CH = D / 16;         // 16-byte chunks per row
    constexpr int RPI = 64 / CH;       // rows filled by one direct-to-LDS instruction of a wavefront
    constexpr int IPW = CH >= NW8 ? CH / NW8 : 1;  // such instructions per wavefront, tensor and tile (with more wavefronts than instructions only the first CH stage)
    constexpr int STAGERS = CH >= NW8 ? NW8 : CH;
    constexpr int TILE_BYTES = KT8 * RB;
    static_assert(IPW * STAGERS == CH, "a tile is CH instructions, spread evenly over the staging wavefronts");
    // separate arrays so that the compiler can tell the tile being filled from the one being read
    __shared__ __attribute__((aligned(1024))) char kbuf0[TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char kbuf1[TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char vbuf0[TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char vbuf1[TILE_BYTES];
    __shared__ float sv_part[NW8];
    __shared__ __attribute__((aligned(16))) float kbias[2][KT8];  // PAD only: 0 for a real key of the tile, -inf for padding
    __shared__ uint32_t kany[2];                                  // PAD only: non-zero if the tile holds any padding (most hold none)

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lq = lane & 31u, h = lane >> 5;
    const uint32_t xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
    const uint32_t lin = xcd * per_xcd + idx;  // each XCD owns a contiguous range of the (unit, tile) order
    if (lin >= total) return;
    const uint32_t unit = lin / q_tiles, qt = lin - unit * q_tiles;  // unit = sb * heads + head
    const uint32_t sb = unit / (uint32_t)a.heads, head = unit - sb * (uint32_t)a.heads;
    const uint32_t n_seq = (uint32_t)a.g.n_sub, n_blk = a.n_blk;
    const uint32_t pq_ = sb / (uint32_t)a.B, b0_ = sb - pq_ * (uint32_t)a.B;
    const uint32_t p_ = a.g.mode == MODE_DENSE ? 0u : pq_ / (uint32_t)a.g.s, q_ = a.g.mode == MODE_DENSE ? 0u : pq_ - p_ * (uint32_t)a.g.s;
    // one wavefront (they take turns) marks the keys of a tile: lane = key
    auto mark_keys = [&](uint32_t t) __attribute__((always_inline)) {
        const uint32_t j = t * KT8 + lane;
        bool real = false;
        if (j < n_seq) (void)src_token_padded(a.g, p_, q_, j, &real);
        kbias[t & 1u][lane] = real ? 0.f : -INFINITY;
        const unsigned long long pads = __builtin_amdgcn_ballot_w64(!real);
        if (lane == 0) kany[t & 1u] = pads != 0 ? 1u : 0u;
    };
    const size_t C = (size_t)a.heads * D;  // bytes per position in the sparse layout
    const size_t unit_off = ((size_t)sb * n_seq) * C + (size_t)head * D;
    const unsigned char* Qg = (const unsigned char*)a.q8 + unit_off;
    const unsigned char* Kg = (const unsigned char*)a.k8 + unit_off;
    const unsigned char* Vg = (const unsigned char*)a.v8 + unit_off;
    const float* skp = a.sk + (size_t)unit * n_blk;
    const float* svp = a.sv + (size_t)unit * n_blk;

    // largest V scale of the unit: the probabilities carry sv / sv_max, the output is multiplied by sv_max at the end
    float svm = 0.f;
    for (uint32_t i = tid; i < n_blk; i += NT8) svm = fmaxf(svm, svp[i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) svm = fmaxf(svm, __shfl_xor(svm, off));
    if (lane == 0) sv_part[wave] = svm;
    __syncthreads();
    float sv_max = sv_part[0];
#pragma unroll
    for (int i = 1; i < NW8; i++) sv_max = fmaxf(sv_max, sv_part[i]);
    const float p_gain = P_GAIN / sv_max;

    // Q fragments: lane = query lq, 32 consecutive channels starting at 64*j + 32*h
    const uint32_t jq = qt * (32u * NW8) + wave * 32u + lq;
    bool q_valid = jq < n_seq;
    uint32_t q_tok = 0;  // PAD: the query's token in the unpadded tensor
    if (PAD) {
        bool real = false;
        q_tok = src_token_padded(a.g, p_, q_, q_valid ? jq : 0u, &real);
        q_valid = q_valid && real;
    }
    const size_t q_off = (size_t)(q_valid ? jq : n_seq - 1u) * C;
    i32x8 qf[NJ];
#pragma unroll
    for (int j = 0; j < NJ; j++) qf[j] = *(const i32x8*)(Qg + q_off + 64 * j + 32 * h);
    // a wavefront's 32 queries lie inside one 128-position scale block (clamped for wavefronts past the end)
    const uint32_t q_blk = (qt * (32u * NW8) + wave * 32u) / 128u;
    const float cq = a.scale * 1.4426950408889634f * a.sq[(size_t)unit * n_blk + (q_blk < n_blk ? q_blk : n_blk - 1u)];

    // staging: lane l of a direct load fetches, for row l/CH of the instruction's RPI rows, the chunk that the swizzle puts at
    // position l%CH; its 16 bytes land at the instruction's LDS base + 16*l
    uint32_t st_row[IPW], st_cb[IPW];
#pragma unroll
    for (int i = 0; i < IPW; i++) {
        st_row[i] = (wave * IPW + i) * RPI + lane / CH;
        st_cb[i] = ((lane % CH) ^ lds_swizzle8<D>(st_row[i])) * 16u;
    }
    auto issue_tile = [&](uint32_t t, char* kb, char* vb) __attribute__((always_inline)) {
        if (STAGERS < NW8 && wave >= (uint32_t)STAGERS) return;
#pragma unroll
        for (int i = 0; i < IPW; i++) {
            uint32_t j = t * KT8 + st_row[i];
            j = j < n_seq ? j : n_seq - 1u;  // rows past the end repeat the last row; their logits are masked
            const uint32_t off = j * (uint32_t)C + st_cb[i];  // fits 32 bits: checked on the host
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Kg + off),
                                             (LDS_PTR(void))(kb + (wave * IPW + i) * 1024u), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Vg + off),
                                             (LDS_PTR(void))(vb + (wave * IPW + i) * 1024u), 16, 0, 0);
        }
    };
    auto tile_landed = [&]() __attribute__((always_inline)) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

    f32x16 oacc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) oacc[mt][r] = 0.f;
    float m_ref = -INFINITY, l_run = 0.f;  // m_ref in log2 units of the scaled logits

    // K fragment of 64-channel step j: row lq (+ 32*kt), chunks 4j + 2h and 4j + 2h + 1 at their swizzled positions (adding 32*kt
    // to the row leaves the swizzle, which depends on the row's low four bits, unchanged)
    // (the position of chunk 4j + e + 2h is that of chunk 2h with (4j + e) * 16 XORed in: one register, an XOR per read)
    const uint32_t k_rd0 = lq * RB + ((2 * h) ^ lds_swizzle8<D>(lq)) * 16u;
    // transposing byte read: a 16-lane group covers 8 keys x 16 channels; lane i addresses key i/2, channels 8*(i%2)..
    const uint32_t li = lane & 15u, lgrp = (lane >> 4) & 1u;
    const uint32_t v_row = 8 * h + (li >> 1);  // + 16*g16 (same swizzle); chunk 2*mt + lgrp: XOR mt * 32 into the position of chunk lgrp
    const uint32_t v_rd0 = v_row * RB + (lgrp ^ lds_swizzle8<D>(v_row)) * 16u + 8 * (li & 1u);

    const uint32_t n_kt = (n_seq + KT8 - 1) / KT8;
    issue_tile(0, kbuf0, vbuf0);
    if (PAD && wave == 0) mark_keys(0);
    tile_landed();
    __syncthreads();

    float sk_cur = skp[0], sv_cur = svp[0], sk_nxt, sv_nxt;
    // one key tile; LAST (compile time) marks the final tile, the only one that may hold keys past the end: the masking code must
    // not be in the other tiles' path at all (the compiler turns a run-time test into 32 compares and selects per tile)
    // The parity of the tile (which buffers) is a compile-time constant as well.
    auto tile_body = [&](auto LASTC, auto PARC, uint32_t t) __attribute__((always_inline)) {
        constexpr bool LAST = decltype(LASTC)::value;
        constexpr int PARITY = decltype(PARC)::value;  // t & 1
        const bool more = !LAST;
        const char* kb = PARITY ? kbuf1 : kbuf0;
        const char* vb = PARITY ? vbuf1 : vbuf0;
        // the next tile's loads have the whole tile to land (enqueued after the QK products instead: 13 % slower; one workgroup of
        // 12 wavefronts sharing a tile instead of three independent ones of 4: 7 % slower)
        if (more) issue_tile(t + 1, PARITY ? kbuf0 : kbuf1, PARITY ? vbuf0 : vbuf1);
        if (PAD && more && wave == ((t + 1u) & (uint32_t)(NW8 - 1))) mark_keys(t + 1u);  // read after this tile's closing barrier
        const float ct = cq * sk_cur;        // logits -> log2 units for this key block
        const float pg = sv_cur * p_gain;    // V scale of this key block, relative to the largest, times the gain
        {   // the next tile's scales are fetched a tile ahead so that no tile waits for them
            uint32_t nb = (t + 1u) >> 1;
            nb = nb < n_blk ? nb : n_blk - 1u;
            sk_nxt = skp[nb];
            sv_nxt = svp[nb];
        }

        // S^T = K Q^T: two blocks of 32 keys
        f32x16 sacc[2];
#pragma unroll
        for (int kt = 0; kt < 2; kt++) {
#pragma unroll
            for (int r = 0; r < 16; r++) sacc[kt][r] = 0.f;
#pragma unroll
            for (int j = 0; j < NJ; j++) {
                const i32x4 k0 = *(const i32x4*)(kb + (k_rd0 ^ (uint32_t)((4 * j) * 16)) + kt * 32 * RB);
                const i32x4 k1 = *(const i32x4*)(kb + (k_rd0 ^ (uint32_t)((4 * j + 1) * 16)) + kt * 32 * RB);
                const i32x8 kf = __builtin_shufflevector(k0, k1, 0, 1, 2, 3, 4, 5, 6, 7);
                sacc[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf, qf[j], sacc[kt], 0, 0, 0, 0, 0, 0);
            }
        }
        if (PAD && __builtin_amdgcn_readfirstlane(kany[PARITY]) != 0) {
            // register r of block kt is key 32*kt + 8*(r/4) + 4*h + r%4; positions past the end carry -inf as well
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const f32x4 b4 = *(const f32x4*)&kbias[PARITY][kt * 32 + 8 * i + 4 * h];
#pragma unroll
                    for (int e = 0; e < 4; e++) sacc[kt][4 * i + e] += b4[e];
                }
        } else if (!PAD && LAST && (n_seq % KT8) != 0) {
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const uint32_t key = t * KT8 + kt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                    sacc[kt][r] = key < n_seq ? sacc[kt][r] : -INFINITY;
                }
        }
        // Online softmax without a per-tile maximum.  The exponentials are taken against the reference the row already
        // has, with log2 of the tile's probability gain folded into the exponent, so one fma and one exp per key give
        // P * gain directly.  Guard: E4M3 has no infinity and the conversion returns NaN above 448, so if a lane's 32
        // scaled probabilities add up to 448 or more (always on the first tile, where the reference is -inf) the
        // wavefront takes the rare path: true maximum, reference raised, tile redone.
        const float lg = __builtin_amdgcn_logf(pg);   // log2 of the gain of this key block
        const float inv_pg = __builtin_amdgcn_rcpf(pg);
        auto probs = [&](float mref_eff, i32x8& dst) __attribute__((always_inline)) -> float {
            float lsum = 0.f;
#pragma unroll
            for (int kt = 0; kt < 2; kt++) {
                int w[4];  // dword i of the block: keys 8*i + 4*h + 0..3
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    float pe[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        pe[e] = __builtin_amdgcn_exp2f(fmaf(sacc[kt][4 * i + e], ct, -mref_eff));
                        lsum += pe[e];
                    }
                    const int pk = __builtin_amdgcn_cvt_pk_fp8_f32(pe[0], pe[1], 0, false);
                    w[i] = __builtin_amdgcn_cvt_pk_fp8_f32(pe[2], pe[3], pk, true);
                }
#pragma unroll
                for (int m2 = 0; m2 < 2; m2++) {
                    // lanes l / l^32 hold keys (4h.., 8+4h..) of the 16-key group; after the swap each holds 8 consecutive keys
                    const auto sw = __builtin_amdgcn_permlane32_swap((unsigned)w[2 * m2], (unsigned)w[2 * m2 + 1], false, false);
                    const unsigned s0 = sw[0], s1 = sw[1];
                    dst[(kt * 2 + m2) * 2] = (int)s0;
                    dst[(kt * 2 + m2) * 2 + 1] = (int)s1;
                }
            }
            return lsum;
        };
        i32x8 pb;  // B operand of O^T += V^T P^T: 32 byte slots per lane half, slot 8*g16 + e <-> key 16*g16 + 8*h + e
        float lsum = probs(m_ref - lg, pb);
        float alpha = 1.0f;
        bool rescale = false;  // wave-uniform
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(lsum < 448.0f)) != 0, 0)) {
            float mx = sacc[0][0];
#pragma unroll
            for (int kt = 0; kt < 2; kt++)
#pragma unroll
                for (int r = 0; r < 16; r++) mx = fmaxf(mx, sacc[kt][r]);
            float lo, hi;
            lane_pair_f(mx, lo, hi);
            const float m_new = fmaxf(m_ref, fmaxf(lo, hi) * ct);
            // a tile of nothing but padding before any real key (any-resolution mode): the reference stays -inf, nothing to rescale,
            // and the exponentials are taken against 0 so that the masked logits give exp2(-inf) = 0
            alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_ref - m_new);  // 0 on the first tile with a real key
            m_ref = m_new;
            lsum = probs(m_new == -INFINITY ? -lg : m_ref - lg, pb);  // now every probability is at most the gain (<= 16)
            rescale = true;
        }
        l_run = fmaf(l_run, alpha, lsum * inv_pg);
        if (__builtin_expect(rescale, 0)) {  // a block of its own: nothing but the in-place multiplies
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int r = 0; r < 16; r++) oacc[mt][r] *= alpha;
        }
        // O^T += V^T P^T: one 64-key MFMA per 32-channel block
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            i32x8 vf;
#pragma unroll
            for (int g16 = 0; g16 < 4; g16++) {
                const i32x2 t8 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((LDS_PTR(i32x2))(LDS_PTR(char))(vb + (v_rd0 ^ (uint32_t)(mt * 32)) + g16 * 16 * RB));
                vf[2 * g16] = t8[0];
                vf[2 * g16 + 1] = t8[1];
            }
            oacc[mt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vf, pb, oacc[mt], 0, 0, 0, 0, 0, 0);
        }
        sk_cur = sk_nxt;
        sv_cur = sv_nxt;
        tile_landed();
        __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    uint32_t t = 0;
    for (; t + 2 < n_kt; t += 2) {
        tile_body(std::false_type{}, P0{}, t);
        tile_body(std::false_type{}, P1{}, t + 1u);
    }
    if (t + 1 < n_kt) {
        tile_body(std::false_type{}, P0{}, t);
        tile_body(std::true_type{}, P1{}, t + 1u);
    } else {
        tile_body(std::true_type{}, P0{}, t);
    }

    // epilogue: O = O^T * sv_max / gain / l, bf16, scattered to the original layout
    float llo, lhi;
    lane_pair_f(l_run, llo, lhi);
    const float inv = sv_max / (P_GAIN * (llo + lhi));
    if (q_valid) {
        const size_t row = (size_t)b0_ * (uint32_t)a.g.n_tok + (PAD ? q_tok : src_token(a.g, p_, q_, jq));
        __bf16* orow = (__bf16*)a.out + row * C + (size_t)head * D;
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; e++) o[e] = (__bf16)(oacc[mt][g * 4 + e] * inv);
                *(bf16x4*)(orow + mt * 32 + g * 8 + 4 * h) = o;
            }
    }
}

template <int D, bool PAD>
static hipError_t launch_fp8_t(const Fp8AttnArgs& a, hipStream_t stream) {
    const uint32_t s2 = a.g.mode == MODE_DENSE ? 1u : (uint32_t)(a.g.s * a.g.s);
    const uint32_t n_units = (uint32_t)a.B * s2 * (uint32_t)a.heads;
    const uint32_t q_tiles = ((uint32_t)a.g.n_sub + 32u * NW8 - 1u) / (32u * NW8);
    const uint64_t total = (uint64_t)n_units * q_tiles;
    if (total > 0x7ffffff0ull) return hipErrorInvalidConfiguration;
    const uint32_t per_xcd = (uint32_t)((total + 7u) / 8u);
    attn_fwd_fp8_kernel<D, PAD><<<8u * per_xcd, NT8, 0, stream>>>(a, q_tiles, (uint32_t)total, per_xcd);
    return hipGetLastError();
}

hipError_t launch_attn_fp8(const Fp8AttnArgs& a, hipStream_t stream) {
    if (a.head_dim == 128) return a.pad ? launch_fp8_t<128, true>(a, stream) : launch_fp8_t<128, false>(a, stream);
    if (a.head_dim == 64) return a.pad ? launch_fp8_t<64, true>(a, stream) : launch_fp8_t<64, false>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace skiparse
