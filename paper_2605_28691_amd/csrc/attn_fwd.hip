// bf16 flash-attention forward for gfx950, with the Skiparse row addressing folded in.
//
// Computes, for every attention unit (a subsequence or batch element, and a head),
//     O = softmax(Q K^T * scale) V                      (Sec. 3.1: attention inside each subsequence)
// without ever forming the N x N matrix: keys are walked in blocks of 32 with a running row maximum and row sum.
//
// Mapping onto the hardware
//   * One workgroup = 8 wavefronts (two per SIMD), each owning 32 query rows for the whole key walk: 256 queries share
//     every K/V tile that is brought into LDS, which halves the L2 -> LDS traffic per MFMA compared with 128 queries.
//     One workgroup per CU (<= 256 VGPRs per lane, 64 KiB LDS).
//   * The products are formed transposed, S^T = K Q^T and O^T = V^T P^T, with v_mfma_f32_32x32x16_bf16.  In the
//     32x32 accumulator layout lane l holds column l%32, so every lane owns ONE query: its 16 registers per 32-key
//     block are 16 keys of that query, and the exponentiated accumulator registers, rounded to bf16, ARE the B operand
//     of the second product -- the probabilities never leave registers.  The key order inside a 16-key MFMA step is
//     whatever the accumulator layout gives (keys 4h..4h+3 and 8+4h..8+4h+3 for lane half h); V^T is fetched in the
//     same order.
//   * Software pipeline over 32-key blocks: step b issues the MFMAs of  S(b+1) = K(b+1) Q^T  and  O += V(b-1)^T P(b-1)^T
//     and does the softmax arithmetic of block b on the vector ALU.  The three are independent inside a step, so the
//     matrix pipe and the vector ALU overlap within one wavefront as well as across the two on a SIMD.
//   * In the steady state the instruction order of a step is written out by hand and fixed with scheduling fences:
//     MFMAs of the two products alternate (so consecutive MFMAs never depend on each other), each followed by its share
//     of the exponentials, and every LDS fragment is read four MFMAs before its use (across the two steps of a window too).
//   * Reference maximum without a per-block maximum: the exponentials are taken against the reference the row already
//     has; the common path computes no maximum at all.  The guard is the row sum: if 16 probabilities of a lane add up
//     to 2^16 or more (always on the first block, where the reference is -inf) the wavefront takes a rare path that finds
//     the true maximum, redoes the block against it and rescales l; O is rescaled at the start of the next step in a
//     block that holds only the in-place multiplies.  Numerator and denominator always use the same reference, so the
//     result is exact up to rounding; probabilities up to 2^16 keep their relative precision in bf16, O and l are fp32.
//   * K and V tiles of 64 keys go from global memory straight into LDS (global_load_lds_dwordx4, no staging registers,
//     no LDS store instructions), double buffered, K one tile ahead of V (a window of two steps reads K tile W and V tile
//     W-1), one barrier per window; the loads of a tile are enqueued half a window before they are waited for (not earlier:
//     see the window loop).  LDS rows are packed (a direct load writes 64 consecutive 16-byte chunks) and bank conflicts are avoided by an XOR swizzle of
//     the chunk position with the row number, chosen so that both the 16-byte fragment reads of K (16 consecutive rows)
//     and the transposing reads of V^T (ds_read_b64_tr_b16, 4 consecutive rows of 64 bytes) touch every bank once; V
//     stays row-major in LDS.  (Three buffers with a two-window lead and a fence-free barrier measured slower.)
//   * Row addresses come from the Skiparse index map: in the dense mode position j is row j, in the sparse modes it is
//     the token the rearrangement (Algorithm 1) would have put at position j, so q, k, v are read and out is written in
//     the original layout and no permuted copy exists.  The rows' byte offsets are formed 8 tiles ahead, one tile (64 rows,
//     lane = row) per window by one wavefront in turn, and kept in a small ring in LDS from which every lane picks up the
//     two rows it fetches: the index arithmetic costs a wavefront one evaluation of the map per 8 tiles.
//   * Workgroups are numbered so that the query tiles of one unit run on the same XCD (workgroup id mod 8 selects
//     the XCD under round-robin dispatch; every XCD owns a contiguous eighth of the (unit, tile) order) and walk K/V in
//     step: the per-XCD L2 then serves the re-reads.
#include <type_traits>

#include "kernels.h"
#include "lds_layout.h"

namespace skiparse {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define LDS_PTR(T) __attribute__((address_space(3))) T*

constexpr int KT = 64;          // keys per staged tile (two 32-key blocks)
constexpr int NW = 8;            // wavefronts per workgroup: two per SIMD, all sharing one K/V tile in LDS
constexpr int NTHREADS = 64 * NW;
constexpr int ATTN_QT = 1;       // 32-query tiles per wavefront
constexpr int RING_AHEAD = NW;   // row offsets are formed this many tiles ahead, by one wavefront per window in turn
constexpr int RING = 16;         // tiles of row offsets (and key validity) kept in LDS: a slot is rewritten RING - RING_AHEAD windows after its last use
static_assert((NW & (NW - 1)) == 0 && (RING & (RING - 1)) == 0 && RING >= RING_AHEAD + 4, "ring sizes");
constexpr int LDS_AHEAD = 4;     // MFMA groups by which the LDS fragment reads run ahead in the steady state
constexpr float RESCALE_LOG2 = 8.0f;  // the reference maximum is only raised when it grew by more than 2^8

template <int D>
struct Tile {
    static constexpr int CH = D / 8;                     // 16-byte chunks per row
    static constexpr int RB = D * 2;                     // row bytes in LDS: rows are packed, bank conflicts are avoided by a swizzle
    static constexpr int RPI = 64 / CH;                  // rows covered by one direct-to-LDS instruction of a wavefront (64 chunks)
    static constexpr int IPW = CH / NW;                  // such instructions per wavefront and 64-row tile
    static constexpr int TILE_BYTES = KT * RB;
    static_assert(IPW >= 1 && IPW * NW == CH, "a tile is CH instructions, spread evenly over the wavefronts");
    // chunk c of row r is stored at chunk position c ^ swz(r): see lds_layout.h
    __host__ __device__ static constexpr uint32_t swz(uint32_t r) { return lds_swizzle<D>(r); }
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

// a value that is the same in every lane, moved to a scalar register
__device__ inline uint32_t uniform(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ inline size_t uniform(size_t x) {
    return ((size_t)uniform((uint32_t)(x >> 32)) << 32) | uniform((uint32_t)x);
}

// PAD selects the any-resolution mode (Sec. 3.2): positions run over the grid padded to multiples of s*s, padding positions
// are masked as keys (a 0 / -inf logit bias per staged row in LDS, from which the logits' accumulators start) and skipped as queries.
// Row of `out` for position j of subsequence sb of the input's sparse layout: the token's row in the original layout, or its
// row in the sparse layout of the other pattern (Alg. 1: tsa_to_orig / gsa_to_orig, tsa_to_gsa / gsa_to_tsa).
__device__ inline size_t scattered_row(const AttnArgs& a, uint32_t sb, uint32_t j) {
    const GridMap& gi = a.g_in;
    const uint32_t s = (uint32_t)gi.s, W = (uint32_t)gi.W, B = (uint32_t)a.out_B;
    const uint32_t pq = sb / B, b = sb - pq * B;
    const uint32_t n = src_token(gi, pq / s, pq % s, j);
    if (a.out_kind == OUT_ORIGINAL) return (size_t)b * (uint32_t)gi.n_tok + n;
    const uint32_t th = n / W, w = n - th * W;  // th = t*H + h
    uint32_t p, q, r, ws;
    if (gi.b != 0) {  // input group-wise -> output token-wise
        p = th % s;
        q = w % s;
        r = th / s;
        ws = w / s;
    } else {          // input token-wise -> output group-wise
        p = (th / s) % s;
        q = (w / s) % s;
        r = (th / (s * s)) * s + th % s;
        ws = (w / (s * s)) * s + w % s;
    }
    return ((size_t)(p * s + q) * B + b) * (uint32_t)gi.n_sub + r * (W / s) + ws;
}

template <int D, int QT, bool PAD>
__global__ __launch_bounds__(NTHREADS, (QT == 1 && NW == 4 ? 2 : 1)) void attn_fwd_bf16_kernel(AttnArgs a, uint32_t q_tiles, uint32_t total, uint32_t per_xcd) {
    using TL = Tile<D>;
    constexpr int KS = D / 16;     // MFMA steps along head_dim for S^T = K Q^T
    constexpr int MT = D / 32;     // 32-row blocks of O^T
    constexpr int BR = 32 * NW * QT;   // query rows per workgroup: QT tiles of 32 per wavefront
    // four separate arrays: the compiler must be able to tell that the tile being filled is not the tile being read
    __shared__ __attribute__((aligned(1024))) char kbuf0[TL::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char kbuf1[TL::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char vbuf0[TL::TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char vbuf1[TL::TILE_BYTES];
    __shared__ __attribute__((aligned(16))) uint32_t rowoff[RING][KT];        // byte offsets of the rows of the next tiles
    __shared__ __attribute__((aligned(16))) float kbias[RING][KT];            // PAD only: logit bias per row of a K tile, 0 = real key, -inf = padding

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = uniform(tid >> 6);
    const uint32_t lq = lane & 31u, h = lane >> 5;

    // workgroup -> (unit, query tile): id%8 is the XCD; each XCD owns a contiguous range of the (unit, tile) order, so that the
    // tiles of a unit run on one XCD (two at a range boundary) and the load is even for any number of units
    const uint32_t xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
    const uint32_t lin = xcd * per_xcd + idx;
    if (lin >= total) return;
    const uint32_t unit = lin / q_tiles, qt = lin - unit * q_tiles;
    const uint32_t bb = unit / (uint32_t)a.heads, head = unit - bb * (uint32_t)a.heads;
    uint32_t p = 0, q = 0, b0 = bb;
    if (a.g.mode != MODE_DENSE) {
        const uint32_t pq = bb / (uint32_t)a.B;
        b0 = bb - pq * (uint32_t)a.B;
        p = pq / (uint32_t)a.g.s;
        q = pq - p * (uint32_t)a.g.s;
    }
    const uint32_t n_seq = (uint32_t)a.g.n_sub;
    const size_t C = (size_t)a.heads * D;
    const size_t unit_off = uniform((size_t)b0 * (uint32_t)a.g.n_tok * C + (size_t)head * D);  // elements
    const __bf16* Qg = (const __bf16*)a.q + unit_off;
    const __bf16* Kg = (const __bf16*)a.k + unit_off;
    const __bf16* Vg = (const __bf16*)a.v + unit_off;
    __bf16* Og = (__bf16*)a.out + unit_off;

    // ---- Q fragments (B operand of S^T = K Q^T): lane = query lq, 8 consecutive channels starting at 16*ks + 8*h
    bf16x8 qf[QT][KS];
    bool q_valid[QT];
    size_t q_row_off[QT];
#pragma unroll
    for (int qi = 0; qi < QT; qi++) {
        const uint32_t jq = qt * BR + (wave * QT + qi) * 32u + lq;
        q_valid[qi] = jq < n_seq;
        if (PAD) {
            bool real;
            const uint32_t tok = src_token_padded(a.g, p, q, q_valid[qi] ? jq : 0u, &real);
            q_valid[qi] = q_valid[qi] && real;
            q_row_off[qi] = q_valid[qi] ? (size_t)tok * C : 0;  // padding queries read token 0 and store nothing
        } else {
            q_row_off[qi] = (size_t)src_token(a.g, p, q, q_valid[qi] ? jq : n_seq - 1u) * C;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ks++) qf[qi][ks] = *(const bf16x8*)(Qg + q_row_off[qi] + ks * 16 + 8 * h);
    }

    // ---- staging: K/V tiles of 64 rows go from global memory straight into LDS (global_load_lds_dwordx4: lane l's 16 bytes
    // land at the instruction's LDS base + 16*l, so one instruction of a wavefront fills RPI whole rows).  A wavefront issues IPW
    // such instructions per tile; lane l fetches, for row l/CH of the instruction's rows, the chunk that the swizzle puts at
    // position l%CH.  The row addresses come from the index map.
    // Byte offsets of the rows relative to the unit's base (they fit 32 bits: checked on the host) come from a small ring in LDS
    // that is filled RING_AHEAD tiles ahead: in every window ONE wavefront (they take turns) forms the 64 offsets of one tile, lane =
    // row, straight from the index map, and every lane of the workgroup later picks up the offsets of the rows it fetches.  The
    // index arithmetic thus costs each wavefront one evaluation per 8 tiles instead of one per tile and fetched row.
    const uint32_t row_bytes = (uint32_t)C * 2u;
    const uint32_t last_off = PAD ? 0u : src_token(a.g, p, q, n_seq - 1u) * row_bytes;  // rows past the end read the last valid row
    auto produce = [&](uint32_t tile) __attribute__((always_inline)) {
        const uint32_t j = tile * KT + lane, jc = j < n_seq ? j : n_seq - 1u;
        uint32_t off;
        if (PAD) {
            bool real;
            const uint32_t tok = src_token_padded(a.g, p, q, jc, &real);
            const bool valid = j < n_seq && real;
            off = valid ? tok * row_bytes : 0u;  // padding rows read token 0; their logits are masked
            kbias[tile % RING][lane] = valid ? 0.f : -INFINITY;
        } else {
            off = j < n_seq ? src_token(a.g, p, q, jc) * row_bytes : last_off;
        }
        rowoff[tile % RING][lane] = off;
    };
    uint32_t st_row[TL::IPW], st_cb[TL::IPW];
#pragma unroll
    for (int i = 0; i < TL::IPW; i++) {
        st_row[i] = (wave * TL::IPW + i) * TL::RPI + lane / TL::CH;  // row of the tile
        st_cb[i] = ((lane % TL::CH) ^ TL::swz(st_row[i])) * 16u;  // byte offset, inside the row, of the chunk this lane fetches
    }
    struct RowOffs {
        uint32_t off[TL::IPW];  // row offset + chunk offset of the lane's fetches of one tile (the same for K and V)
    };
    auto read_offs = [&](uint32_t tile) __attribute__((always_inline)) -> RowOffs {
        RowOffs o;
#pragma unroll
        for (int i = 0; i < TL::IPW; i++) o.off[i] = rowoff[tile % RING][st_row[i]] + st_cb[i];
        return o;
    };
    // enqueue the loads of one tile; they are complete (visible in LDS after the next barrier) once tile_landed() has returned
    auto issue_tile = [&](const __bf16* g, char* buf, const RowOffs& o) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TL::IPW; i++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)((const char*)g + o.off[i]),
                                             (LDS_PTR(void))(buf + (wave * TL::IPW + i) * 1024u), 16, 0, 0);
    };
    auto issue_k = [&](char* buf, const RowOffs& o) __attribute__((always_inline)) { issue_tile(Kg, buf, o); };
    auto issue_v = [&](char* buf, const RowOffs& o) __attribute__((always_inline)) { issue_tile(Vg, buf, o); };
    auto tile_landed = [&]() __attribute__((always_inline)) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

    // ---- running state: every lane tracks its own query (lanes l and l^32 hold the same m_ref; l_run is a partial sum)
    f32x16 oacc[QT][MT];
    f32x16 sreg[2][QT];     // S(b) lives in sreg[b & 1]
    bf16x8 preg[2][QT][2];  // P(b) lives in preg[b & 1][query tile][16-key half]
    float m_ref[QT], l_run[QT];
#pragma unroll
    for (int qi = 0; qi < QT; qi++) {
        m_ref[qi] = -INFINITY;
        l_run[qi] = 0.f;
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int r = 0; r < 16; r++) oacc[qi][mt][r] = 0.f;
    }
    const float c = a.scale * 1.4426950408889634f;  // logits are kept raw; exp(x*scale) = exp2(x*c)
    // A raised reference rescales O one step late: the factor is kept here and applied at the start of the next step
    // (after PV(b-1), before PV(b)), in a block of its own that holds nothing but the in-place multiplies.
    float alpha_pending[QT];
    bool pending = false;  // wave-uniform
#pragma unroll
    for (int qi = 0; qi < QT; qi++) alpha_pending[qi] = 1.f;
    auto apply_pending = [&]() __attribute__((always_inline)) {
        if (__builtin_expect(pending, 0)) {
#pragma unroll
            for (int qi = 0; qi < QT; qi++)
#pragma unroll
                for (int mt = 0; mt < MT; mt++)
#pragma unroll
                    for (int r = 0; r < 16; r++) oacc[qi][mt][r] *= alpha_pending[qi];
            pending = false;
        }
    };

    // LDS read offsets that do not depend on the tile
    uint32_t k_rd[KS];  // K fragment of MFMA step ks: row lq (+ 32 for the second half), chunk 2*ks + h at its swizzled position
#pragma unroll
    for (int ks = 0; ks < KS; ks++) k_rd[ks] = lq * TL::RB + (((uint32_t)(2 * ks) + h) ^ TL::swz(lq)) * 16u;
    // transposing V read: a 16-lane group covers 4 keys x 16 channels; lane i of the group addresses key i/4, channels 4*(i%4)..
    const uint32_t li = lane & 15u, lgrp = (lane >> 4) & 1u;
    uint32_t v_rd[2][MT];  // [second 4-row group][channel block]: + (half*32 + m2*16)*RB
#pragma unroll
    for (int sec = 0; sec < 2; sec++)
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            const uint32_t row = 4 * h + (li >> 2) + 8 * sec;  // adding 16*m2 + 32*half does not change the swizzle (low 4 bits)
            const uint32_t ch = (uint32_t)(mt * 4) + lgrp * 2 + ((li & 3u) >> 1);
            v_rd[sec][mt] = row * TL::RB + ((ch ^ TL::swz(row)) * 16u) + 8 * (li & 1u);
        }

    // Initial accumulator of the logits of 32-key block blkq: zero, or in the any-resolution mode the keys' bias (0 / -inf), which
    // masks the padding positions without any arithmetic of its own.  Register r of the block is key 8*(r/4) + 4*h + r%4.
    auto s_init = [&](uint32_t blkq) __attribute__((always_inline)) -> f32x16 {
        f32x16 v;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            f32x4 b4 = {0.f, 0.f, 0.f, 0.f};
            if (PAD) b4 = *(const f32x4*)&kbias[(blkq >> 1) % RING][(blkq & 1u) * 32u + 8 * i + 4 * h];
#pragma unroll
            for (int e = 0; e < 4; e++) v[4 * i + e] = b4[e];
        }
        return v;
    };
    // S(block blkq) = K(block) Q^T from K tile buffer kb, 32-key half `half`; each K fragment feeds all QT query tiles
    auto qk = [&](const char* kb, int half, f32x16 (&s)[QT], uint32_t blkq) __attribute__((always_inline)) {
        f32x16 acc[QT];
#pragma unroll
        for (int qi = 0; qi < QT; qi++) acc[qi] = s_init(blkq);
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
            const bf16x8 kf = *(const bf16x8*)(kb + k_rd[ks] + half * 32 * TL::RB);
#pragma unroll
            for (int qi = 0; qi < QT; qi++) {
                acc[qi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qi][ks], acc[qi], 0, 0, 0);
            }
        }
#pragma unroll
        for (int qi = 0; qi < QT; qi++) s[qi] = acc[qi];
    };
    // O^T += V(block)^T P(block)^T from V tile buffer vb, 32-key half `half`
    auto pv = [&](const char* vb, int half, const bf16x8 (&pf)[QT][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int m2 = 0; m2 < 2; m2++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const char* va = vb + (half * 32 + m2 * 16) * TL::RB;
                const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(LDS_PTR(char))(va + v_rd[0][mt]));
                const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(LDS_PTR(char))(va + v_rd[1][mt]));
                const bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int qi = 0; qi < QT; qi++)
                    oacc[qi][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qi][m2], oacc[qi][mt], 0, 0, 0);
            }
    };
    auto max3 = [](float x, float y, float z) __attribute__((always_inline)) { return fmaxf(fmaxf(x, y), z); };
    // exponentials of one block against the reference mc (= m_ref * c): bf16 probabilities and their fp32 sum
    auto exps = [&](const f32x16& s, float mc, bf16x8 (&pf)[2]) __attribute__((always_inline)) -> float {
        float lsum = 0.f;
#pragma unroll
        for (int g = 0; g < 2; g++) {
            bf16x8 pk;
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const f32x2 pe = {__builtin_amdgcn_exp2f(fmaf(s[g * 8 + e], c, -mc)), __builtin_amdgcn_exp2f(fmaf(s[g * 8 + e + 1], c, -mc))};
                const bf16x2 pb = __builtin_convertvector(pe, bf16x2);
                lsum += pe[0] + pe[1];  // row sum over the fp32 probabilities (two plain adds measure faster than one bf16 dot2)
                pk[e] = pb[0];
                pk[e + 1] = pb[1];
            }
            pf[g] = pk;
        }
        return lsum;
    };
    // One pipeline step for block b = 2W-1 (PAR = 1) or 2W (PAR = 0) of window W: K tile W in kb, V tile W-1 in vb.
    //   QK(b+1) -> sreg[PAR^1]   softmax(b): sreg[PAR] -> preg[PAR]   PV(b-1) with preg[PAR^1]
    // Generic form, used for the first and last windows (optional QK / PV, key masking); instruction order is left to
    // the compiler.  The steady-state windows use step_manual below.
    auto step = [&](auto DO_QK, auto DO_PV, auto MASK, auto PARC, uint32_t blk, const char* kb, const char* vb) __attribute__((always_inline)) {
        constexpr int PAR = decltype(PARC)::value;
        apply_pending();
        if (decltype(DO_QK)::value) qk(kb, PAR ^ 1, sreg[PAR ^ 1], blk + 1u);
        unsigned long long grow_mask = 0;
#pragma unroll
        for (int qi = 0; qi < QT; qi++) {
            f32x16& s = sreg[PAR][qi];
            if (decltype(MASK)::value && !PAD) {  // PAD: positions past the end carry the -inf bias like every padding position
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const uint32_t key = blk * 32u + 8 * (r >> 2) + 4 * h + (r & 3);
                    s[r] = key < n_seq ? s[r] : -INFINITY;
                }
            }
            const float mx = fmaxf(max3(max3(s[0], s[1], s[2]), max3(s[3], s[4], s[5]), max3(s[6], s[7], s[8])),
                                   max3(max3(s[9], s[10], s[11]), max3(s[12], s[13], s[14]), s[15]));
            float lo, hi;
            lane_pair(mx, lo, hi);
            const float m_new = max3(m_ref[qi], lo, hi);
            const bool grow = (m_new - m_ref[qi]) * c > RESCALE_LOG2;  // same in lanes l and l^32
            grow_mask |= __builtin_amdgcn_ballot_w64(grow);
            const float m_use = grow ? m_new : m_ref[qi];
            // 1 where the reference stays (also while it is still -inf: a block of nothing but masked keys), 0 on the first real block
            alpha_pending[qi] = grow ? __builtin_amdgcn_exp2f((m_ref[qi] - m_use) * c) : 1.0f;
            m_ref[qi] = m_use;
            // while no real key has been seen the reference is -inf: take 0 instead so that masked logits give exp2(-inf) = 0
            const float mc_use = m_use == -INFINITY ? 0.f : m_use * c;
            l_run[qi] = fmaf(l_run[qi], alpha_pending[qi], exps(s, mc_use, preg[PAR][qi]));
        }
        if (decltype(DO_PV)::value) pv(vb, PAR ^ 1, preg[PAR ^ 1]);
        pending = grow_mask != 0;  // O is rescaled at the start of the next step: after PV(b-1), before PV(b)
    };
    // Hand-ordered version of a full, unmasked step: the instruction order is fixed group by group with scheduling
    // fences, and the exponentials are taken against the reference the row already has, so the common path computes no
    // maximum at all: per key only fma, exp, half a bf16 pack and an add (row sum).  The guard is the row sum itself:
    // if a lane's 16 probabilities add up to 2^16 or more (always on the first block, where the reference is -inf), the
    // wavefront takes the rare path, which finds the true maximum, redoes the block's exponentials against it and rescales
    // O and l.  Probabilities up to 2^16 are harmless: bf16 keeps their relative precision and O, l are fp32.
    // LDS fragments are read two MFMA groups ahead and every fragment feeds the MFMAs of all QT query tiles.
    // In the any-resolution mode (PAD) the logits start from the keys' bias instead of zero (see s_init), nothing else differs;
    // `blk` is the block whose softmax this step does (the logits it forms are those of block blk + 1).
    // MFMA groups of a step alternate between the two products (PV, QK, PV, QK, ...: as many of each), so consecutive MFMAs never
    // depend on each other: group g is PV group g/2 when g is even and QK group g/2 when g is odd.
    constexpr int NPV = 2 * MT, NQK = KS, NG = NPV + NQK;
    static_assert(NPV == NQK, "the two products have the same number of MFMA groups");
    // LDS fragment of group g of the step with parity PAR (its PV and QK both work on the half PAR ^ 1 of their tiles)
    auto read_frag = [&](auto PARC, const char* kb, const char* vb, int g) __attribute__((always_inline)) -> bf16x8 {
        constexpr int PAR = decltype(PARC)::value;
        const int i = g / 2;
        if (g % 2 == 0) {  // fragment of PV group i: 16-key group m2 = i / MT, channel block mt = i % MT
            const char* va = vb + ((PAR ^ 1) * 32 + (i / MT) * 16) * TL::RB;
            const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(LDS_PTR(char))(va + v_rd[0][i % MT]));
            const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(LDS_PTR(char))(va + v_rd[1][i % MT]));
            return __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
        }
        return *(const bf16x8*)(kb + k_rd[i] + (PAR ^ 1) * 32 * TL::RB);
    };
    struct Frags {
        bf16x8 f[LDS_AHEAD];  // the first fragments of a step, read before it starts
    };
    auto first_frags = [&](auto PARC, const char* kb, const char* vb) __attribute__((always_inline)) -> Frags {
        Frags p;
#pragma unroll
        for (int g = 0; g < LDS_AHEAD; g++) p.f[g] = read_frag(PARC, kb, vb, g);
        return p;
    };
    // `pre`: the step's first LDS_AHEAD fragments, already on their way.  With NEXT the step's last groups fetch, instead of
    // nothing, the first fragments of the FOLLOWING step on the same tiles (the other parity) into `nxt`, so that the LDS
    // latency is exposed once per window instead of once per step.
    auto step_manual = [&](auto PARC, auto NEXTC, const char* kb, const char* vb, uint32_t blk, const Frags& pre, Frags& nxt) __attribute__((always_inline)) {
        constexpr int PAR = decltype(PARC)::value;
        constexpr bool NEXT = decltype(NEXTC)::value;
        using PARN = std::integral_constant<int, PAR ^ 1>;
        apply_pending();
        bf16x8 fr[NG];  // every fragment has its own name; lifetimes are short, so few registers are live at a time
#pragma unroll
        for (int g = 0; g < LDS_AHEAD; g++) fr[g] = pre.f[g];
        __builtin_amdgcn_sched_barrier(0);
        f32x16 acc[QT];
        float lsum[QT], mc[QT];
        bf16x8 pk[QT][2];
#pragma unroll
        for (int qi = 0; qi < QT; qi++) {
            lsum[qi] = 0.f;
            mc[qi] = m_ref[qi] * c;
        }
#pragma unroll
        for (int g = 0; g < NG; g++) {
            if (g + LDS_AHEAD < NG) fr[g + LDS_AHEAD] = read_frag(PARC, kb, vb, g + LDS_AHEAD);
            else if (NEXT) nxt.f[g + LDS_AHEAD - NG] = read_frag(PARN{}, kb, vb, g + LDS_AHEAD - NG);
            const int i = g / 2;
#pragma unroll
            for (int qi = 0; qi < QT; qi++) {
                if (g % 2 == 0) {
                    oacc[qi][i % MT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g], preg[PAR ^ 1][qi][i / MT], oacc[qi][i % MT], 0, 0, 0);
                } else {
                    if (i == 0) acc[qi] = s_init(blk + 1u);
                    acc[qi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g], qf[qi][i], acc[qi], 0, 0, 0);
                }
            }
            // this group's share of the exponentials: 16 / NG pairs of keys per query tile, rounded so that all 16 are covered
#pragma unroll
            for (int qi = 0; qi < QT; qi++) {
                const f32x16& s = sreg[PAR][qi];
#pragma unroll
                for (int e = 2 * (g * 8 / NG); e < 2 * ((g + 1) * 8 / NG); e += 2) {
                    const f32x2 pe = {__builtin_amdgcn_exp2f(fmaf(s[e], c, -mc[qi])), __builtin_amdgcn_exp2f(fmaf(s[e + 1], c, -mc[qi]))};
                    const bf16x2 pb = __builtin_convertvector(pe, bf16x2);
                    lsum[qi] += pe[0] + pe[1];
                    pk[qi][e / 8][e % 8] = pb[0];
                    pk[qi][e / 8][e % 8 + 1] = pb[1];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        unsigned long long redo = 0;
#pragma unroll
        for (int qi = 0; qi < QT; qi++) {
            sreg[PAR ^ 1][qi] = acc[qi];
            preg[PAR][qi][0] = pk[qi][0];
            preg[PAR][qi][1] = pk[qi][1];
            asm volatile("" ::"v"(preg[PAR][qi][0]), "v"(preg[PAR][qi][1]));
            redo |= __builtin_amdgcn_ballot_w64(!(lsum[qi] < 65536.0f));  // also catches inf and NaN
        }
        if (__builtin_expect(redo != 0, 0)) {
#pragma unroll
            for (int qi = 0; qi < QT; qi++) {
                f32x16& s = sreg[PAR][qi];
                const float mx = fmaxf(max3(max3(s[0], s[1], s[2]), max3(s[3], s[4], s[5]), max3(s[6], s[7], s[8])),
                                       max3(max3(s[9], s[10], s[11]), max3(s[12], s[13], s[14]), s[15]));
                float lo, hi;
                lane_pair(mx, lo, hi);
                const float m_new = max3(m_ref[qi], lo, hi);
                // while no real key has been seen (a block of nothing but padding) the reference stays -inf: factor 1, exponent 0
                alpha_pending[qi] = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f((m_ref[qi] - m_new) * c);  // 0 on the first real block
                m_ref[qi] = m_new;
                l_run[qi] = fmaf(l_run[qi], alpha_pending[qi], exps(s, m_new == -INFINITY ? 0.f : m_new * c, preg[PAR][qi]));
            }
            pending = true;
        } else {
#pragma unroll
            for (int qi = 0; qi < QT; qi++) l_run[qi] += lsum[qi];
        }
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;

    const uint32_t n_tiles = (n_seq + KT - 1) / KT;

    // Staging schedule.  Window W reads K tile W and V tile W-1 from LDS.  Between its two steps it enqueues the direct loads of
    // K tile W+1 (into the K buffer that window W-1 read) and of V tile W (into the V buffer that window W-1 read); they have half
    // a window to land and are waited for just before the window's closing barrier.  The row offsets of tile W+2 are picked up
    // from the ring in window W (so that the LDS read is not waited for), and tile W+RING_AHEAD's are formed by wavefront W%8.
    // ---- prologue: offsets of tiles 0..RING_AHEAD, K tile 0
    produce(wave);
    if (wave == 0) produce(RING_AHEAD);
    __syncthreads();
    RowOffs off_v = read_offs(0);  // offsets of the tile whose V is fetched next
    issue_k(kbuf0, off_v);
    RowOffs off_k = read_offs(1);  // offsets of the tile whose K is fetched next (rows past the end repeat the last row)
    tile_landed();
    __syncthreads();

    // ---- window 0: QK(0), then step 0 without PV
    {
        issue_k(kbuf1, off_k);
        issue_v(vbuf0, off_v);
        off_v = off_k;
        off_k = read_offs(2);
        qk(kbuf0, 0, sreg[0], 0u);
        step(T_{}, F_{}, T_{}, P0{}, 0u, kbuf0, vbuf0);
        tile_landed();
        __syncthreads();
    }
    // ---- windows 1 .. n_tiles-2: all keys valid.  The parity of W selects the buffers at compile time.
    auto window = [&](auto WP, uint32_t Wn) __attribute__((always_inline)) {
        constexpr int WPAR = decltype(WP)::value;  // Wn & 1
        char* const kb = WPAR ? kbuf1 : kbuf0;           // K tile Wn
        char* const kb_fill = WPAR ? kbuf0 : kbuf1;      // K tile Wn+1
        char* const vb = WPAR ? vbuf0 : vbuf1;           // V tile Wn-1
        char* const vb_fill = WPAR ? vbuf1 : vbuf0;      // V tile Wn
        // The next tiles' loads are enqueued between the two steps, i.e. with HALF a window of slack, on purpose.  The workgroups
        // of an XCD that walk the same unit share its K/V tiles through the L2 only while they stay close together, and what keeps
        // them together is that the one in front, which misses the L2, waits for its data while the others, which hit, catch up.
        // With a whole window of slack (loads at the window's start) even the misses are hidden, the workgroups drift apart and
        // the L2 misses quadruple (measured: 2.4e8 instead of 5.7e7 per call, and 1.6 % more time); spreading the issues over the
        // MFMA groups is slower still (each issue stalls the wavefront).
        const RowOffs off_ahead = read_offs(Wn + 2u);
        if (wave == (Wn & (uint32_t)(NW - 1))) produce(Wn + RING_AHEAD);
        const Frags pre = first_frags(P1{}, kb, vb);
        Frags mid, none;
        step_manual(P1{}, T_{}, kb, vb, 2 * Wn - 1, pre, mid);
        issue_k(kb_fill, off_k);
        issue_v(vb_fill, off_v);
        step_manual(P0{}, F_{}, kb, vb, 2 * Wn, mid, none);
        off_v = off_k;
        off_k = off_ahead;
        tile_landed();
        __syncthreads();
    };
    uint32_t W = 1;
    for (; W + 2 < n_tiles; W += 2) {
        window(P1{}, W);
        window(P0{}, W + 1u);
    }
    if (W + 1 < n_tiles) {
        window(P1{}, W);
        W++;
    }
    // ---- window n_tiles-1 (if there is more than one tile): the last K tile, may hold keys past the end
    if (W < n_tiles) {
        const char* kb = (W & 1u) ? kbuf1 : kbuf0;
        const char* vb = (W & 1u) ? vbuf0 : vbuf1;
        issue_v((W & 1u) ? vbuf1 : vbuf0, off_v);  // V tile W, the last one
        step(T_{}, T_{}, T_{}, P1{}, 2 * W - 1, kb, vb);
        step(T_{}, T_{}, T_{}, P0{}, 2 * W, kb, vb);
        tile_landed();
        __syncthreads();
        W++;
    }
    // ---- final window (W == n_tiles): softmax of the last block, the last two PVs
    {
        const char* vb = (W & 1u) ? vbuf0 : vbuf1;  // V tile W-1
        step(F_{}, T_{}, T_{}, P1{}, 2 * W - 1, nullptr, vb);
        apply_pending();
        pv(vb, 1, preg[1]);
    }

    // ---- epilogue: O = O^T / l, rounded to bf16; lane owns query lq, register r of block mt is channel 32*mt + 8*(r/4) + 4*h + r%4
#pragma unroll
    for (int qi = 0; qi < QT; qi++) {
        float llo, lhi;
        lane_pair(l_run[qi], llo, lhi);
        const float inv = 1.0f / (llo + lhi);
        if (a.lse != nullptr && h == 0) {
            // log-sum-exp of the scaled logits: the reference is in raw logit units, the sum is relative to it
            const uint32_t jq = qt * BR + (wave * QT + qi) * 32u + lq;
            if (jq < n_seq) a.lse[(size_t)unit * n_seq + jq] = q_valid[qi] ? m_ref[qi] * a.scale + __logf(llo + lhi) : 0.f;
        }
        if (q_valid[qi]) {
            __bf16* orow = Og + q_row_off[qi];
            if (a.out_kind != OUT_AS_INPUT) {
                // the input is a sparse layout: bb is the subsequence (p, q, b) and this lane's query sits at position jq of it
                const uint32_t jq = qt * BR + (wave * QT + qi) * 32u + lq;
                orow = (__bf16*)a.out + scattered_row(a, bb, jq) * C + (size_t)head * D;
            }
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; e++) o[e] = (__bf16)(oacc[qi][mt][g * 4 + e] * inv);
                    *(bf16x4*)(orow + mt * 32 + g * 8 + 4 * h) = o;
                }
        }
    }
}

template <int D, int QT, bool PAD>
static hipError_t launch_t(const AttnArgs& a, hipStream_t stream) {
    const uint32_t s2 = a.g.mode == MODE_DENSE ? 1u : (uint32_t)(a.g.s * a.g.s);
    const uint32_t n_units = (uint32_t)a.B * s2 * (uint32_t)a.heads;
    const uint32_t q_tiles = ((uint32_t)a.g.n_sub + 32u * NW * QT - 1u) / (32u * NW * QT);
    const uint64_t total = (uint64_t)n_units * q_tiles;
    if (total > 0x7ffffff0ull) return hipErrorInvalidConfiguration;
    const uint32_t per_xcd = (uint32_t)((total + 7u) / 8u);
    attn_fwd_bf16_kernel<D, QT, PAD><<<8u * per_xcd, NTHREADS, 0, stream>>>(a, q_tiles, (uint32_t)total, per_xcd);
    return hipGetLastError();
}

hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t stream) {
    // one kernel serves the token-wise, group-wise and dense index maps: the map is only evaluated when the offset ring is filled
    if (a.head_dim == 128) return a.pad ? launch_t<128, ATTN_QT, true>(a, stream) : launch_t<128, ATTN_QT, false>(a, stream);
    if (a.head_dim == 64) return a.pad ? launch_t<64, ATTN_QT, true>(a, stream) : launch_t<64, ATTN_QT, false>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace skiparse
