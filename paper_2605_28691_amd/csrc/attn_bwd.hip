// bf16 flash-attention backward for gfx950 with the Skiparse row addressing folded in (the layer is fine-tuned, Sec. 4.1, so
// it needs gradients).  For every attention unit (a subsequence and a head), with P = softmax(scale Q K^T) recomputed from
// the forward's log-sum-exp L:
//     delta_i = sum_d dO_id O_id                      (= sum_j P_ij dP_ij; one small kernel)
//     dP = dO V^T,  dS = P o (dP - delta 1^T)
//     dQ = scale dS K,   dK = scale dS^T Q,   dV = P^T dO
// Two launches of one kernel template, each the forward kernel's scheme with the roles of the tensors exchanged: a lane OWNS
// one row (a query in the dQ launch, a key in the dK+dV launch) and the rows of the other side are STREAMED through LDS in
// tiles of 64:
//     M1^T[streamed, owner] = A1 B1^T      (dQ: K Q^T;     dK+dV: Q K^T)         A1 from LDS, B1 = owner (registers)
//     M2^T[streamed, owner] = A2 B2^T      (dQ: V dO^T;    dK+dV: dO V^T)        A2 from LDS, B2 = owner (dQ: registers, dK+dV: LDS)
//     R = elementwise(M1, M2)              (dS; in the dK+dV launch also P)       registers, rounded to bf16
//     acc^T[channel, owner] += A3^T R      (dQ: K^T dS^T;  dK: Q^T dS;  dV: dO^T P)   A3 read from LDS with the transposing read
// As in the forward kernel the 32x32 accumulator layout gives every lane one owner column, so R's registers are directly the
// B operand of the last product, and the owner's gradient rows are accumulated in registers and written once: no atomics, the
// result is deterministic.  dK and dV share one launch (S and dP are formed once for both: 7 matrix products in all against the
// 5 of the definition); their two accumulators take 128 registers at head_dim 128, so the owner's V rows are kept in LDS there.
//   * log-sum-exp and delta are per QUERY: per-lane constants in the dQ launch; in the dK+dV launch per-streamed-row values,
//     staged in LDS next to the tile as -L/scale and -delta and used as the INITIAL accumulators of M1 and M2, so that
//     P = exp2(M1 * c) and dS = P o M2 need no further arithmetic (-inf / 0 for rows that must contribute nothing).
//   * Streamed tiles go from global memory straight into LDS (global_load_lds_dwordx4), rows packed, chunk positions XOR-swizzled
//     with the row number so that a tile serves both the 16-byte fragment reads and ds_read_b64_tr_b16 without bank conflicts.
//   * Rows are addressed through the Skiparse index map (Algorithm 1) exactly as in the forward kernel, so q, k, v, dO and the
//     gradients are all in the original layout.
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

constexpr int BT = 64;             // streamed rows per tile
constexpr int BNW = 8;             // wavefronts per workgroup: 256 owners share every streamed tile
constexpr int BNT = 64 * BNW;
constexpr float LOG2E = 1.4426950408889634f;
constexpr int BRING_AHEAD = BNW;   // row offsets are formed this many tiles ahead, by one wavefront per tile in turn
constexpr int BRING = 16;          // tiles of row offsets kept in LDS
static_assert((BNW & (BNW - 1)) == 0 && (BRING & (BRING - 1)) == 0 && BRING >= BRING_AHEAD + 4, "ring sizes");

// PAD: any-resolution mode (Sec. 3.2): positions run over the grid padded to multiples of s*s; a padding position is skipped as an
// owner and contributes nothing as a streamed row (a -inf bias as the initial accumulator of the logits in both launches).
template <int D, int MODE, bool PAD>
__global__ __launch_bounds__(BNT) void attn_bwd_kernel(BwdArgs a, uint32_t o_tiles, uint32_t total, uint32_t per_xcd) {
    constexpr int KS = D / 16;   // MFMA steps along head_dim
    constexpr int MT = D / 32;   // 32-channel blocks of the gradient row
    constexpr int CH = D / 8;    // 16-byte chunks per row
    constexpr int RB = D * 2;    // row bytes in LDS (packed rows, swizzled chunk positions)
    constexpr int RPI = 64 / CH; // rows filled by one direct-to-LDS instruction of a wavefront
    constexpr int IPW = CH / BNW;  // such instructions per wavefront, tensor and tile
    constexpr bool DKV = MODE == BWD_DKV; // dK and dV together: two accumulators, the owner's second operand (V) lives in LDS
    // LDS fragments are read a few MFMA groups before their use and the order is pinned with scheduling fences, so that an MFMA
    // waits only for its own operands (left to itself the compiler issues each read right before the MFMA that needs it).  The dQ
    // launch reads 4 groups ahead (-7 %).  The dK+dV launch has almost no registers to spare: 1 group ahead in the first two
    // products and 2 in the last two is what fits without spilling into the MFMA chains (-2 %; deeper variants spill and measure
    // 2-14 % slower).  The depths of the dK+dV launch can be overridden at build time for measurements.
#ifndef BWD_DKV_MAN_A
#define BWD_DKV_MAN_A 1
#endif
#ifndef BWD_DKV_MAN_C
#define BWD_DKV_MAN_C 1
#endif
#ifndef BWD_DKV_AH_A
#define BWD_DKV_AH_A 1
#endif
#ifndef BWD_DKV_AH_C
#define BWD_DKV_AH_C 2
#endif
    constexpr int AH_A = DKV ? BWD_DKV_AH_A : 4, AH_C = DKV ? BWD_DKV_AH_C : 4;
    constexpr bool MAN_A = DKV ? (BWD_DKV_MAN_A != 0) : true, MAN_C = DKV ? (BWD_DKV_MAN_C != 0) : true;
    constexpr int TILE_BYTES = BT * RB;
    static_assert(IPW >= 1 && IPW * BNW == CH, "a tile is CH instructions, spread evenly over the wavefronts");
    // two streamed tensors, double buffered; separate arrays so that the compiler can tell the tile being filled from the one
    // being read
    __shared__ __attribute__((aligned(1024))) char s1buf0[TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char s1buf1[TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char s2buf0[TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char s2buf1[TILE_BYTES];
    __shared__ __attribute__((aligned(1024))) char own2buf[DKV ? 32 * BNW * RB : 16];  // DKV: V rows of the 256 owners, swizzled like a tile
    __shared__ __attribute__((aligned(16))) float row_l[2][BT];  // initial M1 per streamed row: dK+dV -L/scale of the query; dQ (PAD) 0 / -inf
    __shared__ __attribute__((aligned(16))) float row_d[2][BT];  // initial M2 per streamed row: dK+dV -delta of the query
    __shared__ __attribute__((aligned(16))) uint32_t rowoff[BRING][BT];     // byte offsets of the streamed rows of the next tiles
    __shared__ __attribute__((aligned(16))) unsigned char rowok[BRING][BT]; // PAD only: 1 = the row is a real token

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lq = lane & 31u, h = lane >> 5;
    const uint32_t xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
    const uint32_t lin = xcd * per_xcd + idx;  // each XCD owns a contiguous range of the (unit, owner tile) order
    if (lin >= total) return;
    const uint32_t unit = lin / o_tiles, ot = lin - unit * o_tiles;  // unit = (subsequence or batch element) * heads + head
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
    const size_t unit_off = (size_t)b0 * (uint32_t)a.g.n_tok * C + (size_t)head * D;  // elements
    const float* lse_u = a.lse + (size_t)unit * n_seq;
    const float* delta_u = a.delta + (size_t)unit * n_seq;

    // tensors by role
    const __bf16* own1_g = (const __bf16*)(MODE == BWD_DQ ? a.q : a.k) + unit_off;
    const __bf16* own2_g = (const __bf16*)(MODE == BWD_DQ ? a.dout : a.v) + unit_off;
    const char* st1_g = (const char*)((const __bf16*)(MODE == BWD_DQ ? a.k : a.q) + unit_off);
    const char* st2_g = (const char*)((const __bf16*)(MODE == BWD_DQ ? a.v : a.dout) + unit_off);
    __bf16* grad_g = (__bf16*)(MODE == BWD_DQ ? a.dq : a.dk) + unit_off;
    __bf16* grad2_g = (__bf16*)a.dv + unit_off;  // DKV: the second gradient

    // ---- owner row: operands in registers (B operands: lane = owner lq, 8 consecutive channels starting at 16*ks + 8*h)
    const uint32_t jo = ot * (32u * BNW) + wave * 32u + lq;
    // token at position j of this unit and whether it is a real one (always, outside the any-resolution mode)
    auto token_at = [&](uint32_t j, bool* real) __attribute__((always_inline)) -> uint32_t {
        if (PAD) return src_token_padded(a.g, p, q, j, real);
        *real = true;
        return src_token(a.g, p, q, j);
    };
    const uint32_t jo_c = jo < n_seq ? jo : n_seq - 1u;
    bool own_real;
    const uint32_t own_tok = token_at(jo_c, &own_real);
    const bool own_valid = jo < n_seq && own_real;
    const size_t own_off = (size_t)(own_real ? own_tok : 0u) * C;  // a padding owner reads token 0 and stores nothing
    bf16x8 own1[KS], own2[DKV ? 1 : KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
        own1[ks] = *(const bf16x8*)(own1_g + own_off + ks * 16 + 8 * h);
        if (!DKV) own2[ks] = *(const bf16x8*)(own2_g + own_off + ks * 16 + 8 * h);
    }
    float own_l = 0.f, own_d = 0.f;  // dQ: the owner is a query
    if (MODE == BWD_DQ) {
        own_l = lse_u[jo_c] * LOG2E;
        own_d = delta_u[jo_c];
    }
    const float c = a.scale * LOG2E;  // exp(x*scale - L) = exp2(x*c - L*log2e)
    const float inv_scale = 1.0f / a.scale;

    // ---- staging of streamed tiles: global memory straight into LDS (global_load_lds_dwordx4: lane l's 16 bytes land at the
    // instruction's LDS base + 16*l, one instruction fills RPI rows).  Chunk c of row r is stored at chunk position c ^ swz(r),
    // which keeps the 16-byte fragment reads (16 consecutive rows) and the transposing reads (4 consecutive rows of 64 bytes)
    // both free of bank conflicts, so a tile that is read both ways is kept once.
    auto swz = [](uint32_t r) __attribute__((always_inline)) -> uint32_t { return lds_swizzle<D>(r); };
    // The byte offsets of the streamed rows (relative to the unit's base; they fit 32 bits: checked on the host) come from a small
    // ring in LDS filled BRING_AHEAD tiles ahead: for every tile ONE wavefront (they take turns) evaluates the index map for the 64
    // rows of a tile, lane = row, and every lane later picks up the offsets of the rows it fetches.
    const uint32_t row_bytes = (uint32_t)C * 2u;
    auto produce = [&](uint32_t tile) __attribute__((always_inline)) {
        const uint32_t j = tile * BT + lane;
        bool real;
        const uint32_t tok = token_at(j < n_seq ? j : n_seq - 1u, &real);  // rows past the end repeat the last row
        rowoff[tile % BRING][lane] = real ? tok * row_bytes : 0u;          // padding rows read token 0
        if (PAD) rowok[tile % BRING][lane] = real ? 1 : 0;
    };
    uint32_t st_row[IPW], st_cb[IPW];
#pragma unroll
    for (int i = 0; i < IPW; i++) {
        st_row[i] = (wave * IPW + i) * RPI + lane / CH;
        st_cb[i] = ((lane % CH) ^ swz(st_row[i])) * 16u;
    }
    struct RowOffs {
        uint32_t off[IPW];  // row offset + chunk offset of the lane's fetches of one tile (the same for both streamed tensors)
    };
    auto read_offs = [&](uint32_t tile) __attribute__((always_inline)) -> RowOffs {
        RowOffs o;
#pragma unroll
        for (int i = 0; i < IPW; i++) o.off[i] = rowoff[tile % BRING][st_row[i]] + st_cb[i];
        return o;
    };
    float rl = 0.f, rd = 0.f;
    auto issue_tile = [&](uint32_t t, const RowOffs& o, char* b1, char* b2) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < IPW; i++) {
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(st1_g + o.off[i]),
                                             (LDS_PTR(void))(b1 + (wave * IPW + i) * 1024u), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(st2_g + o.off[i]),
                                             (LDS_PTR(void))(b2 + (wave * IPW + i) * 1024u), 16, 0, 0);
        }
        if ((DKV || PAD) && tid < BT) {  // per-row values of the streamed rows; rows past the end contribute nothing
            const uint32_t jj = t * BT + tid;
            const bool ok = jj < n_seq && (!PAD || rowok[t % BRING][tid] != 0);
            // The values are the INITIAL accumulators of the two products, so that they cost no arithmetic of their own:
            if (MODE == BWD_DQ) {
                rl = ok ? 0.f : -INFINITY;  // streamed keys: a bias on the raw logit
            } else {
                // streamed queries: raw logit - L/scale, times c = s*c - L*log2e; -inf for a row that contributes nothing (P = 0)
                rl = ok ? -lse_u[jj] * inv_scale : -INFINITY;
                rd = ok ? -delta_u[jj] : 0.f;  // dP - delta
            }
        }
    };
    auto store_rowvals = [&](uint32_t buf) __attribute__((always_inline)) {
        if ((DKV || PAD) && tid < BT) {
            row_l[buf][tid] = rl;
            row_d[buf][tid] = rd;
        }
    };
    auto tile_landed = [&]() __attribute__((always_inline)) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

    f32x16 acc[MT], acc2[DKV ? MT : 1];  // acc2: dV in the DKV launch
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
            acc[mt][r] = 0.f;
            if (DKV) acc2[mt][r] = 0.f;
        }

    // fragment of MFMA step ks: row lq (+ 32*blk), chunk 2*ks + h at its swizzled position.  The position of step ks is that of
    // step 0 with ks*32 XORed in (the row part lies above the chunk bits), so one register and an XOR per read can replace the
    // table; the dK+dV launch, the tightest on registers, does that.
    constexpr bool ADDR_TABLE = !DKV;
    const uint32_t a_rd0 = lq * RB + ((h ^ swz(lq)) * 16u);
    uint32_t a_rd_tab[ADDR_TABLE ? KS : 1];
    if (ADDR_TABLE) {
#pragma unroll
        for (int ks = 0; ks < KS; ks++) a_rd_tab[ks] = a_rd0 ^ (uint32_t)(ks * 32);
    }
    auto a_rd = [&](int ks) __attribute__((always_inline)) -> uint32_t { return ADDR_TABLE ? a_rd_tab[ks] : (a_rd0 ^ (uint32_t)(ks * 32)); };
    // transposing read: a 16-lane group covers 4 rows x 16 channels; lane i of the group addresses row i/4, channels 4*(i%4)..
    const uint32_t li = lane & 15u, lgrp = (lane >> 4) & 1u;
    uint32_t t_rd[2][MT];  // [second 4-row group][channel block]: + (blk*32 + g2*16)*RB
#pragma unroll
    for (int sec = 0; sec < 2; sec++)
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            const uint32_t row = 4 * h + (li >> 2) + 8 * sec;  // adding 16*g2 + 32*blk does not change the swizzle (low 4 bits)
            const uint32_t ch = (uint32_t)(mt * 4) + lgrp * 2 + ((li & 3u) >> 1);
            t_rd[sec][mt] = row * RB + ((ch ^ swz(row)) * 16u) + 8 * (li & 1u);
        }

    const uint32_t n_t = (n_seq + BT - 1) / BT;
    if (DKV) {
        // the wavefront's 32 owner rows of V go straight into LDS (one instruction fills RPI rows; same swizzle as the tiles, so
        // the fragment of MFMA step ks sits at a_rd(ks) of the wavefront's 32-row block); waited for with tile 0
#pragma unroll
        for (int i = 0; i < 32 / RPI; i++) {
            const uint32_t r = (uint32_t)i * RPI + lane / CH;  // row of the wavefront's block
            const uint32_t j = ot * (32u * BNW) + wave * 32u + r;
            bool real;
            const uint32_t tok = token_at(j < n_seq ? j : n_seq - 1u, &real);
            const uint32_t off = (real ? tok : 0u) * row_bytes + (((lane % CH) ^ swz(r)) * 16u);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)((const char*)own2_g + off),
                                             (LDS_PTR(void))(own2buf + wave * 32u * RB + (uint32_t)i * 1024u), 16, 0, 0);
        }
    }
    const char* const own2_lds = own2buf + (DKV ? wave * 32u * RB : 0u);
    produce(wave);  // tiles 0 .. BRING_AHEAD-1
    __syncthreads();
    issue_tile(0, read_offs(0), s1buf0, s2buf0);
    RowOffs off_next = read_offs(1);
    store_rowvals(0);
    tile_landed();
    __syncthreads();
    // one tile: enqueue the loads of the next tile into the other buffers, compute on this one, wait, barrier.  The parity of
    // the tile (which buffers) is a compile-time constant.  Tile t also forms the row offsets of tile t + BRING_AHEAD (written
    // here, first read in tile t + BRING_AHEAD - 2; the slot's previous tenant, tile t + BRING_AHEAD - BRING, was last read in tile
    // t + BRING_AHEAD - BRING - 1: barriers lie between in both directions).
    auto do_tile = [&](auto PARC, uint32_t t) __attribute__((always_inline)) {
        constexpr int PARITY = decltype(PARC)::value;  // t & 1
        const char* t1 = PARITY ? s1buf1 : s1buf0;
        const char* t2 = PARITY ? s2buf1 : s2buf0;
        const bool more = t + 1 < n_t;
        const RowOffs off_now = off_next;
        off_next = read_offs(t + 2u);  // picked up a tile early so that the LDS read is not waited for
        if (wave == (t & (uint32_t)(BNW - 1))) produce(t + BRING_AHEAD);
        const bool tail = MODE == BWD_DQ && !PAD && !more && (n_seq % BT) != 0;  // dQ: streamed keys past the end are masked
#pragma unroll
        for (int blk = 0; blk < 2; blk++) {
            // The next tile's loads are enqueued halfway through this one on purpose: with a whole tile of slack even L2 misses are
            // hidden, the workgroups that walk the same unit drift apart and stop sharing its tiles through the L2.
            if (blk == 1 && more) issue_tile(t + 1, off_now, PARITY ? s1buf0 : s1buf1, PARITY ? s2buf0 : s2buf1);
            // register r of a block is streamed row 8*(r/4) + 4*h + r%4; the per-row values start the accumulators
            f32x16 m1, m2;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                f32x4 i1 = {0.f, 0.f, 0.f, 0.f}, i2 = {0.f, 0.f, 0.f, 0.f};
                if (DKV || PAD) i1 = *(const f32x4*)&row_l[PARITY][blk * 32 + 8 * g + 4 * h];
                if (DKV) i2 = *(const f32x4*)&row_d[PARITY][blk * 32 + 8 * g + 4 * h];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    m1[4 * g + e] = i1[e];
                    m2[4 * g + e] = i2[e];
                }
            }
            // M1 and M2: their MFMA steps alternate (two independent accumulators)
            constexpr int NA = 2 * KS;
            auto frag_a = [&](int g) __attribute__((always_inline)) -> bf16x8 {
                return *(const bf16x8*)((g % 2 == 0 ? t1 : t2) + a_rd(g / 2) + blk * 32 * RB);
            };
            bf16x8 fa[NA], oa[DKV ? KS : 1];
            if (MAN_A) {
#pragma unroll
                for (int g = 0; g < AH_A; g++) {
                    fa[g] = frag_a(g);
                    if (DKV && g % 2 == 1) oa[g / 2] = *(const bf16x8*)(own2_lds + a_rd(g / 2));
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int g = 0; g < NA; g++) {
                if (MAN_A) {
                    if (g + AH_A < NA) {
                        fa[g + AH_A] = frag_a(g + AH_A);
                        if (DKV && (g + AH_A) % 2 == 1) oa[(g + AH_A) / 2] = *(const bf16x8*)(own2_lds + a_rd((g + AH_A) / 2));
                    }
                } else {
                    fa[g] = frag_a(g);
                    if (DKV && g % 2 == 1) oa[g / 2] = *(const bf16x8*)(own2_lds + a_rd(g / 2));
                }
                if (g % 2 == 0) m1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[g], own1[g / 2], m1, 0, 0, 0);
                else m2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[g], DKV ? oa[DKV ? g / 2 : 0] : own2[DKV ? 0 : g / 2], m2, 0, 0, 0);
                if (MAN_A) __builtin_amdgcn_sched_barrier(0);
            }
            // the last product's first fragments are fetched now, under the elementwise arithmetic
            constexpr int NC = (DKV ? 4 : 2) * MT;  // DKV: dK and dV groups alternate
            auto frag_c = [&](int cidx) __attribute__((always_inline)) -> bf16x8 {
                const int pair = DKV ? cidx / 2 : cidx, g2 = pair / MT, mt = pair % MT;
                const char* ta = ((DKV && cidx % 2 == 1) ? t2 : t1) + (blk * 32 + g2 * 16) * RB;  // dV reads the dO tile, dQ and dK the first tensor
                // the offset of channel block mt is that of block 0 with mt * 64 XORed in (the swizzle moves only bits 4-7, and the
                // block number enters through bits 6-7): the dK+dV launch keeps two registers instead of the table
                const uint32_t o0 = ADDR_TABLE ? t_rd[0][mt] : (t_rd[0][0] ^ (uint32_t)(mt * 64));
                const uint32_t o1 = ADDR_TABLE ? t_rd[1][mt] : (t_rd[1][0] ^ (uint32_t)(mt * 64));
                const bf16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(LDS_PTR(char))(ta + o0));
                const bf16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(LDS_PTR(char))(ta + o1));
                return __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
            };
            bf16x8 fc[NC];
            if (MAN_C) {
#pragma unroll
                for (int cidx = 0; cidx < AH_C; cidx++) fc[cidx] = frag_c(cidx);
                __builtin_amdgcn_sched_barrier(0);
            }
            bf16x8 rf[2], rp[DKV ? 2 : 1];  // rp: P itself in the DKV launch (rf holds dS there)
#pragma unroll
            for (int g2 = 0; g2 < 2; g2++) {
                bf16x8 pk, pp;
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    f32x2 val, prob;
#pragma unroll
                    for (int u = 0; u < 2; u++) {
                        const int r = g2 * 8 + e + u;
                        float pr = MODE == BWD_DQ ? __builtin_amdgcn_exp2f(fmaf(m1[r], c, -own_l)) : __builtin_amdgcn_exp2f(m1[r] * c);
                        if (tail) {
                            const uint32_t row = t * BT + blk * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                            pr = row < n_seq ? pr : 0.f;
                        }
                        val[u] = MODE == BWD_DQ ? pr * (m2[r] - own_d) : pr * m2[r];
                        prob[u] = pr;
                    }
                    const bf16x2 vb = __builtin_convertvector(val, bf16x2);
                    pk[e] = vb[0];
                    pk[e + 1] = vb[1];
                    if (DKV) {
                        const bf16x2 pb = __builtin_convertvector(prob, bf16x2);
                        pp[e] = pb[0];
                        pp[e + 1] = pb[1];
                    }
                }
                rf[g2] = pk;
                if (DKV) rp[g2] = pp;
            }
            if (MAN_C) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int cidx = 0; cidx < NC; cidx++) {
                if (MAN_C) {
                    if (cidx + AH_C < NC) fc[cidx + AH_C] = frag_c(cidx + AH_C);
                } else {
                    fc[cidx] = frag_c(cidx);
                }
                const int pair = DKV ? cidx / 2 : cidx, g2 = pair / MT, mt = pair % MT;
                if (DKV && cidx % 2 == 1) acc2[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fc[cidx], rp[DKV ? g2 : 0], acc2[mt], 0, 0, 0);  // dV^T += dO^T P
                else acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fc[cidx], rf[g2], acc[mt], 0, 0, 0);
                if (MAN_C) __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (more) store_rowvals(PARITY ^ 1);
        tile_landed();
        __syncthreads();
    };
    uint32_t t = 0;
    for (; t + 1 < n_t; t += 2) {
        do_tile(std::integral_constant<int, 0>{}, t);
        do_tile(std::integral_constant<int, 1>{}, t + 1u);
    }
    if (t < n_t) do_tile(std::integral_constant<int, 0>{}, t);

    // ---- epilogue: lane owns row jo; register r of block mt is channel 32*mt + 8*(r/4) + 4*h + r%4
    if (own_valid) {
        const float f = a.scale;
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; e++) o[e] = (__bf16)(acc[mt][g * 4 + e] * f);
                *(bf16x4*)(grad_g + own_off + mt * 32 + g * 8 + 4 * h) = o;
            }
        if (DKV) {  // the second row after the first is complete, so that the L2 sees whole lines of one row at a time
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; e++) o[e] = (__bf16)acc2[mt][g * 4 + e];
                    *(bf16x4*)(grad2_g + own_off + mt * 32 + g * 8 + 4 * h) = o;
                }
        }
    }
}

// delta[unit][j] = sum_d dO[row][head][d] * O[row][head][d]: one wavefront per position (sb, j), D/8 lanes per head.
template <int D, bool PAD>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const __bf16* __restrict__ out, const __bf16* __restrict__ dout,
                                                        float* __restrict__ delta, GridMap g, int B, int heads, uint32_t n_rows) {
    constexpr int LPH = D / 8;        // lanes per head (16 bytes each)
    constexpr int HPP = 64 / LPH;     // heads per pass
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t row = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const uint32_t n_sub = (uint32_t)g.n_sub;
    const uint32_t sb = row / n_sub, j = row - sb * n_sub;
    uint32_t p = 0, q = 0, b0 = sb;
    if (g.mode != MODE_DENSE) {
        const uint32_t pq = sb / (uint32_t)B;
        b0 = sb - pq * (uint32_t)B;
        p = pq / (uint32_t)g.s;
        q = pq - p * (uint32_t)g.s;
    }
    const size_t C = (size_t)heads * D;
    bool real = true;
    const uint32_t tok = PAD ? src_token_padded(g, p, q, j, &real) : src_token(g, p, q, j);
    const size_t base = ((size_t)b0 * (uint32_t)g.n_tok + (real ? tok : 0u)) * C;
    for (uint32_t h0 = 0; h0 < (uint32_t)heads; h0 += HPP) {
        const uint32_t head = h0 + lane / LPH;
        float sum = 0.f;
        if (head < (uint32_t)heads && real) {  // a padding position gets delta = 0
            const size_t off = base + (size_t)head * D + (lane % LPH) * 8;
            const bf16x8 o = *(const bf16x8*)(out + off);
            const bf16x8 d = *(const bf16x8*)(dout + off);
#pragma unroll
            for (int e = 0; e < 8; e++) sum = fmaf((float)o[e], (float)d[e], sum);
        }
#pragma unroll
        for (int m = LPH / 2; m >= 1; m >>= 1) sum += __shfl_xor(sum, m);
        if (head < (uint32_t)heads && lane % LPH == 0) delta[((size_t)sb * heads + head) * n_sub + j] = sum;
    }
}

template <int D, int MODE, bool PAD>
static hipError_t launch_mode(const BwdArgs& a, hipStream_t stream) {
    const uint32_t s2 = a.g.mode == MODE_DENSE ? 1u : (uint32_t)(a.g.s * a.g.s);
    const uint32_t n_units = (uint32_t)a.B * s2 * (uint32_t)a.heads;
    const uint32_t o_tiles = ((uint32_t)a.g.n_sub + 32u * BNW - 1u) / (32u * BNW);
    const uint64_t total = (uint64_t)n_units * o_tiles;
    if (total > 0x7ffffff0ull) return hipErrorInvalidConfiguration;
    const uint32_t per_xcd = (uint32_t)((total + 7u) / 8u);
    attn_bwd_kernel<D, MODE, PAD><<<8u * per_xcd, BNT, 0, stream>>>(a, o_tiles, (uint32_t)total, per_xcd);
    return hipGetLastError();
}

template <int D, bool PAD>
static hipError_t launch_all(const BwdArgs& a, hipStream_t stream) {
    const uint32_t s2 = a.g.mode == MODE_DENSE ? 1u : (uint32_t)(a.g.s * a.g.s);
    const uint32_t n_rows = (uint32_t)a.B * s2 * (uint32_t)a.g.n_sub;
    bwd_delta_kernel<D, PAD><<<(n_rows + 3u) / 4u, 256, 0, stream>>>((const __bf16*)a.out, (const __bf16*)a.dout, a.delta, a.g, a.B, a.heads, n_rows);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if ((e = launch_mode<D, BWD_DQ, PAD>(a, stream)) != hipSuccess) return e;
    return launch_mode<D, BWD_DKV, PAD>(a, stream);
}

hipError_t launch_attn_bwd_bf16(const BwdArgs& a, hipStream_t stream) {
    if (a.head_dim == 128) return a.pad ? launch_all<128, true>(a, stream) : launch_all<128, false>(a, stream);
    if (a.head_dim == 64) return a.pad ? launch_all<64, true>(a, stream) : launch_all<64, false>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace skiparse
