// Row gather/scatter between the original and the sparse token order (Algorithm 1, orig_to_tsa / orig_to_gsa and
// their inverses).  Bound by HBM bandwidth: every row of heads*head_dim elements is contiguous in both layouts, so
// one wavefront moves one row with 16-byte accesses per lane (1 KiB contiguous per wavefront instruction) and the
// index arithmetic is done once per row.
#include "kernels.h"

namespace skiparse {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int PERMUTE_WAVES = 4;  // rows per workgroup

// BY_ORIG = false: the wavefronts enumerate the rows of the SPARSE layout (consecutive wavefronts touch consecutive sparse rows) and
// find each row's place in the original layout with the index map; BY_ORIG = true: they enumerate the rows of the ORIGINAL layout
// and find each token's class and position with the inverse formulas.  Either serves both directions; what differs is which
// side of the copy is contiguous across wavefronts.  Contiguous WRITES with gathered reads measure faster than the reverse, so
// the permute (writes the sparse layout) enumerates sparse rows and the unpermute (writes the original layout) original rows.
// ssp_G > 0 (Sparse Sequence Parallelism, Alg. 1 sparse_sequence_parallel, step 3): the sparse side is a buffer as it arrives from the
// all-to-all, [source rank][my subsequence g'][source's subsequence g][b][position]; the algorithm's axis swap to
// [source rank][g][g'][b] = "(p q b')" order is folded into the row number instead of being a pass of its own.
__device__ inline uint32_t ssp_received_sb(uint32_t sb, uint32_t B, uint32_t G) {
    const uint32_t b = B / G;                        // batch elements per subsequence
    const uint32_t pq = sb / B, bi = sb - pq * B;    // class of the source pattern; (g', batch element)
    const uint32_t r = pq / G, gs = pq - r * G, gd = bi / b, bb = bi - gd * b;
    return ((r * G + gd) * G + gs) * b + bb;
}

template <int UNROLL, bool BY_ORIG>
__global__ __launch_bounds__(PERMUTE_WAVES * 64) void permute_rows_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                                          int B, GridMap g, uint32_t chunks_per_row,
                                                                          uint32_t n_rows, int to_sparse, uint32_t ssp_G) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t row = blockIdx.x * PERMUTE_WAVES + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    uint32_t sparse_row, orig_row;
    if (!BY_ORIG) {
        // sparse row -> (sb, j) -> (p, q, b) -> row number in the original layout
        const uint32_t n_sub = (uint32_t)g.n_sub;
        const uint32_t sb = row / n_sub, j = row - sb * n_sub;
        const uint32_t pq = sb / (uint32_t)B, b = sb - pq * (uint32_t)B;
        const uint32_t p = pq / (uint32_t)g.s, q = pq - p * (uint32_t)g.s;
        orig_row = b * (uint32_t)g.n_tok + src_token(g, p, q, j);
        sparse_row = ssp_G ? ssp_received_sb(sb, (uint32_t)B, ssp_G) * n_sub + j : row;
    } else {
        // original row -> (b, t*H + h, w) -> class (p, q) and position (Alg. 1 read backwards; H and W are multiples of s for the
        // token-wise pattern and of s*s for the group-wise one, so t*H + h splits like h)
        orig_row = row;
        sparse_row = row;
        if (g.mode != MODE_DENSE) {
            const uint32_t s = (uint32_t)g.s, W = (uint32_t)g.W;
            const uint32_t b = row / (uint32_t)g.n_tok, n = row - b * (uint32_t)g.n_tok;
            const uint32_t th = n / W, w = n - th * W;
            uint32_t p, q, r, ws;
            if (g.mode == MODE_GROUP) {
                p = (th / s) % s;
                q = (w / s) % s;
                r = (th / (s * s)) * s + th % s;
                ws = (w / (s * s)) * s + w % s;
            } else {
                p = th % s;
                q = w % s;
                r = th / s;
                ws = w / s;
            }
            uint32_t sb = (p * s + q) * (uint32_t)B + b;
            if (ssp_G) sb = ssp_received_sb(sb, (uint32_t)B, ssp_G);
            sparse_row = sb * (uint32_t)g.n_sub + r * (W / s) + ws;
        }
    }
    const u32x4* s = src + (size_t)(to_sparse ? orig_row : sparse_row) * chunks_per_row;
    u32x4* d = dst + (size_t)(to_sparse ? sparse_row : orig_row) * chunks_per_row;
    uint32_t c = lane;
    for (; c + (UNROLL - 1) * 64u < chunks_per_row; c += UNROLL * 64u) {
        u32x4 tmp[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; u++) tmp[u] = __builtin_nontemporal_load(s + c + u * 64u);
#pragma unroll
        for (int u = 0; u < UNROLL; u++) __builtin_nontemporal_store(tmp[u], d + c + u * 64u);
    }
    for (; c < chunks_per_row; c += 64u) __builtin_nontemporal_store(__builtin_nontemporal_load(s + c), d + c);
}

// Direct switch between the two sparse layouts (Algorithm 1, tsa_to_gsa / gsa_to_tsa): one row move per token instead of
// an unpermute followed by a permute.  The destination row (sb', j') of pattern g_to holds token n; the source row is where
// the other pattern keeps n.  Plain integer divisions: they run once per row of heads*head_dim elements.
template <int UNROLL>
__global__ __launch_bounds__(PERMUTE_WAVES * 64) void switch_rows_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int B,
                                                                         GridMap g_to, int from_group, uint32_t H, uint32_t chunks_per_row,
                                                                         uint32_t n_rows) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t row = blockIdx.x * PERMUTE_WAVES + (threadIdx.x >> 6);  // row number in the destination layout
    if (row >= n_rows) return;
    const uint32_t n_sub = (uint32_t)g_to.n_sub, s = (uint32_t)g_to.s, W = (uint32_t)g_to.W;
    const uint32_t sb = row / n_sub, j = row - sb * n_sub;
    const uint32_t pq = sb / (uint32_t)B, b = sb - pq * (uint32_t)B;
    const uint32_t n = src_token(g_to, pq / s, pq % s, j);
    // position of token n in the other pattern: class (p, q) and index r*Ws + ws inside it
    const uint32_t th = n / W, w = n - th * W;  // th = t*H + h
    uint32_t p, q, r, ws;
    if (from_group) {
        p = (th / s) % s;
        q = (w / s) % s;
        r = (th / (s * s)) * s + th % s;
        ws = (w / (s * s)) * s + w % s;
    } else {
        p = th % s;
        q = w % s;
        r = th / s;
        ws = w / s;
    }
    (void)H;
    const uint32_t src_row = ((p * s + q) * (uint32_t)B + b) * n_sub + r * (W / s) + ws;
    const u32x4* sp = src + (size_t)src_row * chunks_per_row;
    u32x4* dp = dst + (size_t)row * chunks_per_row;
    uint32_t c = lane;
    for (; c + (UNROLL - 1) * 64u < chunks_per_row; c += UNROLL * 64u) {
        u32x4 tmp[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; u++) tmp[u] = __builtin_nontemporal_load(sp + c + u * 64u);
#pragma unroll
        for (int u = 0; u < UNROLL; u++) __builtin_nontemporal_store(tmp[u], dp + c + u * 64u);
    }
    for (; c < chunks_per_row; c += 64u) __builtin_nontemporal_store(__builtin_nontemporal_load(sp + c), dp + c);
}

hipError_t launch_switch(const void* src, void* dst, int B, const GridMap& g_to, int from_group, int H, size_t row_bytes,
                         hipStream_t stream) {
    const uint32_t chunks = (uint32_t)(row_bytes / 16);
    const uint32_t n_rows = (uint32_t)B * (uint32_t)(g_to.s * g_to.s) * (uint32_t)g_to.n_sub;
    const uint32_t blocks = (n_rows + PERMUTE_WAVES - 1) / PERMUTE_WAVES;
    if (chunks >= 5 * 64)
        switch_rows_kernel<5><<<blocks, PERMUTE_WAVES * 64, 0, stream>>>((const u32x4*)src, (u32x4*)dst, B, g_to, from_group, (uint32_t)H, chunks, n_rows);
    else
        switch_rows_kernel<1><<<blocks, PERMUTE_WAVES * 64, 0, stream>>>((const u32x4*)src, (u32x4*)dst, B, g_to, from_group, (uint32_t)H, chunks, n_rows);
    return hipGetLastError();
}

#ifndef SKIPARSE_UNPERMUTE_BY_ORIG
#define SKIPARSE_UNPERMUTE_BY_ORIG 1
#endif
#ifndef SKIPARSE_PERMUTE_BY_ORIG
#define SKIPARSE_PERMUTE_BY_ORIG 0
#endif

template <int UNROLL>
static void launch_rows(const void* src, void* dst, int B, const GridMap& g, uint32_t chunks, uint32_t n_rows, int to_sparse,
                        uint32_t ssp_G, hipStream_t stream) {
    const uint32_t blocks = (n_rows + PERMUTE_WAVES - 1) / PERMUTE_WAVES;
    const bool by_orig = to_sparse ? SKIPARSE_PERMUTE_BY_ORIG : SKIPARSE_UNPERMUTE_BY_ORIG;
    if (by_orig)
        permute_rows_kernel<UNROLL, true><<<blocks, PERMUTE_WAVES * 64, 0, stream>>>((const u32x4*)src, (u32x4*)dst, B, g, chunks, n_rows, to_sparse, ssp_G);
    else
        permute_rows_kernel<UNROLL, false><<<blocks, PERMUTE_WAVES * 64, 0, stream>>>((const u32x4*)src, (u32x4*)dst, B, g, chunks, n_rows, to_sparse, ssp_G);
}

hipError_t launch_permute(const void* src, void* dst, int B, const GridMap& g, size_t row_bytes, int to_sparse,
                          hipStream_t stream, int ssp_G) {
    const uint32_t chunks = (uint32_t)(row_bytes / 16);
    const uint32_t s2 = g.mode == MODE_DENSE ? 1u : (uint32_t)(g.s * g.s);
    const uint32_t n_rows = (uint32_t)B * s2 * (uint32_t)g.n_sub;
    if (chunks >= 5 * 64)
        launch_rows<5>(src, dst, B, g, chunks, n_rows, to_sparse, (uint32_t)ssp_G, stream);
    else if (chunks >= 3 * 64)
        launch_rows<3>(src, dst, B, g, chunks, n_rows, to_sparse, (uint32_t)ssp_G, stream);
    else
        launch_rows<1>(src, dst, B, g, chunks, n_rows, to_sparse, (uint32_t)ssp_G, stream);
    return hipGetLastError();
}

}  // namespace skiparse
