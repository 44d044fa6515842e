// Row gather/scatter between the original and the sparse token order (Algorithm 1, orig_to_tsa / orig_to_gsa and
// their inverses).  Bound by HBM bandwidth: every row of heads*head_dim elements is contiguous in both layouts, so
// one wavefront moves one row with 16-byte accesses per lane (1 KiB contiguous per wavefront instruction) and the
// index arithmetic is done once per row.
#include "kernels.h"

namespace skiparse {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int PERMUTE_WAVES = 4;  // rows per workgroup

template <int UNROLL>
__global__ __launch_bounds__(PERMUTE_WAVES * 64) void permute_rows_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                                          int B, GridMap g, uint32_t chunks_per_row,
                                                                          uint32_t n_rows, int to_sparse) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t row = blockIdx.x * PERMUTE_WAVES + (threadIdx.x >> 6);  // row number in the sparse layout
    if (row >= n_rows) return;
    // sparse row -> (sb, j) -> (p, q, b) -> row number in the original layout
    const uint32_t n_sub = (uint32_t)g.n_sub;
    const uint32_t sb = row / n_sub, j = row - sb * n_sub;
    const uint32_t pq = sb / (uint32_t)B, b = sb - pq * (uint32_t)B;
    const uint32_t p = pq / (uint32_t)g.s, q = pq - p * (uint32_t)g.s;
    const uint32_t orig_row = b * (uint32_t)g.n_tok + src_token(g, p, q, j);
    const u32x4* s = src + (size_t)(to_sparse ? orig_row : row) * chunks_per_row;
    u32x4* d = dst + (size_t)(to_sparse ? row : orig_row) * chunks_per_row;
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

hipError_t launch_permute(const void* src, void* dst, int B, const GridMap& g, size_t row_bytes, int to_sparse,
                          hipStream_t stream) {
    const uint32_t chunks = (uint32_t)(row_bytes / 16);
    const uint32_t s2 = g.mode == MODE_DENSE ? 1u : (uint32_t)(g.s * g.s);
    const uint32_t n_rows = (uint32_t)B * s2 * (uint32_t)g.n_sub;
    const uint32_t blocks = (n_rows + PERMUTE_WAVES - 1) / PERMUTE_WAVES;
    if (chunks >= 5 * 64)
        permute_rows_kernel<5><<<blocks, PERMUTE_WAVES * 64, 0, stream>>>((const u32x4*)src, (u32x4*)dst, B, g, chunks, n_rows, to_sparse);
    else if (chunks >= 3 * 64)
        permute_rows_kernel<3><<<blocks, PERMUTE_WAVES * 64, 0, stream>>>((const u32x4*)src, (u32x4*)dst, B, g, chunks, n_rows, to_sparse);
    else
        permute_rows_kernel<1><<<blocks, PERMUTE_WAVES * 64, 0, stream>>>((const u32x4*)src, (u32x4*)dst, B, g, chunks, n_rows, to_sparse);
    return hipGetLastError();
}

}  // namespace skiparse
