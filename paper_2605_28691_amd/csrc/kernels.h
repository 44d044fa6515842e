// Host-side launchers of the HIP kernels; every function only enqueues work on `stream` and returns the
// hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "index_map.h"

namespace skiparse {

// Row gather/scatter between the original and the sparse layout.  `to_sparse` != 0: dst is sparse.  ssp_G > 0: the sparse side is an
// all-to-all receive buffer of Sparse Sequence Parallelism with ssp_G subsequences per rank (Alg. 1, sparse_sequence_parallel, step 3).
hipError_t launch_permute(const void* src, void* dst, int B, const GridMap& g, size_t row_bytes, int to_sparse,
                          hipStream_t stream, int ssp_G = 0);

// Row moves from the sparse layout of one pattern to that of the other; g_to describes the destination pattern.
hipError_t launch_switch(const void* src, void* dst, int B, const GridMap& g_to, int from_group, int H, size_t row_bytes,
                         hipStream_t stream);

// Flash-attention forward, bf16.  Units are (batch-like index, head); with g.mode == MODE_DENSE the batch-like
// index is a batch element of n_sub tokens, otherwise it is a subsequence (p, q, b) addressed inside the
// original layout through src_token().
struct AttnArgs {
    const void* q;
    const void* k;
    const void* v;
    void* out;
    int B;          // batch elements of the original layout
    int heads;
    int head_dim;
    float scale;    // multiplies the logits
    bool pad;       // any-resolution mode: g describes the padded grid, padding positions are masked / skipped
    GridMap g;
    // Where the output rows go.  OUT_AS_INPUT: out is addressed like q.  OUT_ORIGINAL / OUT_OTHER_PATTERN: q, k, v are the
    // sparse layout of pattern g_in (so g is a dense map over its B*s*s subsequences) and the row of query (sb, j) is written
    // at its place in the original layout / in the sparse layout of the other pattern (Alg. 1, tsa_to_gsa / gsa_to_tsa).
    float* lse;     // optional: natural-log log-sum-exp of the scaled logits of every query, [unit][position] (for the backward pass)
    int out_kind;
    int out_B;      // batch elements of the original layout (only for out_kind != OUT_AS_INPUT)
    GridMap g_in;   // index map of the input's pattern (only for out_kind != OUT_AS_INPUT)
};
enum OutKind : int { OUT_AS_INPUT = 0, OUT_ORIGINAL = 1, OUT_OTHER_PATTERN = 2 };
hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t stream);

// Flash-attention backward, bf16: delta = rowsum(dO o O), then dQ, dK and dV (one launch each).  Addressing as in AttnArgs.
enum BwdMode : int { BWD_DQ = 0, BWD_DKV = 1 };  // dQ (owner = query), dK and dV together (owner = key)
struct BwdArgs {
    const void* q;
    const void* k;
    const void* v;
    const void* out;    // the forward's output
    const void* dout;   // gradient of the loss with respect to it
    const float* lse;   // the forward's log-sum-exp, [unit][position]
    float* delta;       // workspace, [unit][position]
    void* dq;
    void* dk;
    void* dv;
    int B;
    int heads;
    int head_dim;
    float scale;
    bool pad;           // any-resolution mode: g describes the padded grid; padding positions are masked keys and skipped rows
    GridMap g;
};
hipError_t launch_attn_bwd_bf16(const BwdArgs& a, hipStream_t stream);

// bf16 (original layout) -> E4M3 codes (sparse layout) + one float32 scale per (subsequence, head, 128 positions).
hipError_t launch_quantize_fp8(const void* x, void* x8, float* scales, int B, int heads, int head_dim, const GridMap& g, bool pad,
                               hipStream_t stream);

// FP8 flash-attention forward on the quantised sparse-layout tensors; bf16 output in the original layout.
struct Fp8AttnArgs {
    const void* q8;
    const void* k8;
    const void* v8;
    const float* sq;
    const float* sk;
    const float* sv;
    void* out;
    int B;            // batch elements of the original layout
    int heads;
    int head_dim;
    float scale;
    uint32_t n_blk;   // scale blocks per (subsequence, head): ceil(n_sub / 128)
    bool pad;         // any-resolution mode: g describes the padded grid; padding positions are masked keys and skipped queries
    GridMap g;
};
hipError_t launch_attn_fp8(const Fp8AttnArgs& a, hipStream_t stream);

}  // namespace skiparse
