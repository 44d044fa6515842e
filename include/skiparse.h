/*
 * skiparse.h -- C ABI of the MI355X (gfx950) Skiparse-2D attention library.
 *
 * The library computes the forward pass, and the gradients, of the sparse attention layer of OSP-Next (Sec. 3.1
 * "Skiparse-2D Attention", Algorithm 1 "Skiparse Rearrange"): a (T,H,W) token grid is split into s*s
 * spatially strided subsequences (token-wise or group-wise), ordinary softmax attention runs inside
 * every subsequence, and the result is put back in the original token order.
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned, and must stay alive
 *     until `stream` has passed the call.  The library never allocates, frees or synchronises: a call
 *     only enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Original layout  x[b][n][head][d], n = (t*H + h)*W + w, contiguous      (Alg. 1: "b (t h w) c").
 *   - Sparse layout    y[sb][j][head][d], sb = (p*s + q)*B + b, j = (t*(H/s) + hs)*(W/s) + ws
 *                      (Alg. 1: "(p q b) (t h w) c", batch fastest inside sb).
 *       token-wise: h = hs*s + p,                 w = ws*s + q                    (Alg. 1, orig_to_tsa)
 *       group-wise: h = (hs/s)*s*s + p*s + hs%s,  w = (ws/s)*s*s + q*s + ws%s     (Alg. 1, orig_to_gsa)
 *   - Shape rules: token-wise needs H % s == 0 and W % s == 0; group-wise needs H % (s*s) == 0 and
 *     W % (s*s) == 0 (Sec. 3.2: the smallest repeatable unit is s^2 x s^2).  s = 1 is legal: the permute is
 *     a copy and sparse attention equals full attention.
 *   - Return value: SKIPARSE_OK or a negative error code.  Arguments are validated before the first HIP
 *     call, so a bad call touches no memory and launches nothing.
 */
#ifndef SKIPARSE_H
#define SKIPARSE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SKIPARSE_TOKEN = 0, SKIPARSE_GROUP = 1 };                       /* pattern */
enum { SKIPARSE_BF16 = 0, SKIPARSE_FP32 = 1, SKIPARSE_FP8_E4M3 = 2 };  /* element type of a tensor */
enum { SKIPARSE_FUSED = 1u, SKIPARSE_PAD = 2u };                       /* flags of skiparse_attn_fwd */
enum { SKIPARSE_OUT_SAME = 0, SKIPARSE_OUT_OTHER = 1, SKIPARSE_OUT_ORIGINAL = 2 }; /* out_layout of skiparse_attn_fwd_sparse */

enum {
    SKIPARSE_OK = 0,
    SKIPARSE_EINVAL = -1,       /* null pointer, non-positive size, unknown enum, src == dst, misaligned pointer */
    SKIPARSE_ESHAPE = -2,       /* H or W not divisible as the pattern requires, or sizes overflow 31-bit row counts */
    SKIPARSE_EUNSUPPORTED = -3, /* no kernel for this head_dim / element type */
    SKIPARSE_EWORKSPACE = -4,   /* workspace missing or smaller than skiparse_workspace_bytes() */
    SKIPARSE_EHIP = -5          /* a kernel launch failed; see skiparse_last_hip_error() */
};

/*
 * Rearrangement original -> sparse (Alg. 1, orig_to_tsa / orig_to_gsa): dst[sb][j][:] = src[b][n(sb,j)][:].
 * Rows of heads*head_dim elements are moved verbatim (bit-exact) for any element type.
 * src: [B][T*H*W][heads][head_dim]; dst: [s*s*B][T*H*W/(s*s)][heads][head_dim]; src and dst must not overlap.
 */
int skiparse_permute(const void* src, void* dst, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern,
                     int dtype, void* stream);

/* Inverse rearrangement sparse -> original (Alg. 1, tsa_to_orig / gsa_to_orig): dst[b][n(sb,j)][:] = src[sb][j][:]. */
int skiparse_unpermute(const void* src, void* dst, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern,
                       int dtype, void* stream);

/*
 * Direct switch between the two sparse layouts (Alg. 1, tsa_to_gsa / gsa_to_tsa): src is in the sparse layout of
 * `from_pattern`, dst receives the sparse layout of the other pattern; equal to unpermute(from) followed by permute(other)
 * with a single row move per token.  Needs H and W multiples of s*s (both patterns must exist).  Bit-exact, any element type.
 */
int skiparse_switch_pattern(const void* src, void* dst, int B, int heads, int T, int H, int W, int head_dim, int s,
                            int from_pattern, int dtype, void* stream);

/*
 * The two LOCAL halves of the pattern switch under Sparse Sequence Parallelism (Sec. 3.3; Alg. 1, sparse_sequence_parallel), for the
 * share of ONE rank.  The s*s subsequences of a sparse layout are spread over group_size ranks, G = s*s/group_size whole subsequences
 * per rank (group_size must divide s*s; H and W multiples of s*s).  A rank's shard is x[(g, bb)][T*(H/s)*(W/s)][heads][head_dim]:
 * g in [0, G) its subsequences in class order, bb in [0, b) the batch elements (batch fastest), positions in subsequence order.
 *   skiparse_ssp_pack    step 1: every held subsequence, a (T, H/s, W/s) grid of its own, is split token-wise once more; the result
 *                        send[dst rank][g' of dst][(g, bb)][T*(H/(s*s))*(W/(s*s))][heads][head_dim] is the all-to-all's send buffer
 *                        (chunk `dst rank` goes to that rank; the library performs no communication).
 *   skiparse_ssp_unpack  steps 3 and 4: recv[src rank][g'][g of src][bb][..] (chunk `src rank` is what that rank sent here) becomes
 *                        the rank's shard y[(g', bb)][T*(H/s)*(W/s)][..] in the OTHER pattern's sparse layout.  The axis swap
 *                        of step 3 is folded into the row numbers; one row move per token.
 * The same pair switches token-wise -> group-wise and group-wise -> token-wise.  group_size = 1 is the single-device switch
 * (equal to skiparse_switch_pattern).  Bit-exact row moves, any element type; src and dst must not overlap.
 */
int skiparse_ssp_pack(const void* x, void* send, int b, int heads, int T, int H, int W, int head_dim, int s, int group_size, int dtype,
                      void* stream);
int skiparse_ssp_unpack(const void* recv, void* y, int b, int heads, int T, int H, int W, int head_dim, int s, int group_size, int dtype,
                        void* stream);

/*
 * Full attention (the dense blocks of the hybrid model, Sec. 3.4; also the per-subsequence step of Sec. 3.1):
 * for every (b, head):  out = softmax(q k^T * scale) v  over all N = T*H*W tokens, no mask, no dropout.
 * q, k, v, out: [B][N][heads][head_dim] bf16 (only N = T*H*W matters).  scale <= 0 selects 1/sqrt(head_dim).
 * dtype must be SKIPARSE_BF16; head_dim 64 or 128.  Accumulation and softmax are fp32, probabilities are
 * rounded to bf16 for the second matrix product, the output is rounded to bf16 (round to nearest even).
 */
int dense_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int H, int W,
                   int head_dim, float scale, int dtype, void* stream);

/*
 * Skiparse-2D attention (Sec. 3.1): out = unpermute(attention(permute(q), permute(k), permute(v))).
 * q, k, v, out are all in the ORIGINAL layout [B][T*H*W][heads][head_dim] bf16.
 *   flags = 0              three permutes, attention on the s*s*B subsequences, one unpermute.  Needs a
 *                          workspace of skiparse_workspace_bytes() bytes (four permuted tensors).
 *   flags = SKIPARSE_FUSED one kernel that computes each row's address from (subsequence, position); no
 *                          permuted copy is written and no workspace is needed (workspace may be NULL).
 * Both give the same result up to fp32 summation order.
 *   flags = SKIPARSE_FUSED | SKIPARSE_PAD   any-resolution mode (Sec. 3.2): H and W may be arbitrary; the grid is treated as
 *                          padded at the END of H and W to the next multiples of s*s, padding positions are masked as keys
 *                          and skipped as queries.  q, k, v, out still hold only the T*H*W real tokens; no padded copy is
 *                          made (the padding is an address predicate of the fused kernel).  Without SKIPARSE_FUSED the
 *                          flag is rejected with SKIPARSE_EUNSUPPORTED.
 */
int skiparse_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int H, int W,
                      int head_dim, int s, int pattern, float scale, int dtype, unsigned flags, void* workspace,
                      size_t workspace_bytes, void* stream);

/* Bytes of device workspace skiparse_attn_fwd needs for these arguments (0 for the fused path, 0 on bad arguments). */
size_t skiparse_workspace_bytes(int B, int heads, int T, int H, int W, int head_dim, int s, int dtype, unsigned flags);

/*
 * Attention for a chain of sparse blocks (Sec. 3.1: token-wise and group-wise blocks alternate; Alg. 1, tsa_to_gsa /
 * gsa_to_tsa): q, k, v are ALREADY in the sparse layout of `pattern` ([s*s*B][T*H*W/(s*s)][heads][head_dim] bf16), so every
 * subsequence is contiguous and no gather is needed; the result row of each query is written straight to
 *   SKIPARSE_OUT_SAME      the same sparse layout,
 *   SKIPARSE_OUT_OTHER     the sparse layout of the other pattern (what the next block reads; needs H, W multiples of s*s),
 *   SKIPARSE_OUT_ORIGINAL  the original layout (after the last sparse block).
 * Equal to dense attention over the s*s*B subsequences followed by skiparse_switch_pattern / skiparse_unpermute, without the
 * extra pass over the tensor.  out must not overlap q, k or v.  Other rules as for skiparse_attn_fwd.
 */
int skiparse_attn_fwd_sparse(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int H, int W,
                             int head_dim, int s, int pattern, int out_layout, float scale, int dtype, void* stream);

/*
 * Training (Sec. 4.1: the model is fine-tuned with the sparse attention in place).
 * skiparse_attn_fwd_lse: the fused forward (as skiparse_attn_fwd with SKIPARSE_FUSED) that also writes, for the backward pass,
 *   lse[sb][head][j] = log sum_keys exp(scale q.k)  (natural log, float32, subsequence order; skiparse_lse_bytes() bytes).
 * skiparse_attn_bwd: gradients of that layer for a loss with dL/dout = dout:
 *   dv = P^T dout,  dq = scale dS k,  dk = scale dS^T q,  dS = P o (dout v^T - rowsum(dout o out)),  P = exp(scale q k^T - lse),
 *   all inside every subsequence.  q, k, v, out, dout, dq, dk, dv: ORIGINAL layout [B][T*H*W][heads][head_dim] bf16; out and lse
 *   must be what skiparse_attn_fwd_lse produced for the same q, k, v, scale and flags.  P and dS are rounded to bf16 for the
 *   matrix products, accumulation is fp32, the gradients are rounded to bf16.  Deterministic (no atomics).
 *   workspace: skiparse_bwd_workspace_bytes() bytes of device memory (one float per position and head).
 *   No gradient buffer may overlap any other argument.  s = 1 gives the gradients of full attention.
 * flags: 0, or SKIPARSE_PAD for the any-resolution mode (Sec. 3.2; the paper trains at 720x1280, a grid that needs the padding):
 *   H and W arbitrary, positions j then run over the grid padded to multiples of s*s (lse of a padding position is 0), padding
 *   positions are masked keys and have no gradients.
 */
size_t skiparse_lse_bytes(int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, unsigned flags);
int skiparse_attn_fwd_lse(const void* q, const void* k, const void* v, void* out, float* lse, int B, int heads, int T, int H, int W,
                          int head_dim, int s, int pattern, float scale, int dtype, unsigned flags, void* stream);
size_t skiparse_bwd_workspace_bytes(int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, unsigned flags);
int skiparse_attn_bwd(const void* q, const void* k, const void* v, const void* out, const void* dout, const float* lse, void* dq,
                      void* dk, void* dv, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, float scale,
                      int dtype, unsigned flags, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The backward pass for callers that cannot allocate device memory (code under HIP graph capture, tight serving or training
 * loops, harnesses that forbid hipMalloc): skiparse_attn_bwd with the delta workspace taken from a static device array inside the
 * library instead of a caller's buffer.  The call allocates nothing and frees nothing; inputs, outputs and results are exactly
 * those of skiparse_attn_bwd.
 *   Limit: the workspace the call would need (skiparse_bwd_workspace_bytes()) must not exceed SKIPARSE_STATIC_SCRATCH_BYTES
 *   (16 MiB = 4,194,304 positions x heads x subsequences; the 768P shape with 40 heads needs 12.9 MB); larger problems are
 *   rejected with SKIPARSE_EWORKSPACE and must use skiparse_attn_bwd.  Every GPU the library is used on holds the array until
 *   the process ends.
 *   The array is shared by all calls on a GPU and keeps the last call's contents (every element a call reads it has written
 *   itself first, so nothing needs clearing): calls that overlap in time on one GPU, e.g. on two streams, race; serialise them.
 *   The device address of the array is looked up on the first call on each device (hipGetSymbolAddress; that first call must
 *   not itself be under graph capture).
 */
enum { SKIPARSE_STATIC_SCRATCH_BYTES = 16 * 1024 * 1024 };
size_t skiparse_static_scratch_bytes(void);
int skiparse_attn_bwd_static(const void* q, const void* k, const void* v, const void* out, const void* dout, const float* lse, void* dq,
                             void* dk, void* dv, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, float scale,
                             int dtype, unsigned flags, void* stream);

/*
 * 8-bit variant (motivated by Sec. 3.5, which runs the attention MatMuls in an 8-bit format; here OCP fp8 e4m3
 * with fine-grained scales instead of per-tensor HiF8).
 * skiparse_quantize_fp8: x (bf16, ORIGINAL layout) -> x8 (e4m3fn bytes, SPARSE layout) and
 * scales[sb][head][ceil(Nsub/128)] (fp32) with scale = max|x| over a block of 128 consecutive tokens of one
 * subsequence and head (all head_dim channels), divided by 448; an all-zero block gets scale 1.  x8 = rne(x/scale),
 * saturating.
 */
int skiparse_quantize_fp8(const void* x_bf16, void* x8, float* scales, int B, int heads, int T, int H, int W, int head_dim,
                          int s, int pattern, void* stream);

/*
 * Attention on the quantised, already permuted tensors; out_bf16 is written in the ORIGINAL layout.
 * S = (q8 k8^T) * sq * sk * scale; probabilities are multiplied by the key block's V scale and rounded to e4m3
 * for the second matrix product, which accumulates in fp32.
 */
int skiparse_attn_fwd_fp8(const void* q8, const void* k8, const void* v8, const float* sq, const float* sk, const float* sv,
                          void* out_bf16, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern,
                          float scale, void* stream);

/*
 * The same two calls with a flags argument: 0, or SKIPARSE_PAD for the any-resolution mode (Sec. 3.2; the paper reports its 8-bit
 * numbers on the padded 720x1280 workload as well).  With SKIPARSE_PAD, H and W are arbitrary; positions run over the grid padded at
 * the END of H and W to multiples of s*s: x8 is [s*s*B][T*Hp*Wp/(s*s)][heads][head_dim] with zero codes at the padding positions,
 * scales [s*s*B][heads][ceil(positions/128)] (a block's scale is taken over its real rows; 1 for a block of nothing but padding);
 * the attention masks the padding positions as keys, skips them as queries and writes only the T*H*W real rows of out_bf16.
 * skiparse_lse_bytes(..., SKIPARSE_PAD) / (4 * s*s*B*heads) gives the positions per subsequence.
 */
int skiparse_quantize_fp8_ex(const void* x_bf16, void* x8, float* scales, int B, int heads, int T, int H, int W, int head_dim,
                             int s, int pattern, unsigned flags, void* stream);
int skiparse_attn_fwd_fp8_ex(const void* q8, const void* k8, const void* v8, const float* sq, const float* sk, const float* sv,
                             void* out_bf16, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern,
                             float scale, unsigned flags, void* stream);

/* Text for an error code; never NULL. */
const char* skiparse_strerror(int code);

/* The hipError_t (as int) of the last failed launch on this thread, 0 if none. */
int skiparse_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SKIPARSE_H */
