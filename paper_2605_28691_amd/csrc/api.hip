// C ABI of the library: argument validation and dispatch.  Everything is checked before the first HIP call, so the
// error paths run on a host without a GPU.
#include "../../include/skiparse.h"

#include <stdint.h>

#include <mutex>

#include "kernels.h"

using namespace skiparse;

// Scratch of skiparse_attn_bwd_static (the backward pass for callers that cannot allocate): the delta array, one float per
// (subsequence, head, position).  Every GPU the library runs on holds its own copy at its own address until the process ends.
// In host code this name is only a stand-in for the symbol: the device address is looked up once per device (static_scratch())
// and that pointer, never the name, is what the kernels get.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)SKIPARSE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip_error = 0;

constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {};  // device address of `scratch` on each device, filled on the first call there
std::mutex g_scratch_mutex;

int elem_size(int dtype) {
    switch (dtype) {
        case SKIPARSE_BF16: return 2;
        case SKIPARSE_FP32: return 4;
        case SKIPARSE_FP8_E4M3: return 1;
        default: return 0;
    }
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// [a, a + a_bytes) and [b, b + b_bytes) share at least one byte
bool overlap2(const void* a, size_t a_bytes, const void* b, size_t b_bytes) {
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y + b_bytes && y < x + a_bytes;
}
bool overlap(const void* a, const void* b, size_t bytes) { return overlap2(a, bytes, b, bytes); }

struct Shape {
    size_t n_tok;     // T*H*W
    size_t n_sub;     // n_tok / s^2
    size_t row_elems; // heads*head_dim
    size_t elems;     // B*n_tok*row_elems
};

// Checks everything that does not involve pointers.  Returns SKIPARSE_OK and fills `sh`, or an error code.
int check_shape(int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, Shape* sh, bool allow_pad = false) {
    if (B < 1 || heads < 1 || T < 1 || H < 1 || W < 1 || head_dim < 1 || s < 1) return SKIPARSE_EINVAL;
    if (pattern != SKIPARSE_TOKEN && pattern != SKIPARSE_GROUP) return SKIPARSE_EINVAL;
    if (s > 1024) return SKIPARSE_ESHAPE;
    const int unit = pattern == SKIPARSE_TOKEN ? s : s * s;
    if (!allow_pad && (H % unit != 0 || W % unit != 0)) return SKIPARSE_ESHAPE;
    const uint64_t n_tok = (uint64_t)T * (uint64_t)H * (uint64_t)W;
    const uint64_t rows = n_tok * (uint64_t)B;
    if (rows >= (1ull << 31)) return SKIPARSE_ESHAPE;  // row numbers are 32-bit in the kernels
    // in the any-resolution mode the subsequences are those of the grid padded to multiples of s*s
    const uint64_t Hp = allow_pad ? ((uint64_t)H + s * s - 1) / (s * s) * (s * s) : (uint64_t)H;
    const uint64_t Wp = allow_pad ? ((uint64_t)W + s * s - 1) / (s * s) * (s * s) : (uint64_t)W;
    if ((uint64_t)T * Hp * Wp >= (1ull << 31)) return SKIPARSE_ESHAPE;
    const uint64_t n_sub = (uint64_t)T * Hp * Wp / ((uint64_t)s * s);
    uint64_t dmax = Wp / (uint64_t)s > (uint64_t)s ? Wp / (uint64_t)s : (uint64_t)s;
    if (allow_pad && Hp > dmax) dmax = Hp;
    if (n_sub * dmax >= (1ull << 32)) return SKIPARSE_ESHAPE;  // range of the multiply-high divisions
    const uint64_t row_elems = (uint64_t)heads * (uint64_t)head_dim;
    if (row_elems >= (1ull << 31) || rows * row_elems >= (1ull << 40)) return SKIPARSE_ESHAPE;
    sh->n_tok = (size_t)n_tok;
    sh->n_sub = (size_t)n_sub;
    sh->row_elems = (size_t)row_elems;
    sh->elems = (size_t)(rows * row_elems);
    return SKIPARSE_OK;
}

GridMap make_gridmap(int T, int H, int W, int s, int pattern, bool pad = false) {
    return skiparse::make_gridmap(T, H, W, s, pattern == SKIPARSE_GROUP, pad);
}

int finish(hipError_t e) {
    if (e == hipSuccess) return SKIPARSE_OK;
    g_last_hip_error = (int)e;
    return SKIPARSE_EHIP;
}

// Device address of the static scratch on the CURRENT device: looked up once per device, with that device current, and kept.
int static_scratch(void** ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return finish(e);
    if (dev < 0 || dev >= MAX_DEVICES) return SKIPARSE_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return finish(e);
        if (p == nullptr) return finish(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return SKIPARSE_OK;
}

int permute_common(const void* src, void* dst, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern,
                   int dtype, void* stream, int to_sparse) {
    if (!src || !dst) return SKIPARSE_EINVAL;
    const int esz = elem_size(dtype);
    if (esz == 0) return SKIPARSE_EINVAL;
    Shape sh;
    const int rc = check_shape(B, heads, T, H, W, head_dim, s, pattern, &sh);
    if (rc != SKIPARSE_OK) return rc;
    if (misaligned(src) || misaligned(dst)) return SKIPARSE_EINVAL;
    const size_t row_bytes = sh.row_elems * (size_t)esz;
    if (row_bytes % 16 != 0) return SKIPARSE_EUNSUPPORTED;
    if (overlap(src, dst, sh.elems * (size_t)esz)) return SKIPARSE_EINVAL;
    const GridMap g = make_gridmap(T, H, W, s, pattern);
    return finish(launch_permute(src, dst, B, g, row_bytes, to_sparse, (hipStream_t)stream));
}

// The attention kernels address rows with 32-bit byte offsets inside one batch element: one batch element must stay below
// 4 GiB (tokens per batch element, row length W and bytes per token row are kept below 2^24 as well).
int check_attn_ranges(const Shape& sh, int W, int elem_bytes) {
    const uint64_t row_bytes = (uint64_t)sh.row_elems * (uint64_t)elem_bytes;
    if (sh.n_tok >= (1u << 24) || (uint64_t)W >= (1u << 24) || row_bytes >= (1u << 24)) return SKIPARSE_ESHAPE;
    if ((uint64_t)sh.n_tok * row_bytes >= (1ull << 32)) return SKIPARSE_ESHAPE;
    return SKIPARSE_OK;
}

int check_attn_ptrs(const void* q, const void* k, const void* v, const void* out, size_t bytes) {
    if (!q || !k || !v || !out) return SKIPARSE_EINVAL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out)) return SKIPARSE_EINVAL;
    if (overlap(out, q, bytes) || overlap(out, k, bytes) || overlap(out, v, bytes)) return SKIPARSE_EINVAL;
    return SKIPARSE_OK;
}

size_t align256(size_t x) { return (x + 255u) & ~(size_t)255u; }

}  // namespace

extern "C" {

int skiparse_permute(const void* src, void* dst, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern,
                     int dtype, void* stream) {
    return permute_common(src, dst, B, heads, T, H, W, head_dim, s, pattern, dtype, stream, 1);
}

int skiparse_unpermute(const void* src, void* dst, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern,
                       int dtype, void* stream) {
    return permute_common(src, dst, B, heads, T, H, W, head_dim, s, pattern, dtype, stream, 0);
}

// Local halves of the pattern switch under Sparse Sequence Parallelism (Sec. 3.3; Alg. 1, sparse_sequence_parallel): shared checks.
static int ssp_common(const void* src, void* dst, int b, int heads, int T, int H, int W, int head_dim, int s, int group_size, int dtype,
                      void* stream, bool pack) {
    if (!src || !dst) return SKIPARSE_EINVAL;
    const int esz = elem_size(dtype);
    if (esz == 0) return SKIPARSE_EINVAL;
    if (b < 1 || s < 1 || s > 1024 || group_size < 1) return SKIPARSE_EINVAL;
    if ((s * s) % group_size != 0) return SKIPARSE_ESHAPE;  // whole subsequences per rank
    const int G = s * s / group_size;
    if ((int64_t)G * b > (int64_t)1 << 24) return SKIPARSE_ESHAPE;
    Shape full;  // the full grid must admit both patterns: H and W multiples of s*s
    int rc = check_shape(b, heads, T, H, W, head_dim, s, SKIPARSE_GROUP, &full);
    if (rc != SKIPARSE_OK) return rc;
    // a rank's shard: G*b batch elements on the reduced grid (T, H/s, W/s), split token-wise once more
    Shape sh;
    rc = check_shape(G * b, heads, T, H / s, W / s, head_dim, s, SKIPARSE_TOKEN, &sh);
    if (rc != SKIPARSE_OK) return rc;
    if (misaligned(src) || misaligned(dst)) return SKIPARSE_EINVAL;
    const size_t row_bytes = sh.row_elems * (size_t)esz;
    if (row_bytes % 16 != 0) return SKIPARSE_EUNSUPPORTED;
    if (overlap(src, dst, sh.elems * (size_t)esz)) return SKIPARSE_EINVAL;
    const GridMap g = make_gridmap(T, H / s, W / s, s, SKIPARSE_TOKEN);
    if (pack) return finish(launch_permute(src, dst, G * b, g, row_bytes, 1, (hipStream_t)stream));
    return finish(launch_permute(src, dst, G * b, g, row_bytes, 0, (hipStream_t)stream, s == 1 ? 0 : G));
}

int skiparse_ssp_pack(const void* x, void* send, int b, int heads, int T, int H, int W, int head_dim, int s, int group_size, int dtype,
                      void* stream) {
    return ssp_common(x, send, b, heads, T, H, W, head_dim, s, group_size, dtype, stream, true);
}

int skiparse_ssp_unpack(const void* recv, void* y, int b, int heads, int T, int H, int W, int head_dim, int s, int group_size, int dtype,
                        void* stream) {
    return ssp_common(recv, y, b, heads, T, H, W, head_dim, s, group_size, dtype, stream, false);
}

int skiparse_switch_pattern(const void* src, void* dst, int B, int heads, int T, int H, int W, int head_dim, int s,
                            int from_pattern, int dtype, void* stream) {
    if (!src || !dst) return SKIPARSE_EINVAL;
    const int esz = elem_size(dtype);
    if (esz == 0) return SKIPARSE_EINVAL;
    if (from_pattern != SKIPARSE_TOKEN && from_pattern != SKIPARSE_GROUP) return SKIPARSE_EINVAL;
    Shape sh;
    const int rc = check_shape(B, heads, T, H, W, head_dim, s, SKIPARSE_GROUP, &sh);  // both patterns must fit: multiples of s*s
    if (rc != SKIPARSE_OK) return rc;
    if (misaligned(src) || misaligned(dst)) return SKIPARSE_EINVAL;
    const size_t row_bytes = sh.row_elems * (size_t)esz;
    if (row_bytes % 16 != 0) return SKIPARSE_EUNSUPPORTED;
    if (overlap(src, dst, sh.elems * (size_t)esz)) return SKIPARSE_EINVAL;
    if (s == 1) return finish(launch_permute(src, dst, B, make_gridmap(T, H, W, 1, SKIPARSE_TOKEN), row_bytes, 1, (hipStream_t)stream));
    const int to_pattern = from_pattern == SKIPARSE_TOKEN ? SKIPARSE_GROUP : SKIPARSE_TOKEN;
    const GridMap g_to = make_gridmap(T, H, W, s, to_pattern);
    return finish(launch_switch(src, dst, B, g_to, from_pattern == SKIPARSE_GROUP, H, row_bytes, (hipStream_t)stream));
}

int dense_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int H, int W,
                   int head_dim, float scale, int dtype, void* stream) {
    Shape sh;
    int rc = check_shape(B, heads, T, H, W, head_dim, 1, SKIPARSE_TOKEN, &sh);
    if (rc != SKIPARSE_OK) return rc;
    if (elem_size(dtype) == 0) return SKIPARSE_EINVAL;
    if (dtype != SKIPARSE_BF16 || (head_dim != 64 && head_dim != 128)) return SKIPARSE_EUNSUPPORTED;
    rc = check_attn_ranges(sh, W, 2);
    if (rc != SKIPARSE_OK) return rc;
    rc = check_attn_ptrs(q, k, v, out, sh.elems * 2);
    if (rc != SKIPARSE_OK) return rc;
    AttnArgs a;
    a.q = q; a.k = k; a.v = v; a.out = out;
    a.B = B; a.heads = heads; a.head_dim = head_dim;
    a.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)head_dim);
    a.g = make_dense_gridmap(sh.n_tok);
    a.pad = false;
    a.out_kind = OUT_AS_INPUT;
    a.lse = nullptr;
    return finish(launch_attn_bf16(a, (hipStream_t)stream));
}

size_t skiparse_workspace_bytes(int B, int heads, int T, int H, int W, int head_dim, int s, int dtype, unsigned flags) {
    Shape sh;
    if (check_shape(B, heads, T, H, W, head_dim, s, SKIPARSE_TOKEN, &sh) != SKIPARSE_OK) return 0;
    if (dtype != SKIPARSE_BF16 || (flags & SKIPARSE_FUSED)) return 0;
    return 4 * align256(sh.elems * 2);
}

int skiparse_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int H, int W,
                      int head_dim, int s, int pattern, float scale, int dtype, unsigned flags, void* workspace,
                      size_t workspace_bytes, void* stream) {
    if (flags & ~(unsigned)(SKIPARSE_FUSED | SKIPARSE_PAD)) return SKIPARSE_EINVAL;
    const bool pad = (flags & SKIPARSE_PAD) != 0 && s > 1;
    Shape sh;
    int rc = check_shape(B, heads, T, H, W, head_dim, s, pattern, &sh, pad);
    if (rc != SKIPARSE_OK) return rc;
    if (elem_size(dtype) == 0) return SKIPARSE_EINVAL;
    if (pad && !(flags & SKIPARSE_FUSED)) return SKIPARSE_EUNSUPPORTED;  // padding exists only as an address predicate of the fused kernel
    if (dtype != SKIPARSE_BF16 || (head_dim != 64 && head_dim != 128)) return SKIPARSE_EUNSUPPORTED;
    const size_t bytes = sh.elems * 2;
    rc = check_attn_ranges(sh, W, 2);
    if (rc != SKIPARSE_OK) return rc;
    rc = check_attn_ptrs(q, k, v, out, bytes);
    if (rc != SKIPARSE_OK) return rc;
    AttnArgs a;
    a.B = B; a.heads = heads; a.head_dim = head_dim;
    a.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)head_dim);
    a.out_kind = OUT_AS_INPUT;
    a.lse = nullptr;
    hipStream_t st = (hipStream_t)stream;
    if (flags & SKIPARSE_FUSED) {
        a.q = q; a.k = k; a.v = v; a.out = out;
        a.g = make_gridmap(T, H, W, s, pattern, pad);
        a.pad = pad;
        return finish(launch_attn_bf16(a, st));
    }
    const size_t need = 4 * align256(bytes);
    if (!workspace || workspace_bytes < need || misaligned(workspace)) return SKIPARSE_EWORKSPACE;
    if (overlap2(workspace, need, q, bytes) || overlap2(workspace, need, k, bytes) || overlap2(workspace, need, v, bytes) ||
        overlap2(workspace, need, out, bytes))
        return SKIPARSE_EINVAL;
    char* w = (char*)workspace;
    void* qp = w;
    void* kp = w + align256(bytes);
    void* vp = w + 2 * align256(bytes);
    void* op = w + 3 * align256(bytes);
    const GridMap g = make_gridmap(T, H, W, s, pattern);
    const size_t row_bytes = sh.row_elems * 2;
    hipError_t e;
    if ((e = launch_permute(q, qp, B, g, row_bytes, 1, st)) != hipSuccess) return finish(e);
    if ((e = launch_permute(k, kp, B, g, row_bytes, 1, st)) != hipSuccess) return finish(e);
    if ((e = launch_permute(v, vp, B, g, row_bytes, 1, st)) != hipSuccess) return finish(e);
    a.q = qp; a.k = kp; a.v = vp; a.out = op;
    a.B = B * s * s;  // the subsequences are the batch of the inner attention (Alg. 1: "(p q b)")
    a.g = make_dense_gridmap(sh.n_sub);
    a.pad = false;
    if ((e = launch_attn_bf16(a, st)) != hipSuccess) return finish(e);
    return finish(launch_permute(op, out, B, g, row_bytes, 0, st));
}

int skiparse_attn_fwd_sparse(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int H, int W,
                             int head_dim, int s, int pattern, int out_layout, float scale, int dtype, void* stream) {
    if (out_layout != SKIPARSE_OUT_SAME && out_layout != SKIPARSE_OUT_OTHER && out_layout != SKIPARSE_OUT_ORIGINAL)
        return SKIPARSE_EINVAL;
    Shape sh;
    // the other pattern's layout exists only when both patterns do: multiples of s*s
    int rc = check_shape(B, heads, T, H, W, head_dim, s, out_layout == SKIPARSE_OUT_OTHER ? SKIPARSE_GROUP : pattern, &sh);
    if (rc != SKIPARSE_OK) return rc;
    if (pattern != SKIPARSE_TOKEN && pattern != SKIPARSE_GROUP) return SKIPARSE_EINVAL;
    if (elem_size(dtype) == 0) return SKIPARSE_EINVAL;
    if (dtype != SKIPARSE_BF16 || (head_dim != 64 && head_dim != 128)) return SKIPARSE_EUNSUPPORTED;
    rc = check_attn_ranges(sh, W, 2);
    if (rc != SKIPARSE_OK) return rc;
    rc = check_attn_ptrs(q, k, v, out, sh.elems * 2);
    if (rc != SKIPARSE_OK) return rc;
    AttnArgs a;
    a.q = q; a.k = k; a.v = v; a.out = out;
    a.B = B * s * s;  // the subsequences are the batch of the attention (Alg. 1: "(p q b)")
    a.heads = heads; a.head_dim = head_dim;
    a.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)head_dim);
    a.g = make_dense_gridmap(sh.n_sub);
    a.pad = false;
    // with s = 1 every layout is the original one
    a.out_kind = (out_layout == SKIPARSE_OUT_SAME || s == 1) ? OUT_AS_INPUT : out_layout == SKIPARSE_OUT_ORIGINAL ? OUT_ORIGINAL : OUT_OTHER_PATTERN;
    a.out_B = B;
    a.lse = nullptr;
    a.g_in = make_gridmap(T, H, W, s, pattern);
    return finish(launch_attn_bf16(a, (hipStream_t)stream));
}

// floats in the log-sum-exp / delta arrays: one per (subsequence, head, position); positions run over the padded grid in the
// any-resolution mode (sh.n_sub is then the padded count)
static size_t lse_elems(int B, int heads, int s, const Shape& sh) { return (size_t)s * s * B * heads * sh.n_sub; }

size_t skiparse_lse_bytes(int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, unsigned flags) {
    if (flags & ~(unsigned)SKIPARSE_PAD) return 0;
    Shape sh;
    if (check_shape(B, heads, T, H, W, head_dim, s, pattern, &sh, (flags & SKIPARSE_PAD) != 0 && s > 1) != SKIPARSE_OK) return 0;
    return lse_elems(B, heads, s, sh) * sizeof(float);
}

int skiparse_attn_fwd_lse(const void* q, const void* k, const void* v, void* out, float* lse, int B, int heads, int T, int H, int W,
                          int head_dim, int s, int pattern, float scale, int dtype, unsigned flags, void* stream) {
    if (flags & ~(unsigned)SKIPARSE_PAD) return SKIPARSE_EINVAL;
    const bool pad = (flags & SKIPARSE_PAD) != 0 && s > 1;
    Shape sh;
    int rc = check_shape(B, heads, T, H, W, head_dim, s, pattern, &sh, pad);
    if (rc != SKIPARSE_OK) return rc;
    if (elem_size(dtype) == 0) return SKIPARSE_EINVAL;
    if (dtype != SKIPARSE_BF16 || (head_dim != 64 && head_dim != 128)) return SKIPARSE_EUNSUPPORTED;
    const size_t bytes = sh.elems * 2, lse_bytes = lse_elems(B, heads, s, sh) * sizeof(float);
    rc = check_attn_ranges(sh, W, 2);
    if (rc != SKIPARSE_OK) return rc;
    rc = check_attn_ptrs(q, k, v, out, bytes);
    if (rc != SKIPARSE_OK) return rc;
    if (!lse || ((uintptr_t)lse & 3u)) return SKIPARSE_EINVAL;
    if (overlap2(lse, lse_bytes, q, bytes) || overlap2(lse, lse_bytes, k, bytes) || overlap2(lse, lse_bytes, v, bytes) ||
        overlap2(lse, lse_bytes, out, bytes))
        return SKIPARSE_EINVAL;
    AttnArgs a;
    a.q = q; a.k = k; a.v = v; a.out = out;
    a.B = B; a.heads = heads; a.head_dim = head_dim;
    a.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)head_dim);
    a.g = make_gridmap(T, H, W, s, pattern, pad);
    a.pad = pad;
    a.out_kind = OUT_AS_INPUT;
    a.lse = lse;
    return finish(launch_attn_bf16(a, (hipStream_t)stream));
}

size_t skiparse_bwd_workspace_bytes(int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, unsigned flags) {
    return align256(skiparse_lse_bytes(B, heads, T, H, W, head_dim, s, pattern, flags));
}

// Shared by skiparse_attn_bwd (caller's workspace) and skiparse_attn_bwd_static (workspace == nullptr: the library's static scratch,
// whose device address is looked up after the arguments have been validated).
static int attn_bwd_common(const void* q, const void* k, const void* v, const void* out, const void* dout, const float* lse, void* dq,
                           void* dk, void* dv, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, float scale,
                           int dtype, unsigned flags, void* workspace, size_t workspace_bytes, bool use_static, void* stream) {
    if (flags & ~(unsigned)SKIPARSE_PAD) return SKIPARSE_EINVAL;
    const bool pad = (flags & SKIPARSE_PAD) != 0 && s > 1;
    Shape sh;
    int rc = check_shape(B, heads, T, H, W, head_dim, s, pattern, &sh, pad);
    if (rc != SKIPARSE_OK) return rc;
    if (elem_size(dtype) == 0) return SKIPARSE_EINVAL;
    if (dtype != SKIPARSE_BF16 || (head_dim != 64 && head_dim != 128)) return SKIPARSE_EUNSUPPORTED;
    const size_t bytes = sh.elems * 2, lse_bytes = lse_elems(B, heads, s, sh) * sizeof(float);
    rc = check_attn_ranges(sh, W, 2);
    if (rc != SKIPARSE_OK) return rc;
    const void* ins[5] = {q, k, v, out, dout};
    void* outs[3] = {dq, dk, dv};
    for (const void* x : ins)
        if (!x || misaligned(x)) return SKIPARSE_EINVAL;
    for (void* y : outs)
        if (!y || misaligned(y)) return SKIPARSE_EINVAL;
    if (!lse || ((uintptr_t)lse & 3u)) return SKIPARSE_EINVAL;
    const size_t need = align256(lse_bytes);
    if (use_static) {
        if (need > STATIC_SCRATCH_BYTES) return SKIPARSE_EWORKSPACE;  // the problem is larger than the static scratch
        rc = static_scratch(&workspace);
        if (rc != SKIPARSE_OK) return rc;
    } else if (!workspace || workspace_bytes < need || misaligned(workspace)) {
        return SKIPARSE_EWORKSPACE;
    }
    // no gradient may alias an input, another gradient, the log-sum-exp or the workspace
    for (int i = 0; i < 3; i++) {
        for (const void* x : ins)
            if (overlap(outs[i], x, bytes)) return SKIPARSE_EINVAL;
        for (int j = i + 1; j < 3; j++)
            if (overlap(outs[i], outs[j], bytes)) return SKIPARSE_EINVAL;
        if (overlap2(outs[i], bytes, lse, lse_bytes) || overlap2(outs[i], bytes, workspace, need)) return SKIPARSE_EINVAL;
    }
    for (const void* x : ins)
        if (overlap2(workspace, need, x, bytes)) return SKIPARSE_EINVAL;
    if (overlap2(workspace, need, lse, lse_bytes)) return SKIPARSE_EINVAL;
    BwdArgs a;
    a.q = q; a.k = k; a.v = v; a.out = out; a.dout = dout; a.lse = lse;
    a.delta = (float*)workspace;
    a.dq = dq; a.dk = dk; a.dv = dv;
    a.B = B; a.heads = heads; a.head_dim = head_dim;
    a.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)head_dim);
    a.pad = pad;
    a.g = make_gridmap(T, H, W, s, pattern, pad);
    return finish(launch_attn_bwd_bf16(a, (hipStream_t)stream));
}

int skiparse_attn_bwd(const void* q, const void* k, const void* v, const void* out, const void* dout, const float* lse, void* dq,
                      void* dk, void* dv, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, float scale,
                      int dtype, unsigned flags, void* workspace, size_t workspace_bytes, void* stream) {
    return attn_bwd_common(q, k, v, out, dout, lse, dq, dk, dv, B, heads, T, H, W, head_dim, s, pattern, scale, dtype, flags, workspace,
                           workspace_bytes, false, stream);
}

size_t skiparse_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int skiparse_attn_bwd_static(const void* q, const void* k, const void* v, const void* out, const void* dout, const float* lse, void* dq,
                             void* dk, void* dv, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern, float scale,
                             int dtype, unsigned flags, void* stream) {
    return attn_bwd_common(q, k, v, out, dout, lse, dq, dk, dv, B, heads, T, H, W, head_dim, s, pattern, scale, dtype, flags, nullptr, 0,
                           true, stream);
}

// elements of a tensor in the sparse layout over the (possibly padded) grid: s*s*B subsequences of sh.n_sub positions
static size_t sparse_elems(int B, int s, const Shape& sh) { return (size_t)s * s * B * sh.n_sub * sh.row_elems; }

int skiparse_quantize_fp8_ex(const void* x_bf16, void* x8, float* scales, int B, int heads, int T, int H, int W, int head_dim,
                             int s, int pattern, unsigned flags, void* stream) {
    if (flags & ~(unsigned)SKIPARSE_PAD) return SKIPARSE_EINVAL;
    const bool pad = (flags & SKIPARSE_PAD) != 0 && s > 1;
    Shape sh;
    const int rc = check_shape(B, heads, T, H, W, head_dim, s, pattern, &sh, pad);
    if (rc != SKIPARSE_OK) return rc;
    if (!x_bf16 || !x8 || !scales) return SKIPARSE_EINVAL;
    if (misaligned(x_bf16) || misaligned(x8) || (reinterpret_cast<uintptr_t>(scales) & 3u)) return SKIPARSE_EINVAL;
    if (head_dim != 64 && head_dim != 128) return SKIPARSE_EUNSUPPORTED;
    if (overlap2(x_bf16, sh.elems * 2, x8, sparse_elems(B, s, sh))) return SKIPARSE_EINVAL;
    const GridMap g = make_gridmap(T, H, W, s, pattern, pad);
    return finish(launch_quantize_fp8(x_bf16, x8, scales, B, heads, head_dim, g, pad, (hipStream_t)stream));
}

int skiparse_quantize_fp8(const void* x_bf16, void* x8, float* scales, int B, int heads, int T, int H, int W, int head_dim,
                          int s, int pattern, void* stream) {
    return skiparse_quantize_fp8_ex(x_bf16, x8, scales, B, heads, T, H, W, head_dim, s, pattern, 0u, stream);
}

int skiparse_attn_fwd_fp8_ex(const void* q8, const void* k8, const void* v8, const float* sq, const float* sk, const float* sv,
                             void* out_bf16, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern,
                             float scale, unsigned flags, void* stream) {
    if (flags & ~(unsigned)SKIPARSE_PAD) return SKIPARSE_EINVAL;
    const bool pad = (flags & SKIPARSE_PAD) != 0 && s > 1;
    Shape sh;
    int rc = check_shape(B, heads, T, H, W, head_dim, s, pattern, &sh, pad);
    if (rc != SKIPARSE_OK) return rc;
    if (!q8 || !k8 || !v8 || !sq || !sk || !sv || !out_bf16) return SKIPARSE_EINVAL;
    if (misaligned(q8) || misaligned(k8) || misaligned(v8) || misaligned(out_bf16)) return SKIPARSE_EINVAL;
    if (head_dim != 64 && head_dim != 128) return SKIPARSE_EUNSUPPORTED;
    rc = check_attn_ranges(sh, W, 2);
    if (rc != SKIPARSE_OK) return rc;
    // the quantised tensors are addressed with 32-bit byte offsets inside one subsequence
    if ((uint64_t)sh.n_sub * sh.row_elems >= (1ull << 32)) return SKIPARSE_ESHAPE;
    const size_t in_bytes = sparse_elems(B, s, sh), out_bytes = sh.elems * 2;
    if (overlap2(out_bf16, out_bytes, q8, in_bytes) || overlap2(out_bf16, out_bytes, k8, in_bytes) ||
        overlap2(out_bf16, out_bytes, v8, in_bytes))
        return SKIPARSE_EINVAL;
    // one float per (subsequence, head, 128 positions); the kernel reads them while it writes out
    const size_t scale_bytes = (size_t)s * s * B * heads * ((sh.n_sub + 127) / 128) * sizeof(float);
    for (const float* sc : {sq, sk, sv})
        if ((reinterpret_cast<uintptr_t>(sc) & 3u) || overlap2(out_bf16, out_bytes, sc, scale_bytes)) return SKIPARSE_EINVAL;
    Fp8AttnArgs a;
    a.q8 = q8; a.k8 = k8; a.v8 = v8; a.sq = sq; a.sk = sk; a.sv = sv; a.out = out_bf16;
    a.B = B; a.heads = heads; a.head_dim = head_dim;
    a.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)head_dim);
    a.n_blk = (uint32_t)((sh.n_sub + 127) / 128);
    a.pad = pad;
    a.g = make_gridmap(T, H, W, s, pattern, pad);
    return finish(launch_attn_fp8(a, (hipStream_t)stream));
}

int skiparse_attn_fwd_fp8(const void* q8, const void* k8, const void* v8, const float* sq, const float* sk, const float* sv,
                          void* out_bf16, int B, int heads, int T, int H, int W, int head_dim, int s, int pattern,
                          float scale, void* stream) {
    return skiparse_attn_fwd_fp8_ex(q8, k8, v8, sq, sk, sv, out_bf16, B, heads, T, H, W, head_dim, s, pattern, scale, 0u, stream);
}

const char* skiparse_strerror(int code) {
    switch (code) {
        case SKIPARSE_OK: return "ok";
        case SKIPARSE_EINVAL: return "invalid argument (null or misaligned pointer, non-positive size, unknown enum, overlapping buffers)";
        case SKIPARSE_ESHAPE: return "grid not divisible as the pattern requires, or sizes out of range";
        case SKIPARSE_EUNSUPPORTED: return "no kernel for this head_dim / element type";
        case SKIPARSE_EWORKSPACE: return "workspace missing, misaligned or too small (or, for the static-scratch entry point, the problem exceeds the scratch)";
        case SKIPARSE_EHIP: return "kernel launch failed (see skiparse_last_hip_error)";
        default: return "unknown error code";
    }
}

int skiparse_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
