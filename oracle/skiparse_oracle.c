/*
 * Skiparse-2D attention -- float64 CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked against.  It shares no
 * code, header, table or helper with the HIP path and must never be linked or called by it; only
 * the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What it computes (OSP-Next paper, Sec. 3.1 "Skiparse-2D Attention" and Algorithm 1 "Skiparse
 * Rearrange"):
 *   1. the token-wise / group-wise rearrangement of a (T,H,W) token grid into s*s subsequences,
 *   2. ordinary softmax attention inside every subsequence (Sec. 3.1: interactions occur only inside
 *      each sub-figure; Sec. 3.3: each subsequence performs global attention),
 *   3. the inverse rearrangement.
 * The method is a re-indexing followed by exact attention, so the oracle is that definition written
 * out: two-pass softmax in float64, no tiling, no online rescaling.
 *
 * Layouts (Algorithm 1):
 *   original  x[b][n][c]        n = (t*H + h)*W + w,  c = head*D + d     ("b (t h w) c")
 *   sparse    y[sb][j][c]       sb = (p*s + q)*B + b                     ("(p q b) ...", batch fastest)
 *                               j  = (t*Hs + hs)*Ws + ws, Hs = H/s, Ws = W/s
 * Token-wise (Alg. 1, orig_to_tsa):  h = hs*s + p,  w = ws*s + q  -> subsequence (h mod s, w mod s).
 * Group-wise (Alg. 1, orig_to_gsa):  the h axis splits as (h_outer, p, h_inner) with h_inner in [0,s):
 *      h = (hs / s)*s*s + p*s + (hs mod s),  same for w with q -> subsequence (floor(h/s) mod s, floor(w/s) mod s).
 *
 * Element types: 0 = bfloat16 bit patterns (uint16), 1 = float32, 2 = float64.  Values are widened to
 * float64 exactly before any arithmetic.
 *
 * All functions return 0 on success and a negative number on a bad argument.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_TOKEN = 0, ORACLE_GROUP = 1 };
enum { ORACLE_BF16 = 0, ORACLE_F32 = 1, ORACLE_F64 = 2 };

static double load_elem(const void *base, int dtype, int64_t i)
{
    if (dtype == ORACLE_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16; /* bf16 = top half of an fp32 */
        float f;
        memcpy(&f, &bits, 4);
        return (double)f;
    }
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[i];
    return ((const double *)base)[i];
}

static int shape_ok(int B, int T, int H, int W, int s, int pattern)
{
    if (B < 1 || T < 1 || H < 1 || W < 1 || s < 1) return 0;
    if (pattern == ORACLE_TOKEN) return H % s == 0 && W % s == 0;
    if (pattern == ORACLE_GROUP) return H % (s * s) == 0 && W % (s * s) == 0;
    return 0;
}

/* Alg. 1, sparse -> original direction: token index n of element j of spatial class (p,q). */
int64_t oracle_src_index(int pattern, int s, int T, int H, int W, int p, int q, int64_t j)
{
    int Hs = H / s, Ws = W / s;
    int64_t ws = j % Ws;
    int64_t hs = (j / Ws) % Hs;
    int64_t t = j / ((int64_t)Ws * Hs);
    int64_t h, w;
    (void)T;
    if (pattern == ORACLE_TOKEN) {
        h = hs * s + p;
        w = ws * s + q;
    } else {
        h = (hs / s) * s * s + (int64_t)p * s + hs % s;
        w = (ws / s) * s * s + (int64_t)q * s + ws % s;
    }
    return (t * H + h) * W + w;
}

/* Alg. 1, original -> sparse direction: token n belongs to class (p,q) and sits at position j there. */
void oracle_dst_index(int pattern, int s, int T, int H, int W, int64_t n, int *p, int *q, int64_t *j)
{
    int Hs = H / s, Ws = W / s;
    int64_t w = n % W;
    int64_t h = (n / W) % H;
    int64_t t = n / ((int64_t)W * H);
    int64_t hs, ws;
    (void)T;
    if (pattern == ORACLE_TOKEN) {
        *p = (int)(h % s);
        *q = (int)(w % s);
        hs = h / s;
        ws = w / s;
    } else {
        *p = (int)((h / s) % s);
        *q = (int)((w / s) % s);
        hs = (h / (s * s)) * s + h % s;
        ws = (w / (s * s)) * s + w % s;
    }
    *j = (t * Hs + hs) * Ws + ws;
}

/* y[sb][j][:] = x[b][src(sb,j)][:] on raw bytes; row_bytes = C * element size. */
int oracle_permute(const void *x, void *y, int B, int T, int H, int W, int64_t row_bytes, int s, int pattern)
{
    if (!x || !y || row_bytes < 1 || !shape_ok(B, T, H, W, s, pattern)) return -1;
    int64_t N = (int64_t)T * H * W, Nsub = N / (s * s);
    for (int p = 0; p < s; p++)
        for (int q = 0; q < s; q++)
            for (int b = 0; b < B; b++) {
                int64_t sb = ((int64_t)p * s + q) * B + b;
                for (int64_t j = 0; j < Nsub; j++) {
                    int64_t n = oracle_src_index(pattern, s, T, H, W, p, q, j);
                    memcpy((char *)y + (sb * Nsub + j) * row_bytes, (const char *)x + ((int64_t)b * N + n) * row_bytes,
                           (size_t)row_bytes);
                }
            }
    return 0;
}

/* x[b][src(sb,j)][:] = y[sb][j][:] */
int oracle_unpermute(const void *y, void *x, int B, int T, int H, int W, int64_t row_bytes, int s, int pattern)
{
    if (!x || !y || row_bytes < 1 || !shape_ok(B, T, H, W, s, pattern)) return -1;
    int64_t N = (int64_t)T * H * W, Nsub = N / (s * s);
    for (int p = 0; p < s; p++)
        for (int q = 0; q < s; q++)
            for (int b = 0; b < B; b++) {
                int64_t sb = ((int64_t)p * s + q) * B + b;
                for (int64_t j = 0; j < Nsub; j++) {
                    int64_t n = oracle_src_index(pattern, s, T, H, W, p, q, j);
                    memcpy((char *)x + ((int64_t)b * N + n) * row_bytes, (const char *)y + (sb * Nsub + j) * row_bytes,
                           (size_t)row_bytes);
                }
            }
    return 0;
}

/*
 * Direct switch between the two sparse layouts (Alg. 1, tsa_to_gsa / gsa_to_tsa): the same tokens, re-sorted from the
 * subsequences of one pattern into those of the other.  Written as the composition it abbreviates: back to the original
 * order with the inverse of `from_pattern`, then forward with the other pattern.  Both patterns must be valid for the grid
 * (H and W multiples of s*s).
 */
int oracle_switch_pattern(const void *y_from, void *y_to, int B, int T, int H, int W, int64_t row_bytes, int s, int from_pattern)
{
    if (!y_from || !y_to || row_bytes < 1 || !shape_ok(B, T, H, W, s, ORACLE_GROUP)) return -1;
    if (from_pattern != ORACLE_TOKEN && from_pattern != ORACLE_GROUP) return -1;
    int to_pattern = from_pattern == ORACLE_TOKEN ? ORACLE_GROUP : ORACLE_TOKEN;
    void *x = malloc((size_t)((int64_t)B * T * H * W * row_bytes));
    if (!x) return -2;
    int rc = oracle_unpermute(y_from, x, B, T, H, W, row_bytes, s, from_pattern);
    if (rc == 0) rc = oracle_permute(x, y_to, B, T, H, W, row_bytes, s, to_pattern);
    free(x);
    return rc;
}

/*
 * One attention output row, plain definition:
 *   S[j] = scale * sum_d Q[d]*K[j][d];  m = max_j S[j];  P[j] = exp(S[j]-m);  O[:] = sum_j P[j] V[j][:] / sum_j P[j]
 * Key/value row j lives at element offset kv_off[j] (so that callers can walk a subsequence of a
 * tensor in the original layout without copying it).  `scores` is scratch of n_keys doubles.
 */
static void attention_row(const void *q, int64_t q_off, const void *k, const void *v, const int64_t *kv_off, int64_t n_keys,
                          int D, double scale, int dtype, double *scores, double *out)
{
    double m = -INFINITY;
    for (int64_t j = 0; j < n_keys; j++) {
        double acc = 0.0;
        for (int d = 0; d < D; d++) acc += load_elem(q, dtype, q_off + d) * load_elem(k, dtype, kv_off[j] + d);
        scores[j] = scale * acc;
        if (scores[j] > m) m = scores[j];
    }
    double denom = 0.0;
    for (int d = 0; d < D; d++) out[d] = 0.0;
    for (int64_t j = 0; j < n_keys; j++) {
        double pj = exp(scores[j] - m);
        denom += pj;
        for (int d = 0; d < D; d++) out[d] += pj * load_elem(v, dtype, kv_off[j] + d);
    }
    for (int d = 0; d < D; d++) out[d] /= denom;
}

/*
 * Attention over a batch of independent sequences: q,k,v are [nb][n][heads][D] contiguous, out is
 * float64 of the same shape.  Every (batch, head) pair is one softmax(Q K^T * scale) V.
 */
int oracle_attention(const void *q, const void *k, const void *v, double *out, int64_t nb, int64_t n, int heads, int D,
                     double scale, int dtype)
{
    if (!q || !k || !v || !out || nb < 1 || n < 1 || heads < 1 || D < 1) return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    int64_t C = (int64_t)heads * D;
    int fail = 0;
#pragma omp parallel
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)n);
        int64_t *off = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
        if (!scores || !off) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 1)
            for (int64_t b = 0; b < nb; b++)
                for (int hd = 0; hd < heads; hd++) {
                    for (int64_t j = 0; j < n; j++) off[j] = (b * n + j) * C + (int64_t)hd * D;
                    for (int64_t i = 0; i < n; i++)
                        attention_row(q, off[i], k, v, off, n, D, scale, dtype, scores, out + off[i]);
                }
        }
        free(scores);
        free(off);
    }
    return fail ? -2 : 0;
}

/*
 * Skiparse-2D attention, inputs and float64 output in the ORIGINAL layout [B][N][heads][D]:
 *   out = unpermute( attention( permute(q), permute(k), permute(v) ) )      (Sec. 3.1, Alg. 1)
 * written exactly as that composition, with whole permuted copies.
 */
int oracle_skiparse_attention(const void *q, const void *k, const void *v, double *out, int B, int heads, int T, int H, int W,
                              int D, int s, int pattern, double scale, int dtype)
{
    if (!q || !k || !v || !out || heads < 1 || D < 1 || !shape_ok(B, T, H, W, s, pattern)) return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    int64_t esz = dtype == ORACLE_BF16 ? 2 : dtype == ORACLE_F32 ? 4 : 8;
    int64_t C = (int64_t)heads * D, N = (int64_t)T * H * W, Nsub = N / (s * s);
    size_t in_bytes = (size_t)(B * N * C * esz), out_bytes = (size_t)(B * N * C) * sizeof(double);
    void *qp = malloc(in_bytes), *kp = malloc(in_bytes), *vp = malloc(in_bytes);
    double *op = (double *)malloc(out_bytes);
    int rc = -2;
    if (qp && kp && vp && op) {
        oracle_permute(q, qp, B, T, H, W, C * esz, s, pattern);
        oracle_permute(k, kp, B, T, H, W, C * esz, s, pattern);
        oracle_permute(v, vp, B, T, H, W, C * esz, s, pattern);
        rc = oracle_attention(qp, kp, vp, op, (int64_t)B * s * s, Nsub, heads, D, scale, dtype);
        if (rc == 0) rc = oracle_unpermute(op, out, B, T, H, W, C * (int64_t)sizeof(double), s, pattern);
    }
    free(qp);
    free(kp);
    free(vp);
    free(op);
    return rc;
}

/*
 * Sampled mode for shapes whose full result is out of reach on a CPU: output rows of
 * oracle_skiparse_attention for a list of (b, head, n) query positions only.  rows = [n_rows][3]
 * int64, out = [n_rows][D] float64.  Each row attends to every token of its own subsequence,
 * found through the same index maps; s = 1 gives sampled rows of full attention.
 */
int oracle_skiparse_attention_rows(const void *q, const void *k, const void *v, const int64_t *rows, int64_t n_rows, double *out,
                                   int B, int heads, int T, int H, int W, int D, int s, int pattern, double scale, int dtype)
{
    if (!q || !k || !v || !rows || !out || n_rows < 0 || heads < 1 || D < 1 || !shape_ok(B, T, H, W, s, pattern)) return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    int64_t C = (int64_t)heads * D, N = (int64_t)T * H * W, Nsub = N / (s * s);
    for (int64_t r = 0; r < n_rows; r++)
        if (rows[3 * r] < 0 || rows[3 * r] >= B || rows[3 * r + 1] < 0 || rows[3 * r + 1] >= heads || rows[3 * r + 2] < 0 ||
            rows[3 * r + 2] >= N)
            return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)Nsub);
        int64_t *off = (int64_t *)malloc(sizeof(int64_t) * (size_t)Nsub);
        if (!scores || !off) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t r = 0; r < n_rows; r++) {
                int64_t b = rows[3 * r], hd = rows[3 * r + 1], n = rows[3 * r + 2];
                int p, qq;
                int64_t jq;
                oracle_dst_index(pattern, s, T, H, W, n, &p, &qq, &jq);
                for (int64_t j = 0; j < Nsub; j++)
                    off[j] = (b * N + oracle_src_index(pattern, s, T, H, W, p, qq, j)) * C + hd * D;
                attention_row(q, (b * N + n) * C + hd * D, k, v, off, Nsub, D, scale, dtype, scores, out + r * D);
            }
        }
        free(scores);
        free(off);
    }
    return fail ? -2 : 0;
}

/*
 * Any-resolution variant (Sec. 3.2): when H or W is not a multiple of s*s the figure is padded at the END of both axes
 * up to the next multiple and the padding tokens are masked out of the attention.  Padding at the end does not change the
 * class of a real token (the class formulas of Sec. 3.1 only look at h and w), so the definition is: every real token
 * attends to all REAL tokens of its own class and batch element.  Written in that mask form, with no padded copy and no
 * position arithmetic; it needs no divisibility at all.  rows = [n_rows][3] (b, head, n), out = [n_rows][D].
 */
static void class_of(int pattern, int s, int H, int W, int64_t n, int *p, int *q)
{
    int64_t w = n % W, h = (n / W) % H;
    if (pattern == ORACLE_TOKEN) {
        *p = (int)(h % s);
        *q = (int)(w % s);
    } else {
        *p = (int)((h / s) % s);
        *q = (int)((w / s) % s);
    }
}

int oracle_skiparse_attention_rows_padded(const void *q, const void *k, const void *v, const int64_t *rows, int64_t n_rows,
                                          double *out, int B, int heads, int T, int H, int W, int D, int s, int pattern,
                                          double scale, int dtype)
{
    if (!q || !k || !v || !rows || !out || n_rows < 0 || heads < 1 || D < 1) return -1;
    if (B < 1 || T < 1 || H < 1 || W < 1 || s < 1 || (pattern != ORACLE_TOKEN && pattern != ORACLE_GROUP)) return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    int64_t C = (int64_t)heads * D, N = (int64_t)T * H * W;
    for (int64_t r = 0; r < n_rows; r++)
        if (rows[3 * r] < 0 || rows[3 * r] >= B || rows[3 * r + 1] < 0 || rows[3 * r + 1] >= heads || rows[3 * r + 2] < 0 ||
            rows[3 * r + 2] >= N)
            return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)N);
        int64_t *off = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
        if (!scores || !off) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t r = 0; r < n_rows; r++) {
                int64_t b = rows[3 * r], hd = rows[3 * r + 1], n = rows[3 * r + 2];
                int pn, qn, pm, qm;
                class_of(pattern, s, H, W, n, &pn, &qn);
                int64_t cnt = 0;
                for (int64_t m = 0; m < N; m++) {
                    class_of(pattern, s, H, W, m, &pm, &qm);
                    if (pm == pn && qm == qn) off[cnt++] = (b * N + m) * C + hd * D;
                }
                attention_row(q, (b * N + n) * C + hd * D, k, v, off, cnt, D, scale, dtype, scores, out + r * D);
            }
        }
        free(scores);
        free(off);
    }
    return fail ? -2 : 0;
}

/*
 * Brute force for tiny grids (Sec. 3.1: a token interacts only with tokens of its own sub-figure):
 * full N x N attention in the original order where the logit of a pair is -inf unless both tokens
 * are in the same batch element and have the same (p,q) class.  Uses only the class of a token,
 * never its position j, and never a permuted copy; H and W need not be divisible (for grids that are
 * not, this is the padded-and-masked attention of Sec. 3.2, since end padding leaves classes unchanged).
 */
int oracle_masked_dense_attention(const void *q, const void *k, const void *v, double *out, int B, int heads, int T, int H, int W,
                                  int D, int s, int pattern, double scale, int dtype)
{
    if (!q || !k || !v || !out || heads < 1 || D < 1 || B < 1 || T < 1 || H < 1 || W < 1 || s < 1) return -1;
    if (pattern != ORACLE_TOKEN && pattern != ORACLE_GROUP) return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    int64_t C = (int64_t)heads * D, N = (int64_t)T * H * W;
    double *logit = (double *)malloc(sizeof(double) * (size_t)N);
    if (!logit) return -2;
    for (int64_t b = 0; b < B; b++)
        for (int hd = 0; hd < heads; hd++)
            for (int64_t n = 0; n < N; n++) {
                int pn, qn, pm, qm;
                int64_t qo = (b * N + n) * C + (int64_t)hd * D;
                class_of(pattern, s, H, W, n, &pn, &qn);
                double m = -INFINITY;
                for (int64_t mm = 0; mm < N; mm++) {
                    class_of(pattern, s, H, W, mm, &pm, &qm);
                    if (pm != pn || qm != qn) {
                        logit[mm] = -INFINITY;
                        continue;
                    }
                    int64_t ko = (b * N + mm) * C + (int64_t)hd * D;
                    double acc = 0.0;
                    for (int d = 0; d < D; d++) acc += load_elem(q, dtype, qo + d) * load_elem(k, dtype, ko + d);
                    logit[mm] = scale * acc;
                    if (logit[mm] > m) m = logit[mm];
                }
                double denom = 0.0;
                for (int d = 0; d < D; d++) out[qo + d] = 0.0;
                for (int64_t mm = 0; mm < N; mm++) {
                    double pj = exp(logit[mm] - m); /* exp(-inf) = 0 for masked pairs */
                    denom += pj;
                    int64_t vo = (b * N + mm) * C + (int64_t)hd * D;
                    for (int d = 0; d < D; d++) out[qo + d] += pj * load_elem(v, dtype, vo + d);
                }
                for (int d = 0; d < D; d++) out[qo + d] /= denom;
            }
    free(logit);
    return 0;
}

/*
 * 8-bit variant (the workload's recipe; the paper's own 8-bit format, HiF8 of Sec. 3.5, is proprietary and is replaced by
 * OCP FP8 E4M3 with fine-grained scales).
 *
 * E4M3 ("fn" flavour: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities, largest finite value 448 =
 * 1.75 * 2^8, smallest subnormal 2^-9).  Encodes a float that already satisfies |y| <= 448, round to nearest, ties to even,
 * written from the format definition.
 */
static uint8_t e4m3_encode(float y)
{
    uint8_t sign = (uint8_t)(signbit(y) ? 0x80 : 0x00);
    double a = fabs((double)y);
    if (a < 0.015625) { /* below the smallest normal 2^-6: multiples of 2^-9 */
        double q = nearbyint(a * 512.0); /* default rounding mode: to nearest, ties to even; q in 0..8 */
        return (uint8_t)(sign | (uint8_t)q); /* q == 8 is the code of 2^-6 (exponent field 1, mantissa 0) */
    }
    int e;
    double f = frexp(a, &e); /* a = f * 2^e, f in [0.5, 1) */
    e -= 1;                  /* a = (2f) * 2^e with 2f in [1, 2) */
    double q = nearbyint((2.0 * f - 1.0) * 8.0); /* mantissa in eighths, 0..8 */
    if (q == 8.0) {
        q = 0.0;
        e += 1;
    }
    return (uint8_t)(sign | (uint8_t)((e + 7) << 3) | (uint8_t)q);
}

double oracle_e4m3_decode(uint8_t code)
{
    int ef = (code >> 3) & 15, m = code & 7;
    double v = ef == 0 ? m / 512.0 : ldexp(1.0 + m / 8.0, ef - 7);
    return (code & 0x80) ? -v : v;
}

uint8_t oracle_e4m3_encode(float y) { return e4m3_encode(y); }

/*
 * ---- Gradients (Sec. 4.1: the model is fine-tuned with the sparse attention in place, so the layer needs a backward pass).
 *
 * The forward definition O = softmax(scale Q K^T) V differentiated by hand, for a scalar loss with dL/dO = dO given:
 *     P  = softmax(S),  S = scale Q K^T
 *     dV = P^T dO
 *     dP = dO V^T
 *     dS = P o (dP - delta 1^T),   delta_i = sum_j P_ij dP_ij         (Jacobian of a row softmax)
 *     dQ = scale dS K,   dK = scale dS^T Q
 * Row i of dQ depends only on query i; rows of dK and dV sum over all queries.  Everything is float64, the N x N
 * matrices are walked row by row and never stored.
 */

/* Softmax row of query i (probabilities into p[0..n_keys)) -- same two-pass form as attention_row. */
static void softmax_row(const void *q, int64_t q_off, const void *k, const int64_t *kv_off, int64_t n_keys, int D, double scale,
                        int dtype, double *p)
{
    double m = -INFINITY, denom = 0.0;
    for (int64_t j = 0; j < n_keys; j++) {
        double acc = 0.0;
        for (int d = 0; d < D; d++) acc += load_elem(q, dtype, q_off + d) * load_elem(k, dtype, kv_off[j] + d);
        p[j] = scale * acc;
        if (p[j] > m) m = p[j];
    }
    for (int64_t j = 0; j < n_keys; j++) {
        p[j] = exp(p[j] - m);
        denom += p[j];
    }
    for (int64_t j = 0; j < n_keys; j++) p[j] /= denom;
}

/*
 * Contribution of query row i to the gradients.  p = its softmax row (input), ds = scratch of n_keys doubles.
 * dq_row (D doubles) is overwritten; dk / dv (may be NULL) are accumulated at dk[acc_off[j] + d] for every key j with
 * acc_off[j] >= 0 (a negative offset means "this key's gradient is not wanted").
 */
static void bwd_row(const void *q, int64_t q_off, const void *k, const void *v, const void *dout, const int64_t *kv_off,
                    int64_t n_keys, int D, double scale, int dtype, const double *p, double *ds, double *dq_row, double *dk,
                    double *dv, const int64_t *acc_off)
{
    double delta = 0.0;
    for (int64_t j = 0; j < n_keys; j++) {
        double dp = 0.0;
        for (int d = 0; d < D; d++) dp += load_elem(dout, dtype, q_off + d) * load_elem(v, dtype, kv_off[j] + d);
        ds[j] = dp;
        delta += p[j] * dp;
    }
    for (int64_t j = 0; j < n_keys; j++) ds[j] = p[j] * (ds[j] - delta);
    if (dq_row) {
        for (int d = 0; d < D; d++) dq_row[d] = 0.0;
        for (int64_t j = 0; j < n_keys; j++)
            for (int d = 0; d < D; d++) dq_row[d] += scale * ds[j] * load_elem(k, dtype, kv_off[j] + d);
    }
    if (dk && dv) {
        for (int64_t j = 0; j < n_keys; j++) {
            if (acc_off[j] < 0) continue;
            for (int d = 0; d < D; d++) {
                dk[acc_off[j] + d] += scale * ds[j] * load_elem(q, dtype, q_off + d);
                dv[acc_off[j] + d] += p[j] * load_elem(dout, dtype, q_off + d);
            }
        }
    }
}

/*
 * Gradients of oracle_attention: q, k, v, dout are [nb][n][heads][D]; dq, dk, dv float64 of the same shape.
 * One thread per (batch, head), so the accumulation into dk / dv needs no synchronisation.
 */
int oracle_attention_bwd(const void *q, const void *k, const void *v, const void *dout, double *dq, double *dk, double *dv,
                         int64_t nb, int64_t n, int heads, int D, double scale, int dtype)
{
    if (!q || !k || !v || !dout || !dq || !dk || !dv || nb < 1 || n < 1 || heads < 1 || D < 1) return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    int64_t C = (int64_t)heads * D;
    int fail = 0;
    memset(dk, 0, sizeof(double) * (size_t)(nb * n * C));
    memset(dv, 0, sizeof(double) * (size_t)(nb * n * C));
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)n);
        double *ds = (double *)malloc(sizeof(double) * (size_t)n);
        int64_t *off = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
        if (!p || !ds || !off) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 1)
            for (int64_t b = 0; b < nb; b++)
                for (int hd = 0; hd < heads; hd++) {
                    for (int64_t j = 0; j < n; j++) off[j] = (b * n + j) * C + (int64_t)hd * D;
                    for (int64_t i = 0; i < n; i++) {
                        softmax_row(q, off[i], k, off, n, D, scale, dtype, p);
                        bwd_row(q, off[i], k, v, dout, off, n, D, scale, dtype, p, ds, dq + off[i], dk, dv, off);
                    }
                }
        }
        free(p);
        free(ds);
        free(off);
    }
    return fail ? -2 : 0;
}

/*
 * Gradients of oracle_skiparse_attention, everything in the ORIGINAL layout: the rearrangement is a permutation of rows,
 * so its transpose is the inverse rearrangement:
 *     (dq, dk, dv) = unpermute( attention_bwd( permute(q), permute(k), permute(v), permute(dout) ) )      (Alg. 1)
 */
int oracle_skiparse_attention_bwd(const void *q, const void *k, const void *v, const void *dout, double *dq, double *dk,
                                  double *dv, int B, int heads, int T, int H, int W, int D, int s, int pattern, double scale,
                                  int dtype)
{
    if (!q || !k || !v || !dout || !dq || !dk || !dv || heads < 1 || D < 1 || !shape_ok(B, T, H, W, s, pattern)) return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    int64_t esz = dtype == ORACLE_BF16 ? 2 : dtype == ORACLE_F32 ? 4 : 8;
    int64_t C = (int64_t)heads * D, N = (int64_t)T * H * W, Nsub = N / (s * s);
    size_t in_bytes = (size_t)(B * N * C * esz), g_bytes = (size_t)(B * N * C) * sizeof(double);
    void *qp = malloc(in_bytes), *kp = malloc(in_bytes), *vp = malloc(in_bytes), *dop = malloc(in_bytes);
    double *gq = (double *)malloc(g_bytes), *gk = (double *)malloc(g_bytes), *gv = (double *)malloc(g_bytes);
    int rc = -2;
    if (qp && kp && vp && dop && gq && gk && gv) {
        oracle_permute(q, qp, B, T, H, W, C * esz, s, pattern);
        oracle_permute(k, kp, B, T, H, W, C * esz, s, pattern);
        oracle_permute(v, vp, B, T, H, W, C * esz, s, pattern);
        oracle_permute(dout, dop, B, T, H, W, C * esz, s, pattern);
        rc = oracle_attention_bwd(qp, kp, vp, dop, gq, gk, gv, (int64_t)B * s * s, Nsub, heads, D, scale, dtype);
        int64_t grow = C * (int64_t)sizeof(double);
        if (rc == 0) rc = oracle_unpermute(gq, dq, B, T, H, W, grow, s, pattern);
        if (rc == 0) rc = oracle_unpermute(gk, dk, B, T, H, W, grow, s, pattern);
        if (rc == 0) rc = oracle_unpermute(gv, dv, B, T, H, W, grow, s, pattern);
    }
    free(qp);
    free(kp);
    free(vp);
    free(dop);
    free(gq);
    free(gk);
    free(gv);
    return rc;
}

/*
 * Sampled mode for shapes whose full gradient is out of reach on a CPU: one attention unit -- batch element b, head hd and
 * the subsequence that contains token n_any -- is walked completely (every query row of the unit), and the gradients are
 * kept for a list of tokens of that unit only.  toks = [n_toks] token numbers n (all must lie in that subsequence);
 * dq, dk, dv = [n_toks][D].  The query loop is split over threads with one private dk / dv accumulator each.
 */
int oracle_skiparse_attention_bwd_unit(const void *q, const void *k, const void *v, const void *dout, const int64_t *toks,
                                       int64_t n_toks, double *dq, double *dk, double *dv, int b, int hd, int64_t n_any, int B,
                                       int heads, int T, int H, int W, int D, int s, int pattern, double scale, int dtype)
{
    if (!q || !k || !v || !dout || !toks || !dq || !dk || !dv || n_toks < 1 || heads < 1 || D < 1 ||
        !shape_ok(B, T, H, W, s, pattern))
        return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    int64_t C = (int64_t)heads * D, N = (int64_t)T * H * W, Nsub = N / (s * s);
    if (b < 0 || b >= B || hd < 0 || hd >= heads || n_any < 0 || n_any >= N) return -1;
    int p0, q0;
    int64_t j0;
    oracle_dst_index(pattern, s, T, H, W, n_any, &p0, &q0, &j0);
    int64_t *off = (int64_t *)malloc(sizeof(int64_t) * (size_t)Nsub);     /* element offset of key j */
    int64_t *acc_off = (int64_t *)malloc(sizeof(int64_t) * (size_t)Nsub); /* where key j's gradient goes, or -1 */
    int64_t *tok_j = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_toks);
    int rc = 0;
    if (!off || !acc_off || !tok_j) rc = -2;
    if (rc == 0) {
        for (int64_t j = 0; j < Nsub; j++) {
            off[j] = ((int64_t)b * N + oracle_src_index(pattern, s, T, H, W, p0, q0, j)) * C + (int64_t)hd * D;
            acc_off[j] = -1;
        }
        for (int64_t t = 0; t < n_toks && rc == 0; t++) {
            int pt, qt;
            if (toks[t] < 0 || toks[t] >= N) { rc = -1; break; }
            oracle_dst_index(pattern, s, T, H, W, toks[t], &pt, &qt, &tok_j[t]);
            if (pt != p0 || qt != q0 || acc_off[tok_j[t]] >= 0) rc = -1; /* wrong subsequence, or listed twice */
            else acc_off[tok_j[t]] = t * D;
        }
    }
    if (rc == 0) {
        int fail = 0;
        memset(dk, 0, sizeof(double) * (size_t)(n_toks * D));
        memset(dv, 0, sizeof(double) * (size_t)(n_toks * D));
#pragma omp parallel
        {
            double *p = (double *)malloc(sizeof(double) * (size_t)Nsub);
            double *ds = (double *)malloc(sizeof(double) * (size_t)Nsub);
            double *dq_row = (double *)malloc(sizeof(double) * (size_t)D);
            double *dk_loc = (double *)calloc((size_t)(n_toks * D), sizeof(double));
            double *dv_loc = (double *)calloc((size_t)(n_toks * D), sizeof(double));
            if (!p || !ds || !dq_row || !dk_loc || !dv_loc) {
#pragma omp atomic write
                fail = 1;
            } else {
#pragma omp for schedule(static)
                for (int64_t i = 0; i < Nsub; i++) {
                    softmax_row(q, off[i], k, off, Nsub, D, scale, dtype, p);
                    bwd_row(q, off[i], k, v, dout, off, Nsub, D, scale, dtype, p, ds, dq_row, dk_loc, dv_loc, acc_off);
                    if (acc_off[i] >= 0)
                        for (int d = 0; d < D; d++) dq[acc_off[i] + d] = dq_row[d];
                }
#pragma omp critical
                for (int64_t e = 0; e < n_toks * D; e++) {
                    dk[e] += dk_loc[e];
                    dv[e] += dv_loc[e];
                }
            }
            free(p);
            free(ds);
            free(dq_row);
            free(dk_loc);
            free(dv_loc);
        }
        if (fail) rc = -2;
    }
    free(off);
    free(acc_off);
    free(tok_j);
    return rc;
}

/*
 * Gradients in the any-resolution mode (Sec. 3.2), mask form as oracle_skiparse_attention_rows_padded: every real token
 * attends to the real tokens of its own class and batch element, whatever H and W are; no padded copy exists, so the
 * gradients are those of that masked attention.  The tokens of one class in raster order form one attention unit.
 *   unit_only = 0: all units; dq, dk, dv = [B][N][heads][D] (float64, original layout).
 *   unit_only = 1: only the unit of (b0, hd0, class of toks[0]); dq, dk, dv = [n_toks][D] for the listed tokens.
 */
static int bwd_padded_impl(const void *q, const void *k, const void *v, const void *dout, double *dq, double *dk, double *dv,
                           int B, int heads, int T, int H, int W, int D, int s, int pattern, double scale, int dtype,
                           int unit_only, int b0, int hd0, const int64_t *toks, int64_t n_toks)
{
    int64_t C = (int64_t)heads * D, N = (int64_t)T * H * W;
    int p0 = 0, q0 = 0;
    if (unit_only) class_of(pattern, s, H, W, toks[0], &p0, &q0);
    int n_units = unit_only ? 1 : B * heads * s * s;
    int fail = 0;
    for (int u = 0; u < n_units && !fail; u++) {
        int b = unit_only ? b0 : u / (heads * s * s), hd = unit_only ? hd0 : (u / (s * s)) % heads;
        int pc = unit_only ? p0 : (u % (s * s)) / s, qc = unit_only ? q0 : u % s;
        /* members of the class, raster order */
        int64_t cnt = 0;
        for (int64_t n = 0; n < N; n++) {
            int pp, qq;
            class_of(pattern, s, H, W, n, &pp, &qq);
            cnt += (pp == pc && qq == qc);
        }
        if (cnt == 0) continue; /* a class with no real token */
        int64_t *off = (int64_t *)malloc(sizeof(int64_t) * (size_t)cnt);
        int64_t *acc_off = (int64_t *)malloc(sizeof(int64_t) * (size_t)cnt);
        int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)cnt);
        if (!off || !acc_off || !tok) {
            free(off); free(acc_off); free(tok);
            return -2;
        }
        int64_t m = 0;
        for (int64_t n = 0; n < N; n++) {
            int pp, qq;
            class_of(pattern, s, H, W, n, &pp, &qq);
            if (pp == pc && qq == qc) {
                tok[m] = n;
                off[m] = ((int64_t)b * N + n) * C + (int64_t)hd * D;
                acc_off[m] = unit_only ? -1 : off[m];
                m++;
            }
        }
        if (unit_only) {
            for (int64_t t = 0; t < n_toks; t++) {
                int64_t pos = -1;
                for (int64_t i = 0; i < cnt; i++)
                    if (tok[i] == toks[t]) pos = i;
                if (pos < 0 || acc_off[pos] >= 0) { free(off); free(acc_off); free(tok); return -1; } /* other class, or twice */
                acc_off[pos] = t * D;
            }
        }
        int64_t n_acc = unit_only ? n_toks * D : 0;
#pragma omp parallel
        {
            double *p = (double *)malloc(sizeof(double) * (size_t)cnt);
            double *ds = (double *)malloc(sizeof(double) * (size_t)cnt);
            double *dq_row = (double *)malloc(sizeof(double) * (size_t)D);
            /* private accumulators: the sampled mode keeps [n_toks][D]; the full mode accumulates the unit's own rows, which no
               other unit touches, but threads of this unit do, so they also go through private copies of the unit's rows */
            int64_t loc_n = unit_only ? n_acc : cnt * D;
            double *dk_loc = (double *)calloc((size_t)loc_n, sizeof(double));
            double *dv_loc = (double *)calloc((size_t)loc_n, sizeof(double));
            int64_t *loc_off = (int64_t *)malloc(sizeof(int64_t) * (size_t)cnt);
            if (!p || !ds || !dq_row || !dk_loc || !dv_loc || !loc_off) {
#pragma omp atomic write
                fail = 1;
            } else {
                for (int64_t i = 0; i < cnt; i++) loc_off[i] = unit_only ? acc_off[i] : i * D;
#pragma omp for schedule(static)
                for (int64_t i = 0; i < cnt; i++) {
                    softmax_row(q, off[i], k, off, cnt, D, scale, dtype, p);
                    bwd_row(q, off[i], k, v, dout, off, cnt, D, scale, dtype, p, ds, dq_row, dk_loc, dv_loc, loc_off);
                    if (acc_off[i] >= 0)
                        for (int d = 0; d < D; d++) dq[acc_off[i] + d] = dq_row[d];
                }
#pragma omp critical
                for (int64_t i = 0; i < cnt; i++) {
                    if (acc_off[i] < 0) continue;
                    for (int d = 0; d < D; d++) {
                        dk[acc_off[i] + d] += dk_loc[loc_off[i] + d];
                        dv[acc_off[i] + d] += dv_loc[loc_off[i] + d];
                    }
                }
            }
            free(p); free(ds); free(dq_row); free(dk_loc); free(dv_loc); free(loc_off);
        }
        free(off); free(acc_off); free(tok);
    }
    return fail ? -2 : 0;
}

int oracle_skiparse_attention_bwd_padded(const void *q, const void *k, const void *v, const void *dout, double *dq, double *dk,
                                         double *dv, int B, int heads, int T, int H, int W, int D, int s, int pattern,
                                         double scale, int dtype)
{
    if (!q || !k || !v || !dout || !dq || !dk || !dv || B < 1 || heads < 1 || T < 1 || H < 1 || W < 1 || D < 1 || s < 1) return -1;
    if (pattern != ORACLE_TOKEN && pattern != ORACLE_GROUP) return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    size_t n = (size_t)B * T * H * W * heads * D;
    memset(dq, 0, sizeof(double) * n);
    memset(dk, 0, sizeof(double) * n);
    memset(dv, 0, sizeof(double) * n);
    return bwd_padded_impl(q, k, v, dout, dq, dk, dv, B, heads, T, H, W, D, s, pattern, scale, dtype, 0, 0, 0, NULL, 0);
}

int oracle_skiparse_attention_bwd_unit_padded(const void *q, const void *k, const void *v, const void *dout, const int64_t *toks,
                                              int64_t n_toks, double *dq, double *dk, double *dv, int b, int hd, int B, int heads,
                                              int T, int H, int W, int D, int s, int pattern, double scale, int dtype)
{
    if (!q || !k || !v || !dout || !toks || !dq || !dk || !dv || n_toks < 1 || B < 1 || heads < 1 || T < 1 || H < 1 || W < 1 ||
        D < 1 || s < 1)
        return -1;
    if (pattern != ORACLE_TOKEN && pattern != ORACLE_GROUP) return -1;
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F64) return -1;
    if (b < 0 || b >= B || hd < 0 || hd >= heads) return -1;
    for (int64_t t = 0; t < n_toks; t++)
        if (toks[t] < 0 || toks[t] >= (int64_t)T * H * W) return -1;
    memset(dq, 0, sizeof(double) * (size_t)(n_toks * D));
    memset(dk, 0, sizeof(double) * (size_t)(n_toks * D));
    memset(dv, 0, sizeof(double) * (size_t)(n_toks * D));
    return bwd_padded_impl(q, k, v, dout, dq, dk, dv, B, heads, T, H, W, D, s, pattern, scale, dtype, 1, b, hd, toks, n_toks);
}

/*
 * Quantise x (bf16 bit patterns, ORIGINAL layout [B][N][heads][D]) to E4M3 codes in the SPARSE layout
 * [s*s*B][Nsub][heads][D] with one float32 scale per (subsequence, head, block of 128 consecutive positions):
 *   amax  = max |x| over the block (all D channels);  scale = amax / 448, inv = 448 / amax  (both float32; 1 if amax = 0)
 *   code  = e4m3( clamp( x * inv, -448, 448 ) )        with x * inv rounded to float32 first
 * scales is [s*s*B][heads][ceil(Nsub/128)].  The decision "which code" is taken in float32 on both sides.
 */
int oracle_quantize_fp8(const uint16_t *x, uint8_t *x8, float *scales, int B, int heads, int T, int H, int W, int D, int s,
                        int pattern)
{
    if (!x || !x8 || !scales || heads < 1 || D < 1 || !shape_ok(B, T, H, W, s, pattern)) return -1;
    int64_t C = (int64_t)heads * D, N = (int64_t)T * H * W, Nsub = N / (s * s), nblk = (Nsub + 127) / 128;
    for (int p = 0; p < s; p++)
        for (int q = 0; q < s; q++)
            for (int b = 0; b < B; b++) {
                int64_t sb = ((int64_t)p * s + q) * B + b;
                for (int hd = 0; hd < heads; hd++)
                    for (int64_t blk = 0; blk < nblk; blk++) {
                        int64_t j0 = blk * 128, j1 = j0 + 128 < Nsub ? j0 + 128 : Nsub;
                        float amax = 0.0f;
                        for (int64_t j = j0; j < j1; j++) {
                            int64_t n = oracle_src_index(pattern, s, T, H, W, p, q, j);
                            for (int d = 0; d < D; d++) {
                                float v = (float)fabs(load_elem(x, ORACLE_BF16, ((int64_t)b * N + n) * C + (int64_t)hd * D + d));
                                if (v > amax) amax = v;
                            }
                        }
                        float scale = amax > 0.0f ? amax / 448.0f : 1.0f;
                        float inv = amax > 0.0f ? 448.0f / amax : 1.0f;
                        scales[(sb * heads + hd) * nblk + blk] = scale;
                        for (int64_t j = j0; j < j1; j++) {
                            int64_t n = oracle_src_index(pattern, s, T, H, W, p, q, j);
                            for (int d = 0; d < D; d++) {
                                float v = (float)load_elem(x, ORACLE_BF16, ((int64_t)b * N + n) * C + (int64_t)hd * D + d);
                                float y = v * inv;
                                if (y > 448.0f) y = 448.0f;
                                if (y < -448.0f) y = -448.0f;
                                x8[(sb * Nsub + j) * C + (int64_t)hd * D + d] = e4m3_encode(y);
                            }
                        }
                    }
            }
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
