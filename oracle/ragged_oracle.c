/*
 * ragged_oracle.c -- CPU reference ("oracle") for the pack -> ragged attention -> unpack path
 * of "Dispatch-Aware Ragged Attention for Pruned Vision Transformers".
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table or helper with the
 * HIP library; nothing in the GPU path may include or link this file.
 *
 * It is deliberately plain and slow: attention is the textbook definition evaluated in fp64, one
 * query row at a time, with no tiling, no running maximum and no fusion.  The paper's Algorithm 1
 * (online softmax over 64x64 tiles) reaches the same result up to rounding order, so the oracle is
 * the definition itself (Section 4.2, "Ragged Attention Kernel": bidirectional attention, softmax
 * of q.k/sqrt(d) over the tokens of the SAME image only, no causal mask, no dropout).
 *
 * Pack / unpack are exact integer / bit-copy operations (Section 4.1, "Fused Token Packing").
 *
 * Readings of the paper taken here (the paper is silent or loose on these points):
 *   - softmax scale is an argument (Alg. 1 hard-codes 1/sqrt(d)); it is an fp32 value widened
 *     to double before multiplying the fp64 dot product;
 *   - only keys j < n_i of the same image take part (Alg. 1 loads whole tiles with no bound);
 *   - packed order is stable: images ascending, tokens ascending inside an image
 *     (Section 4.1 item 1: cumulative sums give the destination indices; Section 4.3 item 5
 *     reads CLS from the front of each packed sequence);
 *   - cu_seqlens and gather_idx are int32; the keep mask is one byte per token, nonzero = keep;
 *   - a sequence with n_i = 0 contributes nothing and produces no output rows;
 *   - unpack (named but not described by the paper) is the inverse scatter of pack; dropped rows
 *     are either left untouched (fill_mode 0) or written with +0 words (fill_mode 1).
 *
 * Also here, for the parts built around the path: attention on the padded layout, packed-to-packed
 * re-pack, CLS extraction, and the linear layer / LayerNorm of the encoder blocks that run on
 * packed rows -- each the plain definition, each with its own pins in tests/test_oracle_*.py.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force padded+masked attention written separately in
 * NumPy; torch's float64 scaled_dot_product_attention for one sequence; closed forms (n=1,
 * scale=0 -> mean of V, identical V rows, two-token sigmoid case, large-scale argmax limit);
 * invariants (rows of softmax sum to 1, key-shift invariance, permutation equivariance, ragged
 * isolation, convex hull); NumPy boolean indexing / cumsum / flatnonzero for pack and unpack.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

/* IEEE binary16 -> double, exact (handles subnormals, infinities, NaN). */
static double decode_f16(uint16_t w)
{
    int sign = (w >> 15) & 1;
    int expo = (w >> 10) & 0x1f;
    int frac = w & 0x3ff;
    double mag;
    if (expo == 0) {
        mag = ldexp((double)frac, -24);              /* subnormal: frac * 2^-10 * 2^-14 */
    } else if (expo == 31) {
        mag = frac ? NAN : INFINITY;
    } else {
        mag = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    }
    return sign ? -mag : mag;
}

/* bfloat16 -> double, exact: a bfloat16 is the upper 16 bits of an IEEE binary32. */
static double decode_bf16(uint16_t w)
{
    uint32_t bits = (uint32_t)w << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double decode(uint16_t w, int dtype)
{
    return dtype == ORACLE_BF16 ? decode_bf16(w) : decode_f16(w);
}

/* Exposed so the tests can pin the decoders against NumPy / torch conversions. */
void oracle_decode(const uint16_t *words, int64_t count, int dtype, double *out)
{
    for (int64_t e = 0; e < count; ++e) out[e] = decode(words[e], dtype);
}

/*
 * Pack (Section 4.1).  x is [B, N, C] 16-bit words, keep is [B, N] bytes.
 * Walks images then tokens in ascending order; every kept token appends its flat source row
 * i*N+t to gather_idx and its C words to the next row of packed.
 * cu_seqlens[0] = 0, cu_seqlens[i+1] = cu_seqlens[i] + n_i.
 * Returns the total kept count T.  packed / gather_idx must have room for B*N rows / entries.
 */
int64_t oracle_pack(const uint16_t *x, const uint8_t *keep, int B, int N, int C,
                    uint16_t *packed, int32_t *cu_seqlens, int32_t *gather_idx)
{
    int64_t next = 0;
    cu_seqlens[0] = 0;
    for (int i = 0; i < B; ++i) {
        for (int t = 0; t < N; ++t) {
            if (keep[(int64_t)i * N + t] != 0) {
                int64_t src = (int64_t)i * N + t;
                gather_idx[next] = (int32_t)src;
                memcpy(packed + next * C, x + src * C, (size_t)C * sizeof(uint16_t));
                ++next;
            }
        }
        cu_seqlens[i + 1] = (int32_t)next;
    }
    return next;
}

/*
 * Unpack: the inverse scatter of pack.  src is [T, C] words; out is [B, N, C] words.
 * A kept token (i,t) with rank r among image i's kept tokens receives row cu_seqlens[i] + r of
 * src.  Dropped tokens: fill_mode 1 writes +0 words, fill_mode 0 leaves out untouched.
 * Walks the mask itself, so it does not depend on gather_idx being right.
 */
void oracle_unpack(const uint16_t *src, const uint8_t *keep, const int32_t *cu_seqlens,
                   int B, int N, int C, uint16_t *out, int fill_mode)
{
    for (int i = 0; i < B; ++i) {
        int64_t rank = 0;
        for (int t = 0; t < N; ++t) {
            uint16_t *dst = out + ((int64_t)i * N + t) * C;
            if (keep[(int64_t)i * N + t] != 0) {
                int64_t row = (int64_t)cu_seqlens[i] + rank;
                memcpy(dst, src + row * C, (size_t)C * sizeof(uint16_t));
                ++rank;
            } else if (fill_mode == 1) {
                memset(dst, 0, (size_t)C * sizeof(uint16_t));
            }
        }
    }
}

/*
 * One query row of one (image, head): the plain definition, on inputs already decoded to double.
 *   S_j = scale * sum_d q[d] k_j[d]          j in [0, n)
 *   M   = max_j S_j ; p_j = exp(S_j - M) ; L = sum_j p_j
 *   o[d] = (sum_j p_j v_j[d]) / L
 * Subtracting M is the usual overflow guard; it cancels in p_j / L.
 * probs (optional, length n) receives p_j / L.
 */
static void attend_row(const double *q, const double *k, const double *v,
                       int64_t s, int n, int r, int h, int H, int D, double scale,
                       double *scores, double *o, double *probs)
{
    const int64_t tok = (int64_t)H * D;            /* elements between consecutive tokens */
    const double *qrow = q + (s + r) * tok + (int64_t)h * D;
    double M = -INFINITY;
    for (int j = 0; j < n; ++j) {
        const double *krow = k + (s + j) * tok + (int64_t)h * D;
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += qrow[d] * krow[d];
        scores[j] = scale * dot;
        if (scores[j] > M) M = scores[j];
    }
    double L = 0.0;
    for (int j = 0; j < n; ++j) {
        scores[j] = exp(scores[j] - M);
        L += scores[j];
    }
    for (int d = 0; d < D; ++d) o[d] = 0.0;
    for (int j = 0; j < n; ++j) {
        const double *vrow = v + (s + j) * tok + (int64_t)h * D;
        for (int d = 0; d < D; ++d) o[d] += scores[j] * vrow[d];
    }
    for (int d = 0; d < D; ++d) o[d] /= L;
    if (probs) for (int j = 0; j < n; ++j) probs[j] = scores[j] / L;
}

/* Decode rows [0, rows) of a [rows, H*D] 16-bit buffer to a freshly allocated double buffer. */
static double *decode_all(const uint16_t *w, int64_t count, int dtype)
{
    double *out = (double *)malloc((size_t)(count > 0 ? count : 1) * sizeof(double));
    if (out) for (int64_t e = 0; e < count; ++e) out[e] = decode(w[e], dtype);
    return out;
}

/*
 * Ragged attention (Section 4.2): q, k, v are [T, H, D] 16-bit words (token-major, then head,
 * then head-dim), out is [T, H, D] doubles.  Image i owns rows [cu[i], cu[i+1]).
 * The inputs are first decoded exactly to double; then every (image, head, row) is evaluated by
 * the definition above.  threads <= 1 runs serially; otherwise (image, head) pairs are spread
 * over that many OpenMP threads -- the arithmetic of every row is unchanged.
 * Returns 0, or -1 if an allocation failed.
 */
int oracle_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v, int dtype,
                const int32_t *cu_seqlens, int B, int H, int D, float scale,
                double *out, int threads)
{
    int nmax = 0;
    for (int i = 0; i < B; ++i) {
        int n = cu_seqlens[i + 1] - cu_seqlens[i];
        if (n > nmax) nmax = n;
    }
    if (nmax == 0) return 0;
    if (threads < 1) threads = 1;
    const int64_t count = (int64_t)cu_seqlens[B] * H * D;
    double *qd = decode_all(q, count, dtype);
    double *kd = decode_all(k, count, dtype);
    double *vd = decode_all(v, count, dtype);
    int failed = !qd || !kd || !vd;
    const int pairs = failed ? 0 : B * H;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads)
#endif
    {
        double *scores = (double *)malloc((size_t)nmax * sizeof(double));
        if (!scores) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int p = 0; p < pairs; ++p) {
            if (!scores) continue;
            int i = p / H, h = p % H;
            int64_t s = cu_seqlens[i];
            int n = cu_seqlens[i + 1] - cu_seqlens[i];
            for (int r = 0; r < n; ++r) {
                double *o = out + ((s + r) * (int64_t)H + h) * D;
                attend_row(qd, kd, vd, s, n, r, h, H, D, (double)scale, scores, o, NULL);
            }
        }
        free(scores);
    }
    free(qd); free(kd); free(vd);
    return failed ? -1 : 0;
}

/*
 * Debug view for the "softmax rows sum to one" invariant, also used to check sampled rows of
 * large batches: the normalised probabilities p_j / L of query row r of image i, head h
 * (length n_i), plus that row's output.  Decodes only that image's rows.
 */
int oracle_attn_row(const uint16_t *q, const uint16_t *k, const uint16_t *v, int dtype,
                    const int32_t *cu_seqlens, int i, int h, int r, int H, int D, float scale,
                    double *probs, double *o)
{
    int64_t s = cu_seqlens[i];
    int n = cu_seqlens[i + 1] - cu_seqlens[i];
    if (r < 0 || r >= n) return -1;
    const int64_t tok = (int64_t)H * D;
    double *scores = (double *)malloc((size_t)n * sizeof(double));
    double *qd = decode_all(q + s * tok, (int64_t)n * tok, dtype);
    double *kd = decode_all(k + s * tok, (int64_t)n * tok, dtype);
    double *vd = decode_all(v + s * tok, (int64_t)n * tok, dtype);
    int ok = scores && qd && kd && vd;
    if (ok) attend_row(qd, kd, vd, 0, n, r, h, H, D, (double)scale, scores, o, probs);
    free(scores); free(qd); free(kd); free(vd);
    return ok ? 0 : -1;
}

/*
 * Attention straight on the padded layout (the single-launch variant of the pipeline, in which the
 * gather of pack and the scatter of unpack are folded into the attention itself): q, k, v are
 * [B, N, H, D] 16-bit words, keep is [B, N] bytes, out is [B, N, H, D] doubles.  For every image
 * the kept tokens, in ascending token order, attend among themselves exactly as in oracle_attn;
 * nothing is computed for dropped tokens, whose rows of out are set to +0.0.
 * Written out on its own (index list + the definition), not by calling pack / attn / unpack, so
 * that the tests can check it against that composition.
 */
int oracle_attn_padded(const uint16_t *q, const uint16_t *k, const uint16_t *v, int dtype,
                       const uint8_t *keep, int B, int N, int H, int D, float scale, double *out)
{
    int *idx = (int *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int));
    double *scores = (double *)malloc((size_t)(N > 0 ? N : 1) * sizeof(double));
    if (!idx || !scores) { free(idx); free(scores); return -1; }
    const int64_t tok = (int64_t)H * D;
    for (int i = 0; i < B; ++i) {
        int n = 0;
        for (int t = 0; t < N; ++t) {
            if (keep[(int64_t)i * N + t] != 0) idx[n++] = t;
            else for (int64_t e = 0; e < tok; ++e) out[((int64_t)i * N + t) * tok + e] = 0.0;
        }
        for (int h = 0; h < H; ++h) {
            for (int r = 0; r < n; ++r) {
                const uint16_t *qrow = q + ((int64_t)i * N + idx[r]) * tok + (int64_t)h * D;
                double M = -INFINITY;
                for (int j = 0; j < n; ++j) {
                    const uint16_t *krow = k + ((int64_t)i * N + idx[j]) * tok + (int64_t)h * D;
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d) dot += decode(qrow[d], dtype) * decode(krow[d], dtype);
                    scores[j] = (double)scale * dot;
                    if (scores[j] > M) M = scores[j];
                }
                double L = 0.0;
                for (int j = 0; j < n; ++j) { scores[j] = exp(scores[j] - M); L += scores[j]; }
                double *o = out + ((int64_t)i * N + idx[r]) * tok + (int64_t)h * D;
                for (int d = 0; d < D; ++d) o[d] = 0.0;
                for (int j = 0; j < n; ++j) {
                    const uint16_t *vrow = v + ((int64_t)i * N + idx[j]) * tok + (int64_t)h * D;
                    for (int d = 0; d < D; ++d) o[d] += scores[j] * decode(vrow[d], dtype);
                }
                for (int d = 0; d < D; ++d) o[d] /= L;
            }
        }
    }
    free(idx); free(scores);
    return 0;
}

/*
 * Re-pack: apply a second keep decision to an ALREADY packed buffer (progressive pruning while
 * staying packed, as in the pipeline of Section 4.3 where the buffer is packed once and later
 * layers keep working on it).  keep_rows has one byte per packed row (only rows < cu_in[B] count).
 * Kept rows are appended in ascending row order; cu_out[i] = kept rows before cu_in[i];
 * gather_out[r'] = the input row that became output row r'.  Returns the new total.
 */
int64_t oracle_repack(const uint16_t *packed_in, const uint8_t *keep_rows, const int32_t *cu_in,
                      int B, int C, uint16_t *packed_out, int32_t *cu_out, int32_t *gather_out)
{
    int64_t next = 0;
    cu_out[0] = 0;
    for (int i = 0; i < B; ++i) {
        for (int64_t r = cu_in[i]; r < cu_in[i + 1]; ++r) {
            if (keep_rows[r] != 0) {
                gather_out[next] = (int32_t)r;
                memcpy(packed_out + next * C, packed_in + r * C, (size_t)C * sizeof(uint16_t));
                ++next;
            }
        }
        cu_out[i + 1] = (int32_t)next;
    }
    return next;
}

/*
 * CLS extraction (Section 4.3, step 5: the class token is read from the packed buffer): the first
 * packed row of every image; an image with no rows yields +0 words.
 */
void oracle_cls_extract(const uint16_t *packed, const int32_t *cu_seqlens, int B, int C, uint16_t *out)
{
    for (int i = 0; i < B; ++i) {
        if (cu_seqlens[i + 1] > cu_seqlens[i])
            memcpy(out + (int64_t)i * C, packed + (int64_t)cu_seqlens[i] * C, (size_t)C * sizeof(uint16_t));
        else
            memset(out + (int64_t)i * C, 0, (size_t)C * sizeof(uint16_t));
    }
}

/* Number of OpenMP threads a parallel region would get by default (1 without OpenMP). */
/*
 * The linear layers of a packed encoder block (Section 4.3 item 4: after the pruning point the
 * projections and the MLP run on the packed buffer, one row per kept token).  The paper does not
 * spell the block out; it is the standard DeiT / ViT pre-norm encoder block:
 *     h = LayerNorm(x);  qkv = h Wqkv^T + b;  x = x + attn(qkv) Wo^T + bo;
 *     h = LayerNorm(x);  x = x + GELU(h W1^T + b1) W2^T + b2
 * with weights stored [out_features][in_features] and the erf form of GELU.
 *
 * oracle_linear:  y[m][n] = act( sum_k x[m][k] * w[n][k] + bias[n] ) + residual[m][n]
 *   act 0 = identity, 1 = GELU(t) = t * (1 + erf(t / sqrt 2)) / 2;  bias and residual may be NULL.
 *   Everything is decoded to double first; the sum runs over k in ascending order.
 */
int oracle_linear(const uint16_t *x, const uint16_t *w, const uint16_t *bias, const uint16_t *residual,
                  int dtype, int M, int N, int K, int act, double *y, int threads)
{
    double *xd = decode_all(x, (int64_t)M * K, dtype);
    double *wd = decode_all(w, (int64_t)N * K, dtype);
    if (!xd || !wd) { free(xd); free(wd); return 1; }
    (void)threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads > 0 ? threads : 1)
#endif
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            double t = 0.0;
            for (int k = 0; k < K; ++k) t += xd[(int64_t)m * K + k] * wd[(int64_t)n * K + k];
            if (bias) t += decode(bias[n], dtype);
            if (act == 1) t = 0.5 * t * (1.0 + erf(t / sqrt(2.0)));
            if (residual) t += decode(residual[(int64_t)m * N + n], dtype);
            y[(int64_t)m * N + n] = t;
        }
    }
    free(xd);
    free(wd);
    return 0;
}

/*
 * oracle_layernorm: per row, y = (x - mean) / sqrt(var + eps) * gamma + beta with the biased
 * variance (divide by C), the definition used by ViT encoders.
 */
void oracle_layernorm(const uint16_t *x, const uint16_t *gamma, const uint16_t *beta, int dtype,
                      int M, int C, double eps, double *y)
{
    for (int m = 0; m < M; ++m) {
        double mean = 0.0, var = 0.0;
        for (int c = 0; c < C; ++c) mean += decode(x[(int64_t)m * C + c], dtype);
        mean /= C;
        for (int c = 0; c < C; ++c) {
            double d = decode(x[(int64_t)m * C + c], dtype) - mean;
            var += d * d;
        }
        var /= C;
        double rstd = 1.0 / sqrt(var + eps);
        for (int c = 0; c < C; ++c)
            y[(int64_t)m * C + c] = (decode(x[(int64_t)m * C + c], dtype) - mean) * rstd *
                                        decode(gamma[c], dtype) + decode(beta[c], dtype);
    }
}

/*
 * A keep-mask producer (Section 5, "Experiments": the timings prune with a threshold on the l2 norm
 * of the token features at a fixed ratio; the paper does not define the method further, and
 * Section 4.3 item 2 accepts any method that yields a per-token keep mask).  Reading taken here:
 * a token's score is the squared l2 norm of its feature row; per image the class token (position 0)
 * is always kept and, of the remaining tokens, the k-1 with the largest score; equal scores are
 * ordered by position (lower first).  k >= N keeps everything.
 *
 * oracle_scores_l2: score[i][t] = sum_c x[i][t][c]^2 in double, c ascending.
 */
void oracle_scores_l2(const uint16_t *x, int dtype, int64_t rows, int C, double *scores)
{
    for (int64_t r = 0; r < rows; ++r) {
        double acc = 0.0;
        for (int c = 0; c < C; ++c) {
            double v = decode(x[r * C + c], dtype);
            acc += v * v;
        }
        scores[r] = acc;
    }
}

/*
 * oracle_keep_topk: keep[i][0] = 1; for t >= 1, keep[i][t] = 1 iff fewer than k-1 tokens u >= 1 of the
 * same image come before t in the order (score descending, position ascending).  Plain O(N^2) count.
 */
void oracle_keep_topk(const double *scores, int B, int N, int k, uint8_t *keep)
{
    for (int i = 0; i < B; ++i) {
        const double *s = scores + (int64_t)i * N;
        for (int t = 0; t < N; ++t) {
            int before = 0;
            for (int u = 1; u < N; ++u)
                if (u != t && (s[u] > s[t] || (s[u] == s[t] && u < t))) ++before;
            keep[(int64_t)i * N + t] = (uint8_t)((t == 0 || before < k - 1) ? 1 : 0);
        }
    }
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
