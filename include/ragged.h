/*
 * ragged.h -- C ABI of the MI355X (gfx950) pack -> ragged attention -> unpack library.
 *
 * The three stages are the pack-attend-unpack pipeline of "Dispatch-Aware Ragged Attention for
 * Pruned Vision Transformers" (Section 4, "Method"): a keep mask produced by any token-pruning
 * method selects the surviving tokens of each image; they are packed into one flat buffer indexed
 * by cu_seqlens, attended per image, and scattered back.
 *
 * Conventions shared by every entry point
 *   - B images, N tokens per image before pruning, H heads, head dim D, row width C = H*D.
 *   - n_i = kept tokens of image i, T = sum_i n_i = cu_seqlens[B].
 *   - Every pointer except `stream` is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or keeps a pointer, never synchronises and never copies to the host: each
 *     call enqueues exactly one kernel on `stream` and returns, so all calls are legal inside a
 *     HIP stream capture.  T is never read on the host; grids are sized by upper bounds and
 *     surplus work-groups exit on the device.
 *   - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *   - 16-bit floating rows are moved as raw words by pack / unpack (bit copy).
 *   - Return value: a ragged_status.  RAGGED_OK means "enqueued".  Arguments are validated on the
 *     host before anything is launched; a validation failure launches nothing.
 *   - x, packed, src, out, q, k, v, o must be 16-byte aligned; C must be a multiple of 8.
 *   - Calls on one stream are ordered; the caller orders calls across streams.
 */
#ifndef RAGGED_H
#define RAGGED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RAGGED_OK = 0,
    RAGGED_ERR_NULL = 1,         /* a required pointer is NULL                                   */
    RAGGED_ERR_SHAPE = 2,        /* a dimension is <= 0, overflows int32 row indexing, or a token
                                    stride is shorter than a row                                  */
    RAGGED_ERR_UNSUPPORTED = 3,  /* dtype pair, head dim, alignment or fill mode not supported    */
    RAGGED_ERR_CAPACITY = 4,     /* a row capacity is < 1 (ragged_pack_attn_unpack: < B*N)        */
    RAGGED_ERR_HIP = 5           /* the HIP runtime refused the launch                            */
} ragged_status;

typedef enum {
    RAGGED_F16 = 0,              /* IEEE binary16                                                 */
    RAGGED_BF16 = 1,             /* bfloat16                                                      */
    RAGGED_F32 = 2               /* IEEE binary32; attention output only                          */
} ragged_dtype;

/*
 * ragged_pack -- Section 4.1 "Fused Token Packing", both phases in ONE launch and without the
 * paper's host read of the total kept count.
 *
 *   x          [B, N, C]   16-bit rows (dt = RAGGED_F16 or RAGGED_BF16; only the width matters)
 *   keep       [B, N]      one byte per token, any nonzero value = keep
 *   packed     [cap_rows, C]  out: kept rows in stable order (images ascending, tokens ascending)
 *   cu_seqlens [B + 1]     out: cu[0] = 0, cu[i+1] = cu[i] + n_i
 *   gather_idx [cap_rows]  out: gather_idx[r] = flat source row i*N + t of packed row r
 *
 * Cost note: every work-group recounts the keep bytes in front of its chunk (no grid-wide scan, no second
 * launch, no workspace), i.e. O(B*N) mask bytes per work-group from L2.  That is free at ViT batch sizes (B*N up to
 * a few 10^4) and grows quadratically with the batch: around B*N = 10^6 the recount costs as much as the copy.
 * ragged_repack and ragged_pack_attn_unpack count the same way.
 *
 * cap_rows is the row capacity of `packed` and `gather_idx`.  B*N always suffices.  Rows whose
 * destination would be >= cap_rows are not written (cu_seqlens still holds the true counts, so the
 * caller can detect the overflow from cu_seqlens[B] afterwards).  Rows >= T are left untouched.
 */
int ragged_pack(const void* x, const uint8_t* keep, int B, int N, int C, ragged_dtype dt,
                void* packed, int64_t cap_rows, int32_t* cu_seqlens, int32_t* gather_idx,
                void* stream);

/*
 * ragged_attn -- Section 4.2 "Ragged Attention Kernel" (Algorithm 1): for every image i, head h
 * and query row r of that image,
 *     o[s+r, h, :] = softmax_j( scale * q[s+r, h, :] . k[s+j, h, :] ) v[s+j, h, :],
 *     s = cu_seqlens[i], j in [0, n_i)
 * bidirectional (no causal mask), no dropout, keys of other images never take part.
 *
 *   q, k, v    [T, H, D]   token-major, then head, then head dim contiguous (in_dt)
 *   o          [T, H, D]   out (out_dt); rows >= T are left untouched
 *   cu_seqlens [B + 1]     as written by ragged_pack
 *   max_seqlen             host-known upper bound on every n_i (N always works); it only sizes
 *                          the grid.  Query rows at positions >= max_seqlen inside an image are
 *                          NOT computed, so a bound that is too small loses rows (ragged_attn_checked
 *                          reports that case on the device).
 *   scale                  finite fp32 softmax scale (the paper uses 1/sqrt(D))
 *
 * Supported: D = 64; (in_dt, out_dt) in {F16->F16, F16->F32, BF16->BF16, BF16->F32}.
 * Limits of the launch (RAGGED_ERR_SHAPE beyond them; the same for every attention entry point, with N in
 * place of max_seqlen where the call has no bound): max_seqlen <= 64 * 65535, B * H <= 512 * 65535, and
 * ceil(B*H / 512) * 512 * ceil(max_seqlen / 64) < 2^31 work-groups.
 * Contractions run on MFMA with fp32 accumulation; the softmax runs in fp32.
 * Images with n_i = 0 produce no rows.  Results are bit-reproducible from run to run with the same arguments.
 * The launch shape follows B, H and max_seqlen (small launches split the keys of a sequence over the wavefronts
 * of a work-group and merge the partial results, large ones walk them in order), so the bits of a sequence
 * longer than 64 tokens may differ in the last place between calls with different B, H or max_seqlen; all the
 * entry points of this header take the same shape for the same (B, H, bound), so they stay bit-identical to
 * each other.
 */
int ragged_attn(const void* q, const void* k, const void* v, void* o,
                const int32_t* cu_seqlens, int B, int max_seqlen, int H, int D,
                float scale, ragged_dtype in_dt, ragged_dtype out_dt, void* stream);

/*
 * ragged_attn_strided -- ragged_attn on token rows that are not contiguous: token t of q, k, v
 * starts in_tok_stride elements after token t-1, token t of o out_tok_stride elements after its
 * predecessor; inside a token the layout stays [H, D].  This is what the late layers of Section 4.3
 * ("End-to-End Pipeline Integration", step 4: attention and MLP run on the packed buffer) need
 * between their linear layers: the QKV projection of packed rows writes one [T, 3, H, D] buffer, and
 * q = base, k = base + H*D, v = base + 2*H*D with in_tok_stride = 3*H*D attends on it in place,
 * without three de-interleaving copies.  ragged_attn is this call with both strides = H*D.
 *
 * Strides are in elements of the respective dtype, must be >= H*D (in_tok_stride also <= 2^23 and
 * out_tok_stride < 2^31, else RAGGED_ERR_SHAPE), and every token row must start
 * on a 16-byte boundary (in_tok_stride a multiple of 8; out_tok_stride a multiple of 8 for 16-bit
 * outputs, of 4 for F32).  Everything else as for ragged_attn; outputs are bit-identical to
 * ragged_attn on contiguous copies of the same rows.
 */
int ragged_attn_strided(const void* q, const void* k, const void* v, void* o,
                        const int32_t* cu_seqlens, int B, int max_seqlen, int H, int D,
                        int64_t in_tok_stride, int64_t out_tok_stride, float scale,
                        ragged_dtype in_dt, ragged_dtype out_dt, void* stream);

/*
 * ragged_attn_checked -- ragged_attn_strided that also reports a `max_seqlen` that was too small.
 * Section 4.2 sizes its grid from the host-known sequence bound; here that bound is an argument, a bound
 * below some n_i silently leaves query rows of that image uncomputed, and the host cannot see n_i without
 * the synchronisation this library avoids.  This entry point closes the gap on the device:
 *
 *   flags      [1]  int32, caller-zeroed.  Bit 0 (RAGGED_FLAG_SEQLEN_EXCEEDED) is OR-ed in when some image
 *                   has n_i > max_seqlen.  The library never clears it; the caller reads it whenever it
 *                   next synchronises (or never).
 *
 * Query rows at positions >= max_seqlen of an offending image may be left uncomputed (such a row of `o` then stays
 * untouched as a whole; rows at positions >= 64 * ceil(max_seqlen / 64) always do); every other row of the batch is
 * computed as by ragged_attn_strided with the same arguments, bit for bit.
 * ragged_pack_attn_unpack and ragged_attn_padded size their grids from N itself and can never lose a row.
 */
#define RAGGED_FLAG_SEQLEN_EXCEEDED 1
int ragged_attn_checked(const void* q, const void* k, const void* v, void* o,
                        const int32_t* cu_seqlens, int B, int max_seqlen, int H, int D,
                        int64_t in_tok_stride, int64_t out_tok_stride, float scale,
                        ragged_dtype in_dt, ragged_dtype out_dt, int32_t* flags, void* stream);

/*
 * ragged_unpack -- the inverse scatter of ragged_pack (the paper names the stage in its
 * "pack-attend-unpack pipeline", Sections 1 and 4, without describing it).
 *
 *   src        [T, C]      packed rows
 *   out        [B, N, C]   out: out[i, t, :] = src[cu[i] + rank(i, t), :] for kept tokens
 *   fill_mode  0: dropped rows of `out` are left untouched.  Reads gather_idx and cu_seqlens[B];
 *                 `keep` may be NULL.
 *              1: dropped rows are written with +0 words, so every byte of `out` is defined.
 *                 Reads keep and cu_seqlens; `gather_idx` may be NULL.
 */
int ragged_unpack(const void* src, const uint8_t* keep, const int32_t* cu_seqlens,
                  const int32_t* gather_idx, int B, int N, int C, ragged_dtype dt,
                  void* out, int fill_mode, void* stream);

/*
 * ragged_attn_padded -- the whole pack-attend-unpack pipeline of Section 4 for ONE attention layer
 * in ONE launch: the kernel turns each image's keep mask into its list of kept token positions and
 * reads / writes Q, K, V, O rows through that list, so no packed copy, no cu_seqlens and no gather
 * index exist.  Same arithmetic as ragged_attn on the packed rows (bit-identical outputs).  The
 * paper's argument (Section 3 and Section 4.2, "Why dispatch overhead is lower") is that at ViT sizes
 * the number of dispatches, not the arithmetic, sets the latency; this entry point removes two of
 * the three.
 *
 *   q, k, v    [B, N, H, D]  padded, token-major inside an image (in_dt); rows of dropped tokens are
 *                            never read
 *   o          [B, N, H, D]  out (out_dt): rows of kept tokens receive the attention output;
 *                            fill_mode 0 leaves rows of dropped tokens untouched, 1 writes +0
 *   keep       [B, N]        one byte per token, any nonzero value = keep
 *
 * Supported: D = 64, N <= 1536, the dtype pairs of ragged_attn.  Images with nothing kept produce no
 * attention rows.
 */
int ragged_attn_padded(const void* q, const void* k, const void* v, void* o, const uint8_t* keep,
                       int B, int N, int H, int D, float scale, ragged_dtype in_dt,
                       ragged_dtype out_dt, int fill_mode, void* stream);

/*
 * ragged_pack_attn_unpack -- ragged_pack, ragged_attn and ragged_unpack of one layer (the three
 * stages of Section 4) in ONE launch, with every output of the three calls produced and bit-identical
 * to theirs.  Section 3 and Section 4.2 ("Why dispatch overhead is lower") argue that at ViT sizes the
 * number of dispatches sets the latency; this entry point is that argument applied to the paper's
 * own pipeline.  Each work-group (image, head, 64-query tile) recounts the image's first packed row
 * and its kept-token list from the keep mask, so there is no dependency between work-groups.
 *
 *   x          [B, N, C]      padded features (dt), C = H*D
 *   keep       [B, N]         one byte per token, nonzero = keep
 *   q, k, v    [cap_rows, H, D]  ALREADY packed query / key / value rows (dt); rows [0, T) are read
 *   packed     [cap_rows, C]  out: as from ragged_pack(x, keep)
 *   cu_seqlens [B + 1]        out: as from ragged_pack
 *   gather_idx [cap_rows]     out: as from ragged_pack
 *   o          [cap_rows, H, D]  out (dt): as from ragged_attn(q, k, v, cu_seqlens)
 *   out        [B, N, C]      out: as from ragged_unpack(o, ..., fill_mode)
 *
 * Supported: D = 64, N <= 1536, dt = F16 or BF16 (o has the input dtype).  cap_rows must be >= B*N
 * (RAGGED_ERR_CAPACITY otherwise), so nothing can overflow.  x, packed, o, out must not overlap.
 */
int ragged_pack_attn_unpack(const void* x, const uint8_t* keep, const void* q, const void* k, const void* v,
                            int B, int N, int H, int D, float scale, ragged_dtype dt, void* packed,
                            int64_t cap_rows, int32_t* cu_seqlens, int32_t* gather_idx, void* o, void* out,
                            int fill_mode, void* stream);

/*
 * ragged_repack -- a second pruning decision applied to rows that are ALREADY packed.  Section 4.3
 * packs once and keeps every later layer on the packed buffer; pruning methods that drop tokens
 * at several depths (Section 2, "Token Pruning for ViTs": DynamicViT and EViT prune progressively)
 * then need a keep mask applied to packed rows, instead of an unpack -> pack round trip through
 * the padded tensor.  Equivalent to ragged_pack with the AND of both masks, in one launch:
 *
 *   packed_in  [cap_in, C]  packed rows; rows [0, T_in) are valid, T_in = cu_in[B] <= cap_in
 *   keep_rows  [cap_in]     one byte per packed row, nonzero = keep; bytes at rows >= T_in are ignored
 *   cu_in      [B + 1]      boundaries of packed_in
 *   packed_out [cap_out, C] out: kept rows in the same order
 *   cu_out     [B + 1]      out: cu_out[i] = number of kept rows before row cu_in[i]
 *   gather_out [cap_out]    out: gather_out[r] = row of packed_in that packed_out row r came from
 *                           (compose with the first gather_idx to get back to the padded tensor)
 *
 * Rows whose destination would be >= cap_out are not written (cu_out still holds the true counts).
 * packed_out must not overlap packed_in; cu_out must not alias cu_in.
 */
int ragged_repack(const void* packed_in, const uint8_t* keep_rows, const int32_t* cu_in, int B,
                  int64_t cap_in, int C, ragged_dtype dt, void* packed_out, int64_t cap_out,
                  int32_t* cu_out, int32_t* gather_out, void* stream);

/*
 * ragged_cls_extract -- step 5 of Section 4.3: the classifier reads each image's class token from
 * the packed buffer.  Packing keeps token order (Section 4.1), so a class token at position 0 that
 * the keep mask retains is the image's first packed row.
 *
 *   packed     [T, C]   packed rows
 *   cu_seqlens [B + 1]
 *   out        [B, C]   out: out[i, :] = packed[cu_seqlens[i], :]; +0 words for an image with no rows
 */
int ragged_cls_extract(const void* packed, const int32_t* cu_seqlens, int B, int C, ragged_dtype dt,
                       void* out, void* stream);

/*
 * ragged_linear -- a linear layer over packed rows, for the encoder blocks that Section 4.3 (item 4)
 * runs on the packed buffer after the pruning point (QKV projection, attention output projection and
 * the two MLP layers; Section 6, "Implications for pruning research", attributes most of the
 * realised speed-up of pruning to these, because their cost is linear in the number of kept tokens):
 *     y[m, n] = act( sum_k x[m, k] * w[n, k] + bias[n] ) + residual[m, n]
 *
 *   x        [rows_cap, K]  packed activations (dt)
 *   w        [N, K]         weights, one output feature per row (dt)
 *   bias     [N] or NULL    (dt)
 *   residual [rows_cap, N] or NULL (dt); may be the same buffer as y (each element is read before
 *                           it is written, by the same thread)
 *   y        [rows_cap, N]  out (dt); must not overlap x
 *   rows_dev                NULL, or a DEVICE pointer to the number of valid rows (for example
 *                           &cu_seqlens[B]); rows processed = min(rows_cap, *rows_dev), read on the
 *                           device, so the call stays capturable.  Rows beyond are left untouched.
 *   rows_hint               0, or the caller's estimate of the valid row count (1 <= rows_hint <=
 *                           rows_cap), e.g. keep ratio * B * N: it only chooses the launch shape (the
 *                           result and the rows written do not depend on it).  0 means rows_cap.
 *   act                     0: none, 1: GELU in its erf form t * Phi(t)
 *
 * Supported: dt = F16 or BF16, N and K multiples of 64, K <= 2^22.  MFMA with fp32
 * accumulation; bias, activation and residual are applied in fp32 before the single rounding to dt.
 */
int ragged_linear(const void* x, const void* w, const void* bias, const void* residual, void* y,
                  int64_t rows_cap, const int32_t* rows_dev, int64_t rows_hint, int N, int K, int act,
                  ragged_dtype dt, void* stream);

/*
 * ragged_layernorm -- LayerNorm over the feature dimension of packed rows (same blocks as above):
 *     y[m, :] = (x[m, :] - mean) / sqrt(var + eps) * gamma + beta,   var = biased variance of the row
 * x, y [rows_cap, C]; gamma, beta [C]; rows_dev as for ragged_linear.  y may be x.
 * Supported: dt = F16 or BF16, C a multiple of 8 and <= 2048, eps >= 0.  Statistics in fp32.
 */
int ragged_layernorm(const void* x, const void* gamma, const void* beta, void* y, int64_t rows_cap,
                     const int32_t* rows_dev, int C, float eps, ragged_dtype dt, void* stream);

/*
 * ragged_token_scores_l2 and ragged_keep_topk -- a keep-mask producer in front of ragged_pack.  The
 * pipeline takes its keep mask from any pruning method (Section 4.3 item 2); the paper's timings use
 * a threshold on the l2 norm of the token features at a fixed ratio (Section 5) and leave the method
 * undefined.  The definition taken here: score = squared l2 norm of the token's feature row; per
 * image the class token (position 0) is kept and, of the other tokens, the k-1 with the largest
 * score, equal scores ordered by position (lower first).  Every image then keeps min(k, N) tokens,
 * the uniform-length setting of the paper's kernel-latency tables.  ragged_keep_topk is independent
 * of how the scores were made (attention-based scores of other pruning methods fit as well).
 *
 *   x      [rows, C]   token features (dt), rows = B*N
 *   scores [rows]      out / in: fp64, 8-byte aligned.  Accumulated in fp64 (squares of 16-bit values
 *                      are exact there), so ranking does not depend on the summation order except
 *                      between scores that agree to the last bit of a rounded sum
 *   keep   [B, N]      out: 1 = keep, 0 = drop
 *
 * Supported: dt = F16 or BF16, C a multiple of 8; N <= 1536, k >= 1 (k >= N keeps everything).
 */
int ragged_token_scores_l2(const void* x, int64_t rows, int C, ragged_dtype dt, double* scores, void* stream);
int ragged_keep_topk(const double* scores, int B, int N, int k, uint8_t* keep, void* stream);

/*
 * ragged_noop -- enqueue an empty kernel of `grid` work-groups of 256 threads on `stream`.
 * It exists to measure the launch floor that Section 3 ("The Dispatch Overhead") is about,
 * separately from the time the real kernels spend on the GPU.
 */
int ragged_noop(int grid, void* stream);

/* Text for a ragged_status (static storage; never free it).  Unknown codes give "unknown". */
const char* ragged_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int ragged_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RAGGED_H */
