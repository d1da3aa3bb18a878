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
    RAGGED_ERR_SHAPE = 2,        /* a dimension is <= 0, overflows int32 row indexing, or C != H*D */
    RAGGED_ERR_UNSUPPORTED = 3,  /* dtype pair, head dim, alignment or fill mode not supported    */
    RAGGED_ERR_CAPACITY = 4,     /* cap_rows < 1                                                  */
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
 *                          NOT computed, so a bound that is too small loses rows.
 *   scale                  finite fp32 softmax scale (the paper uses 1/sqrt(D))
 *
 * Supported: D = 64; (in_dt, out_dt) in {F16->F16, F16->F32, BF16->BF16, BF16->F32}.
 * Contractions run on MFMA with fp32 accumulation; the softmax runs in fp32.
 * Images with n_i = 0 produce no rows.  Results are bit-reproducible from run to run.
 */
int ragged_attn(const void* q, const void* k, const void* v, void* o,
                const int32_t* cu_seqlens, int B, int max_seqlen, int H, int D,
                float scale, ragged_dtype in_dt, ragged_dtype out_dt, void* stream);

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
