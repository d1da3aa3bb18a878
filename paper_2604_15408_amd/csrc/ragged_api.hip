// C ABI of the library (declared in include/ragged.h): argument validation on the host, then
// exactly one kernel launch per call.  No allocation, no synchronisation, no host read-back, so
// every entry point may be recorded into a HIP graph.
#include <math.h>

#include "common.h"

namespace {

constexpr int kVersion = 800;  // 0.8.0

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool is16bit(ragged_dtype dt) { return dt == RAGGED_F16 || dt == RAGGED_BF16; }

// B*N rows must be indexable with int32 (gather_idx and cu_seqlens are int32).
inline bool rows_fit(int B, int N) { return (int64_t)B * N <= (int64_t)INT32_MAX; }

// The attention grid is (pairs of a dispatch batch, 64-row q-tiles, batches of 512 (image, head) pairs): the
// second and third dimension of a grid hold at most 65535, the whole grid fewer than 2^31 work-groups.
inline bool grid_fits(int B, int H, int bound) {
    const int64_t q_tiles = ((int64_t)bound + 63) / 64, batches = ((int64_t)B * H + 511) / 512;
    return q_tiles <= 65535 && batches <= 65535 && batches * 512 * q_tiles <= (int64_t)INT32_MAX;
}

inline int from_hip(hipError_t e) { return e == hipSuccess ? RAGGED_OK : RAGGED_ERR_HIP; }

// ragged_attn, ragged_attn_strided and ragged_attn_checked share the checks and the launch; flags may be null
int attn_call(const void* q, const void* k, const void* v, void* o,
              const int32_t* cu_seqlens, int B, int max_seqlen, int H, int D,
              int64_t in_tok_stride, int64_t out_tok_stride, float scale,
              ragged_dtype in_dt, ragged_dtype out_dt, int32_t* flags, void* stream) {
    if (!q || !k || !v || !o || !cu_seqlens) return RAGGED_ERR_NULL;
    if (B <= 0 || H <= 0 || D <= 0 || max_seqlen < 1) return RAGGED_ERR_SHAPE;
    if (!grid_fits(B, H, max_seqlen)) return RAGGED_ERR_SHAPE;
    const int64_t row = (int64_t)H * D;
    // the kernel addresses the 64 rows of a K/V tile with 32-bit byte offsets and takes the strides as int32
    if (in_tok_stride < row || out_tok_stride < row || in_tok_stride > (int64_t)1 << 23 ||
        out_tok_stride > (int64_t)INT32_MAX)
        return RAGGED_ERR_SHAPE;
    if (D != 64) return RAGGED_ERR_UNSUPPORTED;
    const bool pair_ok = (in_dt == RAGGED_F16 && (out_dt == RAGGED_F16 || out_dt == RAGGED_F32)) ||
                         (in_dt == RAGGED_BF16 && (out_dt == RAGGED_BF16 || out_dt == RAGGED_F32));
    if (!pair_ok || !isfinite(scale)) return RAGGED_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return RAGGED_ERR_UNSUPPORTED;
    // every token row must start on a 16-byte boundary
    const int64_t out_bytes = out_dt == RAGGED_F32 ? 4 : 2;
    if ((in_tok_stride * 2) % 16 != 0 || (out_tok_stride * out_bytes) % 16 != 0) return RAGGED_ERR_UNSUPPORTED;
    return from_hip(ragged::launch_attn(q, k, v, o, cu_seqlens, B, max_seqlen, H, in_tok_stride,
                                        out_tok_stride, scale, in_dt, out_dt, flags,
                                        static_cast<hipStream_t>(stream)));
}

}  // namespace

extern "C" {

int ragged_pack(const void* x, const uint8_t* keep, int B, int N, int C, ragged_dtype dt,
                void* packed, int64_t cap_rows, int32_t* cu_seqlens, int32_t* gather_idx,
                void* stream) {
    if (!x || !keep || !packed || !cu_seqlens || !gather_idx) return RAGGED_ERR_NULL;
    if (B <= 0 || N <= 0 || C <= 0 || !rows_fit(B, N)) return RAGGED_ERR_SHAPE;
    if (!is16bit(dt) || (C & 7) != 0 || !aligned16(x) || !aligned16(packed)) return RAGGED_ERR_UNSUPPORTED;
    if (cap_rows < 1) return RAGGED_ERR_CAPACITY;
    return from_hip(ragged::launch_pack(x, keep, B, N, C, packed, cap_rows, cu_seqlens, gather_idx,
                                        static_cast<hipStream_t>(stream)));
}

int ragged_attn_strided(const void* q, const void* k, const void* v, void* o,
                        const int32_t* cu_seqlens, int B, int max_seqlen, int H, int D,
                        int64_t in_tok_stride, int64_t out_tok_stride, float scale,
                        ragged_dtype in_dt, ragged_dtype out_dt, void* stream) {
    return attn_call(q, k, v, o, cu_seqlens, B, max_seqlen, H, D, in_tok_stride, out_tok_stride, scale, in_dt,
                     out_dt, nullptr, stream);
}

int ragged_attn_checked(const void* q, const void* k, const void* v, void* o,
                        const int32_t* cu_seqlens, int B, int max_seqlen, int H, int D,
                        int64_t in_tok_stride, int64_t out_tok_stride, float scale,
                        ragged_dtype in_dt, ragged_dtype out_dt, int32_t* flags, void* stream) {
    if (!flags) return RAGGED_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(flags) & 3u) != 0) return RAGGED_ERR_UNSUPPORTED;
    return attn_call(q, k, v, o, cu_seqlens, B, max_seqlen, H, D, in_tok_stride, out_tok_stride, scale, in_dt,
                     out_dt, flags, stream);
}

int ragged_attn(const void* q, const void* k, const void* v, void* o,
                const int32_t* cu_seqlens, int B, int max_seqlen, int H, int D,
                float scale, ragged_dtype in_dt, ragged_dtype out_dt, void* stream) {
    const int64_t row = (H > 0 && D > 0) ? (int64_t)H * D : 0;     // contiguous [T, H, D]
    return ragged_attn_strided(q, k, v, o, cu_seqlens, B, max_seqlen, H, D, row, row, scale, in_dt, out_dt,
                               stream);
}

int ragged_attn_padded(const void* q, const void* k, const void* v, void* o, const uint8_t* keep,
                       int B, int N, int H, int D, float scale, ragged_dtype in_dt,
                       ragged_dtype out_dt, int fill_mode, void* stream) {
    if (!q || !k || !v || !o || !keep) return RAGGED_ERR_NULL;
    if (B <= 0 || N <= 0 || H <= 0 || D <= 0 || !rows_fit(B, N)) return RAGGED_ERR_SHAPE;
    if (!grid_fits(B, H, N)) return RAGGED_ERR_SHAPE;
    if (D != 64 || N > ragged::attn_padded_max_tokens()) return RAGGED_ERR_UNSUPPORTED;
    // the kernel addresses the N rows of an image with 32-bit byte offsets
    if ((int64_t)N * H * D * 2 >= (int64_t)1 << 31) return RAGGED_ERR_SHAPE;
    if (fill_mode != 0 && fill_mode != 1) return RAGGED_ERR_UNSUPPORTED;
    const bool pair_ok = (in_dt == RAGGED_F16 && (out_dt == RAGGED_F16 || out_dt == RAGGED_F32)) ||
                         (in_dt == RAGGED_BF16 && (out_dt == RAGGED_BF16 || out_dt == RAGGED_F32));
    if (!pair_ok || !isfinite(scale)) return RAGGED_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return RAGGED_ERR_UNSUPPORTED;
    return from_hip(ragged::launch_attn_padded(q, k, v, o, keep, B, N, H, scale, in_dt, out_dt, fill_mode,
                                               static_cast<hipStream_t>(stream)));
}

int ragged_pack_attn_unpack(const void* x, const uint8_t* keep, const void* q, const void* k, const void* v,
                            int B, int N, int H, int D, float scale, ragged_dtype dt, void* packed,
                            int64_t cap_rows, int32_t* cu_seqlens, int32_t* gather_idx, void* o, void* out,
                            int fill_mode, void* stream) {
    if (!x || !keep || !q || !k || !v || !packed || !cu_seqlens || !gather_idx || !o || !out) return RAGGED_ERR_NULL;
    if (B <= 0 || N <= 0 || H <= 0 || D <= 0 || !rows_fit(B, N)) return RAGGED_ERR_SHAPE;
    if (!grid_fits(B, H, N) || (int64_t)N * H * D * 2 >= (int64_t)1 << 31) return RAGGED_ERR_SHAPE;
    if (D != 64 || N > ragged::attn_padded_max_tokens() || !is16bit(dt)) return RAGGED_ERR_UNSUPPORTED;
    if ((fill_mode != 0 && fill_mode != 1) || !isfinite(scale)) return RAGGED_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(packed) || !aligned16(o) ||
        !aligned16(out))
        return RAGGED_ERR_UNSUPPORTED;
    if (cap_rows < (int64_t)B * N) return RAGGED_ERR_CAPACITY;
    return from_hip(ragged::launch_step(x, keep, q, k, v, B, N, H, scale, dt, packed, cap_rows, cu_seqlens,
                                        gather_idx, o, out, fill_mode, static_cast<hipStream_t>(stream)));
}

int ragged_unpack(const void* src, const uint8_t* keep, const int32_t* cu_seqlens,
                  const int32_t* gather_idx, int B, int N, int C, ragged_dtype dt,
                  void* out, int fill_mode, void* stream) {
    if (fill_mode != 0 && fill_mode != 1) return RAGGED_ERR_UNSUPPORTED;
    if (!src || !cu_seqlens || !out) return RAGGED_ERR_NULL;
    if (fill_mode == 0 && !gather_idx) return RAGGED_ERR_NULL;
    if (fill_mode == 1 && !keep) return RAGGED_ERR_NULL;
    if (B <= 0 || N <= 0 || C <= 0 || !rows_fit(B, N)) return RAGGED_ERR_SHAPE;
    if (!is16bit(dt) || (C & 7) != 0 || !aligned16(src) || !aligned16(out)) return RAGGED_ERR_UNSUPPORTED;
    return from_hip(ragged::launch_unpack(src, keep, cu_seqlens, gather_idx, B, N, C, out, fill_mode,
                                          static_cast<hipStream_t>(stream)));
}

int ragged_repack(const void* packed_in, const uint8_t* keep_rows, const int32_t* cu_in, int B,
                  int64_t cap_in, int C, ragged_dtype dt, void* packed_out, int64_t cap_out,
                  int32_t* cu_out, int32_t* gather_out, void* stream) {
    if (!packed_in || !keep_rows || !cu_in || !packed_out || !cu_out || !gather_out) return RAGGED_ERR_NULL;
    if (B <= 0 || C <= 0 || cap_in > (int64_t)INT32_MAX - 64) return RAGGED_ERR_SHAPE;
    if (!is16bit(dt) || (C & 7) != 0 || !aligned16(packed_in) || !aligned16(packed_out)) return RAGGED_ERR_UNSUPPORTED;
    if (cap_in < 1 || cap_out < 1) return RAGGED_ERR_CAPACITY;
    return from_hip(ragged::launch_repack(packed_in, keep_rows, cu_in, B, cap_in, C, packed_out, cap_out,
                                          cu_out, gather_out, static_cast<hipStream_t>(stream)));
}

int ragged_cls_extract(const void* packed, const int32_t* cu_seqlens, int B, int C, ragged_dtype dt,
                       void* out, void* stream) {
    if (!packed || !cu_seqlens || !out) return RAGGED_ERR_NULL;
    if (B <= 0 || C <= 0) return RAGGED_ERR_SHAPE;
    if (!is16bit(dt) || (C & 7) != 0 || !aligned16(packed) || !aligned16(out)) return RAGGED_ERR_UNSUPPORTED;
    return from_hip(ragged::launch_cls_extract(packed, cu_seqlens, B, C, out, static_cast<hipStream_t>(stream)));
}

int ragged_linear(const void* x, const void* w, const void* bias, const void* residual, void* y,
                  int64_t rows_cap, const int32_t* rows_dev, int64_t rows_hint, int N, int K, int act,
                  ragged_dtype dt, void* stream) {
    if (!x || !w || !y) return RAGGED_ERR_NULL;
    if (rows_hint < 0 || rows_hint > rows_cap) return RAGGED_ERR_SHAPE;
    if (rows_cap < 1 || rows_cap > (int64_t)INT32_MAX - 256 || N <= 0 || K <= 0 || K > (1 << 22)) return RAGGED_ERR_SHAPE;
    if (rows_cap * (int64_t)(N / 64 + 1) > (int64_t)INT32_MAX) return RAGGED_ERR_SHAPE;    // 32-bit grid
    if (!is16bit(dt) || (N % 64) != 0 || (K % 64) != 0 || (act != 0 && act != 1)) return RAGGED_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(bias) || !aligned16(residual))
        return RAGGED_ERR_UNSUPPORTED;
    return from_hip(ragged::launch_linear(x, w, bias, residual, y, (int)rows_cap, rows_dev,
                                          (int)(rows_hint > 0 ? rows_hint : rows_cap), N, K, act, dt,
                                          static_cast<hipStream_t>(stream)));
}

int ragged_layernorm(const void* x, const void* gamma, const void* beta, void* y, int64_t rows_cap,
                     const int32_t* rows_dev, int C, float eps, ragged_dtype dt, void* stream) {
    if (!x || !gamma || !beta || !y) return RAGGED_ERR_NULL;
    if (rows_cap < 1 || rows_cap > (int64_t)INT32_MAX - 256 || C <= 0) return RAGGED_ERR_SHAPE;
    if (!is16bit(dt) || (C & 7) != 0 || C > ragged::layernorm_max_width() || !(eps >= 0.f) || !isfinite(eps))
        return RAGGED_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y)) return RAGGED_ERR_UNSUPPORTED;
    return from_hip(ragged::launch_layernorm(x, gamma, beta, y, (int)rows_cap, rows_dev, C, eps, dt,
                                             static_cast<hipStream_t>(stream)));
}

int ragged_token_scores_l2(const void* x, int64_t rows, int C, ragged_dtype dt, double* scores, void* stream) {
    if (!x || !scores) return RAGGED_ERR_NULL;
    if (rows < 1 || rows > (int64_t)INT32_MAX || C <= 0) return RAGGED_ERR_SHAPE;
    if (!is16bit(dt) || (C & 7) != 0 || !aligned16(x) || (reinterpret_cast<uintptr_t>(scores) & 7u) != 0)
        return RAGGED_ERR_UNSUPPORTED;
    return from_hip(ragged::launch_token_scores_l2(x, rows, C, dt, scores, static_cast<hipStream_t>(stream)));
}

int ragged_keep_topk(const double* scores, int B, int N, int k, uint8_t* keep, void* stream) {
    if (!scores || !keep) return RAGGED_ERR_NULL;
    if (B <= 0 || N <= 0 || k < 1 || !rows_fit(B, N)) return RAGGED_ERR_SHAPE;
    if (N > ragged::keep_topk_max_tokens() || (reinterpret_cast<uintptr_t>(scores) & 7u) != 0)
        return RAGGED_ERR_UNSUPPORTED;
    return from_hip(ragged::launch_keep_topk(scores, B, N, k, keep, static_cast<hipStream_t>(stream)));
}

int ragged_noop(int grid, void* stream) {
    if (grid < 1) return RAGGED_ERR_SHAPE;
    return from_hip(ragged::launch_noop(grid, static_cast<hipStream_t>(stream)));
}

const char* ragged_status_string(int status) {
    switch (status) {
        case RAGGED_OK: return "ok";
        case RAGGED_ERR_NULL: return "a required pointer is NULL";
        case RAGGED_ERR_SHAPE: return "a dimension is non-positive or too large";
        case RAGGED_ERR_UNSUPPORTED: return "unsupported dtype, head dim, alignment, scale or fill mode";
        case RAGGED_ERR_CAPACITY: return "a row capacity is too small";
        case RAGGED_ERR_HIP: return "the HIP runtime refused the launch";
        default: return "unknown";
    }
}

int ragged_version(void) { return kVersion; }

}  // extern "C"
