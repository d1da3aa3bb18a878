// Shared host/device declarations of the gfx950 ragged-attention library (internal; the public
// interface is include/ragged.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ragged.h"

namespace ragged {

constexpr int kWaveSize = 64;          // CDNA wavefront width
constexpr int kBlockThreads = 256;     // 4 wavefronts per work-group in every kernel here
constexpr int kXcds = 8;               // MI355X: 8 accelerator dies, work-groups dealt round-robin

// Enqueue one kernel and return the status of THIS launch.  (hipLaunchKernelGGL followed by
// hipGetLastError would also report -- and clear -- an error that unrelated earlier calls of the
// caller left behind.)  The arguments are converted to the kernel's parameter types.
template <typename T>
struct kernel_param { typedef T type; };
template <typename... Params>
inline hipError_t launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream,
                                typename kernel_param<Params>::type... args) {
    void* ptrs[sizeof...(Params) > 0 ? sizeof...(Params) : 1] = {const_cast<void*>(static_cast<const void*>(&args))...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, stream);
}

// Division by a number the host knows, without the hardware's 40-instruction integer division: with
// magic = floor((2^32 - 1) / d) the high half of n * magic is floor(n / d) or one less (the error
// n * (2^32 - magic*d) / (d * 2^32) is below n / 2^32 < 1), so one correction step makes it exact for
// every 32-bit n and every d >= 1.
inline uint32_t div_magic(uint32_t d) { return 0xFFFFFFFFu / d; }
__device__ __forceinline__ void divmod(uint32_t n, uint32_t d, uint32_t magic, uint32_t& quot, uint32_t& rem) {
    uint32_t q = __umulhi(n, magic);
    uint32_t r = n - q * d;
    if (r >= d) { ++q; r -= d; }
    quot = q;
    rem = r;
}

// Host launchers (one kernel each).  All arguments have been validated by the C ABI layer.
hipError_t launch_pack(const void* x, const uint8_t* keep, int B, int N, int C, void* packed,
                       int64_t cap_rows, int32_t* cu_seqlens, int32_t* gather_idx,
                       hipStream_t stream);
hipError_t launch_unpack(const void* src, const uint8_t* keep, const int32_t* cu_seqlens,
                         const int32_t* gather_idx, int B, int N, int C, void* out, int fill_mode,
                         hipStream_t stream);
// in_tok / out_tok: elements between consecutive tokens of q, k, v / of o
hipError_t launch_attn(const void* q, const void* k, const void* v, void* o,
                       const int32_t* cu_seqlens, int B, int max_seqlen, int H, int64_t in_tok,
                       int64_t out_tok, float scale, ragged_dtype in_dt, ragged_dtype out_dt,
                       int32_t* flags, hipStream_t stream);
hipError_t launch_attn_padded(const void* q, const void* k, const void* v, void* o, const uint8_t* keep,
                              int B, int N, int H, float scale, ragged_dtype in_dt, ragged_dtype out_dt,
                              int fill_mode, hipStream_t stream);
hipError_t launch_repack(const void* packed_in, const uint8_t* keep_rows, const int32_t* cu_in, int B,
                         int64_t cap_in, int C, void* packed_out, int64_t cap_out, int32_t* cu_out,
                         int32_t* gather_out, hipStream_t stream);
hipError_t launch_cls_extract(const void* packed, const int32_t* cu_seqlens, int B, int C, void* out,
                              hipStream_t stream);
// pack + attention + unpack of one layer in one launch (x, packed, o, out, q, k, v all of dtype dt)
hipError_t launch_step(const void* x, const uint8_t* keep, const void* q, const void* k, const void* v,
                       int B, int N, int H, float scale, ragged_dtype dt, void* packed, int64_t cap_rows,
                       int32_t* cu_seqlens, int32_t* gather_idx, void* o, void* out, int fill_mode,
                       hipStream_t stream);
// y = act(x w^T + bias) (+ residual) over packed rows; rows = min(rows_cap, *rows_dev) if rows_dev != null
hipError_t launch_linear(const void* x, const void* w, const void* bias, const void* res, void* y, int rows_cap,
                         const int32_t* rows_dev, int rows_hint, int N, int K, int act, ragged_dtype dt,
                         hipStream_t stream);
hipError_t launch_layernorm(const void* x, const void* gamma, const void* beta, void* y, int rows_cap,
                            const int32_t* rows_dev, int C, float eps, ragged_dtype dt, hipStream_t stream);
int layernorm_max_width();
hipError_t launch_token_scores_l2(const void* x, int64_t rows, int C, ragged_dtype dt, double* scores,
                                  hipStream_t stream);
hipError_t launch_keep_topk(const double* scores, int B, int N, int k, uint8_t* keep, hipStream_t stream);
int keep_topk_max_tokens();
int attn_padded_max_tokens();
hipError_t launch_noop(int grid, hipStream_t stream);

// Tokens of one image handled by one work-group of the pack / zero-filling unpack kernels.
// Small chunks expose more parallelism (the copies are latency-bound at ViT sizes); the chunk
// grows once the grid would exceed max_groups.  Measured: 4096 groups for the zero-filling unpack
// (what the 256 CUs hold resident); 2048 for pack, whose groups each recount the mask in front of
// their chunk -- fewer, larger chunks halve that work from B = 128 on (pack at B = 128, 20 % kept:
// 7.4 -> 5.9 us) and change nothing below.
inline int pick_chunk(int B, int N, int max_groups) {
    const int64_t tokens = (int64_t)B * N;
    int chunk = 8;
    while (chunk < 64 && tokens / chunk > max_groups) chunk *= 2;
    return chunk;
}
constexpr int kPackMaxGroups = 2048;
constexpr int kUnpackFillMaxGroups = 4096;

}  // namespace ragged
