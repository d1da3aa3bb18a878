// A keep-mask producer for the pipeline's first stage (Section 4.3 item 2 accepts any method that
// yields a per-token keep mask; Section 5 prunes by a threshold on the l2 norm of the token features
// at a fixed ratio without defining it further).  Two kernels:
//   token_scores_l2_kernel: score[row] = sum_c x[row][c]^2.  One wavefront per row, fp64
//     accumulation: a square of a 16-bit value is exact in fp64, so for ordinary data the score does
//     not depend on the summation order and ranking decisions agree with any other exact evaluation.
//   keep_topk_kernel: per image, token 0 (the class token) is kept and, of the others, the k-1 with
//     the largest score (equal scores: lower position first).  Scores of the image in LDS, an O(N)
//     count per token split over eight lanes -- N is a few hundred.
#include "common.h"
#include "mfma_lds.h"

namespace ragged {
namespace {

constexpr int kMaxMaskTokens = 1536;

template <typename V8>
__global__ __launch_bounds__(kBlockThreads)
void token_scores_l2_kernel(const uint4* __restrict__ x, int64_t rows, int chunks, double* __restrict__ scores) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int64_t row = (int64_t)blockIdx.x * (kBlockThreads / kWaveSize) + (threadIdx.x >> 6);
    if (row >= rows) return;
    const uint4* src = x + row * chunks;
    double acc = 0.0;
    for (int c = lane; c < chunks; c += kWaveSize) {
        const V8 v = as_vec8<V8>(src[c]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const double d = (double)(float)v[e];
            acc = __builtin_fma(d, d, acc);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, kWaveSize);
    if (lane == 0) scores[row] = acc;
}

// One work-group per (image, 32 tokens): eight lanes share a token and split the range of rivals
// u = 1 .. N-1 between them (u = 1 + part, 9 + part, ...), so the counting loop is an eighth as long and
// the image's scores are read from LDS; the eight partial counts meet in a three-step reduction.
constexpr int kTopkLanes = 8;
constexpr int kTopkTokens = kBlockThreads / kTopkLanes;

__global__ __launch_bounds__(kBlockThreads)
void keep_topk_kernel(const double* __restrict__ scores, int N, int k, int chunks, uint8_t* __restrict__ keep) {
    __shared__ double s[kMaxMaskTokens];
    const int img = blockIdx.x / chunks;
    const int t = (blockIdx.x - img * chunks) * kTopkTokens + threadIdx.x / kTopkLanes;
    const int part = threadIdx.x % kTopkLanes;
    const double* mine = scores + (int64_t)img * N;
    for (int u = threadIdx.x; u < N; u += kBlockThreads) s[u] = mine[u];
    __syncthreads();
    const double st = s[t < N ? t : 0];
    int before = 0;
#pragma unroll 4
    for (int u = 1 + part; u < N; u += kTopkLanes) {
        const double su = s[u];
        before += (u != t && (su > st || (su == st && u < t))) ? 1 : 0;
    }
    before += __shfl_xor(before, 1, kWaveSize);
    before += __shfl_xor(before, 2, kWaveSize);
    before += __shfl_xor(before, 4, kWaveSize);
    if (part == 0 && t < N) keep[(int64_t)img * N + t] = (uint8_t)((t == 0 || before < k - 1) ? 1 : 0);
}

}  // namespace

int keep_topk_max_tokens() { return kMaxMaskTokens; }

hipError_t launch_token_scores_l2(const void* x, int64_t rows, int C, ragged_dtype dt, double* scores,
                                  hipStream_t stream) {
    const int per = kBlockThreads / kWaveSize;
    const dim3 grid((unsigned)((rows + per - 1) / per)), block(kBlockThreads);
    hipError_t err;
    if (dt == RAGGED_F16)
        err = launch_kernel((token_scores_l2_kernel<f16x8>), grid, block, stream, static_cast<const uint4*>(x), rows, C / 8, scores);
    else
        err = launch_kernel((token_scores_l2_kernel<bf16x8>), grid, block, stream, static_cast<const uint4*>(x), rows, C / 8, scores);
    return err;
}

hipError_t launch_keep_topk(const double* scores, int B, int N, int k, uint8_t* keep, hipStream_t stream) {
    const int chunks = (N + kTopkTokens - 1) / kTopkTokens;
    const hipError_t err = launch_kernel(keep_topk_kernel, dim3(B * chunks), dim3(kBlockThreads), stream, scores, N, k, chunks, keep);
    return err;
}

}  // namespace ragged
