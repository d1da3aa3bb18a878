// Achievable ceilings of one MI355X, measured by the benchmark beside the kernels of the library (not
// part of the C ABI in include/ragged.h; built into its own small shared library):
//   * a streaming read and a streaming copy of a large buffer -- what an HBM-bound kernel can approach;
//   * a register-resident MFMA loop (fp16 16x16x32, no memory traffic) -- the matrix-core rate.
// Each entry point enqueues exactly one kernel on the given stream and returns hipError_t as int.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;        // 16-byte loads per thread in flight

// NT: non-temporal loads / stores (the data is touched once, so it need not displace cache contents)
template <bool NT>
__device__ __forceinline__ uint4 load16(const uint4* p) {
    if (NT) {
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
    return *p;
}
template <bool NT>
__device__ __forceinline__ void store16(uint4* p, uint4 v) {
    if (NT) {
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 w = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(p));
    } else {
        *p = v;
    }
}

template <bool NT>
__global__ __launch_bounds__(kThreads)
void stream_read_kernel(const uint4* __restrict__ src, int64_t words, uint32_t* __restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    uint32_t acc = 0;
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    for (; i + (kUnroll - 1) * stride < words; i += kUnroll * stride) {
        uint4 w[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) w[u] = load16<NT>(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc ^= w[u].x ^ w[u].y ^ w[u].z ^ w[u].w;
    }
    for (; i < words; i += stride) {
        const uint4 w = load16<NT>(src + i);
        acc ^= w.x ^ w.y ^ w.z ^ w.w;
    }
    // the buffer is filled with one repeated word by the caller, so the xor of an even number of words is 0;
    // the store below never happens but keeps the loads alive
    if (acc == 0x9e3779b9u) sink[threadIdx.x] = acc;
}

template <bool NT>
__global__ __launch_bounds__(kThreads)
void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t words) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    for (; i + (kUnroll - 1) * stride < words; i += kUnroll * stride) {
        uint4 w[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) w[u] = load16<NT>(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) store16<NT>(dst + i + u * stride, w[u]);
    }
    for (; i < words; i += stride) store16<NT>(dst + i, load16<NT>(src + i));
}

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kChains = 8;        // independent accumulators per wavefront: the matrix core never waits on a result

__global__ __launch_bounds__(kThreads)
void mfma_loop_kernel(int iters, float* __restrict__ sink) {
    f16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (_Float16)(1e-3f * (float)((threadIdx.x + e) & 7));
        b[e] = (_Float16)(1e-3f * (float)((threadIdx.x * 3 + e) & 7));
    }
    f32x4 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kChains; ++c) s += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
    if (s == -1.0f) sink[threadIdx.x] = s;        // sums of non-negative products: never true
}

}  // namespace

extern "C" {

// Reads `bytes` (a multiple of 16) from src once.  sink: at least 1 KiB of device memory (never written when
// the buffer holds one repeated 32-bit word and bytes is a multiple of 32).
int ceiling_stream_read(const void* src, int64_t bytes, void* sink, int groups, int nontemporal, void* stream) {
    if (!src || !sink || bytes < 16 || (bytes & 15) != 0 || groups < 1) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(nontemporal ? stream_read_kernel<true> : stream_read_kernel<false>, dim3(groups), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), bytes / 16, static_cast<uint32_t*>(sink));
    return (int)hipPeekAtLastError();
}

// Copies `bytes` (a multiple of 16) from src to dst: bytes read + bytes written of HBM traffic.
int ceiling_stream_copy(const void* src, void* dst, int64_t bytes, int groups, int nontemporal, void* stream) {
    if (!src || !dst || bytes < 16 || (bytes & 15) != 0 || groups < 1) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(nontemporal ? stream_copy_kernel<true> : stream_copy_kernel<false>, dim3(groups), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
    return (int)hipPeekAtLastError();
}

// groups work-groups of four wavefronts each issue iters * 8 MFMAs (16x16x32 fp16: 16384 flop each).
int ceiling_mfma_loop(int iters, int groups, void* sink, void* stream) {
    if (!sink || iters < 1 || groups < 1) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(groups), dim3(kThreads), 0, static_cast<hipStream_t>(stream), iters,
                       static_cast<float*>(sink));
    return (int)hipPeekAtLastError();
}

int64_t ceiling_mfma_flops(int iters, int groups) {
    return (int64_t)iters * groups * (kThreads / 64) * kChains * 16384;
}

}  // extern "C"
