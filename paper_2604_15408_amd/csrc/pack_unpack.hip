// Pack (keep mask -> cu_seqlens + gather indices + coalesced row gather) and unpack (row scatter)
// for gfx950.  Section 4.1 of the paper does the index phase with several framework ops and a host
// read of the kept count, then a copy kernel; here each stage is a single launch with no host
// read: every work-group recounts the (tiny) mask prefix it needs from L2, so no grid-wide scan or
// second kernel is required.
#include "common.h"

namespace ragged {
namespace {

// Number of nonzero bytes in a 32-bit word.  (b & 0x7f) + 0x7f carries into bit 7 of its own byte
// exactly when the low 7 bits are nonzero, and never into the next byte.
__device__ __forceinline__ int nonzero_bytes(uint32_t w) {
    const uint32_t t = ((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w;
    return __popc(t & 0x80808080u);
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWaveSize);
    return v;
}

// Work-group-wide count of nonzero bytes in base[0, len).  Every thread of the 256-thread group
// must call it; every thread receives the total.  The bulk is read as aligned 16-byte words; the
// unaligned head and the tail go byte by byte, so no byte outside [0, len) is ever touched.
__device__ int block_count_nonzero(const uint8_t* __restrict__ base, int len, int* lds4) {
    const int tid = threadIdx.x;
    int count = 0;
    const int mis = (int)((uintptr_t)base & 15u);
    int head = mis ? 16 - mis : 0;
    if (head > len) head = len;
    if (tid < head) count += base[tid] != 0;
    const int body = (len - head) >> 4;                       // whole 16-byte words
    const uint4* words = reinterpret_cast<const uint4*>(base + head);
    for (int w = tid; w < body; w += kBlockThreads) {
        const uint4 v = words[w];
        count += nonzero_bytes(v.x) + nonzero_bytes(v.y) + nonzero_bytes(v.z) + nonzero_bytes(v.w);
    }
    const int tail0 = head + (body << 4);
    if (tail0 + tid < len) count += base[tail0 + tid] != 0;   // fewer than 16 tail bytes
    count = wave_sum(count);
    __syncthreads();                                          // lds4 may still be read by a prior call
    if ((tid & (kWaveSize - 1)) == 0) lds4[tid >> 6] = count;
    __syncthreads();
    return lds4[0] + lds4[1] + lds4[2] + lds4[3];
}

// Copy one row of `units` 16-byte words with the 64 lanes of a wavefront (coalesced both ways).
__device__ __forceinline__ void wave_copy_row(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                              int units, int lane) {
    for (int u = lane; u < units; u += kWaveSize) dst[u] = src[u];
}

// ------------------------------------------------------------------------------------------------
// pack: one work-group per (image i, chunk of `chunk` <= 64 consecutive tokens).
//   P      = kept tokens before this chunk in the whole batch (flat mask prefix)  -> destination base
//   ballot = keep bits of the chunk; the k-th set bit goes to packed row P + k
// The last chunk of image i also writes cu_seqlens[i+1]; group 0 writes cu_seqlens[0].
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlockThreads)
void pack_kernel(const uint4* __restrict__ x, const uint8_t* __restrict__ keep, int N, int units,
                 uint4* __restrict__ packed, int64_t cap_rows, int32_t* __restrict__ cu_seqlens,
                 int32_t* __restrict__ gather_idx, int chunk, int chunks_per_image) {
    __shared__ int lds4[4];
    const int i = blockIdx.x / chunks_per_image;
    const int c = blockIdx.x - i * chunks_per_image;
    const int t0 = c * chunk;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int row0 = i * N + t0;                               // flat index of the chunk's first token

    const int P = block_count_nonzero(keep, row0, lds4);

    // Every wavefront reads the chunk's <= 64 mask bytes itself: cheaper than a broadcast via LDS.
    const bool mine = lane < chunk && t0 + lane < N && keep[row0 + lane] != 0;
    const uint64_t bits = __ballot(mine);
    const int in_chunk = __popcll(bits);

    if (wave == 0) {
        if (mine) {
            const int64_t dst = (int64_t)P + __popcll(bits & ((1ull << lane) - 1ull));
            if (dst < cap_rows) gather_idx[dst] = row0 + lane;
        }
        if (lane == 0) {
            if (blockIdx.x == 0) cu_seqlens[0] = 0;
            if (c == chunks_per_image - 1) cu_seqlens[i + 1] = P + in_chunk;
        }
    }

    // Rows of the chunk are dealt to the four wavefronts round-robin.
    uint64_t rest = bits;
    for (int k = 0; rest != 0; ++k) {
        const int t = __builtin_ctzll(rest);
        rest &= rest - 1;
        if ((k & 3) != wave) continue;
        const int64_t dst = (int64_t)P + k;
        if (dst >= cap_rows) break;
        wave_copy_row(x + (int64_t)(row0 + t) * units, packed + dst * units, units, lane);
    }
}

// ------------------------------------------------------------------------------------------------
// unpack, fill_mode 0: one work-group per 8 packed rows; out[gather_idx[r]] = src[r].
// Work is proportional to T; groups beyond T (read from cu_seqlens[B]) exit at once.
// ------------------------------------------------------------------------------------------------
constexpr int kUnpackRows = 8;

__global__ __launch_bounds__(kBlockThreads)
void unpack_scatter_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ cu_seqlens,
                           const int32_t* __restrict__ gather_idx, int B, int units,
                           uint4* __restrict__ out) {
    const int T = cu_seqlens[B];
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int r0 = blockIdx.x * kUnpackRows;
    if (r0 >= T) return;
#pragma unroll
    for (int k = 0; k < kUnpackRows / 4; ++k) {
        const int r = r0 + wave + 4 * k;
        if (r < T) {
            const int64_t dst = gather_idx[r];
            wave_copy_row(src + (int64_t)r * units, out + dst * units, units, lane);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// unpack, fill_mode 1: one work-group per (image, chunk) as in pack.  Kept tokens receive their
// packed row (cu_seqlens[i] + rank inside the image); dropped tokens are written with +0 words.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlockThreads)
void unpack_fill_kernel(const uint4* __restrict__ src, const uint8_t* __restrict__ keep,
                        const int32_t* __restrict__ cu_seqlens, int N, int units,
                        uint4* __restrict__ out, int chunk, int chunks_per_image) {
    __shared__ int lds4[4];
    const int i = blockIdx.x / chunks_per_image;
    const int c = blockIdx.x - i * chunks_per_image;
    const int t0 = c * chunk;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = threadIdx.x >> 6;
    const int row0 = i * N + t0;

    const int rank0 = block_count_nonzero(keep + (int64_t)i * N, t0, lds4);
    const int64_t base = (int64_t)cu_seqlens[i] + rank0;

    const bool valid = lane < chunk && t0 + lane < N;
    const bool mine = valid && keep[row0 + lane] != 0;
    const uint64_t bits = __ballot(mine);
    const int live = __popcll(__ballot(valid));                // tokens of this chunk inside the image

    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    for (int t = wave; t < live; t += 4) {
        uint4* dst = out + (int64_t)(row0 + t) * units;
        if ((bits >> t) & 1ull) {
            const int k = __popcll(bits & ((1ull << t) - 1ull));
            wave_copy_row(src + (base + k) * units, dst, units, lane);
        } else {
            for (int u = lane; u < units; u += kWaveSize) dst[u] = zero;
        }
    }
}

__global__ void noop_kernel() {}

}  // namespace

hipError_t launch_pack(const void* x, const uint8_t* keep, int B, int N, int C, void* packed,
                       int64_t cap_rows, int32_t* cu_seqlens, int32_t* gather_idx,
                       hipStream_t stream) {
    const int chunk = pick_chunk(B, N);
    const int cpi = (N + chunk - 1) / chunk;
    hipLaunchKernelGGL(pack_kernel, dim3(B * cpi), dim3(kBlockThreads), 0, stream,
                       static_cast<const uint4*>(x), keep, N, C / 8, static_cast<uint4*>(packed),
                       cap_rows, cu_seqlens, gather_idx, chunk, cpi);
    return hipGetLastError();
}

hipError_t launch_unpack(const void* src, const uint8_t* keep, const int32_t* cu_seqlens,
                         const int32_t* gather_idx, int B, int N, int C, void* out, int fill_mode,
                         hipStream_t stream) {
    if (fill_mode == 0) {
        const int64_t rows = (int64_t)B * N;
        const int grid = (int)((rows + kUnpackRows - 1) / kUnpackRows);
        hipLaunchKernelGGL(unpack_scatter_kernel, dim3(grid), dim3(kBlockThreads), 0, stream,
                           static_cast<const uint4*>(src), cu_seqlens, gather_idx, B, C / 8,
                           static_cast<uint4*>(out));
    } else {
        const int chunk = pick_chunk(B, N);
        const int cpi = (N + chunk - 1) / chunk;
        hipLaunchKernelGGL(unpack_fill_kernel, dim3(B * cpi), dim3(kBlockThreads), 0, stream,
                           static_cast<const uint4*>(src), keep, cu_seqlens, N, C / 8,
                           static_cast<uint4*>(out), chunk, cpi);
    }
    return hipGetLastError();
}

hipError_t launch_noop(int grid, hipStream_t stream) {
    hipLaunchKernelGGL(noop_kernel, dim3(grid), dim3(kBlockThreads), 0, stream);
    return hipGetLastError();
}

}  // namespace ragged
