// Pack (keep mask -> cu_seqlens + gather indices + coalesced row gather) and unpack (row scatter)
// for gfx950.  Section 4.1 of the paper does the index phase with several framework ops and a host
// read of the kept count, then a copy kernel; here each stage is a single launch with no host
// read: every work-group recounts the (tiny) mask prefix it needs from L2, so no grid-wide scan or
// second kernel is required.
#include "common.h"
#include "mask_prefix.h"

namespace ragged {
namespace {

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
constexpr int kMaxEarly = 4;    // rows a wavefront may hold in registers (EARLY needs chunk <= 16)

template <bool EARLY>
__global__ __launch_bounds__(kBlockThreads)
void pack_kernel(const uint4* __restrict__ x, const uint8_t* __restrict__ keep, int N, int units,
                 uint4* __restrict__ packed, int64_t cap_rows, int32_t* __restrict__ cu_seqlens,
                 int32_t* __restrict__ gather_idx, int chunk, int chunks_per_image, uint32_t cpi_magic) {
    __shared__ int lds4[4];
    uint32_t i_u, c_u;
    divmod(blockIdx.x, (uint32_t)chunks_per_image, cpi_magic, i_u, c_u);
    const int i = (int)i_u, c = (int)c_u;
    const int t0 = c * chunk;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // in a scalar register: the bit walks below are scalar code
    const int row0 = i * N + t0;                               // flat index of the chunk's first token

    // Three dependent fabric round trips (mask prefix -> chunk mask -> rows) are folded into two:
    // the chunk's own mask bytes and the prefix words are requested together, and the source rows
    // -- which depend only on the chunk's bits, not on the destination -- are requested before the
    // prefix count is reduced.  Every wavefront reads the chunk's <= 64 mask bytes itself (a clamped,
    // unconditional load: see load_byte_clamped).
    const int in_image = N - t0 < chunk ? N - t0 : chunk;      // tokens of this chunk: >= 1
    const bool in_chunk = lane < in_image;
    const uint8_t my_keep = load_byte_clamped(keep + row0, lane, in_image);
    const PrefixLoads prefix = prefix_issue(keep, row0);

    const bool mine = in_chunk && my_keep != 0;
    const uint64_t bits = __ballot(mine);
    const int in_chunk_count = __popcll(bits);

    // Rows of the chunk are dealt to the four wavefronts round-robin: set bit k -> wavefront k%4.
    // EARLY (chunk <= 16 and rows of at most 128 16-byte words): a wavefront has at most four rows
    // of two words per lane and requests them now, into registers.
    // (the walks over the set bits are straight-line scalar code: a taken branch costs a lone wavefront as much as half a dozen
    // instructions, so no loop per dropped bit)
    uint4 held[kMaxEarly][2];
    if (EARLY) {
#pragma unroll
        for (int r = 0; r < kMaxEarly; ++r) {
            held[r][0] = make_uint4(0u, 0u, 0u, 0u);
            held[r][1] = make_uint4(0u, 0u, 0u, 0u);
        }
        if (wave < in_chunk_count) {                           // this wavefront has a row: set bits wave, wave + 4, ...
            uint32_t m = (uint32_t)bits;                       // chunk <= 16 here: the bits fit
#pragma unroll
            for (int z = 0; z < 3; ++z) m = z < wave ? (m & (m - 1)) : m;   // drop the `wave` lowest set bits
#pragma unroll
            for (int r = 0; r < kMaxEarly; ++r) {
                const uint4* src = x + (int64_t)(row0 + __builtin_ctz(m)) * units;
                if (lane < units) held[r][0] = src[lane];
                if (lane + kWaveSize < units) held[r][1] = src[lane + kWaveSize];
                if (wave + 4 * (r + 1) >= in_chunk_count) break;
#pragma unroll
                for (int z = 0; z < 4; ++z) m &= m - 1;        // on to set bit wave + 4(r+1)
            }
        }
    }

    const int P = prefix_finish(keep, prefix, lds4);           // kept tokens before this chunk in the batch

    if (wave == 0) {
        if (mine) {
            const int64_t dst = (int64_t)P + __popcll(bits & ((1ull << lane) - 1ull));
            if (dst < cap_rows) gather_idx[dst] = row0 + lane;
        }
        if (lane == 0) {
            if (blockIdx.x == 0) cu_seqlens[0] = 0;
            if (c == chunks_per_image - 1) cu_seqlens[i + 1] = P + in_chunk_count;
        }
    }

    if (EARLY) {
#pragma unroll
        for (int r = 0; r < kMaxEarly; ++r) {
            const int64_t dst = (int64_t)P + wave + 4 * r;     // r-th row of this wavefront is set bit wave + 4r
            if (wave + 4 * r < in_chunk_count && dst < cap_rows) {
                uint4* out = packed + dst * units;
                if (lane < units) out[lane] = held[r][0];
                if (lane + kWaveSize < units) out[lane + kWaveSize] = held[r][1];
            }
        }
    } else {
        uint64_t rest = bits;
#pragma unroll
        for (int z = 0; z < 3; ++z) rest = z < wave ? (rest & (rest - 1)) : rest;
        for (int k = wave; rest != 0; k += 4) {                // one iteration per row of this wavefront
            const int t = __builtin_ctzll(rest);
            const int64_t dst = (int64_t)P + k;
            if (dst >= cap_rows) break;
            wave_copy_row(x + (int64_t)(row0 + t) * units, packed + dst * units, units, lane);
#pragma unroll
            for (int z = 0; z < 4; ++z) rest &= rest - 1;
        }
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
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
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
                        uint4* __restrict__ out, int chunk, int chunks_per_image, uint32_t cpi_magic) {
    __shared__ int lds4[4];
    uint32_t i_u, c_u;
    divmod(blockIdx.x, (uint32_t)chunks_per_image, cpi_magic, i_u, c_u);
    const int i = (int)i_u, c = (int)c_u;
    const int t0 = c * chunk;
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row0 = i * N + t0;

    // one memory round trip for everything the addresses depend on: the chunk's own mask bytes, the mask
    // bytes in front of it and the image's first packed row are requested together
    const uint8_t* image_mask = keep + (int64_t)i * N;
    const int live = N - t0 < chunk ? N - t0 : chunk;          // tokens of this chunk inside the image: >= 1
    const uint8_t my_keep = load_byte_clamped(keep + row0, lane, live);
    // (through a pointer held in vector registers, so that it is a vector load issued here with the other
    // requests: a scalar load of it gets scheduled behind the waits of the prefix count)
    typedef const __attribute__((address_space(1))) int32_t* global_i32_ptr;
    global_i32_ptr first_row_ptr = (global_i32_ptr)(cu_seqlens + i);
    asm volatile("" : "+v"(first_row_ptr));
    const int first_row = *first_row_ptr;
    const PrefixLoads prefix = prefix_issue(image_mask, t0);
    const int rank0 = prefix_finish(image_mask, prefix, lds4);
    const int64_t base = (int64_t)first_row + rank0;

    const bool mine = lane < live && my_keep != 0;
    const uint64_t bits = __ballot(mine);

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

// ------------------------------------------------------------------------------------------------
// re-pack: a second keep decision on an already packed buffer.  One work-group per chunk of <= 64
// consecutive packed rows; the structure is that of pack with the flat row index in place of
// (image, token).  cu_out[i] = kept rows before row cu_in[i]: written by the group whose chunk
// contains that row index (the group starting at or just below T_in also runs, for boundaries that
// equal T_in).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlockThreads)
void repack_kernel(const uint4* __restrict__ packed_in, const uint8_t* __restrict__ keep_rows,
                   const int32_t* __restrict__ cu_in, int B, int64_t cap_in, int units,
                   uint4* __restrict__ packed_out, int64_t cap_out, int32_t* __restrict__ cu_out,
                   int32_t* __restrict__ gather_out, int chunk) {
    __shared__ int lds4[4];
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t r0 = (int64_t)blockIdx.x * chunk;            // <= cap_in by the grid size
    const int t_in = cu_in[B];
    // requested before t_in is known: both ranges lie inside the cap_in bytes of keep_rows
    const bool in_cap = lane < chunk && r0 + lane < cap_in;
    const uint8_t my_keep = load_byte_clamped(keep_rows, (int)r0 + lane, (int)cap_in);    // looked at if in_cap
    const PrefixLoads prefix = prefix_issue(keep_rows, (int)r0);
    if (r0 > t_in) return;                                     // whole group; rows >= t_in do not exist

    const bool mine = in_cap && my_keep != 0 && r0 + lane < t_in;
    const uint64_t bits = __ballot(mine);
    const int P = prefix_finish(keep_rows, prefix, lds4);      // kept rows before this chunk

    if (wave == 0 && mine) {
        const int64_t dst = (int64_t)P + __popcll(bits & ((1ull << lane) - 1ull));
        if (dst < cap_out) gather_out[dst] = (int32_t)(r0 + lane);
    }
    for (int i = threadIdx.x; i <= B; i += kBlockThreads) {
        const int64_t c = cu_in[i];
        if (c >= r0 && c < r0 + chunk) cu_out[i] = P + __popcll(bits & ((1ull << (int)(c - r0)) - 1ull));
    }
    uint64_t rest = bits;
#pragma unroll
    for (int z = 0; z < 3; ++z) rest = z < wave ? (rest & (rest - 1)) : rest;   // drop the `wave` lowest set bits
    for (int k = wave; rest != 0; k += 4) {                    // one iteration per row of this wavefront
        const int t = __builtin_ctzll(rest);
        const int64_t dst = (int64_t)P + k;
        if (dst >= cap_out) break;
        wave_copy_row(packed_in + (r0 + t) * units, packed_out + dst * units, units, lane);
#pragma unroll
        for (int z = 0; z < 4; ++z) rest &= rest - 1;
    }
}

// ------------------------------------------------------------------------------------------------
// CLS extraction: one wavefront per image copies the image's first packed row (zeros if it has none).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlockThreads)
void cls_extract_kernel(const uint4* __restrict__ packed, const int32_t* __restrict__ cu_seqlens, int B,
                        int units, uint4* __restrict__ out) {
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int i = blockIdx.x * (kBlockThreads / kWaveSize) + (threadIdx.x >> 6);
    if (i >= B) return;
    const int s = cu_seqlens[i];
    const bool has = cu_seqlens[i + 1] > s;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    for (int u = lane; u < units; u += kWaveSize)
        out[(int64_t)i * units + u] = has ? packed[(int64_t)s * units + u] : zero;
}

__global__ void noop_kernel() {}

}  // namespace

hipError_t launch_pack(const void* x, const uint8_t* keep, int B, int N, int C, void* packed,
                       int64_t cap_rows, int32_t* cu_seqlens, int32_t* gather_idx,
                       hipStream_t stream) {
    const int chunk = pick_chunk(B, N, kPackMaxGroups);
    const int cpi = (N + chunk - 1) / chunk;
    // the early-load variant keeps the first 16 KB of mask prefix in registers; beyond that the
    // remaining prefix loads would queue behind the row loads, so larger masks take the plain order
    const bool early = chunk <= 4 * kMaxEarly && C / 8 <= 2 * kWaveSize && (int64_t)B * N <= 16384;
    const hipError_t err = launch_kernel(early ? pack_kernel<true> : pack_kernel<false>, dim3(B * cpi),
                       dim3(kBlockThreads), stream, static_cast<const uint4*>(x), keep, N, C / 8,
                       static_cast<uint4*>(packed), cap_rows, cu_seqlens, gather_idx, chunk, cpi,
                       div_magic((uint32_t)cpi));
    return err;
}

hipError_t launch_unpack(const void* src, const uint8_t* keep, const int32_t* cu_seqlens,
                         const int32_t* gather_idx, int B, int N, int C, void* out, int fill_mode,
                         hipStream_t stream) {
    hipError_t err;
    if (fill_mode == 0) {
        const int64_t rows = (int64_t)B * N;
        const int grid = (int)((rows + kUnpackRows - 1) / kUnpackRows);
        err = launch_kernel(unpack_scatter_kernel, dim3(grid), dim3(kBlockThreads), stream,
                           static_cast<const uint4*>(src), cu_seqlens, gather_idx, B, C / 8,
                           static_cast<uint4*>(out));
    } else {
        const int chunk = pick_chunk(B, N, kUnpackFillMaxGroups);
        const int cpi = (N + chunk - 1) / chunk;
        err = launch_kernel(unpack_fill_kernel, dim3(B * cpi), dim3(kBlockThreads), stream,
                           static_cast<const uint4*>(src), keep, cu_seqlens, N, C / 8,
                           static_cast<uint4*>(out), chunk, cpi, div_magic((uint32_t)cpi));
    }
    return err;
}

hipError_t launch_repack(const void* packed_in, const uint8_t* keep_rows, const int32_t* cu_in, int B,
                         int64_t cap_in, int C, void* packed_out, int64_t cap_out, int32_t* cu_out,
                         int32_t* gather_out, hipStream_t stream) {
    int chunk = 8;
    while (chunk < 64 && cap_in / chunk > 4096) chunk *= 2;
    const int grid = (int)(cap_in / chunk) + 1;                // covers every chunk start <= cap_in
    const hipError_t err = launch_kernel(repack_kernel, dim3(grid), dim3(kBlockThreads), stream,
                       static_cast<const uint4*>(packed_in), keep_rows, cu_in, B, cap_in, C / 8,
                       static_cast<uint4*>(packed_out), cap_out, cu_out, gather_out, chunk);
    return err;
}

hipError_t launch_cls_extract(const void* packed, const int32_t* cu_seqlens, int B, int C, void* out,
                              hipStream_t stream) {
    const int per = kBlockThreads / kWaveSize;
    const hipError_t err = launch_kernel(cls_extract_kernel, dim3((B + per - 1) / per), dim3(kBlockThreads), stream,
                       static_cast<const uint4*>(packed), cu_seqlens, B, C / 8, static_cast<uint4*>(out));
    return err;
}

hipError_t launch_noop(int grid, hipStream_t stream) {
    const hipError_t err = launch_kernel(noop_kernel, dim3(grid), dim3(kBlockThreads), stream);
    return err;
}

}  // namespace ragged
