// Linear layers and LayerNorm over packed rows (the "late blocks" of Section 4.3 item 4: after the
// pruning point the projections and the MLP run on the packed buffer, so their cost is linear in the
// number of kept tokens), for gfx950.
//
// linear_kernel:  y[m][n] = act( sum_k x[m][k] * w[n][k] + bias[n] ) (+ residual[m][n])
//   x [rows, K] activations, w [N, K] weights (one output feature per row, so both operands are
//   contiguous along k, which is how an MFMA lane wants them: 8 consecutive k per 16-byte read).
//   One work-group computes a 128-token x 128-feature tile; wavefront (wm, wn) owns a 64 x 64
//   quadrant as 4 x 4 MFMA 16x16x32 tiles with fp32 accumulators.  The product is formed
//   TRANSPOSED (features x tokens: W is the A operand, x the B operand), so that a lane ends up
//   with, for one token, 16 consecutive output features -- two 16-byte stores per token -- once the
//   A-operand rows are relabelled: MFMA row m' of feature tile j stands for feature
//   16*(m'/4) + 4*j + m'%4 of the quadrant.
//   Operand tiles (128 rows x 64 k = 128-byte rows) are brought into LDS by direct global->LDS
//   loads, row-major with the chunk swizzle c ^ ((row>>1)&3) that makes every 16-byte operand read
//   conflict-free, double-buffered: the loads of k-step t+1 are in flight while step t is computed.
//   Epilogue in registers: bias, optional GELU (erf form, Abramowitz-Stegun 7.1.26, |error| 1.5e-7,
//   written so the negative tail does not cancel), optional residual, conversion, store.
//
// layernorm_kernel: one wavefront per row, the row held in registers, two passes (mean, then the
//   biased variance of the centred values) in fp32.
//
// Rows: the caller passes a capacity and, optionally, a device pointer to the real row count (for
// example &cu_seqlens[B]); work-groups past it exit, so nothing is read back to the host.
#include "common.h"
#include "mfma_lds.h"

namespace ragged {
namespace {

constexpr int kTM = 128;                         // tokens per work-group tile
constexpr int kTN = 128;                         // output features per work-group tile
constexpr int kTK = 64;                          // contraction elements per stage: 128-byte LDS rows
constexpr int kStages = 2;
constexpr int kOperandBytes = 128 * kTK * 2;     // one operand tile: 16 KB

// GELU(t) = t * Phi(t) with Phi from erfc(z) ~ poly(u) * exp(-z^2), u = 1 / (1 + p z), z = |t| / sqrt 2.
__device__ __forceinline__ float gelu_erf(float t) {
    const float z = fabsf(t) * 0.70710678118654752f;
    const float u = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, z, 1.0f));
    float poly = __builtin_fmaf(u, 1.061405429f, -1.453152027f);
    poly = __builtin_fmaf(poly, u, 1.421413741f);
    poly = __builtin_fmaf(poly, u, -0.284496736f);
    poly = __builtin_fmaf(poly, u, 0.254829592f);
    const float half_erfc = 0.5f * poly * u * __builtin_amdgcn_exp2f(-z * z * 1.4426950408889634f);
    const float phi = t < 0.f ? half_erfc : 1.0f - half_erfc;     // Phi(t) = erfc(-t / sqrt 2) / 2
    return t * phi;
}

__device__ __forceinline__ void unpack16(F16, const uint4& a, const uint4& b, float (&v)[16]) {
    const f16x8 lo = as_vec8<f16x8>(a), hi = as_vec8<f16x8>(b);
#pragma unroll
    for (int e = 0; e < 8; ++e) { v[e] = (float)lo[e]; v[8 + e] = (float)hi[e]; }
}
__device__ __forceinline__ void unpack16(BF16, const uint4& a, const uint4& b, float (&v)[16]) {
    const bf16x8 lo = as_vec8<bf16x8>(a), hi = as_vec8<bf16x8>(b);
#pragma unroll
    for (int e = 0; e < 8; ++e) { v[e] = (float)lo[e]; v[8 + e] = (float)hi[e]; }
}
__device__ __forceinline__ void pack16(F16, const float (&v)[16], uint4& a, uint4& b) {
    f16x8 lo, hi;
#pragma unroll
    for (int e = 0; e < 8; ++e) { lo[e] = (_Float16)v[e]; hi[e] = (_Float16)v[8 + e]; }
    a = __builtin_bit_cast(uint4, lo);
    b = __builtin_bit_cast(uint4, hi);
}
__device__ __forceinline__ void pack16(BF16, const float (&v)[16], uint4& a, uint4& b) {
    bf16x8 lo, hi;
#pragma unroll
    for (int e = 0; e < 8; ++e) { lo[e] = (__bf16)v[e]; hi[e] = (__bf16)v[8 + e]; }
    a = __builtin_bit_cast(uint4, lo);
    b = __builtin_bit_cast(uint4, hi);
}

// Work-group index -> tile.  Consecutive work-groups are dealt round-robin to the 8 XCDs (each with
// its own L2); XCD x takes token tiles x, x+8, ... and walks all feature tiles of one token tile
// before the next, so an activation tile is fetched into one L2 once and the (small) weight matrix
// is what the XCDs share through the Infinity Cache.
template <typename In, int ACT, bool HAS_RES>
__global__ __launch_bounds__(kBlockThreads, 2)
void linear_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                   const uint16_t* __restrict__ bias, const uint16_t* __restrict__ res,
                   uint16_t* __restrict__ y, int rows_cap, const int32_t* __restrict__ rows_dev, int N, int K,
                   int n_tiles) {
    typedef typename In::vec8 vec8;
    __shared__ __attribute__((aligned(1024))) uint4 stage_lds[kStages * 2 * kOperandBytes / 16];   // [stage][x | w]

    const int xcd = blockIdx.x % kXcds;
    const int local = blockIdx.x / kXcds;
    const int m_tile = (local / n_tiles) * kXcds + xcd;
    const int n_tile = local % n_tiles;
    int rows = rows_cap;
    if (rows_dev) { const int r = *rows_dev; rows = r < rows ? r : rows; }
    const int m0 = m_tile * kTM;
    if (m0 >= rows) return;                                    // whole group
    const int n0 = n_tile * kTN;

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15;
    const int g = lane >> 4;
    const int wm = wave & 1, wn = wave >> 1;                   // this wavefront's 64-token / 64-feature quadrant

    // ---- global->LDS loads: instruction i (0..3) of this wavefront covers tile rows 32*wave + 8i + lane/8
    // of x and of w; the lane's LDS slot is position lane%8 of that row = chunk (lane%8) ^ ((row>>1)&3).
    const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) void*)stage_lds);
    const uint32_t row_bytes = (uint32_t)K * 2u;
    const uint32_t chunk = 16u * ((lane & 7) ^ ((lane >> 4) & 3));
    uint32_t voff_x[4], voff_w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 32 * wave + 8 * i + (lane >> 3);
        const int rx = m0 + r < rows ? r : rows - 1 - m0;     // past the last row: that row again (never stored)
        voff_x[i] = (uint32_t)rx * row_bytes + chunk;
        voff_w[i] = (uint32_t)r * row_bytes + chunk;
    }
    const uint16_t* x_base = x + (int64_t)m0 * K;              // wave-uniform; advances by kTK per step
    const uint16_t* w_base = w + (int64_t)n0 * K;
    auto issue = [&](int kt, int s) {
        const uint32_t dst = lds0 + s * 2 * kOperandBytes + wave * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dma16(dst + i * 1024, voff_x[i], x_base + kt * kTK);
            dma16(dst + i * 1024 + kOperandBytes, voff_w[i], w_base + kt * kTK);
        }
    };

    // ---- LDS read addresses inside a stage (x tile first, then w tile)
    //   x operand (B): row wm*64 + 16*mt + col, chunk 2g + ks
    const int x_row = wm * 64 + col;
    const uint32_t x_rel = x_row * 128 + 16 * ((2 * g) ^ ((x_row >> 1) & 3));
    //   w operand (A) of feature tile j: row wn*64 + 16*(col/4) + 4j + col%4, chunk 2g + ks
    uint32_t w_rel[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int w_row = wn * 64 + 16 * (col >> 2) + 4 * j + (col & 3);
        w_rel[j] = kOperandBytes + w_row * 128 + 16 * ((2 * g) ^ ((w_row >> 1) & 3));
    }

    f32x4 acc[4][4];                                           // [feature tile j][token tile mt]
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) acc[j][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int ksteps = K / kTK;
    issue(0, 0);
    for (int kt = 0; kt < ksteps; ++kt) {
        const int s = kt & 1;
        wait_vm<0>();                       // this wavefront's part of step kt has landed
        __syncthreads();                    // step kt visible; every wavefront is past step kt-1's reads
        if (kt + 1 < ksteps) issue(kt + 1, s ^ 1);
        const uint32_t base = lds0 + s * 2 * kOperandBytes;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            uint4 a[4], b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) a[j] = lds_read16(base + (w_rel[j & 1] ^ (16u * ks)) + (j >> 1) * 1024);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) b[mt] = lds_read16(base + (x_rel ^ (16u * ks)) + mt * 2048);
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
                    acc[j][mt] = In::mfma(as_vec8<vec8>(a[j]), as_vec8<vec8>(b[mt]), acc[j][mt]);
        }
    }

    // ---- epilogue: this lane owns, for token m0 + wm*64 + 16*mt + col, features n_base + 4j + r
    const int n_base = n0 + wn * 64 + 16 * g;
    float bias16[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) bias16[e] = 0.f;
    if (bias) {
        const uint4* bp = reinterpret_cast<const uint4*>(bias + n_base);
        unpack16(In{}, bp[0], bp[1], bias16);
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int m = m0 + wm * 64 + 16 * mt + col;
        if (m >= rows) continue;
        float v[16];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float t = acc[j][mt][r] + bias16[4 * j + r];
                if (ACT == 1) t = gelu_erf(t);
                v[4 * j + r] = t;
            }
        if (HAS_RES) {
            const uint4* rp = reinterpret_cast<const uint4*>(res + (int64_t)m * N + n_base);
            float r16[16];
            unpack16(In{}, rp[0], rp[1], r16);
#pragma unroll
            for (int e = 0; e < 16; ++e) v[e] += r16[e];
        }
        uint4 lo, hi;
        pack16(In{}, v, lo, hi);
        uint4* yp = reinterpret_cast<uint4*>(y + (int64_t)m * N + n_base);
        yp[0] = lo;
        yp[1] = hi;
    }
}

// Sum over the 64 lanes of a wavefront (fp32), result in every lane: DPP rotations inside each
// 16-lane row, then the lane-swap instructions across rows.
template <int kCtrl>
__device__ __forceinline__ float dpp_f32(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xf, 0xf, true));
}
__device__ __forceinline__ unsigned opaque_copy_u(unsigned x) {
    unsigned yv;
    asm volatile("v_mov_b32 %0, %1" : "=v"(yv) : "v"(x));
    return yv;
}
__device__ __forceinline__ float wave_sum_f32(float v) {
    v += dpp_f32<0x128>(v);                                    // row_ror:8
    v += dpp_f32<0x124>(v);                                    // row_ror:4
    v += dpp_f32<0x122>(v);                                    // row_ror:2
    v += dpp_f32<0x121>(v);                                    // row_ror:1
    const unsigned u = __builtin_bit_cast(unsigned, v);
    const auto a = __builtin_amdgcn_permlane16_swap(u, opaque_copy_u(u), false, false);
    const unsigned a0 = a[0], a1 = a[1];
    v = __builtin_bit_cast(float, a0) + __builtin_bit_cast(float, a1);
    const unsigned u2 = __builtin_bit_cast(unsigned, v);
    const auto b = __builtin_amdgcn_permlane32_swap(u2, opaque_copy_u(u2), false, false);
    const unsigned b0 = b[0], b1 = b[1];
    return __builtin_bit_cast(float, b0) + __builtin_bit_cast(float, b1);
}

constexpr int kLnChunks = 4;                                   // 16-byte chunks per lane: C <= 64 * 4 * 8 = 2048

template <typename In>
__global__ __launch_bounds__(kBlockThreads)
void layernorm_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ gamma,
                      const uint16_t* __restrict__ beta, uint16_t* __restrict__ y, int rows_cap,
                      const int32_t* __restrict__ rows_dev, int C, float eps) {
    int rows = rows_cap;
    if (rows_dev) { const int r = *rows_dev; rows = r < rows ? r : rows; }
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int row = blockIdx.x * (kBlockThreads / kWaveSize) + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int chunks = C / 8;
    const uint4* src = reinterpret_cast<const uint4*>(x + (int64_t)row * C);
    float v[kLnChunks][8];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kLnChunks; ++i) {
        const int c = lane + kWaveSize * i;
        if (c < chunks) {
            float t[16];
            const uint4 raw = src[c];
            unpack16(In{}, raw, raw, t);
#pragma unroll
            for (int e = 0; e < 8; ++e) { v[i][e] = t[e]; sum += t[e]; }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[i][e] = 0.f;
        }
    }
    const float mean = wave_sum_f32(sum) / (float)C;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < kLnChunks; ++i)
        if (lane + kWaveSize * i < chunks)
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float d = v[i][e] - mean; sq = __builtin_fmaf(d, d, sq); }
    const float rstd = 1.0f / sqrtf(wave_sum_f32(sq) / (float)C + eps);
    uint4* dst = reinterpret_cast<uint4*>(y + (int64_t)row * C);
#pragma unroll
    for (int i = 0; i < kLnChunks; ++i) {
        const int c = lane + kWaveSize * i;
        if (c < chunks) {
            float gm[16], bt[16], o16[16];
            const uint4 graw = reinterpret_cast<const uint4*>(gamma)[c];
            const uint4 braw = reinterpret_cast<const uint4*>(beta)[c];
            unpack16(In{}, graw, graw, gm);
            unpack16(In{}, braw, braw, bt);
#pragma unroll
            for (int e = 0; e < 8; ++e) o16[e] = o16[8 + e] = __builtin_fmaf((v[i][e] - mean) * rstd, gm[e], bt[e]);
            uint4 lo, hi;
            pack16(In{}, o16, lo, hi);
            dst[c] = lo;
        }
    }
}

template <typename In>
hipError_t launch_linear_typed(const void* x, const void* w, const void* bias, const void* res, void* y,
                               int rows_cap, const int32_t* rows_dev, int N, int K, int act, hipStream_t stream) {
    const int n_tiles = N / kTN;
    const int m_tiles = (rows_cap + kTM - 1) / kTM;
    const int m_tiles8 = (m_tiles + kXcds - 1) / kXcds * kXcds;
    const dim3 grid(m_tiles8 * n_tiles), block(kBlockThreads);
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    const uint16_t* wp = static_cast<const uint16_t*>(w);
    const uint16_t* bp = static_cast<const uint16_t*>(bias);
    const uint16_t* rp = static_cast<const uint16_t*>(res);
    uint16_t* yp = static_cast<uint16_t*>(y);
    if (act == 1 && res)
        hipLaunchKernelGGL((linear_kernel<In, 1, true>), grid, block, 0, stream, xp, wp, bp, rp, yp, rows_cap, rows_dev, N, K, n_tiles);
    else if (act == 1)
        hipLaunchKernelGGL((linear_kernel<In, 1, false>), grid, block, 0, stream, xp, wp, bp, rp, yp, rows_cap, rows_dev, N, K, n_tiles);
    else if (res)
        hipLaunchKernelGGL((linear_kernel<In, 0, true>), grid, block, 0, stream, xp, wp, bp, rp, yp, rows_cap, rows_dev, N, K, n_tiles);
    else
        hipLaunchKernelGGL((linear_kernel<In, 0, false>), grid, block, 0, stream, xp, wp, bp, rp, yp, rows_cap, rows_dev, N, K, n_tiles);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear(const void* x, const void* w, const void* bias, const void* res, void* y, int rows_cap,
                         const int32_t* rows_dev, int N, int K, int act, ragged_dtype dt, hipStream_t stream) {
    if (dt == RAGGED_F16) return launch_linear_typed<F16>(x, w, bias, res, y, rows_cap, rows_dev, N, K, act, stream);
    return launch_linear_typed<BF16>(x, w, bias, res, y, rows_cap, rows_dev, N, K, act, stream);
}

int layernorm_max_width() { return kWaveSize * kLnChunks * 8; }

hipError_t launch_layernorm(const void* x, const void* gamma, const void* beta, void* y, int rows_cap,
                            const int32_t* rows_dev, int C, float eps, ragged_dtype dt, hipStream_t stream) {
    const int per = kBlockThreads / kWaveSize;
    const dim3 grid((rows_cap + per - 1) / per), block(kBlockThreads);
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    const uint16_t* gp = static_cast<const uint16_t*>(gamma);
    const uint16_t* bp = static_cast<const uint16_t*>(beta);
    uint16_t* yp = static_cast<uint16_t*>(y);
    if (dt == RAGGED_F16)
        hipLaunchKernelGGL((layernorm_kernel<F16>), grid, block, 0, stream, xp, gp, bp, yp, rows_cap, rows_dev, C, eps);
    else
        hipLaunchKernelGGL((layernorm_kernel<BF16>), grid, block, 0, stream, xp, gp, bp, yp, rows_cap, rows_dev, C, eps);
    return hipGetLastError();
}

}  // namespace ragged
