// Linear layers and LayerNorm over packed rows (the "late blocks" of Section 4.3 item 4: after the
// pruning point the projections and the MLP run on the packed buffer, so their cost is linear in the
// number of kept tokens), for gfx950.
//
// linear_kernel:  y[m][n] = act( sum_k x[m][k] * w[n][k] + bias[n] ) (+ residual[m][n])
//   x [rows, K] activations, w [N, K] weights (one output feature per row, so both operands are
//   contiguous along k, which is how an MFMA lane wants them: 8 consecutive k per 16-byte read).
//   One work-group computes a tile of tokens x features (256 x 256 with eight wavefronts, 128 x 128
//   with four, or 64 x 64 with one wavefront per half of the k-loop); a wavefront owns 64 features
//   x 64 or 128 tokens as 4 x 4 or 4 x 8 MFMA 16x16x32 tiles with fp32 accumulators.  The product is formed
//   TRANSPOSED (features x tokens: W is the A operand, x the B operand), so that a lane ends up
//   with, for one token, 16 consecutive output features -- two 16-byte stores per token -- once the
//   A-operand rows are relabelled: MFMA row m' of feature tile j stands for feature
//   16*(m'/4) + 4*j + m'%4 of the quadrant.
//   Operand tiles (rows x 64 k = 128-byte rows) are brought into LDS by direct global->LDS
//   loads, row-major with the chunk swizzle c ^ ((row>>1)&3) that makes every 16-byte operand read
//   conflict-free, in a ring of two stages; a stage is refilled as soon as every wavefront holds
//   it in registers.
//   Epilogue in registers: bias, optional GELU (erf form, Abramowitz-Stegun 7.1.26, |error| 1.5e-7,
//   written so the negative tail does not cancel), optional residual, conversion, store.
//
// layernorm_kernel: one wavefront per row, the row held in registers, two passes (mean, then the
//   biased variance of the centred values) in fp32.
//
// Rows: the caller passes a capacity and, optionally, a device pointer to the real row count (for
// example &cu_seqlens[B]); work-groups past it exit, so nothing is read back to the host.
#include <type_traits>
#include "common.h"
#include "mfma_lds.h"

namespace ragged {
namespace {

constexpr int kTK = 64;                          // contraction elements per stage: 128-byte LDS rows
constexpr int kBigTileMinGroups = 400;           // use 256 x 256 tiles from this many of them on
constexpr int kSplitMaxGroups = 128;             // 64 x 64 tiles with the k-loop split in the group up to this many 128 x 128 tiles

// GELU(t) = t * Phi(t) = max(t, 0) - |t| * erfc(|t| / sqrt 2) / 2, with erfc(z) ~ poly(u) * exp(-z^2),
// u = 1 / (1 + p z) (Abramowitz-Stegun 7.1.26).  In this form nothing cancels in the negative tail, the
// halving sits in the coefficients and |t| is an operand modifier: 11 VALU + 2 transcendental ops.
__device__ __forceinline__ float gelu_erf(float t) {
    const float at = fabsf(t);
    const float u = __builtin_amdgcn_rcpf(__builtin_fmaf(at, 0.3275911f * 0.70710678118654752f, 1.0f));
    float poly = __builtin_fmaf(u, 0.5f * 1.061405429f, 0.5f * -1.453152027f);
    poly = __builtin_fmaf(poly, u, 0.5f * 1.421413741f);
    poly = __builtin_fmaf(poly, u, 0.5f * -0.284496736f);
    poly = __builtin_fmaf(poly, u, 0.5f * 0.254829592f);
    const float s = at * 0.84932180028801904f;                    // sqrt(log2(e) / 2): exp(-t^2 / 2) = 2^(-s^2)
    const float half_erfc = poly * u * __builtin_amdgcn_exp2f(-s * s);
    return __builtin_fmaf(-at, half_erfc, fmaxf(t, 0.f));
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
//
// Shape of a work-group: WNW x WMW wavefronts, each owning 64 features x 16*MT tokens, i.e. a tile of
// TN = 64*WNW features x TM = 16*MT*WMW tokens.  The L2 -> LDS traffic per flop falls with the tile
// size (a 128 x 128 tile needs 1/64 byte per flop, which at MFMA rate is more than the L2s deliver;
// 256 x 256 halves it), so large problems use 4 x 2 wavefronts of 64 x 128, mid-sized ones 2 x 2
// wavefronts of 64 x 64 and small ones, where filling the 256 CUs matters most, single wavefronts.
//
// KSPLIT > 1 (small grids only): the work-group has KSPLIT sets of WNW x WMW wavefronts; set g runs the
// same loop over the g-th part of the k-steps with a stage ring of its own, so the serial chain of
// k-steps -- what a grid of at most one work-group per CU waits for -- is shorter and more loads are in
// flight per CU.  At the end the other sets hand their accumulators to set 0 through LDS (summed in set
// order: the result does not depend on timing) and set 0 runs the epilogue.
//
// The second launch bound asks for two wavefronts per SIMD, i.e. at most 256 registers; together with the
// compiler option that keeps MFMA results in plain VGPRs (see the build script) it stops the compiler
// from parking accumulators in AGPRs and copying them around every MFMA, which it does as soon as
// the LDS use of a shape limits a CU to one work-group.
template <typename In, int ACT, bool HAS_RES, int WNW, int WMW, int MT, int STAGES, int KSPLIT>
__global__ __launch_bounds__(kWaveSize * WNW * WMW * KSPLIT, (WNW * WMW * KSPLIT >= 8) ? 1 : 8 / (WNW * WMW * KSPLIT))
void linear_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                   const uint16_t* __restrict__ bias, const uint16_t* res,   // res may alias y: no restrict
                   uint16_t* y, int rows_cap, const int32_t* __restrict__ rows_dev, int N, int K,
                   int n_tiles) {
    typedef typename In::vec8 vec8;
    constexpr int WAVES = WNW * WMW;
    constexpr int TN = 64 * WNW, TM = 16 * MT * WMW;
    constexpr int kXBytes = TM * kTK * 2, kWBytes = TN * kTK * 2;       // operand tiles of one stage
    constexpr int kStageBytes = kXBytes + kWBytes;
    __shared__ __attribute__((aligned(1024))) uint4 stage_lds[KSPLIT * STAGES * kStageBytes / 16];   // [set][stage][x | w]
    static_assert(KSPLIT == 1 || STAGES * kStageBytes >= 4 * MT * 16 * kWaveSize * WAVES, "the hand-over needs room in a ring");

    const int xcd = blockIdx.x % kXcds;
    const int local = blockIdx.x / kXcds;
    const int m_tile = (local / n_tiles) * kXcds + xcd;
    const int n_tile = local % n_tiles;
    int rows = rows_cap;
    if (rows_dev) { const int r = *rows_dev; rows = r < rows ? r : rows; }
    const int m0 = m_tile * TM;
    if (m0 >= rows) return;                                    // whole group
    const int n0 = n_tile * TN;

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave_wg = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kset = wave_wg / WAVES;                          // which half of the k-steps (0 if KSPLIT == 1)
    const int wave = wave_wg - kset * WAVES;                   // wavefront inside its set
    const int col = lane & 15;
    const int g = lane >> 4;
    const int wn = wave % WNW, wm = wave / WNW;                // this wavefront's feature / token block

    // ---- global->LDS loads: instruction i of this wavefront covers tile rows 8*(kI*wave + i) + lane/8
    // of x (kXI instructions) and of w (kWI); the lane's LDS slot is position lane%8 of that row =
    // chunk (lane%8) ^ ((row>>1)&3).
    constexpr int kXI = TM / 8 / WAVES, kWI = TN / 8 / WAVES;  // load instructions per wavefront per stage
    static_assert(TM % (8 * WAVES) == 0 && TN % (8 * WAVES) == 0, "tile rows must split over the wavefronts");
    const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) void*)stage_lds) +
                          kset * STAGES * kStageBytes;         // this set's ring
    const uint32_t row_bytes = (uint32_t)K * 2u;
    const uint32_t chunk = 16u * ((lane & 7) ^ ((lane >> 4) & 3));
    uint32_t voff_x[kXI], voff_w[kWI];
#pragma unroll
    for (int i = 0; i < kXI; ++i) {
        const int r = 8 * (kXI * wave + i) + (lane >> 3);
        const int rx = m0 + r < rows ? r : rows - 1 - m0;     // past the last row: that row again (never stored)
        voff_x[i] = (uint32_t)rx * row_bytes + chunk;
    }
#pragma unroll
    for (int i = 0; i < kWI; ++i) voff_w[i] = (uint32_t)(8 * (kWI * wave + i) + (lane >> 3)) * row_bytes + chunk;
    const int ksteps = K / kTK / KSPLIT;                       // k-steps of this set (the host makes it divide)
    const uint16_t* x_base = x + (int64_t)m0 * K + kset * ksteps * kTK;   // wave-uniform; advances by kTK per step
    const uint16_t* w_base = w + (int64_t)n0 * K + kset * ksteps * kTK;
    auto issue = [&](int kt, int s) {
        const uint32_t dst = lds0 + s * kStageBytes;
#pragma unroll
        for (int i = 0; i < kXI; ++i) dma16(dst + (kXI * wave + i) * 1024, voff_x[i], x_base + kt * kTK);
#pragma unroll
        for (int i = 0; i < kWI; ++i) dma16(dst + kXBytes + (kWI * wave + i) * 1024, voff_w[i], w_base + kt * kTK);
    };

    // ---- LDS read addresses inside a stage (x tile first, then w tile)
    //   x operand (B): row wm*16*MT + 16*mt + col, chunk 2g + ks
    const int x_row = wm * 16 * MT + col;
    const uint32_t x_rel = x_row * 128 + 16 * ((2 * g) ^ ((x_row >> 1) & 3));
    //   w operand (A) of feature tile j: row wn*64 + 16*(col/4) + 4j + col%4, chunk 2g + ks
    uint32_t w_rel[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int w_row = wn * 64 + 16 * (col >> 2) + 4 * j + (col & 3);
        w_rel[j] = kXBytes + w_row * 128 + 16 * ((2 * g) ^ ((w_row >> 1) & 3));
    }

    f32x4 acc[4][MT];                                          // [feature tile j][token tile mt]
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[j][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- main loop, software-pipelined in half-steps of 32 k.  F0 / F1 hold the operand fragments
    // of the two halves of a stage; the fragments of the NEXT half are requested from LDS while the
    // 4*MT MFMAs of the current half are issued, one request (and, in the second half, one global->LDS
    // load of the stage being refilled) in front of every second MFMA: a burst of LDS requests or of
    // load instructions would leave the matrix core idle for as long as it takes to issue, and with one
    // wavefront per SIMD nothing else fills that gap.  The barrier sits between the two halves: by then
    // a wavefront holds all of stage t in registers, so the stage's buffer can be refilled (loads for
    // step t + STAGES) a whole step before it is needed.
    auto read_frags = [&](uint32_t base, int ks, uint4 (&a)[4], uint4 (&b)[MT]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) a[j] = lds_read16(base + (w_rel[j & 1] ^ (16u * ks)) + (j >> 1) * 1024);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) b[mt] = lds_read16(base + (x_rel ^ (16u * ks)) + mt * 2048);
    };
    auto mma = [&](const uint4 (&a)[4], const uint4 (&b)[MT]) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[j][mt] = In::mfma(as_vec8<vec8>(a[j]), as_vec8<vec8>(b[mt]), acc[j][mt]);
    };
    constexpr int kPer = kXI + kWI;         // load instructions of this wavefront per stage
    constexpr int kGroups = 2 * MT;         // MFMA pairs per half-step
    constexpr int kDmaPerGroup = (kPer + kGroups - 1) / kGroups;
    static_assert(4 + MT <= kGroups, "one LDS request per MFMA pair must cover a half-step's fragments");
    auto issue_one = [&](int d, int kk, uint32_t dst) {
        if (d < kXI) dma16(dst + (kXI * wave + d) * 1024, voff_x[d], x_base + kk * kTK);
        else dma16(dst + kXBytes + (kWI * wave + (d - kXI)) * 1024, voff_w[d - kXI], w_base + kk * kTK);
    };
    // one half-step: MFMAs on (ca, cb); fragments of (rbase, rks) requested into (na, nb); if DMA, the
    // load instructions of k-step kk into the stage at dst
    auto half_step = [&](auto dma_tag, int kk, uint32_t dst, uint32_t rbase, int rks, uint4 (&na)[4], uint4 (&nb)[MT],
                         const uint4 (&ca)[4], const uint4 (&cb)[MT]) {
        constexpr bool DMA = decltype(dma_tag)::value;
#pragma unroll
        for (int gI = 0; gI < kGroups; ++gI) {
            if (DMA) {
#pragma unroll
                for (int d = gI * kDmaPerGroup; d < (gI + 1) * kDmaPerGroup && d < kPer; ++d) issue_one(d, kk, dst);
            }
            if (gI < 4) na[gI] = lds_read16(rbase + (w_rel[gI & 1] ^ (16u * rks)) + (gI >> 1) * 1024);
            else if (gI < 4 + MT) nb[gI - 4] = lds_read16(rbase + (x_rel ^ (16u * rks)) + (gI - 4) * 2048);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int m = 2 * gI; m < 2 * gI + 2; ++m) {
                const int j = m / MT, mt = m % MT;
                acc[j][mt] = In::mfma(as_vec8<vec8>(ca[j]), as_vec8<vec8>(cb[mt]), acc[j][mt]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // wait until at most `later` stages younger than the wanted one are still in flight
    auto wait_stage = [&](int later) {
        if (later <= 0) wait_vm<0>();
        else if (later == 1) wait_vm<kPer>();
        else if (later == 2) wait_vm<2 * kPer>();
        else wait_vm<3 * kPer>();
    };
#pragma unroll
    for (int st = 0; st < STAGES; ++st)
        if (st < ksteps) issue(st, st);
    wait_stage((ksteps < STAGES ? ksteps : STAGES) - 1);       // step 0 has landed
    __syncthreads();
    uint4 a0[4], b0[MT], a1[4], b1[MT];
    read_frags(lds0, 0, a0, b0);
    int buf = 0;                                               // buffer of step kt
    // Steady state (a next step exists, and first the part in which a later step is still to be loaded)
    // is free of conditional LDS traffic, so that the waits in front of the MFMAs cover exactly the
    // fragments they read and not the ones just requested; the last step is peeled.
    auto step = [&](auto dma_tag, int kt) {
        const int buf_next = buf + 1 == STAGES ? 0 : buf + 1;
        // the first half's fragments were requested a half-step ago: retire them now, so that the wait in
        // front of their MFMAs does not also cover the requests that follow (the LDS counter holds 15)
        __builtin_amdgcn_s_waitcnt(0xC07F);                    // lgkmcnt(0)
        half_step(std::false_type{}, 0, 0u, lds0 + buf * kStageBytes, 1, a1, b1, a0, b0);
        const int last_issued = kt + STAGES - 1 < ksteps - 1 ? kt + STAGES - 1 : ksteps - 1;
        wait_stage(last_issued - (kt + 1));                    // step kt+1 has landed
        __syncthreads();                    // ... for every wavefront, and all of them hold step kt in registers
        half_step(dma_tag, kt + STAGES, lds0 + buf * kStageBytes, lds0 + buf_next * kStageBytes, 0, a0, b0, a1, b1);
        buf = buf_next;
    };
    int kt = 0;
    for (; kt + STAGES < ksteps; ++kt) step(std::true_type{}, kt);
    for (; kt + 1 < ksteps; ++kt) step(std::false_type{}, kt);
    __builtin_amdgcn_s_waitcnt(0xC07F);
    read_frags(lds0 + buf * kStageBytes, 1, a1, b1);
    __builtin_amdgcn_sched_barrier(0);
    mma(a0, b0);
    mma(a1, b1);

    if (KSPLIT > 1) {
        // sets 1.. -> LDS -> set 0, one 16-byte slot per (tile, thread) inside the sender's own ring:
        // conflict-free, and summed in set order, so the result does not depend on timing
        const uint32_t lds_all = (uint32_t)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) void*)stage_lds);
        const uint32_t slot = 16u * (wave * kWaveSize + lane);
        __syncthreads();                                       // every ring is out of use
        if (kset != 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    *reinterpret_cast<__attribute__((address_space(3))) f32x4*>(static_cast<uintptr_t>(
                        lds_all + kset * STAGES * kStageBytes + slot + (j * MT + mt) * 16 * kWaveSize * WAVES)) = acc[j][mt];
        }
        __syncthreads();
        if (kset != 0) return;
#pragma unroll
        for (int s = 1; s < KSPLIT; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[j][mt] += *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(static_cast<uintptr_t>(
                        lds_all + s * STAGES * kStageBytes + slot + (j * MT + mt) * 16 * kWaveSize * WAVES));
    }

    // ---- epilogue: this lane owns, for token m0 + wm*16*MT + 16*mt + col, features n_base + 4j + r
    const int n_base = n0 + wn * 64 + 16 * g;
    float bias16[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) bias16[e] = 0.f;
    if (bias) {
        const uint4* bp = reinterpret_cast<const uint4*>(bias + n_base);
        unpack16(In{}, bp[0], bp[1], bias16);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = m0 + wm * 16 * MT + 16 * mt + col;
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
void layernorm_kernel(const uint16_t* x, const uint16_t* __restrict__ gamma,          // y may be x: no restrict
                      const uint16_t* __restrict__ beta, uint16_t* y, int rows_cap,
                      const int32_t* __restrict__ rows_dev, int C, float eps) {
    int rows = rows_cap;
    if (rows_dev) { const int r = *rows_dev; rows = r < rows ? r : rows; }
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int row = blockIdx.x * (kBlockThreads / kWaveSize) + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int chunks = C / 8;
    const uint4* src = reinterpret_cast<const uint4*>(x + (int64_t)row * C);
    // every load of the kernel is issued up front (the row, and the scale / shift vectors the last
    // pass needs), so the two reductions run while gamma and beta are still on their way
    uint4 raw_x[kLnChunks], raw_g[kLnChunks], raw_b[kLnChunks];
#pragma unroll
    for (int i = 0; i < kLnChunks; ++i) {
        const int c = lane + kWaveSize * i;
        if (c < chunks) {
            raw_x[i] = src[c];
            raw_g[i] = reinterpret_cast<const uint4*>(gamma)[c];
            raw_b[i] = reinterpret_cast<const uint4*>(beta)[c];
        }
    }
    float v[kLnChunks][8];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kLnChunks; ++i) {
        const int c = lane + kWaveSize * i;
        if (c < chunks) {
            float t[16];
            const uint4 raw = raw_x[i];
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
            const uint4 graw = raw_g[i], braw = raw_b[i];
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

template <typename In, int WNW, int WMW, int MT, int STAGES, int KSPLIT>
hipError_t launch_linear_shape(const void* x, const void* w, const void* bias, const void* res, void* y,
                               int rows_cap, const int32_t* rows_dev, int N, int K, int act, hipStream_t stream) {
    constexpr int TN = 64 * WNW, TM = 16 * MT * WMW;
    const int n_tiles = N / TN;
    const int m_tiles = (rows_cap + TM - 1) / TM;
    const int m_tiles8 = (m_tiles + kXcds - 1) / kXcds * kXcds;
    const dim3 grid(m_tiles8 * n_tiles), block(kWaveSize * WNW * WMW * KSPLIT);
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    const uint16_t* wp = static_cast<const uint16_t*>(w);
    const uint16_t* bp = static_cast<const uint16_t*>(bias);
    const uint16_t* rp = static_cast<const uint16_t*>(res);
    uint16_t* yp = static_cast<uint16_t*>(y);
    hipError_t err;
    if (act == 1 && res)
        err = launch_kernel((linear_kernel<In, 1, true, WNW, WMW, MT, STAGES, KSPLIT>), grid, block, stream, xp, wp, bp, rp, yp, rows_cap, rows_dev, N, K, n_tiles);
    else if (act == 1)
        err = launch_kernel((linear_kernel<In, 1, false, WNW, WMW, MT, STAGES, KSPLIT>), grid, block, stream, xp, wp, bp, rp, yp, rows_cap, rows_dev, N, K, n_tiles);
    else if (res)
        err = launch_kernel((linear_kernel<In, 0, true, WNW, WMW, MT, STAGES, KSPLIT>), grid, block, stream, xp, wp, bp, rp, yp, rows_cap, rows_dev, N, K, n_tiles);
    else
        err = launch_kernel((linear_kernel<In, 0, false, WNW, WMW, MT, STAGES, KSPLIT>), grid, block, stream, xp, wp, bp, rp, yp, rows_cap, rows_dev, N, K, n_tiles);
    return err;
}

// Shape choice from what the host knows (the expected row count -- the capacity unless the caller
// gave a better estimate --, N, K); times in us on one MI355X, fp16, no epilogue work:
//   * 256 x 256 tiles (one work-group of eight wavefronts per CU; half the L2 -> LDS bytes per flop of a
//     128 x 128 tile) when there are enough of them for well over one round of the 256 CUs, or when the
//     k-loop is long and the tiles fill at least half the chip (12608 x 768 x 3072: 64 against 75);
//   * 64 x 64 tiles, one wavefront per k-half (two per work-group), when 128 x 128 tiles would leave at
//     least half the CUs idle: what limits a small problem is how many bytes the chip has in flight, and
//     four times as many work-groups, each with two rings, keep more of them going
//     (1334 x 768 x 3072: 19 against 32; 1334 x 768 x 768: 7.9 against 8.7);
//   * else 128 x 128 tiles, four wavefronts, two work-groups per CU (N an odd multiple of 64, as in the
//     192-wide DeiT-Tiny blocks: 64 x 64 tiles whatever the size).
// Rings of three and four stages were measured too: no gain over two except at 1334 x 768 x 3072, where
// the 64 x 64 shape is faster still.
template <typename In>
hipError_t launch_linear_typed(const void* x, const void* w, const void* bias, const void* res, void* y,
                               int rows_cap, const int32_t* rows_dev, int rows_hint, int N, int K, int act,
                               hipStream_t stream) {
    const int ksteps = K / kTK;
    const int64_t big_tiles = (int64_t)((rows_hint + 255) / 256) * (N / 256);
    if (N % 256 == 0 && (big_tiles >= kBigTileMinGroups || (ksteps >= 32 && big_tiles >= 128)))
        return launch_linear_shape<In, 4, 2, 8, 2, 1>(x, w, bias, res, y, rows_cap, rows_dev, N, K, act, stream);
    const int64_t small_tiles = (int64_t)((rows_hint + 127) / 128) * ((N + 127) / 128);
    if ((small_tiles <= kSplitMaxGroups || N % 128 != 0) && ksteps % 2 == 0)
        return launch_linear_shape<In, 1, 1, 4, 2, 2>(x, w, bias, res, y, rows_cap, rows_dev, N, K, act, stream);
    if (N % 128 != 0)          // an odd multiple of 64 features and an odd number of k-steps: 64 x 64 tiles, one wavefront
        return launch_linear_shape<In, 1, 1, 4, 2, 1>(x, w, bias, res, y, rows_cap, rows_dev, N, K, act, stream);
    return launch_linear_shape<In, 2, 2, 4, 2, 1>(x, w, bias, res, y, rows_cap, rows_dev, N, K, act, stream);
}

}  // namespace

hipError_t launch_linear(const void* x, const void* w, const void* bias, const void* res, void* y, int rows_cap,
                         const int32_t* rows_dev, int rows_hint, int N, int K, int act, ragged_dtype dt,
                         hipStream_t stream) {
    if (dt == RAGGED_F16)
        return launch_linear_typed<F16>(x, w, bias, res, y, rows_cap, rows_dev, rows_hint, N, K, act, stream);
    return launch_linear_typed<BF16>(x, w, bias, res, y, rows_cap, rows_dev, rows_hint, N, K, act, stream);
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
    hipError_t err;
    if (dt == RAGGED_F16)
        err = launch_kernel((layernorm_kernel<F16>), grid, block, stream, xp, gp, bp, yp, rows_cap, rows_dev, C, eps);
    else
        err = launch_kernel((layernorm_kernel<BF16>), grid, block, stream, xp, gp, bp, yp, rows_cap, rows_dev, C, eps);
    return err;
}

}  // namespace ragged
