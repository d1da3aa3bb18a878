// Bidirectional multi-head attention over a packed ragged buffer (Section 4.2, Algorithm 1), for
// gfx950.  One launch; one work-group per (image, head) pair and block of up to 16*QW*WAVES query
// rows.  At ViT lengths a whole sequence's K and V fit in LDS (160 KB per CU), so instead of
// streaming 64-key tiles per query tile the group loads K/V ONCE (chunks of up to KC keys, all global
// loads of a chunk in flight together), hits one barrier, and every wavefront then runs its queries
// against LDS-resident keys with MFMA 16x16x32 (fp32 accumulation) and an fp32 online softmax.
//
// Orientation.  A wavefront owns QW subtiles of 16 queries and computes the TRANSPOSED scores
// S^T = K Q^T (keys x queries).  In the MFMA result layout a lane then holds, for ONE query
// (column lane%16), the scores of keys 4*(lane/16)+r of every 16-key subtile.  That is already the
// "B operand" shape of the second contraction O^T = V^T P^T, so P never leaves registers, the
// softmax statistics are per-lane scalars, and a row maximum needs only two cross-lane steps
// (lanes l, l^16, l^32, l^48 share a query).  With QW = 2 each K / V^T operand read from LDS feeds
// two MFMAs.
//
// MFMA 16x16x32 operand layout used below (A: 16 rows x 32 k, B: 32 k x 16 cols, D: 16x16):
//   A: lane l holds row l%16,  k-slots 8*(l/16)+e, e = 0..7
//   B: lane l holds col l%16,  k-slots 8*(l/16)+e
//   D: lane l, register r holds row 4*(l/16)+r, col l%16
// Which contraction index sits in which k-slot is free as long as A and B agree, and which logical
// row/column an MFMA row/column stands for is free as long as loads and stores agree.  Both
// freedoms are used to make every LDS access a 16-byte one and every global access contiguous:
//   * Q (B operand of S^T): lane group g = l/16 loads head-dim elements 16g..16g+15 of its query.
//   * K chunk in LDS, row-major [key][d], row stride 72 halves; A operand = 8 halves at d = 16g+8s.
//   * V chunk in LDS TRANSPOSED, [rho][kappa], row stride KC+8 halves, where
//        rho(d)     = (d%4)*16 + d/4                      (row permutation of the head dim)
//        kappa(key) = 32*(key/32) + 8*((key%16)/4) + 4*((key%32)/16) + key%4
//     so that lane group g reads 8 consecutive kappa = exactly the keys whose probabilities it
//     holds, and ends up owning output elements d = 16g .. 16g+15 of its query (32 contiguous
//     bytes).  The transposition is done once per chunk in registers while filling LDS.
//
// bf16 inputs: Q K^T uses the bf16 MFMA (products are exact in fp32).  A bf16 probability would
// carry only 8 significant bits, so P is split as P = P_hi + P_lo (two bf16 values, 16 bits
// together) and P V is two MFMAs; V stays exact.  The path is not MFMA-bound at ViT lengths.
#include <stdlib.h>

#include "common.h"

namespace ragged {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kHeadDim = 64;
constexpr int kBN = 64;                 // keys per softmax step (four 16-key subtiles)
constexpr int kKStride = 72;            // halves per K row in LDS: 64 + 8 of padding (144 bytes)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazyLog2 = 8.0f;       // probabilities stay below 2^8 between rescales

struct F16 {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ vec8 ones() {
        vec8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (_Float16)1.0f;
        return v;
    }
};
struct BF16 {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ vec8 ones() {
        vec8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (__bf16)1.0f;
        return v;
    }
};

template <typename V>
__device__ __forceinline__ V as_vec8(uint4 raw) { return __builtin_bit_cast(V, raw); }

// O^T += V^T P^T for one 32-key block: p[0..7] are this lane's probabilities (fp32).  The row sums
// of P ride along on the matrix core: with an all-ones A operand every row of the result holds
// sum_k P[k][query], already reduced over the four lane groups, and it is the sum of exactly the
// rounded probabilities that multiply V.
__device__ __forceinline__ void pv_block(F16, const uint4 (&vt)[4], const float (&p)[8], f32x4 (&o)[4],
                                         f32x4& l) {
    f16x8 pb;
#pragma unroll
    for (int e = 0; e < 8; ++e) pb[e] = (_Float16)p[e];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) o[dt] = F16::mfma(as_vec8<f16x8>(vt[dt]), pb, o[dt]);
    l = F16::mfma(F16::ones(), pb, l);
}
__device__ __forceinline__ void pv_block(BF16, const uint4 (&vt)[4], const float (&p)[8], f32x4 (&o)[4],
                                         f32x4& l) {
    bf16x8 hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        hi[e] = (__bf16)p[e];
        lo[e] = (__bf16)(p[e] - (float)hi[e]);
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        o[dt] = BF16::mfma(as_vec8<bf16x8>(vt[dt]), hi, o[dt]);
        o[dt] = BF16::mfma(as_vec8<bf16x8>(vt[dt]), lo, o[dt]);
    }
    l = BF16::mfma(BF16::ones(), hi, l);
    l = BF16::mfma(BF16::ones(), lo, l);
}

// Store 16 consecutive head-dim elements of one output row.
__device__ __forceinline__ void store16(_Float16* dst, const float (&v)[16]) {
    f16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (_Float16)v[e]; b[e] = (_Float16)v[8 + e]; }
    reinterpret_cast<uint4*>(dst)[0] = __builtin_bit_cast(uint4, a);
    reinterpret_cast<uint4*>(dst)[1] = __builtin_bit_cast(uint4, b);
}
__device__ __forceinline__ void store16(__bf16* dst, const float (&v)[16]) {
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)v[e]; b[e] = (__bf16)v[8 + e]; }
    reinterpret_cast<uint4*>(dst)[0] = __builtin_bit_cast(uint4, a);
    reinterpret_cast<uint4*>(dst)[1] = __builtin_bit_cast(uint4, b);
}
__device__ __forceinline__ void store16(float* dst, const float (&v)[16]) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
        reinterpret_cast<float4*>(dst)[e] = make_float4(v[4 * e], v[4 * e + 1], v[4 * e + 2], v[4 * e + 3]);
}

// Maximum over the four lanes that share a query (l, l^16, l^32, l^48) with the gfx950 lane-swap
// instructions (pure VALU, no LDS round trip).  permlane32_swap(a, b) returns {a.lo|b.lo, a.hi|b.hi}
// (32-lane halves); permlane16_swap(a, b) returns {a.row0,b.row0,a.row2,b.row2} and
// {a.row1,b.row1,a.row3,b.row3} (16-lane rows).  With b a copy of a, combining the two results
// reduces across the halves, then across the rows.  The copy is made through an opaque move so the
// two operands can never be folded into one register (the instruction swaps its operands in place).
__device__ __forceinline__ unsigned opaque_copy(unsigned x) {
    unsigned y;
    asm volatile("v_mov_b32 %0, %1" : "=v"(y) : "v"(x));
    return y;
}
__device__ __forceinline__ float as_f32(unsigned u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ unsigned as_u32(float f) { return __builtin_bit_cast(unsigned, f); }
__device__ __forceinline__ float quad_max(float x) {
    const auto a = __builtin_amdgcn_permlane32_swap(as_u32(x), opaque_copy(as_u32(x)), false, false);
    const unsigned a0 = a[0], a1 = a[1];
    x = fmaxf(as_f32(a0), as_f32(a1));
    const auto b = __builtin_amdgcn_permlane16_swap(as_u32(x), opaque_copy(as_u32(x)), false, false);
    const unsigned b0 = b[0], b1 = b[1];
    return fmaxf(as_f32(b0), as_f32(b1));
}

// Per-query-subtile running state of the online softmax.
struct RowState {
    float m;          // reference maximum (log2 domain); -inf before the first step
    f32x4 l;          // running row sum of the probabilities (every register holds the same value)
    f32x4 o[4];       // O^T accumulators: register r of tile dt is head-dim element 16g + 4r + dt
};

// One 64-key step (keys already in LDS) for this wavefront's QW query subtiles:
// S^T = K Q^T, online-softmax update, O^T += V^T P^T.
//   NT   = 16-key subtiles present in the step (1..4)
//   MASK = the last subtile may hold keys past the end of the sequence (index >= rem): masked out
// K and V^T operands are read from LDS once and reused by every query subtile of the wavefront.
// The body is branch-free: a subtile with no real query rows (zero Q) is computed along and never
// stored, which keeps every LDS read of a phase in flight ahead of the MFMAs that consume it.
// scale_log2e >= 0 here (a negative softmax scale is folded into the sign of Q by the caller), so
// the row maximum can be taken on the raw scores and the scale fused into the exponent's FMA.
template <typename In, int QW, int NT, bool MASK>
__device__ __forceinline__ void tile_update(const uint16_t* __restrict__ k_tile,
                                            const uint16_t* __restrict__ vt_tile, int vt_stride,
                                            const typename In::vec8 (&q_frag)[QW][2], int rem, int col, int g,
                                            float scale_log2e, RowState (&rows)[QW]) {
    typedef typename In::vec8 vec8;
    // -------- S^T = K Q^T : NT 16-key subtiles, two k-steps of 32 head-dim elements
    f32x4 st[QW][NT];
#pragma unroll
    for (int j = 0; j < QW; ++j)
#pragma unroll
        for (int kt = 0; kt < NT; ++kt) st[j][kt] = f32x4{0.f, 0.f, 0.f, 0.f};
    vec8 ka[NT][2];
#pragma unroll
    for (int kt = 0; kt < NT; ++kt)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
            ka[kt][ks] = as_vec8<vec8>(*reinterpret_cast<const uint4*>(
                &k_tile[(16 * kt + col) * kKStride + 16 * g + 8 * ks]));
#pragma unroll
    for (int kt = 0; kt < NT; ++kt)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int j = 0; j < QW; ++j) st[j][kt] = In::mfma(ka[kt][ks], q_frag[j][ks], st[j][kt]);
    // -------- online softmax (this lane: one query per subtile, keys 16*kt + 4*g + r of the step)
    const int last_valid = rem - 16 * (NT - 1) - 4 * g;        // r < last_valid is a real key (last subtile)
#pragma unroll
    for (int j = 0; j < QW; ++j) {
        float t_max = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < NT; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                t_max = fmaxf(t_max, (!MASK || kt < NT - 1 || r < last_valid) ? st[j][kt][r] : -INFINITY);
        t_max = quad_max(t_max) * scale_log2e;                  // finite: the step has a valid key
        // Lazy rescaling: the reference maximum only moves when some query's step maximum exceeds
        // it by more than 2^kLazyLog2 (always on the first step, where it is -inf).  Until then
        // probabilities may reach 2^kLazyLog2 instead of 1 -- harmless in fp16/bf16/fp32 -- and
        // the accumulators need no per-step multiply.  Same softmax: the reference cancels.
        RowState& rs = rows[j];
        if (__builtin_amdgcn_ballot_w64(t_max > rs.m + kLazyLog2) != 0) {   // wavefront-uniform
            const float m_new = fmaxf(rs.m, t_max);
            const float alpha = __builtin_amdgcn_exp2f(rs.m - m_new);
            rs.m = m_new;
            rs.l *= alpha;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) rs.o[dt] *= alpha;
        }
#pragma unroll
        for (int kt = 0; kt < NT; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[j][kt][r], scale_log2e, -rs.m));
                if (MASK && kt == NT - 1) p = (r < last_valid) ? p : 0.f;
                st[j][kt][r] = p;
            }
    }
    // -------- O^T += V^T P^T : 32-key blocks x four 16-row head-dim tiles (odd NT: zero upper half)
#pragma unroll
    for (int bb = 0; bb < (NT + 1) / 2; ++bb) {
        uint4 vt[4];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
            vt[dt] = *reinterpret_cast<const uint4*>(&vt_tile[(16 * dt + col) * vt_stride + 32 * bb + 8 * g]);
#pragma unroll
        for (int j = 0; j < QW; ++j) {
            float p[8];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[r] = st[j][2 * bb][r];
                p[4 + r] = (2 * bb + 1 < NT) ? st[j][(2 * bb + 1 < NT) ? 2 * bb + 1 : 0][r] : 0.f;
            }
            pv_block(In{}, vt, p, rows[j].o, rows[j].l);
        }
    }
}

// Work-group index -> (query block, image-head pair): bid = block * pairs8 + pair, pairs8 = B*H
// rounded up to a multiple of 8.  The hardware deals consecutive work-groups round-robin to the 8
// XCDs, so all query blocks of a pair run on XCD pair%8 and share its L2; block 0 of every pair is
// dispatched first, so with ragged lengths the surplus blocks of the upper-bound grid sit at the
// end of the dispatch order and retire while real work is already running.
//
// Template: WAVES wavefronts per group, QW query subtiles (16 rows) per wavefront, KC = keys per
// LDS-resident chunk (a multiple of 64).  Subtile (j*WAVES + wave) of the block belongs to
// wavefront `wave`, so short sequences spread over as many wavefronts as possible.
template <typename In, typename OutT, int WAVES, int QW, int KC, int STEP, int MINW>
__global__ __launch_bounds__(kWaveSize * WAVES, MINW)
void attn_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                 const uint16_t* __restrict__ v, OutT* __restrict__ o,
                 const int32_t* __restrict__ cu_seqlens, int H, int pairs, int pairs8,
                 float scale_log2e, int negate_q) {
    typedef typename In::vec8 vec8;
    constexpr int kThreads = kWaveSize * WAVES;
    constexpr int kBM = 16 * QW * WAVES;                       // query rows per work-group
    constexpr int kVtStride = KC + 8;                          // halves per V^T row in LDS
    constexpr int kKIters = (KC * 8 + kThreads - 1) / kThreads;        // 16-byte K units per thread
    constexpr int kVIters = (KC * 2 + kThreads - 1) / kThreads;        // (4 keys x 8 dims) V units per thread
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* const k_lds = lds;                               // [KC][72]
    uint16_t* const vt_lds = lds + KC * kKStride;              // [64][KC + 8]

    const int block = blockIdx.x / pairs8;
    const int pair = blockIdx.x - block * pairs8;
    if (pair >= pairs) return;
    const int h = pair % H;
    const int img = pair / H;
    const int s = cu_seqlens[img];
    const int n = cu_seqlens[img + 1] - s;
    const int m0 = block * kBM;
    if (m0 >= n) return;                                       // whole group exits together

    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid >> 6;
    const int col = lane & 15;                                 // query inside a 16-row subtile
    const int g = lane >> 4;                                   // lane group
    const int64_t tok = (int64_t)H * kHeadDim;                 // elements between tokens
    const uint16_t* const k_base = k + s * tok + (int64_t)h * kHeadDim;
    const uint16_t* const v_base = v + s * tok + (int64_t)h * kHeadDim;

    // ---- this wavefront's query subtiles
    bool active[QW];
    int q_row[QW];
#pragma unroll
    for (int j = 0; j < QW; ++j) {
        const int row0 = m0 + (j * WAVES + wave) * 16;
        active[j] = row0 < n;
        q_row[j] = row0 + col;
    }

    // ---- chunk loader: all global loads of a chunk are issued before the first LDS write
    uint4 k_raw[kKIters];
    uint4 v_raw[kVIters][4];
    auto issue_loads = [&](int c0, int cn) {                   // keys [c0, c0+cn) of the sequence
#pragma unroll
        for (int it = 0; it < kKIters; ++it) {
            const int u = tid + it * kThreads;                 // unit: key u/8, dims 8*(u%8)..
            k_raw[it] = make_uint4(0, 0, 0, 0);
            if ((u >> 3) < cn)
                k_raw[it] = *reinterpret_cast<const uint4*>(k_base + (c0 + (u >> 3)) * tok + 8 * (u & 7));
        }
#pragma unroll
        for (int it = 0; it < kVIters; ++it) {
            const int u = tid + it * kThreads;                 // unit: keys 4*(u/8)..+3, dims 8*(u%8)..
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int key = 4 * (u >> 3) + a;
                v_raw[it][a] = make_uint4(0, 0, 0, 0);         // keys past the end are zero in LDS
                if (key < cn)
                    v_raw[it][a] = *reinterpret_cast<const uint4*>(v_base + (c0 + key) * tok + 8 * (u & 7));
            }
        }
    };
    auto stage = [&](int cn) {
        const int cn32 = (cn + 31) & ~31;                      // V^T is consumed in 32-key blocks
#pragma unroll
        for (int it = 0; it < kKIters; ++it) {
            const int u = tid + it * kThreads;
            if ((u >> 3) < cn)
                *reinterpret_cast<uint4*>(&k_lds[(u >> 3) * kKStride + 8 * (u & 7)]) = k_raw[it];
        }
#pragma unroll
        for (int it = 0; it < kVIters; ++it) {
            const int u = tid + it * kThreads;
            const int key0 = 4 * (u >> 3);
            if (key0 >= cn32 || key0 >= KC) continue;
            const int kappa = 32 * (key0 >> 5) + 8 * ((key0 & 15) >> 2) + 4 * ((key0 & 31) >> 4);
            const uint32_t w[4][4] = {{v_raw[it][0].x, v_raw[it][0].y, v_raw[it][0].z, v_raw[it][0].w},
                                      {v_raw[it][1].x, v_raw[it][1].y, v_raw[it][1].z, v_raw[it][1].w},
                                      {v_raw[it][2].x, v_raw[it][2].y, v_raw[it][2].z, v_raw[it][2].w},
                                      {v_raw[it][3].x, v_raw[it][3].y, v_raw[it][3].z, v_raw[it][3].w}};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int d = 8 * (u & 7) + e;
                const int rho = (d & 3) * 16 + (d >> 2);
                uint2 packed4;
                if (e & 1) {
                    packed4.x = (w[0][e >> 1] >> 16) | (w[1][e >> 1] & 0xffff0000u);
                    packed4.y = (w[2][e >> 1] >> 16) | (w[3][e >> 1] & 0xffff0000u);
                } else {
                    packed4.x = (w[0][e >> 1] & 0xffffu) | (w[1][e >> 1] << 16);
                    packed4.y = (w[2][e >> 1] & 0xffffu) | (w[3][e >> 1] << 16);
                }
                *reinterpret_cast<uint2*>(&vt_lds[rho * kVtStride + kappa]) = packed4;
            }
        }
    };

    issue_loads(0, min(n, KC));

    // ---- Q: each lane's query rows, head-dim elements 16g .. 16g+15 (zeros past the sequence end)
    vec8 q_frag[QW][2];
#pragma unroll
    for (int j = 0; j < QW; ++j) {
        uint4 q_raw[2] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
        if (q_row[j] < n) {
            const uint4* src = reinterpret_cast<const uint4*>(
                q + (s + q_row[j]) * tok + (int64_t)h * kHeadDim + 16 * g);
            q_raw[0] = src[0];
            q_raw[1] = src[1];
        }
        if (negate_q) {                                        // softmax(-|c| q.k) == softmax(|c| (-q).k)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                q_raw[e].x ^= 0x80008000u; q_raw[e].y ^= 0x80008000u;
                q_raw[e].z ^= 0x80008000u; q_raw[e].w ^= 0x80008000u;
            }
        }
        q_frag[j][0] = as_vec8<vec8>(q_raw[0]);
        q_frag[j][1] = as_vec8<vec8>(q_raw[1]);
    }

    RowState rows[QW];
#pragma unroll
    for (int j = 0; j < QW; ++j) {
        rows[j].m = -INFINITY;
        rows[j].l = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) rows[j].o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int c0 = 0; c0 < n; c0 += KC) {
        const int cn = min(n - c0, KC);                        // keys in this chunk
        if (c0 > 0) {
            __syncthreads();                                   // every wavefront is done with the previous chunk
            issue_loads(c0, cn);
        }
        stage(cn);
        __syncthreads();
        if (!active[0]) continue;                              // no queries here: this wavefront only loads
        for (int t0 = 0; t0 < cn; t0 += STEP) {
            const int rem = cn - t0;
            const uint16_t* kt_ = k_lds + t0 * kKStride;
            const uint16_t* vt_ = vt_lds + t0;                 // kappa permutes inside 32-key blocks only
            if (rem >= STEP) {
                tile_update<In, QW, STEP / 16, false>(kt_, vt_, kVtStride, q_frag, rem, col, g, scale_log2e, rows);
            } else {
                const int nt = (rem + 15) >> 4;
                if (nt == 1) tile_update<In, QW, 1, true>(kt_, vt_, kVtStride, q_frag, rem, col, g, scale_log2e, rows);
                else if (nt == 2 || STEP == 32) tile_update<In, QW, 2, true>(kt_, vt_, kVtStride, q_frag, rem, col, g, scale_log2e, rows);
                else if (nt == 3) tile_update<In, QW, 3, true>(kt_, vt_, kVtStride, q_frag, rem, col, g, scale_log2e, rows);
                else tile_update<In, QW, STEP / 16, true>(kt_, vt_, kVtStride, q_frag, rem, col, g, scale_log2e, rows);
            }
        }
    }

    // ---- normalise and store: a lane owns d = 16g + 4r + dt of its query
#pragma unroll
    for (int j = 0; j < QW; ++j) {
        if (q_row[j] < n) {
            const float inv = 1.0f / rows[j].l[0];
            float out16[16];
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 4; ++r) out16[4 * r + dt] = rows[j].o[dt][r] * inv;
            store16(o + (s + q_row[j]) * tok + (int64_t)h * kHeadDim + 16 * g, out16);
        }
    }
}

template <int KC>
constexpr int lds_bytes() { return (KC * kKStride + kHeadDim * (KC + 8)) * 2; }

template <typename In, typename OutT, int WAVES, int QW, int KC, int STEP, int MINW>
hipError_t launch_config(const void* q, const void* k, const void* v, void* o,
                         const int32_t* cu_seqlens, int B, int max_seqlen, int H, float scale,
                         hipStream_t stream) {
    constexpr int rows = 16 * QW * WAVES;
    constexpr int bytes = lds_bytes<KC>();
    auto kernel = attn_kernel<In, OutT, WAVES, QW, KC, STEP, MINW>;
    if (bytes > 64 * 1024) {
        // more than the default dynamic-LDS limit: raise it once per kernel instance
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (attr != hipSuccess) return attr;
    }
    const int blocks = (max_seqlen + rows - 1) / rows;
    const int pairs = B * H;
    const int pairs8 = (pairs + kXcds - 1) / kXcds * kXcds;
    hipLaunchKernelGGL(kernel, dim3(blocks * pairs8), dim3(kWaveSize * WAVES), bytes, stream,
                       static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                       static_cast<const uint16_t*>(v), static_cast<OutT*>(o), cu_seqlens, H,
                       pairs, pairs8, fabsf(scale) * kLog2e, scale < 0.f ? 1 : 0);
    return hipGetLastError();
}

// Group shape by the host-known upper bound on the sequence lengths:
//   <= 64  : 4 wavefronts x 1 subtile,  64-key chunk  (18 KB LDS)
//   <= 128 : 8 wavefronts x 1 subtile, 128-key chunk  (36 KB LDS)
//   longer : 8 wavefronts x 2 subtiles (256 query rows per group), 256-key chunks (71 KB LDS,
//            two groups per CU); sequences beyond 256 keys take several chunks / query blocks.
template <typename In, typename OutT>
hipError_t launch_typed(const void* q, const void* k, const void* v, void* o,
                        const int32_t* cu_seqlens, int B, int max_seqlen, int H, float scale,
                        hipStream_t stream) {
    static const int variant = getenv("RAGGED_ATTN_VARIANT") ? atoi(getenv("RAGGED_ATTN_VARIANT")) : 0;
    if (max_seqlen <= 64)
        return launch_config<In, OutT, 4, 1, 64, 64, 4>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
    if (max_seqlen <= 128)
        return launch_config<In, OutT, 8, 1, 128, 64, 4>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
    if (variant == 1)
        return launch_config<In, OutT, 16, 1, 256, 64, 4>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
    if (variant == 2)
        return launch_config<In, OutT, 8, 2, 256, 32, 4>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
    if (variant == 3)
        return launch_config<In, OutT, 8, 1, 256, 64, 4>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
    return launch_config<In, OutT, 8, 2, 256, 64, 2>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
}

}  // namespace

hipError_t launch_attn(const void* q, const void* k, const void* v, void* o,
                       const int32_t* cu_seqlens, int B, int max_seqlen, int H, float scale,
                       ragged_dtype in_dt, ragged_dtype out_dt, hipStream_t stream) {
    if (in_dt == RAGGED_F16 && out_dt == RAGGED_F16)
        return launch_typed<F16, _Float16>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
    if (in_dt == RAGGED_F16 && out_dt == RAGGED_F32)
        return launch_typed<F16, float>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
    if (in_dt == RAGGED_BF16 && out_dt == RAGGED_BF16)
        return launch_typed<BF16, __bf16>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
    if (in_dt == RAGGED_BF16 && out_dt == RAGGED_F32)
        return launch_typed<BF16, float>(q, k, v, o, cu_seqlens, B, max_seqlen, H, scale, stream);
    return hipErrorInvalidValue;
}

}  // namespace ragged
