// Bidirectional multi-head attention over a packed ragged buffer (Section 4.2, Algorithm 1), for
// gfx950: one launch, one work-group per (image, head, 64-query tile), K/V tiles staged in LDS,
// MFMA 16x16x32 for both contractions with fp32 accumulation, fp32 online softmax.
//
// Orientation.  Each wavefront owns 16 queries and computes the TRANSPOSED score tile
// S^T = K Q^T (keys x queries).  In the MFMA result layout a lane then holds, for ONE query
// (column lane%16), the scores of keys 4*(lane/16)+r of every 16-key tile.  That is already the
// "B operand" shape of the second contraction O^T = V^T P^T, so P never leaves registers, the
// softmax statistics are per-lane scalars, and a row maximum needs only two cross-lane steps
// (lanes l, l^16, l^32, l^48 share a query).
//
// MFMA 16x16x32 operand layout used below (A: 16 rows x 32 k, B: 32 k x 16 cols, D: 16x16):
//   A: lane l holds row l%16,  k-slots 8*(l/16)+e, e = 0..7
//   B: lane l holds col l%16,  k-slots 8*(l/16)+e
//   D: lane l, register r holds row 4*(l/16)+r, col l%16
// Which contraction index sits in which k-slot is free as long as A and B agree, and which logical
// row/column an MFMA row/column stands for is free as long as loads and stores agree.  Both
// freedoms are used to make every LDS access a conflict-free 16-byte one and every global access a
// contiguous 32 bytes per lane:
//   * Q (B operand of S^T): lane group g = l/16 loads head-dim elements 16g..16g+15 of its query.
//   * K tile in LDS, row-major [key][d], row stride 72 halves; A operand = 8 halves at d = 16g+8s.
//   * V tile in LDS TRANSPOSED, [rho][kappa], stride 72 halves, where
//        rho(d)     = (d%4)*16 + d/4                      (row permutation of the head dim)
//        kappa(key) = 32*(key/32) + 8*((key%16)/4) + 4*((key%32)/16) + key%4
//     so that lane group g reads 8 consecutive kappa = exactly the keys whose probabilities it
//     holds, and ends up owning output elements d = 16g .. 16g+15 of its query (32 contiguous
//     bytes).  The transposition is done once per tile in registers while filling LDS.
//
// bf16 inputs: Q K^T uses the bf16 MFMA (products are exact in fp32).  A bf16 probability would
// carry only 8 significant bits, so P is split as P = P_hi + P_lo (two bf16 values, 16 bits
// together) and P V is two MFMAs; V stays exact.  The path is not MFMA-bound at ViT lengths.
#include "common.h"

namespace ragged {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kHeadDim = 64;
constexpr int kBN = 64;                 // keys per K/V tile
constexpr int kLdsStride = 72;          // halves per LDS row: 64 + 8 of padding (144 bytes)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazyLog2 = 8.0f;       // probabilities stay below 2^8 between rescales
constexpr int kMaxGatherTokens = 1536;  // tokens per image the gather-on-load variant can index in LDS

struct F16 {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};
struct BF16 {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
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
    f16x8 pb, ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) { pb[e] = (_Float16)p[e]; ones[e] = (_Float16)1.0f; }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) o[dt] = F16::mfma(as_vec8<f16x8>(vt[dt]), pb, o[dt]);
    l = F16::mfma(ones, pb, l);
}
__device__ __forceinline__ void pv_block(BF16, const uint4 (&vt)[4], const float (&p)[8], f32x4 (&o)[4],
                                         f32x4& l) {
    bf16x8 hi, lo, ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        hi[e] = (__bf16)p[e];
        lo[e] = (__bf16)(p[e] - (float)hi[e]);
        ones[e] = (__bf16)1.0f;
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        o[dt] = BF16::mfma(as_vec8<bf16x8>(vt[dt]), hi, o[dt]);
        o[dt] = BF16::mfma(as_vec8<bf16x8>(vt[dt]), lo, o[dt]);
    }
    l = BF16::mfma(ones, hi, l);
    l = BF16::mfma(ones, lo, l);
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

// Reductions over the four lanes that share a query (l, l^16, l^32, l^48) with the gfx950 lane-swap
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
// One K/V tile (already in LDS) against this wavefront's 16 queries: S^T = K Q^T, online-softmax
// update, O^T += V^T P^T.  NT = 16-key subtiles present in the tile (1..4); MASK: the last subtile may
// hold keys past the end of the sequence (index >= rem), which are masked out.
// scale_log2e >= 0 here (a negative softmax scale is folded into the sign of Q by the caller), so
// the row maximum can be taken on the raw scores and the scale fused into the exponent's FMA.
template <typename In, int NT, bool MASK>
__device__ __forceinline__ void tile_update(const uint16_t* __restrict__ k_tile,
                                            const uint16_t* __restrict__ vt_tile,
                                            const typename In::vec8 (&q_frag)[2], int rem, int col, int g,
                                            float scale_log2e, float& m_run, f32x4& l_acc,
                                            f32x4 (&o_acc)[4]) {
    typedef typename In::vec8 vec8;
    // -------- S^T = K Q^T : NT 16-key subtiles, two k-steps of 32 head-dim elements
    f32x4 st[NT];
#pragma unroll
    for (int kt = 0; kt < NT; ++kt) {
        st[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const uint4 a = *reinterpret_cast<const uint4*>(
                &k_tile[(16 * kt + col) * kLdsStride + 16 * g + 8 * ks]);
            st[kt] = In::mfma(as_vec8<vec8>(a), q_frag[ks], st[kt]);
        }
    }
    // -------- online softmax (this lane: one query, keys 16*kt + 4*g + r of the tile)
    const int last_valid = rem - 16 * (NT - 1) - 4 * g;        // r < last_valid is a real key (last subtile)
    float t_max = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NT; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            t_max = fmaxf(t_max, (!MASK || kt < NT - 1 || r < last_valid) ? st[kt][r] : -INFINITY);
    t_max = quad_max(t_max) * scale_log2e;                      // finite: the tile has a valid key
    // Lazy rescaling: the reference maximum m_run only moves when some query's tile maximum exceeds
    // it by more than 2^kLazyLog2 (always on the first tile, where m_run = -inf).  Until then
    // probabilities may reach 2^kLazyLog2 instead of 1 -- harmless in fp16/bf16/fp32 -- and the
    // accumulators need no per-tile multiply.  The result is the same softmax: m_run cancels.
    if (__builtin_amdgcn_ballot_w64(t_max > m_run + kLazyLog2) != 0) {   // wavefront-uniform
        const float m_new = fmaxf(m_run, t_max);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        l_acc *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) o_acc[dt] *= alpha;
    }
#pragma unroll
    for (int kt = 0; kt < NT; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kt][r], scale_log2e, -m_run));
            if (MASK && kt == NT - 1) p = (r < last_valid) ? p : 0.f;
            st[kt][r] = p;
        }
    // -------- O^T += V^T P^T : 32-key blocks x four 16-row head-dim tiles (odd NT: zero upper half)
#pragma unroll
    for (int bb = 0; bb < (NT + 1) / 2; ++bb) {
        uint4 vt[4];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
            vt[dt] = *reinterpret_cast<const uint4*>(
                &vt_tile[(16 * dt + col) * kLdsStride + 32 * bb + 8 * g]);
        float p[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p[r] = st[2 * bb][r];
            p[4 + r] = (2 * bb + 1 < NT) ? st[(2 * bb + 1 < NT) ? 2 * bb + 1 : 0][r] : 0.f;
        }
        pv_block(In{}, vt, p, o_acc, l_acc);
    }
}

// Work-group index -> (q-tile, image-head pair).  Pairs are taken in batches of `group` (a multiple
// of 8); inside a batch the order is q-tile-major:  bid = (batch*q_tiles + m_tile)*group + slot,
// pair = batch*group + slot.
//   * The hardware deals consecutive work-groups round-robin to the 8 XCDs (each with its own L2),
//     and group is a multiple of 8, so every q-tile of a pair lands on XCD slot%8 and re-reads that
//     pair's K/V through one L2.
//   * q-tile 0 of every pair of the batch is dispatched first.  The grid is sized by max_seqlen, an
//     upper bound; with ragged lengths most of the surplus tiles are the high ones, which then sit
//     at the end of the batch and retire while the real tiles are already running.
//   * group * q_tiles is about what the chip holds resident, so in the dense case the q-tiles of a
//     pair run together and their K/V re-reads hit L2 instead of going back to the fabric.
//
// A work-group has WAVES wavefronts of 16 queries each (q-tile = 16*WAVES rows).  K/V tiles of 64
// keys are double-buffered in LDS and the next tile's global loads are issued before the current
// tile is computed, so one barrier per tile suffices and the fabric latency of tile t+1 hides
// behind the arithmetic of tile t.  The lower half of the threads copies K, the upper half
// transposes V.
//
// GATHER = false: q, k, v, o are packed [T, H, D] and image i owns rows [cu[i], cu[i+1]).
// GATHER = true : q, k, v, o are padded [B, N, H, D]; the group first turns image i's keep mask
//   into the list of kept token positions (ballot + prefix over the group, in LDS) and then reads
//   and writes rows through that list, so pack and unpack need no launch of their own.  With
//   fill_mode 1 the q-tile-0 group of every (image, head) also zeroes that head's slice of the
//   dropped rows of o.
template <typename In, typename OutT, int WAVES, bool GATHER>
__global__ __launch_bounds__(kWaveSize * WAVES, 4)
void attn_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                 const uint16_t* __restrict__ v, OutT* __restrict__ o,
                 const int32_t* __restrict__ cu_seqlens, const uint8_t* __restrict__ keep, int n_tok,
                 int fill_mode, int H, int64_t tok, int64_t tok_o, int pairs, int q_tiles, int group,
                 float scale_log2e, int negate_q) {
    typedef typename In::vec8 vec8;
    constexpr int kBM = 16 * WAVES;                            // queries per work-group
    constexpr int kHalf = 32 * WAVES;                          // threads per fill role
    constexpr int kKLoads = 512 / kHalf;                       // 16-byte K units per K thread
    constexpr int kKeyStep = kHalf / 8;                        // keys between a K thread's units
    __shared__ __attribute__((aligned(16))) uint16_t k_lds[2][kBN * kLdsStride];
    __shared__ __attribute__((aligned(16))) uint16_t vt_lds[2][kHeadDim * kLdsStride];

    // bid = (batch * q_tiles + m_tile) * group + slot ; pair = batch * group + slot
    const int per_batch = q_tiles * group;
    const int batch = blockIdx.x / per_batch;
    const int in_batch = blockIdx.x - batch * per_batch;
    const int m_tile = in_batch / group;
    const int pair = batch * group + (in_batch - m_tile * group);
    if (pair >= pairs) return;
    const int h = pair % H;
    const int img = pair / H;
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = tid >> 6;
    const int col = lane & 15;                                 // query inside the wavefront's 16
    const int g = lane >> 4;                                   // lane group
    // tok / tok_o: elements between consecutive tokens of q, k, v / of o (H*64 when contiguous)
    const int64_t head_off = (int64_t)h * kHeadDim;
    const int m0 = m_tile * kBM;

    __shared__ uint16_t idx_lds[GATHER ? kMaxGatherTokens : 1];    // kept token positions, ascending
    __shared__ int wave_cnt[WAVES];
    int s, n;
    if (GATHER) {
        constexpr int kThreads = kWaveSize * WAVES;
        constexpr int kPre = 4;                                // mask bytes per thread requested up front
        const uint8_t* mask = keep + (int64_t)img * n_tok;
        s = img * n_tok;
        if (fill_mode == 1 && m_tile == 0) {                   // zero this head's slice of dropped rows
            constexpr int kChunks = kHeadDim * (int)sizeof(OutT) / 16;
            for (int t = tid / kChunks; t < n_tok; t += kThreads / kChunks)
                if (mask[t] == 0)
                    reinterpret_cast<uint4*>(o + (s + t) * tok_o + head_off)[tid % kChunks] = make_uint4(0, 0, 0, 0);
        }
        bool pre[kPre];
#pragma unroll
        for (int j = 0; j < kPre; ++j) {
            const int t = j * kThreads + tid;
            pre[j] = t < n_tok && mask[t] != 0;
        }
        n = 0;
        auto append = [&](bool kept, int t) {                  // every thread of the group calls this
            const uint64_t bits = __ballot(kept);
            if (lane == 0) wave_cnt[wave] = __popcll(bits);
            __syncthreads();
            int before = n, total = 0;
#pragma unroll
            for (int w2 = 0; w2 < WAVES; ++w2) {
                const int c = wave_cnt[w2];
                before += w2 < wave ? c : 0;
                total += c;
            }
            if (kept) idx_lds[before + __popcll(bits & ((1ull << lane) - 1ull))] = (uint16_t)t;
            n += total;
            __syncthreads();
        };
#pragma unroll
        for (int j = 0; j < kPre; ++j)
            if (j * kThreads < n_tok) append(pre[j], j * kThreads + tid);
        for (int base = kPre * kThreads; base < n_tok; base += kThreads) {
            const int t = base + tid;
            append(t < n_tok && mask[t] != 0, t);
        }
    } else {
        s = cu_seqlens[img];
        n = cu_seqlens[img + 1] - s;
    }
    if (m0 >= n) return;                                       // whole group exits together
    // row of the j-th token of this image in q / k / v / o
    auto row_of = [&](int j) -> int64_t { return GATHER ? (int64_t)s + idx_lds[j] : (int64_t)s + j; };
    const bool wave_active = m0 + wave * 16 < n;               // wavefront has at least one real query

    // ---- tile-fill roles
    const bool fills_k = tid < kHalf;
    const int fill = fills_k ? tid : tid - kHalf;
    // K thread: 16-byte units (key = fill/8 + kKeyStep*a, dims 8*(fill%8) ..)
    // V thread, WAVES == 4: keys 4*(fill/8)  .. +3, dims 8*(fill%8)  .. +7  (4 x 16-byte loads)
    //           WAVES == 8: keys 4*(fill/16) .. +3, dims 4*(fill%16) .. +3  (4 x  8-byte loads)
    // The key group of a V thread takes its bit 2 (which 16-key half of a 32-key block, i.e. which
    // 8-byte half of a 16-byte LDS unit) from lane bit 3, so that the 32 lanes of a half-wavefront
    // spread their 8-byte transposed writes evenly over all LDS banks.
    const int v_slot = (WAVES == 4) ? fill >> 3 : fill >> 4;   // 0..15
    const int v_kg = (v_slot & 8) | ((v_slot & 1) << 2) | ((v_slot >> 1) & 3);
    const int v_d0 = (WAVES == 4) ? 8 * (fill & 7) : 4 * (fill & 15);
    const uint16_t* fill_src = fills_k ? k + head_off + 8 * (fill & 7) : v + head_off + v_d0;
    const int fill_key0 = fills_k ? (fill >> 3) : 4 * v_kg;
    const int fill_dkey = fills_k ? kKeyStep : 1;
    // V thread's 4 keys occupy 4 consecutive kappa slots
    const int kappa = 32 * ((4 * v_kg) >> 5) + 8 * (((4 * v_kg) & 15) >> 2) + 4 * (((4 * v_kg) & 31) >> 4);

    constexpr int kLoads = 4;                                  // both roles issue <= 4 loads per tile
    uint4 raw[kLoads];
    auto prefetch = [&](int j0) {
        const int rem = n - j0;
#pragma unroll
        for (int a = 0; a < kLoads; ++a) {
            raw[a] = make_uint4(0, 0, 0, 0);                   // keys past n are zero in LDS
            if (fills_k && a >= kKLoads) continue;
            const int key = fill_key0 + fill_dkey * a;         // key of the tile this load fetches
            if (rem >= kBN || key < rem) {
                const uint16_t* src = fill_src + row_of(j0 + key) * tok;
                if (WAVES == 4 || fills_k) {
                    raw[a] = *reinterpret_cast<const uint4*>(src);
                } else {
                    const uint2 two = *reinterpret_cast<const uint2*>(src);
                    raw[a].x = two.x;
                    raw[a].y = two.y;
                }
            }
        }
    };
    auto stage = [&](int buf) {
        if (fills_k) {
#pragma unroll
            for (int a = 0; a < kKLoads; ++a)
                *reinterpret_cast<uint4*>(
                    &k_lds[buf][((fill >> 3) + kKeyStep * a) * kLdsStride + 8 * (fill & 7)]) = raw[a];
        } else {
            constexpr int kDims = (WAVES == 4) ? 8 : 4;        // head-dim elements this thread transposes
            const uint32_t w[4][4] = {{raw[0].x, raw[0].y, raw[0].z, raw[0].w},
                                      {raw[1].x, raw[1].y, raw[1].z, raw[1].w},
                                      {raw[2].x, raw[2].y, raw[2].z, raw[2].w},
                                      {raw[3].x, raw[3].y, raw[3].z, raw[3].w}};
#pragma unroll
            for (int e = 0; e < kDims; ++e) {
                const int d = v_d0 + e;
                const int rho = (d & 3) * 16 + (d >> 2);
                uint2 packed4;
                if (e & 1) {
                    packed4.x = (w[0][e >> 1] >> 16) | (w[1][e >> 1] & 0xffff0000u);
                    packed4.y = (w[2][e >> 1] >> 16) | (w[3][e >> 1] & 0xffff0000u);
                } else {
                    packed4.x = (w[0][e >> 1] & 0xffffu) | (w[1][e >> 1] << 16);
                    packed4.y = (w[2][e >> 1] & 0xffffu) | (w[3][e >> 1] << 16);
                }
                *reinterpret_cast<uint2*>(&vt_lds[buf][rho * kLdsStride + kappa]) = packed4;
            }
        }
    };

    prefetch(0);

    // ---- Q: this lane's query row, head-dim elements 16g .. 16g+15 (zeros past the sequence end)
    const int q_row = m0 + wave * 16 + col;
    uint4 q_raw[2] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
    if (q_row < n) {
        const uint4* src = reinterpret_cast<const uint4*>(q + row_of(q_row) * tok + head_off + 16 * g);
        q_raw[0] = src[0];
        q_raw[1] = src[1];
    }
    if (negate_q) {                                            // softmax(-|c| q.k) == softmax(|c| (-q).k)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            q_raw[e].x ^= 0x80008000u; q_raw[e].y ^= 0x80008000u;
            q_raw[e].z ^= 0x80008000u; q_raw[e].w ^= 0x80008000u;
        }
    }
    const vec8 q_frag[2] = {as_vec8<vec8>(q_raw[0]), as_vec8<vec8>(q_raw[1])};

    float m_run = -INFINITY;                                   // running max (log2 domain)
    f32x4 l_acc = f32x4{0.f, 0.f, 0.f, 0.f};                   // running row sum (every register equal)
    f32x4 o_acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) o_acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int tiles = (n + kBN - 1) / kBN;
    for (int t = 0; t < tiles; ++t) {
        const int buf = t & 1;
        stage(buf);                         // buffer `buf` was last read two tiles ago: see barrier below
        __syncthreads();                    // tile t visible; every wavefront is past tile t-1's reads
        if (t + 1 < tiles) prefetch((t + 1) * kBN);
        if (wave_active) {
            const int rem = n - t * kBN;
            const uint16_t* kt_ = k_lds[buf];
            const uint16_t* vt_ = vt_lds[buf];
            if (rem >= kBN) {
                tile_update<In, 4, false>(kt_, vt_, q_frag, rem, col, g, scale_log2e, m_run, l_acc, o_acc);
            } else {
                switch ((rem + 15) >> 4) {
                    case 1: tile_update<In, 1, true>(kt_, vt_, q_frag, rem, col, g, scale_log2e, m_run, l_acc, o_acc); break;
                    case 2: tile_update<In, 2, true>(kt_, vt_, q_frag, rem, col, g, scale_log2e, m_run, l_acc, o_acc); break;
                    case 3: tile_update<In, 3, true>(kt_, vt_, q_frag, rem, col, g, scale_log2e, m_run, l_acc, o_acc); break;
                    default: tile_update<In, 4, true>(kt_, vt_, q_frag, rem, col, g, scale_log2e, m_run, l_acc, o_acc); break;
                }
            }
        }
    }

    // ---- normalise and store: this lane owns d = 16g + 4r + dt of its query
    if (wave_active) {
        if (q_row < n) {
            const float inv = 1.0f / l_acc[0];
            float out16[16];
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 4; ++r) out16[4 * r + dt] = o_acc[dt][r] * inv;
            store16(o + row_of(q_row) * tok_o + head_off + 16 * g, out16);
        }
    }
}

template <typename In, typename OutT, bool GATHER>
hipError_t launch_typed(const void* q, const void* k, const void* v, void* o,
                        const int32_t* cu_seqlens, const uint8_t* keep, int n_tok, int fill_mode,
                        int B, int max_seqlen, int H, int64_t in_tok, int64_t out_tok, float scale,
                        hipStream_t stream) {
    constexpr int kWaves = 4;                                  // 64 query rows per work-group
    constexpr int kGroup = 512;                                // pairs per dispatch batch
    const int q_tiles = (max_seqlen + 16 * kWaves - 1) / (16 * kWaves);
    const int pairs = B * H;
    const int pairs8 = (pairs + kXcds - 1) / kXcds * kXcds;
    const int group = pairs8 < kGroup ? pairs8 : kGroup;
    const int batches = (pairs + group - 1) / group;
    hipLaunchKernelGGL((attn_kernel<In, OutT, kWaves, GATHER>), dim3(batches * q_tiles * group),
                       dim3(kWaveSize * kWaves), 0, stream,
                       static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k),
                       static_cast<const uint16_t*>(v), static_cast<OutT*>(o), cu_seqlens, keep, n_tok,
                       fill_mode, H, in_tok, out_tok, pairs, q_tiles, group, fabsf(scale) * kLog2e,
                       scale < 0.f ? 1 : 0);
    return hipGetLastError();
}

template <bool GATHER>
hipError_t launch_any(const void* q, const void* k, const void* v, void* o, const int32_t* cu_seqlens,
                      const uint8_t* keep, int n_tok, int fill_mode, int B, int max_seqlen, int H,
                      int64_t in_tok, int64_t out_tok, float scale, ragged_dtype in_dt,
                      ragged_dtype out_dt, hipStream_t stream) {
    if (in_dt == RAGGED_F16 && out_dt == RAGGED_F16)
        return launch_typed<F16, _Float16, GATHER>(q, k, v, o, cu_seqlens, keep, n_tok, fill_mode, B, max_seqlen, H, in_tok, out_tok, scale, stream);
    if (in_dt == RAGGED_F16 && out_dt == RAGGED_F32)
        return launch_typed<F16, float, GATHER>(q, k, v, o, cu_seqlens, keep, n_tok, fill_mode, B, max_seqlen, H, in_tok, out_tok, scale, stream);
    if (in_dt == RAGGED_BF16 && out_dt == RAGGED_BF16)
        return launch_typed<BF16, __bf16, GATHER>(q, k, v, o, cu_seqlens, keep, n_tok, fill_mode, B, max_seqlen, H, in_tok, out_tok, scale, stream);
    if (in_dt == RAGGED_BF16 && out_dt == RAGGED_F32)
        return launch_typed<BF16, float, GATHER>(q, k, v, o, cu_seqlens, keep, n_tok, fill_mode, B, max_seqlen, H, in_tok, out_tok, scale, stream);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_attn(const void* q, const void* k, const void* v, void* o,
                       const int32_t* cu_seqlens, int B, int max_seqlen, int H, int64_t in_tok,
                       int64_t out_tok, float scale, ragged_dtype in_dt, ragged_dtype out_dt,
                       hipStream_t stream) {
    return launch_any<false>(q, k, v, o, cu_seqlens, nullptr, 0, 0, B, max_seqlen, H, in_tok, out_tok, scale,
                             in_dt, out_dt, stream);
}

int attn_padded_max_tokens() { return kMaxGatherTokens; }

hipError_t launch_attn_padded(const void* q, const void* k, const void* v, void* o, const uint8_t* keep,
                              int B, int N, int H, float scale, ragged_dtype in_dt, ragged_dtype out_dt,
                              int fill_mode, hipStream_t stream) {
    const int64_t tok = (int64_t)H * kHeadDim;
    return launch_any<true>(q, k, v, o, nullptr, keep, N, fill_mode, B, N, H, tok, tok, scale, in_dt, out_dt,
                            stream);
}

}  // namespace ragged
