// Bidirectional multi-head attention over a packed ragged buffer (Section 4.2, Algorithm 1), for
// gfx950: one launch, one work-group per (image, head, 64-query tile), K/V tiles streamed through a
// ring of LDS buffers by direct global->LDS loads, MFMA 16x16x32 for both contractions with fp32
// accumulation, fp32 online softmax.  Small launches take a second form of the same kernel (SPLIT:
// 16-query work-groups whose wavefronts split the keys; described at the kernel).
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
// row/column an MFMA row/column stands for is free as long as loads and stores agree.
//
// Data movement.  A K or V tile is 64 rows of 128 bytes, kept ROW-MAJOR in LDS exactly as the
// hardware's global->LDS load writes it: one wavefront instruction moves 64 x 16 bytes and lane i's
// bytes land at (wave-uniform base) + 16*i, with no register staging and no VALU work.  Which global
// 16-byte chunk a lane fetches is free, and is used to swizzle: row r keeps chunk c at position
// c ^ ((r>>1)&3).  With that
//   * the A operand of S^T (lane: key l%16, head-dim chunk 2*(l/16)+ks) is one conflict-free
//     16-byte LDS read;
//   * the A operand of O^T needs V transposed (for one head-dim element, 8 keys): the transposing
//     LDS read (ds_read_b64_tr_b16: inside a 16-lane group, lane l receives element l%4 of the four
//     values read by lanes 4e + l/4, e = 0..3) delivers it from the row-major tile.  Lane sigma of
//     group g reads key 4g + sigma/4 (+16 for the second half of a 32-key block), head-dim elements
//     16*(sigma%4) + 4*dt .. +3, so lane l's MFMA row stands for element 16*(l%16/4) + 4*dt + l%4 and
//     each lane ends up owning output elements 16g .. 16g+15 of its query (32 contiguous bytes).
// Loads of tile t+kRing-1 are issued while tile t is computed (ring of kRing tiles); completion is
// tracked with the vector-memory counter, one barrier per tile.  Measured: a ring of two (four
// work-groups per CU) beats deeper rings, which cost resident wavefronts.
//
// bf16 inputs: Q K^T uses the bf16 MFMA (products are exact in fp32).  A bf16 probability would
// carry only 8 significant bits, so P is split as P = P_hi + P_lo (two bf16 values, 16 bits
// together) and P V is two MFMAs; V stays exact.  The path is not MFMA-bound at ViT lengths.
#include <type_traits>

#include "common.h"
#include "mask_prefix.h"
#include "mfma_lds.h"

namespace ragged {
namespace {

constexpr int kHeadDim = 64;
constexpr int kBN = 64;                 // keys per K/V tile
// Work-group shape.  Measured on the dense layer (B=64, n=197) and the pruned batches: four
// wavefronts with a ring of two tiles (32 KB, four work-groups per CU) is the fastest; deeper rings
// (3, 4) lose resident wavefronts and gain nothing, eight-wavefront groups with rings of 2..4 tie
// on dense batches and lose on short sequences.
constexpr int kRing = 2;                // K/V tiles resident in LDS per work-group (2..4)
constexpr int kAttnWaves = 4;           // wavefronts per work-group: 4 or 8 (the key-split and single-launch forms need 4)
constexpr int kAttnThreads = kWaveSize * kAttnWaves;
constexpr int kAttnOcc = kAttnWaves == 8 ? 2 : (kRing == 2 ? 4 : (kRing == 3 ? 3 : 2));  // work-groups per CU aimed at
constexpr int kTileBytes = kBN * kHeadDim * 2;   // one K or one V tile: 8 KB
// A sequence's LAST tile takes a tail of up to 16 keys along (n = 64k + 1 .. 64k + 16, k >= 2): 80 keys in one
// pass instead of a pass of its own for a handful of keys -- ViT lengths are 64k + 1 before pruning (197, 577).
// (Not for k = 1: the first tile of a sequence has a form of its own, and a second copy of it for 80 keys
// costs the short launches more in code than the few sequences of 65..80 tokens gain.)
// The tail's K rows and V rows live behind the ring.
constexpr int kExtraRows = 16;
constexpr int kExtraBytes = 2 * kExtraRows * kHeadDim * 2;   // K rows, then V rows: 4 KB
constexpr bool kExtTail = kRing == 2;            // (the load bookkeeping of deeper rings does not count the tail's loads)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazyLog2 = 8.0f;       // probabilities stay below 2^8 between rescales
constexpr int kSplitMaxGroups = 256;    // launches of at most this many 64-row q-tiles split the keys over the wavefronts
constexpr int kMaxGatherTokens = 1536;  // tokens per image the gather-on-load variant can index in LDS
constexpr int kMaxGridYZ = 65535;       // HIP's limit on the second and third grid dimension

// O^T += V^T P^T for one 32-key block: p[0..7] are this lane's probabilities (fp32).  The row sums
// of P ride along on the matrix core: with an all-ones A operand every row of the result holds
// sum_k P[k][query], already reduced over the four lane groups, and it is the sum of exactly the
// rounded probabilities that multiply V.
// START: the accumulators hold nothing yet (first block of a sequence's first tile): they are written, not
// read, so they need no zero-initialisation (the MFMA takes a constant zero as its C operand).
template <bool START>
__device__ __forceinline__ void pv_block(F16, const uint4 (&vt)[4], const float (&p)[8], f32x4 (&o)[4],
                                         f32x4& l) {
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f16x8 pb, ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) { pb[e] = (_Float16)p[e]; ones[e] = (_Float16)1.0f; }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) o[dt] = F16::mfma(as_vec8<f16x8>(vt[dt]), pb, START ? zero : o[dt]);
    l = F16::mfma(ones, pb, START ? zero : l);
}
template <bool START>
__device__ __forceinline__ void pv_block(BF16, const uint4 (&vt)[4], const float (&p)[8], f32x4 (&o)[4],
                                         f32x4& l) {
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    bf16x8 hi, lo, ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        hi[e] = (__bf16)p[e];
        lo[e] = (__bf16)(p[e] - (float)hi[e]);
        ones[e] = (__bf16)1.0f;
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        o[dt] = BF16::mfma(as_vec8<bf16x8>(vt[dt]), hi, START ? zero : o[dt]);
        o[dt] = BF16::mfma(as_vec8<bf16x8>(vt[dt]), lo, o[dt]);
    }
    l = BF16::mfma(ones, hi, START ? zero : l);
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

// Store 4 consecutive head-dim elements of one output row.
__device__ __forceinline__ void store4(_Float16* dst, const float (&v)[4]) {
    typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
    const f16x4 a = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
    *reinterpret_cast<uint2*>(dst) = __builtin_bit_cast(uint2, a);
}
__device__ __forceinline__ void store4(__bf16* dst, const float (&v)[4]) {
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    const bf16x4 a = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
    *reinterpret_cast<uint2*>(dst) = __builtin_bit_cast(uint2, a);
}
__device__ __forceinline__ void store4(float* dst, const float (&v)[4]) {
    *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
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
// update, O^T += V^T P^T.  NT = 16-key subtiles present in the tile (1..4, or 5: a full tile plus the tail
// subtile kept behind the ring, whose K / transposed V operand addresses are ek_a0 / ev_a0 -- the second
// k-step / head-dim pair is at the address xor 16, as for the tile itself); MASK: the last subtile may
// hold keys past the end of the sequence (index >= rem), which are masked out (their LDS rows hold
// a copy of the last real row, so they are finite wherever the inputs are).
// k_a0/k_a1: this lane's LDS byte addresses of its K operand for the two 32-element k-steps of
// subtile 0; v_a0/v_a1: of its transposed V read for head-dim blocks dt = 0,1 / 2,3 of key block 0.
// scale_log2e >= 0 here (a negative softmax scale is folded into the sign of Q by the caller), so
// the row maximum can be taken on the raw scores and the scale fused into the exponent's FMA.
// FIRST: the sequence's first tile.  The running maximum is this tile's maximum and the accumulators are
// written, not updated: no rescaling, no zero-initialised registers.  (The general form would reach the same
// values through alpha = exp2(-inf) = 0 and accumulators cleared beforehand.)
template <typename In, int NT, bool MASK, bool FIRST>
__device__ __forceinline__ void tile_update(uint32_t k_a0, uint32_t k_a1, uint32_t v_a0, uint32_t v_a1,
                                            uint32_t ek_a0, uint32_t ev_a0,
                                            const typename In::vec8 (&q_frag)[2], int rem, int g,
                                            float scale_log2e, float& m_run, f32x4& l_acc,
                                            f32x4 (&o_acc)[4]) {
    typedef typename In::vec8 vec8;
    // -------- S^T = K Q^T : NT 16-key subtiles, two k-steps of 32 head-dim elements
    f32x4 st[NT];
#pragma unroll
    for (int kt = 0; kt < NT; ++kt) {
        const uint4 a0 = lds_read16(kt == 4 ? ek_a0 : k_a0 + kt * 16 * 128);
        const uint4 a1 = lds_read16(kt == 4 ? ek_a0 ^ 16u : k_a1 + kt * 16 * 128);
        st[kt] = In::mfma(as_vec8<vec8>(a0), q_frag[0], f32x4{0.f, 0.f, 0.f, 0.f});
        st[kt] = In::mfma(as_vec8<vec8>(a1), q_frag[1], st[kt]);
    }
    // -------- online softmax (this lane: one query, keys 16*kt + 4*g + r of the tile)
    const int last_valid = rem - 16 * (NT - 1) - 4 * g;        // r < last_valid is a real key (last subtile)
    float t_max = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NT; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            t_max = fmaxf(t_max, (!MASK || kt < NT - 1 || r < last_valid) ? st[kt][r] : -INFINITY);
    // Lazy rescaling: the reference maximum m_run only moves when some query's tile maximum exceeds
    // it by more than 2^kLazyLog2 (always on the first tile, where m_run = -inf).  Until then
    // probabilities may reach 2^kLazyLog2 instead of 1 -- harmless in fp16/bf16/fp32 -- and the
    // accumulators need no per-tile multiply.  The result is the same softmax: m_run cancels.
    // The test is made on each lane's own maximum (a query's four lanes share m_run, so some lane
    // passes it exactly when the query's maximum does); the cross-lane reduction is only paid when
    // the reference really moves.
    if (FIRST) {
        m_run = quad_max(t_max) * scale_log2e;                  // finite: the tile has a valid key
    } else if (__builtin_amdgcn_ballot_w64(t_max * scale_log2e > m_run + kLazyLog2) != 0) {   // wavefront-uniform
        t_max = quad_max(t_max) * scale_log2e;
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
    // -------- O^T += V^T P^T : 32-key blocks x four 16-row head-dim tiles (NT 1 or 3: zero upper half)
    constexpr int kBlocks = NT == 5 ? 2 : (NT + 1) / 2;
#pragma unroll
    for (int bb = 0; bb < kBlocks; ++bb) {
        uint4 vt[4];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const uint32_t a = ((dt & 2) ? v_a1 : v_a0) + 8 * (dt & 1) + bb * 32 * 128;
            const short4v lo = lds_read_tr(a);                  // keys 32bb      + 4g + 0..3
            const short4v hi = lds_read_tr(a + 16 * 128);       // keys 32bb + 16 + 4g + 0..3
            const uint2 lo2 = __builtin_bit_cast(uint2, lo), hi2 = __builtin_bit_cast(uint2, hi);
            vt[dt] = make_uint4(lo2.x, lo2.y, hi2.x, hi2.y);
        }
        float p[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p[r] = st[2 * bb][r];
            p[4 + r] = (2 * bb + 1 < NT) ? st[(2 * bb + 1 < NT) ? 2 * bb + 1 : 0][r] : 0.f;
        }
        if (FIRST && bb == 0) pv_block<true>(In{}, vt, p, o_acc, l_acc);
        else pv_block<false>(In{}, vt, p, o_acc, l_acc);
    }
    if (NT == 5) {
        // the tail subtile: 16 keys in the lower half of a 32-key block whose upper half is zero on both sides
        // (no rows are read for it)
        uint4 vt[4];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const uint2 lo2 = __builtin_bit_cast(uint2, lds_read_tr(((dt & 2) ? ev_a0 ^ 16u : ev_a0) + 8 * (dt & 1)));
            vt[dt] = make_uint4(lo2.x, lo2.y, 0u, 0u);
        }
        const float p[8] = {st[NT - 1][0], st[NT - 1][1], st[NT - 1][2], st[NT - 1][3], 0.f, 0.f, 0.f, 0.f};
        pv_block<false>(In{}, vt, p, o_acc, l_acc);
    }
}

// A tile of `rem` remaining keys at LDS address tile0: full tiles take the unmasked form, a tail is specialised
// on its number of 16-key subtiles.  k_rel0 / v_rel0: this lane's operand offsets inside a tile; ext_tile: a last
// tile of 65..80 keys whose rows 64.. are kept behind the ring at LDS address extra0 (EXT: the kernel form has them).
template <typename In, bool FIRST, bool EXT>
__device__ __forceinline__ void tile_any(int rem, bool ext_tile, uint32_t tile0, uint32_t extra0, uint32_t k_rel0, uint32_t v_rel0,
                                         const typename In::vec8 (&q_frag)[2], int g, float scale_log2e,
                                         float& m_run, f32x4& l_acc, f32x4 (&o_acc)[4]) {
    const uint32_t k_a0 = tile0 + k_rel0, k_a1 = tile0 + (k_rel0 ^ 16u);
    const uint32_t v_a0 = tile0 + v_rel0, v_a1 = tile0 + (v_rel0 ^ 16u);
    const uint32_t ek_a0 = extra0 + k_rel0, ev_a0 = extra0 + kExtraBytes / 2 + (v_rel0 - kTileBytes);
    if (EXT && ext_tile) {
        tile_update<In, 5, true, FIRST>(k_a0, k_a1, v_a0, v_a1, ek_a0, ev_a0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc);
    } else if (rem >= kBN) {
        tile_update<In, 4, false, FIRST>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc);
    } else {
        switch ((rem + 15) >> 4) {
            case 1: tile_update<In, 1, true, FIRST>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc); break;
            case 2: tile_update<In, 2, true, FIRST>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc); break;
            case 3: tile_update<In, 3, true, FIRST>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc); break;
            default: tile_update<In, 4, true, FIRST>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc); break;
        }
    }
}

// Work-group -> (q-tile, image-head pair).  Pairs are taken in batches of `group` (a multiple of 8);
// inside a batch the order is q-tile-major: the grid is (group, q_tiles, batches), dispatched
// x-fastest, so work-group (slot, m_tile, batch) is number (batch*q_tiles + m_tile)*group + slot in
// dispatch order and handles pair = batch*group + slot.
//   * The hardware deals consecutive work-groups round-robin to the 8 XCDs (each with its own L2),
//     and group is a multiple of 8, so every q-tile of a pair lands on XCD slot%8 and re-reads that
//     pair's K/V through one L2.
//   * q-tile 0 of every pair of the batch is dispatched first.  The grid is sized by max_seqlen, an
//     upper bound; with ragged lengths most of the surplus tiles are the high ones, which then sit
//     at the end of the batch and retire while the real tiles are already running.
//   * group * q_tiles is about what the chip holds resident, so in the dense case the q-tiles of a
//     pair run together and their K/V re-reads hit L2 instead of going back to the fabric.
//
// A work-group has four wavefronts of 16 queries each.  Wavefront w issues the loads of rows
// 16w .. 16w+15 of every K and V tile (four instructions per tile); rows past the end of the
// sequence fetch the last real row instead, and a wavefront whose rows lie beyond the 32-key blocks
// the tile's arithmetic touches issues nothing.
//
// MODE kPacked: q, k, v, o are packed [T, H, D] and image i owns rows [cu[i], cu[i+1]).
// MODE kPadded: q, k, v, o are padded [B, N, H, D]; the group first turns image i's keep mask
//   into the list of kept token positions (ballot + prefix over the group, in LDS) and then reads
//   and writes rows through that list, so pack and unpack need no launch of their own.  With
//   fill_mode 1 the groups of every (image, head) also zero that head's slice of the dropped rows
//   of o, a share each.
// MODE kStep  : the whole pack -> attention -> unpack step in this one launch.  q, k, v, o are
//   packed as in kPacked, but the image's first row s is recounted from the keep mask (nonzero
//   bytes before the image) and the kept-position list is built as in kPadded.  Besides its
//   attention rows the group (image, head, q-tile) moves that head's 128-byte slice of its 64 rows
//   from x to the packed buffer and writes each output row twice: to o (packed) and to its padded
//   position in `out`.  Head-0 groups also write gather_idx, and q-tile 0 of head 0 writes
//   cu_seqlens.  Every group derives s and the list itself, so no group waits for another.
enum { kPacked = 0, kPadded = 1, kStep = 2 };

// Extra operands of MODE kStep (null / zero otherwise).
struct StepArgs {
    const uint16_t* x;          // [B, N, C] padded features
    uint16_t* packed;           // [cap_rows, C]
    uint16_t* out;              // [B, N, C]
    int32_t* cu_seqlens;        // [B + 1]
    int32_t* gather_idx;        // [cap_rows]
    int64_t cap_rows;
    int32_t* flags;             // MODE kPacked only, may be null: bit 0 is set when some n_i > max_seqlen
    int max_seqlen;
};

// SPLIT (small launches, where a work-group has a CU to itself and the path is a chain of latencies):
//   the work-group takes only 16 queries and its four wavefronts split the KEYS instead -- wavefront w
//   loads K/V tiles w, w+4, ... into a slot of its own (no barrier in the loop) and runs the same tile
//   arithmetic on them; the four partial results (running maximum, row sum, accumulators) are merged
//   through LDS at the end, each wavefront finishing four of the sixteen head-dim elements a lane owns.
//   A sequence of up to 256 tokens then costs one tile time plus the merge instead of up to four.
template <typename In, typename OutT, int MODE, bool SPLIT>
__global__ __launch_bounds__(kAttnThreads, SPLIT ? 2 : (kAttnOcc < 1 ? 1 : kAttnOcc))
void attn_kernel(const void* __restrict__ index, int n_tok, int fill_mode, int H, uint32_t h_magic, int pairs,
                 int group, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, int tok32,
                 int tok_o32, const uint16_t* __restrict__ q, OutT* __restrict__ o, float scale_log2e,
                 int negate_q, StepArgs step) {
    // The parameters are ordered by when the kernel needs them: the first 14 dwords (up to tok_o32) are
    // delivered in scalar registers with the wavefront (kernel-argument preload), the rest is fetched while
    // the first memory round trip is under way.
    const int32_t* const cu_seqlens = static_cast<const int32_t*>(index);      // MODE kPacked
    const uint8_t* const keep = static_cast<const uint8_t*>(index);            // the modes that read a keep mask
    const int64_t tok = tok32, tok_o = tok_o32;
    typedef typename In::vec8 vec8;
    constexpr bool GATHER = MODE == kPadded;                   // q, k, v, o rows addressed through the kept list
    constexpr bool LIST = MODE != kPacked;                     // the kept list is built from the mask
    static_assert(MODE != kStep || (kAttnThreads == kBlockThreads && kAttnWaves == 4),
                  "the mask prefix count and the x copy of kStep assume 256 threads and 64-row q-tiles");
    static_assert(!SPLIT || kAttnWaves == 4, "the merge of the key-split form gives each of four wavefronts four elements");
    constexpr int WAVES = kAttnWaves;
    constexpr int kI = 8 / WAVES;                              // load instructions per wavefront per K (or V) tile
    constexpr int kPer = 2 * kI;                               // ... per K+V tile
    constexpr int kBM = SPLIT ? 16 : 16 * WAVES;               // queries per work-group
    constexpr bool EXT = kExtTail && !SPLIT;                   // a last tile may take a tail of <= 16 keys along
    constexpr int kRingBytes = (SPLIT ? WAVES : kRing) * 2 * kTileBytes;
    __shared__ __attribute__((aligned(1024))) uint4 ring[(kRingBytes + (EXT ? kExtraBytes : 0)) / 16];   // [slot][K|V], tail rows

    // grid (group, q_tiles, batches): work-groups are dispatched x-fastest, i.e. in the order
    // (batch * q_tiles + m_tile) * group + slot of the mapping described above, with no division to undo it
    const int m_tile = blockIdx.y;
    const int pair = blockIdx.z * group + blockIdx.x;
    if (pair >= pairs) return;
    uint32_t img_u, h_u;
    divmod((uint32_t)pair, (uint32_t)H, h_magic, img_u, h_u);
    const int img = (int)img_u, h = (int)h_u;
    const int tid = threadIdx.x;
    const int lane = tid & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15;                                 // query inside the wavefront's 16
    const int g = lane >> 4;                                   // lane group
    // tok / tok_o: elements between consecutive tokens of q, k, v / of o (H*64 when contiguous)
    const int64_t head_off = (int64_t)h * kHeadDim;
    const int m0 = m_tile * kBM;

    __shared__ uint16_t idx_lds[LIST ? kMaxGatherTokens : 1];      // kept token positions, ascending
    constexpr int kRounds = kMaxGatherTokens / kAttnThreads;       // mask bytes per thread: all requested up front
    __shared__ int wave_cnt[LIST ? kRounds * WAVES : 1];
    __shared__ uint64_t keep_bits[LIST ? kRounds * WAVES : 1];     // fill_mode 1: keep bits of tokens 64e .. 64e+63 in entry e
    __shared__ int lds4[4];
    int s, n;
    if (LIST) {
        constexpr int kThreads = kAttnThreads;
        static_assert(kRounds * kThreads == kMaxGatherTokens, "the mask of an image is read in whole rounds of the group");
        const uint8_t* mask = keep + (int64_t)img * n_tok;
        s = img * n_tok;
        PrefixLoads before_image;
        if (MODE == kStep) before_image = prefix_issue(keep, img * n_tok);   // requested with the image's own mask
        // the image's own mask bytes: every round requested before any is looked at (clamped loads, see
        // load_byte_clamped), so the mask and the prefix words cost ONE memory round trip together
        uint8_t raw[kRounds];
#pragma unroll
        for (int j = 0; j < kRounds; ++j) raw[j] = load_byte_clamped(mask, j * kThreads + tid, n_tok);
        // Count first (one barrier): a group learns the image's length n before anything else is built, and
        // the groups of the upper-bound grid that have no rows leave here.
        // fill_mode 1: the groups of an (image, head) share the zeroing of the head's slice of the dropped rows --
        // group m takes every q_tiles-th pass of the group over the tokens, the groups without rows of their own
        // (most of them, when much is pruned) included, before they leave
        const bool zero_fill = fill_mode == 1;
        const int fill_groups = (int)gridDim.y;
        // kStep, q-tile 0 (with short sequences: the groups that have rows): the count of the kept tokens in front of
        // the image shares the barrier of the length count, so the group knows s and n together.  The other q-tiles
        // count it after the test that lets most of them leave.
        const bool early_s = MODE == kStep && m_tile == 0;
        if (early_s) prefix_post(prefix_count_thread(keep, before_image), lds4);
        // Every mask byte counts as used here, also those of rounds beyond n_tok: a load that the compiler still
        // believes in flight makes it wait for ALL memory traffic (K/V and Q rows by then) before the register is
        // reused further down.
#pragma unroll
        for (int j = 0; j < kRounds; ++j) asm volatile("" : : "v"((uint32_t)raw[j]));
        // (the loops over the rounds leave at the first round beyond n_tok: one scalar branch instead of a
        // skipped block per round -- a taken branch costs a lone wavefront as much as half a dozen instructions)
        uint64_t bits[kRounds];
#pragma unroll
        for (int j = 0; j < kRounds; ++j) {
            if (j * kThreads >= n_tok) break;                  // group-uniform
            bits[j] = __ballot(j * kThreads + tid < n_tok && raw[j] != 0);
            if (lane == 0) {
                wave_cnt[j * WAVES + wave] = __popcll(bits[j]);
                if (zero_fill) keep_bits[j * WAVES + wave] = bits[j];
            }
        }
        __syncthreads();
        n = 0;
        int before[kRounds];                                   // kept tokens in front of this wavefront's 64 of round j
#pragma unroll
        for (int j = 0; j < kRounds; ++j) {
            if (j * kThreads >= n_tok) break;
            before[j] = n;
#pragma unroll
            for (int w2 = 0; w2 < WAVES; ++w2) {
                const int c = wave_cnt[j * WAVES + w2];
                before[j] += w2 < wave ? c : 0;
                n += c;
            }
        }
        if (zero_fill) {                                       // token t's keep bit: entry t / 64, bit t % 64
            if (MODE == kStep) {
                for (int t = tid / 8 + m_tile * (kThreads / 8); t < n_tok; t += fill_groups * (kThreads / 8))
                    if (((keep_bits[t >> 6] >> (t & 63)) & 1ull) == 0)
                        reinterpret_cast<uint4*>(step.out + (int64_t)(s + t) * tok_o + head_off)[tid % 8] =
                            make_uint4(0, 0, 0, 0);
            } else {
                constexpr int kChunks = kHeadDim * (int)sizeof(OutT) / 16;
                for (int t = tid / kChunks + m_tile * (kThreads / kChunks); t < n_tok; t += fill_groups * (kThreads / kChunks))
                    if (((keep_bits[t >> 6] >> (t & 63)) & 1ull) == 0)
                        reinterpret_cast<uint4*>(o + (s + t) * tok_o + head_off)[tid % kChunks] = make_uint4(0, 0, 0, 0);
            }
        }
        n = __builtin_amdgcn_readfirstlane(n);
        // a group with no rows that does not write cu_seqlens either is done (whole group, before any further barrier)
        if (m0 >= n && !(MODE == kStep && h == 0 && m_tile == 0)) return;
#pragma unroll
        for (int j = 0; j < kRounds; ++j) {
            if (j * kThreads >= n_tok) break;
            if (((bits[j] >> lane) & 1ull) != 0)
                idx_lds[before[j] + __popcll(bits[j] & ((1ull << lane) - 1ull))] = (uint16_t)(j * kThreads + tid);
        }
        if (MODE == kStep) {
            // kept tokens of the images before this one; q-tile 0 publishes idx_lds with a barrier further down, once
            // its K/V and Q rows (which need s, not the list) are requested; for the others this barrier does
            s = early_s ? prefix_total(lds4) : prefix_finish(keep, before_image, lds4);
            s = __builtin_amdgcn_readfirstlane(s);
            if (h == 0 && m_tile == 0 && tid == 0) {
                if (img == 0) step.cu_seqlens[0] = 0;
                step.cu_seqlens[img + 1] = s + n;
            }
        } else {
            __syncthreads();                                   // idx_lds complete
        }
    } else {
        s = cu_seqlens[img];
        n = cu_seqlens[img + 1] - s;
        // the caller's bound was too small for this image: say so (one group per image; a vector atomic)
        if (step.flags != nullptr && h == 0 && m_tile == 0 && tid == 0 && n > step.max_seqlen)
            atomicOr(step.flags, RAGGED_FLAG_SEQLEN_EXCEEDED);
    }
    n = __builtin_amdgcn_readfirstlane(n);
    if (m0 >= n) return;                                       // whole group exits together
    const int64_t pad0 = (int64_t)img * n_tok;                 // first padded row of the image (kStep)
    // row of the j-th token of this image in q / k / v / o
    auto row_of = [&](int j) -> int64_t { return GATHER ? (int64_t)s + idx_lds[j] : (int64_t)s + j; };
    const int q_row = m0 + (SPLIT ? 0 : wave * 16) + col;      // this lane's query inside the image
    const bool wave_active = SPLIT || m0 + wave * 16 < n;      // wavefront has at least one real query

    // ---- K/V tile loads.  Instruction i (0, 1) of this wavefront covers tile rows 16*wave + 8i + lane/8;
    // the lane's LDS slot is position lane%8 of that row, which holds chunk (lane%8) ^ ((row>>1)&3).
    const uint32_t ring0 = (uint32_t)reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) void*)ring);
    const uint32_t extra0 = ring0 + kRingBytes;                // the tail rows of a last tile (EXT)
    const uint32_t tok_bytes = (uint32_t)tok * 2u;
    const int load_key = 8 * kI * wave + (lane >> 3);          // + 8i
    const uint32_t load_chunk = 16u * ((lane & 7) ^ ((lane >> 4) & 3));
    const uint16_t* k_base = k + (int64_t)s * tok + head_off;   // wave-uniform
    const uint16_t* v_base = v + (int64_t)s * tok + head_off;
    // tiles of 64 keys; a tail of 1 .. 16 keys behind at least two full tiles rides along with the last one (EXT)
    // (unsigned arithmetic and a select: no branch on the way to the first loads)
    const unsigned tail_keys = (unsigned)n & (kBN - 1);
    const bool rides = EXT && n > 2 * kBN && tail_keys - 1u < (unsigned)kExtraRows;
    const int tiles = (int)(((unsigned)n + kBN - 1) / kBN) - (rides ? 1 : 0);
    const int ride_tile = rides ? tiles - 1 : -1;              // the tile that takes the tail along, if any
    // Returns the number of load instructions issued (0 or kPer).  The per-lane offset is 32 bits wide:
    // packed rows are addressed relative to the tile's first row (the 64-bit part is wave-uniform),
    // gathered rows relative to the image's first token (the host checks that N tokens fit).
    auto issue = [&](int t, int slot, bool may_ride = true) -> int {
        const int rem = n - t * kBN;
        const int need_rows = rem >= kBN ? kBN : 32 * ((rem + 31) >> 5);   // rows the tile's MFMAs touch
        if (8 * kI * wave >= need_rows) return 0;
        const uint32_t dst = ring0 + slot * 2 * kTileBytes + wave * (1024 * kI);
        const int64_t tile_off = GATHER ? 0 : (int64_t)t * kBN * tok;
#pragma unroll
        for (int i = 0; i < kI; ++i) {
            int rel = load_key + 8 * i;
            rel = rel < rem ? rel : rem - 1;                    // past the end: the last real row again
            const uint32_t row = GATHER ? (uint32_t)idx_lds[t * kBN + rel] : (uint32_t)rel;
            const uint32_t voff = row * tok_bytes + load_chunk;
            dma16(dst + i * 1024, voff, k_base + tile_off);
            dma16(dst + i * 1024 + kTileBytes, voff, v_base + tile_off);
        }
        if (__builtin_expect(may_ride && t == ride_tile && wave < kExtraRows / 8, 0)) {
            // the tail rows 64 .. 79 of a last tile: eight rows per instruction, wavefronts 0 and 1
            int rel = kBN + 8 * wave + (lane >> 3);
            rel = rel < rem ? rel : rem - 1;
            const uint32_t row = GATHER ? (uint32_t)idx_lds[t * kBN + rel] : (uint32_t)rel;
            const uint32_t voff = row * tok_bytes + load_chunk;
            dma16(extra0 + wave * 1024, voff, k_base + tile_off);
            dma16(extra0 + wave * 1024 + kExtraBytes / 2, voff, v_base + tile_off);
        }
        return kPer;
    };

    // SPLIT: the whole tile t into this wavefront's own slot (eight instructions per operand)
    auto issue_own = [&](int t) {
        const int rem = n - t * kBN;
        const int need_rows = rem >= kBN ? kBN : 32 * ((rem + 31) >> 5);
        const uint32_t dst = ring0 + wave * 2 * kTileBytes;
        const int64_t tile_off = GATHER ? 0 : (int64_t)t * kBN * tok;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (8 * i < need_rows) {                            // wave-uniform
                int rel = 8 * i + (lane >> 3);
                rel = rel < rem ? rel : rem - 1;
                const uint32_t row = GATHER ? (uint32_t)idx_lds[t * kBN + rel] : (uint32_t)rel;
                const uint32_t voff = row * tok_bytes + load_chunk;
                dma16(dst + i * 1024, voff, k_base + tile_off);
                dma16(dst + i * 1024 + kTileBytes, voff, v_base + tile_off);
            }
        }
    };

    // c_next[d] = load instructions this wavefront has in flight for tile t+1+d (prologue: tiles 1 .. kRing-2)
    int c_next[kRing > 2 ? kRing - 2 : 1] = {0};
    if (SPLIT) {
        if (wave < tiles) issue_own(wave);
    } else {
        issue(0, 0, false);                                    // (a tile that takes a tail along is never the first)
#pragma unroll
        for (int d = 0; d < kRing - 2; ++d) c_next[d] = d + 1 < tiles ? issue(d + 1, d + 1) : 0;
    }

    // ---- Q: this lane's query row, head-dim elements 16g .. 16g+15 (zeros past the sequence end)
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

    // ---- kStep: this head's slice of the group's 64 rows of x (two 16-byte units per thread) is requested
    // now and stored to the packed buffer after the first tile; head 0 also records the source rows
    uint4 x_raw[2] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
    if (MODE == kStep) {
        if (m_tile == 0) __syncthreads();                      // idx_lds complete (see the prefix count above)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = m0 + 32 * i + (tid >> 3);
            if ((!SPLIT || 32 * i + (tid >> 3) < kBM) && j < n)
                x_raw[i] = reinterpret_cast<const uint4*>(step.x + (pad0 + idx_lds[j]) * tok + head_off)[tid & 7];
        }
        if (h == 0 && tid < kBM && m0 + tid < n && (int64_t)s + m0 + tid < step.cap_rows)
            step.gather_idx[s + m0 + tid] = (int32_t)(pad0 + idx_lds[m0 + tid]);
    }

    // ---- LDS read addresses of this lane inside a tile (see the header comment)
    //   K operand: row col (+16kt), chunk 2g + ks at position (2g + ks) ^ ((col>>1)&3)
    const uint32_t k_rel0 = col * 128 + 16 * ((2 * g) ^ ((col >> 1) & 3));
    //   V transposed read: row 4g + sigma/4 (+32bb, +16), chunk 2*(sigma%4) + (dt>>1), half dt&1
    const int sigma = col;
    const int v_row = 4 * g + (sigma >> 2);
    const uint32_t v_rel0 = v_row * 128 + 16 * ((2 * (sigma & 3)) ^ ((v_row >> 1) & 3)) + kTileBytes;

    // running maximum (log2 domain), row sum (every register equal) and output accumulators: written by the
    // sequence's first tile (tile_update<FIRST>), updated by the others
    // (the single-launch step keeps the general form for every tile: with the first tile peeled the compiler
    // settles on a schedule of that kernel that is 4 % slower on the headline batch)
    constexpr bool PEEL = MODE != kStep;
    float m_run;
    f32x4 l_acc;
    f32x4 o_acc[4];
    if (!PEEL) {
        m_run = -INFINITY;
        l_acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) o_acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // kStep: the x rows requested above go to the packed buffer
    auto store_packed_rows = [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int j = m0 + 32 * i + (tid >> 3);
            if ((!SPLIT || 32 * i + (tid >> 3) < kBM) && j < n && (int64_t)s + j < step.cap_rows)
                reinterpret_cast<uint4*>(step.packed + ((int64_t)s + j) * tok + head_off)[tid & 7] = x_raw[i];
        }
    };
    if (SPLIT) {
        // ---- this wavefront's tiles wave, wave + 4, ...: its own slot, its own loads, no barrier
        const uint32_t tile0 = ring0 + wave * 2 * kTileBytes;
        if (wave < tiles) {
            wait_vm<0>();                   // the tile has landed (the loads were this wavefront's own)
            // its results depend on every LDS read of the tile: the slot is free after it
            tile_any<In, PEEL, false>(n - wave * kBN, false, tile0, 0, k_rel0, v_rel0, q_frag, g, scale_log2e, m_run, l_acc, o_acc);
            for (int t = wave + WAVES; t < tiles; t += WAVES) {
                issue_own(t);
                wait_vm<0>();
                tile_any<In, false, false>(n - t * kBN, false, tile0, 0, k_rel0, v_rel0, q_frag, g, scale_log2e, m_run, l_acc, o_acc);
            }
        } else {                            // no tile for this wavefront: it contributes nothing to the merge
            m_run = -INFINITY;
            l_acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) o_acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        if (MODE == kStep) store_packed_rows();
        if (tiles == 1) {                   // a single tile: wavefront 0 holds the whole result, nothing to merge
            if (wave == 0 && q_row < n) {
                const bool row_fits = MODE != kStep || (int64_t)s + q_row < step.cap_rows;
                const float inv = 1.0f / l_acc[0];
                float out16[16];
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) out16[4 * dt + r] = o_acc[dt][r] * inv;
                if (row_fits) store16(o + row_of(q_row) * tok_o + head_off + 16 * g, out16);
                if (MODE == kStep)
                    store16(reinterpret_cast<OutT*>(step.out) + (pad0 + idx_lds[q_row]) * tok_o + head_off + 16 * g, out16);
            }
            return;
        }
        // ---- merge the four partial results: part[j][lane], j = 0: running maximum, 1: row sum, 2 + 4dt + r: accumulators
        float* const part = reinterpret_cast<float*>(ring) + wave * (2 * kTileBytes / 4);
        part[lane] = m_run;
        part[kWaveSize + lane] = l_acc[0];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) part[(2 + 4 * dt + r) * kWaveSize + lane] = o_acc[dt][r];
        __syncthreads();                    // (a wavefront without tiles contributes maximum -inf, sums 0)
        if (q_row < n) {
            const bool row_fits = MODE != kStep || (int64_t)s + q_row < step.cap_rows;
            const float* const all = reinterpret_cast<const float*>(ring);
            float m_w[WAVES], m_all = -INFINITY;
#pragma unroll
            for (int w2 = 0; w2 < WAVES; ++w2) {
                m_w[w2] = all[w2 * (2 * kTileBytes / 4) + lane];
                m_all = fmaxf(m_all, m_w[w2]);  // finite: wavefront 0 always has tile 0
            }
            float l_all = 0.f, o4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w2 = 0; w2 < WAVES; ++w2) {
                const float f = __builtin_amdgcn_exp2f(m_w[w2] - m_all);
                const float* pw = all + w2 * (2 * kTileBytes / 4);
                l_all = __builtin_fmaf(f, pw[kWaveSize + lane], l_all);
#pragma unroll
                for (int r = 0; r < 4; ++r) o4[r] = __builtin_fmaf(f, pw[(2 + 4 * wave + r) * kWaveSize + lane], o4[r]);
            }
            const float inv = 1.0f / l_all;
#pragma unroll
            for (int r = 0; r < 4; ++r) o4[r] *= inv;
            // this wavefront finishes head-dim elements 16g + 4*wave .. +3 of the lane's query
            if (row_fits) store4(o + row_of(q_row) * tok_o + head_off + 16 * g + 4 * wave, o4);
            if (MODE == kStep)
                store4(reinterpret_cast<OutT*>(step.out) + (pad0 + idx_lds[q_row]) * tok_o + head_off + 16 * g + 4 * wave, o4);
        }
        return;
    }

    int slot = 0;                                              // ring slot of tile t
    auto tile_step = [&](int t, auto first) {
        // this wavefront's part of tile t has landed once only the later tiles' loads remain in flight
        int behind = 0;
#pragma unroll
        for (int d = 0; d < kRing - 2; ++d) behind += c_next[d];
        if (behind == 0) wait_vm<0>();
        else if (behind == kPer) wait_vm<kPer>();
        else if (behind == 2 * kPer) wait_vm<2 * kPer>();
        else wait_vm<3 * kPer>();
        __syncthreads();                    // tile t visible; every wavefront is past tile t-1's reads
        const int slot_new = slot == 0 ? kRing - 1 : slot - 1; // slot of tile t-1, just freed, takes tile t+kRing-1
        const int c_new = t + kRing - 1 < tiles ? issue(t + kRing - 1, slot_new) : 0;
#pragma unroll
        for (int d = 0; d + 1 < kRing - 2; ++d) c_next[d] = c_next[d + 1];
        if (kRing > 2) c_next[kRing > 2 ? kRing - 3 : 0] = c_new;
        if (wave_active)
            tile_any<In, decltype(first)::value, EXT && !decltype(first)::value>(n - t * kBN, t == ride_tile,
                                                      ring0 + slot * 2 * kTileBytes, extra0, k_rel0, v_rel0,
                                                      q_frag, g, scale_log2e, m_run, l_acc, o_acc);
        slot = slot == kRing - 1 ? 0 : slot + 1;
    };
    if constexpr (PEEL) {
        tile_step(0, std::true_type{});     // n > m0 >= 0: there is a first tile
        for (int t = 1; t < tiles; ++t) tile_step(t, std::false_type{});
    } else {
        // the same loop written out with the general tile form (see PEEL above: the code generator's schedule
        // of the single-launch step depends on this exact shape)
        for (int t = 0; t < tiles; ++t) {
            int behind = 0;
#pragma unroll
            for (int d = 0; d < kRing - 2; ++d) behind += c_next[d];
            if (behind == 0) wait_vm<0>();
            else if (behind == kPer) wait_vm<kPer>();
            else if (behind == 2 * kPer) wait_vm<2 * kPer>();
            else wait_vm<3 * kPer>();
            __syncthreads();
            const int slot_new = slot == 0 ? kRing - 1 : slot - 1;
            const int c_new = t + kRing - 1 < tiles ? issue(t + kRing - 1, slot_new) : 0;
#pragma unroll
            for (int d = 0; d + 1 < kRing - 2; ++d) c_next[d] = c_next[d + 1];
            if (kRing > 2) c_next[kRing > 2 ? kRing - 3 : 0] = c_new;
            if (wave_active) {
                const int rem = n - t * kBN;
                const uint32_t tile0 = ring0 + slot * 2 * kTileBytes;
                const uint32_t k_a0 = tile0 + k_rel0, k_a1 = tile0 + (k_rel0 ^ 16u);
                const uint32_t v_a0 = tile0 + v_rel0, v_a1 = tile0 + (v_rel0 ^ 16u);
                const uint32_t ek_a0 = extra0 + k_rel0, ev_a0 = extra0 + kExtraBytes / 2 + (v_rel0 - kTileBytes);
                if (t == ride_tile) {
                    tile_update<In, 5, true, false>(k_a0, k_a1, v_a0, v_a1, ek_a0, ev_a0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc);
                } else if (rem >= kBN) {
                    tile_update<In, 4, false, false>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc);
                } else {
                    switch ((rem + 15) >> 4) {
                        case 1: tile_update<In, 1, true, false>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc); break;
                        case 2: tile_update<In, 2, true, false>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc); break;
                        case 3: tile_update<In, 3, true, false>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc); break;
                        default: tile_update<In, 4, true, false>(k_a0, k_a1, v_a0, v_a1, 0, 0, q_frag, rem, g, scale_log2e, m_run, l_acc, o_acc); break;
                    }
                }
            }
            if (t == 0) {
                // the x rows have long arrived: with several tiles the copy drains while the rest is computed
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int j = m0 + 32 * i + (tid >> 3);
                    if (j < n && (int64_t)s + j < step.cap_rows)
                        reinterpret_cast<uint4*>(step.packed + ((int64_t)s + j) * tok + head_off)[tid & 7] = x_raw[i];
                }
            }
            slot = slot == kRing - 1 ? 0 : slot + 1;
        }
    }

    // ---- normalise and store: this lane owns d = 16g + 4dt + r of its query
    const bool row_fits = MODE != kStep || (int64_t)s + q_row < step.cap_rows;
    if (wave_active && q_row < n) {
        const float inv = 1.0f / l_acc[0];
        float out16[16];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) out16[4 * dt + r] = o_acc[dt][r] * inv;
        if (row_fits) store16(o + row_of(q_row) * tok_o + head_off + 16 * g, out16);
        if (MODE == kStep)                                     // the same row at its padded position
            store16(reinterpret_cast<OutT*>(step.out) + (pad0 + idx_lds[q_row]) * tok_o + head_off + 16 * g, out16);
    }
}

template <typename In, typename OutT, int MODE>
hipError_t launch_typed(const void* q, const void* k, const void* v, void* o,
                        const int32_t* cu_seqlens, const uint8_t* keep, int n_tok, int fill_mode,
                        int B, int max_seqlen, int H, int64_t in_tok, int64_t out_tok, float scale,
                        const StepArgs& step, hipStream_t stream) {
    constexpr int kWaves = kAttnWaves;                         // 16 query rows each
    constexpr int kGroup = 512;                                // pairs per dispatch batch
    const int pairs = B * H;
    // Small launches (at most kSplitMaxGroups 64-row q-tiles, sequences that may span several K/V tiles) leave
    // most CUs idle and are a chain of latencies: they take 16-row work-groups whose wavefronts split the keys.
    const bool split = max_seqlen > kBN && (int64_t)pairs * ((max_seqlen + 16 * kWaves - 1) / (16 * kWaves)) <= kSplitMaxGroups;
    const int tile_rows = split ? 16 : 16 * kWaves;
    const int q_tiles = (max_seqlen + tile_rows - 1) / tile_rows;
    const int pairs8 = (pairs + kXcds - 1) / kXcds * kXcds;
    const int group = pairs8 < kGroup ? pairs8 : kGroup;
    const int batches = (pairs + group - 1) / group;
    if (q_tiles > kMaxGridYZ || batches > kMaxGridYZ || in_tok > INT32_MAX || out_tok > INT32_MAX)
        return hipErrorInvalidValue;                            // (the C ABI layer has refused these already)
    const hipError_t err = launch_kernel(split ? attn_kernel<In, OutT, MODE, true> : attn_kernel<In, OutT, MODE, false>,
                       dim3(group, q_tiles, batches), dim3(kAttnThreads), stream,
                       MODE == kPacked ? static_cast<const void*>(cu_seqlens) : static_cast<const void*>(keep),
                       n_tok, fill_mode, H, div_magic((uint32_t)H), pairs, group, static_cast<const uint16_t*>(k),
                       static_cast<const uint16_t*>(v), (int)in_tok, (int)out_tok, static_cast<const uint16_t*>(q),
                       static_cast<OutT*>(o), fabsf(scale) * kLog2e, scale < 0.f ? 1 : 0, step);
    return err;
}

template <int MODE>
hipError_t launch_any(const void* q, const void* k, const void* v, void* o, const int32_t* cu_seqlens,
                      const uint8_t* keep, int n_tok, int fill_mode, int B, int max_seqlen, int H,
                      int64_t in_tok, int64_t out_tok, float scale, ragged_dtype in_dt,
                      ragged_dtype out_dt, const StepArgs& step, hipStream_t stream) {
    if (in_dt == RAGGED_F16 && out_dt == RAGGED_F16)
        return launch_typed<F16, _Float16, MODE>(q, k, v, o, cu_seqlens, keep, n_tok, fill_mode, B, max_seqlen, H, in_tok, out_tok, scale, step, stream);
    if (in_dt == RAGGED_F16 && out_dt == RAGGED_F32)
        return launch_typed<F16, float, MODE>(q, k, v, o, cu_seqlens, keep, n_tok, fill_mode, B, max_seqlen, H, in_tok, out_tok, scale, step, stream);
    if (in_dt == RAGGED_BF16 && out_dt == RAGGED_BF16)
        return launch_typed<BF16, __bf16, MODE>(q, k, v, o, cu_seqlens, keep, n_tok, fill_mode, B, max_seqlen, H, in_tok, out_tok, scale, step, stream);
    if (in_dt == RAGGED_BF16 && out_dt == RAGGED_F32)
        return launch_typed<BF16, float, MODE>(q, k, v, o, cu_seqlens, keep, n_tok, fill_mode, B, max_seqlen, H, in_tok, out_tok, scale, step, stream);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_attn(const void* q, const void* k, const void* v, void* o,
                       const int32_t* cu_seqlens, int B, int max_seqlen, int H, int64_t in_tok,
                       int64_t out_tok, float scale, ragged_dtype in_dt, ragged_dtype out_dt,
                       int32_t* flags, hipStream_t stream) {
    StepArgs extra{};
    extra.flags = flags;
    extra.max_seqlen = max_seqlen;
    return launch_any<kPacked>(q, k, v, o, cu_seqlens, nullptr, 0, 0, B, max_seqlen, H, in_tok, out_tok, scale,
                               in_dt, out_dt, extra, stream);
}

int attn_padded_max_tokens() { return kMaxGatherTokens; }

hipError_t launch_attn_padded(const void* q, const void* k, const void* v, void* o, const uint8_t* keep,
                              int B, int N, int H, float scale, ragged_dtype in_dt, ragged_dtype out_dt,
                              int fill_mode, hipStream_t stream) {
    const int64_t tok = (int64_t)H * kHeadDim;
    return launch_any<kPadded>(q, k, v, o, nullptr, keep, N, fill_mode, B, N, H, tok, tok, scale, in_dt, out_dt,
                               StepArgs{}, stream);
}

hipError_t launch_step(const void* x, const uint8_t* keep, const void* q, const void* k, const void* v,
                       int B, int N, int H, float scale, ragged_dtype dt, void* packed, int64_t cap_rows,
                       int32_t* cu_seqlens, int32_t* gather_idx, void* o, void* out, int fill_mode,
                       hipStream_t stream) {
    const int64_t tok = (int64_t)H * kHeadDim;
    const StepArgs step{static_cast<const uint16_t*>(x), static_cast<uint16_t*>(packed),
                        static_cast<uint16_t*>(out), cu_seqlens, gather_idx, cap_rows, nullptr, 0};
    if (dt == RAGGED_F16)
        return launch_typed<F16, _Float16, kStep>(q, k, v, o, nullptr, keep, N, fill_mode, B, N, H, tok, tok, scale,
                                                  step, stream);
    return launch_typed<BF16, __bf16, kStep>(q, k, v, o, nullptr, keep, N, fill_mode, B, N, H, tok, tok, scale,
                                             step, stream);
}

}  // namespace ragged
