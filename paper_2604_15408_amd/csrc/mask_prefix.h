// Work-group-wide count of the nonzero bytes of a keep-mask prefix (internal; shared by the pack /
// unpack kernels and the single-launch pack + attention + unpack kernel).
#pragma once

#include "common.h"

namespace ragged {

// Number of nonzero bytes in a 32-bit word.  (b & 0x7f) + 0x7f carries into bit 7 of its own byte
// exactly when the low 7 bits are nonzero, and never into the next byte.
__device__ __forceinline__ int nonzero_bytes(uint32_t w) {
    const uint32_t t = ((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w;
    return __popc(t & 0x80808080u);
}

// Sum over the 64 lanes of a wavefront, result in every lane, without going through LDS: four
// rotations inside each 16-lane row (DPP row_ror 8/4/2/1), then the gfx950 lane-swap instructions
// across rows.  permlane16_swap(a, b) returns {a.row0,b.row0,a.row2,b.row2} and
// {a.row1,b.row1,a.row3,b.row3}; permlane32_swap(a, b) returns {a.lo|b.lo} and {a.hi|b.hi}.  The
// second operand is a copy made through an opaque move so it can never share a register with the
// first (the instruction swaps its operands in place).
template <int kCtrl>
__device__ __forceinline__ int dpp_move(int v) {
    return __builtin_amdgcn_update_dpp(0, v, kCtrl, 0xf, 0xf, true);
}
__device__ __forceinline__ int opaque_copy_i(int x) {
    int y;
    asm volatile("v_mov_b32 %0, %1" : "=v"(y) : "v"(x));
    return y;
}
__device__ __forceinline__ int wave_sum(int v) {
    v += dpp_move<0x128>(v);                                   // row_ror:8
    v += dpp_move<0x124>(v);                                   // row_ror:4
    v += dpp_move<0x122>(v);                                   // row_ror:2
    v += dpp_move<0x121>(v);                                   // row_ror:1
    const auto a = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)opaque_copy_i(v), false, false);
    const unsigned a0 = a[0], a1 = a[1];
    v = (int)(a0 + a1);
    const auto b = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)opaque_copy_i(v), false, false);
    const unsigned b0 = b[0], b1 = b[1];
    return (int)(b0 + b1);
}

// Work-group-wide count of nonzero bytes in base[0, len), in two halves so that a caller can put
// other memory traffic between them: prefix_issue() starts the loads (first 16 KB of the range into
// registers), prefix_finish() consumes them, handles any remainder, and reduces over the group.
// Every thread of the 256-thread group must call both; every thread receives the total.  The bulk
// is read as aligned 16-byte words; the unaligned head and the tail go byte by byte.  No byte outside
// [0, len) is touched, except that base[0] is read when len is 0: base must point at a readable byte
// (every caller passes the start of a mask that is not empty).
//
// The byte loads are unconditional, with the index clamped into the range, and their values are only
// looked at in prefix_finish().  A predicated byte load ("in range ? base[i] : 0") is compiled into
// load, wait, compare inside the branch: every such load then costs a memory round trip of its own,
// in front of whatever the caller wanted to have in flight together with the prefix.
constexpr int kPrefixWords = 4;    // 16-byte words per thread kept in flight: 16 KB per pass of the group

// A byte whose use can wait: base[min(i, len - 1)] (base[0] when len <= 0), never predicated.
__device__ __forceinline__ uint8_t load_byte_clamped(const uint8_t* __restrict__ base, int i, int len) {
    int j = i < len ? i : len - 1;
    j = j > 0 ? j : 0;
    return base[j];
}

struct PrefixLoads {
    uint4 w[kPrefixWords];   // words tid + 256*j of the aligned body (zero if absent)
    uint8_t hb, tb;          // a head byte / a tail byte: count only where tid < head / tail0 + tid < len
    int head, body, len;
};

__device__ __forceinline__ PrefixLoads prefix_issue(const uint8_t* __restrict__ base, int len) {
    const int tid = threadIdx.x;
    PrefixLoads p;
    const int mis = (int)((uintptr_t)base & 15u);
    p.head = mis ? 16 - mis : 0;
    if (p.head > len) p.head = len;
    // base and len are the same for the whole group: kept in scalar registers, so that the tests on them are
    // scalar branches
    p.head = __builtin_amdgcn_readfirstlane(p.head);
    p.body = __builtin_amdgcn_readfirstlane((len - p.head) >> 4);   // whole 16-byte words
    p.len = __builtin_amdgcn_readfirstlane(len);
    const uint4* words = reinterpret_cast<const uint4*>(base + p.head);
#pragma unroll
    for (int j = 0; j < kPrefixWords; ++j)
        p.w[j] = tid + j * kBlockThreads < p.body ? words[tid + j * kBlockThreads] : make_uint4(0u, 0u, 0u, 0u);
    p.hb = load_byte_clamped(base, tid, len);
    p.tb = load_byte_clamped(base, p.head + (p.body << 4) + tid, len);   // fewer than 16 tail bytes
    return p;
}

__device__ __forceinline__ int count_word(uint4 v) {
    return nonzero_bytes(v.x) + nonzero_bytes(v.y) + nonzero_bytes(v.z) + nonzero_bytes(v.w);
}

// This thread's share of the count: the words and bytes requested by prefix_issue() plus, for ranges beyond
// 16 KB, the rest of the body.
__device__ inline int prefix_count_thread(const uint8_t* __restrict__ base, const PrefixLoads& p) {
    const int tid = threadIdx.x;
    const int tail0 = p.head + (p.body << 4);
    int count = (tid < p.head && p.hb != 0) + (tail0 + tid < p.len && p.tb != 0);
#pragma unroll
    for (int j = 0; j < kPrefixWords; ++j) {
        if (j * kBlockThreads >= p.body) break;                // group-uniform: no further pass holds a word
        count += count_word(p.w[j]);
    }
    const uint4* words = reinterpret_cast<const uint4*>(base + p.head);
    for (int w0 = tid + kPrefixWords * kBlockThreads; w0 < p.body; w0 += kPrefixWords * kBlockThreads) {
        uint4 more[kPrefixWords];                             // all loads of a pass issued before any is used
#pragma unroll
        for (int j = 0; j < kPrefixWords; ++j)
            more[j] = w0 + j * kBlockThreads < p.body ? words[w0 + j * kBlockThreads] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int j = 0; j < kPrefixWords; ++j) count += count_word(more[j]);
    }
    return count;
}

// The reduction over the group in two steps, for callers that have a barrier of their own to share:
// prefix_post() before it (every thread), prefix_total() after it.  lds4 is used once per kernel.
__device__ __forceinline__ void prefix_post(int thread_count, int* lds4) {
    const int tid = threadIdx.x;
    const int count = wave_sum(thread_count);
    if ((tid & (kWaveSize - 1)) == 0) lds4[tid >> 6] = count;
}
__device__ __forceinline__ int prefix_total(const int* lds4) { return lds4[0] + lds4[1] + lds4[2] + lds4[3]; }

__device__ inline int prefix_finish(const uint8_t* __restrict__ base, const PrefixLoads& p, int* lds4) {
    prefix_post(prefix_count_thread(base, p), lds4);
    __syncthreads();
    return prefix_total(lds4);
}

}  // namespace ragged
