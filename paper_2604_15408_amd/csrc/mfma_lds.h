// MFMA operand types and the LDS / global->LDS primitives shared by the attention and the linear
// kernels (internal).
//
// MFMA 16x16x32 operand layout (A: 16 rows x 32 k, B: 32 k x 16 cols, D: 16x16):
//   A: lane l holds row l%16,  k-slots 8*(l/16)+e, e = 0..7
//   B: lane l holds col l%16,  k-slots 8*(l/16)+e
//   D: lane l, register r holds row 4*(l/16)+r, col l%16
#pragma once

#include "common.h"

namespace ragged {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

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

typedef short short4v __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) short4v lds_short4;

__device__ __forceinline__ uint4 lds_read16(uint32_t addr) {
    const u32x4 w = *reinterpret_cast<const lds_u32x4*>(static_cast<uintptr_t>(addr));
    return make_uint4(w[0], w[1], w[2], w[3]);
}
// transposing 8-byte LDS read (see the header comment)
__device__ __forceinline__ short4v lds_read_tr(uint32_t addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_short4*>(static_cast<uintptr_t>(addr)));
}

// One wavefront instruction of the global->LDS load: lane i fetches the 16 bytes at base + voff and
// the hardware stores them at LDS address lds_dst + 16*i.  The compiler is not told about the LDS
// write; callers order it against LDS reads with wait_vm<>() and a barrier.
// M0 (the LDS destination register of this instruction) is written inside the asm and listed as clobbered,
// so the compiler never keeps a value of its own there across the statement; clang remarks that M0 is a
// reserved register whenever it appears in a clobber list, which is expected here.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(uint32_t lds_dst, uint32_t voff, const void* base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_dst), "v"(voff), "s"(base) : "memory", "m0");
}
#pragma clang diagnostic pop
template <int N>
__device__ __forceinline__ void wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

}  // namespace ragged
