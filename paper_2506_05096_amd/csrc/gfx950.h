// Device-side vocabulary shared by the gfx950 kernels of libastraea: vector types, the hardware bf16
// pack, 16-byte LDS fragment reads, and the global -> LDS tile copy.
#pragma once
#include "common.h"

namespace astraea {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

// Two floats to a bf16 pair, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    floatx2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// One MFMA operand fragment (8 bf16) from LDS; `addr` is an LDS byte address.
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr)
{
    return *reinterpret_cast<const bf16x8 __attribute__((address_space(3))) *>((uintptr_t)addr);
}

// 16 bytes per lane from global memory straight into LDS: lane l of the wave lands at
// lds_wave_base + 16*l.  The LDS base travels in M0, which the statement overwrites (declared, so the
// compiler keeps nothing of its own there across it).  Completion is counted by vmcnt; a kernel waits
// for it explicitly before the barrier that publishes the tile.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"    // m0 is a reserved register; naming it as clobbered is the point
__device__ __forceinline__ void dma16(const void *gbase, uint32_t goff, uint32_t lds_wave_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_wave_base), "v"(goff), "s"(gbase)
                 : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// An index from a caller's idx_sel, forced into [0, n_rows): reads through it stay inside the buffer.
__device__ __forceinline__ int32_t clamp_row(int32_t ix, int32_t n_rows)
{
    return ix < 0 ? 0 : (ix > n_rows - 1 ? n_rows - 1 : ix);
}

// GELU in its tanh form, 0.5 t (1 + tanh u) = t / (1 + e^(-2u)) with u = sqrt(2/pi) (t + 0.044715 t^3).
__device__ __forceinline__ float gelu_tanh(float t)
{
    const float u = 0.79788456080286535588f * __builtin_fmaf(0.044715f * t, t * t, t);
    const float e = __builtin_amdgcn_exp2f(-2.0f * 1.44269504088896340736f * u);
    return t * __builtin_amdgcn_rcpf(1.0f + e);
}

}  // namespace astraea
