// Internal helpers shared by the HIP translation units of libsage_hip (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sage.h"

namespace sage {

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline int launch_status() { return hipGetLastError() == hipSuccess ? SAGE_OK : SAGE_LAUNCH_FAILED; }

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

// fp32 -> bf16, round to nearest even (finite values and infinities; NaN stays NaN).
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}


// 16 bytes per lane from global memory straight into LDS (lane l lands at lds + 16 l; LDS-direct load of gfx950).
// Written as inline assembly so that these loads stay out of the compiler's own bookkeeping of outstanding memory
// operations.  With the builtin the compiler treats them as operations that may complete out of order: every LDS read
// then waits for all earlier LDS reads instead of its own, and a read of a stage that was filled earlier in the same
// loop iteration waits for ALL loads in flight, which drains a prefetch ring.  Kernels that use this keep their own
// count of loads in flight (s_waitcnt vmcnt(N) plus a barrier); the "memory" clobber keeps LDS reads from moving
// across an issue.  M0 carries the LDS address of the load; nothing else in these kernels uses it.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_direct_load16(const unsigned char* gptr, __attribute__((address_space(3))) unsigned char* lds) {
    const unsigned m0v = static_cast<unsigned>(reinterpret_cast<uintptr_t>(lds));
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(m0v)
                 : "m0", "memory");
}
// The same load with the address split into a wave-uniform base (scalar register pair) and a 32-bit per-lane byte
// offset: a stream whose per-lane offsets repeat from tile to tile then advances with scalar arithmetic only.
__device__ __forceinline__ void lds_direct_load16(const unsigned char* sbase, unsigned voff,
                                                  __attribute__((address_space(3))) unsigned char* lds) {
    const unsigned m0v = static_cast<unsigned>(reinterpret_cast<uintptr_t>(lds));
    // the base is uniform by contract; said to the compiler, which otherwise may hand the asm a vector register pair
    const uintptr_t bv = reinterpret_cast<uintptr_t>(sbase);
    const uintptr_t base = (static_cast<uintptr_t>(static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bv >> 32)))) << 32) |
                           static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(bv)));
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(base), "s"(m0v)
                 : "m0", "memory");
}
// The 4-byte form: lane l lands at lds + 4 l.
__device__ __forceinline__ void lds_direct_load4(const unsigned char* gptr, __attribute__((address_space(3))) unsigned char* lds) {
    const unsigned m0v = static_cast<unsigned>(reinterpret_cast<uintptr_t>(lds));
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
                 :
                 : "v"(gptr), "s"(m0v)
                 : "m0", "memory");
}
#pragma clang diagnostic pop

// ---- Wave-wide reductions, result in every lane: four rotations inside each row of 16 lanes, then the 16-lane and
// 32-lane swaps combine the four rows.  About ten vector instructions and no LDS traffic, where the shuffle intrinsics
// go through the LDS crossbar at a round trip per step.
template <int CTRL> __device__ __forceinline__ uint32_t u_dpp(uint32_t v) {
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL> __device__ __forceinline__ float f_dpp(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, u_dpp<0x128>(v));         // row_ror:8
    v = max(v, u_dpp<0x124>(v));         // row_ror:4
    v = max(v, u_dpp<0x122>(v));         // row_ror:2
    v = max(v, u_dpp<0x121>(v));         // row_ror:1
    auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = max(a[0], a[1]);
    a = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return max(a[0], a[1]);
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
    v += u_dpp<0x128>(v); v += u_dpp<0x124>(v); v += u_dpp<0x122>(v); v += u_dpp<0x121>(v);
    auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = a[0] + a[1];
    a = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return a[0] + a[1];
}
__device__ __forceinline__ float wave_sum(float v) {
    v += f_dpp<0x128>(v); v += f_dpp<0x124>(v); v += f_dpp<0x122>(v); v += f_dpp<0x121>(v);
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(a[0]) + __uint_as_float(a[1]);
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, f_dpp<0x128>(v)); v = fmaxf(v, f_dpp<0x124>(v)); v = fmaxf(v, f_dpp<0x122>(v)); v = fmaxf(v, f_dpp<0x121>(v));
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
}
// Lane `lane` (wave-uniform) of a value, through a scalar register.
__device__ __forceinline__ float lane_value(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ uint64_t lane_value(uint64_t v, int lane) {
    const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(v)), lane));
    const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(v >> 32)), lane));
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

}  // namespace sage
