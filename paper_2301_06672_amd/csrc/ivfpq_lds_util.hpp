// Small device helpers of the scan kernels: LDS reads from integer addresses, sub-dword shifts, half-precision
// accumulation in one instruction, compile-time loops.  Included by ivfpq_device.hip only.
#pragma once

#include <cstdint>
#include <type_traits>
#include <utility>

// A W-byte word read from LDS address `a`, counted from the start of the workgroup's LDS, through a pointer to a
// scalar type of that width.  Kernels that form such addresses as plain integers take their dynamic LDS to start
// at LDS address 0, i.e. to have no static LDS: the host verifies that before their first launch.
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
#define IVFPQ_LDS_PTR(T, addr) reinterpret_cast<const __attribute__((address_space(3))) T*>(addr)
template <int W> struct LdsWord;
template <> struct LdsWord<1> { using type = uint32_t; static __device__ __forceinline__ type load(uint32_t a) { return *IVFPQ_LDS_PTR(uint8_t, a); } };
template <> struct LdsWord<2> { using type = uint32_t; static __device__ __forceinline__ type load(uint32_t a) { return *IVFPQ_LDS_PTR(uint16_t, a); } };
template <> struct LdsWord<4> { using type = uint32_t; static __device__ __forceinline__ type load(uint32_t a) { return *IVFPQ_LDS_PTR(uint32_t, a); } };
template <> struct LdsWord<8> {
    using type = u32x2_t;
    static __device__ __forceinline__ type load(uint32_t a) {
        const unsigned long long v = *IVFPQ_LDS_PTR(unsigned long long, a);
        return type{(uint32_t)v, (uint32_t)(v >> 32)};
    }
};
template <> struct LdsWord<16> {
    using type = u32x4_t;
    static __device__ __forceinline__ type load(uint32_t a) {
        const __uint128_t v = *IVFPQ_LDS_PTR(__uint128_t, a);
        return type{(uint32_t)v, (uint32_t)(v >> 32), (uint32_t)(v >> 64), (uint32_t)(v >> 96)};
    }
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// byte BYTE of w, shifted left by SH, in one instruction (sub-dword operand select)
template <int BYTE, int SH>
__device__ __forceinline__ uint32_t byte_shl(uint32_t w) {
    if constexpr (SH == 0) {
        return (w >> (8 * BYTE)) & 255u;
    } else {
        uint32_t r;
        if constexpr (BYTE == 0) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "n"(SH), "v"(w));
        if constexpr (BYTE == 1) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "n"(SH), "v"(w));
        if constexpr (BYTE == 2) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "n"(SH), "v"(w));
        if constexpr (BYTE == 3) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "n"(SH), "v"(w));
        return r;
    }
}

// the lanes of the wave for which `p` holds, as a mask: the compare's own result, with no 0/1 value in between
__device__ __forceinline__ unsigned long long ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// how many lanes below this one are set in `mask` (two count instructions on the mask's halves)
__device__ __forceinline__ uint32_t lanes_below(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): loops whose index must be a constant in
// the body (register arrays indexed by it stay in registers)
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }


// acc + (float)h for the half in the low / high 16 bits of h: a fused multiply-add with 1.0 that converts its half
// operand in the same instruction (exact conversion, one rounding: the value of convert-then-add)
__device__ __forceinline__ float add_half_lo(float acc, uint32_t h) {
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(h), "v"(acc));
    return r;
}
__device__ __forceinline__ float add_half_hi(float acc, uint32_t h) {
    float r;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(h), "v"(acc));
    return r;
}
