// 16-bit storage formats of inputs and table rows, widened exactly to fp32 (the arithmetic is fp32
// throughout; Sec. 3.1 fixes no storage precision).  kind 1 = bf16: the top half of an fp32 pattern;
// kind 2 = IEEE binary16: one hardware conversion (exact, subnormals included).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lffn {

enum ElemKind : int { kElemF32 = 0, kElemBF16 = 1, kElemF16 = 2 };

__device__ __forceinline__ float half_bits_to_float(uint32_t bits)  // low 16 bits
{
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
}

// the element in the low 16 bits of `bits`
__device__ __forceinline__ float widen16(uint32_t bits, int kind)
{
    return kind == kElemF16 ? half_bits_to_float(bits) : __uint_as_float(bits << 16);
}

// both elements of a dword: .x = the low half (the element at the lower address)
template <int KIND>
__device__ __forceinline__ float2 widen16x2(uint32_t w)
{
    static_assert(KIND == kElemBF16 || KIND == kElemF16, "a 16-bit kind");
    if constexpr (KIND == kElemF16)
        return make_float2(half_bits_to_float(w), half_bits_to_float(w >> 16));
    else
        return make_float2(__uint_as_float(w << 16), __uint_as_float(w & 0xFFFF0000u));
}
__device__ __forceinline__ float2 widen16x2(uint32_t w, int kind)
{
    return kind == kElemF16 ? widen16x2<kElemF16>(w) : widen16x2<kElemBF16>(w);
}

}  // namespace lffn
