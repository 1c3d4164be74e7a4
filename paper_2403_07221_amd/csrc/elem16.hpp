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

// fp32 -> 16-bit storage for outputs kept in 16 bits, round to nearest even.  bf16: half an ulp of the kept
// part plus its last bit on a tie is added to the pattern, then the low half is cut (NaN keeps a quiet
// payload); IEEE half: the hardware conversion (round to nearest even is the default mode, never changed).
__device__ __forceinline__ uint32_t narrow16(float f, int kind)
{
    if (kind == kElemF16) return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Stores four consecutive outputs, elements e .. e + 3 of y (e % 4 == 0), in y's storage type, streaming
// (y is written once and not read again by the kernel).
__device__ __forceinline__ void store_y4(void *y, size_t e, float a, float b, float c, float d, int y_kind)
{
    if (y_kind == kElemF32) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const f4 o = {a, b, c, d};
        __builtin_nontemporal_store(o, reinterpret_cast<f4 *>(static_cast<float *>(y) + e));
    } else {
        typedef uint32_t u2 __attribute__((ext_vector_type(2)));
        const u2 o = {narrow16(a, y_kind) | (narrow16(b, y_kind) << 16), narrow16(c, y_kind) | (narrow16(d, y_kind) << 16)};
        __builtin_nontemporal_store(o, reinterpret_cast<u2 *>(static_cast<uint16_t *>(y) + e));
    }
}

}  // namespace lffn
