// Operand types of the gfx950 matrix units as the SpMM kernels use them: vector typedefs, the
// numbering of the types, what each accumulates into, and the MFMA 16x16x32 call per type.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

namespace smat {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x3 __attribute__((ext_vector_type(3)));

// Operand types.  The numbers are those of smat_dtype_t in the public header.
enum : int { kF16 = 0, kBF16 = 1, kE4M3 = 2, kE5M2 = 3, kI8 = 4 };

template <int DT> struct Elem {
    static constexpr int ES = DT <= kBF16 ? 2 : 1;                                  // bytes per element of A and B
    using Acc = typename std::conditional<DT == kI8, i32x4, f32x4>::type;           // one 16x16 output tile, per lane
    using Out = typename std::conditional<DT == kI8, int32_t, float>::type;         // element of C
};

// One matrix instruction: a 16 x 32 piece of A' times 32 x 16 of B.  The 8-bit forms take the
// first two dwords of a and b.
template <int DT>
__device__ __forceinline__ typename Elem<DT>::Acc mfma_pack(u32x4 a, u32x4 b, typename Elem<DT>::Acc c)
{
    if constexpr (DT == kBF16) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else if constexpr (DT == kF16) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    } else {
        const long a8 = __builtin_bit_cast(long, u32x2{a[0], a[1]});
        const long b8 = __builtin_bit_cast(long, u32x2{b[0], b[1]});
        if constexpr (DT == kE4M3) return __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a8, b8, c, 0, 0, 0);
        else if constexpr (DT == kE5M2) return __builtin_amdgcn_mfma_f32_16x16x32_bf8_bf8(a8, b8, c, 0, 0, 0);
        else return __builtin_amdgcn_mfma_i32_16x16x32_i8(a8, b8, c, 0, 0, 0);
    }
}

// int8 with k = 64 (gfx950): a 16 x 64 piece of A' times 64 x 16 of B, sixteen bytes per lane and
// operand; twice the rate of the k = 32 form.
__device__ __forceinline__ i32x4 mfma_i8_k64(u32x4 a, u32x4 b, i32x4 c)
{
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b), c, 0, 0, 0);
}

// The same instructions for the 8-bit types written out, with the result in the registers of the addend.  The
// compiler's own choice for these forms (unlike the 16-bit ones) is a result apart from the addend: a loop with 128
// accumulators per lane then drifts through some 45 further registers and, at the limit of 256, spills inside the
// loop.  The compiler does not see a matrix instruction here and adds none of the waits it would put in front of a
// later ordinary instruction that reads the result (up to 18 clocks): whoever uses these leaves that distance.
// `second` picks dwords 2, 3 of a and b (the second sub-step of 32 k slots) instead of 0, 1.
template <int DT>
__device__ __forceinline__ void mfma_pack8_in_place(u32x4 a, u32x4 b, bool second, typename Elem<DT>::Acc& c)
{
    static_assert(DT == kE4M3 || DT == kE5M2 || DT == kI8, "8-bit operand types");
    const u32x2 a8 = second ? u32x2{a[2], a[3]} : u32x2{a[0], a[1]};
    const u32x2 b8 = second ? u32x2{b[2], b[3]} : u32x2{b[0], b[1]};
    if constexpr (DT == kE4M3) asm("v_mfma_f32_16x16x32_fp8_fp8 %0, %1, %2, %0" : "+v"(c) : "v"(a8), "v"(b8));
    else if constexpr (DT == kE5M2) asm("v_mfma_f32_16x16x32_bf8_bf8 %0, %1, %2, %0" : "+v"(c) : "v"(a8), "v"(b8));
    else asm("v_mfma_i32_16x16x32_i8 %0, %1, %2, %0" : "+v"(c) : "v"(a8), "v"(b8));
}
__device__ __forceinline__ void mfma_i8_k64_in_place(u32x4 a, u32x4 b, i32x4& c)
{
    asm("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
}

}  // namespace smat
