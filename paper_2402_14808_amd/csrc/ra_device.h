// Device-side helpers shared by the gfx950 relay-attention kernels: 16-byte
// vector types, bfloat16 unpacking, DPP lane-group reductions and the merge of
// two softmax partials (the rescaling identity behind Eq. 6-7 of the paper).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ra {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kWave = 64;
constexpr int kThreads = 256;  // every kernel here runs 4 wavefronts per workgroup

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// float -> bfloat16 bits, round to nearest even (NaN kept quiet).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// Sum of a[i]*b[i] over the 8 bfloat16 held in two 16-byte registers.
__device__ __forceinline__ float dot8_bf16(const u32x4 a, const u32x4 b, float acc) {
    // (elements are copied to scalars first: bit-casting a vector element in place picked
    // element 0 for every i with this compiler)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t ai = a[i], bi = b[i];
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, ai),
                                              __builtin_bit_cast(bf16x2, bi), acc, false);
    }
    return acc;
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __int_as_float(
        __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// All-reduce (sum) over aligned groups of LPT = 8 or 16 adjacent lanes; every lane of a
// group ends with the same bits.  quad_perm xor-1, xor-2, then half-row and row mirrors.
template <int LPT>
__device__ __forceinline__ float group_sum(float x) {
    x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);  // row_half_mirror
    if (LPT == 16) x += dpp_move<0x140>(x);  // row_mirror
    return x;
}

// The value lane ^ 32 holds, without a trip through the LDS crossbar (which ds_bpermute, the
// generic shuffle, takes, and whose result is waited for together with every LDS read the
// wavefront has in flight): v_permlane32_swap exchanges the upper half of one register with the
// lower half of another, so swapping two copies of x leaves every lane with its own value in one
// of them and its partner's in the other.
__device__ __forceinline__ float max_with_other_half(float x) {
    const uint32_t bits = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_other_half(float x) {
    const uint32_t bits = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// exp2 that maps -inf to 0 and never sees inf - inf: callers pass a finite `m_use`.
__device__ __forceinline__ float finite_or_zero(float m) { return m == -INFINITY ? 0.f : m; }

}  // namespace ra
