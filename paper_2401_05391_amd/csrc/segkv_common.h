// Shared device-side helpers of libsegkv (gfx950 only): vector types, DPP
// lane reductions, packed beam maps, online-softmax state merging.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace segkv {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr float kLog2e = 1.4426950408889634f;
// "Nothing seen yet" running maximum.  Finite on purpose: exp2(x - kEmptyMax)
// with x = -inf is 0 and kEmptyMax - kEmptyMax is 0, so no inf-inf ever forms.
constexpr float kEmptyMax = -1.0e30f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Between LDS writes of a wave and reads of the same locations by OTHER lanes of
// the same wave: orders the two at wavefront scope for the compiler (the
// hardware issues a wave's LDS operations in order).  Generates no instruction.
__device__ __forceinline__ void wave_lds_exchange_point()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- DPP lane exchange (all patterns used here read a valid lane) ----------
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
constexpr int kDppQuadSwap1 = 0xB1;   // quad_perm:[1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;   // quad_perm:[2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // row_half_mirror (lane i <- 7-i within 8)
constexpr int kDppRowMirror = 0x140;  // row_mirror      (lane i <- 15-i within 16)

// Sum over groups of LANES consecutive lanes (8 or 16); every lane of the
// group ends up holding the total.
template <int LANES>
__device__ __forceinline__ float group_allreduce_sum(float x)
{
    x += dpp_move<kDppQuadSwap1>(x);
    x += dpp_move<kDppQuadSwap2>(x);
    x += dpp_move<kDppHalfMirror>(x);
    if (LANES == 16) x += dpp_move<kDppRowMirror>(x);
    return x;
}

// ---- beam maps: slot permutations/selections packed 4 bits per beam --------
// Nibble j of a map f is f[j].  Slots >= W keep the identity so that every map
// is a total function on 0..7.
constexpr uint32_t kIdentityMap = 0x76543210u;

__device__ __forceinline__ uint32_t map_get(uint32_t f, int j) { return (f >> (4 * j)) & 15u; }

// (f o g)[j] = f[g[j]]
__device__ __forceinline__ uint32_t map_compose(uint32_t f, uint32_t g)
{
    uint32_t r = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) r |= map_get(f, (int)map_get(g, j)) << (4 * j);
    return r;
}

}  // namespace segkv
