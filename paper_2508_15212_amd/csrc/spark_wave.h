// Wave-level building blocks shared by the pruning kernels (gfx950, wave64): data-parallel-primitive scans and
// sums, prefix popcounts, lane writes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace spark {

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// bits 0..15 of x spread to the even bit positions of a 32-bit word
__device__ __forceinline__ uint32_t spread16(uint32_t x)
{
    x &= 0xFFFFu;
    x = (x | (x << 8)) & 0x00FF00FFu;
    x = (x | (x << 4)) & 0x0F0F0F0Fu;
    x = (x | (x << 2)) & 0x33333333u;
    x = (x | (x << 1)) & 0x55555555u;
    return x;
}

__device__ __forceinline__ int mbcnt64(uint64_t m)   // set bits of m below this lane
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

// Inclusive prefix sum over the 64 lanes (lane l gets x_0 + ... + x_l) with data-parallel-primitive
// moves: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0 / 2 is added
// to row 1 / 3 and the last lane of row 1 to rows 2 and 3.  Lanes with no source add 0.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);   // row_shr 1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);   // row_shr 2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);   // row_shr 4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);   // row_shr 8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);   // row_bcast 15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);   // row_bcast 31 -> rows 2, 3
    return v;
}

// Sum over the 64 lanes, returned wave-uniform (same moves as the prefix sum; lane 63 ends with the total).
__device__ __forceinline__ float wave_total_f32(float v)
{
    auto step = [&](auto ctrl, auto rmask) {
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value,
                                                        decltype(rmask)::value, 0xF, false));
    };
    step(std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xF>{});
    step(std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xF>{});
    step(std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xF>{});
    step(std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xF>{});
    step(std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xA>{});
    step(std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xC>{});
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// One wave-uniform value into lane `lane_id` of a register.
__device__ __forceinline__ void write_lane1(uint32_t &a, uint32_t va, int lane_id)
{
    asm("s_mov_b32 m0, %2\n\t"
        "v_writelane_b32 %0, %1, m0"
        : "+v"(a)
        : "s"(va), "s"(lane_id)
        : "m0");
}

__device__ __forceinline__ void prune_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}


}  // namespace spark
