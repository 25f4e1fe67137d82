// Device-side arithmetic shared by the kernels: the two forms of ceil(a/d) of the cost
// model (section 2: execution time c/s, transfer time t/B, each rounded up to whole ticks)
// and lane permutations inside a row of 16 lanes.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "cpeval_internal.hpp"

namespace cpeval {

// ceil(a/d) through the multiply-shift constants of the cost tables; {0, 0} (a free transfer)
// yields 0.  Exact for every a the table was built for.
__device__ __forceinline__ uint32_t magic_div(uint32_t a, Magic mg) {
    uint32_t nn = a + mg.dm1;
    return (uint32_t)(((uint64_t)nn * mg.mul + nn) >> 32);
}

// The same through a 4-byte table entry (d - 1 in the low byte, the upper 24 bits of the
// multiplier above it; the multiplier's low byte is taken as all ones); 0 (a free transfer)
// yields 0 for every a < 2^24.  Exact for every a the entry was built for.
__device__ __forceinline__ uint32_t magic_div(uint32_t a, uint32_t entry) {
    uint32_t nn = a + (entry & 0xffu);
    return (uint32_t)(((uint64_t)nn * (entry | 0xffu) + nn) >> 32);
}

// ceil(a/d) by division; d = 0 marks a free transfer.
__device__ __forceinline__ uint64_t plain_div(uint64_t a, uint64_t d) {
    return d ? (a + d - 1) / d : 0;
}

// x of the lane a DPP control word names (a permutation inside each row of 16 lanes):
// 0xB1 swaps neighbours, 0x4E swaps pairs, 0x141 mirrors halves of 8, 0x140 mirrors the row.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}

template <int CTRL>
__device__ __forceinline__ long long dpp_i64(long long x) {
    const uint32_t lo = dpp_u32<CTRL>((uint32_t)x);
    const uint32_t hi = dpp_u32<CTRL>((uint32_t)((unsigned long long)x >> 32));
    return (long long)(((unsigned long long)hi << 32) | lo);
}

}  // namespace cpeval
