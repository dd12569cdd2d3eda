// The library's counter-based generator (stated in include/moshpit.h): one 64-bit
// mixer shared by the failure schedule, the random order of peers and the donor draw.
// The paper names no generator (Sec. 4.1 only says that peers fail with probability p).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moshpit {

__device__ __forceinline__ uint64_t mix64(uint64_t x)
{
    x ^= x >> 32; x *= 0x9E3779B97F4A7C15ull;
    x ^= x >> 29; x *= 0x6A09E667F3BCC909ull;
    x ^= x >> 32;
    return x;
}

// position of peer i in the random order of round t: smaller key first, ties by index
__device__ __forceinline__ uint64_t order_key(uint64_t seed, int64_t t, int64_t i)
{
    return mix64(mix64(seed + 0xD1B54A32D192ED03ull * static_cast<uint64_t>(t + 1)) ^ static_cast<uint64_t>(i));
}

}  // namespace moshpit
