// How the averaging kernels move VE elements of a row as one memory access and widen them
// to binary32, for gfx950: 128-bit vectors of 4 binary32 or 8 bfloat16 values, and the
// single-element forms used for ragged row ends and misaligned rows.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bf16_round.h"

namespace moshpit {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// How VE elements of storage type DT travel as one memory access and widen to
// binary32.
template <int DT, int VE> struct Vec;

template <> struct Vec<0, 4> {
    typedef f32x4 mem_t;
    static constexpr int NE = 4;
    static __device__ __forceinline__ mem_t zero() { return mem_t{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ void widen(const mem_t &m, float (&f)[NE])
    {
        f[0] = m.x; f[1] = m.y; f[2] = m.z; f[3] = m.w;
    }
    static __device__ __forceinline__ mem_t narrow(const float (&f)[NE]) { return mem_t{f[0], f[1], f[2], f[3]}; }
};

template <> struct Vec<0, 1> {
    typedef float mem_t;
    static constexpr int NE = 1;
    static __device__ __forceinline__ mem_t zero() { return 0.f; }
    static __device__ __forceinline__ void widen(const mem_t &m, float (&f)[NE]) { f[0] = m; }
    static __device__ __forceinline__ mem_t narrow(const float (&f)[NE]) { return f[0]; }
};

template <> struct Vec<1, 8> {
    typedef u32x4 mem_t;
    static constexpr int NE = 8;
    static __device__ __forceinline__ mem_t zero() { return mem_t{0u, 0u, 0u, 0u}; }
    static __device__ __forceinline__ void widen(const mem_t &m, float (&f)[NE])
    {
        const uint32_t w[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f[2 * k] = __uint_as_float(w[k] << 16);             // even element: low half
            f[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u); // odd element: high half
        }
    }
    static __device__ __forceinline__ mem_t narrow(const float (&f)[NE])
    {
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) w[k] = bf16_pair(f[2 * k], f[2 * k + 1]);
        return mem_t{w[0], w[1], w[2], w[3]};
    }
};

template <> struct Vec<1, 1> {
    typedef uint16_t mem_t;
    static constexpr int NE = 1;
    static __device__ __forceinline__ mem_t zero() { return 0; }
    static __device__ __forceinline__ void widen(const mem_t &m, float (&f)[NE])
    {
        f[0] = __uint_as_float(static_cast<uint32_t>(m) << 16);
    }
    static __device__ __forceinline__ mem_t narrow(const float (&f)[NE])
    {
        return bf16_one(f[0]);
    }
};

template <bool NT, typename T> __device__ __forceinline__ T load_vec(const T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename T> __device__ __forceinline__ void store_vec(T *p, const T &v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

}  // namespace moshpit
