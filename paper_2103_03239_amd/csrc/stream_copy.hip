// Streaming copies for gfx950 (MI355X): the plain copy that serves as the measured
// ceiling of a read+write stream (and as the known-size kernel that calibrates HBM
// traffic counters), and the copy of whole rows that lets a returning peer take the
// parameters of an up-to-date peer (App. "Training with a dynamic number of peers").
//
// Shape (measured on MI355X over block sizes 64-256, 1-8 vectors per thread and 4-32
// resident waves per compute unit): one-wave blocks, ONE 128-bit non-temporal load and
// store per lane, and as many resident waves as fit.  A plain copy of 8 GiB runs at
// 6.66 TB/s this way (5.75 TB/s with 256-thread blocks and 4 vectors per thread; every
// limit on the resident waves costs bandwidth here, unlike in the averaging kernel whose
// waves keep 16 loads in flight each).  The row copy reaches 6.3 TB/s with about a
// million blocks that walk the work items; fewer, longer-running blocks are slower
// (5.3 TB/s with 64 per compute unit).
#include "bf16_round.h"
#include "moshpit_internal.h"

namespace moshpit {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kLdsPerCu = 160 * 1024;

struct CopyShape {
    int block;          // threads per block: 64, 128 or 256
    int vecs;           // 128-bit vectors per thread and work item: 1, 2, 4 or 8
    int waves_per_cu;   // resident waves per compute unit (0 = no limit)
    int grid_per_cu;    // refresh only: blocks per compute unit walking the work items
};

size_t throttle_lds(const CopyShape &s)
{
    if (s.waves_per_cu <= 0 || s.waves_per_cu >= 32) return 0;
    int blocks_per_cu = s.waves_per_cu / (s.block / 64);
    if (blocks_per_cu < 1) blocks_per_cu = 1;
    return lds_bytes_for_blocks_per_cu(blocks_per_cu);
}

// Block b copies vectors [b * blockDim * VECS, (b + 1) * blockDim * VECS) of nvec.
template <int VECS>
__global__ __launch_bounds__(256) void copy_probe_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                         int64_t nvec)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * (blockDim.x * VECS) + threadIdx.x;
    u32x4 v[VECS];
#pragma unroll
    for (int u = 0; u < VECS; ++u)
        if (i + u * static_cast<int64_t>(blockDim.x) < nvec) v[u] = __builtin_nontemporal_load(src + i + u * blockDim.x);
#pragma unroll
    for (int u = 0; u < VECS; ++u)
        if (i + u * static_cast<int64_t>(blockDim.x) < nvec) __builtin_nontemporal_store(v[u], dst + i + u * blockDim.x);
}

// Work item w = (returning peer r = w / chunks, chunk c = w % chunks of blockDim * VECS
// vectors of its row); the blocks walk the items grid-stride, the number of items is
// read on the device (counts[1] returning peers).  VEC: rows are 16-byte aligned
// (128-bit copies, the ragged end of a row element by element by the block that has the
// row's last chunk); otherwise everything element by element.
template <int ESIZE, bool VEC, int VECS>
__global__ __launch_bounds__(256) void refresh_copy_kernel(char *__restrict__ X, int64_t row_bytes, int64_t valid_bytes,
                                                           int64_t chunks, const int32_t *__restrict__ donor,
                                                           const int32_t *__restrict__ returning,
                                                           const int32_t *__restrict__ counts)
{
    typedef typename std::conditional<ESIZE == 4, uint32_t, uint16_t>::type elem_t;
    const int64_t total = static_cast<int64_t>(counts[1]) * chunks;
    const int64_t chunk_bytes = static_cast<int64_t>(blockDim.x) * VECS * 16;
    for (int64_t w = blockIdx.x; w < total; w += gridDim.x) {
        const int64_t r = w / chunks, c = w - r * chunks;
        const int64_t i = returning[r];
        const char *src = X + static_cast<int64_t>(donor[i]) * row_bytes;
        char *dst = X + i * row_bytes;
        const int64_t c0 = c * chunk_bytes;
        const int64_t c1 = c0 + chunk_bytes < valid_bytes ? c0 + chunk_bytes : valid_bytes;
        if (VEC) {
            const int64_t v_end = c1 / 16 * 16;
            u32x4 val[VECS];
#pragma unroll
            for (int k = 0; k < VECS; ++k) {
                const int64_t o = c0 + (static_cast<int64_t>(k) * blockDim.x + threadIdx.x) * 16;
                if (o < v_end) val[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
            }
#pragma unroll
            for (int k = 0; k < VECS; ++k) {
                const int64_t o = c0 + (static_cast<int64_t>(k) * blockDim.x + threadIdx.x) * 16;
                if (o < v_end) __builtin_nontemporal_store(val[k], reinterpret_cast<u32x4 *>(dst + o));
            }
            for (int64_t o = v_end + static_cast<int64_t>(threadIdx.x) * ESIZE; o < c1; o += blockDim.x * ESIZE)
                *reinterpret_cast<elem_t *>(dst + o) = *reinterpret_cast<const elem_t *>(src + o);
        } else {
            for (int64_t o = c0 + static_cast<int64_t>(threadIdx.x) * ESIZE; o < c1; o += blockDim.x * ESIZE)
                *reinterpret_cast<elem_t *>(dst + o) = *reinterpret_cast<const elem_t *>(src + o);
        }
    }
}

template <int ESIZE, bool VEC, int VECS>
hipError_t launch_refresh_shape(const CopyShape &s, uint32_t grid, char *X, int64_t row_bytes, int64_t valid,
                                const int32_t *donor, const int32_t *returning, const int32_t *counts,
                                hipStream_t stream)
{
    auto kernel = refresh_copy_kernel<ESIZE, VEC, VECS>;
    const size_t lds = throttle_lds(s);
    if (lds > 0) {
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kernel), kLdsPerCu);
        if (e != hipSuccess) return e;
    }
    const int64_t chunk_bytes = static_cast<int64_t>(s.block) * VECS * 16;
    const int64_t chunks = (valid + chunk_bytes - 1) / chunk_bytes;
    kernel<<<dim3(grid), dim3(s.block), lds, stream>>>(X, row_bytes, valid, chunks, donor, returning, counts);
    return hipGetLastError();
}

template <int ESIZE, bool VEC>
hipError_t launch_refresh_vecs(const CopyShape &s, uint32_t grid, char *X, int64_t row_bytes, int64_t valid,
                               const int32_t *donor, const int32_t *returning, const int32_t *counts,
                               hipStream_t stream)
{
    switch (s.vecs) {
    case 1: return launch_refresh_shape<ESIZE, VEC, 1>(s, grid, X, row_bytes, valid, donor, returning, counts, stream);
    case 2: return launch_refresh_shape<ESIZE, VEC, 2>(s, grid, X, row_bytes, valid, donor, returning, counts, stream);
    case 4: return launch_refresh_shape<ESIZE, VEC, 4>(s, grid, X, row_bytes, valid, donor, returning, counts, stream);
    default: return launch_refresh_shape<ESIZE, VEC, 8>(s, grid, X, row_bytes, valid, donor, returning, counts, stream);
    }
}

}  // namespace

hipError_t launch_refresh_copy(void *X, int dtype, int64_t N, int64_t P, int64_t row_stride, const int32_t *donor,
                               const int32_t *returning, const int32_t *counts, int64_t expected_rows,
                               hipStream_t stream)
{
    if (N <= 0 || P <= 0) return hipSuccess;
    const int64_t esize = dtype == 0 ? 4 : 2;
    const int64_t row_bytes = row_stride * esize, valid = P * esize;
    const CopyShape s{64, 1, 0, 4096};
    int cus = 0;
    hipError_t e = current_compute_units(&cus);
    if (e != hipSuccess) return e;
    // About one block per work item the host expects (the device knows the true number and
    // the blocks walk the items, so a wrong guess costs time only: a block without work
    // costs about 0.2 ns of launch), between 64 and 4096 blocks per compute unit.
    const int64_t chunk_bytes = static_cast<int64_t>(s.block) * s.vecs * 16;
    const int64_t chunks = (valid + chunk_bytes - 1) / chunk_bytes;
    if (expected_rows < 1) expected_rows = 1;
    if (expected_rows > N) expected_rows = N;
    int64_t grid = expected_rows * chunks;
    if (grid < static_cast<int64_t>(cus) * 64) grid = static_cast<int64_t>(cus) * 64;
    if (grid > static_cast<int64_t>(cus) * s.grid_per_cu) grid = static_cast<int64_t>(cus) * s.grid_per_cu;
    if (grid > N * chunks) grid = N * chunks;
    const bool vec = reinterpret_cast<uintptr_t>(X) % 16 == 0 && row_bytes % 16 == 0;
    char *base = static_cast<char *>(X);
    const uint32_t g = static_cast<uint32_t>(grid);
    if (dtype == 0)
        return vec ? launch_refresh_vecs<4, true>(s, g, base, row_bytes, valid, donor, returning, counts, stream)
                   : launch_refresh_vecs<4, false>(s, g, base, row_bytes, valid, donor, returning, counts, stream);
    return vec ? launch_refresh_vecs<2, true>(s, g, base, row_bytes, valid, donor, returning, counts, stream)
               : launch_refresh_vecs<2, false>(s, g, base, row_bytes, valid, donor, returning, counts, stream);
}

namespace {
// Thread i converts the two binary32 numbers with bit patterns 2i and 2i + 1 both ways.
__global__ __launch_bounds__(256) void bf16_rounding_check_kernel(unsigned long long *mismatches)
{
    const uint64_t first = (static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x) * 2;
    const float lo = __uint_as_float(static_cast<uint32_t>(first));
    const float hi = __uint_as_float(static_cast<uint32_t>(first + 1));
    const uint32_t hw = bf16_pair(lo, hi);
    const uint32_t ref = (bf16_bits_reference(lo) & 0xffffu) | (bf16_bits_reference(hi) << 16);
    const uint32_t one = bf16_one(lo);
    const int bad = ((hw & 0xffffu) != (ref & 0xffffu) ? 1 : 0) + ((hw >> 16) != (ref >> 16) ? 1 : 0) +
                    (one != (ref & 0xffffu) ? 1 : 0);
    if (bad != 0) atomicAdd(mismatches, static_cast<unsigned long long>(bad));
}
}  // namespace

hipError_t launch_bf16_rounding_check(unsigned long long *mismatches, hipStream_t stream)
{
    bf16_rounding_check_kernel<<<dim3(1u << 23), dim3(256), 0, stream>>>(mismatches);    // 2^31 pairs
    return hipGetLastError();
}

hipError_t launch_copy_probe(void *dst, const void *src, int64_t nbytes, hipStream_t stream)
{
    const int64_t nvec = nbytes / 16;
    if (nvec <= 0) return hipSuccess;
    const CopyShape s{64, 1, 0, 0};
    const int64_t per_block = static_cast<int64_t>(s.block) * s.vecs;
    const int64_t blocks = (nvec + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t lds = throttle_lds(s);
    const dim3 grid(static_cast<uint32_t>(blocks)), block(s.block);
    u32x4 *d = static_cast<u32x4 *>(dst);
    const u32x4 *sv = static_cast<const u32x4 *>(src);
#define MOSHPIT_COPY(V)                                                                                     \
    if (s.vecs == V) {                                                                                      \
        if (lds > 0) {                                                                                      \
            hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(copy_probe_kernel<V>), kLdsPerCu); \
            if (e != hipSuccess) return e;                                                                  \
        }                                                                                                   \
        copy_probe_kernel<V><<<grid, block, lds, stream>>>(d, sv, nvec);                                    \
    }
    MOSHPIT_COPY(1)
    MOSHPIT_COPY(2)
    MOSHPIT_COPY(4)
    MOSHPIT_COPY(8)
#undef MOSHPIT_COPY
    return hipGetLastError();
}

}  // namespace moshpit
