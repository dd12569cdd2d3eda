// A returning peer takes the parameters of an up-to-date peer before it takes
// part again (App. "Training with a dynamic number of peers"), for gfx950.
//
// Peer i returns in round t when it is present in round t and was absent in
// round t-1; the up-to-date peers it can reach are those present in both
// rounds; its donor is the (u mod c)-th of these c candidates in ascending
// index, u = mix(mix(seed + 0xA0761D6478BD642F*(t+1)) ^ i) with the mixer of
// the failure schedule.  Two kernels: an integer one that draws the donors and
// lists the returning peers, and a copy kernel that moves 2*s*P bytes per
// returning peer at streaming rate.  Donors never return themselves, so the
// copies are independent of each other and run in place.
#include "moshpit_internal.h"

namespace moshpit {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPlanThreads = 1024;
constexpr int kCopyThreads = 256;
constexpr int kCopyVectors = 8;                               // 128-bit vectors per thread and chunk
constexpr int64_t kChunkBytes = int64_t(kCopyThreads) * kCopyVectors * 16;   // 32 KiB of a row per block

__device__ __forceinline__ uint64_t mix64(uint64_t x)
{
    x ^= x >> 32; x *= 0x9E3779B97F4A7C15ull;
    x ^= x >> 29; x *= 0x6A09E667F3BCC909ull;
    x ^= x >> 32;
    return x;
}

// Stable compaction step of one block: every thread passes `flag`, gets the
// number of set flags of the threads before it; *total gets the block's count.
__device__ __forceinline__ int block_rank(bool flag, int *wave_sums, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long ballot = __ballot(flag);
    const int before = __popcll(ballot & ((1ull << lane) - 1ull));
    if (lane == 0) wave_sums[wave] = __popcll(ballot);
    __syncthreads();
    int base = 0, all = 0;
    for (int w = 0; w < kPlanThreads / 64; ++w) {
        const int c = wave_sums[w];
        if (w < wave) base += c;
        all += c;
    }
    __syncthreads();
    *total = all;
    return base + before;
}

// One block.  candidates: scratch, N int32.  donor[i] = donor of peer i or -1;
// returning[0..counts[1]) = the returning peers that have a donor, ascending;
// counts[0] = number of candidates, counts[1] = number of returning peers.
__global__ __launch_bounds__(kPlanThreads) void refresh_plan_kernel(const uint8_t *__restrict__ prev,
                                                                     const uint8_t *__restrict__ cur, int64_t N,
                                                                     uint64_t seed, int64_t t,
                                                                     int32_t *__restrict__ candidates,
                                                                     int32_t *__restrict__ donor,
                                                                     int32_t *__restrict__ returning,
                                                                     int32_t *__restrict__ counts)
{
    __shared__ int wave_sums[kPlanThreads / 64];
    int64_t c = 0;
    for (int64_t j0 = 0; j0 < N; j0 += kPlanThreads) {
        const int64_t j = j0 + threadIdx.x;
        const bool is_cand = j < N && prev[j] != 0 && cur[j] != 0;
        int total = 0;
        const int rank = block_rank(is_cand, wave_sums, &total);
        if (is_cand) candidates[c + rank] = static_cast<int32_t>(j);
        c += total;
    }
    __syncthreads();                                  // candidates[] written by other threads are read below
    const uint64_t round_key = mix64(seed + 0xA0761D6478BD642Full * static_cast<uint64_t>(t + 1));
    int64_t n_ret = 0;
    for (int64_t i0 = 0; i0 < N; i0 += kPlanThreads) {
        const int64_t i = i0 + threadIdx.x;
        const bool returns = i < N && c > 0 && cur[i] != 0 && prev[i] == 0;
        int total = 0;
        const int rank = block_rank(returns, wave_sums, &total);
        if (i < N) {
            int32_t from = -1;
            if (returns) {
                const uint64_t u = mix64(round_key ^ static_cast<uint64_t>(i));
                from = candidates[u % static_cast<uint64_t>(c)];
                returning[n_ret + rank] = static_cast<int32_t>(i);
            }
            donor[i] = from;
        }
        n_ret += total;
    }
    if (threadIdx.x == 0) {
        counts[0] = static_cast<int32_t>(c);
        counts[1] = static_cast<int32_t>(n_ret);
    }
}

// Block (x, y): the x-th 32 KiB chunk of the rows of returning peers y, y +
// gridDim.y, ...  VEC: rows are 16-byte aligned (128-bit copies, the ragged end
// of a row element by element); otherwise everything element by element.
template <int ESIZE, bool VEC>
__global__ __launch_bounds__(kCopyThreads) void refresh_copy_kernel(char *__restrict__ X, int64_t row_bytes,
                                                                     int64_t valid_bytes,
                                                                     const int32_t *__restrict__ donor,
                                                                     const int32_t *__restrict__ returning,
                                                                     const int32_t *__restrict__ counts)
{
    typedef typename std::conditional<ESIZE == 4, uint32_t, uint16_t>::type elem_t;
    const int32_t n_ret = counts[1];
    const int64_t c0 = static_cast<int64_t>(blockIdx.x) * kChunkBytes;
    const int64_t c1 = c0 + kChunkBytes < valid_bytes ? c0 + kChunkBytes : valid_bytes;
    for (int32_t r = blockIdx.y; r < n_ret; r += gridDim.y) {
        const int64_t i = returning[r];
        const char *src = X + static_cast<int64_t>(donor[i]) * row_bytes;
        char *dst = X + i * row_bytes;
        if (VEC) {
            const int64_t v_end = c1 / 16 * 16;
            u32x4 val[kCopyVectors];
#pragma unroll
            for (int k = 0; k < kCopyVectors; ++k) {
                const int64_t o = c0 + (static_cast<int64_t>(k) * kCopyThreads + threadIdx.x) * 16;
                if (o < v_end) val[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + o));
            }
#pragma unroll
            for (int k = 0; k < kCopyVectors; ++k) {
                const int64_t o = c0 + (static_cast<int64_t>(k) * kCopyThreads + threadIdx.x) * 16;
                if (o < v_end) __builtin_nontemporal_store(val[k], reinterpret_cast<u32x4 *>(dst + o));
            }
            for (int64_t o = v_end + static_cast<int64_t>(threadIdx.x) * ESIZE; o < c1; o += kCopyThreads * ESIZE)
                *reinterpret_cast<elem_t *>(dst + o) = *reinterpret_cast<const elem_t *>(src + o);
        } else {
            for (int64_t o = c0 + static_cast<int64_t>(threadIdx.x) * ESIZE; o < c1; o += kCopyThreads * ESIZE)
                *reinterpret_cast<elem_t *>(dst + o) = *reinterpret_cast<const elem_t *>(src + o);
        }
    }
}

}  // namespace

hipError_t launch_refresh_plan(const uint8_t *prev, const uint8_t *cur, int64_t N, uint64_t seed, int64_t t,
                               int32_t *candidates, int32_t *donor, int32_t *returning, int32_t *counts,
                               hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    refresh_plan_kernel<<<dim3(1), dim3(kPlanThreads), 0, stream>>>(prev, cur, N, seed, t, candidates, donor,
                                                                    returning, counts);
    return hipGetLastError();
}

hipError_t launch_refresh_copy(void *X, int dtype, int64_t N, int64_t P, int64_t row_stride, const int32_t *donor,
                               const int32_t *returning, const int32_t *counts, hipStream_t stream)
{
    if (N <= 0 || P <= 0) return hipSuccess;
    const int64_t esize = dtype == 0 ? 4 : 2;
    const int64_t row_bytes = row_stride * esize, valid = P * esize;
    const int64_t chunks = (valid + kChunkBytes - 1) / kChunkBytes;
    if (chunks > 0x7fffffffLL) return hipErrorInvalidValue;
    // the number of returning peers is known on the device only: enough rows of blocks
    // for a few thousand peers at once, further ones are reached by the stride loop
    const uint32_t rows = static_cast<uint32_t>(N < 4096 ? N : 4096);
    const bool vec = reinterpret_cast<uintptr_t>(X) % 16 == 0 && row_bytes % 16 == 0;
    const dim3 grid(static_cast<uint32_t>(chunks), rows), block(kCopyThreads);
    char *base = static_cast<char *>(X);
    if (dtype == 0) {
        if (vec) refresh_copy_kernel<4, true><<<grid, block, 0, stream>>>(base, row_bytes, valid, donor, returning, counts);
        else refresh_copy_kernel<4, false><<<grid, block, 0, stream>>>(base, row_bytes, valid, donor, returning, counts);
    } else {
        if (vec) refresh_copy_kernel<2, true><<<grid, block, 0, stream>>>(base, row_bytes, valid, donor, returning, counts);
        else refresh_copy_kernel<2, false><<<grid, block, 0, stream>>>(base, row_bytes, valid, donor, returning, counts);
    }
    return hipGetLastError();
}

}  // namespace moshpit
