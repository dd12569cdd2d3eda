// Sorting of 128-bit items on the device, for gfx950: the integer side of the rounds
// whose groups come from a random order of the peers (the permutation of Thm 3.2's
// scheme, App. C.3; the random order of peers_t in Alg. 1).
//
// An item is (hi, lo), compared lexicographically.  Callers pack what they sort by into
// it - (order key, peer) or (group key, order key, peer) - so that items are distinct and
// the sorted order is unique: the result is bit-exact whatever the launch shape.
//
// Bitonic network over n = 2^k items (the caller pads with items that compare last).
// Blocks of 1024 threads keep chunks of 4096 items (64 KiB) in LDS: one kernel sorts
// every chunk completely (all stages up to 4096, direction taken from the item's global
// position so that the chunks form the bitonic sequences of the next stage); for larger
// n every further stage is a few one-comparator-per-thread passes over global memory
// (partners >= 4096 apart) and one LDS pass per chunk for the rest.  4096 peers, the
// largest workload here, are one launch.
#include "moshpit_internal.h"

namespace moshpit {
namespace {

constexpr int kChunk = 4096;            // items per block
constexpr int kSortThreads = 1024;

__device__ __forceinline__ bool item_less(const SortItem &a, const SortItem &b)
{
    return a.hi < b.hi || (a.hi == b.hi && a.lo < b.lo);
}

// Steps j = j_first, j_first/2, ..., 1 of stage k on the chunk held in sh[]; base = global
// position of sh[0] (ascending where (position & k) == 0).
__device__ __forceinline__ void chunk_steps(SortItem *sh, int64_t base, int64_t k, int j_first)
{
    for (int j = j_first; j >= 1; j >>= 1) {
#pragma unroll
        for (int c0 = 0; c0 < kChunk / 2; c0 += kSortThreads) {
            const int c = c0 + static_cast<int>(threadIdx.x);
            const int i = ((c & ~(j - 1)) << 1) | (c & (j - 1));
            const int l = i | j;
            const SortItem a = sh[i], b = sh[l];
            const bool ascending = ((base + i) & k) == 0;
            if (item_less(b, a) == ascending) {
                sh[i] = b;
                sh[l] = a;
            }
        }
        __syncthreads();
    }
}

// Every chunk sorted: all stages k = 2 .. kChunk.
__global__ __launch_bounds__(kSortThreads) void sort_chunks_kernel(SortItem *__restrict__ items)
{
    __shared__ SortItem sh[kChunk];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kChunk;
    for (int i = threadIdx.x; i < kChunk; i += kSortThreads) sh[i] = items[base + i];
    __syncthreads();
    for (int k = 2; k <= kChunk; k <<= 1) chunk_steps(sh, base, k, k >> 1);
    for (int i = threadIdx.x; i < kChunk; i += kSortThreads) items[base + i] = sh[i];
}

// One step of stage k with partners j >= kChunk apart: one comparator per thread.
__global__ __launch_bounds__(256) void sort_global_step_kernel(SortItem *__restrict__ items, int64_t n, int64_t k,
                                                               int64_t j)
{
    const int64_t c = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (c >= n / 2) return;
    const int64_t i = ((c & ~(j - 1)) << 1) | (c & (j - 1));
    const int64_t l = i | j;
    const SortItem a = items[i], b = items[l];
    const bool ascending = (i & k) == 0;
    if (item_less(b, a) == ascending) {
        items[i] = b;
        items[l] = a;
    }
}

// The steps j = kChunk/2 .. 1 of stage k > kChunk, chunk by chunk in LDS.
__global__ __launch_bounds__(kSortThreads) void sort_merge_chunks_kernel(SortItem *__restrict__ items, int64_t k)
{
    __shared__ SortItem sh[kChunk];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kChunk;
    for (int i = threadIdx.x; i < kChunk; i += kSortThreads) sh[i] = items[base + i];
    __syncthreads();
    chunk_steps(sh, base, k, kChunk >> 1);
    for (int i = threadIdx.x; i < kChunk; i += kSortThreads) items[base + i] = sh[i];
}

}  // namespace

int64_t sort_padded_count(int64_t n)
{
    int64_t p = kChunk;
    while (p < n) p <<= 1;
    return p;
}

hipError_t launch_sort_items(SortItem *items, int64_t n_padded, hipStream_t stream)
{
    if (n_padded < kChunk || (n_padded & (n_padded - 1)) != 0) return hipErrorInvalidValue;
    const int64_t chunks = n_padded / kChunk;
    if (chunks > 0x7fffffffLL) return hipErrorInvalidValue;
    sort_chunks_kernel<<<dim3(static_cast<uint32_t>(chunks)), dim3(kSortThreads), 0, stream>>>(items);
    for (int64_t k = 2 * kChunk; k <= n_padded; k <<= 1) {
        const uint32_t blocks = static_cast<uint32_t>((n_padded / 2 + 255) / 256);
        for (int64_t j = k >> 1; j >= kChunk; j >>= 1)
            sort_global_step_kernel<<<dim3(blocks), dim3(256), 0, stream>>>(items, n_padded, k, j);
        sort_merge_chunks_kernel<<<dim3(static_cast<uint32_t>(chunks)), dim3(kSortThreads), 0, stream>>>(items, k);
    }
    return hipGetLastError();
}

}  // namespace moshpit
