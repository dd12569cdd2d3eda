// A returning peer takes the parameters of an up-to-date peer before it takes
// part again (App. "Training with a dynamic number of peers"), for gfx950.
//
// Peer i returns in round t when it is present in round t and was absent in
// round t-1; the up-to-date peers it can reach are those present in both
// rounds; its donor is the (u mod c)-th of these c candidates in ascending
// index, u = mix(mix(seed + 0xA0761D6478BD642F*(t+1)) ^ i) with the mixer of
// the failure schedule.  This file holds the integer kernel that draws the donors
// and lists the returning peers; the rows are then copied by the streaming copy
// kernel (2*s*P bytes per returning peer).  Donors never return themselves, so
// the copies are independent of each other and run in place.
#include "mix64.h"
#include "moshpit_internal.h"

namespace moshpit {
namespace {

constexpr int kPlanThreads = 1024;

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

}  // namespace moshpit
