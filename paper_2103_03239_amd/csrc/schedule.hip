// Integer side of a round on the device: the seeded failure schedule and the
// group keys (Eq. 1 on the static grid).  Pure 64-bit integer arithmetic, so
// results are bit-exact and independent of launch shape.
#include "mix64.h"
#include "moshpit_internal.h"

namespace moshpit {
namespace {

// Failure events from the counter-based generator (the paper only says that a
// peer fails in a round with probability p, Sec. 4.1; the mixer is this
// library's own and is stated in the public header).

__device__ __forceinline__ bool failure_event(uint64_t seed, int64_t s, int64_t i, uint32_t threshold)
{
    const uint64_t round_key = mix64(seed + 0x9E3779B97F4A7C15ull * static_cast<uint64_t>(s + 1));
    const uint64_t u = mix64(round_key ^ static_cast<uint64_t>(i));
    return static_cast<uint32_t>(u >> 40) < threshold;
}

// One thread per peer; the thread walks the rounds because a peer's absence
// depends on when its last one started (kind 2).  For kind 2 the walk starts at
// round s_begin <= t0 with away_in[i] rounds still to sit out (s_begin = 0 and
// nothing to sit out when away_in is null), and away_out[i] receives the state
// at the start of round t0 + rounds, from which a later call can go on.
__global__ __launch_bounds__(256) void schedule_kernel(int kind, uint32_t threshold, uint64_t seed, int down,
                                                       int64_t N, int64_t t0, int rounds,
                                                       uint8_t *__restrict__ masks, int64_t s_begin,
                                                       const int32_t *away_in, int32_t *away_out)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= N) return;
    if (kind == 0) {
        for (int r = 0; r < rounds; ++r) masks[static_cast<int64_t>(r) * N + i] = 1;
    } else if (kind == 1) {
        for (int r = 0; r < rounds; ++r)
            masks[static_cast<int64_t>(r) * N + i] = failure_event(seed, t0 + r, i, threshold) ? 0 : 1;
    } else {
        int away = away_in != nullptr ? away_in[i] : 0;   // rounds still to sit out
        for (int64_t s = s_begin; s < t0 + rounds; ++s) {
            if (away == 0 && failure_event(seed, s, i, threshold)) away = down;
            const uint8_t present = away == 0 ? 1 : 0;
            if (away > 0) --away;
            if (s >= t0) masks[(s - t0) * N + i] = present;
        }
        if (away_out != nullptr) away_out[i] = away;
    }
}

// Group-skip behaviour (Sec. 3.1: a peer that fails during the all-reduce makes
// its groupmates skip the round).  One wave per (round, group): if any member
// of the group is absent, every member's byte is cleared.  In place: a group's
// bytes belong to that group alone.
__global__ __launch_bounds__(64) void skip_filter_kernel(uint8_t *__restrict__ masks, int64_t N, int32_t M, int32_t d,
                                                          int64_t t0, int64_t groups)
{
    const int64_t r = blockIdx.x / groups;
    const int64_t g = blockIdx.x - r * groups;
    int64_t S = 1;
    for (int64_t q = 0; q < (t0 + r) % d; ++q) S *= M;
    const int64_t base = (g / S) * S * M + (g % S);
    const int lane = threadIdx.x;
    uint8_t *mine = masks + r * N + base + static_cast<int64_t>(lane) * S;
    const bool absent = lane < M && *mine == 0;
    if (__ballot(absent) != 0 && lane < M) *mine = 0;
}

// Random permutation for the random-group scheme analysed in Thm 3.2 (its proof
// in App. C.3 draws a permutation and cuts it into consecutive groups).  Peers
// are ordered by key(seed,t,i) = mix(mix(seed + 0xD1B54A32D192ED03*(t+1)) ^ i),
// ties by index: the items (key, i) are sorted on the device and perm[r] is the
// peer of the r-th item.
__global__ __launch_bounds__(256) void permutation_items_kernel(uint64_t seed, int64_t t, int64_t N, int64_t n_padded,
                                                                SortItem *__restrict__ items)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n_padded) return;
    items[i] = i < N ? SortItem{order_key(seed, t, i), static_cast<uint64_t>(i)} : SortItem{~0ull, ~0ull};
}

__global__ __launch_bounds__(256) void permutation_extract_kernel(const SortItem *__restrict__ items, int64_t N,
                                                                  int32_t *__restrict__ perm)
{
    const int64_t r = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (r < N) perm[r] = static_cast<int32_t>(items[r].lo);
}

// key(i) = the base-M number formed by the digits of i other than digit a,
// i.e. floor(i / (S*M)) * S + i mod S with S = M^a.
__global__ __launch_bounds__(256) void group_keys_kernel(int64_t N, int32_t M, int64_t S, int32_t *__restrict__ keys)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= N) return;
    keys[i] = static_cast<int32_t>((i / (S * M)) * S + (i % S));
}

}  // namespace

hipError_t launch_schedule(int kind, uint32_t threshold, uint64_t seed, int down, int64_t N, int64_t t0,
                           int rounds, uint8_t *masks, int64_t s_begin, const int32_t *away_in, int32_t *away_out,
                           hipStream_t stream)
{
    if (N <= 0 || rounds <= 0) return hipSuccess;
    const uint32_t blocks = static_cast<uint32_t>((N + 255) / 256);
    schedule_kernel<<<dim3(blocks), dim3(256), 0, stream>>>(kind, threshold, seed, down, N, t0, rounds, masks,
                                                            s_begin, away_in, away_out);
    return hipGetLastError();
}

hipError_t launch_skip_filter(uint8_t *masks, int64_t N, int32_t M, int32_t d, int64_t t0, int rounds,
                              hipStream_t stream)
{
    const int64_t groups = N / M;
    const int64_t blocks = groups * rounds;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    skip_filter_kernel<<<dim3(static_cast<uint32_t>(blocks)), dim3(64), 0, stream>>>(masks, N, M, d, t0, groups);
    return hipGetLastError();
}

hipError_t launch_random_permutation(uint64_t seed, int64_t t, int64_t N, int32_t *perm, SortItem *items,
                                     hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    const int64_t n_padded = sort_padded_count(N);
    permutation_items_kernel<<<dim3(static_cast<uint32_t>((n_padded + 255) / 256)), dim3(256), 0, stream>>>(
        seed, t, N, n_padded, items);
    hipError_t e = launch_sort_items(items, n_padded, stream);
    if (e != hipSuccess) return e;
    permutation_extract_kernel<<<dim3(static_cast<uint32_t>((N + 255) / 256)), dim3(256), 0, stream>>>(items, N, perm);
    return hipGetLastError();
}

hipError_t launch_group_keys(int64_t N, int32_t M, int64_t S, int32_t *keys, hipStream_t stream)
{
    if (N <= 0) return hipSuccess;
    const uint32_t blocks = static_cast<uint32_t>((N + 255) / 256);
    group_keys_kernel<<<dim3(blocks), dim3(256), 0, stream>>>(N, M, S, keys);
    return hipGetLastError();
}

}  // namespace moshpit
