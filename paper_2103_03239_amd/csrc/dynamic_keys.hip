// Alg. 1 with chunk-index keys, integer side, for gfx950.
//
// Every peer carries the key C_i of its d-1 most recent chunk indices (Eq. 1);
// peers with equal keys that take part in a round form a group (cut into
// groups of at most M in the round's random order), and each member shifts its
// position within the group into its key: C_i := (C_i[1:], c_i) (Alg. 1, last
// line of the loop).  These kernels turn (keys, alive, seed, t) into a padded
// peer list - group g occupies entries [g*M, (g+1)*M), unused entries are -1 -
// which the peer-list instantiation of the group-mean kernel then averages,
// and update the keys.  Pure integer work: bit-exact against the CPU oracle.
//
// A peer's rank among the participants that carry its key comes from one device
// sort of the items (key, order key of the round, peer): the participants of a key
// end up next to each other in the round's random order, and the rank is the
// distance to the first of them.
#include "mix64.h"
#include "moshpit_internal.h"

namespace moshpit {
namespace {

// keys[i][q] = coordinate q+1 of peer i (Eq. 2): the first round groups M consecutive peers
__global__ __launch_bounds__(256) void dyn_init_kernel(int64_t N, int32_t M, int32_t kd, int32_t *__restrict__ keys)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= N) return;
    int64_t rest = i / M;
    for (int32_t q = 0; q < kd; ++q) {
        keys[i * kd + q] = static_cast<int32_t>(rest % M);
        rest /= M;
    }
}

// packed[i] = key of peer i as a base-M number, or -1 if it sits the round out; count[] and index[] cleared
__global__ __launch_bounds__(256) void dyn_pack_kernel(int64_t N, int32_t M, int32_t kd, const int32_t *__restrict__ keys,
                                                       const uint8_t *__restrict__ alive, int32_t *__restrict__ packed,
                                                       int32_t *__restrict__ count, int64_t n_keys,
                                                       int32_t *__restrict__ index, int64_t n_index)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < N) {
        int32_t pk = -1;
        if (alive == nullptr || alive[i] != 0) {
            pk = 0;
            int32_t weight = 1;
            for (int32_t q = 0; q < kd; ++q) {
                pk += keys[i * kd + q] * weight;
                weight *= M;
            }
        }
        packed[i] = pk;
    }
    if (i <= n_keys) count[i] = 0;
    if (i < n_index) index[i] = -1;
}

__global__ __launch_bounds__(256) void dyn_count_kernel(int64_t N, const int32_t *__restrict__ packed,
                                                        int32_t *__restrict__ count)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < N && packed[i] >= 0) atomicAdd(&count[packed[i]], 1);
}

// first[k] = number of groups owned by keys < k, a key with c members owning ceil(c / M) groups
__global__ __launch_bounds__(1024) void dyn_scan_kernel(int64_t n_keys, int32_t M, const int32_t *__restrict__ count,
                                                        int32_t *__restrict__ first)
{
    __shared__ int32_t part[1024];
    const int tid = threadIdx.x;
    const int64_t per = (n_keys + 1023) / 1024;
    const int64_t k0 = tid * per, k1 = (k0 + per < n_keys) ? k0 + per : n_keys;
    int32_t sum = 0;
    for (int64_t k = k0; k < k1; ++k) sum += (count[k] + M - 1) / M;
    part[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        int32_t run = 0;
        for (int q = 0; q < 1024; ++q) {
            const int32_t v = part[q];
            part[q] = run;
            run += v;
        }
    }
    __syncthreads();
    int32_t run = part[tid];
    for (int64_t k = k0; k < k1; ++k) {
        first[k] = run;
        run += (count[k] + M - 1) / M;
    }
}

// item of peer i: (key, order key, i) packed as hi = key << 32 | order >> 32,
// lo = order << 32 | i; peers that sit the round out (key -1) and the padding sort last
__global__ __launch_bounds__(256) void dyn_items_kernel(int64_t N, int64_t n_padded, uint64_t seed, int64_t t,
                                                        const int32_t *__restrict__ packed,
                                                        SortItem *__restrict__ items)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n_padded) return;
    SortItem it{~0ull, ~0ull};
    if (i < N) {
        const uint64_t order = order_key(seed, t, i);
        it.hi = (static_cast<uint64_t>(static_cast<uint32_t>(packed[i])) << 32) | (order >> 32);
        it.lo = (order << 32) | static_cast<uint64_t>(i);
    }
    items[i] = it;
}

// sorted position r -> the peer there, its rank among the participants with its key
// (distance to the first item of that key, found by bisection), its slot in the padded
// list and its new key
__global__ __launch_bounds__(256) void dyn_place_kernel(int64_t N, int32_t M, int32_t kd,
                                                        const SortItem *__restrict__ items,
                                                        const int32_t *__restrict__ first, int32_t *__restrict__ keys,
                                                        int32_t *__restrict__ index)
{
    const int64_t r = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (r >= N) return;
    const SortItem it = items[r];
    const uint32_t pk = static_cast<uint32_t>(it.hi >> 32);
    if (pk == 0xffffffffu) return;                     // sits the round out
    const int64_t i = static_cast<int64_t>(it.lo & 0xffffffffull);
    int64_t lo = 0, hi = r;                            // smallest position whose key is pk
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (static_cast<uint32_t>(items[mid].hi >> 32) < pk) lo = mid + 1;
        else hi = mid;
    }
    const int64_t rank = r - lo;
    const int32_t chunk = static_cast<int32_t>(rank % M);   // c_i: position within its group of at most M
    index[(static_cast<int64_t>(first[pk]) + rank / M) * M + chunk] = static_cast<int32_t>(i);
    if (kd > 0) {
        for (int32_t q = 0; q + 1 < kd; ++q) keys[i * kd + q] = keys[i * kd + q + 1];
        keys[i * kd + kd - 1] = chunk;
    }
}

}  // namespace

hipError_t launch_dynamic_init(int64_t N, int32_t M, int32_t d, int32_t *keys, hipStream_t stream)
{
    const uint32_t blocks = static_cast<uint32_t>((N + 255) / 256);
    dyn_init_kernel<<<dim3(blocks), dim3(256), 0, stream>>>(N, M, d - 1, keys);
    return hipGetLastError();
}

hipError_t launch_dynamic_grouping(int64_t N, int32_t M, int32_t d, uint64_t seed, int64_t t, const uint8_t *alive,
                                   int32_t *keys, int32_t *packed, int32_t *count, int32_t *first, int32_t *index,
                                   int64_t n_index, SortItem *items, hipStream_t stream)
{
    int64_t n_keys = 1;
    for (int32_t q = 0; q + 1 < d; ++q) n_keys *= M;
    int64_t span = N > n_keys + 1 ? N : n_keys + 1;
    if (n_index > span) span = n_index;
    const uint32_t blocks_all = static_cast<uint32_t>((span + 255) / 256);
    const uint32_t blocks_n = static_cast<uint32_t>((N + 255) / 256);
    dyn_pack_kernel<<<dim3(blocks_all), dim3(256), 0, stream>>>(N, M, d - 1, keys, alive, packed, count, n_keys, index,
                                                               n_index);
    dyn_count_kernel<<<dim3(blocks_n), dim3(256), 0, stream>>>(N, packed, count);
    dyn_scan_kernel<<<dim3(1), dim3(1024), 0, stream>>>(n_keys, M, count, first);
    const int64_t n_padded = sort_padded_count(N);
    dyn_items_kernel<<<dim3(static_cast<uint32_t>((n_padded + 255) / 256)), dim3(256), 0, stream>>>(N, n_padded, seed, t,
                                                                                                    packed, items);
    hipError_t e = launch_sort_items(items, n_padded, stream);
    if (e != hipSuccess) return e;
    dyn_place_kernel<<<dim3(blocks_n), dim3(256), 0, stream>>>(N, M, d - 1, items, first, keys, index);
    return hipGetLastError();
}

}  // namespace moshpit
