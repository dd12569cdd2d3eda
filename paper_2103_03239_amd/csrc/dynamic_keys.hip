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
// N is at most 65536, so ranks are found by counting (one thread per peer
// scans all peers) instead of sorting.
#include "moshpit_internal.h"

namespace moshpit {
namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t x)
{
    x ^= x >> 32; x *= 0x9E3779B97F4A7C15ull;
    x ^= x >> 29; x *= 0x6A09E667F3BCC909ull;
    x ^= x >> 32;
    return x;
}

// position of peer i in the random order of round t (smaller key first, ties by index)
__device__ __forceinline__ uint64_t order_key(uint64_t seed, int64_t t, int64_t i)
{
    return mix64(mix64(seed + 0xD1B54A32D192ED03ull * static_cast<uint64_t>(t + 1)) ^ static_cast<uint64_t>(i));
}

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

// rank of peer i among the participants with its key -> its slot in the padded list and its new key
__global__ __launch_bounds__(256) void dyn_place_kernel(int64_t N, int32_t M, int32_t kd, uint64_t seed, int64_t t,
                                                        const int32_t *__restrict__ packed,
                                                        const int32_t *__restrict__ first, int32_t *__restrict__ keys,
                                                        int32_t *__restrict__ index)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= N) return;
    const int32_t pk = packed[i];
    if (pk < 0) return;
    const uint64_t ki = order_key(seed, t, i);
    int32_t rank = 0;
    for (int64_t j = 0; j < N; ++j) {
        if (packed[j] != pk) continue;
        const uint64_t kj = order_key(seed, t, j);
        rank += (kj < ki || (kj == ki && j < i)) ? 1 : 0;
    }
    const int32_t chunk = rank % M;                    // c_i: position within its group of at most M
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
                                   int64_t n_index, hipStream_t stream)
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
    dyn_place_kernel<<<dim3(blocks_n), dim3(256), 0, stream>>>(N, M, d - 1, seed, t, packed, first, keys, index);
    return hipGetLastError();
}

}  // namespace moshpit
