// Group-mean round kernel for gfx950 (MI355X).
//
// One averaging round of Moshpit All-Reduce (Alg. 1, the AllReduce line; the
// group-average formula of App. C.3 with the group J_{i,t} of App. C.4) on N
// virtual peers stored as rows of X.  For round t the group g owns the M rows
// base(g) + j*S, S = M^(t mod d); every row whose peer takes part is replaced
// by the mean of the rows that take part.
//
// Mapping.  The reduction runs ACROSS rows, so each lane owns its columns for
// the whole group and no cross-lane traffic or LDS is needed: a work item is
// (group, column tile); a thread loads one 128-bit vector per participating
// row (COLS of them, 256 lanes apart, to keep more loads in flight when M is
// small), sums in binary32 registers, divides by the participant count and
// stores the mean to the same rows.  Rows of absent peers are never touched,
// so HBM traffic is 2 * elem_size * P bytes per participating peer.  In-place
// is safe because a work item reads and writes only its own (group, tile) and
// all its loads retire before its first store.
//
// The participant bitmap of a group is built by the wave itself: lane j < M
// reads alive[base + j*S] and a ballot gives a 64-bit mask (hence M <= 64).
#include "moshpit_internal.h"
#include "row_vec.h"

namespace moshpit {
namespace {

constexpr int kMaxBlock = 256;          // threads per block: 64, 128 or 256
constexpr int kLdsPerCu = 160 * 1024;   // gfx950: LDS bytes per compute unit

// X            state, byte pointer to element (row 0, first column of this launch)
// row_bytes    distance between rows in bytes
// nvec         vectors of VE elements per row covered by this launch
// tiles        ceil(nvec / (blockDim.x * COLS))
// work_items   groups * tiles
// IDX          groups are consecutive chunks of M entries of the peer list
//              index[0..n_index) (e.g. a random permutation) instead of grid lines
// SGD          the Moshpit SGD communication step (Alg. 2): what is averaged is
//              theta_j - gamma * g_j, g read from the matrix G laid out like X
//              (rows g_row_bytes apart); a peer that is alone in its group still
//              takes its local step
template <int DT, int VE, int COLS, int U, bool NT, bool IDX, bool SGD>
__global__ __launch_bounds__(kMaxBlock) void group_mean_kernel(char *X, int64_t row_bytes, int64_t nvec,
                                                            const uint8_t *__restrict__ alive, int32_t M,
                                                            int64_t S, int64_t tiles, int64_t work_items,
                                                            const int32_t *__restrict__ index, int64_t n_index,
                                                            const char *__restrict__ G, int64_t g_row_bytes,
                                                            float gamma, int order)
{
    typedef Vec<DT, VE> V;
    typedef typename V::mem_t mem_t;
    constexpr int NE = V::NE;
    const int lane = threadIdx.x & 63;
    const int kBlock = blockDim.x;

    for (int64_t w0 = blockIdx.x; w0 < work_items; w0 += gridDim.x) {
        int64_t w = w0;
        if (order == 1) {
            // blocks b, b + 8, b + 16, ... (they run on the same one of the 8 dies) take
            // consecutive work items: each die streams through an eighth of the list
            const int64_t per = (work_items + 7) >> 3;
            w = (w0 & 7) * per + (w0 >> 3);
            if (w >= work_items) continue;
        }
        const int64_t g = w / tiles;
        const int64_t tile = w - g * tiles;
        int64_t base = 0;
        int32_t my_row = -1;                         // IDX: the row of position `lane`
        bool takes_part = false;
        if constexpr (IDX) {
            const int64_t pos = g * M + lane;
            if (lane < M && pos < n_index) my_row = index[pos];
            takes_part = my_row >= 0 && ((alive == nullptr) || (alive[my_row] != 0));
        } else {
            base = (g / S) * S * M + (g % S);
            if (lane < M) takes_part = (alive == nullptr) || (alive[base + static_cast<int64_t>(lane) * S] != 0);
        }
        const uint64_t live = __ballot(takes_part);
        const int cnt = __popcll(live);
        if (cnt < (SGD ? 1 : 2)) continue;           // nothing to do: rows stay as they are

        const int64_t v0 = tile * (static_cast<int64_t>(kBlock) * COLS) + threadIdx.x;
        bool in_row[COLS];
#pragma unroll
        for (int c = 0; c < COLS; ++c) in_row[c] = (v0 + c * kBlock) < nvec;

        char *gbase = X + base * row_bytes + v0 * static_cast<int64_t>(sizeof(mem_t));
        const int64_t jstep = S * row_bytes;
        // address of this lane's first vector in the row of position j (j is wave-uniform)
        auto row_ptr = [&](int j) -> char * {
            if constexpr (IDX)
                return gbase + static_cast<int64_t>(__builtin_amdgcn_readlane(my_row, j)) * row_bytes;
            else
                return gbase + j * jstep;
        };

        float acc[COLS][NE];
#pragma unroll
        for (int c = 0; c < COLS; ++c)
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[c][e] = 0.f;

        // Rows are taken in chunks of U by POSITION j (absent rows contribute an
        // exact 0 and cost no load), so the summation order is a fixed balanced
        // tree over the M slots whatever the mask: ((x0+x1)+(x2+x3))+... per
        // chunk, chunks added in ascending order.
        for (int j0 = 0; j0 < M; j0 += U) {
            const uint64_t bits = (live >> j0) & (U >= 64 ? ~0ull : ((1ull << (U % 64)) - 1ull));
            if (bits == 0) continue;
            mem_t buf[U][COLS];
            mem_t gbuf[SGD ? U : 1][COLS];
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int c = 0; c < COLS; ++c) {
                    buf[u][c] = V::zero();
                    if constexpr (SGD) gbuf[u][c] = V::zero();
                }
                if ((bits >> u) & 1ull) {
                    const mem_t *src = reinterpret_cast<const mem_t *>(row_ptr(j0 + u));
#pragma unroll
                    for (int c = 0; c < COLS; ++c)
                        if (in_row[c]) buf[u][c] = load_vec<NT>(src + c * kBlock);
                    if constexpr (SGD) {
                        const mem_t *gsrc = reinterpret_cast<const mem_t *>(
                            G + (base + (j0 + u) * S) * g_row_bytes + v0 * static_cast<int64_t>(sizeof(mem_t)));
#pragma unroll
                        for (int c = 0; c < COLS; ++c)
                            if (in_row[c]) gbuf[u][c] = load_vec<NT>(gsrc + c * kBlock);
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < COLS; ++c) {
                float f[U][NE];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    V::widen(buf[u][c], f[u]);
                    if constexpr (SGD) {
                        float gf[NE];
                        V::widen(gbuf[u][c], gf);
#pragma unroll
                        for (int e = 0; e < NE; ++e) f[u][e] = fmaf(-gamma, gf[e], f[u][e]);
                    }
                }
#pragma unroll
                for (int s = 1; s < U; s *= 2)
#pragma unroll
                    for (int u = 0; u + s < U; u += 2 * s)
#pragma unroll
                        for (int e = 0; e < NE; ++e) f[u][e] += f[u + s][e];
#pragma unroll
                for (int e = 0; e < NE; ++e) acc[c][e] += f[0][e];
            }
        }

        const float k = static_cast<float>(cnt);
        mem_t mean[COLS];
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[c][e] = acc[c][e] / k;
            mean[c] = V::narrow(acc[c]);
        }

        uint64_t rem = live;
        while (rem != 0) {
            const int j = __builtin_ctzll(rem);
            rem &= rem - 1;
            mem_t *dst = reinterpret_cast<mem_t *>(row_ptr(j));
#pragma unroll
            for (int c = 0; c < COLS; ++c)
                if (in_row[c]) store_vec<NT>(dst + c * kBlock, mean[c]);
        }
    }
}

// The kernel uses no LDS.  The dynamic-LDS size of the launch is only a
// throttle: a block that reserves lds bytes lets floor(160 KiB / lds) blocks
// share a compute unit, which bounds the number of row loads in flight.
template <int DT, int VE, int COLS, int U, bool NT, bool IDX = false, bool SGD = false>
hipError_t launch_one(char *X, int64_t row_bytes, int64_t nvec, const uint8_t *alive, const RoundGeom &geom,
                      int block, int waves_per_cu, int order, hipStream_t stream)
{
    if (nvec <= 0) return hipSuccess;
    const int64_t per_tile = static_cast<int64_t>(block) * COLS;
    const int64_t tiles = (nvec + per_tile - 1) / per_tile;
    const int64_t groups = IDX ? (geom.n_index + geom.M - 1) / geom.M : geom.N / geom.M;
    const int64_t work = groups * tiles;
    if (work <= 0) return hipSuccess;
    int64_t grid = work < 0x7fffffffLL ? work : 0x7fffffffLL;
    if (order == 1) {
        grid = ((work + 7) >> 3) << 3;
        if (grid > 0x7fffffffLL) { grid = 0x7fffffffLL; order = 0; }    // (more work items than blocks: plain order)
    }
    auto kernel = group_mean_kernel<DT, VE, COLS, U, NT, IDX, SGD>;
    size_t lds = 0;
    if (waves_per_cu > 0 && waves_per_cu < 32) {
        int blocks_per_cu = waves_per_cu / (block / 64);
        if (blocks_per_cu < 1) blocks_per_cu = 1;
        lds = lds_bytes_for_blocks_per_cu(blocks_per_cu);
        hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kernel), kLdsPerCu);
        if (e != hipSuccess) return e;
    }
    kernel<<<dim3(static_cast<uint32_t>(grid)), dim3(block), lds, stream>>>(X, row_bytes, nvec, alive, geom.M,
                                                                            geom.S, tiles, work, geom.index,
                                                                            geom.n_index, geom.grad, geom.grad_row_bytes,
                                                                            geom.gamma, order);
    return hipGetLastError();
}

template <int DT, int VE>
hipError_t launch_shape(int cols, int unroll, bool nt, char *X, int64_t row_bytes, int64_t nvec,
                        const uint8_t *alive, const RoundGeom &geom, int block, int wpc, int order, hipStream_t stream)
{
    if (geom.index != nullptr) {
        // peer-list groups: the default shapes only, streaming accesses
        if (cols == 1 && unroll == 16) return launch_one<DT, VE, 1, 16, true, true>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream);
        if (cols == 2 && unroll == 8) return launch_one<DT, VE, 2, 8, true, true>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream);
        if (cols == 4 && unroll == 4) return launch_one<DT, VE, 4, 4, true, true>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream);
        if (cols == 4 && unroll == 2) return launch_one<DT, VE, 4, 2, true, true>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream);
        return hipErrorInvalidValue;
    }
    if (geom.grad != nullptr) {
        // Moshpit SGD step: the default shapes only, streaming accesses
        if (cols == 1 && unroll == 16) return launch_one<DT, VE, 1, 16, true, false, true>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream);
        if (cols == 2 && unroll == 8) return launch_one<DT, VE, 2, 8, true, false, true>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream);
        if (cols == 4 && unroll == 4) return launch_one<DT, VE, 4, 4, true, false, true>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream);
        if (cols == 4 && unroll == 2) return launch_one<DT, VE, 4, 2, true, false, true>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream);
        return hipErrorInvalidValue;
    }
#define MOSHPIT_CASE(C, UU)                                                                          \
    if (cols == C && unroll == UU)                                                                   \
        return nt ? launch_one<DT, VE, C, UU, true>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream)   \
                  : launch_one<DT, VE, C, UU, false>(X, row_bytes, nvec, alive, geom, block, wpc, order, stream);
    MOSHPIT_CASE(1, 4)
    MOSHPIT_CASE(1, 8)
    MOSHPIT_CASE(1, 16)
    MOSHPIT_CASE(1, 32)
    MOSHPIT_CASE(2, 2)
    MOSHPIT_CASE(2, 4)
    MOSHPIT_CASE(2, 8)
    MOSHPIT_CASE(2, 16)
    MOSHPIT_CASE(4, 2)
    MOSHPIT_CASE(4, 4)
    MOSHPIT_CASE(4, 8)
#undef MOSHPIT_CASE
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_group_mean(void *X, int dtype, int64_t P, int64_t row_stride, const RoundGeom &geom,
                             const uint8_t *alive, const MeanTuning &tune, hipStream_t stream)
{
    const int64_t esize = dtype == 0 ? 4 : 2;
    const int64_t row_bytes = row_stride * esize;
    const bool aligned = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (row_bytes % 16 == 0) &&
                         (geom.grad == nullptr || (reinterpret_cast<uintptr_t>(geom.grad) % 16 == 0 &&
                                                   geom.grad_row_bytes % 16 == 0));
    const int64_t ve = dtype == 0 ? 4 : 8;
    const int64_t nvec = aligned ? P / ve : 0;          // 128-bit part of every row
    const int64_t tail0 = nvec * ve;                    // first column of the element-wise part

    // Defaults (measured on MI355X over block sizes, rows in flight and resident waves):
    // one-wave blocks, each wave keeps about 16 KiB of row loads in flight
    // (rows per chunk x cols x 1 KiB) and 4-7 waves share a compute unit, i.e.
    // about 16-28 MiB in flight on the chip.  More than that and the HBM
    // controllers see too many open pages; less and latency is not covered.
    int cols = tune.cols, unroll = tune.unroll;
    if (cols <= 0 || unroll <= 0 || geom.index != nullptr || geom.grad != nullptr) {
        if (geom.M > 8) { unroll = 16; cols = 1; }
        else if (geom.M > 4) { unroll = 8; cols = 2; }
        else if (geom.M > 2) {
            // four rows per group: one vector per row and lane and 20 resident waves measured 2 %
            // above four vectors and 5 waves on 100 MB rows (peer lists and the SGD step keep four)
            unroll = 4;
            cols = (geom.index != nullptr || geom.grad != nullptr) ? 4 : 1;
        }
        else { unroll = 2; cols = 4; }
    }
    const bool nt = tune.nt != 0;
    const int block = (tune.block == 64 || tune.block == 128 || tune.block == 256) ? tune.block : 64;
    // Block order (measured on MI355X over row sizes of 128 KiB .. 32 MiB, groups of 16 and of
    // 32 rows).  Work items go to the blocks tile-fastest, so the waves in flight stream a
    // handful of groups: up to 6.4 TB/s when the byte distance between the rows of a group
    // spreads well over the memory channels, 4.3 - 5.4 TB/s when it is 4, 8 or 16 MiB with 16
    // rows per group (2 MiB with 32).  For those distances each die is given an eighth of the
    // work list to stream through (8 times as many row streams in flight): 5.7 - 5.8 TB/s
    // whatever the distance, below the good cases of the plain order, above its bad ones.
    int order = tune.order;
    if (order < 0) {
        order = 0;
        if (geom.index == nullptr) {
            const int64_t member_stride = geom.S * row_bytes;
            const int64_t MiB = 1 << 20;
            if (geom.M <= 16 ? (member_stride >= 4 * MiB && member_stride <= 16 * MiB)
                             : (member_stride >= 2 * MiB && member_stride < 4 * MiB))
                order = 1;
        }
    }
    int wpc = tune.waves_per_cu;
    if (wpc <= 0) {
        // Resident waves per compute unit (measured; the optimum is sharp: on 16 MiB rows in
        // groups of 32, 4 waves give 6.1 TB/s, 3 give 5.8 and 5 give 5.9).  A wave keeps
        // rows x cols KiB of loads in flight (twice that with the gradients of the SGD step).
        const int rows = geom.M < unroll ? geom.M : unroll;
        const int kib_per_wave = rows * cols * (block / 64) * (geom.grad != nullptr ? 2 : 1);
        wpc = (dtype == 0 ? 64 : 80) / kib_per_wave * (block / 64);
        // groups of up to 16 rows (16 KiB in flight per wave): 5 waves; 7 when the rows are
        // shorter than 1 MiB, for groups given as a peer list and when every die streams its
        // own part of the list; 5 for the Moshpit SGD step (which also streams the gradients)
        // The figures above and below were measured with 5 - 20 % of the peers absent.  When
        // (nearly) every peer takes part each wave has more loads in flight and fewer waves do
        // better (16 MiB rows in groups of 32: 3 waves 6.2 TB/s, 4 waves 5.8).
        if (wpc < 4) wpc = 4;
        const bool full = alive == nullptr || geom.present >= 0.97f;
        if (full && geom.grad == nullptr && geom.index == nullptr) wpc -= 1;
        if (rows == 16 && cols == 1 && geom.M <= 16) {
            if (geom.grad != nullptr) wpc = 5;
            else if (geom.index != nullptr) wpc = 7;
            else if (full) wpc = order == 1 ? 6 : 5;
            else wpc = (order == 1 || row_bytes < (1 << 20)) ? 7 : 5;
        }
        // groups of up to 4 rows with one vector per row and lane (4 KiB in flight per wave)
        if (rows * cols <= 4) wpc = full ? 14 : 21;
        if (wpc > 32) wpc = 32;
    }

    char *base = static_cast<char *>(X);
    hipError_t e = hipSuccess;
    if (nvec > 0) {
        e = dtype == 0 ? launch_shape<0, 4>(cols, unroll, nt, base, row_bytes, nvec, alive, geom, block, wpc, order, stream)
                       : launch_shape<1, 8>(cols, unroll, nt, base, row_bytes, nvec, alive, geom, block, wpc, order, stream);
        if (e != hipSuccess) return e;
    }
    if (tail0 < P) {
        char *tbase = base + tail0 * esize;
        if (geom.grad != nullptr) {
            RoundGeom tg = geom;
            tg.grad = geom.grad + tail0 * esize;
            e = dtype == 0 ? launch_one<0, 1, 1, 8, false, false, true>(tbase, row_bytes, P - tail0, alive, tg, 256, 32, 0, stream)
                           : launch_one<1, 1, 1, 8, false, false, true>(tbase, row_bytes, P - tail0, alive, tg, 256, 32, 0, stream);
        } else if (geom.index != nullptr)
            e = dtype == 0 ? launch_one<0, 1, 1, 8, false, true>(tbase, row_bytes, P - tail0, alive, geom, 256, 32, 0, stream)
                           : launch_one<1, 1, 1, 8, false, true>(tbase, row_bytes, P - tail0, alive, geom, 256, 32, 0, stream);
        else
            e = dtype == 0 ? launch_one<0, 1, 1, 8, false>(tbase, row_bytes, P - tail0, alive, geom, 256, 32, 0, stream)
                           : launch_one<1, 1, 1, 8, false>(tbase, row_bytes, P - tail0, alive, geom, 256, 32, 0, stream);
    }
    return e;
}

// ---- local iteration of Moshpit SGD (Alg. 2): theta_i <- theta_i - gamma * g_i ----

namespace {
template <int DT, int VE>
__global__ __launch_bounds__(256) void local_step_kernel(char *X, int64_t row_bytes, const char *__restrict__ G,
                                                         int64_t g_row_bytes, int64_t nvec,
                                                         const uint8_t *__restrict__ alive, float gamma, int64_t tiles)
{
    typedef Vec<DT, VE> V;
    typedef typename V::mem_t mem_t;
    constexpr int NE = V::NE;
    const int64_t row = blockIdx.x / tiles;
    const int64_t tile = blockIdx.x - row * tiles;
    if (alive != nullptr && alive[row] == 0) return;
    const int64_t v = tile * 256 + threadIdx.x;
    if (v >= nvec) return;
    mem_t *x = reinterpret_cast<mem_t *>(X + row * row_bytes) + v;
    const mem_t *g = reinterpret_cast<const mem_t *>(G + row * g_row_bytes) + v;
    float xf[NE], gf[NE];
    V::widen(load_vec<true>(x), xf);
    V::widen(load_vec<true>(g), gf);
#pragma unroll
    for (int e = 0; e < NE; ++e) xf[e] = fmaf(-gamma, gf[e], xf[e]);
    store_vec<true>(x, V::narrow(xf));
}

template <int DT, int VE>
hipError_t launch_local(char *X, int64_t row_bytes, const char *G, int64_t g_row_bytes, int64_t nvec, int64_t N,
                        const uint8_t *alive, float gamma, hipStream_t stream)
{
    if (nvec <= 0) return hipSuccess;
    const int64_t tiles = (nvec + 255) / 256;
    const int64_t blocks = tiles * N;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    local_step_kernel<DT, VE><<<dim3(static_cast<uint32_t>(blocks)), dim3(256), 0, stream>>>(X, row_bytes, G, g_row_bytes,
                                                                                              nvec, alive, gamma, tiles);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_local_step(void *X, int dtype, int64_t N, int64_t P, int64_t row_stride, const void *G,
                             int64_t g_row_stride, const uint8_t *alive, float gamma, hipStream_t stream)
{
    const int64_t esize = dtype == 0 ? 4 : 2;
    const int64_t row_bytes = row_stride * esize, g_row_bytes = g_row_stride * esize;
    const bool aligned = reinterpret_cast<uintptr_t>(X) % 16 == 0 && row_bytes % 16 == 0 &&
                         reinterpret_cast<uintptr_t>(G) % 16 == 0 && g_row_bytes % 16 == 0;
    const int64_t ve = dtype == 0 ? 4 : 8;
    const int64_t nvec = aligned ? P / ve : 0;
    const int64_t tail0 = nvec * ve;
    char *x = static_cast<char *>(X);
    const char *g = static_cast<const char *>(G);
    hipError_t e = dtype == 0 ? launch_local<0, 4>(x, row_bytes, g, g_row_bytes, nvec, N, alive, gamma, stream)
                              : launch_local<1, 8>(x, row_bytes, g, g_row_bytes, nvec, N, alive, gamma, stream);
    if (e != hipSuccess || tail0 >= P) return e;
    return dtype == 0 ? launch_local<0, 1>(x + tail0 * esize, row_bytes, g + tail0 * esize, g_row_bytes, P - tail0, N,
                                           alive, gamma, stream)
                      : launch_local<1, 1>(x + tail0 * esize, row_bytes, g + tail0 * esize, g_row_bytes, P - tail0, N,
                                           alive, gamma, stream);
}

}  // namespace moshpit
