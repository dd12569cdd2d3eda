// Internal launch interface between the C-ABI layer (api.hip) and the kernel
// translation units.  Not installed; the public interface is include/moshpit.h.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>
#include <stdint.h>

namespace moshpit {

// Per-device launch facts, looked up once per device and kept in a table guarded by a
// mutex (handles on different devices, and threads making their first launch at the same
// time, do not disturb each other).
// ensure_dynamic_lds: allow `kernel` to be launched with up to `bytes` of dynamic LDS on
// the current device (a function attribute; set once per kernel and device).
// current_compute_units: number of compute units of the current device.
hipError_t ensure_dynamic_lds(const void *kernel, int bytes);
hipError_t current_compute_units(int *out);

// Dynamic-LDS size that lets `blocks` blocks of a kernel that uses no other LDS share a
// compute unit of gfx950 (and no more, when 128 / blocks is a whole number or nearly so):
// the 160 KiB are handed out in 128 pieces of 1280 bytes (measured: 3 blocks of 52 KiB fit,
// 3 of 53 KiB do not; 2 of 80 KiB and 4 of 40 KiB fit).
inline size_t lds_bytes_for_blocks_per_cu(int blocks)
{
    constexpr size_t kLds = 160 * 1024, kPiece = 1280;
    if (blocks < 1) blocks = 1;
    return kLds / static_cast<size_t>(blocks) / kPiece * kPiece;
}

// 128-bit item of the device sort, compared as (hi, lo).
struct SortItem {
    uint64_t hi, lo;
};

// Items the sort works on for n real ones: the next power of two, at least 4096.
int64_t sort_padded_count(int64_t n);

// Queue the sort of items[0..n_padded) (device; n_padded from sort_padded_count, the
// caller fills the padding with items that compare last), ascending, in place.
hipError_t launch_sort_items(SortItem *items, int64_t n_padded, hipStream_t stream);

// Launch shape of the group-mean kernel.  cols = 128-bit vectors per thread per
// row, unroll = rows whose loads are issued before the first add, nt =
// non-temporal loads and stores, block = threads per block (64/128/256),
// waves_per_cu = resident waves per compute unit (enforced through the
// launch's LDS reservation), order = how work items are dealt to the blocks (0: in
// order, column tiles fastest; 1: each of the 8 dies streams through an eighth of the
// list).  0 / -1 mean "choose from the shape".
struct MeanTuning {
    int cols = 0;
    int unroll = 0;
    int nt = -1;
    int block = 0;
    int waves_per_cu = 0;
    int order = -1;
};

// Geometry of one round: group g (0 <= g < N/M) owns rows base(g) + j*S,
// j = 0..M-1, with S = M^(t mod d) and base(g) = (g / S) * S * M + g % S.
// With index != nullptr the groups are instead consecutive chunks of M entries of
// the peer list index[0..n_index) (device memory), the last chunk possibly short.
struct RoundGeom {
    int64_t N;
    int32_t M;
    int64_t S;
    const int32_t *index = nullptr;
    int64_t n_index = 0;
    // Moshpit SGD step: average theta - gamma * g, g from `grad` (device, laid out like X)
    const char *grad = nullptr;
    int64_t grad_row_bytes = 0;
    float gamma = 0.f;
    // Fraction of the peers expected to take part (sizes the launch only: a wave keeps one row
    // load in flight per participant, so fuller groups want fewer resident waves); < 0 = unknown
    float present = -1.f;
};

// Queue one averaging round on `stream`.  X: device, row-major, `P` valid
// elements per row, rows `row_stride` elements apart.  alive: device, N bytes
// (non-zero = takes part) or nullptr (all take part).
hipError_t launch_group_mean(void *X, int dtype, int64_t P, int64_t row_stride, const RoundGeom &geom,
                             const uint8_t *alive, const MeanTuning &tune, hipStream_t stream);

// Queue the local iteration of Moshpit SGD: X[i] -= gamma * G[i] for the rows that take part.
hipError_t launch_local_step(void *X, int dtype, int64_t N, int64_t P, int64_t row_stride, const void *G,
                             int64_t g_row_stride, const uint8_t *alive, float gamma, hipStream_t stream);

// Number of partial sums launch_dist_partials writes for this shape.
int64_t dist_partials_count(int dtype, int64_t P, int64_t row_stride, const void *X);

// Queue the distortion reduction: partials (device, dist_partials_count
// doubles) then out[0] = (sum of partials) / n.  present: device, N bytes, or
// nullptr (every row counts); first = first row that counts, n = how many do.
hipError_t launch_dist_to_mean(const void *X, int dtype, int64_t N, int64_t P, int64_t row_stride,
                               double *partials, double *out, const uint8_t *present, int64_t first, int64_t n,
                               hipStream_t stream);

// Partial sums the allocation-free distortion entry point can hold, and the device
// address of the array that holds them on the current device (looked up once per
// device; allocates nothing).
constexpr int64_t kStaticPartials = 131072;
hipError_t static_scratch(double **out);

// Queue the failure-schedule generator: masks[r][i] (device, rounds*N bytes).
// Die-and-rejoin schedules (kind 2) depend on the past: the walk starts at round
// s_begin <= t0 from away_in (device, N int32: rounds each peer still sits out at the
// start of round s_begin; nullptr = round 0, nobody away) and leaves the state at the
// start of round t0 + rounds in away_out (device, N int32, may equal away_in; nullptr =
// not wanted).  The other kinds ignore the three arguments.
hipError_t launch_schedule(int kind, uint32_t threshold, uint64_t seed, int down, int64_t N, int64_t t0,
                           int rounds, uint8_t *masks, int64_t s_begin, const int32_t *away_in, int32_t *away_out,
                           hipStream_t stream);

// Alg. 1 with chunk-index keys.  keys: device, N x (d-1) int32.  init writes the initial
// keys; grouping turns (keys, alive, seed, t) into the padded peer list index[0..n_index)
// (group g = entries [g*M, (g+1)*M), unused entries -1; n_index >= (N/M + M^(d-1)) * M) and
// shifts each participant's chunk index into its key.  packed: N int32, count/first:
// M^(d-1)+1 int32 each, items: sort_padded_count(N) entries (device scratch).
hipError_t launch_dynamic_init(int64_t N, int32_t M, int32_t d, int32_t *keys, hipStream_t stream);
hipError_t launch_dynamic_grouping(int64_t N, int32_t M, int32_t d, uint64_t seed, int64_t t, const uint8_t *alive,
                                   int32_t *keys, int32_t *packed, int32_t *count, int32_t *first, int32_t *index,
                                   int64_t n_index, SortItem *items, hipStream_t stream);

// Queue the group-skip filter on masks[rounds][N] (device, in place) for rounds t0..
hipError_t launch_skip_filter(uint8_t *masks, int64_t N, int32_t M, int32_t d, int64_t t0, int rounds,
                              hipStream_t stream);

// Returning peers (present in `cur`, absent in `prev`; device masks of N bytes): draw
// their donors among the peers present in both, list them, then copy the donors' rows.
// candidates, donor, returning: device, N int32 each; counts: device, 2 int32
// (candidates, returning peers).  The copy reads donor/returning/counts on the device.
hipError_t launch_refresh_plan(const uint8_t *prev, const uint8_t *cur, int64_t N, uint64_t seed, int64_t t,
                               int32_t *candidates, int32_t *donor, int32_t *returning, int32_t *counts,
                               hipStream_t stream);
// expected_rows: the host's guess of how many peers return (sizes the launch only).
hipError_t launch_refresh_copy(void *X, int dtype, int64_t N, int64_t P, int64_t row_stride, const int32_t *donor,
                               const int32_t *returning, const int32_t *counts, int64_t expected_rows,
                               hipStream_t stream);

// Queue the random-permutation kernels: perm[r] = peer of rank r when the peers
// are ordered by their 64-bit key of (seed, t), ties by index (device, N int32).
// items: device scratch, sort_padded_count(N) entries.
hipError_t launch_random_permutation(uint64_t seed, int64_t t, int64_t N, int32_t *perm, SortItem *items,
                                     hipStream_t stream);

// Queue the group-key kernel: keys[i] (device, N int32) for axis a, S = M^a.
hipError_t launch_group_keys(int64_t N, int32_t M, int64_t S, int32_t *keys, hipStream_t stream);

// Plan of one fused pass: rounds t0..t0+rounds-1 run on tiles of `rows` = M^F
// rows (one F-dimensional sub-grid) x Wb bytes that stay in LDS.
constexpr int kFusedMaxAxes = 12;
struct FusedPlan {
    int64_t N;
    int32_t M, F;
    int32_t rows, groups;          // M^F rows per tile, rows / M groups per round
    int32_t rows_padded;           // rows rounded up to a multiple of 16
    int32_t rounds;                // rounds fused by this pass
    int32_t blocks_per_cu;         // 1 or 2: which kernel shape the plan was made for
    int32_t spread;                // the next tile's loads are issued in this many portions, one per round
    int32_t local_axis0;           // tile-local axis of the first round
    int32_t n_outer;               // grid axes outside the tile
    int32_t Wb, tile_bytes, lds_bytes;
    int64_t row_bytes, row_valid_bytes;
    int64_t tiles, planes, work_items;
    // Moshpit SGD pass (Alg. 2): rows present in the pass's first round enter the tile as
    // theta - gamma * g, g read from `grad` (device, laid out exactly like the state: same
    // row stride); nullptr = a plain pass
    const char *grad;
    float gamma;
    int64_t gstride[kFusedMaxAxes];   // global row stride of tile-local axis f
    int64_t ostride[40];              // global row strides of the outer axes
};

// Decide whether rounds starting at t0 (at most rounds_wanted) can be fused
// for this state, and how.  false = use the single-round kernel.
bool plan_fused(int dtype, int64_t N, int32_t M, int32_t d, int64_t P, int64_t row_stride, const void *X,
                int64_t t0, int32_t rounds_wanted, FusedPlan *out);

// Queue one fused pass.  masks: device, [plan.rounds][N] for the pass's
// rounds, or nullptr (all peers take part).
hipError_t launch_fused_rounds(void *X, int dtype, const FusedPlan &plan, const uint8_t *masks,
                               hipStream_t stream);

// Queue a plain 128-bit copy of nbytes (multiple of 16) from src to dst.
hipError_t launch_copy_probe(void *dst, const void *src, int64_t nbytes, hipStream_t stream);

// Queue the exhaustive comparison of the hardware binary32 -> bfloat16 conversion with
// its integer definition: mismatches[0] (device, zeroed by the caller) counts the inputs,
// out of all 2^32, on which the two differ.
hipError_t launch_bf16_rounding_check(unsigned long long *mismatches, hipStream_t stream);

}  // namespace moshpit
