// C ABI of libmoshpit (include/moshpit.h): handle, argument checks, scratch,
// and the order in which the kernels of a round / a run are queued.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/moshpit.h"
#include "moshpit_internal.h"

using namespace moshpit;

struct moshpit_ctx {
    int64_t N = 0, P = 0;
    int32_t M = 0, d = 0, dtype = 0;
    int device = 0;

    void *X = nullptr;                 // borrowed
    int64_t row_stride = 0;
    hipStream_t stream = nullptr;

    uint8_t *d_round_mask = nullptr;   // N bytes, for moshpit_round(host mask)
    uint8_t *d_present = nullptr;      // N bytes, for moshpit_dist_to_mean_subset
    int32_t *d_perm = nullptr;         // N, peer list of the list-based rounds
    SortItem *d_sort = nullptr;        // sort_padded_count(N) items: the random orders are sorted here
    int32_t *d_dyn = nullptr;          // chunk-index keys and their scratch (see dyn_layout)
    uint8_t *d_masks = nullptr;        // mask_rounds_cap * N bytes, for runs
    int64_t mask_rounds_cap = 0;
    uint8_t *d_masks_raw = nullptr;    // raw_rounds_cap * N bytes: presence before the group-skip filter
    int64_t raw_rounds_cap = 0;
    int32_t *d_refresh = nullptr;      // 3 N + 2 int32: candidates, donors, returning peers, counts
    uint8_t *d_refresh_masks = nullptr;  // 2 N bytes, for moshpit_refresh(host masks)
    int32_t *d_keys = nullptr;         // N
    double *d_partials = nullptr;      // partials_cap doubles
    int64_t partials_cap = 0;
    double *d_dist = nullptr;          // dist_cap doubles
    int64_t dist_cap = 0;
    std::vector<hipEvent_t> events;    // 2 per timed round

    // Host bytes on their way to the device (masks, peer lists): copied out of the caller's
    // buffer into one of these pinned slots before the call returns, then sent in stream order.
    struct StageSlot {
        void *host = nullptr;
        size_t cap = 0;
        hipEvent_t sent = nullptr;     // recorded after the slot's copy to the device
        bool pending = false;
    };
    static constexpr int kStageSlots = 4;
    StageSlot stage[kStageSlots];
    int stage_next = 0;

    // Die-and-rejoin schedule carried between calls: d_away[i] = rounds peer i still sits
    // out at the start of round away_t under (away_seed, away_threshold, away_down).
    int32_t *d_away = nullptr;
    bool away_valid = false;
    uint64_t away_seed = 0;
    uint32_t away_threshold = 0;
    int32_t away_down = 0;
    int64_t away_t = 0;

    MeanTuning tune;
    char err[512] = {0};
};

namespace {

thread_local char g_create_err[256] = {0};

int fail(moshpit_ctx *h, int code, const char *fmt, ...)
{
    char *dst = h ? h->err : g_create_err;
    const size_t cap = h ? sizeof(h->err) : sizeof(g_create_err);
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, cap, fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(h, call)                                                                         \
    do {                                                                                         \
        hipError_t e_ = (call);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail((h), e_ == hipErrorOutOfMemory ? MOSHPIT_ENOMEM : MOSHPIT_EHIP,          \
                        "%s: %s", #call, hipGetErrorString(e_));                                 \
    } while (0)

int64_t axis_stride(const moshpit_ctx *h, int64_t t)
{
    int64_t S = 1;
    for (int64_t q = 0; q < t % h->d; ++q) S *= h->M;
    return S;
}

int check_ready(moshpit_ctx *h)
{
    if (!h) return MOSHPIT_EINVAL;
    if (!h->X) return fail(h, MOSHPIT_ESTATE, "no state bound: call moshpit_bind_state first");
    return MOSHPIT_OK;
}

int check_schedule(moshpit_ctx *h, const moshpit_schedule *s, int64_t t0, int32_t rounds)
{
    if (t0 < 0 || rounds < 0) return fail(h, MOSHPIT_EINVAL, "t0 and rounds must be >= 0");
    if (!s) return MOSHPIT_OK;
    if (s->kind < MOSHPIT_SCHED_NONE || s->kind > MOSHPIT_SCHED_EXPLICIT)
        return fail(h, MOSHPIT_EINVAL, "unknown schedule kind %d", s->kind);
    if (s->kind == MOSHPIT_SCHED_IID || s->kind == MOSHPIT_SCHED_REJOIN)
        if (!(s->p >= 0.0 && s->p <= 1.0)) return fail(h, MOSHPIT_EINVAL, "failure probability outside [0,1]");
    if (s->kind == MOSHPIT_SCHED_REJOIN && s->down_rounds < 1)
        return fail(h, MOSHPIT_EINVAL, "down_rounds must be >= 1");
    if (s->kind == MOSHPIT_SCHED_EXPLICIT && rounds > 0 && !s->explicit_masks)
        return fail(h, MOSHPIT_EINVAL, "explicit schedule without masks");
    return MOSHPIT_OK;
}

// Send `bytes` of host memory to dst_dev in stream order.  The caller's buffer has been
// read completely when this returns, whatever kind of host memory it is (an asynchronous
// copy straight from pinned memory would still be reading it).
int stage_to_device(moshpit_ctx *h, void *dst_dev, const void *src_host, size_t bytes)
{
    if (bytes == 0) return MOSHPIT_OK;
    moshpit_ctx::StageSlot &s = h->stage[h->stage_next];
    h->stage_next = (h->stage_next + 1) % moshpit_ctx::kStageSlots;
    if (s.pending) {
        HIP_TRY(h, hipEventSynchronize(s.sent));
        s.pending = false;
    }
    if (s.cap < bytes) {
        if (s.host) HIP_TRY(h, hipHostFree(s.host));
        s.host = nullptr;
        s.cap = 0;
        HIP_TRY(h, hipHostMalloc(&s.host, bytes, hipHostMallocDefault));
        s.cap = bytes;
    }
    if (!s.sent) HIP_TRY(h, hipEventCreateWithFlags(&s.sent, hipEventDisableTiming));
    std::memcpy(s.host, src_host, bytes);
    HIP_TRY(h, hipMemcpyAsync(dst_dev, s.host, bytes, hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, hipEventRecord(s.sent, h->stream));
    s.pending = true;
    return MOSHPIT_OK;
}

// Rounds whose groups come from a random order sort 16 bytes per peer and address peers
// by int32: 2^24 peers (a 256 MiB sort buffer) is where this library stops.
constexpr int64_t kMaxOrderedPeers = int64_t(1) << 24;

int reserve_sort(moshpit_ctx *h)
{
    if (h->N > kMaxOrderedPeers)
        return fail(h, MOSHPIT_EINVAL, "rounds over a random order of the peers support at most %lld peers",
                    (long long)kMaxOrderedPeers);
    if (h->d_sort) return MOSHPIT_OK;
    HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_sort), sizeof(SortItem) * static_cast<size_t>(sort_padded_count(h->N))));
    return MOSHPIT_OK;
}

int reserve_masks(moshpit_ctx *h, int64_t rounds)
{
    if (rounds <= h->mask_rounds_cap) return MOSHPIT_OK;
    if (h->d_masks) {
        HIP_TRY(h, hipStreamSynchronize(h->stream));
        HIP_TRY(h, hipFree(h->d_masks));
        h->d_masks = nullptr;
        h->mask_rounds_cap = 0;
    }
    HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_masks), static_cast<size_t>(rounds * h->N)));
    h->mask_rounds_cap = rounds;
    return MOSHPIT_OK;
}

int reserve_dist(moshpit_ctx *h, int64_t count)
{
    if (count <= h->dist_cap) return MOSHPIT_OK;
    if (h->d_dist) {
        HIP_TRY(h, hipStreamSynchronize(h->stream));
        HIP_TRY(h, hipFree(h->d_dist));
        h->d_dist = nullptr;
        h->dist_cap = 0;
    }
    HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_dist), static_cast<size_t>(count) * sizeof(double)));
    h->dist_cap = count;
    return MOSHPIT_OK;
}

int reserve_events(moshpit_ctx *h, size_t count)
{
    while (h->events.size() < count) {
        hipEvent_t ev;
        HIP_TRY(h, hipEventCreate(&ev));
        h->events.push_back(ev);
    }
    return MOSHPIT_OK;
}

// Fill d_masks[0..rounds) for rounds t0.. under schedule s (s may be NULL).
int queue_masks(moshpit_ctx *h, const moshpit_schedule *s, int64_t t0, int32_t rounds)
{
    int rc = reserve_masks(h, rounds);
    if (rc != MOSHPIT_OK || rounds == 0) return rc;
    if (s && s->kind == MOSHPIT_SCHED_EXPLICIT) {
        rc = stage_to_device(h, h->d_masks, s->explicit_masks, static_cast<size_t>(rounds) * h->N);
        if (rc != MOSHPIT_OK) return rc;
    } else {
        const int kind = s ? s->kind : MOSHPIT_SCHED_NONE;
        const double p = s ? s->p : 0.0;
        const uint32_t threshold = static_cast<uint32_t>(std::floor(p * 16777216.0));
        const uint64_t seed = s ? s->seed : 0;
        const int32_t down = s ? s->down_rounds : 0;
        int64_t s_begin = 0;
        const int32_t *away_in = nullptr;
        if (kind == MOSHPIT_SCHED_REJOIN) {
            // go on from the state a previous call left, when it belongs to this schedule and is not past t0
            if (!h->d_away)
                HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_away), sizeof(int32_t) * static_cast<size_t>(h->N)));
            if (h->away_valid && h->away_seed == seed && h->away_threshold == threshold && h->away_down == down &&
                h->away_t <= t0 && h->away_t > 0) {
                s_begin = h->away_t;
                away_in = h->d_away;
            }
            h->away_valid = false;
        }
        HIP_TRY(h, launch_schedule(kind, threshold, seed, down, h->N, t0, rounds, h->d_masks, s_begin, away_in,
                                   kind == MOSHPIT_SCHED_REJOIN ? h->d_away : nullptr, h->stream));
        if (kind == MOSHPIT_SCHED_REJOIN) {
            h->away_valid = true;
            h->away_seed = seed;
            h->away_threshold = threshold;
            h->away_down = down;
            h->away_t = t0 + rounds;
        }
    }
    if (s && s->group_skip) {
        if (s->refresh) {
            // who returns is a matter of presence, not of which groups skipped
            if (rounds > h->raw_rounds_cap) {
                if (h->d_masks_raw) {
                    HIP_TRY(h, hipStreamSynchronize(h->stream));
                    HIP_TRY(h, hipFree(h->d_masks_raw));
                    h->d_masks_raw = nullptr;
                    h->raw_rounds_cap = 0;
                }
                HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_masks_raw), static_cast<size_t>(rounds * h->N)));
                h->raw_rounds_cap = rounds;
            }
            HIP_TRY(h, hipMemcpyAsync(h->d_masks_raw, h->d_masks, static_cast<size_t>(rounds) * h->N,
                                      hipMemcpyDeviceToDevice, h->stream));
        }
        HIP_TRY(h, launch_skip_filter(h->d_masks, h->N, h->M, h->d, t0, rounds, h->stream));
    }
    return MOSHPIT_OK;
}

int reserve_refresh(moshpit_ctx *h)
{
    if (h->d_refresh) return MOSHPIT_OK;
    HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_refresh), sizeof(int32_t) * (3 * static_cast<size_t>(h->N) + 2)));
    return MOSHPIT_OK;
}

// Draw the donors of round t from two device masks and, if asked, copy their rows.
int queue_refresh(moshpit_ctx *h, int64_t t, uint64_t seed, const uint8_t *prev_dev, const uint8_t *cur_dev,
                  bool copy, int64_t expected_rows)
{
    int rc = reserve_refresh(h);
    if (rc != MOSHPIT_OK) return rc;
    int32_t *candidates = h->d_refresh, *donor = candidates + h->N, *returning = donor + h->N;
    int32_t *counts = returning + h->N;
    HIP_TRY(h, launch_refresh_plan(prev_dev, cur_dev, h->N, seed, t, candidates, donor, returning, counts, h->stream));
    if (copy)
        HIP_TRY(h, launch_refresh_copy(h->X, h->dtype, h->N, h->P, h->row_stride, donor, returning, counts, expected_rows,
                                       h->stream));
    return MOSHPIT_OK;
}

int stage_refresh_masks(moshpit_ctx *h, const uint8_t *prev_host, const uint8_t *cur_host)
{
    if (!prev_host || !cur_host) return fail(h, MOSHPIT_EINVAL, "both masks are required");
    if (h->N > 0x7fffffffLL) return fail(h, MOSHPIT_EINVAL, "too many peers for 32-bit donor indices");
    if (!h->d_refresh_masks)
        HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_refresh_masks), 2 * static_cast<size_t>(h->N)));
    int rc = stage_to_device(h, h->d_refresh_masks, prev_host, static_cast<size_t>(h->N));
    if (rc != MOSHPIT_OK) return rc;
    return stage_to_device(h, h->d_refresh_masks + h->N, cur_host, static_cast<size_t>(h->N));
}

// Fraction of non-zero bytes of a host mask, from at most 65,536 evenly spaced samples (it
// sizes launches only).
float present_fraction(const uint8_t *alive_host, int64_t N)
{
    if (!alive_host || N <= 0) return 1.f;
    const int64_t step = (N + 65535) / 65536;
    int64_t n = 0, seen = 0;
    for (int64_t i = 0; i < N; i += step, ++seen) n += alive_host[i] != 0 ? 1 : 0;
    return static_cast<float>(n) / static_cast<float>(seen);
}

// Expected fraction of peers that take part in a round of schedule s (nullptr: everybody).
float present_fraction(const moshpit_schedule *s)
{
    if (!s || s->kind == MOSHPIT_SCHED_NONE) return 1.f;
    if (s->kind == MOSHPIT_SCHED_EXPLICIT) return -1.f;
    return static_cast<float>(1.0 - s->p);
}

int queue_round(moshpit_ctx *h, int64_t t, const uint8_t *alive_dev, float present = -1.f)
{
    RoundGeom geom{h->N, h->M, axis_stride(h, t)};
    geom.present = present;
    HIP_TRY(h, launch_group_mean(h->X, h->dtype, h->P, h->row_stride, geom, alive_dev, h->tune, h->stream));
    return MOSHPIT_OK;
}

int queue_dist(moshpit_ctx *h, double *out_dev)
{
    HIP_TRY(h, launch_dist_to_mean(h->X, h->dtype, h->N, h->P, h->row_stride, h->d_partials, out_dev, nullptr, 0,
                                   h->N, h->stream));
    return MOSHPIT_OK;
}

}  // namespace

extern "C" {

int moshpit_create(int64_t N, int64_t P, int32_t M, int32_t d, int32_t dtype, moshpit_ctx **out)
{
    if (!out) return fail(nullptr, MOSHPIT_EINVAL, "out is NULL");
    *out = nullptr;
    if (M < 2 || M > 64) return fail(nullptr, MOSHPIT_EINVAL, "M must be in [2, 64], got %d", M);
    if (d < 1 || d > 62) return fail(nullptr, MOSHPIT_EINVAL, "d must be in [1, 62], got %d", d);
    if (P < 1) return fail(nullptr, MOSHPIT_EINVAL, "P must be >= 1");
    if (dtype != MOSHPIT_F32 && dtype != MOSHPIT_BF16) return fail(nullptr, MOSHPIT_EINVAL, "unknown dtype %d", dtype);
    int64_t full = 1;
    for (int q = 0; q < d; ++q) {
        if (full > (int64_t(1) << 40) / M) return fail(nullptr, MOSHPIT_EINVAL, "M^d is too large");
        full *= M;
    }
    if (N != full) return fail(nullptr, MOSHPIT_EINVAL, "N = %lld is not M^d = %lld", (long long)N, (long long)full);
    if (N / M > 0x7fffffffLL) return fail(nullptr, MOSHPIT_EINVAL, "too many groups for 32-bit keys");

    moshpit_ctx *h = new (std::nothrow) moshpit_ctx;
    if (!h) return fail(nullptr, MOSHPIT_ENOMEM, "out of host memory");
    h->N = N; h->P = P; h->M = M; h->d = d; h->dtype = dtype;
    hipError_t e = hipGetDevice(&h->device);
    double *static_partials = nullptr;          // set-up of moshpit_dist_to_mean_static on this device
    if (e == hipSuccess) e = static_scratch(&static_partials);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&h->d_round_mask), static_cast<size_t>(N));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&h->d_keys), static_cast<size_t>(N) * sizeof(int32_t));
    if (e != hipSuccess) {
        fail(nullptr, e == hipErrorOutOfMemory ? MOSHPIT_ENOMEM : MOSHPIT_EHIP, "moshpit_create: %s",
             hipGetErrorString(e));
        const int code = e == hipErrorOutOfMemory ? MOSHPIT_ENOMEM : MOSHPIT_EHIP;
        moshpit_destroy(h);
        return code;
    }
    *out = h;
    return MOSHPIT_OK;
}

int moshpit_destroy(moshpit_ctx *h)
{
    if (!h) return MOSHPIT_OK;
    (void)hipStreamSynchronize(h->stream);
    for (hipEvent_t ev : h->events) (void)hipEventDestroy(ev);
    for (moshpit_ctx::StageSlot &slot : h->stage) {
        if (slot.sent) (void)hipEventDestroy(slot.sent);
        if (slot.host) (void)hipHostFree(slot.host);
    }
    if (h->d_away) (void)hipFree(h->d_away);
    if (h->d_round_mask) (void)hipFree(h->d_round_mask);
    if (h->d_present) (void)hipFree(h->d_present);
    if (h->d_perm) (void)hipFree(h->d_perm);
    if (h->d_sort) (void)hipFree(h->d_sort);
    if (h->d_dyn) (void)hipFree(h->d_dyn);
    if (h->d_masks) (void)hipFree(h->d_masks);
    if (h->d_masks_raw) (void)hipFree(h->d_masks_raw);
    if (h->d_refresh) (void)hipFree(h->d_refresh);
    if (h->d_refresh_masks) (void)hipFree(h->d_refresh_masks);
    if (h->d_keys) (void)hipFree(h->d_keys);
    if (h->d_partials) (void)hipFree(h->d_partials);
    if (h->d_dist) (void)hipFree(h->d_dist);
    delete h;
    return MOSHPIT_OK;
}

int moshpit_bind_state(moshpit_ctx *h, void *state_dev, int64_t row_stride_elems, void *hip_stream)
{
    if (!h) return MOSHPIT_EINVAL;
    if (!state_dev) return fail(h, MOSHPIT_EINVAL, "state pointer is NULL");
    if (row_stride_elems < h->P) return fail(h, MOSHPIT_EINVAL, "row stride %lld < P = %lld",
                                             (long long)row_stride_elems, (long long)h->P);
    const int64_t esize = h->dtype == MOSHPIT_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(state_dev) % esize != 0)
        return fail(h, MOSHPIT_EINVAL, "state pointer is not aligned to the element size");
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, state_dev);
    if (e != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return fail(h, MOSHPIT_EINVAL, "state pointer is not device memory");
    }
    if (h->X) HIP_TRY(h, hipStreamSynchronize(h->stream));
    const int64_t need = dist_partials_count(h->dtype, h->P, row_stride_elems, state_dev);
    if (need > h->partials_cap) {
        if (h->d_partials) HIP_TRY(h, hipFree(h->d_partials));
        h->d_partials = nullptr;
        h->partials_cap = 0;
        HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_partials), static_cast<size_t>(need) * sizeof(double)));
        h->partials_cap = need;
    }
    int rc = reserve_dist(h, 64);
    if (rc != MOSHPIT_OK) return rc;
    h->X = state_dev;
    h->row_stride = row_stride_elems;
    h->stream = static_cast<hipStream_t>(hip_stream);
    return MOSHPIT_OK;
}

int moshpit_round(moshpit_ctx *h, int64_t t, const uint8_t *alive_host)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (t < 0) return fail(h, MOSHPIT_EINVAL, "round index must be >= 0");
    if (!alive_host) return queue_round(h, t, nullptr, 1.f);
    rc = stage_to_device(h, h->d_round_mask, alive_host, static_cast<size_t>(h->N));
    if (rc != MOSHPIT_OK) return rc;
    return queue_round(h, t, h->d_round_mask, present_fraction(alive_host, h->N));
}

int moshpit_round_dev(moshpit_ctx *h, int64_t t, const uint8_t *alive_dev)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (t < 0) return fail(h, MOSHPIT_EINVAL, "round index must be >= 0");
    return queue_round(h, t, alive_dev);
}

namespace {
// Rounds t0 .. t0+rounds-1 under schedule s.  grad != nullptr: an iteration of Moshpit SGD -
// the peers present in round t0 first take their local step theta - gamma * g (fused into
// the first pass over the state).
int run_impl(moshpit_ctx *h, int64_t t0, int32_t rounds, const moshpit_schedule *s, int32_t flags,
             double *dist_out_host, float *round_ms_out_host, const void *grad, int64_t grad_row_stride, float gamma)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (flags & ~MOSHPIT_RUN_FUSED) return fail(h, MOSHPIT_EINVAL, "unknown flags 0x%x", flags);
    rc = check_schedule(h, s, t0, rounds);
    if (rc != MOSHPIT_OK) return rc;
    const bool failures = s && s->kind != MOSHPIT_SCHED_NONE;
    const bool refresh = failures && s->refresh != 0;
    if (refresh && h->N > 0x7fffffffLL) return fail(h, MOSHPIT_EINVAL, "too many peers for 32-bit donor indices");
    // a refresh between two rounds moves rows across tiles: such runs go round by round
    const bool fused = (flags & MOSHPIT_RUN_FUSED) != 0 && !refresh;
    if (failures) {
        rc = queue_masks(h, s, t0, rounds);
        if (rc != MOSHPIT_OK) return rc;
    }
    if (dist_out_host) {
        rc = reserve_dist(h, static_cast<int64_t>(rounds) + 1);
        if (rc != MOSHPIT_OK) return rc;
        rc = queue_dist(h, h->d_dist);
        if (rc != MOSHPIT_OK) return rc;
    }
    if (round_ms_out_host) {
        rc = reserve_events(h, 2 * static_cast<size_t>(rounds));
        if (rc != MOSHPIT_OK) return rc;
    }
    // passes: one round each, or several when fusion is allowed and possible
    std::vector<int32_t> pass_rounds;
    std::vector<bool> have_dist(static_cast<size_t>(rounds) + 1, false);
    have_dist[0] = true;
    int32_t r = 0;
    while (r < rounds) {
        const size_t pass = pass_rounds.size();
        const uint8_t *mask_r = failures ? h->d_masks + static_cast<int64_t>(r) * h->N : nullptr;
        FusedPlan plan;
        const bool step_now = grad != nullptr && r == 0;       // the local step rides on the first pass
        const bool grad_fits = !step_now || (grad_row_stride == h->row_stride && reinterpret_cast<uintptr_t>(grad) % 16 == 0);
        const bool fuse = fused && grad_fits && plan_fused(h->dtype, h->N, h->M, h->d, h->P, h->row_stride, h->X, t0 + r,
                                                           rounds - r, &plan);
        if (refresh && r > 0) {
            const uint8_t *presence = s->group_skip ? h->d_masks_raw : h->d_masks;
            // peers that return per round: about p * N under the seeded schedules; unknown for explicit ones
            const int64_t guess = s->kind == MOSHPIT_SCHED_EXPLICIT
                                      ? h->N / 4
                                      : static_cast<int64_t>(1.5 * s->p * static_cast<double>(h->N)) + 16;
            rc = queue_refresh(h, t0 + r, s->seed, presence + static_cast<int64_t>(r - 1) * h->N,
                               presence + static_cast<int64_t>(r) * h->N, true, guess);
            if (rc != MOSHPIT_OK) return rc;
        }
        if (round_ms_out_host) HIP_TRY(h, hipEventRecord(h->events[2 * pass], h->stream));
        int32_t done = 1;
        if (fuse) {
            plan.grad = step_now ? static_cast<const char *>(grad) : nullptr;
            plan.gamma = gamma;
            HIP_TRY(h, launch_fused_rounds(h->X, h->dtype, plan, mask_r, h->stream));
            done = plan.rounds;
        } else if (step_now) {
            RoundGeom geom{h->N, h->M, axis_stride(h, t0 + r)};
            geom.grad = static_cast<const char *>(grad);
            geom.grad_row_bytes = grad_row_stride * (h->dtype == MOSHPIT_F32 ? 4 : 2);
            geom.gamma = gamma;
            HIP_TRY(h, launch_group_mean(h->X, h->dtype, h->P, h->row_stride, geom, mask_r, h->tune, h->stream));
        } else {
            rc = queue_round(h, t0 + r, mask_r, present_fraction(s));
            if (rc != MOSHPIT_OK) return rc;
        }
        if (round_ms_out_host) HIP_TRY(h, hipEventRecord(h->events[2 * pass + 1], h->stream));
        r += done;
        pass_rounds.push_back(done);
        if (dist_out_host) {
            rc = queue_dist(h, h->d_dist + r);
            if (rc != MOSHPIT_OK) return rc;
            have_dist[r] = true;
        }
    }
    if (dist_out_host || round_ms_out_host) {
        if (dist_out_host)
            HIP_TRY(h, hipMemcpyAsync(dist_out_host, h->d_dist, sizeof(double) * (static_cast<size_t>(rounds) + 1),
                                      hipMemcpyDeviceToHost, h->stream));
        HIP_TRY(h, hipStreamSynchronize(h->stream));
        if (dist_out_host)
            for (int32_t i = 0; i <= rounds; ++i)
                if (!have_dist[i]) dist_out_host[i] = std::nan("");
        if (round_ms_out_host) {
            int32_t first = 0;
            for (size_t pass = 0; pass < pass_rounds.size(); ++pass) {
                float ms = 0.f;
                HIP_TRY(h, hipEventElapsedTime(&ms, h->events[2 * pass], h->events[2 * pass + 1]));
                for (int32_t i = 0; i < pass_rounds[pass]; ++i)
                    round_ms_out_host[first + i] = ms / static_cast<float>(pass_rounds[pass]);
                first += pass_rounds[pass];
            }
        }
    }
    return MOSHPIT_OK;
}
}  // namespace

int moshpit_run(moshpit_ctx *h, int64_t t0, int32_t rounds, const moshpit_schedule *s, int32_t flags,
                double *dist_out_host, float *round_ms_out_host)
{
    return run_impl(h, t0, rounds, s, flags, dist_out_host, round_ms_out_host, nullptr, 0, 0.f);
}

int moshpit_dist_to_mean(moshpit_ctx *h, double *out_host)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (!out_host) return fail(h, MOSHPIT_EINVAL, "out is NULL");
    rc = queue_dist(h, h->d_dist);
    if (rc != MOSHPIT_OK) return rc;
    HIP_TRY(h, hipMemcpyAsync(out_host, h->d_dist, sizeof(double), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return MOSHPIT_OK;
}

int moshpit_dist_to_mean_static(const void *state_dev, int64_t N, int64_t P, int64_t row_stride_elems,
                                int32_t dtype, void *hip_stream, double *out_dev)
{
    if (!state_dev || !out_dev) return fail(nullptr, MOSHPIT_EINVAL, "state or output pointer is NULL");
    if (N < 1 || P < 1 || row_stride_elems < P) return fail(nullptr, MOSHPIT_EINVAL, "bad shape: N, P >= 1 and row stride >= P");
    if (dtype != MOSHPIT_F32 && dtype != MOSHPIT_BF16) return fail(nullptr, MOSHPIT_EINVAL, "unknown dtype %d", dtype);
    const int64_t esize = dtype == MOSHPIT_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(state_dev) % esize != 0)
        return fail(nullptr, MOSHPIT_EINVAL, "state pointer is not aligned to the element size");
    if (reinterpret_cast<uintptr_t>(out_dev) % sizeof(double) != 0)
        return fail(nullptr, MOSHPIT_EINVAL, "output pointer is not aligned to 8 bytes");
    const int64_t need = dist_partials_count(dtype, P, row_stride_elems, state_dev);
    if (need > kStaticPartials)
        return fail(nullptr, MOSHPIT_EINVAL,
                    "rows of %lld elements need %lld partial sums, the static scratch holds %lld "
                    "(at most %lld columns in 16-byte-aligned rows): use moshpit_dist_to_mean",
                    (long long)P, (long long)need, (long long)kStaticPartials,
                    (long long)(kStaticPartials * 64 * (16 / esize)));
    double *partials = nullptr;
    hipError_t e = static_scratch(&partials);
    if (e == hipSuccess)
        e = launch_dist_to_mean(state_dev, dtype, N, P, row_stride_elems, partials, out_dev, nullptr, 0, N,
                                static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(nullptr, MOSHPIT_EHIP, "moshpit_dist_to_mean_static: %s", hipGetErrorString(e));
    return MOSHPIT_OK;
}

int moshpit_dist_to_mean_subset(moshpit_ctx *h, const uint8_t *present_host, double *out_host)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (!out_host) return fail(h, MOSHPIT_EINVAL, "out is NULL");
    if (!present_host) return moshpit_dist_to_mean(h, out_host);
    int64_t first = -1, n = 0;
    for (int64_t i = 0; i < h->N; ++i)
        if (present_host[i] != 0) {
            if (first < 0) first = i;
            ++n;
        }
    if (n == 0) {
        *out_host = 0.0;
        return MOSHPIT_OK;
    }
    if (!h->d_present) HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_present), static_cast<size_t>(h->N)));
    rc = stage_to_device(h, h->d_present, present_host, static_cast<size_t>(h->N));
    if (rc != MOSHPIT_OK) return rc;
    HIP_TRY(h, launch_dist_to_mean(h->X, h->dtype, h->N, h->P, h->row_stride, h->d_partials, h->d_dist, h->d_present,
                                   first, n, h->stream));
    HIP_TRY(h, hipMemcpyAsync(out_host, h->d_dist, sizeof(double), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return MOSHPIT_OK;
}

namespace {
// Queue one round over consecutive chunks of `group_size` entries of a device peer list.
int queue_list_round(moshpit_ctx *h, const int32_t *index_dev, int64_t n_index, int32_t group_size,
                     const uint8_t *alive_host)
{
    const uint8_t *alive_dev = nullptr;
    if (alive_host) {
        int rc = stage_to_device(h, h->d_round_mask, alive_host, static_cast<size_t>(h->N));
        if (rc != MOSHPIT_OK) return rc;
        alive_dev = h->d_round_mask;
    }
    RoundGeom geom{h->N, group_size, 1, index_dev, n_index};
    HIP_TRY(h, launch_group_mean(h->X, h->dtype, h->P, h->row_stride, geom, alive_dev, h->tune, h->stream));
    return MOSHPIT_OK;
}
}  // namespace

namespace {
int check_grad(moshpit_ctx *h, const void *grad_dev, int64_t grad_row_stride)
{
    if (!grad_dev) return fail(h, MOSHPIT_EINVAL, "gradient pointer is NULL");
    if (grad_row_stride < h->P) return fail(h, MOSHPIT_EINVAL, "gradient row stride < P");
    const int64_t esize = h->dtype == MOSHPIT_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(grad_dev) % esize != 0)
        return fail(h, MOSHPIT_EINVAL, "gradient pointer is not aligned to the element size");
    return MOSHPIT_OK;
}

const uint8_t *stage_mask(moshpit_ctx *h, const uint8_t *alive_host, int *rc)
{
    *rc = MOSHPIT_OK;
    if (!alive_host) return nullptr;
    *rc = stage_to_device(h, h->d_round_mask, alive_host, static_cast<size_t>(h->N));
    return h->d_round_mask;
}
}  // namespace

int moshpit_sgd_round(moshpit_ctx *h, int64_t t, const uint8_t *alive_host, const void *grad_dev,
                      int64_t grad_row_stride_elems, float gamma)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (t < 0) return fail(h, MOSHPIT_EINVAL, "round index must be >= 0");
    rc = check_grad(h, grad_dev, grad_row_stride_elems);
    if (rc != MOSHPIT_OK) return rc;
    const uint8_t *alive_dev = stage_mask(h, alive_host, &rc);
    if (rc != MOSHPIT_OK) return rc;
    RoundGeom geom{h->N, h->M, axis_stride(h, t)};
    geom.grad = static_cast<const char *>(grad_dev);
    geom.grad_row_bytes = grad_row_stride_elems * (h->dtype == MOSHPIT_F32 ? 4 : 2);
    geom.gamma = gamma;
    HIP_TRY(h, launch_group_mean(h->X, h->dtype, h->P, h->row_stride, geom, alive_dev, h->tune, h->stream));
    return MOSHPIT_OK;
}

int moshpit_sgd_run(moshpit_ctx *h, int64_t t0, int32_t rounds, const moshpit_schedule *s, int32_t flags,
                    const void *grad_dev, int64_t grad_row_stride_elems, float gamma, double *dist_out_host,
                    float *round_ms_out_host)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (rounds < 1) return fail(h, MOSHPIT_EINVAL, "an iteration with averaging needs at least one round");
    rc = check_grad(h, grad_dev, grad_row_stride_elems);
    if (rc != MOSHPIT_OK) return rc;
    return run_impl(h, t0, rounds, s, flags, dist_out_host, round_ms_out_host, grad_dev, grad_row_stride_elems, gamma);
}

int moshpit_local_step(moshpit_ctx *h, const uint8_t *alive_host, const void *grad_dev,
                       int64_t grad_row_stride_elems, float gamma)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    rc = check_grad(h, grad_dev, grad_row_stride_elems);
    if (rc != MOSHPIT_OK) return rc;
    const uint8_t *alive_dev = stage_mask(h, alive_host, &rc);
    if (rc != MOSHPIT_OK) return rc;
    HIP_TRY(h, launch_local_step(h->X, h->dtype, h->N, h->P, h->row_stride, grad_dev, grad_row_stride_elems,
                                 alive_dev, gamma, h->stream));
    return MOSHPIT_OK;
}

namespace {
// one allocation: [keys N*(d-1)][packed N][count K+1][first K+1][index n_index]
struct DynLayout {
    int64_t kd, n_keys, n_index;
    int32_t *keys, *packed, *count, *first, *index;
};

DynLayout dyn_layout(const moshpit_ctx *h)
{
    DynLayout L;
    L.kd = h->d - 1;
    L.n_keys = 1;
    for (int q = 0; q < L.kd; ++q) L.n_keys *= h->M;
    L.n_index = (h->N / h->M + L.n_keys) * h->M;
    L.keys = h->d_dyn;
    L.packed = L.keys + h->N * L.kd;
    L.count = L.packed + h->N;
    L.first = L.count + (L.n_keys + 1);
    L.index = L.first + (L.n_keys + 1);
    return L;
}

int dyn_ensure(moshpit_ctx *h)
{
    int rc = reserve_sort(h);
    if (rc != MOSHPIT_OK) return rc;
    if (h->d_dyn) return MOSHPIT_OK;
    DynLayout L = dyn_layout(h);
    const size_t words = static_cast<size_t>(h->N * L.kd + h->N + 2 * (L.n_keys + 1) + L.n_index);
    HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_dyn), words * sizeof(int32_t)));
    L = dyn_layout(h);
    HIP_TRY(h, launch_dynamic_init(h->N, h->M, h->d, L.keys, h->stream));
    return MOSHPIT_OK;
}
}  // namespace

int moshpit_dynamic_reset(moshpit_ctx *h)
{
    if (!h) return MOSHPIT_EINVAL;
    if (h->d_dyn) {
        HIP_TRY(h, launch_dynamic_init(h->N, h->M, h->d, dyn_layout(h).keys, h->stream));
        return MOSHPIT_OK;
    }
    return dyn_ensure(h);
}

int moshpit_dynamic_round(moshpit_ctx *h, int64_t t, uint64_t seed, const uint8_t *alive_host)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (t < 0) return fail(h, MOSHPIT_EINVAL, "round index must be >= 0");
    rc = dyn_ensure(h);
    if (rc != MOSHPIT_OK) return rc;
    const uint8_t *alive_dev = stage_mask(h, alive_host, &rc);
    if (rc != MOSHPIT_OK) return rc;
    const DynLayout L = dyn_layout(h);
    HIP_TRY(h, launch_dynamic_grouping(h->N, h->M, h->d, seed, t, alive_dev, L.keys, L.packed, L.count, L.first,
                                       L.index, L.n_index, h->d_sort, h->stream));
    RoundGeom geom{h->N, h->M, 1, L.index, L.n_index};
    HIP_TRY(h, launch_group_mean(h->X, h->dtype, h->P, h->row_stride, geom, nullptr, h->tune, h->stream));
    return MOSHPIT_OK;
}

int moshpit_dynamic_keys(moshpit_ctx *h, int32_t *keys_host)
{
    if (!h) return MOSHPIT_EINVAL;
    if (!keys_host && h->d > 1) return fail(h, MOSHPIT_EINVAL, "keys output is NULL");
    int rc = dyn_ensure(h);
    if (rc != MOSHPIT_OK) return rc;
    const DynLayout L = dyn_layout(h);
    if (L.kd > 0)
        HIP_TRY(h, hipMemcpyAsync(keys_host, L.keys, sizeof(int32_t) * static_cast<size_t>(h->N * L.kd),
                                  hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return MOSHPIT_OK;
}

int moshpit_random_permutation(moshpit_ctx *h, int64_t t, uint64_t seed, int32_t *perm_host)
{
    if (!h) return MOSHPIT_EINVAL;
    if (t < 0 || !perm_host) return fail(h, MOSHPIT_EINVAL, "bad round index or NULL output");
    int rc = reserve_sort(h);
    if (rc != MOSHPIT_OK) return rc;
    HIP_TRY(h, launch_random_permutation(seed, t, h->N, h->d_keys, h->d_sort, h->stream));
    HIP_TRY(h, hipMemcpyAsync(perm_host, h->d_keys, sizeof(int32_t) * static_cast<size_t>(h->N),
                              hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return MOSHPIT_OK;
}

int moshpit_random_groups_round(moshpit_ctx *h, int64_t t, uint64_t seed, int32_t group_size,
                                const uint8_t *alive_host)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (t < 0) return fail(h, MOSHPIT_EINVAL, "round index must be >= 0");
    if (group_size < 1 || group_size > 64) return fail(h, MOSHPIT_EINVAL, "group_size must be in [1, 64]");
    rc = reserve_sort(h);
    if (rc != MOSHPIT_OK) return rc;
    if (!h->d_perm) HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_perm), sizeof(int32_t) * static_cast<size_t>(h->N)));
    HIP_TRY(h, launch_random_permutation(seed, t, h->N, h->d_perm, h->d_sort, h->stream));
    return queue_list_round(h, h->d_perm, h->N, group_size, alive_host);
}

int moshpit_refresh(moshpit_ctx *h, int64_t t, uint64_t seed, const uint8_t *alive_prev_host,
                    const uint8_t *alive_cur_host)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (t < 0) return fail(h, MOSHPIT_EINVAL, "round index must be >= 0");
    rc = stage_refresh_masks(h, alive_prev_host, alive_cur_host);
    if (rc != MOSHPIT_OK) return rc;
    int64_t returning = 0;                     // (the masks are on the host: count, to size the copy's launch)
    for (int64_t i = 0; i < h->N; ++i) returning += (alive_cur_host[i] != 0 && alive_prev_host[i] == 0) ? 1 : 0;
    return queue_refresh(h, t, seed, h->d_refresh_masks, h->d_refresh_masks + h->N, true, returning);
}

int moshpit_refresh_donors(moshpit_ctx *h, int64_t t, uint64_t seed, const uint8_t *alive_prev_host,
                           const uint8_t *alive_cur_host, int32_t *donors_host)
{
    if (!h) return MOSHPIT_EINVAL;
    if (t < 0) return fail(h, MOSHPIT_EINVAL, "round index must be >= 0");
    if (!donors_host) return fail(h, MOSHPIT_EINVAL, "donors is NULL");
    int rc = stage_refresh_masks(h, alive_prev_host, alive_cur_host);
    if (rc != MOSHPIT_OK) return rc;
    rc = queue_refresh(h, t, seed, h->d_refresh_masks, h->d_refresh_masks + h->N, false, 0);
    if (rc != MOSHPIT_OK) return rc;
    HIP_TRY(h, hipMemcpyAsync(donors_host, h->d_refresh + h->N, sizeof(int32_t) * static_cast<size_t>(h->N),
                              hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return MOSHPIT_OK;
}

int moshpit_grouped_round(moshpit_ctx *h, const int32_t *index_host, int64_t n_index, int32_t group_size,
                          const uint8_t *alive_host)
{
    int rc = check_ready(h);
    if (rc != MOSHPIT_OK) return rc;
    if (!index_host || n_index < 0 || n_index > h->N)
        return fail(h, MOSHPIT_EINVAL, "peer list is NULL or longer than N");
    if (group_size < 1 || group_size > 64) return fail(h, MOSHPIT_EINVAL, "group_size must be in [1, 64]");
    std::vector<uint8_t> seen(static_cast<size_t>(h->N), 0);
    for (int64_t q = 0; q < n_index; ++q) {
        const int32_t r = index_host[q];
        if (r < 0 || r >= h->N) return fail(h, MOSHPIT_EINVAL, "peer list entry %lld is out of range", (long long)q);
        if (seen[r]) return fail(h, MOSHPIT_EINVAL, "peer %d is listed twice", r);
        seen[r] = 1;
    }
    if (n_index == 0) return MOSHPIT_OK;
    if (!h->d_perm) HIP_TRY(h, hipMalloc(reinterpret_cast<void **>(&h->d_perm), sizeof(int32_t) * static_cast<size_t>(h->N)));
    rc = stage_to_device(h, h->d_perm, index_host, sizeof(int32_t) * static_cast<size_t>(n_index));
    if (rc != MOSHPIT_OK) return rc;
    return queue_list_round(h, h->d_perm, n_index, group_size, alive_host);
}

int moshpit_group_keys(moshpit_ctx *h, int64_t t, int32_t *keys_host)
{
    if (!h) return MOSHPIT_EINVAL;
    if (t < 0 || !keys_host) return fail(h, MOSHPIT_EINVAL, "bad round index or NULL output");
    HIP_TRY(h, launch_group_keys(h->N, h->M, axis_stride(h, t), h->d_keys, h->stream));
    HIP_TRY(h, hipMemcpyAsync(keys_host, h->d_keys, sizeof(int32_t) * static_cast<size_t>(h->N),
                              hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return MOSHPIT_OK;
}

int moshpit_schedule_mask(moshpit_ctx *h, const moshpit_schedule *s, int64_t t0, int32_t rounds,
                          uint8_t *masks_host)
{
    if (!h) return MOSHPIT_EINVAL;
    int rc = check_schedule(h, s, t0, rounds);
    if (rc != MOSHPIT_OK) return rc;
    if (rounds == 0) return MOSHPIT_OK;
    if (!masks_host) return fail(h, MOSHPIT_EINVAL, "masks output is NULL");
    rc = queue_masks(h, s, t0, rounds);
    if (rc != MOSHPIT_OK) return rc;
    HIP_TRY(h, hipMemcpyAsync(masks_host, h->d_masks, static_cast<size_t>(rounds) * h->N, hipMemcpyDeviceToHost,
                              h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return MOSHPIT_OK;
}

int moshpit_sync(moshpit_ctx *h)
{
    if (!h) return MOSHPIT_EINVAL;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return MOSHPIT_OK;
}

int moshpit_set_tuning(moshpit_ctx *h, int32_t cols, int32_t unroll, int32_t nontemporal, int32_t block,
                       int32_t waves_per_cu, int32_t order)
{
    if (!h) return MOSHPIT_EINVAL;
    if (cols > 0 || unroll > 0) {
        static const int ok[][2] = {{1, 4}, {1, 8}, {1, 16}, {1, 32}, {2, 2}, {2, 4}, {2, 8}, {2, 16},
                                   {4, 2}, {4, 4}, {4, 8}};
        bool found = false;
        for (const auto &pair : ok) found = found || (pair[0] == cols && pair[1] == unroll);
        if (!found) return fail(h, MOSHPIT_EINVAL, "unsupported launch shape cols=%d unroll=%d", cols, unroll);
    }
    h->tune.cols = cols;
    h->tune.unroll = unroll;
    if (block != 0 && block != 64 && block != 128 && block != 256)
        return fail(h, MOSHPIT_EINVAL, "block must be 0, 64, 128 or 256");
    if (waves_per_cu < 0 || waves_per_cu > 32) return fail(h, MOSHPIT_EINVAL, "waves_per_cu must be in [0, 32]");
    if (order < -1 || order > 1) return fail(h, MOSHPIT_EINVAL, "order must be -1, 0 or 1");
    h->tune.nt = nontemporal;
    h->tune.block = block;
    h->tune.waves_per_cu = waves_per_cu;
    h->tune.order = order;
    return MOSHPIT_OK;
}

int moshpit_copy_probe(void *dst_dev, const void *src_dev, int64_t nbytes, void *hip_stream)
{
    if (!dst_dev || !src_dev || nbytes < 0 || nbytes % 16 != 0) return MOSHPIT_EINVAL;
    if (reinterpret_cast<uintptr_t>(dst_dev) % 16 || reinterpret_cast<uintptr_t>(src_dev) % 16) return MOSHPIT_EINVAL;
    return launch_copy_probe(dst_dev, src_dev, nbytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? MOSHPIT_OK
               : MOSHPIT_EHIP;
}

int moshpit_check_bf16_rounding(void *hip_stream, uint64_t *mismatches_out_host)
{
    if (!mismatches_out_host) return MOSHPIT_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned long long *count = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&count), sizeof(unsigned long long)) != hipSuccess) return MOSHPIT_EHIP;
    unsigned long long host = 0;
    bool ok = hipMemsetAsync(count, 0, sizeof(unsigned long long), stream) == hipSuccess;
    ok = ok && launch_bf16_rounding_check(count, stream) == hipSuccess;
    ok = ok && hipMemcpyAsync(&host, count, sizeof(host), hipMemcpyDeviceToHost, stream) == hipSuccess;
    ok = ok && hipStreamSynchronize(stream) == hipSuccess;
    (void)hipFree(count);
    if (!ok) return MOSHPIT_EHIP;
    *mismatches_out_host = host;
    return MOSHPIT_OK;
}

const char *moshpit_last_error(moshpit_ctx *h) { return h ? h->err : g_create_err; }

}  // extern "C"
