/*
 * moshpit.h - C ABI of libmoshpit: Moshpit All-Reduce group-averaging rounds
 * for N virtual peers whose parameter vectors are the rows of one matrix in a
 * single MI355X's HBM.  All kernels are hand-written HIP for gfx950.
 *
 * Model (paper: Sec. 3.1, Alg. 1, Eq. 1-2; App. C.1; App. C.4 for notation).
 *   Peers i = 0..N-1 are the vertices of the grid {0..M-1}^d, N = M^d;
 *   coordinate q of peer i is the q-th base-M digit of i.  Round t averages
 *   along coordinate a = t mod d: peers that agree in every other coordinate
 *   form a group (at most M members, row stride M^a), and every member that
 *   takes part in the round replaces its vector by the mean over the members
 *   that take part.  A peer that does not take part keeps its vector and is
 *   neither read nor written.  Rounds are numbered from 0.
 *
 * State layout.  X is row-major [N][row_stride] in device memory, P <=
 * row_stride valid elements per row, element type float (binary32) or
 * bfloat16.  Sums are accumulated in binary32 and rounded once, to nearest
 * even, when stored.  The caller owns X; the library never allocates, frees or
 * copies it.
 *
 * Conventions.  Every function returns MOSHPIT_OK (0) or a negative
 * MOSHPIT_E* code and never throws; moshpit_last_error() gives a message for
 * the last failure on that handle.  "host" / "device" says where a pointer
 * must live.  Calls on one handle must not overlap in time; different handles
 * are independent.  Work is queued on the stream given to
 * moshpit_bind_state(); unless stated otherwise a call returns without waiting
 * for the GPU.
 */
#ifndef MOSHPIT_H
#define MOSHPIT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moshpit_ctx moshpit_ctx;   /* opaque; created/destroyed by the library */

enum { MOSHPIT_F32 = 0, MOSHPIT_BF16 = 1 };

enum {
    MOSHPIT_OK     = 0,
    MOSHPIT_EINVAL = -1,   /* bad argument (shape, alignment, range, NULL)      */
    MOSHPIT_ENOMEM = -2,   /* host or device allocation failed                  */
    MOSHPIT_EHIP   = -3,   /* a HIP runtime call failed; see moshpit_last_error */
    MOSHPIT_ESTATE = -4    /* no state bound yet                                */
};

/* Failure schedule of a multi-round run (Sec. 4.1: each peer fails in a round
 * with probability p and comes back later).  The paper gives no generator; the
 * library uses a counter-based one so a schedule is a pure function of
 * (seed, round, peer):
 *   mix(x): x ^= x>>32; x *= 0x9E3779B97F4A7C15; x ^= x>>29;
 *           x *= 0x6A09E667F3BCC909; x ^= x>>32                  (mod 2^64)
 *   event(s,i) = (mix(mix(seed + 0x9E3779B97F4A7C15*(s+1)) ^ i) >> 40)
 *                < floor(p * 2^24)
 * kind MOSHPIT_SCHED_NONE     nobody ever fails;
 * kind MOSHPIT_SCHED_IID      peer i is absent in round s iff event(s,i);
 * kind MOSHPIT_SCHED_REJOIN   a present peer for which event(s,i) fires is
 *                             absent for rounds s..s+down_rounds-1, draws
 *                             nothing meanwhile and is present again (with its
 *                             stale vector, drawing again) from s+down_rounds;
 *                             the recursion starts at round 0;
 * kind MOSHPIT_SCHED_EXPLICIT masks are given by the caller.
 * A REJOIN schedule depends on its past.  The handle keeps, per peer, the
 * rounds it still sits out at the end of the last schedule it generated, so a
 * run (or moshpit_schedule_mask) that starts at or after that round with the
 * same seed, p and down_rounds goes on from there and costs time proportional
 * to the rounds in between; any other start walks the rounds from 0 once. */
enum {
    MOSHPIT_SCHED_NONE = 0, MOSHPIT_SCHED_IID = 1,
    MOSHPIT_SCHED_REJOIN = 2, MOSHPIT_SCHED_EXPLICIT = 3
};

typedef struct {
    int32_t  kind;
    int32_t  down_rounds;           /* kind REJOIN: >= 1                          */
    double   p;                     /* failure probability in [0,1]               */
    uint64_t seed;
    const uint8_t *explicit_masks;  /* kind EXPLICIT: host, [rounds][N], 1=alive  */
    int32_t  group_skip;            /* 0: the members that are present average
                                       (App. E: a group is formed from whoever
                                       remains); 1: a group with an absent
                                       member sits the round out (Sec. 3.1: a
                                       failure during the all-reduce makes the
                                       groupmates skip the round)               */
    int32_t  refresh;               /* 1: before every round of a run but its
                                       first, a peer that returns takes the
                                       parameters of an up-to-date peer (see
                                       moshpit_refresh), drawn with `seed`; such
                                       a run is never fused                      */
} moshpit_schedule;

/* Flags of moshpit_run.
 * MOSHPIT_RUN_FUSED allows consecutive rounds to run in one pass over HBM: a
 * tile made of the M^F rows of an F-dimensional sub-grid (F distinct axes) and
 * a slice of columns is closed under rounds on those axes, so it is loaded
 * once, averaged F times on chip (any number of times when F = d) and stored
 * once.  The state after a fused pass is bit-identical to the state after the
 * same rounds run one by one.  Where fusion does not apply or does not pay
 * (rows not 16-byte aligned, a sub-grid too tall for on-chip memory, a single
 * round left, two rounds on a sub-grid so tall that its rows get only 128
 * bytes on chip) the rounds run one by one. */
enum {
    MOSHPIT_RUN_DEFAULT = 0,
    MOSHPIT_RUN_FUSED   = 1
};

/* Create a handle for N = M^d peers with P parameters each.
 * Requires 2 <= M <= 64, d >= 1, N == M^d, P >= 1, dtype F32 or BF16;
 * otherwise MOSHPIT_EINVAL and *out = NULL.  Allocates only small device
 * scratch (masks, keys, reduction partials) on the current HIP device. */
int moshpit_create(int64_t N, int64_t P, int32_t M, int32_t d, int32_t dtype, moshpit_ctx **out);

/* Free the handle and its scratch (waits for the bound stream first). */
int moshpit_destroy(moshpit_ctx *h);

/* Attach the peer-state matrix.  state_dev: device, borrowed, must stay valid
 * while the handle uses it.  row_stride_elems >= P.  Rows that start on 16-byte
 * boundaries (state_dev and row_stride_elems*elem_size multiples of 16) take
 * the 128-bit path; anything else is still correct through an element-wise
 * path.  hip_stream: a hipStream_t, or NULL for the default stream. */
int moshpit_bind_state(moshpit_ctx *h, void *state_dev, int64_t row_stride_elems, void *hip_stream);

/* One averaging round t >= 0 (Alg. 1, one pass of its loop body; App. C.3's
 * group-average formula with the group J_{i,t} of App. C.4).
 * alive_host: host, N bytes, non-zero = the peer takes part; NULL = all do.
 * The mask has been read completely when the call returns, whether it lives in
 * pageable or in pinned host memory (the library copies it into a staging
 * buffer of its own first; the same holds for every host mask, explicit
 * schedule and peer list below); the round itself is queued. */
int moshpit_round(moshpit_ctx *h, int64_t t, const uint8_t *alive_host);

/* Same, with the mask already in device memory (device, N bytes, must stay
 * unchanged until the round has run; NULL = all peers take part).  The call
 * only launches kernels on the bound stream, so it may be recorded into a HIP
 * graph by a caller that captures that stream; run one round of each axis
 * outside the capture first (the first launch of a kernel shape also sets a
 * function attribute, which is not a stream operation). */
int moshpit_round_dev(moshpit_ctx *h, int64_t t, const uint8_t *alive_dev);

/* Rounds t0 .. t0+rounds-1 (the loop of Alg. 1) under a failure schedule
 * (NULL = nobody fails).  Masks are generated on the device.
 * dist_out_host: NULL, or host array of rounds+1 doubles that receives the
 *   average distortion (see moshpit_dist_to_mean) before the first round and
 *   after every round.  With MOSHPIT_RUN_FUSED the state between the rounds of
 *   one pass never exists in memory; those entries are NaN.
 * round_ms_out_host: NULL, or host array of `rounds` floats that receives the
 *   GPU time of each round's averaging kernel in milliseconds (a fused pass's
 *   time is split evenly over its rounds).
 * If either output array is given the call waits for the GPU before it
 * returns; otherwise it only queues the work. */
int moshpit_run(moshpit_ctx *h, int64_t t0, int32_t rounds, const moshpit_schedule *s,
                int32_t flags, double *dist_out_host, float *round_ms_out_host);

/* Average distortion (1/N) * sum_i ||theta_i - theta_bar||^2 over all N rows,
 * theta_bar = (1/N) sum_i theta_i (left-hand side of the equation of Thm 3.2;
 * the error measure of Sec. 4.1).  Accumulated in binary64.  Waits for the
 * GPU.  out_host: host, one double. */
int moshpit_dist_to_mean(moshpit_ctx *h, double *out_host);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * serving loops, harnesses that forbid hipMalloc): the average distortion of
 * moshpit_dist_to_mean without a handle and without any allocation, host
 * synchronisation or copy.  The partial sums of its first kernel live in a
 * fixed 1 MiB array inside the library's code object (one copy per GPU, held
 * until the process ends) instead of the handle's scratch.
 * state_dev: device, [N][row_stride_elems], P valid elements per row, dtype
 * MOSHPIT_F32 / MOSHPIT_BF16, borrowed until the queued work has run.
 * out_dev: device, one double, 8-byte aligned; written by the second kernel.
 * hip_stream: a hipStream_t or NULL; the two kernels are queued there and the
 * call returns at once.  Same kernels, same order of additions, hence the same
 * bits as moshpit_dist_to_mean.
 * Limit: at most 131072 partial sums, i.e. P <= 33,554,432 binary32 or
 * 67,108,864 bfloat16 columns when rows are 16-byte aligned (one partial per
 * 64 vectors of 16 bytes), P <= 8,388,608 otherwise (one per 64 elements);
 * beyond that MOSHPIT_EINVAL and nothing is queued.
 * All calls on one GPU share the one array: calls that may overlap in time on
 * the same GPU (different streams, different threads) race and must be ordered
 * by the caller.  Nothing needs clearing between calls: every partial that is
 * read has been written by the same call.  The array's address is looked up
 * once per device (at moshpit_create, else at the first call on that device);
 * make that first call outside a graph capture.
 * Errors: message through moshpit_last_error(NULL). */
int moshpit_dist_to_mean_static(const void *state_dev, int64_t N, int64_t P, int64_t row_stride_elems,
                                int32_t dtype, void *hip_stream, double *out_dev);

/* The same measure over the peers that exist when the grid is only partly
 * filled (Sec. 3.1 after Eq. 2; the partly filled grids of Sec. 4.1 / Table 4):
 * mean and average run over the rows with present_host[i] != 0 only.  A vertex
 * without a peer is modelled as a row that never takes part in a round (its
 * alive byte is 0 in every round) and is left out here.  present_host: host,
 * N bytes, NULL = every row.  Waits for the GPU.  All rows absent gives 0. */
int moshpit_dist_to_mean_subset(moshpit_ctx *h, const uint8_t *present_host, double *out_host);

/* Group key of every peer for round t (Eq. 1 on the static grid: the d-1
 * coordinates other than t mod d, read in increasing coordinate order as a
 * base-M number).  Computed on the device; waits.  keys_host: host, N int32. */
int moshpit_group_keys(moshpit_ctx *h, int64_t t, int32_t *keys_host);

/* The masks moshpit_run would use for rounds t0..t0+rounds-1 under schedule s,
 * generated by the same device kernel; waits.
 * masks_host: host, [rounds][N] bytes, 1 = alive. */
int moshpit_schedule_mask(moshpit_ctx *h, const moshpit_schedule *s, int64_t t0, int32_t rounds,
                          uint8_t *masks_host);

/* Alg. 1 with chunk-index keys (Eq. 1 and the key shift of Alg. 1) instead of
 * fixed grid coordinates.  The handle keeps a key of d-1 chunk indices per
 * peer, initially coordinates 1..d-1 of the peer index (Eq. 2).  Round t:
 * the peers that take part and carry equal keys are ordered by
 *   mix(mix(seed + 0xD1B54A32D192ED03*(t+1)) ^ i), ties by index
 * (the random order of peers_t), cut into consecutive groups of at most M,
 * averaged group by group, and every member shifts its position in its group
 * into its key: C_i := (C_i[1:], c_i).  A peer that sits the round out keeps
 * vector and key.  With all peers present, d rounds give the exact global mean
 * whatever the seed.  N <= 2^24 (the round sorts 16 bytes per peer on the device).
 * moshpit_dynamic_reset restores the initial keys; moshpit_dynamic_keys copies
 * the keys to the host (N x (d-1) int32, row-major; waits). */
int moshpit_dynamic_reset(moshpit_ctx *h);
int moshpit_dynamic_round(moshpit_ctx *h, int64_t t, uint64_t seed, const uint8_t *alive_host);
int moshpit_dynamic_keys(moshpit_ctx *h, int32_t *keys_host);

/* Moshpit SGD (Alg. 2).  grad_dev: device, the stochastic gradients g_i as a
 * matrix laid out like the state (same element type, P valid elements per row,
 * rows grad_row_stride_elems apart), borrowed for the duration of the queued
 * work.  alive_host as in moshpit_round: the peers of P_{k+1}.
 * moshpit_local_step: an iteration without communication,
 *   theta_i <- theta_i - gamma * g_i              for the peers that take part.
 * moshpit_sgd_round: an iteration with one Moshpit All-Reduce round t fused in,
 *   theta_i <- mean over i's round-t group of (theta_j - gamma * g_j);
 * a peer that is alone in its group just takes its local step.  The product
 * theta - gamma*g is formed in binary32 with one fused multiply-add; traffic is
 * 3 * elem_size * P bytes per participating peer. */
int moshpit_local_step(moshpit_ctx *h, const uint8_t *alive_host, const void *grad_dev,
                       int64_t grad_row_stride_elems, float gamma);

/* An iteration of Moshpit SGD whose Moshpit All-Reduce takes several rounds
 * (Alg. 2 with Alg. 1 inside; the paper's ALBERT setup runs two rounds per
 * iteration on an 8 x 8 grid, Sec. 4.3): the peers that are present in round t0
 * take their local step theta_i - gamma * g_i, then rounds t0 .. t0+rounds-1 run
 * under schedule s exactly as in moshpit_run (same flags, same outputs; rounds
 * >= 1; dist_out_host[0] is the distortion before the local step).  With
 * MOSHPIT_RUN_FUSED, a gradient matrix laid out exactly like the state (same
 * row stride, 16-byte aligned) and rounds that fuse, the local step is applied
 * while the first pass loads its tiles: the iteration then moves 3 * elem_size
 * * P bytes per participating peer and pass instead of 5.  There the stepped
 * value is rounded to the storage type before it is averaged (for binary32
 * state the result is bit-identical to moshpit_sgd_round followed by the
 * remaining rounds; for bfloat16 it differs by that one extra rounding).
 * Otherwise the first round runs as moshpit_sgd_round and the others follow. */
int moshpit_sgd_run(moshpit_ctx *h, int64_t t0, int32_t rounds, const moshpit_schedule *s, int32_t flags,
                    const void *grad_dev, int64_t grad_row_stride_elems, float gamma, double *dist_out_host,
                    float *round_ms_out_host);
int moshpit_sgd_round(moshpit_ctx *h, int64_t t, const uint8_t *alive_host, const void *grad_dev,
                      int64_t grad_row_stride_elems, float gamma);

/* Averaging in random groups: the simplified scheme analysed in Thm 3.2 and
 * compared in Sec. 4.1.  Round t orders the peers by the key
 *   mix(mix(seed + 0xD1B54A32D192ED03*(t+1)) ^ i)       (mix as for the schedule)
 * with ties broken by peer index, cuts the resulting permutation into
 * consecutive groups of group_size peers (the last one may be shorter) and
 * replaces the members of every group that take part by their mean (App. C.3,
 * proof of Thm 3.2).  1 <= group_size <= 64, N <= 2^24.  alive_host as in
 * moshpit_round.  Queued on the bound stream.
 * moshpit_random_permutation returns the permutation of round t (host, N
 * int32, perm[r] = peer of rank r), computed by the same device kernel; waits. */
int moshpit_random_groups_round(moshpit_ctx *h, int64_t t, uint64_t seed, int32_t group_size,
                                const uint8_t *alive_host);
int moshpit_random_permutation(moshpit_ctx *h, int64_t t, uint64_t seed, int32_t *perm_host);

/* A returning peer takes the parameters of an up-to-date peer before it takes
 * part again (App. "Training with a dynamic number of peers": a participant that
 * joins or has fallen behind downloads the latest parameters from a random
 * up-to-date peer, so that its stale vector does not undo the others' progress).
 * The paper fixes neither who is up to date nor the draw; here: peer i returns
 * in round t when alive_cur[i] != 0 and alive_prev[i] == 0 (the masks of rounds t
 * and t-1); the candidates are the c peers present in both rounds; the donor of
 * i is the (u mod c)-th candidate in ascending index,
 *   u = mix(mix(seed + 0xA0761D6478BD642F*(t+1)) ^ i)   (mix as for the schedule);
 * with c = 0 nothing happens.  moshpit_refresh copies row donor(i) of the state
 * onto row i for every returning peer (2*elem_size*P bytes each; queued on the
 * bound stream, masks are host pointers of N bytes, copied before return).  Call
 * it before the round t it prepares.  The global mean is NOT conserved by this
 * step.  moshpit_refresh_donors only returns the draw (host, N int32, -1 for
 * peers that do not return), computed by the same device kernel; waits. */
int moshpit_refresh(moshpit_ctx *h, int64_t t, uint64_t seed, const uint8_t *alive_prev_host,
                    const uint8_t *alive_cur_host);
int moshpit_refresh_donors(moshpit_ctx *h, int64_t t, uint64_t seed, const uint8_t *alive_prev_host,
                           const uint8_t *alive_cur_host, int32_t *donors_host);

/* One round over caller-defined groups: consecutive chunks of group_size entries
 * of the peer list index_host[0..n_index) (host; distinct peers in [0, N);
 * n_index <= N; the last chunk may be shorter).  Peers not listed are left
 * alone.  This is the group-average step of Alg. 1 for any group assignment,
 * e.g. one produced by a matchmaking layer above this library. */
int moshpit_grouped_round(moshpit_ctx *h, const int32_t *index_host, int64_t n_index, int32_t group_size,
                          const uint8_t *alive_host);

/* Measurement aids (no counterpart in the paper).
 *
 * moshpit_set_tuning overrides the launch shape of the averaging kernel:
 * cols = 128-bit vectors per thread per row, unroll = rows whose loads are
 * issued before the first add; supported (cols, unroll) pairs are (1,4) (1,8)
 * (1,16) (1,32) (2,2) (2,4) (2,8) (2,16) (4,2) (4,4) (4,8); cols = unroll = 0
 * restores the default
 * chosen from M and the dtype.  nontemporal: 1 = streaming loads/stores, 0 =
 * plain, -1 = default.  block = threads per block (64, 128, 256; 0 = default).
 * waves_per_cu = resident waves per compute unit, 1..32 (0 = default); the
 * kernel runs fastest when the row loads in flight on the whole chip stay
 * near 16-32 MiB, so groups with many rows want few resident waves.
 * order = how the (group, column tile) work items are dealt to the blocks:
 * 0 = in order, column tiles fastest; 1 = each of the 8 dies of the GPU streams
 * through an eighth of the list (steadier when the rows of a group are a few
 * MiB apart, slower otherwise); -1 = chosen from the distance between the rows
 * of a group.
 * Results never depend on nontemporal, block, waves_per_cu or order; they
 * depend on unroll only through the (documented, fixed) summation tree.
 *
 * moshpit_copy_probe queues a plain 128-bit copy of nbytes (multiple of 16,
 * both pointers device, 16-byte aligned) on hip_stream: the streaming ceiling
 * the averaging kernel is compared with, and the known-size kernel used to
 * calibrate HBM traffic counters. */
int moshpit_set_tuning(moshpit_ctx *h, int32_t cols, int32_t unroll, int32_t nontemporal, int32_t block,
                       int32_t waves_per_cu, int32_t order);
int moshpit_copy_probe(void *dst_dev, const void *src_dev, int64_t nbytes, void *hip_stream);

/* bfloat16 states are rounded to nearest, ties to even, after every round (the
 * paper's experiments run in binary32; bfloat16 storage with binary32 sums is
 * this library's option).  The kernels round with the hardware conversion of
 * gfx950; this call runs both that conversion and its definition in integer
 * arithmetic (add 0x7fff plus the lowest kept bit, keep the upper 16 bits; a NaN
 * stays a quiet NaN) over all 2^32 binary32 bit patterns on hip_stream, waits,
 * and writes the number of inputs on which they differ to *mismatches_out_host
 * (host; expected 0).  About 10 ms.  Allocates 8 bytes of device memory for the
 * duration of the call. */
int moshpit_check_bf16_rounding(void *hip_stream, uint64_t *mismatches_out_host);

/* Wait until everything queued on the bound stream has finished. */
int moshpit_sync(moshpit_ctx *h);

/* Message for the last error on this handle (library-owned, valid until the
 * next call on the handle); "" if none.  h == NULL gives the message of the
 * last failed moshpit_create on this thread. */
const char *moshpit_last_error(moshpit_ctx *h);

#ifdef __cplusplus
}
#endif
#endif /* MOSHPIT_H */
