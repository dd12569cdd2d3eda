/*
 * Moshpit All-Reduce group-averaging round: plain fp64 CPU oracle.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, obviously-correct
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or helper with the GPU path and nothing in the product may
 * call it.  Parity status: every function here is pinned by CPU tests against
 * facts the paper or plain mathematics fix (exact global mean after d rounds
 * on a full grid, sum preservation, non-increasing distortion, hand-computed
 * tiny cases, a doubly-stochastic matrix formulation, Table 4's N=1024 p=0
 * entry).  The failure-schedule generator is an input recipe (the paper gives
 * none); it is pinned by its stated distributional properties only.
 *
 * What is computed (paper notation):
 *   - peers i = 0..N-1 sit on the vertices of the hypercube {0..M-1}^d,
 *     N = M^d, one peer per vertex (Sec. 3.1, Eq. 2; App. C.1; proof of the
 *     variance theorem in App. C.4 for the hyperindex notation C_i);
 *   - in round t the peers whose hyperindices agree everywhere except in
 *     coordinate a = t mod d form a group J and every *participating* member
 *     replaces its vector by the group average (Alg. 1, the AllReduce line;
 *     App. C.3, the group-average formula; App. C.4, the definition of
 *     J_{i,t} and b_{i,t});
 *   - a peer that does not take part in a round keeps its vector; the others
 *     of its group still average among themselves (App. E, the guarantee that
 *     a group is formed from whoever remains);
 *   - the error measure is the average distortion (1/N) sum_i ||theta_i -
 *     theta_bar||^2 with theta_bar the mean over all N peers (Thm 3.2, the
 *     left-hand side of its equation; Sec. 4.1).
 *
 * Coordinate convention (a reading of the garbled Eq. 2): coordinate q of
 * peer i is the q-th base-M digit of i, floor(i / M^q) mod M, q = 0..d-1.
 *
 * The state is a row-major double matrix X[N][ld]; a call touches columns
 * 0..W-1 of every row, so a caller may hand in independent column slabs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_D 32

/* ---- hypercube coordinates ------------------------------------------- */

/* digits[q] = q-th base-M digit of i, by repeated division. */
void oracle_digits(int64_t i, int32_t M, int32_t d, int32_t *digits)
{
    int64_t rest = i;
    for (int32_t q = 0; q < d; ++q) {
        digits[q] = (int32_t)(rest % M);
        rest = rest / M;
    }
}

/* 1 when peers i and j agree in every coordinate except coordinate a. */
static int same_group(int64_t i, int64_t j, int32_t M, int32_t d, int32_t a)
{
    int32_t ci[ORACLE_MAX_D], cj[ORACLE_MAX_D];
    oracle_digits(i, M, d, ci);
    oracle_digits(j, M, d, cj);
    for (int32_t q = 0; q < d; ++q) {
        if (q == a) continue;
        if (ci[q] != cj[q]) return 0;
    }
    return 1;
}

/*
 * Group key of every peer for round t (Eq. 1 in its static-grid form: the
 * d-1 coordinates other than a = t mod d), packed into one integer by reading
 * the remaining digits, in increasing q, as a base-M number.
 */
int oracle_group_keys(int64_t N, int32_t M, int32_t d, int64_t t, int32_t *keys)
{
    if (d < 1 || d > ORACLE_MAX_D || M < 1 || t < 0) return -1;
    int32_t a = (int32_t)(t % d);
    for (int64_t i = 0; i < N; ++i) {
        int32_t c[ORACLE_MAX_D];
        oracle_digits(i, M, d, c);
        int64_t key = 0, weight = 1;
        for (int32_t q = 0; q < d; ++q) {
            if (q == a) continue;
            key += (int64_t)c[q] * weight;
            weight *= M;
        }
        keys[i] = (int32_t)key;
    }
    return 0;
}

/*
 * Group membership for round t, derived from the coordinate tuples alone
 * (no packed key, no stride arithmetic): group_id[i] = smallest peer index
 * that shares all coordinates but a with i.  O(N^2), on purpose.
 */
int oracle_group_ids(int64_t N, int32_t M, int32_t d, int64_t t, int64_t *group_id)
{
    if (d < 1 || d > ORACLE_MAX_D || M < 1 || t < 0) return -1;
    int32_t a = (int32_t)(t % d);
    for (int64_t i = 0; i < N; ++i) group_id[i] = -1;
    for (int64_t i = 0; i < N; ++i) {
        if (group_id[i] >= 0) continue;
        for (int64_t j = i; j < N; ++j)
            if (group_id[j] < 0 && same_group(i, j, M, d, a)) group_id[j] = i;
    }
    return 0;
}

/* ---- one averaging round --------------------------------------------- */

/*
 * Round t on columns 0..W-1 of X[N][ld].  alive[i] != 0 means peer i takes
 * part; alive == NULL means everybody does.  For every group the live
 * members' vectors are summed in ascending peer order, divided by their
 * count and written back to exactly those members.
 */
int oracle_round(double *X, int64_t N, int64_t W, int64_t ld,
                 int32_t M, int32_t d, int64_t t, const uint8_t *alive)
{
    int64_t *gid = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    int64_t *members = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    double *mean = (double *)malloc(sizeof(double) * (size_t)(W > 0 ? W : 1));
    if (!gid || !members || !mean) { free(gid); free(members); free(mean); return -2; }
    if (oracle_group_ids(N, M, d, t, gid) != 0) { free(gid); free(members); free(mean); return -1; }

    for (int64_t lead = 0; lead < N; ++lead) {
        if (gid[lead] != lead) continue;          /* one pass per group */
        int64_t k = 0;
        for (int64_t i = lead; i < N; ++i)
            if (gid[i] == lead && (alive == NULL || alive[i] != 0)) members[k++] = i;
        if (k == 0) continue;
        for (int64_t c = 0; c < W; ++c) mean[c] = 0.0;
        for (int64_t m = 0; m < k; ++m) {
            const double *row = X + members[m] * ld;
            for (int64_t c = 0; c < W; ++c) mean[c] += row[c];
        }
        for (int64_t c = 0; c < W; ++c) mean[c] = mean[c] / (double)k;
        for (int64_t m = 0; m < k; ++m) {
            double *row = X + members[m] * ld;
            for (int64_t c = 0; c < W; ++c) row[c] = mean[c];
        }
    }
    free(gid); free(members); free(mean);
    return 0;
}

/* ---- storage rounding (diagnostic mode only) ------------------------- */

/*
 * Nearest bfloat16 (1 sign, 8 exponent, 7 fraction bits), ties to even:
 * write v = m * 2^e with 0.5 <= |m| < 1, keep 8 significant bits of m.
 * Below the normal range the spacing is fixed at 2^-133.
 */
static double round_to_bf16(double v)
{
    if (v == 0.0 || v != v || v - v != 0.0) return v;      /* 0, nan, inf */
    int e;
    double m = frexp(v, &e);
    if (e < -125) return ldexp(nearbyint(ldexp(v, 133)), -133);
    return ldexp(nearbyint(ldexp(m, 8)), e - 8);           /* nearbyint: ties to even */
}

/*
 * Round every entry of columns 0..W-1 to the storage type: 0 = binary32,
 * 1 = bfloat16.  Used by the diagnostic "storage-quantized" run, which mimics
 * a state that lives in the storage type between rounds.
 */
int oracle_quantize(double *X, int64_t N, int64_t W, int64_t ld, int32_t dtype)
{
    if (dtype != 0 && dtype != 1) return -1;
    for (int64_t i = 0; i < N; ++i)
        for (int64_t c = 0; c < W; ++c) {
            double v = X[i * ld + c];
            X[i * ld + c] = (dtype == 0) ? (double)(float)v : round_to_bf16(v);
        }
    return 0;
}

/* ---- average distortion ---------------------------------------------- */

/*
 * (1/N) sum_i sum_{c<W} (X[i][c] - mean_c)^2, mean_c over all N rows
 * (alive or not).  Two passes, as the definition reads.  Column slabs add.
 */
double oracle_dist_to_mean(const double *X, int64_t N, int64_t W, int64_t ld)
{
    double total = 0.0;
    for (int64_t c = 0; c < W; ++c) {
        double s = 0.0;
        for (int64_t i = 0; i < N; ++i) s += X[i * ld + c];
        double mu = s / (double)N;
        double q = 0.0;
        for (int64_t i = 0; i < N; ++i) {
            double e = X[i * ld + c] - mu;
            q += e * e;
        }
        total += q;
    }
    return total / (double)N;
}

/*
 * The same measure restricted to the peers that exist: when the grid is only
 * partly filled (N < M^d, Sec. 3.1 after Eq. 2; the partly filled grids of
 * Sec. 4.1 and Table 4) the mean and the average run over the rows with
 * present[i] != 0 only.  present == NULL means every row.
 */
double oracle_dist_to_mean_subset(const double *X, int64_t N, int64_t W, int64_t ld, const uint8_t *present)
{
    int64_t n = 0;
    for (int64_t i = 0; i < N; ++i)
        if (present == NULL || present[i] != 0) ++n;
    if (n == 0) return 0.0;
    double total = 0.0;
    for (int64_t c = 0; c < W; ++c) {
        double s = 0.0;
        for (int64_t i = 0; i < N; ++i)
            if (present == NULL || present[i] != 0) s += X[i * ld + c];
        double mu = s / (double)n;
        double q = 0.0;
        for (int64_t i = 0; i < N; ++i)
            if (present == NULL || present[i] != 0) {
                double e = X[i * ld + c] - mu;
                q += e * e;
            }
        total += q;
    }
    return total / (double)n;
}

/* ---- seeded failure schedule ------------------------------------------ */

/*
 * The paper draws failures at random with a per-round probability p
 * (Sec. 4.1) and gives no generator.  Both this oracle and the GPU library
 * implement, separately, the same counter-based generator so that the two see
 * identical masks:
 *   mix(x):  x ^= x>>32; x *= 0x9E3779B97F4A7C15; x ^= x>>29;
 *            x *= 0x6A09E667F3BCC909; x ^= x>>32           (mod 2^64)
 *   u(seed,s,i) = mix( mix(seed + 0x9E3779B97F4A7C15*(s+1)) ^ i )
 *   event(s,i)  = (u >> 40) < floor(p * 2^24)
 * kind 0: nobody fails.
 * kind 1: peer i is dead in round s iff event(s,i)  (fails for that round,
 *         back in the next: Sec. 4.1).
 * kind 2: a peer that is up in round s and draws event(s,i) goes down for
 *         `down` consecutive rounds s..s+down-1, draws nothing meanwhile, and
 *         is up (drawing again) from round s+down.  Rounds count from 0.
 */
static uint64_t mix64(uint64_t x)
{
    x ^= x >> 32; x *= 0x9E3779B97F4A7C15ull;
    x ^= x >> 29; x *= 0x6A09E667F3BCC909ull;
    x ^= x >> 32;
    return x;
}

static int failure_event(uint64_t seed, int64_t s, int64_t i, uint32_t thr)
{
    uint64_t u = mix64(mix64(seed + 0x9E3779B97F4A7C15ull * (uint64_t)(s + 1)) ^ (uint64_t)i);
    return (uint32_t)(u >> 40) < thr;
}

/* masks[r][i] = 1 when peer i is alive in round t0 + r, r = 0..rounds-1. */
int oracle_schedule_masks(int32_t kind, double p, uint64_t seed, int32_t down,
                          int64_t N, int64_t t0, int32_t rounds, uint8_t *masks)
{
    if (kind < 0 || kind > 2 || !(p >= 0.0 && p <= 1.0) || t0 < 0 || rounds < 0) return -1;
    if (kind == 2 && down < 1) return -1;
    uint32_t thr = (uint32_t)(p * 16777216.0);     /* floor(p * 2^24) */
    for (int64_t i = 0; i < N; ++i) {
        if (kind == 0) {
            for (int32_t r = 0; r < rounds; ++r) masks[(int64_t)r * N + i] = 1;
        } else if (kind == 1) {
            for (int32_t r = 0; r < rounds; ++r)
                masks[(int64_t)r * N + i] = failure_event(seed, t0 + r, i, thr) ? 0 : 1;
        } else {
            int64_t down_left = 0;                 /* rounds still to sit out */
            for (int64_t s = 0; s < t0 + rounds; ++s) {
                if (down_left == 0 && failure_event(seed, s, i, thr)) down_left = down;
                int is_alive = (down_left == 0);
                if (down_left > 0) --down_left;
                if (s >= t0) masks[(s - t0) * N + i] = (uint8_t)is_alive;
            }
        }
    }
    return 0;
}

/* ---- a returning peer first takes the parameters of an up-to-date peer ---- */

/*
 * App. "Training with a dynamic number of peers": a participant that joins (or
 * comes back desynchronised) downloads the latest parameters from a random
 * up-to-date peer before it takes part again; otherwise its stale vector would
 * undo progress of the others.  The paper fixes neither who counts as up to
 * date nor the draw.  Taken here: peer i returns in round t when it is present
 * in round t and was absent in round t-1; the up-to-date peers it can reach
 * are those present in both rounds; the donor is the (u mod c)-th of these c
 * candidates in ascending index, with
 *   u(seed,t,i) = mix( mix(seed + 0xA0761D6478BD642F*(t+1)) ^ i )
 * (the generator of the failure schedule on a stream of its own).  With no
 * candidate nobody refreshes.  donor[i] = -1 for every peer that does not
 * return.  Donors never return themselves, so the copies of oracle_refresh do
 * not depend on their order.
 */
int oracle_refresh_donors(int64_t N, const uint8_t *prev, const uint8_t *cur, uint64_t seed, int64_t t,
                          int32_t *donor)
{
    if (N < 0 || t < 0 || !prev || !cur || !donor) return -1;
    int64_t c = 0;
    for (int64_t j = 0; j < N; ++j)
        if (prev[j] && cur[j]) ++c;
    for (int64_t i = 0; i < N; ++i) {
        donor[i] = -1;
        if (!(cur[i] && !prev[i]) || c == 0) continue;
        uint64_t u = mix64(mix64(seed + 0xA0761D6478BD642Full * (uint64_t)(t + 1)) ^ (uint64_t)i);
        int64_t want = (int64_t)(u % (uint64_t)c);
        for (int64_t j = 0; j < N; ++j) {
            if (!(prev[j] && cur[j])) continue;
            if (want == 0) { donor[i] = (int32_t)j; break; }
            --want;
        }
    }
    return 0;
}

/* X[i] <- X[donor[i]] for every i with donor[i] >= 0. */
int oracle_refresh(double *X, int64_t N, int64_t W, int64_t ld, const int32_t *donor)
{
    if (!X || !donor || ld < W) return -1;
    for (int64_t i = 0; i < N; ++i) {
        if (donor[i] < 0) continue;
        if (donor[i] >= N || donor[donor[i]] >= 0) return -1;      /* a donor must not be refreshing */
        for (int64_t c = 0; c < W; ++c) X[i * ld + c] = X[(int64_t)donor[i] * ld + c];
    }
    return 0;
}

/* ---- failure during the all-reduce: the whole group skips ---------------- */

/*
 * Sec. 3.1 names a second failure behaviour: a peer that fails during the
 * all-reduce makes its groupmates skip that round.  As a filter on the masks:
 * effective[i] = 1 iff every member of i's round-t group is alive (on a full
 * grid), else 0 for the whole group.  A round run with `effective` is the
 * round with group-skip semantics.
 */
int oracle_skip_filter(int64_t N, int32_t M, int32_t d, int64_t t, const uint8_t *alive, uint8_t *effective)
{
    int64_t *gid = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    if (!gid) return -2;
    if (oracle_group_ids(N, M, d, t, gid) != 0) { free(gid); return -1; }
    for (int64_t i = 0; i < N; ++i) {
        int complete = 1;
        for (int64_t j = 0; j < N; ++j)
            if (gid[j] == gid[i] && alive[j] == 0) complete = 0;
        effective[i] = (uint8_t)complete;
    }
    free(gid);
    return 0;
}

/* ---- averaging in random groups ---------------------------------------- */

/*
 * The simplified scheme analysed in Thm 3.2 (and compared in Sec. 4.1): in
 * every iteration the peers are permuted at random and the permutation is cut
 * into consecutive groups; every group averages (the construction used in the
 * proof of Thm 3.2, App. C.3).
 *
 * The permutation of round t orders the peers by the 64-bit key
 *   key(seed,t,i) = mix( mix(seed + 0xD1B54A32D192ED03*(t+1)) ^ i ),
 * ties broken by peer index (same mixer as the failure schedule, another
 * stream constant).  perm[r] = peer of rank r.  Ranks by plain counting.
 */
static uint64_t order_key(uint64_t seed, int64_t t, int64_t i)
{
    return mix64(mix64(seed + 0xD1B54A32D192ED03ull * (uint64_t)(t + 1)) ^ (uint64_t)i);
}

int oracle_random_permutation(uint64_t seed, int64_t t, int64_t N, int64_t *perm)
{
    if (t < 0 || N < 0) return -1;
    for (int64_t i = 0; i < N; ++i) {
        uint64_t ki = order_key(seed, t, i);
        int64_t rank = 0;
        for (int64_t j = 0; j < N; ++j) {
            uint64_t kj = order_key(seed, t, j);
            if (kj < ki || (kj == ki && j < i)) ++rank;
        }
        perm[rank] = i;
    }
    return 0;
}

/*
 * One round over explicit groups: group g consists of the peers
 * index[g*group_size .. min(n_index, (g+1)*group_size) - 1]; its members that
 * take part (alive != 0; alive == NULL means all) are replaced by their mean.
 * `index` must not list a peer twice.
 */
int oracle_grouped_round(double *X, int64_t N, int64_t W, int64_t ld, const int64_t *index, int64_t n_index,
                         int32_t group_size, const uint8_t *alive)
{
    if (group_size < 1 || n_index < 0) return -1;
    for (int64_t q = 0; q < n_index; ++q)
        if (index[q] < 0 || index[q] >= N) return -1;
    double *mean = (double *)malloc(sizeof(double) * (size_t)(W > 0 ? W : 1));
    if (!mean) return -2;
    for (int64_t g0 = 0; g0 < n_index; g0 += group_size) {
        int64_t g1 = g0 + group_size < n_index ? g0 + group_size : n_index;
        int64_t k = 0;
        for (int64_t c = 0; c < W; ++c) mean[c] = 0.0;
        for (int64_t q = g0; q < g1; ++q) {
            if (alive != NULL && alive[index[q]] == 0) continue;
            const double *row = X + index[q] * ld;
            for (int64_t c = 0; c < W; ++c) mean[c] += row[c];
            ++k;
        }
        if (k == 0) continue;
        for (int64_t c = 0; c < W; ++c) mean[c] = mean[c] / (double)k;
        for (int64_t q = g0; q < g1; ++q) {
            if (alive != NULL && alive[index[q]] == 0) continue;
            double *row = X + index[q] * ld;
            for (int64_t c = 0; c < W; ++c) row[c] = mean[c];
        }
    }
    free(mean);
    return 0;
}

/* Round t of random-group averaging with groups of `group_size` peers. */
int oracle_random_groups_round(double *X, int64_t N, int64_t W, int64_t ld, uint64_t seed, int64_t t,
                               int32_t group_size, const uint8_t *alive)
{
    int64_t *perm = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    if (!perm) return -2;
    int rc = oracle_random_permutation(seed, t, N, perm);
    if (rc == 0) rc = oracle_grouped_round(X, N, W, ld, perm, N, group_size, alive);
    free(perm);
    return rc;
}

/* ---- Alg. 1 with chunk-index keys ---------------------------------------- */

/*
 * Alg. 1 as written: every peer carries the key C_i of its d-1 most recent
 * chunk indices (Eq. 1); peers with equal keys form a group; after the group's
 * all-reduce each member receives a chunk index c_i that is unique within the
 * group (its position in the randomly ordered list peers_t) and shifts it into
 * its key: C_i := (C_i[1:], c_i).  Two peers that just averaged together
 * therefore never share the next group (Sec. 3.1).
 *
 * Readings where the paper is silent:
 *   - initial key (Eq. 2): coordinates 1..d-1 of the peer index, so the first
 *     round groups M consecutive peers, like the static grid;
 *   - the random order of peers_t: ascending order_key(seed, t, i), ties by
 *     index; c_i = rank among the members that take part;
 *   - a peer that does not take part keeps vector and key;
 *   - if more than M peers that take part share a key (possible once peers
 *     with stale keys return), the ordered list is cut into consecutive groups
 *     of M; c_i is the position within its group of at most M.
 * keys: N x (d-1) int32, row-major, updated in place (d == 1: no key, all
 * peers share the empty key).
 */
int oracle_dynamic_init(int64_t N, int32_t M, int32_t d, int32_t *keys)
{
    if (d < 1 || d > ORACLE_MAX_D || M < 1) return -1;
    for (int64_t i = 0; i < N; ++i) {
        int32_t c[ORACLE_MAX_D];
        oracle_digits(i, M, d, c);
        for (int32_t q = 1; q < d; ++q) keys[i * (d - 1) + (q - 1)] = c[q];
    }
    return 0;
}

int oracle_dynamic_round(double *X, int64_t N, int64_t W, int64_t ld, int32_t M, int32_t d, int32_t *keys,
                         uint64_t seed, int64_t t, const uint8_t *alive)
{
    if (d < 1 || d > ORACLE_MAX_D || M < 1 || t < 0) return -1;
    const int32_t kd = d - 1;
    uint8_t *done = (uint8_t *)calloc((size_t)(N > 0 ? N : 1), 1);
    int64_t *members = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    int32_t *chunk = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    double *mean = (double *)malloc(sizeof(double) * (size_t)(W > 0 ? W : 1));
    if (!done || !members || !chunk || !mean) { free(done); free(members); free(chunk); free(mean); return -2; }

    for (int64_t lead = 0; lead < N; ++lead) {
        if (done[lead] || (alive != NULL && alive[lead] == 0)) continue;
        /* everybody who takes part and carries lead's key */
        int64_t k = 0;
        for (int64_t j = lead; j < N; ++j) {
            if (done[j] || (alive != NULL && alive[j] == 0)) continue;
            int same = 1;
            for (int32_t q = 0; q < kd; ++q)
                if (keys[j * kd + q] != keys[lead * kd + q]) same = 0;
            if (same) { members[k++] = j; done[j] = 1; }
        }
        /* the random order of peers_t: insertion sort by (order_key, index) */
        for (int64_t a = 1; a < k; ++a) {
            int64_t m = members[a];
            uint64_t km = order_key(seed, t, m);
            int64_t b = a - 1;
            while (b >= 0) {
                uint64_t kb = order_key(seed, t, members[b]);
                if (kb < km || (kb == km && members[b] < m)) break;
                members[b + 1] = members[b];
                --b;
            }
            members[b + 1] = m;
        }
        /* consecutive groups of at most M: average, hand out chunk indices */
        for (int64_t g0 = 0; g0 < k; g0 += M) {
            int64_t g1 = g0 + M < k ? g0 + M : k;
            for (int64_t c = 0; c < W; ++c) mean[c] = 0.0;
            for (int64_t a = g0; a < g1; ++a)
                for (int64_t c = 0; c < W; ++c) mean[c] += X[members[a] * ld + c];
            for (int64_t c = 0; c < W; ++c) mean[c] = mean[c] / (double)(g1 - g0);
            for (int64_t a = g0; a < g1; ++a) {
                for (int64_t c = 0; c < W; ++c) X[members[a] * ld + c] = mean[c];
                chunk[members[a]] = (int32_t)(a - g0);
            }
        }
    }
    /* C_i := (C_i[1:], c_i) for the peers that took part */
    for (int64_t i = 0; i < N; ++i) {
        if (!done[i] || kd == 0) continue;
        for (int32_t q = 0; q + 1 < kd; ++q) keys[i * kd + q] = keys[i * kd + q + 1];
        keys[i * kd + kd - 1] = chunk[i];
    }
    free(done); free(members); free(chunk); free(mean);
    return 0;
}

/* ---- Moshpit SGD step (Alg. 2) ------------------------------------------ */

/*
 * Local part of an iteration of Alg. 2: every peer of P_{k+1} (alive != 0;
 * NULL = all) moves to theta_i - gamma * g_i.  G is row-major [N][ldg].
 */
int oracle_local_step(double *X, const double *G, int64_t N, int64_t W, int64_t ld, int64_t ldg, double gamma,
                      const uint8_t *alive)
{
    for (int64_t i = 0; i < N; ++i) {
        if (alive != NULL && alive[i] == 0) continue;
        for (int64_t c = 0; c < W; ++c) X[i * ld + c] = X[i * ld + c] - gamma * G[i * ldg + c];
    }
    return 0;
}

/*
 * Communication iteration of Alg. 2 with one Moshpit round:
 * theta_i <- average over i's round-t group of (theta_j - gamma * g_j), the
 * group being formed from the peers of P_{k+1}.
 */
int oracle_sgd_round(double *X, const double *G, int64_t N, int64_t W, int64_t ld, int64_t ldg, double gamma,
                     int32_t M, int32_t d, int64_t t, const uint8_t *alive)
{
    int rc = oracle_local_step(X, G, N, W, ld, ldg, gamma, alive);
    if (rc != 0) return rc;
    return oracle_round(X, N, W, ld, M, d, t, alive);
}

/* ---- several rounds ---------------------------------------------------- */

/*
 * Rounds t0..t0+rounds-1 with masks[r][N] (NULL = no failures).  When
 * dist_out != NULL it receives rounds+1 values: the distortion of the slab
 * before the first round and after each round.  quantize < 0 keeps fp64
 * state between rounds (the graded mode); 0 / 1 re-round the state to
 * binary32 / bfloat16 after every round (diagnostic mode).
 */
int oracle_run(double *X, int64_t N, int64_t W, int64_t ld, int32_t M, int32_t d,
               int64_t t0, int32_t rounds, const uint8_t *masks, int32_t quantize,
               double *dist_out)
{
    if (dist_out) dist_out[0] = oracle_dist_to_mean(X, N, W, ld);
    for (int32_t r = 0; r < rounds; ++r) {
        int rc = oracle_round(X, N, W, ld, M, d, t0 + r, masks ? masks + (int64_t)r * N : NULL);
        if (rc != 0) return rc;
        if (quantize >= 0) {
            rc = oracle_quantize(X, N, W, ld, quantize);
            if (rc != 0) return rc;
        }
        if (dist_out) dist_out[r + 1] = oracle_dist_to_mean(X, N, W, ld);
    }
    return 0;
}
