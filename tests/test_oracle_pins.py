"""Pins for the fp64 CPU oracle: checks against what the paper and plain
mathematics fix, never against the oracle's own formulas or the GPU path.

Each test names the mistake it is meant to catch.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import moshpit_oracle as orc


def read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


# --------------------------------------------------------------------------
# hand-computed cases (tests/golden)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["fig2_nine_peers.txt", "cube_eight_peers.txt"])
def test_hand_cases_full_grid(golden_dir, name):
    """Wrong axis order, wrong stride or a wrong divisor changes these tables."""
    g = read_golden(os.path.join(golden_dir, name))
    M, d = int(g["M"][0]), int(g["d"][0])
    X = np.array(g["x0"], dtype=np.float64).reshape(-1, 1)
    for t in range(d):
        if f"keys{t}" in g:
            assert orc.group_keys(len(X), M, d, t).tolist() == [int(v) for v in g[f"keys{t}"]]
        orc.round_(X, M, d, t)
        assert X[:, 0].tolist() == g[f"x{t + 1}"]


def test_paper_three_vector_example(golden_dir):
    """App. C.1 worked example (an empty grid vertex): a peer that is absent
    must neither contribute nor be overwritten, and a lone survivor keeps its
    value."""
    g = read_golden(os.path.join(golden_dir, "appC1_three_vectors.txt"))
    M, d = int(g["M"][0]), int(g["d"][0])
    alive = np.array(g["alive"], dtype=np.uint8)
    X = np.array(g["x0"], dtype=np.float64).reshape(-1, 1)
    assert orc.dist_to_mean(X) == g["dist"][0]
    for t in range(2):
        orc.round_(X, M, d, t, alive)
        assert X[:, 0].tolist() == g[f"x{t + 1}"]
        assert orc.dist_to_mean(X) == g["dist"][t + 1]
    # the symbolic statement of the paper, with theta_11, theta_21, theta_22 = x0[0], x0[1], x0[3]
    a, b, c = g["x0"][0], g["x0"][1], g["x0"][3]
    assert X[0, 0] == (a + b) / 2
    assert X[1, 0] == X[3, 0] == (a + b) / 4 + c / 2


# --------------------------------------------------------------------------
# P1: exact global mean after d rounds on a full grid (App. C.1 theorem)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("M,d", [(4, 2), (3, 3), (2, 5), (16, 2), (5, 1), (32, 2)])
def test_exact_mean_after_d_rounds(M, d):
    """Any mistake in coordinates (a repeated or skipped axis) leaves some peer
    short of the global mean; checked against numpy's column mean."""
    rng = np.random.default_rng(10 * M + d)
    N, P = M ** d, 7
    X0 = rng.normal(size=(N, P))
    X = X0.copy()
    dist = orc.run(X, M, d, 0, d, want_dist=True)
    want = X0.mean(axis=0)
    assert np.allclose(X, np.broadcast_to(want, X.shape), rtol=0, atol=1e-14)
    assert dist[-1] < 1e-26
    # one round short must NOT be there yet (d >= 2), whichever axis is left out
    if d >= 2:
        for start in range(d):
            Y = X0.copy()
            orc.run(Y, M, d, start, d - 1)
            assert np.abs(Y - want).max() > 1e-3


def test_any_d_consecutive_rounds_give_mean():
    """Axes cycle t mod d: rounds 5,6,7 on a d=3 grid are again a full sweep."""
    rng = np.random.default_rng(3)
    M, d = 3, 3
    X0 = rng.normal(size=(27, 3))
    X = X0.copy()
    orc.run(X, M, d, 5, 3)
    assert np.allclose(X, X0.mean(axis=0), atol=1e-14, rtol=0)


def test_partial_sweep_is_axis_mean():
    """After k < d rounds a peer holds the mean over the first k coordinates
    (recurrence of App. C.1), checked with numpy on the reshaped grid.
    Catches a digit order that is reversed (most-significant digit first)."""
    rng = np.random.default_rng(4)
    M, d, P = 4, 3, 2
    X0 = rng.normal(size=(M ** d, P))
    grid = X0.reshape(M, M, M, P)           # index [c2][c1][c0]: digit 0 is the fastest
    X = X0.copy()
    orc.round_(X, M, d, 0)
    want = np.broadcast_to(grid.mean(axis=2, keepdims=True), grid.shape).reshape(-1, P)
    assert np.allclose(X, want, atol=1e-15, rtol=0)
    orc.round_(X, M, d, 1)
    want = np.broadcast_to(grid.mean(axis=(1, 2), keepdims=True), grid.shape).reshape(-1, P)
    assert np.allclose(X, want, atol=1e-15, rtol=0)


# --------------------------------------------------------------------------
# brute force: the round as an explicit doubly-stochastic matrix
# --------------------------------------------------------------------------

def averaging_matrix(N, M, d, t, alive):
    """W[i][j] from first principles in Python: coordinates by divmod, group =
    equal coordinates except coordinate t mod d."""
    def coords(i):
        c = []
        for _ in range(d):
            i, r = divmod(i, M)
            c.append(r)
        return c
    a = t % d
    W = np.zeros((N, N))
    for i in range(N):
        if not alive[i]:
            W[i, i] = 1.0
            continue
        ci = coords(i)
        mates = [j for j in range(N) if alive[j]
                 and all(cj == cq for q, (cj, cq) in enumerate(zip(coords(j), ci)) if q != a)]
        for j in mates:
            W[i, j] = 1.0 / len(mates)
    return W


@pytest.mark.parametrize("M,d", [(2, 2), (3, 2), (2, 3)])
def test_all_masks_against_matrix_form(M, d):
    """Every one of the 2^N masks, every axis: X <- W X.  A dropped member, a
    divisor M instead of the live count, or a dead peer being overwritten all
    fail here."""
    N = M ** d
    rng = np.random.default_rng(N)
    X0 = rng.normal(size=(N, 3))
    for bits in itertools.product([0, 1], repeat=N):
        alive = np.array(bits, dtype=np.uint8)
        for t in range(d):
            W = averaging_matrix(N, M, d, t, alive)
            assert np.allclose(W.sum(axis=0), 1) and np.allclose(W.sum(axis=1), 1)
            X = X0.copy()
            orc.round_(X, M, d, t, alive)
            assert np.allclose(X, W @ X0, atol=1e-15, rtol=0)


# --------------------------------------------------------------------------
# invariants under arbitrary masks (proof sketch of Thm 3.1; App. C.3)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("M,d,p", [(4, 2, 0.3), (3, 3, 0.2), (8, 2, 0.05), (2, 4, 0.5)])
def test_sum_preserved_and_distortion_monotone(M, d, p):
    rng = np.random.default_rng(100 * M + d)
    N, P, R = M ** d, 5, 9
    X = rng.normal(size=(N, P)) + rng.uniform(-1, 1, size=(N, 1))
    total0 = X.sum(axis=0)
    masks = (rng.random((R, N)) >= p).astype(np.uint8)
    prev = orc.dist_to_mean(X)
    d0 = prev
    for r in range(R):
        gid = orc.group_ids(N, M, d, r)
        before = X.copy()
        orc.round_(X, M, d, r, masks[r])
        # the global sum never moves (first claim of the Thm 3.1 proof sketch)
        assert np.allclose(X.sum(axis=0), total0, rtol=0, atol=1e-12)
        # each group's live-member sum is preserved; dead rows are bit-identical
        for lead in np.unique(gid):
            live = (gid == lead) & (masks[r] == 1)
            assert np.allclose(X[live].sum(axis=0), before[live].sum(axis=0), rtol=0, atol=1e-12)
        dead = masks[r] == 0
        assert np.array_equal(X[dead], before[dead])
        cur = orc.dist_to_mean(X)
        assert cur <= prev + 1e-12 * d0        # distortion never grows (Jensen)
        prev = cur
        # convex hull never expands (App. C.2)
        assert X.max() <= before.max() + 1e-15 and X.min() >= before.min() - 1e-15


def test_dist_to_mean_is_numpy_definition():
    rng = np.random.default_rng(5)
    X = rng.normal(size=(27, 11)) * 3 + 1
    want = ((X - X.mean(axis=0)) ** 2).sum() / X.shape[0]
    assert abs(orc.dist_to_mean(X) - want) <= 1e-13 * want
    # a strided column slab view gives that slab's share
    part = orc.dist_to_mean(X[:, 2:6])
    want = ((X[:, 2:6] - X[:, 2:6].mean(axis=0)) ** 2).sum() / X.shape[0]
    assert abs(part - want) <= 1e-13 * want


def test_special_masks():
    """All dead, one survivor per group, one whole group alive."""
    rng = np.random.default_rng(6)
    M, d = 4, 2
    X0 = rng.normal(size=(16, 4))
    X = X0.copy()
    orc.round_(X, M, d, 0, np.zeros(16, np.uint8))
    assert np.array_equal(X, X0)
    one = np.zeros(16, np.uint8)
    one[[1, 6, 8, 15]] = 1                       # one peer in each round-0 group
    orc.round_(X, M, d, 0, one)
    assert np.array_equal(X, X0)
    grp = np.zeros(16, np.uint8)
    grp[4:8] = 1                                 # round-0 group of peers 4..7
    orc.round_(X, M, d, 0, grp)
    assert np.array_equal(X[:4], X0[:4]) and np.array_equal(X[8:], X0[8:])
    assert np.allclose(X[4:8], X0[4:8].mean(axis=0), atol=1e-15, rtol=0)
    # the same mask in round 1 puts each of them alone in its group
    Y = X0.copy()
    orc.round_(Y, M, d, 1, grp)
    assert np.array_equal(Y, X0)


def test_linearity_and_column_independence():
    rng = np.random.default_rng(7)
    M, d, N = 3, 2, 9
    X0 = rng.normal(size=(N, 6))
    masks = (rng.random((4, N)) > 0.3).astype(np.uint8)
    A = X0.copy()
    orc.run(A, M, d, 0, 4, masks)
    perm = rng.permutation(6)
    B = X0[:, perm].copy()
    orc.run(B, M, d, 0, 4, masks)
    assert np.array_equal(B, A[:, perm])
    C = X0 * 8.0
    orc.run(C, M, d, 0, 4, masks)
    assert np.array_equal(C, A * 8.0)
    # slabs + threads give the same numbers as one call
    D = X0.copy()
    dist_a = orc.run(X0.copy(), M, d, 0, 4, masks, want_dist=True)
    dist_d = orc.run(D, M, d, 0, 4, masks, want_dist=True, threads=3, slab=2)
    assert np.array_equal(D, A)
    assert np.allclose(dist_a, dist_d, rtol=1e-14)


# --------------------------------------------------------------------------
# P5: closed form of the expected distortion on a full grid
# --------------------------------------------------------------------------

def test_expected_distortion_closed_form():
    """iid unit-variance entries: after k <= d rounds every peer holds a mean of
    M^k values, so E[dist_k]/P = M^-k - M^-d (k = 0: 1 - 1/N).  A wrong
    normalisation of the distortion (by N*P, by N-1, or by the live count) is
    off by far more than the 2 % allowed here."""
    rng = np.random.default_rng(8)
    M, d, P = 4, 2, 65536
    X = rng.normal(size=(16, P))
    dist = orc.run(X, M, d, 0, 2, want_dist=True)
    assert abs(dist[0] / P - (1 - 1 / 16)) < 0.02 * (1 - 1 / 16)
    assert abs(dist[1] / P - (1 / 4 - 1 / 16)) < 0.02 * (1 / 4 - 1 / 16)
    assert dist[2] / P < 1e-28


# --------------------------------------------------------------------------
# Table 4 of the paper: all sixteen Moshpit entries (32x32 grid)
# --------------------------------------------------------------------------

def rounds_to_error(n, p, seed, thresholds=(1e-9, 1e-4), max_rounds=50):
    """One restart of the paper's averaging experiment (Sec. 4.1): n peers sit
    on a uniformly random subset of the 32x32 grid's vertices (the other
    vertices stay empty for the whole run), hold scalar N(0,1) values, fail
    independently per round with probability p and return in the next round;
    the error is the average squared difference to the mean over the n peers."""
    rng = np.random.default_rng(seed)
    present = np.zeros(1024, dtype=np.uint8)
    present[rng.choice(1024, size=n, replace=False)] = 1
    X = rng.normal(size=(1024, 1))
    masks = orc.schedule_masks(1, p, seed, 0, 1024, 0, max_rounds)
    hit = [None] * len(thresholds)
    for t in range(max_rounds + 1):
        dist = orc.dist_to_mean_subset(X, present)
        for k, th in enumerate(thresholds):
            if hit[k] is None and dist <= th:
                hit[k] = t
        if all(h is not None for h in hit) or t == max_rounds:
            break
        orc.round_(X, 32, 2, t, present & masks[t])
    return [h if h is not None else max_rounds for h in hit]


def test_table4_moshpit_column(golden_dir):
    """The oracle's semantics (static grid, axes cycling, survivors average, a
    failed peer keeps its stale value and stays in the metric, empty vertices
    never take part) reproduce every Moshpit entry of Table 4.  N = 1024,
    p = 0 is exact; the others are means over 100 restarts and must land within
    0.4 round of the printed value (the paper prints one decimal; the standard
    error of such a mean is about 0.1)."""
    rows = np.loadtxt(os.path.join(golden_dir, "table4_moshpit.txt"), comments="#")
    assert len(rows) == 16
    for n, p, want9, want4 in rows:
        got = np.array([rounds_to_error(int(n), p, 7000 + s) for s in range(100)], dtype=float)
        m9, m4 = got[:, 0].mean(), got[:, 1].mean()
        if n == 1024 and p == 0:
            assert (m9, m4) == (2.0, 2.0)
        else:
            assert abs(m9 - want9) <= 0.4, (n, p, m9, want9)
            assert abs(m4 - want4) <= 0.4, (n, p, m4, want4)


def test_dist_subset_is_numpy_definition():
    rng = np.random.default_rng(12)
    X = rng.normal(size=(30, 5)) + 2
    present = (rng.random(30) < 0.6).astype(np.uint8)
    sub = X[present == 1]
    want = ((sub - sub.mean(axis=0)) ** 2).sum() / len(sub)
    assert abs(orc.dist_to_mean_subset(X, present) - want) <= 1e-13 * want
    assert orc.dist_to_mean_subset(X, None) == orc.dist_to_mean(X)
    assert orc.dist_to_mean_subset(X, np.zeros(30, np.uint8)) == 0.0


# --------------------------------------------------------------------------
# Alg. 1 with chunk-index keys
# --------------------------------------------------------------------------

@pytest.mark.parametrize("M,d", [(4, 2), (3, 3), (2, 4), (8, 2), (5, 1)])
def test_dynamic_keys_exact_mean_without_failures(M, d):
    """Full grid, nobody fails: whatever the random orders, every group has
    exactly M members, peers that just averaged never meet again in the next
    round (Sec. 3.1), and after d rounds every peer holds the global mean
    (equivalence with the torus all-reduce, App. C.1)."""
    N = M ** d
    rng = np.random.default_rng(7 * M + d)
    for seed in range(5):
        X0 = rng.normal(size=(N, 3))
        X = X0.copy()
        keys = orc.dynamic_init(N, M, d)
        for t in range(d):
            before_keys = keys.copy()
            tuples = [tuple(r) for r in before_keys]
            sizes = {k: tuples.count(k) for k in set(tuples)}
            assert set(sizes.values()) == {M}
            orc.dynamic_round(X, M, d, keys, seed, t)
            if d >= 2:
                # members of one group received the chunk indices 0..M-1
                for k in set(tuples):
                    got = sorted(keys[i, -1] for i in range(N) if tuples[i] == k)
                    assert got == list(range(M))
                assert np.array_equal(keys[:, :-1], before_keys[:, 1:])
        assert np.allclose(X, X0.mean(axis=0), atol=1e-14, rtol=0)


def test_dynamic_keys_first_round_is_the_static_grid():
    """With the initial keys of Eq. 2 the first round groups M consecutive
    peers: same values as the static grid's round 0."""
    rng = np.random.default_rng(41)
    M, d, N = 4, 3, 64
    X0 = rng.normal(size=(N, 2))
    alive = (rng.random(N) > 0.2).astype(np.uint8)
    A, B = X0.copy(), X0.copy()
    orc.round_(A, M, d, 0, alive)
    orc.dynamic_round(B, M, d, orc.dynamic_init(N, M, d), 3, 0, alive)
    assert np.allclose(A, B, atol=1e-15, rtol=0)


def test_dynamic_keys_with_failures():
    """Failures: sums preserved, distortion monotone, absent peers keep vector
    and key, groups never exceed M, chunk indices stay below M; first
    principles in Python for the grouping of one round."""
    rng = np.random.default_rng(42)
    M, d, N = 4, 3, 64
    X = rng.normal(size=(N, 3))
    total = X.sum(axis=0)
    keys = orc.dynamic_init(N, M, d)
    masks = orc.schedule_masks(1, 0.25, 9, 0, N, 0, 12)
    prev = orc.dist_to_mean(X)
    for t in range(12):
        bk, bx = keys.copy(), X.copy()
        orc.dynamic_round(X, M, d, keys, 17, t, masks[t])
        dead = masks[t] == 0
        assert np.array_equal(X[dead], bx[dead]) and np.array_equal(keys[dead], bk[dead])
        assert keys.min() >= 0 and keys.max() < M
        assert np.allclose(X.sum(axis=0), total, atol=1e-12, rtol=0)
        cur = orc.dist_to_mean(X)
        assert cur <= prev + 1e-13
        prev = cur
        # python model of this round
        order = {i: (py_mix(py_mix((17 + 0xD1B54A32D192ED03 * (t + 1)) & MASK64) ^ i), i) for i in range(N)}
        groups = {}
        for i in range(N):
            if masks[t][i]:
                groups.setdefault(tuple(bk[i]), []).append(i)
        for members in groups.values():
            members.sort(key=lambda i: order[i])
            for g0 in range(0, len(members), M):
                grp = members[g0:g0 + M]
                assert np.allclose(X[grp], bx[grp].mean(axis=0), atol=1e-15, rtol=0)
                assert [keys[i, -1] for i in grp] == list(range(len(grp)))
                assert all(tuple(keys[i, :-1]) == tuple(bk[i, 1:]) for i in grp)


def test_dynamic_keys_table4_full_grid():
    """N = 1024 on the 32x32 grid with per-round failures.  Table 4 is
    reproduced by the static grid (test above), so this is only a sanity
    bracket: the chunk-index form of Alg. 1, where a returning peer carries a
    stale key, must converge within one round of the printed 3.4/5.4/5.9
    (to 1e-9) and 2.2/2.9/3.0 (to 1e-4)."""
    want = {0.001: (3.4, 2.2), 0.005: (5.4, 2.9), 0.01: (5.9, 3.0)}
    for p, (w9, w4) in want.items():
        res = []
        for s in range(60):
            rng = np.random.default_rng(300 + s)
            X = rng.normal(size=(1024, 1))
            keys = orc.dynamic_init(1024, 32, 2)
            masks = orc.schedule_masks(1, p, 400 + s, 0, 1024, 0, 30)
            r9 = r4 = None
            for t in range(31):
                dist = orc.dist_to_mean(X)
                if r4 is None and dist <= 1e-4:
                    r4 = t
                if dist <= 1e-9:
                    r9 = t
                    break
                orc.dynamic_round(X, 32, 2, keys, 500 + s, t, masks[t])
            res.append((r9 if r9 is not None else 30, r4))
        m9, m4 = np.mean([r[0] for r in res]), np.mean([r[1] for r in res])
        assert abs(m9 - w9) <= 1.0 and abs(m4 - w4) <= 1.0, (p, m9, m4)


# --------------------------------------------------------------------------
# Moshpit SGD step (Alg. 2)
# --------------------------------------------------------------------------

def test_sgd_round_matrix_form():
    """X' = W (X - gamma * A G) with W the averaging matrix and A = diag(alive):
    a wrong sign of gamma, a gradient applied to an absent peer or applied after
    the averaging all change the result."""
    rng = np.random.default_rng(31)
    M, d, N = 3, 2, 9
    X0, G = rng.normal(size=(N, 4)), rng.normal(size=(N, 4))
    for trial in range(20):
        alive = (rng.random(N) > 0.3).astype(np.uint8)
        t, gamma = int(rng.integers(0, 4)), float(rng.uniform(0.01, 0.5))
        W = averaging_matrix(N, M, d, t, alive)
        want = W @ (X0 - gamma * alive[:, None] * G)
        X = X0.copy()
        orc.sgd_round(X, G, gamma, M, d, t, alive)
        assert np.allclose(X, want, atol=1e-14, rtol=0)
        Y = X0.copy()
        orc.sgd_round(Y, G, 0.0, M, d, t, alive)
        Z = X0.copy()
        orc.round_(Z, M, d, t, alive)
        assert np.array_equal(Y, Z)
        L = X0.copy()
        orc.local_step(L, G, gamma, alive)
        assert np.allclose(L, X0 - gamma * alive[:, None] * G, atol=1e-15, rtol=0)


def test_sgd_quadratic_closed_form():
    """Alg. 2 on f_i(theta) = 1/2 ||theta - theta*||^2 with exact gradients and
    all peers present: local steps and group averages both commute with the
    mean over peers, so mean_K = theta* + (1 - gamma)^K (mean_0 - theta*), and
    after a full sweep of d averaging iterations all peers agree."""
    rng = np.random.default_rng(32)
    M, d, N, P = 4, 2, 16, 5
    X = rng.normal(size=(N, P)) * 3
    star = rng.normal(size=P)
    mean0 = X.mean(axis=0)
    gamma, tau, t = 0.1, 3, 0
    for k in range(12):
        G = X - star
        if (k + 1) % tau == 0:
            orc.sgd_round(X, G, gamma, M, d, t)
            t += 1
        else:
            orc.local_step(X, G, gamma)
        want = star + (1 - gamma) ** (k + 1) * (mean0 - star)
        assert np.allclose(X.mean(axis=0), want, atol=1e-13, rtol=0)
    # four averaging iterations = two sweeps; peers drifted apart only by the (identical) local map
    assert np.abs(X - X.mean(axis=0)).max() < 1e-13


# --------------------------------------------------------------------------
# group-skip failure behaviour (Sec. 3.1)
# --------------------------------------------------------------------------

def test_skip_filter_all_masks():
    """From first principles in Python: a peer takes part iff nobody in its
    group failed.  All 2^N masks on 2x2, 3x3 and 2x2x2 grids, every axis."""
    for M, d in ((2, 2), (3, 2), (2, 3)):
        N = M ** d
        for bits in itertools.product([0, 1], repeat=N):
            alive = np.array(bits, dtype=np.uint8)
            for t in range(d):
                a = t % d
                want = np.zeros(N, dtype=np.uint8)
                for i in range(N):
                    mates = [j for j in range(N)
                             if all((j // M ** q) % M == (i // M ** q) % M for q in range(d) if q != a)]
                    want[i] = int(all(alive[j] for j in mates))
                assert np.array_equal(orc.skip_filter(N, M, d, t, alive), want)


def test_skip_semantics_properties():
    """With group-skip every group either averages completely or not at all:
    the global sum is preserved, the distortion never grows, it converges no
    faster than the survivors-average behaviour, and without failures both
    behaviours coincide."""
    rng = np.random.default_rng(21)
    M, d, N = 8, 2, 64
    X0 = rng.normal(size=(N, 3))
    masks = orc.schedule_masks(1, 0.05, 5, 0, N, 0, 12)
    A, B = X0.copy(), X0.copy()
    prev = orc.dist_to_mean(B)
    for t in range(12):
        eff = orc.skip_filter(N, M, d, t, masks[t])
        assert (eff <= masks[t]).all()
        before = B.copy()
        orc.round_(A, M, d, t, masks[t])
        orc.round_(B, M, d, t, eff)
        gid = orc.group_ids(N, M, d, t)
        for lead in np.unique(gid):
            grp = gid == lead
            if masks[t][grp].all():
                assert np.allclose(B[grp], before[grp].mean(axis=0), atol=1e-15, rtol=0)
            else:
                assert np.array_equal(B[grp], before[grp])
        assert np.allclose(B.sum(axis=0), X0.sum(axis=0), atol=1e-12, rtol=0)
        cur = orc.dist_to_mean(B)
        assert cur <= prev + 1e-15
        prev = cur
    assert orc.dist_to_mean(B) >= orc.dist_to_mean(A)
    ones = np.ones(N, dtype=np.uint8)
    assert np.array_equal(orc.skip_filter(N, M, d, 1, ones), ones)


# --------------------------------------------------------------------------
# a returning peer takes the parameters of an up-to-date peer first
# (App. "Training with a dynamic number of peers")
# --------------------------------------------------------------------------

def test_refresh_hand_case():
    """Four peers; peer 1 was away and comes back, peer 3 leaves.  The only peers
    present in both rounds are 0 and 2, so peer 1 ends with the vector of one of
    them and nothing else moves."""
    prev = np.array([1, 0, 1, 1], dtype=np.uint8)
    cur = np.array([1, 1, 1, 0], dtype=np.uint8)
    X0 = np.array([[1.0, 10.0], [2.0, 20.0], [3.0, 30.0], [4.0, 40.0]])
    seen = set()
    for seed in range(40):
        donor = orc.refresh_donors(prev, cur, seed, 5)
        assert donor[0] == donor[2] == donor[3] == -1
        assert donor[1] in (0, 2)
        seen.add(int(donor[1]))
        X = X0.copy()
        orc.refresh(X, donor)
        assert np.array_equal(X[1], X0[donor[1]])
        assert np.array_equal(X[[0, 2, 3]], X0[[0, 2, 3]])
    assert seen == {0, 2}                       # both candidates are drawn
    # nobody present in both rounds: nobody to copy from
    assert (orc.refresh_donors(np.array([0, 0, 1], dtype=np.uint8), np.array([1, 1, 0], dtype=np.uint8), 1, 0) == -1).all()
    # nobody returns
    assert (orc.refresh_donors(cur, cur, 1, 0) == -1).all()


def test_refresh_donor_draw_matches_python_bigint_and_is_uniform():
    """The draw against Python integers (64-bit wrap-around, stream constant, the
    rank-th candidate in ascending order), then its statistics: donors are always
    peers present in both rounds, never returning peers, and uniform over the
    candidates."""
    rng = np.random.default_rng(8)
    N = 300
    prev = (rng.random(N) < 0.7).astype(np.uint8)
    cur = (rng.random(N) < 0.7).astype(np.uint8)
    cand = [j for j in range(N) if prev[j] and cur[j]]
    for t in (0, 3, 1000):
        donor = orc.refresh_donors(prev, cur, 99, t)
        for i in range(N):
            if cur[i] and not prev[i]:
                u = py_mix(py_mix((99 + 0xA0761D6478BD642F * (t + 1)) & MASK64) ^ i)
                assert donor[i] == cand[u % len(cand)]
            else:
                assert donor[i] == -1
    # uniformity: 20 candidates, many returning peers and rounds
    N = 4000
    prev = np.zeros(N, dtype=np.uint8); prev[:20] = 1
    cur = np.ones(N, dtype=np.uint8)
    counts = np.zeros(20)
    for t in range(5):
        donor = orc.refresh_donors(prev, cur, 7, t)
        assert (donor[:20] == -1).all() and donor[20:].min() >= 0 and donor[20:].max() < 20
        counts += np.bincount(donor[20:], minlength=20)
    n = counts.sum()
    chi2 = ((counts - n / 20) ** 2 / (n / 20)).sum()
    assert chi2 < 50.0                           # 19 degrees of freedom: P(chi2 > 50) ~ 1e-4
    # different rounds give different draws
    assert not np.array_equal(orc.refresh_donors(prev, cur, 7, 0), orc.refresh_donors(prev, cur, 7, 1))


def test_refresh_effect_on_a_run():
    """What the step is for.  (a) Once the up-to-date peers agree, a returning peer
    that refreshes agrees with them at once, while one that does not drags the swarm
    back: the paper's reason for the step.  (b) Refreshing breaks the conservation of
    the global sum by exactly the sum of (donor - stale) over the returning peers.
    (c) On a die-and-rejoin schedule the distortion over the peers present at the end
    is smaller with the step than without."""
    rng = np.random.default_rng(31)
    M, d, N, W = 4, 2, 16, 5
    # (a) everybody but peer 5 averages to consensus; peer 5 was away the whole time
    X = rng.normal(size=(N, W))
    away = np.ones(N, dtype=np.uint8); away[5] = 0
    T = 80                                      # with a peer missing the rest converge geometrically
    for t in range(T):
        orc.round_(X, M, d, t, away)
    consensus = X[0].copy()
    assert np.allclose(X[away == 1], consensus, atol=1e-13, rtol=0)
    assert not np.allclose(X[5], consensus, atol=1e-3)
    back = np.ones(N, dtype=np.uint8)
    A, B = X.copy(), X.copy()
    donor = orc.refresh_donors(away, back, 3, T)
    assert donor[5] >= 0 and (np.delete(donor, 5) == -1).all()
    orc.refresh(A, donor)
    assert np.allclose(A, consensus, atol=1e-13, rtol=0)          # with the step: consensus kept
    orc.round_(A, M, d, T, back)
    orc.round_(B, M, d, T, back)                                   # without: the stale vector leaks in
    assert orc.dist_to_mean(A) < 1e-24 < 1e-6 < orc.dist_to_mean(B)
    # (b)
    X = rng.normal(size=(N, W))
    prev = (rng.random(N) < 0.6).astype(np.uint8)
    cur = (rng.random(N) < 0.8).astype(np.uint8)
    donor = orc.refresh_donors(prev, cur, 11, 4)
    Y = X.copy()
    orc.refresh(Y, donor)
    ret = np.flatnonzero(donor >= 0)
    assert len(ret) > 0
    assert np.allclose(Y.sum(axis=0) - X.sum(axis=0), (X[donor[ret]] - X[ret]).sum(axis=0), atol=1e-12, rtol=0)
    # (c)
    M, d, N = 8, 2, 64
    gain = []
    for seed in range(12):
        X0 = rng.normal(size=(N, 8)) + rng.normal(size=(N, 1))
        masks = orc.schedule_masks(2, 0.15, 100 + seed, 2, N, 0, 10)
        A, B = X0.copy(), X0.copy()
        for t in range(10):
            if t > 0:
                orc.refresh(A, orc.refresh_donors(masks[t - 1], masks[t], seed, t))
            orc.round_(A, M, d, t, masks[t])
            orc.round_(B, M, d, t, masks[t])
        gain.append(orc.dist_to_mean_subset(B, masks[-1]) / orc.dist_to_mean_subset(A, masks[-1]))
    assert np.median(gain) > 2.0 and min(gain) > 0.8


# --------------------------------------------------------------------------
# averaging in random groups: the exact contraction rate of Thm 3.2
# --------------------------------------------------------------------------

def test_random_groups_exact_rate_by_enumeration():
    """Thm 3.2 states E[dist after one iteration] = ((r-1)/N + r/N^2) * dist
    before, for a uniformly random permutation cut into r groups.  Its proof
    takes the probability that two given peers share group i as M_i(M_i-1)/N^2;
    for a permutation it is M_i(M_i-1)/(N(N-1)), which turns the rate into
    (r-1)/(N-1) exactly.  The two agree to O(1/N^2) (0.030304 vs 0.030303 for
    N = 1024, r = 32).  Enumerating all N! permutations for tiny N and feeding
    each to the oracle's grouped round must give the exact rate."""
    for N, gs, r in ((4, 2, 2), (5, 2, 3), (6, 3, 2), (6, 2, 3)):
        rng = np.random.default_rng(N)
        X0 = rng.normal(size=(N, 2)) + 1.0
        d0 = orc.dist_to_mean(X0)
        acc, cnt = 0.0, 0
        for perm in itertools.permutations(range(N)):
            X = X0.copy()
            orc.grouped_round(X, perm, gs)
            acc += orc.dist_to_mean(X)
            cnt += 1
            assert np.allclose(X.sum(axis=0), X0.sum(axis=0), atol=1e-13, rtol=0)
        exact = (r - 1) / (N - 1)
        printed = (r - 1) / N + r / N ** 2
        assert abs(acc / cnt - exact * d0) <= 1e-12 * d0, (N, acc / cnt / d0, exact)
        assert abs(printed - exact) <= 1.0 / N ** 2 + 1e-15       # the printed rate is the same to O(1/N^2)


def test_random_groups_seeded_rate():
    """The seeded permutation behaves like a uniform one: the mean contraction
    over 1000 seeds matches the rate of Thm 3.2 for N = 64, r = 8 (printed
    0.11133, exact 0.11111) within 2 %; over T rounds the rate compounds."""
    N, gs, r = 64, 8, 8
    rng = np.random.default_rng(64)
    X0 = rng.normal(size=(N, 4))
    d0 = orc.dist_to_mean(X0)
    rate = (r - 1) / (N - 1)
    one, three = [], []
    for seed in range(1000):
        X = X0.copy()
        for t in range(3):
            orc.random_groups_round(X, seed, t, gs)
            if t == 0:
                one.append(orc.dist_to_mean(X) / d0)
        three.append(orc.dist_to_mean(X) / d0)
    assert abs(np.mean(one) - rate) <= 0.02 * rate
    assert abs(np.mean(three) - rate ** 3) <= 0.08 * rate ** 3


def test_random_permutation_is_a_permutation_and_matches_python():
    N = 300
    perm = orc.random_permutation(11, 5, N)
    assert sorted(perm.tolist()) == list(range(N))
    keys = [py_mix(py_mix((11 + 0xD1B54A32D192ED03 * 6) & MASK64) ^ i) for i in range(N)]
    assert perm.tolist() == sorted(range(N), key=lambda i: (keys[i], i))
    assert not np.array_equal(perm, orc.random_permutation(11, 6, N))
    # a grouped round with failures: the absent peers keep their rows, the others average
    rng = np.random.default_rng(3)
    X0 = rng.normal(size=(N, 3))
    alive = (rng.random(N) > 0.2).astype(np.uint8)
    X = X0.copy()
    orc.random_groups_round(X, 11, 5, 7, alive)
    assert np.array_equal(X[alive == 0], X0[alive == 0])
    for g0 in range(0, N, 7):
        members = [i for i in perm[g0:g0 + 7] if alive[i]]
        if members:
            assert np.allclose(X[members], X0[members].mean(axis=0), atol=1e-15, rtol=0)


# --------------------------------------------------------------------------
# variance bound with peers absent for the whole run (App. C.4)
# --------------------------------------------------------------------------

def m1(M, q):
    """E[min(1/xi, 1)], xi ~ Binom(M, q): the lemma's closed form."""
    return (1 - q) ** M + sum(((1 - q) ** (M - i) - (1 - q) ** M) / i for i in range(1, M + 1))


def m2(M, q):
    return (1 - q) ** M + sum(((1 - q) ** (M - i) - (1 - q) ** M) / i * sum(1 / j for j in range(i, M + 1))
                              for i in range(1, M + 1))


def test_variance_bound_absent_peers():
    """Peers present with probability q for the whole run, iid unit-variance
    inputs: the per-peer output variance after T = d rounds is at most
    M^(T-1) m1(M-1,q) m2(M-1,q)^(T-1).  The oracle is linear, so running it on
    the identity matrix yields the weights and sum_j W_ij^2 is the variance."""
    M, d, q = 6, 2, 0.8
    N = M ** d
    rng = np.random.default_rng(9)
    acc, cnt = 0.0, 0
    for _ in range(200):
        present = (rng.random(N) < q).astype(np.uint8)
        W = np.eye(N)
        orc.run(W, M, d, 0, d, np.tile(present, (d, 1)))
        var = (W ** 2).sum(axis=1)[present == 1]
        acc += var.sum()
        cnt += len(var)
    bound = M ** (d - 1) * m1(M - 1, q) * m2(M - 1, q) ** (d - 1)
    assert acc / cnt <= bound
    assert acc / cnt >= 1.0 / N            # can never beat the exact mean of N values


# --------------------------------------------------------------------------
# failure schedule generator (input recipe)
# --------------------------------------------------------------------------

MASK64 = (1 << 64) - 1


def py_mix(x):
    x ^= x >> 32
    x = (x * 0x9E3779B97F4A7C15) & MASK64
    x ^= x >> 29
    x = (x * 0x6A09E667F3BCC909) & MASK64
    x ^= x >> 32
    return x


def py_event(seed, s, i, p):
    u = py_mix(py_mix((seed + 0x9E3779B97F4A7C15 * (s + 1)) & MASK64) ^ i)
    return (u >> 40) < int(p * (1 << 24))


def test_schedule_iid_matches_python_bigint():
    """64-bit wrap-around and shift widths, against Python integers."""
    masks = orc.schedule_masks(1, 0.3, 77, 0, 50, 3, 6)
    for r in range(6):
        for i in range(50):
            assert masks[r, i] == (0 if py_event(77, 3 + r, i, 0.3) else 1)


def test_schedule_statistics():
    N, R = 4096, 50
    for p in (0.05, 0.2):
        masks = orc.schedule_masks(1, p, 2002, 0, N, 0, R)
        rate = 1.0 - masks.mean()
        assert abs(rate - p) < 4 * np.sqrt(p * (1 - p) / (N * R))
        assert not np.array_equal(masks[0], masks[1])
        # different seeds and different peers decorrelate
        other = orc.schedule_masks(1, p, 2003, 0, N, 0, R)
        both = ((masks == 0) & (other == 0)).mean()
        assert abs(both - p * p) < 5 * np.sqrt(p * p / (N * R))
    assert orc.schedule_masks(0, 0.5, 1, 0, 10, 0, 3).min() == 1
    assert orc.schedule_masks(1, 0.0, 1, 0, 100, 0, 3).min() == 1
    assert orc.schedule_masks(1, 1.0, 1, 0, 100, 0, 3).max() == 0


def test_schedule_rejoin_structure():
    """kind 2: every absence lasts exactly `down` rounds (unless cut by the end
    of the window), a returning peer draws again at once, the stationary dead
    fraction is down*p / (1 + (down-1)*p), and a window that starts later is
    the tail of the window that starts at 0."""
    N, R, p, down = 4096, 40, 0.1, 2
    masks = orc.schedule_masks(2, p, 2005, down, N, 0, R)
    dead = masks == 0
    for i in range(0, N, 37):
        s = 0
        while s < R:
            if dead[s, i]:
                run_len = 1
                while s + run_len < R and dead[s + run_len, i]:
                    run_len += 1
                if s + run_len < R:
                    assert run_len % down == 0        # back-to-back absences are whole multiples
                # the absence starts where the generator's event fires
                assert py_event(2005, s, i, p)
                s += run_len
            else:
                assert not py_event(2005, s, i, p)
                s += 1
    frac = dead[10:].mean()
    want = down * p / (1 + (down - 1) * p)
    assert abs(frac - want) < 0.01
    tail = orc.schedule_masks(2, p, 2005, down, N, 7, 12)
    assert np.array_equal(tail, masks[7:19])


# --------------------------------------------------------------------------
# storage rounding used by the diagnostic mode
# --------------------------------------------------------------------------

def test_quantize_matches_torch_rounding():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11)
    v = np.concatenate([rng.normal(size=5000) * 10.0 ** rng.integers(-6, 6, size=5000),
                        [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.0e-39, 65504.0]])
    A = v.reshape(-1, 1).copy()
    orc.quantize(A, 0)
    assert np.array_equal(A[:, 0], v.astype(np.float32).astype(np.float64))
    B = v.reshape(-1, 1).copy()
    orc.quantize(B, 1)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(B[:, 0], want)


def test_run_quantized_mode_hand_case():
    """The storage-quantised mode of a run, bfloat16, by hand on a 2x2 grid: every mean
    below falls exactly half way between two bfloat16 numbers, so round-to-nearest-even
    decides (a mode that truncates, rounds half away from zero or forgets to round
    between rounds gives other numbers).  Spacing of bfloat16 is 2^-7 in [1,2), 2^-6 in [2,4).
      round 0 (axis 0): (1, 1+2^-7) -> 1+2^-8 -> 1 (even);  (3+2^-6, 3+2^-5) -> 3+1.5*2^-6 -> 3+2^-5 (even)
      round 1 (axis 1): (1, 3+2^-5) -> 2+2^-6 exactly representable
    The unquantised run keeps 1+2^-8 and 3+1.5*2^-6 and ends on 2 + 2^-9 + 1.5*2^-7."""
    x0 = np.array([[1.0], [1.0 + 2.0 ** -7], [3.0 + 2.0 ** -6], [3.0 + 2.0 ** -5]])
    q = x0.copy()
    dist = orc.run(q, 2, 2, 0, 1, None, quantize_dtype=1, want_dist=True)
    assert q[:, 0].tolist() == [1.0, 1.0, 3.0 + 2.0 ** -5, 3.0 + 2.0 ** -5]
    m = 2.0 + 2.0 ** -6
    assert dist[1] == ((1 - m) ** 2 * 2 + (3 + 2.0 ** -5 - m) ** 2 * 2) / 4
    orc.run(q, 2, 2, 1, 1, None, quantize_dtype=1)
    assert q[:, 0].tolist() == [m] * 4
    full = x0.copy()
    orc.run(full, 2, 2, 0, 2, None)
    assert full[:, 0].tolist() == [2.0 + 2.0 ** -9 + 1.5 * 2.0 ** -7] * 4
    # binary32: the mean of 1 and 1+2^-23 is a tie that goes to the even neighbour, 1
    y = np.array([[1.0], [1.0 + 2.0 ** -23], [5.0], [5.0]])
    orc.run(y, 2, 2, 0, 1, None, quantize_dtype=0)
    assert y[:, 0].tolist() == [1.0, 1.0, 5.0, 5.0]


@pytest.mark.parametrize("dtype", [0, 1])
def test_run_quantized_mode_rounds_every_round(dtype):
    """After every round of a quantised run the state holds storage-type numbers only
    (checked with torch's conversion, not the oracle's), peers that sit a round out keep
    their bits, and the run equals the rounds taken one at a time with torch doing the
    rounding in between."""
    torch = pytest.importorskip("torch")
    tt = torch.float32 if dtype == 0 else torch.bfloat16
    M, d, W, rounds = 3, 2, 40, 5
    N = M ** d
    rng = np.random.default_rng(5 + dtype)
    X0 = torch.from_numpy(rng.normal(size=(N, W))).to(tt).to(torch.float64).numpy().copy()
    masks = (rng.random((rounds, N)) > 0.3).astype(np.uint8)
    A = X0.copy()
    dist = orc.run(A, M, d, 1, rounds, masks, quantize_dtype=dtype, want_dist=True)
    B = X0.copy()
    want_dist = [float(((B - B.mean(axis=0)) ** 2).sum() / N)]
    for r in range(rounds):
        before = B.copy()
        orc.round_(B, M, d, 1 + r, masks[r])
        B = torch.from_numpy(B).to(tt).to(torch.float64).numpy().copy()
        assert np.array_equal(B[masks[r] == 0], before[masks[r] == 0])
        want_dist.append(float(((B - B.mean(axis=0)) ** 2).sum() / N))
    assert np.array_equal(A, B)
    assert np.allclose(dist, want_dist, rtol=1e-12, atol=0)
    plain = X0.copy()
    orc.run(plain, M, d, 1, rounds, masks)
    assert not np.array_equal(plain, A), "the quantised mode must differ from the fp64 mode"
    assert np.abs(plain - A).max() <= (2.0 ** -22 if dtype == 0 else 2.0 ** -6) * np.abs(X0).max()
