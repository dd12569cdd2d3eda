"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle,
element by element on the same seeded inputs.

Small cases compare the whole state; the five full-size workloads compare a
sample of whole columns (columns never interact, so the oracle can compute any
column on its own) plus properties that hold at any size.
"""
import numpy as np
import pytest
import torch

from oracle import moshpit_oracle as orc
from paper_2103_03239_amd import binding, inputs
from parity_util import (ELEM_FACTOR, TOL, assert_dist_close, assert_state_close, dist_floor, sample_columns,
                         worst_element_ratio)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def sched_of(w):
    return binding.Schedule(kind=w.kind, p=w.p, seed=w.mask_seed, down_rounds=w.down)


def to_f64(X):
    return X.detach().to("cpu").to(torch.float64).numpy()


def say(msg):
    print(msg, flush=True)


# --------------------------------------------------------------------------
# integer work: keys and masks, bit-exact
# --------------------------------------------------------------------------

@pytest.mark.parametrize("M,d", [(4, 2), (16, 2), (4, 3), (32, 2), (16, 3), (2, 5), (3, 4), (64, 1), (7, 2)])
def test_group_keys_bit_exact(M, d):
    N = M ** d
    with binding.Moshpit(N, 8, M, d, binding.F32) as m:
        for t in range(2 * d + 1):
            say(f"keys M={M} d={d} t={t}")
            assert np.array_equal(m.group_keys(t), orc.group_keys(N, M, d, t))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_schedule_masks_bit_exact(cfg):
    w = inputs.CONFIGS[cfg]
    with binding.Moshpit(w.N, 8, w.M, w.d, w.dtype) as m:
        for t0, rounds in ((0, w.rounds), (5, 9), (0, 0)):
            say(f"masks {w.name} t0={t0} rounds={rounds}")
            got = m.schedule_mask(sched_of(w), t0, rounds)
            want = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, w.N, t0, rounds)
            assert np.array_equal(got, want)
        # p = 0 and p = 1 corner thresholds
        for p in (0.0, 1.0, 0.5):
            s = binding.Schedule(kind=binding.SCHED_IID, p=p, seed=9)
            assert np.array_equal(m.schedule_mask(s, 2, 3), orc.schedule_masks(1, p, 9, 0, w.N, 2, 3))


# --------------------------------------------------------------------------
# whole-state parity on small shapes
# --------------------------------------------------------------------------

SMALL = [
    # M, d, P, dtype, row_stride, offset_elems, p
    (4, 2, 65_536, 0, None, 0, 0.0),        # workload 1 itself
    (16, 2, 5_000, 0, None, 0, 0.05),       # several tiles + ragged last tile
    (4, 3, 9_999, 0, 10_000, 0, 0.1),       # P not a multiple of 4: element-wise tail
    (32, 2, 3_001, 0, 3_004, 0, 0.2),       # M = 32, padded stride
    (16, 3, 2_056, 1, None, 0, 0.1),        # bf16, 4096 peers
    (16, 2, 1_003, 1, 1_008, 0, 0.3),       # bf16 ragged tail, padded stride
    (3, 3, 777, 0, None, 0, 0.25),          # M not a power of two, unaligned rows (777*4 % 16 != 0)
    (2, 6, 1_030, 1, None, 0, 0.3),         # M = 2, bf16 unaligned rows (1030*2 % 16 != 0)
    (64, 1, 2_048, 0, None, 0, 0.1),        # one group of 64 (bit 63 of the live bitmap)
    (5, 2, 1, 0, None, 0, 0.2),             # a single column
    (8, 2, 4_096, 0, 4_100, 1, 0.1),        # base pointer not 16-byte aligned
    (7, 2, 20_000, 1, 20_000, 3, 0.15),     # bf16, base pointer 6 bytes off, M = 7
]


@pytest.mark.parametrize("M,d,P,dtype,stride,offset,p", SMALL)
def test_small_full_state(M, d, P, dtype, stride, offset, p):
    N = M ** d
    rounds = 2 * d + 1
    w = inputs.Workload(f"small-{M}-{d}-{P}", N, M, d, P, dtype, "peer_offset",
                        inputs.KIND_IID if p > 0 else inputs.KIND_NONE, p, 0, rounds, 42 + M + P, 4242 + P)
    say(f"case {w}")
    stride = P if stride is None else stride
    buf = torch.full((N * stride + offset + 64,), 512.0, dtype=w.torch_dtype, device=DEV)
    X = buf[offset: offset + N * stride].view(N, stride)[:, :P]
    X.copy_(inputs.make_state(w, DEV))
    ref = to_f64(X).copy()
    masks = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, N, 0, rounds)
    dist_ref = orc.run(ref, M, d, 0, rounds, masks, want_dist=True)

    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(X)
        dist, ms = m.run(0, rounds, sched_of(w), want_dist=True, want_times=True)
    assert_state_close(to_f64(X), ref, TOL[dtype], w.name)
    assert_dist_close(dist, dist_ref, TOL[dtype], dist_floor(P, dtype, 1.0), w.name)
    assert (ms >= 0).all()
    # padding and guard elements were never written
    whole = buf.to(torch.float32).cpu().numpy()
    assert (whole[:offset] == 512.0).all() and (whole[offset + N * stride:] == 512.0).all()
    if stride > P:
        pad = whole[offset: offset + N * stride].reshape(N, stride)[:, P:]
        assert (pad == 512.0).all()


@pytest.mark.parametrize("M,d,P,dtype,p", [(32, 2, 3_000, 0, 0.2), (16, 2, 5_000, 0, 0.05), (4, 3, 9_999, 0, 0.1),
                                            (3, 3, 777, 0, 0.25), (16, 3, 520, 1, 0.1), (7, 2, 2_000, 1, 0.15),
                                            (64, 1, 1_024, 0, 0.1), (2, 6, 1_030, 1, 0.3)])
def test_each_round_within_rounding_of_the_quantized_oracle(M, d, P, dtype, p):
    """Round by round, from the SAME stored input: the kernel's result against the
    oracle's fp64 mean rounded once to the storage type.  The only differences
    allowed are the kernel's binary32 summation (a tree of depth ceil(log2 M) within
    blocks of 16 and up to 3 more additions across blocks: at most 8 roundings, each
    <= 2^-24 of a partial sum, partial sums <= the sum of |x| over the group's
    participants) and one unit in the last place of the storage type where the two
    sums fall on different sides of a rounding boundary.  Rows that do not take part
    must not change at all.  This localises an error to a round, a group and a
    column, where the tolerance on whole runs cannot."""
    N = M ** d
    rounds = 2 * d
    w = inputs.Workload(f"ulp-{M}-{d}-{P}", N, M, d, P, dtype, "peer_offset", inputs.KIND_IID, p, 0, rounds,
                        4 + M + P, 40 + P)
    say(f"case {w}")
    X = inputs.make_state(w, DEV)
    masks = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, N, 0, rounds)
    ulp = 2.0 ** -23 if dtype == 0 else 2.0 ** -7          # spacing relative to the binade's lower end
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(X)
        for t in range(rounds):
            before = to_f64(X)
            want = before.copy()
            orc.round_(want, M, d, t, masks[t])
            orc.quantize(want, dtype)
            mean_abs = np.abs(before)
            orc.round_(mean_abs, M, d, t, masks[t])        # group mean of |x| for participants
            m.round(t, masks[t])
            got = to_f64(X)
            probe = np.random.default_rng(t).random((N, 1))
            moved = probe.copy()
            orc.round_(moved, M, d, t, masks[t])
            outside = (moved == probe)[:, 0]                # absent peers and lone survivors
            assert np.array_equal(got[outside], before[outside]), f"round {t}: a row outside the round changed"
            bound = 8 * 2.0 ** -24 * mean_abs + ulp * np.abs(want) + 1e-300
            bad = np.abs(got - want) > bound
            assert not bad.any(), (f"round {t}: {int(bad.sum())} elements off by more than the rounding bound; "
                                   f"first at {tuple(np.argwhere(bad)[0])}: got {got[bad][0]!r} want {want[bad][0]!r}")


def test_workload1_is_exact_global_mean():
    """Full grid, no failures, d rounds: every peer ends on the global mean
    (exact-average theorem, App. C.1); distortion follows M^-k - M^-d."""
    w = inputs.CONFIGS[1]
    X = inputs.make_state(w, DEV)
    X0 = to_f64(X)
    with binding.Moshpit(w.N, w.P, w.M, w.d, w.dtype) as m:
        m.bind_state(X)
        dist, _ = m.run(0, w.rounds, None, want_dist=True)
    want = X0.mean(axis=0)
    assert_state_close(to_f64(X), np.broadcast_to(want, X0.shape), TOL[0], w.name)
    assert abs(dist[0] / w.P - (1 - 1 / 16)) < 0.02
    assert abs(dist[1] / w.P - (1 / 4 - 1 / 16)) < 0.02 * (1 / 4 - 1 / 16)
    assert dist[2] <= dist_floor(w.P, 0, 1.0)


def test_round_entry_points_and_special_masks():
    """moshpit_round (host mask), moshpit_round_dev (device mask), explicit
    schedules; all-dead and one-survivor-per-group rounds change nothing."""
    M, d, P = 4, 2, 3000
    N = 16
    w = inputs.Workload("rounds", N, M, d, P, 0, "normal", 0, 0.0, 0, 0, 7, 7)
    X = inputs.make_state(w, DEV)
    X0 = X.clone()
    ref = to_f64(X).copy()
    rng = np.random.default_rng(0)
    with binding.Moshpit(N, P, M, d, 0) as m:
        m.bind_state(X)
        m.round(0, np.zeros(N, np.uint8))
        one = np.zeros(N, np.uint8)
        one[[1, 6, 8, 15]] = 1
        m.round(0, one)
        m.sync()
        assert torch.equal(X, X0)
        masks = (rng.random((5, N)) > 0.3).astype(np.uint8)
        for t in range(5):
            if t % 2 == 0:
                m.round(t, masks[t])
            else:
                m.round_dev(t, torch.from_numpy(masks[t]).to(DEV))
            orc.round_(ref, M, d, t, masks[t])
        m.round(5)                      # NULL mask: everybody
        orc.round_(ref, M, d, 5)
        m.sync()
        assert_state_close(to_f64(X), ref, 1e-6, "round entry points")
        # the same five rounds as one explicit schedule reproduce the same bits
        Y = X0.clone()
        m.bind_state(Y)
        m.run(0, 5, binding.Schedule(kind=binding.SCHED_EXPLICIT, explicit_masks=masks))
        m.round_dev(5, None)
        m.sync()
        assert torch.equal(Y, X)
        assert abs(m.dist_to_mean() - orc.dist_to_mean(ref)) <= 1e-6 * orc.dist_to_mean(ref) + dist_floor(P, 0, 1.0)


def test_errors_are_reported_not_crashed():
    with binding.Moshpit(16, 100, 4, 2, 0) as m:
        with pytest.raises(binding.MoshpitError):
            m.round(0)                                    # nothing bound
        X = torch.zeros(16, 100, device=DEV)
        m.bind_state(X)
        with pytest.raises(binding.MoshpitError):
            m.round(-1)
        with pytest.raises(binding.MoshpitError):
            m.run(0, 2, binding.Schedule(kind=binding.SCHED_IID, p=1.5))
        with pytest.raises(binding.MoshpitError):
            m.run(0, 2, binding.Schedule(kind=binding.SCHED_REJOIN, p=0.1, down_rounds=0))
        with pytest.raises(binding.MoshpitError):
            m.bind_raw(X.data_ptr(), 50)                  # stride < P
        with pytest.raises(binding.MoshpitError):
            m.set_tuning(3, 3)
        m.run(0, 0)                                       # zero rounds is a no-op
        m.sync()


@pytest.mark.parametrize("cols,unroll,nt,block,wpc,order", [
    (1, 4, 0, 64, 4, 0), (1, 8, 1, 64, 3, 1), (1, 16, 0, 128, 2, -1), (2, 2, 1, 256, 32, 1), (2, 4, 0, 64, 1, 0),
    (2, 8, 1, 128, 6, 1), (4, 2, 0, 256, 8, -1), (4, 4, 1, 64, 6, 1), (1, 8, 1, 256, 4, 0), (1, 8, 0, 0, 0, 1)])
def test_every_launch_shape(cols, unroll, nt, block, wpc, order):
    """All launch shapes of the averaging kernel meet the same parity bar."""
    for dtype, M, d, P in ((0, 16, 2, 6_001), (1, 4, 3, 9_000)):
        N = M ** d
        w = inputs.Workload("shape", N, M, d, P, dtype, "normal", 1, 0.2, 0, 5, 5, 6)
        say(f"shape cols={cols} unroll={unroll} nt={nt} block={block} wpc={wpc} order={order} dtype={dtype}")
        X = inputs.make_state(w, DEV, row_stride=P + (8 - P % 8) % 8)
        ref = to_f64(X).copy()
        masks = orc.schedule_masks(1, 0.2, 6, 0, N, 0, 5)
        orc.run(ref, M, d, 0, 5, masks)
        with binding.Moshpit(N, P, M, d, dtype) as m:
            m.bind_state(X)
            m.set_tuning(cols, unroll, nt, block, wpc, order)
            m.run(0, 5, sched_of(w))
            m.sync()
        assert_state_close(to_f64(X), ref, TOL[dtype], "launch shape")


# --------------------------------------------------------------------------
# the five workloads at full size
# --------------------------------------------------------------------------

@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_full_size_workload(cfg):
    """The quick check at full size: sampled columns and size-independent properties
    (test_full_size_full_state compares every element)."""
    w = inputs.CONFIGS[cfg]
    say(f"full-size {w.name}: generating {w.N}x{w.P}")
    X = inputs.make_state(w, DEV, row_stride=inputs.aligned_row_stride(w.P, w.dtype))     # the layout bench.py times
    cols = sample_columns(w.P, 1024 if w.N >= 1024 else 4096, seed=cfg)
    cols_dev = torch.from_numpy(cols).to(DEV)
    ref = to_f64(X.index_select(1, cols_dev)).copy()
    colsum0 = X.sum(dim=0, dtype=torch.float64)
    rms0 = float(np.sqrt((ref ** 2).mean()))

    masks_ref = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, w.N, 0, w.rounds)
    orc.run(ref, w.M, w.d, 0, w.rounds, masks_ref, threads=8, slab=128)

    with binding.Moshpit(w.N, w.P, w.M, w.d, w.dtype) as m:
        m.bind_state(X)
        assert np.array_equal(m.schedule_mask(sched_of(w), 0, w.rounds), masks_ref)
        say("  running")
        dist, ms = m.run(0, w.rounds, sched_of(w), want_dist=True, want_times=True)
        say(f"  round ms: {np.round(ms, 3).tolist()}")
        say(f"  dist/P  : {(dist / w.P).tolist()}")
    worst = assert_state_close(to_f64(X.index_select(1, cols_dev)), ref, TOL[w.dtype], w.name)
    say(f"  worst sampled row error {worst:.3e}")

    # properties that hold at any size
    # (a) the distortion never grows (Jensen; proof sketch of Thm 3.1)
    slack = TOL[w.dtype] * dist[0] + dist_floor(w.P, w.dtype, rms0)
    assert (np.diff(dist) <= slack).all(), dist
    # (b) every column sum is preserved by every round, whatever the masks
    colsum = X.sum(dim=0, dtype=torch.float64)
    scale = rms0 * np.sqrt(w.N)
    drift = float((colsum - colsum0).abs().max()) / scale
    say(f"  column-sum drift / (rms*sqrt(N)) = {drift:.3e}")
    assert drift <= (1e-5 if w.dtype == 0 else 0.05)
    # (c) the distortion of the sampled columns alone agrees with the oracle's
    got_sub = X.index_select(1, cols_dev).to(torch.float64)
    sub = float(((got_sub - got_sub.mean(dim=0)) ** 2).sum() / w.N)
    want_sub = orc.dist_to_mean(ref)
    assert abs(sub - want_sub) <= 10 * TOL[w.dtype] * want_sub + dist_floor(len(cols), w.dtype, rms0)
    if w.kind == 0:
        assert dist[-1] <= dist_floor(w.P, w.dtype, rms0)


def _slab_columns(N):
    """Columns per slab so that one slab of the fp64 reference is about 1 GiB."""
    return max(4096, (2 ** 27 // N) // 4096 * 4096)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_full_size_full_state(cfg):
    """EVERY element of the final state and the WHOLE distortion curve of the five workloads
    at full size, in the layout the benchmark times, against the oracle.  Columns never
    interact, so the state goes to the host in column slabs (about 1 GiB of fp64 each), the
    oracle runs all rounds on each slab and its per-round distortion partial sums add up to
    the curve.  Row errors are accumulated over the slabs; the element guard uses the rms of
    the row within the slab."""
    w = inputs.CONFIGS[cfg]
    tol = TOL[w.dtype]
    say(f"full-state {w.name}: generating {w.N}x{w.P}")
    X = inputs.make_state(w, DEV, row_stride=inputs.aligned_row_stride(w.P, w.dtype))
    X0 = X.clone()
    masks = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, w.N, 0, w.rounds)
    with binding.Moshpit(w.N, w.P, w.M, w.d, w.dtype) as m:
        m.bind_state(X)
        assert np.array_equal(m.schedule_mask(sched_of(w), 0, w.rounds), masks)
        dist, _ = m.run(0, w.rounds, sched_of(w), want_dist=True)
    say(f"  dist/P  : {(dist / w.P).tolist()}")
    slab = _slab_columns(w.N)
    err2 = torch.zeros(w.N, dtype=torch.float64)
    norm2 = torch.zeros(w.N, dtype=torch.float64)
    sum0 = 0.0
    dist_ref = np.zeros(w.rounds + 1)
    worst_el = 0.0
    for k, c0 in enumerate(range(0, w.P, slab)):
        c1 = min(w.P, c0 + slab)
        ref_t = X0[:, c0:c1].cpu().to(torch.float64)
        sum0 += float((ref_t ** 2).sum())
        ref = ref_t.numpy()
        dist_ref += orc.run(ref, w.M, w.d, 0, w.rounds, masks, want_dist=True, threads=16,
                            slab=max(256, (c1 - c0) // 64))
        got_t = X[:, c0:c1].cpu().to(torch.float64)
        diff = (got_t - ref_t).abs_()
        n2 = (ref_t ** 2).sum(dim=1)
        rms = (n2 / (c1 - c0)).sqrt_()
        ratio = float((diff / (ref_t.abs().add_(rms[:, None]).mul_(tol).add_(1e-300))).max())
        worst_el = max(worst_el, ratio)
        err2 += (diff ** 2).sum(dim=1)
        norm2 += n2
        if k % 8 == 0:
            say(f"  slab {k} columns {c0}..{c1}: worst element ratio so far {worst_el:.3f}")
        assert ratio <= ELEM_FACTOR[w.dtype], (f"{w.name}: element outside {ELEM_FACTOR[w.dtype]}*tol*(|x|+rms) in "
                                               f"columns {c0}..{c1}: ratio {ratio:.3f}")
    rel = (err2 / norm2).sqrt().numpy()
    say(f"  worst row error {rel.max():.3e}, worst element error {worst_el:.3f} tol*(|x|+rms)")
    assert rel.max() <= tol, f"{w.name}: worst row relative error {rel.max():.3e} (row {int(rel.argmax())})"
    rms0 = float(np.sqrt(sum0 / (w.N * w.P)))
    say(f"  oracle dist/P: {(dist_ref / w.P).tolist()}")
    assert_dist_close(dist, dist_ref, tol, dist_floor(w.P, w.dtype, rms0), w.name)
    if w.kind == 0:
        assert dist[-1] <= dist_floor(w.P, w.dtype, rms0)



def test_bf16_rounding_of_the_kernels_is_round_to_nearest_even_everywhere():
    """The conversion instruction the kernels round bfloat16 states with, against its
    integer definition, on all 2^32 binary32 inputs (the oracle's rounding is pinned to the
    same definition on the CPU)."""
    assert binding.check_bf16_rounding() == 0


# --------------------------------------------------------------------------
# fused multi-round passes
# --------------------------------------------------------------------------

FUSED = [
    # M, d, P, dtype, p, t0, rounds
    (4, 2, 65_536, 0, 0.0, 0, 2),        # workload 1: whole 4x4 grid in one tile
    (16, 2, 5_000, 0, 0.05, 0, 10),      # 256 rows, ragged last column tile, 5 sweeps in one pass
    (4, 3, 10_000, 0, 0.1, 0, 6),        # 64 rows, d = 3, whole grid
    (32, 2, 4_100, 0, 0.2, 0, 8),        # 1024 rows x 128-byte segments
    (32, 2, 4_100, 0, 0.2, 3, 5),        # start on the second axis, odd number of rounds
    (16, 3, 2_056, 1, 0.1, 0, 12),       # bf16, 4096 peers: planes of 256 rows, 2 rounds per pass
    (16, 3, 2_056, 1, 0.1, 2, 7),        # plane that wraps around (axes 2 and 0), leftover single round
    (16, 3, 1_000, 0, 0.3, 1, 2),        # fewer rounds than axes
    (3, 3, 780, 0, 0.25, 0, 9),          # M not a power of two
    (2, 6, 1_032, 1, 0.3, 4, 13),        # M = 2, six axes in one tile
    (64, 1, 2_048, 0, 0.1, 0, 3),        # one axis only: nothing to fuse, falls back to single rounds
    (8, 2, 12, 0, 0.2, 0, 4),            # rows narrower than a tile
    (7, 2, 20_000, 1, 0.15, 0, 4),
    (5, 4, 1_000, 0, 0.1, 0, 9),         # 625 rows: four axes only with one block per compute unit
    (2, 10, 520, 1, 0.2, 3, 12),         # 1024 rows of a 2^10 grid, bf16
    (10, 3, 300, 0, 0.1, 1, 7),          # 1000 rows, M not a power of two, two 16-position blocks unused
    (20, 2, 1_500, 0, 0.15, 0, 5),       # 400 rows, M = 20: lanes split two 16-position blocks
    (6, 3, 2_000, 1, 0.1, 2, 8),         # 216 rows
    (12, 2, 3_000, 0, 0.05, 0, 6),       # 144 rows, M = 12
    (64, 2, 200, 0, 0.1, 0, 4),          # 4096 rows of 64: does not fit, single rounds
]


@pytest.mark.parametrize("M,d,P,dtype,p,t0,rounds", FUSED)
def test_fused_equals_single_rounds_and_oracle(M, d, P, dtype, p, t0, rounds):
    N = M ** d
    w = inputs.Workload(f"fused-{M}-{d}-{P}", N, M, d, P, dtype, "peer_offset",
                        inputs.KIND_REJOIN if p > 0 else inputs.KIND_NONE, p, 2, rounds, 17 + P, 99 + M)
    say(f"case {w} t0={t0}")
    A = inputs.make_state(w, DEV)
    B = A.clone()
    ref = to_f64(A).copy()
    masks = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, N, t0, rounds)
    dist_ref = orc.run(ref, M, d, t0, rounds, masks, want_dist=True)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(A)
        dist_a, _ = m.run(t0, rounds, sched_of(w), want_dist=True)
        m.bind_state(B)
        dist_b, ms = m.run(t0, rounds, sched_of(w), want_dist=True, want_times=True, flags=binding.RUN_FUSED)
    assert torch.equal(A, B), "fused pass differs from single rounds"
    assert_state_close(to_f64(B), ref, TOL[dtype], w.name)
    have = ~np.isnan(dist_b)
    assert have[0] and have[-1]
    assert np.array_equal(dist_b[have], dist_a[have])
    assert_dist_close(dist_b[have], dist_ref[have], TOL[dtype], dist_floor(P, dtype, 1.0), w.name)
    assert (ms >= 0).all()
    if d >= 2 and rounds >= 2 and M ** 2 * 128 <= 150_000 and P * (2 if dtype else 4) % 16 == 0:
        assert (~have).any(), "expected at least one fused pass"


@pytest.mark.parametrize("M,d,dtype", [(6, 2, 0), (12, 2, 0), (20, 2, 0), (10, 2, 1)])
def test_fused_division_edge_values(M, d, dtype):
    """Sums that are tiny (quotient subnormal), zero, huge or infinite: the fused kernel
    must give the bits of the single-round kernel, NaN for NaN."""
    N, P, rounds = M ** d, 2_048, 4
    say(f"fused division edge values M={M} d={d} dtype={dtype}")
    g = torch.Generator(device="cpu").manual_seed(4242 + M)
    kind = torch.randint(0, 6, (1, P), generator=g).expand(N, P)       # one kind of value per column
    x = torch.randn(N, P, generator=g, dtype=torch.float32)
    scale = torch.ones(N, P)
    scale[kind == 0] = 2.0 ** -130      # subnormal inputs
    scale[kind == 1] = 2.0 ** -122      # normal inputs whose mean is subnormal for larger counts
    scale[kind == 2] = 2.0 ** 120       # huge, finite sums
    x = x * scale
    x[kind == 3] = 0.0
    x[(kind == 4) & (torch.rand(N, P, generator=g) < 0.01)] = float("inf")
    A = x.to(torch.bfloat16 if dtype else torch.float32).to(DEV).contiguous()
    B = A.clone()
    sched = binding.Schedule(kind=inputs.KIND_IID, p=0.2, seed=77 + M)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(A)
        m.run(0, rounds, sched)
        m.bind_state(B)
        m.run(0, rounds, sched, flags=binding.RUN_FUSED)      # whole grid in one tile: one fused pass
    bits = torch.int16 if dtype else torch.int32
    same = (A.view(bits) == B.view(bits)) | (torch.isnan(A) & torch.isnan(B))
    assert bool(same.all()), f"{int((~same).sum())} elements differ in bits"
    tiny = (A != 0) & (A.abs().float() < 2.0 ** -126)
    assert bool(tiny.any()) and bool(torch.isinf(A).any() | torch.isnan(A).any())


@pytest.mark.parametrize("fused", [0, 1])
def test_run_can_be_continued(fused):
    """A run split in two (the second part starting at the round where the first stopped) gives
    the bits of the run in one piece, also when a peer's absence spans the cut (die-and-rejoin
    schedule) and when the cut falls inside what would have been one fused pass."""
    M, d, P, rounds, cut = 16, 2, 3_000, 9, 4
    N = M ** d
    w = inputs.Workload("continued", N, M, d, P, 0, "peer_offset", inputs.KIND_REJOIN, 0.15, 2, rounds, 81, 82)
    say(f"continued run fused={fused}")
    A = inputs.make_state(w, DEV)
    B = A.clone()
    flags = binding.RUN_FUSED if fused else 0
    with binding.Moshpit(N, P, M, d, 0) as m:
        m.bind_state(A)
        da, _ = m.run(0, rounds, sched_of(w), want_dist=True, flags=flags)
        m.bind_state(B)
        d1, _ = m.run(0, cut, sched_of(w), want_dist=True, flags=flags)
        d2, _ = m.run(cut, rounds - cut, sched_of(w), want_dist=True, flags=flags)
        # zero rounds: nothing moves, one distortion value
        before = B.clone()
        d0, _ = m.run(rounds, 0, sched_of(w), want_dist=True, flags=flags)
        m.sync()
    assert torch.equal(A, B) and torch.equal(B, before)
    assert d0.shape == (1,) and d0[0] == d2[-1] == da[-1]
    assert d1[0] == da[0] and d1[-1] == d2[0]


def test_fused_with_explicit_masks_and_dead_rounds():
    """Explicit schedules through the fused path: a round in which nobody is present, a round
    with one survivor per group and a peer absent throughout (its row is never touched)."""
    M, d, P, rounds = 8, 2, 2_048, 6
    N = M ** d
    w = inputs.Workload("explicit", N, M, d, P, 0, "normal", 0, 0.0, 0, rounds, 91, 92)
    say("fused explicit masks")
    masks = orc.schedule_masks(1, 0.2, 92, 0, N, 0, rounds)
    masks[2, :] = 0                                   # nobody
    masks[3, :] = 0
    masks[3, ::M] = 1                                 # round 3 averages along axis 1: peers 0, 8, ... share a group
    masks[4, :] = 0
    masks[4, :M] = 1                                  # round 4 (axis 0): one whole group, the rest absent
    masks[:, 13] = 0                                  # peer 13 never takes part
    A = inputs.make_state(w, DEV)
    B = A.clone()
    ref = to_f64(A).copy()
    orc.run(ref, M, d, 0, rounds, masks)
    sched = binding.Schedule(kind=binding.SCHED_EXPLICIT, explicit_masks=masks)
    with binding.Moshpit(N, P, M, d, 0) as m:
        m.bind_state(A)
        m.run(0, rounds, sched)
        m.bind_state(B)
        dist, _ = m.run(0, rounds, sched, want_dist=True, flags=binding.RUN_FUSED)
    assert np.isnan(dist[1:-1]).all(), "expected one fused pass"
    assert torch.equal(A, B)
    assert_state_close(to_f64(B), ref, TOL[0], w.name)
    assert np.array_equal(to_f64(B)[13], to_f64(inputs.make_state(w, DEV))[13])


def _random_cases(count, seed):
    """Seeded random shapes: grid, width, type, row padding, failure rate, first round, rounds."""
    rng = np.random.default_rng(seed)
    grids = [(2, 3), (2, 7), (3, 2), (3, 4), (4, 2), (4, 4), (5, 2), (5, 3), (6, 2), (8, 2), (8, 3), (9, 2), (11, 2),
             (13, 2), (16, 2), (17, 2), (24, 2), (31, 2), (32, 2), (33, 2), (2, 12), (4, 5), (64, 1), (10, 1)]
    cases = []
    for k in range(count):
        M, d = grids[int(rng.integers(len(grids)))]
        dtype = int(rng.integers(2))
        per16 = 4 if dtype == 0 else 8
        P = int(rng.integers(1, 700))
        if rng.random() < 0.7:
            P = max(per16, P // per16 * per16)            # rows that the fused path accepts
        pad = int(rng.choice([0, 0, per16, 3]))
        p = float(rng.choice([0.0, 0.05, 0.3, 0.7]))
        t0 = int(rng.integers(0, 7))
        rounds = int(rng.integers(1, 3 * d + 3))
        cases.append((M, d, P, dtype, pad, p, t0, rounds, 1000 + k))
    return cases


@pytest.mark.parametrize("M,d,P,dtype,pad,p,t0,rounds,seed", _random_cases(60, 2103))
def test_random_shapes_single_and_fused(M, d, P, dtype, pad, p, t0, rounds, seed):
    """Seeded random small shapes through both paths: the fused run gives the bits of the
    round-by-round run, both agree with the oracle, padding stays untouched."""
    N = M ** d
    w = inputs.Workload(f"rand-{seed}", N, M, d, P, dtype, "peer_offset", inputs.KIND_IID if p > 0 else inputs.KIND_NONE,
                        p, 0, rounds, seed, seed + 1)
    say(f"case {w} pad={pad} t0={t0}")
    stride = P + pad
    bufA = torch.full((N * stride + 16,), 512.0, dtype=w.torch_dtype, device=DEV)
    A = bufA[: N * stride].view(N, stride)[:, :P]
    A.copy_(inputs.make_state(w, DEV))
    bufB = bufA.clone()
    B = bufB[: N * stride].view(N, stride)[:, :P]
    ref = to_f64(A).copy()
    masks = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, N, t0, rounds)
    dist_ref = orc.run(ref, M, d, t0, rounds, masks, want_dist=True)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(A, )
        dist_a, _ = m.run(t0, rounds, sched_of(w), want_dist=True)
        m.bind_state(B)
        dist_b, _ = m.run(t0, rounds, sched_of(w), want_dist=True, flags=binding.RUN_FUSED)
    assert torch.equal(bufA, bufB), "fused run differs from single rounds (or padding was touched)"
    assert_state_close(to_f64(A), ref, TOL[dtype], w.name)
    have = ~np.isnan(dist_b)
    assert np.array_equal(dist_b[have], dist_a[have])
    assert_dist_close(dist_a, dist_ref, TOL[dtype], dist_floor(P, dtype, 1.5), w.name)
    if pad:
        whole = bufA[: N * stride].view(N, stride).to(torch.float32)
        assert bool((whole[:, P:] == 512.0).all()) and bool((bufA[N * stride:].to(torch.float32) == 512.0).all())


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_fused_full_size_matches_single_rounds(cfg):
    """Full-size workloads: the fused path reproduces the single-round path bit for bit,
    on every element of the state."""
    w = inputs.CONFIGS[cfg]
    say(f"fused full-size {w.name}")
    stride = inputs.aligned_row_stride(w.P, w.dtype)
    A = inputs.make_state(w, DEV, row_stride=stride)
    B = inputs.make_state(w, DEV, row_stride=stride)      # same seed, same bytes, same layout
    with binding.Moshpit(w.N, w.P, w.M, w.d, w.dtype) as m:
        m.bind_state(A)
        _, ms_a = m.run(0, w.rounds, sched_of(w), want_times=True)
        m.bind_state(B)
        _, ms_b = m.run(0, w.rounds, sched_of(w), want_times=True, flags=binding.RUN_FUSED)
    say(f"  single rounds {ms_a.sum():.3f} ms, fused {ms_b.sum():.3f} ms")
    assert torch.equal(A, B)


@pytest.mark.parametrize("M,d,P,dtype,p,t0,rounds", [
    (2, 14, 40, 0, 0.1, 12, 3),          # 16,384 peers in groups of 2, axes 12, 13, 0
    (16, 4, 24, 0, 0.1, 2, 3),           # 65,536 peers: planes of 256 rows, rows of 96 bytes, axes 2, 3, 0
    (64, 3, 8, 1, 0.05, 1, 2),           # 262,144 peers in groups of 64, one 16-byte vector per row
])
def test_many_peers_single_and_fused(M, d, P, dtype, p, t0, rounds):
    """Grids of 16,384 to 262,144 peers with short rows (row index arithmetic far beyond
    the workloads' 4,096 rows; the oracle scans all peers per group, which bounds the sizes):
    whole state against the oracle, fused run bit-identical."""
    N = M ** d
    w = inputs.Workload(f"many-{M}-{d}", N, M, d, P, dtype, "normal", inputs.KIND_IID, p, 0, rounds, 31 + M, 32 + d)
    say(f"case {w} t0={t0}")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(w.data_seed)
    A = torch.randn(N, P, generator=gen, device=DEV, dtype=torch.float32).to(w.torch_dtype)
    B = A.clone()
    ref = to_f64(A).copy()
    masks = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, N, t0, rounds)
    orc.run(ref, M, d, t0, rounds, masks)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(A)
        m.run(t0, rounds, sched_of(w))
        m.bind_state(B)
        m.run(t0, rounds, sched_of(w), flags=binding.RUN_FUSED)
        m.sync()
    assert torch.equal(A, B), "fused run differs from single rounds"
    assert_state_close(to_f64(A), ref, TOL[dtype], w.name)


# --------------------------------------------------------------------------
# partly filled grids (N peers on a subset of the M^d vertices)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("M,d,n_present,dtype,P,p", [(32, 2, 512, 0, 1_000, 0.01), (32, 2, 900, 0, 333, 0.0),
                                                      (8, 3, 300, 1, 2_048, 0.05), (4, 2, 1, 0, 64, 0.0)])
def test_partly_filled_grid(M, d, n_present, dtype, P, p):
    """Empty vertices never take part and are left out of the error measure
    (the setting of Table 4's N < 1024 rows)."""
    N, rounds = M ** d, 7
    rng = np.random.default_rng(N + n_present)
    present = np.zeros(N, dtype=np.uint8)
    present[rng.choice(N, size=n_present, replace=False)] = 1
    w = inputs.Workload("partial", N, M, d, P, dtype, "normal", 1, p, 0, rounds, 77, 78)
    say(f"partial grid {w} present={n_present}")
    X = inputs.make_state(w, DEV)
    ref = to_f64(X).copy()
    masks = orc.schedule_masks(1, p, 78, 0, N, 0, rounds) & present
    floor = dist_floor(P, dtype, 1.0)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(X)
        for t in range(rounds):
            got = m.dist_to_mean_subset(present)
            want = orc.dist_to_mean_subset(ref, present)
            assert abs(got - want) <= TOL[dtype] * want + floor, (t, got, want)
            m.round(t, masks[t])
            orc.round_(ref, M, d, t, masks[t])
        m.sync()
        assert_state_close(to_f64(X), ref, TOL[dtype], "partial grid")
        assert m.dist_to_mean_subset(None) == m.dist_to_mean()
        assert m.dist_to_mean_subset(np.zeros(N, np.uint8)) == 0.0
    # rows of empty vertices were never written
    X0 = inputs.make_state(w, DEV)
    empty = torch.from_numpy(present == 0).to(DEV)
    assert torch.equal(X[empty], X0[empty])


# --------------------------------------------------------------------------
# averaging in random groups (the simplified scheme of Thm 3.2) and list-based rounds
# --------------------------------------------------------------------------

@pytest.mark.parametrize("N", [16, 100, 1024, 4096, 6561, 16384])
def test_random_permutation_bit_exact(N):
    # the permutation only depends on N: use any handle with that many peers
    # (6561 and 16384 peers span several chunks of the device sort, the first with padding)
    shapes = {16: (4, 2), 100: (10, 2), 1024: (32, 2), 4096: (16, 3), 6561: (3, 8), 16384: (4, 7)}
    M, d = shapes[N]
    with binding.Moshpit(N, 8, M, d, 0) as m:
        for t, seed in ((0, 1), (3, 2**63 + 5), (7, 12345)):
            say(f"perm N={N} t={t} seed={seed}")
            assert np.array_equal(m.random_permutation(t, seed), orc.random_permutation(seed, t, N))


def _np_mix64(x):
    x = x ^ (x >> np.uint64(32)); x = x * np.uint64(0x9E3779B97F4A7C15)
    x = x ^ (x >> np.uint64(29)); x = x * np.uint64(0x6A09E667F3BCC909)
    return x ^ (x >> np.uint64(32))


@pytest.mark.parametrize("M,d", [(16, 4), (2, 18), (3, 11)])
def test_random_permutation_of_many_peers(M, d):
    """65,536 to 262,144 peers (the oracle's rank-by-counting would take minutes): the
    permutation is the unique ascending order of the keys stated in the header, ties by
    index; checked with the keys recomputed here in 64-bit numpy arithmetic."""
    N = M ** d
    with binding.Moshpit(N, 8, M, d, 0) as m:
        for t, seed in ((2, 7), (9, 2**64 - 3)):
            say(f"perm N={N} t={t} seed={seed}")
            got = m.random_permutation(t, seed)
            with np.errstate(over="ignore"):
                rk = _np_mix64(np.uint64(seed) + np.uint64(0xD1B54A32D192ED03) * np.uint64(t + 1))
                keys = _np_mix64(rk ^ np.arange(N, dtype=np.uint64))
            assert np.array_equal(got, np.lexsort((np.arange(N), keys)).astype(np.int32))
        small = orc.random_permutation(7, 2, 4096)          # the recomputed keys are the oracle's keys
        with np.errstate(over="ignore"):
            rk = _np_mix64(np.uint64(7) + np.uint64(0xD1B54A32D192ED03) * np.uint64(3))
            keys = _np_mix64(rk ^ np.arange(4096, dtype=np.uint64))
        assert np.array_equal(small, np.lexsort((np.arange(4096), keys)))


@pytest.mark.parametrize("M,d,P,dtype,gs,p", [(32, 2, 3_000, 0, 32, 0.0), (32, 2, 1_001, 0, 7, 0.2),
                                              (16, 3, 520, 1, 16, 0.1), (10, 2, 4_096, 0, 64, 0.3),
                                              (4, 2, 999, 1, 2, 0.25), (3, 3, 64, 0, 5, 0.0), (4, 3, 5_000, 0, 1, 0.0)])
def test_random_groups_rounds(M, d, P, dtype, gs, p):
    N, rounds, seed = M ** d, 4, 99
    w = inputs.Workload("random-groups", N, M, d, P, dtype, "peer_offset", 1, p, 0, rounds, 5 + P, 6 + gs)
    say(f"random groups {w} group_size={gs}")
    stride = P + (8 - P % 8) % 8
    X = inputs.make_state(w, DEV, row_stride=stride)
    ref = to_f64(X).copy()
    masks = orc.schedule_masks(1, p, w.mask_seed, 0, N, 0, rounds)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(X)
        for t in range(rounds):
            m.random_groups_round(t, seed, gs, masks[t] if p > 0 else None)
            orc.random_groups_round(ref, seed, t, gs, masks[t] if p > 0 else None)
        m.sync()
        assert_state_close(to_f64(X), ref, TOL[dtype], w.name)
        d_got, d_want = m.dist_to_mean(), orc.dist_to_mean(ref)
        assert abs(d_got - d_want) <= TOL[dtype] * d_want + dist_floor(P, dtype, 1.0)


def test_random_groups_contraction_rate():
    """One round of random groups of 32 among 1024 peers shrinks the distortion
    by (r-1)/(N-1) = 31/1023 in expectation (Thm 3.2, whose printed rate
    31/1024 + 32/1024^2 is the same to 1e-6); with 8192 iid columns a single
    permutation already averages to well within 2 %."""
    N, P, gs = 1024, 8192, 32
    w = inputs.Workload("rate", N, 32, 2, P, 0, "normal", 0, 0.0, 0, 1, 31, 32)
    X = inputs.make_state(w, DEV)
    with binding.Moshpit(N, P, 32, 2, 0) as m:
        m.bind_state(X)
        d0 = m.dist_to_mean()
        m.random_groups_round(0, 7, gs)
        d1 = m.dist_to_mean()
    rate = 31 / 1023
    assert abs(d1 / d0 - rate) <= 0.02 * rate, (d1 / d0, rate)


def test_grouped_round_with_caller_groups():
    N, P = 64, 2_000
    w = inputs.Workload("lists", N, 8, 2, P, 0, "normal", 0, 0.0, 0, 1, 41, 42)
    X = inputs.make_state(w, DEV)
    X0 = X.clone()
    ref = to_f64(X).copy()
    rng = np.random.default_rng(8)
    index = rng.permutation(N)[:50]                      # 14 peers are not listed at all
    alive = (rng.random(N) > 0.2).astype(np.uint8)
    with binding.Moshpit(N, P, 8, 2, 0) as m:
        m.bind_state(X)
        m.grouped_round(index, 6, alive)
        orc.grouped_round(ref, index, 6, alive)
        m.sync()
        assert_state_close(to_f64(X), ref, 1e-6, "caller groups")
        untouched = np.setdiff1d(np.arange(N), index[alive[index] == 1])
        assert torch.equal(X[untouched], X0[untouched])
        m.grouped_round(np.zeros(0, np.int32), 4)       # empty list: nothing happens
        with pytest.raises(binding.MoshpitError):
            m.grouped_round([1, 2, 2], 2)               # a peer listed twice
        with pytest.raises(binding.MoshpitError):
            m.grouped_round([1, 64], 2)                 # out of range
        with pytest.raises(binding.MoshpitError):
            m.random_groups_round(0, 1, 65)


# --------------------------------------------------------------------------
# group-skip failure behaviour
# --------------------------------------------------------------------------

@pytest.mark.parametrize("M,d,P,dtype,p,fused", [(16, 2, 2_000, 0, 0.02, 0), (4, 3, 1_000, 1, 0.1, 0),
                                                  (32, 2, 520, 0, 0.01, 1), (3, 3, 100, 0, 0.05, 1)])
def test_group_skip_schedule(M, d, P, dtype, p, fused):
    N, rounds = M ** d, 6
    w = inputs.Workload("skip", N, M, d, P, dtype, "normal", 1, p, 0, rounds, 51, 52)
    say(f"group skip {w} fused={fused}")
    X = inputs.make_state(w, DEV, row_stride=P + (8 - P % 8) % 8)
    ref = to_f64(X).copy()
    raw = orc.schedule_masks(1, p, 52, 0, N, 0, rounds)
    eff = np.stack([orc.skip_filter(N, M, d, t, raw[t]) for t in range(rounds)])
    orc.run(ref, M, d, 0, rounds, eff)
    sched = binding.Schedule(kind=1, p=p, seed=52, group_skip=True)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(X)
        assert np.array_equal(m.schedule_mask(sched, 0, rounds), eff)
        m.run(0, rounds, sched, flags=binding.RUN_FUSED if fused else 0)
        m.sync()
        # explicit masks go through the same filter
        sched2 = binding.Schedule(kind=binding.SCHED_EXPLICIT, explicit_masks=raw, group_skip=True)
        assert np.array_equal(m.schedule_mask(sched2, 0, rounds), eff)
    assert_state_close(to_f64(X), ref, TOL[dtype], "group skip")


# --------------------------------------------------------------------------
# a returning peer copies an up-to-date peer (App. on a dynamic number of peers)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("M,d", [(4, 2), (7, 2), (16, 2), (32, 2), (16, 3), (2, 11), (64, 1)])
def test_refresh_donors_bit_exact(M, d):
    """The draw of the donors against the oracle's, byte for byte, over random and
    degenerate pairs of masks (more peers than one pass of the planning block,
    nobody to copy from, nobody returning, everybody returning)."""
    N = M ** d
    say(f"refresh donors N={N}")
    rng = np.random.default_rng(N)
    X = torch.zeros(N, 8, device=DEV)
    ones, zeros = np.ones(N, dtype=np.uint8), np.zeros(N, dtype=np.uint8)
    one_left = zeros.copy(); one_left[N // 2] = 1
    cases = [((rng.random(N) < a).astype(np.uint8), (rng.random(N) < b).astype(np.uint8))
             for a, b in ((0.5, 0.5), (0.9, 0.8), (0.1, 0.9), (0.02, 0.98))]
    cases += [(zeros, ones), (ones, ones), (ones, zeros), (one_left, ones), (zeros, zeros)]
    with binding.Moshpit(N, 8, M, d, 0) as m:
        m.bind_state(X)
        for k, (prev, cur) in enumerate(cases):
            for t, seed in ((0, 1), (5, 2**63 + 11), (10**6, 77)):
                got = m.refresh_donors(t, seed, prev, cur)
                assert np.array_equal(got, orc.refresh_donors(prev, cur, seed, t)), f"case {k} t={t}"


@pytest.mark.parametrize("M,d,P,dtype,pad,offset", [(16, 2, 40_000, 0, 0, 0), (4, 3, 9_999, 0, 1, 0), (8, 2, 8_195, 1, 5, 0),
                                                     (32, 2, 3_001, 0, 3, 1), (7, 2, 20_001, 1, 7, 3), (5, 2, 1, 0, 0, 0)])
def test_refresh_copies_rows_exactly(M, d, P, dtype, pad, offset):
    """moshpit_refresh: returning rows become bit copies of their donors' rows, nothing
    else changes (other rows, padding, guard elements) - aligned rows take the 128-bit
    path with an element-wise ragged end, unaligned ones the element-wise path."""
    N = M ** d
    stride = P + pad
    w = inputs.Workload("refresh", N, M, d, P, dtype, "normal", 0, 0.0, 0, 0, 5 + P, 6)
    say(f"refresh copy {w} stride={stride} offset={offset}")
    buf = torch.full((N * stride + offset + 64,), 512.0, dtype=w.torch_dtype, device=DEV)
    X = buf[offset: offset + N * stride].view(N, stride)[:, :P]
    X.copy_(inputs.make_state(w, DEV))
    before = buf.clone()
    rng = np.random.default_rng(P)
    prev = (rng.random(N) < 0.6).astype(np.uint8)
    cur = (rng.random(N) < 0.8).astype(np.uint8)
    donor = orc.refresh_donors(prev, cur, 9, 4)
    assert (donor >= 0).any()
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(X)
        m.refresh(4, 9, prev, cur)
        m.sync()
    want = before.clone()
    Wv = want[offset: offset + N * stride].view(N, stride)
    Bv = before[offset: offset + N * stride].view(N, stride)
    idx = torch.from_numpy(np.flatnonzero(donor >= 0)).to(DEV)
    src = torch.from_numpy(donor[donor >= 0].astype(np.int64)).to(DEV)
    Wv[idx, :P] = Bv[src, :P]
    assert torch.equal(buf, want)


@pytest.mark.parametrize("M,d,P,dtype,kind,p,skip", [(16, 2, 3_000, 0, 2, 0.15, False), (4, 3, 1_001, 0, 1, 0.3, False),
                                                      (16, 3, 264, 1, 2, 0.1, False), (8, 2, 2_048, 0, 2, 0.1, True),
                                                      (32, 2, 520, 1, 1, 0.2, True)])
def test_run_with_refresh(M, d, P, dtype, kind, p, skip):
    """A run whose schedule asks for the refresh: before every round but the first the
    returning peers copy their donors (drawn from the presence masks, also when the
    group-skip filter then thins the participation), then the round runs.  Against the
    oracle taking the same steps one by one; the run is not fused even when allowed."""
    N, rounds, seed = M ** d, 9, 1234
    w = inputs.Workload("run-refresh", N, M, d, P, dtype, "peer_offset", kind, p, 2, rounds, 71, seed)
    say(f"run with refresh {w} skip={skip}")
    X = inputs.make_state(w, DEV)
    ref = to_f64(X).copy()
    presence = orc.schedule_masks(kind, p, seed, 2, N, 0, rounds)
    dist_ref = [orc.dist_to_mean(ref)]
    n_copies = 0
    for t in range(rounds):
        if t > 0:
            donor = orc.refresh_donors(presence[t - 1], presence[t], seed, t)
            n_copies += int((donor >= 0).sum())
            orc.refresh(ref, donor)
        eff = orc.skip_filter(N, M, d, t, presence[t]) if skip else presence[t]
        orc.round_(ref, M, d, t, eff)
        dist_ref.append(orc.dist_to_mean(ref))
    assert n_copies > 0
    sched = binding.Schedule(kind=kind, p=p, seed=seed, down_rounds=2, group_skip=skip, refresh=True)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(X)
        dist, _ = m.run(0, rounds, sched, want_dist=True, flags=binding.RUN_FUSED)
    assert not np.isnan(dist).any(), "a run with refresh must go round by round"
    assert_state_close(to_f64(X), ref, TOL[dtype], w.name)
    assert_dist_close(dist, np.array(dist_ref), TOL[dtype], dist_floor(P, dtype, 1.0), w.name)


def test_refresh_full_size_workload5():
    """Workload 5 at full size (4096 peers that die and come back after 2 rounds): a run
    with the refresh against the oracle on sampled columns."""
    w = inputs.CONFIGS[5]
    say(f"refresh full-size {w.name}")
    X = inputs.make_state(w, DEV)
    cols = sample_columns(w.P, 1024, seed=505)
    tc = torch.from_numpy(cols).to(DEV)
    ref = X[:, tc].to(torch.float64).cpu().numpy().copy()
    presence = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, w.N, 0, w.rounds)
    for t in range(w.rounds):
        if t > 0:
            orc.refresh(ref, orc.refresh_donors(presence[t - 1], presence[t], w.mask_seed, t))
        orc.round_(ref, w.M, w.d, t, presence[t])
    sched = binding.Schedule(kind=w.kind, p=w.p, seed=w.mask_seed, down_rounds=w.down, refresh=True)
    with binding.Moshpit(w.N, w.P, w.M, w.d, w.dtype) as m:
        m.bind_state(X)
        m.run(0, w.rounds, sched)
        m.sync()
    assert_state_close(X[:, tc].to(torch.float64).cpu().numpy(), ref, TOL[w.dtype], w.name)


# --------------------------------------------------------------------------
# Moshpit SGD iterations (Alg. 2)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("M,d,P,dtype,p,pad", [(16, 2, 3_000, 0, 0.1, 0), (4, 3, 1_001, 0, 0.2, 3), (32, 2, 520, 1, 0.1, 0),
                                                (3, 2, 77, 1, 0.3, 1), (8, 2, 4_096, 0, 0.0, 0)])
def test_sgd_iterations(M, d, P, dtype, p, pad):
    """tau = 2: a local step, then a step with the averaging round fused in."""
    N, iters, gamma = M ** d, 6, 0.05
    w = inputs.Workload("sgd", N, M, d, P, dtype, "peer_offset", 1, p, 0, iters, 61, 62)
    say(f"sgd {w}")
    X = inputs.make_state(w, DEV, row_stride=P + pad)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(63)
    ref = to_f64(X).copy()
    masks = orc.schedule_masks(1, p, 62, 0, N, 0, iters)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(X)
        t = 0
        for k in range(iters):
            G = torch.randn(N, P + pad, generator=gen, device=DEV).to(w.torch_dtype)[:, :P]
            Gref = to_f64(G).copy()
            alive = masks[k] if p > 0 else None
            if k % 2 == 1:
                m.sgd_round(t, G, gamma, alive)
                orc.sgd_round(ref, Gref, np.float32(gamma), M, d, t, alive)
                t += 1
            else:
                m.local_step(G, gamma, alive)
                orc.local_step(ref, Gref, np.float32(gamma), alive)
            m.sync()
        assert_state_close(to_f64(X), ref, TOL[dtype], w.name)


@pytest.mark.parametrize("M,d,P,dtype,p,pad,gpad,t0,rounds", [
    (8, 2, 4_096, 0, 0.1, 0, 0, 0, 2),        # the paper's ALBERT shape: two rounds per iteration on an 8 x 8 grid
    (8, 2, 4_096, 1, 0.1, 0, 0, 0, 2),
    (16, 2, 5_000, 0, 0.05, 0, 0, 1, 5),      # ragged last column tile, start on the second axis
    (32, 2, 4_100, 0, 0.2, 0, 0, 0, 8),       # 1024 rows x 128-byte segments, one block per compute unit
    (16, 3, 2_056, 1, 0.1, 0, 0, 0, 6),       # planes: the local step rides on the first of three passes
    (4, 3, 9_999, 0, 0.1, 1, 1, 0, 6),        # rows not 16-byte aligned: nothing fuses
    (4, 3, 10_000, 0, 0.0, 0, 8, 0, 3),       # gradient matrix with another row stride: first round unfused
    (3, 3, 780, 0, 0.25, 0, 0, 2, 4),
    (64, 1, 2_048, 0, 0.1, 0, 0, 0, 1),       # one axis, one round
])
def test_sgd_run(M, d, P, dtype, p, pad, gpad, t0, rounds):
    """An iteration of Moshpit SGD with several averaging rounds: local step of the peers present in
    the first round, then the rounds - against the oracle taking the same steps, through the fused
    and the round-by-round path; for binary32 state both give the bits of moshpit_sgd_round followed
    by the remaining rounds."""
    N, gamma = M ** d, 0.05
    w = inputs.Workload("sgd-run", N, M, d, P, dtype, "peer_offset", inputs.KIND_IID if p > 0 else inputs.KIND_NONE, p, 0,
                        rounds, 161 + P, 162 + M)
    say(f"sgd run {w} pad={pad} gpad={gpad} t0={t0}")
    X0 = inputs.make_state(w, DEV, row_stride=P + pad)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(163)
    G = torch.randn(N, P + gpad, generator=gen, device=DEV).to(w.torch_dtype)[:, :P]
    masks = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, N, t0, rounds)
    ref = to_f64(X0).copy()
    d0 = orc.dist_to_mean(ref)
    orc.local_step(ref, to_f64(G).copy(), np.float32(gamma), masks[0] if p > 0 else None)
    dist_ref = orc.run(ref, M, d, t0, rounds, masks, want_dist=True)
    dist_ref[0] = d0
    results = []
    with binding.Moshpit(N, P, M, d, dtype) as m:
        for flags in (0, binding.RUN_FUSED):
            X = inputs.make_state(w, DEV, row_stride=P + pad)
            m.bind_state(X)
            dist, _ = m.sgd_run(t0, rounds, G, gamma, sched_of(w), want_dist=True, flags=flags)
            assert_state_close(to_f64(X), ref, TOL[dtype], f"{w.name} flags={flags}")
            have = ~np.isnan(dist)
            assert have[0] and have[-1]
            assert_dist_close(dist[have], dist_ref[have], TOL[dtype], dist_floor(P, dtype, 1.5), w.name)
            results.append(X)
        Y = inputs.make_state(w, DEV, row_stride=P + pad)
        m.bind_state(Y)
        m.sgd_round(t0, G, gamma, masks[0] if p > 0 else None)
        if rounds > 1:
            m.run(t0 + 1, rounds - 1, sched_of(w))
        m.sync()
        assert torch.equal(results[0], Y), "round-by-round sgd_run differs from sgd_round + run"
        if dtype == 0:
            assert torch.equal(results[1], Y), "fused sgd_run differs from sgd_round + run"
        with pytest.raises(binding.MoshpitError):
            m.sgd_run(t0, 0, G, gamma)


def test_sgd_quadratic_mean_trajectory():
    """Exact gradients of 1/2 ||theta - theta*||^2, all peers present: the mean
    over peers follows theta* + (1-gamma)^K (mean_0 - theta*) whatever the
    averaging does (closed form pinned for the oracle on the CPU)."""
    M, d, P, gamma = 8, 2, 2_048, 0.1
    N = M * M
    w = inputs.Workload("sgd-quad", N, M, d, P, 0, "peer_offset", 0, 0.0, 0, 1, 71, 72)
    X = inputs.make_state(w, DEV)
    star = torch.linspace(-1, 1, P, device=DEV)
    mean0 = X.double().mean(dim=0)
    with binding.Moshpit(N, P, M, d, 0) as m:
        m.bind_state(X)
        t = 0
        for k in range(8):
            G = X - star
            if k % 2 == 1:
                m.sgd_round(t, G, gamma)
                t += 1
            else:
                m.local_step(G, gamma)
            m.sync()
    want = star.double() + (1 - np.float64(np.float32(gamma))) ** 8 * (mean0 - star.double())
    got = X.double().mean(dim=0)
    assert float((got - want).abs().max()) <= 2e-6 * float(want.abs().max())
    assert float((X - X.mean(dim=0)).abs().max()) <= 1e-5


def test_rounds_replayed_from_a_hip_graph():
    """The round loop captured in a HIP graph (device masks, so a round is kernel launches
    only) and replayed: every replay, with eager work and synchronisations between the
    replays, gives the bits of the eager loop."""
    M, d, P, rounds = 16, 2, 5_000, 6
    N = M ** d
    w = inputs.Workload("graph", N, M, d, P, 0, "peer_offset", inputs.KIND_IID, 0.1, 0, rounds, 31, 32)
    say("hip graph replay")
    X0 = inputs.make_state(w, DEV)
    masks = torch.from_numpy(orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, N, 0, rounds)).to(DEV)
    side = torch.cuda.Stream()
    X = X0.clone()
    with binding.Moshpit(N, P, M, d, 0) as m:
        m.bind_state(X, stream=side)
        with torch.cuda.stream(side):
            for t in range(rounds):                       # eager reference (also the warm-up launches)
                m.round_dev(t, masks[t])
        side.synchronize()
        want = X.clone()
        graph = torch.cuda.CUDAGraph()
        X.copy_(X0)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for t in range(rounds):
                m.round_dev(t, masks[t])
        for replay in range(3):
            X.copy_(X0)
            scratch = (X0 * 2.0).sum()                    # unrelated eager work between replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(X, want), f"replay {replay} differs from the eager rounds"
            assert bool(torch.isfinite(scratch))
        m.sync()


# --------------------------------------------------------------------------
# streams and several handles
# --------------------------------------------------------------------------

def test_user_stream_and_two_handles():
    """Work is queued on the stream given to bind_state; two handles on two
    streams do not disturb each other."""
    M, d, P, rounds = 8, 2, 50_000, 6
    N = M ** d
    wa = inputs.Workload("stream-a", N, M, d, P, 0, "normal", 1, 0.1, 0, rounds, 81, 82)
    wb = inputs.Workload("stream-b", N, M, d, P, 1, "peer_offset", 2, 0.2, 2, rounds, 83, 84)
    A, B = inputs.make_state(wa, DEV), inputs.make_state(wb, DEV)
    ref_a, ref_b = to_f64(A).copy(), to_f64(B).copy()
    orc.run(ref_a, M, d, 0, rounds, orc.schedule_masks(1, 0.1, 82, 0, N, 0, rounds))
    orc.run(ref_b, M, d, 0, rounds, orc.schedule_masks(2, 0.2, 84, 2, N, 0, rounds))
    sa, sb = torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)
    torch.cuda.synchronize()
    with binding.Moshpit(N, P, M, d, 0) as ma, binding.Moshpit(N, P, M, d, 1) as mb:
        ma.bind_state(A, sa)
        mb.bind_state(B, sb)
        for r in range(rounds):                       # interleave the two handles round by round
            ma.run(r, 1, sched_of(wa))
            mb.run(r, 1, sched_of(wb), flags=binding.RUN_FUSED)
        ma.sync()
        mb.sync()
    assert_state_close(to_f64(A), ref_a, TOL[0], "stream a")
    assert_state_close(to_f64(B), ref_b, TOL[1], "stream b")


def test_host_masks_are_read_before_the_call_returns():
    """A mask in PINNED host memory that the caller overwrites right after moshpit_round
    returned, while earlier work still occupies the stream: the round must use the bytes
    the mask held at the call (an asynchronous copy straight from pinned memory would
    read the overwritten ones).  Same for an explicit schedule and the refresh masks."""
    M, d, P = 16, 2, 200_000
    N = M * M
    w = inputs.Workload("pinned", N, M, d, P, 0, "peer_offset", 1, 0.3, 0, 4, 55, 56)
    X = inputs.make_state(w, DEV)
    ref = to_f64(X).copy()
    masks = orc.schedule_masks(1, 0.3, 56, 0, N, 0, 4)
    lib = binding.load_library()
    pinned = torch.empty(4, N, dtype=torch.uint8).pin_memory()
    with binding.Moshpit(N, P, M, d, 0) as m:
        m.bind_state(X)
        for rep in range(3):                                   # keep the stream busy
            m.run(100 + 2 * rep, 2, None)
        pinned[0].copy_(torch.from_numpy(masks[0]))
        assert lib.moshpit_round(m._h, 0, pinned[0].data_ptr()) == 0
        pinned[0].zero_()                                      # the caller reuses its buffer at once
        pinned[:3].copy_(torch.from_numpy(masks[1:4]))
        cs = binding._CSchedule(binding.SCHED_EXPLICIT, 0, 0.0, 0, pinned.data_ptr(), 0, 0)
        import ctypes
        assert lib.moshpit_run(m._h, 1, 3, ctypes.byref(cs), 0, None, None) == 0
        pinned.zero_()
        m.sync()
    for rep in range(3):
        orc.run(ref, M, d, 100 + 2 * rep, 2, None)
    orc.run(ref, M, d, 0, 4, masks)
    assert_state_close(to_f64(X), ref, TOL[0], "pinned masks")


def test_rejoin_schedule_far_into_a_run():
    """Die-and-rejoin masks a million rounds in, and their continuation from the state the
    handle carries, equal the oracle's (which walks every round from 0)."""
    N, M, d, down, p, seed, t0 = 256, 16, 2, 3, 0.2, 4321, 1_000_000
    sched = binding.Schedule(kind=binding.SCHED_REJOIN, p=p, seed=seed, down_rounds=down)
    want = orc.schedule_masks(2, p, seed, down, N, t0, 12)
    with binding.Moshpit(N, 8, M, d, 0) as m:
        assert np.array_equal(m.schedule_mask(sched, t0, 5), want[:5])          # walks from round 0 once
        assert np.array_equal(m.schedule_mask(sched, t0 + 5, 4), want[5:9])     # goes on from the carried state
        assert np.array_equal(m.schedule_mask(sched, t0 + 10, 2), want[10:12])  # skips a round: walks it
        assert np.array_equal(m.schedule_mask(sched, t0 + 2, 3), want[2:5])     # earlier than the carried state
        other = binding.Schedule(kind=binding.SCHED_REJOIN, p=p, seed=seed + 1, down_rounds=down)
        assert np.array_equal(m.schedule_mask(other, 7, 3), orc.schedule_masks(2, p, seed + 1, down, N, 7, 3))
        assert np.array_equal(m.schedule_mask(sched, 0, 6), orc.schedule_masks(2, p, seed, down, N, 0, 6))


def test_first_launches_from_two_threads():
    """Two host threads, each with a handle of its own, make the first launches of the
    process's kernels at the same time (the per-device launch table is shared)."""
    import threading
    M, d, P, rounds = 32, 2, 4_096, 6
    N = M * M
    results = {}

    def work(k):
        w = inputs.Workload(f"thread-{k}", N, M, d, P, k % 2, "peer_offset", 1, 0.1, 0, rounds, 100 + k, 200 + k)
        X = inputs.make_state(w, DEV)
        ref = to_f64(X).copy()
        stream = torch.cuda.Stream(device=DEV)
        torch.cuda.synchronize()
        with binding.Moshpit(N, P, M, d, w.dtype) as m:
            m.bind_state(X, stream)
            m.run(0, rounds, sched_of(w), flags=binding.RUN_FUSED if k >= 2 else 0)
            m.sync()
        orc.run(ref, M, d, 0, rounds, orc.schedule_masks(1, 0.1, 200 + k, 0, N, 0, rounds))
        results[k] = (to_f64(X), ref, w.dtype)

    threads = [threading.Thread(target=work, args=(k,)) for k in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert sorted(results) == [0, 1, 2, 3]
    for k, (got, ref, dtype) in results.items():
        assert_state_close(got, ref, TOL[dtype], f"thread {k}")


# --------------------------------------------------------------------------
# Alg. 1 with chunk-index keys
# --------------------------------------------------------------------------

@pytest.mark.parametrize("M,d,P,dtype,p", [(32, 2, 1_000, 0, 0.05), (16, 3, 264, 1, 0.1), (4, 3, 3_001, 0, 0.3),
                                           (3, 4, 96, 0, 0.2), (2, 5, 512, 1, 0.0), (8, 1, 100, 0, 0.25),
                                           (7, 2, 4_096, 0, 0.0), (4, 7, 64, 0, 0.1), (3, 8, 24, 1, 0.2)])
def test_dynamic_key_rounds(M, d, P, dtype, p):
    N, rounds, seed = M ** d, 2 * d + 2, 1234
    w = inputs.Workload("dynamic", N, M, d, P, dtype, "peer_offset", 1, p, 0, rounds, 91, 92)
    say(f"chunk-index keys {w}")
    X = inputs.make_state(w, DEV, row_stride=P + (8 - P % 8) % 8)
    X0 = to_f64(X).copy()
    ref = X0.copy()
    keys = orc.dynamic_init(N, M, d)
    masks = orc.schedule_masks(1, p, 92, 0, N, 0, rounds)
    with binding.Moshpit(N, P, M, d, dtype) as m:
        m.bind_state(X)
        assert np.array_equal(m.dynamic_keys(), keys)
        for t in range(rounds):
            alive = masks[t] if p > 0 else None
            m.dynamic_round(t, seed, alive)
            orc.dynamic_round(ref, M, d, keys, seed, t, alive)
            assert np.array_equal(m.dynamic_keys(), keys), f"keys differ after round {t}"
            if p == 0 and t == d - 1:
                m.sync()
                assert_state_close(to_f64(X), np.broadcast_to(X0.mean(axis=0), X0.shape), TOL[dtype], "exact mean")
        m.sync()
        assert_state_close(to_f64(X), ref, TOL[dtype], w.name)
        m.dynamic_reset()
        assert np.array_equal(m.dynamic_keys(), orc.dynamic_init(N, M, d))
