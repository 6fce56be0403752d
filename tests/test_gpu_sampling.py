"""GPU parity of the sampling block (section 3.3 of the paper): drift by
ss_detect_stale, per-threshold counts of droppable sampled inputs by
ss_sample_drop, both through the C ABI, against the CPU oracle, which computes
the same counts from the tables and snapshots directly.

Counts are integers and are held to exact equality; a test first makes sure
that no drift lies within 1e-6 relative of a candidate threshold (the two sides
take the verdict in fp64 on drifts that agree to about 1e-15).
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2404_04270_amd import workload as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2404_04270_amd import binding
    return binding


@pytest.fixture(scope="module")
def dev():
    return torch.device("cuda:0")


def problem(rng, T, R, D, H, S, L, thr_mid, hot_share=0.8):
    """Tables, ascending hot ids, snapshots whose drift straddles thr_mid, and
    sampled lookups of which about hot_share land on hot rows."""
    W = [rng.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]
    hot = [np.sort(rng.choice(R, H, replace=False)).astype(np.int32) for _ in range(T)]
    snap = []
    for t in range(T):
        scale = rng.uniform(0, 2 * thr_mid / math.sqrt(D), (H, 1))
        snap.append((W[t][hot[t]] + scale * rng.choice([-1.0, 1.0], (H, D))).astype(np.float32))
    sidx = np.empty((T, S, L), np.int32)
    for t in range(T):
        from_hot = hot[t][rng.integers(0, H, (S, L))]
        anywhere = rng.integers(0, R, (S, L))
        sidx[t] = np.where(rng.random((S, L)) < hot_share, from_hot, anywhere)
    return W, hot, snap, sidx


def device_state(B, dev, W, hot, snap):
    tb = B.Tables([torch.from_numpy(w).to(dev) for w in W])
    tb.new_bits()
    hs = B.HotState(tb, [torch.from_numpy(h).to(dev) for h in hot])
    for t in range(len(W)):
        hs.snapshot[t].copy_(torch.from_numpy(snap[t]))
    return tb, hs


def outside_band(W, hot, snap, thresholds):
    bits = [np.zeros((W[0].shape[0] + 31) // 32, np.uint32) for _ in W]
    _, drift, _ = oracle.detect_stale(W, bits, hot, [s.copy() for s in snap], 0.0, False)
    finite = [t for t in thresholds if 0 < t < math.inf]
    return all((np.abs(drift - t) > 1e-6 * t).all() for t in finite), drift


SAMPLE_CASES = [
    # T, R, D, H, S, L
    (3, 5000, 16, 700, 1000, 1),        # T*L = 3: one lane per input
    (26, 4000, 64, 333, 2500, 1),       # T*L = 26: 8 lanes, ragged last batch
    (8, 3000, 128, 65, 777, 20),        # T*L = 160: 64 lanes, 3 lookups each
    (40, 900, 4, 50, 130, 20),          # T*L = 800: several rounds per lane
    (1, 300, 8, 1, 70, 5),              # a single hot row
    (2, 2000, 32, 2000, 513, 2),        # every row hot
    (5, 1000, 16, 10, 1, 3),            # one sampled input
]


@pytest.mark.parametrize("T,R,D,H,S,L", SAMPLE_CASES)
def test_sample_drop_matches_oracle(B, dev, T, R, D, H, S, L):
    rng = np.random.default_rng(900 + T + H + S)
    thr_mid = 3e-3
    W, hot, snap, sidx = problem(rng, T, R, D, H, S, L, thr_mid)
    ladder = [0.0] + list(np.geomspace(thr_mid / 30, thr_mid * 3, 29)) + [math.inf, 1e-9]
    rng.shuffle(ladder)                               # any order is allowed
    ladder = [float(np.float32(x)) for x in ladder]
    ok, ref_drift = outside_band(W, hot, snap, ladder)
    assert ok
    tb, hs = device_state(B, dev, W, hot, snap)
    B.ss_detect_stale(tb, hs, 0.0, refresh_snapshot=False)
    for t in range(T):
        np.testing.assert_allclose(hs.drift[t].cpu().numpy(), ref_drift[t], rtol=1e-12)
        assert not tb.bits[t].any()                   # threshold 0 flags nothing
        assert np.array_equal(hs.snapshot[t].cpu().numpy(), snap[t])
    sidx_d = torch.from_numpy(sidx).to(dev)
    counts = torch.full((32,), -1, dtype=torch.int32, device=dev)
    seen = set()
    for alpha in sorted({0, 1, 2, T * L // 3, T * L - 1, T * L, T * L + 1}):
        for n_thr in (32, 5):
            counts.fill_(-1)
            B.ss_sample_drop(hs, sidx_d, alpha, ladder[:n_thr], counts)
            got = counts.cpu().numpy()
            ref = oracle.sample_drop(W, hot, snap, sidx, alpha, ladder[:n_thr])
            assert np.array_equal(got[:n_thr].view(np.uint32), ref), (alpha, n_thr)
            assert np.all(got[n_thr:] == -1)          # nothing written past n_thr
            seen.update(int(c) for c in ref)
    assert 0 in seen and S in seen
    if S > 500:
        assert len(seen) > 4                          # the ladder does discriminate


def test_sample_drop_without_samples_gives_zero_counts(B, dev):
    rng = np.random.default_rng(950)
    W, hot, snap, sidx = problem(rng, 2, 100, 8, 10, 4, 1, 1e-3)
    tb, hs = device_state(B, dev, W, hot, snap)
    B.ss_detect_stale(tb, hs, 0.0, refresh_snapshot=False)
    counts = torch.full((3,), 9, dtype=torch.int32, device=dev)
    empty = torch.zeros((2, 0, 1), dtype=torch.int32, device=dev)
    B.ss_sample_drop(hs, empty, 0, [1e-3, 0.0, math.inf], counts)
    assert counts.cpu().tolist() == [0, 0, 0]


def test_sample_drop_agrees_with_detect_then_filter(B, dev):
    """The count for threshold T equals the number of inputs ss_filter_batch
    would skip after ss_detect_stale had run with that T (Eq. 1 and Eq. 6-8 on
    the sample): the three kernels share no code."""
    rng = np.random.default_rng(960)
    T, R, D, H, S, L = 6, 3000, 32, 400, 1500, 2
    thr = 3.6e-3                  # drifts are uniform on (0, 4e-3): most rows stale
    W, hot, snap, sidx = problem(rng, T, R, D, H, S, L, 2e-3, hot_share=0.95)
    tb, hs = device_state(B, dev, W, hot, snap)
    B.ss_detect_stale(tb, hs, 0.0, refresh_snapshot=False)
    sidx_d = torch.from_numpy(sidx).to(dev)
    counts = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(max(256, B.ss_filter_batch_workspace_bytes(T, S, L)),
                     dtype=torch.uint8, device=dev)
    skip = torch.zeros(S, dtype=torch.uint8, device=dev)
    kept = torch.zeros(S, dtype=torch.int32, device=dev)
    nk = torch.zeros(1, dtype=torch.int32, device=dev)
    idx_c = torch.zeros((T, S, L), dtype=torch.int32, device=dev)
    by_sampling = {}
    for alpha in (1, 3, T * L):
        B.ss_sample_drop(hs, sidx_d, alpha, [thr], counts)
        by_sampling[alpha] = int(counts.item())
    B.ss_detect_stale(tb, hs, thr, refresh_snapshot=False)       # now set the bits
    for alpha in (1, 3, T * L):
        B.ss_filter_batch(tb, sidx_d, alpha, skip, kept, nk, idx_c, ws)
        assert S - int(nk.item()) == by_sampling[alpha]
    assert 0 < by_sampling[T * L] < by_sampling[3] <= by_sampling[1] <= S


def test_sampling_block_at_config3_shape_and_threshold_search(B, dev):
    """Full-size tables of config 3, a 0.1 % sample of a million-input pool
    rounded up to 1024 inputs, counts against the oracle on the compact problem
    (hot rows only: lookups elsewhere are never stale), then the search."""
    from paper_2404_04270_amd.sampling import SamplingBlock
    cfg = wl.CONFIGS[3]
    T, R, D, H = cfg.num_tables, cfg.rows, cfg.dim, cfg.hot_rows
    S = 1024
    w = wl.Workload(cfg)
    stream = w.indices(0, 3)                           # [3, T, B, 1]
    hot = wl.hot_set(stream[:2], R, H)
    sidx = np.ascontiguousarray(stream[2][:, :S])      # inputs the hot set has not seen
    rng = np.random.default_rng(970)
    weights = [w.weights_device(t, dev) for t in range(T)]
    tb = B.Tables(weights)
    tb.new_bits()
    hs = B.HotState(tb, [torch.from_numpy(h).to(dev) for h in hot])
    mini, snap = [], []
    for t in range(T):
        rows = weights[t][torch.from_numpy(hot[t]).to(dev).long()].cpu().numpy()
        scale = rng.lognormal(math.log(3e-4 / math.sqrt(D)), 1.0, (H, 1))
        s = (rows + scale * rng.choice([-1.0, 1.0], (H, D))).astype(np.float32)
        hs.snapshot[t].copy_(torch.from_numpy(s))
        mini.append(np.ascontiguousarray(rows))
        snap.append(s)
    # compact problem: hot row h of table t becomes row h; other rows become row H,
    # which is not hot
    mini = [np.vstack([m, np.zeros((1, D), np.float32)]) for m in mini]
    slot = [np.searchsorted(hot[t], sidx[t]) for t in range(T)]
    sidx_m = np.stack([np.where((slot[t] < H) & (hot[t][np.minimum(slot[t], H - 1)] == sidx[t]),
                                slot[t], H).astype(np.int32) for t in range(T)])
    hot_m = [np.arange(H, dtype=np.int32) for _ in range(T)]
    ladder = [float(np.float32(x)) for x in np.geomspace(3e-5, 3e-3, 32)]

    blk = SamplingBlock(tb, hs, torch.from_numpy(sidx).to(dev), alpha=T // 2,
                        population=1_000_000)
    blk.refresh_drift()
    got = blk.counts_for(ladder)
    ref = oracle.sample_drop(mini, hot_m, snap, np.ascontiguousarray(sidx_m), T // 2, ladder)
    assert got == [int(c) for c in ref]
    assert got[0] < got[-1] and all(a <= b for a, b in zip(got, got[1:]))

    est = blk.estimate(ladder[:4])
    for e, c in zip(est, ref[:4]):
        r = oracle.drop_stats(int(c), S, 1_000_000, 1_000_000, 3.340)
        for k in r:
            assert e[k] == pytest.approx(r[k], rel=1e-12, abs=1e-15)

    budget = 0.25
    T_found, tried = blk.find_threshold(budget, 3e-5, 3e-3)
    assert T_found is not None
    hi_at = {t: b for t, b in tried}
    assert hi_at[T_found] <= budget
    assert min(b for t, b in tried if t > T_found) > budget
    # what the oracle says about the threshold that was found
    c = oracle.sample_drop(mini, hot_m, snap, np.ascontiguousarray(sidx_m), T // 2,
                           [float(np.float32(T_found))])[0]
    assert oracle.drop_stats(int(c), S, 1_000_000, 1_000_000, 3.340)["hi"] <= budget
