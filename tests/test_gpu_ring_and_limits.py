"""GPU tests of the snapshot ring, the two halves of the update, argument
checking, and the limits of the table dimension (thousands of tiny tables, and
the largest table count the header allows), plus a sweep of seeded random
geometries through filter -> forward -> update against the CPU oracle.

Bars as everywhere: bit-exact masks, ids, compacted indices, verdicts, bitmaps
and counters; rtol 1e-5 / atol 1e-6 for fp32 outputs and weights.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2404_04270_amd import workload as wl  # noqa: F401  (seeded generators)

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-6

@pytest.fixture(scope="module")
def B():
    from paper_2404_04270_amd import binding
    return binding


@pytest.fixture(scope="module")
def dev():
    return torch.device("cuda:0")


def to_dev(arrs, dev):
    return [torch.from_numpy(np.ascontiguousarray(a)).to(dev) for a in arrs]


def bits_to_dev(bits, dev):
    return [torch.from_numpy(b.view(np.int32).copy()).to(dev) for b in bits]


def bits_from_dev(bits):
    return [b.cpu().numpy().view(np.uint32) for b in bits]


def rand_tables(rng, T, R, D):
    return [rng.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]


def zipf_idx(rng, T, B, L, R, a=1.2):
    return ((rng.zipf(a, (T, B, L)) - 1) % R).astype(np.int32)


def random_bits(rng, T, R, frac):
    out = []
    for _ in range(T):
        flags = rng.random(R) < frac
        pad = np.zeros((R + 31) // 32 * 32, dtype=np.uint8)
        pad[:R] = flags
        out.append(np.packbits(pad, bitorder="little").view(np.uint32).copy())
    return out



def test_prepare_then_apply_equals_update(B, dev):
    rng = np.random.default_rng(460)
    T, R, D, Bc, L = 3, 5000, 64, 3000, 2
    W = rand_tables(rng, T, R, D)
    idx = torch.from_numpy(zipf_idx(rng, T, Bc, L, R)).to(dev)
    grad = torch.from_numpy(rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)).to(dev)
    bits = random_bits(rng, T, R, 0.1)
    nv = torch.tensor([2500], dtype=torch.int32, device=dev)
    a = B.Tables(to_dev(W, dev), bits_to_dev(bits, dev))
    b = B.Tables(to_dev(W, dev), bits_to_dev(bits, dev))
    ws = torch.empty(B.ss_backward_workspace_bytes(T, Bc, L, D), dtype=torch.uint8, device=dev)
    B.ss_embbag_backward_update(a, idx, nv, grad, 0.01, ws)
    ws.fill_(0x5A)
    B.ss_embbag_backward_prepare(b, idx, nv, ws)
    B.ss_embbag_backward_apply(b, Bc, L, grad, 0.01, ws)
    for t in range(T):
        assert torch.equal(a.weights[t], b.weights[t])


# -------------------------------------------------------- error handling
def test_invalid_arguments_are_rejected_before_launch(B, dev):
    rng = np.random.default_rng(500)
    tb = B.Tables(to_dev(rand_tables(rng, 2, 100, 16), dev))
    idx = torch.zeros((2, 8, 1), dtype=torch.int32, device=dev)
    out = torch.zeros((2, 8, 16), dtype=torch.float32, device=dev)
    small = torch.empty(256, dtype=torch.uint8, device=dev)
    with pytest.raises(B.SlipstreamError, match="workspace"):
        B.ss_embbag_backward_update(tb, idx, None, out, 0.01, small)
    hs = B.HotState(tb, [torch.zeros(4, dtype=torch.int32, device=dev)] * 2)
    with pytest.raises(B.SlipstreamError, match="stale_bits"):
        B.ss_detect_stale(tb, hs, 1e-3, True)
    bad = B.Tables(to_dev(rand_tables(rng, 1, 10, 6), dev))
    with pytest.raises(B.SlipstreamError, match="dim"):
        B.ss_embbag_forward(bad, torch.zeros((1, 2, 1), dtype=torch.int32, device=dev),
                            None, torch.zeros((1, 2, 6), dtype=torch.float32, device=dev))
    torch.cuda.synchronize()


# ------------------------------------------------------- snapshot ring
@pytest.mark.parametrize("depth,lag", [(1, 1), (3, 3), (3, 1), (4, 2)])
def test_snapshot_ring_compares_with_the_right_snapshot(B, dev, depth, lag):
    """N temporal snapshots (section 3.1.2): the drift is taken against the
    snapshot `lag` periods back, here checked against the oracle fed with that
    snapshot from a plain host-side history."""
    from paper_2404_04270_amd.step import SnapshotRing
    rng = np.random.default_rng(700 + depth * 10 + lag)
    T, R, D, H = 2, 1500, 32, 300
    W = rand_tables(rng, T, R, D)
    hot = [np.sort(rng.choice(R, H, replace=False)).astype(np.int32) for _ in range(T)]
    tb = B.Tables(to_dev(W, dev))
    tb.new_bits()
    ring = SnapshotRing(tb, to_dev(hot, dev), depth)
    history = []                                  # host copies of every snapshot taken
    ref_bits = [np.zeros((R + 31) // 32, np.uint32) for _ in range(T)]
    thr = 2e-3
    for period in range(depth + 4):
        # the tables move: shrinking steps, so that later periods flag more rows
        step = 4e-3 / (1 + period) / math.sqrt(D)
        for t in range(T):
            W[t][hot[t]] += (step * rng.uniform(0, 1, (H, 1))
                             * rng.choice([-1.0, 1.0], (H, D))).astype(np.float32)
            tb.weights[t].copy_(torch.from_numpy(W[t]))
        if ring.pushed < lag:
            ring.push()
            history.append([W[t][hot[t]].copy() for t in range(T)])
            continue
        snap = [s.copy() for s in history[-lag]]
        r_sh, r_dr, _ = oracle.detect_stale(W, ref_bits, hot, snap, thr, refresh=False)
        slot = ring.detect(thr, lag=lag)
        history.append([W[t][hot[t]].copy() for t in range(T)])
        for t in range(T):
            np.testing.assert_allclose(slot.drift[t].cpu().numpy(), r_dr[t], rtol=1e-12)
            graded = np.abs(r_dr[t] - thr) > 1e-6 * thr
            assert graded.sum() > 0.99 * H
            assert np.array_equal(slot.stale_hot[t].cpu().numpy()[graded], r_sh[t][graded])
            if graded.all():
                assert np.array_equal(bits_from_dev(tb.bits)[t], ref_bits[t])
        # the ring now holds the last `depth` snapshots, newest first by lag
        for k in range(1, min(depth, ring.pushed) + 1):
            for t in range(T):
                assert np.array_equal(ring._slot(k).snapshot[t].cpu().numpy(), history[-k][t])
    assert sum(int(b.sum()) for b in ref_bits) > 0
    with pytest.raises(ValueError):
        ring._slot(depth + 1)


# ------------------------------------------------------- many small tables
def test_every_call_with_two_thousand_tables(B, dev):
    """Grids are laid out as tables x tiles: a model with thousands of tiny
    tables exercises the table dimension of every launch (the limit is 65535)."""
    rng = np.random.default_rng(800)
    T, R, D, Bn, L, H = 2000, 37, 8, 70, 2, 5
    W = rand_tables(rng, T, R, D)
    idx = zipf_idx(rng, T, Bn, L, R)
    bits = random_bits(rng, T, R, 0.2)
    tb = B.Tables(to_dev(W, dev), bits_to_dev(bits, dev))
    idx_d = torch.from_numpy(idx).to(dev)
    # filter
    alpha = T * L // 5
    skip = torch.zeros(Bn, dtype=torch.uint8, device=dev)
    kept = torch.zeros(Bn, dtype=torch.int32, device=dev)
    nk = torch.zeros(1, dtype=torch.int32, device=dev)
    idx_c = torch.zeros((T, Bn, L), dtype=torch.int32, device=dev)
    ws_f = torch.empty(max(256, B.ss_filter_batch_workspace_bytes(T, Bn, L)),
                       dtype=torch.uint8, device=dev)
    B.ss_filter_batch(tb, idx_d, alpha, skip, kept, nk, idx_c, ws_f)
    r_skip, r_kept, r_idx_c = oracle.filter_batch(R, bits, idx, alpha)
    n = int(nk.item())
    assert n == len(r_kept) and 0 < n < Bn
    assert np.array_equal(skip.cpu().numpy(), r_skip)
    assert np.array_equal(idx_c.cpu().numpy()[:, :n], r_idx_c[:, :n])
    # forward
    out = torch.zeros((T, Bn, D), dtype=torch.float32, device=dev)
    B.ss_embbag_forward(tb, idx_c, nk, out)
    ref = oracle.embbag_forward(W, r_idx_c, n)
    np.testing.assert_allclose(out.cpu().numpy()[:, :n], ref[:, :n], rtol=RTOL, atol=ATOL)
    # backward
    grad = rng.normal(0, 0.01, (T, Bn, D)).astype(np.float32)
    ws_b = torch.empty(B.ss_backward_workspace_bytes(T, Bn, L, D), dtype=torch.uint8, device=dev)
    B.ss_embbag_backward_update(tb, idx_c, nk, torch.from_numpy(grad).to(dev), 0.05, ws_b)
    ref_w = [w.copy() for w in W]
    oracle.embbag_backward_update(ref_w, bits, r_idx_c, grad, 0.05, n)
    for t in range(0, T, 97):
        np.testing.assert_allclose(tb.weights[t].cpu().numpy(), ref_w[t], rtol=RTOL, atol=ATOL)
    # detect
    hot = [np.sort(rng.choice(R, H, replace=False)).astype(np.int32) for _ in range(T)]
    hs = B.HotState(tb, to_dev(hot, dev))
    snap = [(ref_w[t][hot[t]] + rng.normal(0, 1e-3, (H, D))).astype(np.float32) for t in range(T)]
    for t in range(T):
        hs.snapshot[t].copy_(torch.from_numpy(snap[t]))
    W_now = [w.cpu().numpy() for w in tb.weights]
    ref_bits = [b.copy() for b in bits]
    r_sh, r_dr, r_cnt = oracle.detect_stale(W_now, ref_bits, hot, [s.copy() for s in snap],
                                            3e-3, True)
    B.ss_detect_stale(tb, hs, 3e-3, True)
    got_bits = bits_from_dev(tb.bits)
    for t in range(T):
        if (np.abs(r_dr[t] - 3e-3) > 1e-6 * 3e-3).all():
            assert np.array_equal(got_bits[t], ref_bits[t])
    assert 0 < int(r_cnt.sum()) < T * H
    # counters and hot set
    ac = B.AccessCounters(T, R, dev)
    B.ss_count_accesses(ac, idx_d)
    cnt = [np.zeros(R, np.uint32) for _ in range(T)]
    oracle.count_accesses(R, idx, cnt)
    ids = [torch.zeros(H, dtype=torch.int32, device=dev) for _ in range(T)]
    ws_s = torch.empty(max(256, B.ss_select_hot_workspace_bytes(T, R)), dtype=torch.uint8,
                       device=dev)
    B.ss_select_hot_top(ac, H, ids, None, ws_s)
    r_ids, _ = oracle.select_hot_top(cnt, H)
    for t in range(T):
        assert np.array_equal(ac.counts[t].cpu().numpy().view(np.uint32), cnt[t])
        assert np.array_equal(ids[t].cpu().numpy(), r_ids[t])


# ------------------------------------------------------------ random shapes
def test_random_small_shapes_through_the_whole_step(B, dev):
    """Forty seeded random geometries (tables, rows, dim, batch, bag, stale share,
    valid count, alpha), each run filter -> forward -> backward against the
    oracle: ragged tiles, strips and classes of every kind in one sweep."""
    rng = np.random.default_rng(4242)
    for case in range(40):
        T = int(rng.integers(1, 7))
        R = int(rng.choice([1, 2, 31, 64, 65, 1000, 4097, 70000]))
        D = int(rng.choice([4, 8, 16, 32, 48, 64, 128, 200, 256, 512]))
        L = int(rng.choice([1, 1, 1, 2, 3, 7, 20]))
        Bn = int(rng.choice([1, 2, 63, 64, 65, 255, 256, 257, 1000, 2049]))
        if Bn * L > 20000:
            Bn = 20000 // L
        frac = float(rng.choice([0.0, 0.05, 0.5, 0.95]))
        za = float(rng.choice([1.05, 1.2, 2.0]))
        W = rand_tables(rng, T, R, D)
        idx = zipf_idx(rng, T, Bn, L, R, za)
        bits = random_bits(rng, T, R, frac) if frac > 0 else None
        alpha = int(rng.choice([1, max(1, T * L // 2), T * L, T * L + 1]))
        tag = (case, T, R, D, L, Bn, frac, za, alpha)
        tb = B.Tables(to_dev(W, dev), None if bits is None else bits_to_dev(bits, dev))
        idx_d = torch.from_numpy(idx).to(dev)
        skip = torch.zeros(Bn, dtype=torch.uint8, device=dev)
        kept = torch.zeros(Bn, dtype=torch.int32, device=dev)
        nk = torch.zeros(1, dtype=torch.int32, device=dev)
        idx_c = torch.full((T, Bn, L), -1, dtype=torch.int32, device=dev)
        ws_f = torch.empty(max(256, B.ss_filter_batch_workspace_bytes(T, Bn, L)),
                           dtype=torch.uint8, device=dev)
        B.ss_filter_batch(tb, idx_d, alpha, skip, kept, nk, idx_c, ws_f)
        r_skip, r_kept, r_idx_c = oracle.filter_batch(R, bits, idx, alpha)
        n = int(nk.item())
        assert n == len(r_kept), tag
        assert np.array_equal(skip.cpu().numpy(), r_skip), tag
        assert np.array_equal(idx_c.cpu().numpy()[:, :n], r_idx_c[:, :n]), tag
        out = torch.full((T, Bn, D), 3.0, dtype=torch.float32, device=dev)
        B.ss_embbag_forward(tb, idx_c, nk, out)
        ref = oracle.embbag_forward(W, r_idx_c, n)
        np.testing.assert_allclose(out.cpu().numpy()[:, :n], ref[:, :n], rtol=RTOL, atol=ATOL,
                                   err_msg=str(tag))
        assert torch.all(out[:, n:] == 3.0), tag
        grad = rng.normal(0, 0.01, (T, Bn, D)).astype(np.float32)
        ws_b = torch.empty(B.ss_backward_workspace_bytes(T, Bn, L, D), dtype=torch.uint8,
                           device=dev)
        B.ss_embbag_backward_update(tb, idx_c, nk, torch.from_numpy(grad).to(dev), 0.02, ws_b)
        ref_w = [w.copy() for w in W]
        oracle.embbag_backward_update(ref_w, bits, r_idx_c, grad, 0.02, n)
        for t in range(T):
            np.testing.assert_allclose(tb.weights[t].cpu().numpy(), ref_w[t], rtol=RTOL,
                                       atol=ATOL, err_msg=str(tag))


def test_the_largest_number_of_tables(B, dev):
    """65535 tables (the limit of the table dimension of a launch), two rows each:
    filter, forward, update and the hot-set calls still address every table."""
    rng = np.random.default_rng(810)
    T, R, D, Bn, L = 65535, 2, 4, 3, 1
    Wall = rng.uniform(-0.05, 0.05, (T, R, D)).astype(np.float32)
    W = [Wall[t] for t in range(T)]
    idx = rng.integers(0, R, (T, Bn, L)).astype(np.int32)
    big = torch.from_numpy(Wall).to(dev)
    tb = B.Tables([big[t] for t in range(T)])            # views of one allocation
    idx_d = torch.from_numpy(idx).to(dev)
    out = torch.zeros((T, Bn, D), dtype=torch.float32, device=dev)
    B.ss_embbag_forward(tb, idx_d, None, out)
    assert np.array_equal(out.cpu().numpy(), Wall[np.arange(T)[:, None], idx[:, :, 0]])
    grad = rng.normal(0, 0.01, (T, Bn, D)).astype(np.float32)
    ws_b = torch.empty(B.ss_backward_workspace_bytes(T, Bn, L, D), dtype=torch.uint8, device=dev)
    B.ss_embbag_backward_update(tb, idx_d, None, torch.from_numpy(grad).to(dev), 0.05, ws_b)
    ref_w = [w.copy() for w in W]
    oracle.embbag_backward_update(ref_w, None, idx, grad, 0.05)
    np.testing.assert_allclose(big.cpu().numpy(), np.stack(ref_w), rtol=RTOL, atol=ATOL)
    # no bitmaps: the filter keeps everything
    skip = torch.ones(Bn, dtype=torch.uint8, device=dev)
    kept = torch.zeros(Bn, dtype=torch.int32, device=dev)
    nk = torch.zeros(1, dtype=torch.int32, device=dev)
    idx_c = torch.zeros((T, Bn, L), dtype=torch.int32, device=dev)
    ws_f = torch.empty(max(256, B.ss_filter_batch_workspace_bytes(T, Bn, L)),
                       dtype=torch.uint8, device=dev)
    B.ss_filter_batch(tb, idx_d, T * L, skip, kept, nk, idx_c, ws_f)
    assert int(nk.item()) == Bn and torch.equal(idx_c, idx_d)
    # counters and the most accessed row of every table
    cnt_all = torch.zeros((T, R), dtype=torch.int32, device=dev)
    ac = B.AccessCounters(T, R, dev, counts=[cnt_all[t] for t in range(T)])
    B.ss_count_accesses(ac, idx_d)
    want = np.stack([np.bincount(idx[t].ravel(), minlength=R) for t in range(T)])
    assert np.array_equal(cnt_all.cpu().numpy(), want)
    ids_all = torch.full((T, 1), -1, dtype=torch.int32, device=dev)
    ws_s = torch.empty(max(256, B.ss_select_hot_workspace_bytes(T, R)), dtype=torch.uint8,
                       device=dev)
    B.ss_select_hot_top(ac, 1, [ids_all[t] for t in range(T)], None, ws_s)
    assert np.array_equal(ids_all.cpu().numpy()[:, 0], np.argmax(want, axis=1))

