"""Seeded random-geometry sweeps of the auxiliary calls (drift test, sampling
block, hot-set identification, feature normalization) against the CPU oracle.
Every input is valid; what varies is the shape: tile, wavefront and bitmap-word
boundaries, one-element extremes, counters that use all 32 bits.  The sweep of
the training step itself is in test_gpu_parity.py.
"""
import math

import numpy as np
import pytest
import torch

import oracle

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


def tables(rng, T, R, D):
    return [rng.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]


def hot_state(B, dev, rng, W, H, spread):
    """Ascending hot ids and snapshots whose drift is uniform on (0, spread)."""
    T, (R, D) = len(W), W[0].shape
    hot = [np.sort(rng.choice(R, H, replace=False)).astype(np.int32) for _ in range(T)]
    snap = [(W[t][hot[t]] + rng.uniform(0, spread / math.sqrt(D), (H, 1))
             * rng.choice([-1.0, 1.0], (H, D))).astype(np.float32) for t in range(T)]
    return hot, snap


def random_bits(rng, T, R, frac):
    out = []
    for _ in range(T):
        pad = np.zeros((R + 31) // 32 * 32, dtype=np.uint8)
        pad[:R] = rng.random(R) < frac
        out.append(np.packbits(pad, bitorder="little").view(np.uint32).copy())
    return out


def test_detect_random_shapes(B, dev):
    rng = np.random.default_rng(5001)
    for case in range(30):
        T = int(rng.integers(1, 6))
        R = int(rng.choice([1, 31, 64, 1000, 5000, 70000]))
        D = int(rng.choice([4, 16, 48, 64, 128, 260, 1024]))
        H = int(min(R, rng.choice([1, 2, 63, 64, 65, 300, 1000])))
        thr = float(rng.choice([0.0, 1e-3, 3e-3, math.inf]))
        refresh = bool(rng.integers(0, 2))
        tag = (case, T, R, D, H, thr, refresh)
        W = tables(rng, T, R, D)
        hot, snap = hot_state(B, dev, rng, W, H, 6e-3)
        bits0 = random_bits(rng, T, R, 0.1)
        tb = B.Tables(to_dev(W, dev), [torch.from_numpy(b.view(np.int32).copy()).to(dev)
                                       for b in bits0])
        hs = B.HotState(tb, to_dev(hot, dev))
        for t in range(T):
            hs.snapshot[t].copy_(torch.from_numpy(snap[t]))
        B.ss_detect_stale(tb, hs, thr, refresh)
        ref_bits = [b.copy() for b in bits0]
        ref_snap = [s.copy() for s in snap]
        r_sh, r_dr, r_cnt = oracle.detect_stale(W, ref_bits, hot, ref_snap, thr, refresh)
        for t in range(T):
            np.testing.assert_allclose(hs.drift[t].cpu().numpy(), r_dr[t], rtol=1e-12, atol=0,
                                       err_msg=str(tag))
            graded = (np.ones(H, bool) if not 0 < thr < math.inf
                      else np.abs(r_dr[t] - thr) > 1e-6 * thr)
            assert np.array_equal(hs.stale_hot[t].cpu().numpy()[graded], r_sh[t][graded]), tag
            if graded.all():
                assert np.array_equal(tb.bits[t].cpu().numpy().view(np.uint32), ref_bits[t]), tag
                assert int(hs.stale_count[t].item()) == int(r_cnt[t]), tag
            assert np.array_equal(hs.snapshot[t].cpu().numpy(), ref_snap[t]), tag


def test_sample_drop_random_shapes(B, dev):
    rng = np.random.default_rng(5002)
    for case in range(30):
        T = int(rng.integers(1, 30))
        R = int(rng.choice([10, 300, 5000]))
        D = int(rng.choice([4, 16, 64]))
        H = int(min(R, rng.choice([1, 2, 50, 333])))
        S = int(rng.choice([1, 2, 63, 64, 65, 500, 3000]))
        L = int(rng.choice([1, 1, 2, 20]))
        while T * S * L > 200000:
            S = max(1, S // 2)
        W = tables(rng, T, R, D)
        hot, snap = hot_state(B, dev, rng, W, H, 6e-3)
        sidx = np.stack([np.where(rng.random((S, L)) < 0.8, hot[t][rng.integers(0, H, (S, L))],
                                  rng.integers(0, R, (S, L))) for t in range(T)]).astype(np.int32)
        n_thr = int(rng.integers(1, 33))
        pool = [0.0, math.inf, 1e-9] + list(np.geomspace(1e-4, 9e-3, 40))
        ladder = [float(np.float32(x)) for x in rng.choice(pool, n_thr)]
        alpha = int(rng.choice([0, 1, 2, max(1, T * L // 3), T * L, T * L + 1]))
        tag = (case, T, R, D, H, S, L, alpha, n_thr)
        bits = [np.zeros((R + 31) // 32, np.uint32) for _ in W]
        _, drift, _ = oracle.detect_stale(W, bits, hot, [s.copy() for s in snap], 0.0, False)
        if any((np.abs(drift - t) <= 1e-6 * t).any() for t in ladder if 0 < t < math.inf):
            continue                         # a drift inside the band of a threshold
        tb = B.Tables(to_dev(W, dev))
        tb.new_bits()
        hs = B.HotState(tb, to_dev(hot, dev))
        for t in range(T):
            hs.snapshot[t].copy_(torch.from_numpy(snap[t]))
        B.ss_detect_stale(tb, hs, 0.0, False)
        counts = torch.full((32,), -1, dtype=torch.int32, device=dev)
        B.ss_sample_drop(hs, torch.from_numpy(sidx).to(dev), alpha, ladder, counts)
        ref = oracle.sample_drop(W, hot, snap, sidx, alpha, ladder)
        assert np.array_equal(counts.cpu().numpy()[:n_thr].view(np.uint32), ref), tag
        assert torch.all(counts[n_thr:] == -1), tag


def test_hot_set_random_shapes(B, dev):
    rng = np.random.default_rng(5003)
    for case in range(40):
        T = int(rng.integers(1, 5))
        R = int(rng.choice([1, 2, 63, 64, 65, 4095, 4096, 4097, 8193, 100000]))
        kind = str(rng.choice(["ties", "zipf", "wide", "flat", "zero"]))
        if kind == "ties":
            counts = [rng.integers(0, 4, R).astype(np.uint32) for _ in range(T)]
        elif kind == "zipf":
            counts = [(rng.zipf(1.3, R) % 70000).astype(np.uint32) for _ in range(T)]
        elif kind == "wide":
            counts = [rng.integers(0, 1 << 32, R, dtype=np.uint64).astype(np.uint32)
                      for _ in range(T)]
        elif kind == "flat":
            counts = [np.full(R, int(rng.integers(0, 1 << 32)), np.uint32) for _ in range(T)]
        else:
            counts = [np.zeros(R, np.uint32) for _ in range(T)]
        H = int(rng.integers(0, R + 1))
        tag = (case, T, R, kind, H)
        ac = B.AccessCounters(T, R, dev)
        for t in range(T):
            ac.counts[t].copy_(torch.from_numpy(counts[t].view(np.int32)))
        ws = torch.empty(max(256, B.ss_select_hot_workspace_bytes(T, R)), dtype=torch.uint8,
                         device=dev)
        ws.fill_(int(rng.integers(0, 256)))
        words = (R + 31) // 32
        ids = [torch.full((max(H, 1),), -7, dtype=torch.int32, device=dev) for _ in range(T)]
        bits = [torch.full((words,), -1, dtype=torch.int32, device=dev) for _ in range(T)]
        B.ss_select_hot_top(ac, H, ids, bits, ws)
        r_ids, r_bits = oracle.select_hot_top(counts, H)
        for t in range(T):
            assert np.array_equal(ids[t].cpu().numpy()[:H], r_ids[t]), tag
            assert np.array_equal(bits[t].cpu().numpy().view(np.uint32), r_bits[t]), tag
        lam = float(rng.choice([0.0, 1e-6, 1e-3, 0.01, 0.3, 1.0, 2.0]))
        total = int(rng.choice([1, 1000, 10 ** 6, 10 ** 9]))
        cap = int(rng.integers(1, R + 1))
        ids = [torch.full((cap,), -1, dtype=torch.int32, device=dev) for _ in range(T)]
        n_hot = torch.full((T,), -1, dtype=torch.int32, device=dev)
        B.ss_select_hot_ratio(ac, lam, total, ids, bits, n_hot, ws)
        q_ids, q_bits, q_n = oracle.select_hot_ratio(counts, lam, total, cap)
        assert np.array_equal(n_hot.cpu().numpy().view(np.uint32), q_n), tag + (lam, total)
        for t in range(T):
            assert np.array_equal(ids[t].cpu().numpy(), q_ids[t]), tag + (lam, total, cap)
            assert np.array_equal(bits[t].cpu().numpy().view(np.uint32), q_bits[t]), tag


def test_count_accesses_random_shapes(B, dev):
    rng = np.random.default_rng(5004)
    for case in range(25):
        T = int(rng.integers(1, 6))
        R = int(rng.choice([1, 7, 1000, 1 << 16, 10 ** 6]))
        Bn = int(rng.choice([1, 64, 2047, 2048, 2049, 9000]))
        L = int(rng.choice([1, 3, 20]))
        nv = int(rng.integers(0, Bn + 1))
        if rng.random() < 0.7:
            idx = ((rng.zipf(float(rng.choice([1.02, 1.3, 3.0])), (T, Bn, L)) - 1) % R)
        else:
            idx = rng.integers(0, R, (T, Bn, L))
        idx = idx.astype(np.int32)
        idx[:, nv:] = -1                         # must not be read
        ref = [rng.integers(0, 9, R).astype(np.uint32) for _ in range(T)]
        ac = B.AccessCounters(T, R, dev)
        for t in range(T):
            ac.counts[t].copy_(torch.from_numpy(ref[t].view(np.int32)))
        B.ss_count_accesses(ac, torch.from_numpy(idx).to(dev),
                            torch.tensor([nv], dtype=torch.int32, device=dev))
        oracle.count_accesses(R, idx, ref, nv)
        for t in range(T):
            assert np.array_equal(ac.counts[t].cpu().numpy().view(np.uint32), ref[t]), \
                (case, T, R, Bn, L, nv, t)


def test_layernorm_random_shapes(B, dev):
    rng = np.random.default_rng(5005)
    for case in range(30):
        T = int(rng.integers(1, 5))
        Bc = int(rng.choice([1, 15, 16, 17, 64, 129, 1000, 3000]))
        D = int(rng.choice([4, 8, 16, 48, 64, 128, 256, 260, 512, 1024]))
        while T * Bc * D > 4_000_000:
            Bc = max(1, Bc // 2)
        nv = int(rng.integers(0, Bc + 1))
        affine = bool(rng.integers(0, 2))
        tag = (case, T, Bc, D, nv, affine)
        x = (rng.normal(0.05, 1.0, (T, Bc, D))
             * rng.uniform(0.05, 3.0, (T, Bc, 1))).astype(np.float32)
        dy = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
        gamma = rng.normal(1, 0.3, (T, D)).astype(np.float32) if affine else None
        beta = rng.normal(0, 0.3, (T, D)).astype(np.float32) if affine else None

        def dv(a):
            return None if a is None else torch.from_numpy(a).to(dev)
        n_valid = torch.tensor([nv], dtype=torch.int32, device=dev)
        y = torch.full((T, Bc, D), 7.0, device=dev)
        mean = torch.full((T, Bc), 7.0, device=dev)
        rstd = torch.full((T, Bc), 7.0, device=dev)
        B.ss_layernorm_forward(dv(x), n_valid, dv(gamma), dv(beta), 1e-5, y, mean, rstd)
        r_y, r_m, r_r = oracle.layernorm_forward(x, gamma, beta, 1e-5, nv)
        np.testing.assert_allclose(y.cpu().numpy()[:, :nv], r_y[:, :nv], rtol=RTOL, atol=ATOL,
                                   err_msg=str(tag))
        np.testing.assert_allclose(rstd.cpu().numpy()[:, :nv], r_r[:, :nv], rtol=RTOL, atol=ATOL)
        assert torch.all(y[:, nv:] == 7.0), tag
        dx = torch.full((T, Bc, D), 7.0, device=dev)
        dg, db = torch.zeros(T, D, device=dev), torch.zeros(T, D, device=dev)
        ws = torch.empty(max(256, B.ss_layernorm_backward_workspace_bytes(T, D, Bc)),
                         dtype=torch.uint8, device=dev)
        ws.fill_(0xEE)
        B.ss_layernorm_backward(dv(dy), dv(x), n_valid, dv(gamma), mean, rstd, dx, dg, db, ws)
        r_dx, r_dg, r_db = oracle.layernorm_backward(dy, x, gamma, 1e-5, nv)
        np.testing.assert_allclose(dx.cpu().numpy()[:, :nv], r_dx[:, :nv], rtol=RTOL, atol=ATOL,
                                   err_msg=str(tag))
        assert torch.all(dx[:, nv:] == 7.0), tag
        sum_atol = ATOL + 1e-7 * math.sqrt(max(nv, 1)) * 0.05      # fp32 sum of nv terms
        np.testing.assert_allclose(dg.cpu().numpy(), r_dg, rtol=RTOL, atol=sum_atol,
                                   err_msg=str(tag))
        np.testing.assert_allclose(db.cpu().numpy(), r_db, rtol=RTOL, atol=sum_atol)
