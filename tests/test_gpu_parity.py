"""GPU parity: every call of the C ABI against the CPU oracle on the same
seeded inputs, element by element.

Bars: bit-exact for skip masks, kept ids, compacted indices, stale verdicts and
bitmaps (rows whose drift lies within 1e-6 relative of the threshold are left
out of the verdict check); rtol 1e-5 / atol 1e-6 for fp32 pooled outputs and
updated weights.  Sizes span several tiles, ragged tails, both sort paths and
all strip lengths of the update kernel.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle.protocol import OracleRun
from paper_2404_04270_amd import workload as wl

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


# --------------------------------------------------------------- forward
@pytest.mark.parametrize("T,R,D,Bc,L,nv", [
    (3, 1000, 16, 700, 1, None),     # one-hot, ragged tile
    (2, 5000, 64, 1025, 1, 999),     # n_valid below capacity
    (2, 3000, 128, 333, 20, None),   # multi-hot with duplicates
    (1, 200, 4, 70, 3, 0),           # nothing valid
    (2, 500, 48, 130, 9, 77),        # dim not a power of two, unroll tail
    (1, 300, 260, 40, 11, None),     # dim above 256: several float4 per lane
    (2, 400, 16, 300, 1, 0),         # one-hot, nothing valid
    (1, 300, 260, 40, 1, 33),        # one-hot, dim above 256
    (3, 700, 48, 1000, 1, 333),      # one-hot, dim not a power of two
    (8, 3000, 16, 70000, 1, 65000),  # one-hot pipeline: 2-3 batches per workgroup
    (26, 5000, 64, 8269, 1, None),   # 3-4 batches per workgroup, ragged last tile
    (26, 5000, 64, 14000, 1, 13999), # 5-6 batches per workgroup
    (2, 3000, 128, 100, 31, None),   # multi-hot: every piece size at once (16+8+4+2+1)
    (2, 3000, 64, 90, 32, 80),       # one full round of 16, then a piece of 16
    (1, 2000, 32, 60, 53, None),     # two full rounds, then 16+4+1
    (2, 500, 48, 50, 40, None),      # long bags, dim not a power of two
    (2, 900, 256, 37, 2, None),      # 64 lanes per row
    (1, 900, 8, 300, 7, None),       # two lanes per row
    (1, 900, 4, 300, 17, None),      # one lane per row
    (2, 3000, 128, 64, 16, None),    # exactly one piece
    (11, 3000, 64, 300, 5, None),    # multi-hot: eight tables pinned to XCDs, three spread
    (16, 2000, 32, 200, 20, 150),    # ... all pinned, two tables per XCD
    (26, 1000, 16, 150, 3, None),    # ... 24 pinned, two spread
])
def test_forward_matches_oracle(B, dev, T, R, D, Bc, L, nv):
    rng = np.random.default_rng(100 + D + L)
    W = rand_tables(rng, T, R, D)
    idx = zipf_idx(rng, T, Bc, L, R)
    if nv is not None:
        idx[:, nv:] = -1             # bags past n_valid hold no usable index
    ref = oracle.embbag_forward(W, idx, nv)
    tb = B.Tables(to_dev(W, dev))
    out = torch.full((T, Bc, D), 7.0, dtype=torch.float32, device=dev)
    n_valid = None if nv is None else torch.tensor([nv], dtype=torch.int32, device=dev)
    B.ss_embbag_forward(tb, torch.from_numpy(idx).to(dev), n_valid, out)
    got = out.cpu().numpy()
    n = Bc if nv is None else nv
    if L == 1:
        assert np.array_equal(got[:, :n], ref[:, :n])          # pure gather
    else:
        np.testing.assert_allclose(got[:, :n], ref[:, :n], rtol=RTOL, atol=ATOL)
    assert np.all(got[:, n:] == 7.0)                           # tail untouched


# ---------------------------------------------------------------- filter
@pytest.mark.parametrize("T,R,Bn,L,frac", [
    (3, 2000, 1000, 1, 0.5), (8, 500, 257, 2, 0.9), (2, 100, 5, 20, 0.97),
    (26, 4000, 4100, 1, 0.8),
    (5, 2000, 300, 20, 0.95),     # 100 lookups per sample: 16 lanes each
    (8, 3000, 700, 20, 0.9),      # 160: 32 lanes
    (26, 1000, 200, 16, 0.97),    # 416: a whole wavefront per sample
    (16, 500, 90, 40, 0.98),      # 640: more than one round of probes per lane; 8 copy parts
    (2, 5000, 70000, 1, 0.7),     # many tiles of samples
    (1, 64, 3000, 7, 0.9),        # one table
])
def test_filter_matches_oracle(B, dev, T, R, Bn, L, frac):
    rng = np.random.default_rng(200 + T + L)
    idx = zipf_idx(rng, T, Bn, L, R)
    bits = random_bits(rng, T, R, frac)
    W = to_dev(rand_tables(rng, T, R, 4), dev)
    tb = B.Tables(W, bits_to_dev(bits, dev))
    ws = torch.empty(max(256, B.ss_filter_batch_workspace_bytes(T, Bn, L)),
                     dtype=torch.uint8, device=dev)
    idx_d = torch.from_numpy(idx).to(dev)
    for alpha in sorted({0, 1, T * L // 2, T * L - 1, T * L, T * L + 1}):
        skip = torch.zeros(Bn, dtype=torch.uint8, device=dev)
        kept = torch.full((Bn,), -1, dtype=torch.int32, device=dev)
        nk = torch.full((1,), -1, dtype=torch.int32, device=dev)
        idx_c = torch.full((T, Bn, L), -1, dtype=torch.int32, device=dev)
        B.ss_filter_batch(tb, idx_d, alpha, skip, kept, nk, idx_c, ws)
        r_skip, r_kept, r_idx_c = oracle.filter_batch(R, bits, idx, alpha)
        n = int(nk.item())
        assert n == len(r_kept), alpha
        assert np.array_equal(skip.cpu().numpy(), r_skip)
        assert np.array_equal(kept.cpu().numpy()[:n], r_kept)
        assert np.all(kept.cpu().numpy()[n:] == -1)
        got_c = idx_c.cpu().numpy()
        assert np.array_equal(got_c[:, :n], r_idx_c[:, :n])
        assert np.all(got_c[:, n:] == -1)


def test_filter_without_bitmaps_keeps_everything(B, dev):
    T, R, Bn, L = 4, 100, 300, 2
    rng = np.random.default_rng(210)
    idx = zipf_idx(rng, T, Bn, L, R)
    tb = B.Tables(to_dev(rand_tables(rng, T, R, 4), dev))
    ws = torch.empty(256, dtype=torch.uint8, device=dev)
    skip = torch.ones(Bn, dtype=torch.uint8, device=dev)
    kept = torch.zeros(Bn, dtype=torch.int32, device=dev)
    nk = torch.zeros(1, dtype=torch.int32, device=dev)
    idx_c = torch.zeros((T, Bn, L), dtype=torch.int32, device=dev)
    B.ss_filter_batch(tb, torch.from_numpy(idx).to(dev), T * L, skip, kept, nk, idx_c, ws)
    assert int(nk.item()) == Bn and not skip.any()
    assert np.array_equal(kept.cpu().numpy(), np.arange(Bn))
    assert np.array_equal(idx_c.cpu().numpy(), idx)


# ---------------------------------------------------------------- detect
def run_detect(B, dev, W, bits, hot, snap, thr, refresh):
    tb = B.Tables(to_dev(W, dev), bits_to_dev(bits, dev))
    hs = B.HotState(tb, to_dev(hot, dev))
    for t in range(len(W)):
        hs.snapshot[t].copy_(torch.from_numpy(snap[t]))
    B.ss_detect_stale(tb, hs, thr, refresh)
    torch.cuda.synchronize()
    return tb, hs


@pytest.mark.parametrize("T,R,D,H,thr", [
    (3, 5000, 16, 700, 2e-3), (2, 3000, 64, 333, 4e-3), (2, 4000, 128, 65, 6e-3),
    (1, 900, 260, 50, 8e-3), (2, 2000, 4, 1000, 1e-3),
])
def test_detect_matches_oracle(B, dev, T, R, D, H, thr):
    rng = np.random.default_rng(300 + D)
    W = rand_tables(rng, T, R, D)
    hot = [np.sort(rng.choice(R, H, replace=False)).astype(np.int32) for _ in range(T)]
    # snapshot = rows plus noise whose norm straddles the threshold
    snap = []
    for t in range(T):
        scale = rng.uniform(0, 2 * thr / math.sqrt(D), (H, 1))
        snap.append((W[t][hot[t]] + scale * rng.choice([-1.0, 1.0], (H, D))).astype(np.float32))
    bits0 = random_bits(rng, T, R, 0.01)
    for refresh in (False, True):
        bits_ref = [b.copy() for b in bits0]
        snap_ref = [s.copy() for s in snap]
        r_sh, r_dr, r_cnt = oracle.detect_stale(W, bits_ref, hot, snap_ref, thr, refresh)
        tb, hs = run_detect(B, dev, W, bits0, hot, snap, thr, refresh)
        for t in range(T):
            dr = hs.drift[t].cpu().numpy()
            np.testing.assert_allclose(dr, r_dr[t], rtol=1e-12, atol=0)
            graded = np.abs(r_dr[t] - thr) > 1e-6 * thr
            assert graded.sum() > 0.9 * H
            sh = hs.stale_hot[t].cpu().numpy()
            assert np.array_equal(sh[graded], r_sh[t][graded])
            assert 0 < r_sh[t].sum() < H
            if graded.all():
                assert np.array_equal(bits_from_dev(tb.bits)[t], bits_ref[t])
                assert int(hs.stale_count[t].item()) == int(r_cnt[t])
            assert np.array_equal(hs.snapshot[t].cpu().numpy(), snap_ref[t])


def test_detect_threshold_zero_captures_and_infinity_flags_all(B, dev):
    rng = np.random.default_rng(310)
    T, R, D, H = 2, 1000, 16, 100
    W = rand_tables(rng, T, R, D)
    hot = [np.sort(rng.choice(R, H, replace=False)).astype(np.int32) for _ in range(T)]
    snap = [np.zeros((H, D), np.float32) for _ in range(T)]
    bits = [np.zeros((R + 31) // 32, np.uint32) for _ in range(T)]
    tb, hs = run_detect(B, dev, W, bits, hot, snap, 0.0, True)      # capture
    for t in range(T):
        assert not bits_from_dev(tb.bits)[t].any()
        assert np.array_equal(hs.snapshot[t].cpu().numpy(), W[t][hot[t]])
        assert int(hs.stale_count[t].item()) == 0
    B.ss_detect_stale(tb, hs, math.inf, False)
    ref_bits = [b.copy() for b in bits]
    oracle.detect_stale(W, ref_bits, hot, [W[t][hot[t]].copy() for t in range(T)],
                        math.inf, False)
    for t in range(T):
        assert np.array_equal(bits_from_dev(tb.bits)[t], ref_bits[t])
        assert int(hs.stale_count[t].item()) == H


# -------------------------------------------------------------- backward
BACKWARD_CASES = [
    # T, R, D, Bcap, L, n_valid, stale fraction, zipf a
    (3, 1000, 16, 700, 1, None, 0.0, 1.2),      # LDS sort, strip 4, D=16
    (2, 50000, 64, 8192, 1, None, 0.1, 1.2),    # LDS sort at 8192 lookups
    (2, 3000, 128, 300, 20, 250, 0.2, 1.2),     # multi-hot, ragged n_valid
    (1, 100, 64, 4096, 4, None, 0.0, 1.05),     # few rows: runs cross workgroups
    (2, 1 << 20, 64, 40000, 1, 39999, 0.05, 1.1),   # global radix sort path
    (1, 70000, 128, 5000, 20, None, 0.1, 1.2),  # global sort + heavy duplicates
    (26, 100000, 64, 8192, 1, None, 0.0, 1.2),  # many workgroups: strip 4
    (8, 200000, 128, 4096, 20, None, 0.02, 1.2),  # strip 8, global sort, tables pinned to XCDs
    (1, 3, 16, 3000, 1, None, 0.0, 1.5),        # three rows only
    (1, 500, 48, 200, 3, None, 0.3, 1.3),       # dim not a power of two
    (1, 300, 260, 100, 2, None, 0.3, 1.3),      # dim above 256
    (2, 400, 4, 5000, 1, 0, 0.0, 1.2),          # nothing valid
    (1, 1, 4, 1, 1, None, 0.0, 1.2),            # one table, one row, one sample
    (2, 9000, 64, 16384, 1, None, 0.05, 1.2),   # largest table the one-launch sort takes
    (2, 9000, 64, 16385, 1, None, 0.05, 1.2),   # one more: global radix sort
    (1, 5000, 32, 2048, 8, 2047, 1.0, 1.2),     # every row stale: nothing may move
    (3, 70000, 16, 2049, 1, 1, 0.0, 1.2),       # a single valid sample
    (4, 64, 64, 1000, 20, None, 0.05, 1.2),     # global sort, rows a power of two: the
    (1, 1024, 16, 20000, 1, None, 0.3, 1.05),   # last row id shares its low bits with
    (2, 1 << 20, 16, 17000, 1, None, 0.2, 1.02),  # the key of dropped lookups
    (2, 3000, 8, 700, 3, None, 0.1, 1.2),       # two lanes per row
    (2, 3000, 256, 300, 5, None, 0.1, 1.2),     # 64 lanes per row, filled exactly
    (1, 2000, 512, 200, 3, 150, 0.1, 1.2),      # two float4 per lane
    (16, 5000, 128, 600, 20, None, 0.1, 1.2),   # multi-hot: tables pinned to XCDs
    (11, 5000, 32, 500, 4, None, 0.1, 1.2),     # ... eight pinned, three spread
    (2, 100000, 8, 250000, 4, 249000, 0.05, 1.1),   # a million lookups per table: 489 sort
    (1, 2000000, 4, 1 << 20, 1, None, 0.0, 1.05),   # tiles; one lane per row, three passes
    # one global pass, then every bucket sorted in LDS (more than a million rows, and the
    # row bits left + the sample number fit one word): 32, 64 and 128 buckets per table
    (3, 3000000, 16, 4096, 6, None, 0.1, 1.2),
    (2, 1500000, 8, 30000, 2, 29000, 0.3, 1.05),
    (2, 10000000, 16, 4096, 20, None, 0.02, 1.2),   # its hottest row alone has 15 000 lookups
    (2, 4194303, 8, 20000, 1, None, 0.5, 1.1),      # the last row id is all ones below bit 22
    (1, 100000000, 4, 512, 40, None, 0.0, 3.0),     # 27 row bits, 22 of them left to the
                                                    # bucket sort; one row has four fifths
                                                    # of the lookups
]


@pytest.mark.parametrize("T,R,D,Bc,L,nv,stale,za", BACKWARD_CASES)
def test_backward_update_matches_oracle(B, dev, T, R, D, Bc, L, nv, stale, za):
    rng = np.random.default_rng(400 + T * 7 + D + L + Bc)
    W = rand_tables(rng, T, R, D)
    idx = zipf_idx(rng, T, Bc, L, R, za)
    grad = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
    bits = random_bits(rng, T, R, stale) if stale > 0 else None
    if bits is not None:
        for b in bits:
            b[0] |= np.uint32(3)               # freeze the two hottest rows too
    ref = [w.copy() for w in W]
    oracle.embbag_backward_update(ref, bits, idx, grad, 0.01, nv)

    tb = B.Tables(to_dev(W, dev), None if bits is None else bits_to_dev(bits, dev))
    ws = torch.empty(B.ss_backward_workspace_bytes(T, Bc, L, D), dtype=torch.uint8, device=dev)
    ws.fill_(0xAB)                              # contents on entry are ignored
    n_valid = None if nv is None else torch.tensor([nv], dtype=torch.int32, device=dev)
    idx_d = torch.from_numpy(idx).to(dev)
    grad_d = torch.from_numpy(grad).to(dev)
    B.ss_embbag_backward_update(tb, idx_d, n_valid, grad_d, 0.01, ws)
    got = [w.cpu().numpy() for w in tb.weights]
    n = Bc if nv is None else nv
    for t in range(T):
        np.testing.assert_allclose(got[t], ref[t], rtol=RTOL, atol=ATOL)
        touched = np.zeros(R, bool)
        touched[idx[t, :n].reshape(-1)] = True
        if bits is not None:
            flags = np.unpackbits(bits[t].view(np.uint8), bitorder="little")[:R].astype(bool)
            touched &= ~flags
            assert np.array_equal(bits_from_dev(tb.bits)[t], bits[t])
        # rows that must not move are bit-identical, rows that must move did
        assert np.array_equal(got[t][~touched], W[t][~touched])
        if touched.any():
            moved = np.any(got[t][touched] != W[t][touched], axis=1)
            assert moved.mean() > 0.99

    # same call again on fresh tables: bit-identical (fixed summation order)
    tb2 = B.Tables(to_dev(W, dev), None if bits is None else bits_to_dev(bits, dev))
    ws.fill_(0x11)
    B.ss_embbag_backward_update(tb2, idx_d, n_valid, grad_d, 0.01, ws)
    for t in range(T):
        assert torch.equal(tb2.weights[t], tb.weights[t])


@pytest.mark.parametrize("T,D,Bc,L,per_row", [(4, 64, 16000, 1, 600), (8, 128, 3000, 20, 700),
                                             (5, 64, 12000, 1, 520), (3, 16, 30000, 1, 2100)])
def test_backward_many_runs_that_cross_several_workgroups(B, dev, T, D, Bc, L, per_row):
    """Rows with `per_row` lookups each, side by side in the grouped list: every run
    leaves its workgroup, most cover about nine of them (just past what a lane group
    of the fixup stage finishes alone), so that one fixup workgroup queues several."""
    rng = np.random.default_rng(455 + T)
    R = 5000
    W = rand_tables(rng, T, R, D)
    flat = (np.arange(Bc * L) // per_row).astype(np.int32)
    idx = np.stack([rng.permutation(flat).reshape(Bc, L) + 3 * t for t in range(T)]).astype(np.int32)
    grad = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
    ref = [w.copy() for w in W]
    oracle.embbag_backward_update(ref, None, idx, grad, 0.01, None)
    tb = B.Tables(to_dev(W, dev))
    ws = torch.empty(B.ss_backward_workspace_bytes(T, Bc, L, D), dtype=torch.uint8, device=dev)
    B.ss_embbag_backward_update(tb, torch.from_numpy(idx).to(dev), None,
                                torch.from_numpy(grad).to(dev), 0.01, ws)
    for t in range(T):
        np.testing.assert_allclose(tb.weights[t].cpu().numpy(), ref[t], rtol=RTOL, atol=ATOL)


@pytest.mark.parametrize("D,L", [(64, 1), (128, 6), (16, 1), (320, 2)])
def test_backward_runs_across_workgroups_are_reproducible(B, dev, D, L):
    """Runs of every length from 1 to several thousand lookups, many of them across
    workgroup borders.  The pieces of such a run are added in a fixed order: 40 calls
    give the same bits, they match the oracle, and a second update stage on the same
    prepared workspace gives the same bits again."""
    rng = np.random.default_rng(4600 + D + L)
    T, R, Bc = 6, 40000, 24000 // L
    W = rand_tables(rng, T, R, D)
    lens = np.concatenate([rng.integers(1, 6, 3000), rng.integers(30, 400, 60),
                           rng.integers(1000, 5000, 3)])
    rows = np.repeat(rng.permutation(R)[:lens.size], lens)
    idx = np.stack([np.resize(rng.permutation(rows), Bc * L).reshape(Bc, L)
                    for _ in range(T)]).astype(np.int32)
    grad = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
    ref = [w.copy() for w in W]
    oracle.embbag_backward_update(ref, None, idx, grad, 0.01, None)
    idx_d, grad_d = torch.from_numpy(idx).to(dev), torch.from_numpy(grad).to(dev)
    ws = torch.empty(B.ss_backward_workspace_bytes(T, Bc, L, D), dtype=torch.uint8, device=dev)
    first = None
    for rep in range(40):
        tb = B.Tables(to_dev(W, dev))
        if rep % 2:        # something else on the device between two calls
            torch.empty(1 << 24, dtype=torch.float32, device=dev).normal_()
        B.ss_embbag_backward_update(tb, idx_d, None, grad_d, 0.01, ws)
        if first is None:
            first = [w.clone() for w in tb.weights]
            for t in range(T):
                np.testing.assert_allclose(first[t].cpu().numpy(), ref[t], rtol=RTOL, atol=ATOL)
        else:
            for t in range(T):
                assert torch.equal(tb.weights[t], first[t]), (rep, t)
    tb = B.Tables(to_dev(W, dev))
    B.ss_embbag_backward_apply(tb, Bc, L, grad_d, 0.01, ws)      # prepared by the last call
    for t in range(T):
        assert torch.equal(tb.weights[t], first[t]), t


@pytest.mark.parametrize("T", [1, 4])
def test_backward_closed_form_heavy_row(B, dev, T):
    # one row hit by every lookup of a large batch: dW = -lr * L * sum_j g_j; the run
    # covers more workgroups than the fixup stages lead states for in one go
    R, D, Bc, L = 64, 64, 20000, 2
    W = [np.ones((R, D), np.float32) for _ in range(T)]
    idx = np.full((T, Bc, L), 17, dtype=np.int32)
    rng = np.random.default_rng(450)
    grad = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
    tb = B.Tables(to_dev(W, dev))
    ws = torch.empty(B.ss_backward_workspace_bytes(T, Bc, L, D), dtype=torch.uint8, device=dev)
    B.ss_embbag_backward_update(tb, torch.from_numpy(idx).to(dev), None,
                                torch.from_numpy(grad).to(dev), 0.5, ws)
    for t in range(T):
        got = tb.weights[t].cpu().numpy()
        exact = 1.0 - 0.5 * L * grad[t].astype(np.float64).sum(axis=0)
        np.testing.assert_allclose(got[17], exact, rtol=RTOL, atol=ATOL)
        assert np.all(np.delete(got, 17, axis=0) == 1.0)


@pytest.mark.parametrize("T,R,D,Bc,L", [(3, 5000, 64, 3000, 1), (26, 1000000, 64, 8192, 1),
                                        (2, 3000, 16, 700, 1), (2, 4000, 128, 500, 3),
                                        (1, 1 << 30, 64, 4096, 1)])
def test_forward_grouped_equals_forward_plus_prepare(B, dev, T, R, D, Bc, L):
    rng = np.random.default_rng(470 + T)
    Rsmall = min(R, 50000)            # tables hold Rsmall rows; indices stay below it
    W = rand_tables(rng, T, Rsmall, D)
    idx = torch.from_numpy(zipf_idx(rng, T, Bc, L, Rsmall)).to(dev)
    grad = torch.from_numpy(rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)).to(dev)
    bits = random_bits(rng, T, Rsmall, 0.1)
    nv = torch.tensor([Bc - 7], dtype=torch.int32, device=dev)

    def tables():
        tb = B.Tables(to_dev(W, dev), bits_to_dev(bits, dev))
        if R > Rsmall:                # claim a wide row-id range: unpacked grouping path
            tb.rows = R
            tb._refresh_struct()
        return tb
    a, b = tables(), tables()
    ws = torch.empty(B.ss_backward_workspace_bytes(T, Bc, L, D), dtype=torch.uint8, device=dev)
    out_a = torch.zeros((T, Bc, D), dtype=torch.float32, device=dev)
    out_b = torch.zeros_like(out_a)
    B.ss_embbag_forward(a, idx, nv, out_a)
    B.ss_embbag_backward_update(a, idx, nv, grad, 0.01, ws)
    ws.fill_(0x33)
    B.ss_embbag_forward_grouped(b, idx, nv, out_b, ws)
    B.ss_embbag_backward_apply(b, Bc, L, grad, 0.01, ws)
    assert torch.equal(out_a, out_b)
    for t in range(T):
        assert torch.equal(a.weights[t], b.weights[t])


# ------------------------------------------------------- whole protocol
def run_lockstep(B, dev, cfg, n_iters, threshold, n_hot=None, overlap=False,
                 grouped_forward=False, pipelined=False, max_ahead=10 ** 9, index_streams=1,
                 issue_thread=False):
    """Oracle and GPU side by side; returns the number of borderline overrides."""
    from paper_2404_04270_amd.step import EmbeddingStep, PipelinedStep
    w = wl.Workload(cfg)
    idx = w.indices(0, n_iters)
    hot = wl.hot_set(idx, cfg.rows, n_hot or cfg.hot_rows)
    W0 = [w.weights(t) for t in range(cfg.num_tables)]
    ref = OracleRun([x.copy() for x in W0], hot, cfg.lr, threshold, cfg.snapshot_every)
    if pipelined:
        gpu = PipelinedStep(to_dev(W0, dev), to_dev(hot, dev), cfg.batch, cfg.bag,
                            cfg.lr, threshold, cfg.snapshot_every, every=pipelined,
                            index_streams=index_streams, issue_thread=issue_thread)
        idx_dev = torch.from_numpy(idx).to(dev)          # resident before any submit
        torch.cuda.synchronize()
        ahead = 0
    else:
        gpu = EmbeddingStep(to_dev(W0, dev), to_dev(hot, dev), cfg.batch, cfg.bag,
                            cfg.lr, threshold, cfg.snapshot_every, overlap=overlap,
                            grouped_forward=grouped_forward)
    overrides = skipped = detects = 0
    for it in range(n_iters):
        g = w.grads(it)
        r = ref.step(idx[it], g)
        if pipelined:
            # index work as far ahead as the ring (or the caller) allows
            while ahead < n_iters and gpu.room() > 0 and ahead - it < max_ahead:
                gpu.submit(idx_dev[ahead])
                ahead += 1
            gpu.forward()
        else:
            gpu.filter_forward(torch.from_numpy(idx[it]).to(dev))
        nk = int(gpu.n_kept.item())
        assert nk == r["n_kept"], it
        assert np.array_equal(gpu.skip_mask.cpu().numpy(), r["skip"]), it
        assert np.array_equal(gpu.kept_ids.cpu().numpy()[:nk], r["kept"]), it
        assert np.array_equal(gpu.idx_c.cpu().numpy()[:, :nk], r["idx_c"][:, :nk]), it
        np.testing.assert_allclose(gpu.pooled.cpu().numpy()[:, :nk], r["pooled"][:, :nk],
                                   rtol=RTOL, atol=ATOL)
        skipped += cfg.batch - nk
        g_c = np.zeros_like(g)
        g_c[:, :nk] = g[:, r["kept"]]
        detected = gpu.backward(torch.from_numpy(g_c).to(dev))
        assert detected == r["detected"]
        if detected:
            detects += 1
            r_sh, r_dr, _ = ref.last_detect
            for t in range(cfg.num_tables):
                sh = gpu.hot.stale_hot[t].cpu().numpy()
                if math.isfinite(threshold) and threshold > 0:
                    # 1e-6 relative, plus three times the 1.5e-9 by which the drifts
                    # of two runs were seen to differ once their tables differ by the
                    # rounding of earlier updates
                    border = np.abs(r_dr[t] - threshold) <= 1e-6 * threshold + 5e-9
                else:
                    border = np.zeros_like(sh, dtype=bool)
                assert np.array_equal(sh[~border], r_sh[t][~border]), (it, t)
                diff = np.flatnonzero(sh != r_sh[t])
                overrides += diff.size
                assert not (pipelined and diff.size)   # the next batch is already classified
                if diff.size:        # keep the two trajectories in lock step
                    gpu.bits[t].copy_(torch.from_numpy(ref.bits[t].view(np.int32)))
                assert np.array_equal(bits_from_dev(gpu.bits)[t], ref.bits[t]), (it, t)
    for t in range(cfg.num_tables):
        np.testing.assert_allclose(gpu.tables.weights[t].cpu().numpy(), ref.W[t],
                                   rtol=RTOL, atol=ATOL)
    n_stale = sum(int(np.unpackbits(b.view(np.uint8)).sum()) for b in ref.bits)
    if pipelined:
        gpu.close()
    return dict(overrides=overrides, skipped=skipped, detects=detects, stale=n_stale)


@pytest.mark.parametrize("pipelined", [0, 1, 4])      # 0: plain step; else events every n batches
def test_protocol_config1_full_run(B, dev, pipelined):
    cfg = wl.CONFIGS[1]
    s = run_lockstep(B, dev, cfg, cfg.iters, cfg.threshold, pipelined=pipelined)
    assert s["detects"] == cfg.iters // cfg.snapshot_every - 1
    assert s["stale"] > 0                       # this workload does flag rows
    assert s["overrides"] == 0


@pytest.mark.parametrize("grouped", [False, True])
def test_protocol_config1_threshold_infinity_skips_all_hot_samples(B, dev, grouped):
    cfg = wl.CONFIGS[1].scaled(zipf_alpha=1.6, num_tables=3)
    s = run_lockstep(B, dev, cfg, 50, math.inf, grouped_forward=grouped)
    assert s["stale"] == cfg.num_tables * cfg.hot_rows
    assert s["skipped"] > 0


@pytest.mark.parametrize("overlap", [False, True])
def test_protocol_config2_prefix(B, dev, overlap):
    cfg = wl.CONFIGS[2]
    s = run_lockstep(B, dev, cfg, 160, cfg.threshold, overlap=overlap)
    assert s["detects"] == 2 and s["overrides"] == 0


@pytest.mark.parametrize("overlap", [False, True])
def test_protocol_multihot_small(B, dev, overlap):
    cfg = wl.CONFIGS[4].scaled(rows=20000, batch=256, snapshot_every=5, hot_frac=0.005,
                               threshold=2e-3)
    s = run_lockstep(B, dev, cfg, 24, cfg.threshold, overlap=overlap)
    assert s["detects"] == 3 and s["overrides"] == 0


def test_protocol_pipelined_skips_and_multihot(B, dev):
    """The pipelined step (index work of batch i+1 next to the kernels of batch i)
    against the oracle: a run in which the skip path is busy (every hot row frozen
    at the first detect pass, detect every 3 batches) and a multi-hot run."""
    cfg = wl.CONFIGS[1].scaled(zipf_alpha=1.6, num_tables=3, snapshot_every=3)
    s = run_lockstep(B, dev, cfg, 40, math.inf, pipelined=2)
    assert s["stale"] == cfg.num_tables * cfg.hot_rows and s["skipped"] > 0
    cfg = wl.CONFIGS[4].scaled(rows=20000, batch=256, snapshot_every=5, hot_frac=0.005,
                               threshold=2e-3)
    s = run_lockstep(B, dev, cfg, 24, cfg.threshold, pipelined=3)
    assert s["detects"] == 3 and s["overrides"] == 0


def test_protocol_pipelined_with_little_lookahead(B, dev):
    """A caller that submits only one batch (or three) ahead: the streams then
    need events that were not recorded on schedule and record them on demand."""
    cfg = wl.CONFIGS[1].scaled(snapshot_every=7)
    for every, ahead in ((4, 1), (4, 3), (2, 2)):
        s = run_lockstep(B, dev, cfg, 45, cfg.threshold, pipelined=every, max_ahead=ahead)
        assert s["detects"] == 45 // 7 - 1 and s["overrides"] == 0


@pytest.mark.parametrize("streams,every,ahead", [(2, 2, 10 ** 9), (3, 1, 10 ** 9), (2, 4, 3)])
def test_protocol_pipelined_over_several_index_streams(B, dev, streams, every, ahead):
    """Index work of consecutive batches on different streams."""
    cfg = wl.CONFIGS[1].scaled(snapshot_every=7)
    s = run_lockstep(B, dev, cfg, 60, cfg.threshold, pipelined=every, max_ahead=ahead,
                     index_streams=streams)
    assert s["detects"] == 60 // 7 - 1 and s["overrides"] == 0


@pytest.mark.parametrize("streams,every,ahead,threads", [
    (1, 1, 10 ** 9, True), (1, 4, 10 ** 9, True), (2, 2, 10 ** 9, True), (2, 4, 3, True),
    (3, 1, 2, True),             # three streams or more: a thread for each
    (3, 2, 10 ** 9, True), (4, 1, 10 ** 9, True),
    (3, 2, 10 ** 9, 2),          # streams 0 and 2 share a thread
    (3, 1, 10 ** 9, 1), (2, 2, 10 ** 9, 2)])
def test_protocol_pipelined_through_the_issue_thread(B, dev, streams, every, ahead, threads):
    """The same lock-step runs with the index work enqueued by the library's own host
    threads (ss_issue_queue): bit-identical index results, weights within tolerance."""
    cfg = wl.CONFIGS[1].scaled(snapshot_every=7)
    s = run_lockstep(B, dev, cfg, 60, cfg.threshold, pipelined=every, max_ahead=ahead,
                     index_streams=streams, issue_thread=threads)
    assert s["detects"] == 60 // 7 - 1 and s["overrides"] == 0


def test_protocol_issue_thread_skips_and_multihot(B, dev):
    cfg = wl.CONFIGS[1].scaled(zipf_alpha=1.6, num_tables=3, snapshot_every=3)
    s = run_lockstep(B, dev, cfg, 40, math.inf, pipelined=2, issue_thread=True)
    assert s["stale"] == cfg.num_tables * cfg.hot_rows and s["skipped"] > 0
    cfg = wl.CONFIGS[4].scaled(rows=20000, batch=256, snapshot_every=5, hot_frac=0.005,
                               threshold=2e-3)
    s = run_lockstep(B, dev, cfg, 24, cfg.threshold, pipelined=3, index_streams=2,
                     issue_thread=True)
    assert s["detects"] == 3 and s["overrides"] == 0
    # global radix sort, three index streams with a thread each, rows frozen midway
    cfg = wl.CONFIGS[5].scaled(rows=300000, batch=20000, snapshot_every=4, hot_frac=0.002)
    s = run_lockstep(B, dev, cfg, 14, math.inf, pipelined=1, index_streams=3, issue_thread=True)
    assert s["detects"] == 2 and s["skipped"] > 0 and s["overrides"] == 0


def test_pipelined_step_refuses_calls_out_of_order(B, dev):
    from paper_2404_04270_amd.step import PipelinedStep
    rng = np.random.default_rng(470)
    T, R, D, Bn = 2, 100, 8, 16
    W = to_dev(rand_tables(rng, T, R, D), dev)
    hot = to_dev([np.arange(5, dtype=np.int32)] * T, dev)
    st = PipelinedStep(W, hot, Bn, 1, 0.01, 1e-3, 4, every=1)      # two batches ahead at most
    idx = torch.from_numpy(zipf_idx(rng, T, Bn, 1, R)).to(dev)
    grad = torch.zeros((T, Bn, D), dtype=torch.float32, device=dev)
    with pytest.raises(RuntimeError):
        st.forward()                    # nothing submitted
    st.submit(idx)
    with pytest.raises(RuntimeError):
        st.backward(grad)               # no forward yet
    st.forward()
    st.submit(idx)
    assert st.room() == 0
    with pytest.raises(RuntimeError):
        st.submit(idx)                  # too far ahead
    with pytest.raises(RuntimeError):
        st.forward()                    # previous batch not finished
    st.backward(grad)
    st.forward()
    st.backward(grad)
    torch.cuda.synchronize()


# ----------------------------------------- filter with the hot / cold split
@pytest.mark.parametrize("T,R,Bn,L,stale_frac,hot_frac", [
    (8, 10000, 128, 1, 0.3, 0.5), (26, 5000, 2049, 1, 0.9, 0.97), (3, 700, 999, 7, 0.5, 0.9),
    (8, 4000, 513, 20, 0.97, 0.99), (1, 64, 300, 1, 0.5, 0.5), (2, 50, 77, 40, 1.0, 1.0),
    (5, 3000, 1000, 3, 0.0, 0.0),
    (26, 1000, 200, 16, 0.97, 0.995),   # 416 lookups per sample: a whole wavefront each
    (16, 500, 90, 40, 0.98, 0.999)])    # 640: more than one round of probes per lane
def test_filter_split_matches_oracle(B, dev, T, R, Bn, L, stale_frac, hot_frac):
    """One pass gives the skip mask (count of stale lookups >= alpha), the compaction
    and the hot / cold membership of every input (section 3.1: hot inputs read only
    hot rows): each against the oracle's classifier, fed the stale bitmaps for the
    one and the hot bitmaps with alpha = T*L for the other."""
    rng = np.random.default_rng(T * 100 + Bn + L)
    idx = zipf_idx(rng, T, Bn, L, R, 1.3)
    stale = random_bits(rng, T, R, stale_frac)
    hot = random_bits(rng, T, R, hot_frac)
    n_forced = Bn // 3 if hot_frac > 0 else 0    # every row these samples read is made hot
    for t in range(T):
        rows = np.unique(idx[t, :n_forced])
        np.bitwise_or.at(hot[t], rows >> 5, np.uint32(1) << (rows & 31).astype(np.uint32))
    tb = B.Tables(to_dev(rand_tables(rng, T, R, 4), dev), bits_to_dev(stale, dev))
    idx_d = torch.from_numpy(idx).to(dev)
    ws = torch.empty(max(256, B.ss_filter_batch_workspace_bytes(T, Bn, L)), dtype=torch.uint8,
                     device=dev)
    want_hot, _, _ = oracle.filter_batch(R, hot, idx, T * L)
    for alpha in (T * L, max(1, T * L // 2), 1, 0, T * L + 1):
        skip = torch.full((Bn,), 7, dtype=torch.uint8, device=dev)
        hot_mask = torch.full((Bn,), 7, dtype=torch.uint8, device=dev)
        kept = torch.zeros(Bn, dtype=torch.int32, device=dev)
        nk = torch.zeros(1, dtype=torch.int32, device=dev)
        idx_c = torch.full((T, Bn, L), -1, dtype=torch.int32, device=dev)
        B.ss_filter_batch_split(tb, bits_to_dev(hot, dev), idx_d, alpha, skip, hot_mask, kept,
                                nk, idx_c, ws)
        r_skip, r_kept, r_idx_c = oracle.filter_batch(R, stale, idx, alpha)
        n = int(nk.item())
        assert n == len(r_kept), alpha
        assert np.array_equal(skip.cpu().numpy(), r_skip), alpha
        assert np.array_equal(kept.cpu().numpy()[:n], r_kept), alpha
        assert np.array_equal(idx_c.cpu().numpy()[:, :n], r_idx_c[:, :n]), alpha
        assert np.array_equal(hot_mask.cpu().numpy(), want_hot), alpha
    # no hot bitmaps at all: no input is hot; one table without a bitmap: likewise
    hot_mask = torch.full((Bn,), 7, dtype=torch.uint8, device=dev)
    B.ss_filter_batch_split(tb, None, idx_d, T * L, skip, hot_mask, kept, nk, idx_c, ws)
    assert int(hot_mask.sum().item()) == 0
    assert want_hot[:n_forced].all()
    if hot_frac == 1.0:
        assert want_hot.all()
    if hot_frac == 0.0:
        assert not want_hot.any()


def test_pipelined_step_waits_for_indices_still_being_produced(B, dev):
    """submit(idx, ready=event): the index tensor is being written by a copy on another
    stream when it is handed over; the index work must wait for the event recorded
    after that copy (checked through both paths: enqueued by the calling thread, and
    by an issue thread)."""
    from paper_2404_04270_amd.step import EmbeddingStep, PipelinedStep
    cfg = wl.CONFIGS[1].scaled(snapshot_every=5, iters=30)
    w = wl.Workload(cfg)
    idx = w.indices(0, cfg.iters)
    hot = wl.hot_set(idx, cfg.rows, cfg.hot_rows)
    W0 = [w.weights(t) for t in range(cfg.num_tables)]
    serial = EmbeddingStep(to_dev(W0, dev), to_dev(hot, dev), cfg.batch, cfg.bag, cfg.lr,
                           cfg.threshold, cfg.snapshot_every)
    grads = [torch.from_numpy(w.grads(it)).to(dev) for it in range(cfg.iters)]
    for it in range(cfg.iters):
        serial.filter_forward(torch.from_numpy(idx[it]).to(dev))
        nk = int(serial.n_kept.item())
        g_c = torch.zeros_like(grads[it])
        g_c[:, :nk] = grads[it][:, serial.kept_ids[:nk].long()]
        grads[it] = g_c
        serial.backward(g_c)
    producer = torch.cuda.Stream(device=dev)
    pinned = torch.from_numpy(idx).pin_memory()
    filler = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
    for threads in (0, 1):
        pipe = PipelinedStep(to_dev(W0, dev), to_dev(hot, dev), cfg.batch, cfg.bag, cfg.lr,
                             cfg.threshold, cfg.snapshot_every, every=2, issue_thread=threads)
        staged = [torch.full(idx[0].shape, -1, dtype=torch.int32, device=dev)
                  for _ in range(cfg.iters)]
        ahead = 0
        for it in range(cfg.iters):
            while ahead < cfg.iters and pipe.room() > 0:
                with torch.cuda.stream(producer):
                    filler.zero_()                       # keeps the producer busy for a while
                    staged[ahead].copy_(pinned[ahead], non_blocking=True)
                    ev = torch.cuda.Event()
                    ev.record(producer)
                pipe.submit(staged[ahead], ready=ev)
                ahead += 1
            pipe.forward()
            pipe.backward(grads[it])
        pipe.flush()
        torch.cuda.synchronize()
        for t in range(cfg.num_tables):
            assert torch.equal(pipe.tables.weights[t], serial.tables.weights[t]), (threads, t)
            assert torch.equal(pipe.bits[t], serial.bits[t]), (threads, t)
        pipe.close()


@pytest.mark.parametrize("host_wait_us,threads", [(0, 0), (2000, 0), (2000, 2)])
def test_free_running_pipelined_step_equals_call_by_call_step(B, dev, host_wait_us, threads):
    """The pipelined step with no synchronisation between its batches, the way a
    training loop and the benchmark drive it: the calling thread runs ahead of the GPU,
    the training stream is made to wait for index work by wait commands
    (host_wait_us = 0) or the calling thread polls for it instead.  Either way it must
    leave bit for bit what the call-by-call step leaves (every sum in the library has a
    fixed order).  Gradients go in uncompacted on both sides: row i stands for the i-th
    kept sample."""
    from paper_2404_04270_amd.step import EmbeddingStep, PipelinedStep
    T, R, D, Bn, L, K, n_iters = 8, 60000, 128, 8192, 4, 25, 160
    rng = np.random.default_rng(97)
    idx = zipf_idx(rng, T, Bn, L, R, 1.2).astype(np.int32)
    ring = [torch.from_numpy(np.roll(idx, s, axis=1).copy()).to(dev) for s in range(6)]
    hot = to_dev(wl.hot_set(idx[None], R, 300), dev)
    W0 = rand_tables(rng, T, R, D)
    grads = [torch.empty(T, Bn, D, dtype=torch.float32, device=dev).normal_(0, 0.01)
             for _ in range(3)]
    # threshold +inf: the second boundary freezes every hot row
    serial = EmbeddingStep(to_dev(W0, dev), hot, Bn, L, 0.05, math.inf, K)
    for it in range(n_iters):
        serial.filter_forward(ring[it % len(ring)])
        serial.backward(grads[it % len(grads)])
    pipe = PipelinedStep(to_dev(W0, dev), hot, Bn, L, 0.05, math.inf, K, index_streams=2,
                         issue_thread=threads, host_wait_us=host_wait_us)
    torch.cuda.synchronize()
    ahead = 0
    for it in range(n_iters):
        while ahead < n_iters and pipe.room() > 0:
            pipe.submit(ring[ahead % len(ring)])
            ahead += 1
        pipe.forward()
        pipe.backward(grads[it % len(grads)])
    pipe.flush()
    torch.cuda.synchronize()
    c = pipe.counters()
    assert c["lookups"] == n_iters
    assert c["host_polls"] >= c["host_polls_done"] >= 0
    if host_wait_us == 0:
        assert c["host_polls"] == 0
    stale = 0
    for t in range(T):
        assert torch.equal(pipe.tables.weights[t], serial.tables.weights[t]), t
        assert torch.equal(pipe.bits[t], serial.bits[t]), t
        assert torch.equal(pipe.hot.snapshot[t], serial.hot.snapshot[t]), t
        stale += int(torch.count_nonzero(serial.bits[t]).item())
    assert stale > 0                       # the run did freeze rows
    print("free-running step, host_wait_us", host_wait_us, "issue threads", threads, c, flush=True)
    pipe.close()


def test_backward_bucket_sort_with_oversized_buckets(B, dev):
    """Tables of more than a million rows: after one global pass each bucket is sorted
    by a workgroup in LDS.  A bucket that is too large for that has its most frequent
    row taken out first; if the rest still does not fit, the workgroup sorts it through
    global memory.  Table 0: every lookup hits one row; table 1: Zipf (its hottest row
    stale); table 2: six rows that share their low bits, 6 800 lookups each (the rest
    does not fit); table 3: as table 0 with that row stale (everything is a dropped
    lookup); table 4: one row with 35 000 lookups and 6 000 lookups of 2 000 other rows
    in the same bucket (they do not fit either: 2 048 do)."""
    T, R, D, Bc, L = 5, 3000000, 8, 4096, 10
    rng = np.random.default_rng(4242)
    idx = zipf_idx(rng, T, Bc, L, R, 1.2)
    idx[0] = 777
    idx[2] = (5 + 64 * rng.integers(0, 6, (Bc, L))).astype(np.int32)
    idx[3] = 123456
    flat = idx[4].reshape(-1)
    flat[:] = 9 + 64 * 7
    where = rng.choice(flat.size, 6000, replace=False)
    flat[where] = (9 + 64 * rng.integers(100, 2100, 6000)).astype(np.int32)
    bits = random_bits(rng, T, R, 0.0)
    bits[3][123456 >> 5] |= np.uint32(1 << (123456 & 31))
    bits[1][0] |= np.uint32(1)
    W = rand_tables(rng, T, R, D)
    grad = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
    ref = [w.copy() for w in W]
    oracle.embbag_backward_update(ref, bits, idx, grad, 0.01, None)
    tb = B.Tables(to_dev(W, dev), bits_to_dev(bits, dev))
    ws = torch.empty(B.ss_backward_workspace_bytes(T, Bc, L, D), dtype=torch.uint8, device=dev)
    ws.fill_(0xCD)
    idx_d, grad_d = torch.from_numpy(idx).to(dev), torch.from_numpy(grad).to(dev)
    B.ss_embbag_backward_update(tb, idx_d, None, grad_d, 0.01, ws)
    got = [w.cpu().numpy() for w in tb.weights]
    for t in range(T):
        np.testing.assert_allclose(got[t], ref[t], rtol=RTOL, atol=ATOL)
    assert np.array_equal(got[3], W[3])            # nothing moved in table 3
    assert not np.array_equal(got[0][777], W[0][777])
    # again on fresh tables: bit-identical (every sum has a fixed order)
    tb2 = B.Tables(to_dev(W, dev), bits_to_dev(bits, dev))
    ws.fill_(0x3C)
    B.ss_embbag_backward_update(tb2, idx_d, None, grad_d, 0.01, ws)
    for t in range(T):
        assert torch.equal(tb2.weights[t], tb.weights[t])
