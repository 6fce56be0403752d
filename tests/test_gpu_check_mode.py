"""Range check of lookup indices: the report of ss_check_indices against a plain
count on the host, and the checked mode, in which an out-of-range id is an error
return and nothing is launched that could fault on it.

No kernel here is ever handed a bad index outside checked mode: ss_check_indices
reads only the indices, and in checked mode the other calls return before they
enqueue anything.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2404_04270_amd import binding
    return binding


@pytest.fixture()
def checked(B):
    B.ss_check_enable(True)
    yield
    B.ss_check_enable(False)


def expected_report(idx, rows, n_valid):
    T, Bn, L = idx.shape
    bad = (idx < 0) | (idx >= rows)
    bad[:, n_valid:] = False
    n = int(bad.sum())
    if n == 0:
        return n, -1
    t, j, l = [int(x[0]) for x in np.nonzero(bad)]
    return n, (t << 32) | (j * L + l)


@pytest.mark.parametrize("T,R,Bn,L,nv,n_bad", [(3, 1000, 5000, 1, None, 0), (3, 1000, 5000, 1, None, 7),
                                               (2, 50, 777, 5, 600, 40), (1, 7, 1, 1, None, 1),
                                               (26, 10 ** 6, 8192, 1, 8000, 3),
                                               (5, 300, 4097, 3, 0, 9)])
def test_check_indices_report(B, T, R, Bn, L, nv, n_bad):
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(T * 1000 + Bn)
    idx = rng.integers(0, R, (T, Bn, L)).astype(np.int32)
    for _ in range(n_bad):
        t, j, l = rng.integers(0, T), rng.integers(0, Bn), rng.integers(0, L)
        idx[t, j, l] = rng.choice([-1, R, R + 5, -2 ** 31, 2 ** 31 - 1])
    n_valid = Bn if nv is None else nv
    report = torch.full((2,), 123, dtype=torch.int64, device=dev)
    nv_d = None if nv is None else torch.tensor([nv], dtype=torch.int32, device=dev)
    B.ss_check_indices(T, R, torch.from_numpy(idx).to(dev), nv_d, report)
    got = report.cpu().numpy()
    want = expected_report(idx, R, n_valid)
    assert (int(got[0]), int(got[1])) == want


def test_checked_mode_turns_bad_ids_into_errors_and_leaves_good_calls_alone(B, checked):
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(9)
    T, R, D, Bn, L, H = 3, 400, 16, 300, 2, 20
    W = [rng.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]
    tb = B.Tables([torch.from_numpy(w).to(dev) for w in W])
    tb.new_bits()
    good = rng.integers(0, R, (T, Bn, L)).astype(np.int32)
    bad = good.copy()
    bad[1, 17, 1] = R                     # one past the last row
    bad[2, 250, 0] = -3
    good_d, bad_d = torch.from_numpy(good).to(dev), torch.from_numpy(bad).to(dev)
    out = torch.zeros(T, Bn, D, device=dev)
    grad = torch.ones(T, Bn, D, device=dev)
    ws_b = torch.empty(B.ss_backward_workspace_bytes(T, Bn, L, D), dtype=torch.uint8, device=dev)
    ws_f = torch.empty(max(256, B.ss_filter_batch_workspace_bytes(T, Bn, L)), dtype=torch.uint8,
                       device=dev)
    skip = torch.zeros(Bn, dtype=torch.uint8, device=dev)
    kept = torch.zeros(Bn, dtype=torch.int32, device=dev)
    nk = torch.zeros(1, dtype=torch.int32, device=dev)
    idx_c = torch.zeros(T, Bn, L, dtype=torch.int32, device=dev)
    before = [w.clone() for w in tb.weights]

    with pytest.raises(B.SlipstreamError, match=r"2 lookup indices are outside \[0, 400\).*table 1 "
                                                r"at position 35 \(entry 17, lookup 1\)"):
        B.ss_embbag_forward(tb, bad_d, None, out)
    with pytest.raises(B.SlipstreamError, match="nothing was enqueued"):
        B.ss_embbag_backward_update(tb, bad_d, None, grad, 0.1, ws_b)
    with pytest.raises(B.SlipstreamError, match="outside"):
        B.ss_filter_batch(tb, bad_d, T * L, skip, kept, nk, idx_c, ws_f)
    with pytest.raises(B.SlipstreamError, match="outside"):
        B.ss_embbag_backward_prepare(tb, bad_d, None, ws_b)
    with pytest.raises(B.SlipstreamError, match="outside"):
        B.ss_count_accesses(B.AccessCounters(T, R, dev), bad_d)
    # entries past n_valid are never read by the kernels, and are not checked either
    nv = torch.tensor([17], dtype=torch.int32, device=dev)
    B.ss_embbag_forward(tb, bad_d, nv, out)
    # hot row ids
    hot_bad = [torch.arange(H, dtype=torch.int32, device=dev) for _ in range(T)]
    hot_bad[2] = hot_bad[2].clone()
    hot_bad[2][5] = R + 1
    with pytest.raises(B.SlipstreamError, match="1 hot row ids are outside.*table 2 at position 5"):
        B.ss_detect_stale(tb, B.HotState(tb, hot_bad), 1e-3, True)
    torch.cuda.synchronize()
    assert float(out[:, 17:].abs().max()) == 0.0          # only the 17 valid bags were pooled
    for t in range(T):
        assert torch.equal(tb.weights[t], before[t])      # no update ran

    # good inputs: same results as with the mode off
    B.ss_embbag_forward(tb, good_d, None, out)
    B.ss_embbag_backward_update(tb, good_d, None, grad, 0.1, ws_b)
    B.ss_check_enable(False)
    tb2 = B.Tables([torch.from_numpy(w).to(dev) for w in W])
    out2 = torch.zeros_like(out)
    B.ss_embbag_forward(tb2, good_d, None, out2)
    B.ss_embbag_backward_update(tb2, good_d, None, grad, 0.1, ws_b)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    for t in range(T):
        assert torch.equal(tb.weights[t], tb2.weights[t])
