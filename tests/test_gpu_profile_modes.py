"""The two profiling modes of the library (event pairs per dispatch; clock stamps
taken by the kernels themselves) on a real GPU: both report every launch of the
kernels they cover, in order, and neither changes a result."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2404_04270_amd import binding
    return binding


@pytest.fixture(scope="module")
def dev():
    return torch.device("cuda:0")


def make_case(dev, T=3, R=5000, D=64, Bc=3000, L=2, seed=81):
    rng = np.random.default_rng(seed)
    W = [rng.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]
    idx = ((rng.zipf(1.2, (T, Bc, L)) - 1) % R).astype(np.int32)
    grad = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
    return W, torch.from_numpy(idx).to(dev), torch.from_numpy(grad).to(dev)


def run_steps(B, dev, W, idx_d, grad_d, steps):
    T, Bc, L = idx_d.shape
    D = W[0].shape[1]
    tb = B.Tables([torch.from_numpy(w.copy()).to(dev) for w in W])
    out = torch.empty(T, Bc, D, dtype=torch.float32, device=dev)
    ws = torch.empty(B.ss_backward_workspace_bytes(T, Bc, L, D), dtype=torch.uint8, device=dev)
    for _ in range(steps):
        B.ss_embbag_forward(tb, idx_d, None, out)
        B.ss_embbag_backward_update(tb, idx_d, None, grad_d, 0.01, ws)
    torch.cuda.synchronize()
    return [w.clone() for w in tb.weights], out.clone()


def test_event_pair_mode_counts_every_launch_and_changes_nothing(B, dev):
    W, idx_d, grad_d = make_case(dev)
    plain_w, plain_out = run_steps(B, dev, W, idx_d, grad_d, 5)
    B.ss_profile_enable(1)
    try:
        prof_w, prof_out = run_steps(B, dev, W, idx_d, grad_d, 5)
    finally:
        B.ss_profile_enable(0)
    rep = B.ss_profile_report()
    for k in ("forward_kernel", "class_sort_kernel", "apply_kernel", "fixup_kernel"):
        assert k in rep, (k, rep)
        launches, total_ms = rep[k]
        assert launches == 5, (k, rep[k])
        assert 0.0 < total_ms < 100.0, (k, rep[k])
    assert torch.equal(prof_out, plain_out)
    for a, b in zip(prof_w, plain_w):
        assert torch.equal(a, b)
    # the report starts afresh
    assert B.ss_profile_report() == {}


def test_trace_mode_lists_every_launch_in_order_and_changes_nothing(B, dev):
    W, idx_d, grad_d = make_case(dev, seed=82)
    plain_w, plain_out = run_steps(B, dev, W, idx_d, grad_d, 6)
    B.ss_profile_enable(2)
    try:
        traced_w, traced_out = run_steps(B, dev, W, idx_d, grad_d, 6)
    finally:
        ev = B.ss_profile_trace()           # also ends the trace
    names = [k for k, _, _ in ev]
    assert names == ["forward_kernel", "class_sort_kernel", "apply_kernel", "fixup_kernel"] * 6, names
    prev_end = 0
    for k, start, end in ev:
        assert start <= end, (k, start, end)
        assert 0 <= end - start < 10_000_000, (k, start, end)        # under 10 ms
        # one stream: a kernel starts after the one before it has ended (the clock
        # ticks every 10 ns)
        assert start + 10 >= prev_end, (k, start, prev_end)
        prev_end = end
    assert ev[0][1] == 0                    # times count from the first start
    assert torch.equal(traced_out, plain_out)
    for a, b in zip(traced_w, plain_w):
        assert torch.equal(a, b)
    # tracing has ended: nothing more is recorded, and a second read is empty
    run_steps(B, dev, W, idx_d, grad_d, 1)
    assert B.ss_profile_trace() == []


def test_trace_mode_stops_recording_when_its_buffer_is_full(B, dev):
    """More launches than the trace holds: the rest run untraced."""
    T, R, D, Bc = 1, 64, 16, 64
    rng = np.random.default_rng(83)
    tb = B.Tables([torch.from_numpy(rng.normal(size=(R, D)).astype(np.float32)).to(dev)])
    idx_d = torch.from_numpy(rng.integers(0, R, (T, Bc, 1)).astype(np.int32)).to(dev)
    out = torch.empty(T, Bc, D, dtype=torch.float32, device=dev)
    limit = 1 << 15
    B.ss_profile_enable(2)
    try:
        for _ in range(limit + 500):
            B.ss_embbag_forward(tb, idx_d, None, out)
        torch.cuda.synchronize()
    finally:
        ev = B.ss_profile_trace()
    assert len(ev) == limit
    assert all(k == "forward_kernel" for k, _, _ in ev)
    ref = tb.weights[0][idx_d[0, :, 0].long()]
    assert torch.equal(out[0], ref)
