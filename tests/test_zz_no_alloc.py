"""ss_embbag_backward_update_noalloc (the update with its workspace inside the
library's device image, for callers that cannot allocate) against
ss_embbag_backward_update on the same inputs, through the C ABI.

Both run the same kernels in the same fixed summation order, so the updated
tables must agree bit for bit, which is tighter than the rtol 1e-5 / atol 1e-6 bar
the update itself is held to against the oracle.  Two calls in a row share the
built-in buffer, the second with a smaller input: what the first left behind must
not leak into the second.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2404_04270_amd import binding
    return binding


def problem(B, dev, seed, T, R, D, Bc, L, nv, stale_frac):
    rng = np.random.default_rng(seed)
    W = [rng.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]
    idx = ((rng.zipf(1.2, (T, Bc, L)) - 1) % R).astype(np.int32)
    grad = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
    bits = []
    for _ in range(T):
        pad = np.zeros((R + 31) // 32 * 32, dtype=np.uint8)
        pad[:R] = rng.random(R) < stale_frac
        bits.append(np.packbits(pad, bitorder="little").view(np.int32).copy())

    def tables():
        return B.Tables([torch.from_numpy(w).to(dev) for w in W],
                        [torch.from_numpy(b).to(dev) for b in bits])
    n_valid = None if nv is None else torch.tensor([nv], dtype=torch.int32, device=dev)
    return (tables, torch.from_numpy(idx).to(dev), torch.from_numpy(grad).to(dev), n_valid,
            W, bits)


def test_noalloc_update_equals_workspace_update_on_two_calls_in_a_row(B):
    dev = torch.device("cuda:0")
    # the larger call first (class sort, 256-byte rows, runs that cross workgroups),
    # then a smaller one (fewer tables, shorter batch, bags of 3, 64-byte rows), then
    # one that takes the global radix sort (more than 16384 lookups per table)
    shapes = [(21, 6, 50000, 64, 7000, 1, 6500, 0.05),
              (22, 3, 900, 16, 500, 3, None, 0.2),
              (23, 2, 30000, 32, 9000, 2, 8000, 0.1)]
    for seed, T, R, D, Bc, L, nv, frac in shapes:
        need = B.ss_backward_workspace_bytes(T, Bc, L, D)
        assert 0 < need <= B.NOALLOC_SCRATCH_BYTES
        mk, idx, grad, n_valid, W, bits = problem(B, dev, seed, T, R, D, Bc, L, nv, frac)
        ref, got = mk(), mk()
        ws = torch.empty(need, dtype=torch.uint8, device=dev)
        B.ss_embbag_backward_update(ref, idx, n_valid, grad, 0.03, ws)
        B.ss_embbag_backward_update_noalloc(got, idx, n_valid, grad, 0.03)
        torch.cuda.synchronize()
        moved = 0
        for t in range(T):
            assert torch.equal(ref.weights[t], got.weights[t]), (seed, t)
            moved += int((got.weights[t].cpu().numpy() != W[t]).any(axis=1).sum())
            # bitmaps are read, never written
            assert np.array_equal(got.bits[t].cpu().numpy(), bits[t])
        assert moved > 0


def test_noalloc_update_rejects_shapes_beyond_its_buffer(B):
    dev = torch.device("cuda:0")
    T, R, D, Bc, L = 8, 64, 128, 4096, 20            # needs about 33 MB of scratch
    assert B.ss_backward_workspace_bytes(T, Bc, L, D) > B.NOALLOC_SCRATCH_BYTES
    w = [torch.zeros(R, D, device=dev) for _ in range(T)]
    tb = B.Tables(w)
    idx = torch.zeros(T, Bc, L, dtype=torch.int32, device=dev)
    grad = torch.ones(T, Bc, D, device=dev)
    with pytest.raises(B.SlipstreamError, match="built-in buffer"):
        B.ss_embbag_backward_update_noalloc(tb, idx, None, grad, 0.1)
    torch.cuda.synchronize()
    assert all(float(x.abs().max()) == 0.0 for x in w)      # nothing was enqueued
