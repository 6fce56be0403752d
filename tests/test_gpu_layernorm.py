"""GPU parity of the feature normalization (section 3.5 of the paper: LayerNorm
over every pooled vector), forward and backward, through the C ABI against the
fp64 CPU oracle.  Tolerance: rtol 1e-5 / atol 1e-6 on fp32 outputs; the batch
sums dgamma / dbeta are compared relative to the size of their terms (atol
scaled by the root of the number of terms, the error of an fp32 sum).
"""
import numpy as np
import pytest
import torch

import oracle
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


def dv(a, dev):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)


CASES = [
    # T, Bcap, D, n_valid, affine
    (3, 700, 16, None, True),
    (2, 1025, 64, 999, True),
    (2, 333, 128, None, False),
    (1, 70, 4, 0, True),             # nothing valid
    (2, 130, 48, 77, True),          # dim not a power of two
    (1, 40, 260, None, True),        # two f4 per lane
    (1, 33, 1024, 20, True),         # four f4 per lane
    (26, 2100, 64, 2000, True),      # several workgroups per table in the backward pass
    (1, 1, 8, None, False),
]


@pytest.mark.parametrize("T,Bc,D,nv,affine", CASES)
def test_layernorm_forward_and_backward_match_oracle(B, dev, T, Bc, D, nv, affine):
    rng = np.random.default_rng(1500 + T + Bc + D)
    x = (rng.normal(0.05, 1.0, (T, Bc, D)) * rng.uniform(0.05, 3.0, (T, Bc, 1))).astype(np.float32)
    dy = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
    gamma = rng.normal(1, 0.3, (T, D)).astype(np.float32) if affine else None
    beta = rng.normal(0, 0.3, (T, D)).astype(np.float32) if affine else None
    eps = 1e-5
    n = Bc if nv is None else nv
    n_valid = None if nv is None else torch.tensor([nv], dtype=torch.int32, device=dev)

    r_y, r_mean, r_rstd = oracle.layernorm_forward(x, gamma, beta, eps, nv)
    x_d = dv(x, dev)
    y = torch.full((T, Bc, D), 7.0, dtype=torch.float32, device=dev)
    mean = torch.full((T, Bc), 7.0, dtype=torch.float32, device=dev)
    rstd = torch.full((T, Bc), 7.0, dtype=torch.float32, device=dev)
    B.ss_layernorm_forward(x_d, n_valid, dv(gamma, dev), dv(beta, dev), eps, y, mean, rstd)
    got = y.cpu().numpy()
    np.testing.assert_allclose(got[:, :n], r_y[:, :n], rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(mean.cpu().numpy()[:, :n], r_mean[:, :n], rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(rstd.cpu().numpy()[:, :n], r_rstd[:, :n], rtol=RTOL, atol=ATOL)
    assert np.all(got[:, n:] == 7.0) and np.all(mean.cpu().numpy()[:, n:] == 7.0)

    r_dx, r_dg, r_db = oracle.layernorm_backward(dy, x, gamma, eps, nv)
    dx = torch.full((T, Bc, D), 7.0, dtype=torch.float32, device=dev)
    dgamma = torch.full((T, D), 7.0, dtype=torch.float32, device=dev)
    dbeta = torch.full((T, D), 7.0, dtype=torch.float32, device=dev)
    ws = torch.empty(max(256, B.ss_layernorm_backward_workspace_bytes(T, D, Bc)),
                     dtype=torch.uint8, device=dev)
    ws.fill_(0xEE)
    dy_d = dv(dy, dev)
    B.ss_layernorm_backward(dy_d, x_d, n_valid, dv(gamma, dev), mean, rstd, dx, dgamma, dbeta, ws)
    got = dx.cpu().numpy()
    np.testing.assert_allclose(got[:, :n], r_dx[:, :n], rtol=RTOL, atol=ATOL)
    assert np.all(got[:, n:] == 7.0)
    # sums of n terms of size ~|dy| (and ~|dy * xhat|): fp32 summation error
    sum_atol = ATOL + 1e-7 * np.sqrt(max(n, 1)) * 0.05
    np.testing.assert_allclose(dgamma.cpu().numpy(), r_dg, rtol=RTOL, atol=sum_atol)
    np.testing.assert_allclose(dbeta.cpu().numpy(), r_db, rtol=RTOL, atol=sum_atol)

    # in place (dx = dy) and without parameter gradients: same dx, bit for bit
    B.ss_layernorm_backward(dy_d, x_d, n_valid, dv(gamma, dev), mean, rstd, dy_d, None, None, None)
    assert torch.equal(dy_d[:, :n], dx[:, :n])
    assert np.array_equal(dy_d.cpu().numpy()[:, n:], dy[:, n:])
    # run to run: the batch sums are taken in a fixed order
    dgamma2 = torch.zeros_like(dgamma)
    dbeta2 = torch.zeros_like(dbeta)
    B.ss_layernorm_backward(dv(dy, dev), x_d, n_valid, dv(gamma, dev), mean, rstd, dx, dgamma2,
                            dbeta2, ws)
    assert torch.equal(dgamma, dgamma2) and torch.equal(dbeta, dbeta2)


def test_layernorm_between_forward_and_update_at_config3_shape(B, dev):
    """Pooled lookup -> LayerNorm -> (gradient) -> LayerNorm backward -> sparse
    update on the full-size tables of config 3, every stage against the oracle on
    the same inputs (the update on the compact problem of the touched rows)."""
    cfg = wl.CONFIGS[3]
    T, R, D, Bn, L = cfg.num_tables, cfg.rows, cfg.dim, cfg.batch, cfg.bag
    w = wl.Workload(cfg)
    idx = w.indices(0, 1)[0]
    dy = w.grads(0)
    weights = [w.weights_device(t, dev) for t in range(T)]
    tb = B.Tables(weights)
    rng = np.random.default_rng(1600)
    gamma = rng.normal(1, 0.2, (T, D)).astype(np.float32)
    beta = rng.normal(0, 0.2, (T, D)).astype(np.float32)
    idx_d = torch.from_numpy(idx).to(dev)
    pooled = torch.empty((T, Bn, D), dtype=torch.float32, device=dev)
    B.ss_embbag_forward(tb, idx_d, None, pooled)
    y = torch.empty_like(pooled)
    mean = torch.empty((T, Bn), dtype=torch.float32, device=dev)
    rstd = torch.empty_like(mean)
    B.ss_layernorm_forward(pooled, None, dv(gamma, dev), dv(beta, dev), 1e-5, y, mean, rstd)
    x = pooled.cpu().numpy()
    r_y, _, _ = oracle.layernorm_forward(x, gamma, beta, 1e-5)
    np.testing.assert_allclose(y.cpu().numpy(), r_y, rtol=RTOL, atol=ATOL)
    # the pooled vectors are rows of uniform(-0.05, 0.05) tables: after the layer
    # every vector has zero mean and unit variance up to the affine map
    z = (y.cpu().numpy().astype(np.float64) - beta[:, None, :]) / gamma[:, None, :]
    assert np.abs(z.mean(-1)).max() < 1e-4 and np.abs(z.var(-1) - 1).max() < 3e-2   # eps = 1e-5 against var ~ 8e-4

    dx = torch.empty_like(pooled)
    dgamma = torch.empty((T, D), dtype=torch.float32, device=dev)
    dbeta = torch.empty_like(dgamma)
    ws = torch.empty(B.ss_layernorm_backward_workspace_bytes(T, D, Bn), dtype=torch.uint8,
                     device=dev)
    B.ss_layernorm_backward(torch.from_numpy(dy).to(dev), pooled, None, dv(gamma, dev), mean,
                            rstd, dx, dgamma, dbeta, ws)
    r_dx, r_dg, r_db = oracle.layernorm_backward(dy, x, gamma, 1e-5)
    # dx is ~ rstd * dy with rstd ~ 35 here: compare relative to its own size
    np.testing.assert_allclose(dx.cpu().numpy(), r_dx, rtol=RTOL, atol=ATOL * 35)
    np.testing.assert_allclose(dgamma.cpu().numpy(), r_dg, rtol=1e-4, atol=1e-4)
    np.testing.assert_allclose(dbeta.cpu().numpy(), r_db, rtol=1e-4, atol=1e-5)

    # the sparse update with the normalised gradient, on the rows the batch touches
    rows = [np.unique(idx[t]) for t in range(T)]
    before = [weights[t][torch.from_numpy(rows[t]).to(dev).long()].cpu().numpy() for t in range(T)]
    rmax = max(b.shape[0] for b in before)
    mini = [np.ascontiguousarray(np.pad(b, ((0, rmax - b.shape[0]), (0, 0)))) for b in before]
    idx_m = np.stack([np.searchsorted(rows[t], idx[t]).astype(np.int32) for t in range(T)])
    dx_host = dx.cpu().numpy()
    oracle.embbag_backward_update(mini, None, idx_m, dx_host, cfg.lr)
    ws_b = torch.empty(B.ss_backward_workspace_bytes(T, Bn, L, D), dtype=torch.uint8, device=dev)
    B.ss_embbag_backward_update(tb, idx_d, None, dx, cfg.lr, ws_b)
    for t in range(T):
        got = weights[t][torch.from_numpy(rows[t]).to(dev).long()].cpu().numpy()
        np.testing.assert_allclose(got, mini[t][:rows[t].size], rtol=RTOL, atol=ATOL * 35)


@pytest.mark.parametrize("T,R,D,Bc,L,nv", [
    (3, 1000, 16, 700, 1, None),
    (2, 5000, 64, 1025, 1, 999),
    (2, 3000, 128, 333, 20, 300),      # multi-hot: the bag is summed on the fly
    (2, 500, 48, 130, 9, 77),
    (1, 300, 260, 40, 3, None),        # two f4 per lane
    (1, 200, 1024, 20, 2, 11),         # four f4 per lane
    (2, 400, 16, 300, 1, 0),
])
def test_pooled_layernorm_in_one_pass_equals_the_two_calls(B, dev, T, R, D, Bc, L, nv):
    """ss_embbag_forward_ln / ss_embbag_ln_backward against the separate calls
    (bit for bit: same arithmetic on the same pooled values) and the oracle."""
    rng = np.random.default_rng(1700 + D + L + Bc)
    W = [rng.uniform(-0.05, 0.05, (R, D)).astype(np.float32) for _ in range(T)]
    idx = ((rng.zipf(1.2, (T, Bc, L)) - 1) % R).astype(np.int32)
    if nv is not None:
        idx[:, nv:] = -1                        # bags past n_valid hold no usable index
    n = Bc if nv is None else nv
    gamma = rng.normal(1, 0.3, (T, D)).astype(np.float32)
    beta = rng.normal(0, 0.3, (T, D)).astype(np.float32)
    dy = rng.normal(0, 0.01, (T, Bc, D)).astype(np.float32)
    eps = 1e-5
    tb = B.Tables([dv(w, dev) for w in W])
    idx_d, n_valid = dv(idx, dev), (None if nv is None else
                                    torch.tensor([nv], dtype=torch.int32, device=dev))
    g_d, b_d, dy_d = dv(gamma, dev), dv(beta, dev), dv(dy, dev)

    def outputs():
        return (torch.full((T, Bc, D), 7.0, dtype=torch.float32, device=dev),
                torch.full((T, Bc), 7.0, dtype=torch.float32, device=dev),
                torch.full((T, Bc), 7.0, dtype=torch.float32, device=dev))
    # the two calls
    x = torch.full((T, Bc, D), 7.0, dtype=torch.float32, device=dev)
    B.ss_embbag_forward(tb, idx_d, n_valid, x)
    y2, mean2, rstd2 = outputs()
    B.ss_layernorm_forward(x, n_valid, g_d, b_d, eps, y2, mean2, rstd2)
    ws = torch.empty(max(256, B.ss_layernorm_backward_workspace_bytes(T, D, Bc)),
                     dtype=torch.uint8, device=dev)
    dx2, dg2, db2 = (torch.full((T, Bc, D), 7.0, device=dev), torch.zeros(T, D, device=dev),
                     torch.zeros(T, D, device=dev))
    B.ss_layernorm_backward(dy_d, x, n_valid, g_d, mean2, rstd2, dx2, dg2, db2, ws)
    # one pass each way
    y1, mean1, rstd1 = outputs()
    B.ss_embbag_forward_ln(tb, idx_d, n_valid, g_d, b_d, eps, y1, mean1, rstd1)
    dx1, dg1, db1 = (torch.full((T, Bc, D), 7.0, device=dev), torch.zeros(T, D, device=dev),
                     torch.zeros(T, D, device=dev))
    B.ss_embbag_ln_backward(tb, idx_d, n_valid, dy_d, g_d, mean1, rstd1, dx1, dg1, db1, ws)
    for a, b in ((y1, y2), (mean1, mean2), (rstd1, rstd2), (dx1, dx2), (dg1, dg2), (db1, db2)):
        assert torch.equal(a, b)
    # and the oracle, from its own pooled vectors
    x_ref = oracle.embbag_forward(W, idx, nv)
    r_y, _, _ = oracle.layernorm_forward(x_ref, gamma, beta, eps, nv)
    r_dx, r_dg, r_db = oracle.layernorm_backward(dy, x_ref, gamma, eps, nv)
    # rstd is ~ 1/(0.03 sqrt(L)): rounding of the pooled value is amplified by it
    amp = 40.0
    np.testing.assert_allclose(y1.cpu().numpy()[:, :n], r_y[:, :n], rtol=RTOL, atol=ATOL * amp)
    np.testing.assert_allclose(dx1.cpu().numpy()[:, :n], r_dx[:, :n], rtol=RTOL, atol=ATOL * amp)
    np.testing.assert_allclose(dg1.cpu().numpy(), r_dg, rtol=1e-4, atol=1e-5 * np.sqrt(max(n, 1)))
    np.testing.assert_allclose(db1.cpu().numpy(), r_db, rtol=1e-4, atol=1e-6 * np.sqrt(max(n, 1)))
    assert torch.all(y1[:, n:] == 7.0) and torch.all(dx1[:, n:] == 7.0)
