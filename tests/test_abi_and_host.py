"""CPU-only checks: the C-ABI library loads and exports every symbol the header
declares, host-side validation works without a GPU, and the input generator is
deterministic and has the stated structure.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2404_04270_amd import workload as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2404_04270_amd", "libslipstream.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return C.CDLL(LIB)


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "slipstream.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ss_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert set(names) >= {"ss_filter_batch", "ss_embbag_forward",
                          "ss_embbag_backward_update", "ss_detect_stale",
                          "ss_last_error", "ss_filter_batch_workspace_bytes",
                          "ss_backward_workspace_bytes"}
    for n in names:
        assert hasattr(lib, n), n


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own (and as C++)."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "slipstream.h"\nint main(void) { return SS_OK; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc,
                    "-fsyntax-only", str(src)], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-I", inc, "-fsyntax-only",
                    "-x", "c++", str(src)], check=True)


def test_binding_names_match_the_header(lib):
    from paper_2404_04270_amd import binding
    assert sorted(binding.SYMBOLS) == declared_symbols()
    for n in binding.SYMBOLS:
        assert callable(getattr(binding, n))


def test_workspace_queries_and_host_side_validation(lib):
    lib.ss_backward_workspace_bytes.restype = C.c_size_t
    lib.ss_filter_batch_workspace_bytes.restype = C.c_size_t
    lib.ss_last_error.restype = C.c_char_p
    small = lib.ss_backward_workspace_bytes(1, 128, 1, 16)
    big = lib.ss_backward_workspace_bytes(8, 4096, 20, 128)
    assert 0 < small < big and small % 256 == 0 and big % 256 == 0
    assert lib.ss_backward_workspace_bytes(1, 128, 1, 6) == 0      # dim % 4
    assert lib.ss_filter_batch_workspace_bytes(26, 8192, 1) >= 32 * 4
    # NULL tables: rejected on the host, nothing launched
    lib.ss_embbag_forward.restype = C.c_int32
    rc = lib.ss_embbag_forward(None, None, 1, 1, None, None, None)
    assert rc == 1 and b"tables is NULL" in lib.ss_last_error()


def test_configs_match_the_stated_workloads():
    c = wl.CONFIGS
    assert [c[i].num_tables for i in range(1, 6)] == [8, 26, 26, 8, 1]
    assert [c[i].rows for i in range(1, 6)] == [10**4, 10**5, 10**6, 10**7, 2 * 10**8]
    assert [c[i].dim for i in range(1, 6)] == [16, 16, 64, 128, 64]
    assert [c[i].batch for i in range(1, 6)] == [128, 2048, 8192, 4096, 65536]
    assert [c[i].bag for i in range(1, 6)] == [1, 1, 1, 20, 1]
    assert [c[i].hot_rows for i in range(1, 6)] == [100, 1000, 5000, 10000, 100000]
    assert [c[i].snapshot_every for i in range(1, 6)] == [10, 50, 100, 100, 200]
    assert c[4].table_bytes == 40_960_000_000 and c[5].table_bytes == 51_200_000_000


def test_generator_is_deterministic_and_zipf_shaped():
    cfg = wl.CONFIGS[1]
    a, b = wl.Workload(cfg), wl.Workload(cfg)
    ia, ib = a.indices(3, 2), b.indices(3, 2)
    assert ia.shape == (2, 8, 128, 1) and ia.dtype == np.int32
    assert np.array_equal(ia, ib)
    assert np.array_equal(a.indices(4, 1)[0], ia[1])          # keyed by iteration
    assert np.array_equal(a.weights(2), b.weights(2))
    assert np.array_equal(a.grads(5), b.grads(5))
    assert ia.min() >= 0 and ia.max() < cfg.rows
    w = a.weights(0)
    assert w.shape == (cfg.rows, cfg.dim) and np.abs(w).max() <= 0.05
    g = a.grads(0)
    assert abs(g.std() - 0.01) < 5e-4
    # bounded Zipf: P(rank 1) = 1 / sum k^-alpha
    cdf = wl.zipf_cdf(cfg.rows, cfg.zipf_alpha)
    p1 = 1.0 / np.sum(np.arange(1, cfg.rows + 1, dtype=np.float64) ** -cfg.zipf_alpha)
    assert abs(cdf[0] - p1) < 1e-12 and cdf[-1] == 1.0
    many = a.indices(0, 50)
    assert abs((many == 0).mean() - p1) < 0.01


def test_permutation_config_and_hot_set_rule():
    cfg = wl.CONFIGS[2].scaled(rows=1000, batch=512, num_tables=2)
    w = wl.Workload(cfg)
    idx = w.indices(0, 4)
    # per-table permutation: the most frequent row differs between tables
    top = [np.bincount(idx[:, t].ravel(), minlength=cfg.rows).argmax() for t in range(2)]
    assert top[0] != top[1]
    stream = np.array([[[[5], [5], [2], [2], [9], [7]]]], dtype=np.int32)  # [1,1,6,1]
    hot = wl.hot_set(stream, 10, 3)
    assert hot.tolist() == [[2, 5, 7]]       # counts 2,2,1,1: tie 7 vs 9 -> lower id
    assert wl.bitmap_words(33) == 2


def test_hot_set_equals_a_full_sort_by_count_then_row():
    """The harness picks the hot rows without sorting every row; the rule it must
    reproduce is "first n by (count descending, row ascending)", here written out
    as a stable full sort, on both of its paths (dense counters; far more rows than
    lookups) and at the edges (everything hot, ties at the cut, unaccessed rows)."""
    rng = np.random.default_rng(12)
    for R, n, H in [(10, 200, 3), (1000, 5000, 37), (50, 10, 50), (50, 10, 49), (7, 0, 3),
                    (100000, 20, 30), (100000, 20, 5), (5000, 30, 4999), (5000, 30, 5000)]:
        for _ in range(5):
            s = rng.integers(0, R, (3, 2, n // 2 + 1 if n else 0, 1)).astype(np.int32)
            got = wl.hot_set(s, R, H)
            for t in range(2):
                cnt = np.bincount(s[:, t].reshape(-1), minlength=R)
                want = np.sort(np.argsort(-cnt, kind="stable")[:H])
                assert np.array_equal(got[t], want), (R, n, H)


# ---------------------------------------------------- sampling block, host side
def drop_stats(lib, count, n, pop, hot, t):
    lib.ss_drop_stats.restype = C.c_int32
    out = (C.c_double * 8)()
    rc = lib.ss_drop_stats(C.c_uint32(count), C.c_int64(n), C.c_int64(pop),
                           C.c_int64(hot), C.c_double(t), out)
    return rc, list(out)


def test_drop_stats_matches_the_oracle_and_rejects_bad_arguments(lib):
    """ss_drop_stats is host arithmetic (Eq. 2-4): no GPU is involved."""
    import oracle
    keys = ("D", "sd", "half", "lo", "hi", "D_bar", "D_bar_lo", "D_bar_hi")
    for count, n, pop, hot, t in [(0, 100, 100000, 100000, 3.340), (100, 100, 1000, 900, 3.340),
                                  (37, 4096, 4_194_304, 3_000_000, 3.340),
                                  (512, 1024, 1024, 1024, 2.0), (1, 3, 7, 5, 0.0)]:
        rc, got = drop_stats(lib, count, n, pop, hot, t)
        assert rc == 0
        ref = oracle.drop_stats(count, n, pop, hot, t)
        np.testing.assert_allclose(got, [ref[k] for k in keys], rtol=1e-12, atol=1e-15)
    lib.ss_last_error.restype = C.c_char_p
    for bad in [(5, 4, 10, 10, 1.0), (0, 0, 10, 10, 1.0), (0, 11, 10, 10, 1.0),
                (0, 5, 10, -1, 1.0), (0, 5, 10, 10, -1.0), (0, 5, 10, 10, float("nan"))]:
        rc, _ = drop_stats(lib, *bad)
        assert rc == 1 and b"ss_drop_stats" in lib.ss_last_error()


def test_sample_drop_validates_on_the_host(lib):
    lib.ss_sample_drop.restype = C.c_int32
    lib.ss_last_error.restype = C.c_char_p
    thr = (C.c_float * 2)(1.0, float("nan"))
    fake = C.c_void_p(256)           # never dereferenced: every call below is rejected
    def call(T=2, H=4, S=8, L=1, alpha=1, n_thr=1, thresholds=thr, counts=fake):
        return lib.ss_sample_drop(C.c_int32(T), fake, C.c_int32(H), fake, fake,
                                  C.c_int32(S), C.c_int32(L), C.c_int32(alpha),
                                  thresholds, C.c_int32(n_thr), counts, None)
    for kwargs, text in [(dict(T=0), b"num_tables"), (dict(H=-1), b"H ="),
                         (dict(S=-1), b"S ="), (dict(L=0), b"L ="),
                         (dict(alpha=-1), b"alpha"), (dict(n_thr=0), b"n_thr"),
                         (dict(n_thr=33), b"n_thr"), (dict(n_thr=2), b"NaN"),
                         (dict(thresholds=None), b"NULL"), (dict(counts=None), b"NULL"),
                         (dict(S=1 << 30, L=4), b"int32")]:
        assert call(**kwargs) != 0, kwargs
        assert text in lib.ss_last_error(), (kwargs, lib.ss_last_error())


def test_ladder_search_finds_the_largest_threshold_within_budget():
    from paper_2404_04270_amd.sampling import geometric_ladder, ladder_search
    lad = geometric_ladder(1e-4, 1e-1, 32)
    assert len(lad) == 32 and all(a < b for a, b in zip(lad, lad[1:]))
    assert 1e-4 < lad[0] and lad[-1] < 1e-1
    np.testing.assert_allclose(np.diff(np.log(lad)), np.log(1e3) / 33, rtol=1e-9)

    rng = np.random.default_rng(5)
    drifts = np.sort(rng.lognormal(np.log(3e-3), 1.0, 5000))
    calls = []
    def bound(ts):               # share of "rows" at or below T: monotone in T
        calls.append(len(ts))
        return [float(np.searchsorted(drifts, t, side="right")) / drifts.size for t in ts]
    for budget in (0.05, 0.3, 0.77):
        calls.clear()
        T, tried = ladder_search(bound, 1e-5, 1.0, budget, passes=2)
        assert bound([T])[0] <= budget
        assert calls[:3] == [2, 32, 32]
        # resolution after two passes: (hi/lo)^(1/33^2); the next point fails
        ratio = (1.0 / 1e-5) ** (1.0 / 33 ** 2)
        assert bound([T * ratio * 1.0001])[0] > budget
        assert all(b <= budget for t, b in tried if t <= T)
    assert ladder_search(bound, 1e-5, 1.0, -0.1)[0] is None        # even lo is over
    assert ladder_search(bound, 1e-5, 1.0, 1.0)[0] == 1.0          # hi itself fits


def test_hot_set_calls_validate_on_the_host(lib):
    lib.ss_select_hot_workspace_bytes.restype = C.c_size_t
    lib.ss_last_error.restype = C.c_char_p
    for name in ("ss_count_accesses", "ss_select_hot_ratio", "ss_select_hot_top"):
        getattr(lib, name).restype = C.c_int32
    small = lib.ss_select_hot_workspace_bytes(C.c_int32(1), C.c_int64(100))
    big = lib.ss_select_hot_workspace_bytes(C.c_int32(26), C.c_int64(1_000_000))
    assert 0 < small < big and small % 256 == 0 and big % 256 == 0
    assert lib.ss_select_hot_workspace_bytes(C.c_int32(0), C.c_int64(100)) == 0
    assert lib.ss_select_hot_workspace_bytes(C.c_int32(1), C.c_int64(1 << 31)) == 0
    fake = C.c_void_p(256)                  # never dereferenced: every call is rejected

    def count(T=2, rows=100, idx=fake, B=4, L=1, counts=fake):
        return lib.ss_count_accesses(C.c_int32(T), C.c_int64(rows), idx, C.c_int32(B),
                                     C.c_int32(L), None, counts, None)
    for kw, text in [(dict(T=0), b"num_tables"), (dict(rows=0), b"rows"),
                     (dict(idx=None), b"idx"), (dict(B=0), b"batch"), (dict(L=0), b"L ="),
                     (dict(counts=None), b"counts")]:
        assert count(**kw) != 0 and text in lib.ss_last_error(), kw

    def ratio(lam=0.5, total=10, cap=4, ids=fake, ws=fake, ws_bytes=1 << 20):
        return lib.ss_select_hot_ratio(C.c_int32(2), C.c_int64(100), fake, C.c_double(lam),
                                       C.c_int64(total), C.c_int32(cap), ids, None, None, ws,
                                       C.c_size_t(ws_bytes), None)
    for kw, text in [(dict(lam=float("nan")), b"NaN"), (dict(total=0), b"total"),
                     (dict(cap=-1), b"cap"), (dict(ids=None), b"hot_ids"),
                     (dict(ws=None), b"workspace"), (dict(ws_bytes=8), b"workspace"),
                     (dict(ws=C.c_void_p(264)), b"aligned")]:
        assert ratio(**kw) != 0 and text in lib.ss_last_error(), kw

    def top(H=5, ids=fake, ws_bytes=1 << 20):
        return lib.ss_select_hot_top(C.c_int32(2), C.c_int64(100), fake, C.c_int32(H), ids,
                                     None, fake, C.c_size_t(ws_bytes), None)
    for kw, text in [(dict(H=-1), b"H ="), (dict(H=101), b"H ="), (dict(ids=None), b"hot_ids"),
                     (dict(ws_bytes=0), b"workspace")]:
        assert top(**kw) != 0 and text in lib.ss_last_error(), kw


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_layernorm_calls_validate_on_the_host(lib):
    lib.ss_last_error.restype = C.c_char_p
    lib.ss_layernorm_forward.restype = C.c_int32
    lib.ss_layernorm_backward.restype = C.c_int32
    lib.ss_layernorm_backward_workspace_bytes.restype = C.c_size_t
    assert lib.ss_layernorm_backward_workspace_bytes(2, 64, 1000) % 256 == 0
    assert lib.ss_layernorm_backward_workspace_bytes(2, 6, 1000) == 0        # dim % 4
    ok = C.c_void_p(256)               # never dereferenced: every call below is rejected
    odd = C.c_void_p(260)

    def fwd(T=2, dim=16, x=ok, Bcap=8, gamma=None, eps=1e-5, y=ok, mean=ok, rstd=ok):
        return lib.ss_layernorm_forward(C.c_int32(T), C.c_int32(dim), x, C.c_int32(Bcap), None,
                                        gamma, None, C.c_float(eps), y, mean, rstd, None)
    for kw, text in [(dict(T=0), b"num_tables"), (dict(dim=6), b"dim"), (dict(Bcap=0), b"Bcap"),
                     (dict(x=None), b"NULL"), (dict(mean=None), b"NULL"),
                     (dict(eps=-1.0), b"eps"), (dict(eps=float("nan")), b"eps"),
                     (dict(x=odd), b"x is not 16-byte"), (dict(y=odd), b"y is not 16-byte"),
                     (dict(gamma=odd), b"gamma is not 16-byte")]:
        assert fwd(**kw) != 0 and text in lib.ss_last_error(), (kw, lib.ss_last_error())

    def bwd(dy=ok, x=ok, dx=ok, dgamma=None, ws=None, ws_bytes=0):
        return lib.ss_layernorm_backward(C.c_int32(2), C.c_int32(16), dy, x, C.c_int32(8), None,
                                         None, ok, ok, dx, dgamma, None, ws, C.c_size_t(ws_bytes),
                                         None)
    for kw, text in [(dict(dy=None), b"NULL"), (dict(dx=odd), b"dx is not 16-byte"),
                     (dict(dgamma=ok), b"workspace"),
                     (dict(dgamma=ok, ws=ok, ws_bytes=16), b"workspace")]:
        assert bwd(**kw) != 0 and text in lib.ss_last_error(), (kw, lib.ss_last_error())


def test_step_plan_picks_streams_threads_and_event_spacing_for_the_shape():
    """Host logic only (ss_step_plan_for): index streams and issue threads by the
    size of a batch's index work, 8 batches between events unless the grouped lists
    of a ring of 3 * every * streams sets would outgrow their share of the
    memory-side cache."""
    from paper_2404_04270_amd import binding
    from paper_2404_04270_amd.step import PipelinedStep as P
    plan = binding.ss_step_plan_for
    assert P.auto_streams(8192, 1) == 1 and P.auto_streams(16384, 1) == 1
    assert P.auto_streams(65536, 1, 1) == 3 and P.auto_streams(4096, 20, 8) == 2
    assert P.auto_streams(65536, 1, 8) == 2 and P.auto_streams(20000, 1, 1) == 3
    # ... and one again where the training kernels of a batch outlast its index work
    assert P.auto_streams(4096, 20, 8, 128) == 1 and P.auto_streams(4096, 20, 8, 64) == 2
    assert P.auto_streams(32768, 1, 8, 64) == 2 and P.auto_streams(65536, 1, 1, 1024) == 3
    assert plan(26, 2048, 1).issue_threads == 1 and plan(1, 65536, 1).issue_threads == 3
    assert plan(26, 8192, 1).issue_threads == 0 and plan(8, 4096, 20).issue_threads == 0
    assert P.auto_every(26, 8192, 1, 1) == 8         # 3.4 MB of lists per batch
    assert P.auto_every(1, 65536, 1, 2) == 8
    assert P.auto_every(8, 4096, 20, 1) == 2         # 10.5 MB per batch
    assert P.auto_every(8, 4096, 20, 4) == 2         # never below 2
    ring_bytes = 96 << 20
    for T, b, L, n in [(26, 8192, 1, 1), (8, 4096, 20, 1), (4, 30000, 3, 2)]:
        e = P.auto_every(T, b, L, n)
        lists = 16 * T * ((b * L + 2047) // 2048) * 2048
        assert e in (2, 4, 8) and (e == 2 or 3 * e * n * lists <= ring_bytes)
        assert e == 8 or 3 * 2 * e * n * lists > ring_bytes        # the largest that fits
    # what the caller fixes stays; the ring follows
    p = plan(26, 8192, 1, every=3, index_streams=2, issue_threads=5)
    assert (p.every, p.index_streams, p.issue_threads, p.num_sets) == (3, 2, 2, 18)
    # the calling thread polls for index work only where that was measured to pay
    # (bags of several lookups), unless the caller says otherwise
    assert plan(8, 4096, 20).host_wait_us == 2000 and plan(26, 8192, 1).host_wait_us == 0
    assert plan(26, 8192, 1, host_wait_us=300).host_wait_us == 300
    assert plan(8, 4096, 20, host_wait_us=0).host_wait_us == 0
    with pytest.raises(binding.SlipstreamError):
        plan(0, 8, 1)
    with pytest.raises(binding.SlipstreamError):
        plan(1, 8, 1, index_streams=17)


def test_step_calls_validate_on_the_host(lib):
    """ss_step_*: a bad plan or a missing argument is refused before any stream, event
    or thread is created; calls on a NULL step are errors, destroying one is not."""
    from paper_2404_04270_amd import binding
    lib.ss_last_error.restype = C.c_char_p
    for n in ("ss_step_create", "ss_step_create_traced", "ss_step_destroy", "ss_step_submit",
              "ss_step_forward", "ss_step_backward", "ss_step_flush", "ss_step_room"):
        getattr(lib, n).restype = C.c_int32
    ok = C.c_void_p(256)               # never dereferenced: every call below is rejected
    plan = binding.StepPlan(2, 1, 0, 7)                  # 3 * 2 * 1 = 6 sets, not 7
    out = C.c_void_p()
    ops = binding.StepTraceOps()
    assert lib.ss_step_create_traced(C.byref(plan), 4, C.byref(ops), C.byref(out)) != 0
    assert b"num_sets" in lib.ss_last_error()
    plan = binding.StepPlan(2, 1, 3, 6)                  # more threads than streams
    assert lib.ss_step_create_traced(C.byref(plan), 4, C.byref(ops), C.byref(out)) != 0
    plan = binding.StepPlan(2, 1, 0, 6, -1)              # host_wait_us left unplanned
    assert lib.ss_step_create_traced(C.byref(plan), 4, C.byref(ops), C.byref(out)) != 0
    assert b"host_wait_us" in lib.ss_last_error()
    plan = binding.StepPlan(2, 1, 0, 6)
    assert lib.ss_step_create_traced(C.byref(plan), 0, C.byref(ops), C.byref(out)) != 0
    assert b"snapshot_every" in lib.ss_last_error()
    assert lib.ss_step_create_traced(C.byref(plan), 4, None, C.byref(out)) != 0
    assert lib.ss_step_create(None, 8, 1, 1, C.c_float(0.1), C.c_float(1e-3), 4, ok, 1, ok, None,
                              None, None, C.byref(plan), ok, ok, None, C.byref(out)) != 0
    assert b"tables is NULL" in lib.ss_last_error()
    assert lib.ss_step_submit(None, ok, None) != 0 and lib.ss_step_forward(None, None) != 0
    assert lib.ss_step_backward(None, ok, None) != 0 and lib.ss_step_flush(None) != 0
    assert lib.ss_step_room(None) == 0 and lib.ss_step_destroy(None) == 0


def test_issue_queue_calls_validate_on_the_host(lib):
    lib.ss_last_error.restype = C.c_char_p
    for n in ("ss_issue_index_batch", "ss_issue_wait_event", "ss_issue_record_event",
              "ss_issue_wait", "ss_event_record", "ss_stream_wait_event", "ss_event_create",
              "ss_issue_queue_create", "ss_issue_queue_destroy", "ss_event_destroy"):
        getattr(lib, n).restype = C.c_int32
    ok = C.c_void_p(256)               # never dereferenced: every call below is rejected
    assert lib.ss_issue_index_batch(None, None, ok, 8, 1, 1, ok, ok, ok, ok, ok, C.c_size_t(256),
                                    ok, C.c_size_t(256), None, None) != 0
    assert b"queue is NULL" in lib.ss_last_error()
    assert lib.ss_issue_wait_event(None, ok, None, None) != 0
    assert lib.ss_issue_record_event(None, ok, None, None) != 0
    assert lib.ss_issue_wait(None, C.c_uint64(1)) != 0
    assert lib.ss_event_record(None, None) != 0 and b"event is NULL" in lib.ss_last_error()
    assert lib.ss_stream_wait_event(None, None) != 0
    assert lib.ss_event_create(None) != 0
    assert lib.ss_issue_queue_create(None) != 0
    assert lib.ss_issue_queue_destroy(None) == 0 and lib.ss_event_destroy(None) == 0


def test_issue_queue_needs_a_device():
    import torch
    from paper_2404_04270_amd import binding
    if torch.cuda.is_available():
        pytest.skip("a device is present: creation succeeds (covered by the GPU tests)")
    with pytest.raises(binding.SlipstreamError, match="no current device"):
        binding.IssueQueue()
