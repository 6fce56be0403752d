#!/usr/bin/env python3
"""Throughput of the embedding hot path on one MI355X.

A step = filter_batch -> forward -> backward_update over one batch of seeded
Zipf lookups, plus detect_stale on the iterations where the snapshot period
ends.  By default the index-only work of the coming batches (filter_batch and the
grouping half of the update) runs on a second stream next to the forward and
update kernels of the current batch; --serial issues everything in order on one
stream.  Inputs are resident in HBM before the timed region starts.  Prints one
JSON line: whole-job samples/s ("value"), the roofline of the dominant kernel
(algorithmic bytes per launch over its measured duration, against 8 TB/s), the
per-kernel durations, the skip fraction, and the CPU oracle timed on this host.
"""
import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The timed region should be long against anything that happens once (a host
    # thread descheduled for some tens of milliseconds would double a 20 ms
    # region), and the warm-up should take every kind of launch once: the first
    # period ends with a snapshot capture, the second with the first detect pass.
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=250)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--threshold", type=float, default=None,
                    help="drift threshold T (default: the config's; inf freezes all hot rows)")
    ap.add_argument("--snapshot-every", type=int, default=0,
                    help="snapshot period K in iterations (default: the config's)")
    ap.add_argument("--ring", type=int, default=16, help="distinct batches cycled through")
    ap.add_argument("--grad-buffers", type=int, default=4,
                    help="distinct gradient tensors cycled through (4: together with the "
                         "pooled output more than the 256 MB memory-side cache holds)")
    ap.add_argument("--overlap", action="store_true",
                    help="issue the grouping half of the backward pass on a second "
                         "stream next to the forward pass (measured slower on one GPU "
                         "when nothing else runs between forward and backward)")
    ap.add_argument("--grouped-forward", action="store_true",
                    help="use ss_embbag_forward_grouped (forward and the grouping half of "
                         "the backward pass in one launch)")
    ap.add_argument("--pipeline-every", type=int, default=0,
                    help="batches between two cross-stream events of the pipelined step "
                         "(0: PipelinedStep's own choice)")
    ap.add_argument("--index-streams", type=int, default=0,
                    help="streams the index work of the pipelined step is spread over "
                         "(0: PipelinedStep's own choice)")
    ap.add_argument("--host-wait-us", type=int, default=-1,
                    help="pipelined step: longest the calling thread polls for a batch's index "
                         "work instead of making the training stream wait for it (0: never; "
                         "-1: the library's choice)")
    ap.add_argument("--issue-thread", type=int, default=-1,
                    help="pipelined step: enqueue the index work from the library's own host "
                         "threads (ss_issue_queue), that many; 0: none; -1: PipelinedStep's own choice")
    ap.add_argument("--serial", action="store_true",
                    help="issue every call of a batch on one stream, one batch after the other "
                         "(EmbeddingStep).  Default: PipelinedStep, which classifies and groups "
                         "the coming batches on a second stream while the current one is in its "
                         "forward and update kernels")
    ap.add_argument("--start-empty", action="store_true",
                    help="pipelined step: submit no index work beyond the last batch of a timed "
                         "region, so that every region starts from an empty pipeline (default: "
                         "the pipeline keeps its lead across regions, and a region holds the "
                         "index work of as many batches as it trains on, the ones further on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prime", action="store_true",
                    help="diagnostic: leave out the untimed priming batches that precede the "
                         "warm-up (two snapshot periods and once round the pipeline's ring), "
                         "so that whatever happens once lands in the warm-up or the timed region")
    ap.add_argument("--no-extra-configs", action="store_true",
                    help="only the workload named by --config: leave out the sub-records of "
                         "the multi-hot workload and of the headline workload with all hot "
                         "rows frozen")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="leave out the measured ceilings (device copy, rows at random places): "
                         "their launches would be averaged into a profiler's per-kernel figures")
    ap.add_argument("--extra-steps", type=int, default=1000,
                    help="timed steps of each sub-record (at least --steps)")
    ap.add_argument("--permute", action="store_true",
                    help="map rank -> row through a per-table random permutation (hot rows "
                         "scattered over the table as in real data; config 2 always does)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy (calibrates rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters against a known size)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--sampling-probe", type=int, default=0, metavar="S",
                    help="after the timed steps, also time the sampling block (drift of "
                         "the hot rows once, then drop counts of S sampled inputs for 32 "
                         "candidate thresholds in one pass) and report it beside the step")
    ap.add_argument("--hotset-probe", action="store_true",
                    help="after the timed steps, also time the hot-set identification "
                         "(access counters over the ring of batches, then the top-H rows "
                         "of every table) and report it beside the step")
    ap.add_argument("--timeline", type=int, default=0, metavar="N",
                    help="after the timed steps, run N more steps in trace mode (the kernels stamp "
                         "the GPU clock themselves, the pipeline runs at its own pace) and report "
                         "durations, gaps and overlap of the training stream's kernels")
    ap.add_argument("--timeline-dump", default=None, metavar="FILE",
                    help="with --timeline: also write every traced launch to FILE, one line each: "
                         "kernel, start and end in ns of the GPU clock")
    ap.add_argument("--row-gather-probe", action="store_true",
                    help="after the timed steps, take the access pattern of the lookup and update "
                         "kernels apart (cold Zipf batches, their distinct rows once each, uniform "
                         "random rows, cache-resident rows, the head of the distribution removed)")
    ap.add_argument("--layernorm-probe", action="store_true",
                    help="after the timed steps, also time LayerNorm forward and backward "
                         "over the pooled vectors of one batch")
    return ap.parse_args()


def unique_rows_per_batch(idx_ring):
    """Mean over the ring of sum over tables of #distinct rows in a batch."""
    tot = 0
    for k in range(idx_ring.shape[0]):
        for t in range(idx_ring.shape[1]):
            tot += np.unique(idx_ring[k, t]).size
    return tot / idx_ring.shape[0]


def prime_batches(step, pipelined, K):
    """Untimed batches run before the warm-up, whatever --warmup says: enough for
    everything that happens once to have happened.  Two snapshot periods (the first
    ends with the capture, the second with the first detect pass) and, for the
    pipelined step, once round the ring of buffer sets plus one more event period,
    so that every set has been used, both streams have recorded events and waited
    for the other's, and the pools the runtime grows on demand (events, completion
    signals, kernel-argument memory) are at their steady size."""
    if not pipelined:
        return 2 * K + 1
    return 2 * K + len(step.sets) + step.every


class Measurement:
    """One workload set up on the device, and the timed runs over it."""

    def __init__(self, args, config_no, threshold):
        import torch
        from paper_2404_04270_amd import workload as wl
        from paper_2404_04270_amd.step import EmbeddingStep, PipelinedStep
        self.torch, self.args = torch, args
        dev = torch.device("cuda:0")
        cfg = wl.CONFIGS[config_no]
        if args.permute and not cfg.permute:
            cfg = cfg.scaled(permute=True, name=cfg.name + "_permuted")
        if args.snapshot_every > 0:
            cfg = cfg.scaled(snapshot_every=args.snapshot_every)
        self.cfg = cfg
        self.thr = cfg.threshold if threshold is None else threshold
        T, R, Bn, L = cfg.num_tables, cfg.rows, cfg.batch, cfg.bag
        self.w = w = wl.Workload(cfg)
        t0 = time.time()
        self.idx_ring = w.indices(0, args.ring)                     # [ring, T, B, L]
        self.hot = wl.hot_set(self.idx_ring, R, cfg.hot_rows)
        weights = [w.weights_device(t, dev) for t in range(T)]
        self.idx_d = torch.from_numpy(self.idx_ring).to(dev)
        self.n_grads = max(1, args.grad_buffers)
        self.grads = [torch.from_numpy(w.grads(k)).to(dev) for k in range(self.n_grads)]
        hot_d = [torch.from_numpy(h).to(dev) for h in self.hot]
        self.pipelined = bool(args.pipeline)
        self.index_streams = args.index_streams if args.index_streams > 0 else \
            PipelinedStep.auto_streams(Bn, L, T, cfg.dim)
        if self.pipelined:
            self.step = PipelinedStep(
                weights, hot_d, Bn, L, cfg.lr, self.thr, cfg.snapshot_every,
                diagnostics=False, every=args.pipeline_every or None,
                index_streams=self.index_streams,
                issue_thread=None if args.issue_thread < 0 else int(args.issue_thread),
                host_wait_us=None if args.host_wait_us < 0 else args.host_wait_us)
        else:
            self.step = EmbeddingStep(weights, hot_d, Bn, L, cfg.lr, self.thr,
                                      cfg.snapshot_every, diagnostics=False,
                                      overlap=args.overlap,
                                      grouped_forward=args.grouped_forward)
        torch.cuda.synchronize()
        self.setup_s = time.time() - t0
        self.done = 0              # batches run so far (the next batch's number)
        self.submitted = 0         # batches whose index work has been submitted
        self.index_submitted_in_run = 0     # ... of them, by the last call of run()

    def run(self, n, stamps=None):
        """Exactly n more batches.  stamps: list that receives the host clock after
        each batch has been enqueued (no synchronisation)."""
        step, ring, grads, n_grads = self.step, self.args.ring, self.grads, self.n_grads
        idx_d, start = self.idx_d, self.done
        if self.pipelined:
            # Index work is submitted ahead of the batch being trained on, at most two new
            # batches per step: the lead grows to what the ring takes (room()) within a few
            # steps, and a run that starts with an empty pipeline does not spend its first
            # quarter millisecond enqueueing index work while the training stream has
            # nothing to do.  By default the pipeline keeps running across calls: a region
            # of n batches holds the lookup and update of those n batches and the index
            # work of the n batches that lie `lead` further on, as any stretch of a training
            # run does.  With --start-empty no index work is submitted beyond the region's
            # last batch, so every region begins with an empty pipeline and holds the index
            # work of exactly its own batches.
            end = start + n
            limit = end if self.args.start_empty else None
            nxt = max(self.submitted, start)
            for it in range(start, end):
                fresh = 0
                while (limit is None or nxt < limit) and step.room() > 0 and \
                        (fresh < 2 or nxt <= it):
                    step.submit(idx_d[nxt % ring])
                    nxt += 1
                    fresh += 1
                step.forward()
                step.backward(grads[it % n_grads])
                if stamps is not None:
                    stamps.append(time.perf_counter())
            self.index_submitted_in_run = nxt - max(self.submitted, start)
            self.submitted = nxt
            step.flush()
        else:
            for it in range(start, start + n):
                step.filter_forward(idx_d[it % ring])
                step.backward(grads[it % n_grads])
                if stamps is not None:
                    stamps.append(time.perf_counter())
            self.index_submitted_in_run = n
        self.done += n

    def timed(self, n):
        """n batches between two device synchronisations: host seconds, the same
        region between two events on the training stream (ms), and the host clock
        after every batch."""
        torch = self.torch
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        stamps = []
        # The interpreter's cyclic garbage collector stays out of the region: a full
        # collection takes 20-60 ms in a process that has imported torch (measured),
        # as long as twenty to forty steps of the default workload.
        gc_was_on = gc.isenabled()
        gc.disable()
        # torch creates an event's HIP object at its first record: not inside the region
        e0.record()
        e1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        e0.record()
        self.run(n, stamps)
        e1.record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t1
        if gc_was_on:
            gc.enable()
        return elapsed, e0.elapsed_time(e1), t1, stamps

    def kept_fraction(self):
        """Share of the submitted samples that were kept, over the batches whose
        counts are still on the device (the ring of buffer sets; the last batch for
        the serial step)."""
        step = self.step
        if self.pipelined:
            used = step.sets[:min(len(step.sets), self.done)]
            return float(sum(int(s.n_kept.item()) for s in used)) / (len(used) * self.cfg.batch)
        return int(step.n_kept.item()) / self.cfg.batch

    def distinct_rows(self):
        """Per batch, averaged over the ring and summed over tables, with the stale
        bitmaps as they are now: (distinct rows the kept samples look up, the
        distinct rows among them that are not stale, gradient rows the update needs =
        kept (table, sample) pairs with at least one lookup of a row that is not
        stale, share of samples kept).  The first is what the forward pass must read,
        the second what the update must read and write, the third what it must read
        of the gradients."""
        cfg = self.cfg
        stale = [np.unpackbits(b.cpu().numpy().view(np.uint8), bitorder="little")[:cfg.rows]
                 .astype(bool) for b in self.step.bits]
        any_stale = any(s.any() for s in stale)
        u_fwd = u_upd = g_rows = kept = 0.0
        for k in range(self.idx_ring.shape[0]):
            idx = self.idx_ring[k]                                   # [T, B, L]
            keep = np.ones(cfg.batch, dtype=bool)
            if any_stale:               # skipped: every lookup of the sample is stale
                all_stale = np.ones(cfg.batch, dtype=bool)
                for t in range(cfg.num_tables):
                    all_stale &= stale[t][idx[t]].all(axis=1)
                keep = ~all_stale
            kept += keep.mean()
            for t in range(cfg.num_tables):
                rows = np.unique(idx[t][keep])
                u_fwd += rows.size
                u_upd += rows.size - (int(stale[t][rows].sum()) if any_stale else 0)
                g_rows += int((~stale[t][idx[t][keep]]).any(axis=1).sum()) if any_stale \
                    else int(keep.sum())
        n = self.idx_ring.shape[0]
        return u_fwd / n, u_upd / n, g_rows / n, kept / n

    def record(self, steps, warmup, pieces=20):
        """Primes, warms up, times `steps` batches, then measures the spread and the
        per-kernel durations; returns the record of this workload."""
        torch, args, cfg, step = self.torch, self.args, self.cfg, self.step
        from paper_2404_04270_amd import binding as B
        T, R, D, Bn, L = cfg.num_tables, cfg.rows, cfg.dim, cfg.batch, cfg.bag
        n_prime = 0 if args.no_prime else prime_batches(step, self.pipelined,
                                                        cfg.snapshot_every)
        self.run(n_prime)
        # A full collection before the warm-up batches, none between them and the
        # region: the collector walks every object of the process, and the first
        # batch after it pays for the caches it has emptied (measured: 140-190 us of
        # host time for that batch instead of 35-45).
        gc.collect()
        gc.disable()
        self.run(warmup)
        c0 = step.counters() if self.pipelined else None
        elapsed, gpu_ms, t1, stamps = self.timed(steps)
        c1 = step.counters() if self.pipelined else None
        gc.enable()
        ms_per_step = 1e3 * elapsed / steps
        value = Bn * steps / elapsed
        per = np.diff(np.array([t1] + stamps)) * 1e6       # host time per batch, us
        timed_region = {
            "host_ms": 1e3 * elapsed, "gpu_event_ms": gpu_ms,
            "first_step_us": float(per[0]), "max_step_us": float(per.max()),
            "argmax": int(per.argmax()), "median_us": float(np.median(per)),
            "host_enqueue_done_ms": 1e3 * (stamps[-1] - t1),
            "note": "host clock after each batch was enqueued (no synchronisation): "
                    "what the calling thread spent per batch, not GPU time",
            "index_batches_submitted": self.index_submitted_in_run,
            # what the scheduler did in the region: wait commands it gave the training
            # stream for index work, and polls of the calling thread instead of them
            "scheduler": None if c0 is None else {k: c1[k] - c0[k] for k in c1},
            "pipeline": ("started empty: the region holds the index work of its own batches "
                         "and no other") if (not self.pipelined or self.args.start_empty) else
                        ("running: the training stream is drained by the synchronisation before "
                         "the region, the index work done ahead of it is kept; the region holds "
                         "the lookup and update of its %d batches and the index work of the %d "
                         "batches that lie %d further on" % (steps, self.index_submitted_in_run,
                                                            self.submitted - self.done))}
        stale_rows = int(sum(int(torch.count_nonzero(b).item()) for b in step.bits))
        kept_frac = self.kept_fraction()

        # spread of the step time: further pieces, each timed on its own (each starts
        # from a synchronisation), outside the timed region
        piece = max(1, min(200, steps))
        spread = sorted(1e6 * self.timed(piece)[0] / piece for _ in range(pieces))

        # host time per batch with the GPU left to run behind (no synchronisation
        # inside): what the calling thread needs to enqueue a batch
        host_us = float(np.median(np.diff(np.array(self.timed(piece)[3])))) * 1e6

        # The same number of steps from an empty pipeline: the batches submitted ahead
        # are trained on without submitting more, then a region submits its own index
        # work and no other (what --start-empty times in the main region).
        from_empty = None
        if self.pipelined and not self.args.start_empty:
            self.args.start_empty = True
            self.run(self.submitted - self.done)
            e_elapsed = self.timed(steps)[0]
            self.args.start_empty = False
            from_empty = {"steps": steps, "ms_per_step": 1e3 * e_elapsed / steps,
                          "value": Bn * steps / e_elapsed}

        # per-kernel durations: the same steps again, each launch bracketed by events
        n_prof = max(steps, 200)
        B.ss_profile_enable(True)
        self.run(n_prof)
        torch.cuda.synchronize()
        B.ss_profile_enable(False)
        prof = B.ss_profile_report()
        kern = {k: {"launches": n, "avg_us": 1e3 * ms / n, "total_ms": ms}
                for k, (n, ms) in prof.items()}

        # algorithmic bytes per launch (all tables are in one launch)
        U_fwd, U_upd, grad_rows, kept_host = self.distinct_rows()
        nnz = T * Bn * L
        row_b = D * 4
        alg = {
            "forward_kernel": U_fwd * row_b + nnz * 4 * kept_frac + T * Bn * row_b * kept_frac,
            "apply_kernel": grad_rows * row_b + nnz * 4 + 2 * U_upd * row_b,
        }
        alg["forward_group_kernel"] = alg["forward_kernel"]
        # the dominant kernel: most GPU time; kernels within 3 % of it count as tied (at
        # one-hot shapes forward and update are, and their order flips from run to run),
        # and among tied ones the kernel that moves more algorithmic bytes is named
        cands = [k for k in kern if k in alg]
        longest = max(kern[k]["total_ms"] for k in cands)
        dom = max((k for k in cands if kern[k]["total_ms"] >= 0.97 * longest),
                  key=lambda k: alg[k])

        def roof(k):
            ach = alg[k] / (kern[k]["avg_us"] * 1e-6) / 1e9
            traffic, src = measured_traffic(cfg.name, k, self.thr == cfg.threshold,
                                            self.thr == float("inf"))
            return {"achieved": ach, "frac": ach / HBM_PEAK_GBS,
                    "algorithmic_bytes_per_launch": alg[k],
                    "avg_kernel_us": kern[k]["avg_us"], "traffic": traffic,
                    "traffic_source": src}
        roofline = {"bound": "hbm", "kernel": dom, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        roofline.update(roof(dom))
        roofline_all = {k: roof(k) for k in kern if k in alg}
        step_bytes = alg["forward_kernel"] + alg["apply_kernel"]
        # "logical" bytes: every lookup counted as a row (nnz in place of the distinct rows)
        logical_bytes = (nnz * row_b + nnz * 4 + T * Bn * row_b) * kept_frac + \
                        (T * Bn * row_b * kept_frac + nnz * 4 + 2 * nnz * row_b * kept_frac)
        # (filter: < 2 % of the step's bytes; grouping and fixup carry no algorithmic bytes)
        med = 0.5 * (spread[(pieces - 1) // 2] + spread[pieces // 2])
        return {
            "value": value, "ms_per_step": ms_per_step, "steps": steps, "warmup": warmup,
            "primed_batches": n_prime,
            "config": {"workload": cfg.name, "tables": T, "rows": R, "dim": D, "batch": Bn,
                       "bag": L, "zipf_alpha": cfg.zipf_alpha, "threshold": self.thr,
                       "snapshot_every": cfg.snapshot_every, "ring": args.ring,
                       "grad_buffers": self.n_grads,
                       "streams": (1 + self.index_streams) if self.pipelined
                       else (2 if args.overlap else 1),
                       "pipelined": self.pipelined,
                       "pipeline_every": step.every if self.pipelined else None,
                       "issue_threads": len(step.queues) if self.pipelined else None,
                       "grouped_forward": bool(args.grouped_forward)},
            "timed_region": timed_region,
            "roofline": roofline, "roofline_all": roofline_all,
            "whole_step": {"algorithmic_bytes": step_bytes,
                           "achieved_GBs": step_bytes / (ms_per_step * 1e-3) / 1e9,
                           "frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9
                           / HBM_PEAK_GBS,
                           "frac_of_hbm_peak_at_spread_median": step_bytes / (med * 1e-6) / 1e9
                           / HBM_PEAK_GBS,
                           "logical_bytes": logical_bytes,
                           "effective_GBs": logical_bytes / (ms_per_step * 1e-3) / 1e9},
            "skip_fraction": 1.0 - kept_frac, "kept_samples_per_s": value * kept_frac,
            "stale_rows": stale_rows,
            "step_us_spread": {"pieces": pieces, "steps_per_piece": piece, "median": med,
                               "min": spread[0], "max": spread[-1]},
            "host_us_per_batch": host_us,
            "from_empty_pipeline": from_empty,
            "kernels": kern, "setup_s": self.setup_s,
        }

    def close(self):
        if self.pipelined:
            self.torch.cuda.synchronize()
            self.step.close()


def copy_rate(torch, dev):
    """What a plain device copy sustains in this process (512 MiB read + 512 MiB
    written): the ceiling the roofline fractions are also put against."""
    ca = torch.empty(1 << 27, dtype=torch.float32, device=dev).normal_()
    cb = torch.empty_like(ca)
    cb.copy_(ca)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        cb.copy_(ca)
    e1.record()
    torch.cuda.synchronize()
    return 5 * 2 * ca.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9


def random_row_rate(torch, B, m):
    """What gathers of random rows of this length sustain on this GPU, through the
    library's own lookup kernel: uniform random rows of the workload's tables (all
    distinct, so every row comes from HBM), eight times the lookups of a batch per
    launch, four index tensors in turn.  One-hot shapes move a row in and a row out
    per lookup, multi-hot ones L rows in per row out; both sides are counted."""
    cfg, dev = m.cfg, torch.device("cuda:0")
    T, R, D, L = cfg.num_tables, cfg.rows, cfg.dim, cfg.bag
    n = min(8 * cfg.batch, max(1, R // (2 * L)))
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    idx = [torch.randint(0, R, (T, n, L), dtype=torch.int32, device=dev, generator=gen)
           for _ in range(4)]
    out = torch.empty(T, n, D, dtype=torch.float32, device=dev)
    for k in range(4):
        B.ss_embbag_forward(m.step.tables, idx[k], None, out)
    torch.cuda.synchronize()
    B.ss_profile_enable(True)
    for k in range(8):
        B.ss_embbag_forward(m.step.tables, idx[k % 4], None, out)
    torch.cuda.synchronize()
    B.ss_profile_enable(False)
    launches, ms = B.ss_profile_report()["forward_kernel"]
    us = 1e3 * ms / launches
    moved = T * n * (L + 1) * D * 4 + T * n * L * 4
    return {"rows_per_launch": T * n * L, "row_bytes": D * 4, "kernel_us": us,
            "GBs": moved / us / 1e3}


def timeline(torch, B, m, n, dump=None):
    """The free-running pipeline seen by the kernels' own clock stamps: per kernel its
    mean duration, per pair of consecutive training-stream kernels the mean gap, and
    how much index-stream kernel time ran beside the training stream's kernels."""
    n = min(n, 32768 // 12)
    m.run(64)
    torch.cuda.synchronize()
    B.ss_profile_enable(2)
    t0 = time.perf_counter()
    m.run(n)
    torch.cuda.synchronize()
    wall_us = 1e6 * (time.perf_counter() - t0) / n
    ev = B.ss_profile_trace()
    if dump:            # every launch: kernel, first workgroup's start, last workgroup's end (ns)
        with open(dump, "w") as f:
            for k, a, b in ev:
                f.write(f"{k} {a} {b}\n")
    main_names = ("forward_kernel", "apply_kernel", "fixup_kernel", "detect_kernel")
    main = sorted((a, b, k) for k, a, b in ev if k in main_names)
    side = sorted((a, b, k) for k, a, b in ev if k not in main_names)
    main = main[len(main) // 8:]                      # past the start of the pipeline
    nb = sum(1 for e in main if e[2] == "apply_kernel")
    span_us = (main[-1][1] - main[0][0]) / 1e3
    dur, gaps = {}, {}
    for a, b, k in main:
        dur.setdefault(k, []).append((b - a) / 1e3)
    for x, y in zip(main, main[1:]):
        gaps.setdefault(x[2] + " -> " + y[2], []).append((y[0] - x[1]) / 1e3)
    side = [e for e in side if e[0] >= main[0][0] and e[1] <= main[-1][1]]
    sdur = {}
    for a, b, k in side:
        sdur.setdefault(k, []).append((b - a) / 1e3)

    def stats(v):
        v = sorted(v)
        return {"n": len(v), "mean_us": sum(v) / len(v), "median_us": v[len(v) // 2],
                "p90_us": v[len(v) * 9 // 10], "max_us": v[-1]}
    return {"steps_traced": n, "wall_us_per_step": wall_us, "batches_analysed": nb,
            "us_per_batch": span_us / max(1, nb),
            "training_stream_kernels": {k: stats(v) for k, v in dur.items()},
            "training_stream_gaps": {k: stats(v) for k, v in gaps.items()},
            "training_stream_busy_us_per_batch": sum(sum(v) for v in dur.values()) / max(1, nb),
            "training_stream_idle_us_per_batch": sum(sum(v) for v in gaps.values()) / max(1, nb),
            "index_stream_kernels": {k: stats(v) for k, v in sdur.items()}}


def row_gather_probe(torch, B, m):
    """Where the time of the lookup and update kernels goes at this workload: the
    same kernels on index tensors that take the access pattern apart.  Every case
    cycles through 16 different batches, so that rows are cold without a flush
    (a fill leaves dirty lines whose write-back would be charged to the kernel)."""
    cfg, dev = m.cfg, torch.device("cuda:0")
    T, R, D, Bn, L = cfg.num_tables, cfg.rows, cfg.dim, cfg.batch, cfg.bag
    NB = 16
    idx = m.w.indices(1000, NB)                                   # [NB, T, B, L]
    tables = B.Tables(m.step.tables.weights)                      # same weights, own bitmaps
    bits = tables.new_bits()
    rng = np.random.default_rng(5)

    def time_forward(batches, reps=2 * NB):
        d = [torch.from_numpy(np.ascontiguousarray(b)).to(dev) for b in batches]
        out = torch.empty(T, batches[0].shape[1], D, dtype=torch.float32, device=dev)
        for k in range(len(d)):
            B.ss_embbag_forward(tables, d[k], None, out)
        torch.cuda.synchronize()
        B.ss_profile_enable(True)
        for k in range(reps):
            B.ss_embbag_forward(tables, d[k % len(d)], None, out)
        torch.cuda.synchronize()
        B.ss_profile_enable(False)
        n, ms = B.ss_profile_report()["forward_kernel"]
        rows = float(np.mean([sum(np.unique(b[t]).size for t in range(T)) for b in batches[:4]]))
        return {"lookups": int(T * batches[0].shape[1] * batches[0].shape[2]),
                "distinct_rows": rows, "distinct_MB": rows * D * 4 / 1e6, "kernel_us": 1e3 * ms / n}

    out = {}
    zipf = [idx[k] for k in range(NB)]
    out["zipf_batches_cold"] = time_forward(zipf)
    out["zipf_batches_two_in_turn"] = time_forward(zipf[:2], reps=16)
    # the distinct rows of each batch, looked up once each (bags of L, random order)
    per = min(np.unique(idx[k, t]).size for k in range(NB) for t in range(T)) // L * L
    once = [np.stack([rng.permutation(np.unique(idx[k, t]))[:per].reshape(-1, L)
                      for t in range(T)]).astype(np.int32) for k in range(NB)]
    out["distinct_rows_once_each"] = time_forward(once)
    out["as_many_uniform_random_rows"] = time_forward(
        [rng.integers(0, R, once[0].shape).astype(np.int32) for _ in range(NB)])
    out["all_lookups_within_128_rows"] = time_forward(
        [(idx[k] % 128).astype(np.int32) for k in range(NB)])

    # the update with the most popular rows taken out (through the stale bitmap), and the
    # lookup with those lookups removed from the bags: what a separate path for the
    # head of the distribution could gain at most
    ws = torch.empty(B.ss_backward_workspace_bytes(T, Bn, L, D), dtype=torch.uint8, device=dev)
    idx_d = [torch.from_numpy(idx[k]).to(dev) for k in range(NB)]
    order = []                                                    # most popular rows per table
    for t in range(T):
        vals, cnt = np.unique(idx[:, t], return_counts=True)
        order.append(vals[np.argsort(-cnt, kind="stable")[:32]])
    backup = [w.clone() for w in tables.weights] if cfg.table_bytes < 8e9 else None
    for nh in (0, 8, 32):
        for t in range(T):
            bits[t].zero_()
            if nh:
                head = torch.from_numpy(order[t][:nh].astype(np.int64)).to(dev)
                flags = torch.zeros(bits[t].numel() * 32, dtype=torch.bool, device=dev)
                flags[head] = True
                words = (flags.view(-1, 32).to(torch.int64) << torch.arange(32, device=dev)).sum(1)
                bits[t].copy_(torch.where(words >= 2 ** 31, words - 2 ** 32, words).to(torch.int32))

        def update(k):
            B.ss_embbag_backward_prepare(tables, idx_d[k % NB], None, ws)
            B.ss_embbag_backward_apply(tables, Bn, L, m.grads[k % m.n_grads], cfg.lr, ws)
        for k in range(NB):
            update(k)
        torch.cuda.synchronize()
        B.ss_profile_enable(True)
        for k in range(2 * NB):
            update(k)
        torch.cuda.synchronize()
        B.ss_profile_enable(False)
        prof = B.ss_profile_report()
        rec = {"apply_us": 1e3 * prof["apply_kernel"][1] / prof["apply_kernel"][0],
               "fixup_us": 1e3 * prof["fixup_kernel"][1] / prof["fixup_kernel"][0]}
        if nh and L > 1:
            is_head = [np.isin(idx[:, t], order[t][:nh]) for t in range(T)]
            share = float(np.mean(is_head))
            Lr = max(1, int(round(L * (1 - share))))
            cold = np.empty((NB, T, Bn, Lr), np.int32)
            for k in range(NB):
                for t in range(T):
                    a = idx[k, t]
                    o = np.argsort(is_head[t][k], axis=1, kind="stable")    # other lookups first
                    srt = np.take_along_axis(a, o, axis=1)[:, :Lr]
                    hd = np.take_along_axis(is_head[t][k], o, axis=1)[:, :Lr]
                    first = np.where(hd[:, :1], (a[:, :1] + 1) % R, srt[:, :1])
                    cold[k, t] = np.where(hd, first, srt)     # short bags repeat a row of theirs
            rec["head_share_of_lookups"] = share
            rec["forward_without_head"] = time_forward([cold[k] for k in range(NB)])
        out["head_rows_removed_%d" % nh] = rec
    if backup is not None:
        for w, b in zip(tables.weights, backup):
            w.copy_(b)
    return out


def main():
    args = parse()
    args.pipeline = not (args.serial or args.overlap or args.grouped_forward)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
              "(no collectives or sharding are part of it)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2404_04270_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")

    if args.copy_probe:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    m = Measurement(args, args.config, args.threshold)
    rec = m.record(args.steps, args.warmup)
    if not args.no_ceilings:
        copy_gbs = copy_rate(torch, dev)
        rec["roofline"]["measured_copy_GBs"] = copy_gbs
        rec["roofline"]["frac_of_measured_copy"] = rec["roofline"]["achieved"] / copy_gbs
        # the other measured ceiling: rows of this length at random places, which is what
        # every kernel of the path reads and writes
        rows = random_row_rate(torch, B, m)
        rec["roofline"]["measured_random_rows"] = rows
        rec["roofline"]["frac_of_measured_random_rows"] = rec["roofline"]["achieved"] / rows["GBs"]

    out = {
        "metric": "train samples/s through embedding fwd+update+stale-skip; achieved HBM GB/s",
        "value": rec.pop("value"), "unit": "samples/s", "n_gpus": 1,
        "steps": rec.pop("steps"), "warmup": rec.pop("warmup"),
        "ms_per_step": rec.pop("ms_per_step"), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
    }
    out.update(rec)

    step, cfg = m.step, m.cfg
    if args.sampling_probe > 0:
        out["sampling_block"] = sampling_probe(B, step, m.idx_d, args.sampling_probe, m.thr)
    if args.timeline > 0:
        out["timeline"] = timeline(torch, B, m, args.timeline, args.timeline_dump)
    if args.row_gather_probe:
        out["row_gather_probe"] = row_gather_probe(torch, B, m)
    if args.layernorm_probe:
        out["layernorm"] = layernorm_probe(B, step, m.grads)
    if args.hotset_probe:
        out["hot_set"] = hotset_probe(B, step, m.idx_d, cfg.hot_rows, m.hot)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, m.w, m.idx_ring, m.hot, m.thr, args.cpu_seconds)
    m.close()
    headline = (args.config, m.thr)
    del m, step
    torch.cuda.empty_cache()

    # The other graded workload, and the headline workload with every hot row frozen
    # (the skip path busy), measured the same way in the same run.
    if not args.no_extra_configs:
        out["configs"] = []
        n_sub = max(args.steps, args.extra_steps)
        for config_no, thr in ((4, None), (3, float("inf"))):
            mm = Measurement(args, config_no, thr)
            if (config_no, mm.thr) == headline:
                mm.close()
                continue
            sub = mm.record(n_sub, args.warmup, pieces=10)
            sub["samples_per_s"] = sub.pop("value")
            out["configs"].append(sub)
            mm.close()
            del mm
            torch.cuda.empty_cache()
    print(json.dumps(out))


def layernorm_probe(B, step, grads):
    """Kernel durations and achieved HBM rates of the feature normalization."""
    import torch
    x = step.pooled
    T, Bn, D = x.shape
    dev = x.device
    gamma = torch.ones(T, D, device=dev)
    beta = torch.zeros(T, D, device=dev)
    y = torch.empty_like(x)
    dx = torch.empty_like(x)
    mean = torch.empty(T, Bn, device=dev)
    rstd = torch.empty(T, Bn, device=dev)
    dgamma, dbeta = torch.empty(T, D, device=dev), torch.empty(T, D, device=dev)
    ws = torch.empty(max(256, B.ss_layernorm_backward_workspace_bytes(T, D, Bn)),
                     dtype=torch.uint8, device=dev)

    def once(k):
        B.ss_layernorm_forward(x, step.n_kept, gamma, beta, 1e-5, y, mean, rstd)
        B.ss_layernorm_backward(grads[k % len(grads)], x, step.n_kept, gamma, mean, rstd, dx,
                                dgamma, dbeta, ws)
        # the same two passes with the pooled vectors formed from the tables on the fly
        B.ss_embbag_forward_ln(step.tables, step.idx_c, step.n_kept, gamma, beta, 1e-5, y,
                               mean, rstd)
        B.ss_embbag_ln_backward(step.tables, step.idx_c, step.n_kept, grads[k % len(grads)],
                                gamma, mean, rstd, dx, dgamma, dbeta, ws)
    for k in range(5):
        once(k)
    torch.cuda.synchronize()
    B.ss_profile_enable(True)
    for k in range(40):
        once(k)
    torch.cuda.synchronize()
    B.ss_profile_enable(False)
    prof = B.ss_profile_report()
    kept = int(step.n_kept.item())
    elems = T * kept * D
    fwd_us = 1e3 * prof["ln_forward_kernel"][1] / prof["ln_forward_kernel"][0]
    bwd_us = 1e3 * prof["ln_backward_kernel"][1] / prof["ln_backward_kernel"][0]
    pf_us = 1e3 * prof["ln_forward_pool_kernel"][1] / prof["ln_forward_pool_kernel"][0]
    pb_us = 1e3 * prof["ln_backward_pool_kernel"][1] / prof["ln_backward_pool_kernel"][0]
    return {"forward_us": fwd_us, "forward_GBs": 8 * elems / fwd_us / 1e3,
            "backward_us": bwd_us, "backward_GBs": 12 * elems / bwd_us / 1e3,
            "algorithmic_bytes": {"forward": 8 * elems, "backward": 12 * elems},
            "pooled_in_one_pass": {"forward_us": pf_us, "backward_us": pb_us}}


def hotset_probe(B, step, idx_d, H, hot_ref):
    """Durations of counting and selecting on the device, checked against the
    hot set the harness derived on the host from the same ring of batches."""
    import torch
    T, R, dev = step.tables.num_tables, step.tables.rows, step.tables.device
    ring = idx_d.shape[0]
    ac = B.AccessCounters(T, R, dev)
    ws = torch.empty(max(256, B.ss_select_hot_workspace_bytes(T, R)), dtype=torch.uint8,
                     device=dev)
    ids = [torch.zeros(H, dtype=torch.int32, device=dev) for _ in range(T)]
    for k in range(ring):                                    # warm-up and the real counts
        B.ss_count_accesses(ac, idx_d[k])
    B.ss_select_hot_top(ac, H, ids, None, ws)
    torch.cuda.synchronize()
    same = all(torch.equal(ids[t].cpu(), torch.from_numpy(hot_ref[t])) for t in range(T))
    scratch = B.AccessCounters(T, R, dev)
    B.ss_profile_enable(True)
    for k in range(ring):
        B.ss_count_accesses(scratch, idx_d[k])
    torch.cuda.synchronize()
    B.ss_profile_enable(False)
    prof = B.ss_profile_report()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 5
    e0.record()
    for _ in range(reps):
        B.ss_select_hot_top(ac, H, ids, None, ws)
    e1.record()
    torch.cuda.synchronize()
    return {"hot_rows_per_table": H, "matches_host_rule": bool(same),
            "count_pass_us_per_batch": 1e3 * prof["count_kernel"][1] / prof["count_kernel"][0],
            "select_top_us": 1e3 * e0.elapsed_time(e1) / reps,
            "counter_bytes": 4 * T * R}


def sampling_probe(B, step, idx_d, S, thr):
    """Kernel durations of the sampling block on the state the steps left behind."""
    import torch
    from paper_2404_04270_amd.sampling import SamplingBlock, geometric_ladder
    T = step.tables.num_tables
    ring, _, Bn, L = idx_d.shape
    S = min(S, ring * Bn)
    # the first S inputs of the ring, as one [T, S, L] array
    sidx = idx_d.permute(1, 0, 2, 3).reshape(T, ring * Bn, L)[:, :S].contiguous()
    hot = B.HotState(step.tables, step.hot.hot_ids, diagnostics=True)
    for dst, src in zip(hot.snapshot, step.hot.snapshot):
        dst.copy_(src)
    blk = SamplingBlock(step.tables, hot, sidx, alpha=T * L, population=ring * Bn)
    centre = thr if 0 < thr < float("inf") else 1e-3
    ladder = geometric_ladder(centre / 30, centre * 30, B.MAX_THRESHOLDS)
    reps = 20
    blk.refresh_drift()
    blk.counts_for(ladder)                                   # warm-up
    B.ss_profile_enable(True)
    for _ in range(reps):
        blk.refresh_drift()
        B.ss_sample_drop(hot, sidx, blk.alpha, ladder, blk.counts)
    torch.cuda.synchronize()
    B.ss_profile_enable(False)
    prof = B.ss_profile_report()
    counts = blk.counts_for(ladder)
    return {"samples": S, "thresholds": len(ladder), "alpha": blk.alpha,
            "hot_rows_per_table": hot.H,
            "drift_pass_us": 1e3 * prof["detect_kernel"][1] / prof["detect_kernel"][0],
            "count_pass_us": 1e3 * prof["sample_drop_kernel"][1] / prof["sample_drop_kernel"][0],
            "counts_first_last": [counts[0], counts[-1]]}


def measured_traffic(workload, kernel, default_threshold=True, frozen=False):
    """(HBM bytes per launch of `kernel`, where the figure comes from): FETCH_SIZE +
    WRITE_SIZE from the committed rocprofv3 counter summary of this workload, each
    already scaled by the copy-kernel calibration.  The counters are not collected
    in this run; (None, reason) if no committed summary covers the kernel."""
    if not default_threshold and not frozen:
        return None, "no committed counter summary for this threshold"
    name = "hbm_traffic_%s%s.txt" % (workload, "_hot_rows_frozen" if frozen else "")
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, "no committed counter summary for this workload"
    for line in open(path):
        f = line.split()
        if len(f) == 4 and f[0] == kernel:
            return float(f[3]), "profiles/" + name + " (rocprofv3 --pmc, separate runs)"
    return None, "profiles/" + name + " has no line for this kernel"


def cpu_baseline(cfg, w, idx_ring, hot, thr, budget_s):
    """The oracle as it stands, on this machine's host cores: one thread (the
    reported baseline), and, as a second figure, the same calls with the tables
    dealt to a pool of threads (the tables of a step are independent but for the
    classifier, which looks at all lookups of a sample and stays on one thread)."""
    from concurrent.futures import ThreadPoolExecutor

    import oracle
    from oracle.protocol import OracleRun
    T = cfg.num_tables

    def tables():
        if cfg.table_bytes <= 8e9:
            return [w.weights(t) for t in range(T)]
        rng = np.random.default_rng(cfg.seed)
        out = []
        for t in range(T):
            a = np.empty((cfg.rows, cfg.dim), dtype=np.float32)
            a[:] = rng.uniform(-cfg.init_bound, cfg.init_bound, cfg.dim).astype(np.float32)
            out.append(a)
        return out
    W = tables()
    run = OracleRun(W, hot, cfg.lr, thr, cfg.snapshot_every)
    g = [w.grads(k) for k in range(2)]
    run.step(idx_ring[0], g[0])                       # warm-up (page faults)
    t0 = time.perf_counter()
    n = 0
    while True:
        run.step(idx_ring[(n + 1) % idx_ring.shape[0]], g[n % 2])
        n += 1
        el = time.perf_counter() - t0
        if el >= budget_s or n >= 2000:
            break
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    out = {"value": cfg.batch * n / el, "unit": "samples/s", "cores": 1,
           "kind": "oracle", "host_nproc": os.cpu_count(), "host_cpu": model,
           "sample": "%d iterations of the same workload after 1 warm-up, "
                     "single thread, %.1f s" % (n, el)}

    # second figure: tables dealt to threads (lookup and update only; the period of the
    # sample holds no detect pass), a third of the budget
    workers = max(1, min(T, 16, os.cpu_count() or 1))
    if workers > 1:
        bits = [np.zeros((cfg.rows + 31) // 32, dtype=np.uint32) for _ in range(T)]
        alpha = T * cfg.bag

        def one_table(t, idx_c, g_c, n_kept):
            oracle.embbag_forward(W[t:t + 1], idx_c[t:t + 1], n_kept)
            oracle.embbag_backward_update(W[t:t + 1], bits[t:t + 1], idx_c[t:t + 1],
                                          g_c[t:t + 1], cfg.lr, n_kept)
        with ThreadPoolExecutor(max_workers=workers) as pool:
            t0 = time.perf_counter()
            m = 0
            while True:
                idx = idx_ring[m % idx_ring.shape[0]]
                _, kept, idx_c = oracle.filter_batch(cfg.rows, bits, idx, alpha)
                g_c = g[m % 2]                        # nothing is stale: every sample is kept
                list(pool.map(lambda t: one_table(t, idx_c, g_c, kept.shape[0]), range(T)))
                m += 1
                el2 = time.perf_counter() - t0
                if el2 >= budget_s / 3 or m >= 2000:
                    break
        out["tables_over_threads"] = {
            "value": cfg.batch * m / el2, "unit": "samples/s", "cores": workers,
            "sample": "%d iterations (classifier on one thread, lookup and update of the "
                      "tables on %d threads), %.1f s" % (m, workers, el2)}
    return out


if __name__ == "__main__":
    main()
