"""Thin ctypes binding of libslipstream.so (include/slipstream.h).

Argument marshalling only: every step of the path runs in the HIP kernels
behind the C ABI.  PyTorch supplies device memory and the current stream.
There is no fallback: if the library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.environ.get("SLIPSTREAM_LIB", os.path.join(_HERE, "libslipstream.so"))

SYMBOLS = (
    "ss_last_error", "ss_filter_batch", "ss_filter_batch_workspace_bytes",
    "ss_embbag_forward", "ss_embbag_backward_update",
    "ss_backward_workspace_bytes", "ss_detect_stale", "ss_profile_enable",
    "ss_profile_report", "ss_embbag_backward_prepare", "ss_embbag_backward_apply",
    "ss_embbag_forward_grouped", "ss_sample_drop", "ss_drop_stats",
    "ss_count_accesses", "ss_select_hot_workspace_bytes", "ss_select_hot_ratio",
    "ss_select_hot_top", "ss_layernorm_forward", "ss_layernorm_backward",
    "ss_layernorm_backward_workspace_bytes", "ss_embbag_forward_ln",
    "ss_embbag_ln_backward", "ss_issue_queue_create", "ss_issue_queue_destroy",
    "ss_issue_index_batch", "ss_issue_wait_event", "ss_issue_record_event",
    "ss_issue_wait", "ss_event_create", "ss_event_destroy", "ss_event_record",
    "ss_stream_wait_event", "ss_embbag_backward_update_noalloc",
    "ss_check_indices", "ss_check_enable",
    "ss_step_plan_for", "ss_step_create", "ss_step_destroy", "ss_step_room",
    "ss_step_submit", "ss_step_forward", "ss_step_backward", "ss_step_flush",
    "ss_step_create_traced", "ss_filter_batch_split", "ss_profile_trace",
    "ss_step_counters",
)


class SlipstreamError(RuntimeError):
    pass


class _CTables(C.Structure):
    _fields_ = [("num_tables", C.c_int32), ("dim", C.c_int32),
                ("rows", C.c_int64), ("weights", C.c_void_p),
                ("stale_bits", C.c_void_p)]


def _load():
    if not os.path.exists(lib_path):
        raise SlipstreamError(
            f"{lib_path} is missing: build it with "
            "`python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no CPU fallback)")
    lib = C.CDLL(lib_path)
    lib.ss_last_error.restype = C.c_char_p
    lib.ss_filter_batch_workspace_bytes.restype = C.c_size_t
    lib.ss_backward_workspace_bytes.restype = C.c_size_t
    lib.ss_select_hot_workspace_bytes.restype = C.c_size_t
    lib.ss_layernorm_backward_workspace_bytes.restype = C.c_size_t
    lib.ss_profile_enable.restype = None
    for n in ("ss_filter_batch", "ss_embbag_forward",
              "ss_embbag_backward_update", "ss_detect_stale",
              "ss_profile_report", "ss_embbag_backward_prepare",
              "ss_embbag_backward_apply", "ss_embbag_forward_grouped",
              "ss_sample_drop", "ss_drop_stats", "ss_count_accesses",
              "ss_select_hot_ratio", "ss_select_hot_top", "ss_layernorm_forward",
              "ss_layernorm_backward", "ss_embbag_forward_ln", "ss_embbag_ln_backward",
              "ss_issue_queue_create", "ss_issue_queue_destroy", "ss_issue_index_batch",
              "ss_issue_wait_event", "ss_issue_record_event", "ss_issue_wait",
              "ss_event_create", "ss_event_destroy", "ss_event_record",
              "ss_stream_wait_event", "ss_embbag_backward_update_noalloc",
              "ss_check_indices", "ss_step_plan_for", "ss_step_create", "ss_step_destroy",
              "ss_step_room", "ss_step_submit", "ss_step_forward", "ss_step_backward",
              "ss_step_flush", "ss_step_create_traced", "ss_filter_batch_split",
              "ss_profile_trace", "ss_step_counters"):
        getattr(lib, n).restype = C.c_int32
    lib.ss_check_enable.restype = None
    return lib


_lib = _load()


def _check(rc: int):
    if rc != 0:
        raise SlipstreamError(
            f"[{rc}] " + _lib.ss_last_error().decode("utf-8", "replace"))


def ss_last_error() -> str:
    return _lib.ss_last_error().decode("utf-8", "replace")


def ss_check_enable(on: bool) -> None:
    """Checked mode: ids are range-checked (with a host synchronisation) before
    every call that takes them; out-of-range ids raise instead of faulting."""
    _lib.ss_check_enable(C.c_int32(int(on)))


def ss_check_indices(num_tables: int, rows: int, idx: torch.Tensor,
                     n_valid: Optional[torch.Tensor], report: torch.Tensor,
                     stream=None) -> None:
    """report: int64 [2] on the device: (number of out-of-range entries,
    table << 32 | position of the first one, or -1)."""
    if idx.dim() != 3 or idx.shape[0] != num_tables:
        raise SlipstreamError("ss_check_indices: idx must be [T, B, L]")
    if report.numel() < 2:
        raise SlipstreamError("ss_check_indices: report needs two words")
    _check(_lib.ss_check_indices(
        C.c_int32(num_tables), C.c_int64(rows), _dev_ptr(idx, torch.int32, "idx"),
        C.c_int32(idx.shape[1]), C.c_int32(idx.shape[2]),
        _dev_ptr(n_valid, torch.int32, "n_valid"), _dev_ptr(report, torch.int64, "report"),
        _stream(stream)))


def ss_profile_enable(on) -> None:
    """False / 0: off; True / 1: an event pair per launch (ss_profile_report);
    2: trace mode (ss_profile_trace)."""
    _lib.ss_profile_enable(C.c_int32(int(on)))


def ss_profile_trace() -> list:
    """[(kernel, start_ns, end_ns)] of the launches traced since ss_profile_enable(2),
    in launch order; stops tracing."""
    buf = C.create_string_buffer(4 << 20)
    _check(_lib.ss_profile_trace(buf, C.c_size_t(len(buf))))
    out = []
    for line in buf.value.decode().splitlines():
        k, a, b = line.split()
        out.append((k, int(a), int(b)))
    return out


def ss_profile_report() -> dict:
    """{kernel: (launches, total_ms)} since the last report."""
    buf = C.create_string_buffer(1 << 16)
    _check(_lib.ss_profile_report(buf, C.c_size_t(len(buf))))
    out = {}
    for line in buf.value.decode().splitlines():
        k, n, ms = line.split()
        out[k] = (int(n), float(ms))
    return out


def _dev_ptr(t: Optional[torch.Tensor], dtype, name: str) -> C.c_void_p:
    if t is None:
        return C.c_void_p(None)
    if not t.is_cuda:
        raise SlipstreamError(f"{name}: need a device tensor")
    if t.dtype != dtype:
        raise SlipstreamError(f"{name}: need dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise SlipstreamError(f"{name}: need a contiguous tensor")
    return C.c_void_p(t.data_ptr())


def _ptr_table(tensors: Sequence[torch.Tensor], device) -> torch.Tensor:
    return torch.tensor([t.data_ptr() for t in tensors], dtype=torch.int64,
                        device=device)


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


class Tables:
    """T embedding tables [R, D] fp32 in HBM plus their stale bitmaps.

    Holds the tensors alive together with the device arrays of pointers the
    library reads.  `bits` may be None (no stale row anywhere).
    """

    def __init__(self, weights: Sequence[torch.Tensor],
                 bits: Optional[Sequence[torch.Tensor]] = None):
        self.weights: List[torch.Tensor] = list(weights)
        w0 = self.weights[0]
        self.device = w0.device
        self.rows, self.dim = int(w0.shape[0]), int(w0.shape[1])
        for w in self.weights:
            _dev_ptr(w, torch.float32, "weights")
            if tuple(w.shape) != (self.rows, self.dim):
                raise SlipstreamError("weights: all tables need the same shape")
        self.num_tables = len(self.weights)
        self._wptr = _ptr_table(self.weights, self.device)
        self.bits: Optional[List[torch.Tensor]] = None
        self._bptr: Optional[torch.Tensor] = None
        if bits is not None:
            self.set_bits(bits)
        self._refresh_struct()

    @staticmethod
    def bitmap_words(rows: int) -> int:
        return (rows + 31) // 32

    def new_bits(self) -> List[torch.Tensor]:
        """Allocates zeroed bitmaps (int32 storage of the 32-bit words)."""
        bits = [torch.zeros(self.bitmap_words(self.rows), dtype=torch.int32,
                            device=self.device) for _ in range(self.num_tables)]
        self.set_bits(bits)
        return bits

    def set_bits(self, bits: Optional[Sequence[torch.Tensor]]):
        if bits is None:
            self.bits, self._bptr = None, None
        else:
            self.bits = list(bits)
            if len(self.bits) != self.num_tables:
                raise SlipstreamError("bits: one bitmap per table")
            for b in self.bits:
                _dev_ptr(b, torch.int32, "bits")
                if b.numel() < self.bitmap_words(self.rows):
                    raise SlipstreamError("bits: bitmap too short")
            self._bptr = _ptr_table(self.bits, self.device)
        self._refresh_struct()

    def _refresh_struct(self):
        self.c = _CTables(
            self.num_tables, self.dim, self.rows, self._wptr.data_ptr(),
            None if self._bptr is None else self._bptr.data_ptr())

    def struct_without_bits(self) -> _CTables:
        return _CTables(self.num_tables, self.dim, self.rows,
                        self._wptr.data_ptr(), None)


def ss_filter_batch_workspace_bytes(T: int, B: int, L: int) -> int:
    return int(_lib.ss_filter_batch_workspace_bytes(
        C.c_int32(T), C.c_int32(B), C.c_int32(L)))


def ss_backward_workspace_bytes(T: int, Bcap: int, L: int, dim: int) -> int:
    return int(_lib.ss_backward_workspace_bytes(
        C.c_int32(T), C.c_int32(Bcap), C.c_int32(L), C.c_int32(dim)))


def _idx_shape(tables: Tables, idx: torch.Tensor):
    if idx.dim() != 3 or idx.shape[0] != tables.num_tables:
        raise SlipstreamError("idx: need int32 [T, B, L]")
    return int(idx.shape[1]), int(idx.shape[2])


def ss_filter_batch(tables: Tables, idx: torch.Tensor, alpha: int,
                    skip_mask: torch.Tensor, kept_ids: torch.Tensor,
                    n_kept: torch.Tensor, idx_c: torch.Tensor,
                    ws: torch.Tensor, stream=None) -> None:
    B, L = _idx_shape(tables, idx)
    if skip_mask.numel() < B or kept_ids.numel() < B or n_kept.numel() < 1 \
            or idx_c.numel() < idx.numel():
        raise SlipstreamError("ss_filter_batch: an output tensor is too small")
    _check(_lib.ss_filter_batch(
        C.byref(tables.c), _dev_ptr(idx, torch.int32, "idx"), C.c_int32(B),
        C.c_int32(L), C.c_int32(alpha),
        _dev_ptr(skip_mask, torch.uint8, "skip_mask"),
        _dev_ptr(kept_ids, torch.int32, "kept_ids"),
        _dev_ptr(n_kept, torch.int32, "n_kept"),
        _dev_ptr(idx_c, torch.int32, "idx_c"),
        _dev_ptr(ws, torch.uint8, "ws"), C.c_size_t(ws.numel()),
        _stream(stream)))


def ss_filter_batch_split(tables: Tables, hot_bits: Optional[Sequence[torch.Tensor]],
                          idx: torch.Tensor, alpha: int, skip_mask: torch.Tensor,
                          hot_mask: torch.Tensor, kept_ids: torch.Tensor, n_kept: torch.Tensor,
                          idx_c: torch.Tensor, ws: torch.Tensor, stream=None) -> None:
    """ss_filter_batch plus hot_mask[b] = every lookup of sample b hits a row whose bit
    is set in hot_bits (T bitmaps in the layout of the stale bitmaps, or None)."""
    B, L = _idx_shape(tables, idx)
    if skip_mask.numel() < B or hot_mask.numel() < B or kept_ids.numel() < B \
            or n_kept.numel() < 1 or idx_c.numel() < idx.numel():
        raise SlipstreamError("ss_filter_batch_split: an output tensor is too small")
    hp = None
    if hot_bits is not None:
        if len(hot_bits) != tables.num_tables or any(
                b.numel() < Tables.bitmap_words(tables.rows) for b in hot_bits):
            raise SlipstreamError("ss_filter_batch_split: one bitmap of ceil(rows/32) words "
                                  "per table")
        hp = _opt_ptr_table(hot_bits, torch.int32, "hot_bits", tables.device)
    _check(_lib.ss_filter_batch_split(
        C.byref(tables.c), C.c_void_p(None if hp is None else hp.data_ptr()),
        _dev_ptr(idx, torch.int32, "idx"), C.c_int32(B), C.c_int32(L), C.c_int32(alpha),
        _dev_ptr(skip_mask, torch.uint8, "skip_mask"), _dev_ptr(hot_mask, torch.uint8, "hot_mask"),
        _dev_ptr(kept_ids, torch.int32, "kept_ids"), _dev_ptr(n_kept, torch.int32, "n_kept"),
        _dev_ptr(idx_c, torch.int32, "idx_c"), _dev_ptr(ws, torch.uint8, "ws"),
        C.c_size_t(ws.numel()), _stream(stream)))


def ss_embbag_forward(tables: Tables, idx: torch.Tensor,
                      n_valid: Optional[torch.Tensor], out: torch.Tensor,
                      stream=None) -> None:
    Bcap, L = _idx_shape(tables, idx)
    if out.numel() < tables.num_tables * Bcap * tables.dim:
        raise SlipstreamError("ss_embbag_forward: out is too small")
    _check(_lib.ss_embbag_forward(
        C.byref(tables.c), _dev_ptr(idx, torch.int32, "idx"), C.c_int32(Bcap),
        C.c_int32(L), _dev_ptr(n_valid, torch.int32, "n_valid"),
        _dev_ptr(out, torch.float32, "out"), _stream(stream)))


def ss_embbag_backward_update(tables: Tables, idx: torch.Tensor,
                              n_valid: Optional[torch.Tensor],
                              grad: torch.Tensor, lr: float, ws: torch.Tensor,
                              stream=None) -> None:
    Bcap, L = _idx_shape(tables, idx)
    if grad.numel() < tables.num_tables * Bcap * tables.dim:
        raise SlipstreamError("ss_embbag_backward_update: grad is too small")
    _check(_lib.ss_embbag_backward_update(
        C.byref(tables.c), _dev_ptr(idx, torch.int32, "idx"), C.c_int32(Bcap),
        C.c_int32(L), _dev_ptr(n_valid, torch.int32, "n_valid"),
        _dev_ptr(grad, torch.float32, "grad"), C.c_float(lr),
        _dev_ptr(ws, torch.uint8, "ws"), C.c_size_t(ws.numel()),
        _stream(stream)))


NOALLOC_SCRATCH_BYTES = 16 << 20


def ss_embbag_backward_update_noalloc(tables: Tables, idx: torch.Tensor,
                                      n_valid: Optional[torch.Tensor],
                                      grad: torch.Tensor, lr: float, stream=None) -> None:
    Bcap, L = _idx_shape(tables, idx)
    if grad.numel() < tables.num_tables * Bcap * tables.dim:
        raise SlipstreamError("ss_embbag_backward_update_noalloc: grad is too small")
    _check(_lib.ss_embbag_backward_update_noalloc(
        C.byref(tables.c), _dev_ptr(idx, torch.int32, "idx"), C.c_int32(Bcap),
        C.c_int32(L), _dev_ptr(n_valid, torch.int32, "n_valid"),
        _dev_ptr(grad, torch.float32, "grad"), C.c_float(lr), _stream(stream)))


def ss_embbag_backward_prepare(tables: Tables, idx: torch.Tensor,
                               n_valid: Optional[torch.Tensor], ws: torch.Tensor,
                               stream=None) -> None:
    Bcap, L = _idx_shape(tables, idx)
    _check(_lib.ss_embbag_backward_prepare(
        C.byref(tables.c), _dev_ptr(idx, torch.int32, "idx"), C.c_int32(Bcap),
        C.c_int32(L), _dev_ptr(n_valid, torch.int32, "n_valid"),
        _dev_ptr(ws, torch.uint8, "ws"), C.c_size_t(ws.numel()), _stream(stream)))


def ss_embbag_forward_grouped(tables: Tables, idx: torch.Tensor,
                              n_valid: Optional[torch.Tensor], out: torch.Tensor,
                              bwd_ws: torch.Tensor, stream=None) -> None:
    Bcap, L = _idx_shape(tables, idx)
    if out.numel() < tables.num_tables * Bcap * tables.dim:
        raise SlipstreamError("ss_embbag_forward_grouped: out is too small")
    _check(_lib.ss_embbag_forward_grouped(
        C.byref(tables.c), _dev_ptr(idx, torch.int32, "idx"), C.c_int32(Bcap),
        C.c_int32(L), _dev_ptr(n_valid, torch.int32, "n_valid"),
        _dev_ptr(out, torch.float32, "out"), _dev_ptr(bwd_ws, torch.uint8, "bwd_ws"),
        C.c_size_t(bwd_ws.numel()), _stream(stream)))


def ss_embbag_backward_apply(tables: Tables, Bcap: int, L: int, grad: torch.Tensor,
                             lr: float, ws: torch.Tensor, stream=None) -> None:
    if grad.numel() < tables.num_tables * Bcap * tables.dim:
        raise SlipstreamError("ss_embbag_backward_apply: grad is too small")
    _check(_lib.ss_embbag_backward_apply(
        C.byref(tables.c), C.c_int32(Bcap), C.c_int32(L),
        _dev_ptr(grad, torch.float32, "grad"), C.c_float(lr),
        _dev_ptr(ws, torch.uint8, "ws"), C.c_size_t(ws.numel()), _stream(stream)))


class HotState:
    """Hot row ids, their snapshots and the optional outputs of ss_detect_stale
    (per-slot verdicts and drifts, per-table counts of flagged rows), with the
    device pointer arrays the call needs.  Without diagnostics none of the
    optional outputs is produced: the counts cost one atomic per workgroup on one
    word per table, which is what a detect pass then mostly waits for once most
    hot rows are flagged (122 against 25 us at 8 tables x 10000 hot rows)."""

    def __init__(self, tables: Tables, hot_ids: Sequence[torch.Tensor],
                 diagnostics: bool = True):
        dev = tables.device
        self.hot_ids = list(hot_ids)
        self.H = int(self.hot_ids[0].numel())
        T = tables.num_tables
        for h in self.hot_ids:
            _dev_ptr(h, torch.int32, "hot_ids")
            if h.numel() != self.H:
                raise SlipstreamError("hot_ids: same H for every table")
        self.snapshot = [torch.zeros(self.H, tables.dim, dtype=torch.float32,
                                     device=dev) for _ in range(T)]
        self.stale_count = (torch.zeros(T, dtype=torch.int32, device=dev)
                            if diagnostics else None)
        self._hptr = _ptr_table(self.hot_ids, dev)
        self._sptr = _ptr_table(self.snapshot, dev)
        self.stale_hot = self.drift = None
        self._shptr = self._dptr = None
        if diagnostics:
            self.stale_hot = [torch.zeros(self.H, dtype=torch.uint8, device=dev)
                              for _ in range(T)]
            self.drift = [torch.zeros(self.H, dtype=torch.float64, device=dev)
                          for _ in range(T)]
            self._shptr = _ptr_table(self.stale_hot, dev)
            self._dptr = _ptr_table(self.drift, dev)


def ss_detect_stale(tables: Tables, hot: HotState, threshold: float,
                    refresh_snapshot: bool = True, stream=None) -> None:
    _check(_lib.ss_detect_stale(
        C.byref(tables.c), C.c_void_p(hot._hptr.data_ptr()), C.c_int32(hot.H),
        C.c_void_p(hot._sptr.data_ptr()), C.c_float(threshold),
        C.c_int32(int(refresh_snapshot)),
        C.c_void_p(None if hot._shptr is None else hot._shptr.data_ptr()),
        C.c_void_p(None if hot._dptr is None else hot._dptr.data_ptr()),
        _dev_ptr(hot.stale_count, torch.int32, "stale_count"), _stream(stream)))


MAX_THRESHOLDS = 32


def ss_sample_drop(hot: HotState, sidx: torch.Tensor, alpha: int,
                   thresholds: Sequence[float], counts: torch.Tensor,
                   stream=None) -> None:
    """sidx int32 [T, S, L]; counts int32 [len(thresholds)] (32-bit words of the
    unsigned counts); reads hot.drift as left by ss_detect_stale."""
    if hot.drift is None:
        raise SlipstreamError("ss_sample_drop: HotState was built without diagnostics")
    if sidx.dim() != 3 or sidx.shape[0] != len(hot.hot_ids):
        raise SlipstreamError("ss_sample_drop: sidx must be [T, S, L]")
    thr = (C.c_float * len(thresholds))(*[float(x) for x in thresholds])
    if counts.numel() < len(thresholds):
        raise SlipstreamError("ss_sample_drop: counts is shorter than thresholds")
    _check(_lib.ss_sample_drop(
        C.c_int32(len(hot.hot_ids)), C.c_void_p(hot._hptr.data_ptr()),
        C.c_int32(hot.H), C.c_void_p(hot._dptr.data_ptr()),
        _dev_ptr(sidx, torch.int32, "sidx"), C.c_int32(sidx.shape[1]),
        C.c_int32(sidx.shape[2]), C.c_int32(alpha), thr,
        C.c_int32(len(thresholds)), _dev_ptr(counts, torch.int32, "counts"),
        _stream(stream)))


_STAT_KEYS = ("D", "sd", "half", "lo", "hi", "D_bar", "D_bar_lo", "D_bar_hi")


def ss_drop_stats(count: int, n_samples: int, population: int, n_hot_inputs: int,
                  t_crit: float) -> dict:
    out = (C.c_double * 8)()
    _check(_lib.ss_drop_stats(C.c_uint32(count), C.c_int64(n_samples),
                              C.c_int64(population), C.c_int64(n_hot_inputs),
                              C.c_double(t_crit), out))
    return dict(zip(_STAT_KEYS, list(out)))


class AccessCounters:
    """uint32 counters [rows] per table (int32 storage) and their pointer array."""

    def __init__(self, num_tables: int, rows: int, device, counts=None):
        """counts: existing int32 tensors [rows], one per table (e.g. views of one
        allocation); allocated and zeroed when omitted."""
        self.rows, self.device = int(rows), device
        if counts is None:
            counts = [torch.zeros(rows, dtype=torch.int32, device=device)
                      for _ in range(num_tables)]
        self.counts = list(counts)
        if len(self.counts) != num_tables:
            raise SlipstreamError("AccessCounters: one counter array per table")
        for c in self.counts:
            _dev_ptr(c, torch.int32, "counts")
            if c.numel() != self.rows:
                raise SlipstreamError("AccessCounters: each array needs `rows` entries")
        self._cptr = _ptr_table(self.counts, device)


def _opt_ptr_table(tensors, dtype, name, device):
    if tensors is None:
        return None
    for x in tensors:
        _dev_ptr(x, dtype, name)
    return _ptr_table(tensors, device)


def ss_count_accesses(counters: AccessCounters, idx: torch.Tensor,
                      n_valid: Optional[torch.Tensor] = None, stream=None) -> None:
    if idx.dim() != 3 or idx.shape[0] != len(counters.counts):
        raise SlipstreamError("ss_count_accesses: idx must be [T, B, L]")
    _check(_lib.ss_count_accesses(
        C.c_int32(len(counters.counts)), C.c_int64(counters.rows),
        _dev_ptr(idx, torch.int32, "idx"), C.c_int32(idx.shape[1]),
        C.c_int32(idx.shape[2]), _dev_ptr(n_valid, torch.int32, "n_valid"),
        C.c_void_p(counters._cptr.data_ptr()), _stream(stream)))


def ss_select_hot_workspace_bytes(T: int, rows: int) -> int:
    return int(_lib.ss_select_hot_workspace_bytes(C.c_int32(T), C.c_int64(rows)))


def ss_select_hot_ratio(counters: AccessCounters, lam: float, total: int,
                        hot_ids: Optional[Sequence[torch.Tensor]],
                        hot_bits: Optional[Sequence[torch.Tensor]],
                        n_hot: Optional[torch.Tensor], ws: torch.Tensor,
                        stream=None) -> None:
    """hot_ids: T int32 tensors of one length (the cap), or None."""
    dev = counters.device
    T = len(counters.counts)
    cap = 0 if hot_ids is None else int(hot_ids[0].numel())
    if hot_ids is not None and any(h.numel() != cap for h in hot_ids):
        raise SlipstreamError("ss_select_hot_ratio: hot_ids need one length")
    if hot_bits is not None and any(b.numel() < Tables.bitmap_words(counters.rows)
                                    for b in hot_bits):
        raise SlipstreamError("ss_select_hot_ratio: bitmap too short")
    if n_hot is not None and n_hot.numel() < T:
        raise SlipstreamError("ss_select_hot_ratio: n_hot is shorter than T")
    ip = _opt_ptr_table(hot_ids, torch.int32, "hot_ids", dev)
    bp = _opt_ptr_table(hot_bits, torch.int32, "hot_bits", dev)
    _check(_lib.ss_select_hot_ratio(
        C.c_int32(T), C.c_int64(counters.rows), C.c_void_p(counters._cptr.data_ptr()),
        C.c_double(lam), C.c_int64(total), C.c_int32(cap),
        C.c_void_p(None if ip is None else ip.data_ptr()),
        C.c_void_p(None if bp is None else bp.data_ptr()),
        _dev_ptr(n_hot, torch.int32, "n_hot"), _dev_ptr(ws, torch.uint8, "ws"),
        C.c_size_t(ws.numel()), _stream(stream)))


def ss_select_hot_top(counters: AccessCounters, H: int,
                      hot_ids: Optional[Sequence[torch.Tensor]],
                      hot_bits: Optional[Sequence[torch.Tensor]], ws: torch.Tensor,
                      stream=None) -> None:
    dev = counters.device
    T = len(counters.counts)
    if hot_ids is not None and any(h.numel() < H for h in hot_ids):
        raise SlipstreamError("ss_select_hot_top: hot_ids shorter than H")
    if hot_bits is not None and any(b.numel() < Tables.bitmap_words(counters.rows)
                                    for b in hot_bits):
        raise SlipstreamError("ss_select_hot_top: bitmap too short")
    ip = _opt_ptr_table(hot_ids, torch.int32, "hot_ids", dev)
    bp = _opt_ptr_table(hot_bits, torch.int32, "hot_bits", dev)
    _check(_lib.ss_select_hot_top(
        C.c_int32(T), C.c_int64(counters.rows), C.c_void_p(counters._cptr.data_ptr()),
        C.c_int32(H), C.c_void_p(None if ip is None else ip.data_ptr()),
        C.c_void_p(None if bp is None else bp.data_ptr()),
        _dev_ptr(ws, torch.uint8, "ws"), C.c_size_t(ws.numel()), _stream(stream)))


def _ln_shape(x: torch.Tensor):
    if x.dim() != 3:
        raise SlipstreamError("layernorm: need fp32 [T, Bcap, D]")
    return int(x.shape[0]), int(x.shape[1]), int(x.shape[2])


def ss_layernorm_forward(x: torch.Tensor, n_valid: Optional[torch.Tensor],
                         gamma: Optional[torch.Tensor], beta: Optional[torch.Tensor],
                         eps: float, y: torch.Tensor, mean: torch.Tensor,
                         rstd: torch.Tensor, stream=None) -> None:
    T, Bcap, D = _ln_shape(x)
    if y.shape != x.shape or mean.numel() < T * Bcap or rstd.numel() < T * Bcap:
        raise SlipstreamError("ss_layernorm_forward: an output tensor is too small")
    for p, name in ((gamma, "gamma"), (beta, "beta")):
        if p is not None and tuple(p.shape) != (T, D):
            raise SlipstreamError(f"ss_layernorm_forward: {name} must be [T, D]")
    _check(_lib.ss_layernorm_forward(
        C.c_int32(T), C.c_int32(D), _dev_ptr(x, torch.float32, "x"), C.c_int32(Bcap),
        _dev_ptr(n_valid, torch.int32, "n_valid"), _dev_ptr(gamma, torch.float32, "gamma"),
        _dev_ptr(beta, torch.float32, "beta"), C.c_float(eps),
        _dev_ptr(y, torch.float32, "y"), _dev_ptr(mean, torch.float32, "mean"),
        _dev_ptr(rstd, torch.float32, "rstd"), _stream(stream)))


def ss_layernorm_backward_workspace_bytes(T: int, dim: int, Bcap: int) -> int:
    return int(_lib.ss_layernorm_backward_workspace_bytes(
        C.c_int32(T), C.c_int32(dim), C.c_int32(Bcap)))


def ss_layernorm_backward(dy: torch.Tensor, x: torch.Tensor,
                          n_valid: Optional[torch.Tensor], gamma: Optional[torch.Tensor],
                          mean: torch.Tensor, rstd: torch.Tensor, dx: torch.Tensor,
                          dgamma: Optional[torch.Tensor], dbeta: Optional[torch.Tensor],
                          ws: Optional[torch.Tensor], stream=None) -> None:
    T, Bcap, D = _ln_shape(x)
    if dy.shape != x.shape or dx.shape != x.shape:
        raise SlipstreamError("ss_layernorm_backward: dy, x and dx need one shape")
    for p, name in ((gamma, "gamma"), (dgamma, "dgamma"), (dbeta, "dbeta")):
        if p is not None and tuple(p.shape) != (T, D):
            raise SlipstreamError(f"ss_layernorm_backward: {name} must be [T, D]")
    _check(_lib.ss_layernorm_backward(
        C.c_int32(T), C.c_int32(D), _dev_ptr(dy, torch.float32, "dy"),
        _dev_ptr(x, torch.float32, "x"), C.c_int32(Bcap),
        _dev_ptr(n_valid, torch.int32, "n_valid"), _dev_ptr(gamma, torch.float32, "gamma"),
        _dev_ptr(mean, torch.float32, "mean"), _dev_ptr(rstd, torch.float32, "rstd"),
        _dev_ptr(dx, torch.float32, "dx"), _dev_ptr(dgamma, torch.float32, "dgamma"),
        _dev_ptr(dbeta, torch.float32, "dbeta"), _dev_ptr(ws, torch.uint8, "ws"),
        C.c_size_t(0 if ws is None else ws.numel()), _stream(stream)))


def ss_embbag_forward_ln(tables: Tables, idx: torch.Tensor, n_valid: Optional[torch.Tensor],
                         gamma: Optional[torch.Tensor], beta: Optional[torch.Tensor],
                         eps: float, y: torch.Tensor, mean: torch.Tensor,
                         rstd: torch.Tensor, stream=None) -> None:
    Bcap, L = _idx_shape(tables, idx)
    T, D = tables.num_tables, tables.dim
    if tuple(y.shape) != (T, Bcap, D) or mean.numel() < T * Bcap or rstd.numel() < T * Bcap:
        raise SlipstreamError("ss_embbag_forward_ln: an output tensor has the wrong size")
    for p, name in ((gamma, "gamma"), (beta, "beta")):
        if p is not None and tuple(p.shape) != (T, D):
            raise SlipstreamError(f"ss_embbag_forward_ln: {name} must be [T, D]")
    _check(_lib.ss_embbag_forward_ln(
        C.byref(tables.c), _dev_ptr(idx, torch.int32, "idx"), C.c_int32(Bcap), C.c_int32(L),
        _dev_ptr(n_valid, torch.int32, "n_valid"), _dev_ptr(gamma, torch.float32, "gamma"),
        _dev_ptr(beta, torch.float32, "beta"), C.c_float(eps),
        _dev_ptr(y, torch.float32, "y"), _dev_ptr(mean, torch.float32, "mean"),
        _dev_ptr(rstd, torch.float32, "rstd"), _stream(stream)))


def ss_embbag_ln_backward(tables: Tables, idx: torch.Tensor, n_valid: Optional[torch.Tensor],
                          dy: torch.Tensor, gamma: Optional[torch.Tensor],
                          mean: torch.Tensor, rstd: torch.Tensor, dx: torch.Tensor,
                          dgamma: Optional[torch.Tensor], dbeta: Optional[torch.Tensor],
                          ws: Optional[torch.Tensor], stream=None) -> None:
    Bcap, L = _idx_shape(tables, idx)
    T, D = tables.num_tables, tables.dim
    if tuple(dy.shape) != (T, Bcap, D) or dx.shape != dy.shape:
        raise SlipstreamError("ss_embbag_ln_backward: dy and dx must be [T, Bcap, D]")
    for p, name in ((gamma, "gamma"), (dgamma, "dgamma"), (dbeta, "dbeta")):
        if p is not None and tuple(p.shape) != (T, D):
            raise SlipstreamError(f"ss_embbag_ln_backward: {name} must be [T, D]")
    _check(_lib.ss_embbag_ln_backward(
        C.byref(tables.c), _dev_ptr(idx, torch.int32, "idx"), C.c_int32(Bcap), C.c_int32(L),
        _dev_ptr(n_valid, torch.int32, "n_valid"), _dev_ptr(dy, torch.float32, "dy"),
        _dev_ptr(gamma, torch.float32, "gamma"), _dev_ptr(mean, torch.float32, "mean"),
        _dev_ptr(rstd, torch.float32, "rstd"), _dev_ptr(dx, torch.float32, "dx"),
        _dev_ptr(dgamma, torch.float32, "dgamma"), _dev_ptr(dbeta, torch.float32, "dbeta"),
        _dev_ptr(ws, torch.uint8, "ws"), C.c_size_t(0 if ws is None else ws.numel()),
        _stream(stream)))


def stream_handle(stream=None) -> C.c_void_p:
    return _stream(stream)


# ---- issue queue (a host thread of the library that enqueues work on streams)
def ss_issue_queue_create() -> C.c_void_p:
    q = C.c_void_p()
    _check(_lib.ss_issue_queue_create(C.byref(q)))
    return q


def ss_issue_queue_destroy(queue: C.c_void_p) -> None:
    _check(_lib.ss_issue_queue_destroy(queue))


def ss_issue_index_batch(queue: C.c_void_p, tables: Tables, idx: torch.Tensor, alpha: int,
                         skip_mask: torch.Tensor, kept_ids: torch.Tensor,
                         n_kept: torch.Tensor, idx_c: torch.Tensor, ws_filter: torch.Tensor,
                         ws_backward: torch.Tensor, stream=None) -> int:
    """ss_filter_batch + ss_embbag_backward_prepare as one queued job; returns its ticket."""
    B, L = _idx_shape(tables, idx)
    if skip_mask.numel() < B or kept_ids.numel() < B or n_kept.numel() < 1 \
            or idx_c.numel() < tables.num_tables * B * L:
        raise SlipstreamError("ss_issue_index_batch: an output tensor is too small")
    t = C.c_uint64()
    _check(_lib.ss_issue_index_batch(
        queue, C.byref(tables.c), _dev_ptr(idx, torch.int32, "idx"), C.c_int32(B), C.c_int32(L),
        C.c_int32(alpha), _dev_ptr(skip_mask, torch.uint8, "skip_mask"),
        _dev_ptr(kept_ids, torch.int32, "kept_ids"), _dev_ptr(n_kept, torch.int32, "n_kept"),
        _dev_ptr(idx_c, torch.int32, "idx_c"), _dev_ptr(ws_filter, torch.uint8, "ws_filter"),
        C.c_size_t(ws_filter.numel()), _dev_ptr(ws_backward, torch.uint8, "ws_backward"),
        C.c_size_t(ws_backward.numel()), _stream(stream), C.byref(t)))
    return t.value


def ss_issue_wait_event(queue: C.c_void_p, event: C.c_void_p, stream=None) -> int:
    t = C.c_uint64()
    _check(_lib.ss_issue_wait_event(queue, event, _stream(stream), C.byref(t)))
    return t.value


def ss_issue_record_event(queue: C.c_void_p, event: C.c_void_p, stream=None) -> int:
    t = C.c_uint64()
    _check(_lib.ss_issue_record_event(queue, event, _stream(stream), C.byref(t)))
    return t.value


def ss_issue_wait(queue: C.c_void_p, ticket: int) -> None:
    _check(_lib.ss_issue_wait(queue, C.c_uint64(ticket)))


def ss_event_create() -> C.c_void_p:
    e = C.c_void_p()
    _check(_lib.ss_event_create(C.byref(e)))
    return e


def ss_event_destroy(event: C.c_void_p) -> None:
    _check(_lib.ss_event_destroy(event))


def ss_event_record(event: C.c_void_p, stream=None) -> None:
    _check(_lib.ss_event_record(event, _stream(stream)))


def ss_stream_wait_event(stream, event: C.c_void_p) -> None:
    _check(_lib.ss_stream_wait_event(_stream(stream), event))


class IssueQueue:
    """The library's issue thread (ss_issue_queue_*) and the plain HIP events that go
    with it.  Tickets are the job numbers ss_issue_wait() takes."""

    def __init__(self):
        q = C.c_void_p()
        _check(_lib.ss_issue_queue_create(C.byref(q)))
        self._q = q
        self._events = []

    def stop(self) -> None:
        """Issues what is still queued and ends the thread; the events stay (jobs of
        another queue may still name them)."""
        if self._q is not None:
            _check(_lib.ss_issue_queue_destroy(self._q))     # issues what is queued, joins
            self._q = None

    def close(self) -> None:
        self.stop()
        for e in self._events:
            _lib.ss_event_destroy(e)
        self._events = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def new_event(self) -> C.c_void_p:
        e = C.c_void_p()
        _check(_lib.ss_event_create(C.byref(e)))
        self._events.append(e)
        return e

    @staticmethod
    def record_now(event: C.c_void_p, handle: C.c_void_p) -> None:
        _check(_lib.ss_event_record(event, handle))

    @staticmethod
    def wait_now(handle: C.c_void_p, event: C.c_void_p) -> None:
        _check(_lib.ss_stream_wait_event(handle, event))

    def wait_event(self, event: C.c_void_p, handle: C.c_void_p) -> int:
        t = C.c_uint64()
        _check(_lib.ss_issue_wait_event(self._q, event, handle, C.byref(t)))
        return t.value

    def record_event(self, event: C.c_void_p, handle: C.c_void_p) -> int:
        t = C.c_uint64()
        _check(_lib.ss_issue_record_event(self._q, event, handle, C.byref(t)))
        return t.value

    def wait_issued(self, ticket: int) -> None:
        _check(_lib.ss_issue_wait(self._q, C.c_uint64(ticket)))


# ---- the training iteration as a whole (ss_step_*) -------------------------
class StepPlan(C.Structure):
    _fields_ = [("every", C.c_int32), ("index_streams", C.c_int32),
                ("issue_threads", C.c_int32), ("num_sets", C.c_int32),
                ("host_wait_us", C.c_int32), ("dim", C.c_int32)]


class StepSet(C.Structure):
    _fields_ = [("skip_mask", C.c_void_p), ("kept_ids", C.c_void_p), ("n_kept", C.c_void_p),
                ("idx_c", C.c_void_p), ("ws_filter", C.c_void_p), ("ws_filter_bytes", C.c_size_t),
                ("ws_backward", C.c_void_p), ("ws_backward_bytes", C.c_size_t)]


_TICKET = C.POINTER(C.c_uint64)


class StepTraceOps(C.Structure):
    """Callbacks of ss_step_create_traced (see include/slipstream.h)."""
    INDEX_NOW = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_int32, C.c_int32)
    Q_INDEX = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _TICKET)
    ON_SET = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_int32)
    EVENT_NOW = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_int32, C.c_int32)
    Q_EVENT = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, _TICKET)
    Q_WAIT_ISSUED = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_int32, C.c_uint64)
    _fields_ = [("user", C.c_void_p), ("index_now", INDEX_NOW), ("q_index", Q_INDEX),
                ("lookup", ON_SET), ("update", ON_SET), ("detect", ON_SET),
                ("record_now", EVENT_NOW), ("wait_now", EVENT_NOW), ("q_record", Q_EVENT),
                ("q_wait", Q_EVENT), ("q_wait_issued", Q_WAIT_ISSUED)]


def ss_step_plan_for(T: int, B: int, L: int, every: int = 0, index_streams: int = 0,
                     issue_threads: int = -1, host_wait_us: int = -1, dim: int = 0) -> StepPlan:
    """The plan for a shape; 0 / 0 / -1 / -1 leave the choice to the library (dim = 0:
    the row length is not known)."""
    plan = StepPlan(int(every), int(index_streams), int(issue_threads), 0, int(host_wait_us),
                    int(dim))
    _check(_lib.ss_step_plan_for(C.c_int32(T), C.c_int32(B), C.c_int32(L), C.byref(plan)))
    return plan


def ss_step_create(tables: Tables, B: int, L: int, alpha: int, lr: float, threshold: float,
                   snapshot_every: int, hot: HotState, plan: StepPlan, sets, pooled: torch.Tensor,
                   stream=None) -> C.c_void_p:
    """sets: plan.num_sets objects with skip_mask, kept_ids, n_kept, idx_c, ws_filter and
    ws_backward tensors.  Returns the handle of the native step."""
    if len(sets) != plan.num_sets:
        raise SlipstreamError("ss_step_create: need plan.num_sets buffer sets")
    if pooled.numel() < tables.num_tables * B * tables.dim:
        raise SlipstreamError("ss_step_create: pooled is too small")
    arr = (StepSet * len(sets))()
    for a, s in zip(arr, sets):
        if s.skip_mask.numel() < B or s.kept_ids.numel() < B or s.n_kept.numel() < 1 \
                or s.idx_c.numel() < tables.num_tables * B * L:
            raise SlipstreamError("ss_step_create: a tensor of a buffer set is too small")
        a.skip_mask = _dev_ptr(s.skip_mask, torch.uint8, "skip_mask").value
        a.kept_ids = _dev_ptr(s.kept_ids, torch.int32, "kept_ids").value
        a.n_kept = _dev_ptr(s.n_kept, torch.int32, "n_kept").value
        a.idx_c = _dev_ptr(s.idx_c, torch.int32, "idx_c").value
        a.ws_filter = _dev_ptr(s.ws_filter, torch.uint8, "ws_filter").value
        a.ws_filter_bytes = s.ws_filter.numel()
        a.ws_backward = _dev_ptr(s.ws_backward, torch.uint8, "ws_backward").value
        a.ws_backward_bytes = s.ws_backward.numel()
    handle = C.c_void_p()
    _check(_lib.ss_step_create(
        C.byref(tables.c), C.c_int32(B), C.c_int32(L), C.c_int32(alpha), C.c_float(lr),
        C.c_float(threshold), C.c_int32(snapshot_every), C.c_void_p(hot._hptr.data_ptr()),
        C.c_int32(hot.H), C.c_void_p(hot._sptr.data_ptr()),
        C.c_void_p(None if hot._shptr is None else hot._shptr.data_ptr()),
        C.c_void_p(None if hot._dptr is None else hot._dptr.data_ptr()),
        _dev_ptr(hot.stale_count, torch.int32, "stale_count"), C.byref(plan), arr,
        _dev_ptr(pooled, torch.float32, "pooled"), _stream(stream), C.byref(handle)))
    return handle


def ss_step_create_traced(plan: StepPlan, snapshot_every: int, ops: StepTraceOps) -> C.c_void_p:
    handle = C.c_void_p()
    _check(_lib.ss_step_create_traced(C.byref(plan), C.c_int32(snapshot_every), C.byref(ops),
                                      C.byref(handle)))
    return handle


def ss_step_destroy(step: C.c_void_p) -> None:
    _check(_lib.ss_step_destroy(step))


def ss_step_room(step: C.c_void_p) -> int:
    return int(_lib.ss_step_room(step))


def ss_step_counters(step: C.c_void_p) -> dict:
    """Lookups enqueued, wait commands given to the training stream for index work,
    polls of the calling thread for index work, polls that found it finished."""
    out = (C.c_int64 * 4)()
    _check(_lib.ss_step_counters(step, out))
    return {"lookups": out[0], "wait_commands": out[1], "host_polls": out[2],
            "host_polls_done": out[3]}


def ss_step_submit(step: C.c_void_p, idx: torch.Tensor, ready_event=None) -> None:
    """idx int32 [T, B, L] contiguous on the device (shape as given at creation, not
    rechecked); ready_event: a torch.cuda.Event recorded after idx's producer, or None."""
    ready = None if ready_event is None else C.c_void_p(ready_event.cuda_event)
    rc = _lib.ss_step_submit(step, C.c_void_p(idx.data_ptr()), ready)
    if rc:
        _check(rc)


def ss_step_forward(step: C.c_void_p) -> int:
    """Returns the ring position of the buffer set that holds this batch's filter outputs."""
    used = C.c_int32(-1)
    rc = _lib.ss_step_forward(step, C.byref(used))
    if rc:
        _check(rc)
    return used.value


def ss_step_backward(step: C.c_void_p, grad: torch.Tensor) -> bool:
    """grad fp32 [T, B, D] contiguous on the device (not rechecked); True after a detect pass."""
    det = C.c_int32(0)
    rc = _lib.ss_step_backward(step, C.c_void_p(grad.data_ptr()), C.byref(det))
    if rc:
        _check(rc)
    return bool(det.value)


def ss_step_flush(step: C.c_void_p) -> None:
    _check(_lib.ss_step_flush(step))
