"""ctypes front end of the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It compiles `ss_oracle.c` with gcc on first use (or when the source
is newer than the library) and exposes its calls on NumPy arrays.
Nothing here touches the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ss_oracle.c")
_LIB = os.path.join(_HERE, "libss_oracle.so")
_lib = None
# A differently built copy of the same source (the sanitizer build of the tests)
# can stand in for the default library: loaded as it is, never rebuilt here.
_LIB_OVERRIDE = os.environ.get("SS_ORACLE_LIB")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the library path."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
             "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"],
            check=True)
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized(out_path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host
    code only); a process that loads it needs the ASan runtime preloaded."""
    subprocess.run(
        ["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", out_path, _SRC, "-lm"],
        check=True)
    return out_path


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_LIB_OVERRIDE if _LIB_OVERRIDE else build())
        for name in ("oracle_embbag_forward", "oracle_embbag_backward_update",
                     "oracle_detect_stale", "oracle_filter_batch",
                     "oracle_sample_drop", "oracle_drop_stats",
                     "oracle_count_accesses", "oracle_select_hot_ratio",
                     "oracle_select_hot_top", "oracle_layernorm_forward",
                     "oracle_layernorm_backward"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _ptr_array(arrays: Optional[Sequence[Optional[np.ndarray]]], n: int):
    """void*[n] holding the data pointers of `arrays` (None -> NULL)."""
    arr = (C.c_void_p * n)()
    if arrays is not None:
        assert len(arrays) == n
        for i, a in enumerate(arrays):
            arr[i] = None if a is None else a.ctypes.data
    return arr


def _check(a: np.ndarray, dtype, name: str):
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need C-contiguous {np.dtype(dtype)}")


def _check_rc(rc: int, what: str):
    if rc == -1:
        raise IndexError(f"{what}: index out of range")
    if rc != 0:
        raise RuntimeError(f"{what}: oracle returned {rc}")


def embbag_forward(weights: Sequence[np.ndarray], idx: np.ndarray,
                   n_valid: Optional[int] = None) -> np.ndarray:
    """weights: T arrays [R, D] fp32; idx int32 [T, Bcap, L] -> [T, Bcap, D].

    Rows j >= n_valid of the result are zero.
    """
    T = len(weights)
    R, D = weights[0].shape
    _check(idx, np.int32, "idx")
    assert idx.shape[0] == T and idx.ndim == 3
    Bcap, L = idx.shape[1], idx.shape[2]
    if n_valid is None:
        n_valid = Bcap
    for w in weights:
        _check(w, np.float32, "weights")
        assert w.shape == (R, D)
    out = np.zeros((T, Bcap, D), dtype=np.float32)
    rc = _load().oracle_embbag_forward(
        C.c_int(T), C.c_int64(R), C.c_int(D), _ptr_array(weights, T),
        C.c_void_p(idx.ctypes.data), C.c_int(Bcap), C.c_int(L),
        C.c_int(n_valid), C.c_void_p(out.ctypes.data))
    _check_rc(rc, "embbag_forward")
    return out


def embbag_backward_update(weights: Sequence[np.ndarray],
                           stale_bits: Optional[Sequence[Optional[np.ndarray]]],
                           idx: np.ndarray, grad: np.ndarray, lr: float,
                           n_valid: Optional[int] = None) -> None:
    """Updates `weights` in place; stale_bits: T uint32 arrays or None."""
    T = len(weights)
    R, D = weights[0].shape
    _check(idx, np.int32, "idx")
    _check(grad, np.float32, "grad")
    Bcap, L = idx.shape[1], idx.shape[2]
    assert idx.shape[0] == T and grad.shape == (T, Bcap, D)
    if n_valid is None:
        n_valid = Bcap
    for w in weights:
        _check(w, np.float32, "weights")
        assert w.shape == (R, D)
    if stale_bits is not None:
        for b in stale_bits:
            if b is not None:
                _check(b, np.uint32, "stale_bits")
                assert b.size >= (R + 31) // 32
    bits = _ptr_array(stale_bits, T) if stale_bits is not None else None
    rc = _load().oracle_embbag_backward_update(
        C.c_int(T), C.c_int64(R), C.c_int(D), _ptr_array(weights, T), bits,
        C.c_void_p(idx.ctypes.data), C.c_int(Bcap), C.c_int(L),
        C.c_int(n_valid), C.c_void_p(grad.ctypes.data), C.c_float(lr))
    _check_rc(rc, "embbag_backward_update")


def detect_stale(weights: Sequence[np.ndarray],
                 stale_bits: Sequence[np.ndarray],
                 hot_ids: Sequence[np.ndarray], snapshot: Sequence[np.ndarray],
                 threshold: float, refresh: bool = True):
    """ORs new stale bits into `stale_bits`, refreshes `snapshot` in place.

    Returns (stale_hot uint8 [T, H], drift fp64 [T, H], stale_count uint32 [T]).
    """
    T = len(weights)
    R, D = weights[0].shape
    H = hot_ids[0].shape[0]
    for t in range(T):
        _check(weights[t], np.float32, "weights")
        _check(stale_bits[t], np.uint32, "stale_bits")
        _check(hot_ids[t], np.int32, "hot_ids")
        _check(snapshot[t], np.float32, "snapshot")
        assert snapshot[t].shape == (H, D) and hot_ids[t].shape == (H,)
        assert stale_bits[t].size >= (R + 31) // 32
    stale_hot = np.zeros((T, H), dtype=np.uint8)
    drift = np.zeros((T, H), dtype=np.float64)
    count = np.zeros(T, dtype=np.uint32)
    rc = _load().oracle_detect_stale(
        C.c_int(T), C.c_int64(R), C.c_int(D), _ptr_array(weights, T),
        _ptr_array(stale_bits, T), _ptr_array(hot_ids, T), C.c_int(H),
        _ptr_array(snapshot, T), C.c_float(threshold), C.c_int(int(refresh)),
        _ptr_array([stale_hot[t] for t in range(T)], T),
        _ptr_array([drift[t] for t in range(T)], T),
        C.c_void_p(count.ctypes.data))
    _check_rc(rc, "detect_stale")
    return stale_hot, drift, count


def filter_batch(rows: int, stale_bits: Optional[Sequence[Optional[np.ndarray]]],
                 idx: np.ndarray, alpha: int):
    """Returns (skip_mask uint8 [B], kept_ids int32 [n_kept], idx_c [T, B, L]).

    idx_c rows j >= n_kept are zero.
    """
    _check(idx, np.int32, "idx")
    T, B, L = idx.shape
    skip = np.zeros(B, dtype=np.uint8)
    kept = np.zeros(B, dtype=np.int32)
    n_kept = C.c_int32(0)
    idx_c = np.zeros_like(idx)
    bits = _ptr_array(stale_bits, T) if stale_bits is not None else None
    rc = _load().oracle_filter_batch(
        C.c_int(T), C.c_int64(rows), bits, C.c_void_p(idx.ctypes.data),
        C.c_int(B), C.c_int(L), C.c_int(alpha), C.c_void_p(skip.ctypes.data),
        C.c_void_p(kept.ctypes.data), C.byref(n_kept),
        C.c_void_p(idx_c.ctypes.data))
    _check_rc(rc, "filter_batch")
    return skip, kept[:n_kept.value].copy(), idx_c


def sample_drop(weights: Sequence[np.ndarray], hot_ids: Sequence[np.ndarray],
                snapshot: Sequence[np.ndarray], sidx: np.ndarray, alpha: int,
                thresholds: Sequence[float]) -> np.ndarray:
    """sidx int32 [T, S, L] -> uint32 [len(thresholds)]: droppable sampled inputs."""
    T = len(weights)
    R, D = weights[0].shape
    H = hot_ids[0].shape[0]
    _check(sidx, np.int32, "sidx")
    assert sidx.ndim == 3 and sidx.shape[0] == T
    S, L = sidx.shape[1], sidx.shape[2]
    for t in range(T):
        _check(weights[t], np.float32, "weights")
        _check(hot_ids[t], np.int32, "hot_ids")
        _check(snapshot[t], np.float32, "snapshot")
        assert snapshot[t].shape == (H, D) and hot_ids[t].shape == (H,)
        assert np.all(np.diff(hot_ids[t]) > 0), "hot_ids must be ascending"
    thr = np.ascontiguousarray(thresholds, dtype=np.float32)
    counts = np.zeros(thr.size, dtype=np.uint32)
    rc = _load().oracle_sample_drop(
        C.c_int(T), C.c_int64(R), C.c_int(D), _ptr_array(weights, T),
        _ptr_array(hot_ids, T), C.c_int(H), _ptr_array(snapshot, T),
        C.c_void_p(sidx.ctypes.data), C.c_int(S), C.c_int(L), C.c_int(alpha),
        C.c_void_p(thr.ctypes.data), C.c_int(thr.size),
        C.c_void_p(counts.ctypes.data))
    _check_rc(rc, "sample_drop")
    return counts


def drop_stats(count: int, n_samples: int, population: int, n_hot_inputs: int,
               t_crit: float) -> dict:
    """Eq. 2-4: share D, sd, interval half-width, and the same on the count scale."""
    out = (C.c_double * 8)()
    rc = _load().oracle_drop_stats(C.c_uint32(count), C.c_int64(n_samples),
                                   C.c_int64(population), C.c_int64(n_hot_inputs),
                                   C.c_double(t_crit), out)
    if rc != 0:
        raise ValueError("drop_stats: inconsistent arguments")
    keys = ("D", "sd", "half", "lo", "hi", "D_bar", "D_bar_lo", "D_bar_hi")
    return dict(zip(keys, list(out)))


def count_accesses(rows: int, idx: np.ndarray, counts: Sequence[np.ndarray],
                   n_valid: Optional[int] = None) -> None:
    """counts: T uint32 arrays [rows], advanced in place."""
    _check(idx, np.int32, "idx")
    T, B, L = idx.shape
    for c in counts:
        _check(c, np.uint32, "counts")
        assert c.shape == (rows,)
    rc = _load().oracle_count_accesses(
        C.c_int(T), C.c_int64(rows), C.c_void_p(idx.ctypes.data), C.c_int(B),
        C.c_int(L), C.c_int(B if n_valid is None else n_valid), _ptr_array(counts, T))
    _check_rc(rc, "count_accesses")


def _hot_outputs(T: int, rows: int, cap: int):
    ids = [np.full(cap, -1, dtype=np.int32) for _ in range(T)]
    bits = [np.zeros((rows + 31) // 32, dtype=np.uint32) for _ in range(T)]
    return ids, bits


def select_hot_ratio(counts: Sequence[np.ndarray], lam: float, total: int, cap: int):
    """Returns (hot_ids: T int32 arrays [cap], -1 past n_hot; bitmaps; n_hot uint32 [T])."""
    T, rows = len(counts), counts[0].shape[0]
    ids, bits = _hot_outputs(T, rows, cap)
    n_hot = np.zeros(T, dtype=np.uint32)
    rc = _load().oracle_select_hot_ratio(
        C.c_int(T), C.c_int64(rows), _ptr_array(counts, T), C.c_double(lam),
        C.c_int64(total), C.c_int(cap), _ptr_array(ids, T), _ptr_array(bits, T),
        C.c_void_p(n_hot.ctypes.data))
    if rc == -3:
        raise ValueError("select_hot_ratio: need total >= 1")
    _check_rc(rc, "select_hot_ratio")
    return ids, bits, n_hot


def select_hot_top(counts: Sequence[np.ndarray], H: int):
    """Returns (hot_ids: T int32 arrays [H] ascending; bitmaps)."""
    T, rows = len(counts), counts[0].shape[0]
    ids, bits = _hot_outputs(T, rows, H)
    rc = _load().oracle_select_hot_top(
        C.c_int(T), C.c_int64(rows), _ptr_array(counts, T), C.c_int(H),
        _ptr_array(ids, T), _ptr_array(bits, T))
    if rc == -3:
        raise ValueError("select_hot_top: need 0 <= H <= rows")
    _check_rc(rc, "select_hot_top")
    return ids, bits


def _opt(a: Optional[np.ndarray], name: str):
    if a is None:
        return None
    _check(a, np.float32, name)
    return C.c_void_p(a.ctypes.data)


def layernorm_forward(x: np.ndarray, gamma: Optional[np.ndarray], beta: Optional[np.ndarray],
                      eps: float, n_valid: Optional[int] = None):
    """x fp32 [T, Bcap, D]; gamma, beta fp32 [T, D] or None.
    Returns (y [T, Bcap, D], mean [T, Bcap], rstd [T, Bcap]); rows j >= n_valid are zero."""
    _check(x, np.float32, "x")
    T, Bcap, D = x.shape
    y = np.zeros_like(x)
    mean = np.zeros((T, Bcap), np.float32)
    rstd = np.zeros((T, Bcap), np.float32)
    rc = _load().oracle_layernorm_forward(
        C.c_int(T), C.c_int(D), C.c_void_p(x.ctypes.data), C.c_int(Bcap),
        C.c_int(Bcap if n_valid is None else n_valid), _opt(gamma, "gamma"),
        _opt(beta, "beta"), C.c_double(eps), C.c_void_p(y.ctypes.data),
        C.c_void_p(mean.ctypes.data), C.c_void_p(rstd.ctypes.data))
    _check_rc(rc, "layernorm_forward")
    return y, mean, rstd


def layernorm_backward(dy: np.ndarray, x: np.ndarray, gamma: Optional[np.ndarray],
                       eps: float, n_valid: Optional[int] = None):
    """Returns (dx [T, Bcap, D], dgamma [T, D], dbeta [T, D])."""
    _check(x, np.float32, "x")
    _check(dy, np.float32, "dy")
    assert dy.shape == x.shape
    T, Bcap, D = x.shape
    dx = np.zeros_like(x)
    dgamma = np.zeros((T, D), np.float32)
    dbeta = np.zeros((T, D), np.float32)
    rc = _load().oracle_layernorm_backward(
        C.c_int(T), C.c_int(D), C.c_void_p(dy.ctypes.data), C.c_void_p(x.ctypes.data),
        C.c_int(Bcap), C.c_int(Bcap if n_valid is None else n_valid), _opt(gamma, "gamma"),
        C.c_double(eps), C.c_void_p(dx.ctypes.data), C.c_void_p(dgamma.ctypes.data),
        C.c_void_p(dbeta.ctypes.data))
    _check_rc(rc, "layernorm_backward")
    return dx, dgamma, dbeta
