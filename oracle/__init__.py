"""CPU oracle for the Elastic Cache hot path -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes wrappers over ``ec_oracle.c`` (plain fp64 C written from the
paper: Sec. 3.3, Eq. 1-3, Alg. 1, Sec. 4.1 Implementation Details).  Nothing in
the product path may import this package; it is for tests, the smoke check and
the benchmark's cpu_baseline leg.  It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ec_oracle.c")
_LIB = os.path.join(_HERE, "libec_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ec_oracle.c with gcc (fp64, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_dp = ctypes.POINTER(ctypes.c_double)
_fp = ctypes.POINTER(ctypes.c_float)
_ip = ctypes.POINTER(ctypes.c_int32)


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_evict_index.argtypes = [ctypes.c_int64] + [ctypes.c_int] * 9
        _lib.oracle_evict_index.restype = ctypes.c_int
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _d(a):
    return None if a is None else a.ctypes.data_as(_dp)


def _i(a):
    return None if a is None else a.ctypes.data_as(_ip)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def prefill_score(q, k, v, scale: float, G: int, want_out=True, want_attn=False):
    """Eq. 1 + importance.  q,k,v [B,H,T,D] -> dict(out, lse, score[, attn]) in fp64."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, H, T, D = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    out = np.empty((B, H, T, D), np.float64) if want_out else None
    lse = np.empty((B, H, T), np.float64)
    score = np.empty((B, G, T), np.float64)
    attn = np.empty((B, H, T, T), np.float64) if want_attn else None
    rc = _load().oracle_prefill_score(_d(q), _d(k), _d(v), B, H, T, D, ctypes.c_double(scale), G,
                                      _d(out), _d(lse), _d(score), _d(attn))
    if rc:
        raise ValueError(f"oracle_prefill_score rc={rc}")
    return {"out": out, "lse": lse, "score": score, "attn": attn}


def chunk_score(q, k, v, P: int, scale: float, G: int, want_out=True):
    """Multi-token pass over [P cached rows | chunk].  q [B,H,Tq,D]; k,v [B,H,P+Tq,D] -> dict(out, lse, score [B,G,P+Tq])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, H, Tq, D = q.shape
    L = P + Tq
    assert k.shape == (B, H, L, D) and v.shape == k.shape
    out = np.empty((B, H, Tq, D), np.float64) if want_out else None
    lse = np.empty((B, H, Tq), np.float64)
    score = np.empty((B, G, L), np.float64)
    rc = _load().oracle_chunk_score(_d(q), _d(k), _d(v), B, H, Tq, P, D, ctypes.c_double(scale), G,
                                    _d(out), _d(lse), _d(score))
    if rc:
        raise ValueError(f"oracle_chunk_score rc={rc}")
    return {"out": out, "lse": lse, "score": score}


def select_anchors(score_f32, n_anchor: int, protect_first: int = 1, protect_last: int = 1):
    """Top-n_anchor positions of each [T] fp32 score row, ascending.  score [B,G,T]."""
    s = np.ascontiguousarray(score_f32, dtype=np.float32)
    B, G, T = s.shape
    idx = np.empty((B, G, n_anchor), np.int32)
    rc = _load().oracle_select_anchors(s.ctypes.data_as(_fp), B, G, T, n_anchor, protect_first,
                                       protect_last, _i(idx))
    if rc:
        raise ValueError(f"oracle_select_anchors rc={rc}")
    return idx


def assign_nearest(anchor_idx, T: int):
    """Exhaustive nearest-anchor assignment -> (assign [B,G,T], counts [B,G,n])."""
    a = np.ascontiguousarray(anchor_idx, dtype=np.int32)
    B, G, n = a.shape
    assign = np.empty((B, G, T), np.int32)
    counts = np.empty((B, G, n), np.int32)
    rc = _load().oracle_assign_nearest(_i(a), B, G, T, n, _i(assign), _i(counts))
    if rc:
        raise ValueError(f"oracle_assign_nearest rc={rc}")
    return assign, counts


def bucket_bounds(anchor_idx, T: int):
    """Eq. 2 inclusive bucket bounds -> (lo, hi), each [B,G,n]."""
    a = np.ascontiguousarray(anchor_idx, dtype=np.int32)
    B, G, n = a.shape
    lo = np.empty((B, G, n), np.int32)
    hi = np.empty((B, G, n), np.int32)
    rc = _load().oracle_bucket_bounds(_i(a), B, G, T, n, _i(lo), _i(hi))
    if rc:
        raise ValueError(f"oracle_bucket_bounds rc={rc}")
    return lo, hi


def merge_compact(x, assign, n_anchor: int, cap: int | None = None):
    """Eq. 3 per-bucket mean.  x [B,H,T,D], assign [B,G,T] -> cache [B,H,cap,D] (rows >= n_anchor zero)."""
    x = _f64(x)
    B, H, T, D = x.shape
    a = np.ascontiguousarray(assign, dtype=np.int32)
    G = a.shape[1]
    cap = n_anchor if cap is None else cap
    cache = np.zeros((B, H, cap, D), np.float64)
    rc = _load().oracle_merge_compact(_d(x), _i(a), B, H, G, T, D, n_anchor, cap, _d(cache))
    if rc:
        raise ValueError(f"oracle_merge_compact rc={rc}")
    return cache


def merge_weighted(x, assign, weights, n_anchor: int, cap: int | None = None):
    """Count-weighted per-bucket mean.  x [B,H,T,D], assign/weights [B,G,T] -> (cache [B,H,cap,D], wsum [B,G,n])."""
    x = _f64(x)
    B, H, T, D = x.shape
    a = np.ascontiguousarray(assign, dtype=np.int32)
    w = np.ascontiguousarray(weights, dtype=np.int32)
    assert a.shape == w.shape
    G = a.shape[1]
    cap = n_anchor if cap is None else cap
    cache = np.zeros((B, H, cap, D), np.float64)
    wsum = np.zeros((B, G, n_anchor), np.int32)
    rc = _load().oracle_merge_weighted(_d(x), _i(a), _i(w), B, H, G, T, D, n_anchor, cap, _d(cache), _i(wsum))
    if rc:
        raise ValueError(f"oracle_merge_weighted rc={rc}")
    return cache, wsum


def evict_compact(x, anchor_idx, cap: int | None = None):
    """Eviction-only ablation (Table 3b): the anchors' own rows.  x [B,H,T,D], anchor_idx [B,G,n]."""
    x = _f64(x)
    B, H, T, D = x.shape
    a = np.ascontiguousarray(anchor_idx, dtype=np.int32)
    G, n = a.shape[1], a.shape[2]
    cap = n if cap is None else cap
    cache = np.zeros((B, H, cap, D), np.float64)
    rc = _load().oracle_evict_compact(_d(x), _i(a), B, H, G, T, D, n, cap, _d(cache))
    if rc:
        raise ValueError(f"oracle_evict_compact rc={rc}")
    return cache


def evict_index(n_seen: int, len_after_append: int, gamma_num: int, gamma_den: int,
                budget_mode: int = 0, fixed_len: int = 0, trunc_mode: int = 0, recent: int = 25,
                n_tl: int = 0, protect_first: int = 1) -> int:
    return int(_load().oracle_evict_index(n_seen, len_after_append, gamma_num, gamma_den,
                                          budget_mode, fixed_len, trunc_mode, recent, n_tl,
                                          protect_first))


def decode_step(q, k_new, v_new, k_cache, v_cache, pos, cache_len: int, evict_idx: int,
                new_pos: int, scale: float, want_probs=False):
    """One generation step, in place on fp64 k_cache/v_cache [B,H,cap,D] and int32 pos [B,G,cap].

    Returns (out [B,H,D], probs [B,H,cache_len+1] or None).
    """
    q, k_new, v_new = _f64(q), _f64(k_new), _f64(v_new)
    for c in (k_cache, v_cache):
        assert c.dtype == np.float64 and c.flags.c_contiguous
    B, H, cap, D = k_cache.shape
    G = 1
    if pos is not None:
        assert pos.dtype == np.int32 and pos.flags.c_contiguous
        G = pos.shape[1]
    out = np.empty((B, H, D), np.float64)
    probs = np.empty((B, H, cache_len + 1), np.float64) if want_probs else None
    rc = _load().oracle_decode_step(_d(q), _d(k_new), _d(v_new), _d(k_cache), _d(v_cache), _i(pos),
                                    B, H, G, D, cap, cache_len, evict_idx, new_pos,
                                    ctypes.c_double(scale), _d(out), _d(probs))
    if rc:
        raise ValueError(f"oracle_decode_step rc={rc}")
    return out, probs


def decode_score_step(q, k_new, v_new, k_cache, v_cache, pos, freq, cache_len: int, new_pos: int, scale: float):
    """Frequency policy: one generation step without removal that also adds its attention row to freq.

    k_cache/v_cache fp64 [B,H,cap,D], pos int32 [B,G,cap] or None, freq fp64 [B,G,cap], all in place.
    Returns (out [B,H,D], probs [B,H,cache_len+1]).
    """
    assert freq.dtype == np.float64 and freq.flags.c_contiguous
    B, H, cap, D = k_cache.shape
    G = freq.shape[1]
    out, probs = decode_step(q, k_new, v_new, k_cache, v_cache, pos, cache_len, -1, new_pos, scale, want_probs=True)
    rc = _load().oracle_freq_accumulate(_d(probs), B, H, G, cache_len + 1, cap, _d(freq))
    if rc:
        raise ValueError(f"oracle_freq_accumulate rc={rc}")
    return out, probs


def evict_min(freq_f32, k_cache, v_cache, pos, length: int, protect_first: int = 1, protect_recent: int = 1):
    """Frequency policy: remove the row of least fp32 mass (lowest index among equals), in place.

    freq_f32 float32 [B,G,cap]; k_cache/v_cache fp64 [B,H,cap,D]; pos int32 [B,G,cap] or None.  Returns victim [B,G].
    """
    assert freq_f32.dtype == np.float32 and freq_f32.flags.c_contiguous
    for c in (k_cache, v_cache):
        assert c.dtype == np.float64 and c.flags.c_contiguous
    B, H, cap, D = k_cache.shape
    G = freq_f32.shape[1]
    victim = np.empty((B, G), np.int32)
    rc = _load().oracle_evict_min(freq_f32.ctypes.data_as(_fp), _d(k_cache), _d(v_cache), _i(pos), B, H, G, D, cap,
                                  length, protect_first, protect_recent, _i(victim))
    if rc:
        raise ValueError(f"oracle_evict_min rc={rc}")
    return victim


def importance_mean(score, Tq: int, P: int = 0):
    """Table 3d's "Mean" metric from the column sums: score [B,G,P+Tq] fp64 -> new array, sum / number of seeing queries."""
    s = np.array(score, dtype=np.float64, order="C", copy=True)
    B, G, L = s.shape
    assert L == P + Tq
    rc = _load().oracle_importance_mean(_d(s), B, G, Tq, P)
    if rc:
        raise ValueError(f"oracle_importance_mean rc={rc}")
    return s
