"""ctypes binding over libelastic_cache.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA tensors (device memory + the current stream come from
PyTorch); every computation happens in the library's HIP kernels.  There is no
CPU fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("EC_LIB_PATH", os.path.join(_HERE, "libelastic_cache.so"))

EC_OK, EC_EINVAL, EC_EUNSUPPORTED, EC_EWORKSPACE, EC_EDEVICE = range(5)
EC_F32, EC_BF16 = 0, 1
(EC_FN_PREFILL_SCORE, EC_FN_SELECT_ANCHORS, EC_FN_MERGE_COMPACT, EC_FN_DECODE_STEP, EC_FN_DECODE_SCORE_STEP,
 EC_FN_EVICT_MIN) = range(6)
EC_BUDGET_RATIO, EC_BUDGET_FIXED = 0, 1
EC_TRUNC_RECENT, EC_TRUNC_ABS = 0, 1
EC_MERGE_MEAN, EC_MERGE_EVICT = 0, 1

SYMBOLS = ("ec_status_string", "ec_workspace_bytes", "ec_prefill_score", "ec_chunk_score", "ec_select_anchors",
           "ec_merge_compact", "ec_remerge_compact", "ec_evict_index", "ec_decode_step", "ec_decode_score_step",
           "ec_evict_min", "ec_prefill_score_varlen", "ec_select_anchors_varlen", "ec_merge_compact_varlen",
           "ec_decode_step_varlen", "ec_importance_mean", "ec_retention_step_varlen", "ec_decode_step_shaped",
           "ec_decode_score_step_static")

_lib = None


class EcError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__(f"{fn}: {status_string(status)}")


def load():
    """Load the in-tree library (build it first with `python -m paper_2407_18121_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_vp, c_sz, c_f = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
    lib.ec_status_string.argtypes = [c_int]
    lib.ec_status_string.restype = ctypes.c_char_p
    lib.ec_workspace_bytes.argtypes = [c_int] * 6
    lib.ec_workspace_bytes.restype = c_sz
    lib.ec_prefill_score.argtypes = [c_vp] * 6 + [c_int] * 6 + [c_f, c_vp, c_sz, c_vp]
    lib.ec_prefill_score.restype = c_int
    lib.ec_chunk_score.argtypes = [c_vp] * 6 + [c_int] * 8 + [c_f, c_vp, c_sz, c_vp]
    lib.ec_chunk_score.restype = c_int
    lib.ec_select_anchors.argtypes = [c_vp] + [c_int] * 6 + [c_vp, c_vp, c_sz, c_vp]
    lib.ec_select_anchors.restype = c_int
    lib.ec_merge_compact.argtypes = [c_vp] * 3 + [c_int] * 8 + [c_vp, c_vp, c_int, c_vp, c_vp, c_vp, c_vp]
    lib.ec_merge_compact.restype = c_int
    lib.ec_remerge_compact.argtypes = ([c_vp, c_vp, c_int, c_vp, c_vp, c_vp] + [c_int] * 8
                                       + [c_vp, c_vp, c_int, c_vp, c_vp, c_vp, c_vp])
    lib.ec_remerge_compact.restype = c_int
    lib.ec_evict_index.argtypes = [ctypes.c_int64] + [c_int] * 9
    lib.ec_evict_index.restype = c_int
    lib.ec_decode_step.argtypes = ([c_vp] * 6 + [c_int] * 7 + [ctypes.c_int32, c_f, c_int, c_vp, c_vp, c_sz, c_vp])
    lib.ec_decode_step.restype = c_int
    lib.ec_decode_step_shaped.argtypes = ([c_vp] * 6 + [c_int] * 7 + [ctypes.c_int32, c_f, c_int, c_vp, c_vp, c_sz]
                                          + [c_int] * 3 + [c_vp])
    lib.ec_decode_step_shaped.restype = c_int
    lib.ec_decode_score_step.argtypes = ([c_vp] * 7 + [c_int] * 6 + [ctypes.c_int32, c_f, c_int, c_vp, c_vp, c_sz, c_vp])
    lib.ec_decode_score_step.restype = c_int
    lib.ec_decode_score_step_static.argtypes = ([c_vp] * 7 + [c_int] * 6 + [ctypes.c_int32, c_f, c_int, c_vp, c_vp])
    lib.ec_decode_score_step_static.restype = c_int
    lib.ec_evict_min.argtypes = [c_vp] * 4 + [c_int] * 9 + [c_vp, c_vp]
    lib.ec_evict_min.restype = c_int
    lib.ec_prefill_score_varlen.argtypes = [c_vp] * 7 + [c_int] * 6 + [c_f, c_vp, c_sz, c_vp]
    lib.ec_prefill_score_varlen.restype = c_int
    lib.ec_select_anchors_varlen.argtypes = [c_vp] * 3 + [c_int] * 6 + [c_vp, c_vp, c_sz, c_vp]
    lib.ec_select_anchors_varlen.restype = c_int
    lib.ec_merge_compact_varlen.argtypes = [c_vp] * 5 + [c_int] * 8 + [c_vp, c_vp, c_int, c_vp, c_vp, c_vp, c_vp]
    lib.ec_merge_compact_varlen.restype = c_int
    lib.ec_decode_step_varlen.argtypes = [c_vp] * 9 + [c_int] * 5 + [c_f, c_int, c_vp, c_vp, c_sz, c_vp]
    lib.ec_decode_step_varlen.restype = c_int
    lib.ec_importance_mean.argtypes = [c_vp] + [c_int] * 4 + [c_vp]
    lib.ec_importance_mean.restype = c_int
    lib.ec_retention_step_varlen.argtypes = [c_vp] * 5 + [c_int] * 10 + [c_vp]
    lib.ec_retention_step_varlen.restype = c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().ec_status_string(int(status)).decode()


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return EC_F32
    if t.dtype == torch.bfloat16:
        return EC_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _chk(t, name, dtype, shape, optional=False):
    """Pointer of a tensor after checking what the C ABI cannot: element type, shape, device, layout.
    A wrong type or shape would make a kernel read or write out of bounds."""
    if t is None:
        if optional:
            return None
        raise ValueError(f"{name} is required")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return _Checked(t, name)


class _Checked:
    """A tensor whose type and shape fit; its device and layout are checked when the pointer is taken, after
    every argument of the call has passed the type and shape checks."""
    __slots__ = ("t", "name")

    def __init__(self, t, name):
        self.t, self.name = t, name


def _call(fn, *args):
    """Call a library function; _Checked arguments become device pointers here, and the stream (passed as the
    function that looks it up) is resolved last, once every tensor has been found in device memory."""
    ptrs = [_ptr(a.t, a.name) if isinstance(a, _Checked) else a for a in args]
    return fn(*[a() if callable(a) else a for a in ptrs])


def _ws(ws):
    """(pointer, bytes) of an optional workspace tensor."""
    if ws is None:
        return None, 0
    return _Checked(ws, "ws"), ws.numel() * ws.element_size()


def _groups(G, H, what):
    if G != 1 and G != H:
        raise ValueError(f"{what}: the number of score groups must be 1 or H={H}, got {G}")
    return G


def _stream():
    return torch.cuda.current_stream().cuda_stream


def ec_workspace_bytes(fn: int, B: int, H: int, T: int, D: int, dt: int) -> int:
    n = load().ec_workspace_bytes(fn, B, H, T, D, dt)
    if n == ctypes.c_size_t(-1).value:
        raise EcError("ec_workspace_bytes", EC_EUNSUPPORTED)
    return int(n)


def new_workspace(fn: int, B: int, H: int, T: int, D: int, dt: int, device="cuda") -> torch.Tensor:
    """Zero-filled workspace of the size the entry point asks for."""
    return torch.zeros(max(ec_workspace_bytes(fn, B, H, T, D, dt), 256), dtype=torch.uint8, device=device)


def ec_prefill_score(q, k, v, out, lse, score, scale: float, ws, check=True) -> int:
    """q,k,v [B,H,T,D]; out [B,H,T,D] or None; lse [B,H,T] f32 or None; score [B,G,T] f32."""
    if q.dim() != 4 or score.dim() != 3:
        raise ValueError("ec_prefill_score: q must be [B,H,T,D] and score [B,G,T]")
    B, H, T, D = q.shape
    G = _groups(score.shape[1], H, "ec_prefill_score")
    dt, f32 = q.dtype, torch.float32
    wp, wb = _ws(ws)
    rc = _call(load().ec_prefill_score, _chk(q, "q", dt, (B, H, T, D)), _chk(k, "k", dt, (B, H, T, D)),
                                 _chk(v, "v", dt, (B, H, T, D)), _chk(out, "out", dt, (B, H, T, D), True),
                                 _chk(lse, "lse", f32, (B, H, T), True), _chk(score, "score", f32, (B, G, T)),
                                 B, H, G, T, D, dtype_code(q), scale, wp, wb, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_prefill_score", rc)
    return rc


def ec_chunk_score(q, k, v, P: int, out, lse, score, scale: float, ws, check=True) -> int:
    """q [B,H,T_new,D]; k,v [B,H,kv_rows,D] holding P cached rows then the chunk's rows; score [B,G,P+T_new]."""
    if q.dim() != 4 or k.dim() != 4 or score.dim() != 3:
        raise ValueError("ec_chunk_score: q, k must be 4-D and score 3-D")
    B, H, T_new, D = q.shape
    kv_rows = k.shape[2]
    G = _groups(score.shape[1], H, "ec_chunk_score")
    dt, f32 = q.dtype, torch.float32
    wp, wb = _ws(ws)
    rc = _call(load().ec_chunk_score, _chk(q, "q", dt, (B, H, T_new, D)), _chk(k, "k", dt, (B, H, kv_rows, D)),
                               _chk(v, "v", dt, (B, H, kv_rows, D)), _chk(out, "out", dt, (B, H, T_new, D), True),
                               _chk(lse, "lse", f32, (B, H, T_new), True),
                               _chk(score, "score", f32, (B, G, P + T_new)), B, H, G, T_new, P, kv_rows, D,
                               dtype_code(q), scale, wp, wb, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_chunk_score", rc)
    return rc


def ec_select_anchors(score, n_anchor: int, protect_first: int, protect_last: int, anchor_idx, check=True) -> int:
    """score [B,G,T] f32 -> anchor_idx [B,G,n_anchor] int32 ascending."""
    if score.dim() != 3:
        raise ValueError("ec_select_anchors: score must be [B,G,T]")
    B, G, T = score.shape
    rc = _call(load().ec_select_anchors, _chk(score, "score", torch.float32, (B, G, T)), B, G, T, n_anchor, protect_first,
                                  protect_last, _chk(anchor_idx, "anchor_idx", torch.int32, (B, G, n_anchor)), None, 0,
                                  _stream)
    if check and rc != EC_OK:
        raise EcError("ec_select_anchors", rc)
    return rc


def ec_merge_compact(k, v, anchor_idx, k_cache, v_cache, counts=None, assign=None, pos=None,
                     merge_mode: int = EC_MERGE_MEAN, check=True) -> int:
    """k,v [B,H,T,D]; anchor_idx [B,G,n]; k_cache,v_cache [B,H,cap,D]."""
    if k.dim() != 4 or anchor_idx.dim() != 3 or k_cache.dim() != 4:
        raise ValueError("ec_merge_compact: k, k_cache must be 4-D and anchor_idx 3-D")
    B, H, T, D = k.shape
    G, n_anchor = _groups(anchor_idx.shape[1], H, "ec_merge_compact"), anchor_idx.shape[2]
    cap = k_cache.shape[2]
    dt, i32 = k.dtype, torch.int32
    rc = _call(load().ec_merge_compact, _chk(k, "k", dt, (B, H, T, D)), _chk(v, "v", dt, (B, H, T, D)),
                                 _chk(anchor_idx, "anchor_idx", i32, (B, G, n_anchor)), B, H, G, T, D, n_anchor,
                                 dtype_code(k), merge_mode, _chk(k_cache, "k_cache", dt, (B, H, cap, D)),
                                 _chk(v_cache, "v_cache", dt, (B, H, cap, D)), cap,
                                 _chk(counts, "counts", i32, (B, G, n_anchor), True),
                                 _chk(assign, "assign", i32, (B, G, T), True), _chk(pos, "pos", i32, (B, G, cap), True),
                                 _stream)
    if check and rc != EC_OK:
        raise EcError("ec_merge_compact", rc)
    return rc


def ec_remerge_compact(k, v, L: int, anchor_idx, k_cache, v_cache, weights=None, src_pos=None, counts=None,
                       assign=None, pos=None, merge_mode: int = EC_MERGE_MEAN, check=True) -> int:
    """k,v [B,H,src_rows,D] of which rows 0..L-1 are merged; weights, src_pos [B,G,L] int32 or None."""
    if k.dim() != 4 or anchor_idx.dim() != 3 or k_cache.dim() != 4:
        raise ValueError("ec_remerge_compact: k, k_cache must be 4-D and anchor_idx 3-D")
    B, H, src_rows, D = k.shape
    G, n_anchor = _groups(anchor_idx.shape[1], H, "ec_remerge_compact"), anchor_idx.shape[2]
    cap = k_cache.shape[2]
    dt, i32 = k.dtype, torch.int32
    rc = _call(load().ec_remerge_compact, _chk(k, "k", dt, (B, H, src_rows, D)), _chk(v, "v", dt, (B, H, src_rows, D)),
                                   src_rows, _chk(weights, "weights", i32, (B, G, L), True),
                                   _chk(src_pos, "src_pos", i32, (B, G, L), True),
                                   _chk(anchor_idx, "anchor_idx", i32, (B, G, n_anchor)), B, H, G, L, D, n_anchor,
                                   dtype_code(k), merge_mode, _chk(k_cache, "k_cache", dt, (B, H, cap, D)),
                                   _chk(v_cache, "v_cache", dt, (B, H, cap, D)), cap,
                                   _chk(counts, "counts", i32, (B, G, n_anchor), True),
                                   _chk(assign, "assign", i32, (B, G, L), True),
                                   _chk(pos, "pos", i32, (B, G, cap), True), _stream)
    if check and rc != EC_OK:
        raise EcError("ec_remerge_compact", rc)
    return rc


def ec_evict_index(n_seen: int, len_after_append: int, gamma_num: int, gamma_den: int,
                   budget_mode: int = EC_BUDGET_RATIO, fixed_len: int = 0, trunc_mode: int = EC_TRUNC_RECENT,
                   recent: int = 25, n_tl: int = 0, protect_first: int = 1) -> int:
    r = load().ec_evict_index(n_seen, len_after_append, gamma_num, gamma_den, budget_mode, fixed_len, trunc_mode,
                              recent, n_tl, protect_first)
    if r == -2:
        raise EcError("ec_evict_index", EC_EINVAL)
    return int(r)


def _decode_args(q, k_new, v_new, k_cache, v_cache, pos, out, G, what):
    """Checked pointers of the tensors every generation-step call takes."""
    if k_cache.dim() != 4:
        raise ValueError(f"{what}: k_cache must be [B,H,cap,D]")
    B, H, cap, D = k_cache.shape
    if G is None:
        G = pos.shape[1] if pos is not None else 1
    _groups(G, H, what)
    dt = k_cache.dtype
    ptrs = (_chk(q, "q", dt, (B, H, D)), _chk(k_new, "k_new", dt, (B, H, D)), _chk(v_new, "v_new", dt, (B, H, D)),
            _chk(k_cache, "k_cache", dt, (B, H, cap, D)), _chk(v_cache, "v_cache", dt, (B, H, cap, D)),
            _chk(pos, "pos", torch.int32, (B, G, cap), True))
    return ptrs, _chk(out, "out", dt, (B, H, D)), (B, H, G, D, cap)


def ec_decode_step(q, k_new, v_new, k_cache, v_cache, pos, cache_len: int, evict_idx: int, new_pos: int,
                   scale: float, out, ws, G: int | None = None, check=True) -> int:
    """q,k_new,v_new,out [B,H,D]; k_cache,v_cache [B,H,cap,D]; pos [B,G,cap] int32 or None."""
    ptrs, po, (B, H, G, D, cap) = _decode_args(q, k_new, v_new, k_cache, v_cache, pos, out, G, "ec_decode_step")
    wp, wb = _ws(ws)
    rc = _call(load().ec_decode_step, *ptrs, B, H, G, D, cap, cache_len, evict_idx, new_pos, scale, dtype_code(k_cache), po,
                               wp, wb, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_decode_step", rc)
    return rc


def ec_decode_step_shaped(q, k_new, v_new, k_cache, v_cache, pos, cache_len: int, evict_idx: int, new_pos: int,
                          scale: float, out, ws, waves: int = 0, unroll: int = 0, splits: int = 0,
                          G: int | None = None, check=True) -> int:
    """ec_decode_step with an explicit launch shape (tests and tuning sweeps)."""
    ptrs, po, (B, H, G, D, cap) = _decode_args(q, k_new, v_new, k_cache, v_cache, pos, out, G, "ec_decode_step_shaped")
    wp, wb = _ws(ws)
    rc = _call(load().ec_decode_step_shaped, *ptrs, B, H, G, D, cap, cache_len, evict_idx, new_pos, scale,
                                      dtype_code(k_cache), po, wp, wb, waves, unroll, splits, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_decode_step_shaped", rc)
    return rc


def ec_decode_score_step(q, k_new, v_new, k_cache, v_cache, pos, freq, cache_len: int, new_pos: int, scale: float,
                         out, ws, check=True) -> int:
    """Frequency policy: append + attend + add the attention row to freq [B,G,cap] f32 (no removal)."""
    if freq.dim() != 3:
        raise ValueError("ec_decode_score_step: freq must be [B,G,cap]")
    ptrs, po, (B, H, G, D, cap) = _decode_args(q, k_new, v_new, k_cache, v_cache, pos, out, freq.shape[1],
                                               "ec_decode_score_step")
    wp, wb = _ws(ws)
    rc = _call(load().ec_decode_score_step, *ptrs, _chk(freq, "freq", torch.float32, (B, G, cap)), B, H, G, D, cap, cache_len,
                                     new_pos, scale, dtype_code(k_cache), po, wp, wb, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_decode_score_step", rc)
    return rc


def ec_decode_score_step_static(q, k_new, v_new, k_cache, v_cache, pos, freq, cache_len: int, new_pos: int,
                                scale: float, out, check=True) -> int:
    """ec_decode_score_step on the library's built-in scratch: no workspace argument, nothing allocated."""
    if freq.dim() != 3:
        raise ValueError("ec_decode_score_step_static: freq must be [B,G,cap]")
    ptrs, po, (B, H, G, D, cap) = _decode_args(q, k_new, v_new, k_cache, v_cache, pos, out, freq.shape[1],
                                               "ec_decode_score_step_static")
    rc = _call(load().ec_decode_score_step_static, *ptrs, _chk(freq, "freq", torch.float32, (B, G, cap)), B, H, G, D,
               cap, cache_len, new_pos, scale, dtype_code(k_cache), po, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_decode_score_step_static", rc)
    return rc


def ec_evict_min(k_cache, v_cache, pos, freq, length: int, protect_first: int, protect_recent: int, victim,
                 check=True) -> int:
    """Frequency policy: remove the least-mass row of every (b,g); victim [B,G] int32 receives the index."""
    if k_cache.dim() != 4 or freq.dim() != 3:
        raise ValueError("ec_evict_min: k_cache must be [B,H,cap,D] and freq [B,G,cap]")
    B, H, cap, D = k_cache.shape
    G = _groups(freq.shape[1], H, "ec_evict_min")
    dt = k_cache.dtype
    rc = _call(load().ec_evict_min, _chk(k_cache, "k_cache", dt, (B, H, cap, D)), _chk(v_cache, "v_cache", dt, (B, H, cap, D)),
                             _chk(pos, "pos", torch.int32, (B, G, cap), True),
                             _chk(freq, "freq", torch.float32, (B, G, cap)), B, H, G, D, cap, length, protect_first,
                             protect_recent, dtype_code(k_cache), _chk(victim, "victim", torch.int32, (B, G)), _stream)
    if check and rc != EC_OK:
        raise EcError("ec_evict_min", rc)
    return rc


def _i32(t, name, n, optional=False):
    if t is None:
        if optional:
            return None
        raise ValueError(f"{name} is required")
    if t.dtype != torch.int32 or t.numel() != n:
        raise ValueError(f"{name} must be an int32 tensor of {n} entries")
    return _Checked(t, name)


def ec_prefill_score_varlen(q, k, v, out, lse, score, seq_len, scale: float, ws, check=True) -> int:
    """Ragged batch: q,k,v [B,H,T_max,D], seq_len int32 [B] on the device."""
    if q.dim() != 4 or score.dim() != 3:
        raise ValueError("ec_prefill_score_varlen: q must be [B,H,T,D] and score [B,G,T]")
    B, H, T, D = q.shape
    G = _groups(score.shape[1], H, "ec_prefill_score_varlen")
    dt, f32 = q.dtype, torch.float32
    wp, wb = _ws(ws)
    rc = _call(load().ec_prefill_score_varlen, _chk(q, "q", dt, (B, H, T, D)), _chk(k, "k", dt, (B, H, T, D)),
                                        _chk(v, "v", dt, (B, H, T, D)), _chk(out, "out", dt, (B, H, T, D), True),
                                        _chk(lse, "lse", f32, (B, H, T), True), _chk(score, "score", f32, (B, G, T)),
                                        _i32(seq_len, "seq_len", B), B, H, G, T, D, dtype_code(q), scale, wp, wb,
                                        _stream)
    if check and rc != EC_OK:
        raise EcError("ec_prefill_score_varlen", rc)
    return rc


def ec_select_anchors_varlen(score, seq_len, n_anchor_b, protect_first: int, protect_last: int, anchor_idx,
                             check=True) -> int:
    """Ragged batch: score [B,G,T_max], anchor_idx [B,G,n_max]; seq_len, n_anchor_b int32 [B] on the device."""
    if score.dim() != 3 or anchor_idx.dim() != 3:
        raise ValueError("ec_select_anchors_varlen: score and anchor_idx must be 3-D")
    B, G, T = score.shape
    n_max = anchor_idx.shape[2]
    rc = _call(load().ec_select_anchors_varlen, _chk(score, "score", torch.float32, (B, G, T)), _i32(seq_len, "seq_len", B),
                                         _i32(n_anchor_b, "n_anchor_b", B), B, G, T, n_max, protect_first,
                                         protect_last, _chk(anchor_idx, "anchor_idx", torch.int32, (B, G, n_max)),
                                         None, 0, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_select_anchors_varlen", rc)
    return rc


def ec_merge_compact_varlen(k, v, anchor_idx, seq_len, n_anchor_b, k_cache, v_cache, counts=None, assign=None, pos=None,
                            merge_mode: int = EC_MERGE_MEAN, check=True) -> int:
    """Ragged batch: k,v [B,H,T_max,D]; anchor_idx [B,G,n_max]; seq_len, n_anchor_b int32 [B] on the device."""
    if k.dim() != 4 or anchor_idx.dim() != 3 or k_cache.dim() != 4:
        raise ValueError("ec_merge_compact_varlen: k, k_cache must be 4-D and anchor_idx 3-D")
    B, H, T, D = k.shape
    G, n_max = _groups(anchor_idx.shape[1], H, "ec_merge_compact_varlen"), anchor_idx.shape[2]
    cap = k_cache.shape[2]
    dt, i32 = k.dtype, torch.int32
    rc = _call(load().ec_merge_compact_varlen, _chk(k, "k", dt, (B, H, T, D)), _chk(v, "v", dt, (B, H, T, D)),
                                        _chk(anchor_idx, "anchor_idx", i32, (B, G, n_max)),
                                        _i32(seq_len, "seq_len", B), _i32(n_anchor_b, "n_anchor_b", B), B, H, G, T, D,
                                        n_max, dtype_code(k), merge_mode, _chk(k_cache, "k_cache", dt, (B, H, cap, D)),
                                        _chk(v_cache, "v_cache", dt, (B, H, cap, D)), cap,
                                        _chk(counts, "counts", i32, (B, G, n_max), True),
                                        _chk(assign, "assign", i32, (B, G, T), True),
                                        _chk(pos, "pos", i32, (B, G, cap), True), _stream)
    if check and rc != EC_OK:
        raise EcError("ec_merge_compact_varlen", rc)
    return rc


def ec_decode_step_varlen(q, k_new, v_new, k_cache, v_cache, pos, cache_len_b, evict_idx_b, new_pos_b, scale: float,
                          out, G: int | None = None, ws=None, check=True) -> int:
    """Ragged batch: per-sequence cache length, victim and position as int32 [B] device tensors."""
    ptrs, po, (B, H, G, D, cap) = _decode_args(q, k_new, v_new, k_cache, v_cache, pos, out, G, "ec_decode_step_varlen")
    wp, wb = _ws(ws)
    rc = _call(load().ec_decode_step_varlen, *ptrs, _i32(cache_len_b, "cache_len_b", B),
                                      _i32(evict_idx_b, "evict_idx_b", B, True), _i32(new_pos_b, "new_pos_b", B, True),
                                      B, H, G, D, cap, scale, dtype_code(k_cache), po, wp, wb, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_decode_step_varlen", rc)
    return rc


def ec_importance_mean(score, T_new: int, P: int = 0, check=True) -> int:
    """A "Mean" metric (this library's reading of Table 3d's row), in place: score [B,G,P+T_new] f32 divided by
    the number of queries that see each row."""
    if score.dim() != 3:
        raise ValueError("ec_importance_mean: score must be [B,G,P+T_new]")
    B, G, L = score.shape
    rc = _call(load().ec_importance_mean, _chk(score, "score", torch.float32, (B, G, P + T_new)), B, G, T_new, P, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_importance_mean", rc)
    return rc


def ec_retention_step_varlen(n_seen_b, cache_len_b, evict_idx_b, new_pos_b, pending_b, gamma_num: int, gamma_den: int,
                             budget_mode: int = EC_BUDGET_RATIO, fixed_len: int = 0, trunc_mode: int = EC_TRUNC_RECENT,
                             recent: int = 25, n_tl: int = 0, protect_first: int = 1, flush_only: bool = False,
                             check=True) -> int:
    """Device-side retention test of a ragged batch; all arrays int32 [B] on the device, updated in place."""
    B = n_seen_b.numel()
    rc = _call(load().ec_retention_step_varlen, _i32(n_seen_b, "n_seen_b", B), _i32(cache_len_b, "cache_len_b", B),
                                         _i32(evict_idx_b, "evict_idx_b", B), _i32(new_pos_b, "new_pos_b", B),
                                         _i32(pending_b, "pending_b", B), B, gamma_num, gamma_den, budget_mode, fixed_len,
                                         trunc_mode, recent, n_tl, protect_first, 1 if flush_only else 0, _stream)
    if check and rc != EC_OK:
        raise EcError("ec_retention_step_varlen", rc)
    return rc
