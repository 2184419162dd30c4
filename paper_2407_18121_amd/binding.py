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
           "ec_decode_step_varlen", "ec_importance_mean", "ec_retention_step_varlen")

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
    lib.ec_decode_score_step.argtypes = ([c_vp] * 7 + [c_int] * 6 + [ctypes.c_int32, c_f, c_int, c_vp, c_vp, c_sz, c_vp])
    lib.ec_decode_score_step.restype = c_int
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
    B, H, T, D = q.shape
    G = score.shape[1]
    rc = load().ec_prefill_score(_ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(out, "out"), _ptr(lse, "lse"),
                                 _ptr(score, "score"), B, H, G, T, D, dtype_code(q), scale, _ptr(ws, "ws"),
                                 0 if ws is None else ws.numel() * ws.element_size(), _stream())
    if check and rc != EC_OK:
        raise EcError("ec_prefill_score", rc)
    return rc


def ec_chunk_score(q, k, v, P: int, out, lse, score, scale: float, ws, check=True) -> int:
    """q [B,H,T_new,D]; k,v [B,H,kv_rows,D] holding P cached rows then the chunk's rows; score [B,G,P+T_new]."""
    B, H, T_new, D = q.shape
    kv_rows = k.shape[2]
    G = score.shape[1]
    if k.shape != v.shape or k.shape[:2] != q.shape[:2] or k.shape[3] != D or score.shape[2] != P + T_new:
        raise ValueError("ec_chunk_score: inconsistent shapes")
    rc = load().ec_chunk_score(_ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(out, "out"), _ptr(lse, "lse"),
                               _ptr(score, "score"), B, H, G, T_new, P, kv_rows, D, dtype_code(q), scale,
                               _ptr(ws, "ws"), 0 if ws is None else ws.numel() * ws.element_size(), _stream())
    if check and rc != EC_OK:
        raise EcError("ec_chunk_score", rc)
    return rc


def ec_select_anchors(score, n_anchor: int, protect_first: int, protect_last: int, anchor_idx, check=True) -> int:
    """score [B,G,T] f32 -> anchor_idx [B,G,n_anchor] int32 ascending."""
    B, G, T = score.shape
    rc = load().ec_select_anchors(_ptr(score, "score"), B, G, T, n_anchor, protect_first, protect_last,
                                  _ptr(anchor_idx, "anchor_idx"), None, 0, _stream())
    if check and rc != EC_OK:
        raise EcError("ec_select_anchors", rc)
    return rc


def ec_merge_compact(k, v, anchor_idx, k_cache, v_cache, counts=None, assign=None, pos=None,
                     merge_mode: int = EC_MERGE_MEAN, check=True) -> int:
    """k,v [B,H,T,D]; anchor_idx [B,G,n]; k_cache,v_cache [B,H,cap,D]."""
    B, H, T, D = k.shape
    G, n_anchor = anchor_idx.shape[1], anchor_idx.shape[2]
    cap = k_cache.shape[2]
    rc = load().ec_merge_compact(_ptr(k, "k"), _ptr(v, "v"), _ptr(anchor_idx, "anchor_idx"), B, H, G, T, D, n_anchor,
                                 dtype_code(k), merge_mode, _ptr(k_cache, "k_cache"), _ptr(v_cache, "v_cache"), cap,
                                 _ptr(counts, "counts"), _ptr(assign, "assign"), _ptr(pos, "pos"), _stream())
    if check and rc != EC_OK:
        raise EcError("ec_merge_compact", rc)
    return rc


def ec_remerge_compact(k, v, L: int, anchor_idx, k_cache, v_cache, weights=None, src_pos=None, counts=None,
                       assign=None, pos=None, merge_mode: int = EC_MERGE_MEAN, check=True) -> int:
    """k,v [B,H,src_rows,D] of which rows 0..L-1 are merged; weights, src_pos [B,G,L] int32 or None."""
    B, H, src_rows, D = k.shape
    G, n_anchor = anchor_idx.shape[1], anchor_idx.shape[2]
    cap = k_cache.shape[2]
    for name, t in (("weights", weights), ("src_pos", src_pos)):
        if t is not None and tuple(t.shape) != (B, G, L):
            raise ValueError(f"ec_remerge_compact: {name} must be [B,G,L]")
    rc = load().ec_remerge_compact(_ptr(k, "k"), _ptr(v, "v"), src_rows, _ptr(weights, "weights"),
                                   _ptr(src_pos, "src_pos"), _ptr(anchor_idx, "anchor_idx"), B, H, G, L, D,
                                   n_anchor, dtype_code(k), merge_mode, _ptr(k_cache, "k_cache"),
                                   _ptr(v_cache, "v_cache"), cap, _ptr(counts, "counts"), _ptr(assign, "assign"),
                                   _ptr(pos, "pos"), _stream())
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


def ec_decode_step(q, k_new, v_new, k_cache, v_cache, pos, cache_len: int, evict_idx: int, new_pos: int,
                   scale: float, out, ws, G: int | None = None, check=True) -> int:
    """q,k_new,v_new,out [B,H,D]; k_cache,v_cache [B,H,cap,D]; pos [B,G,cap] int32 or None."""
    B, H, cap, D = k_cache.shape
    if G is None:
        G = pos.shape[1] if pos is not None else 1
    rc = load().ec_decode_step(_ptr(q, "q"), _ptr(k_new, "k_new"), _ptr(v_new, "v_new"), _ptr(k_cache, "k_cache"),
                               _ptr(v_cache, "v_cache"), _ptr(pos, "pos"), B, H, G, D, cap, cache_len, evict_idx,
                               new_pos, scale, dtype_code(k_cache), _ptr(out, "out"), _ptr(ws, "ws"),
                               0 if ws is None else ws.numel() * ws.element_size(), _stream())
    if check and rc != EC_OK:
        raise EcError("ec_decode_step", rc)
    return rc


def ec_decode_score_step(q, k_new, v_new, k_cache, v_cache, pos, freq, cache_len: int, new_pos: int, scale: float,
                         out, ws, check=True) -> int:
    """Frequency policy: append + attend + add the attention row to freq [B,G,cap] f32 (no removal)."""
    B, H, cap, D = k_cache.shape
    G = freq.shape[1]
    rc = load().ec_decode_score_step(_ptr(q, "q"), _ptr(k_new, "k_new"), _ptr(v_new, "v_new"), _ptr(k_cache, "k_cache"),
                                     _ptr(v_cache, "v_cache"), _ptr(pos, "pos"), _ptr(freq, "freq"), B, H, G, D, cap,
                                     cache_len, new_pos, scale, dtype_code(k_cache), _ptr(out, "out"), _ptr(ws, "ws"),
                                     0 if ws is None else ws.numel() * ws.element_size(), _stream())
    if check and rc != EC_OK:
        raise EcError("ec_decode_score_step", rc)
    return rc


def ec_evict_min(k_cache, v_cache, pos, freq, length: int, protect_first: int, protect_recent: int, victim,
                 check=True) -> int:
    """Frequency policy: remove the least-mass row of every (b,g); victim [B,G] int32 receives the index."""
    B, H, cap, D = k_cache.shape
    G = freq.shape[1]
    rc = load().ec_evict_min(_ptr(k_cache, "k_cache"), _ptr(v_cache, "v_cache"), _ptr(pos, "pos"), _ptr(freq, "freq"),
                             B, H, G, D, cap, length, protect_first, protect_recent, dtype_code(k_cache),
                             _ptr(victim, "victim"), _stream())
    if check and rc != EC_OK:
        raise EcError("ec_evict_min", rc)
    return rc


def _i32(t, name, n):
    if t is None:
        return None
    if t.dtype != torch.int32 or t.numel() != n:
        raise ValueError(f"{name} must be an int32 tensor of {n} entries")
    return _ptr(t, name)


def ec_prefill_score_varlen(q, k, v, out, lse, score, seq_len, scale: float, ws, check=True) -> int:
    """Ragged batch: q,k,v [B,H,T_max,D], seq_len int32 [B] on the device."""
    B, H, T, D = q.shape
    G = score.shape[1]
    rc = load().ec_prefill_score_varlen(_ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(out, "out"), _ptr(lse, "lse"),
                                        _ptr(score, "score"), _i32(seq_len, "seq_len", B), B, H, G, T, D, dtype_code(q),
                                        scale, _ptr(ws, "ws"), 0 if ws is None else ws.numel() * ws.element_size(),
                                        _stream())
    if check and rc != EC_OK:
        raise EcError("ec_prefill_score_varlen", rc)
    return rc


def ec_select_anchors_varlen(score, seq_len, n_anchor_b, protect_first: int, protect_last: int, anchor_idx,
                             check=True) -> int:
    """Ragged batch: score [B,G,T_max], anchor_idx [B,G,n_max]; seq_len, n_anchor_b int32 [B] on the device."""
    B, G, T = score.shape
    rc = load().ec_select_anchors_varlen(_ptr(score, "score"), _i32(seq_len, "seq_len", B),
                                         _i32(n_anchor_b, "n_anchor_b", B), B, G, T, anchor_idx.shape[2], protect_first,
                                         protect_last, _ptr(anchor_idx, "anchor_idx"), None, 0, _stream())
    if check and rc != EC_OK:
        raise EcError("ec_select_anchors_varlen", rc)
    return rc


def ec_merge_compact_varlen(k, v, anchor_idx, seq_len, n_anchor_b, k_cache, v_cache, counts=None, assign=None, pos=None,
                            merge_mode: int = EC_MERGE_MEAN, check=True) -> int:
    """Ragged batch: k,v [B,H,T_max,D]; anchor_idx [B,G,n_max]; seq_len, n_anchor_b int32 [B] on the device."""
    B, H, T, D = k.shape
    G, n_max = anchor_idx.shape[1], anchor_idx.shape[2]
    rc = load().ec_merge_compact_varlen(_ptr(k, "k"), _ptr(v, "v"), _ptr(anchor_idx, "anchor_idx"),
                                        _i32(seq_len, "seq_len", B), _i32(n_anchor_b, "n_anchor_b", B), B, H, G, T, D,
                                        n_max, dtype_code(k), merge_mode, _ptr(k_cache, "k_cache"),
                                        _ptr(v_cache, "v_cache"), k_cache.shape[2], _ptr(counts, "counts"),
                                        _ptr(assign, "assign"), _ptr(pos, "pos"), _stream())
    if check and rc != EC_OK:
        raise EcError("ec_merge_compact_varlen", rc)
    return rc


def ec_decode_step_varlen(q, k_new, v_new, k_cache, v_cache, pos, cache_len_b, evict_idx_b, new_pos_b, scale: float,
                          out, G: int | None = None, check=True) -> int:
    """Ragged batch: per-sequence cache length, victim and position as int32 [B] device tensors."""
    B, H, cap, D = k_cache.shape
    if G is None:
        G = pos.shape[1] if pos is not None else 1
    rc = load().ec_decode_step_varlen(_ptr(q, "q"), _ptr(k_new, "k_new"), _ptr(v_new, "v_new"), _ptr(k_cache, "k_cache"),
                                      _ptr(v_cache, "v_cache"), _ptr(pos, "pos"), _i32(cache_len_b, "cache_len_b", B),
                                      _i32(evict_idx_b, "evict_idx_b", B), _i32(new_pos_b, "new_pos_b", B), B, H, G, D,
                                      cap, scale, dtype_code(k_cache), _ptr(out, "out"), None, 0, _stream())
    if check and rc != EC_OK:
        raise EcError("ec_decode_step_varlen", rc)
    return rc


def ec_importance_mean(score, T_new: int, P: int = 0, check=True) -> int:
    """Table 3d's "Mean" metric, in place: score [B,G,P+T_new] f32 divided by the number of seeing queries."""
    B, G, L = score.shape
    if L != P + T_new or score.dtype != torch.float32:
        raise ValueError("ec_importance_mean: score must be float32 [B,G,P+T_new]")
    rc = load().ec_importance_mean(_ptr(score, "score"), B, G, T_new, P, _stream())
    if check and rc != EC_OK:
        raise EcError("ec_importance_mean", rc)
    return rc


def ec_retention_step_varlen(n_seen_b, cache_len_b, evict_idx_b, new_pos_b, pending_b, gamma_num: int, gamma_den: int,
                             budget_mode: int = EC_BUDGET_RATIO, fixed_len: int = 0, trunc_mode: int = EC_TRUNC_RECENT,
                             recent: int = 25, n_tl: int = 0, protect_first: int = 1, flush_only: bool = False,
                             check=True) -> int:
    """Device-side retention test of a ragged batch; all arrays int32 [B] on the device, updated in place."""
    B = n_seen_b.numel()
    rc = load().ec_retention_step_varlen(_i32(n_seen_b, "n_seen_b", B), _i32(cache_len_b, "cache_len_b", B),
                                         _i32(evict_idx_b, "evict_idx_b", B), _i32(new_pos_b, "new_pos_b", B),
                                         _i32(pending_b, "pending_b", B), B, gamma_num, gamma_den, budget_mode, fixed_len,
                                         trunc_mode, recent, n_tl, protect_first, 1 if flush_only else 0, _stream())
    if check and rc != EC_OK:
        raise EcError("ec_retention_step_varlen", rc)
    return rc
