"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and its
host-only entry points (status strings, workspace sizes, retention test) behave.  No kernels run."""
import ctypes
import os
import re

import pytest

import oracle
from paper_2407_18121_amd import binding as ec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ec.h")).read()
    declared = set(re.findall(r"\b(ec_[a-z_]+)\s*\(", header))
    assert declared == set(ec.SYMBOLS), declared ^ set(ec.SYMBOLS)
    lib = ctypes.CDLL(ec.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings_and_workspace_sizes():
    assert ec.status_string(ec.EC_OK) == "EC_OK"
    for code in (1, 2, 3, 4):
        assert ec.status_string(code).startswith("EC_E")
    assert ec.ec_workspace_bytes(ec.EC_FN_SELECT_ANCHORS, 1, 1, 16, 64, ec.EC_F32) == 0
    n = ec.ec_workspace_bytes(ec.EC_FN_PREFILL_SCORE, 2, 4, 100, 64, ec.EC_F32)
    assert n >= 2 * 2 * 4 * 100 * 4 and n % 256 == 0
    assert ec.ec_workspace_bytes(ec.EC_FN_DECODE_STEP, 2, 4, 100, 128, ec.EC_BF16) == 0
    with pytest.raises(ec.EcError):
        ec.ec_workspace_bytes(ec.EC_FN_DECODE_STEP, 2, 4, 100, 96, ec.EC_BF16)


def test_invalid_arguments_are_rejected_before_any_launch():
    lib = ec.load()
    # NULL pointers / bad shapes: the host returns before touching the device
    assert lib.ec_select_anchors(None, 1, 1, 8, 4, 1, 1, None, None, 0, None) == ec.EC_EINVAL
    assert lib.ec_merge_compact(None, None, None, 1, 1, 1, 8, 64, 4, 0, 0, None, None, 4, None, None, None, None) == ec.EC_EINVAL
    assert lib.ec_decode_step(None, None, None, None, None, None, 1, 1, 1, 64, 8, 0, -1, 0, 1.0, 0, None, None, 0, None) == ec.EC_EINVAL
    assert lib.ec_prefill_score(None, None, None, None, None, None, 1, 1, 1, 8, 64, 0, 1.0, None, 0, None) == ec.EC_EINVAL
    one = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    assert lib.ec_select_anchors(one, 1, 1, 8, 9, 1, 1, one, None, 0, None) == ec.EC_EINVAL       # n_anchor > T
    assert lib.ec_select_anchors(one, 1, 1, 8, 2, 2, 1, one, None, 0, None) == ec.EC_EINVAL       # protected > n_anchor
    assert lib.ec_decode_step(one, one, one, one, one, None, 1, 1, 1, 64, 8, 8, -1, 0, 1.0, 0, one, one, 1 << 20, None) == ec.EC_EINVAL  # full
    assert lib.ec_decode_step(one, one, one, one, one, None, 1, 1, 1, 64, 8, 3, 4, 0, 1.0, 0, one, one, 1 << 20, None) == ec.EC_EINVAL   # evict > len
    assert lib.ec_decode_step(one, one, one, one, one, None, 1, 1, 1, 96, 8, 3, 1, 0, 1.0, 0, one, one, 1 << 20, None) == ec.EC_EUNSUPPORTED
    assert lib.ec_prefill_score(one, one, one, None, None, one, 1, 1, 1, 8, 64, 0, 1.0, one, 16, None) == ec.EC_EWORKSPACE
    assert lib.ec_merge_compact(one, one, one, 1, 4, 2, 8, 64, 4, 0, 0, one, one, 4, None, None, None, None) == ec.EC_EINVAL  # G not in {1,H}
    assert lib.ec_merge_compact(one, one, one, 1, 4, 1, 8, 64, 4, 0, 7, one, one, 4, None, None, None, None) == ec.EC_EINVAL  # merge_mode
    two = ctypes.c_void_p(512)
    assert lib.ec_merge_compact(one, one, one, 1, 4, 1, 8, 64, 4, 0, 0, one, two, 4, None, None, None, None) == ec.EC_EINVAL  # in place
    assert lib.ec_remerge_compact(one, one, 7, None, None, one, 1, 4, 1, 8, 64, 4, 0, 0, two, two, 4, None, None, None, None) == ec.EC_EINVAL  # src_rows < L
    assert lib.ec_chunk_score(None, None, None, None, None, None, 1, 1, 1, 8, 4, 12, 64, 0, 1.0, None, 0, None) == ec.EC_EINVAL
    assert lib.ec_chunk_score(one, one, one, None, None, one, 1, 1, 1, 8, 4, 11, 64, 0, 1.0, one, 1 << 20, None) == ec.EC_EINVAL  # kv_rows < P + T_new
    assert lib.ec_chunk_score(one, one, one, None, None, one, 1, 1, 1, 0, 4, 12, 64, 0, 1.0, one, 1 << 20, None) == ec.EC_EINVAL  # empty chunk
    assert lib.ec_chunk_score(one, one, one, None, None, one, 1, 1, 1, 8, -1, 12, 64, 0, 1.0, one, 1 << 20, None) == ec.EC_EINVAL  # negative prefix
    assert lib.ec_chunk_score(one, one, one, None, None, one, 1, 1, 1, 8, 4, 12, 64, 0, 1.0, one, 16, None) == ec.EC_EWORKSPACE
    # ragged-batch and frequency-policy entry points
    assert lib.ec_prefill_score_varlen(one, one, one, None, None, one, None, 1, 1, 1, 8, 64, 0, 1.0, one, 1 << 20, None) == ec.EC_EINVAL  # no seq_len
    assert lib.ec_select_anchors_varlen(one, one, None, 1, 1, 8, 4, 1, 1, one, None, 0, None) == ec.EC_EINVAL
    assert lib.ec_select_anchors_varlen(one, one, one, 1, 1, 8, 9, 1, 1, one, None, 0, None) == ec.EC_EINVAL  # n_max > T_max
    assert lib.ec_merge_compact_varlen(one, one, one, one, None, 1, 1, 1, 8, 64, 4, 0, 0, two, two, 4, None, None, None, None) == ec.EC_EINVAL
    assert lib.ec_decode_step_varlen(one, one, one, one, one, None, None, None, None, 1, 1, 1, 64, 8, 1.0, 0, one, None, 0, None) == ec.EC_EINVAL
    assert lib.ec_decode_step_varlen(one, one, one, one, one, one, one, None, None, 1, 1, 1, 64, 8, 1.0, 0, one, None, 0, None) == ec.EC_EINVAL  # pos without new_pos_b
    assert lib.ec_decode_score_step(one, one, one, one, one, None, None, 1, 1, 1, 64, 8, 3, 0, 1.0, 0, one, one, 1 << 20, None) == ec.EC_EINVAL  # no freq
    assert lib.ec_decode_score_step(one, one, one, one, one, None, one, 1, 1, 1, 64, 8, 3, 0, 1.0, 0, one, one, 16, None) == ec.EC_EWORKSPACE
    assert lib.ec_evict_min(one, one, None, one, 1, 1, 1, 64, 8, 3, 2, 1, 0, one, None) == ec.EC_EINVAL   # nothing left to choose from
    assert lib.ec_evict_min(one, one, None, one, 1, 1, 1, 64, 8, 9, 1, 1, 0, one, None) == ec.EC_EINVAL   # len > cap
    assert lib.ec_retention_step_varlen(one, one, one, one, None, 4, 1, 2, 0, 0, 0, 25, 0, 1, 0, None) == ec.EC_EINVAL  # no pending_b
    assert lib.ec_retention_step_varlen(one, one, one, one, one, 4, 3, 2, 0, 0, 0, 25, 0, 1, 0, None) == ec.EC_EINVAL   # gamma > 1
    assert lib.ec_retention_step_varlen(one, one, one, one, one, 4, 1, 2, 1, 0, 0, 25, 0, 1, 0, None) == ec.EC_EINVAL   # fixed_len < 1
    assert lib.ec_importance_mean(None, 1, 1, 8, 0, None) == ec.EC_EINVAL
    assert lib.ec_importance_mean(one, 1, 1, 0, 0, None) == ec.EC_EINVAL


def test_evict_index_matches_oracle_everywhere():
    for gamma in ((1, 2), (1, 4), (1, 10), (3, 7), (1, 1)):
        for budget_mode, trunc_mode in ((0, 0), (1, 0), (0, 1), (1, 1)):
            for n_seen in (1, 2, 5, 26, 27, 100, 1025, 9000):
                for length in (1, 2, 3, 26, 27, 28, 60, 513, 900):
                    for pf in (0, 1, 4):
                        kw = dict(budget_mode=budget_mode, fixed_len=50, trunc_mode=trunc_mode, recent=25,
                                  n_tl=40, protect_first=pf)
                        assert (ec.ec_evict_index(n_seen, length, *gamma, **kw)
                                == oracle.evict_index(n_seen, length, *gamma, **kw)), (gamma, kw, n_seen, length)
    with pytest.raises(ec.EcError):
        ec.ec_evict_index(0, 5, 1, 2)
    with pytest.raises(ec.EcError):
        ec.ec_evict_index(5, 5, 3, 2)


def test_config_lengths_match_the_hand_worked_retention_table():
    """The anchor count and cache capacity both sides of every parity test take from the config table are
    Alg. 1's del_num rounding: pinned to tests/golden/retention_lengths.txt (worked in exact rationals)."""
    from paper_2407_18121_amd import synthetic as syn
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "retention_lengths.txt"))
            if l.strip() and not l.startswith("#")]
    assert {r[0] for r in rows} == set(syn.CONFIGS)
    for name, T, p, q, steps, after_prompt, after_gen in rows:
        cfg = syn.CONFIGS[name]
        assert (cfg.T, cfg.gamma, cfg.decode_steps) == (int(T), (int(p), int(q)), int(steps)), name
        assert cfg.n_anchor == int(after_prompt), name
        assert cfg.cap == int(after_gen) + 1, name          # one spare row for the append before the removal
        # and the library's own retention test walks from the first length to the second
        n = cfg.n_anchor
        for step in range(cfg.decode_steps):
            n += 0 if ec.ec_evict_index(cfg.T + step + 1, n + 1, int(p), int(q)) >= 0 else 1
            assert n < cfg.cap
        assert n == int(after_gen), name


def test_binding_rejects_wrong_types_and_shapes_before_any_call():
    """The C ABI sees raw pointers only; the binding refuses tensors whose element type or shape does not fit
    the call (a kernel would otherwise run out of bounds).  Host tensors: nothing is launched."""
    import torch
    B, H, T, D, G, cap, n = 2, 4, 16, 64, 1, 12, 8
    f32, bf16, i32 = torch.float32, torch.bfloat16, torch.int32
    q = torch.zeros((B, H, T, D), dtype=bf16)
    score = torch.zeros((B, G, T), dtype=f32)
    with pytest.raises(ValueError, match="score must be torch.float32"):
        ec.ec_prefill_score(q, q, q, None, None, score.to(bf16), 0.1, None)
    with pytest.raises(ValueError, match="lse must have shape"):
        ec.ec_prefill_score(q, q, q, None, torch.zeros((B, H), dtype=f32), score, 0.1, None)
    with pytest.raises(ValueError, match="k must be torch.bfloat16"):
        ec.ec_prefill_score(q, q.float(), q, None, None, score, 0.1, None)
    with pytest.raises(ValueError, match="v must have shape"):
        ec.ec_prefill_score(q, q, q[:, :, :-1], None, None, score, 0.1, None)
    with pytest.raises(ValueError, match="score groups"):
        ec.ec_prefill_score(q, q, q, None, None, torch.zeros((B, 2, T), dtype=f32), 0.1, None)
    with pytest.raises(ValueError, match="device memory"):   # everything fits: only the device is wrong
        ec.ec_prefill_score(q, q, q, None, None, score, 0.1, None)
    with pytest.raises(ValueError, match="anchor_idx must be torch.int32"):
        ec.ec_select_anchors(score, n, 1, 1, torch.zeros((B, G, n), dtype=torch.int64))
    with pytest.raises(ValueError, match="anchor_idx must have shape"):
        ec.ec_select_anchors(score, n, 1, 1, torch.zeros((B, G, n - 1), dtype=i32))
    kc = torch.zeros((B, H, cap, D), dtype=bf16)
    a = torch.zeros((B, G, n), dtype=i32)
    with pytest.raises(ValueError, match="v_cache must have shape"):
        ec.ec_merge_compact(q, q, a, kc, kc[:, :, :-1], None, None, None)
    with pytest.raises(ValueError, match="counts must have shape"):
        ec.ec_merge_compact(q, q, a, kc, kc, torch.zeros((B, G, n + 1), dtype=i32), None, None)
    with pytest.raises(ValueError, match="pos must be torch.int32"):
        ec.ec_merge_compact(q, q, a, kc, kc, None, None, torch.zeros((B, G, cap), dtype=f32))
    x = torch.zeros((B, H, D), dtype=bf16)
    with pytest.raises(ValueError, match="k_new must have shape"):
        ec.ec_decode_step(x, x[:, :1], x, kc, kc, None, 3, -1, 0, 0.1, x, None, G=1)
    with pytest.raises(ValueError, match="out must be torch.bfloat16"):
        ec.ec_decode_step(x, x, x, kc, kc, None, 3, -1, 0, 0.1, x.float(), None, G=1)
    with pytest.raises(ValueError, match="q must be torch.bfloat16"):
        ec.ec_decode_step(x.float(), x, x, kc, kc, None, 3, -1, 0, 0.1, x, None, G=1)
    with pytest.raises(ValueError, match="freq must be torch.float32"):
        ec.ec_decode_score_step(x, x, x, kc, kc, None, torch.zeros((B, G, cap), dtype=bf16), 3, 0, 0.1, x, None)
    with pytest.raises(ValueError, match="victim must have shape"):
        ec.ec_evict_min(kc, kc, None, torch.zeros((B, G, cap), dtype=f32), 5, 1, 1, torch.zeros((B,), dtype=i32))
    with pytest.raises(ValueError, match="cache_len_b must be an int32 tensor"):
        ec.ec_decode_step_varlen(x, x, x, kc, kc, None, torch.zeros((B + 1,), dtype=i32), None, None, 0.1, x, G=1)


def test_scale_must_be_finite_and_positive():
    lib = ec.load()
    one = ctypes.c_void_p(256)
    for bad in (0.0, -0.5, float("inf"), float("nan")):
        assert lib.ec_prefill_score(one, one, one, None, None, one, 1, 1, 1, 8, 64, 0, bad, one, 1 << 20, None) == ec.EC_EINVAL
        assert lib.ec_decode_step(one, one, one, one, one, None, 1, 1, 1, 64, 8, 3, -1, 0, bad, 0, one, None, 0, None) == ec.EC_EINVAL
        assert lib.ec_decode_step_shaped(one, one, one, one, one, None, 1, 1, 1, 64, 8, 3, -1, 0, bad, 0, one, None, 0,
                                         0, 0, 0, None) == ec.EC_EINVAL


def test_tune_tool_usage():
    """The timing tool prints its usage for an unknown table and refuses to run without a GPU."""
    import torch
    from paper_2407_18121_amd import tune
    assert tune.main(["tune"]) == 2
    assert tune.main(["tune", "nonsense"]) == 2
    if not torch.cuda.is_available():
        assert tune.main(["tune", "decode"]) == 1
