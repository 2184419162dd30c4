"""GPU parity: ec_prefill_score vs the CPU oracle (Sec. 3.3, Eq. 1 and the importance I_n)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_18121_amd import binding as ec
from paper_2407_18121_amd import synthetic as syn
from util import assert_close, to_dev, to_host, torch_dtype

pytestmark = pytest.mark.gpu


def run_gpu_score(q, k, v, dtype, scale, G, want_out=True, want_lse=True):
    B, H, T, D = q.shape
    dq, dk, dv = to_dev(q, dtype), to_dev(k, dtype), to_dev(v, dtype)
    out = torch.full((B, H, T, D), float("nan"), dtype=torch_dtype(dtype), device="cuda") if want_out else None
    lse = torch.full((B, H, T), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    score = torch.full((B, G, T), float("nan"), dtype=torch.float32, device="cuda")
    ws = ec.new_workspace(ec.EC_FN_PREFILL_SCORE, B, H, T, D, ec.dtype_code(dq))
    ec.ec_prefill_score(dq, dk, dv, out, lse, score, scale, ws)
    torch.cuda.synchronize()
    return (None if out is None else to_host(out), None if lse is None else to_host(lse), to_host(score))


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128), ("bf16", 64), ("f32", 128)])
@pytest.mark.parametrize("B,H,T,Gmode", [(1, 2, 1, "layer"), (2, 3, 37, "head"), (1, 4, 256, "layer"),
                                         (2, 2, 321, "layer"), (1, 2, 700, "head")])
def test_prefill_score_parity(dtype, D, B, H, T, Gmode):
    cfg = syn.custom("t", H=H, D=D, B=B, T=T, dtype=dtype, cid=1000 + T)
    q, k, v = syn.prompt_qkv(cfg)
    G = 1 if Gmode == "layer" else H
    ref = oracle.prefill_score(q, k, v, cfg.scale, G)
    out, lse, score = run_gpu_score(q, k, v, dtype, cfg.scale, G)
    assert_close(out, ref["out"], dtype, "out")
    assert_close(lse, ref["lse"], dtype, "lse")
    assert_close(score, ref["score"], dtype, "score")
    np.testing.assert_allclose(score.sum(-1), T, rtol=1e-5)          # rows of A sum to one


def test_prefill_score_optional_outputs_and_literal_eq1_scale():
    cfg = syn.custom("t", H=2, D=64, B=1, T=150, dtype="f32", cid=1234)
    q, k, v = syn.prompt_qkv(cfg)
    q = (q * 0.2).astype(np.float32)
    ref = oracle.prefill_score(q, k, v, 1.0, 1)
    out, lse, score = run_gpu_score(q, k, v, "f32", 1.0, 1, want_out=False, want_lse=False)
    assert out is None and lse is None
    assert_close(score, ref["score"], "f32", "score")


def test_tiny_config_full_layer():
    cfg = syn.CONFIGS["C1"]
    q, k, v = syn.prompt_qkv(cfg)
    for G in (1, cfg.H):
        ref = oracle.prefill_score(q, k, v, cfg.scale, G)
        out, lse, score = run_gpu_score(q, k, v, cfg.dtype, cfg.scale, G)
        assert_close(out, ref["out"], cfg.dtype, "out")
        assert_close(lse, ref["lse"], cfg.dtype, "lse")
        assert_close(score, ref["score"], cfg.dtype, "score")


@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("B,H,T", [
    (1, 2, 255, ),    # one key tile short of the two-group launch shape
    (1, 2, 256, ),    # its first length
    (2, 16, 1024, ),  # 256 workgroups: the largest launch that takes it
    (1, 33, 1024, ),  # 264 workgroups: the smallest that does not
    (1, 3, 1100, ),   # odd number of key and of query tiles, ragged tail
])
def test_prefill_score_launch_shapes_of_short_prompts(D, B, H, T):
    """bf16 launches of at most 256 workgroups run two wave groups per workgroup (alternate key tiles in the
    forward pass, alternate query tiles in the column pass); both sides of every threshold are checked."""
    cfg = syn.custom("t", H=H, D=D, B=B, T=T, dtype="bf16", cid=4000 + T + H)
    q, k, v = syn.prompt_qkv(cfg)
    ref = oracle.prefill_score(q, k, v, cfg.scale, 1)
    out, lse, score = run_gpu_score(q, k, v, "bf16", cfg.scale, 1)
    assert_close(out, ref["out"], "bf16", "out")
    assert_close(lse, ref["lse"], "bf16", "lse")
    assert_close(score, ref["score"], "bf16", "score")
    np.testing.assert_allclose(score.sum(-1), T, rtol=1e-5)


@pytest.mark.parametrize("B,G,Tq,P", [(2, 3, 300, 0), (1, 1, 37, 120), (3, 2, 1, 64), (1, 4, 5000, 700)])
def test_importance_mean_metric(B, G, Tq, P):
    """Table 3d's "Mean" metric: the sums divided by the number of queries that see each row."""
    rng = np.random.default_rng(Tq + P)
    L = P + Tq
    sums = (rng.random((B, G, L)) * (1.0 + 300.0 / (1 + np.arange(L)))).astype(np.float32)
    ref = oracle.importance_mean(sums.astype(np.float64), Tq, P)
    d = torch.from_numpy(sums).cuda()
    ec.ec_importance_mean(d, Tq, P)
    torch.cuda.synchronize()
    np.testing.assert_allclose(d.cpu().numpy().astype(np.float64), ref, rtol=3e-7, atol=0)   # one fp32 division


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_peaked_and_flat_attention(dtype, D):
    """Scores hundreds of units apart (softmax one-hot to fp32 precision) and all-equal scores (uniform rows)."""
    cfg = syn.custom("t", H=2, D=D, B=1, T=300, dtype=dtype, cid=8080)
    q, k, v = syn.prompt_qkv(cfg)
    from util import quantize
    for gain, scale in ((6.0, 1.0), (0.0, 1.0)):
        qq = quantize(q * gain, dtype)
        ref = oracle.prefill_score(qq, k, v, scale, 1)
        out, lse, score = run_gpu_score(qq, k, v, dtype, scale, 1)
        assert np.isfinite(out).all() and np.isfinite(lse).all() and np.isfinite(score).all()
        assert_close(out, ref["out"], dtype, f"out gain {gain}")
        assert_close(score, ref["score"], dtype, f"score gain {gain}")
        # the log-sum-exp itself is hundreds of units large here: compare relative to its size
        np.testing.assert_allclose(lse, ref["lse"], rtol=2e-6 if dtype == "f32" else 1e-5, atol=2e-2 if dtype == "bf16" else 1e-4)
