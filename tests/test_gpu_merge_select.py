"""GPU parity: ec_select_anchors and ec_merge_compact vs the CPU oracle (Sec. 3.3, Eq. 2-3; Sec. 4.1)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_18121_amd import binding as ec
from util import assert_close, quantize, to_dev, to_host, torch_dtype

pytestmark = pytest.mark.gpu


def _gpu_select(score, n, pf, pl):
    B, G, T = score.shape
    idx = torch.full((B, G, n), -1, dtype=torch.int32, device="cuda")
    ec.ec_select_anchors(torch.from_numpy(score).cuda(), n, pf, pl, idx)
    torch.cuda.synchronize()
    return idx.cpu().numpy()


@pytest.mark.parametrize("B,G,T,n,pf,pl", [
    (1, 1, 1, 1, 0, 0), (1, 1, 1, 1, 1, 0), (2, 3, 37, 10, 1, 1), (1, 4, 256, 128, 1, 1), (2, 2, 1024, 512, 1, 1),
    (3, 1, 1500, 1, 0, 0), (1, 2, 1500, 1500, 1, 1), (2, 2, 2048, 512, 4, 8), (1, 3, 8192, 820, 1, 1),
    (2, 1, 8193, 3000, 1, 1), (1, 2, 20000, 2000, 2, 3), (1, 1, 65536, 6554, 1, 1), (4, 8, 1000, 2, 1, 1),
])
def test_select_bit_exact(B, G, T, n, pf, pl):
    rng = np.random.default_rng(T * 31 + n)
    # column-mass-like scores: positive, decaying with position, a few heavy hitters
    score = (rng.random((B, G, T)) * (1.0 + 20.0 / (1 + np.arange(T)))).astype(np.float32)
    score[..., rng.choice(T, max(1, T // 20), replace=False)] *= 30
    np.testing.assert_array_equal(_gpu_select(score, n, pf, pl), oracle.select_anchors(score, n, pf, pl))


@pytest.mark.parametrize("T,n", [(300, 100), (5000, 2500), (9000, 1000)])
def test_select_ties_and_special_values(T, n):
    rng = np.random.default_rng(T)
    s = np.round(rng.random((2, 2, T)) * 8).astype(np.float32) / 8      # heavy ties
    s[0, 0] = 1.0                                                       # all equal
    s[0, 1, ::2] = 0.0
    s[0, 1, 1::4] = -0.0                                                # signed zeros are equal
    s[1, 0, :50] = -rng.random(50).astype(np.float32)                   # negatives
    s[1, 0, 60] = np.inf
    s[1, 0, 61] = -np.inf
    s[1, 1] = np.float32(1e-42) * rng.integers(0, 5, T).astype(np.float32)   # denormals
    for pf, pl in ((1, 1), (0, 0), (3, 0)):
        np.testing.assert_array_equal(_gpu_select(s, n, pf, pl), oracle.select_anchors(s, n, pf, pl))


def _anchors(rng, B, G, T, n):
    return np.stack([np.stack([np.sort(rng.choice(T, n, replace=False)) for _ in range(G)])
                     for _ in range(B)]).astype(np.int32)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)])
@pytest.mark.parametrize("B,H,Gmode,T,n,cap", [
    (1, 2, "layer", 9, 3, 5), (2, 3, "head", 100, 17, 17), (1, 4, "layer", 256, 128, 145),
    (2, 2, "head", 1000, 100, 130), (1, 2, "layer", 1030, 515, 600), (1, 1, "layer", 700, 1, 4),
])
def test_merge_compact_parity(dtype, D, B, H, Gmode, T, n, cap):
    rng = np.random.default_rng(T * 13 + n + D)
    G = 1 if Gmode == "layer" else H
    k = quantize(rng.standard_normal((B, H, T, D)) * 2, dtype)
    v = quantize(rng.standard_normal((B, H, T, D)), dtype)
    k[:, :, 0] = quantize(k[:, :, 0] * 8, dtype)
    a = _anchors(rng, B, G, T, n)
    assign, counts = oracle.assign_nearest(a, T)
    ok, ov = oracle.merge_compact(k, assign, n, cap), oracle.merge_compact(v, assign, n, cap)

    dk_c = torch.full((B, H, cap, D), 9.0, dtype=torch_dtype(dtype), device="cuda")
    dv_c = torch.full((B, H, cap, D), 9.0, dtype=torch_dtype(dtype), device="cuda")
    d_counts = torch.full((B, G, n), -1, dtype=torch.int32, device="cuda")
    d_assign = torch.full((B, G, T), -1, dtype=torch.int32, device="cuda")
    d_pos = torch.full((B, G, cap), -5, dtype=torch.int32, device="cuda")
    ec.ec_merge_compact(to_dev(k, dtype), to_dev(v, dtype), torch.from_numpy(a).cuda(), dk_c, dv_c, d_counts, d_assign, d_pos)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(d_counts.cpu().numpy(), counts)
    np.testing.assert_array_equal(d_assign.cpu().numpy(), assign)
    np.testing.assert_array_equal(d_pos.cpu().numpy()[:, :, :n], a)
    assert (d_pos.cpu().numpy()[:, :, n:] == -5).all()
    assert_close(to_host(dk_c)[:, :, :n], ok[:, :, :n], dtype, "k_cache", stored=True)
    assert_close(to_host(dv_c)[:, :, :n], ov[:, :, :n], dtype, "v_cache", stored=True)
    assert (to_host(dk_c)[:, :, n:] == 9.0).all() and (to_host(dv_c)[:, :, n:] == 9.0).all()
    # conservation of merged count weights (fp32 accumulate, so to rounding)
    assert int(d_counts.sum()) == B * G * T


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_merge_identity_is_a_bit_exact_copy(dtype, D):
    B, H, T = 2, 3, 130
    rng = np.random.default_rng(5)
    k, v = quantize(rng.standard_normal((B, H, T, D)), dtype), quantize(rng.standard_normal((B, H, T, D)), dtype)
    k[:, :, ::7, ::3] = -0.0        # signed zeros and infinities survive a copy too
    v[:, :, 5, :4] = np.inf
    a = np.tile(np.arange(T, dtype=np.int32), (B, 1, 1))
    dk, dv = to_dev(k, dtype), to_dev(v, dtype)
    dk_c, dv_c = torch.zeros_like(dk), torch.zeros_like(dv)
    ec.ec_merge_compact(dk, dv, torch.from_numpy(a).cuda(), dk_c, dv_c)
    torch.cuda.synchronize()
    assert torch.equal(dk.view(torch.int16 if dtype == 'bf16' else torch.int32), dk_c.view(torch.int16 if dtype == 'bf16' else torch.int32))
    assert torch.equal(dv.view(torch.int16 if dtype == 'bf16' else torch.int32), dv_c.view(torch.int16 if dtype == 'bf16' else torch.int32))


def test_merge_optional_outputs_may_be_null_and_batches_are_independent():
    B, H, T, D, n, dtype = 3, 2, 200, 128, 40, "bf16"
    rng = np.random.default_rng(9)
    k, v = quantize(rng.standard_normal((B, H, T, D)), dtype), quantize(rng.standard_normal((B, H, T, D)), dtype)
    a = _anchors(rng, B, 1, T, n)
    full_k = torch.zeros((B, H, n, D), dtype=torch.bfloat16, device="cuda")
    full_v = torch.zeros_like(full_k)
    ec.ec_merge_compact(to_dev(k, dtype), to_dev(v, dtype), torch.from_numpy(a).cuda(), full_k, full_v)
    for b in range(B):
        one_k = torch.zeros((1, H, n, D), dtype=torch.bfloat16, device="cuda")
        one_v = torch.zeros_like(one_k)
        ec.ec_merge_compact(to_dev(k[b:b + 1], dtype), to_dev(v[b:b + 1], dtype), torch.from_numpy(a[b:b + 1]).cuda(), one_k, one_v)
        torch.cuda.synchronize()
        assert torch.equal(one_k[0], full_k[b]) and torch.equal(one_v[0], full_v[b])


@pytest.mark.parametrize("dtype,D,Gmode", [("bf16", 128, "layer"), ("f32", 64, "head"), ("bf16", 64, "head")])
def test_evict_only_mode_copies_anchor_rows(dtype, D, Gmode):
    """Table 3b's eviction-only ablation: anchor rows bit for bit, counts 1, dropped positions -1."""
    B, H, T, n, cap = 2, 4, 333, 70, 80
    G = 1 if Gmode == "layer" else H
    rng = np.random.default_rng(D + n)
    k = quantize(rng.standard_normal((B, H, T, D)) * 3, dtype)
    v = quantize(rng.standard_normal((B, H, T, D)), dtype)
    a = _anchors(rng, B, G, T, n)
    dk_c = torch.full((B, H, cap, D), 9.0, dtype=torch_dtype(dtype), device="cuda")
    dv_c = torch.full((B, H, cap, D), 9.0, dtype=torch_dtype(dtype), device="cuda")
    d_counts = torch.full((B, G, n), -7, dtype=torch.int32, device="cuda")
    d_assign = torch.full((B, G, T), -7, dtype=torch.int32, device="cuda")
    d_pos = torch.full((B, G, cap), -7, dtype=torch.int32, device="cuda")
    ec.ec_merge_compact(to_dev(k, dtype), to_dev(v, dtype), torch.from_numpy(a).cuda(), dk_c, dv_c, d_counts, d_assign,
                        d_pos, merge_mode=ec.EC_MERGE_EVICT)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(dk_c)[:, :, :n], oracle.evict_compact(k, a))
    np.testing.assert_array_equal(to_host(dv_c)[:, :, :n], oracle.evict_compact(v, a))
    assert (to_host(dk_c)[:, :, n:] == 9.0).all()
    assert (d_counts.cpu().numpy() == 1).all()
    np.testing.assert_array_equal(d_pos.cpu().numpy()[:, :, :n], a)
    want_assign = np.full((B, G, T), -1, np.int32)
    for b in range(B):
        for g in range(G):
            want_assign[b, g, a[b, g]] = np.arange(n)
    np.testing.assert_array_equal(d_assign.cpu().numpy(), want_assign)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("f32", 128)])
@pytest.mark.parametrize("weighted", [False, True])
def test_merge_long_buckets_next_to_single_rows(dtype, D, weighted):
    """The shape importance scores produce: anchors packed at the start, then a few buckets of hundreds of rows
    (summed by the whole workgroup) between single-row ones, several of them in one workgroup's chunk."""
    B, H, T = 2, 3, 3000
    rng = np.random.default_rng(D + weighted)
    k = quantize(rng.standard_normal((B, H, T, D)) * 2, dtype)
    v = quantize(rng.standard_normal((B, H, T, D)), dtype)
    a0 = list(range(10)) + [400, 401, 900, 1500, 1501, 1502, 2200, 2998, 2999]
    a1 = [0, 129, 130, 700, 701, 702, 703, 1400, 2100, 2101, 2800, 2801, 2802, 2803, 2804, 2805, 2806, 2900, 2999]
    a = np.array([a0, a1], np.int32).reshape(B, 1, -1)
    n = a.shape[-1]
    assign, counts = oracle.assign_nearest(a, T)
    assert counts.max() > 500 and (counts == 1).any()
    w = rng.integers(1, 9, (B, 1, T)).astype(np.int32)
    if weighted:
        ok, wsum = oracle.merge_weighted(k, assign, w, n)
        ov, _ = oracle.merge_weighted(v, assign, w, n)
    else:
        ok, ov, wsum = oracle.merge_compact(k, assign, n), oracle.merge_compact(v, assign, n), counts
    dk_c = torch.zeros((B, H, n, D), dtype=torch_dtype(dtype), device="cuda")
    dv_c = torch.zeros_like(dk_c)
    d_counts = torch.full((B, 1, n), -1, dtype=torch.int32, device="cuda")
    d_assign = torch.full((B, 1, T), -1, dtype=torch.int32, device="cuda")
    d_pos = torch.full((B, 1, n), -1, dtype=torch.int32, device="cuda")
    ec.ec_remerge_compact(to_dev(k, dtype), to_dev(v, dtype), T, torch.from_numpy(a).cuda(), dk_c, dv_c,
                          weights=torch.from_numpy(w).cuda() if weighted else None, counts=d_counts, assign=d_assign, pos=d_pos)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(d_counts.cpu().numpy(), wsum)
    np.testing.assert_array_equal(d_assign.cpu().numpy(), assign)
    np.testing.assert_array_equal(d_pos.cpu().numpy(), a)
    assert_close(to_host(dk_c), ok, dtype, "k_cache", stored=True)
    assert_close(to_host(dv_c), ov, dtype, "v_cache", stored=True)
    # twice the same call gives the same bits (the long buckets' partial sums are combined in a fixed order)
    dk2, dv2 = torch.zeros_like(dk_c), torch.zeros_like(dv_c)
    ec.ec_remerge_compact(to_dev(k, dtype), to_dev(v, dtype), T, torch.from_numpy(a).cuda(), dk2, dv2,
                          weights=torch.from_numpy(w).cuda() if weighted else None)
    torch.cuda.synchronize()
    assert torch.equal(dk2, dk_c) and torch.equal(dv2, dv_c)
