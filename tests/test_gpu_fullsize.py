"""GPU parity at the full workload shapes, in the launch configuration bench.py times.

Inputs are drawn on the device with the workload recipe; the oracle sees host copies of the same
bits.  Where the fp64 brute force of a whole layer would take minutes, the oracle runs on sampled
batch elements (all heads of each, so the layer-wise head mean is complete) and the rest of the
output is checked through properties that hold at any size.
"""
import functools

import numpy as np
import pytest
import torch

import oracle
from paper_2407_18121_amd import binding as ec
from paper_2407_18121_amd import synthetic as syn
from paper_2407_18121_amd import synthetic_torch as synt
from util import assert_close, to_host

pytestmark = pytest.mark.gpu

# config -> batch elements the oracle recomputes
SAMPLES = {"C2": [0], "C3": [0, 5], "C4": [1], "C5": [11], "T1": [7], "T2": [3], "T3": [0], "T4": [40]}
ALL = ["C2", "C3", "C4", "C5", "T1", "T2", "T3", "T4"]  # T*: the shapes the paper timed (Table 2, budget 0.2)


def _host(t):
    return t.float().cpu().numpy()


def _assert_valid_selection(score, anchors, pf=1, pl=1):
    """The anchors are the protected ends plus the highest scores, equal scores going to the lower position
    (checked from the definition, on whatever fp32 scores the selection was given)."""
    B, G, T = score.shape
    for b in range(B):
        for g in range(G):
            s, a = score[b, g], anchors[b, g]
            sel = np.zeros(T, bool)
            sel[a] = True
            assert sel.sum() == a.size and sel[:pf].all() and sel[T - pl:].all()
            free = np.ones(T, bool)
            free[:pf] = False
            free[T - pl:] = False
            chosen, rest = free & sel, free & ~sel
            if not chosen.any() or not rest.any():
                continue
            thr = s[chosen].min()
            assert s[rest].max() <= thr
            tie_sel, tie_rest = np.flatnonzero(chosen & (s == thr)), np.flatnonzero(rest & (s == thr))
            if tie_rest.size:
                assert tie_sel.max() < tie_rest.min()


@pytest.mark.parametrize("name", ALL)
def test_prefill_chain_full_shape(name):
    cfg = syn.CONFIGS[name]
    B, H, T, D, nA, cap = cfg.B, cfg.H, cfg.T, cfg.D, cfg.n_anchor, cfg.cap
    q, k, v = synt.prompt_qkv_device(cfg, layer=3)
    dt = q.dtype
    out = torch.empty_like(q)
    lse = torch.empty((B, H, T), dtype=torch.float32, device="cuda")
    score = torch.empty((B, 1, T), dtype=torch.float32, device="cuda")
    ws = ec.new_workspace(ec.EC_FN_PREFILL_SCORE, B, H, T, D, ec.EC_BF16)
    ec.ec_prefill_score(q, k, v, out, lse, score, cfg.scale, ws)
    torch.cuda.synchronize()
    del ws
    sc = _host(score)
    # properties at any size: every row of A sums to one; the last key only sees its own query
    np.testing.assert_allclose(sc.sum(-1), T, rtol=2e-5)
    assert (sc[..., -1] <= 1.0 + 1e-5).all() and (sc[..., 0] >= 1.0).all() and np.isfinite(sc).all()

    for b in SAMPLES[name]:
        qb, kb, vb = (_host(x[b:b + 1]) for x in (q, k, v))
        ref = oracle.prefill_score(qb, kb, vb, cfg.scale, 1)
        assert_close(to_host(out[b:b + 1]), ref["out"], cfg.dtype, f"out[{b}]")
        assert_close(to_host(lse[b:b + 1]), ref["lse"], cfg.dtype, f"lse[{b}]")
        assert_close(sc[b:b + 1], ref["score"], cfg.dtype, f"score[{b}]")

        # later stages are fed the oracle's own fp32 scores: indices must then be bit-exact
        sc32 = ref["score"].astype(np.float32)
        a_ref = oracle.select_anchors(sc32, nA, 1, 1)
        a_gpu = torch.empty((1, 1, nA), dtype=torch.int32, device="cuda")
        ec.ec_select_anchors(torch.from_numpy(sc32).cuda(), nA, 1, 1, a_gpu)
        np.testing.assert_array_equal(a_gpu.cpu().numpy(), a_ref)
        assign, counts = oracle.assign_nearest(a_ref, T)
        kc = torch.zeros((1, H, cap, D), dtype=dt, device="cuda")
        vc = torch.zeros_like(kc)
        d_counts = torch.empty((1, 1, nA), dtype=torch.int32, device="cuda")
        d_assign = torch.empty((1, 1, T), dtype=torch.int32, device="cuda")
        d_pos = torch.zeros((1, 1, cap), dtype=torch.int32, device="cuda")
        ec.ec_merge_compact(k[b:b + 1].contiguous(), v[b:b + 1].contiguous(), a_gpu, kc, vc, d_counts, d_assign, d_pos)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_counts.cpu().numpy(), counts)
        np.testing.assert_array_equal(d_assign.cpu().numpy(), assign)
        np.testing.assert_array_equal(d_pos.cpu().numpy()[..., :nA], a_ref)
        assert_close(to_host(kc)[:, :, :nA], oracle.merge_compact(kb, assign, nA), cfg.dtype, "k_cache", stored=True)
        assert_close(to_host(vc)[:, :, :nA], oracle.merge_compact(vb, assign, nA), cfg.dtype, "v_cache", stored=True)

    # the whole batch through select + merge on the GPU's own scores: structural checks at full size
    anchors = torch.empty((B, 1, nA), dtype=torch.int32, device="cuda")
    ec.ec_select_anchors(score, nA, 1, 1, anchors)
    kc = torch.zeros((B, H, cap, D), dtype=dt, device="cuda")
    vc = torch.zeros_like(kc)
    counts = torch.empty((B, 1, nA), dtype=torch.int32, device="cuda")
    ec.ec_merge_compact(k, v, anchors, kc, vc, counts, None, None)
    torch.cuda.synchronize()
    a = anchors.cpu().numpy()
    assert (np.diff(a, axis=-1) > 0).all() and (a[..., 0] == 0).all() and (a[..., -1] == T - 1).all()
    _assert_valid_selection(sc, a)
    cn = counts.cpu().numpy()
    assert (cn.sum(-1) == T).all() and (cn >= 1).all()                        # merged count weights are conserved
    # first moment per head: sum_k count_k * KV_k = sum_t kv_t, up to the bf16 rounding of the stored rows
    for b in SAMPLES[name]:
        w = torch.from_numpy(cn[b, 0]).cuda().float()[None, :, None]
        lhs = (vc[b, :, :nA].float() * w).sum(1)
        rhs = v[b].float().sum(1)
        assert (lhs - rhs).abs().max().item() <= 2.0 ** -8 * float((v[b].float().abs()).sum(1).max()) + 1e-2


@functools.lru_cache(maxsize=None)
def _oracle_merged_cache(name, b):
    """The oracle's own compressed cache of batch element b of the workload's prompt (layer 3): scores, anchors,
    buckets and bucket means, all in fp64 from host copies of the prompt bits.  Returns (anchors, K rows, V rows)."""
    cfg = syn.CONFIGS[name]
    q, k, v = synt.prompt_qkv_device(cfg, layer=3)
    qb, kb, vb = (_host(x[b:b + 1]) for x in (q, k, v))
    del q, k, v
    ref = oracle.prefill_score(qb, kb, vb, cfg.scale, 1, want_out=False)
    a = oracle.select_anchors(ref["score"].astype(np.float32), cfg.n_anchor, 1, 1)
    assign, _ = oracle.assign_nearest(a, cfg.T)
    return a, oracle.merge_compact(kb, assign, cfg.n_anchor), oracle.merge_compact(vb, assign, cfg.n_anchor)


@pytest.mark.parametrize("name", ALL)
def test_decode_full_shape(name):
    """Every generated token of the workload (Alg. 1's last branch over the whole schedule) on one layer, in the
    launch configuration the benchmark times (workspace given: the library picks its launch shape).  The sampled
    batch elements start from the ORACLE's compressed prompt cache, rounded to the storage type on both sides,
    and are compared with the oracle at every step; the other batch elements start from random rows."""
    cfg = syn.CONFIGS[name]
    B, H, D, cap, nA = cfg.B, cfg.H, cfg.D, cfg.cap, cfg.n_anchor
    dt = synt.torch_dtype(cfg)
    g = torch.Generator(device="cuda").manual_seed(1234 + cfg.cid)
    kc = (torch.randn((B, H, cap, D), generator=g, device="cuda") * 1.5).to(dt)
    vc = torch.randn((B, H, cap, D), generator=g, device="cuda").to(dt)
    kc[:, :, 0] *= 8
    pos = (torch.arange(cap, device="cuda", dtype=torch.int32) * 2).repeat(B, 1, 1).contiguous()
    samples = SAMPLES[name]
    for b in samples:
        a, mk, mv = _oracle_merged_cache(name, b)
        kc[b, :, :nA] = torch.from_numpy(mk[0]).to(device="cuda", dtype=dt)
        vc[b, :, :nA] = torch.from_numpy(mv[0]).to(device="cuda", dtype=dt)
        pos[b, 0, :nA] = torch.from_numpy(a[0, 0]).cuda()
    dq, dk, dv = synt.decode_stream_device(cfg, layer=1)
    out = torch.empty((B, H, D), dtype=dt, device="cuda")
    ws = ec.new_workspace(ec.EC_FN_DECODE_STEP, B, H, cap, D, ec.dtype_code(kc))
    p, qd = cfg.gamma
    okc, ovc = (to_host(x[samples]).copy() for x in (kc, vc))   # the same bits, widened exactly
    opos = pos[samples].cpu().numpy().copy()
    hq, hk, hv = (_host(x[:, samples]) for x in (dq, dk, dv))
    N = nA
    worst = 0.0
    for step in range(cfg.decode_steps):
        n_seen = cfg.T + step + 1
        idx = ec.ec_evict_index(n_seen, N + 1, p, qd)
        ec.ec_decode_step(dq[step], dk[step], dv[step], kc, vc, pos, N, idx, n_seen - 1, cfg.scale, out, ws)
        o_ref, _ = oracle.decode_step(hq[step], hk[step], hv[step], okc, ovc, opos, N, idx, n_seen - 1, cfg.scale)
        got = to_host(out[samples])
        worst = max(worst, float(np.abs(got - o_ref).max()))
        assert_close(got, o_ref, cfg.dtype, f"out step {step}")
        N += 0 if idx >= 0 else 1
        assert N == -((-p * n_seen) // qd)                       # ceil(gamma * tokens seen) after every step
    torch.cuda.synchronize()
    assert N == -((-p * (cfg.T + cfg.decode_steps)) // qd) == cap - 1
    np.testing.assert_array_equal(to_host(kc[samples])[:, :, :N], okc[:, :, :N])
    np.testing.assert_array_equal(to_host(vc[samples])[:, :, :N], ovc[:, :, :N])
    np.testing.assert_array_equal(pos[samples].cpu().numpy()[:, :, :N], opos[:, :, :N])
    # every other batch element: finite outputs, positions strictly increasing
    assert torch.isfinite(out.float()).all()
    assert (pos[:, :, 1:N] > pos[:, :, :N - 1]).all()


def test_select_head_wise_full_shape():
    cfg = syn.CONFIGS["C5"]
    g = torch.Generator(device="cuda").manual_seed(5)
    score = torch.rand((cfg.B, cfg.H, cfg.T), generator=g, device="cuda") * 3
    score[..., 0] += 1000
    score = (score * 64).round() / 64          # plenty of exact ties
    idx = torch.empty((cfg.B, cfg.H, cfg.n_anchor), dtype=torch.int32, device="cuda")
    ec.ec_select_anchors(score, cfg.n_anchor, 1, 1, idx)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), oracle.select_anchors(score.cpu().numpy(), cfg.n_anchor, 1, 1))


@pytest.mark.parametrize("name", ["C2", "C3", "C5", "T4"])
def test_second_turn_full_shape(name):
    """A later chunk over the cache a finished generation leaves (multi-turn chat; Alg. 1's multi-token
    branch with a past), at the workload's shape: chunk scoring, selection and weighted re-merge."""
    cfg = syn.CONFIGS[name]
    B, H, D = cfg.B, cfg.H, cfg.D
    dt = synt.torch_dtype(cfg)
    p, qd = cfg.gamma
    P = cfg.n_anchor
    for step in range(cfg.decode_steps):
        P += 0 if ec.ec_evict_index(cfg.T + step + 1, P + 1, p, qd) >= 0 else 1
    Tq = min(cfg.T // 2, 2048)
    L, rows = P + Tq, P + Tq + 5
    n2 = -(-p * (cfg.T + cfg.decode_steps + Tq) // qd)
    g = torch.Generator(device="cuda").manual_seed(4321 + cfg.cid)
    k = (torch.randn((B, H, rows, D), generator=g, device="cuda") * 1.5).to(dt)
    v = torch.randn((B, H, rows, D), generator=g, device="cuda").to(dt)
    k[:, :, 0] *= 8
    k[:, :, L:] = float("nan")      # spare rows of the buffer are never read
    v[:, :, L:] = float("nan")
    q = torch.randn((B, H, Tq, D), generator=g, device="cuda").to(dt)
    out = torch.empty((B, H, Tq, D), dtype=dt, device="cuda")
    lse = torch.empty((B, H, Tq), dtype=torch.float32, device="cuda")
    score = torch.empty((B, 1, L), dtype=torch.float32, device="cuda")
    ws = ec.new_workspace(ec.EC_FN_PREFILL_SCORE, B, H, L, D, ec.EC_BF16)
    ec.ec_chunk_score(q, k, v, P, out, lse, score, cfg.scale, ws)
    torch.cuda.synchronize()
    del ws
    sc = _host(score)
    np.testing.assert_allclose(sc.sum(-1), Tq, rtol=2e-5)
    assert np.isfinite(sc).all() and (sc[..., -1] <= 1.0 + 1e-5).all()

    weights = torch.randint(1, 30, (B, 1, L), generator=g, device="cuda", dtype=torch.int32)
    weights[:, :, P:] = 1
    for b in SAMPLES[name]:
        qb, kb, vb = _host(q[b:b + 1]), _host(k[b:b + 1, :, :L]), _host(v[b:b + 1, :, :L])
        ref = oracle.chunk_score(qb, kb, vb, P, cfg.scale, 1)
        assert_close(to_host(out[b:b + 1]), ref["out"], cfg.dtype, f"out[{b}]")
        assert_close(to_host(lse[b:b + 1]), ref["lse"], cfg.dtype, f"lse[{b}]")
        assert_close(sc[b:b + 1], ref["score"], cfg.dtype, f"score[{b}]")
        sc32 = ref["score"].astype(np.float32)
        a_ref = oracle.select_anchors(sc32, n2, 1, 1)
        a_gpu = torch.empty((1, 1, n2), dtype=torch.int32, device="cuda")
        ec.ec_select_anchors(torch.from_numpy(sc32).cuda(), n2, 1, 1, a_gpu)
        np.testing.assert_array_equal(a_gpu.cpu().numpy(), a_ref)
        assign, _ = oracle.assign_nearest(a_ref, L)
        wb = weights[b:b + 1].cpu().numpy()
        ok, wsum = oracle.merge_weighted(kb, assign, wb, n2)
        ov, _ = oracle.merge_weighted(vb, assign, wb, n2)
        nk = torch.zeros((1, H, n2, D), dtype=dt, device="cuda")
        nv = torch.zeros_like(nk)
        d_counts = torch.empty((1, 1, n2), dtype=torch.int32, device="cuda")
        ec.ec_remerge_compact(k[b:b + 1].contiguous(), v[b:b + 1].contiguous(), L, a_gpu, nk, nv,
                              weights=weights[b:b + 1].contiguous(), counts=d_counts)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_counts.cpu().numpy(), wsum)
        assert_close(to_host(nk), ok, cfg.dtype, "k_cache", stored=True)
        assert_close(to_host(nv), ov, cfg.dtype, "v_cache", stored=True)

    # whole batch on the GPU's own scores: structure at full size
    anchors = torch.empty((B, 1, n2), dtype=torch.int32, device="cuda")
    ec.ec_select_anchors(score, n2, 1, 1, anchors)
    nk = torch.zeros((B, H, n2, D), dtype=dt, device="cuda")
    nv = torch.zeros_like(nk)
    counts = torch.empty((B, 1, n2), dtype=torch.int32, device="cuda")
    ec.ec_remerge_compact(k, v, L, anchors, nk, nv, weights=weights, counts=counts)
    torch.cuda.synchronize()
    a = anchors.cpu().numpy()
    assert (np.diff(a, axis=-1) > 0).all() and (a[..., 0] == 0).all() and (a[..., -1] == L - 1).all()
    _assert_valid_selection(sc, a)
    np.testing.assert_array_equal(counts.cpu().numpy().sum(-1), weights.cpu().numpy().sum(-1))
    assert torch.isfinite(nk.float()).all() and torch.isfinite(nv.float()).all()


def test_long_prompt_beyond_the_workloads():
    """A prompt 2.4x the longest workload, of a length no tile size divides: the select kernel's keys no
    longer fit in LDS, the key-tile loops run 300+ iterations, and a cache of 30000 rows is decoded."""
    B, H, D, T, dtype = 1, 2, 128, 20011, "bf16"
    cfg = syn.custom("long", H=H, D=D, B=B, T=T, dtype=dtype, gamma=(1, 10), cid=4242)
    q, k, v = synt.prompt_qkv_device(cfg, layer=0)
    out = torch.empty_like(q)
    lse = torch.empty((B, H, T), dtype=torch.float32, device="cuda")
    score = torch.empty((B, 1, T), dtype=torch.float32, device="cuda")
    ws = ec.new_workspace(ec.EC_FN_PREFILL_SCORE, B, H, T, D, ec.EC_BF16)
    ec.ec_prefill_score(q, k, v, out, lse, score, cfg.scale, ws)
    torch.cuda.synchronize()
    ref = oracle.prefill_score(_host(q), _host(k), _host(v), cfg.scale, 1)
    assert_close(to_host(out), ref["out"], dtype, "out")
    assert_close(to_host(lse), ref["lse"], dtype, "lse")
    assert_close(_host(score), ref["score"], dtype, "score")
    nA = -(-T // 10)
    sc32 = ref["score"].astype(np.float32)
    a_ref = oracle.select_anchors(sc32, nA, 1, 1)
    a_gpu = torch.empty((B, 1, nA), dtype=torch.int32, device="cuda")
    ec.ec_select_anchors(torch.from_numpy(sc32).cuda(), nA, 1, 1, a_gpu)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(a_gpu.cpu().numpy(), a_ref)
    assign, counts = oracle.assign_nearest(a_ref, T)
    kc = torch.zeros((B, H, nA, D), dtype=q.dtype, device="cuda")
    vc = torch.zeros_like(kc)
    d_counts = torch.empty((B, 1, nA), dtype=torch.int32, device="cuda")
    ec.ec_merge_compact(k, v, a_gpu, kc, vc, d_counts)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(d_counts.cpu().numpy(), counts)
    assert_close(to_host(kc), oracle.merge_compact(_host(k), assign, nA), dtype, "k_cache", stored=True)
    assert_close(to_host(vc), oracle.merge_compact(_host(v), assign, nA), dtype, "v_cache", stored=True)

    # decode over a 30000-row cache with a victim deep inside it
    N, cap = 30000, 30002
    g = torch.Generator(device="cuda").manual_seed(99)
    kc = (torch.randn((B, H, cap, D), generator=g, device="cuda") * 1.5).to(torch.bfloat16)
    vc = torch.randn((B, H, cap, D), generator=g, device="cuda").to(torch.bfloat16)
    pos = torch.arange(cap, dtype=torch.int32, device="cuda").repeat(B, 1, 1).contiguous()
    dq, dk, dv = (torch.randn((B, H, D), generator=g, device="cuda").to(torch.bfloat16) for _ in range(3))
    okc, ovc, opos = to_host(kc), to_host(vc), pos.cpu().numpy().copy()
    dout = torch.empty((B, H, D), dtype=torch.bfloat16, device="cuda")
    ec.ec_decode_step(dq, dk, dv, kc, vc, pos, N, 12345, 777777, cfg.scale, dout, None)
    torch.cuda.synchronize()
    o_ref, _ = oracle.decode_step(_host(dq), _host(dk), _host(dv), okc, ovc, opos, N, 12345, 777777, cfg.scale)
    assert_close(to_host(dout), o_ref, dtype, "decode out")
    np.testing.assert_array_equal(to_host(kc)[:, :, :N], okc[:, :, :N])
    np.testing.assert_array_equal(to_host(vc)[:, :, :N], ovc[:, :, :N])
    np.testing.assert_array_equal(pos.cpu().numpy()[:, :, :N], opos[:, :, :N])
