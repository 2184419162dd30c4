"""GPU parity of the ragged-batch entry points: every batch element must equal the oracle run on that element
alone with its own length (Alg. 1 treats one sequence; a batch is independent sequences)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_18121_amd import binding as ec
from paper_2407_18121_amd import synthetic as syn
from util import assert_close, quantize, to_dev, to_host, torch_dtype

pytestmark = pytest.mark.gpu


def _i32(a):
    return torch.tensor(a, dtype=torch.int32, device="cuda")


def _nan_pad(x, lens, dtype):
    """Device copy of [B,H,T,D] whose rows at or beyond each sequence's length are NaN (never to be read)."""
    t = to_dev(x, dtype)
    for b, n in enumerate(lens):
        t[b, :, n:] = float("nan")
    return t


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("bf16", 64)])
@pytest.mark.parametrize("H,Gmode,lens", [
    (2, "layer", [300, 37, 129, 1]),
    (3, "head", [64, 200, 65]),
    (2, "layer", [5, 0, 130]),          # an empty sequence in the batch
    (2, "layer", [700, 256]),
])
def test_prefill_chain_ragged(dtype, D, H, Gmode, lens):
    B, T = len(lens), max(lens)
    G = 1 if Gmode == "layer" else H
    cfg = syn.custom("t", H=H, D=D, B=B, T=T, dtype=dtype, cid=3000 + T + B)
    q, k, v = syn.prompt_qkv(cfg)
    n_b = [-(-n // 4) for n in lens]
    n_max, cap = max(n_b), max(n_b) + 3
    dq, dk, dv = (_nan_pad(x, lens, dtype) for x in (q, k, v))
    out = torch.full((B, H, T, D), 5.0, dtype=torch_dtype(dtype), device="cuda")
    lse = torch.full((B, H, T), 5.0, dtype=torch.float32, device="cuda")
    score = torch.full((B, G, T), 5.0, dtype=torch.float32, device="cuda")
    ws = ec.new_workspace(ec.EC_FN_PREFILL_SCORE, B, H, T, D, ec.dtype_code(dq))
    ec.ec_prefill_score_varlen(dq, dk, dv, out, lse, score, _i32(lens), cfg.scale, ws)
    torch.cuda.synchronize()

    # stage-fed: the oracle's fp32 scores of every sequence, padded, go into selection; its anchors into merge
    sc_pad = np.full((B, G, T), np.nan, np.float32)
    a_pad = np.zeros((B, G, n_max), np.int32)
    refs = []
    for b, n in enumerate(lens):
        if n == 0:
            refs.append(None)
            continue
        r = oracle.prefill_score(q[b:b + 1, :, :n], k[b:b + 1, :, :n], v[b:b + 1, :, :n], cfg.scale, G)
        assert_close(to_host(out[b:b + 1, :, :n]), r["out"], dtype, f"out[{b}]")
        assert_close(to_host(lse[b:b + 1, :, :n]), r["lse"], dtype, f"lse[{b}]")
        assert_close(to_host(score[b:b + 1, :, :n]), r["score"], dtype, f"score[{b}]")
        sc_pad[b, :, :n] = r["score"][0].astype(np.float32)
        pf = min(1, n_b[b]); pl = min(1, n_b[b] - pf)
        a_pad[b, :, :n_b[b]] = oracle.select_anchors(sc_pad[b:b + 1, :, :n].copy(), n_b[b], pf, pl)[0]
        refs.append(r)
    idx = torch.full((B, G, n_max), -9, dtype=torch.int32, device="cuda")
    ec.ec_select_anchors_varlen(torch.from_numpy(sc_pad).cuda(), _i32(lens), _i32(n_b), 1, 1, idx)
    torch.cuda.synchronize()
    got = idx.cpu().numpy()
    for b in range(B):
        np.testing.assert_array_equal(got[b, :, :n_b[b]], a_pad[b, :, :n_b[b]])
        assert (got[b, :, n_b[b]:] == -9).all()

    kc = torch.full((B, H, cap, D), 9.0, dtype=torch_dtype(dtype), device="cuda")
    vc = torch.full((B, H, cap, D), 9.0, dtype=torch_dtype(dtype), device="cuda")
    counts = torch.full((B, G, n_max), -1, dtype=torch.int32, device="cuda")
    assign = torch.full((B, G, T), -1, dtype=torch.int32, device="cuda")
    pos = torch.full((B, G, cap), -5, dtype=torch.int32, device="cuda")
    ec.ec_merge_compact_varlen(dk, dv, torch.from_numpy(a_pad).cuda(), _i32(lens), _i32(n_b), kc, vc, counts, assign, pos)
    torch.cuda.synchronize()
    for b, n in enumerate(lens):
        nb = n_b[b]
        if n == 0:
            assert (to_host(kc[b]) == 9.0).all() and (counts[b] == -1).all() and (assign[b] == -1).all()
            continue
        a = a_pad[b:b + 1, :, :nb]
        asg, cnt = oracle.assign_nearest(a, n)
        np.testing.assert_array_equal(counts[b:b + 1, :, :nb].cpu().numpy(), cnt)
        np.testing.assert_array_equal(assign[b:b + 1, :, :n].cpu().numpy(), asg)
        np.testing.assert_array_equal(pos[b:b + 1, :, :nb].cpu().numpy(), a)
        assert_close(to_host(kc[b:b + 1, :, :nb]), oracle.merge_compact(k[b:b + 1, :, :n], asg, nb), dtype, f"k_cache[{b}]", stored=True)
        assert_close(to_host(vc[b:b + 1, :, :nb]), oracle.merge_compact(v[b:b + 1, :, :n], asg, nb), dtype, f"v_cache[{b}]", stored=True)
        assert (to_host(kc[b, :, nb:]) == 9.0).all() and (assign[b, :, n:] == -1).all() and (pos[b, :, nb:] == -5).all()


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
@pytest.mark.parametrize("H,G,cap,lens,victims", [
    (2, 1, 40, [5, 0, 39, 17], [-1, 0, 14, 17]),          # append, drop the only row, shift, drop the new row
    (3, 3, 700, [655, 300, 64], [0, 275, -1]),
    (2, 1, 1100, [1029, 1099, 96, 500], [600, 1074, 71, -1]),
])
def test_decode_step_ragged(dtype, D, H, G, cap, lens, victims):
    B = len(lens)
    rng = np.random.default_rng(cap + B + D)
    scale = 1.0 / np.sqrt(D)
    kc = quantize(rng.standard_normal((B, H, cap, D)) * 1.5, dtype)
    vc = quantize(rng.standard_normal((B, H, cap, D)), dtype)
    kc[:, :, 0] = quantize(kc[:, :, 0] * 6, dtype)
    q, kn, vn = (quantize(rng.standard_normal((B, H, D)), dtype) for _ in range(3))
    pos = np.tile(np.arange(cap, dtype=np.int32) * 3 + 1, (B, G, 1))
    new_pos = [4000 + b for b in range(B)]
    dkc, dvc, dpos = to_dev(kc, dtype), to_dev(vc, dtype), torch.from_numpy(pos).cuda()
    for b, n in enumerate(lens):                      # rows beyond a sequence's cache are never read
        dkc[b, :, n:] = float("nan")
        dvc[b, :, n:] = float("nan")
    dout = torch.full((B, H, D), float("nan"), dtype=torch_dtype(dtype), device="cuda")
    ec.ec_decode_step_varlen(to_dev(q, dtype), to_dev(kn, dtype), to_dev(vn, dtype), dkc, dvc, dpos, _i32(lens),
                             _i32(victims), _i32(new_pos), scale, dout)
    torch.cuda.synchronize()
    for b, (n, vic) in enumerate(zip(lens, victims)):
        okc, ovc, opos = kc[b:b + 1].astype(np.float64), vc[b:b + 1].astype(np.float64), pos[b:b + 1].copy()
        oout, _ = oracle.decode_step(q[b:b + 1], kn[b:b + 1], vn[b:b + 1], okc, ovc, opos, n, vic, new_pos[b], scale)
        assert_close(to_host(dout[b:b + 1]), oout, dtype, f"out[{b}]")
        m = n + (0 if vic >= 0 else 1)
        np.testing.assert_array_equal(to_host(dkc[b:b + 1, :, :m]), okc[:, :, :m])
        np.testing.assert_array_equal(to_host(dvc[b:b + 1, :, :m]), ovc[:, :, :m])
        np.testing.assert_array_equal(dpos[b:b + 1, :, :m].cpu().numpy(), opos[:, :, :m])
        assert torch.isnan(dkc[b, :, n + 1:].float()).all()          # nothing beyond the appended row is touched


def test_ragged_with_equal_lengths_is_the_dense_call():
    dtype, B, H, D, T = "bf16", 3, 2, 128, 200
    cfg = syn.custom("t", H=H, D=D, B=B, T=T, dtype=dtype, cid=3100)
    q, k, v = (to_dev(x, dtype) for x in syn.prompt_qkv(cfg))
    ws = ec.new_workspace(ec.EC_FN_PREFILL_SCORE, B, H, T, D, ec.EC_BF16)
    res = []
    for ragged in (False, True):
        out = torch.zeros((B, H, T, D), dtype=torch.bfloat16, device="cuda")
        score = torch.zeros((B, 1, T), dtype=torch.float32, device="cuda")
        idx = torch.zeros((B, 1, 50), dtype=torch.int32, device="cuda")
        kc, vc = torch.zeros((B, H, 50, D), dtype=torch.bfloat16, device="cuda"), torch.zeros((B, H, 50, D), dtype=torch.bfloat16, device="cuda")
        if ragged:
            L, N = _i32([T] * B), _i32([50] * B)
            ec.ec_prefill_score_varlen(q, k, v, out, None, score, L, cfg.scale, ws)
            ec.ec_select_anchors_varlen(score, L, N, 1, 1, idx)
            ec.ec_merge_compact_varlen(k, v, idx, L, N, kc, vc)
        else:
            ec.ec_prefill_score(q, k, v, out, None, score, cfg.scale, ws)
            ec.ec_select_anchors(score, 50, 1, 1, idx)
            ec.ec_merge_compact(k, v, idx, kc, vc)
        torch.cuda.synchronize()
        res.append((out, score, idx, kc, vc))
    for a, b in zip(*res):
        assert torch.equal(a, b)


@pytest.mark.parametrize("budget_mode,trunc_mode", [(0, 0), (1, 0), (0, 1), (1, 1)])
def test_retention_step_on_the_device_matches_the_oracle(budget_mode, trunc_mode):
    """ec_retention_step_varlen = the oracle's retention test for every sequence, step after step (bit-exact)."""
    prompts = [1, 7, 60, 160, 300, 481, 1000, 5000, 26, 27]
    B = len(prompts)
    p, q = 3, 7
    lens = [max(1, -(-p * t // q)) for t in prompts]
    kw = dict(budget_mode=budget_mode, fixed_len=40, trunc_mode=trunc_mode, recent=25, n_tl=9, protect_first=1)
    n_seen, length = _i32(prompts), _i32(lens)
    evict, new_pos, pending = (torch.zeros(B, dtype=torch.int32, device="cuda") for _ in range(3))
    o_seen, o_len = list(prompts), list(lens)
    for step in range(80):
        ec.ec_retention_step_varlen(n_seen, length, evict, new_pos, pending, p, q, **kw)
        o_seen = [n + 1 for n in o_seen]
        o_vic = [oracle.evict_index(o_seen[b], o_len[b] + 1, p, q, **kw) for b in range(B)]
        torch.cuda.synchronize()
        assert n_seen.cpu().tolist() == o_seen and evict.cpu().tolist() == o_vic, step
        assert length.cpu().tolist() == o_len and new_pos.cpu().tolist() == [n - 1 for n in o_seen], step
        o_len = [n + (0 if v >= 0 else 1) for n, v in zip(o_len, o_vic)]
    ec.ec_retention_step_varlen(n_seen, length, evict, new_pos, pending, p, q, flush_only=True, **kw)
    torch.cuda.synchronize()
    assert length.cpu().tolist() == o_len and n_seen.cpu().tolist() == o_seen and pending.cpu().tolist() == [0] * B
