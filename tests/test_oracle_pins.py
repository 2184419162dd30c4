"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the GPU library.  Each test names the passage it checks
(Sec. 3.3 Eq. 1-3, Alg. 1, Sec. 4.1).  Library routines (torch SDPA / softmax /
logsumexp, numpy lexsort / reduceat / delete) and closed forms are the
independent side of every comparison.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


# ----------------------------------------------------------------- scores (Eq. 1, I_n)
def test_score_golden_two_tokens():
    rows = {}
    for line in open(os.path.join(GOLD, "two_token_attention.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        rows[key] = np.array([float(x) for x in vals])
    q = rows["q"].reshape(1, 1, 2, 1)
    k = np.log(rows["k_is_ln"]).reshape(1, 1, 2, 1)
    v = rows["v"].reshape(1, 1, 2, 1)
    r = oracle.prefill_score(q, k, v, 1.0, 1, want_attn=True)
    np.testing.assert_allclose(r["attn"].reshape(-1), rows["A"], atol=1e-14)
    np.testing.assert_allclose(r["score"].reshape(-1), rows["I"], atol=1e-14)
    np.testing.assert_allclose(r["out"].reshape(-1), rows["out"], atol=1e-14)
    np.testing.assert_allclose(r["lse"].reshape(-1), np.log(rows["lse_is_ln"]), atol=1e-13)


@pytest.mark.parametrize("B,H,T,D,scale", [(2, 3, 17, 5, 0.37), (1, 2, 33, 8, 1.0)])
def test_score_against_library_attention(B, H, T, D, scale):
    q, k, v = _rand((B, H, T, D), 1), _rand((B, H, T, D), 2, 1.5), _rand((B, H, T, D), 3)
    r = oracle.prefill_score(q, k, v, scale, H, want_attn=True)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    ref_out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    np.testing.assert_allclose(r["out"], ref_out.numpy(), atol=1e-12)
    s = scale * torch.einsum("bhmd,bhnd->bhmn", tq, tk)
    s = s.masked_fill(~torch.tril(torch.ones(T, T, dtype=torch.bool)), float("-inf"))
    np.testing.assert_allclose(r["lse"], torch.logsumexp(s, -1).numpy(), atol=1e-12)
    A = torch.softmax(s, -1)
    np.testing.assert_allclose(r["attn"], A.numpy(), atol=1e-13)
    np.testing.assert_allclose(r["score"], A.sum(-2).numpy(), atol=1e-12)  # sum over queries m
    # layer-wise importance = mean over heads
    r1 = oracle.prefill_score(q, k, v, scale, 1)
    np.testing.assert_allclose(r1["score"][:, 0], A.sum(-2).mean(1).numpy(), atol=1e-12)


def test_score_closed_form_zero_queries():
    # q = 0 -> A_mn = 1/(m+1) -> I_n = sum_{m=n}^{T-1} 1/(m+1) = H_T - H_n (harmonic numbers)
    T, D, H = 40, 4, 2
    q = np.zeros((1, H, T, D))
    k, v = _rand((1, H, T, D), 4), _rand((1, H, T, D), 5)
    r = oracle.prefill_score(q, k, v, 0.5, 1)
    harm = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, T + 1))])
    np.testing.assert_allclose(r["score"][0, 0], harm[T] - harm[:T], atol=1e-13)
    # out_m = running mean of v
    run_mean = np.cumsum(v, axis=2) / np.arange(1, T + 1)[None, None, :, None]
    np.testing.assert_allclose(r["out"], run_mean, atol=1e-13)


def test_score_invariants():
    B, H, T, D = 2, 4, 64, 16
    q, k, v = _rand((B, H, T, D), 6), _rand((B, H, T, D), 7, 2.0), _rand((B, H, T, D), 8)
    rh = oracle.prefill_score(q, k, v, 0.25, H)
    # every row of A sums to 1 -> total mass = T; last column only sees its own query; column 0 >= 1
    np.testing.assert_allclose(rh["score"].sum(-1), T, rtol=1e-12)
    assert (rh["score"][..., -1] <= 1.0).all() and (rh["score"][..., 0] >= 1.0).all()
    assert (rh["score"] > 0).all()
    # permuting heads leaves the layer-wise score unchanged; batch elements are independent
    r1 = oracle.prefill_score(q, k, v, 0.25, 1)
    perm = [2, 0, 3, 1]
    r1p = oracle.prefill_score(q[:, perm], k[:, perm], v[:, perm], 0.25, 1)
    np.testing.assert_allclose(r1["score"], r1p["score"], atol=1e-13)
    r_b1 = oracle.prefill_score(q[1:], k[1:], v[1:], 0.25, 1)
    np.testing.assert_array_equal(r1["score"][1:], r_b1["score"])
    # T = 1
    r = oracle.prefill_score(q[:, :, :1], k[:, :, :1], v[:, :, :1], 0.25, 1)
    np.testing.assert_allclose(r["score"], 1.0)
    np.testing.assert_allclose(r["out"], v[:, :, :1])


# ----------------------------------------------------------------- selection
def _select_by_lexsort(s, n_anchor, pf, pl):
    T = s.shape[0]
    prot = [t for t in range(T) if t < pf or t >= T - pl]
    free = np.array([t for t in range(T) if not (t < pf or t >= T - pl)], dtype=np.int64)
    order = np.lexsort((free, -s[free].astype(np.float64)))  # primary: score desc, secondary: index asc
    pick = free[order[: n_anchor - len(prot)]]
    return np.sort(np.concatenate([np.array(prot, dtype=np.int64), pick])).astype(np.int32)


@pytest.mark.parametrize("T,n,pf,pl", [(37, 10, 1, 1), (64, 32, 0, 0), (50, 50, 1, 1), (9, 2, 1, 1),
                                         (20, 7, 3, 2), (16, 1, 0, 0), (16, 1, 1, 0)])
def test_select_against_lexsort(T, n, pf, pl):
    rng = np.random.default_rng(T * 100 + n)
    s = rng.random((3, 2, T)).astype(np.float32)
    s[0, 0] = np.round(s[0, 0] * 4) / 4  # many ties
    s[1, 1, ::3] = s[1, 1, 1]
    idx = oracle.select_anchors(s, n, pf, pl)
    for b in range(3):
        for g in range(2):
            np.testing.assert_array_equal(idx[b, g], _select_by_lexsort(s[b, g], n, pf, pl))


def test_select_invariants_and_special_values():
    T, n = 41, 13
    s = np.random.default_rng(5).random((1, 1, T)).astype(np.float32)
    idx = oracle.select_anchors(s, n, 1, 1)[0, 0]
    assert len(idx) == n and (np.diff(idx) > 0).all() and idx[0] == 0 and idx[-1] == T - 1
    unsel = np.setdiff1d(np.arange(T), idx)
    assert s[0, 0, unsel].max() <= s[0, 0, idx[1:-1]].min()
    # all-equal scores -> protected plus the lowest indices
    idx = oracle.select_anchors(np.ones((1, 1, T), np.float32), n, 1, 1)[0, 0]
    np.testing.assert_array_equal(idx, list(range(n - 1)) + [T - 1])
    # -0 == +0 (tie to lower index), +inf tops everything, negatives order correctly
    s = np.array([[[0.0, -0.0, 0.0, -1.0, np.inf, -np.inf, -0.0, 2.0]]], np.float32)
    np.testing.assert_array_equal(oracle.select_anchors(s, 4, 0, 0)[0, 0], [0, 1, 4, 7])
    np.testing.assert_array_equal(oracle.select_anchors(s, 7, 0, 0)[0, 0], [0, 1, 2, 3, 4, 6, 7])


# ----------------------------------------------------------------- buckets (Eq. 2 / Nearest)
def test_buckets_golden():
    for line in open(os.path.join(GOLD, "buckets_small.txt")):
        if line.startswith("#") or not line.strip():
            continue
        T, anchors, bounds = [p.strip() for p in line.split(";")]
        T = int(T)
        a = np.array([[[int(x) for x in anchors.split()]]], np.int32)
        want = [tuple(int(y) for y in x.split("-")) for x in bounds.split()]
        lo, hi = oracle.bucket_bounds(a, T)
        assert list(zip(lo[0, 0], hi[0, 0])) == want
        assign, counts = oracle.assign_nearest(a, T)
        for j, (l, h) in enumerate(want):
            assert (assign[0, 0, l:h + 1] == j).all()
            assert counts[0, 0, j] == h - l + 1


def test_bucket_definitions_coincide_and_partition():
    rng = np.random.default_rng(11)
    for T in (1, 2, 3, 17, 64, 255):
        for n in sorted({1, 2, max(1, T // 3), T}):
            if n > T:
                continue
            a = np.sort(rng.choice(T, size=n, replace=False)).astype(np.int32)[None, None]
            assign, counts = oracle.assign_nearest(a, T)
            lo, hi = oracle.bucket_bounds(a, T)
            assert lo[0, 0, 0] == 0 and hi[0, 0, -1] == T - 1
            assert (lo[0, 0, 1:] == hi[0, 0, :-1] + 1).all()          # contiguous partition
            assert ((lo[0, 0] <= a[0, 0]) & (a[0, 0] <= hi[0, 0])).all()  # anchor inside its bucket
            np.testing.assert_array_equal(counts[0, 0], hi[0, 0] - lo[0, 0] + 1)
            assert counts.sum() == T
            np.testing.assert_array_equal(assign[0, 0], np.repeat(np.arange(n), counts[0, 0]))


# ----------------------------------------------------------------- merge (Eq. 3)
def test_merge_against_reduceat_and_conservation():
    B, H, T, D, n = 2, 3, 50, 6, 11
    rng = np.random.default_rng(21)
    x = rng.standard_normal((B, H, T, D))
    for G in (1, H):
        a = np.stack([np.stack([np.sort(rng.choice(T, n, replace=False)) for _ in range(G)])
                      for _ in range(B)]).astype(np.int32)
        assign, counts = oracle.assign_nearest(a, T)
        lo, _ = oracle.bucket_bounds(a, T)
        cache = oracle.merge_compact(x, assign, n, cap=n + 3)
        assert (cache[:, :, n:] == 0).all()
        for b in range(B):
            for h in range(H):
                g = 0 if G == 1 else h
                sums = np.add.reduceat(x[b, h], lo[b, g], axis=0)
                np.testing.assert_allclose(cache[b, h, :n], sums / counts[b, g][:, None], atol=1e-13)
                # first-moment conservation: sum_k |B_k| KV_k = sum_t kv_t
                np.testing.assert_allclose((cache[b, h, :n] * counts[b, g][:, None]).sum(0),
                                           x[b, h].sum(0), atol=1e-11)


def test_merge_special_cases():
    B, H, T, D = 1, 2, 12, 4
    x = _rand((B, H, T, D), 31)
    ident = np.arange(T, dtype=np.int32)[None, None]
    assign, counts = oracle.assign_nearest(ident, T)
    np.testing.assert_array_equal(oracle.merge_compact(x, assign, T), x)       # N_I = T: copy
    one = np.array([[[5]]], np.int32)
    assign, counts = oracle.assign_nearest(one, T)
    np.testing.assert_allclose(oracle.merge_compact(x, assign, 1)[:, :, 0], x.mean(2), atol=1e-14)
    const = np.full((B, H, T, D), 3.25)
    a = np.array([[[0, 4, 9]]], np.int32)
    assign, _ = oracle.assign_nearest(a, T)
    np.testing.assert_array_equal(oracle.merge_compact(const, assign, 3), np.full((B, H, 3, D), 3.25))


def test_evict_only_variant_is_a_gather():
    # Table 3b "Cache Eviction": anchors keep their own vectors (library gather as the independent side)
    B, H, T, D, n = 2, 3, 40, 5, 9
    rng = np.random.default_rng(77)
    x = rng.standard_normal((B, H, T, D))
    for G in (1, H):
        a = np.stack([np.stack([np.sort(rng.choice(T, n, replace=False)) for _ in range(G)])
                      for _ in range(B)]).astype(np.int32)
        got = oracle.evict_compact(x, a, cap=n + 2)
        idx = np.broadcast_to(a if G == H else np.repeat(a, H, axis=1), (B, H, n))
        want = np.take_along_axis(x, idx[..., None].astype(np.int64), axis=2)
        np.testing.assert_array_equal(got[:, :, :n], want)
        assert (got[:, :, n:] == 0).all()


# ----------------------------------------------------------------- decode attention + removal
def _fresh_cache(B, H, cap, D, n, seed):
    rng = np.random.default_rng(seed)
    kc = np.zeros((B, H, cap, D))
    vc = np.zeros((B, H, cap, D))
    kc[:, :, :n] = rng.standard_normal((B, H, n, D)) * 1.3
    vc[:, :, :n] = rng.standard_normal((B, H, n, D))
    return kc, vc


def test_decode_against_library_attention_and_delete():
    B, H, D, cap, n = 2, 3, 8, 20, 13
    kc, vc = _fresh_cache(B, H, cap, D, n, 41)
    pos = np.tile(np.arange(cap, dtype=np.int32) * 2, (B, 1, 1))
    q, kn, vn = _rand((B, H, D), 42), _rand((B, H, D), 43), _rand((B, H, D), 44)
    kc0, vc0, pos0 = kc.copy(), vc.copy(), pos.copy()
    out, probs = oracle.decode_step(q, kn, vn, kc, vc, pos, n, 4, 777, 0.3, want_probs=True)
    K = np.concatenate([kc0[:, :, :n], kn[:, :, None]], 2)
    V = np.concatenate([vc0[:, :, :n], vn[:, :, None]], 2)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[:, :, None], torch.from_numpy(K), torch.from_numpy(V), scale=0.3)
    np.testing.assert_allclose(out, ref.numpy()[:, :, 0], atol=1e-13)
    np.testing.assert_allclose(probs.sum(-1), 1.0, atol=1e-14)
    np.testing.assert_array_equal(kc[:, :, :n], np.delete(K, 4, axis=2))
    np.testing.assert_array_equal(vc[:, :, :n], np.delete(V, 4, axis=2))
    want_pos = np.delete(np.concatenate([pos0[:, :, :n], np.full((B, 1, 1), 777, np.int32)], 2), 4, axis=2)
    np.testing.assert_array_equal(pos[:, :, :n], want_pos)
    # no eviction: the row is only appended
    kc, vc = kc0.copy(), vc0.copy()
    oracle.decode_step(q, kn, vn, kc, vc, None, n, -1, 0, 0.3)
    np.testing.assert_array_equal(kc[:, :, :n + 1], K)
    assert (kc[:, :, n + 1:] == 0).all()


def test_decode_special_cases():
    B, H, D, cap = 1, 2, 4, 9
    q, kn, vn = _rand((B, H, D), 51), _rand((B, H, D), 52), _rand((B, H, D), 53)
    kc, vc = np.zeros((B, H, cap, D)), np.zeros((B, H, cap, D))
    out, _ = oracle.decode_step(q, kn, vn, kc, vc, None, 0, -1, 0, 1.0)   # empty cache -> v_new
    np.testing.assert_allclose(out, vn, atol=1e-15)
    kc, vc = _fresh_cache(B, H, cap, D, 6, 54)
    kc[:, :, :6] = kn[:, :, None]                                          # identical keys -> mean(V)
    V = np.concatenate([vc[:, :, :6], vn[:, :, None]], 2)
    out, _ = oracle.decode_step(q, kn, vn, kc, vc, None, 6, -1, 0, 1.0)
    np.testing.assert_allclose(out, V.mean(2), atol=1e-14)
    kc, vc = _fresh_cache(B, H, cap, D, 6, 55)                             # row order does not matter
    perm = np.array([3, 0, 5, 1, 4, 2])
    kp, vp = kc.copy(), vc.copy()
    kp[:, :, :6], vp[:, :, :6] = kc[:, :, perm], vc[:, :, perm]
    o1, _ = oracle.decode_step(q, kn, vn, kc, vc, None, 6, -1, 0, 0.7)
    o2, _ = oracle.decode_step(q, kn, vn, kp, vp, None, 6, -1, 0, 0.7)
    np.testing.assert_allclose(o1, o2, atol=1e-14)


# ----------------------------------------------------------------- retention test (Alg. 1)
def _alg1_del_num(seq_len, n, gamma):
    # Alg. 1 literally, in exact rationals: int(seq_len - n*(1-r)) with 1-r = gamma
    x = Fraction(seq_len) - Fraction(n) * gamma
    return int(x)  # truncation toward zero, like Python's int() on a float


def test_evict_index_follows_alg1_and_golden_lengths():
    for line in open(os.path.join(GOLD, "retention_lengths.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, T, p, q, steps, len0, len1 = line.split()
        T, p, q, steps, len0, len1 = (int(x) for x in (T, p, q, steps, len0, len1))
        gamma = Fraction(p, q)
        assert T - _alg1_del_num(T, T, gamma) == len0
        N = len0
        for t in range(steps):
            n = T + t + 1
            idx = oracle.evict_index(n, N + 1, p, q)
            want_del = _alg1_del_num(N + 1, n, gamma)
            assert want_del in (0, 1)
            if want_del >= 1:
                assert idx == N + 1 - 1 - 25   # 25 newest rows (incl. the new one) stay behind it
                N = N + 1 - 1
            else:
                assert idx == -1
                N = N + 1
            assert N == -((-p * n) // q)       # closed form ceil(gamma n)
        assert N == len1


def test_evict_index_modes_and_edges():
    # fixed budget: evict on every step once full
    assert oracle.evict_index(1000, 101, 1, 2, budget_mode=1, fixed_len=100) == 101 - 1 - 25
    assert oracle.evict_index(1000, 100, 1, 2, budget_mode=1, fixed_len=100) == -1
    # absolute truncation location
    assert oracle.evict_index(1000, 101, 1, 2, budget_mode=1, fixed_len=100, trunc_mode=1, n_tl=60) == 60
    # short cache: never below protect_first, never the newest row
    assert oracle.evict_index(10, 6, 1, 2, recent=25, protect_first=1) == 1
    assert oracle.evict_index(10, 6, 1, 2, recent=25, protect_first=0) == 0
    assert oracle.evict_index(3, 2, 1, 2, recent=25, protect_first=1) == -1   # within budget
    assert oracle.evict_index(2, 2, 1, 2, recent=25, protect_first=1) == -1   # only the newest row is left
    assert oracle.evict_index(10, 7, 1, 2, budget_mode=1, fixed_len=3, trunc_mode=1, n_tl=6) == -1


# ----------------------------------------------------------------- multi-token pass over an existing cache
@pytest.mark.parametrize("B,H,Tq,P,D,scale", [(2, 3, 9, 7, 5, 0.37), (1, 2, 5, 20, 8, 1.0), (1, 2, 12, 0, 4, 0.5),
                                               (1, 1, 1, 13, 6, 0.7)])
def test_chunk_score_against_library_attention(B, H, Tq, P, D, scale):
    # Alg. 1's multi-token branch with a past: attn is Tq x (P+Tq), query m sees rows n <= P+m
    L = P + Tq
    q, k, v = _rand((B, H, Tq, D), 31), _rand((B, H, L, D), 32, 1.5), _rand((B, H, L, D), 33)
    r = oracle.chunk_score(q, k, v, P, scale, H)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    mask = torch.arange(L)[None, :] <= (P + torch.arange(Tq))[:, None]
    ref_out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    np.testing.assert_allclose(r["out"], ref_out.numpy(), atol=1e-12)
    s = (scale * torch.einsum("bhmd,bhnd->bhmn", tq, tk)).masked_fill(~mask, float("-inf"))
    np.testing.assert_allclose(r["lse"], torch.logsumexp(s, -1).numpy(), atol=1e-12)
    A = torch.softmax(s, -1)
    np.testing.assert_allclose(r["score"], A.sum(-2).numpy(), atol=1e-12)
    r1 = oracle.chunk_score(q, k, v, P, scale, 1)
    np.testing.assert_allclose(r1["score"][:, 0], A.sum(-2).mean(1).numpy(), atol=1e-12)


def test_chunk_score_closed_form_zero_queries():
    # q = 0 -> A_mn = 1/(P+m+1) for n <= P+m -> I_n = H_{P+Tq} - H_{max(n,P)} (harmonic numbers)
    Tq, P, D, H = 23, 11, 4, 2
    L = P + Tq
    q = np.zeros((1, H, Tq, D))
    k, v = _rand((1, H, L, D), 34), _rand((1, H, L, D), 35)
    r = oracle.chunk_score(q, k, v, P, 0.5, 1)
    harm = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, L + 1))])
    expect = harm[L] - harm[np.maximum(np.arange(L), P)]
    np.testing.assert_allclose(r["score"][0, 0], expect, atol=1e-13)
    run_mean = (np.cumsum(v, axis=2) / np.arange(1, L + 1)[None, None, :, None])[:, :, P:]
    np.testing.assert_allclose(r["out"], run_mean, atol=1e-13)
    np.testing.assert_allclose(r["score"].sum(-1), Tq, rtol=1e-13)  # every query row sums to 1


def test_chunk_score_is_the_tail_of_the_square_pass():
    # the chunk's queries are the last Tq rows of a causal pass over all P+Tq rows
    B, H, Tq, P, D = 1, 2, 10, 14, 6
    L = P + Tq
    qa, k, v = _rand((B, H, L, D), 36), _rand((B, H, L, D), 37), _rand((B, H, L, D), 38)
    full = oracle.prefill_score(qa, k, v, 0.4, H, want_attn=True)
    r = oracle.chunk_score(qa[:, :, P:], k, v, P, 0.4, H)
    np.testing.assert_allclose(r["out"], full["out"][:, :, P:], atol=1e-13)
    np.testing.assert_allclose(r["lse"], full["lse"][:, :, P:], atol=1e-13)
    np.testing.assert_allclose(r["score"], full["attn"][:, :, P:, :].sum(-2), atol=1e-13)
    # P = 0 is the first-turn pass itself
    r0 = oracle.chunk_score(qa, k, v, 0, 0.4, 1)
    f0 = oracle.prefill_score(qa, k, v, 0.4, 1)
    np.testing.assert_allclose(r0["score"], f0["score"], atol=1e-13)


def test_chunk_score_single_query_is_decode_attention():
    # Tq = 1: one query over P cached rows + its own row = the generation step's attention
    B, H, P, D = 2, 3, 17, 8
    q, k, v = _rand((B, H, 1, D), 39), _rand((B, H, P + 1, D), 40), _rand((B, H, P + 1, D), 41)
    r = oracle.chunk_score(q, k, v, P, 0.3, H)
    kc = np.zeros((B, H, P + 2, D)); vc = np.zeros_like(kc)
    kc[:, :, :P] = k[:, :, :P]; vc[:, :, :P] = v[:, :, :P]
    out, probs = oracle.decode_step(q[:, :, 0], k[:, :, P], v[:, :, P], kc, vc, None, P, -1, 0, 0.3, want_probs=True)
    np.testing.assert_allclose(r["out"][:, :, 0], out, atol=1e-13)
    np.testing.assert_allclose(r["score"], probs, atol=1e-13)


# ----------------------------------------------------------------- count-weighted re-merge
def test_merge_weighted_unit_weights_is_eq3():
    B, H, T, D, n = 2, 3, 40, 5, 9
    x = _rand((B, H, T, D), 42)
    rng = np.random.default_rng(43)
    a = np.stack([np.sort(rng.choice(T, n, replace=False)) for _ in range(B)]).astype(np.int32).reshape(B, 1, n)
    assign, counts = oracle.assign_nearest(a, T)
    cache, wsum = oracle.merge_weighted(x, assign, np.ones_like(assign), n)
    np.testing.assert_array_equal(wsum, counts)
    lo, _ = oracle.bucket_bounds(a, T)
    for b in range(B):
        ref = np.add.reduceat(x[b], lo[b, 0], axis=1) / counts[b, 0][None, :, None]
        np.testing.assert_allclose(cache[b], ref, atol=1e-13)


def test_merge_weighted_two_levels_equal_one_level():
    # Merging means with their counts as weights equals merging the original rows into the union
    # buckets directly (the weighted mean is associative); the plain mean of means is not.
    B, H, T, D = 1, 2, 60, 4
    x = _rand((B, H, T, D), 44)
    a1 = np.array([0, 3, 4, 10, 11, 12, 30, 31, 45, 59], np.int32).reshape(1, 1, -1)
    n1 = a1.shape[-1]
    assign1, counts1 = oracle.assign_nearest(a1, T)
    level1 = oracle.merge_compact(x, assign1, n1)
    a2 = np.array([0, 2, 5, 9], np.int32).reshape(1, 1, -1)  # anchors among the n1 level-1 rows
    assign2, _ = oracle.assign_nearest(a2, n1)
    level2, wsum = oracle.merge_weighted(level1, assign2, counts1, 4)
    # union buckets: original position t -> level-1 bucket -> level-2 bucket
    direct_assign = assign2[0, 0][assign1[0, 0]].reshape(1, 1, T)
    direct = oracle.merge_compact(x, direct_assign, 4)
    np.testing.assert_allclose(level2, direct, atol=1e-13)
    np.testing.assert_array_equal(wsum[0, 0], np.bincount(direct_assign[0, 0], minlength=4))
    assert wsum.sum() == T
    plain = oracle.merge_compact(level1, assign2, 4)
    assert np.abs(plain - direct).max() > 1e-3  # the unweighted mean of means differs
    # first moment conservation: sum_k wsum_k * row_k = sum_t x_t
    np.testing.assert_allclose((level2 * wsum[0, 0][None, None, :, None]).sum(2), x.sum(2), atol=1e-12)


# ----------------------------------------------------------------- frequency discard policy (Table 3a "Frequency")
def test_frequency_counts_are_the_column_sums_of_the_generated_rows():
    # Starting from zero counts, Tq generation steps over P cached rows accumulate exactly the column
    # sums of the Tq x (P+Tq) attention matrix, i.e. chunk_score's scores (itself pinned to library SDPA).
    B, H, P, Tq, D, scale = 2, 3, 9, 7, 5, 0.6
    q, k, v = _rand((B, H, Tq, D), 51), _rand((B, H, P + Tq, D), 52), _rand((B, H, P + Tq, D), 53)
    for G in (1, H):
        cap = P + Tq + 1
        kc = np.zeros((B, H, cap, D)); vc = np.zeros_like(kc)
        kc[:, :, :P] = k[:, :, :P]; vc[:, :, :P] = v[:, :, :P]
        freq = np.zeros((B, G, cap))
        outs = []
        for t in range(Tq):
            o, _ = oracle.decode_score_step(q[:, :, t], k[:, :, P + t], v[:, :, P + t], kc, vc, None, freq, P + t, 0, scale)
            outs.append(o)
        ref = oracle.chunk_score(q, k, v, P, scale, G)
        np.testing.assert_allclose(freq[:, :, :P + Tq], ref["score"], atol=1e-13)
        np.testing.assert_allclose(np.stack(outs, 2), ref["out"], atol=1e-13)
        assert (freq[:, :, P + Tq:] == 0).all()


def test_frequency_update_by_hand():
    # two heads, three rows, hand-made probabilities: layer-wise mass is the head mean; the newest row is set
    probs = np.array([[[0.5, 0.25, 0.25], [0.1, 0.3, 0.6]]])          # [B=1,H=2,n=3]
    lib = oracle._load()
    f1 = np.array([[[1.0, 2.0, 99.0, 7.0]]])                            # cap 4; row 2 is the new one, row 3 unused
    assert lib.oracle_freq_accumulate(oracle._d(probs), 1, 2, 1, 3, 4, oracle._d(f1)) == 0
    np.testing.assert_allclose(f1, [[[1.3, 2.275, 0.425, 7.0]]], atol=1e-15)
    fh = np.array([[[1.0, 2.0, 99.0, 7.0], [0.0, 0.0, 99.0, 7.0]]])
    assert lib.oracle_freq_accumulate(oracle._d(probs), 1, 2, 2, 3, 4, oracle._d(fh)) == 0
    np.testing.assert_allclose(fh, [[[1.5, 2.25, 0.25, 7.0], [0.1, 0.3, 0.6, 7.0]]], atol=1e-15)


@pytest.mark.parametrize("G", [1, 3])
def test_evict_min_against_numpy(G):
    B, H, D, cap, length, pf, pr = 2, 3, 4, 12, 10, 1, 2
    rng = np.random.default_rng(60 + G)
    kc, vc = rng.standard_normal((B, H, cap, D)), rng.standard_normal((B, H, cap, D))
    pos = np.tile(np.arange(cap, dtype=np.int32) * 3, (B, G, 1))
    freq = rng.random((B, G, cap)).astype(np.float32)
    freq[0, 0, 0] = -1.0          # protected: never chosen although smallest
    freq[0, 0, 9] = -1.0          # newest rows are protected too
    freq[1, 0, 3] = freq[1, 0, 6] = 0.0   # tie: the lower index goes
    k0, v0, p0, f0 = kc.copy(), vc.copy(), pos.copy(), freq.copy()
    victim = oracle.evict_min(freq, kc, vc, pos, length, pf, pr)
    for b in range(B):
        for g in range(G):
            want = pf + int(np.argmin(f0[b, g, pf:length - pr]))      # first occurrence of the minimum
            assert victim[b, g] == want
            np.testing.assert_array_equal(freq[b, g, :length - 1], np.delete(f0[b, g, :length], want))
            np.testing.assert_array_equal(pos[b, g, :length - 1], np.delete(p0[b, g, :length], want))
            for h in ([g] if G == H else range(H)):
                np.testing.assert_array_equal(kc[b, h, :length - 1], np.delete(k0[b, h, :length], want, axis=0))
                np.testing.assert_array_equal(vc[b, h, :length - 1], np.delete(v0[b, h, :length], want, axis=0))
    assert victim[1, 0] == 3
    with pytest.raises(ValueError):
        oracle.evict_min(freq, kc, vc, pos, 3, 2, 1)   # nothing left to choose from


# ----------------------------------------------------------------- fixed-point elimination over a whole generation
@pytest.mark.parametrize("T,p,q,steps", [(200, 1, 2, 90), (333, 1, 4, 120), (400, 1, 10, 70)])
def test_fixed_point_survivors_in_closed_form(T, p, q, steps):
    """With the recent distance R = 25 (Sec. 4.1) the victim is always the row that has exactly R rows behind
    it, i.e. the row that just left the window of the R newest.  So a row survives iff the step at which it
    leaves that window is one where the retention test keeps everything (Alg. 1's del_num = 0); rows deeper
    than the window at the start are never touched.  The oracle's position bookkeeping must show exactly that.
    (Caches longer than R rows; shorter ones raise the victim to protect_first, covered with the edge cases.)"""
    R, H, D = 25, 1, 2
    n0 = -(-p * T // q)
    assert n0 > R
    cap = n0 + steps + 1
    rng = np.random.default_rng(T)
    kc, vc = rng.standard_normal((1, H, cap, D)), rng.standard_normal((1, H, cap, D))
    anchors = np.sort(rng.choice(T, n0, replace=False)).astype(np.int32)
    pos = np.zeros((1, 1, cap), np.int32)
    pos[0, 0, :n0] = anchors
    N = n0
    evicting = {}
    for t in range(1, steps + 1):
        idx = oracle.evict_index(T + t, N + 1, p, q, recent=R)
        evicting[t] = idx >= 0
        before = pos[0, 0, :N].copy()
        oracle.decode_step(rng.standard_normal((1, H, D)), rng.standard_normal((1, H, D)), rng.standard_normal((1, H, D)),
                           kc, vc, pos, N, idx, T + t - 1, 0.5)
        if idx >= 0:
            np.testing.assert_array_equal(pos[0, 0, :idx], before[:idx])            # rows before the victim stay
            np.testing.assert_array_equal(pos[0, 0, idx:N - 1], before[idx + 1:])   # rows behind it move up by one
            assert pos[0, 0, N - 1] == T + t - 1                                    # the new row closes the cache
        else:
            N += 1
        assert N == -(-p * (T + t) // q)                                            # ceil(gamma * tokens seen)
        assert (np.diff(pos[0, 0, :N]) > 0).all()
    # items in arrival order: the anchors, then the generated tokens T, T+1, ...
    items = list(anchors) + [T + t - 1 for t in range(1, steps + 1)]
    survivors = []
    for i, item in enumerate(items):
        leaves_at = i - (n0 - R) + 1          # the step at which R rows stand behind it
        if leaves_at < 1 or leaves_at > steps or not evicting[leaves_at]:
            survivors.append(item)
    np.testing.assert_array_equal(pos[0, 0, :N], np.array(survivors, np.int32))


# ----------------------------------------------------------------- "Mean" importance metric (Table 3d)
@pytest.mark.parametrize("Tq,P", [(13, 0), (9, 6), (1, 5)])
def test_importance_mean_is_the_mean_over_the_seeing_queries(Tq, P):
    B, H, D, L = 2, 2, 4, P + Tq
    q, k, v = _rand((B, H, Tq, D), 71), _rand((B, H, L, D), 72), _rand((B, H, L, D), 73)
    r = oracle.chunk_score(q, k, v, P, 0.5, H)
    got = oracle.importance_mean(r["score"], Tq, P)
    tq, tk = torch.from_numpy(q), torch.from_numpy(k)
    mask = torch.arange(L)[None, :] <= (P + torch.arange(Tq))[:, None]
    s = (0.5 * torch.einsum("bhmd,bhnd->bhmn", tq, tk)).masked_fill(~mask, float("-inf"))
    A = torch.softmax(s, -1).numpy()
    A[..., ~mask.numpy()] = np.nan                     # entries a query cannot see do not enter the mean
    np.testing.assert_allclose(got, np.nanmean(A, axis=-2), atol=1e-13)
    assert got is not r["score"] and not np.shares_memory(got, r["score"])
