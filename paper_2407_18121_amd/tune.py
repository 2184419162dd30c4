"""Timing of single entry points over launch shapes and input structure, through the ctypes binding.

    python -m paper_2407_18121_amd.tune decode   # ec_decode_step_shaped: fused launch against every split shape
    python -m paper_2407_18121_amd.tune merge    # ec_merge_compact on three anchor distributions
    python -m paper_2407_18121_amd.tune select   # ec_select_anchors
    python -m paper_2407_18121_amd.tune score    # ec_prefill_score

Every measurement replays one HIP graph that walks several distinct sets of buffers (so that nothing is served
from a cache a real layer loop would not have) and reports microseconds per call by HIP events on the launch
stream.  Inputs are seeded random numbers: this tool times kernels, it checks nothing.
"""
from __future__ import annotations

import sys

import torch

from . import binding as ec

BF16 = torch.bfloat16


def graph_time_ms(fn, iters: int = 5) -> float:
    """Milliseconds per replay of the launches fn() makes, captured once into a HIP graph."""
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            fn()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def _randn(*shape):
    return torch.randn(*shape, device="cuda").to(BF16)


def time_decode(B, H, D, N, waves, unroll, splits, sets=32):
    """(us per launch, algorithmic GB/s) of one generation step over N cached rows with an eviction."""
    cap = N + 2
    kc = [_randn(B, H, cap, D) for _ in range(sets)]
    vc = [_randn(B, H, cap, D) for _ in range(sets)]
    q, kn, vn = (_randn(B, H, D) for _ in range(3))
    out = torch.empty(B, H, D, device="cuda", dtype=BF16)
    pos = torch.zeros(B, 1, cap, dtype=torch.int32, device="cuda")
    ws = torch.zeros(4 * B * H * max(splits, 1) * (D + 2) + 256, dtype=torch.uint8, device="cuda")

    def fn():
        for l in range(sets):
            ec.ec_decode_step_shaped(q, kn, vn, kc[l], vc[l], pos, N, N - 25, 5, 0.088, out, ws,
                                     waves=waves, unroll=unroll, splits=splits)

    ms = graph_time_ms(fn) / sets
    return ms * 1e3, 2 * B * H * (N + 1) * D * 2 / (ms * 1e-3) / 1e9


DECODE_SHAPES = {  # name: (B, H, D, cached rows in the middle of the generation)
    "C2": (1, 32, 128, 640), "C4": (4, 40, 128, 640), "C3": (8, 32, 128, 576), "T1": (8, 40, 128, 256),
    "T3": (16, 32, 128, 256), "C5": (16, 32, 128, 870), "T4": (48, 32, 128, 150)}


def tune_decode():
    for name, (B, H, D, N) in DECODE_SHAPES.items():
        sets = 16 if name == "C5" else 32
        us, gbps = time_decode(B, H, D, N, 0, 0, 1, sets)
        print(f"decode {name} B{B} H{H} rows {N}: one launch (library's choice) {us:7.2f} us {gbps:7.0f} GB/s", flush=True)
        for waves, unroll in ((2, 4), (2, 8), (4, 4), (4, 6), (4, 8), (4, 12), (8, 4), (8, 8), (16, 4)):
            us, gbps = time_decode(B, H, D, N, waves, unroll, 1, sets)
            print(f"decode {name}:   one launch, {waves:2d} waves x {unroll:2d} loads in flight {us:7.2f} us {gbps:7.0f} GB/s", flush=True)
        best = None
        for splits in (2, 3, 4, 6, 8, 12, 16):
            if B * H * splits > 4096 or N // splits < 32:
                continue
            for waves, unroll in ((4, 4), (8, 4), (4, 8), (2, 8)):
                us, gbps = time_decode(B, H, D, N, waves, unroll, splits, sets)
                if best is None or us < best[0]:
                    best = (us, gbps, splits, waves, unroll)
        if best:
            print(f"decode {name}: best split + merging launch: {best[0]:7.2f} us {best[1]:7.0f} GB/s "
                  f"(splits {best[2]}, waves {best[3]}, unroll {best[4]})", flush=True)


def anchors(kind, B, T, n):
    """[B,1,n] ascending anchor positions.  uniform: random positions; prompt: the first positions plus 5 %
    of T scattered behind them (what column masses of prompts with heavy hitters select); giant: the first and
    the last positions with one bucket of everything between."""
    rows = []
    for _ in range(B):
        if kind == "uniform":
            a = torch.randperm(T, device="cuda")[:n]
        elif kind == "prompt":
            nh = int(0.05 * T)
            a = torch.cat([torch.arange(n - nh, device="cuda"),
                           torch.randperm(T - (n - nh), device="cuda")[:nh] + (n - nh)])
        else:
            a = torch.cat([torch.arange(n - 25, device="cuda"), torch.arange(T - 25, T, device="cuda")])
        rows.append(torch.sort(a)[0])
    return torch.stack(rows).to(torch.int32).view(B, 1, n).contiguous()


def time_merge(B, H, D, T, n, kind, sets=8):
    k = [_randn(B, H, T, D) for _ in range(sets)]
    v = [_randn(B, H, T, D) for _ in range(sets)]
    a = anchors(kind, B, T, n)
    kc = torch.empty(B, H, n + 8, D, device="cuda", dtype=BF16)
    vc = torch.empty_like(kc)
    cnt = torch.empty(B, 1, n, dtype=torch.int32, device="cuda")
    pos = torch.empty(B, 1, n + 8, dtype=torch.int32, device="cuda")

    def fn():
        for l in range(sets):
            ec.ec_merge_compact(k[l], v[l], a, kc, vc, cnt, None, pos)

    ms = graph_time_ms(fn) / sets
    return ms * 1e3, 2 * B * H * D * 2 * (T + n) / (ms * 1e-3) / 1e9


def tune_merge():
    shapes = {"C2": (1, 32, 128, 1024, 512), "C3": (8, 32, 128, 2048, 512), "C5 (4 of 16 batch elements)": (4, 32, 128, 8192, 820)}
    for name, (B, H, D, T, n) in shapes.items():
        for kind in ("uniform", "prompt", "giant"):
            us, gbps = time_merge(B, H, D, T, n, kind)
            print(f"merge {name} anchors {kind:8s}: {us:8.2f} us {gbps:7.0f} GB/s", flush=True)


def tune_select():
    for name, (B, T, n) in {"C2": (1, 1024, 512), "C3": (8, 2048, 512), "C5": (16, 8192, 820)}.items():
        sc = [torch.rand(B, 1, T, device="cuda") * 10 for _ in range(8)]
        idx = torch.empty(B, 1, n, dtype=torch.int32, device="cuda")

        def fn():
            for l in range(8):
                ec.ec_select_anchors(sc[l], n, 1, 1, idx)

        print(f"select {name} B{B} T{T} n{n}: {graph_time_ms(fn) / 8 * 1e3:7.2f} us", flush=True)


def tune_score():
    shapes = {"C2": (1, 32, 128, 1024), "C3": (8, 32, 128, 2048), "C5 (4 of 16 batch elements)": (4, 32, 128, 8192)}
    for name, (B, H, D, T) in shapes.items():
        sets = 2
        q, k, v = ([_randn(B, H, T, D) for _ in range(sets)] for _ in range(3))
        out = torch.empty(B, H, T, D, device="cuda", dtype=BF16)
        sc = torch.empty(B, 1, T, device="cuda")
        ws = ec.new_workspace(ec.EC_FN_PREFILL_SCORE, B, H, T, D, ec.dtype_code(out))

        def fn():
            for l in range(sets):
                ec.ec_prefill_score(q[l], k[l], v[l], out, None, sc, 0.088, ws)

        ms = graph_time_ms(fn, iters=3) / sets
        print(f"score {name}: {ms * 1e3:9.1f} us {3.0 * D * T * (T + 1) * B * H / (ms * 1e-3) / 1e12:7.1f} TFLOP/s", flush=True)


def main(argv):
    what = argv[1] if len(argv) > 1 else ""
    table = {"decode": tune_decode, "merge": tune_merge, "select": tune_select, "score": tune_score}
    if what not in table:
        print(__doc__)
        return 2
    if not torch.cuda.is_available():
        print("tune: no GPU", file=sys.stderr)
        return 1
    ec.load()
    torch.manual_seed(1)
    table[what]()
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
