#!/usr/bin/env python3
"""Benchmark of the Elastic Cache hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic prompts:
for every layer ec_prefill_score -> ec_select_anchors -> ec_merge_compact, then
`decode_steps` generated tokens, each walking every layer with ec_evict_index
(host) -> ec_decode_step on that layer's own compressed cache.  All inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

After the timed region it also times, outside `value`, a second turn (`detail.turn2`): a new chunk of
`--turn2` tokens (default: half the prompt) is encoded over the cache the generation left behind with
ec_chunk_score -> ec_select_anchors -> ec_remerge_compact; and `--freq-steps` generated tokens under the
"Frequency" discard policy (`detail.frequency_policy`: ec_decode_score_step + ec_evict_min per layer-step); and, for
batches of two or more, `--ragged-steps` tokens of a mixed-length batch through ec_decode_step_varlen
(`detail.ragged_decode`).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C2] [--score-mode layer|head]
                    [--no-graph] [--no-cpu-baseline] [--turn2 N] [--freq-steps N] [--ragged-steps N] [--no-extras]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA
FP32_VALU_PEAK_TFLOPS = 157.3
# HBM bytes actually moved per algorithmic byte, from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in
# profiles/decode_step_hbm_traffic.txt (counters scaled by a 256 MiB device copy in the same run)
DECODE_TRAFFIC_RATIO = {"C2": 1.04, "C3": 1.04, "C4": 1.03, "C5": 1.03}
PROMPT_BUDGET_GB = 160       # HBM set aside for the prompts' Q, K, V (of 288 GB)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C5", choices=["C1", "C2", "C3", "C4", "C5", "T1", "T2", "T3", "T4"],
                    help="workload (default C5: the largest single-GPU one, on which the roofline bars are defined)")
    ap.add_argument("--score-mode", default="layer", choices=["layer", "head"])
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--decode-steps", type=int, default=0,
                    help="profiling aid: run only the first N generated tokens (the JSON line says so)")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also launch one plain device copy of this many MiB (reference dispatch for HBM counters)")
    ap.add_argument("--turn2", type=int, default=-1,
                    help="tokens of the second-turn chunk timed after the main step (-1 = half the prompt, 0 = skip)")
    ap.add_argument("--freq-steps", type=int, default=32,
                    help="generated tokens timed under the frequency discard policy after the main step (0 = skip)")
    ap.add_argument("--ragged-steps", type=int, default=16,
                    help="generated tokens timed through ec_decode_step_varlen on a mixed-length batch (0 = skip; needs B >= 2)")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the main step: no second turn, frequency policy, ragged or layers-folded runs "
                         "(kernel traces then hold the main path's launches alone)")
    ap.add_argument("--distinct-layers", type=int, default=0,
                    help="distinct prompt tensors to generate (0 = one per layer, or as many as fit in "
                         f"{PROMPT_BUDGET_GB} GB of HBM; fewer than the layers are cycled, and the JSON line says so)")
    args = ap.parse_args()
    if args.no_extras:
        args.turn2 = args.freq_steps = args.ragged_steps = 0
    return args


class Workload:
    """Device buffers + the precomputed call list of one hot-path step."""

    def __init__(self, cfg, score_mode, distinct_layers):
        import torch
        from paper_2407_18121_amd import binding as ec
        from paper_2407_18121_amd import synthetic_torch as synt
        self.cfg, self.ec, self.torch = cfg, ec, torch
        self.lib = ec.load()
        dt = synt.torch_dtype(cfg)
        self.dt_code = ec.EC_F32 if cfg.dtype == "f32" else ec.EC_BF16
        B, H, T, D, L = cfg.B, cfg.H, cfg.T, cfg.D, cfg.layers
        self.G = 1 if score_mode == "layer" else H
        per_layer = 3.0 * B * H * T * D * cfg.esize
        fit = max(1, int(PROMPT_BUDGET_GB * 1e9 // per_layer))
        n_distinct = min(L, fit) if distinct_layers <= 0 else min(L, distinct_layers)
        self.n_distinct = n_distinct
        self.prompts = [synt.prompt_qkv_device(cfg, l) for l in range(n_distinct)]
        self.dec = [synt.decode_stream_device(cfg, l) for l in range(L)]
        cap, nA, G = cfg.cap, cfg.n_anchor, self.G
        self.k_cache = [torch.zeros((B, H, cap, D), dtype=dt, device="cuda") for _ in range(L)]
        self.v_cache = [torch.zeros((B, H, cap, D), dtype=dt, device="cuda") for _ in range(L)]
        self.pos = [torch.zeros((B, G, cap), dtype=torch.int32, device="cuda") for _ in range(L)]
        self.score = [torch.empty((B, G, T), dtype=torch.float32, device="cuda") for _ in range(L)]
        self.anchor = [torch.empty((B, G, nA), dtype=torch.int32, device="cuda") for _ in range(L)]
        self.counts = [torch.empty((B, G, nA), dtype=torch.int32, device="cuda") for _ in range(L)]
        self.attn_out = torch.empty((B, H, T, D), dtype=dt, device="cuda")  # consumed by the (absent) model
        self.dec_out = torch.empty((B, H, D), dtype=dt, device="cuda")
        self.ws_prefill = ec.new_workspace(ec.EC_FN_PREFILL_SCORE, B, H, T, D, self.dt_code)
        self.ws_decode = ec.new_workspace(ec.EC_FN_DECODE_STEP, B, H, cap, D, self.dt_code)
        self._build_calls()

    def _build_calls(self):
        cfg, lib, G = self.cfg, self.lib, self.G
        B, H, T, D, L = cfg.B, cfg.H, cfg.T, cfg.D, cfg.layers
        cap, nA, dtc, scale = cfg.cap, cfg.n_anchor, self.dt_code, cfg.scale
        ws_p, ws_pb = self.ws_prefill.data_ptr(), self.ws_prefill.numel()
        ws_d, ws_db = self.ws_decode.data_ptr(), self.ws_decode.numel()
        self.score_calls, self.select_calls, self.merge_calls = [], [], []
        for l in range(L):
            q, k, v = self.prompts[l % len(self.prompts)]
            self.score_calls.append((q.data_ptr(), k.data_ptr(), v.data_ptr(), self.attn_out.data_ptr(), None,
                                     self.score[l].data_ptr(), B, H, G, T, D, dtc, scale, ws_p, ws_pb))
            self.select_calls.append((self.score[l].data_ptr(), B, G, T, nA, 1, 1, self.anchor[l].data_ptr(), None, 0))
            self.merge_calls.append((k.data_ptr(), v.data_ptr(), self.anchor[l].data_ptr(), B, H, G, T, D, nA, dtc, 0,
                                     self.k_cache[l].data_ptr(), self.v_cache[l].data_ptr(), cap,
                                     self.counts[l].data_ptr(), None, self.pos[l].data_ptr()))
        # decode schedule: the retention test is pure host integer arithmetic (Alg. 1)
        self.decode_calls = []
        self.decode_bytes = 0
        p, qd = cfg.gamma
        N = nA
        esz = cfg.esize
        row = D * esz
        for step in range(cfg.decode_steps):
            n_seen = T + step + 1
            idx = self.ec.ec_evict_index(n_seen, N + 1, p, qd)
            for l in range(L):
                dq, dk, dv = self.dec[l]
                self.decode_calls.append((dq[step].data_ptr(), dk[step].data_ptr(), dv[step].data_ptr(),
                                          self.k_cache[l].data_ptr(), self.v_cache[l].data_ptr(), self.pos[l].data_ptr(),
                                          B, H, G, D, cap, N, idx, n_seen - 1, scale, dtc, self.dec_out.data_ptr(),
                                          ws_d, ws_db))
            # algorithmic bytes of one launch: K and V rows read once (incl. the new row)
            self.decode_bytes += L * 2 * B * H * (N + 1) * row
            N += 0 if idx >= 0 else 1
        self.final_len = N
        self.score_flops_per_layer = 3.0 * D * T * (T + 1) * B * H
        self.merge_bytes_per_layer = 2.0 * B * H * D * esz * (T + nA)

    # --- launch helpers (stream = torch's current stream) ---
    def _stream(self):
        return self.torch.cuda.current_stream().cuda_stream

    def run_score(self, s):
        f = self.lib.ec_prefill_score
        for a in self.score_calls:
            rc = f(*a, s)
            assert rc == 0, rc

    def run_select(self, s):
        f = self.lib.ec_select_anchors
        for a in self.select_calls:
            rc = f(*a, s)
            assert rc == 0, rc

    def run_merge(self, s):
        f = self.lib.ec_merge_compact
        for a in self.merge_calls:
            rc = f(*a, s)
            assert rc == 0, rc

    def run_prefill(self, s):
        fs, fa, fm = self.lib.ec_prefill_score, self.lib.ec_select_anchors, self.lib.ec_merge_compact
        for a, b, c in zip(self.score_calls, self.select_calls, self.merge_calls):
            rc = fs(*a, s) | fa(*b, s) | fm(*c, s)
            assert rc == 0, rc

    def run_decode(self, s):
        f = self.lib.ec_decode_step
        for a in self.decode_calls:
            rc = f(*a, s)
            assert rc == 0, rc


class Turn2:
    """A second turn over the cache the generation left: chunk scoring, anchor selection, re-merge (all layers)."""

    def __init__(self, wl, T_new):
        import torch
        from paper_2407_18121_amd import synthetic as syn
        from paper_2407_18121_amd import synthetic_torch as synt
        cfg, ec = wl.cfg, wl.ec
        self.wl, self.lib = wl, wl.lib
        B, H, D, L, G = cfg.B, cfg.H, cfg.D, cfg.layers, wl.G
        dt = synt.torch_dtype(cfg)
        self.P, self.Tq = wl.final_len, T_new
        self.Lr = Lr = self.P + T_new
        n_seen = cfg.T + cfg.decode_steps + T_new
        self.n2 = n2 = min(Lr, -(-cfg.gamma[0] * n_seen // cfg.gamma[1]))
        n_src = min(L, 4)   # distinct source buffers, cycled over the layers
        chunk_cfg = syn.custom(cfg.name + "-turn2", H=H, D=D, B=B, T=T_new, dtype=cfg.dtype, cid=cfg.cid + 500)
        self.q, self.k, self.v = [], [], []
        for i in range(n_src):
            q, k, v = synt.prompt_qkv_device(chunk_cfg, i)
            kb = torch.zeros((B, H, Lr, D), dtype=dt, device="cuda")
            vb = torch.zeros((B, H, Lr, D), dtype=dt, device="cuda")
            kb[:, :, :self.P] = wl.k_cache[i][:, :, :self.P]
            vb[:, :, :self.P] = wl.v_cache[i][:, :, :self.P]
            kb[:, :, self.P:] = k
            vb[:, :, self.P:] = v
            self.q.append(q); self.k.append(kb); self.v.append(vb)
        self.out = torch.empty((B, H, T_new, D), dtype=dt, device="cuda")
        self.score = torch.empty((B, G, Lr), dtype=torch.float32, device="cuda")
        self.anchor = torch.empty((B, G, n2), dtype=torch.int32, device="cuda")
        self.counts = torch.empty((B, G, n2), dtype=torch.int32, device="cuda")
        self.nk = torch.empty((B, H, n2, D), dtype=dt, device="cuda")
        self.nv = torch.empty((B, H, n2, D), dtype=dt, device="cuda")
        self.ws = ec.new_workspace(ec.EC_FN_PREFILL_SCORE, B, H, Lr, D, wl.dt_code)
        ws, wsb = self.ws.data_ptr(), self.ws.numel()
        self.score_calls, self.select_calls, self.merge_calls = [], [], []
        for l in range(L):
            i = l % n_src
            self.score_calls.append((self.q[i].data_ptr(), self.k[i].data_ptr(), self.v[i].data_ptr(), self.out.data_ptr(),
                                     None, self.score.data_ptr(), B, H, G, T_new, self.P, Lr, D, wl.dt_code, cfg.scale, ws, wsb))
            self.select_calls.append((self.score.data_ptr(), B, G, Lr, n2, 1, 1, self.anchor.data_ptr(), None, 0))
            self.merge_calls.append((self.k[i].data_ptr(), self.v[i].data_ptr(), Lr, None, None, self.anchor.data_ptr(), B, H, G,
                                     Lr, D, n2, wl.dt_code, 0, self.nk.data_ptr(), self.nv.data_ptr(), n2,
                                     self.counts.data_ptr(), None, None))
        pairs = float(T_new) * self.P + T_new * (T_new + 1) / 2.0   # visible (query, key) pairs per head
        self.score_flops_per_layer = 6.0 * D * pairs * B * H
        self.merge_bytes_per_layer = 2.0 * B * H * D * cfg.esize * (Lr + n2)

    def run_score(self, s):
        for a in self.score_calls:
            rc = self.lib.ec_chunk_score(*a, s)
            assert rc == 0, rc

    def run_select(self, s):
        for a in self.select_calls:
            rc = self.lib.ec_select_anchors(*a, s)
            assert rc == 0, rc

    def run_merge(self, s):
        for a in self.merge_calls:
            rc = self.lib.ec_remerge_compact(*a, s)
            assert rc == 0, rc

    def run_all(self, s):
        for a, b, c in zip(self.score_calls, self.select_calls, self.merge_calls):
            rc = self.lib.ec_chunk_score(*a, s) | self.lib.ec_select_anchors(*b, s) | self.lib.ec_remerge_compact(*c, s)
            assert rc == 0, rc


class FrequencyDecode:
    """Generation under the "Frequency" discard policy (Table 3a) at a constant cache length: every layer-step is
    ec_decode_score_step followed by ec_evict_min, on the caches the main step left."""

    def __init__(self, wl, steps):
        import torch
        cfg, ec = wl.cfg, wl.ec
        self.wl, self.lib = wl, wl.lib
        B, H, D, L, G, cap = cfg.B, cfg.H, cfg.D, cfg.layers, wl.G, cfg.cap
        N = min(wl.final_len, cap - 1)
        self.N, self.steps = N, min(steps, cfg.decode_steps)
        g = torch.Generator(device="cuda").manual_seed(7)
        self.freq = [torch.rand((B, G, cap), generator=g, device="cuda") * 0.05 for _ in range(L)]
        self.victim = torch.empty((B, G), dtype=torch.int32, device="cuda")
        self.ws = ec.new_workspace(ec.EC_FN_DECODE_SCORE_STEP, B, H, cap, D, wl.dt_code)
        ws, wsb = self.ws.data_ptr(), self.ws.numel()
        self.calls = []
        for step in range(self.steps):
            for l in range(L):
                dq, dk, dv = wl.dec[l]
                self.calls.append(((dq[step].data_ptr(), dk[step].data_ptr(), dv[step].data_ptr(), wl.k_cache[l].data_ptr(),
                                    wl.v_cache[l].data_ptr(), wl.pos[l].data_ptr(), self.freq[l].data_ptr(), B, H, G, D, cap,
                                    N, cfg.T + step, cfg.scale, wl.dt_code, wl.dec_out.data_ptr(), ws, wsb),
                                   (wl.k_cache[l].data_ptr(), wl.v_cache[l].data_ptr(), wl.pos[l].data_ptr(),
                                    self.freq[l].data_ptr(), B, H, G, D, cap, N + 1, 1, 1, wl.dt_code, self.victim.data_ptr())))
        self.bytes_per_layer_step = 2.0 * B * H * (N + 1) * D * cfg.esize

    def run(self, s):
        f, e = self.lib.ec_decode_score_step, self.lib.ec_evict_min
        for a, b in self.calls:
            rc = f(*a, s) | e(*b, s)
            assert rc == 0, rc


class RaggedDecode:
    """ec_decode_step_varlen on a batch whose caches hold between half and all of the rows the main step ends
    with (evenly spread), every sequence evicting at its own recent-distance location so that lengths stay put."""

    def __init__(self, wl, steps):
        import torch
        cfg = wl.cfg
        self.wl, self.lib = wl, wl.lib
        B, H, D, L, G, cap = cfg.B, cfg.H, cfg.D, cfg.layers, wl.G, cfg.cap
        N = min(wl.final_len, cap - 1)
        lens = [N // 2 + (N - N // 2) * b // max(B - 1, 1) for b in range(B)]
        self.lens, self.steps = lens, min(steps, cfg.decode_steps)
        self.len_b = torch.tensor(lens, dtype=torch.int32, device="cuda")
        self.vic_b = torch.tensor([max(n - 25, 1) for n in lens], dtype=torch.int32, device="cuda")
        self.pos_b = torch.tensor([cfg.T + 7] * B, dtype=torch.int32, device="cuda")
        self.calls = []
        for step in range(self.steps):
            for l in range(L):
                dq, dk, dv = wl.dec[l]
                self.calls.append((dq[step].data_ptr(), dk[step].data_ptr(), dv[step].data_ptr(), wl.k_cache[l].data_ptr(),
                                   wl.v_cache[l].data_ptr(), wl.pos[l].data_ptr(), self.len_b.data_ptr(), self.vic_b.data_ptr(),
                                   self.pos_b.data_ptr(), B, H, G, D, cap, cfg.scale, wl.dt_code, wl.dec_out.data_ptr(), None, 0))
        self.bytes_per_launch = sum(2.0 * H * (n + 1) * D * cfg.esize for n in lens)

    def run(self, s):
        f = self.lib.ec_decode_step_varlen
        for a in self.calls:
            rc = f(*a, s)
            assert rc == 0, rc


class FoldedDecode:
    """Layers folded into the batch: ONE ec_decode_step launch over all layers' caches of a token step.  Legal only
    because the synthetic decode inputs of a layer do not depend on the layer below; reported for small batches,
    where a per-layer launch has too few (batch, head) pairs to fill the chip."""

    def __init__(self, wl, launches):
        import torch
        from paper_2407_18121_amd import synthetic_torch as synt
        cfg = wl.cfg
        self.wl, self.lib = wl, wl.lib
        B, H, D, L, G, cap = cfg.B, cfg.H, cfg.D, cfg.layers, wl.G, cfg.cap
        dt = synt.torch_dtype(cfg)
        N = min(wl.final_len, cap - 1)
        self.N, self.launches = N, launches
        g = torch.Generator(device="cuda").manual_seed(11)
        self.kc = torch.randn((L * B, H, cap, D), generator=g, device="cuda").to(dt)
        self.vc = torch.randn((L * B, H, cap, D), generator=g, device="cuda").to(dt)
        self.q, self.kn, self.vn = (torch.randn((L * B, H, D), generator=g, device="cuda").to(dt) for _ in range(3))
        self.out = torch.empty((L * B, H, D), dtype=dt, device="cuda")
        self.call = (self.q.data_ptr(), self.kn.data_ptr(), self.vn.data_ptr(), self.kc.data_ptr(), self.vc.data_ptr(), None,
                     L * B, H, G, D, cap, N, max(N - 25, 1), 0, cfg.scale, wl.dt_code, self.out.data_ptr(), None, 0)
        self.bytes_per_launch = 2.0 * L * B * H * (N + 1) * D * cfg.esize

    def run(self, s):
        for _ in range(self.launches):
            rc = self.lib.ec_decode_step(*self.call, s)
            assert rc == 0, rc


def capture(torch, fn):
    """Record fn(stream) into a HIP graph; returns a replay callable, or None if capture is not possible."""
    try:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                fn(torch.cuda.current_stream().cuda_stream)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        return g.replay
    except Exception as e:  # pragma: no cover
        print(f"[bench] graph capture unavailable ({type(e).__name__}: {e}); launching eagerly", file=sys.stderr)
        return None


def timed(torch, fn, reps):
    """Average milliseconds of fn() over reps, measured with HIP events on the current stream."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def cpu_baseline(cfg, wl, G, budget_s=20.0):
    """Time the fp64 oracle (as it stands) on a bounded sample of the same workload, scaled to whole-job tokens/s."""
    import numpy as np
    import oracle
    B, H, T, D, L = cfg.B, cfg.H, cfg.T, cfg.D, cfg.layers
    # one layer of the fp64 brute force costs ~4*D*T^2/2*B*H flop; bound one sample layer to ~6e11 flop
    flops_per_b = 2.0 * D * T * (T + 1) * H
    nb = max(1, min(B, int(6e11 // flops_per_b)))
    frac = nb / B
    t_start = time.perf_counter()
    t_prefill, n_layers = [], 0
    kc = vc = None
    for l in range(L):
        q, k, v = (x[:nb].float().cpu().numpy() for x in wl.prompts[l % len(wl.prompts)])
        t0 = time.perf_counter()
        r = oracle.prefill_score(q, k, v, cfg.scale, G, want_out=True)
        a = oracle.select_anchors(r["score"].astype(np.float32), cfg.n_anchor, 1, 1)
        assign, _ = oracle.assign_nearest(a, T)
        kc = oracle.merge_compact(k, assign, cfg.n_anchor, cfg.cap)
        vc = oracle.merge_compact(v, assign, cfg.n_anchor, cfg.cap)
        t_prefill.append(time.perf_counter() - t0)
        n_layers += 1
        if time.perf_counter() - t_start > 0.6 * budget_s:
            break
    # decode: steps spread over the run, each at the cache length the schedule has there
    p, qd = cfg.gamma
    lens, N = [], cfg.n_anchor
    for step in range(cfg.decode_steps):
        idx = oracle.evict_index(T + step + 1, N + 1, p, qd)
        lens.append((N, idx))
        N += 0 if idx >= 0 else 1
    t_dec, n_dec_layers = [], 0
    for l in range(L):          # whole decode runs of successive layers until the budget is used
        dq, dk, dv = (x[:, :nb].float().cpu().numpy() for x in wl.dec[l])
        for step in range(cfg.decode_steps):
            n, idx = lens[step]
            t0 = time.perf_counter()
            oracle.decode_step(dq[step], dk[step], dv[step], kc, vc, None, n, idx, T + step, cfg.scale)
            t_dec.append(time.perf_counter() - t0)
        n_dec_layers += 1
        if time.perf_counter() - t_start > budget_s:
            break
    t_prefill_layer = float(np.mean(t_prefill)) / frac
    t_decode_layer_step = float(np.mean(t_dec)) / frac
    total = L * t_prefill_layer + L * cfg.decode_steps * t_decode_layer_step
    return {
        "value": B * cfg.decode_steps / total, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": (f"{nb}/{B} batch elements, all {H} heads: score+select+merge of {n_layers} layer(s) "
                   f"{sum(t_prefill):.2f} s, all {cfg.decode_steps} decode steps of {n_dec_layers} layer(s) {sum(t_dec):.2f} s; "
                   f"scaled linearly to {L} layers x {cfg.decode_steps} steps x full batch"),
        "prefill_s_per_layer": t_prefill_layer, "decode_s_per_layer_step": t_decode_layer_step,
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the hot path has no cross-GPU exchange); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2407_18121_amd import synthetic as syn
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    cfg = syn.CONFIGS[args.config]
    truncated = 0 < args.decode_steps < cfg.decode_steps
    if truncated:
        import dataclasses
        cfg = dataclasses.replace(cfg, decode_steps=args.decode_steps)
    wl = Workload(cfg, args.score_mode, args.distinct_layers)
    L, B = cfg.layers, cfg.B
    torch.cuda.synchronize()
    if args.calib_copy_mb > 0:  # a copy of known size, so that profiler byte counters can be scaled
        src = torch.empty(args.calib_copy_mb << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    print(f"[bench] workload {cfg.name} resident; eager pass", file=sys.stderr, flush=True)
    eager_prefill = lambda: wl.run_prefill(wl._stream())
    eager_decode = lambda: wl.run_decode(wl._stream())
    # eager pass first: also validates every argument before anything is captured
    eager_prefill()
    eager_decode()
    torch.cuda.synchronize()
    replay_prefill = replay_decode = None
    if not args.no_graph:
        replay_prefill = capture(torch, wl.run_prefill)
        replay_decode = capture(torch, wl.run_decode) if replay_prefill else None
    use_graph = replay_prefill is not None and replay_decode is not None
    do_prefill = replay_prefill if use_graph else eager_prefill
    do_decode = replay_decode if use_graph else eager_decode

    print(f"[bench] launch mode {'hipgraph' if use_graph else 'eager'}; warmup + timed steps", file=sys.stderr, flush=True)
    for _ in range(args.warmup):
        do_prefill()
        do_decode()
    torch.cuda.synchronize()

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        do_prefill()
        ev[i][1].record()
        do_decode()
        ev[i][2].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall0) * 1e3 / args.steps
    prefill_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    decode_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    ms_per_step = max(wall_ms, prefill_ms + decode_ms)

    print("[bench] timed region done; per-call breakdown", file=sys.stderr, flush=True)
    # ---- per-call breakdown (outside the timed region above, same buffers, same launch mode) ----
    def per_layer_ms(run):
        fn = (capture(torch, run) if use_graph else None) or (lambda: run(wl._stream()))
        fn()
        return timed(torch, fn, 3) / L
    score_ms = per_layer_ms(wl.run_score)
    select_ms = per_layer_ms(wl.run_select)
    merge_ms = per_layer_ms(wl.run_merge)
    do_prefill()  # restore the compressed caches for whoever looks at them next
    torch.cuda.synchronize()

    # ---- rows beyond the core path, each outside `value`; a failure in one is reported, not fatal ----
    def graph_or_eager(run):
        fn = (capture(torch, run) if use_graph else None) or (lambda: run(wl._stream()))
        fn()
        return fn

    def extra_turn2(t2_len):
        do_decode()   # leaves every layer's cache as the generation ends
        torch.cuda.synchronize()
        t2 = Turn2(wl, t2_len)
        t2.run_all(wl._stream())   # eager validation pass
        torch.cuda.synchronize()
        t2_ms = lambda run: timed(torch, graph_or_eager(run), 3) / L
        a_ms, s_ms, sel_ms, m_ms = t2_ms(t2.run_all), t2_ms(t2.run_score), t2_ms(t2.run_select), t2_ms(t2.run_merge)
        return {"chunk_tokens": t2_len, "cache_rows_before": t2.P, "cache_rows_after": t2.n2,
                "us_per_layer": a_ms * 1e3, "score_us_per_layer": s_ms * 1e3, "select_us_per_layer": sel_ms * 1e3,
                "merge_us_per_layer": m_ms * 1e3, "score_TFLOPs": t2.score_flops_per_layer / (s_ms * 1e-3) / 1e12,
                "merge_GBps": t2.merge_bytes_per_layer / (m_ms * 1e-3) / 1e9}

    def extra_frequency():
        do_decode()
        torch.cuda.synchronize()
        fd = FrequencyDecode(wl, args.freq_steps)
        fd.run(wl._stream())
        torch.cuda.synchronize()
        f_ms = timed(torch, graph_or_eager(fd.run), 3) / (fd.steps * L)
        return {"cache_rows": fd.N, "steps": fd.steps, "us_per_layer_step": f_ms * 1e3,
                "attn_GBps": fd.bytes_per_layer_step / (f_ms * 1e-3) / 1e9, "launches_per_layer_step": 4}

    def extra_ragged():
        do_decode()
        torch.cuda.synchronize()
        rd = RaggedDecode(wl, args.ragged_steps)
        rd.run(wl._stream())
        torch.cuda.synchronize()
        r_ms = timed(torch, graph_or_eager(rd.run), 3) / (rd.steps * L)
        return {"cache_rows": [min(rd.lens), max(rd.lens)], "us_per_launch": r_ms * 1e3,
                "attn_GBps": rd.bytes_per_launch / (r_ms * 1e-3) / 1e9}

    def extra_folded():
        fo = FoldedDecode(wl, 16)
        fo.run(wl._stream())
        torch.cuda.synchronize()
        fo_ms = timed(torch, graph_or_eager(fo.run), 3) / fo.launches
        gbps = fo.bytes_per_launch / (fo_ms * 1e-3) / 1e9
        return {"note": "all layers of one token step in ONE launch (layers as batch); legal only for synthetic inputs",
                "cache_rows": fo.N, "us_per_launch": fo_ms * 1e3, "attn_GBps": gbps,
                "frac_of_hbm_peak": gbps / HBM_PEAK_GBPS, "tokens_per_s_if_folded": B / (fo_ms * 1e-3)}

    def guarded(what, fn, *a):
        print(f"[bench] {what}", file=sys.stderr, flush=True)
        try:
            r = fn(*a)
        except Exception as e:   # the main line must still be printed
            r = {"error": f"{type(e).__name__}: {e}"}
        torch.cuda.synchronize()
        do_prefill()             # back to the compressed caches of the main step
        torch.cuda.synchronize()
        return r

    t2_len = cfg.T // 2 if args.turn2 < 0 else args.turn2
    turn2 = guarded(f"second turn: chunk of {t2_len} tokens over the generated cache", extra_turn2, t2_len) if t2_len > 0 else None
    freq_detail = guarded("frequency discard policy at constant cache length", extra_frequency) if args.freq_steps > 0 else None
    ragged = guarded("ragged batch through ec_decode_step_varlen", extra_ragged) if args.ragged_steps > 0 and B >= 2 else None
    folded = guarded("layers-folded decode launch", extra_folded) if B * cfg.H < 256 and L > 1 and not args.no_extras else None
    # a plain device copy on the same box, for a measured ceiling beside the nominal one
    cp_src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    cp_dst = torch.empty_like(cp_src)
    cp_dst.copy_(cp_src)
    copy_ms = timed(torch, lambda: cp_dst.copy_(cp_src), 5)
    copy_gbps = 2.0 * cp_src.numel() / (copy_ms * 1e-3) / 1e9
    del cp_src, cp_dst
    step_ms = sorted(e[0].elapsed_time(e[2]) for e in ev)

    n_dec = len(wl.decode_calls)
    dec_launch_us = decode_ms * 1e3 / n_dec
    dec_gbps = wl.decode_bytes / (decode_ms * 1e-3) / 1e9
    score_tflops = wl.score_flops_per_layer / (score_ms * 1e-3) / 1e12
    merge_gbps = wl.merge_bytes_per_layer / (merge_ms * 1e-3) / 1e9
    score_peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else FP32_VALU_PEAK_TFLOPS

    res = {
        "metric": "decode-attn GB/s + tokens/s over merged KV; prefill score+merge us/layer",
        "value": B * cfg.decode_steps / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {L} layers, {cfg.H} heads, head_dim {cfg.D}, batch {B}, prompt {cfg.T}, "
                               f"budget {cfg.gamma[0]}/{cfg.gamma[1]}, {cfg.decode_steps} decode steps, {cfg.dtype}",
                   "score_mode": args.score_mode, "launch": "hipgraph" if use_graph else "eager", "truncated_decode": truncated,
                   "cache_len": [cfg.n_anchor, wl.final_len], "distinct_prompt_layers": wl.n_distinct},
        "detail": {
            "decode_attn_GBps": dec_gbps, "decode_tokens_per_s": B * cfg.decode_steps / (decode_ms * 1e-3),
            "decode_us_per_launch": dec_launch_us, "decode_launches": n_dec,
            "prefill_score_merge_us_per_layer": prefill_ms * 1e3 / L,
            "score_us_per_layer": score_ms * 1e3, "select_us_per_layer": select_ms * 1e3,
            "merge_us_per_layer": merge_ms * 1e3,
            "score_TFLOPs": score_tflops, "score_frac_of_peak": score_tflops / score_peak,
            "merge_GBps": merge_gbps, "merge_frac_of_hbm_peak": merge_gbps / HBM_PEAK_GBPS,
            "wall_ms_per_step": wall_ms, "event_ms_per_step": prefill_ms + decode_ms,
            "event_ms_per_step_min": step_ms[0], "event_ms_per_step_median": step_ms[len(step_ms) // 2],
            "device_copy_GBps": copy_gbps,
        },
        "roofline": {
            "kernel": "decode_step_kernel", "bound": "hbm", "achieved": dec_gbps, "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": dec_gbps / HBM_PEAK_GBPS,
            "traffic": (DECODE_TRAFFIC_RATIO[cfg.name] * wl.decode_bytes / n_dec) if cfg.name in DECODE_TRAFFIC_RATIO else None,
            "traffic_source": "algorithmic bytes of this run x the FETCH_SIZE+WRITE_SIZE / algorithmic ratio of the "
                              "rocprofv3 --pmc runs in profiles/decode_step_hbm_traffic.txt",
            "bytes_per_launch": wl.decode_bytes / n_dec, "us_per_launch": dec_launch_us,
            "frac_of_measured_copy": dec_gbps / copy_gbps,
        },
        "roofline_score": {
            "kernel": "prefill score (attention + column mass)", "bound": "mfma" if cfg.dtype == "bf16" else "alu",
            "achieved": score_tflops, "peak": score_peak, "unit": "TFLOP/s", "frac": score_tflops / score_peak,
            "traffic": None,
        },
    }
    if turn2 is not None:
        res["detail"]["turn2"] = turn2
    if freq_detail is not None:
        res["detail"]["frequency_policy"] = freq_detail
    if ragged is not None:
        res["detail"]["ragged_decode"] = ragged
    if folded is not None:
        res["detail"]["decode_layers_folded"] = folded
    if not args.no_cpu_baseline:
        print("[bench] timing the CPU oracle on a bounded sample", file=sys.stderr, flush=True)
        res["cpu_baseline"] = cpu_baseline(cfg, wl, wl.G)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
