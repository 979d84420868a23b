#!/usr/bin/env python3
"""Benchmark of the SQAP-VLA hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input of
the batched-prefill workload (16 observations x 276 tokens, each pruned to
128 + 20 = 148 tokens, M = 2368):

    prune_rows (top-k + kept rows) -> quantize_act (gather fused) -> W4A4 gate/up
    linear (4096 -> 11008) -> quantize_act (K = 11008) -> W4A4 down linear
    (11008 -> 4096)

Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
`value` is 2*M*N*K of the two linears divided by the whole step time (TOPS).
`roofline` is for the prefill GEMM kernel (int8 MFMA bound), timed with HIP
events recorded on the launch stream around its launches.  `decode` reports the
small-M path over the 32-layer stack + lm_head (HBM bound), with its own
roofline object.  `cpu_baseline` times the CPU oracle on the same step.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5033.0      # 8192 op/clk/CU x 256 CU x 2.4 GHz (dense), = 5.0 POP/s
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-layers", action="store_true")
    ap.add_argument("--no-variants", action="store_true", help="skip the cold-weight / rotated / outlier-free GEMM timings")
    ap.add_argument("--only", default="", help="prefill|decode|decoder|calib: run just that loop --steps times (for profilers)")
    return ap.parse_args()


def quantize_and_pack(torch, B, W, flags=0):
    N, K = W.shape
    Wq = torch.empty((N, K // 2), dtype=torch.uint8, device=W.device)
    sw = torch.empty((N,), dtype=torch.float16, device=W.device)
    B.sqap_quantize_weight(W, Wq, sw, flags)
    h = B.sqap_weight_pack(Wq, sw)
    torch.cuda.synchronize()
    return h


class Prefill:
    """Configuration 3 resident on the GPU."""

    def __init__(self, torch, B, wl, dev, variant="workload"):
        """variant: "workload" (1 % outlier channels x30, no rotation: the configuration as defined), "rotated"
        (same inputs, quantized with the Hadamard rotation: codes spread over the whole 4-bit range) or
        "outlier_free" (plain N(0,1) inputs).  The GEMM's work is the same; its power draw, hence its clock, is not."""
        c = wl.CONFIGS[3]
        self.torch, self.B = torch, B
        self.flags = B.ROTATE_HADAMARD if variant == "rotated" else 0
        frac = 0.0 if variant == "outlier_free" else 0.01
        self.batch, self.keep = c["batch"], c["keep_k"]
        self.S, self.nv = wl.SEQ_LEN, wl.N_VISUAL
        self.M = self.batch * (self.keep + wl.N_TEXT)
        H, F = wl.HIDDEN, wl.FFN
        self.H, self.F = H, F
        t = lambda a: torch.from_numpy(a).to(dev)
        self.scores = t(wl.scores(self.batch, self.nv, wl.rng_for(3, 0, wl.T_SCORES)))
        self.X = t(wl.layer_input(3, 0, 4, self.batch * self.S, outlier_frac=frac))   # gate/up input, all tokens
        self.Xd = t(wl.layer_input(3, 0, 6, self.M, outlier_frac=frac))                # down input, kept tokens
        self.W_gate = quantize_and_pack(torch, B, t(wl.layer_weight(3, 0, 4)), self.flags)
        self.W_down = quantize_and_pack(torch, B, t(wl.layer_weight(3, 0, 6)), self.flags)
        self.cold = None                 # list of (W_gate, W_down) used in turn: see make_cold_weights
        i32, u8, f16 = torch.int32, torch.uint8, torch.float16
        self.idx = torch.empty((self.batch, self.keep), dtype=i32, device=dev)
        self.rows = torch.empty((self.M,), dtype=i32, device=dev)
        self.Xq = torch.empty((self.M, H // 2), dtype=u8, device=dev)
        self.sx = torch.empty((self.M,), dtype=f16, device=dev)
        self.Xdq = torch.empty((self.M, F // 2), dtype=u8, device=dev)
        self.sxd = torch.empty((self.M,), dtype=f16, device=dev)
        self.Yg = torch.empty((self.M, F), dtype=f16, device=dev)
        self.Yd = torch.empty((self.M, H), dtype=f16, device=dev)
        nws = max(B.sqap_workspace_bytes(self.M, F, H), B.sqap_workspace_bytes(self.M, H, F), 256)
        self.ws = torch.zeros((nws,), dtype=u8, device=dev)
        self.ops = 2.0 * self.M * (F * H + H * F)
        self.gemm_events = None

    def make_cold_weights(self, wl, total_bytes=1.1e9):
        """Distinct weight pairs summing to more than a gigabyte (the last-level cache holds 256 MB), used in
        turn by step(): every launch then streams its weights from HBM."""
        torch, B = self.torch, self.B
        g = torch.Generator(device=self.X.device)
        g.manual_seed(wl.BASE_SEED + 3)
        per_pair = self.F * self.H          # two weights of F x H codes, half a byte each
        self.cold, self.turn = [], 0
        for _ in range(int(total_bytes // per_pair) + 1):
            mk = lambda N, K: quantize_and_pack(torch, B, (torch.randn((N, K), generator=g, device=self.X.device,
                                                                       dtype=torch.float32) * 0.02).half())
            self.cold.append((mk(self.F, self.H), mk(self.H, self.F)))

    def step(self):
        B, ev = self.B, self.gemm_events
        Wg, Wd = self.W_gate, self.W_down
        if self.cold:
            Wg, Wd = self.cold[self.turn % len(self.cold)]
            self.turn += 1
        B.sqap_prune_rows(self.scores, self.keep, self.S, 0, self.idx, self.rows)
        B.sqap_quantize_act(self.X, self.rows, self.Xq, self.sx, flags=self.flags)
        if ev is not None:
            ev[0].record()
        B.sqap_w4a4_linear(self.Xq, self.sx, Wg, self.Yg, None, self.ws)
        if ev is not None:
            ev[1].record()
        B.sqap_quantize_act(self.Xd, None, self.Xdq, self.sxd, flags=self.flags)
        if ev is not None:
            ev[2].record()
        B.sqap_w4a4_linear(self.Xdq, self.sxd, Wd, self.Yd, None, self.ws)
        if ev is not None:
            ev[3].record()

    def free(self):
        for w in [self.W_gate, self.W_down] + [w for pair in (self.cold or []) for w in pair]:
            w.free()


def time_gemm_launches(torch, wk, steps):
    """Duration of the prefill GEMM launches, from HIP events recorded on the launch stream directly around
    each linear call inside whole steps that run back to back (no synchronisation between the steps, as
    in the timed region; one at the end).  Returns (mean ms per launch, per-GEMM mean ms, stats in us)."""
    all_ev = []
    for _ in range(steps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        wk.gemm_events = ev
        wk.step()
        all_ev.append(ev)
    wk.gemm_events = None
    torch.cuda.synchronize()
    gate = [ev[0].elapsed_time(ev[1]) for ev in all_ev]
    down = [ev[2].elapsed_time(ev[3]) for ev in all_ev]
    both = sorted(gate + down)
    stats = {"mean": 1e3 * sum(both) / len(both), "median": 1e3 * both[len(both) // 2], "min": 1e3 * both[0],
             "max": 1e3 * both[-1], "launches": len(both)}
    return sum(both) / len(both), {"gate_up": sum(gate) / steps, "down": sum(down) / steps}, stats


def settle_clocks(torch, wk, max_steps=300, window=25, tol=0.01):
    """Untimed pre-warm, whatever --warmup says: the first dozens of launches after an idle period run 5-10 %
    slower (clocks and power management settle).  Runs whole steps in windows of `window` until the mean
    step time of two consecutive windows differs by less than `tol`, or max_steps have run."""
    prev, done, ms = None, 0, 0.0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    while done < max_steps:
        e0.record()
        for _ in range(window):
            wk.step()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / window
        done += window
        if prev is not None and abs(ms - prev) <= tol * prev:
            break
        prev = ms
    return {"steps": done, "last_window_us_per_step": ms * 1e3}


def read_sclk_mhz():
    """Current shader clock of the first GPU that reports one (sysfs pp_dpm_sclk, the starred level), or None."""
    import glob
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
        try:
            for line in open(path):
                if "*" in line:
                    return int(line.split(":")[1].strip().lower().replace("mhz", "").replace("*", "").strip())
        except (OSError, ValueError, IndexError):
            continue
    return None


def sclk_under_load(torch, wk, steps=150):
    """Shader clock read from the host while `steps` steps are in flight on the GPU (launches are asynchronous)."""
    for _ in range(steps):
        wk.step()
    mhz = read_sclk_mhz()
    torch.cuda.synchronize()
    return mhz


class Stack:
    """The 32-layer linear stack + lm_head as packed W4 weights (3.30 GB), from a seeded
    GPU generator (host generation of 6.6 G normals would take minutes)."""

    def __init__(self, torch, B, wl, dev, layers=None):
        self.torch, self.B, self.wl, self.dev = torch, B, wl, dev
        g = torch.Generator(device=dev)
        g.manual_seed(wl.BASE_SEED)
        self.g = g
        self.layers = wl.N_LAYERS if layers is None else layers
        self.weights = []
        for _ in range(self.layers):
            row = []
            for (_, N, K) in wl.LAYER_LINEARS:
                W = (torch.randn((N, K), generator=g, device=dev, dtype=torch.float32) * 0.02).half()
                row.append(quantize_and_pack(torch, B, W))
                del W
            self.weights.append(row)
        _, V, Hd = wl.LM_HEAD
        W = (torch.randn((V, Hd), generator=g, device=dev, dtype=torch.float32) * 0.02).half()
        self.lm_head = quantize_and_pack(torch, B, W)
        del W
        self.weight_bytes = self.layers * sum(N * K // 2 for (_, N, K) in wl.LAYER_LINEARS) + V * Hd // 2
        self.scale_bytes = 2 * (self.layers * sum(N for (_, N, K) in wl.LAYER_LINEARS) + V)

    def activation(self, M, K):
        """Quantized [M, K] input: N(0,1) with 1 % outlier channels x30 (fixed channels)."""
        torch, B, wl = self.torch, self.B, self.wl
        x = torch.randn((M, K), generator=self.g, device=self.dev, dtype=torch.float32)
        ch = torch.randperm(K, generator=self.g, device=self.dev)[: wl.n_outliers_for(K)]
        x[:, ch] *= 30.0
        x = x.half()
        Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=self.dev)
        sx = torch.empty((M,), dtype=torch.float16, device=self.dev)
        B.sqap_quantize_act(x, None, Xq, sx)
        return Xq, sx


def decode_leg(torch, B, wl, stack, steps_per_m=7):
    """Configuration 4: M in {1, 8} through every linear of the stack + lm_head.  Each linear
    has its own input (the workload has no glue between linears), so a whole step is one
    group launch; the dependency-respecting variant (4 launches per layer) is timed too."""
    out = {}
    dev = stack.dev
    H, F = wl.HIDDEN, wl.FFN
    for M in (1, 2, 4, 8):
        xq_h = [stack.activation(M, H) for _ in range(3)]      # qkv input, o input, gate/up input
        xq_f = stack.activation(M, F)
        problems, levels = [], []
        for l in range(stack.layers):
            ys = []
            for i, (name, N, K) in enumerate(wl.LAYER_LINEARS):
                src = xq_f if K == F else (xq_h[0] if i < 3 else xq_h[1] if i == 3 else xq_h[2])
                Y = torch.empty((M, N), dtype=torch.float16, device=dev)
                ys.append((src[0], src[1], stack.weights[l][i], Y))
            problems += ys
            levels += [ys[0:3], ys[3:4], ys[4:6], ys[6:7]]
        _, V, _ = wl.LM_HEAD
        lm = (xq_h[0][0], xq_h[0][1], stack.lm_head, torch.empty((M, V), dtype=torch.float16, device=dev))
        problems.append(lm)
        levels.append([lm])
        whole = B.sqap_group_create(problems)
        per_level = [B.sqap_group_create(lv) for lv in levels]

        def timed(fn):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps_per_m):            # 7 sequential action tokens
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / steps_per_m

        ms_whole = timed(whole.run)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for gq in per_level:
                gq.run()
        ms_levels = timed(graph.replay)
        alg_bytes = stack.weight_bytes + stack.scale_bytes + M * sum(
            K // 2 + 2 * N for (_, N, K) in wl.LAYER_LINEARS) * stack.layers
        out["M%d" % M] = {
            "us_per_step": ms_whole * 1e3, "GBps": alg_bytes / (ms_whole * 1e-3) / 1e9,
            "frac_of_hbm_peak": alg_bytes / (ms_whole * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "launches": 1,
            "per_level": {"launches": len(per_level), "us_per_step": ms_levels * 1e3,
                          "GBps": alg_bytes / (ms_levels * 1e-3) / 1e9},
        }
        whole.free()
        for gq in per_level:
            gq.free()
    # Two formulations of a step.  "whole_group": the 225 linears as independent problems in ONE launch (the
    # workload definition has no glue between linears, so this is permitted, but no token generation could
    # issue it: layer l + 1 consumes layer l's output): the ceiling of the weight stream.  "per_level": the
    # linears that may run together (q|k|v, o, gate|up, down, head) as one launch each, in order: what a decode
    # step's dependencies allow.  The roofline object is for the second; the first is kept beside it.
    alg = stack.weight_bytes + stack.scale_bytes
    dep, ceil_ = out["M1"]["per_level"], out["M1"]
    out["roofline"] = {"bound": "hbm", "kernel": "skinny_kernel<S, 8> (129 launches per step, replayed from a HIP graph)",
                       "formulation": "dependency-respecting: one launch per group of linears that can run together",
                       "achieved": dep["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dep["GBps"] / HBM_PEAK_GBS,
                       "target_frac": 0.70, "traffic": None, "algorithmic_bytes_per_step": alg}
    out["weight_stream_ceiling"] = {"kernel": "skinny_kernel<1, 16>", "formulation": "all 225 linears as independent "
                                    "problems in one launch (no dependencies: not a decode step)",
                                    "achieved": ceil_["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": ceil_["GBps"] / HBM_PEAK_GBS, "traffic": None,
                                    "algorithmic_bytes_per_launch": alg}
    out["weights_GB"] = stack.weight_bytes / 1e9
    return out


def layer_leg(torch, B, wl, stack):
    """Configurations 1 and 2: per-layer latency of the 7 linears at M = 148 (one layer) and the
    32-layer stack at M = 276 for 2 layers then M = 84; one launch per linear, distinct weights."""
    dev = stack.dev
    H, F = wl.HIDDEN, wl.FFN
    res = {}

    def run_layers(M, layer_ids):
        xh, xf = stack.activation(M, H), stack.activation(M, F)
        ys = {N: torch.empty((M, N), dtype=torch.float16, device=dev) for N in (H, F)}
        nws = max([B.sqap_workspace_bytes(M, N, K) for (_, N, K) in wl.LAYER_LINEARS] + [256])
        ws = torch.zeros((nws,), dtype=torch.uint8, device=dev)

        def go():
            for l in layer_ids:
                for i, (_, N, K) in enumerate(wl.LAYER_LINEARS):
                    x = xf if K == F else xh
                    B.sqap_w4a4_linear(x[0], x[1], stack.weights[l][i], ys[N], None, ws)
        go()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 3
        e0.record()
        for _ in range(reps):
            go()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3        # us for all the listed layers

    n = stack.layers
    ops_layer = lambda M: 2.0 * M * sum(N * K for (_, N, K) in wl.LAYER_LINEARS)
    us148 = run_layers(148, range(n)) / n
    res["cfg1_M148"] = {"us_per_layer": us148, "TOPS": ops_layer(148) / us148 / 1e6,
                        "floor_us": 14.6, "note": "average over %d distinct layers (no cache reuse)" % n}
    us276 = run_layers(276, range(min(2, n))) / min(2, n)
    us84 = run_layers(84, range(min(2, n), n)) / max(1, n - 2)
    total = 2 * us276 + 30 * us84
    res["cfg2_stack"] = {"us_per_layer_M276": us276, "us_per_layer_M84": us84, "us_total_32_layers": total,
                         "floor_us": 456.0, "TOPS": (2 * ops_layer(276) + 30 * ops_layer(84)) / total / 1e6}

    # the vocabulary head (4096 -> 32000) at the stack's two token counts
    for M in (84, 276):
        xh = stack.activation(M, H)
        yv = torch.empty((M, wl.LM_HEAD[1]), dtype=torch.float16, device=dev)
        wsv = torch.zeros((max(B.sqap_workspace_bytes(M, wl.LM_HEAD[1], H), 256),), dtype=torch.uint8, device=dev)
        res["cfg2_stack"]["us_lm_head_M%d" % M] = graph_time_us(
            torch, lambda: B.sqap_w4a4_linear(xh[0], xh[1], stack.lm_head, yv, None, wsv), 20)

    # pruning-ratio sweep on the same layers: 256 visual tokens pruned by 0.3 .. 0.6, plus 20 text tokens
    few = range(min(4, n))
    res["ratio_sweep"] = {"M%d" % M: run_layers(M, few) / len(few) for M in (199, 174, 148, 122)}
    res["ratio_sweep"]["note"] = "us per layer (7 launches), pruning ratio 0.3 / 0.4 / 0.5 / 0.6 of 256 visual tokens"

    # the same layer with q/k/v and gate/up packed as single weights: 4 launches instead of 7
    g = stack.g
    mk = lambda N, K: quantize_and_pack(torch, B, (torch.randn((N, K), generator=g, device=dev,
                                                               dtype=torch.float32) * 0.02).half())
    fused = [[mk(3 * H, H), mk(H, H), mk(2 * F, H), mk(H, F)] for _ in few]
    shapes = [(3 * H, H), (H, H), (2 * F, H), (H, F)]
    M = 148
    xh, xf = stack.activation(M, H), stack.activation(M, F)
    ys = [torch.empty((M, N), dtype=torch.float16, device=dev) for (N, _) in shapes]
    nws = max([B.sqap_workspace_bytes(M, N, K) for (N, K) in shapes] + [256])
    ws = torch.zeros((nws,), dtype=torch.uint8, device=dev)

    def go_fused():
        for row in fused:
            for i, (N, K) in enumerate(shapes):
                x = xf if K == F else xh
                B.sqap_w4a4_linear(x[0], x[1], row[i], ys[i], None, ws)
    go_fused()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        go_fused()
    e1.record()
    torch.cuda.synchronize()
    res["cfg1_M148"]["us_per_layer_fused_qkv_gateup"] = e0.elapsed_time(e1) / 3 * 1e3 / len(fused)
    for row in fused:
        for w in row:
            w.free()
    return res


def decoder_leg(torch, B, wl, dev, distinct_layers=8):
    """Configuration 2 as a real forward: 32 Llama-2-7B-shaped layers at batch 1 (RMSNorm, fused q|k|v,
    rotary embedding, causal attention, o, RMSNorm, fused gate|up, SwiGLU, down, residuals; every linear
    W4A4), 276 tokens for two layers, then the retention score of the last text token from that layer's
    own rotated queries and keys, top-k 256 -> 64 visual tokens, and 84 tokens for the other 30 layers.
    Weights: 8 distinct random layers used in turn (0.8 GB, more than the caches hold)."""
    from paper_2509_09090_amd import decoder
    H, F, nh, hd = wl.HIDDEN, wl.FFN, wl.N_HEADS, wl.HEAD_DIM
    S, nv, keep = wl.SEQ_LEN, wl.N_VISUAL, 64
    Mk = S - nv + keep
    g = torch.Generator(device=dev)
    g.manual_seed(wl.BASE_SEED + 2)
    mk = lambda N, K: quantize_and_pack(torch, B, (torch.randn((N, K), generator=g, device=dev,
                                                               dtype=torch.float32) * 0.02).half())
    gain = lambda: (1 + 0.1 * torch.randn((H,), generator=g, device=dev, dtype=torch.float32)).half()
    layers = [decoder.LayerWeights(mk(3 * H, H), mk(H, H), mk(2 * F, H), mk(H, F), gain(), gain())
              for _ in range(distinct_layers)]
    buf = decoder.LayerBuffers(S, H, F, device=dev)
    x0 = torch.randn((S, H), generator=g, device=dev, dtype=torch.float32)
    ch = torch.randperm(H, generator=g, device=dev)[: wl.n_outliers_for(H)]
    x0[:, ch] *= 30.0
    x0 = x0.half()
    x = torch.empty_like(x0)
    xa, xb = torch.empty((S, H), dtype=torch.float16, device=dev), torch.empty((S, H), dtype=torch.float16, device=dev)
    da, db = torch.empty_like(xa), torch.empty_like(xa)
    pos_full = torch.arange(S, dtype=torch.int32, device=dev)
    kdense = torch.empty((S, H), dtype=torch.float16, device=dev)
    scores = torch.empty((1, nv), dtype=torch.float32, device=dev)
    score_ws = torch.zeros((B.sqap_attn_scores_workspace_bytes(1, S, nh, hd, nv),), dtype=torch.uint8, device=dev)
    idx = torch.empty((1, keep), dtype=torch.int32, device=dev)
    rows = torch.empty((Mk,), dtype=torch.int32, device=dev)

    def forward():
        x.copy_(x0)
        # layers 0, 1 on the full sequence
        decoder.layer_forward(layers[0], buf, x, None, pos_full, 1, nh, hd, xa, da)
        decoder.layer_forward(layers[1 % distinct_layers], buf, xa, da, pos_full, 1, nh, hd, xb, db)
        # retention score of the last (text) token from this layer's rotated q and k, then the kept rows
        B.sqap_gather_rows(buf.qkv[:S, H:2 * H], pos_full, kdense)
        B.sqap_attn_scores(buf.qkv[S - 1, :H], kdense.view(S, nh, hd), 0, nv, scores[0], score_ws)
        B.sqap_prune_rows(scores, keep, S, 0, idx, rows)
        B.sqap_residual_add(xb, db)                       # the pending update lands before the gather
        src, pend, use_rows, pos = xb, None, rows, rows
        outs = ((xa[:Mk], da[:Mk]), (xb[:Mk], db[:Mk]))
        for l in range(2, wl.N_LAYERS):
            xo, do = outs[l & 1]
            if use_rows is not None:                      # first pruned layer: gather fused into its first call
                xo, do = xa[:Mk], da[:Mk]
            decoder.layer_forward(layers[l % distinct_layers], buf, src, pend, pos, 1, nh, hd, xo, do, rows=use_rows)
            src, pend, use_rows = xo, do, None
        B.sqap_residual_add(src, pend)
        return src

    forward()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 3
    e0.record()
    for _ in range(reps):
        forward()
    e1.record()
    torch.cuda.synchronize()
    eager_us = e0.elapsed_time(e1) / reps * 1e3
    res = {"us_forward_eager": eager_us, "launches": 2 * 10 + 4 + 30 * 10 + 2,
           "note": "32 layers, 276 tokens for 2 layers then 84; includes the pruning step"}
    # the same forward replayed from a HIP graph (no host launch cost)
    try:
        sidestream = torch.cuda.Stream()
        sidestream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(sidestream):
            forward()
        torch.cuda.current_stream().wait_stream(sidestream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            out_ref = forward()
        graph.replay()
        torch.cuda.synchronize()
        first = out_ref.clone()
        e0.record()
        for _ in range(reps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        res["us_forward_graph"] = e0.elapsed_time(e1) / reps * 1e3
        eager_out = forward().clone()
        torch.cuda.synchronize()
        res["graph_matches_eager"] = bool(torch.equal(first, eager_out) and torch.equal(out_ref, eager_out))
    except Exception as exc:                              # report, never hide: the eager number stands on its own
        res["graph_error"] = repr(exc)[:200]
    ops = lambda M: 2.0 * M * (3 * H * H + H * H + 2 * F * H + H * F)
    total_ops = 2 * ops(S) + 30 * ops(Mk)
    res["TOPS_eager"] = total_ops / eager_us / 1e6
    res["decode"] = decode_forward_leg(torch, B, wl, dev, layers, buf, g)
    # one layer at configuration 3's batch: 16 observations x 148 tokens = 2368 rows
    nb, Sp = 16, 148
    big = decoder.LayerBuffers(nb * Sp, H, F, device=dev)
    xb3 = torch.randn((nb * Sp, H), generator=g, device=dev, dtype=torch.float32).half()
    pend3 = torch.randn((nb * Sp, H), generator=g, device=dev, dtype=torch.float32).half()
    pos3 = torch.arange(Sp, dtype=torch.int32, device=dev).repeat(nb)
    xo3, do3 = torch.empty_like(xb3), torch.empty_like(xb3)
    res["us_layer_cfg3_batch16"] = graph_time_us(
        torch, lambda: decoder.layer_forward(layers[0], big, xb3, pend3, pos3, nb, nh, hd, xo3, do3), 10, per_graph=2)
    del big
    for lw in layers:
        lw.free()
    return res


def decode_forward_leg(torch, B, wl, dev, layers, buf, g, prefix=148, new_tokens=7):
    """Configuration 4 as a real decode: the 148 pruned tokens are prefilled into per-layer key/value caches,
    then action tokens are generated one at a time at batch 1: 32 layers (norm, q|k|v, rotary + cache append,
    attention over the cache, o, norm, gate|up, SwiGLU, down; every linear W4A4 through the small-M kernel),
    final norm and the 4096 -> 32000 head.  Time per generated token."""
    from paper_2509_09090_amd import decoder
    H, F, nh, hd, V = wl.HIDDEN, wl.FFN, wl.N_HEADS, wl.HEAD_DIM, wl.LM_HEAD[1]
    nl, nd = wl.N_LAYERS, len(layers)
    head = quantize_and_pack(torch, B, (torch.randn((V, H), generator=g, device=dev, dtype=torch.float32) * 0.02).half())
    gamma_f = (1 + 0.1 * torch.randn((H,), generator=g, device=dev, dtype=torch.float32)).half()
    caches = [torch.zeros((prefix + new_tokens, 2 * H), dtype=torch.float16, device=dev) for _ in range(nl)]
    x0 = torch.randn((prefix, H), generator=g, device=dev, dtype=torch.float32).half()
    pos = torch.arange(prefix, dtype=torch.int32, device=dev)
    xa, xb = (torch.empty((prefix, H), dtype=torch.float16, device=dev) for _ in range(2))
    da, db = (torch.empty((prefix, H), dtype=torch.float16, device=dev) for _ in range(2))
    src, pend = x0, None
    for l in range(nl):                                  # prefill (not timed): fills the caches
        xo, do = (xa, da) if l % 2 == 0 else (xb, db)
        decoder.layer_forward(layers[l % nd], buf, src, pend, pos, 1, nh, hd, xo, do, kv=caches[l], past=0)
        src, pend = xo, do
    tok = torch.randn((1, H), generator=g, device=dev, dtype=torch.float32).half()
    logits = torch.empty((1, V), dtype=torch.float16, device=dev)
    x1a, x1b, d1a, d1b = (torch.empty((1, H), dtype=torch.float16, device=dev) for _ in range(4))
    p1 = [torch.tensor([prefix + i], dtype=torch.int32, device=dev) for i in range(new_tokens)]

    def step(i):
        src, pend = tok, None
        for l in range(nl):
            xo, do = (x1a, d1a) if l % 2 == 0 else (x1b, d1b)
            decoder.layer_forward(layers[l % nd], buf, src, pend, p1[i], 1, nh, hd, xo, do, kv=caches[l], past=prefix + i)
            src, pend = xo, do
        B.sqap_rmsnorm_quantize_act(src, None, gamma_f, 1e-5, buf.xq[:1], buf.sx[:1], delta=pend)
        B.sqap_w4a4_linear(buf.xq[:1], buf.sx[:1], head, logits, None, buf.ws)

    def generate():
        for i in range(new_tokens):
            step(i)

    generate()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        generate()
    e1.record()
    torch.cuda.synchronize()
    us_eager = e0.elapsed_time(e1) * 1e3 / (3 * new_tokens)
    res = {"us_per_token_eager": us_eager, "launches_per_token": nl * 9 + 2, "prefix": prefix,
           "new_tokens": new_tokens}
    try:
        res["us_per_token_graph"] = graph_time_us(torch, generate, 3, per_graph=1) / new_tokens
    except Exception as exc:
        res["graph_error"] = repr(exc)[:200]
    weight_bytes = nl * (3 * H * H + H * H + 2 * F * H + H * F) // 2 + V * H // 2
    res["GBps_weights_graph"] = weight_bytes / res.get("us_per_token_graph", us_eager) / 1e3
    res["formulation"] = "chain of launches (nine per layer): every dependency of a real decode step"
    chain_logits = logits.clone()                         # of the last token generated above
    # The same step as ONE persistent launch (sqap_decoder_step): same caches, same weights, same token.
    dec = B.sqap_decoder_create([(layers[l % nd].qkv, layers[l % nd].o, layers[l % nd].gate_up, layers[l % nd].down,
                                  layers[l % nd].gamma_attn, layers[l % nd].gamma_mlp, caches[l]) for l in range(nl)],
                                nh, hd, gamma_f, head)
    logits1 = torch.empty((V,), dtype=torch.float16, device=dev)

    def generate1():
        for i in range(new_tokens):
            dec.step(tok[0], p1[i], prefix + i, logits1)

    generate1()
    torch.cuda.synchronize()
    one = {"launches_per_token": 1, "status": dec.status(),
           "logits_equal_chain": bool(torch.equal(logits1.view(torch.int16), chain_logits[0].view(torch.int16)))}
    e0.record()
    for _ in range(3):
        generate1()
    e1.record()
    torch.cuda.synchronize()
    one["us_per_token_eager"] = e0.elapsed_time(e1) * 1e3 / (3 * new_tokens)
    try:
        one["us_per_token_graph"] = graph_time_us(torch, generate1, 3, per_graph=1) / new_tokens
    except Exception as exc:
        one["graph_error"] = repr(exc)[:200]
    us1 = min(one["us_per_token_eager"], one.get("us_per_token_graph", float("inf")))
    one["status_after"] = dec.status()
    one["GBps_weights"] = weight_bytes / us1 / 1e3
    one["frac_of_hbm_peak"] = one["GBps_weights"] / HBM_PEAK_GBS
    one["weight_bytes_per_token"] = weight_bytes
    one["formulation"] = ("one persistent launch per token (decoder_step_kernel): every dependency of a real decode step, "
                          "rows between the linears handed from workgroup to workgroup inside the launch")
    res["step_kernel"] = one
    dec.free()
    head.free()
    return res


def selection_leg(torch, B, wl, dev, iters=50):
    """The full selection rule (top-k + projected ring + farthest point sampling) at configuration 3's
    batch: 16 observations of a 16 x 16 token grid, 64 attention tokens, ring radius 2, 128 kept."""
    batch, gw, gh, k_attn, total, radius = 16, 16, 16, 64, 128, 2
    s = torch.from_numpy(wl.scores(batch, gw * gh, wl.rng_for(3, 0, wl.T_SCORES))).to(dev)
    cam = torch.from_numpy(wl.cameras(batch, gw, gh, 14.0, wl.rng_for(3, 0, wl.T_CAMERA))).to(dev)
    idx = torch.empty((batch, total + (2 * radius + 1) ** 2), dtype=torch.int32, device=dev)
    cnt = torch.empty((batch,), dtype=torch.int32, device=dev)
    us = graph_time_us(torch, lambda: B.sqap_prune_select(s, gw, gh, k_attn, total, cam, radius, idx, cnt), iters)
    return {"us_per_call": us, "batch": batch, "grid": [gw, gh], "k_attn": k_attn, "keep_total": total,
            "ring_radius": radius, "note": "GPU time, back-to-back launches replayed from a HIP graph"}


def graph_time_us(torch, fn, iters, per_graph=10):
    """Microseconds of GPU time per call of fn: per_graph calls captured into a HIP graph and replayed, so
    that the host's launch cost (several microseconds per call through Python) does not count."""
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(per_graph):
            fn()
    graph.replay()
    torch.cuda.synchronize()
    reps = max(1, iters // per_graph)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (reps * per_graph)


def prefill_variants(torch, B, wl, dev, wk, steps=60):
    """The two prefill GEMMs timed again (HIP events around each launch, back-to-back steps, clocks settled
    first) with cold weights and with other input data: the work is the same, the power draw and so the
    clock are not."""
    res = {}

    def measure(w):
        settle_clocks(torch, w, max_steps=150)
        ms, per, st = time_gemm_launches(torch, w, steps)
        return {"avg_launch_us": ms * 1e3, "median_us": st["median"], "min_us": st["min"],
                "gate_up_us": per["gate_up"] * 1e3, "down_us": per["down"] * 1e3,
                "TOPs": wk.ops / 2.0 / (ms * 1e-3) / 1e12, "sclk_mhz_under_load": sclk_under_load(torch, w, 100)}

    wk.make_cold_weights(wl)
    res["cold_weights"] = measure(wk)
    res["cold_weights"]["note"] = "%d distinct weight pairs (%.2f GB) used in turn: every launch streams its weights " \
                                  "from HBM" % (len(wk.cold), len(wk.cold) * wk.F * wk.H / 1e9)
    for pair in wk.cold:
        for w in pair:
            w.free()
    wk.cold = None
    for variant in ("rotated", "outlier_free"):
        w = Prefill(torch, B, wl, dev, variant)
        res[variant] = measure(w)
        w.free()
        del w
    res["note"] = "rotated: activations and weights rotated (Eq. 6) before quantization; outlier_free: N(0,1) inputs"
    return res


def small_kernel_leg(torch, B, wl, wk, dev, iters=50):
    """Microseconds per call of the selection and quantization kernels at configuration 3's sizes
    (back-to-back launches on one stream, HIP events around the run)."""
    def timed(fn):
        return graph_time_us(torch, fn, iters)

    q, k = wl.query_and_keys(wl.SEQ_LEN, wl.N_HEADS, wl.HEAD_DIM, wl.rng_for(3, 2, wl.T_Q))
    q, k = torch.from_numpy(q).to(dev), torch.from_numpy(k).to(dev)
    a_q = torch.empty((wl.N_VISUAL,), dtype=torch.float32, device=dev)
    gathered = torch.empty((wk.M, wk.H), dtype=torch.float16, device=dev)
    nb = 16
    qb = q.unsqueeze(0).repeat(nb, 1, 1).contiguous()
    kb = k.unsqueeze(0).repeat(nb, 1, 1, 1).contiguous()
    a_qb = torch.empty((nb, wl.N_VISUAL), dtype=torch.float32, device=dev)
    ws_a = torch.zeros((B.sqap_attn_scores_workspace_bytes(nb, wl.SEQ_LEN, wl.N_HEADS, wl.HEAD_DIM, wl.N_VISUAL),),
                       dtype=torch.uint8, device=dev)
    out = {
        "attn_scores_S276_H32_d128": timed(lambda: B.sqap_attn_scores(q, k, 0, wl.N_VISUAL, a_q, ws_a)),
        "attn_scores_batch16_S276_H32_d128": timed(lambda: B.sqap_attn_scores_batch(qb, kb, 0, wl.N_VISUAL, a_qb, ws_a)),
        "prune_rows_16x256_to_128": timed(lambda: B.sqap_prune_rows(wk.scores, wk.keep, wk.S, 0, wk.idx, wk.rows)),
        "gather_rows_2368x4096": timed(lambda: B.sqap_gather_rows(wk.X, wk.rows, gathered)),
        "quantize_act_2368x4096_fused_gather": timed(lambda: B.sqap_quantize_act(wk.X, wk.rows, wk.Xq, wk.sx)),
        "quantize_act_2368x11008": timed(lambda: B.sqap_quantize_act(wk.Xd, None, wk.Xdq, wk.sxd)),
        "quantize_act_2368x4096_rotated": timed(
            lambda: B.sqap_quantize_act(wk.X, wk.rows, wk.Xq, wk.sx, flags=B.ROTATE_HADAMARD)),
    }
    # algorithmic bytes: 2 B read + 0.5 B written per element (+ scales)
    for name, (rows_, cols) in (("quantize_act_2368x4096_fused_gather", (wk.M, wk.H)),
                                ("quantize_act_2368x11008", (wk.M, wk.F))):
        out[name + "_GBps"] = rows_ * cols * 2.5 / out[name] / 1e3
    out["note"] = "us of GPU time per call, back-to-back launches replayed from a HIP graph"
    return out


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return None


def cpu_baseline(wl, timed_outputs=None, n_samples=4000):
    """The oracle, as it stands, on the same step (all 16 observations), all host threads; the same on one
    observation's share with one thread; and, when the GPU's outputs of the timed buffers are given
    (Yg, Yd as numpy arrays copied back after the timed region), a comparison of sampled outputs with
    what the oracle computes for them one by one (bit equality of the fp16 values)."""
    import ctypes
    import numpy as np
    import oracle
    H, F, S, nv = wl.HIDDEN, wl.FFN, wl.SEQ_LEN, wl.N_VISUAL
    keep, batch = wl.CONFIGS[3]["keep_k"], wl.CONFIGS[3]["batch"]
    M = batch * (keep + wl.N_TEXT)
    scores = wl.scores(batch, nv, wl.rng_for(3, 0, wl.T_SCORES))
    X = wl.layer_input(3, 0, 4, batch * S)
    Xd = wl.layer_input(3, 0, 6, M)
    Wg, sg, _ = oracle.quantize_rows(wl.layer_weight(3, 0, 4))       # offline step, not timed
    Wd, sd, _ = oracle.quantize_rows(wl.layer_weight(3, 0, 6))
    t0 = time.perf_counter()
    idx = oracle.prune_topk(scores, keep)
    rows = oracle.kept_rows(idx, S, 0, nv)
    Xq, sx, _ = oracle.quantize_rows(X, rows=rows)
    oracle.w4a4_linear(Xq, sx, Wg, sg)
    Xdq, sxd, _ = oracle.quantize_rows(Xd)
    oracle.w4a4_linear(Xdq, sxd, Wd, sd)
    dt = time.perf_counter() - t0
    ops = 2.0 * M * (F * H + H * F)
    threads = ctypes.CDLL("libgomp.so.1").omp_get_max_threads()
    out = {"value": ops / dt / 1e12, "unit": "TOPS", "cores": int(threads), "kind": "oracle",
           "seconds": dt, "cpu_model": cpu_model(),
           "sample": "one whole step of the same workload (16 observations, M=%d): "
                     "prune, rows, quantize, gate/up, quantize, down" % M}
    # one thread, one observation's 148 kept rows (a sixteenth of the step)
    m1 = keep + wl.N_TEXT
    old = oracle.set_threads(1)
    t0 = time.perf_counter()
    i1 = oracle.prune_topk(scores[:1], keep)
    r1 = oracle.kept_rows(i1, S, 0, nv)
    q1, s1, _ = oracle.quantize_rows(X, rows=r1)
    oracle.w4a4_linear(q1, s1, Wg, sg)
    qd1, sd1, _ = oracle.quantize_rows(Xd[:m1])
    oracle.w4a4_linear(qd1, sd1, Wd, sd)
    dt1 = time.perf_counter() - t0
    oracle.set_threads(old)
    out["single_thread"] = {"value": 2.0 * m1 * (F * H + H * F) / dt1 / 1e12, "unit": "TOPS", "cores": 1,
                            "seconds": dt1, "sample": "one observation of the step (M=%d)" % m1}
    if timed_outputs is not None:
        Yg, Yd = timed_outputs
        rng = np.random.default_rng(12345)
        bad = 0
        for (Y, xq, s_x, wq, s_w) in ((Yg, Xq, sx, Wg, sg), (Yd, Xdq, sxd, Wd, sd)):
            ms = rng.integers(0, Y.shape[0], n_samples).astype(np.int32)
            ns = rng.integers(0, Y.shape[1], n_samples).astype(np.int32)
            ms[:4], ns[:4] = [0, Y.shape[0] - 1, 0, Y.shape[0] - 1], [0, 0, Y.shape[1] - 1, Y.shape[1] - 1]
            _, y_o = oracle.linear_samples(xq, s_x, wq, s_w, ms, ns)
            bad += int(np.count_nonzero(Y[ms, ns].view(np.uint16) != y_o.view(np.uint16)))
        out["parity_samples"] = 2 * n_samples
        out["parity_mismatches"] = bad
    return out


def stored_traffic(kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc (see profiles/); None if not recorded."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(kernel)
    except (OSError, ValueError):
        return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); no multi-GPU path exists",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2509_09090_amd import binding as B, workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.only == "calib":
        # plain copy of known size: reference reading for the FETCH_SIZE / WRITE_SIZE counters
        n = 1 << 30
        src = torch.ones((n,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        return
    if args.only == "decoder":
        print(json.dumps(decoder_leg(torch, B, wl, dev)))
        return
    if args.only == "decode":
        stack = Stack(torch, B, wl, dev)
        print(json.dumps(decode_leg(torch, B, wl, stack, steps_per_m=args.steps)))
        return

    wk = Prefill(torch, B, wl, dev)
    if args.only == "prefill":
        for _ in range(args.steps):
            wk.step()
        torch.cuda.synchronize()
        return

    B.sqap_init()
    settled = settle_clocks(torch, wk)
    for _ in range(args.warmup):
        wk.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wk.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    tops = wk.ops / (dt / args.steps) / 1e12

    gemm_ms, per_gemm, launch_stats = time_gemm_launches(torch, wk, args.steps)
    gemm_ops = wk.ops / 2.0                                  # each of the two launches: 2*M*N*K
    achieved = gemm_ops / (gemm_ms * 1e-3) / 1e12
    ws_error = B.workspace_error(wk.ws)
    timed_outputs = (wk.Yg.cpu().numpy(), wk.Yd.cpu().numpy())      # the buffers the timed region wrote
    sclk = sclk_under_load(torch, wk)

    out = {
        "metric": "W4A4 linear TOPS (prefill, pruned tokens) + decode GB/s, fraction of peak",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "configs[3]: batched prefill, 16 obs x 276 tokens pruned to 148, M=2368; "
                               "gate/up 4096->11008 and down 11008->4096, int4 codes widened to int8 MFMA",
                   "M": wk.M, "step": "prune_rows(top-k+kept rows)+quantize_act+linear+quantize_act+linear"},
        "roofline": {"bound": "mfma", "kernel": "gemm_streamk_kernel<Cfg<256,256,2,4>>", "achieved": achieved,
                     "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / INT8_MFMA_PEAK_TOPS,
                     "avg_launch_ms": gemm_ms, "per_gemm_ms": per_gemm, "launch_us": launch_stats,
                     "algorithmic_ops_per_launch": gemm_ops,
                     "traffic": stored_traffic("gemm_streamk_kernel"),
                     "sclk_mhz_under_load": sclk, "workspace_error_word": ws_error,
                     "operands": "warm: one layer's weights (45 MB) reused by every step"},
        "prewarm": settled,
    }
    if not args.no_variants:
        out["roofline"]["variants"] = prefill_variants(torch, B, wl, dev, wk)
    out["kernels_us"] = small_kernel_leg(torch, B, wl, wk, dev)
    del wk
    torch.cuda.empty_cache()
    if not (args.no_decode and args.no_layers):
        stack = Stack(torch, B, wl, dev)
        if not args.no_decode:
            out["decode"] = decode_leg(torch, B, wl, stack)
            out["decode"]["roofline"]["traffic"] = stored_traffic("skinny_kernel")
        if not args.no_layers:
            out["layers"] = layer_leg(torch, B, wl, stack)
        del stack
        torch.cuda.empty_cache()
    if not args.no_layers:
        out["decoder_forward"] = decoder_leg(torch, B, wl, dev)
        if "decode" in out and "decode" in out["decoder_forward"]:
            # the real decode step (attention, norms and caches included) beside the linears-only figures above
            real = out["decoder_forward"]["decode"]
            out["decode"]["real_step"] = {
                "chain_of_launches_us_per_token": real.get("us_per_token_graph", real["us_per_token_eager"]),
                "one_launch_us_per_token": min(real["step_kernel"]["us_per_token_eager"],
                                               real["step_kernel"].get("us_per_token_graph", float("inf"))),
                "one_launch_GBps_weights": real["step_kernel"]["GBps_weights"],
                "one_launch_frac_of_hbm_peak": real["step_kernel"]["frac_of_hbm_peak"],
                "logits_equal": real["step_kernel"]["logits_equal_chain"],
                "roofline": {"bound": "hbm", "kernel": "decoder_step_kernel (one launch per token)",
                             "achieved": real["step_kernel"]["GBps_weights"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": real["step_kernel"]["frac_of_hbm_peak"],
                             "algorithmic_bytes_per_launch": real["step_kernel"]["weight_bytes_per_token"],
                             "traffic": stored_traffic("decoder_step_kernel")},
                "formulation": "dependency-respecting, whole model: 32 layers with attention over the cache, norms, "
                               "SwiGLU, cache append, final norm and head; batch 1, 148 cached tokens"}
    out["selection"] = selection_leg(torch, B, wl, dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, timed_outputs)
        out["parity_checked"] = out["cpu_baseline"].get("parity_mismatches") == 0 and ws_error == 0
    print(json.dumps(out))


if __name__ == "__main__":
    main()
