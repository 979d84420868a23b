#!/usr/bin/env python3
"""Benchmark of the SQAP-VLA hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input of
the batched-prefill workload (16 observations x 276 tokens, each pruned to
128 + 20 = 148 tokens, M = 2368):

    prune_topk -> kept_rows -> quantize_act (gather fused) -> W4A4 gate/up
    linear (4096 -> 11008) -> quantize_act (K = 11008) -> W4A4 down linear
    (11008 -> 4096)

Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
`value` is 2*M*N*K of the two linears divided by the whole step time (TOPS).
The `roofline` object is for the prefill GEMM kernel (int8 MFMA bound), timed
with HIP events around its launches; `decode` reports the small-M path
(HBM bound); `cpu_baseline` times the CPU oracle on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5033.0      # 8192 op/clk/CU x 256 CU x 2.4 GHz (dense)
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--only", default="", help="run only the main loop this many times (for profilers)")
    return ap.parse_args()


class Prefill:
    """Configuration 3 resident on the GPU."""

    def __init__(self, torch, B, wl, dev):
        c = wl.CONFIGS[3]
        self.torch, self.B = torch, B
        self.batch, self.keep = c["batch"], c["keep_k"]
        self.S, self.nv = wl.SEQ_LEN, wl.N_VISUAL
        self.M = self.batch * (self.keep + wl.N_TEXT)
        H, F = wl.HIDDEN, wl.FFN
        self.H, self.F = H, F
        t = lambda a: torch.from_numpy(a).to(dev)
        self.scores = t(wl.scores(self.batch, self.nv, wl.rng_for(3, 0, wl.T_SCORES)))
        self.X = t(wl.layer_input(3, 0, 4, self.batch * self.S))          # gate/up input, all tokens
        self.Xd = t(wl.layer_input(3, 0, 6, self.M))                       # down input, kept tokens
        self.W_gate = self._weight(t(wl.layer_weight(3, 0, 4)))
        self.W_down = self._weight(t(wl.layer_weight(3, 0, 6)))
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
        self.ws = torch.empty((nws,), dtype=u8, device=dev)
        self.ops = 2.0 * self.M * (F * H + H * F)
        self.gemm_events = None

    def _weight(self, W):
        torch, B = self.torch, self.B
        N, K = W.shape
        Wq = torch.empty((N, K // 2), dtype=torch.uint8, device=W.device)
        sw = torch.empty((N,), dtype=torch.float16, device=W.device)
        B.sqap_quantize_weight(W, Wq, sw)
        h = B.sqap_weight_pack(Wq, sw)
        torch.cuda.synchronize()
        return h

    def step(self):
        B, ev = self.B, self.gemm_events
        B.sqap_prune_topk(self.scores, self.keep, self.idx)
        B.sqap_kept_rows(self.idx, self.S, 0, self.nv, self.rows)
        B.sqap_quantize_act(self.X, self.rows, self.Xq, self.sx)
        if ev is not None:
            ev[0].record()
        B.sqap_w4a4_linear(self.Xq, self.sx, self.W_gate, self.Yg, None, self.ws)
        if ev is not None:
            ev[1].record()
        B.sqap_quantize_act(self.Xd, None, self.Xdq, self.sxd)
        if ev is not None:
            ev[2].record()
        B.sqap_w4a4_linear(self.Xdq, self.sxd, self.W_down, self.Yd, None, self.ws)
        if ev is not None:
            ev[3].record()


def time_gemm_launches(torch, wk, steps):
    """Average duration of one prefill GEMM launch, from HIP events recorded on
    the launch stream directly around each linear call inside whole steps."""
    total_ms, launches = 0.0, 0
    per = {"gate_up": 0.0, "down": 0.0}
    for _ in range(steps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        wk.gemm_events = ev
        wk.step()
        torch.cuda.synchronize()
        a, b = ev[0].elapsed_time(ev[1]), ev[2].elapsed_time(ev[3])
        per["gate_up"] += a
        per["down"] += b
        total_ms += a + b
        launches += 2
    wk.gemm_events = None
    return total_ms / launches, {k: v / steps for k, v in per.items()}


def cpu_baseline(wl, wk_M_per_obs, n_obs=4):
    """The oracle, as it stands, on 4 of the 16 observations of the same workload."""
    import numpy as np
    import oracle
    H, F, S, nv, keep = wl.HIDDEN, wl.FFN, wl.SEQ_LEN, wl.N_VISUAL, wl.CONFIGS[3]["keep_k"]
    scores = wl.scores(16, nv, wl.rng_for(3, 0, wl.T_SCORES))[:n_obs]
    X = wl.layer_input(3, 0, 4, 16 * S)[: n_obs * S]
    M = n_obs * wk_M_per_obs
    Xd = wl.layer_input(3, 0, 6, 16 * wk_M_per_obs)[:M]
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
    import ctypes
    threads = ctypes.CDLL("libgomp.so.1").omp_get_max_threads()
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": int(threads), "kind": "oracle",
            "seconds": dt,
            "sample": "%d of 16 observations (M=%d) through the same prune/quantize/gate-up/down path"
                      % (n_obs, M)}


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
    wk = Prefill(torch, B, wl, dev)

    if args.only:
        for _ in range(int(args.only)):
            wk.step()
        torch.cuda.synchronize()
        return

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

    gemm_ms, per_gemm = time_gemm_launches(torch, wk, min(args.steps, 50))
    gemm_ops = wk.ops / 2.0                                  # each of the two launches: 2*M*N*K
    achieved = gemm_ops / (gemm_ms * 1e-3) / 1e12

    out = {
        "metric": "W4A4 linear TOPS (prefill, pruned tokens)",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4 codes -> int8 MFMA -> int32 acc -> fp16",
        "data": "synthetic",
        "config": {"workload": "configs[3]: batched prefill, 16 obs x 276 tokens pruned to 148, M=2368; "
                               "gate/up 4096->11008 and down 11008->4096",
                   "M": wk.M, "step": "prune_topk+kept_rows+quantize_act+linear+quantize_act+linear"},
        "roofline": {"bound": "mfma", "kernel": "gemm_tiled_kernel<256,256>", "achieved": achieved,
                     "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / INT8_MFMA_PEAK_TOPS,
                     "avg_launch_ms": gemm_ms, "per_gemm_ms": per_gemm, "traffic": None},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, wk.keep + wl.N_TEXT)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
