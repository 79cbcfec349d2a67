#!/usr/bin/env python3
"""Benchmark of the W4A4 hot path on one MI355X.

A step is one pass of the whole path over one synthetic layer: sq_rotate_quantize_prepared on X,
then sq_w4a4_gemm; the weights were rotated and quantized beforehand and R1, R2 were put into the
matrix cores' operand order beforehand (the offline phase; the plain sq_rotate_quantize entry,
which takes R1 and R2 as they are, is timed beside it as rotate_quant_us_unprepared_entry).
The headline workload is the attention-projection shape T=2048, K=N=4096.  Inputs are resident in
HBM before the clock starts, and the step cycles through a ring of buffer sets larger than the
256 MB last-level cache so that "HBM" numbers are not cache numbers.

Prints ONE JSON line: layer time (us), the per-kernel rates, the roofline of the dominant kernel
(the GEMM: int8 MFMA) and of the rotate+quantize kernel (HBM), and the CPU oracle timed on this
box's host cores beside them.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
INT8_MFMA_PEAK_TOPS = 5000.0    # MI355X dense int8 matrix peak
RING_BYTES = 640 << 20          # > 2x the 256 MB Infinity Cache

# HBM-side bytes per launch, from the rocprofv3 --pmc runs summarised in
# profiles/w4a4_gemm_<workload>.md and profiles/rotate_quantize_<workload>.md (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the counter reads for a plain 256 MiB copy: x2.000 and x1.000).
PROFILED_TRAFFIC = {
    "attn_proj": {"gemm": {"fetch": 33797816, "write": 16777216},
                  "rotate_quantize": {"fetch": 17064267, "write": 4227072}},
    "mlp_down": {"gemm": {"fetch": 90415209, "write": 16777216},
                 "rotate_quantize": {"fetch": 45744638, "write": 11337728}},
    "decode": {"gemm": {"fetch": 117976009, "write": 468416},
               "rotate_quantize": {"fetch": 652215, "write": 33024}},
    "large_prefill": {"gemm": {"fetch": 1412787392, "write": 469762048},
                      "rotate_quantize": {"fetch": 134738700, "write": 33816576}},
}


def rq_bytes(T: int, K: int) -> float:
    """Algorithmic HBM bytes of rotate+quantize: fp16 row in, nibble codes and one fp32 step out."""
    return 2.5 * T * K + 4.0 * T


def gemm_ops(T: int, K: int, N: int) -> float:
    return 2.0 * T * K * N


class LayerBuffers:
    """Ring of device buffer sets for one layer shape."""

    def __init__(self, cfg, torch, sq, synth, sets=None):
        self.cfg, self.torch, self.sq = cfg, torch, sq
        self.ws = None
        dev = torch.device("cuda:0")
        L = synth.layer(cfg)
        self.L = L
        T, K, N = cfg.T, cfg.K, cfg.N
        per_set = 2 * T * K + T * K // 2 + 2 * T * N + N * K // 2
        self.sets = sets or max(2, min(16, -(-RING_BYTES // per_set)))
        self.R1 = torch.from_numpy(L.R1).to(dev)
        self.R2 = torch.from_numpy(L.R2).to(dev)
        X0 = torch.from_numpy(L.X).to(dev)
        # offline phase: W^T rows get the same transform and quantizer (Sec. 4.2), on the GPU
        Qw0 = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
        sw0 = torch.empty((N,), dtype=torch.float32, device=dev)
        slab = 4096
        for lo in range(0, N, slab):
            hi = min(N, lo + slab)
            Wt = torch.from_numpy(synth.weight_rows_t(cfg, np.arange(lo, hi))).to(dev)
            sq.sq_rotate_quantize(Wt, L.giv_i, L.giv_j, L.giv_theta, self.R1, self.R2, Qw0[lo:hi], sw0[lo:hi])
        # offline as well: R1, R2 in the operand order of the matrix cores (constants of the layer)
        self.prepared = torch.empty((sq.sq_prepared_rotation_bytes(cfg.n1, cfg.n2),), dtype=torch.uint8, device=dev)
        sq.sq_prepare_rotation(self.R1, self.R2, self.prepared)
        torch.cuda.synchronize()
        self.X, self.Qw, self.sw, self.Q, self.s, self.Y = [], [], [], [], [], []
        for i in range(self.sets):
            # other sets: the same rows in another order (same distribution, other addresses)
            self.X.append(X0 if i == 0 else torch.roll(X0, shifts=7 * i, dims=0).contiguous())
            self.Qw.append(Qw0 if i == 0 else torch.roll(Qw0, shifts=5 * i, dims=0).contiguous())
            self.sw.append(sw0 if i == 0 else torch.roll(sw0, shifts=5 * i, dims=0).contiguous())
            self.Q.append(torch.empty((T, K // 2), dtype=torch.uint8, device=dev))
            self.s.append(torch.empty((T,), dtype=torch.float32, device=dev))
            self.Y.append(torch.empty((T, N), dtype=torch.float16, device=dev))
        torch.cuda.synchronize()

    def rotate_quantize(self, i):
        L = self.L
        self.sq.sq_rotate_quantize_prepared(self.X[i], L.giv_i, L.giv_j, L.giv_theta, self.prepared,
                                            self.cfg.n1, self.cfg.n2, self.Q[i], self.s[i])

    def rotate_quantize_plain(self, i):
        """The entry point that takes R1 and R2 as they are: same results, slower start."""
        L = self.L
        self.sq.sq_rotate_quantize(self.X[i], L.giv_i, L.giv_j, L.giv_theta, self.R1, self.R2, self.Q[i], self.s[i])

    def gemm(self, i):
        self.sq.sq_w4a4_gemm(self.Q[i], self.s[i], self.Qw[i], self.sw[i], self.Y[i])

    def step(self, i):
        self.rotate_quantize(i)
        self.gemm(i)

    def single_launch(self, i):
        """The same layer through sq_decode_layer (at most 32 tokens)."""
        L = self.L
        if self.ws is None:
            self.ws = self.torch.zeros((self.sq.sq_decode_layer_workspace_bytes(self.cfg.T, self.cfg.K),),
                                       dtype=self.torch.uint8, device=self.Y[0].device)
        self.sq.sq_decode_layer(self.X[i], L.giv_i, L.giv_j, L.giv_theta, self.prepared, self.cfg.n1, self.cfg.n2,
                                self.Qw[i], self.sw[i], self.Y[i], self.ws)


SETTLE_SECONDS = 0.08           # load put on the GPU before anything is timed (see settle())


def settle(torch, fn, sets):
    """The GPU's clocks take some tens of milliseconds under load to reach their working point: the
    first few hundred layer steps on a fresh process run 10-20 % slower than all later ones.  So
    before any timing the same step is run, untimed, for SETTLE_SECONDS; the W warmup steps of
    timed() come on top.  Returns the number of steps it ran."""
    n, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < SETTLE_SECONDS:
        for _ in range(50):
            fn(n % sets)
            n += 1
        torch.cuda.synchronize()
    return n


def timed(torch, fn, sets, steps, warmup):
    """(wall ms per call, event ms per call): events are recorded on the stream the kernels use."""
    for w in range(warmup):
        fn(w % sets)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for k in range(steps):
        fn(k % sets)
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return wall, e0.elapsed_time(e1) / steps


def measure_layer(cfg, torch, sq, synth, steps, warmup):
    B = LayerBuffers(cfg, torch, sq, synth)
    T, K, N = cfg.T, cfg.K, cfg.N
    settled = settle(torch, B.step, B.sets)
    wall_ms, ev_ms = timed(torch, B.step, B.sets, steps, warmup)
    _, rq_ms = timed(torch, B.rotate_quantize, B.sets, steps, warmup)
    _, gm_ms = timed(torch, B.gemm, B.sets, steps, warmup)
    _, rq_plain_ms = timed(torch, B.rotate_quantize_plain, B.sets, steps, warmup)
    single_ms = None
    if T <= 32 and (cfg.n1, cfg.n2) in ((16, 32), (32, 32), (32, 64), (64, 64), (64, 128)):
        single_ms, _ = timed(torch, B.single_launch, B.sets, steps, warmup)
    out = {
        "workload": cfg.name, "T": T, "K": K, "N": N, "n1": cfg.n1, "n2": cfg.n2, "givens_pairs": cfg.P,
        "layer_us": wall_ms * 1e3, "layer_us_events": ev_ms * 1e3,
        "rotate_quant_us": rq_ms * 1e3, "gemm_us": gm_ms * 1e3,
        "rotate_quant_us_unprepared_entry": rq_plain_ms * 1e3,
        "layer_us_single_launch": None if single_ms is None else single_ms * 1e3,
        "rotate_quant_GBps": rq_bytes(T, K) / (rq_ms * 1e-3) / 1e9,
        "gemm_int_TOPS": gemm_ops(T, K, N) / (gm_ms * 1e-3) / 1e12,
        "gemm_weight_stream_GBps": (N * K / 2) / (gm_ms * 1e-3) / 1e9,
        "ring_sets": B.sets, "settle_steps": settled,
        "massive_channels": [int(c) for c in synth.massive_channels(cfg)],
    }
    out["rotate_quant_frac_of_hbm_peak"] = out["rotate_quant_GBps"] / HBM_PEAK_GBPS
    out["gemm_frac_of_int8_peak"] = out["gemm_int_TOPS"] / INT8_MFMA_PEAK_TOPS
    out["gemm_weight_stream_frac_of_hbm_peak"] = out["gemm_weight_stream_GBps"] / HBM_PEAK_GBPS
    del B
    torch.cuda.empty_cache()
    return out


def measure_build_rotation(cfg, torch, sq, synth, steps, warmup):
    """The offline constructor (sq_build_rotation) on the workload's activations as calibration
    batch.  Not part of the layer time.  Its one large kernel reads X once (2*T*K bytes); the rest
    is a few small launches, so the whole-call rate is a lower bound on that kernel's."""
    dev = torch.device("cuda:0")
    X0 = torch.from_numpy(synth.activations(cfg)).to(dev)
    sets = max(2, min(16, -(-RING_BYTES // (2 * cfg.T * cfg.K))))
    Xs = [X0 if i == 0 else torch.roll(X0, shifts=7 * i, dims=0).contiguous() for i in range(sets)]
    gi = torch.empty((cfg.P,), dtype=torch.int32, device=dev)
    gj = torch.empty((cfg.P,), dtype=torch.int32, device=dev)
    gt = torch.empty((cfg.P,), dtype=torch.float32, device=dev)
    R1 = torch.empty((cfg.n1, cfg.n1), dtype=torch.float16, device=dev)
    R2 = torch.empty((cfg.n2, cfg.n2), dtype=torch.float16, device=dev)
    ws = torch.empty((sq.sq_build_rotation_workspace_bytes(cfg.T, cfg.n1, cfg.n2),), dtype=torch.uint8, device=dev)
    call = lambda i: sq.sq_build_rotation(Xs[i], cfg.n1, cfg.n2, gi, gj, gt, R1, R2, ws)
    settle(torch, call, sets)
    _, ms = timed(torch, call, sets, steps, warmup)
    return {"workload": cfg.name, "T": cfg.T, "n1": cfg.n1, "n2": cfg.n2, "art_steps": cfg.P, "us": ms * 1e3,
            "calibration_bytes": 2.0 * cfg.T * cfg.K, "whole_call_GBps": 2.0 * cfg.T * cfg.K / (ms * 1e-3) / 1e9,
            "ring_sets": sets}


def cpu_baseline(cfg, synth):
    """The CPU oracle, as it stands, on this machine's host cores: rotate+quantize of every token, then
    the integer GEMM with its dequantization on every token (for layers much larger than the
    headline one the GEMM is timed on the first 2048 tokens and scaled linearly in T)."""
    import oracle
    oracle.build()
    L = synth.layer(cfg)
    Ts = min(cfg.T, 2048)
    Wt = synth.weights_t(cfg)
    Qw, sw = oracle.prepare_weights(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)   # offline, untimed
    t0 = time.perf_counter()
    Qx, sx = oracle.quantize_rows(oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2))
    t_rq = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.gemm(Qx[:Ts], sx[:Ts], Qw, sw)
    t_gemm = (time.perf_counter() - t0) * (cfg.T / Ts)
    gemm_note = (f"GEMM of all {cfg.T} tokens x {cfg.N} outputs timed in full" if Ts == cfg.T else
                 f"GEMM timed on the first {Ts} tokens x all {cfg.N} outputs and scaled by {cfg.T / Ts:g}")
    return {
        "value": (t_rq + t_gemm) * 1e6, "unit": "us", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": f"one layer: rotate+quantize of all {cfg.T} tokens timed in full; {gemm_note}",
        "rotate_quant_GBps": rq_bytes(cfg.T, cfg.K) / t_rq / 1e9,
        "gemm_int_TOPS": gemm_ops(cfg.T, cfg.K, cfg.N) / t_gemm / 1e12,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="attn_proj", help="layer shape for the headline number")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the other layer shapes")
    ap.add_argument("--only-build-rotation", action="store_true",
                    help="time only the offline constructor on --workload and print its numbers")
    ap.add_argument("--only-single-launch", action="store_true",
                    help="time only sq_decode_layer (the layer in one launch, at most 32 tokens) on --workload")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run three plain 256 MiB device copies (known traffic: the scale for "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        return 2

    import torch
    import paper_2511_22316_amd as sq
    from paper_2511_22316_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    if not os.path.exists(sq.library_path()):
        from paper_2511_22316_amd import build
        build.build()

    cfg = synth.CONFIGS[args.workload]
    if args.copy_calibration:
        src = torch.ones((256 << 20) // 2, dtype=torch.float16, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.only_build_rotation:
        print(json.dumps({"build_rotation": measure_build_rotation(cfg, torch, sq, synth, args.steps, args.warmup)}))
        return 0
    if args.only_single_launch:
        B = LayerBuffers(cfg, torch, sq, synth)
        settle(torch, B.single_launch, B.sets)
        _, ms = timed(torch, B.single_launch, B.sets, args.steps, args.warmup)
        print(json.dumps({"workload": cfg.name, "layer_us_single_launch": ms * 1e3, "ring_sets": B.sets,
                          "weight_stream_GBps": cfg.N * cfg.K / 2 / (ms * 1e-3) / 1e9}))
        return 0
    head = measure_layer(cfg, torch, sq, synth, args.steps, args.warmup)
    extra = {}
    if not args.no_extra:
        for name, st in (("tiny", args.steps), ("mlp_down", max(10, args.steps // 4)), ("decode", args.steps),
                         ("large_prefill", max(5, args.steps // 20))):
            if name != args.workload:
                extra[name] = measure_layer(synth.CONFIGS[name], torch, sq, synth, st, max(2, args.warmup // 4))

    gemm_tops = head["gemm_int_TOPS"]
    prof = PROFILED_TRAFFIC.get(cfg.name, {})
    traffic = lambda k: (prof[k]["fetch"] + prof[k]["write"]) if k in prof else None
    if cfg.T <= 64:      # decode-shaped GEMM: one pass over the weights, HBM-bound
        gemm_roofline = {"kernel": "w4a4_gemm_skinny_kernel", "bound": "hbm", "achieved": head["gemm_weight_stream_GBps"],
                         "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": head["gemm_weight_stream_GBps"] / HBM_PEAK_GBPS,
                         "bytes_per_launch": cfg.N * cfg.K / 2.0, "traffic": traffic("gemm"),
                         "traffic_detail": prof.get("gemm")}
    else:
        gemm_roofline = {"kernel": "w4a4_gemm_kernel", "bound": "mfma", "achieved": gemm_tops,
                         "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": gemm_tops / INT8_MFMA_PEAK_TOPS,
                         "ops_per_launch": gemm_ops(cfg.T, cfg.K, cfg.N), "traffic": traffic("gemm"),
                         "traffic_detail": prof.get("gemm")}
    result = {
        "metric": f"layer time, rotate+quant then W4A4 GEMM, T={cfg.T} K={cfg.K} N={cfg.N} (also: rotate+quant HBM GB/s, GEMM int TOPS)",
        "value": head["layer_us"], "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["layer_us"] / 1e3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4 codes on int8 MFMA, int32 accumulate; fp32 rotation",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} K={cfg.K} ({cfg.n1}x{cfg.n2}) N={cfg.N}, {cfg.P} Givens pairs",
                   "ring_sets": head["ring_sets"], "settle_steps_before_warmup": head["settle_steps"],
                   "massive_channels": head["massive_channels"]},
        "rotate_quant_GBps": head["rotate_quant_GBps"], "gemm_int_TOPS": gemm_tops,
        "rotate_quant_us": head["rotate_quant_us"], "gemm_us": head["gemm_us"],
        "rotate_quant_us_unprepared_entry": head["rotate_quant_us_unprepared_entry"],
        "layer_us_single_launch": head["layer_us_single_launch"],
        "roofline": gemm_roofline,
        "roofline_rotate_quant": {"kernel": "rotate_quantize", "bound": "hbm", "achieved": head["rotate_quant_GBps"],
                                  "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                  "frac": head["rotate_quant_GBps"] / HBM_PEAK_GBPS,
                                  "bytes_per_launch": rq_bytes(cfg.T, cfg.K),
                                  "traffic": traffic("rotate_quantize"),
                                  "traffic_detail": prof.get("rotate_quantize")},
        "other_workloads": extra,
    }
    if not args.no_extra and cfg.n2 & (cfg.n2 - 1) == 0:
        result["build_rotation"] = measure_build_rotation(cfg, torch, sq, synth, max(10, args.steps // 4),
                                                          max(2, args.warmup // 4))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, synth)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
