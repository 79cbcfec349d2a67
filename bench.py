#!/usr/bin/env python3
"""Benchmark of the W4A4 hot path on one MI355X.

A step is one pass of the whole path over one synthetic layer: sq_rotate_quantize_prepared on X,
then sq_w4a4_gemm; the weights were rotated and quantized beforehand and R1, R2 were put into the
matrix cores' operand order beforehand (the offline phase; the plain sq_rotate_quantize entry,
which takes R1 and R2 as they are, is timed beside it as rotate_quant_us_unprepared_entry).
The headline workload is the attention-projection shape T=2048, K=N=4096.  Inputs are resident in
HBM before the clock starts, and the step cycles through a ring of buffer sets larger than the
256 MB last-level cache so that "HBM" numbers are not cache numbers.

How the times are taken.  Every figure comes from HIP events recorded on the stream the kernels
run on.  After W warm-up steps the step is timed in blocks of exactly K steps (--steps), as many
blocks as it takes to reach 100 steps (at least three): the headline `value` is the median
block's time per step, the minimum is beside it.  Each kernel is also timed alone, the same
way; where a kernel is shorter than the host's Python -> C call path (about 10 us per call: the
rotate+quantize kernel at 2048 tokens is just that long, at 8 tokens it takes 6 us) the host
enqueues whole batches while a spin kernel holds the stream, so that the GPU runs them back to
back between two events.  The roofline figures come from these per-kernel times.  (A HIP graph of
the same launches was tried for this and replays 1-5 us per node slower than the stream runs
them; the held stream is used only where needed because the clocks sag during the hold.)

Prints ONE JSON line: layer time (us), the per-kernel rates, the roofline of the dominant kernel
(the GEMM: int8 MFMA) and of the rotate+quantize kernel (HBM), and the CPU oracle timed on this
box's host cores beside them (all cores and one thread; the headline layer and large_prefill).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
INT8_MFMA_PEAK_TOPS = 5000.0    # MI355X dense int8 matrix peak
RING_BYTES = 640 << 20          # > 2x the 256 MB Infinity Cache
MIN_TIMED_STEPS = 100           # per figure, whatever --steps says
MIN_BLOCKS = 3

# HBM-side bytes per launch.  NOT measured in this run: constants copied from the rocprofv3 --pmc
# summaries profiles/w4a4_gemm_<workload>.md and profiles/rotate_quantize_<workload>.md (FETCH_SIZE
# and WRITE_SIZE, each scaled by what the counter reads for a plain 256 MiB copy: x2.000, x1.000).
PROFILED_TRAFFIC = {
    "attn_proj": {"gemm": {"fetch": 33825466, "write": 16777216},
                  "rotate_quantize": {"fetch": 17075532, "write": 4227072}},
    "mlp_down": {"gemm": {"fetch": 90541107, "write": 16777216},
                 "rotate_quantize": {"fetch": 45743076, "write": 11337728}},
    "decode": {"gemm": {"fetch": 118156413, "write": 458752},
               "rotate_quantize": {"fetch": 659389, "write": 33024}},
    "large_prefill": {"gemm": {"fetch": 1414240495, "write": 469762048},
                      "rotate_quantize": {"fetch": 134742838, "write": 33816576}},
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
        # at most 32 tokens: the GEMM reads the decode layout of the codes (a second copy, made once per layer)
        self.Qt = []
        if T <= 32 and K % 256 == 0:
            for i in range(self.sets):
                self.Qt.append(torch.empty((sq.sq_decode_weights_bytes(K, N),), dtype=torch.uint8, device=dev))
                sq.sq_tile_weights_decode(self.Qw[i], self.Qt[i])
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
        if self.Qt:
            self.sq.sq_w4a4_gemm_decode(self.Q[i], self.s[i], self.Qt[i], self.sw[i], self.Y[i])
        else:
            self.sq.sq_w4a4_gemm(self.Q[i], self.s[i], self.Qw[i], self.sw[i], self.Y[i])

    def gemm_canonical(self, i):
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


def _summary(per_call_ms, blocks, calls_per_block):
    us = [m * 1e3 for m in per_call_ms]
    return {"median_us": statistics.median(us), "min_us": min(us), "mean_us": sum(us) / len(us),
            "blocks": blocks, "calls_per_block": calls_per_block}


def timed(torch, fn, sets, steps, warmup):
    """Eager launches.  W warm-up calls, then blocks of exactly `steps` calls each, enough of them
    for MIN_TIMED_STEPS calls (at least MIN_BLOCKS), an event between blocks and one host
    synchronization at the end.  -> summary of the per-call times of the blocks, with the wall
    time per call over all blocks beside it."""
    for w in range(warmup):
        fn(w % sets)
    torch.cuda.synchronize()
    blocks = max(MIN_BLOCKS, -(-MIN_TIMED_STEPS // steps))
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(blocks + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    k = 0
    for b in range(blocks):
        for _ in range(steps):
            fn(k % sets)
            k += 1
        ev[b + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / (blocks * steps)
    out = _summary([ev[b].elapsed_time(ev[b + 1]) / steps for b in range(blocks)], blocks, steps)
    out["wall_us"] = wall_ms * 1e3
    return out


_SLEEP_CYCLES_PER_MS = None


def _hold_stream(torch, ms):
    """Keep the current stream busy for about `ms` milliseconds with torch's spin kernel (one
    wave), so that launches enqueued meanwhile pile up behind it."""
    global _SLEEP_CYCLES_PER_MS
    if _SLEEP_CYCLES_PER_MS is None:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda._sleep(1000000)
        e0.record()
        torch.cuda._sleep(10000000)
        e1.record()
        torch.cuda.synchronize()
        _SLEEP_CYCLES_PER_MS = 10000000 / max(e0.elapsed_time(e1), 1e-3)
    torch.cuda._sleep(int(ms * _SLEEP_CYCLES_PER_MS))


HOST_CALL_US = 16.0             # a Python -> C launch call costs the host 8-11 us; kernels at least this long
                                # are never waiting for the host in a plain eager loop


def timed_queued(torch, fn, sets, steps, kernel_us):
    """Eager launches with the host taken out of the timed region, for kernels shorter than the
    host's call path (about 10 us per Python -> C call; the kernel at hand takes about kernel_us):
    the stream is held by a spin kernel just long enough for the host to get ahead, the host
    enqueues a whole batch of launches meanwhile, and the GPU then runs the batch back to back
    between two events.  Batches of max(steps, MIN_TIMED_STEPS) launches (at most 400, to stay
    inside the hardware queue), MIN_BLOCKS of them.  The hold is kept short because the clocks sag
    while the one-wave spin kernel runs (after a hold of 2.5 ms a batch of GEMMs ran 3-10 % slower
    than in a plain eager loop).  -> summary of the per-launch times of the batches."""
    n = min(400, max(MIN_TIMED_STEPS, steps))
    for i in range(min(sets, 4)):
        fn(i)
    torch.cuda.synchronize()
    ev = []
    for b in range(MIN_BLOCKS):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for k in range(40):                    # the clocks' working point: the same launches, untimed
            fn(k % sets)
        _hold_stream(torch, (n + 40) * max(0.5, HOST_CALL_US - kernel_us) * 1e-3)
        e0.record()
        for k in range(n):
            fn(k % sets)
        e1.record()
        torch.cuda.synchronize()
        ev.append((e0, e1))
    return _summary([e0.elapsed_time(e1) / n for e0, e1 in ev], MIN_BLOCKS, n)


def kernel_time(torch, fn, sets, steps, warmup):
    """Launch duration of one call in a stream of the same calls.  Plain eager blocks (timed) when
    the call keeps the GPU busy longer than the host needs for the next call; otherwise batches
    enqueued behind a held stream (timed_queued).  -> summary with the method named."""
    eager = timed(torch, fn, sets, steps, warmup)
    if eager["median_us"] >= HOST_CALL_US:
        eager["method"] = "eager blocks (host call path shorter than the kernel)"
        eager["eager_median_us"] = eager["median_us"]
        return eager
    queued = timed_queued(torch, fn, sets, steps, eager["median_us"])
    queued["method"] = "batches enqueued behind a held stream"
    queued["eager_median_us"] = eager["median_us"]
    if queued["median_us"] > eager["median_us"]:           # the host was not the limit after all
        eager["method"] = "eager blocks (no slower than queued batches)"
        eager["eager_median_us"] = eager["median_us"]
        return eager
    return queued


def measure_layer(cfg, torch, sq, synth, steps, warmup):
    B = LayerBuffers(cfg, torch, sq, synth)
    T, K, N = cfg.T, cfg.K, cfg.N
    settled = settle(torch, B.step, B.sets)
    layer = timed(torch, B.step, B.sets, steps, warmup)
    rq = kernel_time(torch, B.rotate_quantize, B.sets, steps, warmup)
    gm = kernel_time(torch, B.gemm, B.sets, steps, warmup)
    rq_plain = kernel_time(torch, B.rotate_quantize_plain, B.sets, steps, warmup)
    gm_canonical = kernel_time(torch, B.gemm_canonical, B.sets, steps, warmup) if B.Qt else None
    single = single_k = None
    if T <= 32 and (cfg.n1, cfg.n2) in ((16, 32), (32, 32), (32, 64), (64, 64), (64, 128)):
        single = timed(torch, B.single_launch, B.sets, steps, warmup)
        single_k = kernel_time(torch, B.single_launch, B.sets, steps, warmup)
    rq_us, gm_us = rq["mean_us"], gm["mean_us"]
    out = {
        "workload": cfg.name, "T": T, "K": K, "N": N, "n1": cfg.n1, "n2": cfg.n2, "givens_pairs": cfg.P,
        "layer_us": layer["median_us"], "layer_us_min": layer["min_us"], "layer_us_wall": layer["wall_us"],
        "timing_blocks": layer["blocks"], "steps_per_block": steps,
        # per kernel: mean = the average launch duration the rooflines use
        "rotate_quant_us": rq_us, "rotate_quant_us_median": rq["median_us"], "rotate_quant_us_min": rq["min_us"],
        "rotate_quant_timing": rq["method"], "rotate_quant_us_eager": rq["eager_median_us"],
        "gemm_us": gm_us, "gemm_us_median": gm["median_us"], "gemm_us_min": gm["min_us"],
        "gemm_timing": gm["method"], "gemm_us_eager": gm["eager_median_us"],
        "rotate_quant_us_unprepared_entry": rq_plain["mean_us"],
        "gemm_entry": "sq_w4a4_gemm_decode (decode layout of the weight codes)" if B.Qt else "sq_w4a4_gemm",
        "gemm_us_canonical_layout": None if gm_canonical is None else gm_canonical["mean_us"],
        "layer_us_single_launch": None if single is None else single["median_us"],
        "single_launch_kernel_us": None if single_k is None else single_k["mean_us"],
        "rotate_quant_GBps": rq_bytes(T, K) / (rq_us * 1e-6) / 1e9,
        "gemm_int_TOPS": gemm_ops(T, K, N) / (gm_us * 1e-6) / 1e12,
        "gemm_weight_stream_GBps": (N * K / 2) / (gm_us * 1e-6) / 1e9,
        "ring_sets": B.sets, "settle_steps": settled,
        "massive_channels": [int(c) for c in synth.massive_channels(cfg)],
    }
    out["rotate_quant_frac_of_hbm_peak"] = out["rotate_quant_GBps"] / HBM_PEAK_GBPS
    out["gemm_frac_of_int8_peak"] = out["gemm_int_TOPS"] / INT8_MFMA_PEAK_TOPS
    out["gemm_weight_stream_frac_of_hbm_peak"] = out["gemm_weight_stream_GBps"] / HBM_PEAK_GBPS
    del B
    torch.cuda.empty_cache()
    return out


FP16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense fp16 matrix peak


def measure_weight_only(cfg, torch, sq, synth, steps, warmup):
    """The weight-only setting (W4A16, the paper's appendix): sq_rotate_fp16 then sq_w4a16_gemm on
    the same layer, same ring of buffer sets.  Rotation: HBM-bound, 2 T K bytes in and 2 T K out;
    GEMM: 2 T K N flops on the fp16 matrix cores."""
    B = LayerBuffers(cfg, torch, sq, synth)
    T, K, N = cfg.T, cfg.K, cfg.N
    L = B.L
    Xr = [torch.empty((T, K), dtype=torch.float16, device=B.Y[0].device) for _ in range(B.sets)]
    rot = lambda i: sq.sq_rotate_fp16(B.X[i], L.giv_i, L.giv_j, L.giv_theta, B.R1, B.R2, Xr[i])
    mm = lambda i: sq.sq_w4a16_gemm(Xr[i], B.Qw[i], B.sw[i], B.Y[i])

    def both(i):
        rot(i)
        mm(i)
    settle(torch, both, B.sets)
    layer = timed(torch, both, B.sets, steps, warmup)
    r = kernel_time(torch, rot, B.sets, steps, warmup)
    g = kernel_time(torch, mm, B.sets, steps, warmup)
    flops = 2.0 * T * K * N
    out = {"workload": cfg.name, "layer_us": layer["median_us"], "layer_us_min": layer["min_us"],
           "rotate_fp16_us": r["mean_us"], "rotate_fp16_GBps": 4.0 * T * K / (r["mean_us"] * 1e-6) / 1e9,
           "rotate_fp16_frac_of_hbm_peak": 4.0 * T * K / (r["mean_us"] * 1e-6) / 1e9 / HBM_PEAK_GBPS,
           "gemm_us": g["mean_us"], "gemm_TFLOPS": flops / (g["mean_us"] * 1e-6) / 1e12,
           "gemm_frac_of_fp16_peak": flops / (g["mean_us"] * 1e-6) / 1e12 / FP16_MFMA_PEAK_TFLOPS,
           "ring_sets": B.sets}
    if T <= 32:      # decode-shaped: one pass over the weight codes, HBM-bound
        out["gemm_weight_stream_GBps"] = N * K / 2.0 / (g["mean_us"] * 1e-6) / 1e9
        out["gemm_frac_of_hbm_peak"] = out["gemm_weight_stream_GBps"] / HBM_PEAK_GBPS
        # W3A16: the same weights through the 3-bit quantizer and the 3-bit storage (3K/8 bytes a row)
        dev = B.Y[0].device
        Q3n = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
        s3 = torch.empty((N,), dtype=torch.float32, device=dev)
        for lo in range(0, N, 4096):
            hi = min(N, lo + 4096)
            Wt = torch.from_numpy(synth.weight_rows_t(cfg, np.arange(lo, hi))).to(dev)
            sq.sq_rotate_quantize_variant(Wt, L.giv_i, L.giv_j, L.giv_theta, B.R1, B.R2, 3, 1.0, Q3n[lo:hi], s3[lo:hi])
        Q3 = []
        for i in range(B.sets):
            Q3.append(torch.empty((N, 3 * K // 8), dtype=torch.uint8, device=dev))
            sq.sq_pack_w3(Q3n if i == 0 else torch.roll(Q3n, shifts=5 * i, dims=0).contiguous(), Q3[i])
        del Q3n
        g3 = kernel_time(torch, lambda i: sq.sq_w3a16_gemm(Xr[i], Q3[i], s3, B.Y[i]), B.sets, steps, warmup)
        out["w3a16_gemm_us"] = g3["mean_us"]
        out["w3a16_weight_stream_GBps"] = N * K * 3.0 / 8.0 / (g3["mean_us"] * 1e-6) / 1e9
        out["w3a16_frac_of_hbm_peak"] = out["w3a16_weight_stream_GBps"] / HBM_PEAK_GBPS
        del Q3
    del B, Xr
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
    us = timed(torch, call, sets, steps, warmup)["median_us"]
    return {"workload": cfg.name, "T": cfg.T, "n1": cfg.n1, "n2": cfg.n2, "art_steps": cfg.P, "us": us,
            "calibration_bytes": 2.0 * cfg.T * cfg.K, "whole_call_GBps": 2.0 * cfg.T * cfg.K / (us * 1e-6) / 1e9,
            "ring_sets": sets}


def _oracle_sample(oracle, synth, cfg, L, Qw, sw, tokens_rq, tokens_gemm):
    """Seconds the oracle needs for rotate+quantize of the first tokens_rq tokens and for its GEMM
    of the first tokens_gemm tokens against the weight rows in Qw."""
    t0 = time.perf_counter()
    Qx, sx = oracle.quantize_rows(oracle.rotate(L.X[:tokens_rq], L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2))
    t_rq = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.gemm(Qx[:tokens_gemm], sx[:tokens_gemm], Qw, sw)
    return t_rq, time.perf_counter() - t0


def cpu_baseline(cfg, synth, channels=None, tokens_rq=None, tokens_gemm=None, one_thread_fraction=16):
    """The CPU oracle, as it stands, on this machine's host cores, on a bounded sample of the layer:
    rotate+quantize of the first tokens_rq tokens, then the integer GEMM with its dequantization of
    the first tokens_gemm tokens against the first `channels` output channels (defaults: the
    whole layer); each part is scaled linearly to the whole layer, and the sample is named.
    Once with every core and once, on a sample one_thread_fraction times smaller, with one thread
    (the thread count is set through the OpenMP runtime the oracle library is linked with)."""
    import oracle
    oracle.build()
    T, K, N = cfg.T, cfg.K, cfg.N
    channels = N if channels is None else min(N, channels)
    tokens_rq = T if tokens_rq is None else min(T, tokens_rq)
    tokens_gemm = T if tokens_gemm is None else min(T, tokens_gemm)
    L = synth.layer(cfg, max(tokens_rq, tokens_gemm))
    Wt = synth.weight_rows_t(cfg, np.arange(channels))
    Qw, sw = oracle.prepare_weights(Wt, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2)   # offline, untimed
    cores = oracle.num_threads()

    def run(trq, tgm, label):
        t_rq, t_gm = _oracle_sample(oracle, synth, cfg, L, Qw, sw, trq, tgm)
        t_rq_full, t_gm_full = t_rq * (T / trq), t_gm * (T / tgm) * (N / channels)
        return {"value": (t_rq_full + t_gm_full) * 1e6, "unit": "us", "kind": "oracle",
                "sample": (f"{label}: rotate+quantize of {trq} of {T} tokens (scaled x{T / trq:g}); GEMM of "
                           f"{tgm} tokens x {channels} of {N} output channels (scaled x{T / tgm * N / channels:g})"),
                "sampled_seconds": t_rq + t_gm,
                "rotate_quant_GBps": rq_bytes(T, K) / t_rq_full / 1e9,
                "gemm_int_TOPS": gemm_ops(T, K, N) / t_gm_full / 1e12}

    out = run(tokens_rq, tokens_gemm, f"one {cfg.name} layer")
    out["cores"] = cores
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(1)
    try:
        single = run(max(1, tokens_rq // one_thread_fraction), max(1, tokens_gemm // one_thread_fraction),
                     f"one {cfg.name} layer, one thread")
    finally:
        omp.omp_set_num_threads(cores)
    single["cores"] = 1
    out["one_thread"] = single
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="attn_proj", help="layer shape for the headline number")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the other layer shapes")
    ap.add_argument("--only-build-rotation", action="store_true",
                    help="time only the offline constructor on --workload and print its numbers")
    ap.add_argument("--only-single-launch", action="store_true",
                    help="time only sq_decode_layer (the layer in one launch, at most 32 tokens) on --workload")
    ap.add_argument("--only-kernels", action="store_true",
                    help="run only the two kernels of --workload, each in queued batches (what the rocprofv3 "
                         "summaries under profiles/ are taken from)")
    ap.add_argument("--only-weight-only", action="store_true",
                    help="time only the weight-only setting (sq_rotate_fp16, sq_w4a16_gemm) on --workload")
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
        us = kernel_time(torch, B.single_launch, B.sets, args.steps, args.warmup)["mean_us"]
        print(json.dumps({"workload": cfg.name, "layer_us_single_launch": us, "ring_sets": B.sets,
                          "weight_stream_GBps": cfg.N * cfg.K / 2 / (us * 1e-6) / 1e9}))
        return 0
    if args.only_weight_only:
        print(json.dumps({"weight_only_w4a16": measure_weight_only(cfg, torch, sq, synth, args.steps, args.warmup)}))
        return 0
    if args.only_kernels:
        B = LayerBuffers(cfg, torch, sq, synth)
        settle(torch, B.step, B.sets)
        rq = kernel_time(torch, B.rotate_quantize, B.sets, args.steps, args.warmup)
        gm = kernel_time(torch, B.gemm, B.sets, args.steps, args.warmup)
        print(json.dumps({"workload": cfg.name, "ring_sets": B.sets, "rotate_quant_us": rq["mean_us"],
                          "gemm_us": gm["mean_us"], "launches_each": rq["blocks"] * rq["calls_per_block"]}))
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
    source = lambda stem: (f"constant from profiles/{stem}_{cfg.name}.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE), "
                           "not measured in this run") if cfg.name in PROFILED_TRAFFIC else None
    timing_note = "average launch duration between HIP events on the launch stream; "
    if cfg.T <= 64:      # decode-shaped GEMM: one pass over the weights, HBM-bound
        gemm_roofline = {"kernel": "w4a4_gemm_skinny_kernel" + (" on the decode layout (sq_w4a4_gemm_decode)" if cfg.T <= 32 and cfg.K % 256 == 0 else ""),
                         "bound": "hbm", "achieved": head["gemm_weight_stream_GBps"],
                         "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": head["gemm_weight_stream_GBps"] / HBM_PEAK_GBPS,
                         "bytes_per_launch": cfg.N * cfg.K / 2.0, "launch_us": head["gemm_us"], "timing": timing_note + head["gemm_timing"],
                         "traffic": traffic("gemm"), "traffic_detail": prof.get("gemm"),
                         "traffic_source": source("w4a4_gemm")}
    else:
        gemm_roofline = {"kernel": "w4a4_gemm_kernel", "bound": "mfma", "achieved": gemm_tops,
                         "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": gemm_tops / INT8_MFMA_PEAK_TOPS,
                         "ops_per_launch": gemm_ops(cfg.T, cfg.K, cfg.N), "launch_us": head["gemm_us"],
                         "timing": timing_note + head["gemm_timing"], "traffic": traffic("gemm"), "traffic_detail": prof.get("gemm"),
                         "traffic_source": source("w4a4_gemm")}
    result = {
        "metric": f"layer time, rotate+quant then W4A4 GEMM, T={cfg.T} K={cfg.K} N={cfg.N} (also: rotate+quant HBM GB/s, GEMM int TOPS)",
        "value": head["layer_us"], "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["layer_us"] / 1e3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4 codes on int8 MFMA, int32 accumulate; fp32 rotation",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} K={cfg.K} ({cfg.n1}x{cfg.n2}) N={cfg.N}, {cfg.P} Givens pairs",
                   "ring_sets": head["ring_sets"], "settle_steps_before_warmup": head["settle_steps"],
                   "value_is": f"median over {head['timing_blocks']} blocks of {args.steps} eager steps each, HIP events",
                   "massive_channels": head["massive_channels"]},
        "layer_us_min": head["layer_us_min"], "layer_us_wall": head["layer_us_wall"],
        "rotate_quant_GBps": head["rotate_quant_GBps"], "gemm_int_TOPS": gemm_tops,
        "rotate_quant_us": head["rotate_quant_us"], "gemm_us": head["gemm_us"],
        "rotate_quant_us_min": head["rotate_quant_us_min"], "gemm_us_min": head["gemm_us_min"],
        "rotate_quant_us_eager": head["rotate_quant_us_eager"], "gemm_us_eager": head["gemm_us_eager"],
        "rotate_quant_us_unprepared_entry": head["rotate_quant_us_unprepared_entry"],
        "gemm_entry": head["gemm_entry"], "gemm_us_canonical_layout": head["gemm_us_canonical_layout"],
        "layer_us_single_launch": head["layer_us_single_launch"],
        "roofline": gemm_roofline,
        "roofline_rotate_quant": {"kernel": "rotate_quantize_mfma_kernel", "bound": "hbm",
                                  "achieved": head["rotate_quant_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                  "frac": head["rotate_quant_GBps"] / HBM_PEAK_GBPS,
                                  "bytes_per_launch": rq_bytes(cfg.T, cfg.K), "launch_us": head["rotate_quant_us"],
                                  "timing": timing_note + head["rotate_quant_timing"],
                                  "traffic": traffic("rotate_quantize"),
                                  "traffic_detail": prof.get("rotate_quantize"),
                                  "traffic_source": source("rotate_quantize")},
        "other_workloads": extra,
    }
    if not args.no_extra and cfg.n2 & (cfg.n2 - 1) == 0:
        result["build_rotation"] = measure_build_rotation(cfg, torch, sq, synth, max(10, args.steps // 4),
                                                          max(2, args.warmup // 4))
    if not args.no_extra:
        result["weight_only_w4a16"] = measure_weight_only(cfg, torch, sq, synth, max(10, args.steps // 2),
                                                          max(2, args.warmup // 4))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, synth)
        if not args.no_extra and cfg.name != "large_prefill":
            # beside the large layer as well: 1024 of its 8192 tokens through rotate+quantize, 64 tokens
            # x 4096 of its 28672 output channels through the GEMM
            result["cpu_baseline_large_prefill"] = cpu_baseline(synth.CONFIGS["large_prefill"], synth, channels=4096,
                                                                tokens_rq=1024, tokens_gemm=64, one_thread_fraction=8)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
