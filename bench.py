#!/usr/bin/env python3
"""Benchmark of the W8A8 layer forward (libhero) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload bert-large|gpt-prefill|gpt-decode|bert-base]

One "step" is one pass of the whole hot path -- every layer of the workload's stack, each
layer = LN^quant, QKV / O / FC1 / FC2 GeMM^quant, INT8 attention -- over one batch of
seeded synthetic input that is already resident in HBM.  Prints ONE JSON line:
  value     W8A8 layer tokens/s = tokens x layers / second
  roofline  the dominant kernel (the FC1 GeMM^quant with its GELU^quant epilogue) timed
            alone with HIP events on the same stream, against the dense INT8 MFMA peak
  cpu_baseline  the CPU oracle timed on a bounded slice of the same workload
Extra keys report the stand-alone GEMM sweep (TOP/s) and the fused LN+quant kernel (GB/s).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs, scaled by the same
# counters on a plain copy of known size) are NOT typed in here: they are read from profiles/measured_traffic.json,
# which names the commit and the commands they were taken with (written from the rocprofv3 summaries beside it).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "measured_traffic.json")

# the roofline bound of a whole layer per workload, in layer-tokens/s: its integer operations at the 5.0 POP/s INT8
# MFMA peak for the prefill stacks (446 GOP / 6.87 TOP per layer), its HBM bytes at 8 TB/s for the decode step
# (1.3 GB per layer-step); bert-base is latency-bound and has none
LAYER_BOUND = {"bert-large-32x512": 185e6, "gpt-prefill-8x2048": 12e6, "gpt-decode-64x1": 0.39e6}

PEAK_INT8_TOPS = 5000.0      # MI355X dense INT8 MFMA, TOP/s
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense FP8 MFMA, TFLOP/s
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, GB/s

WORKLOADS = {"bert-base": 0, "bert-large": 2, "gpt-prefill": 3, "gpt-decode": 4}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(key):
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
        e = dict(t["kernels"][key])
        e["measured_at_commit"] = t.get("commit")
        return e
    except (OSError, KeyError, ValueError):
        return None


RAMP_MS = 60.0    # device time of back-to-back work in front of every timed leg (see time_gpu)


def time_gpu(fn, iters, warmup=3, graph=False, repeats=5, ramp_ms=RAMP_MS):
    """ms per call of fn: HIP events (on the current stream, the one the library launches on) around `iters`
    back-to-back calls, the MEDIAN of `repeats` such measurements.  graph=True: the calls are captured into a HIP
    graph once and the replays are timed, so a short kernel is not hidden behind the ~10 us one call costs on the
    host (Python -> ctypes -> launch); nothing in the library allocates or clears memory, so its calls capture as
    they are.
    Steady state: after any idle period (the host-side preparation of a leg is one) this GPU runs its first ~35 ms
    of work up to 25 % slower than what follows (measured: the same kernel 116 -> 92.7 us per launch over the first
    few hundred launches, again after every 20 ms pause).  The 24-layer stack is timed long after that, so every leg
    first queues about ramp_ms of the same calls, and the repeats follow back to back with no host synchronisation
    between them."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    run, per = (lambda: [fn() for _ in range(iters)]), iters
    if graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(iters):
                fn()
        g.replay()
        torch.cuda.synchronize()
        run = g.replay
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(repeats + 1)]
    if ramp_ms > 0:
        ev[0].record()
        run()
        ev[1].record()
        torch.cuda.synchronize()
        for _ in range(min(400, max(1, int(ramp_ms / max(ev[0].elapsed_time(ev[1]), 1e-3))))):
            run()
    ev[0].record()
    for r in range(repeats):
        run()
        ev[r + 1].record()
    torch.cuda.synchronize()
    return float(np.median([ev[r].elapsed_time(ev[r + 1]) / per for r in range(repeats)]))      # ms per call


class Stack:
    """Device-resident prepared weights + activations of one workload."""

    def __init__(self, hero, shape, seed, mode, layers=None, fp8=False, share=None):
        """share: another Stack of the same model (config 4 decodes with config 3's layers): its prepared
        weights are reused instead of being calibrated and quantized again."""
        import torch
        from paper_2310_17723_amd import binding as HB, prep, synth
        self.hero, self.shape, self.mode = hero, shape, mode
        self.layers = shape.layers if layers is None else layers
        dev = torch.device("cuda")
        B, S, d = shape.B, shape.S, shape.d
        self.T = B * S
        post = shape.arch == synth.POST_LN
        decode = shape.cache_len > 0
        # ---- calibration input: a small batch of the same distribution, propagated
        # through the UNQUANTIZED stack layer by layer (Sec. 3: forward pass only)
        Sc = min(S if not decode else 128, 256)
        Bc = 2
        xc = torch.from_numpy(synth.activations(seed, shape, Bc * Sc, stream=1)).to(dev).double()
        emb = synth.embedding_ln_params(seed, shape)
        self.emb = {k: torch.from_numpy(v).to(dev) for k, v in emb.items()}
        if post:
            xc = torch.nn.functional.layer_norm(xc, (d,), self.emb["g"].double(), self.emb["b"].double(), shape.eps)
        cal_mask = shape.mask if not decode else HB.MASK_CAUSAL
        self.fp8 = fp8
        self.desc = hero.layer_desc(shape.arch, d, shape.H, shape.Dh, shape.f, shape.eps, shape.mask,
                                    mode | (HB.M_FP8 if fp8 else 0))
        self.weights, self.keep = [], []
        if share is not None:
            assert (share.shape.d, share.shape.f, share.shape.H, share.mode, share.fp8) == (d, shape.f, shape.H, mode, fp8)
            self.weights, self.keep = share.weights[:self.layers], share.keep[:self.layers]
        for l in range(self.layers if share is None else 0):
            p = {k: torch.from_numpy(v).to(dev) for k, v in synth.layer_params(seed, shape, l).items()}
            sc, xc = prep.calibrate(p, xc, shape.arch, shape.H, shape.Dh, shape.eps,
                                    cal_mask if cal_mask != HB.MASK_PADDING else HB.MASK_NONE, Bc, Sc, hero=hero, fp8=fp8)
            t, qk, ps = prep.prepare(p, sc, shape.arch, d, shape.Dh, mode, hero=hero, fp8=fp8)
            self.keep.append(t)
            self.weights.append(hero.layer_weights(t, qk, ps))
            del p
        # ---- inputs, resident in HBM
        h0 = torch.from_numpy(synth.activations(seed, shape, self.T)).to(dev)
        self.kv_len = None
        if shape.mask == HB.MASK_PADDING and not decode:
            self.kv_len = torch.from_numpy(synth.kv_lengths(seed, shape)).to(dev)
        self.ws = torch.empty(hero.hero_layer_workspace_bytes(self.desc, B, S), dtype=torch.uint8, device=dev)
        if post:
            self.x0_q, self.x0_s, _ = hero.hero_ln_quant(h0.to(torch.bfloat16), None, None, None, self.emb["g"],
                                                         self.emb["b"], shape.eps, fp8=fp8)
            self.buf = [(torch.empty_like(self.x0_q), torch.empty_like(self.x0_s)) for _ in range(2)]
        else:
            self.h0 = h0.to(torch.bfloat16)
            self.h = torch.empty_like(self.h0)
        self.caches = None
        if decode:
            Smax = shape.cache_len + shape.steps
            self.Smax = Smax
            self.caches = []
            gen = torch.Generator(device="cuda").manual_seed(seed)      # uniform INT8 codes, drawn on the GPU (4.6 GB)
            for l in range(self.layers):
                kc = torch.randint(-127, 128, (B, shape.H, Smax, shape.Dh), dtype=torch.int8, device=dev, generator=gen)
                vc = torch.randint(-127, 128, (B, shape.H, Smax, shape.Dh), dtype=torch.int8, device=dev, generator=gen)
                if fp8:                                   # the bytes are E4M3 codes here: no NaN patterns (0x7F / 0xFF)
                    for c in (kc, vc):
                        c[(c & 0x7F) == 0x7F] -= 1
                self.caches.append((kc, vc))
            # kv_len for every decode step, precomputed: the caller owns the counter
            self.kv_steps = torch.stack([torch.full((B,), shape.cache_len + t + 1, dtype=torch.int32)
                                         for t in range(shape.steps)]).to(dev)
        torch.cuda.synchronize()

    def step(self):
        """One pass of the whole stack.  Decode: `steps` tokens, each through every layer."""
        hero, sh = self.hero, self.shape
        B, S = sh.B, sh.S
        # the hint a caller of a stack gives: what the next call reads first (the next layer's QKV weights)
        nxt = lambda l: self.keep[(l + 1) % self.layers].get("w_qkv")
        if sh.arch == 0:
            xq, xs = self.x0_q, self.x0_s
            for l in range(self.layers):
                oq, os_ = self.buf[l & 1]
                hero.hero_layer_fwd(self.desc, self.weights[l], B, S, self.ws, x_q=xq, x_scale=xs, out_q=oq,
                                    out_scale=os_, kv_len=self.kv_len, next_read=nxt(l))
                xq, xs = oq, os_
        elif self.caches is None:
            self.h.copy_(self.h0)
            for l in range(self.layers):
                hero.hero_layer_fwd(self.desc, self.weights[l], B, S, self.ws, h=self.h, next_read=nxt(l))
        else:
            for t in range(sh.steps):
                self.h.copy_(self.h0)
                for l in range(self.layers):
                    kc, vc = self.caches[l]
                    hero.hero_layer_fwd(self.desc, self.weights[l], B, 1, self.ws, h=self.h, kv_len=self.kv_steps[t],
                                        k_cache=kc, v_cache=vc)

    def sanity(self):
        """Cheap check of what the LAST pass left behind, so that a stack that produced garbage cannot post a
        number: finite values in a plausible range, TWQ rows that reach the code +-127, codes not all saturated."""
        import torch
        sh = self.shape
        if sh.arch == 0:
            oq, os_ = self.buf[(self.layers - 1) & 1]
            rows = torch.ones(self.T, dtype=torch.bool, device=oq.device)
            if self.kv_len is not None:
                rows = (torch.arange(sh.S, device=oq.device)[None, :] < self.kv_len[:, None]).reshape(-1)
            sc = os_[rows]
            ok_scale = bool(torch.isfinite(sc).all() and (sc > 1e-6).all() and (sc < 1e3).all())
            if self.fp8:
                v = oq.view(torch.uint8)[rows]
                sat = float(((v & 0x7F) >= 0x7E).float().mean())
                return {"ok": ok_scale and sat < 0.2, "scales_finite_in_range": ok_scale, "saturated_code_fraction": round(sat, 5)}
            q = oq[rows].to(torch.int16).abs()
            reach = bool((q.amax(dim=1) == 127).all())
            sat = float((q == 127).float().mean())
            return {"ok": ok_scale and reach and sat < 0.2, "scales_finite_in_range": ok_scale,
                    "every_row_reaches_127": reach, "saturated_code_fraction": round(sat, 5)}
        h = self.h.float()
        fin = bool(torch.isfinite(h).all())
        rms = float(h.pow(2).mean().sqrt()) if fin else float("nan")
        return {"ok": fin and 0.1 < rms < 100.0, "finite": fin, "rms": round(rms, 3)}

    def tokens_layers_per_step(self):
        sh = self.shape
        return self.T * self.layers * (sh.steps if self.caches is not None else 1)


def fc1_roofline(hero, shape, seed, iters=40, tile=None):
    """The dominant kernel alone, under the conditions it meets in the stack: FC1 GeMM^quant + GELU^quant at the
    workload's shape, its operands rotating over more buffers than the 256 MB memory-side cache holds (in the stack
    every layer brings its own weights from HBM; with one resident set the kernel looks 10 % faster than it is there),
    timed after 60 ms of back-to-back launches (after an idle period the first ~35 ms of launches run up to 25 %
    slower, and the stack is timed long after that), events only, no host synchronisation between the repeats."""
    import torch
    from paper_2310_17723_amd import binding as HB, synth
    M, K, N = shape.B * shape.S, shape.d, shape.f
    c = synth.gemm_case(seed, M, K, N)
    A0, B0 = torch.from_numpy(c["A"]).cuda(), torch.from_numpy(c["Bt"]).cuda()
    rs, cs, bias = (torch.from_numpy(c[k]).cuda() for k in ("a_row_scale", "b_col_scale", "bias"))
    cs = cs * (30.0 / K ** 0.5)
    sa = torch.full((N,), 0.03, dtype=torch.float32, device="cuda")
    n_w, n_a, n_c = max(2, (128 << 20) // (N * K)), max(2, (128 << 20) // (M * K)), max(2, (192 << 20) // (M * N))
    As, Bs = [A0.clone() for _ in range(n_a)], [B0.clone() for _ in range(n_w)]
    Cs = [torch.empty((M, N), dtype=torch.int8, device="cuda") for _ in range(n_c)]
    count = [0]

    def fn():
        i = count[0] = count[0] + 1
        hero.hero_int8_gemm(As[i % n_a], Bs[i % n_w], rs, cs, bias, epi=HB.EPI_GELU_REQUANT, out_col_scale=sa,
                            C_out=Cs[i % n_c], tile=tile)
    fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    ev[0].record()
    fn()
    ev[1].record()
    torch.cuda.synchronize()
    for _ in range(min(600, max(20, int(60.0 / ev[0].elapsed_time(ev[1]))))):      # about 60 ms of device time, queued
        fn()
    ev[0].record()
    for r in range(5):
        for _ in range(iters):
            fn()
        ev[r + 1].record()
    torch.cuda.synchronize()
    ms = float(np.median([ev[r].elapsed_time(ev[r + 1]) / iters for r in range(5)]))
    ops = 2.0 * M * N * K
    tops = ops / (ms * 1e-3) / 1e12
    return {"bound": "mfma", "kernel": ("int8_gemm_ovl_kernel" if K < 2048 and tile in (None, 9) else "int8_gemm_persistent_kernel") + "<GELU_REQUANT> (FC1)", "shape_mnk": [M, N, K],
            "achieved": round(tops, 2), "peak": PEAK_INT8_TOPS, "unit": "TOP/s", "frac": round(tops / PEAK_INT8_TOPS, 4),
            "avg_launch_us": round(ms * 1e3, 2), "ops_per_launch": ops,
            "timing": f"median of 5 x {iters} back-to-back launches after 60 ms of them, HIP events; operands rotate over {n_a} / {n_w} / {n_c} buffers (A / W / C)",
            "algorithmic_bytes": M * K + N * K + M * N + 4 * (M + 3 * N),
            "traffic": measured_traffic(f"fc1_gelu_requant_{M}x{N}x{K}")}


def measured_ceilings():
    """What this machine sustains, beside the nameplate peaks the fractions are quoted against, from the
    instruments of libhero_probe (a library of its own, loaded only here).  Matrix cores: a register-only INT8
    MFMA loop on near-constant and on random operand bytes (the clock under the matrix cores is power-limited and
    depends on the data), and the same loop with 4 / 8 fp32 vector instructions behind every matrix instruction of
    a wave, or in the other wave of the SIMD (does the vector ALU issue while the matrix pipe is busy?).  HBM: five
    instruments on 256 MiB buffers (read only, write only, copy with 1 and with 4 independent 16-byte loads in
    flight per lane, the runtime's device-to-device copy) and a copy of one LN^quant call's volume on rotating buffers."""
    import torch
    from paper_2310_17723_amd.probe import Probe
    pr = Probe()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = {}
    for name, rnd in (("mfma_int8_constant_operands_tops", 0), ("mfma_int8_random_operands_tops", 1)):
        ops = [0.0]

        def fn():
            ops[0] = pr.mfma_i8(rnd, 2048, sink)
        ms = time_gpu(fn, 5, warmup=2, repeats=3)
        out[name] = round(ops[0] / (ms * 1e-3) / 1e12, 1)
    co = {}
    for name, mode, V in (("mfma_only", 0, 0), ("valu4_only", 1, 4), ("valu8_only", 1, 8), ("in_wave_mfma_valu4", 0, 4),
                          ("in_wave_mfma_valu8", 0, 8), ("cross_wave_mfma_valu4", 2, 4), ("cross_wave_mfma_valu8", 2, 8)):
        ms = time_gpu(lambda: pr.coissue(mode, V, 1000, sink), 3, warmup=1, repeats=3)
        co[name + "_us"] = round(ms * 1e3, 1)
    co["hidden_fraction_in_wave_valu4"] = round(1.0 - (co["in_wave_mfma_valu4_us"] - co["mfma_only_us"]) / co["valu4_only_us"], 3)
    co["hidden_fraction_in_wave_valu8"] = round(1.0 - (co["in_wave_mfma_valu8_us"] - co["mfma_only_us"]) / co["valu8_only_us"], 3)
    co["hidden_fraction_cross_wave_valu4"] = round(1.0 - (co["cross_wave_mfma_valu4_us"] - co["mfma_only_us"]) / co["valu4_only_us"], 3)
    out["mfma_valu_coissue"] = co
    n = 256 << 20
    src = torch.randint(-127, 128, (n,), dtype=torch.int8, device="cuda")
    dst = torch.empty_like(src)
    gbs = lambda moved, ms: round(moved / (ms * 1e-3) / 1e9, 1)
    out["hbm_read_only_256MiB_gbs"] = gbs(n, time_gpu(lambda: pr.read(src, sink), 5, warmup=2, repeats=3))
    out["hbm_write_only_256MiB_gbs"] = gbs(n, time_gpu(lambda: pr.write(dst), 5, warmup=2, repeats=3))
    out["copy_256MiB_gbs"] = gbs(2 * n, time_gpu(lambda: pr.copy(src, dst, 1), 5, warmup=2, repeats=3))      # read + write
    out["copy_256MiB_4_loads_in_flight_gbs"] = gbs(2 * n, time_gpu(lambda: pr.copy(src, dst, 4), 5, warmup=2, repeats=3))
    out["hip_memcpy_dtod_256MiB_gbs"] = gbs(2 * n, time_gpu(lambda: pr.memcpy(src, dst), 5, warmup=2, repeats=3))
    del src, dst
    # a copy that moves what one LN^quant call of the bench moves (48 MiB), on rotating buffers like that leg
    n, nbuf = 24 << 20, 8
    bufs = [(torch.randint(-127, 128, (n,), dtype=torch.int8, device="cuda"), torch.empty(n, dtype=torch.int8, device="cuda"))
            for _ in range(nbuf)]
    i = [0]

    def cp():
        a, b = bufs[i[0] % nbuf]
        i[0] += 1
        pr.copy(a, b, 4)
    ms = time_gpu(cp, 40, warmup=nbuf, graph=True, repeats=5)
    out["copy_24MiB_rotating_gbs"] = round(2.0 * n / (ms * 1e-3) / 1e9, 1)
    out["hbm_best_copy_gbs"] = max(out["copy_256MiB_gbs"], out["copy_256MiB_4_loads_in_flight_gbs"], out["hip_memcpy_dtod_256MiB_gbs"])
    return out


def gemm_sweep(hero, seed, iters=10):
    import torch
    from paper_2310_17723_amd import binding as HB, synth
    rows = []
    for (K, N) in synth.GEMM_KN:
        for M in synth.GEMM_M:
            c = synth.gemm_case(seed, M, K, N)
            A, Bt = torch.from_numpy(c["A"]).cuda(), torch.from_numpy(c["Bt"]).cuda()
            rs, cs, bias = (torch.from_numpy(c[k]).cuda() for k in ("a_row_scale", "b_col_scale", "bias"))
            for name, epi, dt in (("fp16", HB.EPI_DEQUANT, torch.float16), ("int8", HB.EPI_REQUANT, torch.int8)):
                out = torch.empty((M, N), dtype=dt, device="cuda")
                ms = time_gpu(lambda: hero.hero_int8_gemm(A, Bt, rs, cs, bias, epi=epi, C_out=out), iters, graph=True)
                tops = 2.0 * M * N * K / (ms * 1e-3) / 1e12
                rows.append({"M": M, "K": K, "N": N, "out": name, "us": round(ms * 1e3, 2), "tops": round(tops, 1),
                             "frac_peak": round(tops / PEAK_INT8_TOPS, 4)})
    return rows


def gemm_cpu_baseline(seed):
    """The oracle's GeMM^quant beside the config-1 sweep: M = 512 in full, and 64 seeded output rows of the M = 8192
    problem (the oracle computes row by row, so the rate of a sample of rows is the rate of the problem)."""
    import oracle as O
    from paper_2310_17723_amd import synth
    out = []
    K, N = synth.GEMM_KN[0]
    for M, rows, what in ((512, 512, "in full"), (8192, 64, "64 seeded output rows")):
        c = synth.gemm_case(seed, M, K, N)
        sel = np.sort(synth.rng(seed + M).choice(M, rows, replace=False)) if rows < M else np.arange(M)
        A, rs = np.ascontiguousarray(c["A"][sel]), np.ascontiguousarray(c["a_row_scale"][sel])
        t0 = time.perf_counter()
        O.int8_gemm(A, c["Bt"], a_row_scale=rs, b_col_scale=c["b_col_scale"], bias=c["bias"], epi=O.EPI_REQUANT, c_dt=O.I8)
        dt = time.perf_counter() - t0
        out.append({"value": round(2.0 * rows * N * K / dt / 1e9, 2), "unit": "GOP/s", "cores": O.num_threads(), "kind": "oracle",
                    "sample": f"REQUANT {M}x{N}x{K}: {what}", "seconds": round(dt, 3)})
    return out


def fp8_gemm_leg(hero, shape, seed, iters=20):
    """The FP8 variant of the layer's two big GEMMs (Sec. 2.1 names FP8 as the alternative 8-bit format):
    E4M3 operands from Gaussian data under token-wise / column-wise scales, E4M3 outputs."""
    import torch
    from paper_2310_17723_amd import binding as HB
    g = torch.Generator(device="cuda").manual_seed(seed)
    M, d, f = shape.B * shape.S, shape.d, shape.f
    rows = []
    for name, N, K, epi in (("FC1 GELU^quant", f, d, HB.EPI_GELU_REQUANT), ("FC2 requant", d, f, HB.EPI_REQUANT)):
        X = torch.randn((M, K), device="cuda", generator=g)
        W = torch.randn((N, K), device="cuda", generator=g) * 0.03
        rs = X.abs().amax(dim=1) / 448
        cs = W.abs().amax(dim=1) / 448
        A = (X / rs[:, None]).to(torch.float8_e4m3fn)
        Bt = (W / cs[:, None]).to(torch.float8_e4m3fn)
        bias = torch.randn(N, device="cuda", generator=g) * 0.02
        s_out = torch.full((N,), 0.03, dtype=torch.float32, device="cuda")
        cs2 = cs / 0.05 if epi == HB.EPI_REQUANT else cs
        out = torch.empty((M, N), dtype=torch.float8_e4m3fn, device="cuda")
        ms = time_gpu(lambda: hero.hero_fp8_gemm(A, Bt, rs, cs2, bias, epi=epi, out_col_scale=s_out, C_out=out), iters)
        tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        rows.append({"gemm": name, "shape_mnk": [M, N, K], "us": round(ms * 1e3, 2), "tflops": round(tf, 1),
                     "peak": PEAK_FP8_TFLOPS, "frac_peak": round(tf / PEAK_FP8_TFLOPS, 4)})
    return rows


def fp8_layer_leg(hero, shape, seed, iters=10):
    """One layer of the workload in the FP8 variant (mode bit M_FP8: E4M3 codes in every 8-bit buffer).  Timing
    only: Gaussian weights quantized column-wise to E4M3 here with torch, static scales set to the ranges such a
    layer has (its parity against the oracle's FP8 layer is in the tests); prefill workloads only."""
    import torch
    from paper_2310_17723_amd import binding as HB
    g = torch.Generator(device="cuda").manual_seed(seed + 7)
    B, S, d, f, H, Dh = shape.B, shape.S, shape.d, shape.f, shape.H, shape.Dh
    T = B * S

    def wq(N, K, std):
        W = torch.randn((N, K), device="cuda", generator=g) * std
        cs = W.abs().amax(dim=1) / 448
        return (W / cs[:, None]).to(torch.float8_e4m3fn), cs

    t = {}
    t["w_qkv"], t["w_qkv_s"] = wq(3 * d, d, 0.02)
    t["w_o"], t["w_o_s"] = wq(d, d, 0.02)
    t["w_1"], t["w_1_s"] = wq(f, d, 0.02)
    t["w_2"], t["w_2_s"] = wq(d, f, 0.02)
    t["w_qkv_s"] = t["w_qkv_s"] * 4.0                    # folded 1 / S_{q,k,v}: codes spread over the E4M3 range
    for n, k in (("b_qkv", 3 * d), ("b_o", d), ("b_1", f), ("b_2", d)):
        t[n] = torch.randn(k, device="cuda", generator=g) * 0.02
    for n in ("ln1_g", "ln2_g"):
        t[n] = torch.ones(d, device="cuda")
    for n in ("ln1_b", "ln2_b"):
        t[n] = torch.zeros(d, device="cuda")
    t["S_o"] = torch.full((d,), 2.0 / 448, device="cuda")
    t["S_x2"] = torch.full((d,), 2.0 / 448, device="cuda")
    t["S_a"] = torch.full((f,), 4.0 / 448, device="cuda")
    t["attn_out_scale"] = torch.full((d,), 1.0 / 448 * 4.0, device="cuda")
    W = hero.layer_weights(t, 1.5 / (100 * 100 * Dh ** 0.5), 1.0 / 448)
    desc = hero.layer_desc(shape.arch, d, H, Dh, f, shape.eps, shape.mask, HB.MODE_M3 | HB.M_FP8)
    ws = torch.empty(hero.hero_layer_workspace_bytes(desc, B, S), dtype=torch.uint8, device="cuda")
    kvl = None
    if shape.mask == 1:
        kvl = torch.randint(shape.kv_lo or S // 2, (shape.kv_hi or S) + 1, (B,), dtype=torch.int32, device="cuda", generator=g)
    h0 = torch.randn((T, d), device="cuda", generator=g).to(torch.bfloat16)
    if shape.arch == 0:
        xq, xs, _ = hero.hero_ln_quant(h0, None, None, None, t["ln1_g"], t["ln1_b"], shape.eps, fp8=True)
        oq, os_ = torch.empty_like(xq), torch.empty_like(xs)
        fn = lambda: hero.hero_layer_fwd(desc, W, B, S, ws, x_q=xq, x_scale=xs, out_q=oq, out_scale=os_, kv_len=kvl)
    else:
        h = h0.clone()
        fn = lambda: hero.hero_layer_fwd(desc, W, B, S, ws, h=h)
    ms = time_gpu(fn, iters)
    return {"workload": shape.name, "mode": "M3 + FP8 (E4M3)", "us_per_layer": round(ms * 1e3, 2),
            "layer_tokens_per_s": round(T / (ms * 1e-3), 1)}


def attn_variants(hero, shape, seed, iters=20):
    """The attention kernel alone at the workload's shape: the two-pass Softmax^quant of Sec. 2.2.2 (what the
    layer runs) beside the single-sweep online variant (a different quantization of the probabilities) and the
    FP8 variant of the two-pass flow."""
    import torch
    from paper_2310_17723_amd import binding as HB
    g = torch.Generator(device="cuda").manual_seed(seed)
    B, S, H, Dh = shape.B, shape.S, shape.H, shape.Dh
    d = H * Dh
    qkv = torch.clamp(torch.round(torch.randn((B * S, 3 * d), device="cuda", generator=g) * 30), -127, 127).to(torch.int8)
    v = qkv.view(B, S, 3, H, Dh)
    cs = torch.full((d,), 0.005, device="cuda")
    kvl = None
    if shape.mask == 1:
        kvl = torch.randint(shape.kv_lo or S // 2, (shape.kv_hi or S) + 1, (B,), dtype=torch.int32, device="cuda", generator=g)
    out = torch.empty((B * S, d), dtype=torch.int8, device="cuda")
    dt = 4.0 / (30 * 30 * Dh)                                   # logits of a few units
    dth = torch.full((H,), dt, device="cuda")
    ops = 4.0 * B * H * S * S * Dh * (0.5 if shape.mask == 2 else 1.0)
    res = {"shape_bshd": [B, S, H, Dh], "mask": ["none", "padding", "causal"][shape.mask], "useful_ops": ops}
    if kvl is not None:
        # padded positions neither ask nor are asked: the fraction of the S x S (query, key) pairs that are computed
        res["real_pair_fraction"] = round(float((kvl.double() ** 2).mean().item()) / (S * S), 4)
    ms = time_gpu(lambda: hero.hero_int8_attn(v[:, :, 0], v[:, :, 1], v[:, :, 2], dt, 1 / 255, cs, mask=shape.mask,
                                              kv_len=kvl, out=out), iters)
    res["two_pass_us"] = round(ms * 1e3, 2)
    ms = time_gpu(lambda: hero.hero_int8_attn_online(v[:, :, 0], v[:, :, 1], v[:, :, 2], dth, 1 / 255, cs, mask=shape.mask,
                                                     kv_len=kvl, out=out), iters)
    res["online_us"] = round(ms * 1e3, 2)
    q8 = (torch.randn((B * S, 3 * d), device="cuda", generator=g) * 40).to(torch.float8_e4m3fn)
    v8 = q8.view(B, S, 3, H, Dh)
    out8 = torch.empty((B * S, d), dtype=torch.float8_e4m3fn, device="cuda")
    ms = time_gpu(lambda: hero.hero_fp8_attn(v8[:, :, 0], v8[:, :, 1], v8[:, :, 2], 1.5 / (40 * 40 * Dh ** 0.5), 1 / 448, cs,
                                             mask=shape.mask, kv_len=kvl, out=out8), iters)
    res["fp8_two_pass_us"] = round(ms * 1e3, 2)
    return res


def ln_bandwidth(hero, T, D, iters=40, nbuf=8):
    """Fused LN + per-token quant on rotating buffers (working set >> the 256 MB cache)."""
    import torch
    g = torch.Generator(device="cuda").manual_seed(1)
    sets = []
    for _ in range(nbuf):
        x = torch.randint(-127, 128, (T, D), dtype=torch.int8, device="cuda", generator=g)
        r = torch.randint(-127, 128, (T, D), dtype=torch.int8, device="cuda", generator=g)
        xs = torch.rand(T, device="cuda", generator=g) * 0.04 + 0.01
        sets.append((x, r, xs, torch.empty_like(x), torch.empty(T, device="cuda")))
    rc = torch.rand(D, device="cuda", generator=g) * 0.02 + 0.001
    gam = torch.ones(D, device="cuda")
    bet = torch.zeros(D, device="cuda")
    i = [0]

    def fn():
        x, r, xs, yq, ys = sets[i[0] % nbuf]
        i[0] += 1
        hero.hero_ln_quant(x, xs, r, rc, gam, bet, 1e-12, y_q=yq, y_scale=ys)
    ms = time_gpu(fn, iters, warmup=nbuf, graph=True)            # replays of a HIP graph: no host time in the figure
    bytes_ = T * (3 * D + 8)
    gbs = bytes_ / (ms * 1e-3) / 1e9
    return {"T": T, "D": D, "form": "int8+int8->int8", "us": round(ms * 1e3, 2), "bytes_per_launch": bytes_,
            "gbs": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4), "working_set_mb": nbuf * bytes_ // 2 ** 20,
            "timing": f"median of 5 replays of a HIP graph of {iters} launches on {nbuf} rotating buffer sets",
            "counters": measured_traffic(f"ln_quant_{T}x{D}")}


def embed_bandwidth(hero, B, S, D, V=30522, iters=40, nbuf=8):
    """Embedding LN^quant (Sec. 2.2.1): INT8 token-table gather + bf16 position / type rows -> LN -> TWQ INT8.
    Algorithmic bytes: one INT8 table row, its scale and three ids read and one INT8 row + scale written per
    token, the position / type tables once."""
    import torch
    from paper_2310_17723_amd import synth
    T = B * S
    g = torch.Generator(device="cuda").manual_seed(2)
    tok = torch.randint(-127, 128, (V, D), dtype=torch.int8, device="cuda", generator=g)
    ts = torch.rand(V, device="cuda", generator=g) * 1e-3 + 1e-4
    pos = (torch.randn((S, D), device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    typ = (torch.randn((2, D), device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    gam = torch.ones(D, device="cuda")
    bet = torch.zeros(D, device="cuda")
    sets = []
    for k in range(nbuf):
        ids = synth.embedding_ids(100 + k, B, S, V, 2)
        sets.append((torch.from_numpy(ids["tok"]).cuda(), torch.from_numpy(ids["pos"]).cuda(), torch.from_numpy(ids["type"]).cuda(),
                     torch.empty((T, D), dtype=torch.int8, device="cuda"), torch.empty(T, device="cuda")))
    i = [0]

    def fn():
        a, b, c, yq, ys = sets[i[0] % nbuf]
        i[0] += 1
        hero.hero_embed_ln_quant(a, b, c, tok, ts, pos, typ, gam, bet, 1e-12, y_q=yq, y_scale=ys)
    ms = time_gpu(fn, iters, warmup=nbuf, graph=True)
    bytes_ = T * (2 * D + 20) + (S + 2) * D * 2
    gbs = bytes_ / (ms * 1e-3) / 1e9
    return {"T": T, "D": D, "vocab": V, "form": "int8 table + bf16 tables -> int8", "us": round(ms * 1e3, 2),
            "bytes_per_launch": bytes_, "gbs": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4),
            "timing": f"median of 5 replays of a HIP graph of {iters} launches on {nbuf} rotating id / output sets"}


def cpu_baseline(shape, seed, mode_name="M3", prepared=None):
    """The oracle, as it stands, timed on a bounded slice of the workload (the forward passes only; calibration
    and weight preparation are outside the clock).  Slices: BERT-base in full; BERT-large one sequence x 512
    tokens through all 24 layers (M3) or one layer (M1); GPT prefill one sequence x 2048 tokens through one layer;
    GPT decode two batch rows x 4 steps against a 2048-key cache through one layer.  `prepared`: oracle weights
    of the same model to reuse (the decode slice takes the prefill slice's).  Returns (record, prepared)."""
    import oracle as O
    from oracle import layer as OL
    from paper_2310_17723_amd import synth
    decode = shape.cache_len > 0
    mode = {"M1": OL.MODE_M1, "M2": OL.MODE_M2, "M3": OL.MODE_M3}[mode_name]
    if decode:
        B, S, L = 2, 1, 1
    elif shape.d > 1024:
        B, S, L = 1, shape.S, 1
    elif shape.layers > 1:
        B, S, L = 1, shape.S, (shape.layers if mode_name == "M3" else 1)
    else:
        B, S, L = shape.B, shape.S, 1
    sh = synth.small(shape, B=B, S=S)
    emb = synth.embedding_ln_params(seed, sh)
    if prepared is None:
        Sc = 128
        xc = synth.activations(seed, sh, Sc, stream=1).astype(np.float64)
        if sh.arch == synth.POST_LN:
            xc = OL._ln64(xc, emb["g"].astype(np.float64), emb["b"].astype(np.float64), sh.eps)
        cal = synth.small(sh, mask=synth.MASK_NONE if sh.mask == synth.MASK_PADDING else sh.mask)
        if decode:
            cal = synth.small(cal, mask=synth.MASK_CAUSAL)
        prepared = []
        for l in range(L):
            p = synth.layer_params(seed, sh, l)
            sc, xc = OL.calibrate(p, xc, cal, 1, Sc)
            prepared.append(OL.prepare(p, sc, sh, mode))
            del p
    h0 = synth.activations(seed, sh, B * S)
    steps = 1
    t0 = time.perf_counter()
    if sh.arch == synth.POST_LN:
        xq, xs, _ = O.ln_quant(h0, O.F32, None, None, 0, None, emb["g"], emb["b"], sh.eps)
        kv = np.full(B, S, np.int32) if sh.mask == synth.MASK_PADDING else None
        for l in range(L):
            xq, xs = OL.layer_fwd(prepared[l], sh, B, S, x_q=xq, x_s=xs, kv_len=kv)
        sample = f"{B} sequence(s) x {S} tokens through {L} layer(s) of {shape.name} ({mode_name})"
    elif not decode:
        OL.layer_fwd(prepared[0], sh, B, S, h=O.f32_to_bf16(h0))
        sample = f"{B} sequence x {S} tokens through 1 layer of {shape.name}"
    else:
        steps = 4
        Smax = shape.cache_len + steps
        cache = {"k": synth.int8_codes(seed, (B, sh.H, Smax, sh.Dh), 0), "v": synth.int8_codes(seed, (B, sh.H, Smax, sh.Dh), 1)}
        t0 = time.perf_counter()
        for t in range(steps):
            OL.layer_fwd(prepared[0], sh, B, 1, h=O.f32_to_bf16(h0), kv_len=np.full(B, shape.cache_len + t + 1, np.int32), cache=cache)
        sample = f"{B} sequences x {steps} decode steps (cache {shape.cache_len}) through 1 layer of {shape.name}"
    dt = time.perf_counter() - t0
    return ({"value": round(B * S * L * steps / dt, 2), "unit": "layer-tokens/s", "cores": O.num_threads(), "kind": "oracle",
             "sample": sample, "seconds": round(dt, 2)}, prepared)


def time_stack(st, steps, repeats=5, graph=False):
    """ms per pass of the stack: HIP events around `steps` passes, median of `repeats`."""
    import torch
    st.step()
    torch.cuda.synchronize()
    run = st.step
    if graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            st.step()
        g.replay()
        torch.cuda.synchronize()
        run = g.replay
    ts = []
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            run()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) / steps)
    return float(np.median(ts)), [round(t, 4) for t in ts]


def workload_record(st, ms_per_step, mode_name, graph, launches=None):
    sh = st.shape
    decode = st.caches is not None
    per_layer_us = ms_per_step * 1e3 / (st.layers * (sh.steps if decode else 1))
    tps = st.tokens_layers_per_step() / (ms_per_step * 1e-3)
    rec = {"workload": sh.name, "mode": mode_name, "layers": st.layers, "tokens_per_step": st.T * (sh.steps if decode else 1),
           "hip_graph": bool(graph), "ms_per_step": round(ms_per_step, 4), "us_per_layer": round(per_layer_us, 2),
           "layer_tokens_per_s": round(tps, 1), "timing": "median of 5 repeats, HIP events around whole passes"}
    bound = LAYER_BOUND.get(sh.name)
    if bound:
        rec["roofline_bound_layer_tokens_per_s"] = bound
        rec["frac_of_bound"] = round(tps / bound, 4)
    if launches:
        rec["launches_per_layer"] = launches
    rec["sanity"] = st.sanity()
    return rec


def other_workloads(hero, seed):
    """Configs 0, 3, 4 and config 2 in the mixed mode M1 (attention core, attention-output linear and FC2 in BF16):
    each timed like the headline stack, each with the oracle beside it on its own slice."""
    import torch
    from paper_2310_17723_amd import binding as HB, synth
    out = {}
    # ---- config 2, M1
    log("[bench] config 2 in M1 (BF16 attention / attention-output / FC2)")
    sh = synth.CONFIGS[2]
    st = Stack(hero, sh, seed, HB.MODE_M1)
    ms, _ = time_stack(st, 3)
    out["bert-large-32x512_M1"] = workload_record(st, ms, "M1", False)
    del st
    torch.cuda.empty_cache()
    out["bert-large-32x512_M1"]["cpu_baseline"], _ = cpu_baseline(sh, seed, "M1")
    # ---- config 0: eager and as a HIP graph (9 launches of a few microseconds each)
    log("[bench] config 0 (BERT-base 1 x 128): eager and HIP graph")
    sh = synth.CONFIGS[0]
    st = Stack(hero, sh, seed, HB.MODE_M3)
    ms, _ = time_stack(st, 50)
    out["bert-base-1x128_eager"] = workload_record(st, ms, "M3", False, launches=9)
    ms, _ = time_stack(st, 50, graph=True)
    out["bert-base-1x128_graph"] = workload_record(st, ms, "M3", True, launches=9)
    del st
    cb, _ = cpu_baseline(sh, seed, "M3")
    out["bert-base-1x128_eager"]["cpu_baseline"] = cb
    out["bert-base-1x128_graph"]["cpu_baseline"] = cb
    # ---- config 3, then config 4 on the same prepared layers
    log("[bench] config 3 (GPT prefill 8 x 2048, d 4096, 4 layers)")
    sh3, sh4 = synth.CONFIGS[3], synth.CONFIGS[4]
    st3 = Stack(hero, sh3, seed, HB.MODE_M3)
    ms, _ = time_stack(st3, 2)
    out["gpt-prefill-8x2048"] = workload_record(st3, ms, "M3", False)
    log("[bench] config 4 (GPT decode 64 x 1 against a 2048-token INT8 cache, 128 steps, 4 layers)")
    st4 = Stack(hero, sh4, seed, HB.MODE_M3, share=st3)
    st3.ws = st3.h = st3.h0 = None
    torch.cuda.empty_cache()
    ms, _ = time_stack(st4, 1, repeats=3)
    out["gpt-decode-64x1"] = workload_record(st4, ms, "M3", False)
    out["gpt-decode-64x1"]["timing"] = "median of 3 repeats of the 128-step pass"
    del st3, st4
    torch.cuda.empty_cache()
    log("[bench] CPU oracle on the config 3 / 4 slices")
    out["gpt-prefill-8x2048"]["cpu_baseline"], prepared = cpu_baseline(sh3, seed, "M3")
    out["gpt-decode-64x1"]["cpu_baseline"], _ = cpu_baseline(sh4, seed, "M3", prepared=prepared)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="bert-large", choices=sorted(WORKLOADS))
    ap.add_argument("--mode", default="M3", choices=["M1", "M2", "M3"])
    ap.add_argument("--layers", type=int, default=None, help="override the stack depth")
    ap.add_argument("--seed", type=int, default=2310)
    ap.add_argument("--no-extras", action="store_true", help="skip the GEMM sweep / LN / other-workload / CPU legs")
    ap.add_argument("--no-workloads", action="store_true", help="skip the legs of the other configs (0, 3, 4, config 2 in M1)")
    ap.add_argument("--fp8", action="store_true",
                    help="run the stack in the FP8 variant (E4M3 codes in every 8-bit buffer; mode M3 only)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one pass of the stack in a HIP graph and time its replays (launch-bound workloads)")
    ap.add_argument("--only", default=None, choices=["ln", "coissue", "fc1", "attention"],
                    help="run one leg alone and print its record (for rocprofv3 counter runs): the LN^quant bandwidth legs, "
                         "the MFMA + VALU co-issue probe, the FC1 GeMM^quant (with --tile), the attention kernels")
    ap.add_argument("--tile", type=int, default=None, help="with --only fc1: force a GEMM kernel through the test hook (7, 8, 9)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy 5 times (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards without exchange along tokens; "
              "no collective is built) -- run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2310_17723_amd as pkg
    from paper_2310_17723_amd import binding as HB, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    if args.copy_calibration:
        src = torch.randint(-127, 128, (256 << 20,), dtype=torch.int8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 256 << 20, "copy_bytes_written": 256 << 20, "launches": 5}))
        return
    hero = pkg.load()                     # raises if libhero.so is missing: no fallback
    shape = synth.CONFIGS[WORKLOADS[args.workload]]
    if args.only == "ln":
        print(json.dumps({"ln_quant": ln_bandwidth(hero, 16384, shape.d), "ln_quant_large": ln_bandwidth(hero, 65536, shape.d, nbuf=4),
                          "embed_ln_quant": embed_bandwidth(hero, 32, 512, shape.d)}))
        return
    if args.only == "coissue":
        from paper_2310_17723_amd.probe import Probe
        pr, sink = Probe(), torch.zeros(1, dtype=torch.int32, device="cuda")
        for mode, V in ((0, 0), (1, 4), (1, 8), (0, 4), (0, 8), (2, 4), (2, 8)):
            pr.coissue(mode, V, 1000, sink)
            pr.coissue(mode, V, 1000, sink)
        torch.cuda.synchronize()
        print(json.dumps({"launched": "probe_coissue_kernel<mode, V> twice each: (0,0) (1,4) (1,8) (0,4) (0,8) (2,4) (2,8), 1000 iterations"}))
        return
    if args.only == "fc1":
        print(json.dumps(fc1_roofline(hero, shape, args.seed, tile=args.tile)))
        return
    if args.only == "attention":
        print(json.dumps(attn_variants(hero, shape, args.seed)))
        return
    mode = {"M1": HB.MODE_M1, "M2": HB.MODE_M2, "M3": HB.MODE_M3}[args.mode]
    decode = shape.cache_len > 0
    steps = args.steps if args.steps is not None else (1 if decode else 10)
    # default warm-up: long enough (about 45 ms of the BERT-large stack) that the timed steps begin behind the slow
    # first ~35 ms this GPU shows after every idle period (see time_gpu)
    warmup = args.warmup if args.warmup is not None else (1 if decode else 6)

    log(f"[bench] preparing {shape.name} ({args.mode}) ...")
    if args.fp8 and args.mode != "M3":
        print("bench.py: --fp8 runs every module in 8 bits (mode M3)", file=sys.stderr)
        sys.exit(2)
    st = Stack(hero, shape, args.seed, mode, args.layers, fp8=args.fp8)
    log("[bench] warm-up")
    for _ in range(warmup):
        st.step()
    torch.cuda.synchronize()
    run = st.step
    if args.graph:
        # every launch of the stack goes to the current stream and nothing allocates, so the pass can be
        # captured as it is; the replays then cost one launch
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            st.step()
        graph.replay()
        torch.cuda.synchronize()
        run = graph.replay
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = e0.elapsed_time(e1) / steps
    tl = st.tokens_layers_per_step()
    value = tl / (ms_per_step * 1e-3)
    sanity = st.sanity()
    if not sanity["ok"]:
        print(f"bench.py: the timed stack left implausible outputs behind: {sanity}", file=sys.stderr)
        sys.exit(4)
    # four more timings of the same K steps: `value` is the first one (the contract's K steps), the spread is reported
    reps = [round(ms_per_step, 4)]
    for _ in range(4 if not decode else 0):
        e0.record()
        for _ in range(steps):
            run()
        e1.record()
        torch.cuda.synchronize()
        reps.append(round(e0.elapsed_time(e1) / steps, 4))

    rec = {
        "metric": "W8A8 layer tokens/s", "value": round(value, 1), "unit": "layer-tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f8e4m3" if args.fp8 else "int8", "data": "synthetic",
        "config": {"workload": shape.name, "arch": "post-LN" if shape.arch == 0 else "pre-LN", "mode": args.mode + ("+FP8" if args.fp8 else ""),
                   "layers": st.layers, "batch": shape.B, "seq_len": shape.S, "hidden": shape.d, "heads": shape.H,
                   "ffn": shape.f, "tokens_per_step": st.T * (shape.steps if decode else 1),
                   "mask": ["none", "padding", "causal"][shape.mask], "hip_graph": bool(args.graph)},
        "stack_tokens_per_s": round(value / st.layers, 1),
        "us_per_layer": round(ms_per_step * 1e3 / (st.layers * (shape.steps if decode else 1)), 2),
        "wall_ms_timed_region": round(wall_ms, 2),
        "ms_per_step_repeats": reps, "ms_per_step_median": round(float(np.median(reps)), 4),
        "sanity": sanity,
    }
    if st.kv_len is not None:
        real = int(st.kv_len.sum().item())
        rec["real_token_fraction"] = round(real / st.T, 4)
    log("[bench] dominant kernel alone (FC1 GeMM^quant + GELU^quant)")
    rec["roofline"] = fc1_roofline(hero, shape, args.seed)
    if not args.no_extras:
        log("[bench] LN^quant bandwidth")
        rec["ln_quant"] = ln_bandwidth(hero, max(st.T, 16384), shape.d)
        rec["ln_quant_large"] = ln_bandwidth(hero, 65536, shape.d, nbuf=4)
        rec["embed_ln_quant"] = embed_bandwidth(hero, 32, 512, shape.d)
        if shape.S > 1:
            log("[bench] attention alone: two-pass and online Softmax^quant")
            rec["attention"] = attn_variants(hero, shape, args.seed)
        log("[bench] FP8 variant of the FC1 / FC2 GEMMs")
        rec["fp8_gemm"] = fp8_gemm_leg(hero, shape, args.seed)
        if not decode:
            log("[bench] FP8 variant of the whole layer")
            rec["fp8_layer"] = fp8_layer_leg(hero, shape, args.seed)
        log("[bench] measured ceilings (MFMA loops, MFMA + VALU co-issue, HBM streams)")
        rec["roofline"]["measured_ceilings"] = measured_ceilings()
        mc = rec["roofline"]["measured_ceilings"]
        # beside `frac` (against the nameplate peak): against what a register-only loop of the same matrix instruction
        # sustains on random operand bytes on this machine, right now
        rec["roofline"]["frac_of_measured_mfma_rate"] = round(rec["roofline"]["achieved"] / mc["mfma_int8_random_operands_tops"], 4)
        rec["ln_quant"]["frac_of_same_size_copy"] = round(rec["ln_quant"]["gbs"] / mc["copy_24MiB_rotating_gbs"], 4)
        rec["ln_quant_large"]["frac_of_best_large_copy"] = round(rec["ln_quant_large"]["gbs"] / mc["hbm_best_copy_gbs"], 4)
        log("[bench] GEMM sweep")
        rec["gemm_sweep"] = gemm_sweep(hero, args.seed)
        rec["gemm_sweep_cpu_baseline"] = gemm_cpu_baseline(args.seed)
        del st
        torch.cuda.empty_cache()
        log("[bench] CPU oracle baseline")
        rec["cpu_baseline"], _ = cpu_baseline(shape, args.seed, args.mode)
        if not args.no_workloads and args.workload == "bert-large" and args.mode == "M3" and not args.fp8:
            rec["workloads"] = other_workloads(hero, args.seed)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
