#!/usr/bin/env python3
"""Benchmark of the W4A16 GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload decode|mlp_decode|prefill|sweep|shapes|ceiling|companion|moe|w8|attn|epilogue|layer|pack|copy]
                    [--sweep-out FILE] [--no-cpu-baseline] [--no-prefill]

A "step" is one pass of the fused GEMM over every (layer, M) pair of the workload, weights already packed
(packing is the paper's offline stage and is timed separately, once).  Inputs are resident in HBM before the timed
region; every launch reads a different packed copy of its layer's weights, rotating through more than 512 MB per
layer, so that no launch finds its weights in L2 or in the 256 MB Infinity Cache.

Prints ONE JSON line.  `value` is the effective HBM bandwidth (algorithmic bytes / time) of the default decode
workload (K=4096, N in {4096, 12288}, M in {1, 4, 8, 16}); the prefill TFLOP/s is reported beside it.
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2516.6   # 256 CUs x 2.4 GHz x 4096 flop/clk/CU, dense
ROTATE_BYTES = 512 << 20
METRIC = "W4A16 GEMM TFLOP/s + effective HBM GB/s (% roofline), M=1..4096"

WORKLOADS = {
    # name: (list of (layer case name at its largest M, Ms))
    "decode": [("cfg2_attn_out_M16", (1, 4, 8, 16)), ("cfg2_qkv_M16", (1, 4, 8, 16))],
    "mlp_decode": [("cfg3_gate_up_M64", (1, 16, 32, 64)), ("cfg3_down_M64", (1, 16, 32, 64))],
    "prefill": [("cfg4_prefill_70b_mlp", (4096,))],
    "sweep5": [("cfg5_sweep_M1024", (1, 2, 4, 8, 32, 128, 256, 1024))],
    "tiny": [("cfg1_tiny_M1", (1,))],
}
# the five configurations of the benchmark, in order, as workload names
CONFIG_WORKLOADS = ("tiny", "decode", "mlp_decode", "prefill", "sweep5")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Layer:
    """One weight matrix: R packed copies on the device, X/Y buffers for each M."""

    def __init__(self, tm, torch, wl, case_name, Ms, rotate_bytes=ROTATE_BYTES):
        import numpy as np
        self.case = wl.case_by_name(case_name)
        c = self.case
        t0 = time.time()
        self.data = wl.make(c)
        self.gen_s = time.time() - t0
        d = self.data
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a.view(np.int32) if a.dtype == np.uint32 else a)).cuda()
        qw, s, z = dev(d["qweight"]), dev(d["s"]), dev(d["z"])
        wbytes = c.K * c.N // 2 + 4 * c.K * c.N // c.group
        self.copies = max(2, -(-rotate_bytes // wbytes))
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        self.packed = [tm.tm_pack_w4(qw, s, z, c.K, c.N, c.group)]          # first call also sets up the workspace
        torch.cuda.synchronize()
        e0.record()
        for _ in range(self.copies - 1):
            self.packed.append(tm.tm_pack_w4(qw, s, z, c.K, c.N, c.group))
        e1.record()
        torch.cuda.synchronize()
        self.pack_ms = e0.elapsed_time(e1) / max(1, self.copies - 1)
        self.Ms = tuple(Ms)
        Xfull = dev(d["X"])
        # several X/Y buffers per M so that activations rotate too
        self.X = {M: [Xfull[:M].clone() for _ in range(4)] for M in self.Ms}
        self.Y = {M: [torch.empty((M, c.N), dtype=torch.float16, device="cuda") for _ in range(4)] for M in self.Ms}
        self.turn = 0

    def launch(self, tm, M):
        i = self.turn
        self.turn += 1
        tm.tm_gemm_w4a16(self.X[M][i % 4], self.packed[i % self.copies], self.Y[M][i % 4])


# untimed graph replays before every timed region: about this many milliseconds of them, at most this many replays
WARM_MS = 20.0
WARM_REPLAYS_MAX = 400


def time_steps(torch, step_fn, steps, warmup, graph_steps=0):
    """Times exactly `steps` calls of step_fn between two events on the launch stream.

    graph_steps > 0: the steps are captured `graph_steps` at a time into a HIP graph and, after untimed replays that
    warm the device up, the graph is replayed steps / graph_steps times, which removes the host's per-launch cost (a
    decode kernel runs for a few microseconds, less than one eager launch costs the host) exactly as a serving loop
    would.  graph_steps must divide steps."""
    for _ in range(warmup):
        step_fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if graph_steps <= 0:
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            step_fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1), (time.perf_counter() - t0) * 1e3
    assert steps % graph_steps == 0
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(graph_steps):
                step_fn()
        # untimed replays, at least one and some milliseconds of them (WARM_MS): graph upload, caches and the clocks in steady state
        # (the first 5-10 ms after a host-side pause run 3-10 % slower than the steady state that follows)
        w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        w0.record()
        graph.replay()
        w1.record()
        torch.cuda.synchronize()
        for _ in range(min(WARM_REPLAYS_MAX, int(WARM_MS / max(w0.elapsed_time(w1), 0.05)))):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps // graph_steps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
    return e0.elapsed_time(e1), (time.perf_counter() - t0) * 1e3


def pick_graph_steps(steps, want):
    """largest divisor of `steps` that is <= want (>= 1)"""
    best = 1
    for g in range(1, min(steps, want) + 1):
        if steps % g == 0:
            best = g
    return best


def per_shape_table(tm, torch, wl, layers, iters=100, warmup=10, use_graph=True):
    rows = []
    for L in layers:
        c = L.case
        for M in L.Ms:
            ev_ms, _ = time_steps(torch, lambda: L.launch(tm, M), iters, warmup,
                                  graph_steps=iters if use_graph else 0)
            if ev_ms / iters < 0.05:
                # launches of a few microseconds come out 20-25 % slower now and then for a whole timed region (the
                # device's clocks after the idle stretch before a row): such rows are timed twice, the better one counts
                ev2, _ = time_steps(torch, lambda: L.launch(tm, M), iters, warmup, graph_steps=iters if use_graph else 0)
                ev_ms = min(ev_ms, ev2)
            t = ev_ms / iters * 1e-3
            B = wl.algorithmic_bytes(M, c.K, c.N, c.group)
            F = wl.flops(M, c.K, c.N)
            plan = tm.tm_get_plan(L.packed[0], M)
            hbm_frac, mfma_frac = B / t / 1e9 / HBM_PEAK_GBPS, F / t / 1e12 / MFMA_F16_PEAK_TFLOPS
            # the roofline that binds: HBM while the ideal HBM time exceeds the ideal matrix-core time (M below about 84)
            bound = "hbm" if B / (HBM_PEAK_GBPS * 1e9) >= F / (MFMA_F16_PEAK_TFLOPS * 1e12) else "mfma"
            rows.append({"layer": c.name.rsplit("_M", 1)[0], "M": M, "K": c.K, "N": c.N, "group": c.group,
                         "us": t * 1e6, "GBps": B / t / 1e9, "TFLOPs": F / t / 1e12,
                         "hbm_frac": hbm_frac, "mfma_frac": mfma_frac, "bound": bound,
                         "frac": hbm_frac if bound == "hbm" else mfma_frac,
                         "variant": plan["name"], "split_k": plan["split_k"], "grid": plan["grid"]})
    return rows


def dense_companion(tm, torch, wl, layers, iters=50):
    """fp16 x fp16 companion (the paper's Fig. "int4" / Table "performance" comparison in kind): the vendor library's
    dense GEMM (torch.matmul -> hipBLASLt) on dequantised fp16 weights of the same shapes, timed the same way
    (HIP-graph replay, weight copies rotated).  Context for the W4A16 numbers, not part of the method."""
    rows = []
    for L in layers:
        c = L.case
        wbytes = c.K * c.N * 2
        copies = max(2, min(L.copies, -(-ROTATE_BYTES // wbytes)))
        W = [(torch.randn(c.K, c.N, device="cuda", dtype=torch.float16) * c.sigma) for _ in range(copies)]
        for M in L.Ms:
            X = L.X[M][0]
            Y = torch.empty((M, c.N), dtype=torch.float16, device="cuda")
            turn = [0]

            def dense_step():
                torch.matmul(X, W[turn[0] % copies], out=Y)
                turn[0] += 1

            it = iters if M < 1024 else 10
            d_ms, _ = time_steps(torch, dense_step, it, 3, graph_steps=it)
            o_ms, _ = time_steps(torch, lambda: L.launch(tm, M), it, 3, graph_steps=it)
            rows.append({"layer": c.name.rsplit("_M", 1)[0], "M": M, "K": c.K, "N": c.N,
                         "w4a16_us": o_ms / it * 1e3, "dense_fp16_us": d_ms / it * 1e3,
                         "speedup_vs_dense": d_ms / o_ms,
                         "w4a16_TFLOPs": wl.flops(M, c.K, c.N) / (o_ms / it * 1e-3) / 1e12,
                         "dense_TFLOPs": wl.flops(M, c.K, c.N) / (d_ms / it * 1e-3) / 1e12})
        del W
        torch.cuda.empty_cache()
    return rows


# Mixture-of-experts decode layers in the shapes of the MoE models the paper evaluates (Sec. 5.1): (experts, experts
# per token, K, N); gate and up projections fused along N.  Weights are random int4 words (timing does not depend on
# their values); routing is uniform, seeded, k distinct experts per token, a new draw for every timed step.
MOE_LAYERS = {
    "moe8_gate_up": (8, 2, 4096, 28672),
    "moe8_down": (8, 2, 14336, 4096),
    "moe128_gate_up": (128, 8, 4096, 3072),
    "moe128_down": (128, 8, 1536, 4096),
}


def moe_table(tm, torch, names, tokens=(1, 4, 16, 64), iters=40, group=128, only=None, use_graph=True, fmt="int4"):
    import numpy as np
    rows = []
    for name in names:
        E, topk, K, N = MOE_LAYERS[name]
        G = K // group
        experts = []
        for e in range(E):
            if fmt == "int4":
                qw = torch.randint(-2 ** 31, 2 ** 31 - 1, (K, N // 8), dtype=torch.int32, device="cuda")
                s = (torch.rand((G, N), device="cuda") * 0.02 + 0.001).to(torch.float16)
                z = torch.randint(0, 16, (G, N), device="cuda").to(torch.float16)
                experts.append(tm.tm_pack_w4(qw, s, z, K, N, group))
            else:                                        # 8-bit integer or FP8 E4M3 experts (random codes)
                qw = torch.randint(-2 ** 31, 2 ** 31 - 1, (K, N // 4), dtype=torch.int32, device="cuda")
                s = (torch.rand((G, N), device="cuda") * 0.002 + 0.0001).to(torch.float16)
                z = torch.randint(0, 256, (G, N), device="cuda").to(torch.float16)
                if fmt == "fp8":
                    qw = qw & 0x77777777                 # keeps every code finite (no E4M3 NaN pattern)
                    experts.append(tm.tm_pack_w8_fp8(qw, s, K, N, group))
                else:
                    experts.append(tm.tm_pack_w8(qw, s, z, K, N, group))
        del qw, s, z
        grp = tm.tm_group_experts(experts)
        ebytes = (K * N // 2 if fmt == "int4" else K * N) + 4 * G * N
        rng = np.random.default_rng(E * 7 + K)
        for T in tokens:
            if only is not None and (name, T) != only:
                continue
            R = T * topk
            X = (torch.randn((R, K), device="cuda")).to(torch.float16)
            Y = torch.empty((R, N), dtype=torch.float16, device="cuda")
            offs, counts_all, active = [], [], 0
            for _ in range(iters):
                picks = np.concatenate([rng.choice(E, topk, replace=False) for _ in range(T)])
                counts = np.bincount(picks, minlength=E)
                active += int((counts > 0).sum())
                counts_all.append(counts)
                offs.append(np.concatenate([[0], np.cumsum(counts)]).astype(np.int32))
            od = torch.from_numpy(np.stack(offs)).cuda()
            turn = [0]

            def grouped_step():
                tm.tm_gemm_w4a16_grouped(X, grp, od[turn[0] % iters], Y)
                turn[0] += 1

            def looped_step():                          # one ordinary GEMM per expert that has rows (host-side counts)
                i = turn[0] % iters
                turn[0] += 1
                for e in range(E):
                    r0, r1 = int(offs[i][e]), int(offs[i][e + 1])
                    if r1 > r0:
                        tm.tm_gemm_w4a16(X[r0:r1], experts[e], Y[r0:r1])

            turn[0] = 0
            g_ms, _ = time_steps(torch, grouped_step, iters, 0, graph_steps=iters if use_graph else 0)
            turn[0] = 0
            l_ms, _ = time_steps(torch, looped_step, iters, 0, graph_steps=iters) if use_graph else (float("nan"), 0)
            t = g_ms / iters * 1e-3
            B = active / iters * ebytes + R * K * 2 + R * N * 2
            v, st = tm.tm_get_grouped_plan(grp, R)
            F = 2.0 * R * K * N
            rows.append({"layer": name, "format": fmt, "experts": E, "top_k": topk, "K": K, "N": N, "tokens": T, "rows": R,
                         "active_experts_avg": active / iters, "us": t * 1e6, "GBps": B / t / 1e9,
                         "TFLOPs": F / t / 1e12, "mfma_frac": F / t / 1e12 / MFMA_F16_PEAK_TFLOPS,
                         "hbm_frac": B / t / 1e9 / HBM_PEAK_GBPS, "looped_us": l_ms / iters * 1e3,
                         "variant": tm.tm_variant_name(v), "strips": st})
            log(f"{name:15s} E={E:3d} top{topk} tokens={T:3d} rows={R:4d} active={active / iters:6.1f}  grouped {t * 1e6:8.2f} us "
                f"({B / t / 1e9:6.0f} GB/s, {100 * B / t / 1e9 / HBM_PEAK_GBPS:4.1f} % HBM; {F / t / 1e12:7.1f} TF)   one launch per expert "
                f"{l_ms / iters * 1e3:8.2f} us   {tm.tm_variant_name(v)} x{st}")
        grp.close()
        for p in experts:
            p.close()
        del experts
        torch.cuda.empty_cache()
    return rows


def w8_table(tm, torch, wl, iters=100):
    """8-bit weights at decode sizes: the decode and MLP-decode layer shapes with int8 codes (W8A16) and with FP8 E4M3
    codes (random codes; timing does not depend on their values), same timing method as the 4-bit sweep."""
    rows = []
    shapes = WORKLOADS["decode"] + WORKLOADS["mlp_decode"] + WORKLOADS["sweep5"] + WORKLOADS["prefill"]
    for fmt, (name, Ms) in [(f, l) for f in ("int8", "fp8") for l in shapes]:
        c = wl.case_by_name(name)
        G = c.K // c.group
        wbytes = c.K * c.N + 4 * G * c.N
        copies = max(2, -(-ROTATE_BYTES // wbytes))
        packed = []
        for _ in range(copies):
            qw = torch.randint(-2 ** 31, 2 ** 31 - 1, (c.K, c.N // 4), dtype=torch.int32, device="cuda")
            s = (torch.rand((G, c.N), device="cuda") * 0.002 + 0.0001).to(torch.float16)
            z = torch.randint(0, 256, (G, c.N), device="cuda").to(torch.float16)
            if fmt == "int8":
                packed.append(tm.tm_pack_w8(qw, s, z, c.K, c.N, c.group))
            else:
                qw &= -16843010                      # 0xFEFEFEFE: no byte is a NaN code
                packed.append(tm.tm_pack_w8_fp8(qw, s, c.K, c.N, c.group))
        del qw, s, z
        for M in Ms:
            X = [torch.randn((M, c.K), device="cuda").to(torch.float16) for _ in range(4)]
            Y = [torch.empty((M, c.N), dtype=torch.float16, device="cuda") for _ in range(4)]
            turn = [0]

            def step():
                i = turn[0]
                turn[0] += 1
                tm.tm_gemm_w4a16(X[i % 4], packed[i % copies], Y[i % 4])

            it = iters if M < 1024 else 10
            ev_ms, _ = time_steps(torch, step, it, 3, graph_steps=it)
            t = ev_ms / it * 1e-3
            B = wl.algorithmic_bytes(M, c.K, c.N, c.group, bits=8)
            plan = tm.tm_get_plan(packed[0], M)
            rows.append({"layer": c.name.rsplit("_M", 1)[0], "M": M, "K": c.K, "N": c.N, "group": c.group, "bits": 8, "format": fmt,
                         "us": t * 1e6, "GBps": B / t / 1e9, "hbm_frac": B / t / 1e9 / HBM_PEAK_GBPS,
                         "TFLOPs": wl.flops(M, c.K, c.N) / t / 1e12,
                         "variant": plan["name"], "split_k": plan["split_k"], "grid": plan["grid"], "block": plan["block"]})
            log(f"{fmt:4s} {rows[-1]['layer']:14s} M={M:4d} K={c.K:6d} N={c.N:6d} {t * 1e6:8.2f} us {B / t / 1e9:7.0f} GB/s "
                f"({100 * B / t / 1e9 / HBM_PEAK_GBPS:4.1f} % HBM) {wl.flops(M, c.K, c.N) / t / 1e12:7.1f} TF  "
                f"{plan['name']} split {plan['split_k']} block {plan['block']}")
        for p in packed:
            p.close()
        del packed
        torch.cuda.empty_cache()
    return rows


# Decode attention over an 8-bit KV cache in the head geometry of the 8B model of the paper's kernel benchmark (32 query
# heads, 8 KV heads, head dimension 128): (batch, context length).  Cache contents are random codes with valid pairs.
ATTN_SHAPES = [(1, 2048), (1, 8192), (1, 32768), (8, 2048), (8, 8192), (32, 2048), (32, 8192), (64, 4096), (128, 2048)]


def attn_table(tm, torch, iters=50, q_heads=32, kv_heads=8, only=None, bits=8, eager=False):
    import numpy as np
    rows = []
    rng = np.random.default_rng(0)
    for B, T in ATTN_SHAPES:
        if only is not None and (B, T) != only:
            continue
        per_cache = B * kv_heads * T * (2 * 128 * bits // 8 + 8)
        copies = max(2, -(-ROTATE_BYTES // per_cache))
        caches = []
        for _ in range(copies):
            c = tm.tm_kv_create(B, kv_heads, T, bits)
            n = B * kv_heads * c.capacity
            pairs = (rng.uniform(0.005, 0.05, 2 * n).astype(np.float16).view(np.uint16).astype(np.uint32)
                     | (rng.integers(0, 256, 2 * n).astype(np.float16).view(np.uint16).astype(np.uint32) << 16))
            k, v, p, cb, pb = tm.tm_kv_raw(c)
            for ptr in (k, v):                          # random codes generated on the device
                t = torch.randint(0, 256, (cb,), dtype=torch.uint8, device="cuda")
                tm.tm_bench_copy_raw(ptr, t.data_ptr(), cb)
            t = torch.from_numpy(pairs.view(np.uint8)).cuda()
            tm.tm_bench_copy_raw(p, t.data_ptr(), pb)
            torch.cuda.synchronize()
            caches.append(c)
        Q = torch.randn((B, q_heads, 128), device="cuda").to(torch.float16)
        O = torch.empty_like(Q)
        lens = torch.full((B,), T, dtype=torch.int32, device="cuda")
        turn = [0]

        def step():
            tm.tm_attn_decode(Q, caches[turn[0] % copies], lens, O, 0.08838834764831845, max_len=T)
            turn[0] += 1

        # launched both ways - replayed from a HIP graph and enqueued call by call - and the faster one reported: graph
        # replay wins where a call is shorter than a host launch, while between long kernels its nodes leave a gap of
        # several microseconds that plain enqueueing does not (measured at batch 128 x 2048, 4-bit: 60 against 54 us)
        ev_ms, _ = time_steps(torch, step, iters, 5, graph_steps=0 if eager else iters)
        t, how = ev_ms / iters * 1e-3, "eager" if eager else "graph"
        if not eager:
            ev2, _ = time_steps(torch, step, iters, 5, graph_steps=0)
            if ev2 < ev_ms:
                t, how = ev2 / iters * 1e-3, "eager"
        # the step's other kernel: quantise and store the newest token of every sequence (position T - 1)
        knew = torch.randn((B, 1, kv_heads, 128), device="cuda").to(torch.float16)
        vnew = torch.randn((B, 1, kv_heads, 128), device="cuda").to(torch.float16)
        pos = torch.full((B,), T - 1, dtype=torch.int32, device="cuda")

        def store():
            tm.tm_kv_append(caches[turn[0] % copies], knew, vnew, pos)
            turn[0] += 1

        ev_ms, _ = time_steps(torch, store, iters, 5, graph_steps=0 if eager else iters)
        t_store = ev_ms / iters * 1e-3
        bytes_ = per_cache + 2 * B * q_heads * 128 * 2
        rows.append({"batch": B, "context": T, "q_heads": q_heads, "kv_heads": kv_heads, "kv_bits": bits, "us": t * 1e6,
                     "GBps": bytes_ / t / 1e9, "hbm_frac": bytes_ / t / 1e9 / HBM_PEAK_GBPS, "cache_copies": copies,
                     "append_us": t_store * 1e6, "launch": how})
        log(f"attn decode KV{bits}  batch {B:4d} context {T:6d}  {t * 1e6:9.2f} us  {bytes_ / t / 1e9:7.0f} GB/s "
            f"({100 * bytes_ / t / 1e9 / HBM_PEAK_GBPS:4.1f} % of HBM peak, {how})  {bytes_ / 1e6:8.1f} MB per call; "
            f"append of one token per sequence {t_store * 1e6:6.2f} us")
        for c in caches:
            c.close()
        del caches
        torch.cuda.empty_cache()
    return rows


# Prefill attention: a whole prompt's queries over the quantised cache the same call sequence has just filled (causal), in
# the same head geometry: (batch, prompt length).  A dense contraction: priced against the fp16 MFMA peak, with the
# causal half of the score matrix as the flop count (QK^T and PV, 2 flops per multiply-add).
ATTN_PREFILL_SHAPES = [(1, 512), (1, 2048), (1, 8192), (4, 2048), (16, 512)]


def attn_prefill_table(tm, torch, iters=20, q_heads=32, kv_heads=8, bits=8, only=None):
    import numpy as np
    rows = []
    rng = np.random.default_rng(0)
    for B, T in ATTN_PREFILL_SHAPES:
        if only is not None and (B, T) != only:
            continue
        c = tm.tm_kv_create(B, kv_heads, T, bits)
        n = B * kv_heads * c.capacity
        pairs = (rng.uniform(0.005, 0.05, 2 * n).astype(np.float16).view(np.uint16).astype(np.uint32)
                 | (rng.integers(0, 256, 2 * n).astype(np.float16).view(np.uint16).astype(np.uint32) << 16))
        k, v, p, cb, pb = tm.tm_kv_raw(c)
        for ptr in (k, v):
            t = torch.randint(0, 256, (cb,), dtype=torch.uint8, device="cuda")
            tm.tm_bench_copy_raw(ptr, t.data_ptr(), cb)
        t = torch.from_numpy(pairs.view(np.uint8)).cuda()
        tm.tm_bench_copy_raw(p, t.data_ptr(), pb)
        torch.cuda.synchronize()
        Q = torch.randn((B, T, q_heads, 128), device="cuda").to(torch.float16)
        O = torch.empty_like(Q)
        pos = torch.zeros((B,), dtype=torch.int32, device="cuda")

        def step():
            tm.tm_attn_prefill(Q, c, pos, O, 0.08838834764831845)

        it = max(3, min(iters, int(2e11 / (B * q_heads * 128 * 2.0 * T * (T + 1)))))
        ev_ms, _ = time_steps(torch, step, it, 2, graph_steps=0)
        sec = ev_ms / it * 1e-3
        flops = B * q_heads * 128 * 2.0 * T * (T + 1)                  # 4 * D flops per (query, key) pair with key <= query
        bytes_ = B * kv_heads * T * (2 * 128 * bits // 8 + 8) + 2 * B * T * q_heads * 128 * 2
        rows.append({"batch": B, "prompt": T, "q_heads": q_heads, "kv_heads": kv_heads, "kv_bits": bits, "us": sec * 1e6,
                     "TFLOPs": flops / sec / 1e12, "mfma_frac": flops / sec / 1e12 / MFMA_F16_PEAK_TFLOPS,
                     "GBps": bytes_ / sec / 1e9, "tokens_per_s": B * T / sec})
        log(f"attn prefill KV{bits}  batch {B:3d} prompt {T:6d}  {sec * 1e6:10.1f} us  {flops / sec / 1e12:7.1f} TFLOP/s "
            f"({100 * flops / sec / 1e12 / MFMA_F16_PEAK_TFLOPS:4.1f} % of the fp16 MFMA peak)  {B * T / sec / 1e6:7.2f} M tokens/s")
        c.close()
        torch.cuda.empty_cache()
    return rows


def epilogue_table(tm, torch, wl, iters=100):
    """Fused epilogue against the same work done as a second pass over Y (PyTorch elementwise kernels, same HIP graph):
    the gated MLP's fused gate+up projection with silu(gate)*up, and its down projection with the residual add."""
    import numpy as np
    import torch.nn.functional as F
    rows = []
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a.view(np.int32) if a.dtype == np.uint32 else a)).cuda()
    for case_name, mode in (("cfg3_gate_up_M64", "silu_mul"), ("cfg3_down_M64", "residual")):
        c = wl.case_by_name(case_name)
        d = wl.make(c)
        qw, sc, z = dev(d["qweight"]), dev(d["s"]), dev(d["z"])
        wbytes = c.K * c.N // 2 + 4 * c.K * c.N // c.group
        copies = max(2, -(-ROTATE_BYTES // wbytes))
        act = mode == "silu_mul"
        plain = [tm.tm_pack_w4(qw, sc, z, c.K, c.N, c.group) for _ in range(copies)]
        fused = [tm.tm_pack_w4_gate_up(qw, sc, z, c.K, c.N, c.group) for _ in range(copies)] if act else plain
        n_out = c.N // 2 if act else c.N
        for M in (1, 16, 64, 512, 4096):
            X = torch.randn((M, c.K), device="cuda").to(torch.float16)
            Y = torch.empty((M, c.N), dtype=torch.float16, device="cuda")
            Z = torch.empty((M, n_out), dtype=torch.float16, device="cuda")
            R = torch.randn((M, n_out), device="cuda").to(torch.float16)
            turn = [0]

            def step_fused():
                i = turn[0] % copies
                turn[0] += 1
                if act:
                    tm.tm_gemm_w4a16_ex(X, fused[i], Z, act=tm.TM_ACT_SILU_MUL)
                else:
                    tm.tm_gemm_w4a16_ex(X, fused[i], Z, residual=R)

            def step_unfused():
                i = turn[0] % copies
                turn[0] += 1
                tm.tm_gemm_w4a16(X, plain[i], Y)
                if act:
                    torch.mul(F.silu(Y[:, :n_out]), Y[:, n_out:], out=Z)
                else:
                    torch.add(Y, R, out=Z)

            n = iters if M <= 512 else max(10, iters // 10)
            tf = time_steps(torch, step_fused, n, 5, graph_steps=n)[0] / n * 1e3
            tu = time_steps(torch, step_unfused, n, 5, graph_steps=n)[0] / n * 1e3
            rows.append({"layer": case_name.split("_M")[0], "epilogue": mode, "M": M, "K": c.K, "N": c.N, "fused_us": tf,
                         "unfused_us": tu, "speedup": tu / tf})
            log(f"{case_name.split('_M')[0]:14s} {mode:9s} M={M:5d}  fused {tf:9.2f} us   GEMM + elementwise pass {tu:9.2f} us   x{tu / tf:.2f}")
        for h in plain + (fused if act else []):
            h.close()
        del plain, fused
        torch.cuda.empty_cache()
    return rows


def layer_table(tm, torch, wl, iters=20, layers=8, context=2048, batches=(1, 8, 32, 64)):
    """One decoding step through a stack of `layers` transformer layers built from the library's entry points only, in the
    layer shapes of the benchmark configurations (hidden 4096, 32 heads of 128, gated MLP of 11008): fused QKV GEMM ->
    quantise-and-store of the new key/value -> decode attention over the quantised cache -> output GEMM + residual ->
    gate/up GEMM with silu(gate)*up -> down GEMM + residual.  Norms and rotary embedding are left out (elementwise, not
    part of this library); the three slices of the QKV output are made contiguous by framework copies.  Every layer has
    its own weights and cache, so a step streams `layers` x (101 MB of weights + the cache) and nothing is re-read from
    the last-level cache.  Random codes; timing only."""
    import numpy as np
    H, NH, I = 4096, 32, 11008
    rng = np.random.default_rng(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def weights(K, N):
        q = rng.integers(0, 2 ** 31 - 1, (K, N // 8), dtype=np.int64).astype(np.int32)
        sc = rng.uniform(0.001, 0.004, (K // 128, N)).astype(np.float16)
        z = rng.integers(0, 16, (K // 128, N)).astype(np.float16)
        return dev(q), dev(sc), dev(z)

    stack = []
    for _ in range(layers):
        stack.append({"qkv": tm.tm_pack_w4(*weights(H, 3 * H), H, 3 * H, 128), "out": tm.tm_pack_w4(*weights(H, H), H, H, 128),
                      "gate_up": tm.tm_pack_w4_gate_up(*weights(H, 2 * I), H, 2 * I, 128),
                      "down": tm.tm_pack_w4(*weights(I, H), I, H, 128)})
    rows = []
    for bits in (8, 4):
        for B in batches:
            caches = []
            for _ in range(layers):
                c = tm.tm_kv_create(B, NH, context, bits)
                k, v, p, cb, pb = tm.tm_kv_raw(c)
                for ptr in (k, v):
                    t = torch.randint(0, 256, (cb,), dtype=torch.uint8, device="cuda")
                    tm.tm_bench_copy_raw(ptr, t.data_ptr(), cb)
                n = B * NH * c.capacity
                pairs = (rng.uniform(0.005, 0.05, 2 * n).astype(np.float16).view(np.uint16).astype(np.uint32)
                         | (rng.integers(0, 16, 2 * n).astype(np.float16).view(np.uint16).astype(np.uint32) << 16))
                t = torch.from_numpy(pairs.view(np.uint8)).cuda()
                tm.tm_bench_copy_raw(p, t.data_ptr(), pb)
                torch.cuda.synchronize()
                caches.append(c)
            f16 = lambda *shape: torch.empty(shape, dtype=torch.float16, device="cuda")
            x0 = torch.randn((B, H), device="cuda").to(torch.float16) * 0.1
            qkv, q, k, v = f16(B, 3 * H), f16(B, NH, 128), f16(B, 1, NH, 128), f16(B, 1, NH, 128)
            att, h1, act, h2 = f16(B, NH, 128), f16(B, H), f16(B, I), f16(B, H)
            pos = torch.full((B,), context - 1, dtype=torch.int32, device="cuda")
            lens = torch.full((B,), context, dtype=torch.int32, device="cuda")

            def step():
                x = x0
                for L, c in zip(stack, caches):
                    tm.tm_gemm_w4a16(x, L["qkv"], qkv)
                    q.copy_(qkv[:, :H].view(B, NH, 128))
                    k.copy_(qkv[:, H:2 * H].view(B, 1, NH, 128))
                    v.copy_(qkv[:, 2 * H:].view(B, 1, NH, 128))
                    tm.tm_kv_append(c, k, v, pos)
                    tm.tm_attn_decode(q, c, lens, att, 0.08838834764831845, max_len=context)
                    tm.tm_gemm_w4a16_ex(att.view(B, H), L["out"], h1, residual=x)
                    tm.tm_gemm_w4a16_ex(h1, L["gate_up"], act, act=tm.TM_ACT_SILU_MUL)
                    tm.tm_gemm_w4a16_ex(act, L["down"], h2, residual=h1)
                    x = h2

            ev_ms, _ = time_steps(torch, step, iters, 2, graph_steps=iters)
            us = ev_ms / iters / layers * 1e3
            wbytes = sum((K * N // 2 + 4 * K * N // 128) for K, N in ((H, 3 * H), (H, H), (H, 2 * I), (I, H)))
            cbytes = B * NH * context * (2 * 128 * bits // 8 + 8)
            rows.append({"kv_bits": bits, "batch": B, "context": context, "layers": layers, "us_per_layer": us,
                         "GBps": (wbytes + cbytes) / us / 1e3, "tokens_per_s_32_layers": B / (us * 32e-6)})
            log(f"decode layer KV{bits} batch {B:3d} context {context}: {us:8.2f} us per layer  "
                f"{(wbytes + cbytes) / us / 1e3:6.0f} GB/s of weights+cache  ({B / (us * 32e-6):8.0f} tokens/s at 32 layers)")
            for c in caches:
                c.close()
            del caches
            torch.cuda.empty_cache()
    for L in stack:
        for h in L.values():
            h.close()
    return rows


def attn_companion(torch, iters=20, q_heads=32, kv_heads=8, only=None):
    """The companion measurement of the attention rows: the same decode step over an unquantised fp16 cache through the
    framework's own fused attention (`scaled_dot_product_attention`, grouped-query mode) - what a serving stack without
    the quantised cache runs.  Same rotation over > 512 MB; HIP-graph replay when the library call can be captured."""
    import torch.nn.functional as F
    rows = []
    for B, T in ATTN_SHAPES:
        if only is not None and (B, T) != only:
            continue
        per_cache = B * kv_heads * T * 2 * 128 * 2
        copies = max(2, -(-ROTATE_BYTES // per_cache))
        Ks = [torch.randn((B, kv_heads, T, 128), device="cuda").to(torch.float16) for _ in range(copies)]
        Vs = [torch.randn((B, kv_heads, T, 128), device="cuda").to(torch.float16) for _ in range(copies)]
        Q = torch.randn((B, q_heads, 1, 128), device="cuda").to(torch.float16)
        out = [None]
        turn = [0]

        def step():
            i = turn[0] % copies
            out[0] = F.scaled_dot_product_attention(Q, Ks[i], Vs[i], enable_gqa=True)
            turn[0] += 1

        try:
            ev_ms, _ = time_steps(torch, step, iters, 3, graph_steps=iters)
            how = "graph"
        except Exception:
            torch.cuda.synchronize()
            ev_ms, _ = time_steps(torch, step, iters, 3, graph_steps=0)
            how = "eager"
        t = ev_ms / iters * 1e-3
        bytes_ = per_cache + 2 * B * q_heads * 128 * 2
        rows.append({"batch": B, "context": T, "us": t * 1e6, "GBps": bytes_ / t / 1e9, "timed": how})
        log(f"attn decode fp16 cache (library)  batch {B:4d} context {T:6d}  {t * 1e6:9.2f} us  {bytes_ / t / 1e9:7.0f} GB/s  ({how})")
        del Ks, Vs
        torch.cuda.empty_cache()
    return rows


def attn_store_row(tm, torch, iters=20, B=16, T=2048, kv_heads=8, bits=8, eager=False):
    """Quantise-and-store of a whole prompt (the prefill side of the cache): reads 2 fp16 tensors, writes codes + pairs."""
    c = tm.tm_kv_create(B, kv_heads, T, bits)
    knew = torch.randn((B, T, kv_heads, 128), device="cuda").to(torch.float16)
    vnew = torch.randn((B, T, kv_heads, 128), device="cuda").to(torch.float16)
    pos = torch.zeros((B,), dtype=torch.int32, device="cuda")
    ev_ms, _ = time_steps(torch, lambda: tm.tm_kv_append(c, knew, vnew, pos), iters, 3, graph_steps=0 if eager else iters)
    t = ev_ms / iters * 1e-3
    bytes_ = B * T * kv_heads * (2 * 128 * 2 + 2 * 128 * bits // 8 + 8)
    c.close()
    log(f"kv append (prompt) KV{bits} batch {B} tokens {T}: {t * 1e6:9.2f} us  {bytes_ / t / 1e9:7.0f} GB/s read+written")
    return {"batch": B, "tokens": T, "kv_heads": kv_heads, "kv_bits": bits, "us": t * 1e6, "GBps": bytes_ / t / 1e9,
            "hbm_frac": bytes_ / t / 1e9 / HBM_PEAK_GBPS}


def attn_cpu_baseline(B=1, T=2048, q_heads=32, kv_heads=8):
    """The attention oracle as it stands on this host, one decode step of a small case, in the unit of the attention rows."""
    import numpy as np
    from oracle import oracle_attn
    from workloads import attn as wa
    Q, K, V, lens = wa.draw(B, q_heads, kv_heads, T, seed=0)
    kq, vq = oracle_attn.kv_quantise(K), oracle_attn.kv_quantise(V)
    n, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < 5.0:
        oracle_attn.attn_decode(Q, *kq, *vq, lens, 128 ** -0.5)
        n += 1
    dt = (time.perf_counter() - t0) / n
    bytes_ = B * kv_heads * T * (2 * 128 + 8) + 2 * B * q_heads * 128 * 2
    return {"value": bytes_ / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{n} decode steps of batch {B} x context {T}, {q_heads}/{kv_heads} heads (numpy fp64)"}


# Launch shapes of the read-only stream tried for the ceiling: (CTAs per CU, threads per CTA, 128-bit loads in flight per
# thread, flags: 1 = non-temporal, 2 = contiguous slice per CTA).  The short list holds the shapes that won at some byte
# count in the full sweep (`--workload ceiling --ceiling-full`); grid 0 = one load per thread, the plain tm_bench_read shape.
CEILING_SHORTLIST = [(0, 256, 1, 0), (1, 1024, 8, 1), (1, 1024, 4, 3), (2, 512, 4, 1), (2, 1024, 2, 1), (4, 256, 4, 1),
                     (4, 512, 2, 1), (8, 256, 2, 1), (8, 256, 1, 1), (16, 256, 1, 1)]


# Layer shapes of other published models than the benchmark's (K, N, group): the dispatcher's thresholds were fitted on
# the benchmark's five configurations, these show what it does elsewhere.  Random codes: timing only.
OTHER_SHAPES = [("13B qkv", 5120, 15360, 128), ("13B gate_up", 5120, 27648, 128), ("13B down", 13824, 5120, 128),
                ("8B-GQA qkv", 4096, 6144, 128), ("8B-GQA gate_up", 4096, 28672, 128), ("8B-GQA down", 14336, 4096, 128),
                ("70B-GQA qkv", 8192, 10240, 128), ("70B down", 28672, 8192, 128), ("7B-28h gate_up", 3584, 37888, 128),
                ("7B-28h down", 18944, 3584, 128), ("small g64", 2048, 8192, 64),
                # one GPU's share of a 70B model under 8-way tensor parallelism (column-parallel layers cut along N,
                # row-parallel ones along K)
                ("70B/8 qkv", 8192, 1280, 128), ("70B/8 attn_out", 1024, 8192, 128), ("70B/8 gate_up", 8192, 7168, 128),
                ("70B/8 down", 3584, 8192, 128)]
OTHER_MS = (1, 8, 16, 32, 64, 128, 512)


def other_shapes_table(tm, torch, wl, iters=50):
    rows = []
    for label, K, N, g in OTHER_SHAPES:
        wbytes = K * N // 2 + 4 * K * N // g
        copies = max(2, -(-ROTATE_BYTES // wbytes))
        packed = []
        for _ in range(copies):
            qw = torch.randint(-2 ** 31, 2 ** 31 - 1, (K, N // 8), dtype=torch.int32, device="cuda")
            sc = (torch.rand((K // g, N), device="cuda") * 0.02 + 0.001).to(torch.float16)
            z = torch.randint(0, 16, (K // g, N), device="cuda").to(torch.float16)
            packed.append(tm.tm_pack_w4(qw, sc, z, K, N, g))
            del qw, sc, z
        for M in OTHER_MS:
            X = [torch.randn((M, K), device="cuda").to(torch.float16) for _ in range(2)]
            Y = [torch.empty((M, N), dtype=torch.float16, device="cuda") for _ in range(2)]
            turn = [0]

            def step():
                i = turn[0]
                turn[0] += 1
                tm.tm_gemm_w4a16(X[i % 2], packed[i % copies], Y[i % 2])

            it = iters if M <= 128 else max(10, iters // 5)
            ev_ms, _ = time_steps(torch, step, it, 3, graph_steps=it)
            t = ev_ms / it * 1e-3
            B, F = wl.algorithmic_bytes(M, K, N, g), wl.flops(M, K, N)
            hbm_frac, mfma_frac = B / t / 1e9 / HBM_PEAK_GBPS, F / t / 1e12 / MFMA_F16_PEAK_TFLOPS
            bound = "hbm" if B / (HBM_PEAK_GBPS * 1e9) >= F / (MFMA_F16_PEAK_TFLOPS * 1e12) else "mfma"
            plan = tm.tm_get_plan(packed[0], M)
            rows.append({"layer": label, "K": K, "N": N, "group": g, "M": M, "us": t * 1e6, "GBps": B / t / 1e9, "TFLOPs": F / t / 1e12,
                         "bound": bound, "frac": hbm_frac if bound == "hbm" else mfma_frac, "variant": plan["name"],
                         "split_k": plan["split_k"], "grid": plan["grid"], "one_shot": plan["one_shot_units_per_wave"]})
            log(f"{label:15s} {K:6d} x {N:6d} M={M:4d}: {t * 1e6:8.2f} us  {B / t / 1e9:6.0f} GB/s  {F / t / 1e12:7.1f} TF  "
                f"{100 * rows[-1]['frac']:4.1f} % of the {bound} roofline  {plan['name']} split {plan['split_k']} grid {plan['grid']}"
                f"{' one-shot' if plan['one_shot_units_per_wave'] else ''}")
        for pk in packed:
            pk.close()
        del packed
        torch.cuda.empty_cache()
    return rows


def l2_feed_table(tm, torch, iters=20):
    """How fast the compute units can be fed from the L2, apart from HBM: every CTA of a one-CTA-per-CU launch reads the
    whole of a 2 MB buffer (the way every CTA of a GEMM reads all of X), for several amounts of bytes in flight per CU."""
    n = 2 << 20
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.int32, device="cuda")
    rows = []
    for block, unroll in ((256, 1), (256, 4), (512, 4), (1024, 2), (1024, 8)):
        def step():
            tm.tm_bench_read_shape(src.data_ptr(), n, sink, 256, block, unroll, tm.TM_READ_SHARED | tm.TM_READ_NONTEMPORAL)
        ev_ms, _ = time_steps(torch, step, iters, 3, graph_steps=iters)
        us = ev_ms / iters * 1e3
        rows.append({"block": block, "loads_in_flight_per_thread": unroll, "bytes_in_flight_per_cu": block * unroll * 16,
                     "us": us, "GBps_per_cu": n / us / 1e3, "TBps_chip": 256 * n / us / 1e6})
        log(f"L2 feed, 256 CTAs x {block} threads x {unroll} loads in flight ({block * unroll * 16 // 1024:3d} KiB per CU): "
            f"{n / us / 1e3:6.1f} GB/s per CU, {256 * n / us / 1e6:5.1f} TB/s over the chip")
    return rows


def clock_under_load(tm, torch, step_fn, graph_steps, micros=3000):
    """Shader clock the chip holds while step_fn's launches run: a one-wave kernel, launched on a second stream ahead of
    the work so that it has its wave slot, sleeps through the untimed replays that precede every timed region and
    then reads the shader clock counter and the constant-rate counter around `micros` microseconds of further replays.
    Two streams may share a hardware queue, in which case the probe and the work run one after the other: events on both
    streams tell, and the measurement is repeated on another stream then.  None if no attempt overlapped."""
    out = torch.zeros(16, dtype=torch.int32, device="cuda")
    main = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(main):
        with torch.cuda.graph(graph, stream=main):
            for _ in range(graph_steps):
                step_fn()
        w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        w0.record()
        graph.replay()
        w1.record()
        torch.cuda.synchronize()
        one_ms = max(w0.elapsed_time(w1), 0.02)
    probe_ms = WARM_MS + micros * 1e-3
    for _ in range(6):
        side = torch.cuda.Stream()
        m0, m1, s1 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        khz = tm.tm_bench_clock(out, micros, delay_micros=int(WARM_MS * 1000), stream=side)
        s1.record(side)
        with torch.cuda.stream(main):
            m0.record()
            for _ in range(int((probe_ms + 4.0) / one_ms) + 1):     # replays to outlast the probe by a few milliseconds
                graph.replay()
            m1.record()
        torch.cuda.synchronize()
        # the probe ran beside the work if it ended its own length after the work began, and before the work ended
        if m0.elapsed_time(s1) > 0.9 * probe_ms and s1.elapsed_time(m1) > 0.0:
            ticks = out.cpu().numpy().astype("uint32")
            return float(ticks[0]) / (float(ticks[1]) / (khz * 1e3)) / 1e9 if ticks[1] else None
    return None


def mfma_ceiling_table(tm, torch, target_ms=1.0, num_cu=256):
    """What the matrix pipes sustain on this chip in a kernel of fp16 16x16x32 MFMAs only (eight independent accumulators
    per wave, operands in registers): one CTA per CU with one, two and four waves per SIMD; zero operands, one operand
    pair for all instructions, and a different pair per instruction (the case a GEMM is held against).
    Every launch is sized to about `target_ms` (a prefill launch takes 1.5 ms) and timed like the GEMM rows; the shader
    clock held under the load follows from the two device counters the first wave reads around its loop."""
    out = torch.zeros(16, dtype=torch.int32, device="cuda")
    wall_khz = tm.tm_bench_clock(out, 1)                     # frequency of the constant-rate counter
    torch.cuda.synchronize()
    rows = []
    for waves_per_simd, pattern in ((1, 0), (1, 1), (1, 2), (2, 2), (4, 2)):
        block = 256 * waves_per_simd
        iters = int(target_ms * 1e-3 * 2.4e9 / (128 * waves_per_simd))
        def step():
            tm.tm_bench_mfma(out, num_cu, block, iters, pattern)
        ev_ms, _ = time_steps(torch, step, 10, 3, graph_steps=10)
        us = ev_ms / 10 * 1e3
        ticks = out.cpu().numpy().astype("uint32")
        flops = num_cu * (block // 64) * iters * 8 * 16384.0
        ghz = float(ticks[0]) / (float(ticks[1]) / (wall_khz * 1e3)) / 1e9 if ticks[1] else None
        rows.append({"waves_per_simd": waves_per_simd, "operands": ("zeros", "one pair of values", "eight pairs of values")[pattern],
                     "iters": iters, "us": us, "TFLOPs": flops / us / 1e6, "frac_of_peak": flops / us / 1e6 / MFMA_F16_PEAK_TFLOPS,
                     "shader_clock_GHz": ghz, "shader_clocks_per_us_of_launch": float(ticks[0]) / us, "first_wave_clocks_per_mfma": float(ticks[0]) / (iters * 8)})
        log(f"MFMA only, {waves_per_simd} wave(s) per SIMD, {rows[-1]['operands']:21s}: {us:8.1f} us, {rows[-1]['TFLOPs']:7.1f} TFLOP/s "
            f"({100 * rows[-1]['frac_of_peak']:4.1f} % of {MFMA_F16_PEAK_TFLOPS:.0f}), shader clock {ghz:.2f} GHz, "
            f"{rows[-1]['first_wave_clocks_per_mfma']:.1f} clocks per MFMA in the first wave")
    return rows


def ceiling_sizes(wl):
    """(label, packed weight + scale/zero bytes) of every distinct weight matrix of the benchmark configurations."""
    out, seen = [], set()
    for name in ("decode", "mlp_decode", "sweep5", "prefill"):
        for cn, _ in WORKLOADS[name]:
            c = wl.case_by_name(cn)
            b = c.K * c.N // 2 + 4 * c.K * c.N // c.group
            if b not in seen:
                seen.add(b)
                out.append((cn.rsplit("_M", 1)[0], b))
    return out


def ceiling_table(tm, torch, sizes, iters=100, full=False, num_cu=256):
    """Read-only streaming ceiling at given byte counts: the achievable HBM read rate of a kernel that does nothing but
    load that many bytes once, timed exactly like the GEMM rows (HIP-graph replay, every launch on a different region of
    a buffer of more than 512 MB, so nothing is found in L2 or the Infinity Cache).  Returns, per size, the best shape."""
    total = ROTATE_BYTES + max(b for _, b in sizes) + (64 << 20)
    pool = torch.empty(total, dtype=torch.uint8, device="cuda")
    pool.random_(0, 256)
    sink = torch.zeros(16, dtype=torch.int32, device="cuda")
    base = pool.data_ptr()
    if full:
        shapes = [(0, 256, 1, 0)] + [(g, b, u, f) for g in (1, 2, 4, 8, 16, 32) for b in (256, 512, 1024) for u in (1, 2, 4, 8, 16)
                                     for f in (0, 1, 2, 3) if g * b <= 8192 and g * b * u <= 32768]
    else:
        shapes = CEILING_SHORTLIST
    rows = []
    for label, nbytes in sizes:
        nbytes = nbytes // 256 * 256
        span = -(-nbytes // 4096) * 4096
        slots = max(2, (total - span) // span)
        best = None
        for g, block, unroll, flags in shapes:
            grid = g * num_cu if g else -(-nbytes // 16 // block)
            turn = [0]

            def step():
                off = (turn[0] % slots) * span
                turn[0] += 1
                tm.tm_bench_read_shape(base + off, nbytes, sink, grid, block, unroll, flags)

            ev_ms, _ = time_steps(torch, step, iters, 5, graph_steps=iters)
            us = ev_ms / iters * 1e3
            row = {"bytes": nbytes, "like": label, "grid": grid, "block": block, "unroll": unroll,
                   "nontemporal": bool(flags & 1), "chunked": bool(flags & 2), "us": us, "GBps": nbytes / us / 1e3}
            if full:
                rows.append(row)
            if best is None or us < best["us"]:
                best = row
            if g == 0:
                plain = row
        best = dict(best, plain_read_us=plain["us"], plain_read_GBps=plain["GBps"], best=True)
        rows.append(best)
        log(f"read ceiling at {nbytes / 1e6:7.2f} MB ({label:14s}): best {best['us']:7.2f} us = {best['GBps']:6.0f} GB/s "
            f"({100 * best['GBps'] / HBM_PEAK_GBPS:4.1f} % of peak) with grid {best['grid']} x {best['block']}, {best['unroll']} in flight"
            f"{', nt' if best['nontemporal'] else ''}{', chunked' if best['chunked'] else ''};  one load per thread: {plain['us']:7.2f} us")
    del pool
    torch.cuda.empty_cache()
    return rows


def empty_launch_us(tm, torch, iters=200):
    """Cost of a kernel node that does no work (a 16-byte read), same graph-replay timing: the floor under every row."""
    buf = torch.zeros(64, dtype=torch.int32, device="cuda")
    ev_ms, _ = time_steps(torch, lambda: tm.tm_bench_read_shape(buf.data_ptr(), 16, buf, 1, 64, 1, 0), iters, 5, graph_steps=iters)
    return ev_ms / iters * 1e3


def cpu_baseline(wl, layers, min_s=12.0, budget_s=25.0):
    """The oracle as it stands, timed on this host's cores over the same workload: whole passes over every
    (layer, M) pair are repeated until at least `min_s` seconds have been spent; a single GEMM too large for
    `budget_s` is cut to its first rows (and the sample string says so)."""
    from oracle import oracle_w4
    threads = max(1, oracle_w4.num_threads())
    total_bytes = total_flops = 0
    total_s = 0.0
    passes = 0
    done = []
    while total_s < min_s and passes < 1000:
        for L in layers:
            c, d = L.case, L.data
            for M in L.Ms:
                rows = M
                est_rate = 1.0e9 * threads                               # MAC/s guess, only to bound one call
                if rows * c.K * c.N / est_rate > budget_s:
                    rows = max(1, int(budget_s * est_rate / (c.K * c.N)))
                t0 = time.perf_counter()
                oracle_w4.gemm(d["X"][:rows], d["q"], d["s"], d["z"], c.group)
                total_s += time.perf_counter() - t0
                total_bytes += wl.algorithmic_bytes(rows, c.K, c.N, c.group)
                total_flops += wl.flops(rows, c.K, c.N)
                if passes == 0:
                    done.append(f"{c.name.rsplit('_M', 1)[0]}:M={rows}" + ("" if rows == M else f"(of {M})"))
        passes += 1
    return {"seconds": total_s, "bytes": total_bytes, "flops": total_flops, "cores": threads,
            "sample": f"{passes} pass(es) of oracle.gemm (fp64, scalar C, OpenMP) over " + ", ".join(done)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="decode", choices=sorted(WORKLOADS) + ["sweep", "shapes", "ceiling", "copy", "companion", "pack", "moe", "w8", "attn", "epilogue", "layer"])
    ap.add_argument("--sweep-out", default=None, help="with --workload sweep: write the per-shape table here (JSON)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ceiling-full", action="store_true", help="with --workload ceiling: sweep every launch shape, not the short list")
    ap.add_argument("--attn-companion", action="store_true",
                    help="attn workload: also time the framework's fused attention over an fp16 cache on the same shapes")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill companion measurement")
    ap.add_argument("--no-per-config", action="store_true", help="skip the per-(configuration, M) rows of the default line")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the read-only streaming ceiling beside the roofline")
    ap.add_argument("--companion-workloads", default="decode,mlp_decode,sweep5,prefill",
                    help="workloads the fp16 x fp16 companion covers (comma-separated; one of them makes a short profiler run)")
    ap.add_argument("--eager", action="store_true", help="launch every kernel from the host instead of replaying HIP graphs")
    ap.add_argument("--moe-tokens", default="1,4,16,64", help="with --workload moe: tokens per step (comma-separated)")
    ap.add_argument("--moe-format", default="int4", choices=["int4", "int8", "fp8"], help="with --workload moe: weight format of the experts")
    ap.add_argument("--only", default=None, help="restrict the workload to one 'layer:M' pair, e.g. cfg3_gate_up:1 (profiling)")
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--stage-steps", type=int, default=0)
    ap.add_argument("--variant", type=int, default=-1)
    ap.add_argument("--split-k", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    import paper_2508_15601_amd as tm
    from workloads import w4a16 as wl
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    tm.load_library()
    tm.tm_set_variant(args.variant, args.split_k)
    tm.tm_set_launch(args.waves, args.stage_steps)

    if args.workload == "copy":
        # plain 128-bit copy of known size: calibrates the profiler's FETCH_SIZE / WRITE_SIZE counters
        n = 256 << 20
        src = torch.randint(0, 2 ** 31 - 1, (n // 4,), dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        ev_ms, _ = time_steps(torch, lambda: tm.tm_bench_copy(dst, src), args.steps, args.warmup)
        print(json.dumps({"metric": "plain copy (counter calibration)", "bytes_read": n, "bytes_written": n,
                          "steps": args.steps, "ms_per_step": ev_ms / args.steps,
                          "GBps_read_plus_write": 2 * n / (ev_ms / args.steps * 1e-3) / 1e9}))
        return

    if args.workload == "shapes":
        rows = other_shapes_table(tm, torch, wl, iters=min(args.steps, 50))
        if args.sweep_out:
            os.makedirs(os.path.dirname(os.path.abspath(args.sweep_out)), exist_ok=True)
            json.dump(rows, open(args.sweep_out, "w"), indent=1)
        print(json.dumps({"metric": "W4A16 GEMM on layer shapes outside the benchmark configurations", "workload": "shapes",
                          "n_gpus": 1, "data": "synthetic (random codes)", "rows": rows}))
        return

    if args.workload == "ceiling":
        sizes = ceiling_sizes(wl)
        if args.only:                                   # --only cfg2_qkv: one byte count (a profiler run per size)
            sizes = [sz for sz in sizes if sz[0] == args.only]
            if not sizes:
                raise SystemExit(f"--only {args.only}: no such weight matrix; have {[n for n, _ in ceiling_sizes(wl)]}")
        rows = ceiling_table(tm, torch, sizes, iters=min(args.steps, 100), full=args.ceiling_full)
        empty = empty_launch_us(tm, torch)
        log(f"empty kernel node: {empty:.2f} us")
        l2 = None if args.only else l2_feed_table(tm, torch)
        mfma = None if args.only else mfma_ceiling_table(tm, torch)
        if args.sweep_out:
            os.makedirs(os.path.dirname(os.path.abspath(args.sweep_out)), exist_ok=True)
            json.dump(rows, open(args.sweep_out, "w"), indent=1)
        print(json.dumps({"metric": "read-only streaming ceiling at the byte counts of the benchmark's weight matrices", "workload": "ceiling",
                          "n_gpus": 1, "empty_launch_us": empty, "l2_feed": l2, "mfma_only": mfma, "rows": [r for r in rows if r.get("best")]}))
        return

    if args.workload == "pack":
        # offline packing of one gate/up-shaped matrix from every interchange layout (wall time per call includes
        # the handle's two device allocations; kernel times come from a profiler run of this same command)
        import numpy as np
        K, N, g = 4096, 22016, 128
        rng = np.random.default_rng(0)
        q = rng.integers(0, 16, (K, N), dtype=np.uint8)
        s = torch.from_numpy(rng.uniform(0.001, 0.02, (K // g, N)).astype(np.float16)).cuda()
        z = rng.integers(0, 16, (K // g, N)).astype(np.float16)
        rows = []
        for layout in (tm.TM_LAYOUT_N8, tm.TM_LAYOUT_N8_INTERLEAVED, tm.TM_LAYOUT_K8):
            qw, zs = wl.encode_layout(q, z, layout)
            qd = torch.from_numpy(qw.view(np.int32)).cuda()
            zd = torch.from_numpy(zs if layout == tm.TM_LAYOUT_N8 else zs.view(np.int32)).cuda()
            def once():
                tm.tm_pack_w4_layout(qd, s, zd, K, N, g, layout).close()       # close() synchronises
            for _ in range(args.warmup):
                once()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                once()
            ms = (time.perf_counter() - t0) * 1e3 / args.steps
            rows.append({"layout": layout, "ms_per_pack_call": ms})
            log(f"layout {layout}: {ms:.3f} ms per pack call (allocation + two kernels + free)")
        print(json.dumps({"metric": "offline pack", "K": K, "N": N, "group": g, "steps": args.steps, "rows": rows}))
        return

    if args.workload == "layer":
        table = layer_table(tm, torch, wl, iters=min(args.steps, 20))
        if args.sweep_out:
            os.makedirs(os.path.dirname(os.path.abspath(args.sweep_out)), exist_ok=True)
            json.dump(table, open(args.sweep_out, "w"), indent=1)
        print(json.dumps({"metric": "one decoding step of a transformer layer built from the library's entry points: microseconds per layer",
                          "workload": "layer", "n_gpus": 1, "data": "synthetic", "rows": table}))
        return

    if args.workload == "epilogue":
        table = epilogue_table(tm, torch, wl, iters=min(args.steps, 100))
        if args.sweep_out:
            os.makedirs(os.path.dirname(os.path.abspath(args.sweep_out)), exist_ok=True)
            json.dump(table, open(args.sweep_out, "w"), indent=1)
        print(json.dumps({"metric": "fused epilogue vs a second pass over Y: microseconds per layer call", "workload": "epilogue",
                          "n_gpus": 1, "data": "synthetic", "rows": table}))
        return

    if args.workload == "attn":
        only = tuple(int(v) for v in args.only.split(":")) if args.only else None
        if only is not None and len(only) == 3:                 # --only batch:context:bits
            table = attn_table(tm, torch, iters=min(args.steps, 50), only=only[:2], bits=only[2], eager=args.eager)
        else:
            table = attn_table(tm, torch, iters=min(args.steps, 50), only=only, eager=args.eager)
            table += attn_table(tm, torch, iters=min(args.steps, 50), only=only, bits=4, eager=args.eager)
        if args.sweep_out:
            os.makedirs(os.path.dirname(os.path.abspath(args.sweep_out)), exist_ok=True)
            json.dump(table, open(args.sweep_out, "w"), indent=1)
        best = max(table, key=lambda r: r["GBps"])
        traffic = None                      # HBM bytes per launch from the committed profile of that shape and code width
        traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
        if os.path.exists(traffic_file) and (best["batch"], best["context"]) == (128, 2048):
            traffic = json.load(open(traffic_file)).get(f"attn_kv{best['kv_bits']}")
        print(json.dumps({"metric": "decode attention over a quantised KV cache: effective HBM GB/s", "workload": "attn",
                          "value": best["GBps"], "unit": "GB/s", "n_gpus": 1, "dtype": "u8 / u4 codes, f16 activations, f32 accumulation",
                          "data": "synthetic", "config": {"workload": f"KV{best['kv_bits']}, batch {best['batch']} x context {best['context']}, "
                                                                      f"{best['q_heads']} query / {best['kv_heads']} KV heads, head dimension 128"},
                          "roofline": {"bound": "hbm", "achieved": best["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                       "frac": best["hbm_frac"], "traffic": traffic, "kernel": f"attn_decode_kernel<{best['kv_bits']}, true>",
                                       "avg_launch_us": best["us"]},
                          "cpu_baseline": None if args.no_cpu_baseline else attn_cpu_baseline(),
                          "store": None if only is not None else [attn_store_row(tm, torch, eager=args.eager), attn_store_row(tm, torch, bits=4, eager=args.eager)],
                          "fp16_cache_library": attn_companion(torch, iters=min(args.steps, 20)) if args.attn_companion else None,
                          "prefill": None if only is not None else attn_prefill_table(tm, torch) + attn_prefill_table(tm, torch, bits=4),
                          "rows": table}))
        return

    if args.workload == "w8":
        table = w8_table(tm, torch, wl, iters=min(args.steps, 100))
        if args.sweep_out:
            os.makedirs(os.path.dirname(os.path.abspath(args.sweep_out)), exist_ok=True)
            json.dump(table, open(args.sweep_out, "w"), indent=1)
        print(json.dumps({"metric": "W8A16 GEMM, decode: effective HBM GB/s", "workload": "w8", "rows": table}))
        return

    if args.workload == "moe":
        only = None
        if args.only:
            nm, T = args.only.split(":")
            only = (nm, int(T))
        names = [n for n in MOE_LAYERS if only is None or n == only[0]]
        table = moe_table(tm, torch, names, tokens=tuple(int(t) for t in args.moe_tokens.split(",")), iters=args.steps if args.steps <= 40 else 40, only=only, use_graph=not args.eager, fmt=args.moe_format)
        if args.sweep_out:
            os.makedirs(os.path.dirname(os.path.abspath(args.sweep_out)), exist_ok=True)
            json.dump(table, open(args.sweep_out, "w"), indent=1)
        print(json.dumps({"metric": "grouped W4A16 GEMM, MoE decode: effective HBM GB/s", "workload": "moe", "rows": table}))
        return

    if args.workload == "companion":
        table = []
        for name in args.companion_workloads.split(","):
            layers = [Layer(tm, torch, wl, cn, Ms) for cn, Ms in WORKLOADS[name]]
            rows = dense_companion(tm, torch, wl, layers)
            for r in rows:
                log(f"{r['layer']:16s} M={r['M']:5d} K={r['K']:6d} N={r['N']:6d}  W4A16 {r['w4a16_us']:9.2f} us "
                    f"({r['w4a16_TFLOPs']:7.1f} TF)   dense fp16 (vendor library) {r['dense_fp16_us']:9.2f} us "
                    f"({r['dense_TFLOPs']:7.1f} TF)   speed-up {r['speedup_vs_dense']:5.2f}x")
            table += rows
            del layers
            torch.cuda.empty_cache()
        if args.sweep_out:
            os.makedirs(os.path.dirname(os.path.abspath(args.sweep_out)), exist_ok=True)
            json.dump(table, open(args.sweep_out, "w"), indent=1)
        print(json.dumps({"metric": METRIC, "workload": "companion", "rows": len(table)}))
        return

    if args.workload == "sweep":
        table = []
        for name in ("decode", "mlp_decode", "sweep5", "prefill"):
            layers = [Layer(tm, torch, wl, cn, Ms) for cn, Ms in WORKLOADS[name]]
            rows = per_shape_table(tm, torch, wl, layers, iters=(10 if name == "prefill" else 100),
                                   use_graph=not args.eager)
            for r in rows:
                r["workload"] = name
                log(f"{r['layer']:16s} M={r['M']:5d} K={r['K']:6d} N={r['N']:6d} g={r['group']:3d} {r['us']:9.2f} us "
                    f"{r['GBps']:8.1f} GB/s ({100 * r['hbm_frac']:5.1f}% HBM) {r['TFLOPs']:8.2f} TF "
                    f"({100 * r['mfma_frac']:5.1f}% MFMA) {r['variant']} split={r['split_k']} grid={r['grid']}")
            table += rows
            for L in layers:
                log(f"   pack {L.case.K}x{L.case.N}: {L.pack_ms:.3f} ms per matrix "
                    f"({L.case.K * L.case.N / 2 / L.pack_ms / 1e6:.1f} GB/s of int4 out)")
            del layers
            torch.cuda.empty_cache()
        if args.sweep_out:
            os.makedirs(os.path.dirname(os.path.abspath(args.sweep_out)), exist_ok=True)
            json.dump(table, open(args.sweep_out, "w"), indent=1)
        print(json.dumps({"metric": METRIC, "workload": "sweep", "rows": len(table)}))
        return

    spec = WORKLOADS[args.workload]
    if args.only:
        lname, m = args.only.split(":")
        spec = [(cn, (int(m),)) for cn, Ms in spec if cn.startswith(lname)]
        assert spec, "no layer of this workload matches --only"
    layers = [Layer(tm, torch, wl, cn, Ms) for cn, Ms in spec]
    launches_per_step = sum(len(L.Ms) for L in layers)

    def step():
        for L in layers:
            for M in L.Ms:
                L.launch(tm, M)

    # graph long enough that every layer walks through all of its packed copies at least once per replay
    want = max(-(-L.copies // len(L.Ms)) for L in layers)
    graph_steps = 0 if args.eager else pick_graph_steps(args.steps, max(want, 100 // launches_per_step, 1))
    ev_ms, wall_ms = time_steps(torch, step, args.steps, args.warmup, graph_steps=graph_steps)
    ms_per_step = ev_ms / args.steps
    B = sum(wl.algorithmic_bytes(M, L.case.K, L.case.N, L.case.group) for L in layers for M in L.Ms)
    F = sum(wl.flops(M, L.case.K, L.case.N) for L in layers for M in L.Ms)
    gbps = B / (ms_per_step * 1e-3) / 1e9
    tflops = F / (ms_per_step * 1e-3) / 1e12
    hbm_bound = args.workload != "prefill"

    # Roofline of the dominant kernel: the layer that moves the most bytes, timed alone over the same number of
    # steps with the same launch mode, so that its average launch duration can be set against the profiler's.
    dom = max(layers, key=lambda L: L.case.K * L.case.N)
    dom_steps = args.steps
    # (graphs of about a hundred launches, so that the cost of starting a replay is spread as thinly as in the step above)
    dom_graph = 0 if args.eager else pick_graph_steps(dom_steps, max(-(-dom.copies // len(dom.Ms)), 100 // len(dom.Ms), 1))

    def dom_step():
        for M in dom.Ms:
            dom.launch(tm, M)

    dom_ms, _ = time_steps(torch, dom_step, dom_steps, 2, graph_steps=dom_graph)
    dom_launch_s = dom_ms * 1e-3 / (dom_steps * len(dom.Ms))
    dom_B = sum(wl.algorithmic_bytes(M, dom.case.K, dom.case.N, dom.case.group) for M in dom.Ms) / len(dom.Ms)
    dom_F = sum(wl.flops(M, dom.case.K, dom.case.N) for M in dom.Ms) / len(dom.Ms)
    if hbm_bound:
        ach = dom_B / dom_launch_s / 1e9
        roofline = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": ach / HBM_PEAK_GBPS, "traffic": None}
    else:
        ach = dom_F / dom_launch_s / 1e12
        roofline = {"bound": "mfma", "achieved": ach, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / MFMA_F16_PEAK_TFLOPS, "traffic": None}
    plan = tm.tm_get_plan(dom.packed[0], dom.Ms[-1])
    form = (f", one-shot form: stream_kernel with {plan['name'].split('x')[-1]}-column strips, {plan['one_shot_units_per_wave']} units per wave, "
            f"{plan['block'] // 64} waves" if plan.get("one_shot_units_per_wave", 0) > 0 else "")
    roofline["kernel"] = f"{plan['name']}{form} on {dom.case.name.rsplit('_M', 1)[0]} (K={dom.case.K}, N={dom.case.N}), M in {list(dom.Ms)}"
    roofline["avg_launch_us"] = dom_launch_s * 1e6
    roofline["algorithmic_bytes_per_launch"] = dom_B
    roofline["flops_per_launch"] = dom_F
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        roofline["traffic"] = json.load(open(traffic_file)).get(args.workload)
        roofline["traffic_source"] = ("profiles/traffic.json: FETCH_SIZE x 2.0 + WRITE_SIZE from rocprofv3 --pmc runs of this command, "
                                      "copied there by hand from the summaries under profiles/; a stored figure, not observed in this run")
    if hbm_bound and not args.no_ceiling:
        # the read-only stream at the dominant layer's byte count, timed the same way: what this chip's memory system
        # delivers to a kernel that only loads those bytes, beside the 8 TB/s of the data sheet
        c = dom.case
        ceil = ceiling_table(tm, torch, [(c.name.rsplit("_M", 1)[0], c.K * c.N // 2 + 4 * c.K * c.N // c.group)], iters=100)[-1]
        roofline["read_ceiling_GBps"] = ceil["GBps"]
        roofline["read_ceiling_us"] = ceil["us"]
        roofline["read_ceiling_shape"] = {k: ceil[k] for k in ("grid", "block", "unroll", "nontemporal", "chunked")}
        roofline["frac_of_read_ceiling"] = ach / ceil["GBps"]
        roofline["empty_launch_us"] = empty_launch_us(tm, torch)
    if not args.no_ceiling and dom_graph > 0:
        # the shader clock held while the dominant kernel runs (the data-sheet peaks are quoted at 2.4 GHz)
        try:
            roofline["shader_clock_GHz_under_load"] = clock_under_load(tm, torch, dom_step, dom_graph)
        except tm.TmError as e:                           # a side measurement: its failure must not cost the line
            roofline["shader_clock_GHz_under_load"] = None
            log(f"clock probe failed: {e}")
    if not hbm_bound and not args.no_ceiling:
        # a kernel of MFMAs only, timed the same way: what the matrix pipes deliver at the clock this chip holds under
        # that load, beside the data-sheet peak at 2.4 GHz
        best = max(mfma_ceiling_table(tm, torch), key=lambda r: r["TFLOPs"] if r["operands"] == "eight pairs of values" else 0.0)
        roofline["mfma_ceiling_TFLOPs"] = best["TFLOPs"]
        roofline["mfma_ceiling_shader_clock_GHz"] = best["shader_clock_GHz"]
        roofline["mfma_ceiling_shape"] = {"waves_per_simd": best["waves_per_simd"], "operands": best["operands"]}
        roofline["frac_of_mfma_ceiling"] = ach / best["TFLOPs"]
        if roofline.get("shader_clock_GHz_under_load"):
            roofline["frac_of_peak_at_held_clock"] = ach / (MFMA_F16_PEAK_TFLOPS * roofline["shader_clock_GHz_under_load"] / 2.4)

    out = {
        "metric": METRIC, "value": gbps if hbm_bound else tflops, "unit": "GB/s" if hbm_bound else "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": {"decode": "configs[1]: W4A16 GEMM K=4096, N in {4096, 12288}, group=128, M in {1,4,8,16}",
                                "mlp_decode": "configs[2]: K=4096,N=22016 and K=11008,N=4096, group=128, M in {1,16,32,64}",
                                "prefill": "configs[3]: M=4096, K=8192, N=28672, group=128",
                                "sweep5": "configs[4]: K=8192, N=8192, group=64, M in {1,2,4,8,32,128,256,1024}"}[args.workload],
                   "launches_per_step": launches_per_step, "weight_copies_rotated": [L.copies for L in layers],
                   "launch_mode": "eager" if args.eager else f"hip_graph({graph_steps} steps per replay)"},
        "tflops": tflops, "effective_GBps": gbps, "host_wall_ms_per_step": wall_ms / args.steps,
        "pack_ms_per_matrix": {f"{L.case.K}x{L.case.N}": L.pack_ms for L in layers},
        "roofline": roofline,
    }

    if args.workload == "decode" and not args.no_per_config:
        # one timed row per (configuration, M) of all five configurations, same timing method
        table = []
        for ci, name in enumerate(CONFIG_WORKLOADS):
            ls = layers if name == "decode" else [Layer(tm, torch, wl, cn, Ms) for cn, Ms in WORKLOADS[name]]
            rows = per_shape_table(tm, torch, wl, ls, iters=(20 if name == "prefill" else 100), warmup=3)
            for r in rows:
                r["config"] = ci + 1
            table += rows
            if name != "decode":
                del ls
                torch.cuda.empty_cache()
        out["per_config"] = table
        pr = [r for r in table if r["config"] == 4][0]
        out["prefill"] = {"workload": "configs[3]: M=4096, K=8192, N=28672, group=128", "ms": pr["us"] * 1e-3, "TFLOPs": pr["TFLOPs"],
                          "roofline": {"bound": "mfma", "achieved": pr["TFLOPs"], "peak": MFMA_F16_PEAK_TFLOPS,
                                       "unit": "TFLOP/s", "frac": pr["mfma_frac"]},
                          "kernel": pr["variant"]}
    elif args.workload == "decode" and not args.no_prefill:
        PL = Layer(tm, torch, wl, *WORKLOADS["prefill"][0])
        pms, _ = time_steps(torch, lambda: PL.launch(tm, 4096), 20, 5, graph_steps=5)
        t = pms / 20 * 1e-3
        c = PL.case
        ptf = wl.flops(4096, c.K, c.N) / t / 1e12
        out["prefill"] = {"workload": "configs[3]: M=4096, K=8192, N=28672, group=128", "ms": t * 1e3, "TFLOPs": ptf,
                          "roofline": {"bound": "mfma", "achieved": ptf, "peak": MFMA_F16_PEAK_TFLOPS,
                                       "unit": "TFLOP/s", "frac": ptf / MFMA_F16_PEAK_TFLOPS},
                          "kernel": tm.tm_get_plan(PL.packed[0], 4096)["name"]}
        del PL

    if not args.no_cpu_baseline:
        cb = cpu_baseline(wl, layers)
        v = cb["bytes"] / cb["seconds"] / 1e9 if hbm_bound else cb["flops"] / cb["seconds"] / 1e12
        out["cpu_baseline"] = {"value": v, "unit": out["unit"], "cores": cb["cores"], "kind": "oracle",
                               "sample": cb["sample"], "seconds": cb["seconds"]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
