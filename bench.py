#!/usr/bin/env python3
"""Benchmark of the PVQ hot path on one MI355X.

A step is one pass of the whole path over the Llama-3-70B gate-projection shape (28672 x 8192,
bf16 source, D = 8, K = 16 -> 24-bit indices, 2-bit amplitude codes = 3.25 bits per weight):
    pvq_encode  ->  pvq_decode (to bf16)  ->  pvq_decode_gemv at batch 1, 4 and 16.
Inputs are resident in HBM before the timed region.  Steps rotate over several sets of packed
planes so that the fused product reads its codes from HBM rather than from the last-level cache.

Prints ONE JSON line.  `value` is the fused decode+GEMV's algorithmic bandwidth at batch 1
(bytes the method must move per launch / the kernel's mean duration inside the timed steps, HIP
events on the launch stream); the other kernels' rates are extra keys of the same line, and so are,
timed after the steps, the benchmark's other workloads (`configs`: the 14336 x 4096 matrix with 8-bit
amplitude codes, with groups of 16 and 32, decode-only over the seven Llama-3-70B shapes) and the
device's plain copy rate.
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
ROWS, COLS = 28672, 8192        # Llama-3-70B gate projection (out x in)
D, INDEX_BUDGET, SCALE_BITS = 8, 24, 2
BATCHES = (1, 4, 16)


def algorithmic_bytes(rows, cols, index_bits, scale_bits, batch):
    """What one launch has to move (per weight: (index_bits + scale_bits)/8/D bytes of codes)."""
    G = cols // D
    codes = rows * ((G * index_bits + 31) // 32 + (G * scale_bits + 31) // 32) * 4
    gemv = codes + rows * 4 + batch * cols * 2 + batch * rows * 4
    decode = codes + rows * 4 + rows * cols * 2
    encode = rows * cols * 2 + codes + rows * 4
    return {"gemv": gemv, "decode": decode, "encode": encode}


def cpu_baseline(wf_rows, xf, K, threads):
    """The CPU oracle, as it stands, on a row sample of the same workload: encode, then
    decode + product at batch 1.  Returns rates in the units of the GPU figures."""
    import numpy as np

    from oracle import pvq_oracle as oracle
    rows, cols = wf_rows.shape
    G = cols // D
    edges, centers = oracle.beta_tables(D, G, SCALE_BITS)
    t0 = time.perf_counter()
    enc = oracle.encode(wf_rows, D, K, SCALE_BITS, edges, want_pulses=False, nthreads=threads)
    t1 = time.perf_counter()
    oracle.decode(enc, centers, x=xf.astype(np.float64), want_weights=False, nthreads=threads)
    t2 = time.perf_counter()
    ab = algorithmic_bytes(rows, cols, enc.index_bits, SCALE_BITS, 1)
    return {
        "value": ab["gemv"] / (t2 - t1) / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": f"first {rows} of {ROWS} rows of the same matrix ({rows * cols / 1e6:.1f} M weights), "
                  f"decode + product at batch 1; encode timed beside it",
        "decode_gemv_gweights_per_s": rows * cols / (t2 - t1) / 1e9,
        "encode_gweights_per_s": rows * cols / (t1 - t0) / 1e9,
        "seconds": round(t2 - t0, 2),
    }


TRAFFIC_FILE = "profiles/hbm_traffic_gate_70b.txt"


def read_traffic(kernel="gemv_b1"):
    """HBM bytes per launch of a kernel from the COMMITTED counter summary (rocprofv3 --pmc FETCH_SIZE
    and WRITE_SIZE runs, scaled by a copy of known size; see the file), or None if it is not there.
    Not measured by this run: counters need the profiler."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(f"{kernel}_traffic_bytes_per_launch"):
                    return int(line.split("=")[1])
    except (OSError, ValueError):
        pass
    return None


def timed_ms(torch, fn, reps=10, warm_ms=30.0):
    """Median duration of fn() in ms: HIP events on the current stream around each call, after the GPU has been kept
    busy with fn for warm_ms (after a pause on the host the clocks of this part sag for some tens of milliseconds:
    the same kernel measured 0.235 ms at first and 0.295 ms ten launches later)."""
    fn(); torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < warm_ms:
        for _ in range(4):
            fn()
        torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    for i in range(reps):
        ev[i].record(); fn()
    ev[reps].record(); torch.cuda.synchronize()
    return sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))[reps // 2]


def other_configs(torch, pvq, si, dev):
    """The other workloads of the benchmark definition, timed after the steps (not part of ms_per_step):
    config 1 (Llama-3-8B up projection, 8-bit amplitude codes, encode and decode), config 2 (the same matrix
    with groups of 16 and 32, 52- and 104-bit indices), config 3 (decode only, to bf16, over the seven weight
    shapes of a Llama-3-70B decoder layer at 3.25 bits per weight), and the device's own copy rate as the
    practical ceiling of the HBM-bound kernels.  Rates are algorithmic bytes / mean kernel time."""
    out = {}
    gbps = lambda nbytes, t_ms: round(nbytes / (t_ms * 1e-3) / 1e9, 1)
    gw = lambda n, t_ms: round(n / (t_ms * 1e-3) / 1e9, 2)

    # what a plain copy and a plain fill reach on this device (256 MiB; bytes read + bytes written)
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    t_copy = timed_ms(torch, lambda: dst.copy_(src))
    t_fill = timed_ms(torch, lambda: dst.zero_())
    out["device_copy_GBps"] = gbps(2 * src.numel(), t_copy)
    out["device_fill_GBps"] = gbps(src.numel(), t_fill)
    del src, dst

    # config 1 and config 2: 14336 x 4096, bf16 source
    r8, c8 = si.LLAMA3_8B_UP
    W8 = si.gaussian_weights_device(r8, c8, 0.015, si.BASE_SEED + 1, dev)
    Wo8 = torch.empty((r8, c8), dtype=torch.bfloat16, device=dev)
    n8 = r8 * c8

    def enc_dec(Dg, budget, sbits, label):
        Kg = pvq.pvq_max_k(Dg, budget)
        if sbits:
            e, c = pvq.pvq_beta_tables(Dg, c8 // Dg, sbits)
            cx = pvq.pvq_ctx_create(Dg, Kg, sbits, e, c)
        else:
            cx = pvq.pvq_ctx_create(Dg, Kg)
        pk = pvq.alloc_packed(cx, r8, c8, dev)
        te = timed_ms(torch, lambda: pvq.pvq_encode(cx, W8, out=pk), reps=5)
        td = timed_ms(torch, lambda: pvq.pvq_decode(cx, pk, out=Wo8), reps=5)
        G_ = c8 // Dg
        codes = r8 * ((G_ * cx.index_bits + 31) // 32 * 4 + ((G_ * sbits + 31) // 32 * 4 if sbits else G_ * 4))
        rown = r8 * 4 if sbits else 0
        out[label] = {
            "shape": [r8, c8], "D": Dg, "K": Kg, "index_bits": cx.index_bits, "scale_bits": sbits,
            "bits_per_weight": round(8.0 * codes / n8, 3),
            "encode_ms": round(te, 4), "encode_gweights_per_s": gw(n8, te), "encode_GBps": gbps(2 * n8 + codes + rown, te),
            "decode_ms": round(td, 4), "decode_gweights_per_s": gw(n8, td), "decode_GBps": gbps(2 * n8 + codes + rown, td),
        }
        cx.close()

    enc_dec(8, 24, 8, "config1_llama3_8b_up_D8_8bit_codes")
    enc_dec(16, 52, 0, "config2_D16_52bit_index_f32_amplitudes")
    enc_dec(32, 104, 0, "config2_D32_104bit_index_f32_amplitudes")
    del W8, Wo8

    # config 3: decode only over the seven shapes (3.25 bits per weight: 24-bit index + 2-bit code per 8 weights)
    K = pvq.pvq_max_k(8, 24)
    ctxs, layers = {}, []
    total_w = total_b = 0
    for i, (name, (r, c)) in enumerate(si.LLAMA3_70B_SHAPES.items()):
        if c not in ctxs:
            e, cc = pvq.pvq_beta_tables(8, c // 8, 2)
            ctxs[c] = pvq.pvq_ctx_create(8, K, 2, e, cc)
        Wl = si.gaussian_weights_device(r, c, 0.015, si.BASE_SEED + 30 + i, dev)
        pk = pvq.pvq_encode(ctxs[c], Wl)
        del Wl
        nbytes = pk.index.numel() * 4 + pk.scale.numel() * 4 + r * 4 + 2 * r * c
        layers.append((name, r, c, pk, nbytes))
        total_w += r * c
        total_b += nbytes
    biggest = max(r * c for _, r, c, _, _ in layers)
    Wo = torch.empty(biggest, dtype=torch.bfloat16, device=dev)

    def decode_layer():
        for _, r, c, pk, _ in layers:
            pvq.pvq_decode(ctxs[c], pk, out=Wo[: r * c].view(r, c))
    t_all = timed_ms(torch, decode_layer, reps=5)
    per = {}
    for name, r, c, pk, nbytes in layers:
        t = timed_ms(torch, lambda: pvq.pvq_decode(ctxs[c], pk, out=Wo[: r * c].view(r, c)), reps=5)
        per[name] = {"shape": [r, c], "ms": round(t, 4), "GBps": gbps(nbytes, t)}
    out["config3_llama3_70b_layer_decode_bf16"] = {
        "weights": total_w, "algorithmic_bytes": total_b, "ms": round(t_all, 4),
        "gweights_per_s": gw(total_w, t_all), "GBps": gbps(total_b, t_all),
        "frac_of_hbm_peak": round(total_b / (t_all * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4), "per_shape": per,
    }
    for cx in ctxs.values():
        cx.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of the oracle's sample (0 = auto)")
    ap.add_argument("--sets", type=int, default=4, help="sets of packed planes the steps rotate over")
    ap.add_argument("--only", default="", help="comma-separated subset of encode,decode,gemv_b1,gemv_b4,"
                    "gemv_b16 to run in the timed steps (profiling aid; the JSON line is then partial)")
    ap.add_argument("--steps-only", action="store_true",
                    help="leave out the back-to-back and cache-warm loops of the batch-1 kernel, so that a kernel "
                         "trace of the run holds the launches of the timed steps and the warm-up only")
    ap.add_argument("--extras", action="store_true",
                    help="after the timed steps also time, on the same matrix: pvq_encode with least-squares "
                    "amplitudes, and the D=16 / 52-bit index / 4-bit amplitude setting (generic kernels)")
    ap.add_argument("--no-configs", action="store_true",
                    help="leave out the other workloads (configs 1-3) and the device copy rate that follow the steps")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of a known size (256 MiB read + 256 MiB written), so "
                    "that a counter run can scale FETCH_SIZE / WRITE_SIZE against a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus must be 1 (rows would shard across "
                 "GPUs without any exchange; nothing here runs on a second GPU)")

    import numpy as np
    import torch

    import paper_2410_16926_amd as pvq
    import synth_inputs as si

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    K = pvq.pvq_max_k(D, INDEX_BUDGET)
    G = COLS // D
    edges, centers = pvq.pvq_beta_tables(D, G, SCALE_BITS)
    ctx = pvq.pvq_ctx_create(D, K, SCALE_BITS, edges, centers)

    # synthetic weights: Gaussian, block Hadamard rotation along the input dim, bf16
    t_gen = time.perf_counter()
    W = si.gaussian_weights_device(ROWS, COLS, 0.015, si.BASE_SEED + 4, dev)
    xs = {}
    xf1 = None
    for B in BATCHES:
        xf, xb = si.activations(B, COLS, seed=si.BASE_SEED + 4 + B)
        xs[B] = torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16)
        if B == 1:
            xf1 = xf
    t_gen = time.perf_counter() - t_gen

    sets = [pvq.alloc_packed(ctx, ROWS, COLS, dev) for _ in range(max(1, args.sets))]
    Wout = torch.empty((ROWS, COLS), dtype=torch.bfloat16, device=dev)
    ys = {B: torch.empty((B, ROWS), dtype=torch.float32, device=dev) for B in BATCHES}

    names = ["encode", "decode"] + [f"gemv_b{B}" for B in BATCHES]
    only = set(filter(None, args.only.split(",")))
    if only - set(names):
        sys.exit(f"bench.py: --only takes names from {names}")
    # every set holds valid codes before the first step: a step's products read other sets than the one it encodes
    for p in sets:
        pvq.pvq_encode(ctx, W, out=p)

    def step(i, events=None):
        p = sets[i % len(sets)]
        ev = events
        if ev: ev[0].record()
        if not only or "encode" in only:
            pvq.pvq_encode(ctx, W, out=p)
        if ev: ev[1].record()
        if not only or "decode" in only:
            pvq.pvq_decode(ctx, p, out=Wout)
        if ev: ev[2].record()
        for j, B in enumerate(BATCHES):
            # each product reads the set that has gone longest without being touched (all sets hold the same
            # codes), so that its codes come from HBM and not from the last-level cache
            if not only or f"gemv_b{B}" in only:
                pvq.pvq_decode_gemv(ctx, sets[(i + 1 + j) % len(sets)], xs[B], out=ys[B])
            if ev: ev[3 + j].record()

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    all_events = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)]
                  for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, all_events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    per_step = {n: [ev[j].elapsed_time(ev[j + 1]) for ev in all_events] for j, n in enumerate(names)}
    ms = {n: sum(v) / len(v) for n, v in per_step.items()}
    for n in names:
        if only and n not in only:
            ms[n] = float("nan")
    g1 = sorted(per_step["gemv_b1"])

    weights = ROWS * COLS
    ab = {B: algorithmic_bytes(ROWS, COLS, ctx.index_bits, SCALE_BITS, B) for B in BATCHES}
    gbps = lambda nbytes, t_ms: nbytes / (t_ms * 1e-3) / 1e9

    # Extra figure: the dominant kernel launched back to back between two events.  The per-step events
    # above (which `value` and `roofline` use) also count the event packets and the gaps between unlike
    # kernels, a few us per kernel, and every launch there follows a kernel that has just swept the
    # caches; back to back the tables stay cached and launches overlap their ends.
    b2b = ms["gemv_b1"]
    if args.steps_only:
        b2b = warm = float("nan")
    elif not only or "gemv_b1" in only:
        n = max(args.steps, 10)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            pvq.pvq_decode_gemv(ctx, sets[i % len(sets)], xs[1], out=ys[1])
        e1.record()
        torch.cuda.synchronize()
        b2b = e0.elapsed_time(e1) / n
        # and with one set of packed planes only (95 MB: it stays in the last-level cache)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            pvq.pvq_decode_gemv(ctx, sets[0], xs[1], out=ys[1])
        e1.record()
        torch.cuda.synchronize()
        warm = e0.elapsed_time(e1) / n
    else:
        warm = float("nan")
    gemv1 = gbps(ab[1]["gemv"], ms["gemv_b1"] if ms["gemv_b1"] == ms["gemv_b1"] else b2b)

    result = {
        "metric": "pvq_decode_gemv_hbm_GBps",
        "value": round(gemv1, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall * 1e3 / args.steps, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {
            "workload": "llama3-70b gate_proj 28672x8192 bf16, D=8 K=16 (24-bit index) + 2-bit Beta "
                        "amplitude code = 3.25 bpw; step = encode + decode(bf16) + decode_gemv batch 1/4/16",
            "rows": ROWS, "cols": COLS, "D": D, "K": K, "index_bits": ctx.index_bits,
            "scale_bits": SCALE_BITS, "packed_sets": len(sets),
        },
        "kernel_ms": {n: round(v, 4) for n, v in ms.items()},
        "gemv_b1_ms_median_min": [round(g1[len(g1) // 2], 4), round(g1[0], 4)],
        "gemv_b1_back_to_back_ms": round(b2b, 4),
        "gemv_b1_single_set_cache_warm_ms": round(warm, 4),
        # the products' arithmetic against the vector ALU (2*rows*cols*batch flop; fp32 vector peak 157.3 TFLOP/s):
        # far below it at every batch size, the kernels are bound by decoding, not by HBM or by the products
        "gemv_tflops": {f"b{B}": round(2.0 * weights * B / (ms[f"gemv_b{B}"] * 1e-3) / 1e12, 2) for B in BATCHES},
        "pct_of_hbm_peak": round(100 * gemv1 / HBM_PEAK_GBPS, 2),
        "encode_gweights_per_s": round(weights / (ms["encode"] * 1e-3) / 1e9, 2),
        "decode_gweights_per_s": round(weights / (ms["decode"] * 1e-3) / 1e9, 2),
        "decode_GBps": round(gbps(ab[1]["decode"], ms["decode"]), 1),
        "gemv_gweights_per_s": {f"b{B}": round(weights / (ms[f"gemv_b{B}"] * 1e-3) / 1e9, 2) for B in BATCHES},
        "gemv_GBps": {f"b{B}": round(gbps(ab[B]["gemv"], ms[f"gemv_b{B}"]), 1) for B in BATCHES},
        "roofline": {
            "kernel": "pvq_decode_gemv batch 1",
            "bound": "hbm",
            "achieved": round(gemv1, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(gemv1 / HBM_PEAK_GBPS, 4),
            "traffic": read_traffic(),
            "traffic_source": TRAFFIC_FILE + " (committed rocprofv3 counter summary of this kernel; "
                              "not measured by this run)",
            "algorithmic_bytes_per_launch": ab[1]["gemv"],
        },
        "input_generation_s": round(t_gen, 1),
    }
    # which kernels each batch size ran on, and its fraction of both roofs: HBM (algorithmic bytes) and the
    # arithmetic unit of its path (fp32 vector ALU 157.3 TFLOP/s; dense bf16 matrix cores 2500 TFLOP/s: the
    # pulses go in as they are, exact in bf16, so the unit does the product's flops once, in 4 x 4 x 4 blocks
    # whose own rate is a quarter of that peak)
    paths = {}
    for B in BATCHES:
        plan = pvq.pvq_decode_gemv_plan(ctx, ROWS, COLS, B)
        t = ms[f"gemv_b{B}"]
        flops = 2.0 * weights * B / (t * 1e-3) / 1e12
        mfma = any(k.startswith("mfma") for k, _ in plan)
        paths[f"b{B}"] = {
            "passes": [f"{k} x{n}" for k, n in plan],
            "frac_of_hbm_peak": round(gbps(ab[B]["gemv"], t) / HBM_PEAK_GBPS, 4),
            "arithmetic_roof": "mfma_bf16" if mfma else "valu_fp32",
            "frac_of_arithmetic_peak": round(flops / 2500.0 if mfma else flops / 157.3, 4),
            "binds": "neither: decoding (LDS table lookups and integer work)",
        }
    result["gemv_paths"] = paths
    if not only and not args.steps_only and not args.no_configs:
        result["configs"] = other_configs(torch, pvq, si, dev)

    if args.extras:
        def timed(fn, reps=5):
            return timed_ms(torch, fn, reps=max(reps, 9))
        ex = {}
        ctx.set_amplitude("ls")
        ex["encode_ls_ms"] = round(timed(lambda: pvq.pvq_encode(ctx, W, out=sets[0])), 4)
        ctx.set_amplitude("norm")
        K16 = pvq.pvq_max_k(16, 52)
        e16, c16 = pvq.pvq_beta_tables(16, COLS // 16, 4)
        ctx16 = pvq.pvq_ctx_create(16, K16, 4, e16, c16)
        ctx16.set_amplitude("ls")
        p16 = pvq.alloc_packed(ctx16, ROWS, COLS, dev)
        ex["d16_k33_4bit"] = {
            "encode_ms": round(timed(lambda: pvq.pvq_encode(ctx16, W, out=p16)), 4),
            "decode_ms": round(timed(lambda: pvq.pvq_decode(ctx16, p16, out=Wout)), 4),
            "gemv_b1_ms": round(timed(lambda: pvq.pvq_decode_gemv(ctx16, p16, xs[1], out=ys[1])), 4),
        }
        ctx16.close()
        K32 = pvq.pvq_max_k(32, 104)
        ctx32 = pvq.pvq_ctx_create(32, K32)
        p32 = pvq.alloc_packed(ctx32, ROWS, COLS, dev)
        ex["d32_k60_f32_amplitudes"] = {
            "encode_ms": round(timed(lambda: pvq.pvq_encode(ctx32, W, out=p32)), 4),
            "decode_ms": round(timed(lambda: pvq.pvq_decode(ctx32, p32, out=Wout)), 4),
            "gemv_b1_ms": round(timed(lambda: pvq.pvq_decode_gemv(ctx32, p32, xs[1], out=ys[1])), 4),
        }
        ctx32.close()
        del p16, p32
        # App. C.2: the size table on the GPU (one workgroup, a latency-bound scan), and the oracle's beside it
        from oracle import pvq_oracle as oracle
        for (d_, k_, w_) in ((32, 60, 4), (128, 187, 12)):
            t_gpu = timed(lambda: pvq.pvq_size_table_device(d_, k_, w_, dev), reps=20)
            t0 = time.perf_counter(); oracle.size_table(d_, k_); t_cpu = time.perf_counter() - t0
            ex[f"size_table_D{d_}_K{k_}"] = {"gpu_ms": round(t_gpu, 4), "oracle_cpu_ms": round(t_cpu * 1e3, 3)}
        # Sec. 3.3 Step 1: randomised Hadamard rotation of the rows, bf16 in and out (HBM-bound: one read,
        # one write of the matrix)
        sg = torch.randint(0, 2, (COLS,), dtype=torch.uint8, device=dev)
        had = {}
        for blk in (64, 512, 4096, 8192):
            ms = timed(lambda: pvq.pvq_hadamard(W, blk, sg, out=Wout), reps=10)
            had[f"block_{blk}"] = {"ms": round(ms, 4), "GBps": round(2 * W.numel() * W.element_size() / ms / 1e6, 1)}
        ex["hadamard_bf16"] = had
        # the same rotation fused in front of the D = 8 encoder (the rotated values are never written), against
        # the two calls with a float32 matrix in between
        Wf = torch.empty((ROWS, COLS), dtype=torch.float32, device=dev)
        rot8 = {}
        for blk in (64, 512, 4096, 8192):
            tf = timed(lambda: pvq.pvq_rotate_encode(ctx, W, blk, sg, out=sets[0]), reps=10)
            t2 = timed(lambda: (pvq.pvq_hadamard(W, blk, sg, out=Wf), pvq.pvq_encode(ctx, Wf, out=sets[0])), reps=10)
            rot8[f"block_{blk}"] = {"fused_ms": round(tf, 4), "two_calls_ms": round(t2, 4)}
        ex["rotate_encode_d8"] = rot8
        del Wf
        # on-the-fly activation quantisation (Sec. 3.2, Sec. 4.3): groups of 128 values, 3 bits per value
        # (K = 187, 384-bit indices), a prefill batch and a decode batch of hidden size 8192
        K128 = pvq.pvq_max_k(128, 384)
        ctxa = pvq.pvq_ctx_create(128, K128)
        act = {"D": 128, "K": K128, "index_bits": ctxa.index_bits}
        for tokens in (4096, 16):
            _, xb = si.activation_matrix(tokens, 8192, seed=7)
            X = torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16)
            pa = pvq.alloc_packed(ctxa, tokens, 8192, dev)
            Xo = torch.empty_like(X)
            te = timed(lambda: pvq.pvq_encode(ctxa, X, out=pa), reps=10)
            td = timed(lambda: pvq.pvq_decode(ctxa, pa, out=Xo), reps=10)
            sga = torch.randint(0, 2, (8192,), dtype=torch.uint8, device=dev)
            tf = timed(lambda: pvq.pvq_rotate_encode(ctxa, X, 8192, sga, out=pa), reps=10)
            act[f"tokens_{tokens}"] = {"encode_ms": round(te, 4), "decode_ms": round(td, 4),
                                       "encode_Gvalues_per_s": round(tokens * 8192 / te / 1e6, 2),
                                       "rotate_encode_ms": round(tf, 4)}
            if tokens == 16:
                xf = si.bf16_bits_to_f32(xb)
                t0 = time.perf_counter(); oracle.encode(xf, 128, K128, nthreads=1); t_cpu = time.perf_counter() - t0
                act["oracle_one_core_Gvalues_per_s"] = round(tokens * 8192 / t_cpu / 1e9, 5)
        ctxa.close()
        ex["activation_pvq"] = act
        # Sec. 3.3 Step 6: error correction group after group: a key / value projection (1024 x 8192), a square
        # projection (8192 x 8192) and the benchmark's matrix, float32 in place.  For timing the factor is any well-conditioned upper triangular matrix; the oracle beside it
        # on 8 rows (rows are independent), one core.
        gcor = torch.Generator(device=dev); gcor.manual_seed(11)
        Uc = torch.triu(torch.randn((COLS, COLS), generator=gcor, device=dev) * (0.3 / COLS ** 0.5)) + torch.eye(COLS, device=dev)
        ctxc = pvq.pvq_ctx_create(8, K)
        for cr, cc in ((1024, COLS), (8192, COLS), (ROWS, COLS)):
            Wc0 = torch.randn((cr, cc), generator=gcor, device=dev) * 0.02
            work = torch.empty((cr * 1024,), dtype=torch.uint8, device=dev)
            Wc = Wc0.clone()
            pvq.pvq_correct(ctxc, Wc, Uc, work=work); torch.cuda.synchronize()
            ms = []
            for _ in range(3):
                Wc.copy_(Wc0); torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); pvq.pvq_correct(ctxc, Wc, Uc, work=work); e1.record(); torch.cuda.synchronize()
                ms.append(e0.elapsed_time(e1))
            t_ms = sorted(ms)[1]
            flop = float(cr) * cc * cc          # one multiply-add per element and earlier column: 2 x rows x cols^2 / 2
            ex[f"correct_{cr}x{cc}"] = {"ms": round(t_ms, 3), "TFLOPs": round(flop / t_ms / 1e9, 2),
                                        "frac_of_fp32_alu_peak": round(flop / t_ms / 1e9 / 78.6, 3),
                                        "gpu_rows_per_s": round(cr / t_ms * 1e3, 1)}
            if cr == 8192:
                w8, u8 = Wc0[:8].cpu().numpy(), Uc.cpu().numpy()
                t0 = time.perf_counter(); oracle.correct(w8, u8, 8, K); t_cpu = time.perf_counter() - t0
                ex[f"correct_{cr}x{cc}"]["oracle_one_core_rows_per_s"] = round(8 / t_cpu, 3)
            del Wc0, Wc, work
        ctxc.close()
        del Uc
        result["extras"] = ex

    if not args.no_cpu_baseline:
        threads = min(os.cpu_count() or 1, 16)
        rows = args.cpu_rows or 1024 * threads    # about 20-40 core-seconds of the oracle
        rows = min(rows, ROWS)
        sample = W[:rows].to(torch.float32).cpu().numpy()      # the bf16 values, widened exactly
        result["cpu_baseline"] = cpu_baseline(np.ascontiguousarray(sample), xf1, K, threads)
        one = cpu_baseline(np.ascontiguousarray(sample[:max(1, rows // threads)]), xf1, K, 1)
        result["cpu_baseline"]["one_core"] = {k: one[k] for k in ("value", "decode_gemv_gweights_per_s",
                                                                   "encode_gweights_per_s", "seconds")}

    ctx.close()

    def clean(v):   # a partial run (--only) leaves figures undefined: null, not NaN, in the JSON line
        if isinstance(v, float) and v != v:
            return None
        if isinstance(v, dict):
            return {k: clean(x) for k, x in v.items()}
        if isinstance(v, list):
            return [clean(x) for x in v]
        return v

    print(json.dumps(clean(result)))


if __name__ == "__main__":
    main()
