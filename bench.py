"""Benchmark of libyoco on one MI355X.

One "step" is one pass of the whole attention hot path over one synthetic
batch at the headline shape (T=32768, 24 query heads x 128, window 1024):
  SWA prefill (24 KV heads)  ->  global K^/V^ write of the T rows (8 KV heads)
  ->  cross-attention prefill of the last position  ->  one split-KV decode
  step (pass 1 + log-sum-exp merge) over that cache.
`value` is T / step time. The roofline object is for the dominant kernel, the
SWA prefill (algorithmic flops = 4 * d * unmasked (query, key) pairs). The two
decode workloads the metric also names (16 x 32K and 1 x 512K caches, 13
cross-decoder layers back to back) are timed in the same run and reported
under "decode" as GB/s against the HBM peak. The fp64 oracle is timed on a
bounded sample of the same SWA workload on the host cores ("cpu_baseline").
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2516.6    # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "hbm_traffic_swa_prefill_32k_and_decode.md")


def swa_traffic_from_profile():
    """HBM bytes of one SWA prefill launch at the headline shape, read at run time from the committed rocprofv3
    summary (two --pmc runs, FETCH_SIZE then WRITE_SIZE, each scaled by what the counter reads for a 1 GiB copy; the
    file gives commands and factors). Returns (fetch_bytes, write_bytes) or None when the file or its rows are missing:
    the line then carries traffic = null rather than a stale constant."""
    try:
        got = {}
        with open(TRAFFIC_PROFILE) as f:
            for line in f:
                cells = [c.strip() for c in line.split("|")]
                if len(cells) > 6 and cells[1].startswith("swa_mfma_kernel") and cells[2] in ("FETCH_SIZE", "WRITE_SIZE"):
                    got[cells[2]] = float(cells[5])          # the "scaled bytes" column
        return (got["FETCH_SIZE"], got["WRITE_SIZE"])
    except (OSError, KeyError, ValueError):
        return None


def swa_flops(T, H, d, C):
    pairs = C * (C + 1) // 2 + (T - C) * C if T > C else T * (T + 1) // 2
    return 4.0 * d * pairs * H


def graph_ms(step, reps):
    """Average duration of `step` (a run of library launches on the current stream) replayed from a HIP graph:
    the launch-bound decode loops as a serving loop would issue them, without the per-call host time of Python."""
    import torch
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    times = []
    for rep in range(2 + reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        if rep >= 2:
            times.append(e0.elapsed_time(e1))
    return sum(times) / len(times)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-decode", action="store_true", help="skip the two decode workloads")
    ap.add_argument("--only", choices=["all", "swa", "decode", "gret", "calib"], default="all",
                    help="profiling aid: 'swa' runs only the SWA prefill launches, 'decode' only the decode workloads, "
                         "'gret' only the gated-retention launches, "
                         "'calib' only a 1 GiB device-to-device copy (the known-size kernel the HBM byte counters are scaled by)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-e2e", action="store_true", help="skip the whole-stack prefill timing at T = 131072")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2405_05254_amd as yoco
    import yoco_synth as ys

    yoco.lib()                                   # no library, no benchmark: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda"
    if args.only == "calib":
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calib": "3 device-to-device copies of 1 GiB (reads 2^30 B, writes 2^30 B each)"}))
        return
    c = ys.CONFIGS["swa_prefill_32k"]
    T, H, d, C = c["T"], c["Hq"], c["d"], c["window"]
    Hkv_cache = ys.CONFIGS["decode_b16_32k"]["Hkv"]
    scale = 1.0 / math.sqrt(d)

    # ---- inputs, resident in HBM before any timing
    qn, kn, vn = ys.qkv(c["seed"], T, H, H, d, c["std"], "bf16")
    q, k, v = (torch.from_numpy(x[None]).to(dev).to(torch.bfloat16) for x in (qn, kn, vn))
    o = torch.empty_like(q)
    khat = ys.device_normal((T, Hkv_cache, d), 11, 1.0, torch.bfloat16, dev)
    vhat = ys.device_normal((T, Hkv_cache, d), 12, 1.0, torch.bfloat16, dev)
    cache = yoco.KVCache(1, Hkv_cache, d, T, torch.bfloat16)
    q_last = ys.device_normal((1, H, d), 13, 1.0, torch.bfloat16, dev)
    o_last = torch.empty_like(q_last)
    o_dec = torch.empty_like(q_last)
    lens = torch.tensor([T], dtype=torch.int64, device=dev)
    nbytes, _ = yoco.cross_attn_decode_workspace(cache, H)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    if args.only != "all":
        args.no_cpu_baseline = True
    if args.only == "swa":
        args.no_decode = True

    def step(ev=None):
        if args.only in ("decode", "gret"):
            return
        if ev:
            ev[0].record()
        yoco.swa_prefill(q, k, v, C, scale, out=o)
        if ev:
            ev[1].record()
        if args.only == "swa":
            return
        yoco.global_kv_write(cache, khat, vhat, 0, 0)
        yoco.cross_attn_prefill(cache, q_last, 0, T - 1, scale, out=o_last, workspace=ws)
        yoco.cross_attn_decode(cache, q_last, lens, scale, ws, out=o_dec)

    # The chip raises its clock over the first tens of milliseconds of work: a step timed right after idle runs 10 %
    # slower than the sustained rate (measured: 0.62 ms per SWA launch with no warm-up, 0.585 after 10 steps, 0.555
    # after 100 or 1000). A serving process runs sustained, so the first steps after idle are timed for the record
    # (`after_idle`), then the step runs untimed until the clock has settled, then come the W warm-up steps and the K
    # timed steps of the contract.
    after_idle = None
    if args.only in ("all", "swa"):
        torch.cuda.synchronize()
        t_idle = time.perf_counter()
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        after_idle = dict(steps=10, ms_per_step=round((time.perf_counter() - t_idle) * 1e3 / 10, 4))
        settle_steps, t_settle = 0, time.perf_counter()
        while time.perf_counter() - t_settle < 0.25:
            for _ in range(20):
                step()
            torch.cuda.synchronize()
            settle_steps += 20
        after_idle["untimed_settle_steps"] = settle_steps
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    swa_times = sorted(a.elapsed_time(b) for a, b in evs) if args.only not in ("decode", "gret") else [float("nan")]
    swa_ms = sum(swa_times) / len(swa_times)
    flops = swa_flops(T, H, d, C)
    swa_tflops = flops / (swa_ms * 1e-3) / 1e12
    # the same launch with the caches flushed before it (a 512 MiB buffer is rewritten between repetitions)
    swa_flushed = None
    if args.only in ("all", "swa"):
        flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
        ft = []
        for rep in range(20):
            flush.fill_(rep & 0xff)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            yoco.swa_prefill(q, k, v, C, scale, out=o)
            e1.record()
            torch.cuda.synchronize()
            ft.append(e0.elapsed_time(e1))
        ft.sort()
        swa_flushed = dict(ms_median=round(ft[len(ft) // 2], 4), ms_min=round(ft[0], 4))
        del flush

    # ---- what this machine can do: an MFMA-only loop and a streaming read, measured in the same run
    ceilings = None
    if args.only == "all":
        g = torch.Generator(device=dev)
        g.manual_seed(5)
        seed_rand = torch.empty(8192, dtype=torch.float32, device=dev).normal_(0.0, 0.5, generator=g).to(torch.bfloat16)
        seed_zero = torch.zeros(8192, dtype=torch.bfloat16, device=dev)
        sink = torch.zeros(4, dtype=torch.float32, device=dev)
        big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
        big.fill_(1)

        def rate(fn, reps):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            work = sum(fn() for _ in range(reps))
            e1.record()
            torch.cuda.synchronize()
            return work / (e0.elapsed_time(e1) * 1e-3)

        ceilings = dict(
            mfma_bf16_TFLOPs_random_operands=round(rate(lambda: yoco.ceiling_mfma(seed_rand, sink, 20000, 256), 3) / 1e12, 1),
            mfma_bf16_TFLOPs_zero_operands=round(rate(lambda: yoco.ceiling_mfma(seed_zero, sink, 20000, 256), 3) / 1e12, 1),
            attn_loop_lds_fed_TFLOPs=round(rate(lambda: yoco.ceiling_attn_loop(seed_rand, sink, 4000, 256, 1), 3) / 1e12, 1),
            attn_loop_lds_fed_with_softmax_TFLOPs=round(rate(lambda: yoco.ceiling_attn_loop(seed_rand, sink, 4000, 256, 2), 3) / 1e12, 1),
            stream_read_GBps=round(max(rate(lambda n=n: yoco.ceiling_stream_read(big, sink, n), 10) for n in (256, 512, 1024)) / 1e9, 1),
            note="MFMA-only loop (2 wavefronts per SIMD, register operands); the attention inner loop on its own with random "
                 "operands (every MFMA's A operand a fresh LDS fragment; then with the softmax work of 32 scores per lane and 32 "
                 "MFMAs interleaved): no staging, masks, barriers or tile walk, i.e. what the prefill kernel could reach at best; "
                 "and a 2 GiB streaming read with 128-bit nontemporal loads (best of 1, 2 and 4 workgroups per CU)")
        # the MFMA-only loop keeps the matrix pipe full (32 clocks per v_mfma_f32_32x32x16, measured), so its rate is a
        # reading of the clock the chip holds under that load: 2516.6 TFLOP/s is the pipe at 2.4 GHz
        ceilings["clock_GHz_in_the_mfma_loop"] = dict(
            random_operands=round(2.4 * ceilings["mfma_bf16_TFLOPs_random_operands"] / MFMA_BF16_PEAK_TFLOPS, 3),
            zero_operands=round(2.4 * ceilings["mfma_bf16_TFLOPs_zero_operands"] / MFMA_BF16_PEAK_TFLOPS, 3))
        del big

    # ---- the decode workloads of the metric: 13 cross-decoder layers over one shared cache
    decode = {}
    if not args.no_decode and args.only != "gret":
        del q, k, v, o
        for name in ("decode_b16_32k", "decode_b1_512k", "decode_b16_32k_int8", "decode_b1_512k_int8"):
            coded = name.endswith("_int8")                       # the same workload over the 8-bit cache
            dc = ys.CONFIGS[name[:-5] if coded else name]
            B, N, Hq, Hkv, layers = dc["B"], dc["N"], dc["Hq"], dc["Hkv"], dc["layers"]
            kvc = yoco.KVCache(B, Hkv, d, N, torch.int8 if coded else torch.bfloat16)
            if coded:
                for b in range(B):                               # rows are coded by the library's own write call
                    yoco.global_kv_write(kvc, ys.device_normal((N, Hkv, d), dc["seed"] + 2 * b, dc["std"], torch.bfloat16, dev),
                                         ys.device_normal((N, Hkv, d), dc["seed"] + 2 * b + 1, dc["std"], torch.bfloat16, dev), b, 0)
            else:
                Kp, Vp = kvc.planes()
                Kp.copy_(ys.device_normal(Kp.shape, dc["seed"], dc["std"], torch.bfloat16, dev))
                Vp.copy_(ys.device_normal(Vp.shape, dc["seed"] + 1, dc["std"], torch.bfloat16, dev))
                del Kp, Vp
            qs = [ys.device_normal((B, Hq, d), 100 + i, dc["std"], torch.bfloat16, dev) for i in range(layers)]
            od = torch.empty_like(qs[0])
            ln = torch.full((B,), N, dtype=torch.int64, device=dev)
            nb, splits = yoco.cross_attn_decode_workspace(kvc, Hq)
            w = torch.empty(nb, dtype=torch.uint8, device=dev)
            reps = max(3, min(20, args.steps // 2))
            times = []
            for rep in range(2 + reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(layers):
                    yoco.cross_attn_decode(kvc, qs[i], ln, scale, w, out=od)
                e1.record()
                torch.cuda.synchronize()
                if rep >= 2:
                    times.append(e0.elapsed_time(e1))
            ms = sum(times) / len(times)
            cache_bytes = 2.0 * B * N * Hkv * (d + 4 if coded else d * 2)     # codes + one fp32 scale per row, or bf16
            gbs = layers * cache_bytes / (ms * 1e-3) / 1e9
            decode[name] = dict(ms_per_13_layers=round(ms, 4), ms_per_layer=round(ms / layers, 4), min_ms=round(min(times), 4),
                                GBps=round(gbs, 1), frac_of_hbm_peak=round(gbs / HBM_PEAK_GBS, 4), splits=splits,
                                cache_bytes=int(cache_bytes))
            if coded:
                decode[name]["speedup_over_bf16_cache"] = round(decode[name[:-5]]["ms_per_13_layers"] / ms, 3)
            del kvc, w, qs
            # No torch.cuda.empty_cache() anywhere in this file: a 2 GiB block handed back to the driver and mapped again
            # measures 6 % slower in the next workload (0.323 against 0.303 ms per layer, whatever its shape); torch's
            # caching allocator keeps the blocks and the 288 GB hold all of them.
        # one generation step of the self-decoder: 13 layers, each stores the new row in its own rolling
        # window cache (window 1024, 24 heads) and attends to it in the same launch, 16 sequences at position 32767
        sc = ys.CONFIGS["swa_prefill_32k"]
        B, Cw, Hs, layers = 16, sc["window"], sc["Hq"], 13
        rings = [yoco.KVCache(B, Hs, d, Cw, torch.bfloat16) for _ in range(layers)]
        for i, r in enumerate(rings):
            for pl in r.planes():
                pl.copy_(ys.device_normal(pl.shape, 300 + i, 1.0, torch.bfloat16, dev))
        qs = [ys.device_normal((B, Hs, d), 400 + i, 1.0, torch.bfloat16, dev) for i in range(layers)]
        k_new = ys.device_normal((B, Hs, d), 500, 1.0, torch.bfloat16, dev)
        od = torch.empty_like(qs[0])
        pos = torch.full((B,), 32767, dtype=torch.int64, device=dev)
        ln = pos + 1
        nb, splits = yoco.cross_attn_decode_workspace(rings[0], Hs)
        w = torch.empty(nb, dtype=torch.uint8, device=dev)
        times = []
        for rep in range(2 + max(3, min(20, args.steps // 2))):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(layers):
                yoco.swa_decode(rings[i], qs[i], ln, scale, w, out=od, k_new=k_new, v_new=k_new)   # stores the new row itself
            e1.record()
            torch.cuda.synchronize()
            if rep >= 2:
                times.append(e0.elapsed_time(e1))
        ms = sum(times) / len(times)
        ring_bytes = 2.0 * B * Cw * Hs * d * 2
        gbs = layers * ring_bytes / (ms * 1e-3) / 1e9

        def swa_step():
            for i in range(layers):
                yoco.swa_decode(rings[i], qs[i], ln, scale, w, out=od, k_new=k_new, v_new=k_new)
        gms = graph_ms(swa_step, len(times))
        decode["swa_decode_b16_w1024"] = dict(ms_per_13_layers=round(ms, 4), ms_per_layer=round(ms / layers, 4),
                                              GBps=round(gbs, 1), frac_of_hbm_peak=round(gbs / HBM_PEAK_GBS, 4),
                                              hip_graph_ms_per_13_layers=round(gms, 4),
                                              hip_graph_frac_of_hbm_peak=round(layers * ring_bytes / (gms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                              splits=splits, ring_bytes_per_layer=int(ring_bytes))
        del rings, qs, w

    # ---- gated retention, the paper's other self-decoder module, at the same shape (reported, not part of `value`)
    gret = None
    if not args.no_decode and args.only in ("all", "gret"):
        gq, gk, gv, glg = ys.gret_inputs(c["seed"], 1, T, H, d, d, 1.0, "bf16")
        gq, gk, gv = (torch.from_numpy(x).to(dev).to(torch.bfloat16) for x in (gq, gk, gv))
        glg = torch.from_numpy(glg).to(dev)
        go = torch.empty_like(gv)
        chunk = 256
        gws = torch.empty(yoco.gret_prefill_workspace(1, T, H, d, d, chunk, yoco.BF16), dtype=torch.uint8, device=dev)
        gst = torch.empty(1, H, d, d, dtype=torch.float32, device=dev)
        times = []
        for rep in range(3 + max(3, min(20, args.steps // 2))):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            yoco.gret_prefill(gq, gk, gv, glg, scale, chunk=chunk, state_out=gst, workspace=gws, out=go)
            e1.record()
            torch.cuda.synchronize()
            if rep >= 3:
                times.append(e0.elapsed_time(e1))
        ms = sum(times) / len(times)
        gflops = T * H * (4.0 * d * (chunk + 1) / 2 + 4.0 * d * d)       # inner chunk (causal half) + cross-chunk + state
        gret = {"prefill_32k": dict(ms=round(ms, 4), tokens_per_s=round(T / (ms * 1e-3), 1), chunk=chunk,
                                    TFLOPs=round(gflops / (ms * 1e-3) / 1e12, 1),
                                    workspace_bytes=gws.numel())}
        del gq, gk, gv, go, gws
        Bd, layers = 16, 13
        states = [torch.zeros(Bd, H, d, d, dtype=torch.float32, device=dev) for _ in range(layers)]
        dq = ys.device_normal((Bd, H, d), 600, 1.0, torch.bfloat16, dev)
        dlg = -torch.rand(Bd, H, device=dev) * 0.1
        do = torch.empty_like(dq)
        times = []
        for rep in range(2 + max(3, min(20, args.steps // 2))):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(layers):
                yoco.gret_decode(dq, dq, dq, dlg, states[i], scale, out=do)
            e1.record()
            torch.cuda.synchronize()
            if rep >= 2:
                times.append(e0.elapsed_time(e1))
        ms = sum(times) / len(times)
        sbytes = 2.0 * Bd * H * d * d * 4                                  # the state read and written once

        def gret_step():
            for i in range(layers):
                yoco.gret_decode(dq, dq, dq, dlg, states[i], scale, out=do)
        gms = graph_ms(gret_step, len(times))
        gret["decode_b16"] = dict(ms_per_13_layers=round(ms, 4), ms_per_layer=round(ms / layers, 4),
                                  GBps=round(layers * sbytes / (ms * 1e-3) / 1e9, 1),
                                  frac_of_hbm_peak=round(layers * sbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                  hip_graph_ms_per_13_layers=round(gms, 4),
                                  hip_graph_frac_of_hbm_peak=round(layers * sbytes / (gms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                  state_bytes_per_layer=int(sbytes / 2))
        del states

    # ---- whole-stack context (not part of `value`): the end-to-end configuration's prefill at T = 131072, once
    # with the early exit of Fig. 3 and once with every row sent through the cross-decoder. The projections,
    # norms and FFNs are torch bf16 GEMMs (not part of the library); attention and the cache are libyoco's.
    e2e = None
    if args.only == "all" and not args.no_e2e:
        from paper_2405_05254_amd.stack import YocoStack
        ec = ys.CONFIGS["e2e_early_exit_128k"]
        with torch.no_grad():
            w = ys.stack_weights_device(ec["seed"], ec["stack"], torch.bfloat16, dev)
            st = YocoStack(w, torch.bfloat16, glue_dtype=torch.bfloat16)
            del w
            tok = torch.from_numpy(ys.tokens(ec["seed"], ec["T"], ec["stack"]["vocab"])).to(dev)

            def timed(fn):
                fn()                                  # warm-up (GEMM heuristics, allocator)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                fn()
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) * 1e3

            ee_ms = timed(lambda: st.forward_early_exit(tok))
            full_ms = timed(lambda: st.forward_full(tok, rows=slice(ec["T"] - 1, ec["T"])))
            es = ec["stack"]
            eq = ys.device_normal((1, ec["T"], es["Hq"], es["d"]), 700, 0.5, torch.bfloat16, dev)
            swa_layer_ms = timed(lambda: yoco.swa_prefill(eq, eq, eq, es["window"], scale))
            # Eq. 2 on all T rows (norm, two projections, cache write), as the stack does it and with the norm folded
            # into the write call (yoco_global_kv_write_scaled)
            xm = ys.device_normal((ec["T"], es["d_model"]), 701, 1.0, torch.bfloat16, dev)
            kvc = yoco.KVCache(1, st.Hkv, st.d, ec["T"], torch.bfloat16, dev)

            def best(fn, reps=5):
                return min(timed(fn) for _ in range(reps))

            eq2_plain_ms = best(lambda: st.write_cache(xm, kvc))
            st.fused_kv_norm = True
            st.kv["gW_K"] = (st.kv["ln"].float()[:, None] * st.kv["W_K"].float()).to(torch.bfloat16)
            st.kv["gW_V"] = (st.kv["ln"].float()[:, None] * st.kv["W_V"].float()).to(torch.bfloat16)
            eq2_folded_ms = best(lambda: st.write_cache(xm, kvc))
            del st, tok, eq, xm, kvc
        e2e = dict(T=ec["T"], early_exit_prefill_ms=round(ee_ms, 1), full_forward_ms=round(full_ms, 1),
                   eq2_all_rows_ms=dict(norm_then_projections_then_write=round(eq2_plain_ms, 3),
                                        norm_folded_into_the_write=round(eq2_folded_ms, 3)),
                   early_exit_speedup=round(full_ms / ee_ms, 2), early_exit_tokens_per_s=round(ec["T"] / (ee_ms * 1e-3), 1),
                   swa_ms_per_layer=round(swa_layer_ms, 2),
                   swa_share_of_early_exit_prefill=round(es["n_self"] * swa_layer_ms / ee_ms, 3),
                   note="1.4B-shape random-init stack, 12 + 12 layers, bf16 torch GEMMs around libyoco's attention")

    # ---- the oracle on the host cores, bounded sample of the same SWA workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        rng = np.random.default_rng(1)
        n, t0, c0 = 0, time.perf_counter(), time.process_time()
        while time.perf_counter() - t0 < args.cpu_seconds:
            for _ in range(64):
                oracle.swa_row(qn, kn, vn, int(rng.integers(C, T)), int(rng.integers(0, H)), C, scale)
            n += 64
        dt = time.perf_counter() - t0
        cores = max(1, int(round((time.process_time() - c0) / dt)))      # threads that were actually busy (CPU time / wall time)
        cpu = dict(value=round(n / H / dt, 3), unit="tokens/s", cores=cores, kind="oracle",
                   sample="%d sampled (row, head) outputs of the same T=32768 x 24-head SWA workload in %.1f s; "
                          "a token = 24 head rows" % (n, dt))

    traffic = swa_traffic_from_profile()
    out = {
        "metric": "swa_prefill_tokens_per_s", "value": round(T / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "swa_prefill_32k: B=1 T=32768 24x128 heads window 1024 (+ K^/V^ write of T rows x 8 KV heads, "
                               "last-token cross-attention, one split-KV decode step)", "seed": c["seed"]},
        "swa_prefill": {"ms": round(swa_ms, 4), "ms_median": round(swa_times[len(swa_times) // 2], 4), "ms_min": round(swa_times[0], 4),
                        "tokens_per_s": round(T / (swa_ms * 1e-3), 1),
                        "TFLOPs": round(swa_tflops, 1), "frac_of_mfma_peak": round(swa_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                        "caches_flushed": swa_flushed},
        "clock_settling": None if after_idle is None else dict(
            first_steps_after_idle=dict(steps=after_idle["steps"], ms_per_step=after_idle["ms_per_step"]),
            untimed_settle_steps=after_idle["untimed_settle_steps"],
            note="the first steps of the process, timed for the record; then the step ran untimed for 0.25 s so that the chip's "
                 "clock had settled before the W warm-up steps and the K timed steps"),
        "peaks": {"mfma_bf16_TFLOPs": MFMA_BF16_PEAK_TFLOPS, "hbm_GBps": HBM_PEAK_GBS, "measured": ceilings},
        "roofline": {"kernel": "yoco_swa_prefill", "bound": "mfma", "achieved": round(swa_tflops, 1),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(swa_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": None if traffic is None else int(traffic[0] + traffic[1]),
                     "traffic_note": "not measured in this run" if traffic is None else
                     "HBM bytes per launch read from profiles/%s (rocprofv3 --pmc FETCH_SIZE %.3f GB + WRITE_SIZE %.3f GB, "
                     "scaled by a 1 GiB copy) against 0.805 GB algorithmic" % (os.path.basename(TRAFFIC_PROFILE), traffic[0] / 1e9, traffic[1] / 1e9)},
        "decode": decode,
        "gated_retention": gret,
        "e2e_early_exit_128k": e2e,
        "cpu_baseline": cpu,
        # the paper's own profiling figures (section 4.4), another machine and the whole model: context, not a target
        "paper_context": {"hardware": "H100-80GB", "model": "YOCO-3B with the gated-retention self-decoder, whole model",
                          "prefill_512k_s": {"transformer": 180, "yoco": "< 6"}, "prefill_speedup": {"32k": 2.87, "1m": 71.8},
                          "throughput_512k_tokens_per_s": {"transformer": 4.5, "yoco": 43.1}, "memory_1m_gb": 12.4},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
