#!/usr/bin/env python3
"""Benchmark of the MoE expert layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mixtral_T4096]

One "step" is one moe_layer_forward call (router, dispatch, both expert GEMMs, combine) over one
batch of seeded synthetic tokens already resident in HBM.  Prints one JSON line: whole-layer
useful TFLOP/s, ms per step, the roofline figures of the dominant kernel (GEMM1 + SwiGLU), and the
CPU oracle timed on a bounded sample of the same workload on this machine's host cores.

`--curve` additionally sweeps the skewed Mixtral-shaped workload over token loads and writes the
latency-vs-token-load table (the per-GPU profile the paper's mapping search consumes, Sec. 3.3.2)
to latency_curve.json in the output folder (--out-dir).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (published)
PEAK_HBM_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


OUT_DIR_DEFAULT = "bench_out"


def make_workload(name, seed, weights):
    import workloads as wl
    if name.startswith("mixtral_skewed_T"):
        return wl.mixtral_skewed(int(name.split("T")[-1]), seed, weights=weights)
    if name.startswith("mixtral_T"):
        return wl.mixtral(int(name.split("T")[-1]), seed, weights=weights)
    if name.startswith("fine_grained_T"):
        return wl.fine_grained(int(name.split("T")[-1]), seed, weights=weights)
    if name.startswith("ep_share_T"):
        return wl.ep_share_layer(int(name.split("T")[-1]), seed, weights=weights)
    if name.startswith("wide_few_T"):
        return wl.wide_few_experts(int(name.split("T")[-1]), seed, weights=weights)
    if name.startswith("mid_grained_T"):
        return wl.mid_grained(int(name.split("T")[-1]), seed, weights=weights)
    if name == "tiny":
        return wl.tiny(seed)
    raise SystemExit(f"unknown workload {name}")


def profiled_traffic(workload, kernel):
    """HBM-side bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary
    of this workload (FETCH_SIZE + WRITE_SIZE, scaled by the copy-kernel calibration); None if no
    summary exists for this workload."""
    path = os.path.join(ROOT, "profiles", f"gemm_{workload}_pmc.txt")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel:
                return float(parts[2])
    except OSError:
        pass
    return None


def time_layer(ctx, x, rp, bias, packed, out, steps, warmup):
    import torch
    for _ in range(warmup):
        ctx.moe_layer_forward(x, rp, bias, packed, out=out)
    torch.cuda.synchronize()
    try:
        ctx.moe_stage_times()          # drop earlier calls from the stage averages
    except Exception:
        pass
    t0 = time.perf_counter()
    for _ in range(steps):
        ctx.moe_layer_forward(x, rp, bias, packed, out=out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dt / steps * 1e3, ctx.moe_stage_times()


def time_layer_graph(moe, s, x, rp, bias, packed, out, steps, warmup):
    """The same layer call captured once into a HIP graph and replayed (a context without stage events:
    those record events into the stream)."""
    import torch
    ctx = moe.MoEContext(s.T, s.d, s.f, s.E, s.k, s.e_lo, s.E_local)
    ctx.moe_layer_forward(x, rp, bias, packed, out=out)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.moe_layer_forward(x, rp, bias, packed, out=out)
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    del graph
    ctx.close()
    return dt / steps * 1e3


def time_calls(fn, iters, warmup=3):
    """Mean milliseconds of fn() over `iters` back-to-back calls (HIP events on the current stream)."""
    import torch
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def hbm_stages(moe, s, T, seed, iters=30):
    """The three memory-bound stages on their own, each as `iters` back-to-back calls of its C-ABI entry point
    on T tokens of the workload's shape (the router of the workload, Gaussian activations): algorithmic bytes
    per call / mean time per call against the 8 TB/s HBM peak.  Algorithmic bytes: route 2*T*d + 8*T*k (+ the
    packed router); permute, with the row copy, 2*(T + A)*d + 12*A; combine 2*(A + T)*d + 8*A, A = T*k local
    assignments (all experts resident)."""
    import torch
    ctx = moe.MoEContext(T, s.d, 64, s.E, s.k)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x = torch.randn(T, s.d, device="cuda", generator=g).bfloat16()
    Wg = torch.randn(s.d, s.E, device="cuda", generator=g) * 0.02
    rp = ctx.moe_pack_router(Wg)
    idx = torch.empty((T, s.k), dtype=torch.int32, device="cuda")
    w = torch.empty((T, s.k), dtype=torch.float32, device="cuda")
    counts = torch.empty(s.E, dtype=torch.int32, device="cuda")
    A = T * s.k
    out = {}
    ms = time_calls(lambda: ctx.moe_route(x, rp, None, idx=idx, w=w, counts=counts), iters)
    out["route"] = (2.0 * T * s.d + 8.0 * A + rp.numel() * 2, ms)
    xp, offsets, row_of, tok_of = ctx.moe_permute(x, idx)
    lib, cptr = ctx.lib, ctx._ctx
    import ctypes as C
    p = lambda t: C.c_void_p(t.data_ptr())
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    ms = time_calls(lambda: lib.moe_permute(cptr, p(x), p(idx), T, p(xp), p(offsets), p(row_of), p(tok_of), st), iters)
    out["permute"] = (2.0 * (T + A) * s.d + 12.0 * A, ms)
    y = xp                                     # any [A, d] bf16 buffer serves as the experts' output
    o = torch.empty((T, s.d), dtype=torch.bfloat16, device="cuda")
    ms = time_calls(lambda: ctx.moe_combine(y, row_of, w, out=o), iters)
    out["combine"] = (2.0 * (A + T) * s.d + 8.0 * A, ms)
    ctx.close()
    return {k: {"T": T, "bytes": b, "us": ms * 1e3, "GBps": b / ms / 1e6, "frac": b / ms / 1e6 / PEAK_HBM_GBS}
            for k, (b, ms) in out.items()}


class ClockSampler:
    """Shader clock (MHz) while a load runs, read from `rocm-smi --showclocks --json` a few times a second in a
    thread of its own.  The device lowers its clock to stay inside its power limit, so the clock a kernel
    sustains is part of what bounds it."""

    def __init__(self, period=0.15):
        self.period, self.samples, self._stop, self._th = period, [], False, None

    def _run(self):
        import subprocess
        while not self._stop:
            try:
                r = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=5)
                for card in json.loads(r.stdout).values():
                    for key, val in card.items():
                        if "sclk" in key.lower() and "speed" in key.lower():
                            self.samples.append(float(str(val).strip("()Mhz ")))
            except Exception:
                pass
            time.sleep(self.period)

    def __enter__(self):
        import threading
        self._th = threading.Thread(target=self._run, daemon=True)
        self._th.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        self._th.join()

    def mean(self):
        v = self.samples[2:] if len(self.samples) > 4 else self.samples   # the first readings predate the load
        return sum(v) / len(v) if v else None


def run_gemm_trail(moe, ctx, s, cnt, packed, secs):
    """What bounds the grouped GEMM: rate and sustained shader clock of (a) an MFMA-only kernel, (b) the two
    expert GEMMs of this library on the workload's per-expert loads, (c) the vendor library's dense GEMM
    (torch.matmul, i.e. hipBLASLt) on ONE matrix of the same total size, in both operand layouts.  Every load
    loops for `secs` seconds while the clock is sampled."""
    import torch
    rows = []

    def loop(name, fn, flop, per_sync=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        with ClockSampler() as cs:
            t0 = time.perf_counter()
            n = 0
            while time.perf_counter() - t0 < secs:
                for _ in range(per_sync):
                    fn()
                torch.cuda.synchronize()
                n += per_sync
            dt = time.perf_counter() - t0
        rate = flop * n / dt / 1e12
        rows.append({"load": name, "TFLOPs": rate, "sclk_MHz": cs.mean(), "ms": dt / n * 1e3})

    # (a) MFMA only: the library's own rate kernel reports its rate; sample the clock around it
    for shape, name in ((1, "v_mfma_f32_16x16x32_bf16, the grouped GEMM's instruction"), (0, "v_mfma_f32_32x32x16_bf16")):
        with ClockSampler() as cs:
            t0 = time.perf_counter()
            rates = []
            while time.perf_counter() - t0 < secs:
                rates.append(moe.moe_measure_mfma_rate(2500, 5, shape=shape))
        rows.append({"load": f"MFMA only ({name}; no loads)", "TFLOPs": sum(rates) / len(rates),
                     "sclk_MHz": cs.mean(), "ms": None})
    # (b) this library: both expert GEMMs on the workload's loads (rows already expert-contiguous)
    local = [int(c) for c in cnt[s.e_lo:s.e_lo + s.E_local]]
    A = sum(local)
    off = torch.tensor([0] + list(__import__("itertools").accumulate(local)), dtype=torch.int32, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    xp = torch.randn(A, s.d, device="cuda", generator=g).bfloat16()
    y = torch.empty(A, s.d, dtype=torch.bfloat16, device="cuda")
    loop(f"moe_grouped_ffn, loads {local}", lambda: ctx.moe_grouped_ffn(xp, off, A, packed, y=y),
         6.0 * A * s.d * s.f)
    # (c) vendor dense GEMM of the same size: [A, d] x [d, 2f] and [A, f] x [f, d]
    Wa = (torch.randn(2 * s.f, s.d, device="cuda", generator=g) * 0.02).bfloat16()
    loop(f"torch.matmul {A}x{2 * s.f}x{s.d}, weights [2f, d] (k contiguous)", lambda: xp @ Wa.t(),
         4.0 * A * s.d * s.f)
    Wb = Wa.t().contiguous()
    loop(f"torch.matmul {A}x{2 * s.f}x{s.d}, weights [d, 2f] (n contiguous)", lambda: xp @ Wb,
         4.0 * A * s.d * s.f)
    del Wa, Wb
    h = torch.randn(A, s.f, device="cuda", generator=g).bfloat16()
    Wc = (torch.randn(s.d, s.f, device="cuda", generator=g) * 0.02).bfloat16()
    loop(f"torch.matmul {A}x{s.d}x{s.f}, weights [d, f] (k contiguous)", lambda: h @ Wc.t(), 2.0 * A * s.d * s.f)
    for r in rows:
        clk = r["sclk_MHz"]
        r["TFLOPs_per_GHz"] = r["TFLOPs"] / clk * 1e3 if clk else None
        log(f"gemm-trail: {r['load']:78s} {r['TFLOPs']:7.0f} TFLOP/s at "
            + (f"{clk:5.0f} MHz = {r['TFLOPs_per_GHz']:.0f} TFLOP/s per GHz" if clk else "(no clock reading)"))
    log(f"gemm-trail: the published peak is {PEAK_BF16_TFLOPS:.0f} TFLOP/s at 2400 MHz = "
        f"{PEAK_BF16_TFLOPS / 2.4:.0f} TFLOP/s per GHz")
    return rows


def cpu_baseline(inp, sample_tokens):
    """The oracle as it stands, on a bounded sample of the workload's tokens, on the host cores."""
    import numpy as np
    from oracle import moe_oracle as orc          # bench's cpu_baseline leg may use the oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    s = inp.shape
    n = min(sample_tokens, s.T)
    tokens = np.linspace(0, s.T - 1, n).astype(np.int64)
    t0 = time.perf_counter()
    r = orc.layer_forward(inp.x, inp.Wg, inp.bias, inp.W1, inp.W3, inp.W2, s.k, e_lo=s.e_lo, tokens=tokens)
    dt = time.perf_counter() - t0
    local = ((r["idx"][tokens] >= s.e_lo) & (r["idx"][tokens] < s.e_lo + s.E_local)).sum()
    flops = 6.0 * local * s.d * s.f + 2.0 * s.T * s.d * s.E
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle", "cpu": model,
            "sample": f"{n} of {s.T} tokens ({int(local)} expert rows) of the same workload, fp64 numpy + OpenBLAS, "
                      f"{dt:.1f} s wall"}


def roofline_bound_ms(d, f, rows_per_expert, T_in=0):
    """Lower bound of the expert FFN (plus, with T_in > 0, the layer's activation traffic) on one MI355X:
    max(useful flop / bf16 MFMA peak, algorithmic bytes / HBM peak).  Bytes: packed weights of the experts that
    have rows (6*d*f each), token rows in (2*d per row), the intermediate written and read (2 * 2*f per row),
    expert outputs (2*d per row), and for a whole layer x read and out written (2 * 2*d per token)."""
    rows = float(sum(rows_per_expert))
    touched = sum(1 for n in rows_per_expert if n > 0)
    flops = 6.0 * rows * d * f
    bytes_ = 6.0 * d * f * touched + rows * (2 * d + 4 * f + 2 * d) + 4.0 * T_in * d
    t_flop, t_byte = flops / (PEAK_BF16_TFLOPS * 1e12), bytes_ / (PEAK_HBM_GBS * 1e9)
    return max(t_flop, t_byte) * 1e3, ("mfma" if t_flop >= t_byte else "hbm")


def run_curve(moe, gu, weights_dev_packed, args):
    """Latency vs per-GPU token load: the skewed Mixtral-shaped workload (config 3), the fine-grained layer
    (config 4) and one GPU's expert-parallel share (config 5: already-routed groups and the decode-sized layer),
    every row with its roofline bound and the fraction of it that was reached."""
    import torch
    import workloads as wl
    rows = []

    def record(name, tokens, ms, n_e, d, f, T_in, extra=None):
        bound, kind = roofline_bound_ms(d, f, n_e, T_in)
        flops = 6.0 * sum(n_e) * d * f
        row = {"workload": name, "tokens": tokens, "ms": ms, "tflops": flops / ms / 1e9, "bound_ms": bound,
               "bound": kind, "frac_of_bound": bound / ms, "rows_per_expert_max": int(max(n_e)), "rows": int(sum(n_e))}
        row.update(extra or {})
        rows.append(row)
        log(f"curve {name} n={tokens}: {ms:.3f} ms  {row['tflops']:.1f} TFLOP/s  bound {bound:.3f} ms ({kind}) -> "
            f"{row['frac_of_bound']:.1%} of the roofline")

    # config 3
    loads = [int(v) for v in args.curve_loads.split(",")]
    ctx = moe.MoEContext(max(loads), wl.MIXTRAL_D, wl.MIXTRAL_F, wl.MIXTRAL_E, wl.MIXTRAL_K, flags=moe.FLAG_STAGE_EVENTS)
    for T in loads:
        inp = wl.mixtral_skewed(T, args.seed, weights=False)
        x = gu.to_dev_bf16(inp.x)
        rp = ctx.moe_pack_router(gu.to_dev(inp.Wg))
        bias = gu.to_dev(inp.bias)
        out = torch.empty(T, wl.MIXTRAL_D, dtype=torch.bfloat16, device="cuda")
        counts = torch.empty(wl.MIXTRAL_E, dtype=torch.int32, device="cuda")
        ctx.moe_layer_forward(x, rp, bias, weights_dev_packed, out=out, counts_out=counts)
        ms, stages = time_layer(ctx, x, rp, bias, weights_dev_packed, out, args.curve_steps, 3)
        record("mixtral_skewed", T, ms, counts.cpu().tolist(), wl.MIXTRAL_D, wl.MIXTRAL_F, T,
               {"tile_rows": ctx.moe_tile_rows(), "expert_counts": counts.cpu().tolist(), "stages_ms": stages})
    ctx.close()
    del weights_dev_packed
    torch.cuda.empty_cache()

    def layer_point(name, inp):
        s = inp.shape
        c = moe.MoEContext(s.T, s.d, s.f, s.E, s.k, s.e_lo, s.E_local, flags=moe.FLAG_STAGE_EVENTS)
        x = gu.to_dev_bf16(inp.x)
        rp = c.moe_pack_router(gu.to_dev(inp.Wg))
        bias = gu.to_dev(inp.bias) if inp.bias is not None else None
        packed = c.moe_pack_weights(gu.to_dev_bf16(inp.W1), gu.to_dev_bf16(inp.W3), gu.to_dev_bf16(inp.W2))
        out = torch.empty(s.T, s.d, dtype=torch.bfloat16, device="cuda")
        counts = torch.empty(s.E, dtype=torch.int32, device="cuda")
        c.moe_layer_forward(x, rp, bias, packed, out=out, counts_out=counts)
        ms, stages = time_layer(c, x, rp, bias, packed, out, args.curve_steps, 3)
        n_e = counts.cpu().tolist()[s.e_lo:s.e_lo + s.E_local]
        record(name, s.T, ms, n_e, s.d, s.f, s.T, {"tile_rows": c.moe_tile_rows(), "stages_ms": stages})
        c.close()
        return packed

    # config 4
    layer_point("fine_grained", wl.fine_grained(8192, args.seed))
    torch.cuda.empty_cache()
    # config 5: the decode-sized layer, then the already-routed groups on the same packed weights
    ep_w = wl.expert_weights(args.seed, wl.EP_ELOCAL, wl.EP_D, wl.EP_F)
    packed = layer_point("ep_share_layer", wl.ep_share_layer(128, args.seed, weights=ep_w))
    for N in (256, 1024, 4096, 16384):
        xp_bits, off = wl.ep_share_groups(N, args.seed)
        c = moe.MoEContext(N, wl.EP_D, wl.EP_F, wl.EP_ELOCAL, 1)
        xp, offd = gu.to_dev_bf16(xp_bits), gu.to_dev(off)
        y = torch.empty((N, wl.EP_D), dtype=torch.bfloat16, device="cuda")
        ms = time_calls(lambda: c.moe_grouped_ffn(xp, offd, N, packed, y=y), args.curve_steps)
        record("ep_share_groups", N, ms, np_diff(off), wl.EP_D, wl.EP_F, 0, {"tile_rows": c.moe_tile_rows()})
        c.close()
    os.makedirs(os.path.join(ROOT, args.out_dir), exist_ok=True)
    with open(os.path.join(ROOT, args.out_dir, "latency_curve.json"), "w") as fh:
        json.dump({"rows": rows}, fh, indent=1)


def np_diff(off):
    return [int(off[i + 1] - off[i]) for i in range(len(off) - 1)]


def run_profile_curve(moe, s, packed, args):
    """Token-vs-latency curve of the isolated expert kernels, sampled at the tile boundaries
    (paper Sec. 3.3.2, Step-2) -> cg_curve.json in the output folder."""
    import torch
    from paper_2605_19945_amd import latency_curve as lc
    boundary = s.E_local * 32            # row tiles grow in steps of 32 rows per expert
    dense_max = s.E_local * 2048         # every boundary up to 2K tokens per expert
    n_max, sparse_step = 4 * dense_max, dense_max // 2
    after = s.E_local                    # n = m*boundary + E_local: every expert has crossed its boundary
    counts = lc.sample_counts(boundary, dense_max, n_max, sparse_step, after)
    ctx = moe.MoEContext(n_max, s.d, s.f, s.E_local, 1)
    g = torch.Generator(device="cuda")
    g.manual_seed(args.seed)
    xp = torch.randn(n_max, s.d, device="cuda", generator=g).bfloat16()
    t0 = time.perf_counter()
    ms = ctx.moe_profile_ffn(xp, packed, counts, warmup=2, iters=args.profile_iters)
    wall = time.perf_counter() - t0
    curve = lc.LatencyCurve(counts, ms)
    dense_end = min(dense_max, n_max) // boundary * boundary
    jumps = [(c, ms[i], ms[i + 1]) for i, c in enumerate(counts[:-1]) if c % boundary == 0 and counts[i + 1] == c + after]
    flat = [ms[i + 1] / ms[i] - 1.0 for i, c in enumerate(counts[:-1]) if c % boundary == after and c > after and counts[i + 1] == c - after + boundary]
    tile = s.E_local * ctx.moe_tile_rows()   # tokens per GPU at which every expert gets one more row tile
    big = [b / a - 1.0 for c, a, b in jumps if c % tile == 0]
    rel = [b / a - 1.0 for c, a, b in jumps if c % tile != 0]
    cost, sweep = curve.profiling_cost_ms(args.profile_iters), curve.full_sweep_cost_ms(args.profile_iters)
    log(f"profile: {len(counts)} token counts x {args.profile_iters} launches in {wall:.1f} s wall; "
        f"kernel time {cost / 1e3:.2f} s vs {sweep / 1e3:.0f} s for a sweep of every count 1..{n_max} ({sweep / cost:.0f}x)")
    log(f"profile: latency jump when a row-tile boundary is crossed (n = m*{tile} -> +{after}): "
        + ", ".join(f"{100 * v:.1f} %" for v in big))
    log(f"profile: latency jump when a 32-row boundary is crossed (n = m*{boundary} -> +{after}): median {100 * sorted(rel)[len(rel) // 2]:.1f} %; "
        f"change across the rest of a step (m*{boundary}+{after} -> (m+1)*{boundary}): median {100 * sorted(flat)[len(flat) // 2]:.1f} %")
    for n in (1, boundary, boundary + after, 1024, 4096, 8192, dense_max, n_max):
        log(f"   C_g({n}) = {curve.at(n):.3f} ms")
    os.makedirs(os.path.join(ROOT, args.out_dir), exist_ok=True)
    with open(os.path.join(ROOT, args.out_dir, "cg_curve.json"), "w") as fh:
        json.dump({"boundary": boundary, "after": after, "dense_end": dense_end, "iters": args.profile_iters,
                   "counts": counts, "ms": ms, "profiling_kernel_ms": cost, "full_sweep_kernel_ms": sweep}, fh)
    ctx.close()


def run_gem_demo(moe, gu, s, packed, args):
    """The paper's pipeline end to end on one GPU: Step-2 profile of the expert kernels at E/G experts
    per GPU, Step-1 trace of S router steps, Step-3 mapping search.  GPU-to-GPU variability is emulated
    as in the paper's sensitivity study (Sec. 5): G copies of the measured curve, the last one 12 % slower."""
    import numpy as np
    import torch
    import workloads as wl
    from paper_2605_19945_amd import latency_curve as lc, trace as tr
    G, S, T = 4, 16, 2048
    per_gpu = s.E // G
    # Step-2: curve of one GPU holding per_gpu experts
    ctx = moe.MoEContext(S * 0 + 4 * T * s.k, s.d, s.f, per_gpu, 1)
    n_max = ctx.rows_capacity(4 * T * s.k)
    counts = lc.sample_counts(per_gpu * 32, min(n_max, per_gpu * 2048), n_max, 2048, per_gpu)
    xp = torch.randn(n_max, s.d, device="cuda").bfloat16()
    sub = packed[: ctx.lib.moe_packed_weight_bytes(__import__("ctypes").byref(ctx.shape)) // 2]
    ms = ctx.moe_profile_ffn(xp, sub, counts, warmup=2, iters=args.profile_iters)
    ctx.close()
    curves = [(counts, [m * (1.12 if g == G - 1 else 1.0) for m in ms]) for g in range(G)]
    # Step-1: trace of S steps through the router on the GPU
    steps, active = wl.trace_steps(S, T, args.seed, d=s.d, E=s.E, k=s.k)
    rctx = moe.MoEContext(T, s.d, 64, s.E, s.k)
    rp = rctx.moe_pack_router(gu.to_dev(steps[0].Wg))
    bias = gu.to_dev(steps[0].bias)
    trace_dev = torch.zeros(S, s.E, dtype=torch.int32, device="cuda")
    for t, inp in enumerate(steps):
        rctx.moe_route(gu.to_dev_bf16(inp.x), rp, bias, counts=trace_dev[t])
    torch.cuda.synchronize()
    trace = trace_dev.cpu().numpy()
    rctx.close()
    # Step-3: mapping search (30 restarts, noise drawn here and handed in)
    K = 30
    noise = np.random.default_rng(args.seed).uniform(-1.0, 1.0, (K, s.E)).astype(np.float32)
    t0 = time.perf_counter()
    M, score, swaps = moe.moe_gem_place(trace, curves, noise, K)
    dt = time.perf_counter() - t0
    linear = [e // per_gpu for e in range(s.E)]
    s_lin = moe.moe_gem_score(trace, curves, linear)
    a, b = wl.TRACE_PAIR
    log(f"gem-demo: {S}-step trace, mean utilisation {tr.mean_utilisation(trace).round(0).tolist()}, "
        f"pair {wl.TRACE_PAIR} r = {tr.pearson(trace, a, b):.2f}, active steps {[t for t in range(S) if active[t]]}")
    log(f"gem-demo: C_g sampled at {len(counts)} counts; GPU {G - 1} emulated 12 % slower")
    log(f"gem-demo: linear mapping {linear} score {s_lin:.3f} ms; searched mapping {M.tolist()} score {score:.3f} ms "
        f"({100 * (1 - score / s_lin):.1f} % lower predicted straggler latency; {swaps} swaps; search {dt * 1e3:.1f} ms)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mixtral_T4096")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--tile-class", type=int, default=-1)
    ap.add_argument("--cpu-sample-tokens", type=int, default=2048)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--out-dir", default=OUT_DIR_DEFAULT, help="folder (under the repo root) for the curve JSON files")
    ap.add_argument("--graph", action="store_true",
                    help="also time the layer call captured into a HIP graph and replayed")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the measurement of the bf16 MFMA rate the device sustains under an MFMA-only load")
    ap.add_argument("--no-hbm-stages", action="store_true",
                    help="skip the separate measurement of the memory-bound stages (route, permute, combine)")
    ap.add_argument("--hbm-stage-tokens", default="4096,65536")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (reference for HBM byte counters)")
    ap.add_argument("--profile-curve", action="store_true",
                    help="also run the tile-boundary latency profiler (C_g(n) of the isolated expert kernels)")
    ap.add_argument("--profile-iters", type=int, default=10)
    ap.add_argument("--gem-demo", action="store_true",
                    help="profile -> trace -> mapping search on emulated GPU variability (paper Steps 1-3)")
    ap.add_argument("--gemm-trail", action="store_true",
                    help="rate and sustained shader clock of an MFMA-only load, of this library's expert GEMMs and "
                         "of the vendor library's dense GEMM of the same size (what bounds the grouped GEMM)")
    ap.add_argument("--trail-secs", type=float, default=4.0)
    ap.add_argument("--curve", action="store_true")
    ap.add_argument("--curve-loads", default="512,1024,2048,4096,8192")
    ap.add_argument("--curve-steps", type=int, default=20)
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU's expert layer: this build has no multi-GPU path; "
                         "run with --gpus 1")
    if args.steps > 64:
        raise SystemExit("--steps is limited to 64 (the per-stage event ring holds 64 calls)")

    import torch
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (the HIP path has no CPU fallback)")
    import paper_2605_19945_amd as moe
    from paper_2605_19945_amd import tensors as gu
    moe.load_library()

    t0 = time.perf_counter()
    inp = make_workload(args.workload, args.seed, None)
    s = inp.shape
    log(f"workload {inp.name}: T={s.T} d={s.d} f={s.f} E={s.E} k={s.k} local=[{s.e_lo},{s.e_lo + s.E_local}) "
        f"generated in {time.perf_counter() - t0:.1f} s")

    ctx = moe.MoEContext(s.T, s.d, s.f, s.E, s.k, s.e_lo, s.E_local, flags=moe.FLAG_STAGE_EVENTS)
    ctx.moe_set_tile_class(args.tile_class)
    x = gu.to_dev_bf16(inp.x)
    rp = ctx.moe_pack_router(gu.to_dev(inp.Wg))
    bias = gu.to_dev(inp.bias) if inp.bias is not None else None
    W1, W3, W2 = gu.to_dev_bf16(inp.W1), gu.to_dev_bf16(inp.W3), gu.to_dev_bf16(inp.W2)
    packed = ctx.moe_pack_weights(W1, W3, W2)
    torch.cuda.synchronize()
    del W1, W3, W2
    torch.cuda.empty_cache()
    out = torch.empty(s.T, s.d, dtype=torch.bfloat16, device="cuda")
    counts = torch.empty(s.E, dtype=torch.int32, device="cuda")
    ctx.moe_layer_forward(x, rp, bias, packed, out=out, counts_out=counts)
    torch.cuda.synchronize()
    cnt = counts.cpu().numpy()
    A_local = int(cnt[s.e_lo:s.e_lo + s.E_local].sum())

    ms, stages = time_layer(ctx, x, rp, bias, packed, out, args.steps, args.warmup)
    flops_ffn = 6.0 * A_local * s.d * s.f
    flops = flops_ffn + 2.0 * s.T * s.d * s.E
    tflops = flops / ms / 1e9
    g1 = 4.0 * A_local * s.d * s.f / stages["gemm1"] / 1e9
    g2 = 2.0 * A_local * s.d * s.f / stages["gemm2"] / 1e9
    route_gbs = (s.T * s.d * 2 + s.T * s.k * 8) / stages["route"] / 1e6
    combine_gbs = ((A_local + s.T) * s.d * 2 + A_local * 8) / stages["combine"] / 1e6
    log(f"layer {ms:.3f} ms/step -> {tflops:.1f} TFLOP/s; stages (ms): "
        + ", ".join(f"{k}={v:.4f}" for k, v in stages.items()))
    log(f"gemm1 {g1:.1f} TFLOP/s ({g1 / PEAK_BF16_TFLOPS:.1%} of bf16 peak), gemm2 {g2:.1f} TFLOP/s "
        f"({g2 / PEAK_BF16_TFLOPS:.1%}); route {route_gbs:.0f} GB/s, combine {combine_gbs:.0f} GB/s "
        f"(stage intervals include launch gaps); tile rows {ctx.moe_tile_rows()}; counts {cnt.tolist()}")

    # the dominant kernel (GEMM1) against the roofline that bounds it at this load: MFMA, or HBM when the
    # launch mostly streams the weights of the loaded experts (bytes: W1|W3 of every expert with rows, the
    # token rows in, the activated rows out)
    loaded = int((cnt[s.e_lo:s.e_lo + s.E_local] > 0).sum())
    g1_bytes = loaded * 2.0 * s.f * s.d * 2 + A_local * s.d * 2.0 + A_local * s.f * 2.0
    g1_hbm_gbs = g1_bytes / stages["gemm1"] / 1e6
    g1_flop = 4.0 * A_local * s.d * s.f
    hbm_bound = g1_bytes / (PEAK_HBM_GBS * 1e9) > g1_flop / (PEAK_BF16_TFLOPS * 1e12)
    if hbm_bound:
        log(f"gemm1 is bound by weight streaming at this load: {g1_bytes / 1e9:.3f} GB in {stages['gemm1'] * 1e3:.0f} us = "
            f"{g1_hbm_gbs:.0f} GB/s ({g1_hbm_gbs / PEAK_HBM_GBS:.1%} of HBM peak)")
    result = {
        "metric": "MoE layer TFLOP/s + latency vs per-GPU token load (Mixtral-8x7B shape, 1 GPU)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": inp.name, "T": s.T, "d": s.d, "f": s.f, "E": s.E, "k": s.k,
                   "E_local": s.E_local, "local_assignments": A_local, "tile_rows": ctx.moe_tile_rows(),
                   "stages_ms": stages},
        "roofline": {"bound": "hbm" if hbm_bound else "mfma", "kernel": "grouped_gemm_kernel<SwiGLU> (GEMM1)",
                     "achieved": g1_hbm_gbs if hbm_bound else g1,
                     "peak": PEAK_HBM_GBS if hbm_bound else PEAK_BF16_TFLOPS,
                     "unit": "GB/s" if hbm_bound else "TFLOP/s",
                     "frac": g1_hbm_gbs / PEAK_HBM_GBS if hbm_bound else g1 / PEAK_BF16_TFLOPS,
                     "mfma_frac": g1 / PEAK_BF16_TFLOPS, "hbm_frac": g1_hbm_gbs / PEAK_HBM_GBS,
                     "traffic": profiled_traffic(inp.name, "gemm1") if args.tile_class < 0 else None,
                     "traffic_source": "committed rocprofv3 --pmc summary of this command (profiles/), not this run",
                     "gemm2": {"achieved": g2, "frac": g2 / PEAK_BF16_TFLOPS}},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(inp, args.cpu_sample_tokens)
    if args.graph:
        gms = time_layer_graph(moe, s, x, rp, bias, packed, out, args.steps, args.warmup)
        log(f"graph replay {gms:.3f} ms/step ({100 * (gms / ms - 1):+.1f} % against the eager calls)")
        result["graph_replay_ms_per_step"] = gms
    if not args.no_hbm_stages:
        # route / permute / combine against the HBM roofline, at the workload's token count and at a large one
        stages_hbm = []
        for T in [int(v) for v in args.hbm_stage_tokens.split(",")]:
            r = hbm_stages(moe, s, T, args.seed)
            stages_hbm.append(r)
            log(f"memory-bound stages at T={T}: " + ", ".join(
                f"{k} {v['us']:.1f} us {v['GBps']:.0f} GB/s ({v['frac']:.0%} of HBM peak)" for k, v in r.items()))
        result["roofline"]["hbm_stages"] = stages_hbm
    if not args.no_mfma_ceiling:
        # context for roofline.frac, not a replacement of the published peak it is computed against
        sustained = moe.moe_measure_mfma_rate(2500, 5)
        log(f"sustained MFMA-only rate: {sustained:.0f} TFLOP/s = {100 * sustained / PEAK_BF16_TFLOPS:.1f} % of the "
            f"{PEAK_BF16_TFLOPS:.0f} TFLOP/s peak; GEMM1 reaches {100 * g1 / sustained:.1f} % of it")
        result["roofline"]["sustained_mfma_only"] = sustained
        # the same for HBM: what a read-only streaming kernel reaches over the expert weights
        hbm = {"bytes": packed.numel() * packed.element_size(),
               "plain_GBps": moe.moe_measure_hbm_read_rate(packed, nontemporal=False),
               "nontemporal_GBps": moe.moe_measure_hbm_read_rate(packed, nontemporal=True)}
        log(f"sustained read-only streaming over the {hbm['bytes'] / 1e9:.2f} GB of expert weights: "
            f"{hbm['plain_GBps']:.0f} GB/s with plain loads, {hbm['nontemporal_GBps']:.0f} GB/s with the "
            f"non-temporal hint ({100 * hbm['nontemporal_GBps'] / PEAK_HBM_GBS:.0f} % of the {PEAK_HBM_GBS:.0f} GB/s peak)")
        result["roofline"]["sustained_hbm_read"] = hbm
    if args.gemm_trail:
        result["roofline"]["gemm_trail"] = run_gemm_trail(moe, ctx, s, cnt, packed, args.trail_secs)
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.curve:
        run_curve(moe, gu, packed, args)
    if args.profile_curve:
        run_profile_curve(moe, s, packed, args)
    if args.gem_demo:
        run_gem_demo(moe, gu, s, packed, args)
    ctx.close()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
