#!/usr/bin/env python3
"""Benchmark of the LoRAct hot path on one MI355X.

One "step" = one pass of the whole hot path over one activation site resident in HBM:
loract_compress (sample, sketch, orthonormalise, project) + loract_reconstruct +
loract_lora_grad, on the LLaMA-7B-shaped pre-norm activation (8192 x 4096 bf16, rank 128,
LoRA rank 16, dY 8192 x 4096).  Inputs are seeded synthetic stand-ins (workloads/synth.py).

Prints ONE JSON line: metric/value = activation GB/s through compress + reconstruct (+ the LoRA
gradient, which is inside the step), plus
  roofline     the dominant kernel's algorithmic HBM bytes per launch / its mean duration,
               measured with HIP events on the library's stream inside this run;
  cpu_baseline the fp64 numpy oracle timed on this machine's host cores on the same workload.
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

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
FP64_VECTOR_PEAK_TFLOPS = 78.6   # MI355X published fp64 vector rate
BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix rate


def algorithmic_cost(name: str, m: int, n: int, k: int, b: int, n_out: int, r: int, launches: float):
    """(bound, amount per launch, unit) for a kernel name: algorithmic HBM bytes for the
    streaming kernels, flops for the float64 small-matrix kernels.  `launches` = launches of
    that name per step (a name used by two different calls gets the mean of their amounts)."""
    fb = b                                      # factor bytes per element (= input dtype here)
    kp = (k + 15) // 16 * 16
    rp = (r + 15) // 16 * 16
    hbm = {
        # reads X once and the k sampled rows, writes Y (fp32, possibly as split partials)
        "sketch": m * n * b + k * n * b + m * kp * 4,
        # reads X once and U, writes V
        "project": m * n * b + m * k * fb + k * n * fb,
        # writes Xhat, reads U and V
        "reconstruct": m * n * b + (m + n) * k * fb,
        # reads dY once and B_lora, writes G
        "lora_dyb": m * n_out * b + r * n_out * b + m * rp * 4,
        # reads U and the split G, writes T
        "lora_utg": m * k * fb + m * 2 * rp * 2 + k * 2 * rp * 4,
        "lora_vtt": k * n * fb + n * r * 4,
        # Newton-Schulz finish, one kernel: U = Q1 + Q1b T (reads the bf16 copy of Q1, T and the
        # fp32 Q1, writes U); the separate finalize kernel only runs for ranks not a multiple of 64
        "ns_correct": m * kp * 2 + kp * kp * 2 + m * kp * 4 + m * k * fb,
        "ns_finalize": m * kp * 4 + m * k * fb,
    }
    if name in hbm:
        return "hbm", float(hbm[name]), "GB/s"
    flops = {
        # the lower 64 x 64 blocks of the kp x kp matrix, diagonal included
        "gram": 2.0 * m * 4096.0 * (((kp + 63) // 64) * ((kp + 63) // 64 + 1) // 2),
        "trsm_apply": 1.0 * m * kp * kp + 2.0 * m * kp * 16,
        "chol": kp ** 3 / 3.0,
        # factorisation and triangular solve of a round in one launch (round 2 usually ends at once:
        # the mean over its two launches per step is what `launches` divides)
        "chol_trsm": (kp ** 3 / 3.0 + 1.0 * m * kp * kp + 2.0 * m * kp * 16) / max(launches, 1.0),
        # degree-4 finish of round 2: E^2, then E^3 and E^4 (float64 products of kp x kp matrices)
        "ns_poly_square": 2.0 * kp ** 3,
        "ns_poly_finish": 4.0 * kp ** 3,
    }
    if name in flops:
        return "alu", flops[name], "TFLOP/s"
    return "hbm", 0.0, "GB/s"


def c5_stream(args, L, torch, np) -> int:
    """Config 5: long-context stream, 16 x 4096 tokens per site, 7 sites per decoder layer (six
    4096-wide, one 11008-wide), rank 256.  Sites are generated on the GPU on one HIP stream
    (harness code: X = c (G1 diag(s)) G2^T + 1e-3 N with Gaussian G1, G2 scaled to near-orthonormal
    columns, 1024 spectrum terms, s_i = i^-1.5, per-site seed) while the previous site is compressed
    on another stream; two X buffers alternate.  Factors of every site are kept, as in training."""
    from workloads import gpu_sites
    m, k = gpu_sites.C5_ROWS, gpu_sites.C5_RANK
    widths = list(gpu_sites.C5_WIDTHS)
    sites = [(layer, s) for layer in range(args.layers) for s in range(7)]
    gen_stream, cmp_stream = torch.cuda.Stream(), torch.cuda.Stream()
    xbuf = [torch.empty((m, 11008), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    factors, errs = [], []
    gen_done = [torch.cuda.Event() for _ in sites]
    cmp_done = [torch.cuda.Event() for _ in sites]

    def generate(i):
        layer, s = sites[i]
        n = widths[s]
        x = xbuf[i % 2].view(-1)[: m * n].view(m, n)
        return gpu_sites.c5_site_on_gpu(torch, layer, s, out=x)

    def run(check):
        factors.clear()
        errs.clear()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        views = [None, None]
        for i in range(len(sites) + 1):
            if i < len(sites):
                with torch.cuda.stream(gen_stream):
                    if i >= 2:
                        gen_stream.wait_event(cmp_done[i - 2])      # buffer i % 2 is free again
                    views[i % 2] = generate(i)
                    gen_done[i].record(gen_stream)
            j = i - 1
            if j >= 0:
                with torch.cuda.stream(cmp_stream):
                    cmp_stream.wait_event(gen_done[j])
                    x = views[j % 2]
                    u, v = L.loract_compress(x, k, seed=50_000 + j)
                    if check:
                        xh = L.loract_reconstruct(u, v)
                        errs.append(torch.linalg.norm(xh.float() - x.float()) / torch.linalg.norm(x.float()))
                        del xh
                    cmp_done[j].record(cmp_stream)
                    factors.append((u, v))
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    run(False)                                    # warm-up (allocations, first-use set-up)
    seconds = run(False)
    run(True)
    total_bytes = sum(m * widths[s] * 2 for _, s in sites)
    # compress-only time of the same sites, back to back on one stream, inputs resident
    x4096 = xbuf[0].view(-1)[: m * 4096].view(m, 4096)
    x11008 = xbuf[1].view(-1)[: m * 11008].view(m, 11008)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _, s in sites:
        L.loract_compress(x11008 if s == 6 else x4096, k, seed=1)
    torch.cuda.synchronize()
    compress_only = time.perf_counter() - t0
    out = {
        "metric": "activation GB/s compressed (long-context stream, generation overlapped)",
        "value": round(total_bytes / seconds / 1e9, 2), "unit": "GB/s", "n_gpus": 1,
        "steps": len(sites), "warmup": len(sites), "ms_per_step": round(seconds * 1e3 / len(sites), 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "c5stream: %d layers x 7 sites of 65536 x {4096 x6, 11008 x1} bf16, rank 256, "
                               "two HIP streams (generate || compress), double-buffered X" % args.layers},
        "layers": args.layers, "sites": len(sites),
        "full_configuration": bool(args.layers == 32),
        "compress_only_gbps": round(total_bytes / compress_only / 1e9, 2),
        # two passes over X, the sampled rows, Y out and in, the factors: the algorithmic bytes of a
        # compress as Algorithm 1 is written, against the 8 TB/s of the part
        "compress_only_hbm_frac_two_pass": round(
            sum(2 * m * widths[s] * 2 + k * widths[s] * 2 + 2 * m * k * 4 + (m + widths[s]) * k * 2
                for _, s in sites) / compress_only / 1e9 / HBM_PEAK_GBS, 4),
        "compress_only_ms_per_site": round(compress_only * 1e3 / len(sites), 3),
        "rel_fro_err_min_max": [round(float(min(errs)), 5), round(float(max(errs)), 5)],
        "factor_bytes_kept": int(sum(u.numel() * 2 + v.numel() * 2 for u, v in factors)),
    }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2a", "c2b", "c3", "c4", "c5", "coherent", "c5stream"])
    ap.add_argument("--layers", type=int, default=32,
                    help="c5stream only: decoder layers to stream (7 sites each; the configuration is 32 layers, "
                         "fewer is a subsample of it and is labelled so)")
    ap.add_argument("--streams", type=int, default=3,
                    help="independent sites in flight for the `pipelined` figure (hardware queues per process: 4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-comparator", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run 5 plain device copies of X (2*|X| bytes of known traffic each) so "
                         "that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
    ap.add_argument("--profile-pass", action="store_true",
                    help="run only warm single-stream steps (no cold-cache flush, no pipelined section, no "
                         "comparator, no event profiling) and print a short JSON line: the run to put under "
                         "rocprofv3 --kernel-trace / --pmc, so that every kernel average is one role's warm figure")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "traffic.json"))
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (each GPU compresses "
              "its own micro-batch independently); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2509_23472_amd as L
    from workloads import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    if args.workload == "c5stream":
        return c5_stream(args, L, torch, np)
    if args.workload == "c3":
        w = synth.c3_llama()
    else:
        w = synth.FULL_SIZE[args.workload]()
    m, n, k = w.m, w.n, w.k
    # config 1 is float32 (float64 accumulation on the device); the others are bf16
    is_f32 = w.dtype == "f32"
    b = 4 if is_f32 else 2
    dt = torch.float32 if is_f32 else torch.bfloat16
    dt_name = "f32" if is_f32 else "bf16"
    rng = np.random.default_rng(123)
    dy_h = w.extras.get("dY")
    bl_h = w.extras.get("B_lora")
    if dy_h is None:       # the LoRA operands are part of every step; other sites reuse the recipe
        r_l = 16
        dy_h = synth.round_to_bf16(rng.standard_normal((m, n)).astype(np.float32))
        bl_h = synth.round_to_bf16((rng.standard_normal((r_l, n)) / 4.0).astype(np.float32))
    r_l, n_out = bl_h.shape[0], dy_h.shape[1]

    def up(a):
        if is_f32:
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        return torch.from_numpy(synth.f32_to_bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)

    x, dy, bl = up(w.x), up(dy_h), up(bl_h)
    u = torch.empty((m, k), dtype=dt, device="cuda")
    v = torch.empty((k, n), dtype=dt, device="cuda")
    xhat = torch.empty((m, n), dtype=dt, device="cuda")
    ga = torch.empty((n, r_l), dtype=torch.float32, device="cuda")

    def compress():
        L.loract_compress(x, k, seed=w.seed, out=(u, v))

    def reconstruct():
        L.loract_reconstruct(u, v, out=xhat)

    def lora():
        L.loract_lora_grad(u, v, dy, bl, scale=1.0, out=ga)

    def step():
        compress()
        reconstruct()
        lora()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    x_bytes = m * n * b

    if args.profile_pass:
        if args.pmc_calibration:
            scratch = torch.empty_like(x)
            for _ in range(5):
                scratch.copy_(x)
            torch.cuda.synchronize()
        print(json.dumps({"profile_pass": True, "workload": args.workload, "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
                          "launch_order": "compress, reconstruct, lora_grad per step, one stream"}))
        return 0

    # per-phase times (separate region, events on the stream the library launches on)
    def timed(fn):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / args.steps     # microseconds

    us_c, us_r, us_l = timed(compress), timed(reconstruct), timed(lora)

    # cold-cache figures: X (and dY) fit in the 256 MB memory-side cache for the single-site
    # configurations, so a back-to-back loop re-reads them from there.  Here a 512 MB fill between
    # calls pushes them out, which is what a training step does between the forward and backward
    # use of a site.
    flush = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")

    def timed_cold(fn, reps):
        tot = 0.0
        for _ in range(reps):
            flush.fill_(1)
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            tot += e0.elapsed_time(e1)
        return tot * 1e3 / reps

    cold_reps = max(5, args.steps // 5)
    us_c_cold, us_r_cold, us_l_cold = (timed_cold(compress, cold_reps), timed_cold(reconstruct, cold_reps),
                                       timed_cold(lora, cold_reps))
    del flush

    # per-kernel times: HIP events recorded by the library around each of its launches
    L.loract_profile_begin()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = L.loract_profile_end()
    kernels = {}
    for name, (ms, cnt) in prof.items():
        bound, amount, unit = algorithmic_cost(name, m, n, k, b, n_out, r_l, cnt / args.steps)
        avg_us = ms * 1e3 / cnt
        kernels[name] = {"avg_us": round(avg_us, 2), "launches_per_step": cnt / args.steps,
                         "share": 0.0, "bound": bound,
                         "achieved": round(amount / (avg_us * 1e-6) / (1e9 if unit == "GB/s" else 1e12), 2)
                         if amount else None, "unit": unit}
    total_ms = sum(ms for ms, _ in prof.values())
    for name, (ms, cnt) in prof.items():
        kernels[name]["share"] = round(ms / total_ms, 3)
    # matrix-core utilisation of the three dense contractions (2 m n k flops each) against the
    # published dense bf16 peak
    for name in ("sketch", "project", "reconstruct"):
        if name in kernels:
            tf = 2.0 * m * n * k / (kernels[name]["avg_us"] * 1e-6) / 1e12
            kernels[name]["mfma_tflops"] = round(tf, 1)
            kernels[name]["mfma_frac"] = round(tf / BF16_MFMA_PEAK_TFLOPS, 4)
    dom = max(prof.items(), key=lambda kv: kv[1][0])[0]
    d_bound, d_amount, d_unit = algorithmic_cost(dom, m, n, k, b, n_out, r_l, prof[dom][1] / args.steps)
    d_avg_s = prof[dom][0] * 1e-3 / prof[dom][1]
    if d_unit == "GB/s":
        achieved, peak = d_amount / d_avg_s / 1e9, HBM_PEAK_GBS
    else:
        achieved, peak = d_amount / d_avg_s / 1e12, FP64_VECTOR_PEAK_TFLOPS
    # HBM bytes per launch from the committed rocprofv3 --pmc summary, only if that summary was taken
    # from this very build of the library (same source hash); otherwise null
    traffic, traffic_of = None, {}
    if os.path.exists(args.traffic_json):
        try:
            from paper_2509_23472_amd.build import source_hash
            tj = json.load(open(args.traffic_json))
            if tj.get("source_hash") == source_hash():
                traffic_of = tj.get(args.workload, {})
                traffic = traffic_of.get(dom)
        except Exception:
            traffic, traffic_of = None, {}
    roofline = {"kernel": dom, "bound": d_bound, "achieved": round(achieved, 2), "peak": peak,
                "unit": d_unit, "frac": round(achieved / peak, 4), "traffic": traffic,
                "avg_us": round(d_avg_s * 1e6, 2), "algorithmic_per_launch": d_amount}
    if dom in ("chol_trsm", "chol"):
        # a chain of k dependent pivots on one CU (the triangular solve runs beside it in the same
        # launch): priced against the float64 vector peak only because the line wants a number
        roofline["note"] = ("latency-bound: k sequential pivots on one CU, solve hidden behind them; "
                            "roofline_streaming is the bandwidth-bound figure")

    # the slowest HBM-streaming kernel as well (the dominant kernel may be a latency-bound one)
    streaming = {kn: kv for kn, kv in kernels.items() if kv["bound"] == "hbm" and kv["achieved"]}
    roofline_streaming = None
    if streaming:
        sn = max(streaming, key=lambda kn: prof[kn][0])
        s_bound, s_amount, _ = algorithmic_cost(sn, m, n, k, b, n_out, r_l, prof[sn][1] / args.steps)
        s_avg = prof[sn][0] * 1e-3 / prof[sn][1]
        roofline_streaming = {"kernel": sn, "bound": "hbm", "achieved": round(s_amount / s_avg / 1e9, 2),
                              "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": round(s_amount / s_avg / 1e9 / HBM_PEAK_GBS, 4),
                              "traffic": traffic_of.get(sn),
                              "avg_us": round(s_avg * 1e6, 2), "algorithmic_per_launch": s_amount}

    # several independent sites in flight on separate HIP streams (as the sites of a layer are in
    # training): the latency-bound single-workgroup kernels of one site overlap the streaming
    # kernels of the others
    pipelined = None
    if not args.no_comparator:
        nstreams = args.streams
        streams = [torch.cuda.Stream() for _ in range(nstreams)]
        held = []
        for _ in range(nstreams):
            held.append((x.clone(), torch.empty_like(u), torch.empty_like(v), torch.empty_like(xhat),
                         torch.empty_like(ga)))

        def round_of_sites():
            for st, (xs, us, vs, xh, gs) in zip(streams, held):
                with torch.cuda.stream(st):
                    L.loract_compress(xs, k, seed=w.seed, out=(us, vs))
                    L.loract_reconstruct(us, vs, out=xh)
                    L.loract_lora_grad(us, vs, dy, bl, scale=1.0, out=gs)

        for _ in range(3):
            round_of_sites()
        torch.cuda.synchronize()
        tp0 = time.perf_counter()
        for _ in range(args.steps):
            round_of_sites()
        torch.cuda.synchronize()
        us_site = (time.perf_counter() - tp0) * 1e6 / (args.steps * nstreams)
        same = all(torch.equal(h[1], u) and torch.equal(h[3], xhat) for h in held)
        pipelined = {"streams": nstreams, "us_per_site": round(us_site, 1),
                     "gbps": round(x_bytes / us_site / 1e3, 1), "bit_identical_to_single_stream": bool(same)}

    # The same sites as HIP graphs: one captured site (compress + reconstruct + lora_grad) per stream,
    # replayed round after round.  A graph launch costs the host one call per site instead of ~25,
    # which removes the host's launch rate from the figure above.  Every replay is checked against
    # the eager result (the library records kernels only: no copies, no memsets, ids in the kernel
    # arguments), with eager work and synchronisations between replays.
    pipelined_graph = None
    if not args.no_comparator and not is_f32:
        nstreams = min(args.streams, 4)
        streams = [torch.cuda.Stream() for _ in range(nstreams)]
        gheld, graphs = [], []
        for st in streams:
            bufs = (x.clone(), torch.empty_like(u), torch.empty_like(v), torch.empty_like(xhat),
                    torch.empty_like(ga))
            gheld.append(bufs)

            def site(bufs=bufs):
                xs, us, vs, xh, gs = bufs
                L.loract_compress(xs, k, seed=w.seed, out=(us, vs))
                L.loract_reconstruct(us, vs, out=xh)
                L.loract_lora_grad(us, vs, dy, bl, scale=1.0, out=gs)

            with torch.cuda.stream(st):
                site()                      # workspaces and first-use set-up happen outside the capture
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=st):
                site()
            graphs.append(g)
        torch.cuda.synchronize()

        def replay_round():
            for st, g in zip(streams, graphs):
                with torch.cuda.stream(st):
                    g.replay()

        identical = True
        for rep in range(3):
            for bufs in gheld:
                bufs[1].zero_(); bufs[2].zero_(); bufs[3].zero_(); bufs[4].zero_()
            step()                          # eager work between the replays
            torch.cuda.synchronize()
            replay_round()
            torch.cuda.synchronize()
            identical = identical and all(torch.equal(h[1], u) and torch.equal(h[2], v) and
                                          torch.equal(h[3], xhat) and torch.equal(h[4], ga) for h in gheld)
        tg0 = time.perf_counter()
        for _ in range(args.steps):
            replay_round()
        torch.cuda.synchronize()
        us_site_g = (time.perf_counter() - tg0) * 1e6 / (args.steps * nstreams)
        pipelined_graph = {"streams": nstreams, "us_per_site": round(us_site_g, 1),
                           "gbps": round(x_bytes / us_site_g / 1e3, 1),
                           "site": "compress + reconstruct + lora_grad captured as one HIP graph per stream",
                           "bit_identical_to_eager_on_every_checked_replay": bool(identical)}
        del graphs, gheld

    # pre-norm unit (Section 3.3) at the same shape: bandwidth-bound row kernels
    gamma = torch.ones((n,), dtype=torch.float32, device="cuda")
    a_n, rms_n = L.loract_prenorm_forward(x, gamma)
    us_pf = timed(lambda: L.loract_prenorm_forward(x, gamma))
    us_pb = timed(lambda: L.loract_prenorm_backward(xhat, rms_n, gamma, dy[:, :n] if n_out >= n else xhat))
    prenorm = {"forward_us": round(us_pf, 1), "forward_gbps": round(2 * x_bytes / us_pf / 1e3, 1),
               "backward_us": round(us_pb, 1), "backward_gbps": round(3 * x_bytes / us_pb / 1e3, 1),
               "note": "algorithmic bytes: forward reads X writes A (2|X|), backward reads A, dA writes dX (3|X|)"}
    del a_n

    if args.pmc_calibration:
        scratch = torch.empty_like(x)
        for _ in range(5):
            scratch.copy_(x)
        torch.cuda.synchronize()

    # comparator of Section 3.2 at equal rank on the same input: oversampling 8, one power iteration
    comparator = None
    if not args.no_comparator:
        def rsvd():
            L.loract_rsvd(x, k, oversample=8, power_iters=1, seed=w.seed)
        rsteps = max(3, args.steps // 5)
        for _ in range(2):
            rsvd()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(rsteps):
            rsvd()
        e1.record()
        torch.cuda.synchronize()
        us_rsvd = e0.elapsed_time(e1) * 1e3 / rsteps
        L.loract_profile_begin()
        for _ in range(rsteps):
            rsvd()
        torch.cuda.synchronize()
        rprof = L.loract_profile_end()
        us_trunc = sum(ms for nm, (ms, cnt) in rprof.items()
                       if nm in ("jacobi_eig", "truncate_bbt", "truncate_qw", "truncate_wtb")) * 1e3 / rsteps
        ur, vr = L.loract_rsvd(x, k, oversample=8, power_iters=1, seed=w.seed)
        xr = L.loract_reconstruct(ur, vr)
        err_rsvd = float((torch.linalg.norm(xr.float() - x.float()) / torch.linalg.norm(x.float())).item())
        ur0, vr0 = L.loract_rsvd(x, k, oversample=0, power_iters=0, seed=w.seed)
        xr0 = L.loract_reconstruct(ur0, vr0)
        err_rsvd0 = float((torch.linalg.norm(xr0.float() - x.float()) / torch.linalg.norm(x.float())).item())
        del ur, vr, xr, ur0, vr0, xr0
        comparator = {"method": "rsvd (oversampling 8, 1 power iteration, rank %d)" % k,
                      "rel_fro_err_rsvd": round(err_rsvd, 6),
                      "rel_fro_err_rsvd_plain": round(err_rsvd0, 6),
                      "note_err": "rsvd_plain = Gaussian test matrix of k columns, no power iteration: "
                                  "the method Algorithm 1 differs from only in the test matrix",
                      "total_us": round(us_rsvd, 1), "truncation_us": round(us_trunc, 1),
                      "range_finder_us": round(us_rsvd - us_trunc, 1),
                      "loract_compress_us": round(us_c, 1),
                      "speedup_vs_range_finder": round((us_rsvd - us_trunc) / us_c, 2)}

    # Error against time: the power rounds of Algorithm 1 (t = 0, 1, 2) beside the randomized SVD it
    # is compared with in Section 3.2 (Gaussian test matrix; q power rounds; with and without the
    # oversampling of 8 columns that the comparator's truncation to rank k goes with).
    error_vs_time = None
    if not args.no_comparator:
        x32n = torch.linalg.norm(x.float())

        def measure(fn):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            reps = max(3, args.steps // 5)
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                uu, vv = fn()
            e1.record()
            torch.cuda.synchronize()
            xr = L.loract_reconstruct(uu, vv)
            e = float((torch.linalg.norm(xr.float() - x.float()) / x32n).item())
            return round(e0.elapsed_time(e1) * 1e3 / reps, 1), round(e, 6)

        rows = []
        for t_it in (0, 1, 2):
            us_t, e_t = measure(lambda: L.loract_compress(x, k, t=t_it, seed=w.seed))
            rows.append({"method": "Algorithm 1, t = %d" % t_it, "us": us_t, "rel_fro_err": e_t})
        for q_it, p_over in ((0, 0), (1, 0), (1, 8)):
            us_t, e_t = measure(lambda: L.loract_rsvd(x, k, oversample=p_over, power_iters=q_it, seed=w.seed))
            rows.append({"method": "randomized SVD, q = %d, oversampling %d" % (q_it, p_over), "us": us_t,
                         "rel_fro_err": e_t})
        error_vs_time = {"rank": k, "rank_k_floor": (round(float(w.extras["rank_k_floor"]), 6)
                                                      if "rank_k_floor" in w.extras else None), "rows": rows}

    # accuracy of the timed outputs (cheap GPU-side figure; full parity lives in tests/)
    err = float((torch.linalg.norm(xhat.float() - x.float()) / torch.linalg.norm(x.float())).item())

    out = {
        "metric": "activation GB/s compressed+reconstructed",
        "value": round(x_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dt_name, "data": "synthetic",
        "config": {"workload": "%s: %dx%d %s, rank %d, LoRA rank %d, dY %dx%d; step = compress + "
                               "reconstruct + lora_grad" % (args.workload, m, n, dt_name, k, r_l, m, n_out)},
        "phases_us": {"compress": round(us_c, 1), "reconstruct": round(us_r, 1), "lora_grad": round(us_l, 1)},
        "phases_us_cold_cache": {"compress": round(us_c_cold, 1), "reconstruct": round(us_r_cold, 1),
                                 "lora_grad": round(us_l_cold, 1),
                                 "note": "512 MB fill between calls (inputs evicted from the memory-side cache)"},
        "gbps": {"compress": round(x_bytes / us_c / 1e3, 1), "reconstruct": round(x_bytes / us_r / 1e3, 1),
                 "round_trip": round(x_bytes / (us_c + us_r) / 1e3, 1)},
        "hbm_frac_two_pass": round((2 * x_bytes + k * n * b + 2 * m * k * 4 + 2 * (m + n) * k * b + x_bytes)
                                   / ((us_c + us_r) * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
        "rel_fro_err": round(err, 6),
        "rel_fro_err_rank_k_floor": (round(float(w.extras["rank_k_floor"]), 6)
                                     if "rank_k_floor" in w.extras else None),
        "roofline": roofline,
        "roofline_streaming": roofline_streaming,
        "comparator": comparator,
        "pipelined": pipelined,
        "pipelined_graph": pipelined_graph,
        "error_vs_time": error_vs_time,
        "prenorm": prenorm,
        "kernels": kernels,
    }

    if not args.no_cpu_baseline:
        from oracle import loract_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        x64 = w.x.astype(np.float64)
        reps, t_start = 0, time.perf_counter()
        while True:
            uo, vo = orc.decompose(x64, k, seed=w.seed)
            xo = orc.reconstruct(uo, vo)
            orc.lora_grad(uo, vo, dy_h, bl_h, 1.0)
            reps += 1
            elapsed = time.perf_counter() - t_start
            if elapsed >= 10.0 or reps >= 200:
                break
        out["cpu_baseline"] = {"value": round(x_bytes / (elapsed / reps) / 1e9, 4), "unit": "GB/s",
                               "cores": int(cores), "kind": "oracle",
                               "sample": "%d full steps of the same %s workload (fp64 numpy oracle, "
                                         "%.1f s)" % (reps, args.workload, elapsed)}
        out["parity_vs_oracle"] = round(orc.rel_fro(xhat.float().cpu().numpy(), xo), 6)

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
