#!/usr/bin/env python3
"""Benchmark of the QTIP inference hot path on one MI355X.

Workload (the one the headline metric is quoted on): a 8192 x 28672 layer stored as
2-bit 3INST trellis codes (L = 16, V = 1), batch 1.  One step = the whole hot path
once: the input-side random Hadamard transform of the activation (qtip_rht) followed
by the fused decode + matrix-vector product (qtip_decode_matvec).  All inputs are
seeded synthetic buffers already resident in HBM.  Consecutive steps rotate over
enough distinct copies of the code stream (>= 512 MiB in total) that the 256 MiB
last-level cache cannot serve them: the reported rate is an HBM rate.

Prints ONE JSON line.  `value` is effective GB/s on compressed-weight bytes per step;
`roofline` is the decode + matvec kernel alone, timed with HIP events on the stream it
is launched on; `cpu_baseline` is the CPU oracle timed on a bounded slab of the same
workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
WORKLOAD = "metric_3inst_k2_8192x28672"

# Counter figures for the decode + matvec kernel come from rocprofv3 --pmc runs of this file,
# whose summaries live in profiles/<workload>_counters.txt as `key = value` lines: HBM bytes per
# launch (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a plain copy
# of known size), vector-ALU wave instructions per launch (SQ_INSTS_VALU), and the SHA-256 of the
# kernel sources they were measured on.  They are reported only while that hash still matches
# the sources in the tree; after any kernel change they are dropped until the profile is redone.
PROFILE_DIR = os.path.join(ROOT, "profiles")
KERNEL_SOURCE_DIR = os.path.join(ROOT, "paper_2406_11235_amd", "csrc")


def kernel_sources_sha256():
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(KERNEL_SOURCE_DIR)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            with open(os.path.join(KERNEL_SOURCE_DIR, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def measured_counters(workload):
    """{key: value} from profiles/<workload>_counters.txt, or {} if the file is missing or was
    taken on other kernel sources than the tree holds (said on stderr)."""
    path = os.path.join(PROFILE_DIR, workload + "_counters.txt")
    if not os.path.exists(path):
        return {}
    vals = {}
    with open(path) as f:
        for line in f:
            if "=" in line and not line.lstrip().startswith("#"):
                key, v = line.split("=", 1)
                vals[key.strip()] = v.strip()
    if vals.get("kernel_sources_sha256") != kernel_sources_sha256():
        log(f"bench.py: {os.path.relpath(path, ROOT)} was measured on other kernel sources than the "
            f"tree holds: its counter figures (traffic, vector-ALU instructions) are left out")
        return {}
    vals["file"] = os.path.relpath(path, ROOT)
    return vals


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def bench_quantize(args, q, torch, np):
    """The GPU tail-biting Viterbi quantizer on a 2048 x 2048 matrix of i.i.d. Gaussian
    weights scaled to the code (16384 tiles), 2-bit 3INST: one step = the whole matrix.
    The rate is in trellis state updates: per tile 2 passes (Algorithm 4) x 256 steps x
    2^16 states.  ALU roof: an update is three dependent binary32 instructions (subtract,
    fused multiply-add onto the minimum, compare-for-minimum), against 256 CUs x 4 SIMDs x
    16 lanes x 2.4 GHz lane-instructions per second (no packed FP32 in this build)."""
    import qtip_synth as synth
    code_id, k, V, m, n = synth.CODE_3INST, 2, 1, 2048, 2048
    steps = max(1, min(args.steps, 3))
    warmup = max(1, min(args.warmup, 1))
    ntiles = (m // 16) * (n // 16)
    rng = np.random.default_rng(240611235 + 77)
    sd = 1.2437                                  # standard deviation of the 3INST code values
    Wh = (rng.standard_normal((m, n)) * sd).astype(np.float32)
    W = torch.from_numpy(Wh).cuda()
    in_flight = 4096
    ws_bytes = q.qtip_quantize_gpu_workspace(k, V, in_flight)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    codes = torch.zeros((ntiles, 8 * k), dtype=torch.int32, device="cuda")
    err = torch.zeros(ntiles, dtype=torch.float32, device="cuda")
    run = lambda: q.qtip_quantize_gpu(W, m, n, 16, k, V, code_id, None, codes, err, ws, ws_bytes)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    updates = ntiles * 2 * 256 * 65536
    rate = updates / (ms * 1e-3)
    mse = float(err.double().sum()) / (m * n)
    log(f"quantize: {ms:.1f} ms per {m}x{n} matrix = {ms*1e3/ntiles:.2f} us/tile, "
        f"{rate/1e12:.2f} T state updates/s, mse/var {mse/sd**2:.4f}")
    peak = 256 * 4 * 16 * 2.4e9
    roofline = {"bound": "alu", "kernel": "viterbi_forward_kernel", "unit": "T lane-instructions/s",
                "achieved": 3 * rate / 1e12, "peak": peak / 1e12, "frac": 3 * rate / peak,
                "traffic": None, "instructions_per_state_update": 3,
                "tflops": 4 * rate / 1e12, "frac_of_published_fp32_vector_peak_157.3": 4 * rate / 157.3e12}
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        C = oracle.codebook(16, V, code_id)
        codes_h = codes.cpu().numpy().view(np.uint32)
        t0 = time.perf_counter()
        done = 0
        same = 0
        while time.perf_counter() - t0 < 10.0 and done < 64:
            S = Wh[0:16, 16 * done:16 * done + 16].reshape(-1)
            d, words = oracle.tailbiting_quantize_f32(S, 16, k, V, C)
            same += int(np.array_equal(words, codes_h[done]))
            done += 1
        dt = time.perf_counter() - t0
        cpu_baseline = {"value": done * 2 * 256 * 65536 / dt, "unit": "state updates/s", "cores": 1,
                        "kind": "oracle",
                        "sample": f"first {done} tiles of the matrix, binary32 Algorithm 4 of the "
                                  f"oracle, {dt:.1f} s; {same} of {done} streams equal the GPU's",
                        "tiles_per_s": done / dt}
        log(f"cpu oracle: {done/dt:.2f} tiles/s on one thread; {same}/{done} streams identical")
    # the same matrix through BlockLDLQ (Algorithm 5) with a strongly correlated synthetic
    # proxy Hessian: decomposition and loop on the GPU; reported beside the headline figure
    X = torch.randn(2 * n, n, dtype=torch.float64, device="cuda",
                    generator=torch.Generator(device="cuda").manual_seed(11))
    X = 0.9 * X[:, :1] + 0.1 * X
    H = X.T @ X / (2 * n) + 1e-3 * torch.eye(n, dtype=torch.float64, device="cuda")
    A = torch.empty((n, n), dtype=torch.float32, device="cuda")
    lws_bytes = q.qtip_block_ldl_workspace(n)
    lws = torch.empty(lws_bytes, dtype=torch.uint8, device="cuda")
    q.qtip_block_ldl(H, n, 16, A, None, lws, lws_bytes)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    q.qtip_block_ldl(H, n, 16, A, None, lws, lws_bytes)
    torch.cuda.synchronize()
    ms_ldl = (time.perf_counter() - t0) * 1e3
    del lws
    qws_bytes = q.qtip_quantize_ldlq_workspace(m, n, k, V, m // 16)
    qws = ws if qws_bytes <= ws_bytes else torch.empty(qws_bytes, dtype=torch.uint8, device="cuda")
    What = torch.empty((m, n), dtype=torch.float32, device="cuda")
    proxy = {}
    for name, fb in (("feedback", A), ("none", torch.zeros_like(A))):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        q.qtip_quantize_ldlq(W, fb, m, n, 16, k, V, code_id, None, codes, What, err, qws, max(qws_bytes, 0))
        torch.cuda.synchronize()
        if name == "feedback":
            ms_ldlq = (time.perf_counter() - t0) * 1e3
        Ed = (What - W).double()
        proxy[name] = float(torch.trace(Ed @ H @ Ed.T))
    ldlq = {"ms_block_ldl": ms_ldl, "ms_quantize_ldlq": ms_ldlq, "us_per_tile": ms_ldlq * 1e3 / ntiles,
            "proxy_loss": proxy["feedback"], "proxy_loss_without_feedback": proxy["none"]}
    log(f"BlockLDLQ {m}x{n}: block LDL {ms_ldl:.1f} ms, loop {ms_ldlq:.1f} ms = "
        f"{ms_ldlq*1e3/ntiles:.2f} us/tile; proxy loss {proxy['feedback']:.4g} against "
        f"{proxy['none']:.4g} without feedback")

    return {"metric": "tail-biting Viterbi quantization (L=16, 2-bit 3INST, T=256), trellis state "
                      "updates per second",
            "value": rate, "unit": "state updates/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"quantize_3inst_k2_{m}x{n}", "m": m, "n": n, "code": "3INST",
                       "L": 16, "k": k, "V": V, "tiles": ntiles, "tiles_in_flight": in_flight},
            "us_per_tile": ms * 1e3 / ntiles, "mse_over_variance": mse / sd ** 2,
            "roofline": roofline, "cpu_baseline": cpu_baseline, "block_ldlq": ldlq}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=WORKLOAD)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy five times, so that a rocprofv3 "
                         "--pmc FETCH_SIZE / WRITE_SIZE run of this file has a kernel of known "
                         "traffic to scale the counters by")
    ap.add_argument("--all", action="store_true",
                    help="also time every configured workload (report on stderr)")
    ap.add_argument("--quantize", action="store_true",
                    help="instead of the inference path, time the GPU quantizer "
                         "(qtip_quantize_gpu) and print its JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no sharding, no collectives); "
            "--gpus must be 1")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2406_11235_amd as q
    import qtip_synth as synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    q.lib()
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()

    if args.quantize:
        print(json.dumps(bench_quantize(args, q, torch, np)), flush=True)
        return

    def prepare(w, min_total=512 << 20):
        inp = synth.make_inputs(w)
        copies = max(2, -(-min_total // w.code_bytes))
        rng = np.random.default_rng(w.seed + 1)
        bufs = [dev(inp.codes)]
        for _ in range(copies - 1):
            # distinct random streams of the same shape (decode time does not depend on bits)
            words = rng.integers(0, 1 << 32, size=inp.codes.shape, dtype=np.uint64)
            bufs.append(dev(words.astype(np.uint32)))
        st = dict(w=w, inp=inp, bufs=bufs, lut=dev(inp.lut), X=dev(inp.X),
                  signs=dev(inp.signs_n), scale=dev(inp.row_scale),
                  xt=torch.empty((w.B, w.n), dtype=torch.float16, device="cuda"),
                  Y=torch.empty((w.B, w.m), dtype=torch.float32, device="cuda"))
        return st

    def rht(st):
        w = st["w"]
        q.qtip_rht(st["X"], st["signs"], w.n, w.block_n, w.B, 0, st["xt"])

    def mult(st, i):
        w = st["w"]
        codes = st["bufs"][i % len(st["bufs"])]
        if w.B == 1 and st["scale"] is None:
            q.qtip_decode_matvec(codes, w.L, w.k, w.V, w.code_id, st["lut"], w.m, w.n, st["xt"],
                                 st["Y"])
        else:
            q.qtip_decode_matmat(codes, w.L, w.k, w.V, w.code_id, st["lut"], w.m, w.n, st["xt"],
                                 w.B, st["scale"], st["Y"])

    ROUNDS = 11          # timed rounds of `steps` launches each; the median round is reported
    MIN_WARM_MS = 50.0   # warm-up lasts at least this long (clocks ramp over some milliseconds)

    class Timing(float):
        """Median ms per call over the rounds (the float), plus the spread."""
        def __new__(cls, per_round):
            per_round = sorted(per_round)
            self = super().__new__(cls, per_round[len(per_round) // 2])
            self.min, self.max, self.rounds = per_round[0], per_round[-1], len(per_round)
            return self

    def warm(fn, warmup):
        """`warmup` calls, then more of the same until MIN_WARM_MS of wall time have passed."""
        t0 = time.perf_counter()
        i = 0
        while True:
            for _ in range(max(1, warmup)):
                fn(i)
                i += 1
            torch.cuda.synchronize()
            if (time.perf_counter() - t0) * 1e3 >= MIN_WARM_MS:
                return i

    def timed(fn, steps, warmup):
        """ms per call of fn(i): ROUNDS rounds of exactly `steps` calls, each bracketed by HIP
        events on the launch stream; the median round is the figure, min and max go with it."""
        i = warm(fn, warmup)
        events = []
        for _ in range(ROUNDS):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                fn(i)
                i += 1
            e1.record()
            torch.cuda.synchronize()
            events.append((e0, e1))
        return Timing([a.elapsed_time(b) / steps for a, b in events])

    def timed_graph(step, period, steps, warmup):
        """The same steps captured once into a HIP graph (`period` steps = one pass over
        the rotating buffers) and replayed: launch overhead leaves the timed region."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(period):
                step(i)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(period):
                step(i)
        replays = max(1, -(-steps // period))
        warm(lambda i: g.replay(), max(1, warmup // period))
        events = []
        for _ in range(ROUNDS):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(replays):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            events.append((e0, e1))
        return Timing([a.elapsed_time(b) / (replays * period) for a, b in events])

    def measure(name, steps, warmup):
        st = prepare(synth.WORKLOADS[name])
        w = st["w"]

        def step(i):
            rht(st)
            mult(st, i)

        ms_step = timed(step, steps, warmup)
        ms_step_graph = timed_graph(step, len(st["bufs"]), steps, warmup)
        rht(st)
        ms_kernel = timed(lambda i: mult(st, i), steps, warmup)
        # the same launches replayed from a HIP graph: for kernels of a few microseconds the
        # host cannot issue launches as fast as the GPU finishes them, and the loop above
        # then times the host
        ms_kernel_graph = timed_graph(lambda i: mult(st, i), len(st["bufs"]), steps, warmup)
        ms_hot = timed(lambda i: mult(st, 0), steps, warmup)
        ms_rht = timed(lambda i: rht(st), steps, warmup)
        return st, dict(ms_step=ms_step, ms_step_graph=ms_step_graph, ms_kernel_graph=ms_kernel_graph,
                        ms_kernel=ms_kernel, ms_hot=ms_hot, ms_rht=ms_rht, bytes=w.code_bytes,
                        copies=len(st["bufs"]))

    st, r = measure(args.workload, args.steps, args.warmup)
    w = st["w"]
    gbs = lambda ms: w.code_bytes / (ms * 1e-3) / 1e9
    spread = lambda t: f"{t*1e3:.2f} us (min {t.min*1e3:.2f}, max {t.max*1e3:.2f})"
    log(f"[{w.name}] median of {ROUNDS} rounds of {args.steps} steps: step {spread(r['ms_step'])}, "
        f"{r['ms_step_graph']*1e3:.2f} us replayed from a HIP graph; "
        f"decode+matvec kernel {spread(r['ms_kernel'])} cold = {gbs(r['ms_kernel']):.0f} GB/s "
        f"({gbs(r['ms_kernel'])/HBM_PEAK_GBS*100:.1f}% of 8 TB/s), {r['ms_kernel_graph']*1e3:.2f} us replayed "
        f"from a HIP graph, {spread(r['ms_hot'])} "
        f"cache-resident, rht {r['ms_rht']*1e3:.2f} us back to back, {r['copies']} rotating buffers")

    counters = measured_counters(w.name)
    # algorithmic bytes per launch: code stream + activation + output
    alg_bytes = w.code_bytes + 2 * w.n * w.B + 4 * w.m * w.B
    roofline = {"bound": "hbm", "kernel": "decode+matvec", "achieved": alg_bytes / (r["ms_kernel"] * 1e-3) / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": alg_bytes / (r["ms_kernel"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "traffic": int(counters["traffic_bytes_per_launch"]) if "traffic_bytes_per_launch" in counters else None,
                "traffic_from": counters.get("file"), "us_per_launch": r["ms_kernel"] * 1e3,
                "us_per_launch_min": r["ms_kernel"].min * 1e3, "us_per_launch_max": r["ms_kernel"].max * 1e3,
                "us_per_launch_hipgraph": r["ms_kernel_graph"] * 1e3,
                "us_per_launch_cache_resident": r["ms_hot"] * 1e3,
                "algorithmic_bytes": alg_bytes}

    # The same kernel against the vector-ALU roof: wave instructions per launch (SQ_INSTS_VALU),
    # 64 lanes each, against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second
    # (the rate of the four-cycle instructions that make up most of the loop; the simplest
    # 32-bit operations issue in two cycles, so the fraction could pass 1 for other code).
    valu = None
    if "valu_wave_instructions_per_launch" in counters:
        winsts = int(counters["valu_wave_instructions_per_launch"])
        peak = 256 * 4 * 16 * 2.4e9
        valu = {"bound": "alu", "kernel": "decode+matvec", "unit": "T lane-instructions/s",
                "achieved": winsts * 64 / (r["ms_hot"] * 1e-3) / 1e12, "peak": peak / 1e12,
                "frac": winsts * 64 / (r["ms_hot"] * 1e-3) / peak,
                "valu_wave_instructions_per_launch": winsts, "counters_from": counters["file"]}

    # The lookup-only code is bound by its table reads: one 2-byte LDS read per weight at random
    # addresses.  Peak: 32 four-byte banks per CU, each serving one address per cycle.
    lds = None
    if w.code_id == synth.CODE_LUT:
        lookups = w.m * w.n
        peak = 256 * 32 * 2.4e9
        lds = {"bound": "lds", "kernel": "decode+matvec", "unit": "T table reads/s",
               "achieved": lookups / (r["ms_hot"] * 1e-3) / 1e12, "peak": peak / 1e12,
               "frac": lookups / (r["ms_hot"] * 1e-3) / peak, "table_reads_per_launch": lookups}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        rows = 2048
        slab = st["inp"].codes[: (rows // w.tile[0]) * (w.n // w.tile[1])]
        xt = st["xt"].cpu().numpy()
        t0 = time.perf_counter()
        Wd = oracle.dequantize(slab, w.L, w.k, w.V, w.code_id, rows, w.n, st["inp"].lut, tile=w.tile)
        yref = oracle.matmat_dense(Wd, xt)
        dt = time.perf_counter() - t0
        reps = 1
        while dt < 10.0 and reps < 64:          # extend to about 10 s of CPU work
            t1 = time.perf_counter()
            Wd = oracle.dequantize(slab, w.L, w.k, w.V, w.code_id, rows, w.n, st["inp"].lut, tile=w.tile)
            yref = oracle.matmat_dense(Wd, xt)
            dt += time.perf_counter() - t1
            reps += 1
        sample_bytes = rows * w.n * w.k // 8
        mult(st, 0)
        torch.cuda.synchronize()
        ygpu = st["Y"].cpu().numpy()[:, :rows]
        err = float(np.abs(ygpu - yref).max() / np.abs(yref).max())
        cpu_baseline = {"value": sample_bytes * reps / dt / 1e9, "unit": "GB/s",
                        "cores": oracle.threads(), "kind": "oracle",
                        "sample": f"first {rows} of {w.m} output rows (all {w.n} inputs), "
                                  f"oracle dequantize + fp64 matvec, {reps} repetitions, "
                                  f"{dt:.1f} s",
                        "us_per_matvec_extrapolated": dt / reps * (w.m / rows) * 1e6,
                        "gpu_vs_oracle_max_rel_err": err}
        log(f"cpu oracle: {cpu_baseline['value']:.4f} GB/s on {cpu_baseline['cores']} threads; "
            f"GPU vs oracle on the sample: max rel err {err:.2e}")

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.all:
        for name in synth.WORKLOADS:
            if name == args.workload:
                continue
            st2, r2 = measure(name, max(20, args.steps // 4), args.warmup)
            w2 = st2["w"]
            g2 = w2.code_bytes / (r2["ms_kernel_graph"] * 1e-3) / 1e9
            log(f"[{name}] kernel {r2['ms_kernel_graph']*1e3:.2f} us cold from a HIP graph ({g2:.0f} GB/s, "
                f"{g2/HBM_PEAK_GBS*100:.1f}%), {r2['ms_kernel']*1e3:.2f} us launched one by one, "
                f"{r2['ms_hot']*1e3:.2f} us hot, rht "
                f"{r2['ms_rht']*1e3:.2f} us (launch-bound), step {r2['ms_step']*1e3:.2f} us")
            del st2
            torch.cuda.empty_cache()

    out = {
        "metric": "batch-1 decode+matvec effective HBM GB/s on compressed-weight bytes, "
                  + ("2-bit 3INST 8192x28672" if w.name == WORKLOAD else w.name),
        "value": gbs(r["ms_step"]), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": float(r["ms_step"]), "ms_per_step_min": r["ms_step"].min,
        "ms_per_step_max": r["ms_step"].max, "rounds": ROUNDS, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": w.name, "m": w.m, "n": w.n, "code": synth.CODE_NAMES[w.code_id],
                   "L": w.L, "k": w.k, "V": w.V, "batch": w.B, "rht_block": w.block_n,
                   "step": "qtip_rht + qtip_decode_matvec",
                   "rotating_code_buffers": r["copies"]},
        "us_per_matvec": r["ms_kernel"] * 1e3, "us_rht": r["ms_rht"] * 1e3,
        "ms_per_step_hipgraph": float(r["ms_step_graph"]),
        "pct_of_hbm_peak": gbs(r["ms_kernel"]) / HBM_PEAK_GBS * 100,
        "roofline": roofline, "roofline_alu": valu, "roofline_lds": lds, "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
