#!/usr/bin/env python3
"""Benchmark of the MGLU forward pass on one MI355X.

A step is one mglu_forward call (the whole hot path: stream W and the packed masks,
accumulate, reduce, fused Swish/gate*value/mixture epilogue, store) on synthetic inputs
already resident in HBM.  The headline workload is the largest single-GPU decode
configuration (d_model 8192, d_ff 28672, eight masks, one token, bf16); every step reads a
different copy of (W, masks) out of a ring larger than the 256 MB last-level cache, so the
rate is an HBM rate, not a cache rate.  One JSON line is printed; the other configurations
ride along under "extra", each with the step counts it was timed with.

Timing method (every row): W warm-up steps, then an untimed settle phase (more of the same
steps until the GPU has been busy for ~100 ms, so that the shader clock has settled), then a
blocker (a few launches of the library's plain read kernel) behind which the K timed steps
are queued, so that they run back to back on the device whatever the host's launch rate;
HIP events on the launch stream bracket exactly the K steps, with a synchronisation on both
sides.
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
LLC_BYTES = 256 * 2 ** 20    # last-level (Infinity) cache
HEADLINE = "large 8192x28672 n_m=8 T=1"
HEADLINE_KERNEL = "mglu::stream_resident_kernel<mglu::Bf16Traits, 8, 0, 2, false>"
HEADLINE_TRAFFIC_KEY = "large_nm8_T1"
SETTLE_MS = 100.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-extra", action="store_true", help="headline workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-refs", action="store_true",
                    help="skip the SwiGLU-reference and read-ceiling legs of the headline")
    ap.add_argument("--probe", default="",
                    help="profiling aid: launch only this workload ('headline', a substring of an extra "
                         "workload's name, or 'routed decode_8b' / 'routed large') 20 times, then one mglu_stream_read and one device copy of "
                         "exactly 1 GiB each (known sizes to scale byte counters by), print nothing")
    ap.add_argument("--only", default="", help="comma list of extra workloads to run (names as printed)")
    return ap.parse_args()


class Workload:
    """One (config, tokens) case with a ring of packed (W, masks) copies on the GPU."""

    def __init__(self, name, cfg, ring_bytes=2 * LLC_BYTES, swiglu=True, max_ring=64, keep_inputs=False):
        import torch
        from paper_2506_23225_amd import api, costmodel, synth
        self.name, self.cfg = name, cfg
        self.torch, self.api = torch, api
        T, h, d, n_m = cfg["tokens"], cfg["d_model"], cfg["d_ff"], cfg["n_masks"]
        dt = synth.TORCH_DTYPE[cfg["dtype"]]
        self.desc = api.make_desc(T, h, d, n_m, dt)
        self.plan = api.mglu_describe_plan(self.desc)
        x, W, masks = synth.make_inputs(**cfg, seed=0, device="cuda:0")
        self.x = x
        Wp = api.mglu_pack_weights(self.desc, W)
        Mp = api.mglu_pack_masks(self.desc, masks)
        self.inputs = (x, W, masks) if keep_inputs else None   # for the CPU-oracle leg
        del masks
        per_copy = Wp.numel() + Mp.numel()
        self.copies = max(1, min(max_ring, -(-ring_bytes // per_copy)))
        self.ring = [(Wp, Mp)] + [(Wp.clone(), Mp.clone()) for _ in range(self.copies - 1)]
        self.out = torch.empty(T, d, dtype=dt, device="cuda:0")
        ws = api.mglu_workspace_bytes(self.desc)
        self.ws = torch.zeros(max(ws, 16), dtype=torch.uint8, device="cuda:0")
        self.bytes = costmodel.mglu_bytes(h, d, n_m, T, cfg["dtype"])
        self.flops = costmodel.mglu_flops(h, d, n_m, T)
        self.glu_bytes = costmodel.glu_bytes(h, d, T, cfg["dtype"])
        self.glu_flops = costmodel.glu_flops(h, d, T)
        self.swiglu_ring = None
        if swiglu:
            # same-shape two-matrix SwiGLU: the second matrix is an independent draw
            _, Wv, _ = synth.make_inputs(h, d, 1, 1, cfg["dtype"], cfg["w_std"], seed=1, device="cuda:0")
            Wvp = api.mglu_pack_weights(self.desc, Wv)
            n = max(1, min(max_ring, -(-ring_bytes // (2 * Wp.numel()))))
            self.swiglu_ring = [(Wp, Wvp)] + [(Wp.clone(), Wvp.clone()) for _ in range(n - 1)]
        del W

    def step(self, i):
        Wp, Mp = self.ring[i % self.copies]
        self.api.mglu_forward(self.desc, self.x, Wp, Mp, out=self.out, workspace=self.ws)

    # ---- widened rows: Top-K routed layer and the whole FFN block (layer + output projection) ----
    def enable_routing(self, k):
        """Route weights from the library's router on a seeded random W_r; routed_step then runs the routed layer."""
        torch = self.torch
        gen = torch.Generator(device="cuda:0").manual_seed(2)
        Wr = (torch.randn(self.cfg["d_model"], self.cfg["n_masks"], generator=gen, device="cuda:0") * 0.1).to(self.x.dtype)
        self.route = self.api.mglu_route_topk(self.desc, self.x, Wr, k)

    def routed_step(self, i):
        Wp, Mp = self.ring[i % self.copies]
        self.api.mglu_forward_variant(self.desc, self.x, Wp, Mp, route_weights=self.route, out=self.out, workspace=self.ws)

    def enable_planar_routing(self, k, masks):
        """The same routed layer on the planar mask format: a ring of (W, planar masks) copies; only k planes are read."""
        from paper_2506_23225_amd import costmodel
        self.route_k = k
        Mpl = self.api.mglu_pack_masks_planar(self.desc, masks)
        self.planar_ring = [(Wp, Mpl if j == 0 else Mpl.clone()) for j, (Wp, _) in enumerate(self.ring)]
        c = self.cfg
        self.routed_bytes = costmodel.mglu_bytes(c["d_model"], c["d_ff"], k, c["tokens"], c["dtype"])   # W + k planes
        self.routed_flops = costmodel.mglu_flops(c["d_model"], c["d_ff"], k, c["tokens"])               # t + k masked sums

    def planar_routed_step(self, i):
        Wp, Mpl = self.planar_ring[i % self.copies]
        self.api.mglu_forward_routed(self.desc, self.x, Wp, Mpl, self.route, self.route_k, out=self.out)

    def enable_ffn(self, ring_bytes=2 * LLC_BYTES):
        torch = self.torch
        T, h, d = self.cfg["tokens"], self.cfg["d_model"], self.cfg["d_ff"]
        gen = torch.Generator(device="cuda:0").manual_seed(3)
        Wo = (torch.randn(d, h, generator=gen, device="cuda:0") * 0.02).to(self.x.dtype)
        self.down = self.api.make_desc(T, d, h, 1, self.x.dtype)
        Wop = self.api.mglu_pack_weights(self.down, Wo)
        self.wo_ring = [Wop] + [Wop.clone() for _ in range(self.copies - 1)]
        self.y = torch.empty(T, h, dtype=self.x.dtype, device="cuda:0")
        self.ffn_bytes = self.bytes + Wop.numel() + 2 * T * d + 2 * T * h   # + Wo, hidden in again, y out
        self.ffn_flops = self.flops + 2 * T * d * h

    def ffn_step(self, i):
        Wp, Mp = self.ring[i % self.copies]
        self.api.mglu_ffn_forward(self.desc, self.x, Wp, Mp, self.wo_ring[i % self.copies], hidden=self.out, y=self.y,
                                  workspace=self.ws)

    def swiglu_step(self, i):
        Wg, Wv = self.swiglu_ring[i % len(self.swiglu_ring)]
        self.api.swiglu_forward(self.desc, self.x, Wg, Wv, out=self.out, workspace=self.ws)


class Timer:
    """HIP-event timing of exactly K steps that run back to back on the device (see the module docstring)."""

    def __init__(self, torch, api):
        self.torch, self.api = torch, api
        self.block_buf = torch.empty(2 ** 30, dtype=torch.uint8, device="cuda:0").random_(0, 255)
        self.sink = torch.zeros(256, dtype=torch.int32, device="cuda:0")
        self.block_ms = None      # duration of one blocker launch, measured once

    def _blocker(self, n):
        for _ in range(n):
            self.api.mglu_stream_read(self.block_buf, self.sink)

    def run(self, fn, steps, warmup):
        """-> dict(ms, wall_ms, steps, warmup, settle_steps, blocker_launches)."""
        torch = self.torch
        if self.block_ms is None:
            self._blocker(2)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            self._blocker(4)
            b.record()
            torch.cuda.synchronize()
            self.block_ms = a.elapsed_time(b) / 4
        # warm-up: W steps as asked, timed on the host side to learn the enqueue cost of one step
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(warmup):
            fn(i)
        # enqueue cost only (nothing synchronises inside the loop); too few steps to tell: assume a slow host
        host_ms = (time.perf_counter() - t0) * 1e3 / warmup if warmup >= 3 else 0.03
        torch.cuda.synchronize()
        # settle: untimed steps until ~SETTLE_MS of GPU work has gone by since the warm-up began
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn(warmup)
        b.record()
        torch.cuda.synchronize()
        one_ms = max(a.elapsed_time(b), 1e-3)
        settle = int(min(20000, max(0, SETTLE_MS / one_ms - warmup)))
        for i in range(settle):
            fn(warmup + 1 + i)
        base = warmup + 1 + settle
        # blocker long enough for the host to enqueue all K steps behind it
        host_ms = max(host_ms, 0.004)
        n_block = int(min(4000, steps * host_ms * 1.5 / self.block_ms + 2))
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        self._blocker(n_block)
        start.record()
        for i in range(steps):
            fn(base + i)
        stop.record()
        enqueue_ms = (time.perf_counter() - t0) * 1e3
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        return {"ms": start.elapsed_time(stop) / steps, "wall_ms": wall_ms / steps, "steps": steps, "warmup": warmup,
                "settle_steps": settle + 1, "blocker_launches": n_block,
                "host_enqueue_ms_per_step": enqueue_ms / (steps + n_block)}


def summarize(w, t, bound):
    T = w.cfg["tokens"]
    ms = t["ms"]
    rec = {
        "workload": w.name, "kernel": w.plan, "tokens": T, "d_model": w.cfg["d_model"], "d_ff": w.cfg["d_ff"],
        "n_masks": w.cfg["n_masks"], "dtype": w.cfg["dtype"], "ring_copies": w.copies,
        "ms": ms, "steps": t["steps"], "warmup": t["warmup"], "settle_steps": t["settle_steps"],
        "GBps": w.bytes / ms / 1e6, "hbm_frac": w.bytes / ms / 1e6 / HBM_PEAK_GBS,
        "TFLOPs": w.flops / ms / 1e9, "mfma_frac": w.flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
        "tokens_per_s": T / ms * 1e3, "bound": bound,
    }
    return rec


ONE_THREAD_C2 = r"""
import sys, time
sys.path.insert(0, %r)
from oracle import mglu_oracle as oracle
from paper_2506_23225_amd import synth
cfg = synth.config("decode_gemv")
x, W, masks = synth.make_inputs(**cfg, seed=0, device="cpu")
xn, Wn, Mn = x.double().numpy(), W.double().numpy(), masks.numpy()
oracle.mglu_forward(xn[:, :64], Wn[:64, :64], Mn[:, :64, :64])
oracle._load().omp_set_num_threads(1)   # the OpenMP runtime the oracle library is linked to; its source is untouched
best = 1e9
for _ in range(3):
    t0 = time.perf_counter(); oracle.mglu_forward(xn, Wn, Mn); best = min(best, time.perf_counter() - t0)
print(oracle.threads(), best)
"""


def cpu_baseline(head, budget_s=12.0, sample_cols=4096):
    """The fp64 oracle, as it stands, on the host cores, on a bounded sample of the headline workload: the
    first `sample_cols` output columns (all of d_model, all masks, the one token), repeated within a time budget."""
    from oracle import mglu_oracle as oracle
    from paper_2506_23225_amd import costmodel
    x, W, masks = head.inputs
    cfg = head.cfg
    xn = x.double().cpu().numpy()
    Wn = W[:, :sample_cols].double().cpu().numpy()
    Mn = masks[:, :, :sample_cols].cpu().numpy()
    oracle.mglu_forward(xn[:, :64], Wn[:64, :64], Mn[:, :64, :64])  # load the library
    times = []
    t_start = time.perf_counter()
    while len(times) < 100 and (time.perf_counter() - t_start) < budget_s:
        t0 = time.perf_counter()
        oracle.mglu_forward(xn, Wn, Mn)
        times.append(time.perf_counter() - t0)
    best = min(times)
    frac = sample_cols / cfg["d_ff"]
    sample_bytes = costmodel.mglu_bytes(cfg["d_model"], sample_cols, cfg["n_masks"], cfg["tokens"], cfg["dtype"])
    rec = {
        "value": sample_bytes / best / 1e9, "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
        "sample": "%s: the first %d of %d output columns (%.4f of the layer; every k, every mask, the one token), "
                  "best of %d runs in %.1f s, %.3f s per run (median %.3f s); extrapolated full layer %.2f s"
                  % (head.name, sample_cols, cfg["d_ff"], frac, len(times), time.perf_counter() - t_start, best,
                     sorted(times)[len(times) // 2], best / frac),
        "tokens_per_s": cfg["tokens"] / (best / frac),
    }
    # one-thread time of the oracle on the decode GEMV configuration (2048 x 5632, 4 masks), in a process of its own
    try:
        out = subprocess.run([sys.executable, "-c", ONE_THREAD_C2 % ROOT], capture_output=True, text=True,
                             timeout=120).stdout.split()
        rec["decode_gemv_one_thread"] = {"threads": int(out[0]), "seconds": float(out[1]),
                                         "note": "full decode_gemv workload, best of 3"}
    except Exception as e:   # the baseline leg must not take the bench line down
        rec["decode_gemv_one_thread"] = {"error": repr(e)}
    return rec


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the layer shards by d_ff "
              "columns with no exchange between the shards). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2506_23225_amd import _lib, api, synth
    _lib.load()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.probe:
        return probe(torch, synth, args)
    timer = Timer(torch, api)

    # ---- headline: the largest decode configuration, cold ring ----
    head_cfg = synth.config("large", n_masks=8, tokens=1)
    head = Workload(HEADLINE, head_cfg, swiglu=not args.no_refs, keep_inputs=not args.no_cpu)
    t = timer.run(head.step, args.steps, args.warmup)
    rec = summarize(head, t, "hbm")
    ms = t["ms"]

    result = {
        "metric": "MGLU decode HBM GB/s (frac of peak) + prefill TFLOP/s, tokens/s per layer",
        "value": rec["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": HEADLINE, "d_model": 8192, "d_ff": 28672, "n_masks": 8, "tokens": 1,
                   "ring_copies": head.copies, "cache": "cold (ring of copies > 2x last-level cache)"},
        "timing": {"method": "HIP events around exactly `steps` launches queued behind a blocker launch, after "
                             "`warmup` steps and an untimed settle phase",
                   "settle_steps": t["settle_steps"], "blocker_launches": t["blocker_launches"],
                   "host_enqueue_ms_per_step": t["host_enqueue_ms_per_step"], "wall_ms_per_step": t["wall_ms"]},
        "tokens_per_s": rec["tokens_per_s"], "hbm_frac": rec["hbm_frac"],
        "roofline": {"bound": "hbm", "achieved": rec["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": rec["hbm_frac"], "traffic": measured_traffic(HEADLINE_TRAFFIC_KEY),
                     "traffic_source": "profiles/traffic.txt: committed rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE "
                                       "summary of this workload, a constant, not measured in this run",
                     "kernel": HEADLINE_KERNEL, "kernel_from_plan_query": head.plan,
                     "bytes_per_launch": head.bytes},
    }
    if not args.no_refs:
        sw = timer.run(head.swiglu_step, args.steps, args.warmup)
        # measured streaming-read ceiling of this GPU (same load pattern, nothing else), 1 GiB
        rd = timer.run(lambda i: api.mglu_stream_read(timer.block_buf, timer.sink), 50, 5)
        result["swiglu_reference"] = {"ms": sw["ms"], "GBps": head.glu_bytes / sw["ms"] / 1e6,
                                      "mglu_over_swiglu_time": ms / sw["ms"],
                                      "byte_model_ratio": (16 + head_cfg["n_masks"]) / 32.0}
        result["measured_read_ceiling_GBps"] = 2 ** 30 / rd["ms"] / 1e6
        # what a step costs with (next to) no work in it under this timing method: a 4 KiB read by the same kernel.
        # Every row's time includes this launch-to-launch floor; it is reported, never subtracted.
        floor = timer.run(lambda i: api.mglu_stream_read(timer.block_buf[:4096], timer.sink), 200, 20)
        result["timing"]["empty_launch_us"] = floor["ms"] * 1e3
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(head)
        result["gpu_over_cpu"] = result["value"] / result["cpu_baseline"]["value"]
    del head
    torch.cuda.empty_cache()

    if not args.no_extra:
        result["extra"] = run_extras(torch, synth, args, timer)
        for e in result["extra"]:
            if e["workload"].startswith("prefill_8b 4096x14336 n_m=4"):
                result["prefill_TFLOPs"] = e["TFLOPs"]
                result["prefill_mfma_frac"] = e["mfma_frac"]
                result["prefill_tokens_per_s"] = e["tokens_per_s"]
    print(json.dumps(result))


def measured_traffic(key):
    """HBM bytes per launch from the committed rocprofv3 counter summary (profiles/traffic.txt), or None."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        for line in f:
            parts = line.split()
            if len(parts) >= 2 and parts[0] == key:
                return float(parts[1])
    return None


def extra_cases(synth):
    """(name, config, bound, steps, warmup): every row is timed with its own counts, recorded in its record."""
    cases = [("decode_gemv 2048x5632 n_m=4 T=1", synth.config("decode_gemv"), "hbm", 1000, 200)]
    for T in (1, 4, 16):
        cases.append(("decode_8b 4096x14336 n_m=8 T=%d" % T, synth.config("decode_8b", tokens=T), "hbm", 400, 100))
    for n_m in (1, 2, 4, 8):
        for T in (1, 32):
            if (n_m, T) == (8, 1):
                continue   # the headline
            cases.append(("large 8192x28672 n_m=%d T=%d" % (n_m, T),
                          synth.config("large", n_masks=n_m, tokens=T), "hbm", 100, 30))
    # the paper's own precision on the shape of its kernel timings (4096 x 14336, 4 masks, batch 1), and its prefill twin
    cases.append(("fp16 4096x14336 n_m=4 T=1", synth.config("prefill_8b", tokens=1, dtype="f16"), "hbm", 400, 100))
    cases.append(("prefill_8b 4096x14336 n_m=4 T=4096", synth.config("prefill_8b"), "mfma", 20, 10))
    cases.append(("fp16 4096x14336 n_m=4 T=4096", synth.config("prefill_8b", dtype="f16"), "mfma", 20, 10))
    # 16 masks, the paper's largest ablation
    cases.append(("decode_8b 4096x14336 n_m=16 T=1", synth.config("decode_8b", n_masks=16, tokens=1), "hbm", 300, 100))
    cases.append(("prefill_8b 4096x14336 n_m=16 T=4096", synth.config("prefill_8b", n_masks=16), "mfma", 8, 4))
    for n_m in (1, 2, 4, 8):
        cases.append(("large 8192x28672 n_m=%d T=2048" % n_m,
                      synth.config("large", n_masks=n_m, tokens=2048), "mfma", 10, 5))
    return cases


def probe(torch, synth, args):
    """For rocprofv3 counter runs: 20 launches of one workload, then two kernels of known size (1 GiB):
    the library's streaming read, which issues the same 16-byte-per-lane loads as the MGLU kernels
    (read counters), and a plain device copy (write counters)."""
    routed = args.probe.startswith("routed")
    if args.probe == "headline":
        name, cfg = HEADLINE, synth.config("large", n_masks=8, tokens=1)
    elif routed:   # "routed decode_8b" / "routed large": top-2 of 8 on the planar mask format
        name, cfg = args.probe, synth.config("large" if "large" in args.probe else "decode_8b", n_masks=8, tokens=1)
    else:
        name, cfg = next((n, c) for n, c, _, _, _ in extra_cases(synth) if args.probe in n)
    w = Workload(name, cfg, swiglu=False, keep_inputs=routed)
    if routed:
        w.enable_routing(2)
        w.enable_planar_routing(2, w.inputs[2])
    for i in range(20):
        (w.planar_routed_step if routed else w.step)(i)
    from paper_2506_23225_amd import api
    src = torch.empty(2 ** 30, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    sink = torch.zeros(256, dtype=torch.int32, device="cuda:0")
    torch.cuda.synchronize()
    api.mglu_stream_read(src, sink)
    dst.copy_(src)
    torch.cuda.synchronize()


def run_extras(torch, synth, args, timer):
    cases = extra_cases(synth)
    only = [s.strip() for s in args.only.split(",") if s.strip()]
    out = []
    for name, cfg, bound, steps, warmup in cases:
        if only and not any(o in name for o in only):
            continue
        w = Workload(name, cfg)
        t = timer.run(w.step, steps, warmup)
        rec = summarize(w, t, bound)
        sw = timer.run(w.swiglu_step, steps, warmup)
        rec["swiglu_ms"] = sw["ms"]
        rec["swiglu_GBps"] = w.glu_bytes / sw["ms"] / 1e6
        rec["swiglu_TFLOPs"] = w.glu_flops / sw["ms"] / 1e9
        rec["mglu_over_swiglu_time"] = t["ms"] / sw["ms"]
        out.append(rec)
        print("[bench] %-40s %9.4f ms  %8.1f GB/s (%.1f%% HBM)  %8.1f TFLOP/s (%.1f%% MFMA)  swiglu %9.4f ms"
              % (name, t["ms"], rec["GBps"], 100 * rec["hbm_frac"], rec["TFLOPs"], 100 * rec["mfma_frac"], sw["ms"]),
              file=sys.stderr, flush=True)
        del w
        torch.cuda.empty_cache()
    out.extend(run_widened(torch, synth, only, timer))
    return out


def run_widened(torch, synth, only, timer):
    """Rows beyond the up-projection itself: the Top-K routed layer and the whole FFN block."""
    out = []
    cases = [("routed top-2 of 8, decode_8b 4096x14336 T=1", synth.config("decode_8b", tokens=1), "routed", 400, 100),
             ("routed top-2 of 8, large 8192x28672 T=1", synth.config("large", n_masks=8, tokens=1), "routed", 100, 30),
             ("ffn (layer + output projection), decode_8b 4096x14336 n_m=8 T=1", synth.config("decode_8b", tokens=1), "ffn", 400, 100),
             ("ffn (layer + output projection), prefill_8b 4096x14336 n_m=4 T=4096", synth.config("prefill_8b"), "ffn", 20, 10)]
    for name, cfg, kind, steps, warmup in cases:
        if only and not any(o in name for o in only):
            continue
        w = Workload(name, cfg, swiglu=False, keep_inputs=(kind == "routed"))
        if kind == "routed":
            w.enable_routing(2)
            w.enable_planar_routing(2, w.inputs[2])
            w.inputs = None
            # interleaved mask format first (every mask's bits stream, the unselected masks' sums are skipped) ...
            ti = timer.run(w.routed_step, steps, warmup)
            # ... then the planar format: only the two selected planes are read; bytes credited = W + 2 planes
            t = timer.run(w.planar_routed_step, steps, warmup)
            w.bytes, w.flops = w.routed_bytes, w.routed_flops
            rec = summarize(w, t, "hbm")
            rec["kernel"] = w.api.mglu_describe_plan(w.desc, "forward_routed", 2)
            rec["interleaved_format_ms"] = ti["ms"]
            rec["interleaved_format_kernel"] = w.api.mglu_describe_plan(w.desc, "forward_variant")
            rec["note"] = "planar mask format: bytes credited are W + the 2 selected mask planes"
        else:
            w.enable_ffn()
            t = timer.run(w.ffn_step, steps, warmup)
            w.bytes, w.flops = w.ffn_bytes, w.ffn_flops
            rec = summarize(w, t, "hbm" if cfg["tokens"] <= 64 else "mfma")
            rec["kernel"] = w.plan + " + " + w.api.mglu_describe_plan(w.down, "linear")
            rec["note"] = "two launches; bytes and FLOPs include the output projection"
        out.append(rec)
        print("[bench] %-62s %9.4f ms  %8.1f GB/s (%.1f%% HBM)  %8.1f TFLOP/s (%.1f%% MFMA)"
              % (name, t["ms"], rec["GBps"], 100 * rec["hbm_frac"], rec["TFLOPs"], 100 * rec["mfma_frac"]),
              file=sys.stderr, flush=True)
        del w
        torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
