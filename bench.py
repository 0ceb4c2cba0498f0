#!/usr/bin/env python3
"""Benchmark of the MGLU forward pass on one MI355X.

A step is one mglu_forward call (the whole hot path: stream W and the packed masks,
accumulate, reduce, fused Swish/gate*value/mixture epilogue, store) on synthetic inputs
already resident in HBM.  The headline workload is the decode GEMV configuration
(d_model 2048, d_ff 5632, four masks, one token, bf16); every step reads a different copy
of (W, masks) out of a ring larger than the 256 MB last-level cache, so the rate is an HBM
rate, not a cache rate.  One JSON line is printed; the other configurations ride along
under "extra".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
LLC_BYTES = 256 * 2 ** 20    # last-level (Infinity) cache
HEADLINE = "decode_gemv 2048x5632 n_m=4 T=1"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5000)
    ap.add_argument("--warmup", type=int, default=1000)
    ap.add_argument("--no-extra", action="store_true", help="headline workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-refs", action="store_true",
                    help="skip the warm-cache, SwiGLU-reference and read-ceiling legs of the headline")
    ap.add_argument("--probe", default="",
                    help="profiling aid: launch only this workload ('headline' or a substring of an extra "
                         "workload's name) 20 times, then one mglu_stream_read and one device copy of "
                         "exactly 1 GiB each (known sizes to scale byte counters by), print nothing")
    ap.add_argument("--only", default="", help="comma list of extra workloads to run (names as printed)")
    return ap.parse_args()


class Workload:
    """One (config, tokens) case with a ring of packed (W, masks) copies on the GPU."""

    def __init__(self, name, cfg, ring_bytes=2 * LLC_BYTES, swiglu=True, max_ring=64):
        import torch
        from paper_2506_23225_amd import api, costmodel, synth
        self.name, self.cfg = name, cfg
        self.torch, self.api = torch, api
        T, h, d, n_m = cfg["tokens"], cfg["d_model"], cfg["d_ff"], cfg["n_masks"]
        dt = synth.TORCH_DTYPE[cfg["dtype"]]
        self.desc = api.make_desc(T, h, d, n_m, dt)
        x, W, masks = synth.make_inputs(**cfg, seed=0, device="cuda:0")
        self.x = x
        Wp = api.mglu_pack_weights(self.desc, W)
        Mp = api.mglu_pack_masks(self.desc, masks)
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


def time_steps(torch, fn, steps, warmup):
    """ms per step over exactly `steps` calls, HIP events on the launch stream, synchronised on both sides."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for i in range(steps):
        fn(warmup + i)
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return start.elapsed_time(stop) / steps, wall_ms / steps


def summarize(w, ms, wall_ms, bound):
    T = w.cfg["tokens"]
    rec = {
        "workload": w.name, "tokens": T, "d_model": w.cfg["d_model"], "d_ff": w.cfg["d_ff"],
        "n_masks": w.cfg["n_masks"], "dtype": w.cfg["dtype"], "ring_copies": w.copies,
        "ms": ms, "wall_ms": wall_ms,
        "GBps": w.bytes / ms / 1e6, "hbm_frac": w.bytes / ms / 1e6 / HBM_PEAK_GBS,
        "TFLOPs": w.flops / ms / 1e9, "mfma_frac": w.flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
        "tokens_per_s": T / ms * 1e3, "bound": bound,
    }
    return rec


def cpu_baseline(cfg, unit_bytes, budget_s=10.0):
    """The fp64 oracle, as it stands, on the host cores: full decode-GEMV workload, repeated within a time budget."""
    import numpy as np
    from oracle import mglu_oracle as oracle
    from paper_2506_23225_amd import synth
    x, W, masks = synth.make_inputs(**cfg, seed=0, device="cpu")
    xn, Wn, Mn = x.double().numpy(), W.double().numpy(), masks.numpy()
    oracle.mglu_forward(xn[:, :64], Wn[:64, :64], Mn[:, :64, :64])  # load the library
    times = []
    t_start = time.perf_counter()
    while len(times) < 200 and (time.perf_counter() - t_start) < budget_s:
        t0 = time.perf_counter()
        oracle.mglu_forward(xn, Wn, Mn)
        times.append(time.perf_counter() - t0)
    best = min(times)
    return {
        "value": unit_bytes / best / 1e9, "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
        "sample": "full %s workload (%d token, all %d columns), best of %d runs in %.1f s, %.3f s per run (median %.3f s)"
                  % (cfg["name"], cfg["tokens"], cfg["d_ff"], len(times), time.perf_counter() - t_start, best,
                     sorted(times)[len(times) // 2]),
        "tokens_per_s": cfg["tokens"] / best,
    }


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

    # ---- headline: decode GEMV, cold ring ----
    head_cfg = synth.config("decode_gemv")
    head = Workload(HEADLINE, head_cfg, swiglu=not args.no_refs)
    ms, wall_ms = time_steps(torch, head.step, args.steps, args.warmup)
    rec = summarize(head, ms, wall_ms, "hbm")

    result = {
        "metric": "MGLU decode HBM GB/s (frac of peak) + prefill TFLOP/s, tokens/s per layer",
        "value": rec["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": HEADLINE, "d_model": 2048, "d_ff": 5632, "n_masks": 4, "tokens": 1,
                   "ring_copies": head.copies, "cache": "cold (ring of copies > 2x last-level cache)"},
        "tokens_per_s": rec["tokens_per_s"], "hbm_frac": rec["hbm_frac"],
        "wall_ms_per_step": wall_ms,
        "roofline": {"bound": "hbm", "achieved": rec["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": rec["hbm_frac"], "traffic": measured_traffic("decode_gemv"),
                     "kernel": "mglu::stream_resident_kernel<mglu::Bf16Traits, 4, 0, 2, true>",
                     "bytes_per_launch": head.bytes},
    }
    if not args.no_refs:
        sw_ms, _ = time_steps(torch, head.swiglu_step, args.steps, args.warmup)
        warm = Workload("decode_gemv warm", head_cfg, ring_bytes=1, swiglu=False)
        warm_ms, _ = time_steps(torch, warm.step, args.steps, args.warmup)
        del warm
        # measured streaming-read ceiling of this GPU (same load pattern, nothing else)
        buf = torch.empty(2 ** 30, dtype=torch.uint8, device="cuda:0").random_(0, 255)
        sink = torch.zeros(256, dtype=torch.int32, device="cuda:0")
        read_ms, _ = time_steps(torch, lambda i: api.mglu_stream_read(buf, sink), 50, 5)
        del buf
        # the same number of bytes as one headline step, read cold by the plain read kernel: what a
        # launch that only streams them costs on this GPU (start-up and drain included)
        n_small = head.bytes // 16 * 16
        smalls = [torch.empty(n_small, dtype=torch.uint8, device="cuda:0").random_(0, 255)
                  for _ in range(max(2, int(2 * LLC_BYTES // n_small) + 1))]
        small_ms, _ = time_steps(torch, lambda i: api.mglu_stream_read(smalls[i % len(smalls)], sink),
                                 args.steps, args.warmup)
        del smalls
        result["plain_read_same_bytes"] = {"ms": small_ms, "GBps": n_small / small_ms / 1e6,
                                           "note": "events around back-to-back launches; at this size the "
                                                   "host's launch rate and the kernel time are about equal"}
        # the same cold-ring steps captured once into a HIP graph and replayed: launch gaps of the host gone
        gsteps = 4 * head.copies
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(cap):
            head.step(0)
            cap.synchronize()
            with torch.cuda.graph(graph, stream=cap):
                for i in range(gsteps):
                    head.step(i)
        torch.cuda.current_stream().wait_stream(cap)
        graph_ms, _ = time_steps(torch, lambda i: graph.replay(), 20, 3)
        result["graph_replay"] = {"ms_per_step": graph_ms / gsteps, "GBps": head.bytes / (graph_ms / gsteps) / 1e6,
                                  "steps_per_graph": gsteps}
        del graph
        result["warm_cache"] = {"ms": warm_ms, "GBps": head.bytes / warm_ms / 1e6}
        result["swiglu_reference"] = {"ms": sw_ms, "GBps": head.glu_bytes / sw_ms / 1e6,
                                      "mglu_over_swiglu_time": ms / sw_ms,
                                      "byte_model_ratio": (16 + head_cfg["n_masks"]) / 32.0}
        result["measured_read_ceiling_GBps"] = 2 ** 30 / read_ms / 1e6
    del head

    if not args.no_extra:
        result["extra"] = run_extras(torch, synth, args)
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(head_cfg, rec_bytes(head_cfg))
        result["gpu_over_cpu"] = result["value"] / result["cpu_baseline"]["value"]
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
    cases = []
    for T in (1, 4, 16):
        cases.append(("decode_8b 4096x14336 n_m=8 T=%d" % T, synth.config("decode_8b", tokens=T), "hbm", 400, 200))
    for n_m in (1, 2, 4, 8):
        for T in (1, 32):
            cases.append(("large 8192x28672 n_m=%d T=%d" % (n_m, T),
                          synth.config("large", n_masks=n_m, tokens=T), "hbm", 100, 60))
    # the paper's own precision on the shape of its kernel timings (4096 x 14336, 4 masks, batch 1), and its prefill twin
    cases.append(("fp16 4096x14336 n_m=4 T=1", synth.config("prefill_8b", tokens=1, dtype="f16"), "hbm", 400, 200))
    cases.append(("prefill_8b 4096x14336 n_m=4 T=4096", synth.config("prefill_8b"), "mfma", 20, 20))
    cases.append(("fp16 4096x14336 n_m=4 T=4096", synth.config("prefill_8b", dtype="f16"), "mfma", 20, 20))
    # 16 masks, the paper's largest ablation
    cases.append(("decode_8b 4096x14336 n_m=16 T=1", synth.config("decode_8b", n_masks=16, tokens=1), "hbm", 300, 150))
    cases.append(("prefill_8b 4096x14336 n_m=16 T=4096", synth.config("prefill_8b", n_masks=16), "mfma", 8, 8))
    for n_m in (1, 2, 4, 8):
        cases.append(("large 8192x28672 n_m=%d T=2048" % n_m,
                      synth.config("large", n_masks=n_m, tokens=2048), "mfma", 10, 10))
    return cases


def probe(torch, synth, args):
    """For rocprofv3 counter runs: 20 launches of one workload, then two kernels of known size (1 GiB):
    the library's streaming read, which issues the same 16-byte-per-lane loads as the MGLU kernels
    (read counters), and a plain device copy (write counters)."""
    if args.probe == "headline":
        name, cfg = HEADLINE, synth.config("decode_gemv")
    else:
        name, cfg = next((n, c) for n, c, _, _, _ in extra_cases(synth) if args.probe in n)
    w = Workload(name, cfg, swiglu=False)
    for i in range(20):
        w.step(i)
    from paper_2506_23225_amd import api
    src = torch.empty(2 ** 30, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    sink = torch.zeros(256, dtype=torch.int32, device="cuda:0")
    torch.cuda.synchronize()
    api.mglu_stream_read(src, sink)
    dst.copy_(src)
    torch.cuda.synchronize()


def rec_bytes(cfg):
    from paper_2506_23225_amd import costmodel
    return costmodel.mglu_bytes(cfg["d_model"], cfg["d_ff"], cfg["n_masks"], cfg["tokens"], cfg["dtype"])


def run_extras(torch, synth, args):
    cases = extra_cases(synth)
    only = [s.strip() for s in args.only.split(",") if s.strip()]
    out = []
    for name, cfg, bound, steps, warmup in cases:
        if only and not any(o in name for o in only):
            continue
        w = Workload(name, cfg)
        ms, wall_ms = time_steps(torch, w.step, steps, warmup)
        rec = summarize(w, ms, wall_ms, bound)
        sw_ms, _ = time_steps(torch, w.swiglu_step, steps, warmup)
        rec["swiglu_ms"] = sw_ms
        rec["swiglu_GBps"] = w.glu_bytes / sw_ms / 1e6
        rec["swiglu_TFLOPs"] = w.glu_flops / sw_ms / 1e9
        rec["mglu_over_swiglu_time"] = ms / sw_ms
        out.append(rec)
        print("[bench] %-40s %9.4f ms  %8.1f GB/s (%.1f%% HBM)  %8.1f TFLOP/s (%.1f%% MFMA)  swiglu %9.4f ms"
              % (name, ms, rec["GBps"], 100 * rec["hbm_frac"], rec["TFLOPs"], 100 * rec["mfma_frac"], sw_ms),
              file=sys.stderr, flush=True)
        del w
        torch.cuda.empty_cache()
    out.extend(run_widened(torch, synth, only))
    return out


def run_widened(torch, synth, only):
    """Rows beyond the up-projection itself: the Top-K routed layer and the whole FFN block."""
    out = []
    cases = [("routed top-2 of 8, decode_8b 4096x14336 T=1", synth.config("decode_8b", tokens=1), "routed", 400, 200),
             ("routed top-2 of 8, large 8192x28672 T=1", synth.config("large", n_masks=8, tokens=1), "routed", 100, 60),
             ("ffn (layer + output projection), decode_8b 4096x14336 n_m=8 T=1", synth.config("decode_8b", tokens=1), "ffn", 400, 200),
             ("ffn (layer + output projection), prefill_8b 4096x14336 n_m=4 T=4096", synth.config("prefill_8b"), "ffn", 20, 20)]
    for name, cfg, kind, steps, warmup in cases:
        if only and not any(o in name for o in only):
            continue
        w = Workload(name, cfg, swiglu=False)
        if kind == "routed":
            w.enable_routing(2)
            ms, wall_ms = time_steps(torch, w.routed_step, steps, warmup)
            rec = summarize(w, ms, wall_ms, "hbm")
            rec["note"] = "same bytes as the unrouted layer; sums of the unselected masks are skipped"
        else:
            w.enable_ffn()
            ms, wall_ms = time_steps(torch, w.ffn_step, steps, warmup)
            w.bytes, w.flops = w.ffn_bytes, w.ffn_flops
            rec = summarize(w, ms, wall_ms, "hbm" if cfg["tokens"] <= 64 else "mfma")
            rec["note"] = "two launches; bytes and FLOPs include the output projection"
        out.append(rec)
        print("[bench] %-62s %9.4f ms  %8.1f GB/s (%.1f%% HBM)  %8.1f TFLOP/s (%.1f%% MFMA)"
              % (name, ms, rec["GBps"], 100 * rec["hbm_frac"], rec["TFLOPs"], 100 * rec["mfma_frac"]),
              file=sys.stderr, flush=True)
        del w
        torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
