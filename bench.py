#!/usr/bin/env python3
"""Throughput of the two-way error-feedback compression hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic gradients:
n x bpc_compress (worker: q = g + e, C(q), residual), 1 x bpc_server_aggregate (decode n
messages, average, + server residual, recompress, residual), 1 x bpc_adaptive_update (decode
the pulled message fused with the moment / parameter update).  Inputs are resident in HBM
before the clock starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-others] [--no-cpu]
                  [--no-stream-probe]

Stage times are medians over per-call HIP event pairs on the launch stream; after every timed
region the workspace's status word is checked (a device-side wait that gave up would make the
numbers meaningless, so it aborts the run).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, vendor figure


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="bert_large")
    ap.add_argument("--no-others", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--worker-streams", type=int, default=2, choices=(1, 2),
                    help="streams the workers of the sparse kinds take turns on")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-partitions", type=int, default=8, help="partitions in the CPU sample")
    ap.add_argument("--cpu-steps", type=int, default=6, help="pipeline steps the CPU sample runs")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy a few times (reference for hardware counters)")
    ap.add_argument("--no-stream-probe", action="store_true",
                    help="skip the plain streaming kernels that measure the achievable bandwidth")
    ap.add_argument("--cpu-single-partitions", type=int, default=3,
                    help="partitions in the single-threaded CPU sample (one step)")
    return ap.parse_args()


def payload_bytes_per_elem(w):
    k = w["kind"]
    if k == "sign":
        return 1.0 / 8
    if k in ("dither", "natdither"):
        # a nibble, plus one bit for each level bit above the third (linear levels beyond 7)
        levels, planes = w.get("levels", 4), 0
        while k == "dither" and (levels >> (3 + planes)):
            planes += 1
        return 0.5 + planes / 8
    if k == "fp16":
        return 2.0
    if k == "topk":
        return 8 * w["k_ratio"]
    if k == "topk16":
        return 6 * w["k_ratio"]
    if k == "randk":
        return 4 * w["k_ratio"]
    return 4.0


def algorithmic_bytes_per_elem(w):
    """Bytes the method must move per gradient element: every input read once, every output
    written once."""
    G = 4 if w["dtype"] == "f32" else 2
    pl = payload_bytes_per_elem(w)
    n = w["n_workers"]
    return {"W": G + 8 + pl, "S": n * pl + 8 + pl, "U": pl + 24}


class Pipeline:
    """Device state of one workload and the three stage calls."""

    def __init__(self, name, w, torch, bpc, synth, worker_streams=2):
        self.name, self.w, self.torch, self.bpc = name, w, torch, bpc
        dev = "cuda"
        self.D, self.n = w["D"], w["n_workers"]
        self.pe = synth.part_elems(w["dtype"])
        kind = {"sign": bpc.SIGN, "topk": bpc.TOPK, "randk": bpc.RANDK, "dither": bpc.DITHER,
                "natdither": bpc.NATDITHER, "fp16": bpc.FP16, "topk16": bpc.TOPK16}[w["kind"]]
        self.kw = dict(k_ratio=w.get("k_ratio", 0.01), levels=w.get("levels", 4),
                       value_scale=w.get("value_scale", 1.0), seed=synth.BASE_SEED)
        self.kind = kind
        p0 = bpc.make_params(kind, self.pe, **self.kw)
        self.grads = [synth.device_gradient(w["dist"], self.D, w["dtype"], worker=i, device=dev)
                      for i in range(self.n)]
        self.res = [torch.zeros(self.D, dtype=torch.float32, device=dev) for _ in range(self.n)]
        self.sres = torch.zeros(self.D, dtype=torch.float32, device=dev)
        pb = bpc.payload_bytes(p0, self.D)
        self.pay = [torch.zeros(pb, dtype=torch.uint8, device=dev) for _ in range(self.n)]
        self.pay_out = torch.zeros(pb, dtype=torch.uint8, device=dev)
        blocks = synth.layer_blocks(self.D, 768 if name.startswith("bert_base") else 1024)
        self.blocks = torch.from_numpy(blocks.astype("int64")).to(dev)
        self.ws = torch.empty(max(bpc.workspace_bytes(p0, self.D, self.n),
                                  bpc.update_workspace_bytes(p0, self.D, len(blocks) - 1)), dtype=torch.uint8, device=dev)
        # Workers whose call does not fill the device (the sparse kinds: the selection pass of
        # top-k runs on one workgroup per partition) take turns on two streams, each with a
        # workspace of its own, so that one worker's selection overlaps the next one's streaming
        # pass; the server call joins them.  (The single-pass kernels of the other kinds fill the
        # device and are kept apart by the library anyway.)
        self.side = []
        if w["kind"] in ("topk", "topk16", "randk") and self.n > 1 and worker_streams > 1:
            self.side = [torch.cuda.Stream(), torch.cuda.Stream()]
            self.ws_side = [torch.empty_like(self.ws) for _ in self.side]
        self.x = synth.device_params(self.D, device=dev)
        self.m = torch.zeros(self.D, dtype=torch.float32, device=dev)
        self.v = torch.zeros(self.D, dtype=torch.float32, device=dev)
        self.t = 0

    def params(self, role, worker):
        return self.bpc.make_params(self.kind, self.pe, stream_id=(self.t << 32) | (role << 16) | worker, **self.kw)

    def stage_w(self, i, ws=None):
        self.bpc.bpc_compress(self.params(0, i), self.grads[i], self.res[i], self.pay[i], self.ws if ws is None else ws)

    def workers(self):
        """All n worker calls of a step: one after the other, or alternating over two streams."""
        if not self.side:
            for i in range(self.n):
                self.stage_w(i)
            return
        torch = self.torch
        main = torch.cuda.current_stream()
        for s in self.side:
            s.wait_stream(main)
        for i in range(self.n):
            k = i % len(self.side)
            with torch.cuda.stream(self.side[k]):
                self.stage_w(i, ws=self.ws_side[k])
        for s in self.side:
            main.wait_stream(s)

    def stage_s(self):
        ins = [self.params(0, i) for i in range(self.n)]
        self.bpc.bpc_server_aggregate(ins, self.pay, self.params(1, 0), self.sres, self.D, self.pay_out, self.ws)

    def stage_u(self):
        t = max(self.t, 1)
        opt = self.bpc.make_opt(self.bpc.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, t)
        self.bpc.bpc_adaptive_update(self.params(1, 0), self.pay_out, self.x, self.m, self.v, opt, self.ws)

    def stage_u_lans(self):
        """The update as Algorithm 5 prints it (block-normalised, the partitions as blocks); timed
        beside the Adam-style update of the step, on the same buffers."""
        t = max(self.t, 1)
        opt = self.bpc.make_opt(self.bpc.OPT_LANS, 1e-3, 0.9, 0.999, 1e-8, 0.01, t)
        self.bpc.bpc_adaptive_update(self.params(1, 0), self.pay_out, self.x, self.m, self.v, opt, self.ws)

    def stage_u_lans_layers(self):
        """The same update with the blocks Algorithm 5 means: layers (offsets shaped like the
        tensors of a BERT encoder stack, synth.layer_blocks), not partitions."""
        t = max(self.t, 1)
        opt = self.bpc.make_opt(self.bpc.OPT_LANS, 1e-3, 0.9, 0.999, 1e-8, 0.01, t, block_offsets=self.blocks)
        self.bpc.bpc_adaptive_update(self.params(1, 0), self.pay_out, self.x, self.m, self.v, opt, self.ws)

    def step(self):
        self.t += 1
        self.workers()
        self.stage_s()
        self.stage_u()

    def check(self, where):
        """Waits for the stream; raises if a device-side wait of the last call gave up."""
        try:
            for ws in [self.ws] + (self.ws_side if self.side else []):
                self.bpc.workspace_check(self.params(0, 0), self.D, ws)
        except self.bpc.BpcError as err:
            raise SystemExit(f"bench.py: {self.name}, {where}: {err}")


def timed(torch, fn, reps):
    """Median milliseconds of fn() over reps calls: one HIP event before each call and one after
    the last, on the stream fn launches on (torch's current stream, which the binding passes to
    the library)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    torch.cuda.synchronize()
    for i in range(reps):
        ev[i].record()
        fn()
    ev[reps].record()
    torch.cuda.synchronize()
    per_call = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
    mid = reps // 2
    return per_call[mid] if reps % 2 else 0.5 * (per_call[mid - 1] + per_call[mid])


def run_workload(name, w, steps, warmup, torch, bpc, synth, worker_streams=2):
    pipe = Pipeline(name, w, torch, bpc, synth, worker_streams)
    for _ in range(warmup):
        pipe.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        pipe.step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    pipe.check("timed steps")
    # per-stage medians, steady state (non-zero residuals)
    reps = max(steps, 5)
    ms_w = timed(torch, lambda: pipe.stage_w(0), reps)
    pipe.check("worker stage")
    ms_s = timed(torch, pipe.stage_s, reps)
    pipe.check("server stage")
    ms_u = timed(torch, pipe.stage_u, reps)
    pipe.check("update stage")
    ms_ul = timed(torch, pipe.stage_u_lans, reps)
    pipe.check("LANS update stage")
    ms_ulb = timed(torch, pipe.stage_u_lans_layers, reps)
    pipe.check("LANS update stage, layer blocks")
    G = 4 if w["dtype"] == "f32" else 2
    D, n = w["D"], w["n_workers"]
    alg = algorithmic_bytes_per_elem(w)
    stages = {}
    for key, ms in (("W", ms_w), ("S", ms_s), ("U", ms_u), ("U_lans", ms_ul), ("U_lans_layers", ms_ulb)):
        a = alg[key[0]]
        stages[key] = {"ms": round(ms, 4), "gradient_GBps": round(D * G / ms / 1e6, 1),
                       "algorithmic_GBps": round(D * a / ms / 1e6, 1),
                       "frac_of_hbm_peak": round(D * a / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    out = {"workload": name, "D": D, "dtype": w["dtype"], "compressor": w["kind"], "n_workers": n,
           "worker_streams": max(1, len(pipe.side)),
           "ms_per_step": round(ms_step, 4), "value_GBps": round(n * D * G / ms_step / 1e6, 1),
           "pipeline_GBps_one_worker": round(D * G / (ms_w + ms_s + ms_u) / 1e6, 1), "stages": stages}
    if D <= (1 << 25):
        # small workloads are bound by launches: the same step recorded once into a HIP graph
        # and replayed (the recorded stream ids repeat, which does not change the work)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            pipe.step()
        out["ms_per_step_graph"] = round(timed(torch, graph.replay, reps), 4)
        del graph
    del pipe
    torch.cuda.empty_cache()
    return out


def stream_probe(torch, bpc, D):
    """What the memory system of this device delivers for the stages' access patterns: plain
    streaming kernels of the library (bpc_stream_probe: the traffic of a stage, none of its
    arithmetic) over D elements, GB/s from the median of HIP-event timings."""
    dev = "cuda"
    a16 = torch.zeros(D, dtype=torch.float16, device=dev)
    a, b, c = (torch.zeros(D, dtype=torch.float32, device=dev) for _ in range(3))
    out = {"elements": D}
    for key, mix, args in (("copy_GBps", bpc.PROBE_COPY, (a, None, c)),
                           ("worker_mix_GBps", bpc.PROBE_WORKER_MIX, (a16, b, c)),
                           ("update_mix_GBps", bpc.PROBE_UPDATE_MIX, (a, b, c))):
        for _ in range(3):
            bpc.bpc_stream_probe(mix, *args)
        ms = timed(torch, lambda: bpc.bpc_stream_probe(mix, *args), 15)
        out[key] = round(D * bpc.PROBE_BYTES_PER_ELEMENT[mix] / ms / 1e6, 1)
    del a16, a, b, c
    torch.cuda.empty_cache()
    return out


def sources_digest():
    """sha256 over the kernel sources: the profile summaries record the digest they were measured
    at, so a stored traffic figure can be told from one that predates a change to a kernel."""
    import hashlib

    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2105_07829_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hip", ".hpp")):
            h.update(f.encode())
            h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def cpu_baseline(name, w, n_parts, n_steps, synth, threads=None):
    """The CPU oracle as it stands, on `n_parts` full partitions of the same workload (all n
    workers, server, update) for `n_steps` steps, partitions spread over the host cores with a
    thread pool."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor

    import oracle

    oracle.build()
    pe = synth.part_elems(w["dtype"])
    n = w["n_workers"]
    D = pe * n_parts
    cores = threads or min(os.cpu_count() or 1, 16)
    kind = {"sign": oracle.SIGN, "topk": oracle.TOPK, "randk": oracle.RANDK, "dither": oracle.DITHER,
            "natdither": oracle.NATDITHER, "fp16": oracle.FP16, "topk16": oracle.TOPK16}[w["kind"]]
    kw = dict(k_ratio=w.get("k_ratio", 0.01), levels=w.get("levels", 4), value_scale=w.get("value_scale", 1.0),
              seed=synth.BASE_SEED)
    grads = [synth.host_gradient(w["dist"], D, w["dtype"], worker=i) for i in range(n)]
    res = [np.zeros(D, np.float32) for _ in range(n)]
    sres = np.zeros(D, np.float32)
    x, m, v = synth.host_params(D), np.zeros(D, np.float32), np.zeros(D, np.float32)
    strd = None

    step = [1]

    def prm(role, worker, part):
        return oracle.make_params(kind, pe, stream_id=(step[0] << 32) | (role << 16) | worker,
                                  first_partition=part, **kw)

    pays = [[None] * n_parts for _ in range(n)]
    outs = [None] * n_parts

    def work_w(job):
        i, p = job
        sl = slice(p * pe, (p + 1) * pe)
        pays[i][p] = oracle.compress(prm(0, i, p), grads[i][sl], res[i][sl])

    def work_su(p):
        sl = slice(p * pe, (p + 1) * pe)
        ins = [prm(0, i, p) for i in range(n)]
        outs[p] = oracle.server_aggregate(ins, [pays[i][p] for i in range(n)], prm(1, 0, p), sres[sl], pe)
        opt = oracle.make_opt(oracle.OPT_ADAM, 1e-3, 0.9, 0.999, 1e-8, 0.01, step[0])
        oracle.adaptive_update(prm(1, 0, p), outs[p], pe, x[sl], m[sl], v[sl], opt)

    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        for t in range(1, n_steps + 1):
            step[0] = t
            list(ex.map(work_w, [(i, p) for i in range(n) for p in range(n_parts)]))
            list(ex.map(work_su, range(n_parts)))
    dt = time.perf_counter() - t0
    G = 4 if w["dtype"] == "f32" else 2
    return {"value": round(n_steps * n * D * G / dt / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_steps} steps on {n_parts} full partitions ({D} elements) of {name}: {n} workers "
                      f"compress + server aggregate + update per step, {dt:.1f} s wall on {cores} threads"}


def recorded_traffic(workload, stage):
    """(HBM bytes per launch of a stage as measured with rocprofv3 counters and recorded under
    profiles/, digest of the kernel sources it was measured at), or (None, None)."""
    names = {"bert_large": "bench_bert_large_dither.txt", "resnet50": "bench_resnet50_topk.txt",
             "vgg16": "bench_vgg16_randk.txt", "bert_base": "bench_bert_base_sign.txt"}
    path = os.path.join(ROOT, "profiles", names.get(workload, f"bench_{workload}.txt"))
    total, digest = None, None
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 9 and f[0] == "TRAFFIC" and f[1] == workload and f[2] == stage:
                total = float(f[f.index("total_bytes") + 1])
            if len(f) >= 2 and f[0] == "SOURCES":
                digest = f[1]
    except OSError:
        pass
    return total, digest


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2105_07829_amd as bpc
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    bpc.lib()   # raises if the HIP library was not built: there is no fallback
    torch.cuda.set_device(0)
    head = run_workload(args.workload, synth.WORKLOADS[args.workload], args.steps, args.warmup, torch, bpc, synth,
                        args.worker_streams)
    others = []
    if not args.no_others:
        for name, w in synth.WORKLOADS.items():
            if name != args.workload:
                others.append(run_workload(name, w, max(3, args.steps // 2), 2, torch, bpc, synth, args.worker_streams))
    w = synth.WORKLOADS[args.workload]
    # dominant stage of the step: the worker compress call runs n times per step
    dom = max(("W", "S", "U"), key=lambda k: head["stages"][k]["ms"] * (w["n_workers"] if k == "W" else 1))
    alg = algorithmic_bytes_per_elem(w)[dom]
    ach = head["stages"][dom]["algorithmic_GBps"]
    call = {"W": "bpc_compress", "S": "bpc_server_aggregate", "U": "bpc_adaptive_update"}[dom]
    traffic, traffic_digest = recorded_traffic(args.workload, dom)
    if traffic is not None and traffic_digest != sources_digest():
        print(f"bench.py: the traffic figure under profiles/ was measured at kernel sources {traffic_digest}, "
              f"these are {sources_digest()}", file=sys.stderr)
    result = {
        "metric": "GB/s of gradient compressed+EF+decompressed, % of HBM peak, per compressor",
        "value": head["value_GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "elements": w["D"], "gradient_dtype": w["dtype"],
                   "compressor": w["kind"], "n_workers": w["n_workers"], "partition_bytes": synth.PART_BYTES,
                   "error_feedback": "two-way", "update": "adam-style"},
        "roofline": {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_measured_at_sources": traffic_digest, "sources": sources_digest(),
                     "kernel": f"{call} ({w['kind']})", "algorithmic_bytes_per_element": alg,
                     "elements_per_launch": w["D"]},
        "stages": head["stages"],
        "pipeline_GBps_one_worker": head["pipeline_GBps_one_worker"],
        "other_workloads": others,
    }
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["copy_calibration"] = {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "launches": 3}
    if not args.no_stream_probe:
        # the ceiling the 8 TB/s figure has to be read against: plain streams of the same shapes
        result["roofline"]["achieved_stream"] = stream_probe(torch, bpc, w["D"])
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(args.workload, w, args.cpu_partitions, args.cpu_steps, synth)
        single = cpu_baseline(args.workload, w, args.cpu_single_partitions, 1, synth, threads=1)
        result["cpu_baseline"]["single_thread"] = {"value": single["value"], "unit": "GB/s", "sample": single["sample"]}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
