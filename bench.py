#!/usr/bin/env python3
"""Benchmark of the HCCS hot path on one MI355X.

A step is one call of hccs_calibrated_softmax_i8 over one batch of the "long row"
workload, the largest of the stand-alone configurations: int8 logits [4,16,4096,4096]
-> uint8 probabilities (Alg. 1 with the 8-bit output path of Sec. III-B), 1.07 GB read
and 1.07 GB written per step.  The batch is resident in HBM before the timed region;
consecutive steps alternate between buffer sets.

Every timed launch, of the headline and of the other workloads, runs inside a replayed
HIP graph whose replays are bracketed by HIP events on the stream they run on: for any
--steps K the timed region is K launches from graphs (K // per replays of a graph of
`per` launches plus one replay of a graph holding the K % per remaining ones), never a
Python launch loop.

Prints ONE JSON line.  `value` is rows/s over the timed region (wall clock between device
synchronisations).  `roofline` prices the headline kernel against the HBM peak from the
event durations of the timed region; `rooflines` holds the same object for each of the
other workloads (kernel name, algorithmic bytes or operations per launch, average launch
time) so that every fraction can be recomputed from the committed kernel statistics.
`cpu_baseline` is the CPU oracle timed on the host's cores on the same batch.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
INT8_MFMA_PEAK_TOPS = 5000.0   # dense int8 MFMA peak
MALL_BYTES = 256 << 20         # memory-side cache: rotating buffer sets must exceed it
KERNEL_SOURCES = ["paper_2604_02292_amd/csrc/hccs_softmax.hip", "paper_2604_02292_amd/csrc/hccs_device.h"]

# the row kernel each stand-alone workload is dispatched to (hccs_softmax.hip, launch_mode)
ROW_KERNELS = {"pr1_ref": "hccs_rows_kernel<4,1,1,1,0,false>", "edge_encoder": "hccs_rows_kernel<8,1,1,1,0,false>",
               "stress_rows": "hccs_rows_kernel<16,2,1,4,0,false>", "long_row": "hccs_row_block_kernel<2,2,0,false>",
               "ragged_rows": "hccs_rows_staged_kernel<8,2,2,0>"}
HEADLINE = "long_row"


def kernel_hash():
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def counter_traffic(workload):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload's kernel,
    or None when there is none or the kernel sources changed after the counters were taken."""
    path = os.path.join(ROOT, "profiles", f"hccs_rows_{workload}_pmc.md")
    if not os.path.exists(path):
        return None
    rec = None
    with open(path) as fh:
        for line in fh:
            if line.startswith("TRAFFIC_RECORD "):
                rec = json.loads(line[len("TRAFFIC_RECORD "):])
    if rec is None or rec.get("kernel_hash") != kernel_hash():
        return None
    return rec.get("traffic_bytes_per_launch")


class GraphLoop:
    """Runs exact numbers of launches out of replayed HIP graphs.

    `launches` is a list of closures (one per buffer set); a graph of n launches cycles through
    them in order.  The kernels allocate nothing and use no memset nodes, so a graph holds kernel
    nodes only.  Every graph is replayed three times, untimed, right after its capture (the first
    replay also uploads it; the others let the clocks settle before anything is timed)."""

    def __init__(self, torch, launches, per):
        self.torch, self.launches, self.per = torch, launches, max(1, per)
        self.graphs = {}
        self.side = torch.cuda.Stream()

    def graph(self, n):
        if n not in self.graphs:
            torch = self.torch
            seq = [self.launches[i % len(self.launches)] for i in range(n)]
            self.side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(self.side):
                seq[0]()                       # one eager launch on the capture stream first
            self.side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=self.side):
                for f in seq:
                    f()
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            self.graphs[n] = g
        return self.graphs[n]

    def plan(self, n):
        """[(graph, launches)] covering exactly n launches."""
        per = min(self.per, n) if n > 0 else self.per
        out = [(self.graph(per), per)] * (n // per) if n > 0 else []
        if n > 0 and n % per:
            out.append((self.graph(n % per), n % per))
        return out

    def run(self, n):
        """n untimed launches."""
        for g, _ in self.plan(n):
            g.replay()

    def time(self, n):
        """n launches; returns (wall seconds between device synchronisations, per-replay
        (milliseconds, launches) from HIP events on the replaying stream)."""
        torch = self.torch
        plan = self.plan(n)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in plan]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for (g, _), (a, b) in zip(plan, ev):
            a.record()
            g.replay()
            b.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return t1 - t0, [(a.elapsed_time(b), c) for (a, b), (_, c) in zip(ev, plan)]

    def describe(self, n):
        per = min(self.per, n)
        tail = n % per
        return (f"{n // per} replay(s) of a HIP graph of {per} launches" +
                (f" + 1 replay of a graph of {tail}" if tail else ""))


def launch_ms(pairs):
    """Average and median duration of one launch from per-replay (milliseconds, launches)."""
    total = sum(c for _, c in pairs)
    per = sorted(ms / c for ms, c in pairs)
    return sum(ms for ms, _ in pairs) / total, per[len(per) // 2], total


def hbm_roofline(alg_bytes, avg_ms, kernel, extra=None):
    achieved = alg_bytes / (avg_ms * 1e-3) / 1e9
    r = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(achieved / HBM_PEAK_GBS, 4), "kernel": kernel, "algorithmic_bytes_per_launch": alg_bytes,
         "avg_launch_ms": round(avg_ms, 5)}
    if extra:
        r.update(extra)
    return r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--no-extras", action="store_true", help="headline workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--counter-run", choices=["rows", "attention", "attention_stream"], default=None,
                    help="for rocprofv3 --pmc: --steps eager launches of one workload's kernel, nothing else; "
                         "`rows` also launches the plain copy kernel on the same buffers (counter scaling)")
    ap.add_argument("--workload", default=HEADLINE, help="stand-alone workload of a `rows` counter run")
    ap.add_argument("--tokens", type=int, default=None,
                    help="tokens per (batch, head) item of an `attention` counter run (default: the 256 of the fused workload)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: rows are independent and shard with no exchange step, "
                 "so a multi-GPU figure would only restate this one; run with --gpus 1")
    if args.steps < 1 or args.warmup < 0:
        sys.exit("--steps must be positive, --warmup non-negative")

    import numpy as np
    import torch
    from paper_2604_02292_amd import binding, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    binding.lib()
    dev = torch.device("cuda:0")
    ncpu = min(os.cpu_count() or 1, 16)

    def rows_workload(name):
        if name == "ragged_rows":   # the edge-encoder recipe at a token count that is no multiple of 16
            return synth.make_workload("edge_encoder", threads=ncpu, shape=(64, 12, 197, 197))
        return synth.make_workload(name, threads=ncpu)

    def streaming_case():
        gq = np.random.default_rng(7)
        Bs, Hs, Ls, ds = 4, 12, 2048, 64
        qs, ks, vs = (torch.from_numpy(gq.integers(-64, 64, size=(Bs, Hs, Ls, ds), dtype=np.int8)).to(dev)
                      for _ in range(3))
        os_ = torch.empty((Bs, Hs, Ls, ds), dtype=torch.int32, device=dev)
        tab_s = synth.head_params(Hs, Ls, synth.BAND_U8, seed=11)
        rq_s = synth.requant_params(Hs, seed=11)
        return (Bs, Hs, Ls, ds), (lambda: binding.attention_i8(qs, ks, vs, tab_s, rq_s, synth.BAND_U8, out=os_))

    if args.counter_run == "attention":
        a = synth.make_workload("fused_attention", shape=None if args.tokens is None else (64, 12, args.tokens, 64))
        q, k, v = (torch.from_numpy(a[t]).to(dev) for t in ("q", "k", "v"))
        o = torch.empty(a["q"].shape, dtype=torch.int32, device=dev)
        launch = binding.prepare_attention(q, k, v, o, a["table"], a["requant"], a["band"])
        o2 = torch.empty_like(o)
        for _ in range(args.steps):
            launch()
            binding.copy_bytes(o, o2)                 # copy kernel of known size beside it (counter scaling)
        torch.cuda.synchronize()
        print(json.dumps({"counter_run": "attention", "launches": args.steps, "shape": list(a["q"].shape),
                          "bytes_read_per_launch": 3 * q.numel(), "bytes_written_per_launch": 4 * o.numel(),
                          "copy_bytes_each_way": 4 * o.numel()}))
        return
    if args.counter_run == "attention_stream":
        shape, launch = streaming_case()
        cp = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
        for _ in range(args.steps):
            launch()
            binding.copy_bytes(cp[:32 << 20], cp[32 << 20:])
        torch.cuda.synchronize()
        n = shape[0] * shape[1] * shape[2] * shape[3]
        print(json.dumps({"counter_run": "attention_stream", "launches": args.steps, "shape": list(shape),
                          "bytes_read_per_launch": 3 * n, "bytes_written_per_launch": 4 * n,
                          "copy_bytes_each_way": 32 << 20}))
        return
    if args.counter_run == "rows":
        w = rows_workload(args.workload)
        x = torch.from_numpy(w["logits"]).to(dev)
        out = torch.empty_like(x, dtype=torch.uint8)
        launch = binding.prepare_softmax(x, out, w["table"], w["band"])
        for _ in range(args.steps):
            launch()
            binding.copy_bytes(x, out)
        launch()                                       # leave the kernel's result, not the copy's, in `out`
        torch.cuda.synchronize()
        print(json.dumps({"counter_run": "rows", "workload": args.workload, "launches_each": args.steps,
                          "bytes_read_per_launch": x.numel(), "bytes_written_per_launch": x.numel(),
                          "kernel_hash": kernel_hash()}))
        return

    # ------------------------------------------------------------------ headline workload
    name = HEADLINE
    w = rows_workload(name)
    x_host, table, band = w["logits"], w["table"], w["band"]
    Bt, H, Lq, Lk = x_host.shape
    rows = Bt * H * Lq
    elems = rows * Lk
    alg_bytes = 2 * elems                     # 1 byte read + 1 byte written per element
    nsets = max(2, -(-6 * MALL_BYTES // alg_bytes))   # in+out of all sets > 6x the memory-side cache
    x0 = torch.from_numpy(x_host).to(dev)
    xs = [x0] + [x0.clone() for _ in range(nsets - 1)]
    outs = [torch.empty_like(x0, dtype=torch.uint8) for _ in range(nsets)]
    loop = GraphLoop(torch, [binding.prepare_softmax(xs[i], outs[i], table, band) for i in range(nsets)], per=64)

    loop.plan(args.steps)                      # capture (and upload) every graph of the timed region first
    loop.run(args.warmup)
    wall_s, pairs = loop.time(args.steps)
    wall_ms_per_step = wall_s * 1e3 / args.steps
    rows_per_s = rows * args.steps / wall_s
    kern_ms, kern_median, timed = launch_ms(pairs)
    roofline = hbm_roofline(alg_bytes, kern_ms, ROW_KERNELS[name],
                            {"traffic": counter_traffic(name), "median_launch_ms": round(kern_median, 5),
                             "launches_timed": timed,
                             "how": "HIP events around each graph replay of the timed region, summed and divided by "
                                    "the launches they hold"})
    roofline = {k: roofline[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel",
                                         "algorithmic_bytes_per_launch", "avg_launch_ms", "median_launch_ms",
                                         "launches_timed", "how")}

    result = {
        "metric": "HCCS logit rows/sec + achieved HBM GB/s (fraction of peak), int8 logits->u8 probs",
        "value": round(rows_per_s, 1), "unit": "rows/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall_ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"{name} int8 logits [{Bt},{H},{Lq},{Lk}] (causal mask as -128), 8-bit-path band, "
                               f"{nsets} alternating buffer sets",
                   "rows_per_step": rows, "row_length": Lk,
                   "launch": loop.describe(args.steps) + "; warm-up " +
                             (loop.describe(args.warmup) if args.warmup else "none") +
                             "; every graph also replayed 3 times untimed right after its capture"},
        "whole_job_GBps": round(alg_bytes / (wall_ms_per_step * 1e-3) / 1e9, 1),
        "elements_per_s": round(rows_per_s * Lk, 1),
        "roofline": roofline,
    }

    # ------------------------------------------------------------------ CPU oracle baseline
    if not args.no_cpu:
        import oracle
        oracle.load()
        oracle.softmax(x_host[:1, :1], table[:1], band, threads=ncpu)     # page in, spin up threads
        c0 = time.perf_counter()
        want, rc = oracle.softmax(x_host, table, band, threads=ncpu)
        c1 = time.perf_counter()
        assert rc == 0
        same = all(bool(np.array_equal(o.cpu().numpy(), want)) for o in outs)   # every buffer set, every element
        # about 1.5 s of wall time on all cores (the sample), then a slice of the batch on one thread
        reps = max(1, min(64, int(1.5 / max(c1 - c0, 1e-4))))
        c0 = time.perf_counter()
        for _ in range(reps):
            oracle.softmax(x_host, table, band, threads=ncpu)
        c1 = time.perf_counter()
        part = x_host[:1, :2]                                            # 2 of the 64 (batch, head) slabs
        prow = part.shape[0] * part.shape[1] * part.shape[2]
        s0 = time.perf_counter()
        oracle.softmax(part, table[:2], band, threads=1)
        s1 = time.perf_counter()
        reps1 = max(1, min(64, int(2.0 / max(s1 - s0, 1e-4))))
        s0 = time.perf_counter()
        for _ in range(reps1):
            oracle.softmax(part, table[:2], band, threads=1)
        s1 = time.perf_counter()
        result["cpu_baseline"] = {"value": round(rows * reps / (c1 - c0), 1), "unit": "rows/s", "cores": ncpu,
                                  "kind": "oracle",
                                  "sample": f"the whole {name} batch ({rows} rows of {Lk}) {reps} time(s) on {ncpu} "
                                            f"threads ({c1 - c0:.2f} s), then {prow} rows of it {reps1} time(s) on one "
                                            f"thread ({s1 - s0:.2f} s)",
                                  "single_thread_rows_per_s": round(prow * reps1 / (s1 - s0), 1),
                                  "gpu_output_equals_oracle": same}
        del want

    if not args.no_extras:
        rooflines = {name: {k: v for k, v in roofline.items() if k not in ("how", "traffic")}}
        del xs, outs, loop, x0
        torch.cuda.empty_cache()

        def timed_graphs(launches, per, total, warm=None):
            lp = GraphLoop(torch, launches, per)
            lp.run(2 * per if warm is None else warm)
            _, pr = lp.time(total)
            return launch_ms(pr)[0]

        # ---- the other stand-alone workloads, same launch path
        for other in ("pr1_ref", "edge_encoder", "stress_rows", "ragged_rows"):
            wo = rows_workload(other)
            xh = wo["logits"]
            nb = 2 * xh.size
            sets = max(2, min(32, -(-6 * MALL_BYTES // nb)))
            xi = [torch.from_numpy(xh).to(dev)]
            xi += [xi[0].clone() for _ in range(sets - 1)]
            oi = [torch.empty_like(xi[0], dtype=torch.uint8) for _ in range(sets)]
            per = 128 if nb < (256 << 20) else 32
            ms = timed_graphs([binding.prepare_softmax(xi[i], oi[i], wo["table"], wo["band"]) for i in range(sets)],
                              per, 16 * per if per == 128 else 4 * per)
            r = xh.shape[0] * xh.shape[1] * xh.shape[2]
            rooflines[other] = hbm_roofline(nb, ms, ROW_KERNELS[other],
                                            {"shape": list(xh.shape), "rows_per_s": round(r / (ms * 1e-3), 1),
                                             "traffic": counter_traffic(other)})
            if other == "edge_encoder":
                # same batch: exact exponential in float32, a plain copy, and the other output modes
                H2 = xh.shape[1]
                ms = timed_graphs([(lambda i=i: binding.exp_softmax_i8_f32(xi[i], [0.125] * H2, out=oi[i]))
                                   for i in range(sets)], per, 4 * per)
                result["exp_softmax_f32"] = {"avg_launch_ms": round(ms, 5), "GBps": round(nb / (ms * 1e-3) / 1e9, 1),
                                             "note": "same-run exact-exp float32 softmax on the edge-encoder batch, "
                                                     "same bytes, not parity-checked"}
                ms = timed_graphs([(lambda i=i: binding.copy_bytes(xi[i], oi[i])) for i in range(sets)], per, 4 * per)
                result["copy_kernel"] = {"avg_launch_ms": round(ms, 5), "GBps": round(nb / (ms * 1e-3) / 1e9, 1),
                                         "frac_of_hbm_peak": round(nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                         "note": "plain 16-byte-per-lane copy of the edge-encoder buffers"}
                modes = {}
                o16 = [torch.empty(xi[0].shape, dtype=torch.int16, device=dev) for _ in range(sets)]
                for label, T, recip in (("i16_exact", 32767, 0), ("u8_leading_bit", 255, 1),
                                        ("i16_leading_bit", 32767, 1)):
                    dst = o16 if T == 32767 else oi
                    ms = timed_graphs([(lambda i=i: binding.calibrated_softmax_i8_ex(
                        xi[i], wo["table"], wo["band"], out_scale_T=T, reciprocal=recip, out=dst[i]))
                        for i in range(sets)], per, 4 * per)
                    mb = xh.size * (3 if T == 32767 else 2)
                    modes[label] = hbm_roofline(mb, ms, f"hccs_rows_kernel mode {label}",
                                                {"rows_per_s": round(r / (ms * 1e-3), 1)})
                result["other_modes"] = modes
                del o16
            del xi, oi
            torch.cuda.empty_cache()

        # ---- fused int8 attention block (resident kernels): the 256-token shape, and a vision encoder's 197 tokens
        for label, shape, kernel in (("fused_attention", None, "hccs_attention_direct_kernel<16,0,8,false,false>"),
                                     ("fused_attention_197", (64, 12, 197, 64), "hccs_attention_direct_kernel<16,0,8,true,false>"),
                                     ("fused_attention_577", (64, 12, 577, 64), "hccs_attention_direct_kernel<40,0,8,true,false>")):
            a = synth.make_workload("fused_attention", shape=shape)
            sets = 18 if label != "fused_attention_577" else 8   # 1.5 GB of inputs and outputs: six times the memory-side cache
            q, k, v = ([torch.from_numpy(a[t]).to(dev).clone() for _ in range(sets)] for t in ("q", "k", "v"))
            o = [torch.empty(a["q"].shape, dtype=torch.int32, device=dev) for _ in range(sets)]
            ms = timed_graphs([binding.prepare_attention(q[i], k[i], v[i], o[i], a["table"], a["requant"], a["band"])
                               for i in range(sets)], 32, 512, warm=512)   # ~10 ms of launches before the timed ones
            Ba, Ha, La, da = a["q"].shape
            ops = 2 * (2 * Ba * Ha * La * La * da)
            nb = 3 * a["q"].size + 4 * a["q"].size
            t = ms * 1e-3
            rooflines[label] = hbm_roofline(
                nb, ms, kernel,
                {"shape": [Ba, Ha, La, da], "logit_rows_per_s": round(Ba * Ha * La / t, 1),
                 "algorithmic_int8_ops_per_launch": ops, "int8_TOPs": round(ops / t / 1e12, 2),
                 "mfma_utilisation": round(ops / t / 1e12 / INT8_MFMA_PEAK_TOPS, 4),
                 "note": "one round of 768 blocks: loads, then arithmetic bound by vector-instruction issue (requantisation "
                         "and HCCS stage; the matrix unit carries only the two contractions), then the last tile's stores"
                         + {"fused_attention": "", "fused_attention_197": "; 13 of the 16 query tiles and 197 of the 256 key slots of a block exist",
                            "fused_attention_577": "; 37 of the 40 query tiles and 577 of the 640 key slots of a block exist, one block per "
                                                   "compute unit, three rounds"}[label]})
            del q, k, v, o
            torch.cuda.empty_cache()

        # ---- streaming fused block: keys beyond what a query tile can hold as 16-bit pairs
        (Bs, Hs, Ls, ds), launch = streaming_case()
        ms = timed_graphs([launch], 8, 64, warm=96)   # ~7 ms of launches before the timed ones
        t = ms * 1e-3
        ops = 2 * (2 * Bs * Hs * Ls * Ls * ds)
        rooflines["fused_attention_streaming"] = {
            "bound": "mfma", "achieved": round(ops / t / 1e12, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
            "frac": round(ops / t / 1e12 / INT8_MFMA_PEAK_TOPS, 4), "kernel": "hccs_attention_stream2_kernel<16,1,0,2,true,2,false>",
            "algorithmic_int8_ops_per_launch": ops, "avg_launch_ms": round(ms, 5), "shape": [Bs, Hs, Ls, Ls, ds],
            "logit_rows_per_s": round(Bs * Hs * Ls / t, 1),
            "note": "K/V streamed through LDS in chunks; up to 2048 keys the logits stay in registers as bytes "
                    "(2 passes), beyond that Q.K^T is recomputed (3 passes); vector-issue bound"}
        result["rooflines"] = rooflines

        # ---- offline calibration by grid search on 64 batches of the edge-encoder workload (Sec. III-C, V-A)
        calib_x = torch.from_numpy(synth.make_workload("edge_encoder", threads=ncpu, shape=(64, 8, 128, 128))
                                   ["logits"]).to(dev)
        gcal = np.random.default_rng(0)
        cand = np.stack([gcal.integers(2, 256, 4096), gcal.integers(0, 4, 4096), gcal.integers(1, 128, 4096)], 1)
        alphas = [0.05 + 0.02 * h for h in range(8)]
        binding.calibrate_grid(calib_x, alphas, cand)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        obj, best = binding.calibrate_grid(calib_x, alphas, cand)
        torch.cuda.synchronize()
        c1 = time.perf_counter()
        result["calibration_grid_search"] = {"logits": list(calib_x.shape), "candidates": int(cand.shape[0]),
                                             "wall_ms": round((c1 - c0) * 1e3, 3),
                                             "admissible": int(torch.isfinite(obj[0]).sum()),
                                             "note": "mean KL(softmax || HCCS) in the 16-bit space per head and "
                                                     "candidate, arg-min per head; includes the binding's allocations"}
        result["paper_context"] = ("paper, AIE-ML/AIE-MLv2 cycle-accurate simulator, one tile, n=128: HCCS i8+CLB "
                                   "2.18-2.21 G elem/s; 184 tiles extrapolated 407 G elem/s (Tab. III, Sec. V-D); "
                                   "different hardware, context only")

    print(json.dumps(result))


if __name__ == "__main__":
    main()
