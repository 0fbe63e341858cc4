#!/usr/bin/env python3
"""Benchmark of the PPV + fused masked-sampling hot path on one MI355X.

Default workload: the N = 1M, V = 32k configuration (C3) -- the full constrained decode loop of
Algorithm 1's SampleCandidate for B = 256 rows that start from the empty prefix and extend by
their sampled token until they are members of S.  One benchmark "step" is one whole loop: l_max
fused decode-step launches through the C ABI, every launch streaming that decode step's own
pre-generated bf16 logits [256, 32000] (distinct buffers per decode step, already resident in HBM).
`value` = prefix-steps (row x decode-step pairs that were actually processed) per second.

Prints ONE JSON line.  `roofline` is for the dominant kernel (the fused decode step): algorithmic
bytes per launch / average launch duration measured with HIP events on the launch stream.
`cpu_baseline` is the CPU oracle timed on this machine's host cores on the same loop.
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

HBM_PEAK_GBS = 8000.0  # MI355X published peak HBM3E bandwidth

# HBM bytes per launch of the dominant kernel from rocprofv3 counter runs (FETCH_SIZE + WRITE_SIZE, each
# scaled by what the same counter reads for a plain copy of known size); see profiles/.  Keyed by
# (workload, batch); None until measured for that shape.
TRAFFIC_BYTES_PER_LAUNCH = {
    ("C3", 256): (9819569, "profiles/decode_kernel_C3_B256.md: FETCH_SIZE + WRITE_SIZE of the per-step decode_kernel, "
                           "mean over the 32 launches of a loop, copy-calibrated"),
    ("C5", 1024): (529872422, "profiles/mask_sample_kernels_C5.md: FETCH_SIZE + WRITE_SIZE of the one-call kernel, "
                              "copy-calibrated"),
}


def algorithmic_bytes_per_prefix_step(V: int, elem: int, n_children: float) -> float:
    """What one row of one fused decode step has to move through HBM: the logits row once; the
    valid set, either the children's entries (8 bytes each, plus the one that closes them) or, for a
    heavy prefix, its V-bit image plus three 128-byte lines to find the sampled child; and about 96
    bytes of per-row state, scalars and the appended token.  The mask never leaves the chip here."""
    return V * elem + min(8.0 * (n_children + 1.0), V / 8.0 + 384.0) + 96.0


class LoopBench:
    """The decode loop of one batch: buffers, the eager loop and its HIP graph."""

    def __init__(self, torch, ppv, W, index, logits, uniforms, use_graph=True):
        self.torch, self.ppv, self.index = torch, ppv, index
        L, B, V = logits.shape
        self.L, self.B, self.V = L, B, V
        dev = logits.device
        self.prefixes = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=dev)
        self.lens = torch.zeros((B,), dtype=torch.int32, device=dev)
        self.active = torch.zeros((B,), dtype=torch.uint8, device=dev)
        self.state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=dev)
        self.logx = torch.zeros((B,), dtype=torch.float32, device=dev)
        self.ids = torch.zeros((B,), dtype=torch.int32, device=dev)
        self.lz = torch.zeros((B,), dtype=torch.float32, device=dev)
        self.logits, self.uniforms = logits, uniforms
        self.step_logits = [logits[s] for s in range(L)]
        self.step_uniforms = [uniforms[s] for s in range(L)]
        self.loop()                                            # eager once: loads the kernels
        torch.cuda.synchronize()
        self.graph = None
        if use_graph:
            # the launch-bound inner loop is captured once in a HIP graph and replayed
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                self.loop()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            # (captured on the stream that has just run the loop: a stream under capture cannot allocate, and the
            # library keeps per-stream scratch for rows it spreads over several workgroups)
            self.graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(self.graph, stream=side):
                self.loop()
        self.run = self.graph.replay if self.graph is not None else self.loop

    def loop(self, events=None):
        """One whole decode loop: start from the empty prefix, then l_max fused step launches."""
        ppv = self.ppv
        for s in range(self.L):
            if events is not None:
                events[s][0].record()
            # the first step starts every row from the empty candidate (a = [], x = 1) in the same launch
            step = ppv.ppv_decode_first_step if s == 0 else ppv.ppv_decode_step
            step(self.index, self.prefixes, self.lens, self.active, self.step_logits[s],
                 self.step_uniforms[s], self.ids, self.lz, self.logx, state=self.state)
            if events is not None:
                events[s][1].record()

    def single_launch(self):
        """The same loop as ONE ppv_decode_loop launch (possible here because every step's logits are resident up front)."""
        ppv = self.ppv
        ppv.ppv_decode_begin_empty(self.index, self.lens, self.state, self.active, self.logx)
        ppv.ppv_decode_loop(self.index, self.prefixes, self.lens, self.active, self.logits, self.uniforms, None, None,
                            self.logx, state=self.state)

    def time(self, warmup, steps, single_launch=False):
        """Wall-clock seconds of `steps` loops (synchronised on both sides), the same region in GPU time
        by HIP events on the launch stream, and the rows' final lengths."""
        torch = self.torch
        run = self.single_launch if single_launch else self.run
        for _ in range(warmup):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            run()
        e1.record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        self.gpu_seconds = e0.elapsed_time(e1) * 1e-3
        assert not self.active.any().item(), "a row did not finish"
        final_lens = self.lens.cpu().numpy().astype("int64")
        return elapsed, final_lens

    def saturated_launch_seconds(self, reps=5):
        """GPU seconds of the launch of decode step 3 alone (every row still active: no member of S is shorter than 4
        tokens), as the difference between two captured graphs, begin + steps 0..3 and begin + steps 0..2."""
        torch, ppv = self.torch, self.ppv

        def partial(n):
            for s in range(n):
                step = ppv.ppv_decode_first_step if s == 0 else ppv.ppv_decode_step
                step(self.index, self.prefixes, self.lens, self.active, self.step_logits[s],
                     self.step_uniforms[s], self.ids, self.lz, self.logx, state=self.state)

        times = []
        for n in (3, 4):
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                partial(n)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                partial(n)
            graph.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                graph.replay()
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e-3 / reps)
        return max(times[1] - times[0], 1e-9)

    def per_loop_ms(self, n):
        """GPU milliseconds of n single loops, each between its own pair of HIP events."""
        import numpy as np
        torch = self.torch
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        self.run()
        torch.cuda.synchronize()
        for a, b in ev:
            a.record()
            self.run()
            b.record()
        torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) for a, b in ev])

    def launch_durations(self, loops=5):
        """Average duration of each of the L step launches: HIP events around every eager launch on the
        launch stream; two graph replays run ahead each time so that the GPU is busy and clocked up."""
        import numpy as np
        torch = self.torch
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(self.L)]
        dur_ms = np.zeros(self.L)
        for _ in range(loops):
            self.run()
            self.run()
            self.loop(events)
            torch.cuda.synchronize()
            dur_ms += np.array([a.elapsed_time(b) for a, b in events]) / loops
        return dur_ms


def measured_copy_bandwidth(torch, dev, n_bytes=1 << 30, reps=5):
    """What a plain device-to-device copy reaches on this machine (bytes read + bytes written per second), GB/s:
    the practical roof beside the published 8 TB/s."""
    src = torch.empty(n_bytes // 4, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return round(2.0 * n_bytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C3", choices=["C1", "C2", "C3", "C4", "C5"],
                    help="C3 (default): the N=1M, V=32k decode loop the metric is quoted on; C1/C2/C4/C5: one "
                         "ppv_next_token_mask + constrained_sample call on that config's batch")
    ap.add_argument("--n-seq", type=int, default=0, help="override |S| (debugging only; invalidates the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch every decode step eagerly from Python")
    ap.add_argument("--no-sweep", action="store_true", help="skip the batch sweep (B = 1024, 4096 replicas)")
    ap.add_argument("--verbose", action="store_true", help="per-decode-step table on stderr")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy a few times (reference for the HBM counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); the path is data-parallel "
              "over rows with a replicated index and needs no collective", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2504_09135_amd import binding as ppv
    from paper_2504_09135_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    dev = "cuda:0"
    if args.copy_calibration:
        n = 256 << 20
        src = torch.full((n // 4,), 1.0, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1.0, out=dst)                       # one elementwise kernel: reads n bytes, writes n bytes
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "launches": 5}))
        return 0
    cfg = W.CONFIGS[args.config]
    if args.n_seq:
        cfg = W.scaled(cfg, args.n_seq)
    B, V = cfg.batch, cfg.vocab
    if not cfg.loop:
        return single_call_bench(args, cfg, torch, ppv, W, dev)

    S = W.make_constraint_set(cfg)
    t0 = time.perf_counter()
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t0
    L = index.l_max
    import tempfile
    with tempfile.TemporaryDirectory() as td:                  # persistence: written once, loaded instead of rebuilt
        t0 = time.perf_counter()
        ppv.ppv_index_save(index, os.path.join(td, "index.ppv"))
        t_save = time.perf_counter() - t0
        t0 = time.perf_counter()
        ppv.ppv_index_load(os.path.join(td, "index.ppv")).free()
        t_load = time.perf_counter() - t0

    # every decode step's logits and uniforms, resident in HBM before anything is timed
    logits = torch.empty((L, B, V), dtype=torch.bfloat16, device=dev)
    uniforms = torch.empty((L, B), dtype=torch.float32, device=dev)
    for s in range(L):
        logits[s] = torch.from_numpy(W.make_logits(cfg, step=s).view(np.int16)).to(dev).view(torch.bfloat16)
        uniforms[s] = torch.from_numpy(W.make_uniforms(cfg, step=s)).to(dev)

    lb = LoopBench(torch, ppv, W, index, logits, uniforms, use_graph=not args.no_graph)
    elapsed, final_lens = lb.time(args.warmup, args.steps)
    prefix_steps = int(final_lens.sum())                       # row x decode-step pairs per loop
    active_per_step = np.array([(final_lens > s).sum() for s in range(L)], dtype=np.int64)
    ms_per_step = elapsed / args.steps * 1e3
    value = prefix_steps * args.steps / elapsed
    per_loop_ms = lb.per_loop_ms(min(args.steps, 30))         # spread of single loops (HIP events around each)
    copy_gbs = measured_copy_bandwidth(torch, dev)

    # ---- dominant kernel (the fused decode step): algorithmic bytes per launch / average launch duration.
    # Average duration = GPU time of the timed region (HIP events on the launch stream) / launches in it;
    # (the first launch of a loop is ppv_decode_first_step, which also starts the rows)
    gpu_seconds = lb.gpu_seconds
    dur_ms = lb.launch_durations() if args.verbose else None
    seqs = lb.prefixes.cpu().numpy()
    fan = fanout_along(index, ppv, torch, seqs, final_lens, L, dev)  # mean children of the prefixes reached at step s
    bytes_per_launch = np.array([active_per_step[s] * algorithmic_bytes_per_prefix_step(V, 2, fan[s]) for s in range(L)])
    if args.verbose:
        print("per-launch figures below are eager launches with an event pair around each (a few us of event "
              "overhead included)", file=sys.stderr)
        for s_ in range(L):
            print(f"step {s_:2d} active {active_per_step[s_]:4d} fanout {fan[s_]:9.1f} launch {dur_ms[s_] * 1e3:8.2f} us "
                  f"{bytes_per_launch[s_] / max(dur_ms[s_], 1e-9) / 1e6:8.1f} GB/s", file=sys.stderr)
    n_launch = L                                               # every loop launches all l_max steps
    avg_launch_s = gpu_seconds / (args.steps * n_launch)
    bytes_per_launch_avg = float(bytes_per_launch.sum() / n_launch)
    achieved = bytes_per_launch_avg / avg_launch_s / 1e9
    roofline = {"bound": "hbm", "kernel": "decode_kernel<bf16, per-step>", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": TRAFFIC_BYTES_PER_LAUNCH.get((cfg.name, B), (None, None))[0],
                "traffic_source": TRAFFIC_BYTES_PER_LAUNCH.get((cfg.name, B), (None, "not measured for this shape"))[1],
                "avg_launch_us": round(avg_launch_s * 1e6, 2), "launches_per_step": n_launch,
                "bytes_per_launch": int(bytes_per_launch_avg),
                "rows_per_launch_avg": round(float(active_per_step.mean()), 1),
                "device_copy_GBs": copy_gbs}

    out = {
        "metric": "constrained decode steps (prefixes)/sec at N=1M, V=32k", "value": round(value, 1),
        "unit": "prefix-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(float(np.median(per_loop_ms)), 4),
        "ms_per_step_min": round(float(per_loop_ms.min()), 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 logits, f32/f64 accumulate, u32 index", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: |S|={index.n_distinct} lengths U[4,32] Zipf(1.1) V={V}; full decode loop, "
                               f"B={B} rows from the empty prefix, {L} fused step launches per loop, "
                               f"{prefix_steps} prefix-steps per loop",
                   "launch": ("one ppv_decode_step per decode step through the C ABI (the first one ppv_decode_first_step, which starts the rows from the empty prefix), " +
                              ("captured once in a HIP graph and replayed" if lb.graph is not None else "launched eagerly") +
                              ", no host sync inside a loop")},
        "roofline": roofline,
        "index_build_s": round(t_build, 3), "index_device_MB": round(index.device_bytes / 1e6, 1),
        "index_save_s": round(t_save, 3), "index_load_s": round(t_load, 3),
    }

    # The same loop, same rows, as one launch (ppv_decode_loop): every workgroup stays with its row, so there
    # is no launch boundary between decode steps.  Only possible because the logits of all steps are resident up
    # front; with a model between the steps the per-step launch above is the real path.
    ref_seqs, ref_lens = lb.prefixes.clone(), lb.lens.clone()
    el1, fl1 = lb.time(args.warmup, args.steps, single_launch=True)
    assert torch.equal(lb.prefixes, ref_seqs) and torch.equal(lb.lens, ref_lens), "single-launch loop differs"
    out["single_launch_loop"] = {"prefix_steps_per_s": round(prefix_steps * args.steps / el1, 1),
                                 "ms_per_loop": round(el1 / args.steps * 1e3, 4),
                                 "GBs": round(float(bytes_per_launch.sum()) * args.steps / el1 / 1e9, 1),
                                 "frac_of_peak": round(float(bytes_per_launch.sum()) * args.steps / el1 / 1e9 / HBM_PEAK_GBS, 4)}

    if not args.no_graph:
        # one launch of the timed kernel with all B rows active (decode step 3), beside the loop's average launch
        sat = lb.saturated_launch_seconds(reps=20)
        bps1 = algorithmic_bytes_per_prefix_step(V, 2, 1.0)
        out["roofline"]["launch_all_rows_active"] = {"us": round(sat * 1e6, 2), "GBs": round(B * bps1 / sat / 1e9, 1),
                                                     "frac_of_peak": round(B * bps1 / sat / 1e9 / HBM_PEAK_GBS, 4)}

    if not args.no_sweep:
        # Same loop with R replicas of the batch (logits drawn on the device: same distribution, not
        # checked against the oracle) to show where the kernel goes once the launch is large enough.
        out["batch_sweep"] = []
        del lb
        for Bs in (1024, 4096, 16384):
            g = torch.Generator(device=dev)
            g.manual_seed(cfg.seed + Bs)
            lg = torch.empty((L, Bs, V), dtype=torch.bfloat16, device=dev)
            for s in range(L):
                lg[s] = (torch.randn((Bs, V), generator=g, device=dev, dtype=torch.float32) * cfg.sigma).to(torch.bfloat16)
            un = torch.rand((L, Bs), generator=g, device=dev, dtype=torch.float32)
            sb = LoopBench(torch, ppv, W, index, lg, un, use_graph=not args.no_graph)
            el, fl = sb.time(2, 10)
            ps = int(fl.sum())
            el1, _ = sb.time(2, 10, single_launch=True)
            bps = algorithmic_bytes_per_prefix_step(V, 2, 1.0)
            sat = sb.saturated_launch_seconds() if not args.no_graph else None
            out["batch_sweep"].append({"B": Bs, "prefix_steps_per_s": round(ps * 10 / el, 1),
                                       "GBs": round(ps * bps * 10 / el / 1e9, 1),
                                       "frac_of_peak": round(ps * bps * 10 / el / 1e9 / HBM_PEAK_GBS, 4),
                                       "single_launch_prefix_steps_per_s": round(ps * 10 / el1, 1),
                                       "single_launch_GBs": round(ps * bps * 10 / el1 / 1e9, 1),
                                       # one launch with every row still active (decode step 3: no member is shorter
                                       # than 4 tokens), the loop's own figure being an average over launches that
                                       # get sparser as rows retire
                                       "launch_all_rows_active": None if sat is None else {
                                           "us": round(sat * 1e6, 2), "GBs": round(Bs * bps / sat / 1e9, 1),
                                           "frac_of_peak": round(Bs * bps / sat / 1e9 / HBM_PEAK_GBS, 4)}})
            del sb, lg, un

    if not args.no_sweep:
        out["topm_sweep"] = topm_sweep(cfg, S, index, logits[0], torch, ppv, W, dev)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, S, B, seqs, final_lens)
    print(json.dumps(out))
    return 0


def topm_sweep(cfg, S, index, logits0, torch, ppv, W, dev, reps=40):
    """Algorithm 2 with M candidates (ppv_topm_mask) against the full-vocabulary mask (ppv_next_token_mask) on
    the config's prefix batch: microseconds per call, HIP events on the launch stream."""
    pb = W.make_prefix_batch(cfg, S)
    B = pb.prefixes.shape[0]
    P, Ln = torch.from_numpy(pb.prefixes).to(dev), torch.from_numpy(pb.lens).to(dev)
    mask = torch.zeros((B, index.n_words), dtype=torch.int32, device=dev)

    def us_per_call(fn):
        # `reps` calls captured in one HIP graph: the figure is GPU time per call (launch gaps included), not the
        # rate at which Python can issue calls
        fn()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(reps):
                fn()
        graph.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        graph.replay()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        return round(e0.elapsed_time(e1) * 1e3 / (2 * reps), 2)

    res = {"B": B, "full_mask_us": us_per_call(lambda: ppv.ppv_next_token_mask(index, P, Ln, mask)), "topm_us": {}}
    for M in (50, 100, 500, 1000):
        res["topm_us"][str(M)] = us_per_call(lambda: ppv.ppv_topm_mask(index, P, Ln, logits0, M, mask))
    return res


def single_call_bench(args, cfg, torch, ppv, W, dev):
    """C2 / C4 / C5: the two-call path (mask, then sample) on the config's own batch.  A step = one mask call +
    one sample call over the batch; the logits of every timed step are a fresh buffer resident in HBM."""
    import numpy as np
    B, V = cfg.batch, cfg.vocab
    e = 2 if cfg.dtype == "bf16" else 4
    S = W.make_constraint_set(cfg)
    t0 = time.perf_counter()
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t0
    pb = W.make_prefix_batch(cfg, S)
    P, Ln = torch.from_numpy(pb.prefixes).to(dev), torch.from_numpy(pb.lens).to(dev)
    host_logits = W.make_logits(cfg)
    first = (torch.from_numpy(host_logits.view(np.int16)).to(dev).view(torch.bfloat16) if cfg.dtype == "bf16"
             else torch.from_numpy(host_logits).to(dev))
    n_buf = max(2, min(args.steps, int(3e9 // (B * V * e))))            # distinct buffers so that steps stream cold data
    g = torch.Generator(device=dev)
    g.manual_seed(cfg.seed)
    bufs = [first]
    for _ in range(n_buf - 1):
        x = torch.randn((B, V), generator=g, device=dev, dtype=torch.float32) * cfg.sigma
        bufs.append(x.to(torch.bfloat16) if cfg.dtype == "bf16" else x)
    un = torch.from_numpy(W.make_uniforms(cfg)).to(dev)
    mask = torch.zeros((B, index.n_words), dtype=torch.int32, device=dev)
    lo = torch.zeros(B, dtype=torch.int32, device=dev)
    hi = torch.zeros_like(lo)
    mem = torch.zeros(B, dtype=torch.uint8, device=dev)
    ids = torch.zeros(B, dtype=torch.int32, device=dev)
    lz = torch.zeros(B, dtype=torch.float32, device=dev)

    def step(k):
        ppv.ppv_next_token_mask(index, P, Ln, mask, lo, hi, mem)
        ppv.constrained_sample(bufs[k % n_buf], mask, un, ids, lz)

    def region(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for k in range(n):
            fn(k)
        e1.record()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, e0.elapsed_time(e1) * 1e-3

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()

    def graph_region(fn, n):
        """(wall seconds, GPU seconds) of n calls captured in one HIP graph and replayed once: the GPU's figure, not
        the rate at which Python issues calls."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for k in range(n):
                fn(k)
        graph.replay()
        return region(lambda k: graph.replay(), 1)

    timed = region if args.no_graph else graph_region
    launch = "launched eagerly" if args.no_graph else f"{args.steps} steps captured in one HIP graph and replayed"

    def fused(k):
        ppv.ppv_sample_next(index, P, Ln, bufs[k % n_buf], un, ids1, lz1)
    ids1, lz1 = torch.zeros_like(ids), torch.zeros_like(lz)
    fused(0)
    torch.cuda.synchronize()
    elapsed2, _ = timed(step, args.steps)                                # mask call + sample call
    _, t_mask = timed(lambda k: ppv.ppv_next_token_mask(index, P, Ln, mask, lo, hi, mem), args.steps)
    _, t_samp = timed(lambda k: ppv.constrained_sample(bufs[k % n_buf], mask, un, ids, lz), args.steps)
    elapsed1, t_fused = timed(fused, args.steps)                         # one call, the mask never written
    step(0)
    fused(0)
    torch.cuda.synchronize()
    n_valid = int((ids >= 0).sum().item())
    same = int((ids == ids1).sum().item())
    # algorithmic bytes: two calls = logits once, mask written and read, scalars; one call = logits once, the
    # children entries (or the heavy prefix's image), scalars
    children = np.unpackbits(mask.cpu().numpy().view(np.uint8), axis=1).sum(axis=1).astype(np.float64)
    bytes_sample = B * (V * e + V / 8.0 + 12.0)
    bytes_two = B * (V * e + 2.0 * V / 8.0 + 96.0)
    bytes_fused = float(sum(algorithmic_bytes_per_prefix_step(V, e, c) for c in children))
    two = {"prefixes_per_s": round(B * args.steps / elapsed2, 1), "us_per_step": round(elapsed2 / args.steps * 1e6, 2),
           "GBs": round(bytes_two / (elapsed2 / args.steps) / 1e9, 1),
           "frac_of_peak": round(bytes_two / (elapsed2 / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
           "mask_us": round(t_mask / args.steps * 1e6, 2), "sample_us": round(t_samp / args.steps * 1e6, 2),
           "sample_GBs": round(bytes_sample / (t_samp / args.steps) / 1e9, 1),
           "mask_GBs_written": round(B * V / 8.0 / (t_mask / args.steps) / 1e9, 1)}
    one = {"prefixes_per_s": round(B * args.steps / elapsed1, 1), "us_per_step": round(elapsed1 / args.steps * 1e6, 2),
           "GBs": round(bytes_fused / (t_fused / args.steps) / 1e9, 1),
           "frac_of_peak": round(bytes_fused / (t_fused / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
           "ids_equal_to_two_calls": f"{same}/{B}"}
    use_fused = elapsed1 <= elapsed2
    elapsed = elapsed1 if use_fused else elapsed2
    one_tile = V <= (1024 if cfg.dtype == "f32" else 2048)
    if use_fused:
        kernel = f"sample_next_one_tile_kernel<{cfg.dtype}>" if one_tile else f"decode_kernel<{cfg.dtype}> (ppv_sample_next)"
        k_bytes, k_time = bytes_fused, t_fused
    else:
        kernel, k_bytes, k_time = f"sample_kernel<{cfg.dtype}>", bytes_sample, t_samp
    achieved = k_bytes / (k_time / args.steps) / 1e9
    out = {
        "metric": f"constrained decode steps (prefixes)/sec on config {cfg.name}", "value": round(B * args.steps / elapsed, 1),
        "unit": "prefixes/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": f"{cfg.dtype} logits, f32/f64 accumulate, u32 index", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: |S|={index.n_distinct} V={V} B={B} ({n_valid} rows with a valid token); " +
                               ("one ppv_sample_next call per step (valid set and sample fused, no mask written), "
                                if use_fused else "one ppv_next_token_mask + one constrained_sample per step, ") + launch},
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": TRAFFIC_BYTES_PER_LAUNCH.get((cfg.name, B), (None, None))[0] if use_fused else None,
                     "traffic_source": (TRAFFIC_BYTES_PER_LAUNCH.get((cfg.name, B), (None, "not measured for this shape"))[1]
                                        if use_fused else "not measured for this pipeline"),
                     "avg_launch_us": round(k_time / args.steps * 1e6, 2), "bytes_per_launch": int(k_bytes),
                     "device_copy_GBs": measured_copy_bandwidth(torch, dev)},
        "pipelines": {"one_call": one, "two_calls": two},
        "index_build_s": round(t_build, 3), "index_device_MB": round(index.device_bytes / 1e6, 1),
    }
    if not args.no_sweep:
        out["topm_sweep"] = topm_sweep(cfg, S, index, bufs[0], torch, ppv, W, dev, reps=10)
    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.max_threads()
        trie = oracle.Trie(S.tokens, S.offsets, V)
        lf = W.logits_as_f32(cfg, host_logits)
        unh = W.make_uniforms(cfg)
        rows = min(B, max(threads, int(4e9 // (V * 40))))               # bounded sample of the batch
        reps, dt = 0, 0.0
        t0 = time.perf_counter()
        while dt < 1.0 and reps < 200:                                  # repeated until about a second of wall time
            ref = trie.step(pb.prefixes[:rows], pb.lens[:rows], lf[:rows], unh[:rows], want_mask=True, threads=threads)
            reps += 1
            dt = time.perf_counter() - t0
        same = int((ref.ids == (ids1 if use_fused else ids)[:rows].cpu().numpy()).sum())
        t0 = time.perf_counter()
        trie.step(pb.prefixes[:rows], pb.lens[:rows], lf[:rows], unh[:rows], want_mask=True, threads=1)
        dt1 = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(rows * reps / dt, 1), "unit": "prefixes/s", "cores": threads, "kind": "oracle",
                               "value_one_thread": round(rows / dt1, 1),
                               "sample": f"the first {rows} rows of the same batch, one mask + step each, {reps} times "
                                         f"({dt:.2f} s wall, about {dt * threads:.0f} core-seconds), OpenMP over rows; "
                                         f"trie build excluded; {same}/{rows} ids equal the GPU's"}
    print(json.dumps(out))
    return 0


def fanout_along(index, ppv, torch, seqs, final_lens, L, dev):
    """Mean number of valid next tokens of the prefixes the rows went through, per decode step
    (bookkeeping for the byte count only, after the timed region: one mask call per step)."""
    import numpy as np
    B = seqs.shape[0]
    out = np.zeros(L)
    P = torch.from_numpy(np.ascontiguousarray(seqs)).to(dev)
    mask = torch.zeros((B, index.n_words), dtype=torch.int32, device=dev)
    for s in range(L):
        on = final_lens > s
        if not on.any():
            break
        ppv.ppv_next_token_mask(index, P, torch.full((B,), s, dtype=torch.int32, device=dev), mask)
        bits = np.unpackbits(mask.cpu().numpy().view(np.uint8), axis=1).sum(axis=1)
        out[s] = bits[on].mean()
    return out


def cpu_baseline(cfg, S, B, gpu_seqs, gpu_lens, repeats=8):
    """The CPU oracle (never tuned for this) on the same decode loop, on this machine's cores."""
    import numpy as np
    import oracle
    from paper_2504_09135_amd import workloads as W
    threads = oracle.max_threads()
    trie = oracle.Trie(S.tokens, S.offsets, cfg.vocab)
    # inputs are generated outside the timed region, like the GPU side's
    cache_l = {s: W.logits_as_f32(cfg, W.make_logits(cfg, step=s)) for s in range(trie.l_max)}
    cache_u = {s: W.make_uniforms(cfg, step=s) for s in range(trie.l_max)}
    t0 = time.perf_counter()
    for _ in range(repeats):
        res = oracle.decode_loop(trie, B, lambda s, *_: cache_l[s], lambda s: cache_u[s], threads=threads)
    dt = time.perf_counter() - t0
    steps = int(res.lens.sum())
    same = int(sum(np.array_equal(res.seqs[b, :res.lens[b]], gpu_seqs[b, :gpu_lens[b]]) for b in range(B)))
    t0 = time.perf_counter()
    oracle.decode_loop(trie, B, lambda s, *_: cache_l[s], lambda s: cache_u[s], threads=1)
    dt1 = time.perf_counter() - t0
    return {"value": round(steps * repeats / dt, 1), "unit": "prefix-steps/s", "cores": threads, "kind": "oracle",
            "value_one_thread": round(steps / dt1, 1),
            "sample": f"the same full decode loop, all {B} rows, {repeats} times ({steps * repeats} prefix-steps, "
                      f"{dt:.1f} s wall, about {dt * threads:.0f} core-seconds), OpenMP over rows; then once on one "
                      f"thread ({dt1:.1f} s); trie build excluded; {same}/{B} rows end on the GPU's sequence"}


if __name__ == "__main__":
    sys.exit(main())
