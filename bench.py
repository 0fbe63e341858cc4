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


def algorithmic_bytes_per_prefix_step(V: int, elem: int, n_children: float, depth: float, stride_read: float) -> float:
    """What one row of one decode step has to move through HBM: the logits row once, the children
    tokens of the reached prefix (4 bytes each) or at most a V-bit image, one 128-byte line per
    level of the walk for each of the three per-depth arrays it touches, the prefix itself, and
    the few scalars written back.  The mask stays on chip in the fused step."""
    return V * elem + min(4.0 * n_children, V / 8.0) + 3 * 128.0 * depth + 4.0 * stride_read + 24.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C3", choices=["C3"])
    ap.add_argument("--n-seq", type=int, default=0, help="override |S| (debugging only; invalidates the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--verbose", action="store_true", help="per-decode-step table on stderr")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); the path is data-parallel "
              "over rows with a replicated index and needs no collective, see DESIGN.md", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2504_09135_amd import binding as ppv
    from paper_2504_09135_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    dev = "cuda:0"
    cfg = W.CONFIGS[args.config]
    if args.n_seq:
        cfg = W.scaled(cfg, args.n_seq)
    B, V = cfg.batch, cfg.vocab

    t0 = time.perf_counter()
    S = W.make_constraint_set(cfg)
    t_gen = time.perf_counter() - t0
    t0 = time.perf_counter()
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t0
    L = index.l_max

    # every decode step's logits and uniforms, resident in HBM before anything is timed
    logits = torch.empty((L, B, V), dtype=torch.bfloat16, device=dev)
    uniforms = torch.empty((L, B), dtype=torch.float32, device=dev)
    for s in range(L):
        logits[s] = torch.from_numpy(W.make_logits(cfg, step=s).view(np.int16)).to(dev).view(torch.bfloat16)
        uniforms[s] = torch.from_numpy(W.make_uniforms(cfg, step=s)).to(dev)

    reps = args.warmup + args.steps + 1                    # +1: the pass that times single launches
    prefixes = torch.full((reps, B, L), W.PAD_TOKEN, dtype=torch.int32, device=dev)
    lens = torch.zeros((reps, B), dtype=torch.int32, device=dev)
    active = torch.ones((reps, B), dtype=torch.uint8, device=dev)
    logx = torch.zeros((reps, B), dtype=torch.float32, device=dev)
    ids = torch.zeros((B,), dtype=torch.int32, device=dev)
    lz = torch.zeros((B,), dtype=torch.float32, device=dev)

    def loop(r: int, events=None):
        for s in range(L):
            if events is not None:
                events[s][0].record()
            ppv.ppv_decode_step(index, prefixes[r], lens[r], active[r], logits[s], uniforms[s], ids, lz, logx[r])
            if events is not None:
                events[s][1].record()

    for r in range(args.warmup):
        loop(r)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for r in range(args.warmup, args.warmup + args.steps):
        loop(r)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # ---- what was processed
    final_lens = lens[args.warmup].cpu().numpy().astype(np.int64)
    assert not active[args.warmup:args.warmup + args.steps].any().item(), "a row did not finish"
    assert (lens[args.warmup:args.warmup + args.steps] == lens[args.warmup]).all().item(), "loops differ"
    prefix_steps = int(final_lens.sum())                   # row x decode-step pairs per loop
    active_per_step = np.array([(final_lens > s).sum() for s in range(L)], dtype=np.int64)
    ms_per_step = elapsed / args.steps * 1e3
    value = prefix_steps * args.steps / elapsed

    # ---- dominant kernel: average launch duration by HIP events around every launch of one more loop
    r = reps - 1
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(L)]
    loop(r, events)
    torch.cuda.synchronize()
    dur_ms = np.array([a.elapsed_time(b) for a, b in events])
    # algorithmic bytes: per row of step s the reached prefix has depth s; its child count comes from the run
    seqs = prefixes[args.warmup].cpu().numpy()
    fan = fanout_along(index, ppv, torch, seqs, final_lens, L, dev)             # [L] mean children of the prefixes reached at step s
    bytes_per_launch = np.array([
        active_per_step[s] * algorithmic_bytes_per_prefix_step(V, 2, fan[s], s, s) for s in range(L)])
    if args.verbose:
        for s_ in range(L):
            print(f"step {s_:2d} active {active_per_step[s_]:4d} fanout {fan[s_]:9.1f} launch {dur_ms[s_] * 1e3:8.2f} us "
                  f"{bytes_per_launch[s_] / max(dur_ms[s_], 1e-9) / 1e6:8.1f} GB/s", file=sys.stderr)
    launches = int((active_per_step > 0).sum())
    busy = active_per_step > 0
    achieved = float(bytes_per_launch[busy].sum() / (dur_ms[busy].sum() * 1e-3) / 1e9)
    roofline = {"bound": "hbm", "kernel": "decode_step_kernel<bf16>", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "avg_launch_us": round(float(dur_ms[busy].mean() * 1e3), 2), "launches_per_step": launches,
                "bytes_per_launch_avg": int(bytes_per_launch[busy].mean()),
                "first_launch_us": round(float(dur_ms[0] * 1e3), 2),
                "first_launch_GBs": round(float(bytes_per_launch[0] / (dur_ms[0] * 1e-3) / 1e9), 1)}

    out = {
        "metric": "constrained decode steps (prefixes)/sec at N=1M, V=32k", "value": round(value, 1),
        "unit": "prefix-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 logits, f32/f64 accumulate, u32 index", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: |S|={index.n_distinct} lengths U[4,32] Zipf(1.1) V={V}; full decode loop, "
                               f"B={B} rows from the empty prefix, {L} fused step launches per loop, "
                               f"{prefix_steps} prefix-steps per loop",
                   "launch": "one ppv_decode_step per decode step via the C ABI, no host sync inside a loop"},
        "roofline": roofline,
        "index_build_s": round(t_build, 3), "index_device_MB": round(index.device_bytes / 1e6, 1),
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, S, B, seqs, final_lens)
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


def cpu_baseline(cfg, S, B, gpu_seqs, gpu_lens):
    """The CPU oracle (never tuned for this) on the same decode loop, on this machine's cores."""
    import numpy as np
    import oracle
    from paper_2504_09135_amd import workloads as W
    threads = oracle.max_threads()
    trie = oracle.Trie(S.tokens, S.offsets, cfg.vocab)
    rows = B
    lg = lambda s, *_: W.logits_as_f32(cfg, W.make_logits(cfg, step=s))[:rows]
    un = lambda s: W.make_uniforms(cfg, step=s)[:rows]
    # pre-generate outside the timed region, like the GPU side
    cache_l, cache_u = {}, {}
    for s in range(trie.l_max):
        cache_l[s], cache_u[s] = lg(s), un(s)
    t0 = time.perf_counter()
    res = oracle.decode_loop(trie, rows, lambda s, *_: cache_l[s], lambda s: cache_u[s], threads=threads)
    dt = time.perf_counter() - t0
    steps = int(res.lens.sum())
    same = int(sum(np.array_equal(res.seqs[b, :res.lens[b]], gpu_seqs[b, :gpu_lens[b]]) for b in range(rows)))
    return {"value": round(steps / dt, 1), "unit": "prefix-steps/s", "cores": threads, "kind": "oracle",
            "sample": f"the same full decode loop, all {rows} rows ({steps} prefix-steps, {dt:.1f} s), "
                      f"OpenMP over rows; trie build excluded; {same}/{rows} rows end on the GPU's sequence"}


if __name__ == "__main__":
    sys.exit(main())
