#!/usr/bin/env python3
"""Benchmark of the paged-attention hot path on one MI355X.

Default workload ("c2"): batched GQA decode, Llama-3-8B layer shape, batch 128, 32/8 heads,
D 128, bf16, page 16, KV lengths Zipf(1.2) over [256, 32768] (seeded synthetic; see
workloads.config2).  One step = one pass of the whole hot path over the batch:
fi_plan (host scheduler + async copy of the plan) -> fi_run (persistent attention launch +
merge launch).  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: metric = achieved HBM bandwidth of the step (algorithmic bytes / step
time), plus `roofline` for the dominant kernel (timed with HIP events recorded by the library
around that kernel on the launch stream, on every --event-stride-th launch of the timed region:
a pair of event records costs the step about 10 us here, which would otherwise be charged to
the step time) and `cpu_baseline` (the fp64 oracle on host cores).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2516.6


class HipEvents:
    """Raw HIP events (the library records them around its attention kernel)."""

    def __init__(self, n: int):
        import torch  # noqa: F401  (torch's HIP runtime is the one in this process)
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.start, self.stop = [], []
        for _ in range(n):
            for lst in (self.start, self.stop):
                e = ctypes.c_void_p()
                rc = self.hip.hipEventCreate(ctypes.byref(e))
                if rc != 0:
                    raise RuntimeError(f"hipEventCreate failed: {rc}")
                lst.append(e)

    def elapsed_ms(self, i: int) -> float:
        self.hip.hipEventSynchronize(self.stop[i])
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.start[i], self.stop[i])
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def close(self):
        for e in self.start + self.stop:
            self.hip.hipEventDestroy(e)


def decode_algorithmic_bytes(batch, plan_view) -> dict:
    """Algorithmic HBM bytes of one decode step: K and V of every attended token once per
    kv head (head-group fusion: not once per query head), q, the (o, lse) rows, one int32 per
    page, and for every split chunk the partial state written by the attention kernel and read
    again by the merge."""
    H, Hk, D = batch.num_qo_heads, batch.num_kv_heads, batch.head_dim
    tokens = int(batch.kv_lens().sum())
    kv = tokens * Hk * D * 2 * (1 if batch.kv_dtype else 2)   # an 8-bit KV cache stores one byte per element
    n_rows = int(batch.qo_indptr[-1]) * H
    q = n_rows * D * 2
    out = n_rows * (D + 1) * 4
    idx = int(batch.kv_indptr[-1]) * 4
    n_split = int((plan_view["w_out_slot"] >= 0).sum())
    part = n_split * plan_view["t_pos"] * H * (D + 1) * 4
    final_rows_by_attn = n_rows - int(plan_view["m_n_pos"].sum()) * H
    attn = kv + q + idx + part + final_rows_by_attn * (D + 1) * 4
    return dict(kv=kv, q=q, out=out, idx=idx, partial_write=part, attention_kernel=attn,
                step=kv + q + out + idx + 2 * part, tokens=tokens)


def append_algorithmic_flops(batch) -> int:
    """4*D flop per unmasked (query row, key) pair per query head."""
    qo, kv = batch.qo_lens().astype(np.int64), batch.kv_lens().astype(np.int64)
    pairs = 0
    for lq, lk in zip(qo, kv):
        j = np.arange(lq)
        pairs += int(np.clip(lk - lq + j + 1, 0, lk).sum()) if batch.causal else int(lq * lk)
    return pairs * batch.num_qo_heads * 4 * batch.head_dim


def cpu_baseline(batch, unit_work: float, unit: str, budget_s: float = 10.0) -> dict:
    import oracle
    cores = len(os.sched_getaffinity(0))
    passes, t_total = 0, 0.0
    best = float("inf")
    while passes < 3 and t_total < budget_s:
        t0 = time.perf_counter()
        oracle.run_batch(batch)
        dt = time.perf_counter() - t0
        best = min(best, dt)
        t_total += dt
        passes += 1
    return {"value": unit_work / best, "unit": unit, "cores": cores, "kind": "oracle",
            "sample": f"whole batch ({batch.batch} requests), best of {passes} pass(es), {best:.2f} s per pass",
            "seconds_per_batch": best}


def bench_shared_prefix(args) -> int:
    """Workload c5: one decode step of 64 requests sharing a 4096-token prefix.  Composable
    formats (Sec. 3.1.2): prefix pass = one 64-query row block through the append tile kernel,
    suffix pass = paged decode, then fi_merge_state_pair; timed against the single-format decode
    of the same problem on the same box (the comparison of the paper's shared-prefix table)."""
    import torch
    import workloads
    import paper_2501_01005_amd as fi
    from paper_2501_01005_amd.device import DeviceBatch, formats_of, make_formats_wrapper, make_wrapper

    c = workloads.config5(small=args.small)
    dev_p, dev_s, dev_1 = DeviceBatch(c.prefix), DeviceBatch(c.suffix), DeviceBatch(c.single)
    wp = make_wrapper(c.prefix, "append", num_ctas=args.num_ctas, min_chunk=args.min_chunk)
    ws = make_wrapper(c.suffix, "decode", merge=args.merge, min_chunk=args.suffix_min_chunk)
    w1 = make_wrapper(c.single, "decode", merge=args.merge)
    n, H, D = dev_p.q.shape[0], c.prefix.num_qo_heads, c.prefix.head_dim
    o_p = torch.empty((n, H, D), dtype=torch.float32, device="cuda:0"); l_p = torch.empty((n, H), dtype=torch.float32, device="cuda:0")
    o_s = torch.empty_like(o_p); l_s = torch.empty_like(l_p)
    o_1 = torch.empty_like(o_p); l_1 = torch.empty_like(l_p)
    stream = torch.cuda.current_stream().cuda_stream

    side = torch.cuda.Stream() if args.graph and args.c5_path != "formats" else None  # default priority
    # both formats as one plan of one handle (fi_plan_formats): one attention launch + one contraction launch
    formats, ids = formats_of([c.prefix, c.suffix])
    wf = make_formats_wrapper([c.prefix, c.suffix], mode=args.tile_mode, num_ctas=args.num_ctas, min_chunk=args.min_chunk,
                              alpha=args.alpha, beta=args.beta)
    ids_dev = torch.from_numpy(ids).to("cuda:0")

    def composed(plan=True):
        if args.c5_path == "formats":
            if plan:
                wf.plan_formats(formats)
            wf.run(dev_p.q, dev_p.k_pool, dev_p.v_pool, ids_dev, c.prefix.sm_scale, o=o_p, lse=l_p)
            return
        if plan:
            wp.plan(c.prefix.qo_indptr, c.prefix.kv_indptr, c.prefix.last_page_len, causal=False)
            ws.plan(c.suffix.qo_indptr, c.suffix.kv_indptr, c.suffix.last_page_len, causal=False)
        if side is not None:
            # the two passes do not depend on each other: in the captured graph they are parallel branches
            main = torch.cuda.current_stream()
            side.wait_stream(main)
            with torch.cuda.stream(side):
                wp.run(dev_p.q, dev_p.k_pool, dev_p.v_pool, dev_p.kv_indices, c.prefix.sm_scale, o=o_p, lse=l_p)
            ws.run(dev_s.q, dev_s.k_pool, dev_s.v_pool, dev_s.kv_indices, c.suffix.sm_scale, o=o_s, lse=l_s)
            main.wait_stream(side)
            fi.fi_merge_state_pair(o_p, l_p, o_s, l_s, n * H, D, o_p, l_p, main.cuda_stream)
            return
        if args.c5_path == "composed":
            # both attention launches, then one contraction launch over the partial states of both passes
            wp.run_composed(ws, dev_p.q, dev_p.k_pool, dev_p.v_pool, dev_p.kv_indices, dev_s.kv_indices, c.prefix.sm_scale,
                            o=o_p, lse=l_p)
            return
        wp.run(dev_p.q, dev_p.k_pool, dev_p.v_pool, dev_p.kv_indices, c.prefix.sm_scale, o=o_p, lse=l_p)
        ws.run(dev_s.q, dev_s.k_pool, dev_s.v_pool, dev_s.kv_indices, c.suffix.sm_scale, o=o_s, lse=l_s)
        fi.fi_merge_state_pair(o_p, l_p, o_s, l_s, n * H, D, o_p, l_p, stream)

    def single(plan=True):
        if plan:
            w1.plan(c.single.qo_indptr, c.single.kv_indptr, c.single.last_page_len, causal=False)
        w1.run(dev_1.q, dev_1.k_pool, dev_1.v_pool, dev_1.kv_indices, c.single.sm_scale, o=o_1, lse=l_1)

    def timeit(fn, plan):
        fn(True)
        for _ in range(args.warmup):
            fn(plan)
        torch.cuda.synchronize()
        step = lambda: fn(plan)
        if args.graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                fn(False)
            step = graph.replay
            for _ in range(args.warmup):
                step()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps * 1e6

    us_comp = timeit(composed, not args.no_plan)
    us_single = timeit(single, not args.no_plan)
    bytes_comp = c.prefix.kv_bytes() + c.suffix.kv_bytes() + n * H * D * 2 + 3 * n * H * (D + 1) * 4
    bytes_single = c.single.kv_bytes() + n * H * D * 2 + n * H * (D + 1) * 4
    line = {
        "metric": "achieved HBM bandwidth, shared-prefix decode step in composable formats (algorithmic bytes, prefix once / step time)",
        "value": bytes_comp / (us_comp * 1e-6) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": us_comp * 1e-3, "us_per_batch": us_comp, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": c.prefix.dtype, "data": "synthetic",
        "config": {"workload": "c5_shared_prefix" + ("_small" if args.small else ""), "requests": n,
                   "prefix_tokens": int(c.prefix.kv_lens()[0]),
                   "step": (("one captured graph, replayed: " if args.graph else "") +
                            {"formats": "both formats in one plan: 1 attention launch + 1 contraction launch (fi_plan_formats, fi_run; "
                                        + args.tile_mode + ")",
                             "composed": "2 attention launches + 1 contraction launch (fi_run_composed)",
                             "separate": "2 attention launches + 3 merge launches"}[args.c5_path] +
                            ("" if args.no_plan else ", planned every step"))},
        "frac_of_peak": bytes_comp / (us_comp * 1e-6) / 1e9 / HBM_PEAK_GBS,
        "composable_us": us_comp, "single_format_us": us_single, "speedup_vs_single_format": us_single / us_comp,
        "algorithmic_bytes_composable": bytes_comp, "algorithmic_bytes_single_format": bytes_single,
        "single_format_GBps": bytes_single / (us_single * 1e-6) / 1e9,
        "roofline": {"bound": "hbm", "kernel": "latency-bound (dependent small launches); see single_format_GBps for the streaming rate",
                     "achieved": bytes_comp / (us_comp * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": bytes_comp / (us_comp * 1e-6) / 1e9 / HBM_PEAK_GBS, "traffic": None},
    }
    print(json.dumps(line))
    return 0


E2_WORKLOADS = [f"e2-{k}-{d}" for k in ("decode", "prefill") for d in ("constant", "uniform", "zipf")]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # 250 back-to-back steps are 0.1 s of GPU time; shorter runs after an idle period catch the power
    # management's transient (the matrix-bound append kernel swings between 334 and 392 us per launch in its
    # first 15 ms and settles near 329 us)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "sa"] + E2_WORKLOADS,
                    help="c1..c5: the benchmark configurations; e2-<decode|prefill>-<constant|uniform|zipf>: batch 16 "
                         "with the three length distributions of the paper's kernel experiment (Sec. 4.2); sa: short "
                         "appends (--sa-qo tokens per request, --sa-batch requests, caches up to --sa-kv-max tokens) through "
                         "the handle mode --handle-mode")
    ap.add_argument("--e2-len", type=int, default=1024,
                    help="e2-*-constant: the sequence length (the paper's experiment has 1024)")
    ap.add_argument("--sa-qo", type=int, default=16)
    ap.add_argument("--sa-batch", type=int, default=64)
    ap.add_argument("--sa-kv-max", type=int, default=4096)
    ap.add_argument("--handle-mode", default="append", choices=["decode", "tile16", "tile64", "append"],
                    help="sa: the query tile of the handle (decode needs --sa-qo 1)")
    ap.add_argument("--small", action="store_true", help="small variant of the workload (debug)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-plan", action="store_true", help="time fi_run only (plan once, as for layers 2..L)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of the workload, launch a plain elementwise kernel that reads 1 GiB and writes "
                         "1 GiB per launch (scale reference for the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--event-stride", type=int, default=5,
                    help="bracket every n-th attention launch of the timed region with HIP events (recording a pair "
                         "costs the step about 10 us on this box, so not every launch carries one)")
    ap.add_argument("--page-order", default="random", choices=["random", "identity"],
                    help="identity: every request's pages are consecutive in the pool (with --kv-layout NHD that is a "
                         "contiguous ragged KV tensor); c2, c3, c4 only")
    ap.add_argument("--kv-contiguous", action="store_true",
                    help="with --page-order identity: run without a page table (fi_run with kv_indices = NULL: affine "
                         "addressing, the dense baseline of App. B's comparison); c2, c3, c4")
    ap.add_argument("--kv-layout", default="HND", choices=["HND", "NHD"],
                    help="pool layout in memory: [page, head, slot, D] (default, tuned) or [page, slot, head, D]")
    ap.add_argument("--kv-dtype", default="same", choices=["same", "fp8"],
                    help="fp8: K/V stored as E4M3 codes with scales (App. F), decode workloads c2 and c4 only")
    ap.add_argument("--page-size", type=int, default=16, help="tokens per page (c2 and c3; 16 is the tuned size)")
    ap.add_argument("--rope-theta", type=float, default=0.0,
                    help="> 0: the rotary embedding fused into the kernel (fi_run_variant; the cache holds unrotated keys, "
                         "Sec. 4.3); 16-bit decode and causal append workloads")
    ap.add_argument("--soft-cap", type=float, default=0.0,
                    help="> 0: logits soft cap c * tanh(s / c) (fi_run_variant, Sec. 3.2.3); 16-bit decode and causal append workloads")
    ap.add_argument("--alibi", action="store_true",
                    help="ALiBi bias slope[head] * (t - pos) on the logits (fi_run_variant); 16-bit decode and causal append workloads")
    ap.add_argument("--window-left", type=int, default=-1,
                    help=">= 0: decode with a sliding window of that many tokens behind the query (fi_run_variant)")
    ap.add_argument("--plan-window", action="store_true",
                    help="with --window-left: the planner knows the window (fi_config.plan_window) and leaves the hidden "
                         "keys out of the work items")
    ap.add_argument("--graph", action="store_true",
                    help="with --no-plan: capture fi_run (attention + merge launches) in a HIP graph once and time its "
                         "replays; c5: the prefix and the suffix pass become parallel branches of the graph")
    ap.add_argument("--num-ctas", type=int, default=0)
    ap.add_argument("--min-chunk", type=int, default=0)
    ap.add_argument("--balance", type=int, default=0, help="fi_config.balance (0 = default of the mode)")
    ap.add_argument("--merge", type=int, default=0,
                    help="fi_config.merge: 1 = partial states folded by a second launch, 2 = inside the attention launch "
                         "(decode), 0 = default")
    ap.add_argument("--suffix-min-chunk", type=int, default=0, help="c5: fi_config.min_chunk of the suffix (decode) handle")
    ap.add_argument("--tile-mode", default="tile16", choices=["tile16", "tile64"],
                    help="c5 with --c5-path formats: the handle's query tile: 16 fused rows, one wavefront per CTA, or 64 "
                         "fused rows, four wavefronts per CTA that share the K/V rows of a wide tile through LDS")
    ap.add_argument("--c5-path", default="formats", choices=["formats", "composed", "separate"],
                    help="c5: formats = both formats planned as one work list on one 16-row-tile handle (fi_plan_formats; one "
                         "attention launch + one contraction launch); composed = a handle per format, fi_run_composed (two "
                         "attention launches + one contraction launch); separate = fi_run on each and fi_merge_state_pair (five)")
    ap.add_argument("--out16", action="store_true",
                    help="append workloads: write the output in the input type only (fi_run with o = NULL), not as fp32 rows")
    ap.add_argument("--alpha", type=int, default=0, help="fi_config.alpha (with --beta; 0, 0 = default)")
    ap.add_argument("--beta", type=int, default=0)
    args = ap.parse_args()
    if args.graph and not args.no_plan:
        print("bench.py: --graph times replays of a captured fi_run and needs --no-plan", file=sys.stderr)
        return 2
    if args.kv_contiguous and (args.page_order != "identity" or args.workload not in ("c2", "c3", "c4")):
        print("bench.py: --kv-contiguous needs --page-order identity and one of c2, c3, c4", file=sys.stderr)
        return 2
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no multi-GPU path exists); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    import workloads
    import paper_2501_01005_amd as fi
    from paper_2501_01005_amd.device import DeviceBatch, make_wrapper

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    # the driver's invocation (no workload or variant flag): the headline workload plus an "also" block
    plain_default = all(getattr(args, k) == ap.get_default(k) for k in vars(args) if k not in ("gpus", "steps", "warmup"))
    if args.calibrate_copy:
        n = (1 << 30) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(args.warmup + args.steps):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "torch.add(src, 1.0, out=dst)", "read_bytes_per_launch": n * 4,
                          "write_bytes_per_launch": n * 4, "launches": args.warmup + args.steps}))
        return 0
    if args.workload == "c5":
        return bench_shared_prefix(args)
    line = run_workload(args)
    if isinstance(line, int):
        return line
    if plain_default:
        # the other two roofline-bound workloads in the same process, each with its own settled warm-up: the
        # matrix-bound append kernel (c3) and the long-context decode with split KV and merge (c4)
        line["also"] = []
        for wl in ("c3", "c4"):
            sub = argparse.Namespace(**vars(args))
            sub.workload, sub.no_cpu_baseline = wl, True
            sub.warmup, sub.steps = max(args.warmup, 50), max(args.steps, 100)
            extra = run_workload(sub)
            if isinstance(extra, int):
                return extra
            line["also"].append({k: extra[k] for k in ("metric", "value", "unit", "steps", "warmup", "us_per_batch", "dtype",
                                                       "config", "frac_of_peak", "host_plan_us", "roofline")})
    print(json.dumps(line))
    return 0


def run_workload(args):
    """One workload: set-up, warm-up, timed steps; returns the JSON line as a dict (or an exit code)."""
    import torch
    import workloads
    import paper_2501_01005_amd as fi
    from paper_2501_01005_amd.device import DeviceBatch, make_wrapper

    cfg_kw = {"permute_pages": False} if args.page_order == "identity" and args.workload in ("c2", "c3", "c4") else {}
    if args.kv_dtype == "fp8":
        if args.workload not in ("c2", "c4"):
            print("bench.py: --kv-dtype fp8 is for the decode workloads c2 and c4", file=sys.stderr)
            return 2
        cfg_kw["kv_dtype"] = workloads.FP8
    if args.page_size != 16:
        if args.workload not in ("c2", "c3"):
            print("bench.py: --page-size is for c2 and c3", file=sys.stderr)
            return 2
        cfg_kw["page_size"] = args.page_size
    if args.workload == "sa":
        if args.handle_mode == "decode" and args.sa_qo != 1:
            print("bench.py: a decode-mode handle takes one query position per request (--sa-qo 1)", file=sys.stderr)
            return 2
        batch = workloads.short_append(args.sa_qo, args.sa_batch, args.sa_kv_max)
        mode = args.handle_mode
    elif args.workload in E2_WORKLOADS:
        _, kind, dist = args.workload.split("-")
        batch = workloads.config_e2(kind, dist, args.e2_len)
        mode = "append" if kind == "prefill" else "decode"
    else:
        batch = getattr(workloads, "config" + args.workload[1])(small=args.small, **cfg_kw)
        mode = "append" if args.workload == "c3" else "decode"
    dev = DeviceBatch(batch, kv_layout=args.kv_layout)
    w = make_wrapper(batch, mode, num_ctas=args.num_ctas, min_chunk=args.min_chunk, balance=args.balance,
                     alpha=args.alpha, beta=args.beta, merge=args.merge,
                     plan_window=args.window_left + 1 if args.plan_window and args.window_left >= 0 else 0)
    nnz = dev.q.shape[0]
    o = torch.empty((nnz, batch.num_qo_heads, batch.head_dim), dtype=torch.float32, device=dev.device)
    lse = torch.empty((nnz, batch.num_qo_heads), dtype=torch.float32, device=dev.device)

    run_kw = dict(dev.scales)
    if args.out16:
        if mode != "append":
            print("bench.py: --out16 is for the append workloads (the decode byte counts assume fp32 rows)", file=sys.stderr)
            return 2
        run_kw["o_cast"] = torch.empty((nnz, batch.num_qo_heads, batch.head_dim), dtype=dev.q.dtype, device=dev.device)
        o = False
    if args.rope_theta > 0 or args.window_left >= 0 or args.soft_cap > 0 or args.alibi:
        if batch.kv_dtype or args.page_size != 16 or (mode != "decode" and not batch.causal):
            print("bench.py: --rope-theta, --window-left, --alibi and --soft-cap are for the 16-bit decode workloads with "
                  "page size 16 and the causal append workloads", file=sys.stderr)
            return 2
        run_kw["variant"] = dict(
            kv_indptr=torch.from_numpy(np.ascontiguousarray(batch.kv_indptr, dtype=np.int32)).to(dev.device),
            last_page_len=torch.from_numpy(np.ascontiguousarray(batch.last_page_len, dtype=np.int32)).to(dev.device),
            rope_theta=args.rope_theta, window_left=args.window_left, logits_soft_cap=args.soft_cap)
        if args.alibi:   # the usual geometric slopes 2^(-8 (h + 1) / H)
            h = batch.num_qo_heads
            run_kw["variant"]["alibi_slopes"] = torch.tensor([2.0 ** (-8.0 * (i + 1) / h) for i in range(h)],
                                                             dtype=torch.float32, device=dev.device)

    stride = max(1, args.event_stride)
    n_samples = (args.steps + stride - 1) // stride
    ev = HipEvents(n_samples)

    def step(i_timed: int = -1):
        if not args.no_plan or i_timed == -2:
            w.plan(batch.qo_indptr, batch.kv_indptr, batch.last_page_len, causal=batch.causal)
        sampled = i_timed >= 0 and i_timed % stride == 0
        if sampled:
            fi.lib.fi_set_timing_events(w.handle, ev.start[i_timed // stride], ev.stop[i_timed // stride])
        w.run(dev.q, dev.k_pool, dev.v_pool, None if args.kv_contiguous else dev.kv_indices, batch.sm_scale, o=o, lse=lse,
              **run_kw)
        if sampled:
            fi.lib.fi_set_timing_events(w.handle, None, None)

    step(-2)
    view = fi.fi_plan_view(w.handle)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        # one captured launch sequence, replayed (the kernel's own time is taken from eager launches afterwards)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        for i in range(n_samples):  # kernel time: eager launches with events, outside the timed region
            step(i * stride)
        torch.cuda.synchronize()
    else:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    kern_ms = [ev.elapsed_ms(i) for i in range(n_samples)]
    kern_avg_ms = float(np.mean(kern_ms))

    # host planner alone
    tp = time.perf_counter()
    for _ in range(20):
        fi.fi_plan(w.handle, batch.qo_indptr, batch.kv_indptr, batch.last_page_len, batch.causal)
    plan_us = (time.perf_counter() - tp) / 20 * 1e6

    traffic = None  # HBM bytes per launch by hardware counters: taken in an earlier profiled run of this command, not live
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    measured_setup = (args.page_size == 16 and args.page_order == "random" and args.kv_layout == "HND" and
                      args.window_left < 0 and args.soft_cap == 0 and not args.alibi and not args.small)  # the counters were taken on these settings only
    if os.path.exists(tpath) and measured_setup:
        traffic = json.load(open(tpath)).get(args.workload + ("_fp8" if batch.kv_dtype else "") +
                                             ("_rope" if args.rope_theta > 0 else "") +
                                             ("_small" if args.small else ""))

    if mode != "append" or args.workload == "sa":   # bound by the K/V bytes: every attended token once per kv head
        ab = decode_algorithmic_bytes(batch, view)
        value = ab["step"] / (ms_per_step * 1e-3) / 1e9
        achieved = ab["attention_kernel"] / (kern_avg_ms * 1e-3) / 1e9
        metric, unit = ("achieved HBM bandwidth, short causal appends (algorithmic bytes / step time)" if args.workload == "sa" else
                        "achieved HBM bandwidth, paged GQA decode step (algorithmic bytes / step time)"), "GB/s"
        roof = {"bound": "hbm", "kernel": {"decode": "decode_kernel", "tile16": "tile_kernel", "tile64": "tile64_kernel",
                                           "append": "append_kernel"}[mode], "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "traffic_source": "profiles/traffic.json: rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this workload, not of this run",
                "algorithmic_bytes_per_launch": ab["attention_kernel"], "avg_kernel_us": kern_avg_ms * 1e3,
                "min_kernel_us": float(np.min(kern_ms)) * 1e3, "timed_launches": n_samples}
        base_work, base_unit = ab["step"] / 1e9, "GB/s"
        extra = {"kv_tokens": ab["tokens"], "algorithmic_bytes_per_step": ab["step"]}
    else:
        fl = append_algorithmic_flops(batch)
        value = fl / (ms_per_step * 1e-3) / 1e12
        achieved = fl / (kern_avg_ms * 1e-3) / 1e12
        metric, unit = "achieved MFMA throughput, causal paged append step (algorithmic flop / step time)", "TFLOP/s"
        roof = {"bound": "mfma", "kernel": "append_kernel", "achieved": achieved, "peak": MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / MFMA_PEAK_TFLOPS, "traffic": traffic,
                "traffic_source": "profiles/traffic.json: rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this workload, not of this run",
                "algorithmic_flop_per_launch": fl, "avg_kernel_us": kern_avg_ms * 1e3,
                "min_kernel_us": float(np.min(kern_ms)) * 1e3, "timed_launches": n_samples}
        base_work, base_unit = fl / 1e12, "TFLOP/s"
        extra = {"algorithmic_flop_per_step": fl}

    line = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "us_per_batch": ms_per_step * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": batch.dtype, "data": "synthetic",
        "config": {"workload": batch.name, "batch": batch.batch, "num_qo_heads": batch.num_qo_heads,
                   "num_kv_heads": batch.num_kv_heads, "head_dim": batch.head_dim, "page_size": batch.page_size, "handle_mode": mode, "page_order": args.page_order, "kv_layout": args.kv_layout,
                   "page_table": "none (contiguous KV, affine addressing)" if args.kv_contiguous else "kv_indices",
                   "kv_dtype": batch.kv_dtype or batch.dtype, "o_dtype": batch.dtype if args.out16 else "f32",
                   **({"fused_rope_theta": args.rope_theta} if args.rope_theta > 0 else {}),
                   **({"logits_soft_cap": args.soft_cap} if args.soft_cap > 0 else {}),
                   **({"alibi": True} if args.alibi else {}),
                   **({"window_left": args.window_left, "planned": bool(args.plan_window)} if args.window_left >= 0 else {}),
                   "step": ("fi_run captured in a HIP graph, replayed (plan reused)" if args.graph else
                            "fi_run only (plan reused)" if args.no_plan else "fi_plan + fi_run"),
                   "ctas_per_head": int(view["ctas_per_head"]), "l_kv_chunk": int(view["l_kv_chunk"]),
                   "n_work": int(view["n_work"]), "n_split_tiles": int(view["n_merge"])},
        "frac_of_peak": (value / HBM_PEAK_GBS) if unit == "GB/s" else (value / MFMA_PEAK_TFLOPS),
        "host_plan_us": plan_us, "roofline": roof, **extra,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(batch, base_work, base_unit)
    ev.close()
    w.close()
    return line


if __name__ == "__main__":
    sys.exit(main())
