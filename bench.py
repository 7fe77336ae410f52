#!/usr/bin/env python3
"""Benchmark of the shared-decode step on one MI355X.

A "step" is one full decode step (all layers, lm_head, argmax) over one synthetic mixed-model
batch whose weights, KV pool, page tables and lengths are resident in HBM before timing starts.
Prints ONE JSON line: tokens/s (= batch / step time), TPOT (= step time), the roofline of the
dominant kernel (paged attention, HBM bound) measured with HIP events inside this run, and the
CPU oracle timed on a bounded sample of the same workload on this machine's host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg3|cfg5a|cfg5b] [--quant asym|sym|sym_noz]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "int8": 5000.0}   # dense matrix-core peaks of the MI355X


def measured_traffic_bytes(workload: str, quant):
    """HBM bytes per attention launch from the counter summaries under profiles/ (two rocprofv3 --pmc runs of
    this script, FETCH_SIZE then WRITE_SIZE, each scaled by what the same counter reads for a plain 1 GiB copy:
    --copy-calibration).  The summary of a workload carries a line `traffic_bytes_per_launch: <bytes>`; a
    workload (or weight format) that was not counted reports null.  Not a reading of this run."""
    name = f"attn_split_{workload}{'_qsun' if quant else ''}_hbm_traffic_pmc.txt"
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def w4_bytes_per_weight(quant) -> float:
    """4-bit codes + an fp16 scale per 128 weights, + an fp16 zero point unless the layout stores none."""
    return 0.515625 if quant == "sym_noz" else 0.53125


def algorithmic_bytes(shape, work, quant, logits_out: bool = True):
    """Bytes the method must move per step: weights once, lm_head (bf16), embedding rows,
    KV read for every cached position incl. the new one, KV write, fp32 logits."""
    el = 4 if getattr(work, "dtype", "bf16") == "f32" else 2   # bytes of a dense weight
    b_w = w4_bytes_per_weight(quant) if quant else float(el)
    weights = shape.body_params * b_w + shape.vocab * shape.hidden * el
    kv_tok = shape.kv_bytes_per_token()
    kv_read = float(work.kv_tokens_read) * kv_tok
    kv_write = work.batch * kv_tok
    other = work.batch * shape.hidden * el + (work.batch * shape.vocab * 4 if logits_out else 0)
    return {"weights": weights, "kv_read": kv_read, "kv_write": kv_write, "other": other,
            "total": weights + kv_read + kv_write + other}


def build_workload(name: str):
    from paper_2603_02599_amd import workloads as wl
    if name.startswith("b") and "x" in name:      # "b<batch>x<len>": 8B shape, that many requests, all that long
        batch, length = (int(v) for v in name[1:].split("x"))
        return (wl.make_workload("cfg2", batch=batch, lo=length, hi=length, n_models=min(4, batch), seed=100 + batch),
                f"8B-shaped shared decode, batch {batch}, every cache {length} long (the grid of --sweep-step-times)")
    if name == "cfg1":
        return wl.make_workload("cfg1"), "tiny fp32 shape, 8 requests over 3 source models, L~U[16,128] (the oracle runs it whole)"
    if name == "cfg2":
        return wl.make_workload("cfg2"), "8B-shaped shared decode, batch 64 over 4 source models, L~U[512,4096]"
    if name == "cfg3":
        return wl.make_workload("cfg3"), "8B-shaped shared decode, batch 256 over 8 Zipf(1.2) source models, log-normal L (median 1024, clip [64,16384])"
    if name == "cfg5b":
        w = wl.make_workload("cfg5b")
        return w, (f"14B-shaped shared decode, the first {w.batch} of 128 Zipf(1.2)-tagged requests, L~U[2048,32768], whose "
                   "caches fit a 200 GB pool (no aliasing)")
    if name == "cfg5a":
        w = wl.make_workload("cfg5a")
        return w, (f"14B-shaped shared decode, batch 128 over 16 Zipf(1.2) source models, L~U[2048,32768], over a "
                   f"{w.n_pages}-page (206 GB) pool: own tail pages, history pages shared read-only")
    if name == "small":
        return (wl.make_workload("cfg2", shape=wl.SMALL128, batch=64, lo=64, hi=512, seed=7),
                "small128 test shape, batch 64 (not a benchmark configuration)")
    raise SystemExit(f"unknown workload {name}")


def cpu_baseline(case, work, n_sample: int):
    """Times the oracle (as it stands) on n_sample requests spread over the length distribution.  The only
    part of this script that touches the oracle: it hands it host copies of the weights and of the sampled
    requests' cache pages."""
    import torch
    from oracle import oracle as orc
    from paper_2603_02599_amd.device_case import layout_strides, to_np, weights_to_np
    order = np.argsort(work.seq_lens)
    rows = sorted({int(order[int(round(q * (work.batch - 1)))]) for q in np.linspace(0, 1, n_sample)})
    wnp = weights_to_np(case.w)
    qnp = None
    if case.quant is not None:
        def triple(t):
            q, sc, z = t
            scn = to_np(sc)
            return to_np(q), scn, (to_np(z) if z is not None else np.full(scn.shape, 0x4800, np.uint16))
        qnp = {k: [triple(t) for t in v] for k, v in case.quant.items()}
        for k, v in qnp.items():        # the dense sources of the quantised matrices have left the device
            if k not in wnp:
                wnp[k] = [np.empty((0, 2 * t[0].shape[1]), np.float32) for t in v]
    params = orc.params_from_arrays(wnp, qnp)
    # compact host copy of the pages the sampled requests reference, same in-page layout
    lay = case.lay
    tabs = work.page_tables[rows]
    used = np.unique(tabs[tabs >= 0])
    remap = np.full(int(lay.n_pages), -1, np.int64)
    remap[used] = np.arange(len(used))
    new_tabs = np.where(tabs >= 0, remap[np.maximum(tabs, 0)], -1).astype(np.int32)
    view = case.pool_mem.view(work.shape.n_layers, int(lay.n_pages), int(lay.k_page))
    host = to_np(view.index_select(1, torch.from_numpy(used.astype(np.int64)).to(view.device)).contiguous()).reshape(-1).copy()
    st = layout_strides(lay)
    st["k_layer"] = st["v_layer"] = len(used) * int(lay.k_page)
    pool = orc.make_pool(host, len(used), 16, st)
    ocfg = orc.make_cfg(work.shape)

    def timed():
        t0 = time.perf_counter()
        orc.decode_step(ocfg, params, pool, work.tokens[rows], new_tabs, work.seq_lens[rows], work.model_ids[rows])
        return time.perf_counter() - t0

    dt = timed()
    out = {"value": len(rows) / dt, "unit": "tokens/s", "cores": orc.threads(), "kind": "oracle",
           "sample": f"{len(rows)} of {work.batch} requests of the same batch (lengths "
                     f"{[int(work.seq_lens[r]) for r in rows]}), all {work.shape.n_layers} layers + lm_head, "
                     f"one oracle step took {dt:.3g} s; gcc -O2 -fopenmp, fp64"}
    if len(rows) == work.batch and dt < 2.0:
        # a batch the oracle finishes at once is also timed on one thread (the OpenMP runtime's own switch;
        # the oracle's code is untouched)
        import ctypes
        omp = ctypes.CDLL("libgomp.so.1")
        n = orc.threads()
        omp.omp_set_num_threads(1)
        try:
            out["one_thread"] = {"value": len(rows) / timed(), "unit": "tokens/s", "cores": 1}
        finally:
            omp.omp_set_num_threads(n)
    return out


def bench_run(args, sun, case, work, shape, desc, free_list):
    """K steps of greedy decoding in one library call: tokens/s over the run and TPOT = time / K."""
    import torch
    d_free = torch.from_numpy(free_list).cuda()
    d_head = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_status = torch.zeros(1, dtype=torch.int32, device="cuda")
    n_out = max(args.steps, args.warmup, 1)
    d_out = torch.empty((n_out, work.batch), dtype=torch.int32, device="cuda")
    tok, tab, lens = case.tokens.clone(), case.tables.clone(), case.lens.clone()

    def run(n, flags=0):
        sun.sun_decode_run(case.pool, case.weights, n, tok, tab, lens, case.ids, d_free, d_head, d_status, d_out,
                           case.logits, case.ws, flags=flags)

    if args.warmup:
        run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert int(d_status.cpu()[0]) == 0, "a request ran out of pages during the run"
    ms_per_step = wall * 1e3 / args.steps
    pn = min(8, args.steps)  # per-kernel event timing on the steps that follow the timed run
    if not args.no_profile:
        sun.sun_profile_reset()
        run(pn, sun.SUN_PROFILE)
        torch.cuda.synchronize()
    # bytes: the caches grow by one token per request and step
    start = work.seq_lens.astype(np.int64) + args.warmup
    kv_tokens = sum(int((start + s + 1).sum()) for s in range(args.steps)) / args.steps
    roof, kernels = None, {}
    if not args.no_profile:
        prof = sun.sun_profile_read()
        sun.sun_profile_reset()
        for k, v in prof.items():
            if v["launches"]:
                kernels[k] = {"avg_us": 1e3 * v["ms"] / v["launches"], "launches_per_step": v["launches"] // pn,
                              "ms_per_step": v["ms"] / pn}
        att = prof["attn_split"]
        after = work.seq_lens.astype(np.int64) + args.warmup + args.steps
        per_launch = sum(int((after + s + 1).sum()) for s in range(pn)) / pn * 2 * shape.n_kv_heads * shape.head_dim * 2
        avg_s = att["ms"] / att["launches"] * 1e-3
        roof = {"bound": "hbm", "kernel": "attn_split_kernel", "achieved": per_launch / avg_s / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": per_launch / avg_s / 1e9 / HBM_PEAK_GBS,
                "traffic": None, "bytes_per_launch": per_launch, "avg_launch_us": avg_s * 1e6}

    class _W:  # the average step of the run, for the byte count
        batch = work.batch
        kv_tokens_read = kv_tokens
    alg = algorithmic_bytes(shape, _W, args.quant, logits_out=False)
    alg["total"] += work.batch * shape.vocab * 4 / args.steps  # logits are written by the last step only
    out = {
        "metric": "shared-decode tokens/sec", "value": work.batch / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "tpot_ms": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("f32" if work.dtype == "f32" else "bf16") if not args.quant else "bf16 activations, 4-bit group-128 weights", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc}; one sun_decode_run of {args.steps} steps after "
                               f"{args.warmup} warm-up steps (greedy feedback, caches grow, pages from a free list)",
                   "shape": shape.name, "batch": work.batch, "quant": args.quant, "mode": "run",
                   "output_length": args.steps, "mean_kv_tokens_per_step": kv_tokens,
                   "pages_taken": int(d_head.cpu()[0])},
        "algorithmic_GB_per_step": alg["total"] / 1e9,
        "step_GBps": alg["total"] / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": alg["total"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": roof, "kernels": kernels,
        "cpu_baseline": None,
    }
    print(json.dumps(out))


def bench_serve(args, sun, H):
    """K iterations of continuous batching in one library call: the rows of the --workload batch are kept
    busy from a queue of prefilled requests that retire at their output budget and are replaced on the
    device; tokens/s counts generated tokens only (idle rows count for nothing)."""
    import torch
    base, desc = build_workload(args.workload)
    shape, slots = base.shape, base.batch
    rng = np.random.default_rng(2025)
    n_wait = 3 * slots
    total_steps = args.warmup + args.steps
    lens = rng.choice(base.seq_lens, size=n_wait).astype(np.int32)            # the workload's own length mix
    budgets = rng.integers(max(2, total_steps // 4), max(3, total_steps) + 1, size=n_wait).astype(np.int32)
    cols = int(lens.max() + budgets.max()) // 16 + 1
    have = lens // 16 + 1
    ring_n = slots * (int(budgets.max()) // 16 + 2)
    n_pages = 1 + int(have.sum()) + ring_n
    perm = rng.permutation(n_pages).astype(np.int32)
    tables = np.full((n_wait, cols), -1, np.int32)
    o = 1
    for r in range(n_wait):
        tables[r, :have[r]] = perm[o:o + have[r]]
        o += int(have[r])
    work = base
    work.page_tables, work.n_pages = np.full((slots, cols), -1, np.int32), n_pages
    t_setup = time.perf_counter()
    case = H.DeviceCase(work, quant_mode=args.quant)
    if args.quant:
        for k in sun.QUANT_KEYS:
            case.w[k] = None
    waiting = {"req": np.arange(n_wait, dtype=np.int32), "token": rng.integers(0, shape.vocab, size=n_wait).astype(np.int32),
               "tables": tables, "lens": lens, "model": rng.integers(0, work.n_models, size=n_wait).astype(np.int32),
               "budget": budgets}
    state = sun.ServeTensors(slots, cols, waiting, perm[o:].tolist(), n_pages, int(perm[0]))
    ws = torch.empty(sun.sun_serve_workspace_bytes(case.cfg, slots, cols), dtype=torch.uint8, device="cuda")
    n_out = max(args.steps, args.warmup, 1)
    toks = torch.empty((n_out, slots), dtype=torch.int32, device="cuda")
    reqs = torch.empty((n_out, slots), dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    print(f"[bench] setup {time.perf_counter() - t_setup:.1f} s; pool {n_pages} pages, {n_wait} requests waiting",
          file=sys.stderr, flush=True)
    sun.sun_decode_serve(case.pool, case.weights, max(args.warmup, 1), state, toks, reqs, None, ws,
                         flags=sun.SUN_VALIDATE | sun.SUN_SERVE_RESET)
    torch.cuda.synchronize()
    c0 = state.counters.cpu().tolist()
    t0 = time.perf_counter()
    sun.sun_decode_serve(case.pool, case.weights, args.steps, state, toks, reqs, None, ws)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    c1 = state.counters.cpu().tolist()
    assert c1[3] == 0, f"status {c1[3]}"
    gen = c1[6] - c0[6]
    ms_per_step = wall * 1e3 / args.steps
    print(json.dumps({
        "metric": "shared-decode tokens/sec", "value": gen / wall, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": max(args.warmup, 1), "ms_per_step": ms_per_step, "tpot_ms": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": ("f32" if work.dtype == "f32" else "bf16") if not args.quant else "bf16 activations, 4-bit group-128 weights", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc}; continuous batching: one sun_decode_serve call of {args.steps} "
                               f"iterations over {slots} rows fed from {n_wait} prefilled requests (lengths drawn from the "
                               f"workload's, output budgets U[{int(budgets.min())},{int(budgets.max())}]), retirement, page "
                               "return and admission on the device",
                   "shape": shape.name, "rows": slots, "quant": args.quant, "mode": "serve",
                   "tokens_generated": gen, "row_occupancy": gen / (args.steps * slots),
                   "admitted": c1[5] - c0[5], "retired": c1[4] - c0[4], "still_waiting": n_wait - c1[0]},
        "roofline": None, "cpu_baseline": None}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None,
                    help="one workload only: cfg2 (the headline configuration), cfg1 (tiny fp32), cfg3, cfg5a, cfg5b, small, or "
                         "b<batch>x<len>.  Default (step mode): cfg2 and cfg3, each with bf16 and with 4-bit weights, in one "
                         "process; the JSON line is cfg2/bf16 and carries the other three under \"legs\"")
    ap.add_argument("--quant", default=None, choices=[None, "asym", "sym", "sym_noz"],
                    help="4-bit group-128 decode weights: affine, symmetric, or symmetric without stored zero points")
    ap.add_argument("--cpu-sample", type=int, default=24, help="requests the oracle is timed on (0 = skip); 24 are about 10 s of CPU work")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event pass")
    ap.add_argument("--graph", action="store_true", help="replay the step from a captured HIP graph")
    ap.add_argument("--ingest-tokens", type=int, default=0,
                    help="instead of decoding: time sun_kv_pool_ingest of one prompt cache of this many tokens "
                         "(shape of --workload), K times; prints its own JSON line (tokens/s and GB/s read+written)")
    ap.add_argument("--prefill-tokens", type=int, default=0,
                    help="instead of decoding: time sun_prefill of one prompt of this many tokens (shape of "
                         "--workload, bf16), K times; prints its own JSON line (prompt tokens/s)")
    ap.add_argument("--mode", default="step", choices=["step", "run", "serve"],
                    help="step: K independent calls of the decode step on the same inputs (default). "
                         "run: one sun_decode_run call of K steps with token feedback, growing caches and page "
                         "allocation on the device (TPOT over an output length of K). "
                         "serve: one sun_decode_serve call of K iterations: rows retire at their output budget and "
                         "take waiting requests, on the device (continuous batching)")
    ap.add_argument("--sweep-step-times", action="store_true",
                    help="instead of one workload: time the decode step of the --workload shape over a grid of batch "
                         "sizes and cache lengths (all requests of a point equally long) and print one JSON table; "
                         "this is the input of paper_2603_02599_amd/placement.py")
    ap.add_argument("--hbm-read-probe", action="store_true",
                    help="only time a kernel that reads 8 GiB and does nothing else (address order, shuffled 4 KiB blocks): the "
                         "practical ceiling the HBM-bound kernels are compared with")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy (known size) to calibrate FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.copy_calibration:
        import torch
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "launches": 6, "ms_per_copy": ms,
                          "read_plus_write_GBps": 2.0 * (1 << 30) / (ms * 1e-3) / 1e9}))
        return
    if args.hbm_read_probe:
        # the yardstick: what a kernel that only reads reaches on this device (sun_hbm_read_probe), over buffers far
        # larger than the 256 MB memory-side cache, in address order and in shuffled 4 KiB blocks (the size of one
        # (page, head) K or V block of the pool)
        import torch
        from paper_2603_02599_amd import binding as sun
        sun.lib()
        nbytes = 8 << 30
        src = torch.empty(nbytes // 4, dtype=torch.int32, device="cuda")
        src.random_(0, 1 << 30)
        perm = torch.randperm(nbytes // 4096, device="cuda").to(torch.int32)
        out = {"what": "read-only streaming kernel", "bytes": nbytes, "hbm_peak_GBps": HBM_PEAK_GBS, "runs": []}
        for block, order, wgs, streaming in ((4096, None, 2048, False), (4096, perm, 2048, False), (4096, perm, 1024, False),
                                             (4096, perm, 4096, False), (65536, None, 2048, False), (4096, None, 2048, True),
                                             (4096, perm, 2048, True), (4096, perm, 512, True), (4096, perm, 8192, True)):
            sink = torch.empty(wgs * 256, dtype=torch.int32, device="cuda")
            p = order if block == 4096 else None
            for _ in range(2):
                sun.sun_hbm_read_probe(src, block, p, wgs, sink, streaming_loads=streaming)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                sun.sun_hbm_read_probe(src, block, p, wgs, sink, streaming_loads=streaming)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            out["runs"].append({"block_bytes": block, "order": "shuffled" if p is not None else "address", "workgroups": wgs,
                                "loads": "streaming" if streaming else "plain",
                                "ms": ms, "GBps": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS})
        print(json.dumps(out))
        return
    if args.gpus != 1:
        raise SystemExit("bench.py: this build measures one GPU only (one decode worker holds a full copy of the "
                         "shared decode weights; more GPUs are more independent workers). Run with --gpus 1.")
    import torch
    from paper_2603_02599_amd import binding as sun
    sun.lib()  # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    from paper_2603_02599_amd import device_case as H   # device buffers and handles; nothing of the oracle

    all_legs = (args.workload is None and args.mode == "step" and not args.ingest_tokens and not args.prefill_tokens
                and not args.sweep_step_times)
    if not all_legs and args.workload is None:
        args.workload = "cfg2"
    if args.ingest_tokens > 0:
        from paper_2603_02599_amd import workloads as wl
        shape = {"cfg2": wl.LLAMA_8B, "cfg3": wl.LLAMA_8B, "cfg5a": wl.QWEN_14B, "cfg5b": wl.QWEN_14B, "small": wl.SMALL128}[args.workload]
        n = args.ingest_tokens
        pages = (n + 15) // 16
        cfg = sun.make_cfg(shape, "bf16")
        mem = torch.empty(sun.sun_kv_pool_bytes(cfg, pages) // 2, dtype=torch.bfloat16, device="cuda")
        pool = sun.sun_kv_pool_create(cfg, mem, 16, 1)
        k = torch.randn((shape.n_layers, n, shape.n_kv_heads, shape.head_dim), device="cuda").to(torch.bfloat16)
        v = torch.randn_like(k)
        row = torch.randperm(pages, device="cuda").to(torch.int32)
        for _ in range(args.warmup):
            sun.sun_kv_pool_ingest(pool, 0, k, v, 0, row)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            sun.sun_kv_pool_ingest(pool, 0, k, v, 0, row)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        moved = 2.0 * 2 * k.numel() * 2   # K and V, read and written, 2 bytes each
        print(json.dumps({"metric": "kv-ingest tokens/sec", "value": n / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
                          "dtype": "bf16 (byte copy)", "data": "synthetic",
                          "config": {"workload": f"one prompt cache of {n} tokens, {shape.name} shape, shuffled pages"},
                          "roofline": {"bound": "hbm", "kernel": "kv_ingest_kernel", "achieved": moved / (ms * 1e-3) / 1e9,
                                       "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                       "traffic": None, "bytes_per_launch": moved}}))
        return
    if args.prefill_tokens > 0:
        from paper_2603_02599_amd import workloads as wl
        shape = {"cfg2": wl.LLAMA_8B, "cfg3": wl.LLAMA_8B, "cfg5a": wl.QWEN_14B, "cfg5b": wl.QWEN_14B, "small": wl.SMALL128}[args.workload]
        n = args.prefill_tokens
        pages = n // 16 + 1
        cfg = sun.make_cfg(shape, "bf16")
        mem = torch.empty(sun.sun_kv_pool_bytes(cfg, pages) // 2, dtype=torch.bfloat16, device="cuda")
        pool = sun.sun_kv_pool_create(cfg, mem, 16, 1)
        w = wl.make_weights(shape, "bf16", "cuda", 11)
        weights = sun.sun_weights_create(cfg, w)
        toks = torch.randint(0, shape.vocab, (n,), device="cuda", dtype=torch.int32)
        row = torch.randperm(pages, device="cuda").to(torch.int32)
        ws = torch.empty(sun.sun_prefill_workspace_bytes(cfg, n, pages), dtype=torch.uint8, device="cuda")
        logits = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
        nxt = torch.empty(1, dtype=torch.int32, device="cuda")
        for _ in range(args.warmup):
            sun.sun_prefill(pool, weights, toks, row, 0, 0, logits, nxt, ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            sun.sun_prefill(pool, weights, toks, row, 0, 0, logits, nxt, ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        print(json.dumps({"metric": "prefill prompt tokens/sec", "value": n / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
                          "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": f"one prompt of {n} tokens, {shape.name} shape, shuffled pages, "
                                                 "through the decode step's kernels in blocks of 256 rows"}}))
        return
    if args.sweep_step_times:
        from paper_2603_02599_amd import workloads as wl
        shape = {"cfg2": wl.LLAMA_8B, "cfg3": wl.LLAMA_8B, "cfg5a": wl.QWEN_14B, "cfg5b": wl.QWEN_14B, "small": wl.SMALL128}[args.workload]
        shared = H.DeviceWeights(shape, "bf16", 11, quant_mode=args.quant)
        fn = sun.sun_qdecode_step if args.quant else sun.sun_decode_step
        points = []
        for B in (1, 4, 16, 32, 64, 128, 256):
            for L in (256, 1024, 2048, 4096, 8192):
                if B * L > (1 << 20):
                    continue
                work = wl.make_workload("cfg2", shape=shape, batch=B, lo=L, hi=L, seed=100 + B)
                case = H.DeviceCase(work, shared=shared)
                host_lens = work.seq_lens.copy()
                for _ in range(3):
                    fn(case.pool, case.weights, case.tokens, case.tables, case.lens, case.ids, None, case.next, case.ws,
                       seq_lens_host=host_lens)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    fn(case.pool, case.weights, case.tokens, case.tables, case.lens, case.ids, None, case.next, case.ws,
                       seq_lens_host=host_lens)
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t0) * 1e3 / args.steps
                points.append({"batch": B, "len": L, "kv_tokens": int(work.kv_tokens_read), "ms_per_step": ms})
                print(f"[sweep] batch {B} len {L}: {ms:.3f} ms", file=sys.stderr, flush=True)
                del case
                torch.cuda.empty_cache()
        print(json.dumps({"what": "decode step time", "shape": shape.name, "quant": args.quant, "device": "MI355X",
                          "steps_per_point": args.steps, "points": points}))
        return
    if args.mode == "serve":
        return bench_serve(args, sun, H)
    if args.mode == "run":
        return bench_run_setup(args, sun, H)
    if args.workload is not None:
        print(json.dumps(step_leg(args, sun, H, args.workload, args.quant, None, args.cpu_sample)))
        return
    # Default: the whole metric in one process.  The headline line is cfg2 with bf16 weights; the same step with
    # 4-bit weights, and both at batch 256 (cfg3), ride along under "legs", each with its own roofline.  The
    # two weight sets are built once and shared by the workloads.
    from paper_2603_02599_amd import workloads as wl
    legs = {}
    head = None
    for quant in (None, args.quant or "asym"):
        shared = H.DeviceWeights(wl.LLAMA_8B, "bf16", wl.SEED_BASE + 3, quant_mode=quant)
        if quant:
            for k in sun.QUANT_KEYS:
                shared.w[k] = None
            torch.cuda.empty_cache()
        for name in ("cfg2", "cfg3"):
            first = name == "cfg2" and quant is None
            leg = step_leg(args, sun, H, name, quant, shared, args.cpu_sample if first else 0)
            if first:
                head = leg
            else:
                legs[f"{name}_{'qsun' if quant else 'bf16'}"] = {k: leg[k] for k in (
                    "value", "unit", "ms_per_step", "step_ms_p10_p50_p90", "dtype", "config", "algorithmic_GB_per_step",
                    "step_GBps", "step_frac_of_hbm_peak", "roofline", "kernels")}
        del shared
        torch.cuda.empty_cache()
    b16, q4 = head["ms_per_step"], legs["cfg2_qsun"]["ms_per_step"]
    head["legs"] = legs
    head["qsun_step_time_gain"] = {"cfg2": 1.0 - q4 / b16, "cfg3": 1.0 - legs["cfg3_qsun"]["ms_per_step"] / legs["cfg3_bf16"]["ms_per_step"]}
    print(json.dumps(head))


def projection_figures(shape, work, quant, kernels):
    """Per projection: weight bytes per second, and the method's arithmetic (2 N K per row: the second activation
    plane of the kernels is not counted) per second against the matrix-core peak of the operand type the kernel
    multiplies in; `bound` names the larger of the two floors (weights once from HBM at 8 TB/s, arithmetic at
    the matrix-core peak)."""
    el = 4.0 if work.dtype == "f32" else 2.0
    b_w = w4_bytes_per_weight(quant) if quant else el
    H_, QD, KD, F = shape.hidden, shape.q_dim, shape.kv_dim, shape.ffn
    mats = {"qkv_proj": ((QD + 2 * KD), H_, b_w, quant), "o_proj": (H_, QD, b_w, quant), "gate_up_proj": (2 * F, H_, b_w, quant),
            "down_proj": (H_, F, b_w, quant), "lm_head": (shape.vocab, H_, el, None)}
    for k, (N, K, bpw, q) in mats.items():
        if k not in kernels:
            continue
        t = kernels[k]["avg_us"] * 1e-6
        nbytes, flops = N * K * bpw, 2.0 * work.batch * N * K
        peak = MFMA_PEAK_TFLOPS["int8" if q else "bf16"]
        kernels[k]["weight_GBps"] = nbytes / t / 1e9
        kernels[k]["frac_of_hbm_peak"] = nbytes / t / 1e9 / HBM_PEAK_GBS
        if work.dtype != "f32":
            kernels[k]["TFLOPs"] = flops / t / 1e12
            kernels[k]["mfma_operands"] = "int8" if q else "bf16"
            kernels[k]["frac_of_mfma_peak"] = flops / t / 1e12 / peak
            kernels[k]["bound"] = "mfma" if flops / (peak * 1e12) > nbytes / (HBM_PEAK_GBS * 1e9) else "hbm"


def step_leg(args, sun, H, workload, quant, shared, cpu_sample):
    """Times K independent calls of the decode step on one resident workload; returns the JSON object."""
    import torch
    work, desc = build_workload(workload)
    shape = work.shape
    t_setup = time.perf_counter()
    if shared is not None:
        case = H.DeviceCase(work, shared=shared)
    else:
        case = H.DeviceCase(work, quant_mode=quant)
        if quant:  # the dense projection sources are no longer needed on the device
            for k in sun.QUANT_KEYS:
                case.w[k] = None
    torch.cuda.synchronize()
    print(f"[bench] {workload} quant={quant}: setup {time.perf_counter() - t_setup:.1f} s; pool {work.n_pages} pages, "
          f"{work.kv_tokens_read} KV tokens read per layer-step", file=sys.stderr, flush=True)
    host_lens = work.seq_lens.copy()
    fn = sun.sun_qdecode_step if quant else sun.sun_decode_step

    def one_step(flags=0):
        # seq_lens is held fixed so every step overwrites the same slot and moves identical bytes
        fn(case.pool, case.weights, case.tokens, case.tables, case.lens, case.ids, case.logits, case.next, case.ws,
           seq_lens_host=host_lens, flags=flags)

    graph = None
    if args.graph:
        one_step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one_step()
        run = graph.replay
    else:
        run = one_step

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        run()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_step = np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps)])
    ms_per_step = wall * 1e3 / args.steps

    alg = algorithmic_bytes(shape, work, quant)
    roof = None
    kernels = {}
    launches_per_step = None
    if not args.no_profile:
        sun.sun_profile_reset()
        for _ in range(args.steps):
            one_step(flags=sun.SUN_PROFILE)
        torch.cuda.synchronize()
        prof = sun.sun_profile_read()
        sun.sun_profile_reset()
        for k, v in prof.items():
            if v["launches"]:
                kernels[k] = {"avg_us": 1e3 * v["ms"] / v["launches"], "launches_per_step": v["launches"] // args.steps,
                              "ms_per_step": v["ms"] / args.steps}
        launches_per_step = sum(v["launches_per_step"] for v in kernels.values())
        att = prof["attn_split"]
        # one launch = one layer: K and V of every cached position of every request, once
        per_launch = float(work.kv_tokens_read) * 2 * shape.n_kv_heads * shape.head_dim * 2
        avg_s = att["ms"] / att["launches"] * 1e-3
        roof = {"bound": "hbm", "kernel": "attn_split_kernel", "achieved": per_launch / avg_s / 1e9,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": per_launch / avg_s / 1e9 / HBM_PEAK_GBS,
                "traffic": measured_traffic_bytes(workload, quant), "traffic_source": "profiles/ (counter runs of this command, not this run)",
                "bytes_per_launch": per_launch, "avg_launch_us": avg_s * 1e6}
        projection_figures(shape, work, quant, kernels)

    cpu = None
    if cpu_sample > 0:
        cpu = cpu_baseline(case, work, cpu_sample)

    out = {
        "metric": "shared-decode tokens/sec",
        "value": work.batch / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "tpot_ms": ms_per_step,
        "step_ms_p10_p50_p90": [float(np.percentile(per_step, p)) for p in (10, 50, 90)],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("f32" if work.dtype == "f32" else "bf16") if not quant else "bf16 activations, 4-bit group-128 weights",
        "data": "synthetic",
        "config": {"workload": f"{workload}: {desc}", "shape": shape.name, "batch": work.batch,
                   "quant": quant, "kv_tokens": work.kv_tokens_read, "graph": bool(args.graph)},
        "algorithmic_GB_per_step": alg["total"] / 1e9,
        "step_GBps": alg["total"] / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": alg["total"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "launches_per_step": launches_per_step,
        "roofline": roof,
        "kernels": kernels,
        "cpu_baseline": cpu,
    }
    del case
    torch.cuda.empty_cache()
    return out


def bench_run_setup(args, sun, H):
    """--mode run: widen the page tables for the tokens the run generates, then time it."""
    import torch
    workload = args.workload or "cfg2"
    work, desc = build_workload(workload)
    shape = work.shape
    grow = args.steps + args.warmup + 8  # + a short per-kernel timing pass after the timed run
    cols = (int(work.seq_lens.max()) + grow) // 16 + 1
    wide = np.full((work.batch, cols), -1, np.int32)
    wide[:, :work.max_pages] = work.page_tables
    referenced = np.zeros(work.n_pages, bool)
    referenced[work.page_tables[work.page_tables >= 0]] = True
    free_list = np.flatnonzero(~referenced).astype(np.int32)
    assert len(free_list) >= work.batch * (grow // 16 + 1), "pool has too few spare pages for this output length"
    work.page_tables = wide
    case = H.DeviceCase(work, quant_mode=args.quant)
    if args.quant:
        for k in sun.QUANT_KEYS:
            case.w[k] = None
    torch.cuda.synchronize()
    args.workload = workload
    return bench_run(args, sun, case, work, shape, desc, free_list)


if __name__ == "__main__":
    main()
