"""Host-side simulator of decode-worker placement in multi-model disaggregated serving (Section 3.2.3,
Appendix A.2): N task-specific models, each with its own prefill worker, and decode workers that are either
isolated per model (the baseline, one decode worker per model) or pooled and model-agnostic (SUN: any of K
workers can decode any request, because all tasks share the one frozen decode module).

Every decode worker runs the continuous-batching loop of `sun_decode_serve` (rows retire at their output
length, waiting requests enter first in, first out).  The time of one iteration comes from step times
measured on one MI355X with `bench.py --sweep-step-times` (a JSON table of batch size, cache length and
milliseconds): t(B, T) = a(B) + b * T, a(B) interpolated linearly between the measured batch sizes, T the
number of cached tokens the step reads.  Everything else is bookkeeping in simulated time, so the
simulator says how the *measured* single-GPU step scales into the system-level curves of Figures 3 and 4
(throughput per GPU, interactivity = 1000 / TPOT_ms, achieved / offered load), not how any real
multi-GPU system performed.

Traffic follows Appendix A.2: open-loop Poisson arrivals at a total rate R split over the models by
P(i) = i^-alpha / sum_j j^-alpha, fixed input and output lengths, metrics over requests that complete
inside a measurement window after a grace period.

No GPU is needed here; nothing in the decode path imports this module.
"""
from __future__ import annotations

import argparse
import heapq
import json
import os
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np

DATA_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "data")


def zipf_split(n_models: int, alpha: float) -> np.ndarray:
    """Share of the total request rate per model, by popularity rank (Appendix A.2)."""
    w = np.arange(1, n_models + 1, dtype=np.float64) ** (-alpha)
    return w / w.sum()


class StepTimeModel:
    """t_ms(B, T) = a(B) + b * T fitted by least squares to measured points; a(B) is one intercept per
    measured batch size, interpolated linearly in B in between (and held constant outside)."""

    def __init__(self, points: Sequence[Dict[str, float]]):
        bs = sorted({int(p["batch"]) for p in points})
        col = {b: i for i, b in enumerate(bs)}
        A = np.zeros((len(points), len(bs) + 1))
        y = np.zeros(len(points))
        for r, p in enumerate(points):
            A[r, col[int(p["batch"])]] = 1.0
            A[r, -1] = float(p["kv_tokens"])
            y[r] = float(p["ms_per_step"])
        sol, *_ = np.linalg.lstsq(A, y, rcond=None)
        self.batches = np.array(bs, dtype=np.float64)
        self.intercepts = sol[:-1]
        self.ms_per_kv_token = float(sol[-1])
        self.max_rel_err = float(np.max(np.abs(A @ sol - y) / y))

    @classmethod
    def from_file(cls, path: str) -> "StepTimeModel":
        with open(path) as f:
            return cls(json.load(f)["points"])

    def ms(self, batch: int, kv_tokens: float) -> float:
        return float(np.interp(batch, self.batches, self.intercepts)) + self.ms_per_kv_token * kv_tokens


@dataclass
class Request:
    model: int
    arrival: float        # s, when its prompt cache is ready on the decode side
    isl: int
    osl: int
    first_token: float = -1.0
    last_token: float = -1.0
    generated: int = 0


class Worker:
    """One decode GPU: `rows` batch rows, a first-in first-out queue, one iteration at a time."""

    def __init__(self, rows: int, model: StepTimeModel):
        self.rows, self.model = rows, model
        self.active: List[Request] = []
        self.queue: List[Request] = []
        self.busy_until: Optional[float] = None

    def load(self) -> int:
        return len(self.active) + len(self.queue)

    def start_step(self, now: float) -> Optional[float]:
        """Admits from the queue, then starts an iteration if any row is occupied; returns its end time."""
        while self.queue and len(self.active) < self.rows:
            self.active.append(self.queue.pop(0))
        if not self.active:
            self.busy_until = None
            return None
        kv = sum(r.isl + r.generated + 1 for r in self.active)
        self.busy_until = now + 1e-3 * self.model.ms(len(self.active), kv)
        return self.busy_until

    def finish_step(self, now: float, done: List[Request], window, counters) -> None:
        still = []
        for r in self.active:
            r.generated += 1
            if r.first_token < 0:
                r.first_token = now
            r.last_token = now
            if window[0] <= now < window[1]:
                counters["tokens"] += 1
            if r.generated >= r.osl:
                done.append(r)
            else:
                still.append(r)
        self.active = still


def simulate(step_model: StepTimeModel, policy: str, n_models: int = 4, n_workers: int = 4, rps_total: float = 2.0,
             alpha: float = 0.0, isl: int = 1024, osl: int = 512, rows: int = 64, grace_s: float = 30.0,
             window_s: float = 60.0, seed: int = 0) -> Dict[str, float]:
    """policy "isolated": model i decodes on worker i (n_workers must equal n_models); "shared": a request goes
    to the worker with the fewest requests running or queued when its cache is ready, lowest index on ties,
    whatever its model.  Returns throughput (output tokens/s inside the window), TPOT (mean over requests that
    completed inside the window, ms), interactivity (1000 / TPOT), achieved / offered request rate."""
    if policy not in ("isolated", "shared"):
        raise ValueError(policy)
    if policy == "isolated" and n_workers != n_models:
        raise ValueError("the isolated baseline has one decode worker per model")
    rng = np.random.default_rng(seed)
    horizon = grace_s + window_s
    window = (grace_s, horizon)
    shares = zipf_split(n_models, alpha)
    events = []   # (time, order, kind, payload)
    order = 0
    for m in range(n_models):
        rate = rps_total * shares[m]
        t = 0.0
        while rate > 0:
            t += rng.exponential(1.0 / rate)
            if t >= horizon:
                break
            events.append((t, order, 0, Request(m, t, isl, osl)))
            order += 1
    heapq.heapify(events)
    workers = [Worker(rows, step_model) for _ in range(n_workers)]
    done: List[Request] = []
    counters = {"tokens": 0}
    offered = len(events)
    while events:
        now, _, kind, payload = heapq.heappop(events)
        if now >= horizon:
            break
        if kind == 0:
            req = payload
            w = req.model if policy == "isolated" else min(range(n_workers), key=lambda i: (workers[i].load(), i))
            workers[w].queue.append(req)
            if workers[w].busy_until is None:
                end = workers[w].start_step(now)
                heapq.heappush(events, (end, order, 1, w))
                order += 1
        else:
            w = payload
            workers[w].finish_step(now, done, window, counters)
            end = workers[w].start_step(now)
            if end is not None:
                heapq.heappush(events, (end, order, 1, w))
                order += 1
    in_window = [r for r in done if window[0] <= r.last_token < window[1] and r.generated > 1]
    tpot = float(np.mean([(r.last_token - r.first_token) / (r.generated - 1) for r in in_window])) * 1e3 if in_window else float("nan")
    return {"policy": policy, "n_workers": n_workers, "alpha": alpha, "isl": isl, "osl": osl, "rps": rps_total,
            "throughput_tok_s": counters["tokens"] / window_s, "tpot_ms": tpot,
            "interactivity_tok_s": 1000.0 / tpot if tpot == tpot else float("nan"),
            "completed_in_window": len(in_window),
            "achieved_over_offered": len(in_window) / (rps_total * window_s) if rps_total > 0 else float("nan"),
            "offered_requests": offered,
            "backlog_at_end": sum(w.load() for w in workers)}


def closed_loop(step_model: StepTimeModel, concurrency: int, isl: int, osl: int, ttft_ms: float = 0.0) -> Dict[str, float]:
    """One decode worker kept at `concurrency` requests in lockstep (the closed-loop client of the paper's
    concurrency table): TPOT is the mean step time over the osl - 1 steps after the first token, with every
    row at length isl + t; a request takes ttft + (osl - 1) * TPOT, so the worker delivers
    TPUT = concurrency * osl / (ttft + (osl - 1) * TPOT) output tokens per second."""
    steps = [step_model.ms(concurrency, concurrency * (isl + t + 1)) for t in range(1, osl)]
    tpot = float(np.mean(steps)) if steps else step_model.ms(concurrency, concurrency * (isl + 1))
    total_ms = ttft_ms + (osl - 1) * tpot
    return {"concurrency": concurrency, "isl": isl, "osl": osl, "tpot_ms": tpot, "interactivity_tok_s": 1000.0 / tpot,
            "throughput_tok_s": throughput_from_latencies(concurrency, osl, ttft_ms, tpot) if total_ms > 0 else float("nan")}


def throughput_from_latencies(concurrency: int, osl: int, ttft_ms: float, tpot_ms: float) -> float:
    """Output tokens per second of `concurrency` requests in flight, each taking ttft + (osl - 1) * TPOT."""
    return concurrency * osl / ((ttft_ms + (osl - 1) * tpot_ms) * 1e-3)


def saturation_rps(step_model: StepTimeModel, isl: int, osl: int, rows: int) -> float:
    """Requests/s one worker sustains with every row busy: rows / (osl * step time at the mean cache length)."""
    t = 1e-3 * step_model.ms(rows, rows * (isl + osl / 2.0))
    return rows / (osl * t)


def figure3(step_model: StepTimeModel, load: float = 0.45, rows: int = 64, seed: int = 1) -> List[Dict[str, float]]:
    """The sweep of Figure 3: isolated 4x(1P/1D) against pooled 4P/KD for K = 4..1, alpha in {0, 1.5}, output
    lengths 128, 256, 512.  The offered rate is `load` times what the four isolated decode workers sustain in
    total (the paper fixes a rate on its own hardware; here it is set relative to the measured capacity)."""
    out = []
    for alpha in (0.0, 1.5):
        for osl in (128, 256, 512):
            rps = load * 4 * saturation_rps(step_model, 1024, osl, rows)
            runs = [("4x(1P/1D)", "isolated", 4)] + [(f"4P/{k}D", "shared", k) for k in (4, 3, 2, 1)]
            for name, policy, k in runs:
                r = simulate(step_model, policy, 4, k, rps, alpha, 1024, osl, rows, seed=seed)
                r["config"] = name
                r["throughput_per_gpu"] = r["throughput_tok_s"] / (4 + k)
                out.append(r)
    return out


def figure4(step_model: StepTimeModel, load: float = 0.6, rows: int = 64, seed: int = 1) -> List[Dict[str, float]]:
    """The skew sweep of Figure 4: input 1024, output 2048, isolated 4x(1P/1D) against pooled 4P/4D, alpha 0..2."""
    out = []
    rps = load * 4 * saturation_rps(step_model, 1024, 2048, rows)
    for alpha in (0.0, 0.5, 1.0, 1.5, 2.0):
        for name, policy in (("4x(1P/1D)", "isolated"), ("4P/4D", "shared")):
            r = simulate(step_model, policy, 4, 4, rps, alpha, 1024, 2048, rows, grace_s=60.0, window_s=180.0, seed=seed)
            r["config"] = name
            out.append(r)
    return out


def _table(rows: List[Dict[str, float]]) -> str:
    head = f"{'config':<10} {'alpha':>5} {'osl':>5} {'rps':>7} {'tput tok/s':>11} {'tput/GPU':>9} {'TPOT ms':>8} {'interact.':>9} {'ach/off':>7}"
    lines = [head]
    for r in rows:
        per_gpu = r.get("throughput_per_gpu", r["throughput_tok_s"] / (4 + r["n_workers"]))
        lines.append(f"{r['config']:<10} {r['alpha']:>5.1f} {r['osl']:>5d} {r['rps']:>7.2f} {r['throughput_tok_s']:>11.0f} "
                     f"{per_gpu:>9.0f} {r['tpot_ms']:>8.2f} {r['interactivity_tok_s']:>9.1f} {r['achieved_over_offered']:>7.2f}")
    return "\n".join(lines)


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--step-times", default=os.path.join(DATA_DIR, "step_times_llama8b_bf16_mi355x.json"))
    ap.add_argument("--figure", type=int, choices=[3, 4], default=3)
    ap.add_argument("--concurrency-table", action="store_true",
                    help="instead of a figure: TPOT and throughput at concurrency 1/4/16 and input 1024/2048/4096, output "
                         "1024 (the grid of the paper's concurrency table), from the measured step times alone (TTFT 0)")
    ap.add_argument("--load", type=float, default=None,
                    help="offered rate as a fraction of what four isolated decode workers sustain (default 0.45 for "
                         "figure 3, 0.6 for figure 4)")
    ap.add_argument("--rows", type=int, default=64)
    ap.add_argument("--seed", type=int, default=1)
    args = ap.parse_args()
    model = StepTimeModel.from_file(args.step_times)
    print(f"step-time model: {model.ms_per_kv_token * 1e3:.4f} us per cached token + a(B); worst fit error {model.max_rel_err:.1%}")
    if args.concurrency_table:
        print(f"{'isl':>5} {'conc':>5} {'TPOT ms':>8} {'TPUT tok/s':>11}")
        for isl in (1024, 2048, 4096):
            for c in (1, 4, 16):
                r = closed_loop(model, c, isl, 1024)
                print(f"{isl:>5d} {c:>5d} {r['tpot_ms']:>8.2f} {r['throughput_tok_s']:>11.1f}")
        return
    load = args.load if args.load is not None else (0.45 if args.figure == 3 else 0.6)
    rows = (figure3 if args.figure == 3 else figure4)(model, load, args.rows, args.seed)
    print(_table(rows))


if __name__ == "__main__":
    main()
