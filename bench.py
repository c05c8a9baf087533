#!/usr/bin/env python3
"""Throughput of the merged multi-task serving forward pass on one MI355X.

One step = the forward pass over one synthetic request batch (embeddings, shared trunk once, all task
branches, poolers and heads), inputs and weights already resident in HBM.  Request batches keep the
workload's batch size (32 sequences for `base`); the server hands several of them to the library in one
call (mt_forward_multi, --requests-per-call), which runs them as one combined batch so that every
contraction has enough rows to fill the chip.  Prints ONE JSON line: sequences/s (whole job), the
roofline position of the dominant kernel (the bf16 MFMA contraction) from per-launch HIP events recorded
inside the library on the forward's stream, the CPU oracle timed on a bounded sample of the same workload
on this host, and short runs of the other workloads (`workloads`).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16 matrix-core peak
PEAK_FP8_MFMA_TFLOPS = 5000.0      # ... and dense FP8
PEAK_FP32_VALU_TFLOPS = 157.3


def layer_kinds(spec):
    """(#layers evaluated on every token row, #layers evaluated on the first token only).

    Only position 0 of a branch's output feeds its pooler, so the library computes the last own layer
    of every branch for that position alone (its keys and values still come from every row)."""
    tok = [getattr(t, "token_level", False) for t in spec.tasks]       # a tagging task needs every row of its last layer
    n_full = spec.n_trunk_layers + sum(t.n_layers if k else max(t.n_layers - 1, 0) for t, k in zip(spec.tasks, tok))
    n_first = sum(1 for t, k in zip(spec.tasks, tok) if t.n_layers >= 1 and not k)
    return n_full, n_first


def gemm_flops_per_forward(spec, rows, batch):
    """EXECUTED FLOPs of the linear layers, per profile class, for one forward over `rows` token rows.

    The library drops padded positions before the first layer, so `rows` is the number of real
    tokens of the batch (sum of sequence lengths), not batch*seq.  A first-token-only layer (bf16 path)
    projects no keys or values: per sequence it computes the query, Wk^T q per head, the raw scores
    x_j . (Wk^T q) over the sequence's rows, Wv applied to the per-head weighted row sums, and the output
    projection and feed-forward layers on one row."""
    H, F, A = spec.hidden, spec.ffn, spec.heads
    n_full, n_first = layer_kinds(spec)
    kvfree = spec.precision in ("bf16", "fp8", "fp8_all") and A <= 16
    first = 2.0 * batch * (2 * H * H + 2 * H * F)                      # query, output projection, FFN1, FFN2
    qkv_last = 0.0
    if kvfree:
        first += 2.0 * batch * 2 * H * H + 2.0 * rows * H * A          # Wk^T q and Wv xbar (H^2 each), raw scores
    else:
        qkv_last = 2.0 * rows * 2 * H * H                              # K|V projection over all rows
    return {"gemm_qkv": n_full * 2.0 * rows * 3 * H * H + n_first * qkv_last,
            "gemm_out": n_full * 2.0 * rows * H * H,
            "gemm_ffn1": n_full * 2.0 * rows * F * H,
            "gemm_ffn2": n_full * 2.0 * rows * H * F,
            "gemm_first": n_first * first}


def forward(model, batch, out=None, out_tokens=None):
    """One forward of the whole model: the token-level entry point when the model has tagging tasks."""
    if model.n_token_logits > 0:
        return model.forward_tokens(*batch, out=out, out_tokens=out_tokens)[0]
    return model.forward(*batch, out=out)


def host_description():
    """Logical CPUs visible to this process and the processor's model name, for reading the CPU baseline."""
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return {"logical_cpus": os.cpu_count(), "usable_cpus": usable, "model": model}


TRAFFIC_SOURCES = ("gemm_bf16.hip", "gemm_bf16_persist.hip", "mt_model.cpp")     # kernels and the host code that picks launch shapes


def traffic_source_hash():
    """One hash over the sources that decide the tiled contractions' HBM traffic: both kernels and the scheduler."""
    import hashlib
    h = hashlib.sha256()
    for f in TRAFFIC_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2107_05377_amd", "csrc", f), "rb").read())
    return h.hexdigest()


def stored_traffic(workload_name, requests_per_call):
    """HBM-side bytes per launch of the tiled contraction kernels from the committed counter summary (stored, not
    measured in this run), or None when there is none for this workload and call size or any of TRAFFIC_SOURCES has
    changed since the counters were taken."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", f"bench_{workload_name}_hbm_traffic*.txt"))):
        vals = {}
        for line in open(path):
            if " = " in line:
                k, v = line.split(" = ", 1)
                vals[k.strip()] = v.split()[0]
        if "traffic_bytes_per_launch" not in vals or int(vals.get("requests_per_call", "1")) != requests_per_call:
            continue
        if vals.get("kernel_source_sha256") != traffic_source_hash():
            continue
        return float(vals["traffic_bytes_per_launch"])
    return None


def latency_sweep(mt, ms, spec, model, calls):
    """One forward at a time, host clock around launch + stream sync, per batch size: p50 / p99 / sequences/s."""
    import numpy as np
    import torch
    res = []
    for b in (1, 2, 4, 8):
        if b > spec.batch:
            continue
        sets = []
        for i in range(8):
            ids, mask, _ = ms.make_inputs(spec, batch=b, batch_index=i)
            sets.append((torch.from_numpy(ids).cuda(), torch.from_numpy(mask).cuda()))
        out = torch.zeros((b, model.n_logits), dtype=torch.float32, device="cuda")
        tok = torch.zeros((b, spec.seq, model.n_token_logits), dtype=torch.float32, device="cuda") if model.n_token_logits else None
        for i in range(50):
            forward(model, sets[i % 8], out, tok)
        torch.cuda.synchronize()
        t = np.empty(calls)
        for i in range(calls):
            t0 = time.perf_counter()
            forward(model, sets[i % 8], out, tok)
            torch.cuda.synchronize()
            t[i] = time.perf_counter() - t0
        ent = {"batch": b, "calls": calls, "p50_ms": float(np.percentile(t, 50) * 1e3), "p99_ms": float(np.percentile(t, 99) * 1e3),
               "mean_ms": float(t.mean() * 1e3), "sequences_per_s": float(b / t.mean())}
        # the same forward captured once as a HIP graph and replayed (the forward only enqueues kernels: nothing in it
        # allocates, copies, clears or waits); every replay is checked against the launched result
        forward(model, sets[0], out, tok)
        torch.cuda.synchronize()
        launched = out.clone()
        out_g = torch.zeros_like(out)
        tok_g = torch.zeros_like(tok) if tok is not None else None
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            forward(model, sets[0], out_g, tok_g)
        same = True
        n_rep = max(50, calls // 4)
        tg = np.empty(n_rep)
        for i in range(n_rep):
            if i < 3:
                out_g.zero_()
                forward(model, sets[1], out, tok)          # launched work between the replays
                torch.cuda.synchronize()
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            tg[i] = time.perf_counter() - t0
            if i < 3:
                same = same and bool(torch.equal(out_g, launched))
        ent["graph_replay"] = {"calls": n_rep, "p50_ms": float(np.percentile(tg, 50) * 1e3), "p99_ms": float(np.percentile(tg, 99) * 1e3),
                               "bit_identical_to_launched": same}
        del graph
        res.append(ent)
    return res


def qps_stream(ms, spec, model, rates, n_requests, seed=7):
    """Open-loop request stream (Appendix E reports the 99th-percentile latency of the deployed model under a
    request rate): single-sequence requests arrive as a Poisson process; the server loop takes whatever has
    arrived (at most the model's batch size), copies the ids and masks from pinned host memory, runs one forward,
    copies the logits back and waits for them.  A request's latency runs from its arrival to that moment, so it
    includes queueing, both PCIe copies and the launch path."""
    import numpy as np
    import torch
    B, S = spec.batch, spec.seq
    pool_ids, pool_mask = [], []
    for i in range(8):
        ids, mask, _ = ms.make_inputs(spec, batch=B, batch_index=i)
        pool_ids.append(ids)
        pool_mask.append(mask)
    pool_ids, pool_mask = np.concatenate(pool_ids), np.concatenate(pool_mask)         # 8*B single-sequence requests
    h_ids = torch.empty((B, S), dtype=torch.int32).pin_memory()
    h_mask = torch.empty((B, S), dtype=torch.int32).pin_memory()
    d_ids = torch.empty((B, S), dtype=torch.int32, device="cuda")
    d_mask = torch.empty((B, S), dtype=torch.int32, device="cuda")
    out = torch.zeros((B, model.n_logits), dtype=torch.float32, device="cuda")
    tok = torch.zeros((B, S, model.n_token_logits), dtype=torch.float32, device="cuda") if model.n_token_logits else None
    h_out = torch.empty((B, model.n_logits), dtype=torch.float32).pin_memory()
    h_tok = torch.empty((B, S, model.n_token_logits), dtype=torch.float32).pin_memory() if model.n_token_logits else None
    np_ids, np_mask = h_ids.numpy(), h_mask.numpy()

    def serve(req):
        n = len(req)
        np_ids[:n] = pool_ids[req]
        np_mask[:n] = pool_mask[req]
        d_ids[:n].copy_(h_ids[:n], non_blocking=True)
        d_mask[:n].copy_(h_mask[:n], non_blocking=True)
        forward(model, (d_ids[:n], d_mask[:n]), out[:n], tok[:n] if tok is not None else None)
        h_out[:n].copy_(out[:n], non_blocking=True)
        if tok is not None:
            h_tok[:n].copy_(tok[:n], non_blocking=True)
        torch.cuda.synchronize()

    for n in (1, B):                                   # warm both ends of the batch range
        for _ in range(20):
            serve(np.arange(n))
    res = []
    rng = np.random.default_rng(seed)
    for rate in rates:
        arrive = np.cumsum(rng.exponential(1.0 / rate, n_requests))
        which = rng.integers(0, len(pool_ids), n_requests)
        done = np.empty(n_requests)
        nxt, n_batches = 0, 0
        t0 = time.perf_counter()
        while nxt < n_requests:
            now = time.perf_counter() - t0
            hi = min(int(np.searchsorted(arrive, now, side="right")), nxt + B)
            if hi == nxt:                                # nothing waiting: idle until the next arrival
                while time.perf_counter() - t0 < arrive[nxt]:
                    pass
                continue
            serve(which[nxt:hi])
            done[nxt:hi] = time.perf_counter() - t0
            nxt = hi
            n_batches += 1
        lat = (done - arrive) * 1e3
        res.append({"offered_qps": float(rate), "served_qps": float(n_requests / done[-1]), "requests": int(n_requests),
                    "mean_batch": float(n_requests / n_batches), "p50_ms": float(np.percentile(lat, 50)),
                    "p99_ms": float(np.percentile(lat, 99)), "max_ms": float(lat.max())})
    return res


class Served:
    """A loaded model plus the replicas, streams and request batches one measurement needs."""

    def __init__(self, mt, ms, spec, B, R, n_fly, n_batches=8):
        import numpy as np
        import torch
        self.mt, self.spec, self.B, self.R, self.S = mt, spec, B, max(1, R), spec.seq
        self.multi = self.R > 1
        t0 = time.time()
        self.model, _ = mt.load_synthetic(spec, max_batch=B * self.R, max_seq=spec.seq)
        self.load_s = time.time() - t0
        self.n_batches = n_batches
        self.batches, self.real_tokens, self.sq_lengths = [], [], []
        for i in range(n_batches):
            ids, mask, lengths = ms.make_inputs(spec, batch=B, batch_index=i)
            self.batches.append((torch.from_numpy(ids).cuda(), torch.from_numpy(mask).cuda()))
            self.real_tokens.append(int(mask.sum()))
            self.sq_lengths.append(float((lengths.astype(np.float64) ** 2).sum()))
        self.stream = torch.cuda.current_stream()
        self.n_fly = max(1, n_fly)
        self.models = [self.model] + [self.model.replica() for _ in range(self.n_fly - 1)]
        self.streams = [torch.cuda.Stream() for _ in range(self.n_fly)]          # default priority
        m = self.model
        self.outs = [[torch.zeros((B, m.n_logits), dtype=torch.float32, device="cuda") for _ in range(self.R)] for _ in range(self.n_fly)]
        self.tok_outs = [torch.zeros((B, self.S, m.n_token_logits), dtype=torch.float32, device="cuda") if m.n_token_logits else None
                         for _ in range(self.n_fly)]

    def call(self, j, first, n):
        """One library call on replica j: request batches first .. first+n-1 (indices into the cycled batches)."""
        reqs = [self.batches[(first + r) % self.n_batches] for r in range(n)]
        if self.multi:
            self.models[j].forward_multi(reqs, outs=self.outs[j][:n])
        else:
            forward(self.models[j], reqs[0], self.outs[j][0], self.tok_outs[j])

    def run_steps(self, k, fly):
        """k request batches, R per call, calls round-robin over the replicas' streams; elapsed milliseconds."""
        import torch
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(self.stream)
        for st in self.streams[:fly]:
            st.wait_event(e0)
        done, c = 0, 0
        while done < k:
            n = min(self.R, k - done)
            with torch.cuda.stream(self.streams[c % fly]):
                self.call(c % fly, done, n)
            done += n
            c += 1
        for st in self.streams[:fly]:
            self.stream.wait_stream(st)
        e1.record(self.stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def rows_per_step(self, steps):
        import numpy as np
        rows = float(np.mean([self.real_tokens[i % self.n_batches] for i in range(steps)]))
        sumsq = float(np.mean([self.sq_lengths[i % self.n_batches] for i in range(steps)]))
        return rows, sumsq

    def profile(self, steps):
        """Per-kernel-class durations (ms per request batch, event overhead taken off) with one call in flight."""
        import torch
        # the chip's clocks settle over the first tenths of a second of load: repeat the (untimed-for-the-headline) pass
        # until 0.2 s of device time have gone by and keep the last repetition
        spent, ms_serial = 0.0, 0.0
        for _ in range(50):
            t = self.run_steps(steps, 1)
            spent += t
            ms_serial = t / steps
            if spent >= 200.0:
                break
        self.model.profile_enable(True)
        done = 0
        while done < steps:
            n = min(self.R, steps - done)
            self.call(0, done, n)
            done += n
        torch.cuda.synchronize()
        prof = self.model.profile_read()
        self.model.profile_enable(False)
        # An event record costs the command processor a few microseconds, so the event-bracketed durations sum to
        # more than the same launches take back to back without events (ms_serial; kernels of one forward run
        # gap-free on one stream).  The excess, spread evenly over the launches, is taken off every duration.
        launches_total = sum(n for _, n in prof.values()) / steps
        raw_sum_ms = sum(ms_tot for ms_tot, _ in prof.values()) / steps
        event_overhead_ms = max(0.0, (raw_sum_ms - ms_serial) / launches_total)
        dur, kernels = {}, {}
        for k, (ms_tot, n) in prof.items():
            if n == 0:
                continue
            dur[k] = max(1e-6, ms_tot / steps - event_overhead_ms * n / steps)
            kernels[k] = {"launches_per_step": n / steps, "ms_per_step": dur[k], "avg_us": 1e3 * dur[k] / (n / steps),
                          "ms_per_step_raw_events": ms_tot / steps}
        return ms_serial, prof, dur, kernels, event_overhead_ms

    def close(self):
        for m in self.models[1:]:
            m.close()
        self.model.close()


def gemm_summary(spec, B, rows, prof, dur, kernels, steps, peak):
    """Adds TFLOP/s and the fraction of the matrix-core peak to the contraction classes; returns the totals over the
    tiled contractions (the dominant kernel)."""
    flops = gemm_flops_per_forward(spec, rows, B)
    for k in flops:
        if k in kernels:
            kernels[k]["tflops"] = flops[k] / (dur[k] * 1e-3) / 1e12
            kernels[k]["frac"] = kernels[k]["tflops"] / peak
    main = [k for k in flops if k != "gemm_first" and k in dur]
    main_flops = sum(flops[k] for k in main)
    gemm_ms = sum(dur[k] for k in main)
    gemm_ms_raw = sum(prof[k][0] for k in main) / steps
    gemm_launches = sum(prof[k][1] for k in main) / steps
    return flops, main_flops, gemm_ms, gemm_ms_raw, gemm_launches


def side_workload(mt, ms, name, R, fly, steps, warmup, latency_calls=0, precision=None):
    """A short run of another workload: sequences/s and the tiled contraction's TFLOP/s; for the small-batch serving
    workloads also the per-call latency sweep.  precision "fp8": the same shapes in the FP8 variant (E4M3 feed-forward
    contractions, whose two classes are then also given against the FP8 matrix-core peak)."""
    import dataclasses
    import torch
    spec = ms.get_config(name)
    if precision:
        spec = dataclasses.replace(spec, precision=precision)
    sv = Served(mt, ms, spec, spec.batch, R, fly)
    ms_serial, prof, dur, kernels, _ = sv.profile(steps)      # first, as in the headline run: it also settles the clocks
    sv.run_steps(warmup, sv.n_fly)
    ms_step = sv.run_steps(steps, sv.n_fly) / steps
    rows, _ = sv.rows_per_step(steps)
    _, main_flops, gemm_ms, _, gemm_launches = gemm_summary(spec, spec.batch, rows, prof, dur, kernels, steps, PEAK_BF16_MFMA_TFLOPS)
    ent = {"workload": f"{spec.name}: H={spec.hidden} trunk={spec.n_trunk_layers} tasks={spec.n_tasks} layers={sv.model.layer_count()} "
                       f"B={spec.batch} S={spec.seq}",
           "requests_per_call": sv.R, "calls_in_flight": sv.n_fly, "steps": steps,
           "sequences_per_s": spec.batch / (ms_step * 1e-3), "ms_per_step": ms_step, "ms_per_step_one_call_in_flight": ms_serial,
           "gemm_tflops": main_flops / (gemm_ms * 1e-3) / 1e12, "gemm_frac": main_flops / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
           "gemm_launches_per_step": gemm_launches}
    if spec.precision in ("fp8", "fp8_all"):
        ent["precision"] = ("bf16, feed-forward contractions in FP8 E4M3" if spec.precision == "fp8" else
                            "bf16, all four contractions of a layer in FP8 E4M3")
        for k in (("gemm_ffn1", "gemm_ffn2") if spec.precision == "fp8" else ("gemm_qkv", "gemm_out", "gemm_ffn1", "gemm_ffn2")):
            ent[k] = {"tflops": kernels[k]["tflops"], "frac_of_fp8_peak": kernels[k]["tflops"] / PEAK_FP8_MFMA_TFLOPS,
                      "avg_us": kernels[k]["avg_us"]}
    if latency_calls > 0:
        ent["latency"] = latency_sweep(mt, ms, spec, sv.model, latency_calls)
    sv.close()
    del sv
    torch.cuda.empty_cache()
    return ent


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="base", help="tiny | base | hetero | latency | large | industrial | wo_kd | mixed | assistant")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--requests-per-call", type=int, default=None,
                    help="request batches handed to the library per call (mt_forward_multi); 1 = plain mt_forward.  Default for "
                         "sequence-level workloads of up to 64 sequences per batch: the smallest of 8 .. 16 that divides --steps "
                         "(8 if none does); else 1")
    ap.add_argument("--in-flight", type=int, default=2,
                    help="calls in flight: calls are issued round-robin to this many model replicas (shared "
                         "weights, own workspace) on as many streams; 1 = strictly one call after another")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-workloads", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--cpu-sample", type=int, default=64, help="sequences the CPU oracle is timed on")
    ap.add_argument("--latency-calls", type=int, default=2000,
                    help="small-batch serving workloads: forwards timed one by one (host clock, stream sync per call) per "
                         "batch size; 0 skips that sweep")
    ap.add_argument("--qps", default="", help="comma-separated request rates (requests/s): also serve an open-loop Poisson "
                                              "stream of single-sequence requests at each rate and report p50/p99 latency")
    ap.add_argument("--qps-requests", type=int, default=20000, help="requests per rate of --qps")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="before the warm-up, run one plain 256 MiB device copy (a kernel of known traffic to scale "
                         "hardware byte counters by); untimed")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this benchmark measures one GPU only (sequences are independent, so N GPUs would run N "
              "replicas with no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import mt_synth as ms
    import paper_2107_05377_amd as mt
    from paper_2107_05377_amd import build as mtbuild

    if not os.path.exists(mt.LIB_PATH):
        mtbuild.build()
    mt.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    spec = ms.get_config(args.config)
    B = args.batch or spec.batch
    S = spec.seq
    has_tokens = any(getattr(t, "token_level", False) for t in spec.tasks)
    # default: calls of 8 request batches; when the timed steps do not fill calls of 8 but do fill calls of 9 .. 16, take that
    # size, so that every timed call is a full one
    full = [r for r in range(8, 17) if args.steps % r == 0]
    R = args.requests_per_call if args.requests_per_call else ((full[0] if full else 8) if (B <= 64 and not has_tokens) else 1)
    if has_tokens:
        R = 1
    sv = Served(mt, ms, spec, B, R, args.in_flight)
    model, n_fly = sv.model, sv.n_fly

    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")       # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Order of the measurements: first the same steps with one call in flight (what the per-kernel figures are measured
    # on, so that no other call's kernels share the chip with a timed launch) and with HIP events around every launch;
    # then the headline: W untimed warm-up steps and exactly K timed steps with `n_fly` calls in flight.
    sv.run_steps(min(args.warmup, 3 * sv.R), 1)
    ms_serial, prof, dur, kernels, event_overhead_ms = sv.profile(args.steps)
    sv.run_steps(args.warmup, n_fly)
    ms_per_step = sv.run_steps(args.steps, n_fly) / args.steps
    seq_per_s = B / (ms_per_step * 1e-3)
    for o in sv.outs[0][:min(sv.R, args.steps)]:
        assert torch.isfinite(o).all()
    # ... and call by call with an event pair around every call: median and minimum per request batch
    n_calls = (args.steps + sv.R - 1) // sv.R
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_calls + 1)]
    torch.cuda.synchronize()
    marks[0].record(sv.stream)
    done, sizes = 0, []
    for i in range(n_calls):
        n = min(sv.R, args.steps - done)
        sv.call(0, done, n)
        marks[i + 1].record(sv.stream)
        done += n
        sizes.append(n)
    torch.cuda.synchronize()
    per_step = np.array([marks[i].elapsed_time(marks[i + 1]) / sizes[i] for i in range(n_calls)])

    n_layers = model.layer_count()
    rows, sumsq = sv.rows_per_step(args.steps)
    n_full, n_first = layer_kinds(spec)
    assert n_full + n_first == n_layers
    bf16 = spec.precision == "bf16"
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_FP32_VALU_TFLOPS
    flops, main_flops, gemm_ms, gemm_ms_raw, gemm_launches = gemm_summary(spec, B, rows, prof, dur, kernels, args.steps, peak)
    gemm_tflops = main_flops / (gemm_ms * 1e-3) / 1e12
    kname = ("gemm_bf16_kernel + gemm_bf16_persist_kernel" if rows * sv.R > 256 else "gemm_skinny_bf16_kernel") if bf16 else "gemm_f32_kernel"
    traffic = stored_traffic(spec.name, sv.R) if (bf16 and B == spec.batch and rows * sv.R > 256) else None
    measured_peak = mt.mfma_peak() if bf16 else None
    # per LAUNCH: a launch serves the rows of all request batches of its call
    roofline = {"kernel": kname, "bound": "mfma" if bf16 else "alu",
                "achieved": gemm_tflops, "peak": peak, "unit": "TFLOP/s", "frac": gemm_tflops / peak, "traffic": traffic,
                "traffic_source": "stored rocprofv3 counter summary under profiles/ (null: none for this kernel source)",
                "peak_measured_mfma_only": measured_peak,
                "frac_of_measured_peak": (gemm_tflops / measured_peak) if measured_peak else None,
                "flops_per_launch": main_flops / gemm_launches, "avg_launch_us": 1e3 * gemm_ms / gemm_launches,
                "flops_counted": "executed: real (unpadded) token rows only",
                "launches_per_step": gemm_launches, "gemm_ms_per_step": gemm_ms,
                "rows_per_launch": rows * min(sv.R, args.steps),
                "avg_launch_us_raw_events": 1e3 * gemm_ms_raw / gemm_launches, "event_overhead_us_per_launch": 1e3 * event_overhead_ms}

    h = spec.hidden
    per_layer = 8.0 * S * h * h + 4.0 * S * h * spec.ffn + 4.0 * S * S * h
    flops_per_seq_dense = n_layers * per_layer + spec.n_tasks * 2.0 * h * h          # dense, padded convention
    first_attn = 2.0 * h * rows * spec.heads if (bf16 and spec.heads <= 16) else 4.0 * h * rows   # weighted row sums per head
    executed_per_step = (sum(flops.values()) + n_full * 4.0 * h * sumsq + n_first * first_attn
                         + spec.n_tasks * 2.0 * B * 2 * h * h)
    e2e_tflops = executed_per_step / (ms_per_step * 1e-3) / 1e12
    e2e_tflops_dense = flops_per_seq_dense * seq_per_s / 1e12

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        trunk, _ = ms.make_trunk_params(spec)
        tasks = [ms.make_task_params(spec, t)[0] for t in range(spec.n_tasks)]
        orc = oracle.Oracle(spec, trunk, tasks)
        left, dt, n_done, err = max(1, args.cpu_sample), 0.0, 0, 0.0
        for bi in range(sv.n_batches):
            if left <= 0:
                break
            n = min(left, B)
            ids, mask, _ = ms.make_inputs(spec, batch=B, batch_index=bi)
            t0 = time.time()
            ref = orc.mt_forward(ids[:n], mask[:n])
            dt += time.time() - t0
            sv.call(0, bi, 1)
            got = sv.outs[0][0].cpu().numpy()[:n]
            err = max(err, float(np.abs(got - ref).max()))
            left -= n
            n_done += n
        cpu = {"value": n_done / dt, "unit": "sequences/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"the first {n_done} sequences of the same workload's batches, one pass, {dt:.1f} s",
               "max_abs_dlogit_vs_gpu": err, "host": host_description()}
        # the same oracle on one thread, on a smaller sample
        n1 = max(1, min(4, n_done))
        all_threads = oracle.num_threads()
        oracle.set_num_threads(1)
        ids, mask, _ = ms.make_inputs(spec, batch=B, batch_index=0)
        t0 = time.time()
        orc.mt_forward(ids[:n1], mask[:n1])
        dt1 = time.time() - t0
        oracle.set_num_threads(all_threads)
        cpu["one_thread"] = {"value": n1 / dt1, "unit": "sequences/s", "sample": f"first {n1} sequences of batch 0, {dt1:.1f} s"}

    line = {
        "metric": "sequences/sec (8-task MT forward, BERT-base, seq128) + % bf16 MFMA peak",
        "value": seq_per_s, "unit": "sequences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{spec.name}: H={spec.hidden} A={spec.heads} F={spec.ffn} trunk={spec.n_trunk_layers} "
                               f"tasks={spec.n_tasks} layers={n_layers} B={B} S={S} len~U[{spec.len_lo},{spec.len_hi}]",
                   "batch": B, "seq_len": S, "layer_evals": n_layers, "layers_on_all_rows": n_full,
                   "layers_on_first_token_only": n_first, "real_tokens_per_batch": rows, "padding_skipped": True,
                   "step": "one request batch of `batch` sequences", "requests_per_call": sv.R, "calls_in_flight": n_fly},
        "ms_per_step_one_call_in_flight": ms_serial, "sequences_per_s_one_call_in_flight": B / (ms_serial * 1e-3),
        "ms_per_step_one_call_in_flight_median": float(np.median(per_step)), "ms_per_step_one_call_in_flight_min": float(per_step.min()),
        "e2e_tflops_executed": e2e_tflops, "e2e_frac_of_peak": e2e_tflops / peak,
        "e2e_tflops_dense_padded_equivalent": e2e_tflops_dense,
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "weights_load_s": sv.load_s,
    }
    if spec.name in ("latency", "industrial") and args.latency_calls > 0:
        line["latency"] = latency_sweep(mt, ms, spec, model, args.latency_calls)
    if args.qps:
        line["qps_stream"] = qps_stream(ms, spec, model, [float(r) for r in args.qps.split(",")], args.qps_requests)
    if spec.name == "base" and not args.no_workloads:
        # the other workloads, driver-timed: short runs (a few seconds each), same measurement as above
        sv.close()
        del sv, model
        torch.cuda.empty_cache()
        side = {}
        side["base_one_request_per_call"] = side_workload(mt, ms, "base", 1, 3, 192, 24)
        side["base_fp8_ffn"] = side_workload(mt, ms, "base", 8, 2, 48, 8, precision="fp8")
        side["base_fp8_layer"] = side_workload(mt, ms, "base", 8, 2, 48, 8, precision="fp8_all")
        side["hetero"] = side_workload(mt, ms, "hetero", 4, 2, 32, 4)
        side["large"] = side_workload(mt, ms, "large", 1, 2, 16, 2)
        side["industrial"] = side_workload(mt, ms, "industrial", 32, 2, 256, 64)   # short utterances: 32 requests fill a call
        side["latency"] = side_workload(mt, ms, "latency", 1, 1, 64, 8, latency_calls=args.latency_calls)
        line["workloads"] = side
    print(json.dumps(line))


if __name__ == "__main__":
    main()
