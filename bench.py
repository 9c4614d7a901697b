#!/usr/bin/env python3
"""Benchmark of the RanDeS hot path on one MI355X.

One *step* is one pass of the whole hot path over one synthetic batch: merge
(compress) the K task deltas once, then serve a stream of retrieve requests that
cycle over the task ids.  The headline workload is the Llama-7B-shaped bf16 stack
(32 blocks, d = 4096, ffn 11008, K = 8, 64 requests).  Inputs are generated on
the device and are resident in HBM before the timed region starts.

Prints ONE JSON line: whole-step throughput in GB/s of algorithmic bytes
(merge: K*b_in + b_merged per element; retrieve: b_merged + b_base + b_out per
element), the HBM roofline of the dominant kernel (retrieve) and of the merge
kernel, and the CPU oracle timed on a bounded sample of the same workload.
After the timed region of the headline workload the same line gathers, under
`config`: the headline workload once more with ordinary allocations
(`plain_placement`), the other model-shaped workloads (`other_workloads`: ViT-B/32,
ViT-L/14 with K = 20, T5-base, and T5-base's LoRA variant), the other entry
points, and what a cached call costs on the host.
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2505_11204_amd import binding as rb          # noqa: E402
from paper_2505_11204_amd import placement              # noqa: E402
from paper_2505_11204_amd import workloads as wl        # noqa: E402

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth

WORKLOADS = {
    # name: (stack fn, storage dtype, K, requests, delta std, per-task scales?)
    "llama_7b": (wl.llama_7b, "bf16", 8, 64, 5e-4, False),
    "vit_l14": (wl.vit_l14, "f32", 20, 20, 1e-3, True),
    "vit_b32": (wl.vit_b32, "f32", 8, 8, 1e-3, False),
    "t5_base": (wl.t5_base, "bf16", 8, 8, 1e-3, False),
    "tiny": (wl.tiny, "f32", 4, 4, 1e-3, False),
}
HEADLINE = "llama_7b"
OTHERS = ("vit_b32", "vit_l14", "t5_base")

# What the paper itself times (Sec. "Performance Analysis", repeated in "Scalability Analysis"):
# regenerating one model's transforms and retrieving it, on a CPU.  Another machine and an
# implementation that is not published: context beside the retrieve figures, not a target.
PAPER_RETRIEVE_MS = {
    "vit_b32": {"ms": 292.70, "hardware": "Intel Xeon Gold 6448Y (CPU)", "workload": "CLIP-ViT-B/32, 8 models"},
    "vit_l14": {"ms": 658.19, "hardware": "Intel Xeon Gold 6448Y (CPU)", "workload": "CLIP-ViT-L/14"},
}

# rocprofv3 summaries that hold the HBM byte counters of a workload's kernels, and the sources
# whose hash the summary records: counters taken on other kernels are not reported as traffic.
PROFILES = {
    "llama_7b": "profiles/llama_7b_bf16_k8_merge_retrieve.txt",
    "vit_l14": "profiles/vit_l14_f32_k20_merge_retrieve.txt",
    "vit_b32": "profiles/vit_b32_f32_k8_merge_retrieve.txt",
    "t5_base": "profiles/t5_base_bf16_k8_merge_retrieve.txt",
}
KERNEL_SOURCES = ("paper_2505_11204_amd/csrc/kernels.hip", "paper_2505_11204_amd/csrc/device_util.hpp",
                  "paper_2505_11204_amd/csrc/philox.hpp", "paper_2505_11204_amd/csrc/plan.cpp",
                  "paper_2505_11204_amd/csrc/plan.hpp")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(WORKLOADS))
    ap.add_argument("--requests", type=int, default=0, help="retrieve requests per step (0 = workload default)")
    ap.add_argument("--merge-rows", type=int, default=0, help="rows per merge tile (0 = library default)")
    ap.add_argument("--retrieve-rows", type=int, default=0, help="rows per retrieve tile (0 = library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 4 GiB device copy (torch.mul(src, 1.0, out=dst)) three times, so that HBM byte "
                         "counters collected over this command can be scaled by a kernel of known traffic")
    ap.add_argument("--cpu-sample-elems", type=int, default=1_600_000_000,
                    help="size of the oracle's sample (elements per model)")
    ap.add_argument("--placement", choices=("groups", "plain"), default="groups",
                    help="groups: find the memory's address groups by timing copies and place read and "
                         "write streams in different ones (stacks of 256 MiB and more); plain: one "
                         "allocation per stack, wherever the allocator puts it")
    ap.add_argument("--tasks", type=int, default=0, help="number of merged models (0 = the workload's own)")
    ap.add_argument("--no-fold", action="store_true",
                    help="hand every layer to the kernels row by row (see randes_set_fold)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the plain-streaming probe")
    ap.add_argument("--no-extras", action="store_true", help="skip the other entry points of the library")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the other workloads and the second run of the headline workload with plain allocations")
    return ap.parse_args()


def cpu_model():
    """Model name of the host CPU with its family and model numbers (a virtual machine may shorten the name)."""
    want = {"model name": None, "cpu family": None, "model": None}
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                key = line.split(":", 1)[0].strip().lower()
                if key in want and want[key] is None:
                    want[key] = line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "%s (family %s, model %s)" % (want["model name"] or "unknown", want["cpu family"] or "?", want["model"] or "?")


def sources_sha256(paths=KERNEL_SOURCES):
    h = hashlib.sha256()
    for p in paths:
        with open(os.path.join(ROOT, p), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def profile_traffic(workload):
    """HBM bytes per launch of the workload's kernels as the tracked rocprofv3 summary records them
    (lines `@ traffic_bytes <kernel> = <bytes>`), or a reason why there is none to report: no
    summary, or one taken on kernel sources with another hash (`@ sources_sha256 = ...`)."""
    path = PROFILES.get(workload)
    if path is None or not os.path.exists(os.path.join(ROOT, path)):
        return {}, "no tracked counter summary for this workload"
    sha, traffic = None, {}
    with open(os.path.join(ROOT, path)) as f:
        for line in f:
            m = re.match(r"@ sources_sha256 = ([0-9a-f]{64})", line)
            if m:
                sha = m.group(1)
            m = re.match(r"@ traffic_bytes (\w+) = ([0-9.eE+]+)", line)
            if m:
                traffic[m.group(1)] = float(m.group(2))
    if sha != sources_sha256():
        return {}, "%s holds counters of other kernel sources (sha256 %s..., now %s...): take them again" % (
            path, (sha or "none")[:12], sources_sha256()[:12])
    return traffic, None


class Placement:
    """Where the stacks of a run live: in one large allocation cut into the memory's address groups
    (found by timing copies), or in ordinary allocations.  One instance serves every workload of a run."""

    def __init__(self, mode, headline_bytes, headline_tasks):
        self.arena = self.labels = None
        self.fallback = False
        self.info = {"policy": "plain"}
        if mode != "groups":
            return
        free_bytes, _ = torch.cuda.mem_get_info()
        try:
            # everything but a reserve for temporaries goes into one allocation, cut by measurement
            self.arena = placement.Arena(free_bytes - (12 << 30))
            t_cls = time.perf_counter()
            ok = False
            for attempt in range(3):        # the copy rates differ by a few per cent only: measure again if need be
                self.labels = self.arena.classify()
                if placement.plan_serving_layout(self.labels, self.arena.chunk_bytes, headline_bytes,
                                                 headline_tasks) is not None:
                    ok = True
                    break
            self.info = {"classify_s": time.perf_counter() - t_cls, "classify_attempts": attempt + 1,
                         "runs_gib": [(g, a, b) for g, a, b in placement.runs_of(self.labels)]}
            if not ok:
                self.info["policy"] = "plain (no usable address groups found)"
                self.fallback = True
                self.close()
        except (RuntimeError, ValueError) as e:      # the large allocation itself failed
            self.info = {"policy": "plain (arena not available: %s)" % str(e).splitlines()[0][:120]}
            self.fallback = True
            self.close()

    def close(self):
        self.arena = self.labels = None
        torch.cuda.empty_cache()

    def layout(self, stack_bytes, n_tasks, more_outputs=0):
        """(byte offsets of the stacks inside the arena, description), or (None, description) for
        ordinary allocations."""
        if self.arena is None or stack_bytes < (256 << 20):
            return None, dict(self.info, policy=self.info.get("policy", "plain") if self.arena is None
                              else "plain (stack under 256 MiB)")
        lay = None
        for more in (more_outputs, 0):
            lay = placement.plan_serving_layout(self.labels, self.arena.chunk_bytes, stack_bytes, n_tasks, more)
            if lay is not None:
                break
        gib = lambda off: round(off / (1 << 30), 2)      # noqa: E731
        if lay is None:
            # groups were found but do not hold this workload's layout: stacks one after the other
            step = (stack_bytes + 255) // 256 * 256
            if step * (n_tasks + 3) > self.arena.buf.numel():
                raise RuntimeError("workload does not fit the device")
            lay = {"base": 0, "merged": step, "out": 2 * step, "deltas": [(3 + i) * step for i in range(n_tasks)],
                   "more_outputs": []}
            return lay, dict(self.info, policy="stacks one after the other inside the large allocation "
                                               "(its groups do not hold this layout)")
        desc = dict(self.info)
        desc.update({
            "policy": "merged and base in one address group, out across the boundary of two others, "
                      "deltas in what is left of every group but the first",
            "read_group": lay["read_group"], "write_groups": lay["write_groups"],
            "offsets_gib": {"merged": gib(lay["merged"]), "base": gib(lay["base"]), "out": gib(lay["out"]),
                            "deltas": [gib(d) for d in lay["deltas"]],
                            "more_outputs": [gib(d) for d in lay["more_outputs"]]}})
        return lay, desc


class Setup:
    """One workload resident in HBM: base, K deltas, the merged stack, one output stack and the
    library's tables for them."""

    def __init__(self, name, pl, n_tasks=0, n_req=0, more_outputs=0):
        stack_fn, self.dtype, K, req, delta_std, scaled = WORKLOADS[name]
        self.name = name
        self.K = n_tasks or K
        self.n_req = n_req or req
        self.stack = stack_fn()
        self.layers = [(l.rows, l.cols, l.group, l.flags) for l in self.stack]
        self.n_elem = wl.n_elements(self.stack)
        self.eb = 4 if self.dtype == "f32" else 2
        self.seeds = [42 + i for i in range(self.K)]
        self.td = wl.torch_dtype(self.dtype)
        self.stack_elems = wl.stack_elements(self.stack, self.td)
        lay, self.placed = pl.layout(self.stack_elems * self.eb, self.K, more_outputs)
        place = merged_into = out_into = None
        self.more_out_into = []
        if lay is not None:
            flat = lambda off: pl.arena.flat(off, self.stack_elems, self.td)     # noqa: E731
            place = lambda who: flat(lay["base"] if who == "base" else lay["deltas"][who])   # noqa: E731
            merged_into, out_into = flat(lay["merged"]), flat(lay["out"])
            self.more_out_into = [flat(off) for off in lay["more_outputs"]]
        self.flats = []
        scales = wl.task_scales(self.K, 1234) if scaled else None
        self.base, self.deltas = wl.make_inputs(self.stack, self.K, dtype=self.dtype, device="cuda", data_seed=1234,
                                                delta_std=delta_std, scales=scales, flats=self.flats, place=place)
        self.merged_flat, self.merged = wl.alloc_stack(self.stack, self.td, "cuda", into=merged_into)
        self.out_flat, self.out = wl.alloc_stack(self.stack, self.td, "cuda", into=out_into)
        self.lt = rb.LayerTable(self.layers)
        self.t_deltas = rb.PtrTable([t for per in self.deltas for t in per], self.lt)
        self.t_merged = rb.PtrTable(self.merged, self.lt)
        self.t_base = rb.PtrTable(self.base, self.lt)
        self.t_out = rb.PtrTable(self.out, self.lt)
        self.bytes_merge = self.n_elem * (self.K * self.eb + self.eb)
        self.bytes_retr = self.n_elem * 3 * self.eb
        self.bytes_step = self.bytes_merge + self.n_req * self.bytes_retr
        torch.cuda.synchronize()

    def describe(self):
        return "%s-shaped stack: %d matrices, %d elements, %s storage with f32 arithmetic, K=%d, one merge + %d " \
               "retrieve requests per step" % (self.name, len(self.stack), self.n_elem, self.dtype, self.K, self.n_req)

    def step(self, events=None):
        """One pass of the hot path.  With `events`, every launch is bracketed by HIP events recorded on
        the stream the library launches on (torch's current stream)."""
        if events is not None:
            e0 = torch.cuda.Event(enable_timing=True); e0.record()
        rb.merge(self.lt, self.t_deltas, self.seeds, merged=self.t_merged)
        if events is not None:
            e1 = torch.cuda.Event(enable_timing=True); e1.record()
            events["merge"].append((e0, e1))
        for q in range(self.n_req):
            if events is not None:
                a = torch.cuda.Event(enable_timing=True); a.record()
            rb.retrieve(self.lt, self.t_merged, self.t_base, self.seeds[q % self.K], 1.0, out=self.t_out)
            if events is not None:
                b = torch.cuda.Event(enable_timing=True); b.record()
                events["retrieve"].append((a, b))

    def step_in_a_graph(self, reps=10):
        """The same step recorded once into a HIP graph and replayed (cached calls are kernel launches only):
        what a serving loop pays per step when it replays its launches, which matters for the stacks whose
        kernels last a fraction of a millisecond."""
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            self.step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            graph.capture_begin()
            try:
                self.step()
            finally:
                graph.capture_end()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / reps
        gbs = self.bytes_step / (ms * 1e-3) / 1e9
        return {"ms_per_step": ms, "GBs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS, "replays": reps}

    def first_calls(self):
        """The first call with a given (layers, pointers, seed) builds the tile tables on the host and
        uploads them; later calls find them cached.  Timed once, outside the timed region."""
        first = {}
        tf = time.perf_counter()
        rb.merge(self.lt, self.t_deltas, self.seeds, merged=self.t_merged)
        torch.cuda.synchronize()
        first["merge_ms"] = (time.perf_counter() - tf) * 1e3
        tf = time.perf_counter()
        rb.retrieve(self.lt, self.t_merged, self.t_base, self.seeds[0], 1.0, out=self.t_out)
        torch.cuda.synchronize()
        first["retrieve_ms"] = (time.perf_counter() - tf) * 1e3
        return first

    def measure(self, steps, warmup):
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        events = {"merge": [], "retrieve": []}
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(events)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / max(steps, 1)
        merge_ms = sorted(a.elapsed_time(b) for a, b in events["merge"])
        retr_ms = sorted(a.elapsed_time(b) for a, b in events["retrieve"])
        avg = lambda xs: sum(xs) / len(xs)          # noqa: E731
        pct = lambda xs, p: xs[min(len(xs) - 1, int(p * len(xs)))]   # noqa: E731
        retr_avg, merge_avg = avg(retr_ms), avg(merge_ms)
        retr_gbs = self.bytes_retr / (retr_avg * 1e-3) / 1e9
        merge_gbs = self.bytes_merge / (merge_avg * 1e-3) / 1e9
        step_gbs = self.bytes_step / (ms_per_step * 1e-3) / 1e9
        return {
            "ms_per_step": ms_per_step, "GBs": step_gbs, "frac_of_hbm_peak": step_gbs / HBM_PEAK_GBS,
            "algorithmic_bytes_per_step": self.bytes_step,
            "merge": {"GBs": merge_gbs, "frac_of_hbm_peak": merge_gbs / HBM_PEAK_GBS, "ms_avg": merge_avg,
                      "ms_min": merge_ms[0], "bytes": self.bytes_merge},
            "retrieve": {"GBs": retr_gbs, "frac_of_hbm_peak": retr_gbs / HBM_PEAK_GBS, "ms_avg": retr_avg,
                         "ms_median": pct(retr_ms, 0.5), "ms_p95": pct(retr_ms, 0.95), "ms_min": retr_ms[0],
                         "bytes": self.bytes_retr},
        }

    def host_time_per_cached_call(self):
        """Microseconds the calling thread spends inside one call whose tables are cached (argument
        marshalling of the Python binding, key hashing, lookup, overlap checks, kernel launches); the
        GPU work it enqueues runs behind it."""
        out = {}
        torch.cuda.synchronize()
        for what, n, fn in (
                ("retrieve", 32, lambda q: rb.retrieve(self.lt, self.t_merged, self.t_base, self.seeds[q % self.K], 1.0,
                                                        out=self.t_out)),
                ("merge", 6, lambda q: rb.merge(self.lt, self.t_deltas, self.seeds, merged=self.t_merged))):
            ts = []
            for q in range(n):
                t = time.perf_counter()
                fn(q)
                ts.append(time.perf_counter() - t)
            torch.cuda.synchronize()
            ts.sort()
            out[what + "_us_median"] = ts[len(ts) // 2] * 1e6
            out[what + "_us_max"] = ts[-1] * 1e6
        return out


def cpu_baseline(S, target_elems):
    """The oracle, as it stands, on a bounded sample of the same workload: the leading
    grouped layers of the stack (whole matrices, about `target_elems` elements), copied
    from the device, merged once and retrieved for a few tasks with all host threads."""
    import oracle
    stack, deltas, base, seeds, dtype, n_requests = S.stack, S.deltas, S.base, S.seeds, S.dtype, S.n_req
    code = {"f32": 0, "bf16": 1}[dtype]
    pick, n_elem = [], 0
    for idx, l in enumerate(stack):
        if l.group < 0:
            continue
        pick.append(idx)
        n_elem += l.rows * l.cols
        if n_elem >= target_elems:
            break
    sub = [(stack[i].rows, stack[i].cols, stack[i].group, stack[i].flags) for i in pick]
    K = len(seeds)
    host_d = [[wl.to_numpy(deltas[i][p]) for p in pick] for i in range(K)]
    host_b = [wl.to_numpy(base[p]) for p in pick]
    threads = oracle.max_threads()
    t0 = time.perf_counter()
    merged = oracle.merge(sub, host_d, seeds, code, code, n_threads=threads)
    t1 = time.perf_counter()
    n_retr = min(4, n_requests)
    for q in range(n_retr):
        oracle.retrieve(sub, merged, host_b, seeds[q % K], 1.0, code, code, code, n_threads=threads)
    t2 = time.perf_counter()
    eb = 4 if dtype == "f32" else 2
    # one thread, on the first matrix of the sample only
    one = [sub[0][:2] + (-1, sub[0][3] & 1)]
    n_one = sub[0][0] * sub[0][1]
    t3 = time.perf_counter()
    m1 = oracle.merge(one, [[d[0]] for d in host_d], seeds, code, code, n_threads=1)
    t4 = time.perf_counter()
    oracle.retrieve(one, m1, host_b[:1], seeds[0], 1.0, code, code, code, n_threads=1)
    t5 = time.perf_counter()
    bytes_merge = n_elem * (K * eb + eb)
    bytes_retr = n_elem * 3 * eb
    t_merge, t_retr = t1 - t0, (t2 - t1) / n_retr
    t_step = t_merge + n_requests * t_retr
    return {
        "value": (bytes_merge + n_requests * bytes_retr) / t_step / 1e9,
        "unit": "GB/s",
        "cores": threads,
        "cpu_model": cpu_model(),
        "kind": "oracle",
        "sample": "the first %d grouped matrices of the stack (%d elements, K=%d): one merge %.2f s + %d retrieves "
                  "%.2f s each; value combines them as 1 merge + %d retrieves" % (
                      len(sub), n_elem, K, t_merge, n_retr, t_retr, n_requests),
        "merge_GBs": bytes_merge / t_merge / 1e9,
        "retrieve_GBs": bytes_retr / t_retr / 1e9,
        "one_thread": {"merge_GBs": n_one * (K * eb + eb) / (t4 - t3) / 1e9,
                       "retrieve_GBs": n_one * 3 * eb / (t5 - t4) / 1e9,
                       "sample": "the first matrix of the sample (%d elements)" % n_one},
    }


def ceilings(flats, merged_flat, out_flat):
    """What a plain streaming kernel with nothing of the method in it reaches on this machine, on this
    workload's own buffers (not part of the timed region).  A point of comparison, not an upper
    bound: its launch shape is one of many."""
    nb = min(f.numel() * f.element_size() for f in flats + [merged_flat, out_flat]) // 16384 * 16384
    def cut(t):
        return t.view(torch.uint8)[:nb]
    base, deltas = cut(flats[0]), [cut(f) for f in flats[1:]]
    m, o = cut(merged_flat), cut(out_flat)
    K = min(8, len(deltas))

    def run(inputs, output, write):
        ts = []
        for _ in range(4):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            rb.probe_stream(inputs, output, write)
            b.record()
            b.synchronize()
            ts.append(a.elapsed_time(b))
        ts = sorted(ts[1:])
        n_streams = len(inputs) + (1 if write else 0)
        return n_streams * nb / (ts[len(ts) // 2] * 1e-3) / 1e9
    # the probe overwrites merged and out; both are rewritten by every timed step
    return {
        "unit": "GB/s",
        "bytes_per_stream": nb,
        "read_%d_streams" % K: run(deltas[:K], o, False),
        "add_%d_reads_1_write" % K: run(deltas[:K], m, True),
        "add_2_reads_1_write": run([m, base], o, True),
        "copy_1_read_1_write": run([base], o, True),
    }


def timed_calls(fn, reps=10, burst=20):
    """(median ms of one call bracketed by its own pair of HIP events, which includes the latency of
    a launch into an idle queue; ms per call of `burst` calls issued back to back between one pair,
    which is what the kernels themselves take; microseconds the host spends issuing one such call)."""
    fn(); fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); fn(); b.record(); b.synchronize()
        ts.append(a.elapsed_time(b))
    bs, hs = [], []
    for _ in range(3):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        t0 = time.perf_counter()
        for _ in range(burst):
            fn()
        hs.append((time.perf_counter() - t0) / burst * 1e6)
        b.record(); b.synchronize()
        bs.append(a.elapsed_time(b) / burst)
    return sorted(ts)[len(ts) // 2], sorted(bs)[1], sorted(hs)[1]


def across_a_boundary(pl, nbytes):
    """Byte offset inside the placed allocation at which nbytes lie half in one address group and half in
    the next (a write-only stream is fastest there), or None."""
    if pl is None or pl.arena is None or pl.labels is None:
        return None
    cb = pl.arena.chunk_bytes
    need = -(-(nbytes // 2) // cb)
    runs = placement.runs_of(pl.labels)
    for (_, a0, b0), (_, a1, b1) in zip(runs[:-1], runs[1:]):
        if b0 - a0 >= need and b1 - a1 >= need:
            return (b0 * cb - nbytes // 2) // 256 * 256
    return None


def lora_variant(pl=None):
    """The LoRA variant of the T5-base workload (PEFT section): K = 8 models, each a rank-16 adapter on
    72 of the stack's 768 x 768 matrices.  The front end either materialises the 576 dense deltas
    B.A, which the streaming merge then superposes, or superposes straight from the factors and writes the
    72 merged matrices once; retrieval is the ordinary one on the 72-matrix stack.  All write-bound
    or launch-bound at this size (85 MB per stack), so rates are GB/s of HBM.  With a placed allocation at
    hand (no other workload uses it at this point) the 680 MB of materialised deltas are also written
    across a boundary of two address groups, next to the run with ordinary allocations."""
    stack_full = wl.t5_base()
    stack = [stack_full[t] for t in wl.t5_lora_targets(stack_full)]
    layers = [(l.rows, l.cols, l.group, l.flags) for l in stack]
    K, rank = 8, 16
    factors = wl.make_lora_factors(stack, list(range(len(stack))), K, rank=rank, dtype="bf16", device="cuda")
    Bs = [f[0] for per in factors for f in per]
    As = [f[1] for per in factors for f in per]
    batch = rb.LoraBatch(Bs, As)
    placed_batch = None
    per = [l.rows * l.cols for l in stack] * K
    off = across_a_boundary(pl, 2 * sum(per))
    if off is not None:
        flat = pl.arena.flat(off, sum(per), torch.bfloat16)
        starts = [sum(per[:q]) for q in range(len(per))]
        placed_batch = rb.LoraBatch(Bs, As, [flat[s:s + n].view(Bs[q].shape[0], As[q].shape[1])
                                             for q, (s, n) in enumerate(zip(starts, per))])
    seeds = [42 + i for i in range(K)]
    fused = rb.LoraMerge(layers, factors, seeds, merged_dtype=torch.bfloat16)
    lt = rb.LayerTable(layers)
    t_dense = rb.PtrTable(batch.outs, lt)
    merged = fused.merged
    t_merged = rb.PtrTable(merged, lt)
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    base = [torch.empty(l.rows, l.cols, dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=g)
            .to(torch.bfloat16) for l in stack]
    out = [torch.empty_like(b) for b in base]
    t_base, t_out = rb.PtrTable(base, lt), rb.PtrTable(out, lt)

    n_out = sum(l.rows * l.cols for l in stack)
    in_bytes = K * sum((l.rows + l.cols) * rank * 2 for l in stack)
    flop = 2.0 * K * n_out * rank
    rows = {}

    def row(name, nbytes, fn, with_flop=False):
        ms_call, ms_burst, host_us = timed_calls(fn)
        rows[name] = {"ms_per_call_alone": ms_call, "ms_back_to_back": ms_burst, "host_us_per_call": host_us, "bytes": nbytes,
                      "GBs": nbytes / (ms_burst * 1e-3) / 1e9,
                      "frac_of_hbm_peak": nbytes / (ms_burst * 1e-3) / 1e9 / HBM_PEAK_GBS}
        if with_flop:
            rows[name]["TFLOPs"] = flop / (ms_burst * 1e-3) / 1e12
    row("materialize (576 deltas written)", K * n_out * 2 + in_bytes, lambda: batch.run(1.0), True)
    if placed_batch is not None:
        row("materialize_across_groups (the same, outputs half and half across a boundary of two address groups)",
            K * n_out * 2 + in_bytes, lambda: placed_batch.run(1.0), True)
    row("merge of the materialised deltas", n_out * 2 * (K + 1), lambda: rb.merge(lt, t_dense, seeds, merged=t_merged))
    row("fused_merge (factors in, 72 merged matrices written)", n_out * 2 + in_bytes, lambda: fused.run(1.0), True)
    q = [0]

    def one_retrieve():
        q[0] += 1
        rb.retrieve(lt, t_merged, t_base, seeds[q[0] % K], 1.0, out=t_out)
    row("retrieve", n_out * 6, one_retrieve)
    return {"shapes": "72 x (768 x 768), rank 16, K = 8, bf16; GB/s and TFLOP/s from the back-to-back time", **rows}


def widened_rows(S):
    """The other streaming entry points on the same stacks, after the timed region (they overwrite
    the merged stack): hot add of one model, the diagnostics reduction, merge from weights."""
    lt, K, eb, seeds = S.lt, S.K, S.eb, S.seeds
    per_model = [rb.PtrTable(S.deltas[i], lt) for i in range(min(K, 2))]

    def timed(fn, reps=4):
        fn()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record(); b.synchronize()
            ts.append(a.elapsed_time(b))
        return sorted(ts)[len(ts) // 2]
    stats_out = torch.empty(3, dtype=torch.float64, device="cuda")
    rows = {
        "hot_add (reads delta + merged, writes merged)":
            (3 * eb, timed(lambda: rb.update(lt, S.t_merged, per_model[0], seeds[0]))),
        "delta_stats (reads two deltas)":
            (2 * eb, timed(lambda: rb.delta_stats(lt, per_model[0], seeds[0], per_model[1 % K],
                                                  seeds[1 % K], out=stats_out))),
        # timing only: the delta stacks stand in for fine-tuned weights.  Task i's term of slot l is
        # weights_i[src_i(l)] - base[src_i(l)]: the base layer differs per task, so 2K read streams.
        "merge_from_weights (reads K weights + K base layers, writes merged)":
            ((2 * K + 1) * eb, timed(lambda: rb.merge_weights(lt, S.t_deltas, S.t_base, seeds, merged=S.t_merged))),
    }
    return {name: {"ms": ms, "GBs": S.n_elem * bpe / (ms * 1e-3) / 1e9} for name, (bpe, ms) in rows.items()}


MANY_Q = 4     # models retrieved per pass in the several-models measurement


def many_extras(S, single_ms):
    """MANY_Q models retrieved in one pass (the merged stack is read once for all of them), after the
    timed region.  Reported per request, as algorithmic bytes of MANY_Q single retrievals and as the
    bytes the pass really moves.  None when the further output stacks do not fit."""
    outs = [S.out]
    try:
        for i in range(MANY_Q - 1):
            into = S.more_out_into[i] if i < len(S.more_out_into) else None
            if into is None and torch.cuda.mem_get_info()[0] < S.stack_elems * S.eb + (4 << 30):
                return None
            outs.append(wl.alloc_stack(S.stack, S.td, "cuda", into=into)[1])
    except RuntimeError:
        return None
    q = len(outs)
    t_outs = rb.PtrTable([t for per in outs for t in per], S.lt)
    req = [S.seeds[i % len(S.seeds)] for i in range(q)]
    lams = [1.0] * q

    def run():
        rb.retrieve_many(S.lt, S.t_merged, S.t_base, req, lams, outs=t_outs)
    run()
    ts = []
    for _ in range(6):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); run(); b.record(); b.synchronize()
        ts.append(a.elapsed_time(b))
    ms = sorted(ts)[len(ts) // 2]
    moved = S.n_elem * S.eb * (1 + 2 * q)
    return {"requests_per_pass": q, "ms_per_pass": ms, "ms_per_request": ms / q,
            "speedup_over_single_requests": single_ms * q / ms,
            "GBs_algorithmic (3 streams per request)": S.n_elem * S.eb * 3 * q / (ms * 1e-3) / 1e9,
            "GBs_moved (1 + 2 q streams)": moved / (ms * 1e-3) / 1e9}


def brief(m):
    """The figures of one measured workload that go into the lists of the JSON line."""
    return {"ms_per_step": m["ms_per_step"], "GBs": m["GBs"], "frac_of_hbm_peak": m["frac_of_hbm_peak"],
            "merge": {k: m["merge"][k] for k in ("ms_avg", "GBs", "frac_of_hbm_peak")},
            "retrieve": {k: m["retrieve"][k] for k in ("ms_avg", "ms_min", "GBs", "frac_of_hbm_peak")}}


def one_line(name, m):
    return "%s: step %.0f GB/s (%.3f), merge %.3f ms %.0f GB/s (%.3f), retrieve %.3f ms %.0f GB/s (%.3f)" % (
        name, m["GBs"], m["frac_of_hbm_peak"], m["merge"]["ms_avg"], m["merge"]["GBs"], m["merge"]["frac_of_hbm_peak"],
        m["retrieve"]["ms_avg"], m["retrieve"]["GBs"], m["retrieve"]["frac_of_hbm_peak"])


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this benchmark runs on one GPU only (the path would shard by rows with no "
              "communication, so more GPUs add nothing to measure); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    rb.lib()
    torch.cuda.set_device(0)
    rb.set_tile_rows(args.merge_rows, args.retrieve_rows)
    rb.set_fold(not args.no_fold)

    head_fn, head_dtype, head_K = WORKLOADS[args.workload][:3]
    head_stack = head_fn()
    head_bytes = wl.stack_elements(head_stack, wl.torch_dtype(head_dtype)) * (4 if head_dtype == "f32" else 2)
    small = head_bytes < (256 << 20) and args.no_others      # nothing in this run is large enough to place
    pl = Placement("plain" if small else args.placement, head_bytes, args.tasks or head_K)
    S = Setup(args.workload, pl, args.tasks, args.requests, MANY_Q - 1)

    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    ceil = None
    if not args.no_ceilings and S.n_elem * S.eb >= (1 << 28):
        ceil = ceilings(S.flats, S.merged_flat, S.out_flat)
        torch.cuda.synchronize()

    first = S.first_calls()
    m = S.measure(args.steps, args.warmup)
    traffic, stale = profile_traffic(args.workload)

    result = {
        "metric": "merge & retrieve GB/s (bytes moved) and % of MI355X HBM peak",
        "value": m["GBs"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "%s storage, f32 accumulate" % S.dtype,
        "data": "synthetic",
        "placement_fallback": bool(args.placement == "groups" and pl.fallback),
        "config": {
            "workload": S.describe(),
            "storage": S.dtype, "n_tasks": S.K, "requests_per_step": S.n_req, "lambda": 1.0,
            "algorithmic_bytes_per_step": S.bytes_step,
            "pct_of_hbm_peak": 100.0 * m["frac_of_hbm_peak"],
            "merge": dict(m["merge"], pct_of_hbm_peak=100.0 * m["merge"]["frac_of_hbm_peak"]),
            "retrieve": dict(m["retrieve"], pct_of_hbm_peak=100.0 * m["retrieve"]["frac_of_hbm_peak"]),
            "first_call_with_table_build_and_upload": first,
            "hbm_placement": S.placed,
        },
        "roofline": {"kernel": "retrieve_kernel", "bound": "hbm", "achieved": m["retrieve"]["GBs"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": m["retrieve"]["frac_of_hbm_peak"],
                     "traffic": traffic.get("retrieve_kernel")},
        "roofline_merge": {"kernel": "merge_kernel", "bound": "hbm", "achieved": m["merge"]["GBs"],
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": m["merge"]["frac_of_hbm_peak"],
                           "traffic": traffic.get("merge_kernel")},
    }
    if stale:
        result["roofline"]["traffic_stale"] = result["roofline_merge"]["traffic_stale"] = stale
    cfg = result["config"]
    cfg["host_time_per_cached_call"] = S.host_time_per_cached_call()
    if ceil is not None:
        cfg["plain_streaming_probe"] = ceil
    if not args.no_extras:
        cfg["other_entry_points"] = widened_rows(S)
        many = many_extras(S, m["retrieve"]["ms_avg"])
        if many is not None:
            cfg["retrieve_many"] = many
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(S, args.cpu_sample_elems)
    head_name, head_tasks, head_req = S.name, S.K, S.n_req
    del S
    torch.cuda.empty_cache()

    if not args.no_others:
        others, lines = {}, []
        for name in OTHERS:
            if name == head_name:
                continue
            W = Setup(name, pl)
            W.first_calls()
            mw = W.measure(5, 2)
            entry = dict(brief(mw), workload=W.describe(), placement=W.placed["policy"])
            try:
                gs = W.step_in_a_graph()
            except Exception as e:      # the timed figures above do not depend on this extra
                gs = {"error": (str(e).splitlines() or [type(e).__name__])[0][:200]}
                torch.cuda.synchronize()
            entry["step_replayed_from_a_hip_graph"] = gs
            tw, stale_w = profile_traffic(name)
            if tw:
                entry["traffic"] = {"merge_kernel": tw.get("merge_kernel"), "retrieve_kernel": tw.get("retrieve_kernel")}
            if name in PAPER_RETRIEVE_MS:
                entry["paper_retrieve_one_model (context: another machine, not a target)"] = PAPER_RETRIEVE_MS[name]
            others[name] = entry
            lines.append(one_line(name, mw) + (", step replayed from a HIP graph %.0f GB/s (%.3f)" % (
                gs["GBs"], gs["frac_of_hbm_peak"]) if "GBs" in gs else ", step replayed from a HIP graph: failed"))
            del W
            torch.cuda.empty_cache()
        lv = lora_variant(pl)
        others["t5_base_lora_rank16"] = lv
        lines.append("t5_base_lora_rank16: " + ", ".join(
            "%s %.1f us %.0f GB/s (%.3f)" % (k.split(" ")[0], v["ms_back_to_back"] * 1e3, v["GBs"], v["frac_of_hbm_peak"])
            for k, v in lv.items() if isinstance(v, dict)))
        cfg["other_workloads"] = others
        cfg["other_workloads_summary"] = "; ".join(lines)
        # the headline workload once more, every stack in an allocation of its own
        if pl.arena is not None:
            pl.close()
            P = Setup(head_name, Placement("plain", 0, 0), head_tasks, head_req)
            P.first_calls()
            plain, plain_run = P.measure(3, 1), {"steps": 3, "warmup": 1}
            del P
            torch.cuda.empty_cache()
            note = ("the same workload with one ordinary allocation per stack: what a caller gets who does not "
                    "place the stacks by address group")
        else:
            plain, plain_run = m, {"steps": args.steps, "warmup": args.warmup}
            note = "the headline run itself used ordinary allocations"
        cfg["plain_placement"] = dict(brief(plain), value=plain["GBs"], note=note, **plain_run)
        cfg["plain_placement_summary"] = one_line(head_name + " with ordinary allocations", plain)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
