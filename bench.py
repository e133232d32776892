#!/usr/bin/env python3
"""Benchmark of the replay-evaluation hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one candidate evaluation through r3_eval_candidate: batched restore of the
recorded prologue, launch of the candidate kernel, fused compare+checksum against the
recorded epilogue, summary back to the host.  Inputs (snapshots, golden state, tables) are
resident in HBM before the timed region starts.  Prints ONE JSON line.

Workloads (shapes of the five benchmark configurations):
  large_snapshot  16 x 2 GiB regions (fp32 / bf16), 32 GiB per arena (default: the largest state
                  that fits one GPU and the one the HBM-roofline figure is quoted on)
  jacobi          256^3 fp64 7-point Jacobi, 8 candidate variants
  replay_small    3 x 2^20 fp32 inputs + 2^20 fp32 output, pure restore -> validate replays
  many_regions    4096 regions, 256 B .. 1 MiB, ~0.5 GiB: restore + validate the whole table
  spmv            CSR SpMV, 2^21 rows x 27 nnz, 64 launch configurations
The default run also records short legs of the other four workloads (evaluations/s, stage rates,
their own CPU baseline), the bandwidth yardsticks (plain copy, two-stream read) and the validation
of states that differ from the recorded one in every element.
"""
import argparse
import collections
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE (profiles/bench_large_snapshot_and_other_workloads_hbm_counters.txt),
# each scaled by what the same counter reads for a plain 1 GiB copy (FETCH 2.0, WRITE 1.0).
# Valid only for the kernel source they were taken with: reported as null otherwise.
COUNTERS = {
    "kernels_sha256_16": "1ee79119fcf5ac86",
    "jacobi": {"restore": 541105126, "validate": 269493419},
    "large_snapshot": {"restore": 68754965277, "validate": 68734378414},
}


def measured_traffic(workload, stage):
    import hashlib
    src = os.path.join(ROOT, "paper_2604_11109_amd", "csrc", "r3_kernels.hip")
    try:
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    if sha != COUNTERS["kernels_sha256_16"]:
        return None
    return COUNTERS.get(workload, {}).get(stage)


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=None)
    p.add_argument("--warmup", type=int, default=None)
    p.add_argument("--workload", default="large_snapshot",
                   choices=["jacobi", "replay_small", "many_regions", "large_snapshot", "spmv"])
    p.add_argument("--inflight", type=int, default=2,
                   help="evaluations kept in flight (r3_eval_submit / r3_eval_wait); 1 = the synchronous "
                        "r3_eval_candidate")
    p.add_argument("--no-all-differ", action="store_true", help="skip the every-element-differs validation leg")
    p.add_argument("--no-others", action="store_true", help="skip the short legs of the other workloads")
    p.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run 5 plain copies of 1 GiB (plain_copy_kernel), the yardstick for "
                        "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    return p.parse_args()


class Replay:
    """Everything one workload keeps resident: tables, snapshots, live arena, candidates."""

    def __init__(self, name, r3, wl, ctx, torch):
        import numpy as np

        import r3_inputs as ri
        self.name, self.r3, self.ctx, self.torch = name, r3, ctx, torch
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
        self.launch, self.candidates, self.expect_pass = None, [None], [None]
        self.host_case = None
        self.baseline_index = 0
        if name == "jacobi":
            c = ri.jacobi(256)
            A = c["arena_bytes"]
            self.restore_tbl = r3.Table(ctx, c["restore_rows"], A)
            self.check_tbl = r3.Table(ctx, [c["check_rows"][1]], A)
            self.d_live = up(c["prologue"])
            self.d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
            self.d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
            self.launch = wl.jacobi_launch()
            base = wl.jacobi_args(c, 64, 1, 0)
            r3.r3_record(ctx, self.restore_tbl, self.d_live, self.launch, base, self.d_pro, self.d_epi)
            self.candidates = [wl.jacobi_args(c, b, u, g) for b, u, g in ri.JACOBI_VARIANTS]
            self.expect_pass = [g == 0 for _, _, g in ri.JACOBI_VARIANTS]
            self.host_case = c
            self.desc = "7-point Jacobi 256^3 fp64, 8 candidate variants, restore 2x128 MiB, validate 128 MiB"
        elif name == "replay_small":
            c = ri.replay_small()
            A = c["arena_bytes"]
            self.restore_tbl = r3.Table(ctx, c["restore_rows"], A)
            self.check_tbl = r3.Table(ctx, c["check_rows"], A)
            self.d_pro, self.d_epi, self.d_live = up(c["prologue"]), up(c["epilogue"]), up(c["live"])
            self.expect_pass = [False]
            self.host_case = c
            self.desc = "3 x 2^20 fp32 inputs restored, 2^20 fp32 output validated (rtol 1e-5, atol 1e-7)"
        elif name == "many_regions":
            c = ri.many_regions()
            A = c["arena_bytes"]
            self.restore_tbl = self.check_tbl = r3.Table(ctx, c["rows"], A)
            self.d_pro = up(c["snapshot"])
            self.d_epi = self.d_pro
            self.d_live = up(c["live"])
            self.expect_pass = [True]
            self.host_case = c
            self.desc = "4096 regions 256 B..1 MiB (fp32/fp64/int32/bf16), %.0f MiB, restore + validate" % (A / 2**20)
        elif name == "large_snapshot":
            c = ri.large_snapshot_device()
            A = c["arena_bytes"]
            self.restore_tbl = self.check_tbl = r3.Table(ctx, c["rows"], A)
            self.d_pro, self.d_epi = c["snapshot"], c["golden"]
            self.d_live = torch.empty(A, dtype=torch.uint8, device="cuda:0")
            self.expect_pass = [False]
            self.n_planted = sum(len(i) for i in c["planted"])
            self.desc = "16 regions x 2 GiB (8 fp32, 8 bf16), restore 32 GiB + validate against golden"
        elif name == "spmv":
            c = ri.spmv()
            A = c["arena_bytes"]
            self.restore_tbl = r3.Table(ctx, c["table_rows"], A)
            self.check_tbl = r3.Table(ctx, c["y_rows"], A)
            self.d_live = up(c["prologue"])
            self.d_pro = torch.empty(A, dtype=torch.uint8, device="cuda:0")
            self.d_epi = torch.empty(A, dtype=torch.uint8, device="cuda:0")
            self.launch = wl.spmv_launch()
            r3.r3_record(ctx, self.restore_tbl, self.d_live, self.launch, wl.spmv_args(c, 64, 256),
                         self.d_pro, self.d_epi)
            self.candidates = [wl.spmv_args(c, r, b) for r, b in ri.SPMV_VARIANTS]
            self.baseline_index = ri.SPMV_VARIANTS.index((64, 256))
            self.expect_pass = [True if r >= 64 else None for r, _ in ri.SPMV_VARIANTS]
            self.host_case = c
            self.desc = "CSR SpMV 2^21 rows x 27 nnz fp64, 64 launch configurations, full-arena restore 688 MiB"
        self.arena_bytes = A
        self.d_regions = torch.zeros(40 * self.check_tbl.n, dtype=torch.uint8, device="cuda:0")
        self.d_regions_ring = []  # one result array per evaluation in flight
        self.restore_bytes = 2 * self.restore_tbl.info()["total_bytes"]
        self.validate_bytes = 2 * self.check_tbl.info()["total_bytes"]

    def enable_writeset(self, page=4096):
        """Record once more with the dirty bitmap and build the write-set / guard tables."""
        import numpy as np
        r3, ctx, torch = self.r3, self.ctx, self.torch
        A = self.arena_bytes
        d_bm = torch.zeros(r3.bitmap_words(A, page), dtype=torch.int64, device="cuda:0")
        self.d_live.copy_(self.d_pro)
        r3.r3_record(ctx, self.restore_tbl, self.d_live, self.launch, self.candidates[self.baseline_index],
                     self.d_pro, self.d_epi, page, d_bm)
        bm = d_bm.cpu().numpy().view(np.uint64)
        self.ws_tbl = r3.Table(ctx, r3.r3_writeset_regions(bm, A, page, 1), A)
        self.guard_tbl = r3.Table(ctx, r3.r3_writeset_regions(bm, A, page, 0), A)
        self.heal_tbl = r3.Table(ctx, [(0, A, 0, 0, 0.0, 0.0)], A)
        self.d_expected = torch.zeros(self.guard_tbl.n, dtype=torch.int64, device="cuda:0")
        self.d_scratch = torch.zeros(self.guard_tbl.n, dtype=torch.int64, device="cuda:0")
        r3.r3_checksum(ctx, self.guard_tbl, self.d_pro, self.d_expected)
        torch.cuda.synchronize()
        self.d_live.copy_(self.d_pro)
        return {"write_set_bytes": self.ws_tbl.info()["total_bytes"],
                "guarded_bytes": self.guard_tbl.info()["total_bytes"]}

    def step_writeset(self, i, guard_every=8):
        """Restore only the recorded write-set; every guard_every-th evaluation also checks that
        the rest of the state still carries its recorded checksums."""
        k = i % len(self.candidates)
        if i % guard_every == guard_every - 1:
            rc, out, g = self.r3.r3_eval_candidate_guarded(
                self.ctx, self.ws_tbl, self.d_pro, self.check_tbl, self.d_epi, self.d_live, self.launch,
                self.candidates[k], 0, 1, self.r3.EVERY, self.d_regions, self.guard_tbl, self.d_expected,
                self.d_scratch, every=0, heal_tbl=self.heal_tbl)
            if g.failed_checks:
                raise RuntimeError("guard failed for candidate %d" % k)
        else:
            rc, out = self.r3.r3_eval_candidate(self.ctx, self.ws_tbl, self.d_pro, self.check_tbl, self.d_epi,
                                                self.d_live, self.launch, self.candidates[k], 0, 1,
                                                self.r3.EVERY, self.d_regions)
        want = self.expect_pass[k]
        if rc != 0 or (want is not None and bool(out.passed) != want):
            raise RuntimeError("write-set evaluation %d of %s gave pass=%d (expected %s), status %d"
                               % (i, self.name, out.passed, want, rc))
        return out

    def submit_writeset(self, i, slot, guard_every=8):
        k = i % len(self.candidates)
        while len(self.d_regions_ring) <= slot:
            self.d_regions_ring.append(self.torch.zeros_like(self.d_regions))
        guarded = i % guard_every == guard_every - 1
        if guarded:
            t = self.r3.r3_eval_submit_guarded(
                self.ctx, self.ws_tbl, self.d_pro, self.check_tbl, self.d_epi, self.d_live, self.launch,
                self.candidates[k], 0, 1, self.r3.EVERY, self.d_regions_ring[slot], self.guard_tbl,
                self.d_expected, self.d_scratch, every=0, heal_tbl=self.heal_tbl)
        else:
            t = self.r3.r3_eval_submit(self.ctx, self.ws_tbl, self.d_pro, self.check_tbl, self.d_epi,
                                       self.d_live, self.launch, self.candidates[k], 0, 1, self.r3.EVERY,
                                       self.d_regions_ring[slot])
        return t, i, k

    def finish_writeset(self, t, i, k):
        rc, out, g = self.r3.r3_eval_wait(self.ctx, t, with_guard=True)
        if g.failed_checks:
            raise RuntimeError("guard failed for candidate %d" % k)
        want = self.expect_pass[k]
        if rc != 0 or (want is not None and bool(out.passed) != want):
            raise RuntimeError("write-set evaluation %d of %s gave pass=%d (expected %s), status %d"
                               % (i, self.name, out.passed, want, rc))
        return out

    def step(self, i):
        k = i % len(self.candidates)
        rc, out = self.r3.r3_eval_candidate(self.ctx, self.restore_tbl, self.d_pro, self.check_tbl,
                                            self.d_epi, self.d_live, self.launch, self.candidates[k],
                                            0, 1, self.r3.EVERY, self.d_regions)
        want = self.expect_pass[k]
        if rc != 0 or (want is not None and bool(out.passed) != want):
            raise RuntimeError("evaluation %d of %s gave pass=%d (expected %s), status %d"
                               % (i, self.name, out.passed, want, rc))
        return out


    def submit(self, i, slot):
        k = i % len(self.candidates)
        while len(self.d_regions_ring) <= slot:
            self.d_regions_ring.append(self.torch.zeros_like(self.d_regions))
        t = self.r3.r3_eval_submit(self.ctx, self.restore_tbl, self.d_pro, self.check_tbl, self.d_epi,
                                   self.d_live, self.launch, self.candidates[k], 0, 1, self.r3.EVERY,
                                   self.d_regions_ring[slot])
        return t, i, k

    def submit_overlapped(self, i, slot):
        """The same evaluation through the double-buffered pipeline: live arenas alternate."""
        k = i % len(self.candidates)
        while len(self.d_regions_ring) <= slot:
            self.d_regions_ring.append(self.torch.zeros_like(self.d_regions))
        if getattr(self, "d_live_pair", None) is None:
            self.d_live_pair = [self.d_live, self.d_live.clone()]
        t = self.r3.r3_eval_submit_overlapped(self.ctx, self.restore_tbl, self.d_pro, self.check_tbl, self.d_epi,
                                              self.d_live_pair[i % 2], self.launch, self.candidates[k], 0, 1,
                                              self.r3.EVERY, self.d_regions_ring[slot])
        return t, i, k

    def finish(self, t, i, k):
        rc, out = self.r3.r3_eval_wait(self.ctx, t)
        want = self.expect_pass[k]
        if rc != 0 or (want is not None and bool(out.passed) != want):
            raise RuntimeError("evaluation %d of %s gave pass=%d (expected %s), status %d"
                               % (i, self.name, out.passed, want, rc))
        return out


def run_steps(rp, n, inflight):
    """n evaluations, each a whole restore -> candidate -> validate -> verdict on the host; with
    inflight > 1 the next ones are enqueued before the verdict of the oldest is waited for."""
    if inflight <= 1:
        for i in range(n):
            rp.step(i)
        return
    q = collections.deque()
    for i in range(n):
        q.append(rp.submit(i, i % inflight))
        if len(q) == inflight:
            rp.finish(*q.popleft())
    while q:
        rp.finish(*q.popleft())


def overlapped_leg(rp, steps, warmup, inflight=2):
    """Evaluations/s with two live arenas on the context's two streams (restore of one evaluation
    beside the validation of the one before; candidates still alone on the GPU)."""
    torch = rp.torch

    def run(n):
        q = collections.deque()
        for i in range(n):
            q.append(rp.submit_overlapped(i, i % inflight))
            if len(q) == inflight:
                rp.finish(*q.popleft())
        while q:
            rp.finish(*q.popleft())
    run(warmup + (warmup & 1))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return {"value": steps / dt, "unit": "evals/s", "ms_per_step": dt / steps * 1e3, "steps": steps,
            "evaluations_in_flight": inflight}


def timed_run(rp, steps, warmup, inflight=1):
    torch, ctx = rp.torch, rp.ctx
    run_steps(rp, warmup, inflight)
    ctx.profile(4 if steps >= 16 else 1)  # stage events on every 4th evaluation of the timed region
    ctx.profile_read(reset=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(rp, steps, inflight)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = ctx.profile_read(reset=True)
    ctx.profile(0)
    return t1 - t0, prof


def writeset_leg(rp, steps, warmup, inflight=1):
    """The same workload with write-set driven restore and a periodic whole-state guard."""
    info = rp.enable_writeset()
    torch = rp.torch

    def run(n):
        if inflight <= 1:
            for i in range(n):
                rp.step_writeset(i)
            return
        q = collections.deque()
        for i in range(n):
            q.append(rp.submit_writeset(i, i % inflight))
            if len(q) == inflight:
                rp.finish_writeset(*q.popleft())
        while q:
            rp.finish_writeset(*q.popleft())
    run(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    info.update({"value": steps / dt, "unit": "evals/s", "ms_per_step": dt / steps * 1e3, "steps": steps,
                 "guard_every": 8, "evaluations_in_flight": inflight,
                 "note": "restore covers only the pages the recorded kernel wrote; every 8th evaluation also "
                         "checksums the rest of the arena against the recorded checksums"})
    return info


def record_path_leg(rp, reps=10):
    """The record-time kernels on this workload's arena: checksum only, page dirty-diff and the
    whole-arena copy, each timed alone with events on the stream it runs on."""
    r3, ctx, torch = rp.r3, rp.ctx, rp.torch
    A = rp.arena_bytes
    tbl = rp.restore_tbl
    d_cs = torch.zeros(tbl.n, dtype=torch.int64, device="cuda:0")
    d_bm = torch.zeros(r3.bitmap_words(A, 4096), dtype=torch.int64, device="cuda:0")
    d_cnt = torch.zeros(1, dtype=torch.int64, device="cuda:0")

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    out = {}
    ms = timed(lambda: r3.r3_checksum(ctx, tbl, rp.d_pro, d_cs))
    b = tbl.info()["total_bytes"]
    out["checksum"] = {"ms": ms, "algorithmic_bytes": b, "GB/s": b / ms / 1e6}
    ms = timed(lambda: r3.r3_dirty_diff(ctx, rp.d_pro, rp.d_epi, A, 4096, d_bm, d_cnt))
    out["dirty_diff"] = {"ms": ms, "algorithmic_bytes": 2 * A, "GB/s": 2 * A / ms / 1e6,
                         "dirty_pages": int(d_cnt.cpu()[0])}
    return out


def stage_report(rp, prof):
    out = {}
    if prof.restore_launches:
        ms = prof.restore_ms / prof.restore_launches
        out["restore"] = {"ms": ms, "algorithmic_bytes": rp.restore_bytes,
                          "GB/s": rp.restore_bytes / ms / 1e6}
    if prof.validate_launches:
        ms = prof.validate_ms / prof.validate_launches
        out["validate"] = {"ms": ms, "algorithmic_bytes": rp.validate_bytes,
                           "GB/s": rp.validate_bytes / ms / 1e6}
    if prof.candidate_launches:
        out["candidate"] = {"ms": prof.candidate_ms / prof.candidate_launches}
    if "restore" in out and "validate" in out:
        tot_ms = out["restore"]["ms"] + out["validate"]["ms"]
        tot_b = rp.restore_bytes + rp.validate_bytes
        out["restore+validate"] = {"ms": tot_ms, "algorithmic_bytes": tot_b, "GB/s": tot_b / tot_ms / 1e6,
                                   "frac_of_hbm_peak": tot_b / tot_ms / 1e6 / HBM_PEAK_GBS}
    return out


def roofline(rp, stages):
    """The dominant kernel of the path (whichever of restore / validate takes longer per launch), plus
    the whole pipeline: all algorithmic bytes of one replay over the time of both stages."""
    cands = [(k, stages[k]) for k in ("restore", "validate") if k in stages]
    name, st = max(cands, key=lambda kv: kv[1]["ms"])
    kernel = "restore_kernel" if name == "restore" else "compare_kernel + compare_finalize_kernel"
    ach = st["GB/s"]
    out = {"bound": "hbm", "kernel": kernel, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
           "frac": ach / HBM_PEAK_GBS, "traffic": measured_traffic(rp.name, name),
           "algorithmic_bytes_per_launch": st["algorithmic_bytes"], "avg_launch_ms": st["ms"],
           "stage_fracs": {k: v["GB/s"] / HBM_PEAK_GBS for k, v in cands}}
    if "restore+validate" in stages:
        both = stages["restore+validate"]
        out["pipeline"] = {"achieved": both["GB/s"], "frac": both["frac_of_hbm_peak"], "ms": both["ms"],
                           "algorithmic_bytes": both["algorithmic_bytes"],
                           "slowest_stage": min(cands, key=lambda kv: kv[1]["GB/s"])[0]}
    if rp.restore_bytes + rp.validate_bytes < (256 << 20):
        out["note"] = ("the working set of this workload stays in the caches and a launch lasts microseconds: "
                       "latency-bound, the fraction is not a roofline claim (evaluations/s is the figure)")
    return out


def host_threads():
    """Threads the CPU baseline may use: the machine's CPU share (16 for one GPU), never more than the host has."""
    return max(1, min(16, os.cpu_count() or 1))


def cpu_model():
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(rp, budget_s=10.0):
    """The CPU oracle, untuned, on a bounded sample of the same workload: one thread, and for the large
    snapshot also one oracle call per host thread on disjoint chunks."""
    import numpy as np

    import r3_inputs as ri
    from oracle import r3_oracle as o
    if rp.name == "jacobi":
        c = rp.host_case
        n = c["n"]
        pro = c["prologue"]
        epi = rp.d_epi.cpu().numpy()
        rt = o.make_table(c["restore_rows"])
        ct = o.make_table([c["check_rows"][1]])
        live = np.zeros_like(pro)

        def sweep(a):
            g = a[c["in_off"]:c["in_off"] + c["grid_bytes"]].view("<f8").reshape(n, n, n)
            a[c["out_off"]:c["out_off"] + c["grid_bytes"]] = ri.jacobi_reference(g).reshape(-1).view(np.uint8)
            return 0
        evals = 0
        t0 = time.perf_counter()
        while True:
            res = o.eval_candidate(rt, pro, ct, epi, live, sweep, 0, 1)
            evals += 1
            if time.perf_counter() - t0 > budget_s or evals >= 8:
                break
        dt = time.perf_counter() - t0
        assert res["pass"] == 1
        return {"value": evals / dt, "unit": "evals/s", "cores": 1, "kind": "oracle",
                "sample": "%d evaluations of the 256^3 Jacobi replay (oracle restore 256 MiB, numpy sweep as the "
                          "candidate, oracle compare of the 128 MiB output)" % evals}
    if rp.name == "replay_small":
        c = rp.host_case
        rt, ct = o.make_table(c["restore_rows"]), o.make_table(c["check_rows"])
        live = c["live"].copy()
        evals, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < budget_s:
            o.eval_candidate(rt, c["prologue"], ct, c["epilogue"], live, None, 0, 1)
            evals += 1
        dt = time.perf_counter() - t0
        return {"value": evals / dt, "unit": "evals/s", "cores": 1, "kind": "oracle",
                "sample": "%d pure restore->validate replays at full size" % evals}
    if rp.name == "many_regions":
        c = rp.host_case
        t = o.make_table(c["rows"])
        live = c["live"].copy()
        evals, t0 = 0, time.perf_counter()
        while evals < 4 and (evals == 0 or time.perf_counter() - t0 < budget_s):
            res = o.eval_candidate(t, c["snapshot"], t, c["snapshot"], live, None, 0, 1)
            evals += 1
        dt = time.perf_counter() - t0
        assert res["pass"] == 1
        return {"value": evals / dt, "unit": "evals/s", "cores": 1, "kind": "oracle",
                "sample": "%d restore->validate replays of all 4096 regions" % evals}
    if rp.name == "spmv":
        c = rp.host_case
        rows = c["rows"]
        row_ptr, col, vals, x = c["csr"]
        y_off, y_bytes = c["offsets"]["y"], c["sizes"]["y"]
        rt, ct = o.make_table(c["table_rows"]), o.make_table(c["y_rows"])
        epi = rp.d_epi.cpu().numpy()
        live = np.zeros_like(c["prologue"])

        def product(a):
            y = (vals.reshape(rows, 27) * x[col]).sum(axis=1)
            a[y_off:y_off + y_bytes] = y.astype("<f8").view(np.uint8)
            return 0
        evals, t0 = 0, time.perf_counter()
        while evals < 4 and (evals == 0 or time.perf_counter() - t0 < budget_s):
            o.eval_candidate(rt, c["prologue"], ct, epi, live, product, 0, 1)
            evals += 1
        dt = time.perf_counter() - t0
        return {"value": evals / dt, "unit": "evals/s", "cores": 1, "kind": "oracle",
                "sample": "%d evaluations: oracle restore of the 688 MiB arena, numpy row sums as the "
                          "candidate, oracle compare of y (16 MiB)" % evals}
    if rp.name == "large_snapshot":
        return cpu_baseline_large(rp, o, np)
    return None


def cpu_baseline_large(rp, o, np):
    """Regions 0 (fp32) and 8 (bf16) of the 16, i.e. 4 GiB of the 32 GiB state, downloaded from the device.
    T = 1: the oracle's restore + compare on each of the two regions, one after the other.  T = host
    threads: the same bytes cut into 16 chunks of 256 MiB, each chunk a region of its own, one plain oracle
    call per chunk on a pool of T threads (the oracle itself stays single-threaded; counts add, indices
    take the minimum, maxima the maximum).  Times are scaled by 8 to the whole state."""
    import concurrent.futures as cf
    picked = (0, 8)
    host = []
    for r in picked:
        row = rp.check_tbl.host[r]
        off, nb = int(row["offset"]), int(row["bytes"])
        host.append((rp.d_pro[off:off + nb].cpu().numpy(), rp.d_epi[off:off + nb].cpu().numpy(),
                     tuple(row.tolist()[2:]), nb))
    scale = 16.0 / len(picked)
    bytes_per_eval = 4.0 * sum(h[3] for h in host) * scale       # restore 2 B/B + compare 2 B/B
    # T = 1
    t_single, counts = 0.0, []
    for snap, gold, tail, nb in host:
        live = np.empty_like(snap)
        tbl = o.make_table([(0, nb) + tail])
        t0 = time.perf_counter()
        res = o.eval_candidate(tbl, snap, tbl, gold, live, None, 0, 1)
        t_single += time.perf_counter() - t0
        counts.append(int(res["total_mismatch"]))
        del live
    per_eval = t_single * scale
    out = {"value": 1.0 / per_eval, "unit": "evals/s", "cores": 1, "kind": "oracle", "cpu": cpu_model(),
           "GB/s": bytes_per_eval / per_eval / 1e9,
           "sample": "restore+validate of regions 0 (fp32) and 8 (bf16), 4 GiB of the 32 GiB state (%.1f s of "
                     "CPU); time scaled by 8 to the whole state" % t_single}
    # T = host threads
    T = host_threads()
    jobs = []
    for snap, gold, tail, nb in host:
        step = nb // 8
        for k in range(8):
            jobs.append((snap[k * step:(k + 1) * step], gold[k * step:(k + 1) * step],
                         o.make_table([(0, step) + tail])))
    lives = [np.empty_like(j[0]) for j in jobs]

    def one(i):
        snap, gold, tbl = jobs[i]
        return int(o.eval_candidate(tbl, snap, tbl, gold, lives[i], None, 0, 1)["total_mismatch"])
    t0 = time.perf_counter()
    with cf.ThreadPoolExecutor(max_workers=T) as pool:
        chunk_counts = list(pool.map(one, range(len(jobs))))
    t_threads = time.perf_counter() - t0
    assert sum(chunk_counts) == sum(counts), "chunked oracle run disagrees with the whole-region run"
    per_eval_t = t_threads * scale
    out["threads"] = {"value": 1.0 / per_eval_t, "unit": "evals/s", "cores": T, "GB/s": bytes_per_eval / per_eval_t / 1e9,
                      "sample": "the same 4 GiB as 16 chunks of 256 MiB, one single-thread oracle call per chunk on "
                                "%d host threads (%.1f s); time scaled by 8" % (T, t_threads)}
    return out


def ceilings_leg(wl, torch, reps=10):
    """What this GPU gives the plainest kernels with the replay path's traffic shapes: a copy (one read
    and one write stream) and a two-stream read of 2 GiB per stream, 16-byte accesses, no table, no
    arithmetic beyond an XOR.  The best shape of each is the yardstick the stage rates are held against."""
    nbytes = 2 << 30
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    b = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    a.fill_(1)
    b.fill_(1)
    sink = torch.zeros(4, dtype=torch.uint8, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    out = {"bytes_per_stream": nbytes, "shapes": {}}
    for kib in (1, 4, 16):
        ms_c = timed(lambda: wl.yard_copy(a, b, nbytes, kib, stream))
        ms_r = timed(lambda: wl.yard_read2(a, b, nbytes, sink, kib, stream))
        out["shapes"]["%d KiB per wavefront" % kib] = {"copy_GBs": 2 * nbytes / ms_c / 1e6,
                                                       "read2_GBs": 2 * nbytes / ms_r / 1e6}
    out["copy_GBs"] = max(v["copy_GBs"] for v in out["shapes"].values())
    out["read2_GBs"] = max(v["read2_GBs"] for v in out["shapes"].values())
    del a, b
    torch.cuda.empty_cache()
    return out


def against_ceilings(stages, ceil):
    out = {}
    if "restore" in stages:
        out["restore_vs_copy"] = stages["restore"]["GB/s"] / ceil["copy_GBs"]
    if "validate" in stages:
        out["validate_vs_read2"] = stages["validate"]["GB/s"] / ceil["read2_GBs"]
    return out


def all_differ_leg(r3, ctx, torch, nbytes=256 << 20, reps=10):
    """Validation of a state that differs from the recorded one in EVERY element by one bit-pattern step
    (the pattern of a numerically equivalent rewrite under the relaxed criterion, Section V-C): one
    region of 256 MiB per element type, tolerance mode, rates incl. the finalize launch."""
    import r3_inputs as ri
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(4711)
    kinds = [("fp64", ri.F64, torch.float64, torch.int64, 1e-12, 0.0),
             ("fp32", ri.F32, torch.float32, torch.int32, 1e-5, 1e-7),
             ("bf16", ri.BF16, torch.bfloat16, torch.int16, 1e-2, 1e-3),
             ("fp16", ri.F16, torch.float16, torch.int16, 1e-2, 1e-3),
             ("int32", ri.I32, None, torch.int32, 0.0, 1.0),
             ("u8", ri.U8, None, torch.uint8, 0.0, 1.0)]
    d_out = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    d_sum = torch.zeros(40, dtype=torch.uint8, device="cuda:0")
    out = {}
    for name, dt, fdt, idt, rtol, atol in kinds:
        es = ri.ELEM_SIZE[dt]
        n = nbytes // es
        gold = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        if fdt is not None:
            for lo in range(0, n, 1 << 26):
                hi = min(n, lo + (1 << 26))
                gold.view(fdt)[lo:hi] = torch.randn(hi - lo, generator=gen, device="cuda:0",
                                                    dtype=torch.float32).to(fdt)
        else:
            gold.copy_(torch.randint(0, 256, (nbytes,), generator=gen, device="cuda:0", dtype=torch.uint8))
            if dt == ri.I32:
                gold.view(torch.int32).bitwise_and_(0x3FFFFFFF)
        live = gold.clone()
        live.view(idt).add_(1)                     # every element one pattern step away
        tbl = r3.Table(ctx, [(0, nbytes, dt, ri.TOL, rtol, atol)], nbytes)

        def run():
            r3.r3_compare(ctx, tbl, live, gold, d_out, d_sum)
        run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        res = r3.results_to_numpy(d_out, 1)[0]
        out[name] = {"ms": ms, "algorithmic_bytes": 2 * nbytes, "GB/s": 2 * nbytes / ms / 1e6,
                     "frac_of_hbm_peak": 2 * nbytes / ms / 1e6 / HBM_PEAK_GBS,
                     "mismatch_count": int(res["mismatch_count"]), "max_rel_err": float(res["max_rel_err"])}
        # the same region with nothing different, for comparison
        live.copy_(gold)
        run()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        out[name]["identical_GB/s"] = 2 * nbytes / (e0.elapsed_time(e1) / reps) / 1e6
        del tbl, live, gold
        torch.cuda.empty_cache()
    return out


def other_legs(r3, wl, ctx, torch, skip, inflight, defaults, ceil, with_cpu):
    """Evaluations/s, stage rates and the oracle's rate for the workloads that are not the headline one,
    so that one run records all five."""
    out = {}
    for name in ("jacobi", "replay_small", "many_regions", "spmv", "large_snapshot"):
        if name == skip:
            continue
        if name == "large_snapshot":
            free, _ = torch.cuda.mem_get_info()
            if free < 110 * (1 << 30):
                out[name] = {"skipped": "needs 96 GiB of free device memory, %.0f GiB free" % (free / 2**30)}
                continue
        rp = Replay(name, r3, wl, ctx, torch)
        steps, warmup = defaults[name]
        if name != "large_snapshot":
            steps = max(64, steps // 2)
        dt, prof = timed_run(rp, steps, warmup, inflight)
        st = stage_report(rp, prof)
        leg = {"workload": rp.desc, "value": steps / dt, "unit": "evals/s", "steps": steps,
               "ms_per_step": dt / steps * 1e3, "evaluations_in_flight": inflight, "stages": st,
               "roofline": roofline(rp, st), "vs_ceilings": against_ceilings(st, ceil)}
        if inflight > 1:
            dt1, _ = timed_run(rp, steps, warmup, 1)
            leg["synchronous"] = {"value": steps / dt1, "unit": "evals/s", "ms_per_step": dt1 / steps * 1e3}
        if name != "large_snapshot":
            leg["overlapped"] = overlapped_leg(rp, steps, warmup, max(2, inflight))
        if with_cpu:
            leg["cpu_baseline"] = cpu_baseline(rp, budget_s=3.0)
        if name in ("jacobi", "spmv"):
            leg["write_set_replay"] = writeset_leg(rp, steps, warmup, inflight)
        out[name] = leg
        del rp
        torch.cuda.empty_cache()
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (--gpus %d refused)" % a.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2604_11109_amd import binding as r3
    from paper_2604_11109_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    r3.lib()
    wl.lib()
    ctx = r3.Context(0)
    defaults = {"jacobi": (200, 16), "replay_small": (2000, 100), "many_regions": (200, 10),
                "large_snapshot": (20, 2), "spmv": (128, 8)}
    steps = a.steps if a.steps is not None else defaults[a.workload][0]
    warmup = a.warmup if a.warmup is not None else defaults[a.workload][1]
    if not 1 <= a.inflight <= 8:
        print("--inflight must be 1 .. 8", file=sys.stderr)
        sys.exit(2)
    if a.workload == "large_snapshot":
        free, _ = torch.cuda.mem_get_info()
        if free < 110 * (1 << 30):
            print("the large snapshot needs 96 GiB of free device memory, %.0f GiB free" % (free / 2**30),
                  file=sys.stderr)
            sys.exit(2)

    if a.calibrate_copy:
        buf = torch.zeros(2 << 30, dtype=torch.uint8, device="cuda:0")
        buf[:1 << 30].fill_(7)
        for _ in range(5):
            wl.plain_copy(buf, 0, 1 << 30, 1 << 30)
        torch.cuda.synchronize()
        del buf
        torch.cuda.empty_cache()

    ceil = ceilings_leg(wl, torch)
    rp = Replay(a.workload, r3, wl, ctx, torch)
    dt, prof = timed_run(rp, steps, warmup, a.inflight)
    stages = stage_report(rp, prof)
    line = {
        "metric": "candidate evals/sec per kernel; restore+compare GB/s as % of HBM peak",
        "value": steps / dt, "unit": "evals/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "%s: %s" % (a.workload, rp.desc), "evaluations_in_flight": a.inflight},
        "roofline": roofline(rp, stages),
        "stages": stages,
        "ceilings": ceil,
        "vs_ceilings": against_ceilings(stages, ceil),
    }
    if a.inflight > 1:
        dt1, _ = timed_run(rp, steps, warmup, 1)
        line["synchronous"] = {"value": steps / dt1, "unit": "evals/s", "ms_per_step": dt1 / steps * 1e3,
                               "note": "the same evaluations through r3_eval_candidate, one at a time"}
    if a.workload != "large_snapshot":
        line["overlapped"] = overlapped_leg(rp, steps, warmup, max(2, a.inflight))
    line["cpu_baseline"] = None if a.no_cpu else cpu_baseline(rp)
    line["record_path"] = record_path_leg(rp, reps=3 if a.workload == "large_snapshot" else 10)
    if a.workload in ("jacobi", "spmv"):
        line["write_set_replay"] = writeset_leg(rp, steps, warmup, a.inflight)
    del rp
    torch.cuda.empty_cache()
    if not a.no_all_differ:
        line["all_differ"] = all_differ_leg(r3, ctx, torch)
    if not a.no_others:
        line["other_workloads"] = other_legs(r3, wl, ctx, torch, a.workload, a.inflight, defaults, ceil,
                                             not a.no_cpu)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
