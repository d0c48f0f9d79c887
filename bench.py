#!/usr/bin/env python3
"""Benchmark of the deduplicated-embedding hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic session-structured batch:
  recd_build_ikjt -> recd_pooled_lookup_unique -> recd_expand_inverse (--one-pass-forward:
  recd_build_ikjt_runs -> recd_pooled_lookup_expand) -> recd_backward_plan / recd_backward_apply
  (inverse aggregation, sorted segment-reduce, row-wise Adagrad).
Inputs (KJT, tables, upstream gradient) are resident in HBM before the timed region; steps rotate
over several different seeded batches so that table rows are not served from a warm cache.
The non-deduplicated KJT lookup (comparison path) is timed separately on the same batches.

Prints ONE JSON line.  `value` = pooled lookups per second = B*F / step time (median of the
HIP-event-timed steps; the wall-clock mean is reported beside it).  The default run also measures the
other benchmark configurations (cfg1-cfg3, forward only) and the duplication sweep (cfg4).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="cfg5",
                    help="cfg1..cfg5 or cfg4_S<k> (duplication sweep member)")
    ap.add_argument("--batches", type=int, default=4, help="distinct seeded batches to rotate over")
    ap.add_argument("--cpu-features", type=int, default=64,
                    help="features of batch 0 the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-sweep", dest="sweep", action="store_false",
                    help="skip the duplication sweep (cfg4, S in 1,2,4,8,32)")
    ap.add_argument("--no-others", dest="others", action="store_false",
                    help="skip the other configurations (cfg1, cfg2, cfg3, forward only)")
    ap.add_argument("--forward", choices=("auto", "two-call", "one-pass"), default="auto",
                    help="how the step runs the unique lookup and the expand: as two calls (recd_build_ikjt + "
                         "recd_pooled_lookup_unique + recd_expand_inverse), as the one-pass call "
                         "(recd_build_ikjt_runs + recd_pooled_lookup_expand), or auto = whichever is the faster "
                         "on this chip for the workload's shape (one pass for batches of at most 16384 rows, "
                         "where launches count, and for 16-bit tables; two calls otherwise); the step is also "
                         "timed in the other form, and both calls are timed alone in `regions` either way")
    ap.add_argument("--one-pass-forward", dest="forward", action="store_const", const="one-pass",
                    help="same as --forward one-pass")
    ap.add_argument("--steps-only", action="store_true",
                    help="run only the warm-up and the timed steps of the workload (the run to profile: no "
                         "per-call passes, no comparison path, no CPU baseline, no other configurations)")
    ap.add_argument("--forward-only", action="store_true", help="leave the backward pass out of the step")
    ap.add_argument("--store-grad", action="store_true",
                    help="also store the per-row gradients (default: the fused Adagrad update consumes them "
                         "from registers)")
    ap.add_argument("--sequence", action="store_true",
                    help="also time the unpooled path (sequence lookup on the unique lists + jagged expand) "
                         "and its non-deduplicated comparison; reported beside the step, not part of it")
    ap.add_argument("--groups", type=int, default=0,
                    help="also time the grouped IKJT path with groups of this many consecutive features "
                         "(builder, group-sum module on the unique rows, one expand per group) beside the "
                         "same module run on the expanded KJT rows")
    ap.add_argument("--partial", type=float, default=0.0,
                    help="also time the partial IKJT path on the workload with this probability of a "
                         "sample's lists shifting by one id within a session (0 = skip)")
    ap.add_argument("--plan-from-runs", dest="run_plan", action="store_true",
                    help="the backward's plan sorts the batch's runs (recd_build_ikjt_runs + "
                         "recd_backward_plan_runs) instead of all F*B rows by unique list (recd_build_ikjt + "
                         "recd_backward_plan); measured a few microseconds slower per step at cfg5")
    ap.add_argument("--one-call-backward", dest="planned", action="store_false",
                    help="run the backward as one call after the expand instead of plan (next to the forward "
                         "calls) + apply")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from captured HIP graphs (launches sized by host upper "
                         "bounds of U and M; reported beside `value`)")
    ap.add_argument("--weights", action="store_true",
                    help="also time the per-id-weight calls (weighted builder, lookups, backward) on the same "
                         "batches with seeded weights, and the backward of average and max pooling")
    ap.add_argument("--reader", action="store_true",
                    help="also report the builder alone (the conversion step of a reader) beside the CPU "
                         "oracle's builder run feature-parallel on the host cores")
    ap.add_argument("--pipeline", action="store_true",
                    help="also run the steps with the builder on a second stream (reported beside the step, "
                         "never as `value`)")
    ap.add_argument("--tune", type=int, default=0, help="launch-shape override of the gather-sum kernel (tuning runs; 0 = automatic)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (calibrates hardware byte counters)")
    return ap.parse_args()


_TABLE_CACHE = {}


def make_tables(torch, synth, w, tdt):
    """F seeded tables on the device (N(0, 0.01^2), cast to the table dtype).  Workloads that differ
    only in their session structure (the sweep) share one set."""
    key = (w.index, w.F, w.rows, w.D, w.table_dtype)
    if key not in _TABLE_CACHE:
        _TABLE_CACHE.clear()   # one set at a time: cfg5's tables are 33 GB
        torch.cuda.empty_cache()
        gen = torch.Generator(device="cuda")
        gen.manual_seed(synth.BASE_SEED + 1000 * w.index + 777)
        tabs = []
        for _ in range(w.F):
            t = torch.empty(w.rows, w.D, dtype=torch.float32, device="cuda")
            t.normal_(0.0, 0.01, generator=gen)
            tabs.append(t.to(tdt) if tdt != torch.float32 else t)
        _TABLE_CACHE[key] = tabs
    return _TABLE_CACHE[key]


class DeviceProblem:
    """Everything one workload needs on the device, allocated once at worst-case sizes."""

    def __init__(self, torch, recd, synth, w, n_batches, need_backward, store_grad=False, tune=0):
        self.torch, self.w, self.recd = torch, w, recd
        F, B, D = w.F, w.B, w.D
        self.tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[w.table_dtype]
        self.batches = [synth.make_batch(w, i) for i in range(n_batches)]
        self.values = [torch.from_numpy(b.values).cuda() for b in self.batches]
        self.offsets = [torch.from_numpy(b.offsets).cuda() for b in self.batches]
        self.tables = make_tables(torch, synth, w, self.tdt)
        Nmax = max(b.N for b in self.batches)
        # one IKJT per batch, so that the per-call timings can run the same call on all batches
        # back to back
        self.u_values = [torch.zeros(b.N, dtype=torch.int64, device="cuda") for b in self.batches]
        self.u_offsets = [torch.zeros(F * B + 1, dtype=torch.int64, device="cuda") for _ in self.batches]
        self.inverse = [torch.zeros(F * B, dtype=torch.int32, device="cuda") for _ in self.batches]
        self.feat_uoff = [torch.zeros(F + 1, dtype=torch.int64, device="cuda") for _ in self.batches]
        self.runs = [torch.zeros(3 * (F * B + 2), dtype=torch.int64, device="cuda") for _ in self.batches]
        self.pooled = torch.zeros(F * B, D, dtype=self.tdt, device="cuda")
        self.out = torch.zeros(F, B, D, dtype=self.tdt, device="cuda")
        self.kjt_out = torch.zeros(F, B, D, dtype=self.tdt, device="cuda")
        self.need_backward = need_backward
        self.planned = True
        self.fused_forward = False
        self.run_plan = False
        ws = recd.workspace_bytes(F, B, Nmax, D)
        self.ctx = recd.Context(0, workspace_hint_bytes=ws)
        if tune:
            self.ctx.set_option(recd._OPT_INTERNAL_TUNE_SEGSUM, tune)
        # unique-list counts of every batch (U, M): size the backward outputs by the largest M
        self.counts = [self.build(i) for i in range(n_batches)]
        if need_backward:
            Mmax = max(c[1] for c in self.counts)
            g = torch.Generator(device="cuda")
            g.manual_seed(synth.BASE_SEED + 1000 * w.index + 500)
            self.grad_out = torch.empty(F, B, D, dtype=torch.float32, device="cuda")
            self.grad_out.normal_(0.0, 0.01, generator=g)
            self.touched = torch.zeros(Mmax, dtype=torch.int64, device="cuda")
            self.feat_roff = torch.zeros(F + 1, dtype=torch.int64, device="cuda")
            self.grad_rows = torch.zeros(Mmax, D, dtype=torch.float32, device="cuda") if store_grad else None
            self.state = [torch.zeros(w.rows, dtype=torch.float32, device="cuda") for _ in range(F)]
        self.rows = [w.rows] * F
        self.u_hint = F * B

    # --- the calls of one step; each returns nothing and enqueues on torch's current stream ----
    def build(self, i, counts=True, runs=None):
        w = self.w
        if runs is None:
            runs = self.fused_forward or (self.run_plan and self.planned and self.need_backward)
        if not runs:
            return self.ctx.build_ikjt(w.F, w.B, self.values[i], self.offsets[i], self.u_values[i],
                                       self.u_offsets[i], self.inverse[i], self.feat_uoff[i], want_counts=counts)
        return self.ctx.build_ikjt_runs(w.F, w.B, self.values[i], self.offsets[i], self.u_values[i],
                                        self.u_offsets[i], self.inverse[i], self.feat_uoff[i], self.runs[i],
                                        want_counts=counts)

    def lookup(self, i, U=None):
        w = self.w
        self.ctx.pooled_lookup_unique(self.tables, self.u_values[i], self.u_offsets[i],
                                      self.feat_uoff[i], w.F * w.B if U is None else U, self.pooled)

    def expand(self, i):
        w = self.w
        self.ctx.expand_inverse(w.F, w.B, self.pooled, self.feat_uoff[i], self.inverse[i], self.out)

    def fused(self, i, U=None):
        w = self.w
        # U + U/16: the runs are the unique lists plus the lists that come back later in the batch
        est = w.F * w.B if U is None else U + U // 16
        self.ctx.pooled_lookup_expand(self.tables, w.B, self.u_values[i], self.runs[i], est, self.pooled, self.out)

    def forward(self, i, U=None):
        if self.fused_forward:
            self.fused(i, U)
        else:
            self.lookup(i, U)
            self.expand(i)

    def backward(self, i, U, M, want_count=False):
        w = self.w
        return self.ctx.backward_dedup(w.F, w.B, self.grad_out, self.inverse[i], self.feat_uoff[i],
                                       self.u_values[i], self.u_offsets[i], self.rows, U, M, self.touched,
                                       self.feat_roff, self.grad_rows, tables=self.tables,
                                       adagrad_state=self.state, lr=0.01, eps=1e-8,
                                       want_count=want_count)

    def kjt(self, i):
        w = self.w
        self.ctx.kjt_pooled_lookup(self.tables, w.B, self.values[i], self.offsets[i], self.kjt_out)

    def step(self, i):
        # The lookup and the expand need no host-side count (any max_lists sizes the launch; the last
        # step's U is the estimate), so they are enqueued right behind the build; U and M come back to
        # the host while they run and bound the backward's sorts.
        self.build(i, counts=False)
        self.forward(i, self.u_hint)
        U, M = self.ctx.last_ikjt_counts()
        self.u_hint = max(U, 1)
        if self.need_backward:
            if self.planned:
                # the backward's grouping half depends on the IKJT only: it runs on the context's side
                # streams from the end of the build on, next to lookup and expand; the sums follow
                w = self.w
                if self.run_plan:
                    self.ctx.backward_plan_runs(w.F, w.B, w.D, self.inverse[i], self.feat_uoff[i], self.u_values[i],
                                                self.u_offsets[i], self.rows, U, M, self.runs[i],
                                                self.ctx.last_ikjt_run_count(), self.touched, self.feat_roff)
                else:
                    self.ctx.backward_plan(w.F, w.B, w.D, self.inverse[i], self.feat_uoff[i], self.u_values[i],
                                           self.u_offsets[i], self.rows, U, M, self.touched, self.feat_roff)
                self.ctx.backward_apply(self.grad_out, self.grad_rows, tables=self.tables,
                                        adagrad_state=self.state, lr=0.01, eps=1e-8)
            else:
                self.backward(i, U, M)
        return U, M

    def ikjt_shape(self, i, U):
        """(distinct (feature, row) pairs of the unique ids, batch rows in the first run of their list)
        of batch i's resident IKJT: sizes of the bytes model, counted with torch on the device."""
        torch, w = self.torch, self.w
        F, B = w.F, w.B
        fu = self.feat_uoff[i].cpu().tolist()
        uo = self.u_offsets[i]
        R = 0
        for f in range(F):
            lo, hi = int(uo[fu[f]].item()), int(uo[fu[f + 1]].item())
            if hi > lo:
                R += int(torch.unique(self.u_values[i][lo:hi]).numel())
        # rows of the first runs: run r covers [row_r, row_{r+1}); the flag is bit 63 of its first word
        ri = self.runs[i]
        n_runs = int(ri[0].item())
        w0 = ri[3:3 * (n_runs + 2):3]
        row = w0 & 0xffffffff
        covered = int(((row[1:] - row[:-1]) * (w0[:-1] < 0)).sum().item())
        self.n_runs = n_runs
        return R, covered


def pipelined_steps(torch, recd, P, args):
    """The same K steps with the builder of batch k+1 on a second stream (its own context and
    workspace) next to lookup, expand and backward of batch k on the main stream.  Every step still
    runs all four calls on its batch, in order; only the host's wait for U and M no longer idles
    the GPU.  Returns ms per step."""
    w = P.w
    nb = len(P.batches)
    s2 = torch.cuda.Stream()
    ctx2 = recd.Context(0, workspace_hint_bytes=recd.workspace_bytes(w.F, w.B, max(b.N for b in P.batches), w.D),
                        stream=s2.cuda_stream)
    done = [torch.cuda.Event() for _ in range(nb)]   # main stream has finished with batch i's IKJT

    def build_on_s2(i):
        s2.wait_event(done[i])
        if not P.fused_forward:
            return ctx2.build_ikjt(w.F, w.B, P.values[i], P.offsets[i], P.u_values[i], P.u_offsets[i],
                                   P.inverse[i], P.feat_uoff[i], want_counts=True)
        return ctx2.build_ikjt_runs(w.F, w.B, P.values[i], P.offsets[i], P.u_values[i], P.u_offsets[i],
                                    P.inverse[i], P.feat_uoff[i], P.runs[i], want_counts=True)

    def run(steps):
        pending = build_on_s2(0)
        for k in range(steps):
            i = k % nb
            U, M = pending
            torch.cuda.current_stream().wait_stream(s2)   # the IKJT of batch i is complete
            P.forward(i, U)
            if P.need_backward:
                P.backward(i, U, M)
            done[i].record()
            if k + 1 < steps:
                pending = build_on_s2((k + 1) % nb)
        torch.cuda.synchronize()

    for i in range(nb):
        done[i].record()
    run(max(args.warmup, 2))
    t0 = time.perf_counter()
    run(args.steps)
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ctx2.close()
    return ms


def graph_steps(torch, recd, P, args, stats):
    """The same K steps replayed from HIP graphs, one graph per resident batch, captured on a stream
    of their own.  Inside a graph nothing can come back to the host, so the later calls are sized by
    host upper bounds (the largest U and M of the rotated batches) instead of the builder's counts;
    the kernels read the true counts on the device.  Returns ms per step."""
    w = P.w
    F, B = w.F, w.B
    nb = len(P.batches)
    U_cap = int(max(st[0] for st in stats))
    M_cap = int(max(st[1] for st in stats))
    s3 = torch.cuda.Stream()
    ctx3 = recd.Context(0, workspace_hint_bytes=recd.workspace_bytes(F, B, max(b.N for b in P.batches), w.D),
                        stream=s3.cuda_stream)

    def step(i):
        if P.fused_forward:
            ctx3.build_ikjt_runs(F, B, P.values[i], P.offsets[i], P.u_values[i], P.u_offsets[i], P.inverse[i],
                                 P.feat_uoff[i], P.runs[i])
            ctx3.pooled_lookup_expand(P.tables, B, P.u_values[i], P.runs[i], U_cap + U_cap // 16, P.pooled, P.out)
        else:
            ctx3.build_ikjt(F, B, P.values[i], P.offsets[i], P.u_values[i], P.u_offsets[i], P.inverse[i],
                            P.feat_uoff[i])
            ctx3.pooled_lookup_unique(P.tables, P.u_values[i], P.u_offsets[i], P.feat_uoff[i], U_cap, P.pooled)
            ctx3.expand_inverse(F, B, P.pooled, P.feat_uoff[i], P.inverse[i], P.out)
        if P.need_backward:
            ctx3.backward_dedup(F, B, P.grad_out, P.inverse[i], P.feat_uoff[i], P.u_values[i], P.u_offsets[i],
                                P.rows, U_cap, M_cap, P.touched, P.feat_roff, P.grad_rows, tables=P.tables,
                                adagrad_state=P.state, lr=0.01, eps=1e-8)

    graphs = []
    with torch.cuda.stream(s3):
        for i in range(nb):
            step(i)                      # eager once: sizes the workspace before any capture
        torch.cuda.synchronize()
        for i in range(nb):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s3):
                step(i)
            graphs.append(g)
        for k in range(max(args.warmup, 2)):
            graphs[k % nb].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            graphs[k % nb].replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
    del graphs
    ctx3.close()
    return ms


KERNELS_OF_STEP = ("hash_insert", "emit", "lookup_expand", "expand_uncovered", "lookup_unique", "expand",
                   "grad_lists_sum", "grad_rows_sum")


def kernel_bytes(name, sh):
    """Algorithmic bytes per launch of one of the step's kernels (compulsory form: every distinct table
    row once) from the batch's sizes."""
    N, U, M, R, FB, D, e, o, cov, runs = (sh[k] for k in ("N", "U", "M", "R", "FB", "D", "e", "o", "covered", "runs"))
    look = M * 8 + (U + 1) * 8 + R * D * e + U * D * o
    return {
        # ids of every list (the predecessor compare re-reads them from cache), offsets, slot numbers,
        # one table slot written and read per run head (about U of them)
        "hash_insert": N * 8 + FB * (8 + 4) + U * 16,
        # rep + number read, inverse written, unique ids copied, the hash tables cleared (2 B slots a feature)
        "emit": FB * (4 + 4 + 4) + M * 16 + U * (4 + 8) + 2 * FB * 8,
        "lookup_unique": look,
        "expand": FB * 4 + U * D * o + FB * D * o,
        # lookup without the offsets (the run entries hold them) + run entries read, the first runs' output rows
        "lookup_expand": look - (U + 1) * 8 + runs * 24 + cov * D * o,
        # run entries read again, the later runs' rows copied from pooled
        "expand_uncovered": runs * 8 + (FB - cov) * D * o + min(FB - cov, U) * D * o,
        "kjt_lookup": N * 8 + (FB + 1) * 8 + R * D * e + FB * D * o,
        # every grad_out row once, sorted payload, segment starts, g_u written
        "grad_lists_sum": FB * D * 4 + FB * 4 + U * 8 + U * D * 4,
        # table row and accumulator read-modify-write, row id + feature + segment start per row,
        # payload per entry, every g_u row once
        "grad_rows_sum": R * (2 * D * 4 + 2 * 4 + 8 + 4 + 8) + M * 4 + U * D * 4,
    }[name]


def one_pass_forward(w, args):
    """Whether the step of workload w runs the forward pass as the one-pass call."""
    form = getattr(args, "forward", "auto")
    if form == "auto":
        return w.F * w.B <= 16384 or w.table_dtype != "f32"
    return form == "one-pass"


def run_workload(torch, recd, synth, w, args, need_backward, detail=True, pipeline=True, steps=None):
    P = DeviceProblem(torch, recd, synth, w, args.batches, need_backward, getattr(args, "store_grad", False), getattr(args, "tune", 0))
    P.planned = getattr(args, "planned", True)
    P.fused_forward = one_pass_forward(w, args)
    P.run_plan = getattr(args, "run_plan", False)
    nb = len(P.batches)
    F, B, D = w.F, w.B, w.D
    e = 4 if w.table_dtype == "f32" else 2
    o = e
    steps = steps or args.steps

    stats = []
    for i in range(nb):  # per-batch sizes (also warms the workspace)
        U, M = P.build(i, runs=True)
        P.forward(i, U)
        Rb = P.backward(i, U, M, want_count=True) if need_backward else None
        Rd, covered = P.ikjt_shape(i, U)
        assert Rb is None or Rb == Rd
        stats.append((U, M, Rd, covered, P.n_runs))
    for k in range(args.warmup):
        P.step(k % nb)
    # The timed region: K steps, wall clock around all of them (synchronised on both sides) and one
    # pair of HIP events around every step on the library's stream (= torch's current stream).
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        ev[k][0].record()
        P.step(k % nb)
        ev[k][1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    per_step = sorted(a.elapsed_time(b) for a, b in ev)
    step_ms = float(per_step[len(per_step) // 2])
    # ... and in the other form of the forward pass (event-timed median), for comparison; left out of
    # the run that is profiled kernel by kernel, whose kernels are those of one form only
    other_ms = None
    if detail:
        P.fused_forward = not P.fused_forward
        for k in range(max(args.warmup, 2)):
            P.step(k % nb)
        ev2 = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for k in range(steps):
            ev2[k][0].record()
            P.step(k % nb)
            ev2[k][1].record()
        torch.cuda.synchronize()
        other_ms = float(sorted(a.elapsed_time(b) for a, b in ev2)[steps // 2])
        P.fused_forward = not P.fused_forward
        for k in range(2):
            P.step(k % nb)
    # The same K steps once more with the library's own event pairs around the step's main kernels
    # (on the stream each is launched on): per-kernel launch times inside the running step, next to
    # whatever the side streams do meanwhile.  Kept out of the pass above: a pair of events per kernel
    # costs the stream a few microseconds per step.
    P.ctx.set_option(recd._OPT_INTERNAL_TIMING, 1)
    for name in recd.KERNEL_SLOTS:
        P.ctx.kernel_ms(name)   # reset
    for k in range(steps):
        P.step(k % nb)
    torch.cuda.synchronize()
    live = {}
    for name in KERNELS_OF_STEP:
        avg, med, n = P.ctx.kernel_ms(name)
        if n:
            live[name] = {"avg_ms": avg, "median_ms": med, "launches": n}
    P.ctx.set_option(recd._OPT_INTERNAL_TIMING, 0)

    res = {"step_ms": step_ms, "step_ms_wall_mean": wall_ms, "step_ms_event_mean": float(np.mean(per_step)),
           "forward": "one-pass" if P.fused_forward else "two-call",
           "step_ms_one_pass_forward": step_ms if P.fused_forward else other_ms,
           "step_ms_two_call_forward": other_ms if P.fused_forward else step_ms,
           "B": B, "F": F, "D": D}
    N = float(np.mean([b.N for b in P.batches]))
    U = float(np.mean([s[0] for s in stats]))
    M = float(np.mean([s[1] for s in stats]))
    R = float(np.mean([s[2] for s in stats]))
    covered = float(np.mean([s[3] for s in stats]))
    runs = float(np.mean([s[4] for s in stats]))
    shape = {"N": N, "U": U, "M": M, "R": R, "FB": float(F * B), "D": D, "e": e, "o": o, "covered": covered,
             "runs": runs}
    res.update({"N": N, "U": U, "M": M, "R": R, "runs": runs, "rows_in_first_runs": covered, "dedupe_factor": N / max(M, 1.0),
                "mean_session": float(np.mean([b.mean_session for b in P.batches]))})
    for name, k in live.items():
        by = kernel_bytes(name, shape)
        k.update({"algorithmic_bytes": by, "gbs": by / k["avg_ms"] / 1e6, "frac_of_peak": by / k["avg_ms"] / 1e6 / HBM_PEAK_GBS})
    res["kernels_in_timed_steps"] = live
    if not detail:
        return res, P
    if pipeline and getattr(args, "pipeline", False):
        res["pipelined_step_ms"] = pipelined_steps(torch, recd, P, args)
    if getattr(args, "graph", False):
        res["graph_step_ms"] = graph_steps(torch, recd, P, args, stats)

    reps = max(steps // nb, 3)
    # Per-call HIP-event timings on the library's stream (torch's current stream).  Each call is
    # issued for all batches back to back between one pair of events, behind a kernel that keeps
    # the GPU busy while the host marshals the first call, so the pair brackets GPU time only.
    # lookup, expand and kjt are one kernel launch per call; the one-pass call is two.
    cnt = [P.build(i, runs=True) for i in range(nb)]     # every batch's IKJT (and run index) is resident from here on

    def timed(fn):
        s_ev, e_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        P.expand(0)
        s_ev.record()
        for i in range(nb):
            fn(i)
        e_ev.record()
        torch.cuda.synchronize()
        return s_ev.elapsed_time(e_ev) / nb

    t = {k: [] for k in ("lookup", "expand", "fused", "kjt", "build", "build_runs", "bwd")}
    for _ in range(reps):
        t["lookup"].append(timed(lambda i: P.lookup(i, cnt[i][0])))
        t["expand"].append(timed(P.expand))
        t["fused"].append(timed(lambda i: P.fused(i, cnt[i][0])))
        t["kjt"].append(timed(P.kjt))
        t["build"].append(timed(lambda i: P.build(i, counts=False, runs=False)))
        t["build_runs"].append(timed(lambda i: P.build(i, counts=False, runs=True)))
        if need_backward:
            t["bwd"].append(timed(lambda i: P.backward(i, cnt[i][0], cnt[i][1])))
    if need_backward and getattr(args, "kjt_backward", True):
        # Comparison path of the backward: the same call on the KJT taken as an IKJT in which every row
        # is its own unique list (identity inverse): no deduplication, every id position sorted and summed.
        ident_inv = torch.arange(B, dtype=torch.int32, device="cuda").repeat(F)
        ident_uoff = torch.arange(F + 1, dtype=torch.int64, device="cuda") * B
        Nmax = max(b.N for b in P.batches)
        touched_kjt = torch.zeros(Nmax, dtype=torch.int64, device="cuda")
        P.ctx.set_option(recd.RECD_OPT_LONG_SEGMENT_CUT, 64)   # most of its work is in long rows

        def kjt_backward(i):
            P.ctx.backward_dedup(F, B, P.grad_out, ident_inv, ident_uoff, P.values[i], P.offsets[i], P.rows,
                                 F * B, P.batches[i].N, touched_kjt, P.feat_roff, None, tables=P.tables,
                                 adagrad_state=P.state, lr=0.01, eps=1e-8)

        kjt_backward(0)   # grows the workspace once, outside the timing
        kjt_bwd_t = [timed(kjt_backward) for _ in range(max(reps // 3, 2))]
        P.ctx.set_option(recd.RECD_OPT_LONG_SEGMENT_CUT, 32)
        res["kjt_backward_ms"] = float(np.mean(kjt_bwd_t))
        del touched_kjt, ident_inv
    ms = {k: float(np.mean(v)) for k, v in t.items() if v}
    build_ms, lookup_ms, expand_ms, fused_ms, kjt_ms = (ms[k] for k in ("build", "lookup", "expand", "fused", "kjt"))
    res.update({"build_ms": build_ms, "build_with_run_index_ms": ms["build_runs"], "lookup_unique_ms": lookup_ms, "expand_ms": expand_ms,
                "lookup_expand_one_pass_ms": fused_ms, "kjt_lookup_ms": kjt_ms})
    if need_backward:
        res["backward_ms"] = ms["bwd"]

    # algorithmic bytes per launch (upper: every gathered row counted; compulsory: each distinct
    # row once per launch)
    look_upper = M * 8 + (U + 1) * 8 + M * D * e + U * D * o
    look_comp = kernel_bytes("lookup_unique", shape)
    exp_bytes = kernel_bytes("expand", shape)
    fused_bytes = kernel_bytes("lookup_expand", shape) + kernel_bytes("expand_uncovered", shape)
    kjt_upper = N * 8 + (F * B + 1) * 8 + N * D * e + F * B * D * o
    kjt_comp = kernel_bytes("kjt_lookup", shape)
    res["bytes"] = {"lookup_unique_upper": look_upper, "lookup_unique_compulsory": look_comp, "expand": exp_bytes,
                    "lookup_expand_one_pass_compulsory": fused_bytes, "kjt_upper": kjt_upper,
                    "kjt_compulsory": kjt_comp}
    res["gbs"] = {
        "lookup_unique_upper": look_upper / lookup_ms / 1e6,
        "lookup_unique_compulsory": look_comp / lookup_ms / 1e6,
        "expand": exp_bytes / expand_ms / 1e6,
        # lookup + expand together (the region the 60 %-of-peak target is stated for), compulsory bytes:
        # as two kernels, and as the one-pass call (which never re-reads the pooled rows)
        "lookup_plus_expand_upper": (look_upper + exp_bytes) / (lookup_ms + expand_ms) / 1e6,
        "lookup_plus_expand_compulsory": (look_comp + exp_bytes) / (lookup_ms + expand_ms) / 1e6,
        "lookup_plus_expand_one_pass_compulsory": fused_bytes / fused_ms / 1e6,
        "kjt_upper": kjt_upper / kjt_ms / 1e6,
        "kjt_compulsory": kjt_comp / kjt_ms / 1e6,
    }
    res["frac_of_peak"] = {"lookup_plus_expand_compulsory": res["gbs"]["lookup_plus_expand_compulsory"] / HBM_PEAK_GBS,
                           "lookup_plus_expand_one_pass_compulsory":
                               res["gbs"]["lookup_plus_expand_one_pass_compulsory"] / HBM_PEAK_GBS}
    tr = [measured_traffic(w.name, k) for k in ("lookup_unique", "expand")]
    if all(x is not None for x in tr):
        res["bytes"]["lookup_plus_expand_traffic"] = sum(tr)
        res["gbs"]["lookup_plus_expand_traffic"] = sum(tr) / (lookup_ms + expand_ms) / 1e6
        # the same region with the HBM bytes the profiler measured for the two kernels (read from the
        # committed profile, see traffic_source) in the place of the algorithmic bytes
        res["frac_of_peak"]["lookup_plus_expand_traffic"] = res["gbs"]["lookup_plus_expand_traffic"] / HBM_PEAK_GBS
    if need_backward and "kjt_backward_ms" in res:
        res["backward_speedup_vs_kjt"] = res["kjt_backward_ms"] / res["backward_ms"]
    # Speedup of the deduplicated forward over the KJT lookup, and what the bytes predict for it:
    # bytes(KJT lookup) / bytes(lookup + expand), every gathered row counted on both sides ("upper":
    # the yardstick for ids without cache help), and with each distinct row counted once on both
    # sides ("compulsory": what is left when caches serve every repeated row).
    res["speedup_vs_kjt"] = kjt_ms / (lookup_ms + expand_ms)
    res["speedup_vs_kjt_one_pass"] = kjt_ms / fused_ms
    res["speedup_vs_kjt_with_build"] = kjt_ms / (build_ms + lookup_ms + expand_ms)
    res["predicted_speedup_bytes_model"] = kjt_upper / (look_upper + exp_bytes)
    res["predicted_speedup_compulsory_bytes"] = kjt_comp / (look_comp + exp_bytes)
    if getattr(args, "sequence", False):
        res["sequence"] = sequence_regions(torch, P, cnt, timed, reps, R)
    if getattr(args, "groups", 0) > 0:
        res["grouped"] = grouped_regions(torch, P, timed, reps, args.groups)
    if getattr(args, "partial", 0.0) > 0.0:
        res["partial"] = partial_regions(torch, synth, P, timed, reps, args.partial)
    if getattr(args, "weights", False):
        res["weighted"] = weighted_regions(torch, synth, P, timed, reps)
    return res, P


def weighted_regions(torch, synth, P, timed, reps):
    """Per-id weights: every id of the same batches carries a seeded fp32 weight (a function of id and
    position, so the duplication of the batch is kept).  Times the weighted builder, the weighted
    unique and KJT lookups and the weighted backward (fused update) beside their plain forms."""
    w = P.w
    F, B, D = w.F, w.B, w.D
    nb = len(P.batches)
    wts = [torch.from_numpy(synth.make_weights(b, i)).cuda() for i, b in enumerate(P.batches)]
    u_w = [torch.zeros(b.N, dtype=torch.float32, device="cuda") for b in P.batches]

    def build(i, counts=False):
        return P.ctx.build_ikjt_weighted(F, B, P.values[i], wts[i], P.offsets[i], P.u_values[i], u_w[i],
                                         P.u_offsets[i], P.inverse[i], P.feat_uoff[i], want_counts=counts)

    cnt = [build(i, True) for i in range(nb)]

    def lookup(i):
        P.ctx.pooled_lookup_unique_weighted(P.tables, P.u_values[i], u_w[i], P.u_offsets[i], P.feat_uoff[i],
                                            cnt[i][0], P.pooled)

    def kjt(i):
        P.ctx.kjt_pooled_lookup_weighted(P.tables, B, P.values[i], wts[i], P.offsets[i], P.kjt_out)

    def backward(i):
        P.ctx.backward_dedup_weighted(F, B, P.grad_out, P.inverse[i], P.feat_uoff[i], P.u_values[i], u_w[i],
                                      P.u_offsets[i], P.rows, cnt[i][0], cnt[i][1], P.touched, P.feat_roff,
                                      P.grad_rows, tables=P.tables, adagrad_state=P.state, lr=0.01, eps=1e-8)

    names = {"build": build, "lookup": lookup, "kjt": kjt}
    if P.need_backward:
        names["backward"] = backward
    t = {n: [] for n in names}
    for _ in range(max(reps // 2, 2)):
        for n, fn in names.items():
            t[n].append(timed(fn))
    ms = {n: float(np.mean(v)) for n, v in t.items()}
    out = {"build_weighted_ms": ms["build"], "lookup_unique_weighted_ms": ms["lookup"],
           "kjt_lookup_weighted_ms": ms["kjt"], "U": float(np.mean([c[0] for c in cnt])),
           "M": float(np.mean([c[1] for c in cnt]))}
    if P.need_backward:
        out["backward_weighted_ms"] = ms["backward"]
    cnt_plain = [P.build(i) for i in range(nb)]   # leave the plain IKJTs behind
    if P.need_backward:
        # the backward of the other pooling functions on the plain IKJTs (same batches, fused update)
        def bwd_mean(i):
            P.ctx.backward_dedup(F, B, P.grad_out, P.inverse[i], P.feat_uoff[i], P.u_values[i], P.u_offsets[i],
                                 P.rows, cnt_plain[i][0], cnt_plain[i][1], P.touched, P.feat_roff, P.grad_rows,
                                 tables=P.tables, adagrad_state=P.state, lr=0.01, eps=1e-8, mode="mean")

        def bwd_max(i):
            P.ctx.backward_dedup_max(F, B, P.grad_out, P.inverse[i], P.feat_uoff[i], P.u_values[i], P.u_offsets[i],
                                     P.rows, cnt_plain[i][0], cnt_plain[i][1], P.tables, P.touched, P.feat_roff,
                                     P.grad_rows, tables=P.tables, adagrad_state=P.state, lr=0.01, eps=1e-8)

        bwd_max(0)   # grows the workspace once, outside the timing
        tm = {"backward_mean_ms": [], "backward_max_ms": []}
        for _ in range(max(reps // 2, 2)):
            tm["backward_mean_ms"].append(timed(bwd_mean))
            tm["backward_max_ms"].append(timed(bwd_max))
        out.update({k: float(np.mean(v)) for k, v in tm.items()})
    return out


def partial_regions(torch, synth, P, timed, reps, shift):
    """Partial IKJTs on batches whose lists slide within a session: the partial builder and the pooled
    lookup on its windows beside the IKJT builder and lookup on the same batches."""
    import dataclasses
    w = dataclasses.replace(P.w, shift=shift)
    F, B, D = w.F, w.B, w.D
    nb = min(len(P.batches), 2)
    batches = [synth.make_batch(w, i) for i in range(nb)]
    values = [torch.from_numpy(b.values).cuda() for b in batches]
    offsets = [torch.from_numpy(b.offsets).cuda() for b in batches]
    i64 = dict(dtype=torch.int64, device="cuda")
    Nmax = max(b.N for b in batches)
    pv = [torch.zeros(b.N, **i64) for b in batches]
    ws = [torch.zeros(F * B, **i64) for _ in batches]
    wl = [torch.zeros(F * B, **i64) for _ in batches]
    inv = torch.zeros(F * B, dtype=torch.int32, device="cuda")
    fu = [torch.zeros(F + 1, **i64) for _ in batches]
    fp = torch.zeros(F + 1, **i64)
    uv = [torch.zeros(b.N, **i64) for b in batches]
    uo = [torch.zeros(F * B + 1, **i64) for _ in batches]
    fu2 = [torch.zeros(F + 1, **i64) for _ in batches]

    def build_p(i, counts=False):
        return P.ctx.build_partial_ikjt(F, B, values[i], offsets[i], pv[i], ws[i], wl[i], inv, fu[i], fp,
                                        None, want_counts=counts)

    def build_i(i, counts=False):
        return P.ctx.build_ikjt(F, B, values[i], offsets[i], uv[i], uo[i], inv, fu2[i], want_counts=counts)

    cp = [build_p(i, True) for i in range(nb)]
    ci = [build_i(i, True) for i in range(nb)]

    def look_p(i):
        P.ctx.pooled_lookup_partial(P.tables, pv[i], ws[i], wl[i], fu[i], cp[i][0], P.pooled)

    def look_i(i):
        P.ctx.pooled_lookup_unique(P.tables, uv[i], uo[i], fu2[i], ci[i][0], P.pooled)

    def timed_n(fn):   # as `timed`, over this region's batches
        s_ev, e_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        P.expand(0)
        s_ev.record()
        for i in range(nb):
            fn(i)
        e_ev.record()
        torch.cuda.synchronize()
        return s_ev.elapsed_time(e_ev) / nb

    t = {n: [] for n in ("build_p", "build_i", "look_p", "look_i")}
    for _ in range(max(reps // 2, 2)):
        t["build_p"].append(timed_n(build_p))
        t["build_i"].append(timed_n(build_i))
        t["look_p"].append(timed_n(look_p))
        t["look_i"].append(timed_n(look_i))
    ms = {n: float(np.mean(v)) for n, v in t.items()}
    for i in range(len(P.batches)):
        P.build(i)
    N = float(np.mean([b.N for b in batches]))
    Pn = float(np.mean([c[1] for c in cp]))
    M = float(np.mean([c[2] for c in cp]))
    return {"shift_probability": shift, "N": N, "U": float(np.mean([c[0] for c in cp])), "M_ikjt": M,
            "P_partial": Pn, "extra_values_removed_fraction_of_N": (M - Pn) / N,
            "dedupe_factor_ikjt": N / M, "dedupe_factor_partial": N / Pn,
            "build_partial_ms": ms["build_p"], "build_ikjt_ms": ms["build_i"],
            "lookup_partial_ms": ms["look_p"], "lookup_ikjt_ms": ms["look_i"]}


def grouped_regions(torch, P, timed, reps, k):
    """Grouped IKJTs: features in groups of k share one inverse.  Times the grouped builder, the
    element-wise sum over a group's features on the unique rows and the single expand per group;
    beside them the same sum on the expanded [F,B,D] rows (the module run without deduplication)."""
    w = P.w
    F, B, D = w.F, w.B, w.D
    groups = list(range(0, F, k)) + [F]
    G = len(groups) - 1
    nb = len(P.batches)
    inv_g = [torch.zeros(G * B, dtype=torch.int32, device="cuda") for _ in range(nb)]
    g_uoff = [torch.zeros(G + 1, dtype=torch.int64, device="cuda") for _ in range(nb)]
    inv_f = torch.zeros(F * B, dtype=torch.int32, device="cuda")
    comb = torch.zeros(G * B, D, dtype=P.tdt, device="cuda")
    gout = torch.zeros(G, B, D, dtype=P.tdt, device="cuda")
    ident_f = torch.arange(F + 1, dtype=torch.int64, device="cuda") * B
    ident_g = torch.arange(G + 1, dtype=torch.int64, device="cuda") * B

    def build(i, counts=False):
        return P.ctx.build_ikjt_grouped(F, B, groups, P.values[i], P.offsets[i], P.u_values[i], P.u_offsets[i],
                                        inv_g[i], g_uoff[i], P.feat_uoff[i], inv_f, want_counts=counts)

    cnt = [build(i, True) for i in range(nb)]  # the per-batch IKJTs are now the grouped ones

    def lookup(i):
        P.ctx.pooled_lookup_unique(P.tables, P.u_values[i], P.u_offsets[i], P.feat_uoff[i], cnt[i][0], P.pooled)

    def gsum(i):
        P.ctx.group_sum_unique(F, groups, P.pooled, P.feat_uoff[i], g_uoff[i], comb)

    def gexpand(i):
        P.ctx.expand_inverse(G, B, comb, g_uoff[i], inv_g[i], gout)

    def kjt_sum(i):  # the same module on the expanded rows: every "slot" is a sample
        P.ctx.group_sum_unique(F, groups, P.out.view(F * B, D), ident_f, ident_g, comb)

    t = {n: [] for n in ("build", "lookup", "gsum", "gexpand", "kjt_sum")}
    for _ in range(max(reps // 2, 2)):
        t["build"].append(timed(build))
        t["lookup"].append(timed(lookup))
        t["gsum"].append(timed(gsum))
        t["gexpand"].append(timed(gexpand))
        t["kjt_sum"].append(timed(kjt_sum))
    ms = {n: float(np.mean(v)) for n, v in t.items()}
    for i in range(nb):   # leave the ungrouped IKJTs behind, as the other regions expect them
        P.build(i)
    return {"features_per_group": k, "G": G, "build_grouped_ms": ms["build"],
            "lookup_unique_ms": ms["lookup"], "group_sum_unique_ms": ms["gsum"],
            "expand_groups_ms": ms["gexpand"], "group_sum_on_kjt_rows_ms": ms["kjt_sum"],
            "U_lists": float(np.mean([c[0] for c in cnt])), "M": float(np.mean([c[1] for c in cnt])),
            "U_groups": float(np.mean([c[2] for c in cnt])),
            "module_speedup": ms["kjt_sum"] / (ms["gsum"] + ms["gexpand"])}


def sequence_regions(torch, P, cnt, timed, reps, R):
    """Unpooled path on the resident IKJTs: one activation row per id.  Every call is one copy
    kernel; bytes are ids read + rows read + rows written (compulsory form: each distinct source
    row once per launch)."""
    w = P.w
    F, B, D = w.F, w.B, w.D
    e = 4 if w.table_dtype == "f32" else 2
    Nmax = max(b.N for b in P.batches)
    Mmax = max(c[1] for c in cnt)
    emb = torch.empty(Mmax, D, dtype=P.tdt, device="cuda")
    out = torch.empty(Nmax, D, dtype=P.tdt, device="cuda")

    def seq(i):
        P.ctx.sequence_lookup_unique(P.tables, P.u_values[i], P.u_offsets[i], P.feat_uoff[i], cnt[i][0], emb)

    def jag(i):
        P.ctx.jagged_expand_inverse(F, B, emb, P.u_offsets[i], P.feat_uoff[i], P.inverse[i], P.offsets[i],
                                    out[:P.batches[i].N])

    def kjt(i):
        P.ctx.kjt_sequence_lookup(P.tables, B, P.values[i], P.offsets[i], out[:P.batches[i].N])

    for i in range(len(P.batches)):
        seq(i), jag(i), kjt(i)
    t = {"seq": [], "jag": [], "kjt": [], "bwd": []}
    for _ in range(max(reps // 2, 2)):
        t["seq"].append(timed(seq))
        t["jag"].append(timed(jag))
        t["kjt"].append(timed(kjt))
    seq_ms, jag_ms, kjt_ms = (float(np.mean(t[k])) for k in ("seq", "jag", "kjt"))
    bwd_ms = None
    if P.need_backward:
        # backward of the sequence path: the KJT-shaped buffer now plays the upstream gradient
        grad_emb = emb if emb.dtype == torch.float32 else torch.empty(Mmax, D, dtype=torch.float32, device="cuda")
        gout = out if out.dtype == torch.float32 else None
        if gout is not None:
            gout.normal_(0.0, 0.01)

            def bwd(i):
                P.ctx.backward_sequence_dedup(F, B, gout[:P.batches[i].N], P.offsets[i], P.inverse[i],
                                              P.feat_uoff[i], P.u_values[i], P.u_offsets[i], P.rows, cnt[i][0],
                                              cnt[i][1], grad_emb, P.touched, P.feat_roff, None, tables=P.tables,
                                              adagrad_state=P.state, lr=0.01, eps=1e-8)

            for i in range(len(P.batches)):
                bwd(i)
            for _ in range(max(reps // 2, 2)):
                t["bwd"].append(timed(bwd))
            bwd_ms = float(np.mean(t["bwd"]))
    N = float(np.mean([b.N for b in P.batches]))
    U = float(np.mean([c[0] for c in cnt]))
    M = float(np.mean([c[1] for c in cnt]))
    rd = M if R is None else R
    by = {"sequence_lookup_unique": M * 8 + rd * D * e + M * D * e,
          "jagged_expand": F * B * (4 + 8) + U * 8 + M * D * e + N * D * e,
          "kjt_sequence": N * 8 + rd * D * e + N * D * e}
    ms = {"sequence_lookup_unique": seq_ms, "jagged_expand": jag_ms, "kjt_sequence": kjt_ms}
    if bwd_ms is not None:
        Rr = M if R is None else R
        by["backward_sequence"] = N * D * 4 + F * B * (4 + 8) + M * D * 4 * 2 + Rr * (2 * D * 4 + 8)
        ms["backward_sequence"] = bwd_ms
    return {"sequence_lookup_unique_ms": seq_ms, "jagged_expand_ms": jag_ms, "kjt_sequence_ms": kjt_ms,
            "backward_sequence_ms": bwd_ms,
            "bytes": by, "gbs": {k: by[k] / ms[k] / 1e6 for k in by},
            "activation_bytes_unique": M * D * e, "activation_bytes_kjt": N * D * e,
            "speedup_vs_kjt": kjt_ms / (seq_ms + jag_ms)}


def cpu_baseline(torch, synth, P, n_feat):
    """The CPU oracle, as it stands, single thread, on the first n_feat features (features are
    independent) of every rotated batch: build + unique lookup + expand (+ backward + Adagrad)."""
    from oracle import recd_oracle as orc
    w = P.w
    n_feat = min(n_feat, w.F)
    B = w.B
    dt = w.table_dtype
    tabs = []
    for f in range(n_feat):
        t = P.tables[f]
        tabs.append(t.view(torch.int16).cpu().numpy().view(np.uint16) if dt == "bf16" else t.cpu().numpy())
    gout = P.grad_out[:n_feat].cpu().numpy() if P.need_backward else None

    def one_batch(b):
        hi = int(b.offsets[n_feat * B])
        values, offsets = b.values[:hi], b.offsets[:n_feat * B + 1]
        t0 = time.perf_counter()
        uv, uo, inv, fu = orc.build_ikjt(n_feat, B, values, offsets)
        pooled = orc.pooled_lookup(tabs, dt, uv, uo, fu)
        orc.expand_inverse(n_feat, B, pooled, fu, inv)
        if gout is not None:
            tr, fr, gr = orc.backward_dedup(n_feat, B, gout, inv, fu, uv, uo)
            for f in range(n_feat):
                rows_f = tr[fr[f]:fr[f + 1]]
                orc.rowwise_adagrad(gr[fr[f]:fr[f + 1]], tabs[f][rows_f].astype(np.float64),
                                    np.zeros(len(rows_f)), 0.01, 1e-8)
        return time.perf_counter() - t0

    # the rotated batches in turn until about 10 s of CPU work are timed (every batch at least
    # once, unless that alone passes 20 s)
    total_s, n_done = 0.0, 0
    while total_s < 20.0 and (total_s < 10.0 or n_done < len(P.batches)):
        total_s += one_batch(P.batches[n_done % len(P.batches)])
        n_done += 1
    return {"value": B * n_feat * n_done / total_s, "unit": "pooled lookups/s", "cores": 1,
            "kind": "oracle", "seconds": total_s,
            "sample": f"features 0..{n_feat - 1} ({n_feat} of {w.F}), {n_done} batch passes over the "
                      f"{len(P.batches)} rotated batches, all B={B} rows: "
                      f"build + unique lookup + expand" + (" + backward + Adagrad" if gout is not None else "")}


def reader_regions(P, build_ms, max_seconds=20.0):
    """The KJT -> IKJT conversion alone: the GPU builder's time per batch beside the CPU oracle's
    builder, one thread per group of features (features are independent; the oracle's C code runs
    outside the interpreter lock), on as many features of batch 0 as fit the time bound."""
    import concurrent.futures as cf
    from oracle import recd_oracle as orc
    w, b = P.w, P.batches[0]
    B = w.B
    cores = min(os.cpu_count() or 1, 16)

    def one(f):
        lo, hi = int(b.offsets[f * B]), int(b.offsets[(f + 1) * B])
        orc.build_ikjt(1, B, b.values[lo:hi], b.offsets[f * B:(f + 1) * B + 1] - lo)

    t0 = time.perf_counter()
    one(0)
    per_feature = time.perf_counter() - t0
    n_feat = int(min(w.F, max(cores, cores * (max_seconds / max(per_feature, 1e-6)) // 1)))
    t0 = time.perf_counter()
    with cf.ThreadPoolExecutor(max_workers=cores) as ex:
        list(ex.map(one, range(n_feat)))
    cpu_s = time.perf_counter() - t0
    gpu_lists_s = B * w.F / (build_ms * 1e-3)
    cpu_lists_s = B * n_feat / cpu_s
    return {"gpu_build_ms": build_ms, "gpu_lists_per_s": gpu_lists_s, "gpu_ids_per_s": b.N / (build_ms * 1e-3),
            "cpu_oracle_lists_per_s": cpu_lists_s, "cpu_threads": cores,
            "cpu_sample": f"oracle builder on features 0..{n_feat - 1} of batch 0, {cores} threads",
            "gpu_over_cpu": gpu_lists_s / cpu_lists_s}


def cpu_baseline_parallel(torch, P, max_seconds=20.0):
    """The same oracle work feature-parallel: one task per feature of batch 0 (features are
    independent; the oracle's C code runs outside the interpreter lock) on the host's cores."""
    import concurrent.futures as cf
    from oracle import recd_oracle as orc
    w, b = P.w, P.batches[0]
    B, dt = w.B, w.table_dtype
    cores = min(os.cpu_count() or 1, 16)
    gout = P.grad_out.cpu().numpy() if P.need_backward else None

    tabs = [t.view(torch.int16).cpu().numpy().view(np.uint16) if dt == "bf16" else t.cpu().numpy()
            for t in P.tables]

    def one(f):
        tab = tabs[f]
        lo, hi = int(b.offsets[f * B]), int(b.offsets[(f + 1) * B])
        values, offsets = b.values[lo:hi], b.offsets[f * B:(f + 1) * B + 1] - lo
        t0 = time.perf_counter()
        uv, uo, inv, fu = orc.build_ikjt(1, B, values, offsets)
        pooled = orc.pooled_lookup([tab], dt, uv, uo, fu)
        orc.expand_inverse(1, B, pooled, fu, inv)
        if gout is not None:
            tr, fr, gr = orc.backward_dedup(1, B, gout[f:f + 1], inv, fu, uv, uo)
            orc.rowwise_adagrad(gr, tab[tr].astype(np.float64), np.zeros(len(tr)), 0.01, 1e-8)
        return time.perf_counter() - t0

    per = one(0)
    n_feat = int(min(w.F, max(cores, cores * (max_seconds / max(per, 1e-6)) // 1)))
    t0 = time.perf_counter()
    with cf.ThreadPoolExecutor(max_workers=cores) as ex:
        list(ex.map(one, range(n_feat)))
    wall = time.perf_counter() - t0
    return {"value": B * n_feat / wall, "unit": "pooled lookups/s", "cores": cores, "kind": "oracle",
            "seconds": wall, "sample": f"features 0..{n_feat - 1} of batch 0, one task per feature on {cores} threads"}


def traffic_file(workload_name):
    return os.path.join("profiles", f"hbm_traffic_{workload_name}.md")


def measured_traffic(workload_name, kernel="lookup_expand"):
    """HBM bytes per launch of one kernel from the committed rocprofv3 --pmc summary of this workload
    (FETCH_SIZE and WRITE_SIZE, calibrated against a plain copy); None if there is none.  The figure is
    read from the file, not measured in this run (`traffic_source` names the file)."""
    try:
        for line in open(os.path.join(ROOT, traffic_file(workload_name))):
            if line.startswith(f"{kernel}_traffic_bytes:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def summary_of(r):
    """The figures of one forward-only configuration that the targets are judged on."""
    keys = ("step_ms", "step_ms_wall_mean", "forward", "step_ms_one_pass_forward", "step_ms_two_call_forward", "N", "U", "M", "R", "dedupe_factor", "mean_session", "build_ms",
            "build_with_run_index_ms", "lookup_unique_ms", "expand_ms", "lookup_expand_one_pass_ms", "kjt_lookup_ms", "speedup_vs_kjt",
            "speedup_vs_kjt_one_pass", "speedup_vs_kjt_with_build", "predicted_speedup_bytes_model",
            "predicted_speedup_compulsory_bytes")
    out = {k: r[k] for k in keys}
    out["lookup_plus_expand_gbs_compulsory"] = r["gbs"]["lookup_plus_expand_compulsory"]
    out["lookup_plus_expand_frac_of_peak"] = r["frac_of_peak"]["lookup_plus_expand_compulsory"]
    out["lookup_plus_expand_one_pass_gbs_compulsory"] = r["gbs"]["lookup_plus_expand_one_pass_compulsory"]
    out["lookup_plus_expand_one_pass_frac_of_peak"] = r["frac_of_peak"]["lookup_plus_expand_one_pass_compulsory"]
    out["kjt_gbs_upper"] = r["gbs"]["kjt_upper"]
    return out


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2211_05239_amd import recd, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    if args.calib_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        b = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        for _ in range(3):
            a.copy_(b)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()

    name = args.workload
    if name.startswith("cfg4_S"):
        w = synth.sweep_workload(int(name[6:]))
    else:
        w = synth.WORKLOADS[name]
    need_backward = not args.forward_only
    res, P = run_workload(torch, recd, synth, w, args, need_backward, detail=not args.steps_only)

    value = w.B * w.F / (res["step_ms"] * 1e-3)
    # the kernel that takes the most time in the timed steps, by the library's own event pairs
    live = res["kernels_in_timed_steps"]
    dom = max(live, key=lambda k: live[k]["avg_ms"])
    fused = one_pass_forward(w, args)
    with_runs = fused or (args.run_plan and args.planned and need_backward)
    forward = ("build_ikjt_runs" if with_runs else "build_ikjt") + (
        " + pooled_lookup_expand (one pass)" if fused else " + pooled_lookup_unique + expand_inverse")
    line = {
        "metric": "deduped pooled lookups/sec",
        "value": value,
        "unit": "pooled lookups/s",
        "samples_per_s": w.B / (res["step_ms"] * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["step_ms"],
        "ms_per_step_timing": "median of the HIP-event-timed steps",
        "ms_per_step_wall_mean": res["step_ms_wall_mean"],
        "value_from_wall_mean": w.B * w.F / (res["step_ms_wall_mean"] * 1e-3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.table_dtype == "f32" else f"{w.table_dtype} tables, f32 accumulation",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B}, F={w.F}, mean session {w.S}, rows={w.rows}, D={w.D}, "
                               f"{w.table_dtype} tables; step = {forward}"
                               + (((" + backward_plan_runs / backward_apply" if args.run_plan else " + backward_plan / backward_apply")
                                    if getattr(args, "planned", True)
                                    else " + backward_dedup") + " with fused row-wise Adagrad"
                                  + ("" if args.store_grad else " (gradient rows consumed in registers, not stored)")
                                  if need_backward else " (forward only)"),
                   "batches_rotated": len(P.batches)},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": live[dom]["gbs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": live[dom]["frac_of_peak"],
                     "traffic": measured_traffic(w.name, dom),
                     "traffic_source": traffic_file(w.name) if measured_traffic(w.name, dom) is not None else None,
                     "algorithmic_bytes": live[dom]["algorithmic_bytes"],
                     "bytes_form": "compulsory (each distinct table row once per launch)",
                     "avg_launch_ms": live[dom]["avg_ms"],
                     "timing": "HIP event pairs around every launch of the kernel inside the timed steps, on the "
                               "stream it is launched on",
                     "kernels": {k: dict(v, traffic=measured_traffic(w.name, k)) for k, v in live.items()}},
        "regions": res,
    }
    if "pipelined_step_ms" in res:
        line["pipelined"] = {"ms_per_step": res["pipelined_step_ms"],
                             "value": w.B * w.F / (res["pipelined_step_ms"] * 1e-3), "unit": "pooled lookups/s",
                             "note": "same K steps, builder of the next batch on a second stream; not `value`"}
    if "graph_step_ms" in res:
        line["graph"] = {"ms_per_step": res["graph_step_ms"],
                         "value": w.B * w.F / (res["graph_step_ms"] * 1e-3), "unit": "pooled lookups/s",
                         "note": "same K steps replayed from captured HIP graphs, later calls sized by host upper "
                                 "bounds of U and M; not `value`"}
    if args.steps_only:
        P.ctx.close()
        print(json.dumps(line))
        return
    if args.cpu_features > 0:
        line["cpu_baseline"] = cpu_baseline(torch, synth, P, args.cpu_features)
        line["cpu_baseline_parallel"] = cpu_baseline_parallel(torch, P)
    if args.reader:
        line["regions"]["reader"] = reader_regions(P, res["build_ms"])
    P.ctx.close()
    del P
    torch.cuda.empty_cache()

    short = max(min(args.steps, 16), 4)
    if args.others:
        others = {}
        for cfg in ("cfg1", "cfg2", "cfg3"):
            if cfg == w.name:
                continue
            r, Po = run_workload(torch, recd, synth, synth.WORKLOADS[cfg], args, need_backward=False, steps=short)
            Po.ctx.close()
            del Po
            others[cfg] = summary_of(r)
        line["other_configs"] = others
    if args.sweep:
        sweep = []
        for S in synth.SWEEP_SESSION_SIZES:
            ws = synth.sweep_workload(S)
            r, Ps = run_workload(torch, recd, synth, ws, args, need_backward=False, steps=short)
            Ps.ctx.close()
            del Ps
            sweep.append(dict(summary_of(r), S=S))
        line["duplication_sweep"] = sweep
    print(json.dumps(line))


if __name__ == "__main__":
    main()
