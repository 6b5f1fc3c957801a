#!/usr/bin/env python3
"""Benchmark of the rehearsal-buffer hot path on one MI355X.

A step is one update of the buffer with a mini-batch plus one sampling of r
representatives into the augmented mini-batch, on synthetic input that is
already resident in HBM.  The headline drives it through rb_update_sample_many
(with the next call announced), which puts several steps into one launch where
the shape allows; the same steps issued one launch per step, as the fused
single call and as rb_update + rb_sample_augment are reported beside it.
Every figure is the median of several timed regions of exactly --steps steps
each, enqueued back to back behind a pre-roll of the same calls (so that the
GPU never waits for the host), with HIP events on the side stream between them.
Prints ONE JSON line: augmented samples/s of the whole job, the HBM roofline
of the dominant kernel, and the CPU oracle timed on the host.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--prefill]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
POOL_BYTES = 2 << 30           # inputs/outputs rotate through at least this much memory (>> 256 MB of last-level cache)
# HBM bytes per STEP of the dominant kernel as counted by two `rocprofv3 --pmc` runs (FETCH_SIZE, WRITE_SIZE) of
# `bench.py --pmc-run`, each scaled by the reading of a plain copy of known size in the same run; the text summaries
# with the exact commands are the files named here.  Not measured by this run: the line says where it is from.
PROFILED_TRAFFIC = {
    ("C4-1000x300-bf16-3x224x224-zipf", "rb_window_kernel"): (75656761, "profiles/rb_window_kernel_C4_pmc_hbm_traffic.txt"),   # algorithmic 77070336: slot losers are not moved, forwarded rows hit the cache
    ("C3-1000x130-f32-3x224x224", "rb_window_kernel"): (19325318, "profiles/rb_window_kernel_C3_pmc_hbm_traffic.txt"),          # algorithmic 19267584
    ("C5-10000x1000-f32-2048-active50", "rb_bigwin_kernel"): (34013328, "profiles/rb_bigwin_kernel_C5_pmc_hbm_traffic.txt"),    # algorithmic 33554432
}

MANY = 64           # steps handed to one rb_update_sample_many call
REPEATS = 5         # timed regions per figure (the median is reported, with the smallest and the largest)
PREROLL = 64        # steps enqueued, untimed, right in front of the first timed region (the GPU works on them while the host queues the rest)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Rig:
    """Device-side state of one workload: the buffer, a side stream and a rotating pool of augmented batches."""

    def __init__(self, w, torch, rb, wl, pool_slots=None, storage="hbm", store_dtype=None):
        self.w, self.torch, self.rb = w, torch, rb
        self.dev = torch.device("cuda:0")
        self.stream = torch.cuda.Stream(self.dev)
        self.buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=self.dev, stream=self.stream,
                                      storage=storage, store_dtype=store_dtype)
        aug_bytes = (w.b + w.r) * w.row_bytes
        self.P = pool_slots or min(1024, max(32, -(-POOL_BYTES // aug_bytes)))
        self.aug_x = torch.empty((self.P, w.b + w.r, *w.shape), dtype=w.torch_dtype, device=self.dev)
        self.aug_y = torch.empty((self.P, w.b + w.r), dtype=torch.int64, device=self.dev)
        # distinct sample bytes for a few slots, replicated over the pool (generation is not what is measured);
        # labels are generated for every slot, they drive the plan.
        distinct = min(self.P, 4)
        for i in range(distinct):
            self.aug_x[i, :w.b].copy_(wl.make_samples(w, i, self.dev))
        for i in range(distinct, self.P):
            self.aug_x[i, :w.b].copy_(self.aug_x[i % distinct, :w.b])
        for i in range(self.P):
            self.aug_y[i, :w.b].copy_(wl.make_labels(w, i, self.dev))
        self.aug_x[:, w.b:].zero_()
        self.aug_y[:, w.b:].fill_(-1)
        torch.cuda.synchronize()
        rs = w.row_bytes
        self.args = []
        for i in range(self.P):
            bx, by = self.aug_x[i].data_ptr(), self.aug_y[i].data_ptr()
            self.args.append((bx, by, bx + w.b * rs, by + w.b * 8))
        # host arrays of the same pointers for rb_update_sample_many: the pool several times over, so that any run
        # of up to MANY consecutive steps is contiguous (the pool has at least 32 slots: the steps that share a
        # launch never share a slot)
        self.ptrs = [rb.pointer_array([a[i] for a in self.args] * (2 + MANY // self.P)) for i in range(4)]
        self.step = 0

    def prefill(self):
        """Fill every slot: updates with c = b and round-robin labels until F = K*S."""
        w, torch = self.w, self.torch
        h = self.buf.handle
        y = torch.empty(w.b, dtype=torch.int64, device=self.dev)
        total = w.K * w.S
        done = 0
        with torch.cuda.stream(self.stream):
            while done < total + w.b:
                y.copy_((torch.arange(w.b, device=self.dev) + done) % w.K)
                rc = self.rb.rb_update(h, self.args[0][0], y, w.b, w.b, 12345, 1 << 40 | done)
                assert rc == 0, rc
                done += w.b
        self.stream.synchronize()
        fill, _, _ = self.buf.read_state()
        assert int(fill.sum()) == total, (int(fill.sum()), total)

    def enqueue(self, n, do_update=True, do_sample=True, single_call=False, many=0, ahead=False):
        """Enqueue n consecutive steps on the side stream (no synchronisation).
        many: hand the steps to rb_update_sample_many, `many` of them per call.
        ahead: announce the labels that come next before every call (plan-ahead forms): the next pool slot's
        with single_call, those of the next call's first steps (up to 16) with many."""
        w, rb, h, P, args = self.w, self.rb, self.buf.handle, self.P, self.args
        upd, smp, both = rb.rb_update, rb.rb_sample_augment, rb.rb_update_sample
        b, c, r, seed = w.b, w.c, w.r, w.lib_seed
        t = self.step
        if many:
            assert many <= MANY
            import ctypes as C
            for at in range(0, n, many):
                k = min(many, n - at)
                o = (t % P) * C.sizeof(C.c_void_p)
                px, py, ox, oy = (C.cast(C.byref(a, o), C.POINTER(C.c_void_p)) for a in self.ptrs)
                if ahead:
                    o_next = ((t + k) % P) * C.sizeof(C.c_void_p)
                    nxt = min(many, n - (at + k)) or many           # steps of the call that follows (the next enqueue's first, at the end)
                    rb.rb_announce_next_many(h, min(32, nxt), C.cast(C.byref(self.ptrs[1], o_next), C.POINTER(C.c_void_p)))
                rc = rb.rb_update_sample_many(h, k, px, py, b, c, r, seed, t, ox, oy)
                if rc:
                    raise RuntimeError(f"rb_update_sample_many -> {rc}")
                t += k
            self.step = t
            return
        for _ in range(n):
            bx, by, ox, oy = args[t % P]
            if single_call:
                if ahead:
                    rb.rb_announce_next(h, args[(t + 1) % P][1])
                rc = both(h, bx, by, b, c, r, seed, t, ox, oy)
                if rc:
                    raise RuntimeError(f"rb_update_sample -> {rc}")
                t += 1
                continue
            if do_update:
                rc = upd(h, bx, by, b, c, seed, t)
                if rc:
                    raise RuntimeError(f"rb_update -> {rc}")
            if do_sample:
                rc = smp(h, r, seed, t, ox, oy)
                if rc:
                    raise RuntimeError(f"rb_sample_augment -> {rc}")
            t += 1
        self.step = t

    def timed_regions(self, n, repeats=REPEATS, **kw):
        """ms per step of `repeats` regions of exactly n steps each.  Everything is enqueued back to back on the
        side stream, behind a pre-roll of the same calls that keeps the GPU busy while the host queues the timed
        launches (so the regions hold no time in which the GPU waits for the host, as in a training loop whose data
        pipeline runs ahead); HIP events on that stream mark the regions, the device is drained only at the end."""
        torch = self.torch
        per = kw.get("many") or 1
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(repeats + 1)]
        torch.cuda.synchronize()
        self.enqueue(-(-PREROLL // per) * per, **kw)
        ev[0].record(self.stream)
        for i in range(repeats):
            self.enqueue(n, **kw)
            ev[i + 1].record(self.stream)
        torch.cuda.synchronize()
        return [ev[i].elapsed_time(ev[i + 1]) / n for i in range(repeats)]

    def timed(self, n, repeats=3, **kw):
        """Median ms per step over `repeats` regions of n steps (see timed_regions)."""
        ms = sorted(self.timed_regions(n, repeats, **kw))
        return ms[len(ms) // 2]

    def close(self):
        self.buf.close()
        del self.aug_x, self.aug_y, self.buf
        self.torch.cuda.empty_cache()


def copy_ceiling(torch, rb, nbytes=1 << 30, reps=20):
    """GB/s (read + write) of a plain large device copy with the mover's inner loop: the best of 1 to 8 vectors per
    thread, plain / streaming with paced stores / streaming with burst stores."""
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    src.fill_(1)
    best = 0.0
    for unroll in (1, 2, 4, 8):
        for nt in (0, 1, 2):
            for _ in range(3):
                rb.rb_copy_bytes(None, dst, src, nbytes, unroll, nt)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                rb.rb_copy_bytes(None, dst, src, nbytes, unroll, nt)
            e1.record()
            torch.cuda.synchronize()
            gbs = 2 * nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
            best = max(best, gbs)
    del src, dst
    torch.cuda.empty_cache()
    return best


def overlap_leg(rig, steps, target_ms, kind="fma"):
    """Steps of the asynchronous pipeline of Sec. IV-D: buffer work on the side stream under a stand-in
    for the training computation on the main stream (kind "fma": register-only multiply-add loop on all
    compute units; kind "hbm": a large streaming copy, the worst case for a bandwidth-bound path).
    Returns ms per iteration: stand-in alone, buffer alone, both overlapped."""
    torch, rb, w = rig.torch, rig.rb, rig.w
    main = torch.cuda.current_stream(rig.dev)
    blocks = 256 * 8
    sink = torch.empty(blocks * 256, dtype=torch.float32, device=rig.dev)
    big = None
    if kind == "hbm":
        big = torch.empty((2, 1 << 30), dtype=torch.uint8, device=rig.dev)
        big.fill_(3)

    def standin(amount):
        if kind == "fma":
            rb.rb_standin_compute(None, sink, blocks, amount)
        else:
            rb.rb_copy_bytes(None, big[1], big[0], amount, 2, 1)

    def standin_ms(amount, n=5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(main)
        for _ in range(n):
            standin(amount)
        e1.record(main)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    probe = 20000 if kind == "fma" else (256 << 20)
    standin_ms(probe)
    amount = max(1, int(probe * target_ms / standin_ms(probe)))
    if kind == "hbm":
        amount = min(1 << 30, max(1 << 20, amount // 4096 * 4096))
    t_alone = standin_ms(amount, steps)
    t_rb = rig.timed(steps, single_call=True)
    pipe = rb.Pipeline(rig.buf)
    h, P, args = pipe.handle, rig.P, rig.args
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(main)
    for _ in range(steps):
        t = rig.step
        bx, by = args[t % P][:2]
        nx, ny = args[(t + 1) % P][2:]                 # tail of the next augmented mini-batch
        # (1) wait for the representatives sampled during the previous iteration; (2) update with this
        # mini-batch, then sample the next representatives, on the buffer's stream
        rc, _ = rb.rb_pipeline_step(h, bx, by, w.b, w.c, w.r, w.lib_seed, t, nx, ny, main)
        if rc:
            raise RuntimeError(f"rb_pipeline_step -> {rc}")
        rig.step = t + 1
        standin(amount)                                # (3), (4) forward and backward pass stand-in
    pipe.drain(main)
    e1.record(main)
    torch.cuda.synchronize()
    t_both = e0.elapsed_time(e1) / steps
    # The same loop with a data pipeline that is a whole launch ahead: one rb_pipeline_step_many call per `group`
    # iterations (the group's launch runs under the first iteration's stand-in, the other iterations follow
    # rb_pipeline_drain), every call announced to the one before.
    import ctypes as C
    group = rig.buf.steps_per_launch(w.b, w.c, w.r)
    t_rb_many = t_both_many = None
    if group > 1:
        n_groups = max(2, steps // group)
        t_rb_many = rig.timed(n_groups * group, many=group, ahead=True)
        torch.cuda.synchronize()
        e0.record(main)
        for _ in range(n_groups):
            t = rig.step
            o, o_next = (t % P) * C.sizeof(C.c_void_p), ((t + group) % P) * C.sizeof(C.c_void_p)
            px, py, ox, oy = (C.cast(C.byref(a, o), C.POINTER(C.c_void_p)) for a in rig.ptrs)
            rb.rb_announce_next_many(rig.buf.handle, group, C.cast(C.byref(rig.ptrs[1], o_next), C.POINTER(C.c_void_p)))
            rc, _ = rb.rb_pipeline_step_many(h, group, px, py, w.b, w.c, w.r, w.lib_seed, t, ox, oy, main)
            if rc:
                raise RuntimeError(f"rb_pipeline_step_many -> {rc}")
            rig.step = t + group
            standin(amount)                            # iteration t: overlaps the group's launch
            pipe.drain(main)
            for _ in range(group - 1):
                standin(amount)                        # the group's other iterations
        e1.record(main)
        torch.cuda.synchronize()
        t_both_many = e0.elapsed_time(e1) / (n_groups * group)
    pipe.close()
    del big
    out = {"standin": kind, "standin_ms": round(t_alone, 4), "buffer_ms": round(t_rb, 4), "overlapped_ms": round(t_both, 4),
           "overhead_frac": round((t_both - t_alone) / t_alone, 4)}
    if group > 1:
        out.update({"iterations_per_call": group, "many_buffer_ms": round(t_rb_many, 5), "many_overlapped_ms": round(t_both_many, 4),
                    "many_overhead_frac": round((t_both_many - t_alone) / t_alone, 4)})
    return out


def cpu_baseline(w, wl, budget_s=12.0, max_steps=4000, threads=0, pool=None):
    """The CPU oracle as it stands on the same workload from an empty buffer, host batches cycled from a pool
    larger than the host's last-level cache.  threads > 0: the oracle's timing variant, policy sequential, the row
    copies of every call spread over that many host threads."""
    from oracle import rbo
    import numpy as np
    if pool is None:
        pool = cpu_pool(w, wl)
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    workers = rbo.Pool(threads) if threads else None
    out = np.zeros((w.r, w.row_bytes), dtype=np.uint8)
    t0 = time.perf_counter()
    steps = 0
    while steps < max_steps:
        x, y = pool[steps % len(pool)]
        if workers:
            orc.update_mt(workers, x, y, w.c, w.lib_seed, steps)
            orc.sample_augment_mt(workers, w.r, w.lib_seed, steps, out_x=out)
        else:
            orc.update(x, y, w.c, w.lib_seed, steps)
            orc.sample_augment(w.r, w.lib_seed, steps, out_x=out)
        steps += 1
        if steps % 10 == 0 and time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    orc.close()
    if workers:
        workers.close()
    pool_mb = sum(x.nbytes for x, _ in pool) / 1e6
    return {"value": round((w.b + w.r) * steps / dt, 1), "unit": "augmented samples/s", "cores": threads or 1, "kind": "oracle",
            "sample": f"first {steps} steps of {w.name} from an empty buffer, {dt:.1f} s, host batches cycled from a pool of "
                      f"{len(pool)} ({pool_mb:.0f} MB); rows are allocated on first write" +
                      (f"; policy sequential, row copies of each call spread over {threads} threads" if threads else ""),
            "ms_per_step": round(dt / steps * 1e3, 4),
            "gb_per_s": round(w.bytes_per_step() * steps / dt / 1e9, 3)}


def cpu_pool(w, wl, min_bytes=1 << 30, max_batches=12):
    """Host mini-batches for the CPU baseline: at least min_bytes of them (more than a last-level cache)."""
    n = max(3, min(max_batches, -(-min_bytes // (w.b * w.row_bytes))))
    pool = []
    for i in range(n):
        x, y = wl.make_batch(w, i)
        pool.append((wl.as_row_bytes(x), y.numpy()))
    return pool


def call_sizes(n, per_call):
    """Steps per rb_update_sample_many call of a region of n steps."""
    return [min(per_call, n - at) for at in range(0, n, per_call)]


def spread(ms):
    """median, smallest and largest of a list of timings"""
    o = sorted(ms)
    return o[len(o) // 2], o[0], o[-1]


def headline(rig, steps, warmup=0):
    """The headline figure on one rig: REPEATS regions of exactly `steps` steps through announced
    rb_update_sample_many calls of at most MANY steps.  Returns a dict with the median, the spread, the launches
    of one region and the rows that were really moved per step (counted by the kernels, read outside the regions)."""
    w = rig.w
    per_call = min(MANY, steps)
    if warmup:
        rig.enqueue(warmup, many=min(MANY, warmup), ahead=True)
    rows0, steps0 = rig.buf.moved_rows(), rig.step          # (synchronises; outside the timed regions)
    ms_all = rig.timed_regions(steps, REPEATS, many=per_call, ahead=True)
    rows1, steps1 = rig.buf.moved_rows(), rig.step
    ms, lo, hi = spread(ms_all)
    launches = [k for n in call_sizes(steps, per_call) for k in launch_sizes(rig, n)]
    moved_per_step = (rows1 - rows0) / (steps1 - steps0)
    return {"ms_per_step": ms, "ms_per_step_min": lo, "ms_per_step_max": hi, "regions": REPEATS, "ms_per_step_regions": ms_all,
            "steps_per_call": call_sizes(steps, per_call) if steps <= 4 * MANY else f"{steps // per_call} x {per_call} + {steps % per_call}",
            "launch_steps": launches if len(launches) <= 16 else f"{len(launches)} launches, {max(launches)} steps at most",
            "n_launches": len(launches), "rows_moved_per_step": moved_per_step,
            "gb_per_s_actual": 2 * moved_per_step * w.row_bytes / (ms * 1e-3) / 1e9}


def measure(w, torch, rb, wl, steps, warmup, prefill):
    rig = Rig(w, torch, rb, wl)
    if prefill:
        rig.prefill()
    # One launch per step is possible for at most 64 candidates and representatives and at most 1024 classes;
    # the labels of the next mini-batch are then announced before every call (they are resident, like every
    # input), so that each launch also plans the following step and only moves rows itself.
    # Larger counts (up to 1024 candidates and representatives, 10240 classes) have a plan-ahead form of their
    # own: one launch per step that moves rows by the plan a 1024-thread workgroup of the launch before made.
    small = 1 <= w.c <= 64 and 1 <= w.r <= 64 and w.K <= 1024
    fused = small or (1 <= w.c <= 1024 and 1 <= w.r <= 1024 and w.b <= 4096 and w.K <= 10240)
    windowed = rig.buf.steps_per_launch(w.b, w.c, w.r) > 1
    rig.enqueue(warmup, single_call=True, ahead=fused)
    # Headline: exactly `steps` steps per timed region through rb_update_sample_many, at most MANY steps per host
    # call, the labels of the next call's first steps announced before every call.  The mini-batches of all those
    # steps are resident (like every input); when the step is eligible, up to 16 steps share one launch whose plan
    # the launch before made (also across calls: that is what the announcement is for).
    head = headline(rig, steps)
    ms = head["ms_per_step"]
    n_side = min(max(steps, 256), 1000)
    ms_many_plain = rig.timed(n_side // MANY * MANY or MANY, many=MANY)    # the same without announcing the next call
    # ... and with calls of exactly one launch each (what a loader that prefetches 8 or 16 mini-batches can feed)
    per_launch = rig.buf.steps_per_launch(w.b, w.c, w.r)
    ms_launch_calls = None
    if per_launch > 1:
        ms_launch_calls = rig.timed(n_side // per_launch * per_launch, many=per_launch, ahead=True)
    ms_ahead = rig.timed(n_side, single_call=True, ahead=fused)   # one rb_update_sample per step, next labels announced
    ms_plain = rig.timed(n_side, single_call=True)                # ... not announced
    ms_two = rig.timed(n_side)
    rig.buf.set_option(rb.RB_OPT_WINDOW, 1)
    ms_many1 = rig.timed(n_side // MANY * MANY or MANY, many=MANY)   # rb_update_sample_many held to one launch per step
    rig.buf.set_option(rb.RB_OPT_WINDOW, 32)
    # One kernel alone, launched back to back on the same stream with HIP events around the whole
    # loop: launches pipeline, so the time per launch is that kernel's duration plus the dispatch
    # gap (an event pair around every single launch would add several microseconds to each).
    ms_update = rig.timed(n_side, do_sample=False)
    ms_sample = rig.timed(n_side, do_update=False)
    fill, last_n, flags = rig.buf.read_state()
    res = {
        "workload": w.name, "ms_per_step": ms, "aug_samples_per_s": (w.b + w.r) / (ms * 1e-3),
        "reps_per_s": w.r / (ms * 1e-3), "gb_per_s": w.bytes_per_step() / (ms * 1e-3) / 1e9,
        "hbm_frac": w.bytes_per_step() / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "headline": head,
        "launches_per_step": head["n_launches"] / steps if windowed else (1 if fused else 2),
        "steps_per_launch": per_launch if windowed else 1,
        "next_call_not_announced_ms_per_step": ms_many_plain, "one_launch_per_call_announced_ms_per_step": ms_launch_calls,
        "one_launch_per_step_ms": ms_ahead, "one_launch_per_step_gb_per_s": w.bytes_per_step() / (ms_ahead * 1e-3) / 1e9,
        "next_labels_announced": fused, "plan_ahead_kernel": None if not fused else ("rb_step_planned_kernel" if small else "rb_step_big_kernel"),
        "not_announced_ms_per_step": ms_plain, "not_announced_gb_per_s": w.bytes_per_step() / (ms_plain * 1e-3) / 1e9,
        "two_call_ms_per_step": ms_two, "two_call_gb_per_s": w.bytes_per_step() / (ms_two * 1e-3) / 1e9,
        "many_call_one_launch_per_step_ms": ms_many1,
        "update_kernel_ms": ms_update, "sample_kernel_ms": ms_sample,
        "side_legs_steps_per_region": n_side,
        "stored_samples": int(fill.sum()), "last_n": int(last_n), "prefilled": bool(prefill),
    }
    return rig, res


def rows_per_call_sweep(rig, counts=(8, 16, 32, 64)):
    """The same rig with c = r = 8 ... 64 rows per step (announced rb_update_sample_many calls, steps per launch as
    the library chooses): how the achieved rate approaches the plain-copy ceiling as a launch carries more rows."""
    import dataclasses
    w0 = rig.w
    out = []
    for k in counts:
        if k > w0.b or k > w0.r:          # the pool's augmented mini-batches have room for w0.r representatives
            continue
        rig.w = dataclasses.replace(w0, c=k, r=k)
        per = rig.buf.steps_per_launch(w0.b, k, k)
        n = max(MANY, 512 // MANY * MANY)
        ms = rig.timed(n, many=MANY, ahead=True)
        out.append({"c": k, "r": k, "rows_per_step": 2 * k, "steps_per_launch": per, "rows_per_launch": 2 * k * per,
                    "mb_per_launch": round(2 * 2 * k * per * w0.row_bytes / 1e6, 2), "ms_per_step": round(ms, 5),
                    "gb_per_s": round(2 * 2 * k * w0.row_bytes / (ms * 1e-3) / 1e9, 1),
                    "hbm_frac": round(2 * 2 * k * w0.row_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
    rig.w = w0
    return out


def launch_sizes(rig, n):
    """Steps per launch of one rb_update_sample_many call of n steps in a stream of calls that are announced to each
    other: the library's limit for the shape, and a remainder."""
    w = rig.w
    per = rig.buf.steps_per_launch(w.b, w.c, w.r)
    return [min(per, n - at) for at in range(0, n, per)]


def host_pinned_leg(torch, rb, wl, steps=200):
    """Where the paper keeps its buffers (Sec. IV-C): sample rows in pinned host memory, moved by the same
    kernels over the host link.  Workload C3 with 4 slots per class (2.4 GB of pinned rows)."""
    w = wl.variant(wl.C3, name="C3-rows-in-pinned-host-memory-S4", S=4)
    rig = Rig(w, torch, rb, wl, storage="host_pinned")
    rig.enqueue(50, single_call=True)
    torch.cuda.synchronize()
    ms = rig.timed(steps, single_call=True)
    rig.close()
    return {"workload": w.name, "ms_per_step": round(ms, 5), "aug_samples_per_s": round((w.b + w.r) / (ms * 1e-3), 1),
            "host_link_gb_per_s": round((w.c + w.r) * w.row_bytes / (ms * 1e-3) / 1e9, 2)}


def reduced_precision_leg(torch, rb, wl, steps=1000):
    """Data reduction of the stored samples (Sec. VII): workload C3 (float32 samples) with rows stored as
    bfloat16.  A candidate is read at 4 bytes and written at 2 bytes per element, a representative the other
    way round: 3/4 of the bytes of the plain workload, and half the buffer."""
    w = wl.C3
    rig = Rig(w, torch, rb, wl, store_dtype=torch.bfloat16)
    rig.enqueue(100, single_call=True, ahead=True)
    rig.enqueue(MANY, many=MANY, ahead=True)
    torch.cuda.synchronize()
    n = max(MANY, steps // MANY * MANY)
    ms = rig.timed(n, many=MANY, ahead=True)                  # 16 steps per launch, calls announced
    ms_ahead = rig.timed(steps, single_call=True, ahead=True)  # one launch per step, plan made one step ahead
    ms_plain = rig.timed(steps, single_call=True)             # general kernels, two launches per step
    moved = (w.c + w.r) * (w.row_bytes + w.row_bytes // 2)
    steps_per_launch = rig.buf.steps_per_launch(w.b, w.c, w.r)
    rig.close()
    return {"workload": w.name + " stored as bf16", "ms_per_step": round(ms, 5),
            "aug_samples_per_s": round((w.b + w.r) / (ms * 1e-3), 1), "bytes_per_step": moved,
            "gb_per_s": round(moved / (ms * 1e-3) / 1e9, 1), "hbm_frac": round(moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "buffer_gb": round(w.buffer_bytes / 2 / 1e9, 1), "steps_per_launch": steps_per_launch,
            "one_launch_per_step_ms": round(ms_ahead, 5), "not_announced_ms_per_step": round(ms_plain, 5)}


def eight_bit_leg(torch, rb, wl, steps=1000):
    """Workload C3 (float32 images with values in [0, 1)) with rows stored in 8 bits per element (Sec. VII): a quarter
    of the buffer, 5/8 of the bytes per step.  Several steps per launch through announced multi-step calls; a single
    step is served by the general kernels (two launches)."""
    w = wl.C3
    rig = Rig(w, torch, rb, wl, store_dtype=torch.uint8)
    rig.enqueue(100, single_call=True)
    rig.enqueue(MANY, many=MANY, ahead=True)
    torch.cuda.synchronize()
    n = max(MANY, steps // MANY * MANY)
    ms = rig.timed(n, many=MANY, ahead=True)
    ms_plain = rig.timed(steps, single_call=True)
    moved = (w.c + w.r) * (w.row_bytes + w.row_bytes // 4)
    steps_per_launch = rig.buf.steps_per_launch(w.b, w.c, w.r)
    rig.close()
    return {"workload": w.name + " stored as u8", "ms_per_step": round(ms, 5), "aug_samples_per_s": round((w.b + w.r) / (ms * 1e-3), 1),
            "bytes_per_step": moved, "gb_per_s": round(moved / (ms * 1e-3) / 1e9, 1),
            "hbm_frac": round(moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "buffer_gb": round(w.buffer_bytes / 4 / 1e9, 1),
            "steps_per_launch": steps_per_launch, "two_launches_per_step_ms": round(ms_plain, 5)}


def variants_leg(w, torch, rb, wl, steps):
    """The policy variants of Algorithm 1 on the same workload, all through the same announced multi-step calls as
    the headline: the other replacement strategies in the same several-steps launch, the Bernoulli selection (whose
    number of candidates is only bounded by b) in the several-steps launch for large counts."""
    out = {}
    names = {(1, 0): "bernoulli+uniform", (0, 1): "exact+fifo", (0, 2): "exact+reservoir", (1, 1): "bernoulli+fifo"}
    small = 1 <= w.c <= 64 and 1 <= w.r <= 64 and w.K <= 1024
    for (sel, ev), name in names.items():
        rig = Rig(w, torch, rb, wl)
        rig.buf.set_policy(sel, ev)
        rig.prefill()                       # every slot filled, so that every insertion exercises the eviction strategy
        # plan-ahead launches: exact selection with small counts, Bernoulli selection with b <= 1024
        planned = (small and sel == 0) or (sel == 1 and w.b <= 1024 and w.K <= 10240)
        per = rig.buf.steps_per_launch(w.b, w.c, w.r)            # several steps per launch (exact selection only)
        rig.enqueue(100, single_call=True, ahead=planned)
        if per > 1:
            rig.enqueue(MANY, many=MANY, ahead=True)
        torch.cuda.synchronize()
        if per > 1:
            ms = rig.timed(max(MANY, steps // MANY * MANY), many=MANY, ahead=True)
        else:
            ms = rig.timed(steps, single_call=True, ahead=planned)
        out[name] = {"ms_per_step": round(ms, 5), "aug_samples_per_s": round((w.b + w.r) / (ms * 1e-3), 1),
                     "gb_per_s_nominal": round(w.bytes_per_step() / (ms * 1e-3) / 1e9, 1), "prefilled": True,
                     "steps_per_launch": per, "launches_per_step": 1 / per if per > 1 else (1 if planned else 2)}
        if planned:
            out[name]["one_launch_per_step_ms"] = round(rig.timed(steps, single_call=True, ahead=True), 5)
            out[name]["not_announced_ms_per_step"] = round(rig.timed(steps, single_call=True), 5)
        rig.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--prefill", action="store_true", help="fill every slot before timing (all inserts replace)")
    ap.add_argument("--others", default="C3,C5,C5F,C2,C1", help="comma list of further workloads reported inside the line ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true")
    ap.add_argument("--no-variants", action="store_true")
    ap.add_argument("--pmc-run", action="store_true",
                    help="short fixed sequence for `rocprofv3 --pmc`: 120 two-call steps, 120 single-call steps, 120 single-call steps with "
                         "the next labels announced, 320 steps through announced rb_update_sample_many calls, then 3 plain copies "
                         "of 256 MiB whose known traffic calibrates the counters; prints no JSON line")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build covers one GPU's local buffer only (no collectives); run with --gpus 1")

    import torch
    import rb_workloads as wl
    import __graft_entry__
    __graft_entry__.ensure_built()          # compiles only when no library has been built yet
    import paper_2406_03285_amd as rb
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; there is no CPU path")

    w = wl.by_name(a.workload)
    if a.pmc_run:
        rig = Rig(w, torch, rb, wl)
        if a.prefill:
            rig.prefill()
        rig.enqueue(120)
        rig.enqueue(120, single_call=True)
        rig.enqueue(120, single_call=True, ahead=True)
        rig.enqueue(320, many=64, ahead=True)
        torch.cuda.synchronize()
        nbytes = 256 << 20
        src = torch.full((nbytes,), 7, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            rb.rb_copy_bytes(None, dst, src, nbytes, 4, 1)
        torch.cuda.synchronize()
        log(f"[bench] pmc run done: {w.name}, 120 steps, 3 copies of {nbytes} bytes")
        return
    log(f"[bench] {w.name}: buffer {w.buffer_bytes / 1e9:.1f} GB, {w.bytes_per_step() / 1e6:.2f} MB/step")
    ceiling = copy_ceiling(torch, rb)
    log(f"[bench] plain copy ceiling {ceiling:.0f} GB/s")
    rig, res = measure(w, torch, rb, wl, a.steps, a.warmup, a.prefill)
    log(f"[bench] {json.dumps(res)}")
    sweeps = {}
    if not a.no_variants:
        sweeps[w.name] = rows_per_call_sweep(rig)
        log(f"[bench] rows-per-call sweep {json.dumps(sweeps[w.name])}")
    rig.close()
    # The same headline on a second, fresh allocation of the buffer and the pool: the rate depends a little on the
    # physical placement the driver hands out, so two draws of it are shown.
    rig = Rig(w, torch, rb, wl)
    if a.prefill:
        rig.prefill()
    again = headline(rig, a.steps, warmup=max(a.warmup, MANY))
    log(f"[bench] second allocation {json.dumps(again)}")
    rig.close()
    pre = None
    if not a.prefill:
        rig, pre = measure(w, torch, rb, wl, min(a.steps, 500), a.warmup, True)
        log(f"[bench] prefilled {json.dumps(pre)}")
        rig.close()

    others = {}
    for name in [s for s in a.others.split(",") if s]:
        ow = wl.by_name(name)
        # (regions of at least 256 steps: with fewer, a region is one or two launches and mostly their start and end)
        orig, ores = measure(ow, torch, rb, wl, max(256, min(a.steps, ow.steps)), a.warmup, False)
        ores["steps_per_region"] = max(256, min(a.steps, ow.steps))
        if ow.name.startswith("C3") and not a.no_overlap:
            ores["overlap"] = {f"fma_{d}ms": overlap_leg(orig, 200, d) for d in (0.5, 2.0, 10.0)}
            ores["overlap"]["hbm_copy_0.3ms"] = overlap_leg(orig, 200, 0.3, kind="hbm")
        orig.close()
        if ow.name.startswith("C3") and not a.no_variants:
            # the sweep at this row size needs room for 64 representatives behind every pooled mini-batch
            srig = Rig(wl.variant(ow, r=64), torch, rb, wl)
            srig.enqueue(MANY, many=MANY, ahead=True)
            sweeps[ow.name] = rows_per_call_sweep(srig)
            srig.close()
            log(f"[bench] rows-per-call sweep {json.dumps(sweeps[ow.name])}")
        others[ow.name] = rounded(ores)
        log(f"[bench] {json.dumps(others[ow.name])}")

    variants = None if a.no_variants else variants_leg(w, torch, rb, wl, min(a.steps, 500))
    if variants:
        log(f"[bench] variants {json.dumps(variants)}")
    pinned = None if a.no_variants else host_pinned_leg(torch, rb, wl)
    if pinned:
        log(f"[bench] host-pinned {json.dumps(pinned)}")
    reduced = None if a.no_variants else reduced_precision_leg(torch, rb, wl)
    if reduced:
        log(f"[bench] reduced-precision {json.dumps(reduced)}")
    eight = None if a.no_variants else eight_bit_leg(torch, rb, wl)
    if eight:
        log(f"[bench] 8-bit storage {json.dumps(eight)}")

    # Roofline of the dominant kernel over the timed regions of the headline.  With one or several whole steps per
    # launch that kernel is the step (rb_window_kernel / rb_step_big_kernel: every inserted row and every
    # representative row read once and written once, plus the workgroups that plan what comes next), launched back
    # to back with nothing else in the stream: its average launch is a region's bytes and a region's time divided
    # by the launches of a region.  Otherwise it is the gather of rb_sample_augment, timed alone.
    n_rows = min(w.r, res["last_n"])
    head = res["headline"]
    if res["launches_per_step"] <= 1:
        small = 1 <= w.c <= 64 and 1 <= w.r <= 64 and w.K <= 1024
        kernel = ("rb_window_kernel" if small else "rb_bigwin_kernel") if res["steps_per_launch"] > 1 else res["plan_ahead_kernel"]
        launches = head["n_launches"]
        k_ms = res["ms_per_step"] * a.steps / launches
        k_bytes = 2 * (w.c + n_rows) * w.row_bytes * a.steps / launches
        steps_per_avg_launch = a.steps / launches
    else:
        kernel, k_ms, k_bytes, steps_per_avg_launch = "rb_sample_kernel", res["sample_kernel_ms"], 2 * n_rows * w.row_bytes, 1
    achieved = k_bytes / (k_ms * 1e-3) / 1e9
    profiled = PROFILED_TRAFFIC.get((w.name, kernel)) if not a.prefill else None
    calls = call_sizes(a.steps, min(MANY, a.steps))
    line = {
        "metric": "augmented samples/sec and achieved HBM GB/s (% of peak) per update+sample step",
        "value": round(res["aug_samples_per_s"], 1), "unit": "augmented samples/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(res["ms_per_step"], 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": w.name, "classes": w.K, "slots_per_class": w.S, "sample_shape": list(w.shape),
                   "sample_dtype": w.dtype, "b": w.b, "c": w.c, "r": w.r, "prefilled": bool(a.prefill),
                   "api": f"rb_announce_next_many + rb_update_sample_many, calls of {sorted(set(calls), reverse=True)} steps, launches of "
                          f"{sorted(set(launch_sizes_of(calls, res['steps_per_launch'])), reverse=True)} steps (each planned by the launch before)",
                   "timing": f"median of {REPEATS} regions of {a.steps} steps each, back to back behind {PREROLL} untimed steps of the same calls",
                   "stream": "side stream, inputs resident in HBM, pool rotation"},
        "gb_per_s": round(res["gb_per_s"], 1), "hbm_frac": round(res["hbm_frac"], 4),
        "gb_per_s_actual": round(head["gb_per_s_actual"], 1),
        "ms_per_step_min_max": [round(head["ms_per_step_min"], 5), round(head["ms_per_step_max"], 5)],
        "second_allocation": {"ms_per_step": round(again["ms_per_step"], 5),
                              "ms_per_step_min_max": [round(again["ms_per_step_min"], 5), round(again["ms_per_step_max"], 5)],
                              "hbm_frac": round(w.bytes_per_step() / (again["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "reps_per_s": round(res["reps_per_s"], 1),
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": None if profiled is None else round(profiled[0] * steps_per_avg_launch),
                     "traffic_source": None if profiled is None else f"{profiled[1]}: {profiled[0]} bytes per step, times the "
                                                                     f"{steps_per_avg_launch:.2f} steps of this run's average launch (not measured by this run)",
                     "bytes_per_launch": round(k_bytes), "kernel_ms": round(k_ms, 5),
                     "launches_per_region": head["n_launches"] if res["launches_per_step"] <= 1 else None,
                     "copy_ceiling_gbs": round(ceiling, 1)},
        "rows_per_call_sweep": sweeps or None,
        "detail": rounded(res),
        "prefilled": None if pre is None else rounded(pre),
        "others": others,
        "policy_variants": variants,
        "host_pinned_rows": pinned,
        "bf16_stored_rows": reduced,
        "u8_stored_rows": eight,
    }
    if not a.no_cpu_baseline:
        pool = cpu_pool(w, wl)
        line["cpu_baseline"] = cpu_baseline(w, wl, pool=pool)
        log(f"[bench] cpu {json.dumps(line['cpu_baseline'])}")
        line["cpu_baseline_mt"] = cpu_baseline(w, wl, pool=pool, threads=max(2, min(os.cpu_count() or 2, 16)))
        log(f"[bench] cpu mt {json.dumps(line['cpu_baseline_mt'])}")
    print(json.dumps(line), flush=True)


def launch_sizes_of(calls, per_launch):
    """Steps per launch of announced calls of these sizes: the library makes a call's launches as equal as it can."""
    out = []
    for n in calls:
        left = n
        while left > 0:
            launches = -(-left // per_launch)
            w = -(-left // launches)
            out.append(w)
            left -= w
    return out


def rounded(d):
    out = {}
    for k, v in d.items():
        if isinstance(v, float):
            v = round(v, 5)
        elif isinstance(v, dict):
            v = rounded(v)
        elif isinstance(v, list):
            v = [round(x, 5) if isinstance(x, float) else x for x in v]
        out[k] = v
    return out


if __name__ == "__main__":
    main()
