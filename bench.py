#!/usr/bin/env python3
"""Benchmark of the rehearsal-buffer hot path on one MI355X.

A step is one update of the buffer with a mini-batch plus one sampling of r
representatives into the augmented mini-batch, on synthetic input that is
already resident in HBM.  The headline drives it through the single-call
primitive rb_update_sample (one kernel launch per step where eligible); the
same step issued as rb_update + rb_sample_augment (two launches) is reported
beside it.  Prints ONE JSON line: augmented samples/s of the whole job, the HBM
roofline of the dominant kernel, and the CPU oracle timed on the host.

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
# HBM bytes per launch of the dominant kernel as counted by two
# `rocprofv3 --pmc` runs (FETCH_SIZE, WRITE_SIZE), each scaled by the reading of a plain copy of
# known size; the text summaries with the exact commands are kept under profiles/.
# rb_window_kernel: a launch of 8 steps at C4 (algorithmic 616.56 MB; candidates that lose their slot within a launch,
# and representatives taken from a mini-batch row still in cache, are not moved) and of 16 steps at C3 (308.28 MB).
MEASURED_TRAFFIC = {("C4-1000x300-bf16-3x224x224-zipf", "rb_window_kernel"): 605764878,
                    ("C3-1000x130-f32-3x224x224", "rb_window_kernel"): 308354440,
                    ("C4-1000x300-bf16-3x224x224-zipf", "rb_step_planned_kernel"): 77116977,
                    ("C4-1000x300-bf16-3x224x224-zipf", "rb_step_small_kernel"): 77312701,
                    ("C5-10000x1000-f32-2048-active50", "rb_step_big_kernel"): 34009498}      # algorithmic 33.55 MB


MANY = 64           # steps handed to one rb_update_sample_many call


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
        self.P = pool_slots or min(1024, max(16, -(-POOL_BYTES // aug_bytes)))
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
        # of up to MANY consecutive steps is contiguous (the pool has at least 16 slots: the steps that share a
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
                    rb.rb_announce_next_many(h, min(16, nxt), C.cast(C.byref(self.ptrs[1], o_next), C.POINTER(C.c_void_p)))
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

    def timed(self, n, **kw):
        """ms per step over n steps enqueued back to back, HIP events on the side stream."""
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(self.stream)
        self.enqueue(n, **kw)
        e1.record(self.stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

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
    pipe.close()
    del big
    return {"standin": kind, "standin_ms": round(t_alone, 4), "buffer_ms": round(t_rb, 4), "overlapped_ms": round(t_both, 4),
            "overhead_frac": round((t_both - t_alone) / t_alone, 4)}


def cpu_baseline(w, wl, budget_s=12.0, max_steps=4000):
    """The CPU oracle on the same workload from an empty buffer, host batches cycled from a small pool."""
    from oracle import rbo
    import numpy as np
    pool = []
    for i in range(3):
        x, y = wl.make_batch(w, i)
        pool.append((wl.as_row_bytes(x), y.numpy()))
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    out = np.zeros((w.r, w.row_bytes), dtype=np.uint8)
    t0 = time.perf_counter()
    steps = 0
    while steps < max_steps:
        x, y = pool[steps % len(pool)]
        orc.update(x, y, w.c, w.lib_seed, steps)
        orc.sample_augment(w.r, w.lib_seed, steps, out_x=out)
        steps += 1
        if steps % 10 == 0 and time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    orc.close()
    return {"value": round((w.b + w.r) * steps / dt, 1), "unit": "augmented samples/s", "cores": 1, "kind": "oracle",
            "sample": f"first {steps} steps of {w.name} from an empty buffer, {dt:.1f} s, host batches cycled from a pool of {len(pool)}",
            "ms_per_step": round(dt / steps * 1e3, 4),
            "gb_per_s": round(w.bytes_per_step() * steps / dt / 1e9, 3)}


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
    rig.enqueue(MANY, many=MANY, ahead=True)
    torch.cuda.synchronize()
    # Headline: K steps enqueued back to back on the side stream through rb_update_sample_many, MANY steps per
    # host call, the labels of the next call's first steps announced before every call.  The mini-batches
    # of all those steps are resident (like every input); when the step is eligible, up to 16 steps share one
    # launch whose plan the launch before made (also across calls: that is what the announcement is for).
    ms = rig.timed(steps, many=min(MANY, steps), ahead=True)     # exactly `steps` steps: the last call takes what is left
    n_side = min(steps, 1000)
    ms_many_plain = rig.timed(n_side // MANY * MANY or MANY, many=MANY)    # the same without announcing the next call
    # ... and with calls of exactly one launch each (what a loader that prefetches 8 or 16 mini-batches can feed)
    per_launch = rig.buf.steps_per_launch(w.b, w.c, w.r)
    ms_launch_calls = None
    if per_launch > 1:
        rig.enqueue(per_launch, many=per_launch, ahead=True)
        ms_launch_calls = rig.timed(n_side // per_launch * per_launch, many=per_launch, ahead=True)
    ms_ahead = rig.timed(n_side, single_call=True, ahead=fused)   # one rb_update_sample per step, next labels announced
    ms_plain = rig.timed(n_side, single_call=True)                # ... not announced
    ms_two = rig.timed(n_side)
    rig.buf.set_option(rb.RB_OPT_WINDOW, 1)
    ms_many1 = rig.timed(n_side // MANY * MANY or MANY, many=MANY)   # rb_update_sample_many held to one launch per step
    rig.buf.set_option(rb.RB_OPT_WINDOW, 16)
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
        "launches_per_step": len(launch_sizes(rig, MANY)) / MANY if windowed else (1 if fused else 2),
        "steps_per_launch": max(launch_sizes(rig, MANY)) if windowed else 1,
        "steps_per_launch_schedule": launch_sizes(rig, MANY) if windowed else None,
        "next_call_not_announced_ms_per_step": ms_many_plain, "one_launch_per_call_announced_ms_per_step": ms_launch_calls,
        "steps_per_host_call": MANY,
        "one_launch_per_step_ms": ms_ahead, "one_launch_per_step_gb_per_s": w.bytes_per_step() / (ms_ahead * 1e-3) / 1e9,
        "next_labels_announced": fused, "plan_ahead_kernel": None if not fused else ("rb_step_planned_kernel" if small else "rb_step_big_kernel"),
        "not_announced_ms_per_step": ms_plain, "not_announced_gb_per_s": w.bytes_per_step() / (ms_plain * 1e-3) / 1e9,
        "two_call_ms_per_step": ms_two, "two_call_gb_per_s": w.bytes_per_step() / (ms_two * 1e-3) / 1e9,
        "many_call_one_launch_per_step_ms": ms_many1,
        "update_kernel_ms": ms_update, "sample_kernel_ms": ms_sample,
        "stored_samples": int(fill.sum()), "last_n": int(last_n), "prefilled": bool(prefill),
    }
    return rig, res


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


def variants_leg(w, torch, rb, wl, steps):
    """The policy variants of Algorithm 1 on the same workload.  The other replacement strategies go through the
    same announced multi-step calls as the headline (several steps per launch); the Bernoulli selection has no
    bound on its number of candidates and always takes the general kernels (two launches per step)."""
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
    ap.add_argument("--others", default="C3,C5,C2,C1", help="comma list of further workloads reported inside the line ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true")
    ap.add_argument("--no-variants", action="store_true")
    ap.add_argument("--pmc-run", action="store_true",
                    help="short fixed sequence for `rocprofv3 --pmc`: 120 two-call steps, 120 single-call steps, 120 single-call steps with "
                         "the next labels announced, 192 steps through announced rb_update_sample_many calls, then 3 plain copies "
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
        rig.enqueue(192, many=64, ahead=True)
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
    pre = None
    if not a.prefill:
        rig.close()
        rig, pre = measure(w, torch, rb, wl, min(a.steps, 500), a.warmup, True)
        log(f"[bench] prefilled {json.dumps(pre)}")
    rig.close()

    others = {}
    for name in [s for s in a.others.split(",") if s]:
        ow = wl.by_name(name)
        orig, ores = measure(ow, torch, rb, wl, min(a.steps, ow.steps), a.warmup, False)
        if ow.name.startswith("C3") and not a.no_overlap:
            ores["overlap"] = {f"fma_{d}ms": overlap_leg(orig, 200, d) for d in (0.5, 2.0, 10.0)}
            ores["overlap"]["hbm_copy_0.3ms"] = overlap_leg(orig, 200, 0.3, kind="hbm")
        orig.close()
        others[ow.name] = {k: (round(v, 5) if isinstance(v, float) else v) for k, v in ores.items()}
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

    # Roofline of the dominant kernel.  With one or several whole steps per launch that kernel is the
    # step (rb_window_kernel / rb_step_planned_kernel: every inserted row and every representative row
    # read once and written once, plus the one workgroup that plans what comes next); otherwise it is
    # the gather of rb_sample_augment.
    n_rows = min(w.r, res["last_n"])
    if res["steps_per_launch"] > 1:
        # several steps per launch, every launch of a call of MANY steps the same size
        per = res["steps_per_launch"]
        assert MANY % per == 0
        kernel = "rb_window_kernel"
        k_ms, k_bytes = res["ms_per_step"] * per, 2 * (w.c + n_rows) * w.row_bytes * per
    elif res["launches_per_step"] == 1:
        # rb_update_sample_many announces every next step's labels for itself: one planned launch per step
        kernel, k_ms, k_bytes = res["plan_ahead_kernel"], res["ms_per_step"], 2 * (w.c + n_rows) * w.row_bytes
    else:
        kernel, k_ms, k_bytes = "rb_sample_kernel", res["sample_kernel_ms"], 2 * n_rows * w.row_bytes
    achieved = k_bytes / (k_ms * 1e-3) / 1e9
    line = {
        "metric": "augmented samples/sec and achieved HBM GB/s (% of peak) per update+sample step",
        "value": round(res["aug_samples_per_s"], 1), "unit": "augmented samples/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(res["ms_per_step"], 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": w.name, "classes": w.K, "slots_per_class": w.S, "sample_shape": list(w.shape),
                   "sample_dtype": w.dtype, "b": w.b, "c": w.c, "r": w.r, "prefilled": bool(a.prefill),
                   "api": f"rb_announce_next_many + rb_update_sample_many, {MANY} steps per call" +
                          (f", {res['steps_per_launch']} steps per launch (planned by the launch before)" if res["steps_per_launch"] > 1 else ""),
                   "stream": "side stream, inputs resident in HBM, pool rotation"},
        "gb_per_s": round(res["gb_per_s"], 1), "hbm_frac": round(res["hbm_frac"], 4),
        "reps_per_s": round(res["reps_per_s"], 1),
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_TRAFFIC.get((w.name, kernel)) if not a.prefill else None,
                     "bytes_per_launch": k_bytes, "kernel_ms": round(k_ms, 5),
                     "copy_ceiling_gbs": round(ceiling, 1)},
        "detail": {k: (round(v, 5) if isinstance(v, float) else v) for k, v in res.items()},
        "prefilled": None if pre is None else {k: (round(v, 5) if isinstance(v, float) else v) for k, v in pre.items()},
        "others": others,
        "policy_variants": variants,
        "host_pinned_rows": pinned,
        "bf16_stored_rows": reduced,
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, wl)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
