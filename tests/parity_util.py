"""Drive the HIP library and the CPU oracle side by side on the same seeded inputs
and compare everything observable, byte for byte."""
import numpy as np
import torch

import rb_workloads as wl
from oracle import rbo

SENTINEL = 0x5A


def _bytes(t):
    """uint8 view [rows, row_bytes] of a contiguous sample tensor (stays on its device)."""
    row_bytes = t.element_size()
    for d in t.shape[1:]:
        row_bytes *= d
    return t.view(torch.uint8).reshape(t.shape[0], row_bytes)


def compare_state(buf, orc, tag):
    fill, last_n, flags = buf.read_state()
    assert np.array_equal(fill, orc.fill), f"{tag}: per-class fill differs"
    assert flags == orc.flags, f"{tag}: flags {flags} != {orc.flags}"
    return fill


def compare_buffers(buf, orc, tag, chunk_bytes=256 << 20):
    """Labels of all slots, and sample bytes of every filled slot."""
    fill = compare_state(buf, orc, tag)
    gy = buf.buf_y.cpu().numpy()
    assert np.array_equal(gy, orc.buf_y), f"{tag}: buf_y differs"
    rows_per_chunk = max(1, chunk_bytes // buf.row_bytes)
    bx = buf.buf_x.view(buf.K * buf.S, -1).view(torch.uint8)      # [K*S, row_bytes] on the device
    pending, count = [], 0

    def flush():
        nonlocal pending, count
        if not pending:
            return
        host = np.concatenate([orc.export_rows(first, n) for first, n in pending])
        idx = torch.cat([torch.arange(first, first + n) for first, n in pending]).to(bx.device)
        want = torch.from_numpy(host).to(bx.device)   # bx is on the device, or in pinned host memory
        got = bx.index_select(0, idx)
        if not torch.equal(got, want):
            bad = (got != want).any(dim=1).nonzero().flatten()[:5].tolist()
            raise AssertionError(f"{tag}: stored rows differ at slots {[int(idx[i]) for i in bad]}")
        pending, count = [], 0

    for k in range(buf.K):
        f = int(fill[k])
        at = 0
        while at < f:
            n = min(f - at, rows_per_chunk - count)
            pending.append((k * buf.S + at, n))
            count += n
            at += n
            if count >= rows_per_chunk:
                flush()
    flush()


def run_parity(w, steps=None, device="cuda:0", stream=None, options=(), check_state_every=0,
               first_step=0, progress=None, buf=None, orc=None, final_check=True, single_call=False,
               policy=None, storage="hbm", store_bf16=False, store_u8=False):
    """Runs `steps` update+sample steps of workload `w` on both sides.

    single_call: drive the HIP side through rb_update_sample instead of the two calls.
    policy: (selection, eviction) variant codes, set on both sides (the codes are the same numbers).
    store_bf16 / store_u8: float32 samples stored as bfloat16 / in 8 bits per element on both sides.
    Every step: out_y equal, the n sampled rows byte-equal, rows >= n untouched.
    At the end (and every `check_state_every` steps): fill, flags, buf_y and all
    filled buf_x rows.  Returns (buf, orc) for further checks.
    """
    import paper_2406_03285_amd as rb

    steps = w.steps if steps is None else steps
    dev = torch.device(device)
    own = buf is None
    if own:
        buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev, stream=stream, storage=storage,
                                 store_dtype=_store_dtype(store_bf16, store_u8))
        orc = rbo.Buffer(w.K, w.S, w.row_bytes)
        _set_oracle_storage(orc, store_bf16, store_u8)
        for opt, val in options:
            buf.set_option(opt, val)
        if policy is not None:
            buf.set_policy(*policy)
            orc.set_policy(*policy)
    aug_x = torch.empty((w.b + w.r, *w.shape), dtype=w.torch_dtype, device=dev)
    aug_y = torch.empty(w.b + w.r, dtype=torch.int64, device=dev)
    for step in range(first_step, first_step + steps):
        x, y = wl.make_batch(w, step, dev)
        aug_x[:w.b].copy_(x)
        aug_y[:w.b].copy_(y)
        _bytes(aug_x[w.b:]).fill_(SENTINEL)
        aug_y[w.b:].fill_(-7)
        if stream is not None:
            stream.wait_stream(torch.cuda.current_stream(dev))
        if single_call:
            buf.update_sample(aug_x[:w.b], aug_y[:w.b], w.c, w.r, w.lib_seed, step, aug_x[w.b:], aug_y[w.b:])
        else:
            buf.update(aug_x[:w.b], aug_y[:w.b], w.c, w.lib_seed, step)
            buf.sample_augment(w.r, w.lib_seed, step, aug_x[w.b:], aug_y[w.b:])
        if stream is not None:
            torch.cuda.current_stream(dev).wait_stream(stream)
        # oracle on the host copies of the very same bytes
        hx = _bytes(aug_x[:w.b]).cpu().numpy()
        hy = aug_y[:w.b].cpu().numpy()
        orc.update(hx, hy, w.c, w.lib_seed, step)
        ref_x = np.full((w.r, w.row_bytes), SENTINEL, dtype=np.uint8)
        n, ref_x, ref_y = orc.sample_augment(w.r, w.lib_seed, step, out_x=ref_x)
        got_y = aug_y[w.b:].cpu().numpy()
        tag = f"{w.name} step {step}"
        assert np.array_equal(got_y, ref_y), f"{tag}: out_y differs\n gpu {got_y[:16]}\n ref {ref_y[:16]}"
        got_x = _bytes(aug_x[w.b:]).cpu().numpy()
        if not np.array_equal(got_x, ref_x):
            bad = np.nonzero((got_x != ref_x).any(axis=1))[0]
            raise AssertionError(f"{tag}: out_x rows {bad[:8].tolist()} differ (n={n})")
        if check_state_every and (step + 1) % check_state_every == 0:
            compare_buffers(buf, orc, tag)
            _, last_n, _ = buf.read_state()
            assert last_n == n
        if progress and (step + 1) % progress == 0:
            print(f"  {tag} ok", flush=True)
    if final_check:
        compare_buffers(buf, orc, f"{w.name} final")
    return buf, orc


def _store_dtype(store_bf16, store_u8):
    return torch.bfloat16 if store_bf16 else torch.uint8 if store_u8 else None


def _set_oracle_storage(orc, store_bf16, store_u8):
    if store_bf16:
        orc.set_storage(rbo.STORE_BF16)
    elif store_u8:
        orc.set_storage(rbo.STORE_U8)


def run_ahead_parity(w, steps, schedule_seed=None, store_bf16=False, policy=None, options=(), store_u8=False):
    """update_sample with the next mini-batch's labels announced; with a schedule seed, promises are
    broken at random (other labels, other arguments, other calls in between) and the plan must be
    dropped without a trace."""
    import paper_2406_03285_amd as rb

    dev = torch.device("cuda:0")
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev, store_dtype=_store_dtype(store_bf16, store_u8))
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    _set_oracle_storage(orc, store_bf16, store_u8)
    if policy is not None:
        buf.set_policy(*policy)
        orc.set_policy(*policy)
    for opt, val in options:
        buf.set_option(opt, val)

    def batch(t):
        x, y = wl.make_batch(w, t, dev)
        return x.contiguous(), y.contiguous()

    nxt = batch(0)
    out_x = torch.empty((w.r, *w.shape), dtype=w.torch_dtype, device=dev)
    out_y = torch.empty(w.r, dtype=torch.int64, device=dev)
    rng = np.random.default_rng(schedule_seed)
    for t in range(steps):
        (x, y), nxt = nxt, batch(t + 1)         # the next mini-batch is there before this step is enqueued
        c, r = w.c, w.r
        _bytes(out_x).fill_(SENTINEL)
        out_y.fill_(-7)
        what = "keep" if schedule_seed is None else rng.choice(["keep", "keep", "keep", "other-labels", "other-c", "two-calls",
                                                                "read-state", "no-announce"])
        if what != "no-announce":
            buf.announce_next(nxt[1])
        if what == "other-labels":              # the step that comes is not the one that was announced
            y = y.clone()
        if what == "other-c":
            c = max(1, w.c - 1)
        if what == "read-state":
            assert np.array_equal(buf.read_state()[0], orc.fill)
        if what == "two-calls":
            buf.update(x, y, c, w.lib_seed, t)
            buf.sample_augment(r, w.lib_seed, t, out_x, out_y)
        else:
            buf.update_sample(x, y, c, r, w.lib_seed, t, out_x, out_y)
        orc.update(_bytes(x).cpu().numpy(), y.cpu().numpy(), c, w.lib_seed, t)
        ref = np.full((r, w.row_bytes), SENTINEL, dtype=np.uint8)
        n, ref_x, ref_y = orc.sample_augment(r, w.lib_seed, t, out_x=ref)
        tag = f"{w.name} step {t} ({what})"
        assert np.array_equal(out_y.cpu().numpy(), ref_y), f"{tag}: out_y differs"
        assert np.array_equal(_bytes(out_x).cpu().numpy(), ref_x), f"{tag}: out_x differs (n={n})"
        if (t + 1) % max(1, steps // 3) == 0:
            compare_buffers(buf, orc, tag)
            assert buf.read_state()[1] == n
    compare_buffers(buf, orc, f"{w.name} final")
    assert buf.read_state()[2] == orc.flags


def run_many_parity(w, steps, per_call=24, window=None, announce=False, schedule_seed=None, store_bf16=False, policy=None,
                    options=(), store_u8=False, planners=None):
    """rb_update_sample_many, `per_call` steps per call (several launches, each of as many steps as the shape allows),
    against the oracle step by step.  announce: the labels of the next call's first steps are announced
    before every call (the last launch of a call then plans them); with a schedule seed some of those
    promises are broken (other labels, another c, fewer steps than planned, another call in between).
    planners: RB_OPT_PLANNERS (1: one planner workgroup per launch, 2: two per step, 0: the library's choice); None: runs of
    up to 200 steps go through both forms when the shape allows either, longer ones through the library's choice."""
    import paper_2406_03285_amd as rb

    if planners is None:
        exact = policy is None or policy[0] == 0
        either = 1 <= w.c <= 64 and 1 <= w.r <= 64 and w.K <= 1024 and w.b <= 2048 and exact
        if either and steps <= 200 and (window is None or window > 1) and not any(opt == rb.RB_OPT_PLANNERS for opt, _ in options):
            for form in (1, 2):
                run_many_parity(w, steps, per_call, window, announce, schedule_seed, store_bf16, policy, options, store_u8, form)
            return
        planners = 0
    dev = torch.device("cuda:0")
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev, store_dtype=_store_dtype(store_bf16, store_u8))
    buf.set_option(rb.RB_OPT_PLANNERS, planners)
    if window is not None:
        buf.set_option(rb.RB_OPT_WINDOW, window)
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    _set_oracle_storage(orc, store_bf16, store_u8)
    if policy is not None:
        buf.set_policy(*policy)
        orc.set_policy(*policy)
    for opt, val in options:
        buf.set_option(opt, val)
    oxs = [torch.empty((w.r, *w.shape), dtype=w.torch_dtype, device=dev) for _ in range(per_call)]
    oys = [torch.empty(w.r, dtype=torch.int64, device=dev) for _ in range(per_call)]
    rng = np.random.default_rng(schedule_seed)

    def make(first):
        n = max(0, min(per_call, steps - first))
        batches = [wl.make_batch(w, first + i, dev) for i in range(n)]
        return [x.contiguous() for x, _ in batches], [y.contiguous() for _, y in batches]

    first = 0
    xs, ys = make(0)
    while first < steps:
        n = len(xs)
        nxs, nys = make(first + n)              # the next call's mini-batches are there before this call is enqueued
        what = "keep" if schedule_seed is None else rng.choice(["keep", "keep", "other-labels", "other-c", "fewer-steps", "read-state"])
        c = w.c
        if what == "other-labels" and n > 1:    # the call that comes is not the one that was announced
            ys[min(1, n - 1)] = ys[min(1, n - 1)].clone()
        if what == "other-c":
            c = max(1, w.c - 1)
        if what == "fewer-steps" and n > 2:     # fewer steps than the launch before may have planned
            nxs, nys = xs[2:] + nxs, ys[2:] + nys
            nxs, nys = nxs[:per_call], nys[:per_call]
            xs, ys, n = xs[:2], ys[:2], 2
        if what == "read-state":
            assert np.array_equal(buf.read_state()[0], orc.fill)
        for i in range(n):
            _bytes(oxs[i]).fill_(SENTINEL)
            oys[i].fill_(-7)
        if announce and nys:
            buf.announce_next_many(nys[:32])
        if first % (2 * per_call) == 0:
            rc = rb.rb_update_sample_many(buf.handle, n, xs, ys, w.b, c, w.r, w.lib_seed, first, oxs[:n], oys[:n])
            assert rc == rb.RB_OK, rc
        else:           # the same through the class
            buf.update_sample_many(xs, ys, c, w.r, w.lib_seed, first, oxs[:n], oys[:n])
        torch.cuda.synchronize()
        for i in range(n):
            t = first + i
            orc.update(_bytes(xs[i]).cpu().numpy(), ys[i].cpu().numpy(), c, w.lib_seed, t)
            ref = np.full((w.r, w.row_bytes), SENTINEL, dtype=np.uint8)
            nn, ref_x, ref_y = orc.sample_augment(w.r, w.lib_seed, t, out_x=ref)
            assert np.array_equal(oys[i].cpu().numpy(), ref_y), f"{w.name} step {t} ({what}): out_y differs"
            assert np.array_equal(_bytes(oxs[i]).cpu().numpy(), ref_x), f"{w.name} step {t} ({what}): out_x differs (n={nn})"
        if not announce:        # (reading the state would drop a window that was planned across calls)
            compare_state(buf, orc, f"{w.name} step {first + n - 1}")
            assert buf.read_state()[1] == nn
        first += n
        xs, ys = nxs, nys
    compare_buffers(buf, orc, f"{w.name} final")
    assert buf.read_state()[1] == nn
