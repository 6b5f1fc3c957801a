"""rb_bind_static: the entry point that allocates nothing (its workspace is an array the library holds in device
memory) against rb_bind with a caller's workspace: same results, byte for byte, on two uses of the array in a row,
the second by a smaller buffer."""
import numpy as np
import pytest
import torch

import rb_workloads as wl
from oracle import rbo
import parity_util
from parity_util import compare_buffers

pytestmark = pytest.mark.gpu


def _drive(w, steps, static):
    """`steps` steps of w: the first third through the two calls, the rest through announced several-steps calls.
    Returns the buffer and every step's labels and rows."""
    import paper_2406_03285_amd as rb
    dev = torch.device("cuda:0")
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    if static:
        # the tensors first, so that the call under test is the only thing between the two readings
        buf_x = torch.empty((w.K, w.S, *w.shape), dtype=w.torch_dtype, device=dev)
        buf_y = torch.empty((w.K, w.S), dtype=torch.int64, device=dev)
        rc, h = rb.rb_create(w.K, w.S, w.shape, rb.RB_F32 if w.dtype == "f32" else rb.RB_BF16)
        assert rc == rb.RB_OK
        # (the HIP runtime loads a library's device code, static arrays included, at the library's first launch
        # in the process: an ordinary bind first, so that this is not taken for an allocation of the call under test)
        warm = rb.RehearsalBuffer(2, 2, (4,), torch.float32, device=dev)
        torch.cuda.synchronize()
        del warm
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        assert rb.rb_bind_static(h, buf_x, buf_y, None) == rb.RB_OK
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before, "rb_bind_static changed the free device memory"
        rb.rb_destroy(h)
        del buf_x, buf_y
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev, static_workspace=static)
    assert (buf.workspace is None) == static
    batches = [wl.make_batch(w, t, dev) for t in range(steps)]
    xs, ys = [x.contiguous() for x, _ in batches], [y.contiguous() for _, y in batches]
    oxs = [torch.full((w.r, *w.shape), 3, dtype=w.torch_dtype, device=dev) for _ in range(steps)]
    oys = [torch.full((w.r,), -7, dtype=torch.int64, device=dev) for _ in range(steps)]
    third = steps // 3
    for t in range(third):
        buf.update(xs[t], ys[t], w.c, w.lib_seed, t)
        buf.sample_augment(w.r, w.lib_seed, t, oxs[t], oys[t])
    per_call = 9
    for first in range(third, steps, per_call):
        n = min(per_call, steps - first)
        nxt = ys[first + n:first + 2 * n]
        if nxt:
            buf.announce_next_many(nxt)
        buf.update_sample_many(xs[first:first + n], ys[first:first + n], w.c, w.r, w.lib_seed, first, oxs[first:first + n], oys[first:first + n])
    torch.cuda.synchronize()
    return buf, xs, ys, [y.cpu().numpy() for y in oys], [parity_util._bytes(x).cpu().numpy() for x in oxs]


def _same_as_rb_bind_and_the_oracle(w, steps):
    import paper_2406_03285_amd as rb
    sbuf, xs, ys, s_y, s_x = _drive(w, steps, static=True)
    pbuf, _, _, p_y, p_x = _drive(w, steps, static=False)
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    untouched = parity_util._bytes(torch.full((w.r, *w.shape), 3, dtype=w.torch_dtype)).numpy()
    for t in range(steps):
        assert np.array_equal(s_y[t], p_y[t]), f"{w.name} step {t}: labels differ from rb_bind's"
        assert np.array_equal(s_x[t], p_x[t]), f"{w.name} step {t}: rows differ from rb_bind's"
        orc.update(parity_util._bytes(xs[t]).cpu().numpy(), ys[t].cpu().numpy(), w.c, w.lib_seed, t)
        n, ref_x, ref_y = orc.sample_augment(w.r, w.lib_seed, t, out_x=untouched.copy())
        assert np.array_equal(s_y[t], ref_y) and np.array_equal(s_x[t], ref_x), f"{w.name} step {t}: differs from the oracle"
    assert np.array_equal(sbuf.read_state()[0], pbuf.read_state()[0])
    assert torch.equal(sbuf.buf_y, pbuf.buf_y)
    compare_buffers(sbuf, orc, f"{w.name} (static workspace) final")
    compare_buffers(pbuf, orc, f"{w.name} (caller's workspace) final")
    assert sbuf.moved_rows() == pbuf.moved_rows()
    return sbuf


def test_static_workspace_twice_in_a_row_the_second_time_smaller():
    import paper_2406_03285_amd as rb
    big = wl.variant(wl.C2, name="C2-static", K=1000, S=3, b=128, c=40, r=40)        # fills up, replaces, several steps per launch
    first = _same_as_rb_bind_and_the_oracle(big, 60)
    # the array now holds the last plans and counts of that buffer; a smaller one takes it over
    small = wl.variant(wl.C1, name="C1-static", S=5)
    second = _same_as_rb_bind_and_the_oracle(small, 60)
    # ... and the handle that held it before is unbound (its state is gone), with a clear status
    x, y = wl.make_batch(big, 0, "cuda:0")
    assert rb.rb_update(first.handle, x, y, big.b, big.c, 0, 0) == rb.RB_ESTATE
    assert rb.rb_read_state(first.handle, big.K)[0] == rb.RB_ESTATE
    # large counts (1024-thread planners, the large tables of the workspace) through the static array as well
    third = _same_as_rb_bind_and_the_oracle(wl.variant(wl.C5, name="C5-static", K=3000, S=4, shape=(64,), b=512, c=200, r=150), 30)
    assert rb.rb_update(second.handle, x, y, small.b, small.c, 0, 0) == rb.RB_ESTATE
    del third


def test_static_workspace_limit_and_argument_checks():
    import paper_2406_03285_amd as rb
    rc, h = rb.rb_create(rb.RB_MAX_CLASSES, 1, (4,), rb.RB_F32)                   # 2^20 classes: about 16 MB of workspace
    assert rc == rb.RB_OK
    assert rb.rb_query_sizes(h)[3] > rb.RB_STATIC_WORKSPACE_BYTES
    y = torch.zeros(16, dtype=torch.int64, device="cuda:0")
    assert rb.rb_bind_static(h, y, y, None) == rb.RB_ELIMIT
    assert "static scratch" in rb.rb_strerror(rb.RB_ELIMIT)
    rb.rb_destroy(h)
    rc, h = rb.rb_create(4, 2, (4,), rb.RB_F32)
    assert rb.rb_bind_static(h, None, y, None) == rb.RB_EINVAL
    assert rb.rb_bind_static(h, y.data_ptr() + 8, y, None) == rb.RB_EINVAL       # buf_x not 16-byte aligned
    assert rb.rb_bind_static(None, y, y, None) == rb.RB_EINVAL
    assert rb.rb_update(h, y, y, 4, 2, 0, 0) == rb.RB_ESTATE                      # none of them bound it
    rb.rb_destroy(h)
