"""Thin ctypes binding of the C ABI in include/rb.h (argument marshalling only).

Every function has the name and argument order of its C counterpart; tensors
are passed as device pointers.  PyTorch is used for device memory and streams
only.  There is no fallback: if librb.so is missing the import fails.
"""
import ctypes as C
import os

import torch  # first: the library must bind to the HIP runtime PyTorch has loaded

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("RB_LIBRARY") or os.path.join(HERE, "librb.so")   # RB_LIBRARY: another build of the same library

RB_F32, RB_BF16 = 0, 1
RB_OK, RB_EINVAL, RB_ENOMEM, RB_ESTATE, RB_EHIP, RB_ELIMIT = 0, -1, -2, -3, -4, -5
RB_STATIC_WORKSPACE_BYTES = 4 << 20
RB_MAX_BATCH = 4096
RB_MAX_CLASSES = 1 << 20
RB_FLAG_BAD_LABEL = 1
RB_OPT_UNROLL, RB_OPT_NONTEMPORAL, RB_OPT_ROWS_PER_BLOCK, RB_OPT_FUSE, RB_OPT_WINDOW, RB_OPT_PLANNERS = 0, 1, 2, 3, 4, 5
RB_SELECT_EXACT, RB_SELECT_BERNOULLI = 0, 1
RB_STORE_SAME, RB_STORE_BF16, RB_STORE_U8 = 0, 1, 2
RB_EVICT_UNIFORM, RB_EVICT_FIFO, RB_EVICT_RESERVOIR = 0, 1, 2

EXPORTS = (
    "rb_create", "rb_query_sizes", "rb_set_storage", "rb_bind", "rb_bind_static", "rb_set_policy", "rb_set_stream", "rb_update", "rb_sample_augment", "rb_update_sample",
    "rb_announce_next", "rb_announce_next_many", "rb_query_steps_per_launch", "rb_update_sample_many", "rb_pipeline_create", "rb_pipeline_step", "rb_pipeline_step_many", "rb_pipeline_drain", "rb_pipeline_destroy",
    "rb_read_state", "rb_read_moved_rows", "rb_set_option", "rb_destroy", "rb_strerror", "rb_standin_compute", "rb_copy_bytes",
)


class RbError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {rb_strerror(status)} ({status})")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python paper_2406_03285_amd/build.py` "
            "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i64, u64, i32, sz = C.c_void_p, C.c_int64, C.c_uint64, C.c_int32, C.c_size_t
    L.rb_create.argtypes = [C.POINTER(vp), i64, i64, C.POINTER(i64), i32, i32]
    L.rb_query_sizes.argtypes = [vp, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
    L.rb_bind.argtypes = [vp, vp, vp, vp, vp]
    L.rb_bind_static.argtypes = [vp, vp, vp, vp]
    L.rb_set_policy.argtypes = [vp, i32, i32]
    L.rb_set_storage.argtypes = [vp, i32]
    L.rb_set_stream.argtypes = [vp, vp]
    L.rb_update.argtypes = [vp, vp, vp, i64, i64, u64, u64]
    L.rb_sample_augment.argtypes = [vp, i64, u64, u64, vp, vp]
    L.rb_update_sample.argtypes = [vp, vp, vp, i64, i64, i64, u64, u64, vp, vp]
    L.rb_announce_next.argtypes = [vp, vp]
    L.rb_announce_next_many.argtypes = [vp, i64, C.POINTER(vp)]
    L.rb_query_steps_per_launch.argtypes = [vp, i64, i64, i64, C.POINTER(i64)]
    L.rb_update_sample_many.argtypes = [vp, i64, C.POINTER(vp), C.POINTER(vp), i64, i64, i64, u64, u64, C.POINTER(vp), C.POINTER(vp)]
    L.rb_pipeline_create.argtypes = [C.POINTER(vp), vp]
    L.rb_pipeline_step.argtypes = [vp, vp, vp, i64, i64, i64, u64, u64, vp, vp, vp, C.POINTER(i64)]
    L.rb_pipeline_step_many.argtypes = [vp, i64, C.POINTER(vp), C.POINTER(vp), i64, i64, i64, u64, u64, C.POINTER(vp), C.POINTER(vp), vp,
                                        C.POINTER(i64)]
    L.rb_pipeline_drain.argtypes = [vp, vp, C.POINTER(i64)]
    L.rb_read_moved_rows.argtypes = [vp, C.POINTER(u64)]
    L.rb_pipeline_destroy.argtypes = [vp]
    L.rb_read_state.argtypes = [vp, vp, C.POINTER(i64), C.POINTER(C.c_uint32)]
    L.rb_set_option.argtypes = [vp, i32, i64]
    L.rb_destroy.argtypes = [vp]
    L.rb_strerror.argtypes = [C.c_int]
    L.rb_strerror.restype = C.c_char_p
    L.rb_standin_compute.argtypes = [vp, vp, i64, i64]
    L.rb_copy_bytes.argtypes = [vp, vp, vp, sz, i32, i32]
    for name in EXPORTS:
        if name != "rb_strerror":
            getattr(L, name).restype = C.c_int
    return L


_L = _load()


def _ptr(t):
    """Device (or null) pointer of a tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s or None
    return s.cuda_stream or None


def rb_strerror(status):
    return _L.rb_strerror(int(status)).decode()


def rb_create(classes, slots_per_class, sample_shape, dtype):
    h = C.c_void_p()
    shape = (C.c_int64 * len(sample_shape))(*[int(v) for v in sample_shape])
    rc = _L.rb_create(C.byref(h), int(classes), int(slots_per_class), shape, len(sample_shape), int(dtype))
    return rc, h.value


def rb_query_sizes(rb):
    x, y, w = C.c_size_t(), C.c_size_t(), C.c_size_t()
    rc = _L.rb_query_sizes(rb, C.byref(x), C.byref(y), C.byref(w))
    return rc, x.value, y.value, w.value


def rb_bind(rb, buf_x, buf_y, workspace, hip_stream=None):
    return _L.rb_bind(rb, _ptr(buf_x), _ptr(buf_y), _ptr(workspace), _stream(hip_stream))


def rb_bind_static(rb, buf_x, buf_y, hip_stream=None):
    return _L.rb_bind_static(rb, _ptr(buf_x), _ptr(buf_y), _stream(hip_stream))


def rb_set_storage(rb, storage):
    return _L.rb_set_storage(rb, int(storage))


def rb_set_policy(rb, selection, eviction):
    return _L.rb_set_policy(rb, int(selection), int(eviction))


def rb_set_stream(rb, hip_stream):
    return _L.rb_set_stream(rb, _stream(hip_stream))


def rb_update(rb, batch_x, batch_y, b, c, seed, step):
    return _L.rb_update(rb, _ptr(batch_x), _ptr(batch_y), int(b), int(c), int(seed), int(step))


def rb_sample_augment(rb, r, seed, step, out_x, out_y):
    return _L.rb_sample_augment(rb, int(r), int(seed), int(step), _ptr(out_x), _ptr(out_y))


def rb_update_sample(rb, batch_x, batch_y, b, c, r, seed, step, out_x, out_y):
    return _L.rb_update_sample(rb, _ptr(batch_x), _ptr(batch_y), int(b), int(c), int(r), int(seed), int(step),
                               _ptr(out_x), _ptr(out_y))


def rb_announce_next(rb, next_batch_y):
    return _L.rb_announce_next(rb, _ptr(next_batch_y))


def rb_announce_next_many(rb, n, next_batch_y):
    """next_batch_y: sequence of n label tensors / addresses, or an array made by pointer_array."""
    arr = next_batch_y if next_batch_y is None or isinstance(next_batch_y, (C.Array, C._Pointer)) else pointer_array(next_batch_y)
    return _L.rb_announce_next_many(rb, int(n), arr)


def rb_query_steps_per_launch(rb, b, c, r):
    steps = C.c_int64(0)
    rc = _L.rb_query_steps_per_launch(rb, int(b), int(c), int(r), C.byref(steps))
    return rc, steps.value


def pointer_array(items):
    """Host array of device pointers (tensors or ints), reusable across rb_update_sample_many calls."""
    return (C.c_void_p * len(items))(*[_ptr(t) for t in items])


def rb_update_sample_many(rb, n, batch_x, batch_y, b, c, r, seed, first_step, out_x, out_y):
    """batch_x, batch_y, out_x, out_y: sequences of n tensors / addresses, or arrays made by pointer_array."""
    arrs = [a if a is None or isinstance(a, (C.Array, C._Pointer)) else pointer_array(a) for a in (batch_x, batch_y, out_x, out_y)]
    return _L.rb_update_sample_many(rb, int(n), arrs[0], arrs[1], int(b), int(c), int(r), int(seed), int(first_step),
                                    arrs[2], arrs[3])


def rb_pipeline_create(rb):
    h = C.c_void_p()
    rc = _L.rb_pipeline_create(C.byref(h), rb)
    return rc, h.value


def rb_pipeline_step(p, batch_x, batch_y, b, c, r, seed, step, next_x, next_y, train_stream=None):
    """Returns (status, ready_rows)."""
    n = C.c_int64()
    rc = _L.rb_pipeline_step(p, _ptr(batch_x), _ptr(batch_y), int(b), int(c), int(r), int(seed), int(step),
                             _ptr(next_x), _ptr(next_y), _stream(train_stream), C.byref(n))
    return rc, n.value


def rb_pipeline_step_many(p, n, batch_x, batch_y, b, c, r, seed, first_step, next_x, next_y, train_stream=None):
    """batch_x, batch_y, next_x, next_y: sequences of n tensors / addresses, or arrays made by pointer_array.
    Returns (status, ready_rows)."""
    arrs = [a if a is None or isinstance(a, (C.Array, C._Pointer)) else pointer_array(a) for a in (batch_x, batch_y, next_x, next_y)]
    rows = C.c_int64()
    rc = _L.rb_pipeline_step_many(p, int(n), arrs[0], arrs[1], int(b), int(c), int(r), int(seed), int(first_step),
                                  arrs[2], arrs[3], _stream(train_stream), C.byref(rows))
    return rc, rows.value


def rb_pipeline_drain(p, train_stream=None):
    """Returns (status, ready_rows)."""
    n = C.c_int64()
    rc = _L.rb_pipeline_drain(p, _stream(train_stream), C.byref(n))
    return rc, n.value


def rb_pipeline_destroy(p):
    return _L.rb_pipeline_destroy(p)


def rb_read_state(rb, classes):
    """Returns (status, fill [classes] int32 numpy array, last_n, flags)."""
    import numpy as np
    fill = np.zeros(int(classes), dtype=np.int32)
    n, fl = C.c_int64(), C.c_uint32()
    rc = _L.rb_read_state(rb, fill.ctypes.data, C.byref(n), C.byref(fl))
    return rc, fill, n.value, fl.value


def rb_read_moved_rows(rb):
    """Returns (status, rows moved since the last bind)."""
    rows = C.c_uint64()
    rc = _L.rb_read_moved_rows(rb, C.byref(rows))
    return rc, rows.value


def rb_set_option(rb, option, value):
    return _L.rb_set_option(rb, int(option), int(value))


def rb_destroy(rb):
    return _L.rb_destroy(rb)


def rb_standin_compute(hip_stream, sink, blocks, iters):
    return _L.rb_standin_compute(_stream(hip_stream), _ptr(sink), int(blocks), int(iters))


def rb_copy_bytes(hip_stream, dst, src, nbytes, unroll=4, nontemporal=1):
    return _L.rb_copy_bytes(_stream(hip_stream), _ptr(dst), _ptr(src), int(nbytes), int(unroll), int(nontemporal))


def _check(rc, where):
    if rc != RB_OK:
        raise RbError(rc, where)


class RehearsalBuffer:
    """Owns the device tensors of one buffer and forwards to the C ABI.

    Convenience only: allocates buf_x / buf_y / workspace with PyTorch, keeps the
    handle, raises RbError on a non-zero status.  All work is done by the library.
    """

    def __init__(self, classes, slots_per_class, sample_shape, dtype=torch.float32, device="cuda:0", stream=None,
                 storage="hbm", store_dtype=None, static_workspace=False):
        """storage: "hbm" keeps the sample rows in device memory; "host_pinned" keeps them in pinned host
        memory that the kernels read and write directly over the host link (where the paper keeps its
        buffers, Sec. IV-C); labels and workspace stay on the device either way.
        store_dtype: None keeps rows as they come; with dtype float32, torch.bfloat16 stores them at half size and
        torch.uint8 (values in [0, 1] as bytes) at a quarter.
        static_workspace: bind with rb_bind_static (the library's own scratch array instead of a workspace tensor)."""
        code = {torch.float32: RB_F32, torch.bfloat16: RB_BF16}[dtype]
        rc, self.handle = rb_create(classes, slots_per_class, tuple(sample_shape), code)
        _check(rc, "rb_create")
        self.K, self.S, self.sample_shape, self.dtype = int(classes), int(slots_per_class), tuple(sample_shape), dtype
        self.store_dtype = dtype if store_dtype is None else store_dtype
        if self.store_dtype != dtype:
            if dtype != torch.float32 or self.store_dtype not in (torch.bfloat16, torch.uint8):
                raise ValueError("only float32 samples stored as bfloat16 or uint8")
            _check(rb_set_storage(self.handle, RB_STORE_BF16 if self.store_dtype == torch.bfloat16 else RB_STORE_U8), "rb_set_storage")
        rc, xb, yb, wb = rb_query_sizes(self.handle)
        _check(rc, "rb_query_sizes")
        self.row_bytes = xb // (self.K * self.S)          # of a stored row
        self.device = torch.device(device)
        if storage == "hbm":
            self.buf_x = torch.empty((self.K, self.S, *self.sample_shape), dtype=self.store_dtype, device=self.device)
        elif storage == "host_pinned":
            self.buf_x = torch.empty((self.K, self.S, *self.sample_shape), dtype=self.store_dtype, pin_memory=True)
        else:
            raise ValueError(storage)
        self.storage = storage
        self.buf_y = torch.empty((self.K, self.S), dtype=torch.int64, device=self.device)
        assert self.buf_x.numel() * self.buf_x.element_size() == xb and self.buf_y.numel() * 8 == yb
        self.stream = stream
        if static_workspace:
            self.workspace = None
            _check(rb_bind_static(self.handle, self.buf_x, self.buf_y, stream), "rb_bind_static")
        else:
            self.workspace = torch.empty(wb, dtype=torch.uint8, device=self.device)
            _check(rb_bind(self.handle, self.buf_x, self.buf_y, self.workspace, stream), "rb_bind")

    def set_policy(self, selection, eviction):
        _check(rb_set_policy(self.handle, selection, eviction), "rb_set_policy")

    def set_stream(self, stream):
        self.stream = stream
        _check(rb_set_stream(self.handle, stream), "rb_set_stream")

    def update(self, batch_x, batch_y, c, seed, step):
        assert batch_x.is_contiguous() and batch_y.is_contiguous() and batch_y.dtype == torch.int64
        assert batch_x.dtype == self.dtype and tuple(batch_x.shape[1:]) == self.sample_shape
        assert batch_x.device == self.device and batch_y.device == self.device
        b = batch_y.shape[0]
        assert batch_x.shape[0] == b
        _check(rb_update(self.handle, batch_x, batch_y, b, c, seed, step), "rb_update")

    def sample_augment(self, r, seed, step, out_x, out_y):
        """out_x: [>= r, *sample_shape] contiguous, out_y: [>= r] int64; typically the tail of a (b+r)-row batch."""
        if r > 0:
            assert out_x.is_contiguous() and out_y.is_contiguous() and out_y.dtype == torch.int64
            assert out_x.dtype == self.dtype and tuple(out_x.shape[1:]) == self.sample_shape
            assert out_x.shape[0] >= r and out_y.shape[0] >= r
            assert out_x.device == self.device and out_y.device == self.device
        _check(rb_sample_augment(self.handle, r, seed, step, out_x, out_y), "rb_sample_augment")

    def announce_next(self, next_batch_y):
        """Labels of the next mini-batch (or None), so that the next update_sample also plans the step after it."""
        if next_batch_y is not None:
            assert next_batch_y.is_contiguous() and next_batch_y.dtype == torch.int64
        _check(rb_announce_next(self.handle, next_batch_y), "rb_announce_next")

    def update_sample(self, batch_x, batch_y, c, r, seed, step, out_x, out_y):
        assert batch_x.is_contiguous() and batch_y.is_contiguous() and batch_y.dtype == torch.int64
        assert batch_x.dtype == self.dtype and tuple(batch_x.shape[1:]) == self.sample_shape
        b = batch_y.shape[0]
        assert batch_x.shape[0] == b
        if r > 0:
            assert out_x.is_contiguous() and out_y.is_contiguous() and out_y.dtype == torch.int64
            assert out_x.dtype == self.dtype and tuple(out_x.shape[1:]) == self.sample_shape
            assert out_x.shape[0] >= r and out_y.shape[0] >= r
        _check(rb_update_sample(self.handle, batch_x, batch_y, b, c, r, seed, step, out_x, out_y), "rb_update_sample")

    def update_sample_many(self, batch_x, batch_y, c, r, seed, first_step, out_x, out_y):
        """len(batch_x) consecutive steps from one call (sequences of tensors, one per step)."""
        n = len(batch_x)
        assert len(batch_y) == n and (r == 0 or (len(out_x) == n and len(out_y) == n))
        b = batch_y[0].shape[0] if n else 1
        for i in range(n):
            assert batch_x[i].is_contiguous() and batch_y[i].is_contiguous() and batch_y[i].dtype == torch.int64
            assert batch_x[i].dtype == self.dtype and tuple(batch_x[i].shape[1:]) == self.sample_shape
            assert batch_x[i].shape[0] == b and batch_y[i].shape[0] == b
            if r > 0:
                assert out_x[i].is_contiguous() and out_y[i].is_contiguous() and out_y[i].dtype == torch.int64
                assert out_x[i].dtype == self.dtype and tuple(out_x[i].shape[1:]) == self.sample_shape
                assert out_x[i].shape[0] >= r and out_y[i].shape[0] >= r
        _check(rb_update_sample_many(self.handle, n, batch_x, batch_y, b, c, r, seed, first_step,
                                     out_x if r > 0 else None, out_y if r > 0 else None), "rb_update_sample_many")

    def announce_next_many(self, next_batch_y):
        """Labels of the first steps of the update_sample_many call after the next one."""
        for y in next_batch_y:
            assert y.is_contiguous() and y.dtype == torch.int64
        _check(rb_announce_next_many(self.handle, len(next_batch_y), next_batch_y), "rb_announce_next_many")

    def steps_per_launch(self, b, c, r):
        rc, steps = rb_query_steps_per_launch(self.handle, b, c, r)
        _check(rc, "rb_query_steps_per_launch")
        return steps

    def read_state(self):
        rc, fill, last_n, flags = rb_read_state(self.handle, self.K)
        _check(rc, "rb_read_state")
        return fill, last_n, flags

    def moved_rows(self):
        rc, rows = rb_read_moved_rows(self.handle)
        _check(rc, "rb_read_moved_rows")
        return rows

    def set_option(self, option, value):
        _check(rb_set_option(self.handle, option, value), "rb_set_option")

    def close(self):
        if getattr(self, "handle", None):
            rb_destroy(self.handle)
            self.handle = None

    def __del__(self):
        self.close()


class Pipeline:
    """The asynchronous `update` primitive on top of a RehearsalBuffer (argument marshalling only).

    step(batch_x, batch_y, c, r, seed, t, next_x, next_y, train_stream) returns the number of rows that the
    previous call's representatives hold (0 on the first call) once `train_stream` has been told to wait for them.
    """

    def __init__(self, buf):
        self.buf = buf
        rc, self.handle = rb_pipeline_create(buf.handle)
        _check(rc, "rb_pipeline_create")

    def step(self, batch_x, batch_y, c, r, seed, step, next_x, next_y, train_stream=None):
        buf = self.buf
        assert batch_x.is_contiguous() and batch_y.is_contiguous() and batch_y.dtype == torch.int64
        assert batch_x.dtype == buf.dtype and tuple(batch_x.shape[1:]) == buf.sample_shape
        b = batch_y.shape[0]
        assert batch_x.shape[0] == b
        if r > 0:
            assert next_x.is_contiguous() and next_y.is_contiguous() and next_y.dtype == torch.int64
            assert next_x.dtype == buf.dtype and tuple(next_x.shape[1:]) == buf.sample_shape
            assert next_x.shape[0] >= r and next_y.shape[0] >= r
        rc, rows = rb_pipeline_step(self.handle, batch_x, batch_y, b, c, r, seed, step, next_x, next_y, train_stream)
        _check(rc, "rb_pipeline_step")
        return rows

    def step_many(self, batch_x, batch_y, c, r, seed, first_step, next_x, next_y, train_stream=None):
        """len(batch_x) consecutive iterations from one call (sequences of tensors or pointer arrays are passed through)."""
        n = len(batch_x)
        b = batch_y[0].shape[0] if n else 1
        rc, rows = rb_pipeline_step_many(self.handle, n, batch_x, batch_y, b, c, r, seed, first_step, next_x, next_y, train_stream)
        _check(rc, "rb_pipeline_step_many")
        return rows

    def drain(self, train_stream=None):
        rc, rows = rb_pipeline_drain(self.handle, train_stream)
        _check(rc, "rb_pipeline_drain")
        return rows

    def close(self):
        if getattr(self, "handle", None):
            rb_pipeline_destroy(self.handle)
            self.handle = None

    def __del__(self):
        self.close()
