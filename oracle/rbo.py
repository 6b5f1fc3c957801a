"""ctypes front of the C oracle (oracle/rbo.c).  Test infrastructure only.

Every array crossing this boundary is a C-contiguous numpy array on the host.
The functions mirror the C ones one to one; see rbo.c for what each computes
and which passage of the paper it follows (Sec. IV-A, Algorithm 1, Sec. IV-C).
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

SELECT, EVICT, SAMPLE, COIN = 1, 2, 3, 4
SELECT_EXACT, SELECT_BERNOULLI = 0, 1
EVICT_UNIFORM, EVICT_FIFO, EVICT_RESERVOIR = 0, 1, 2
STORE_SAME, STORE_BF16, STORE_U8 = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        L = C.CDLL(path)
        vp, i64, u64, u32 = C.c_void_p, C.c_int64, C.c_uint64, C.c_uint32
        L.rbo_philox4x32_10.argtypes = [vp, vp, vp]
        L.rbo_philox4x32_10.restype = None
        L.rbo_draw64.argtypes = [u64, u64, u32, u32]
        L.rbo_draw64.restype = u64
        L.rbo_bounded.argtypes = [u64, u64, u32, u32, u64]
        L.rbo_bounded.restype = u64
        L.rbo_floyd.argtypes = [u64, u64, u32, i64, i64, vp]
        L.rbo_floyd.restype = None
        L.rbo_create.argtypes = [i64, i64, i64]
        L.rbo_create.restype = vp
        L.rbo_destroy.argtypes = [vp]
        L.rbo_destroy.restype = None
        L.rbo_set_policy.argtypes = [vp, C.c_int, C.c_int]
        L.rbo_set_policy.restype = C.c_int
        L.rbo_set_storage.argtypes = [vp, C.c_int]
        L.rbo_set_storage.restype = C.c_int
        L.rbo_stored_row_bytes.argtypes = [vp]
        L.rbo_stored_row_bytes.restype = i64
        L.rbo_f32_to_bf16.argtypes = [u32]
        L.rbo_f32_to_bf16.restype = C.c_uint16
        L.rbo_bf16_to_f32.argtypes = [C.c_uint16]
        L.rbo_bf16_to_f32.restype = u32
        L.rbo_f32_to_u8.argtypes = [u32]
        L.rbo_f32_to_u8.restype = C.c_uint8
        L.rbo_u8_to_f32.argtypes = [C.c_uint8]
        L.rbo_u8_to_f32.restype = u32
        L.rbo_update.argtypes = [vp, vp, vp, i64, i64, u64, u64]
        L.rbo_update.restype = C.c_int
        L.rbo_sample_augment.argtypes = [vp, i64, u64, u64, vp, vp]
        L.rbo_sample_augment.restype = i64
        for name in ("rbo_fill", "rbo_buf_y", "rbo_ins_pos", "rbo_ins_class", "rbo_ins_slot", "rbo_sampled_g"):
            getattr(L, name).argtypes = [vp]
            getattr(L, name).restype = vp
        L.rbo_flags.argtypes = [vp]
        L.rbo_flags.restype = u32
        L.rbo_last_n.argtypes = [vp]
        L.rbo_last_n.restype = i64
        L.rbo_n_inserted.argtypes = [vp]
        L.rbo_n_inserted.restype = i64
        L.rbo_row.argtypes = [vp, i64, i64]
        L.rbo_row.restype = vp
        L.rbo_export_rows.argtypes = [vp, i64, i64, vp]
        L.rbo_export_rows.restype = None
        L.rbo_pool_create.argtypes = [C.c_int]
        L.rbo_pool_create.restype = vp
        L.rbo_pool_destroy.argtypes = [vp]
        L.rbo_pool_destroy.restype = None
        L.rbo_update_mt.argtypes = [vp, vp, vp, vp, i64, i64, u64, u64]
        L.rbo_update_mt.restype = C.c_int
        L.rbo_sample_augment_mt.argtypes = [vp, vp, i64, u64, u64, vp, vp]
        L.rbo_sample_augment_mt.restype = i64
        _lib = L
    return _lib


def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    lib().rbo_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def draw64(seed, step, purpose, index):
    return int(lib().rbo_draw64(seed, step, purpose, index))


def bounded(seed, step, purpose, index, n):
    return int(lib().rbo_bounded(seed, step, purpose, index, n))


def floyd(seed, step, purpose, n, m):
    out = np.empty(m, dtype=np.int64)
    lib().rbo_floyd(seed, step, purpose, n, m, out.ctypes.data)
    return out


def f32_to_bf16(bits):
    """bfloat16 bit pattern of the binary32 with bit pattern `bits`."""
    return int(lib().rbo_f32_to_bf16(int(bits)))


def bf16_to_f32(h):
    return int(lib().rbo_bf16_to_f32(int(h)))


def f32_to_u8(bits):
    """Byte that stores the binary32 with bit pattern `bits` (8-bit storage form)."""
    return int(lib().rbo_f32_to_u8(int(bits)))


def u8_to_f32(q):
    """Bit pattern of the binary32 that byte q is handed out as."""
    return int(lib().rbo_u8_to_f32(int(q)))


def _view(ptr, n, dtype):
    if n == 0 or not ptr:
        return np.empty(0, dtype=dtype)
    ct = {np.int32: C.c_int32, np.int64: C.c_int64}[dtype]
    return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(ct)), shape=(n,)).copy()


class Buffer:
    """One process's local rehearsal buffer B_n on the host."""

    def __init__(self, classes, slots_per_class, row_bytes):
        self.K, self.S, self.row_bytes = int(classes), int(slots_per_class), int(row_bytes)
        self._h = lib().rbo_create(self.K, self.S, self.row_bytes)
        if not self._h:
            raise ValueError("rbo_create rejected the arguments")

    def set_storage(self, storage):
        if lib().rbo_set_storage(self._h, int(storage)) != 0:
            raise ValueError("rbo_set_storage rejected the arguments (unknown variant, rows not made of 4-byte elements, "
                             "or the buffer is not empty)")

    @property
    def stored_row_bytes(self):
        return int(lib().rbo_stored_row_bytes(self._h))

    def set_policy(self, selection, eviction):
        if lib().rbo_set_policy(self._h, int(selection), int(eviction)) != 0:
            raise ValueError("rbo_set_policy rejected the arguments (unknown variant, or the buffer is not empty)")

    def close(self):
        if self._h:
            lib().rbo_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    @staticmethod
    def _bytes2d(a):
        a = np.ascontiguousarray(a)
        return a.view(np.uint8).reshape(a.shape[0], -1)

    def update(self, batch_x, batch_y, c, seed, step):
        x = self._bytes2d(batch_x)
        y = np.ascontiguousarray(batch_y, dtype=np.int64)
        b = y.shape[0]
        assert x.shape == (b, self.row_bytes), (x.shape, b, self.row_bytes)
        rc = lib().rbo_update(self._h, x.ctypes.data, y.ctypes.data, b, int(c), int(seed), int(step))
        if rc != 0:
            raise ValueError("rbo_update rejected the arguments")

    def sample_augment(self, r, seed, step, out_x=None):
        """Returns (n, out_x as uint8 [r,row_bytes], out_y int64 [r]); rows >= n of out_x keep what they held."""
        r = int(r)
        if out_x is None:
            out_x = np.zeros((r, self.row_bytes), dtype=np.uint8)
        out_y = np.empty(r, dtype=np.int64)
        assert out_x.dtype == np.uint8 and out_x.shape == (r, self.row_bytes) and out_x.flags.c_contiguous
        n = lib().rbo_sample_augment(self._h, r, int(seed), int(step), out_x.ctypes.data, out_y.ctypes.data)
        if n < 0:
            raise ValueError("rbo_sample_augment rejected the arguments")
        return int(n), out_x, out_y

    # ---- timing variant: the row copies of a call spread over the threads of a Pool ----
    def update_mt(self, pool, batch_x, batch_y, c, seed, step):
        x = self._bytes2d(batch_x)
        y = np.ascontiguousarray(batch_y, dtype=np.int64)
        b = y.shape[0]
        assert x.shape == (b, self.row_bytes), (x.shape, b, self.row_bytes)
        rc = lib().rbo_update_mt(pool._h, self._h, x.ctypes.data, y.ctypes.data, b, int(c), int(seed), int(step))
        if rc != 0:
            raise ValueError("rbo_update_mt rejected the arguments")

    def sample_augment_mt(self, pool, r, seed, step, out_x=None):
        r = int(r)
        if out_x is None:
            out_x = np.zeros((r, self.row_bytes), dtype=np.uint8)
        out_y = np.empty(r, dtype=np.int64)
        assert out_x.dtype == np.uint8 and out_x.shape == (r, self.row_bytes) and out_x.flags.c_contiguous
        n = lib().rbo_sample_augment_mt(pool._h, self._h, r, int(seed), int(step), out_x.ctypes.data, out_y.ctypes.data)
        if n < 0:
            raise ValueError("rbo_sample_augment_mt rejected the arguments")
        return int(n), out_x, out_y

    @property
    def fill(self):
        return _view(lib().rbo_fill(self._h), self.K, np.int32)

    @property
    def buf_y(self):
        return _view(lib().rbo_buf_y(self._h), self.K * self.S, np.int64).reshape(self.K, self.S)

    @property
    def flags(self):
        return int(lib().rbo_flags(self._h))

    @property
    def last_n(self):
        return int(lib().rbo_last_n(self._h))

    def last_insertions(self):
        """(pos, class, slot) of every insertion of the last update, in insertion order."""
        n = int(lib().rbo_n_inserted(self._h))
        L = lib()
        return (_view(L.rbo_ins_pos(self._h), n, np.int64), _view(L.rbo_ins_class(self._h), n, np.int64),
                _view(L.rbo_ins_slot(self._h), n, np.int64))

    def last_sampled_g(self):
        return _view(lib().rbo_sampled_g(self._h), self.last_n, np.int64)

    def row(self, k, s):
        p = lib().rbo_row(self._h, int(k), int(s))
        if not p:
            return None
        return np.ctypeslib.as_array(C.cast(p, C.POINTER(C.c_uint8)), shape=(self.stored_row_bytes,)).copy()

    def export_rows(self, first, count):
        """Rows as stored (stored_row_bytes each)."""
        out = np.empty((int(count), self.stored_row_bytes), dtype=np.uint8)
        lib().rbo_export_rows(self._h, int(first), int(count), out.ctypes.data)
        return out


class Pool:
    """Host threads that carry out the row copies of Buffer.update_mt / sample_augment_mt."""

    def __init__(self, threads):
        self.threads = int(threads)
        self._h = lib().rbo_pool_create(self.threads)
        if not self._h:
            raise ValueError("rbo_pool_create rejected the thread count")

    def close(self):
        if self._h:
            lib().rbo_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()
