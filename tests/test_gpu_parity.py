"""GPU parity: the HIP library against the CPU oracle, byte for byte, through the C ABI.

Integer / byte work only, so the bar is bit-exact: per-class fill, flags, every
slot label, every stored row, every augmented row and label, on every step.
"""
import os

import numpy as np
import pytest
import torch

import rb_workloads as wl
from oracle import rbo
from parity_util import SENTINEL, compare_buffers, run_parity

pytestmark = pytest.mark.gpu

FULL = os.environ.get("RB_FULL", "0") == "1"      # run the large workloads for all their steps


@pytest.fixture(autouse=True)
def _free_device_memory():
    yield
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


def _rb():
    import paper_2406_03285_amd as rb
    return rb


# ------------------------------------------------------ the five workloads ---

def test_c1_tiny_all_steps():
    run_parity(wl.C1, check_state_every=10)


def test_c2_all_steps():
    run_parity(wl.C2, check_state_every=250, progress=250)


@pytest.mark.parametrize("w,steps", [(wl.C3, 120), (wl.C4, 50), (wl.C5, 40)], ids=["C3", "C4", "C5"])
def test_full_size_workloads(w, steps):
    """Real shapes (78-90 GB buffers) in the launch configuration the bench times."""
    print(f"\n{w.name}: buffer {w.buffer_bytes / 1e9:.1f} GB", flush=True)
    run_parity(w, steps=w.steps if FULL else steps, progress=10 if not FULL else 100)


def test_c3_on_a_side_stream():
    s = torch.cuda.Stream()
    run_parity(wl.variant(wl.C3, name="C3-side-stream", S=8), steps=30, stream=s)


# ------------------------------ the single-call primitive (one fused launch) ---

@pytest.mark.parametrize("w,steps", [
    (wl.C1, 100),                                                              # fills up: forwarding of appended and overwritten slots
    (wl.C2, 300),
    (wl.variant(wl.C3, name="C3-S4-single", S=4), 120),
    (wl.variant(wl.C4, name="C4-S8-single", S=8, shape=(3, 32, 32)), 100),     # Zipf head: several overwrites of one class per step
    (wl.variant(wl.C1, name="C1-one-class", K=1, S=7, c=16, r=16), 40),        # every representative competes with this step's writes
    (wl.variant(wl.C1, name="C1-r-large", S=3, c=16, r=64, b=64), 40),         # r above what is stored for a while, then r = F
    (wl.variant(wl.C2, name="C2-odd-b", b=77, c=33, r=21, S=2), 60),           # odd b: LDS table alignment
    (wl.variant(wl.C5, name="C5-fallback", K=2000, S=4, shape=(64,), b=256, c=100, r=30), 20),   # not eligible: two launches
])
def test_single_call_primitive(w, steps):
    run_parity(w, steps=steps, check_state_every=max(1, steps // 4), single_call=True)


@pytest.mark.parametrize("w,steps", [(wl.C3, 60), (wl.C4, 40)], ids=["C3", "C4"])
def test_single_call_full_size(w, steps):
    run_parity(w, steps=w.steps if FULL else steps, progress=10 if not FULL else 100, single_call=True)


def test_single_call_equals_two_calls_without_fusion():
    rb = _rb()
    w = wl.variant(wl.C1, name="C1-nofuse", S=5)
    run_parity(w, steps=40, options=((rb.RB_OPT_FUSE, 0),), single_call=True)


# ------------------------------------- policy variants of Algorithm 1 (NEXT-1) ---

POLICIES = {"bernoulli-uniform": (1, 0), "exact-fifo": (0, 1), "exact-reservoir": (0, 2), "bernoulli-fifo": (1, 1),
            "bernoulli-reservoir": (1, 2)}


@pytest.mark.parametrize("policy", sorted(POLICIES))
@pytest.mark.parametrize("w,steps", [
    (wl.C1, 100),                                                                  # fills up: every strategy replaces
    (wl.variant(wl.C2, name="C2-S3-policy", S=3), 120),
    (wl.variant(wl.C4, name="C4-S8-policy", S=8, shape=(3, 32, 32)), 60),          # Zipf head: many class-mates per step
    (wl.variant(wl.C5, name="C5-S16-K200-policy", K=200, S=16, shape=(64,)), 25),  # ~20 candidates per class and step into 16 slots
    (wl.variant(wl.C5, name="C5-S50-K5-policy", K=5, S=50, shape=(64,)), 12),      # ~200 candidates per class: more than one wavefront of class-mates
    (wl.Workload("laps", 9, 3, 2, (8,), "f32", 4096, 4096, 64, 6, "normal", "uniform"), 6),   # ~1365 candidates per class into 2 slots
    (wl.Workload("one-class", 9, 1, 5000, (8,), "bf16", 4096, 2000, 4096, 8, "normal", "uniform"), 8),
], ids=["C1", "C2-S3", "C4-S8", "C5-S16", "C5-K5", "laps", "one-class"])
def test_policy_variants(policy, w, steps):
    run_parity(w, steps=steps, check_state_every=max(1, steps // 3), policy=POLICIES[policy])


def test_policy_variant_through_the_single_call_and_at_full_size():
    run_parity(wl.C4, steps=30, policy=POLICIES["bernoulli-fifo"], single_call=True, progress=10)


def test_policy_cannot_change_after_an_update():
    rb = _rb()
    w = wl.C1
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype)
    assert rb.rb_set_policy(buf.handle, 2, 0) == rb.RB_EINVAL
    assert rb.rb_set_policy(buf.handle, 0, 3) == rb.RB_EINVAL
    assert rb.rb_set_policy(buf.handle, rb.RB_SELECT_BERNOULLI, rb.RB_EVICT_FIFO) == rb.RB_OK
    x, y = wl.make_batch(w, 0, "cuda:0")
    buf.update(x, y, w.c, 0, 0)
    assert rb.rb_set_policy(buf.handle, 0, 0) == rb.RB_ESTATE
    assert rb.rb_bind(buf.handle, buf.buf_x, buf.buf_y, buf.workspace, None) == rb.RB_OK
    assert rb.rb_set_policy(buf.handle, 0, 0) == rb.RB_OK


# ------------------------------------------- stress variants (replace path) ---

@pytest.mark.parametrize("w,steps", [
    (wl.variant(wl.C3, name="C3-S4", S=4), 150),                               # 16 per class > 4 slots: heavy replacement
    (wl.variant(wl.C4, name="C4-S8", S=8, shape=(3, 32, 32)), 100),            # Zipf head: many same-class evictions per step
    (wl.variant(wl.C5, name="C5-S16-K200", K=200, S=16, shape=(64,)), 40),     # 1024 candidates into 50 classes x 16 slots
    (wl.variant(wl.C5, name="C5-S50-K5", K=5, S=50, shape=(64,)), 20),         # ~200 candidates per class: more than one wavefront of class-mates
    (wl.variant(wl.C2, name="C2-S3", S=3), 200),
    (wl.variant(wl.C5, name="C5-small-rows", S=40, shape=(256,)), 30),         # K = 10000: two-level fill index, append chains
])
def test_stress_variants(w, steps):
    run_parity(w, steps=steps, check_state_every=max(1, steps // 3))


# -------------------------------------------------- launch-shape invariance ---

@pytest.mark.parametrize("unroll", [1, 2, 4, 8])
@pytest.mark.parametrize("nt", [0, 1])
def test_launch_shape_does_not_change_results(unroll, nt):
    rb = _rb()
    w = wl.variant(wl.C1, name=f"C1-u{unroll}-nt{nt}", shape=(777, 4), S=6, steps=40)   # 777 vectors per row: ragged tiles
    run_parity(w, options=((rb.RB_OPT_UNROLL, unroll), (rb.RB_OPT_NONTEMPORAL, nt)))


@pytest.mark.parametrize("rpb", [1, 2, 3, 16])
def test_rows_per_block(rpb):
    rb = _rb()
    w = wl.variant(wl.C2, name=f"C2-rpb{rpb}", shape=(64,), S=5, b=200, c=77, r=61, steps=30)
    run_parity(w, options=((rb.RB_OPT_ROWS_PER_BLOCK, rpb),))


# ------------------------------------------ buffer rows in pinned host memory ---

@pytest.mark.parametrize("single", [False, True])
def test_rows_in_pinned_host_memory(single):
    """The paper keeps the buffers in pinned host memory; the same kernels run on such storage."""
    w = wl.variant(wl.C3, name="C3-host-pinned", K=40, S=5, shape=(3, 64, 64))        # 9.8 MB of pinned rows
    run_parity(w, steps=40, storage="host_pinned", single_call=single, check_state_every=10)
    w = wl.variant(wl.C5, name="C5-host-pinned", K=300, S=8, shape=(256,), b=512, c=200, r=150)
    run_parity(w, steps=10, storage="host_pinned", single_call=single)


# ------------------------------------------------------ random configurations ---

def _random_workload(rng, i):
    big = rng.random() < 0.3                                  # sometimes large counts (general kernels)
    b = int(rng.integers(1, 4097 if big else 200))
    c = int(rng.integers(0, b + 1)) if rng.random() < 0.7 else int(min(b, rng.integers(0, 65)))
    r = int(rng.integers(0, 4097 if big else 130))
    K = int(rng.choice([1, 2, 7, 100, 1000, 1024, 1025, 3000, 20000]))
    S = int(rng.choice([1, 2, 3, 10, 60]))
    vecs = int(rng.choice([1, 2, 63, 64, 65, 255, 256, 257, 1000, 2049]))   # 16-byte vectors per row
    dtype = "f32" if rng.random() < 0.5 else "bf16"
    shape = (vecs * (4 if dtype == "f32" else 8),)
    labels = str(rng.choice(["uniform", "zipf", "active50"]))
    return wl.Workload(f"rand{i}-K{K}-S{S}-b{b}-c{c}-r{r}-v{vecs}", 9, K, S, shape, dtype, b, c, r, 6, "normal", labels)


@pytest.mark.parametrize("chunk", range(6))
def test_random_configurations(chunk):
    """Seeded random shapes, counts, policies, launch options and call styles, a few steps each."""
    rb = _rb()
    rng = np.random.default_rng(1000 + chunk)
    for i in range(12):
        w = _random_workload(rng, chunk * 100 + i)
        policy = (int(rng.integers(0, 2)), int(rng.integers(0, 3))) if rng.random() < 0.5 else None
        options = ((rb.RB_OPT_UNROLL, int(rng.choice([0, 1, 2, 4, 8]))), (rb.RB_OPT_NONTEMPORAL, int(rng.integers(0, 2))),
                   (rb.RB_OPT_ROWS_PER_BLOCK, int(rng.choice([0, 1, 3, 16]))), (rb.RB_OPT_FUSE, int(rng.integers(0, 2))))
        single = bool(rng.integers(0, 2))
        print(f"  {w.name} policy={policy} options={[v for _, v in options]} single_call={single}", flush=True)
        run_parity(w, steps=6, check_state_every=3, policy=policy, options=options, single_call=single)


# ------------------------------------------------------------- edge cases ---

@pytest.mark.parametrize("K,S,shape,dtype,b,c,r", [
    (1, 1, (4,), "f32", 1, 1, 1),                    # smallest everything: 16-byte rows
    (1, 5000, (8,), "bf16", 4096, 4096, 4096),       # maximum b = c = r, one class, append then replace
    (3, 2, (8,), "f32", 4096, 4096, 4096),           # maximum sizes into 6 slots: collisions everywhere; r >> F
    (257, 3, (12,), "f32", 64, 64, 100),             # two chunks of classes, ragged second chunk
    (70000, 2, (4,), "f32", 4096, 2048, 512),        # 274 chunks: several chunk sums per thread
    (5, 4, (3, 5, 8), "bf16", 33, 7, 9),
    (10, 20, (3, 32, 32), "f32", 16, 16, 300),       # c = b; r above capacity (200)
])
def test_edge_shapes(K, S, shape, dtype, b, c, r):
    w = wl.Workload(f"edge-{K}x{S}-{b}-{c}-{r}", 9, K, S, shape, dtype, b, c, r, 12, "normal", "uniform")
    run_parity(w, check_state_every=4)


def test_noop_calls_and_empty_buffer():
    rb = _rb()
    w = wl.C1
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype)
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    x, y = wl.make_batch(w, 0, "cuda:0")
    out_x = torch.zeros((w.r, *w.shape), device="cuda:0")
    out_y = torch.full((w.r,), 5, dtype=torch.int64, device="cuda:0")
    # sampling from an empty buffer: n = 0, labels -1, rows untouched
    buf.sample_augment(w.r, 0, 0, out_x, out_y)
    fill, last_n, flags = buf.read_state()
    assert last_n == 0 and fill.sum() == 0 and flags == 0
    assert out_y.tolist() == [-1] * w.r and not out_x.any()
    # c = 0 and r = 0 are no-ops
    buf.update(x, y, 0, 0, 0)
    buf.sample_augment(0, 0, 0, None, None)
    assert buf.read_state()[0].sum() == 0
    assert torch.all(buf.buf_y == -1)
    # several updates without sampling, then several samplings without update
    for step in range(5):
        x, y = wl.make_batch(w, step, "cuda:0")
        buf.update(x, y, w.c, 3, step)
        orc.update(wl.as_row_bytes(x), y.cpu().numpy(), w.c, 3, step)
    compare_buffers(buf, orc, "updates only")
    for step in range(5):
        buf.sample_augment(w.r, 3, 100 + step, out_x, out_y)
        n, rx, ry = orc.sample_augment(w.r, 3, 100 + step)
        assert out_y.cpu().numpy().tolist() == ry.tolist()
        assert np.array_equal(wl.as_row_bytes(out_x), rx)
        assert buf.read_state()[1] == n == w.r


def test_bad_labels_are_dropped_and_flagged():
    rb = _rb()
    K, S, b = 4, 8, 8
    buf = rb.RehearsalBuffer(K, S, (4,), torch.float32)
    orc = rbo.Buffer(K, S, 16)
    x = torch.randn(b, 4, device="cuda:0")
    y = torch.tensor([0, -1, 1, K, 2, 10**12, 3, -7], dtype=torch.int64, device="cuda:0")
    assert buf.read_state()[2] == 0
    buf.update(x, y, b, 0, 0)
    orc.update(wl.as_row_bytes(x), y.cpu().numpy(), b, 0, 0)
    fill, _, flags = buf.read_state()
    assert flags & rb.RB_FLAG_BAD_LABEL and fill.tolist() == [1, 1, 1, 1]
    compare_buffers(buf, orc, "bad labels")


def test_bind_again_resets():
    rb = _rb()
    w = wl.C1
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype)
    x, y = wl.make_batch(w, 0, "cuda:0")
    buf.update(x, y, w.c, 0, 0)
    assert buf.read_state()[0].sum() == w.c
    assert rb.rb_bind(buf.handle, buf.buf_x, buf.buf_y, buf.workspace, None) == rb.RB_OK
    assert buf.read_state()[0].sum() == 0 and torch.all(buf.buf_y == -1)
    run_parity(w, steps=20, buf=buf, orc=rbo.Buffer(w.K, w.S, w.row_bytes))


def test_device_pointer_validation_on_gpu():
    rb = _rb()
    buf = rb.RehearsalBuffer(4, 4, (8,), torch.float32)
    x = torch.zeros(9, 8, device="cuda:0")
    y = torch.zeros(9, dtype=torch.int64, device="cuda:0")
    assert rb.rb_update(buf.handle, x.data_ptr() + 4, y, 8, 2, 0, 0) == rb.RB_EINVAL
    assert rb.rb_sample_augment(buf.handle, 2, 0, 0, x.data_ptr() + 8, y) == rb.RB_EINVAL
    assert rb.rb_update(buf.handle, x, y, 8, 2, 0, 0) == rb.RB_OK


def test_copy_helper_moves_bytes():
    rb = _rb()
    src = torch.randint(0, 255, (3_000_016,), dtype=torch.uint8, device="cuda:0")
    for unroll in (1, 2, 4, 8):
        for nt in (0, 1):
            dst = torch.zeros_like(src)
            assert rb.rb_copy_bytes(None, dst, src, src.numel(), unroll, nt) == rb.RB_OK
            assert torch.equal(dst, src)
    assert rb.rb_copy_bytes(None, dst, src, 24, 4, 1) == rb.RB_EINVAL


def test_standin_compute_runs():
    rb = _rb()
    sink = torch.zeros(8 * 256, device="cuda:0")
    assert rb.rb_standin_compute(None, sink, 8, 1000) == rb.RB_OK
    torch.cuda.synchronize()
    assert torch.isfinite(sink).all() and sink.abs().sum() > 0
