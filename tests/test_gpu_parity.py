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
import parity_util
from parity_util import compare_buffers, run_ahead_parity, run_many_parity, run_parity

pytestmark = pytest.mark.gpu

# The three large workloads run for ALL their configured steps (2000 / 2000 / 500) through the two calls and through
# the call form the bench times (announced several-steps calls for C3 and C4, announced single steps for C5); the
# other call forms run them for fewer steps unless RB_FULL=1 asks for everything.
FULL = os.environ.get("RB_FULL", "0") == "1"


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


@pytest.mark.parametrize("w", [wl.C3, wl.C4, wl.C5], ids=["C3", "C4", "C5"])
def test_full_size_workloads(w):
    """Real shapes (78-90 GB buffers), every configured step, rb_update + rb_sample_augment."""
    print(f"\n{w.name}: buffer {w.buffer_bytes / 1e9:.1f} GB, {w.steps} steps", flush=True)
    run_parity(w, steps=w.steps, progress=100)


def test_c5_with_one_fixed_set_of_active_classes():
    """C5's shape with the same 50 active classes in every step: they are full after about 50 steps, then every
    step overwrites about 20 slots of each and several candidates share a slot (the configured C5, whose active
    classes change every step, never fills a class).  The two general kernels, all 500 steps."""
    buf, orc = run_parity(wl.C5F, steps=wl.C5F.steps, progress=100)
    assert int((orc.fill == wl.C5F.S).sum()) == 50


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


# ---------------------------------------------- reduced-precision storage ---

_plain_make_batch = wl.make_batch


def _special_values_batch(w, step, dev):
    """A mini-batch whose float32 elements include every kind of rounding case: ties, values next to
    ties, subnormals, the largest finite values, infinities and NaNs of both signs."""
    x, y = _plain_make_batch(w, step, dev)
    bits = x.view(torch.int32).reshape(-1)
    special = torch.tensor([0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0x7F7FFFFF, 0x7F7F7FFF, 0x7F7F8000,
                            0x00000001, 0x00008000, 0x00008001, 0x00018000, 0x7F800000, 0x7FC00000, 0x7F800001,
                            0x00000000], dtype=torch.int64)
    special = torch.cat([special, special | 0x80000000])
    special = torch.where(special >= 2**31, special - 2**32, special).to(torch.int32).to(dev)
    g = torch.Generator(device="cpu")
    g.manual_seed(step)
    where = torch.randint(0, bits.numel(), (special.numel() * 40,), generator=g).to(dev)
    bits[where] = special.repeat(40)
    return x, y


@pytest.mark.parametrize("w,steps", [
    (wl.variant(wl.C2, name="C2-bf16-store", S=4), 60),
    (wl.variant(wl.C5, name="C5-bf16-store", K=300, S=12, shape=(264,), b=512, c=200, r=150), 25),   # 33 stored vectors per row: ragged tiles
    (wl.variant(wl.C3, name="C3-bf16-store", K=50, S=6), 20),                                       # 301 056-byte stored rows
], ids=["C2", "C5", "C3"])
def test_float32_samples_stored_as_bfloat16(w, steps):
    buf, orc = run_parity(w, steps=steps, check_state_every=max(1, steps // 2), store_bf16=True)
    assert buf.buf_x.dtype == torch.bfloat16 and buf.row_bytes == w.row_bytes // 2


def test_bfloat16_storage_rounds_every_special_value_like_the_oracle(monkeypatch):
    w = wl.variant(wl.C2, name="C2-bf16-special", S=3, c=64, r=64)
    monkeypatch.setattr(wl, "make_batch", lambda ww, step, dev="cpu": _special_values_batch(ww, step, dev))
    run_parity(w, steps=12, check_state_every=4, store_bf16=True)


@pytest.mark.parametrize("w,steps", [
    (wl.variant(wl.C2, name="C2-bf16-ahead", S=4), 60),                             # replaces from step ~25 on; forwarding through the rounding
    (wl.variant(wl.C1, name="C1-bf16-one-class-ahead", K=1, S=7, c=16, r=16), 40),  # every representative competes with this step's writes
    (wl.variant(wl.C3, name="C3-bf16-ahead", K=50, S=6), 25),                       # 301 056-byte stored rows, many tiles
], ids=["C2", "one-class", "C3"])
def test_bfloat16_storage_with_plan_ahead_steps(w, steps):
    run_ahead_parity(w, steps, store_bf16=True)


def test_bfloat16_storage_plan_ahead_special_values_and_broken_promises(monkeypatch):
    monkeypatch.setattr(wl, "make_batch", lambda ww, step, dev="cpu": _special_values_batch(ww, step, dev))
    run_ahead_parity(wl.variant(wl.C1, name="C1-bf16-special-ahead", K=2, S=5, c=12, r=12), 40, schedule_seed=5, store_bf16=True)


def test_bfloat16_storage_with_a_policy_variant_and_the_single_call():
    w = wl.variant(wl.C5, name="C5-bf16-fifo", K=40, S=16, shape=(64,), b=512, c=200, r=150)
    run_parity(w, steps=15, store_bf16=True, policy=POLICIES["bernoulli-fifo"], single_call=True)


def test_storage_variant_argument_checks():
    rb = _rb()
    rc, h = rb.rb_create(4, 2, (8,), rb.RB_BF16)
    assert rc == rb.RB_OK
    assert rb.rb_set_storage(h, rb.RB_STORE_BF16) == rb.RB_EINVAL      # samples are not binary32
    rb.rb_destroy(h)
    rc, h = rb.rb_create(4, 2, (4,), rb.RB_F32)
    assert rb.rb_set_storage(h, rb.RB_STORE_BF16) == rb.RB_EINVAL      # 16-byte samples: a stored row would be 8 bytes
    rb.rb_destroy(h)
    rc, h = rb.rb_create(4, 2, (8,), rb.RB_F32)
    assert rb.rb_set_storage(h, 2) == rb.RB_EINVAL
    assert rb.rb_query_sizes(h)[1] == 4 * 2 * 32
    assert rb.rb_set_storage(h, rb.RB_STORE_BF16) == rb.RB_OK
    assert rb.rb_query_sizes(h)[1] == 4 * 2 * 16
    assert rb.rb_set_storage(h, rb.RB_STORE_SAME) == rb.RB_OK
    rb.rb_destroy(h)
    buf = rb.RehearsalBuffer(4, 2, (8,), torch.float32)
    assert rb.rb_set_storage(buf.handle, rb.RB_STORE_BF16) == rb.RB_ESTATE   # already bound


# ------------------------------------------------- 8-bit storage (Sec. VII) ---

def _image_like_batch(w, step, dev):
    """Values as an image pipeline gives them, plus everything the conversion has to decide: every k/255, the values
    around every tie (k + 1/2)/255, values outside [0, 1], zeros of both signs, subnormals, infinities and NaNs."""
    x, y = _plain_make_batch(w, step, dev)
    x = x.abs().fmod(1.0) if w.values == "normal" else x
    flat = x.reshape(-1)
    k = torch.arange(256, dtype=torch.float32)
    ties = ((torch.arange(255, dtype=torch.float32) + 0.5) / 255.0)
    special = torch.cat([k / 255.0, ties, torch.nextafter(ties, torch.zeros(())), torch.nextafter(ties, torch.ones(())),
                         torch.tensor([-0.0, -0.25, 1.0000001, 7.5, float("inf"), -float("inf"), float("nan"), 1e-45, -1e-45])])
    g = torch.Generator(device="cpu")
    g.manual_seed(step)
    where = torch.randint(0, flat.numel(), (special.numel() * 3,), generator=g).to(dev)
    flat[where] = special.repeat(3).to(dev)
    return x, y


@pytest.mark.parametrize("w,steps", [
    (wl.variant(wl.C2, name="C2-u8-store", S=4), 60),                                                 # N(0,1) values: half of them saturate
    (wl.variant(wl.C5, name="C5-u8-store", K=300, S=12, shape=(272,), b=512, c=200, r=150), 25),     # 17 stored vectors per row: ragged tiles
    (wl.variant(wl.C3, name="C3-u8-store", K=50, S=6), 20),                                          # U(0,1) images, 150 528-byte stored rows
], ids=["C2", "C5", "C3"])
def test_float32_samples_stored_in_8_bits(w, steps):
    buf, orc = run_parity(w, steps=steps, check_state_every=max(1, steps // 2), store_u8=True)
    assert buf.buf_x.dtype == torch.uint8 and buf.row_bytes == w.row_bytes // 4


def test_8_bit_storage_decides_every_value_like_the_oracle(monkeypatch):
    w = wl.variant(wl.C2, name="C2-u8-special", S=3, c=64, r=64, values="uniform")
    monkeypatch.setattr(wl, "make_batch", lambda ww, step, dev="cpu": _image_like_batch(ww, step, dev))
    buf, orc = run_parity(w, steps=12, check_state_every=4, store_u8=True)
    assert len(torch.unique(buf.buf_x)) == 256                       # every byte value is in use


def test_8_bit_storage_decides_every_value_like_the_oracle_with_several_steps_per_launch(monkeypatch):
    """Few classes: most representatives of a launch come from mini-batch rows of the same launch (through the 8-bit code
    the slot will hold) or are handed the slot's old content by the candidate that overwrites it."""
    w = wl.variant(wl.C2, name="C2-u8-special-many", K=3, S=30, c=32, r=32, values="uniform")
    monkeypatch.setattr(wl, "make_batch", lambda ww, step, dev="cpu": _image_like_batch(ww, step, dev))
    run_many_parity(w, 48, per_call=16, announce=True, store_u8=True)
    run_many_parity(w, 40, per_call=19, store_u8=True, policy=POLICIES["exact-fifo"])


@pytest.mark.parametrize("w,steps,per_call", [
    (wl.variant(wl.C3, name="C3-u8-many", K=50, S=6), 96, 64),                                       # full-size rows, 32 steps per launch
    (wl.variant(wl.C4, name="C4-u8-many", S=3, K=40, dtype="f32", shape=(3, 64, 64)), 60, 20),        # 64 + 64 rows per step, 8 steps per launch
    (wl.variant(wl.C1, name="C1-u8-many-ragged", shape=(3, 20, 20), S=4), 70, 33),                    # 75 stored vectors per row
], ids=["C3", "C4", "ragged"])
def test_8_bit_storage_with_several_steps_per_launch(w, steps, per_call):
    run_many_parity(w, steps, per_call=per_call, announce=True, store_u8=True)
    run_many_parity(w, steps // 2, per_call=per_call, store_u8=True)


@pytest.mark.parametrize("w,policy", [
    (wl.variant(wl.C5, name="bw-u8-two-classes", K=2, S=40, shape=(64,), b=256, c=100, r=70), None),                # 4 stored vectors per row; every step reads and rewrites most slots
    (wl.variant(wl.C5, name="bw-u8-K300-fifo", K=300, S=12, shape=(272,), b=512, c=200, r=150), "exact-fifo"),        # 17 stored vectors: ragged
    (wl.variant(wl.C5, name="bw-u8-long-rows", K=6, S=30, shape=(3, 64, 64), b=256, c=100, r=70), None),              # 768 stored vectors: tiles for 256 threads
    (wl.variant(wl.C5, name="bw-u8-bernoulli-reservoir", K=2, S=40, shape=(64,), b=256, c=100, r=70), "bernoulli-reservoir"),
    (wl.variant(wl.C5, name="bw-u8-C5-rows", K=40, S=30, b=1024, c=300, r=300), None),                               # C5's rows: one wavefront per 2 KiB stored row
], ids=lambda v: v.name if hasattr(v, "name") else None)
def test_8_bit_storage_with_large_counts(w, policy):
    pol = POLICIES[policy] if policy else None
    run_many_parity(w, 40, per_call=19, policy=pol, store_u8=True)
    run_many_parity(w, 40, per_call=16, announce=True, policy=pol, store_u8=True)
    run_ahead_parity(w, 30, policy=pol, store_u8=True)                 # one launch per step, planned by the launch before
    run_ahead_parity(w, 30, schedule_seed=3, policy=pol, store_u8=True)


def test_8_bit_storage_decides_every_value_like_the_oracle_with_large_counts(monkeypatch):
    w = wl.variant(wl.C5, name="bw-u8-special", K=3, S=60, shape=(3, 32, 32), b=256, c=100, r=100, values="uniform")
    monkeypatch.setattr(wl, "make_batch", lambda ww, step, dev="cpu": _image_like_batch(ww, step, dev))
    run_many_parity(w, 40, per_call=16, announce=True, store_u8=True)
    run_ahead_parity(w, 20, store_u8=True)


@pytest.mark.parametrize("style", ["single", "ahead", "many", "many-announced", "fifo-bernoulli"])
def test_8_bit_storage_through_every_call_form(style):
    """The 8-bit form is served by the general kernels, the plan-ahead steps and the several-steps launches; the bytes are
    the oracle's in every call form."""
    w = wl.variant(wl.C4, name=f"C4-u8-{style}", S=8, shape=(3, 32, 32), dtype="f32", b=128, c=40, r=40)
    if style == "single":
        run_parity(w, steps=40, store_u8=True, single_call=True)
    elif style == "ahead":
        run_ahead_parity(w, 40, schedule_seed=4, store_u8=True)
    elif style == "many":
        run_many_parity(w, 48, per_call=16, store_u8=True)
    elif style == "many-announced":
        run_many_parity(w, 48, per_call=16, announce=True, schedule_seed=6, store_u8=True)
    else:
        run_many_parity(w, 48, per_call=16, announce=True, store_u8=True, policy=POLICIES["bernoulli-fifo"])


def test_8_bit_storage_argument_checks():
    rb = _rb()
    rc, h = rb.rb_create(4, 2, (16,), rb.RB_BF16)
    assert rb.rb_set_storage(h, rb.RB_STORE_U8) == rb.RB_EINVAL       # samples are not binary32
    rb.rb_destroy(h)
    rc, h = rb.rb_create(4, 2, (8,), rb.RB_F32)
    assert rb.rb_set_storage(h, rb.RB_STORE_U8) == rb.RB_EINVAL       # 32-byte samples: a stored row would be 8 bytes
    rb.rb_destroy(h)
    rc, h = rb.rb_create(4, 2, (16,), rb.RB_F32)
    assert rb.rb_set_storage(h, 3) == rb.RB_EINVAL
    assert rb.rb_set_storage(h, rb.RB_STORE_U8) == rb.RB_OK and rb.rb_query_sizes(h)[1] == 4 * 2 * 16
    assert rb.rb_query_steps_per_launch(h, 512, 65, 8) == (rb.RB_OK, 16)  # the several-steps launch for large counts serves it
    assert rb.rb_set_option(h, rb.RB_OPT_PLANNERS, 1) == rb.RB_OK
    assert rb.rb_query_steps_per_launch(h, 64, 8, 8) == (rb.RB_OK, 32)   # ... and so does the one for small counts
    rb.rb_destroy(h)


# ------------------------------------------------------- plan-ahead steps ---

@pytest.mark.parametrize("w,steps", [
    (wl.C1, 100),                                                                   # fills up: append, replace, collisions
    (wl.variant(wl.C4, name="C4-S8-ahead", S=8, shape=(3, 32, 32)), 80),            # Zipf head: several overwrites of one class per step
    (wl.variant(wl.C1, name="C1-one-class-ahead", K=1, S=7, c=16, r=16), 40),       # every representative competes with this step's writes
    (wl.variant(wl.C1, name="C1-r-large-ahead", S=3, c=16, r=64, b=64), 40),        # r above what is stored, then r = F
    (wl.variant(wl.C2, name="C2-odd-b-ahead", b=77, c=33, r=21, S=2), 60),
    (wl.variant(wl.C3, name="C3-S4-ahead", S=4, K=1000), 40),                       # full-size rows, many tiles
    (wl.variant(wl.C5, name="C5-fallback-ahead", K=20000, S=4, shape=(64,), b=256, c=100, r=30), 15),  # not eligible (too many classes): announcement ignored
], ids=["C1", "C4-S8", "one-class", "r-large", "odd-b", "C3-S4", "not-eligible"])
def test_plan_ahead_steps(w, steps):
    run_ahead_parity(w, steps)


@pytest.mark.parametrize("w,steps", [
    (wl.variant(wl.C5, name="C5-K300-big", K=300, S=12, shape=(256,), b=512, c=200, r=150), 40),      # classes fill up: drawn slots, shared slots
    (wl.variant(wl.C5, name="C5-K2000-big", K=2000, S=4, shape=(64,), b=256, c=100, r=30), 25),
    (wl.variant(wl.C5, name="C5-limits-big", K=10240, S=3, shape=(16,), b=4096, c=1024, r=1024), 12), # every limit at once
    (wl.variant(wl.C4, name="C4-zipf-big", K=1000, S=8, shape=(3, 8, 8), b=2048, c=700, r=900), 20),  # Zipf head: a class list of hundreds
    (wl.variant(wl.C1, name="C1-one-class-big", K=1, S=50, b=300, c=300, r=100), 10),                 # one list of 300, every slot contested
    (wl.variant(wl.C2, name="C2-r-large-big", K=100, S=2, b=128, c=70, r=500), 12),                   # r above what is stored, then r = F
    (wl.variant(wl.C3, name="C3-K1100-big", K=1100, S=2), 12),                                        # few full-size rows (many tiles each), too many classes for the small plan
    (wl.variant(wl.C5, name="C5-K5000-odd-big", K=5003, S=7, shape=(12,), b=777, c=333, r=211), 25),
], ids=["K300", "K2000", "limits", "zipf", "one-class", "r-large", "C3-K1100", "odd"])
def test_plan_ahead_steps_with_large_counts(w, steps):
    """More than 64 candidates or representatives, or more than 1024 classes: the plan of a 1024-thread workgroup."""
    run_ahead_parity(w, steps)


@pytest.mark.parametrize("w,steps", [
    (wl.C1, 100),                                                                               # 16 positions, about 4 candidates: fills up, replaces
    (wl.variant(wl.C2, name="C2-S3-bernoulli-ahead", S=3), 80),
    (wl.variant(wl.C4, name="C4-S8-bernoulli-ahead", S=8, shape=(3, 32, 32)), 60),              # 512 positions, Zipf head
    (wl.variant(wl.C5, name="C5-b1024-bernoulli-ahead", K=300, S=12, shape=(256,), b=1024, c=400, r=150), 30),   # the largest mini-batch this form takes
    (wl.variant(wl.C5, name="C5-b1025-bernoulli-ahead", K=300, S=12, shape=(64,), b=1025, c=400, r=150), 10),    # one more: not eligible, announcement ignored
    (wl.variant(wl.C1, name="C1-c-equals-b-bernoulli-ahead", b=64, c=64, r=20, S=3), 30),       # every coin shows heads
], ids=["C1", "C2-S3", "C4-S8", "b1024", "b1025", "c=b"])
def test_plan_ahead_with_the_bernoulli_selection(w, steps):
    run_ahead_parity(w, steps, policy=POLICIES["bernoulli-uniform"])
    run_many_parity(w, min(steps, 40), per_call=7, announce=True, policy=POLICIES["bernoulli-uniform"])


@pytest.mark.parametrize("policy", ["exact-fifo", "exact-reservoir", "bernoulli-fifo", "bernoulli-reservoir"])
@pytest.mark.parametrize("w,steps", [
    (wl.variant(wl.C5, name="C5-K300-big-policy", K=300, S=12, shape=(256,), b=512, c=200, r=150), 40),   # classes fill up, then every strategy replaces
    (wl.Workload("laps-big", 9, 3, 2, (8,), "f32", 600, 300, 100, 20, "normal", "uniform"), 20),          # ~100 candidates per class into 2 slots: many rounds within a step
    (wl.variant(wl.C4, name="C4-zipf-big-policy", K=1000, S=8, shape=(3, 8, 8), b=1024, c=700, r=900), 20),
    (wl.variant(wl.C2, name="C2-K1100-big-policy", K=1100, S=2), 60),                                     # few candidates, too many classes for the small plan
], ids=["K300", "laps", "zipf", "K1100"])
def test_plan_ahead_with_large_counts_and_other_policies(policy, w, steps):
    run_ahead_parity(w, steps, policy=POLICIES[policy])


@pytest.mark.parametrize("w,steps,policy", [
    (wl.variant(wl.C5, name="C5-K300-big-bf16", K=300, S=12, shape=(256,), b=512, c=200, r=150), 40, None),          # forwarding through the rounded row
    (wl.variant(wl.C5, name="C5-K300-big-bf16-fifo", K=300, S=12, shape=(256,), b=512, c=200, r=150), 30, "exact-fifo"),
    (wl.variant(wl.C3, name="C3-K1100-big-bf16", K=1100, S=2), 12, None),                                            # full-size rows, many tiles
    (wl.variant(wl.C1, name="C1-bernoulli-big-bf16", S=3), 60, "bernoulli-uniform"),
], ids=["K300", "K300-fifo", "C3-K1100", "bernoulli"])
def test_plan_ahead_with_large_counts_and_bfloat16_storage(w, steps, policy):
    run_ahead_parity(w, steps, store_bf16=True, policy=POLICIES[policy] if policy else None)


def _long(name, vecs, b, c, r, K=12, S=3, dtype="f32"):
    """A few classes of a few slots with rows of `vecs` 16-byte vectors: every step replaces and collides."""
    return wl.Workload(name, 9, K, S, (vecs * (4 if dtype == "f32" else 8),), dtype, b, c, r, 8, "normal", "uniform")


@pytest.mark.parametrize("w,bf16,policy", [
    (_long("long-u12", 18816, 512, 65, 64), False, None),            # 129 rows in 7 tiles of up to 2688 vectors: one workgroup per compute unit
    (_long("long-u8", 9000, 300, 100, 100), False, None),            # 5 tiles of 1856
    (_long("long-u6-ragged", 5003, 400, 150, 100), False, None),     # row length not a multiple of the tile unit
    (_long("long-u10", 12001, 200, 80, 90), False, "exact-fifo"),
    (_long("long-two-per-cu", 6000, 700, 300, 300), False, None),    # too many rows for one workgroup per compute unit: two
    (_long("long-bf16", 18816, 512, 65, 64), True, None),            # stored rows of 9408 vectors, converting mover
    (_long("long-bf16-wide", 37632, 128, 65, 64, K=6, S=2), True, "exact-reservoir"),
    (_long("long-bernoulli", 18816, 512, 64, 64, dtype="bf16"), False, "bernoulli-uniform"),   # the grid covers 128 candidate entries
], ids=lambda v: v.name if hasattr(v, "name") else None)
def test_plan_ahead_with_large_counts_and_long_rows(w, bf16, policy):
    """The large-count launch cuts long rows so that its workgroups spread evenly over the compute units."""
    pol = POLICIES[policy] if policy else None
    run_ahead_parity(w, 8, policy=pol, store_bf16=bf16)
    run_many_parity(w, 12, per_call=5, announce=True, policy=pol, store_bf16=bf16)


def test_plan_ahead_with_the_bernoulli_selection_survives_broken_promises():
    run_ahead_parity(wl.variant(wl.C4, name="C4-S8-bernoulli-promises", S=8, shape=(3, 32, 32), b=128, c=40, r=40), 90, schedule_seed=3,
                     policy=POLICIES["bernoulli-uniform"])


@pytest.mark.parametrize("seed", [4, 5])
def test_plan_ahead_with_large_counts_survives_broken_promises(seed):
    run_ahead_parity(wl.variant(wl.C5, name=f"C5-big-promises-{seed}", K=300, S=12, shape=(256,), b=512, c=200, r=150), 70, schedule_seed=seed)


def test_plan_ahead_with_large_counts_drops_and_flags_bad_labels():
    rb = _rb()
    dev = torch.device("cuda:0")
    K, S, b, c, r, n = 1500, 2, 200, 150, 90, 6
    buf = rb.RehearsalBuffer(K, S, (8,), torch.float32, device=dev)
    orc = rbo.Buffer(K, S, 32)
    g = torch.Generator(device="cpu")
    g.manual_seed(6)
    xs = [torch.randn((b, 8), generator=g).to(dev) for _ in range(n)]
    ys = [torch.randint(0, K, (b,), generator=g, dtype=torch.int64) for _ in range(n)]
    ys[2][::3] = -1
    ys[4][1::4] = K
    ys[4][5] = 10**12
    ys = [y.to(dev) for y in ys]
    out_x = torch.zeros((r, 8), device=dev)
    out_y = torch.full((r,), -7, dtype=torch.int64, device=dev)
    for t in range(n):
        if t + 1 < n:
            buf.announce_next(ys[t + 1])
        buf.update_sample(xs[t], ys[t], c, r, 21, t, out_x, out_y)
        if t < 2:
            assert buf.read_state()[2] == 0          # step 2 is planned during step 1, its flag is raised when it runs
        orc.update(parity_util._bytes(xs[t]).cpu().numpy(), ys[t].cpu().numpy(), c, 21, t)
        m, ref_x, ref_y = orc.sample_augment(r, 21, t)
        assert np.array_equal(out_y.cpu().numpy(), ref_y), f"step {t}: labels differ"
        assert np.array_equal(parity_util._bytes(out_x).cpu().numpy()[:m], ref_x[:m]), f"step {t}: rows differ"
    assert buf.read_state()[2] == rb.RB_FLAG_BAD_LABEL == orc.flags
    compare_buffers(buf, orc, "bad labels, large counts")


@pytest.mark.parametrize("w,steps", [(wl.C3, 60), (wl.C4, 40), (wl.C5, wl.C5.steps), (wl.C5F, wl.C5F.steps)], ids=["C3", "C4", "C5", "C5F"])
def test_plan_ahead_at_full_size(w, steps):
    """Real shapes, one launch per step, next labels announced; C5 (the form the bench times it in) and its
    variant with a fixed set of active classes for all their steps."""
    run_ahead_parity(w, w.steps if FULL else steps)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_plan_ahead_survives_broken_promises(seed):
    run_ahead_parity(wl.variant(wl.C4, name=f"C4-S8-promises-{seed}", S=8, shape=(3, 32, 32), b=128, c=40, r=40), 90, schedule_seed=seed)
    run_ahead_parity(wl.variant(wl.C1, name=f"C1-promises-{seed}"), 90, schedule_seed=seed + 10)


@pytest.mark.parametrize("policy", ["exact-fifo", "exact-reservoir"])
@pytest.mark.parametrize("w,steps", [
    (wl.C1, 100),                                                                           # fills up: every strategy replaces
    (wl.variant(wl.C4, name="C4-S8-ahead-policy", S=8, shape=(3, 32, 32)), 60),             # Zipf head: many class-mates per step
    (wl.Workload("laps-ahead", 9, 3, 2, (8,), "f32", 64, 64, 64, 30, "normal", "uniform"), 30),   # ~21 candidates per class into 2 slots
    (wl.variant(wl.C2, name="C2-S3-ahead-policy", S=3), 80),
], ids=["C1", "C4-S8", "laps", "C2-S3"])
def test_plan_ahead_with_other_replacement_strategies(policy, w, steps):
    run_ahead_parity(w, steps, policy=POLICIES[policy])


def test_plan_ahead_policy_bf16_and_broken_promises_together():
    w = wl.variant(wl.C1, name="C1-fifo-bf16-promises", K=4, S=5, c=12, r=12)
    run_ahead_parity(w, 60, schedule_seed=7, store_bf16=True, policy=POLICIES["exact-fifo"])
    run_ahead_parity(w, 60, schedule_seed=8, store_bf16=True, policy=POLICIES["exact-reservoir"])
    # the Bernoulli selection has no bound of 64 on its candidates: announcements are ignored, results unchanged
    run_ahead_parity(w, 30, policy=POLICIES["bernoulli-fifo"])


def test_an_announcement_that_was_not_used_is_forgotten():
    """Labels are announced, then other calls come instead of rb_update_sample.  The announcement
    must not linger and be taken for the labels of a later step that happens to reuse the memory."""
    rb = _rb()
    dev = torch.device("cuda:0")
    w = wl.C1
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev)
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    out_x = torch.empty((w.r, *w.shape), dtype=w.torch_dtype, device=dev)
    out_y = torch.empty(w.r, dtype=torch.int64, device=dev)
    lab = torch.empty(w.b, dtype=torch.int64, device=dev)          # one piece of memory for every step's labels
    for t in range(12):
        x, y = wl.make_batch(w, t, dev)
        lab.copy_(y)
        if t % 3 == 0:
            buf.announce_next(lab)                                 # never followed by rb_update_sample
            buf.update(x, lab, w.c, w.lib_seed, t)
            buf.sample_augment(w.r, w.lib_seed, t, out_x, out_y)
        else:
            buf.update_sample(x, lab, w.c, w.r, w.lib_seed, t, out_x, out_y)
        orc.update(parity_util._bytes(x).cpu().numpy(), y.cpu().numpy(), w.c, w.lib_seed, t)
        n, ref_x, ref_y = orc.sample_augment(w.r, w.lib_seed, t)
        assert np.array_equal(out_y.cpu().numpy(), ref_y), f"step {t}"
        assert np.array_equal(parity_util._bytes(out_x).cpu().numpy()[:n], ref_x[:n]), f"step {t}"
    compare_buffers(buf, orc, "final")


def test_plan_ahead_flags_a_bad_label_only_when_its_step_runs():
    rb = _rb()
    dev = torch.device("cuda:0")
    w = wl.C1
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev)
    x0, y0 = wl.make_batch(w, 0, dev)
    x1, y1 = wl.make_batch(w, 1, dev)
    y1 = torch.full_like(y1, w.K + 5)                  # every candidate of step 1 is out of range
    out_x = torch.empty((w.r, *w.shape), dtype=w.torch_dtype, device=dev)
    out_y = torch.empty(w.r, dtype=torch.int64, device=dev)
    buf.announce_next(y1)
    buf.update_sample(x0, y0, w.c, w.r, 0, 0, out_x, out_y)      # plans step 1, which has the bad labels
    assert buf.read_state()[2] == 0                              # ... but step 1 has not run (and its plan is dropped here)
    buf.announce_next(None)
    buf.update_sample(x1, y1, w.c, w.r, 0, 1, out_x, out_y)
    assert buf.read_state()[2] == rb.RB_FLAG_BAD_LABEL
    # the same through the planned step itself
    buf2 = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev)
    buf2.announce_next(y1)
    buf2.update_sample(x0, y0, w.c, w.r, 0, 0, out_x, out_y)
    buf2.update_sample(x1, y1, w.c, w.r, 0, 1, out_x, out_y)     # moves rows by the plan: none is stored
    fill, last_n, flags = buf2.read_state()
    assert flags == rb.RB_FLAG_BAD_LABEL and int(fill.sum()) == w.c and last_n == min(w.r, w.c)


# ------------------------------------------------ several steps from one call ---

@pytest.mark.parametrize("window", [32, 16, 8, 3, 1])
@pytest.mark.parametrize("w", [
    wl.variant(wl.C2, name="C2-many", S=4),
    wl.variant(wl.C5, name="C5-many", K=300, S=12, shape=(256,), b=512, c=200, r=150),
    wl.variant(wl.C1, name="C1-many-one-class", K=1, S=7, c=16, r=16),     # every step rewrites slots that representatives of the same launch read
    wl.variant(wl.C1, name="C1-many-one-slot", K=2, S=1, c=6, r=2),        # two slots in all: each is read and rewritten in every step
    wl.variant(wl.C4, name="C4-many-S2", S=2, shape=(3, 32, 32)),          # Zipf head: the hot classes' two slots are hit again and again
    wl.variant(wl.C1, name="C1-many", S=20),
], ids=["small", "general", "one-class", "one-slot", "zipf-S2", "C1"])
@pytest.mark.parametrize("planners", [1, 2], ids=["one-planner", "planners-side-by-side"])
def test_many_steps_from_one_call(w, window, planners):
    rb = _rb()
    dev = torch.device("cuda:0")
    n = 36 if window == 32 else 18
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev)
    buf.set_option(rb.RB_OPT_WINDOW, window)
    buf.set_option(rb.RB_OPT_PLANNERS, planners)
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    xs, ys, oxs, oys = [], [], [], []
    for t in range(2 * n):
        x, y = wl.make_batch(w, t, dev)
        xs.append(x.contiguous())
        ys.append(y)
        oxs.append(torch.full((w.r, *w.shape), 3, dtype=w.torch_dtype, device=dev))
        oys.append(torch.full((w.r,), -7, dtype=torch.int64, device=dev))
    # a bad argument anywhere: nothing is enqueued
    broken = list(oxs[:n])
    broken[n - 1] = oxs[n - 1].data_ptr() + 4
    assert rb.rb_update_sample_many(buf.handle, n, xs[:n], ys[:n], w.b, w.c, w.r, w.lib_seed, 0, broken, oys[:n]) == rb.RB_EINVAL
    assert int(buf.read_state()[0].sum()) == 0
    assert rb.rb_update_sample_many(buf.handle, 0, xs[:0], ys[:0], w.b, w.c, w.r, w.lib_seed, 0, oxs[:0], oys[:0]) == rb.RB_OK
    for first in (0, n):
        sl = slice(first, first + n)
        assert rb.rb_update_sample_many(buf.handle, n, xs[sl], ys[sl], w.b, w.c, w.r, w.lib_seed, first, oxs[sl], oys[sl]) == rb.RB_OK
    torch.cuda.synchronize()
    untouched = parity_util._bytes(torch.full((w.r, *w.shape), 3, dtype=w.torch_dtype)).numpy()
    for t in range(2 * n):
        orc.update(parity_util._bytes(xs[t]).cpu().numpy(), ys[t].cpu().numpy(), w.c, w.lib_seed, t)
        nn, ref_x, ref_y = orc.sample_augment(w.r, w.lib_seed, t)
        got_y = oys[t].cpu().numpy()
        assert np.array_equal(got_y, ref_y), f"{w.name} step {t}: labels differ"
        got_x = parity_util._bytes(oxs[t]).cpu().numpy()
        assert np.array_equal(got_x[:nn], ref_x[:nn]), f"{w.name} step {t}: rows differ"
        assert np.array_equal(got_x[nn:], untouched[nn:]), f"{w.name} step {t}: rows beyond n were written"
    compare_buffers(buf, orc, f"{w.name} final")


@pytest.mark.parametrize("announce", [False, True], ids=["plain", "announced"])
@pytest.mark.parametrize("w,steps", [(wl.C3, 72), (wl.C4, 48)], ids=["C3", "C4"])
def test_many_steps_at_full_size(w, steps, announce):
    """The configuration the bench times: real shapes, 32 (C3) or 9 to 10 (C4) steps per launch, calls announced: every
    configured step.  Without the announcement: a shorter run."""
    run_many_parity(w, w.steps if FULL or announce else steps, per_call=64 if announce else 24, announce=announce)


@pytest.mark.parametrize("form", ["u8", "bf16"])
def test_many_steps_at_full_size_with_reduced_storage(form):
    """C3 at its real shape with the rows stored in 8 bits resp. as bfloat16, as the bench's legs run it (announced calls of
    64 steps, 32 steps per launch), 600 steps."""
    run_many_parity(wl.C3, wl.C3.steps if FULL else 600, per_call=64, announce=True, store_u8=form == "u8", store_bf16=form == "bf16")


@pytest.mark.parametrize("w,steps,per_call", [
    (wl.C1, 100, 17),                                                              # fills up: append, replace, collisions
    (wl.C2, 200, 64),
    (wl.variant(wl.C4, name="C4-S8-many", S=8, shape=(3, 32, 32)), 96, 32),        # Zipf head: several overwrites of one class per step
    (wl.variant(wl.C4, name="C4-S1-many", S=1, K=40, shape=(3, 32, 32)), 64, 32),  # 40 slots in all, 64 written and 64 read per step
    (wl.variant(wl.C1, name="C1-r-large-many", S=3, c=16, r=64, b=64), 40, 9),     # r above what is stored, then r = F
    (wl.variant(wl.C2, name="C2-odd-b-many", b=77, c=33, r=21, S=2), 60, 11),
    (wl.variant(wl.C2, name="C2-b1500-many", b=1500, c=40, r=30, S=3, shape=(3, 8, 8)), 40, 17),   # more positions than one selecting wavefront per step gets scratch for
    (wl.variant(wl.C4, name="C4-b2048-many", b=2048, c=64, r=64, S=2, K=1024, shape=(64,)), 32, 16),   # every limit of the several-steps launch at once
    (wl.variant(wl.C1, name="C1-c1-many", c=1, r=1, S=2), 50, 13),
], ids=["C1", "C2", "C4-S8", "C4-S1", "r-large", "odd-b", "b1500", "b2048", "c1"])
def test_many_steps_longer_runs(w, steps, per_call):
    run_many_parity(w, steps, per_call=per_call)


@pytest.mark.parametrize("w,steps,per_call", [
    (wl.C1, 100, 17),
    (wl.C2, 96, 8),                                                                # every call is one launch, planned by the call before
    (wl.variant(wl.C4, name="C4-S8-announced", S=8, shape=(3, 32, 32)), 96, 32),
    (wl.variant(wl.C4, name="C4-S1-announced", S=1, K=40, shape=(3, 32, 32)), 60, 20),
    (wl.variant(wl.C3, name="C3-S4-announced", S=4), 30, 10),                      # full-size rows
    (wl.variant(wl.C5, name="C5-announced", K=300, S=12, shape=(256,), b=512, c=200, r=150), 30, 7),   # steps go out one by one: plan-ahead chain across calls
], ids=["C1", "C2-one-launch", "C4-S8", "C4-S1", "C3-S4", "one-by-one"])
def test_many_steps_with_the_next_call_announced(w, steps, per_call):
    run_many_parity(w, steps, per_call=per_call, announce=True)


@pytest.mark.parametrize("w,steps,per_call,announce", [
    (wl.variant(wl.C1, name="C1-many-bf16"), 100, 17, False),                                  # fills up: append, replace, collisions
    (wl.variant(wl.C1, name="C1-many-bf16-one-class", K=1, S=7, c=16, r=16), 60, 20, True),    # old content handed on by the writers, forwarding
    (wl.variant(wl.C1, name="C1-many-bf16-one-slot", K=2, S=1, c=6, r=2), 48, 16, True),
    (wl.variant(wl.C3, name="C3-many-bf16", K=50, S=6), 36, 18, True),                         # 301 056-byte stored rows, many tiles
    (wl.variant(wl.C2, name="C2-many-bf16", S=3, shape=(3, 8, 8)), 96, 32, True),
], ids=["C1", "one-class", "one-slot", "C3-rows", "C2-S3"])
def test_many_steps_with_float32_samples_stored_as_bfloat16(w, steps, per_call, announce):
    run_many_parity(w, steps, per_call=per_call, announce=announce, store_bf16=True)


@pytest.mark.parametrize("policy", ["exact-fifo", "exact-reservoir"])
@pytest.mark.parametrize("w,steps,per_call", [
    (wl.C1, 100, 17),                                                                           # fills up: every strategy replaces
    (wl.variant(wl.C4, name="C4-S8-many-policy", S=8, shape=(3, 32, 32)), 64, 32),              # Zipf head: many class-mates per step
    (wl.Workload("laps-many", 9, 3, 2, (8,), "f32", 64, 64, 64, 30, "normal", "uniform"), 32, 8),   # ~21 candidates per class into 2 slots: whole rounds within a step
    (wl.variant(wl.C2, name="C2-S3-many-policy", S=3), 96, 16),
    (wl.variant(wl.C1, name="C1-one-class-many-policy", K=1, S=7, c=16, r=16), 48, 16),         # every hazard between the steps of a launch
], ids=["C1", "C4-S8", "laps", "C2-S3", "one-class"])
def test_many_steps_with_other_replacement_strategies(policy, w, steps, per_call):
    run_many_parity(w, steps, per_call=per_call, announce=True, policy=POLICIES[policy])


def test_many_steps_policy_bf16_and_broken_promises_together():
    w = wl.variant(wl.C1, name="C1-many-fifo-bf16-promises", K=4, S=5, c=12, r=12)
    run_many_parity(w, 90, per_call=9, announce=True, schedule_seed=7, store_bf16=True, policy=POLICIES["exact-fifo"])
    run_many_parity(w, 90, per_call=9, announce=True, schedule_seed=8, store_bf16=True, policy=POLICIES["exact-reservoir"])
    # the Bernoulli selection has no bound of 64 on its candidates: the large-count form takes these steps, results unchanged
    run_many_parity(w, 30, per_call=9, announce=True, policy=POLICIES["bernoulli-fifo"])


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_many_steps_announced_survive_broken_promises(seed):
    run_many_parity(wl.variant(wl.C4, name=f"C4-S8-many-promises-{seed}", S=8, shape=(3, 32, 32), b=128, c=40, r=40), 160, per_call=12,
                    announce=True, schedule_seed=seed)
    run_many_parity(wl.variant(wl.C1, name=f"C1-many-promises-{seed}"), 120, per_call=9, announce=True, schedule_seed=seed + 10)


def test_an_announced_call_that_never_comes_is_forgotten():
    """Labels of a next call are announced and planned, then single steps come instead."""
    rb = _rb()
    dev = torch.device("cuda:0")
    w = wl.C1
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev)
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    batches = [wl.make_batch(w, t, dev) for t in range(20)]
    xs, ys = [x.contiguous() for x, _ in batches], [y.contiguous() for _, y in batches]
    oxs = [torch.empty((w.r, *w.shape), dtype=w.torch_dtype, device=dev) for _ in range(20)]
    oys = [torch.empty(w.r, dtype=torch.int64, device=dev) for _ in range(20)]
    buf.announce_next_many(ys[6:12])
    buf.update_sample_many(xs[:6], ys[:6], w.c, w.r, w.lib_seed, 0, oxs[:6], oys[:6])       # plans steps 6.. as well
    buf.update_sample(xs[6], ys[6], w.c, w.r, w.lib_seed, 6, oxs[6], oys[6])               # a single step instead
    buf.announce_next_many(ys[7:9])                                                        # announced, but the wrong call follows
    buf.update(xs[7], ys[7], w.c, w.lib_seed, 7)
    buf.sample_augment(w.r, w.lib_seed, 7, oxs[7], oys[7])
    buf.update_sample_many(xs[8:14], ys[8:14], w.c, w.r, w.lib_seed, 8, oxs[8:14], oys[8:14])
    buf.announce_next_many(ys[14:20])
    buf.update_sample_many(xs[14:14], ys[14:14], w.c, w.r, w.lib_seed, 14, oxs[14:14], oys[14:14])   # no steps: the announcement is spent
    buf.update_sample_many(xs[14:20], ys[14:20], w.c, w.r, w.lib_seed, 14, oxs[14:20], oys[14:20])
    torch.cuda.synchronize()
    for t in range(20):
        orc.update(parity_util._bytes(xs[t]).cpu().numpy(), ys[t].cpu().numpy(), w.c, w.lib_seed, t)
        n, ref_x, ref_y = orc.sample_augment(w.r, w.lib_seed, t)
        assert np.array_equal(oys[t].cpu().numpy(), ref_y), f"step {t}: labels differ"
        assert np.array_equal(parity_util._bytes(oxs[t]).cpu().numpy()[:n], ref_x[:n]), f"step {t}: rows differ"
    compare_buffers(buf, orc, "final")


@pytest.mark.parametrize("window", [32, 16, 8, 4, 2])
@pytest.mark.parametrize("planners", [1, 2], ids=["one-planner", "planners-side-by-side"])
def test_many_steps_with_every_hazard_between_the_steps_of_one_launch(window, planners):
    """Eight classes of one slot each, every step samples all eight rows and rewrites one class (the label
    sequence decides which): rows that are read before a later step of the same launch overwrites them, rows
    that are read after an earlier step wrote them, rows written twice."""
    rb = _rb()
    dev = torch.device("cuda:0")
    K, S, b, c, r = 8, 1, 4, 4, 8
    shape = (3, 40)                                     # 480-byte rows
    buf = rb.RehearsalBuffer(K, S, shape, torch.float32, device=dev)
    buf.set_option(rb.RB_OPT_WINDOW, window)
    buf.set_option(rb.RB_OPT_PLANNERS, planners)
    orc = rbo.Buffer(K, S, 480)
    sequence = list(range(8)) + [7, 6, 5, 4, 3, 2, 1, 0] + [0, 0, 1, 1, 0, 2, 2, 0] + [5, 5, 5, 5, 5, 5, 5, 5] + [3, 4, 3, 4, 3, 4, 3, 4]
    g = torch.Generator(device="cpu")
    g.manual_seed(99)
    xs = [torch.randn((b, *shape), generator=g).to(dev) for _ in sequence]
    ys = [torch.full((b,), k, dtype=torch.int64, device=dev) for k in sequence]
    oxs = [torch.zeros((r, *shape), device=dev) for _ in sequence]
    oys = [torch.full((r,), -7, dtype=torch.int64, device=dev) for _ in sequence]
    per = max(8, window)
    for first in range(0, len(sequence), per):
        sl = slice(first, first + per)
        n = len(xs[sl])
        assert rb.rb_update_sample_many(buf.handle, n, xs[sl], ys[sl], b, c, r, 3, first, oxs[sl], oys[sl]) == rb.RB_OK
    torch.cuda.synchronize()
    for t, k in enumerate(sequence):
        orc.update(parity_util._bytes(xs[t]).cpu().numpy(), ys[t].cpu().numpy(), c, 3, t)
        n, ref_x, ref_y = orc.sample_augment(r, 3, t)
        assert np.array_equal(oys[t].cpu().numpy(), ref_y), f"step {t}: labels differ"
        assert np.array_equal(parity_util._bytes(oxs[t]).cpu().numpy()[:n], ref_x[:n]), f"step {t}: rows differ"
    compare_buffers(buf, orc, "final")


# ------------------------- several steps per launch with large counts (1024-thread planners side by side) ---

@pytest.mark.parametrize("window", [16, 11, 5, 2])
@pytest.mark.parametrize("w,policy,bf16", [
    (wl.variant(wl.C5, name="bw-two-classes", K=2, S=40, shape=(64,), b=256, c=100, r=70), None, False),        # 80 slots in all: every step reads and rewrites most of them
    (wl.variant(wl.C5, name="bw-one-class", K=1, S=150, shape=(32,), b=300, c=120, r=150), None, False),        # r = everything stored: every slot is read in every step
    (wl.variant(wl.C5, name="bw-K300", K=300, S=12, shape=(256,), b=512, c=200, r=150), None, False),           # fills up, then replaces
    (wl.variant(wl.C5, name="bw-K300-fifo", K=300, S=12, shape=(256,), b=512, c=200, r=150), "exact-fifo", False),
    (wl.variant(wl.C5, name="bw-K40-reservoir", K=40, S=10, shape=(64,), b=512, c=200, r=150), "exact-reservoir", False),
    (wl.variant(wl.C5, name="bw-two-classes-bf16", K=2, S=40, shape=(64,), b=256, c=100, r=70), None, True),    # old content handed on through the conversion
    (wl.variant(wl.C5, name="bw-K300-bf16-fifo", K=300, S=12, shape=(264,), b=512, c=200, r=150), "exact-fifo", True),
    (wl.variant(wl.C5, name="bw-K300-bernoulli", K=300, S=12, shape=(256,), b=1024, c=400, r=150), "bernoulli-uniform", False),   # the largest mini-batch the Bernoulli selection may have here
    (wl.variant(wl.C4, name="bw-C4-S8-bernoulli", S=8, shape=(3, 32, 32)), "bernoulli-uniform", False),        # small counts: the small form does not take this selection
    (wl.variant(wl.C1, name="bw-C1-bernoulli-fifo", S=5), "bernoulli-fifo", False),                             # about 4 of 16 positions; fills up, replaces
    (wl.variant(wl.C5, name="bw-two-classes-bernoulli-reservoir-bf16", K=2, S=40, shape=(64,), b=256, c=100, r=70), "bernoulli-reservoir", True),
    (wl.variant(wl.C1, name="bw-c-equals-b-bernoulli", b=64, c=64, r=20, S=3), "bernoulli-uniform", False),     # every coin shows heads
    (wl.variant(wl.C2, name="bw-K1100-few", K=1100, S=2), None, False),                                         # few candidates, too many classes for the small form
    (wl.variant(wl.C5, name="bw-limits", K=10240, S=3, shape=(16,), b=4096, c=1024, r=1024), None, False),      # every limit at once
], ids=lambda v: v.name if hasattr(v, "name") else None)
def test_many_steps_with_large_counts(w, policy, bf16, window):
    """rb_update_sample_many for shapes beyond the small several-steps form: up to 16 steps per launch, planned by
    two 1024-thread workgroups per step that settle between them what the steps do to each other's slots."""
    rb = _rb()
    pol = POLICIES[policy] if policy else None
    run_many_parity(w, 40, per_call=19, window=window, policy=pol, store_bf16=bf16)
    run_many_parity(w, 40, per_call=16, window=window, announce=True, policy=pol, store_bf16=bf16)
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, store_dtype=torch.bfloat16 if bf16 else None)
    if pol:
        buf.set_policy(*pol)
    buf.set_option(rb.RB_OPT_WINDOW, window)
    assert buf.steps_per_launch(w.b, w.c, w.r) == window


@pytest.mark.parametrize("seed", [1, 2])
def test_many_steps_with_large_counts_survive_broken_promises(seed):
    run_many_parity(wl.variant(wl.C5, name=f"bw-promises-{seed}", K=30, S=12, shape=(64,), b=512, c=200, r=150), 160, per_call=12,
                    announce=True, schedule_seed=seed)
    run_many_parity(wl.variant(wl.C4, name=f"bw-promises-bernoulli-{seed}", S=8, shape=(3, 32, 32), b=128, c=40, r=40), 120, per_call=12,
                    announce=True, schedule_seed=seed + 20, policy=POLICIES["bernoulli-uniform"])


def test_many_steps_with_large_counts_drop_and_flag_bad_labels():
    rb = _rb()
    dev = torch.device("cuda:0")
    K, S, b, c, r, n = 1500, 2, 200, 150, 90, 14
    buf = rb.RehearsalBuffer(K, S, (8,), torch.float32, device=dev)
    assert buf.steps_per_launch(b, c, r) == 16
    orc = rbo.Buffer(K, S, 32)
    g = torch.Generator(device="cpu")
    g.manual_seed(6)
    xs = [torch.randn((b, 8), generator=g).to(dev) for _ in range(n)]
    ys = [torch.randint(0, K, (b,), generator=g, dtype=torch.int64) for _ in range(n)]
    ys[5][::3] = -1
    ys[9][1::4] = K
    ys[9][5] = 10**12
    ys = [y.to(dev) for y in ys]
    oxs = [torch.zeros((r, 8), device=dev) for _ in range(n)]
    oys = [torch.full((r,), -7, dtype=torch.int64, device=dev) for _ in range(n)]
    buf.update_sample_many(xs[:4], ys[:4], c, r, 21, 0, oxs[:4], oys[:4])
    assert buf.read_state()[2] == 0
    buf.update_sample_many(xs[4:], ys[4:], c, r, 21, 4, oxs[4:], oys[4:])
    torch.cuda.synchronize()
    for t in range(n):
        orc.update(parity_util._bytes(xs[t]).cpu().numpy(), ys[t].cpu().numpy(), c, 21, t)
        m, ref_x, ref_y = orc.sample_augment(r, 21, t)
        assert np.array_equal(oys[t].cpu().numpy(), ref_y), f"step {t}: labels differ"
        assert np.array_equal(parity_util._bytes(oxs[t]).cpu().numpy()[:m], ref_x[:m]), f"step {t}: rows differ"
    assert buf.read_state()[2] == rb.RB_FLAG_BAD_LABEL == orc.flags
    compare_buffers(buf, orc, "bad labels, large counts, several steps per launch")


@pytest.mark.parametrize("w", [wl.C5, wl.C5F], ids=["C5", "C5F"])
def test_many_steps_with_large_counts_at_full_size(w):
    """C5 and its variant with a fixed set of active classes in the form the bench times them in: announced
    rb_update_sample_many calls, 16 steps per launch, every configured step."""
    run_many_parity(w, w.steps, per_call=32, announce=True)


@pytest.mark.parametrize("planners", [1, 2], ids=["one-planner", "planners-side-by-side"])
def test_many_steps_drop_and_flag_bad_labels(planners):
    """Labels outside [0, K) among the candidates of steps in the middle of a launch: not stored, flag raised."""
    rb = _rb()
    dev = torch.device("cuda:0")
    K, S, b, c, r, n = 5, 3, 12, 12, 6, 16
    buf = rb.RehearsalBuffer(K, S, (8,), torch.float32, device=dev)
    buf.set_option(rb.RB_OPT_PLANNERS, planners)
    orc = rbo.Buffer(K, S, 32)
    g = torch.Generator(device="cpu")
    g.manual_seed(5)
    xs = [torch.randn((b, 8), generator=g).to(dev) for _ in range(n)]
    ys = [torch.randint(0, K, (b,), generator=g, dtype=torch.int64) for _ in range(n)]
    ys[3][::3] = -1
    ys[9][1::4] = K
    ys[10][5] = 10**12
    ys = [y.to(dev) for y in ys]
    oxs = [torch.zeros((r, 8), device=dev) for _ in range(n)]
    oys = [torch.full((r,), -7, dtype=torch.int64, device=dev) for _ in range(n)]
    buf.update_sample_many(xs[:3], ys[:3], c, r, 11, 0, oxs[:3], oys[:3])
    assert buf.read_state()[2] == 0
    buf.update_sample_many(xs[3:], ys[3:], c, r, 11, 3, oxs[3:], oys[3:])
    torch.cuda.synchronize()
    for t in range(n):
        orc.update(parity_util._bytes(xs[t]).cpu().numpy(), ys[t].cpu().numpy(), c, 11, t)
        m, ref_x, ref_y = orc.sample_augment(r, 11, t)
        assert np.array_equal(oys[t].cpu().numpy(), ref_y), f"step {t}: labels differ"
        assert np.array_equal(parity_util._bytes(oxs[t]).cpu().numpy()[:m], ref_x[:m]), f"step {t}: rows differ"
    assert buf.read_state()[2] == rb.RB_FLAG_BAD_LABEL == orc.flags
    compare_buffers(buf, orc, "bad labels in a window")


# ----------------------------------------- the asynchronous primitive (Sec. IV-D) ---

@pytest.mark.parametrize("w,steps", [
    (wl.variant(wl.C2, name="C2-pipeline", S=6), 60),                                      # fused single launch
    (wl.variant(wl.C5, name="C5-pipeline", K=300, S=12, shape=(256,), b=512, c=200, r=150), 25),   # two general kernels
], ids=["small", "general"])
def test_pipelined_primitive_returns_the_previous_iterations_representatives(w, steps):
    """Iteration t trains on the representatives that iteration t-1 started to collect, while the
    update with mini-batch t and the next sampling run on the buffer's stream under a stand-in
    for the training computation."""
    rb = _rb()
    dev = torch.device("cuda:0")
    side = torch.cuda.Stream(dev)
    train = torch.cuda.current_stream(dev)
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev, stream=side)
    pipe = rb.Pipeline(buf)
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    aug_x = torch.empty((2, w.b + w.r, *w.shape), dtype=w.torch_dtype, device=dev)    # two augmented mini-batches in turn
    aug_y = torch.empty((2, w.b + w.r), dtype=torch.int64, device=dev)
    sink = torch.empty(64 * 256, dtype=torch.float32, device=dev)
    want = None                                     # what the oracle sampled in the previous iteration
    for t in range(steps + 1):
        cur, nxt = t % 2, (t + 1) % 2
        if t < steps:
            x, y = wl.make_batch(w, t, dev)             # produced on the training stream
            aug_x[cur, :w.b].copy_(x)
            aug_y[cur, :w.b].copy_(y)
            # the tail of the NEXT augmented mini-batch receives this iteration's sampling
            parity_util._bytes(aug_x[nxt, w.b:]).fill_(parity_util.SENTINEL)
            aug_y[nxt, w.b:].fill_(-7)
            rows = pipe.step(aug_x[cur, :w.b], aug_y[cur, :w.b], w.c, w.r, w.lib_seed, t,
                             aug_x[nxt, w.b:], aug_y[nxt, w.b:], train_stream=train)
            assert rb.rb_standin_compute(train, sink, 64, 2000) == rb.RB_OK     # "forward and backward pass"
        else:
            rows = pipe.drain(train)
        assert rows == (0 if t == 0 else w.r)
        if t > 0:
            # ordered on the training stream after the wait that the call enqueued
            got_y = aug_y[cur, w.b:].cpu().numpy()
            got_x = parity_util._bytes(aug_x[cur, w.b:]).cpu().numpy()
            n, ref_x, ref_y = want
            assert np.array_equal(got_y, ref_y), f"{w.name} iteration {t}: labels of the representatives differ"
            assert np.array_equal(got_x, ref_x), f"{w.name} iteration {t}: representatives differ (n={n})"
        if t < steps:
            hx = parity_util._bytes(aug_x[cur, :w.b]).cpu().numpy()
            hy = aug_y[cur, :w.b].cpu().numpy()
            orc.update(hx, hy, w.c, w.lib_seed, t)
            ref = np.full((w.r, w.row_bytes), parity_util.SENTINEL, dtype=np.uint8)
            want = orc.sample_augment(w.r, w.lib_seed, t, out_x=ref)
    compare_buffers(buf, orc, f"{w.name} final")
    pipe.close()


@pytest.mark.parametrize("w,steps,group,announce", [
    (wl.variant(wl.C2, name="C2-pipeline-many", S=6), 64, 16, True),                            # 16 steps per launch, planned by the call before
    (wl.variant(wl.C3, name="C3-pipeline-many", K=50, S=6), 40, 8, True),                       # full-size rows; windows of 8
    (wl.variant(wl.C4, name="C4-pipeline-many", S=2, shape=(3, 32, 32)), 30, 7, False),         # every call plans its own first window
    (wl.variant(wl.C5, name="C5-pipeline-many", K=300, S=12, shape=(256,), b=512, c=200, r=150), 24, 6, True),   # steps go out one by one
], ids=["C2", "C3-rows", "C4-S2", "one-by-one"])
def test_pipelined_primitive_with_several_iterations_per_call(w, steps, group, announce):
    """One rb_pipeline_step_many call per `group` training iterations: the first iteration of a group trains (a
    stand-in) while the group's launch runs on the buffer's stream, the others after rb_pipeline_drain; every
    iteration must see exactly the representatives that the step before it sampled."""
    rb = _rb()
    dev = torch.device("cuda:0")
    side = torch.cuda.Stream(dev)
    train = torch.cuda.current_stream(dev)
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev, stream=side)
    pipe = rb.Pipeline(buf)
    orc = rbo.Buffer(w.K, w.S, w.row_bytes)
    # one augmented mini-batch per iteration (the data pipeline is `group` iterations ahead, and one group more when it announces)
    aug_x = torch.empty((steps + 1, w.b + w.r, *w.shape), dtype=w.torch_dtype, device=dev)
    aug_y = torch.empty((steps + 1, w.b + w.r), dtype=torch.int64, device=dev)
    sink = torch.empty(64 * 256, dtype=torch.float32, device=dev)
    produced = 0

    def produce(upto):
        nonlocal produced
        for t in range(produced, min(upto, steps)):
            x, y = wl.make_batch(w, t, dev)
            aug_x[t, :w.b].copy_(x)
            aug_y[t, :w.b].copy_(y)
            parity_util._bytes(aug_x[t + 1, w.b:]).fill_(parity_util.SENTINEL)     # where iteration t's sampling goes
            aug_y[t + 1, w.b:].fill_(-7)
        produced = max(produced, min(upto, steps))

    want = {}

    def check(t):
        """Iteration t reads its representatives on the training stream."""
        if t == 0:
            return
        n, ref_x, ref_y = want.pop(t)
        assert np.array_equal(aug_y[t, w.b:].cpu().numpy(), ref_y), f"{w.name} iteration {t}: labels of the representatives differ"
        assert np.array_equal(parity_util._bytes(aug_x[t, w.b:]).cpu().numpy(), ref_x), f"{w.name} iteration {t}: representatives differ (n={n})"

    for g in range(0, steps, group):
        n = min(group, steps - g)
        produce(g + n + (group if announce else 0))
        if announce and g + n < steps:
            buf.announce_next_many([aug_y[t, :w.b] for t in range(g + n, min(g + 2 * n, steps))][:16])
        ts = range(g, g + n)
        rows = pipe.step_many([aug_x[t, :w.b] for t in ts], [aug_y[t, :w.b] for t in ts], w.c, w.r, w.lib_seed, g,
                              [aug_x[t + 1, w.b:] for t in ts], [aug_y[t + 1, w.b:] for t in ts], train_stream=train)
        assert rows == (0 if g == 0 else w.r)
        assert rb.rb_standin_compute(train, sink, 64, 2000) == rb.RB_OK     # iteration g's "forward and backward pass"
        check(g)
        for t in ts:
            orc.update(parity_util._bytes(aug_x[t, :w.b]).cpu().numpy(), aug_y[t, :w.b].cpu().numpy(), w.c, w.lib_seed, t)
            ref = np.full((w.r, w.row_bytes), parity_util.SENTINEL, dtype=np.uint8)
            want[t + 1] = orc.sample_augment(w.r, w.lib_seed, t, out_x=ref)
        assert pipe.drain(train) == w.r
        for t in range(g + 1, g + n):
            assert rb.rb_standin_compute(train, sink, 64, 500) == rb.RB_OK
            check(t)
    check(steps)                                    # what the last step sampled (drained above)
    compare_buffers(buf, orc, f"{w.name} final")
    # argument checks: nothing enqueued, pipeline unchanged
    bad = [aug_x[0, :w.b], aug_x[1, :w.b].data_ptr() + 4]
    rc, _ = rb.rb_pipeline_step_many(pipe.handle, 2, bad, [aug_y[0, :w.b], aug_y[1, :w.b]], w.b, w.c, w.r, w.lib_seed, steps,
                                     [aug_x[1, w.b:], aug_x[2, w.b:]], [aug_y[1, w.b:], aug_y[2, w.b:]], train)
    assert rc == rb.RB_EINVAL
    assert rb.rb_pipeline_step_many(pipe.handle, 0, [], [], w.b, w.c, w.r, w.lib_seed, steps, [], [], train) == (rb.RB_OK, w.r)
    assert rb.rb_pipeline_step_many(None, 0, [], [], w.b, w.c, w.r, w.lib_seed, steps, [], [], train)[0] == rb.RB_EINVAL
    torch.cuda.synchronize()
    compare_buffers(buf, orc, f"{w.name} after rejected calls")
    pipe.close()


def test_moved_rows_counter_counts_stored_candidates_and_representatives():
    """rb_read_moved_rows against the oracle's record of every step, through each family of kernels."""
    rb = _rb()
    dev = torch.device("cuda:0")
    for w, style in [(wl.variant(wl.C1, name="C1-moved"), "two"), (wl.variant(wl.C1, name="C1-moved-single"), "single"),
                     (wl.variant(wl.C1, name="C1-moved-ahead"), "ahead"), (wl.variant(wl.C1, name="C1-moved-many"), "many"),
                     (wl.variant(wl.C5, name="C5-moved", K=20, S=8, shape=(64,), b=512, c=200, r=150), "two"),
                     (wl.variant(wl.C5, name="C5-moved-ahead", K=20, S=8, shape=(64,), b=512, c=200, r=150), "ahead")]:
        buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev)
        orc = rbo.Buffer(w.K, w.S, w.row_bytes)
        steps = 48
        batches = [wl.make_batch(w, t, dev) for t in range(steps + 1)]
        xs, ys = [x.contiguous() for x, _ in batches], [y.contiguous() for _, y in batches]
        oxs = [torch.empty((w.r, *w.shape), dtype=w.torch_dtype, device=dev) for _ in range(steps)]
        oys = [torch.empty(w.r, dtype=torch.int64, device=dev) for _ in range(steps)]
        expect = 0
        for t in range(steps):
            orc.update(parity_util._bytes(xs[t]).cpu().numpy(), ys[t].cpu().numpy(), w.c, w.lib_seed, t)
            pos, cls, slot = orc.last_insertions()
            expect += len(set(zip(cls.tolist(), slot.tolist())))      # of the insertions into one slot only the last is moved
            expect += orc.sample_augment(w.r, w.lib_seed, t)[0]
        if style == "many":
            for first in range(0, steps, 16):
                buf.update_sample_many(xs[first:first + 16], ys[first:first + 16], w.c, w.r, w.lib_seed, first, oxs[first:first + 16], oys[first:first + 16])
        else:
            for t in range(steps):
                if style == "two":
                    buf.update(xs[t], ys[t], w.c, w.lib_seed, t)
                    buf.sample_augment(w.r, w.lib_seed, t, oxs[t], oys[t])
                else:
                    if style == "ahead":
                        buf.announce_next(ys[t + 1])
                    buf.update_sample(xs[t], ys[t], w.c, w.r, w.lib_seed, t, oxs[t], oys[t])
        if style == "many":
            # within a launch of several steps a slot written twice is moved once, and the oracle's per-step count is an upper bound
            assert buf.moved_rows() <= expect, (w.name, style)
            assert buf.moved_rows() >= expect - steps * w.c
        else:
            assert buf.moved_rows() == expect, (w.name, style, buf.moved_rows(), expect)
        assert rb.rb_read_moved_rows(None)[0] == rb.RB_EINVAL


def test_pipeline_argument_checks_leave_it_unchanged():
    rb = _rb()
    w = wl.C1
    dev = torch.device("cuda:0")
    buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev, stream=torch.cuda.Stream(dev))
    rc, p = rb.rb_pipeline_create(buf.handle)
    assert rc == rb.RB_OK
    assert rb.rb_pipeline_create(None)[0] == rb.RB_EINVAL
    x, y = wl.make_batch(w, 0, dev)
    out_x = torch.empty((w.r, *w.shape), dtype=w.torch_dtype, device=dev)
    out_y = torch.empty(w.r, dtype=torch.int64, device=dev)
    assert rb.rb_pipeline_step(p, x, y, w.b, w.b + 1, w.r, 0, 0, out_x, out_y)[0] == rb.RB_EINVAL
    assert rb.rb_pipeline_step(p, x, y, w.b, w.c, w.r, 0, 0, None, out_y)[0] == rb.RB_EINVAL
    assert rb.rb_pipeline_drain(p) == (rb.RB_OK, 0)                      # nothing was started
    assert rb.rb_pipeline_step(p, x, y, w.b, w.c, w.r, 0, 0, out_x, out_y) == (rb.RB_OK, 0)
    assert rb.rb_pipeline_step(p, x, y, w.b, w.c, 3, 0, 1, out_x, out_y) == (rb.RB_OK, w.r)
    assert rb.rb_pipeline_drain(p) == (rb.RB_OK, 3)
    torch.cuda.synchronize()
    assert rb.rb_pipeline_destroy(p) == rb.RB_OK
    assert rb.rb_pipeline_destroy(None) == rb.RB_EINVAL


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


def _random_planned_workload(rng, i):
    """Shapes around the limits of the plan-ahead forms: at most 64 / 1024 candidates and representatives,
    1024 / 10240 classes, mini-batches of 2048 / 4096."""
    kind = rng.choice(["small", "large", "any"])
    if kind == "small":
        b = int(rng.choice([1, 5, 64, 65, 700, 2048, 2049]))
        c, r = int(min(b, rng.integers(1, 66))), int(rng.integers(1, 66))
        K = int(rng.choice([1, 3, 50, 1000, 1024, 1025]))
    elif kind == "large":
        b = int(rng.choice([100, 1024, 1500, 4096]))
        c, r = int(min(b, rng.integers(1, 1100))), int(rng.integers(1, 1100))
        K = int(rng.choice([1, 40, 1025, 5000, 10240, 10241]))
    else:
        b = int(rng.integers(1, 4097))
        c, r = int(rng.integers(0, b + 1)), int(rng.integers(0, 1500))
        K = int(rng.choice([2, 100, 3000, 20000]))
    S = int(rng.choice([1, 2, 3, 10, 60]))
    vecs = int(rng.choice([1, 2, 64, 65, 257, 1000]))        # 16-byte vectors per row
    dtype = "f32" if rng.random() < 0.5 else "bf16"
    shape = (vecs * (4 if dtype == "f32" else 8),)
    labels = str(rng.choice(["uniform", "zipf", "active50"]))
    return wl.Workload(f"randp{i}-{kind}-K{K}-S{S}-b{b}-c{c}-r{r}-v{vecs}", 9, K, S, shape, dtype, b, c, r, 6, "normal", labels)


@pytest.mark.parametrize("chunk", range(6))
def test_random_configurations_planned_ahead(chunk):
    """Seeded random shapes through the calls that plan ahead: one announced step at a time, and several steps
    per call (with and without the next call announced, sometimes with promises broken)."""
    rb = _rb()
    rng = np.random.default_rng(2000 + chunk)
    for i in range(10):
        w = _random_planned_workload(rng, chunk * 100 + i)
        style = str(rng.choice(["ahead", "ahead-broken", "many", "many-announced", "many-broken"]))
        per_call = int(rng.choice([3, 8, 17, 33]))
        options = ((rb.RB_OPT_UNROLL, int(rng.choice([0, 1, 2, 4, 8]))), (rb.RB_OPT_NONTEMPORAL, int(rng.integers(0, 2))),
                   (rb.RB_OPT_WINDOW, int(rng.choice([32, 32, 16, 7, 2, 1]))), (rb.RB_OPT_FUSE, int(rng.choice([1, 1, 1, 0]))),
                   (rb.RB_OPT_PLANNERS, int(rng.choice([0, 1, 2]))))
        print(f"  {w.name} {style} per_call={per_call} options={[v for _, v in options]}", flush=True)
        policy = POLICIES[str(rng.choice(sorted(POLICIES)))] if rng.random() < 0.5 else None
        bf16 = bool(rng.random() < 0.4 and w.dtype == "f32" and (w.row_bytes // 2) % 16 == 0)   # binary32 samples stored as bfloat16
        if style == "ahead":
            run_ahead_parity(w, 8, policy=policy, options=options, store_bf16=bf16)
        elif style == "ahead-broken":
            run_ahead_parity(w, 12, schedule_seed=int(rng.integers(1, 1000)), policy=policy, options=options, store_bf16=bf16)
        elif style == "many":
            run_many_parity(w, 40, per_call=per_call, policy=policy, options=options, store_bf16=bf16)
        elif style == "many-announced":
            run_many_parity(w, 40, per_call=per_call, announce=True, policy=policy, options=options, store_bf16=bf16)
        else:
            run_many_parity(w, 40, per_call=per_call, announce=True, schedule_seed=int(rng.integers(1, 1000)), policy=policy, options=options,
                            store_bf16=bf16)


# ------------------------------------------- two buffers at the same time ---

def test_two_buffers_on_two_streams_do_not_disturb_each_other():
    """Two handles of different shape, each on a stream of its own, enqueued alternately with no host
    synchronisation until the end: every handle has its own workspace and plans, the library keeps no
    state outside them."""
    rb = _rb()
    from oracle import rbo
    from parity_util import _bytes, compare_buffers
    dev = torch.device("cuda:0")
    wa = wl.variant(wl.C3, name="two-a", K=40, S=3, shape=(3, 32, 32))                               # several steps per launch
    wb = wl.variant(wl.C5, name="two-b", K=300, S=4, shape=(256,), b=512, c=200, r=150)              # large-count launches
    sides = []
    for w in (wa, wb):
        st = torch.cuda.Stream(dev)
        buf = rb.RehearsalBuffer(w.K, w.S, w.shape, w.torch_dtype, device=dev, stream=st)
        steps, per_call = 36, 12
        batches = [wl.make_batch(w, t, dev) for t in range(steps)]
        xs, ys = [x.contiguous() for x, _ in batches], [y.contiguous() for _, y in batches]
        oxs = [torch.full((w.r, *w.shape), 3, dtype=w.torch_dtype, device=dev) for _ in range(steps)]
        oys = [torch.full((w.r,), -7, dtype=torch.int64, device=dev) for _ in range(steps)]
        sides.append((w, st, buf, xs, ys, oxs, oys, steps, per_call))
    torch.cuda.synchronize()
    for first in range(0, 36, 12):
        for w, st, buf, xs, ys, oxs, oys, steps, per_call in sides:
            nxt = ys[first + per_call:first + 2 * per_call]
            if nxt:
                buf.announce_next_many(nxt)
            buf.update_sample_many(xs[first:first + per_call], ys[first:first + per_call], w.c, w.r, w.lib_seed, first,
                                   oxs[first:first + per_call], oys[first:first + per_call])
    torch.cuda.synchronize()
    for w, st, buf, xs, ys, oxs, oys, steps, per_call in sides:
        orc = rbo.Buffer(w.K, w.S, w.row_bytes)
        for t in range(steps):
            orc.update(_bytes(xs[t]).cpu().numpy(), ys[t].cpu().numpy(), w.c, w.lib_seed, t)
            ref = _bytes(torch.full((w.r, *w.shape), 3, dtype=w.torch_dtype)).numpy().copy()
            n, ref_x, ref_y = orc.sample_augment(w.r, w.lib_seed, t, out_x=ref)
            assert np.array_equal(oys[t].cpu().numpy(), ref_y), f"{w.name} step {t}: out_y differs"
            assert np.array_equal(_bytes(oxs[t]).cpu().numpy(), ref_x), f"{w.name} step {t}: out_x differs (n={n})"
        compare_buffers(buf, orc, f"{w.name} final")
        buf.close()


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
        for nt in (0, 1, 2):
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
