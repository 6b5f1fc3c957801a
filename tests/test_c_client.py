"""The C ABI from C: a small client compiled with gcc against include/rb.h and linked to the built library
(host-side calls only: create, sizes, option and policy setters, the launch-size query, error strings; no GPU
needed), and, on a GPU, tests/c_client/rb_client.c: a C program with its own device memory that runs a whole
workload through the library and whose dump is compared with the oracle."""
import os
import subprocess
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB_DIR = os.path.join(ROOT, "paper_2406_03285_amd")

CLIENT = textwrap.dedent(r"""
    #include <stdio.h>
    #include <stdint.h>
    #include "rb.h"

    int main(void)
    {
        rb_buffer *rb = NULL;
        const int64_t shape[3] = {3, 224, 224};
        static int64_t fake[4] __attribute__((aligned(16)));     /* stands for device memory: never dereferenced by these calls */
        size_t xb = 0, yb = 0, wb = 0;
        int64_t steps = 0;
        if (rb_create(&rb, 1000, 130, shape, 3, RB_F32) != RB_OK || !rb) return 1;
        if (rb_query_sizes(rb, &xb, &yb, &wb) != RB_OK) return 2;
        if (xb != (size_t)1000 * 130 * 602112 || yb != (size_t)1000 * 130 * 8 || wb == 0 || wb % 256 != 0) return 3;
        if (rb_query_steps_per_launch(rb, 64, 8, 8, &steps) != RB_OK || steps != 32) return 4;
        if (rb_set_option(rb, RB_OPT_WINDOW, 4) != RB_OK) return 5;
        if (rb_query_steps_per_launch(rb, 64, 8, 8, &steps) != RB_OK || steps != 4) return 6;
        if (rb_set_policy(rb, RB_SELECT_EXACT, RB_EVICT_RESERVOIR) != RB_OK) return 7;
        if (rb_update(rb, fake, fake, 8, 2, 0, 0) != RB_ESTATE) return 8;            /* nothing bound yet */
        if (rb_update(rb, NULL, NULL, 8, 2, 0, 0) != RB_EINVAL) return 9;
        if (rb_create(&rb, 0, 1, shape, 3, RB_F32) != RB_EINVAL) return 10;          /* rb is reset to NULL */
        if (rb != NULL) return 11;
        if (!rb_strerror(RB_EINVAL) || !rb_strerror(RB_OK)) return 12;
        printf("c client ok\n");
        return 0;
    }
""")


def test_a_c_program_can_use_the_library(tmp_path):
    lib = os.path.join(LIB_DIR, "librb.so")
    assert os.path.exists(lib), "build the library first"
    src = tmp_path / "client.c"
    src.write_text(CLIENT)
    exe = tmp_path / "client"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", LIB_DIR, "-lrb", "-Wl,-rpath," + LIB_DIR], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, (out.returncode, out.stdout, out.stderr)
    assert "c client ok" in out.stdout


@pytest.mark.gpu
@pytest.mark.parametrize("K,S,vecs,b,c,r,steps", [
    (10, 20, 768, 16, 4, 4, 100),          # the tiny workload's shape: fills up, replaces, collides
    (3, 4, 5, 64, 40, 30, 24),             # few slots: every step overwrites, r above what is stored at first
], ids=["C1-shape", "crowded"])
def test_a_c_program_drives_the_gpu_path(tmp_path, K, S, vecs, b, c, r, steps):
    import numpy as np
    from oracle import rbo
    exe = os.path.join(ROOT, "tests", "c_client", "rb_client")
    assert os.path.exists(exe), "build first (python __graft_entry__.py): the client is compiled with the library"
    row_bytes, seed = 16 * vecs, 17
    rng = np.random.default_rng(K * 1000 + S)
    xs = rng.integers(0, 256, (steps, b, row_bytes), dtype=np.uint8)
    ys = rng.integers(0, K, (steps, b)).astype(np.int64)
    ys[steps // 3, :] = K + 2                       # labels outside [0, K): every candidate of this step is dropped and flagged
    with open(tmp_path / "in.bin", "wb") as f:
        f.write(np.array([K, S, row_bytes, b, c, r, steps, seed], dtype=np.int64).tobytes())
        for t in range(steps):
            f.write(xs[t].tobytes())
            f.write(ys[t].tobytes())
    out = subprocess.run([exe, str(tmp_path / "in.bin"), str(tmp_path / "out.bin")], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, (out.returncode, out.stdout, out.stderr)
    data = np.fromfile(tmp_path / "out.bin", dtype=np.uint8)
    orc = rbo.Buffer(K, S, row_bytes)
    at = 0
    n = 0
    for t in range(steps):
        orc.update(xs[t], ys[t], c, seed, t)
        ref = np.full((r, row_bytes), 0x5A, dtype=np.uint8)
        n, ref_x, ref_y = orc.sample_augment(r, seed, t, out_x=ref)
        got_y = data[at:at + 8 * r].view(np.int64)
        at += 8 * r
        got_x = data[at:at + r * row_bytes].reshape(r, row_bytes)
        at += r * row_bytes
        assert np.array_equal(got_y, ref_y), f"step {t}: labels differ"
        assert np.array_equal(got_x, ref_x), f"step {t}: rows differ (n={n})"
    fill = data[at:at + 4 * K].view(np.int32)
    at += 4 * K
    last_n = int(data[at:at + 8].view(np.int64)[0])
    flags = int(data[at + 8:at + 12].view(np.uint32)[0])
    moved = int(data[at + 12:at + 20].view(np.uint64)[0])
    at += 20
    assert np.array_equal(fill, orc.fill) and last_n == n and flags == orc.flags == 1
    assert 0 < moved <= steps * (c + r)
    buf_y = data[at:at + 8 * K * S].view(np.int64).reshape(K, S)
    at += 8 * K * S
    assert np.array_equal(buf_y, orc.buf_y)
    buf_x = data[at:at + K * S * row_bytes].reshape(K * S, row_bytes)
    assert at + K * S * row_bytes == data.size
    want = orc.export_rows(0, K * S)
    filled = (orc.buf_y.reshape(-1) >= 0)
    assert np.array_equal(buf_x[filled], want[filled])
