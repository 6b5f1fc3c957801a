"""The C ABI from C: a small client compiled with gcc against include/rb.h and linked to the built library.
Host-side calls only (create, sizes, option and policy setters, the launch-size query, error strings): no GPU needed."""
import os
import subprocess
import sys
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
        if (rb_query_steps_per_launch(rb, 64, 8, 8, &steps) != RB_OK || steps != 16) return 4;
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
