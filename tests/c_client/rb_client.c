/*
 * A caller of the library that is not Python: plain C against include/rb.h and the HIP runtime API.
 * It allocates its own device memory, reads a seeded workload from a file (written by the test that
 * starts it), drives the first half of the steps through rb_update + rb_sample_augment and the
 * second half through rb_announce_next_many + rb_update_sample_many, and dumps everything
 * observable (every step's augmented rows and labels, then fill counts, state words, slot labels and
 * all stored rows) for the test to compare with the oracle.
 *
 *   rb_client <input file> <output file>
 *
 * Input:  int64 K, S, row_bytes, b, c, r, steps, seed; then per step b*row_bytes sample bytes and b int64 labels.
 * Output: per step r int64 labels and r*row_bytes bytes (rows beyond n keep the byte 0x5A);
 *         then K int32 fill counts, int64 last_n, uint32 flags, uint64 moved rows, K*S int64 labels, K*S rows.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "rb.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_RB(x) do { int s_ = (x); if (s_ != RB_OK) { fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, rb_strerror(s_)); return 3; } } while (0)

enum { GROUP = 8 };      /* steps per rb_update_sample_many call */

int main(int argc, char **argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s <input> <output>\n", argv[0]); return 1; }
    FILE *in = fopen(argv[1], "rb");
    FILE *out = fopen(argv[2], "wb");
    if (!in || !out) { perror("open"); return 1; }
    int64_t h[8];
    if (fread(h, sizeof h, 1, in) != 1) return 1;
    const int64_t K = h[0], S = h[1], row_bytes = h[2], b = h[3], c = h[4], r = h[5], steps = h[6];
    const uint64_t seed = (uint64_t)h[7];
    if (row_bytes % 16 != 0 || steps < 1 || steps > 4096) return 1;
    const size_t batch_x_bytes = (size_t)b * (size_t)row_bytes, out_x_bytes = (size_t)r * (size_t)row_bytes;

    /* host copies of all inputs, device copies of all inputs and outputs (small workloads only) */
    unsigned char *hx = (unsigned char *)malloc(batch_x_bytes);
    int64_t *hy = (int64_t *)malloc((size_t)b * 8);
    unsigned char *hox = (unsigned char *)malloc(out_x_bytes ? out_x_bytes : 1);
    int64_t *hoy = (int64_t *)malloc((size_t)(r ? r : 1) * 8);
    void **dx = (void **)calloc((size_t)steps, sizeof(void *));
    int64_t **dy = (int64_t **)calloc((size_t)steps, sizeof(int64_t *));
    void **dox = (void **)calloc((size_t)steps, sizeof(void *));
    int64_t **doy = (int64_t **)calloc((size_t)steps, sizeof(int64_t *));
    if (!hx || !hy || !hox || !hoy || !dx || !dy || !dox || !doy) return 1;
    for (int64_t t = 0; t < steps; ++t) {
        if (fread(hx, 1, batch_x_bytes, in) != batch_x_bytes || fread(hy, 8, (size_t)b, in) != (size_t)b) return 1;
        CHECK_HIP(hipMalloc(&dx[t], batch_x_bytes));
        CHECK_HIP(hipMalloc((void **)&dy[t], (size_t)b * 8));
        CHECK_HIP(hipMalloc(&dox[t], out_x_bytes ? out_x_bytes : 16));
        CHECK_HIP(hipMalloc((void **)&doy[t], (size_t)(r ? r : 1) * 8));
        CHECK_HIP(hipMemcpy(dx[t], hx, batch_x_bytes, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemcpy(dy[t], hy, (size_t)b * 8, hipMemcpyHostToDevice));
        CHECK_HIP(hipMemset(dox[t], 0x5A, out_x_bytes ? out_x_bytes : 16));
        CHECK_HIP(hipMemset(doy[t], 0xFF, (size_t)(r ? r : 1) * 8));
    }
    fclose(in);

    rb_buffer *rb = NULL;
    const int64_t shape[1] = { row_bytes / 4 };
    CHECK_RB(rb_create(&rb, K, S, shape, 1, RB_F32));
    size_t xb = 0, yb = 0, wb = 0;
    CHECK_RB(rb_query_sizes(rb, &xb, &yb, &wb));
    void *buf_x = NULL, *ws = NULL;
    int64_t *buf_y = NULL;
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_HIP(hipMalloc(&buf_x, xb));
    CHECK_HIP(hipMalloc((void **)&buf_y, yb));
    CHECK_HIP(hipMalloc(&ws, wb));
    CHECK_HIP(hipMemset(buf_x, 0, xb));          /* never-written slots are dumped too */
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_RB(rb_bind(rb, buf_x, buf_y, ws, stream));

    const int64_t half = steps / 2;
    for (int64_t t = 0; t < half; ++t) {
        CHECK_RB(rb_update(rb, dx[t], dy[t], b, c, seed, (uint64_t)t));
        CHECK_RB(rb_sample_augment(rb, r, seed, (uint64_t)t, dox[t], doy[t]));
    }
    for (int64_t t = half; t < steps; t += GROUP) {
        const int64_t n = steps - t < GROUP ? steps - t : GROUP;
        const int64_t after = steps - (t + n) < GROUP ? steps - (t + n) : GROUP;
        if (after > 0) CHECK_RB(rb_announce_next_many(rb, after, (const int64_t *const *)(dy + t + n)));
        CHECK_RB(rb_update_sample_many(rb, n, (const void *const *)(dx + t), (const int64_t *const *)(dy + t), b, c, r, seed,
                                       (uint64_t)t, dox + t, doy + t));
    }
    CHECK_HIP(hipStreamSynchronize(stream));

    for (int64_t t = 0; t < steps; ++t) {
        CHECK_HIP(hipMemcpy(hoy, doy[t], (size_t)r * 8, hipMemcpyDeviceToHost));
        CHECK_HIP(hipMemcpy(hox, dox[t], out_x_bytes, hipMemcpyDeviceToHost));
        if (fwrite(hoy, 8, (size_t)r, out) != (size_t)r || fwrite(hox, 1, out_x_bytes, out) != out_x_bytes) return 1;
    }
    int32_t *fill = (int32_t *)malloc((size_t)K * 4);
    int64_t last_n = -1;
    uint32_t flags = 0;
    uint64_t moved = 0;
    CHECK_RB(rb_read_state(rb, fill, &last_n, &flags));
    CHECK_RB(rb_read_moved_rows(rb, &moved));
    fwrite(fill, 4, (size_t)K, out);
    fwrite(&last_n, 8, 1, out);
    fwrite(&flags, 4, 1, out);
    fwrite(&moved, 8, 1, out);
    unsigned char *all = (unsigned char *)malloc(xb > yb ? xb : yb);
    if (!all) return 1;
    CHECK_HIP(hipMemcpy(all, buf_y, yb, hipMemcpyDeviceToHost));
    fwrite(all, 1, yb, out);
    CHECK_HIP(hipMemcpy(all, buf_x, xb, hipMemcpyDeviceToHost));
    fwrite(all, 1, xb, out);
    if (fclose(out) != 0) return 1;
    CHECK_RB(rb_destroy(rb));
    printf("rb_client ok: %lld steps\n", (long long)steps);
    return 0;
}
