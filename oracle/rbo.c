/*
 * CPU oracle of the per-process rehearsal buffer (TEST INFRASTRUCTURE ONLY).
 *
 * A plain, sequential, single-threaded C implementation of what one process
 * of the paper does each training iteration with its local buffer B_n:
 *
 *   - the buffer is one sub-buffer R^i_n per class i, each of the same
 *     capacity (Sec. IV-A);
 *   - update_buffer(m) (Algorithm 1): pick c random candidates of the
 *     mini-batch m, then for every candidate append it to the sub-buffer of
 *     its class while that sub-buffer has room, otherwise overwrite a random
 *     representative of that class;
 *   - mini-batch augmentation (Sec. IV-C): draw r representatives uniformly,
 *     without replacement, from everything stored, and hand them out so the
 *     caller can concatenate them to the mini-batch (Listing 1).
 *
 * The paper names no random generator, no subset-sampling algorithm and no
 * insertion order; the readings taken here (Philox4x32-10 counter-based
 * draws, multiply-high range reduction, Floyd's subset sampling, insertion in
 * ascending mini-batch position) are chosen so that every random choice is a
 * pure function of (seed, step, purpose, index) and a parallel implementation
 * can reproduce the sequential result bit for bit.
 *
 * Nothing here is shared with the GPU library: no header, no table, no
 * helper.  Only tests, the smoke check and the bench's cpu_baseline leg may
 * use this file.  Parity status: every function below is pinned by the CPU
 * test-suite (known-answer vectors for Philox, closed forms / library
 * routines for the policy, chi-square tests for the distributions); the exact
 * seeded result at the five workload shapes is fixed by no printed example in
 * the paper (its two-iteration figures carry no numbers) -- "parity unpinned
 * by the paper" for those, pinned only through the properties above.
 */
#define _POSIX_C_SOURCE 200809L   /* pthread barriers (timing variant at the end of the file) */
#include <limits.h>
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define RBO_SELECT 1u   /* purpose tag of the draws that choose candidates       */
#define RBO_EVICT  2u   /* purpose tag of the draws that choose a slot to replace */
#define RBO_SAMPLE 3u   /* purpose tag of the draws that choose representatives   */
#define RBO_COIN   4u   /* purpose tag of the per-sample coin of the Bernoulli selection */

/* Policy variants (the default pair is what Algorithm 1 prints).
 * Selection: EXACT  - first step of Algorithm 1: a uniform subset of exactly c positions;
 *            BERNOULLI - the wording of Sec. IV-B (each sample is inserted with probability c/b):
 *                        an independent coin of probability c/b per sample.
 * Eviction (Sec. IV-A allows strategies other than random replacement of old representatives):
 *            UNIFORM   - overwrite a uniformly drawn slot of the class;
 *            FIFO      - overwrite the oldest representative of the class;
 *            RESERVOIR - reservoir sampling per class (Vitter's Algorithm R): the n-th sample ever
 *                        offered to a full class replaces a uniformly drawn slot with probability
 *                        S/n and is discarded otherwise, so that the class holds a uniform sample
 *                        of everything it was offered. */
enum { RBO_SELECT_EXACT = 0, RBO_SELECT_BERNOULLI = 1 };
enum { RBO_EVICT_UNIFORM = 0, RBO_EVICT_FIFO = 1, RBO_EVICT_RESERVOIR = 2 };

/* Storage variants.  The discussion section (Sec. VII) notes that data reduction can be applied to the
 * stored representatives and names no technique; the one built here is the plainest for floating-point
 * samples: keep every IEEE binary32 element as a bfloat16.
 *   SAME - a stored row is the sample's bytes;
 *   BF16 - the sample is an array of binary32 values; each is stored as the bfloat16 nearest to it (ties
 *          to the one whose last bit is 0), and handed out widened back to binary32, which is exact.
 *   U8   - the sample is an array of binary32 values meant to lie in [0, 1] (an image tensor); each value x is
 *          stored as one byte, the integer nearest to 255 * x, and handed out as that integer divided by 255.
 *          So that two implementations agree on every bit, the arithmetic is fixed: the product 255 * x is the
 *          binary32 product, it is rounded to an integer in the nearest-even sense, values not above 0 (and
 *          NaN) give 0 and products of 255 or more give 255; the quotient is the binary32 quotient. */
enum { RBO_STORE_SAME = 0, RBO_STORE_BF16 = 1, RBO_STORE_U8 = 2 };

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as  */
/* easy as 1, 2, 3", SC'11, Sec. 3.3 and Table 2 for the constants).        */
/* ------------------------------------------------------------------------ */
void rbo_philox4x32_10(const uint32_t ctr_in[4], const uint32_t key_in[2], uint32_t out[4])
{
    uint32_t c0 = ctr_in[0], c1 = ctr_in[1], c2 = ctr_in[2], c3 = ctr_in[3];
    uint32_t k0 = key_in[0], k1 = key_in[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;   /* multiplier of word 0 */
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;   /* multiplier of word 2 */
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;                          /* Weyl key schedule    */
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* One 64-bit uniform draw per (seed, step, purpose, index). */
uint64_t rbo_draw64(uint64_t seed, uint64_t step, uint32_t purpose, uint32_t index)
{
    uint32_t ctr[4] = { index, purpose, (uint32_t)step, (uint32_t)(step >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    rbo_philox4x32_10(ctr, key, w);
    return (uint64_t)w[0] | ((uint64_t)w[1] << 32);
}

/* Uniform integer in [0, n): floor(u * n / 2^64) of the 64-bit draw u. */
uint64_t rbo_bounded(uint64_t seed, uint64_t step, uint32_t purpose, uint32_t index, uint64_t n)
{
    unsigned __int128 prod = (unsigned __int128)rbo_draw64(seed, step, purpose, index) * n;
    return (uint64_t)(prod >> 64);
}

/*
 * Floyd's algorithm for a uniformly distributed m-subset of {0..n-1}
 * (Bentley & Floyd, "Programming pearls: a sample of brilliance", CACM 1987).
 * out[i] is the element added in iteration i.  Membership is tested by a
 * plain linear search over what was emitted so far.
 */
void rbo_floyd(uint64_t seed, uint64_t step, uint32_t purpose, int64_t n, int64_t m, int64_t *out)
{
    for (int64_t i = 0; i < m; ++i) {
        int64_t j = n - m + i;
        int64_t t = (int64_t)rbo_bounded(seed, step, purpose, (uint32_t)i, (uint64_t)j + 1);
        int seen = 0;
        for (int64_t q = 0; q < i; ++q)
            if (out[q] == t) { seen = 1; break; }
        out[i] = seen ? j : t;
    }
}

/* ------------------------------------------------------------------------ */
/* binary32 -> bfloat16, round to nearest, ties to even, written out from   */
/* the definition.  A bfloat16 is the upper 16 bits of a binary32, so the   */
/* two neighbours of a value are its bit pattern with the lower half        */
/* cleared (towards zero) and that plus one unit in bit 16 (away from zero; */
/* from the largest finite bfloat16 this is infinity, as rounding demands). */
/* NaN stays NaN: sign and upper payload bits kept, quiet bit set.          */
/* ------------------------------------------------------------------------ */
uint16_t rbo_f32_to_bf16(uint32_t bits)
{
    uint32_t magnitude = bits & 0x7FFFFFFFu;
    if (magnitude > 0x7F800000u) return (uint16_t)((bits >> 16) | 0x0040u);
    uint32_t down = bits >> 16;             /* neighbour towards zero  */
    uint32_t up = down + 1u;                /* neighbour away from zero */
    uint32_t rest = bits & 0xFFFFu;         /* distance from `down`, in units of 2^-16 of the gap */
    if (rest < 0x8000u) return (uint16_t)down;
    if (rest > 0x8000u) return (uint16_t)up;
    return (uint16_t)((down & 1u) ? up : down);
}

uint32_t rbo_bf16_to_f32(uint16_t h) { return (uint32_t)h << 16; }

/* binary32 (given by its bit pattern) -> byte, and back; see RBO_STORE_U8. */
uint8_t rbo_f32_to_u8(uint32_t bits)
{
    float x;
    memcpy(&x, &bits, 4);
    volatile float product = x * 255.0f;     /* (volatile: rounded to binary32 here, whatever the compiler keeps in registers) */
    float t = product;
    if (!(t > 0.0f)) return 0;               /* not above zero, or NaN */
    if (t >= 255.0f) return 255;
    return (uint8_t)lrintf(t);               /* nearest integer, ties to even (the default rounding mode) */
}

uint32_t rbo_u8_to_f32(uint8_t q)
{
    volatile float quotient = (float)q / 255.0f;
    float y = quotient;
    uint32_t bits;
    memcpy(&bits, &y, 4);
    return bits;
}

/* ------------------------------------------------------------------------ */
/* The buffer                                                                */
/* ------------------------------------------------------------------------ */
typedef struct rbo_buffer {
    int64_t K;            /* number of classes                                   */
    int64_t S;            /* capacity of every per-class sub-buffer, in samples  */
    int64_t row_bytes;    /* bytes of one sample as the caller hands it in and gets it back */
    int64_t stored_bytes; /* bytes of one stored sample (row_bytes, or half of it) */
    int storage;          /* RBO_STORE_*                                          */
    int32_t *fill;        /* [K]   samples currently held per class              */
    int64_t *buf_y;       /* [K*S] label of each slot, -1 while never written    */
    unsigned char **rows; /* [K*S] sample bytes of each slot, NULL until written */
    uint32_t flags;       /* bit 0: a candidate carried a label outside [0,K)    */
    int64_t last_n;       /* representatives handed out by the last sampling     */
    /* record of the last calls, for tests that inspect the decisions */
    int64_t n_ins;        /* insertions performed by the last update             */
    int64_t *ins_pos;     /* [c] mini-batch position of each insertion           */
    int64_t *ins_class;   /* [c] its class                                       */
    int64_t *ins_slot;    /* [c] the slot it went to                             */
    int64_t *smp_g;       /* [last_n] index, among the filled slots in class-major order, of each representative */
    int64_t cap_ins, cap_smp;
    int selection, eviction;   /* policy variant, see the enums above */
    int32_t *head;        /* [K] FIFO: slot of the oldest representative of a full class       */
    int32_t *seen;        /* [K] RESERVOIR: samples offered to the class so far (saturating)   */
    /* timing variant only (see the end of this file): row copies are listed instead of carried out */
    int defer;
    struct rbo_copy *jobs;
    int64_t n_jobs, cap_jobs;
} rbo_buffer;

struct rbo_copy { unsigned char *dst; const unsigned char *src; };

/* Timing variant: remember a row copy for later.  Returns 0, or -1 when out of memory. */
static int defer_copy(rbo_buffer *rb, unsigned char *dst, const unsigned char *src)
{
    if (rb->n_jobs == rb->cap_jobs) {
        int64_t cap = rb->cap_jobs ? 2 * rb->cap_jobs : 256;
        struct rbo_copy *j = (struct rbo_copy *)realloc(rb->jobs, (size_t)cap * sizeof *j);
        if (!j) return -1;
        rb->jobs = j; rb->cap_jobs = cap;
    }
    rb->jobs[rb->n_jobs].dst = dst; rb->jobs[rb->n_jobs].src = src;
    rb->n_jobs += 1;
    return 0;
}

rbo_buffer *rbo_create(int64_t classes, int64_t slots_per_class, int64_t row_bytes)
{
    if (classes < 1 || slots_per_class < 1 || row_bytes < 1) return NULL;
    rbo_buffer *rb = (rbo_buffer *)calloc(1, sizeof *rb);
    if (!rb) return NULL;
    rb->K = classes; rb->S = slots_per_class; rb->row_bytes = row_bytes;
    rb->stored_bytes = row_bytes; rb->storage = RBO_STORE_SAME;
    size_t slots = (size_t)classes * (size_t)slots_per_class;
    rb->fill = (int32_t *)calloc((size_t)classes, sizeof(int32_t));
    rb->head = (int32_t *)calloc((size_t)classes, sizeof(int32_t));
    rb->seen = (int32_t *)calloc((size_t)classes, sizeof(int32_t));
    rb->buf_y = (int64_t *)malloc(slots * sizeof(int64_t));
    rb->rows = (unsigned char **)calloc(slots, sizeof(unsigned char *));
    if (!rb->fill || !rb->head || !rb->seen || !rb->buf_y || !rb->rows) {
        free(rb->fill); free(rb->head); free(rb->seen); free(rb->buf_y); free(rb->rows); free(rb); return NULL;
    }
    for (size_t i = 0; i < slots; ++i) rb->buf_y[i] = -1;
    return rb;
}

void rbo_destroy(rbo_buffer *rb)
{
    if (!rb) return;
    size_t slots = (size_t)rb->K * (size_t)rb->S;
    for (size_t i = 0; i < slots; ++i) free(rb->rows[i]);
    free(rb->rows); free(rb->buf_y); free(rb->fill); free(rb->head); free(rb->seen);
    free(rb->ins_pos); free(rb->ins_class); free(rb->ins_slot); free(rb->smp_g); free(rb->jobs);
    free(rb);
}

/* Choose the policy variant; only while the buffer is still empty.  Returns 0, or -1. */
int rbo_set_policy(rbo_buffer *rb, int selection, int eviction)
{
    if (!rb || selection < 0 || selection > 1 || eviction < 0 || eviction > 2) return -1;
    for (int64_t k = 0; k < rb->K; ++k)
        if (rb->fill[k] != 0 || rb->seen[k] != 0) return -1;
    rb->selection = selection;
    rb->eviction = eviction;
    return 0;
}

/* Choose the storage variant; only while the buffer is still empty.  BF16 needs rows made of
 * binary32 elements.  Returns 0, or -1. */
int rbo_set_storage(rbo_buffer *rb, int storage)
{
    if (!rb || (storage != RBO_STORE_SAME && storage != RBO_STORE_BF16 && storage != RBO_STORE_U8)) return -1;
    if (storage != RBO_STORE_SAME && rb->row_bytes % 4 != 0) return -1;
    for (int64_t k = 0; k < rb->K; ++k)
        if (rb->fill[k] != 0 || rb->seen[k] != 0) return -1;
    rb->storage = storage;
    rb->stored_bytes = storage == RBO_STORE_BF16 ? rb->row_bytes / 2 : storage == RBO_STORE_U8 ? rb->row_bytes / 4 : rb->row_bytes;
    return 0;
}

/* One sample into its stored form / back (both rows may be unaligned: bytes are assembled by hand,
 * little-endian like the machines this runs on). */
static void store_row(rbo_buffer *rb, unsigned char *stored, const unsigned char *sample)
{
    if (rb->defer && defer_copy(rb, stored, sample) == 0) return;
    if (rb->storage == RBO_STORE_SAME) { memcpy(stored, sample, (size_t)rb->row_bytes); return; }
    for (int64_t e = 0; e < rb->row_bytes / 4; ++e) {
        uint32_t bits;
        memcpy(&bits, sample + 4 * e, 4);
        if (rb->storage == RBO_STORE_U8) { stored[e] = rbo_f32_to_u8(bits); continue; }
        uint16_t h = rbo_f32_to_bf16(bits);
        memcpy(stored + 2 * e, &h, 2);
    }
}

static void load_row(rbo_buffer *rb, unsigned char *sample, const unsigned char *stored)
{
    if (rb->defer && defer_copy(rb, sample, stored) == 0) return;
    if (rb->storage == RBO_STORE_SAME) { memcpy(sample, stored, (size_t)rb->row_bytes); return; }
    for (int64_t e = 0; e < rb->row_bytes / 4; ++e) {
        uint32_t bits;
        if (rb->storage == RBO_STORE_U8) {
            bits = rbo_u8_to_f32(stored[e]);
        } else {
            uint16_t h;
            memcpy(&h, stored + 2 * e, 2);
            bits = rbo_bf16_to_f32(h);
        }
        memcpy(sample + 4 * e, &bits, 4);
    }
}

static int cmp_i64(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

/*
 * Algorithm 1, update_buffer(m).  batch_x: b rows of row_bytes; batch_y: b
 * labels.  Returns 0, or -1 on invalid arguments / out of memory.
 */
int rbo_update(rbo_buffer *rb, const void *batch_x, const int64_t *batch_y,
               int64_t b, int64_t c, uint64_t seed, uint64_t step)
{
    if (!rb || !batch_x || !batch_y || b < 1 || c < 0 || c > b) return -1;
    /* at most c candidates with the exact selection, at most b with the Bernoulli one */
    int64_t cap = rb->selection == RBO_SELECT_BERNOULLI ? b : c;
    if (cap > rb->cap_ins) {
        free(rb->ins_pos); free(rb->ins_class); free(rb->ins_slot);
        rb->ins_pos = (int64_t *)malloc((size_t)cap * sizeof(int64_t));
        rb->ins_class = (int64_t *)malloc((size_t)cap * sizeof(int64_t));
        rb->ins_slot = (int64_t *)malloc((size_t)cap * sizeof(int64_t));
        rb->cap_ins = cap;
        if (!rb->ins_pos || !rb->ins_class || !rb->ins_slot) return -1;
    }
    rb->n_ins = 0;
    if (c == 0) return 0;

    int64_t *cand = (int64_t *)malloc((size_t)cap * sizeof(int64_t));
    if (!cand) return -1;
    int64_t ncand;
    if (rb->selection == RBO_SELECT_BERNOULLI) {
        /* Sec. IV-B wording: each sample is a candidate with probability c/b.  One coin per
         * position, heads iff a uniform integer below b is below c. */
        ncand = 0;
        for (int64_t pos = 0; pos < b; ++pos)
            if ((int64_t)rbo_bounded(seed, step, RBO_COIN, (uint32_t)pos, (uint64_t)b) < c) cand[ncand++] = pos;
    } else {
        /* Algorithm 1, first step (choose c candidates of the mini-batch at random): a
         * uniform c-subset of the b positions. */
        rbo_floyd(seed, step, RBO_SELECT, b, c, cand);
        ncand = c;
        /* Algorithm 1, loop over the candidates: visited in ascending mini-batch position. */
        qsort(cand, (size_t)c, sizeof(int64_t), cmp_i64);
    }

    const unsigned char *src = (const unsigned char *)batch_x;
    for (int64_t q = 0; q < ncand; ++q) {
        int64_t pos = cand[q];
        int64_t k = batch_y[pos];
        if (k < 0 || k >= rb->K) { rb->flags |= 1u; continue; }
        int64_t s;
        int64_t offered = rb->seen[k];          /* samples offered to class k before this one */
        if (rb->seen[k] < INT32_MAX) rb->seen[k] += 1;
        if (rb->fill[k] < rb->S) {
            /* Algorithm 1, else-branch: the class still has room, the candidate is appended */
            s = rb->fill[k];
            rb->fill[k] += 1;
        } else if (rb->eviction == RBO_EVICT_FIFO) {
            /* replace the oldest representative */
            s = rb->head[k];
            rb->head[k] = (int32_t)((rb->head[k] + 1) % rb->S);
        } else if (rb->eviction == RBO_EVICT_RESERVOIR) {
            /* Algorithm R: sample number `offered` (0-based) stays with probability S/(offered+1) */
            s = (int64_t)rbo_bounded(seed, step, RBO_EVICT, (uint32_t)pos, (uint64_t)offered + 1);
            if (s >= rb->S) continue;
        } else {
            /* Algorithm 1, if-branch: the class is full, a random representative is replaced:
             * every slot of the class equally likely, whatever its age. */
            s = (int64_t)rbo_bounded(seed, step, RBO_EVICT, (uint32_t)pos, (uint64_t)rb->S);
        }
        size_t slot = (size_t)k * (size_t)rb->S + (size_t)s;
        if (!rb->rows[slot]) {
            rb->rows[slot] = (unsigned char *)malloc((size_t)rb->stored_bytes);
            if (!rb->rows[slot]) { free(cand); return -1; }
        }
        store_row(rb, rb->rows[slot], src + (size_t)pos * (size_t)rb->row_bytes);
        rb->buf_y[slot] = k;
        rb->ins_pos[rb->n_ins] = pos; rb->ins_class[rb->n_ins] = k; rb->ins_slot[rb->n_ins] = s;
        rb->n_ins += 1;
    }
    free(cand);
    return 0;
}

/*
 * Mini-batch augmentation: draw n = min(r, F) representatives uniformly and
 * without replacement from the F stored samples and copy them (and their
 * labels) to out_x / out_y; out_y[j] = -1 for n <= j < r, the matching out_x
 * rows are left alone.  Returns n, or -1 on invalid arguments.
 */
int64_t rbo_sample_augment(rbo_buffer *rb, int64_t r, uint64_t seed, uint64_t step,
                           void *out_x, int64_t *out_y)
{
    if (!rb || r < 0 || (r > 0 && (!out_x || !out_y))) return -1;
    int64_t F = 0;
    for (int64_t k = 0; k < rb->K; ++k) F += rb->fill[k];
    int64_t n = r < F ? r : F;
    if (n > rb->cap_smp) {
        free(rb->smp_g);
        rb->smp_g = (int64_t *)malloc((size_t)n * sizeof(int64_t));
        rb->cap_smp = n;
        if (!rb->smp_g) return -1;
    }
    rb->last_n = n;
    if (n > 0) rbo_floyd(seed, step, RBO_SAMPLE, F, n, rb->smp_g);

    unsigned char *dst = (unsigned char *)out_x;
    for (int64_t j = 0; j < n; ++j) {
        /* the g-th stored sample, counting class 0's slots first, then class
         * 1's, ... (a fuller class is therefore drawn more often). */
        int64_t g = rb->smp_g[j], k = 0;
        while (g >= rb->fill[k]) { g -= rb->fill[k]; ++k; }
        size_t slot = (size_t)k * (size_t)rb->S + (size_t)g;
        load_row(rb, dst + (size_t)j * (size_t)rb->row_bytes, rb->rows[slot]);
        out_y[j] = k;
    }
    for (int64_t j = n; j < r; ++j) out_y[j] = -1;
    return n;
}

/* ------------------------------------------------------------------------ */
/* Read-only access for the tests                                            */
/* ------------------------------------------------------------------------ */
const int32_t *rbo_fill(const rbo_buffer *rb) { return rb->fill; }
const int64_t *rbo_buf_y(const rbo_buffer *rb) { return rb->buf_y; }
uint32_t rbo_flags(const rbo_buffer *rb) { return rb->flags; }
int64_t rbo_last_n(const rbo_buffer *rb) { return rb->last_n; }
int64_t rbo_n_inserted(const rbo_buffer *rb) { return rb->n_ins; }
const int64_t *rbo_ins_pos(const rbo_buffer *rb) { return rb->ins_pos; }
const int64_t *rbo_ins_class(const rbo_buffer *rb) { return rb->ins_class; }
const int64_t *rbo_ins_slot(const rbo_buffer *rb) { return rb->ins_slot; }
const int64_t *rbo_sampled_g(const rbo_buffer *rb) { return rb->smp_g; }
int64_t rbo_stored_row_bytes(const rbo_buffer *rb) { return rb->stored_bytes; }

/* Stored bytes (rbo_stored_row_bytes of them) of slot s of class k, or NULL while that slot was never written. */
const void *rbo_row(const rbo_buffer *rb, int64_t k, int64_t s)
{
    if (k < 0 || k >= rb->K || s < 0 || s >= rb->S) return NULL;
    return rb->rows[(size_t)k * (size_t)rb->S + (size_t)s];
}

/* Copy slots [first, first+count) (flat index k*S+s), as stored, into dst, row after row;
 * never-written slots are filled with zero bytes. */
void rbo_export_rows(const rbo_buffer *rb, int64_t first, int64_t count, void *dst)
{
    unsigned char *d = (unsigned char *)dst;
    for (int64_t i = 0; i < count; ++i) {
        const unsigned char *src = rb->rows[(size_t)(first + i)];
        if (src) memcpy(d + (size_t)i * (size_t)rb->stored_bytes, src, (size_t)rb->stored_bytes);
        else memset(d + (size_t)i * (size_t)rb->stored_bytes, 0, (size_t)rb->stored_bytes);
    }
}

/* ------------------------------------------------------------------------ */
/* Timing variant: the same two calls with the row copies of a call spread   */
/* over host threads.  The policy (selection, slot assignment, sampling)     */
/* stays the sequential code above, which only lists its row copies instead  */
/* of carrying them out; then every thread walks the list in order and       */
/* copies its own slice of every row.  Copies to one destination therefore   */
/* still land in list order, byte for byte, so the result is that of the     */
/* plain calls.  Only for the storage form RBO_STORE_SAME.  This is a        */
/* reported baseline of the benchmark, not the parity reference.             */
/* ------------------------------------------------------------------------ */
typedef struct rbo_pool {
    int n;                          /* worker threads                              */
    pthread_t *threads;
    pthread_barrier_t start, done;  /* workers and the caller meet at both         */
    const struct rbo_copy *jobs;
    int64_t n_jobs, row_bytes;
    int quit;
} rbo_pool;

struct rbo_worker { rbo_pool *pool; int index; };

static void *pool_worker(void *arg)
{
    struct rbo_worker *me = (struct rbo_worker *)arg;
    rbo_pool *pool = me->pool;
    const int t = me->index;
    free(me);
    for (;;) {
        pthread_barrier_wait(&pool->start);
        if (pool->quit) return NULL;
        /* slice t of every row, in multiples of 64 bytes */
        int64_t units = (pool->row_bytes + 63) / 64;
        int64_t lo = units * t / pool->n * 64, hi = units * (t + 1) / pool->n * 64;
        if (hi > pool->row_bytes) hi = pool->row_bytes;
        if (lo < hi)
            for (int64_t j = 0; j < pool->n_jobs; ++j)
                memcpy(pool->jobs[j].dst + lo, pool->jobs[j].src + lo, (size_t)(hi - lo));
        pthread_barrier_wait(&pool->done);
    }
}

rbo_pool *rbo_pool_create(int threads)
{
    if (threads < 1 || threads > 1024) return NULL;
    rbo_pool *pool = (rbo_pool *)calloc(1, sizeof *pool);
    if (!pool) return NULL;
    pool->threads = (pthread_t *)calloc((size_t)threads, sizeof(pthread_t));
    if (!pool->threads) { free(pool); return NULL; }
    pthread_barrier_init(&pool->start, NULL, (unsigned)threads + 1);
    pthread_barrier_init(&pool->done, NULL, (unsigned)threads + 1);
    pool->n = threads;
    for (int t = 0; t < threads; ++t) {
        struct rbo_worker *w = (struct rbo_worker *)malloc(sizeof *w);
        if (!w) abort();
        w->pool = pool; w->index = t;
        if (pthread_create(&pool->threads[t], NULL, pool_worker, w) != 0) abort();
    }
    return pool;
}

void rbo_pool_destroy(rbo_pool *pool)
{
    if (!pool) return;
    pool->quit = 1;
    pthread_barrier_wait(&pool->start);
    for (int t = 0; t < pool->n; ++t) pthread_join(pool->threads[t], NULL);
    pthread_barrier_destroy(&pool->start);
    pthread_barrier_destroy(&pool->done);
    free(pool->threads);
    free(pool);
}

static void pool_run(rbo_pool *pool, rbo_buffer *rb)
{
    pool->jobs = rb->jobs; pool->n_jobs = rb->n_jobs; pool->row_bytes = rb->row_bytes;
    pthread_barrier_wait(&pool->start);
    pthread_barrier_wait(&pool->done);
    rb->n_jobs = 0;
}

int rbo_update_mt(rbo_pool *pool, rbo_buffer *rb, const void *batch_x, const int64_t *batch_y,
                  int64_t b, int64_t c, uint64_t seed, uint64_t step)
{
    if (!pool || !rb || rb->storage != RBO_STORE_SAME) return -1;
    rb->defer = 1; rb->n_jobs = 0;
    int rc = rbo_update(rb, batch_x, batch_y, b, c, seed, step);
    rb->defer = 0;
    pool_run(pool, rb);
    return rc;
}

int64_t rbo_sample_augment_mt(rbo_pool *pool, rbo_buffer *rb, int64_t r, uint64_t seed, uint64_t step,
                              void *out_x, int64_t *out_y)
{
    if (!pool || !rb || rb->storage != RBO_STORE_SAME) return -1;
    rb->defer = 1; rb->n_jobs = 0;
    int64_t n = rbo_sample_augment(rb, r, seed, step, out_x, out_y);
    rb->defer = 0;
    pool_run(pool, rb);
    return n;
}
