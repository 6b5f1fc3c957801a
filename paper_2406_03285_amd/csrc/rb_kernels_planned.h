// Plan-ahead kernels for the single-launch step with at most 64 candidates and representatives:
// the plan of a step (which rows go where) is worked out by ONE workgroup during the previous
// step's launch and left in a table; the step's own launch then only moves rows by that table.
// Included by rb.hip only, after rb_kernels_small.h (whose candidate selection it uses).
#pragma once

#include "rb_device.h"
#include "rb_kernels_small.h"

namespace {

// The table of one step, in the caller's workspace.
struct PlanHeader {
    int32_t n;            // representatives the step hands out: min(r, F)
    uint32_t flags;       // RB_FLAG_* raised by the step
    int32_t c, r;         // what the plan was made for
};
struct PlanEntry {        // 16 bytes
    // candidate e < c:       pos = its mini-batch position, row = slot row it is stored to (-1: not stored)
    // representative e - c:  pos = mini-batch position it is copied from when its slot is written in the
    //                        same step (-1: read the slot), label = its class (-1: fewer stored than asked
    //                        for), row = slot row it is read from
    int32_t pos;
    int32_t label;
    int64_t row;
};
constexpr int PLAN_ROWS = 2 * WAVE;
constexpr size_t PLAN_BYTES = (sizeof(PlanHeader) + PLAN_ROWS * sizeof(PlanEntry) + 255) / 256 * 256;

struct PlanArgs {
    const int64_t* batch_y;   // labels of the step that is planned
    const int32_t* fill_old;  // fill counts before that step
    int32_t* fill_new;        // ... and after it
    int32_t* chunk_new;
    char* table;              // PlanHeader, then c + r entries
    Seed sd;
    int32_t b, c, r;
    int32_t K, nchunks;
    int64_t S;
    int32_t eviction;         // RB_EVICT_*
    const int32_t* aux_old;   // per class: FIFO: slot of the oldest sample; RESERVOIR: samples offered so far
    int32_t* aux_new;
    int32_t selection;        // RB_SELECT_* (the large-count form only; the others are for the exact selection)
    int32_t ce;               // candidate entries of the table: c, or b with the Bernoulli selection (one per position)
};

struct MoveArgs {
    const vec16* batch_x;
    vec16* buf_x;
    int64_t* buf_y;
    vec16* out_x;
    int64_t* out_y;
    const char* table;
    DevState* state;
    int32_t c, r;
    int64_t S;
    int64_t row_vec;
    int32_t tpr, tile_vec, tile_rem;
    int32_t plan_next;        // 1: workgroup 0 plans the next step and the movers start at workgroup 1
    int32_t cgrid;            // large-count form: candidate rows the grid covers (c; with the Bernoulli selection c plus a margin)
};

// ---------------------------------------------------------------------------
// The whole plan of one step by one workgroup (all TPB threads call it).
// Wavefront 0: one lane per candidate (selection, class, insertion number, slot,
// last writer wins); all threads: fill counts after the update and their prefix
// sums over the classes; wavefront 1: one lane per representative (Floyd draw,
// class-major locate, forwarding from the mini-batch when the slot is written in
// this very step).  Same decisions as rb_step_small_kernel, candidate by
// candidate and representative by representative.
//
// LDS (dynamic): s_first[b] u32, s_y[b] i32.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void plan_step(const PlanArgs& a, uint32_t* lds)
{
    constexpr int NCLS = DIRECT_CHUNKS * CH;
    uint32_t* s_first = lds;                                   // [b]
    int32_t* s_y = reinterpret_cast<int32_t*>(lds + a.b);      // [b]
    __shared__ int32_t s_old[NCLS];     // fill counts before the step
    __shared__ int32_t s_cnt[NCLS];     // candidates of each class in this step
    __shared__ int32_t s_pre[NCLS];     // stored samples in the classes before each class, after the update
    __shared__ int32_t s_aux[NCLS];     // per-class state of the FIFO / reservoir strategies before the step
    __shared__ int s_wave[NWAVE];
    __shared__ uint64_t s_bits[WAVE];   // random bits of sampling draw i
    __shared__ __align__(16) int32_t s_ck[WAVE], s_cslot[WAVE], s_cx[WAVE];   // per candidate: class (-1: none), slot, position
    __shared__ __align__(16) int32_t s_cw[WAVE];                              // per candidate: the slot it drew if it overwrites, else -2
    __shared__ __align__(16) uint32_t s_t[WAVE];                              // per representative: its Floyd draw
    __shared__ uint32_t s_flags;

    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int b = a.b, c = a.c, r = a.r;
    PlanHeader* head = reinterpret_cast<PlanHeader*>(a.table);
    PlanEntry* entry = reinterpret_cast<PlanEntry*>(a.table + sizeof(PlanHeader));

    int64_t yv[YPRE];
#pragma unroll
    for (int u = 0; u < YPRE; ++u) {
        const int q = tid + u * TPB;
        yv[u] = q < b ? a.batch_y[q] : -1;
    }
    int4 fo = make_int4(0, 0, 0, 0), ao = make_int4(0, 0, 0, 0);
    if (4 * tid < a.nchunks * CH) {
        fo = *reinterpret_cast<const int4*>(a.fill_old + 4 * tid);
        if (a.eviction != RB_EVICT_UNIFORM) ao = *reinterpret_cast<const int4*>(a.aux_old + 4 * tid);
    }

    bool active = false;
    int x = 0;
    if (wave == 0) {
        x = wave_select(a.sd, b, c, s_first, active);
    } else if (wave == 1) {
        if (lane < r) s_bits[lane] = draw64(a.sd, PURPOSE_SAMPLE, (uint32_t)lane);
    }
    park_labels(yv, a.batch_y, b, a.K, s_y);
    *reinterpret_cast<int4*>(s_old + 4 * tid) = fo;
    *reinterpret_cast<int4*>(s_aux + 4 * tid) = ao;
    *reinterpret_cast<int4*>(s_cnt + 4 * tid) = make_int4(0, 0, 0, 0);
    __syncthreads();

    // ---- classes of the candidates: lane i of wavefront 0 = candidate i of Floyd's emission order ----
    int32_t k = LAB_UNSELECTED;
    bool valid = false;
    if (wave == 0) {
        k = active ? s_y[x] : LAB_UNSELECTED;
        valid = active && k >= 0;
        const bool bad = __ballot(active && k == LAB_INVALID) != 0;
        // Every lane's class and position go to LDS; the loops over the candidates below read them
        // back four at a time (one address for the whole wavefront).  Lanes without a candidate, or
        // with a label outside [0, K), hold class -1 and match nobody.
        s_ck[lane] = valid ? k : -1;
        s_cx[lane] = x;
        if (valid) atomicAdd(&s_cnt[k], 1);
        if (lane == 0) s_flags = bad ? RB_FLAG_BAD_LABEL : 0u;
    }
    __syncthreads();

    // ---- fill counts after the update, four consecutive classes per thread ----
    int nf[4];
    int local = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t v = (int64_t)s_old[4 * tid + u] + s_cnt[4 * tid + u];
        nf[u] = (int)(v < a.S ? v : a.S);
        local += nf[u];
    }
    if (4 * tid < a.nchunks * CH) {
        *reinterpret_cast<int4*>(a.fill_new + 4 * tid) = make_int4(nf[0], nf[1], nf[2], nf[3]);
        if (a.eviction != RB_EVICT_UNIFORM) {
            int na[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t before_k = s_aux[4 * tid + u], v = (int64_t)s_old[4 * tid + u] + s_cnt[4 * tid + u];
                if (a.eviction == RB_EVICT_FIFO) {
                    // the oldest sample moves on by the number of overwrites
                    na[u] = (int)((before_k + (v > a.S ? v - a.S : 0)) % a.S);
                } else {
                    const int64_t seen = before_k + s_cnt[4 * tid + u];
                    na[u] = (int)(seen < INT32_MAX ? seen : INT32_MAX);
                }
            }
            *reinterpret_cast<int4*>(a.aux_new + 4 * tid) = make_int4(na[0], na[1], na[2], na[3]);
        }
    }
    {
        // a wavefront covers exactly one chunk of CH classes
        const int wsum = lane_read(wave_scan_incl(local), WAVE - 1);
        if (lane == 0 && wave < a.nchunks) a.chunk_new[wave] = wsum;
    }
    int F;
    int before = block_scan_excl(local, F, s_wave);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        s_pre[4 * tid + u] = before;
        before += nf[u];
    }
    __syncthreads();

    // From here wavefront 0 places the candidates while wavefront 1 draws and locates the
    // representatives; the two meet again for the forwarding check.
    int pk = 0, ps = 0, n = 0;
    if (wave == 0) {
        // insertion number within the class: fill0 + class-mates earlier in the mini-batch
        const int64_t fill0 = valid ? s_old[k] : 0;
        const int64_t aux0 = valid ? s_aux[k] : 0;
        int rank = 0, total = 0;
#pragma unroll 4
        for (int m = 0; m < c; m += 4) {
            const int4 km = *reinterpret_cast<const int4*>(s_ck + m);
            const int4 xm = *reinterpret_cast<const int4*>(s_cx + m);
            rank += (int)(km.x == k && xm.x < x) + (int)(km.y == k && xm.y < x) + (int)(km.z == k && xm.z < x) +
                    (int)(km.w == k && xm.w < x);
            total += (int)(km.x == k) + (int)(km.y == k) + (int)(km.z == k) + (int)(km.w == k);
        }
        const int64_t at = fill0 + rank;
        int slot = valid ? (int)at : -1;
        bool beaten = false;
        if (a.eviction == RB_EVICT_FIFO) {
            // beyond the capacity the oldest sample is overwritten; a candidate is itself overwritten in this
            // step if a class-mate comes a whole round of S later (the same slot: the later one is what it holds)
            if (valid && at >= a.S) slot = (int)((aux0 + at - a.S) % a.S);
            beaten = valid && at + a.S < fill0 + total;
        } else {
            const bool reservoir = a.eviction == RB_EVICT_RESERVOIR;
            bool over = valid && at >= a.S;            // beyond the capacity: overwrites a drawn slot, if it is kept
            if (__ballot(over) != 0) {
                if (over) {
                    const int64_t offers = aux0 + rank < INT32_MAX ? aux0 + rank : INT32_MAX;   // to the class, before this one
                    const int64_t draw = (int64_t)below(a.sd, PURPOSE_EVICT, (uint32_t)x, reservoir ? (uint64_t)offers + 1 : (uint64_t)a.S);
                    over = draw < a.S;                 // reservoir: otherwise the candidate is not kept
                    slot = over ? (int)draw : -1;
                }
                s_cw[lane] = over ? slot : -2;         // slot an overwriting candidate drew
                // not stored if a later class-mate overwrites the same slot
#pragma unroll 4
                for (int m = 0; m < c; m += 4) {
                    const int4 km = *reinterpret_cast<const int4*>(s_ck + m);
                    const int4 xm = *reinterpret_cast<const int4*>(s_cx + m);
                    const int4 wm = *reinterpret_cast<const int4*>(s_cw + m);
                    beaten |= (km.x == k && xm.x > x && wm.x == slot) | (km.y == k && xm.y > x && wm.y == slot) |
                              (km.z == k && xm.z > x && wm.z == slot) | (km.w == k && xm.w > x && wm.w == slot);
                }
            }
        }
        s_cslot[lane] = slot;                          // -1 without a candidate
        if (lane < c) {
            PlanEntry e;
            e.pos = x;
            e.label = valid ? k : -1;
            e.row = (valid && slot >= 0 && !beaten) ? (int64_t)k * a.S + slot : -1;
            entry[lane] = e;
        }
    } else if (wave == 1) {
        // ---- representatives: lane j = draw j of Floyd's n-subset of the F stored samples ----
        n = r < F ? r : F;
        const int base = F - n;
        const uint32_t t = lane < n ? (uint32_t)__umul64hi(s_bits[lane], (uint64_t)base + lane + 1) : 0xFFFFFFFFu;
        s_t[lane] = t;
        bool dup = false;                               // an earlier draw had the same value
#pragma unroll 4
        for (int i = 0; i < n; i += 4) {
            const uint4 ti = *reinterpret_cast<const uint4*>(s_t + i);
            dup |= (i < lane && ti.x == t) | (i + 1 < lane && ti.y == t) | (i + 2 < lane && ti.z == t) | (i + 3 < lane && ti.w == t);
        }
        // replaced by base + j iff dup, or t = base + q for an earlier q whose own draw was replaced
        int cur = lane;
        bool taken = false, done = lane >= n;
        while (__ballot(!done) != 0) {
            const uint32_t tc = (uint32_t)__shfl((int)t, cur, WAVE);
            const int dc = __shfl((int)dup, cur, WAVE);
            if (!done) {
                if (dc) {
                    taken = true;
                    done = true;
                } else {
                    const int64_t q = (int64_t)tc - base;
                    if (q < 0 || q >= cur) done = true;
                    else cur = (int)q;
                }
            }
        }
        const int g = taken ? base + lane : (int)t;     // class-major index of the sample
        // its class: the last one whose prefix does not exceed g (empty classes share the prefix of
        // the next non-empty one, which is the one meant)
        int lo = 0, hi = NCLS - 1;
        if (lane < n) {
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (s_pre[mid] <= g) lo = mid; else hi = mid - 1;
            }
        }
        pk = lo;
        ps = lane < n ? g - s_pre[lo] : 0;
    }
    __syncthreads();

    if (wave == 1) {
        // written in this very step?  Then the latest candidate that goes there is what the slot holds.
        int fwd = -1;
#pragma unroll 4
        for (int m = 0; m < c; m += 4) {
            const int4 km = *reinterpret_cast<const int4*>(s_ck + m);
            const int4 sm = *reinterpret_cast<const int4*>(s_cslot + m);
            const int4 xm = *reinterpret_cast<const int4*>(s_cx + m);
            if (km.x == pk && sm.x == ps) fwd = xm.x > fwd ? xm.x : fwd;
            if (km.y == pk && sm.y == ps) fwd = xm.y > fwd ? xm.y : fwd;
            if (km.z == pk && sm.z == ps) fwd = xm.z > fwd ? xm.z : fwd;
            if (km.w == pk && sm.w == ps) fwd = xm.w > fwd ? xm.w : fwd;
        }
        if (lane < r) {
            PlanEntry e;
            e.pos = lane < n ? fwd : -1;
            e.label = lane < n ? pk : -1;
            e.row = lane < n ? (int64_t)pk * a.S + ps : -1;
            entry[c + lane] = e;
        }
        if (lane == 0) {
            PlanHeader h;
            h.n = n;
            h.flags = s_flags;
            h.c = c;
            h.r = r;
            *head = h;
        }
    }
}

// The plan of one step on its own (first step of a sequence).
__global__ void __launch_bounds__(TPB) rb_plan_kernel(const PlanArgs a)
{
    extern __shared__ uint32_t lds[];
    plan_step(a, lds);
}

// ---------------------------------------------------------------------------
// One step by its table: workgroup (e, tile) moves one tile of row e (candidates
// first, then representatives); with plan_next the first workgroup of the grid
// plans the next step instead.
// ---------------------------------------------------------------------------
template <int U, bool NT, int ST>           // ST: RB_STORE_*, the form binary32 samples are stored in (row_vec counts stored vectors)
__global__ void __launch_bounds__(TPB) rb_step_planned_kernel(const MoveArgs m, const PlanArgs next)
{
    extern __shared__ uint32_t lds[];
    const bool plan_next = m.plan_next != 0;
    if (plan_next && blockIdx.x == 0) {        // dispatched first: it has the longest way to go
        plan_step(next, lds);
        return;
    }
    const int mover = blockIdx.x - (plan_next ? 1 : 0);
    // Consecutive workgroups go to the eight accelerator dies in turn, and each die translates
    // addresses for itself: all tiles of a row are given to workgroups of one die (rows are dealt
    // to the dies in turn), so that a die touches an eighth of the rows' pages instead of all.
    int e, tile;
    const int rows = m.c + m.r, dealt = rows / XCDS * XCDS;
    if (mover < dealt * m.tpr) {
        const int die = mover % XCDS, i = mover / XCDS;
        e = i / m.tpr * XCDS + die;
        tile = i % m.tpr;
    } else {
        e = mover / m.tpr;
        tile = mover % m.tpr;
    }
    const PlanHeader* head = reinterpret_cast<const PlanHeader*>(m.table);
    const PlanEntry en = reinterpret_cast<const PlanEntry*>(m.table + sizeof(PlanHeader))[e];
    int64_t v_lo, v_hi;
    tile_bounds(tile, m.tile_vec, m.tile_rem, m.row_vec, v_lo, v_hi);
    const bool first = tile == 0 && threadIdx.x == 0;
    if (mover == 0 && threadIdx.x == 0) {
        const PlanHeader h = *head;
        m.state->last_n = h.n;
        if (h.flags != 0) atomicOr(&m.state->flags, h.flags);
    }
    constexpr int WIDE = stored_wide(ST);         // vectors of a mini-batch / output row per vector of a stored row
    if (e < m.c) {
        if (en.row < 0) return;                 // label outside [0, K), or a later class-mate takes the slot
        if (first) { m.buf_y[en.row] = en.label; count_moved(m.state); }
        Tile<U, NT, TPB, true, stored_cv(ST, CV_NARROW)> t;
        t.load(m.batch_x + (int64_t)en.pos * m.row_vec * WIDE, v_lo, v_hi);
        t.store(m.buf_x + en.row * m.row_vec, v_lo, v_hi);
        return;
    }
    const int j = e - m.c;
    if (first) m.out_y[j] = en.label;           // -1 when fewer samples are stored than asked for
    if (en.label < 0) return;
    if (first) count_moved(m.state);
    vec16* dst = m.out_x + (int64_t)j * m.row_vec * WIDE;
    if (ST != RB_STORE_SAME && en.pos >= 0) {
        // forwarded from the mini-batch: what the slot will hold is the row in its stored form
        Tile<U, NT, TPB, true, stored_cv(ST, CV_BOTH)> t;
        t.load(m.batch_x + (int64_t)en.pos * m.row_vec * WIDE, v_lo, v_hi);
        t.store(dst, v_lo, v_hi);
    } else {
        const vec16* src = en.pos >= 0 ? m.batch_x + (int64_t)en.pos * m.row_vec : m.buf_x + en.row * m.row_vec;
        Tile<U, NT, TPB, true, stored_cv(ST, CV_WIDEN)> t;
        t.load(src, v_lo, v_hi);
        t.store(dst, v_lo, v_hi);
    }
}

}  // namespace
