// Small-count kernels (at most 64 candidates / representatives): the plan is computed by one wavefront per workgroup; includes the single-launch update + sample kernel.
// Included by rb.hip only, after rb_device.h.
#pragma once

#include "rb_device.h"

namespace {

constexpr int YPRE = 4;    // label loads per thread issued before anything else (covers b <= 1024)

// Labels of the whole mini-batch into LDS (LAB_INVALID when outside [0, K)).  The
// first YPRE per thread were requested earlier into yv[]; called by all threads.
__device__ __forceinline__ void park_labels(const int64_t (&yv)[YPRE], const int64_t* __restrict__ batch_y,
                                            int b, int K, int32_t* s_y)
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int u = 0; u < YPRE; ++u) {
        const int q = tid + u * TPB;
        int64_t y = yv[u];
        // keeps the compiler from evaluating the range test (and so waiting for the load) any
        // earlier than here; the loads are meant to stay in flight across the code before
        asm volatile("" : "+v"(y));
        if (q < b) s_y[q] = (y >= 0 && y < K) ? (int32_t)y : LAB_INVALID;
    }
    for (int q = tid + YPRE * TPB; q < b; q += TPB) {
        const int64_t y = batch_y[q];
        s_y[q] = (y >= 0 && y < K) ? (int32_t)y : LAB_INVALID;
    }
}

// ---------------------------------------------------------------------------
// Pieces of the plan shared by the small-count kernels.  Called by wavefront 0
// only, with all of its 64 lanes active.
// ---------------------------------------------------------------------------

// Floyd's c-subset of the b mini-batch positions, all draws at once: lane i < c
// draws t_i uniform in [0, b-c+i]; the sequential algorithm replaces t_i by
// b-c+i when t_i was chosen before, which is the case iff an earlier lane drew
// the same value, or t_i = b-c+q for an earlier q whose own draw was replaced.
// Returns the lane's candidate position (0 for lanes >= c); s_first: b words of LDS.
__device__ __forceinline__ int wave_select(const Seed& sd, int b, int c, uint32_t* s_first, bool& active)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int base = b - c;
    active = lane < c;
    const uint32_t t = active ? (uint32_t)below(sd, PURPOSE_SELECT, (uint32_t)lane, (uint64_t)(base + lane + 1)) : 0u;
    if (active) s_first[t] = 0xFFFFFFFFu;
    if (active) atomicMin(&s_first[t], (uint32_t)lane);
    const bool dup = active && s_first[t] != (uint32_t)lane;
    const int packed = (int)(t | (dup ? 0x80000000u : 0u));      // t < 4096: bit 31 is free for the flag
    int cur = lane;
    bool taken = false, done = !active;
    while (__ballot(!done) != 0) {
        const int pc = __shfl(packed, cur, WAVE);
        if (!done) {
            if (pc < 0) {
                taken = true;
                done = true;
            } else {
                const int q = pc - base;
                if (q < 0 || q >= cur) done = true;
                else cur = q;
            }
        }
    }
    return active ? (taken ? base + lane : (int)t) : 0;
}

// Where candidate i (mini-batch position p, class ki, fill0 samples of that class stored before
// the step) is stored: row index ki*S + slot, or -1 if it is not stored (label outside [0, K),
// or a later class-mate overwrites its slot).  Lane l holds candidate l: position x, class k.
__device__ __forceinline__ int64_t wave_place(const Seed& sd, bool active, int x, int32_t k, int i, int p,
                                              int32_t ki, int64_t fill0, int64_t S)
{
    if (ki < 0) return -1;
    // candidates of class ki; in mini-batch order the one with `rank` class-mates
    // before it is insertion number fill0 + rank of the class
    const bool same = active && k == ki;
    const int total = __popcll(__ballot(same));
    const int rank = __popcll(__ballot(same && x < p));
    if (fill0 + total <= S) return (int64_t)ki * S + fill0 + rank;     // all append: distinct slots
    // Insertions beyond the capacity overwrite a uniformly drawn slot.  This
    // candidate is not stored if a later class-mate overwrites its slot.
    const int draw = same ? (int)below(sd, PURPOSE_EVICT, (uint32_t)x, (uint64_t)S) : -1;
    const int own = fill0 + rank < S ? (int)(fill0 + rank) : lane_read(draw, i);
    uint64_t rivals = __ballot(same && x > p && draw == own);
    while (rivals != 0) {
        const int m = __builtin_ctzll(rivals);
        rivals &= rivals - 1;
        const int xm = __builtin_amdgcn_readlane(x, m);
        const int rank_m = __popcll(__ballot(same && x < xm));
        if (fill0 + rank_m >= S) return -1;                            // m does overwrite
    }
    return (int64_t)ki * S + own;
}

// ---------------------------------------------------------------------------
// rb_update for c <= WAVE candidates: the plan is computed by the first
// wavefront of each workgroup alone, one lane per candidate, with ballots and
// lane reads instead of workgroup scans; the other three wavefronts only move
// data.  Same grid and arguments as rb_update_kernel.
//
// LDS (dynamic): s_first[b] u32 (lowest lane that drew a value), s_y[b] i32
// (label of every mini-batch position, LAB_INVALID when outside [0, K)).
// ---------------------------------------------------------------------------
template <int U, bool NT>
__global__ void __launch_bounds__(TPB) rb_update_small_kernel(const UpdateArgs a)
{
    extern __shared__ uint32_t lds[];
    uint32_t* s_first = lds;                                   // [b]
    int32_t* s_y = reinterpret_cast<int32_t*>(lds + a.b);      // [b]
    __shared__ int s_wave[NWAVE];
    __shared__ int s_hist[CH];
    __shared__ int s_p[2];          // mini-batch position of the current candidate (double-buffered over rows)
    __shared__ int64_t s_dst[2];    // slot row it is stored to, -1: not stored

    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const bool w0 = tid < WAVE;
    const int b = a.b, c = a.c;

    // all labels of the mini-batch: requested now, parked in LDS once the selection is done
    int64_t yv[YPRE];
#pragma unroll
    for (int u = 0; u < YPRE; ++u) {
        const int q = tid + u * TPB;
        yv[u] = q < b ? a.batch_y[q] : -1;
    }

    // wavefront 0: lane i computes candidate i of Floyd's emission order
    bool active = false;
    int x = 0;                       // its mini-batch position
    if (w0) x = wave_select(a.sd, b, c, s_first, active);

    if ((int)blockIdx.x < a.nchunks) {
        // ---- bookkeeping: fill_new = min(fill_old + candidates of the class, S) ----
        park_labels(yv, a.batch_y, b, a.K, s_y);
        const int k_lo = blockIdx.x * CH;
        s_hist[tid] = 0;
        __syncthreads();
        if (w0) {
            const int32_t k = active ? s_y[x] : LAB_UNSELECTED;
            if (active && k >= k_lo && k < k_lo + CH) atomicAdd(&s_hist[k - k_lo], 1);
            if (blockIdx.x == 0 && __ballot(active && k == LAB_INVALID) != 0 && lane == 0)
                atomicOr(&a.state->flags, RB_FLAG_BAD_LABEL);
        }
        __syncthreads();
        const int kk = k_lo + tid;
        int32_t nf = 0;
        if (kk < a.K) {
            int64_t v = (int64_t)a.fill_old[kk] + s_hist[tid];
            nf = (int32_t)(v < a.S ? v : a.S);
            a.fill_new[kk] = nf;
        }
        int total;
        block_scan_excl(nf, total, s_wave);
        if (tid == 0) a.chunk_new[blockIdx.x] = total;
        return;
    }

    // ---- movers ---------------------------------------------------------------
    const int mover = blockIdx.x - a.nchunks;
    const int group = mover / a.tpr, tile = mover % a.tpr;
    int64_t v_lo, v_hi;
    tile_bounds(tile, a.tile_vec, a.tile_rem, a.row_vec, v_lo, v_hi);

    // The first row is handled outside the loop over further rows: the label loads are still in
    // flight here and a loop header would make the compiler wait for them before the barrier.
    int32_t k = LAB_UNSELECTED;      // wavefront 0: class of the lane's candidate
    {
        const int i = group * a.rpb;           // candidate, in Floyd emission order
        if (i >= c) return;
        if (w0) {
            const int pi = lane_read(x, i);
            if (lane == 0) s_p[0] = pi;
        }
        __syncthreads();
        const int p = s_p[0];
        // The row is requested as soon as its position is known: before the labels have
        // arrived, and long before wavefront 0 has worked out where it goes.
        Tile<U, NT> t;
        t.load(a.batch_x + (int64_t)p * a.row_vec, v_lo, v_hi);
        park_labels(yv, a.batch_y, b, a.K, s_y);
        __syncthreads();
        if (w0) {
            k = active ? s_y[x] : LAB_UNSELECTED;
            const int32_t ki = lane_read(k, i);
            const int64_t dst = wave_place(a.sd, active, x, k, i, p, ki, ki >= 0 ? a.fill_old[ki] : 0, a.S);
            if (lane == 0) s_dst[0] = dst;
        }
        __syncthreads();
        const int64_t dst_row = s_dst[0];
        if (dst_row >= 0) {
            t.store(a.buf_x + dst_row * a.row_vec, v_lo, v_hi);
            if (tile == 0 && tid == 0) { a.buf_y[dst_row] = dst_row / a.S; count_moved(a.state); }
        }
    }
    for (int rr = 1; rr < a.rpb; ++rr) {
        const int i = group * a.rpb + rr;
        if (i >= c) break;
        const int par = rr & 1;
        if (w0) {
            const int pi = lane_read(x, i);
            if (lane == 0) s_p[par] = pi;
        }
        __syncthreads();
        const int p = s_p[par];
        Tile<U, NT> t;
        t.load(a.batch_x + (int64_t)p * a.row_vec, v_lo, v_hi);
        if (w0) {
            const int32_t ki = lane_read(k, i);
            const int64_t dst = wave_place(a.sd, active, x, k, i, p, ki, ki >= 0 ? a.fill_old[ki] : 0, a.S);
            if (lane == 0) s_dst[par] = dst;
        }
        __syncthreads();
        const int64_t dst_row = s_dst[par];
        if (dst_row >= 0) {
            t.store(a.buf_x + dst_row * a.row_vec, v_lo, v_hi);
            if (tile == 0 && tid == 0) { a.buf_y[dst_row] = dst_row / a.S; count_moved(a.state); }
        }
    }
}

// ---------------------------------------------------------------------------
// rb_sample_augment for r <= WAVE representatives and at most WAVE chunks of
// classes: the first wavefront of each workgroup computes the plan, the others
// only move data.  Up to DIRECT_CHUNKS chunks the wavefront reads every fill
// count at once (16 consecutive classes per lane); above, lane ch reads the sum
// of chunk ch and the CH counts of the one chunk that holds the wanted sample
// are read afterwards (4 consecutive classes per lane).
// ---------------------------------------------------------------------------
constexpr int DIRECT_CHUNKS = 4;

template <int U, bool NT>
__global__ void __launch_bounds__(TPB) rb_sample_small_kernel(const SampleArgs a)
{
    __shared__ int s_pick[2][2];    // (class, slot) of the current row, double-buffered over rows
    __shared__ int s_n;

    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const bool w0 = tid < WAVE;
    const bool direct = a.nchunks <= DIRECT_CHUNKS;

    int n = 0, base = 0;
    uint32_t t = 0xFFFFFFFFu;       // wavefront 0, lane i < n: Floyd draw i
    int fv[16];                     // direct: fill counts of classes [16*lane, 16*lane + 16)
    int cs = 0, incl = 0;           // direct: samples in / up to the lane's 16 classes; else: in / up to chunk `lane`
    if (w0) {
        // the fill counts are requested first; the random bits do not depend on them
        // (only their reduction to [0, F-n+i] does) and are computed while the loads fly
        if (direct) {
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const int first = 16 * lane + 4 * m;
                int4 f = make_int4(0, 0, 0, 0);
                if (first < a.nchunks * CH) f = *reinterpret_cast<const int4*>(a.fill + first);
                fv[4 * m] = f.x; fv[4 * m + 1] = f.y; fv[4 * m + 2] = f.z; fv[4 * m + 3] = f.w;
            }
        } else {
            cs = lane < a.nchunks ? a.chunk[lane] : 0;
        }
        const uint64_t bits = lane < a.r ? draw64(a.sd, PURPOSE_SAMPLE, (uint32_t)lane) : 0;
        if (direct) {
#pragma unroll
            for (int m = 0; m < 16; ++m) cs += fv[m];
        }
        incl = wave_scan_incl(cs);
        const int F = lane_read(incl, WAVE - 1);
        n = a.r < F ? a.r : F;
        base = F - n;
        if (lane < n) t = (uint32_t)__umul64hi(bits, (uint64_t)base + lane + 1);
        if (lane == 0) {
            s_n = n;
            if (blockIdx.x == 0) a.state->last_n = n;
        }
    }

    const int group = blockIdx.x / a.tpr, tile = blockIdx.x % a.tpr;
    int64_t v_lo, v_hi;
    tile_bounds(tile, a.tile_vec, a.tile_rem, a.row_vec, v_lo, v_hi);

    for (int rr = 0; rr < a.rpb; ++rr) {
        const int j = group * a.rpb + rr;      // output row
        if (j >= a.r) break;
        const int par = rr & 1;
        if (w0 && j < n) {
            if (lane == 0) { s_pick[par][0] = 0; s_pick[par][1] = 0; }   // never left undefined
            // Floyd: draw j is replaced by base + j iff an earlier draw had the same value, or
            // it equals base + q for an earlier q whose own draw was replaced.
            int cur = j;
            bool taken = false;
            for (;;) {
                const uint32_t tc = (uint32_t)lane_read((int)t, cur);
                if (__ballot(lane < cur && t == tc) != 0) { taken = true; break; }
                const int64_t q = (int64_t)tc - base;
                if (q < 0 || q >= cur) break;
                cur = (int)q;
            }
            const int gj = taken ? base + j : lane_read((int)t, j);   // class-major index of the sample
            if (direct) {
                int acc = incl - cs;
                if (gj >= acc && gj < incl) {
                    int u = 0;
#pragma unroll
                    for (int m = 0; m < 15; ++m) {
                        if (u == m && gj >= acc + fv[m]) { acc += fv[m]; u = m + 1; }
                    }
                    s_pick[par][0] = 16 * lane + u;
                    s_pick[par][1] = gj - acc;
                }
            } else {
                // chunk holding gj: the number of chunks that end at or before it
                const int ch = __popcll(__ballot(lane < a.nchunks && incl <= gj));
                const int gl = gj - (lane_read(incl, ch) - lane_read(cs, ch));
                const int4 f = *reinterpret_cast<const int4*>(a.fill + (int64_t)ch * CH + 4 * lane);
                const int local = f.x + f.y + f.z + f.w;
                const int lincl = wave_scan_incl(local);
                int acc = lincl - local;
                if (gl >= acc && gl < lincl) {
                    int u = 0;
                    if (gl >= acc + f.x) { acc += f.x; u = 1;
                        if (gl >= acc + f.y) { acc += f.y; u = 2;
                            if (gl >= acc + f.z) { acc += f.z; u = 3; } } }
                    s_pick[par][0] = ch * CH + 4 * lane + u;
                    s_pick[par][1] = gl - acc;
                }
            }
        }
        __syncthreads();
        if (j >= s_n) {                        // fewer stored samples than asked for
            if (tile == 0 && tid == 0) a.out_y[j] = -1;
            continue;
        }
        const int pk = s_pick[par][0], ps = s_pick[par][1];
        Tile<U, NT> t2;
        t2.load(a.buf_x + ((int64_t)pk * a.S + ps) * a.row_vec, v_lo, v_hi);
        t2.store(a.out_x + (int64_t)j * a.row_vec, v_lo, v_hi);
        if (tile == 0 && tid == 0) { a.out_y[j] = pk; count_moved(a.state); }
    }
}

// ---------------------------------------------------------------------------
// rb_update_sample, c <= WAVE, r <= WAVE, at most DIRECT_CHUNKS chunks of
// classes: update and sampling of one step in ONE launch.
//
// Grid: bookkeeping workgroups, then the movers of the c candidate rows
// (exactly as in rb_update_small_kernel), then the movers of the r
// representative rows.  A representative mover cannot read the fill counts
// the bookkeeping workgroups of the same launch are writing, so it derives
// them itself: old counts + a histogram of this step's candidates.  A
// representative whose slot is written in this very step is copied from the
// mini-batch row that is being stored there ("forwarding"), never from the
// slot, so no workgroup reads a row another one is writing.
//
// LDS (dynamic): s_first[b], s_y[b] as in rb_update_small_kernel, then
// s_old[DIRECT_CHUNKS*CH] (fill counts before the step) and
// s_cnt[DIRECT_CHUNKS*CH] (candidates of each class in this step).
// ---------------------------------------------------------------------------

template <int U, bool NT>
__global__ void __launch_bounds__(TPB) rb_step_small_kernel(const StepArgs sa)
{
    const UpdateArgs& a = sa.u;
    constexpr int NCLS = DIRECT_CHUNKS * CH;
    extern __shared__ uint32_t lds[];
    uint32_t* s_first = lds;                                       // [b]
    int32_t* s_y = reinterpret_cast<int32_t*>(lds + a.b);          // [b]
    int32_t* s_old = reinterpret_cast<int32_t*>(lds + ((2 * a.b + 3) & ~3));   // [NCLS], 16-byte aligned
    int32_t* s_cnt = s_old + NCLS;                                 // [NCLS]
    __shared__ int s_wave[NWAVE];
    __shared__ int s_hist[CH];
    __shared__ int s_p;             // candidate mover: mini-batch position of the row
    __shared__ int64_t s_dst;       // candidate mover: slot row it is stored to, -1: not stored
    __shared__ int s_n;             // representative mover: n = min(r, F)
    __shared__ int s_pick[3];       // representative mover: class, slot, forwarding position (-1: read the slot)
    __shared__ uint64_t s_bits[WAVE];   // representative mover: random bits of sampling draw i, made by wavefront 1

    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const bool w0 = tid < WAVE;
    const int b = a.b, c = a.c;
    const bool gather = (int)blockIdx.x >= sa.first_gather;

    // labels of the mini-batch (and, for representative movers, the fill counts): requested now
    int64_t yv[YPRE];
#pragma unroll
    for (int u = 0; u < YPRE; ++u) {
        const int q = tid + u * TPB;
        yv[u] = q < b ? a.batch_y[q] : -1;
    }
    int4 fo = make_int4(0, 0, 0, 0);
    if (gather && 4 * tid < a.nchunks * CH) fo = *reinterpret_cast<const int4*>(a.fill_old + 4 * tid);

    // wavefront 0 selects the candidates while wavefront 1 makes the random bits of the sampling draws
    bool active = false;
    int x = 0;
    if (w0) {
        x = wave_select(a.sd, b, c, s_first, active);
    } else if (gather && tid < 2 * WAVE) {
        if (lane < sa.r) s_bits[lane] = draw64(a.sd, PURPOSE_SAMPLE, (uint32_t)lane);
    }

    if ((int)blockIdx.x < a.nchunks) {
        // ---- bookkeeping: fill_new = min(fill_old + candidates of the class, S) ----
        park_labels(yv, a.batch_y, b, a.K, s_y);
        const int k_lo = blockIdx.x * CH;
        s_hist[tid] = 0;
        __syncthreads();
        if (w0) {
            const int32_t k = active ? s_y[x] : LAB_UNSELECTED;
            if (active && k >= k_lo && k < k_lo + CH) atomicAdd(&s_hist[k - k_lo], 1);
            if (blockIdx.x == 0 && __ballot(active && k == LAB_INVALID) != 0 && lane == 0)
                atomicOr(&a.state->flags, RB_FLAG_BAD_LABEL);
        }
        __syncthreads();
        const int kk = k_lo + tid;
        int32_t nf = 0;
        if (kk < a.K) {
            int64_t v = (int64_t)a.fill_old[kk] + s_hist[tid];
            nf = (int32_t)(v < a.S ? v : a.S);
            a.fill_new[kk] = nf;
        }
        int total;
        block_scan_excl(nf, total, s_wave);
        if (tid == 0) a.chunk_new[blockIdx.x] = total;
        return;
    }

    if (!gather) {
        // ---- candidate movers (rows of the mini-batch into their slots) ----------
        const int mover = blockIdx.x - a.nchunks;
        const int i = mover / a.tpr, tile = mover % a.tpr;     // candidate in Floyd emission order, tile of its row
        int64_t v_lo, v_hi;
        tile_bounds(tile, a.tile_vec, a.tile_rem, a.row_vec, v_lo, v_hi);
        if (w0) {
            const int pi = lane_read(x, i);
            if (lane == 0) s_p = pi;
        }
        __syncthreads();
        const int p = s_p;
        // requested as soon as the position is known, before the labels have arrived
        Tile<U, NT> t;
        t.load(a.batch_x + (int64_t)p * a.row_vec, v_lo, v_hi);
        park_labels(yv, a.batch_y, b, a.K, s_y);
        __syncthreads();
        if (w0) {
            const int32_t k = active ? s_y[x] : LAB_UNSELECTED;
            const int32_t ki = lane_read(k, i);
            const int64_t dst = wave_place(a.sd, active, x, k, i, p, ki, ki >= 0 ? a.fill_old[ki] : 0, a.S);
            if (lane == 0) s_dst = dst;
        }
        __syncthreads();
        const int64_t dst_row = s_dst;
        if (dst_row >= 0) {
            t.store(a.buf_x + dst_row * a.row_vec, v_lo, v_hi);
            if (tile == 0 && tid == 0) { a.buf_y[dst_row] = dst_row / a.S; count_moved(a.state); }
        }
        return;
    }

    // ---- representative movers (stored samples into the augmented mini-batch) ---
    const int mover = blockIdx.x - sa.first_gather;
    const int j = mover / a.tpr, tile = mover % a.tpr;         // output row, tile of it
    int64_t v_lo, v_hi;
    tile_bounds(tile, a.tile_vec, a.tile_rem, a.row_vec, v_lo, v_hi);

    park_labels(yv, a.batch_y, b, a.K, s_y);
    *reinterpret_cast<int4*>(s_old + 4 * tid) = fo;
    *reinterpret_cast<int4*>(s_cnt + 4 * tid) = make_int4(0, 0, 0, 0);
    __syncthreads();
    if (w0) {
        const int32_t k = active ? s_y[x] : LAB_UNSELECTED;
        if (active && k >= 0) atomicAdd(&s_cnt[k], 1);
        // fill counts after this step's update, 16 consecutive classes per lane
        int fv[16];
        int cs = 0;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int64_t v = (int64_t)s_old[16 * lane + m] + s_cnt[16 * lane + m];
            fv[m] = (int)(v < a.S ? v : a.S);
            cs += fv[m];
        }
        const int incl = wave_scan_incl(cs);
        const int F = lane_read(incl, WAVE - 1);
        const int n = sa.r < F ? sa.r : F;
        const int base = F - n;
        uint32_t t = 0xFFFFFFFFu;
        if (lane < n) t = (uint32_t)__umul64hi(s_bits[lane], (uint64_t)base + lane + 1);
        if (lane == 0) {
            s_n = n;
            s_pick[0] = 0; s_pick[1] = 0; s_pick[2] = -1;
            if (mover == 0) a.state->last_n = n;
        }
        if (j < n) {
            // Floyd: draw j is replaced by base + j iff an earlier draw had the same value, or
            // it equals base + q for an earlier q whose own draw was replaced.
            int cur = j;
            bool taken = false;
            for (;;) {
                const uint32_t tc = (uint32_t)lane_read((int)t, cur);
                if (__ballot(lane < cur && t == tc) != 0) { taken = true; break; }
                const int64_t q = (int64_t)tc - base;
                if (q < 0 || q >= cur) break;
                cur = (int)q;
            }
            const int gj = taken ? base + j : lane_read((int)t, j);   // class-major index of the sample
            // locate it: the lane whose 16 classes hold it walks them
            int acc = incl - cs;
            const bool mine = gj >= acc && gj < incl;
            int u = 0;
            if (mine) {
#pragma unroll
                for (int m = 0; m < 15; ++m) {
                    if (u == m && gj >= acc + fv[m]) { acc += fv[m]; u = m + 1; }
                }
            }
            const int owner = __builtin_ctzll(__ballot(mine) | (1ull << 63));
            const int pk = lane_read(16 * lane + u, owner);
            const int ps = lane_read(gj - acc, owner);

            // Is slot ps of class pk written in this step, and by which candidate?
            const bool same = active && k == pk;
            const uint64_t same_mask = __ballot(same);
            const int64_t fill0 = s_old[pk];
            int fwd = -1;
            if (same_mask != 0 && (ps >= fill0 || fill0 + __popcll(same_mask) > a.S)) {
                int my_rank = 0;                       // class-mates earlier in the mini-batch
                uint64_t sm = same_mask;
                while (sm != 0) {
                    const int m = __builtin_ctzll(sm);
                    sm &= sm - 1;
                    my_rank += (int)(__builtin_amdgcn_readlane(x, m) < x);
                }
                int slot = -1;
                if (same) {
                    const int64_t at = fill0 + my_rank;
                    slot = (int)(at < a.S ? at : (int64_t)below(a.sd, PURPOSE_EVICT, (uint32_t)x, (uint64_t)a.S));
                }
                uint64_t writers = __ballot(same && slot == ps);
                while (writers != 0) {                 // the one latest in the mini-batch is what the slot holds
                    const int m = __builtin_ctzll(writers);
                    writers &= writers - 1;
                    const int xm = __builtin_amdgcn_readlane(x, m);
                    fwd = xm > fwd ? xm : fwd;
                }
            }
            if (lane == 0) { s_pick[0] = pk; s_pick[1] = ps; s_pick[2] = fwd; }
        }
    }
    __syncthreads();
    if (j >= s_n) {                            // fewer stored samples than asked for
        if (tile == 0 && tid == 0) sa.out_y[j] = -1;
        return;
    }
    const int pk = s_pick[0], ps = s_pick[1], fwd = s_pick[2];
    const vec16* src = fwd >= 0 ? a.batch_x + (int64_t)fwd * a.row_vec
                                : a.buf_x + ((int64_t)pk * a.S + ps) * a.row_vec;
    Tile<U, NT> t;
    t.load(src, v_lo, v_hi);
    t.store(sa.out_x + (int64_t)j * a.row_vec, v_lo, v_hi);
    if (tile == 0 && tid == 0) { sa.out_y[j] = pk; count_moved(a.state); }
}

}  // namespace
