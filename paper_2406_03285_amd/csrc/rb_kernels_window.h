// Several steps per launch (rb_update_sample_many, at most 64 candidates and representatives, at
// most 1024 classes, exact selection; any replacement strategy, any storage form): one workgroup
// plans a whole window of steps, one after the other, while the other workgroups of the same launch
// move the previous window's rows; the window's own launch then moves the rows of all its steps at
// once by the table the planner left.  (The host sends shapes whose rows move sooner than that one
// workgroup plans to rb_kernels_bigwin.h, whose planners work side by side.)
// Included by rb.hip only, after rb_kernels_small.h (whose candidate selection it uses).
#pragma once

#include "rb_device.h"
#include "rb_kernels_small.h"

namespace {

constexpr int WIN_MAX = 32;                   // most steps one launch covers ...
constexpr int WIN_ENTRIES = 1280;             // ... as long as steps * (c + r) table entries do not exceed this
constexpr int WIN_SLOTS = 640;                // ... and steps * max(c, r) not this (per-step arrays of the planner)
constexpr int WIN_PACE = 64;                  // stores of a tile go out in one burst once its loads have arrived (no wait between them)
constexpr int WIN_HASH = 2048;                // slots of the window's table of buffer rows (at most WIN_ENTRIES keys)
// (The planner's LDS, 32.5 KB - 36.6 KB with the replacement strategies' state -, is reserved for every workgroup of the launch, the movers included: four of them
// share a compute unit.  Tables of twice the size left room for two, which cost the 16-row steps 8 % of their rate.)
constexpr uint32_t WIN_NONE = 0xFFFFu;        // "no entry" in the 16-bit links below
constexpr uint32_t WIN_EMPTY = 0xFFFFFFFFu;   // free slot of the row table (no buffer row has this index)

// Steps of one launch share the buffer, so the planner resolves what the stream order resolves
// between separate launches:
//   - a representative whose slot is written earlier in the window (or in its own step) is copied
//     from the mini-batch row that was stored there;
//   - of several writes to one slot only the last one is carried out;
//   - a representative that needs what a slot held BEFORE the window, while a later step of the
//     window overwrites that slot, is served by the workgroups that carry out that write: each of
//     them first copies its tile of the old content to the representative's row, then overwrites it.
struct WinHeader {        // one per step
    int32_t n;            // representatives the step hands out: min(r, F)
    uint32_t flags;       // RB_FLAG_* raised by the step
    int32_t pad[2];
};
struct WinEntry {         // 32 bytes; entry index = step * (c + r) + (candidate i | c + representative j)
    int32_t src;          // candidate: its mini-batch position.  representative: -1 = read the slot, else
                          // (step in the window << 16 | mini-batch position) of the row stored there
    int32_t label;        // class; representative: -1 = fewer samples stored than asked for
    int64_t row;          // candidate: slot row it is written to, -1 = not written by this launch.
                          // representative: slot row it is read from
    int32_t chain;        // candidate: first representative (entry index) that gets the slot's old content
                          // from this candidate's workgroups, -1 = none.  representative: the next one of that chain
    int32_t handled;      // representative: 1 = served by a candidate's workgroups, its own do nothing
    int32_t pad[2];
};
constexpr size_t WIN_TABLE_BYTES = (WIN_MAX * sizeof(WinHeader) + WIN_ENTRIES * sizeof(WinEntry) + 255) / 256 * 256;

struct WinPlanArgs {
    const int64_t* batch_y[WIN_MAX];   // labels of the steps that are planned
    const int32_t* fill_old;           // fill counts before the window
    int32_t* fill_new;                 // ... and after it
    int32_t* chunk_new;
    char* table;
    uint32_t seed_lo, seed_hi;
    uint64_t first_step;
    int32_t w;                         // steps in the window
    int32_t b, c, r;
    int32_t K, nchunks;
    int64_t S;
    int32_t eviction;                  // RB_EVICT_*
    const int32_t* aux_old;            // per class: FIFO: slot of the oldest sample; RESERVOIR: samples offered so far
    int32_t* aux_new;
};

struct WinMoveArgs {
    const vec16* batch_x[WIN_MAX];
    vec16* out_x[WIN_MAX];
    int64_t* out_y[WIN_MAX];
    vec16* buf_x;
    int64_t* buf_y;
    const char* table;
    DevState* state;
    int32_t w, c, r;
    int64_t S;
    int64_t row_vec;
    int32_t tpr, tile_vec, tile_rem;
};

// block_scan_excl of rb_device.h with that barrier.
__device__ __forceinline__ int block_scan_excl_lds(int v, int& total, int* s_wave)
{
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    const int inc = wave_scan_incl(v);
    if (lane == WAVE - 1) s_wave[w] = inc;
    lds_barrier();
    int before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < NWAVE; ++i) {
        const int x = s_wave[i];
        all += x;
        if (i < w) before += x;
    }
    lds_barrier();
    total = all;
    return before + inc - v;
}

__device__ __forceinline__ uint32_t win_hash(uint32_t row)
{
    return (row * 2654435761u) >> 21;          // 11 bits: WIN_HASH slots
}

// Slot of `row` in the row table, inserting it if it is not there (open addressing; the table
// never fills: at most WIN_ENTRIES of its WIN_HASH slots are ever used).
__device__ __forceinline__ int win_find_or_insert(uint32_t* s_hkey, uint32_t row)
{
    uint32_t h = win_hash(row);
    for (;;) {
        const uint32_t prev = atomicCAS(&s_hkey[h], WIN_EMPTY, row);
        if (prev == WIN_EMPTY || prev == row) return (int)h;
        h = (h + 1) & (WIN_HASH - 1);
    }
}

// Orders the LDS traffic of ONE wavefront: what its lanes wrote before is what its lanes read after
// (the lanes run in lockstep; this only keeps the compiler from moving or merging the accesses).
__device__ __forceinline__ void wave_fence()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
}

// What wavefront 0 knows of a step's candidates before they enter the row table (one lane each).
struct WinCand {
    int x;            // mini-batch position
    int32_t k;        // class, LAB_* when not a valid candidate
    int fill0;        // samples of the class stored before the step
    int rank, total;  // class-mates earlier in the mini-batch / in all
    int slot;         // slot within the class: appended, or the one it overwrites when the class is full; -1: not kept
    int32_t aux0;     // the class's FIFO / reservoir state before the step
    bool valid, bad, any_over;
};

// ---------------------------------------------------------------------------
// The plan of a.w consecutive steps by one workgroup (all TPB threads call it).
// Before the first step the wavefronts share the steps: each selects the
// candidates of its steps (which depends on nothing but the seed) and requests
// their labels, so that the only global loads the steps wait for are issued once,
// all together.  Then, per step: wavefront 0 = one lane per candidate, all
// threads = prefix of the fill counts over the classes, wavefront 1 = one lane
// per representative; the fill counts stay in LDS from step to step.  The part
// of a step's candidates that does not need the row table (insertion numbers,
// eviction draws: win_candidates) runs in wavefront 0 while wavefront 1 still
// works on the representatives of the step before; only entering the row table
// is serial.  No dynamic LDS.
// ---------------------------------------------------------------------------
struct WinLds {
    int32_t* s_fill;      // [NCLS] fill counts, carried from step to step
    int32_t* s_ck;        // [WAVE] candidate classes, positions, scratch (wavefront 0 only)
    int32_t* s_cx;
    int32_t* s_cw;
    const int32_t* s_aux;     // [NCLS] per-class state of the FIFO / reservoir strategies (only with them)
    const uint16_t* s_wpos;   // [WIN_SLOTS] mini-batch position of every step's candidates (step * max(c, r) + i)
    const int16_t* s_lab;     // [WIN_SLOTS] ... and their classes (LAB_INVALID when outside [0, K))
    int stride;               // of the per-step arrays: max(c, r)
};

__device__ __forceinline__ Seed win_seed(const WinPlanArgs& a, int s)
{
    Seed sd;
    sd.seed_lo = a.seed_lo; sd.seed_hi = a.seed_hi;
    sd.step_lo = (uint32_t)(a.first_step + s); sd.step_hi = (uint32_t)((a.first_step + s) >> 32);
    return sd;
}

// Labels of step s of the window.  All WIN_MAX pointers are read from the kernel arguments at fixed offsets (one
// batch of scalar loads at kernel entry) and the one asked for is picked by comparisons: an argument read at a
// computed offset is a second, dependent trip to wherever the arguments live.
__device__ __forceinline__ const int64_t* win_labels(const WinPlanArgs& a, int s)
{
    const int64_t* p = a.batch_y[0];
#pragma unroll
    for (int i = 1; i < WIN_MAX; ++i) p = s == i ? a.batch_y[i] : p;
    return p;
}

// Wavefront 0: candidates of step s, up to the slot each one asks for.  Needs the fill counts after step s-1.
// AUX: the replacement strategy is FIFO or reservoir (Alg. 1 with the variants of its line 5).
template <bool AUX>
__device__ __forceinline__ WinCand win_candidates(const WinPlanArgs& a, int s, const WinLds& l)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const Seed sd = win_seed(a, s);
    WinCand cd;
    const int x = lane < a.c ? l.s_wpos[s * l.stride + lane] : 0;
    const int32_t k = lane < a.c ? l.s_lab[s * l.stride + lane] : LAB_UNSELECTED;
    cd.x = x;
    cd.k = k;
    cd.valid = k >= 0;
    cd.bad = __ballot(k == LAB_INVALID) != 0;
    l.s_ck[lane] = cd.valid ? k : -1;
    l.s_cx[lane] = x;
    cd.fill0 = cd.valid ? l.s_fill[k] : 0;
    wave_fence();
    // insertion number within the class: fill0 + class-mates earlier in the mini-batch
    int rank = 0, total = 0;
#pragma unroll 4
    for (int m = 0; m < a.c; m += 4) {
        const int4 km = *reinterpret_cast<const int4*>(l.s_ck + m);
        const int4 xm = *reinterpret_cast<const int4*>(l.s_cx + m);
        rank += (int)(km.x == k && xm.x < x) + (int)(km.y == k && xm.y < x) + (int)(km.z == k && xm.z < x) +
                (int)(km.w == k && xm.w < x);
        total += (int)(km.x == k) + (int)(km.y == k) + (int)(km.z == k) + (int)(km.w == k);
    }
    cd.rank = rank;
    cd.total = total;
    const int64_t at = (int64_t)cd.fill0 + rank;
    const bool over = cd.valid && at >= a.S;       // beyond the capacity: overwrites a stored sample
    cd.slot = cd.valid ? (int)at : -1;
    cd.any_over = __ballot(over) != 0;
    cd.aux0 = 0;
    if (!AUX) {
        if (over) cd.slot = (int)below(sd, PURPOSE_EVICT, (uint32_t)x, (uint64_t)a.S);      // a uniformly drawn one
    } else {
        cd.aux0 = cd.valid ? l.s_aux[k] : 0;
        if (a.eviction == RB_EVICT_FIFO) {
            if (over) cd.slot = (int)(((int64_t)cd.aux0 + at - a.S) % a.S);                   // the oldest one
        } else if (over) {
            // reservoir: kept with probability S / (samples offered to the class so far + 1), then in a uniform slot
            const int64_t offers = (int64_t)cd.aux0 + rank < INT32_MAX ? (int64_t)cd.aux0 + rank : INT32_MAX;
            const int64_t draw = (int64_t)below(sd, PURPOSE_EVICT, (uint32_t)x, (uint64_t)offers + 1);
            cd.slot = draw < a.S ? (int)draw : -1;
        }
    }
    return cd;
}

template <bool AUX>
__device__ __forceinline__ void plan_window(const WinPlanArgs& a)
{
    constexpr int NCLS = DIRECT_CHUNKS * CH;
    __shared__ __align__(16) int32_t s_fill[NCLS];    // fill counts, carried from step to step
    __shared__ __align__(16) int32_t s_aux[AUX ? NCLS : 4];   // FIFO / reservoir state of the classes, carried likewise
    __shared__ __align__(16) int32_t s_pre[NCLS];     // stored samples in the classes before each class, after the step's update
    __shared__ uint32_t s_h[2 * WIN_HASH];
    uint32_t* s_hkey = s_h;                           // buffer rows the window touches ...
    uint32_t* s_hval = s_h + WIN_HASH;                // ... low half: entry of the last candidate written there; high half:
                                                      //     head of the chain of representatives that read its old content
                                                      // (before the first step: the scratch of the candidate selection)
    __shared__ uint64_t s_bits[WIN_SLOTS];            // random bits of every step's sampling draws (step * max(c, r) + j)
    __shared__ uint16_t s_next[WIN_SLOTS];            // per representative (step * max(c, r) + j): next entry of its chain
    __shared__ uint16_t s_wpos[WIN_SLOTS];            // per candidate (step * max(c, r) + i): its mini-batch position
    __shared__ int16_t s_lab[WIN_SLOTS];              // ... and its class (LAB_INVALID when outside [0, K))
    __shared__ int s_wave[NWAVE];
    __shared__ __align__(16) int32_t s_ck[WAVE], s_cx[WAVE];
    __shared__ __align__(16) uint32_t s_t[WAVE];      // wavefront 1, while it works on the representatives
    int32_t* s_cw = reinterpret_cast<int32_t*>(s_t);  // wavefront 0, while the candidates enter the row table (wavefront 1 waits then)
    __shared__ uint32_t s_flags;

    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const int b = a.b, c = a.c, r = a.r, w = a.w;
    const int stride = c > r ? c : r, rows = c + r;   // of the per-step arrays, and of the table
    WinHeader* head = reinterpret_cast<WinHeader*>(a.table);
    WinEntry* entry = reinterpret_cast<WinEntry*>(a.table + WIN_MAX * sizeof(WinHeader));
    WinLds l;
    l.s_fill = s_fill; l.s_aux = s_aux; l.s_ck = s_ck; l.s_cx = s_cx; l.s_cw = s_cw; l.s_wpos = s_wpos; l.s_lab = s_lab; l.stride = stride;

    // ---- before the first step ----
    int4 fo = make_int4(0, 0, 0, 0), ao = make_int4(0, 0, 0, 0);
    if (4 * tid < a.nchunks * CH) {
        fo = *reinterpret_cast<const int4*>(a.fill_old + 4 * tid);
        if (AUX) ao = *reinterpret_cast<const int4*>(a.aux_old + 4 * tid);
    }
    // candidates of all steps and their labels; a selecting wavefront needs b words of scratch
    const int nsel = b <= 2 * WIN_HASH / NWAVE ? NWAVE : 2;
    constexpr int SEL_MAX = WIN_MAX / 2;              // steps per selecting wavefront at most
    int64_t ylab[SEL_MAX];
    if (wave < nsel) {
        for (int s = wave; s < w; s += nsel) {
            bool active = false;
            const int x = wave_select(win_seed(a, s), b, c, s_h + wave * b, active);
            if (active) s_wpos[s * stride + lane] = (uint16_t)x;
        }
#pragma unroll
        for (int u = 0; u < SEL_MAX; ++u) {           // (every lane reads back what it wrote itself)
            const int s = wave + u * nsel;
            ylab[u] = -1;
            if (s < w && lane < c) ylab[u] = win_labels(a, s)[s_wpos[s * stride + lane]];
        }
    }
    // all sampling bits
    for (int s = wave; s < w; s += NWAVE)
        if (lane < r) s_bits[s * stride + lane] = draw64(win_seed(a, s), PURPOSE_SAMPLE, (uint32_t)lane);
    lds_barrier();
    for (int i = tid; i < WIN_HASH; i += TPB) {       // empty row table
        s_hkey[i] = WIN_EMPTY;
        s_hval[i] = 0xFFFFFFFFu;
    }
    *reinterpret_cast<int4*>(s_fill + 4 * tid) = fo;
    if (AUX) *reinterpret_cast<int4*>(s_aux + 4 * tid) = ao;
    if (tid == 0) s_flags = 0;
    if (wave < nsel) {
#pragma unroll
        for (int u = 0; u < SEL_MAX; ++u) {
            const int s = wave + u * nsel;
            const int64_t y = ylab[u];
            if (s < w && lane < c) s_lab[s * stride + lane] = (int16_t)((y >= 0 && y < a.K) ? (int32_t)y : LAB_INVALID);
        }
    }
    lds_barrier();
    WinCand cd = {};
    if (wave == 0) cd = win_candidates<AUX>(a, 0, l);

    for (int s = 0; s < w; ++s) {
        if (wave == 0) {
            // ---- win_enter: the candidates of step s enter the row table ----
            const int x = cd.x;
            const int32_t k = cd.k;
            const bool valid = cd.valid;
            const bool placed = valid && cd.slot >= 0;       // (a reservoir may not keep a candidate)
            const int64_t row = placed ? (int64_t)k * a.S + cd.slot : -1;
            const int me = s * rows + lane;
            int h = 0;
            // candidates that share a slot share a table slot
            if (placed) h = win_find_or_insert(s_hkey, (uint32_t)row);
            wave_fence();
            const uint32_t v = placed ? s_hval[h] : 0xFFFFFFFFu;
            bool stored = placed;
            if (cd.any_over) {
                // of the candidates that ask for one slot only the last of the mini-batch is stored:
                // one of them (whose lane number lands in the table slot) collects the largest position
                s_cw[lane] = -1;
                wave_fence();
                if (placed) s_hval[h] = (uint32_t)lane;
                wave_fence();
                const int leader = placed ? (int)s_hval[h] : lane;
                wave_fence();
                if (placed) atomicMax(&s_cw[leader], x);
                wave_fence();
                stored = placed && s_cw[leader] == x;
                wave_fence();
            }
            int chain = -1;
            if (stored) {
                const uint32_t before = v & 0xFFFFu, readers = v >> 16;
                if (before != WIN_NONE) {              // an earlier step of the window wrote this slot: that write is dropped
                    entry[before].row = -1;
                    entry[before].chain = -1;
                }
                if (readers != WIN_NONE) chain = (int)readers;   // they read what the slot held before the window
                s_hval[h] = (readers << 16) | (uint32_t)me;
            }
            if (lane < c) {
                WinEntry e;
                e.src = x;
                e.label = valid ? k : -1;
                e.row = stored ? row : -1;
                e.chain = chain;
                e.handled = 0;
                e.pad[0] = 0; e.pad[1] = 0;
                entry[me] = e;
            }
            // the class's fill count (and strategy state) after this step (one lane per class: its first candidate)
            if (valid && cd.rank == 0) {
                const int64_t f = (int64_t)cd.fill0 + cd.total;
                s_fill[k] = (int32_t)(f < a.S ? f : a.S);
                if (AUX) {
                    if (a.eviction == RB_EVICT_FIFO) {
                        // the oldest sample moves on by the number of overwrites
                        s_aux[k] = (int32_t)(((int64_t)cd.aux0 + (f > a.S ? f - a.S : 0)) % a.S);
                    } else {
                        const int64_t seen = (int64_t)cd.aux0 + cd.total;
                        s_aux[k] = (int32_t)(seen < INT32_MAX ? seen : INT32_MAX);
                    }
                }
            }
            if (cd.bad && lane == 0) s_flags |= RB_FLAG_BAD_LABEL;
        }
        lds_barrier();

        // ---- prefix of the fill counts over the classes, four consecutive classes per thread ----
        const int4 f4 = *reinterpret_cast<const int4*>(s_fill + 4 * tid);
        int F;
        int before = block_scan_excl_lds(f4.x + f4.y + f4.z + f4.w, F, s_wave);
        s_pre[4 * tid] = before;
        s_pre[4 * tid + 1] = before + f4.x;
        s_pre[4 * tid + 2] = before + f4.x + f4.y;
        s_pre[4 * tid + 3] = before + f4.x + f4.y + f4.z;
        lds_barrier();

        if (wave == 0) {
            if (s + 1 < w) cd = win_candidates<AUX>(a, s + 1, l);
        } else if (wave == 1) {
            // ---- representatives of step s: lane j = draw j of Floyd's n-subset of the F stored samples ----
            const int n = r < F ? r : F;
            const int base = F - n;
            const uint32_t t = lane < n ? (uint32_t)__umul64hi(s_bits[s * stride + lane], (uint64_t)base + lane + 1) : 0xFFFFFFFFu;
            s_t[lane] = t;
            bool dup = false;                           // an earlier draw had the same value
#pragma unroll 4
            for (int i = 0; i < n; i += 4) {
                const uint4 ti = *reinterpret_cast<const uint4*>(s_t + i);
                dup |= (i < lane && ti.x == t) | (i + 1 < lane && ti.y == t) | (i + 2 < lane && ti.z == t) | (i + 3 < lane && ti.w == t);
            }
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
            const int g = taken ? base + lane : (int)t;
            // class of stored sample number g: the last class with s_pre <= g, by three rounds of
            // independent reads (every 64th class, every 4th, single ones)
            int lo = 0;
            if (lane < n) {
                int cnt = 0;
#pragma unroll
                for (int i = 1; i < NCLS / 64; ++i) cnt += (int)(s_pre[64 * i] <= g);
                lo = 64 * cnt;
                cnt = 0;
#pragma unroll
                for (int i = 1; i < 16; ++i) cnt += (int)(s_pre[lo + 4 * i] <= g);
                lo += 4 * cnt;
                const int4 p4 = *reinterpret_cast<const int4*>(s_pre + lo);
                lo += (int)(p4.y <= g) + (int)(p4.z <= g) + (int)(p4.w <= g);
            }
            const int pk = lo, ps = lane < n ? g - s_pre[lo] : 0;
            const int64_t row = (int64_t)pk * a.S + ps;
            const int me = s * rows + c + lane;
            int src = -1, chain = -1;
            if (lane < n) {
                // the representatives of one step are different samples, so no two lanes share a table slot here
                const int h = win_find_or_insert(s_hkey, (uint32_t)row);
                const uint32_t v = s_hval[h];
                const uint32_t writer = v & 0xFFFFu, readers = v >> 16;
                if (writer != WIN_NONE) {
                    // written in this window (this step included): take the row that was stored there
                    const int ws = (int)writer / rows, wi = (int)writer % rows;
                    src = (ws << 16) | (int)s_wpos[ws * stride + wi];
                } else {
                    // what the slot held before the window: remembered, in case a later step overwrites it
                    chain = readers != WIN_NONE ? (int)readers : -1;
                    s_hval[h] = ((uint32_t)me << 16) | WIN_NONE;
                }
            }
            if (lane < r) s_next[s * stride + lane] = (uint16_t)(chain >= 0 ? chain : (int)WIN_NONE);
            if (lane < r) {
                WinEntry e;
                e.src = src;
                e.label = lane < n ? pk : -1;
                e.row = lane < n ? row : -1;
                e.chain = chain;
                e.handled = 0;
                e.pad[0] = 0; e.pad[1] = 0;
                entry[me] = e;
            }
            if (lane == 0) {
                WinHeader hd;
                hd.n = n;
                hd.flags = s_flags;
                hd.pad[0] = 0; hd.pad[1] = 0;
                head[s] = hd;
            }
        }
        lds_barrier();
    }

    // every table entry has left before any of them is patched below
    __syncthreads();

    // ---- representatives that a candidate's workgroups serve do nothing themselves ----
    for (int i = tid; i < WIN_HASH; i += TPB) {
        const uint32_t v = s_hval[i];
        if (s_hkey[i] == WIN_EMPTY || (v & 0xFFFFu) == WIN_NONE) continue;
        uint32_t e = v >> 16;
        while (e != WIN_NONE) {
            entry[e].handled = 1;
            e = s_next[(e / rows) * stride + (e % rows - c)];
        }
    }

    // ---- fill counts after the window ----
    if (4 * tid < a.nchunks * CH) {
        *reinterpret_cast<int4*>(a.fill_new + 4 * tid) = *reinterpret_cast<const int4*>(s_fill + 4 * tid);
        if (AUX) *reinterpret_cast<int4*>(a.aux_new + 4 * tid) = *reinterpret_cast<const int4*>(s_aux + 4 * tid);
    }
    {
        const int4 f4 = *reinterpret_cast<const int4*>(s_fill + 4 * tid);
        const int wsum = lane_read(wave_scan_incl(f4.x + f4.y + f4.z + f4.w), WAVE - 1);   // a wavefront covers one chunk of CH classes
        if (lane == 0 && wave < a.nchunks) a.chunk_new[wave] = wsum;
    }
}

// The plan of the first window of a call, on its own.
template <bool AUX>
__global__ void __launch_bounds__(TPB) rb_window_plan_kernel(const WinPlanArgs a)
{
    plan_window<AUX>(a);
}

// ---------------------------------------------------------------------------
// All steps of one window by its table: workgroup (step, entry, tile) moves one
// tile of one row; if there is a next window, workgroup 0 plans it instead.  (The
// planner's LDS limits every compute unit to four workgroups of this kernel; five measured no better.  Measured alternatives: the planner as a launch of its own on a second
// stream frees the movers but the events that order the two streams cost more than
// that gains.)
// ---------------------------------------------------------------------------
template <int U, bool NT, int ST, bool AUX>      // ST: RB_STORE_*: binary32 samples are stored as they are, as bfloat16 or as 8-bit
                                                 // codes (row_vec counts stored vectors);
                                                 // AUX: FIFO or reservoir replacement (the planner carries their per-class state)
__global__ void __launch_bounds__(TPB) rb_window_kernel(const WinMoveArgs m, const WinPlanArgs next)
{
    if (next.w > 0 && blockIdx.x == 0) {
        // dispatched first, and first in line whenever it has an instruction ready: the next launch
        // waits for this one workgroup as much as for all the movers
        __builtin_amdgcn_s_setprio(3);
        plan_window<AUX>(next);
        return;
    }
    const int mover = blockIdx.x - (next.w > 0 ? 1 : 0);
    const int rows = m.c + m.r, per_step = rows * m.tpr;
    const int s = mover / per_step, in_step = mover % per_step;
    // all tiles of a row go to workgroups of one die (see rb_step_planned_kernel)
    int e, tile;
    const int dealt = rows / XCDS * XCDS;
    if (in_step < dealt * m.tpr) {
        const int die = in_step % XCDS, i = in_step / XCDS;
        e = i / m.tpr * XCDS + die;
        tile = i % m.tpr;
    } else {
        e = in_step / m.tpr;
        tile = in_step % m.tpr;
    }
    const WinHeader* head = reinterpret_cast<const WinHeader*>(m.table);
    const WinEntry* entry = reinterpret_cast<const WinEntry*>(m.table + WIN_MAX * sizeof(WinHeader));
    const WinEntry en = entry[s * rows + e];
    int64_t v_lo, v_hi;
    tile_bounds(tile, m.tile_vec, m.tile_rem, m.row_vec, v_lo, v_hi);
    const bool first = tile == 0 && threadIdx.x == 0;
    if (mover == 0 && threadIdx.x == 0) {
        uint32_t flags = 0;
        for (int q = 0; q < m.w; ++q) flags |= head[q].flags;
        m.state->last_n = head[m.w - 1].n;
        if (flags != 0) atomicOr(&m.state->flags, flags);
    }
    constexpr int WIDE = stored_wide(ST);       // vectors of a mini-batch / output row per vector of a stored row
    if (e < m.c) {
        if (en.row < 0) return;                 // dropped within its step, or overwritten again later in the window
        vec16* slot = m.buf_x + en.row * m.row_vec;
        // representatives that need the slot's old content get it from here, before it is overwritten
        for (int q = en.chain; q >= 0;) {
            const WinEntry rq = entry[q];
            const int qs = q / rows, qj = q % rows - m.c;
            if (first) { m.out_y[qs][qj] = rq.label; count_moved(m.state); }
            Tile<U, NT, TPB, WIN_PACE, stored_cv(ST, CV_WIDEN)> old;
            old.load(slot, v_lo, v_hi);
            old.store(m.out_x[qs] + (int64_t)qj * m.row_vec * WIDE, v_lo, v_hi);
            q = rq.chain;
        }
        // Lanes past the end of a tile move its last vector again, so a vector may be read by one
        // wavefront and overwritten by another: everybody has read before anybody overwrites.
        if (en.chain >= 0) __syncthreads();
        if (first) { m.buf_y[en.row] = en.label; count_moved(m.state); }
        Tile<U, NT, TPB, WIN_PACE, stored_cv(ST, CV_NARROW)> t;
        t.load(m.batch_x[s] + (int64_t)en.src * m.row_vec * WIDE, v_lo, v_hi);
        t.store(slot, v_lo, v_hi);
        return;
    }
    if (en.handled) return;
    const int j = e - m.c;
    if (first) m.out_y[s][j] = en.label;        // -1 when fewer samples are stored than asked for
    if (en.label < 0) return;
    if (first) count_moved(m.state);
    vec16* dst = m.out_x[s] + (int64_t)j * m.row_vec * WIDE;
    if (ST != RB_STORE_SAME && en.src >= 0) {
        // taken from a mini-batch row of this launch: what the slot will hold is that row in its stored form
        Tile<U, NT, TPB, WIN_PACE, stored_cv(ST, CV_BOTH)> t;
        t.load(m.batch_x[en.src >> 16] + (int64_t)(en.src & 0xFFFF) * m.row_vec * WIDE, v_lo, v_hi);
        t.store(dst, v_lo, v_hi);
    } else {
        const vec16* src = en.src >= 0 ? m.batch_x[en.src >> 16] + (int64_t)(en.src & 0xFFFF) * m.row_vec
                                       : m.buf_x + en.row * m.row_vec;
        Tile<U, NT, TPB, WIN_PACE, stored_cv(ST, CV_WIDEN)> t;
        t.load(src, v_lo, v_hi);
        t.store(dst, v_lo, v_hi);
    }
}

}  // namespace
