// Plan-ahead kernels for the single-launch step with up to 1024 candidates and representatives and up
// to 10240 classes (any replacement strategy, any storage form; exact selection, or the Bernoulli
// selection for mini-batches of at most 1024 samples): as in rb_kernels_planned.h the plan of a step is worked out by
// extra workgroups of the previous step's launch and left in a table, and the step's own launch only
// moves rows by that table - but the planning workgroups (two: update, sampling) have 1024 threads
// (one per candidate, resp. representative) and find class-mates, shared slots and repeated draws
// through hash tables in LDS instead of loops over all candidates.
// Included by rb.hip only, after rb_kernels_planned.h (whose table format and argument structs it uses).
#pragma once

#include "rb_device.h"
#include "rb_kernels_planned.h"

namespace {

constexpr int BIG_TPB = 1024;                 // threads of a workgroup of these kernels
constexpr int BIG_NWAVE = BIG_TPB / WAVE;
constexpr int BIG_MAX = 1024;                 // most candidates / representatives: one thread each
constexpr int BIG_PER = 10;                   // classes per thread in the prefix sums
constexpr int BIG_CLASSES = BIG_TPB * BIG_PER;   // most classes
constexpr int BIG_FILL = BIG_CLASSES + WAVE;  // words of the prefix table: one more than classes, rounded up
constexpr int BIG_BATCH = 4096;               // largest mini-batch (words of the first-occurrence table)
constexpr int BIG_HASH = 2048;                // slots of each hash table (at most BIG_MAX keys)
constexpr uint32_t BIG_EMPTY = 0xFFFFFFFFu;   // free slot (no class, row or draw has this value)
constexpr int BIG_GROUP = TPB;                // threads that move one tile together
constexpr int BIG_GROUPS = BIG_TPB / BIG_GROUP;
// LDS words: fill counts | region U | region V | selection / sampling draws
constexpr size_t BIG_LDS_BYTES = (size_t)(BIG_FILL + 2 * BIG_HASH + 2 * BIG_HASH + BIG_MAX + 4) * 4;
constexpr size_t BIG_TABLE_BYTES = (sizeof(PlanHeader) + 2 * BIG_MAX * sizeof(PlanEntry) + 255) / 256 * 256;
// in memory: the table of the slot rows a step writes, and the number of candidate entries of its plan
constexpr size_t BIG_FWD_BYTES = (((size_t)2 * BIG_HASH + 1) * 4 + 255) / 256 * 256;

__device__ __forceinline__ uint32_t big_hash(uint32_t key)
{
    return (key * 2654435761u) >> 21;          // 11 bits: BIG_HASH slots
}

// Slot of `key`, inserting it if it is not there (open addressing; at most half of the slots are ever used).
__device__ __forceinline__ int big_find_or_insert(uint32_t* keys, uint32_t key)
{
    uint32_t h = big_hash(key);
    for (;;) {
        const uint32_t prev = atomicCAS(&keys[h], BIG_EMPTY, key);
        if (prev == BIG_EMPTY || prev == key) return (int)h;
        h = (h + 1) & (BIG_HASH - 1);
    }
}

// Slot of `key`, -1 if it is not in the table (nobody inserts meanwhile).
__device__ __forceinline__ int big_find(const uint32_t* keys, uint32_t key)
{
    uint32_t h = big_hash(key);
    for (;;) {
        const uint32_t at = keys[h];
        if (at == key) return (int)h;
        if (at == BIG_EMPTY) return -1;
        h = (h + 1) & (BIG_HASH - 1);
    }
}

// Floyd's subset, all draws at once (see wave_select): draw i is replaced by base + i iff an earlier
// draw has the same value (`dup`, bit 31 of s_draw[i]), or it equals base + q for an earlier q whose
// own draw was replaced.  s_draw holds every draw; returns whether draw `i` (value t) is replaced.
__device__ __forceinline__ bool big_replaced(const uint32_t* s_draw, int i, int64_t base)
{
    int cur = i;
    for (;;) {
        const uint32_t pc = s_draw[cur];
        if (pc >> 31) return true;
        const int64_t q = (int64_t)pc - base;
        if (q < 0 || q >= cur) return false;
        cur = (int)q;
    }
}

// Exclusive prefix sum of one int per thread over the BIG_TPB threads.  s_wave: BIG_NWAVE ints of LDS.
__device__ __forceinline__ int big_scan_excl(int v, int& total, int* s_wave)
{
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    const int inc = wave_scan_incl(v);
    if (lane == WAVE - 1) s_wave[w] = inc;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < BIG_NWAVE; ++i) {
        const int x = s_wave[i];
        all += x;
        if (i < w) before += x;
    }
    __syncthreads();
    total = all;
    return before + inc - v;
}

// ---------------------------------------------------------------------------
// The plan of one step by TWO workgroups of BIG_TPB threads that run side by side
// and do not talk to each other: one plans the update (Alg. 1), the other the
// sampling (Sec. IV-C).  Thread i = candidate i of Floyd's emission order, resp.
// representative i.  Same decisions as rb_update_kernel followed by
// rb_sample_kernel, candidate by candidate and representative by representative.
// Both start with the selection (first occurrence of every draw through a table
// over the b positions, then the chain walk) and the candidates' classes (all b
// labels parked in LDS at entry).  Then
//   update    the candidates of a class are collected in a list (hash table keyed
//             by class -> counter; list starts by a prefix sum over the table's
//             slots); a candidate's insertion number is the class's fill count
//             plus the list members earlier in the mini-batch; last writer wins
//             through a hash table keyed by slot row -> largest mini-batch position
//             among the candidates that go there.  That table also goes out to
//             memory: a representative whose slot is written in this very step is
//             copied from the mini-batch row stored there, and only this
//             workgroup knows which row that is (big_forwarded, called by the
//             workgroups that move the representative).
//   sampling  needs of the update only how many candidates every class gets: the
//             fill counts after the step (out to memory, this workgroup owns
//             them) and their prefix sums over the classes, in LDS; repeated draws
//             through a hash table keyed by the draw's value, chain walk, class of
//             the sample by binary search of the prefix sums.  A representative of
//             a class that gets candidates in this step is marked "look it up".
//
// LDS (dynamic, BIG_LDS_BYTES): s_fill[BIG_FILL], regions U and V of 2 * BIG_HASH
// words each, s_draw[BIG_MAX] (+4 words: the class lists, kept there, are read
// four members at a time).
// ---------------------------------------------------------------------------
struct BigSelected {
    int x;           // mini-batch position of the thread's candidate
    int32_t k;       // its class, LAB_INVALID, or LAB_UNSELECTED for threads without a candidate
};

// Selection and classes; by all threads of either workgroup.  Uses region U (first occurrences), region V (labels)
// and s_draw; ends with a barrier after which U and s_draw are free, V still holds the labels.  The fill counts
// before the step are requested behind the labels (which are needed first) and parked in s_fill on the way.
__device__ __forceinline__ BigSelected big_select(const PlanArgs& a, int32_t* s_fill, uint32_t* s_u, uint32_t* s_v, uint32_t* s_draw)
{
    const int tid = threadIdx.x;
    const int b = a.b, c = a.c, K = a.K;
    static_assert(BIG_BATCH == 4 * BIG_TPB && BIG_BATCH <= 2 * BIG_HASH, "four labels per thread, parked in region V");
    int64_t yv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int q = tid + u * BIG_TPB;
        yv[u] = q < b ? a.batch_y[q] : -1;
    }
    int32_t fo[BIG_PER];
#pragma unroll
    for (int u = 0; u < BIG_PER; ++u) {
        const int q = tid + u * BIG_TPB;
        fo[u] = q < K ? a.fill_old[q] : 0;
    }
    // Bernoulli selection (b <= BIG_MAX): thread i = mini-batch position i, selected by its own coin; the rounds
    // of Floyd's subset below then run empty
    const bool bernoulli = a.selection == RB_SELECT_BERNOULLI;
    const bool heads = bernoulli && tid < b && (int64_t)below(a.sd, PURPOSE_COIN, (uint32_t)tid, (uint64_t)b) < c;
    const bool active = !bernoulli && tid < c;
    const int sel_base = b - c;
    const uint32_t t = active ? (uint32_t)below(a.sd, PURPOSE_SELECT, (uint32_t)tid, (uint64_t)(sel_base + tid + 1)) : 0u;
    if (active) s_u[t] = 0xFFFFFFFFu;
    __syncthreads();
    if (active) atomicMin(&s_u[t], (uint32_t)tid);
    __syncthreads();
    if (active) s_draw[tid] = t | ((s_u[t] != (uint32_t)tid) ? 0x80000000u : 0u);     // t < 4096
    // the loads have had the two rounds above to arrive
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t y = yv[u];
        s_v[tid + u * BIG_TPB] = (uint32_t)((y >= 0 && y < K) ? (int32_t)y : LAB_INVALID);
    }
#pragma unroll
    for (int u = 0; u < BIG_PER; ++u) s_fill[tid + u * BIG_TPB] = fo[u];
    __syncthreads();
    BigSelected sel;
    sel.x = active ? (big_replaced(s_draw, tid, sel_base) ? sel_base + tid : (int)t) : (heads ? tid : 0);
    sel.k = active || heads ? (int32_t)s_v[sel.x] : LAB_UNSELECTED;
    __syncthreads();
    return sel;
}

// fwd: 2 * BIG_HASH words in memory: the slot rows written in the step, and 1 + the mini-batch position stored there.
__device__ __forceinline__ void plan_big_update(const PlanArgs& a, uint32_t* lds, uint32_t* fwd)
{
    int32_t* s_fill = reinterpret_cast<int32_t*>(lds);         // fill counts before the step
    uint32_t* s_u = lds + BIG_FILL;                        // first occurrences | class table
    uint32_t* s_v = s_u + 2 * BIG_HASH;                    // the mini-batch's labels | starts of the class lists | row table
    uint32_t* s_draw = s_v + 2 * BIG_HASH;                 // selection draws (bit 31: repeated), then the class lists
    __shared__ int s_wave[BIG_NWAVE];

    const int tid = threadIdx.x;
    const int64_t S = a.S;
    PlanEntry* entry = reinterpret_cast<PlanEntry*>(a.table + sizeof(PlanHeader));

    const BigSelected sel = big_select(a, s_fill, s_u, s_v, s_draw);
    const int x = sel.x;
    const int32_t k = sel.k;
    const bool valid = k >= 0;
    const int64_t fill0 = valid ? s_fill[k] : 0;
    // FIFO / reservoir replacement: the class's state before the step (slot of the oldest sample / samples offered so
    // far), on its way while the class table is built; this workgroup owns that state and writes its next copy
    const bool strategy = a.eviction != RB_EVICT_UNIFORM;
    const int64_t aux0 = strategy && valid ? a.aux_old[k] : 0;
    // table entry of the thread's candidate: its number in Floyd's emission order, or, with the Bernoulli
    // selection, its number among the selected positions
    int ent = tid, count = a.ce;
    if (a.selection == RB_SELECT_BERNOULLI) ent = big_scan_excl(k != LAB_UNSELECTED ? 1 : 0, count, s_wave);
    // class table: keys in U[0, BIG_HASH), members per class in U[BIG_HASH, 2 BIG_HASH)
    uint32_t* ckey = s_u;
    uint32_t* ccnt = s_u + BIG_HASH;
    uint32_t* list = s_draw;                    // [BIG_MAX]: position << 10 | candidate
    uint32_t* cstart = s_v + BIG_MAX;           // [BIG_HASH]: start of the class's list
    for (int i = tid; i < BIG_HASH; i += BIG_TPB) {
        ckey[i] = BIG_EMPTY;
        ccnt[i] = 0;
    }
    __syncthreads();
    int h = 0, arrival = 0;
    if (valid) {
        h = big_find_or_insert(ckey, (uint32_t)k);
        arrival = (int)atomicAdd(&ccnt[h], 1u);
    }
    __syncthreads();
    const int total = valid ? (int)ccnt[h] : 0;
    {
        // the lists of the classes follow each other in the order of the table's slots: two slots per thread
        static_assert(BIG_HASH == 2 * BIG_TPB, "two table slots per thread");
        const int c0 = (int)ccnt[2 * tid], c1 = (int)ccnt[2 * tid + 1];
        int all;
        const int lbefore = big_scan_excl(c0 + c1, all, s_wave);
        cstart[2 * tid] = (uint32_t)lbefore;
        cstart[2 * tid + 1] = (uint32_t)(lbefore + c0);
    }
    __syncthreads();
    const int start = valid ? (int)cstart[h] : 0;
    if (valid) list[start + arrival] = ((uint32_t)x << 10) | (uint32_t)tid;
    __syncthreads();

    // ---- insertion number and slot ----
    int rank = 0;
    for (int i = 0; i < total; i += 4) {             // four members per round; what is read past the class's list is not counted
        const uint32_t m0 = list[start + i], m1 = list[start + i + 1], m2 = list[start + i + 2], m3 = list[start + i + 3];
        rank += (int)((int)(m0 >> 10) < x) + (int)(i + 1 < total && (int)(m1 >> 10) < x) + (int)(i + 2 < total && (int)(m2 >> 10) < x) +
                (int)(i + 3 < total && (int)(m3 >> 10) < x);
    }
    const int64_t at = fill0 + rank;
    const bool over = valid && at >= S;              // beyond the capacity: overwrites a stored sample
    int64_t slot = at;
    if (over) {
        if (a.eviction == RB_EVICT_FIFO) {
            slot = (aux0 + at - S) % S;                                                      // the oldest one
        } else if (a.eviction == RB_EVICT_RESERVOIR) {
            // kept with probability S / (samples offered to the class so far + 1), then in a uniform slot
            const int64_t offers = aux0 + rank < INT32_MAX ? aux0 + rank : INT32_MAX;
            const int64_t draw = (int64_t)below(a.sd, PURPOSE_EVICT, (uint32_t)x, (uint64_t)offers + 1);
            slot = draw < S ? draw : -1;
        } else {
            slot = (int64_t)below(a.sd, PURPOSE_EVICT, (uint32_t)x, (uint64_t)S);           // a uniformly drawn one
        }
    }
    const bool placed = valid && slot >= 0;          // (a reservoir may not keep a candidate)
    const int64_t row = placed ? (int64_t)k * S + slot : -1;
    if (strategy) {
        // the strategy's state after the step: classes with candidates by their first arrival, the others copied
        if (valid && arrival == 0) {
            const int64_t f = fill0 + total;
            int64_t next;
            if (a.eviction == RB_EVICT_FIFO) next = (aux0 + (f > S ? f - S : 0)) % S;     // the oldest sample moves on by the overwrites
            else next = aux0 + total < INT32_MAX ? aux0 + total : INT32_MAX;
            a.aux_new[k] = (int32_t)next;
        }
        for (int q = tid; q < a.K; q += BIG_TPB)
            if (big_find(ckey, (uint32_t)q) < 0) a.aux_new[q] = a.aux_old[q];
    }
    uint32_t* rkey = s_v;                            // slot rows written in this step (the list starts in region V have been read)
    uint32_t* rmax = s_v + BIG_HASH;                 // 1 + the largest mini-batch position that goes there
    for (int i = tid; i < BIG_HASH; i += BIG_TPB) {
        rkey[i] = BIG_EMPTY;
        rmax[i] = 0;
    }
    __syncthreads();
    int hr = 0;
    if (placed) {
        hr = big_find_or_insert(rkey, (uint32_t)row);
        atomicMax(&rmax[hr], (uint32_t)x + 1u);
    }
    __syncthreads();
    // of the candidates that go to one slot the last of the mini-batch is stored
    const bool stored = placed && rmax[hr] == (uint32_t)x + 1u;
    if (a.selection == RB_SELECT_BERNOULLI ? k != LAB_UNSELECTED : tid < a.ce) {
        PlanEntry e;
        e.pos = x;
        e.label = valid ? k : -1;
        e.row = stored ? row : -1;
        entry[ent] = e;
    }
    for (int i = tid; i < 2 * BIG_HASH; i += BIG_TPB) fwd[i] = s_v[i];
    if (tid == 0) fwd[2 * BIG_HASH] = (uint32_t)count;
}

// Mini-batch position of the candidate that the step stores in slot row `row`, -1 if the step does not write it.
__device__ __forceinline__ int big_forwarded(const uint32_t* __restrict__ fwd, uint32_t row)
{
    uint32_t h = big_hash(row);
    for (;;) {
        const uint32_t at = fwd[h];
        if (at == row) return (int)fwd[BIG_HASH + h] - 1;
        if (at == BIG_EMPTY) return -1;
        h = (h + 1) & (BIG_HASH - 1);
    }
}

constexpr int32_t BIG_LOOK_UP = -2;      // PlanEntry::pos of a representative: its class gets candidates in this step

__device__ __forceinline__ void plan_big_sample(const PlanArgs& a, uint32_t* lds)
{
    int32_t* s_fill = reinterpret_cast<int32_t*>(lds);     // fill counts before the step, then after it, then their prefix sums
    uint32_t* s_u = lds + BIG_FILL;                        // first occurrences | draw table
    uint32_t* s_v = s_u + 2 * BIG_HASH;                    // the mini-batch's labels
    uint32_t* s_draw = s_v + 2 * BIG_HASH;                 // selection draws, then sampling draws (bit 31: repeated)
    __shared__ int s_wave[BIG_NWAVE];
    __shared__ uint32_t s_flags;
    __shared__ uint32_t s_hit[BIG_CLASSES / 32];           // one bit per class: it gets candidates in this step

    const int tid = threadIdx.x;
    const int r = a.r, K = a.K;
    const int64_t S = a.S;
    PlanHeader* head = reinterpret_cast<PlanHeader*>(a.table);
    PlanEntry* entry = reinterpret_cast<PlanEntry*>(a.table + sizeof(PlanHeader));

    if (tid == 0) s_flags = 0;
    if (tid < BIG_CLASSES / 32) s_hit[tid] = 0;
    const BigSelected sel = big_select(a, s_fill, s_u, s_v, s_draw);      // (its barriers also cover the stores above)
    const int32_t k = sel.k;

    // ---- how many candidates every class gets; the sampling bits; empty draw table ----
    if (k >= 0) {
        atomicAdd(&s_fill[k], 1);                           // may pass the capacity: cut back below
        atomicOr(&s_hit[k >> 5], 1u << (k & 31));
    }
    if (k == LAB_INVALID) atomicOr(&s_flags, (uint32_t)RB_FLAG_BAD_LABEL);
    const uint64_t bits = tid < r ? draw64(a.sd, PURPOSE_SAMPLE, (uint32_t)tid) : 0;
    uint32_t* dkey = s_u;                            // values of the sampling draws
    uint32_t* dfirst = s_u + BIG_HASH;               // first draw with that value
    for (int i = tid; i < BIG_HASH; i += BIG_TPB) {
        dkey[i] = BIG_EMPTY;
        dfirst[i] = 0xFFFFFFFFu;
    }
    __syncthreads();

    // ---- fill counts after the step: out to memory; sums of ten classes per thread ----
    const int32_t cap = (int32_t)(S < INT32_MAX ? S : INT32_MAX);
#pragma unroll
    for (int u = 0; u < BIG_PER; ++u) {
        const int q = tid + u * BIG_TPB;
        const int32_t f = s_fill[q];
        if (q < K) a.fill_new[q] = f < cap ? f : cap;
    }
    int nf[BIG_PER], local = 0;
#pragma unroll
    for (int u = 0; u < BIG_PER; ++u) {
        const int32_t f = s_fill[BIG_PER * tid + u];
        nf[u] = f < cap ? f : cap;
        local += nf[u];
    }
    // prefix sums over the threads, and (in registers) over the wavefronts: stretches of WAVE * BIG_PER classes
    const int lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int inc = wave_scan_incl(local);
    if (lane == WAVE - 1) s_wave[wave] = inc;
    lds_barrier();                                   // also ends the reads of s_fill above; the fill counts stay on their way out
    int wpre[BIG_NWAVE];                             // stored samples before the classes of wavefront i
    int F = 0;
#pragma unroll
    for (int i = 0; i < BIG_NWAVE; ++i) {
        wpre[i] = F;
        F += s_wave[i];
    }
    int before = inc - local;
#pragma unroll
    for (int i = 0; i < BIG_NWAVE; ++i) before += i == wave ? wpre[i] : 0;
#pragma unroll
    for (int u = 0; u < BIG_PER; ++u) {
        s_fill[BIG_PER * tid + u] = before;
        before += nf[u];
    }
    for (int i = BIG_CLASSES + tid; i < BIG_FILL; i += BIG_TPB) s_fill[i] = F;
    lds_barrier();
    if (tid < a.nchunks) {
        // stored samples per chunk of CH classes
        const int lo = tid * CH, hi = lo + CH;
        a.chunk_new[tid] = s_fill[hi] - s_fill[lo];
    }

    // ---- thread j = draw j of Floyd's n-subset of the F stored samples ----
    const int n = r < F ? r : F;
    const int64_t base = (int64_t)F - n;
    const bool drawing = tid < n;
    const uint32_t g0 = drawing ? (uint32_t)__umul64hi(bits, (uint64_t)base + (uint64_t)tid + 1u) : 0u;   // < 2^31
    int hd = 0;
    if (drawing) {
        hd = big_find_or_insert(dkey, g0);
        atomicMin(&dfirst[hd], (uint32_t)tid);
    }
    lds_barrier();
    if (drawing) s_draw[tid] = g0 | ((dfirst[hd] != (uint32_t)tid) ? 0x80000000u : 0u);
    lds_barrier();
    int32_t pk = -1;
    int64_t prow = -1;
    int32_t pos = -1;
    if (drawing) {
        const int64_t g = big_replaced(s_draw, tid, base) ? base + tid : (int64_t)g0;     // class-major index of the sample
        // its class: the last one whose prefix does not exceed g (empty classes share the prefix of the
        // next non-empty one, which is the one meant; classes past K hold F > g)
        // first which wavefront's stretch of classes (registers), then inside it (LDS)
        int seg = 0;
#pragma unroll
        for (int i = 1; i < BIG_NWAVE; ++i) seg += (int)(wpre[i] <= g);
        int lo = seg * WAVE * BIG_PER, hi = lo + WAVE * BIG_PER - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (s_fill[mid] <= g) lo = mid; else hi = mid - 1;
        }
        pk = lo;
        prow = (int64_t)pk * S + (g - s_fill[lo]);
        if ((s_hit[pk >> 5] >> (pk & 31)) & 1u) pos = BIG_LOOK_UP;      // its slot may be written in this very step
    }
    if (tid < r) {
        PlanEntry e;
        e.pos = pos;
        e.label = pk;                           // -1 when fewer samples are stored than asked for
        e.row = prow;
        entry[a.ce + tid] = e;
    }
    if (tid == 0) {
        PlanHeader hh;
        hh.n = n;
        hh.flags = s_flags;
        hh.c = a.ce;
        hh.r = r;
        *head = hh;
    }
}

// The plan of one step on its own (first step of a sequence): two workgroups.
__global__ void __launch_bounds__(BIG_TPB) rb_big_plan_kernel(const PlanArgs a, uint32_t* fwd)
{
    extern __shared__ uint32_t lds[];
    if (blockIdx.x == 0) plan_big_update(a, lds, fwd);
    else plan_big_sample(a, lds);
}

// ---------------------------------------------------------------------------
// One step by its table: every group of BIG_GROUP threads moves one tile of one
// row (candidates first, then representatives); with plan_next the first
// workgroup of the grid plans the next step instead.
// ---------------------------------------------------------------------------
template <int U, bool NT, int ST>           // ST: RB_STORE_*, the form binary32 samples are stored in (row_vec counts stored vectors)
__global__ void __launch_bounds__(BIG_TPB) rb_step_big_kernel(const MoveArgs m, const PlanArgs next, const uint32_t* fwd, uint32_t* fwd_next)
{
    extern __shared__ uint32_t lds[];
    const int planners = m.plan_next != 0 ? 2 : 0;
    if ((int)blockIdx.x < planners) {          // dispatched first: they have the longest way to go
        __builtin_amdgcn_s_setprio(3);
        if (blockIdx.x == 0) plan_big_update(next, lds, fwd_next);
        else plan_big_sample(next, lds);
        return;
    }
    const int64_t item = (int64_t)((int)blockIdx.x - planners) * BIG_GROUPS + threadIdx.x / BIG_GROUP;
    const int64_t items = (int64_t)(m.cgrid + m.r) * m.tpr;
    if (item >= items) return;
    int e, tile;
    split_item(item, m.tpr, e, tile);
    const PlanHeader* head = reinterpret_cast<const PlanHeader*>(m.table);
    const PlanEntry* entry = reinterpret_cast<const PlanEntry*>(m.table + sizeof(PlanHeader));
    int64_t v_lo, v_hi;
    tile_bounds(tile, m.tile_vec, m.tile_rem, m.row_vec, v_lo, v_hi);
    const bool first = tile == 0 && (threadIdx.x & (BIG_GROUP - 1)) == 0;
    if (item == 0 && first) {
        const PlanHeader hh = *head;
        m.state->last_n = hh.n;
        if (hh.flags != 0) atomicOr(&m.state->flags, hh.flags);
    }
    constexpr int WIDE = stored_wide(ST);         // vectors of a mini-batch / output row per vector of a stored row
    if (e < m.cgrid) {
        // the grid covers cgrid candidate rows; when the plan has more (Bernoulli selection: their number is random),
        // a group goes on to the entry cgrid further on
        const int count = (int)fwd[2 * BIG_HASH];
        for (int ee = e; ee < count; ee += m.cgrid) {
            const PlanEntry en = entry[ee];
            if (en.row < 0) continue;           // label outside [0, K), or a later class-mate takes the slot
            if (first) { m.buf_y[en.row] = en.label; count_moved(m.state); }
            Tile<U, NT, BIG_GROUP, true, stored_cv(ST, CV_NARROW)> t;
            t.load(m.batch_x + (int64_t)en.pos * m.row_vec * WIDE, v_lo, v_hi);
            t.store(m.buf_x + en.row * m.row_vec, v_lo, v_hi);
        }
        return;
    }
    const int j = e - m.cgrid;
    const PlanEntry en = entry[m.c + j];
    if (first) m.out_y[j] = en.label;           // -1 when fewer samples are stored than asked for
    if (en.label < 0) return;
    if (first) count_moved(m.state);
    // written in this very step?  Then the stored candidate's mini-batch row is what the slot will hold.
    const int pos = en.pos == BIG_LOOK_UP ? big_forwarded(fwd, (uint32_t)en.row) : -1;
    vec16* dst = m.out_x + (int64_t)j * m.row_vec * WIDE;
    if (ST != RB_STORE_SAME && pos >= 0) {
        // forwarded from the mini-batch: what the slot will hold is the row in its stored form
        Tile<U, NT, BIG_GROUP, true, stored_cv(ST, CV_BOTH)> t;
        t.load(m.batch_x + (int64_t)pos * m.row_vec * WIDE, v_lo, v_hi);
        t.store(dst, v_lo, v_hi);
    } else {
        const vec16* src = pos >= 0 ? m.batch_x + (int64_t)pos * m.row_vec : m.buf_x + en.row * m.row_vec;
        Tile<U, NT, BIG_GROUP, true, stored_cv(ST, CV_WIDEN)> t;
        t.load(src, v_lo, v_hi);
        t.store(dst, v_lo, v_hi);
    }
}

}  // namespace
