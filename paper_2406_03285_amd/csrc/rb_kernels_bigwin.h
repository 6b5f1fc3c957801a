// Several steps per launch for large counts, and for short rows (rb_update_sample_many with up to 1024 candidates and
// representatives, up to 10240 classes; exact selection, or the Bernoulli selection for mini-batches of at most 1024
// samples; any replacement strategy, any storage form).
// As in rb_kernels_window.h a launch moves the rows of all steps of a window by a table that extra
// workgroups of the launch before made; as in rb_kernels_big.h those workgroups have 1024 threads, one per
// candidate or representative, and there are two per step (update, sampling).  The 2 w planners of a window of
// w steps run side by side and tell each other, through the workspace, the little that one step needs of
// the others:
//   A  every update planner selects its step's candidates and publishes their classes.  The fill counts at
//      the start of step s are the counts before the window plus the candidates that the steps before s bring
//      (cut off at the capacity: min(min(f + a, S) + b, S) = min(f + a + b, S)), and the per-class state of the
//      FIFO / reservoir strategies follows from the same sums in closed form; so a planner waits for the
//      classes of the steps before its own and needs nothing else of them to plan its step as
//      rb_kernels_big.h does;
//   B  every planner writes its step's table entries; an update planner also publishes a hash table of the slot
//      rows its step writes;
//   C  what the order of separate launches would settle between steps (rb_kernels_window.h) every planner
//      settles for its OWN entries by looking rows up in the other steps' tables: of several writes to one slot
//      only the last is carried out; a representative whose slot an earlier step of the window (or its own)
//      writes is copied from the mini-batch row stored there; and a representative that needs what a slot held
//      before the window while a later step overwrites it is left to the workgroups that carry out that write:
//      its planner puts it on a list that hangs off the writing candidate (an exchange on the list's head), and
//      those workgroups copy the old content out to the list's members before they overwrite it.
// What planners read of each other (classes, row tables, list heads, flags) is written with stores that go
// through to memory and read with loads that do not stop at a cache of their own die (agent-scope atomics: the
// dies of the chip do not see each other's caches), and a flag is set only when the stores before it have been
// acknowledged; the table entries and list links have one writer each and are only read by the next launch.  No
// cache is written back or invalidated as a whole: with the movers' traffic in them that took longer than the plan.
// The planners are the first workgroups of their launch, which starts when the launch before has ended: they
// are all resident from the start and never wait for a workgroup that has not been dispatched.  Every wait is
// bounded all the same (BW_TIMEOUT_TICKS): a planner that gives up marks the window's table as failed, the
// window's launch then moves nothing and raises RB_FLAG_PLAN_TIMEOUT.
// Included by rb.hip only, after rb_kernels_window.h (table entry format) and rb_kernels_big.h (selection, hash tables).
#pragma once

#include <type_traits>

#include "rb_device.h"
#include "rb_kernels_window.h"
#include "rb_kernels_big.h"

namespace {

constexpr int BW_MAX = 16;                          // most steps one launch covers
constexpr int BW_HALF = 8;                          // steps whose tables one batch of lookups covers (registers)
static_assert(BW_MAX % BW_HALF == 0 && BW_MAX <= 16, "step masks are 16-bit");
constexpr uint64_t BW_TIMEOUT_TICKS = 200000000ull; // bound of every wait: 2 s of the 100 MHz wall clock

// The table of one window in the workspace (two of them, used in turn).
struct BwFlags {
    uint32_t classes[BW_MAX];   // = the window's number once step s's candidate classes are published (A)
    uint32_t update[BW_MAX];    // ... once step s's update planner has published entries, write table and list heads (B)
    uint32_t failed;            // = the window's number if a planner gave up waiting
    uint32_t pad[7];
    uint32_t count[BW_MAX];     // candidate entries of step s (the Bernoulli selection yields any number of them)
};
constexpr size_t BW_OFF_HEAD = 0;                                                    // BW_MAX WinHeader
constexpr size_t BW_OFF_FLAGS = BW_OFF_HEAD + BW_MAX * sizeof(WinHeader);            // BwFlags
constexpr size_t BW_OFF_ENTRY = BW_OFF_FLAGS + sizeof(BwFlags);                      // entry index = step * (c + r) + (candidate i | c + representative j)
constexpr size_t BW_OFF_CLASS = BW_OFF_ENTRY + (size_t)BW_MAX * 2 * BIG_MAX * sizeof(WinEntry);   // [step][BIG_MAX] candidate classes
constexpr size_t BW_OFF_WROTE = BW_OFF_CLASS + (size_t)BW_MAX * BIG_MAX * 4;         // [step][BIG_HASH] 64-bit words: see BwTable
constexpr size_t BW_OFF_FIRST = BW_OFF_WROTE + (size_t)BW_MAX * 2 * BIG_HASH * 4;    // [step][BIG_MAX] list heads, by candidate entry
constexpr size_t BW_OFF_NEXT = BW_OFF_FIRST + (size_t)BW_MAX * BIG_MAX * 4;          // [step][BIG_MAX] list links, by representative
constexpr size_t BW_TABLE_BYTES = (BW_OFF_NEXT + (size_t)BW_MAX * BIG_MAX * 4 + 255) / 256 * 256;
constexpr uint32_t BW_NONE = 0xFFFFFFFFu;           // end of a list; otherwise step << 16 | representative
static_assert(sizeof(BwFlags) % 16 == 0 && BW_OFF_ENTRY % 16 == 0, "entries are 16-byte aligned");

struct BwPlanArgs {
    const int64_t* batch_y[BW_MAX];    // labels of the steps that are planned
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
    uint32_t number;                   // the window's number (never 0): what its flags are set to
    int32_t selection;                 // RB_SELECT_*
    int32_t ce;                        // candidate entries per step in the table: c, or b with the Bernoulli selection (one thread per position)
    const int32_t* aux_old;            // per class: FIFO: slot of the oldest sample; RESERVOIR: samples offered so far
    int32_t* aux_new;
};

struct BwMoveArgs {
    const vec16* batch_x[BW_MAX];
    vec16* out_x[BW_MAX];
    int64_t* out_y[BW_MAX];
    vec16* buf_x;
    int64_t* buf_y;
    const char* table;
    DevState* state;
    int32_t w, c, r;                   // c: candidate entries per step in the table (BwPlanArgs::ce)
    int32_t cgrid;                     // candidate rows per step that the grid covers (with the Bernoulli selection c and a margin; the groups go round)
    uint32_t number;                   // the number of the window this table was planned as
    int64_t S;
    int64_t row_vec;
    int32_t tpr, tile_vec, tile_rem;
};

// Pointer number i of one of the per-step pointer arrays of BwMoveArgs, for kernels whose FIRST argument that struct is
// (it then starts the kernel's argument segment, `args`).  One load at a computed offset in place of a choice among
// BW_MAX values; where i is the same in all lanes it is a scalar load.
// bw_kernel_args() has a meaning in the kernel function itself only (elsewhere the compiler yields a null pointer):
// functions that are called take `args` as a parameter.
typedef const char __attribute__((address_space(4))) * BwArgBytes;
__device__ __forceinline__ BwArgBytes bw_kernel_args()
{
    return (BwArgBytes)__builtin_amdgcn_kernarg_segment_ptr();
}
template <typename T>
__device__ __forceinline__ T* bw_step_pointer(BwArgBytes args, size_t array_offset, int i)
{
    typedef T* const __attribute__((address_space(4))) * ArgPointer;
    return *(ArgPointer)(args + array_offset + sizeof(void*) * (size_t)i);
}

__device__ __forceinline__ const int64_t* bw_labels(const BwPlanArgs& a, int s)
{
    const int64_t* p = a.batch_y[0];   // (fixed offsets into the kernel arguments, see win_labels)
#pragma unroll
    for (int i = 1; i < BW_MAX; ++i) p = s == i ? a.batch_y[i] : p;
    return p;
}

// Stores and loads of what planners tell each other within a launch.
__device__ __forceinline__ void bw_put(uint32_t* p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t bw_get(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// What this workgroup has told the others (bw_put) so far has arrived when they see `flag` = number.  All threads call it.
__device__ __forceinline__ void bw_publish(uint32_t* flag, uint32_t number)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) bw_put(flag, number);
}

// Wait until flags[lo .. hi) all show `number` (thread i watches flag lo + i; at most BW_MAX of them).
// All threads call it; false if a wait ran out.
__device__ __forceinline__ bool bw_await(const uint32_t* flags, int lo, int hi, uint32_t number, int* s_ok)
{
    const int i = (int)threadIdx.x;
    if (i == 0) *s_ok = 1;
    __syncthreads();
    if (i < hi - lo) {
        const uint64_t t0 = wall_clock64();
        while (bw_get(flags + lo + i) != number) {
            if (wall_clock64() - t0 > BW_TIMEOUT_TICKS) {
                *s_ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(4);
        }
    }
    __syncthreads();
    const bool ok = *s_ok != 0;
    __syncthreads();                                  // (everybody has read the verdict before the next wait resets it)
    return ok;
}

__device__ __forceinline__ void bw_put64(uint64_t* p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t bw_get64(const uint64_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A published table: BIG_HASH words of (value << 32 | row), open addressing as in the planners' LDS tables, free
// slots hold BIG_EMPTY as row.
// `row` looked up in the tables of all steps q with bit q of `steps` set, all at once: a round trip to memory per
// probe round, not per table (a dependent trip costs 1 to 2 us while the movers are running).  Returns the steps
// whose table holds the row, their values in val[q].
__device__ __forceinline__ uint32_t bw_lookup_half(const uint64_t* tabs, uint32_t row, uint32_t steps, uint32_t (&val)[BW_HALF])
{
    uint32_t h[BW_HALF];
#pragma unroll
    for (int q = 0; q < BW_HALF; ++q) h[q] = big_hash(row);
    uint32_t pending = steps, found = 0;
    // two consecutive slots per table and round: the tables are half full, so most walks end in the first round
    for (int probes = 0; pending != 0 && probes < BIG_HASH; probes += 2) {
        uint64_t at[BW_HALF], nx[BW_HALF];
#pragma unroll
        for (int q = 0; q < BW_HALF; ++q)
            if ((pending >> q) & 1u) {
                const uint64_t* tab = tabs + (size_t)q * BIG_HASH;
                const uint32_t h1 = (h[q] + 1) & (BIG_HASH - 1);
                at[q] = bw_get64(tab + h[q]);
                nx[q] = bw_get64(tab + h1);
            }
#pragma unroll
        for (int q = 0; q < BW_HALF; ++q) {
            if (!((pending >> q) & 1u)) continue;
            if ((uint32_t)at[q] == row || ((uint32_t)at[q] != BIG_EMPTY && (uint32_t)nx[q] == row)) {
                found |= 1u << q;
                val[q] = (uint32_t)(((uint32_t)at[q] == row ? at[q] : nx[q]) >> 32);
                pending &= ~(1u << q);
            } else if ((uint32_t)at[q] == BIG_EMPTY || (uint32_t)nx[q] == BIG_EMPTY) {
                pending &= ~(1u << q);
            } else {
                h[q] = (h[q] + 2) & (BIG_HASH - 1);
            }
        }
    }
    return found;
}
// (BW_HALF tables at a time: their words of one round are all in registers together)
__device__ __forceinline__ uint32_t bw_lookup_steps(const uint64_t* tabs, uint32_t row, uint32_t steps, uint32_t (&val)[BW_MAX])
{
    uint32_t found = 0;
#pragma unroll
    for (int p = 0; p < BW_MAX / BW_HALF; ++p) {
        const uint32_t part = (steps >> (p * BW_HALF)) & ((1u << BW_HALF) - 1u);
        if (part == 0) continue;
        uint32_t v[BW_HALF];
        const uint32_t f = bw_lookup_half(tabs + (size_t)p * BW_HALF * BIG_HASH, row, part, v);
#pragma unroll
        for (int q = 0; q < BW_HALF; ++q)
            if ((f >> q) & 1u) val[p * BW_HALF + q] = v[q];
        found |= f << (p * BW_HALF);
    }
    return found;
}

struct BwTable {
    WinHeader* head;
    BwFlags* flags;
    WinEntry* entry;
    int32_t* classes;
    uint64_t* wrote;      // [step][BIG_HASH]: rows the step writes -> mini-batch position << 16 | candidate entry
    uint32_t* first;      // [step][BIG_MAX]: by candidate entry: the first representative (step << 16 | number) that
                          // gets the slot's old content from the candidate's workgroups, BW_NONE: none
    uint32_t* next;       // [step][BIG_MAX]: by representative: the one after it on that list
};
__device__ __forceinline__ BwTable bw_table(char* table)
{
    BwTable t;
    t.head = reinterpret_cast<WinHeader*>(table + BW_OFF_HEAD);
    t.flags = reinterpret_cast<BwFlags*>(table + BW_OFF_FLAGS);
    t.entry = reinterpret_cast<WinEntry*>(table + BW_OFF_ENTRY);
    t.classes = reinterpret_cast<int32_t*>(table + BW_OFF_CLASS);
    t.wrote = reinterpret_cast<uint64_t*>(table + BW_OFF_WROTE);
    t.first = reinterpret_cast<uint32_t*>(table + BW_OFF_FIRST);
    t.next = reinterpret_cast<uint32_t*>(table + BW_OFF_NEXT);
    return t;
}

// The arguments of rb_kernels_big.h's selection for step s of the window.
__device__ __forceinline__ PlanArgs bw_step_args(const BwPlanArgs& a, int s)
{
    PlanArgs p;
    p.batch_y = bw_labels(a, s);
    p.fill_old = a.fill_old;
    p.fill_new = nullptr; p.chunk_new = nullptr; p.table = nullptr;
    p.sd.seed_lo = a.seed_lo; p.sd.seed_hi = a.seed_hi;
    p.sd.step_lo = (uint32_t)(a.first_step + s); p.sd.step_hi = (uint32_t)((a.first_step + s) >> 32);
    p.b = a.b; p.c = a.c; p.r = a.r;
    p.K = a.K; p.nchunks = a.nchunks;
    p.S = a.S;
    p.eviction = a.eviction;
    p.aux_old = a.aux_old; p.aux_new = nullptr;
    p.selection = a.selection;
    p.ce = a.ce;
    return p;
}

// ---------------------------------------------------------------------------
// Update planner of step s of the window (Alg. 1): thread i = candidate i of Floyd's emission order, or, with the
// Bernoulli selection (mini-batches of at most BIG_MAX), mini-batch position i, which is a candidate if its coin says so.
// LDS as in plan_big_update.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void bw_plan_update(const BwPlanArgs& a, int s, uint32_t* lds)
{
    int32_t* s_fill = reinterpret_cast<int32_t*>(lds);     // fill counts before the window, then at the start of step s (not cut off)
    uint32_t* s_u = lds + BIG_FILL;                        // first occurrences | class table
    uint32_t* s_v = s_u + 2 * BIG_HASH;                    // the mini-batch's labels | starts of the class lists | row table
    uint32_t* s_draw = s_v + 2 * BIG_HASH;                 // selection draws (bit 31: repeated), then the class lists
    __shared__ int s_wave[BIG_NWAVE];
    __shared__ int s_ok;

    const int tid = threadIdx.x;
    const int ce = a.ce, w = a.w, rows = a.ce + a.r;
    const int64_t S = a.S;
    const BwTable t = bw_table(a.table);
    const PlanArgs pa = bw_step_args(a, s);

    // ---- A: selection, classes ----
    const BigSelected sel = big_select(pa, s_fill, s_u, s_v, s_draw);
    const int x = sel.x;
    const int32_t k = sel.k;
    const bool valid = k >= 0;
    const bool strategy = a.eviction != RB_EVICT_UNIFORM;
    const int64_t before_window = valid ? s_fill[k] : 0;             // samples of the class stored before the window
    const int64_t aux_window = strategy && valid ? a.aux_old[k] : 0;  // the strategy's state before the window
    if (tid < ce) bw_put(reinterpret_cast<uint32_t*>(t.classes) + s * BIG_MAX + tid, (uint32_t)k);   // LAB_INVALID: label outside [0, K); LAB_UNSELECTED: tails
    // table entry of the thread's candidate: its number in Floyd's emission order, or its number among the selected positions
    int ent = tid, count = ce;
    if (a.selection == RB_SELECT_BERNOULLI) ent = big_scan_excl(k != LAB_UNSELECTED ? 1 : 0, count, s_wave);
    const bool has_entry = a.selection == RB_SELECT_BERNOULLI ? k != LAB_UNSELECTED : tid < ce;
    if (tid == 0) t.flags->count[s] = (uint32_t)count;
    bw_publish(&t.flags->classes[s], a.number);
    bool ok = bw_await(t.flags->classes, 0, s, a.number, &s_ok);
    // the candidates that the steps before this one bring
    if (ok && tid < ce) {
        int32_t kq[BW_MAX];                          // (all steps' loads first: one trip to memory, not one per step)
#pragma unroll
        for (int q = 0; q < BW_MAX; ++q) kq[q] = q < s ? (int32_t)bw_get(reinterpret_cast<const uint32_t*>(t.classes) + q * BIG_MAX + tid) : -1;
#pragma unroll
        for (int q = 0; q < BW_MAX; ++q)
            if (kq[q] >= 0) atomicAdd(&s_fill[kq[q]], 1);
    }

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
    // the class at the start of this step: what it would hold without a capacity, what it holds, the strategy's state
    const int64_t offered = valid ? s_fill[k] : 0;                   // before_window + candidates of the earlier steps
    const int64_t fill0 = offered < S ? offered : S;
    int64_t aux0 = 0;
    if (a.eviction == RB_EVICT_FIFO) aux0 = (aux_window + (offered > S ? offered - S : 0)) % S;   // the oldest sample moved on by the overwrites
    else if (a.eviction == RB_EVICT_RESERVOIR) aux0 = aux_window + (offered - before_window) < INT32_MAX ? aux_window + (offered - before_window) : INT32_MAX;
    int h = 0, arrival = 0;
    if (valid) {
        h = big_find_or_insert(ckey, (uint32_t)k);
        arrival = (int)atomicAdd(&ccnt[h], 1u);
    }
    __syncthreads();
    const int total = valid ? (int)ccnt[h] : 0;
    {
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

    // ---- insertion number and slot (as plan_big_update) ----
    int rank = 0;
    for (int i = 0; i < total; i += 4) {
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
            const int64_t offers = aux0 + rank < INT32_MAX ? aux0 + rank : INT32_MAX;
            const int64_t draw = (int64_t)below(pa.sd, PURPOSE_EVICT, (uint32_t)x, (uint64_t)offers + 1);
            slot = draw < S ? draw : -1;
        } else {
            slot = (int64_t)below(pa.sd, PURPOSE_EVICT, (uint32_t)x, (uint64_t)S);          // a uniformly drawn one
        }
    }
    const bool placed = valid && slot >= 0;          // (a reservoir may not keep a candidate)
    const int64_t row = placed ? (int64_t)k * S + slot : -1;
    uint32_t* rkey = s_v;                            // slot rows written in this step
    uint32_t* rval = s_v + BIG_HASH;                 // 1 + the largest mini-batch position that goes there, then position << 16 | candidate entry
    for (int i = tid; i < BIG_HASH; i += BIG_TPB) {
        rkey[i] = BIG_EMPTY;
        rval[i] = 0;
    }
    __syncthreads();
    int hr = 0;
    if (placed) {
        hr = big_find_or_insert(rkey, (uint32_t)row);
        atomicMax(&rval[hr], (uint32_t)x + 1u);
    }
    __syncthreads();
    // of the candidates of this step that go to one slot the last of the mini-batch is stored
    const bool stored = placed && rval[hr] == (uint32_t)x + 1u;
    __syncthreads();
    if (stored) rval[hr] = ((uint32_t)x << 16) | (uint32_t)ent;
    const int me = s * rows + ent;
    if (has_entry) {
        WinEntry e;
        e.src = x;
        e.label = valid ? k : -1;
        e.row = stored ? row : -1;
        e.chain = -1;
        e.handled = 0;
        e.pad[0] = 0; e.pad[1] = 0;
        t.entry[me] = e;
        bw_put(t.first + s * BIG_MAX + ent, BW_NONE);          // nobody waits for the slot's old content yet
    }
    __syncthreads();
    for (int i = tid; i < BIG_HASH; i += BIG_TPB) bw_put64(t.wrote + (size_t)s * BIG_HASH + i, (uint64_t)rval[i] << 32 | rkey[i]);
    bw_publish(&t.flags->update[s], a.number);

    // ---- C: this step's writes against the later steps of the window ----
    ok = bw_await(t.flags->update, s + 1, w, a.number, &s_ok) && ok;
    // Which later steps bring candidates of this step's classes (16 step bits per slot of the class table, in the
    // words that held the class lists): only their tables can hold this step's rows.
    uint32_t* cmask = s_draw;
    static_assert(BIG_HASH / 2 <= BIG_MAX + 4, "the step bits fit where the class lists were");
    for (int i = tid; i < BIG_HASH / 2; i += BIG_TPB) cmask[i] = 0;
    __syncthreads();
    if (ok && tid < ce) {
        int32_t kq[BW_MAX];
#pragma unroll
        for (int q = 0; q < BW_MAX; ++q) kq[q] = q < w && q > s ? (int32_t)bw_get(reinterpret_cast<const uint32_t*>(t.classes) + q * BIG_MAX + tid) : -1;
#pragma unroll
        for (int q = 0; q < BW_MAX; ++q) {
            if (kq[q] < 0) continue;
            const int hq = big_find(ckey, (uint32_t)kq[q]);
            if (hq >= 0) atomicOr(&cmask[hq >> 1], (1u << q) << (16 * (hq & 1)));
        }
    }
    __syncthreads();
    if (ok && stored) {
        const uint32_t later = (cmask[h >> 1] >> (16 * (h & 1))) & 0xFFFFu;
        uint32_t val[BW_MAX];
        // a later step writes the same slot: this write is not carried out
        if (later != 0 && bw_lookup_steps(t.wrote, (uint32_t)row, later, val) != 0) t.entry[me].row = -1;
    }
    if (!ok && tid == 0) bw_put(&t.flags->failed, a.number);
}

// ---------------------------------------------------------------------------
// Sampling planner of step s of the window (Sec. IV-C): thread j = representative j.
// LDS as in plan_big_sample.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void bw_plan_sample(const BwPlanArgs& a, int s, uint32_t* lds)
{
    int32_t* s_fill = reinterpret_cast<int32_t*>(lds);     // fill counts before the window, after step s, then their prefix sums
    uint32_t* s_u = lds + BIG_FILL;                        // draw table
    uint32_t* s_hit = s_u + 2 * BIG_HASH;                  // one byte per class: bit i: a step q of the window with q mod 8 = i brings it candidates
    uint32_t* s_draw = s_u + 4 * BIG_HASH;                 // sampling draws (bit 31: repeated)
    static_assert(BIG_CLASSES / 4 <= 2 * BIG_HASH, "a byte per class in the second table region");
    __shared__ int s_wave[BIG_NWAVE];
    __shared__ int s_ok;
    __shared__ uint32_t s_flags;

    const int tid = threadIdx.x;
    const int ce = a.ce, r = a.r, K = a.K, w = a.w, rows = a.ce + a.r;
    const int64_t S = a.S;
    const bool last = s == w - 1;
    const BwTable t = bw_table(a.table);
    Seed sd;
    sd.seed_lo = a.seed_lo; sd.seed_hi = a.seed_hi;
    sd.step_lo = (uint32_t)(a.first_step + s); sd.step_hi = (uint32_t)((a.first_step + s) >> 32);

    int32_t fo[BIG_PER];
#pragma unroll
    for (int u = 0; u < BIG_PER; ++u) {
        const int q = tid + u * BIG_TPB;
        fo[u] = q < K ? a.fill_old[q] : 0;
    }
    if (tid == 0) s_flags = 0;
    for (int i = tid; i < BIG_CLASSES / 4; i += BIG_TPB) s_hit[i] = 0;
    const uint64_t bits = tid < r ? draw64(sd, PURPOSE_SAMPLE, (uint32_t)tid) : 0;
    uint32_t* dkey = s_u;                            // values of the sampling draws
    uint32_t* dfirst = s_u + BIG_HASH;               // first draw with that value
    for (int i = tid; i < BIG_HASH; i += BIG_TPB) {
        dkey[i] = BIG_EMPTY;
        dfirst[i] = 0xFFFFFFFFu;
    }
#pragma unroll
    for (int u = 0; u < BIG_PER; ++u) s_fill[tid + u * BIG_TPB] = fo[u];
    for (int i = BIG_CLASSES + tid; i < BIG_FILL; i += BIG_TPB) s_fill[i] = 0;

    // ---- the candidates of this step and of the steps before it: how many every class gets; which classes the later steps touch ----
    bool ok = bw_await(t.flags->classes, 0, w, a.number, &s_ok);
    if (ok && tid < ce) {
        int32_t kq[BW_MAX];                          // (all steps' loads first: one trip to memory, not one per step)
#pragma unroll
        for (int q = 0; q < BW_MAX; ++q) kq[q] = q < w ? (int32_t)bw_get(reinterpret_cast<const uint32_t*>(t.classes) + q * BIG_MAX + tid) : -1;
#pragma unroll
        for (int q = 0; q < BW_MAX; ++q) {
            if (kq[q] >= 0) {
                if (q <= s) atomicAdd(&s_fill[kq[q]], 1);        // may pass the capacity: cut back below
                atomicOr(&s_hit[kq[q] >> 2], (1u << (q & 7)) << (8 * (kq[q] & 3)));
            } else if (q == s && kq[q] == LAB_INVALID) {
                atomicOr(&s_flags, (uint32_t)RB_FLAG_BAD_LABEL);
            }
        }
    }
    __syncthreads();

    // ---- fill counts after the step; after the last step of the window they go out to memory, with the strategies' state ----
    const int32_t cap = (int32_t)(S < INT32_MAX ? S : INT32_MAX);
    if (last) {
#pragma unroll
        for (int u = 0; u < BIG_PER; ++u) {
            const int q = tid + u * BIG_TPB;
            if (q >= K) continue;
            const int32_t f = s_fill[q];
            a.fill_new[q] = f < cap ? f : cap;
            if (a.eviction == RB_EVICT_FIFO) {
                a.aux_new[q] = (int32_t)(((int64_t)a.aux_old[q] + (f > cap ? f - cap : 0)) % S);
            } else if (a.eviction == RB_EVICT_RESERVOIR) {
                const int64_t seen = (int64_t)a.aux_old[q] + (f - fo[u]);
                a.aux_new[q] = (int32_t)(seen < INT32_MAX ? seen : INT32_MAX);
            }
        }
    }
    int nf[BIG_PER], local = 0;
#pragma unroll
    for (int u = 0; u < BIG_PER; ++u) {
        const int32_t f = s_fill[BIG_PER * tid + u];
        nf[u] = f < cap ? f : cap;
        local += nf[u];
    }
    const int lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int inc = wave_scan_incl(local);
    if (lane == WAVE - 1) s_wave[wave] = inc;
    __syncthreads();                                 // also ends the reads of s_fill above
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
    __syncthreads();
    if (last && tid < a.nchunks) {
        const int lo = tid * CH, hi = lo + CH;
        a.chunk_new[tid] = s_fill[hi] - s_fill[lo];
    }

    // ---- thread j = draw j of Floyd's n-subset of the F stored samples (as plan_big_sample) ----
    const int n = r < F ? r : F;
    const int64_t base = (int64_t)F - n;
    const bool drawing = tid < n;
    const uint32_t g0 = drawing ? (uint32_t)__umul64hi(bits, (uint64_t)base + (uint64_t)tid + 1u) : 0u;   // < 2^31
    int hd = 0;
    if (drawing) {
        hd = big_find_or_insert(dkey, g0);
        atomicMin(&dfirst[hd], (uint32_t)tid);
    }
    __syncthreads();
    if (drawing) s_draw[tid] = g0 | ((dfirst[hd] != (uint32_t)tid) ? 0x80000000u : 0u);
    __syncthreads();
    int32_t pk = -1;
    int64_t prow = -1;
    uint32_t touched = 0;                            // steps of the window that may bring candidates to the sample's class
    if (drawing) {
        const int64_t g = big_replaced(s_draw, tid, base) ? base + tid : (int64_t)g0;     // class-major index of the sample
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
        const uint32_t hit = (s_hit[pk >> 2] >> (8 * (pk & 3))) & 0xFFu;
        touched = (hit | hit << 8) & ((1u << w) - 1u);
        static_assert(BW_MAX <= 16, "two steps per bit at most");
    }
    const int me = s * rows + ce + tid;
    if (tid < r) {
        WinEntry e;
        e.src = -1;
        e.label = pk;                           // -1 when fewer samples are stored than asked for
        e.row = prow;
        e.chain = -1;
        e.handled = 0;
        e.pad[0] = 0; e.pad[1] = 0;
        t.entry[me] = e;
    }
    if (tid == 0) {
        WinHeader hh;
        hh.n = n;
        hh.flags = s_flags;
        hh.pad[0] = 0; hh.pad[1] = 0;
        t.head[s] = hh;
    }

    // ---- C: a slot that this step or an earlier one of the window writes is read from the mini-batch row stored there;
    //         what a later step overwrites is handed out by the workgroups that overwrite it ----
    ok = bw_await(t.flags->update, 0, w, a.number, &s_ok) && ok;
    if (ok && touched != 0) {
        uint32_t val[BW_MAX];
        const uint32_t writers = bw_lookup_steps(t.wrote, (uint32_t)prow, touched, val);
        const uint32_t upto = writers & ((2u << s) - 1u);
        const int q = 31 - __builtin_clz(upto != 0 ? upto : (writers | 1u));   // the latest write up to this step, else the last one of the window
        uint32_t v = 0;
#pragma unroll
        for (int i = 0; i < BW_MAX; ++i) v = i == q ? val[i] : v;
        if (upto != 0) {
            t.entry[me].src = (q << 16) | (int)(v >> 16);
        } else if (writers != 0) {
            // Overwritten later in the window; of those writes the last is the one carried out.  This representative joins
            // the list of that candidate, whose workgroups hand the slot's old content out to the list's members.
            t.entry[me].handled = 1;
            const uint32_t before = __hip_atomic_exchange(t.first + q * BIG_MAX + (int)(v & 0xFFFFu), ((uint32_t)s << 16) | (uint32_t)tid,
                                                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            t.next[s * BIG_MAX + tid] = before;
        }
    }
    if (!ok && tid == 0) bw_put(&t.flags->failed, a.number);
}

// The plan of the first window of a call, on its own: 2 w workgroups.
__global__ void __launch_bounds__(BIG_TPB) rb_bigwin_plan_kernel(const BwPlanArgs a)
{
    extern __shared__ uint32_t lds[];
    const int s = (int)blockIdx.x >> 1;
    if (blockIdx.x & 1) bw_plan_sample(a, s, lds);
    else bw_plan_update(a, s, lds);
}

// A candidate's row stored in a slot whose content from before the window representatives of earlier steps of the
// window still need: the members of the list that starts with `heir` (their sampling planners put them there).  Every
// lane copies its own vectors out to them and only then overwrites these same vectors, so no lane waits for another.
// args: the calling kernel's argument segment, which BwMoveArgs starts (bw_step_pointer).
template <int U, int W, int ST>
__device__ __forceinline__ void bw_hand_off(BwArgBytes args, const uint32_t* next, DevState* state, vec16* slot, const vec16* fresh,
                                            uint32_t heir, int32_t label, int w, int r, int64_t row_vec, int64_t v_lo, int64_t v_hi, bool first)
{
    constexpr int WIDE = stored_wide(ST);       // vectors of an output row per vector of a stored row
    constexpr int UB = U > 4 ? 4 : U;           // a lane's vectors go in batches of that many (registers)
    constexpr int PART = WIDE * U / UB;
    // what a lane holds of the stored row per vector of the sample: the vector itself, half of one (four bfloat16), a quarter (four bytes)
    typedef typename std::conditional<ST == RB_STORE_U8, uint32_t, typename std::conditional<ST == RB_STORE_BF16, vec8, vec16>::type>::type Stored;
    const int lane = threadIdx.x & (W - 1);
    Stored* stored = reinterpret_cast<Stored*>(slot);
    const int64_t lo = WIDE * v_lo, hi = WIDE * v_hi;       // in vectors of the output rows
#pragma unroll
    for (int g = 0; g < PART; ++g) {
        // (all of a lane's vectors are read before any is written: the reads are in flight together)
        Stored old[UB];
        vec16 in[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int64_t i = lo + lane + (int64_t)(g * UB + u) * W;
            const int64_t at = i < hi ? i : hi - 1;          // (beyond the tile: its last vector again, not used)
            old[u] = stored[at];
            in[u] = fresh[at];
        }
        // (a list has at most one member per earlier step of the window; the bounds keep a walk finite and inside the
        // outputs whatever the list's words hold)
        uint32_t member = heir;
        for (int walked = 0; member != BW_NONE && walked < BW_MAX; ++walked) {
            const int q = (int)(member >> 16), j = (int)(member & 0xFFFFu);
            if (q >= w || j >= r) break;
            const uint32_t after = next[q * BIG_MAX + j];
            vec16* out = bw_step_pointer<vec16>(args, offsetof(BwMoveArgs, out_x), q) + (int64_t)j * row_vec * WIDE;
            if (first && g == 0) {
                bw_step_pointer<int64_t>(args, offsetof(BwMoveArgs, out_y), q)[j] = label;
                count_moved(state);
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const int64_t i = lo + lane + (int64_t)(g * UB + u) * W;
                if (i >= hi) continue;
                if constexpr (ST == RB_STORE_U8) out[i] = unpack4_u8(old[u]);
                else if constexpr (ST == RB_STORE_BF16) out[i] = widen4(old[u]);
                else out[i] = old[u];
            }
            member = after;
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int64_t i = lo + lane + (int64_t)(g * UB + u) * W;
            if (i >= hi) continue;
            if constexpr (ST == RB_STORE_U8) stored[i] = pack4_u8(in[u]);
            else if constexpr (ST == RB_STORE_BF16) stored[i] = narrow4(in[u]);
            else stored[i] = in[u];
        }
    }
}

// ---------------------------------------------------------------------------
// All steps of one window by its table: every group of BIG_GROUP threads moves one tile of one row; the
// first 2 next.w workgroups plan the next window instead.
// ---------------------------------------------------------------------------
template <int U, int W, bool NT, int ST>      // W: threads that move one tile together (short rows: one wavefront, which then has the
                                              // most bytes in flight; a compute unit holds a fixed number of wavefronts, not of bytes);
                                              // ST: RB_STORE_*, the form binary32 samples are stored in (row_vec counts stored vectors)
__global__ void __launch_bounds__(BIG_TPB) rb_bigwin_kernel(const BwMoveArgs m, const BwPlanArgs next)
{
    extern __shared__ uint32_t lds[];
    const int planners = 2 * next.w;
    if ((int)blockIdx.x < planners) {          // dispatched first: they have the longest way to go
        __builtin_amdgcn_s_setprio(3);
        const int s = (int)blockIdx.x >> 1;
        if (blockIdx.x & 1) bw_plan_sample(next, s, lds);
        else bw_plan_update(next, s, lds);
        return;
    }
    // the per-step pointers of m, by step number
    const BwArgBytes args = bw_kernel_args();
    const auto batch_x_of = [args](int q) { return bw_step_pointer<const vec16>(args, offsetof(BwMoveArgs, batch_x), q); };
    const auto out_x_of = [args](int q) { return bw_step_pointer<vec16>(args, offsetof(BwMoveArgs, out_x), q); };
    const auto out_y_of = [args](int q) { return bw_step_pointer<int64_t>(args, offsetof(BwMoveArgs, out_y), q); };
    const int rows = m.c + m.r;                 // entries per step in the table
    const int64_t per_step = (int64_t)(m.cgrid + m.r) * m.tpr;
    static_assert(W % WAVE == 0, "a wavefront works on one tile: what follows from its number is the same in all lanes");
    const int64_t item = (int64_t)((int)blockIdx.x - planners) * (BIG_TPB / W) + __builtin_amdgcn_readfirstlane((int)threadIdx.x / W);
    if (item >= per_step * m.w) return;
    const int s = (int)(item / per_step);
    int e, tile;
    split_item(item - (int64_t)s * per_step, m.tpr, e, tile);
    const WinHeader* head = reinterpret_cast<const WinHeader*>(m.table + BW_OFF_HEAD);
    const BwFlags* flags = reinterpret_cast<const BwFlags*>(m.table + BW_OFF_FLAGS);
    const WinEntry* entry = reinterpret_cast<const WinEntry*>(m.table + BW_OFF_ENTRY);
    const int lane = threadIdx.x & (W - 1);
    const bool first = tile == 0 && lane == 0;
    if (flags->failed == m.number) {           // the planners of this window gave up on each other: nothing is moved
        if (item == 0 && first) atomicOr(&m.state->flags, (uint32_t)RB_FLAG_PLAN_TIMEOUT);
        return;
    }
    int64_t v_lo, v_hi;
    tile_bounds(tile, m.tile_vec, m.tile_rem, m.row_vec, v_lo, v_hi);
    if (item == 0 && first) {
        uint32_t raised = 0;
        for (int q = 0; q < m.w; ++q) raised |= head[q].flags;
        m.state->last_n = head[m.w - 1].n;
        if (raised != 0) atomicOr(&m.state->flags, raised);
    }
    constexpr int WIDE = stored_wide(ST);         // vectors of a mini-batch / output row per vector of a stored row
    if (e < m.cgrid) {
        const uint32_t* first_of = reinterpret_cast<const uint32_t*>(m.table + BW_OFF_FIRST) + s * BIG_MAX;
        const uint32_t* next = reinterpret_cast<const uint32_t*>(m.table + BW_OFF_NEXT);
        const auto store_candidate = [&](const WinEntry& en, uint32_t heir) {
            if (en.row < 0) return;             // dropped within its step, or overwritten again later in the window
            vec16* slot = m.buf_x + en.row * m.row_vec;
            const vec16* fresh = batch_x_of(s) + (int64_t)en.src * m.row_vec * WIDE;
            if (first) { m.buf_y[en.row] = en.label; count_moved(m.state); }
            if (__builtin_expect(heir == BW_NONE, 1)) {
                Tile<U, NT, W, WIN_PACE, stored_cv(ST, CV_NARROW)> t;
                t.load(fresh, v_lo, v_hi);
                t.store(slot, v_lo, v_hi);
                return;
            }
            bw_hand_off<U, W, ST>(args, next, m.state, slot, fresh, heir, en.label, m.w, m.r, m.row_vec, v_lo, v_hi, first);
        };
        // The grid covers cgrid candidate rows per step; when the plan has more (Bernoulli selection), a group goes on to
        // the entry cgrid further on.  (The first entry is asked for before the step's count is known: it is inside the
        // step's part of the table whatever the count.)
        int ee = e;
        WinEntry en = entry[s * rows + ee];
        uint32_t heir = first_of[ee];
        const int count = (int)flags->count[s];
        while (ee < count) {
            store_candidate(en, heir);
            ee += m.cgrid;
            if (ee < count) {
                en = entry[s * rows + ee];
                heir = first_of[ee];
            }
        }
        return;
    }
    const int j = e - m.cgrid;
    const WinEntry en = entry[s * rows + m.c + j];
    if (en.handled) return;
    if (first) out_y_of(s)[j] = en.label;        // -1 when fewer samples are stored than asked for
    if (en.label < 0) return;
    if (first) count_moved(m.state);
    vec16* dst = out_x_of(s) + (int64_t)j * m.row_vec * WIDE;
    if (ST != RB_STORE_SAME && en.src >= 0) {
        // taken from a mini-batch row of this launch: what the slot will hold is that row in its stored form
        Tile<U, NT, W, WIN_PACE, stored_cv(ST, CV_BOTH)> t;
        t.load(batch_x_of(en.src >> 16) + (int64_t)(en.src & 0xFFFF) * m.row_vec * WIDE, v_lo, v_hi);
        t.store(dst, v_lo, v_hi);
    } else {
        const vec16* src = en.src >= 0 ? batch_x_of(en.src >> 16) + (int64_t)(en.src & 0xFFFF) * m.row_vec
                                       : m.buf_x + en.row * m.row_vec;
        Tile<U, NT, W, WIN_PACE, stored_cv(ST, CV_WIDEN)> t;
        t.load(src, v_lo, v_hi);
        t.store(dst, v_lo, v_hi);
    }
}

}  // namespace
