// Rehearsal-buffer hot path for gfx950 (MI355X): the C ABI of include/rb.h (host side); the
// kernels are in rb_kernels_small.h (at most 64 candidates / representatives, and the
// single-launch step), rb_kernels_planned.h (the same step with its plan made during the previous
// launch), rb_kernels_general.h (any counts, policy variants, reduced-precision storage) and
// rb_kernels_aux.h, their common device code in rb_device.h.
//
// One kernel launch per hot call.  Every workgroup first re-derives, in LDS,
// the few integers of the step's plan it needs (which mini-batch positions are
// candidates, which slot a candidate goes to, which stored sample a
// representative is) and then moves its share of one sample row with 16-byte
// vector loads and stores.  The plan is O(b + K) integers while a row is
// hundreds of kilobytes, so recomputing it per workgroup is cheaper than a
// second, dependent launch.  Nothing is staged through LDS: a row is read once
// and written once, so the data path is global -> registers -> global.
// When the labels of the next mini-batch are known in advance (rb_announce_next)
// the plan is not recomputed per workgroup at all: one workgroup of the previous
// launch leaves it as a table in the workspace and the step's launch only moves rows.
//
// Per-class fill counts are kept twice (ping-pong): an update reads the "old"
// copy everywhere and a few bookkeeping workgroups write the "new" one, so no
// workgroup can observe a count another workgroup of the same launch changed.
// The same two copies let a plan made ahead be dropped: the host just points
// back at the copy the planner read.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <new>

#include "rb.h"
#include "rb_device.h"
#include "rb_kernels_general.h"
#include "rb_kernels_small.h"
#include "rb_kernels_planned.h"
#include "rb_kernels_window.h"
#include "rb_kernels_big.h"
#include "rb_kernels_bigwin.h"
#include "rb_kernels_aux.h"

// ===========================================================================
// Host side: the C ABI
// ===========================================================================
struct rb_buffer {
    int64_t K, S;
    int64_t row_bytes;       // bytes of one stored row
    int64_t row_vec;         // 16-byte vectors of one stored row
    int64_t sample_bytes;    // bytes of one sample as the caller hands it in and gets it back
    int32_t dtype;
    int32_t storage;         // RB_STORE_*
    int32_t nchunks;
    // device storage (borrowed)
    void* buf_x;
    int64_t* buf_y;
    char* ws;
    hipStream_t stream;
    bool bound;
    int cur;                 // which of the two fill-count copies is current
    // workspace layout (byte offsets)
    size_t off_fill[2], off_chunk[2], ws_bytes;
    // launch-shape knobs
    int opt_unroll, opt_nt, opt_rpb, opt_fuse, opt_window, opt_planners;
    // policy variant and its per-class state (two copies, like the fill counts)
    int selection, eviction;
    size_t off_aux[2];
    int64_t updates;         // rb_update calls since the last rb_bind
    // plan-ahead form of the single-launch step
    size_t off_tbl[2];       // the two plan tables
    size_t off_wtbl[2];      // the two plan tables of the several-steps-per-launch form (and of the large-count form)
    size_t off_bfwd[2];      // large-count form: the two tables of the slot rows a step writes
    size_t off_bwtbl[2];     // the two plan tables of the several-steps-per-launch form for large counts
    uint32_t bw_number;      // number of the last window planned in that form (its planners' flags are set to it)
    uint32_t bw_table_number[2];   // ... and which window each of the two tables holds
    int tbl_next;            // table the next plan is written to
    int tbl_planned;         // table that holds the pending plan
    bool plan_valid;         // a step has been planned (and the fill counts advanced) but not yet executed
    const int64_t* plan_y;   // ... for these arguments
    int64_t plan_b, plan_c, plan_r;
    uint64_t plan_seed, plan_step;
    const int64_t* next_y;   // announced labels of the next mini-batch, consumed by the next rb_update_sample
    // several steps per launch: labels announced for the call after the next rb_update_sample_many, and the
    // window that the last launch of a call planned for them
    const int64_t* ann_y[WIN_MAX];
    int64_t ann_n;
    bool wplan_valid;        // a window has been planned (and the fill counts advanced) but not yet executed
    const int64_t* wplan_y[WIN_MAX];
    int wplan_form;          // MANY_SMALL or MANY_LARGE: whose table it is in
    int64_t wplan_w, wplan_b, wplan_c, wplan_r;
    uint64_t wplan_seed, wplan_first;
    int wplan_tbl;           // table that holds it
    int64_t wplan_nat;       // size the windows have grown to (the planned one may be shorter: what was left, what was announced)
    int static_dev;          // device whose static scratch array is this handle's workspace, -1: the caller's workspace
};

// Workspace of rb_bind_static: callers that cannot allocate get their workspace from here.  One copy per GPU
// that loads this library, at an address of its own on each; in host code the array's name only stands for the
// symbol (it is no device address), so the address is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[RB_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
void* scratch_ptr[MAX_DEVICES] = {};          // device address of `scratch` on each device, once known
rb_buffer* scratch_holder[MAX_DEVICES] = {};  // the handle that is bound to it

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// How rb_update_sample_many carries out a call: step by step, or several steps per launch planned by one workgroup per
// launch (rb_kernels_window.h) or by two per step (rb_kernels_bigwin.h).
enum { MANY_SINGLE = 0, MANY_SMALL = 1, MANY_LARGE = 2 };

struct Shape {
    int unroll, tpr, tile_vec, tile_rem, rpb;
    int64_t groups;
};

// Split `rows` rows of `row_vec` vectors into tiles of at most width * unroll vectors, where `width`
// is the number of threads that share a tile: TPB in the small-count kernels (a workgroup per tile),
// WAVE in the general ones (a wavefront per tile).
// most: the most vectors per thread the caller's kernel can hold (the converting movers hold several accesses per
// vector); preferred: what the caller's kernel does best with, taken when the option leaves the choice open.
Shape plan_shape(const rb_buffer* rb, int64_t rows, int width, int most = 8, int preferred = 0)
{
    Shape s;
    const int64_t row_vec = rb->row_vec;
    int u = rb->opt_unroll != 0 ? rb->opt_unroll : preferred;
    if (u == 0) {
        // Largest unroll that still leaves at least 1024 tiles (four workgroups per compute unit in
        // the small-count kernels, four wavefronts in the general ones); never below two vectors in
        // flight per thread (one was slower at every size measured) unless the row is shorter.
        u = 8;
        while (u > 2 && rows * ((row_vec + (int64_t)width * u - 1) / ((int64_t)width * u)) < 1024) u >>= 1;
        while (u > 1 && (int64_t)width * (u / 2) >= row_vec) u >>= 1;
    }
    if (u > most) u = most;
    s.unroll = u;
    const int64_t cap = (int64_t)width * u;
    s.tpr = (int)((row_vec + cap - 1) / cap);
    // even split in units of TILE_UNIT vectors: every tile holds nunits / tpr units, the first nunits % tpr one more
    const int64_t nunits = (row_vec + TILE_UNIT - 1) / TILE_UNIT;
    s.tile_vec = (int)(nunits / s.tpr);
    s.tile_rem = (int)(nunits % s.tpr);
    s.rpb = 1;
    if (width == TPB && s.tpr == 1) {
        int r = rb->opt_rpb;
        if (r == 0) {
            r = 1;
            while (r < 16 && (rows + r - 1) / r > 1024) r <<= 1;
        }
        s.rpb = r;
    }
    s.groups = (rows + s.rpb - 1) / s.rpb;
    return s;
}

template <bool NT>
hipError_t launch_update(const UpdateArgs& a, bool small, int narrow, int unroll, dim3 grid, size_t lds, hipStream_t st)
{
    if (small) {
        switch (unroll) {
        case 1: rb_update_small_kernel<1, NT><<<grid, TPB, lds, st>>>(a); break;
        case 2: rb_update_small_kernel<2, NT><<<grid, TPB, lds, st>>>(a); break;
        case 4: rb_update_small_kernel<4, NT><<<grid, TPB, lds, st>>>(a); break;
        default: rb_update_small_kernel<8, NT><<<grid, TPB, lds, st>>>(a); break;
        }
        return hipGetLastError();
    }
    if (narrow == 2) {                  // 8 bits per element: a lane holds four accesses per vector of the tile (at most four vectors)
        if (unroll == 1) rb_update_kernel<1, NT, 2><<<grid, TPB, lds, st>>>(a);
        else if (unroll == 2) rb_update_kernel<2, NT, 2><<<grid, TPB, lds, st>>>(a);
        else rb_update_kernel<4, NT, 2><<<grid, TPB, lds, st>>>(a);
        return hipGetLastError();
    }
    if (narrow == 1) {
        switch (unroll) {
        case 1: rb_update_kernel<1, NT, 1><<<grid, TPB, lds, st>>>(a); break;
        case 2: rb_update_kernel<2, NT, 1><<<grid, TPB, lds, st>>>(a); break;
        case 4: rb_update_kernel<4, NT, 1><<<grid, TPB, lds, st>>>(a); break;
        default: rb_update_kernel<8, NT, 1><<<grid, TPB, lds, st>>>(a); break;
        }
        return hipGetLastError();
    }
    switch (unroll) {
    case 1: rb_update_kernel<1, NT, 0><<<grid, TPB, lds, st>>>(a); break;
    case 2: rb_update_kernel<2, NT, 0><<<grid, TPB, lds, st>>>(a); break;
    case 4: rb_update_kernel<4, NT, 0><<<grid, TPB, lds, st>>>(a); break;
    default: rb_update_kernel<8, NT, 0><<<grid, TPB, lds, st>>>(a); break;
    }
    return hipGetLastError();
}

template <bool NT>
hipError_t launch_sample(const SampleArgs& a, bool small, int widen, int unroll, dim3 grid, size_t lds, hipStream_t st)
{
    if (small) {
        switch (unroll) {
        case 1: rb_sample_small_kernel<1, NT><<<grid, TPB, lds, st>>>(a); break;
        case 2: rb_sample_small_kernel<2, NT><<<grid, TPB, lds, st>>>(a); break;
        case 4: rb_sample_small_kernel<4, NT><<<grid, TPB, lds, st>>>(a); break;
        default: rb_sample_small_kernel<8, NT><<<grid, TPB, lds, st>>>(a); break;
        }
        return hipGetLastError();
    }
    if (widen == 2) {
        if (unroll == 1) rb_sample_kernel<1, NT, 2><<<grid, TPB, lds, st>>>(a);
        else if (unroll == 2) rb_sample_kernel<2, NT, 2><<<grid, TPB, lds, st>>>(a);
        else rb_sample_kernel<4, NT, 2><<<grid, TPB, lds, st>>>(a);
        return hipGetLastError();
    }
    if (widen == 1) {
        switch (unroll) {
        case 1: rb_sample_kernel<1, NT, 1><<<grid, TPB, lds, st>>>(a); break;
        case 2: rb_sample_kernel<2, NT, 1><<<grid, TPB, lds, st>>>(a); break;
        case 4: rb_sample_kernel<4, NT, 1><<<grid, TPB, lds, st>>>(a); break;
        default: rb_sample_kernel<8, NT, 1><<<grid, TPB, lds, st>>>(a); break;
        }
        return hipGetLastError();
    }
    switch (unroll) {
    case 1: rb_sample_kernel<1, NT, 0><<<grid, TPB, lds, st>>>(a); break;
    case 2: rb_sample_kernel<2, NT, 0><<<grid, TPB, lds, st>>>(a); break;
    case 4: rb_sample_kernel<4, NT, 0><<<grid, TPB, lds, st>>>(a); break;
    default: rb_sample_kernel<8, NT, 0><<<grid, TPB, lds, st>>>(a); break;
    }
    return hipGetLastError();
}

template <bool NT>
hipError_t launch_step(const StepArgs& a, int unroll, dim3 grid, size_t lds, hipStream_t st)
{
    switch (unroll) {
    case 1: rb_step_small_kernel<1, NT><<<grid, TPB, lds, st>>>(a); break;
    case 2: rb_step_small_kernel<2, NT><<<grid, TPB, lds, st>>>(a); break;
    case 4: rb_step_small_kernel<4, NT><<<grid, TPB, lds, st>>>(a); break;
    default: rb_step_small_kernel<8, NT><<<grid, TPB, lds, st>>>(a); break;
    }
    return hipGetLastError();
}

template <bool NT, int PACE>
hipError_t launch_copy(vec16* dst, const vec16* src, int64_t nvec, int unroll, hipStream_t st)
{
    const int64_t cap = (int64_t)TPB * unroll;
    dim3 grid((unsigned)((nvec + cap - 1) / cap));
    switch (unroll) {
    case 1: rb_copy_kernel<1, NT, PACE><<<grid, TPB, 0, st>>>(dst, src, nvec); break;
    case 2: rb_copy_kernel<2, NT, PACE><<<grid, TPB, 0, st>>>(dst, src, nvec); break;
    case 4: rb_copy_kernel<4, NT, PACE><<<grid, TPB, 0, st>>>(dst, src, nvec); break;
    default: rb_copy_kernel<8, NT, PACE><<<grid, TPB, 0, st>>>(dst, src, nvec); break;
    }
    return hipGetLastError();
}

Seed make_seed(uint64_t seed, uint64_t step)
{
    Seed s;
    s.seed_lo = (uint32_t)seed;
    s.seed_hi = (uint32_t)(seed >> 32);
    s.step_lo = (uint32_t)step;
    s.step_hi = (uint32_t)(step >> 32);
    return s;
}

template <bool NT, int ST>
hipError_t launch_planned_s(const MoveArgs& m, const PlanArgs& next, int unroll, dim3 grid, size_t lds, hipStream_t st)
{
    switch (unroll) {
    case 1: rb_step_planned_kernel<1, NT, ST><<<grid, TPB, lds, st>>>(m, next); break;
    case 2: rb_step_planned_kernel<2, NT, ST><<<grid, TPB, lds, st>>>(m, next); break;
    case 4: rb_step_planned_kernel<4, NT, ST><<<grid, TPB, lds, st>>>(m, next); break;
    default:
        if constexpr (ST == RB_STORE_U8) return hipErrorInvalidValue;    // (at most four vectors per lane: step_planned)
        else rb_step_planned_kernel<8, NT, ST><<<grid, TPB, lds, st>>>(m, next);
        break;
    }
    return hipGetLastError();
}

template <bool NT>
hipError_t launch_planned(const MoveArgs& m, const PlanArgs& next, int storage, int unroll, dim3 grid, size_t lds, hipStream_t st)
{
    switch (storage) {
    case RB_STORE_BF16: return launch_planned_s<NT, RB_STORE_BF16>(m, next, unroll, grid, lds, st);
    case RB_STORE_U8: return launch_planned_s<NT, RB_STORE_U8>(m, next, unroll, grid, lds, st);
    default: return launch_planned_s<NT, RB_STORE_SAME>(m, next, unroll, grid, lds, st);
    }
}

// Called by every entry point other than rb_update_sample.  A step that was planned ahead will not
// be executed as planned: the fill counts go back to the copy the planner read (it only wrote the
// other one).  An announcement that has not been used yet is forgotten as well: it was made for the
// call that should have come next.
void discard_window_plan(rb_buffer* rb)
{
    if (rb->wplan_valid) {
        rb->cur ^= 1;
        rb->wplan_valid = false;
    }
}

// Whether the window that the call before planned ahead (window_plan_kept) is the start of this call: same shape, seed
// and step number, and the very label arrays that were announced.
bool window_plan_matches(const rb_buffer* rb, int form, int64_t n, const int64_t* const* batch_y, int64_t b, int64_t c, int64_t r,
                         uint64_t seed, uint64_t first_step)
{
    bool same = rb->wplan_valid && rb->wplan_form == form && rb->wplan_w <= n && rb->wplan_b == b && rb->wplan_c == c && rb->wplan_r == r &&
                rb->wplan_seed == seed && rb->wplan_first == first_step;
    for (int64_t k = 0; same && k < rb->wplan_w; ++k) same = rb->wplan_y[k] == batch_y[k];
    return same;
}

// The last launch of a call has planned the first w steps of the call that was announced, into table tbl of the given
// form (MANY_SMALL, MANY_LARGE).
void window_plan_kept(rb_buffer* rb, int form, int64_t w, int64_t b, int64_t c, int64_t r, uint64_t seed, uint64_t first_step, int tbl,
                      int64_t nat, const int64_t* const* ann_y)
{
    rb->wplan_valid = true;
    rb->wplan_form = form;
    rb->wplan_w = w; rb->wplan_b = b; rb->wplan_c = c; rb->wplan_r = r;
    rb->wplan_seed = seed; rb->wplan_first = first_step;
    rb->wplan_tbl = tbl;
    rb->wplan_nat = nat;
    for (int64_t k = 0; k < w; ++k) rb->wplan_y[k] = ann_y[k];
}

void discard_plan(rb_buffer* rb)
{
    if (rb->plan_valid) {
        rb->cur ^= 1;
        rb->plan_valid = false;
    }
    discard_window_plan(rb);
    rb->next_y = nullptr;
    rb->ann_n = 0;
}

PlanArgs make_plan(const rb_buffer* rb, const int64_t* batch_y, int64_t b, int64_t c, int64_t r, uint64_t seed, uint64_t step)
{
    PlanArgs p;
    p.batch_y = batch_y;
    p.fill_old = reinterpret_cast<const int32_t*>(rb->ws + rb->off_fill[rb->cur]);
    p.fill_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_fill[rb->cur ^ 1]);
    p.chunk_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_chunk[rb->cur ^ 1]);
    p.table = rb->ws + rb->off_tbl[rb->tbl_next];
    p.sd = make_seed(seed, step);
    p.b = (int32_t)b; p.c = (int32_t)c; p.r = (int32_t)r;
    p.K = (int32_t)rb->K; p.nchunks = rb->nchunks;
    p.S = rb->S;
    p.eviction = rb->eviction;
    p.aux_old = reinterpret_cast<const int32_t*>(rb->ws + rb->off_aux[rb->cur]);
    p.aux_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_aux[rb->cur ^ 1]);
    p.selection = rb->selection;
    p.ce = (int32_t)(rb->selection == RB_SELECT_BERNOULLI ? b : c);
    return p;
}

// Host bookkeeping after a plan has been enqueued.
void plan_enqueued(rb_buffer* rb, const int64_t* batch_y, int64_t b, int64_t c, int64_t r, uint64_t seed, uint64_t step)
{
    rb->cur ^= 1;
    rb->tbl_planned = rb->tbl_next;
    rb->tbl_next ^= 1;
    rb->plan_valid = true;
    rb->plan_y = batch_y; rb->plan_b = b; rb->plan_c = c; rb->plan_r = r; rb->plan_seed = seed; rb->plan_step = step;
}

// One step of the plan-ahead form: plan it now unless the previous launch already did, move its
// rows by the table, and let the same launch plan the following step when its labels are known.
int step_planned(rb_buffer* rb, const void* batch_x, const int64_t* batch_y, int64_t b, int64_t c, int64_t r,
                 uint64_t seed, uint64_t step, void* out_x, int64_t* out_y, const int64_t* next_y)
{
    if (!rb->plan_valid) {
        const PlanArgs now = make_plan(rb, batch_y, b, c, r, seed, step);
        rb_plan_kernel<<<dim3(1), TPB, (size_t)b * 8, rb->stream>>>(now);
        if (hipGetLastError() != hipSuccess) return RB_EHIP;
        plan_enqueued(rb, batch_y, b, c, r, seed, step);
    }
    // (with 8-bit storage a lane holds four accesses per vector: at most four vectors)
    const Shape sh = plan_shape(rb, c + r, TPB, rb->storage == RB_STORE_U8 ? 4 : 8);
    MoveArgs m;
    m.batch_x = static_cast<const vec16*>(batch_x);
    m.buf_x = static_cast<vec16*>(rb->buf_x);
    m.buf_y = rb->buf_y;
    m.out_x = static_cast<vec16*>(out_x);
    m.out_y = out_y;
    m.table = rb->ws + rb->off_tbl[rb->tbl_planned];
    m.state = reinterpret_cast<DevState*>(rb->ws);
    m.c = (int32_t)c; m.r = (int32_t)r; m.cgrid = (int32_t)c;
    m.S = rb->S;
    m.row_vec = rb->row_vec;
    m.tpr = sh.tpr; m.tile_vec = sh.tile_vec; m.tile_rem = sh.tile_rem;
    const int64_t movers = (c + r) * sh.tpr;
    rb->plan_valid = false;                     // this step is being executed
    m.plan_next = next_y ? 1 : 0;
    PlanArgs next = {};
    if (next_y) next = make_plan(rb, next_y, b, c, r, seed, step + 1);
    const dim3 grid((unsigned)(movers + m.plan_next));
    const size_t lds = next_y ? (size_t)b * 8 : 0;
    const hipError_t e = rb->opt_nt ? launch_planned<true>(m, next, rb->storage, sh.unroll, grid, lds, rb->stream)
                                    : launch_planned<false>(m, next, rb->storage, sh.unroll, grid, lds, rb->stream);
    if (e == hipSuccess && next_y) plan_enqueued(rb, next_y, b, c, r, seed, step + 1);
    if (e != hipSuccess) return RB_EHIP;
    rb->updates += 1;
    return RB_OK;
}

// The 1024-thread kernels ask for more dynamic LDS than a kernel gets by default: allowed once per kernel and device.
template <auto kernel>
hipError_t allow_big_lds()
{
    static bool allowed[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    if (dev < 0 || dev >= 64 || !allowed[dev]) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 (int)BIG_LDS_BYTES);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) allowed[dev] = true;
    }
    return hipSuccess;
}

template <int U, bool NT, int ST>
hipError_t launch_big_u(const MoveArgs& m, const PlanArgs& next, const uint32_t* fwd, uint32_t* fwd_next, dim3 grid, hipStream_t st)
{
    // (the converting movers have to fit the 128 registers per lane of a 1024-thread workgroup: big_shape)
    if constexpr ((ST == RB_STORE_U8 && U > 2) || (ST == RB_STORE_BF16 && U > 8)) {
        return hipErrorInvalidValue;
    } else {
        const size_t lds = m.plan_next ? BIG_LDS_BYTES : 0;
        if (lds != 0) {
            const hipError_t e = allow_big_lds<&rb_step_big_kernel<U, NT, ST>>();
            if (e != hipSuccess) return e;
        }
        rb_step_big_kernel<U, NT, ST><<<grid, BIG_TPB, lds, st>>>(m, next, fwd, fwd_next);
        return hipGetLastError();
    }
}

template <bool NT, int ST>
hipError_t launch_big_s(const MoveArgs& m, const PlanArgs& next, const uint32_t* fwd, uint32_t* fwd_next, int unroll, dim3 grid,
                        hipStream_t st)
{
    switch (unroll) {
    case 1: return launch_big_u<1, NT, ST>(m, next, fwd, fwd_next, grid, st);
    case 2: return launch_big_u<2, NT, ST>(m, next, fwd, fwd_next, grid, st);
    case 4: return launch_big_u<4, NT, ST>(m, next, fwd, fwd_next, grid, st);
    case 6: return launch_big_u<6, NT, ST>(m, next, fwd, fwd_next, grid, st);
    case 8: return launch_big_u<8, NT, ST>(m, next, fwd, fwd_next, grid, st);
    case 10: return launch_big_u<10, NT, ST>(m, next, fwd, fwd_next, grid, st);
    case 12: return launch_big_u<12, NT, ST>(m, next, fwd, fwd_next, grid, st);
    default: return hipErrorInvalidValue;
    }
}

template <bool NT>
hipError_t launch_big(const MoveArgs& m, const PlanArgs& next, const uint32_t* fwd, uint32_t* fwd_next, int storage, int unroll,
                      dim3 grid, hipStream_t st)
{
    switch (storage) {
    case RB_STORE_BF16: return launch_big_s<NT, RB_STORE_BF16>(m, next, fwd, fwd_next, unroll, grid, st);
    case RB_STORE_U8: return launch_big_s<NT, RB_STORE_U8>(m, next, fwd, fwd_next, unroll, grid, st);
    default: return launch_big_s<NT, RB_STORE_SAME>(m, next, fwd, fwd_next, unroll, grid, st);
    }
}

// Tiles of the large-count launch.  Its workgroups hold four groups of movers each, and a compute unit holds one such
// workgroup at a time (traced: of 325 workgroups the last 69 start when the first ones end), so a launch of a few
// hundred workgroups runs in rounds of 256, and a round that is nearly empty costs as much as a full one (measured
// on MI355X with a bare mover, 129 rows of 301 056 bytes: 323 workgroups of four 32 KiB tiles 18.9 us, 226
// workgroups of four 42 KiB tiles 14.9 us, 258 workgroups 20.1 us; 256 rows: 640 workgroups 33.6 us, 448
// workgroups 31.4 us; the whole step gains less: 65 candidates and 64 representatives 17.3 -> 16.5 us, 128 and 128
// 33.0 -> 32.0 us).  So, when the rows are long enough (tiles of 12 KiB and more), a row gets as many tiles as keep
// the whole launch, planners included, within one round, or else within two.  Measured and not adopted: at most
// one mover workgroup per compute unit whose groups go round the tiles themselves (5 to 10 % slower than letting
// the second round of workgroups start as the first ones end); for many short rows a wavefront per row, sixteen
// rows per workgroup, so that one round suffices (10000 classes, 1024 + 1024 rows of 8 KiB: no change, the step is
// bound by the planners and the launch itself).
Shape big_shape(const rb_buffer* rb, int64_t rows, int planners)
{
    // (with 8-bit storage a lane holds four accesses per vector, and these workgroups have 128 registers per lane: two vectors)
    if (rb->storage == RB_STORE_U8) return plan_shape(rb, rows, BIG_GROUP, 2);
    Shape s = plan_shape(rb, rows, BIG_GROUP);
    if (rb->opt_unroll != 0) return s;
    constexpr int64_t CUS = 256;
    const int64_t nunits = (rb->row_vec + TILE_UNIT - 1) / TILE_UNIT;
    for (int64_t k = 1; k <= 2; ++k) {
        int64_t tpr = (CUS * k - planners) * BIG_GROUPS / rows;
        if (tpr > nunits) tpr = nunits;
        if (tpr < 1) continue;
        const int64_t tile = (nunits / tpr + (nunits % tpr ? 1 : 0)) * TILE_UNIT;      // vectors of the longest tile
        int u = (int)((tile + BIG_GROUP - 1) / BIG_GROUP);
        if (u > (rb->storage == RB_STORE_BF16 ? 8 : 12)) continue;
        if (u < 4) break;                                                                 // short rows: the plain split
        u = (u + 1) / 2 * 2;                                                              // 4, 6, 8, 10 or 12
        s.unroll = u;
        s.tpr = (int)tpr;
        s.tile_vec = (int)(nunits / tpr);
        s.tile_rem = (int)(nunits % tpr);
        s.rpb = 1;
        s.groups = rows;
        return s;
    }
    return s;
}

// One step of the plan-ahead form for large counts (up to BIG_MAX candidates and representatives, up to
// BIG_CLASSES classes); same bookkeeping as step_planned, the tables are the (larger) ones that the
// several-steps-per-launch form uses for shapes this form does not serve.  Two workgroups plan.
int step_big(rb_buffer* rb, const void* batch_x, const int64_t* batch_y, int64_t b, int64_t c, int64_t r,
             uint64_t seed, uint64_t step, void* out_x, int64_t* out_y, const int64_t* next_y)
{
    static_assert(BIG_TABLE_BYTES <= WIN_TABLE_BYTES, "the big plan's table must fit the window table");
    if (!rb->plan_valid) {
        PlanArgs now = make_plan(rb, batch_y, b, c, r, seed, step);
        now.table = rb->ws + rb->off_wtbl[rb->tbl_next];
        if (allow_big_lds<&rb_big_plan_kernel>() != hipSuccess) return RB_EHIP;
        rb_big_plan_kernel<<<dim3(2), BIG_TPB, BIG_LDS_BYTES, rb->stream>>>(now, reinterpret_cast<uint32_t*>(rb->ws + rb->off_bfwd[rb->tbl_next]));
        if (hipGetLastError() != hipSuccess) return RB_EHIP;
        plan_enqueued(rb, batch_y, b, c, r, seed, step);
    }
    // candidate entries of the table, and how many of them the grid covers: all c, or, with the Bernoulli selection
    // (about c of the b positions are selected), c and eight standard deviations (more are served by going round)
    const bool bernoulli = rb->selection == RB_SELECT_BERNOULLI;
    const int64_t ce = bernoulli ? b : c;
    int64_t margin = 16;
    while (margin * margin < 64 * c) ++margin;
    const int64_t cgrid = bernoulli ? std::min(b, c + margin) : c;
    const Shape sh = big_shape(rb, cgrid + r, next_y ? 2 : 0);
    MoveArgs m;
    m.batch_x = static_cast<const vec16*>(batch_x);
    m.buf_x = static_cast<vec16*>(rb->buf_x);
    m.buf_y = rb->buf_y;
    m.out_x = static_cast<vec16*>(out_x);
    m.out_y = out_y;
    m.table = rb->ws + rb->off_wtbl[rb->tbl_planned];
    m.state = reinterpret_cast<DevState*>(rb->ws);
    m.c = (int32_t)ce; m.r = (int32_t)r; m.cgrid = (int32_t)cgrid;
    m.S = rb->S;
    m.row_vec = rb->row_vec;
    m.tpr = sh.tpr; m.tile_vec = sh.tile_vec; m.tile_rem = sh.tile_rem;
    const int64_t items = (cgrid + r) * sh.tpr;
    rb->plan_valid = false;                     // this step is being executed
    m.plan_next = next_y ? 1 : 0;
    PlanArgs next = {};
    if (next_y) {
        next = make_plan(rb, next_y, b, c, r, seed, step + 1);
        next.table = rb->ws + rb->off_wtbl[rb->tbl_next];
    }
    const uint32_t* fwd = reinterpret_cast<const uint32_t*>(rb->ws + rb->off_bfwd[rb->tbl_planned]);
    uint32_t* fwd_next = reinterpret_cast<uint32_t*>(rb->ws + rb->off_bfwd[rb->tbl_next]);
    const dim3 grid((unsigned)((items + BIG_GROUPS - 1) / BIG_GROUPS + 2 * m.plan_next));
    const hipError_t e = rb->opt_nt ? launch_big<true>(m, next, fwd, fwd_next, rb->storage, sh.unroll, grid, rb->stream)
                                    : launch_big<false>(m, next, fwd, fwd_next, rb->storage, sh.unroll, grid, rb->stream);
    if (e == hipSuccess && next_y) plan_enqueued(rb, next_y, b, c, r, seed, step + 1);
    if (e != hipSuccess) return RB_EHIP;
    rb->updates += 1;
    return RB_OK;
}

template <bool NT, int ST, bool AUX>
hipError_t launch_window_u(const WinMoveArgs& m, const WinPlanArgs& next, int unroll, dim3 grid, hipStream_t st)
{
    switch (unroll) {
    case 1: rb_window_kernel<1, NT, ST, AUX><<<grid, TPB, 0, st>>>(m, next); break;
    case 2: rb_window_kernel<2, NT, ST, AUX><<<grid, TPB, 0, st>>>(m, next); break;
    case 4: rb_window_kernel<4, NT, ST, AUX><<<grid, TPB, 0, st>>>(m, next); break;
    default:
        if constexpr (ST == RB_STORE_U8) return hipErrorInvalidValue;    // (a lane holds four accesses per vector: at most four vectors)
        else rb_window_kernel<8, NT, ST, AUX><<<grid, TPB, 0, st>>>(m, next);
        break;
    }
    return hipGetLastError();
}

// aux: the replacement strategy keeps per-class state (FIFO, reservoir)
template <bool NT>
hipError_t launch_window(const WinMoveArgs& m, const WinPlanArgs& next, int storage, bool aux, int unroll, dim3 grid, hipStream_t st)
{
    switch (storage) {
    case RB_STORE_BF16:
        return aux ? launch_window_u<NT, RB_STORE_BF16, true>(m, next, unroll, grid, st) : launch_window_u<NT, RB_STORE_BF16, false>(m, next, unroll, grid, st);
    case RB_STORE_U8:
        return aux ? launch_window_u<NT, RB_STORE_U8, true>(m, next, unroll, grid, st) : launch_window_u<NT, RB_STORE_U8, false>(m, next, unroll, grid, st);
    default:
        return aux ? launch_window_u<NT, RB_STORE_SAME, true>(m, next, unroll, grid, st) : launch_window_u<NT, RB_STORE_SAME, false>(m, next, unroll, grid, st);
    }
}

WinPlanArgs window_plan_args(rb_buffer* rb, const int64_t* const* batch_y, int64_t at, int64_t w, int64_t b, int64_t c, int64_t r,
                             uint64_t seed, uint64_t first_step, int table)
{
    WinPlanArgs p = {};
    for (int64_t i = 0; i < w; ++i) p.batch_y[i] = batch_y[at + i];
    p.fill_old = reinterpret_cast<const int32_t*>(rb->ws + rb->off_fill[rb->cur]);
    p.fill_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_fill[rb->cur ^ 1]);
    p.chunk_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_chunk[rb->cur ^ 1]);
    p.table = rb->ws + rb->off_wtbl[table];
    p.seed_lo = (uint32_t)seed; p.seed_hi = (uint32_t)(seed >> 32);
    p.first_step = first_step + (uint64_t)at;
    p.w = (int32_t)w;
    p.b = (int32_t)b; p.c = (int32_t)c; p.r = (int32_t)r;
    p.K = (int32_t)rb->K; p.nchunks = rb->nchunks;
    p.S = rb->S;
    p.eviction = rb->eviction;
    p.aux_old = reinterpret_cast<const int32_t*>(rb->ws + rb->off_aux[rb->cur]);
    p.aux_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_aux[rb->cur ^ 1]);
    return p;
}

// `left` steps go into launches of at most `cap` steps: the size of the first of them when they are made as equal
// as possible (20 steps, 16 at most: 10 and 10, not 16 and 4 - a short launch hides little of the next window's plan).
int64_t even_share(int64_t left, int64_t cap)
{
    if (left <= 0) return 0;
    const int64_t launches = (left + cap - 1) / cap;
    return (left + launches - 1) / launches;
}

// Whether rb_update_sample_many puts several steps of this shape into one launch, and how many at most: the option,
// and what the planner's tables hold.  1: one launch (or two) per step.
int64_t window_limit(const rb_buffer* rb, int64_t b, int64_t c, int64_t r)
{
    const bool windowed = c >= 1 && c <= WAVE && r >= 1 && r <= WAVE && rb->nchunks <= DIRECT_CHUNKS && b <= 2048 && rb->opt_fuse &&
                          rb->opt_window >= 2 && rb->selection == RB_SELECT_EXACT;
    if (!windowed) return 1;
    return std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(WIN_MAX, rb->opt_window),
                                                  std::min<int64_t>(WIN_ENTRIES / (c + r), WIN_SLOTS / std::max(c, r))));
}

// n steps as launches of up to WIN_MAX steps each.  Workgroup 0 of every launch plans the next
// window while the others move the rows of this one; the first window is planned by a launch of its
// own and kept short, so that the movers get going early - unless the last launch of the call before
// planned it (ann_y: labels announced for the first ann_n steps of the call after this one).
int steps_windowed(rb_buffer* rb, int64_t n, const void* const* batch_x, const int64_t* const* batch_y, int64_t b, int64_t c,
                   int64_t r, uint64_t seed, uint64_t first_step, void* const* out_x, int64_t* const* out_y,
                   int64_t ann_n, const int64_t* const* ann_y)
{
    static_assert(sizeof(rb_buffer::ann_y) / sizeof(void*) >= WIN_MAX, "announced labels and planned windows are kept for a whole launch");
    const int64_t wmax = window_limit(rb, b, c, r);
    // With thousands of workgroups per launch, and the planner's LDS leaving room for four workgroups per
    // compute unit, tiles of four vectors per thread measured best (1000 classes of 3x224x224 bfloat16 samples,
    // 64 candidates and representatives: 13.1 us per step against 14.1 with two and 14.2 with eight; binary32
    // samples, 8 and 8: 3.9 against 4.1 and 4.1).  With binary32 samples stored as bfloat16 a thread holds twice as
    // many half vectors, and two per thread measured best (8 and 8: 2.6 us against 2.7).
    // With 8-bit storage a thread holds four quarter vectors per vector of the tile (16 bytes of the sample each): one.
    const int unroll_option = rb->opt_unroll;
    Shape sh = plan_shape(rb, wmax * (c + r), TPB, rb->storage == RB_STORE_U8 ? 4 : 8,
                          rb->storage == RB_STORE_U8 ? 1 : rb->storage == RB_STORE_BF16 ? 2 : 4);
    // ... and a third more tiles than that needs, i.e. tiles about three quarters full (most threads hold three vectors):
    // the launch's workgroups come in more and shorter rounds.  Measured with 301 KB rows, 64 + 64 per step: 12.42 us per step
    // with 25 to 28 tiles per row against 12.74 with the 19 that four vectors per thread need, 13.4 with 38; 602 KB rows,
    // 8 + 8 per step: 3.06 with 38 to 46 against 3.07 with 37, 3.12 with 56.
    if (unroll_option == 0 && sh.unroll == 4 && sh.tpr > 1) {
        const int64_t nunits = (rb->row_vec + TILE_UNIT - 1) / TILE_UNIT;
        sh.tpr = (int)((rb->row_vec + (int64_t)TPB * 3 - 1) / ((int64_t)TPB * 3));
        sh.tile_vec = (int)(nunits / sh.tpr);
        sh.tile_rem = (int)(nunits % sh.tpr);
    }
    // Window sizes.  A launch of w steps should not have to wait for the plan of the next window, which the one
    // planner workgroup makes meanwhile; so the windows grow as fast as that allows, and the first one (planned
    // with nothing to hide behind) is the smallest from which they can grow.  Measured on MI355X: rows move at
    // about 5.5 TB/s; a window's plan takes about 3 us more than a launch's own fixed cost, plus 1.6 us and
    // 0.04 us per candidate or representative for every step.
    const double move_us = (double)(c + r) * (double)(rb->row_bytes + rb->sample_bytes) / 5.5e6;
    const double plan_us = 1.6 + 0.04 * (double)std::max(c, r);
    const auto grown = [&](int64_t w) {
        return std::max<int64_t>(1, std::min<int64_t>(wmax, (int64_t)((move_us * (double)w - 3.0) / plan_us)));
    };
    int64_t w0 = 1;
    while (w0 < wmax && grown(w0) <= w0) ++w0;
    int64_t at = 0, w;
    int tbl;
    const bool resume = window_plan_matches(rb, MANY_SMALL, n, batch_y, b, c, r, seed, first_step);
    int64_t nat;                                // size the windows have grown to, whatever a call's end cut them down to
    if (resume) {
        w = rb->wplan_w;
        tbl = rb->wplan_tbl;
        nat = rb->wplan_nat;
        rb->wplan_valid = false;                // it is being executed
    } else {
        discard_window_plan(rb);
        w = std::min(w0, n);
        nat = w0;
        tbl = 0;
        const WinPlanArgs p = window_plan_args(rb, batch_y, 0, w, b, c, r, seed, first_step, tbl);
        if (rb->eviction != RB_EVICT_UNIFORM) rb_window_plan_kernel<true><<<dim3(1), TPB, 0, rb->stream>>>(p);
        else rb_window_plan_kernel<false><<<dim3(1), TPB, 0, rb->stream>>>(p);
        if (hipGetLastError() != hipSuccess) return RB_EHIP;
        rb->cur ^= 1;
    }
    while (at < n) {
        const int64_t next_at = at + w;
        nat = std::min(wmax, std::max(nat, grown(nat)));
        // the next window: the steps that are left in equal parts rather than full windows and a short one
        int64_t next_w = even_share(n - next_at, nat);
        // the last launch of the call plans the first steps of the call that was announced
        const bool ahead = next_w == 0 && ann_n > 0;
        if (ahead) next_w = even_share(ann_n, nat);
        WinPlanArgs next = {};
        if (ahead) next = window_plan_args(rb, ann_y, 0, next_w, b, c, r, seed, first_step + (uint64_t)n, tbl ^ 1);
        else if (next_w > 0) next = window_plan_args(rb, batch_y, next_at, next_w, b, c, r, seed, first_step, tbl ^ 1);
        WinMoveArgs m = {};
        for (int64_t k = 0; k < w; ++k) {
            m.batch_x[k] = static_cast<const vec16*>(batch_x[at + k]);
            m.out_x[k] = static_cast<vec16*>(out_x[at + k]);
            m.out_y[k] = out_y[at + k];
        }
        m.buf_x = static_cast<vec16*>(rb->buf_x);
        m.buf_y = rb->buf_y;
        m.table = rb->ws + rb->off_wtbl[tbl];
        m.state = reinterpret_cast<DevState*>(rb->ws);
        m.w = (int32_t)w; m.c = (int32_t)c; m.r = (int32_t)r;
        m.S = rb->S;
        m.row_vec = rb->row_vec;
        m.tpr = sh.tpr; m.tile_vec = sh.tile_vec; m.tile_rem = sh.tile_rem;
        const dim3 grid((unsigned)(w * (c + r) * sh.tpr + (next_w > 0 ? 1 : 0)));
        const bool aux = rb->eviction != RB_EVICT_UNIFORM;
        const hipError_t e = rb->opt_nt ? launch_window<true>(m, next, rb->storage, aux, sh.unroll, grid, rb->stream)
                                        : launch_window<false>(m, next, rb->storage, aux, sh.unroll, grid, rb->stream);
        if (e != hipSuccess) return RB_EHIP;
        if (next_w > 0) rb->cur ^= 1;
        if (ahead) window_plan_kept(rb, MANY_SMALL, next_w, b, c, r, seed, first_step + (uint64_t)n, tbl ^ 1, nat, ann_y);
        at = next_at;
        w = ahead ? 0 : next_w;
        tbl ^= 1;
    }
    rb->updates += n;
    return RB_OK;
}

template <int U, int W, bool NT, int ST>
hipError_t launch_bigwin_u(const BwMoveArgs& m, const BwPlanArgs& next, dim3 grid, hipStream_t st)
{
    if constexpr (ST == RB_STORE_U8 && U > 2) {
        return hipErrorInvalidValue;           // (a lane holds four accesses per vector, and these workgroups have 128 registers per lane: bigwin_shape)
    } else {
        const size_t lds = next.w > 0 ? BIG_LDS_BYTES : 0;
        if (lds != 0) {
            const hipError_t e = allow_big_lds<&rb_bigwin_kernel<U, W, NT, ST>>();
            if (e != hipSuccess) return e;
        }
        rb_bigwin_kernel<U, W, NT, ST><<<grid, BIG_TPB, lds, st>>>(m, next);
        return hipGetLastError();
    }
}

// width: threads per tile (bigwin_width), unroll: vectors per thread
template <bool NT, int ST>
hipError_t launch_bigwin_s(const BwMoveArgs& m, const BwPlanArgs& next, int width, int unroll, dim3 grid, hipStream_t st)
{
    if (width == WAVE) return unroll == 2 ? launch_bigwin_u<2, WAVE, NT, ST>(m, next, grid, st) : launch_bigwin_u<8, WAVE, NT, ST>(m, next, grid, st);
    if (width == 2 * WAVE) return launch_bigwin_u<8, 2 * WAVE, NT, ST>(m, next, grid, st);
    switch (unroll) {
    case 1: return launch_bigwin_u<1, TPB, NT, ST>(m, next, grid, st);
    case 2: return launch_bigwin_u<2, TPB, NT, ST>(m, next, grid, st);
    case 4: return launch_bigwin_u<4, TPB, NT, ST>(m, next, grid, st);
    default: return launch_bigwin_u<8, TPB, NT, ST>(m, next, grid, st);
    }
}

template <bool NT>
hipError_t launch_bigwin(const BwMoveArgs& m, const BwPlanArgs& next, int storage, int width, int unroll, dim3 grid, hipStream_t st)
{
    switch (storage) {
    case RB_STORE_BF16: return launch_bigwin_s<NT, RB_STORE_BF16>(m, next, width, unroll, grid, st);
    case RB_STORE_U8: return launch_bigwin_s<NT, RB_STORE_U8>(m, next, width, unroll, grid, st);
    default: return launch_bigwin_s<NT, RB_STORE_SAME>(m, next, width, unroll, grid, st);
    }
}

// Tiles of the several-steps launch for large counts.  A compute unit holds a fixed number of wavefronts, so the bytes it
// has in flight are what a wavefront has in flight: rows of up to 8 KiB are moved by one wavefront each (eight vectors per
// lane), rows of up to 16 KiB by two; longer rows are cut into tiles for 256 threads like everywhere else.
Shape bigwin_shape(const rb_buffer* rb, int64_t rows, int& width)
{
    width = TPB;
    const bool q8 = rb->storage == RB_STORE_U8;        // at most two vectors per lane: a wavefront per row up to 128 vectors
    if (rb->opt_unroll == 0 && rb->row_vec <= (q8 ? WAVE * 2 : 2 * WAVE * 8)) width = rb->row_vec <= WAVE * 8 ? WAVE : 2 * WAVE;
    // (long rows stored as bfloat16: a lane holds two half vectors per vector, four vectors measured best - 1000 classes of
    // 3x224x224 samples, 8 + 8 rows per step: 2.86 us per step against 3.05 with two and 3.39 with eight)
    if (width == TPB) return plan_shape(rb, rows, TPB, q8 ? 2 : 8, rb->storage == RB_STORE_BF16 ? 4 : 0);
    Shape s;
    s.unroll = width == WAVE && rb->row_vec <= WAVE * 2 ? 2 : 8;
    s.tpr = 1;
    const int64_t nunits = (rb->row_vec + TILE_UNIT - 1) / TILE_UNIT;
    s.tile_vec = (int)nunits;
    s.tile_rem = 0;
    s.rpb = 1;
    s.groups = rows;
    return s;
}

// Whether rb_update_sample_many puts several steps of this shape into one launch of the large-count form, and how
// many at most (1: it does not).  Shapes that the small form takes (window_limit) are not meant.
int64_t bigwin_limit(const rb_buffer* rb, int64_t b, int64_t c, int64_t r)
{
    const bool eligible = c >= 1 && c <= BIG_MAX && r >= 1 && r <= BIG_MAX && b <= BIG_BATCH &&
                          rb->K <= BIG_CLASSES && rb->opt_fuse &&
                          rb->opt_window >= 2 && (rb->selection == RB_SELECT_EXACT || b <= BIG_MAX) && rb->K * rb->S <= INT64_C(0x7FFFFFFF) &&
                          rb->S <= INT32_MAX - (int64_t)BW_MAX * RB_MAX_BATCH;
    if (!eligible) return 1;
    return std::min<int64_t>(BW_MAX, rb->opt_window);
}

BwPlanArgs bigwin_plan_args(rb_buffer* rb, const int64_t* const* batch_y, int64_t at, int64_t w, int64_t b, int64_t c, int64_t r,
                            uint64_t seed, uint64_t first_step, int table)
{
    BwPlanArgs p = {};
    for (int64_t i = 0; i < w; ++i) p.batch_y[i] = batch_y[at + i];
    p.fill_old = reinterpret_cast<const int32_t*>(rb->ws + rb->off_fill[rb->cur]);
    p.fill_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_fill[rb->cur ^ 1]);
    p.chunk_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_chunk[rb->cur ^ 1]);
    p.table = rb->ws + rb->off_bwtbl[table];
    p.seed_lo = (uint32_t)seed; p.seed_hi = (uint32_t)(seed >> 32);
    p.first_step = first_step + (uint64_t)at;
    p.w = (int32_t)w;
    p.b = (int32_t)b; p.c = (int32_t)c; p.r = (int32_t)r;
    p.K = (int32_t)rb->K; p.nchunks = rb->nchunks;
    p.S = rb->S;
    p.eviction = rb->eviction;
    p.selection = rb->selection;
    p.ce = (int32_t)(rb->selection == RB_SELECT_BERNOULLI ? b : c);     // with the Bernoulli selection one thread and one entry per position
    rb->bw_number += 1;
    if (rb->bw_number == 0) rb->bw_number = 1;          // 0 is what a cleared flag shows
    p.number = rb->bw_number;
    rb->bw_table_number[table] = p.number;
    p.aux_old = reinterpret_cast<const int32_t*>(rb->ws + rb->off_aux[rb->cur]);
    p.aux_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_aux[rb->cur ^ 1]);
    return p;
}

// n steps of the large-count form as launches of up to BW_MAX steps each: the first 2 w' workgroups of every launch
// plan the next window of w' steps (rb_kernels_bigwin.h) while the others move the rows of this one.  Bookkeeping as
// in steps_windowed.  The planners of a window work side by side, so a plan takes about as long whatever the
// window's size: a chain of about fifteen dependent trips to memory (measured on MI355X, 1024 candidates and
// representatives of 10000 classes: 20 to 26 us on an idle chip, 30 to 45 us under the movers' traffic), so the
// windows are of full size from the second launch on; the first window, planned with nothing to hide behind, is
// short, so that rows start to move early.
int steps_bigwin(rb_buffer* rb, int64_t n, const void* const* batch_x, const int64_t* const* batch_y, int64_t b, int64_t c,
                 int64_t r, uint64_t seed, uint64_t first_step, void* const* out_x, int64_t* const* out_y,
                 int64_t ann_n, const int64_t* const* ann_y)
{
    static_assert(BW_MAX <= WIN_MAX, "announced labels and planned windows are kept for at most WIN_MAX steps");
    const int64_t wmax = bigwin_limit(rb, b, c, r);
    // candidate entries of a step in the table, and how many of them the grid covers: all c, or, with the Bernoulli selection
    // (about c of the b positions are selected), c and eight standard deviations (more are served by going round)
    const bool bernoulli = rb->selection == RB_SELECT_BERNOULLI;
    const int64_t ce = bernoulli ? b : c;
    int64_t margin = 16;
    while (margin * margin < 64 * c) ++margin;
    const int64_t cgrid = bernoulli ? std::min(b, c + margin) : c;
    int width;
    const Shape sh = bigwin_shape(rb, wmax * (cgrid + r), width);
    const double move_us = (double)(c + r) * (double)(rb->row_bytes + rb->sample_bytes) / 5.5e6;
    int64_t w0 = 1;
    while (w0 < wmax && move_us * (double)w0 < 12.0) ++w0;
    if (allow_big_lds<&rb_bigwin_plan_kernel>() != hipSuccess) return RB_EHIP;
    int64_t at = 0, w;
    int tbl;
    const bool resume = window_plan_matches(rb, MANY_LARGE, n, batch_y, b, c, r, seed, first_step);
    if (resume) {
        w = rb->wplan_w;
        tbl = rb->wplan_tbl;
        rb->wplan_valid = false;                // it is being executed
    } else {
        discard_window_plan(rb);
        w = std::min(w0, n);
        tbl = 0;
        const BwPlanArgs p = bigwin_plan_args(rb, batch_y, 0, w, b, c, r, seed, first_step, tbl);
        rb_bigwin_plan_kernel<<<dim3((unsigned)(2 * w)), BIG_TPB, BIG_LDS_BYTES, rb->stream>>>(p);
        if (hipGetLastError() != hipSuccess) return RB_EHIP;
        rb->cur ^= 1;
    }
    while (at < n) {
        const int64_t next_at = at + w;
        int64_t next_w = even_share(n - next_at, wmax);
        // the last launch of the call plans the first steps of the call that was announced
        const bool ahead = next_w == 0 && ann_n > 0;
        if (ahead) next_w = even_share(ann_n, wmax);
        BwMoveArgs m = {};
        for (int64_t k = 0; k < w; ++k) {
            m.batch_x[k] = static_cast<const vec16*>(batch_x[at + k]);
            m.out_x[k] = static_cast<vec16*>(out_x[at + k]);
            m.out_y[k] = out_y[at + k];
        }
        m.buf_x = static_cast<vec16*>(rb->buf_x);
        m.buf_y = rb->buf_y;
        m.table = rb->ws + rb->off_bwtbl[tbl];
        m.state = reinterpret_cast<DevState*>(rb->ws);
        m.w = (int32_t)w; m.c = (int32_t)ce; m.r = (int32_t)r; m.cgrid = (int32_t)cgrid;
        m.number = rb->bw_table_number[tbl];
        m.S = rb->S;
        m.row_vec = rb->row_vec;
        m.tpr = sh.tpr; m.tile_vec = sh.tile_vec; m.tile_rem = sh.tile_rem;
        BwPlanArgs next = {};
        if (ahead) next = bigwin_plan_args(rb, ann_y, 0, next_w, b, c, r, seed, first_step + (uint64_t)n, tbl ^ 1);
        else if (next_w > 0) next = bigwin_plan_args(rb, batch_y, next_at, next_w, b, c, r, seed, first_step, tbl ^ 1);
        const int64_t items = w * (cgrid + r) * sh.tpr;
        const int64_t per_block = BIG_TPB / width;
        const dim3 grid((unsigned)((items + per_block - 1) / per_block + 2 * next_w));
        const hipError_t e = rb->opt_nt ? launch_bigwin<true>(m, next, rb->storage, width, sh.unroll, grid, rb->stream)
                                        : launch_bigwin<false>(m, next, rb->storage, width, sh.unroll, grid, rb->stream);
        if (e != hipSuccess) return RB_EHIP;
        if (next_w > 0) rb->cur ^= 1;
        if (ahead) window_plan_kept(rb, MANY_LARGE, next_w, b, c, r, seed, first_step + (uint64_t)n, tbl ^ 1, wmax, ann_y);
        at = next_at;
        w = ahead ? 0 : next_w;
        tbl ^= 1;
    }
    rb->updates += n;
    return RB_OK;
}

// Which several-steps form serves this shape (MANY_SINGLE: none) and how many steps it puts into one launch at most.
// Where both forms could: the one workgroup that plans a window of the small form does so step after step (about
// 1.6 us + 0.04 us per candidate or representative each, 2.3 to 2.7 us under load), which is hidden as long as the rows
// of a step take longer to move; the two planners per step of the large form work side by side and take as long for
// sixteen steps as for one, but their launch moves long rows about 6 % slower, and rows that are converted on the way
// 15 to 25 % slower.  Measured on MI355X, us per step, small form against large form: 8 + 8 rows of 12 KB 2.7 : 1.05;
// 8 + 8 rows of 301 KB 2.59 : 2.07, 12 + 12 of them 2.88 : 2.86, 16 + 16 3.09 : 3.37; 4 + 4 rows of 602 KB 2.26 : 2.07,
// 6 + 6 2.52 : 2.58, 8 + 8 3.08 : 3.32; 8 + 8 rows of 602 KB stored as bfloat16 2.54 : 3.22, in 8 bits 2.5 : 2.9.  So the
// large form takes a shape when its rows move (at 5.5 TB/s) in less than 1.25 times the small form's nominal plan time,
// in less than 0.8 times when they are converted.  RB_OPT_PLANNERS overrides the choice where the shape allows.
int many_form(const rb_buffer* rb, int64_t b, int64_t c, int64_t r, int64_t& steps)
{
    const int64_t small = window_limit(rb, b, c, r), large = bigwin_limit(rb, b, c, r);
    int form = MANY_SINGLE;
    if (small >= 2 && large >= 2) {
        const double move_us = (double)(c + r) * (double)(rb->row_bytes + rb->sample_bytes) / 5.5e6;
        const double plan_us = 1.6 + 0.04 * (double)std::max(c, r);
        form = move_us < (rb->storage == RB_STORE_SAME ? 1.25 : 0.8) * plan_us ? MANY_LARGE : MANY_SMALL;
        if (rb->opt_planners != 0) form = rb->opt_planners;
    } else if (small >= 2) {
        form = MANY_SMALL;
    } else if (large >= 2) {
        form = MANY_LARGE;
    }
    steps = form == MANY_SMALL ? small : form == MANY_LARGE ? large : 1;
    return form;
}

// What the host can check of the arguments of one update + sample step.
int check_step(const rb_buffer* rb, const void* batch_x, const int64_t* batch_y, int64_t b, int64_t c, int64_t r,
               const void* out_x, const int64_t* out_y)
{
    if (!rb || !batch_x || !batch_y) return RB_EINVAL;
    if (b < 1 || b > RB_MAX_BATCH || c < 0 || c > b) return RB_EINVAL;
    if (!aligned(batch_x, 16) || !aligned(batch_y, 8)) return RB_EINVAL;
    if (r < 0 || r > RB_MAX_BATCH) return RB_EINVAL;
    if (r > 0 && (!out_x || !out_y || !aligned(out_x, 16) || !aligned(out_y, 8))) return RB_EINVAL;
    if (!rb->bound) return RB_ESTATE;
    return RB_OK;
}

}  // namespace

// The asynchronous form of the single primitive: two events order the training stream and the
// buffer's stream against each other.
struct rb_pipeline {
    rb_buffer* rb;
    hipEvent_t ready;     // on the training stream: mini-batch produced, earlier representatives consumed
    hipEvent_t done;      // on the buffer's stream: the latest step's update and sampling are complete
    int64_t prev_r;       // rows the latest step asked for
    bool started;         // at least one step has been enqueued
};

extern "C" {

int rb_create(rb_buffer** out, int64_t classes, int64_t slots_per_class,
              const int64_t* sample_shape, int32_t ndim, int32_t dtype)
{
    if (!out) return RB_EINVAL;
    *out = nullptr;
    if (!sample_shape || ndim < 1 || ndim > 16) return RB_EINVAL;
    if (classes < 1 || classes > RB_MAX_CLASSES || slots_per_class < 1) return RB_EINVAL;
    if (slots_per_class > RB_MAX_SLOTS / classes) return RB_EINVAL;
    if (dtype != RB_F32 && dtype != RB_BF16) return RB_EINVAL;
    int64_t elems = 1;
    for (int i = 0; i < ndim; ++i) {
        if (sample_shape[i] < 1) return RB_EINVAL;
        if (elems > (INT64_C(1) << 40) / sample_shape[i]) return RB_EINVAL;   // a row of more than 2^40 elements
        elems *= sample_shape[i];
    }
    const int64_t row_bytes = elems * (dtype == RB_F32 ? 4 : 2);
    if (row_bytes % 16 != 0) return RB_EINVAL;
    rb_buffer* rb = new (std::nothrow) rb_buffer();
    if (!rb) return RB_ENOMEM;
    rb->K = classes;
    rb->S = slots_per_class;
    rb->row_bytes = row_bytes;
    rb->row_vec = row_bytes / 16;
    rb->sample_bytes = row_bytes;
    rb->dtype = dtype;
    rb->storage = RB_STORE_SAME;
    rb->nchunks = (int32_t)((classes + CH - 1) / CH);
    rb->buf_x = nullptr; rb->buf_y = nullptr; rb->ws = nullptr; rb->stream = nullptr;
    rb->bound = false;
    rb->static_dev = -1;
    rb->cur = 0;
    size_t off = STATE_BYTES;
    const size_t fill_bytes = round_up((size_t)rb->nchunks * CH * sizeof(int32_t), 256);
    const size_t chunk_bytes = round_up((size_t)rb->nchunks * sizeof(int32_t), 256);
    rb->off_fill[0] = off; off += fill_bytes;
    rb->off_fill[1] = off; off += fill_bytes;
    rb->off_chunk[0] = off; off += chunk_bytes;
    rb->off_chunk[1] = off; off += chunk_bytes;
    rb->off_aux[0] = off; off += fill_bytes;
    rb->off_aux[1] = off; off += fill_bytes;
    rb->off_tbl[0] = off; off += PLAN_BYTES;
    rb->off_tbl[1] = off; off += PLAN_BYTES;
    rb->off_wtbl[0] = off; off += WIN_TABLE_BYTES;
    rb->off_wtbl[1] = off; off += WIN_TABLE_BYTES;
    rb->off_bfwd[0] = off; off += BIG_FWD_BYTES;
    rb->off_bfwd[1] = off; off += BIG_FWD_BYTES;
    rb->off_bwtbl[0] = off; off += BW_TABLE_BYTES;
    rb->off_bwtbl[1] = off; off += BW_TABLE_BYTES;
    rb->bw_number = 0; rb->bw_table_number[0] = 0; rb->bw_table_number[1] = 0;
    rb->ws_bytes = off;
    rb->tbl_next = 0; rb->tbl_planned = 0; rb->plan_valid = false; rb->plan_y = nullptr; rb->next_y = nullptr;
    rb->ann_n = 0; rb->wplan_valid = false; rb->wplan_tbl = 0;
    rb->selection = RB_SELECT_EXACT; rb->eviction = RB_EVICT_UNIFORM; rb->updates = 0;
    rb->opt_unroll = 0; rb->opt_nt = 1; rb->opt_rpb = 0; rb->opt_fuse = 1; rb->opt_window = WIN_MAX; rb->opt_planners = 0;
    *out = rb;
    return RB_OK;
}

int rb_query_sizes(const rb_buffer* rb, size_t* x_bytes, size_t* y_bytes, size_t* workspace_bytes)
{
    if (!rb) return RB_EINVAL;
    if (x_bytes) *x_bytes = (size_t)rb->K * (size_t)rb->S * (size_t)rb->row_bytes;
    if (y_bytes) *y_bytes = (size_t)rb->K * (size_t)rb->S * sizeof(int64_t);
    if (workspace_bytes) *workspace_bytes = rb->ws_bytes;
    return RB_OK;
}

int rb_set_storage(rb_buffer* rb, int32_t storage)
{
    if (!rb) return RB_EINVAL;
    if (storage != RB_STORE_SAME && storage != RB_STORE_BF16 && storage != RB_STORE_U8) return RB_EINVAL;
    if (rb->bound) return RB_ESTATE;                 // the storage the caller bound was sized for the other form
    if (storage == RB_STORE_BF16 && (rb->dtype != RB_F32 || rb->sample_bytes % 32 != 0)) return RB_EINVAL;
    if (storage == RB_STORE_U8 && (rb->dtype != RB_F32 || rb->sample_bytes % 64 != 0)) return RB_EINVAL;
    rb->storage = storage;
    rb->row_bytes = storage == RB_STORE_BF16 ? rb->sample_bytes / 2 : storage == RB_STORE_U8 ? rb->sample_bytes / 4 : rb->sample_bytes;
    rb->row_vec = rb->row_bytes / 16;
    return RB_OK;
}

namespace {
// The handle no longer uses a device's static scratch array.
void release_scratch(rb_buffer* rb)
{
    if (rb->static_dev >= 0 && scratch_holder[rb->static_dev] == rb) scratch_holder[rb->static_dev] = nullptr;
    rb->static_dev = -1;
}
}  // namespace

int rb_bind(rb_buffer* rb, void* buf_x, int64_t* buf_y, void* workspace, void* hip_stream)
{
    if (!rb || !buf_x || !buf_y || !workspace) return RB_EINVAL;
    if (!aligned(buf_x, 16) || !aligned(buf_y, 8) || !aligned(workspace, 256)) return RB_EINVAL;
    if (rb->static_dev >= 0 && workspace != scratch_ptr[rb->static_dev]) release_scratch(rb);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int64_t slots = rb->K * rb->S;
    int64_t blocks = (slots + TPB - 1) / TPB;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    rb_reset_kernel<<<dim3((unsigned)blocks), TPB, 0, st>>>(static_cast<uint32_t*>(workspace),
                                                           (int64_t)(rb->ws_bytes / 4), buf_y, slots);
    if (hipGetLastError() != hipSuccess) return RB_EHIP;
    rb->buf_x = buf_x;
    rb->buf_y = buf_y;
    rb->ws = static_cast<char*>(workspace);
    rb->stream = st;
    rb->cur = 0;
    rb->updates = 0;
    rb->plan_valid = false; rb->next_y = nullptr; rb->tbl_next = 0;
    rb->ann_n = 0; rb->wplan_valid = false;
    rb->bw_number = 0; rb->bw_table_number[0] = 0; rb->bw_table_number[1] = 0;     // (the reset clears the planners' flags)
    rb->bound = true;
    return RB_OK;
}

int rb_bind_static(rb_buffer* rb, void* buf_x, int64_t* buf_y, void* hip_stream)
{
    if (!rb || !buf_x || !buf_y) return RB_EINVAL;
    if (!aligned(buf_x, 16) || !aligned(buf_y, 8)) return RB_EINVAL;
    if (rb->ws_bytes > sizeof scratch) return RB_ELIMIT;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return RB_EHIP;
    if (!scratch_ptr[dev]) {
        // first use on this device (which is current): where this device's copy of the array lives
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RB_EHIP;
        scratch_ptr[dev] = p;
    }
    rb_buffer* before = scratch_holder[dev];
    if (rb->static_dev >= 0 && rb->static_dev != dev) release_scratch(rb);
    rb->static_dev = dev;                          // (rb_bind keeps the array with this handle)
    const int rc = rb_bind(rb, buf_x, buf_y, scratch_ptr[dev], hip_stream);   // clears what the handle uses of the array, on the stream
    if (rc != RB_OK) {
        if (before != rb) rb->static_dev = -1;
        return rc;
    }
    if (before && before != rb) {                  // the array changes hands: the other handle has no workspace any more
        before->bound = false;
        before->static_dev = -1;
    }
    scratch_holder[dev] = rb;
    return RB_OK;
}

int rb_set_stream(rb_buffer* rb, void* hip_stream)
{
    if (!rb) return RB_EINVAL;
    rb->stream = static_cast<hipStream_t>(hip_stream);
    return RB_OK;
}

int rb_set_policy(rb_buffer* rb, int32_t selection, int32_t eviction)
{
    if (!rb) return RB_EINVAL;
    if (selection != RB_SELECT_EXACT && selection != RB_SELECT_BERNOULLI) return RB_EINVAL;
    if (eviction != RB_EVICT_UNIFORM && eviction != RB_EVICT_FIFO && eviction != RB_EVICT_RESERVOIR) return RB_EINVAL;
    if (rb->updates != 0) return RB_ESTATE;      // the per-class state of one strategy means nothing to another
    rb->selection = selection;
    rb->eviction = eviction;
    return RB_OK;
}

int rb_update(rb_buffer* rb, const void* batch_x, const int64_t* batch_y,
              int64_t b, int64_t c, uint64_t seed, uint64_t step)
{
    if (!rb || !batch_x || !batch_y) return RB_EINVAL;
    if (b < 1 || b > RB_MAX_BATCH || c < 0 || c > b) return RB_EINVAL;
    if (!aligned(batch_x, 16) || !aligned(batch_y, 8)) return RB_EINVAL;
    if (!rb->bound) return RB_ESTATE;
    discard_plan(rb);
    if (c == 0) return RB_OK;

    const bool variant = rb->selection != RB_SELECT_EXACT || rb->eviction != RB_EVICT_UNIFORM;
    const int narrow = rb->storage == RB_STORE_BF16 ? 1 : rb->storage == RB_STORE_U8 ? 2 : 0;
    const bool small = c <= WAVE && !variant && !narrow;
    // Rows the grid is sized for.  The Bernoulli selection yields a random number of candidates
    // (mean c, at most b); the movers loop over the work items, so any number is handled, and
    // the grid only has to be large enough for the usual case.
    int64_t rows = c;
    if (rb->selection == RB_SELECT_BERNOULLI) {
        int64_t slack = 16;
        while (slack * slack < 36 * c) ++slack;          // about six standard deviations
        rows = c + slack < b ? c + slack : b;
    }
    const Shape sh = plan_shape(rb, rows, small ? TPB : WAVE, narrow == 2 ? 4 : 8);   // (the 8-bit mover holds at most four vectors per lane)
    UpdateArgs a;
    a.batch_x = static_cast<const vec16*>(batch_x);
    a.batch_y = batch_y;
    a.buf_x = static_cast<vec16*>(rb->buf_x);
    a.buf_y = rb->buf_y;
    a.fill_old = reinterpret_cast<const int32_t*>(rb->ws + rb->off_fill[rb->cur]);
    a.fill_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_fill[rb->cur ^ 1]);
    a.chunk_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_chunk[rb->cur ^ 1]);
    a.state = reinterpret_cast<DevState*>(rb->ws);
    a.sd = make_seed(seed, step);
    a.b = (int32_t)b; a.c = (int32_t)c;
    a.K = (int32_t)rb->K; a.nchunks = rb->nchunks;
    a.S = rb->S;
    a.row_vec = rb->row_vec;
    a.tpr = sh.tpr; a.tile_vec = sh.tile_vec; a.tile_rem = sh.tile_rem; a.rpb = sh.rpb;
    a.selection = rb->selection; a.eviction = rb->eviction;
    a.cap = (int32_t)(rb->selection == RB_SELECT_BERNOULLI ? b : c);
    a.aux_old = reinterpret_cast<const int32_t*>(rb->ws + rb->off_aux[rb->cur]);
    a.aux_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_aux[rb->cur ^ 1]);
    const dim3 grid((unsigned)(rb->nchunks + (small ? sh.groups * sh.tpr : (rows * sh.tpr + NWAVE - 1) / NWAVE)));
    const size_t lds = small ? (size_t)b * 8 : (size_t)b * 4 + (size_t)a.cap * 8;
    hipError_t e = rb->opt_nt ? launch_update<true>(a, small, narrow, sh.unroll, grid, lds, rb->stream)
                              : launch_update<false>(a, small, narrow, sh.unroll, grid, lds, rb->stream);
    if (e != hipSuccess) return RB_EHIP;
    rb->cur ^= 1;
    rb->updates += 1;
    return RB_OK;
}

int rb_sample_augment(rb_buffer* rb, int64_t r, uint64_t seed, uint64_t step, void* out_x, int64_t* out_y)
{
    if (!rb || r < 0 || r > RB_MAX_BATCH) return RB_EINVAL;
    if (r > 0 && (!out_x || !out_y || !aligned(out_x, 16) || !aligned(out_y, 8))) return RB_EINVAL;
    if (!rb->bound) return RB_ESTATE;
    discard_plan(rb);
    if (r == 0) return RB_OK;

    const int widen = rb->storage == RB_STORE_BF16 ? 1 : rb->storage == RB_STORE_U8 ? 2 : 0;
    const bool small = r <= WAVE && rb->nchunks <= WAVE && !widen;
    const Shape sh = plan_shape(rb, r, small ? TPB : WAVE, widen == 2 ? 4 : 8);
    SampleArgs a;
    a.buf_x = static_cast<const vec16*>(rb->buf_x);
    a.out_x = static_cast<vec16*>(out_x);
    a.out_y = out_y;
    a.fill = reinterpret_cast<const int32_t*>(rb->ws + rb->off_fill[rb->cur]);
    a.chunk = reinterpret_cast<const int32_t*>(rb->ws + rb->off_chunk[rb->cur]);
    a.state = reinterpret_cast<DevState*>(rb->ws);
    a.sd = make_seed(seed, step);
    a.r = (int32_t)r;
    a.K = (int32_t)rb->K; a.nchunks = rb->nchunks;
    a.S = rb->S;
    a.row_vec = rb->row_vec;
    a.tpr = sh.tpr; a.tile_vec = sh.tile_vec; a.tile_rem = sh.tile_rem; a.rpb = sh.rpb;
    const dim3 grid((unsigned)(small ? sh.groups * sh.tpr : (r * sh.tpr + NWAVE - 1) / NWAVE));
    const size_t lds = small ? 0 : ((size_t)rb->nchunks + (size_t)r) * 4;
    hipError_t e = rb->opt_nt ? launch_sample<true>(a, small, widen, sh.unroll, grid, lds, rb->stream)
                              : launch_sample<false>(a, small, widen, sh.unroll, grid, lds, rb->stream);
    return e == hipSuccess ? RB_OK : RB_EHIP;
}

int rb_update_sample(rb_buffer* rb, const void* batch_x, const int64_t* batch_y, int64_t b, int64_t c,
                     int64_t r, uint64_t seed, uint64_t step, void* out_x, int64_t* out_y)
{
    const int bad = check_step(rb, batch_x, batch_y, b, c, r, out_x, out_y);
    if (bad != RB_OK) return bad;
    discard_window_plan(rb);                     // a single step is not what a planned window was made for
    rb->ann_n = 0;

    // the plan-ahead form covers both storage forms; the kernel that plans and moves in one launch only the plain one
    const bool plannable = c >= 1 && c <= WAVE && r >= 1 && r <= WAVE && rb->nchunks <= DIRECT_CHUNKS && rb->opt_fuse &&
                           rb->selection == RB_SELECT_EXACT;
    const bool fused = plannable && rb->storage == RB_STORE_SAME && rb->eviction == RB_EVICT_UNIFORM;
    // larger counts have a plan-ahead form of their own
    // (with the Bernoulli selection, whose number of candidates is only bounded by b, for mini-batches of at most BIG_MAX)
    const bool big = !plannable && c >= 1 && c <= BIG_MAX && r >= 1 && r <= BIG_MAX && b <= BIG_BATCH &&
                     rb->K <= BIG_CLASSES && rb->opt_fuse && (rb->selection == RB_SELECT_EXACT || b <= BIG_MAX) &&
                     rb->K * rb->S <= INT64_C(0x7FFFFFFF) && rb->S <= INT32_MAX - RB_MAX_BATCH;
    const int64_t* next_y = rb->next_y;
    rb->next_y = nullptr;                        // an announcement serves one call
    if (rb->plan_valid && !((plannable || big) && rb->plan_y == batch_y && rb->plan_b == b && rb->plan_c == c && rb->plan_r == r &&
                            rb->plan_seed == seed && rb->plan_step == step))
        discard_plan(rb);
    if (plannable && (rb->plan_valid || next_y))
        return step_planned(rb, batch_x, batch_y, b, c, r, seed, step, out_x, out_y, next_y);
    if (big && (rb->plan_valid || next_y))
        return step_big(rb, batch_x, batch_y, b, c, r, seed, step, out_x, out_y, next_y);
    if (!fused) {
        const int rc = rb_update(rb, batch_x, batch_y, b, c, seed, step);
        if (rc != RB_OK) return rc;
        return rb_sample_augment(rb, r, seed, step, out_x, out_y);
    }
    const Shape sh = plan_shape(rb, c + r, TPB);
    StepArgs sa;
    UpdateArgs& a = sa.u;
    a.batch_x = static_cast<const vec16*>(batch_x);
    a.batch_y = batch_y;
    a.buf_x = static_cast<vec16*>(rb->buf_x);
    a.buf_y = rb->buf_y;
    a.fill_old = reinterpret_cast<const int32_t*>(rb->ws + rb->off_fill[rb->cur]);
    a.fill_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_fill[rb->cur ^ 1]);
    a.chunk_new = reinterpret_cast<int32_t*>(rb->ws + rb->off_chunk[rb->cur ^ 1]);
    a.state = reinterpret_cast<DevState*>(rb->ws);
    a.sd = make_seed(seed, step);
    a.b = (int32_t)b; a.c = (int32_t)c;
    a.K = (int32_t)rb->K; a.nchunks = rb->nchunks;
    a.S = rb->S;
    a.row_vec = rb->row_vec;
    a.tpr = sh.tpr; a.tile_vec = sh.tile_vec; a.tile_rem = sh.tile_rem; a.rpb = 1;
    a.selection = RB_SELECT_EXACT; a.eviction = RB_EVICT_UNIFORM; a.cap = (int32_t)c;
    a.aux_old = nullptr; a.aux_new = nullptr;
    sa.out_x = static_cast<vec16*>(out_x);
    sa.out_y = out_y;
    sa.r = (int32_t)r;
    sa.first_gather = (int32_t)(rb->nchunks + c * sh.tpr);
    const dim3 grid((unsigned)(rb->nchunks + (c + r) * sh.tpr));
    const size_t lds = (((size_t)b * 2 + 3) & ~(size_t)3) * 4 + (size_t)DIRECT_CHUNKS * CH * 8;
    hipError_t e = rb->opt_nt ? launch_step<true>(sa, sh.unroll, grid, lds, rb->stream)
                              : launch_step<false>(sa, sh.unroll, grid, lds, rb->stream);
    if (e != hipSuccess) return RB_EHIP;
    rb->cur ^= 1;
    rb->updates += 1;
    return RB_OK;
}

int rb_announce_next(rb_buffer* rb, const int64_t* next_batch_y)
{
    if (!rb) return RB_EINVAL;
    if (next_batch_y && !aligned(next_batch_y, 8)) return RB_EINVAL;
    rb->next_y = next_batch_y;
    return RB_OK;
}

int rb_query_steps_per_launch(const rb_buffer* rb, int64_t b, int64_t c, int64_t r, int64_t* steps)
{
    if (!rb || !steps) return RB_EINVAL;
    if (b < 1 || b > RB_MAX_BATCH || c < 0 || c > b || r < 0 || r > RB_MAX_BATCH) return RB_EINVAL;
    (void)many_form(rb, b, c, r, *steps);
    return RB_OK;
}

int rb_announce_next_many(rb_buffer* rb, int64_t n, const int64_t* const* next_batch_y)
{
    if (!rb || n < 0 || (n > 0 && !next_batch_y)) return RB_EINVAL;
    const int64_t keep = std::min<int64_t>(n, WIN_MAX);        // more than one launch can cover is of no use
    for (int64_t i = 0; i < keep; ++i)
        if (!next_batch_y[i] || !aligned(next_batch_y[i], 8)) return RB_EINVAL;
    for (int64_t i = 0; i < keep; ++i) rb->ann_y[i] = next_batch_y[i];
    rb->ann_n = keep;
    return RB_OK;
}

int rb_update_sample_many(rb_buffer* rb, int64_t n, const void* const* batch_x, const int64_t* const* batch_y,
                          int64_t b, int64_t c, int64_t r, uint64_t seed, uint64_t first_step,
                          void* const* out_x, int64_t* const* out_y)
{
    if (!rb || n < 0 || !batch_x || !batch_y) return RB_EINVAL;
    if (r > 0 && (!out_x || !out_y)) return RB_EINVAL;
    // what was announced is about the call after this one and serves this call only
    const int64_t ann_n = rb->ann_n;
    const int64_t* ann_y[WIN_MAX];
    for (int64_t i = 0; i < ann_n; ++i) ann_y[i] = rb->ann_y[i];
    rb->ann_n = 0;
    for (int64_t i = 0; i < n; ++i) {
        const int bad = check_step(rb, batch_x[i], batch_y[i], b, c, r, r > 0 ? out_x[i] : nullptr, r > 0 ? out_y[i] : nullptr);
        if (bad != RB_OK) return bad;
    }
    int64_t per_launch;
    const int form = n >= 2 ? many_form(rb, b, c, r, per_launch) : MANY_SINGLE;
    if (form != MANY_SINGLE) {
        if (rb->plan_valid) {                    // a single step that was planned ahead is not executed as planned
            rb->cur ^= 1;
            rb->plan_valid = false;
        }
        rb->next_y = nullptr;
        return form == MANY_SMALL ? steps_windowed(rb, n, batch_x, batch_y, b, c, r, seed, first_step, out_x, out_y, ann_n, ann_y)
                                  : steps_bigwin(rb, n, batch_x, batch_y, b, c, r, seed, first_step, out_x, out_y, ann_n, ann_y);
    }
    discard_window_plan(rb);
    for (int64_t i = 0; i < n; ++i) {
        // the next step's labels are known: plan ahead (also across calls when the next call's first labels were announced)
        rb->next_y = i + 1 < n ? batch_y[i + 1] : (ann_n > 0 ? ann_y[0] : nullptr);
        const int rc = rb_update_sample(rb, batch_x[i], batch_y[i], b, c, r, seed, first_step + (uint64_t)i,
                                        r > 0 ? out_x[i] : nullptr, r > 0 ? out_y[i] : nullptr);
        if (rc != RB_OK) return rc;      // only a failed launch can get here
    }
    return RB_OK;
}

int rb_pipeline_create(rb_pipeline** out, rb_buffer* rb)
{
    if (!out) return RB_EINVAL;
    *out = nullptr;
    if (!rb) return RB_EINVAL;
    rb_pipeline* p = new (std::nothrow) rb_pipeline();
    if (!p) return RB_ENOMEM;
    p->rb = rb;
    p->prev_r = 0;
    p->started = false;
    if (hipEventCreateWithFlags(&p->ready, hipEventDisableTiming) != hipSuccess) {
        delete p;
        return RB_EHIP;
    }
    if (hipEventCreateWithFlags(&p->done, hipEventDisableTiming) != hipSuccess) {
        (void)hipEventDestroy(p->ready);
        delete p;
        return RB_EHIP;
    }
    *out = p;
    return RB_OK;
}

int rb_pipeline_step(rb_pipeline* p, const void* batch_x, const int64_t* batch_y, int64_t b, int64_t c,
                     int64_t r, uint64_t seed, uint64_t step, void* next_x, int64_t* next_y,
                     void* train_stream, int64_t* ready_rows)
{
    if (!p) return RB_EINVAL;
    rb_buffer* rb = p->rb;
    const int bad = check_step(rb, batch_x, batch_y, b, c, r, next_x, next_y);
    if (bad != RB_OK) return bad;
    hipStream_t train = static_cast<hipStream_t>(train_stream);
    const bool two_streams = train != rb->stream;
    if (two_streams) {
        // (1) the training stream may go on once the previous step's representatives are complete
        if (p->started && hipStreamWaitEvent(train, p->done, 0) != hipSuccess) return RB_EHIP;
        // the buffer's stream starts this step once the training stream has got this far
        if (hipEventRecord(p->ready, train) != hipSuccess) return RB_EHIP;
        if (hipStreamWaitEvent(rb->stream, p->ready, 0) != hipSuccess) return RB_EHIP;
    }
    // (2) update with this mini-batch, then collect the next representatives
    const int rc = rb_update_sample(rb, batch_x, batch_y, b, c, r, seed, step, next_x, next_y);
    if (rc != RB_OK) return rc;
    if (two_streams && hipEventRecord(p->done, rb->stream) != hipSuccess) return RB_EHIP;
    if (ready_rows) *ready_rows = p->started ? p->prev_r : 0;
    p->prev_r = r;
    p->started = true;
    return RB_OK;
}

int rb_pipeline_drain(rb_pipeline* p, void* train_stream, int64_t* ready_rows)
{
    if (!p) return RB_EINVAL;
    hipStream_t train = static_cast<hipStream_t>(train_stream);
    if (p->started && train != p->rb->stream && hipStreamWaitEvent(train, p->done, 0) != hipSuccess) return RB_EHIP;
    if (ready_rows) *ready_rows = p->started ? p->prev_r : 0;
    return RB_OK;
}

int rb_pipeline_step_many(rb_pipeline* p, int64_t n, const void* const* batch_x, const int64_t* const* batch_y,
                          int64_t b, int64_t c, int64_t r, uint64_t seed, uint64_t first_step,
                          void* const* next_x, int64_t* const* next_y, void* train_stream, int64_t* ready_rows)
{
    if (!p || n < 0 || !batch_x || !batch_y) return RB_EINVAL;
    if (r > 0 && (!next_x || !next_y)) return RB_EINVAL;
    rb_buffer* rb = p->rb;
    // everything is checked before the first stream operation, so that an error leaves nothing behind
    for (int64_t i = 0; i < n; ++i) {
        const int bad = check_step(rb, batch_x[i], batch_y[i], b, c, r, r > 0 ? next_x[i] : nullptr, r > 0 ? next_y[i] : nullptr);
        if (bad != RB_OK) return bad;
    }
    if (n == 0) {
        if (ready_rows) *ready_rows = p->started ? p->prev_r : 0;
        return RB_OK;
    }
    hipStream_t train = static_cast<hipStream_t>(train_stream);
    const bool two_streams = train != rb->stream;
    if (two_streams) {
        // (1) the training stream may go on once the previous call's representatives are complete
        if (p->started && hipStreamWaitEvent(train, p->done, 0) != hipSuccess) return RB_EHIP;
        // the buffer's stream starts these steps once the training stream has got this far
        if (hipEventRecord(p->ready, train) != hipSuccess) return RB_EHIP;
        if (hipStreamWaitEvent(rb->stream, p->ready, 0) != hipSuccess) return RB_EHIP;
    }
    // (2) the n updates, each followed by the collection of the next representatives
    const int rc = rb_update_sample_many(rb, n, batch_x, batch_y, b, c, r, seed, first_step, next_x, next_y);
    if (rc != RB_OK) return rc;
    if (two_streams && hipEventRecord(p->done, rb->stream) != hipSuccess) return RB_EHIP;
    if (ready_rows) *ready_rows = p->started ? p->prev_r : 0;
    p->prev_r = r;
    p->started = true;
    return RB_OK;
}

int rb_pipeline_destroy(rb_pipeline* p)
{
    if (!p) return RB_EINVAL;
    const bool ok = hipEventDestroy(p->ready) == hipSuccess;
    const bool ok2 = hipEventDestroy(p->done) == hipSuccess;
    delete p;
    return ok && ok2 ? RB_OK : RB_EHIP;
}

int rb_read_state(rb_buffer* rb, int32_t* fill_host, int64_t* last_n_host, uint32_t* flags_host)
{
    if (!rb) return RB_EINVAL;
    if (!rb->bound) return RB_ESTATE;
    discard_plan(rb);
    if (hipStreamSynchronize(rb->stream) != hipSuccess) return RB_EHIP;
    DevState st;
    if (hipMemcpy(&st, rb->ws, sizeof st, hipMemcpyDeviceToHost) != hipSuccess) return RB_EHIP;
    if (fill_host &&
        hipMemcpy(fill_host, rb->ws + rb->off_fill[rb->cur], (size_t)rb->K * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
        return RB_EHIP;
    if (last_n_host) *last_n_host = st.last_n;
    if (flags_host) *flags_host = st.flags;
    return RB_OK;
}

int rb_read_moved_rows(rb_buffer* rb, uint64_t* rows_host)
{
    if (!rb || !rows_host) return RB_EINVAL;
    if (!rb->bound) return RB_ESTATE;
    discard_plan(rb);
    if (hipStreamSynchronize(rb->stream) != hipSuccess) return RB_EHIP;
    static_assert(MOVED_STRIDE % sizeof(uint64_t) == 0, "counters are read as an array of 64-bit words");
    uint64_t words[MOVED_COUNTERS * MOVED_STRIDE / sizeof(uint64_t)];
    if (hipMemcpy(words, rb->ws + STATE_HEAD_BYTES, sizeof words, hipMemcpyDeviceToHost) != hipSuccess) return RB_EHIP;
    uint64_t sum = 0;
    for (int i = 0; i < MOVED_COUNTERS; ++i) sum += words[i * (MOVED_STRIDE / sizeof(uint64_t))];
    *rows_host = sum;
    return RB_OK;
}

int rb_set_option(rb_buffer* rb, int32_t option, int64_t value)
{
    if (!rb) return RB_EINVAL;
    switch (option) {
    case RB_OPT_UNROLL:
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return RB_EINVAL;
        rb->opt_unroll = (int)value;
        return RB_OK;
    case RB_OPT_NONTEMPORAL:
        if (value != 0 && value != 1) return RB_EINVAL;
        rb->opt_nt = (int)value;
        return RB_OK;
    case RB_OPT_ROWS_PER_BLOCK:
        if (value < 0 || value > 16) return RB_EINVAL;
        rb->opt_rpb = (int)value;
        return RB_OK;
    case RB_OPT_FUSE:
        if (value != 0 && value != 1) return RB_EINVAL;
        rb->opt_fuse = (int)value;
        return RB_OK;
    case RB_OPT_WINDOW:
        if (value < 1 || value > WIN_MAX) return RB_EINVAL;
        rb->opt_window = (int)value;
        return RB_OK;
    case RB_OPT_PLANNERS:
        if (value < 0 || value > 2) return RB_EINVAL;
        rb->opt_planners = (int)value;
        return RB_OK;
    default:
        return RB_EINVAL;
    }
}

int rb_destroy(rb_buffer* rb)
{
    if (rb) release_scratch(rb);
    delete rb;
    return RB_OK;
}

const char* rb_strerror(int status)
{
    switch (status) {
    case RB_OK: return "ok";
    case RB_EINVAL: return "invalid argument";
    case RB_ENOMEM: return "out of host memory";
    case RB_ESTATE: return "buffer is not bound to device storage";
    case RB_EHIP: return "a HIP call failed";
    case RB_ELIMIT: return "the buffer needs more workspace than the library's static scratch array holds";
    default: return "unknown status";
    }
}

int rb_standin_compute(void* hip_stream, float* sink, int64_t blocks, int64_t iters)
{
    if (!sink || blocks < 1 || blocks > (1 << 20) || iters < 0) return RB_EINVAL;
    rb_standin_kernel<<<dim3((unsigned)blocks), TPB, 0, static_cast<hipStream_t>(hip_stream)>>>(sink, iters);
    return hipGetLastError() == hipSuccess ? RB_OK : RB_EHIP;
}

int rb_copy_bytes(void* hip_stream, void* dst, const void* src, size_t bytes, int32_t unroll, int32_t nontemporal)
{
    if (!dst || !src || bytes == 0 || bytes % 16 != 0 || !aligned(dst, 16) || !aligned(src, 16)) return RB_EINVAL;
    if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8) return RB_EINVAL;
    const int64_t nvec = (int64_t)(bytes / 16);
    if ((nvec + (int64_t)TPB * unroll - 1) / ((int64_t)TPB * unroll) > 0x7FFFFFFF) return RB_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    vec16* d = static_cast<vec16*>(dst);
    const vec16* s = static_cast<const vec16*>(src);
    hipError_t e = nontemporal == 2 ? launch_copy<true, 64>(d, s, nvec, unroll, st)
                 : nontemporal      ? launch_copy<true, 1>(d, s, nvec, unroll, st)
                                    : launch_copy<false, 1>(d, s, nvec, unroll, st);
    return e == hipSuccess ? RB_OK : RB_EHIP;
}

}  // extern "C"
