// Rehearsal-buffer hot path for gfx950 (MI355X): kernels and the C ABI of include/rb.h.
//
// One kernel launch per hot call.  Every workgroup first re-derives, in LDS,
// the few integers of the step's plan it needs (which mini-batch positions are
// candidates, which slot a candidate goes to, which stored sample a
// representative is) and then moves its share of one sample row with 16-byte
// vector loads and stores.  The plan is O(b + K) integers while a row is
// hundreds of kilobytes, so recomputing it per workgroup is cheaper than a
// second, dependent launch.  Nothing is staged through LDS: a row is read once
// and written once, so the data path is global -> registers -> global.
//
// Per-class fill counts are kept twice (ping-pong): an update reads the "old"
// copy everywhere and a few bookkeeping workgroups write the "new" one, so no
// workgroup can observe a count another workgroup of the same launch changed.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <new>

#include "rb.h"

namespace {

constexpr int TPB = 256;               // threads per workgroup: four 64-wide wavefronts
constexpr int WAVE = 64;
constexpr int NWAVE = TPB / WAVE;
constexpr int CH = 256;                // classes per chunk of the two-level fill index
constexpr int TILE_UNIT = 64;          // granularity, in 16-byte vectors, at which a row is cut into tiles
constexpr uint32_t PURPOSE_SELECT = 1; // counter word that separates the three kinds of draws
constexpr uint32_t PURPOSE_EVICT = 2;
constexpr uint32_t PURPOSE_SAMPLE = 3;
constexpr uint32_t PURPOSE_COIN = 4;   // per-sample coin of the Bernoulli selection
constexpr int32_t LAB_UNSELECTED = -2; // LDS label table: position is not a candidate
constexpr int32_t LAB_INVALID = -1;    // candidate whose label is outside [0, K)

typedef uint32_t vec16 __attribute__((ext_vector_type(4)));   // one 16-byte transfer

// Device-resident state words at the start of the workspace.
struct DevState {
    uint32_t flags;
    uint32_t pad;
    int64_t last_n;
};
constexpr size_t STATE_BYTES = 256;

struct Seed {
    uint32_t seed_lo, seed_hi, step_lo, step_hi;
};

// ---------------------------------------------------------------------------
// Counter-based random draws: Philox4x32-10 (Salmon et al., SC'11).  Counter =
// (index, purpose, step), key = seed; the low two output words form one 64-bit
// draw.  An integer in [0, n) is the high half of draw * n.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint64_t draw64(const Seed& sd, uint32_t purpose, uint32_t index)
{
    uint32_t x0 = index, x1 = purpose, x2 = sd.step_lo, x3 = sd.step_hi;
    uint32_t ka = sd.seed_lo, kb = sd.seed_hi;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        // one 32x32->64 multiply per word pair (v_mad_u64_u32) instead of separate high and low halves
        const uint64_t pa = (uint64_t)0xD2511F53u * x0;
        const uint64_t pb = (uint64_t)0xCD9E8D57u * x2;
        x0 = (uint32_t)(pb >> 32) ^ x1 ^ ka;
        x2 = (uint32_t)(pa >> 32) ^ x3 ^ kb;
        x1 = (uint32_t)pb;
        x3 = (uint32_t)pa;
        ka += 0x9E3779B9u;
        kb += 0xBB67AE85u;
    }
    return (uint64_t)x0 | ((uint64_t)x1 << 32);
}

__device__ __forceinline__ uint64_t below(const Seed& sd, uint32_t purpose, uint32_t index, uint64_t n)
{
    return __umul64hi(draw64(sd, purpose, index), n);
}

// ---------------------------------------------------------------------------
// Wavefront-level pieces of the small-count kernels (at most WAVE candidates or
// representatives: one lane per item, all 64 lanes of the wavefront active).
// ---------------------------------------------------------------------------
// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (no LDS round
// trips): Hillis-Steele steps of 1, 2, 4, 8 lanes inside each row of 16 lanes, then the last
// lane of row 0 / row 2 is added to row 1 / row 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ int wave_scan_incl(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// Value of `v` in lane `src`, the same lane for the whole wavefront.
__device__ __forceinline__ int lane_read(int v, int src)
{
    return __builtin_amdgcn_readlane(v, src);
}

// ---------------------------------------------------------------------------
// Workgroup-wide exclusive prefix sum of one int per thread.  s_wave: NWAVE
// ints of LDS.  Must be called by all threads of the workgroup.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int block_scan_excl(int v, int& total, int* s_wave)
{
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    const int inc = wave_scan_incl(v);
    if (lane == WAVE - 1) s_wave[w] = inc;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < NWAVE; ++i) {
        int x = s_wave[i];
        all += x;
        if (i < w) before += x;
    }
    __syncthreads();
    total = all;
    return before + inc - v;
}

// ---------------------------------------------------------------------------
// Row mover: one tile of one row, U vectors per thread in flight.
// ---------------------------------------------------------------------------
template <int U, bool NT, int W = TPB, bool PACED = true>   // W: threads that share the tile (a workgroup or one wavefront)
struct Tile {
    vec16 v[U];

    // Requires lo < hi.  No lane is ever masked off: a lane whose index falls past the end of
    // the tile moves the tile's last vector again (same source, same destination, same bytes as
    // the lane that owns it), so the copy stays correct and branch-free.  That keeps the number
    // of loads in flight known at compile time - a wait for an earlier load then does not have
    // to drain these - and keeps the compiler from moving loads down into a guarded store.
    __device__ __forceinline__ void load(const vec16* __restrict__ src, int64_t lo, int64_t hi)
    {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t i = lo + (int64_t)u * W + (threadIdx.x & (W - 1));
            i = i < hi ? i : hi - 1;
            v[u] = NT ? __builtin_nontemporal_load(src + i) : src[i];
        }
    }
    // All loads are waited for first and every store is waited for before the next one is
    // issued.  Measured on MI355X with a bare mover of the same shape (64 rows of 301 056 bytes,
    // U = 4): 7.6 us against 8.6 us when each store is issued as soon as its load has arrived
    // and 8.9 us with the guarded form; the memory system does better with few writes in flight.
    __device__ __forceinline__ void store(vec16* __restrict__ dst, int64_t lo, int64_t hi) const
    {
        if (PACED) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t i = lo + (int64_t)u * W + (threadIdx.x & (W - 1));
            i = i < hi ? i : hi - 1;
            if (NT) __builtin_nontemporal_store(v[u], dst + i);
            else dst[i] = v[u];
            if (PACED) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    }
};

// Vector range [lo, hi) of tile `tile` of a row of row_vec vectors.  The row is cut into units of
// TILE_UNIT vectors (1 KiB: what one wavefront moves per instruction, so that a wavefront's access
// does not straddle two such blocks of a 1 KiB-aligned row) and the units are dealt evenly: the
// first `rem` tiles get `units + 1`, the others `units` (>= 1).  Tiles are never empty and never
// longer than W * U vectors for the tile width W the host planned for.
__device__ __forceinline__ void tile_bounds(int tile, int units, int rem, int64_t row_vec, int64_t& lo, int64_t& hi)
{
    const int64_t ulo = (int64_t)tile * units + (tile < rem ? tile : rem);
    const int64_t uhi = ulo + units + (tile < rem ? 1 : 0);
    lo = ulo * TILE_UNIT;
    hi = uhi * TILE_UNIT < row_vec ? uhi * TILE_UNIT : row_vec;
}

// ---------------------------------------------------------------------------
// Reset: fill counts, partial sums and state words to zero, labels to -1.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(TPB) rb_reset_kernel(uint32_t* __restrict__ ws, int64_t ws_words,
                                                        int64_t* __restrict__ buf_y, int64_t slots)
{
    const int64_t stride = (int64_t)gridDim.x * TPB;
    const int64_t first = (int64_t)blockIdx.x * TPB + threadIdx.x;
    for (int64_t i = first; i < ws_words; i += stride) ws[i] = 0u;
    for (int64_t i = first; i < slots; i += stride) buf_y[i] = -1;
}

// ---------------------------------------------------------------------------
// rb_update: Algorithm 1, any c (used for c > WAVE).
//
// The whole workgroup first computes, once, what every candidate is (its
// mini-batch position and class) into LDS; then each of its four wavefronts
// takes one work item (candidate row, tile of WAVE * U vectors) and works out
// alone, with ballots over the candidate list, where that candidate goes.
//
// LDS (dynamic): s_first[b] u32 (lowest candidate index that drew a value),
// s_k[c] i32 (class per candidate, LAB_INVALID outside [0, K)), s_t[c] u16
// (Floyd draws), s_x[c] u16 (candidate positions in Floyd emission order).
//
// Grid: `nchunks` bookkeeping workgroups (new fill counts and chunk sums for CH
// classes each), then ceil(c * tpr / NWAVE) mover workgroups.
// ---------------------------------------------------------------------------
struct UpdateArgs {
    const vec16* batch_x;
    const int64_t* batch_y;
    vec16* buf_x;
    int64_t* buf_y;
    const int32_t* fill_old;
    int32_t* fill_new;
    int32_t* chunk_new;
    DevState* state;
    Seed sd;
    int32_t b, c;
    int32_t K, nchunks;
    int64_t S;
    int64_t row_vec;      // 16-byte vectors per row
    int32_t tpr;          // tiles per row
    int32_t tile_vec;     // a row is split evenly into tpr tiles in units of TILE_UNIT vectors: the first
    int32_t tile_rem;     // tile_rem tiles hold tile_vec + 1 units, the others tile_vec; see tile_bounds
    int32_t rpb;          // small kernels: rows per mover workgroup (1 unless tpr == 1)
    // policy variants (general kernel only)
    int32_t selection;    // RB_SELECT_*
    int32_t eviction;     // RB_EVICT_*
    int32_t cap;          // most candidates a step can have: c (exact selection) or b (Bernoulli)
    const int32_t* aux_old;   // per class: FIFO: slot of the oldest sample; RESERVOIR: samples offered so far
    int32_t* aux_new;
};

template <int U, bool NT>
__global__ void __launch_bounds__(TPB) rb_update_kernel(const UpdateArgs a)
{
    extern __shared__ uint32_t lds[];
    uint32_t* s_first = lds;                                          // [b]
    int32_t* s_k = reinterpret_cast<int32_t*>(lds + a.b);             // [cap]
    uint16_t* s_t = reinterpret_cast<uint16_t*>(lds + a.b + a.cap);   // [cap]
    uint16_t* s_x = s_t + a.cap;                                      // [cap]
    __shared__ int s_wave[NWAVE];
    __shared__ int s_hist[CH];
    __shared__ uint16_t s_pend[NWAVE][2 * WAVE];    // per wavefront: later class-mates waiting for their evict draw
    __shared__ uint32_t s_cm[NWAVE][RB_MAX_BATCH / 32];     // per wavefront: bitmap of the class-mates' positions
    __shared__ uint16_t s_cmpre[NWAVE][RB_MAX_BATCH / 32];  // class-mates before each bitmap word

    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int b = a.b, c = a.c;
    int m;      // number of candidates of this step (the same in every workgroup)

    if (a.selection == RB_SELECT_BERNOULLI) {
        // ---- one coin per sample, heads with probability c/b; candidates in mini-batch order ----
        const int per = (b + TPB - 1) / TPB;
        const int q_lo = tid * per;
        int mine = 0;
        for (int u = 0; u < per; ++u) {
            const int q = q_lo + u;
            if (q < b && (int64_t)below(a.sd, PURPOSE_COIN, (uint32_t)q, (uint64_t)b) < c) {
                s_first[q] = 1u;
                ++mine;
            } else if (q < b) {
                s_first[q] = 0u;
            }
        }
        int at = block_scan_excl(mine, m, s_wave);
        for (int u = 0; u < per; ++u) {
            const int q = q_lo + u;
            if (q < b && s_first[q] != 0u) {
                s_x[at] = (uint16_t)q;
                const int64_t y = a.batch_y[q];
                s_k[at] = (y >= 0 && y < a.K) ? (int32_t)y : LAB_INVALID;
                ++at;
            }
        }
        __syncthreads();
    } else {
        // ---- candidate selection: Floyd's c-subset of [0, b), all draws at once --
        // Draw i is t_i in [0, b-c+i]; it is "taken" iff an earlier draw had the same
        // value, or it equals b-c+q for an earlier q whose own draw was taken; a
        // taken draw is replaced by b-c+i.
        m = c;
        for (int q = tid; q < b; q += TPB) s_first[q] = 0xFFFFFFFFu;
        __syncthreads();
        const int base = b - c;
        for (int i = tid; i < c; i += TPB) {
            uint32_t t = (uint32_t)below(a.sd, PURPOSE_SELECT, (uint32_t)i, (uint64_t)(base + i + 1));
            s_t[i] = (uint16_t)t;
            atomicMin(&s_first[t], (uint32_t)i);
        }
        __syncthreads();
        for (int i = tid; i < c; i += TPB) {
            int cur = i;
            bool taken = false;
            for (;;) {
                int t = s_t[cur];
                if (s_first[t] != (uint32_t)cur) { taken = true; break; }   // an earlier draw had this value
                int q = t - base;                                           // the step whose fallback value is t
                if (q < 0 || q >= cur) break;
                cur = q;                                                    // taken iff that step fell back
            }
            int x = taken ? base + i : (int)s_t[i];
            s_x[i] = (uint16_t)x;
            int64_t y = a.batch_y[x];
            s_k[i] = (y >= 0 && y < a.K) ? (int32_t)y : LAB_INVALID;
        }
        __syncthreads();
    }

    if ((int)blockIdx.x < a.nchunks) {
        // ---- bookkeeping: fill_new = min(fill_old + candidates of the class, S) ----
        const int k_lo = blockIdx.x * CH;
        s_hist[tid] = 0;
        __syncthreads();
        bool bad = false;
        for (int i = tid; i < m; i += TPB) {
            const int32_t k = s_k[i];
            if (k >= k_lo && k < k_lo + CH) atomicAdd(&s_hist[k - k_lo], 1);
            bad |= (k == LAB_INVALID);
        }
        __syncthreads();
        const int k = k_lo + tid;
        int32_t nf = 0;
        if (k < a.K) {
            const int64_t old = a.fill_old[k];
            const int64_t v = old + s_hist[tid];
            nf = (int32_t)(v < a.S ? v : a.S);
            a.fill_new[k] = nf;
            if (a.eviction == RB_EVICT_FIFO) {
                // the oldest sample moves on by the number of overwrites
                const int64_t over = v > a.S ? v - a.S : 0;
                a.aux_new[k] = (int32_t)(((int64_t)a.aux_old[k] + over) % a.S);
            } else if (a.eviction == RB_EVICT_RESERVOIR) {
                const int64_t seen = (int64_t)a.aux_old[k] + s_hist[tid];
                a.aux_new[k] = (int32_t)(seen < INT32_MAX ? seen : INT32_MAX);
            }
        }
        int total;
        block_scan_excl(nf, total, s_wave);
        if (tid == 0) a.chunk_new[blockIdx.x] = total;
        if (blockIdx.x == 0 && bad) atomicOr(&a.state->flags, RB_FLAG_BAD_LABEL);
        return;
    }

    // ---- movers: one work item per wavefront and round, no workgroup barrier from here on ----
    const int64_t stride = (int64_t)(gridDim.x - a.nchunks) * NWAVE;
    for (int64_t item = (int64_t)(blockIdx.x - a.nchunks) * NWAVE + wave; item < (int64_t)m * a.tpr; item += stride) {
        const int i = (int)(item / a.tpr), tile = (int)(item % a.tpr);   // candidate, tile of its row
        const int p = s_x[i];                                             // its mini-batch position
        const int32_t ki = s_k[i];
        if (ki < 0) continue;                  // label outside [0, K): dropped (flagged by bookkeeping)
        int64_t v_lo, v_hi;
        tile_bounds(tile, a.tile_vec, a.tile_rem, a.row_vec, v_lo, v_hi);

        const int64_t fill0 = a.fill_old[ki];
        const int64_t aux0 = a.eviction != RB_EVICT_UNIFORM ? a.aux_old[ki] : 0;
        // the row is read while the wavefront works out where it goes
        Tile<U, NT, WAVE, false> t;
        t.load(a.batch_x + (int64_t)p * a.row_vec, v_lo, v_hi);

        // Candidates of class ki, in mini-batch order: the one with `rank` class-mates before it is
        // insertion number fill0 + rank of the class.
        int total = 0, rank = 0;
        for (int m0 = 0; m0 < m; m0 += WAVE) {
            const int q = m0 + lane;
            const bool same = q < m && s_k[q] == ki;
            const int xq = q < m ? s_x[q] : 0;
            total += __popcll(__ballot(same));
            rank += __popcll(__ballot(same && xq < p));
        }
        int64_t slot;
        if (fill0 + total <= a.S) {
            slot = fill0 + rank;               // all of them append: distinct slots
        } else if (a.eviction == RB_EVICT_FIFO) {
            // insertion number fill0 + rank overwrites the oldest sample once the class is full; it is
            // itself overwritten in this step if a class-mate comes a whole round of S later
            const int64_t at = fill0 + rank;
            if (at + a.S < fill0 + total) continue;
            slot = at < a.S ? at : (aux0 + at - a.S) % a.S;
        } else {
            const bool reservoir = a.eviction == RB_EVICT_RESERVOIR;
            // Insertions beyond the capacity overwrite a uniformly drawn slot (or, with reservoir
            // sampling, are kept with probability S / offers).  This candidate is not stored if a
            // later class-mate overwrites its slot.
            int64_t own = fill0 + rank;
            if (own >= a.S) {
                const int64_t offers = aux0 + rank < INT32_MAX ? aux0 + rank : INT32_MAX;   // to the class, before this one
                own = (int64_t)below(a.sd, PURPOSE_EVICT, (uint32_t)p, reservoir ? (uint64_t)offers + 1 : (uint64_t)a.S);
                if (own >= a.S) continue;      // reservoir: not kept
            }
            // bitmap of the class-mates' positions: rank of a position = class-mates below it
            uint32_t* cm = s_cm[wave];
            uint16_t* cmpre = s_cmpre[wave];
            cm[2 * lane] = 0u;
            cm[2 * lane + 1] = 0u;
            for (int m0 = 0; m0 < m; m0 += WAVE) {
                const int q = m0 + lane;
                if (q < m && s_k[q] == ki) atomicOr(&cm[s_x[q] >> 5], 1u << (s_x[q] & 31));
            }
            {
                const int p0 = __popc(cm[2 * lane]), p1 = __popc(cm[2 * lane + 1]);
                const int before = wave_scan_incl(p0 + p1) - (p0 + p1);
                cmpre[2 * lane] = (uint16_t)before;
                cmpre[2 * lane + 1] = (uint16_t)(before + p0);
            }
            // later class-mates are gathered WAVE at a time so that their draws are made with full wavefronts
            uint16_t* pend = s_pend[wave];
            int npend = 0;
            bool beaten = false;
            for (int m0 = 0; m0 < m + WAVE; m0 += WAVE) {
                if (m0 < m) {
                    const int q = m0 + lane;
                    const int xq = q < m ? s_x[q] : 0;
                    const bool later = q < m && s_k[q] == ki && xq > p;
                    const uint64_t mask = __ballot(later);
                    if (later) pend[npend + __popcll(mask & ((1ull << lane) - 1))] = (uint16_t)xq;
                    npend += __popcll(mask);
                }
                if (npend >= WAVE || (m0 >= m && npend > 0)) {
                    const int take = npend < WAVE ? npend : WAVE;
                    const int xr = lane < take ? pend[lane] : 0;
                    // the rival's insertion number decides whether it overwrites at all, and (reservoir) its odds
                    const int rank_r = cmpre[xr >> 5] + __popc(cm[xr >> 5] & ((1u << (xr & 31)) - 1u));
                    bool hit = false;
                    if (lane < take && fill0 + rank_r >= a.S) {
                        const int64_t offers = aux0 + rank_r < INT32_MAX ? aux0 + rank_r : INT32_MAX;
                        hit = (int64_t)below(a.sd, PURPOSE_EVICT, (uint32_t)xr, reservoir ? (uint64_t)offers + 1 : (uint64_t)a.S) == own;
                    }
                    beaten |= __ballot(hit) != 0;
                    const int rest = lane + take < npend ? pend[lane + take] : 0;    // at most WAVE - 1 left over
                    if (lane + take < npend) pend[lane] = (uint16_t)rest;
                    npend -= take;
                }
            }
            if (beaten) continue;
            slot = own;
        }
        const int64_t dst_row = (int64_t)ki * a.S + slot;
        t.store(a.buf_x + dst_row * a.row_vec, v_lo, v_hi);
        if (tile == 0 && lane == 0) a.buf_y[dst_row] = ki;
    }
}

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
            if (tile == 0 && tid == 0) a.buf_y[dst_row] = dst_row / a.S;
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
            if (tile == 0 && tid == 0) a.buf_y[dst_row] = dst_row / a.S;
        }
    }
}

// ---------------------------------------------------------------------------
// rb_sample_augment: n = min(r, F) distinct stored samples, uniformly; any r
// and any number of classes (used when r > WAVE or there are more than WAVE
// chunks of classes).
//
// The workgroup computes F, the number of stored samples before every chunk of
// CH classes, and all n Floyd draws into LDS once; then each wavefront takes
// one work item (output row, tile of WAVE * U vectors): it decides whether its
// draw is taken, finds the chunk that holds the wanted sample, reads that
// chunk's CH fill counts (four consecutive classes per lane) and moves its tile.
//
// LDS (dynamic): s_cpre[nchunks] i32, s_t[r] u32.
// Grid: ceil(r * tpr / NWAVE) workgroups.
// ---------------------------------------------------------------------------
struct SampleArgs {
    const vec16* buf_x;
    vec16* out_x;
    int64_t* out_y;
    const int32_t* fill;
    const int32_t* chunk;
    DevState* state;
    Seed sd;
    int32_t r;
    int32_t K, nchunks;
    int64_t S;
    int64_t row_vec;
    int32_t tpr;
    int32_t tile_vec;
    int32_t tile_rem;
    int32_t rpb;          // small kernel: rows per workgroup (1 unless tpr == 1)
};

template <int U, bool NT>
__global__ void __launch_bounds__(TPB) rb_sample_kernel(const SampleArgs a)
{
    extern __shared__ uint32_t lds[];
    int32_t* s_cpre = reinterpret_cast<int32_t*>(lds);    // [nchunks]
    uint32_t* s_t = lds + a.nchunks;                      // [r]
    __shared__ int s_wave[NWAVE];

    const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;

    // ---- F and the number of stored samples before every chunk -----------------
    const int cper = (a.nchunks + TPB - 1) / TPB;
    int csum = 0;
    for (int u = 0; u < cper; ++u) {
        int ch = tid * cper + u;
        if (ch < a.nchunks) csum += a.chunk[ch];
    }
    int F;
    int cbefore = block_scan_excl(csum, F, s_wave);
    for (int u = 0; u < cper; ++u) {
        int ch = tid * cper + u;
        if (ch < a.nchunks) {
            s_cpre[ch] = cbefore;
            cbefore += a.chunk[ch];
        }
    }
    const int n = a.r < F ? a.r : F;
    if (blockIdx.x == 0 && tid == 0) a.state->last_n = n;

    // ---- Floyd's n-subset of [0, F): all draws ----------------------------------
    const int base = F - n;
    for (int i = tid; i < n; i += TPB)
        s_t[i] = (uint32_t)below(a.sd, PURPOSE_SAMPLE, (uint32_t)i, (uint64_t)base + i + 1);
    __syncthreads();

    // ---- one work item per wavefront, no workgroup barrier from here on ---------
    const int64_t item = (int64_t)blockIdx.x * NWAVE + wave;
    if (item >= (int64_t)a.r * a.tpr) return;
    const int j = (int)(item / a.tpr), tile = (int)(item % a.tpr);    // output row, tile of it
    if (j >= n) {                              // fewer stored samples than asked for
        if (tile == 0 && lane == 0) a.out_y[j] = -1;
        return;
    }
    int64_t v_lo, v_hi;
    tile_bounds(tile, a.tile_vec, a.tile_rem, a.row_vec, v_lo, v_hi);

    // Draw j is replaced by base + j iff an earlier draw had the same value, or it equals
    // base + q for an earlier q whose own draw was replaced.
    int cur = j;
    bool taken = false;
    for (;;) {
        const uint32_t t = s_t[cur];
        bool same = false;
        for (int q = lane; q < cur; q += WAVE) same |= (s_t[q] == t);
        if (__ballot(same) != 0) { taken = true; break; }
        const int64_t q = (int64_t)t - base;
        if (q < 0 || q >= cur) break;
        cur = (int)q;
    }
    const int g = taken ? base + j : (int)s_t[j];      // g-th stored sample, class-major

    // chunk holding g: the last one with s_cpre <= g
    int lo = 0, hi = a.nchunks - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (s_cpre[mid] <= g) lo = mid; else hi = mid - 1;
    }
    const int gl = g - s_cpre[lo];
    const int4 f = *reinterpret_cast<const int4*>(a.fill + (int64_t)lo * CH + 4 * lane);
    const int local = f.x + f.y + f.z + f.w;
    const int lincl = wave_scan_incl(local);
    int acc = lincl - local;
    const bool mine = gl >= acc && gl < lincl;
    int u = 0;
    if (mine) {
        if (gl >= acc + f.x) { acc += f.x; u = 1;
            if (gl >= acc + f.y) { acc += f.y; u = 2;
                if (gl >= acc + f.z) { acc += f.z; u = 3; } } }
    }
    const int owner = __builtin_ctzll(__ballot(mine) | (1ull << 63));
    const int pk = lane_read(lo * CH + 4 * lane + u, owner);
    const int ps = lane_read(gl - acc, owner);

    Tile<U, NT, WAVE, false> t;
    t.load(a.buf_x + ((int64_t)pk * a.S + ps) * a.row_vec, v_lo, v_hi);
    t.store(a.out_x + (int64_t)j * a.row_vec, v_lo, v_hi);
    if (tile == 0 && lane == 0) a.out_y[j] = pk;
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
        if (tile == 0 && tid == 0) a.out_y[j] = pk;
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
struct StepArgs {
    UpdateArgs u;
    vec16* out_x;
    int64_t* out_y;
    int32_t r;
    int32_t first_gather;   // index of the first representative mover (the candidate movers come before)
};

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
            if (tile == 0 && tid == 0) a.buf_y[dst_row] = dst_row / a.S;
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
    if (tile == 0 && tid == 0) sa.out_y[j] = pk;
}

// ---------------------------------------------------------------------------
// Measurement helpers
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(TPB) rb_standin_kernel(float* __restrict__ sink, int64_t iters)
{
    float x0 = threadIdx.x * 1e-3f, x1 = x0 + 1.f, x2 = x0 + 2.f, x3 = x0 + 3.f;
    const float m = 0.999f, d = 1e-3f;
    for (int64_t i = 0; i < iters; ++i) {
        x0 = fmaf(x0, m, d); x1 = fmaf(x1, m, d); x2 = fmaf(x2, m, d); x3 = fmaf(x3, m, d);
        x0 = fmaf(x0, m, d); x1 = fmaf(x1, m, d); x2 = fmaf(x2, m, d); x3 = fmaf(x3, m, d);
    }
    sink[(int64_t)blockIdx.x * TPB + threadIdx.x] = x0 + x1 + x2 + x3;
}

template <int U, bool NT>
__global__ void __launch_bounds__(TPB) rb_copy_kernel(vec16* __restrict__ dst, const vec16* __restrict__ src, int64_t nvec)
{
    const int64_t lo = (int64_t)blockIdx.x * (TPB * U);
    const int64_t hi = lo + TPB * U < nvec ? lo + TPB * U : nvec;
    Tile<U, NT> t;
    t.load(src, lo, hi);
    t.store(dst, lo, hi);
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

// ===========================================================================
// Host side: the C ABI
// ===========================================================================
struct rb_buffer {
    int64_t K, S, row_bytes, row_vec;
    int32_t dtype;
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
    int opt_unroll, opt_nt, opt_rpb, opt_fuse;
    // policy variant and its per-class state (two copies, like the fill counts)
    int selection, eviction;
    size_t off_aux[2];
    int64_t updates;         // rb_update calls since the last rb_bind
};

namespace {

struct Shape {
    int unroll, tpr, tile_vec, tile_rem, rpb;
    int64_t groups;
};

// Split `rows` rows of `row_vec` vectors into tiles of at most width * unroll vectors, where `width`
// is the number of threads that share a tile: TPB in the small-count kernels (a workgroup per tile),
// WAVE in the general ones (a wavefront per tile).
Shape plan_shape(const rb_buffer* rb, int64_t rows, int width)
{
    Shape s;
    const int64_t row_vec = rb->row_vec;
    int u = rb->opt_unroll;
    if (u == 0) {
        // Largest unroll that still leaves at least 1024 tiles (four workgroups per compute unit in
        // the small-count kernels, four wavefronts in the general ones); never below two vectors in
        // flight per thread (one was slower at every size measured) unless the row is shorter.
        u = 8;
        while (u > 2 && rows * ((row_vec + (int64_t)width * u - 1) / ((int64_t)width * u)) < 1024) u >>= 1;
        while (u > 1 && (int64_t)width * (u / 2) >= row_vec) u >>= 1;
    }
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
hipError_t launch_update(const UpdateArgs& a, bool small, int unroll, dim3 grid, size_t lds, hipStream_t st)
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
    switch (unroll) {
    case 1: rb_update_kernel<1, NT><<<grid, TPB, lds, st>>>(a); break;
    case 2: rb_update_kernel<2, NT><<<grid, TPB, lds, st>>>(a); break;
    case 4: rb_update_kernel<4, NT><<<grid, TPB, lds, st>>>(a); break;
    default: rb_update_kernel<8, NT><<<grid, TPB, lds, st>>>(a); break;
    }
    return hipGetLastError();
}

template <bool NT>
hipError_t launch_sample(const SampleArgs& a, int unroll, dim3 grid, size_t lds, hipStream_t st)
{
    if (a.r <= WAVE && a.nchunks <= WAVE) {
        switch (unroll) {
        case 1: rb_sample_small_kernel<1, NT><<<grid, TPB, lds, st>>>(a); break;
        case 2: rb_sample_small_kernel<2, NT><<<grid, TPB, lds, st>>>(a); break;
        case 4: rb_sample_small_kernel<4, NT><<<grid, TPB, lds, st>>>(a); break;
        default: rb_sample_small_kernel<8, NT><<<grid, TPB, lds, st>>>(a); break;
        }
        return hipGetLastError();
    }
    switch (unroll) {
    case 1: rb_sample_kernel<1, NT><<<grid, TPB, lds, st>>>(a); break;
    case 2: rb_sample_kernel<2, NT><<<grid, TPB, lds, st>>>(a); break;
    case 4: rb_sample_kernel<4, NT><<<grid, TPB, lds, st>>>(a); break;
    default: rb_sample_kernel<8, NT><<<grid, TPB, lds, st>>>(a); break;
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

template <bool NT>
hipError_t launch_copy(vec16* dst, const vec16* src, int64_t nvec, int unroll, hipStream_t st)
{
    const int64_t cap = (int64_t)TPB * unroll;
    dim3 grid((unsigned)((nvec + cap - 1) / cap));
    switch (unroll) {
    case 1: rb_copy_kernel<1, NT><<<grid, TPB, 0, st>>>(dst, src, nvec); break;
    case 2: rb_copy_kernel<2, NT><<<grid, TPB, 0, st>>>(dst, src, nvec); break;
    case 4: rb_copy_kernel<4, NT><<<grid, TPB, 0, st>>>(dst, src, nvec); break;
    default: rb_copy_kernel<8, NT><<<grid, TPB, 0, st>>>(dst, src, nvec); break;
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

}  // namespace

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
    rb->dtype = dtype;
    rb->nchunks = (int32_t)((classes + CH - 1) / CH);
    rb->buf_x = nullptr; rb->buf_y = nullptr; rb->ws = nullptr; rb->stream = nullptr;
    rb->bound = false;
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
    rb->ws_bytes = off;
    rb->selection = RB_SELECT_EXACT; rb->eviction = RB_EVICT_UNIFORM; rb->updates = 0;
    rb->opt_unroll = 0; rb->opt_nt = 1; rb->opt_rpb = 0; rb->opt_fuse = 1;
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

int rb_bind(rb_buffer* rb, void* buf_x, int64_t* buf_y, void* workspace, void* hip_stream)
{
    if (!rb || !buf_x || !buf_y || !workspace) return RB_EINVAL;
    if (!aligned(buf_x, 16) || !aligned(buf_y, 8) || !aligned(workspace, 256)) return RB_EINVAL;
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
    rb->bound = true;
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
    if (c == 0) return RB_OK;

    const bool variant = rb->selection != RB_SELECT_EXACT || rb->eviction != RB_EVICT_UNIFORM;
    const bool small = c <= WAVE && !variant;
    // Rows the grid is sized for.  The Bernoulli selection yields a random number of candidates
    // (mean c, at most b); the movers loop over the work items, so any number is handled, and
    // the grid only has to be large enough for the usual case.
    int64_t rows = c;
    if (rb->selection == RB_SELECT_BERNOULLI) {
        int64_t slack = 16;
        while (slack * slack < 36 * c) ++slack;          // about six standard deviations
        rows = c + slack < b ? c + slack : b;
    }
    const Shape sh = plan_shape(rb, rows, small ? TPB : WAVE);
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
    hipError_t e = rb->opt_nt ? launch_update<true>(a, small, sh.unroll, grid, lds, rb->stream)
                              : launch_update<false>(a, small, sh.unroll, grid, lds, rb->stream);
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
    if (r == 0) return RB_OK;

    const bool small = r <= WAVE && rb->nchunks <= WAVE;
    const Shape sh = plan_shape(rb, r, small ? TPB : WAVE);
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
    hipError_t e = rb->opt_nt ? launch_sample<true>(a, sh.unroll, grid, lds, rb->stream)
                              : launch_sample<false>(a, sh.unroll, grid, lds, rb->stream);
    return e == hipSuccess ? RB_OK : RB_EHIP;
}

int rb_update_sample(rb_buffer* rb, const void* batch_x, const int64_t* batch_y, int64_t b, int64_t c,
                     int64_t r, uint64_t seed, uint64_t step, void* out_x, int64_t* out_y)
{
    if (!rb || !batch_x || !batch_y) return RB_EINVAL;
    if (b < 1 || b > RB_MAX_BATCH || c < 0 || c > b) return RB_EINVAL;
    if (!aligned(batch_x, 16) || !aligned(batch_y, 8)) return RB_EINVAL;
    if (r < 0 || r > RB_MAX_BATCH) return RB_EINVAL;
    if (r > 0 && (!out_x || !out_y || !aligned(out_x, 16) || !aligned(out_y, 8))) return RB_EINVAL;
    if (!rb->bound) return RB_ESTATE;

    const bool fused = c >= 1 && c <= WAVE && r >= 1 && r <= WAVE && rb->nchunks <= DIRECT_CHUNKS && rb->opt_fuse &&
                       rb->selection == RB_SELECT_EXACT && rb->eviction == RB_EVICT_UNIFORM;
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

int rb_read_state(rb_buffer* rb, int32_t* fill_host, int64_t* last_n_host, uint32_t* flags_host)
{
    if (!rb) return RB_EINVAL;
    if (!rb->bound) return RB_ESTATE;
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
    default:
        return RB_EINVAL;
    }
}

int rb_destroy(rb_buffer* rb)
{
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
    hipError_t e = nontemporal ? launch_copy<true>(static_cast<vec16*>(dst), static_cast<const vec16*>(src), nvec, unroll, st)
                               : launch_copy<false>(static_cast<vec16*>(dst), static_cast<const vec16*>(src), nvec, unroll, st);
    return e == hipSuccess ? RB_OK : RB_EHIP;
}

}  // extern "C"
