// General kernels: buffer reset, rb_update and rb_sample_augment for any candidate / representative count and any policy variant.
// Included by rb.hip only, after rb_device.h.
#pragma once

#include "rb_device.h"

namespace {

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
// LDS (dynamic): s_first[b] u32 (lowest candidate index that drew a value;
// with the Bernoulli selection: the class of every position whose coin came up heads),
// s_k[cap] i32 (class per candidate, LAB_INVALID outside [0, K)), s_t[cap] u16
// (Floyd draws), s_x[cap] u16 (candidate positions, Floyd emission order or,
// with the Bernoulli selection, mini-batch order); cap = c, or b for Bernoulli.
//
// Grid: `nchunks` bookkeeping workgroups (new fill counts and chunk sums for CH
// classes each), then ceil(c * tpr / NWAVE) mover workgroups.
// ---------------------------------------------------------------------------

template <int U, bool NT, int NARROW>       // NARROW: binary32 mini-batch rows are stored 0 - as they come, 1 - as bfloat16, 2 - in 8 bits per element
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
        // s_lab[q] = class of sample q if its coin came up heads, LAB_UNSELECTED otherwise.  All labels
        // are requested first (coalesced, MAX_PER = RB_MAX_BATCH / TPB per thread) so that their memory
        // round trip overlaps the coin draws.
        int32_t* s_lab = reinterpret_cast<int32_t*>(s_first);
        constexpr int MAX_PER = RB_MAX_BATCH / TPB;
        int64_t yl[MAX_PER];
#pragma unroll
        for (int u = 0; u < MAX_PER; ++u) {
            const int q = tid + u * TPB;
            yl[u] = q < b ? a.batch_y[q] : -1;
        }
        uint32_t heads = 0;                    // bit u: the coin of sample tid + u * TPB
        for (int q = tid, u = 0; q < b; q += TPB, ++u)
            heads |= (uint32_t)((int64_t)below(a.sd, PURPOSE_COIN, (uint32_t)q, (uint64_t)b) < c) << u;
#pragma unroll
        for (int u = 0; u < MAX_PER; ++u) {
            const int q = tid + u * TPB;
            if (q < b) s_lab[q] = !((heads >> u) & 1u) ? LAB_UNSELECTED : (yl[u] >= 0 && yl[u] < a.K) ? (int32_t)yl[u] : LAB_INVALID;
        }
        __syncthreads();
        const int per = (b + TPB - 1) / TPB;
        const int q_lo = tid * per, q_hi = q_lo + per < b ? q_lo + per : b;
        int mine = 0;
        for (int q = q_lo; q < q_hi; ++q) mine += s_lab[q] != LAB_UNSELECTED;
        int at = block_scan_excl(mine, m, s_wave);
        for (int q = q_lo; q < q_hi; ++q) {
            const int32_t k = s_lab[q];
            if (k != LAB_UNSELECTED) {
                s_x[at] = (uint16_t)q;
                s_k[at] = k;
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
        const int base = b - c;
        // s_first[v] = lowest candidate index that drew v: only the entries that are drawn at all
        // are initialised (by every thread that drew them), then minimised
        for (int i = tid; i < c; i += TPB) {
            uint32_t t = (uint32_t)below(a.sd, PURPOSE_SELECT, (uint32_t)i, (uint64_t)(base + i + 1));
            s_t[i] = (uint16_t)t;
            s_first[t] = 0xFFFFFFFFu;
        }
        __syncthreads();
        for (int i = tid; i < c; i += TPB) atomicMin(&s_first[s_t[i]], (uint32_t)i);
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
            s_x[i] = (uint16_t)(taken ? base + i : (int)s_t[i]);
        }
        // the candidates' labels, four loads in flight per thread
        for (int i0 = tid; i0 < c; i0 += 4 * TPB) {
            int64_t y[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * TPB;
                y[u] = i < c ? a.batch_y[s_x[i]] : -1;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * TPB;
                if (i < c) s_k[i] = (y[u] >= 0 && y[u] < a.K) ? (int32_t)y[u] : LAB_INVALID;
            }
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
        int i, tile;                           // candidate, tile of its row
        split_item(item, a.tpr, i, tile);
        const int p = s_x[i];                                             // its mini-batch position
        const int32_t ki = s_k[i];
        if (ki < 0) continue;                  // label outside [0, K): dropped (flagged by bookkeeping)
        int64_t v_lo, v_hi;
        tile_bounds(tile, a.tile_vec, a.tile_rem, a.row_vec, v_lo, v_hi);

        const int64_t fill0 = a.fill_old[ki];
        const int64_t aux0 = a.eviction != RB_EVICT_UNIFORM ? a.aux_old[ki] : 0;
        // the row is read while the wavefront works out where it goes
        Tile<U, NT, WAVE, false, NARROW == 2 ? CV_NARROW8 : NARROW ? CV_NARROW : CV_NONE> t;
        t.load(a.batch_x + (int64_t)p * a.row_vec * (NARROW == 2 ? 4 : NARROW ? 2 : 1), v_lo, v_hi);

        // Candidates of class ki, in mini-batch order: the one with `rank` class-mates before it is
        // insertion number fill0 + rank of the class.  Each lane looks at every WAVE-th candidate,
        // remembers in a bit mask which of them are class-mates, and the counts are summed over the
        // wavefront once at the end (no ballot, hence no scalar dependency, per round).
        uint64_t hit = 0;                      // bit `round`: candidate round * WAVE + lane is a class-mate (m <= 64 * WAVE)
        int my_rank = 0;
        for (int m0 = 0, round = 0; m0 < m; m0 += WAVE, ++round) {
            const int q = m0 + lane;
            const bool same = q < m && s_k[q] == ki;
            const int xq = q < m ? s_x[q] : 0;
            hit |= (uint64_t)same << round;
            my_rank += same && xq < p;
        }
        const int mine = __popcll(hit);
        const int incl = wave_scan_incl(mine | (my_rank << 16));      // both sums are <= 4096
        const int total = lane_read(incl, WAVE - 1) & 0xFFFF, rank = lane_read(incl, WAVE - 1) >> 16;
        int64_t slot;
        if (fill0 + total <= a.S) {
            slot = fill0 + rank;               // all of them append: distinct slots
        } else if (a.eviction == RB_EVICT_FIFO) {
            // insertion number fill0 + rank overwrites the oldest sample once the class is full; it is
            // itself overwritten in this step if a class-mate comes a whole round of S later
            const int64_t at = fill0 + rank;
            if (at + a.S < fill0 + total) continue;
            slot = at < a.S ? at : (aux0 + at - a.S) % a.S;
        } else if (total <= WAVE) {
            // Insertions beyond the capacity overwrite a uniformly drawn slot (or, with reservoir
            // sampling, are kept with probability S / offers).  This candidate is not stored if a
            // later class-mate overwrites its slot.  The usual case: every class-mate gets a lane
            // (in no particular order), which works out its insertion number (class-mates before it)
            // and, if it overwrites, the slot it draws.
            const bool reservoir = a.eviction == RB_EVICT_RESERVOIR;
            uint16_t* pend = s_pend[wave];
            int at = (incl & 0xFFFF) - mine;
            for (uint64_t h = hit; h != 0; h &= h - 1) pend[at++] = s_x[__builtin_ctzll(h) * WAVE + lane];
            const bool has = lane < total;
            const int xl = has ? pend[lane] : 0;
            int rl = 0;
            for (int j = 0; j < total; ++j) rl += lane_read(xl, j) < xl;
            const bool draws = has && xl >= p && fill0 + rl >= a.S;     // this candidate and the later ones
            int dr = -1;
            if (draws) {
                const int64_t offers = aux0 + rl < INT32_MAX ? aux0 + rl : INT32_MAX;   // to the class, before this one
                dr = (int)below(a.sd, PURPOSE_EVICT, (uint32_t)xl, reservoir ? (uint64_t)offers + 1 : (uint64_t)a.S);
            }
            int64_t own = fill0 + rank;
            if (own >= a.S) {
                const int me = __builtin_ctzll(__ballot(has && xl == p) | (1ull << 63));
                own = lane_read(dr, me);
                if (own >= a.S) continue;      // reservoir: not kept
            }
            if (__ballot(draws && xl > p && dr == (int)own) != 0) continue;
            slot = own;
        } else {
            // the same for a class with more than WAVE candidates in this step
            const bool reservoir = a.eviction == RB_EVICT_RESERVOIR;
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
        if (tile == 0 && lane == 0) { a.buf_y[dst_row] = ki; count_moved(a.state); }
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

template <int U, bool NT, int WIDEN>        // WIDEN: rows are handed out 0 - as stored, 1 - widened from bfloat16, 2 - from 8 bits per element to binary32
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
    int j, tile;                               // output row, tile of it
    split_item(item, a.tpr, j, tile);
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

    Tile<U, NT, WAVE, false, WIDEN == 2 ? CV_WIDEN8 : WIDEN ? CV_WIDEN : CV_NONE> t;
    t.load(a.buf_x + ((int64_t)pk * a.S + ps) * a.row_vec, v_lo, v_hi);
    t.store(a.out_x + (int64_t)j * a.row_vec * (WIDEN == 2 ? 4 : WIDEN ? 2 : 1), v_lo, v_hi);
    if (tile == 0 && lane == 0) { a.out_y[j] = pk; count_moved(a.state); }
}

}  // namespace
