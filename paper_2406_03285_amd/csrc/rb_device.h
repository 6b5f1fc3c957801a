// Device-side building blocks of the rehearsal-buffer kernels (gfx950): constants, counter-based
// random draws, wavefront and workgroup primitives, the row mover and the launch-argument structs.
// Included by rb.hip only.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "rb.h"

namespace {

constexpr int TPB = 256;               // threads per workgroup: four 64-wide wavefronts
constexpr int WAVE = 64;
constexpr int NWAVE = TPB / WAVE;
constexpr int CH = 256;                // classes per chunk of the two-level fill index
constexpr int XCDS = 8;               // accelerator dies of the chip; workgroup w of a grid runs on die w % XCDS
constexpr int TILE_UNIT = 64;          // granularity, in 16-byte vectors, at which a row is cut into tiles
constexpr uint32_t PURPOSE_SELECT = 1; // counter word that separates the three kinds of draws
constexpr uint32_t PURPOSE_EVICT = 2;
constexpr uint32_t PURPOSE_SAMPLE = 3;
constexpr uint32_t PURPOSE_COIN = 4;   // per-sample coin of the Bernoulli selection
constexpr int32_t LAB_UNSELECTED = -2; // LDS label table: position is not a candidate
constexpr int32_t LAB_INVALID = -1;    // candidate whose label is outside [0, K)

typedef uint32_t vec16 __attribute__((ext_vector_type(4)));   // one 16-byte transfer
typedef uint32_t vec8 __attribute__((ext_vector_type(2)));    // half of one: four bfloat16

// Device-resident state words at the start of the workspace.
struct DevState {
    uint32_t flags;
    uint32_t pad;
    int64_t last_n;
};
// Behind them: counters of the rows moved since the last bind (stored candidates + representatives handed out).
// One thread per moved row adds to one of MOVED_COUNTERS counters, picked by its workgroup's number and kept
// MOVED_STRIDE bytes apart: additions to ONE address are carried out one after the other (measured on MI355X: about
// 8.5 ns each, 17 us for the 2048 rows of one step with 1024 candidates and representatives, which the launch
// cannot end before), additions to addresses in different memory channels side by side.  The host adds them up.
constexpr int MOVED_COUNTERS = 64;
constexpr size_t MOVED_STRIDE = 256;
constexpr size_t STATE_HEAD_BYTES = 256;
constexpr size_t STATE_BYTES = STATE_HEAD_BYTES + MOVED_COUNTERS * MOVED_STRIDE;

// One more row is being moved (called by the one thread that also writes the row's label).
__device__ __forceinline__ void count_moved(DevState* state)
{
    char* counters = reinterpret_cast<char*>(state) + STATE_HEAD_BYTES;
    atomicAdd(reinterpret_cast<unsigned long long*>(counters + (blockIdx.x & (MOVED_COUNTERS - 1)) * MOVED_STRIDE), 1ull);
}

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

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global load
// and store the wavefront has in flight; the planners keep loads on their way in and table entries
// and fill counts on their way out across these barriers (nobody in the same launch reads them).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
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
// Reduced-precision storage: binary32 elements kept as bfloat16 (the upper half of the binary32,
// rounded to nearest, ties to even; NaN keeps its sign and upper payload bits and is made quiet).
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t bf16_of(uint32_t u)
{
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;    // carries into the exponent where rounding demands it
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? ((u >> 16) | 0x0040u) : rounded;
}

// Four consecutive binary32 elements (one vector) -> four bfloat16 (half a vector), element order kept; and back: exact
__device__ __forceinline__ vec8 narrow4(const vec16 a)
{
    vec8 o;
    o.x = bf16_of(a.x) | (bf16_of(a.y) << 16);
    o.y = bf16_of(a.z) | (bf16_of(a.w) << 16);
    return o;
}
__device__ __forceinline__ vec16 widen4(const vec8 s)
{
    vec16 a;
    a.x = s.x << 16; a.y = s.x & 0xFFFF0000u; a.z = s.y << 16; a.w = s.y & 0xFFFF0000u;
    return a;
}

// Reduced-precision storage in 8 bits (Sec. VII: data reduction of the stored samples): a binary32 element x is kept as the
// byte nearest to 255 x (product and rounding in binary32, ties to even; below 0 and NaN give 0, above 255 gives 255)
// and handed out as byte / 255 (binary32 division, correctly rounded).  Meant for samples in [0, 1], like image tensors.
__device__ __forceinline__ uint32_t u8_of(uint32_t bits)
{
    const float t = __uint_as_float(bits) * 255.0f;
    if (!(t > 0.0f)) return 0u;                 // not above zero, or NaN
    if (t >= 255.0f) return 255u;
    return (uint32_t)(int)rintf(t);             // nearest, ties to even
}
__device__ __forceinline__ uint32_t pack4_u8(const vec16 a)      // four consecutive elements -> four bytes, element order kept
{
    return u8_of(a.x) | (u8_of(a.y) << 8) | (u8_of(a.z) << 16) | (u8_of(a.w) << 24);
}
__device__ __forceinline__ vec16 unpack4_u8(const uint32_t s)
{
    vec16 a;
    a.x = __float_as_uint((float)(s & 0xFFu) / 255.0f);
    a.y = __float_as_uint((float)((s >> 8) & 0xFFu) / 255.0f);
    a.z = __float_as_uint((float)((s >> 16) & 0xFFu) / 255.0f);
    a.w = __float_as_uint((float)(s >> 24) / 255.0f);
    return a;
}

// bit 0: convert while loading, bit 1: while storing; bit 2: the narrow form is 8 bits per element instead of bfloat16
enum { CV_NONE = 0, CV_NARROW = 1, CV_WIDEN = 2, CV_BOTH = 3, CV_Q8 = 4, CV_NARROW8 = CV_Q8 | CV_NARROW, CV_WIDEN8 = CV_Q8 | CV_WIDEN };

// The Tile conversion of a mover whose stored rows have the form `storage` (RB_STORE_*); dir: CV_NARROW (a sample is
// stored), CV_WIDEN (a stored sample is handed out), CV_BOTH (sample to sample through the stored form).  And the vectors
// of a sample per vector of its stored row.
constexpr int stored_cv(int storage, int dir)
{
    return storage == RB_STORE_U8 ? (CV_Q8 | dir) : storage == RB_STORE_BF16 ? dir : CV_NONE;
}
constexpr int stored_wide(int storage)
{
    return storage == RB_STORE_U8 ? 4 : storage == RB_STORE_BF16 ? 2 : 1;
}

// ---------------------------------------------------------------------------
// Row mover: one tile of one row, U vectors per thread in flight.
// ---------------------------------------------------------------------------
// W: threads that share the tile (a workgroup or one wavefront).  CV: CV_NARROW - the source row is
// binary32 (two vectors per vector of the tile), converted to bfloat16 while it is loaded; CV_WIDEN -
// the destination row is binary32, converted from the tile's bfloat16 while it is stored; CV_BOTH -
// binary32 to binary32 through the bfloat16 a stored copy would hold.  Tile indices always count
// vectors of the narrow (stored) row.
template <int U, bool NT, int W = TPB, int PACED = 1, int CV = CV_NONE>
struct Tile {
    // Without conversion a lane holds U vectors.  With one, it holds 2 U half vectors (four bfloat16 each):
    // a lane then touches 8 bytes of the narrow row and 16 bytes of the binary32 row per access, so every
    // instruction of a wavefront covers one contiguous run of bytes on either side.
    vec16 v[CV ? 1 : U];
    vec8 h[CV && !(CV & CV_Q8) ? 2 * U : 1];
    // 8-bit storage: 4 U quarter vectors (four bytes of the stored row against 16 bytes of the binary32 row per access)
    uint32_t q[CV & CV_Q8 ? 4 * U : 1];

    // Requires lo < hi.  No lane is ever masked off: a lane whose index falls past the end of
    // the tile moves the tile's last vector again (same source, same destination, same bytes as
    // the lane that owns it), so the copy stays correct and branch-free.  That keeps the number
    // of loads in flight known at compile time - a wait for an earlier load then does not have
    // to drain these - and keeps the compiler from moving loads down into a guarded store.
    __device__ __forceinline__ void load(const vec16* __restrict__ src, int64_t lo, int64_t hi)
    {
        if (CV & CV_Q8) {
#pragma unroll
            for (int u = 0; u < 4 * U; ++u) {
                int64_t j = 4 * lo + (int64_t)u * W + (threadIdx.x & (W - 1));
                j = j < 4 * hi ? j : 4 * hi - 1;
                if (CV & CV_NARROW) {
                    q[u] = pack4_u8(NT ? __builtin_nontemporal_load(src + j) : src[j]);
                } else {
                    const uint32_t* quarter = reinterpret_cast<const uint32_t*>(src);
                    q[u] = NT ? __builtin_nontemporal_load(quarter + j) : quarter[j];
                }
            }
            return;
        }
        if (CV) {
#pragma unroll
            for (int u = 0; u < 2 * U; ++u) {
                int64_t j = 2 * lo + (int64_t)u * W + (threadIdx.x & (W - 1));
                j = j < 2 * hi ? j : 2 * hi - 1;
                if (CV & CV_NARROW) {
                    h[u] = narrow4(NT ? __builtin_nontemporal_load(src + j) : src[j]);
                } else {
                    const vec8* half = reinterpret_cast<const vec8*>(src);
                    h[u] = NT ? __builtin_nontemporal_load(half + j) : half[j];
                }
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t i = lo + (int64_t)u * W + (threadIdx.x & (W - 1));
            i = i < hi ? i : hi - 1;
            v[u] = NT ? __builtin_nontemporal_load(src + i) : src[i];
        }
    }
    // PACED = 1: all loads are waited for first and every store is waited for before the next one
    // is issued.  Measured on MI355X with a bare mover of the same shape (64 rows of 301 056 bytes,
    // U = 4): 7.6 us against 8.6 us when each store is issued as soon as its load has arrived
    // and 8.9 us with the guarded form; a launch of about one workgroup wave does better with few
    // writes in flight.  PACED = n > 1: a wait after every n-th store; n > U: the stores go out in
    // one burst once the loads have arrived, which is what launches of many workgroup waves do
    // best with (1024 rows of 301 056 bytes in 19 456 tiles: 105.6 us against 107.1 us paced;
    // 256 rows of 602 112 bytes: 52.1 against 54.1).  PACED = 0: no waits of its own.
    __device__ __forceinline__ void store(vec16* __restrict__ dst, int64_t lo, int64_t hi) const
    {
        if (PACED) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (CV & CV_Q8) {
#pragma unroll
            for (int u = 0; u < 4 * U; ++u) {
                int64_t j = 4 * lo + (int64_t)u * W + (threadIdx.x & (W - 1));
                j = j < 4 * hi ? j : 4 * hi - 1;
                if (CV & CV_WIDEN) {
                    const vec16 a = unpack4_u8(q[u]);
                    if (NT) __builtin_nontemporal_store(a, dst + j);
                    else dst[j] = a;
                } else {
                    uint32_t* quarter = reinterpret_cast<uint32_t*>(dst);
                    if (NT) __builtin_nontemporal_store(q[u], quarter + j);
                    else quarter[j] = q[u];
                }
                if (PACED && (u + 1) % PACED == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            return;
        }
        if (CV) {
#pragma unroll
            for (int u = 0; u < 2 * U; ++u) {
                int64_t j = 2 * lo + (int64_t)u * W + (threadIdx.x & (W - 1));
                j = j < 2 * hi ? j : 2 * hi - 1;
                if (CV & CV_WIDEN) {
                    const vec16 a = widen4(h[u]);
                    if (NT) __builtin_nontemporal_store(a, dst + j);
                    else dst[j] = a;
                } else {
                    vec8* half = reinterpret_cast<vec8*>(dst);
                    if (NT) __builtin_nontemporal_store(h[u], half + j);
                    else half[j] = h[u];
                }
                if (PACED && (u + 1) % PACED == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int64_t i = lo + (int64_t)u * W + (threadIdx.x & (W - 1));
            i = i < hi ? i : hi - 1;
            if (NT) __builtin_nontemporal_store(v[u], dst + i);
            else dst[i] = v[u];
            if (PACED && (u + 1) % PACED == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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

// Work item -> (row, tile of the row), tpr tiles per row.  The common cases avoid the 64-bit division.
__device__ __forceinline__ void split_item(int64_t item, int tpr, int& row, int& tile)
{
    if (tpr == 1) {
        row = (int)item;
        tile = 0;
    } else if (item <= 0x7FFFFFFF) {
        const uint32_t it = (uint32_t)item;
        row = (int)(it / (uint32_t)tpr);
        tile = (int)(it - (uint32_t)row * (uint32_t)tpr);
    } else {
        row = (int)(item / tpr);
        tile = (int)(item % tpr);
    }
}

// ---------------------------------------------------------------------------
// Launch arguments
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
    int64_t row_vec;      // 16-byte vectors per stored row (a mini-batch row has twice as many with bfloat16 storage)
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

struct StepArgs {
    UpdateArgs u;
    vec16* out_x;
    int64_t* out_y;
    int32_t r;
    int32_t first_gather;   // index of the first representative mover (the candidate movers come before)
};

}  // namespace
