// adacomp_apply: loop body of Alg. 2 (eqs. 3, 4, 5) for a queue of sparse updates.
//
// Two execution plans for the part of the work inside one call, chosen on the host from
// sizes alone:
//
//   scatter  one launch per update, in queue order.  Per-parameter staleness without
//            searching a history: cnt[k] is incremented by every applied non-zero entry for
//            k, so the sum of indicators of eq. 3 over u = j .. i-1 is cnt_k(at time i) -
//            cnt_k(at time j).  The reading cnt_k(j) is taken by a gather ("snapshot") of cnt
//            at the update's own indices, enqueued where PS time equals the update's pull
//            timestamp.  Only differences of cnt are used, so its starting values do not
//            matter, and an update that no later snapshot of the call looks back on is not
//            counted at all.  Indices inside one update are unique, so the scatter needs no atomics.
//            Each random 4-byte access moves a whole cache line: right for short or very
//            sparse queues.
//
//   sweep    one launch for the whole queue.  Parameters are independent of each other
//            (the result for k depends only on the touches of k, in time order), so a
//            workgroup owns a tile of consecutive coordinates, collects the slices of
//            all Q sorted index lists that fall into its tile (slice bounds come from a
//            bisection kernel), groups them by coordinate with a counting sort in LDS,
//            and replays every coordinate's touches in time order.  For a touch by update q
//            pulled at j, sigma_k is the number of earlier non-zero touches of k by updates
//            u with j <= u < q: eq. 3 evaluated on the tile's own lists; cnt is not needed.
//            Theta is read and written once per touched coordinate instead of once per
//            touch.  A tile whose lists do not fit LDS is replayed update by update by a
//            second kernel, one workgroup per such tile (queues of up to 64 updates: out of
//            LDS, with a mask of non-zero touches per coordinate; longer ones: from global
//            memory, snapshot scheme on cnt).  Dense queues (about one queued entry per parameter or more, up to
//            256 updates) take a kernel of their own that needs no sorting: a thread per
//            coordinate, the coordinate's non-zero touches as a bit mask over the queue.
//
// The part of an update's window that lies before the call is searched in the remembered
// updates (k_history) and handed to either plan as a per-entry addend.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "common.h"

namespace adacomp {
namespace {

constexpr uint32_t BLOCK = 256;
constexpr uint32_t WAVES = BLOCK / WAVE;
constexpr uint32_t ITEMS = 4;          // scatter plan: entries per thread
constexpr uint32_t TILE_MAX = 2048;    // sweep plan: most coordinates per tile of the sorting kernels (power of two); dense queues get smaller tiles
constexpr uint32_t TILE_MAX_SPARSE = 2048;  // ... and of the kernel for sparse queues
constexpr uint32_t HOT_TILE_MAX = TILE_MAX_SPARSE;  // largest tile the kernel for overflowing tiles keeps in LDS
constexpr uint32_t STAGE_CAP = 512;    // sweep plan: entries of the whole queue a tile can hold in LDS
constexpr uint32_t SLOW_GRID = 1024;
constexpr uint32_t PASS = 256;           // sweep plan: updates whose slices are staged together
constexpr uint32_t PASS_SHORT = 64;      // sweep plan: longest queue the kernel for short queues takes (one lane of wave 0 per update)
constexpr uint32_t DENSE_QMAX = 256;     // sweep plan: longest queue the kernel for dense queues takes
// ... and the queued entries per parameter from which it is used, for queues of up to 64 updates
// and for longer ones (measured crossovers against the sorting kernels: 0.5-1.0 and 1.4-1.8)
constexpr double DENSE_PER_COORD = 1.0, DENSE_PER_COORD_LONG = 1.75;
// ... and the queued entries per parameter up to which the kernel for sparse queues is used (measured against the
// sorting kernel on the mid-size model, 64 updates: 0.19 entries per parameter 0.34 against 0.32 ms per queue, 0.64
// entries per parameter 0.68 against 0.91 ms: its smaller table of slice bounds weighs more as the tiles shrink)
constexpr double SPARSE_PER_COORD = 0.75;
// one launch costs about as much as this many bytes of memory traffic (4 us at 5 TB/s)
constexpr double LAUNCH_COST_BYTES = 20e6;
static_assert((TILE_MAX & (TILE_MAX - 1)) == 0 && TILE_MAX >= BLOCK && STAGE_CAP % BLOCK == 0 && STAGE_CAP <= 65535,
              "tile and stage sizes");

struct ParamDesc {
    float *theta;
    uint32_t *cnt;
    uint64_t n;
    uint64_t tile_base;  // sweep plan: first tile of this tensor (entry L: number of tiles)
};
static_assert(sizeof(ParamDesc) % 8 == 0, "table is uploaded as 64-bit words");

struct UpdDesc {
    const uint32_t *idx;
    const float *val;
    const uint64_t *off;  // layer_off_dev
    uint32_t *snap;       // scratch: counter readings at pull time, one per entry
    const uint32_t *pre;  // staleness already accumulated before this call (pulled earlier), or nullptr
    uint32_t pull;        // pull timestamp relative to the first update of the call (0 if pulled earlier)
    uint32_t pad;
};
static_assert(sizeof(UpdDesc) % 8 == 0, "table is uploaded as 64-bit words");

// eqs. 5 and 4 for one entry: one divide, one multiply, one subtract, each rounded once.
__device__ __forceinline__ float step(float theta, float lr, uint32_t sigma, float v) {
    float alpha = lr;
    if (sigma != 0) alpha = __fdiv_rn(lr, (float)sigma);
    return __fsub_rn(theta, __fmul_rn(alpha, v));
}

__device__ __forceinline__ bool is_nonzero(float v) {  // indicator of eq. 3
    return (__float_as_uint(v) & KEY_MASK) != 0;
}

// An update applied by an earlier call, as the trace of Sec. 4 "Complexity" keeps it: its
// sorted index lists (and values, for the non-zero test of eq. 3).
struct HistDesc {
    const uint32_t *idx;
    const float *val;
    const uint64_t *off;  // layer_off_dev
};
static_assert(sizeof(HistDesc) % 8 == 0, "table is uploaded as 64-bit words");

// ------------------------------------------------------------------ scatter plan

// Tensor that holds entry e: the last l with off[l] <= e.
__device__ __forceinline__ uint32_t layer_of(const uint64_t *off, uint32_t L, uint64_t e) {
    uint32_t lo = 0, hi = L;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (off[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

// snap[e] = cnt[idx[e]]: the reading of the counters at the worker's pull time.
__global__ __launch_bounds__(BLOCK) void k_snapshot(const ParamDesc *P, uint32_t L, const uint64_t *off,
                                                    const uint32_t *idx, uint32_t *snap, uint64_t total) {
    uint64_t e = (uint64_t)blockIdx.x * (BLOCK * ITEMS) + threadIdx.x;
    if (e >= total) return;
    uint32_t l = layer_of(off, L, e);
#pragma unroll
    for (uint32_t i = 0; i < ITEMS; ++i, e += BLOCK) {
        if (e >= total) break;
        while (e >= off[l + 1]) ++l;
        const uint32_t k = idx[e];
        if (k < P[l].n) snap[e] = P[l].cnt[k];  // an index outside the tensor (malformed update) is skipped
    }
}

// The part of eq. 3 that lies before the current call: for every entry of an update pulled
// at an earlier timestamp, the number of remembered updates H[first..nh) (= timestamps pull ..
// t0-1) that hold a non-zero entry for the same parameter, by bisection in their sorted
// index lists -- the search the paper describes (Sec. 4 "Complexity").
__global__ __launch_bounds__(BLOCK) void k_history(const HistDesc *H, uint32_t first, uint32_t nh, uint32_t L,
                                                   const uint64_t *off, const uint32_t *idx, uint32_t *pre,
                                                   uint64_t total) {
    const uint64_t e = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (e >= total) return;
    const uint32_t l = layer_of(off, L, e);
    const uint32_t k = idx[e];
    uint32_t sigma = 0;
    for (uint32_t h = first; h < nh; ++h) {
        const HistDesc u = H[h];
        if (!u.off) continue;  // an empty update was applied at that timestamp
        uint64_t lo = u.off[l], hi = u.off[l + 1];
        const uint64_t end = hi;
        while (lo < hi) {
            const uint64_t mid = lo + ((hi - lo) >> 1);
            if (u.idx[mid] < k) lo = mid + 1; else hi = mid;
        }
        if (lo < end && u.idx[lo] == k && is_nonzero(u.val[lo])) ++sigma;
    }
    pre[e] = sigma;
}

// One PS iteration.  STALE: the update has a snapshot of the counters taken at its pull time
// (or at the start of the call if it was pulled earlier); PRE: it was pulled before this call
// and carries the staleness accumulated until the call.  Without either, sigma_k is 0 or 1
// for every entry and alpha_k = alpha.  COUNT: a later update of the call takes the difference
// of two counter readings around this one, so its non-zero entries must be counted; the last
// updates of a call (the only one, when the server applies update by update) leave the
// counters alone.
template <bool STALE, bool PRE, bool COUNT>
__global__ __launch_bounds__(BLOCK) void k_scatter_apply(const ParamDesc *P, uint32_t L, const uint64_t *off,
                                                         const uint32_t *idx, const float *val,
                                                         const uint32_t *snap, const uint32_t *pre, uint64_t total,
                                                         float lr) {
    uint64_t e = (uint64_t)blockIdx.x * (BLOCK * ITEMS) + threadIdx.x;
    if (e >= total) return;
    uint32_t l = layer_of(off, L, e);
#pragma unroll
    for (uint32_t i = 0; i < ITEMS; ++i, e += BLOCK) {
        if (e >= total) break;
        while (e >= off[l + 1]) ++l;
        const uint32_t k = idx[e];
        if (k >= P[l].n) continue;  // malformed update: skipped, never dereferenced
        const float v = val[e];
        const bool nonzero = is_nonzero(v);
        float *theta = P[l].theta + k;
        uint32_t *cnt = P[l].cnt + k;
        uint32_t c = 0, sigma = 0;
        if (STALE || (COUNT && nonzero)) c = *cnt;
        if (STALE) sigma = c - snap[e];  // eq. 3, the part inside this call
        if (PRE) sigma += pre[e];        // eq. 3, the part before it
        *theta = step(*theta, lr, sigma, v);
        if (COUNT && nonzero) *cnt = c + 1;
    }
}

// The rule the paper ascribes to its competitors (Sec. 5.2): one learning rate per update,
// alpha divided by the update's global staleness i - j.
__global__ __launch_bounds__(BLOCK) void k_scatter_apply_global(const ParamDesc *P, uint32_t L, const uint64_t *off,
                                                                const uint32_t *idx, const float *val,
                                                                uint64_t total, float lr, uint32_t sigma) {
    uint64_t e = (uint64_t)blockIdx.x * (BLOCK * ITEMS) + threadIdx.x;
    if (e >= total) return;
    uint32_t l = layer_of(off, L, e);
#pragma unroll
    for (uint32_t i = 0; i < ITEMS; ++i, e += BLOCK) {
        if (e >= total) break;
        while (e >= off[l + 1]) ++l;
        const uint32_t k = idx[e];
        if (k >= P[l].n) continue;
        float *theta = P[l].theta + k;
        *theta = step(*theta, lr, sigma, val[e]);
    }
}

// flags[0] |= 1 if an index is outside its tensor, |= 2 if the indices of a tensor are not
// strictly ascending, |= 4 if the device copy of the offsets differs from the host's total.
__global__ __launch_bounds__(BLOCK) void k_validate(const uint64_t *n, uint32_t L, const uint64_t *off,
                                                    const uint32_t *idx, uint64_t total, uint32_t *flags) {
    const uint64_t e = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (e == 0 && off[L] != total) atomicOr(flags, 4u);
    if (e >= total || off[L] != total) return;
    const uint32_t l = layer_of(off, L, e);
    uint32_t bad = 0;
    if (idx[e] >= n[l]) bad |= 1u;
    if (e > off[l] && idx[e - 1] >= idx[e]) bad |= 2u;
    if (bad) atomicOr(flags, bad);
}

// ------------------------------------------------------------------ sweep plan

struct Sweep {
    const ParamDesc *P;   // [L+1]
    const UpdDesc *U;     // [Q]
    const uint32_t *B;    // [Q][ntiles+1]: first entry of update q at or after the start of tile t
    const uint32_t *tile_tensor;  // [ntiles] tensor that owns tile t
    const uint32_t *pa_off;   // [Q+1] CSR over PS time: updates pulled at that time and applied >= 2 later
    const uint32_t *pa_list;
    uint32_t *ovf;        // ovf[0] = number of tiles left to the slow kernel, ovf[1..] = their ids
    uint32_t L, Q;
    uint32_t ntiles, tile_shift;
    float lr;
};

__device__ __forceinline__ uint32_t tile_layer(const ParamDesc *P, uint32_t L, uint32_t t) {
    uint32_t lo = 0, hi = L;  // the last l with tile_base[l] <= t; t < tile_base[L], the number of tiles
    {   // first probe by proportion: the answer when the tensors are equally large
        uint32_t g = (uint32_t)((float)t * (float)L / (float)P[L].tile_base);
        if (g >= L) g = L - 1;
        const uint64_t b_g = P[g].tile_base, b_next = P[g + 1].tile_base;
        if (b_g <= t) {
            if (b_next > t) return g;
            lo = g + 1;  // tile_base[g + 1] <= t
        } else {
            hi = g;
        }
    }
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (P[mid].tile_base <= t) lo = mid; else hi = mid;
    }
    return lo;
}

constexpr uint32_t BOUNDS_WAYS = 4;

// B[q][t] by search in the sorted index list of the tile's tensor; tile_tensor[t].
__global__ __launch_bounds__(BLOCK) void k_bounds(Sweep sw, uint32_t *B, uint32_t *tile_tensor) {
    const uint64_t g = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    const uint64_t per = (uint64_t)sw.ntiles + 1;
    if (g >= per * sw.Q) return;
    const uint32_t q = (uint32_t)(g / per), t = (uint32_t)(g % per);
    const UpdDesc u = sw.U[q];
    if (t == sw.ntiles) {
        B[g] = (uint32_t)u.off[sw.L];
        return;
    }
    const uint32_t l = tile_layer(sw.P, sw.L, t);
    if (q == 0) tile_tensor[t] = l;
    const uint32_t c0 = (t - (uint32_t)sw.P[l].tile_base) << sw.tile_shift;
    // The kernel is bound by the length of its chain of dependent loads: BOUNDS_WAYS - 1 probes per round, loaded
    // together, cut the range into BOUNDS_WAYS parts, so log(n)/log(BOUNDS_WAYS) rounds instead of log2(n).
    uint64_t lo = u.off[l], hi = u.off[l + 1];  // the answer lies in [lo, hi]
    while (hi - lo >= BOUNDS_WAYS) {
        const uint64_t step = (hi - lo) / BOUNDS_WAYS;  // >= 1
        uint32_t v[BOUNDS_WAYS - 1];
#pragma unroll
        for (uint32_t j = 0; j < BOUNDS_WAYS - 1; ++j) v[j] = u.idx[lo + (j + 1) * step];  // positions < hi
        uint32_t below = 0;  // probes with a smaller index: a prefix of them when the list is sorted
#pragma unroll
        for (uint32_t j = 0; j < BOUNDS_WAYS - 1; ++j) below += v[j] < c0 ? 1u : 0u;
        const uint64_t base = lo;
        if (below) lo = base + below * step + 1;                       // idx[base + below * step] < c0
        if (below < BOUNDS_WAYS - 1) hi = base + (below + 1) * step;   // idx[that] >= c0
    }
    while (lo < hi) {
        const uint64_t mid = lo + ((hi - lo) >> 1);
        if (u.idx[mid] < c0) lo = mid + 1; else hi = mid;
    }
    B[g] = (uint32_t)lo;
}

// Slices of up to PASS consecutive updates (q0 ..) inside tile t, laid end to end.
struct Slices {
    uint32_t off[PASS + 1];      // position of the first entry of update q0+i; off[n] = entries
    uint32_t b0[PASS];           // its entry number inside the update
    const uint32_t *idx[PASS];   // the update's arrays
    const float *val[PASS];
    const uint32_t *pre[PASS];   // staleness accumulated before the call, per entry, or nullptr
    uint32_t tag[PASS];          // update number | staleness inside the call << 15 (key bits of its touches)
};

// The bounds of the calling thread's update in a tile, fetched by the kernel ahead of time for a
// queue of at most PASS updates (then thread q serves update q in every tile of the workgroup).
struct Fetched {
    bool valid;   // bounds are in b0 / b1
    bool first;   // first tile of the workgroup: the update's arrays are not yet in `sl`
    uint32_t b0, b1;
};

__device__ __forceinline__ uint32_t load_slices(const Sweep &sw, uint32_t t, uint32_t q0, Slices &sl,
                                                uint32_t *s_wave, const Fetched &f) {
    const uint32_t q = q0 + threadIdx.x;
    const bool mine = threadIdx.x < PASS && q < sw.Q;
    uint32_t b0 = 0, len = 0;
    if (mine) {
        uint32_t b1;
        if (f.valid) {
            b0 = f.b0;
            b1 = f.b1;
        } else {
            const uint32_t *row = sw.B + (uint64_t)q * (sw.ntiles + 1) + t;
            b0 = row[0];
            b1 = row[1];
        }
        len = b1 >= b0 ? b1 - b0 : 0u;  // bounds of an unsorted (malformed) list may cross
        if (!f.valid || f.first) {
            const UpdDesc u = sw.U[q];
            sl.idx[threadIdx.x] = u.idx;
            sl.val[threadIdx.x] = u.val;
            sl.pre[threadIdx.x] = u.pre;
            sl.tag[threadIdx.x] = q | ((q - u.pull) << 15);
        }
    }
    uint32_t total;
    const uint32_t o = block_exclusive_scan<WAVES>(len, s_wave, total);
    if (threadIdx.x <= PASS) sl.off[threadIdx.x] = o;  // off[n_slices .. PASS] = total
    if (mine) sl.b0[threadIdx.x] = b0;
    __syncthreads();
    return total;
}

// Update (relative to q0) that owns staged position p: the last i with off[i] <= p.
__device__ __forceinline__ uint32_t slice_of(const uint32_t *off, uint32_t n_slices, uint32_t p) {
    uint32_t lo = 0, hi = n_slices;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (off[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

constexpr uint32_t PER_THREAD = STAGE_CAP / BLOCK;  // staged entries per thread and pass

__device__ __forceinline__ uint32_t slot(uint32_t c) { return c + (c >> 4); }

// A touch in LDS: key = update number (15 bits) | staleness field (15 bits, from bit 15) |
// pulled-before-the-call (bit 30) | value-is-non-zero (bit 31); value separately.  The
// staleness field is q - pull for an update pulled inside the call; for one pulled earlier
// its window covers the whole call so far, and the field holds the staleness it had
// accumulated before the call.
__device__ __forceinline__ void sweep_tile(const Sweep &sw, const uint32_t t, const Fetched &fetched) {
    // per coordinate: count, then start, then end of its list; slot(c) skews the index so
    // that the scan's 16-consecutive-per-thread accesses fall into distinct banks
    __shared__ uint32_t s_cur[TILE_MAX + TILE_MAX / 16];
    __shared__ uint32_t s_key[STAGE_CAP];
    __shared__ float s_val[STAGE_CAP];
    __shared__ float s_prod[STAGE_CAP];      // alpha_k * value of every touch, per coordinate in time order
    __shared__ uint16_t s_coord[STAGE_CAP];  // coordinate (inside the tile) of every touch
    __shared__ Slices sl;
    __shared__ uint32_t s_wave[WAVES];
    __shared__ uint32_t s_bad;

    const uint32_t tid = threadIdx.x;
    const uint32_t tile = 1u << sw.tile_shift;
    const ParamDesc pd = sw.P[sw.tile_tensor[t]];
    const uint32_t c0 = (t - (uint32_t)pd.tile_base) << sw.tile_shift;
    // the scan over the tile's coordinates: per_thread consecutive ones per thread; a tile
    // smaller than the workgroup leaves the upper threads without any
    const uint32_t per_thread = tile >= BLOCK ? tile / BLOCK : 1u;
    const bool scans = tid * per_thread < tile;

    const uint32_t ncoord = pd.n - c0 < tile ? (uint32_t)(pd.n - c0) : tile;

    for (uint32_t c = tid; c < tile + tile / 16; c += BLOCK) s_cur[c] = 0;
    if (tid == 0) s_bad = 0;
    __syncthreads();

    // pass A: count the touches of every coordinate.  With a queue of at most PASS updates
    // there is one pass and the entries stay in registers for pass B.
    uint32_t c[PER_THREAD], key[PER_THREAD];
    float v[PER_THREAD];
    uint32_t total = 0;
    for (uint32_t q0 = 0; q0 < sw.Q; q0 += PASS) {
        const uint32_t n_pass = load_slices(sw, t, q0, sl, s_wave, fetched);
        const uint32_t n_slices = sw.Q - q0 < PASS ? sw.Q - q0 : PASS;
        total += n_pass;
        if (total > STAGE_CAP) break;  // uniform
#pragma unroll
        for (uint32_t j = 0; j < PER_THREAD; ++j) {  // all loads in flight together
            const uint32_t p = tid + j * BLOCK;
            c[j] = 0xffffffffu;
            if (p < n_pass) {
                const uint32_t i = slice_of(sl.off, n_slices, p);
                const uint32_t e = sl.b0[i] + (p - sl.off[i]);
                c[j] = sl.idx[i][e] - c0;
                v[j] = sl.val[i][e];
                key[j] = sl.tag[i];
                if (sl.pre[i]) {
                    const uint32_t before = sl.pre[i][e];
                    if (before > 0x7fffu) s_bad = 1;  // does not fit the key: leave the tile to the slow kernel
                    key[j] = (key[j] & 0x7fffu) | (before << 15) | 0x40000000u;
                }
            }
        }
#pragma unroll
        for (uint32_t j = 0; j < PER_THREAD; ++j) {
            if (tid + j * BLOCK >= n_pass) continue;
            if (c[j] >= ncoord) s_bad = 1;  // only a malformed (unsorted) index list gets here
            else atomicAdd(&s_cur[slot(c[j])], 1u);
        }
        __syncthreads();
    }
    if (total > STAGE_CAP || s_bad) {  // leave the tile untouched for the slow kernel
        if (tid == 0) sw.ovf[1 + atomicAdd(&sw.ovf[0], 1u)] = t;
        return;
    }
    if (total == 0) return;

    // counts -> list starts (exclusive scan, per_thread consecutive coordinates per thread)
    {
        uint32_t sum = 0;
        if (scans)
            for (uint32_t j = 0; j < per_thread; ++j) sum += s_cur[slot(tid * per_thread + j)];
        uint32_t all;
        uint32_t run = block_exclusive_scan<WAVES>(sum, s_wave, all);
        if (scans)
            for (uint32_t j = 0; j < per_thread; ++j) {
                const uint32_t n_touch = s_cur[slot(tid * per_thread + j)];
                s_cur[slot(tid * per_thread + j)] = run;
                run += n_touch;
            }
        __syncthreads();
    }

    // pass B: group the touches by coordinate (list order is arbitrary, time is in the key)
    for (uint32_t q0 = 0; q0 < sw.Q; q0 += PASS) {
        uint32_t n_pass = total;
        if (sw.Q > PASS) {  // several passes: fetch this pass's entries again (cache hits)
            n_pass = load_slices(sw, t, q0, sl, s_wave, fetched);
            const uint32_t n_slices = sw.Q - q0 < PASS ? sw.Q - q0 : PASS;
#pragma unroll
            for (uint32_t j = 0; j < PER_THREAD; ++j) {
                const uint32_t p = tid + j * BLOCK;
                if (p < n_pass) {
                    const uint32_t i = slice_of(sl.off, n_slices, p);
                    const uint32_t e = sl.b0[i] + (p - sl.off[i]);
                    c[j] = sl.idx[i][e] - c0;
                    v[j] = sl.val[i][e];
                    key[j] = sl.tag[i];
                    if (sl.pre[i]) key[j] = (key[j] & 0x7fffu) | (sl.pre[i][e] << 15) | 0x40000000u;
                }
            }
        }
#pragma unroll
        for (uint32_t j = 0; j < PER_THREAD; ++j) {
            if (tid + j * BLOCK >= n_pass) continue;
            const uint32_t pos = atomicAdd(&s_cur[slot(c[j])], 1u);
            s_key[pos] = key[j] | (is_nonzero(v[j]) ? 0x80000000u : 0u);
            s_val[pos] = v[j];
            s_coord[pos] = (uint16_t)c[j];
        }
        __syncthreads();
    }

    // per touch (dense over the lists, PER_THREAD touches per thread): its rank in time among
    // the touches of its coordinate, its staleness sigma (eq. 3 on the coordinate's own list),
    // and the product alpha_k * value (eq. 5 and the multiply of eq. 4), stored in time order.
    // The earliest touch of a coordinate also fetches Theta_k and will fold the list.
    float theta[PER_THREAD];
    uint32_t lo[PER_THREAD], hi[PER_THREAD], coord[PER_THREAD];
#pragma unroll
    for (uint32_t j = 0; j < PER_THREAD; ++j) {
        const uint32_t x = tid + j * BLOCK;
        lo[j] = hi[j] = 0;
        if (x >= total) continue;
        const uint32_t kx = s_key[x], cx = s_coord[x];
        const uint32_t qx = kx & 0x7fffu;
        const bool earlier = (kx >> 30) & 1u;  // pulled before the call
        const uint32_t field = (kx >> 15) & 0x7fffu;
        const uint32_t pull = earlier ? 0u : qx - field;
        const uint32_t beg = cx ? s_cur[slot(cx - 1)] : 0u, end = s_cur[slot(cx)];
        uint32_t rank = 0, sigma = earlier ? field : 0u;
        for (uint32_t y = beg; y < end; ++y) {
            const uint32_t ky = s_key[y];
            const uint32_t qy = ky & 0x7fffu;
            rank += qy < qx;
            sigma += (ky >> 31) & (uint32_t)(qy >= pull && qy < qx);
        }
        float alpha = sw.lr;
        if (sigma != 0) alpha = __fdiv_rn(sw.lr, (float)sigma);
        s_prod[beg + rank] = __fmul_rn(alpha, s_val[x]);
        if (rank == 0) {
            lo[j] = beg;
            hi[j] = end;
            coord[j] = cx;
            theta[j] = pd.theta[c0 + cx];
        }
    }
    __syncthreads();

    // per coordinate: subtract its products in time order (eq. 4)
#pragma unroll
    for (uint32_t j = 0; j < PER_THREAD; ++j) {
        if (hi[j] <= lo[j]) continue;
        float th = theta[j];
        for (uint32_t m = lo[j]; m < hi[j]; ++m) th = __fsub_rn(th, s_prod[m]);
        pd.theta[c0 + coord[j]] = th;
    }
}

// A workgroup takes TPB consecutive tiles, one after the other.  A tile is a few microseconds
// of work behind a chain of dependent loads (bounds -> entries -> parameters); with a queue
// of at most PASS updates thread q fetches the bounds of update q for all TPB tiles at once
// (they are neighbours in memory) and the update's descriptor once, which takes the first
// link of the chain off all tiles but the first.
template <uint32_t TPB>
__global__ __launch_bounds__(BLOCK) void k_sweep(Sweep sw) {
    const uint32_t t0 = blockIdx.x * TPB;
    const bool ahead = sw.Q <= PASS;
    uint32_t row[TPB + 1];
    if (ahead && threadIdx.x < sw.Q) {
        const uint32_t *b = sw.B + (uint64_t)threadIdx.x * (sw.ntiles + 1) + t0;
#pragma unroll
        for (uint32_t i = 0; i <= TPB; ++i) row[i] = t0 + i <= sw.ntiles ? b[i] : 0u;
    }
#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) {
        const uint32_t t = t0 + i;
        if (t >= sw.ntiles) return;
        sweep_tile(sw, t, Fetched{ahead, i == 0, row[i], row[i + 1]});
        __syncthreads();  // the next tile reuses the LDS arrays
    }
}

// The same sweep for queues of at most PASS_SHORT updates, arranged so that the chain of
// dependent loads (bounds -> entries -> parameters) is paid once per workgroup instead of
// once per tile: wave 0 fetches the bounds of every update in all TPB tiles and scans them
// with lane shuffles; then every thread requests its entries of all TPB tiles together, then
// the parameters those entries touch; only then the tiles are sorted and replayed one after
// the other out of registers and LDS.
template <uint32_t TPB>
__global__ __launch_bounds__(BLOCK) void k_sweep_short(Sweep sw) {
    constexpr uint32_t QS = PASS_SHORT;
    __shared__ uint32_t s_cur[TILE_MAX + TILE_MAX / 16];
    __shared__ uint32_t s_key[STAGE_CAP];
    __shared__ float s_val[STAGE_CAP];
    __shared__ float s_theta[STAGE_CAP];     // Theta of the touch's coordinate, as fetched ahead
    __shared__ float s_prod[STAGE_CAP];
    __shared__ uint16_t s_coord[STAGE_CAP];
    __shared__ const uint32_t *s_idx[QS];
    __shared__ const float *s_valp[QS];
    __shared__ const uint32_t *s_pre[QS];
    __shared__ uint32_t s_tag[QS];
    static_assert(QS == WAVE, "wave 0 serves one update per lane");
    __shared__ uint32_t s_off[TPB][QS + 1];  // per tile: staged position of the first entry of update q; [Q..QS] = entries
    __shared__ uint32_t s_b0[TPB][QS];
    __shared__ uint32_t s_wave[WAVES];
    __shared__ uint32_t s_bad[TPB];

    const uint32_t tid = threadIdx.x, t0 = blockIdx.x * TPB;
    const uint32_t tile = 1u << sw.tile_shift;
    const uint32_t per_thread = tile >= BLOCK ? tile / BLOCK : 1u;
    const bool scans = tid * per_thread < tile;

    // the tiles' tensors (independent of the bounds: both requests are in flight together)
    uint32_t tensor[TPB];
#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) tensor[i] = t0 + i < sw.ntiles ? sw.tile_tensor[t0 + i] : 0u;

    if (tid < WAVE) {  // wave 0: bounds, their scans, the updates' arrays
        const bool mine = tid < sw.Q;
        uint32_t row[TPB + 1];
        if (mine) {
            const uint32_t *b = sw.B + (uint64_t)tid * (sw.ntiles + 1) + t0;
#pragma unroll
            for (uint32_t i = 0; i <= TPB; ++i) row[i] = t0 + i <= sw.ntiles ? b[i] : 0u;
            const UpdDesc u = sw.U[tid];
            s_idx[tid] = u.idx;
            s_valp[tid] = u.val;
            s_pre[tid] = u.pre;
            s_tag[tid] = tid | ((tid - u.pull) << 15);
        }
#pragma unroll
        for (uint32_t i = 0; i < TPB; ++i) {
            // bounds of an unsorted (malformed) list may cross
            const uint32_t len = (mine && t0 + i < sw.ntiles && row[i + 1] >= row[i]) ? row[i + 1] - row[i] : 0u;
            uint32_t incl = len;
#pragma unroll
            for (int d = 1; d < WAVE; d <<= 1) {
                const uint32_t y = __shfl_up(incl, d);
                if (tid >= (uint32_t)d) incl += y;
            }
            s_off[i][tid] = incl - len;  // lanes at or beyond Q hold the total
            if (tid == WAVE - 1) s_off[i][QS] = incl;
            if (mine) s_b0[i][tid] = row[i];
        }
    }
    if (tid < TPB) s_bad[tid] = 0;
    __syncthreads();

    float *theta_of[TPB];  // first parameter of the tile
    uint32_t c0[TPB], ncoord[TPB], total[TPB];
#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) {
        const ParamDesc pd = sw.P[tensor[i]];
        c0[i] = (t0 + i - (uint32_t)pd.tile_base) << sw.tile_shift;
        ncoord[i] = pd.n - c0[i] < tile ? (uint32_t)(pd.n - c0[i]) : tile;
        theta_of[i] = pd.theta + c0[i];
        total[i] = s_off[i][QS];
    }

    // every entry of every tile of the workgroup: requested together
    uint32_t c[TPB][PER_THREAD], key[TPB][PER_THREAD];
    float v[TPB][PER_THREAD], th[TPB][PER_THREAD];
#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) {
#pragma unroll
        for (uint32_t j = 0; j < PER_THREAD; ++j) {
            const uint32_t p = tid + j * BLOCK;
            c[i][j] = 0xffffffffu;
            v[i][j] = 0.f;
            key[i][j] = 0;
            if (total[i] <= STAGE_CAP && p < total[i]) {
                const uint32_t u = slice_of(s_off[i], sw.Q, p);
                const uint32_t e = s_b0[i][u] + (p - s_off[i][u]);
                c[i][j] = s_idx[u][e] - c0[i];
                v[i][j] = s_valp[u][e];
                key[i][j] = s_tag[u];
                if (s_pre[u]) {
                    const uint32_t before = s_pre[u][e];
                    if (before > 0x7fffu) s_bad[i] = 1;  // does not fit the key: leave the tile to the slow kernel
                    key[i][j] = (key[i][j] & 0x7fffu) | (before << 15) | 0x40000000u;
                }
            }
        }
    }
    // the parameters they touch: requested together as well
#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) {
#pragma unroll
        for (uint32_t j = 0; j < PER_THREAD; ++j) {
            th[i][j] = 0.f;
            if (c[i][j] < ncoord[i]) th[i][j] = theta_of[i][c[i][j]];
        }
    }

#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) {
        if (t0 + i >= sw.ntiles || total[i] == 0) continue;  // uniform
        for (uint32_t x = tid; x < tile + tile / 16; x += BLOCK) s_cur[x] = 0;
        __syncthreads();
        if (total[i] <= STAGE_CAP) {
#pragma unroll
            for (uint32_t j = 0; j < PER_THREAD; ++j) {
                if (tid + j * BLOCK >= total[i]) continue;
                if (c[i][j] >= ncoord[i]) s_bad[i] = 1;  // only a malformed (unsorted) index list gets here
                else atomicAdd(&s_cur[slot(c[i][j])], 1u);
            }
        }
        __syncthreads();
        if (total[i] > STAGE_CAP || s_bad[i]) {  // leave the tile untouched for the slow kernel
            if (tid == 0) sw.ovf[1 + atomicAdd(&sw.ovf[0], 1u)] = t0 + i;
            continue;
        }
        {  // counts -> list starts
            uint32_t sum = 0;
            if (scans)
                for (uint32_t j = 0; j < per_thread; ++j) sum += s_cur[slot(tid * per_thread + j)];
            uint32_t all;
            uint32_t run = block_exclusive_scan<WAVES>(sum, s_wave, all);
            if (scans)
                for (uint32_t j = 0; j < per_thread; ++j) {
                    const uint32_t n_touch = s_cur[slot(tid * per_thread + j)];
                    s_cur[slot(tid * per_thread + j)] = run;
                    run += n_touch;
                }
            __syncthreads();
        }
#pragma unroll
        for (uint32_t j = 0; j < PER_THREAD; ++j) {  // group the touches by coordinate
            if (tid + j * BLOCK >= total[i]) continue;
            const uint32_t pos = atomicAdd(&s_cur[slot(c[i][j])], 1u);
            s_key[pos] = key[i][j] | (is_nonzero(v[i][j]) ? 0x80000000u : 0u);
            s_val[pos] = v[i][j];
            s_theta[pos] = th[i][j];
            s_coord[pos] = (uint16_t)c[i][j];
        }
        __syncthreads();
        // per touch: rank in time, sigma (eq. 3), alpha_k * value (eq. 5 and the multiply of eq. 4)
        float theta[PER_THREAD];
        uint32_t lo[PER_THREAD], hi[PER_THREAD], coord[PER_THREAD];
#pragma unroll
        for (uint32_t j = 0; j < PER_THREAD; ++j) {
            const uint32_t x = tid + j * BLOCK;
            lo[j] = hi[j] = 0;
            if (x >= total[i]) continue;
            const uint32_t kx = s_key[x], cx = s_coord[x];
            const uint32_t qx = kx & 0x7fffu;
            const bool earlier = (kx >> 30) & 1u;
            const uint32_t field = (kx >> 15) & 0x7fffu;
            const uint32_t pull = earlier ? 0u : qx - field;
            const uint32_t beg = cx ? s_cur[slot(cx - 1)] : 0u, end = s_cur[slot(cx)];
            uint32_t rank = 0, sigma = earlier ? field : 0u;
            for (uint32_t y = beg; y < end; ++y) {
                const uint32_t ky = s_key[y];
                const uint32_t qy = ky & 0x7fffu;
                rank += qy < qx;
                sigma += (ky >> 31) & (uint32_t)(qy >= pull && qy < qx);
            }
            float alpha = sw.lr;
            if (sigma != 0) alpha = __fdiv_rn(sw.lr, (float)sigma);
            s_prod[beg + rank] = __fmul_rn(alpha, s_val[x]);
            if (rank == 0) {  // every touch of a coordinate fetched the same Theta; the earliest one folds
                lo[j] = beg;
                hi[j] = end;
                coord[j] = cx;
                theta[j] = s_theta[x];
            }
        }
        __syncthreads();
#pragma unroll
        for (uint32_t j = 0; j < PER_THREAD; ++j) {  // eq. 4, in time order
            if (hi[j] <= lo[j]) continue;
            float t_k = theta[j];
            for (uint32_t m = lo[j]; m < hi[j]; ++m) t_k = __fsub_rn(t_k, s_prod[m]);
            theta_of[i][coord[j]] = t_k;
        }
        __syncthreads();  // the next tile reuses the LDS arrays
    }
}

// The sweep for sparse queues of at most PASS_SHORT updates: most parameters that the queue
// touches at all are touched once (16 workers at 0.5 %: 93 % of them), and such a touch needs no
// list, no rank and no sorting: sigma_k counts earlier touches of k (eq. 3) and there are none,
// so the step is Theta_k - alpha * v straight from the registers that hold the entry.  Which
// touches are alone is read off two bitmaps over the tile's coordinates (touched at all / touched
// at least twice), filled with LDS atomics.  Only the entries of coordinates touched twice or more
// are grouped: the coordinate's number among those coordinates is a population count over the
// second bitmap, so the counting sort runs over a few dozen slots instead of the tile's thousands.
// A workgroup takes TPB consecutive tiles of up to TILE_MAX_SPARSE coordinates: wave 0 fetches
// the bounds of every update in all of them, then every thread requests its entries of all TPB
// tiles together, then the parameters they name (the chain bounds -> entries -> parameters is paid
// once per workgroup), and only then the tiles are worked through one after the other.  A tile
// with more than SP_CAP queued entries or SP_MULTI entries on shared coordinates is left untouched
// for the kernel for overflowing tiles.
constexpr uint32_t SP_PER = 3;                 // entries per thread and tile
constexpr uint32_t SP_CAP = BLOCK * SP_PER;    // entries per tile
constexpr uint32_t SP_MULTI = 512;             // entries on coordinates touched more than once
constexpr uint32_t SP_WORDS = TILE_MAX_SPARSE / 32;
static_assert(SP_WORDS <= BLOCK && SP_MULTI % BLOCK == 0 && SP_MULTI / 2 <= BLOCK,
              "one bitmap word, two list slots, one shared coordinate per thread");

template <uint32_t TPB>
__global__ __launch_bounds__(BLOCK) void k_sweep_sparse(Sweep sw) {
    constexpr uint32_t QS = PASS_SHORT;
    __shared__ uint32_t s_b1[SP_WORDS], s_b2[SP_WORDS];  // coordinate touched / touched at least twice
    __shared__ uint32_t s_pref[SP_WORDS];                // coordinates with the second bit set before this word
    __shared__ uint32_t s_start[SP_MULTI / 2 + 1];       // per shared coordinate: count, then start of its list
    __shared__ uint32_t s_fill[SP_MULTI / 2];
    __shared__ uint32_t s_key[SP_MULTI];
    __shared__ float s_val[SP_MULTI], s_theta[SP_MULTI], s_prod[SP_MULTI];
    __shared__ uint16_t s_coord[SP_MULTI], s_slot[SP_MULTI];
    __shared__ const uint32_t *s_idx[QS];
    __shared__ const float *s_valp[QS];
    __shared__ const uint32_t *s_pre[QS];
    __shared__ uint32_t s_tag[QS];
    __shared__ uint32_t s_off[TPB][QS + 1];  // per tile: staged position of the first entry of update q; [Q..QS] = entries
    __shared__ uint32_t s_b0[TPB][QS];
    __shared__ uint32_t s_wave[WAVES];
    __shared__ uint32_t s_bad[TPB];
    static_assert(QS == WAVE, "wave 0 serves one update per lane");

    const uint32_t tid = threadIdx.x, t0 = blockIdx.x * TPB;
    const uint32_t tile = 1u << sw.tile_shift;
    uint32_t tensor[TPB];
#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) tensor[i] = t0 + i < sw.ntiles ? sw.tile_tensor[t0 + i] : 0u;
    if (tid < WAVE) {  // wave 0: the slices of every update in the TPB tiles, their scans, the updates' arrays
        const bool mine = tid < sw.Q;
        uint32_t row[TPB + 1];
        if (mine) {
            const uint32_t *b = sw.B + (uint64_t)tid * (sw.ntiles + 1) + t0;
#pragma unroll
            for (uint32_t i = 0; i <= TPB; ++i) row[i] = t0 + i <= sw.ntiles ? b[i] : 0u;
            const UpdDesc u = sw.U[tid];
            s_idx[tid] = u.idx;
            s_valp[tid] = u.val;
            s_pre[tid] = u.pre;
            s_tag[tid] = tid | ((tid - u.pull) << 15);
        }
#pragma unroll
        for (uint32_t i = 0; i < TPB; ++i) {
            // bounds of an unsorted (malformed) list may cross
            const uint32_t len = (mine && t0 + i < sw.ntiles && row[i + 1] >= row[i]) ? row[i + 1] - row[i] : 0u;
            uint32_t incl = len;
#pragma unroll
            for (int d = 1; d < WAVE; d <<= 1) {
                const uint32_t y = __shfl_up(incl, d);
                if (tid >= (uint32_t)d) incl += y;
            }
            s_off[i][tid] = incl - len;  // lanes at or beyond Q hold the total
            if (tid == WAVE - 1) s_off[i][QS] = incl;
            if (mine) s_b0[i][tid] = row[i];
        }
    }
    if (tid < TPB) s_bad[tid] = 0;
    __syncthreads();

    float *theta_of[TPB];  // first parameter of the tile
    uint32_t c0[TPB], ncoord[TPB], total[TPB];
#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) {
        const ParamDesc pd = sw.P[tensor[i]];
        c0[i] = (t0 + i - (uint32_t)pd.tile_base) << sw.tile_shift;
        ncoord[i] = pd.n - c0[i] < tile ? (uint32_t)(pd.n - c0[i]) : tile;
        theta_of[i] = pd.theta + c0[i];
        total[i] = t0 + i < sw.ntiles ? s_off[i][QS] : 0u;
    }
    // every entry of every tile of the workgroup, then the parameters they name: two rounds of requests
    uint32_t c[TPB][SP_PER], key[TPB][SP_PER];
    float v[TPB][SP_PER], th[TPB][SP_PER];
#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) {
#pragma unroll
        for (uint32_t j = 0; j < SP_PER; ++j) {
            const uint32_t p = tid + j * BLOCK;
            c[i][j] = 0xffffffffu;
            v[i][j] = 0.f;
            key[i][j] = 0;
            if (total[i] <= SP_CAP && p < total[i]) {
                const uint32_t u = slice_of(s_off[i], sw.Q, p);
                const uint32_t e = s_b0[i][u] + (p - s_off[i][u]);
                c[i][j] = s_idx[u][e] - c0[i];
                v[i][j] = s_valp[u][e];
                key[i][j] = s_tag[u];
                if (s_pre[u]) {
                    const uint32_t before = s_pre[u][e];
                    if (before > 0x7fffu) s_bad[i] = 1;  // does not fit the key
                    key[i][j] = (key[i][j] & 0x7fffu) | (before << 15) | 0x40000000u;
                }
                if (c[i][j] >= ncoord[i]) s_bad[i] = 1;  // only a malformed (unsorted) index list gets here
            }
        }
    }
#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) {
#pragma unroll
        for (uint32_t j = 0; j < SP_PER; ++j) {
            th[i][j] = 0.f;
            if (c[i][j] < ncoord[i]) th[i][j] = theta_of[i][c[i][j]];
        }
    }

#pragma unroll
    for (uint32_t i = 0; i < TPB; ++i) {
        if (total[i] == 0) continue;  // uniform
        if (total[i] > SP_CAP) {      // uniform: leave the tile untouched for the kernel for overflowing tiles
            if (tid == 0) sw.ovf[1 + atomicAdd(&sw.ovf[0], 1u)] = t0 + i;
            continue;
        }
        __syncthreads();  // the previous tile is done with the LDS arrays
        if (tid < SP_WORDS) {
            s_b1[tid] = 0;
            s_b2[tid] = 0;
        }
        for (uint32_t x = tid; x < SP_MULTI / 2; x += BLOCK) {
            s_start[x] = 0;
            s_fill[x] = 0;
        }
        __syncthreads();
#pragma unroll
        for (uint32_t j = 0; j < SP_PER; ++j) {
            if (c[i][j] < ncoord[i]) {
                const uint32_t bit = 1u << (c[i][j] & 31u);
                if (atomicOr(&s_b1[c[i][j] >> 5], bit) & bit) atomicOr(&s_b2[c[i][j] >> 5], bit);
            }
        }
        __syncthreads();
        // shared coordinates numbered in coordinate order: prefix population count of the second bitmap
        uint32_t shared_all;
        {
            const uint32_t mine = tid < SP_WORDS ? (uint32_t)__popc(s_b2[tid]) : 0u;
            const uint32_t before = block_exclusive_scan<WAVES>(mine, s_wave, shared_all);
            if (tid < SP_WORDS) s_pref[tid] = before;
        }
        __syncthreads();
        if (s_bad[i] || shared_all > SP_MULTI / 2) {  // uniform
            if (tid == 0) sw.ovf[1 + atomicAdd(&sw.ovf[0], 1u)] = t0 + i;
            continue;
        }
        // the entries on shared coordinates are counted per coordinate; nothing is stored before the
        // tile is known to fit, so that a tile left to the other kernel is found untouched
        uint32_t slot[SP_PER];
#pragma unroll
        for (uint32_t j = 0; j < SP_PER; ++j) {
            slot[j] = 0xffffffffu;
            if (c[i][j] >= ncoord[i]) continue;
            const uint32_t w = c[i][j] >> 5, bit = 1u << (c[i][j] & 31u);
            const uint32_t twice = s_b2[w];
            if (twice & bit) {
                slot[j] = s_pref[w] + (uint32_t)__popc(twice & (bit - 1u));
                atomicAdd(&s_start[slot[j]], 1u);
            }
        }
        uint32_t multi = 0;  // entries on shared coordinates
        if (shared_all) {    // uniform
            __syncthreads();
            const uint32_t n_touch = tid < shared_all ? s_start[tid] : 0u;
            const uint32_t before = block_exclusive_scan<WAVES>(n_touch, s_wave, multi);  // counts -> list starts
            if (tid < shared_all) s_start[tid] = before;
            if (tid == 0) s_start[shared_all] = multi;
            __syncthreads();
            if (multi > SP_MULTI) {  // uniform
                if (tid == 0) sw.ovf[1 + atomicAdd(&sw.ovf[0], 1u)] = t0 + i;
                continue;
            }
        }
#pragma unroll
        for (uint32_t j = 0; j < SP_PER; ++j) {
            if (c[i][j] >= ncoord[i]) continue;
            if (slot[j] == 0xffffffffu) {
                // a touch that is alone on its coordinate: eqs. 3-5 on the spot
                const bool earlier = (key[i][j] >> 30) & 1u;
                const uint32_t sigma = earlier ? (key[i][j] >> 15) & 0x7fffu : 0u;  // what it had accumulated before the call
                theta_of[i][c[i][j]] = step(th[i][j], sw.lr, sigma, v[i][j]);
            } else {
                const uint32_t pos = s_start[slot[j]] + atomicAdd(&s_fill[slot[j]], 1u);
                s_key[pos] = key[i][j] | (is_nonzero(v[i][j]) ? 0x80000000u : 0u);
                s_val[pos] = v[i][j];
                s_theta[pos] = th[i][j];
                s_coord[pos] = (uint16_t)c[i][j];
                s_slot[pos] = (uint16_t)slot[j];
            }
        }
        if (multi == 0) continue;  // uniform
        __syncthreads();
        // per touch on a shared coordinate: rank in time, sigma (eq. 3), alpha_k * value (eq. 5 and the multiply of eq. 4)
        constexpr uint32_t MP = SP_MULTI / BLOCK;
        float theta[MP];
        uint32_t lo[MP], hi[MP], coord[MP];
#pragma unroll
        for (uint32_t j = 0; j < MP; ++j) {
            const uint32_t x = tid + j * BLOCK;
            lo[j] = hi[j] = 0;
            if (x >= multi) continue;
            const uint32_t kx = s_key[x], sx = s_slot[x];
            const uint32_t qx = kx & 0x7fffu;
            const bool earlier = (kx >> 30) & 1u;
            const uint32_t field = (kx >> 15) & 0x7fffu;
            const uint32_t pull = earlier ? 0u : qx - field;
            const uint32_t beg = s_start[sx], end = s_start[sx + 1];
            uint32_t rank = 0, sigma = earlier ? field : 0u;
            for (uint32_t y = beg; y < end; ++y) {
                const uint32_t ky = s_key[y];
                const uint32_t qy = ky & 0x7fffu;
                rank += qy < qx;
                sigma += (ky >> 31) & (uint32_t)(qy >= pull && qy < qx);
            }
            float alpha = sw.lr;
            if (sigma != 0) alpha = __fdiv_rn(sw.lr, (float)sigma);
            s_prod[beg + rank] = __fmul_rn(alpha, s_val[x]);
            if (rank == 0) {  // every touch of a coordinate fetched the same Theta; the earliest one folds
                lo[j] = beg;
                hi[j] = end;
                coord[j] = s_coord[x];
                theta[j] = s_theta[x];
            }
        }
        __syncthreads();
#pragma unroll
        for (uint32_t j = 0; j < MP; ++j) {  // eq. 4, in time order
            if (hi[j] <= lo[j]) continue;
            float t_k = theta[j];
            for (uint32_t m = lo[j]; m < hi[j]; ++m) t_k = __fsub_rn(t_k, s_prod[m]);
            theta_of[i][coord[j]] = t_k;
        }
    }
}

// The sweep for dense queues (about one queued entry per parameter or more).  There the lists
// of a coordinate need no sorting: a tile is DTILE consecutive coordinates, thread c owns
// coordinate c with Theta_c in a register, and the queue passes through LDS DQ updates at a
// time as a dense [update][coordinate] array of values plus one presence word per coordinate.
// The owner replays its touches in time order.  Its non-zero touches so far are one bit per
// update in Z, so eq. 3 for a touch by update q pulled at j is a population count of Z over
// the bits j .. q-1 (plus what the update had accumulated before the call).  alpha / sigma
// comes from a table built with the same correctly rounded divide as everywhere else.
// Queues of at most 64 * NW updates.  A slice of a sorted list inside a tile has at most DTILE
// entries; what a malformed list adds beyond that, or outside the tile, is skipped.
constexpr uint32_t DTILE = BLOCK;
constexpr uint32_t DTILE_SHIFT = 8;
static_assert(DTILE == 1u << DTILE_SHIFT, "dense sweep: one thread per coordinate of a tile");

typedef const __attribute__((address_space(1))) uint32_t *global_u32;
typedef const __attribute__((address_space(1))) float *global_f32;

template <uint32_t NW, uint32_t DQ, bool PRE>
__global__ __launch_bounds__(BLOCK) void k_sweep_dense(Sweep sw) {
    constexpr uint32_t QMAX = 64 * NW;
    constexpr uint32_t PER_WAVE = DQ / WAVES;
    static_assert(DQ <= 32 && DQ % WAVES == 0 && QMAX <= BLOCK, "presence bits fit a word; thread q serves update q");
    __shared__ float s_v[DQ][DTILE];
    __shared__ uint32_t s_pr[PRE ? DQ : 1][DTILE];
    __shared__ uint32_t s_p[DTILE];
    __shared__ const uint32_t *s_idx[QMAX];
    __shared__ const float *s_valp[QMAX];
    __shared__ const uint32_t *s_pre[QMAX];
    __shared__ uint32_t s_b0[QMAX], s_len[QMAX], s_pull[QMAX];
    __shared__ float s_alpha[QMAX];

    const uint32_t tid = threadIdx.x, t = blockIdx.x;
    const uint32_t lane = tid & (WAVE - 1);
    const uint32_t wv = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const ParamDesc pd = sw.P[sw.tile_tensor[t]];
    const uint32_t c0 = (t - (uint32_t)pd.tile_base) << DTILE_SHIFT;
    const uint32_t ncoord = pd.n - c0 < DTILE ? (uint32_t)(pd.n - c0) : DTILE;
    float th = 0.f;
    if (tid < ncoord) th = pd.theta[c0 + tid];
    if (tid < sw.Q) {
        const uint32_t *row = sw.B + (uint64_t)tid * (sw.ntiles + 1) + t;
        const uint32_t b0 = row[0], b1 = row[1];
        const UpdDesc u = sw.U[tid];
        s_b0[tid] = b0;
        const uint32_t len = b1 >= b0 ? b1 - b0 : 0u;  // bounds of an unsorted (malformed) list may cross
        s_len[tid] = len < DTILE ? len : DTILE;
        s_idx[tid] = u.idx;
        s_valp[tid] = u.val;
        s_pre[tid] = u.pre;
        s_pull[tid] = u.pull;
    }
    for (uint32_t x = tid; x < QMAX; x += BLOCK) s_alpha[x] = x ? __fdiv_rn(sw.lr, (float)x) : sw.lr;
    s_p[tid] = 0;

    uint64_t Z[NW];  // bit q: update q touched this coordinate with a non-zero value
#pragma unroll
    for (uint32_t w = 0; w < NW; ++w) Z[w] = 0;
    bool touched = false;

    // A group of up to 64 consecutive updates: the first 64 entries of each slice go to
    // registers in one round of requests (wave w: updates g0 + w, g0 + w + WAVES, ...), then the
    // group passes through LDS DQ updates at a time.
    constexpr uint32_t GROUP = 64, GW = GROUP / WAVES, PASSES = GROUP / DQ;
    static_assert(GW == PASSES * PER_WAVE, "a wave's slices of a group, pass by pass");
    __syncthreads();  // tables ready
    for (uint32_t g0 = 0; g0 < sw.Q; g0 += GROUP) {
        uint32_t k[GW], pr[GW];
        float v[GW];
        uint32_t have = 0;
#pragma unroll
        for (uint32_t j = 0; j < GW; ++j) {
            // register j: pass j / PER_WAVE, slice wv + (j % PER_WAVE) * WAVES of that pass
            const uint32_t q = g0 + (j / PER_WAVE) * DQ + wv + (j % PER_WAVE) * WAVES;
            k[j] = 0;
            v[j] = 0.f;
            pr[j] = 0;
            if (q < sw.Q && lane < s_len[q]) {
                have |= 1u << j;
                const uint32_t e = s_b0[q] + lane;
                k[j] = ((global_u32)s_idx[q])[e];
                v[j] = ((global_f32)s_valp[q])[e];
                if (PRE && s_pre[q]) pr[j] = ((global_u32)s_pre[q])[e];
            }
        }
#pragma unroll
        for (uint32_t p = 0; p < PASSES; ++p) {
            const uint32_t q0 = g0 + p * DQ;
            if (q0 >= sw.Q) break;  // uniform
            const uint32_t nq = sw.Q - q0 < DQ ? sw.Q - q0 : DQ;
            if (p || g0) __syncthreads();  // the previous pass has been replayed
#pragma unroll
            for (uint32_t jj = 0; jj < PER_WAVE; ++jj) {
                const uint32_t j = p * PER_WAVE + jj, ql = wv + jj * WAVES;
                const uint32_t c = k[j] - c0;
                if (((have >> j) & 1u) && c < ncoord) {
                    s_v[ql][c] = v[j];
                    if (PRE) s_pr[ql][c] = pr[j];
                    atomicOr(&s_p[c], 1u << ql);
                }
            }
            for (uint32_t ql = wv; ql < nq; ql += WAVES) {  // slices longer than a wavefront
                const uint32_t len = s_len[q0 + ql], b0 = s_b0[q0 + ql];
                for (uint32_t i = WAVE + lane; i < len; i += WAVE) {
                    const uint32_t e = b0 + i;
                    const uint32_t c = ((global_u32)s_idx[q0 + ql])[e] - c0;
                    if (c >= ncoord) continue;
                    s_v[ql][c] = ((global_f32)s_valp[q0 + ql])[e];
                    if (PRE) s_pr[ql][c] = s_pre[q0 + ql] ? ((global_u32)s_pre[q0 + ql])[e] : 0u;
                    atomicOr(&s_p[c], 1u << ql);
                }
            }
            __syncthreads();
            // replay: the touches of coordinate `tid` by the updates of this pass, in time order
            uint32_t pm = s_p[tid];
            s_p[tid] = 0;
            touched |= pm != 0;
            while (pm) {
                const uint32_t ql = (uint32_t)__builtin_ctz(pm);
                pm &= pm - 1;
                const uint32_t q = q0 + ql;
                const float val = s_v[ql][tid];
                const uint32_t pull = s_pull[q];
                uint32_t sigma = PRE ? s_pr[ql][tid] : 0u;
#pragma unroll
                for (uint32_t w = 0; w < NW; ++w) {  // bits pull .. q-1 of Z, word by word
                    const uint32_t base = 64 * w;
                    const uint32_t lo = pull > base ? pull - base : 0u;
                    const uint32_t hi = q > base ? (q - base < 64u ? q - base : 64u) : 0u;
                    if (hi > lo) {
                        const uint64_t upto = hi == 64u ? ~0ull : (1ull << hi) - 1ull;
                        sigma += popc64(Z[w] & upto & ~((1ull << lo) - 1ull));
                    }
                }
                const float alpha = sigma < QMAX ? s_alpha[sigma] : __fdiv_rn(sw.lr, (float)sigma);
                th = __fsub_rn(th, __fmul_rn(alpha, val));
                if (is_nonzero(val)) {
#pragma unroll
                    for (uint32_t w = 0; w < NW; ++w)
                        if ((q >> 6) == w) Z[w] |= 1ull << (q & 63u);
                }
            }
        }
    }
    if (touched) pd.theta[c0 + tid] = th;
}

// Tiles the fast kernel declined: update by update from global memory, one workgroup per
// tile, with the snapshot scheme of the scatter plan restricted to the tile.
__global__ __launch_bounds__(BLOCK) void k_sweep_slow(Sweep sw) {
    const uint32_t n_ovf = sw.ovf[0];
    for (uint32_t o = blockIdx.x; o < n_ovf; o += gridDim.x) {
        const uint32_t t = sw.ovf[1 + o];
        const ParamDesc pd = sw.P[sw.tile_tensor[t]];
        for (uint32_t q = 0; q < sw.Q; ++q) {
            for (uint32_t a = sw.pa_off[q]; a < sw.pa_off[q + 1]; ++a) {
                const UpdDesc u = sw.U[sw.pa_list[a]];
                const uint32_t *row = sw.B + (uint64_t)sw.pa_list[a] * (sw.ntiles + 1) + t;
                for (uint32_t e = row[0] + threadIdx.x; e < row[1]; e += BLOCK) {
                    const uint32_t k = u.idx[e];
                    if (k < pd.n) u.snap[e] = pd.cnt[k];
                }
            }
            __syncthreads();
            const UpdDesc u = sw.U[q];
            const uint32_t *row = sw.B + (uint64_t)q * (sw.ntiles + 1) + t;
            const bool stale = q - u.pull >= (u.pre ? 1u : 2u);  // has a snapshot (host: same rule)
            for (uint32_t e = row[0] + threadIdx.x; e < row[1]; e += BLOCK) {
                const uint32_t k = u.idx[e];
                if (k >= pd.n) continue;
                const float v = u.val[e];
                const uint32_t c = pd.cnt[k];
                const uint32_t sigma = (stale ? c - u.snap[e] : 0u) + (u.pre ? u.pre[e] : 0u);
                pd.theta[k] = step(pd.theta[k], sw.lr, sigma, v);
                if (is_nonzero(v)) pd.cnt[k] = c + 1;
            }
            __syncthreads();
        }
    }
}

// Tiles the sorting kernels declined, for queues of at most 64 updates: where the same rows are
// large in every worker's gradient, a tile holds thousands of queued entries.  The tile's
// parameters stay in LDS while the queue is replayed update by update; sigma_k is a population
// count over the coordinate's mask of non-zero touches, as in the kernel for dense queues, so no
// counters and no snapshots are read or written.  The first 256 entries of the next update's
// slice are requested before the current update is applied.
__global__ __launch_bounds__(BLOCK) void k_sweep_hot(Sweep sw) {
    constexpr uint32_t QMAX = 64;
    __shared__ float s_theta[HOT_TILE_MAX];
    __shared__ uint64_t s_Z[HOT_TILE_MAX];
    __shared__ const uint32_t *s_idx[QMAX];
    __shared__ const float *s_valp[QMAX];
    __shared__ const uint32_t *s_pre[QMAX];
    __shared__ uint32_t s_b0[QMAX], s_len[QMAX], s_pull[QMAX];
    __shared__ float s_alpha[QMAX];
    const uint32_t tid = threadIdx.x;
    const uint32_t n_ovf = sw.ovf[0];
    const uint32_t tile = 1u << sw.tile_shift;
    if (tid < sw.Q) {
        const UpdDesc u = sw.U[tid];
        s_idx[tid] = u.idx;
        s_valp[tid] = u.val;
        s_pre[tid] = u.pre;
        s_pull[tid] = u.pull;
    }
    if (tid < QMAX) s_alpha[tid] = tid ? __fdiv_rn(sw.lr, (float)tid) : sw.lr;
    for (uint32_t o = blockIdx.x; o < n_ovf; o += gridDim.x) {
        const uint32_t t = sw.ovf[1 + o];
        const ParamDesc pd = sw.P[sw.tile_tensor[t]];
        const uint32_t c0 = (t - (uint32_t)pd.tile_base) << sw.tile_shift;
        const uint32_t ncoord = pd.n - c0 < tile ? (uint32_t)(pd.n - c0) : tile;
        __syncthreads();  // tables ready; the previous tile has been written back
        for (uint32_t c = tid; c < ncoord; c += BLOCK) {
            s_theta[c] = pd.theta[c0 + c];
            s_Z[c] = 0;
        }
        if (tid < sw.Q) {
            const uint32_t *row = sw.B + (uint64_t)tid * (sw.ntiles + 1) + t;
            const uint32_t b0 = row[0], b1 = row[1];
            s_b0[tid] = b0;
            const uint32_t len = b1 >= b0 ? b1 - b0 : 0u;  // bounds of an unsorted (malformed) list may cross
            s_len[tid] = len < tile ? len : tile;          // a sorted list has at most one entry per coordinate
        }
        __syncthreads();
        auto apply_entry = [&](uint32_t q, uint64_t window, uint32_t k, float v, uint32_t before) {
            const uint32_t c = k - c0;
            if (c >= ncoord) return;  // only a malformed (unsorted) index list gets here
            const uint32_t sigma = before + popc64(s_Z[c] & window);
            const float alpha = sigma < QMAX ? s_alpha[sigma] : __fdiv_rn(sw.lr, (float)sigma);
            s_theta[c] = __fsub_rn(s_theta[c], __fmul_rn(alpha, v));
            if (is_nonzero(v)) s_Z[c] |= 1ull << q;
        };
        uint32_t next_k = 0, next_before = 0;
        float next_v = 0.f;
        bool next_have = tid < s_len[0];
        if (next_have) {
            const uint32_t e = s_b0[0] + tid;
            next_k = ((global_u32)s_idx[0])[e];
            next_v = ((global_f32)s_valp[0])[e];
            if (s_pre[0]) next_before = ((global_u32)s_pre[0])[e];
        }
        for (uint32_t q = 0; q < sw.Q; ++q) {
            const uint32_t k = next_k, before = next_before;
            const float v = next_v;
            const bool have = next_have;
            next_have = q + 1 < sw.Q && tid < s_len[q + 1];
            next_before = 0;
            if (next_have) {
                const uint32_t e = s_b0[q + 1] + tid;
                next_k = ((global_u32)s_idx[q + 1])[e];
                next_v = ((global_f32)s_valp[q + 1])[e];
                if (s_pre[q + 1]) next_before = ((global_u32)s_pre[q + 1])[e];
            }
            const uint32_t pull = s_pull[q];
            const uint64_t window = (q ? (1ull << q) - 1ull : 0ull) & ~((1ull << pull) - 1ull);  // updates pull .. q-1
            if (have) apply_entry(q, window, k, v, before);
            const uint32_t len = s_len[q], b0 = s_b0[q];
            for (uint32_t i = BLOCK + tid; i < len; i += BLOCK) {  // slices longer than the workgroup
                const uint32_t e = b0 + i;
                apply_entry(q, window, ((global_u32)s_idx[q])[e], ((global_f32)s_valp[q])[e],
                            s_pre[q] ? ((global_u32)s_pre[q])[e] : 0u);
            }
            __syncthreads();
        }
        for (uint32_t c = tid; c < ncoord; c += BLOCK) pd.theta[c0 + c] = s_theta[c];
    }
}

// ------------------------------------------------------------------ host side

// Test hooks: environment switches that choose between execution plans with identical results.
// They exist for tests and measurements, are read once at the start of a call, and are no part
// of the interface.
struct ApplyHooks {
    enum Plan { AUTO, SCATTER, SWEEP } plan = AUTO;            // ADACOMP_APPLY_PLAN=scatter|sweep
    enum Kernel { ANY, LONG, DENSE, TILED, SPARSE } kernel = ANY;  // ADACOMP_SWEEP_KERNEL=long|dense|tiled|sparse
    uint32_t tpb = 0;                                          // ADACOMP_TPB=1|2|4 (0: the library's choice)
};

ApplyHooks read_apply_hooks() {
    ApplyHooks hk;
    if (const char *e = std::getenv("ADACOMP_APPLY_PLAN")) {
        if (std::strcmp(e, "scatter") == 0) hk.plan = ApplyHooks::SCATTER;
        else if (std::strcmp(e, "sweep") == 0) hk.plan = ApplyHooks::SWEEP;
    }
    if (const char *e = std::getenv("ADACOMP_SWEEP_KERNEL")) {
        if (std::strcmp(e, "long") == 0) hk.kernel = ApplyHooks::LONG;
        else if (std::strcmp(e, "dense") == 0) hk.kernel = ApplyHooks::DENSE;
        else if (std::strcmp(e, "tiled") == 0) hk.kernel = ApplyHooks::TILED;
        else if (std::strcmp(e, "sparse") == 0) hk.kernel = ApplyHooks::SPARSE;
    }
    if (const char *e = std::getenv("ADACOMP_TPB")) {
        const int t = std::atoi(e);
        hk.tpb = t == 4 || t == 2 ? (uint32_t)t : 1u;
    }
    return hk;
}

struct Layout {
    bool sweep = false;
    bool dense = false;   // sweep plan: one thread per coordinate (k_sweep_dense)
    bool sparse = false;  // sweep plan: touches that are alone on their coordinate need no list (k_sweep_sparse)
    uint32_t tile_shift = 0;
    uint64_t ntiles = 0;
    uint32_t n_hist = 0;  // remembered updates this call reaches back to
    size_t table = 0, upd = 0, pa_off = 0, pa_list = 0, bounds = 0, tile_tensor = 0, ovf = 0, hist = 0;
    std::vector<size_t> snap;  // byte offset per update
    std::vector<size_t> pre;   // byte offset per update pulled before the call, else SIZE_MAX
    size_t bytes = 0;
};

int check_updates(uint32_t L, const adacomp_update_t *updates, uint32_t Q) {
    if (Q && !updates) return ADACOMP_ERR_NULL;
    for (uint32_t q = 0; q < Q; ++q) {
        const adacomp_update_t &u = updates[q];
        if (u.num_layers != L) return ADACOMP_ERR_LAYER_MISMATCH;
        if (!u.layer_off) return ADACOMP_ERR_NULL;
        if (u.layer_off[0] != 0) return ADACOMP_ERR_LAYER_MISMATCH;
        for (uint32_t l = 0; l < L; ++l)
            if (u.layer_off[l + 1] < u.layer_off[l]) return ADACOMP_ERR_LAYER_MISMATCH;
    }
    return ADACOMP_OK;
}

// Timestamps against the state: every update must have been pulled no later than it is
// applied and no earlier than the oldest remembered update.
int check_pulls(const adacomp_state_t *st, const adacomp_update_t *updates, uint32_t Q) {
    const uint64_t t0 = st ? st->t : 0;
    uint64_t remembered = 0;
    if (st && st->history_cap) {
        if (!st->history || !st->history_off) return ADACOMP_ERR_NULL;
        remembered = st->history_len < st->history_cap ? st->history_len : st->history_cap;
        if (remembered > t0) remembered = t0;
    }
    for (uint32_t q = 0; q < Q; ++q) {
        if (updates[q].pull_ts > t0 + q) return ADACOMP_ERR_FUTURE_PULL;
        const bool empty = updates[q].layer_off[updates[q].num_layers] == 0;  // no entry, no staleness to look up
        if (!empty && updates[q].pull_ts + remembered < t0) return ADACOMP_ERR_HISTORY;
    }
    return ADACOMP_OK;
}

// Plan and workspace layout from sizes and timestamps alone.  The sweep pays 16 bytes per
// parameter plus about 30 per entry and three launches; the scatter about 440 bytes per entry
// (measured line traffic) and one or two launches per update.
void make_layout(const uint64_t *n, uint32_t L, uint64_t t0, const adacomp_update_t *updates, uint32_t Q,
                 const ApplyHooks &hk, Layout &lay) {
    double entries = 0, params = 0;
    bool fits32 = true;
    uint64_t oldest = t0;
    for (uint32_t q = 0; q < Q; ++q) {
        entries += (double)updates[q].layer_off[L];
        fits32 = fits32 && updates[q].layer_off[L] <= 0xffff0000ull;  // 32-bit entry numbers, with room for the loops' strides
        if (updates[q].pull_ts < oldest && updates[q].layer_off[L] > 0) oldest = updates[q].pull_ts;
    }
    lay.n_hist = (uint32_t)(t0 - oldest);
    for (uint32_t l = 0; l < L; ++l) params += (double)n[l];
    const bool never = hk.plan == ApplyHooks::SCATTER;  // the hooks override the cost model
    const bool always = hk.plan == ApplyHooks::SWEEP;
    if (!never && Q >= 2 && Q <= 0x7fffu && fits32 && L > 0 && params > 0 && entries > 0) {
        // tile: about STAGE_CAP / 2 queued entries per tile on average, as long as the table of
        // slice bounds (Q x tiles) stays below twice the size of the updates themselves
        const double per_coord = entries / params;
        auto tiles_at = [&](uint32_t sh) {
            uint64_t t = 0;
            for (uint32_t l = 0; l < L; ++l) t += (n[l] + (1ull << sh) - 1) >> sh;
            return t;
        };
        uint32_t shift = 0;
        while ((2u << shift) <= TILE_MAX) ++shift;  // log2(TILE_MAX)
        const double table_budget = std::max(64.0 * 1048576.0, 16.0 * entries);
        const bool dense_forced = hk.kernel == ApplyHooks::DENSE;
        const bool dense_allowed = hk.kernel == ApplyHooks::ANY || dense_forced;  // the other names are those of the other kernels
        const bool dense = Q <= DENSE_QMAX && dense_allowed && (dense_forced || per_coord >= (Q <= 64 ? DENSE_PER_COORD : DENSE_PER_COORD_LONG)) &&
                           (dense_forced || 4.0 * (double)Q * (double)tiles_at(DTILE_SHIFT) <= table_budget);
        // few entries per parameter, short queue: most touches are alone on their coordinate
        const bool sparse = !dense && Q <= PASS_SHORT &&
                            (hk.kernel == ApplyHooks::SPARSE || (hk.kernel == ApplyHooks::ANY && per_coord <= SPARSE_PER_COORD));
        if (dense) {
            shift = DTILE_SHIFT;
        } else if (sparse) {
            shift = 0;
            while ((2u << shift) <= TILE_MAX_SPARSE) ++shift;  // log2(TILE_MAX_SPARSE)
            while (shift > 0 && (double)(1u << shift) * per_coord > SP_CAP * 0.45 &&
                   4.0 * (double)Q * (double)tiles_at(shift - 1) <= table_budget)
                --shift;
        } else {
            while (shift > 0 && (double)(1u << shift) * per_coord > STAGE_CAP / 2 &&
                   4.0 * (double)Q * (double)tiles_at(shift - 1) <= table_budget)
                --shift;
        }
        const uint64_t ntiles = tiles_at(shift);
        uint32_t launches = 0;  // of the scatter plan
        for (uint32_t q = 0; q < Q; ++q)
            if (updates[q].layer_off[L] > 0) launches += (t0 + q - updates[q].pull_ts >= 2) ? 2u : 1u;
        const double sweep_cost = 1.25 * (16.0 * params + 30.0 * entries + 8.0 * (double)Q * (double)ntiles) +
                                  3.0 * LAUNCH_COST_BYTES;
        const double scatter_cost = 440.0 * entries + LAUNCH_COST_BYTES * launches;
        if (ntiles < 0x7fffffffull && (always || scatter_cost > sweep_cost)) {
            lay.sweep = true;
            lay.dense = dense;
            lay.sparse = sparse;
            lay.tile_shift = shift;
            lay.ntiles = ntiles;
        }
    }
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align_up(bytes ? bytes : 1, 256);
        return at;
    };
    lay.table = take(((size_t)L + 1) * sizeof(ParamDesc));
    lay.hist = take((size_t)lay.n_hist * sizeof(HistDesc));
    if (lay.sweep) {
        lay.upd = take((size_t)Q * sizeof(UpdDesc));
        lay.pa_off = take(((size_t)Q + 1) * sizeof(uint32_t));
        lay.pa_list = take((size_t)Q * sizeof(uint32_t));
        lay.bounds = take((size_t)Q * (lay.ntiles + 1) * sizeof(uint32_t));
        lay.tile_tensor = take(lay.ntiles * sizeof(uint32_t));
        lay.ovf = take((lay.ntiles + 1) * sizeof(uint32_t));
    }
    lay.snap.resize(Q);
    lay.pre.assign(Q, SIZE_MAX);
    for (uint32_t q = 0; q < Q; ++q) {
        lay.snap[q] = take((size_t)updates[q].layer_off[L] * sizeof(uint32_t));
        if (updates[q].pull_ts < t0 && updates[q].layer_off[L] > 0)
            lay.pre[q] = take((size_t)updates[q].layer_off[L] * sizeof(uint32_t));
    }
    lay.bytes = off;
}

// Remember the applied updates: slot (timestamp mod history_cap) of the trace.
void remember(adacomp_state_t *st, const adacomp_update_t *updates, uint32_t Q, uint32_t L, uint64_t t0) {
    const uint32_t first = Q > st->history_cap ? Q - st->history_cap : 0;
    for (uint32_t q = first; q < Q; ++q) {
        const uint64_t slot = (t0 + q) % st->history_cap;
        uint64_t *off = st->history_off + slot * ((uint64_t)L + 1);
        std::memcpy(off, updates[q].layer_off, ((size_t)L + 1) * sizeof(uint64_t));
        st->history[slot] = updates[q];
        st->history[slot].layer_off = off;
    }
    const uint64_t len = (uint64_t)st->history_len + Q;
    st->history_len = (uint32_t)(len < st->history_cap ? len : st->history_cap);
}

}  // namespace
}  // namespace adacomp

using namespace adacomp;

extern "C" int adacomp_apply_workspace(const uint64_t *n, uint32_t L, const adacomp_state_t *st,
                                       const adacomp_update_t *updates, uint32_t Q, size_t *bytes) {
    if (!bytes || (L && !n)) return ADACOMP_ERR_NULL;
    int rc = check_updates(L, updates, Q);
    if (rc) return rc;
    rc = check_pulls(st, updates, Q);
    if (rc) return rc;
    Layout lay;
    make_layout(n, L, st ? st->t : 0, updates, Q, read_apply_hooks(), lay);
    *bytes = lay.bytes;
    return ADACOMP_OK;
}

#define CHECK_LAUNCH()                                               \
    do {                                                             \
        if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP; \
    } while (0)

extern "C" int adacomp_apply(const adacomp_param_layer_t *params, uint32_t L, adacomp_state_t *st,
                             const adacomp_update_t *updates, uint32_t Q, float lr,
                             void *workspace, size_t ws_bytes, void *hip_stream) {
    if (!st || (L && (!params || !st->cnt))) return ADACOMP_ERR_NULL;
    if (st->num_layers != L) return ADACOMP_ERR_LAYER_MISMATCH;
    if (!std::isfinite(lr)) return ADACOMP_ERR_LR;
    int rc = check_updates(L, updates, Q);
    if (rc) return rc;
    std::vector<ParamDesc> table((size_t)L + 1);
    std::vector<uint64_t> n(L);
    for (uint32_t l = 0; l < L; ++l) {
        if (params[l].n > 0xffffffffull) return ADACOMP_ERR_LAYER_TOO_LARGE;
        if (params[l].n && (!params[l].data || !st->cnt[l])) return ADACOMP_ERR_NULL;
        if (((uintptr_t)params[l].data & 3u) || ((uintptr_t)st->cnt[l] & 3u)) return ADACOMP_ERR_ALIGNMENT;
        table[l] = ParamDesc{params[l].data, st->cnt[l], params[l].n, 0};
        n[l] = params[l].n;
    }
    table[L] = ParamDesc{nullptr, nullptr, 0, 0};
    const uint64_t t0 = st->t;
    for (uint32_t q = 0; q < Q; ++q) {
        const adacomp_update_t &u = updates[q];
        const uint64_t total = u.layer_off[L];
        for (uint32_t l = 0; l < L; ++l)
            if (u.layer_off[l + 1] - u.layer_off[l] > params[l].n) return ADACOMP_ERR_LAYER_MISMATCH;
        if (total > u.cap) return ADACOMP_ERR_CAPACITY;
        if (total && (!u.idx || !u.val || !u.layer_off_dev)) return ADACOMP_ERR_NULL;
        if (((uintptr_t)u.idx & 3u) || ((uintptr_t)u.val & 3u) || ((uintptr_t)u.layer_off_dev & 7u))
            return ADACOMP_ERR_ALIGNMENT;
    }
    rc = check_pulls(st, updates, Q);
    if (rc) return rc;
    const ApplyHooks hk = read_apply_hooks();
    Layout lay;
    make_layout(n.data(), L, t0, updates, Q, hk, lay);
    if (!workspace || ((uintptr_t)workspace & 255u) || ws_bytes < lay.bytes) return ADACOMP_ERR_WORKSPACE;
    if (Q == 0) return ADACOMP_OK;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char *wsb = static_cast<char *>(workspace);
    ParamDesc *P = reinterpret_cast<ParamDesc *>(wsb + lay.table);

    // Staleness accumulated before this call (eq. 3, u = pull .. t0-1) for the updates that
    // were pulled earlier: searched in the remembered updates t0 - n_hist .. t0 - 1.
    if (lay.n_hist) {
        std::vector<HistDesc> hist(lay.n_hist);
        for (uint32_t h = 0; h < lay.n_hist; ++h) {
            const adacomp_update_t &u = st->history[(t0 - lay.n_hist + h) % st->history_cap];
            hist[h] = u.layer_off[L] ? HistDesc{u.idx, u.val, u.layer_off_dev} : HistDesc{nullptr, nullptr, nullptr};
        }
        const HistDesc *H = reinterpret_cast<const HistDesc *>(wsb + lay.hist);
        if (put_async(wsb + lay.hist, hist.data(), hist.size() * sizeof(HistDesc), s) != hipSuccess)
            return ADACOMP_ERR_HIP;
        for (uint32_t q = 0; q < Q; ++q) {
            if (lay.pre[q] == SIZE_MAX) continue;
            const adacomp_update_t &u = updates[q];
            const uint64_t total = u.layer_off[L];
            const uint32_t first = lay.n_hist - (uint32_t)(t0 - u.pull_ts);
            ADACOMP_LAUNCH(ADACOMP_KERNEL_HISTORY, k_history, dim3((unsigned)((total + BLOCK - 1) / BLOCK)),
                           dim3(BLOCK), s, H, first, lay.n_hist, L, u.layer_off_dev, u.idx,
                           reinterpret_cast<uint32_t *>(wsb + lay.pre[q]), total);
            CHECK_LAUNCH();
        }
    }

    // Inside the call an update pulled earlier behaves as if pulled at the call's first
    // timestamp.  pulled_at[q]: updates whose counters are read just before update q is
    // applied (Alg. 1 "Pull" / Alg. 2 "Get").  A snapshot is needed when the window inside
    // the call can change alpha: two or more iterations, or one on top of earlier staleness.
    std::vector<std::vector<uint32_t>> pulled_at(Q);
    std::vector<char> stale(Q, 0);
    std::vector<uint32_t> pull_rel(Q);
    for (uint32_t q = 0; q < Q; ++q) {
        const bool earlier = updates[q].pull_ts < t0;
        pull_rel[q] = earlier ? 0u : (uint32_t)(updates[q].pull_ts - t0);
        if (updates[q].layer_off[L] > 0 && q - pull_rel[q] >= (lay.pre[q] != SIZE_MAX ? 1u : 2u)) {
            stale[q] = 1;
            pulled_at[pull_rel[q]].push_back(q);
        }
    }
    auto pre_of = [&](uint32_t q) {
        return lay.pre[q] == SIZE_MAX ? nullptr : reinterpret_cast<const uint32_t *>(wsb + lay.pre[q]);
    };

    if (lay.sweep) {
        uint64_t tiles = 0;
        for (uint32_t l = 0; l < L; ++l) {
            table[l].tile_base = tiles;
            tiles += (n[l] + (1ull << lay.tile_shift) - 1) >> lay.tile_shift;
        }
        table[L].tile_base = tiles;
        std::vector<UpdDesc> upd(Q);
        std::vector<uint32_t> pa_off((size_t)Q + 1, 0), pa_list;
        for (uint32_t q = 0; q < Q; ++q) {
            const adacomp_update_t &u = updates[q];
            upd[q] = UpdDesc{u.idx, u.val, u.layer_off_dev, reinterpret_cast<uint32_t *>(wsb + lay.snap[q]),
                             pre_of(q), pull_rel[q], 0};
            pa_off[q] = (uint32_t)pa_list.size();
            pa_list.insert(pa_list.end(), pulled_at[q].begin(), pulled_at[q].end());
        }
        pa_off[Q] = (uint32_t)pa_list.size();
        pa_list.resize(Q, 0);
        Sweep sw;
        sw.P = P;
        sw.U = reinterpret_cast<const UpdDesc *>(wsb + lay.upd);
        sw.B = reinterpret_cast<const uint32_t *>(wsb + lay.bounds);
        sw.tile_tensor = reinterpret_cast<const uint32_t *>(wsb + lay.tile_tensor);
        sw.pa_off = reinterpret_cast<const uint32_t *>(wsb + lay.pa_off);
        sw.pa_list = reinterpret_cast<const uint32_t *>(wsb + lay.pa_list);
        sw.ovf = reinterpret_cast<uint32_t *>(wsb + lay.ovf);
        sw.L = L;
        sw.Q = Q;
        sw.ntiles = (uint32_t)lay.ntiles;
        sw.tile_shift = lay.tile_shift;
        sw.lr = lr;
        if (put_async(P, table.data(), table.size() * sizeof(ParamDesc), s) != hipSuccess ||
            put_async(wsb + lay.upd, upd.data(), upd.size() * sizeof(UpdDesc), s) != hipSuccess ||
            put_async(wsb + lay.pa_off, pa_off.data(), pa_off.size() * sizeof(uint32_t), s) != hipSuccess ||
            put_async(wsb + lay.pa_list, pa_list.data(), pa_list.size() * sizeof(uint32_t), s) != hipSuccess ||
            fill_u32_async(sw.ovf, 0u, 1, s) != hipSuccess)
            return ADACOMP_ERR_HIP;
        const uint64_t nb = ((uint64_t)Q * (lay.ntiles + 1) + BLOCK - 1) / BLOCK;
        if (nb > 0x7fffffffull) return ADACOMP_ERR_LAYER_TOO_LARGE;
        ADACOMP_LAUNCH(ADACOMP_KERNEL_BOUNDS, k_bounds, dim3((unsigned)nb), dim3(BLOCK), s, sw,
                       reinterpret_cast<uint32_t *>(wsb + lay.bounds),
                       reinterpret_cast<uint32_t *>(wsb + lay.tile_tensor));
        CHECK_LAUNCH();
        if (lay.dense) {
            bool any_pre = false;
            for (uint32_t q = 0; q < Q; ++q) any_pre = any_pre || lay.pre[q] != SIZE_MAX;
            const dim3 grid((unsigned)lay.ntiles);
#define DENSE(NW, DQ, PRE) ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, (k_sweep_dense<NW, DQ, PRE>), grid, dim3(BLOCK), s, sw)
            if (Q <= 64 && any_pre) DENSE(1, 16, true);
            else if (Q <= 64) DENSE(1, 16, false);
            else if (any_pre) DENSE(4, 16, true);
            else DENSE(4, 16, false);
#undef DENSE
            CHECK_LAUNCH();
            if (st->history_cap) remember(st, updates, Q, L, t0);
            st->t = t0 + Q;
            return ADACOMP_OK;
        }
        // several tiles per workgroup once there are enough tiles to fill the chip many times over
        // (the kernel for sparse queues is bound by its memory traffic, not by the chain of dependent loads: measured
        // 1.61 / 1.73 / 1.82 ms per queue of the 1e9-parameter workload with 1 / 2 / 4 tiles per workgroup)
        const uint32_t tpb = hk.tpb ? hk.tpb : (lay.sparse ? 1u : (lay.ntiles >= 65536 ? 4u : 1u));
        const dim3 grid((unsigned)((lay.ntiles + tpb - 1) / tpb));
        const bool short_queue = Q <= PASS_SHORT && hk.kernel != ApplyHooks::LONG;  // else the general kernel also for short queues
        if (lay.sparse && tpb == 4) ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, k_sweep_sparse<4>, grid, dim3(BLOCK), s, sw);
        else if (lay.sparse && tpb == 2) ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, k_sweep_sparse<2>, grid, dim3(BLOCK), s, sw);
        else if (lay.sparse) ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, k_sweep_sparse<1>, dim3((unsigned)lay.ntiles), dim3(BLOCK), s, sw);
        else if (short_queue && tpb == 4) ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, k_sweep_short<4>, grid, dim3(BLOCK), s, sw);
        else if (short_queue && tpb == 2) ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, k_sweep_short<2>, grid, dim3(BLOCK), s, sw);
        else if (short_queue) ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, k_sweep_short<1>, dim3((unsigned)lay.ntiles), dim3(BLOCK), s, sw);
        else if (tpb == 4) ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, k_sweep<4>, grid, dim3(BLOCK), s, sw);
        else if (tpb == 2) ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, k_sweep<2>, grid, dim3(BLOCK), s, sw);
        else ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP, k_sweep<1>, dim3((unsigned)lay.ntiles), dim3(BLOCK), s, sw);
        CHECK_LAUNCH();
        if (Q <= 64)
            ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP_SLOW, k_sweep_hot,
                           dim3((unsigned)std::min<uint64_t>(lay.ntiles, 2 * SLOW_GRID)), dim3(BLOCK), s, sw);
        else
            ADACOMP_LAUNCH(ADACOMP_KERNEL_SWEEP_SLOW, k_sweep_slow,
                           dim3((unsigned)std::min<uint64_t>(lay.ntiles, SLOW_GRID)), dim3(BLOCK), s, sw);
        CHECK_LAUNCH();
    } else {
        if (L && put_async(P, table.data(), table.size() * sizeof(ParamDesc), s) != hipSuccess)
            return ADACOMP_ERR_HIP;
        // counted[q]: some later update has a snapshot taken at or before update q
        std::vector<char> counted(Q, 0);
        uint32_t first_snapshot = UINT32_MAX;
        for (uint32_t q = Q; q-- > 0;) {
            counted[q] = first_snapshot <= q;
            if (stale[q]) first_snapshot = std::min(first_snapshot, pull_rel[q]);
        }
        for (uint32_t q = 0; q < Q; ++q) {
            for (uint32_t w : pulled_at[q]) {
                const adacomp_update_t &u = updates[w];
                const uint64_t total = u.layer_off[L];
                const unsigned grid = (unsigned)((total + BLOCK * ITEMS - 1) / (BLOCK * ITEMS));
                ADACOMP_LAUNCH(ADACOMP_KERNEL_SNAPSHOT, k_snapshot, dim3(grid), dim3(BLOCK), s, P, L,
                               u.layer_off_dev, u.idx, reinterpret_cast<uint32_t *>(wsb + lay.snap[w]), total);
                CHECK_LAUNCH();
            }
            const adacomp_update_t &u = updates[q];
            const uint64_t total = u.layer_off[L];
            if (total == 0) continue;  // an empty push only advances the timestamp
            const dim3 grid((unsigned)((total + BLOCK * ITEMS - 1) / (BLOCK * ITEMS)));
            const uint32_t *snap = reinterpret_cast<const uint32_t *>(wsb + lay.snap[q]);
            const uint32_t *pre = pre_of(q);
#define SCATTER(STALE, PRE)                                                                                        \
    do {                                                                                                           \
        if (counted[q])                                                                                            \
            ADACOMP_LAUNCH(ADACOMP_KERNEL_SCATTER_APPLY, (k_scatter_apply<STALE, PRE, true>), grid, dim3(BLOCK),   \
                           s, P, L, u.layer_off_dev, u.idx, u.val, snap, pre, total, lr);                          \
        else                                                                                                       \
            ADACOMP_LAUNCH(ADACOMP_KERNEL_SCATTER_APPLY, (k_scatter_apply<STALE, PRE, false>), grid, dim3(BLOCK),  \
                           s, P, L, u.layer_off_dev, u.idx, u.val, snap, pre, total, lr);                          \
    } while (0)
            if (stale[q] && pre) SCATTER(true, true);
            else if (stale[q]) SCATTER(true, false);
            else if (pre) SCATTER(false, true);
            else SCATTER(false, false);
#undef SCATTER
            CHECK_LAUNCH();
        }
    }

    if (st->history_cap) remember(st, updates, Q, L, t0);
    st->t = t0 + Q;
    return ADACOMP_OK;
}

extern "C" int adacomp_apply_global_staleness(const adacomp_param_layer_t *params, uint32_t L, adacomp_state_t *st,
                                              const adacomp_update_t *updates, uint32_t Q, float lr,
                                              void *workspace, size_t ws_bytes, void *hip_stream) {
    if (!st || (L && !params)) return ADACOMP_ERR_NULL;
    if (st->num_layers != L) return ADACOMP_ERR_LAYER_MISMATCH;
    if (st->history_cap && (!st->history || !st->history_off)) return ADACOMP_ERR_NULL;
    if (!std::isfinite(lr)) return ADACOMP_ERR_LR;
    int rc = check_updates(L, updates, Q);
    if (rc) return rc;
    std::vector<ParamDesc> table((size_t)L + 1, ParamDesc{nullptr, nullptr, 0, 0});
    for (uint32_t l = 0; l < L; ++l) {
        if (params[l].n > 0xffffffffull) return ADACOMP_ERR_LAYER_TOO_LARGE;
        if (params[l].n && !params[l].data) return ADACOMP_ERR_NULL;
        if ((uintptr_t)params[l].data & 3u) return ADACOMP_ERR_ALIGNMENT;
        table[l] = ParamDesc{params[l].data, nullptr, params[l].n, 0};
    }
    const uint64_t t0 = st->t;
    for (uint32_t q = 0; q < Q; ++q) {
        const adacomp_update_t &u = updates[q];
        const uint64_t total = u.layer_off[L];
        for (uint32_t l = 0; l < L; ++l)
            if (u.layer_off[l + 1] - u.layer_off[l] > params[l].n) return ADACOMP_ERR_LAYER_MISMATCH;
        if (total > u.cap) return ADACOMP_ERR_CAPACITY;
        if (total && (!u.idx || !u.val || !u.layer_off_dev)) return ADACOMP_ERR_NULL;
        if (((uintptr_t)u.idx & 3u) || ((uintptr_t)u.val & 3u) || ((uintptr_t)u.layer_off_dev & 7u))
            return ADACOMP_ERR_ALIGNMENT;
        if (u.pull_ts > t0 + q) return ADACOMP_ERR_FUTURE_PULL;
        if (t0 + q - u.pull_ts > 0xffffffffull) return ADACOMP_ERR_HISTORY;
    }
    const size_t need = align_up(((size_t)L + 1) * sizeof(ParamDesc), 256);
    if (!workspace || ((uintptr_t)workspace & 255u) || ws_bytes < need) return ADACOMP_ERR_WORKSPACE;
    if (Q == 0) return ADACOMP_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    ParamDesc *P = static_cast<ParamDesc *>(workspace);
    bool any = false;
    for (uint32_t q = 0; q < Q; ++q) any = any || updates[q].layer_off[L] > 0;
    if (!any) {  // empty pushes only: nothing to enqueue
        if (st->history_cap) remember(st, updates, Q, L, t0);
        st->t = t0 + Q;
        return ADACOMP_OK;
    }
    if (put_async(P, table.data(), table.size() * sizeof(ParamDesc), s) != hipSuccess) return ADACOMP_ERR_HIP;
    for (uint32_t q = 0; q < Q; ++q) {
        const adacomp_update_t &u = updates[q];
        const uint64_t total = u.layer_off[L];
        if (total == 0) continue;
        const dim3 grid((unsigned)((total + BLOCK * ITEMS - 1) / (BLOCK * ITEMS)));
        ADACOMP_LAUNCH(ADACOMP_KERNEL_SCATTER_APPLY, k_scatter_apply_global, grid, dim3(BLOCK), s, P, L,
                       u.layer_off_dev, u.idx, u.val, total, lr, (uint32_t)(t0 + q - u.pull_ts));
        CHECK_LAUNCH();
    }
    // the trace records which parameters an update touched, whichever rule set its step: a later
    // adacomp_apply on this state may look back across these timestamps (eq. 3)
    if (st->history_cap) remember(st, updates, Q, L, t0);
    st->t = t0 + Q;
    return ADACOMP_OK;
}

extern "C" int adacomp_update_validate(const adacomp_update_t *update, const uint64_t *n_dev, uint32_t L,
                                       uint32_t *flags_dev, void *hip_stream) {
    if (!update || !flags_dev || (L && !n_dev)) return ADACOMP_ERR_NULL;
    int rc = check_updates(L, update, 1);
    if (rc) return rc;
    const uint64_t total = update->layer_off[L];
    if (total > update->cap) return ADACOMP_ERR_CAPACITY;
    if (!update->layer_off_dev || (total && !update->idx)) return ADACOMP_ERR_NULL;
    if (((uintptr_t)update->idx & 3u) || ((uintptr_t)update->layer_off_dev & 7u) || ((uintptr_t)n_dev & 7u) ||
        ((uintptr_t)flags_dev & 3u))
        return ADACOMP_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (fill_u32_async(flags_dev, 0u, 1, s) != hipSuccess) return ADACOMP_ERR_HIP;
    const dim3 grid((unsigned)((total + BLOCK) / BLOCK));
    ADACOMP_LAUNCH(ADACOMP_KERNEL_VALIDATE, k_validate, grid, dim3(BLOCK), s, n_dev, L, update->layer_off_dev,
                   update->idx, total, flags_dev);
    CHECK_LAUNCH();
    return ADACOMP_OK;
}
