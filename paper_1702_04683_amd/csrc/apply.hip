// adacomp_apply: loop body of Alg. 2 (eqs. 3, 4, 5) for a queue of sparse updates.
//
// Per-parameter staleness without searching a history: cnt[k] counts the applied
// updates whose entry for parameter k was non-zero, so the sum of indicators of eq. 3
// over u = j .. i-1 is cnt_k(at time i) - cnt_k(at time j).  The index set of every
// queued update is known when the call starts, so the second reading is taken by a
// gather ("snapshot") of cnt at the update's own indices, enqueued at the point of the
// queue where PS time equals the update's pull timestamp j.  Indices inside one update
// are unique, so the scatter needs no atomics; updates are serialised by stream order.
#include <cmath>
#include <vector>

#include "common.h"

namespace adacomp {
namespace {

constexpr uint32_t BLOCK = 256;
constexpr uint32_t ITEMS = 4;  // entries per thread

struct ParamDesc {
    float *theta;
    uint32_t *cnt;
    uint64_t n;
};
static_assert(sizeof(ParamDesc) % 8 == 0, "table is uploaded as 64-bit words");

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
        snap[e] = P[l].cnt[idx[e]];
    }
}

// One PS iteration.  STALE: the update was pulled two or more iterations ago and has a
// snapshot; otherwise sigma_k is 0 or 1 for every entry and alpha_k = alpha.
template <bool STALE>
__global__ __launch_bounds__(BLOCK) void k_scatter_apply(const ParamDesc *P, uint32_t L, const uint64_t *off,
                                                         const uint32_t *idx, const float *val,
                                                         const uint32_t *snap, uint64_t total, float lr) {
    uint64_t e = (uint64_t)blockIdx.x * (BLOCK * ITEMS) + threadIdx.x;
    if (e >= total) return;
    uint32_t l = layer_of(off, L, e);
#pragma unroll
    for (uint32_t i = 0; i < ITEMS; ++i, e += BLOCK) {
        if (e >= total) break;
        while (e >= off[l + 1]) ++l;
        const uint32_t k = idx[e];
        const float v = val[e];
        const bool nonzero = (__float_as_uint(v) & KEY_MASK) != 0;  // indicator of eq. 3
        float *theta = P[l].theta + k;
        uint32_t *cnt = P[l].cnt + k;
        float alpha = lr;
        uint32_t c = 0;
        if (STALE || nonzero) c = *cnt;
        if (STALE) {
            const uint32_t sigma = c - snap[e];                      // eq. 3
            if (sigma != 0) alpha = __fdiv_rn(lr, (float)sigma);     // eq. 5
        }
        *theta = __fsub_rn(*theta, __fmul_rn(alpha, v));             // eq. 4
        if (nonzero) *cnt = c + 1;
    }
}

struct Layout {
    size_t table = 0;
    std::vector<size_t> snap;  // byte offset per update
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

void make_layout(uint32_t L, const adacomp_update_t *updates, uint32_t Q, Layout &lay) {
    size_t off = 0;
    lay.table = off;
    off += align_up((size_t)(L ? L : 1) * sizeof(ParamDesc), 256);
    lay.snap.resize(Q);
    for (uint32_t q = 0; q < Q; ++q) {
        lay.snap[q] = off;
        off += align_up((size_t)updates[q].layer_off[L] * sizeof(uint32_t) + 1, 256);
    }
    lay.bytes = off;
}

}  // namespace
}  // namespace adacomp

using namespace adacomp;

extern "C" int adacomp_apply_workspace(uint32_t L, const adacomp_update_t *updates, uint32_t Q,
                                       size_t *bytes) {
    if (!bytes) return ADACOMP_ERR_NULL;
    int rc = check_updates(L, updates, Q);
    if (rc) return rc;
    Layout lay;
    make_layout(L, updates, Q, lay);
    *bytes = lay.bytes;
    return ADACOMP_OK;
}

extern "C" int adacomp_apply(const adacomp_param_layer_t *params, uint32_t L, adacomp_state_t *st,
                             const adacomp_update_t *updates, uint32_t Q, float lr,
                             void *workspace, size_t ws_bytes, void *hip_stream) {
    if (!st || (L && (!params || !st->cnt))) return ADACOMP_ERR_NULL;
    if (st->num_layers != L) return ADACOMP_ERR_LAYER_MISMATCH;
    if (!std::isfinite(lr)) return ADACOMP_ERR_LR;
    int rc = check_updates(L, updates, Q);
    if (rc) return rc;
    std::vector<ParamDesc> table(L);
    for (uint32_t l = 0; l < L; ++l) {
        if (params[l].n > 0xffffffffull) return ADACOMP_ERR_LAYER_TOO_LARGE;
        if (params[l].n && (!params[l].data || !st->cnt[l])) return ADACOMP_ERR_NULL;
        if (((uintptr_t)params[l].data & 3u) || ((uintptr_t)st->cnt[l] & 3u)) return ADACOMP_ERR_ALIGNMENT;
        table[l] = ParamDesc{params[l].data, st->cnt[l], params[l].n};
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
        if (u.pull_ts < t0) return ADACOMP_ERR_HISTORY;
    }
    Layout lay;
    make_layout(L, updates, Q, lay);
    if (!workspace || ((uintptr_t)workspace & 255u) || ws_bytes < lay.bytes) return ADACOMP_ERR_WORKSPACE;
    if (Q == 0) return ADACOMP_OK;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char *wsb = static_cast<char *>(workspace);
    ParamDesc *P = reinterpret_cast<ParamDesc *>(wsb + lay.table);
    if (L && put_async(P, table.data(), table.size() * sizeof(ParamDesc), s) != hipSuccess)
        return ADACOMP_ERR_HIP;

    // pulled_at[q]: updates whose worker pulled at PS time t0 + q and that arrive two
    // or more iterations later (Alg. 1 "Pull" / Alg. 2 "Get"): their counters are
    // read just before update q is applied.
    std::vector<std::vector<uint32_t>> pulled_at(Q);
    std::vector<char> stale(Q, 0);
    for (uint32_t q = 0; q < Q; ++q) {
        const uint64_t j = updates[q].pull_ts - t0;
        if (q - j >= 2 && updates[q].layer_off[L] > 0) {
            stale[q] = 1;
            pulled_at[j].push_back(q);
        }
    }
    for (uint32_t q = 0; q < Q; ++q) {
        for (uint32_t w : pulled_at[q]) {
            const adacomp_update_t &u = updates[w];
            const uint64_t total = u.layer_off[L];
            const unsigned grid = (unsigned)((total + BLOCK * ITEMS - 1) / (BLOCK * ITEMS));
            ADACOMP_LAUNCH(ADACOMP_KERNEL_SNAPSHOT, k_snapshot, dim3(grid), dim3(BLOCK), s, P, L,
                           u.layer_off_dev, u.idx, reinterpret_cast<uint32_t *>(wsb + lay.snap[w]), total);
            if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP;
        }
        const adacomp_update_t &u = updates[q];
        const uint64_t total = u.layer_off[L];
        if (total == 0) continue;  // an empty push only advances the timestamp
        const unsigned grid = (unsigned)((total + BLOCK * ITEMS - 1) / (BLOCK * ITEMS));
        const uint32_t *snap = reinterpret_cast<const uint32_t *>(wsb + lay.snap[q]);
        if (stale[q])
            ADACOMP_LAUNCH(ADACOMP_KERNEL_SCATTER_APPLY, k_scatter_apply<true>, dim3(grid), dim3(BLOCK), s, P, L,
                           u.layer_off_dev, u.idx, u.val, snap, total, lr);
        else
            ADACOMP_LAUNCH(ADACOMP_KERNEL_SCATTER_APPLY, k_scatter_apply<false>, dim3(grid), dim3(BLOCK), s, P, L,
                           u.layer_off_dev, u.idx, u.val, snap, total, lr);
        if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP;
    }
    st->t = t0 + Q;
    return ADACOMP_OK;
}
