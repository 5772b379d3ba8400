// Optional per-kernel timing with HIP events attached to the kernel dispatch itself
// (hipExtLaunchKernelGGL start/stop events: the span is the kernel's own begin..end on
// its stream, not the gap before it).  Off unless adacomp_profile_start() was called;
// when off a launch costs one predictable branch.  Not thread-safe: meant for a
// benchmark's single thread.
#include <vector>

#include "common.h"

namespace adacomp {
namespace {

struct Span {
    int id;
    hipEvent_t beg, end;
};

uint64_t g_mask = 0;
std::vector<Span> g_spans;
std::vector<hipEvent_t> g_pool;

hipEvent_t take_event() {
    hipEvent_t e = nullptr;
    if (!g_pool.empty()) {
        e = g_pool.back();
        g_pool.pop_back();
    } else if (hipEventCreate(&e) != hipSuccess) {
        e = nullptr;
    }
    return e;
}

}  // namespace

ProfScope::ProfScope(int id) : beg_(nullptr), end_(nullptr) {
    if (!((g_mask >> id) & 1u)) return;
    Span sp{id, take_event(), take_event()};
    if (!sp.beg || !sp.end) return;
    g_spans.push_back(sp);
    beg_ = sp.beg;
    end_ = sp.end;
}

}  // namespace adacomp

using namespace adacomp;

extern "C" int adacomp_profile_start(uint64_t kernel_mask) {
    for (Span &sp : g_spans) {
        g_pool.push_back(sp.beg);
        g_pool.push_back(sp.end);
    }
    g_spans.clear();
    g_mask = kernel_mask;
    return ADACOMP_OK;
}

extern "C" int adacomp_profile_stop(double *total_ms, uint64_t *launches) {
    g_mask = 0;
    for (int i = 0; i < ADACOMP_KERNEL_COUNT; ++i) {
        if (total_ms) total_ms[i] = 0.0;
        if (launches) launches[i] = 0;
    }
    int rc = ADACOMP_OK;
    for (Span &sp : g_spans) {
        float ms = 0.f;
        if (hipEventSynchronize(sp.end) != hipSuccess || hipEventElapsedTime(&ms, sp.beg, sp.end) != hipSuccess) {
            rc = ADACOMP_ERR_HIP;
        } else {
            if (total_ms) total_ms[sp.id] += ms;
            if (launches) launches[sp.id] += 1;
        }
        g_pool.push_back(sp.beg);
        g_pool.push_back(sp.end);
    }
    g_spans.clear();
    return rc;
}

extern "C" const char *adacomp_kernel_name(int id) {
    switch (id) {
        case ADACOMP_KERNEL_PUT: return "put";
        case ADACOMP_KERNEL_FILL: return "fill";
        case ADACOMP_KERNEL_SAMPLE_HIST: return "sample_hist";
        case ADACOMP_KERNEL_PICK: return "pick";
        case ADACOMP_KERNEL_FILTER: return "filter";
        case ADACOMP_KERNEL_FINISH: return "finish";
        case ADACOMP_KERNEL_GATHER: return "gather";
        case ADACOMP_KERNEL_WORK: return "work";
        case ADACOMP_KERNEL_HIST: return "hist";
        case ADACOMP_KERNEL_RESOLVE: return "resolve";
        case ADACOMP_KERNEL_COUNT_SEG: return "count";
        case ADACOMP_KERNEL_SCAN: return "scan";
        case ADACOMP_KERNEL_EMIT: return "emit";
        case ADACOMP_KERNEL_IDENTITY: return "identity";
        case ADACOMP_KERNEL_HISTORY: return "history";
        case ADACOMP_KERNEL_SNAPSHOT: return "snapshot";
        case ADACOMP_KERNEL_SCATTER_APPLY: return "scatter_apply";
        case ADACOMP_KERNEL_BOUNDS: return "bounds";
        case ADACOMP_KERNEL_SWEEP: return "sweep";
        case ADACOMP_KERNEL_SWEEP_SLOW: return "sweep_slow";
        case ADACOMP_KERNEL_VALIDATE: return "validate";
        case ADACOMP_KERNEL_WIRE_MEASURE: return "wire_measure";
        case ADACOMP_KERNEL_WIRE_SCAN: return "wire_scan";
        case ADACOMP_KERNEL_WIRE_WRITE: return "wire_write";
        case ADACOMP_KERNEL_WIRE_READ: return "wire_read";
        case ADACOMP_KERNEL_SMALL: return "small";
        default: return "?";
    }
}
