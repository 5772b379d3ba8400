// adacomp_select: SELECT_GRAD of Alg. 1 on gfx950.
//
// Exact per-tensor top-k by magnitude, output in ascending index order, ties at the
// threshold broken towards the lower index.  Everything is integer work on the
// magnitude key (sign-cleared IEEE bits); no floating-point comparison is made.
//
// Pipeline (all tensors of the update go through each launch together):
//   1. sample histogram   a strided sample of 1 KB pieces of every tensor is binned on
//                         the top 12 key bits (LDS histogram per workgroup);
//   2. pick               from it a conservative filter threshold t_lo is chosen so that
//                         #{key >= t_lo} >= k with overwhelming probability and not
//                         much more (exactly, when the sample is the whole tensor);
//   3. filter             the one full streaming read: every wave owns a contiguous
//                         8192-element segment and compacts, in index order, the
//                         entries with key >= t_lo into its own candidate region;
//   4. check              per tensor: scan of the candidate counts; a tensor whose
//                         candidates are fewer than k or exceed a quarter of the tensor
//                         is switched to the dense source (the tensor itself), so
//                         exactness never depends on the sample;
//   5. gather             the regions are packed, in index order, into one dense
//                         (index, value) array per tensor; a segment with more
//                         candidates than its region holds (large entries clustered in
//                         one stretch) is read and filtered again on the spot;
//   6. radix descent      12 + 12 + 7 bit histograms over the packed candidates (or the
//                         dense source) give the exact threshold key T and tie quota r;
//   7. count / scan / emit  per-chunk counts of key > T and key == T, their exclusive
//                         scans, and the order-preserving write of exactly k
//                         (index, value) pairs.
// Steps 3-5 are launched once per group of consecutive tensors; all groups use the same
// candidate-region memory, sized so that what a group writes there is still in the
// last-level cache when its gather reads it.
// Tensors with k == n are copied (identity), tensors with k == 0 produce nothing,
// tensors with k > n/8 skip steps 1-5.
//
// Small tensors (the whole CNN of Sec. 5.1 has 211,690 parameters) would pay about twenty
// launches for microseconds of work: when the small tensors of a call fit the last-level
// cache, each is selected by one workgroup in a single launch (k_small: the same 12 + 12 + 7
// bit descent with LDS histograms, then the ordered write), and the pipeline above runs for
// the large tensors only.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <cmath>
#include <mutex>
#include <vector>

#include "common.h"

namespace adacomp {
namespace {

constexpr uint32_t WSEG = 8192;     // elements per wave segment
constexpr int FILTER_NLOAD = 1;     // 16-byte loads per lane in flight in the filter: at 8 waves per SIMD one keeps 32 KB per compute unit
                                    // in flight, which is what the memory system takes; two are 3 % slower, half the waves 25 %
constexpr uint32_t PIECE = 256;     // elements per wave-wide float4 load
constexpr uint32_t BINS = 4096;     // histogram bins (12 key bits)
constexpr uint32_t VCHUNK = 2048;   // packed candidates per wave chunk (descent, count, emit)
// Segments per wave in the gather, by the capacity of a candidate region (three times its expected fill): fuller
// regions mean longer chains of loads per segment, so fewer segments per wave and more waves.  Measured per step:
// capacity 100: 54 us at 16, 66 at 4; 247: 0.42 ms at 8, 0.50 at 16, 0.47 at 4; 410: 0.176 ms at 4, 0.188 at 8,
// 0.230 at 16; 3260: 1.68 ms at 4, 2.44 at 8, 3.76 at 16.
constexpr uint32_t GSEGS = 16, GSEGS_MID = 8, GSEGS_FULL = 4;
constexpr uint32_t GATHER_MID_CAP = 128, GATHER_FULL_CAP = 320;
constexpr uint32_t TAIL_BLOCKS = 1024;  // workgroups of the descent / count / emit kernels
constexpr uint32_t SPIECES = 64;    // sampled pieces per sample-histogram workgroup
constexpr uint32_t BLOCK = 256;     // threads per workgroup = 4 waves
constexpr uint32_t WAVES = BLOCK / WAVE;
constexpr uint32_t IDENT_TILE = BLOCK * 16;  // elements per identity-copy workgroup
constexpr uint32_t SMALL_MAX = 1u << 18;     // largest tensor that one workgroup selects on its own
constexpr uint64_t SMALL_TOTAL = 1ull << 26; // ... as long as all such tensors of the call hold no more elements than this
constexpr uint32_t SBLOCK = 1024;            // threads of that workgroup
constexpr uint32_t SWAVES = SBLOCK / WAVE;
// k_finish: one workgroup takes a tensor from the candidates its filter left to its output
constexpr uint32_t FUSE_MAX_SEG = 2048;      // most segments of such a tensor (16.7M elements)
constexpr uint32_t FUSE_MAX_CAND = 1u << 17; // ... and most candidates the plan expects for it (the kernel accepts twice as many)
constexpr uint32_t FUSE_MAX_CAP = 320;       // ... and largest region: fuller segments are packed faster by the gather's many waves
constexpr uint32_t FUSE_SHIFT = 11;          // key bits resolved by its second histogram; the first takes the 12 above
constexpr uint32_t FUSE_ROWS = 8;           // rows of 64 candidates that a packing wave of k_finish has in flight

// Candidate regions of one group of tensors: consecutive tensors are filtered and finished (or
// checked and packed) together, and the next group reuses the same region memory, which bounds the
// workspace.  The filter writes the regions with streaming stores and k_finish gives every tensor of
// the group one workgroup, in as many rounds as it takes; the tensors of a call are spread evenly
// over the groups that these limits ask for.  Whole steps on 16 x 4 GB gradients (1600 tensors,
// 5 GB of regions) on a settled box: 7 groups of up to 256 tensors 12.23 ms, 512 + 512 + 512 + 64
// tensors 12.13, three groups of 534 12.18, 768 + 768 + 64 12.08, two groups of 800 12.03,
// 1024 + 576 12.08, one group 12.13.
constexpr uint64_t GROUP_BYTES = 2560ull << 20;
constexpr uint32_t GROUP_TENSORS = 1024;

enum : uint32_t { MODE_EMPTY = 0, MODE_IDENTITY = 1, MODE_FILTER = 2, MODE_DENSE = 3, MODE_SMALL = 4 };

struct SmallDesc {  // a tensor selected by one workgroup
    const float *g;
    uint64_t out_off;
    uint32_t n, k;
};
// What is uploaded for it: the count and the output position come from the update's own
// offsets on the device, 16 bytes per tensor instead of 24 (a third fewer upload launches for
// a call that is nothing but small tensors).
struct SmallEntry {
    const float *g;
    uint32_t n;
    uint32_t l;  // tensor number in the call
};
static_assert(sizeof(SmallEntry) % 8 == 0, "descriptor table is uploaded as 64-bit words");

struct LayerDesc {
    const float *g;
    uint64_t out_off;    // first output entry of this tensor (layer_off[l])
    uint64_t cand_base;  // first candidate slot of this tensor's regions (slots are reused group after group)
    uint64_t pack_base;  // first slot of this tensor's packed candidates
    uint32_t n, k;
    uint32_t mode;
    uint32_t vec;        // data pointer is 16-byte aligned
    uint32_t nseg;       // wave segments taking part in filter / descent / emit
    uint32_t seg_base;   // first global segment id
    uint32_t cap;        // candidate slots per segment
    uint32_t stride;     // one piece sampled out of `stride`
    uint32_t npieces;    // pieces in the tensor
    uint32_t npieces_s;  // sampled pieces
    uint32_t target;     // sample count the filter threshold must cover
    uint32_t sblk_base;  // prefix sums of workgroup counts, one per kernel shape
    uint32_t wblk_base;  //   one segment per wave
    uint32_t iblk_base;  //   identity copy
    uint32_t gblk_base;  //   gather: Plan::gsegs segments per wave
    uint32_t fused;      // few enough segments for one workgroup to finish the tensor right after its filter (k_finish)
};
static_assert(sizeof(LayerDesc) % 8 == 0, "descriptor table is uploaded as 64-bit words");

// What the host uploads per tensor of the pipeline: a quarter of a LayerDesc.  Everything else in
// the descriptor follows from these fields, the update's own offsets and prefix sums over the
// tensors, which k_expand computes on the device (uploads travel in kernel-argument packets of
// 3.5 KB: a call over 1600 tensors needs 11 of them this way instead of 43).
struct CompactDesc {
    const float *g;
    uint32_t n;
    uint32_t l;       // tensor number in the call: its count and output position are the update's offsets
    uint32_t target;
    uint32_t bits;    // mode (3 bits) | fused << 3 | first filtered tensor of a group << 4 | log2(stride) << 5 | cap << 8
};
static_assert(sizeof(CompactDesc) == 24, "table is uploaded as 64-bit words");

struct LayerState {
    uint32_t t_lo;       // candidates are the entries with key >= t_lo
    uint32_t use_dense;  // descent and emit read the tensor itself, not the candidates
    uint32_t prefix;     // key bits fixed so far by the radix descent
    uint32_t k_rem;      // rank still to resolve inside the prefix
    uint32_t T;          // threshold key
    uint32_t r;          // number of entries with key == T to keep (lowest indices)
    uint32_t m;          // elements of the source the descent reads: n, or the number of candidates
    uint32_t nchunk;     // chunks of that source (WSEG elements of the tensor, VCHUNK candidates)
    uint32_t t_reserve;  // a lower, safer threshold the filter only counts against (<= t_lo)
    uint32_t refilter;   // t_lo fell short and was replaced by t_reserve: the gather filters every segment again
    uint32_t done;       // k_finish has written this tensor's output: nothing is left for the later kernels
    uint32_t pad;
};

struct Workspace {
    LayerDesc *desc;      // [L+1]
    LayerState *state;    // [L]
    uint32_t *hist;       // [L][BINS]
    uint32_t *seg_cnt;    // [nseg_total] candidates found per segment
    uint32_t *seg_res;    // [nseg_total] entries with key >= t_reserve per segment
    uint32_t *seg_gt;     // [nseg_total] #key > T, then exclusive prefix within the tensor
    uint32_t *seg_eq;     // [nseg_total] #key == T, then exclusive prefix within the tensor
    uint32_t *chunk_base; // [L+1] first chunk of every tensor in the global chunk numbering
    uint32_t *seg_off;    // [nseg_total] candidates of the tensor before this segment
    uint2 *cand;          // [cand_total] per-segment regions of (index, value bits) of one group of tensors
    uint32_t *pack_idx;   // [pack_total] the candidates packed per tensor
    uint32_t *pack_val;
    SmallEntry *small;    // [nsmall]
    uint32_t *redo;       // [L+1] redo[0] = number of tensors k_finish handed back, redo[1..] = their numbers
    CompactDesc *compact; // [L]
    size_t bytes;
};

// Consecutive tensors whose candidate regions are filled, checked and packed together before
// the next group reuses the same region memory: a group's regions stay in the last-level
// cache between the filter that writes them and the gather that reads them.
struct Group {
    uint32_t l0, l1;  // tensors [l0, l1)
    uint32_t filters; // of them through the filter
    uint32_t unfused; // of those, tensors too large for k_finish: the group needs its own gather
};

struct Plan {
    std::vector<LayerDesc> desc;  // the tensors that go through the pipeline, in order, then one entry with the totals
    std::vector<uint32_t> number; // their numbers in the call
    std::vector<char> opens;      // the tensor is the first filtered one of a group after the first
    std::vector<uint64_t> off;    // [L+1] first output entry of every tensor of the call
    std::vector<Group> groups;    // ranges of `desc`
    uint32_t gsegs = GSEGS;       // segments per wave in the gather
    uint64_t pack_total = 0;
    std::vector<SmallEntry> small; // tensors left to k_small, largest first
    uint64_t nseg_total = 0, cand_total = 0, out_total = 0;
    bool any_fused = false;
};

uint32_t sample_piece(uint32_t p, uint32_t stride, uint32_t npieces) {
    uint32_t j = ((p * 2654435761u) >> 16) & (stride - 1);
    uint64_t q = (uint64_t)p * stride + j;
    return q < npieces ? (uint32_t)q : npieces - 1;
}

// Test hooks: environment switches that choose between execution plans with identical results.
// They exist for tests and measurements, are read once at the start of a call, and are no part
// of the interface.
struct SelectHooks {
    bool small = true;    // ADACOMP_SELECT_SMALL=0: small tensors take the streaming pipeline too
    bool fused = true;    // ADACOMP_SELECT_FUSED=0: no tensor is finished by k_finish
    bool group_tensors = true;  // false with ADACOMP_SELECT_GROUP_MB: only the size limits a group
    uint64_t group_slots_max = GROUP_BYTES / sizeof(uint2);  // ADACOMP_SELECT_GROUP_MB=<n> (0: one group)
};

SelectHooks read_select_hooks() {
    SelectHooks hk;
    if (const char *e = std::getenv("ADACOMP_SELECT_SMALL")) hk.small = e[0] != '0';
    if (const char *e = std::getenv("ADACOMP_SELECT_FUSED")) hk.fused = e[0] != '0';
    if (const char *gm = std::getenv("ADACOMP_SELECT_GROUP_MB")) {
        const long mb = std::atol(gm);
        hk.group_slots_max = mb > 0 ? (uint64_t)mb * 1048576ull / sizeof(uint2) : ~0ull;
        hk.group_tensors = false;
    }
    return hk;
}

int make_plan(const uint64_t *n, const float *const *data, uint32_t L, double rate,
              const uint64_t *k_override, const SelectHooks &hk, Plan &plan) {
    if (!(rate >= 0.0 && rate <= 1.0)) return ADACOMP_ERR_RATE;
    plan.desc.clear();
    plan.number.clear();
    plan.opens.clear();
    plan.off.assign((size_t)L + 1, 0);
    uint64_t seg = 0, cand = 0, out = 0, sblk = 0, wblk = 0, iblk = 0;
    // one workgroup per small tensor, if together they stay cache-sized
    uint64_t small_elems = 0;
    for (uint32_t l = 0; l < L; ++l)
        if (n[l] <= SMALL_MAX) small_elems += n[l];
    const bool small_ok = small_elems <= SMALL_TOTAL && hk.small;
    const uint64_t group_slots_max = hk.group_slots_max;
    uint64_t pack = 0, cand_max = 0;
    Group grp{0, 0, 0, 0};
    for (uint32_t l = 0; l < L; ++l) {
        if (n[l] > 0xffffffffull) return ADACOMP_ERR_LAYER_TOO_LARGE;
        uint64_t k64 = k_override ? k_override[l] : adacomp_count(n[l], rate);
        if (k64 > n[l]) return ADACOMP_ERR_K_RANGE;
        LayerDesc d{};
        bool opens = false;
        plan.off[l] = out;
        d.g = data ? data[l] : nullptr;
        d.n = (uint32_t)n[l];
        d.k = (uint32_t)k64;
        d.vec = data ? (((uintptr_t)data[l] & 15u) == 0) : 1;
        d.out_off = out;
        d.cand_base = cand;
        d.seg_base = (uint32_t)seg;
        d.sblk_base = (uint32_t)sblk;
        d.wblk_base = (uint32_t)wblk;
        d.iblk_base = (uint32_t)iblk;
        d.npieces = (uint32_t)((n[l] + PIECE - 1) / PIECE);
        d.stride = 1;
        if (d.n == 0 || d.k == 0) {
            d.mode = MODE_EMPTY;
        } else if (d.k == d.n) {
            d.mode = MODE_IDENTITY;
            iblk += (n[l] + IDENT_TILE - 1) / IDENT_TILE;
        } else if (small_ok && d.n <= SMALL_MAX) {
            d.mode = MODE_SMALL;
            plan.small.push_back(SmallEntry{d.g, d.n, l});
        } else {
            d.nseg = (uint32_t)((n[l] + WSEG - 1) / WSEG);
            d.mode = (8ull * d.k > d.n) ? MODE_DENSE : MODE_FILTER;
            if (d.mode == MODE_FILTER) {
                // sample about 128K elements or more, at most one piece in 64
                uint32_t stride = 64;
                while (stride > 1 && d.npieces / stride < 512) stride >>= 1;
                double m_est = 0;
                for (;; stride >>= 1) {
                    d.stride = stride;
                    d.npieces_s = (d.npieces + stride - 1) / stride;
                    if (stride == 1) {
                        d.target = d.k;
                        m_est = (double)d.k * 1.5;
                        break;
                    }
                    // exact number of sampled elements: only the last piece can be short
                    uint64_t ns = (uint64_t)d.npieces_s * PIECE;
                    if (sample_piece(d.npieces_s - 1, stride, d.npieces) == d.npieces - 1)
                        ns -= (uint64_t)d.npieces * PIECE - n[l];
                    double f = (double)ns / (double)n[l];
                    double kf = (double)d.k * f;
                    double tgt = std::ceil(kf + 6.0 * std::sqrt(kf) + 8.0);
                    m_est = 1.5 * tgt / f;
                    if (m_est <= (double)n[l] / 4.0) {
                        d.target = (uint32_t)tgt;
                        break;
                    }
                }
                double per_seg = m_est * (double)WSEG / (double)n[l];
                // a multiple of 16 entries: every region starts on a 128-byte line and is
                // written in whole lines
                uint64_t cap = ((uint64_t)std::ceil(3.0 * per_seg) + 64 + 15) & ~15ull;
                d.cap = (uint32_t)std::min<uint64_t>(cap, WSEG);
                const uint64_t slots = (uint64_t)d.nseg * d.cap;
                if (grp.filters && (cand + slots > group_slots_max ||
                                    (hk.group_tensors && grp.filters >= GROUP_TENSORS))) {  // close the group, reuse the regions
                    grp.l1 = (uint32_t)plan.desc.size();
                    plan.groups.push_back(grp);
                    grp = Group{grp.l1, grp.l1, 0, 0};
                    cand = 0;
                    opens = true;
                }
                d.cand_base = cand;
                d.pack_base = pack;
                cand += slots;
                pack += slots;
                cand_max = std::max(cand_max, cand);
                ++grp.filters;
                d.fused = hk.fused && d.nseg <= FUSE_MAX_SEG && m_est <= (double)FUSE_MAX_CAND && d.cap <= FUSE_MAX_CAP;
                if (d.fused) plan.any_fused = true;
                else ++grp.unfused;
                sblk += (d.npieces_s + SPIECES - 1) / SPIECES;
            }
            seg += d.nseg;
            wblk += (d.nseg + WAVES - 1) / WAVES;
        }
        // small and empty tensors never reach the pipeline's kernels: no descriptor, nothing to upload
        if (d.mode != MODE_EMPTY && d.mode != MODE_SMALL) {
            plan.desc.push_back(d);
            plan.number.push_back(l);
            plan.opens.push_back(opens);
        }
        out += d.k;
    }
    // the gather's shape follows the fullest regions of the call
    uint32_t cap_max = 0;
    for (const LayerDesc &d : plan.desc)
        if (d.mode == MODE_FILTER) cap_max = std::max(cap_max, d.cap);
    plan.gsegs = cap_max >= GATHER_FULL_CAP ? GSEGS_FULL : cap_max >= GATHER_MID_CAP ? GSEGS_MID : GSEGS;
    uint64_t gblk = 0;
    for (LayerDesc &d : plan.desc) {
        d.gblk_base = (uint32_t)gblk;
        if (d.mode == MODE_FILTER) gblk += (d.nseg + WAVES * plan.gsegs - 1) / (WAVES * plan.gsegs);
    }
    if (seg > 0xffffffffull || sblk > 0x7fffffffull || wblk > 0x7fffffffull ||
        iblk > 0x7fffffffull || gblk > 0x7fffffffull)
        return ADACOMP_ERR_LAYER_TOO_LARGE;
    grp.l1 = (uint32_t)plan.desc.size();
    plan.groups.push_back(grp);
    if (plan.groups.size() > 1) {
        // The pass above says how many groups the limits ask for.  The same number of groups with the
        // filtered tensors spread evenly over them makes the launches equally long (1600 equal tensors:
        // 800 + 800 instead of 1024 + 576); kept unless a group would then exceed the size limit.
        const size_t ng = plan.groups.size();
        uint32_t nf = 0;
        for (const Group &g : plan.groups) nf += g.filters;
        const uint32_t per = (uint32_t)((nf + ng - 1) / ng);
        std::vector<Group> even;
        std::vector<char> opens(plan.desc.size(), 0);
        std::vector<uint64_t> base(plan.desc.size(), 0);
        Group cur{0, 0, 0, 0};
        uint64_t c = 0, c_max = 0;
        bool fits = true;
        for (uint32_t i = 0; i < plan.desc.size() && fits; ++i) {
            const LayerDesc &d = plan.desc[i];
            if (d.mode != MODE_FILTER) continue;
            const uint64_t slots = (uint64_t)d.nseg * d.cap;
            if (cur.filters >= per) {
                cur.l1 = i;
                even.push_back(cur);
                cur = Group{i, i, 0, 0};
                c = 0;
                opens[i] = 1;
            }
            if (cur.filters && c + slots > group_slots_max) fits = false;
            base[i] = c;
            c += slots;
            c_max = std::max(c_max, c);
            ++cur.filters;
            if (!d.fused) ++cur.unfused;
        }
        if (fits) {
            cur.l1 = (uint32_t)plan.desc.size();
            even.push_back(cur);
            plan.groups = even;
            plan.opens = opens;
            for (uint32_t i = 0; i < plan.desc.size(); ++i)
                if (plan.desc[i].mode == MODE_FILTER) plan.desc[i].cand_base = base[i];
            cand_max = c_max;
        }
    }
    plan.off[L] = out;
    plan.desc.push_back(LayerDesc{});
    LayerDesc &e = plan.desc.back();
    e.out_off = out;
    e.cand_base = cand_max;
    e.pack_base = pack;
    e.seg_base = (uint32_t)seg;
    e.sblk_base = (uint32_t)sblk;
    e.wblk_base = (uint32_t)wblk;
    e.iblk_base = (uint32_t)iblk;
    e.gblk_base = (uint32_t)gblk;
    plan.nseg_total = seg;
    plan.cand_total = cand_max;
    plan.pack_total = pack;
    plan.out_total = out;
    std::stable_sort(plan.small.begin(), plan.small.end(),
                     [](const SmallEntry &a, const SmallEntry &b) { return a.n > b.n; });
    return ADACOMP_OK;
}

// L: the tensors of the pipeline (plan.desc.size() - 1)
void carve(const Plan &plan, uint32_t L, void *base, Workspace &ws) {
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void *p = base ? (char *)base + off : nullptr;
        off += align_up(bytes ? bytes : 1, 256);
        return p;
    };
    ws.desc = (LayerDesc *)take(((size_t)L + 1) * sizeof(LayerDesc));
    ws.state = (LayerState *)take((size_t)L * sizeof(LayerState));
    ws.hist = (uint32_t *)take((size_t)L * BINS * sizeof(uint32_t));
    ws.redo = (uint32_t *)take(((size_t)L + 1) * sizeof(uint32_t));
    ws.seg_cnt = (uint32_t *)take(plan.nseg_total * sizeof(uint32_t));
    ws.seg_res = (uint32_t *)take(plan.nseg_total * sizeof(uint32_t));
    ws.seg_gt = (uint32_t *)take(plan.nseg_total * sizeof(uint32_t));
    ws.seg_eq = (uint32_t *)take(plan.nseg_total * sizeof(uint32_t));
    ws.chunk_base = (uint32_t *)take(((size_t)L + 1) * sizeof(uint32_t));
    ws.seg_off = (uint32_t *)take(plan.nseg_total * sizeof(uint32_t));
    ws.cand = (uint2 *)take(plan.cand_total * sizeof(uint2));
    ws.pack_idx = (uint32_t *)take(plan.pack_total * sizeof(uint32_t));
    ws.pack_val = (uint32_t *)take(plan.pack_total * sizeof(uint32_t));
    ws.small = (SmallEntry *)take(plan.small.size() * sizeof(SmallEntry));
    ws.compact = (CompactDesc *)take((size_t)L * sizeof(CompactDesc));
    ws.bytes = off;
}

// ------------------------------------------------------------------ device side

template <uint32_t LayerDesc::*BASE>
__device__ __forceinline__ uint32_t find_layer(const LayerDesc *d, uint32_t L, uint32_t blk) {
    uint32_t lo = 0, hi = L;  // the last l with d[l].*BASE <= blk owns workgroup blk
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (d[mid].*BASE <= blk) lo = mid; else hi = mid;
    }
    return lo;
}

// The same among the tensors [lo, hi) when d[lo].*BASE <= blk < d[hi].*BASE (d[hi] exists: the table
// ends with an entry of totals).  The first probe is placed by proportion, which is the answer when
// the tensors of the range are equally large: two rounds of loads instead of log2(L) dependent ones
// in front of a workgroup's first data load.  Any other layout falls through to the bisection.
template <uint32_t LayerDesc::*BASE>
__device__ __forceinline__ uint32_t find_layer_in(const LayerDesc *d, uint32_t lo, uint32_t hi, uint32_t blk) {
    const uint32_t b_lo = d[lo].*BASE, b_hi = d[hi].*BASE;
    uint32_t g = lo + (uint32_t)((float)(blk - b_lo) * (float)(hi - lo) / (float)(b_hi - b_lo));
    if (g >= hi) g = hi - 1;
    const uint32_t b_g = d[g].*BASE, b_next = d[g + 1].*BASE;
    if (b_g <= blk) {
        if (b_next > blk) return g;
        lo = g + 1;  // d[g + 1].*BASE <= blk
    } else {
        hi = g;
    }
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (d[mid].*BASE <= blk) lo = mid; else hi = mid;
    }
    return lo;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// Tensor pointers come out of descriptor tables in memory, so the compiler cannot tell that
// they point to device global memory and would emit generic (flat) loads; these typedefs say so.
typedef const __attribute__((address_space(1))) uint32_t *global_u32_ptr;
typedef const __attribute__((address_space(1))) u32x4 *global_u32x4_ptr;

// 16 bytes at element `base` of a 16-byte aligned array.  STREAM marks data that is read
// once (non-temporal: it does not displace cached lines).
template <bool STREAM>
__device__ __forceinline__ uint4 load4_full(const float *g, uint32_t base) {
    global_u32x4_ptr p = (global_u32x4_ptr)(reinterpret_cast<const uint32_t *>(g) + base);
    const u32x4 t = STREAM ? __builtin_nontemporal_load(p) : *p;
    return make_uint4(t.x, t.y, t.z, t.w);
}

// Four consecutive elements starting at `base`; elements at or beyond `lim` read as 0.
template <bool STREAM = false>
__device__ __forceinline__ uint4 load4(const float *g, uint32_t base, uint32_t lim, bool vec) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (base >= lim) return v;
    if (vec && lim - base >= 4) return load4_full<STREAM>(g, base);
    global_u32_ptr p = (global_u32_ptr)(reinterpret_cast<const uint32_t *>(g) + base);
    v.x = p[0];
    if (lim - base > 1) v.y = p[1];
    if (lim - base > 2) v.z = p[2];
    if (lim - base > 3) v.w = p[3];
    return v;
}

// What the descent, count and emit kernels read for one tensor: the tensor itself (position
// is the index) or its packed candidates (explicit index array).
struct Source {
    const uint32_t *val;  // value bits
    const uint32_t *idx;  // explicit indices, or nullptr when the position is the index
    uint32_t m;           // elements
    uint32_t chunk;       // elements per wave chunk
    bool vec;             // 16-byte aligned
};

// Visit the elements [lo, hi) of a source with one wave, in order: the visitor is called
// wave-wide once per piece of up to 256 elements with each lane holding 4 consecutive elements
// (idx[c], bits[c]); nvalid of them are inside the range.  WITH_IDX loads explicit indices.
// A tensor that does not start on a 16-byte boundary (a view into a flat buffer) is read on the
// aligned grid all the same: the up to 3 elements in front of the first boundary inside the
// range make a short piece of their own, and the pieces after it are shifted by that much.
template <bool WITH_IDX, bool STREAM = false, int NLOAD = 4, class F>
__device__ __forceinline__ void visit_range(const Source &src, uint32_t lo, uint32_t hi, F &&f) {
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    const float *vals = reinterpret_cast<const float *>(src.val);
    const float *idxs = reinterpret_cast<const float *>(src.idx);
    const bool with_idx = WITH_IDX && idxs != nullptr;
    constexpr uint32_t round = NLOAD * PIECE;  // elements per wave iteration: NLOAD 16-byte loads per lane in flight
    uint32_t r = lo;
    bool aligned = src.vec;  // element r of the source lies on a 16-byte boundary
    if (!aligned && r < hi) {
        const uint32_t mis = (uint32_t)((reinterpret_cast<uintptr_t>(vals) >> 2) & 3u);  // elements past a boundary at element 0
        const uint32_t head = (4u - ((r + mis) & 3u)) & 3u;
        if (head) {  // uniform
            const uint32_t h_hi = hi - r > head ? r + head : hi;
            const uint32_t first = r + lane * 4;
            const uint4 v = load4<STREAM>(vals, first, h_hi, false);
            uint32_t idx[4] = {first, first + 1, first + 2, first + 3};
            const uint32_t bits[4] = {v.x, v.y, v.z, v.w};
            const uint32_t nvalid = first >= h_hi ? 0u : (h_hi - first < 4u ? h_hi - first : 4u);
            f(idx, bits, nvalid);
            r = h_hi;
        }
        aligned = true;
    }
    if (aligned) {
        // whole rounds of an aligned source: plain vector loads, every element valid
        for (; hi - r >= round; r += round) {
            uint4 v[NLOAD], x[NLOAD];
#pragma unroll
            for (int j = 0; j < NLOAD; ++j) v[j] = load4_full<STREAM>(vals, r + j * PIECE + lane * 4);
            if (with_idx) {
#pragma unroll
                for (int j = 0; j < NLOAD; ++j) x[j] = load4_full<false>(idxs, r + j * PIECE + lane * 4);
            }
#pragma unroll
            for (int j = 0; j < NLOAD; ++j) {
                const uint32_t first = r + j * PIECE + lane * 4;
                uint32_t idx[4] = {first, first + 1, first + 2, first + 3};
                if (with_idx) {
                    idx[0] = x[j].x;
                    idx[1] = x[j].y;
                    idx[2] = x[j].z;
                    idx[3] = x[j].w;
                }
                const uint32_t bits[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
                f(idx, bits, 4u);
            }
        }
    }
    // the rest: an unaligned source, or the ragged end of the range (hi may be 2^32 - 1: the
    // position is advanced only while it stays below hi, it must not wrap)
    for (; r < hi; r = hi - r > PIECE ? r + PIECE : hi) {
        const uint32_t first = r + lane * 4;
        const uint4 v = load4<STREAM>(vals, first, hi, aligned);
        uint32_t idx[4] = {first, first + 1, first + 2, first + 3};
        if (with_idx) {
            const uint4 x = load4(idxs, first, hi, true);
            idx[0] = x.x;
            idx[1] = x.y;
            idx[2] = x.z;
            idx[3] = x.w;
        }
        const uint32_t bits[4] = {v.x, v.y, v.z, v.w};
        const uint32_t nvalid = first >= hi ? 0u : (hi - first < 4u ? hi - first : 4u);
        f(idx, bits, nvalid);
    }
}

__device__ __forceinline__ Source source_of(const LayerDesc &d, const LayerState &st, const Workspace &ws) {
    if (st.use_dense) return Source{reinterpret_cast<const uint32_t *>(d.g), nullptr, d.n, WSEG, d.vec != 0};
    return Source{ws.pack_val + d.pack_base, ws.pack_idx + d.pack_base, st.m, VCHUNK, true};
}

// Workgroup-wide: the largest bin b of h[0..nbins) whose suffix sum (bins >= b) reaches
// `target`, and the sum `above` of the bins > b.  If even the total falls short, b = 0.
// nbins <= BINS, BLOCK threads, 16 consecutive bins per thread.  All threads return
// the same pair.
__device__ void find_bin_from_top(const uint32_t *h, uint32_t nbins, uint32_t target,
                                  uint32_t &bin, uint32_t &above) {
    __shared__ uint32_t s_suffix[BLOCK + 1];
    __shared__ uint32_t s_bin, s_above;
    const uint32_t t = threadIdx.x;
    uint32_t c[16];
    uint32_t sum = 0;
#pragma unroll
    for (int b = 0; b < 16; ++b) {
        const uint32_t i = t * 16 + b;
        c[b] = i < nbins ? h[i] : 0u;
        sum += c[b];
    }
    if (t == 0) {
        s_bin = 0;
        s_above = 0;
        s_suffix[BLOCK] = 0;
    }
    s_suffix[t] = sum;
    __syncthreads();
    for (uint32_t step = 1; step < BLOCK; step <<= 1) {  // inclusive suffix scan
        const uint32_t add = t + step < BLOCK ? s_suffix[t + step] : 0u;
        __syncthreads();
        s_suffix[t] += add;
        __syncthreads();
    }
    const uint32_t incl = s_suffix[t], excl = s_suffix[t + 1];
    if (excl < target && target <= incl) {
        uint32_t acc = excl;
        for (int b = 15; b >= 0; --b) {
            if (acc + c[b] >= target) {
                s_bin = t * 16 + b;
                s_above = acc;
                break;
            }
            acc += c[b];
        }
    }
    if (t == 0 && incl < target) s_above = incl - c[0];
    __syncthreads();
    bin = s_bin;
    above = s_above;
    __syncthreads();
}

// LDS histogram helpers ---------------------------------------------------------
__device__ __forceinline__ void lds_hist_clear(uint32_t *h) {
    for (uint32_t i = threadIdx.x; i < BINS; i += BLOCK) h[i] = 0;
    __syncthreads();
}

__device__ __forceinline__ void lds_hist_flush(const uint32_t *h, uint32_t *global_hist, uint32_t nbins) {
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < nbins; i += BLOCK) {
        const uint32_t c = h[i];
        if (c) atomicAdd(global_hist + i, c);
    }
}

// Add one matching element per (lane, component) to an LDS histogram.  Zero keys, which
// can be half of a tensor, are counted with a ballot instead of 64 colliding atomics.
template <int NC>
__device__ __forceinline__ void lds_hist_add(uint32_t *h, const uint32_t (&key)[NC], const bool (&match)[NC],
                                             const uint32_t (&bin)[NC], uint32_t &zero_run) {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const bool z = match[c] && key[c] == 0;
        zero_run += popc64(__ballot(z));
        if (match[c] && !z) atomicAdd(&h[bin[c]], 1u);
    }
}

// Elements [lo, hi) of segment s of a tensor.  Segments are WSEG elements long; in a tensor that does
// not start on a 128-byte boundary (a view into a flat buffer) the borders between them are moved to
// the next such boundary (by the `head` < 32 elements in front of the tensor's first one), so that
// only the tensor's first segment has a head to peel or loads that straddle cache lines.
__device__ __forceinline__ void segment_range(const LayerDesc &d, uint32_t s, uint32_t &lo, uint32_t &hi) {
    const uint32_t head = (uint32_t)((0u - (reinterpret_cast<uintptr_t>(d.g) >> 2)) & 31u);
    const uint64_t b0 = s ? (uint64_t)s * WSEG + head : 0u, b1 = (uint64_t)(s + 1) * WSEG + head;
    lo = b0 < d.n ? (uint32_t)b0 : d.n;
    hi = (b1 < d.n && s + 1 < d.nseg) ? (uint32_t)b1 : d.n;  // the last segment ends with the tensor
}

// ---- step 1: sample histogram on the top 12 key bits -----------------------------
__global__ __launch_bounds__(BLOCK) void k_sample_hist(Workspace ws, uint32_t L) {
    __shared__ uint32_t h[BINS];
    const uint32_t l = find_layer_in<&LayerDesc::sblk_base>(ws.desc, 0, L, blockIdx.x);
    const LayerDesc d = ws.desc[l];
    const uint32_t b = blockIdx.x - d.sblk_base;
    const uint32_t wave = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
    lds_hist_clear(h);
    const uint32_t p_lo = b * SPIECES;
    const uint32_t p_hi = p_lo + SPIECES < d.npieces_s ? p_lo + SPIECES : d.npieces_s;
    // a tensor that does not start on a 16-byte boundary: a true sample (one piece in several) reads the
    // 256 elements from the first boundary inside each sampled piece, so that the loads are 16 bytes wide
    // (which elements are sampled does not matter to the result); a tensor read completely keeps its pieces
    const uint32_t shift = (!d.vec && d.stride > 1) ? (4u - (uint32_t)((reinterpret_cast<uintptr_t>(d.g) >> 2) & 3u)) & 3u : 0u;
    const bool wide = d.vec != 0 || shift != 0;
    uint32_t zero_run = 0;
    for (uint32_t p0 = p_lo + wave * 4; p0 < p_hi; p0 += WAVES * 4) {
        uint4 v[4];
        uint32_t first[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t p = p0 + j;
            uint32_t piece = 0;
            if (p < p_hi) {
                const uint32_t jit = ((p * 2654435761u) >> 16) & (d.stride - 1);
                const uint64_t q = (uint64_t)p * d.stride + jit;
                piece = q < d.npieces ? (uint32_t)q : d.npieces - 1;
            }
            first[j] = piece * PIECE + shift + lane * 4;
            v[j] = load4<true>(d.g, first[j], p < p_hi ? d.n : 0u, wide);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (p0 + j >= p_hi) break;
            const uint32_t nvalid = first[j] >= d.n ? 0u : (d.n - first[j] < 4u ? d.n - first[j] : 4u);
            const uint32_t bits[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
            uint32_t key[4], bin[4];
            bool match[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                key[c] = mag_key(bits[c]);
                bin[c] = key[c] >> 19;
                match[c] = (uint32_t)c < nvalid;
            }
            lds_hist_add<4>(h, key, match, bin, zero_run);
        }
    }
    if (lane == 0 && zero_run) atomicAdd(&h[0], zero_run);
    lds_hist_flush(h, ws.hist + (size_t)l * BINS, BINS);
}

// ---- step 2: initialise per-tensor state, choose the filter threshold -----------
__global__ __launch_bounds__(BLOCK) void k_pick(Workspace ws) {
    const uint32_t l = blockIdx.x;
    const LayerDesc d = ws.desc[l];
    uint32_t *h = ws.hist + (size_t)l * BINS;
    uint32_t t_lo = 0, t_reserve = 0;
    if (d.mode == MODE_FILTER) {
        uint32_t bin, above;
        find_bin_from_top(h, BINS, d.target, bin, above);
        t_lo = bin << 19;
        t_reserve = t_lo;
        if (d.stride > 1) {
            // The margin in d.target is that of independent draws.  Where large entries cluster (rows
            // of a weight matrix), a sample of 1 KB pieces can be off by far more: the filter also
            // counts against the threshold that three times as many sampled entries reach, and
            // check / gather fall back on that one before giving up on the candidates altogether.
            const uint32_t wide = d.target > 0x55555555u ? 0xffffffffu : 3u * d.target;
            find_bin_from_top(h, BINS, wide, bin, above);
            t_reserve = bin << 19;
        }
        for (uint32_t i = threadIdx.x; i < BINS; i += BLOCK) h[i] = 0;
    }
    if (threadIdx.x == 0) {
        LayerState st;
        st.t_lo = t_lo;
        st.t_reserve = t_reserve;
        st.refilter = 0;
        st.use_dense = d.mode == MODE_DENSE;
        st.prefix = 0;
        st.k_rem = d.k;
        st.T = 0;
        st.r = 0;
        st.m = d.n;          // the dense source, unless the check finds the candidates usable
        st.nchunk = d.nseg;
        st.done = 0;
        st.pad = 0;
        ws.state[l] = st;
        if (l == 0) ws.redo[0] = 0;
    }
}

// ---- step 3: the streaming read; ordered compaction of key >= t_lo per wave ------
// Candidates are staged in LDS (one private buffer per wave) and leave as coalesced
// 8-byte (index, value) stores of whole 128-byte lines into the segment's own region of `cap`
// slots; what does not fit is counted, not stored (a count above `cap` tells the readers to
// filter that segment again).
constexpr uint32_t FSTAGE = 272;  // staged candidates per wave: a 256-element piece on top of a 15-entry remainder

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__global__ __launch_bounds__(BLOCK) void k_filter(Workspace ws, uint32_t l0, uint32_t l1, uint32_t blk0) {
    __shared__ uint2 s_stage[WAVES][FSTAGE];
    const uint32_t blk = blk0 + xcd_contiguous_block();  // workgroup number across all groups of tensors; the launch covers tensors [l0, l1)
    const uint32_t l = find_layer_in<&LayerDesc::wblk_base>(ws.desc, l0, l1, blk);
    const LayerDesc d = ws.desc[l];
    if (d.mode != MODE_FILTER) return;
    const uint32_t wave = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
    const uint32_t seg = (blk - d.wblk_base) * WAVES + wave;
    if (seg >= d.nseg) return;
    const uint32_t t_lo = ws.state[l].t_lo, t_reserve = ws.state[l].t_reserve;
    uint32_t reserve = 0;  // entries with key >= t_reserve (wave-uniform)
    uint2 *region = ws.cand + d.cand_base + (uint64_t)seg * d.cap;
    uint2 *stage = s_stage[wave];
    const uint32_t cap = d.cap;
    uint32_t lo, hi;
    segment_range(d, seg, lo, hi);
    const Source src{reinterpret_cast<const uint32_t *>(d.g), nullptr, d.n, WSEG, d.vec != 0};
    uint32_t staged = 0;   // candidates in the stage (wave-uniform)
    uint32_t written = 0;  // candidates of this segment already flushed (may exceed cap: those are dropped)
    // Whole 128-byte lines (16 entries) only: `written` stays a multiple of 16 until the last
    // flush, which rounds up (the slack holds stale LDS contents and is never read, the
    // region's fill count says where it ends).  Entries past cap are counted, not stored.
    auto flush = [&](bool last) {
        wave_lds_fence();
        const uint32_t n_out = last ? (staged + 15u) & ~15u : staged & ~15u;
        for (uint32_t e = lane; e < n_out; e += WAVE) {
            // streaming stores: the lines are read once more, by the finish (or gather) of the group, and
            // written whole.  Whole steps on a settled box: filter 9.28 against 9.61 ms with plain stores,
            // finish 0.84 against 0.81 ms
            if (written + e < cap) {
                const uint2 t = stage[e];
                u32x2 w;
                w.x = t.x;
                w.y = t.y;
                __builtin_nontemporal_store(w, (__attribute__((address_space(1))) u32x2 *)&region[written + e]);
            }
        }
        const uint32_t keep = last ? 0u : staged - n_out;  // < 16 entries move to the front
        uint2 moved = make_uint2(0, 0);
        if (lane < keep) moved = stage[n_out + lane];
        wave_lds_fence();
        if (lane < keep) stage[lane] = moved;
        wave_lds_fence();
        written += last ? staged : n_out;
        staged = keep;
    };
    visit_range<false, true, FILTER_NLOAD>(src, lo, hi, [&](const uint32_t(&idx)[4], const uint32_t(&bits)[4], uint32_t nvalid) {
        bool f[4];
        uint64_t m[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            f[c] = (uint32_t)c < nvalid && mag_key(bits[c]) >= t_lo;
            m[c] = __ballot(f[c]);
            reserve += popc64(__ballot((uint32_t)c < nvalid && mag_key(bits[c]) >= t_reserve));
        }
        if ((m[0] | m[1] | m[2] | m[3]) == 0) return;
        const uint32_t found = popc64(m[0]) + popc64(m[1]) + popc64(m[2]) + popc64(m[3]);
        if (staged + found > FSTAGE) flush(false);
        uint32_t pos = staged + lanes_below(m[0]) + lanes_below(m[1]) + lanes_below(m[2]) + lanes_below(m[3]);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (f[c]) stage[pos++] = make_uint2(idx[c], bits[c]);
        }
        staged += found;
    });
    flush(true);
    if (lane == 0) {
        ws.seg_cnt[d.seg_base + seg] = written;
        ws.seg_res[d.seg_base + seg] = reserve;
    }
}

// ---- step 4: candidate offsets per segment; are the candidates usable? -------------
// One workgroup per tensor.  A tensor of a billion elements has 122,000 segments: 1024 threads
// with 4 consecutive counts each, so that the serial part is tens of rounds, not hundreds.
constexpr uint32_t CBLOCK = 1024, CITEMS = 4;

// out[i] = load(0) + ... + load(i - 1) for i < n, by one workgroup of CBLOCK threads; returns the
// total (the same in all threads).  `out` may be the array that `load` reads.
template <class Load, class Store>
__device__ __forceinline__ uint32_t scan_store(Load load, Store store, uint32_t n, uint32_t *s_wave) {
    uint32_t carry = 0;
    for (uint32_t i0 = 0; i0 < n; i0 += CBLOCK * CITEMS) {
        const uint32_t i = i0 + threadIdx.x * CITEMS;
        uint32_t c[CITEMS], sum = 0;
#pragma unroll
        for (uint32_t j = 0; j < CITEMS; ++j) {
            c[j] = i + j < n ? load(i + j) : 0u;
            sum += c[j];
        }
        uint32_t total;
        uint32_t run = carry + block_exclusive_scan<CBLOCK / WAVE>(sum, s_wave, total);
#pragma unroll
        for (uint32_t j = 0; j < CITEMS; ++j) {
            if (i + j < n) store(i + j, run);
            run += c[j];
        }
        carry += total;  // the callers' sums stay below 2^32
    }
    return carry;
}

template <class Load>
__device__ __forceinline__ uint32_t scan_array(Load load, uint32_t *out, uint32_t n, uint32_t *s_wave) {
    return scan_store(load, [&](uint32_t i, uint32_t v) { out[i] = v; }, n, s_wave);
}

// ---- descriptors from their compact form ----------------------------------------------
// One workgroup: per tensor the fields that follow from its own size and count, then the
// prefix sums over the tensors that place its segments, workgroups and candidates.
__global__ __launch_bounds__(CBLOCK) void k_expand(Workspace ws, uint32_t L, const uint64_t *layer_off, uint32_t gsegs) {
    __shared__ uint32_t s_wave[CBLOCK / WAVE];
    __shared__ uint32_t s_carry;
    for (uint32_t i = threadIdx.x; i < L; i += CBLOCK) {
        const CompactDesc c = ws.compact[i];
        LayerDesc d{};
        d.g = c.g;
        d.n = c.n;
        d.out_off = layer_off[c.l];
        d.k = (uint32_t)(layer_off[c.l + 1] - d.out_off);
        d.mode = c.bits & 7u;
        d.fused = (c.bits >> 3) & 1u;
        d.stride = 1u << ((c.bits >> 5) & 7u);
        d.cap = c.bits >> 8;
        d.target = c.target;
        d.vec = ((uintptr_t)c.g & 15u) == 0;
        d.npieces = (uint32_t)(((uint64_t)c.n + PIECE - 1) / PIECE);
        if (d.mode == MODE_FILTER) d.npieces_s = (d.npieces + d.stride - 1) / d.stride;
        if (d.mode == MODE_FILTER || d.mode == MODE_DENSE) d.nseg = (uint32_t)(((uint64_t)c.n + WSEG - 1) / WSEG);
        ws.desc[i] = d;
    }
    __syncthreads();
    LayerDesc *D = ws.desc;
    uint32_t tot;
    tot = scan_store([&](uint32_t i) { return D[i].nseg; }, [&](uint32_t i, uint32_t v) { D[i].seg_base = v; }, L, s_wave);
    if (threadIdx.x == 0) D[L].seg_base = tot;
    tot = scan_store([&](uint32_t i) { return D[i].mode == MODE_FILTER ? (D[i].npieces_s + SPIECES - 1) / SPIECES : 0u; },
                     [&](uint32_t i, uint32_t v) { D[i].sblk_base = v; }, L, s_wave);
    if (threadIdx.x == 0) D[L].sblk_base = tot;
    tot = scan_store([&](uint32_t i) { return (D[i].nseg + WAVES - 1) / WAVES; }, [&](uint32_t i, uint32_t v) { D[i].wblk_base = v; }, L, s_wave);
    if (threadIdx.x == 0) D[L].wblk_base = tot;
    tot = scan_store([&](uint32_t i) { return D[i].mode == MODE_IDENTITY ? (uint32_t)(((uint64_t)D[i].n + IDENT_TILE - 1) / IDENT_TILE) : 0u; },
                     [&](uint32_t i, uint32_t v) { D[i].iblk_base = v; }, L, s_wave);
    if (threadIdx.x == 0) D[L].iblk_base = tot;
    tot = scan_store([&](uint32_t i) { return D[i].mode == MODE_FILTER ? (D[i].nseg + WAVES * gsegs - 1) / (WAVES * gsegs) : 0u; },
                     [&](uint32_t i, uint32_t v) { D[i].gblk_base = v; }, L, s_wave);
    if (threadIdx.x == 0) D[L].gblk_base = tot;
    // candidate slots in units of 16 (a region is whole 128-byte lines): the packed arrays run through
    // all tensors; the regions start again at 0 with every group
    tot = scan_store([&](uint32_t i) { return D[i].mode == MODE_FILTER ? (uint32_t)((uint64_t)D[i].nseg * D[i].cap / 16) : 0u; },
                     [&](uint32_t i, uint32_t v) { D[i].pack_base = 16ull * v; }, L, s_wave);
    if (threadIdx.x == 0) D[L].pack_base = 16ull * tot;
    __syncthreads();
    // slots before the tensor's group: the running maximum of (slots before a tensor that opens a group)
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (uint32_t i0 = 0; i0 < L; i0 += CBLOCK) {
        const uint32_t i = i0 + threadIdx.x;
        const uint32_t lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
        const uint32_t before = i < L ? (uint32_t)(D[i].pack_base / 16) : 0u;
        uint32_t m = i < L && ((ws.compact[i].bits >> 4) & 1u) ? before : 0u;
#pragma unroll
        for (int o = 1; o < WAVE; o <<= 1) {
            const uint32_t y = __shfl_up(m, o);
            if (lane >= (uint32_t)o && y > m) m = y;
        }
        if (lane == WAVE - 1) s_wave[wave] = m;
        __syncthreads();
        uint32_t prev = s_carry;
        for (uint32_t w = 0; w < wave; ++w) prev = s_wave[w] > prev ? s_wave[w] : prev;
        if (prev > m) m = prev;
        if (i < L) D[i].cand_base = 16ull * (before - m);
        __syncthreads();
        if (threadIdx.x == CBLOCK - 1) s_carry = m;
        __syncthreads();
    }
}

// Whole workgroup.  Returns true if the packed candidates will be the source of the descent.
__device__ __forceinline__ bool check_tensor(const Workspace &ws, uint32_t l, const LayerDesc &d, uint32_t *s_wave) {
    // the count is exact also where the region overflowed (the gather reads such a segment again)
    const uint32_t *cnt = ws.seg_cnt + d.seg_base, *res = ws.seg_res + d.seg_base;
    uint32_t m = scan_array([&](uint32_t i) { return cnt[i]; }, ws.seg_off + d.seg_base, d.nseg, s_wave);
    const uint64_t room = std::min<uint64_t>((uint64_t)d.nseg * d.cap, d.n / 4);  // what the packed array holds, and is worth packing
    bool refilter = false;
    if (m < d.k) {
        // the sample misjudged: the candidates of the reserve threshold, which the filter only counted
        m = scan_array([&](uint32_t i) { return res[i]; }, ws.seg_off + d.seg_base, d.nseg, s_wave);
        refilter = true;
    }
    const bool usable = !(m < d.k || m > room);
    if (threadIdx.x == 0) {
        if (!usable) {
            ws.state[l].use_dense = 1;  // m and nchunk keep the dense-source values
        } else {
            ws.state[l].m = m;
            ws.state[l].nchunk = (m + VCHUNK - 1) / VCHUNK;
            if (refilter) {
                ws.state[l].t_lo = ws.state[l].t_reserve;
                ws.state[l].refilter = 1;
            }
        }
    }
    return usable;
}

// ---- step 5: pack the candidates of a tensor, in index order --------------------------
// One wave packs the segments s0 .. s0 + GS - 1 of tensor l.  refilter_all: the regions do not hold
// the candidates of the threshold in force (it was replaced by the reserve threshold, or the
// regions have been reused since): every segment is read from the tensor and filtered again.
template <uint32_t GS>
__device__ __forceinline__ void gather_segments(const Workspace &ws, uint32_t l, const LayerDesc &d, uint32_t s0,
                                                bool refilter_all) {
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    uint32_t my_cnt = 0, my_off = 0;
    if (lane < GS && s0 + lane < d.nseg) {
        my_cnt = refilter_all ? 0xffffffffu : ws.seg_cnt[d.seg_base + s0 + lane];
        my_off = ws.seg_off[d.seg_base + s0 + lane];
    }
    const uint2 *__restrict__ cand = ws.cand + d.cand_base + (uint64_t)s0 * d.cap;
    uint32_t *__restrict__ pidx = ws.pack_idx + d.pack_base;
    uint32_t *__restrict__ pval = ws.pack_val + d.pack_base;
    uint32_t cnt[GS], off[GS];
    uint2 rc[GS];
    uint32_t overflowed = 0;  // segments whose region could not hold their candidates (bit i)
#pragma unroll
    for (uint32_t i = 0; i < GS; ++i) {  // first 64 candidates of every segment, loads together
        cnt[i] = __shfl(my_cnt, i);
        if (cnt[i] > d.cap) {
            overflowed |= 1u << i;
            cnt[i] = 0;
        }
        off[i] = __shfl(my_off, i);
        if (lane < cnt[i]) rc[i] = cand[(uint64_t)i * d.cap + lane];
    }
#pragma unroll
    for (uint32_t i = 0; i < GS; ++i) {
        if (lane < cnt[i]) {
            pidx[off[i] + lane] = rc[i].x;
            pval[off[i] + lane] = rc[i].y;
        }
        for (uint32_t e = WAVE + lane; e < cnt[i]; e += 2 * WAVE) {  // fuller segments: two loads in flight
            uint2 c0, c1;
            const bool second = e + WAVE < cnt[i];
            c0 = cand[(uint64_t)i * d.cap + e];
            if (second) c1 = cand[(uint64_t)i * d.cap + e + WAVE];
            pidx[off[i] + e] = c0.x;
            pval[off[i] + e] = c0.y;
            if (second) {
                pidx[off[i] + e + WAVE] = c1.x;
                pval[off[i] + e + WAVE] = c1.y;
            }
        }
    }
    // A region that overflowed (large entries clustered in one stretch of the tensor) holds only
    // the first `cap` candidates of its segment: the segment is read and filtered again,
    // straight into the packed arrays.  Only these segments pay for it.
    if (overflowed) {
        const uint32_t t_lo = ws.state[l].t_lo;
        const Source src{reinterpret_cast<const uint32_t *>(d.g), nullptr, d.n, WSEG, d.vec != 0};
        for (uint32_t i = 0; i < GS; ++i) {
            if (!((overflowed >> i) & 1u)) continue;
            uint32_t lo, hi;
            segment_range(d, s0 + i, lo, hi);
            uint32_t pos = __shfl(my_off, i);
            visit_range<false, false, 4>(src, lo, hi, [&](const uint32_t(&idx)[4], const uint32_t(&bits)[4], uint32_t nvalid) {
                bool f[4];
                uint64_t m[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    f[c] = (uint32_t)c < nvalid && mag_key(bits[c]) >= t_lo;
                    m[c] = __ballot(f[c]);
                }
                uint32_t p = pos + lanes_below(m[0]) + lanes_below(m[1]) + lanes_below(m[2]) + lanes_below(m[3]);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (f[c]) {
                        pidx[p] = idx[c];
                        pval[p] = bits[c];
                        ++p;
                    }
                }
                pos += popc64(m[0]) + popc64(m[1]) + popc64(m[2]) + popc64(m[3]);
            });
        }
    }
}

// The tensors of one group that k_finish does not take (too many segments for one workgroup).
template <uint32_t GS>
__global__ __launch_bounds__(BLOCK) void k_gather(Workspace ws, uint32_t L, uint32_t blk0) {
    const uint32_t blk = blk0 + blockIdx.x;
    const uint32_t l = find_layer<&LayerDesc::gblk_base>(ws.desc, L, blk);
    const LayerDesc d = ws.desc[l];
    if (d.mode != MODE_FILTER || d.fused || ws.state[l].use_dense) return;
    const uint32_t wave = threadIdx.x / WAVE;
    const uint32_t s0 = ((blk - d.gblk_base) * WAVES + wave) * GS;
    if (s0 >= d.nseg) return;
    gather_segments<GS>(ws, l, d, s0, ws.state[l].refilter != 0);
}

// The tensors that k_finish handed back, after all groups: their regions have been reused by
// later groups, so every segment is read and filtered again (fixed grid; nothing to do when the
// list is empty, which is the rule).
template <uint32_t GS>
__global__ __launch_bounds__(BLOCK) void k_regather(Workspace ws) {
    const uint32_t n_redo = ws.redo[0];
    const uint32_t wave = threadIdx.x / WAVE;
    constexpr uint32_t NB = (FUSE_MAX_SEG + WAVES * GS - 1) / (WAVES * GS);  // workgroups' worth of segments of the largest such tensor
    for (uint64_t g = blockIdx.x; g < (uint64_t)n_redo * NB; g += gridDim.x) {
        const uint32_t l = ws.redo[1 + g / NB];
        const LayerDesc d = ws.desc[l];
        const uint32_t s0 = ((uint32_t)(g % NB) * WAVES + wave) * GS;
        if (s0 < d.nseg && !ws.state[l].use_dense) gather_segments<GS>(ws, l, d, s0, true);
    }
}

// ---- small tensors: the whole selection of one tensor in one workgroup -------------
// s_res[0] = the largest bin b with #{entries in bins >= b} >= want, s_res[1] = #{entries in
// bins > b}.  The histogram holds at least `want` entries.  SBLOCK threads, nbins <= BINS.
__device__ __forceinline__ void small_find_bin(const uint32_t *s_hist, uint32_t nbins, uint32_t want,
                                               uint32_t *s_wave, uint32_t *s_res) {
    const uint32_t per = nbins >= SBLOCK ? nbins / SBLOCK : 1u;  // bins per thread, taken from the top
    const uint32_t first = threadIdx.x * per;
    uint32_t sum = 0;
    if (first < nbins)
        for (uint32_t j = 0; j < per; ++j) sum += s_hist[nbins - 1 - (first + j)];
    uint32_t all;
    uint32_t run = block_exclusive_scan<SWAVES>(sum, s_wave, all);  // entries above this thread's bins
    if (first < nbins && run < want && run + sum >= want) {       // exactly one thread
        for (uint32_t j = 0; j < per; ++j) {
            const uint32_t b = nbins - 1 - (first + j);
            const uint32_t c = s_hist[b];
            if (run + c >= want) {
                s_res[0] = b;
                s_res[1] = run;
                break;
            }
            run += c;
        }
    }
    __syncthreads();
}

constexpr uint32_t SCAND = 448;  // candidate slots per wave of k_small (16 waves: 56 KB of LDS)
constexpr uint32_t TINY_MAX = 512;            // largest tensor k_small ranks by all-pairs comparison (at most SBLOCK, and BINS / 2)
constexpr uint32_t SMALL_SAMPLE_MIN = 32768;  // smallest tensor k_small samples before reading it whole

// Digit of `key` at a level of the descent, if the bits above the digit equal `prefix`.
__device__ __forceinline__ bool small_digit(uint32_t key, uint32_t prefix, uint32_t pshift, uint32_t shift,
                                            uint32_t nbins, uint32_t &digit) {
    digit = (key >> shift) & (nbins - 1);
    return (key >> pshift) == prefix;
}

// The quads q0 + u * stride (u < U) of a tensor; quads at or beyond q_end read as zeros.  A
// single workgroup has few waves to hide memory latency with, so the aligned full quads are
// fetched by U unconditional loads that are all in flight together (addresses past the range
// are clamped and the result dropped); only a ragged last quad or an unaligned tensor takes
// the conditional element-wise path.
template <uint32_t U>
__device__ __forceinline__ void small_load(const SmallDesc &d, bool vec, uint32_t q0, uint32_t stride,
                                           uint32_t q_end, uint4 (&v)[U]) {
    const uint32_t nfull = vec ? d.n / 4 : 0u;  // quads that one aligned 16-byte load can fetch
    if (nfull) {
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t q = q0 + u * stride;
            v[u] = load4_full<false>(d.g, (q < nfull ? q : nfull - 1) * 4);
        }
    }
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) {
        const uint32_t q = q0 + u * stride;
        if (q >= nfull) v[u] = q < q_end ? load4(d.g, q * 4, d.n, vec) : make_uint4(0, 0, 0, 0);
    }
}

// Histogram of one level over the whole tensor.
__device__ __forceinline__ void small_hist_global(const SmallDesc &d, bool vec, uint32_t *s_hist, uint32_t prefix,
                                                  uint32_t pshift, uint32_t shift, uint32_t nbins) {
    constexpr uint32_t U = 8;
    const uint32_t nquads = (d.n + 3) / 4;
    uint32_t zeros = 0;  // digit 0 (all exact zeros at the first level) is counted in a register
    for (uint32_t q0 = threadIdx.x; q0 < nquads; q0 += U * SBLOCK) {
        uint4 v[U];
        small_load<U>(d, vec, q0, SBLOCK, nquads, v);
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t q = q0 + u * SBLOCK;
            const uint32_t bits[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (uint32_t c = 0; c < 4; ++c) {
                uint32_t digit;
                if (q < nquads && q * 4 + c < d.n && small_digit(mag_key(bits[c]), prefix, pshift, shift, nbins, digit)) {
                    if (digit == 0) ++zeros;
                    else atomicAdd(&s_hist[digit], 1u);
                }
            }
        }
    }
    if (zeros) atomicAdd(&s_hist[0], zeros);
}

// One workgroup selects one tensor: level-0 histogram over the tensor; then, in a second and
// last read, every wave compacts the entries of its contiguous share that lie in the threshold
// bin or above, in index order, into LDS; the two lower levels of the descent and the ordered
// write work on those.  If the candidates do not fit LDS, the lower levels and the write read
// the tensor again instead.  Larger tensors are sampled first (like the streaming pipeline
// does), which usually replaces the level-0 pass over the whole tensor by one over an eighth.
__global__ __launch_bounds__(SBLOCK) void k_small(const SmallEntry *S, const uint64_t *layer_off, uint32_t *out_idx,
                                                  uint32_t *out_val) {
    __shared__ __align__(8) uint32_t s_hist[BINS];  // also used as 64-bit words by the all-pairs path
    __shared__ uint32_t s_cidx[SWAVES][SCAND];
    __shared__ uint32_t s_cval[SWAVES][SCAND];
    __shared__ uint32_t s_wave[SWAVES];
    __shared__ uint32_t s_cnt[SWAVES], s_gt[SWAVES], s_eq[SWAVES];
    __shared__ uint32_t s_res[2];
    __shared__ uint32_t s_fail, s_ns;
    const SmallEntry entry = S[blockIdx.x];
    const uint64_t out_first = layer_off[entry.l];
    const SmallDesc d{entry.g, out_first, entry.n, (uint32_t)(layer_off[entry.l + 1] - out_first)};
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wv = tid / WAVE;
    const bool vec = ((uintptr_t)d.g & 15u) == 0;
    const uint32_t nquads = (d.n + 3) / 4;

    // A tensor of a few hundred elements (a bias vector, a small convolution kernel) needs none of
    // the machinery below: one element per thread, its rank in the order of the selection (larger
    // key first, lower index first among equal keys) by comparison with every other element, and
    // the selected ones written at the number of selected elements before them.
    if (d.n <= TINY_MAX) {
        uint64_t *s_order = reinterpret_cast<uint64_t *>(s_hist);  // key << 32 | ~index: greater = earlier in the order
        uint32_t bits = 0;
        uint64_t mine = 0;
        if (tid < d.n) {
            bits = reinterpret_cast<const uint32_t *>(d.g)[tid];
            mine = ((uint64_t)mag_key(bits) << 32) | (uint32_t)~tid;
            s_order[tid] = mine;
        }
        __syncthreads();
        uint32_t rank = 0;
        if (tid < d.n)
            for (uint32_t j = 0; j < d.n; ++j) rank += s_order[j] > mine ? 1u : 0u;
        const bool selected = tid < d.n && rank < d.k;
        uint32_t total;
        const uint32_t before = block_exclusive_scan<SWAVES>(selected ? 1u : 0u, s_wave, total);
        if (selected) {
            out_idx[d.out_off + before] = tid;
            out_val[d.out_off + before] = bits;
        }
        return;
    }

    // Ordered compaction of the entries whose key lies in bin `bin_lo` (of level 0) or above, wave
    // by wave over contiguous shares, into the waves' LDS slots.  False if a wave ran out of slots.
    auto collect = [&](uint32_t bin_lo) -> bool {
        if (tid == 0) s_fail = 0;
        __syncthreads();
        const uint32_t share = (nquads + SWAVES - 1) / SWAVES;
        const uint32_t q_lo = wv * share, q_hi = q_lo + share < nquads ? q_lo + share : nquads;
        uint32_t filled = 0;
        bool ok = true;
        constexpr uint32_t U = 8;
        for (uint32_t p = q_lo; p < q_hi && ok; p += U * WAVE) {
            uint4 v[U];
            small_load<U>(d, vec, p + lane, WAVE, q_hi, v);
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                const uint32_t q = p + u * WAVE + lane;
                const uint32_t bits[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
                bool take[4];
                uint32_t before = 0, total = 0;  // candidates in lower lanes; in the whole piece
#pragma unroll
                for (uint32_t c = 0; c < 4; ++c) {
                    take[c] = q < q_hi && q * 4 + c < d.n && (mag_key(bits[c]) >> 19) >= bin_lo;
                    const uint64_t m = __ballot(take[c]);
                    before += lanes_below(m);
                    total += popc64(m);
                }
                if (filled + total > SCAND) {  // wave-uniform
                    ok = false;
                    break;
                }
                uint32_t at = filled + before;
#pragma unroll
                for (uint32_t c = 0; c < 4; ++c) {
                    if (take[c]) {
                        s_cidx[wv][at] = q * 4 + c;
                        s_cval[wv][at] = bits[c];
                        ++at;
                    }
                }
                filled += total;
            }
        }
        if (lane == 0) {
            s_cnt[wv] = filled;
            if (!ok) s_fail = 1;
        }
        __syncthreads();
        return s_fail == 0;
    };
    // Histogram of one level of the descent over the candidates in LDS (s_hist zeroed by the caller).
    auto hist_candidates = [&](uint32_t pre, uint32_t pshift, uint32_t shift, uint32_t nbins) {
        uint32_t zeros = 0;
        for (uint32_t e = lane; e < s_cnt[wv]; e += WAVE) {
            uint32_t digit;
            if (small_digit(mag_key(s_cval[wv][e]), pre, pshift, shift, nbins, digit)) {
                if (digit == 0) ++zeros;
                else atomicAdd(&s_hist[digit], 1u);
            }
        }
        if (zeros) atomicAdd(&s_hist[0], zeros);
    };

    uint32_t prefix = 0, k_rem = d.k;
    bool in_lds = false, level0_done = false;

    // A tensor that is worth it is first sampled, one 1 KB piece in eight: from the sample a
    // conservative bin is chosen, one read of the tensor collects everything in that bin or above,
    // and if that is at least k entries (and fits LDS) the whole descent runs on them.
    if (d.n >= SMALL_SAMPLE_MIN && 2 * d.k <= SWAVES * SCAND) {
        for (uint32_t i = tid; i < BINS; i += SBLOCK) s_hist[i] = 0;
        if (tid == 0) s_ns = 0;
        __syncthreads();
        const uint32_t npieces = (nquads + WAVE - 1) / WAVE;
        uint32_t zeros = 0, mine = 0;
        for (uint32_t j = wv; j * 8 < npieces; j += SWAVES) {
            uint32_t p = j * 8 + ((j * 5u) & 7u);  // a different piece of every eight
            if (p >= npieces) p = npieces - 1;
            const uint32_t q = p * WAVE + lane;
            if (q >= nquads) continue;
            const uint4 v = load4(d.g, q * 4, d.n, vec);
            const uint32_t bits[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (uint32_t c = 0; c < 4; ++c) {
                if (q * 4 + c >= d.n) continue;
                ++mine;
                const uint32_t digit = mag_key(bits[c]) >> 19;
                if (digit == 0) ++zeros;
                else atomicAdd(&s_hist[digit], 1u);
            }
        }
        if (zeros) atomicAdd(&s_hist[0], zeros);
        if (mine) atomicAdd(&s_ns, mine);
        __syncthreads();
        const uint32_t ns = s_ns;
        const float kf = (float)d.k * (float)ns / (float)d.n;
        const uint32_t want = (uint32_t)ceilf(kf + 6.0f * sqrtf(kf) + 8.0f) + 1u;
        if (want <= ns) {  // uniform
            small_find_bin(s_hist, BINS, want, s_wave, s_res);
            const uint32_t bin_lo = s_res[0];
            __syncthreads();
            if (bin_lo > 0 && collect(bin_lo)) {
                uint32_t m = 0;
                for (uint32_t w = 0; w < SWAVES; ++w) m += s_cnt[w];
                if (m >= d.k) {  // the k largest are all among the candidates
                    in_lds = true;
                    for (uint32_t i = tid; i < BINS; i += SBLOCK) s_hist[i] = 0;
                    __syncthreads();
                    hist_candidates(0u, 31u, 19u, BINS);
                    __syncthreads();
                    small_find_bin(s_hist, BINS, d.k, s_wave, s_res);
                    prefix = s_res[0];
                    k_rem = d.k - s_res[1];
                    level0_done = true;
                    __syncthreads();
                }
            }
        }
    }

    if (!level0_done) {
        // level 0 from the whole tensor: bits 30..19 of the key
        __syncthreads();
        for (uint32_t i = tid; i < BINS; i += SBLOCK) s_hist[i] = 0;
        __syncthreads();
        small_hist_global(d, vec, s_hist, 0u, 31u, 19u, BINS);
        __syncthreads();
        small_find_bin(s_hist, BINS, d.k, s_wave, s_res);
        const uint32_t bin0 = s_res[0];
        prefix = bin0;
        k_rem = d.k - s_res[1];
        const uint32_t ncand = s_res[1] + s_hist[bin0];  // entries in the threshold bin or above
        __syncthreads();
        in_lds = ncand <= SWAVES * SCAND && collect(bin0);
    }

    // levels 1 and 2: bits 18..7 and 6..0, among the entries that share the prefix found so far
#pragma unroll 1
    for (int level = 1; level < 3; ++level) {
        const uint32_t shift = level == 1 ? 7u : 0u;
        const uint32_t nbins = level == 1 ? BINS : 128u;
        const uint32_t pshift = level == 1 ? 19u : 7u;
        for (uint32_t i = tid; i < nbins; i += SBLOCK) s_hist[i] = 0;
        __syncthreads();
        if (in_lds) {
            hist_candidates(prefix, pshift, shift, nbins);
        } else {
            small_hist_global(d, vec, s_hist, prefix, pshift, shift, nbins);
        }
        __syncthreads();
        small_find_bin(s_hist, nbins, k_rem, s_wave, s_res);
        prefix = (prefix << (level == 1 ? 12 : 7)) | s_res[0];
        k_rem -= s_res[1];
        __syncthreads();
    }
    const uint32_t T = prefix, r = k_rem;  // threshold key; entries equal to it to keep (lowest indices)

    if (in_lds) {
        // ordered write from the candidates: counts per wave, then every wave places its own
        uint32_t n_gt = 0, n_eq = 0;
        for (uint32_t e0 = 0; e0 < s_cnt[wv]; e0 += WAVE) {
            const uint32_t e = e0 + lane;
            const uint32_t key = e < s_cnt[wv] ? mag_key(s_cval[wv][e]) : 0u;
            n_gt += popc64(__ballot(e < s_cnt[wv] && key > T));
            n_eq += popc64(__ballot(e < s_cnt[wv] && key == T));
        }
        if (lane == 0) {
            s_gt[wv] = n_gt;
            s_eq[wv] = n_eq;
        }
        __syncthreads();
        uint32_t g = 0, q = 0;  // selected-above and equal entries before this wave's share
        for (uint32_t w = 0; w < wv; ++w) {
            g += s_gt[w];
            q += s_eq[w];
        }
        for (uint32_t e0 = 0; e0 < s_cnt[wv]; e0 += WAVE) {
            const uint32_t e = e0 + lane;
            const bool live = e < s_cnt[wv];
            const uint32_t bits = live ? s_cval[wv][e] : 0u;
            const uint32_t key = mag_key(bits);
            const bool gt = live && key > T, eq = live && key == T;
            const uint64_t m_gt = __ballot(gt), m_eq = __ballot(eq);
            const uint32_t g_before = g + lanes_below(m_gt), q_before = q + lanes_below(m_eq);
            if (gt || (eq && q_before < r)) {
                const uint64_t pos = d.out_off + g_before + (q_before < r ? q_before : r);
                out_idx[pos] = s_cidx[wv][e];
                out_val[pos] = bits;
            }
            g += popc64(m_gt);
            q += popc64(m_eq);
        }
        return;
    }

    // ordered write from the tensor: entry e goes to position #{selected entries before e}
    uint32_t gt_before = 0, eq_before = 0;
    for (uint32_t q0 = 0; q0 < nquads; q0 += SBLOCK) {
        const uint32_t q = q0 + tid;
        const uint4 v = q < nquads ? load4(d.g, q * 4, d.n, vec) : make_uint4(0, 0, 0, 0);
        const uint32_t bits[4] = {v.x, v.y, v.z, v.w};
        bool gt[4], eq[4];
        uint32_t cnt = 0;
#pragma unroll
        for (uint32_t c = 0; c < 4; ++c) {
            const uint32_t key = mag_key(bits[c]);
            const bool valid = q < nquads && q * 4 + c < d.n;
            gt[c] = valid && key > T;
            eq[c] = valid && key == T;
            cnt += (gt[c] ? 1u : 0u) + (eq[c] ? 0x10000u : 0u);
        }
        uint32_t tot;  // both counts in one scan: at most 4096 each per round
        const uint32_t o = block_exclusive_scan<SWAVES>(cnt, s_wave, tot);
        uint32_t g = gt_before + (o & 0xffffu), e = eq_before + (o >> 16);
#pragma unroll
        for (uint32_t c = 0; c < 4; ++c) {
            if (gt[c]) {
                const uint64_t pos = d.out_off + g + (e < r ? e : r);
                out_idx[pos] = q * 4 + c;
                out_val[pos] = bits[c];
                ++g;
            } else if (eq[c]) {
                if (e < r) {
                    const uint64_t pos = d.out_off + g + e;
                    out_idx[pos] = q * 4 + c;
                    out_val[pos] = bits[c];
                }
                ++e;
            }
        }
        gt_before += tot & 0xffffu;
        eq_before += tot >> 16;
        if (gt_before + (eq_before < r ? eq_before : r) == d.k) break;  // uniform: all k written
    }
}

// ---- steps 4-7 for one tensor in one workgroup ---------------------------------------
// A tensor of up to a couple of thousand segments has tens of thousands of candidates: half a
// megabyte that the filter of its group has just written and that is still in cache.  One
// workgroup per tensor, launched right after that filter, takes it from there to its output with
// no further launches:
//   pack     the regions' candidates are copied to the packed arrays in index order: every wave fills
//            an even share of the packed positions (whole rows of 64), gathering each row from the
//            regions it falls into (a segment whose region overflowed is read from the tensor and
//            filtered again), and bins (key - t_lo) >> 11 into 4096 bins (keys a factor two or more
//            above t_lo share the last bin) -> the bin of the k-th largest key;
//   level 2  histogram of the low 11 bits inside that bin over the packed candidates -> the exact
//            threshold key T and the tie quota r;
//   count    every wave counts key > T and key == T in its even share of the packed candidates;
//   emit     ordered write: a wave's first output position follows from the counts of the waves
//            before it; the selected pairs pass through an LDS buffer and leave in whole runs.
// The last three are dense reads of data the workgroup has just written.  The workgroup does
// the check of the multi-launch path instead and leaves the tensor to those kernels when the
// candidates are too few (the sample misjudged: filtered again after all groups) or too many,
// and after packing when the threshold lies a factor two above t_lo (the packed arrays are then
// ready for the descent).  A tensor that the plan does not give to this kernel (more than
// FUSE_MAX_SEG segments or FUSE_MAX_CAND expected candidates) only gets the check here.
constexpr uint32_t ESTAGE = 384;  // selected pairs a wave of k_finish collects before it writes them out

__global__ __launch_bounds__(SBLOCK) void k_finish(Workspace ws, uint32_t l0, uint32_t *out_idx, uint32_t *out_val) {
    static_assert(SBLOCK == CBLOCK, "the check and the finish share a workgroup");
    static_assert(ESTAGE > PIECE && ESTAGE * 2 * SWAVES >= BINS, "emit buffer: more than a piece; it shares LDS with the histogram");
    __shared__ uint32_t s_buf[2 * ESTAGE * SWAVES];  // first the histogram, then the waves' emit buffers (index, value)
    __shared__ uint32_t s_pre[FUSE_MAX_SEG + 1];  // packed position of each segment's first candidate; [nseg] = all
    __shared__ uint32_t s_wave[SWAVES];
    __shared__ uint32_t s_gt[SWAVES], s_eq[SWAVES];
    __shared__ uint32_t s_res[2];
    uint32_t *s_hist = s_buf;
    const uint32_t l = l0 + blockIdx.x;
    const LayerDesc d = ws.desc[l];
    if (d.mode != MODE_FILTER) return;
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wv = tid / WAVE;
    const uint32_t per = (d.nseg + SWAVES - 1) / SWAVES;  // segments per wave (for the segments that overflowed)
    const uint32_t s_lo = wv * per < d.nseg ? wv * per : d.nseg;
    const uint32_t s_hi = s_lo + per < d.nseg ? s_lo + per : d.nseg;
    bool take = d.fused != 0;
    uint32_t m = 0;
    if (take) {
        // packed position of every segment's first candidate = prefix sums of the counts, in LDS
        const uint32_t *cnt = ws.seg_cnt + d.seg_base;
        for (uint32_t i = tid; i < BINS; i += SBLOCK) s_hist[i] = 0;
        m = scan_store([&](uint32_t i) { return cnt[i]; }, [&](uint32_t i, uint32_t v) { s_pre[i] = v; }, d.nseg, s_wave);
        if (tid == 0) s_pre[d.nseg] = m;
        __syncthreads();
        const uint64_t room = std::min<uint64_t>((uint64_t)d.nseg * d.cap, d.n / 4);
        take = m >= d.k && m <= 2 * FUSE_MAX_CAND && m <= room;
    }
    if (!take) {
        // the multi-launch path; a tensor that was meant to be finished here has no gather in its
        // group: it is entered into the list of tensors to be filtered again after all groups
        const bool usable = check_tensor(ws, l, d, s_wave);
        if (tid == 0 && d.fused && usable) {
            ws.state[l].refilter = 1;
            ws.redo[1 + atomicAdd(&ws.redo[0], 1u)] = l;
        }
        return;
    }
    const uint32_t t_lo = ws.state[l].t_lo;
    uint32_t *__restrict__ pidx = ws.pack_idx + d.pack_base;
    uint32_t *__restrict__ pval = ws.pack_val + d.pack_base;
    // the wave's even share of the packed candidates, in whole pieces
    const uint32_t share = ((m + SWAVES - 1) / SWAVES + PIECE - 1) / PIECE * PIECE;
    const uint32_t wv_u = __builtin_amdgcn_readfirstlane(wv);  // tells the compiler that the share is wave-uniform
    const uint32_t c_lo = wv_u * share < m ? wv_u * share : m;
    const uint32_t c_hi = m - c_lo < share ? m : c_lo + share;
    {   // pack + first histogram
        const uint2 *__restrict__ regions = ws.cand + d.cand_base;
        const uint32_t cap = d.cap;
        auto bin_of = [&](uint32_t bits) {
            const uint32_t b = (mag_key(bits) - t_lo) >> FUSE_SHIFT;
            return b < BINS - 1 ? b : BINS - 1;
        };
        // Packed position c belongs to the segment seg with s_pre[seg] <= c < s_pre[seg + 1] and is entry
        // c - s_pre[seg] of its region.  A lane visits the positions c_lo + lane, + 64, ...: it looks its
        // first segment up by bisection and walks on from there.  Each row of 64 positions is one gather
        // from two or three regions and two full-width stores; FUSE_ROWS rows are requested, then stored.
        // Positions of a segment whose region overflowed are left out here.
        const uint32_t rows = (c_hi - c_lo + WAVE - 1) / WAVE;  // wave-uniform
        uint32_t seg = 0;
        {
            const uint32_t c0 = c_lo + lane < m ? c_lo + lane : m - 1;  // m >= k >= 1
            uint32_t hi = d.nseg;
            while (hi - seg > 1) {
                const uint32_t mid = (seg + hi) / 2;
                if (s_pre[mid] <= c0) seg = mid;
                else hi = mid;
            }
        }
        uint32_t base = s_pre[seg], lim = s_pre[seg + 1];
        uint2 a[FUSE_ROWS];
        uint32_t have = 0;  // bit j: a[j] holds a candidate
        // Every lane loads in every slot, from entry 0 of the first region where it has nothing to fetch:
        // only when the number of loads issued after a given one is known at compile time can the wait
        // for that one leave the later ones in flight.
        auto request = [&](uint32_t j, uint32_t row) {
            const uint32_t c = c_lo + row * WAVE + lane;
            uint64_t at = 0;
            bool real = false;
            if (c < c_hi) {
                while (c >= lim) {  // ends: c < m = s_pre[nseg]
                    ++seg;
                    base = lim;
                    lim = s_pre[seg + 1];
                }
                if (lim - base <= cap) {
                    at = (uint64_t)seg * cap + (c - base);
                    real = true;
                }
            }
            a[j] = regions[at];
            have = real ? have | (1u << j) : have & ~(1u << j);
        };
        auto retire = [&](uint32_t j, uint32_t row) {
            if ((have >> j) & 1u) {
                const uint32_t c = c_lo + row * WAVE + lane;
                pidx[c] = a[j].x;
                pval[c] = a[j].y;
                atomicAdd(&s_hist[bin_of(a[j].y)], 1u);
            }
        };
        for (uint32_t row0 = 0; row0 < rows; row0 += FUSE_ROWS) {
#pragma unroll
            for (uint32_t j = 0; j < FUSE_ROWS; ++j) request(j, row0 + j);
#pragma unroll
            for (uint32_t j = 0; j < FUSE_ROWS; ++j) retire(j, row0 + j);
        }
        // a region that overflowed holds only its first `cap` candidates: the wave filters such a segment
        // of its range of segments again, from the tensor, to the segment's packed positions
        const Source dense{reinterpret_cast<const uint32_t *>(d.g), nullptr, d.n, WSEG, d.vec != 0};
        for (uint32_t s0 = s_lo; s0 < s_hi; s0 += WAVE) {
            const uint32_t sg = s0 + lane;
            uint64_t over = __ballot(sg < s_hi && s_pre[sg + 1] - s_pre[sg] > cap);
            while (over) {  // uniform
                const uint32_t os = s0 + (uint32_t)__builtin_ctzll(over);
                over &= over - 1;
                uint32_t lo, hi;
                segment_range(d, os, lo, hi);
                uint32_t q0 = s_pre[os];
                visit_range<false, false, 4>(dense, lo, hi, [&](const uint32_t(&idx)[4], const uint32_t(&bits)[4], uint32_t nvalid) {
                    bool f[4];
                    uint64_t mk[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        f[c] = (uint32_t)c < nvalid && mag_key(bits[c]) >= t_lo;
                        mk[c] = __ballot(f[c]);
                    }
                    uint32_t p = q0 + lanes_below(mk[0]) + lanes_below(mk[1]) + lanes_below(mk[2]) + lanes_below(mk[3]);
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (f[c]) {
                            pidx[p] = idx[c];
                            pval[p] = bits[c];
                            atomicAdd(&s_hist[bin_of(bits[c])], 1u);
                            ++p;
                        }
                    }
                    q0 += popc64(mk[0]) + popc64(mk[1]) + popc64(mk[2]) + popc64(mk[3]);
                });
            }
        }
    }
    __syncthreads();  // the packed arrays are complete and visible to the whole workgroup
    small_find_bin(s_hist, BINS, d.k, s_wave, s_res);
    const uint32_t b0 = s_res[0];
    const uint32_t k_rem = d.k - s_res[1];
    __syncthreads();
    if (b0 == BINS - 1) {  // keys of different upper bits share the last bin: the general descent resolves it
        if (tid == 0) {
            ws.state[l].m = m;
            ws.state[l].nchunk = (m + VCHUNK - 1) / VCHUNK;
        }
        return;
    }
    const Source packed{pval, pidx, m, VCHUNK, true};
    for (uint32_t i = tid; i < (1u << FUSE_SHIFT); i += SBLOCK) s_hist[i] = 0;
    __syncthreads();
    visit_range<false, false, 4>(packed, c_lo, c_hi, [&](const uint32_t(&)[4], const uint32_t(&bits)[4], uint32_t nvalid) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t rel = mag_key(bits[c]) - t_lo;
            if ((uint32_t)c < nvalid && (rel >> FUSE_SHIFT) == b0) atomicAdd(&s_hist[rel & ((1u << FUSE_SHIFT) - 1u)], 1u);
        }
    });
    __syncthreads();
    small_find_bin(s_hist, 1u << FUSE_SHIFT, k_rem, s_wave, s_res);
    const uint32_t T = t_lo + (b0 << FUSE_SHIFT) + s_res[0];  // threshold key
    const uint32_t r = k_rem - s_res[1];                      // entries equal to it to keep (lowest indices)
    uint32_t n_gt = 0, n_eq = 0;
    visit_range<false, false, 4>(packed, c_lo, c_hi, [&](const uint32_t(&)[4], const uint32_t(&bits)[4], uint32_t nvalid) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t key = mag_key(bits[c]);
            const bool ok = (uint32_t)c < nvalid;
            n_gt += popc64(__ballot(ok && key > T));
            n_eq += popc64(__ballot(ok && key == T));
        }
    });
    if (lane == 0) {
        s_gt[wv] = n_gt;
        s_eq[wv] = n_eq;
    }
    __syncthreads();  // also: the histogram is no longer needed, its memory becomes the emit buffers
    uint32_t run_gt = 0, run_eq = 0;  // entries with key > T / key == T before the current ones (in the tensor)
    for (uint32_t w = 0; w < wv; ++w) {
        run_gt += s_gt[w];
        run_eq += s_eq[w];
    }
    // Selected pairs go to this wave's LDS buffer in order and leave as runs of consecutive
    // output entries: a few full-width stores instead of eight narrow strided ones per piece.
    const uint32_t first_out = run_gt + (run_eq < r ? run_eq : r);  // output position of the wave's first selected entry
    uint32_t *e_idx = s_buf + wv * 2 * ESTAGE, *e_val = e_idx + ESTAGE;
    uint32_t *oi = out_idx + d.out_off + first_out;
    uint32_t *ov = out_val + d.out_off + first_out;
    uint32_t staged = 0, written = 0;  // wave-uniform
    auto drain = [&]() {
        wave_lds_fence();
        for (uint32_t e = lane; e < staged; e += WAVE) {
            oi[written + e] = e_idx[e];
            ov[written + e] = e_val[e];
        }
        wave_lds_fence();
        written += staged;
        staged = 0;
    };
    visit_range<true, false, 4>(packed, c_lo, c_hi, [&](const uint32_t(&idx)[4], const uint32_t(&bits)[4], uint32_t nvalid) {
        bool g[4], e[4];
        uint64_t any = 0;
        uint32_t gt_b = run_gt, eq_b = run_eq, tot_g = 0, tot_e = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t key = mag_key(bits[c]);
            const bool ok = (uint32_t)c < nvalid;
            g[c] = ok && key > T;
            e[c] = ok && key == T;
            const uint64_t mg = __ballot(g[c]), me = __ballot(e[c]);
            any |= mg | me;
            gt_b += lanes_below(mg);
            eq_b += lanes_below(me);
            tot_g += popc64(mg);
            tot_e += popc64(me);
        }
        if (any == 0) return;
        if (staged + PIECE > ESTAGE) drain();  // uniform: a piece adds at most PIECE entries
        const uint32_t origin = first_out + written;  // output position of buffer slot 0
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            // an entry at the threshold is kept iff fewer than r equal keys precede it in the tensor
            if (g[c]) {
                const uint32_t slot = gt_b + (eq_b < r ? eq_b : r) - origin;
                e_idx[slot] = idx[c];
                e_val[slot] = bits[c];
                ++gt_b;
            } else if (e[c]) {
                if (eq_b < r) {
                    const uint32_t slot = gt_b + eq_b - origin;
                    e_idx[slot] = idx[c];
                    e_val[slot] = bits[c];
                }
                ++eq_b;
            }
        }
        run_gt += tot_g;
        run_eq += tot_e;
        staged = run_gt + (run_eq < r ? run_eq : r) - origin;
    });
    drain();
    if (tid == 0) {
        ws.state[l].T = T;
        ws.state[l].r = r;
        ws.state[l].done = 1;
        ws.state[l].m = 0;
        ws.state[l].nchunk = 0;  // nothing for the descent, count and emit kernels
    }
}

// ---- chunk numbering across tensors ------------------------------------------------
// The descent, count and emit kernels run with a fixed number of workgroups; each worker
// (workgroup or wave) takes a contiguous range of the global chunk numbering.
__global__ __launch_bounds__(CBLOCK) void k_work(Workspace ws, uint32_t L) {
    __shared__ uint32_t s_wave[CBLOCK / WAVE];
    const uint32_t total = scan_array([&](uint32_t l) { return ws.state[l].nchunk; }, ws.chunk_base, L, s_wave);
    if (threadIdx.x == 0) ws.chunk_base[L] = total;
}

// Range of global chunk numbers of worker `w` out of `nworkers`, and the tensor of its first chunk.
__device__ __forceinline__ bool chunk_range(const Workspace &ws, uint32_t L, uint32_t w, uint32_t nworkers,
                                            uint32_t &lo, uint32_t &hi, uint32_t &l) {
    const uint32_t total = ws.chunk_base[L];
    const uint32_t per = (total + nworkers - 1) / nworkers;
    lo = w * per;
    if (per == 0 || lo >= total) return false;
    hi = total - lo < per ? total : lo + per;
    uint32_t a = 0, b = L;  // the last tensor with chunk_base <= lo
    while (b - a > 1) {
        const uint32_t mid = (a + b) >> 1;
        if (ws.chunk_base[mid] <= lo) a = mid; else b = mid;
    }
    l = a;
    return true;
}

// ---- step 6: radix descent, one histogram + one resolve per level ----------------
// level 0: bins = key[30:19]; level 1: key[30:19] == prefix, bins = key[18:7];
// level 2: key[30:7] == prefix, bins = key[6:0].
template <int LEVEL>
__global__ __launch_bounds__(BLOCK) void k_hist(Workspace ws, uint32_t L) {
    __shared__ uint32_t h[BINS];
    uint32_t w_lo, w_hi, l;
    if (!chunk_range(ws, L, blockIdx.x, gridDim.x, w_lo, w_hi, l)) return;
    const uint32_t wave = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
    while (w_lo < w_hi) {  // one tensor at a time: the LDS histogram belongs to one tensor
        while (w_lo >= ws.chunk_base[l + 1]) ++l;
        const uint32_t base = ws.chunk_base[l];
        const uint32_t end = ws.chunk_base[l + 1] < w_hi ? ws.chunk_base[l + 1] : w_hi;
        const LayerDesc d = ws.desc[l];
        const LayerState st = ws.state[l];
        const Source src = source_of(d, st, ws);
        const uint32_t prefix = st.prefix;
        lds_hist_clear(h);
        uint32_t zero_run = 0;
        for (uint32_t w = w_lo + wave; w < end; w += WAVES) {
            const uint32_t lo = (w - base) * src.chunk;
            const uint32_t hi = src.m - lo < src.chunk ? src.m : lo + src.chunk;
            visit_range<false>(src, lo, hi, [&](const uint32_t(&idx)[4], const uint32_t(&bits)[4], uint32_t nvalid) {
                uint32_t key[4], bin[4];
                bool match[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    key[c] = mag_key(bits[c]);
                    match[c] = (uint32_t)c < nvalid;
                    if (LEVEL == 0) {
                        bin[c] = key[c] >> 19;
                    } else if (LEVEL == 1) {
                        match[c] = match[c] && (key[c] >> 19) == prefix;
                        bin[c] = (key[c] >> 7) & 0xfffu;
                    } else {
                        match[c] = match[c] && (key[c] >> 7) == prefix;
                        bin[c] = key[c] & 0x7fu;
                    }
                }
                (void)idx;
                lds_hist_add<4>(h, key, match, bin, zero_run);
            });
        }
        if (lane == 0 && zero_run) atomicAdd(&h[0], zero_run);
        lds_hist_flush(h, ws.hist + (size_t)l * BINS, LEVEL == 2 ? 128u : BINS);
        __syncthreads();
        w_lo = end;
    }
}

template <int LEVEL>
__global__ __launch_bounds__(BLOCK) void k_resolve(Workspace ws) {
    const uint32_t l = blockIdx.x;
    const LayerDesc d = ws.desc[l];
    if (d.nseg == 0) return;
    uint32_t *h = ws.hist + (size_t)l * BINS;
    const LayerState st = ws.state[l];
    if (st.done) return;
    constexpr uint32_t nbins = LEVEL == 2 ? 128u : BINS;
    uint32_t bin, above;
    find_bin_from_top(h, nbins, st.k_rem, bin, above);
    for (uint32_t i = threadIdx.x; i < nbins; i += BLOCK) h[i] = 0;
    if (threadIdx.x == 0) {
        const uint32_t prefix = (st.prefix << (LEVEL == 2 ? 7 : 12)) | bin;
        const uint32_t k_rem = st.k_rem - above;
        ws.state[l].prefix = prefix;
        ws.state[l].k_rem = k_rem;
        if (LEVEL == 2) {
            ws.state[l].T = prefix;
            ws.state[l].r = k_rem;
        }
    }
}

// ---- step 7: per-chunk counts, scans, ordered emit ------------------------------
__global__ __launch_bounds__(BLOCK) void k_count(Workspace ws, uint32_t L) {
    const uint32_t wave = threadIdx.x / WAVE, lane = threadIdx.x & (WAVE - 1);
    uint32_t w_lo, w_hi, l;
    if (!chunk_range(ws, L, blockIdx.x * WAVES + wave, gridDim.x * WAVES, w_lo, w_hi, l)) return;
    uint32_t cur = 0xffffffffu;
    LayerDesc d;
    LayerState st;
    Source src;
    for (uint32_t w = w_lo; w < w_hi; ++w) {
        while (w >= ws.chunk_base[l + 1]) ++l;
        if (l != cur) {
            cur = l;
            d = ws.desc[l];
            st = ws.state[l];
            src = source_of(d, st, ws);
        }
        const uint32_t j = w - ws.chunk_base[l];
        const uint32_t lo = j * src.chunk;
        const uint32_t hi = src.m - lo < src.chunk ? src.m : lo + src.chunk;
        const uint32_t T = st.T;
        uint32_t gt = 0, eq = 0;
        visit_range<false>(src, lo, hi, [&](const uint32_t(&idx)[4], const uint32_t(&bits)[4], uint32_t nvalid) {
            (void)idx;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t key = mag_key(bits[c]);
                const bool ok = (uint32_t)c < nvalid;
                gt += popc64(__ballot(ok && key > T));
                eq += popc64(__ballot(ok && key == T));
            }
        });
        if (lane == 0) {
            ws.seg_gt[d.seg_base + j] = gt;
            ws.seg_eq[d.seg_base + j] = eq;
        }
    }
}

// Exclusive scan over the chunks of one tensor of both count arrays, in place.
__global__ __launch_bounds__(CBLOCK) void k_scan(Workspace ws) {
    __shared__ uint32_t s_wave[CBLOCK / WAVE];
    const uint32_t l = blockIdx.x;
    const LayerDesc d = ws.desc[l];
    if (d.nseg == 0) return;
    const uint32_t nchunk = ws.state[l].nchunk;
    uint32_t *gt = ws.seg_gt + d.seg_base, *eq = ws.seg_eq + d.seg_base;
    scan_array([&](uint32_t i) { return gt[i]; }, gt, nchunk, s_wave);
    scan_array([&](uint32_t i) { return eq[i]; }, eq, nchunk, s_wave);
}

__global__ __launch_bounds__(BLOCK) void k_emit(Workspace ws, uint32_t L, uint32_t *out_idx, uint32_t *out_val) {
    const uint32_t wave = threadIdx.x / WAVE;
    uint32_t w_lo, w_hi, l;
    if (!chunk_range(ws, L, blockIdx.x * WAVES + wave, gridDim.x * WAVES, w_lo, w_hi, l)) return;
    uint32_t cur = 0xffffffffu;
    LayerDesc d;
    LayerState st;
    Source src;
    for (uint32_t w = w_lo; w < w_hi; ++w) {
        while (w >= ws.chunk_base[l + 1]) ++l;
        if (l != cur) {
            cur = l;
            d = ws.desc[l];
            st = ws.state[l];
            src = source_of(d, st, ws);
        }
        const uint32_t j = w - ws.chunk_base[l];
        const uint32_t lo = j * src.chunk;
        const uint32_t hi = src.m - lo < src.chunk ? src.m : lo + src.chunk;
        const uint32_t T = st.T, r = st.r;
        uint32_t run_gt = ws.seg_gt[d.seg_base + j];  // entries with key > T before this chunk
        uint32_t run_eq = ws.seg_eq[d.seg_base + j];  // entries with key == T before this chunk
        uint32_t *oi = out_idx + d.out_off;
        uint32_t *ov = out_val + d.out_off;
        visit_range<true>(src, lo, hi, [&](const uint32_t(&idx)[4], const uint32_t(&bits)[4], uint32_t nvalid) {
            bool g[4], e[4];
            uint64_t mg[4], me[4];
            uint64_t any = 0;
            uint32_t gt_b = run_gt, eq_b = run_eq, tot_g = 0, tot_e = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t key = mag_key(bits[c]);
                const bool ok = (uint32_t)c < nvalid;
                g[c] = ok && key > T;
                e[c] = ok && key == T;
                mg[c] = __ballot(g[c]);
                me[c] = __ballot(e[c]);
                any |= mg[c] | me[c];
                gt_b += lanes_below(mg[c]);
                eq_b += lanes_below(me[c]);
                tot_g += popc64(mg[c]);
                tot_e += popc64(me[c]);
            }
            if (any == 0) return;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (g[c]) {
                    const uint32_t pos = gt_b + (eq_b < r ? eq_b : r);
                    oi[pos] = idx[c];
                    ov[pos] = bits[c];
                    ++gt_b;
                } else if (e[c]) {
                    if (eq_b < r) {
                        const uint32_t pos = gt_b + eq_b;
                        oi[pos] = idx[c];
                        ov[pos] = bits[c];
                    }
                    ++eq_b;
                }
            }
            run_gt += tot_g;
            run_eq += tot_e;
        });
    }
}

// ---- k == n: the update is the tensor itself --------------------------------------
__global__ __launch_bounds__(BLOCK) void k_identity(Workspace ws, uint32_t L, uint32_t *out_idx, uint32_t *out_val) {
    const uint32_t l = find_layer<&LayerDesc::iblk_base>(ws.desc, L, blockIdx.x);
    const LayerDesc d = ws.desc[l];
    const uint32_t lo = (blockIdx.x - d.iblk_base) * IDENT_TILE;
    const uint32_t hi = d.n - lo < IDENT_TILE ? d.n : lo + IDENT_TILE;
    const uint32_t *g = reinterpret_cast<const uint32_t *>(d.g);
    for (uint64_t i = (uint64_t)lo + threadIdx.x; i < hi; i += BLOCK) {  // 64-bit: hi may be 2^32 - 1
        out_idx[d.out_off + i] = (uint32_t)i;
        out_val[d.out_off + i] = g[i];
    }
}

__global__ void k_put(uint64_t *dst, PutPayload a, uint32_t nwords) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nwords) dst[i] = a.w[i];
}

__global__ void k_fill(uint32_t *dst, uint32_t value, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += step) dst[i] = value;
}

}  // namespace

hipError_t put_async(void *dst_dev, const void *src_host, size_t bytes, hipStream_t s) {
    const size_t words = (bytes + 7) / 8;
    const char *src = static_cast<const char *>(src_host);
    for (size_t w0 = 0; w0 < words; w0 += PUT_WORDS) {
        PutPayload a;
        const size_t nw = std::min<size_t>(PUT_WORDS, words - w0);
        const size_t nb = std::min<size_t>(nw * 8, bytes - w0 * 8);
        a.w[nw - 1] = 0;
        std::memcpy(a.w, src + w0 * 8, nb);
        ADACOMP_LAUNCH(ADACOMP_KERNEL_PUT, k_put, dim3((unsigned)((nw + 255) / 256)), dim3(256), s,
                       static_cast<uint64_t *>(dst_dev) + w0, a, (uint32_t)nw);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t fill_u32_async(uint32_t *dst_dev, uint32_t value, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<size_t>((n + 1023) / 1024, 4096);
    ADACOMP_LAUNCH(ADACOMP_KERNEL_FILL, k_fill, dim3(blocks), dim3(256), s, dst_dev, value, n);
    return hipGetLastError();
}

}  // namespace adacomp

using namespace adacomp;

extern "C" uint64_t adacomp_count(uint64_t n, double rate) {
    if (n == 0 || !(rate > 0.0) || rate > 1.0) return 0;
    if (rate == 1.0) return n;
    const double scaled = rate * (double)n;
    const double guarded = scaled * (1.0 - 0x1p-40);
    double k = std::ceil(guarded);
    if (k < 1.0) k = 1.0;
    if (k > (double)n) return n;
    return (uint64_t)k;
}

extern "C" int adacomp_select_workspace(const uint64_t *n, uint32_t L, double rate,
                                        const uint64_t *k_override, size_t *bytes) {
    if (!bytes || (L && !n)) return ADACOMP_ERR_NULL;
    Plan plan;
    int rc = make_plan(n, nullptr, L, rate, k_override, read_select_hooks(), plan);
    if (rc) return rc;
    Workspace ws;
    carve(plan, (uint32_t)plan.desc.size() - 1, nullptr, ws);
    *bytes = ws.bytes;
    return ADACOMP_OK;
}

#define LAUNCH(id, kernel, grid, ...)                                               \
    do {                                                                            \
        if ((grid) > 0) {                                                           \
            ADACOMP_LAUNCH(id, kernel, dim3((unsigned)(grid)), dim3(BLOCK), s, __VA_ARGS__); \
            if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP;            \
        }                                                                           \
    } while (0)

// Scratch of adacomp_select_noalloc: one copy per GPU, held until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; kernels are given the address that
// call returns for the current device.
static __device__ __align__(256) unsigned char scratch[ADACOMP_SELECT_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES];  // device address of `scratch` on device d, once looked up

// Address of `scratch` on the current device (looked up once per device).
int scratch_of_current_device(void **ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return ADACOMP_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ADACOMP_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return ADACOMP_OK;
}

// static_scratch: the workspace is the library's own array; its address is looked up only once
// the sizes are known to fit, and a call that needs more is refused with its own error code.
int select_impl(const adacomp_layer_t *layers, uint32_t L, double rate, const uint64_t *k_override,
                adacomp_update_t *out, void *workspace, size_t ws_bytes, bool static_scratch, void *hip_stream);

}  // namespace

extern "C" int adacomp_select(const adacomp_layer_t *layers, uint32_t L, double rate,
                              const uint64_t *k_override, adacomp_update_t *out,
                              void *workspace, size_t ws_bytes, void *hip_stream) {
    return select_impl(layers, L, rate, k_override, out, workspace, ws_bytes, false, hip_stream);
}

extern "C" int adacomp_select_noalloc(const adacomp_layer_t *layers, uint32_t L, double rate,
                                      const uint64_t *k_override, adacomp_update_t *out, void *hip_stream) {
    return select_impl(layers, L, rate, k_override, out, nullptr, 0, true, hip_stream);
}

namespace {

int select_impl(const adacomp_layer_t *layers, uint32_t L, double rate, const uint64_t *k_override,
                adacomp_update_t *out, void *workspace, size_t ws_bytes, bool static_scratch, void *hip_stream) {
    if (!out || (L && !layers) || !out->layer_off || !out->layer_off_dev) return ADACOMP_ERR_NULL;
    if (out->num_layers != L) return ADACOMP_ERR_LAYER_MISMATCH;
    std::vector<uint64_t> n(L);
    std::vector<const float *> data(L);
    for (uint32_t l = 0; l < L; ++l) {
        n[l] = layers[l].n;
        data[l] = layers[l].data;
        if (n[l] && !data[l]) return ADACOMP_ERR_NULL;
        if ((uintptr_t)data[l] & 3u) return ADACOMP_ERR_ALIGNMENT;
    }
    Plan plan;
    int rc = make_plan(n.data(), data.data(), L, rate, k_override, read_select_hooks(), plan);
    if (rc) return rc;
    if (plan.out_total > out->cap) return ADACOMP_ERR_CAPACITY;
    if (plan.out_total && (!out->idx || !out->val)) return ADACOMP_ERR_NULL;
    if (((uintptr_t)out->idx & 3u) || ((uintptr_t)out->val & 3u) || ((uintptr_t)out->layer_off_dev & 7u))
        return ADACOMP_ERR_ALIGNMENT;
    const uint32_t Lp = (uint32_t)plan.desc.size() - 1;  // the tensors of the pipeline (small and empty ones are not among them)
    Workspace ws;
    if (static_scratch) {
        carve(plan, Lp, nullptr, ws);
        if (ws.bytes > ADACOMP_SELECT_NOALLOC_SCRATCH_BYTES) return ADACOMP_ERR_SCRATCH_LIMIT;
        rc = scratch_of_current_device(&workspace);
        if (rc) return rc;
        ws_bytes = ADACOMP_SELECT_NOALLOC_SCRATCH_BYTES;
    }
    carve(plan, Lp, workspace, ws);
    if (!workspace || ((uintptr_t)workspace & 255u) || ws_bytes < ws.bytes) return ADACOMP_ERR_WORKSPACE;

    for (uint32_t l = 0; l <= L; ++l) out->layer_off[l] = plan.off[l];

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (put_async(out->layer_off_dev, plan.off.data(), plan.off.size() * sizeof(uint64_t), s) != hipSuccess)
        return ADACOMP_ERR_HIP;
    if (L == 0) return ADACOMP_OK;
    const LayerDesc &tot = plan.desc[Lp];
    uint32_t *out_idx = out->idx;
    uint32_t *out_val = reinterpret_cast<uint32_t *>(out->val);
    if (!plan.small.empty()) {
        if (put_async(ws.small, plan.small.data(), plan.small.size() * sizeof(SmallEntry), s) != hipSuccess)
            return ADACOMP_ERR_HIP;
        ADACOMP_LAUNCH(ADACOMP_KERNEL_SMALL, k_small, dim3((unsigned)plan.small.size()), dim3(SBLOCK), s, ws.small,
                       out->layer_off_dev, out_idx, out_val);
        if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP;
    }
    if (tot.seg_base == 0 && tot.iblk_base == 0) return ADACOMP_OK;  // nothing for the pipeline
    {
        std::vector<CompactDesc> compact(Lp);
        for (uint32_t i = 0; i < Lp; ++i) {
            const LayerDesc &d = plan.desc[i];
            uint32_t lg = 0;
            while ((1u << lg) < d.stride) ++lg;
            compact[i] = CompactDesc{d.g, d.n, plan.number[i], d.target,
                                     d.mode | (d.fused << 3) | ((uint32_t)plan.opens[i] << 4) | (lg << 5) | (d.cap << 8)};
        }
        if (put_async(ws.compact, compact.data(), compact.size() * sizeof(CompactDesc), s) != hipSuccess)
            return ADACOMP_ERR_HIP;
        ADACOMP_LAUNCH(ADACOMP_KERNEL_PUT, k_expand, dim3(1), dim3(CBLOCK), s, ws, Lp, out->layer_off_dev, plan.gsegs);
        if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP;
    }
    if (tot.seg_base) {
        if (fill_u32_async(ws.hist, 0u, (size_t)Lp * BINS, s) != hipSuccess) return ADACOMP_ERR_HIP;
        LAUNCH(ADACOMP_KERNEL_SAMPLE_HIST, k_sample_hist, tot.sblk_base, ws, Lp);
        LAUNCH(ADACOMP_KERNEL_PICK, k_pick, Lp, ws);
    }
    if (tot.sblk_base) {  // at least one tensor goes through the filter
        for (const Group &g : plan.groups) {
            if (!g.filters) continue;
            const uint32_t w0 = plan.desc[g.l0].wblk_base, g0 = plan.desc[g.l0].gblk_base;
            LAUNCH(ADACOMP_KERNEL_FILTER, k_filter, plan.desc[g.l1].wblk_base - w0, ws, g.l0, g.l1, w0);
            // per tensor: finished on the spot, or checked and left to the kernels below
            ADACOMP_LAUNCH(ADACOMP_KERNEL_FINISH, k_finish, dim3(g.l1 - g.l0), dim3(SBLOCK), s, ws, g.l0, out_idx, out_val);
            if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP;
            if (!g.unfused) continue;  // no tensor of this group needs its regions packed before they are reused
            const uint32_t g_blocks = plan.desc[g.l1].gblk_base - g0;
            if (plan.gsegs == GSEGS) LAUNCH(ADACOMP_KERNEL_GATHER, k_gather<GSEGS>, g_blocks, ws, Lp, g0);
            else if (plan.gsegs == GSEGS_MID) LAUNCH(ADACOMP_KERNEL_GATHER, k_gather<GSEGS_MID>, g_blocks, ws, Lp, g0);
            else LAUNCH(ADACOMP_KERNEL_GATHER, k_gather<GSEGS_FULL>, g_blocks, ws, Lp, g0);
        }
        if (plan.any_fused) {  // the tensors that k_finish handed back (usually none)
            const uint32_t r_blocks = (uint32_t)std::min<uint64_t>(2 * TAIL_BLOCKS, (tot.seg_base + WAVES - 1) / WAVES);
            if (plan.gsegs == GSEGS) LAUNCH(ADACOMP_KERNEL_GATHER, k_regather<GSEGS>, r_blocks, ws);
            else if (plan.gsegs == GSEGS_MID) LAUNCH(ADACOMP_KERNEL_GATHER, k_regather<GSEGS_MID>, r_blocks, ws);
            else LAUNCH(ADACOMP_KERNEL_GATHER, k_regather<GSEGS_FULL>, r_blocks, ws);
        }
    }
    if (tot.seg_base) {
        // fixed grids: the number of chunks is known on the device only (<= the segments)
        const uint32_t tail_blocks = (uint32_t)std::min<uint64_t>(TAIL_BLOCKS, (tot.seg_base + WAVES - 1) / WAVES);
        ADACOMP_LAUNCH(ADACOMP_KERNEL_WORK, k_work, dim3(1), dim3(CBLOCK), s, ws, Lp);
        if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP;
        LAUNCH(ADACOMP_KERNEL_HIST, k_hist<0>, tail_blocks, ws, Lp);
        LAUNCH(ADACOMP_KERNEL_RESOLVE, k_resolve<0>, Lp, ws);
        LAUNCH(ADACOMP_KERNEL_HIST, k_hist<1>, tail_blocks, ws, Lp);
        LAUNCH(ADACOMP_KERNEL_RESOLVE, k_resolve<1>, Lp, ws);
        LAUNCH(ADACOMP_KERNEL_HIST, k_hist<2>, tail_blocks, ws, Lp);
        LAUNCH(ADACOMP_KERNEL_RESOLVE, k_resolve<2>, Lp, ws);
        LAUNCH(ADACOMP_KERNEL_COUNT_SEG, k_count, tail_blocks, ws, Lp);
        ADACOMP_LAUNCH(ADACOMP_KERNEL_SCAN, k_scan, dim3(Lp), dim3(CBLOCK), s, ws);
        if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP;
        LAUNCH(ADACOMP_KERNEL_EMIT, k_emit, tail_blocks, ws, Lp, out_idx, out_val);
    }
    LAUNCH(ADACOMP_KERNEL_IDENTITY, k_identity, tot.iblk_base, ws, Lp, out_idx, out_val);
    return ADACOMP_OK;
}

}  // namespace

extern "C" const char *adacomp_strerror(int code) {
    switch (code) {
        case ADACOMP_OK: return "success";
        case ADACOMP_ERR_NULL: return "a required pointer is NULL";
        case ADACOMP_ERR_RATE: return "rate is NaN or outside [0, 1]";
        case ADACOMP_ERR_LAYER_TOO_LARGE: return "a tensor has 2^32 or more elements";
        case ADACOMP_ERR_CAPACITY: return "update buffers are smaller than the selected count";
        case ADACOMP_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned or too small";
        case ADACOMP_ERR_LAYER_MISMATCH: return "tensor count or sizes of update/state differ from the parameters";
        case ADACOMP_ERR_FUTURE_PULL: return "an update was pulled after the time it is applied";
        case ADACOMP_ERR_K_RANGE: return "k_override exceeds the tensor size";
        case ADACOMP_ERR_HISTORY: return "an update was pulled before the oldest remembered update";
        case ADACOMP_ERR_LR: return "learning rate is not finite";
        case ADACOMP_ERR_ALIGNMENT: return "a device pointer is not aligned to its element size";
        case ADACOMP_ERR_HIP: return "a HIP runtime call failed";
        case ADACOMP_ERR_SCRATCH_LIMIT: return "the call needs more scratch than the library's built-in buffer holds";
        default: return "unknown adacomp error code";
    }
}
