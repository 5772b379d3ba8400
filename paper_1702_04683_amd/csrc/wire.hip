// adacomp_wire_pack / adacomp_wire_unpack: a compressed update as a stream of 32-bit words.
//
// The paper leaves the byte encoding of an update open (footnote of Sec. 4 "Overview") and
// models the traffic as I x M x c (Sec. 3.2), i.e. values only.  This format is what the
// library puts on the wire so that the real figure can be stated: indices are strictly
// ascending per tensor, so a block of up to 64 consecutive entries (one wavefront) stores its
// first index in full and the 63 gaps minus one in as many bits as the largest needs.  The
// layout is defined in include/adacomp.h.
//
// One wave owns one block in every kernel: the gaps come from a lane shuffle, the width from
// a wave-wide OR, the packed bits are assembled in LDS and leave as whole words.  Where a
// block's words start depends on the widths of all earlier blocks: the first pass leaves
// every block's offset inside its group of 16 blocks and the group's total, a single-workgroup
// scan over the group totals sits between the two passes.  The unpacker trusts nothing in the stream: every read is bounded
// by the stream length the host states and every write by the counts the host expects.
#include <algorithm>
#include <vector>

#include "common.h"

namespace adacomp {
namespace {

constexpr uint32_t BLOCK = 256;
constexpr uint32_t WAVES = BLOCK / WAVE;
constexpr uint32_t SCAN_BLOCK = 1024;
constexpr uint32_t SCAN_ITEMS = 4;   // consecutive counts per thread and stretch of the single-workgroup scan
constexpr uint32_t SCAN_SUB = 4;     // stretches per round
constexpr uint32_t MAGIC = 0x31434441u;
constexpr uint32_t SUPER = 16;       // blocks per group of the two-level scan (one 1024-thread workgroup of the packer)

struct Wire {
    const uint64_t *off;      // layer_off_dev of the update [L+1]
    const uint32_t *blk_base; // [L+1] first block of every tensor
    uint32_t *nw;             // [B] delta words of the earlier blocks of the same group
    uint32_t *ng;             // [G+1] delta words per group of SUPER blocks, then their exclusive scan; ng[G] = sum
    uint32_t L, B, G;
    uint64_t total;           // entries
    uint64_t first_at, width_at, delta_at;  // word positions in the stream
};

// Block b: its tensor, first entry and number of entries.
__device__ __forceinline__ void locate(const Wire &w, uint32_t b, uint32_t &l, uint64_t &e0, uint32_t &m) {
    uint32_t lo = 0, hi = w.L;  // the last l with blk_base[l] <= b
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (w.blk_base[mid] <= b) lo = mid; else hi = mid;
    }
    l = lo;
    e0 = w.off[l] + (uint64_t)(b - w.blk_base[l]) * WAVE;
    const uint64_t left = w.off[l + 1] - e0;
    m = left < WAVE ? (uint32_t)left : (uint32_t)WAVE;
}

__device__ __forceinline__ uint32_t wave_or(uint32_t x) {
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) x |= __shfl_xor(x, d);
    return x;
}

// gap minus one to the previous entry of the block (0 for its first entry and for idle lanes)
__device__ __forceinline__ uint32_t gap_of(uint32_t mine, uint32_t lane, uint32_t m) {
    const uint32_t prev = __shfl_up(mine, 1);
    return (lane >= 1 && lane < m) ? mine - prev - 1u : 0u;
}

__device__ __forceinline__ uint32_t bit_length(uint32_t x) { return x ? 32u - (uint32_t)__clz((int)x) : 0u; }

// pass 1 of the packer: first index and width of every block; its word count as an offset inside
// its group (one workgroup = one group of SUPER blocks) and the group's total
__global__ __launch_bounds__(SUPER * WAVE) void k_wire_measure(Wire w, const uint32_t *idx, uint32_t *out, uint64_t cap) {
    __shared__ uint32_t s_n[SUPER];
    const uint32_t lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
    const uint32_t b = blockIdx.x * SUPER + wv;
    uint32_t count = 0;
    if (b < w.B) {
        uint32_t l, m;
        uint64_t e0;
        locate(w, b, l, e0, m);
        const uint32_t mine = lane < m ? idx[e0 + lane] : 0u;
        // OR of the gaps has the bit length of the largest gap
        const uint32_t width = bit_length(wave_or(gap_of(mine, lane, m)));
        count = ((m - 1) * width + 31u) >> 5;
        if (lane == 0) {
            if (w.first_at + b < cap) out[w.first_at + b] = mine;
            const uint64_t byte = w.width_at * 4 + b;
            if (byte < cap * 4) reinterpret_cast<uint8_t *>(out)[byte] = (uint8_t)width;
            if (b == w.B - 1)  // zero padding of the width bytes
                for (uint64_t p = byte + 1; p < w.delta_at * 4 && p < cap * 4; ++p) reinterpret_cast<uint8_t *>(out)[p] = 0;
        }
    }
    if (lane == 0) s_n[wv] = count;
    __syncthreads();
    if (lane == 0) {
        uint32_t before = 0, all = 0;
        for (uint32_t i = 0; i < SUPER; ++i) {
            if (i < wv) before += s_n[i];
            all += s_n[i];
        }
        if (b < w.B) w.nw[b] = before;
        if (wv == 0) w.ng[blockIdx.x] = all;
    }
}

// ng[0..G) -> exclusive prefix sums, ng[G] = sum.  One workgroup.  A round covers SCAN_SUB
// stretches of SCAN_BLOCK * SCAN_ITEMS counts; their loads are issued together, so that the
// memory latency is paid once per round and not once per stretch.
__device__ __forceinline__ void scan_words(const Wire &w, uint32_t *s_wave) {
    constexpr uint32_t STRETCH = SCAN_BLOCK * SCAN_ITEMS;
    uint32_t carry = 0;
    for (uint32_t base = 0; base < w.G; base += STRETCH * SCAN_SUB) {
        uint32_t v[SCAN_SUB][SCAN_ITEMS];
#pragma unroll
        for (uint32_t u = 0; u < SCAN_SUB; ++u) {
            const uint32_t i0 = base + u * STRETCH + threadIdx.x * SCAN_ITEMS;
#pragma unroll
            for (uint32_t j = 0; j < SCAN_ITEMS; ++j) v[u][j] = i0 + j < w.G ? w.ng[i0 + j] : 0u;
        }
#pragma unroll
        for (uint32_t u = 0; u < SCAN_SUB; ++u) {
            const uint32_t i0 = base + u * STRETCH + threadIdx.x * SCAN_ITEMS;
            uint32_t sum = 0;
#pragma unroll
            for (uint32_t j = 0; j < SCAN_ITEMS; ++j) sum += v[u][j];
            uint32_t all;
            uint32_t run = carry + block_exclusive_scan<SCAN_BLOCK / WAVE>(sum, s_wave, all);
#pragma unroll
            for (uint32_t j = 0; j < SCAN_ITEMS; ++j) {
                if (i0 + j < w.G) w.ng[i0 + j] = run;
                run += v[u][j];
            }
            carry += all;
        }
    }
    if (threadIdx.x == 0) w.ng[w.G] = carry;
}

// packer: offsets of the blocks' words, the header, and the length of the stream
__global__ __launch_bounds__(SCAN_BLOCK) void k_wire_scan_pack(Wire w, uint32_t *out, uint64_t cap, uint64_t *words_out) {
    __shared__ uint32_t s_wave[SCAN_BLOCK / WAVE];
    scan_words(w, s_wave);
    __syncthreads();
    if (threadIdx.x == 0) *words_out = w.delta_at + w.ng[w.G] + w.total;
    if (4 + (uint64_t)w.L > cap) return;
    if (threadIdx.x == 0) {
        out[0] = MAGIC;
        out[1] = w.L;
        out[2] = (uint32_t)w.total;
        out[3] = (uint32_t)(w.total >> 32);
    }
    for (uint32_t l = threadIdx.x; l < w.L; l += SCAN_BLOCK) out[4 + l] = (uint32_t)(w.off[l + 1] - w.off[l]);
}

// pass 2 of the packer: the delta words of every block and its values
__global__ __launch_bounds__(BLOCK) void k_wire_write(Wire w, const uint32_t *idx, const uint32_t *val, uint32_t *out,
                                                      uint64_t cap) {
    __shared__ uint32_t s_bits[WAVES][WAVE];
    const uint32_t lane = threadIdx.x & (WAVE - 1), wv = threadIdx.x / WAVE;
    const uint32_t b = blockIdx.x * WAVES + wv;
    if (b >= w.B) return;  // whole waves leave; no workgroup barrier below
    uint32_t l, m;
    uint64_t e0;
    locate(w, b, l, e0, m);
    const uint32_t mine = lane < m ? idx[e0 + lane] : 0u;
    const uint32_t gap = gap_of(mine, lane, m);
    const uint32_t width = bit_length(wave_or(gap));
    const uint32_t nwords = ((m - 1) * width + 31u) >> 5;
    s_bits[wv][lane] = 0;
    __builtin_amdgcn_wave_barrier();
    if (lane >= 1 && lane < m && width) {
        const uint32_t p = (lane - 1) * width, at = p >> 5, sh = p & 31u;
        atomicOr(&s_bits[wv][at], gap << sh);
        if (sh + width > 32) atomicOr(&s_bits[wv][at + 1], gap >> (32 - sh));
    }
    __builtin_amdgcn_wave_barrier();
    const uint64_t pos = w.delta_at + w.ng[b / SUPER] + w.nw[b];
    if (lane < nwords && pos + lane < cap) out[pos + lane] = s_bits[wv][lane];
    const uint64_t vpos = w.delta_at + w.ng[w.G] + e0 + lane;
    if (lane < m && vpos < cap) out[vpos] = val[e0 + lane];
}

// flags of the unpacker
enum : uint32_t { BAD_HEADER = 1, BAD_WIDTH = 2, BAD_LENGTH = 4, BAD_INDEX = 8 };

// unpacker, pass 1: word count of every block from its width byte, as an offset inside its
// group of SUPER blocks (16 neighbouring lanes), and the group's total
__global__ __launch_bounds__(BLOCK) void k_wire_widths(Wire w, const uint32_t *in, uint64_t nwords, uint32_t *flags) {
    const uint32_t b = blockIdx.x * BLOCK + threadIdx.x;
    uint32_t count = 0;
    if (b < w.B) {
        uint32_t l, m;
        uint64_t e0;
        locate(w, b, l, e0, m);
        const uint64_t byte = w.width_at * 4 + b;
        uint32_t width = byte < nwords * 4 ? reinterpret_cast<const uint8_t *>(in)[byte] : 0u;
        if (width > 32) {
            atomicOr(flags, (uint32_t)BAD_WIDTH);
            width = 32;
        }
        count = ((m - 1) * width + 31u) >> 5;
    }
    uint32_t incl = count;
#pragma unroll
    for (uint32_t d = 1; d < SUPER; d <<= 1) {
        const uint32_t y = __shfl_up(incl, d, SUPER);
        if ((threadIdx.x & (SUPER - 1)) >= d) incl += y;
    }
    if (b < w.B) w.nw[b] = incl - count;
    if ((b & (SUPER - 1)) == SUPER - 1 && b / SUPER < w.G) w.ng[b / SUPER] = incl;
}

// unpacker: offsets of the blocks' words; header and stream length against what the host expects
__global__ __launch_bounds__(SCAN_BLOCK) void k_wire_scan_unpack(Wire w, const uint32_t *in, uint64_t nwords,
                                                                 uint32_t *flags) {
    __shared__ uint32_t s_wave[SCAN_BLOCK / WAVE];
    scan_words(w, s_wave);
    __syncthreads();
    uint32_t bad = 0;
    if (threadIdx.x == 0) {
        if (nwords < 4 || in[0] != MAGIC || in[1] != w.L || in[2] != (uint32_t)w.total || in[3] != (uint32_t)(w.total >> 32))
            bad |= BAD_HEADER;
        if (w.delta_at + w.ng[w.G] + w.total != nwords) bad |= BAD_LENGTH;
    }
    for (uint32_t l = threadIdx.x; l < w.L; l += SCAN_BLOCK)
        if (4 + (uint64_t)l >= nwords || in[4 + l] != (uint32_t)(w.off[l + 1] - w.off[l])) bad |= BAD_HEADER;
    if (bad) atomicOr(flags, bad);
}

// unpacker, pass 2: indices by a wave prefix sum over the gaps, values copied
__global__ __launch_bounds__(BLOCK) void k_wire_read(Wire w, const uint32_t *in, uint64_t nwords, uint32_t *idx,
                                                     uint32_t *val, uint32_t *flags) {
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    const uint32_t b = blockIdx.x * WAVES + threadIdx.x / WAVE;
    if (b >= w.B) return;
    uint32_t l, m;
    uint64_t e0;
    locate(w, b, l, e0, m);
    const uint64_t byte = w.width_at * 4 + b;
    uint32_t width = byte < nwords * 4 ? reinterpret_cast<const uint8_t *>(in)[byte] : 0u;
    if (width > 32) width = 32;
    const uint64_t pos = w.delta_at + w.ng[b / SUPER] + w.nw[b];
    unsigned long long step = 0;  // distance to the previous entry
    if (lane >= 1 && lane < m) {
        uint32_t gap = 0;
        if (width) {
            const uint32_t p = (lane - 1) * width, sh = p & 31u;
            const uint64_t at = pos + (p >> 5);
            gap = at < nwords ? in[at] >> sh : 0u;
            if (sh + width > 32 && at + 1 < nwords) gap |= in[at + 1] << (32 - sh);
            if (width < 32) gap &= (1u << width) - 1u;
        }
        step = (unsigned long long)gap + 1ull;
    }
    if (lane == 0) step = w.first_at + b < nwords ? in[w.first_at + b] : 0u;
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {  // inclusive prefix sum: lane i holds its index
        const unsigned long long y = __shfl_up(step, d);
        if (lane >= (uint32_t)d) step += y;
    }
    if (lane < m) {
        if (step > 0xffffffffull) atomicOr(flags, (uint32_t)BAD_INDEX);
        idx[e0 + lane] = (uint32_t)step;
        const uint64_t vpos = w.delta_at + w.ng[w.G] + e0 + lane;
        val[e0 + lane] = vpos < nwords ? in[vpos] : 0u;
    }
}

struct WirePlan {
    std::vector<uint32_t> blk_base;
    uint64_t B = 0, total = 0, first_at = 0, width_at = 0, delta_at = 0;
    size_t blk_base_at = 0, nw_at = 0, ng_at = 0, bytes = 0;
    uint64_t G = 0;
};

int make_wire_plan(const uint64_t *layer_off, uint32_t L, WirePlan &p) {
    if (!layer_off) return ADACOMP_ERR_NULL;
    if (layer_off[0] != 0) return ADACOMP_ERR_LAYER_MISMATCH;
    p.blk_base.assign((size_t)L + 1, 0);
    uint64_t B = 0;
    for (uint32_t l = 0; l < L; ++l) {
        if (layer_off[l + 1] < layer_off[l]) return ADACOMP_ERR_LAYER_MISMATCH;
        if (layer_off[l + 1] - layer_off[l] > 0xffffffffull) return ADACOMP_ERR_LAYER_TOO_LARGE;
        p.blk_base[l] = (uint32_t)B;
        B += (layer_off[l + 1] - layer_off[l] + WAVE - 1) / WAVE;
        if (B > 0x7fffffffull) return ADACOMP_ERR_LAYER_TOO_LARGE;
    }
    p.blk_base[L] = (uint32_t)B;
    p.B = B;
    p.total = layer_off[L];
    if (p.total > 0xffffffffull) return ADACOMP_ERR_LAYER_TOO_LARGE;  // word offsets are 32-bit
    p.first_at = 4 + (uint64_t)L;
    p.width_at = p.first_at + B;
    p.delta_at = p.width_at + (B + 3) / 4;
    p.blk_base_at = 0;
    p.G = (B + SUPER - 1) / SUPER;
    p.nw_at = align_up(((size_t)L + 1) * sizeof(uint32_t), 256);
    p.ng_at = p.nw_at + align_up(((size_t)B + 1) * sizeof(uint32_t), 256);
    p.bytes = p.ng_at + align_up(((size_t)p.G + 1) * sizeof(uint32_t), 256);
    return ADACOMP_OK;
}

Wire device_view(const WirePlan &p, uint32_t L, const uint64_t *off_dev, char *wsb) {
    Wire w;
    w.off = off_dev;
    w.blk_base = reinterpret_cast<const uint32_t *>(wsb + p.blk_base_at);
    w.nw = reinterpret_cast<uint32_t *>(wsb + p.nw_at);
    w.ng = reinterpret_cast<uint32_t *>(wsb + p.ng_at);
    w.L = L;
    w.B = (uint32_t)p.B;
    w.G = (uint32_t)p.G;
    w.total = p.total;
    w.first_at = p.first_at;
    w.width_at = p.width_at;
    w.delta_at = p.delta_at;
    return w;
}

int check_update(const adacomp_update_t *u, const WirePlan &p) {
    if (p.total > u->cap) return ADACOMP_ERR_CAPACITY;
    if (!u->layer_off_dev || (p.total && (!u->idx || !u->val))) return ADACOMP_ERR_NULL;
    if (((uintptr_t)u->idx & 3u) || ((uintptr_t)u->val & 3u) || ((uintptr_t)u->layer_off_dev & 7u))
        return ADACOMP_ERR_ALIGNMENT;
    return ADACOMP_OK;
}

}  // namespace
}  // namespace adacomp

using namespace adacomp;

#define CHECK_LAUNCH()                                               \
    do {                                                             \
        if (hipGetLastError() != hipSuccess) return ADACOMP_ERR_HIP; \
    } while (0)

extern "C" int adacomp_wire_bound(const uint64_t *layer_off, uint32_t L, uint64_t *words) {
    if (!words) return ADACOMP_ERR_NULL;
    WirePlan p;
    const int rc = make_wire_plan(layer_off, L, p);
    if (rc) return rc;
    *words = p.delta_at + p.total /* at most one delta word per entry */ + p.total;
    return ADACOMP_OK;
}

extern "C" int adacomp_wire_workspace(const uint64_t *layer_off, uint32_t L, size_t *bytes) {
    if (!bytes) return ADACOMP_ERR_NULL;
    WirePlan p;
    const int rc = make_wire_plan(layer_off, L, p);
    if (rc) return rc;
    *bytes = p.bytes;
    return ADACOMP_OK;
}

extern "C" int adacomp_wire_pack(const adacomp_update_t *update, uint32_t *wire, uint64_t wire_cap,
                                 uint64_t *wire_words_dev, void *workspace, size_t ws_bytes, void *hip_stream) {
    if (!update || !wire_words_dev || (wire_cap && !wire)) return ADACOMP_ERR_NULL;
    const uint32_t L = update->num_layers;
    WirePlan p;
    int rc = make_wire_plan(update->layer_off, L, p);
    if (rc) return rc;
    rc = check_update(update, p);
    if (rc) return rc;
    if (((uintptr_t)wire & 3u) || ((uintptr_t)wire_words_dev & 7u)) return ADACOMP_ERR_ALIGNMENT;
    if (!workspace || ((uintptr_t)workspace & 255u) || ws_bytes < p.bytes) return ADACOMP_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char *wsb = static_cast<char *>(workspace);
    const Wire w = device_view(p, L, update->layer_off_dev, wsb);
    if (put_async(wsb + p.blk_base_at, p.blk_base.data(), p.blk_base.size() * sizeof(uint32_t), s) != hipSuccess)
        return ADACOMP_ERR_HIP;
    const unsigned grid = (unsigned)((p.B + WAVES - 1) / WAVES);
    if (p.B) {
        ADACOMP_LAUNCH(ADACOMP_KERNEL_WIRE_MEASURE, k_wire_measure, dim3((unsigned)p.G), dim3(SUPER * WAVE), s, w,
                       update->idx, wire, wire_cap);
        CHECK_LAUNCH();
    }
    ADACOMP_LAUNCH(ADACOMP_KERNEL_WIRE_SCAN, k_wire_scan_pack, dim3(1), dim3(SCAN_BLOCK), s, w, wire, wire_cap,
                   wire_words_dev);
    CHECK_LAUNCH();
    if (p.B) {
        ADACOMP_LAUNCH(ADACOMP_KERNEL_WIRE_WRITE, k_wire_write, dim3(grid), dim3(BLOCK), s, w, update->idx,
                       reinterpret_cast<const uint32_t *>(update->val), wire, wire_cap);
        CHECK_LAUNCH();
    }
    return ADACOMP_OK;
}

extern "C" int adacomp_wire_unpack(const uint32_t *wire, uint64_t wire_words, const adacomp_update_t *update,
                                   uint32_t *flags_dev, void *workspace, size_t ws_bytes, void *hip_stream) {
    if (!update || !flags_dev || (wire_words && !wire)) return ADACOMP_ERR_NULL;
    const uint32_t L = update->num_layers;
    WirePlan p;
    int rc = make_wire_plan(update->layer_off, L, p);
    if (rc) return rc;
    rc = check_update(update, p);
    if (rc) return rc;
    if (((uintptr_t)wire & 3u) || ((uintptr_t)flags_dev & 3u)) return ADACOMP_ERR_ALIGNMENT;
    if (!workspace || ((uintptr_t)workspace & 255u) || ws_bytes < p.bytes) return ADACOMP_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char *wsb = static_cast<char *>(workspace);
    const Wire w = device_view(p, L, update->layer_off_dev, wsb);
    if (put_async(wsb + p.blk_base_at, p.blk_base.data(), p.blk_base.size() * sizeof(uint32_t), s) != hipSuccess ||
        put_async(update->layer_off_dev, update->layer_off, ((size_t)L + 1) * sizeof(uint64_t), s) != hipSuccess ||
        fill_u32_async(flags_dev, 0u, 1, s) != hipSuccess)
        return ADACOMP_ERR_HIP;
    if (p.B) {
        ADACOMP_LAUNCH(ADACOMP_KERNEL_WIRE_MEASURE, k_wire_widths, dim3((unsigned)((p.B + BLOCK - 1) / BLOCK)),
                       dim3(BLOCK), s, w, wire, wire_words, flags_dev);
        CHECK_LAUNCH();
    }
    ADACOMP_LAUNCH(ADACOMP_KERNEL_WIRE_SCAN, k_wire_scan_unpack, dim3(1), dim3(SCAN_BLOCK), s, w, wire, wire_words,
                   flags_dev);
    CHECK_LAUNCH();
    if (p.B) {
        ADACOMP_LAUNCH(ADACOMP_KERNEL_WIRE_READ, k_wire_read, dim3((unsigned)((p.B + WAVES - 1) / WAVES)), dim3(BLOCK),
                       s, w, wire, wire_words, update->idx, reinterpret_cast<uint32_t *>(update->val), flags_dev);
        CHECK_LAUNCH();
    }
    return ADACOMP_OK;
}
