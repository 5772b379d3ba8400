/*
 * AdaComp CPU oracle  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A deliberately plain, slow, single-threaded restatement of the two halves of
 * AdaComp's data-parallel hot path, written from the paper alone:
 *
 *   - worker side, SELECT_GRAD (Alg. 1; Sec. 4 "Selection method"; Table 1 row c):
 *     for every weight matrix V_l and bias vector beta_l separately, keep the
 *     (100*c)% entries that are largest in absolute value;
 *   - parameter-server side (Alg. 2; eqs. 3, 4, 5): for every entry of a received
 *     sparse update, count how many updates applied since the sender's pull
 *     changed that very parameter (sigma_k, eq. 3), divide the learning rate by
 *     that count when it is non-zero (alpha_k, eq. 5), and step the parameter
 *     (eq. 4).  The history is what Sec. 4 "Complexity" describes: per applied
 *     update the sorted list of indices of its non-zero entries, searched by
 *     bisection; a bitmap variant exists only as a brute-force cross-check.
 *
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
 * this file.  It shares no code, header, table or helper with the HIP library.
 *
 * Readings of points the paper leaves open (each isolated in one function):
 *   count rule        oracle_count()      k = 0 if c == 0, N if c == 1, else
 *                                         min(N, max(1, ceil((c*N)*(1-2^-40))))
 *   magnitude order   mag_key()           unsigned order of the IEEE-754 bit
 *                                         pattern with the sign bit cleared
 *   ties              select              equal magnitudes: lower index first
 *   "!= 0" in eq. 3   is_nonzero()        value != +-0 (denormals count)
 *   op order eq. 4-5  step_f32/step_f64   divide, multiply, subtract, each rounded
 *
 * A third part is not from the paper, which leaves the byte encoding of an update
 * open (footnote of Sec. 4 "Overview"): the wire format of this library (block-wise
 * delta coding of the sorted indices, values as they are), written out from its
 * definition in include/adacomp.h so that real bytes per update can be set against
 * the paper's traffic model (Sec. 3.2: I x M x c).  Pins: tests/test_oracle_wire.py.
 *
 * Parity pins: tests/test_oracle_select.py, tests/test_oracle_apply.py (closed
 * forms, brute force, library cross-checks, hand examples in tests/golden/).
 * The count rule and the "!= 0" reading are choices the paper does not
 * determine: parity unpinned by the paper for those two, pinned by definition.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ helpers */

static uint32_t f32_bits(float x) {
    uint32_t b;
    memcpy(&b, &x, sizeof b);
    return b;
}

/* |x| as an integer that orders exactly like the absolute value (Alg. 1,
 * SELECT_GRAD: "largest ... in absolute value"); +x and -x tie, +-0 -> 0. */
static uint32_t mag_key(float x) { return f32_bits(x) & 0x7fffffffu; }

/* indicator of eq. 3: Delta Theta_k(u) != 0 */
static int is_nonzero(float x) { return mag_key(x) != 0u; }

static int cmp_u64(const void *a, const void *b) {
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x > y) - (x < y);
}

static int cmp_u32(const void *a, const void *b) {
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return (x > y) - (x < y);
}

/* ------------------------------------------------------------------- select */

/* Number of entries "(100*c)%" of an N-entry tensor stands for (Alg. 1,
 * SELECT_GRAD; c in (0,1], Sec. 3.2).  The paper gives no rounding rule. */
uint64_t adacomp_oracle_count(uint64_t n, double rate) {
    if (n == 0 || !(rate > 0.0)) return 0;
    if (rate >= 1.0) return n;
    double x = rate * (double)n;
    double y = x * (1.0 - 0x1p-40);
    double k = ceil(y);
    if (k < 1.0) k = 1.0;
    if (k > (double)n) k = (double)n;
    return (uint64_t)k;
}

/* One tensor: order all entries by magnitude (descending) with the lower index
 * first among equals, keep the first k, report them in ascending index order
 * with the value copied bit for bit.  Returns 0, or -1 on allocation failure /
 * bad arguments. */
int adacomp_oracle_select_layer(const float *g, uint64_t n, uint64_t k,
                                uint32_t *idx_out, float *val_out) {
    if (k > n || n > 0xffffffffull) return -1;
    if (k == 0) return 0;
    uint64_t *order = (uint64_t *)malloc(n * sizeof *order);
    if (!order) return -1;
    for (uint64_t i = 0; i < n; ++i) {
        /* ascending sort of (inverted magnitude, index) == descending magnitude,
         * ascending index among equal magnitudes */
        uint64_t inv = 0x7fffffffu - mag_key(g[i]);
        order[i] = (inv << 32) | i;
    }
    qsort(order, n, sizeof *order, cmp_u64);
    for (uint64_t e = 0; e < k; ++e) idx_out[e] = (uint32_t)(order[e] & 0xffffffffu);
    free(order);
    qsort(idx_out, k, sizeof *idx_out, cmp_u32);
    for (uint64_t e = 0; e < k; ++e) val_out[e] = g[idx_out[e]];
    return 0;
}

/* All tensors of one update.  layer_off[L+1], idx[cap], val[cap] are outputs;
 * k_override (NULL or [L]) replaces the count rule per tensor. */
int adacomp_oracle_select(const float *const *layer_data, const uint64_t *layer_n,
                          uint32_t L, double rate, const uint64_t *k_override,
                          uint64_t *layer_off, uint32_t *idx, float *val,
                          uint64_t cap) {
    uint64_t off = 0;
    for (uint32_t l = 0; l < L; ++l) {
        uint64_t k = k_override ? k_override[l] : adacomp_oracle_count(layer_n[l], rate);
        if (k > layer_n[l] || off + k > cap) return -1;
        layer_off[l] = off;
        int rc = adacomp_oracle_select_layer(layer_data[l], layer_n[l], k, idx + off, val + off);
        if (rc) return rc;
        off += k;
    }
    layer_off[L] = off;
    return 0;
}

/* -------------------------------------------------------- parameter server */

enum { ORACLE_HISTORY_LISTS = 0, ORACLE_HISTORY_BITMAP = 1 };
enum { ORACLE_STALENESS_PER_PARAMETER = 0, ORACLE_STALENESS_GLOBAL = 1 };

typedef struct {
    /* sorted-list form: for tensor l, entries nz[off[l] .. off[l+1]) */
    uint64_t *off;   /* [L+1] */
    uint32_t *nz;    /* indices whose value was != 0, ascending per tensor */
    /* bitmap form: bit (base[l] + k) */
    uint8_t *bits;
} history_entry_t;

typedef struct {
    uint32_t L;
    uint64_t *n;        /* [L] tensor sizes */
    uint64_t *base;     /* [L+1] offsets of tensors in the flat coordinate space */
    int method;         /* ORACLE_HISTORY_* */
    uint64_t t;         /* PS timestamp i = number of updates applied so far */
    history_entry_t *H; /* H[u] for every applied update u (complete trace) */
    uint64_t H_cap;
} oracle_ps_t;

oracle_ps_t *adacomp_oracle_ps_create(uint32_t L, const uint64_t *n, int method) {
    oracle_ps_t *ps = (oracle_ps_t *)calloc(1, sizeof *ps);
    if (!ps) return NULL;
    ps->L = L;
    ps->method = method;
    ps->n = (uint64_t *)malloc((L ? L : 1) * sizeof *ps->n);
    ps->base = (uint64_t *)malloc((L + 1) * sizeof *ps->base);
    if (!ps->n || !ps->base) return NULL;
    ps->base[0] = 0;
    for (uint32_t l = 0; l < L; ++l) {
        ps->n[l] = n[l];
        ps->base[l + 1] = ps->base[l] + n[l];
    }
    return ps;
}

void adacomp_oracle_ps_destroy(oracle_ps_t *ps) {
    if (!ps) return;
    for (uint64_t u = 0; u < ps->t; ++u) {
        free(ps->H[u].off);
        free(ps->H[u].nz);
        free(ps->H[u].bits);
    }
    free(ps->H);
    free(ps->n);
    free(ps->base);
    free(ps);
}

uint64_t adacomp_oracle_ps_timestamp(const oracle_ps_t *ps) { return ps->t; }

/* 1 if update u changed parameter k of tensor l (the indicator of eq. 3) */
static int touched(const oracle_ps_t *ps, uint64_t u, uint32_t l, uint32_t k) {
    const history_entry_t *h = &ps->H[u];
    if (ps->method == ORACLE_HISTORY_BITMAP) {
        uint64_t b = ps->base[l] + k;
        return (h->bits[b >> 3] >> (b & 7)) & 1;
    }
    /* bisection in the sorted index list of that update (Sec. 4 "Complexity") */
    uint64_t lo = h->off[l], hi = h->off[l + 1];
    while (lo < hi) {
        uint64_t mid = lo + (hi - lo) / 2;
        if (h->nz[mid] < k) lo = mid + 1; else hi = mid;
    }
    return lo < h->off[l + 1] && h->nz[lo] == k;
}

/* eq. 3: number of updates u in [j, i-1] that changed parameter k */
static uint64_t sigma_k(const oracle_ps_t *ps, uint64_t j, uint64_t i, uint32_t l, uint32_t k) {
    uint64_t s = 0;
    for (uint64_t u = j; u < i; ++u) s += (uint64_t)touched(ps, u, l, k);
    return s;
}

/* eqs. 5 then 4 in single precision: one divide, one multiply, one subtract */
static float step_f32(float theta, float alpha, uint64_t sigma, float delta) {
    float a = alpha;
    if (sigma != 0) a = alpha / (float)sigma;
    float p = a * delta;
    return theta - p;
}

/* the same in double precision (parameters kept in double by the caller) */
static double step_f64(double theta, double alpha, uint64_t sigma, double delta) {
    double a = alpha;
    if (sigma != 0) a = alpha / (double)sigma;
    double p = a * delta;
    return theta - p;
}

static int history_append(oracle_ps_t *ps, const uint64_t *layer_off,
                          const uint32_t *idx, const float *val) {
    if (ps->t == ps->H_cap) {
        uint64_t nc = ps->H_cap ? 2 * ps->H_cap : 64;
        history_entry_t *nh = (history_entry_t *)realloc(ps->H, nc * sizeof *nh);
        if (!nh) return -1;
        ps->H = nh;
        ps->H_cap = nc;
    }
    history_entry_t *h = &ps->H[ps->t];
    memset(h, 0, sizeof *h);
    if (ps->method == ORACLE_HISTORY_BITMAP) {
        uint64_t nbytes = (ps->base[ps->L] + 7) / 8;
        h->bits = (uint8_t *)calloc(nbytes ? nbytes : 1, 1);
        if (!h->bits) return -1;
        for (uint32_t l = 0; l < ps->L; ++l)
            for (uint64_t e = layer_off[l]; e < layer_off[l + 1]; ++e)
                if (is_nonzero(val[e])) {
                    uint64_t b = ps->base[l] + idx[e];
                    h->bits[b >> 3] |= (uint8_t)(1u << (b & 7));
                }
    } else {
        uint64_t total = layer_off[ps->L];
        h->off = (uint64_t *)malloc((ps->L + 1) * sizeof *h->off);
        h->nz = (uint32_t *)malloc((total ? total : 1) * sizeof *h->nz);
        if (!h->off || !h->nz) return -1;
        uint64_t w = 0;
        for (uint32_t l = 0; l < ps->L; ++l) {
            h->off[l] = w;
            for (uint64_t e = layer_off[l]; e < layer_off[l + 1]; ++e)
                if (is_nonzero(val[e])) h->nz[w++] = idx[e];
        }
        h->off[ps->L] = w;
    }
    return 0;
}

/* One PS iteration (Alg. 2, body of the for loop): apply one received sparse
 * update whose sender pulled at timestamp pull_ts = j, then advance the
 * timestamp.  theta32 (array of L float pointers) or theta64 (L double
 * pointers) is updated in place; exactly one of them is non-NULL.
 * staleness_mode GLOBAL replaces sigma_k by i - j for every entry (the rule the
 * paper ascribes to its competitors, Sec. 5.2); PER_PARAMETER is AdaComp.
 * sigma_out, if non-NULL, receives the staleness used for each entry.
 * Returns 0; -1 bad argument / allocation; -2 pull_ts in the future. */
int adacomp_oracle_ps_apply(oracle_ps_t *ps, float *const *theta32, double *const *theta64,
                            const uint64_t *layer_off, const uint32_t *idx, const float *val,
                            uint64_t pull_ts, double lr, int staleness_mode,
                            uint64_t *sigma_out) {
    if (!ps || (!theta32) == (!theta64)) return -1;
    const uint64_t i = ps->t, j = pull_ts;
    if (j > i) return -2;
    for (uint32_t l = 0; l < ps->L; ++l)
        for (uint64_t e = layer_off[l]; e < layer_off[l + 1]; ++e)
            if (idx[e] >= ps->n[l]) return -1;

    const float lr32 = (float)lr;
    for (uint32_t l = 0; l < ps->L; ++l) {
        for (uint64_t e = layer_off[l]; e < layer_off[l + 1]; ++e) {
            const uint32_t k = idx[e];
            uint64_t s = (staleness_mode == ORACLE_STALENESS_GLOBAL)
                             ? (i - j)
                             : sigma_k(ps, j, i, l, k);
            if (sigma_out) sigma_out[e] = s;
            if (theta32)
                theta32[l][k] = step_f32(theta32[l][k], lr32, s, val[e]);
            else
                theta64[l][k] = step_f64(theta64[l][k], (double)lr32, s, (double)val[e]);
        }
    }
    if (history_append(ps, layer_off, idx, val)) return -1;
    ps->t = i + 1;
    return 0;
}


/* ------------------------------------------------------------------ wire format
 *
 * Not from the paper (it leaves the encoding open).  Little-endian 32-bit words:
 *
 *   [0] magic 0x31434441   [1] L   [2],[3] total entries (low, high)
 *   [4 .. 4+L)             k_l, entries of tensor l
 *   first[B]               B = sum_l ceil(k_l / 64) blocks; a block is up to 64 consecutive
 *                          entries of one tensor; first[b] = index of its first entry
 *   width[B]               one byte per block, zero-padded to a whole word
 *   deltas                 block after block: for the entries i = 1 .. m-1 of the block
 *                          d_i = idx_i - idx_{i-1} - 1 (indices ascend strictly), each in
 *                          w = width[b] bits, d_1 first, least significant bit first, bit p
 *                          of the block's stream = bit (p mod 32) of its word p / 32; the
 *                          last word is zero-padded; w = bit length of the largest d_i
 *   values[total]          the fp32 bit patterns, in entry order
 */

#define WIRE_MAGIC 0x31434441u
#define WIRE_BLOCK 64u

static uint32_t bit_length(uint32_t x) {
    uint32_t n = 0;
    while (x) {
        ++n;
        x >>= 1;
    }
    return n;
}

/* Upper bound of the words adacomp_oracle_wire_pack can produce (every width 32). */
uint64_t adacomp_oracle_wire_bound(const uint64_t *layer_off, uint32_t L) {
    uint64_t blocks = 0, delta_words = 0;
    for (uint32_t l = 0; l < L; ++l) {
        const uint64_t k = layer_off[l + 1] - layer_off[l];
        blocks += (k + WIRE_BLOCK - 1) / WIRE_BLOCK;
        delta_words += k; /* at most one word per entry */
    }
    return 4 + (uint64_t)L + blocks + (blocks + 3) / 4 + delta_words + layer_off[L];
}

/* Returns the number of words written, or 0 if `cap` words do not suffice / the
 * indices of a tensor do not ascend strictly. */
uint64_t adacomp_oracle_wire_pack(const uint64_t *layer_off, const uint32_t *idx, const float *val,
                                  uint32_t L, uint32_t *out, uint64_t cap) {
    const uint64_t total = layer_off[L];
    uint64_t blocks = 0;
    for (uint32_t l = 0; l < L; ++l) blocks += (layer_off[l + 1] - layer_off[l] + WIRE_BLOCK - 1) / WIRE_BLOCK;
    const uint64_t first_at = 4 + (uint64_t)L;
    const uint64_t width_at = first_at + blocks;
    const uint64_t delta_at = width_at + (blocks + 3) / 4;
    if (delta_at > cap) return 0;
    out[0] = WIRE_MAGIC;
    out[1] = L;
    out[2] = (uint32_t)(total & 0xffffffffu);
    out[3] = (uint32_t)(total >> 32);
    for (uint32_t l = 0; l < L; ++l) out[4 + l] = (uint32_t)(layer_off[l + 1] - layer_off[l]);
    for (uint64_t w = width_at; w < delta_at; ++w) out[w] = 0;
    uint64_t b = 0, pos = delta_at;
    for (uint32_t l = 0; l < L; ++l) {
        for (uint64_t e0 = layer_off[l]; e0 < layer_off[l + 1]; e0 += WIRE_BLOCK, ++b) {
            const uint64_t e1 = e0 + WIRE_BLOCK < layer_off[l + 1] ? e0 + WIRE_BLOCK : layer_off[l + 1];
            uint32_t largest = 0;
            for (uint64_t e = e0 + 1; e < e1; ++e) {
                if (idx[e] <= idx[e - 1]) return 0;
                const uint32_t d = idx[e] - idx[e - 1] - 1;
                if (d > largest) largest = d;
            }
            const uint32_t w = bit_length(largest);
            out[first_at + b] = idx[e0];
            out[width_at + b / 4] |= w << (8 * (b % 4));
            const uint64_t bits = (e1 - e0 - 1) * w, words = (bits + 31) / 32;
            if (pos + words > cap) return 0;
            for (uint64_t x = 0; x < words; ++x) out[pos + x] = 0;
            uint64_t p = 0; /* bit position in the block's stream */
            for (uint64_t e = e0 + 1; e < e1; ++e) {
                const uint32_t d = idx[e] - idx[e - 1] - 1;
                for (uint32_t i = 0; i < w; ++i, ++p)
                    if ((d >> i) & 1u) out[pos + p / 32] |= 1u << (p % 32);
            }
            pos += words;
        }
    }
    if (pos + total > cap) return 0;
    for (uint64_t e = 0; e < total; ++e) out[pos + e] = f32_bits(val[e]);
    return pos + total;
}

/* Inverse.  layer_off (L+1), idx and val (cap entries) are outputs.  Returns 0, or a
 * negative number naming what is wrong with the stream. */
int adacomp_oracle_wire_unpack(const uint32_t *in, uint64_t nwords, uint32_t L, uint64_t cap,
                               uint64_t *layer_off, uint32_t *idx, float *val) {
    if (nwords < 4 || in[0] != WIRE_MAGIC) return -1;
    if (in[1] != L || nwords < 4 + (uint64_t)L) return -2;
    const uint64_t total = (uint64_t)in[2] | ((uint64_t)in[3] << 32);
    uint64_t blocks = 0, sum = 0;
    layer_off[0] = 0;
    for (uint32_t l = 0; l < L; ++l) {
        sum += in[4 + l];
        layer_off[l + 1] = sum;
        blocks += ((uint64_t)in[4 + l] + WIRE_BLOCK - 1) / WIRE_BLOCK;
    }
    if (sum != total || total > cap) return -3;
    const uint64_t first_at = 4 + (uint64_t)L;
    const uint64_t width_at = first_at + blocks;
    const uint64_t delta_at = width_at + (blocks + 3) / 4;
    if (delta_at > nwords) return -4;
    uint64_t b = 0, pos = delta_at;
    for (uint32_t l = 0; l < L; ++l) {
        for (uint64_t e0 = layer_off[l]; e0 < layer_off[l + 1]; e0 += WIRE_BLOCK, ++b) {
            const uint64_t e1 = e0 + WIRE_BLOCK < layer_off[l + 1] ? e0 + WIRE_BLOCK : layer_off[l + 1];
            const uint32_t w = (in[width_at + b / 4] >> (8 * (b % 4))) & 0xffu;
            if (w > 32) return -5;
            const uint64_t words = ((e1 - e0 - 1) * w + 31) / 32;
            if (pos + words > nwords) return -4;
            uint64_t prev = in[first_at + b], p = 0;
            idx[e0] = (uint32_t)prev;
            for (uint64_t e = e0 + 1; e < e1; ++e) {
                uint64_t d = 0;
                for (uint32_t i = 0; i < w; ++i, ++p) d |= (uint64_t)((in[pos + p / 32] >> (p % 32)) & 1u) << i;
                prev += d + 1;
                if (prev > 0xffffffffull) return -6;
                idx[e] = (uint32_t)prev;
            }
            pos += words;
        }
    }
    if (pos + total != nwords) return -7;
    memcpy(val, in + pos, total * sizeof(float));
    return 0;
}
