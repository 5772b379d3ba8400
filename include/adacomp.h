/*
 * adacomp.h -- C ABI of the MI355X (gfx950) implementation of AdaComp's
 * data-parallel hot path.
 *
 *   worker side            adacomp_select()  SELECT_GRAD of Alg. 1: per tensor (each
 *                                            weight matrix V_l and bias vector beta_l
 *                                            on its own), keep the (100*c)% entries
 *                                            largest in absolute value
 *   parameter-server side  adacomp_apply()   loop body of Alg. 2 for a queue of
 *                                            received updates: per-parameter staleness
 *                                            (eq. 3), learning rate alpha/sigma_k
 *                                            (eq. 5), parameter step (eq. 4)
 *
 * Conventions common to all calls
 *   - "DEVICE" pointers are HIP device memory of the current device, "HOST" pointers
 *     ordinary host memory.  Every buffer is allocated and owned by the caller; the
 *     library allocates no device memory, keeps no global state (aside from the optional event
 *     timing at the end of this header and the built-in scratch of adacomp_select_noalloc) and
 *     never synchronises the device.
 *     All device work is enqueued on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and is complete when that stream has drained.
 *     Host arrays are read before the call returns.
 *   - Return value 0 on success, a negative ADACOMP_ERR_* otherwise.  Arguments are
 *     checked before anything is enqueued: a failing call has no side effect.
 *   - Sizes are in elements unless a name says bytes.  A tensor has at most
 *     2^32 - 1 elements.  Zero-element tensors are legal.
 *   - Test hooks.  A few environment variables choose between execution plans that give
 *     identical results (ADACOMP_APPLY_PLAN, ADACOMP_SWEEP_KERNEL, ADACOMP_TPB,
 *     ADACOMP_SELECT_SMALL, ADACOMP_SELECT_FUSED, ADACOMP_SELECT_GROUP_MB).  They exist for the
 *     library's own tests and measurements, are read once at the start of a call, and are not
 *     part of this interface: leave them unset.  A *_workspace call and the call it sizes each
 *     derive the plan from what they see; if a hook changes in between and the plan then needs
 *     more bytes, the call is refused with ADACOMP_ERR_WORKSPACE.
 */
#ifndef ADACOMP_H
#define ADACOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ADACOMP_OK = 0,
    ADACOMP_ERR_NULL = -1,            /* a required pointer is NULL                          */
    ADACOMP_ERR_RATE = -2,            /* rate is NaN or outside [0, 1]                       */
    ADACOMP_ERR_LAYER_TOO_LARGE = -3, /* a tensor has 2^32 or more elements                  */
    ADACOMP_ERR_CAPACITY = -4,        /* update buffers hold fewer than sum_l k_l entries    */
    ADACOMP_ERR_WORKSPACE = -5,       /* workspace NULL, misaligned (256 B) or too small     */
    ADACOMP_ERR_LAYER_MISMATCH = -6,  /* update / state tensor count or sizes differ from params */
    ADACOMP_ERR_FUTURE_PULL = -7,     /* an update's pull_ts is later than its apply time    */
    ADACOMP_ERR_K_RANGE = -8,         /* k_override[l] > n_l                                 */
    ADACOMP_ERR_HISTORY = -9,         /* pull_ts precedes the oldest remembered update       */
    ADACOMP_ERR_LR = -10,             /* learning rate is not finite                         */
    ADACOMP_ERR_ALIGNMENT = -11,      /* a float/uint32 device pointer is not 4-byte aligned */
    ADACOMP_ERR_HIP = -12,            /* a HIP runtime call (kernel launch) failed           */
    ADACOMP_ERR_SCRATCH_LIMIT = -13   /* adacomp_select_noalloc: the call needs more scratch than
                                         ADACOMP_SELECT_NOALLOC_SCRATCH_BYTES                */
};

/* One tensor of a worker's dense update Delta Theta^(w): a V_l or a beta_l
 * (Sec. 4 "Selection method").  data: DEVICE, n floats, read only. */
typedef struct {
    const float *data;
    uint64_t n;
} adacomp_layer_t;

/* The slice of Theta that corresponds to one tensor; data: DEVICE, n floats,
 * updated in place by adacomp_apply (eq. 4). */
typedef struct {
    float *data;
    uint64_t n;
} adacomp_param_layer_t;

/* A compressed update Delta~Theta^(w) (Table 1; Alg. 1 lines "SELECT_GRAD" and
 * "Push") together with the timestamp the worker pulled.  The paper leaves the
 * encoding open (footnote of Sec. 4); here: per tensor, the selected entries as
 * (index within the tensor, value) pairs in strictly ascending index order, the
 * tensors laid end to end, structure-of-arrays.
 *   layer_off      HOST   [num_layers+1]  entries of tensor l are [off[l], off[l+1])
 *   layer_off_dev  DEVICE [num_layers+1]  the same numbers, for the kernels
 *   idx            DEVICE [cap]           uint32 index local to the tensor
 *   val            DEVICE [cap]           value, bit-identical to the dense entry
 *   cap                                   capacity of idx/val in entries
 *   pull_ts                               j: PS timestamp the worker fetched (Alg. 1
 *                                         "Pull"); not touched by adacomp_select
 * adacomp_select fills layer_off, layer_off_dev, idx, val.  adacomp_apply reads all. */
typedef struct {
    uint32_t num_layers;
    uint64_t *layer_off;
    uint64_t *layer_off_dev;
    uint32_t *idx;
    float *val;
    uint64_t cap;
    uint64_t pull_ts;
} adacomp_update_t;

/* Parameter-server staleness state (Alg. 2; Sec. 4 "Algorithm details": the PS keeps a
 * timestamp and a trace of received updates).  Caller-owned memory whose contents the
 * library defines; zero-initialise t and history_len for a fresh server.
 *   t            i: number of updates applied so far (advanced by adacomp_apply)
 *   cnt          HOST array [num_layers] of DEVICE pointers; cnt[l] holds n_l uint32
 *                counters, one per parameter of tensor l.  Scratch of the library: when a
 *                call executes update by update, an applied non-zero entry for k
 *                increments cnt[l][k] (unless no later update of the call looks back on
 *                it), and the part of sigma_k (eq. 3) that lies inside the call is a
 *                difference of two readings of it.  Only differences are used: the values
 *                need no initialisation and mean nothing between calls.
 *   history_cap  d: how many applied updates the trace remembers (Sec. 4 "Complexity":
 *                the last d updates, d = the worst delay); 0 = none
 *   history_len  remembered so far (maintained by adacomp_apply)
 *   history      HOST ring [history_cap], maintained by adacomp_apply: slot (u mod
 *                history_cap) describes applied update u.  Only descriptors are kept: the
 *                DEVICE buffers idx/val/layer_off_dev of an applied update must stay
 *                allocated and unchanged until history_cap later updates have been
 *                applied and their stream work has finished
 *   history_off  HOST [history_cap * (num_layers + 1)], maintained by adacomp_apply
 *                (copies of the remembered updates' layer_off)
 * With history_cap = 0, history and history_off may be NULL. */
typedef struct {
    uint64_t t;
    uint32_t num_layers;
    uint32_t **cnt;
    uint32_t history_cap;
    uint32_t history_len;
    adacomp_update_t *history;
    uint64_t *history_off;
} adacomp_state_t;

/* k_l: how many entries "(100*c)%" of an n-entry tensor means (Alg. 1,
 * SELECT_GRAD; c = rate in [0,1], Table 1).  The paper states no rounding:
 * 0 if rate == 0 or n == 0; n if rate == 1; otherwise
 * min(n, max(1, ceil((rate*n) * (1 - 2^-40)))) in IEEE double.  Returns 0 for an
 * invalid rate.  Pure host function. */
uint64_t adacomp_count(uint64_t n, double rate);

/* Bytes of DEVICE workspace adacomp_select needs for tensors of sizes n[0..L) at
 * `rate` (k_override as in adacomp_select).  Depends only on these arguments,
 * never on data.  HOST pointers.  Pure host function. */
int adacomp_select_workspace(const uint64_t *n, uint32_t L, double rate,
                             const uint64_t *k_override, size_t *bytes);

/* SELECT_GRAD (Alg. 1): for each of the L tensors keep the k_l entries of largest
 * magnitude, k_l = k_override[l] if k_override != NULL else adacomp_count(n_l, rate).
 * Magnitudes are compared exactly (IEEE bit pattern without the sign: denormals
 * are not flushed, +x ties -x, +-0 are the smallest, NaN patterns order above
 * infinity); among equal magnitudes the lower index is kept.  Exactly k_l entries
 * are produced per tensor, explicit zeros included if k_l exceeds the number of
 * non-zeros.
 *   layers      HOST [L]; layers[l].data DEVICE
 *   k_override  HOST [L] or NULL
 *   out         HOST struct; out->num_layers must equal L; out->layer_off (HOST,
 *               L+1) is filled before the call returns, since k_l does not depend
 *               on the data; out->layer_off_dev, idx, val (DEVICE) are filled by the
 *               enqueued kernels; out->cap >= sum_l k_l
 *   workspace   DEVICE, 256-byte aligned, >= adacomp_select_workspace() bytes;
 *               contents are scratch, may be reused by the next call on the same stream
 * Calls sharing a workspace must be on the same stream. */
int adacomp_select(const adacomp_layer_t *layers, uint32_t L, double rate,
                   const uint64_t *k_override, adacomp_update_t *out,
                   void *workspace, size_t ws_bytes, void *hip_stream);

/* adacomp_select for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, result and errors as adacomp_select, except that the scratch memory is a buffer of
 * ADACOMP_SELECT_NOALLOC_SCRATCH_BYTES that is part of the library's device code: every GPU the
 * library runs on holds one copy until the process ends.  The call allocates nothing on the
 * device and frees nothing.  The device that hip_stream belongs to must be the current device.
 * A call whose tensors need more scratch than that (adacomp_select_workspace() tells how much:
 * about 3 MB for a 3.3M-parameter model at 1 %) is refused with ADACOMP_ERR_SCRATCH_LIMIT before
 * anything is enqueued.  All calls on one GPU share that GPU's buffer, which keeps the previous
 * call's contents (the kernels clear what they need cleared): calls on the same stream run one
 * after the other and are safe, calls that overlap on one GPU (different streams, or threads
 * with streams of their own) race. */
#define ADACOMP_SELECT_NOALLOC_SCRATCH_BYTES (32u << 20)
int adacomp_select_noalloc(const adacomp_layer_t *layers, uint32_t L, double rate,
                           const uint64_t *k_override, adacomp_update_t *out, void *hip_stream);

/* Bytes of DEVICE workspace adacomp_apply needs for a queue of Q updates (HOST array;
 * num_layers, layer_off and pull_ts are read) on L parameter tensors of sizes n[0..L)
 * (HOST), applied to state st (HOST; only t and the history fields are read; NULL = a
 * fresh state).  Depends on these sizes and timestamps only.  Returns the same timestamp
 * errors as adacomp_apply would. */
int adacomp_apply_workspace(const uint64_t *n, uint32_t L, const adacomp_state_t *st,
                            const adacomp_update_t *updates, uint32_t Q, size_t *bytes);

/* Parameter-server iterations (Alg. 2, loop body) for a queue: updates[0..Q) are
 * applied in array order as iterations i = st->t, st->t + 1, ...; for each entry
 * (k, v) of update q with pull timestamp j:
 *     sigma_k = #{ u in [j, i-1] : update u had a non-zero entry for k }   (eq. 3)
 *     alpha_k = lr / sigma_k if sigma_k != 0 else lr                        (eq. 5)
 *     Theta_k = Theta_k - alpha_k * v                                       (eq. 4)
 * in fp32, as one correctly rounded divide, one multiply and one subtract.  An
 * entry counts as non-zero iff its value is not +-0.  An empty update still
 * advances the timestamp.  On success st->t += Q (at enqueue time).
 *   params   HOST [L]; data DEVICE, updated in place
 *   st       HOST struct; st->num_layers == L; st->cnt HOST [L] of DEVICE pointers
 *   updates  HOST [Q]; each must have num_layers == L, idx < n_l, strictly ascending
 *            per tensor (see adacomp_update_validate for updates from elsewhere);
 *            pull_ts <= apply time of that update (else ADACOMP_ERR_FUTURE_PULL) and
 *            pull_ts >= st->t - (remembered updates) (else ADACOMP_ERR_HISTORY): an
 *            update pulled before this call has the earlier part of its window
 *            searched in the remembered updates' sorted index lists, by bisection, as
 *            Sec. 4 "Complexity" describes; with history_cap = 0 every pull_ts must be
 *            >= st->t; an update without entries has no staleness to look up and may
 *            carry any pull_ts that is not in the future
 *   lr       alpha, finite
 *   workspace DEVICE, 256-byte aligned, >= adacomp_apply_workspace() bytes
 * The queue is executed either update by update (scatter) or in one sweep over
 * coordinate tiles; the choice is made from the sizes and does not change the result. */
int adacomp_apply(const adacomp_param_layer_t *params, uint32_t L, adacomp_state_t *st,
                  const adacomp_update_t *updates, uint32_t Q, float lr,
                  void *workspace, size_t ws_bytes, void *hip_stream);

/* The same queue under the learning-rate rule that Sec. 5.2 describes for the competitors, ASGD
 * and Comp-ASGD: one staleness per update, sigma = i - j for every entry of it, alpha = lr / sigma
 * if sigma != 0.  (Their selection, the largest entries across the whole model, is
 * adacomp_select on the model passed as one tensor.)  Arguments, checks and stream semantics as
 * adacomp_apply; no counters are needed and st->cnt is neither read nor written; any
 * pull_ts <= apply time is accepted.  With history_cap > 0 the applied updates are entered
 * into the trace exactly as adacomp_apply enters them (same lifetime rule for their buffers), so
 * the two calls can be mixed on one state.  workspace: DEVICE, 256-byte aligned, at least
 * 32 * (L + 1) bytes rounded up to 256. */
int adacomp_apply_global_staleness(const adacomp_param_layer_t *params, uint32_t L, adacomp_state_t *st,
                                   const adacomp_update_t *updates, uint32_t Q, float lr,
                                   void *workspace, size_t ws_bytes, void *hip_stream);

/* Check an update that did not come from adacomp_select (adacomp_apply skips entries whose
 * index is outside the tensor, but otherwise trusts its input: an index list that is not
 * strictly ascending gives unspecified parameter values).  Enqueues one pass over the
 * indices that leaves in *flags_dev (DEVICE uint32, read it after the stream has drained):
 * 0 = well formed; bit 0: an index >= its tensor's size; bit 1: indices of a tensor not
 * strictly ascending; bit 2: layer_off_dev[L] differs from the host layer_off[L].
 *   n_dev  DEVICE [L] tensor sizes */
int adacomp_update_validate(const adacomp_update_t *update, const uint64_t *n_dev, uint32_t L,
                            uint32_t *flags_dev, void *hip_stream);

/* ---- wire format (not an operation of the paper) -----------------------------------
 * The paper leaves the byte encoding of an update open (footnote of Sec. 4 "Overview")
 * and models traffic as I x M x c (Sec. 3.2), values only.  These two calls turn an
 * update into the stream of little-endian 32-bit words this library would send, and back,
 * so that real bytes per update can be stated.  A block is up to 64 consecutive entries of
 * one tensor; B = sum_l ceil(k_l / 64).
 *
 *   [0] magic 0x31434441  [1] L  [2],[3] total entries (low, high word)
 *   [4 .. 4+L)            k_l
 *   first[B]              index of the first entry of every block
 *   width[B]              one byte per block, zero-padded to a whole word
 *   deltas                block after block: for entries i = 1 .. m-1 of the block
 *                         d_i = idx_i - idx_(i-1) - 1 in width[b] bits each, d_1 first,
 *                         least significant bit first, bit p of the block's stream = bit
 *                         (p mod 32) of its word p / 32, last word zero-padded;
 *                         width[b] = bit length of the block's largest d_i (0 .. 32)
 *   values[total]         fp32 bit patterns in entry order
 *
 * adacomp_wire_bound: *words = the most words a stream for these HOST offsets can take.
 * adacomp_wire_workspace: *bytes of DEVICE workspace either call needs (256-byte aligned). */
int adacomp_wire_bound(const uint64_t *layer_off, uint32_t L, uint64_t *words);
int adacomp_wire_workspace(const uint64_t *layer_off, uint32_t L, size_t *bytes);

/* Encode `update` (as adacomp_select leaves it; totals above 2^32 - 1 entries are refused
 * with ADACOMP_ERR_LAYER_TOO_LARGE) into wire[0 .. wire_cap) (DEVICE, 4-byte aligned).
 * *wire_words_dev (DEVICE uint64, 8-byte aligned) receives the length of the stream; if it
 * exceeds wire_cap the stream is incomplete (nothing is written beyond wire_cap), so size the
 * buffer with adacomp_wire_bound.  Asynchronous on hip_stream; allocates nothing. */
int adacomp_wire_pack(const adacomp_update_t *update, uint32_t *wire, uint64_t wire_cap,
                      uint64_t *wire_words_dev, void *workspace, size_t ws_bytes, void *hip_stream);

/* Decode wire[0 .. wire_words) (DEVICE) into `update`.  The receiver knows what it expects:
 * update->num_layers and the HOST update->layer_off (k_l follows from (n_l, c) alone, Alg. 1)
 * must be filled in by the caller; idx, val (cap >= total) and layer_off_dev are written.
 * The stream is not trusted: no read goes beyond wire_words and no write beyond the expected
 * counts, and *flags_dev (DEVICE uint32, valid once the stream has drained) reports
 * 0 = decoded; bit 0: header differs from what was expected; bit 1: a width above 32;
 * bit 2: stream length inconsistent with its widths; bit 3: an index beyond 2^32 - 1.
 * With a flag set the output arrays hold unspecified values. */
int adacomp_wire_unpack(const uint32_t *wire, uint64_t wire_words, const adacomp_update_t *update,
                        uint32_t *flags_dev, void *workspace, size_t ws_bytes, void *hip_stream);

/* Static, human-readable text for a return code. */
const char *adacomp_strerror(int code);

/* ---- measurement aid (not an operation of the paper) -------------------------------
 * Kernels of the library, for the optional event timing below. */
enum {
    ADACOMP_KERNEL_PUT = 0,        /* small host->device table upload through kernel arguments */
    ADACOMP_KERNEL_FILL,           /* clear histograms                                          */
    ADACOMP_KERNEL_SAMPLE_HIST,    /* select: histogram of a strided sample                     */
    ADACOMP_KERNEL_PICK,           /* select: choose the filter threshold                       */
    ADACOMP_KERNEL_FILTER,         /* select: streaming read + ordered candidate compaction     */
    ADACOMP_KERNEL_FINISH,         /* select: per tensor, threshold and ordered write straight from the
                                      candidate regions; or the check that leaves it to the kernels below */
    ADACOMP_KERNEL_GATHER,         /* select: pack the candidate regions per tensor             */
    ADACOMP_KERNEL_WORK,           /* select: chunk numbering across tensors                    */
    ADACOMP_KERNEL_HIST,           /* select: radix-descent histogram (3 levels)                */
    ADACOMP_KERNEL_RESOLVE,        /* select: radix-descent bin choice (3 levels)               */
    ADACOMP_KERNEL_COUNT_SEG,      /* select: per-segment counts above / at the threshold       */
    ADACOMP_KERNEL_SCAN,           /* select: exclusive scan of the segment counts              */
    ADACOMP_KERNEL_EMIT,           /* select: ordered write of the (index, value) pairs         */
    ADACOMP_KERNEL_IDENTITY,       /* select: k == n copy                                       */
    ADACOMP_KERNEL_HISTORY,        /* apply: staleness accumulated before the call (bisection)  */
    ADACOMP_KERNEL_SNAPSHOT,       /* apply: counter reading at pull time                       */
    ADACOMP_KERNEL_SCATTER_APPLY,  /* apply: eqs. 3-5 scatter, one update                       */
    ADACOMP_KERNEL_BOUNDS,         /* apply: slice of every update per coordinate tile          */
    ADACOMP_KERNEL_SWEEP,          /* apply: eqs. 3-5 for the whole queue, tile by tile         */
    ADACOMP_KERNEL_SWEEP_SLOW,     /* apply: tiles whose touch lists exceed LDS                 */
    ADACOMP_KERNEL_VALIDATE,       /* adacomp_update_validate                                   */
    ADACOMP_KERNEL_WIRE_MEASURE,   /* wire: width and word count of every 64-entry block        */
    ADACOMP_KERNEL_WIRE_SCAN,      /* wire: word offsets of the blocks, header                  */
    ADACOMP_KERNEL_WIRE_WRITE,     /* wire: packed index gaps and values out                    */
    ADACOMP_KERNEL_WIRE_READ,      /* wire: indices and values back                             */
    ADACOMP_KERNEL_SMALL,          /* select: a small tensor start to end in one workgroup      */
    ADACOMP_KERNEL_COUNT
};

/* Start timing every launch of the kernels whose bit (1 << ADACOMP_KERNEL_*) is set in
 * kernel_mask: a HIP event is recorded before and after each such launch on the stream
 * the kernel is enqueued on.  The only process-global state of the library; not
 * thread-safe.  Events are host objects; no device memory is allocated. */
int adacomp_profile_start(uint64_t kernel_mask);

/* Stop timing, wait for the recorded events and report, per kernel id, the summed
 * duration in milliseconds and the number of launches.  total_ms, launches: HOST arrays
 * of ADACOMP_KERNEL_COUNT elements (either may be NULL). */
int adacomp_profile_stop(double *total_ms, uint64_t *launches);

/* Short static name of a kernel id. */
const char *adacomp_kernel_name(int id);

#ifdef __cplusplus
}
#endif
#endif /* ADACOMP_H */
