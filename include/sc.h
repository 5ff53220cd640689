/*
 * sc.h — C ABI of the budgeted KV cache for autoregressive decoding on MI355X (gfx950).
 *
 * The library implements the per-step hot path of Scissorhands (arxiv 2305.17118):
 *   - Alg. 1 (inference with a budget KV cache): every step appends one key/value row per
 *     (sequence, head) unit; when the cache reaches its trigger size it must be compressed.
 *   - Sec. 4.1 estimator: attention of one query over the n resident rows only.
 *   - Alg. 2 (compress): importance record I = number of steps inside the history window
 *     at which a row's attention probability was below 1/t, kept online during generation
 *     as Sec. 4.1 "Overhead Tradeoff" allows; the r most recent rows are protected; the m
 *     rows with the largest record are dropped; survivors are compacted, n <- n - m.
 *
 * General conventions
 *   Units.     A unit is one (sequence, head) pair; U = batch*heads.  By default all units
 *              advance in lock step; with the *_ragged calls every sequence has its own
 *              counters.  Either way the counters t (tokens seen) and n (resident rows) are
 *              host integers and no call ever reads device memory back.
 *   Memory.    Every pointer marked "device" is device memory owned by the caller and must
 *              stay valid until the work enqueued by the call has run.  The library never
 *              allocates or frees device memory; the cache lives in a caller-provided
 *              workspace (256-byte aligned, sc_workspace_bytes() long) that must outlive
 *              the handle.  The handle owns host metadata only.
 *   Streams.   `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *              Calls only enqueue kernels on it and never synchronise.  The work of two calls
 *              on one handle must not overlap on the device (the workspace holds scratch and
 *              counters that a launch expects to find as the previous one left them): use one
 *              stream per handle, or order the streams.
 *   Errors.    Functions return sc_status; nothing throws, aborts or prints.  Every argument
 *              and state check is made before anything is enqueued or changed: on
 *              SC_ERR_INVALID_ARG, _WORKSPACE, _FULL, _STATE, _UNSUPPORTED, _SCRATCH and
 *              _HOST_MEMORY the cache (t, n, device contents) is unchanged and out-params are
 *              untouched.  SC_ERR_DEVICE (a launch was refused by the runtime) can arrive in
 *              the middle of a call that enqueues several launches (sc_prefill and its ragged
 *              form, sc_compress with the record rebuilt first, the ragged step after its
 *              table upload): the cache is then in no defined state and must be put back to
 *              empty with sc_cache_reset before it is used again.
 *   Threads.   A handle is not thread-safe; distinct handles are independent.
 *   Element types.  SC_KV_F32: q/k/v/out are float.  SC_KV_F16 and SC_KV_I4G64: q/k/v/out
 *              are IEEE binary16.  All dot products, the softmax and the weighted value sum
 *              accumulate in fp32; `out` is rounded to nearest-even on store.
 */
#ifndef SC_H_
#define SC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sc_cache sc_cache; /* opaque, host side */

typedef enum {
    SC_OK = 0,
    SC_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, m > trigger size - r, ...    */
    SC_ERR_WORKSPACE = 2,   /* workspace too small or not 256-byte aligned                    */
    SC_ERR_FULL = 3,        /* sc_decode_step while a compression is due                      */
    SC_ERR_STATE = 4,       /* sc_compress when none is due; lock-step call on a ragged handle */
    SC_ERR_UNSUPPORTED = 5, /* head_dim / kv_dtype / sizes this build does not cover          */
    SC_ERR_DEVICE = 6,      /* a kernel launch failed (hipGetLastError)                       */
    SC_ERR_SCRATCH = 7,     /* sc_compress_static: the cache needs more scratch than the
                               library's static array holds (SC_STATIC_SCRATCH_BYTES)          */
    SC_ERR_HOST_MEMORY = 8  /* host memory for the handle's own bookkeeping could not be had  */
} sc_status;

/* Storage format of the cached K/V rows. */
typedef enum {
    SC_KV_F32 = 0,  /* fp32 rows                                                              */
    SC_KV_F16 = 1,  /* fp16 rows                                                              */
    SC_KV_I4G64 = 2 /* 4-bit codes, asymmetric, one (scale, zero) fp16 pair per 64 channels   */
} sc_kv_dtype;

/* When Alg. 1 compresses.  Alg. 1 says "if n > B ... such that n <= B" and Alg. 2 removes
 * exactly m rows, so the literal reading leaves B+1-m rows; Sec. 4.2 states the cache holds
 * exactly B rows for m = 1.  Both readings are offered. */
typedef enum {
    SC_TRIGGER_HARD_CAP = 0,  /* compress when n == B+1; afterwards n == B+1-m (<= B)         */
    SC_TRIGGER_HIGH_WATER = 1 /* compress when n == B+m; afterwards n == B exactly            */
} sc_trigger;

/* Threshold below which a probability counts as "low" (Alg. 2 uses 1/t; Sec. 3.1 motivates
 * it as the average score). */
typedef enum {
    SC_THRESH_INV_POS = 0, /* 1/t, t = tokens seen so far including the current one (paper)   */
    SC_THRESH_INV_LEN = 1  /* 1/n, n = resident rows (the true average over a compacted cache)*/
} sc_thresh;

/* How the importance record of Alg. 2 (low-score counts over the last w steps) is stored.
 * Both reproduce the history window exactly at every compression; they differ in cost. */
typedef enum {
    SC_WINDOW_AUTO = 0,   /* buckets when w is a multiple of m, else the exact ring           */
    SC_WINDOW_RING = 1    /* one bit per (row, step) in a ring of w bits: any w, w/8 bytes/row */
} sc_window;

/* When the importance record of Alg. 2 is collected.  Sec. 4.1 ("Overhead Tradeoff") names
 * both: Alg. 2 as printed spends "an extra attention computation" at the compression step,
 * or a little memory keeps the record up to date during the generation steps. */
typedef enum {
    SC_RECORD_ONLINE = 0,    /* counted at every step from that step's own probabilities        */
    SC_RECORD_RECOMPUTE = 1  /* the last w queries are kept; at a compression each is replayed
                                over the rows resident then that its step could see (stream
                                position <= its own), softmax over exactly those rows, low =
                                below that step's threshold                                     */
} sc_record;

/* Problem statement of Def. 4.1 / inputs of Alg. 1 and Alg. 2. */
typedef struct {
    int32_t batch, heads; /* U = batch*heads independent units                               */
    int32_t head_dim;     /* d in {64, 128}                                                  */
    int32_t kv_dtype;     /* sc_kv_dtype                                                     */
    int32_t budget;       /* B: token budget per unit (Alg. 1)                               */
    int32_t recent;       /* r: most recent rows never evicted (Alg. 2), r >= 1              */
    int32_t history;      /* w: history window in steps (Alg. 2), 1 <= w <= 8192             */
    int32_t drop;         /* m: rows dropped per compression (Alg. 2), 1 <= m <= n_trig - r  */
    int32_t trigger;      /* sc_trigger                                                      */
    int32_t thresh_mode;  /* sc_thresh                                                       */
    int32_t window_mode;  /* sc_window                                                       */
    int32_t record_mode;  /* sc_record                                                       */
    float scale;          /* score scale; 0 selects 1/sqrt(head_dim)                         */
} sc_config;

/* Derived sizes of a configuration (host only, no GPU needed).
 *   n_trig   : number of resident rows at which a compression becomes due
 *   capacity : row stride of every per-unit array (n_trig rounded up to a multiple of 64);
 *              also the leading dimension of probs_out
 *   buckets  : E = w/m 16-bit counter buckets kept per row (0 when the exact ring is used;
 *              1 with SC_RECORD_RECOMPUTE: the record itself, rebuilt at every compression)
 *   ring_words : ceil(w/32) 32-bit ring words kept per row (0 when buckets are used)
 * Returns SC_ERR_INVALID_ARG for an inconsistent configuration (m > n_trig - r, sizes < 1,
 * unknown enum values, more than 2^24 units) and SC_ERR_UNSUPPORTED for one outside what the
 * kernels cover: head_dim other than 64 or 128, w > 8192, n_trig > 12288 (a unit's scores are
 * held in LDS during a step), capacity > 6144 with SC_RECORD_RECOMPUTE (the replay's LDS). */
sc_status sc_config_sizes(const sc_config *cfg, int32_t *n_trig, int32_t *capacity, int32_t *buckets,
                          int32_t *ring_words);

/* Bytes of device workspace a cache of this configuration needs; 0 if cfg is invalid. */
size_t sc_workspace_bytes(const sc_config *cfg);

/* Where step number t (1-based count of tokens seen) falls in the counter schedule (host
 * only).  Compressions happen at t = n_trig + k*m; `epoch` is the k of the next compression
 * at or after t (may be negative), `bucket` = epoch mod E the counter bucket that step t
 * increments, `counted` = 0 for steps so early that they have left every history window
 * before the first compression.  The union of the E buckets at a compression step is
 * exactly the history window (t-w, t] of Alg. 2.  With the exact ring every step is counted,
 * step t owns ring bit t mod w, and `bucket` is the index (t mod w)/32 of the word holding it. */
sc_status sc_schedule(const sc_config *cfg, int64_t t, int64_t *epoch, int32_t *bucket, int32_t *counted);

/* Create an empty cache (n = 0, t = 0) inside dev_workspace (device, 256-byte aligned,
 * `bytes` >= sc_workspace_bytes(cfg)).  Enqueues a clear of the counters on `stream`. */
sc_status sc_cache_create(const sc_config *cfg, void *dev_workspace, size_t bytes, void *stream,
                          sc_cache **out);

/* Back to the empty state (n = 0, t = 0) for a new batch of sequences in the same workspace:
 * the Alg. 1 loop starts over.  Enqueues a clear of the counters on `stream`; K, V and
 * positions need none (only slots below n are ever read). */
sc_status sc_cache_reset(sc_cache *c, void *stream);

/* Free the host metadata.  The workspace is the caller's. */
void sc_cache_destroy(sc_cache *c);

/* One decode step (Alg. 1 loop body + Sec. 4.1 estimator + one update of the Alg. 2 record):
 * append k_new/v_new as row n of every unit, attend q over the n+1 resident rows, add one
 * to the record of every row whose probability is below the threshold, n <- n+1, t <- t+1.
 *   q, k_new, v_new : device, U rows of head_dim elements; consecutive units are `in_stride`
 *                     elements apart (0 = densely packed [batch, heads, head_dim])
 *   out             : device, dense [batch, heads, head_dim]
 *   probs_out       : device fp32 [U][capacity] or NULL, 8-byte aligned (probabilities are
 *                     stored in pairs); receives, for slots < n, exactly the probabilities the
 *                     threshold test was applied to (slot n is written as 0 when n is odd,
 *                     other slots >= n are untouched)
 * q, k_new, v_new and out must be 16-byte aligned, in_stride a multiple of 16 bytes.
 *   compress_due    : host int or NULL; set to 1 when n has reached n_trig, i.e. the caller
 *                     must call sc_compress before the next step, else 0
 * SC_ERR_FULL if a compression is due. */
sc_status sc_decode_step(sc_cache *c, const void *q, const void *k_new, const void *v_new,
                         int64_t in_stride, void *out, float *probs_out, int32_t *compress_due,
                         void *stream);

/* Alg. 2 on every unit: select the m candidates (slots < n - r) with the largest record,
 * equal records lowest slot first; compact K, V, positions and counters in place keeping
 * order; n <- n - m.
 *   evicted_out : device int32 [U][m] or NULL; the dropped slots (numbering before
 *                 compaction) of each unit in ascending order
 *   probs_out   : SC_RECORD_RECOMPUTE only (ignored otherwise), device fp32
 *                 [U][min(w, t)][capacity] or NULL: row k receives, for the rows that replayed
 *                 step t - min(w, t) + 1 + k sees, exactly the probabilities its threshold
 *                 test was applied to; other elements are untouched
 * SC_ERR_STATE unless the previous step reported compress_due. */
sc_status sc_compress(sc_cache *c, int32_t *evicted_out, float *probs_out, void *stream);

/* sc_compress for callers that can neither allocate device memory nor hand over scratch of
 * their own: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same result, same kernels as sc_compress; the only difference is
 * where the hand-over between selection and compaction lives (per unit: the source slot of
 * every surviving row and the first slot that moves).  sc_compress keeps it in the caller's
 * workspace; this call keeps it in a file-scope device array of SC_STATIC_SCRATCH_BYTES that is
 * part of the library's code object (every GPU the library runs on holds its own copy until
 * the process ends).  The call allocates and frees nothing, on the host or on the device.
 *   Limit.    256*ceil(4*U/256) + 4*U*capacity bytes must fit in SC_STATIC_SCRATCH_BYTES
 *             (cfg4's 9216 units x 704 slots need 24.8 MiB); otherwise SC_ERR_SCRATCH and
 *             nothing is enqueued or changed.
 *   Sharing.  Every call on a GPU uses that GPU's one array, on whatever cache: two calls that
 *             may run at the same time on one GPU (different streams, or graphs replayed
 *             concurrently) race.  Calls ordered on one stream are safe.  Nothing in the array
 *             has to start at zero: selection writes every element compaction reads.
 *   Device.   The array is looked up on the device that is current (hipGetDevice) when the
 *             call is made; that must be the device of `stream` and of the cache.
 * SC_ERR_STATE unless the previous step reported compress_due, or on a ragged handle. */
#define SC_STATIC_SCRATCH_BYTES (32u << 20)
sc_status sc_compress_static(sc_cache *c, int32_t *evicted_out, float *probs_out, void *stream);

/* How sc_prefill computes.  The result is the same function of the inputs either way; the
 * floating-point rounding differs (summation order, fp16 probabilities in P.V). */
typedef enum {
    SC_PREFILL_AUTO = 0,     /* dense causal blocks on the matrix cores where supported (runs of
                                >= 16 positions, capacity <= 6144 slots), else streamed           */
    SC_PREFILL_STREAMED = 1  /* one decode step per position: bit-identical to calling
                                sc_decode_step / sc_compress in a loop                            */
} sc_prefill_mode;

/* Stream a prompt through Alg. 1 (Def. 4.1 treats prompt and generated tokens as one
 * stream): for each of the prompt_len positions in order, one decode step, then a
 * compression whenever one is due.  The cache need not be empty: the positions continue its
 * stream from wherever it stands (a prompt handed over in chunks, a later turn of a
 * conversation); SC_ERR_FULL if a compression is due.  Between two compressions the
 * cache only grows, so the positions in between form one dense causal attention block
 * (Sec. 4.1 estimator per position, Alg. 2 record update per position); SC_PREFILL_AUTO
 * computes them that way.
 *   q, k, v   : device, [U][>= prompt_len][head_dim]; consecutive units are `unit_stride`
 *               elements apart (0 = prompt_len*head_dim)
 *   out       : device dense [U][prompt_len][head_dim], or NULL to discard the outputs
 *   probs_out : device fp32 [U][prompt_len][capacity] or NULL; row i receives, for the slots
 *               resident at position i (numbering at that step), exactly the probabilities
 *               the threshold test was applied to; other elements are untouched (a slot just
 *               past the resident ones may be written as 0)
 *   mode      : sc_prefill_mode */
sc_status sc_prefill(sc_cache *c, const void *q, const void *k, const void *v, int32_t prompt_len,
                     int64_t unit_stride, void *out, float *probs_out, int32_t mode, void *stream);

/* The runs sc_prefill cuts a prompt into (host only, no GPU needed): consecutive positions
 * that share one counter bucket with no compression in between.  Entry i of the output
 * arrays (any may be NULL; at most max_runs entries are written) describes run i:
 *   run_len      : positions in the run
 *   run_dense    : 1 if computed as one dense causal block, 0 if streamed step by step
 *   run_compress : 1 if a compression (Alg. 2) follows the run
 * *n_runs receives the total number of runs, which may exceed max_runs. */
sc_status sc_prefill_plan(const sc_config *cfg, int32_t prompt_len, int32_t mode, int32_t max_runs,
                          int32_t *run_len, int32_t *run_dense, int32_t *run_compress, int32_t *n_runs);

/* Resident rows n and tokens seen t (either pointer may be NULL).  SC_ERR_STATE once the handle
 * keeps per-sequence counters (see sc_cache_len_seq). */
sc_status sc_cache_len(const sc_cache *c, int32_t *n, int64_t *t);

/* ---- Ragged batches -------------------------------------------------------------------------
 * Alg. 1 keeps its counters per sequence: prompts of different lengths, or sequences that stop
 * generating at different steps, give every sequence b its own t_b and n_b, hence its own
 * threshold 1/t_b (Alg. 2), its own place in the history window and its own steps at which a
 * compression is due.  The three calls below run the same kernels with those quantities taken
 * per sequence (a device table of one integer per sequence, rewritten only when a sequence
 * joins, leaves or is prefilled); all sequences of a call still share one launch.
 * The first *_ragged call switches the handle to per-sequence counters (SC_ERR_FULL if a
 * lock-step compression is still due); from then on the lock-step calls (sc_decode_step,
 * sc_compress, sc_prefill, sc_cache_len, sc_diag_kept_mass) return SC_ERR_STATE until
 * sc_cache_reset. */

/* Empty the cache of sequence b alone (n_b = 0, t_b = 0) so that a new request can take its
 * place in the batch while the other sequences go on (the Alg. 1 loop of that sequence starts
 * over; a compression it had pending is dropped with it).  Enqueues a clear of that
 * sequence's counters on `stream`.  Switches the handle to per-sequence counters like the
 * other ragged calls. */
sc_status sc_cache_reset_seq(sc_cache *c, int32_t b, void *stream);

/* Host only: the resident rows of a sequence right after its step t (t >= 1, counting the row
 * that step appended, before the compression that may then be due) and whether a compression is
 * due after it, given that every due compression was carried out (Alg. 1).  This closed form is
 * what the kernels evaluate per sequence for ragged batches.  Either pointer may be NULL. */
sc_status sc_schedule_rows(const sc_config *cfg, int64_t t, int32_t *rows, int32_t *due);

/* Prompts of different lengths: sequence b streams its first prompt_len[b] positions through
 * Alg. 1 exactly as sc_prefill does for a whole batch (consecutive sequences of equal length
 * share their launches when their counters are equal too).  Sequences with prompt_len[b] == 0
 * are left alone; the others continue from wherever they stand (SC_ERR_FULL if one of them has
 * a compression due).
 *   prompt_len : host int32 [batch]
 *   q, k, v    : device, [U][>= max prompt_len][head_dim], units `unit_stride` elements apart
 *                (0 = max prompt_len * head_dim)
 *   out        : device dense [U][max prompt_len][head_dim] or NULL; rows past a sequence's
 *                prompt are untouched
 *   probs_out  : device fp32 [U][max prompt_len][capacity] or NULL, rows as in sc_prefill */
sc_status sc_prefill_ragged(sc_cache *c, const void *q, const void *k, const void *v,
                            const int32_t *prompt_len, int64_t unit_stride, void *out, float *probs_out,
                            int32_t mode, void *stream);

/* One decode step of the sequences with active[b] != 0 (all when active is NULL; at least one),
 * each at its own t_b and n_b; arguments as in sc_decode_step.  Units of idle sequences are
 * neither read nor written (q/k_new/v_new/out/probs_out rows included).
 *   active : host uint8 [batch] or NULL
 *   n_due  : host int or NULL; receives the number of sequences whose cache has reached its
 *            trigger size: when it is not 0 the caller must call sc_compress_ragged before the
 *            next step
 * SC_ERR_FULL if a compression is due for any sequence. */
sc_status sc_decode_step_ragged(sc_cache *c, const void *q, const void *k_new, const void *v_new,
                                int64_t in_stride, void *out, float *probs_out, const uint8_t *active,
                                int32_t *n_due, void *stream);

/* Replaying a decode step (HIP graphs).  By default the step count travels to the kernels as an
 * argument, so the work a call enqueues is only valid once.  With the device clock enabled the
 * count lives in the workspace: sc_decode_step_ragged then enqueues the attention launch, whose
 * arguments no longer change from step to step, followed by a one-thread launch that advances
 * the count.  That pair can be captured in a graph and replayed for as long as the same
 * sequences take part and no compression becomes due, across compressions and prompts handled
 * by eager calls in between (the caller rewrites q, k_new, v_new in place before each replay):
 *   1. make one eager call with the active set to be captured (it brings the device table up
 *      to date, so the captured call contains no table write);
 *   2. capture one sc_decode_step_ragged call: the handle counts it as a step although nothing
 *      runs; the first replay executes it;
 *   3. after every further replay call sc_cache_note_replays(c, 1, ...) (or once with k for k
 *      replays) so that the host counters follow; sc_steps_until_due says how many steps may
 *      be taken before a compression (SC_ERR_FULL from sc_cache_note_replays beyond that).
 * Enabling or disabling switches the handle to per-sequence counters like the other ragged calls. */
sc_status sc_cache_device_clock(sc_cache *c, int32_t enable);

/* Steps the sequences with active[b] != 0 (all when NULL) can still take before one of them
 * reaches its trigger size (0: a compression is due now).  Host only. */
sc_status sc_steps_until_due(const sc_cache *c, const uint8_t *active, int32_t *steps);

/* The work enqueued by the most recent sc_decode_step_ragged call has been executed k more
 * times (graph replays): advance the counters of the sequences that took part in it.
 *   n_due : host int or NULL; number of sequences now due
 * SC_ERR_STATE without the device clock or before any ragged decode step; SC_ERR_FULL (nothing
 * changed) if k steps would pass a due compression. */
sc_status sc_cache_note_replays(sc_cache *c, int32_t k, int32_t *n_due);

/* Alg. 2 on the units of every sequence that is due (one launch pair for all of them; with
 * SC_RECORD_RECOMPUTE preceded by one replay of the kept queries per range of due sequences
 * with equal token counts).
 *   evicted_out : device int32 [U][m] or NULL; rows of sequences that were not due are untouched
 *   probs_out   : SC_RECORD_RECOMPUTE only (ignored otherwise), device fp32 [U][w][capacity] or
 *                 NULL: for the units of a due sequence b, row k < min(w, t_b) receives the
 *                 probabilities of replayed step t_b - min(w, t_b) + 1 + k as in sc_compress
 * SC_ERR_STATE when no sequence is due. */
sc_status sc_compress_ragged(sc_cache *c, int32_t *evicted_out, float *probs_out, void *stream);

/* Resident rows and tokens seen of sequence b (works for lock-step handles too). */
sc_status sc_cache_len_seq(const sc_cache *c, int32_t b, int32_t *n, int64_t *t);

/* ---- One cache per transformer layer, each with its own budget ------------------------------
 * Sec. 4.1 "Allocating Budgets Across Attention Heads": a total budget is distributed over the
 * layers (more to later layers, whose persistence ratio is lower) and evenly over the heads of
 * a layer.  A layer set is L caches that share every parameter of `cfg` except the per-layer
 * budget B_l and rows dropped per compression m_l (the paper ties m to B, m = B/2), carved out
 * of one caller-provided workspace.  Each layer is an ordinary sc_cache: the handle returned by
 * sc_layers_get is used with every call above (lock step or ragged) and is owned by the set. */
typedef struct sc_layers sc_layers; /* opaque, host side */

/* Bytes of 256-byte aligned device workspace for the whole set; 0 if any layer's configuration
 * is invalid.  budgets: host int32 [layers]; drops: host int32 [layers] or NULL (cfg->drop). */
size_t sc_layers_workspace_bytes(const sc_config *cfg, int32_t layers, const int32_t *budgets,
                                 const int32_t *drops);

/* Create the L empty caches.  Errors as sc_cache_create (the first failing layer's status). */
sc_status sc_layers_create(const sc_config *cfg, int32_t layers, const int32_t *budgets,
                           const int32_t *drops, void *dev_workspace, size_t bytes, void *stream,
                           sc_layers **out);

/* The cache of one layer (NULL when out of range).  Owned by the set: do not destroy it. */
sc_cache *sc_layers_get(sc_layers *ls, int32_t layer);

/* Number of layers. */
int32_t sc_layers_count(const sc_layers *ls);

/* One decode step of every layer in ONE call: layer l runs sc_decode_step_ragged on its own
 * cache with its own inputs and outputs (a model's layers step one after another on one stream;
 * the launches are independent, the set only spares the caller L round trips through the ABI
 * and gives a HIP graph one call to capture).
 *   q, k_new, v_new  : device; layer l's rows start layer_stride elements after layer l-1's
 *                      (>= U*head_dim, or (U-1)*in_stride + head_dim with in_stride != 0), inside a
 *                      layer units are in_stride elements apart (0 = densely packed)
 *   out              : device; layer l's dense [U][head_dim] block starts out_layer_stride elements
 *                      after layer l-1's
 *   active           : host uint8 [batch] or NULL (all), the same sequences in every layer
 *   n_due            : host int or NULL; receives the number of (layer, sequence) pairs whose
 *                      cache has reached its trigger size; when not 0 call sc_layers_compress
 * SC_ERR_FULL, with nothing enqueued or changed, if a compression is due in any layer.  A device
 * error in layer l leaves layers < l one step ahead of the others.
 * Replaying it from a HIP graph works exactly as for one cache (sc_cache_device_clock):
 * sc_layers_device_clock(1), one eager call, capture one call, then per replay
 * sc_layers_note_replays(ls, 1, ...); sc_layers_steps_until_due says how far the graph may run
 * (layers with different budgets become due at different steps; compress eagerly, then go on
 * replaying the same graph). */
sc_status sc_layers_decode_step(sc_layers *ls, const void *q, const void *k_new, const void *v_new,
                                int64_t layer_stride, int64_t in_stride, void *out,
                                int64_t out_layer_stride, const uint8_t *active, int32_t *n_due,
                                void *stream);

/* sc_cache_device_clock for every layer of the set. */
sc_status sc_layers_device_clock(sc_layers *ls, int32_t enable);

/* sc_cache_note_replays for every layer: the work enqueued by the most recent
 * sc_layers_decode_step has been executed k more times.  SC_ERR_FULL (nothing changed) if k steps
 * would pass a due compression in any layer. */
sc_status sc_layers_note_replays(sc_layers *ls, int32_t k, int32_t *n_due);

/* The smallest sc_steps_until_due over the layers. */
sc_status sc_layers_steps_until_due(const sc_layers *ls, const uint8_t *active, int32_t *steps);

/* Alg. 2 on every layer in which a compression is due (sc_compress / sc_compress_ragged as the
 * layer's handle requires, no outputs).  n_compressed: host int or NULL, the number of layers
 * compressed.  SC_ERR_STATE when no layer is due. */
sc_status sc_layers_compress(sc_layers *ls, int32_t *n_compressed, void *stream);

/* Free the host metadata of the set and of its caches. */
void sc_layers_destroy(sc_layers *ls);

/* Device pointers into the workspace, for inspection (any pointer may be NULL):
 *   K, V    : [U][capacity] rows; F32/F16: head_dim elements; I4G64: head_dim/2 bytes of
 *             codes, channel 2i in the low nibble of byte i
 *   K_meta, V_meta : I4G64 only (else NULL): [U][capacity][head_dim/64] pairs of fp16
 *             (scale, zero); value = code*scale + zero
 *   pos     : int32 [U][capacity], 0-based position in the stream of the row in each slot
 *   cnt     : buckets: uint16 [U][buckets][capacity], a row's record I is the sum over buckets;
 *             exact ring: the same pointer addresses uint32 [U][ring_words][capacity], bit
 *             (s mod w) of a row's ring is the low-score flag of step s, I is the popcount */
sc_status sc_cache_view(const sc_cache *c, const void **K, const void **V, const void **K_meta,
                        const void **V_meta, const int32_t **pos, const uint16_t **cnt,
                        int32_t *capacity, int32_t *buckets);

/* Diagnostic of Sec. 3.1 ("Verification"): the pivotal-token sets behind the persistence
 * ratio, from full-attention probabilities (e.g. sc_prefill's probs_out of a cache whose budget
 * is at least the length, so that slot j holds token j).  A token j is pivotal for position i
 * (0-based; t = i+1 tokens seen) when probs[i][j] > 1/t.  With S_first the tokens j < split
 * pivotal for some position i < split and S_later those pivotal for some i >= split,
 *   counts_out[u] = { |S_first|, |S_later|, |S_first ^ S_later| },
 * so the persistence ratio is counts[2]/counts[1] and |S_first|/split the size the paper
 * reports beside it (the paper uses split = length/2).
 *   probs      : device fp32; row i of unit u starts at probs + u*unit_stride + i*row_stride
 *                and holds at least i+1 probabilities
 *   counts_out : device int32 [units][3] */
sc_status sc_diag_persistence(const float *probs, int32_t units, int32_t length, int64_t row_stride,
                              int64_t unit_stride, int32_t split, int32_t *counts_out, void *stream);

/* Diagnostic behind the attention-score change ratio of Sec. 5: the share of one step's
 * full attention that falls on the rows the budgeted cache still holds,
 *   mass_out[u] = sum over resident slots j of probs_full[u][pos[u][j]].
 * By the restricted-softmax identity (proof of Lemma A.4) every surviving token's budgeted
 * score is its full score divided by this mass, so the change ratio (a_s - a_o)/a_o is
 * 1/mass - 1 for every survivor and -1 for every evicted token.
 *   probs_full : device fp32, unit u's full-attention probabilities by stream position start
 *                at probs_full + u*unit_stride (at least t entries)
 *   mass_out   : device fp32 [U] */
sc_status sc_diag_kept_mass(const sc_cache *c, const float *probs_full, int64_t unit_stride,
                            float *mass_out, void *stream);

/* Reference point for the roofline fractions: one launch that reads `bytes` of device memory and
 * does nothing else (16-byte loads, eight in flight per thread, 1024 workgroups of 256 threads,
 * each on its own contiguous share).  Timing it (HIP events, rocprofv3) gives the read bandwidth
 * this chip reaches in practice, which the decode kernels, bound by the same reads (Sec. 4.1's
 * estimator touches every resident row once per step), cannot exceed.
 *   buf         : device, 16-byte aligned, at least `bytes` long; bytes a multiple of 32 MiB
 *   nontemporal : non-zero = streaming loads (as the decode kernels use), 0 = plain loads
 *   sink        : device uint32, written only if the folded data equals a fixed constant (it
 *                 keeps the loads alive; in practice it stays untouched)
 * SC_ERR_INVALID_ARG for null or misaligned pointers or a size that is no multiple of 32 MiB. */
sc_status sc_diag_read_bandwidth(const void *buf, size_t bytes, int32_t nontemporal, uint32_t *sink,
                                 void *stream);

/* Diagnostic of the decode-attention launch itself (where the time of a step goes): while a
 * buffer is set, every workgroup of the launches made by sc_decode_step / sc_decode_step_ragged
 * (one workgroup per unit; units of idle sequences write nothing) records
 *   trace_out[u] = { clock at its start, clock when its K/V stream ended, clock at its end,
 *                    where it ran: low word (XCD << 6) | (shader engine << 4) | CU, high word
 *                    the wave's raw hardware-id register (wave slot, SIMD, ...) }
 * with `clock` the GPU's constant-rate counter (100 MHz, shared by all workgroups).  Each launch
 * overwrites the previous one's readings; results of the step are not affected.
 *   trace_out : device uint64 [U][4], 8-byte aligned; NULL switches the recording off
 * SC_ERR_UNSUPPORTED for a cache whose decode step shares a unit among several workgroups (at most
 * 64 units of fp32/fp16 rows with a capacity of 512 slots or more). */
sc_status sc_diag_trace(sc_cache *c, uint64_t *trace_out);

/* Static description of a status code. */
const char *sc_status_str(sc_status s);

#ifdef __cplusplus
}
#endif
#endif /* SC_H_ */
