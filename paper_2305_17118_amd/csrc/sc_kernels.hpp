// Internal interface between the host state machine (sc_host.cpp) and the gfx950 kernels.
// Not part of the public ABI (that is include/sc.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sc {

enum : int { KV_F32 = 0, KV_F16 = 1, KV_I4G64 = 2 };

// Device addresses of one cache inside the caller's workspace.  Every per-unit array has a
// row stride of `C` slots.
struct Layout {
    int U, d, kv_dtype;
    int C;          // slots per unit (multiple of 64)
    int E;          // counter buckets per slot (bucket mode)
    int W32;        // 32-bit ring words per slot (exact ring mode), 0 in bucket mode
    void* K;        // F32/F16: [U][C][d] elements; I4: [U][C][d/2] bytes of codes
    void* V;
    void* K_meta;   // I4 only: [U][C][d/64] x {fp16 scale, fp16 zero}
    void* V_meta;
    int32_t* pos;   // [U][C]
    uint16_t* cnt;  // bucket mode: [U][E][C] uint16; ring mode: the same memory as uint32 [U][W32][C]
    void* Qh;       // record recomputed at compression time: ring of the last w queries [U][w][d], else null
    int w;          // history window in steps
    int32_t* srcmap;  // [U][C] scratch written by select, read by compact
    int32_t* first;   // [U] scratch: first slot whose row moves
    int32_t* ticket;  // one counter, zero between launches: units of a decode launch handed out by ticket
    int split;        // fp32/fp16 decode: workgroups per unit when there are very few units with long caches, else 0
    float* shares;    // [U][8][d + 32] shares of a split step (srcmap doubles as its [U][C] raw scores)
    int32_t* arrive;  // [U] workgroups of a split step that have published, zero between launches
};

// ---- Ragged batches: every sequence runs Alg. 1 on its own clock ----------------------------
// The schedule of a sequence is a function of the number of tokens it has seen: as long as every
// due compression is carried out before the next step, the resident rows, the history bucket (or
// ring bit), the threshold and the steps at which a compression is due all follow from t_b.  The
// device therefore only needs t_b per sequence: a table off[b] = t_b - step that stays valid
// while a sequence takes part in consecutive steps (both sides advance by one per call), and is
// rewritten only when a sequence joins, leaves or is prefilled.
constexpr int32_t kSeqIdle = INT32_MIN;  // table entry of a sequence that does not take part

struct SeqSched {
    const int32_t* off;  // device [batch], or null: all units in lock step (scalar arguments apply)
    int step;            // t_b = off[b] + step is the step being computed (decode) or just computed (compress)
    const int32_t* step_dev;  // decode only: when not null the device keeps the count of completed
                              // steps and t_b = off[b] + *step_dev + 1 (`step` is ignored); a launch
                              // whose arguments do not change from step to step can be replayed
    int heads;           // units per sequence
    int n_trig, m, w;    // trigger size, rows dropped per compression, history window
    int E, W32;          // record layout (buckets, or ring words)
    int thresh_len;      // threshold 1/n instead of 1/t
    int recompute;       // record rebuilt at compression time: steps count nothing, queries are kept
};

struct SeqStep {
    int n;          // resident rows including the one this step appends
    int pos_value;  // stream position of that row
    int bucket;     // counter bucket, or ring word, of this step
    int counted;
    uint32_t ring_bit;
    float tau;
};

// ceil((t - n_trig) / m) for any sign.
__host__ __device__ inline long sched_epoch(long t, long n_trig, long m) {
    const long a = t - n_trig;
    return a >= 0 ? (a + m - 1) / m : -((-a) / m);
}

// Resident rows right after step t (before the compression that may then be due).
__host__ __device__ inline int sched_rows(long t, int n_trig, int m) {
    return t <= n_trig ? (int)t : n_trig - m + (int)((t - n_trig - 1) % m) + 1;
}

// A compression is due right after step t.
__host__ __device__ inline bool sched_due(long t, int n_trig, int m) {
    return t >= n_trig && (t - n_trig) % m == 0;
}

__host__ __device__ inline SeqStep sched_step(const SeqSched& s, long t1) {
    SeqStep r;
    r.n = sched_rows(t1, s.n_trig, s.m);
    r.pos_value = (int)(t1 - 1);
    if (s.recompute) {
        r.bucket = 0;
        r.ring_bit = 0;
        r.counted = 0;
    } else if (s.W32) {
        const long rho = t1 % s.w;  // ring bit owned by this step
        r.bucket = (int)(rho >> 5);
        r.ring_bit = 1u << (rho & 31);
        r.counted = 1;
    } else {
        const long ep = sched_epoch(t1, s.n_trig, s.m);
        r.bucket = (int)(((ep % s.E) + s.E) % s.E);
        r.ring_bit = 0;
        r.counted = ep > -(long)s.E;
    }
    const float x = (float)(s.thresh_len ? (long)r.n : t1);
#if defined(__HIP_DEVICE_COMPILE__)
    r.tau = __fdiv_rn(1.0f, x);
#else
    r.tau = 1.0f / x;
#endif
    return r;
}

// Write `count` table entries (host values) to device memory on `stream`.
hipError_t launch_write_seq_table(int32_t* dst, const int32_t* host_values, int count, hipStream_t stream);

// *counters[i] += 1 for i < count on `stream` (the device-side step counts of ragged batches; one
// launch serves up to 64 caches).
hipError_t launch_tick(int32_t* const* counters, int count, hipStream_t stream);

struct StepArgs {
    const void* q;
    const void* k_new;
    const void* v_new;
    long in_stride;   // elements between units in q/k_new/v_new
    void* out;        // [U][d]
    long out_stride;  // elements between units in out
    float* probs;     // unit 0's row of C floats, or null
    long probs_stride;  // floats between units in probs
    int n;            // resident rows including the one appended by this step
    int pos_value;    // stream position of the appended row (t-1)
    int bucket;       // counter bucket this step increments (ring mode: ring word of this step)
    int counted;      // 0: this step falls outside every history window, do not count
    uint32_t ring_bit;  // ring mode: mask of this step's bit inside its word
    float qk_log2;    // score scale * log2(e)
    float tau;        // low-score threshold
    void* q_keep;     // ring slot of this step for unit 0 (units are w*d elements apart), or null
    SeqSched seq{};   // seq.off != null: n, pos_value, bucket, counted, ring_bit and tau above are
                      // ignored and derived per sequence on the device
    unsigned long long* trace = nullptr;  // diagnostics: [U][4] clock readings per workgroup, or null
};

// One launch on `stream`: append the new row and attend.
hipError_t launch_decode_step(const Layout& L, const StepArgs& a, hipStream_t stream);

struct CompressArgs {
    int n;          // resident rows before compression (== trigger size)
    int r, m;       // recent window, rows to drop
    int zero_bucket;  // bucket the following epoch will count into (cleared here)
    int32_t* evicted; // [U][m] or null
    SeqSched seq{};   // seq.off != null: only the units of sequences that are due after step
                      // off[b] + step are compressed (n is the trigger size for all of them),
                      // zero_bucket is derived per sequence
};

hipError_t launch_compress(const Layout& L, const CompressArgs& a, hipStream_t stream);

// Scratch for select -> compact that belongs to the library instead of the caller's workspace: a
// file-scope device array of kStaticScratchBytes, one copy per device.  Returns its address on
// the current device (looked up with hipGetSymbolAddress the first time a device asks, kept
// afterwards); allocates nothing.
constexpr size_t kStaticScratchBytes = 32u << 20;
hipError_t static_scratch(void** ptr);

// A run of `c` consecutive prompt positions with no compression inside and a single counter
// bucket (the host cuts the prompt accordingly), processed as one dense causal block.
struct ChunkArgs {
    const void* q;    // first prompt row of the run, unit 0
    const void* k;
    const void* v;
    long unit_stride;      // elements between units in q, k and v
    void* out;             // first output row of the run, unit 0, or null; rows are d apart
    long out_unit_stride;  // elements between units in out
    float* probs;          // row of the run's first position, unit 0, or null; rows are C apart
    long probs_unit_stride;  // floats between units in probs
    int n0;           // resident rows before the run
    int c;            // positions in the run; n0 + c <= trigger size
    long t0;          // tokens seen before the run
    int bucket;       // counter bucket every position of the run increments
    int counted;      // 0: the run falls outside every history window
    int thresh_len;   // threshold 1/n (1) or 1/t (0)
    float qk_log2;
};

// Whether launch_prefill_chunk handles such a cache: every storage type and head size it does
// (fp32, fp16, 4-bit; 64 or 128 channels; bucket counters, the one-bit-per-step ring, or the
// record rebuilt at compression time); what limits it is the per-slot LDS array that has to fit
// beside the tiles.
inline bool prefill_chunk_supported(int kv_dtype, int d, int E, int W32, int C) {
    if (C > 6144) return false;
    (void)kv_dtype;
    (void)d;
    return E > 0 || W32 > 0;
}

// Two launches on `stream`: append the run's rows, then attention + counting.
hipError_t launch_prefill_chunk(const Layout& L, const ChunkArgs& a, hipStream_t stream);

// Keep the queries of `count` consecutive steps, the first being step t0+1, in the ring
// L.Qh (step i goes to slot (i-1) mod w).  q points at the first of them for unit 0; rows
// are d elements apart, units unit_stride elements.
hipError_t launch_store_queries(const Layout& L, const void* q, long unit_stride, int count, long t0,
                                hipStream_t stream);

// Alg. 2 as printed: rebuild the record (16-bit counts in L.cnt, cleared first) by replaying
// the kept queries of steps (t - min(w,t), t] over the n resident rows.
struct ReplayArgs {
    long probs_unit_stride;  // floats between units in probs (0: min(w, t) * C, densely packed)
    int n;
    long t;
    int thresh_len;
    float qk_log2;
    float* probs;  // [U][min(w,t)][C] or null
};
hipError_t launch_recompute_record(const Layout& L, const ReplayArgs& a, hipStream_t stream);

// Diagnostics (diag.hip): pivotal-token counts behind the persistence ratio of Sec. 3.1, and the
// full-attention mass held by the resident rows.
hipError_t launch_persistence(const float* probs, int units, int length, long row_stride, long unit_stride,
                              int split, int32_t* counts, hipStream_t stream);
// Pure read of `bytes` (a multiple of 32 MiB) from buf with 16-byte loads, 1024 workgroups.
hipError_t launch_read_stream(const void* buf, size_t bytes, bool nontemporal, uint32_t* sink, hipStream_t stream);
hipError_t launch_kept_mass(const Layout& L, int n, const float* full, long unit_stride, float* mass,
                            hipStream_t stream);

// Zero all counters (cache creation).
hipError_t launch_clear_counters(const Layout& L, hipStream_t stream);

}  // namespace sc
