// Host side of the C ABI declared in include/sc.h: configuration checks, workspace carving,
// and the lock-step state machine of Alg. 1 (t tokens seen, n resident rows, when a
// compression is due, which counter bucket a step increments).  All device work is enqueued
// through sc_kernels.hpp; nothing here reads device memory or synchronises.
#include "../../include/sc.h"

#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

#include "sc_kernels.hpp"

struct sc_cache {
    sc_config cfg;
    sc::Layout L;
    int32_t n_trig;
    int32_t n;
    int64_t t;
    float qk_log2;
    // Ragged batches: once a *_ragged call has been made every sequence has its own counters
    // (ts, ns) and the lock-step pair (n, t) above is no longer used.
    bool ragged;
    std::vector<int64_t> ts;       // tokens seen by each sequence
    std::vector<int32_t> ns;       // resident rows of each sequence
    std::vector<int32_t> table;    // what the device table holds (t_b - step, or kSeqIdle)
    std::vector<int32_t> wanted;   // scratch for building the next table
    bool table_known;              // false until the first upload
    int32_t step;                  // ragged decode calls made so far
    int32_t* seq_off;              // device [batch], followed by the device-side step count and the ticket counter
    bool device_clock;             // ragged decode launches read the step count from the device
    bool step_dev_known;           // the device-side count equals `step`
    std::vector<uint8_t> last_active;  // sequences of the most recent ragged decode step
    size_t row_bytes, meta_bytes;  // per K (or V) row, for views of a range of sequences
    unsigned long long* trace;     // diagnostics buffer of the decode launches, or null
};

struct sc_layers {
    std::vector<sc_cache*> layer;
    std::vector<int32_t*> clocks;  // scratch of sc_layers_decode_step: device step counts to advance
};

namespace {

static_assert(SC_STATIC_SCRATCH_BYTES == sc::kStaticScratchBytes, "sc.h and the kernels disagree");

constexpr size_t kAlign = 256;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Sizes {
    int32_t n_trig, C, E, W32;
    size_t row_bytes, meta_bytes;  // per K (or V) row
    size_t off_K, off_V, off_Km, off_Vm, off_pos, off_cnt, off_qh, off_map, off_first, off_seq, off_shares, off_arrive, total;
    int32_t split;  // workgroups per unit of a decode step (very few units with long caches), else 0
    bool recompute;
};

sc_status derive(const sc_config* cfg, Sizes* s) {
    if (!cfg) return SC_ERR_INVALID_ARG;
    if (cfg->batch < 1 || cfg->heads < 1 || cfg->budget < 1 || cfg->recent < 1 || cfg->history < 1 ||
        cfg->drop < 1)
        return SC_ERR_INVALID_ARG;
    if (cfg->trigger != SC_TRIGGER_HARD_CAP && cfg->trigger != SC_TRIGGER_HIGH_WATER)
        return SC_ERR_INVALID_ARG;
    if (cfg->thresh_mode != SC_THRESH_INV_POS && cfg->thresh_mode != SC_THRESH_INV_LEN)
        return SC_ERR_INVALID_ARG;
    if (!(cfg->scale >= 0.0f) || std::isinf(cfg->scale)) return SC_ERR_INVALID_ARG;
    if ((int64_t)cfg->batch * cfg->heads > (1 << 24)) return SC_ERR_INVALID_ARG;
    if (cfg->budget > (1 << 20) || cfg->drop > (1 << 20)) return SC_ERR_INVALID_ARG;
    if (cfg->head_dim != 64 && cfg->head_dim != 128) return SC_ERR_UNSUPPORTED;
    if (cfg->kv_dtype < SC_KV_F32 || cfg->kv_dtype > SC_KV_I4G64) return SC_ERR_UNSUPPORTED;
    if (cfg->window_mode != SC_WINDOW_AUTO && cfg->window_mode != SC_WINDOW_RING) return SC_ERR_INVALID_ARG;
    if (cfg->record_mode != SC_RECORD_ONLINE && cfg->record_mode != SC_RECORD_RECOMPUTE)
        return SC_ERR_INVALID_ARG;
    if (cfg->history > 8192) return SC_ERR_UNSUPPORTED;
    const int64_t n_trig =
        cfg->trigger == SC_TRIGGER_HIGH_WATER ? (int64_t)cfg->budget + cfg->drop : (int64_t)cfg->budget + 1;
    if (cfg->drop > n_trig - cfg->recent) return SC_ERR_INVALID_ARG;
    if (n_trig > 12288) return SC_ERR_UNSUPPORTED;  // one unit's scores must fit in LDS
    s->n_trig = (int32_t)n_trig;
    s->C = (int32_t)((n_trig + 63) / 64 * 64);
    // Recomputed record: one 16-bit count per slot, rebuilt at every compression; the window
    // is exact for any w because the kept queries are replayed one by one.
    s->recompute = cfg->record_mode == SC_RECORD_RECOMPUTE;
    const bool ring = !s->recompute && (cfg->window_mode == SC_WINDOW_RING || cfg->history % cfg->drop != 0);
    s->E = s->recompute ? 1 : ring ? 0 : cfg->history / cfg->drop;
    s->W32 = ring ? (cfg->history + 31) / 32 : 0;
    if (s->recompute && s->C > 6144) return SC_ERR_UNSUPPORTED;  // the replay kernel's LDS budget
    const size_t d = (size_t)cfg->head_dim;
    s->row_bytes = cfg->kv_dtype == SC_KV_F32 ? d * 4 : cfg->kv_dtype == SC_KV_F16 ? d * 2 : d / 2;
    s->meta_bytes = cfg->kv_dtype == SC_KV_I4G64 ? d / 64 * 4 : 0;
    const size_t rows = (size_t)cfg->batch * cfg->heads * (size_t)s->C;
    size_t off = 0;
    s->off_K = off;     off = align_up(off + rows * s->row_bytes);
    s->off_V = off;     off = align_up(off + rows * s->row_bytes);
    s->off_Km = off;    off = align_up(off + rows * s->meta_bytes);
    s->off_Vm = off;    off = align_up(off + rows * s->meta_bytes);
    s->off_pos = off;   off = align_up(off + rows * 4);
    s->off_cnt = off;   off = align_up(off + rows * ((size_t)s->E * 2 + (size_t)s->W32 * 4));
    s->off_qh = off;
    if (s->recompute)
        off = align_up(off + (size_t)cfg->batch * cfg->heads * (size_t)cfg->history * d *
                                 (cfg->kv_dtype == SC_KV_F32 ? 4 : 2));
    s->off_map = off;   off = align_up(off + rows * 4);
    s->off_first = off; off = align_up(off + (size_t)cfg->batch * cfg->heads * 4);
    s->off_seq = off;   off = align_up(off + ((size_t)cfg->batch + 2) * 4);  // table, step count, ticket counter
    // Very few units with long caches leave most CUs idle with one workgroup per unit: the decode
    // step then splits a unit's rows over 8 workgroups (up to 32 units) or 4 (up to 64), fp32/fp16
    // rows only.  Measured on 32 heads x 1050 rows of fp16: 13.4 -> 10.7 us per step at batch 1,
    // 14.0 -> 12.8 at batch 2; from 128 units on (and with 8 workgroups at 64 units) the merge
    // costs more than the extra workgroups gain.
    const int64_t units = (int64_t)cfg->batch * cfg->heads;
    s->split = (cfg->kv_dtype == SC_KV_I4G64 || s->C < 512) ? 0 : units <= 32 ? 8 : units <= 64 ? 4 : 0;
    s->off_shares = off; off = align_up(off + (s->split ? (size_t)units * 8 * (d + 32) * 4 : 0));
    s->off_arrive = off; off = align_up(off + (s->split ? (size_t)units * 4 : 0));
    s->total = off;
    return SC_OK;
}

// ceil((t - n_trig) / m) for any sign.
int64_t epoch_of(int64_t t, int64_t n_trig, int64_t m) {
    const int64_t a = t - n_trig;
    return a >= 0 ? (a + m - 1) / m : -((-a) / m);
}

int32_t bucket_of(int64_t epoch, int32_t E) { return (int32_t)(((epoch % E) + E) % E); }

// How sc_prefill cuts a prompt: positions up to the next boundary of the counter schedule
// share one bucket and no compression falls inside a run; the boundaries are the steps
// t = n_trig + k*m, the same steps after which a compression is due.
constexpr int64_t kMinDenseRun = 16;  // a workgroup of the dense kernel serves 64 positions

struct Run {
    int64_t len, epoch;
    bool dense;
};

Run next_run(const sc_config& cfg, const Sizes& z, int32_t mode, int64_t t, int64_t remaining) {
    Run r;
    r.epoch = epoch_of(t + 1, z.n_trig, cfg.drop);
    r.len = std::min<int64_t>(remaining, z.n_trig + r.epoch * cfg.drop - t);
    const int64_t units = (int64_t)cfg.batch * cfg.heads;
    r.dense = mode == SC_PREFILL_AUTO && r.len >= kMinDenseRun &&
              sc::prefill_chunk_supported(cfg.kv_dtype, cfg.head_dim, z.E, z.W32, z.C) &&
              units * ((r.len + 63) / 64) < (1ll << 31);
    return r;
}

size_t elem_bytes(const sc_config& c) { return c.kv_dtype == SC_KV_F32 ? 4 : 2; }

sc_status step_impl(sc_cache* c, const void* q, const void* k_new, const void* v_new, int64_t in_stride,
                    void* out, int64_t out_stride, float* probs_out, int64_t probs_stride,
                    hipStream_t stream) {
    const int64_t t1 = c->t + 1;
    const int32_t n1 = c->n + 1;
    sc::StepArgs a;
    a.q = q;
    a.k_new = k_new;
    a.v_new = v_new;
    a.in_stride = (long)in_stride;
    a.out = out;
    a.out_stride = (long)out_stride;
    a.probs = probs_out;
    a.probs_stride = (long)probs_stride;
    a.n = n1;
    a.pos_value = (int)(t1 - 1);
    if (c->L.Qh) {  // the record is rebuilt at compression time: nothing is counted here
        a.bucket = 0;
        a.ring_bit = 0;
        a.counted = 0;
    } else if (c->L.W32) {
        const int64_t rho = t1 % c->cfg.history;  // ring bit owned by this step
        a.bucket = (int)(rho >> 5);
        a.ring_bit = 1u << (rho & 31);
        a.counted = 1;
    } else {
        const int64_t ep = epoch_of(t1, c->n_trig, c->cfg.drop);
        a.bucket = bucket_of(ep, c->L.E);
        a.ring_bit = 0;
        a.counted = ep > -(int64_t)c->L.E;
    }
    a.qk_log2 = c->qk_log2;
    a.tau = c->cfg.thresh_mode == SC_THRESH_INV_LEN ? 1.0f / (float)n1 : 1.0f / (float)t1;
    // Record rebuilt at compression time: the attention kernel also keeps this step's query
    // (step t1 in ring slot (t1-1) mod w).
    a.q_keep = c->L.Qh ? static_cast<char*>(c->L.Qh) +
                             (size_t)((t1 - 1) % c->cfg.history) * c->cfg.head_dim * elem_bytes(c->cfg)
                       : nullptr;
    a.trace = c->trace;
    if (sc::launch_decode_step(c->L, a, stream) != hipSuccess) return SC_ERR_DEVICE;
    c->t = t1;
    c->n = n1;
    return SC_OK;
}

sc_status compress_impl(sc_cache* c, int32_t* evicted_out, float* probs_out, hipStream_t stream) {
    if (c->L.Qh) {  // Alg. 2 as printed: the extra attention computation over the history window
        sc::ReplayArgs r;
        r.n = c->n;
        r.t = (long)c->t;
        r.thresh_len = c->cfg.thresh_mode == SC_THRESH_INV_LEN;
        r.qk_log2 = c->qk_log2;
        r.probs = probs_out;
        r.probs_unit_stride = 0;
        if (sc::launch_recompute_record(c->L, r, stream) != hipSuccess) return SC_ERR_DEVICE;
    }
    sc::CompressArgs a;
    a.n = c->n;
    a.r = c->cfg.recent;
    a.m = c->cfg.drop;
    // The step that made the cache full closed epoch k; the following steps count into k+1.
    a.zero_bucket = -1;
    if (c->L.E && !c->L.Qh) {
        const int64_t ep = epoch_of(c->t, c->n_trig, c->cfg.drop);
        a.zero_bucket = bucket_of(ep + 1, c->L.E);
    }
    a.evicted = evicted_out;
    if (sc::launch_compress(c->L, a, stream) != hipSuccess) return SC_ERR_DEVICE;
    c->n -= c->cfg.drop;
    return SC_OK;
}

// The same cache restricted to the units of sequences [b0, b1).
sc::Layout view_of(const sc_cache* c, const sc::Layout& whole, int b0, int b1) {
    sc::Layout L = whole;
    const size_t u0 = (size_t)b0 * c->cfg.heads, C = (size_t)whole.C;
    L.U = (b1 - b0) * c->cfg.heads;
    L.K = static_cast<char*>(whole.K) + u0 * C * c->row_bytes;
    L.V = static_cast<char*>(whole.V) + u0 * C * c->row_bytes;
    if (whole.K_meta) {
        L.K_meta = static_cast<char*>(whole.K_meta) + u0 * C * c->meta_bytes;
        L.V_meta = static_cast<char*>(whole.V_meta) + u0 * C * c->meta_bytes;
    }
    L.pos = whole.pos + u0 * C;
    L.cnt = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(whole.cnt) +
                                        u0 * C * ((size_t)whole.E * 2 + (size_t)whole.W32 * 4));
    if (whole.Qh) L.Qh = static_cast<char*>(whole.Qh) + u0 * (size_t)whole.w * whole.d * elem_bytes(c->cfg);
    L.srcmap = whole.srcmap + u0 * C;
    L.first = whole.first + u0;
    if (whole.shares) {
        L.shares = whole.shares + u0 * 8 * ((size_t)whole.d + 32);
        L.arrive = whole.arrive + u0;
    }
    return L;
}

// From lock step to per-sequence counters (nothing on the device changes).
sc_status enter_ragged(sc_cache* c) {
    if (c->ragged) return SC_OK;
    if (c->n >= c->n_trig) return SC_ERR_FULL;  // the pending lock-step compression comes first
    const size_t B = (size_t)c->cfg.batch;
    try {  // nothing may be thrown across the C ABI
        c->ts.assign(B, c->t);
        c->ns.assign(B, c->n);
        c->table.assign(B, sc::kSeqIdle);
        c->wanted.assign(B, sc::kSeqIdle);
        c->last_active.assign(B, 0);
    } catch (const std::bad_alloc&) {
        return SC_ERR_HOST_MEMORY;
    }
    c->table_known = false;
    c->step = 0;
    c->step_dev_known = false;
    c->ragged = true;
    return SC_OK;
}

sc::SeqSched make_sched(const sc_cache* c, int32_t step) {
    sc::SeqSched q;
    q.off = c->seq_off;
    q.step = step;
    q.heads = c->cfg.heads;
    q.n_trig = c->n_trig;
    q.m = c->cfg.drop;
    q.w = c->cfg.history;
    q.E = c->L.E;
    q.W32 = c->L.W32;
    q.thresh_len = c->cfg.thresh_mode == SC_THRESH_INV_LEN;
    q.recompute = c->L.Qh != nullptr;
    q.step_dev = nullptr;
    return q;
}

// Make the device table equal to c->wanted (uploaded only when it differs).
sc_status sync_table(sc_cache* c, hipStream_t s) {
    if (c->table_known && c->table == c->wanted) return SC_OK;
    if (sc::launch_write_seq_table(c->seq_off, c->wanted.data(), c->cfg.batch, s) != hipSuccess)
        return SC_ERR_DEVICE;
    c->table = c->wanted;
    c->table_known = true;
    return SC_OK;
}

// The prompt of all units of c->L (which may be a view of a range of sequences), cut into runs.
// stride / out_stride / probs_stride: elements between units in q,k,v / out / probs_out.
sc_status prefill_core(sc_cache* c, const void* q, const void* k, const void* v, int64_t prompt_len,
                       int64_t stride, void* out, int64_t out_stride, float* probs_out, int64_t probs_stride,
                       int32_t mode, hipStream_t s) {
    const int64_t d = c->cfg.head_dim;
    const size_t eb = elem_bytes(c->cfg);
    Sizes z;
    if (derive(&c->cfg, &z) != SC_OK) return SC_ERR_INVALID_ARG;
    int64_t i = 0;
    while (i < prompt_len) {
        const Run r = next_run(c->cfg, z, mode, c->t, prompt_len - i);
        const int64_t run = r.len, ep = r.epoch;
        const size_t off = (size_t)i * d * eb;
        void* o = out ? static_cast<char*>(out) + off : nullptr;
        float* pr = probs_out ? probs_out + (size_t)i * c->L.C : nullptr;
        if (r.dense) {
            sc::ChunkArgs a;
            a.q = static_cast<const char*>(q) + off;
            a.k = static_cast<const char*>(k) + off;
            a.v = static_cast<const char*>(v) + off;
            a.unit_stride = (long)stride;
            a.out = o;
            a.out_unit_stride = (long)out_stride;
            a.probs = pr;
            a.probs_unit_stride = (long)probs_stride;
            a.n0 = c->n;
            a.c = (int)run;
            a.t0 = (long)c->t;
            a.bucket = c->L.E ? bucket_of(ep, c->L.E) : 0;
            // the ring records every step; counters skip steps older than every window
            a.counted = c->L.W32 ? 1 : (!c->L.Qh && ep > -(int64_t)c->L.E);
            a.thresh_len = c->cfg.thresh_mode == SC_THRESH_INV_LEN;
            a.qk_log2 = c->qk_log2;
            if (sc::launch_prefill_chunk(c->L, a, s) != hipSuccess) return SC_ERR_DEVICE;
            if (c->L.Qh && sc::launch_store_queries(c->L, a.q, (long)stride, (int)run, (long)c->t, s) != hipSuccess)
                return SC_ERR_DEVICE;
            c->t += run;
            c->n += (int32_t)run;
        } else {
            for (int64_t j = 0; j < run; ++j) {
                const size_t offj = off + (size_t)j * d * eb;
                sc_status st = step_impl(c, static_cast<const char*>(q) + offj, static_cast<const char*>(k) + offj,
                                         static_cast<const char*>(v) + offj, stride,
                                         o ? static_cast<char*>(o) + (size_t)j * d * eb : nullptr,
                                         out_stride, pr ? pr + (size_t)j * c->L.C : nullptr,
                                         probs_stride, s);
                if (st != SC_OK) return st;
            }
        }
        i += run;
        if (c->n == c->n_trig) {
            const sc_status st = compress_impl(c, nullptr, nullptr, s);
            if (st != SC_OK) return st;
        }
    }
    return SC_OK;
}

}  // namespace

extern "C" {

sc_status sc_config_sizes(const sc_config* cfg, int32_t* n_trig, int32_t* capacity, int32_t* buckets,
                          int32_t* ring_words) {
    Sizes s;
    const sc_status st = derive(cfg, &s);
    if (st != SC_OK) return st;
    if (n_trig) *n_trig = s.n_trig;
    if (capacity) *capacity = s.C;
    if (buckets) *buckets = s.E;
    if (ring_words) *ring_words = s.W32;
    return SC_OK;
}

size_t sc_workspace_bytes(const sc_config* cfg) {
    Sizes s;
    return derive(cfg, &s) == SC_OK ? s.total : 0;
}

sc_status sc_schedule(const sc_config* cfg, int64_t t, int64_t* epoch, int32_t* bucket, int32_t* counted) {
    Sizes s;
    const sc_status st = derive(cfg, &s);
    if (st != SC_OK) return st;
    if (t < 1) return SC_ERR_INVALID_ARG;
    const int64_t ep = epoch_of(t, s.n_trig, cfg->drop);
    if (epoch) *epoch = ep;
    if (s.W32) {
        if (bucket) *bucket = (int32_t)((t % cfg->history) >> 5);
        if (counted) *counted = 1;
        return SC_OK;
    }
    if (bucket) *bucket = bucket_of(ep, s.E);
    if (counted) *counted = ep > -(int64_t)s.E;
    return SC_OK;
}

sc_status sc_schedule_rows(const sc_config* cfg, int64_t t, int32_t* rows, int32_t* due) {
    Sizes s;
    const sc_status st = derive(cfg, &s);
    if (st != SC_OK) return st;
    if (t < 1) return SC_ERR_INVALID_ARG;
    if (rows) *rows = sc::sched_rows((long)t, s.n_trig, cfg->drop);
    if (due) *due = sc::sched_due((long)t, s.n_trig, cfg->drop);
    return SC_OK;
}

sc_status sc_cache_create(const sc_config* cfg, void* dev_workspace, size_t bytes, void* stream,
                          sc_cache** out) {
    if (!out) return SC_ERR_INVALID_ARG;
    Sizes s;
    const sc_status st = derive(cfg, &s);
    if (st != SC_OK) return st;
    if (!dev_workspace) return SC_ERR_INVALID_ARG;
    if (bytes < s.total || (reinterpret_cast<uintptr_t>(dev_workspace) % kAlign) != 0)
        return SC_ERR_WORKSPACE;
    sc_cache* c = new (std::nothrow) sc_cache;
    if (!c) return SC_ERR_HOST_MEMORY;
    c->cfg = *cfg;
    char* base = static_cast<char*>(dev_workspace);
    sc::Layout& L = c->L;
    L.U = cfg->batch * cfg->heads;
    L.d = cfg->head_dim;
    L.kv_dtype = cfg->kv_dtype;
    L.C = s.C;
    L.E = s.E;
    L.W32 = s.W32;
    L.K = base + s.off_K;
    L.V = base + s.off_V;
    L.K_meta = s.meta_bytes ? base + s.off_Km : nullptr;
    L.V_meta = s.meta_bytes ? base + s.off_Vm : nullptr;
    L.pos = reinterpret_cast<int32_t*>(base + s.off_pos);
    L.cnt = reinterpret_cast<uint16_t*>(base + s.off_cnt);
    L.Qh = s.recompute ? base + s.off_qh : nullptr;
    L.w = cfg->history;
    L.srcmap = reinterpret_cast<int32_t*>(base + s.off_map);
    L.first = reinterpret_cast<int32_t*>(base + s.off_first);
    L.ticket = reinterpret_cast<int32_t*>(base + s.off_seq) + cfg->batch + 1;
    L.split = s.split;
    L.shares = s.split ? reinterpret_cast<float*>(base + s.off_shares) : nullptr;
    L.arrive = s.split ? reinterpret_cast<int32_t*>(base + s.off_arrive) : nullptr;
    c->ragged = false;
    c->table_known = false;
    c->step = 0;
    c->device_clock = false;
    c->step_dev_known = false;
    c->seq_off = reinterpret_cast<int32_t*>(base + s.off_seq);
    c->row_bytes = s.row_bytes;
    c->meta_bytes = s.meta_bytes;
    c->trace = nullptr;
    c->n_trig = s.n_trig;
    c->n = 0;
    c->t = 0;
    const float scale = cfg->scale > 0.0f ? cfg->scale : 1.0f / std::sqrt((float)cfg->head_dim);
    c->qk_log2 = scale * 1.4426950408889634f;
    if (sc::launch_clear_counters(L, static_cast<hipStream_t>(stream)) != hipSuccess) {
        delete c;
        return SC_ERR_DEVICE;
    }
    *out = c;
    return SC_OK;
}

sc_status sc_cache_reset(sc_cache* c, void* stream) {
    if (!c) return SC_ERR_INVALID_ARG;
    if (sc::launch_clear_counters(c->L, static_cast<hipStream_t>(stream)) != hipSuccess) return SC_ERR_DEVICE;
    c->n = 0;
    c->t = 0;
    c->ragged = false;
    c->table_known = false;
    c->step = 0;
    c->step_dev_known = false;
    return SC_OK;
}

void sc_cache_destroy(sc_cache* c) { delete c; }

sc_status sc_decode_step(sc_cache* c, const void* q, const void* k_new, const void* v_new,
                         int64_t in_stride, void* out, float* probs_out, int32_t* compress_due,
                         void* stream) {
    if (!c || !q || !k_new || !v_new || !out) return SC_ERR_INVALID_ARG;
    if (in_stride < 0 || (in_stride != 0 && in_stride < c->cfg.head_dim)) return SC_ERR_INVALID_ARG;
    const size_t eb = elem_bytes(c->cfg);
    if (in_stride != 0 && (in_stride * eb) % 16 != 0) return SC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_new) |
         reinterpret_cast<uintptr_t>(v_new) | reinterpret_cast<uintptr_t>(out)) % 16 != 0)
        return SC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(probs_out) % 8 != 0) return SC_ERR_INVALID_ARG;  // stored in pairs
    if (c->ragged) return SC_ERR_STATE;
    if (c->n >= c->n_trig) return SC_ERR_FULL;
    const int64_t stride = in_stride ? in_stride : c->cfg.head_dim;
    const sc_status st = step_impl(c, q, k_new, v_new, stride, out, c->cfg.head_dim, probs_out, c->L.C,
                                   static_cast<hipStream_t>(stream));
    if (st != SC_OK) return st;
    if (compress_due) *compress_due = (c->n == c->n_trig);
    return SC_OK;
}

sc_status sc_compress(sc_cache* c, int32_t* evicted_out, float* probs_out, void* stream) {
    if (!c) return SC_ERR_INVALID_ARG;
    if (c->ragged || c->n != c->n_trig) return SC_ERR_STATE;
    return compress_impl(c, evicted_out, probs_out, static_cast<hipStream_t>(stream));
}

sc_status sc_compress_static(sc_cache* c, int32_t* evicted_out, float* probs_out, void* stream) {
    if (!c) return SC_ERR_INVALID_ARG;
    if (c->ragged || c->n != c->n_trig) return SC_ERR_STATE;
    // `first` [U] then `srcmap` [U][C], both 256-byte aligned inside the library's array.
    const size_t first_bytes = align_up((size_t)c->L.U * sizeof(int32_t));
    const size_t need = first_bytes + (size_t)c->L.U * (size_t)c->L.C * sizeof(int32_t);
    if (need > sc::kStaticScratchBytes) return SC_ERR_SCRATCH;
    void* base = nullptr;
    if (sc::static_scratch(&base) != hipSuccess) return SC_ERR_DEVICE;
    int32_t* const ws_map = c->L.srcmap;
    int32_t* const ws_first = c->L.first;
    c->L.first = static_cast<int32_t*>(base);
    c->L.srcmap = reinterpret_cast<int32_t*>(static_cast<char*>(base) + first_bytes);
    const sc_status st = compress_impl(c, evicted_out, probs_out, static_cast<hipStream_t>(stream));
    c->L.srcmap = ws_map;
    c->L.first = ws_first;
    return st;
}

sc_status sc_prefill(sc_cache* c, const void* q, const void* k, const void* v, int32_t prompt_len,
                     int64_t unit_stride, void* out, float* probs_out, int32_t mode, void* stream) {
    if (!c || !q || !k || !v || prompt_len < 1) return SC_ERR_INVALID_ARG;
    if (mode != SC_PREFILL_AUTO && mode != SC_PREFILL_STREAMED) return SC_ERR_INVALID_ARG;
    if (c->ragged) return SC_ERR_STATE;
    if (c->n >= c->n_trig) return SC_ERR_FULL;
    const int64_t d = c->cfg.head_dim;
    const int64_t stride = unit_stride ? unit_stride : (int64_t)prompt_len * d;
    if (stride < (int64_t)prompt_len * d) return SC_ERR_INVALID_ARG;
    const size_t eb = elem_bytes(c->cfg);
    if ((stride * eb) % 16 != 0) return SC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(v) |
         reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(probs_out)) % 16 != 0)
        return SC_ERR_INVALID_ARG;
    return prefill_core(c, q, k, v, prompt_len, stride, out, (int64_t)prompt_len * d, probs_out,
                        (int64_t)prompt_len * c->L.C, mode, static_cast<hipStream_t>(stream));
}

sc_status sc_prefill_plan(const sc_config* cfg, int32_t prompt_len, int32_t mode, int32_t max_runs,
                          int32_t* run_len, int32_t* run_dense, int32_t* run_compress, int32_t* n_runs) {
    Sizes z;
    const sc_status st = derive(cfg, &z);
    if (st != SC_OK) return st;
    if (prompt_len < 1 || max_runs < 0 || !n_runs) return SC_ERR_INVALID_ARG;
    if (mode != SC_PREFILL_AUTO && mode != SC_PREFILL_STREAMED) return SC_ERR_INVALID_ARG;
    int64_t t = 0, n = 0, i = 0;
    int32_t count = 0;
    while (i < prompt_len) {
        const Run r = next_run(*cfg, z, mode, t, prompt_len - i);
        t += r.len;
        n += r.len;
        const bool due = n == z.n_trig;
        if (due) n -= cfg->drop;
        if (count < max_runs) {
            if (run_len) run_len[count] = (int32_t)r.len;
            if (run_dense) run_dense[count] = r.dense;
            if (run_compress) run_compress[count] = due;
        }
        ++count;
        i += r.len;
    }
    *n_runs = count;
    return SC_OK;
}

sc_status sc_cache_len(const sc_cache* c, int32_t* n, int64_t* t) {
    if (!c) return SC_ERR_INVALID_ARG;
    if (c->ragged) return SC_ERR_STATE;
    if (n) *n = c->n;
    if (t) *t = c->t;
    return SC_OK;
}

sc_status sc_cache_len_seq(const sc_cache* c, int32_t b, int32_t* n, int64_t* t) {
    if (!c || b < 0 || b >= c->cfg.batch) return SC_ERR_INVALID_ARG;
    if (n) *n = c->ragged ? c->ns[b] : c->n;
    if (t) *t = c->ragged ? c->ts[b] : c->t;
    return SC_OK;
}

sc_status sc_cache_reset_seq(sc_cache* c, int32_t b, void* stream) {
    if (!c || b < 0 || b >= c->cfg.batch) return SC_ERR_INVALID_ARG;
    const sc_status st0 = enter_ragged(c);
    if (st0 != SC_OK) return st0;
    if (sc::launch_clear_counters(view_of(c, c->L, b, b + 1), static_cast<hipStream_t>(stream)) != hipSuccess)
        return SC_ERR_DEVICE;
    c->ts[b] = 0;
    c->ns[b] = 0;
    return SC_OK;
}

sc_status sc_prefill_ragged(sc_cache* c, const void* q, const void* k, const void* v,
                            const int32_t* prompt_len, int64_t unit_stride, void* out, float* probs_out,
                            int32_t mode, void* stream) {
    if (!c || !q || !k || !v || !prompt_len) return SC_ERR_INVALID_ARG;
    if (mode != SC_PREFILL_AUTO && mode != SC_PREFILL_STREAMED) return SC_ERR_INVALID_ARG;
    const int B = c->cfg.batch;
    int64_t longest = 0;
    for (int b = 0; b < B; ++b) {
        if (prompt_len[b] < 0) return SC_ERR_INVALID_ARG;
        if (prompt_len[b] > 0 && (c->ragged ? c->ns[b] : c->n) >= c->n_trig) return SC_ERR_FULL;
        longest = std::max<int64_t>(longest, prompt_len[b]);
    }
    if (longest == 0) return SC_ERR_INVALID_ARG;
    const int64_t d = c->cfg.head_dim;
    const int64_t stride = unit_stride ? unit_stride : longest * d;
    if (stride < longest * d) return SC_ERR_INVALID_ARG;
    const size_t eb = elem_bytes(c->cfg);
    if ((stride * eb) % 16 != 0) return SC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(v) |
         reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(probs_out)) % 16 != 0)
        return SC_ERR_INVALID_ARG;
    const sc_status st0 = enter_ragged(c);
    if (st0 != SC_OK) return st0;
    // Consecutive sequences with the same counters and the same prompt length advance in lock
    // step: each such range is prefilled as a view of the cache, with the same kernels as a
    // whole batch.
    const sc::Layout whole = c->L;
    const int32_t n_saved = c->n;
    const int64_t t_saved = c->t;
    const int64_t out_stride = longest * d, probs_stride = longest * whole.C;
    sc_status st = SC_OK;
    for (int b0 = 0; b0 < B && st == SC_OK;) {
        int b1 = b0 + 1;
        while (b1 < B && prompt_len[b1] == prompt_len[b0] && c->ts[b1] == c->ts[b0] && c->ns[b1] == c->ns[b0])
            ++b1;
        if (prompt_len[b0] > 0) {
            const size_t u0 = (size_t)b0 * c->cfg.heads;
            c->L = view_of(c, whole, b0, b1);
            c->n = c->ns[b0];
            c->t = c->ts[b0];
            st = prefill_core(c, static_cast<const char*>(q) + u0 * stride * eb,
                              static_cast<const char*>(k) + u0 * stride * eb,
                              static_cast<const char*>(v) + u0 * stride * eb, prompt_len[b0], stride,
                              out ? static_cast<char*>(out) + u0 * out_stride * eb : nullptr, out_stride,
                              probs_out ? probs_out + u0 * probs_stride : nullptr, probs_stride, mode,
                              static_cast<hipStream_t>(stream));
            for (int b = b0; b < b1; ++b) {
                c->ts[b] = c->t;
                c->ns[b] = c->n;
            }
        }
        b0 = b1;
    }
    c->L = whole;
    c->n = n_saved;
    c->t = t_saved;
    return st;
}

// `tick`: advance the device-side step count right after the launch (a layer set advances the
// counts of all its caches with one launch instead).
static sc_status decode_step_ragged_impl(sc_cache* c, const void* q, const void* k_new, const void* v_new,
                                         int64_t in_stride, void* out, float* probs_out, const uint8_t* active,
                                         int32_t* n_due, void* stream, bool tick) {
    if (!c || !q || !k_new || !v_new || !out) return SC_ERR_INVALID_ARG;
    if (in_stride < 0 || (in_stride != 0 && in_stride < c->cfg.head_dim)) return SC_ERR_INVALID_ARG;
    const size_t eb = elem_bytes(c->cfg);
    if (in_stride != 0 && (in_stride * eb) % 16 != 0) return SC_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_new) |
         reinterpret_cast<uintptr_t>(v_new) | reinterpret_cast<uintptr_t>(out)) % 16 != 0)
        return SC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(probs_out) % 8 != 0) return SC_ERR_INVALID_ARG;  // stored in pairs
    const int B = c->cfg.batch;
    bool any = false;
    for (int b = 0; b < B; ++b) any = any || !active || active[b];
    if (!any) return SC_ERR_INVALID_ARG;
    for (int b = 0; b < B; ++b)  // checked before anything changes, the counters' mode included
        if ((c->ragged ? c->ns[b] : c->n) >= c->n_trig) return SC_ERR_FULL;
    const sc_status st0 = enter_ragged(c);
    if (st0 != SC_OK) return st0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // t_b of the step being computed = table[b] + (step + 1)
    for (int b = 0; b < B; ++b)
        c->wanted[b] = (!active || active[b]) ? (int32_t)(c->ts[b] - c->step) : sc::kSeqIdle;
    const sc_status stt = sync_table(c, s);
    if (stt != SC_OK) return stt;
    sc::StepArgs a;
    a.q = q;
    a.k_new = k_new;
    a.v_new = v_new;
    a.in_stride = (long)(in_stride ? in_stride : c->cfg.head_dim);
    a.out = out;
    a.out_stride = c->cfg.head_dim;
    a.probs = probs_out;
    a.probs_stride = c->L.C;
    a.n = 0;
    a.pos_value = 0;
    a.bucket = 0;
    a.counted = 0;
    a.ring_bit = 0;
    a.qk_log2 = c->qk_log2;
    a.tau = 0.f;
    a.q_keep = c->L.Qh;  // kept queries: the kernels pick each sequence's own ring slot
    a.seq = make_sched(c, c->step + 1);
    if (c->device_clock) {
        int32_t* step_dev = c->seq_off + B;
        if (!c->step_dev_known) {
            if (sc::launch_write_seq_table(step_dev, &c->step, 1, s) != hipSuccess) return SC_ERR_DEVICE;
            c->step_dev_known = true;
        }
        a.seq.step_dev = step_dev;
        a.seq.step = 0;
    }
    a.trace = c->trace;
    if (sc::launch_decode_step(c->L, a, s) != hipSuccess) return SC_ERR_DEVICE;
    if (c->device_clock && tick) {
        int32_t* const counter = c->seq_off + B;
        if (sc::launch_tick(&counter, 1, s) != hipSuccess) return SC_ERR_DEVICE;
    }
    c->step += 1;
    int32_t due = 0;
    for (int b = 0; b < B; ++b) {
        c->last_active[b] = c->wanted[b] != sc::kSeqIdle;
        if (c->wanted[b] == sc::kSeqIdle) continue;
        c->ts[b] += 1;
        c->ns[b] += 1;
        due += c->ns[b] == c->n_trig;
    }
    if (n_due) *n_due = due;
    return SC_OK;
}

sc_status sc_decode_step_ragged(sc_cache* c, const void* q, const void* k_new, const void* v_new,
                                int64_t in_stride, void* out, float* probs_out, const uint8_t* active,
                                int32_t* n_due, void* stream) {
    return decode_step_ragged_impl(c, q, k_new, v_new, in_stride, out, probs_out, active, n_due, stream, true);
}

sc_status sc_cache_device_clock(sc_cache* c, int32_t enable) {
    if (!c) return SC_ERR_INVALID_ARG;
    const sc_status st0 = enter_ragged(c);
    if (st0 != SC_OK) return st0;
    c->device_clock = enable != 0;
    c->step_dev_known = false;
    return SC_OK;
}

sc_status sc_steps_until_due(const sc_cache* c, const uint8_t* active, int32_t* steps) {
    if (!c || !steps) return SC_ERR_INVALID_ARG;
    int32_t least = INT32_MAX;
    for (int b = 0; b < c->cfg.batch; ++b) {
        if (active && !active[b]) continue;
        least = std::min<int32_t>(least, c->n_trig - (c->ragged ? c->ns[b] : c->n));
    }
    if (least == INT32_MAX) return SC_ERR_INVALID_ARG;
    *steps = least;
    return SC_OK;
}

sc_status sc_cache_note_replays(sc_cache* c, int32_t k, int32_t* n_due) {
    if (!c || k < 0) return SC_ERR_INVALID_ARG;
    if (!c->ragged || !c->device_clock || c->step == 0) return SC_ERR_STATE;
    const int B = c->cfg.batch;
    for (int b = 0; b < B; ++b)
        if (c->last_active[b] && c->ns[b] + k > c->n_trig) return SC_ERR_FULL;
    int32_t due = 0;
    for (int b = 0; b < B; ++b) {
        if (c->last_active[b]) {
            c->ts[b] += k;
            c->ns[b] += k;
        }
        due += c->ns[b] == c->n_trig;
    }
    c->step += k;
    if (n_due) *n_due = due;
    return SC_OK;
}

sc_status sc_compress_ragged(sc_cache* c, int32_t* evicted_out, float* probs_out, void* stream) {
    if (!c) return SC_ERR_INVALID_ARG;
    if (!c->ragged) return SC_ERR_STATE;
    const int B = c->cfg.batch;
    bool any = false, table_fits = c->table_known;
    for (int b = 0; b < B; ++b) {
        const bool pending = c->ns[b] == c->n_trig;
        any = any || pending;
        c->wanted[b] = pending ? (int32_t)(c->ts[b] - c->step) : sc::kSeqIdle;
        if (!table_fits) continue;
        // The table of the latest step serves as it is when it marks exactly the pending
        // sequences as due (the others are idle or stand between two compressions).
        const int32_t e = c->table[b];
        const bool due_by_table = e != sc::kSeqIdle && sc::sched_due((long)e + c->step, c->n_trig, c->cfg.drop);
        table_fits = pending ? (e == c->wanted[b]) : !due_by_table;
    }
    if (!any) return SC_ERR_STATE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!table_fits) {
        c->table_known = false;
        const sc_status stt = sync_table(c, s);
        if (stt != SC_OK) return stt;
    }
    if (c->L.Qh) {
        // Alg. 2 as printed: every range of due sequences with the same token count replays its
        // kept queries as one dense block over its own units.
        for (int b0 = 0; b0 < B;) {
            int b1 = b0 + 1;
            if (c->ns[b0] != c->n_trig) {
                b0 = b1;
                continue;
            }
            while (b1 < B && c->ns[b1] == c->n_trig && c->ts[b1] == c->ts[b0]) ++b1;
            sc::ReplayArgs r;
            r.n = c->n_trig;
            r.t = (long)c->ts[b0];
            r.thresh_len = c->cfg.thresh_mode == SC_THRESH_INV_LEN;
            r.qk_log2 = c->qk_log2;
            r.probs_unit_stride = (long)c->cfg.history * c->L.C;
            r.probs = probs_out ? probs_out + (size_t)b0 * c->cfg.heads * (size_t)r.probs_unit_stride : nullptr;
            if (sc::launch_recompute_record(view_of(c, c->L, b0, b1), r, s) != hipSuccess) return SC_ERR_DEVICE;
            b0 = b1;
        }
    }
    sc::CompressArgs a;
    a.n = c->n_trig;
    a.r = c->cfg.recent;
    a.m = c->cfg.drop;
    a.zero_bucket = -1;
    a.evicted = evicted_out;
    a.seq = make_sched(c, c->step);
    if (sc::launch_compress(c->L, a, s) != hipSuccess) return SC_ERR_DEVICE;
    for (int b = 0; b < B; ++b)
        if (c->ns[b] == c->n_trig) c->ns[b] -= c->cfg.drop;
    return SC_OK;
}

sc_status sc_cache_view(const sc_cache* c, const void** K, const void** V, const void** K_meta,
                        const void** V_meta, const int32_t** pos, const uint16_t** cnt, int32_t* capacity,
                        int32_t* buckets) {
    if (!c) return SC_ERR_INVALID_ARG;
    if (K) *K = c->L.K;
    if (V) *V = c->L.V;
    if (K_meta) *K_meta = c->L.K_meta;
    if (V_meta) *V_meta = c->L.V_meta;
    if (pos) *pos = c->L.pos;
    if (cnt) *cnt = c->L.cnt;
    if (capacity) *capacity = c->L.C;
    if (buckets) *buckets = c->L.E ? c->L.E : c->L.W32;
    return SC_OK;
}

sc_status sc_diag_trace(sc_cache* c, uint64_t* trace_out) {
    if (!c) return SC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(trace_out) % 8 != 0) return SC_ERR_INVALID_ARG;
    if (trace_out && c->L.split) return SC_ERR_UNSUPPORTED;  // several workgroups per unit
    c->trace = reinterpret_cast<unsigned long long*>(trace_out);
    return SC_OK;
}

sc_status sc_diag_read_bandwidth(const void* buf, size_t bytes, int32_t nontemporal, uint32_t* sink,
                                 void* stream) {
    if (!buf || !sink || bytes == 0 || bytes % ((size_t)32 << 20) != 0) return SC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(buf) % 16 != 0 || reinterpret_cast<uintptr_t>(sink) % 4 != 0)
        return SC_ERR_INVALID_ARG;
    if (sc::launch_read_stream(buf, bytes, nontemporal != 0, sink, static_cast<hipStream_t>(stream)) != hipSuccess)
        return SC_ERR_DEVICE;
    return SC_OK;
}

sc_status sc_diag_persistence(const float* probs, int32_t units, int32_t length, int64_t row_stride,
                              int64_t unit_stride, int32_t split, int32_t* counts_out, void* stream) {
    if (!probs || !counts_out || units < 1 || length < 1 || split < 0 || split > length) return SC_ERR_INVALID_ARG;
    if (row_stride < length || unit_stride < (int64_t)(length - 1) * row_stride + length) return SC_ERR_INVALID_ARG;
    if (sc::launch_persistence(probs, units, length, (long)row_stride, (long)unit_stride, split, counts_out,
                               static_cast<hipStream_t>(stream)) != hipSuccess)
        return SC_ERR_DEVICE;
    return SC_OK;
}

sc_status sc_diag_kept_mass(const sc_cache* c, const float* probs_full, int64_t unit_stride, float* mass_out,
                            void* stream) {
    if (!c || !probs_full || !mass_out || unit_stride < c->t) return SC_ERR_INVALID_ARG;
    if (c->ragged) return SC_ERR_STATE;
    if (sc::launch_kept_mass(c->L, c->n, probs_full, (long)unit_stride, mass_out,
                             static_cast<hipStream_t>(stream)) != hipSuccess)
        return SC_ERR_DEVICE;
    return SC_OK;
}

size_t sc_layers_workspace_bytes(const sc_config* cfg, int32_t layers, const int32_t* budgets,
                                 const int32_t* drops) {
    if (!cfg || layers < 1 || !budgets) return 0;
    size_t total = 0;
    for (int32_t l = 0; l < layers; ++l) {
        sc_config c = *cfg;
        c.budget = budgets[l];
        if (drops) c.drop = drops[l];
        const size_t b = sc_workspace_bytes(&c);
        if (b == 0) return 0;
        total += b;  // every cache's size is a multiple of the alignment
    }
    return total;
}

sc_status sc_layers_create(const sc_config* cfg, int32_t layers, const int32_t* budgets, const int32_t* drops,
                           void* dev_workspace, size_t bytes, void* stream, sc_layers** out) {
    if (!cfg || layers < 1 || !budgets || !out) return SC_ERR_INVALID_ARG;
    if (!dev_workspace) return SC_ERR_INVALID_ARG;
    sc_layers* ls = new (std::nothrow) sc_layers;
    if (!ls) return SC_ERR_HOST_MEMORY;
    size_t off = 0;
    for (int32_t l = 0; l < layers; ++l) {
        sc_config c = *cfg;
        c.budget = budgets[l];
        if (drops) c.drop = drops[l];
        Sizes z;
        sc_status st = derive(&c, &z);
        if (st == SC_OK && off + z.total > bytes) st = SC_ERR_WORKSPACE;
        sc_cache* h = nullptr;
        if (st == SC_OK) st = sc_cache_create(&c, static_cast<char*>(dev_workspace) + off, z.total, stream, &h);
        if (st != SC_OK) {
            sc_layers_destroy(ls);
            return st;
        }
        try {  // nothing may be thrown across the C ABI
            ls->layer.push_back(h);
        } catch (const std::bad_alloc&) {
            sc_cache_destroy(h);
            sc_layers_destroy(ls);
            return SC_ERR_HOST_MEMORY;
        }
        off += z.total;
    }
    try {
        ls->clocks.reserve(ls->layer.size());
    } catch (const std::bad_alloc&) {
        sc_layers_destroy(ls);
        return SC_ERR_HOST_MEMORY;
    }
    *out = ls;
    return SC_OK;
}

sc_cache* sc_layers_get(sc_layers* ls, int32_t layer) {
    return ls && layer >= 0 && (size_t)layer < ls->layer.size() ? ls->layer[(size_t)layer] : nullptr;
}

int32_t sc_layers_count(const sc_layers* ls) { return ls ? (int32_t)ls->layer.size() : 0; }

sc_status sc_layers_device_clock(sc_layers* ls, int32_t enable) {
    if (!ls) return SC_ERR_INVALID_ARG;
    for (sc_cache* h : ls->layer) {
        const sc_status st = sc_cache_device_clock(h, enable);
        if (st != SC_OK) return st;
    }
    return SC_OK;
}

sc_status sc_layers_decode_step(sc_layers* ls, const void* q, const void* k_new, const void* v_new,
                                int64_t layer_stride, int64_t in_stride, void* out, int64_t out_layer_stride,
                                const uint8_t* active, int32_t* n_due, void* stream) {
    if (!ls || ls->layer.empty() || !q || !k_new || !v_new || !out) return SC_ERR_INVALID_ARG;
    const sc_cache* c0 = ls->layer[0];
    const size_t eb = elem_bytes(c0->cfg);
    const int64_t row = in_stride ? in_stride : c0->cfg.head_dim;
    const int64_t units = (int64_t)c0->cfg.batch * c0->cfg.heads;
    if (layer_stride < (units - 1) * row + c0->cfg.head_dim || (layer_stride * (int64_t)eb) % 16 != 0)
        return SC_ERR_INVALID_ARG;
    if (out_layer_stride < units * c0->cfg.head_dim || (out_layer_stride * (int64_t)eb) % 16 != 0)
        return SC_ERR_INVALID_ARG;
    // nothing is enqueued unless every layer can take the step
    for (const sc_cache* h : ls->layer)
        for (int b = 0; b < h->cfg.batch; ++b)
            if ((!active || active[b]) && (h->ragged ? h->ns[b] : h->n) >= h->n_trig) return SC_ERR_FULL;
    int32_t total = 0;
    ls->clocks.clear();  // (capacity reserved at creation: nothing is allocated here)
    sc_status st = SC_OK;
    for (size_t l = 0; l < ls->layer.size() && st == SC_OK; ++l) {
        const size_t in_off = l * (size_t)layer_stride * eb, out_off = l * (size_t)out_layer_stride * eb;
        int32_t due = 0;
        sc_cache* h = ls->layer[l];
        st = decode_step_ragged_impl(h, static_cast<const char*>(q) + in_off,
                                     static_cast<const char*>(k_new) + in_off,
                                     static_cast<const char*>(v_new) + in_off, in_stride,
                                     static_cast<char*>(out) + out_off, nullptr, active, &due, stream, false);
        if (st == SC_OK && h->device_clock) ls->clocks.push_back(h->seq_off + h->cfg.batch);
        total += due;
    }
    // the device-side step counts of the layers that took the step advance with one launch
    if (!ls->clocks.empty() &&
        sc::launch_tick(ls->clocks.data(), (int)ls->clocks.size(), static_cast<hipStream_t>(stream)) != hipSuccess)
        return SC_ERR_DEVICE;
    if (st != SC_OK) return st;
    if (n_due) *n_due = total;
    return SC_OK;
}

sc_status sc_layers_note_replays(sc_layers* ls, int32_t k, int32_t* n_due) {
    if (!ls || k < 0) return SC_ERR_INVALID_ARG;
    for (const sc_cache* h : ls->layer) {  // checked for every layer before any layer advances
        if (!h->ragged || !h->device_clock || h->step == 0) return SC_ERR_STATE;
        for (int b = 0; b < h->cfg.batch; ++b)
            if (h->last_active[b] && h->ns[b] + k > h->n_trig) return SC_ERR_FULL;
    }
    int32_t total = 0;
    for (sc_cache* h : ls->layer) {
        int32_t due = 0;
        const sc_status st = sc_cache_note_replays(h, k, &due);
        if (st != SC_OK) return st;
        total += due;
    }
    if (n_due) *n_due = total;
    return SC_OK;
}

sc_status sc_layers_steps_until_due(const sc_layers* ls, const uint8_t* active, int32_t* steps) {
    if (!ls || ls->layer.empty() || !steps) return SC_ERR_INVALID_ARG;
    int32_t least = INT32_MAX;
    for (const sc_cache* h : ls->layer) {
        int32_t k = 0;
        const sc_status st = sc_steps_until_due(h, active, &k);
        if (st != SC_OK) return st;
        least = std::min(least, k);
    }
    *steps = least;
    return SC_OK;
}

sc_status sc_layers_compress(sc_layers* ls, int32_t* n_compressed, void* stream) {
    if (!ls) return SC_ERR_INVALID_ARG;
    int32_t count = 0;
    for (sc_cache* h : ls->layer) {
        bool due = false;
        if (h->ragged) {
            for (int b = 0; b < h->cfg.batch; ++b) due = due || h->ns[b] == h->n_trig;
        } else {
            due = h->n == h->n_trig;
        }
        if (!due) continue;
        const sc_status st = h->ragged ? sc_compress_ragged(h, nullptr, nullptr, stream)
                                       : sc_compress(h, nullptr, nullptr, stream);
        if (st != SC_OK) return st;
        ++count;
    }
    if (n_compressed) *n_compressed = count;
    return count ? SC_OK : SC_ERR_STATE;
}

void sc_layers_destroy(sc_layers* ls) {
    if (!ls) return;
    for (sc_cache* h : ls->layer) sc_cache_destroy(h);
    delete ls;
}

const char* sc_status_str(sc_status s) {
    switch (s) {
        case SC_OK: return "ok";
        case SC_ERR_INVALID_ARG: return "invalid argument";
        case SC_ERR_WORKSPACE: return "workspace too small or misaligned";
        case SC_ERR_FULL: return "cache full: a compression is due";
        case SC_ERR_STATE: return "call not legal in the current cache state";
        case SC_ERR_UNSUPPORTED: return "configuration not supported by this build";
        case SC_ERR_DEVICE: return "kernel launch failed";
        case SC_ERR_SCRATCH: return "cache needs more scratch than the library's static array holds";
        case SC_ERR_HOST_MEMORY: return "out of host memory";
    }
    return "unknown status";
}

}  // extern "C"
