// Decode-step kernels for gfx950: row append (Alg. 1 "model update") and the budgeted
// attention estimator of Sec. 4.1 with the Alg. 2 importance record updated in the softmax
// epilogue (the online variant of Sec. 4.1 "Overhead Tradeoff").
//
// One workgroup owns one (sequence, head) unit and does the whole step for it in a single
// launch: the new row is taken from k_new/v_new (quantised first for 4-bit storage), written
// to its slot and attended to from registers / LDS, so nothing is read back from a slot
// written in the same launch.  K and V rows already resident are streamed exactly once,
// together, with 16-byte loads per lane; a row of 16*LPR bytes is spread over LPR adjacent
// lanes, so one wave instruction fetches 64/LPR whole rows (1 KiB, fully coalesced).  Each
// lane group keeps a running softmax (max, sum, weighted value partial) that is rescaled only
// when the maximum moves; raw scores are parked in LDS so that, once the unit's global max
// and sum are known, the epilogue can form every probability, test it against the
// threshold, bump the counters and (optionally) dump the probabilities.
#include "quant.hpp"
#include "sc_kernels.hpp"

#include <type_traits>

namespace sc {
namespace {

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over the LPR adjacent lanes that share a row; every lane ends with the same bits.
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
    if constexpr (LPR >= 2) v += dpp_f32<0xB1>(v);   // quad_perm [1,0,3,2]
    if constexpr (LPR >= 4) v += dpp_f32<0x4E>(v);   // quad_perm [2,3,0,1]
    if constexpr (LPR >= 8) v += dpp_f32<0x141>(v);  // row_half_mirror
    if constexpr (LPR >= 16) v += dpp_f32<0x140>(v); // row_mirror
    if constexpr (LPR >= 32) v += __shfl_xor(v, 16);
    return v;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct AttnArgs {
    const void* q;
    const void* k_new;
    const void* v_new;
    long in_stride;  // elements between units in q, k_new and v_new
    const void* K;
    const void* V;
    const void* K_meta;
    const void* V_meta;
    int32_t* pos;
    int pos_value;
    void* out;
    long out_stride;
    float* probs;
    long probs_stride;  // floats between units in probs
    uint16_t* cnt;  // bucket mode: current bucket of unit 0; ring mode: this step's word plane
    long cnt_unit_stride;  // in 16-bit units
    uint32_t ring_bit;     // ring mode: this step's bit inside its word; 0 selects bucket mode
    int n, C;  // n counts the row appended by this launch
    float qk_log2, tau;
    int counted;
    void* q_keep;         // where unit 0's query of this step is kept (record rebuilt at
    long q_keep_stride;   // compression time), elements between units; null: not kept
    SeqSched seq;         // ragged batches (seq.off != null): the fields above that depend on the
    uint16_t* cnt_base;   // step are derived per sequence; cnt_base = bucket (ring word) 0 of unit 0
    long q_keep_slot_bytes;  // ragged + kept queries: q_keep = slot 0 of unit 0, slots this far apart
    unsigned long long* trace;  // diagnostics, normally null: [U][4] clock readings per workgroup
    int through;  // counters and outputs are written through the L2 (see store_through)
    // Units handed out by ticket (fp32/fp16 kernel, lock step, many units; null otherwise):
    // workgroups below n_static own the unit of their index, the n_ticket_wgs workgroups from
    // there on draw a number from *ticket and take unit n_static + number while it is below
    // n_tail (the rest return at once); the last to draw sets the counter back to zero.
    int32_t* ticket;
    int n_static, n_tail, n_ticket_wgs;
    // Very few units with long caches (fp32/fp16 kernel): `split` workgroups share a unit's rows.
    // Each publishes its share (acc[D], m, l; `share_stride` floats apart) and the raw scores of
    // its rows, then counts itself in arrive[u]; the last to arrive merges the shares and runs the
    // epilogue.  0: one workgroup per unit.
    int split, share_stride;
    float* shares;     // [U][8][share_stride]
    float* raw;        // [U][C] raw scores
    int32_t* arrive;   // [U], zero between launches
};

// Diagnostics (a.trace set): every workgroup reports when it started, when its K/V stream ended
// and when it finished (constant-rate 100 MHz clock) and where it ran (XCD, shader engine, CU).
struct TraceClock {
    long long t0 = 0, t1 = 0;
    __device__ __forceinline__ void start(const AttnArgs& a) {
        if (a.trace) t0 = wall_clock64();
    }
    __device__ __forceinline__ void streamed(const AttnArgs& a) {
        if (a.trace) t1 = wall_clock64();
    }
    __device__ __forceinline__ void finish(const AttnArgs& a, int u) {
        if (a.trace && threadIdx.x == 0) {
            unsigned long long* o = a.trace + 4 * (size_t)u;
            o[0] = (unsigned long long)t0;
            o[1] = (unsigned long long)t1;
            o[2] = (unsigned long long)wall_clock64();
            const unsigned hw = __builtin_amdgcn_s_getreg(GETREG_IMMED(31, 0, HW_ID));
            o[3] = ((unsigned long long)hw << 32) | __smid();
        }
    }
};

// Ragged batches: replace the lock-step scalars by those of unit u's sequence.  False when the
// sequence does not take part in this step (the workgroup then has nothing to do).
__device__ __forceinline__ bool seq_apply(AttnArgs& a, int u) {
    const int off = a.seq.off[u / a.seq.heads];
    if (off == kSeqIdle) return false;
    const int step = a.seq.step_dev ? *a.seq.step_dev + 1 : a.seq.step;
    const SeqStep s = sched_step(a.seq, (long)off + step);
    a.n = s.n;
    a.pos_value = s.pos_value;
    a.tau = s.tau;
    a.counted = s.counted;
    a.ring_bit = s.ring_bit;
    if (a.q_keep)  // step t keeps its query in ring slot (t-1) mod w
        a.q_keep = static_cast<char*>(a.q_keep) + (size_t)(s.pos_value % a.seq.w) * a.q_keep_slot_bytes;
    a.cnt = a.seq.W32 ? reinterpret_cast<uint16_t*>(reinterpret_cast<uint32_t*>(a.cnt_base) + (size_t)s.bucket * a.C)
                      : a.cnt_base + (size_t)s.bucket * a.C;
    return true;
}

template <typename T, int N>
union Frag {
    uint4 raw;
    T e[N];
};

// Running softmax of one lane group: m = max score so far (log2 domain), l = sum of
// exp2(score - m), acc = sum of exp2(score - m) * value fragment.
template <int N>
struct Running {
    float m, l, acc[N];
    __device__ __forceinline__ void init() {
        m = -INFINITY;
        l = 0.f;
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = 0.f;
    }
    // Account for one row with score s; returns its weight exp2(s - m) (0 when !valid).
    __device__ __forceinline__ float admit(float s, bool valid) {
        if (valid && s > m) {
            const float al = fast_exp2(m - s);
            l *= al;
#pragma unroll
            for (int i = 0; i < N; ++i) acc[i] *= al;
            m = s;
        }
        const float e = valid ? fast_exp2(s - m) : 0.f;
        l += e;
        return e;
    }
    // Merge with the lane `off` away (both lanes end with the merged state).
    __device__ __forceinline__ void merge_xor(int off) {
        const float mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
        const float mn = fmaxf(m, mo);
        const float sa = (m == mn) ? 1.0f : fast_exp2(m - mn);
        const float sb = (mo == mn) ? 1.0f : fast_exp2(mo - mn);
        l = l * sa + lo * sb;
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = acc[i] * sa + __shfl_xor(acc[i], off) * sb;
        m = mn;
    }
};

// Counter words: two 16-bit counters (slots 2i and 2i+1) per 32-bit word.  Each thread owns
// the words i = tid, tid + NT, ...; the first cnt_pf(NT) of them (enough for 768 resident
// rows, more with many threads) are fetched when the kernel starts so that their latency is
// hidden behind the K/V stream: a dependent load per word in the epilogue costs a full
// memory round trip each.
constexpr int cnt_pf(int nt) { return nt >= 384 ? 1 : 384 / nt; }

template <int NT>
__device__ __forceinline__ void prefetch_counters(const AttnArgs& a, int u, uint32_t (&pre)[cnt_pf(NT)]) {
    constexpr int CNT_PF = cnt_pf(NT);
    const uint32_t* cw = reinterpret_cast<const uint32_t*>(a.cnt + (size_t)u * a.cnt_unit_stride);
    const int per_word = a.ring_bit ? 1 : 2;  // slots covered by one 32-bit word
#pragma unroll
    for (int k = 0; k < CNT_PF; ++k) {
        const int i = threadIdx.x + k * NT;
        pre[k] = (a.counted && per_word * i < a.n) ? cw[i] : 0u;
    }
}

// The appended row, the counters and the outputs are results nobody reads again inside the
// launch.  A plain store leaves them in the XCD's L2 as dirty lines until they are displaced or
// the kernel's end writes them back; a device-scope store is written through at once, but its
// wave waits longer for the acknowledgement.  Measured on MI355X: a launch that writes much
// (9216 units x 562 rows: 17 MB per launch) runs 3 to 4.4% faster written through (counters
// and outputs 1.9 to 3.3%, the rows another 1.2%), launches that write little run up to 1.3%
// slower (2560 units x 347 rows, 3.7 MB), so the host chooses per launch.
__device__ __forceinline__ void store_through(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_through(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_through(_Float16* p, _Float16 v) {
    union { _Float16 h; unsigned short u; } c;
    c.h = v;
    __hip_atomic_store(reinterpret_cast<unsigned short*>(p), c.u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The probability epilogue with the update of the importance record (Alg. 2, kept online):
// p_j = exp2(s_j - M) / L for every resident slot, tested against the threshold.
// Bucket mode: two 16-bit counters per word, +1 where the probability is below the threshold.
// Ring mode: one 32-bit ring word per slot; this step's bit is set or cleared.
// The scores of all the prefetched words of a thread are read from LDS before any of them is
// used, whether or not the word lies below n (LDS holds C >= n scores and the partials behind
// them, so the read is in bounds; the value is then unused): behind a condition every read
// would be waited for on its own, one LDS round trip after the other.
template <int NT>
__device__ __forceinline__ void finish_counters(const AttnArgs& a, int u, const float* s_lds, float M, float invL,
                                                const uint32_t (&pre)[cnt_pf(NT)]) {
    constexpr int CNT_PF = cnt_pf(NT);
    const int tid = threadIdx.x;
    uint32_t* cw = reinterpret_cast<uint32_t*>(a.cnt + (size_t)u * a.cnt_unit_stride);
    const int n = a.n;
    if (a.ring_bit) {
        float* probs = a.probs ? a.probs + (size_t)u * a.probs_stride : nullptr;
        auto do_slot = [&](int j, uint32_t word, float score) {
            const float p = fast_exp2(score - M) * invL;
            if (probs) probs[j] = p;
            const uint32_t upd = (p < a.tau) ? (word | a.ring_bit) : (word & ~a.ring_bit);
            if (upd != word) {
                if (a.through) store_through(cw + j, upd); else cw[j] = upd;
            }
        };
        float sc[CNT_PF];
#pragma unroll
        for (int k = 0; k < CNT_PF; ++k) {
            const int j = tid + k * NT;
            sc[k] = s_lds[j < n ? j : 0];
        }
#pragma unroll
        for (int k = 0; k < CNT_PF; ++k) {
            const int j = tid + k * NT;
            if (j < n) do_slot(j, pre[k], sc[k]);
        }
        for (int j = tid + CNT_PF * NT; j < n; j += NT) do_slot(j, cw[j], s_lds[j]);
        return;
    }
    float2* probs = a.probs ? reinterpret_cast<float2*>(a.probs + (size_t)u * a.probs_stride) : nullptr;
    auto do_word = [&](int i, uint32_t word, float2 score) {
        const int j = 2 * i;  // j < n here; slot j+1 may be the first free one
        const float p0 = fast_exp2(score.x - M) * invL;
        const float p1 = (j + 1 < n) ? fast_exp2(score.y - M) * invL : 0.f;
        if (probs) probs[i] = make_float2(p0, p1);
        const uint32_t inc = (p0 < a.tau ? 1u : 0u) | ((j + 1 < n && p1 < a.tau) ? 0x10000u : 0u);
        if (a.counted && inc) {
            if (a.through) store_through(cw + i, word + inc); else cw[i] = word + inc;
        }
    };
    const float2* s2 = reinterpret_cast<const float2*>(s_lds);  // slots 2i, 2i+1
    float2 sc[CNT_PF];
#pragma unroll
    for (int k = 0; k < CNT_PF; ++k) {
        const int i = tid + k * NT;
        sc[k] = s2[2 * i < n ? i : 0];
    }
#pragma unroll
    for (int k = 0; k < CNT_PF; ++k) {
        const int i = tid + k * NT;
        if (2 * i < n) do_word(i, pre[k], sc[k]);
    }
    for (int i = tid + CNT_PF * NT; 2 * i < n; i += NT) do_word(i, a.counted ? cw[i] : 0u, s2[i]);
}

// Shared tail of the attention kernels: combine the partials, write `out`, then the
// probability epilogue.  NT = threads of the workgroup, NP = number of partial (m, l, acc[D])
// triples published in LDS.
template <typename TOut, int D, int NT, int NP>
__device__ __forceinline__ void finish_unit(const AttnArgs& a, int u, const float* s_lds,
                                            const float* part_m, const float* part_l,
                                            const float* part_acc, const uint32_t (&pre)[cnt_pf(NT)]) {
    const int tid = threadIdx.x;
    float M = part_m[0];
#pragma unroll
    for (int w = 1; w < NP; ++w) M = fmaxf(M, part_m[w]);
    float Lsum = 0.f;
#pragma unroll
    for (int w = 0; w < NP; ++w) Lsum += part_l[w] * fast_exp2(part_m[w] - M);
    const float invL = 1.0f / Lsum;
    if (a.out) {
        for (int ch = tid; ch < D; ch += NT) {
            float o = 0.f;
#pragma unroll
            for (int w = 0; w < NP; ++w) o += part_acc[w * D + ch] * fast_exp2(part_m[w] - M);
            TOut* dst = (TOut*)a.out + (size_t)u * a.out_stride + ch;
            if (a.through) store_through(dst, (TOut)(o * invL)); else *dst = (TOut)(o * invL);
        }
    }
    finish_counters<NT>(a, u, s_lds, M, invL, pre);
}

// ---------------------------------------------------------------------------------------
// fp32 / fp16 rows.
// ---------------------------------------------------------------------------------------
// K/V rows are read exactly once per launch: stream them with non-temporal loads so that they
// do not displace anything in the cache hierarchy (measurably faster than plain loads here).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* base, uint32_t byte_off) {
    const u32x4 v = __builtin_nontemporal_load(
        reinterpret_cast<const u32x4*>(static_cast<const char*>(base) + byte_off));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// 16 bytes per lane, written through like store_through (there is no 128-bit atomic store to
// express it with).
__device__ __forceinline__ void store_through16(void* p, const uint4& v) {
    const u32x4 d = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(d) : "memory");
}

// Loads of what another workgroup of this launch, possibly on another XCD, has published with
// store_through: device-scope loads, which are not served from this XCD's own copy of the line.
__device__ __forceinline__ float load_published(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// (At most 80 scalar registers: with the 90 the split variant would otherwise take, two workgroups
// of 16 waves no longer fit on a CU -- measured: the second 256 workgroups of a launch then
// start only as the first ones leave.)
template <typename T, int D, int NW, int UNR, bool SPLIT>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_num_sgpr(80))) attn_rows_kernel(AttnArgs a) {
    TraceClock clk;
    clk.start(a);
    // SPLIT: a.split consecutive workgroups share one unit, each taking a contiguous range of rows
    const int wg = SPLIT ? (int)blockIdx.x / a.split : (int)blockIdx.x;
    const int part = SPLIT ? (int)blockIdx.x - wg * a.split : 0;
    if (a.seq.off && !seq_apply(a, wg)) return;
    constexpr int EPL = 16 / (int)sizeof(T);  // elements per lane
    constexpr int LPR = D / EPL;              // lanes per row
    constexpr int RPW = 64 / LPR;             // rows per wave load
    constexpr int CHUNK = RPW * UNR;          // rows a wave fetches per batch of loads
    constexpr int STRIDE = NW * CHUNK;
    constexpr uint32_t ROWB = D * sizeof(T);
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* s_lds = reinterpret_cast<float*>(smem_raw);
    float* part_m = s_lds + a.C;
    float* part_l = part_m + NW;
    float* part_acc = part_l + NW;

    // Workgroup i runs on XCD i mod 8 whatever the XCDs' progress, and the XCDs are not equally
    // fast (measured: the odd ones about 4% behind on 9216 units), so with one unit per workgroup
    // index the launch lasts as long as the slowest XCD.  The last units are therefore not tied
    // to a workgroup index: twice as many workgroups as there are such units draw tickets, an XCD
    // that gets to its ticket workgroups early takes more of the units, and workgroups that draw
    // when none is left return.
    int u = wg;
    if (!SPLIT && a.ticket && u >= a.n_static) {
        __shared__ int drawn;
        if (threadIdx.x == 0) {
            const int k = __hip_atomic_fetch_add(a.ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (k == a.n_ticket_wgs - 1)  // every workgroup has drawn: ready for the next launch
                __hip_atomic_store(a.ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            drawn = k;
        }
        __syncthreads();
        const int k = __builtin_amdgcn_readfirstlane(drawn);
        if (k >= a.n_tail) return;
        u = a.n_static + k;
    }
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = lane / LPR, c = lane % LPR;
    const int nc = a.n - 1;  // rows resident before this step; the new row goes to slot nc
    // unit-uniform bases (scalar registers) + 32-bit per-lane byte offsets
    char* Kb = (char*)a.K + (size_t)u * a.C * ROWB;
    char* Vb = (char*)a.V + (size_t)u * a.C * ROWB;
    const uint32_t lane_off = (uint32_t)g * ROWB + (uint32_t)c * 16u;
    const size_t in_off = (size_t)u * a.in_stride + c * EPL;
    using F = Frag<T, EPL>;

    // Everything the kernel needs from memory up front is requested before anything is
    // waited for: q, the new row (its owner only), the counters.
    F qr;
    qr.raw = *reinterpret_cast<const uint4*>((const T*)a.q + in_off);
    // Rows [lo, hi) are this workgroup's (all resident rows unless the unit is split; ranges start
    // at multiples of 32 rows so that no two workgroups write scores into one 128-byte line); the
    // new row belongs to the workgroup that has the last range.
    int lo = 0, hi = nc;
    if constexpr (SPLIT) {
        const int per = ((nc + a.split - 1) / a.split + 31) / 32 * 32;
        lo = part * per < nc ? part * per : nc;
        hi = lo + per < nc ? lo + per : nc;
    }
    const bool last_part = !SPLIT || part == a.split - 1;
    const bool owner = (wv == 0) && (g == 0) && last_part;  // Alg. 1 model update: who holds the new row
    if (a.q_keep && owner)  // Alg. 2 as printed replays this query at the next compressions
        *reinterpret_cast<uint4*>((T*)a.q_keep + (size_t)u * a.q_keep_stride + c * EPL) = qr.raw;
    F k_own, v_own;
    k_own.raw = make_uint4(0, 0, 0, 0);
    v_own.raw = make_uint4(0, 0, 0, 0);
    if (owner) {
        k_own.raw = *reinterpret_cast<const uint4*>((const T*)a.k_new + in_off);
        v_own.raw = *reinterpret_cast<const uint4*>((const T*)a.v_new + in_off);
    }
    uint32_t cpre[cnt_pf(NW * 64)];
    prefetch_counters<NW * 64>(a, u, cpre);

    float qf[EPL];
    Running<EPL> run;
    run.init();
    auto take_row = [&](const F& kr, const F& vr, int j, bool valid) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) s = fmaf((float)kr.e[i], qf[i], s);
        s = group_sum<LPR>(s);
        if (valid && c == 0) s_lds[j] = s;
        const float e = run.admit(s, valid);
#pragma unroll
        for (int i = 0; i < EPL; ++i) run.acc[i] = fmaf(e, (float)vr.e[i], run.acc[i]);
    };
    // Full chunks need no bounds checks; one ragged chunk at most is handled with masks.
    auto load_full = [&](F (&kr)[UNR], F (&vr)[UNR], int base) {
        const uint32_t off = (uint32_t)base * ROWB + lane_off;
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            kr[x].raw = load_stream16(Kb, off + (uint32_t)x * (RPW * ROWB));
            vr[x].raw = load_stream16(Vb, off + (uint32_t)x * (RPW * ROWB));
        }
    };
    auto take_full = [&](const F (&kr)[UNR], const F (&vr)[UNR], int base) {
#pragma unroll
        for (int x = 0; x < UNR; ++x) take_row(kr[x], vr[x], base + x * RPW + g, true);
    };

#pragma unroll
    for (int i = 0; i < EPL; ++i) qf[i] = (float)qr.e[i] * a.qk_log2;
    int base = lo + wv * CHUNK;
    for (; base + CHUNK <= hi; base += STRIDE) {
        F kr[UNR], vr[UNR];
        load_full(kr, vr, base);
        take_full(kr, vr, base);
    }
    if (base < hi) {  // ragged tail of this wave
        F kr[UNR], vr[UNR];
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            const int j = base + x * RPW + g;
            const uint32_t off = (j < hi ? (uint32_t)j : 0u) * ROWB + (uint32_t)c * 16u;
            kr[x].raw = load_stream16(Kb, off);
            vr[x].raw = load_stream16(Vb, off);
        }
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            const int j = base + x * RPW + g;
            take_row(kr[x], vr[x], j, j < hi);
        }
    }
    if (owner) {
        if (a.through) {
            store_through16(Kb + (size_t)nc * ROWB + c * 16, k_own.raw);
            store_through16(Vb + (size_t)nc * ROWB + c * 16, v_own.raw);
        } else {
            *reinterpret_cast<uint4*>(Kb + (size_t)nc * ROWB + c * 16) = k_own.raw;
            *reinterpret_cast<uint4*>(Vb + (size_t)nc * ROWB + c * 16) = v_own.raw;
        }
        if (c == 0) a.pos[(size_t)u * a.C + nc] = a.pos_value;
    }
    if (wv == 0 && last_part) take_row(k_own, v_own, nc, owner);
    clk.streamed(a);

#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) run.merge_xor(off);
    if (g == 0) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) part_acc[wv * D + c * EPL + i] = run.acc[i];
        if (c == 0) {
            part_m[wv] = run.m;
            part_l[wv] = run.l;
        }
    }
    __syncthreads();
    if constexpr (SPLIT) {
        static_assert(NW >= 8, "the shares of up to 8 workgroups are merged in the per-wave LDS arrays");
        __shared__ int arrived;
        const int tid = threadIdx.x;
        // 1. Publish this workgroup's share (its waves merged) and the raw scores of its rows,
        //    written through to where every XCD sees them.
        float M = part_m[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, part_m[w]);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) L += part_m[w] == -INFINITY ? 0.f : part_l[w] * fast_exp2(part_m[w] - M);
        float* share = a.shares + ((size_t)u * 8 + part) * a.share_stride;
        for (int ch = tid; ch < D; ch += NW * 64) {
            float o = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w)
                o += part_m[w] == -INFINITY ? 0.f : part_acc[w * D + ch] * fast_exp2(part_m[w] - M);
            store_through(share + ch, o);
        }
        if (tid == 0) {
            store_through(share + D, M);  // -inf when the range holds no row
            store_through(share + D + 1, L);
        }
        float* raw = a.raw + (size_t)u * a.C;
        for (int j = lo + tid; j < hi; j += NW * 64) store_through(raw + j, s_lds[j]);
        if (last_part && tid == 0) store_through(raw + nc, s_lds[nc]);
        // 2. Once all of it has arrived in memory, count this workgroup in; all but the last leave.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const int k = __hip_atomic_fetch_add(a.arrive + u, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (k == a.split - 1)  // ready for the next launch
                __hip_atomic_store(a.arrive + u, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            arrived = k;
        }
        __syncthreads();
        if (__builtin_amdgcn_readfirstlane(arrived) != a.split - 1) return;
        // 3. The last to arrive: fetch the others' scores and all shares, then finish the unit as
        //    a workgroup that had streamed all of it would (shares take the place of waves).
        for (int j = tid; j < a.n; j += NW * 64)
            if (j < lo || (j >= hi && !(last_part && j == nc))) s_lds[j] = load_published(raw + j);
        for (int i = tid; i < 8 * D; i += NW * 64) {
            const int p = i / D, ch = i - p * D;
            part_acc[i] = p < a.split ? load_published(a.shares + ((size_t)u * 8 + p) * a.share_stride + ch) : 0.f;
        }
        if (tid < 8) {
            const float* sh = a.shares + ((size_t)u * 8 + tid) * a.share_stride;
            part_m[tid] = tid < a.split ? load_published(sh + D) : -INFINITY;
            part_l[tid] = tid < a.split ? load_published(sh + D + 1) : 0.f;
        }
        __syncthreads();
        finish_unit<T, D, NW * 64, 8>(a, u, s_lds, part_m, part_l, part_acc, cpre);
    } else {
        finish_unit<T, D, NW * 64, NW>(a, u, s_lds, part_m, part_l, part_acc, cpre);
        clk.finish(a, u);
    }
}

// ---------------------------------------------------------------------------------------
// 4-bit rows: 16 bytes of codes (32 channels) per lane, D/32 lanes per row, one
// (scale, zero) fp16 pair per 64 channels.  value = code*scale + zero, so
//   <q, k>   = sum_groups scale_g * sum_c q_c*code_c + zero_g * sum_c q_c
//   sum_j p_j v_j[c] = sum_j (p_j*scale_jg) * code_jc + sum_j p_j*zero_jg
// ---------------------------------------------------------------------------------------
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// Two 4-bit codes of a 32-bit word, bits [lo, lo+4) of each 16-bit half, as a pair of fp16
// numbers without any int->float conversion: OR-ing the bits into the mantissa of 1024.0
// (0x6400, whose ulp is 1) gives 1024 + code for lo = 0 and 1024 + 16*code for lo = 4.
// The masks live in vector registers and the constant in a scalar one (made opaque to the
// compiler once per kernel), because the single-instruction form (w & mask) | magic takes no
// literals and one scalar operand; written as plain C so that the compiler, not inline
// assembly, emits it and inserts the wait states a matrix instruction reading the result needs.
struct NibbleConsts {
    uint32_t lo, hi, magic;
    __device__ __forceinline__ void init() {
        asm volatile("v_mov_b32 %0, 0x000F000F" : "=v"(lo));
        asm volatile("v_mov_b32 %0, 0x00F000F0" : "=v"(hi));
        asm volatile("s_mov_b32 %0, 0x64006400" : "=s"(magic));
    }
};

__device__ __forceinline__ half2_t nibble_pair(uint32_t w, uint32_t mask, uint32_t magic) {
    return __builtin_bit_cast(half2_t, (w & mask) | magic);
}

// The eight codes of word w as four such pairs: {n0,n4}, {n1,n5}x16, {n2,n6}, {n3,n7}x16.
__device__ __forceinline__ void unpack8(uint32_t w, half2_t (&h)[4], const NibbleConsts& nk) {
    const uint32_t t = w >> 8;
    h[0] = nibble_pair(w, nk.lo, nk.magic);
    h[1] = nibble_pair(w, nk.hi, nk.magic);
    h[2] = nibble_pair(t, nk.lo, nk.magic);
    h[3] = nibble_pair(t, nk.hi, nk.magic);
}

template <int CTRL>
__device__ __forceinline__ float dpp_max(float v) { return fmaxf(v, dpp_f32<CTRL>(v)); }

// DPP row_ror:n (rotate right by n lanes inside each row of 16 lanes).
#define SC_ROW_ROR(n) (0x120 + (n))

// Sum / max over the lane groups that share a row of 16 lanes (groups are LPR lanes wide, so
// lanes LPR, 2*LPR, ... apart hold the same channels of different cache rows).
template <int LPR>
__device__ __forceinline__ float row_groups_sum(float v) {
    if constexpr (LPR <= 2) v += dpp_f32<SC_ROW_ROR(2)>(v);
    if constexpr (LPR <= 4) v += dpp_f32<SC_ROW_ROR(4)>(v);
    if constexpr (LPR <= 8) v += dpp_f32<SC_ROW_ROR(8)>(v);
    return v;
}
template <int LPR>
__device__ __forceinline__ float row_groups_max(float v) {
    if constexpr (LPR <= 2) v = dpp_max<SC_ROW_ROR(2)>(v);
    if constexpr (LPR <= 4) v = dpp_max<SC_ROW_ROR(4)>(v);
    if constexpr (LPR <= 8) v = dpp_max<SC_ROW_ROR(8)>(v);
    return v;
}

// The kernel is bound by plain ALU work as much as by HBM (256 codes per 144 bytes), so the
// inner loop avoids per-code conversions: codes become fp16 pairs with one AND-OR each, the
// key side uses the packed fp16 dot product with fp32 accumulation, the value side the mixed
// fp16 x fp32 fused multiply-add; the +1024 offsets of the pairs and the zero points are
// folded out of the loop.  All lane groups of a 16-lane row share one running maximum, so
// their partial sums merge with plain DPP adds.
template <int D, int NW, int UNR>
__global__ void __launch_bounds__(NW * 64) attn_i4_kernel(AttnArgs a) {
    TraceClock clk;
    clk.start(a);
    if (a.seq.off && !seq_apply(a, blockIdx.x)) return;
    constexpr int LPR = D / 32;   // lanes per cache row (16 bytes = 32 codes per lane)
    constexpr int RPW = 64 / LPR; // cache rows per wave load
    constexpr int GPR = D / 64;   // quantisation groups per cache row
    constexpr uint32_t ROWB = D / 2;  // bytes of codes per cache row
    constexpr int NP = NW * 4;        // one partial per 16-lane row
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* s_lds = reinterpret_cast<float*>(smem_raw);
    float* part_m = s_lds + a.C;
    float* part_l = part_m + NP;
    float* part_acc = part_l + NP;
    __shared__ __align__(16) unsigned char new_codes[2][ROWB];  // [0] key row, [1] value row
    __shared__ uint32_t new_meta[2][GPR];

    const int u = blockIdx.x;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = lane / LPR, c = lane % LPR;
    const int gi = c / 2;  // 64-channel group this lane's 32 channels fall in
    const int nc = a.n - 1;
    NibbleConsts nk;
    nk.init();
    unsigned char* Kb = (unsigned char*)a.K + (size_t)u * a.C * ROWB;
    unsigned char* Vb = (unsigned char*)a.V + (size_t)u * a.C * ROWB;
    uint32_t* Kmb = (uint32_t*)a.K_meta + (size_t)u * a.C * GPR;
    uint32_t* Vmb = (uint32_t*)a.V_meta + (size_t)u * a.C * GPR;

    // Alg. 1 model update: wave 0 quantises the key row, wave 1 (wave 0 again when the
    // workgroup is a single wave) the value row.
    for (int which = wv; which < 2; which += NW) {
        const _Float16* src = (const _Float16*)(which ? a.v_new : a.k_new) + (size_t)u * a.in_stride;
        const float x0 = lane < D / 2 ? (float)src[2 * lane] : 0.f;
        const float x1 = lane < D / 2 ? (float)src[2 * lane + 1] : 0.f;
        quantise_row<D>(x0, x1, (which ? Vb : Kb) + (size_t)nc * ROWB,
                        (which ? Vmb : Kmb) + (size_t)nc * GPR, new_codes[which], new_meta[which], lane);
        if (which == 0 && lane == 0) a.pos[(size_t)u * a.C + nc] = a.pos_value;
    }
    uint32_t cpre[cnt_pf(NW * 64)];
    prefetch_counters<NW * 64>(a, u, cpre);

    // q of this lane's 32 channels as fp16 pairs matching unpack8, and the constants that
    // cancel the +1024 of every pair: qa0/qb0 = -1024 * (sum of q over the channels that go
    // through the plain / the x16 pairs); qsum for the zero point.
    half2_t qh[16];
    float qa0, qb0, qsum;
    {
        const _Float16* qu = (const _Float16*)a.q + (size_t)u * a.in_stride + c * 32;
        float sa = 0.f, sb = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            Frag<_Float16, 8> qr;
            qr.raw = *reinterpret_cast<const uint4*>(qu + w * 8);
            if (a.q_keep && wv == 0 && g == 0)  // kept for the replay at the next compressions
                *reinterpret_cast<uint4*>((_Float16*)a.q_keep + (size_t)u * a.q_keep_stride + c * 32 + w * 8) = qr.raw;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                qh[w * 4 + k] = half2_t{qr.e[k], qr.e[k + 4]};
                const float pair = (float)qr.e[k] + (float)qr.e[k + 4];
                if (k & 1) sb += pair; else sa += pair;
            }
        }
        qa0 = -1024.f * sa;
        qb0 = -1024.f * sb;
        qsum = sa + sb;
    }
    // Running softmax shared by the 16 lanes of a row: m, and per lane l (its own cache rows),
    // acc (32 channels, still carrying the pair offsets), wsum (sum of weight*scale, to remove
    // those offsets) and zacc (sum of weight*zero).
    float m = -INFINITY, l = 0.f, wsum = 0.f, zacc = 0.f, acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.f;

    // One cache row per lane group.  `masked` (a compile-time tag) is only true for the one
    // ragged tile at the end of the cache and for the new row, where some groups hold no row.
    auto take_row = [&](auto masked, const uint4& kr, const uint4& vr, uint32_t kmw, uint32_t vmw, int j,
                        bool valid) {
        constexpr bool MASKED = decltype(masked)::value;
        const uint32_t kw[4] = {kr.x, kr.y, kr.z, kr.w};
        float da = qa0, db = qb0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            half2_t h[4];
            unpack8(kw[w], h, nk);
            da = __builtin_amdgcn_fdot2(h[0], qh[w * 4 + 0], da, false);
            db = __builtin_amdgcn_fdot2(h[1], qh[w * 4 + 1], db, false);
            da = __builtin_amdgcn_fdot2(h[2], qh[w * 4 + 2], da, false);
            db = __builtin_amdgcn_fdot2(h[3], qh[w * 4 + 3], db, false);
        }
        MetaWord km, vm;
        km.u32 = kmw;
        vm.u32 = vmw;
        const float dotc = fmaf(db, 0.0625f, da);  // sum of q*code over this lane's channels
        float s = group_sum<LPR>(fmaf((float)km.h[0], dotc, (float)km.h[1] * qsum)) * a.qk_log2;
        if constexpr (MASKED) {
            if (valid && c == 0) s_lds[j] = s;
            s = valid ? s : -INFINITY;
        } else {
            s_lds[j] = s;  // the LPR lanes of a group store the same value to the same address
        }
        // The running maximum moves rarely: only when some lane of the wave sees a score above
        // its row's maximum is the row maximum formed (same decision in all 16 lanes of a row).
        if (__builtin_amdgcn_ballot_w64(s > m) != 0ull) {
            const float smax = row_groups_max<LPR>(s);
            if (smax > m) {
                const float al = fast_exp2(m - smax);
                l *= al;
                wsum *= al;
                zacc *= al;
#pragma unroll
                for (int i = 0; i < 32; ++i) acc[i] *= al;
                m = smax;
            }
        }
        float e = fast_exp2(s - m);
        if constexpr (MASKED) e = valid ? e : 0.f;
        l += e;
        const float es = e * (float)vm.h[0];
        const float es16 = es * 0.0625f;
        wsum += es;
        zacc = fmaf(e, (float)vm.h[1], zacc);
        const uint32_t vw[4] = {vr.x, vr.y, vr.z, vr.w};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            half2_t h[4];
            unpack8(vw[w], h, nk);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float wk = (k & 1) ? es16 : es;
                acc[w * 8 + k] = fmaf((float)h[k][0], wk, acc[w * 8 + k]);
                acc[w * 8 + k + 4] = fmaf((float)h[k][1], wk, acc[w * 8 + k + 4]);
            }
        }
    };
    using Full = std::integral_constant<bool, false>;
    using Ragged = std::integral_constant<bool, true>;

    // A ring of UNR tiles (RPW cache rows each) per wave: as soon as a tile has been consumed
    // its registers are refilled with the tile UNR positions ahead, so UNR-1 tiles of loads
    // stay in flight behind the arithmetic.  Wave w owns tiles w, w+NW, w+2NW, ...  Every
    // request is unconditional and has the same form (rows beyond the last resident one repeat
    // that row: in bounds, finite, never used), so that the number of loads issued after the
    // ones a tile waits for is a compile-time constant and a wait covers that tile only.
    const int ntiles = (nc + RPW - 1) / RPW;
    const int nloc = ntiles > wv ? (ntiles - wv + NW - 1) / NW : 0;  // tiles of this wave
    uint4 kr[UNR], vr[UNR];
    uint32_t km[UNR], vm[UNR];
    int next_row = wv * RPW + g;  // row this lane group holds in the tile requested next
    auto request = [&](int x) {
        const uint32_t jj = (uint32_t)(next_row < nc ? next_row : nc - 1);
        kr[x] = load_stream16(Kb, jj * ROWB + (uint32_t)c * 16u);
        vr[x] = load_stream16(Vb, jj * ROWB + (uint32_t)c * 16u);
        km[x] = Kmb[jj * GPR + gi];
        vm[x] = Vmb[jj * GPR + gi];
        next_row += NW * RPW;
    };
    if (nloc > 0) {
#pragma unroll
        for (int x = 0; x < UNR; ++x) request(x);
    }
    // All rounds but the last hold complete tiles only (a later tile of this wave exists, so
    // every row of these is resident) and refill each slot; the last round checks both.
    const int rounds = (nloc + UNR - 1) / UNR;
    int li = 0;
    for (int rr = 0; rr + 1 < rounds; ++rr, li += UNR) {
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            take_row(Full{}, kr[x], vr[x], km[x], vm[x], (wv + (li + x) * NW) * RPW + g, true);
            request(x);
        }
    }
    if (nloc > 0) {
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            if (li + x < nloc) {
                const int j = (wv + (li + x) * NW) * RPW + g;
                take_row(Ragged{}, kr[x], vr[x], km[x], vm[x], j, j < nc);
            }
        }
    }
    clk.streamed(a);
    __syncthreads();  // the quantised new row is in LDS
    if (wv == 0) {
        const uint4 kr = *reinterpret_cast<const uint4*>(&new_codes[0][c * 16]);
        const uint4 vr = *reinterpret_cast<const uint4*>(&new_codes[1][c * 16]);
        take_row(Ragged{}, kr, vr, new_meta[0][gi], new_meta[1][gi], nc, g == 0);
    }
    // Remove the pair offsets (1024*weight, resp. 1024*weight/16), add the zero points, then
    // add up the lane groups of each 16-lane row (they share m, so plain sums).
    {
        const float off_a = 1024.f * wsum, off_b = 64.f * wsum;
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float o = (k & 1) ? off_b : off_a;
                acc[w * 8 + k] = row_groups_sum<LPR>(acc[w * 8 + k] - o + zacc);
                acc[w * 8 + k + 4] = row_groups_sum<LPR>(acc[w * 8 + k + 4] - o + zacc);
            }
        l = row_groups_sum<LPR>(l);
    }
    if ((lane & 15) < LPR) {
        const int p = wv * 4 + (lane >> 4);
#pragma unroll
        for (int i = 0; i < 32; ++i) part_acc[p * D + c * 32 + i] = acc[i];
        if (c == 0) {
            part_m[p] = m;
            part_l[p] = l;
        }
    }
    __syncthreads();
    finish_unit<_Float16, D, NW * 64, NP>(a, u, s_lds, part_m, part_l, part_acc, cpre);
    clk.finish(a, u);
}

// ---------------------------------------------------------------------------------------
// 4-bit rows, head_dim 128, key side on the matrix cores.
//
// The 4-bit kernel above is limited by vector-ALU issue, not by HBM.  Here the q.k products
// move to MFMA (v_mfma_f32_16x16x32_f16), which runs beside the vector ALU: a tile of 16 cache
// rows is the B operand (lane l = row l%16, 16 bytes = channels 32*(l/16) .. +31; one 32-bit
// word of codes becomes the 8 fp16 values a lane owes one MFMA with four AND-ORs), q is the A
// operand, laid out once per launch.  The M dimension, useless for a single query, separates
// the two quantisation groups of a row (output row 0: channels 0-63, row 1: channels 64-127)
// and repeats them for every 16-lane row, so each lane finds both sums for its own cache row
// in its accumulator registers and no shuffle is needed.  The value side stays on the vector
// ALU (its contraction runs over cache rows, which no lane holds contiguously).
// ---------------------------------------------------------------------------------------
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

union CodeOctet {  // the 8 codes of one 32-bit word as fp16: {n0, n4, 16*n1, 16*n5, n2, n6, 16*n3, 16*n7} + 1024
    half2_t h2[4];
    half8_t h8;
};

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) { return v + dpp_f32<CTRL>(v); }

// Sum / max over the 16 lanes of a DPP row (every lane ends with the result).
__device__ __forceinline__ float row16_sum(float v) {
    v = dpp_add<0xB1>(v);
    v = dpp_add<0x4E>(v);
    v = dpp_add<0x141>(v);
    return dpp_add<0x140>(v);
}
__device__ __forceinline__ float row16_max(float v) {
    v = dpp_max<0xB1>(v);
    v = dpp_max<0x4E>(v);
    v = dpp_max<0x141>(v);
    return dpp_max<0x140>(v);
}

// The waves that share a SIMD do not get equal shares of its issue slots by themselves (one of
// them can end a third later than another although their work is identical), and a launch is
// only over when its slowest wave is.  Each wave therefore walks through the priority levels
// as it advances, offset by its slot on the SIMD, so that over any few tiles every wave has
// held every level.
__device__ __forceinline__ void rotate_priority(int k) {
    switch (k % 3) {
        case 0: __builtin_amdgcn_s_setprio(0); break;
        case 1: __builtin_amdgcn_s_setprio(1); break;
        default: __builtin_amdgcn_s_setprio(2); break;
    }
}

template <int NW, int UNR>
__global__ void __launch_bounds__(NW * 64) attn_i4_mfma_kernel(AttnArgs a) {
    TraceClock clk;
    clk.start(a);
    if (a.seq.off && !seq_apply(a, blockIdx.x)) return;
    constexpr int D = 128;
    constexpr int RPW = 16;           // cache rows per tile (one wave load)
    constexpr int GPR = 2;            // quantisation groups per cache row
    constexpr uint32_t ROWB = D / 2;  // bytes of codes per cache row
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* s_lds = reinterpret_cast<float*>(smem_raw);
    float* part_m = s_lds + a.C;
    float* part_l = part_m + NW;
    float* part_acc = part_l + NW;
    __shared__ __align__(16) unsigned char new_codes[2][ROWB];  // [0] key row, [1] value row
    __shared__ __align__(8) uint32_t new_meta[2][GPR];

    const int u = blockIdx.x;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int r = lane & 15;   // cache row inside a tile
    const int kb = lane >> 4;  // which 32 channels of the row this lane holds
    const int gi = kb >> 1;    // their quantisation group
    const int nc = a.n - 1;
    NibbleConsts nk;
    nk.init();
    unsigned char* Kb = (unsigned char*)a.K + (size_t)u * a.C * ROWB;
    unsigned char* Vb = (unsigned char*)a.V + (size_t)u * a.C * ROWB;
    uint32_t* Kmb = (uint32_t*)a.K_meta + (size_t)u * a.C * GPR;
    uint32_t* Vmb = (uint32_t*)a.V_meta + (size_t)u * a.C * GPR;

    // Everything small the kernel needs is requested first (the raw new row, q, the counter
    // words), then the first tiles of the K/V stream; the set-up below only waits for the
    // former while the latter are already in flight.
    constexpr int NQ = NW == 1 ? 2 : 1;  // new rows this wave may have to quantise
    _Float16 nx[NQ][2];
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        const int which = wv + i * NW;
        nx[i][0] = nx[i][1] = (_Float16)0.f;
        if (which < 2) {
            const _Float16* src = (const _Float16*)(which ? a.v_new : a.k_new) + (size_t)u * a.in_stride;
            const half2_t pair = *reinterpret_cast<const half2_t*>(src + 2 * lane);
            nx[i][0] = pair[0];
            nx[i][1] = pair[1];
        }
    }
    Frag<_Float16, 8> qraw[4];
    {
        const _Float16* qu = (const _Float16*)a.q + (size_t)u * a.in_stride + kb * 32;
#pragma unroll
        for (int t = 0; t < 4; ++t) qraw[t].raw = *reinterpret_cast<const uint4*>(qu + t * 8);
        if (a.q_keep && wv == 0 && r == 0) {  // kept for the replay at the next compressions
            _Float16* qk = (_Float16*)a.q_keep + (size_t)u * a.q_keep_stride + kb * 32;
#pragma unroll
            for (int t = 0; t < 4; ++t) *reinterpret_cast<uint4*>(qk + t * 8) = qraw[t].raw;
        }
    }
    uint32_t cpre[cnt_pf(NW * 64)];
    prefetch_counters<NW * 64>(a, u, cpre);

    // Ring of UNR tiles per wave, refilled as soon as consumed.  Wave w owns tiles w, w+NW, ...;
    // every request is unconditional and has the same form (rows beyond the last resident one
    // repeat that row: in bounds, finite, never used), so that the number of loads issued after
    // the ones a tile waits for is a compile-time constant everywhere and a wait covers that
    // tile only: behind a condition the compiler has to wait for everything outstanding.
    const int ntiles = (nc + RPW - 1) / RPW;
    const int nloc = ntiles > wv ? (ntiles - wv + NW - 1) / NW : 0;  // tiles of this wave
    uint4 kr[UNR], vr[UNR];
    uint2 km[UNR];
    uint32_t vm[UNR];
    int next_row = wv * RPW + r;  // row this lane holds in the tile requested next
    auto request = [&](int x) {
        const uint32_t jj = (uint32_t)(next_row < nc ? next_row : nc - 1);
        const uint32_t off = jj * ROWB + (uint32_t)kb * 16u;
        kr[x] = load_stream16(Kb, off);
        vr[x] = load_stream16(Vb, off);
        km[x] = *reinterpret_cast<const uint2*>(Kmb + jj * GPR);
        vm[x] = Vmb[jj * GPR + gi];
        next_row += NW * RPW;
    };
    if (nloc > 0) {
#pragma unroll
        for (int x = 0; x < UNR; ++x) request(x);
    }

    // Alg. 1 model update: wave 0 quantises the key row, wave 1 (wave 0 again when the
    // workgroup is a single wave) the value row.
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        const int which = wv + i * NW;
        if (which < 2) {
            quantise_row<D>((float)nx[i][0], (float)nx[i][1], (which ? Vb : Kb) + (size_t)nc * ROWB,
                            (which ? Vmb : Kmb) + (size_t)nc * GPR, new_codes[which], new_meta[which], lane);
            if (which == 0 && lane == 0) a.pos[(size_t)u * a.C + nc] = a.pos_value;
        }
    }

    // A operands: qa[t] feeds the MFMA that consumes word t of every lane's 16 bytes.  Lane l
    // holds A[i = l%16][k = 8*(l/16) .. +7]; k-block kb, element e stands for channel
    // 32*kb + 8*t + {0,4,1,5,2,6,3,7}[e], divided by 16 where the code arrives multiplied by
    // 16.  Output rows i%4 == 0 take the channels of group 0 (k-blocks 0,1), rows i%4 == 1
    // those of group 1 (k-blocks 2,3), other rows are zero.  c0[g] = -(what the +1024 of every
    // code adds up to for group g), qs[g] = sum of q over group g (for the zero points).
    half8_t qa[4];
    float c0[2], qs[2];
    {
        const bool mine = ((r & 3) == 0 && gi == 0) || ((r & 3) == 1 && gi == 1);
        float sa = 0.f, sb = 0.f;  // sums over the plain / the x16 positions of this lane's 32 channels
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const Frag<_Float16, 8>& qr = qraw[t];
            const _Float16 sixteenth = (_Float16)0.0625f;
            half8_t v = {qr.e[0], qr.e[4], qr.e[1] * sixteenth, qr.e[5] * sixteenth,
                         qr.e[2], qr.e[6], qr.e[3] * sixteenth, qr.e[7] * sixteenth};
            sa += (float)qr.e[0] + (float)qr.e[4] + (float)qr.e[2] + (float)qr.e[6];
            sb += (float)qr.e[1] + (float)qr.e[5] + (float)qr.e[3] + (float)qr.e[7];
            const half8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
            qa[t] = mine ? v : zero;
        }
        // the other half of this lane's group sits 16 lanes away, the other group 32 lanes away
        const float off = 1024.f * sa + 64.f * sb, sum = sa + sb;
        const float off_g = off + __shfl_xor(off, 16), sum_g = sum + __shfl_xor(sum, 16);
        const float off_o = __shfl_xor(off_g, 32), sum_o = __shfl_xor(sum_g, 32);
        c0[0] = -(gi == 0 ? off_g : off_o);
        c0[1] = -(gi == 0 ? off_o : off_g);
        qs[0] = gi == 0 ? sum_g : sum_o;
        qs[1] = gi == 0 ? sum_o : sum_g;
    }

    // Running softmax, one maximum per wave: m; per lane l (sum of weights of its cache rows),
    // acc (32 channels, still carrying the pair offsets), wsum (sum of weight*scale, to remove
    // those offsets) and zacc (sum of weight*zero).
    float m = -INFINITY, l = 0.f, wsum = 0.f, zacc = 0.f, acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.f;

    auto take_tile = [&](auto masked, const uint4& kr, const uint4& vr, uint2 kmw, uint32_t vmw, int j,
                         bool valid) {
        constexpr bool MASKED = decltype(masked)::value;
        const uint32_t kw[4] = {kr.x, kr.y, kr.z, kr.w};
        float4_t d = {c0[0], c0[1], 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            CodeOctet b;
            unpack8(kw[t], b.h2, nk);
            d = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[t], b.h8, d, 0, 0, 0);
        }
        MetaWord k0, k1, vm;
        k0.u32 = kmw.x;
        k1.u32 = kmw.y;
        vm.u32 = vmw;
        float s = fmaf((float)k0.h[0], d[0], (float)k0.h[1] * qs[0]);
        s = fmaf((float)k1.h[0], d[1], s);
        s = fmaf((float)k1.h[1], qs[1], s) * a.qk_log2;
        if constexpr (MASKED) {
            if (valid && kb == 0) s_lds[j] = s;
            s = valid ? s : -INFINITY;
        } else {
            s_lds[j] = s;  // the four lanes that hold row j store the same value
        }
        if (__builtin_amdgcn_ballot_w64(s > m) != 0ull) {  // rare once the maximum has settled
            float smax = row16_max(s);  // over the 16 rows of the tile ...
            smax = fmaxf(smax, __shfl_xor(smax, 16));  // ... and made identical in all four
            smax = fmaxf(smax, __shfl_xor(smax, 32));  // 16-lane rows, whatever their rounding
            const float al = fast_exp2(m - smax);
            l *= al;
            wsum *= al;
            zacc *= al;
#pragma unroll
            for (int i = 0; i < 32; ++i) acc[i] *= al;
            m = smax;
        }
        float e = fast_exp2(s - m);
        if constexpr (MASKED) e = valid ? e : 0.f;
        l += e;
        const float es = e * (float)vm.h[0];
        const float es16 = es * 0.0625f;
        wsum += es;
        zacc = fmaf(e, (float)vm.h[1], zacc);
        const uint32_t vw[4] = {vr.x, vr.y, vr.z, vr.w};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            half2_t h[4];
            unpack8(vw[w], h, nk);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float wk = (k & 1) ? es16 : es;
                acc[w * 8 + k] = fmaf((float)h[k][0], wk, acc[w * 8 + k]);
                acc[w * 8 + k + 4] = fmaf((float)h[k][1], wk, acc[w * 8 + k + 4]);
            }
        }
    };
    using Full = std::integral_constant<bool, false>;
    using Ragged = std::integral_constant<bool, true>;

    // All rounds but the last: UNR tiles taken and replaced, no condition anywhere.  The last
    // round (the only one that can hold the cache's ragged last tile, or fewer than UNR tiles)
    // takes what is left with masks and requests nothing.
    const int slot = (int)(__builtin_amdgcn_s_getreg(GETREG_IMMED(3, 0, HW_ID)) % 3u);  // slot on the SIMD
    const int rounds = (nloc + UNR - 1) / UNR;
    int li = 0;  // local index of the round's first tile
    int turn = slot;
    for (int rr = 0; rr + 1 < rounds; ++rr, li += UNR) {
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            // every other tile at the level of the wave's slot (the hardware's own order among
            // equal levels favours the low slots; this leans the other way), the tiles in
            // between walking through the three levels
            if (x & 1) rotate_priority(slot); else rotate_priority(turn++);
            take_tile(Full{}, kr[x], vr[x], km[x], vm[x], (wv + (li + x) * NW) * RPW + r, true);
            request(x);
        }
    }
    // The new row (quantised into LDS at the start) is attended to here, while the last round's
    // loads are still on their way, rather than after them at the very end of the wave.
    if constexpr (NW > 1) __syncthreads();  // (a single wave reads what it wrote itself)
    if (wv == 0) {
        const uint4 nk = *reinterpret_cast<const uint4*>(&new_codes[0][kb * 16]);
        const uint4 nv = *reinterpret_cast<const uint4*>(&new_codes[1][kb * 16]);
        take_tile(Ragged{}, nk, nv, make_uint2(new_meta[0][0], new_meta[0][1]), new_meta[1][gi], nc, r == 0);
    }
    if (nloc > 0) {
        rotate_priority(slot);
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            if (li + x < nloc) {
                const int j = (wv + (li + x) * NW) * RPW + r;
                take_tile(Ragged{}, kr[x], vr[x], km[x], vm[x], j, j < nc);
            }
        }
    }
    __builtin_amdgcn_s_setprio(0);
    clk.streamed(a);
    // Add up the 16 cache rows of every DPP row, then remove the pair offsets (1024*weight,
    // resp. 1024*weight/16) and add the zero points.
    {
        wsum = row16_sum(wsum);
        zacc = row16_sum(zacc);
        l = row16_sum(l);
        const float off_a = 1024.f * wsum, off_b = 64.f * wsum;
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float o = zacc - ((k & 1) ? off_b : off_a);
                acc[w * 8 + k] = row16_sum(acc[w * 8 + k]) + o;
                acc[w * 8 + k + 4] = row16_sum(acc[w * 8 + k + 4]) + o;
            }
    }
    if constexpr (NW == 1) {
        // A single wave already holds everything: m is the wave's maximum, l the sum over all
        // rows, and lane (r = 0, kb) the 32 output channels 32*kb ..; no trip through LDS.
        const float invL = 1.0f / l;
        if (a.out && r == 0) {
            _Float16* dst = (_Float16*)a.out + (size_t)u * a.out_stride + kb * 32;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                Frag<_Float16, 8> o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o.e[e] = (_Float16)(acc[w * 8 + e] * invL);
                if (a.through) store_through16(dst + w * 8, o.raw); else *reinterpret_cast<uint4*>(dst + w * 8) = o.raw;
            }
        }
        __syncthreads();  // the scores in LDS are complete
        finish_counters<64>(a, u, s_lds, m, invL, cpre);
    } else {
        if (r == 0) {
#pragma unroll
            for (int i = 0; i < 32; ++i) part_acc[wv * D + kb * 32 + i] = acc[i];
            if (kb == 0) {
                part_m[wv] = m;
                part_l[wv] = l;
            }
        }
        __syncthreads();
        finish_unit<_Float16, D, NW * 64, NW>(a, u, s_lds, part_m, part_l, part_acc, cpre);
    }
    clk.finish(a, u);
}

__global__ void clear_u32_kernel(uint32_t* p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0u;
}

template <typename T, int D, int UNR>
hipError_t launch_rows(const AttnArgs& a, int U, int grid, hipStream_t stream) {
    // 16 waves per workgroup with two K and two V loads in flight per lane (<= 64 VGPRs, so two
    // workgroups share a CU): measured on MI355X over unit counts from 128 to 9216 and 350 to 1000
    // resident rows, the fastest or within 2% of it everywhere (4 or 8 waves: up to 65% slower on
    // few units, 1 to 2% on many).
    constexpr int NW = 16;
    const size_t lds = ((size_t)a.C + 2 * NW + (size_t)NW * D) * sizeof(float);
    if (a.split)
        attn_rows_kernel<T, D, NW, UNR, true><<<U * a.split, NW * 64, lds, stream>>>(a);
    else
        attn_rows_kernel<T, D, NW, UNR, false><<<grid, NW * 64, lds, stream>>>(a);
    return hipGetLastError();
}

template <int D, int UNR>
hipError_t launch_i4(const AttnArgs& a, int U, int nw, hipStream_t stream) {
    const size_t lds = ((size_t)a.C + 8 * nw + (size_t)4 * nw * D) * sizeof(float);
    switch (nw) {
        case 1: attn_i4_kernel<D, 1, UNR><<<U, 64, lds, stream>>>(a); break;
        case 2: attn_i4_kernel<D, 2, UNR><<<U, 128, lds, stream>>>(a); break;
        default: attn_i4_kernel<D, 4, UNR><<<U, 256, lds, stream>>>(a); break;
    }
    return hipGetLastError();
}

template <int UNR>
hipError_t launch_i4_mfma(const AttnArgs& a, int U, int nw, hipStream_t stream) {
    const size_t lds = ((size_t)a.C + 2 * nw + (size_t)nw * 128) * sizeof(float);
    switch (nw) {
        case 1: attn_i4_mfma_kernel<1, UNR><<<U, 64, lds, stream>>>(a); break;
        case 2: attn_i4_mfma_kernel<2, UNR><<<U, 128, lds, stream>>>(a); break;
        default: attn_i4_mfma_kernel<4, UNR><<<U, 256, lds, stream>>>(a); break;
    }
    return hipGetLastError();
}

// The 4-bit kernel's per-wave fixed work (query set-up, merging 32 accumulators, the epilogue)
// is paid once per wave, so a unit gets as few waves as still fill the chip.  Measured on
// MI355X on 96*b units of 570 rows (us per launch with 1 / 2 / 4 / 8 waves per unit):
// 96 units 17.0 / 11.7 / 9.2 / 10.3, 192: 17.4 / 12.0 / 9.9 / 10.3, 384: 18.4 / 14.5 / 12.5 / 18.4,
// 768: 19.6 / 16.5 / 17.8 / 28.3, 1536: 27.4 / 27.4 / 33.1 / 53.9, 3072: one wave.
int pick_waves_i4(int U) {
    if (U > 1536) return 1;
    if (U > 512) return 2;
    return 4;
}

}  // namespace

hipError_t launch_decode_step(const Layout& L, const StepArgs& s, hipStream_t stream) {
    AttnArgs a;
    a.q = s.q;
    a.k_new = s.k_new;
    a.v_new = s.v_new;
    a.in_stride = s.in_stride;
    a.K = L.K;
    a.V = L.V;
    a.K_meta = L.K_meta;
    a.V_meta = L.V_meta;
    a.pos = L.pos;
    a.pos_value = s.pos_value;
    a.out = s.out;
    a.out_stride = s.out_stride;
    a.probs = s.probs;
    a.probs_stride = s.probs_stride;
    if (L.W32) {  // ring mode: word plane `bucket` of the uint32 [U][W32][C] ring
        a.cnt = reinterpret_cast<uint16_t*>(reinterpret_cast<uint32_t*>(L.cnt) + (size_t)s.bucket * L.C);
        a.cnt_unit_stride = 2L * L.W32 * L.C;
    } else {
        a.cnt = L.cnt + (size_t)s.bucket * L.C;
        a.cnt_unit_stride = (long)L.E * L.C;
    }
    a.ring_bit = s.ring_bit;
    a.n = s.n;
    a.C = L.C;
    a.qk_log2 = s.qk_log2;
    a.tau = s.tau;
    a.counted = s.counted;
    a.q_keep = s.q_keep;
    a.q_keep_stride = (long)L.w * L.d;
    a.seq = s.seq;
    a.cnt_base = L.cnt;
    a.q_keep_slot_bytes = (long)L.d * (L.kv_dtype == KV_F32 ? 4 : 2);
    a.trace = s.trace;
    {   // bytes this launch writes (counters, outputs, the new rows) against a quarter of the eight
        // 4 MB L2s
        const size_t rows = s.seq.off ? (size_t)L.C : (size_t)s.n;
        const size_t elem = L.kv_dtype == KV_F32 ? 4 : 2;
        const size_t row = L.kv_dtype == KV_I4G64 ? (size_t)L.d / 2 + L.d / 16 : (size_t)L.d * elem;
        const size_t per_unit = rows * (L.W32 ? 4 : 2) + (size_t)L.d * elem + 2 * row;
        a.through = (size_t)L.U * per_unit >= ((size_t)8 << 20);
    }
    // Tickets for the last sixteenth of the units once a launch has several generations of
    // workgroups per XCD (512 workgroups are resident at a time).
    a.ticket = nullptr;
    a.n_static = L.U;
    a.n_tail = a.n_ticket_wgs = 0;
    if (L.ticket && !s.seq.off && L.kv_dtype != KV_I4G64 && L.U >= 2048) {
        a.ticket = L.ticket;
        a.n_tail = L.U / 16;
        a.n_static = L.U - a.n_tail;
        a.n_ticket_wgs = 2 * a.n_tail;
    }
    const int grid = a.n_static + a.n_ticket_wgs;
    a.split = L.kv_dtype != KV_I4G64 ? L.split : 0;
    a.share_stride = L.d + 32;  // acc[d], m, l, padded to whole 128-byte lines
    a.shares = L.shares;
    a.raw = reinterpret_cast<float*>(L.srcmap);  // idle between compressions, same size [U][C]
    a.arrive = L.arrive;
    if (a.split) a.trace = nullptr;  // (the clocks are per workgroup-is-a-unit)
    if (L.kv_dtype == KV_F32)
        return L.d == 64 ? launch_rows<float, 64, 2>(a, L.U, grid, stream)
                         : launch_rows<float, 128, 2>(a, L.U, grid, stream);
    if (L.kv_dtype == KV_F16)
        return L.d == 64 ? launch_rows<_Float16, 64, 2>(a, L.U, grid, stream)
                         : launch_rows<_Float16, 128, 2>(a, L.U, grid, stream);
    const int nw4 = pick_waves_i4(L.U);
    return L.d == 64 ? launch_i4<64, 4>(a, L.U, nw4, stream) : launch_i4_mfma<4>(a, L.U, nw4, stream);
}

hipError_t launch_clear_counters(const Layout& L, hipStream_t stream) {
    const size_t words = L.W32 ? (size_t)L.U * L.W32 * L.C : (size_t)L.U * L.E * L.C / 2;  // C is even
    clear_u32_kernel<<<1024, 256, 0, stream>>>(reinterpret_cast<uint32_t*>(L.cnt), words);
    if (L.ticket) clear_u32_kernel<<<1, 64, 0, stream>>>(reinterpret_cast<uint32_t*>(L.ticket), 1);
    if (L.arrive) clear_u32_kernel<<<1, 64, 0, stream>>>(reinterpret_cast<uint32_t*>(L.arrive), (size_t)L.U);
    return hipGetLastError();
}

}  // namespace sc
