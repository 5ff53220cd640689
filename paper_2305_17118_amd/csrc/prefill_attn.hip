// Prompt phase on the matrix cores (gfx950): a run of consecutive prompt positions between two
// compressions is one dense causal block.  Def. 4.1 treats prompt and generated tokens as one
// stream, so position i of the run must see exactly what a decode step would: the rows that
// were resident before the run plus the run's own rows up to and including i (Alg. 1 appends
// before it attends), and it adds one count to the record of every such row whose
// probability is below its threshold 1/t (Alg. 2, record kept online as Sec. 4.1 allows).
// Inside a run the cache only grows and, with the run cut at the boundaries of the counter
// schedule, every position counts into the same bucket, so the whole run is
//   S = Q K^T (causal), P = softmax(S), out = P V, cnt[j] += #{i : P[i][j] < 1/t_i}.
//
// Every storage type (fp16, fp32 and 4-bit rows; bucket counters or the one-bit-per-step ring).
// One launch per run, one workgroup per (unit, block of queries), which makes two passes over
// the visible rows in tiles of 64 staged in LDS: pass 1 is the usual running-softmax attention
// (scores and P.V on the matrix cores: v_mfma_f32_16x16x32_f16, or v_mfma_f32_16x16x4_f32 for
// fp32 rows), pass 2 recomputes the scores against the final maximum and sum to form the very
// probabilities the threshold is applied to, counts the low ones per cache row and adds the
// counts to the 16-bit counters (two per 32-bit atomic).  The run's own fp16/fp32 rows reach
// their slots through the registers of the workgroup that holds the last query block; 4-bit
// rows are quantised into their slots by a small launch of their own first.
#include "quant.hpp"
#include "sc_kernels.hpp"

#include <type_traits>

namespace sc {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// grid (U, pieces/256): one 16-byte piece of a query row per thread; step t0+1+row goes to
// ring slot (t0 + row) mod w.  count <= w, so no two rows share a slot.
__global__ void __launch_bounds__(256)
store_queries_kernel(const char* __restrict__ q, long unit_stride_bytes, char* __restrict__ ring, int w,
                     int row16, int count, long t0) {
    const int u = blockIdx.x;
    const int e = blockIdx.y * 256 + threadIdx.x;
    if (e >= count * row16) return;
    const int row = e / row16, piece = e - row * row16;
    const size_t slot = (size_t)((t0 + row) % w);
    *reinterpret_cast<uint4*>(ring + (((size_t)u * w + slot) * row16 + piece) * 16) =
        *reinterpret_cast<const uint4*>(q + (size_t)u * unit_stride_bytes + (size_t)e * 16);
}

struct PrefillArgs {
    const void* q;  // fp16, or fp32 with fp32 rows
    long unit_stride;
    const void* K;  // fp16 rows, or 4-bit codes
    const void* V;
    const uint32_t* K_meta;  // 4-bit only: {fp16 scale, fp16 zero} per row and 64 channels
    const uint32_t* V_meta;
    void* out;  // same element type as q
    long out_unit_stride;
    float* probs;
    long probs_unit_stride;
    uint16_t* cnt;  // current bucket of unit 0
    long cnt_unit_stride;
    int C, n0, c, nqb;
    long t0;
    int counted, thresh_len;
    float qk_log2;
    // Replay of kept queries (record collected at compression time): positions of the resident
    // rows, their number, and the length of the query ring; null / 0 for a prompt run.
    const int32_t* pos;
    int n_rows;
    int ring_w;
    // Prompt run with the row copy fused in (fp16): the run's key/value rows as handed in
    // (unit 0; units are unit_stride elements apart) and where their positions go; null
    // when the rows are already in their slots.
    const void* k_run;
    const void* v_run;
    int32_t* pos_w;
    // Exact one-bit-per-step record instead of counters: uint32 [U][ring_words][C], step i owns
    // bit i mod ring_bits of every row; null with bucket counters.
    uint32_t* ring;
    int ring_words, ring_bits;
};

// Write the low/not-low flags of 16 consecutive steps into one row's ring.  `first_bit` is the
// bit the first of them owns; bit k of `touch` says step k saw the row (its bit is rewritten:
// set where `set` has it, cleared otherwise), steps that did not see it leave their bit alone.
// The run of bits is cut at word ends and where the ring wraps.  Other waves update other bits
// of the same words at the same time, hence the atomics.
__device__ __forceinline__ void ring_write16(uint32_t* row_ring, int C, int first_bit, int ring_bits,
                                             uint32_t set, uint32_t touch) {
    int b = first_bit, left = 16;
    while (left > 0) {
        const int off = b & 31;
        int take = 32 - off;
        if (take > ring_bits - b) take = ring_bits - b;
        if (take > left) take = left;
        const uint32_t m = take == 32 ? 0xFFFFFFFFu : ((1u << take) - 1u);
        const uint32_t t = (touch & m) << off, v = (set & m) << off;
        if (t) {
            uint32_t* word = row_ring + (size_t)(b >> 5) * C;
            if (t & ~v) atomicAnd(word, ~(t & ~v));
            if (v) atomicOr(word, v);
        }
        set >>= take;
        touch >>= take;
        left -= take;
        b += take;
        if (b == ring_bits) b = 0;
    }
}

// ---------------------------------------------------------------------------------------
// 4-bit storage (head size 128).  The run's rows are quantised into their slots first (16
// lanes per row, the same single-operation fp32 arithmetic as the decode kernel, so the
// codes are identical to what stepping would have stored).  prefill_chunk_kernel<128, ., ., true>
// then differs from the fp16 instantiation in how a tile is staged and how a score is finished:
//  * keys stay codes: the staged K tile holds the codes as fp16 integers (exact), the matrix
//    instructions accumulate sum_c q_c*code_c per group of 64 channels, and the score is
//    scale_0*S_0 + scale_1*S_1 + zero_0*sum(q over group 0) + zero_1*sum(q over group 1)
//    in fp32, i.e. <q, code*scale + zero> without ever rounding a dequantised key;
//  * values are dequantised while they are transposed into LDS: fp16(code*scale + zero).
// Unpacking a word of eight codes with two masks gives the channel pairs (0,4) (1,5) (2,6)
// (3,7); the staged K tile keeps that order inside every 8 channels and the query operand is
// permuted once to match.
// ---------------------------------------------------------------------------------------
// Quantise 8 consecutive channels held by one lane; the 8 lanes that share a group of 64
// channels are adjacent (half a DPP row).  Same single-operation fp32 arithmetic as
// quantise_row, so the codes and meta words are identical; returns the 8 codes packed into one
// word (channel e in nibble e) and the group's meta word.
__device__ __forceinline__ uint32_t quantise_octet(const half8_t x, uint32_t& meta_word) {
    float f[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (float)x[e];
    float mn = fminf(fminf(fminf(f[0], f[1]), fminf(f[2], f[3])), fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
    float mx = fmaxf(fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3])), fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
    auto dpp = [](float v, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v),
                                                                     decltype(ctrl)::value, 0xF, 0xF, true));
    };
    using X1 = std::integral_constant<int, 0xB1>;   // quad_perm [1,0,3,2]
    using X2 = std::integral_constant<int, 0x4E>;   // quad_perm [2,3,0,1]
    using HM = std::integral_constant<int, 0x141>;  // row_half_mirror: the other quad of these 8 lanes
    mn = fminf(mn, dpp(mn, X1{}));
    mx = fmaxf(mx, dpp(mx, X1{}));
    mn = fminf(mn, dpp(mn, X2{}));
    mx = fmaxf(mx, dpp(mx, X2{}));
    mn = fminf(mn, dpp(mn, HM{}));
    mx = fmaxf(mx, dpp(mx, HM{}));
    const float range = __fsub_rn(mx, mn);
    _Float16 sh = (_Float16)__fdiv_rn(range, 15.0f);
    float sc = (float)sh;
    if (sc == 0.0f) {
        sc = 1.0f;
        sh = (_Float16)1.0f;
    }
    const _Float16 zh = (_Float16)mn;
    const float z = (float)zh;
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float c = rintf(__fdiv_rn(__fsub_rn(f[e], z), sc));
        c = fminf(fmaxf(c, 0.f), 15.f);
        word |= (uint32_t)c << (4 * e);
    }
    MetaWord mw;
    mw.h[0] = sh;
    mw.h[1] = zh;
    meta_word = mw.u32;
    return word;
}

// Quantise the run's rows into slots n0.. : D/8 lanes per row (8 channels each), 2048/D rows
// per workgroup; grid (U, rows / (2048/D)).
template <int D>
__global__ void __launch_bounds__(256)
append_rows_i4_kernel(const _Float16* __restrict__ k, const _Float16* __restrict__ v, long unit_stride,
                      unsigned char* __restrict__ K, unsigned char* __restrict__ V,
                      uint32_t* __restrict__ Km, uint32_t* __restrict__ Vm, int32_t* __restrict__ pos,
                      int C, int n0, int c, int t0) {
    constexpr int LPR = D / 8;  // lanes per row
    const int u = blockIdx.x, l8 = threadIdx.x & (LPR - 1);
    int row = blockIdx.y * (256 / LPR) + (threadIdx.x / LPR);
    const bool live = row < c;
    row = live ? row : c - 1;  // idle lanes shadow the last row (the reductions need every lane)
    const size_t src = (size_t)u * unit_stride + (size_t)row * D + 8 * l8;
    const size_t slot = (size_t)u * C + n0 + row;
    const half8_t kk = *reinterpret_cast<const half8_t*>(k + src);
    const half8_t vv = *reinterpret_cast<const half8_t*>(v + src);
    uint32_t kmw, vmw;
    const uint32_t kc = quantise_octet(kk, kmw);
    const uint32_t vc = quantise_octet(vv, vmw);
    if (!live) return;
    reinterpret_cast<uint32_t*>(K + slot * (D / 2))[l8] = kc;
    reinterpret_cast<uint32_t*>(V + slot * (D / 2))[l8] = vc;
    if ((l8 & 7) == 0) {
        Km[slot * (D / 64) + (l8 >> 3)] = kmw;
        Vm[slot * (D / 64) + (l8 >> 3)] = vmw;
    }
    if (l8 == 0) pos[slot] = t0 + row;
}

// The eight codes of word w as fp16 integers, in the order (n0,n4) (n1,n5) (n2,n6) (n3,n7).
__device__ __forceinline__ void codes_to_half(uint32_t w, half2_t (&h)[4]) {
    const uint32_t t = w >> 8;
    const half2_t k1024 = {(_Float16)1024.f, (_Float16)1024.f};
    const half2_t k64 = {(_Float16)64.f, (_Float16)64.f};
    const half2_t sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    // (w & mask) | 0x6400 per half is the fp16 number 1024 + code (low nibble) or 1024 + 16*code
    h[0] = __builtin_bit_cast(half2_t, (w & 0x000F000Fu) | 0x64006400u) - k1024;
    h[1] = __builtin_bit_cast(half2_t, (w & 0x00F000F0u) | 0x64006400u) * sixteenth - k64;
    h[2] = __builtin_bit_cast(half2_t, (t & 0x000F000Fu) | 0x64006400u) - k1024;
    h[3] = __builtin_bit_cast(half2_t, (t & 0x00F000F0u) | 0x64006400u) * sixteenth - k64;
}


// Matrix-instruction operand layout (16x16x32, fp16 in, fp32 out), lane l, i = l%16, g = l/16:
//   A: lane holds A[i][8g .. 8g+7]      B: lane holds B[8g .. 8g+7][i]      D: lane holds D[4g + r][i]
// Scores are computed transposed, S^T = K Q^T (A = 16 cache rows, B = 16 queries), so a lane
// ends up with four consecutive cache rows of ONE query: softmax statistics are per lane
// (plus a reduction over g), and the probabilities are already laid out as the B operand of
// out^T = V^T P^T, whose contraction index (lane group g, element e) stands for cache row
// 4g + e of one 16-row block (e < 4) or of the next one (e >= 4).  V is staged transposed in
// LDS so that its A operand is two 8-byte reads.
// At least three waves per SIMD: the register budget that goes with it (168) also makes the
// compiler keep the matrix accumulators in ordinary vector registers, where the running-softmax
// rescale can reach them without copies.
//
// WITH_PV = false drops the value side (no V tile, no P.V, no output): that is the replay of
// Alg. 2 as printed, which recomputes the attention of the last w queries over the rows
// resident at compression time only to count low probabilities.  There the queries come
// from a ring (step i in slot (i-1) mod w) and the last row step i may see is found from the
// rows' stream positions (rows are kept in order of position): the last one with
// position <= i-1.
//
// SB = blocks of 16 queries per wave.  With SB = 2 every K and V fragment read from LDS feeds
// two matrix instructions (LDS operand traffic, the busiest resource of this kernel, is halved
// per query) at the price of twice the accumulators, i.e. two instead of three waves per SIMD.
//
// I4 = true: 4-bit rows (see above); the rows are already in their slots (quantised by
// append_rows_i4_kernel), so nothing is read from the caller's arrays or written here.
//
// F32 = true: fp32 rows, queries and outputs.  The same two passes on the fp32 matrix
// instruction (16x16x4: lane l holds A[l%16][l/16], B[l/16][l%16], D[4(l/16)+r][l%16]):
// probabilities stay fp32, V is staged row-major (its operand is one float per lane), and
// tiles go from global memory straight into LDS without a register stage (a path kept for
// completeness: fp32 rows cost twice the traffic of fp16 ones).
template <int D, bool WITH_PV, int SB, bool I4, bool F32 = false>
__global__ void __launch_bounds__(256)
__attribute__((amdgpu_waves_per_eu(SB == 1 && !(F32 && D == 128) ? 3 : 2)))  // fp32, d = 128: 67 KB of LDS allow two anyway
prefill_chunk_kernel(PrefillArgs a) {
    static_assert(!(I4 && F32) && (!F32 || SB == 1), "fp32 rows: one query block per wave");
    constexpr int GPR = D / 64;   // 4-bit rows: groups of 64 channels, each with its own scale and zero
    constexpr int KB = 64;        // cache rows per tile
    constexpr int WQ = 16 * SB;   // queries per wave
    constexpr int QB = 4 * WQ;    // queries per workgroup
    constexpr int LDK = F32 ? D + 4 : D + 8;  // elements per staged K row (the padding keeps operand reads conflict-free)
    constexpr int LDV = KB + 4;   // halfs per channel of the transposed V tile
    constexpr int LDVF = D + 4;   // fp32: floats per row of the row-major V tile
    constexpr int KS4 = D / 4;    // fp32: matrix instructions per 16 scores
    constexpr int KS = D / 32;    // matrix instructions per 16 scores
    constexpr int CB = D / 16;    // 16-channel blocks of the output
    constexpr int PIECES = KB * D / 8 / 256;  // 16-byte pieces of a tile per thread
    __shared__ __align__(16) unsigned char ks_raw[KB * LDK * (F32 ? 4 : 2)];
    __shared__ __align__(16) unsigned char vt_raw[F32 ? KB * LDVF * 4 : D * LDV * 2];
    _Float16* const Ks = reinterpret_cast<_Float16*>(ks_raw);
    _Float16* const Vt = reinterpret_cast<_Float16*>(vt_raw);
    float* const Ksf = reinterpret_cast<float*>(ks_raw);
    float* const Vsf = reinterpret_cast<float*>(vt_raw);
    __shared__ float stat_m[QB], stat_inv[QB];  // per query: final maximum, 1/sum (pass 1 -> pass 2)
    __shared__ __align__(16) float Kmeta[I4 ? KB * 4 : 4];  // 4-bit: per tile row scale, zero of group 0; of group 1
    __shared__ float stat_q0[I4 ? QB : 1], stat_q1[I4 ? QB : 1];  // 4-bit: per query, sum of q over each group
    __shared__ int stat_lim[QB];                // per query: last row it sees (-1: none)
    extern __shared__ int cnt_lds[];  // [tiles * 64] low-score counts of this workgroup's queries

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int li = lane & 15, g = lane >> 4;
    // A prompt run handed in with its rows still in the caller's arrays (k_run): every
    // workgroup reads the run's rows from there, and the workgroup of the last query block,
    // which sees all of them, also writes them into their slots as they pass through its
    // registers (Alg. 1 "model update"): no separate copy pass, no second read.
    const bool fused = a.k_run != nullptr;
    // Workgroups are handed to the 8 XCDs round-robin by their index; each XCD has its own L2.
    // Renumber them so that an XCD receives consecutive numbers: the query blocks of one unit,
    // which read the same K/V rows, then run on one XCD at about the same time and share its L2.
    unsigned blk;
    {
        const unsigned per = gridDim.x / 8, rem = gridDim.x % 8, xcd = blockIdx.x % 8, idx = blockIdx.x / 8;
        blk = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + idx;
    }
    const int u = blk / a.nqb;
    const int q0 = (a.nqb - 1 - (int)(blk % a.nqb)) * QB;  // longest query blocks first
    const bool writer = fused && blk % a.nqb == 0;
    int qi[SB], qc[SB];  // this lane's queries (positions in the run); padding lanes shadow the last one
#pragma unroll
    for (int sb = 0; sb < SB; ++sb) {
        qi[sb] = q0 + WQ * w + 16 * sb + li;
        qc[sb] = qi[sb] < a.c ? qi[sb] : a.c - 1;
    }
    const int q_last = (q0 + QB < a.c ? q0 + QB : a.c) - 1;
    // Last cache row each of the workgroup's queries sees.  Prompt run: n0 + query index.
    // Replay: rows with position <= t0 + query index (binary search over the positions, staged
    // in the LDS array that later holds the counts).
    if (a.pos) {
        const int32_t* pu = a.pos + (size_t)u * a.C;
        for (int i = tid; i < a.n_rows; i += 256) cnt_lds[i] = pu[i];
        __syncthreads();
        if (tid < QB) {
            const int q = q0 + tid < a.c ? q0 + tid : a.c - 1;
            const int want = (int)a.t0 + q;
            int lo = 0, up = a.n_rows;
            while (lo < up) {
                const int mid = (lo + up) >> 1;
                if (cnt_lds[mid] <= want) lo = mid + 1; else up = mid;
            }
            stat_lim[tid] = lo - 1;
        }
    } else if (tid < QB) {
        stat_lim[tid] = a.n0 + (q0 + tid < a.c ? q0 + tid : a.c - 1);
    }
    __syncthreads();
    bool valid[SB];  // a real query that sees at least one row
    int lim[SB];     // last row it sees (a query that sees nothing shadows row 0, never stored)
    int sub_first_lim[SB];  // last row ALL queries of the 16-block see
#pragma unroll
    for (int sb = 0; sb < SB; ++sb) {
        const int lim_raw = stat_lim[WQ * w + 16 * sb + li];
        valid[sb] = qi[sb] < a.c && lim_raw >= 0;
        lim[sb] = lim_raw > 0 ? lim_raw : 0;
        sub_first_lim[sb] = stat_lim[WQ * w + 16 * sb] > 0 ? stat_lim[WQ * w + 16 * sb] : 0;
    }
    const int hi = (stat_lim[q_last - q0] > 0 ? stat_lim[q_last - q0] : 0) + 1;  // rows visible to this workgroup
    const int ntiles = (hi + KB - 1) / KB;
    const int wave_lim = stat_lim[WQ * w + WQ - 1] > 0 ? stat_lim[WQ * w + WQ - 1] : 0;  // last row any query of the wave sees

    const _Float16* Kb = static_cast<const _Float16*>(a.K) + (size_t)u * a.C * D;
    const _Float16* Vb = static_cast<const _Float16*>(a.V) + (size_t)u * a.C * D;
    // rows n0.. of a fused run are read from the caller's arrays
    const _Float16* Krun = fused ? static_cast<const _Float16*>(a.k_run) + (size_t)u * a.unit_stride : nullptr;
    const _Float16* Vrun = fused ? static_cast<const _Float16*>(a.v_run) + (size_t)u * a.unit_stride : nullptr;
    // fp32 rows
    const float* Kbf = static_cast<const float*>(a.K) + (size_t)u * a.C * D;
    const float* Vbf = static_cast<const float*>(a.V) + (size_t)u * a.C * D;
    const float* Krunf = fused ? static_cast<const float*>(a.k_run) + (size_t)u * a.unit_stride : nullptr;
    const float* Vrunf = fused ? static_cast<const float*>(a.v_run) + (size_t)u * a.unit_stride : nullptr;

    // 4-bit rows: codes, and one meta word per row and group
    const unsigned char* Kc = static_cast<const unsigned char*>(a.K) + (size_t)u * a.C * (D / 2);
    const unsigned char* Vc = static_cast<const unsigned char*>(a.V) + (size_t)u * a.C * (D / 2);
    const uint32_t* Kmb = I4 ? a.K_meta + (size_t)u * a.C * GPR : nullptr;
    const uint32_t* Vmb = I4 ? a.V_meta + (size_t)u * a.C * GPR : nullptr;

    // Query operand.  4-bit: channels 32*ks + 8*g + {0,4,1,5,2,6,3,7} (the order the codes are
    // unpacked in), plus the sums of q over the two groups for the zero points.
    half8_t qB[SB][KS];
    float qF[F32 ? KS4 : 1];  // fp32: q[query li][4*ks + g]
    float qsum0[SB], qsum1[SB];
    if constexpr (F32) {
        const long qslot = a.ring_w ? (a.t0 + qc[0]) % a.ring_w : qc[0];
        const float* qrow = static_cast<const float*>(a.q) + (size_t)u * a.unit_stride + (size_t)qslot * D + g;
#pragma unroll
        for (int ks = 0; ks < KS4; ++ks) qF[ks] = qrow[4 * ks];
        qsum0[0] = qsum1[0] = 0.f;
    }
#pragma unroll
    for (int sb = 0; sb < (F32 ? 0 : SB); ++sb) {
        const long qslot = a.ring_w ? (a.t0 + qc[sb]) % a.ring_w : qc[sb];
        const _Float16* qrow = static_cast<const _Float16*>(a.q) + (size_t)u * a.unit_stride + (size_t)qslot * D + 8 * g;
        float part[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const half8_t x = *reinterpret_cast<const half8_t*>(qrow + 32 * ks);
            qB[sb][ks] = I4 ? __builtin_shufflevector(x, x, 0, 4, 1, 5, 2, 6, 3, 7) : x;
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += (float)x[e];
            part[ks] = acc;
        }
        qsum0[sb] = qsum1[sb] = 0.f;
        if constexpr (I4) {
            float s0 = part[0] + part[1], s1 = part[KS - 2] + part[KS - 1];
            s0 += __shfl_xor(s0, 16);
            s0 += __shfl_xor(s0, 32);
            s1 += __shfl_xor(s1, 16);
            s1 += __shfl_xor(s1, 32);
            qsum0[sb] = s0;
            qsum1[sb] = s1;
        }
    }

    // A tile travels global -> registers -> LDS; the loads of tile kt+1 are issued before
    // tile kt is computed on.  K pieces: 16 bytes of one row per thread and piece.  V pieces come
    // in pairs (the same 8 channels of rows 2*rp and 2*rp+1) so that the transposed tile is
    // written one 32-bit word (two rows of a channel) at a time.  The row index of the
    // transposed tile is XORed with 8*(channel/32): with that the 64 lanes of a store hit 64
    // different banks, and groups of four rows stay contiguous for the operand reads.
    u32x4_t kreg[PIECES];
    half8_t vreg[PIECES];
    constexpr int RPP = 256 / (D / 8);  // tile rows covered by one K piece index step
    const int prow_k = tid / (D / 8), pcb8 = tid % (D / 8);
    const uint32_t koff = (uint32_t)(prow_k * D + pcb8 * 8) * 2u;       // bytes inside a tile
    const uint32_t voff = (uint32_t)(2 * prow_k * D + pcb8 * 8) * 2u;
    // 4-bit staging: thread = (tile row tid/4, 32 channels starting at 32*(tid%4))
    const int srow = tid >> 2, sp = tid & 3;
    u32x4_t kcodes, vcodes;
    uint32_t kmreg = 0, vmreg = 0;
    auto fetch = [&](int kt, bool with_v) {
        const int r0 = kt * KB;
        if constexpr (F32) return;  // fp32 tiles go straight to LDS in stage()
        if constexpr (I4) {
            if (sp >= D / 32) return;  // rows of 64 channels: two of a row's four threads carry it
            int grow = r0 + srow;
            grow = grow < hi ? grow : hi - 1;  // stay inside rows that hold data
            kcodes = *reinterpret_cast<const u32x4_t*>(Kc + (size_t)grow * (D / 2) + sp * 16);
            kmreg = Kmb[(size_t)grow * GPR + (sp >> 1)];
            if (with_v) {
                vcodes = *reinterpret_cast<const u32x4_t*>(Vc + (size_t)grow * (D / 2) + sp * 16);
                vmreg = Vmb[(size_t)grow * GPR + (sp >> 1)];
            }
            return;
        }
        const bool in_cache = !fused || r0 + KB <= a.n0, in_run = fused && r0 >= a.n0;
        if (r0 + KB <= hi && (in_cache || in_run)) {  // a whole tile of data from one array
            const char* kt_base = in_cache ? reinterpret_cast<const char*>(Kb) + (size_t)r0 * D * 2
                                           : reinterpret_cast<const char*>(Krun) + (size_t)(r0 - a.n0) * D * 2;
            const char* vt_base = in_cache ? reinterpret_cast<const char*>(Vb) + (size_t)r0 * D * 2
                                           : reinterpret_cast<const char*>(Vrun) + (size_t)(r0 - a.n0) * D * 2;
#pragma unroll
            for (int x = 0; x < PIECES; ++x)
                kreg[x] = *reinterpret_cast<const u32x4_t*>(kt_base + koff + (uint32_t)(x * RPP * D * 2));
            if (with_v) {
#pragma unroll
                for (int x = 0; x < PIECES / 2; ++x)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        vreg[2 * x + h] = *reinterpret_cast<const half8_t*>(
                            vt_base + voff + (uint32_t)((2 * x * RPP + h) * D * 2));
            }
        } else {
            // Last tile (rows past the data are read from the last row that holds some) or a
            // tile that straddles the boundary between resident rows and the run's own.
            auto row_of = [&](const _Float16* cache, const _Float16* run, int row) {
                int grow = r0 + row;
                grow = grow < hi ? grow : hi - 1;
                return (!fused || grow < a.n0) ? cache + (size_t)grow * D : run + (size_t)(grow - a.n0) * D;
            };
#pragma unroll
            for (int x = 0; x < PIECES; ++x)
                kreg[x] = *reinterpret_cast<const u32x4_t*>(row_of(Kb, Krun, prow_k + x * RPP) + pcb8 * 8);
            if (with_v) {
#pragma unroll
                for (int x = 0; x < PIECES / 2; ++x)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        vreg[2 * x + h] = *reinterpret_cast<const half8_t*>(
                            row_of(Vb, Vrun, 2 * (prow_k + x * RPP) + h) + pcb8 * 8);
            }
        }
    };
    _Float16* Kw = const_cast<_Float16*>(Kb);
    _Float16* Vw = const_cast<_Float16*>(Vb);
    auto stage = [&](bool with_v, int kt) {
        const int r0 = kt * KB;
        if constexpr (F32) {
            constexpr int P4 = D / 4;  // 16-byte pieces per row
            const bool keep = writer && with_v && r0 + KB > a.n0;
            float* Kwf = const_cast<float*>(Kbf);
            float* Vwf = const_cast<float*>(Vbf);
#pragma unroll 4
            for (int p = tid; p < KB * P4; p += 256) {
                const int row = p / P4, c4 = p - row * P4;
                int grow = r0 + row;
                const bool real = grow < hi;
                grow = real ? grow : hi - 1;  // rows past the data shadow the last one that holds some
                const bool cached = !fused || grow < a.n0;
                const size_t off = cached ? (size_t)grow * D + 4 * c4 : (size_t)(grow - a.n0) * D + 4 * c4;
                const float4_t kv = *reinterpret_cast<const float4_t*>((cached ? Kbf : Krunf) + off);
                *reinterpret_cast<float4_t*>(&Ksf[row * LDK + 4 * c4]) = kv;
                const bool store = keep && real && !cached;
                if (store) {
                    *reinterpret_cast<float4_t*>(Kwf + (size_t)grow * D + 4 * c4) = kv;
                    if (c4 == 0) a.pos_w[(size_t)u * a.C + grow] = (int)a.t0 + grow - a.n0;
                }
                if (with_v) {
                    const float4_t vv = *reinterpret_cast<const float4_t*>((cached ? Vbf : Vrunf) + off);
                    *reinterpret_cast<float4_t*>(&Vsf[row * LDVF + 4 * c4]) = vv;
                    if (store) *reinterpret_cast<float4_t*>(Vwf + (size_t)grow * D + 4 * c4) = vv;
                }
            }
            return;
        }
        if constexpr (I4) {
            if (sp >= D / 32) return;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                half2_t h[4];
                codes_to_half(kcodes[i], h);
                const half4_t lo = __builtin_shufflevector(h[0], h[1], 0, 1, 2, 3);
                const half4_t hi4 = __builtin_shufflevector(h[2], h[3], 0, 1, 2, 3);
                *reinterpret_cast<half8_t*>(&Ks[srow * LDK + 32 * sp + 8 * i]) =
                    __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
            }
            if ((sp & 1) == 0) {
                MetaWord kw;
                kw.u32 = kmreg;
                *reinterpret_cast<float2*>(&Kmeta[srow * 4 + (sp >> 1) * 2]) = make_float2((float)kw.h[0], (float)kw.h[1]);
                if (GPR == 1) *reinterpret_cast<float2*>(&Kmeta[srow * 4 + 2]) = make_float2(0.f, 0.f);  // no second group
            }
            if (with_v) {
                MetaWord mw;
                mw.u32 = vmreg;
                const half2_t sc2 = {mw.h[0], mw.h[0]}, zr2 = {mw.h[1], mw.h[1]};
                // P[i][k] = values of channels 32*sp + 8*i + k and + 4 of this thread's row as fp16:
                // code*scale + zero in one fused fp16 operation (the codes are exact integers, so
                // this is the real value rounded once)
                half2_t P[4][4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    half2_t h[4];
                    codes_to_half(vcodes[i], h);
#pragma unroll
                    for (int k = 0; k < 4; ++k) P[i][k] = __builtin_elementwise_fma(h[k], sc2, zr2);
                }
                // Rows 2k and 2k+1 sit four lanes apart.  The even-row thread ends up with channels
                // 0..15 of both rows, the odd-row thread with channels 16..31, so that each writes
                // 32-bit words {row 2k, row 2k+1} of the transposed tile.
                const bool odd = srow & 1;
                const int col = (srow & ~1) ^ (8 * sp);  // swizzle: channel/32 == sp
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const half2_t lower = P[i][k], upper = P[2 + i][k];
                        const uint32_t send = __builtin_bit_cast(uint32_t, odd ? lower : upper);
                        const half2_t got = __builtin_bit_cast(half2_t, (uint32_t)__shfl_xor((int)send, 4));
                        const half2_t mine = odd ? upper : lower;
                        const half2_t r0h = odd ? got : mine, r1h = odd ? mine : got;  // rows 2k, 2k+1
                        const int ch = 32 * sp + (odd ? 16 : 0) + 8 * i + k;
                        const half2_t w0 = {r0h[0], r1h[0]}, w1 = {r0h[1], r1h[1]};
                        *reinterpret_cast<half2_t*>(&Vt[ch * LDV + col]) = w0;
                        *reinterpret_cast<half2_t*>(&Vt[(ch + 4) * LDV + col]) = w1;
                    }
            }
            return;
        }
        // the writer keeps the run's rows (slots n0 .. n0+c-1) as they come by, in pass 1
        const bool keep = writer && with_v && r0 + KB > a.n0;
#pragma unroll
        for (int x = 0; x < PIECES; ++x) {
            *reinterpret_cast<u32x4_t*>(&Ks[(prow_k + x * RPP) * LDK + pcb8 * 8]) = kreg[x];
            const int grow = r0 + prow_k + x * RPP;
            if (keep && grow >= a.n0 && grow < hi) {
                *reinterpret_cast<u32x4_t*>(Kw + (size_t)grow * D + pcb8 * 8) = kreg[x];
                if (pcb8 == 0) a.pos_w[(size_t)u * a.C + grow] = (int)a.t0 + grow - a.n0;
            }
        }
        if (with_v) {
#pragma unroll
            for (int x = 0; x < PIECES / 2; ++x) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int grow = r0 + 2 * (prow_k + x * RPP) + h;
                    if (keep && grow >= a.n0 && grow < hi)
                        *reinterpret_cast<half8_t*>(Vw + (size_t)grow * D + pcb8 * 8) = vreg[2 * x + h];
                }
                const int col = (2 * (prow_k + x * RPP)) ^ (8 * (pcb8 >> 2));
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const half2_t two = {vreg[2 * x][e], vreg[2 * x + 1][e]};
                    *reinterpret_cast<half2_t*>(&Vt[(pcb8 * 8 + e) * LDV + col]) = two;
                }
            }
        }
    };
    // Raw dot products of a 64-row tile with the wave's SB blocks of 16 queries.
    // TRANSPOSED: d[sb][rb][r] = <k_j, q_i> for cache row j = 64*kt + 16*rb + 4*g + r and query
    //             i = li of block sb (a lane holds one query per block: what the running
    //             softmax and P.V want);
    // otherwise:  d[sb][rb][r] = <k_j, q_i> for cache row j = 64*kt + 16*rb + li and query
    //             i = 4*g + r of block sb (a lane holds one cache row: what the counts want).
    // Every K fragment is read from LDS once and used for all SB blocks.
    // 4-bit: the matrix instructions give sum_c q_c*code_c per group of 64 channels; the score is
    // scale_0*S_0 + scale_1*S_1 + zero_0*sum(q over group 0) + zero_1*sum(q over group 1) in fp32.
    float qs0p[SB][4], qs1p[SB][4];  // pass 2: group sums of this lane's four queries per block
    auto finish_score = [](float s0, float s1, float4_t meta, float q0s, float q1s) {
        float s = meta[1] * q0s;
        s = fmaf(meta[3], q1s, s);
        s = fmaf(meta[0], s0, s);
        return fmaf(meta[2], s1, s);
    };
    auto scores = [&](auto transposed, float4_t (&d)[SB][4]) {
        constexpr bool TRANSPOSED = decltype(transposed)::value;
        if constexpr (F32) {
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                float4_t acc4 = {0.f, 0.f, 0.f, 0.f};
                const float* krow = &Ksf[(16 * rb + li) * LDK + g];
#pragma unroll
                for (int ks = 0; ks < KS4; ++ks) {
                    const float kv = krow[4 * ks];  // K[row 16rb+li][channel 4ks+g]: A of S^T, B of S
                    acc4 = TRANSPOSED ? __builtin_amdgcn_mfma_f32_16x16x4f32(kv, qF[ks], acc4, 0, 0, 0)
                                      : __builtin_amdgcn_mfma_f32_16x16x4f32(qF[ks], kv, acc4, 0, 0, 0);
                }
                d[0][rb] = acc4;
            }
            return;
        }
        if constexpr (I4) {
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                half8_t kf[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    kf[ks] = *reinterpret_cast<const half8_t*>(&Ks[(16 * rb + li) * LDK + 32 * ks + 8 * g]);
                float4_t meta[4];  // transposed: rows 4g + r of the block; plain: row li (entry 0)
                if constexpr (TRANSPOSED) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        meta[r] = *reinterpret_cast<const float4_t*>(&Kmeta[(16 * rb + 4 * g + r) * 4]);
                } else {
                    meta[0] = *reinterpret_cast<const float4_t*>(&Kmeta[(16 * rb + li) * 4]);
                }
#pragma unroll
                for (int sb = 0; sb < SB; ++sb) {
                    float4_t g0 = {0.f, 0.f, 0.f, 0.f}, g1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        if constexpr (TRANSPOSED) {
                            g0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[ks], qB[sb][ks], g0, 0, 0, 0);
                            if constexpr (GPR == 2)
                                g1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[2 + ks], qB[sb][2 + ks], g1, 0, 0, 0);
                        } else {
                            g0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(qB[sb][ks], kf[ks], g0, 0, 0, 0);
                            if constexpr (GPR == 2)
                                g1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(qB[sb][2 + ks], kf[2 + ks], g1, 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        d[sb][rb][r] = TRANSPOSED ? finish_score(g0[r], g1[r], meta[r], qsum0[sb], qsum1[sb])
                                                  : finish_score(g0[r], g1[r], meta[0], qs0p[sb][r], qs1p[sb][r]);
                }
            }
            return;
        }
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) d[sb][rb] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const half8_t kf = *reinterpret_cast<const half8_t*>(&Ks[(16 * rb + li) * LDK + 32 * ks + 8 * g]);
#pragma unroll
                for (int sb = 0; sb < SB; ++sb) {
                    if constexpr (TRANSPOSED)
                        d[sb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf, qB[sb][ks], d[sb][rb], 0, 0, 0);
                    else
                        d[sb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qB[sb][ks], kf, d[sb][rb], 0, 0, 0);
                }
            }
    };
    using Transposed = std::integral_constant<bool, true>;
    using Plain = std::integral_constant<bool, false>;

    // ---- pass 1: running softmax and P.V --------------------------------------------------
    // m is kept in the scaled (log2) domain; the scale is positive, so the maximum can be
    // taken over the raw dot products and scaled once.
    const float c2 = a.qk_log2;
    float m[SB], lsum[SB];
    float4_t acc[SB][CB];
#pragma unroll
    for (int sb = 0; sb < SB; ++sb) {
        m[sb] = -INFINITY;
        lsum[sb] = 0.f;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) acc[sb][cb] = float4_t{0.f, 0.f, 0.f, 0.f};
    }
    fetch(0, WITH_PV);
    for (int kt = 0; kt < ntiles; ++kt) {
        __syncthreads();
        stage(WITH_PV, kt);
        __syncthreads();
        if (kt + 1 < ntiles) fetch(kt + 1, WITH_PV);
        if (kt * KB > wave_lim) continue;  // nothing in this tile is visible to this wave
        float4_t d[SB][4];
        scores(Transposed{}, d);
        half4_t ph[SB][4];
        float4_t pf[F32 ? 4 : 1];  // fp32 rows: the probabilities stay fp32
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) {
            if (kt * KB + KB - 1 > sub_first_lim[sb]) {  // the causal boundary crosses this tile
                const int rel = lim[sb] - (kt * KB + 4 * g);  // rows 16*rb + r <= rel are visible
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) d[sb][rb][r] = (16 * rb + r <= rel) ? d[sb][rb][r] : -INFINITY;
            }
            float tmax = fmaxf(fmaxf(d[sb][0][0], d[sb][0][1]), fmaxf(d[sb][0][2], d[sb][0][3]));
#pragma unroll
            for (int rb = 1; rb < 4; ++rb)
                tmax = fmaxf(tmax, fmaxf(fmaxf(d[sb][rb][0], d[sb][rb][1]), fmaxf(d[sb][rb][2], d[sb][rb][3])));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            // finite from tile 0 on: row 0 is visible to every query
            const float m_new = fmaxf(m[sb], tmax * c2);
            if (__builtin_amdgcn_ballot_w64(m_new != m[sb]) != 0ull) {
                const float alpha = fast_exp2(m[sb] - m_new);
                lsum[sb] *= alpha;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) acc[sb][cb] *= alpha;
                m[sb] = m_new;
            }
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                float4_t p;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    p[r] = fast_exp2(fmaf(d[sb][rb][r], c2, -m[sb]));
                    lsum[sb] += p[r];
                }
                if constexpr (F32) pf[rb] = p;
                else ph[sb][rb] = __builtin_convertvector(p, half4_t);
            }
        }
        if constexpr (WITH_PV && F32) {
            // out^T = V^T P^T four cache rows at a time: for rows 16rb + 4g' + r (g' = 0..3) the A
            // operand is V[that row][channel 16cb + li] and the B operand this lane's p[rb][r].
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float* vrow = &Vsf[(16 * rb + 4 * g + r) * LDVF + li];
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
                        acc[0][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(vrow[16 * cb], pf[rb][r], acc[0][cb], 0, 0, 0);
                }
        }
        if constexpr (WITH_PV && !F32) {
#pragma unroll
            for (int kp = 0; kp < 2; ++kp) {
                // The swizzle of the transposed tile decides which of the two 4-row groups of a
                // lane sits at the lower LDS address; the probabilities are ordered to match,
                // so that the operand is one two-address read with no register shuffling.
                half8_t B01[SB], B10[SB];
#pragma unroll
                for (int sb = 0; sb < SB; ++sb) {
                    B01[sb] = __builtin_shufflevector(ph[sb][2 * kp], ph[sb][2 * kp + 1], 0, 1, 2, 3, 4, 5, 6, 7);
                    B10[sb] = __builtin_shufflevector(ph[sb][2 * kp + 1], ph[sb][2 * kp], 0, 1, 2, 3, 4, 5, 6, 7);
                }
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    const int swz = 8 * (cb >> 1);  // channel/32 == cb/2
                    const _Float16* vrow = &Vt[(16 * cb + li) * LDV + (((32 * kp + 4 * g) ^ swz) & ~16)];
                    const half4_t a0 = *reinterpret_cast<const half4_t*>(vrow);
                    const half4_t a1 = *reinterpret_cast<const half4_t*>(vrow + 16);
                    const half8_t A = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int sb = 0; sb < SB; ++sb)
                        acc[sb][cb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, (swz & 16) ? B10[sb] : B01[sb],
                                                                              acc[sb][cb], 0, 0, 0);
                }
            }
        }
    }
    const bool pass2 = a.counted || a.probs;
    // Pass 2 runs backwards and starts on the K tile that pass 1 left staged; the tile before it
    // is in flight while the outputs are written.
    if (pass2 && ntiles > 1) fetch(ntiles - 2, false);
    float invL[SB];
#pragma unroll
    for (int sb = 0; sb < SB; ++sb) {
        lsum[sb] += __shfl_xor(lsum[sb], 16);
        lsum[sb] += __shfl_xor(lsum[sb], 32);
        invL[sb] = 1.0f / lsum[sb];
        if (WITH_PV && a.out && valid[sb]) {
            if constexpr (F32) {
                float* orow = static_cast<float*>(a.out) + (size_t)u * a.out_unit_stride + (size_t)qi[sb] * D + 4 * g;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) *reinterpret_cast<float4_t*>(orow + 16 * cb) = acc[sb][cb] * invL[sb];
            } else {
                _Float16* orow = static_cast<_Float16*>(a.out) + (size_t)u * a.out_unit_stride + (size_t)qi[sb] * D + 4 * g;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    *reinterpret_cast<half4_t*>(orow + 16 * cb) = __builtin_convertvector(acc[sb][cb] * invL[sb], half4_t);
            }
        }
    }
    if (!pass2) return;

    // ---- pass 2: the probabilities themselves, thresholds, counts ---------------------------
    // Scores are recomputed untransposed, so a lane holds ONE cache row and four queries per
    // block (4*g + r): the per-row count is a sum inside the lane plus one LDS atomic.  Each
    // query's maximum and 1/sum come from the lane that owned it in pass 1, through LDS.
    if (g == 0) {
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) {
            stat_m[WQ * w + 16 * sb + li] = m[sb];
            stat_inv[WQ * w + 16 * sb + li] = invL[sb];
            if constexpr (I4) {
                stat_q0[WQ * w + 16 * sb + li] = qsum0[sb];
                stat_q1[WQ * w + 16 * sb + li] = qsum1[sb];
            }
        }
    }
    for (int i = tid; i < ntiles * KB; i += 256) cnt_lds[i] = 0;
    __syncthreads();
    float qm[SB][4], qinv[SB][4], qtau[SB][4];
    int qlim[SB][4];
    // ring record: which of this lane's queries write their bit (real, see a row, and among the
    // last ring_bits steps of the run: an earlier step's bit is overwritten within the run)
    // and the bit the first query of each 16-block owns
    uint32_t qwrites[SB];
    int blk_bit[SB];
#pragma unroll
    for (int sb = 0; sb < SB; ++sb) {
        const int qbase = q0 + WQ * w + 16 * sb + 4 * g;  // this lane's first query of the block
        qwrites[sb] = 0;
        blk_bit[sb] = a.ring ? (int)((a.t0 + q0 + WQ * w + 16 * sb + 1) % a.ring_bits) : 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int si = WQ * w + 16 * sb + 4 * g + r;
            if (qbase + r < a.c && stat_lim[si] >= 0 && qbase + r >= a.c - a.ring_bits) qwrites[sb] |= 1u << r;
            qm[sb][r] = stat_m[si];
            qinv[sb][r] = stat_inv[si];
            qs0p[sb][r] = I4 ? stat_q0[si] : 0.f;
            qs1p[sb][r] = I4 ? stat_q1[si] : 0.f;
            qlim[sb][r] = stat_lim[si];
            // threshold 1/t (tokens seen at that step) or 1/(rows it sees)
            const long tq = a.thresh_len ? (long)qlim[sb][r] + 1 : a.t0 + qbase + r + 1;
            // a padding query (past the end of the run) or one that sees no row never counts: no
            // probability is below -1
            qtau[sb][r] = (qbase + r < a.c && qlim[sb][r] >= 0) ? __fdiv_rn(1.0f, (float)tq) : -1.0f;
        }
    }
    // Last tile first: it is still staged in LDS, and the K rows that pass 1 read last are the
    // ones most likely still in L2.
    for (int kt = ntiles - 1; kt >= 0; --kt) {
        if (kt != ntiles - 1) {
            __syncthreads();
            stage(false, kt);
            __syncthreads();
            if (kt > 0) fetch(kt - 1, false);
        }
        if (kt * KB > wave_lim) continue;
        float4_t d[SB][4];
        scores(Plain{}, d);
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            const int j = kt * KB + 16 * rb + li;
            int cnt = 0;
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                const bool diag = kt * KB + KB - 1 > sub_first_lim[sb];
                const int qbase = q0 + WQ * w + 16 * sb + 4 * g;
                float4_t p;
                uint32_t setn = 0, seen = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    p[r] = fast_exp2(fmaf(d[sb][rb][r], c2, -qm[sb][r])) * qinv[sb][r];
                    bool low = p[r] < qtau[sb][r];
                    const bool sees = !diag || j <= qlim[sb][r];
                    low = low && sees;
                    cnt += low ? 1 : 0;
                    setn |= (low ? 1u : 0u) << r;
                    seen |= (sees ? 1u : 0u) << r;
                }
                if (a.ring) {
                    // the 16 queries of the block: this lane's four sit at bits 4g .. 4g+3
                    uint32_t both = ((setn & qwrites[sb]) << (4 * g)) | ((seen & qwrites[sb]) << (4 * g + 16));
                    both |= (uint32_t)__shfl_xor((int)both, 16);
                    both |= (uint32_t)__shfl_xor((int)both, 32);
                    if (g == 0 && (both >> 16))
                        ring_write16(a.ring + (size_t)u * a.ring_words * a.C + j, a.C, blk_bit[sb], a.ring_bits,
                                     both & 0xFFFFu, both >> 16);
                }
                if (a.probs) {
                    float* pbase = a.probs + (size_t)u * a.probs_unit_stride + (size_t)qbase * a.C;
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (qbase + r < a.c && j <= qlim[sb][r]) pbase[(size_t)r * a.C + j] = p[r];
                }
            }
            if (cnt && !a.ring) atomicAdd(&cnt_lds[j], cnt);
        }
    }
    __syncthreads();
    if (!a.counted || a.ring) return;
    uint32_t* cw = reinterpret_cast<uint32_t*>(a.cnt + (size_t)u * a.cnt_unit_stride);
    for (int i = tid; 2 * i < hi; i += 256) {
        const uint32_t word = (uint32_t)cnt_lds[2 * i] | ((uint32_t)cnt_lds[2 * i + 1] << 16);
        if (word) atomicAdd(&cw[i], word);
    }
}


}  // namespace

hipError_t launch_prefill_chunk(const Layout& L, const ChunkArgs& c, hipStream_t stream) {
    const bool i4 = L.kv_dtype == KV_I4G64;
    if (i4) {
        const int rows_per_wg = 2048 / L.d;
        const dim3 grid_a(L.U, (c.c + rows_per_wg - 1) / rows_per_wg);
        auto* append = L.d == 64 ? append_rows_i4_kernel<64> : append_rows_i4_kernel<128>;
        append<<<grid_a, 256, 0, stream>>>(
            static_cast<const _Float16*>(c.k), static_cast<const _Float16*>(c.v), c.unit_stride,
            static_cast<unsigned char*>(L.K), static_cast<unsigned char*>(L.V),
            static_cast<uint32_t*>(L.K_meta), static_cast<uint32_t*>(L.V_meta), L.pos, L.C, c.n0, c.c,
            (int)c.t0);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    PrefillArgs a;
    a.q = c.q;
    a.unit_stride = c.unit_stride;
    a.K = L.K;
    a.V = L.V;
    a.K_meta = static_cast<const uint32_t*>(L.K_meta);
    a.V_meta = static_cast<const uint32_t*>(L.V_meta);
    a.out = c.out;
    a.out_unit_stride = c.out_unit_stride;
    a.probs = c.probs;
    a.probs_unit_stride = c.probs_unit_stride;
    a.cnt = L.cnt + (size_t)c.bucket * L.C;
    a.cnt_unit_stride = (long)L.E * L.C;
    a.C = L.C;
    a.n0 = c.n0;
    a.c = c.c;
    const bool f32 = L.kv_dtype == KV_F32;
    const bool wide = !i4 && !f32 && c.c > 64;  // two blocks of 16 queries per wave (4-bit: too many registers)
    a.nqb = wide ? (c.c + 127) / 128 : (c.c + 63) / 64;
    a.t0 = c.t0;
    a.counted = c.counted;
    a.thresh_len = c.thresh_len;
    a.qk_log2 = c.qk_log2;
    a.pos = nullptr;
    a.n_rows = 0;
    a.ring_w = 0;
    // fp16: the run's rows are written into their slots by the attention kernel itself
    a.k_run = i4 ? nullptr : c.k;
    a.v_run = i4 ? nullptr : c.v;
    a.pos_w = L.pos;
    a.ring = L.W32 ? reinterpret_cast<uint32_t*>(L.cnt) : nullptr;
    a.ring_words = L.W32;
    a.ring_bits = L.W32 ? L.w : (1 << 30);
    const size_t lds = (size_t)L.C * sizeof(int);
    const unsigned grid = (unsigned)L.U * (unsigned)a.nqb;
    if (f32 && L.d == 64)
        prefill_chunk_kernel<64, true, 1, false, true><<<grid, 256, lds, stream>>>(a);
    else if (f32)
        prefill_chunk_kernel<128, true, 1, false, true><<<grid, 256, lds, stream>>>(a);
    else if (i4 && L.d == 64)
        prefill_chunk_kernel<64, true, 1, true><<<grid, 256, lds, stream>>>(a);
    else if (i4)
        prefill_chunk_kernel<128, true, 1, true><<<grid, 256, lds, stream>>>(a);
    else if (L.d == 64 && wide)
        prefill_chunk_kernel<64, true, 2, false><<<grid, 256, lds, stream>>>(a);
    else if (L.d == 64)
        prefill_chunk_kernel<64, true, 1, false><<<grid, 256, lds, stream>>>(a);
    else if (wide)
        prefill_chunk_kernel<128, true, 2, false><<<grid, 256, lds, stream>>>(a);
    else
        prefill_chunk_kernel<128, true, 1, false><<<grid, 256, lds, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_store_queries(const Layout& L, const void* q, long unit_stride, int count, long t0,
                                hipStream_t stream) {
    const int eb = L.kv_dtype == KV_F32 ? 4 : 2;
    const int row16 = L.d * eb / 16;
    const char* src = static_cast<const char*>(q);
    if (count > L.w) {  // only the last w matter
        src += (size_t)(count - L.w) * L.d * eb;
        t0 += count - L.w;
        count = L.w;
    }
    const dim3 grid(L.U, (count * row16 + 255) / 256);
    store_queries_kernel<<<grid, 256, 0, stream>>>(src, unit_stride * eb, static_cast<char*>(L.Qh), L.w, row16,
                                                   count, t0);
    return hipGetLastError();
}

hipError_t launch_recompute_record(const Layout& L, const ReplayArgs& r, hipStream_t stream) {
    hipError_t err = launch_clear_counters(L, stream);
    if (err != hipSuccess) return err;
    const int W = r.t < (long)L.w ? (int)r.t : L.w;
    PrefillArgs a;
    a.q = L.Qh;
    a.unit_stride = (long)L.w * L.d;
    a.K = L.K;
    a.V = L.V;
    a.K_meta = static_cast<const uint32_t*>(L.K_meta);
    a.V_meta = static_cast<const uint32_t*>(L.V_meta);
    a.out = nullptr;
    a.out_unit_stride = 0;
    a.probs = r.probs;
    a.probs_unit_stride = r.probs_unit_stride ? r.probs_unit_stride : (long)W * L.C;
    a.cnt = L.cnt;
    a.cnt_unit_stride = (long)L.E * L.C;
    a.C = L.C;
    a.n0 = 0;
    a.c = W;
    const bool wide = L.kv_dtype == KV_F16 && W > 64;
    a.nqb = wide ? (W + 127) / 128 : (W + 63) / 64;
    a.t0 = r.t - W;
    a.counted = 1;
    a.thresh_len = r.thresh_len;
    a.qk_log2 = r.qk_log2;
    a.pos = L.pos;
    a.n_rows = r.n;
    a.ring_w = L.w;
    a.k_run = nullptr;
    a.v_run = nullptr;
    a.pos_w = nullptr;
    a.ring = nullptr;
    a.ring_words = 0;
    a.ring_bits = 1 << 30;
    const size_t lds = (size_t)L.C * sizeof(int);
    const unsigned grid = (unsigned)L.U * (unsigned)a.nqb;
    if (L.kv_dtype == KV_F32 && L.d == 64)
        prefill_chunk_kernel<64, false, 1, false, true><<<grid, 256, lds, stream>>>(a);
    else if (L.kv_dtype == KV_F32)
        prefill_chunk_kernel<128, false, 1, false, true><<<grid, 256, lds, stream>>>(a);
    else if (L.kv_dtype == KV_I4G64 && L.d == 64)
        prefill_chunk_kernel<64, false, 1, true><<<grid, 256, lds, stream>>>(a);
    else if (L.kv_dtype == KV_I4G64)
        prefill_chunk_kernel<128, false, 1, true><<<grid, 256, lds, stream>>>(a);
    else if (L.d == 64 && wide)
        prefill_chunk_kernel<64, false, 2, false><<<grid, 256, lds, stream>>>(a);
    else if (L.d == 64)
        prefill_chunk_kernel<64, false, 1, false><<<grid, 256, lds, stream>>>(a);
    else if (wide)
        prefill_chunk_kernel<128, false, 2, false><<<grid, 256, lds, stream>>>(a);
    else
        prefill_chunk_kernel<128, false, 1, false><<<grid, 256, lds, stream>>>(a);
    return hipGetLastError();
}

}  // namespace sc
