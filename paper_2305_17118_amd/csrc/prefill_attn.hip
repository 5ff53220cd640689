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
// fp16 storage only.  Two kernels per run: the rows are copied into their slots first, then
// one workgroup per (unit, 64 queries) makes two passes over the visible rows in tiles of 64:
// pass 1 is the usual running-softmax attention (scores and P.V on v_mfma_f32_16x16x32_f16),
// pass 2 recomputes the scores against the final maximum and sum to form the very
// probabilities the threshold is applied to, counts the low ones per cache row and adds the
// counts to the 16-bit counters (two per 32-bit atomic).
#include "sc_kernels.hpp"

namespace sc {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Copy the run's key/value rows into slots n0.. of every unit and record their positions.
// grid (U, pieces/256): one 16-byte piece of a K row and of a V row per thread.
__global__ void __launch_bounds__(256)
append_rows_kernel(const char* __restrict__ k, const char* __restrict__ v, long unit_stride_bytes,
                   char* __restrict__ K, char* __restrict__ V, int32_t* __restrict__ pos, int C,
                   int row16, int n0, int c, int t0) {
    const int u = blockIdx.x;
    const int e = blockIdx.y * 256 + threadIdx.x;
    if (e >= c * row16) return;
    const int row = e / row16;
    const size_t src = (size_t)u * unit_stride_bytes + (size_t)e * 16;
    const size_t dst = ((size_t)u * C + n0) * row16 * 16 + (size_t)e * 16;
    *reinterpret_cast<uint4*>(K + dst) = *reinterpret_cast<const uint4*>(k + src);
    *reinterpret_cast<uint4*>(V + dst) = *reinterpret_cast<const uint4*>(v + src);
    if (e - row * row16 == 0) pos[(size_t)u * C + n0 + row] = t0 + row;
}

struct PrefillArgs {
    const _Float16* q;
    long unit_stride;
    const _Float16* K;
    const _Float16* V;
    _Float16* out;
    long out_unit_stride;
    float* probs;
    long probs_unit_stride;
    uint16_t* cnt;  // current bucket of unit 0
    long cnt_unit_stride;
    int C, n0, c, nqb;
    long t0;
    int counted, thresh_len;
    float qk_log2;
};

// Matrix-instruction operand layout (16x16x32, fp16 in, fp32 out), lane l, i = l%16, g = l/16:
//   A: lane holds A[i][8g .. 8g+7]      B: lane holds B[8g .. 8g+7][i]      D: lane holds D[4g + r][i]
// Scores are computed transposed, S^T = K Q^T (A = 16 cache rows, B = 16 queries), so a lane
// ends up with four consecutive cache rows of ONE query: softmax statistics are per lane
// (plus a reduction over g), and the probabilities are already laid out as the B operand of
// out^T = V^T P^T, whose contraction index (lane group g, element e) stands for cache row
// 4g + e of one 16-row block (e < 4) or of the next one (e >= 4).  V is staged transposed in
// LDS so that its A operand is two 8-byte reads.
template <int D>
__global__ void __launch_bounds__(256) prefill_chunk_kernel(PrefillArgs a) {
    constexpr int KB = 64;        // cache rows per tile
    constexpr int QB = 64;        // queries per workgroup (16 per wave)
    constexpr int LDK = D + 8;    // halfs per staged K row (padding keeps 16-byte reads conflict-free)
    constexpr int LDV = KB + 4;   // halfs per channel of the transposed V tile
    constexpr int KS = D / 32;    // matrix instructions per 16 scores
    constexpr int CB = D / 16;    // 16-channel blocks of the output
    constexpr int PIECES = KB * D / 8 / 256;  // 16-byte pieces of a tile per thread
    __shared__ __align__(16) _Float16 Ks[KB * LDK];
    __shared__ __align__(16) _Float16 Vt[D * LDV];
    extern __shared__ int cnt_lds[];  // [tiles * 64] low-score counts of this workgroup's queries

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int li = lane & 15, g = lane >> 4;
    const int u = blockIdx.x / a.nqb;
    const int q0 = (a.nqb - 1 - (int)(blockIdx.x % a.nqb)) * QB;  // longest query blocks first
    const int qi = q0 + 16 * w + li;                 // this lane's query (position in the run)
    const int qc = qi < a.c ? qi : a.c - 1;          // clamped: padding lanes shadow the last query
    const int lim = a.n0 + qc;                       // last cache row query qc sees
    const int q_last = (q0 + QB < a.c ? q0 + QB : a.c) - 1;
    const int hi = a.n0 + q_last + 1;                // rows visible to this workgroup
    const int ntiles = (hi + KB - 1) / KB;
    const int wave_lim = a.n0 + (q0 + 16 * w + 15 < a.c ? q0 + 16 * w + 15 : a.c - 1);

    const _Float16* Kb = a.K + (size_t)u * a.C * D;
    const _Float16* Vb = a.V + (size_t)u * a.C * D;

    half8_t qB[KS];
    {
        const _Float16* qrow = a.q + (size_t)u * a.unit_stride + (size_t)qc * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qB[ks] = *reinterpret_cast<const half8_t*>(qrow + 32 * ks);
    }

    auto load_tile = [&](int kt, bool with_v) {
#pragma unroll
        for (int x = 0; x < PIECES; ++x) {
            const int idx = tid + 256 * x;
            const int row = idx / (D / 8), cb8 = idx % (D / 8);
            int grow = kt * KB + row;
            grow = grow < hi ? grow : hi - 1;  // stay inside rows that hold data
            const size_t off = (size_t)grow * D + cb8 * 8;
            *reinterpret_cast<uint4*>(&Ks[row * LDK + cb8 * 8]) = *reinterpret_cast<const uint4*>(Kb + off);
            if (with_v) {
                const half8_t vv = *reinterpret_cast<const half8_t*>(Vb + off);
#pragma unroll
                for (int e = 0; e < 8; ++e) Vt[(cb8 * 8 + e) * LDV + row] = vv[e];
            }
        }
    };
    // d[rb][r] = <k_j, q> for cache row j = 64*kt + 16*rb + 4*g + r and this lane's query
    auto scores = [&](float4_t (&d)[4]) {
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) d[rb] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const half8_t A = *reinterpret_cast<const half8_t*>(&Ks[(16 * rb + li) * LDK + 32 * ks + 8 * g]);
                d[rb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, qB[ks], d[rb], 0, 0, 0);
            }
    };

    // ---- pass 1: running softmax and P.V --------------------------------------------------
    float m = -INFINITY, l32 = 0.f, l16 = 0.f;
    float4_t acc[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) acc[cb] = float4_t{0.f, 0.f, 0.f, 0.f};
    for (int kt = 0; kt < ntiles; ++kt) {
        __syncthreads();
        load_tile(kt, true);
        __syncthreads();
        if (kt * KB > wave_lim) continue;  // nothing in this tile is visible to this wave
        float4_t d[4];
        scores(d);
        float tmax = -INFINITY;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = kt * KB + 16 * rb + 4 * g + r;
                const float s = j <= lim ? d[rb][r] * a.qk_log2 : -INFINITY;
                d[rb][r] = s;
                tmax = fmaxf(tmax, s);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m, tmax);  // finite: row 0 of tile 0 is visible to every query
        const float alpha = fast_exp2(m - m_new);
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0ull) {
            l32 *= alpha;
            l16 *= alpha;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) acc[cb] *= alpha;
        }
        m = m_new;
        half4_t ph[4];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = fast_exp2(d[rb][r] - m);
                const _Float16 p16 = (_Float16)p;
                l32 += p;
                l16 += (float)p16;
                ph[rb][r] = p16;
            }
#pragma unroll
        for (int kp = 0; kp < 2; ++kp) {
            const half8_t B = __builtin_shufflevector(ph[2 * kp], ph[2 * kp + 1], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const _Float16* vrow = &Vt[(16 * cb + li) * LDV + 32 * kp + 4 * g];
                const half4_t a0 = *reinterpret_cast<const half4_t*>(vrow);
                const half4_t a1 = *reinterpret_cast<const half4_t*>(vrow + 16);
                const half8_t A = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(A, B, acc[cb], 0, 0, 0);
            }
        }
    }
    l32 += __shfl_xor(l32, 16);
    l32 += __shfl_xor(l32, 32);
    l16 += __shfl_xor(l16, 16);
    l16 += __shfl_xor(l16, 32);
    if (a.out && qi < a.c) {
        const float inv = 1.0f / l16;
        _Float16* orow = a.out + (size_t)u * a.out_unit_stride + (size_t)qi * D + 4 * g;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            half4_t o;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (_Float16)(acc[cb][r] * inv);
            *reinterpret_cast<half4_t*>(orow + 16 * cb) = o;
        }
    }
    if (!a.counted && !a.probs) return;

    // ---- pass 2: the probabilities themselves, thresholds, counts ---------------------------
    for (int i = tid; i < ntiles * KB; i += 256) cnt_lds[i] = 0;
    const float invL = 1.0f / l32;
    const long tq = a.thresh_len ? (long)a.n0 + qi + 1 : a.t0 + qi + 1;
    const float tau = __fdiv_rn(1.0f, (float)tq);
    const bool real = qi < a.c;
    float* prow = a.probs ? a.probs + (size_t)u * a.probs_unit_stride + (size_t)qc * a.C : nullptr;
    const int rb_l = lane >> 4, g_l = (lane >> 2) & 3, r_l = lane & 3;  // the tile row this lane counts for
    for (int kt = 0; kt < ntiles; ++kt) {
        __syncthreads();
        load_tile(kt, false);
        __syncthreads();
        if (kt * KB > wave_lim) continue;
        float4_t d[4];
        scores(d);
        uint32_t mine = 0;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            const int j0 = kt * KB + 16 * rb + 4 * g;
            float4_t p;
#pragma unroll
            for (int r = 0; r < 4; ++r) p[r] = fast_exp2(d[rb][r] * a.qk_log2 - m) * invL;
            if (prow && real) {
                if (j0 + 3 <= lim) {
                    *reinterpret_cast<float4_t*>(prow + j0) = p;
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (j0 + r <= lim) prow[j0 + r] = p[r];
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool low = real && (j0 + r <= lim) && (p[r] < tau);
                const unsigned long long bal = __builtin_amdgcn_ballot_w64(low);
                const uint32_t half = (g_l & 2) ? (uint32_t)(bal >> 32) : (uint32_t)bal;
                const uint32_t cnt = __popc((half >> ((g_l & 1) * 16)) & 0xFFFFu);
                mine = (rb == rb_l && r == r_l) ? cnt : mine;
            }
        }
        if (mine) atomicAdd(&cnt_lds[kt * KB + lane], (int)mine);
    }
    __syncthreads();
    if (!a.counted) return;
    uint32_t* cw = reinterpret_cast<uint32_t*>(a.cnt + (size_t)u * a.cnt_unit_stride);
    for (int i = tid; 2 * i < hi; i += 256) {
        const uint32_t word = (uint32_t)cnt_lds[2 * i] | ((uint32_t)cnt_lds[2 * i + 1] << 16);
        if (word) atomicAdd(&cw[i], word);
    }
}

}  // namespace

bool prefill_chunk_supported(const Layout& L) {
    return L.kv_dtype == KV_F16 && L.E > 0 && L.C <= 6144;
}

hipError_t launch_prefill_chunk(const Layout& L, const ChunkArgs& c, hipStream_t stream) {
    const int row16 = L.d * 2 / 16;
    const dim3 grid_a(L.U, (c.c * row16 + 255) / 256);
    append_rows_kernel<<<grid_a, 256, 0, stream>>>(
        static_cast<const char*>(c.k), static_cast<const char*>(c.v), c.unit_stride * 2,
        static_cast<char*>(L.K), static_cast<char*>(L.V), L.pos, L.C, row16, c.n0, c.c, (int)c.t0);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    PrefillArgs a;
    a.q = static_cast<const _Float16*>(c.q);
    a.unit_stride = c.unit_stride;
    a.K = static_cast<const _Float16*>(L.K);
    a.V = static_cast<const _Float16*>(L.V);
    a.out = static_cast<_Float16*>(c.out);
    a.out_unit_stride = c.out_unit_stride;
    a.probs = c.probs;
    a.probs_unit_stride = c.probs_unit_stride;
    a.cnt = L.cnt + (size_t)c.bucket * L.C;
    a.cnt_unit_stride = (long)L.E * L.C;
    a.C = L.C;
    a.n0 = c.n0;
    a.c = c.c;
    a.nqb = (c.c + 63) / 64;
    a.t0 = c.t0;
    a.counted = c.counted;
    a.thresh_len = c.thresh_len;
    a.qk_log2 = c.qk_log2;
    const size_t lds = (size_t)L.C * sizeof(int);
    const unsigned grid = (unsigned)L.U * (unsigned)a.nqb;
    if (L.d == 64)
        prefill_chunk_kernel<64><<<grid, 256, lds, stream>>>(a);
    else
        prefill_chunk_kernel<128><<<grid, 256, lds, stream>>>(a);
    return hipGetLastError();
}

}  // namespace sc
