// Decode-step kernels for gfx950: row append (Alg. 1 "model update") and the budgeted
// attention estimator of Sec. 4.1 with the Alg. 2 importance record updated in the softmax
// epilogue (the online variant of Sec. 4.1 "Overhead Tradeoff").
//
// One workgroup owns one (sequence, head) unit.  K and V rows are streamed exactly once,
// together, with 16-byte loads per lane; a row of 16*LPR bytes is spread over LPR adjacent
// lanes, so one wave instruction fetches 64/LPR whole rows (1 KiB, fully coalesced).  Each
// lane group keeps a running softmax (max, sum, weighted value partial) that is rescaled only
// when the maximum moves; raw scores are parked in LDS so that, once the unit's global max
// and sum are known, the epilogue can form every probability, test it against the
// threshold, bump the counters and (optionally) dump the probabilities.
#include "sc_kernels.hpp"

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
    long q_stride;
    const void* K;
    const void* V;
    const void* K_meta;
    const void* V_meta;
    void* out;
    long out_stride;
    float* probs;
    uint16_t* cnt;  // current bucket of unit 0
    long cnt_unit_stride;
    int n, C;
    float qk_log2, tau;
    int counted;
};

template <typename T, int N>
union Frag {
    uint4 raw;
    T e[N];
};

// Merge the running softmax of lane groups / waves: (m, l, acc) <- combine with (mo, lo, acco).
__device__ __forceinline__ void merge_scales(float m, float mo, float& mn, float& a, float& b) {
    mn = fmaxf(m, mo);
    a = (m == mn) ? 1.0f : fast_exp2(m - mn);
    b = (mo == mn) ? 1.0f : fast_exp2(mo - mn);
}

// Shared tail of both attention kernels: combine the per-wave partials, write `out`, then the
// probability epilogue with the counter update.
template <typename TOut, int D, int NW>
__device__ __forceinline__ void finish_unit(const AttnArgs& a, int u, float* s_lds, float* part_m,
                                            float* part_l, float* part_acc) {
    const int tid = threadIdx.x;
    float M = part_m[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, part_m[w]);
    float Lsum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) Lsum += part_l[w] * fast_exp2(part_m[w] - M);
    const float invL = 1.0f / Lsum;
    if (a.out && tid < D) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) o += part_acc[w * D + tid] * fast_exp2(part_m[w] - M);
        ((TOut*)a.out)[(size_t)u * a.out_stride + tid] = (TOut)(o * invL);
    }
    uint16_t* cnt = a.cnt + (size_t)u * a.cnt_unit_stride;
    float* probs = a.probs ? a.probs + (size_t)u * a.C : nullptr;
    for (int j = tid; j < a.n; j += NW * 64) {
        const float p = fast_exp2(s_lds[j] - M) * invL;
        if (probs) probs[j] = p;
        if (a.counted && p < a.tau) cnt[j] = (uint16_t)(cnt[j] + 1);
    }
}

// ---------------------------------------------------------------------------------------
// fp32 / fp16 rows.
// ---------------------------------------------------------------------------------------
template <typename T, int D, int NW, int UNR>
__global__ void __launch_bounds__(NW * 64) attn_rows_kernel(AttnArgs a) {
    constexpr int EPL = 16 / (int)sizeof(T);  // elements per lane
    constexpr int LPR = D / EPL;              // lanes per row
    constexpr int RPW = 64 / LPR;             // rows per wave load
    constexpr int CHUNK = RPW * UNR;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* s_lds = reinterpret_cast<float*>(smem_raw);
    float* part_m = s_lds + a.C;
    float* part_l = part_m + NW;
    float* part_acc = part_l + NW;

    const int u = blockIdx.x;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = lane / LPR, c = lane % LPR;
    const int n = a.n;
    const T* Ku = (const T*)a.K + (size_t)u * a.C * D + c * EPL;
    const T* Vu = (const T*)a.V + (size_t)u * a.C * D + c * EPL;

    float qf[EPL];
    {
        Frag<T, EPL> qr;
        qr.raw = *reinterpret_cast<const uint4*>((const T*)a.q + (size_t)u * a.q_stride + c * EPL);
#pragma unroll
        for (int i = 0; i < EPL; ++i) qf[i] = (float)qr.e[i] * a.qk_log2;
    }
    float m = -INFINITY, l = 0.f, acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;

    for (int base = wv * CHUNK; base < n; base += NW * CHUNK) {
        Frag<T, EPL> kr[UNR], vr[UNR];
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            const int j = base + x * RPW + g;
            const int jj = j < n ? j : n - 1;
            kr[x].raw = *reinterpret_cast<const uint4*>(Ku + (size_t)jj * D);
            vr[x].raw = *reinterpret_cast<const uint4*>(Vu + (size_t)jj * D);
        }
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            const int j = base + x * RPW + g;
            const bool valid = j < n;
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < EPL; ++i) s = fmaf((float)kr[x].e[i], qf[i], s);
            s = group_sum<LPR>(s);
            if (valid && c == 0) s_lds[j] = s;
            if (valid && s > m) {
                const float al = fast_exp2(m - s);
                l *= al;
#pragma unroll
                for (int i = 0; i < EPL; ++i) acc[i] *= al;
                m = s;
            }
            const float e = valid ? fast_exp2(s - m) : 0.f;
            l += e;
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] = fmaf(e, (float)vr[x].e[i], acc[i]);
        }
    }
    // lane groups of one wave
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
        const float mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
        float mn, sa, sb;
        merge_scales(m, mo, mn, sa, sb);
        l = l * sa + lo * sb;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] = acc[i] * sa + __shfl_xor(acc[i], off) * sb;
        m = mn;
    }
    if (g == 0) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) part_acc[wv * D + c * EPL + i] = acc[i];
        if (c == 0) {
            part_m[wv] = m;
            part_l[wv] = l;
        }
    }
    __syncthreads();
    finish_unit<T, D, NW>(a, u, s_lds, part_m, part_l, part_acc);
}

// ---------------------------------------------------------------------------------------
// 4-bit rows: 16 bytes of codes (32 channels) per lane, D/32 lanes per row, one
// (scale, zero) fp16 pair per 64 channels.  value = code*scale + zero, so
//   <q, k>   = sum_groups scale_g * sum_c q_c*code_c + zero_g * sum_c q_c
//   sum_j p_j v_j[c] = sum_j (p_j*scale_jg) * code_jc + sum_j p_j*zero_jg
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float2 unpack_meta(uint32_t w) {
    union {
        uint32_t u;
        _Float16 h[2];
    } cv;
    cv.u = w;
    return make_float2((float)cv.h[0], (float)cv.h[1]);
}

template <int D, int NW, int UNR>
__global__ void __launch_bounds__(NW * 64) attn_i4_kernel(AttnArgs a) {
    constexpr int LPR = D / 32;
    constexpr int RPW = 64 / LPR;
    constexpr int GPR = D / 64;  // groups per row
    constexpr int CHUNK = RPW * UNR;
    constexpr int ROWB = D / 2;  // bytes of codes per row
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* s_lds = reinterpret_cast<float*>(smem_raw);
    float* part_m = s_lds + a.C;
    float* part_l = part_m + NW;
    float* part_acc = part_l + NW;

    const int u = blockIdx.x;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = lane / LPR, c = lane % LPR;
    const int gi = c / 2;  // 64-channel group this lane's 32 channels fall in
    const int n = a.n;
    const unsigned char* Ku = (const unsigned char*)a.K + (size_t)u * a.C * ROWB + c * 16;
    const unsigned char* Vu = (const unsigned char*)a.V + (size_t)u * a.C * ROWB + c * 16;
    const uint32_t* Km = (const uint32_t*)a.K_meta + (size_t)u * a.C * GPR + gi;
    const uint32_t* Vm = (const uint32_t*)a.V_meta + (size_t)u * a.C * GPR + gi;

    float qf[32];
    float qsum = 0.f;
    {
        const _Float16* qu = (const _Float16*)a.q + (size_t)u * a.q_stride + c * 32;
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            Frag<_Float16, 8> qr;
            qr.raw = *reinterpret_cast<const uint4*>(qu + v4 * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                qf[v4 * 8 + i] = (float)qr.e[i] * a.qk_log2;
                qsum += qf[v4 * 8 + i];
            }
        }
    }
    float m = -INFINITY, l = 0.f, zacc = 0.f, acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = 0.f;

    for (int base = wv * CHUNK; base < n; base += NW * CHUNK) {
        uint4 kr[UNR], vr[UNR];
        uint32_t km[UNR], vm[UNR];
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            const int j = base + x * RPW + g;
            const int jj = j < n ? j : n - 1;
            kr[x] = *reinterpret_cast<const uint4*>(Ku + (size_t)jj * ROWB);
            vr[x] = *reinterpret_cast<const uint4*>(Vu + (size_t)jj * ROWB);
            km[x] = Km[(size_t)jj * GPR];
            vm[x] = Vm[(size_t)jj * GPR];
        }
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            const int j = base + x * RPW + g;
            const bool valid = j < n;
            const uint32_t kw[4] = {kr[x].x, kr[x].y, kr[x].z, kr[x].w};
            float dotc = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w)
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    dotc = fmaf((float)((kw[w] >> (4 * k)) & 15u), qf[w * 8 + k], dotc);
            const float2 kmeta = unpack_meta(km[x]);
            float s = group_sum<LPR>(fmaf(kmeta.x, dotc, kmeta.y * qsum));
            if (valid && c == 0) s_lds[j] = s;
            if (valid && s > m) {
                const float al = fast_exp2(m - s);
                l *= al;
                zacc *= al;
#pragma unroll
                for (int i = 0; i < 32; ++i) acc[i] *= al;
                m = s;
            }
            const float e = valid ? fast_exp2(s - m) : 0.f;
            l += e;
            const float2 vmeta = unpack_meta(vm[x]);
            const float es = e * vmeta.x;
            zacc = fmaf(e, vmeta.y, zacc);
            const uint32_t vw[4] = {vr[x].x, vr[x].y, vr[x].z, vr[x].w};
#pragma unroll
            for (int w = 0; w < 4; ++w)
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    acc[w * 8 + k] = fmaf(es, (float)((vw[w] >> (4 * k)) & 15u), acc[w * 8 + k]);
        }
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] += zacc;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
        const float mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
        float mn, sa, sb;
        merge_scales(m, mo, mn, sa, sb);
        l = l * sa + lo * sb;
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[i] = acc[i] * sa + __shfl_xor(acc[i], off) * sb;
        m = mn;
    }
    if (g == 0) {
#pragma unroll
        for (int i = 0; i < 32; ++i) part_acc[wv * D + c * 32 + i] = acc[i];
        if (c == 0) {
            part_m[wv] = m;
            part_l[wv] = l;
        }
    }
    __syncthreads();
    finish_unit<_Float16, D, NW>(a, u, s_lds, part_m, part_l, part_acc);
}

// ---------------------------------------------------------------------------------------
// Append: copy (or quantise) this step's k/v row into slot n-1 and record its position.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(64) append_rows_kernel(const T* k_new, const T* v_new, long in_stride,
                                                         T* K, T* V, int32_t* pos, int C, int slot,
                                                         int pos_value) {
    constexpr int EPL = 16 / (int)sizeof(T);
    constexpr int LPR = D / EPL;
    const int u = blockIdx.x, lane = threadIdx.x;
    if (lane < LPR) {
        *reinterpret_cast<uint4*>(K + ((size_t)u * C + slot) * D + lane * EPL) =
            *reinterpret_cast<const uint4*>(k_new + (size_t)u * in_stride + lane * EPL);
    } else if (lane < 2 * LPR) {
        const int c = lane - LPR;
        *reinterpret_cast<uint4*>(V + ((size_t)u * C + slot) * D + c * EPL) =
            *reinterpret_cast<const uint4*>(v_new + (size_t)u * in_stride + c * EPL);
    }
    if (lane == 63) pos[(size_t)u * C + slot] = pos_value;
}

// 4-bit append.  Wave 0 quantises the key row, wave 1 the value row; lane i owns channels
// 2i and 2i+1 (one byte of codes).  Every operation is a single IEEE fp32 operation so the
// codes are reproducible: zero = min, scale = fp16((max-min)/15) (1 when that is 0),
// code = clamp(rint((x-zero)/scale), 0, 15).
template <int D>
__global__ void __launch_bounds__(128) append_i4_kernel(const _Float16* k_new, const _Float16* v_new,
                                                        long in_stride, unsigned char* K,
                                                        unsigned char* V, uint32_t* K_meta,
                                                        uint32_t* V_meta, int32_t* pos, int C, int slot,
                                                        int pos_value) {
    constexpr int GPR = D / 64;
    const int u = blockIdx.x, lane = threadIdx.x & 63, which = threadIdx.x >> 6;
    const _Float16* src = (which ? v_new : k_new) + (size_t)u * in_stride;
    unsigned char* dst = (which ? V : K) + ((size_t)u * C + slot) * (D / 2);
    uint32_t* meta = (which ? V_meta : K_meta) + ((size_t)u * C + slot) * GPR;
    if (lane < D / 2) {
        const float x0 = (float)src[2 * lane], x1 = (float)src[2 * lane + 1];
        float mn = fminf(x0, x1), mx = fmaxf(x0, x1);
#pragma unroll
        for (int off = 1; off < 32; off <<= 1) {
            mn = fminf(mn, __shfl_xor(mn, off));
            mx = fmaxf(mx, __shfl_xor(mx, off));
        }
        const float range = __fsub_rn(mx, mn);
        _Float16 sh = (_Float16)__fdiv_rn(range, 15.0f);
        float s = (float)sh;
        if (s == 0.0f) {
            s = 1.0f;
            sh = (_Float16)1.0f;
        }
        const _Float16 zh = (_Float16)mn;
        const float z = (float)zh;
        float c0 = rintf(__fdiv_rn(__fsub_rn(x0, z), s));
        float c1 = rintf(__fdiv_rn(__fsub_rn(x1, z), s));
        c0 = fminf(fmaxf(c0, 0.f), 15.f);
        c1 = fminf(fmaxf(c1, 0.f), 15.f);
        dst[lane] = (unsigned char)((uint32_t)c0 | ((uint32_t)c1 << 4));
        if ((lane & 31) == 0) {
            union {
                uint32_t u32;
                _Float16 h[2];
            } cv;
            cv.h[0] = sh;
            cv.h[1] = zh;
            meta[lane >> 5] = cv.u32;
        }
    }
    if (threadIdx.x == 127) pos[(size_t)u * C + slot] = pos_value;
}

__global__ void clear_u32_kernel(uint32_t* p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0u;
}

template <typename T, int D, int UNR>
hipError_t launch_rows(const AttnArgs& a, int U, int nw, hipStream_t stream) {
    const size_t lds = ((size_t)a.C + 2 * nw + (size_t)nw * D) * sizeof(float);
    switch (nw) {
        case 4: attn_rows_kernel<T, D, 4, UNR><<<U, 256, lds, stream>>>(a); break;
        case 8: attn_rows_kernel<T, D, 8, UNR><<<U, 512, lds, stream>>>(a); break;
        default: attn_rows_kernel<T, D, 16, UNR><<<U, 1024, lds, stream>>>(a); break;
    }
    return hipGetLastError();
}

template <int D, int UNR>
hipError_t launch_i4(const AttnArgs& a, int U, int nw, hipStream_t stream) {
    const size_t lds = ((size_t)a.C + 2 * nw + (size_t)nw * D) * sizeof(float);
    switch (nw) {
        case 4: attn_i4_kernel<D, 4, UNR><<<U, 256, lds, stream>>>(a); break;
        case 8: attn_i4_kernel<D, 8, UNR><<<U, 512, lds, stream>>>(a); break;
        default: attn_i4_kernel<D, 16, UNR><<<U, 1024, lds, stream>>>(a); break;
    }
    return hipGetLastError();
}

// Waves per workgroup: enough waves chip-wide (256 CUs) to keep many loads in flight even
// when there are few units.
int pick_waves(int U) {
    if (U >= 2048) return 4;
    if (U >= 1024) return 8;
    return 16;
}

}  // namespace

hipError_t launch_decode_step(const Layout& L, const StepArgs& s, hipStream_t stream) {
    const int slot = s.n - 1;
    hipError_t err;
    if (L.kv_dtype == KV_F32) {
        if (L.d == 64)
            append_rows_kernel<float, 64><<<L.U, 64, 0, stream>>>(
                (const float*)s.k_new, (const float*)s.v_new, s.in_stride, (float*)L.K, (float*)L.V,
                L.pos, L.C, slot, s.pos_value);
        else
            append_rows_kernel<float, 128><<<L.U, 64, 0, stream>>>(
                (const float*)s.k_new, (const float*)s.v_new, s.in_stride, (float*)L.K, (float*)L.V,
                L.pos, L.C, slot, s.pos_value);
    } else if (L.kv_dtype == KV_F16) {
        if (L.d == 64)
            append_rows_kernel<_Float16, 64><<<L.U, 64, 0, stream>>>(
                (const _Float16*)s.k_new, (const _Float16*)s.v_new, s.in_stride, (_Float16*)L.K,
                (_Float16*)L.V, L.pos, L.C, slot, s.pos_value);
        else
            append_rows_kernel<_Float16, 128><<<L.U, 64, 0, stream>>>(
                (const _Float16*)s.k_new, (const _Float16*)s.v_new, s.in_stride, (_Float16*)L.K,
                (_Float16*)L.V, L.pos, L.C, slot, s.pos_value);
    } else {
        if (L.d == 64)
            append_i4_kernel<64><<<L.U, 128, 0, stream>>>(
                (const _Float16*)s.k_new, (const _Float16*)s.v_new, s.in_stride, (unsigned char*)L.K,
                (unsigned char*)L.V, (uint32_t*)L.K_meta, (uint32_t*)L.V_meta, L.pos, L.C, slot,
                s.pos_value);
        else
            append_i4_kernel<128><<<L.U, 128, 0, stream>>>(
                (const _Float16*)s.k_new, (const _Float16*)s.v_new, s.in_stride, (unsigned char*)L.K,
                (unsigned char*)L.V, (uint32_t*)L.K_meta, (uint32_t*)L.V_meta, L.pos, L.C, slot,
                s.pos_value);
    }
    err = hipGetLastError();
    if (err != hipSuccess) return err;

    AttnArgs a;
    a.q = s.q;
    a.q_stride = s.in_stride;
    a.K = L.K;
    a.V = L.V;
    a.K_meta = L.K_meta;
    a.V_meta = L.V_meta;
    a.out = s.out;
    a.out_stride = s.out_stride;
    a.probs = s.probs;
    a.cnt = L.cnt + (size_t)s.bucket * L.C;
    a.cnt_unit_stride = (long)L.E * L.C;
    a.n = s.n;
    a.C = L.C;
    a.qk_log2 = s.qk_log2;
    a.tau = s.tau;
    a.counted = s.counted;
    const int nw = pick_waves(L.U);
    if (L.kv_dtype == KV_F32)
        return L.d == 64 ? launch_rows<float, 64, 4>(a, L.U, nw, stream)
                         : launch_rows<float, 128, 4>(a, L.U, nw, stream);
    if (L.kv_dtype == KV_F16)
        return L.d == 64 ? launch_rows<_Float16, 64, 4>(a, L.U, nw, stream)
                         : launch_rows<_Float16, 128, 4>(a, L.U, nw, stream);
    return L.d == 64 ? launch_i4<64, 2>(a, L.U, nw, stream) : launch_i4<128, 2>(a, L.U, nw, stream);
}

hipError_t launch_clear_counters(const Layout& L, hipStream_t stream) {
    const size_t words = (size_t)L.U * L.E * L.C / 2;  // C is even
    clear_u32_kernel<<<1024, 256, 0, stream>>>(reinterpret_cast<uint32_t*>(L.cnt), words);
    return hipGetLastError();
}

}  // namespace sc
