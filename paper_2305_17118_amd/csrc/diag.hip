// Diagnostics the paper plots, computed on the device from dumped probabilities (gfx950).
//  * Persistence ratio (Sec. 3.1, "Verification"): a token is pivotal for position t when it
//    receives more than 1/t of that position's attention; S(0->t) and S(t+1->l) are the unions
//    of the pivotal sets over the first and the later positions, both restricted to the
//    tokens x_1..x_t; the ratio is |S(t+1->l) ^ S(0->t)| / |S(t+1->l)|.
//  * Attention kept by the budgeted cache (ablation on the attention score error, Sec. 5): by
//    the restricted-softmax identity in the proof of Lemma A.4 every surviving token's score
//    is the full-attention score divided by the attention mass the survivors hold, so the
//    change ratio (a_s - a_o)/a_o is 1/mass - 1 for every survivor and -1 for every evicted
//    token; the mass is the one number to measure.
#include "sc_kernels.hpp"

namespace sc {
namespace {

// One workgroup per unit; thread j owns token j < split and walks down its column.
// counts[u] = {|S_first|, |S_later|, |S_first ^ S_later|} over tokens [0, split).
__global__ void __launch_bounds__(256)
persistence_kernel(const float* __restrict__ probs, int length, long row_stride, long unit_stride, int split,
                   int32_t* __restrict__ counts) {
    __shared__ int tot[3];
    if (threadIdx.x < 3) tot[threadIdx.x] = 0;
    __syncthreads();
    const float* pu = probs + (size_t)blockIdx.x * unit_stride;
    int c_first = 0, c_later = 0, c_both = 0;
    for (int j = threadIdx.x; j < split; j += 256) {
        bool first = false, later = false;
        for (int i = j; i < length; ++i) {  // position i (0-based) sees tokens 0..i; t = i+1 tokens seen
            const bool pivotal = pu[(size_t)i * row_stride + j] > __fdiv_rn(1.0f, (float)(i + 1));
            first = first || (pivotal && i < split);
            later = later || (pivotal && i >= split);
        }
        c_first += first;
        c_later += later;
        c_both += first && later;
    }
    atomicAdd(&tot[0], c_first);
    atomicAdd(&tot[1], c_later);
    atomicAdd(&tot[2], c_both);
    __syncthreads();
    if (threadIdx.x < 3) counts[(size_t)blockIdx.x * 3 + threadIdx.x] = tot[threadIdx.x];
}

// One workgroup per unit: mass[u] = sum over resident slots j < n of full[u][pos[u][j]].
__global__ void __launch_bounds__(256)
kept_mass_kernel(const int32_t* __restrict__ pos, int C, int n, const float* __restrict__ full,
                 long unit_stride, float* __restrict__ mass) {
    __shared__ float part[4];
    const int u = blockIdx.x;
    float acc = 0.f;
    for (int j = threadIdx.x; j < n; j += 256) acc += full[(size_t)u * unit_stride + pos[(size_t)u * C + j]];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) mass[u] = (part[0] + part[1]) + (part[2] + part[3]);
}

// What reading a buffer and nothing else reaches on this chip: every thread fetches 16 bytes
// at a time, eight loads in flight, workgroup b owns the b-th contiguous share of the buffer.
// The reference point for the decode kernels' fraction of peak (they can at best stream their
// bytes this fast).  The loaded words are folded into a value that is stored only if it equals
// a constant it never equals in practice, so that the loads cannot be dropped.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <bool NT>
__global__ void __launch_bounds__(256)
read_stream_kernel(const u32x4_t* __restrict__ p, size_t pieces_per_wg, uint32_t* __restrict__ sink) {
    constexpr int UNR = 8;
    const u32x4_t* base = p + (size_t)blockIdx.x * pieces_per_wg;
    uint32_t acc = 0;
    for (size_t i = threadIdx.x; i + (UNR - 1) * 256 < pieces_per_wg; i += UNR * 256) {
        u32x4_t r[UNR];
#pragma unroll
        for (int x = 0; x < UNR; ++x) r[x] = NT ? __builtin_nontemporal_load(base + i + x * 256) : base[i + x * 256];
#pragma unroll
        for (int x = 0; x < UNR; ++x) acc ^= r[x].x ^ r[x].y ^ r[x].z ^ r[x].w;
    }
    if (acc == 0x9E3779B9u) *sink = acc;
}

}  // namespace

hipError_t launch_read_stream(const void* buf, size_t bytes, bool nontemporal, uint32_t* sink, hipStream_t stream) {
    const size_t pieces_per_wg = bytes / 16 / 1024;  // bytes is a multiple of 1024 * 8 * 256 * 16
    if (nontemporal)
        read_stream_kernel<true><<<1024, 256, 0, stream>>>(static_cast<const u32x4_t*>(buf), pieces_per_wg, sink);
    else
        read_stream_kernel<false><<<1024, 256, 0, stream>>>(static_cast<const u32x4_t*>(buf), pieces_per_wg, sink);
    return hipGetLastError();
}

hipError_t launch_persistence(const float* probs, int units, int length, long row_stride, long unit_stride,
                              int split, int32_t* counts, hipStream_t stream) {
    persistence_kernel<<<units, 256, 0, stream>>>(probs, length, row_stride, unit_stride, split, counts);
    return hipGetLastError();
}

hipError_t launch_kept_mass(const Layout& L, int n, const float* full, long unit_stride, float* mass,
                            hipStream_t stream) {
    kept_mass_kernel<<<L.U, 256, 0, stream>>>(L.pos, L.C, n, full, unit_stride, mass);
    return hipGetLastError();
}

}  // namespace sc
