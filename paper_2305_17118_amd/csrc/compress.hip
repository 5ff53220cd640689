// Compression kernels for gfx950 (Alg. 2): per-unit selection of the m rows with the largest
// importance record outside the recent window, then stable in-place compaction of every
// per-row array.  All of it is integer / byte work and exact.
#include "sc_kernels.hpp"

#include <mutex>

namespace sc {
namespace {

// Scratch owned by the library (select -> compact hand-over: `first` then `srcmap`), for the
// one entry point whose callers cannot provide or allocate any.  In host code this name is
// only a handle for hipGetSymbolAddress; every device holds its own copy at its own address,
// looked up once per device in static_scratch() below.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, null until looked up

constexpr int SEL_THREADS = 256;
constexpr int SEL_WAVES = SEL_THREADS / 64;

// Exclusive prefix of a 0/1 flag over the workgroup in thread order; returns this thread's
// prefix and the workgroup total.  `wave_tot` is LDS scratch of SEL_WAVES ints.
__device__ __forceinline__ int block_prefix(bool flag, int* wave_tot, int& total) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const unsigned long long bal = __ballot(flag);
    const int in_wave = __popcll(bal & ((1ull << lane) - 1ull));
    __syncthreads();  // previous use of wave_tot is over
    if (lane == 0) wave_tot[wv] = __popcll(bal);
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) {
        const int v = wave_tot[w];
        before += (w < wv) ? v : 0;
        tot += v;
    }
    total = tot;
    return before + in_wave;
}

// Among 256 histogram bins (LDS, one per thread) find the bin b with
//   count(bins > b) < need <= count(bins >= b)
// and publish (b, count(bins > b)) through `res`.  `scan` is LDS scratch of 256 ints.
__device__ __forceinline__ void find_cut_bin(const int* hist, int* scan, int need, int* res) {
    const int t = threadIdx.x;
    scan[t] = hist[t];
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {  // inclusive suffix sum
        const int add = (t + off < 256) ? scan[t + off] : 0;
        __syncthreads();
        scan[t] += add;
        __syncthreads();
    }
    const int ge = scan[t];
    const int gt = (t + 1 < 256) ? scan[t + 1] : 0;
    if (gt < need && need <= ge) {
        res[0] = t;
        res[1] = gt;
    }
    __syncthreads();
}

// Ragged batches: whether the sequence of unit u stands at its trigger size after the latest step.
__device__ __forceinline__ bool seq_due(const SeqSched& s, int u) {
    const int off = s.off[u / s.heads];
    return off != kSeqIdle && sched_due((long)off + s.step, s.n_trig, s.m);
}

// One workgroup per unit.  Writes srcmap[u][i] = source slot of the row that ends in slot i
// (i < n-m), first[u] = first slot whose row moves, and optionally the ascending list of
// evicted slots.
__global__ void __launch_bounds__(SEL_THREADS)
select_evict_kernel(const uint16_t* __restrict__ cnt, int32_t* __restrict__ srcmap,
                    int32_t* __restrict__ first, int32_t* __restrict__ evicted, int n, int C, int E,
                    int W32, int r, int m, SeqSched seq) {
    if (seq.off && !seq_due(seq, blockIdx.x)) return;  // ragged batch: this unit's sequence is not due
    extern __shared__ int smem[];
    int* I = smem;            // [C] record of every slot
    int* hist = I + C;        // [256]
    int* scan = hist + 256;   // [256]
    int* wave_tot = scan + 256;  // [SEL_WAVES]
    int* res = wave_tot + SEL_WAVES;  // [2]
    const int u = blockIdx.x, t = threadIdx.x;
    const int ncand = n - r;
    if (W32) {  // exact ring: the record is the number of set bits in the slot's ring
        const uint32_t* ru = reinterpret_cast<const uint32_t*>(cnt) + (size_t)u * W32 * C;
        for (int j = t; j < n; j += SEL_THREADS) {
            int acc = 0;
            for (int b = 0; b < W32; ++b) acc += __popc(ru[(size_t)b * C + j]);
            I[j] = acc;
        }
    } else {
        const uint16_t* cu = cnt + (size_t)u * E * C;
        for (int j = t; j < n; j += SEL_THREADS) {
            int acc = 0;
            for (int b = 0; b < E; ++b) acc += cu[(size_t)b * C + j];
            I[j] = acc;
        }
    }
    // m-th largest record among the candidates, by two 8-bit digit passes.
    hist[t] = 0;
    __syncthreads();
    for (int j = t; j < ncand; j += SEL_THREADS) atomicAdd(&hist[(I[j] >> 8) & 255], 1);
    __syncthreads();
    find_cut_bin(hist, scan, m, res);
    const int hi = res[0];
    const int above_hi = res[1];
    __syncthreads();
    hist[t] = 0;
    __syncthreads();
    for (int j = t; j < ncand; j += SEL_THREADS)
        if (((I[j] >> 8) & 255) == hi) atomicAdd(&hist[I[j] & 255], 1);
    __syncthreads();
    find_cut_bin(hist, scan, m - above_hi, res);
    const int cut = (hi << 8) | res[0];            // every record above `cut` is evicted
    const int ties_needed = m - above_hi - res[1]; // plus this many records equal to it
    __syncthreads();

    // Sweep the slots in ascending order: rank ties, decide, and number the survivors.
    int tie_base = 0, keep_base = 0, first_moved = n;
    for (int j0 = 0; j0 < n; j0 += SEL_THREADS) {
        const int j = j0 + t;
        const bool in = j < n;
        const bool cand = j < ncand;
        const int v = in ? I[j] : 0;
        const bool tie = cand && v == cut;
        int tot;
        const int tie_rank = tie_base + block_prefix(tie, wave_tot, tot);
        tie_base += tot;
        const bool evict = cand && (v > cut || (tie && tie_rank < ties_needed));
        const bool keep = in && !evict;
        const int dest = keep_base + block_prefix(keep, wave_tot, tot);
        keep_base += tot;
        if (keep) srcmap[(size_t)u * C + dest] = j;
        if (evict) {
            const int k = j - dest;  // evicted slots before j
            if (evicted) evicted[(size_t)u * m + k] = j;
            if (k == 0) first_moved = j;
        }
    }
    if (first_moved < n) first[u] = first_moved;  // exactly one thread saw k == 0
}

// Move `lanes_per_row`-element rows of `base` (element type VT) so that slot i receives the
// row of slot srcmap[i], for i in [first, n_new).  In place: elements are handled in
// ascending chunks, a chunk is loaded completely before any of it is stored, and a row's
// source never lies below its destination, so no store can hit data still to be read.
// Rows are read once and written once per compression: non-temporal accesses keep them from
// displacing anything in the caches.
typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
template <typename VT>
__device__ __forceinline__ VT nt_load(const VT* p) {
    if constexpr (sizeof(VT) == 16) {
        const u32x4_nt v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(p));
        return __builtin_bit_cast(VT, v);
    } else {
        return __builtin_nontemporal_load(p);
    }
}
template <typename VT>
__device__ __forceinline__ void nt_store(VT* p, VT v) {
    if constexpr (sizeof(VT) == 16) {
        __builtin_nontemporal_store(__builtin_bit_cast(u32x4_nt, v), reinterpret_cast<u32x4_nt*>(p));
    } else {
        __builtin_nontemporal_store(v, p);
    }
}

template <typename VT, int UNR>
__device__ __forceinline__ void compact_array(VT* base, int lanes_per_row, const int32_t* srcmap,
                                              int first, int n_new) {
    const int total = (n_new - first) * lanes_per_row;
    const int nthreads = blockDim.x;
    for (int e0 = 0; e0 < total; e0 += nthreads * UNR) {
        VT val[UNR];
        int dst_idx[UNR];
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            const int e = e0 + x * nthreads + threadIdx.x;
            dst_idx[x] = -1;
            if (e < total) {
                const int row = first + e / lanes_per_row;
                const int ln = e - (row - first) * lanes_per_row;
                val[x] = nt_load(&base[(size_t)srcmap[row] * lanes_per_row + ln]);
                dst_idx[x] = row * lanes_per_row + ln;
            }
        }
        __syncthreads();
#pragma unroll
        for (int x = 0; x < UNR; ++x)
            if (dst_idx[x] >= 0) nt_store(&base[dst_idx[x]], val[x]);
    }
    __syncthreads();
}

struct CompactArgs {
    void* K;
    void* V;
    void* K_meta;
    void* V_meta;
    int32_t* pos;
    uint16_t* cnt;
    const int32_t* srcmap;
    const int32_t* first;
    int C, E, W32;
    int row_lanes16;   // 16-byte pieces per K (or V) row
    int meta_words;    // 32-bit words of meta per row (0 when not 4-bit)
    int n_old, n_new;
    int zero_bucket;
    SeqSched seq;
};

// grid (U, 3): part 0 moves K (+K_meta), part 1 moves V (+V_meta), part 2 moves positions and
// counters, then clears the counters of the freed tail slots and of the bucket that the next
// epoch counts into.
__global__ void __launch_bounds__(1024) compact_kernel(CompactArgs a) {
    const int u = blockIdx.x, part = blockIdx.y;
    if (a.seq.off) {  // ragged batch: only due sequences, each clearing the bucket its next epoch counts into
        if (!seq_due(a.seq, u)) return;
        if (a.E) {
            const long ep = sched_epoch((long)a.seq.off[u / a.seq.heads] + a.seq.step, a.seq.n_trig, a.seq.m) + 1;
            a.zero_bucket = (int)(((ep % a.E) + a.E) % a.E);
        }
    }
    const int32_t* map = a.srcmap + (size_t)u * a.C;
    const int first = a.first[u];
    if (part < 2) {
        uint4* rows = reinterpret_cast<uint4*>(part ? a.V : a.K) + (size_t)u * a.C * a.row_lanes16;
        compact_array<uint4, 4>(rows, a.row_lanes16, map, first, a.n_new);
        if (a.meta_words) {
            uint32_t* meta =
                reinterpret_cast<uint32_t*>(part ? a.V_meta : a.K_meta) + (size_t)u * a.C * a.meta_words;
            compact_array<uint32_t, 4>(meta, a.meta_words, map, first, a.n_new);
        }
        return;
    }
    compact_array<int32_t, 4>(a.pos + (size_t)u * a.C, 1, map, first, a.n_new);
    for (int b = 0; b < a.W32; ++b) {  // exact ring: every word plane moves with its row
        uint32_t* rb = reinterpret_cast<uint32_t*>(a.cnt) + ((size_t)u * a.W32 + b) * a.C;
        compact_array<uint32_t, 4>(rb, 1, map, first, a.n_new);
        for (int j = a.n_new + threadIdx.x; j < a.n_old; j += blockDim.x) rb[j] = 0;
    }
    for (int b = 0; b < a.E; ++b) {
        uint16_t* cb = a.cnt + ((size_t)u * a.E + b) * a.C;
        if (b == a.zero_bucket) {
            for (int j = threadIdx.x; j < a.n_old; j += blockDim.x) cb[j] = 0;
        } else {
            compact_array<uint16_t, 4>(cb, 1, map, first, a.n_new);
            for (int j = a.n_new + threadIdx.x; j < a.n_old; j += blockDim.x) cb[j] = 0;
        }
    }
}

// The per-sequence table travels as kernel arguments (no host buffer has to outlive the call).
struct SeqChunk {
    int32_t v[256];
};

__global__ void __launch_bounds__(256) write_seq_table_kernel(int32_t* __restrict__ dst, SeqChunk c, int count) {
    if ((int)threadIdx.x < count) dst[threadIdx.x] = c.v[threadIdx.x];
}

// Up to 64 step counts (one per cache of a layer set) advanced by one launch.
struct TickList {
    int32_t* counter[64];
};
__global__ void __launch_bounds__(64) tick_kernel(TickList t, int count) {
    if ((int)threadIdx.x < count) *t.counter[threadIdx.x] += 1;
}

}  // namespace

hipError_t static_scratch(void** ptr) {
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return err;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t launch_write_seq_table(int32_t* dst, const int32_t* host_values, int count, hipStream_t stream) {
    for (int base = 0; base < count; base += 256) {
        SeqChunk c;
        const int k = count - base < 256 ? count - base : 256;
        for (int i = 0; i < 256; ++i) c.v[i] = i < k ? host_values[base + i] : kSeqIdle;
        write_seq_table_kernel<<<1, 256, 0, stream>>>(dst + base, c, k);
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

hipError_t launch_tick(int32_t* const* counters, int count, hipStream_t stream) {
    for (int base = 0; base < count; base += 64) {
        TickList t;
        const int k = count - base < 64 ? count - base : 64;
        for (int i = 0; i < 64; ++i) t.counter[i] = i < k ? counters[base + i] : nullptr;
        tick_kernel<<<1, 64, 0, stream>>>(t, k);
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

hipError_t launch_compress(const Layout& L, const CompressArgs& c, hipStream_t stream) {
    const size_t lds = ((size_t)L.C + 512 + SEL_WAVES + 2) * sizeof(int);
    select_evict_kernel<<<L.U, SEL_THREADS, lds, stream>>>(L.cnt, L.srcmap, L.first, c.evicted, c.n, L.C,
                                                           L.E, L.W32, c.r, c.m, c.seq);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    CompactArgs a;
    a.K = L.K;
    a.V = L.V;
    a.K_meta = L.K_meta;
    a.V_meta = L.V_meta;
    a.pos = L.pos;
    a.cnt = L.cnt;
    a.srcmap = L.srcmap;
    a.first = L.first;
    a.C = L.C;
    a.E = L.E;
    a.W32 = L.W32;
    if (L.kv_dtype == KV_F32) {
        a.row_lanes16 = L.d * 4 / 16;
        a.meta_words = 0;
    } else if (L.kv_dtype == KV_F16) {
        a.row_lanes16 = L.d * 2 / 16;
        a.meta_words = 0;
    } else {
        a.row_lanes16 = L.d / 2 / 16;
        a.meta_words = L.d / 64;
    }
    a.n_old = c.n;
    a.n_new = c.n - c.m;
    a.zero_bucket = c.zero_bucket;
    a.seq = c.seq;
    // 1024 threads per workgroup: a workgroup needs all the loads in flight it can have to move its
    // unit quickly, and with every unit compacting (lock step) it is no slower than smaller
    // workgroups that share a CU (measured per event, 256 against 1024 threads: 9216 units 0.82
    // -> 0.80 ms, 2560 units 0.159 -> 0.149; one ragged sequence of 32 units 68 -> 25 us).
    compact_kernel<<<dim3(L.U, 3), 1024, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace sc
