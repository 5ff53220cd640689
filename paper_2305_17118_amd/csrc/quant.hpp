// 4-bit row format shared by the kernels that write or read quantised rows (device code only).
// Per row and per group of 64 consecutive channels: zero = min, scale = fp16((max-min)/15)
// (1 when that is 0), code = clamp(rint((x-zero)/scale), 0, 15); value = code*scale + zero.
// Two codes per byte, channel 2i in the low nibble of byte i; one 32-bit meta word
// {fp16 scale, fp16 zero} per group.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sc {

union MetaWord {
    uint32_t u32;
    _Float16 h[2];  // scale, zero
};

// Quantise one row of D fp16 channels held two per lane (lane i holds x0 = channel 2i and
// x1 = channel 2i+1; lanes >= D/2 idle) and store codes and meta to `codes` / `meta` (global)
// and, when given, to their LDS copies.
// Every operation is a single IEEE fp32 operation so the codes are reproducible anywhere:
// zero = min, scale = fp16((max-min)/15) (1 when that is 0),
// code = clamp(rint((x-zero)/scale), 0, 15).
template <int D>
__device__ __forceinline__ void quantise_row(float x0, float x1, unsigned char* codes, uint32_t* meta,
                                             unsigned char* lds_codes, uint32_t* lds_meta, int lane) {
    if (lane < D / 2) {
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
        const unsigned char byte = (unsigned char)((uint32_t)c0 | ((uint32_t)c1 << 4));
        codes[lane] = byte;
        if (lds_codes) lds_codes[lane] = byte;
        if ((lane & 31) == 0) {
            MetaWord mw;
            mw.h[0] = sh;
            mw.h[1] = zh;
            meta[lane >> 5] = mw.u32;
            if (lds_meta) lds_meta[lane >> 5] = mw.u32;
        }
    }
}

}  // namespace sc
