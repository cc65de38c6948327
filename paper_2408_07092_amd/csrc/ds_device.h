// Device-side helpers shared by the kernels of libdsattn (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ds_internal.h"

namespace ds {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

// Monotone map from a binary32 score to an unsigned key: a larger score gives a
// larger key, and -0 maps to the key of +0 so the two tie.
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Algorithm 1 step 3 as a predicate: with T the exact k-th largest key of the
// unit, a token is selected iff its key beats T, or equals T and is among the
// lowest-index ties that still fit (token <= tcut).
__device__ __forceinline__ bool is_selected(uint32_t key, int t, uint32_t T, int tcut)
{
    return key > T || (key == T && t <= tcut);
}

__device__ __forceinline__ int wave_inclusive_scan(int x, int lane)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int y = __shfl_up(x, o);
        if (lane >= o) x += y;
    }
    return x;
}

// Ordered compaction: writes the selected tokens of [t0, t1) to sel[] in
// ascending token order and returns how many there are (same value in every
// thread).  keys_u points at the unit's key array; t0 % 4 == 0.  s_w is LDS
// scratch of 4 ints.  All 256 threads must call it.
__device__ __forceinline__ int compact_selected(const uint32_t *__restrict__ keys_u, int t0, int t1,
                                                uint32_t T, int tcut, int *sel, int *s_w)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int base = 0;
    for (int p0 = t0; p0 < t1; p0 += kWG * 4) {
        const int t = p0 + tid * 4;
        uint32_t kv[4] = {0u, 0u, 0u, 0u};
        if (t < t1) {
            const uint4 v = *reinterpret_cast<const uint4 *>(keys_u + t);
            kv[0] = v.x; kv[1] = v.y; kv[2] = v.z; kv[3] = v.w;
        }
        bool f[4];
        int cnt = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[e] = (t + e < t1) && is_selected(kv[e], t + e, T, tcut);
            cnt += f[e] ? 1 : 0;
        }
        const int incl = wave_inclusive_scan(cnt, lane);
        if (lane == 63) s_w[wave] = incl;
        __syncthreads();
        int woff = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int c = s_w[w];
            if (w < wave) woff += c;
            total += c;
        }
        int pos = base + woff + incl - cnt;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (f[e]) sel[pos++] = t + e;
        base += total;
        __syncthreads();
    }
    return base;
}

}  // namespace ds
