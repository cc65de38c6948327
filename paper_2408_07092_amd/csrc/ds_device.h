// Device-side helpers shared by the kernels of libdsattn (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "ds_internal.h"

namespace ds {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

constexpr float kNegInf = -__builtin_inff();

// Loads of data that is read once per call (label rows, K/V rows) are marked non-temporal, which
// streams them past the caches' replacement (measured on this part: dense decode over 1 GiB 191 ->
// 176 us).  ST = false: the variants for calls that move only a few MiB, which do better without.
//
// A 16-byte piece of a label row of NV pieces.  Rows of one piece stream; of rows of two pieces a
// wavefront's first load leaves every other 16 bytes of its lines for the second, which finds them
// in the cache only if the first load was an ordinary one (measured on 16-channel labels:
// streaming mark +3 us per layer).  (k_refine_attend loads such rows as whole lines, two tokens'
// halves per lane, and lets neighbouring lanes swap: see swap_pairs.)
template <int NV, bool ST = true>
__device__ __forceinline__ half8 label_load(const half8 *p)
{
    if constexpr (NV == 1 && ST) return __builtin_nontemporal_load(p);
    else return *p;
}
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <bool ST = true>
__device__ __forceinline__ uint4 stream_load(const uint4 *p)
{
    if constexpr (!ST) return *p;
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Neighbouring lanes (2j, 2j + 1) exchange a 16-byte piece.
__device__ __forceinline__ half8 swap_pairs(half8 v)
{
    typedef int int4v __attribute__((ext_vector_type(4)));
    int4v x = __builtin_bit_cast(int4v, v);
#pragma unroll
    for (int k = 0; k < 4; ++k) x[k] = __builtin_amdgcn_update_dpp(0, x[k], 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
    return __builtin_bit_cast(half8, x);
}

// Development aid, compiled out unless the library is built with -DDS_TRACE:
// thread 0 of every workgroup stamps the device clock at numbered stages into a
// per-source-file buffer that ds_trace_read_* copies out.
#ifdef DS_TRACE
#define DS_TRACE_BUFFER __device__ long long g_trace[1 << 18];
#define DS_TR(stage)                                                                              \
    do {                                                                                          \
        if (threadIdx.x == 0)                                                                     \
            g_trace[(((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 16 + (stage)) & ((1 << 18) - 1)] = \
                wall_clock64();                                                                   \
    } while (0)
#else
#define DS_TRACE_BUFFER
#define DS_TR(stage) do { } while (0)
#endif

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

// In-launch hand-over.  These workspace arrays are written by one workgroup and read by another
// inside the same launch: the unit histograms (`hist`, `coarse`), the candidate list (`cand`), the
// per-chunk counts and offsets (`ndef`, `offs`), the attention partials (`part`) and the words of
// the UnitCtl records.  Every such read goes through ld_dev and every such write through st_dev
// or an agent-scope atomic -- never through a plain load, which could be served from a stale line
// of the reader's L2 without any error and only now and then.  Plain stores to them are allowed
// only for clearing what nobody reads again in this launch.  tests/test_abi_host.py greps the
// kernels for reads that break the rule.  (The reason for not using fences instead is measured:
// see below.)
//
// Data that one workgroup hands to another inside a kernel goes through these
// device-scope accesses: the stores are written through to the device's
// coherence point and the loads read it there, so no cache needs flushing.
// (A device-wide fence per workgroup writes back and invalidates the whole L2
// of its XCD, which costs far more than the kernels themselves.)
__device__ __forceinline__ uint32_t ld_dev(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint2 ld_dev(const uint2 *p)
{
    const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p),
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint2((uint32_t)v, (uint32_t)(v >> 32));
}
__device__ __forceinline__ float2 ld_dev(const float2 *p)
{
    const uint2 v = ld_dev(reinterpret_cast<const uint2 *>(p));
    return make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
}
__device__ __forceinline__ void st_dev(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(float *p, float v)
{
    __hip_atomic_store(reinterpret_cast<uint32_t *>(p), __float_as_uint(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(uint2 *p, uint2 v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p),
                       (unsigned long long)v.x | ((unsigned long long)v.y << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// "Last workgroup done" hand-over: every workgroup of a group of `total` calls
// this after its st_dev stores / global atomics; exactly one of them (the last
// to arrive) gets true in all its threads and may then read what the others
// wrote with ld_dev.  Each thread first waits until its own stores and atomics
// have been performed, the barrier collects the workgroup, then one thread
// bumps the counter.  The counter must be 0 before the first arrival; the
// workgroup that gets true resets it.
// (Data whose reader can check its completeness itself -- the unit histograms of
// k_refine_attend, by their sums -- is handed over without the wait.)
__device__ __forceinline__ bool last_arrival(uint32_t *counter, uint32_t total, uint32_t *s_flag)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t t = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = (t == total - 1u) ? 1u : 0u;
    }
    __syncthreads();
    return *s_flag != 0u;
}

// The same with a 64-bit counter whose high word counts the arrivals and whose low word is a
// sum the arriving workgroups have added to before (agent-scope adds of their contributions):
// the workgroup that completes the count also learns the full sum (*low) without another load.
__device__ __forceinline__ bool last_arrival_sum(unsigned long long *counter, uint32_t total,
                                                 uint32_t *s_flag, uint32_t *s_low)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long t =
            __hip_atomic_fetch_add(counter, 1ull << 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = ((uint32_t)(t >> 32) == total - 1u) ? 1u : 0u;
        *s_low = (uint32_t)t;
    }
    __syncthreads();
    return *s_flag != 0u;
}

// Inclusive prefix sum over the 64 lanes of a wavefront with DPP moves: four
// shifted adds inside each row of 16 lanes, then the row totals are carried
// forward (lane 15 of a row into the next row, lane 31 into rows 2 and 3).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_take(int x)
{
    // lanes without a source (shifted in from outside the row, or rows masked off) read 0
    return __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xF, true);
}
__device__ __forceinline__ int wave_inclusive_scan(int x, int /*lane*/)
{
    x += dpp_take<0x111, 0xF>(x);  // row_shr:1
    x += dpp_take<0x112, 0xF>(x);  // row_shr:2
    x += dpp_take<0x114, 0xF>(x);  // row_shr:4
    x += dpp_take<0x118, 0xF>(x);  // row_shr:8
    x += dpp_take<0x142, 0xA>(x);  // row_bcast:15 into rows 1 and 3
    x += dpp_take<0x143, 0xC>(x);  // row_bcast:31 into rows 2 and 3
    return x;
}

// Exclusive prefix sum over the threads of the workgroup (thread order; NW wavefronts, 256
// threads unless said otherwise); *total receives the sum.  s_w: NW words of LDS.  Contains two
// barriers.
template <int NW = 4>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t *s_w, uint32_t *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t incl = (uint32_t)wave_inclusive_scan((int)x, lane);
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    uint32_t woff = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const uint32_t c = s_w[w];
        if (w < wave) woff += c;
        tot += c;
    }
    __syncthreads();
    *total = tot;
    return woff + incl - x;
}

// Fixed-order reductions over the workgroup (same tree every run).
__device__ __forceinline__ float block_max(float x, float *s_w)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = x;
    __syncthreads();
    const float r = fmaxf(fmaxf(s_w[0], s_w[1]), fmaxf(s_w[2], s_w[3]));
    __syncthreads();
    return r;
}
__device__ __forceinline__ float block_sum(float x, float *s_w)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = x;
    __syncthreads();
    const float r = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
    __syncthreads();
    return r;
}

// Histogram select over 64*NW*PER bins (256*PER unless NW is given) whose counts come from get(bin): finds the
// bin holding the kth element (1-based) counted from the top bin down
// (FROM_TOP) or from bin 0 up.  res[0] = bin, res[1] = rank of the element
// inside that bin, counted the same way.  Exactly one thread writes res when
// 1 <= kth <= total count (otherwise res = {0, 1}); all threads may read res
// after the call, and must have finished reading an earlier result before it.
template <int PER, bool FROM_TOP, int NW = 4, class Get>
__device__ __forceinline__ void hist_select(Get get, uint32_t kth, uint32_t *s_w, uint32_t *res)
{
    const int tid = threadIdx.x;
    constexpr int NB = 64 * NW * PER;
    // in-range result even when the counts do not reach kth (a workspace that was not cleared)
    if (tid == 0) {
        res[0] = 0u;
        res[1] = 1u;
    }
    // A thread owns PER consecutive bins.  Their sum is taken in an order that starts at a
    // different bin in every lane: read in the same order, the lanes of a wavefront would sit
    // PER words apart -- on 32 / PER LDS banks, each read served in PER turns.
    auto bin_at = [&](int i) { return FROM_TOP ? (NB - 1 - (tid * PER + i)) : tid * PER + i; };
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) sum += get(bin_at(PER > 1 ? ((i + tid) % PER) : i));
    uint32_t total;
    uint32_t before = block_exclusive_scan<NW>(sum, s_w, &total);
    // (one thread at most: it reads its bins once more, all at once, and walks them in order)
    if (before < kth && before + sum >= kth) {
        uint32_t loc[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) loc[i] = PER > 1 ? get(bin_at(i)) : sum;  // (a single bin may have come from memory)
        bool done = false;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (!done) {
                if (before + loc[i] >= kth) {
                    res[0] = (uint32_t)bin_at(i);
                    res[1] = kth - before;
                    done = true;
                } else {
                    before += loc[i];
                }
            }
        }
    }
    __syncthreads();
}

// One radix pass over the candidates of a unit: histogram `digit(e)` of those
// with `match(e)`, then pick the bin holding the `want`-th of them.
template <int PER, bool FROM_TOP, int NW = 4, class Each, class Match, class Digit>
__device__ __forceinline__ void svc_radix_pass(Each each, Match match, Digit digit, uint32_t want,
                                               uint32_t *lh, uint32_t *s_w, uint32_t *res)
{
    for (int i = threadIdx.x; i < 64 * NW * PER; i += 64 * NW) lh[i] = 0u;
    __syncthreads();
    each([&](uint2 e) {
        if (match(e)) atomicAdd(&lh[digit(e)], 1u);
    });
    __syncthreads();
    hist_select<PER, FROM_TOP, NW>([&](int bin) { return lh[bin]; }, want, s_w, res);
}

// Ordered compaction: writes the selected tokens of [t0, t1) to sel[] in
// ascending token order and returns how many there are (same value in every
// thread).  keys_u points at the unit's key array; t0 % 4 == 0.  s_w is LDS
// scratch of 4 words.  All 256 threads must call it.
__device__ __forceinline__ int compact_selected(const uint32_t *__restrict__ keys_u, int t0, int t1,
                                                uint32_t T, int tcut, int *sel, uint32_t *s_w)
{
    const int tid = threadIdx.x;
    int base = 0;
    for (int p0 = t0; p0 < t1; p0 += kWG * 4) {
        const int t = p0 + tid * 4;
        uint32_t kv[4] = {0u, 0u, 0u, 0u};
        if (t < t1) {
            const uint4 v = *reinterpret_cast<const uint4 *>(keys_u + t);
            kv[0] = v.x; kv[1] = v.y; kv[2] = v.z; kv[3] = v.w;
        }
        bool f[4];
        uint32_t cnt = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[e] = (t + e < t1) && is_selected(kv[e], t + e, T, tcut);
            cnt += f[e] ? 1u : 0u;
        }
        uint32_t total;
        int pos = base + (int)block_exclusive_scan(cnt, s_w, &total);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (f[e]) sel[pos++] = t + e;
        base += (int)total;
    }
    __syncthreads();
    return base;
}

}  // namespace ds
