// Steps 1-2 of Algorithm 1 on gfx950: label-cache scoring and exact per-unit
// top-k as a radix select.
//
//   k_score   streams the label cache, forms the binary32 approximate score of
//             every token, stores it as an ordered 32-bit key and builds a
//             4096-bin histogram of the keys' top 12 bits per unit.
//   k_thresh  finds the histogram bin b* that holds the k-th largest key.
//   k_cand    collects the keys of bin b* (the only ones whose fate is open)
//             and counts, per token chunk, the keys above b*.
//   k_refine  radix-selects the exact k-th key T inside bin b*, resolves equal
//             keys towards the lowest token index, and turns the per-chunk
//             counts into offsets of the ascending index list.
//   k_compact writes that index list (used when the caller wants indices).
// All counters are integers, so the result does not depend on the order in
// which workgroups or atomics complete.
#include "ds_device.h"

namespace ds {

// ---------------------------------------------------------------- zero
__global__ __launch_bounds__(kWG) void k_zero(uint32_t *p, size_t n_words)
{
    size_t i = (size_t)blockIdx.x * kWG + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kWG;
    for (; i < n_words; i += stride) p[i] = 0u;
}

// ---------------------------------------------------------------- score
// RMODE 8 / 16: r known at compile time (one or two 16-byte loads per token);
// RMODE 0: r % 8 == 0 (r/8 16-byte loads); RMODE -1: any r, 2-byte loads.
template <int RMODE>
__device__ __forceinline__ float label_dot(const _Float16 *__restrict__ row, const float *qs, int r)
{
    float acc = 0.0f;
    if constexpr (RMODE == 8 || RMODE == 16) {
        constexpr int NV = RMODE / 8;
        half8 v[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) v[i] = reinterpret_cast<const half8 *>(row)[i];
#pragma unroll
        for (int i = 0; i < NV; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc = __builtin_fmaf(qs[i * 8 + j], (float)v[i][j], acc);
    } else if constexpr (RMODE == 0) {
        for (int i = 0; i < r / 8; ++i) {
            const half8 v = reinterpret_cast<const half8 *>(row)[i];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc = __builtin_fmaf(qs[i * 8 + j], (float)v[j], acc);
        }
    } else {
        for (int j = 0; j < r; ++j) acc = __builtin_fmaf(qs[j], (float)row[j], acc);
    }
    return acc;
}

template <int RMODE>
__global__ __launch_bounds__(kWG) void k_score(const _Float16 *__restrict__ q,
                                               const _Float16 *__restrict__ label,
                                               const int32_t *__restrict__ channels,
                                               uint32_t *__restrict__ keys,
                                               uint32_t *__restrict__ hist, int Hq, int Hkv, int G,
                                               int L, int L_max, int r, int key_stride, int sc_chunk)
{
    __shared__ uint32_t lh[kHistBins];
    __shared__ float qs_sh[kD];
    const int tid = threadIdx.x;
    const int u = blockIdx.y, b = u / Hkv, h = u % Hkv;

    for (int i = tid; i < kHistBins; i += kWG) lh[i] = 0u;
    if (tid < r) {
        // label query of the group: sum over its heads (g ascending) of q_g[C[j]]
        const int c = channels[h * r + tid];
        float a = 0.0f;
        for (int g = 0; g < G; ++g) a = a + (float)q[((size_t)b * Hq + (size_t)h * G + g) * kD + c];
        qs_sh[tid] = a;
    }
    __syncthreads();

    float qs[(RMODE > 0) ? RMODE : 1];
    if (RMODE > 0) {
#pragma unroll
        for (int j = 0; j < ((RMODE > 0) ? RMODE : 1); ++j) qs[j] = qs_sh[j];
    }
    const float *qp = (RMODE > 0) ? qs : qs_sh;

    const int t_begin = blockIdx.x * sc_chunk;
    const int t_end = min(L, t_begin + sc_chunk);
    const _Float16 *lab = label + (size_t)u * L_max * r;
    uint32_t *ku = keys + (size_t)u * key_stride;

    constexpr int UNR = 4;
    for (int t0 = t_begin + tid; t0 < t_end; t0 += kWG * UNR) {
        float s[UNR];
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int t = t0 + i * kWG;
            s[i] = (t < t_end) ? label_dot<RMODE>(lab + (size_t)t * r, qp, r) : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int t = t0 + i * kWG;
            if (t < t_end) {
                const uint32_t key = score_key(s[i]);
                ku[t] = key;
                atomicAdd(&lh[key >> kKeyShift], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t *hu = hist + (size_t)u * kHistBins;
    for (int i = tid; i < kHistBins; i += kWG) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&hu[i], c);
    }
}

// ---------------------------------------------------------------- histogram select
// LDS histogram lh[256*PER]; finds the bin holding the kth element (1-based)
// counted from the top bin down (FROM_TOP) or from bin 0 up.  res[0] = bin,
// res[1] = rank of the element inside that bin, counted the same way.
// Exactly one thread writes res when 1 <= kth <= total count.
template <int PER, bool FROM_TOP>
__device__ __forceinline__ void hist_select(const uint32_t *lh, uint32_t kth, uint32_t *s_part,
                                            uint32_t *res)
{
    const int tid = threadIdx.x;
    constexpr int NB = kWG * PER;
    uint32_t loc[PER];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int pos = tid * PER + i;
        loc[i] = lh[FROM_TOP ? (NB - 1 - pos) : pos];
        sum += loc[i];
    }
    s_part[tid] = sum;
    __syncthreads();
    uint32_t before = 0;
    for (int j = 0; j < tid; ++j) before += s_part[j];
    if (before < kth && before + sum >= kth) {
        bool done = false;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (!done) {
                if (before + loc[i] >= kth) {
                    const int pos = tid * PER + i;
                    res[0] = (uint32_t)(FROM_TOP ? (NB - 1 - pos) : pos);
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

__global__ __launch_bounds__(kWG) void k_thresh(const uint32_t *__restrict__ hist, UnitCtl *ctl,
                                                int k_eff)
{
    __shared__ uint32_t lh[kHistBins];
    __shared__ uint32_t s_part[kWG];
    __shared__ uint32_t res[2];
    const int tid = threadIdx.x, u = blockIdx.x;
    const uint32_t *hu = hist + (size_t)u * kHistBins;
    for (int i = tid; i < kHistBins; i += kWG) lh[i] = hu[i];
    __syncthreads();
    hist_select<kHistBins / kWG, true>(lh, (uint32_t)k_eff, s_part, res);
    if (tid == 0) {
        ctl[u].bstar = res[0];
        ctl[u].krem = res[1];
    }
}

// ---------------------------------------------------------------- candidates
__global__ __launch_bounds__(kWG) void k_cand(const uint32_t *__restrict__ keys, UnitCtl *ctl,
                                              uint2 *__restrict__ cand, uint32_t *__restrict__ ndef,
                                              int L, int key_stride, int ch, int n_ch)
{
    extern __shared__ uint2 lc[];  // ch entries
    __shared__ uint32_t s_cnt, s_def, s_base;
    const int tid = threadIdx.x, u = blockIdx.y, c = blockIdx.x;
    if (tid == 0) { s_cnt = 0u; s_def = 0u; }
    __syncthreads();
    const uint32_t bstar = ctl[u].bstar;
    const int t0 = c * ch, t1 = min(L, t0 + ch);
    const uint32_t *ku = keys + (size_t)u * key_stride;
    uint32_t mydef = 0;
    for (int t = t0 + tid * 4; t < t1; t += kWG * 4) {
        const uint4 v = *reinterpret_cast<const uint4 *>(ku + t);
        const uint32_t kv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (t + e < t1) {
                const uint32_t bin = kv[e] >> kKeyShift;
                if (bin > bstar) {
                    ++mydef;
                } else if (bin == bstar) {
                    const uint32_t slot = atomicAdd(&s_cnt, 1u);
                    lc[slot] = make_uint2(kv[e], (uint32_t)(t + e));
                }
            }
        }
    }
    if (mydef) atomicAdd(&s_def, mydef);
    __syncthreads();
    if (tid == 0) {
        ndef[(size_t)u * n_ch + c] = s_def;
        s_base = s_cnt ? atomicAdd(&ctl[u].ncand, s_cnt) : 0u;
    }
    __syncthreads();
    const uint32_t n = s_cnt, base = s_base;
    uint2 *cu = cand + (size_t)u * L;
    for (uint32_t i = tid; i < n; i += kWG) cu[base + i] = lc[i];
}

// ---------------------------------------------------------------- refine
__global__ __launch_bounds__(kWG) void k_refine(const uint2 *__restrict__ cand, UnitCtl *ctl,
                                                const uint32_t *__restrict__ ndef,
                                                uint32_t *__restrict__ offs, int L, int ch, int n_ch)
{
    __shared__ uint32_t lh[2048];
    __shared__ uint32_t s_part[kWG];
    __shared__ uint32_t res[2];
    extern __shared__ uint32_t cnt[];  // n_ch entries
    const int tid = threadIdx.x, u = blockIdx.x;
    const uint2 *cu = cand + (size_t)u * L;
    const uint32_t n = ctl[u].ncand;
    const uint32_t bstar = ctl[u].bstar;
    uint32_t krem = ctl[u].krem;

    // key bits [19:10] of the candidates (all share the top 12 bits)
    for (int i = tid; i < 1024; i += kWG) lh[i] = 0u;
    __syncthreads();
    for (uint32_t i = tid; i < n; i += kWG) atomicAdd(&lh[(cu[i].x >> 10) & 1023u], 1u);
    __syncthreads();
    hist_select<4, true>(lh, krem, s_part, res);
    const uint32_t mid = res[0];
    krem = res[1];
    __syncthreads();
    // key bits [9:0] among candidates matching so far
    for (int i = tid; i < 1024; i += kWG) lh[i] = 0u;
    __syncthreads();
    const uint32_t pre22 = (bstar << 10) | mid;
    for (uint32_t i = tid; i < n; i += kWG) {
        const uint32_t key = cu[i].x;
        if ((key >> 10) == pre22) atomicAdd(&lh[key & 1023u], 1u);
    }
    __syncthreads();
    hist_select<4, true>(lh, krem, s_part, res);
    const uint32_t T = (pre22 << 10) | res[0];
    const uint32_t m_ties = res[1];          // how many keys equal to T are selected
    const uint32_t n_ties = lh[res[0]];      // how many keys equal T
    __syncthreads();

    // Equal keys: keep the m_ties lowest token indices -> tcut = m_ties-th smallest
    // index among them (radix select on the index, 11 + 10 + 10 bits, ascending).
    int tcut = 0x7fffffff;
    if (m_ties < n_ties) {
        uint32_t want = m_ties, prefix = 0u;
        // bits [30:20]
        for (int i = tid; i < 2048; i += kWG) lh[i] = 0u;
        __syncthreads();
        for (uint32_t i = tid; i < n; i += kWG)
            if (cu[i].x == T) atomicAdd(&lh[cu[i].y >> 20], 1u);
        __syncthreads();
        hist_select<8, false>(lh, want, s_part, res);
        prefix = res[0];
        want = res[1];
        __syncthreads();
        // bits [19:10]
        for (int i = tid; i < 1024; i += kWG) lh[i] = 0u;
        __syncthreads();
        for (uint32_t i = tid; i < n; i += kWG)
            if (cu[i].x == T && (cu[i].y >> 20) == prefix) atomicAdd(&lh[(cu[i].y >> 10) & 1023u], 1u);
        __syncthreads();
        hist_select<4, false>(lh, want, s_part, res);
        prefix = (prefix << 10) | res[0];
        want = res[1];
        __syncthreads();
        // bits [9:0]
        for (int i = tid; i < 1024; i += kWG) lh[i] = 0u;
        __syncthreads();
        for (uint32_t i = tid; i < n; i += kWG)
            if (cu[i].x == T && (cu[i].y >> 10) == prefix) atomicAdd(&lh[cu[i].y & 1023u], 1u);
        __syncthreads();
        hist_select<4, false>(lh, want, s_part, res);
        tcut = (int)((prefix << 10) | res[0]);
        __syncthreads();
    }
    if (tid == 0) {
        ctl[u].T = T;
        ctl[u].tcut = tcut;
    }

    // selected tokens per chunk = keys above bin b* (ndef) + selected candidates
    for (int i = tid; i < n_ch; i += kWG) cnt[i] = ndef[(size_t)u * n_ch + i];
    __syncthreads();
    for (uint32_t i = tid; i < n; i += kWG) {
        const uint2 e = cu[i];
        if (is_selected(e.x, (int)e.y, T, tcut)) atomicAdd(&cnt[e.y / (uint32_t)ch], 1u);
    }
    __syncthreads();
    // exclusive prefix over chunks -> offsets into the ascending index list
    const int per = (n_ch + kWG - 1) / kWG;
    const int c0 = tid * per, c1 = min(n_ch, c0 + per);
    uint32_t sum = 0;
    for (int i = c0; i < c1; ++i) sum += cnt[i];
    s_part[tid] = sum;
    __syncthreads();
    uint32_t run = 0;
    for (int j = 0; j < tid; ++j) run += s_part[j];
    for (int i = c0; i < c1; ++i) {
        offs[(size_t)u * n_ch + i] = run;
        run += cnt[i];
    }
}

// ---------------------------------------------------------------- compact
// Writes idx_out[u, 0..k_eff) ascending and -1 beyond.
__global__ __launch_bounds__(kWG) void k_compact(const uint32_t *__restrict__ keys,
                                                 const UnitCtl *__restrict__ ctl,
                                                 const uint32_t *__restrict__ offs,
                                                 int32_t *__restrict__ idx_out, int L, int key_stride,
                                                 int ch, int n_ch, int k, int k_eff)
{
    extern __shared__ int sel[];  // ch entries
    __shared__ int s_w[4];
    const int tid = threadIdx.x, u = blockIdx.y, c = blockIdx.x;
    const int t0 = c * ch, t1 = min(L, t0 + ch);
    const uint32_t T = ctl[u].T;
    const int tcut = ctl[u].tcut;
    const int n = compact_selected(keys + (size_t)u * key_stride, t0, t1, T, tcut, sel, s_w);
    __syncthreads();
    int32_t *io = idx_out + (size_t)u * k;
    const uint32_t off = offs[(size_t)u * n_ch + c];
    for (int i = tid; i < n; i += kWG)
        if (off + i < (uint32_t)k_eff) io[off + i] = sel[i];
    if (c == 0)
        for (int i = k_eff + tid; i < k; i += kWG) io[i] = -1;
}

// ---------------------------------------------------------------- launchers
static inline char *wsp(void *ws, size_t off) { return static_cast<char *>(ws) + off; }

hipError_t launch_zero(void *ws, const Plan &p, hipStream_t st)
{
    // ctl and hist are adjacent in the workspace
    const size_t n_words = (p.off_keys - p.off_ctl) / 4;
    const int blocks = (int)((n_words + kWG * 4 - 1) / (kWG * 4));
    prof_begin(KID_ZERO, st);
    hipLaunchKernelGGL(k_zero, dim3(blocks < 1 ? 1 : blocks), dim3(kWG), 0, st,
                       reinterpret_cast<uint32_t *>(wsp(ws, p.off_ctl)), n_words);
    prof_end(KID_ZERO, st);
    return hipGetLastError();
}

hipError_t launch_score(const void *q, const void *label, const int32_t *channels, void *ws,
                        const Plan &p, const ds_shape_t &s, hipStream_t st)
{
    const dim3 grid(p.n_sc, p.units), block(kWG);
    auto *keys = reinterpret_cast<uint32_t *>(wsp(ws, p.off_keys));
    auto *hist = reinterpret_cast<uint32_t *>(wsp(ws, p.off_hist));
    const auto *qh = static_cast<const _Float16 *>(q);
    const auto *lh = static_cast<const _Float16 *>(label);
    prof_begin(KID_SCORE, st);
#define DS_SCORE(MODE)                                                                         \
    hipLaunchKernelGGL(k_score<MODE>, grid, block, 0, st, qh, lh, channels, keys, hist, s.Hq,   \
                       s.Hkv, p.G, s.L, s.L_max, s.r, p.key_stride, p.sc_chunk)
    if (s.r == 8) DS_SCORE(8);
    else if (s.r == 16) DS_SCORE(16);
    else if (s.r % 8 == 0) DS_SCORE(0);
    else DS_SCORE(-1);
#undef DS_SCORE
    prof_end(KID_SCORE, st);
    return hipGetLastError();
}

hipError_t launch_thresh(void *ws, const Plan &p, hipStream_t st)
{
    prof_begin(KID_THRESH, st);
    hipLaunchKernelGGL(k_thresh, dim3(p.units), dim3(kWG), 0, st,
                       reinterpret_cast<const uint32_t *>(wsp(ws, p.off_hist)),
                       reinterpret_cast<UnitCtl *>(wsp(ws, p.off_ctl)), p.k_eff);
    prof_end(KID_THRESH, st);
    return hipGetLastError();
}

hipError_t launch_cand(void *ws, const Plan &p, const ds_shape_t &s, hipStream_t st)
{
    prof_begin(KID_CAND, st);
    hipLaunchKernelGGL(k_cand, dim3(p.n_ch, p.units), dim3(kWG), (size_t)p.ch * sizeof(uint2), st,
                       reinterpret_cast<const uint32_t *>(wsp(ws, p.off_keys)),
                       reinterpret_cast<UnitCtl *>(wsp(ws, p.off_ctl)),
                       reinterpret_cast<uint2 *>(wsp(ws, p.off_cand)),
                       reinterpret_cast<uint32_t *>(wsp(ws, p.off_ndef)), s.L, p.key_stride, p.ch,
                       p.n_ch);
    prof_end(KID_CAND, st);
    return hipGetLastError();
}

hipError_t launch_refine(void *ws, const Plan &p, const ds_shape_t &s, hipStream_t st)
{
    prof_begin(KID_REFINE, st);
    hipLaunchKernelGGL(k_refine, dim3(p.units), dim3(kWG), (size_t)p.n_ch * sizeof(uint32_t), st,
                       reinterpret_cast<const uint2 *>(wsp(ws, p.off_cand)),
                       reinterpret_cast<UnitCtl *>(wsp(ws, p.off_ctl)),
                       reinterpret_cast<const uint32_t *>(wsp(ws, p.off_ndef)),
                       reinterpret_cast<uint32_t *>(wsp(ws, p.off_offs)), s.L, p.ch, p.n_ch);
    prof_end(KID_REFINE, st);
    return hipGetLastError();
}

hipError_t launch_compact(void *ws, int32_t *idx_out, const Plan &p, const ds_shape_t &s,
                          hipStream_t st)
{
    prof_begin(KID_COMPACT, st);
    hipLaunchKernelGGL(k_compact, dim3(p.n_ch, p.units), dim3(kWG), (size_t)p.ch * sizeof(int), st,
                       reinterpret_cast<const uint32_t *>(wsp(ws, p.off_keys)),
                       reinterpret_cast<const UnitCtl *>(wsp(ws, p.off_ctl)),
                       reinterpret_cast<const uint32_t *>(wsp(ws, p.off_offs)), idx_out, s.L,
                       p.key_stride, p.ch, p.n_ch, s.k, p.k_eff);
    prof_end(KID_COMPACT, st);
    return hipGetLastError();
}

}  // namespace ds
