// Steps 1-2 of Algorithm 1 on gfx950: approximate scoring and exact per-unit
// top-k as a radix select.
//
//   k_score  streams the label cache (or, in its other modes, the K rows or the
//            4-bit label cache), forms the binary32 approximate score of every
//            token, stores it as an ordered 32-bit key and builds a 4096-bin and
//            a 256-bin histogram of the keys' top bits per unit.  The last
//            workgroup to finish a unit finds the bin b* that holds the k-th
//            largest key and clears the histograms for the next call; for short
//            units it also settles the exact threshold from the keys.
//   k_cand   collects the keys of bin b* (the only ones whose fate is open) and
//            counts, per token chunk, the keys above b*.  The last workgroup of
//            a unit radix-selects the exact k-th key T among the candidates,
//            resolves equal keys towards the lowest token index (tcut), and
//            turns the per-chunk counts into offsets of the ascending index list.
//            (The default decode path does this inside its attention launch
//            instead; ds_select and the three-launch shape use k_cand.)
//   k_compact writes that index list (for callers that only want indices).
// All counters are integers, so the result does not depend on the order in
// which workgroups or atomics complete.
#include <type_traits>

#include "ds_device.h"

namespace ds {

DS_TRACE_BUFFER

// ---------------------------------------------------------------- init
__global__ __launch_bounds__(kWG) void k_init(uint4 *p, size_t n16)
{
    size_t i = (size_t)blockIdx.x * kWG + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * kWG;
    for (; i < n16; i += stride) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// ---------------------------------------------------------------- score
// RMODE 8 / 16: r known at compile time (one or two 16-byte loads per token);
// RMODE 0: r % 8 == 0 (r/8 16-byte loads); RMODE -1: any r, 2-byte loads;
// RMODE -2: no label cache -- `label` is the K cache itself and the r channels of a token are
// picked out of its 256-byte row, the access pattern the label cache exists to avoid (Sec. 4.2,
// ablation in the appendix "Forward without Label Cache").  Same arithmetic, same keys.
// RMODE -3: 4-bit label cache -- `label` holds packed codes (eight nibbles per 32-bit word,
// ceil(r/8) words per token) and the label query carries the channel's step:
// w[j] = (sum_g q_g[C[j]]) * (amax[j] / 7), acc = fma(w[j], code[t,j], acc), j ascending.
template <int RMODE>
__device__ __forceinline__ float label_dot(const _Float16 *__restrict__ row, const float *qs, int r)
{
    float acc = 0.0f;
    if constexpr (RMODE == 0) {
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
                                               const float *__restrict__ amax,
                                               uint32_t *__restrict__ keys, uint32_t *hist,
                                               uint32_t *coarse, UnitCtl *ctl, uint32_t *offs, int Hq, int Hkv,
                                               int G, int L, int L_max, int r, int key_stride, int sc_chunk,
                                               int k_eff, int tail_refine, int want_offsets, int ch, int n_ch)
{
    extern __shared__ uint32_t cnt_sh[];  // n_ch words, used by the refining tail
    __shared__ uint32_t lh[kHistBins];
    __shared__ uint32_t rh[2048];
    __shared__ float qs_sh[kD];
    __shared__ int ch_sh[kD];
    __shared__ __attribute__((aligned(16))) _Float16 qrow_sh[8][kD];
    __shared__ uint32_t s_w[4], s_res[2], s_flag, s_fine[16], s_n;
    const int tid = threadIdx.x;
    const int u = blockIdx.y, b = u / Hkv, h = u % Hkv;
    const int t_begin = blockIdx.x * sc_chunk;
    const int t_end = min(L, t_begin + sc_chunk);
    const _Float16 *lab = label + (size_t)u * L_max * r;
    uint32_t *ku = keys + (size_t)u * key_stride;
    // keys are written through only when this launch's own tail reads them back
    auto put_key = [&](uint32_t *p, uint32_t key) {
        if (tail_refine) st_dev(p, key);
        else *p = key;
    };

    // Fast modes: eight tokens per thread per pass, every load of a pass issued before the
    // first use; lanes past the end re-read the chunk's last token (in bounds) and drop the
    // result.  The first pass is put in flight before the label query is formed.
    constexpr int NV = (RMODE > 0) ? RMODE / 8 : 1;
    constexpr int UNR = 8;
    half8 v[UNR][NV];
    auto issue = [&](int t0) {
#pragma unroll
        for (int i = 0; i < UNR; ++i) {
            const int t = min(t0 + i * kWG, t_end - 1);
            const half8 *row = reinterpret_cast<const half8 *>(lab + (size_t)t * (NV * 8));
#pragma unroll
            for (int j = 0; j < NV; ++j) v[i][j] = label_load<NV>(row + j);
        }
    };
    DS_TR(0);
    // Label query of the group: sum over its heads (g ascending) of q_g[C[j]].  The channel
    // ids and whole query rows (up to 8 heads at a time) are requested together with the first
    // label rows -- one memory round trip instead of two dependent ones -- and the r values are
    // then picked out of LDS.
    int c_q = 0;
    if (tid < r) c_q = channels[h * r + tid];
    float a_q = 0.0f;
    for (int g0 = 0; g0 < G; g0 += 8) {
        const int ng = min(8, G - g0);
        if (g0) __syncthreads();
        if (tid >= 128 && tid - 128 < ng * 16) {
            const int g = (tid - 128) >> 4, pp = (tid - 128) & 15;
            const _Float16 *src = q + ((size_t)b * Hq + (size_t)h * G + g0 + g) * kD + pp * 8;
            *reinterpret_cast<uint4 *>(&qrow_sh[g][pp * 8]) = *reinterpret_cast<const uint4 *>(src);
        }
        if (g0 == 0) {
            if constexpr (RMODE > 0) {
                issue(t_begin + tid);
                __builtin_amdgcn_sched_barrier(0);
            }
            for (int i = tid; i < kHistBins; i += kWG) lh[i] = 0u;
        }
        __syncthreads();
        if (tid < r)
            for (int g = 0; g < ng; ++g) a_q = a_q + (float)qrow_sh[g][c_q];
    }
    if (tid < r) {
        if constexpr (RMODE == -3) a_q = a_q * (amax[(size_t)u * r + tid] / 7.0f);
        qs_sh[tid] = a_q;
        ch_sh[tid] = c_q;
    }
    __syncthreads();

    DS_TR(1);
    if constexpr (RMODE > 0) {
        float qs[RMODE];
#pragma unroll
        for (int j = 0; j < RMODE; ++j) qs[j] = qs_sh[j];
        for (int t0 = t_begin + tid; t0 < t_end;) {
#pragma unroll
            for (int i = 0; i < UNR; ++i) {
                float acc = 0.0f;
#pragma unroll
                for (int j = 0; j < NV; ++j)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(qs[j * 8 + e], (float)v[i][j][e], acc);
                const int t = t0 + i * kWG;
                if (t < t_end) {
                    const uint32_t key = score_key(acc);
                    put_key(ku + t, key);
                    atomicAdd(&lh[key >> kKeyShift], 1u);
                }
            }
            t0 += kWG * UNR;
            if (t0 < t_end) issue(t0);
        }
    } else if constexpr (RMODE == -3) {
        const int W = (r + 7) / 8;
        const uint32_t *cu = reinterpret_cast<const uint32_t *>(label) + (size_t)u * L_max * W;
        auto nib = [](uint32_t word, int i) { return (float)(((int32_t)(word << (28 - 4 * i))) >> 28); };
        // One or two words per token: 16-byte loads of four or two tokens, four loads in flight;
        // w[j] = 0 beyond r (a product of zero leaves the sum as it is).
        auto run_packed = [&](auto wc) {
            constexpr int WW = decltype(wc)::value;  // words per token
            constexpr int TPL = 4 / WW;              // tokens per 16-byte load
            float wr[8 * WW];
#pragma unroll
            for (int j = 0; j < 8 * WW; ++j) wr[j] = j < r ? qs_sh[j] : 0.0f;
            const int t_lastq = (t_end - 1) & ~(TPL - 1);
            for (int t0 = t_begin + tid * TPL; t0 < t_end; t0 += kWG * TPL * 4) {
                uint4 cv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    cv[i] = stream_load(reinterpret_cast<const uint4 *>(cu + (size_t)min(t0 + i * kWG * TPL, t_lastq) * WW));
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t c4[4] = {cv[i].x, cv[i].y, cv[i].z, cv[i].w};
#pragma unroll
                    for (int e = 0; e < TPL; ++e) {
                        const int t = t0 + i * kWG * TPL + e;
                        float acc = 0.0f;
#pragma unroll
                        for (int w = 0; w < WW; ++w)
#pragma unroll
                            for (int j = 0; j < 8; ++j)
                                acc = __builtin_fmaf(wr[w * 8 + j], nib(c4[e * WW + w], j), acc);
                        if (t < t_end) {
                            const uint32_t key = score_key(acc);
                            put_key(ku + t, key);
                            atomicAdd(&lh[key >> kKeyShift], 1u);
                        }
                    }
                }
            }
        };
        if (W == 1 && (L_max & 3) == 0) {
            run_packed(std::integral_constant<int, 1>{});
        } else if (W == 2 && (L_max & 1) == 0) {
            run_packed(std::integral_constant<int, 2>{});
        } else {
            for (int t = t_begin + tid; t < t_end; t += kWG) {
                float acc = 0.0f;
                for (int w = 0; w < W; ++w) {
                    const uint32_t word = cu[(size_t)t * W + w];
                    for (int i = 0; i < 8 && w * 8 + i < r; ++i)
                        acc = __builtin_fmaf(qs_sh[w * 8 + i], nib(word, i), acc);
                }
                const uint32_t key = score_key(acc);
                put_key(ku + t, key);
                atomicAdd(&lh[key >> kKeyShift], 1u);
            }
        }
    } else if constexpr (RMODE == -2) {
        const _Float16 *Ku = label + (size_t)u * L_max * kD;
        for (int t0 = t_begin + tid; t0 < t_end; t0 += kWG * 4) {
            const _Float16 *row[4];
            float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int i = 0; i < 4; ++i) row[i] = Ku + (size_t)min(t0 + i * kWG, t_end - 1) * kD;
#pragma unroll 8
            for (int j = 0; j < r; ++j) {
                const int cj = ch_sh[j];
                const float qj = qs_sh[j];
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] = __builtin_fmaf(qj, (float)row[i][cj], acc[i]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = t0 + i * kWG;
                if (t < t_end) {
                    const uint32_t key = score_key(acc[i]);
                    put_key(ku + t, key);
                    atomicAdd(&lh[key >> kKeyShift], 1u);
                }
            }
        }
    } else {
        for (int t = t_begin + tid; t < t_end; t += kWG) {
            const uint32_t key = score_key(label_dot<RMODE>(lab + (size_t)t * r, qs_sh, r));
            put_key(ku + t, key);
            atomicAdd(&lh[key >> kKeyShift], 1u);
        }
    }
    DS_TR(2);
    __syncthreads();
    uint32_t *hu = hist + (size_t)u * kHistBins;
    uint32_t *cu = coarse + (size_t)u * 256;
    const bool whole_unit = gridDim.x == 1;  // this workgroup scored every token of the unit
    if (!whole_unit) {
        // neighbouring lanes add to neighbouring words (a wavefront's atomics that fall into one
        // cache line are served together); coarse bin tid = fine bins 16*tid .. 16*tid+15
        uint32_t c[kHistBins / kWG], cc = 0;
#pragma unroll
        for (int i = 0; i < kHistBins / kWG; ++i) {
            c[i] = lh[tid + i * kWG];
            cc += lh[tid * 16 + ((i + tid) & 15)];  // (an order of its own per lane: see hist_select)
        }
#pragma unroll
        for (int i = 0; i < kHistBins / kWG; ++i)
            if (c[i]) atomicAdd(&hu[tid + i * kWG], c[i]);
        if (cc) atomicAdd(&cu[tid], cc);
    }

    DS_TR(3);
    if (whole_unit) {
        // The workgroup's own histogram is the unit's: the threshold bin comes straight out of
        // LDS, nothing goes through the unit histograms in memory and no arrival is counted.
        hist_select<kHistBins / kWG, true>([&](int bin) { return lh[bin]; }, (uint32_t)k_eff, s_w, s_res);
        if (tid == 0) {
            ctl[u].bstar = s_res[0];
            ctl[u].krem = s_res[1];
            s_n = 0u;
        }
        if (!tail_refine) return;
        // the tail below reads the keys back: wait until this workgroup's own stores are done
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
        // ---- last workgroup of the unit: threshold bin (coarse bin first, then its 16 fine
        // bins), then leave the histograms clean
        {
            const bool last = last_arrival(&ctl[u].arrive_a, gridDim.x, &s_flag);
            DS_TR(4);
            if (!last) return;
        }
        hist_select<1, true>([&](int bin) { return ld_dev(cu + bin); }, (uint32_t)k_eff, s_w, s_res);
        const uint32_t cb = s_res[0], rank = s_res[1];
        if (tid < 16) s_fine[tid] = ld_dev(hu + cb * 16 + 15 - tid);  // from the top fine bin down
        __syncthreads();
        DS_TR(5);
        if (tid == 0) {
            uint32_t before = 0, bin = 0, krem = 1;
            for (int i = 0; i < 16; ++i) {
                if (before + s_fine[i] >= rank) {
                    bin = cb * 16 + 15 - i;
                    krem = rank - before;
                    break;
                }
                before += s_fine[i];
            }
            ctl[u].bstar = bin;
            ctl[u].krem = krem;
            ctl[u].arrive_a = 0u;
            s_res[0] = bin;
            s_res[1] = krem;
            s_n = 0u;
        }
        for (int i = tid; i < kHistBins; i += kWG) hu[i] = 0u;
        cu[tid] = 0u;
        if (!tail_refine) return;
    }

    // ---- the same workgroup settles the exact threshold: one pass over the unit's keys (all
    // written through by now) collects the keys of bin b*, which are then radix-selected in LDS.
    // For units of up to ~128K tokens this is cheaper than a launch that spreads the pass out.
    __syncthreads();
    const uint32_t bstar = s_res[0];
    uint32_t krem = s_res[1];
    __syncthreads();
    uint2 *cl = reinterpret_cast<uint2 *>(lh);  // the chunk histogram is dead: 2048 candidate slots
    constexpr uint32_t kCap = kHistBins / 2;
    if (want_offsets)
        for (int i = tid; i < n_ch; i += kWG) cnt_sh[i] = 0u;
    __syncthreads();
    // A thread's four consecutive keys lie in one attend chunk (ch % 4 == 0).  Keys of bin b*
    // are rare, so the common case per load is a handful of compares and no branch taken.
    const uint32_t lo_key = bstar << kKeyShift;
    const bool ch_pow2 = (ch & (ch - 1)) == 0;
    const int ch_shift = __builtin_ctz(ch);
    for (int t0 = tid * 4; t0 < L; t0 += kWG * 4 * 8) {
        uint4 kv[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int t = min(t0 + x * kWG * 4, ((L - 1) & ~3));
            const uint2 lo = ld_dev(reinterpret_cast<const uint2 *>(ku + t));
            const uint2 hi = ld_dev(reinterpret_cast<const uint2 *>(ku + t + 2));
            kv[x] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
        uint32_t hits = 0;  // bit 4x+e: key e of load x lies in bin b*
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int t = t0 + x * kWG * 4;
            const uint32_t k4[4] = {kv[x].x, kv[x].y, kv[x].z, kv[x].w};
            uint32_t above = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t rel = k4[e] - lo_key;  // < 2^20 inside b*; wraps to huge below it
                const bool live = t + e < L;
                hits |= (live && rel < (1u << kKeyShift)) ? (1u << (4 * x + e)) : 0u;
                above += (live && k4[e] >= lo_key && rel >= (1u << kKeyShift)) ? 1u : 0u;
            }
            if (want_offsets && above) atomicAdd(&cnt_sh[ch_pow2 ? (t >> ch_shift) : (t / ch)], above);
        }
        if (hits) {
            // one returning LDS atomic per thread and batch, not one per hit
            uint32_t slot = atomicAdd(&s_n, (uint32_t)__builtin_popcount(hits));
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const uint32_t k4[4] = {kv[x].x, kv[x].y, kv[x].z, kv[x].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (hits & (1u << (4 * x + e))) {
                        if (slot < kCap) cl[slot] = make_uint2(k4[e], (uint32_t)(t0 + x * kWG * 4 + e));
                        ++slot;
                    }
                }
            }
        }
    }
    __syncthreads();
    DS_TR(6);
    const uint32_t n = s_n;
    const bool in_lds = n <= kCap;
    auto each = [&](auto f) {
        if (in_lds) {
            for (uint32_t i = tid; i < n; i += kWG) f(cl[i]);
        } else {
            // more candidates than LDS slots (massive ties): walk the keys again
            for (int t = tid; t < L; t += kWG) {
                const uint32_t key = ld_dev(ku + t);
                if ((key >> kKeyShift) == bstar) f(make_uint2(key, (uint32_t)t));
            }
        }
    };
    svc_radix_pass<4, true>(each, [](uint2) { return true; },
                            [](uint2 e) { return (e.x >> 10) & 1023u; }, krem, rh, s_w, s_res);
    const uint32_t pre22 = (bstar << 10) | s_res[0];
    krem = s_res[1];
    __syncthreads();
    svc_radix_pass<4, true>(each, [&](uint2 e) { return (e.x >> 10) == pre22; },
                            [](uint2 e) { return e.x & 1023u; }, krem, rh, s_w, s_res);
    const uint32_t T = (pre22 << 10) | s_res[0];
    const uint32_t m_ties = s_res[1];
    const uint32_t n_ties = rh[s_res[0]];
    __syncthreads();
    int tcut = 0x7fffffff;
    if (m_ties < n_ties) {
        svc_radix_pass<8, false>(each, [&](uint2 e) { return e.x == T; },
                                 [](uint2 e) { return e.y >> 20; }, m_ties, rh, s_w, s_res);
        uint32_t prefix = s_res[0], want = s_res[1];
        __syncthreads();
        svc_radix_pass<4, false>(each, [&](uint2 e) { return e.x == T && (e.y >> 20) == prefix; },
                                 [](uint2 e) { return (e.y >> 10) & 1023u; }, want, rh, s_w, s_res);
        prefix = (prefix << 10) | s_res[0];
        want = s_res[1];
        __syncthreads();
        svc_radix_pass<4, false>(each, [&](uint2 e) { return e.x == T && (e.y >> 10) == prefix; },
                                 [](uint2 e) { return e.y & 1023u; }, want, rh, s_w, s_res);
        tcut = (int)((prefix << 10) | s_res[0]);
        __syncthreads();
    }
    DS_TR(7);
    if (tid == 0) {
        ctl[u].T = T;
        ctl[u].tcut = tcut;
    }
    if (!want_offsets) return;
    each([&](uint2 e) {
        if (is_selected(e.x, (int)e.y, T, tcut)) atomicAdd(&cnt_sh[e.y / (uint32_t)ch], 1u);
    });
    __syncthreads();
    const int per = (n_ch + kWG - 1) / kWG;
    const int c0 = min(n_ch, tid * per), c1 = min(n_ch, c0 + per);
    uint32_t sum = 0;
    for (int i = c0; i < c1; ++i) sum += cnt_sh[i];
    uint32_t total;
    uint32_t run = block_exclusive_scan(sum, s_w, &total);
    for (int i = c0; i < c1; ++i) {
        offs[(size_t)u * n_ch + i] = run;
        run += cnt_sh[i];
    }
    DS_TR(14);
}

// ---------------------------------------------------------------- candidates + exact threshold
// One radix pass of the refinement: histogram `digit(e)` over the candidates
// that satisfy `match(e)`, then pick the bin holding the `want`-th of them.
template <int PER, bool FROM_TOP, class At, class Match, class Digit>
__device__ __forceinline__ void radix_pass(uint32_t n, At at, Match match, Digit digit, uint32_t want,
                                           uint32_t *lh, uint32_t *s_w, uint32_t *res)
{
    for (int i = threadIdx.x; i < kWG * PER; i += kWG) lh[i] = 0u;
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < n; i += kWG) {
        const uint2 e = at(i);
        if (match(e)) atomicAdd(&lh[digit(e)], 1u);
    }
    __syncthreads();
    hist_select<PER, FROM_TOP>([&](int bin) { return lh[bin]; }, want, s_w, res);
}

__global__ __launch_bounds__(kWG) void k_cand(const uint32_t *__restrict__ keys, UnitCtl *ctl,
                                              uint2 *cand, uint32_t *ndef, uint32_t *offs, int L,
                                              int key_stride, int ch, int n_ch, int cap_lds,
                                              int want_offsets)
{
    extern __shared__ uint2 lc[];  // cap_lds candidate slots, then n_ch counters
    __shared__ uint32_t lh[2048];
    __shared__ uint32_t s_cnt, s_def, s_base, s_flag;
    __shared__ uint32_t s_w[4], s_res[2];
    const int tid = threadIdx.x, u = blockIdx.y, c = blockIdx.x;
    if (tid == 0) { s_cnt = 0u; s_def = 0u; }
    __syncthreads();
    DS_TR(8);
    const uint32_t bstar = ctl[u].bstar;
    const int t0 = c * ch, t1 = min(L, t0 + ch);
    const uint32_t *ku = keys + (size_t)u * key_stride;
    uint2 *cu = cand + (size_t)u * L;
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
                    const uint32_t slot = atomicAdd(&s_cnt, 1u);  // slot < tokens of the chunk <= ch
                    lc[slot] = make_uint2(kv[e], (uint32_t)(t + e));
                }
            }
        }
    }
    DS_TR(9);
    if (want_offsets && mydef) atomicAdd(&s_def, mydef);
    __syncthreads();
    if (tid == 0) {
        if (want_offsets) st_dev(ndef + (size_t)u * n_ch + c, s_def);
        s_base = s_cnt ? atomicAdd(&ctl[u].ncand, s_cnt) : 0u;
    }
    __syncthreads();
    {
        // (a unit has L candidates at most; a base beyond that means the workspace was not cleared)
        const uint32_t n = s_cnt, base = s_base;
        if (base + n <= (uint32_t)L) {
            for (uint32_t i = tid; i < n; i += kWG) st_dev(cu + base + i, lc[i]);
        } else if (tid == 0) {
            st_dev(&ctl[u].err, 8u);
        }
    }

    // ---- last workgroup of the unit: exact k-th key among the candidates
    DS_TR(10);
    {
        const bool last = last_arrival(&ctl[u].arrive_b, gridDim.x, &s_flag);
        DS_TR(11);
        if (!last) return;
    }
    const uint32_t n = min(ld_dev(&ctl[u].ncand), (uint32_t)L);
    const bool in_lds = n <= (uint32_t)cap_lds;
    if (in_lds) {
        // up to four loads per thread in flight
        for (uint32_t i0 = tid; i0 < n; i0 += kWG * 4) {
            uint2 e[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) e[x] = ld_dev(cu + min(i0 + x * kWG, n - 1));
#pragma unroll
            for (int x = 0; x < 4; ++x)
                if (i0 + x * kWG < n) lc[i0 + x * kWG] = e[x];
        }
    }
    __syncthreads();
    auto at = [&](uint32_t i) { return in_lds ? lc[i] : ld_dev(cu + i); };
    DS_TR(12);
    uint32_t krem = ctl[u].krem;

    // key bits [19:10] (all candidates share the top 12 bits), then bits [9:0]
    radix_pass<4, true>(n, at, [](uint2) { return true; },
                        [](uint2 e) { return (e.x >> 10) & 1023u; }, krem, lh, s_w, s_res);
    const uint32_t pre22 = (bstar << 10) | s_res[0];
    krem = s_res[1];
    __syncthreads();
    radix_pass<4, true>(n, at, [&](uint2 e) { return (e.x >> 10) == pre22; },
                        [](uint2 e) { return e.x & 1023u; }, krem, lh, s_w, s_res);
    const uint32_t T = (pre22 << 10) | s_res[0];
    const uint32_t m_ties = s_res[1];       // how many keys equal to T are selected
    const uint32_t n_ties = lh[s_res[0]];   // how many keys equal T
    __syncthreads();

    // Equal keys: keep the m_ties lowest token indices -> tcut = the m_ties-th smallest
    // index among them (radix select on the index, 11 + 10 + 10 bits, ascending).
    int tcut = 0x7fffffff;
    if (m_ties < n_ties) {
        radix_pass<8, false>(n, at, [&](uint2 e) { return e.x == T; },
                             [](uint2 e) { return e.y >> 20; }, m_ties, lh, s_w, s_res);
        uint32_t prefix = s_res[0], want = s_res[1];
        __syncthreads();
        radix_pass<4, false>(n, at, [&](uint2 e) { return e.x == T && (e.y >> 20) == prefix; },
                             [](uint2 e) { return (e.y >> 10) & 1023u; }, want, lh, s_w, s_res);
        prefix = (prefix << 10) | s_res[0];
        want = s_res[1];
        __syncthreads();
        radix_pass<4, false>(n, at, [&](uint2 e) { return e.x == T && (e.y >> 10) == prefix; },
                             [](uint2 e) { return e.y & 1023u; }, want, lh, s_w, s_res);
        tcut = (int)((prefix << 10) | s_res[0]);
        __syncthreads();
    }
    DS_TR(13);
    if (tid == 0) {
        ctl[u].T = T;
        ctl[u].tcut = tcut;
        ctl[u].ncand = 0u;
        ctl[u].arrive_b = 0u;
    }
    if (!want_offsets) return;

    // selected tokens per chunk = keys above bin b* (ndef) + selected candidates;
    // exclusive prefix over chunks -> offsets into the ascending index list
    uint32_t *cnt = reinterpret_cast<uint32_t *>(lc + cap_lds);
    for (int i = tid; i < n_ch; i += kWG) cnt[i] = ld_dev(ndef + (size_t)u * n_ch + i);
    __syncthreads();
    for (uint32_t i = tid; i < n; i += kWG) {
        const uint2 e = at(i);
        if (is_selected(e.x, (int)e.y, T, tcut)) atomicAdd(&cnt[e.y / (uint32_t)ch], 1u);
    }
    __syncthreads();
    const int per = (n_ch + kWG - 1) / kWG;
    const int c0 = min(n_ch, tid * per), c1 = min(n_ch, c0 + per);
    uint32_t sum = 0;
    for (int i = c0; i < c1; ++i) sum += cnt[i];
    uint32_t total;
    uint32_t run = block_exclusive_scan(sum, s_w, &total);
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
    __shared__ uint32_t s_w[4];
    const int tid = threadIdx.x, u = blockIdx.y, c = blockIdx.x;
    const int t0 = c * ch, t1 = min(L, t0 + ch);
    const uint32_t T = ctl[u].T;
    const int tcut = ctl[u].tcut;
    const int n = compact_selected(keys + (size_t)u * key_stride, t0, t1, T, tcut, sel, s_w);
    int32_t *io = idx_out + (size_t)u * k;
    const uint32_t off = offs[(size_t)u * n_ch + c];
    for (int i = tid; i < n; i += kWG)
        if (off + i < (uint32_t)k_eff) io[off + i] = sel[i];
    if (c == 0)
        for (int i = k_eff + tid; i < k; i += kWG) io[i] = -1;
}

// ---------------------------------------------------------------- launchers
static inline char *wsp(void *ws, size_t off) { return static_cast<char *>(ws) + off; }

hipError_t launch_init(void *ws, size_t bytes, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + kWG * 4 - 1) / (kWG * 4);
    if (blocks < 1) blocks = 1;
    if (blocks > 65536) blocks = 65536;
    DS_LAUNCH(KID_INIT, k_init, dim3((unsigned)blocks), dim3(kWG), 0, st, static_cast<uint4 *>(ws), n16);
    return hipGetLastError();
}

hipError_t launch_score(const void *q, const void *label, const int32_t *channels, void *ws,
                        const Plan &p, const ds_shape_t &s, bool tail_refine, bool want_offsets,
                        hipStream_t st, ScoreSrc src)
{
    const dim3 grid(p.n_sc, p.units), block(kWG);
    auto *keys = reinterpret_cast<uint32_t *>(wsp(ws, p.off_keys));
    auto *hist = reinterpret_cast<uint32_t *>(wsp(ws, p.off_hist));
    auto *coarse = reinterpret_cast<uint32_t *>(wsp(ws, p.off_coarse));
    auto *ctl = reinterpret_cast<UnitCtl *>(wsp(ws, p.off_ctl));
    auto *offs = reinterpret_cast<uint32_t *>(wsp(ws, p.off_offs));
    const auto *qh = static_cast<const _Float16 *>(q);
    const auto *lh = static_cast<const _Float16 *>(label);
#define DS_SCORE(MODE)                                                                            \
    DS_LAUNCH(KID_SCORE, k_score<MODE>, grid, block, (size_t)p.n_ch * 4, st, qh, lh, channels, src.amax, keys, hist, \
                       coarse, ctl, offs, s.Hq, s.Hkv, p.G, s.L, s.L_max, s.r, p.key_stride, p.sc_chunk,       \
                       p.k_eff, tail_refine ? 1 : 0, want_offsets ? 1 : 0, p.ch, p.n_ch)
    if (src.kind == SRC_Q4) DS_SCORE(-3);
    else if (src.kind == SRC_K_ROWS) DS_SCORE(-2);
    else if (s.r == 8) DS_SCORE(8);
    else if (s.r == 16) DS_SCORE(16);
    else if (s.r % 8 == 0) DS_SCORE(0);
    else DS_SCORE(-1);
#undef DS_SCORE
    return hipGetLastError();
}

hipError_t launch_cand(void *ws, const Plan &p, const ds_shape_t &s, bool want_offsets,
                       hipStream_t st)
{
    const int cap_lds = p.ch > 2048 ? p.ch : 2048;
    const size_t shmem = (size_t)cap_lds * sizeof(uint2) + (size_t)p.n_ch * sizeof(uint32_t);
    DS_LAUNCH(KID_CAND, k_cand, dim3(p.n_ch, p.units), dim3(kWG), shmem, st,
                       reinterpret_cast<const uint32_t *>(wsp(ws, p.off_keys)),
                       reinterpret_cast<UnitCtl *>(wsp(ws, p.off_ctl)),
                       reinterpret_cast<uint2 *>(wsp(ws, p.off_cand)),
                       reinterpret_cast<uint32_t *>(wsp(ws, p.off_ndef)),
                       reinterpret_cast<uint32_t *>(wsp(ws, p.off_offs)), s.L, p.key_stride, p.ch,
                       p.n_ch, cap_lds, want_offsets ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_compact(void *ws, int32_t *idx_out, const Plan &p, const ds_shape_t &s,
                          hipStream_t st)
{
    DS_LAUNCH(KID_COMPACT, k_compact, dim3(p.n_ch, p.units), dim3(kWG), (size_t)p.ch * sizeof(int), st,
                       reinterpret_cast<const uint32_t *>(wsp(ws, p.off_keys)),
                       reinterpret_cast<const UnitCtl *>(wsp(ws, p.off_ctl)),
                       reinterpret_cast<const uint32_t *>(wsp(ws, p.off_offs)), idx_out, s.L,
                       p.key_stride, p.ch, p.n_ch, s.k, p.k_eff);
    return hipGetLastError();
}

}  // namespace ds

#ifdef DS_TRACE
extern "C" int ds_trace_read_select(void *dst, size_t bytes)
{
    return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(ds::g_trace), bytes, 0, hipMemcpyDeviceToHost);
}
#endif

