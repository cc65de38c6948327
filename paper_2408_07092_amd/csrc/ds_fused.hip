// Algorithm 1 in ONE launch: score -> top-k -> gather -> softmax.V for every
// (batch, KV head) unit, with no kernel boundary between the steps.
//
// The grid is sized so that every workgroup is resident at once and has two
// kinds of workgroups:
//   * workers own "items" (one unit's chunk of 1024 tokens).  A worker first
//     scores all its items (keys stay in its LDS, the chunk's key histogram is
//     added to the unit's histogram in the workspace), then extracts the
//     threshold candidates of all its items, then gathers and attends them.
//   * reducers each own a few units.  For a unit they wait until all chunks are
//     scored, find the histogram bin b* holding the k-th largest key and
//     publish it; wait for the chunks' candidates, radix-select the exact k-th
//     key T (ties to the lowest token index) and publish it; wait for the
//     chunks' attention partials and merge them in a fixed order into the output.
// Hand-over: a producer writes its data with device-scope stores or atomics,
// waits until they have been performed, then bumps the unit's counter; the
// reducer polls the counter.  Reducers publish by writing the value, waiting,
// then setting a ready word that workers poll.  Every counter, ready word and
// histogram is cleared by the reducer after its last use, so the workspace is
// clean for the next call.
// A worker runs phase X of ALL its items before phase X+1 of any, and a reducer
// runs step X of all its units before step X+1, so every wait is on work that
// never waits on the waiter; every poll loop is also bounded and raises the
// unit's error word instead of spinning for ever.
// Results are independent of arrival order: counters are integers and every
// floating-point reduction has a fixed order.
#include <algorithm>
#include <mutex>
#include <vector>

#include "ds_attend_core.h"

namespace ds {

DS_TRACE_BUFFER

constexpr int kItemTokens = 1024;  // tokens per item (4 per thread)
constexpr int kCandLds = 2048;     // candidates a reducer keeps in LDS
constexpr int kMaxItems = 12;      // items one worker may own

struct FusedArgs {
    const _Float16 *q, *label, *K, *V;
    const int32_t *channels;
    UnitCtl *ctl;          // [units]
    uint32_t *hist;        // [units][4096] fine histogram (top 12 key bits), zero between calls
    uint32_t *coarse;      // [units][256] coarse histogram (top 8 key bits), zero between calls
    uint32_t *ncd, *ndef;  // [items] candidates / keys above b* of each chunk
    uint32_t *offs;        // [items] offset of the chunk in the ascending index list
    uint2 *mb_cand;        // [items][1024] (key, token)
    uint16_t *deflist;     // [items][1024] tokens above b* (offset in the chunk), two-launch mode
    float *part;           // [units * G][n_ch][kPartStride]
    float *out;
    int32_t *idx_out;
    int Hq, Hkv, G, L, L_max, r, k, k_eff;
    int units, n_ch, items, P, n_svc, max_items;
    int two_launch;        // 1: stop after the candidate phase; k_attend2 finishes the call
    uint32_t spin_limit;
};

__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Polls *p until it equals `want`; false after `limit` polls.
__device__ __forceinline__ bool spin_equals(const uint32_t *p, uint32_t want, uint32_t limit)
{
    for (uint32_t it = 0; it < limit; ++it) {
        if (ld_dev(p) == want) return true;
        __builtin_amdgcn_s_sleep(1);
    }
    return false;
}
// Fire-and-forget device-scope increment.
__device__ __forceinline__ void bump(uint32_t *p)
{
    (void)__hip_atomic_fetch_add(p, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Same compaction as compact_selected, keys of the item in LDS.
__device__ __forceinline__ int compact_item(const uint32_t *keys_item, int t0, int t1, uint32_t T, int tcut,
                                            int *sel, uint32_t *s_w)
{
    const int tid = threadIdx.x;
    const int t = t0 + tid * 4;
    bool f[4];
    uint32_t cnt = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[e] = (t + e < t1) && is_selected(keys_item[tid * 4 + e], t + e, T, tcut);
        cnt += f[e] ? 1u : 0u;
    }
    uint32_t total;
    int pos = (int)block_exclusive_scan(cnt, s_w, &total);
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (f[e]) sel[pos++] = t + e;
    __syncthreads();
    return (int)total;
}

// ---------------------------------------------------------------- worker
template <int GT, int RMODE>
__device__ __forceinline__ void fused_worker(const FusedArgs &a, char *smem, int p)
{
    constexpr int RQ = (RMODE > 0) ? RMODE : kD;
    constexpr int NV = (RMODE > 0) ? RMODE / 8 : 1;
    constexpr int TPT = kItemTokens / kWG;
    __shared__ uint32_t s_bstar[kMaxItems], s_rdy[1], s_val[1][2], s_w[4];
    __shared__ __attribute__((aligned(16))) float sc_sh[4][16];

    uint32_t *hist16 = reinterpret_cast<uint32_t *>(smem);                    // 2048 words, 2 bins each
    uint32_t *keys = hist16 + kHistBins / 2;                                   // max_items * 1024
    float *qs = reinterpret_cast<float *>(keys + (size_t)a.max_items * kItemTokens);
    _Float16 *qsh = reinterpret_cast<_Float16 *>(qs + (size_t)a.max_items * RQ);
    int *sel = reinterpret_cast<int *>(qsh + (size_t)a.max_items * GT * kD);
    float(*wpart)[GT][kPartStride] = reinterpret_cast<float(*)[GT][kPartStride]>(sel + 2 * kItemTokens);

    const int tid = threadIdx.x;
    if (p >= a.items) return;
    const int nj = (a.items - p + a.P - 1) / a.P;
    DS_TR(0);

    // ---- phase S: score every item; keys stay in LDS, the chunk histogram joins the unit's.
    // The first item's label rows, the channel ids and the query rows of all my items are
    // requested together; the label queries are then formed from LDS.
    half8 v[TPT][NV], vn[TPT][NV];
    auto issue = [&](int j, half8(&dst)[TPT][NV]) {
        const int i = p + j * a.P, u = i / a.n_ch, t0 = (i % a.n_ch) * kItemTokens;
        const _Float16 *lab = a.label + (size_t)u * a.L_max * a.r;
#pragma unroll
        for (int e = 0; e < TPT; ++e) {
            const int t = min(t0 + tid + e * kWG, a.L - 1);
            const half8 *row = reinterpret_cast<const half8 *>(lab + (size_t)t * (NV * 8));
#pragma unroll
            for (int x = 0; x < NV; ++x) dst[e][x] = row[x];
        }
    };
    if constexpr (RMODE > 0) {
        issue(0, v);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int idx = tid; idx < nj * GT * 16; idx += kWG) {
        const int j = idx / (GT * 16), g = (idx / 16) % GT, pp = idx % 16;
        const int u = (p + j * a.P) / a.n_ch, b = u / a.Hkv, h = u % a.Hkv;
        const _Float16 *src = a.q + ((size_t)b * a.Hq + (size_t)h * a.G + g) * kD + pp * 8;
        *reinterpret_cast<uint4 *>(&qsh[((size_t)j * GT + g) * kD + pp * 8]) = *reinterpret_cast<const uint4 *>(src);
    }
    int my_ch[(kMaxItems * kD + kWG - 1) / kWG];
#pragma unroll
    for (int e = 0; e < (kMaxItems * kD + kWG - 1) / kWG; ++e) {
        const int idx = tid + e * kWG;
        my_ch[e] = 0;
        if (idx < nj * a.r) {
            const int j = idx / a.r, x = idx % a.r;
            const int h = ((p + j * a.P) / a.n_ch) % a.Hkv;
            my_ch[e] = a.channels[h * a.r + x];
        }
    }
    __syncthreads();
    // label query of the group: sum over its heads (g ascending) of q_g[C[j]]
#pragma unroll
    for (int e = 0; e < (kMaxItems * kD + kWG - 1) / kWG; ++e) {
        const int idx = tid + e * kWG;
        if (idx < nj * a.r) {
            const int j = idx / a.r, x = idx % a.r;
            float sum = 0.0f;
            for (int g = 0; g < a.G; ++g) sum = sum + (float)qsh[((size_t)j * GT + g) * kD + my_ch[e]];
            qs[j * RQ + x] = sum;
        }
    }
    DS_TR(1);
    for (int j = 0; j < nj; ++j) {
        const int i = p + j * a.P, u = i / a.n_ch, t0 = (i % a.n_ch) * kItemTokens;
        if constexpr (RMODE > 0)
            if (j + 1 < nj) issue(j + 1, vn);
#pragma unroll
        for (int e = 0; e < kHistBins / 2 / kWG; ++e) hist16[tid + e * kWG] = 0u;
        __syncthreads();
        uint32_t *kj = keys + (size_t)j * kItemTokens;
        if constexpr (RMODE > 0) {
            float qr[RMODE];
#pragma unroll
            for (int x = 0; x < RMODE; ++x) qr[x] = qs[j * RQ + x];
#pragma unroll
            for (int e = 0; e < TPT; ++e) {
                float acc = 0.0f;
#pragma unroll
                for (int x = 0; x < NV; ++x)
#pragma unroll
                    for (int y = 0; y < 8; ++y) acc = __builtin_fmaf(qr[x * 8 + y], (float)v[e][x][y], acc);
                const int t = t0 + tid + e * kWG;
                const uint32_t key = (t < a.L) ? score_key(acc) : 0u;
                kj[tid + e * kWG] = key;
                if (t < a.L) {
                    const uint32_t bin = key >> kKeyShift;
                    atomicAdd(&hist16[bin >> 1], 1u << ((bin & 1u) * 16u));
                }
            }
        } else {
            const _Float16 *lab = a.label + (size_t)u * a.L_max * a.r;
            for (int e = 0; e < TPT; ++e) {
                const int t = t0 + tid + e * kWG;
                uint32_t key = 0u;
                if (t < a.L) {
                    const _Float16 *row = lab + (size_t)t * a.r;
                    float acc = 0.0f;
                    for (int x = 0; x < a.r; ++x) acc = __builtin_fmaf(qs[j * RQ + x], (float)row[x], acc);
                    key = score_key(acc);
                    const uint32_t bin = key >> kKeyShift;
                    atomicAdd(&hist16[bin >> 1], 1u << ((bin & 1u) * 16u));
                }
                kj[tid + e * kWG] = key;
            }
        }
        __syncthreads();
        {
            // neighbouring lanes add to neighbouring words (atomics of a wave that fall into one
            // cache line are served together); coarse bin tid = fine bins 16*tid .. 16*tid+15
            uint32_t *hu = a.hist + (size_t)u * kHistBins;
            uint32_t w[8], cw[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                w[e] = hist16[tid + e * kWG];
                cw[e] = hist16[tid * 8 + e];
            }
            uint32_t csum = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t lo = w[e] & 0xffffu, hi = w[e] >> 16;
                if (lo) atomicAdd(&hu[2 * (tid + e * kWG)], lo);
                if (hi) atomicAdd(&hu[2 * (tid + e * kWG) + 1], hi);
                csum += (cw[e] & 0xffffu) + (cw[e] >> 16);
            }
            if (csum) atomicAdd(&a.coarse[(size_t)u * 256 + tid], csum);
        }
        wait_stores();
        __syncthreads();
        if (tid == 0) bump(&a.ctl[u].cnt_a);
        if constexpr (RMODE > 0) {
#pragma unroll
            for (int e = 0; e < TPT; ++e)
#pragma unroll
                for (int x = 0; x < NV; ++x) v[e][x] = vn[e][x];
        }
    }
    DS_TR(2);

    // ---- phase C: candidates (keys in the threshold bin) of every item, in step order
    for (int j = 0; j < nj; ++j) {
        const int i = p + j * a.P, u = i / a.n_ch, t0 = (i % a.n_ch) * kItemTokens;
        const int t1 = min(a.L, t0 + kItemTokens);
        const uint32_t *kj = keys + (size_t)j * kItemTokens;
        if (tid == 0) {
            s_rdy[0] = spin_equals(&a.ctl[u].arrive_a, 1u, a.spin_limit) ? 1u : 0u;
            s_bstar[j] = ld_dev(&a.ctl[u].bstar);
        }
        __syncthreads();
        if (j == 0) DS_TR(3);
        if (!s_rdy[0]) {
            if (tid == 0) st_dev(&a.ctl[u].err, 1u);
            return;
        }
        const uint32_t bstar = s_bstar[j];
        bool fc[4];
        uint32_t kd = 0, kc = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int t = t0 + tid * 4 + e;
            const uint32_t bin = kj[tid * 4 + e] >> kKeyShift;
            fc[e] = t < t1 && bin == bstar;
            kd += (t < t1 && bin > bstar) ? 1u : 0u;
            kc += fc[e] ? 1u : 0u;
        }
        uint32_t n_def, n_cand;
        uint32_t pd = block_exclusive_scan(kd, s_w, &n_def);
        uint32_t pc = block_exclusive_scan(kc, s_w, &n_cand);
        uint2 *mb = a.mb_cand + (size_t)i * kItemTokens;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (fc[e]) st_dev(mb + pc++, make_uint2(kj[tid * 4 + e], (uint32_t)(t0 + tid * 4 + e)));
        if (tid == 0) {
            st_dev(a.ncd + i, n_cand);
            st_dev(a.ndef + i, n_def);
        }
        if (a.two_launch) {
            // the attention launch reads the tokens above b* as a list (ascending)
            uint16_t *dl = a.deflist + (size_t)i * kItemTokens;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int t = t0 + tid * 4 + e;
                if (t < t1 && (kj[tid * 4 + e] >> kKeyShift) > bstar) dl[pd++] = (uint16_t)(tid * 4 + e);
            }
            continue;
        }
        wait_stores();
        __syncthreads();
        if (tid == 0) bump(&a.ctl[u].cnt_b);
    }
    if (a.two_launch) return;
    DS_TR(4);

    // ---- phase A, item by item.  The tokens above the threshold bin are certainly selected:
    // their rows are gathered and attended while the reducer settles the exact threshold T
    // among the candidates; the selected candidates' rows follow.  Row order (tokens above b*
    // ascending, then selected candidates ascending) is fixed, so the result is reproducible.
    int *csel = sel + kItemTokens;
    for (int j = 0; j < nj; ++j) {
        const int i = p + j * a.P, u = i / a.n_ch, c = i % a.n_ch, t0 = c * kItemTokens;
        const int t1 = min(a.L, t0 + kItemTokens);
        const uint32_t *kj = keys + (size_t)j * kItemTokens;
        const uint32_t bstar = s_bstar[j];
        uint32_t n_def, n_cand;
        {
            // ordered split of the item's tokens: above b* -> sel[], in b* -> csel[]
            bool fd[4], fc[4];
            uint32_t kd = 0, kc = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int t = t0 + tid * 4 + e;
                const uint32_t bin = kj[tid * 4 + e] >> kKeyShift;
                fd[e] = t < t1 && bin > bstar;
                fc[e] = t < t1 && bin == bstar;
                kd += fd[e] ? 1u : 0u;
                kc += fc[e] ? 1u : 0u;
            }
            uint32_t pd = block_exclusive_scan(kd, s_w, &n_def);
            uint32_t pc = block_exclusive_scan(kc, s_w, &n_cand);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int t = t0 + tid * 4 + e;
                if (fd[e]) sel[pd++] = t;
                if (fc[e]) csel[pc++] = t;
            }
            __syncthreads();
        }
        const char *Ku = reinterpret_cast<const char *>(a.K + (size_t)u * a.L_max * kD);
        const char *Vu = reinterpret_cast<const char *>(a.V + (size_t)u * a.L_max * kD);
        const _Float16(*qj)[kD] = reinterpret_cast<const _Float16(*)[kD]>(qsh + (size_t)j * GT * kD);
        // query groups of 4 or 8 heads run on the matrix cores, 1 or 2 heads on the vector ALUs
        RowState<(GT >= 4 ? 1 : GT)> stv;
        MfmaState stm;
        half8 qreg[4];
        if constexpr (GT >= 4) {
            load_q_mfma(qsh + (size_t)j * GT * kD, GT, qreg);
            stm.init();
        } else {
            stv.init();
        }
        auto attend = [&](const int *list, int n_rows) {
            if constexpr (GT >= 4)
                attend_rows_mfma(Ku, Vu, 2 * kD, n_rows, [&](int ri) { return list[ri]; }, qreg, stm,
                                 sc_sh[tid >> 6]);
            else
                attend_rows<GT>(Ku, Vu, 2 * kD, n_rows, [&](int ri) { return list[ri]; }, qj, stv);
        };
        attend(sel, (int)n_def);

        if (tid == 0) {
            s_rdy[0] = spin_equals(&a.ctl[u].arrive_b, 1u, a.spin_limit) ? 1u : 0u;
            s_val[0][0] = ld_dev(&a.ctl[u].T);
            s_val[0][1] = ld_dev(reinterpret_cast<const uint32_t *>(&a.ctl[u].tcut));
        }
        __syncthreads();
        if (j == 0) DS_TR(5);
        if (!s_rdy[0]) {
            if (tid == 0) st_dev(&a.ctl[u].err, 2u);
            return;
        }
        const uint32_t T = s_val[0][0];
        const int tcut = (int)s_val[0][1];
        uint32_t n_csel;
        {
            // selected candidates, ascending (csel is ascending): compact in place
            int tok[4];
            bool fs[4];
            uint32_t ks = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t x = tid * 4 + e;
                tok[e] = x < n_cand ? csel[x] : t0;
                fs[e] = x < n_cand && is_selected(kj[tok[e] - t0], tok[e], T, tcut);
                ks += fs[e] ? 1u : 0u;
            }
            uint32_t ps = block_exclusive_scan(ks, s_w, &n_csel);  // barriers: all reads of csel done
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (fs[e]) csel[ps++] = tok[e];
            __syncthreads();
        }
        attend(csel, (int)n_csel);
        float *po = a.part + (((size_t)u * a.G) * a.n_ch + c) * kPartStride;
        if constexpr (GT >= 4) wg_store_partial_mfma<GT>(stm, wpart, GT, po, (size_t)a.n_ch * kPartStride);
        else wg_store_partial<GT>(stv, wpart, po, (size_t)a.n_ch * kPartStride);
        if (a.idx_out) {
            // the caller's index list is ascending over all selected tokens of the unit
            __syncthreads();
            const int n = compact_item(kj, t0, t1, T, tcut, sel, s_w);
            int32_t *io = a.idx_out + (size_t)u * a.k;
            const uint32_t off = ld_dev(a.offs + i);
            for (int x = tid; x < n; x += kWG)
                if (off + x < (uint32_t)a.k_eff) io[off + x] = sel[x];
            if (c == 0)
                for (int x = a.k_eff + tid; x < a.k; x += kWG) io[x] = -1;
        }
        wait_stores();
        __syncthreads();
        if (tid == 0) bump(&a.ctl[u].cnt_c);
    }
    DS_TR(6);
}

// ---------------------------------------------------------------- reducer
__device__ __forceinline__ void fused_reducer(const FusedArgs &a, char *smem, int s)
{
    __shared__ uint32_t s_w[4], s_res[2], s_ok, s_fine[16];
    uint32_t *lh = reinterpret_cast<uint32_t *>(smem);                // 2048 words: radix passes
    uint2 *cl = reinterpret_cast<uint2 *>(lh + 2048);                 // kCandLds entries
    uint32_t *cnt = reinterpret_cast<uint32_t *>(cl + kCandLds);      // n_ch words: per-chunk counts
    uint32_t *pos = cnt + a.n_ch;                                     // n_ch (+1) words: per-chunk candidates
    float(*red)[kD] = reinterpret_cast<float(*)[kD]>(pos + ((a.n_ch + 1 + 3) & ~3));
    float(*red_ml)[2] = reinterpret_cast<float(*)[2]>(red + 8);
    const int tid = threadIdx.x;
    __builtin_amdgcn_s_setprio(3);  // the few reducer waves go ahead of the workers sharing their CU
    DS_TR(8);

    // ---- step A: threshold bin b* from the unit's histograms (coarse bin first, then its 16 fine bins)
    for (int u = s; u < a.units; u += a.n_svc) {
        if (tid == 0) s_ok = spin_equals(&a.ctl[u].cnt_a, (uint32_t)a.n_ch, a.spin_limit) ? 1u : 0u;
        __syncthreads();
        if (!s_ok) {
            if (tid == 0) st_dev(&a.ctl[u].err, 3u);
            return;
        }
        uint32_t *cu = a.coarse + (size_t)u * 256, *hu = a.hist + (size_t)u * kHistBins;
        hist_select<1, true>([&](int bin) { return ld_dev(cu + bin); }, (uint32_t)a.k_eff, s_w, s_res);
        const uint32_t cb = s_res[0], rank = s_res[1];
        if (tid < 16) s_fine[tid] = ld_dev(hu + cb * 16 + 15 - tid);  // from the top fine bin down
        __syncthreads();
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
                st_dev(&a.ctl[u].bstar, bin);
            st_dev(&a.ctl[u].krem, krem);
            wait_stores();
            st_dev(&a.ctl[u].arrive_a, 1u);
                st_dev(&a.ctl[u].cnt_a, 0u);
        }
        // all chunks are in: leave the histograms clean for the next call
        for (int i = tid; i < kHistBins; i += kWG) hu[i] = 0u;
        cu[tid] = 0u;
        __syncthreads();
    }
    DS_TR(9);
    if (a.two_launch) return;

    // ---- step B: exact k-th key T among the candidates, tie cut, index-list offsets
    for (int u = s; u < a.units; u += a.n_svc) {
        if (tid == 0) s_ok = spin_equals(&a.ctl[u].cnt_b, (uint32_t)a.n_ch, a.spin_limit) ? 1u : 0u;
        __syncthreads();
        if (!s_ok) {
            if (tid == 0) st_dev(&a.ctl[u].err, 4u);
            return;
        }
        if (u == s) DS_TR(12);
        const uint32_t bstar = ld_dev(&a.ctl[u].bstar);
        uint32_t krem = ld_dev(&a.ctl[u].krem);
        // Four threads per chunk fetch the chunk's counts and its first 16 candidates in one
        // round trip (a chunk rarely has more; the rest follows in a second round); the
        // entries are then packed into LDS behind an exclusive scan of the per-thread counts.
        uint32_t n = 0;
        for (int cbase = 0; cbase < a.n_ch; cbase += kWG / 4) {
            const int c = cbase + (tid >> 2), sub = tid & 3;
            const bool live = c < a.n_ch;
            const size_t i = (size_t)u * a.n_ch + (live ? c : 0);
            const uint32_t nc = live ? ld_dev(a.ncd + i) : 0u;
            const uint32_t nd = live ? ld_dev(a.ndef + i) : 0u;
            const uint2 *mb = a.mb_cand + i * kItemTokens;
            uint2 e[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) e[x] = ld_dev(mb + sub + 4 * x);
            if (live && sub == 0) {
                cnt[c] = nd;
                pos[c] = nc;
            }
            const uint32_t mine = nc > (uint32_t)sub ? (nc - sub + 3) / 4 : 0u;  // entries sub, sub+4, ..
            uint32_t total;
            uint32_t at = n + block_exclusive_scan(mine, s_w, &total);
            n += total;
#pragma unroll
            for (int x = 0; x < 4; ++x)
                if ((uint32_t)x < mine && at + x < (uint32_t)kCandLds) cl[at + x] = e[x];
            for (uint32_t x = 4; x < mine; ++x) {
                const uint2 ex = ld_dev(mb + sub + 4 * x);
                if (at + x < (uint32_t)kCandLds) cl[at + x] = ex;
            }
        }
        const bool in_lds = n <= (uint32_t)kCandLds;
        __syncthreads();
        if (u == s) DS_TR(14);
        auto each = [&](auto f) {
            if (in_lds) {
                for (uint32_t i = tid; i < n; i += kWG) f(cl[i]);
            } else {
                for (int c = 0; c < a.n_ch; ++c) {
                    const uint2 *mb = a.mb_cand + ((size_t)u * a.n_ch + c) * kItemTokens;
                    for (uint32_t e = tid; e < pos[c]; e += kWG) f(ld_dev(mb + e));
                }
            }
        };
        svc_radix_pass<4, true>(each, [](uint2) { return true; },
                                [](uint2 e) { return (e.x >> 10) & 1023u; }, krem, lh, s_w, s_res);
        const uint32_t pre22 = (bstar << 10) | s_res[0];
        krem = s_res[1];
        __syncthreads();
        svc_radix_pass<4, true>(each, [&](uint2 e) { return (e.x >> 10) == pre22; },
                                [](uint2 e) { return e.x & 1023u; }, krem, lh, s_w, s_res);
        const uint32_t T = (pre22 << 10) | s_res[0];
        const uint32_t m_ties = s_res[1];
        const uint32_t n_ties = lh[s_res[0]];
        __syncthreads();
        if (u == s) DS_TR(15);
        int tcut = 0x7fffffff;
        if (m_ties < n_ties) {
            // keep the m_ties lowest token indices among the keys equal to T
            svc_radix_pass<8, false>(each, [&](uint2 e) { return e.x == T; },
                                     [](uint2 e) { return e.y >> 20; }, m_ties, lh, s_w, s_res);
            uint32_t prefix = s_res[0], want = s_res[1];
            __syncthreads();
            svc_radix_pass<4, false>(each, [&](uint2 e) { return e.x == T && (e.y >> 20) == prefix; },
                                     [](uint2 e) { return (e.y >> 10) & 1023u; }, want, lh, s_w, s_res);
            prefix = (prefix << 10) | s_res[0];
            want = s_res[1];
            __syncthreads();
            svc_radix_pass<4, false>(each, [&](uint2 e) { return e.x == T && (e.y >> 10) == prefix; },
                                     [](uint2 e) { return e.y & 1023u; }, want, lh, s_w, s_res);
            tcut = (int)((prefix << 10) | s_res[0]);
            __syncthreads();
        }
        if (a.idx_out) {
            // selected tokens per chunk = keys above b* + selected candidates; prefix -> offsets
            each([&](uint2 e) {
                if (is_selected(e.x, (int)e.y, T, tcut)) atomicAdd(&cnt[e.y / (uint32_t)kItemTokens], 1u);
            });
            __syncthreads();
            const int per = (a.n_ch + kWG - 1) / kWG;
            const int c0 = min(a.n_ch, tid * per), c1 = min(a.n_ch, c0 + per);
            uint32_t sum = 0;
            for (int i = c0; i < c1; ++i) sum += cnt[i];
            uint32_t total;
            uint32_t run = block_exclusive_scan(sum, s_w, &total);
            for (int i = c0; i < c1; ++i) {
                st_dev(a.offs + (size_t)u * a.n_ch + i, run);
                run += cnt[i];
            }
            wait_stores();
        }
        __syncthreads();
        if (tid == 0) {
            st_dev(&a.ctl[u].T, T);
            st_dev(reinterpret_cast<uint32_t *>(&a.ctl[u].tcut), (uint32_t)tcut);
            wait_stores();
            st_dev(&a.ctl[u].arrive_b, 1u);
            st_dev(&a.ctl[u].cnt_b, 0u);
        }
        __syncthreads();
    }
    DS_TR(10);

    // ---- step C: merge the chunk partials of each head in a fixed order
    for (int u = s; u < a.units; u += a.n_svc) {
        if (tid == 0) s_ok = spin_equals(&a.ctl[u].cnt_c, (uint32_t)a.n_ch, a.spin_limit) ? 1u : 0u;
        __syncthreads();
        if (!s_ok) {
            if (tid == 0) st_dev(&a.ctl[u].err, 5u);
            return;
        }
        merge_partials(a.part + (size_t)u * a.G * a.n_ch * kPartStride, a.G, a.n_ch,
                       a.out + (size_t)u * a.G * kD, red, red_ml, [](int, bool) {});
        // every wait on this unit is over: leave its words clean for the next call
        if (tid == 0) {
            st_dev(&a.ctl[u].cnt_c, 0u);
            st_dev(&a.ctl[u].arrive_a, 0u);
            st_dev(&a.ctl[u].arrive_b, 0u);
        }
        __syncthreads();
    }
    DS_TR(11);
}

template <int GT, int RMODE>
__global__ __launch_bounds__(kWG) void k_fused(FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    if ((int)blockIdx.x < a.n_svc) fused_reducer(a, smem, blockIdx.x);
    else fused_worker<GT, RMODE>(a, smem, (int)blockIdx.x - a.n_svc);
}

// ---------------------------------------------------------------- second launch of the two-launch path
// After k_fused stopped behind the candidate phase, every unit has its threshold bin b*, and
// every chunk its list of tokens above b*, its candidates (keys in b*) and their counts.
// Each workgroup of this launch settles the exact threshold for its unit itself -- all
// candidates of the unit (about 1-2 % of its tokens) go to LDS and are radix-selected there;
// doing that in each workgroup costs less than a hand-over between workgroups -- and then
// gathers and attends its own chunks: tokens above b* first, then its selected candidates.
struct Attend2Args {
    const _Float16 *q, *K, *V;
    UnitCtl *ctl;
    const uint32_t *ncd, *ndef;
    const uint2 *mb_cand;
    const uint16_t *deflist;
    float *part, *out;
    int32_t *idx_out;
    int Hq, Hkv, G, L, L_max, k, k_eff, n_ch, m, n_wg;
};

template <int GT>
__global__ __launch_bounds__(kWG) void k_attend2(Attend2Args a)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ uint32_t s_w[4], s_res[2], s_flag;
    __shared__ __attribute__((aligned(16))) float sc_sh[4][16];
    __shared__ __attribute__((aligned(16))) float red[8][kD];
    __shared__ float red_ml[8][2];
    uint32_t *lh = reinterpret_cast<uint32_t *>(smem);                     // 2048 words
    uint2 *cl = reinterpret_cast<uint2 *>(lh + 2048);                      // kCandLds entries
    uint32_t *cnt = reinterpret_cast<uint32_t *>(cl + kCandLds);           // n_ch: selected per chunk
    uint32_t *ncs = cnt + ((a.n_ch + 3) & ~3);                             // n_ch: candidates per chunk
    int *sel = reinterpret_cast<int *>(ncs + ((a.n_ch + 3) & ~3));         // m * 1024 rows
    _Float16 *qsh = reinterpret_cast<_Float16 *>(sel + (size_t)a.m * kItemTokens);  // GT rows
    float(*wpart)[GT][kPartStride] = reinterpret_cast<float(*)[GT][kPartStride]>(qsh + GT * kD);

    const int tid = threadIdx.x;
    const int u = blockIdx.y, cw = blockIdx.x;
    const int b = u / a.Hkv, h = u % a.Hkv;
    const int c_lo = cw * a.m, c_hi = min(a.n_ch, c_lo + a.m);
    const uint32_t bstar = a.ctl[u].bstar;
    uint32_t krem = a.ctl[u].krem;

    if (GT < 4 && tid < GT * 16) {
        const int g = tid >> 4, p = tid & 15;
        const _Float16 *src = a.q + ((size_t)b * a.Hq + (size_t)h * a.G + g) * kD + p * 8;
        *reinterpret_cast<uint4 *>(&qsh[g * kD + p * 8]) = *reinterpret_cast<const uint4 *>(src);
    }

    // ---- all candidates of the unit -> LDS: four threads per chunk fetch the chunk's counts and
    // its first 16 candidates in one round trip; the rest (rare) follows
    uint32_t n = 0;
    for (int cbase = 0; cbase < a.n_ch; cbase += kWG / 4) {
        const int c = cbase + (tid >> 2), sub = tid & 3;
        const bool live = c < a.n_ch;
        const size_t i = (size_t)u * a.n_ch + (live ? c : 0);
        const uint32_t nc = live ? a.ncd[i] : 0u;
        const uint32_t nd = live ? a.ndef[i] : 0u;
        const uint2 *mb = a.mb_cand + i * kItemTokens;
        uint2 e[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) e[x] = mb[sub + 4 * x];
        if (live && sub == 0) {
            cnt[c] = nd;
            ncs[c] = nc;
        }
        const uint32_t mine = nc > (uint32_t)sub ? (nc - sub + 3) / 4 : 0u;
        uint32_t total;
        uint32_t at = n + block_exclusive_scan(mine, s_w, &total);
        n += total;
#pragma unroll
        for (int x = 0; x < 4; ++x)
            if ((uint32_t)x < mine && at + x < (uint32_t)kCandLds) cl[at + x] = e[x];
        for (uint32_t x = 4; x < mine; ++x) {
            const uint2 ex = mb[sub + 4 * x];
            if (at + x < (uint32_t)kCandLds) cl[at + x] = ex;
        }
    }
    const bool in_lds = n <= (uint32_t)kCandLds;
    __syncthreads();
    auto each = [&](auto f) {
        if (in_lds) {
            for (uint32_t i = tid; i < n; i += kWG) f(cl[i]);
        } else {
            for (int c = 0; c < a.n_ch; ++c) {
                const uint2 *mb = a.mb_cand + ((size_t)u * a.n_ch + c) * kItemTokens;
                for (uint32_t e = tid; e < ncs[c]; e += kWG) f(mb[e]);
            }
        }
    };
    // ---- exact k-th key T (10 + 10 key bits), ties towards the lowest token index
    svc_radix_pass<4, true>(each, [](uint2) { return true; },
                            [](uint2 e) { return (e.x >> 10) & 1023u; }, krem, lh, s_w, s_res);
    const uint32_t pre22 = (bstar << 10) | s_res[0];
    krem = s_res[1];
    __syncthreads();
    svc_radix_pass<4, true>(each, [&](uint2 e) { return (e.x >> 10) == pre22; },
                            [](uint2 e) { return e.x & 1023u; }, krem, lh, s_w, s_res);
    const uint32_t T = (pre22 << 10) | s_res[0];
    const uint32_t m_ties = s_res[1];
    const uint32_t n_ties = lh[s_res[0]];
    __syncthreads();
    int tcut = 0x7fffffff;
    if (m_ties < n_ties) {
        svc_radix_pass<8, false>(each, [&](uint2 e) { return e.x == T; },
                                 [](uint2 e) { return e.y >> 20; }, m_ties, lh, s_w, s_res);
        uint32_t prefix = s_res[0], want = s_res[1];
        __syncthreads();
        svc_radix_pass<4, false>(each, [&](uint2 e) { return e.x == T && (e.y >> 20) == prefix; },
                                 [](uint2 e) { return (e.y >> 10) & 1023u; }, want, lh, s_w, s_res);
        prefix = (prefix << 10) | s_res[0];
        want = s_res[1];
        __syncthreads();
        svc_radix_pass<4, false>(each, [&](uint2 e) { return e.x == T && (e.y >> 10) == prefix; },
                                 [](uint2 e) { return e.y & 1023u; }, want, lh, s_w, s_res);
        tcut = (int)((prefix << 10) | s_res[0]);
        __syncthreads();
    }

    // ---- rows of my chunks: tokens above b* (ascending), then the chunk's selected candidates
    int n_rows = 0;
    for (int c = c_lo; c < c_hi; ++c) {
        const size_t i = (size_t)u * a.n_ch + c;
        const int t0 = c * kItemTokens;
        const int nd = (int)a.ndef[i];
        const uint16_t *dl = a.deflist + i * kItemTokens;
        for (int x = tid; x < nd; x += kWG) sel[n_rows + x] = t0 + dl[x];
        n_rows += nd;
        const uint2 *mb = a.mb_cand + i * kItemTokens;
        const uint32_t nc = ncs[c];
        for (uint32_t x0 = 0; x0 < nc; x0 += kWG) {
            const uint32_t x = x0 + tid;
            uint2 e = make_uint2(0u, 0u);
            if (x < nc) e = mb[x];
            const bool f = x < nc && is_selected(e.x, (int)e.y, T, tcut);
            uint32_t total;
            const uint32_t at = block_exclusive_scan(f ? 1u : 0u, s_w, &total);
            if (f) sel[n_rows + at] = (int)e.y;
            n_rows += (int)total;
        }
    }
    __syncthreads();

    if (a.idx_out) {
        // ascending index list: per-chunk counts -> offsets; my chunks merge their two lists via flags
        each([&](uint2 e) {
            if (is_selected(e.x, (int)e.y, T, tcut)) atomicAdd(&cnt[e.y / (uint32_t)kItemTokens], 1u);
        });
        __syncthreads();
        uint32_t *flags = lh;  // 1024 words
        int32_t *io = a.idx_out + (size_t)u * a.k;
        for (int c = c_lo; c < c_hi; ++c) {
            uint32_t off = 0;
            for (int cc = tid; cc < c; cc += kWG) off += cnt[cc];
            uint32_t tot_off;
            (void)block_exclusive_scan(off, s_w, &tot_off);
            for (int x = tid; x < kItemTokens; x += kWG) flags[x] = 0u;
            __syncthreads();
            const size_t i = (size_t)u * a.n_ch + c;
            const int nd = (int)a.ndef[i];
            const uint16_t *dl = a.deflist + i * kItemTokens;
            for (int x = tid; x < nd; x += kWG) flags[dl[x]] = 1u;
            const uint2 *mb = a.mb_cand + i * kItemTokens;
            for (uint32_t x = tid; x < ncs[c]; x += kWG) {
                const uint2 e = mb[x];
                if (is_selected(e.x, (int)e.y, T, tcut)) flags[e.y - (uint32_t)(c * kItemTokens)] = 1u;
            }
            __syncthreads();
            uint32_t mine = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) mine += flags[tid * 4 + e];
            uint32_t total;
            uint32_t at = tot_off + block_exclusive_scan(mine, s_w, &total);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (flags[tid * 4 + e] && at < (uint32_t)a.k_eff) io[at++] = c * kItemTokens + tid * 4 + e;
            __syncthreads();
        }
        if (cw == 0)
            for (int x = a.k_eff + tid; x < a.k; x += kWG) io[x] = -1;
    }

    // ---- gather + attention over my rows, one partial per head
    const char *Ku = reinterpret_cast<const char *>(a.K + (size_t)u * a.L_max * kD);
    const char *Vu = reinterpret_cast<const char *>(a.V + (size_t)u * a.L_max * kD);
    float *po = a.part + (((size_t)u * a.G) * a.n_wg + cw) * kPartStride;
    if constexpr (GT >= 4) {
        half8 qreg[4];
        load_q_mfma(a.q + ((size_t)b * a.Hq + (size_t)h * a.G) * kD, a.G, qreg);
        MfmaState st;
        st.init();
        attend_rows_mfma(Ku, Vu, 2 * kD, n_rows, [&](int ri) { return sel[ri]; }, qreg, st, sc_sh[tid >> 6]);
        wg_store_partial_mfma<GT>(st, wpart, a.G, po, (size_t)a.n_wg * kPartStride);
    } else {
        RowState<GT> st;
        st.init();
        attend_rows<GT>(Ku, Vu, 2 * kD, n_rows, [&](int ri) { return sel[ri]; },
                        reinterpret_cast<const _Float16(*)[kD]>(qsh), st);
        wg_store_partial<GT>(st, wpart, po, (size_t)a.n_wg * kPartStride);
    }

    // ---- last workgroup of the unit: merge the partials, leave the unit's words clean
    if (!last_arrival(&a.ctl[u].arrive_c, gridDim.x, &s_flag)) return;
    if (tid == 0) {
        a.ctl[u].arrive_c = 0u;
        a.ctl[u].arrive_a = 0u;
    }
    merge_partials(a.part + (size_t)u * a.G * a.n_wg * kPartStride, a.G, a.n_wg,
                   a.out + (size_t)u * a.G * kD, red, red_ml, [](int, bool) {});
}

// ---------------------------------------------------------------- host side
static size_t worker_lds(int max_items, int GT, int rq)
{
    return (size_t)(kHistBins / 2) * 4 + (size_t)max_items * kItemTokens * 4 + (size_t)max_items * rq * 4 +
           (size_t)max_items * GT * kD * 2 + (size_t)2 * kItemTokens * 4 + (size_t)4 * GT * kPartStride * 4;
}
static size_t reducer_lds(int n_ch)
{
    return (size_t)2048 * 4 + (size_t)kCandLds * 8 + (size_t)n_ch * 4 + (size_t)((n_ch + 1 + 3) & ~3) * 4 +
           (size_t)8 * kD * 4 + 64 + 16;
}

template <int GT>
static const void *fused_fn(int rmode)
{
    switch (rmode) {
    case 8: return reinterpret_cast<const void *>(&k_fused<GT, 8>);
    case 16: return reinterpret_cast<const void *>(&k_fused<GT, 16>);
    default: return reinterpret_cast<const void *>(&k_fused<GT, -1>);
    }
}
static const void *fused_fn(int G, int rmode)
{
    switch (G) {
    case 1: return fused_fn<1>(rmode);
    case 2: return fused_fn<2>(rmode);
    case 4: return fused_fn<4>(rmode);
    case 8: return fused_fn<8>(rmode);
    default: return nullptr;
    }
}

// The launch shape depends on the device (CU count, occupancy of the kernel); it is looked
// up once per (G, r mode, units, chunks) and remembered.
struct FusedKey { int G, rmode, units, n_ch; FusedPlan plan; };
static std::mutex g_fused_mu;
static std::vector<FusedKey> g_fused_cache;

static bool compute_fused_plan(const ds_shape_t &s, const Plan &p, FusedPlan *f);

bool make_fused_plan(const ds_shape_t &s, const Plan &p, FusedPlan *f)
{
    f->ok = false;
    if (tune_get(3) != 2 && tune_get(3) != 3) return false;  // opt-in: knob 3 = 2 (one launch) or 3 (two)
    const int n_ch = (s.L + kItemTokens - 1) / kItemTokens;
    const int rmode = (s.r == 8) ? 8 : (s.r == 16) ? 16 : -1;
    std::lock_guard<std::mutex> lk(g_fused_mu);
    for (const auto &e : g_fused_cache)
        if (e.G == p.G && e.rmode == rmode && e.units == p.units && e.n_ch == n_ch) {
            *f = e.plan;
            return f->ok;
        }
    compute_fused_plan(s, p, f);
    g_fused_cache.push_back({p.G, rmode, p.units, n_ch, *f});
    return f->ok;
}

static bool compute_fused_plan(const ds_shape_t &s, const Plan &p, FusedPlan *f)
{
    f->ok = false;
    if (p.G != 1 && p.G != 2 && p.G != 4 && p.G != 8) return false;
    const int n_ch = (s.L + kItemTokens - 1) / kItemTokens;
    const long long items = (long long)p.units * n_ch;
    if (items > (1 << 20) || n_ch > 4096) return false;
    const int rmode = (s.r == 8) ? 8 : (s.r == 16) ? 16 : -1;
    const int rq = rmode > 0 ? rmode : kD;
    const void *fn = fused_fn(p.G, rmode);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return false;
    const int n_svc = std::min(p.units, std::max(1, cus / 4));
    for (int mi = 1; mi <= kMaxItems; ++mi) {
        const size_t lds = std::max(worker_lds(mi, p.G, rq), reducer_lds(n_ch));
        if (lds > 64 * 1024) break;
        int per_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kWG, lds) != hipSuccess) return false;
        const long long cap = (long long)per_cu * cus - n_svc;
        if (cap < 1) continue;
        const long long need = (items + mi - 1) / mi;
        if (need > cap) continue;
        if (cap < n_ch) continue;  // a worker must never own two chunks of one unit
        f->P = (int)std::min<long long>(cap, items);
        // spread the items evenly: no worker gets more than max_items
        f->max_items = (int)((items + f->P - 1) / f->P);
        f->P = (int)((items + f->max_items - 1) / f->max_items);
        if (f->max_items > 1 && f->P < n_ch) continue;
        f->n_svc = n_svc;
        f->n_ch = n_ch;
        f->items = (int)items;
        f->lds = std::max(worker_lds(f->max_items, p.G, rq), reducer_lds(n_ch));
        f->rmode = rmode;
        f->ok = true;
        return true;
    }
    return false;
}

hipError_t launch_fused(const void *q, const void *label, const void *K, const void *V,
                        const int32_t *channels, void *ws, float *out, int32_t *idx_out, const Plan &p,
                        const FusedPlan &f, const ds_shape_t &s, hipStream_t st, int two_launch)
{
    char *base = static_cast<char *>(ws);
    FusedArgs a{};
    a.q = static_cast<const _Float16 *>(q);
    a.label = static_cast<const _Float16 *>(label);
    a.K = static_cast<const _Float16 *>(K);
    a.V = static_cast<const _Float16 *>(V);
    a.channels = channels;
    a.ctl = reinterpret_cast<UnitCtl *>(base + p.off_ctl);
    a.hist = reinterpret_cast<uint32_t *>(base + p.off_hist);
    a.coarse = reinterpret_cast<uint32_t *>(base + p.off_coarse);
    a.ncd = reinterpret_cast<uint32_t *>(base + p.off_fused);
    a.ndef = a.ncd + f.items;
    a.offs = a.ndef + f.items;
    a.mb_cand = reinterpret_cast<uint2 *>(a.offs + f.items + (f.items & 1));
    a.part = reinterpret_cast<float *>(a.mb_cand + (size_t)f.items * kItemTokens);
    a.deflist = reinterpret_cast<uint16_t *>(a.part + (size_t)p.units * p.G * f.n_ch * kPartStride);
    a.two_launch = two_launch;
    a.out = out;
    a.idx_out = idx_out;
    a.Hq = s.Hq; a.Hkv = s.Hkv; a.G = p.G; a.L = s.L; a.L_max = s.L_max; a.r = s.r; a.k = s.k;
    a.k_eff = p.k_eff;
    a.units = p.units; a.n_ch = f.n_ch; a.items = f.items; a.P = f.P; a.n_svc = f.n_svc;
    a.max_items = f.max_items;
    a.spin_limit = 1u << 21;
    const void *fn = fused_fn(p.G, f.rmode);
    void *params[] = {&a};
    hipEvent_t ev_a = nullptr, ev_b = nullptr;
    hipError_t e = prof_events(KID_FUSED, &ev_a, &ev_b)
                       ? hipExtLaunchKernel(fn, dim3(f.n_svc + f.P), dim3(kWG), params, f.lds, st, ev_a, ev_b, 0)
                       : hipLaunchKernel(fn, dim3(f.n_svc + f.P), dim3(kWG), params, f.lds, st);
    return e != hipSuccess ? e : hipGetLastError();
}

template <int GT>
static void launch_attend2_gt(const Attend2Args &a, dim3 grid, size_t lds, hipStream_t st)
{
    DS_LAUNCH(KID_ATTEND2, (k_attend2<GT>), grid, dim3(kWG), lds, st, a);
}

hipError_t launch_two(const void *q, const void *label, const void *K, const void *V,
                      const int32_t *channels, void *ws, float *out, int32_t *idx_out, const Plan &p,
                      const FusedPlan &f, const ds_shape_t &s, hipStream_t st)
{
    hipError_t e = launch_fused(q, label, K, V, channels, ws, out, idx_out, p, f, s, st, 1);
    if (e != hipSuccess) return e;
    char *base = static_cast<char *>(ws);
    Attend2Args a{};
    a.q = static_cast<const _Float16 *>(q);
    a.K = static_cast<const _Float16 *>(K);
    a.V = static_cast<const _Float16 *>(V);
    a.ctl = reinterpret_cast<UnitCtl *>(base + p.off_ctl);
    uint32_t *ncd = reinterpret_cast<uint32_t *>(base + p.off_fused);
    a.ncd = ncd;
    a.ndef = ncd + f.items;
    uint32_t *offs = ncd + 2 * (size_t)f.items;
    a.mb_cand = reinterpret_cast<const uint2 *>(offs + f.items + (f.items & 1));
    float *part = reinterpret_cast<float *>(const_cast<uint2 *>(a.mb_cand) + (size_t)f.items * kItemTokens);
    a.part = part;
    a.deflist = reinterpret_cast<const uint16_t *>(part + (size_t)p.units * p.G * f.n_ch * kPartStride);
    a.out = out;
    a.idx_out = idx_out;
    a.Hq = s.Hq; a.Hkv = s.Hkv; a.G = p.G; a.L = s.L; a.L_max = s.L_max; a.k = s.k; a.k_eff = p.k_eff;
    a.n_ch = f.n_ch;
    // chunks per workgroup: about 2048 workgroups for single heads, larger tiles for query groups
    int m = (int)(((long long)p.units * f.n_ch + 2047) / 2048);
    if (p.G >= 4) m *= 2;
    m = std::max(1, std::min(m, 4));
    a.m = m;
    a.n_wg = (f.n_ch + m - 1) / m;
    const int gt = p.G;  // 1, 2, 4 or 8 (checked by the plan)
    const size_t lds = (size_t)2048 * 4 + (size_t)kCandLds * 8 + (size_t)((f.n_ch + 3) & ~3) * 8 + (size_t)m * kItemTokens * 4 + (size_t)gt * kD * 2 +
                       (size_t)4 * gt * kPartStride * 4;
    const dim3 grid(a.n_wg, p.units);
    switch (gt) {
    case 8: launch_attend2_gt<8>(a, grid, lds, st); break;
    case 4: launch_attend2_gt<4>(a, grid, lds, st); break;
    case 2: launch_attend2_gt<2>(a, grid, lds, st); break;
    default: launch_attend2_gt<1>(a, grid, lds, st); break;
    }
    return hipGetLastError();
}

size_t fused_workspace_bytes(const ds_shape_t &s, const Plan &p)
{
    const int n_ch = (s.L + kItemTokens - 1) / kItemTokens;
    const size_t items = (size_t)p.units * n_ch;
    return items * 4 * 3 + 8 + items * kItemTokens * 8 + (size_t)p.units * p.G * n_ch * kPartStride * 4 +
           items * kItemTokens * 2 + 256;
}

}  // namespace ds

#ifdef DS_TRACE
extern "C" int ds_trace_read_fused(void *dst, size_t bytes)
{
    return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(ds::g_trace), bytes, 0, hipMemcpyDeviceToHost);
}
#endif
