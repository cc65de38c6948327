// Steps 3-5 of Algorithm 1 on gfx950: gather the selected K/V rows as whole
// 256-byte rows and run exact softmax attention over them; the same kernel body
// serves dense decode (all rows of a token chunk) and attention over rows that
// were gathered beforehand.
//
// Work split: one workgroup per (token chunk, unit).  A wavefront loads four
// rows per instruction -- 16 lanes x 16 bytes cover one row -- so each 16-lane
// group ("slot") owns a row at a time and keeps its own online-softmax state
// (running max m, denominator l, 8 output channels per lane).  The 16 slots of
// a workgroup are merged in a fixed order and written as one partial per chunk;
// the last workgroup of a unit to finish combines the chunk partials of its
// heads in a fixed order, so results are bit-reproducible whichever workgroup
// that happens to be.
// Logits are kept in the log2 domain: s2 = (q.k) * log2(e)/sqrt(d), p = 2^(s2-m).
#include <algorithm>
#include <map>
#include <mutex>
#include <tuple>

#include "ds_attend_core.h"

#define DS_PRIO(x) __builtin_amdgcn_s_setprio(x)

namespace ds {

constexpr int kRowsPerSlot = 4;   // rows of a 16-lane slot in flight (2: -0.2 us on the 64K workload, 8: +0.5)
// ... on the vector path of the 256-thread variants: five, i.e. rounds of 80 rows.  A chunk of the
// 64K workload has 128 +- 11 selected rows; with rounds of 64 nearly half the workgroups run a
// third, almost empty round (31.1 -> 30.9 us/layer; batch 4 x 16K tokens 30.9 -> 30.5; six rows
// per slot: 31.4).
constexpr int kRowsPerSlotVector = 5;
constexpr int kScoreDepth = 8;    // label loads of a thread in flight (4: +1.1 us; 12, 16: no gain)

DS_TRACE_BUFFER

struct AttendArgs {
    const _Float16 *q, *K, *V;
    const uint32_t *keys;
    const UnitCtl *ctl;
    const uint32_t *offs;
    int32_t *idx_out;
    float *part;
    float *out;
    UnitCtl *ctl_rw;
    int Hq, Hkv, G, L, L_max, key_stride, ch, n_ch, k, k_eff, n_rows;
    int kv_stride;       // halves from one token's K (V) row to the next: d, or 2d when K|V interleave
    int unit0;           // k_refine_attend: first unit of this launch (a launch may take a share of the units)
    // k_refine_attend only
    uint2 *cand;         // [units][L] (key, token) of the keys in bin b*, unordered
    uint32_t *ndef;      // [units][n_ch] keys above bin b* per chunk
    uint32_t *offs_rw;   // [units][n_ch] offset of the chunk in the ascending index list
    uint32_t spin_limit;
    // k_refine_attend with the scoring done in the same launch (one workgroup per unit)
    const _Float16 *label;     // [units][L_max][r]
    const int32_t *channels;   // [Hkv][r]
    uint32_t *hist, *coarse;   // unit histograms (4096 / 256 bins), zero between calls
    const float *amax;         // 4-bit label cache: [units][r] largest magnitude per channel
    int r;                     // label channels (4-bit label cache; fp16 labels have it in the kernel's type)
};

// MODE 0: rows = tokens of the chunk that pass the selection predicate
// MODE 1: rows = all tokens of the chunk (dense)
// MODE 2: rows = pre-gathered [k][2][d] K|V pairs
template <int GT, int MODE>
__global__ __launch_bounds__(kWG, (GT == 1 ? 8 : 1)) void k_attend(AttendArgs a)
{
    extern __shared__ int sel[];  // ch words: selected tokens of the chunk (sparse mode only)
    __shared__ uint32_t s_w[4], s_flag;
    __shared__ __attribute__((aligned(16))) float red[8][kD];
    __shared__ float red_ml[8][2];
    __shared__ __attribute__((aligned(16))) _Float16 qsh[GT >= 4 ? 1 : GT][kD];
    __shared__ __attribute__((aligned(16))) float sc_sh[4][16];
    __shared__ __attribute__((aligned(16))) float wpart[4][GT][kPartStride];

    const int tid = threadIdx.x;
    const int u = blockIdx.y, c = blockIdx.x;
    const int b = u / a.Hkv, h = u % a.Hkv;
    const int t0 = c * a.ch;
    int n;
    DS_TR(0);
    if (MODE == 0) {
        const int t1 = min(a.L, t0 + a.ch);
        const uint32_t T = a.ctl[u].T;
        const int tcut = a.ctl[u].tcut;
        n = compact_selected(a.keys + (size_t)u * a.key_stride, t0, t1, T, tcut, sel, s_w);
        if (a.idx_out) {
            int32_t *io = a.idx_out + (size_t)u * a.k;
            const uint32_t off = a.offs[(size_t)u * a.n_ch + c];
            for (int i = tid; i < n; i += kWG)
                if (off + i < (uint32_t)a.k_eff) io[off + i] = sel[i];
            if (c == 0)
                for (int i = a.k_eff + tid; i < a.k; i += kWG) io[i] = -1;
        }
    } else if (MODE == 1) {
        n = min(a.L, t0 + a.ch) - t0;
    } else {
        n = min(a.n_rows, t0 + a.ch) - t0;
    }

    DS_TR(1);
    // unit base pointers are uniform; a row is addressed by a 32-bit byte offset from them
    const char *Ku, *Vu;
    uint32_t row_bytes;
    if (MODE == 2) {
        Ku = reinterpret_cast<const char *>(a.K + ((size_t)u * a.k + t0) * 2 * kD);
        Vu = Ku + kD * 2;
        row_bytes = 4 * kD;
    } else {
        Ku = reinterpret_cast<const char *>(a.K + (size_t)u * a.L_max * a.kv_stride);
        Vu = reinterpret_cast<const char *>(a.V + (size_t)u * a.L_max * a.kv_stride);
        row_bytes = 2 * a.kv_stride;
    }

    auto row_of = [&](int ri) { return (MODE == 0) ? sel[ri] : (MODE == 1) ? (t0 + ri) : ri; };
    const bool single = gridDim.x == 1;  // the unit's only workgroup writes the result itself
    for (int g0 = 0; g0 < a.G; g0 += GT) {
        float *po = a.part + (((size_t)u * a.G + g0) * a.n_ch + c) * kPartStride;
        float *od = single ? a.out + ((size_t)u * a.G + g0) * kD : nullptr;
        const _Float16 *q0 = a.q + ((size_t)b * a.Hq + (size_t)h * a.G + g0) * kD;
        __syncthreads();
        if constexpr (GT >= 4) {
            // query group on the matrix cores: up to GT heads share every gathered row
            const int n_heads = min(GT, a.G - g0);
            half8 qreg[4];
            load_q_mfma(q0, n_heads, qreg);
            MfmaState st;
            st.init();
            attend_rows_mfma(Ku, Vu, row_bytes, n, row_of, qreg, st, sc_sh[tid >> 6]);
            DS_TR(2);
            wg_store_partial_mfma<GT>(st, wpart, n_heads, po, (size_t)a.n_ch * kPartStride, od);
        } else {
            if (tid < GT * 16) {
                const int g = tid >> 4, p = tid & 15;
                *reinterpret_cast<uint4 *>(&qsh[g][p * 8]) = *reinterpret_cast<const uint4 *>(q0 + (size_t)g * kD + p * 8);
            }
            __syncthreads();
            RowState<GT> st;
            st.init();
            attend_rows<GT>(Ku, Vu, row_bytes, n, row_of, qsh, st);
            DS_TR(2);
            wg_store_partial<GT>(st, wpart, po, (size_t)a.n_ch * kPartStride, od);
        }
    }

    // ---- last workgroup of the unit: combine the chunk partials of every head of the group
    DS_TR(3);
    if (single) return;
    {
        const bool last = last_arrival(&a.ctl_rw[u].arrive_c, gridDim.x, &s_flag);
        DS_TR(4);
        if (!last) return;
    }
    if (tid == 0) a.ctl_rw[u].arrive_c = 0u;
    merge_partials(a.part + (size_t)u * a.G * a.n_ch * kPartStride, a.G, a.n_ch,
                   a.out + (size_t)u * a.G * kD, red, red_ml, [](int, bool) {});
    DS_TR(5);
}


// ---------------------------------------------------------------- exact threshold + attention, one launch
// Runs after k_score has left the unit's keys and the threshold bin b* (with the
// rank krem of the k-th key inside it) -- or, with SMODE != 0, does that part itself
// first (Algorithm 1 steps 1-2: label rows streamed, keys kept in LDS, chunk
// histograms met in the unit's histograms in memory; see step 0 in the body), so
// that the whole decode is this one launch.  Tokens whose key lies in a bin above b*
// are selected whatever the exact threshold turns out to be, so a workgroup
//   1. splits its chunk's keys into definite tokens, candidates (bin b*) and the rest,
//      appends the candidates to the unit's list and arrives at the unit's counter;
//   2. attends the definite rows -- the bulk of the traffic -- straight away;
//   3. picks up the exact k-th key T and the tie cut, appends its selected
//      candidates and attends those;
//   4. writes its partial; the unit's last workgroup merges the partials.
// The workgroup whose arrival completes the unit radix-selects T from the
// candidate list before its own step 2 and publishes (T, tie cut, ready) as one
// 64-bit word, so the refinement hides behind the other workgroups' row traffic.
// (A refiner workgroup of its own per unit was tried: it costs a place among the
// resident workgroups and gains nothing measurable.)
// Waiting: a workgroup waits only for the publishing workgroup, which is running
// by then and never waits itself; every workgroup of the unit arrives before
// any waits, and workgroups are dispatched in grid order, so all of a unit's
// workgroups get to run as long as one XCD can hold its share (every eighth) of
// the n_ch of them (checked on the host).  (With SMODE != 0 a workgroup also waits
// for its unit's histogram to be complete, i.e. for workgroups that may not have
// started: the host then sizes the chunks so that the whole grid is resident.)
// Every wait is bounded as well: on expiry the unit's error word is raised and
// the workgroup carries on with a value that keeps all accesses in range.
//
// The body, in order (the "----" comments mark the parts):
//   0.  (SMODE != 0) score the chunk: label query, label rows -> keys in LDS + chunk histogram;
//       threshold bin b*: from the workgroup's own histogram (one workgroup per unit), or the
//       chunk histograms meet in memory and every workgroup finds b* there (vector variants) /
//       the last to arrive finds and publishes it (matrix-core variants)
//   1.  (SMODE == 0) keys and b* of the scoring launch are loaded instead
//   --  classify the keys against b*: row list (definite rows from the front, candidates from the
//       back), candidates to the unit's list in memory, arrival
//   --  (the workgroup that completes the unit) exact threshold T and tie cut by radix select over
//       the candidates; published
//   2-4 definite rows in whole rounds; settle() = wait for (T, tie cut), add the selected
//       candidates (and write the index list if asked); the remaining rows; partial
//   --  (the unit's last workgroup) merge of the partials
// Template: GT heads per pass (1, 2 on the vector ALUs; 4, 8, 16 on the matrix cores), SMODE see
// 0./1., RPS rows per 16-lane slot in flight (4; 8 = the 1024-thread variant of one workgroup
// per unit that has a CU to itself).
template <int GT, int SMODE, int RPS = 4, bool ST = true>
__global__ __launch_bounds__((RPS > 4 ? 1024 : 256), (RPS > 4 ? 1 : (!ST ? 2 : GT == 1 ? 4 : 3))) void k_refine_attend(AttendArgs a)
{
    // Workgroup size: 256 threads; 1024 (four wavefronts per SIMD, 128 registers each: RPS = 8)
    // for the variant that has a CU to itself (RPS > 4: one workgroup per unit, launched with
    // gridDim.x == 1 only), where a single wavefront per SIMD would leave every instruction's
    // latency exposed (C2: 256 threads 56.9, 512 threads 55.7, 1024 threads 55.1 us/layer).
    constexpr int NW = RPS > 4 ? 16 : 4;
    constexpr int WGT = 64 * NW;
    extern __shared__ __attribute__((aligned(16))) uint32_t dyn_sh[];  // ch keys | ch 16-bit row list | n_ch counters
    uint32_t *keys_sh = dyn_sh;
    uint16_t *sel = reinterpret_cast<uint16_t *>(dyn_sh + a.ch);
    uint32_t *cnt = dyn_sh + a.ch + a.ch / 2;
    __shared__ uint32_t s_w[NW], s_flag, s_res[2], s_base, s_T[2], s_ok, s_cnt2;
    __shared__ float red_ml[8][2];
    __shared__ __attribute__((aligned(16))) _Float16 qsh[GT >= 4 ? 1 : GT][kD];
    __shared__ __attribute__((aligned(16))) float sc_sh[4][16];
    // 4 KiB serve the radix bins of the refinement, later the merge of the unit's partials; the
    // workgroup's own wavefront partials lie between the two in time and share the space when
    // they are at least that large
    // On the matrix-core variants, where LDS limits the workgroups per CU, the chunk histogram of
    // the launch that scores as well lives there too (it is dead before any of the above), with
    // the array padded to its 16 KiB where four heads make it smaller.
    constexpr bool kAliasHist = SMODE != 0 && GT >= 4;
    constexpr int kWpartRows = (kAliasHist && 4 * GT * kPartStride < kHistBins) ? 8 : NW;
    __shared__ __attribute__((aligned(16))) float wpart[kWpartRows][GT][kPartStride];
    __shared__ __attribute__((aligned(16))) float red_own[GT >= 2 ? 1 : 8][kD];
    float(*red)[kD] = GT >= 2 ? reinterpret_cast<float(*)[kD]>(&wpart[0][0][0]) : red_own;
    uint32_t *lh = reinterpret_cast<uint32_t *>(&red[0][0]);  // 1024 radix bins

    const int tid = threadIdx.x;
    const int u = blockIdx.y + a.unit0, c = blockIdx.x;
    const int b = u / a.Hkv, h = u % a.Hkv;
    const int t0 = c * a.ch, t1 = min(a.L, t0 + a.ch);
    constexpr int kMaxPass = 8;                              // ch <= 8192
    const int n_pass = (t1 - t0 + WGT * 4 - 1) / (WGT * 4);  // <= kMaxPass
    const uint32_t *ku = a.keys + (size_t)u * a.key_stride;
    uint2 *cu = a.cand + (size_t)u * a.L;
    UnitCtl *ctl = a.ctl_rw + u;
    uint2 *ready = reinterpret_cast<uint2 *>(&ctl->cnt_a);  // {T, tie cut | 1<<31}
    unsigned long long *cand_arrive = reinterpret_cast<unsigned long long *>(&ctl->pad[2]);
    DS_TR(0);
    // A wait for another workgroup that ran out: the unit's error word is raised (it stays up until
    // the workspace is cleared) and the workgroup remembers it for its last arrival, so that the
    // workgroup that would merge the unit writes NaN instead.  A unit whose word is up when the
    // launch starts is not computed at all: its output is NaN again.
    __shared__ uint32_t s_failed;
    auto raise_err = [&](uint32_t code) {
        uint32_t none = 0u;  // (the unit's first code stays)
        __hip_atomic_compare_exchange_strong(&ctl->err, &none, code, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
        s_failed = 1u;
    };
    auto poison_out = [&]() {
        float *ou = a.out + (size_t)u * a.G * kD;
        for (int i = tid; i < a.G * kD; i += WGT) ou[i] = __builtin_nanf("");
    };
    // (the word is asked for here and looked at after the chunk has been scored, before the first
    //  thing that another workgroup could see: the load is off the path)
    const uint32_t sticky = a.ctl[u].err;
    auto refuse_if_poisoned = [&]() {
        if (sticky != 0u && c == 0) poison_out();
        return sticky != 0u;
    };
    if (tid == 0) s_failed = 0u;
    if constexpr (SMODE == 0) {
        if (refuse_if_poisoned()) return;
    }

    // the group's query rows (up to eight at a time), loaded for the label query; single heads and
    // pairs attend with them too, so that no load of q sits between the lists and the rows
    __shared__ __attribute__((aligned(16))) _Float16 qrow_sh[SMODE != 0 ? 8 : 1][kD];
    if constexpr (SMODE == 0 && GT <= 2) {
        if (tid < GT * 16) {
            const int g = tid >> 4, p = tid & 15;
            const _Float16 *q0 = a.q + ((size_t)b * a.Hq + (size_t)h * a.G) * kD;
            *reinterpret_cast<uint4 *>(&qsh[g][p * 8]) = *reinterpret_cast<const uint4 *>(q0 + (size_t)g * kD + p * 8);
        }
    }
    uint32_t bstar = kHistBins - 1, krem_unit = 1;
    if constexpr (SMODE != 0) {
        // ---- 0. Algorithm 1 steps 1-2 right here: stream the chunk's label rows, keys go to LDS
        // only; with one workgroup per unit the threshold bin comes out of its own histogram.
        // Same arithmetic and order as k_score.  SMODE = r for fp16 labels (8 or 16); SMODE = -8 /
        // -16 for the 4-bit label cache of up to 8 / 16 channels (one / two words per token).
        constexpr bool kQ4 = SMODE < 0;
        constexpr int RR = kQ4 ? -SMODE : SMODE;
        constexpr int NV = RR / 8;
        __shared__ uint32_t hist_own[kAliasHist ? 1 : kHistBins];
        auto hist_at = [&](int i) -> uint32_t & {
            if constexpr (kAliasHist) return reinterpret_cast<uint32_t *>(&wpart[0][0][0])[i];
            else return hist_own[i];
        };
        __shared__ float qs_sh[RR];
        if constexpr (kQ4) {
            // label query of the group times the step of each channel (amax / 7); zero beyond r
            int c_q = 0;
            if (tid < a.r) c_q = a.channels[h * a.r + tid];
            float a_q = 0.0f;
            for (int g0 = 0; g0 < a.G; g0 += 8) {
                const int ng = min(8, a.G - g0);
                if (g0) __syncthreads();
                if (tid >= 128 && tid - 128 < ng * 16) {
                    const int g = (tid - 128) >> 4, pp = (tid - 128) & 15;
                    const _Float16 *src = a.q + ((size_t)b * a.Hq + (size_t)h * a.G + g0 + g) * kD + pp * 8;
                    *reinterpret_cast<uint4 *>(&qrow_sh[g][pp * 8]) = *reinterpret_cast<const uint4 *>(src);
                }
                if (g0 == 0)
                    for (int i = tid; i < kHistBins; i += WGT) hist_at(i) = 0u;
                __syncthreads();
                if (tid < a.r)
                    for (int g = 0; g < ng; ++g) a_q = a_q + (float)qrow_sh[g][c_q];
            }
            if (tid < RR) qs_sh[tid] = tid < a.r ? a_q * (a.amax[(size_t)u * a.r + tid] / 7.0f) : 0.0f;
            __syncthreads();
            float wr[RR];
#pragma unroll
            for (int j = 0; j < RR; ++j) wr[j] = qs_sh[j];
            // 16-byte loads of four (two) tokens, four loads per thread in flight
            constexpr int WW = NV, TPL = 4 / WW;
            const uint32_t *codes = reinterpret_cast<const uint32_t *>(a.label) + (size_t)u * a.L_max * WW;
            auto nib = [](uint32_t word, int i) { return (float)(((int32_t)(word << (28 - 4 * i))) >> 28); };
            const int t_lastq = (t1 - 1) & ~(TPL - 1);
            for (int tb = t0 + tid * TPL; tb < t1; tb += WGT * TPL * 4) {
                uint4 cv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    cv[i] = stream_load<ST>(reinterpret_cast<const uint4 *>(codes + (size_t)min(tb + i * WGT * TPL, t_lastq) * WW));
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t c4[4] = {cv[i].x, cv[i].y, cv[i].z, cv[i].w};
#pragma unroll
                    for (int e = 0; e < TPL; ++e) {
                        const int t = tb + i * WGT * TPL + e;
                        float acc = 0.0f;
#pragma unroll
                        for (int w = 0; w < WW; ++w)
#pragma unroll
                            for (int j = 0; j < 8; ++j)
                                acc = __builtin_fmaf(wr[w * 8 + j], nib(c4[e * WW + w], j), acc);
                        if (t < t1) {
                            const uint32_t key = score_key(acc);
                            keys_sh[t - t0] = key;
                            atomicAdd(&hist_at(key >> kKeyShift), 1u);
                        }
                    }
                }
            }
        }
        if constexpr (!kQ4) {
        const _Float16 *lab = a.label + (size_t)u * a.L_max * SMODE;
        constexpr int SD = ST ? kScoreDepth : 2 * kScoreDepth;  // (a mostly idle device: fewer round trips)
        half8 v[SD][NV];
        // (rows past the end of the chunk re-read its last row; their scores are dropped)
        // Rows of two 16-byte pieces (16 channels): a wavefront's two loads take 64 consecutive
        // pieces each -- whole cache lines, so they can carry the streaming mark --, which leaves
        // every lane with the same half of two tokens; neighbouring lanes then swap one piece, and
        // the even lane holds token l/2 of the wavefront's 64, the odd lane token 32 + l/2, whole.
        // (One token per lane straight away means every load takes every other 16 bytes of its
        //  lines: measured 2 us per layer slower on the batch-8 workload.)
        const int lane_ = tid & 63;
        auto token_of = [&](int tb, int i) {
            if constexpr (NV == 2) return tb - lane_ + i * WGT + (lane_ >> 1) + ((lane_ & 1) ? 32 : 0);
            else return tb + i * WGT;
        };
        auto issue = [&](int tb) {
#pragma unroll
            for (int i = 0; i < SD; ++i) {
                if constexpr (NV == 2) {
                    const int p0 = 2 * (tb - lane_ + i * WGT) + lane_, p_last = 2 * t1 - 1;
                    const half8 *pieces = reinterpret_cast<const half8 *>(lab);
                    v[i][0] = label_load<1, ST>(pieces + min(p0, p_last));
                    v[i][1] = label_load<1, ST>(pieces + min(p0 + 64, p_last));
                } else {
                    const half8 *row = reinterpret_cast<const half8 *>(lab + (size_t)min(tb + i * WGT, t1 - 1) * SMODE);
#pragma unroll
                    for (int j = 0; j < NV; ++j) v[i][j] = label_load<NV, ST>(row + j);
                }
            }
        };
        // (NV == 2) the lane's two pieces -> its token's two halves
        auto own_row = [&](half8 (&r)[NV]) {
            if constexpr (NV == 2) {
                const bool odd = lane_ & 1;
                const half8 got = swap_pairs(odd ? r[0] : r[1]);
                if (odd) r[0] = got;
                else r[1] = got;
            }
        };
        int c_q = 0;
        if (tid < SMODE) c_q = a.channels[h * SMODE + tid];
        float a_q = 0.0f;
        for (int g0 = 0; g0 < a.G; g0 += 8) {
            const int ng = min(8, a.G - g0);
            if (g0) __syncthreads();
            if (tid >= 128 && tid - 128 < ng * 16) {
                const int g = (tid - 128) >> 4, pp = (tid - 128) & 15;
                const _Float16 *src = a.q + ((size_t)b * a.Hq + (size_t)h * a.G + g0 + g) * kD + pp * 8;
                *reinterpret_cast<uint4 *>(&qrow_sh[g][pp * 8]) = *reinterpret_cast<const uint4 *>(src);
            }
            if (g0 == 0) {
                issue(t0 + tid);
                __builtin_amdgcn_sched_barrier(0);
                for (int i = tid; i < kHistBins; i += WGT) hist_at(i) = 0u;
            }
            __syncthreads();
            if (tid < SMODE)
                for (int g = 0; g < ng; ++g) a_q = a_q + (float)qrow_sh[g][c_q];
        }
        if (tid < SMODE) qs_sh[tid] = a_q;
        __syncthreads();
        float qs[SMODE];
#pragma unroll
        for (int j = 0; j < SMODE; ++j) qs[j] = qs_sh[j];
        // (NV == 2: a lane's token is not the one of its place, so a wavefront stays together)
        auto more = [&](int tb) { return (NV == 2 ? tb - lane_ : tb) < t1; };
        for (int tb = t0 + tid; more(tb);) {
#pragma unroll
            for (int i = 0; i < SD; ++i) {
                own_row(v[i]);
                float acc = 0.0f;
#pragma unroll
                for (int j = 0; j < NV; ++j)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(qs[j * 8 + e], (float)v[i][j][e], acc);
                const int t = token_of(tb, i);
                if (t < t1) {
                    const uint32_t key = score_key(acc);
                    keys_sh[t - t0] = key;
                    atomicAdd(&hist_at(key >> kKeyShift), 1u);
                }
            }
            tb += WGT * SD;
            if (more(tb)) issue(tb);
        }
        }  // fp16 labels
        DS_PRIO(3);
        if (refuse_if_poisoned()) return;
        __syncthreads();
        DS_TR(11);
        if (gridDim.x == 1) {
            hist_select<kHistBins / WGT, true, NW>([&](int bin) { return hist_at(bin); }, (uint32_t)a.k_eff, s_w, s_res);
            bstar = s_res[0];
            krem_unit = s_res[1];
            __syncthreads();
        } else if constexpr (NW == 4) {
            {
                // Several workgroups per unit: the chunk histograms meet in the unit's histograms in
                // memory (as in k_score).  Every workgroup then waits until all of the unit's have
                // arrived and finds the threshold bin itself, with one round of loads: the 256 coarse
                // bins, and with them the fine bins of the three coarse bins around the one that its
                // own histogram points to (another round only if the unit's lies elsewhere).  Nobody
                // has to publish anything; the histograms are cleared at the launch's end, by the
                // workgroup that merges the unit, when every workgroup has long read them.  (The last
                // to arrive finding the bin and publishing it measured the same or slower.)
                uint32_t *hu = a.hist + (size_t)u * kHistBins;
                uint32_t *cuh = a.coarse + (size_t)u * 256;
                {
                    uint32_t cbin[kHistBins / WGT], cc = 0;
    #pragma unroll
                    for (int i = 0; i < kHistBins / WGT; ++i) {
                        cbin[i] = hist_at(tid + i * WGT);
                        cc += hist_at(tid * 16 + ((i + tid) & 15));  // (an order of its own per lane: see hist_select)
                    }
    #pragma unroll
                    for (int i = 0; i < kHistBins / WGT; ++i)
                        if (cbin[i]) atomicAdd(&hu[tid + i * WGT], cbin[i]);
                    if (cc) atomicAdd(&cuh[tid], cc);
                }
                // (No wait for the adds to be performed before the arrival: an arrival that overtakes
                //  its workgroup's adds is caught by the reader, who checks that the coarse counts add
                //  up to L and the fine counts of the unit's coarse bin to its count, and looks again
                //  if they do not.  One round trip less on every workgroup's path.)
                __syncthreads();
                uint32_t seen = 0;
                if (tid == 0)
                    seen = __hip_atomic_fetch_add(&ctl->arrive_a, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
                // (while the arrival is under way) the coarse bin holding the chunk's share of k
                uint32_t cb0;
                {
                    const uint32_t n_tok = (uint32_t)(t1 - t0);
                    uint32_t k_loc = (uint32_t)(((unsigned long long)a.k_eff * n_tok + (uint32_t)a.L - 1u) / (uint32_t)a.L);
                    k_loc = min(max(k_loc, 1u), n_tok);
                    hist_select<kHistBins / WGT, true, NW>([&](int bin) { return hist_at(bin); }, k_loc, s_w, s_res);
                    cb0 = min(max(s_res[0] >> 4, 1u) - 1u, 253u);  // fine bins of coarse bins cb0 .. cb0 + 2
                }
                if (tid == 0) {
                    const uint32_t n_wg = gridDim.x;
                    uint32_t ok = 1u;
                    if (seen != n_wg) {
                        ok = 0u;
                        for (uint32_t it = 0; it < a.spin_limit; ++it) {
                            if (ld_dev(&ctl->arrive_a) == n_wg) { ok = 1u; break; }
                            __builtin_amdgcn_s_sleep(1);
                        }
                    }
                    s_ok = ok;
                    if (!ok) raise_err(9u);
                }
                __syncthreads();
                DS_TR(12);
                if (s_ok) {
                    __shared__ uint32_t s_fine[16], s_cbn, s_valid;
                    for (uint32_t attempt = 0;; ++attempt) {
                        uint32_t fv = 0;
                        if (tid < 48) fv = ld_dev(hu + cb0 * 16 + tid);
                        const uint32_t myc = ld_dev(cuh + 255 - tid);  // (thread = coarse bin, from the top)
                        if (tid == 0) {
                            s_res[0] = 0u;
                            s_res[1] = 1u;
                            s_cbn = 0xffffffffu;
                        }
                        uint32_t tot;
                        const uint32_t above = block_exclusive_scan<NW>(myc, s_w, &tot);
                        if (above < (uint32_t)a.k_eff && above + myc >= (uint32_t)a.k_eff) {
                            s_res[0] = 255u - (uint32_t)tid;
                            s_res[1] = (uint32_t)a.k_eff - above;
                            s_cbn = myc;
                        }
                        __syncthreads();
                        const uint32_t cb = s_res[0], rank = s_res[1];
                        if (cb - cb0 < 3u) {
                            if (tid < 48 && (uint32_t)(tid >> 4) == cb - cb0) s_fine[15 - (tid & 15)] = fv;
                        } else if (tid < 16) {
                            s_fine[tid] = ld_dev(hu + cb * 16 + 15 - tid);
                        }
                        __syncthreads();
                        if (tid == 0) {
                            // (s_fine runs from the coarse bin's top fine bin down)
                            uint32_t fsum = 0;
                            for (int i = 0; i < 16; ++i) fsum += s_fine[i];
                            const bool valid = tot == (uint32_t)a.L && fsum == s_cbn;
                            uint32_t before = 0, bin = cb * 16, krem = 1;
                            for (int i = 0; i < 16; ++i) {
                                if (before + s_fine[i] >= rank) {
                                    bin = cb * 16 + 15 - i;
                                    krem = rank - before;
                                    break;
                                }
                                before += s_fine[i];
                            }
                            s_T[0] = bin;
                            s_T[1] = krem;
                            s_valid = valid ? 1u : 0u;
                            // (counts that never add up: a workspace that was not cleared, or adds that
                            //  do not arrive)
                            if (!valid && attempt + 1u >= a.spin_limit) {
                                raise_err(9u);
                                s_T[0] = (uint32_t)(kHistBins - 1);
                                s_T[1] = 1u;
                                s_valid = 2u;
                            }
                        }
                        __syncthreads();
                        if (s_valid) break;
                        __builtin_amdgcn_s_sleep(8);
                    }
                } else if (tid == 0) {
                    s_T[0] = (uint32_t)(kHistBins - 1);
                    s_T[1] = 1u;
                }
            }
            __syncthreads();
            bstar = s_T[0];
            krem_unit = s_T[1];
            __syncthreads();
        }
        DS_TR(10);
    } else {
        // ---- 1. the chunk's keys come from the scoring launch, with the unit's threshold bin;
        // all of the thread's key loads are in flight together; the keys then live in LDS
        bstar = ctl->bstar;
        krem_unit = ctl->krem;
        uint4 kv[kMaxPass];
#pragma unroll
        for (int p = 0; p < kMaxPass; ++p) {
            const int t = t0 + (p * WGT + tid) * 4;
            kv[p] = make_uint4(0u, 0u, 0u, 0u);
            if (p < n_pass && t < t1) kv[p] = *reinterpret_cast<const uint4 *>(ku + t);
        }
#pragma unroll
        for (int p = 0; p < kMaxPass; ++p) {
            const int lt = (p * WGT + tid) * 4;
            if (p < n_pass && t0 + lt < t1) *reinterpret_cast<uint4 *>(keys_sh + lt) = kv[p];
        }
    }
    // ---- classify the chunk's keys against bin b*
    const uint32_t lo_key = bstar << kKeyShift;
    // own_keys(p): the thread's four keys of pass p (zeros past the end of the chunk)
    auto own_keys = [&](int p, uint32_t (&k4)[4]) {
        const int lt = (p * WGT + tid) * 4;
        k4[0] = k4[1] = k4[2] = k4[3] = 0u;
        if (t0 + lt < t1) {
            const uint4 v = *reinterpret_cast<const uint4 *>(keys_sh + lt);
            k4[0] = v.x; k4[1] = v.y; k4[2] = v.z; k4[3] = v.w;
        }
    };
    int n_def = 0;
    uint32_t n_cand = 0;
    uint32_t early_base = 0;  // (thread 0, several workgroups per unit, lists made by the single scan)
    // A workgroup that owns a CU (RPS > 4) has nobody else to hide its list work behind, so
    // instructions count: it looks at each key once and orders the lists thread by thread with one
    // scan (any fixed order of the row list will do; only the index list has to be in token order).
    constexpr bool kAllKeys = RPS > 4;
    // (kAllKeys) bit 4 p + e of a mask <-> the thread's key e of pass p, at this place in the chunk:
    auto key_slot = [&](int j) { return ((j >> 2) * WGT + tid) * 4 + (j & 3); };
    uint32_t mcan[2] = {0u, 0u};  // the thread's candidates
    constexpr int kAllPasses = 16384 / (WGT * 4);  // ch <= 16384
    if constexpr (kAllKeys) {
        __syncthreads();  // the keys were stored by other threads
        // One look at each key: which of the thread's keys are definite / candidates goes into two
        // 64-bit masks (few keys are either), and the list writes -- now and when the exact
        // threshold is in -- walk the set bits only.
        uint32_t mdef[2] = {0u, 0u};
#pragma unroll
        for (int p = 0; p < kAllPasses; ++p) {
            const int lt = (p * WGT + tid) * 4;
            uint4 kq = make_uint4(0u, 0u, 0u, 0u);
            if (p < n_pass && t0 + lt < t1) kq = *reinterpret_cast<const uint4 *>(keys_sh + lt);
            const uint32_t k4[4] = {kq.x, kq.y, kq.z, kq.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = p * 4 + e;
                const bool live = p < n_pass && t0 + lt + e < t1;
                const uint32_t bin = k4[e] >> kKeyShift;
                if (live && bin > bstar) mdef[j >> 5] |= 1u << (j & 31);
                if (live && bin == bstar) mcan[j >> 5] |= 1u << (j & 31);
            }
        }
        const uint32_t packed = (uint32_t)(__builtin_popcount(mdef[0]) + __builtin_popcount(mdef[1])) |
                                (uint32_t)(__builtin_popcount(mcan[0]) + __builtin_popcount(mcan[1])) << 16;
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<NW>(packed, s_w, &total);
        int dpos = (int)(ex & 0xffffu);
        int cp = a.ch - 1 - (int)(ex >> 16);
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            for (uint32_t m = mdef[w]; m; m &= m - 1u) sel[dpos++] = (uint16_t)key_slot(w * 32 + __builtin_ctz(m));
            for (uint32_t m = mcan[w]; m; m &= m - 1u) sel[cp--] = (uint16_t)key_slot(w * 32 + __builtin_ctz(m));
        }
        n_def = (int)(total & 0xffffu);
        n_cand = total >> 16;
    }
    if constexpr (!kAllKeys) {
        if constexpr (SMODE == 0) __syncthreads();  // the keys were stored by other threads
        // Each thread owns n_pass groups of four consecutive keys (group p of thread t: keys
        // 4 (p WGT + t) ..: a wavefront's loads then cover the LDS banks evenly).  Both lists are
        // written in thread order, which is the same on every run (only the index list has to be
        // in token order, and that is written further down).
        auto block_keys = [&](int p, uint32_t (&k4)[4]) {
            const int lt = (p * WGT + tid) * 4;
            k4[0] = k4[1] = k4[2] = k4[3] = 0u;
            if (t0 + lt < t1) {
                const uint4 v = *reinterpret_cast<const uint4 *>(keys_sh + lt);
                k4[0] = v.x; k4[1] = v.y; k4[2] = v.z; k4[3] = v.w;
            }
            return lt;
        };
        // One look at each key: which of the thread's keys (64 at most) are definite and which are
        // candidates goes into two masks, and the writes walk the set bits, few as they are
        // (against a counting pass and a writing pass over the keys: C3 -0.2, C4a -0.9 us/layer).
        unsigned long long mdef = 0, mcd = 0;
        for (int p = 0; p < n_pass; ++p) {
            uint32_t k4[4];
            const int lt = block_keys(p, k4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool in = t0 + lt + e < t1 && k4[e] >= lo_key;
                const bool cand = k4[e] - lo_key < (1u << kKeyShift);
                if (in && !cand) mdef |= 1ull << (4 * p + e);
                if (in && cand) mcd |= 1ull << (4 * p + e);
            }
        }
        const uint32_t packed = (uint32_t)__builtin_popcountll(mdef) | ((uint32_t)__builtin_popcountll(mcd) << 16);
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<NW>(packed, s_w, &total);
        DS_TR(13);
        // the chunk's place in the unit's candidate list is fetched while the lists are written
        if (gridDim.x != 1 && tid == 0 && (total >> 16))
            early_base = (uint32_t)__hip_atomic_fetch_add(cand_arrive, (unsigned long long)(total >> 16), __ATOMIC_RELAXED,
                                                          __HIP_MEMORY_SCOPE_AGENT);
        // the candidates follow the definite rows in the row list; both in the thread's key order
        uint32_t dpos = ex & 0xffffu;
        uint32_t cp = (total & 0xffffu) + (ex >> 16);
        for (unsigned long long m = mdef; m; m &= m - 1ull) {
            const int j = __builtin_ctzll(m);
            sel[dpos++] = (uint16_t)(((j >> 2) * WGT + tid) * 4 + (j & 3));
        }
        for (unsigned long long m = mcd; m; m &= m - 1ull) {
            const int j = __builtin_ctzll(m);
            sel[cp++] = (uint16_t)(((j >> 2) * WGT + tid) * 4 + (j & 3));
        }
        n_def = (int)(total & 0xffffu);
        n_cand = total >> 16;
    }
    // where the chunk's i-th candidate waits in the row list: behind the definite rows, or (the
    // variant that looks at each key once) at the list's end, filled from the back
    auto cand_slot = [&](uint32_t i) { return kAllKeys ? a.ch - 1 - (int)i : n_def + (int)i; };
    // A unit with this one workgroup keeps everything in LDS: no candidate list in memory, no
    // arrival, nothing to publish.
    const bool single = gridDim.x == 1;
    if (!single && tid == 0) {
        // candidate count of the unit (low word) and arrivals (high word) share one 64-bit counter
        if constexpr (kAllKeys)
            s_base = n_cand ? (uint32_t)__hip_atomic_fetch_add(cand_arrive, (unsigned long long)n_cand, __ATOMIC_RELAXED,
                                                              __HIP_MEMORY_SCOPE_AGENT)
                            : 0u;
        else
            s_base = early_base;
        if (a.idx_out) st_dev(a.ndef + (size_t)u * a.n_ch + c, (uint32_t)n_def);
    }
    __syncthreads();
    if (!single) {
        // (a unit has L candidates at most; a base beyond that means the workspace was not cleared)
        const uint32_t base = s_base;
        if (base + n_cand <= (uint32_t)a.L) {
            for (uint32_t i = tid; i < n_cand; i += WGT) {
                const int lt = sel[cand_slot(i)];
                st_dev(cu + base + i, make_uint2(keys_sh[lt], (uint32_t)(t0 + lt)));
            }
        } else if (tid == 0) {
            raise_err(8u);
        }
    }
    DS_TR(1);
    bool have_T = single ? true : last_arrival_sum(cand_arrive, gridDim.x, &s_flag, &s_base);
    DS_TR(2);
    uint32_t T = 0;
    int tcut = 0x7fffffff;
    if (have_T) {
        // ---- the unit is complete: exact k-th key among the candidates (10 + 10 key bits), ties
        // to the lowest token (4 + 10 + 10 index bits; tokens are below 2^24).  Up to 2048
        // candidates stay in registers; beyond that every pass re-reads the list.
        const uint32_t n = single ? n_cand : min(s_base, (uint32_t)a.L);  // the completed count came with the arrival
        const bool in_regs = n <= 8u * WGT;
        // candidate i of the unit: out of the list in memory, or (single workgroup) the i-th
        // staged token of this chunk
        auto cand_at = [&](uint32_t i) {
            if (single) {
                const int lt = sel[cand_slot(i)];
                return make_uint2(keys_sh[lt], (uint32_t)(t0 + lt));
            }
            return ld_dev(cu + i);
        };
        uint2 ce[8];
        if (in_regs && n) {
#pragma unroll
            for (int x = 0; x < 8; ++x) ce[x] = cand_at(min((uint32_t)(tid + x * WGT), n - 1));
        }
        auto each = [&](auto f) {
            if (in_regs) {
#pragma unroll
                for (int x = 0; x < 8; ++x)
                    if ((uint32_t)(tid + x * WGT) < n) f(ce[x]);
            } else {
                for (uint32_t i = tid; i < n; i += WGT) f(cand_at(i));
            }
        };
        if (tid == 0) s_cnt2 = 0u;  // (pass 1 has barriers before its first use)
        DS_TR(8);
        uint32_t krem = krem_unit;
        bool settled = false;
        // Up to 256 candidates (short units, as a rule): one per thread, each counts the candidates
        // that sort before it -- key descending, token ascending -- out of LDS, sixteen per step;
        // the one with krem - 1 before it is the unit's k-th key, and its token is the tie cut.
        constexpr uint32_t kRankAll = 256;
        if (n >= 1u && n <= kRankAll) {
            // (key and inverted token as one 64-bit number: sorts before <=> larger; 0 for the rest)
            unsigned long long *s_c = reinterpret_cast<unsigned long long *>(lh);  // (2 KiB of the radix bins' 4)
            const uint2 me2 = ce[0];
            const unsigned long long me =
                (uint32_t)tid < n ? ((unsigned long long)me2.x << 32) | (unsigned long long)(0xffffffffu - me2.y) : 0ull;
            if (tid < (int)kRankAll) s_c[tid] = me;
            __syncthreads();
            if ((uint32_t)tid < n) {
                uint32_t before = 0;
                for (uint32_t j = 0; j < n; j += 16) {
                    unsigned long long o[16];
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[e] = s_c[j + e];
#pragma unroll
                    for (int e = 0; e < 16; ++e) before += o[e] > me ? 1u : 0u;
                }
                if (before + 1u == krem) {
                    s_T[0] = me2.x;
                    s_T[1] = me2.y;
                }
            }
            __syncthreads();
            // (a rank beyond the list means a workspace that was not cleared: take the long way)
            if (krem >= 1u && krem <= n) {
                T = s_T[0];
                tcut = (int)s_T[1];
                settled = true;
            }
        }
        uint32_t pre22 = 0, n22 = 0xffffffffu;
        if (!settled) {
            svc_radix_pass<1024 / WGT, true, NW>(each, [](uint2) { return true; },
                                    [](uint2 e) { return (e.x >> 10) & 1023u; }, krem, lh, s_w, s_res);
            pre22 = (bstar << 10) | s_res[0];
            krem = s_res[1];
            n22 = lh[s_res[0]];  // candidates that share the k-th key's 22-bit prefix
            __syncthreads();
        }
        DS_TR(14);
        if (!settled && n22 <= 64u) {
            // One or two candidates as a rule: they are ranked among themselves by one wavefront,
            // in the order (key descending, token ascending); the one of rank krem is the unit's
            // k-th key, and its token is the tie cut.
            __shared__ uint2 s_small[64];
            each([&](uint2 e) {
                if ((e.x >> 10) == pre22) {
                    const uint32_t slot = atomicAdd(&s_cnt2, 1u);
                    if (slot < 64u) s_small[slot] = e;
                }
            });
            __syncthreads();
            const uint32_t m = min(s_cnt2, 64u);
            if (tid < 64 && (uint32_t)tid < m) {
                const uint2 mine = s_small[tid];
                uint32_t before = 0;
                for (uint32_t j = 0; j < m; ++j) {
                    const uint2 o = s_small[j];
                    before += (o.x > mine.x || (o.x == mine.x && o.y < mine.y)) ? 1u : 0u;
                }
                if (before + 1u == krem) {
                    s_T[0] = mine.x;
                    s_T[1] = mine.y;
                }
            }
            __syncthreads();
            // (counts that do not add up mean a workspace that was not cleared: take the long way)
            if (m == n22 && krem >= 1u && krem <= m) {
                T = s_T[0];
                tcut = (int)s_T[1];
                settled = true;
            }
        }
        if (!settled) {
            svc_radix_pass<1024 / WGT, true, NW>(each, [&](uint2 e) { return (e.x >> 10) == pre22; },
                                    [](uint2 e) { return e.x & 1023u; }, krem, lh, s_w, s_res);
            T = (pre22 << 10) | s_res[0];
            const uint32_t m_ties = s_res[1];
            const uint32_t n_ties = lh[s_res[0]];
            __syncthreads();
            if (m_ties < n_ties) {
                svc_radix_pass<1, false, NW>(each, [&](uint2 e) { return e.x == T; },
                                         [](uint2 e) { return (e.y >> 20) & 255u; }, m_ties, lh, s_w, s_res);
                uint32_t prefix = s_res[0], want = s_res[1];
                __syncthreads();
                svc_radix_pass<1024 / WGT, false, NW>(each, [&](uint2 e) { return e.x == T && (e.y >> 20) == prefix; },
                                         [](uint2 e) { return (e.y >> 10) & 1023u; }, want, lh, s_w, s_res);
                prefix = (prefix << 10) | s_res[0];
                want = s_res[1];
                __syncthreads();
                svc_radix_pass<1024 / WGT, false, NW>(each, [&](uint2 e) { return e.x == T && (e.y >> 10) == prefix; },
                                         [](uint2 e) { return e.y & 1023u; }, want, lh, s_w, s_res);
                tcut = (int)((prefix << 10) | s_res[0]);
                __syncthreads();
            }
        }
        if (a.idx_out && !single) {
            // selected tokens per chunk = keys above b* + selected candidates; prefix -> offsets
            for (int i = tid; i < a.n_ch; i += WGT) cnt[i] = ld_dev(a.ndef + (size_t)u * a.n_ch + i);
            __syncthreads();
            each([&](uint2 e) {
                if (is_selected(e.x, (int)e.y, T, tcut)) atomicAdd(&cnt[e.y / (uint32_t)a.ch], 1u);
            });
            __syncthreads();
            const int per = (a.n_ch + WGT - 1) / WGT;
            const int c0 = min(a.n_ch, tid * per), c1 = min(a.n_ch, c0 + per);
            uint32_t sum = 0;
            for (int i = c0; i < c1; ++i) sum += cnt[i];
            uint32_t total;
            uint32_t run = block_exclusive_scan<NW>(sum, s_w, &total);
            for (int i = c0; i < c1; ++i) {
                st_dev(a.offs_rw + (size_t)u * a.n_ch + i, run);
                run += cnt[i];
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
        DS_TR(15);
        if (!single && tid == 0) {
            st_dev(ready, make_uint2(T, (uint32_t)tcut | 0x80000000u));
            __hip_atomic_store(cand_arrive, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        DS_TR(9);
    }

    // ---- 2..4 per pass over the query group
    const char *Ku = reinterpret_cast<const char *>(a.K + (size_t)u * a.L_max * a.kv_stride);
    const char *Vu = reinterpret_cast<const char *>(a.V + (size_t)u * a.L_max * a.kv_stride);
    const uint32_t row_bytes = 2 * a.kv_stride;
    int n_sel = 0;
    // First the definite rows that fill whole rounds of the workgroup's wavefronts (64 rows a round,
    // or 4 * RPS per wavefront on the vector path); the rest of them joins the selected candidates in one list, so
    // that at most one round of the workgroup runs partly empty.
    // (the variants for calls that move little data run on a mostly idle device, where a round
    //  trip is all that a round of rows costs: eight rows per slot in flight there)
    constexpr int kRowsInFlight = !ST ? 8 : (RPS > 4 || GT > 2) ? RPS : kRowsPerSlotVector;
    constexpr int kRound = (GT >= 4) ? 64 : 4 * NW * kRowsInFlight;
    const int n_first = (n_def / kRound) * kRound;
    auto row_def = [&](int ri) { return t0 + (int)sel[ri]; };
    auto row_rest = [&](int ri) { return t0 + (int)sel[n_first + ri]; };
    // After the definite rows of the first pass: fetch (T, tie cut), append the selected candidates
    // to the row list and write the chunk's slice of the index list.
    auto settle = [&]() {
        if (!have_T) {
            if (tid == 0) {
                uint2 w = make_uint2(0u, 0u);
                uint32_t ok = 0;
                for (uint32_t it = 0; it < a.spin_limit; ++it) {
                    w = ld_dev(ready);
                    if (w.y & 0x80000000u) { ok = 1u; break; }
                    __builtin_amdgcn_s_sleep(1);
                }
                s_T[0] = w.x;
                s_T[1] = w.y & 0x7fffffffu;
                s_ok = ok;
                if (!ok) raise_err(6u);
            }
            __syncthreads();
            T = s_T[0];
            tcut = (int)s_T[1];
            if (!s_ok) { T = 0xffffffffu; tcut = -1; }  // nothing more is selected
            have_T = true;
        }
        DS_TR(4);
        const uint32_t off = (a.idx_out && !single) ? ld_dev(a.offs_rw + (size_t)u * a.n_ch + c) : 0u;
        int32_t *io = a.idx_out ? a.idx_out + (size_t)u * a.k : nullptr;
        int all_base = 0;
        // the row list in thread-major order (any fixed order will do); an index list, if wanted,
        // is written in token order by the pass loop further down
        if constexpr (kAllKeys) {
            uint32_t msel[2] = {0u, 0u};
#pragma unroll
            for (int w = 0; w < 2; ++w)
                for (uint32_t m = mcan[w]; m; m &= m - 1u) {
                    const int bit = __builtin_ctz(m);
                    const int lt = key_slot(w * 32 + bit);
                    if (is_selected(keys_sh[lt], t0 + lt, T, tcut)) msel[w] |= 1u << bit;
                }
            uint32_t total;
            int cp = n_def + (int)block_exclusive_scan<NW>((uint32_t)(__builtin_popcount(msel[0]) + __builtin_popcount(msel[1])),
                                                       s_w, &total);
#pragma unroll
            for (int w = 0; w < 2; ++w)
                for (uint32_t m = msel[w]; m; m &= m - 1u) sel[cp++] = (uint16_t)key_slot(w * 32 + __builtin_ctz(m));
            n_sel = (int)total;
        }
        // The chunk's candidates -- already listed, behind the definite rows -- are all there is to
        // look at for the row list: one scan per 256 of them.  The selected ones close up to the
        // definite rows in place (a batch is read before it is written, and what it writes never
        // reaches the next batch).
        if constexpr (!kAllKeys) {
            for (uint32_t c0 = 0; c0 < n_cand; c0 += WGT) {
                const uint32_t i = c0 + tid;
                int lt = 0;
                bool hit = false;
                if (i < n_cand) {
                    lt = sel[cand_slot(i)];
                    hit = is_selected(keys_sh[lt], t0 + lt, T, tcut);
                }
                uint32_t total;
                const uint32_t ex = block_exclusive_scan<NW>(hit ? 1u : 0u, s_w, &total);
                if (hit) sel[n_def + n_sel + (int)ex] = (uint16_t)lt;
                n_sel += (int)total;
            }
        }
        // the chunk's slice of the index list, in token order: one scan per 1024 keys
        for (int p = 0; p < (io ? n_pass : 0); ++p) {
            const int lt = (p * WGT + tid) * 4;
            uint32_t k4[4];
            own_keys(p, k4);
            bool fs[4];
            uint32_t mine = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                fs[e] = (t0 + lt + e < t1) && is_selected(k4[e], t0 + lt + e, T, tcut);
                mine += fs[e] ? 1u : 0u;
            }
            uint32_t total;
            const uint32_t ex = block_exclusive_scan<NW>(mine, s_w, &total);
            uint32_t ap = off + (uint32_t)all_base + ex;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (fs[e]) {
                    if (ap < (uint32_t)a.k_eff) io[ap] = t0 + lt + e;
                    ++ap;
                }
            }
            all_base += (int)total;
        }
        if (io && c == 0)
            for (int i = a.k_eff + tid; i < a.k; i += WGT) io[i] = -1;
        __syncthreads();
    };

    for (int g0 = 0; g0 < a.G; g0 += GT) {
        float *po = a.part + (((size_t)u * a.G + g0) * a.n_ch + c) * kPartStride;
        float *od = single ? a.out + ((size_t)u * a.G + g0) * kD : nullptr;
        const _Float16 *q0 = a.q + ((size_t)b * a.Hq + (size_t)h * a.G + g0) * kD;
        __syncthreads();
        if constexpr (GT >= 4) {
            const int n_heads = min(GT, a.G - g0);
            half8 qreg[4];
            load_q_mfma(q0, n_heads, qreg);
            MfmaState st;
            st.init();
            // (row loops at the lowest priority, hand-over sections at the highest: a workgroup
            //  that is still making its lists shares the compute unit with two that stream rows)
            DS_PRIO(0);
            attend_rows_mfma<false>(Ku, Vu, row_bytes, n_first, row_def, qreg, st, sc_sh[tid >> 6]);
            DS_PRIO(3);
            if (g0 == 0) { DS_TR(3); settle(); }
            DS_PRIO(2);
            attend_rows_mfma<false>(Ku, Vu, row_bytes, n_def - n_first + n_sel, row_rest, qreg, st, sc_sh[tid >> 6]);
            DS_PRIO(3);
            DS_TR(5);
            wg_store_partial_mfma<GT>(st, wpart, n_heads, po, (size_t)a.n_ch * kPartStride, od);
        } else {
            // (the query rows have been in LDS since the kernel's first steps, barriers passed)
            const _Float16(*qrows)[kD] = SMODE != 0 ? qrow_sh : qsh;
            RowState<GT> st;
            st.init();
            DS_PRIO(0);
            attend_rows<GT, kRowsInFlight, NW, ST>(Ku, Vu, row_bytes, n_first, row_def, qrows, st);
            DS_PRIO(3);
            if (g0 == 0) { DS_TR(3); settle(); }
            DS_PRIO(2);
            attend_rows<GT, kRowsInFlight, NW, ST>(Ku, Vu, row_bytes, n_def - n_first + n_sel, row_rest, qrows, st);
            DS_PRIO(3);
            DS_TR(5);
            wg_store_partial<GT, NW>(st, wpart, po, (size_t)a.n_ch * kPartStride, od);
        }
    }

    // ---- last workgroup of the unit: merge the chunk partials, leave the control words clean
    if (single) return;
    {
        // (the arrival count in the low half of the word; a workgroup whose wait ran out adds a
        //  mark in the high half, which the last one to arrive sees without another load)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const uint32_t mine = s_failed ? 0x10000u : 0u;
            const uint32_t t = __hip_atomic_fetch_add(&ctl->arrive_c, 1u + mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_flag = ((t & 0xffffu) == gridDim.x - 1u) ? 1u : 0u;
            s_ok = ((t >> 16) != 0u || mine != 0u) ? 0u : 1u;
        }
        __syncthreads();
        DS_TR(6);
        if (!s_flag) return;
    }
    const bool unit_ok = s_ok != 0u;
    if (tid == 0) {
        ctl->arrive_c = 0u;
        ctl->cnt_a = 0u;
        ctl->cnt_b = 0u;
    }
    if (!unit_ok) {
        poison_out();
    } else if constexpr (NW == 4) {  // (written for 256 threads; the wider variant never gets here)
        merge_partials(a.part + (size_t)u * a.G * a.n_ch * kPartStride, a.G, a.n_ch,
                       a.out + (size_t)u * a.G * kD, red, red_ml, [](int, bool) {});
    }
    DS_TR(7);
    if constexpr (SMODE != 0 && NW == 4) {
        // every workgroup of the unit has long read the unit's histograms and passed their arrival
        // counter: clean for the next call (off everybody's path but the launch's very end)
        uint4 *hu = reinterpret_cast<uint4 *>(a.hist + (size_t)u * kHistBins);
        for (int i = tid; i < kHistBins / 4; i += WGT) hu[i] = make_uint4(0u, 0u, 0u, 0u);
        a.coarse[(size_t)u * 256 + tid] = 0u;
        if (tid == 0) ctl->arrive_a = 0u;
    }
}

// ---------------------------------------------------------------- launchers
static inline char *wsp(void *ws, size_t off) { return static_cast<char *>(ws) + off; }

// Heads handled per pass over the rows: 1 or 2 on the vector ALUs, 4 / 8 / 16 (padded) on the
// matrix cores; larger groups take several passes of 16.
static int pick_gt(int G)
{
    if (G <= 2) return G;
    if (G <= 4) return 4;
    if (G <= 8) return 8;
    return 16;
}

template <int MODE>
static void launch_attend_mode(int kid, const AttendArgs &a, dim3 grid, size_t shmem, hipStream_t st)
{
    switch (pick_gt(a.G)) {
    case 16: DS_LAUNCH(kid, (k_attend<16, MODE>), grid, dim3(kWG), shmem, st, a); break;
    case 8: DS_LAUNCH(kid, (k_attend<8, MODE>), grid, dim3(kWG), shmem, st, a); break;
    case 4: DS_LAUNCH(kid, (k_attend<4, MODE>), grid, dim3(kWG), shmem, st, a); break;
    case 2: DS_LAUNCH(kid, (k_attend<2, MODE>), grid, dim3(kWG), shmem, st, a); break;
    default: DS_LAUNCH(kid, (k_attend<1, MODE>), grid, dim3(kWG), shmem, st, a); break;
    }
}

hipError_t launch_attend_sparse(const void *q, const void *K, const void *V, void *ws, float *out,
                                int32_t *idx_out, const Plan &p, const ds_shape_t &s,
                                hipStream_t st, int kv_stride)
{
    AttendArgs a{};
    a.q = static_cast<const _Float16 *>(q);
    a.K = static_cast<const _Float16 *>(K);
    a.V = static_cast<const _Float16 *>(V);
    a.keys = reinterpret_cast<const uint32_t *>(wsp(ws, p.off_keys));
    a.ctl = reinterpret_cast<const UnitCtl *>(wsp(ws, p.off_ctl));
    a.ctl_rw = reinterpret_cast<UnitCtl *>(wsp(ws, p.off_ctl));
    a.out = out;
    a.offs = reinterpret_cast<const uint32_t *>(wsp(ws, p.off_offs));
    a.idx_out = idx_out;
    a.part = reinterpret_cast<float *>(wsp(ws, p.off_part));
    a.Hq = s.Hq; a.Hkv = s.Hkv; a.G = p.G; a.L = s.L; a.L_max = s.L_max;
    a.key_stride = p.key_stride; a.ch = p.ch; a.n_ch = p.n_ch; a.k = s.k; a.k_eff = p.k_eff;
    a.n_rows = 0;
    a.kv_stride = kv_stride;
    launch_attend_mode<0>(KID_ATTEND, a, dim3(p.n_ch, p.units), (size_t)p.ch * sizeof(int), st);
    return hipGetLastError();
}

// Whether k_refine_attend can take this plan's chunks: keys loaded from memory come in at most
// eight passes of 1024; a workgroup that scores its unit itself writes them to LDS directly
// (16-bit row offsets: up to 16384 tokens).
bool refine_attend_ok(const Plan &p, bool scores_itself)
{
    return p.ch <= (scores_itself ? 16384 : 8192) && (p.ch & 3) == 0;
}

// ---- the instantiation that serves a launch, by function pointer
using RaFn = void (*)(AttendArgs);
struct RaKernel {
    RaFn fn;
    int threads;
};

// smode: 0 = keys and threshold bin come from the scoring launch; 8 / 16 = fp16 labels of that
// many channels scored here; -8 / -16 = 4-bit labels of up to that many channels scored here.
template <int GT, int RPS, bool ST = true>
static RaFn ra_fn(int smode)
{
    switch (smode) {
    case 0: return RPS > 4 ? nullptr : static_cast<RaFn>(k_refine_attend<GT, 0, 4, ST>);
    case 8: return k_refine_attend<GT, 8, RPS, ST>;
    case 16: return k_refine_attend<GT, 16, RPS, ST>;
    case -8: return k_refine_attend<GT, -8, RPS, ST>;
    default: return k_refine_attend<GT, -16, RPS, ST>;
    }
}

// Whether a sparse decode call marks its loads of label and K/V rows as streaming: when it moves
// 16 MiB or more (the headline shape moves 96 MiB).  A call of a few MiB that finds its rows in the
// caches is up to 1 us of 15 slower with the mark; single heads and pairs have a variant without.
static bool streams_past_caches(const Plan &p, const ds_shape_t &s)
{
    const size_t per_unit = (size_t)s.L * s.r * 2 + (size_t)p.k_eff * 2 * kD * 2;
    return (size_t)p.units * per_unit >= ((size_t)16 << 20);
}

static size_t ra_shmem(const Plan &p) { return (size_t)p.ch * 4 + (size_t)p.ch * 2 + (size_t)p.n_ch * 4; }

static RaKernel ra_kernel(const Plan &p, const ds_shape_t &s, int smode)
{
    const int gt = pick_gt(p.G);
    if (gt <= 2 && !streams_past_caches(p, s) && !(smode && gt == 1 && ra_shmem(p) > (64u << 10) && p.n_ch == 1))
        return {gt == 2 ? ra_fn<2, kRowsPerSlot, false>(smode) : ra_fn<1, kRowsPerSlot, false>(smode), 256};
    // one workgroup per unit that has a CU to itself (LDS): 1024 threads, eight rows per slot in flight
    if (smode && gt == 1 && ra_shmem(p) > (64u << 10) && p.n_ch == 1) return {ra_fn<1, 8>(smode), 1024};
    switch (gt) {
    case 16: return {ra_fn<16, kRowsPerSlot>(smode), 256};
    case 8: return {ra_fn<8, kRowsPerSlot>(smode), 256};
    case 4: return {ra_fn<4, kRowsPerSlot>(smode), 256};
    case 2: return {ra_fn<2, kRowsPerSlot>(smode), 256};
    default: return {ra_fn<1, kRowsPerSlot>(smode), 256};
    }
}

// 0 when the labels cannot be scored in the attention launch
static int ra_smode(const ds_shape_t &s, bool scores_itself, bool q4)
{
    if (!scores_itself) return 0;
    if (q4) return (s.r > 16 || (s.L_max & (s.r > 8 ? 1 : 3))) ? 0 : (s.r > 8 ? -16 : -8);
    return (s.r == 8 || s.r == 16) ? s.r : 0;
}

// What the runtime says of a kernel, asked once per (kernel, dynamic LDS): more than 64 KiB of
// dynamic LDS has to be granted first (all that the compute unit has beyond the kernel's static
// arrays); then the number of its workgroups that one compute unit holds at a time.
static int ra_workgroups_per_cu(const RaKernel &k, size_t shmem, const DeviceCaps &caps)
{
    struct Key {
        const void *fn;
        size_t shmem;
        int dev;
        bool operator<(const Key &o) const { return std::tie(fn, shmem, dev) < std::tie(o.fn, o.shmem, o.dev); }
    };
    static std::mutex mu;
    static std::map<Key, int> cache;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    const void *fn = reinterpret_cast<const void *>(k.fn);
    std::lock_guard<std::mutex> lk(mu);
    const Key key{fn, shmem, dev};
    auto it = cache.find(key);
    if (it != cache.end()) return it->second;
    int per_cu = 0;
    bool ok = true;
    if (shmem > (64u << 10)) {
        hipFuncAttributes fa;
        ok = hipFuncGetAttributes(&fa, fn) == hipSuccess;
        const int room = ok ? caps.lds_per_cu - (int)fa.sharedSizeBytes : 0;
        ok = ok && (size_t)room >= shmem &&
             hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, room) == hipSuccess;
    }
    if (ok && hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, k.threads, shmem) != hipSuccess) per_cu = 0;
    if (!ok) per_cu = 0;
    (void)hipGetLastError();
    cache[key] = per_cu;
    return per_cu;
}

// Whether the device holds, at the same time, all the workgroups that a launch of this plan lets
// wait for each other.  A launch that scores as well waits (for its unit's histogram) for
// workgroups that may not have started: the whole grid has to be resident.  After a scoring
// launch a workgroup waits only for one that is running; workgroups start in grid order and are
// dealt out to the dies in turn, so one die has to hold its share of a unit's workgroups.  A unit
// with a single workgroup waits for nobody.
static bool ra_fits(const RaKernel &k, const Plan &p, int smode)
{
    if (!k.fn) return false;
    const DeviceCaps caps = device_caps();
    const int per_cu = ra_workgroups_per_cu(k, ra_shmem(p), caps);
    if (per_cu < 1) return false;
    if (p.n_ch == 1) return true;
    if (smode != 0) return (int64_t)p.n_ch * ((p.units + p.unit_groups - 1) / p.unit_groups) <= (int64_t)per_cu * caps.cus;
    const int dies = std::max(1, caps.xccs);
    return (p.n_ch + dies - 1) / dies <= per_cu * std::max(1, caps.cus / dies);
}

bool refine_attend_fits(const Plan &p, const ds_shape_t &s, bool scores_itself, bool q4)
{
    const int smode = ra_smode(s, scores_itself, q4);
    if (scores_itself && smode == 0) return false;
    return ra_fits(ra_kernel(p, s, smode), p, smode);
}

// score_label / score_channels: non-null to run the scoring in the same launch (fp16 labels of 8
// or 16 channels; with score_amax the 4-bit label cache of up to 16 channels, whose token rows
// must be 16-byte loadable: L_max % 4 == 0 for one word per token, L_max % 2 == 0 for two);
// otherwise the keys and the threshold bin of a preceding k_score launch are read from the
// workspace.  kNotResident, with nothing enqueued, when the device cannot hold the workgroups
// that would wait for each other.
hipError_t launch_refine_attend(const void *q, const void *K, const void *V, void *ws, float *out,
                                int32_t *idx_out, const Plan &p, const ds_shape_t &s, hipStream_t st,
                                int kv_stride, const void *score_label, const int32_t *score_channels,
                                const float *score_amax)
{
    AttendArgs a{};
    a.q = static_cast<const _Float16 *>(q);
    a.K = static_cast<const _Float16 *>(K);
    a.V = static_cast<const _Float16 *>(V);
    a.keys = reinterpret_cast<const uint32_t *>(wsp(ws, p.off_keys));
    a.ctl = reinterpret_cast<const UnitCtl *>(wsp(ws, p.off_ctl));
    a.ctl_rw = reinterpret_cast<UnitCtl *>(wsp(ws, p.off_ctl));
    a.out = out;
    a.offs = reinterpret_cast<const uint32_t *>(wsp(ws, p.off_offs));
    a.offs_rw = reinterpret_cast<uint32_t *>(wsp(ws, p.off_offs));
    a.cand = reinterpret_cast<uint2 *>(wsp(ws, p.off_cand));
    a.ndef = reinterpret_cast<uint32_t *>(wsp(ws, p.off_ndef));
    a.idx_out = idx_out;
    a.part = reinterpret_cast<float *>(wsp(ws, p.off_part));
    a.Hq = s.Hq; a.Hkv = s.Hkv; a.G = p.G; a.L = s.L; a.L_max = s.L_max;
    a.key_stride = p.key_stride; a.ch = p.ch; a.n_ch = p.n_ch; a.k = s.k; a.k_eff = p.k_eff;
    a.spin_limit = tune_get(5) ? (uint32_t)tune_get(5) : 1u << 21;
    a.kv_stride = kv_stride;
    a.label = static_cast<const _Float16 *>(score_label);
    a.channels = score_channels;
    a.hist = reinterpret_cast<uint32_t *>(wsp(ws, p.off_hist));
    a.coarse = reinterpret_cast<uint32_t *>(wsp(ws, p.off_coarse));
    a.amax = score_amax;
    a.r = s.r;
    const int smode = ra_smode(s, score_label != nullptr, score_amax != nullptr);
    if (score_label && smode == 0) return hipErrorInvalidValue;
    const RaKernel k = ra_kernel(p, s, smode);
    if (!k.fn) return hipErrorInvalidValue;
    if (!ra_fits(k, p, smode)) return kNotResident;
    // (a launch that scores as well may take a share of the units at a time: see make_plan)
    const int groups = smode != 0 ? std::max(1, p.unit_groups) : 1;
    const int per_group = (p.units + groups - 1) / groups;
    for (int u0 = 0; u0 < p.units; u0 += per_group) {
        a.unit0 = u0;
        const dim3 grid(p.n_ch, std::min(per_group, p.units - u0)), block(k.threads);
        void *args[] = {&a};
        hipEvent_t ev_a = nullptr, ev_b = nullptr;
        hipError_t e;
        if (prof_events(KID_REFINE_ATTEND, &ev_a, &ev_b))
            e = hipExtLaunchKernel(reinterpret_cast<const void *>(k.fn), grid, block, args, ra_shmem(p), st, ev_a, ev_b, 0);
        else
            e = hipLaunchKernel(reinterpret_cast<const void *>(k.fn), grid, block, args, ra_shmem(p), st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_attend_dense(const void *q, const void *K, const void *V, void *ws, float *out,
                               const DensePlan &p, const ds_shape_t &s, hipStream_t st)
{
    AttendArgs a{};
    a.q = static_cast<const _Float16 *>(q);
    a.K = static_cast<const _Float16 *>(K);
    a.V = static_cast<const _Float16 *>(V);
    a.part = reinterpret_cast<float *>(wsp(ws, p.off_part));
    a.ctl_rw = reinterpret_cast<UnitCtl *>(wsp(ws, p.off_ctl));
    a.out = out;
    a.Hq = s.Hq; a.Hkv = s.Hkv; a.G = p.G; a.L = s.L; a.L_max = s.L_max;
    a.ch = p.ch; a.n_ch = p.n_ch;
    a.kv_stride = kD;
    launch_attend_mode<1>(KID_DENSE, a, dim3(p.n_ch, p.units), 0, st);
    return hipGetLastError();
}

hipError_t launch_attend_rows(const void *q, const void *KV_rows, void *ws, float *out,
                              const DensePlan &p, const ds_shape_t &s, int n_rows, hipStream_t st)
{
    AttendArgs a{};
    a.q = static_cast<const _Float16 *>(q);
    a.K = static_cast<const _Float16 *>(KV_rows);
    a.V = nullptr;
    a.part = reinterpret_cast<float *>(wsp(ws, p.off_part));
    a.ctl_rw = reinterpret_cast<UnitCtl *>(wsp(ws, p.off_ctl));
    a.out = out;
    a.Hq = s.Hq; a.Hkv = s.Hkv; a.G = p.G; a.L = s.L; a.L_max = s.L_max;
    a.ch = p.ch; a.n_ch = p.n_ch; a.k = s.k; a.n_rows = n_rows;
    launch_attend_mode<2>(KID_ATTEND_ROWS, a, dim3(p.n_ch, p.units), 0, st);
    return hipGetLastError();
}

}  // namespace ds

#ifdef DS_TRACE
extern "C" int ds_trace_read_attend(void *dst, size_t bytes)
{
    return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(ds::g_trace), bytes, 0, hipMemcpyDeviceToHost);
}
#endif

