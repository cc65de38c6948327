// Attention building blocks of the attention kernels
// (Algorithm 1 steps 3-5 / Sec. 2.1).
//
// Row processing: a wavefront loads four rows per instruction -- 16 lanes x 16
// bytes cover one 256-byte row -- so each 16-lane group ("slot") owns a row at
// a time and keeps its own online-softmax state (running max m, denominator l,
// 8 output channels per lane).  Logits live in the log2 domain:
// s2 = (q.k) * log2(e)/sqrt(d), p = 2^(s2 - m).
// Every reduction runs in an order fixed by the launch shape, so results are
// bit-reproducible.
#pragma once

#include <type_traits>

#include "ds_device.h"

namespace ds {

constexpr float kScaleLog2 = 1.4426950408889634f * 0.08838834764831845f;  // log2(e) / sqrt(128)

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// Sum over the 16 lanes of a row; every lane of the row ends with the total.
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);  // row_half_mirror
    v += dpp_move<0x140>(v);  // row_mirror
    return v;
}

__device__ __forceinline__ float dot8(half8 a, half8 b)
{
    float acc = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        half2v x = {a[2 * i], a[2 * i + 1]};
        half2v y = {b[2 * i], b[2 * i + 1]};
        acc = __builtin_amdgcn_fdot2(x, y, acc, false);
    }
    return acc;
}

template <int GT>
struct RowState {
    float m[GT], l[GT], acc[GT][8];
    __device__ __forceinline__ void init()
    {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            m[g] = kNegInf;
            l[g] = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[g][j] = 0.0f;
        }
    }
};

// A 16-byte piece of a K or V row: read once per call, gathered or front to back, so the load is
// marked as streaming (measured: dense decode 191 -> 176 us on the 64K workload, the gathers of the
// sparse path 0.7 to 2.5 us per layer).
template <bool ST = true>
__device__ __forceinline__ half8 row_load(const half8 *p)
{
    if constexpr (ST) return __builtin_nontemporal_load(p);
    else return *p;
}

// The calling wavefront's share of the workgroup's n rows: with RPS rows per 16-lane slot in
// flight, rows wave*4*RPS + NW*4*RPS*i ..  (NW wavefronts; RPS = 4: 64 rows of a 256-thread
// workgroup per round trip and 8 loads per lane; larger RPS for a workgroup that has a CU to itself).
// row_of(ri) gives the row number of list entry ri; a row's K (V) bytes start at
// Ku (Vu) + row * row_bytes.  qsh holds the GT query rows in LDS.
template <int GT, int RPS = 4, int NW = 4, bool ST = true, class RowOf>
__device__ __forceinline__ void attend_rows(const char *Ku, const char *Vu, uint32_t row_bytes, int n,
                                            RowOf row_of, const _Float16 (*qsh)[kD], RowState<GT> &st)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int slot = lane >> 4, part = lane & 15;
    if constexpr (NW > 4) {
        // A workgroup with a CU to itself has nobody else to cover its memory latency, so the
        // RPS rows of a slot travel in two halves, the loads of one
        // issued before the other is folded in.  Rows reach a slot's state in the same order and
        // the same groups of four as in the plain loop below.
        constexpr int HB = RPS / 2;
        const int base = wave * 4 * RPS;
        if (base >= n) return;
        half8 k0[HB], v0[HB], k1[HB], v1[HB];
        // first row of the wavefront's h-th half
        auto first_row = [&](int h) { return base + (h >> 1) * 4 * NW * RPS + (h & 1) * 4 * HB; };
        auto issue = [&](half8 (&kr)[HB], half8 (&vr)[HB], int rr) {
#pragma unroll
            for (int i = 0; i < HB; ++i) {
                const uint32_t off = (uint32_t)row_of(min(rr + i * 4 + slot, n - 1)) * row_bytes + (uint32_t)part * 16u;
                kr[i] = row_load<ST>(reinterpret_cast<const half8 *>(Ku + off));
                vr[i] = row_load<ST>(reinterpret_cast<const half8 *>(Vu + off));
            }
        };
        auto fold = [&](half8 (&kr)[HB], half8 (&vr)[HB], int rr) {
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                const half8 qv = *reinterpret_cast<const half8 *>(&qsh[g][part * 8]);
#pragma unroll
                for (int i0 = 0; i0 < HB; i0 += 4) {
                    float s[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        s[i] = row16_sum(dot8(qv, kr[i0 + i])) * kScaleLog2;
                        if (rr + (i0 + i) * 4 + slot >= n) s[i] = kNegInf;
                    }
                    const float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
                    const float mn = fmaxf(st.m[g], mx);
                    if (mn != kNegInf) {
                        const float sc = (st.m[g] == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(st.m[g] - mn);
                        st.m[g] = mn;
                        st.l[g] *= sc;
#pragma unroll
                        for (int j = 0; j < 8; ++j) st.acc[g][j] *= sc;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float p = __builtin_amdgcn_exp2f(s[i] - mn);
                            st.l[g] += p;
#pragma unroll
                            for (int j = 0; j < 8; ++j)
                                st.acc[g][j] = __builtin_fmaf(p, (float)vr[i0 + i][j], st.acc[g][j]);
                        }
                    }
                }
            }
        };
        issue(k0, v0, first_row(0));
        for (int h = 0; first_row(h) < n; h += 2) {
            issue(k1, v1, first_row(h + 1));
            __builtin_amdgcn_sched_barrier(0);
            fold(k0, v0, first_row(h));
            issue(k0, v0, first_row(h + 2));
            __builtin_amdgcn_sched_barrier(0);
            if (first_row(h + 1) < n) fold(k1, v1, first_row(h + 1));
        }
        return;
    }
    for (int r0 = wave * 4 * RPS; r0 < n; r0 += 16 * RPS) {
        // all row loads of the pass are issued before the first use; lanes past the
        // end re-read the last row of the list (in bounds) and mask its score below
        half8 kr[RPS], vr[RPS];
        bool ok[RPS];
        uint32_t off[RPS];
#pragma unroll
        for (int i = 0; i < RPS; ++i) {
            const int want = r0 + i * 4 + slot;
            ok[i] = want < n;
            off[i] = (uint32_t)row_of(min(want, n - 1)) * row_bytes + (uint32_t)part * 16u;
        }
#pragma unroll
        for (int i = 0; i < RPS; ++i) {
            kr[i] = row_load<ST>(reinterpret_cast<const half8 *>(Ku + off[i]));
            vr[i] = row_load<ST>(reinterpret_cast<const half8 *>(Vu + off[i]));
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the loads ahead of the arithmetic
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const half8 qv = *reinterpret_cast<const half8 *>(&qsh[g][part * 8]);
            // the rows of a slot are folded into its state four at a time (the last group may be
            // smaller), in row order
            auto fold_group = [&](auto i0c, auto fgc) {
                constexpr int i0 = decltype(i0c)::value, FG = decltype(fgc)::value;
                float s[FG];
                float mx = kNegInf;
#pragma unroll
                for (int i = 0; i < FG; ++i) {
                    s[i] = row16_sum(dot8(qv, kr[i0 + i])) * kScaleLog2;
                    if (!ok[i0 + i]) s[i] = kNegInf;
                    mx = fmaxf(mx, s[i]);
                }
                // a slot may have no valid row yet (m stays -inf); slot 0 always has one here
                const float mn = fmaxf(st.m[g], mx);
                if (mn != kNegInf) {
                    const float sc = (st.m[g] == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(st.m[g] - mn);
                    st.m[g] = mn;
                    st.l[g] *= sc;
#pragma unroll
                    for (int j = 0; j < 8; ++j) st.acc[g][j] *= sc;
#pragma unroll
                    for (int i = 0; i < FG; ++i) {
                        const float p = __builtin_amdgcn_exp2f(s[i] - mn);  // 2^-inf = 0 for masked rows
                        st.l[g] += p;
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            st.acc[g][j] = __builtin_fmaf(p, (float)vr[i0 + i][j], st.acc[g][j]);
                    }
                }
            };
            if constexpr (RPS >= 4) fold_group(std::integral_constant<int, 0>{}, std::integral_constant<int, 4>{});
            if constexpr (RPS >= 8) fold_group(std::integral_constant<int, 4>{}, std::integral_constant<int, 4>{});
            if constexpr (RPS % 4 != 0)
                fold_group(std::integral_constant<int, RPS / 4 * 4>{}, std::integral_constant<int, RPS % 4>{});
        }
    }
}

// Second half of a workgroup's partial: the four wavefronts' states in
// wpart[wave][head] = {m, l, -, -, acc[128]} (LDS) are merged in wave order and
// written as one partial per head to po + g * head_stride with device-scope
// stores.  With out_direct (a unit that has this one workgroup only) the final
// result acc / l goes to out_direct + g * kD instead; that is what merging the
// single partial would give, bit for bit.
// Starts with a barrier; callers put a barrier between two uses of wpart.
template <int GH, int NW = 4>
__device__ __forceinline__ void wg_combine_store(float (*wpart)[GH][kPartStride], int n_heads, float *po,
                                                 size_t head_stride, float *out_direct = nullptr)
{
    const int tid = threadIdx.x;
    __syncthreads();
    if (tid < kD) {
#pragma unroll
        for (int g = 0; g < GH; ++g) {
            if (g < n_heads) {
                float M = kNegInf;
#pragma unroll
                for (int w = 0; w < NW; ++w) M = fmaxf(M, wpart[w][g][0]);
                float A = 0.0f, Ls = 0.0f;
#pragma unroll
                for (int w = 0; w < NW; ++w) {
                    const float mw = wpart[w][g][0];
                    const float f = (mw == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(mw - M);
                    A += f * wpart[w][g][4 + tid];
                    Ls += f * wpart[w][g][1];
                }
                if (out_direct) {
                    out_direct[(size_t)g * kD + tid] = A / Ls;
                } else {
                    float *pg = po + (size_t)g * head_stride;
                    st_dev(pg + 4 + tid, A);
                    if (tid == 0) {
                        st_dev(pg + 0, M);
                        st_dev(pg + 1, Ls);
                    }
                }
            }
        }
    }
}

// Merges the 16 slot states of the workgroup (4 slots per wave in slot order,
// then the 4 waves in wave order) and writes one partial per head.
template <int GT, int NW = 4>
__device__ __forceinline__ void wg_store_partial(const RowState<GT> &st,
                                                 float (*wpart)[GT][kPartStride], float *po,
                                                 size_t head_stride, float *out_direct = nullptr)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int slot = lane >> 4, part = lane & 15;
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        float mm = fmaxf(st.m[g], __shfl_xor(st.m[g], 16));
        mm = fmaxf(mm, __shfl_xor(mm, 32));
        const float w = (st.m[g] == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(st.m[g] - mm);
        float lv = st.l[g] * w;
        lv += __shfl_xor(lv, 16);
        lv += __shfl_xor(lv, 32);
        float av[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            av[j] = st.acc[g][j] * w;
            av[j] += __shfl_xor(av[j], 16);
            av[j] += __shfl_xor(av[j], 32);
        }
        if (slot == 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) wpart[wave][g][4 + part * 8 + j] = av[j];
            if (part == 0) {
                wpart[wave][g][0] = mm;
                wpart[wave][g][1] = lv;
            }
        }
    }
    wg_combine_store<GT, NW>(wpart, GT, po, head_stride, out_direct);
}

// ---------------------------------------------------------------- matrix-core path for query groups
// When several query heads share a KV head, scores and P.V are small dense
// contractions over the gathered rows: S[token][head] = K[token,:] . q[head,:]
// (16 tokens x up to 16 heads x 128 channels, fp16 MFMA 16x16x32, four issues) and
// O[head][channel] += P[token][head] * V[token][channel] (fp16 MFMA 16x16x16 with
// fp32 accumulation: V as stored, each weight as the sum of two fp16 numbers, which
// carries it to about 22 bits).  A wavefront owns tiles of 16 rows.
//
// Lane roles (l = lane, lo = l % 16, hi = l / 16):
//   K operand   : token lo of the tile, 16-byte pieces at channels 8*(4x + hi), x = 0..3
//   q operand   : head lo, the same channel pieces (loaded once per item)
//   S result    : head lo, tokens 4*hi + r, r = 0..3   -> softmax state per lane for head lo
//   V operand   : token 4*hi + r, channels 8*lo .. 8*lo+7 (the whole 256-byte row per 16 lanes)
//   O result e  : heads 4*hi + rr, channel 8*lo + e     (8 accumulators of 4 values)
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

// Softmax weights on the matrix-core path carry this factor, numerators and denominators alike (it
// cancels in every quotient and every merge): 2^14, so that the low half of a weight's two-part
// fp16 form is a normal number down to weights of 2^-17 of the largest.
constexpr float kPScaleLog2 = 14.0f;

struct MfmaState {
    float m, l;       // running max / partial denominator (times 2^kPScaleLog2) of head lo over this lane's tokens
    float4v O[8];     // O[e][rr]: head 4*hi + rr, channel 8*lo + e
    __device__ __forceinline__ void init()
    {
        m = kNegInf;
        l = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) O[e] = (float4v){0.f, 0.f, 0.f, 0.f};
    }
};

// q rows of the heads [g0, g0 + 16) of a unit as MFMA operands (zeros beyond n_heads).
__device__ __forceinline__ void load_q_mfma(const _Float16 *q_unit, int n_heads, half8 (&qreg)[4])
{
    const int lane = threadIdx.x & 63, lo = lane & 15, hi = lane >> 4;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        qreg[x] = (half8)(_Float16)0;
        if (lo < n_heads) qreg[x] = *reinterpret_cast<const half8 *>(q_unit + (size_t)lo * kD + 8 * (4 * x + hi));
    }
}

// sc_lds: 16 floats of LDS private to the calling wavefront.
// KST: whether the K loads carry the streaming mark.  A K load takes 64 bytes of each of 16 rows,
// so two loads in a row share every 128-byte line; when the rows are gathered, the second finds
// the line more cheaply after an ordinary load (measured on the two query-group workloads:
// -1.2 and -1.0 us per layer; the V loads, whole rows, do better with the mark: +1 us without).
template <bool KST = true, class RowOf>
__device__ __forceinline__ void attend_rows_mfma(const char *Ku, const char *Vu, uint32_t row_bytes, int n,
                                                 RowOf row_of, const half8 (&qreg)[4], MfmaState &st,
                                                 float *sc_lds)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lo = lane & 15, hi = lane >> 4;
    // The K pieces of a tile are dead once its scores are formed, the V pieces once they are
    // folded in: the next tile's K loads are issued right after the scores and its V loads right
    // after the fold, into the same registers, so that a wavefront has loads in flight while it
    // computes.  Rows past the end re-read the last row of the list (in bounds) and their scores
    // are masked.
    half8 kr[4], vr[4];
    auto issue_k = [&](int r0) {
        const uint32_t krow = (uint32_t)row_of(min(r0 + lo, n - 1)) * row_bytes;
#pragma unroll
        for (int x = 0; x < 4; ++x)
            kr[x] = row_load<KST>(reinterpret_cast<const half8 *>(Ku + krow + 16u * (uint32_t)(4 * x + hi)));
    };
    auto issue_v = [&](int r0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t vrow = (uint32_t)row_of(min(r0 + 4 * hi + r, n - 1)) * row_bytes;
            vr[r] = row_load(reinterpret_cast<const half8 *>(Vu + vrow + 16u * (uint32_t)lo));
        }
    };
    if (wave * 16 >= n) return;
    issue_k(wave * 16);
    issue_v(wave * 16);
    for (int r0 = wave * 16; r0 < n; r0 += 64) {
        const bool more = r0 + 64 < n;
        __builtin_amdgcn_sched_barrier(0);
        float4v S = (float4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int x = 0; x < 4; ++x) S = __builtin_amdgcn_mfma_f32_16x16x32_f16(kr[x], qreg[x], S, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (more) issue_k(r0 + 64);
        __builtin_amdgcn_sched_barrier(0);
        float s[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) s[r] = (r0 + 4 * hi + r < n) ? S[r] * kScaleLog2 : kNegInf;
        float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));  // over the 16 tokens of the tile, per head (token r0 is valid)
        const float mn = fmaxf(st.m, mx);
        const float sc = (st.m == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(st.m - mn);
        st.m = mn;
        float p[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) p[r] = __builtin_amdgcn_exp2f(s[r] - mn + kPScaleLog2);  // (masked rows: 2^-inf = 0)
        st.l = st.l * sc + ((p[0] + p[1]) + (p[2] + p[3]));
        if (__any(sc != 1.0f)) {
            // the accumulators of heads 4*hi .. 4*hi+3 live in this lane; their scale factors sit in
            // lanes 4*hi .. 4*hi+3 of the wavefront: pass them through the wavefront's LDS words
            if (hi == 0) sc_lds[lo] = sc;
            const float4v f = *reinterpret_cast<const float4v *>(sc_lds + 4 * hi);
#pragma unroll
            for (int e = 0; e < 8; ++e) st.O[e] *= f;
        }
        // P.V on the fp16 matrix cores with fp32 accumulation: V is fp16 as stored; a weight goes
        // in as the sum of two fp16 numbers, hi = fp16(p) and lo = fp16(p - hi), which carries it to
        // about 22 bits (the weights are scaled by kPScale beforehand, see above, so that lo stays a
        // normal fp16 number for every weight that matters).  16 short issues per tile against 32
        // long ones with weights and V widened to fp32 (measured: C4a 52.0 -> 49.5 us/layer).
        half4v p_hi, p_lo;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p_hi[r] = (_Float16)p[r];
            p_lo[r] = (_Float16)(p[r] - (float)p_hi[r]);
        }
        // (the eight high parts first, then the eight low parts: two issues in a row into the
        //  same accumulator would wait for each other)
        half4v vb[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vb[e] = (half4v){vr[0][e], vr[1][e], vr[2][e], vr[3][e]};
#pragma unroll
        for (int e = 0; e < 8; ++e) st.O[e] = __builtin_amdgcn_mfma_f32_16x16x16f16(p_hi, vb[e], st.O[e], 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 8; ++e) st.O[e] = __builtin_amdgcn_mfma_f32_16x16x16f16(p_lo, vb[e], st.O[e], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (more) issue_v(r0 + 64);
    }
}

// Writes the calling wavefront's state to wpart[wave][head] and runs the workgroup combine.
template <int GH>
__device__ __forceinline__ void wg_store_partial_mfma(const MfmaState &st, float (*wpart)[GH][kPartStride],
                                                      int n_heads, float *po, size_t head_stride,
                                                      float *out_direct = nullptr)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lo = lane & 15, hi = lane >> 4;
    float lv = st.l;
    lv += __shfl_xor(lv, 16);
    lv += __shfl_xor(lv, 32);
    if (hi == 0 && lo < n_heads) {
        wpart[wave][lo][0] = st.m;
        wpart[wave][lo][1] = lv;
    }
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int head = 4 * hi + rr;
        if (head < n_heads) {
#pragma unroll
            for (int e = 0; e < 8; ++e) wpart[wave][head][4 + 8 * lo + e] = st.O[e][rr];
        }
    }
    wg_combine_store<GH>(wpart, n_heads, po, head_stride, out_direct);
}

// Combines the n_ch chunk partials of each of the G heads of one unit:
//   y = sum_c acc_c 2^(m_c - M) / sum_c l_c 2^(m_c - M),  M = max_c m_c.
// The workgroup is cut into 8 groups of 32 threads; a group owns 4 output
// channels per thread and walks its share of a head's chunks in ascending
// order with a running (max, denominator, numerator) state; the groups of a
// head are then combined in group order.  The schedule depends only on
// (G, n_ch).  wait_chunk(cc, active) is called by every lane of a group before
// the group reads chunk cc (a no-op when all partials are already complete).
// red: LDS [8][kD], red_ml: LDS [8][2].  All 256 threads must call it.
template <class Wait>
__device__ __forceinline__ void merge_partials(const float *part_unit, int G, int n_ch, float *out_unit,
                                               float (*red)[kD], float (*red_ml)[2], Wait wait_chunk)
{
    const int tid = threadIdx.x;
    const int gph = (G >= 8) ? 1 : (G >= 4) ? 2 : (G >= 2) ? 4 : 8;  // groups per head
    const int hpr = 8 / gph;                                          // heads per round
    const int cl = tid >> 5, cg = tid & 31;
    const int hr = cl / gph, sub = cl % gph;
    for (int g0 = 0; g0 < G; g0 += hpr) {
        const int g = g0 + hr;
        float m = kNegInf, l = 0.0f;
        float4 A = make_float4(0.f, 0.f, 0.f, 0.f);
        const bool active = g < G;
        const float *ph = part_unit + (size_t)(active ? g : 0) * n_ch * kPartStride;
        // every group runs the same number of batches so that wait_chunk stays wave-uniform
        for (int c0 = sub; c0 - sub < n_ch; c0 += gph * 4) {
            float2 ml[4];
            float4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int cc = c0 + i * gph;
                const bool have = active && cc < n_ch;
                wait_chunk(cc, have);
                if (have) {
                    const float *pc = ph + (size_t)cc * kPartStride;
                    ml[i] = ld_dev(reinterpret_cast<const float2 *>(pc));
                    const float2 lo = ld_dev(reinterpret_cast<const float2 *>(pc + 4 + cg * 4));
                    const float2 hi = ld_dev(reinterpret_cast<const float2 *>(pc + 6 + cg * 4));
                    v[i] = make_float4(lo.x, lo.y, hi.x, hi.y);
                } else {
                    ml[i] = make_float2(kNegInf, 0.f);
                    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (ml[i].x != kNegInf) {
                    const float mn = fmaxf(m, ml[i].x);
                    const float so = (m == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(m - mn);
                    const float sn = __builtin_amdgcn_exp2f(ml[i].x - mn);
                    l = l * so + ml[i].y * sn;
                    A.x = A.x * so + v[i].x * sn;
                    A.y = A.y * so + v[i].y * sn;
                    A.z = A.z * so + v[i].z * sn;
                    A.w = A.w * so + v[i].w * sn;
                    m = mn;
                }
            }
        }
        *reinterpret_cast<float4 *>(&red[cl][cg * 4]) = A;
        if (cg == 0) {
            red_ml[cl][0] = m;
            red_ml[cl][1] = l;
        }
        __syncthreads();
        for (int hh = tid >> 7; hh < hpr; hh += 2) {
            const int g2 = g0 + hh, cc = tid & (kD - 1);
            if (g2 < G) {
                float M = kNegInf;
                for (int sgi = 0; sgi < gph; ++sgi) M = fmaxf(M, red_ml[hh * gph + sgi][0]);
                float As = 0.0f, Ls = 0.0f;
                for (int sgi = 0; sgi < gph; ++sgi) {
                    const float ms = red_ml[hh * gph + sgi][0];
                    const float f = (ms == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(ms - M);
                    As += f * red[hh * gph + sgi][cc];
                    Ls += f * red_ml[hh * gph + sgi][1];
                }
                out_unit[(size_t)g2 * kD + cc] = As / Ls;
            }
        }
        __syncthreads();
    }
}

}  // namespace ds
