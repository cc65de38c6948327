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
#include "ds_device.h"

namespace ds {

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
};

__device__ __forceinline__ float dpp_add_xor1(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_add_xor2(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_add_half_mirror(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));
}
__device__ __forceinline__ float dpp_add_mirror(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));
}
// Sum over the 16 lanes of a row; every lane of the row ends with the total.
__device__ __forceinline__ float row16_sum(float v)
{
    v = dpp_add_xor1(v);
    v = dpp_add_xor2(v);
    v = dpp_add_half_mirror(v);
    v = dpp_add_mirror(v);
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
    __shared__ __attribute__((aligned(16))) _Float16 qsh[GT][kD];
    __shared__ __attribute__((aligned(16))) float wpart[4][GT][kPartStride];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slot = lane >> 4, part = lane & 15;
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
        Ku = reinterpret_cast<const char *>(a.K + (size_t)u * a.L_max * kD);
        Vu = reinterpret_cast<const char *>(a.V + (size_t)u * a.L_max * kD);
        row_bytes = 2 * kD;
    }
    const float scale_log2 = 1.4426950408889634f * 0.08838834764831845f;  // log2(e) / sqrt(128)

    for (int g0 = 0; g0 < a.G; g0 += GT) {
        __syncthreads();
        if (tid < GT * 16) {
            const int g = tid >> 4, p = tid & 15;
            const _Float16 *src = a.q + ((size_t)b * a.Hq + (size_t)h * a.G + g0 + g) * kD + p * 8;
            *reinterpret_cast<uint4 *>(&qsh[g][p * 8]) = *reinterpret_cast<const uint4 *>(src);
        }
        __syncthreads();

        float m[GT], l[GT], acc[GT][8];
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            m[g] = kNegInf;
            l[g] = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[g][j] = 0.0f;
        }

        for (int r0 = wave * 16; r0 < n; r0 += 64) {
            // all eight row loads of the pass are issued before the first use; lanes past the
            // end re-read the last row of the list (in bounds) and mask its score below
            half8 kr[4], vr[4];
            bool ok[4];
            uint32_t off[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int want = r0 + i * 4 + slot;
                ok[i] = want < n;
                const int ri = min(want, n - 1);
                const uint32_t row = (MODE == 0) ? (uint32_t)sel[ri] : (MODE == 1) ? (uint32_t)(t0 + ri) : (uint32_t)ri;
                off[i] = row * row_bytes + (uint32_t)part * 16u;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                kr[i] = *reinterpret_cast<const half8 *>(Ku + off[i]);
                vr[i] = *reinterpret_cast<const half8 *>(Vu + off[i]);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the eight loads ahead of the arithmetic
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                const half8 qv = *reinterpret_cast<const half8 *>(&qsh[g][part * 8]);
                float s[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    s[i] = row16_sum(dot8(qv, kr[i])) * scale_log2;
                    if (!ok[i]) s[i] = kNegInf;
                }
                // rows of one slot are taken in order i = 0..3; slot 0 / i = 0 is valid whenever
                // the wave is in this loop, other slots may have no valid row yet
                const float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
                const float mn = fmaxf(m[g], mx);
                if (mn != kNegInf) {
                    const float sc = (m[g] == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(m[g] - mn);
                    m[g] = mn;
                    l[g] *= sc;
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[g][j] *= sc;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float p = __builtin_amdgcn_exp2f(s[i] - mn);  // 2^-inf = 0 for masked rows
                        l[g] += p;
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[g][j] = __builtin_fmaf(p, (float)vr[i][j], acc[g][j]);
                    }
                }
            }
        }

        DS_TR(2);
        // merge the four slots of the wave (fixed order), then the four waves
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            float mm = fmaxf(m[g], __shfl_xor(m[g], 16));
            mm = fmaxf(mm, __shfl_xor(mm, 32));
            const float w = (m[g] == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(m[g] - mm);
            float lv = l[g] * w;
            lv += __shfl_xor(lv, 16);
            lv += __shfl_xor(lv, 32);
            float av[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                av[j] = acc[g][j] * w;
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
        __syncthreads();
        if (tid < kD) {
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float M = kNegInf;
#pragma unroll
                for (int w = 0; w < 4; ++w) M = fmaxf(M, wpart[w][g][0]);
                float A = 0.0f, Ls = 0.0f;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float mw = wpart[w][g][0];
                    const float f = (mw == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(mw - M);
                    A += f * wpart[w][g][4 + tid];
                    Ls += f * wpart[w][g][1];
                }
                float *po = a.part + (((size_t)u * a.G + g0 + g) * a.n_ch + c) * kPartStride;
                st_dev(po + 4 + tid, A);
                if (tid == 0) {
                    st_dev(po + 0, M);
                    st_dev(po + 1, Ls);
                }
            }
        }
    }

    // ---- last workgroup of the unit: combine the chunk partials of every head of the group.
    // The workgroup is cut into 8 groups of 32 threads; a group owns 4 output channels per
    // thread and walks its share of a head's chunks in ascending order with a running
    // (max, denominator, numerator) state; the `gph` groups of a head are then combined in
    // group order.  The schedule depends only on (G, n_ch), never on arrival order.
    DS_TR(3);
    {
        const bool last = last_arrival(&a.ctl_rw[u].arrive_c, gridDim.x, &s_flag);
        DS_TR(4);
        if (!last) return;
    }
    if (tid == 0) a.ctl_rw[u].arrive_c = 0u;
    const int gph = (a.G >= 8) ? 1 : (a.G >= 4) ? 2 : (a.G >= 2) ? 4 : 8;  // groups per head
    const int hpr = 8 / gph;                                               // heads per round
    const int cl = tid >> 5, cg = tid & 31;
    const int hr = cl / gph, sub = cl % gph;
    for (int g0 = 0; g0 < a.G; g0 += hpr) {
        const int g = g0 + hr;
        float m = kNegInf, l = 0.0f;
        float4 A = make_float4(0.f, 0.f, 0.f, 0.f);
        if (g < a.G) {
            const float *ph = a.part + ((size_t)u * a.G + g) * a.n_ch * kPartStride;
            for (int c0 = sub; c0 < a.n_ch; c0 += gph * 4) {
                float2 ml[4];
                float4 v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int cc = c0 + i * gph;
                    if (cc < a.n_ch) {
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
        }
        *reinterpret_cast<float4 *>(&red[cl][cg * 4]) = A;
        if (cg == 0) {
            red_ml[cl][0] = m;
            red_ml[cl][1] = l;
        }
        __syncthreads();
        for (int hh = tid >> 7; hh < hpr; hh += 2) {
            const int g2 = g0 + hh, cc = tid & (kD - 1);
            if (g2 < a.G) {
                float M = kNegInf;
                for (int sgi = 0; sgi < gph; ++sgi) M = fmaxf(M, red_ml[hh * gph + sgi][0]);
                float As = 0.0f, Ls = 0.0f;
                for (int sgi = 0; sgi < gph; ++sgi) {
                    const float ms = red_ml[hh * gph + sgi][0];
                    const float f = (ms == kNegInf) ? 0.0f : __builtin_amdgcn_exp2f(ms - M);
                    As += f * red[hh * gph + sgi][cc];
                    Ls += f * red_ml[hh * gph + sgi][1];
                }
                a.out[((size_t)u * a.G + g2) * kD + cc] = As / Ls;
            }
        }
        __syncthreads();
    }
    DS_TR(5);
}

// ---------------------------------------------------------------- launchers
static inline char *wsp(void *ws, size_t off) { return static_cast<char *>(ws) + off; }

static int pick_gt(int G)
{
    if (G % 8 == 0) return 8;
    if (G % 4 == 0) return 4;
    if (G % 2 == 0) return 2;
    return 1;
}

template <int MODE>
static void launch_attend_mode(const AttendArgs &a, dim3 grid, size_t shmem, hipStream_t st)
{
    switch (pick_gt(a.G)) {
    case 8: hipLaunchKernelGGL((k_attend<8, MODE>), grid, dim3(kWG), shmem, st, a); break;
    case 4: hipLaunchKernelGGL((k_attend<4, MODE>), grid, dim3(kWG), shmem, st, a); break;
    case 2: hipLaunchKernelGGL((k_attend<2, MODE>), grid, dim3(kWG), shmem, st, a); break;
    default: hipLaunchKernelGGL((k_attend<1, MODE>), grid, dim3(kWG), shmem, st, a); break;
    }
}

hipError_t launch_attend_sparse(const void *q, const void *K, const void *V, void *ws, float *out,
                                int32_t *idx_out, const Plan &p, const ds_shape_t &s,
                                hipStream_t st)
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
    prof_begin(KID_ATTEND, st);
    launch_attend_mode<0>(a, dim3(p.n_ch, p.units), (size_t)p.ch * sizeof(int), st);
    prof_end(KID_ATTEND, st);
    return hipGetLastError();
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
    prof_begin(KID_DENSE, st);
    launch_attend_mode<1>(a, dim3(p.n_ch, p.units), 0, st);
    prof_end(KID_DENSE, st);
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
    prof_begin(KID_ATTEND_ROWS, st);
    launch_attend_mode<2>(a, dim3(p.n_ch, p.units), 0, st);
    prof_end(KID_ATTEND_ROWS, st);
    return hipGetLastError();
}

}  // namespace ds

#ifdef DS_TRACE
extern "C" int ds_trace_read_attend(void *dst, size_t bytes)
{
    return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(ds::g_trace), bytes, 0, hipMemcpyDeviceToHost);
}
#endif

