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
#include "ds_attend_core.h"

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
        Ku = reinterpret_cast<const char *>(a.K + (size_t)u * a.L_max * kD);
        Vu = reinterpret_cast<const char *>(a.V + (size_t)u * a.L_max * kD);
        row_bytes = 2 * kD;
    }

    auto row_of = [&](int ri) { return (MODE == 0) ? sel[ri] : (MODE == 1) ? (t0 + ri) : ri; };
    for (int g0 = 0; g0 < a.G; g0 += GT) {
        float *po = a.part + (((size_t)u * a.G + g0) * a.n_ch + c) * kPartStride;
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
            wg_store_partial_mfma<GT>(st, wpart, n_heads, po, (size_t)a.n_ch * kPartStride);
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
            wg_store_partial<GT>(st, wpart, po, (size_t)a.n_ch * kPartStride);
        }
    }

    // ---- last workgroup of the unit: combine the chunk partials of every head of the group
    DS_TR(3);
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
static void launch_attend_mode(const AttendArgs &a, dim3 grid, size_t shmem, hipStream_t st)
{
    switch (pick_gt(a.G)) {
    case 16: hipLaunchKernelGGL((k_attend<16, MODE>), grid, dim3(kWG), shmem, st, a); break;
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

