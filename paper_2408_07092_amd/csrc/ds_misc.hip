// Label-cache maintenance (Sec. 4.2), the host-row gather of the offload
// arrangement (Sec. 5.1) and the read-bandwidth probe.
#include <algorithm>

#include "ds_device.h"

namespace ds {

// label[u, t, j] = K[u, t, channels[h, j]] for t in [t0, t0 + n): a bit copy.
// One thread per label element; writes are contiguous, reads pick 2-byte
// elements out of the 256-byte K rows (kv_stride halves apart: d, or 2d when
// each K row is followed by the token's V row).
__global__ __launch_bounds__(kWG) void k_label(const uint16_t *__restrict__ K,
                                               const int32_t *__restrict__ channels,
                                               uint16_t *__restrict__ label, int Hkv, int L_max,
                                               int r, int t0, int n, int kv_stride)
{
    __shared__ int ch_sh[kD];
    const int u = blockIdx.y, h = u % Hkv;
    if (threadIdx.x < r) ch_sh[threadIdx.x] = channels[h * r + threadIdx.x];
    __syncthreads();
    const size_t total = (size_t)n * r;
    const size_t stride = (size_t)gridDim.x * kWG;
    for (size_t e = (size_t)blockIdx.x * kWG + threadIdx.x; e < total; e += stride) {
        const size_t t = t0 + e / r;
        const int j = (int)(e % r);
        const size_t row = (size_t)u * L_max + t;
        label[row * r + j] = K[row * kv_stride + ch_sh[j]];
    }
}

// Decode-step cache maintenance in one launch (Sec. 4.2: a decode step extends the label cache
// by the new tokens' r selected channels only): the n new tokens' K and V rows go into
// the caches at tokens [t0, t0 + n) and their r label values into the label cache.
// 16 lanes move one 256-byte row; the label values are picked out of the new rows afterwards.
__global__ __launch_bounds__(kWG) void k_append_kv(const uint4 *__restrict__ k_new,
                                                   const uint4 *__restrict__ v_new, uint4 *K, uint4 *V,
                                                   const int32_t *__restrict__ channels,
                                                   uint16_t *__restrict__ label, int Hkv, int L_max,
                                                   int r, int t0, int n, int kv_stride16)
{
    __shared__ int ch_sh[kD];
    const int u = blockIdx.y, h = u % Hkv;
    if (threadIdx.x < r) ch_sh[threadIdx.x] = channels[h * r + threadIdx.x];
    __syncthreads();
    const int p = threadIdx.x & 15;
    for (int i = blockIdx.x * 16 + (threadIdx.x >> 4); i < n; i += gridDim.x * 16) {
        const size_t src = ((size_t)u * n + i) * 16 + p;
        const size_t dst = ((size_t)u * L_max + t0 + i) * kv_stride16 + p;
        K[dst] = k_new[src];
        V[dst] = v_new[src];
    }
    const uint16_t *kn = reinterpret_cast<const uint16_t *>(k_new);
    const size_t total = (size_t)n * r;
    for (size_t e = (size_t)blockIdx.x * kWG + threadIdx.x; e < total; e += (size_t)gridDim.x * kWG) {
        const size_t i = e / r;
        const int j = (int)(e % r);
        label[((size_t)u * L_max + t0 + i) * r + j] = kn[((size_t)u * n + i) * kD + ch_sh[j]];
    }
}

// ---------------------------------------------------------------- 4-bit label cache (Sec. 4.2)
// The paper says only that the label cache can be kept in 4 bits.  Quantiser used here:
// symmetric, one step per (unit, label channel), fixed at build time:
//   amax[u, j] = max_t |K[u, t, C[j]]|,  code = clamp(rint(x * (7 / amax)), -8, 7),
//   label value = code * (amax / 7); eight two's-complement nibbles per 32-bit word,
//   channel j of a token in bits [4 (j mod 8), +4) of the token's word j / 8.
// k_q4_amax: non-negative binary32 values order like their bit patterns, so the maximum is an
// integer atomicMax (exact, order-free).  amax must be zero on entry.
__global__ __launch_bounds__(kWG) void k_q4_zero(uint32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * kWG + threadIdx.x; i < n; i += (size_t)gridDim.x * kWG) p[i] = 0u;
}

__global__ __launch_bounds__(kWG) void k_q4_amax(const _Float16 *__restrict__ K,
                                                 const int32_t *__restrict__ channels,
                                                 uint32_t *amax_bits, int Hkv, int L_max, int r, int n)
{
    __shared__ int ch_sh[kD];
    __shared__ uint32_t mx_sh[kD];
    const int u = blockIdx.y, h = u % Hkv;
    if (threadIdx.x < kD) {
        mx_sh[threadIdx.x] = 0u;
        if (threadIdx.x < r) ch_sh[threadIdx.x] = channels[h * r + threadIdx.x];
    }
    __syncthreads();
    const size_t total = (size_t)n * r;
    for (size_t e = (size_t)blockIdx.x * kWG + threadIdx.x; e < total; e += (size_t)gridDim.x * kWG) {
        const size_t t = e / r;
        const int j = (int)(e % r);
        const float x = __builtin_fabsf((float)K[((size_t)u * L_max + t) * kD + ch_sh[j]]);
        atomicMax(&mx_sh[j], __float_as_uint(x));
    }
    __syncthreads();
    if (threadIdx.x < r && mx_sh[threadIdx.x]) atomicMax(&amax_bits[(size_t)u * r + threadIdx.x], mx_sh[threadIdx.x]);
}

// One thread per (token, word): up to eight codes packed into the word.
__global__ __launch_bounds__(kWG) void k_q4_write(const _Float16 *__restrict__ K,
                                                  const int32_t *__restrict__ channels,
                                                  const float *__restrict__ amax,
                                                  uint32_t *__restrict__ codes, int Hkv, int L_max,
                                                  int r, int t0, int n)
{
    __shared__ int ch_sh[kD];
    __shared__ float inv_sh[kD];
    const int u = blockIdx.y, h = u % Hkv;
    if (threadIdx.x < r) {
        ch_sh[threadIdx.x] = channels[h * r + threadIdx.x];
        const float a = amax[(size_t)u * r + threadIdx.x];
        inv_sh[threadIdx.x] = a > 0.0f ? 7.0f / a : 0.0f;
    }
    __syncthreads();
    const int W = (r + 7) / 8;
    const size_t total = (size_t)n * W;
    for (size_t e = (size_t)blockIdx.x * kWG + threadIdx.x; e < total; e += (size_t)gridDim.x * kWG) {
        const size_t row = (size_t)u * L_max + t0 + e / W;
        const int w = (int)(e % W);
        uint32_t word = 0u;
        for (int i = 0; i < 8 && w * 8 + i < r; ++i) {
            const int j = w * 8 + i;
            const float y = __builtin_rintf((float)K[row * kD + ch_sh[j]] * inv_sh[j]);
            const int c = y < -8.0f ? -8 : (y > 7.0f ? 7 : (int)y);
            word |= ((uint32_t)c & 0xfu) << (4 * i);
        }
        codes[row * W + w] = word;
    }
}

// ---------------------------------------------------------------- next-layer query prediction (Sec. 5.1)
// q_out[b, n] = sum_m Wq[n, m] * x[b, m], the shape of the step that turns a layer's input
// embedding into an approximate query of the NEXT layer so that its rows can be fetched early.
// Bound by the one read of Wq.  A wavefront owns an output feature n at a time: its 64 lanes
// split m in 16-byte pieces, products are exact (fp16 x fp16) and accumulated in binary32, the
// lanes are summed in a fixed butterfly, the result is rounded once to fp16.  Up to four batch
// rows share a pass over Wq (x sits in LDS); larger batches take several passes.
constexpr int kPredBatch = 4;

__global__ __launch_bounds__(kWG) void k_predict_query(const _Float16 *__restrict__ x,
                                                       const _Float16 *__restrict__ Wq,
                                                       _Float16 *__restrict__ q_out, int B, int Dm,
                                                       int N, int rows_per_wg)
{
    extern __shared__ __attribute__((aligned(16))) _Float16 x_sh[];  // [min(B, kPredBatch)][Dm]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_lo = blockIdx.x * rows_per_wg, n_hi = min(N, n_lo + rows_per_wg);
    for (int b0 = 0; b0 < B; b0 += kPredBatch) {
        const int nb = min(kPredBatch, B - b0);
        __syncthreads();
        for (int i = tid * 8; i < nb * Dm; i += kWG * 8)
            *reinterpret_cast<uint4 *>(x_sh + i) = *reinterpret_cast<const uint4 *>(x + (size_t)b0 * Dm + i);
        __syncthreads();
        for (int n = n_lo + wave; n < n_hi; n += 4) {
            const _Float16 *wrow = Wq + (size_t)n * Dm;
            float acc[kPredBatch] = {0.0f, 0.0f, 0.0f, 0.0f};
            for (int m = lane * 8; m < Dm; m += 64 * 8) {
                const half8 wv = *reinterpret_cast<const half8 *>(wrow + m);
#pragma unroll
                for (int b = 0; b < kPredBatch; ++b) {
                    if (b < nb) {
                        const half8 xv = *reinterpret_cast<const half8 *>(x_sh + b * Dm + m);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const half2v a2 = {wv[2 * e], wv[2 * e + 1]};
                            const half2v b2 = {xv[2 * e], xv[2 * e + 1]};
                            acc[b] = __builtin_amdgcn_fdot2(a2, b2, acc[b], false);
                        }
                    }
                }
            }
#pragma unroll
            for (int b = 0; b < kPredBatch; ++b) {
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) acc[b] += __shfl_xor(acc[b], o);
                if (lane == 0 && b < nb) q_out[(size_t)(b0 + b) * N + n] = (_Float16)acc[b];
            }
        }
    }
}

// rows[u, i, 0, :] = K_host[u, idx[u, i], :], rows[u, i, 1, :] = V_host[...]:
// 16 lanes move one 256-byte row; K_host / V_host are pinned host memory read
// over the host link by the kernel itself.
__global__ __launch_bounds__(kWG) void k_gather_host(const uint4 *__restrict__ Kh,
                                                     const uint4 *__restrict__ Vh,
                                                     const int32_t *__restrict__ idx,
                                                     uint4 *__restrict__ rows, int L_max, int k)
{
    const int u = blockIdx.y;
    const int i = blockIdx.x * 16 + (threadIdx.x >> 4), p = threadIdx.x & 15;
    if (i >= k) return;
    const int tok = idx[(size_t)u * k + i];
    uint4 kv = make_uint4(0, 0, 0, 0), vv = kv;
    if (tok >= 0) {
        const size_t src = ((size_t)u * L_max + tok) * 16 + p;
        kv = Kh[src];
        vv = Vh[src];
    }
    const size_t dst = ((size_t)u * k + i) * 32 + p;
    rows[dst] = kv;
    rows[dst + 16] = vv;
}

// Plain streaming read: every workgroup reads 64 KiB as 16-byte loads marked as streaming (the
// mark is worth about 10 % on reads far larger than the caches), sixteen per thread in flight
// (eight leave about 8 % of the rate on the table).
constexpr int kProbeLoads = 16;
__global__ __launch_bounds__(kWG) void k_probe(const uint4 *__restrict__ src, size_t n16,
                                               uint32_t *sink)
{
    const size_t base = (size_t)blockIdx.x * (kWG * kProbeLoads) + threadIdx.x;
    uint4 v[kProbeLoads];
#pragma unroll
    for (int i = 0; i < kProbeLoads; ++i) {
        const size_t e = base + (size_t)i * kWG;
        v[i] = (e < n16) ? stream_load(src + e) : make_uint4(0, 0, 0, 0);
    }
    uint32_t x = 0;
#pragma unroll
    for (int i = 0; i < kProbeLoads; ++i) x ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o);
    if ((threadIdx.x & 63) == 0 && x != 0x9e3779b9u) atomicXor(&sink[blockIdx.x & 1023], x);
}

hipError_t launch_label(const void *K, const int32_t *channels, void *label, const ds_shape_t &s,
                        int t0, int n, hipStream_t st, int kv_stride)
{
    if (n <= 0) return hipSuccess;
    const size_t total = (size_t)n * s.r;
    size_t blocks = (total + kWG - 1) / kWG;
    if (blocks > 4096) blocks = 4096;
    DS_LAUNCH(KID_LABEL, k_label, dim3((unsigned)blocks, s.B * s.Hkv), dim3(kWG), 0, st,
                       static_cast<const uint16_t *>(K), channels, static_cast<uint16_t *>(label),
                       s.Hkv, s.L_max, s.r, t0, n, kv_stride);
    return hipGetLastError();
}

hipError_t launch_q4_amax(const void *K, const int32_t *channels, float *amax, const ds_shape_t &s,
                          hipStream_t st)
{
    const size_t n_amax = (size_t)s.B * s.Hkv * s.r;
    hipLaunchKernelGGL(k_q4_zero, dim3((unsigned)std::min<size_t>((n_amax + kWG - 1) / kWG, 1024)), dim3(kWG),
                       0, st, reinterpret_cast<uint32_t *>(amax), n_amax);
    const size_t total = (size_t)s.L * s.r;
    size_t blocks = (total + kWG * 8 - 1) / (kWG * 8);
    if (blocks > 1024) blocks = 1024;
    DS_LAUNCH(KID_Q4_AMAX, k_q4_amax, dim3((unsigned)blocks, s.B * s.Hkv), dim3(kWG), 0, st,
              static_cast<const _Float16 *>(K), channels, reinterpret_cast<uint32_t *>(amax), s.Hkv,
              s.L_max, s.r, s.L);
    return hipGetLastError();
}

hipError_t launch_q4_write(const void *K, const int32_t *channels, const float *amax, void *codes,
                           const ds_shape_t &s, int t0, int n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    const size_t total = (size_t)n * ((s.r + 7) / 8);
    size_t blocks = (total + kWG - 1) / kWG;
    if (blocks > 4096) blocks = 4096;
    DS_LAUNCH(KID_Q4_WRITE, k_q4_write, dim3((unsigned)blocks, s.B * s.Hkv), dim3(kWG), 0, st,
              static_cast<const _Float16 *>(K), channels, amax, static_cast<uint32_t *>(codes), s.Hkv,
              s.L_max, s.r, t0, n);
    return hipGetLastError();
}

hipError_t launch_predict_query(const void *x, const void *Wq, void *q_out, int B, int Dm, int N,
                                hipStream_t st)
{
    // about two workgroups per CU; every workgroup re-reads x once per batch pass
    int rows_per_wg = (N + 511) / 512;
    rows_per_wg = (rows_per_wg + 3) & ~3;
    const int blocks = (N + rows_per_wg - 1) / rows_per_wg;
    const size_t shmem = (size_t)std::min(B, kPredBatch) * Dm * sizeof(_Float16);
    DS_LAUNCH(KID_PREDICT, k_predict_query, dim3((unsigned)blocks), dim3(kWG), shmem, st,
              static_cast<const _Float16 *>(x), static_cast<const _Float16 *>(Wq),
              static_cast<_Float16 *>(q_out), B, Dm, N, rows_per_wg);
    return hipGetLastError();
}

hipError_t launch_append_kv(const void *k_new, const void *v_new, void *K, void *V,
                            const int32_t *channels, void *label, const ds_shape_t &s, int t0, int n,
                            int kv_stride, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    size_t blocks = ((size_t)n + 15) / 16;
    if (blocks > 2048) blocks = 2048;
    DS_LAUNCH(KID_APPEND_KV, k_append_kv, dim3((unsigned)blocks, s.B * s.Hkv), dim3(kWG), 0, st,
              static_cast<const uint4 *>(k_new), static_cast<const uint4 *>(v_new),
              static_cast<uint4 *>(K), static_cast<uint4 *>(V), channels,
              static_cast<uint16_t *>(label), s.Hkv, s.L_max, s.r, t0, n, kv_stride / 8);
    return hipGetLastError();
}

hipError_t launch_gather_host(const void *Kh, const void *Vh, const int32_t *idx, void *rows,
                              const ds_shape_t &s, hipStream_t st)
{
    DS_LAUNCH(KID_GATHER_HOST, k_gather_host, dim3((s.k + 15) / 16, s.B * s.Hkv), dim3(kWG), 0, st,
                       static_cast<const uint4 *>(Kh), static_cast<const uint4 *>(Vh), idx,
                       static_cast<uint4 *>(rows), s.L_max, s.k);
    return hipGetLastError();
}

hipError_t launch_probe(const void *src, size_t bytes, uint32_t *sink, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    const size_t blocks = (n16 + kWG * kProbeLoads - 1) / (kWG * kProbeLoads);
    DS_LAUNCH(KID_PROBE, k_probe, dim3((unsigned)blocks), dim3(kWG), 0, st,
                       static_cast<const uint4 *>(src), n16, sink);
    return hipGetLastError();
}

}  // namespace ds
