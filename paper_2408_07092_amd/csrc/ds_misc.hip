// Label-cache maintenance (Sec. 4.2), the host-row gather of the offload
// arrangement (Sec. 5.1) and the read-bandwidth probe.
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

// Decode-step cache maintenance in one launch (Sec. 4.2: in decoding only the new tokens'
// heavy-channel values are added to the label cache): the n new tokens' K and V rows go into
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

// Plain streaming read: every workgroup reads 32 KiB as 16-byte loads.
__global__ __launch_bounds__(kWG) void k_probe(const uint4 *__restrict__ src, size_t n16,
                                               uint32_t *sink)
{
    const size_t base = (size_t)blockIdx.x * (kWG * 8) + threadIdx.x;
    uint4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const size_t e = base + (size_t)i * kWG;
        v[i] = (e < n16) ? src[e] : make_uint4(0, 0, 0, 0);
    }
    uint32_t x = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) x ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
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
    const size_t blocks = (n16 + kWG * 8 - 1) / (kWG * 8);
    DS_LAUNCH(KID_PROBE, k_probe, dim3((unsigned)blocks), dim3(kWG), 0, st,
                       static_cast<const uint4 *>(src), n16, sink);
    return hipGetLastError();
}

}  // namespace ds
