// C-ABI layer of libdsattn: argument validation, launch plans / workspace
// layout, the host-side offline calibration and the per-kernel event timing.
// No kernel code lives here; every device step is enqueued through the
// launchers declared in ds_internal.h.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include <hip/hip_runtime.h>

#include "ds_internal.h"

// Scratch of ds_sparse_decode_static: device memory that the library itself holds, one copy per
// GPU from the moment the code object is loaded there until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels get the resolved address.
#define DS_STATIC_SCRATCH_BYTES (32u << 20)
static __device__ __align__(256) unsigned char scratch[DS_STATIC_SCRATCH_BYTES];

namespace ds {

// ---------------------------------------------------------------- knobs
// (process-wide, for sweeps and tests; atomic so that a set in one thread and plans made in
//  another do not race -- a plan reads each knob once)
static std::atomic<int> g_tune[6];
int tune_get(int knob) { return (knob >= 0 && knob < 6) ? g_tune[knob].load(std::memory_order_relaxed) : 0; }

// ---------------------------------------------------------------- device
static thread_local const DeviceCaps *t_pretend = nullptr;
static thread_local DeviceCaps t_pretend_caps;

void device_caps_pretend(const DeviceCaps *caps)
{
    if (caps) {
        t_pretend_caps = *caps;
        t_pretend = &t_pretend_caps;
    } else {
        t_pretend = nullptr;
    }
}

DeviceCaps device_caps()
{
    if (t_pretend) return *t_pretend;
    static std::mutex mu;
    static DeviceCaps cache[64];
    static bool have[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();  // no device: the plan of an MI355X
        return DeviceCaps();
    }
    std::lock_guard<std::mutex> lk(mu);
    if (!have[dev]) {
        DeviceCaps c;
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) c.cus = v;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeNumberOfXccs, dev) == hipSuccess && v > 0) c.xccs = v;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) == hipSuccess && v > 0)
            c.lds_per_cu = v;
        (void)hipGetLastError();
        cache[dev] = c;
        have[dev] = true;
    }
    return cache[dev];
}

// ---------------------------------------------------------------- plans
static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static bool shape_ok(const ds_shape_t &s, bool need_rk)
{
    if (s.B < 1 || s.Hq < 1 || s.Hkv < 1 || s.d != kD) return false;
    if (s.Hq % s.Hkv != 0) return false;
    if (s.L < 1 || s.L > s.L_max) return false;
    if (need_rk && (s.r < 1 || s.r > s.d || s.k < 1)) return false;
    if ((int64_t)s.B * s.Hkv > 65535) return false;  // units ride on gridDim.y
    if ((int64_t)s.L_max * kD * 2 > 0xffffffffll) return false;  // rows are addressed by 32-bit byte offsets
    if (need_rk && (int64_t)std::min(s.k, s.L) * kD * 4 > 0xffffffffll) return false;
    return true;
}

// Workgroups of the refine-and-attend kernel that one CU holds when the kernel scores as well
// (matrix-core variants, query groups of 3+ heads): LDS is what limits them -- the chunk's keys and
// row list (6 bytes a token), the chunk histogram or the wavefront partials, whichever is larger,
// and about 3 KiB of small arrays -- and registers allow three.
static int group_wgs_per_cu(int G, int ch, int n_ch, const DeviceCaps &caps)
{
    const int gt = G <= 4 ? 4 : G <= 8 ? 8 : 16;
    const size_t lds = (size_t)ch * 6 + (size_t)n_ch * 4 + 512 + 3072 +
                       4 * (size_t)std::max(kHistBins, 4 * gt * kPartStride);
    return (int)std::min<size_t>(3, (size_t)caps.lds_per_cu / lds);
}

bool make_plan(const ds_shape_t &s, Plan *p, PlanFor purpose)
{
    if (!shape_ok(s, true)) return false;
    const DeviceCaps caps = device_caps();
    p->cus = caps.cus;
    p->units = s.B * s.Hkv;
    p->G = s.Hq / s.Hkv;
    p->k_eff = std::min(s.k, s.L);
    const int64_t tokens = (int64_t)p->units * s.L;

    int sc = tune_get(0);
    // fewer, larger workgroups: every workgroup pays an arrival atomic and a histogram flush
    if (sc == 0) {
        sc = (tokens >= (1 << 21)) ? 4096 : (tokens >= (1 << 20)) ? 2048 : 1024;
        // enough units to fill the device on their own: one workgroup scores a whole short unit
        // and takes the threshold bin from its own histogram, with no traffic between workgroups
        if (p->units >= caps.cus && s.L <= 8192) sc = (s.L + 255) & ~255;
    }
    p->sc_chunk = sc;
    p->n_sc = (s.L + sc - 1) / sc;

    // Launch shape of ds_sparse_decode: units of more than 8K tokens refine the threshold behind
    // the attention (two launches).  Short units get one workgroup each, which refines and attends
    // the whole unit out of LDS and writes the result itself (and scores it too when the label
    // cache is plain fp16 with 8 or 16 channels): everything between workgroups -- keys in memory,
    // histograms, arrival counting, partials -- costs more than it spreads at that size.  "Short"
    // is 4K tokens; 8K when there are enough units (256) to fill the device; 16K for a workgroup
    // that scores its unit itself, single heads or pairs, with 192 units or more (one 96 KiB
    // workgroup per CU).  Units of 4K to 8K tokens that are too few for that take the long units'
    // path when the attention launch can score (batch 4 x 8K tokens, 32 heads: 30.5 -> 25.1 us);
    // what is left refines the threshold in the scoring launch's tail.
    const bool one_wg_units =
        purpose != PLAN_SELECT &&
        (s.L <= 4096 || (p->units >= caps.cus && s.L <= 8192) ||
         (purpose == PLAN_DECODE_SCORING && p->units >= caps.cus * 3 / 4 && p->G <= 2 && s.L <= 16384));
    p->refine_attend = purpose != PLAN_SELECT &&
                       (tune_get(3) == 4 ||
                        (tune_get(3) == 0 && (s.L > (1 << 13) || one_wg_units ||
                                            (purpose == PLAN_DECODE_SCORING && s.L > (1 << 12)))));
    int ch = tune_get(1);
    p->group_scores_itself = false;
    p->unit_groups = 1;
    if (ch == 0 && p->refine_attend && !one_wg_units && p->G > 2 && purpose == PLAN_DECODE_SCORING) {
        // Query groups: one launch that scores as well pays off when all of its workgroups are
        // resident at once (a workgroup waits for the others of its unit twice).  Most
        // workgroups per CU first: the largest number of chunks per unit that still fits.
        // (units that do not fit at once even with one workgroup per CU go in two to four launches
        //  of a share of the units each)
        for (int g = 1; g <= 4 && ch == 0; ++g) {
            const int units_g = (p->units + g - 1) / g;
            for (int w = 3; w >= 1 && ch == 0; --w) {
                const int n = std::min((caps.cus * w) / units_g, kMaxChunks);
                if (n < 1) continue;
                const int c = std::max(2048, (((s.L + n - 1) / n) + 63) & ~63);  // (no point in tiny chunks)
                if (c <= 8192 && group_wgs_per_cu(p->G, c, (s.L + c - 1) / c, caps) >= w) {
                    ch = c;
                    p->group_scores_itself = true;
                    p->unit_groups = g;
                }
            }
        }
    }
    if (ch != 0) {
        // (set by the knob or just above)
    } else if (p->refine_attend && one_wg_units) {
        ch = (s.L + 255) & ~255;
    } else if (p->refine_attend) {
        // every workgroup resident at once (six per CU on the vector path, three on the matrix
        // cores) when chunks of up to 4096 / 6144 tokens allow it
        if (p->G <= 2) {
            // A launch that scores as well needs its whole grid resident, and LDS decides how many
            // workgroups a CU holds (6 bytes a token for keys and row list, about 26 KiB of fixed
            // arrays): the largest number of chunks per unit that gives four, else three, two, one
            // workgroup per CU.  (Fixed chunks of up to 4096 tokens left 128 units of 32K tokens
            // with 1024 workgroups of which 768 fit: scoring became a launch of its own, 55 us per
            // layer against 46.5 with four chunks of 8192 tokens in one launch.)
            // Units that do not fit at once even so (256 units of 32K tokens) go in two to four
            // launches of a share of the units each, every one of them resident at once (two
            // launches of 128 units: 93 us per layer against 105 with scoring as a launch of its own).
            if (purpose == PLAN_DECODE_SCORING) {
                for (int g = 1; g <= 4 && ch == 0; ++g) {
                    const int units_g = (p->units + g - 1) / g;
                    for (int w = 4; w >= 1 && ch == 0; --w) {
                        const int n = std::min((caps.cus * w) / units_g, kMaxChunks);
                        if (n < 2) continue;
                        const int c = std::max(1024, (((s.L + n - 1) / n) + 63) & ~63);
                        const size_t lds = (size_t)c * 6 + (size_t)((s.L + c - 1) / c) * 4 + (26u << 10);
                        if (c <= 16384 && lds * w <= (size_t)caps.lds_per_cu) {
                            ch = c;
                            p->unit_groups = g;
                        }
                    }
                }
            }
            if (ch == 0) {
                ch = 1024;
                while (ch < 4096 && (int64_t)p->units * ((s.L + ch - 1) / ch) > 6 * caps.cus) ch *= 2;
            }
        } else {
            ch = 2048;
            while (ch < 6144 && ch < s.L && (int64_t)p->units * ((s.L + ch - 1) / ch) > 3 * caps.cus) ch += 256;
        }
    } else {
        ch = (tokens >= (1 << 21)) ? 2048 : (tokens >= (1 << 20)) ? 1024 : (tokens >= (1 << 18)) ? 512 : 256;
        if (p->G >= 4 && ch < 4096) ch *= 2;  // a query group writes G partials per chunk
        while ((s.L + ch - 1) / ch > kMaxChunks && ch < 4096) ch *= 2;
        // The matrix-core attention holds three workgroups per CU (768 on the device).  A launch
        // slightly over that runs a nearly empty second round: grow the chunks to fit in one.
        if (p->G >= 4)
            while ((int64_t)p->units * ((s.L + ch - 1) / ch) > 3 * caps.cus && ch < 6144 && ch < s.L) ch += 256;
    }
    p->ch = ch;
    p->n_ch = (s.L + ch - 1) / ch;
    if (p->n_ch > kMaxChunks) return false;
    p->key_stride = (s.L + 3) & ~3;

    size_t off = 0;
    p->off_ctl = off;   off = align_up(off + (size_t)p->units * sizeof(UnitCtl), 256);
    p->off_hist = off;  off = align_up(off + (size_t)p->units * kHistBins * 4, 256);
    p->off_coarse = off; off = align_up(off + (size_t)p->units * 256 * 4, 256);
    p->off_keys = off;  off = align_up(off + (size_t)p->units * p->key_stride * 4, 256);
    p->off_cand = off;  off = align_up(off + (size_t)p->units * s.L * 8, 256);
    p->off_ndef = off;  off = align_up(off + (size_t)p->units * p->n_ch * 4, 256);
    p->off_offs = off;  off = align_up(off + (size_t)p->units * p->n_ch * 4, 256);
    p->off_part = off;  off = align_up(off + (size_t)p->units * p->G * p->n_ch * kPartStride * 4, 256);
    p->total = off;
    return true;
}

bool make_dense_plan(const ds_shape_t &s, int n_tokens, DensePlan *p)
{
    if (!shape_ok(s, false) || n_tokens < 1) return false;
    p->units = s.B * s.Hkv;
    p->G = s.Hq / s.Hkv;
    int ch = tune_get(2);
    if (ch == 0) {
        const int64_t tokens = (int64_t)p->units * n_tokens;
        ch = (tokens >= (1 << 20)) ? 1024 : (tokens >= (1 << 18)) ? 256 : 64;
    }
    p->ch = ch;
    p->n_ch = (n_tokens + ch - 1) / ch;
    // same control prefix (records + histograms) as the sparse plan, so that sparse and dense
    // calls may alternate on one workspace without disturbing each other's zeroed counters
    size_t off = 0;
    p->off_ctl = off;   off = align_up(off + (size_t)p->units * sizeof(UnitCtl), 256);
    off = align_up(off + (size_t)p->units * kHistBins * 4, 256);
    off = align_up(off + (size_t)p->units * 256 * 4, 256);
    p->off_part = off;  off = align_up(off + (size_t)p->units * p->G * p->n_ch * kPartStride * 4, 256);
    p->total = off;
    return true;
}

// ---------------------------------------------------------------- per-kernel event timing
static const char *const kKernelNames[KID_COUNT] = {
    "k_init", "k_score", "k_cand", "k_attend", "k_compact", "k_dense",
    "k_attend_rows", "k_label", "k_gather_host", "k_probe",
    "k_refine_attend", "k_append_kv", "k_q4_amax", "k_q4_write", "k_predict_query"};

struct ProfRec { int id; hipEvent_t a, b; };
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof_recs;
static std::vector<hipEvent_t> g_prof_pool;

static hipEvent_t prof_event()
{
    if (!g_prof_pool.empty()) {
        hipEvent_t e = g_prof_pool.back();
        g_prof_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

bool prof_events(int id, hipEvent_t *start, hipEvent_t *stop)
{
    if (!g_prof_on) return false;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    hipEvent_t a = prof_event();
    if (!a) return false;
    hipEvent_t b = prof_event();
    if (!b) { g_prof_pool.push_back(a); return false; }
    g_prof_recs.push_back({id, a, b});
    *start = a;
    *stop = b;
    return true;
}

}  // namespace ds

using namespace ds;

// ---------------------------------------------------------------- helpers
static bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

#define DS_TRY(expr)                                  \
    do {                                              \
        if ((expr) != hipSuccess) return DS_ERR_HIP;  \
    } while (0)

extern "C" {

const char *ds_strerror(ds_status_t status)
{
    switch (status) {
    case DS_OK: return "ok";
    case DS_ERR_NULL: return "required pointer is NULL";
    case DS_ERR_SHAPE: return "invalid shape or size argument";
    case DS_ERR_ALIGN: return "pointer is not sufficiently aligned";
    case DS_ERR_WORKSPACE: return "workspace is too small (static-scratch call: the shape needs more than ds_static_scratch_bytes())";
    case DS_ERR_UNSUPPORTED: return "configuration not supported";
    case DS_ERR_HIP: return "HIP runtime reported an error";
    }
    return "unknown status";
}

int ds_version(void) { return 109; }

ds_status_t ds_calibrate_channels(const uint16_t *q_calib, const uint16_t *k_calib, int32_t N,
                                  int32_t Hq, int32_t Hkv, int32_t d, int32_t r,
                                  ds_calib_mode_t mode, int32_t *channels_out)
{
    if (!q_calib || !k_calib || !channels_out) return DS_ERR_NULL;
    if (N < 1 || Hq < 1 || Hkv < 1 || d < 1 || r < 1 || r > d || Hq % Hkv != 0) return DS_ERR_SHAPE;
    if (mode != DS_CALIB_Q && mode != DS_CALIB_K && mode != DS_CALIB_QK) return DS_ERR_SHAPE;
    const int G = Hq / Hkv;
    // |x| of a binary16 bit pattern, widened through binary32 bit assembly
    auto habs = [](uint16_t h) -> double {
        const uint32_t e = (h >> 10) & 0x1f, m = h & 0x3ff;
        if (e == 0) return std::ldexp((double)m, -24);
        if (e == 31) return m ? NAN : INFINITY;
        return std::ldexp((double)(m | 0x400), (int)e - 25);
    };
    std::vector<double> mq(d), mk(d), w(d);
    std::vector<int32_t> order(d);
    for (int h = 0; h < Hkv; ++h) {
        std::fill(mq.begin(), mq.end(), 0.0);
        std::fill(mk.begin(), mk.end(), 0.0);
        for (int n = 0; n < N; ++n) {
            for (int g = 0; g < G; ++g) {
                const uint16_t *row = q_calib + ((size_t)n * Hq + (size_t)h * G + g) * d;
                for (int c = 0; c < d; ++c) mq[c] += habs(row[c]);
            }
            const uint16_t *krow = k_calib + ((size_t)n * Hkv + h) * d;
            for (int c = 0; c < d; ++c) mk[c] += habs(krow[c]);
        }
        for (int c = 0; c < d; ++c) {
            const double a = mq[c] / ((double)N * G), b = mk[c] / (double)N;
            w[c] = mode == DS_CALIB_Q ? a : mode == DS_CALIB_K ? b : a * b;
            order[c] = c;
        }
        std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return w[x] > w[y]; });
        std::sort(order.begin(), order.begin() + r);
        std::copy(order.begin(), order.begin() + r, channels_out + (size_t)h * r);
    }
    return DS_OK;
}

static ds_status_t check_label_args(const void *K, const int32_t *channels, void *label,
                                    const ds_shape_t *s)
{
    if (!K || !channels || !label || !s) return DS_ERR_NULL;
    if (s->B < 1 || s->Hkv < 1 || s->d != kD || s->r < 1 || s->r > s->d || s->L_max < 1)
        return DS_ERR_SHAPE;
    if ((int64_t)s->B * s->Hkv > 65535) return DS_ERR_SHAPE;
    if (!aligned(K, 256) || !aligned(label, 16)) return DS_ERR_ALIGN;
    return DS_OK;
}

ds_status_t ds_build_label(const void *K, const int32_t *channels, void *label,
                           const ds_shape_t *shape, void *stream)
{
    ds_status_t st = check_label_args(K, channels, label, shape);
    if (st != DS_OK) return st;
    if (shape->L < 1 || shape->L > shape->L_max) return DS_ERR_SHAPE;
    DS_TRY(launch_label(K, channels, label, *shape, 0, shape->L, (hipStream_t)stream));
    return DS_OK;
}

ds_status_t ds_append_label(const void *K, const int32_t *channels, void *label,
                            const ds_shape_t *shape, int32_t t0, int32_t n_new, void *stream)
{
    ds_status_t st = check_label_args(K, channels, label, shape);
    if (st != DS_OK) return st;
    if (t0 < 0 || n_new < 0 || (int64_t)t0 + n_new > shape->L_max) return DS_ERR_SHAPE;
    DS_TRY(launch_label(K, channels, label, *shape, t0, n_new, (hipStream_t)stream));
    return DS_OK;
}

ds_status_t ds_build_label_q4(const void *K, const int32_t *channels, void *label_q4, float *amax,
                              const ds_shape_t *shape, void *stream)
{
    if (!amax) return DS_ERR_NULL;
    ds_status_t st = check_label_args(K, channels, label_q4, shape);
    if (st != DS_OK) return st;
    if (shape->L < 1 || shape->L > shape->L_max) return DS_ERR_SHAPE;
    if (!aligned(amax, 4)) return DS_ERR_ALIGN;
    DS_TRY(launch_q4_amax(K, channels, amax, *shape, (hipStream_t)stream));
    DS_TRY(launch_q4_write(K, channels, amax, label_q4, *shape, 0, shape->L, (hipStream_t)stream));
    return DS_OK;
}

ds_status_t ds_append_label_q4(const void *K, const int32_t *channels, void *label_q4,
                               const float *amax, const ds_shape_t *shape, int32_t t0,
                               int32_t n_new, void *stream)
{
    if (!amax) return DS_ERR_NULL;
    ds_status_t st = check_label_args(K, channels, label_q4, shape);
    if (st != DS_OK) return st;
    if (t0 < 0 || n_new < 0 || (int64_t)t0 + n_new > shape->L_max) return DS_ERR_SHAPE;
    DS_TRY(launch_q4_write(K, channels, amax, label_q4, *shape, t0, n_new, (hipStream_t)stream));
    return DS_OK;
}

ds_status_t ds_build_label_kv(const void *KV, const int32_t *channels, void *label,
                              const ds_shape_t *shape, void *stream)
{
    ds_status_t st = check_label_args(KV, channels, label, shape);
    if (st != DS_OK) return st;
    if (shape->L < 1 || shape->L > shape->L_max) return DS_ERR_SHAPE;
    DS_TRY(launch_label(KV, channels, label, *shape, 0, shape->L, (hipStream_t)stream, 2 * kD));
    return DS_OK;
}

ds_status_t ds_append_kv(const void *k_new, const void *v_new, void *K, void *V,
                         const int32_t *channels, void *label, const ds_shape_t *shape, int32_t t0,
                         int32_t n_new, ds_kv_layout_t layout, void *stream)
{
    if (!k_new || !v_new) return DS_ERR_NULL;
    if (layout != DS_KV_SPLIT && layout != DS_KV_INTERLEAVED) return DS_ERR_SHAPE;
    if (layout == DS_KV_SPLIT && !V) return DS_ERR_NULL;
    ds_status_t st = check_label_args(K, channels, label, shape);
    if (st != DS_OK) return st;
    if (t0 < 0 || n_new < 0 || (int64_t)t0 + n_new > shape->L_max) return DS_ERR_SHAPE;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || (layout == DS_KV_SPLIT && !aligned(V, 256)))
        return DS_ERR_ALIGN;
    const bool il = layout == DS_KV_INTERLEAVED;
    void *Vp = il ? static_cast<void *>(static_cast<char *>(K) + kD * 2) : V;
    DS_TRY(launch_append_kv(k_new, v_new, K, Vp, channels, label, *shape, t0, n_new, il ? 2 * kD : kD,
                            (hipStream_t)stream));
    return DS_OK;
}

size_t ds_workspace_bytes(const ds_shape_t *shape)
{
    if (!shape) return 0;
    Plan p;
    DensePlan dp, rp;
    size_t need = 0;
    for (PlanFor purpose : {PLAN_SELECT, PLAN_DECODE, PLAN_DECODE_SCORING}) {
        if (make_plan(*shape, &p, purpose)) {
            need = std::max(need, p.total);
            if (make_dense_plan(*shape, p.k_eff, &rp)) need = std::max(need, rp.total);
        }
    }
    if (make_dense_plan(*shape, shape->L, &dp)) need = std::max(need, dp.total);
    return need;
}

ds_status_t ds_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return DS_ERR_NULL;
    if (workspace_bytes == 0 || workspace_bytes % 16 != 0) return DS_ERR_SHAPE;
    if (!aligned(workspace, 16)) return DS_ERR_ALIGN;
    DS_TRY(launch_init(workspace, workspace_bytes, (hipStream_t)stream));
    return DS_OK;
}

ds_status_t ds_workspace_errors(const void *workspace, size_t workspace_bytes, const ds_shape_t *shape,
                                void *stream, int32_t *n_failed, int32_t *first_code)
{
    if (!workspace || !shape) return DS_ERR_NULL;
    Plan p;
    if (!shape_ok(*shape, true)) return DS_ERR_SHAPE;
    if (!make_plan(*shape, &p, PLAN_DECODE)) return DS_ERR_UNSUPPORTED;
    const size_t bytes = (size_t)p.units * sizeof(UnitCtl);
    if (workspace_bytes < p.off_ctl + bytes) return DS_ERR_WORKSPACE;
    std::vector<UnitCtl> ctl((size_t)p.units);
    if (hipMemcpyAsync(ctl.data(), static_cast<const char *>(workspace) + p.off_ctl, bytes, hipMemcpyDeviceToHost,
                       (hipStream_t)stream) != hipSuccess ||
        hipStreamSynchronize((hipStream_t)stream) != hipSuccess)
        return DS_ERR_HIP;
    int32_t n = 0, first = 0;
    for (const UnitCtl &c : ctl)
        if (c.err) {
            if (!n) first = (int32_t)c.err;
            ++n;
        }
    if (n_failed) *n_failed = n;
    if (first_code) *first_code = first;
    return DS_OK;
}

static ds_status_t select_common(const void *q, const void *label, const int32_t *channels,
                                 void *workspace, size_t workspace_bytes, const ds_shape_t *shape,
                                 Plan *p, PlanFor purpose = PLAN_SELECT)
{
    if (!q || !label || !channels || !workspace || !shape) return DS_ERR_NULL;
    if (!shape_ok(*shape, true)) return DS_ERR_SHAPE;
    if (!make_plan(*shape, p, purpose)) return DS_ERR_UNSUPPORTED;
    if (!aligned(q, 16) || !aligned(label, 16) || !aligned(workspace, 16)) return DS_ERR_ALIGN;
    if (workspace_bytes < p->total) return DS_ERR_WORKSPACE;
    return DS_OK;
}

static ds_status_t enqueue_select(const void *q, const void *label, const int32_t *channels,
                                  void *ws, const Plan &p, const ds_shape_t &s, bool want_offsets,
                                  hipStream_t st, ScoreSrc src = ScoreSrc())
{
    // Units of up to 8K tokens: the scoring launch's last workgroup per unit also settles the
    // exact threshold (knob 4 = 1 forces the separate candidate launch, 2 forces the tail).
    const int mode = tune_get(4);
    const bool tail_refine = mode == 2 || (mode == 0 && s.L <= (1 << 13));
    DS_TRY(launch_score(q, label, channels, ws, p, s, tail_refine, want_offsets, st, src));
    if (!tail_refine) DS_TRY(launch_cand(ws, p, s, want_offsets, st));
    return DS_OK;
}

static bool label_may_score(const ds_shape_t &s, ScoreSrcKind kind)
{
    // the attention launch can score as well when the labels are plain fp16 with 8 or 16 channels,
    // or 4-bit codes of up to 16 channels in rows that 16-byte loads can take (knob 4 = 1 keeps
    // the separate scoring launch)
    return tune_get(4) != 1 && ((kind == SRC_LABEL && (s.r == 8 || s.r == 16)) ||
                                (kind == SRC_Q4 && s.r <= 16 && (s.L_max & (s.r > 8 ? 1 : 3)) == 0));
}

// Whether the attention launch of a decode call scores as well: a unit with one workgroup always
// can; several workgroups per unit wait for each other before all of them have started, so the
// whole grid has to be resident at once -- single heads and pairs: four workgroups per compute
// unit; larger query groups: when the plan found chunks that make it so.  Knob 4 = 2 forces it,
// 1 forbids it.  (The launcher checks the grid against the occupancy the runtime reports.)
static bool plan_scores_itself(const Plan &p, bool may_score)
{
    return may_score && (p.n_ch == 1 || tune_get(4) == 2 ||
                         (tune_get(4) == 0 && p.G <= 2 &&
                          (int64_t)((p.units + p.unit_groups - 1) / p.unit_groups) * p.n_ch <= 4 * (int64_t)p.cus) ||
                         (tune_get(4) == 0 && p.group_scores_itself));
}

// ds_sparse_decode with the scores taken from the label cache, from the K rows themselves or from
// the 4-bit label cache (`label` is then that source's array).
static ds_status_t sparse_decode_impl(const void *q, const void *label, const void *K, const void *V,
                                      const int32_t *channels, float *out, int32_t *idx_out,
                                      void *workspace, size_t workspace_bytes,
                                      const ds_shape_t *shape, void *stream, ScoreSrc src,
                                      int kv_stride = kD, bool clear_first = false)
{
    if (!K || !V || !out) return DS_ERR_NULL;
    Plan p;
    const bool may_score = shape && label_may_score(*shape, src.kind);
    ds_status_t rc = select_common(q, label, channels, workspace, workspace_bytes, shape, &p,
                                   may_score ? PLAN_DECODE_SCORING : PLAN_DECODE);
    if (rc != DS_OK) return rc;
    if (!aligned(K, 256) || !aligned(V, 256) || !aligned(out, 16) || (idx_out && !aligned(idx_out, 16)))
        return DS_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    // (a workspace shared by calls of different shapes: counters, histograms and error words start
    //  from zero whatever the last call left there -- a fill kernel, so that the call can be captured)
    if (clear_first) DS_TRY(launch_init(workspace, p.off_keys, st));
    // a workgroup that may score its tokens itself: one launch, keys never leave LDS
    // ... and so can several workgroups per unit (their chunk histograms meet in memory and the
    // threshold bin is published to them) as long as the whole grid is resident at once: single
    // heads and pairs, four workgroups per CU; larger query groups when the plan found chunks that
    // make it so (up to three workgroups per CU).  Knob 4 = 2 forces it, 1 forbids it.
    bool scores_itself = plan_scores_itself(p, may_score);
    const bool q4 = src.kind == SRC_Q4;
    if (p.refine_attend && refine_attend_ok(p, scores_itself)) {
        // (the runtime's occupancy figure for the kernel decides whether the workgroups that wait
        //  for each other are all resident; if not, the separate scoring launch needs less room,
        //  and the three launches below need none)
        if (scores_itself && !refine_attend_fits(p, *shape, true, q4)) scores_itself = false;
        if (scores_itself) {
            DS_TRY(launch_refine_attend(q, K, V, workspace, out, idx_out, p, *shape, st, kv_stride, label, channels,
                                        q4 ? src.amax : nullptr));
            return DS_OK;
        }
        // otherwise scoring leaves keys and the threshold bin; one more launch settles the exact
        // threshold behind the attention over the rows that are selected either way
        if (refine_attend_ok(p, false) && refine_attend_fits(p, *shape, false, q4)) {
            DS_TRY(launch_score(q, label, channels, workspace, p, *shape, false, false, st, src));
            DS_TRY(launch_refine_attend(q, K, V, workspace, out, idx_out, p, *shape, st, kv_stride));
            return DS_OK;
        }
    }
    rc = enqueue_select(q, label, channels, workspace, p, *shape, idx_out != nullptr, st, src);
    if (rc != DS_OK) return rc;
    DS_TRY(launch_attend_sparse(q, K, V, workspace, out, idx_out, p, *shape, st, kv_stride));
    return DS_OK;
}

ds_status_t ds_pretend_device(int32_t cus, int32_t xccs, int32_t lds_per_cu)
{
    if (cus == 0 && xccs == 0 && lds_per_cu == 0) {
        device_caps_pretend(nullptr);
        return DS_OK;
    }
    if (cus < 1 || xccs < 1 || cus % xccs != 0 || lds_per_cu < (64 << 10)) return DS_ERR_SHAPE;
    DeviceCaps c;
    c.cus = cus;
    c.xccs = xccs;
    c.lds_per_cu = lds_per_cu;
    device_caps_pretend(&c);
    return DS_OK;
}

ds_status_t ds_plan_describe(const ds_shape_t *shape, int32_t label_kind, int32_t out[8])
{
    if (!shape || !out) return DS_ERR_NULL;
    if (label_kind < 0 || label_kind > 2 || !shape_ok(*shape, true)) return DS_ERR_SHAPE;
    const ScoreSrcKind kind = static_cast<ScoreSrcKind>(label_kind);
    const bool may_score = label_may_score(*shape, kind);
    Plan p;
    if (!make_plan(*shape, &p, may_score ? PLAN_DECODE_SCORING : PLAN_DECODE)) return DS_ERR_UNSUPPORTED;
    const bool si = plan_scores_itself(p, may_score);
    const bool ra = p.refine_attend && refine_attend_ok(p, si);
    const int planned = !ra ? 3 : si ? p.unit_groups : 2;
    int actual = -1;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) == hipSuccess && n_dev > 0) {
        actual = 3;
        if (ra) {
            const bool q4 = kind == SRC_Q4;
            if (si && refine_attend_fits(p, *shape, true, q4)) actual = p.unit_groups;
            else if (refine_attend_ok(p, false) && refine_attend_fits(p, *shape, false, q4)) actual = 2;
        }
    }
    (void)hipGetLastError();
    out[0] = planned;
    out[1] = actual;
    out[2] = p.ch;
    out[3] = p.n_ch;
    out[4] = p.units * p.n_ch;
    out[5] = p.cus;
    out[6] = si ? 1 : 0;
    out[7] = p.G;
    return DS_OK;
}

ds_status_t ds_sparse_decode(const void *q, const void *label, const void *K, const void *V,
                             const int32_t *channels, float *out, int32_t *idx_out,
                             void *workspace, size_t workspace_bytes, const ds_shape_t *shape,
                             void *stream)
{
    return sparse_decode_impl(q, label, K, V, channels, out, idx_out, workspace, workspace_bytes, shape,
                              stream, ScoreSrc());
}

// Address of this device's copy of the static scratch array, resolved once per device.
static ds_status_t static_scratch(void **ptr)
{
    static std::mutex mu;
    static void *per_device[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return DS_ERR_HIP;
    if (dev < 0 || dev >= 64) return DS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lk(mu);
    if (!per_device[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DS_ERR_HIP;
        per_device[dev] = p;
    }
    *ptr = per_device[dev];
    return DS_OK;
}

size_t ds_static_scratch_bytes(void) { return DS_STATIC_SCRATCH_BYTES; }

ds_status_t ds_static_init(void)
{
    void *p = nullptr;
    return static_scratch(&p);
}

ds_status_t ds_sparse_decode_static(const void *q, const void *label, const void *K, const void *V,
                                    const int32_t *channels, float *out, int32_t *idx_out,
                                    const ds_shape_t *shape, void *stream)
{
    if (!q || !label || !K || !V || !channels || !out || !shape) return DS_ERR_NULL;
    void *ws = nullptr;
    ds_status_t rc = static_scratch(&ws);
    if (rc != DS_OK) return rc;
    // shapes whose scratch layout is larger than the array come back as DS_ERR_WORKSPACE
    return sparse_decode_impl(q, label, K, V, channels, out, idx_out, ws, DS_STATIC_SCRATCH_BYTES, shape,
                              stream, ScoreSrc(), kD, true);
}

ds_status_t ds_sparse_decode_nolabel(const void *q, const void *K, const void *V,
                                     const int32_t *channels, float *out, int32_t *idx_out,
                                     void *workspace, size_t workspace_bytes,
                                     const ds_shape_t *shape, void *stream)
{
    ScoreSrc src;
    src.kind = SRC_K_ROWS;
    return sparse_decode_impl(q, K, K, V, channels, out, idx_out, workspace, workspace_bytes, shape,
                              stream, src);
}

ds_status_t ds_sparse_decode_q4(const void *q, const void *label_q4, const float *amax, const void *K,
                                const void *V, const int32_t *channels, float *out,
                                int32_t *idx_out, void *workspace, size_t workspace_bytes,
                                const ds_shape_t *shape, void *stream)
{
    if (!amax) return DS_ERR_NULL;
    if (!aligned(amax, 4)) return DS_ERR_ALIGN;
    ScoreSrc src;
    src.kind = SRC_Q4;
    src.amax = amax;
    return sparse_decode_impl(q, label_q4, K, V, channels, out, idx_out, workspace, workspace_bytes,
                              shape, stream, src);
}

ds_status_t ds_sparse_decode_kv(const void *q, const void *label, const void *KV,
                                const int32_t *channels, float *out, int32_t *idx_out,
                                void *workspace, size_t workspace_bytes, const ds_shape_t *shape,
                                void *stream)
{
    if (!KV) return DS_ERR_NULL;
    // a row is addressed by a 32-bit byte offset inside its unit: 512-byte steps here
    if (shape && (int64_t)shape->L_max * 4 * kD > 0xffffffffll) return DS_ERR_SHAPE;
    const void *V = static_cast<const char *>(KV) + kD * 2;
    return sparse_decode_impl(q, label, KV, V, channels, out, idx_out, workspace, workspace_bytes, shape,
                              stream, ScoreSrc(), 2 * kD);
}

ds_status_t ds_select(const void *q, const void *label, const int32_t *channels, int32_t *idx_out,
                      void *workspace, size_t workspace_bytes, const ds_shape_t *shape, void *stream)
{
    if (!idx_out) return DS_ERR_NULL;
    Plan p;
    ds_status_t rc = select_common(q, label, channels, workspace, workspace_bytes, shape, &p);
    if (rc != DS_OK) return rc;
    if (!aligned(idx_out, 16)) return DS_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    rc = enqueue_select(q, label, channels, workspace, p, *shape, true, st);
    if (rc != DS_OK) return rc;
    DS_TRY(launch_compact(workspace, idx_out, p, *shape, st));
    return DS_OK;
}

ds_status_t ds_dense_decode(const void *q, const void *K, const void *V, float *out,
                            void *workspace, size_t workspace_bytes, const ds_shape_t *shape,
                            void *stream)
{
    if (!q || !K || !V || !out || !workspace || !shape) return DS_ERR_NULL;
    if (!shape_ok(*shape, false)) return DS_ERR_SHAPE;
    DensePlan p;
    if (!make_dense_plan(*shape, shape->L, &p)) return DS_ERR_UNSUPPORTED;
    if (!aligned(K, 256) || !aligned(V, 256) || !aligned(q, 16) || !aligned(out, 16) ||
        !aligned(workspace, 16))
        return DS_ERR_ALIGN;
    if (workspace_bytes < p.total) return DS_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    DS_TRY(launch_attend_dense(q, K, V, workspace, out, p, *shape, st));
    return DS_OK;
}

ds_status_t ds_predict_query(const void *x, const void *Wq, void *q_out, int32_t B, int32_t Dm,
                             int32_t N, void *stream)
{
    if (!x || !Wq || !q_out) return DS_ERR_NULL;
    // 16-byte pieces of a row; x for up to four batch rows has to fit the 64 KiB of LDS asked for
    if (B < 1 || N < 1 || Dm < 8 || Dm % 8 != 0 || Dm > 8192) return DS_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(Wq, 16) || !aligned(q_out, 2)) return DS_ERR_ALIGN;
    DS_TRY(launch_predict_query(x, Wq, q_out, B, Dm, N, (hipStream_t)stream));
    return DS_OK;
}

ds_status_t ds_gather_rows_host(const void *K_host, const void *V_host, const int32_t *idx,
                                void *KV_rows, const ds_shape_t *shape, void *stream)
{
    if (!K_host || !V_host || !idx || !KV_rows || !shape) return DS_ERR_NULL;
    if (!shape_ok(*shape, true)) return DS_ERR_SHAPE;
    if (!aligned(K_host, 256) || !aligned(V_host, 256) || !aligned(KV_rows, 256) || !aligned(idx, 4))
        return DS_ERR_ALIGN;
    DS_TRY(launch_gather_host(K_host, V_host, idx, KV_rows, *shape, (hipStream_t)stream));
    return DS_OK;
}

ds_status_t ds_attend_rows(const void *q, const void *KV_rows, float *out, void *workspace,
                           size_t workspace_bytes, const ds_shape_t *shape, void *stream)
{
    if (!q || !KV_rows || !out || !workspace || !shape) return DS_ERR_NULL;
    if (!shape_ok(*shape, true)) return DS_ERR_SHAPE;
    const int n_rows = std::min(shape->k, shape->L);
    DensePlan p;
    if (!make_dense_plan(*shape, n_rows, &p)) return DS_ERR_UNSUPPORTED;
    if (!aligned(KV_rows, 256) || !aligned(q, 16) || !aligned(out, 16) || !aligned(workspace, 16))
        return DS_ERR_ALIGN;
    if (workspace_bytes < p.total) return DS_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    DS_TRY(launch_attend_rows(q, KV_rows, workspace, out, p, *shape, n_rows, st));
    return DS_OK;
}

ds_status_t ds_probe_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink) return DS_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || bytes / 16 / (kWG * 8) > 0x7fffffffull) return DS_ERR_SHAPE;
    if (!aligned(src, 16) || !aligned(sink, 4)) return DS_ERR_ALIGN;
    DS_TRY(launch_probe(src, bytes, sink, (hipStream_t)stream));
    return DS_OK;
}

int ds_profile_kernel_count(void) { return KID_COUNT; }

const char *ds_profile_kernel_name(int id)
{
    return (id >= 0 && id < KID_COUNT) ? kKernelNames[id] : "";
}

ds_status_t ds_profile_enable(int on)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = on != 0;
    return DS_OK;
}

ds_status_t ds_profile_reset(void)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto &r : g_prof_recs) {
        g_prof_pool.push_back(r.a);
        g_prof_pool.push_back(r.b);
    }
    g_prof_recs.clear();
    return DS_OK;
}

ds_status_t ds_profile_read(int id, double *total_ms, int64_t *launches)
{
    if (!total_ms || !launches) return DS_ERR_NULL;
    if (id < 0 || id >= KID_COUNT) return DS_ERR_SHAPE;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    double tot = 0.0;
    int64_t n = 0;
    for (auto &r : g_prof_recs) {
        if (r.id != id) continue;
        if (hipEventSynchronize(r.b) != hipSuccess) return DS_ERR_HIP;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return DS_ERR_HIP;
        tot += ms;
        ++n;
    }
    *total_ms = tot;
    *launches = n;
    return DS_OK;
}

ds_status_t ds_tune_set(int knob, int value)
{
    if (knob < 0 || knob > 5) return DS_ERR_SHAPE;
    if (value < 0) return DS_ERR_SHAPE;
    if (value != 0) {
        if (knob == 0 && (value % 256 != 0 || value > (1 << 20))) return DS_ERR_SHAPE;
        if (knob == 1 && (value % 64 != 0 || value > 16384)) return DS_ERR_SHAPE;
        if (knob == 2 && (value % 16 != 0 || value > (1 << 20))) return DS_ERR_SHAPE;
        if (knob == 3 && value != 1 && value != 4) return DS_ERR_SHAPE;
        if (knob == 4 && value > 2) return DS_ERR_SHAPE;
    }
    g_tune[knob].store(value, std::memory_order_relaxed);
    return DS_OK;
}

int ds_tune_get(int knob) { return tune_get(knob); }

}  // extern "C"
