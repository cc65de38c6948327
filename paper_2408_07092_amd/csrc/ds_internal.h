// Internal declarations shared by the translation units of libdsattn.
// Host-side plan (launch shapes + workspace layout) and the launcher functions
// each .hip file exports to the C-ABI layer.
#pragma once

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

#include "ds_attn.h"

namespace ds {

constexpr int kD = 128;          // head dimension the kernels are written for
constexpr int kWG = 256;         // threads per workgroup (4 wavefronts of 64)
constexpr int kHistBits = 12;    // first-level radix: top 12 bits of the ordered key
constexpr int kHistBins = 1 << kHistBits;
constexpr int kKeyShift = 32 - kHistBits;
constexpr int kPartStride = 132; // floats per attention partial: m, l, 2 pad, acc[128]
constexpr int kMaxChunks = 8192; // chunk offsets of one unit must fit one workgroup's LDS

// Per-unit selection state in the workspace (64 bytes).  Counters and hand-over words are zero
// between calls: the workgroup that consumes one resets it (see ds_workspace_init); err stays.
struct UnitCtl {
    uint32_t bstar;     // first-level bin holding the k-th largest key (left by k_score / k_cand)
    uint32_t krem;      // how many keys of that bin are selected (>= 1)
    uint32_t ncand;     // k_cand: candidates appended so far (keys in bin bstar)
    uint32_t T;         // k_cand / k_score's tail: exact k-th largest key
    int32_t tcut;       // keys equal to T are selected iff token <= tcut
    uint32_t arrive_a;  // workgroups that have added their chunk histogram to the unit's (k_score, or
                        // k_refine_attend when it scores itself)
    uint32_t arrive_b;  // workgroups of k_cand that finished this unit
    uint32_t arrive_c;  // workgroups of an attention kernel whose partial is written (k_refine_attend:
                        // the high half counts those whose wait for another workgroup ran out)
    uint32_t cnt_a;     // k_refine_attend: the exact threshold as published by the workgroup that
    uint32_t cnt_b;     //   settled it, one 64-bit word {T, tie cut | 1 << 31}
    uint32_t cnt_c;
    uint32_t err;       // non-zero once a bounded wait between workgroups gave up (the first code stays)
    uint32_t pad[4];    // pad[2..3]: k_refine_attend's 64-bit counter {candidates so far, arrivals << 32}
};
static_assert(sizeof(UnitCtl) == 64, "UnitCtl is one 64-byte record");

enum KernelId {
    KID_INIT = 0,
    KID_SCORE,
    KID_CAND,
    KID_ATTEND,
    KID_COMPACT,
    KID_DENSE,
    KID_ATTEND_ROWS,
    KID_LABEL,
    KID_GATHER_HOST,
    KID_PROBE,
    KID_REFINE_ATTEND,
    KID_APPEND_KV,
    KID_Q4_AMAX,
    KID_Q4_WRITE,
    KID_PREDICT,
    KID_COUNT
};

// Launch plan of one sparse decode / select call and its workspace layout.
struct Plan {
    int units, G, k_eff;
    int cus;             // compute units of the device the plan was made for
    int sc_chunk, n_sc;  // tokens per workgroup / workgroups per unit, scoring
    int ch, n_ch;        // same for candidate collection, compaction and attention
    int key_stride;      // uint32 keys per unit (L rounded up to 4)
    bool refine_attend;  // ds_sparse_decode as scoring + one refine-and-attend launch
    bool group_scores_itself;  // query groups of 3+ heads: chunks sized so that this launch can do the scoring too
    int unit_groups;     // the attention launch that scores as well is enqueued this many times, a share of the units each
    size_t off_ctl, off_hist, off_coarse, off_keys, off_cand, off_ndef, off_offs, off_part;
    size_t total;
};
// Plan of dense / gathered-rows attention (token chunks of dn_chunk).
struct DensePlan {
    int units, G;
    int ch, n_ch;
    size_t off_ctl, off_part, total;  // same control prefix as Plan
};

// Where the approximate scores come from: the fp16 label cache, the K rows themselves (no label
// cache), or the 4-bit label cache (packed codes + per-channel amax).
enum ScoreSrcKind { SRC_LABEL = 0, SRC_K_ROWS = 1, SRC_Q4 = 2 };
struct ScoreSrc {
    ScoreSrcKind kind = SRC_LABEL;
    const float *amax = nullptr;  // SRC_Q4: [units][r]
};

// What the launch plans need to know of the device: compute units, the dies (XCDs) that workgroups
// are dealt out to in turn, and LDS bytes per compute unit.  Taken from the current device, or the
// figures of an MI355X when no device is visible (a plan made on a host without one).
struct DeviceCaps {
    int cus = 256, xccs = 8, lds_per_cu = 160 << 10;
};
DeviceCaps device_caps();                  // of the current device (cached per device)
void device_caps_pretend(const DeviceCaps *caps);  // test hook: overrides device_caps() for this thread (nullptr: off)

// What the plan is for: the split select call (and anything that runs the candidate launch), a
// decode call, or a decode call whose attention launch may do the scoring as well.
enum PlanFor { PLAN_SELECT = 0, PLAN_DECODE = 1, PLAN_DECODE_SCORING = 2 };
bool make_plan(const ds_shape_t &s, Plan *p, PlanFor purpose = PLAN_SELECT);
bool make_dense_plan(const ds_shape_t &s, int n_tokens, DensePlan *p);

// Per-kernel timing: while it is on, prof_events hands out a start and a stop event for one
// launch of kernel `id` (false when it is off or no event could be made) and remembers the pair.
bool prof_events(int id, hipEvent_t *start, hipEvent_t *stop);

// launchers: enqueue only; return the launch error (hipSuccess if fine)
hipError_t launch_init(void *ws, size_t bytes, hipStream_t st);
hipError_t launch_score(const void *q, const void *label, const int32_t *channels, void *ws,
                        const Plan &p, const ds_shape_t &s, bool tail_refine, bool want_offsets,
                        hipStream_t st, ScoreSrc src = ScoreSrc());
hipError_t launch_cand(void *ws, const Plan &p, const ds_shape_t &s, bool want_offsets,
                       hipStream_t st);
hipError_t launch_compact(void *ws, int32_t *idx_out, const Plan &p, const ds_shape_t &s,
                          hipStream_t st);
hipError_t launch_attend_sparse(const void *q, const void *K, const void *V, void *ws, float *out,
                                int32_t *idx_out, const Plan &p, const ds_shape_t &s,
                                hipStream_t st, int kv_stride = kD);
bool refine_attend_ok(const Plan &p, bool scores_itself);
// Returned by launch_refine_attend (nothing enqueued) when the launch would wait for workgroups
// that the device cannot hold at the same time as the waiting ones.
constexpr hipError_t kNotResident = hipErrorLaunchOutOfResources;
bool refine_attend_fits(const Plan &p, const ds_shape_t &s, bool scores_itself, bool q4);
hipError_t launch_refine_attend(const void *q, const void *K, const void *V, void *ws, float *out,
                                int32_t *idx_out, const Plan &p, const ds_shape_t &s, hipStream_t st,
                                int kv_stride = kD, const void *score_label = nullptr,
                                const int32_t *score_channels = nullptr, const float *score_amax = nullptr);
hipError_t launch_attend_dense(const void *q, const void *K, const void *V, void *ws, float *out,
                               const DensePlan &p, const ds_shape_t &s, hipStream_t st);
hipError_t launch_attend_rows(const void *q, const void *KV_rows, void *ws, float *out,
                              const DensePlan &p, const ds_shape_t &s, int n_rows, hipStream_t st);
hipError_t launch_label(const void *K, const int32_t *channels, void *label, const ds_shape_t &s,
                        int t0, int n, hipStream_t st, int kv_stride = kD);
hipError_t launch_q4_amax(const void *K, const int32_t *channels, float *amax, const ds_shape_t &s,
                          hipStream_t st);
hipError_t launch_q4_write(const void *K, const int32_t *channels, const float *amax, void *codes,
                           const ds_shape_t &s, int t0, int n, hipStream_t st);
hipError_t launch_predict_query(const void *x, const void *Wq, void *q_out, int B, int Dm, int N,
                                hipStream_t st);
hipError_t launch_append_kv(const void *k_new, const void *v_new, void *K, void *V,
                            const int32_t *channels, void *label, const ds_shape_t &s, int t0, int n,
                            int kv_stride, hipStream_t st);
hipError_t launch_gather_host(const void *Kh, const void *Vh, const int32_t *idx, void *rows,
                              const ds_shape_t &s, hipStream_t st);
hipError_t launch_probe(const void *src, size_t bytes, uint32_t *sink, hipStream_t st);

int tune_get(int knob);

}  // namespace ds

// Launches a kernel.  While per-kernel timing is on, the dispatch itself carries the start and
// stop events, so the interval is the kernel's own begin-to-end time without the launch latency
// that events recorded around the launch would add.
#define DS_LAUNCH(kid, kernel, grid, block, shmem, st, ...)                                          \
    do {                                                                                             \
        hipEvent_t ds_ev_a_ = nullptr, ds_ev_b_ = nullptr;                                           \
        if (ds::prof_events((kid), &ds_ev_a_, &ds_ev_b_))                                            \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, st, ds_ev_a_, ds_ev_b_, 0, __VA_ARGS__); \
        else                                                                                         \
            hipLaunchKernelGGL(kernel, grid, block, shmem, st, __VA_ARGS__);                         \
    } while (0)
