/*
 * ds_attn.h -- C ABI of libdsattn: Double Sparsity decode attention on gfx950.
 *
 * The decode step of "Post-Training Sparse Attention with Double Sparsity"
 * (Algorithm 1): for every (batch, KV head) unit
 *   1. gather the r calibrated channels of the query and score every cached
 *      token against the label cache (the same r channels of K),
 *   2. keep the k best-scoring tokens,
 *   3. gather those k full K and V rows,
 *   4. run exact softmax attention over them.
 *
 * General conventions
 *   - fp16 means IEEE binary16 stored as 2 bytes; all arithmetic accumulates in
 *     binary32.  d (head dimension) must be 128.
 *   - A "unit" is one (batch b, KV head h); query head hq uses KV head hq / G,
 *     G = Hq / Hkv (G = 1 is multi-head attention, G > 1 grouped-query).
 *   - Layouts are dense row-major:
 *       q        [B, Hq, d]           fp16
 *       K, V     [B, Hkv, L_max, d]   fp16   one token = one 256-byte row
 *       label    [B, Hkv, L_max, r]   fp16
 *       channels [Hkv, r]             int32  distinct, in [0, d); shared over batch
 *       out      [B, Hq, d]           fp32
 *       idx      [B, Hkv, k]          int32
 *     Tokens [0, L) are valid; L_max is the allocated token count (row stride).
 *   - Ownership: the caller owns every buffer.  The library allocates and frees
 *     no device memory and keeps no pointer after a call returns.  Scratch comes
 *     from a caller-provided workspace of ds_workspace_bytes() bytes.  The
 *     workspace carries a few counters that every call leaves at zero again, so
 *     it must be cleared once with ds_workspace_init() after allocation, must
 *     not be written by the caller, and must be cleared again before it is used
 *     with a different shape, after a call that returned DS_ERR_HIP or after a
 *     call whose output came back as NaN (see ds_workspace_errors).  Two calls
 *     that overlap in time must not share a workspace, and a decode call expects
 *     the device to itself while it runs.
 *   - Device entry points only enqueue work on `stream` (a hipStream_t passed
 *     as void*, NULL = the null stream) and return without synchronising.
 *     DS_OK means "validated and enqueued".
 *   - Errors: every entry point returns a ds_status_t and never throws or
 *     aborts.  On any error nothing is enqueued and no output is touched.
 *     NULL required pointer -> DS_ERR_NULL.  d != 128, Hq % Hkv != 0,
 *     r outside [1, d], k < 1, L < 1, L > L_max, B/Hq/Hkv < 1 -> DS_ERR_SHAPE.
 *     Misaligned base pointer -> DS_ERR_ALIGN (K, V: 256 bytes; label, q, out,
 *     idx, workspace: 16 bytes).  Workspace too small -> DS_ERR_WORKSPACE.
 *     A failed launch -> DS_ERR_HIP.  k > L is not an error: k_eff = min(k, L).
 *   - Inputs must be finite; behaviour on NaN/Inf is unspecified.
 *   - Results are bit-identical from run to run for the same inputs and shape.
 */
#ifndef DS_ATTN_H
#define DS_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DS_OK = 0,
    DS_ERR_NULL = -1,
    DS_ERR_SHAPE = -2,
    DS_ERR_ALIGN = -3,
    DS_ERR_WORKSPACE = -4,
    DS_ERR_UNSUPPORTED = -5,
    DS_ERR_HIP = -6
} ds_status_t;

/* Which statistic ranks the channels (the q / k / qk outlier variants of the
 * paper's outlier-type ablation, Table 3). */
typedef enum { DS_CALIB_Q = 0, DS_CALIB_K = 1, DS_CALIB_QK = 2 } ds_calib_mode_t;

typedef struct {
    int32_t B, Hq, Hkv, d; /* batch, query heads, KV heads, head dim (=128)      */
    int32_t L, L_max;      /* valid tokens, allocated tokens                      */
    int32_t r, k;          /* label channels (alpha*d), selected tokens (beta*S)  */
} ds_shape_t;

/* Static string for a status code (never NULL). */
const char *ds_strerror(ds_status_t status);
/* Library version, major*10000 + minor*100 + patch. */
int ds_version(void);

/*
 * Offline calibration (Sec. 4.1).  HOST pointers, synchronous, CPU only.
 * The attention logit is a sum over channels, A = sum_c q_c k_c; the channels
 * whose terms are largest in magnitude over a calibration set are kept.
 *   q_calib [N, Hq, d] fp16, k_calib [N, Hkv, d] fp16 : N sample rows.
 *   mode Q : importance(h, c) = mean over samples and the group's query heads of |q_c|
 *   mode K : importance(h, c) = mean over samples of |k_c|
 *   mode QK: product of the two (= mean |q_c k_c| over all query/key pairs).
 *   channels_out [Hkv, r]: the r most important channels of each KV head in
 *   ascending channel order; equal importance keeps the lower channel.
 * Errors: DS_ERR_NULL, DS_ERR_SHAPE (N < 1, r outside [1, d], d < 1,
 * Hq % Hkv != 0, bad mode).  d is not restricted to 128 here.
 */
ds_status_t ds_calibrate_channels(const uint16_t *q_calib, const uint16_t *k_calib,
                                  int32_t N, int32_t Hq, int32_t Hkv, int32_t d,
                                  int32_t r, ds_calib_mode_t mode,
                                  int32_t *channels_out);

/*
 * Label cache maintenance (Sec. 4.2).  DEVICE pointers.
 *   label[b, h, t, j] = K[b, h, t, channels[h, j]]   (bit copy)
 * ds_build_label writes tokens [0, L) (prefill); ds_append_label writes tokens
 * [t0, t0 + n_new) (decode: call it after the new token's K row is in the cache
 * and before ds_sparse_decode; L then counts the new token).
 * Uses shape->{B, Hkv, d, L, L_max, r}; ds_append_label ignores L and needs
 * 0 <= t0, n_new >= 0, t0 + n_new <= L_max (else DS_ERR_SHAPE).
 */
ds_status_t ds_build_label(const void *K, const int32_t *channels, void *label,
                           const ds_shape_t *shape, void *stream);
ds_status_t ds_append_label(const void *K, const int32_t *channels, void *label,
                            const ds_shape_t *shape, int32_t t0, int32_t n_new,
                            void *stream);

/*
 * K/V cache layouts.  DS_KV_SPLIT: K and V are separate [B, Hkv, L_max, d]
 * arrays (the layout of every call above and below unless it says otherwise).
 * DS_KV_INTERLEAVED: one array KV [B, Hkv, L_max, 2, d] in which a token's K
 * row is followed by its V row, so that the decode gathers one 512-byte piece
 * per selected token instead of two 256-byte rows (Sec. 5.3: the cost of the
 * path is the gather of the selected rows).  KV base 256-byte aligned;
 * L_max * 512 must fit 32 bits.
 */
typedef enum { DS_KV_SPLIT = 0, DS_KV_INTERLEAVED = 1 } ds_kv_layout_t;

/*
 * Decode-step cache maintenance in one launch (Sec. 4.2: a decode step extends
 * the label cache by the new tokens' r selected channels only).  Writes the n_new new tokens' rows k_new, v_new [B, Hkv, n_new, d]
 * fp16 (device, 16-byte aligned) into the caches at tokens [t0, t0 + n_new) and
 * label[b, h, t0 + i, j] = k_new[b, h, i, channels[h, j]].  With
 * DS_KV_INTERLEAVED pass the KV array as K; V is ignored.  Uses
 * shape->{B, Hkv, d, L_max, r}; t0 + n_new <= L_max.  Equal to copying the rows
 * and calling ds_append_label.
 */
ds_status_t ds_append_kv(const void *k_new, const void *v_new, void *K, void *V,
                         const int32_t *channels, void *label, const ds_shape_t *shape,
                         int32_t t0, int32_t n_new, ds_kv_layout_t layout, void *stream);
/* ds_build_label for an interleaved cache KV [B, Hkv, L_max, 2, d]. */
ds_status_t ds_build_label_kv(const void *KV, const int32_t *channels, void *label,
                              const ds_shape_t *shape, void *stream);

/*
 * Label cache kept in 4 bits (Sec. 4.2 says the label cache can be stored in
 * 4-bit and gives no quantiser; this one is symmetric with one step per batch
 * entry, KV head and label channel, fixed when the cache is built):
 *   amax[b, h, j]  = max over t < L of |K[b, h, t, channels[h, j]]|
 *   code[t, j]     = clamp(rint(K[t, channels[j]] * (7 / amax[j])), -8, 7)
 *                    (binary32 product of the binary32 quotient, half to even)
 *   label value    = code * (amax / 7)
 * label_q4 [B, Hkv, L_max, ceil(r/8)] uint32: channel j of a token is the
 * two's-complement nibble in bits [4 (j mod 8), +4) of the token's word j / 8,
 * nibbles past r are zero; amax [B, Hkv, r] fp32.  DEVICE pointers.
 * ds_build_label_q4 computes amax over tokens [0, L) and codes them;
 * ds_append_label_q4 codes tokens [t0, t0 + n_new) with the amax given (values
 * beyond it saturate).  Argument checks as ds_build_label / ds_append_label.
 */
ds_status_t ds_build_label_q4(const void *K, const int32_t *channels, void *label_q4,
                              float *amax, const ds_shape_t *shape, void *stream);
ds_status_t ds_append_label_q4(const void *K, const int32_t *channels, void *label_q4,
                               const float *amax, const ds_shape_t *shape, int32_t t0,
                               int32_t n_new, void *stream);

/* Bytes of workspace any decode/select/attend call with this shape needs
 * (a multiple of 256).  Pure host function; 0 if the shape is invalid. */
size_t ds_workspace_bytes(const ds_shape_t *shape);
/* Enqueues the clearing of a freshly allocated workspace (all workspace_bytes,
 * a multiple of 16).  Required once before the first call that uses it: the
 * clearing must have completed, or be ordered on the same stream, before that
 * call runs.  A call on a workspace that was not cleared gives wrong results
 * (out-of-range counters are caught where they would index memory). */
ds_status_t ds_workspace_init(void *workspace, size_t workspace_bytes, void *stream);
/* Waits for `stream` and reads back the per-unit error words of the workspace
 * (DEVICE pointer) for this shape.  Inside a launch a workgroup sometimes waits
 * for another workgroup of its unit (Algorithm 1 steps 2-5 done in one launch).
 * The library only enqueues such a launch when the occupancy that the runtime
 * reports for the kernel holds all the workgroups that wait for each other at the
 * same time (otherwise it takes launch shapes that need less, down to three
 * launches that need nothing); that figure assumes that the decode call has the
 * device to itself -- kernels of other streams or processes that occupy compute
 * units while it runs can keep workgroups from starting.  Every wait is therefore
 * bounded as well: a workgroup whose wait runs out raises its unit's error word
 * and carries on without the value it waited for, the launch always ends, and
 * that unit's rows of `out` are written as NaN instead of a wrong result.  The
 * word stays set until ds_workspace_init(): later calls on the workspace write
 * NaN for that unit again without computing it, so the failure cannot pass
 * unnoticed by a caller that never asks here.  *n_failed = units whose word is
 * set, *first_code = the first such word (which wait it was; 0 if none); either
 * pointer may be NULL.  DS_OK when the words could be read (whatever they say),
 * DS_ERR_HIP when the copy failed.  Synchronises: not for the hot path. */
ds_status_t ds_workspace_errors(const void *workspace, size_t workspace_bytes,
                                const ds_shape_t *shape, void *stream,
                                int32_t *n_failed, int32_t *first_code);

/*
 * Double Sparsity decode (Algorithm 1), all four steps.  DEVICE pointers.
 *   s_hat[t] = sum_{g in group} sum_j q_g[channels[j]] * label[t, j]   (no scale)
 *   I        = the k_eff tokens with the largest s_hat; equal scores keep the
 *              lower token index (-0 and +0 are equal)
 *   out[hq]  = softmax(q_hq . K[I,:]^T / sqrt(d)) . V[I,:]   for each head of the group
 * The selection is taken on binary32 scores accumulated as fma over j ascending
 * from 0, with the group's label queries summed first (g ascending).
 * idx_out may be NULL; otherwise it receives I in ascending token order in
 * idx_out[b, h, 0 .. k_eff) and -1 in [k_eff, k).
 */
ds_status_t ds_sparse_decode(const void *q, const void *label, const void *K,
                             const void *V, const int32_t *channels, float *out,
                             int32_t *idx_out, void *workspace,
                             size_t workspace_bytes, const ds_shape_t *shape,
                             void *stream);

/*
 * ds_sparse_decode for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The scratch is a device array inside the library
 * (ds_static_scratch_bytes() = 32 MiB, held once per GPU for the life of the
 * process); this call allocates and frees nothing, and neither does anything it
 * calls.  Same arguments, results (bit for bit) and errors as ds_sparse_decode,
 * minus the workspace; a shape whose scratch layout exceeds the array is refused
 * with DS_ERR_WORKSPACE and nothing is enqueued (the headline shape B = 1, 32
 * heads, L = 65536 needs 25 MiB; 12 bytes per cached token of all units plus
 * 20 KiB per unit is a safe estimate).  Every call first clears the control part
 * of the scratch with a fill kernel on `stream`, so calls of different shapes may
 * follow each other.  All calls on one GPU share the one array: calls that overlap
 * in time on the same GPU (different streams, different threads) race and give
 * wrong results; serialise them.  ds_static_init() resolves the array's address
 * on the current device ahead of time (optional; the first call does it
 * otherwise); call it once per device before capturing.
 */
size_t ds_static_scratch_bytes(void);
ds_status_t ds_static_init(void);
ds_status_t ds_sparse_decode_static(const void *q, const void *label, const void *K,
                                    const void *V, const int32_t *channels, float *out,
                                    int32_t *idx_out, const ds_shape_t *shape,
                                    void *stream);

/*
 * The same decode without a label cache (Sec. 4.2 and the appendix ablation
 * "Forward without Label Cache"): s_hat[t] is formed from K[t, channels[j]] read
 * out of the 256-byte K rows, the strided access the label cache removes.  Same
 * arithmetic as ds_sparse_decode, hence the same selection and output for a
 * label cache that matches K; it exists to measure what the label cache buys.
 * Arguments as ds_sparse_decode, minus label.
 */
ds_status_t ds_sparse_decode_nolabel(const void *q, const void *K, const void *V,
                                     const int32_t *channels, float *out,
                                     int32_t *idx_out, void *workspace,
                                     size_t workspace_bytes, const ds_shape_t *shape,
                                     void *stream);

/*
 * ds_sparse_decode with the approximate scores taken from the 4-bit label cache:
 *   s_hat[t] = sum_j w[j] * code[t, j],  w[j] = (sum_{g in group} q_g[channels[j]]) * (amax[j] / 7)
 * in binary32 (g ascending, then fma over j ascending from 0); steps 3-5 of
 * Algorithm 1 are unchanged (exact attention over the k selected fp16 rows).
 */
ds_status_t ds_sparse_decode_q4(const void *q, const void *label_q4, const float *amax,
                                const void *K, const void *V, const int32_t *channels,
                                float *out, int32_t *idx_out, void *workspace,
                                size_t workspace_bytes, const ds_shape_t *shape,
                                void *stream);

/* ds_sparse_decode over an interleaved cache KV [B, Hkv, L_max, 2, d]
 * (DS_KV_INTERLEAVED); everything else as ds_sparse_decode. */
ds_status_t ds_sparse_decode_kv(const void *q, const void *label, const void *KV,
                                const int32_t *channels, float *out, int32_t *idx_out,
                                void *workspace, size_t workspace_bytes,
                                const ds_shape_t *shape, void *stream);

/*
 * Dense decode attention over all L tokens (Sec. 2.1), the in-library
 * comparison point:  out[hq] = softmax(q_hq . K^T / sqrt(d)) . V.
 * Uses shape->{B, Hq, Hkv, d, L, L_max}; r and k are ignored.
 */
ds_status_t ds_dense_decode(const void *q, const void *K, const void *V, float *out,
                            void *workspace, size_t workspace_bytes,
                            const ds_shape_t *shape, void *stream);

/*
 * Query prediction of the offload schedule (Sec. 5.1): a layer's input
 * embedding is passed through the NEXT layer's query projection to get an
 * approximate query for that layer, whose selected rows can then be fetched
 * while the current layer still computes.
 *   q_out[b, n] = sum_m Wq[n, m] * x[b, m]
 * x [B, Dm] fp16, Wq [N, Dm] fp16 (row n = output feature n; N = Hq * d gives
 * q_out the [B, Hq, d] layout of the decode calls), q_out [B, N] fp16.  DEVICE
 * pointers; x and Wq 16-byte aligned; Dm a multiple of 8, at most 8192.
 * Products are exact, sums are binary32 in a fixed order, one rounding to fp16.
 * (Positional encoding and normalisation belong to the model around this call.)
 */
ds_status_t ds_predict_query(const void *x, const void *Wq, void *q_out, int32_t B,
                             int32_t Dm, int32_t N, void *stream);

/*
 * Split entry points for the offload arrangement (Sec. 5.1: label cache on the
 * GPU, full K/V in host memory, only the selected rows fetched).
 * ds_select      = steps 1-2 of Algorithm 1; idx_out (required) as above.
 * ds_gather_rows_host copies the selected rows: K_host, V_host are pinned host
 *                  buffers [B, Hkv, L_max, d] addressable from the device;
 *                  KV_rows (device) is [B, Hkv, k, 2, d]: row i holds K[idx[i]]
 *                  then V[idx[i]].  Rows with idx < 0 are zero-filled.
 * ds_attend_rows = steps 4-5 over gathered rows; n_rows_per_unit = k_eff is
 *                  taken from shape (min(k, L)).
 */
ds_status_t ds_select(const void *q, const void *label, const int32_t *channels,
                      int32_t *idx_out, void *workspace, size_t workspace_bytes,
                      const ds_shape_t *shape, void *stream);
ds_status_t ds_gather_rows_host(const void *K_host, const void *V_host,
                                const int32_t *idx, void *KV_rows,
                                const ds_shape_t *shape, void *stream);
ds_status_t ds_attend_rows(const void *q, const void *KV_rows, float *out,
                           void *workspace, size_t workspace_bytes,
                           const ds_shape_t *shape, void *stream);

/*
 * Measurement aids (not part of the method).
 * ds_probe_stream_read: one pass of plain 16-byte loads over `bytes` bytes of
 *   device memory (bytes % 16 == 0), xor-folded into sink[0..1023] (uint32,
 *   device) so the loads cannot be dropped: the read-bandwidth ceiling of the
 *   device as seen by a kernel of this library.
 * Per-kernel timing: while enabled, every kernel the library launches is
 *   bracketed by HIP events on its stream.  ds_profile_read synchronises the
 *   recorded events of kernel `id` and returns their summed duration and count
 *   since the last reset.  ids run from 0 to ds_profile_kernel_count() - 1.
 *   Enabling it perturbs end-to-end timing; leave it off when timing whole calls.
 */
ds_status_t ds_probe_stream_read(const void *src, size_t bytes, uint32_t *sink,
                                 void *stream);
int ds_profile_kernel_count(void);
const char *ds_profile_kernel_name(int id);
ds_status_t ds_profile_enable(int on);
ds_status_t ds_profile_reset(void);
ds_status_t ds_profile_read(int id, double *total_ms, int64_t *launches);

/*
 * Launch-shape knobs, for sweeps (defaults are chosen from the shape):
 *   knob 0: tokens per workgroup in the scoring kernel   (0 = automatic; multiple of 256)
 *   knob 1: tokens per workgroup in select/attend        (0 = automatic; multiple of 64, <= 16384;
 *           the candidate launch of shape 1 and ds_select take up to 6144)
 *   knob 2: tokens per workgroup in dense/rows attention (0 = automatic; multiple of 16)
 *   knob 3: how ds_sparse_decode is launched: 0 = automatic (4 for units of more than 8K
 *           tokens -- more than 4K when the attention launch can score as well, see knob 4 --
 *           and for units short enough for one workgroup each: up to 4K tokens, up to 8K when
 *           there are 256 units or more; else 1), 1 = three launches
 *           (score, candidates, attend), 4 = scoring (keys and threshold bin), then one launch
 *           in which a unit's workgroups attend the rows above the threshold bin while the last
 *           of them to have listed its candidates settles the exact threshold for the rest
 *           (one launch in all when that launch can score as well, see knob 4)
 *   knob 4: where the exact top-k threshold is settled on the three-launch path: 0 = automatic
 *           (in the scoring launch for units of up to 8K tokens), 1 = always in a separate
 *           candidate launch, 2 = always in the scoring launch.  On launch shape 4 with a label
 *           cache of 8 or 16 fp16 channels, or a 4-bit one of up to 16 channels whose token
 *           rows 16-byte loads can take (L_max a multiple of 4, of 2 above 8 channels), the
 *           attention launch can do the scoring as well (one launch in all): 0 = when a unit
 *           has one workgroup, or the whole grid is resident at once (single heads and pairs:
 *           up to 1024 workgroups; larger query groups: chunks sized for it when that fits);
 *           1 = never; 2 = always
 *   knob 5: launch shape 4: polls after which a workgroup's wait for another workgroup gives
 *           up (0 = the default of 2^21, far beyond any wait that ends; small values are for
 *           testing the give-up path: see ds_workspace_errors)
 * DS_ERR_SHAPE for a knob or value the kernels cannot run with.  Process-wide;
 * changing a knob changes ds_workspace_bytes() and the workspace layout, so
 * re-query the size and clear the workspace again afterwards.
 */
ds_status_t ds_tune_set(int knob, int value);
int ds_tune_get(int knob);

/*
 * How ds_sparse_decode would be launched for a shape (diagnostics and tests; pure host work
 * apart from asking the runtime for the kernel's occupancy).  label_kind: 0 = fp16 label cache,
 * 1 = no label cache, 2 = 4-bit label cache.  out[0] = launches by the planner's own model of the
 * device (with out[6] = 1: launches that score, select and attend, one as a rule, two to four
 * of a share of the units each when the units do not fit the device at once; otherwise 2:
 * scoring, then selection behind the attention; 3: scoring, candidates, attention); out[1] =
 * launches once the occupancy that the
 * runtime reports for the kernels has been taken into account (-1 when no device is visible);
 * out[2] = tokens per workgroup, out[3] = workgroups per unit, out[4] = workgroups of the
 * attention launches together, out[5] = compute units planned for, out[6] = 1 if the attention launch
 * scores as well, out[7] = query heads per KV head.
 * ds_pretend_device makes the calling thread's plans (and residency checks) assume a device of
 * `cus` compute units on `xccs` dies with `lds_per_cu` bytes of LDS each, instead of the current
 * one; (0, 0, 0) ends it.  The workspace layout follows the plan: query ds_workspace_bytes() and
 * clear the workspace again after switching.  DS_ERR_SHAPE for cus < 1, xccs < 1, cus not a
 * multiple of xccs, or less than 64 KiB of LDS.
 */
ds_status_t ds_plan_describe(const ds_shape_t *shape, int32_t label_kind, int32_t out[8]);
ds_status_t ds_pretend_device(int32_t cus, int32_t xccs, int32_t lds_per_cu);

#ifdef __cplusplus
}
#endif
#endif /* DS_ATTN_H */
