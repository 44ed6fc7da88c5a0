/* preserve.h - C ABI of the MI355X request-load-predictor + load-anticipator library.
 *
 * The library implements the per-request hot path of PreServe's prediction-based management:
 *   - the request load predictor (paper Sec. 3.3 "Tier-2: Request Load Prediction"): prompt
 *     token ids -> predicted number of response tokens, by a DistilBERT-shaped encoder whose
 *     [CLS] state feeds a two-layer regression head, with M learnable prompt vectors appended
 *     to the text tokens;
 *   - the instance load anticipator (paper Sec. 3.4.1 "Instance Load Anticipator"): per-request
 *     predictions -> per-instance future-load curves, updated per request.
 *
 * Conventions
 *   - Every array argument is a DEVICE pointer unless marked "host".  The caller owns every
 *     buffer it passes in, including workspaces; the library allocates device memory only in
 *     ps_model_load() and releases it in ps_model_free().
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and return without synchronising.  Outputs of one call may be passed to the
 *     next call on the same stream (pred_tokens of ps_predict_load -> ps_anticipate).
 *   - Return value: PS_OK or a negative PS_E* code for faults the host can see.  Faults only
 *     visible in device data are recorded in a caller-provided ps_status block (below).
 *   - One model may be used from one stream at a time; calls sharing a workspace must be
 *     ordered by the caller.
 */
#ifndef PRESERVE_H
#define PRESERVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PS_OK            0
#define PS_EINVAL       -1   /* null pointer, negative size, inconsistent arguments          */
#define PS_EIO          -2   /* model file cannot be read                                    */
#define PS_EFORMAT      -3   /* model file header or size is wrong                           */
#define PS_ENOMEM       -4   /* host or device allocation failed                             */
#define PS_EWORKSPACE   -5   /* workspace too small or misaligned (256 B)                    */
#define PS_EUNSUPPORTED -6   /* shape outside what the kernels are built for                 */
#define PS_EHIP         -7   /* a HIP runtime call failed                                    */

/* Device-side fault record.  The caller zeroes it (device memory, 16 bytes, 8-byte aligned)
 * before a call or a series of calls and reads it back with ps_status_read().  `flags` is the
 * OR of PS_ST_* bits.  `first_bad`, as ps_status_read() returns it, is the smallest request /
 * record index that raised one, or -1 if none carried an index; in device memory the field
 * holds an encoding of it that only ps_status_read() interprets. */
typedef struct ps_status {
    int32_t flags;
    int32_t reserved;
    int64_t first_bad;
} ps_status;

#define PS_ST_BAD_TOKEN    0x01  /* token id outside [0, vocab)                               */
#define PS_ST_BAD_LENGTH   0x02  /* request length < 1, > its span, or + n_soft > max_pos; a span
                                    outside [0, n_tokens]; or overlapping spans that together need
                                    more rows than n_tokens token slots can (the requests from the
                                    first one that does not fit onwards)                      */
#define PS_ST_NAN          0x04  /* a prediction is NaN                                       */
#define PS_ST_BAD_RECORD   0x10  /* anticipator or look-ahead record skipped: pred_tokens < 0 or > PS_MAX_PRED,
                                    instance outside [0, n_inst), arrival outside [0, horizon),
                                    or rate[instance] < 1                                     */
#define PS_ST_RANGE        0x20  /* a load bucket left the int32 range (its low 32 bits are stored),
                                    or a workgroup folded so many tokens (2^27 per wavefront)
                                    that it cannot rule that out                              */

#define PS_MAX_PRED  65535       /* largest pred_tokens value ps_anticipate accepts           */

typedef struct ps_model ps_model;   /* opaque; owns the device copy of the weights */

typedef struct ps_model_info {
    int32_t layers, hidden, heads, ffn, vocab, max_pos, n_soft, head_hidden;
    int32_t dtype;     /* 0 = fp32 weights and arithmetic, 1 = bf16 storage / fp32 accumulate */
    int32_t d_max;     /* predictions are clamped to [0, d_max] tokens                        */
} ps_model_info;

/* Load a predictor (Sec. 3.3) from `path` (host string; file layout: 64-byte header, then the
 * tensors in a fixed order, see the package's workload module) onto HIP device `device`.
 * On success *out owns the device weights.  Errors: PS_EINVAL, PS_EIO, PS_EFORMAT, PS_ENOMEM,
 * PS_EUNSUPPORTED (bf16 models need hidden % 256 == 0, ffn % 256 == 0 and head size 64),
 * PS_EHIP. */
int ps_model_load(const char* path /*host*/, int device, ps_model** out /*host*/);

/* Release a model and its device memory.  NULL is allowed. */
void ps_model_free(ps_model* model);

/* Copy the model's shape into *out (host). */
int ps_model_get_info(const ps_model* model, ps_model_info* out /*host*/);

/* Bytes of device workspace ps_predict_load() needs for calls with at most `max_tokens` token
 * slots (n_tokens below) and `max_req` requests.  0 on invalid arguments or a size ps_predict_load()
 * refuses. */
size_t ps_workspace_bytes(const ps_model* model, int64_t max_tokens, int32_t max_req);

/* Predict the response length of n_req requests (Sec. 3.3).
 *   token_ids   [n_tokens] int32; request r's text tokens start at offsets[r]; the caller puts
 *               the [CLS] id first: the state of a request's first token is what is pooled.
 *   offsets     [n_req + 1] int32, non-decreasing, offsets[n_req] == n_tokens.  Checked on the device: a
 *               request whose span breaks this is faulty (PS_ST_BAD_LENGTH), nothing is read out of bounds.
 *   lengths     NULL: packed layout, request r has offsets[r+1] - offsets[r] tokens.
 *               else [n_req]: padded layout, request r has lengths[r] valid tokens at the start
 *               of its span; the rest of the span is padding and takes no part in anything.
 *   n_tokens    host scalar, number of token slots (= offsets[n_req]).
 *   pred_f      [n_req] float, out: raw regression output (NaN for a faulty request).
 *   pred_tokens [n_req] int32, out: pred_f rounded half-to-even and clamped to [0, d_max]
 *               (-1 for a faulty request).
 *   workspace   device scratch of at least ps_workspace_bytes(model, n_tokens, n_req) bytes,
 *               256-byte aligned; contents are undefined before and after.
 *   status      device ps_status or NULL; see above.  A request with a fault gets NaN / -1 and
 *               does not disturb the others.
 * Every request is processed with the model's n_soft learnable prompt rows appended after its
 * text tokens.  n_req == 0 is allowed and does nothing.
 * Errors: PS_EINVAL (null pointers, negative sizes), PS_EWORKSPACE (too small or misaligned),
 * PS_EUNSUPPORTED (n_tokens + n_req * (n_soft + 8) above 2^27 activation rows), PS_EHIP. */
int ps_predict_load(ps_model* model, const int32_t* token_ids, const int32_t* offsets,
                    const int32_t* lengths, int32_t n_req, int64_t n_tokens,
                    float* pred_f, int32_t* pred_tokens,
                    void* workspace, size_t workspace_bytes, ps_status* status, void* hip_stream);

/* Bytes of device workspace ps_anticipate() needs (partial curves of its workgroups, for both of its
 * first kernels).  0 on invalid arguments. */
size_t ps_anticipate_workspace_bytes(int64_t n_req, int32_t n_inst, int32_t horizon);

/* Fold n_req predictions into the per-instance future-load curves (Sec. 3.4.1: the look-ahead
 * map is updated per request from its predicted response length).  Request r, assigned to
 * instance_id[r] and arriving in one-second bucket arrival_bucket[r], decodes pred_tokens[r]
 * tokens over `dur` consecutive buckets from its arrival bucket, spread as evenly as integers
 * allow (the first pred % dur buckets take one more):
 *     rate == NULL : dur = horizon - arrival          (spread to the end of the horizon)
 *     otherwise    : dur = ceil(pred / rate[instance]) (rate[k] = tokens/s instance k decodes)
 *   load      [n_inst * horizon] int32, row-major [instance][bucket]; ACCUMULATED into: the map
 *             is persistent, the caller zeroes it to start afresh.
 *   overflow  [n_inst] int64, accumulated: tokens that fall at or after `horizon`.  May be NULL
 *             only if rate == NULL (nothing can overflow then).
 *   Records may come in any order and the result does not depend on it.  Long streams (262144 records
 *   or more, rate given, horizon <= 4096) whose records are in arrival order (non-decreasing
 *   arrival_bucket, as in a request log) are folded by a cheaper kernel; if a record turns out to lie
 *   outside the bucket window of its part of the stream, the general kernel redoes the call.
 *   workspace at least ps_anticipate_workspace_bytes(n_req, n_inst, horizon) bytes, 256-byte
 *             aligned.
 *   status    device ps_status or NULL.  Faulty records are skipped (PS_ST_BAD_RECORD).
 * Integer arithmetic throughout: the result does not depend on record order and is bit-exact.
 * pred_tokens, instance_id and arrival_bucket must be 16-byte aligned (PS_EINVAL otherwise).
 * Errors: PS_EINVAL, PS_EWORKSPACE, PS_EUNSUPPORTED (horizon above 65535, or too long for one row
 * of the map to fit a compute unit's local memory), PS_EHIP.  n_req == 0 is allowed. */
int ps_anticipate(const int32_t* pred_tokens, const int32_t* instance_id,
                  const int32_t* arrival_bucket, const int32_t* rate,
                  int64_t n_req, int32_t n_inst, int32_t horizon,
                  int32_t* load, int64_t* overflow,
                  void* workspace, size_t workspace_bytes, ps_status* status, void* hip_stream);

/* ps_anticipate() for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result and errors as
 * ps_anticipate() without `workspace`: the partial curves go to an array of PS_ANTICIPATE_STATIC_BYTES bytes
 * that is part of the library's device image (every GPU the library runs on holds its copy until the process
 * ends).  The call allocates and frees nothing.  Calls whose ps_anticipate_workspace_bytes() exceeds the
 * array are refused with PS_EWORKSPACE (with 256 instances x 600 buckets the array holds calls of up to
 * 212992 records; the long request-log streams need ps_anticipate()).  The device is the calling thread's
 * current one, and `hip_stream` must belong to it.  All calls on one GPU share that GPU's array: the caller
 * orders them (one stream, or events); calls that overlap on one GPU race on it.  Nothing needs clearing
 * between calls: the kernels write every scratch cell they later read. */
#define PS_ANTICIPATE_STATIC_BYTES  (8u << 20)
int ps_anticipate_static(const int32_t* pred_tokens, const int32_t* instance_id,
                         const int32_t* arrival_bucket, const int32_t* rate,
                         int64_t n_req, int32_t n_inst, int32_t horizon,
                         int32_t* load, int64_t* overflow, ps_status* status, void* hip_stream);

/* The load-look-ahead map in the paper's own units (Sec. 3.4.1): kv_tokens[k][t] is the number of
 * KV-cache tokens instance k is expected to hold at the t-th decoding iteration from now (the paper
 * records U = tokens / M, the fraction of the instance's token capacity M; see `fraction` below).
 * Record j adds sign[j] * (prompt_tokens[j] + i) to slot start_iter[j] + i of instance
 * instance_id[j] for every i in [i_begin[j], i_end[j]):
 *   - a new request with P prompt tokens and D predicted response tokens whose first decoding
 *     iteration is slot s:                      (k, s, P, 0, D, +1)    U'_i = (U_i M + (P + i)) / M
 *   - one that finished after D' < D iterations: (k, s, P, D', D, -1)   the rest is subtracted
 *   - one still running after D iterations:      (k, s, P, D, D + ext, +1)  a virtual extension, whose
 *     unused part is subtracted like an early finish once the request completes.
 *   instance_id, start_iter, prompt_tokens, i_begin, i_end, sign   [n_rec] int32 each
 *   n_rec, n_inst, map_len  host scalars; map_len <= PS_MAX_ITER + 1
 *   kv_tokens  [n_inst * map_len] int32, row-major, ACCUMULATED into (zero it to build from scratch)
 *   overflow   [n_inst] int64 or NULL, accumulated: signed tokens of iterations at or beyond map_len
 *   capacity   [n_inst] int32 token capacities M, needed only with `fraction`
 *   fraction   [n_inst * map_len] float or NULL, out: kv_tokens / capacity after the update (NaN for
 *              an instance whose capacity is < 1)
 *   workspace  device scratch of at least ps_lookahead_workspace_bytes(n_rec, n_inst, map_len) bytes,
 *              256-byte aligned; contents undefined before and after
 *   status     device ps_status or NULL.  A record with instance outside [0, n_inst), start_iter
 *              outside [0, map_len), prompt_tokens outside [0, PS_MAX_PROMPT), i_begin < 0, i_end < i_begin,
 *              i_end > PS_MAX_ITER or sign not +1 / -1 is skipped (PS_ST_BAD_RECORD); a slot that
 *              leaves the int32 range keeps its low 32 bits (PS_ST_RANGE).
 * Integer arithmetic throughout: the result does not depend on record order and is bit-exact, however many
 * records start or end in one slot (lists of 65536 records or more over maps of at most 12800 slots and 4096
 * instances are binned by instance and folded in LDS with wide counters; other calls use packed global counters
 * and are folded in parts of 2^22 records, within which no intermediate sum can leave its field).
 * n_rec == 0 is allowed (with `fraction` it recomputes the fractions of the map as it stands).
 * Errors: PS_EINVAL, PS_EWORKSPACE, PS_EUNSUPPORTED (map_len above PS_MAX_ITER + 1), PS_EHIP. */
#define PS_MAX_ITER  65535       /* largest i_end ps_lookahead_update accepts                 */
#define PS_MAX_PROMPT 131072     /* prompt_tokens must be below this (2^17)                   */
size_t ps_lookahead_workspace_bytes(int64_t n_rec, int32_t n_inst, int32_t map_len);
int ps_lookahead_update(const int32_t* instance_id, const int32_t* start_iter,
                        const int32_t* prompt_tokens, const int32_t* i_begin, const int32_t* i_end,
                        const int32_t* sign, int64_t n_rec, int32_t n_inst, int32_t map_len,
                        int32_t* kv_tokens, int64_t* overflow, const int32_t* capacity, float* fraction,
                        void* workspace, size_t workspace_bytes, ps_status* status, void* hip_stream);

/* In-window checks of the proactive instance scaler (Sec. 3.4.2) on the look-ahead maps of
 * ps_lookahead_update().  Over the next `window` iterations (clipped to map_len), U = tokens / capacity:
 *   over_count[k]   iterations in which instance k's usage exceeds over_pct % (the paper: 95)
 *   peak_tokens[k]  its largest token count in the window
 *   overloaded[k]   1 if over_count[k] is more than share_pct % of the window (the paper: 10), else 0
 *   summary[0]      number of overloaded instances (each asks for one more instance)
 *   summary[1]      1 if every instance stays below idle_pct % (the paper's T_f = 30) throughout the
 *                   window, i.e. a scale-down may be triggered, else 0
 *   scale_down[0]   n_inst - sum_k(peak_tokens[k] / capacity[k]) / (idle_pct / 100): the number of
 *                   instances to isolate if summary[1] is set (a double; the caller rounds)
 * kv_tokens [n_inst * map_len] int32, capacity [n_inst] int32; over_count, peak_tokens, overloaded
 * [n_inst] int32; summary [2] int32; scale_down [1] double; all device, all outputs overwritten.
 * Thresholds are whole percents and compared in integers, so the flags are exact.  An instance with
 * capacity < 1 is left out (zeros) and clears summary[1].  Errors: PS_EINVAL, PS_EHIP. */
int ps_scaler_scan(const int32_t* kv_tokens, const int32_t* capacity, int32_t n_inst, int32_t map_len,
                   int32_t window, int32_t over_pct, int32_t share_pct, int32_t idle_pct,
                   int32_t* over_count, int32_t* peak_tokens, int32_t* overloaded, int32_t* summary,
                   double* scale_down, void* hip_stream);

/* Load-aware request router (Sec. 3.4.3): dispatch the n_req requests of a micro-batch one after the
 * other, each to the instance with the smallest estimated load
 *     L_i = (queued_p[i] + P) + (current_d[i] + D) + beta * max(0, U_i - T_mem) * M_i,
 * U_i = the peak, over the next `window` iterations, of instance i's look-ahead map with the request
 * virtually added (P + t tokens at iteration t < D), M_i = capacity[i].  Ties go to the lowest
 * index.  After each decision the chosen instance's queued_p, current_d and window are updated, so
 * the next request sees it.  Scores are integers: score100 = 100 L with T_mem as a whole percent.
 *   prompt_tokens, pred_tokens  [n_req] int32 (P, D; a request with either negative is not dispatched:
 *                  assigned = -1, PS_ST_BAD_RECORD)
 *   window_tokens  [n_inst * window] int32, in/out: the first `window` slots of every instance's map
 *   capacity       [n_inst] int32
 *   queued_p, current_d  [n_inst] int64, in/out: tokens waiting to be prefilled / still to be decoded
 *   assigned       [n_req] int32, out; score100 [n_req] int64, out: 100 L of the chosen instance
 * All arrays are device pointers.  One workgroup walks the batch: n_inst <= 1024 and
 * n_inst * (20 + 4 * window) bytes plus 21 KB must fit in 160 KB of LDS (PS_EUNSUPPORTED otherwise).
 * The full-length maps are brought up to date by passing `assigned` as instance_id to
 * ps_lookahead_update().  A window value that leaves the int32 range keeps its low 32 bits (PS_ST_RANGE);
 * the flag is also raised, conservatively, once the largest window value so far plus a request's P + window
 * reaches 2^31.  Errors: PS_EINVAL, PS_EUNSUPPORTED, PS_EHIP. */
int ps_route(const int32_t* prompt_tokens, const int32_t* pred_tokens, int32_t n_req, int32_t n_inst,
             int32_t window, int32_t* window_tokens, const int32_t* capacity, int64_t* queued_p,
             int64_t* current_d, int32_t t_mem_pct, int32_t beta, int32_t* assigned, int64_t* score100,
             ps_status* status, void* hip_stream);

/* Online phase of the service workload predictor (Sec. 3.2, Alg. 2).  For each of n_services services
 * two multiplicative LSTMs (Krause et al. 2016), one for prompt tokens and one for response tokens,
 * forecast the token count of the current time window from the counts of the k past windows, then,
 * with that forecast appended to the history, the count of the next window; the next window's
 * counts give the number of instances  N = max(P / mu_p, D / mu_d, (P + D) / mu_t).
 *   weights  [n_services][2][5 H^2 + 10 H + 1] float, H = hidden <= 64; per model, in this order:
 *            w_mx[H] W_mh[H][H] w_hx[H] W_hm[H][H] b_h[H] w_ix[H] W_im[H][H] b_i[H] w_ox[H] W_om[H][H]
 *            b_o[H] w_fx[H] W_fm[H][H] b_f[H] w_out[H] b_out, for the recurrence
 *              m = (w_mx x) * (W_mh h),  hh = w_hx x + W_hm m + b_h,  i, o, f = sigmoid(w_.x x + W_.m m + b_.),
 *              c = f c + i tanh(hh),  h = tanh(c) o
 *            on the input sequence min-max normalised as in Alg. 1: x = (count - min) / (max - min) over the
 *            sequence the model is applied to (a flat sequence takes the range as 1), and
 *            forecast = max(0, min + (max - min) (w_out . h + b_out)).  The second step's sequence is the k
 *            past windows plus the first forecast, normalised over those k + 1 values.
 *            each H x H matrix is stored input-major: the weight from input unit i to output unit j at [i * H + j];
 *            model 0 of a service is the prompt-token model, model 1 the response-token model
 *   hist_p, hist_d  [n_services][k] float: token counts of the k past windows, oldest first
 *   mu       [n_services][3] float: one instance's prefill, decode and total token capacity per window
 *   out      [n_services][5] float: forecasts (P current, D current, P next, D next) and N (not rounded)
 * All arrays are device pointers; fp32 arithmetic.  Errors: PS_EINVAL, PS_EUNSUPPORTED (hidden above
 * 64), PS_EHIP. */
int ps_forecast(const float* weights, int32_t hidden, const float* hist_p, const float* hist_d,
                int32_t n_services, int32_t k, const float* mu, float* out, void* hip_stream);

/* Kernel-family timing for benchmarks.  While enabled, ps_predict_load() brackets every kernel
 * launch with HIP events on the call's stream (the paper reports only the predictor's end-to-end
 * latency, Sec. 4.5; this splits it by kernel).  ps_profile_read() waits for `hip_stream`, adds
 * up the elapsed time and launch count of each family since the last read into ms[] and
 * launches[] (host arrays of PS_N_FAMILIES) and clears the record. */
#define PS_N_FAMILIES 6
#define PS_FAM_EMBED     0   /* bookkeeping + embedding gather + embedding LayerNorm */
#define PS_FAM_GEMM      1   /* QKV, output projection and feed-forward GEMMs         */
#define PS_FAM_ATTENTION 2
#define PS_FAM_LAYERNORM 3
#define PS_FAM_HEAD      4   /* [CLS] pooling + regression head                        */
#define PS_FAM_REFINE    5   /* error-compensated feed-forward pass over the [CLS] rows */
int ps_profile_enable(ps_model* model, int on);
int ps_profile_read(ps_model* model, void* hip_stream, double* ms /*host*/, int64_t* launches /*host*/);
/* Core clock the GPU sustained during the last large GEMM launched while profiling was enabled
 * (bf16 models): one workgroup of that launch counts core cycles against the device's constant-rate
 * timer.  Waits for `hip_stream`; *core_ghz (host) is 0 if no such launch has run.  The clock under
 * matrix-core load is what the achieved rate has to be read against: it sits well below the
 * nominal peak clock.  Errors: PS_EINVAL, PS_EHIP. */
int ps_profile_clock(ps_model* model, void* hip_stream, double* core_ghz /*host*/);

/* Bandwidth yardstick for benchmarks: enqueue one kernel that reads `bytes` bytes at `data` (device, 16-byte
 * aligned, bytes a multiple of 16) once and XORs the buffer's 64-bit words into *sink (device; accumulated
 * into, so clear it first to get the buffer's XOR).  It does what the anticipator's record kernels
 * (Sec. 3.4.1) do to their input and nothing else, so its rate is the ceiling such a kernel can be read
 * against on a given machine.  Allocates nothing.  Errors: PS_EINVAL (null pointer, negative or unaligned
 * size, unaligned data), PS_EHIP. */
int ps_profile_stream_read(const void* data /*device*/, int64_t bytes, uint64_t* sink /*device*/, void* hip_stream);

/* Wait for `hip_stream` and copy a device ps_status to *out (host). */
int ps_status_read(const ps_status* status /*device*/, void* hip_stream, ps_status* out /*host*/);

/* Text for a PS_E* code (host string, static storage). */
const char* ps_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* PRESERVE_H */
