// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "preserve.h"

typedef uint16_t bf16_t;   // raw bf16 bit pattern

#define PS_ROW_ALIGN   8     // every request starts at a multiple of this many activation rows
#define PS_ROW_TILE    256   // activation buffers are padded to a multiple of this many rows
#define PS_ATT_BQ      128   // query rows per attention workgroup (bf16 path)
#define PS_MAX_ROWS    ((int64_t)1 << 27)   // most activation rows one call may need (tokens + requests * (M + 8))
#define PS_KEY_SLACK   64    // the last key tile of a request reads up to this many rows past its end: they
                             // must hold finite numbers (their weights are exactly zero), so the embedding
                             // zero-fills and the GEMMs cover that many rows beyond the last request

// Device weights of one encoder layer.  bf16 models: matrices are bf16, stored [out][in]
// (the contraction index contiguous) for the MFMA kernels; fp32 models: float, [in][out].
struct LayerWeights {
    void *w_qkv, *w_o, *w_1, *w_2;
    void *w_od, *w_1d, *w_2d;    // bf16 models: W_o, W_1, W_2 with the contraction index repeated ([out][2 in])
    float *b_qkv, *b_o, *b_1, *b_2;
    // bf16 models: the LayerNorm in front of the QKV and the first feed-forward map is folded into them.
    // With x = (y - mean) * rstd * gamma + beta:  x W + b = rstd * (y (gamma W) - mean * c) + d,
    // c[n] = sum_k gamma[k] W[k][n], d[n] = b[n] + sum_k beta[k] W[k][n].  w_qkv and w_1 hold gamma W,
    // b_qkv holds d of the QKV map, d_1 that of W_1 (b_1 stays the plain bias: the first-row pass uses it
    // with the plain w_1d), c_qkv and c_1 the column sums taken over the rounded gamma W.
    float *c_qkv, *c_1, *d_1;
    float *ln1_g, *ln1_b, *ln2_g, *ln2_b;
};

struct ProfRecord {
    int family;
    hipEvent_t start, stop;
};

struct ps_model {
    // event records of ps_profile_enable(); mutable so launch code holding a const model can log
    mutable bool profiling = false;
    mutable std::vector<ProfRecord> prof;
    mutable std::vector<hipEvent_t> event_pool;
    ps_model_info info;
    float ln_eps;
    int device;
    int lds_max;                 // largest LDS allocation of one workgroup on this device
    int64_t* clk_slot;           // device: {core cycles, timer ticks} of the last profiled GEMM launch
    void* blob;                  // the one device allocation everything below points into
    size_t blob_bytes;
    void *e_tok, *e_pos, *e_soft;     // embedding tables in the model's dtype, [rows][hidden]
    float *lne_g, *lne_b;
    std::vector<LayerWeights> layers;
    float *w_h1t;                // [head_hidden][hidden]
    float *b_h1, *w_h2;
    float b_h2;
};

// Per-call bookkeeping the prep kernel writes at the start of the workspace.
struct BatchMeta {
    int32_t total_rows;          // activation rows in use (padded request starts included)
    int32_t total_qtiles;        // attention query tiles over all requests
    int32_t n_req;               // requests in this call (row count of the per-request side GEMMs)
    int32_t qkv_rows;            // total_rows + PS_KEY_SLACK: rows the QKV projection covers
};

// Carved-up workspace of one ps_predict_load call.
struct Workspace {
    BatchMeta* meta;
    int32_t *seq_len;            // [B]   rows of request r (text + learnable prompts), 0 if faulty
    int32_t *row_start;          // [B+1] first activation row of request r
    int32_t *qtile_start;        // [B+1] first attention query tile of request r
    int32_t *bad_req;            // [B]   set when a request's text holds an invalid token id
    void *x, *qkv, *vt, *att, *y, *x1, *g;
    // bf16 path: the residual stream is kept as the pre-LayerNorm sums of the last two sublayers,
    // each sum as two bf16 values hi + lo (16 significant bits), plus each row's (mean, 1/std); its
    // LayerNorm is recomputed wherever it is needed.  The hi parts are x (sums entering a layer) and x1
    // (sums after the attention sublayer): exactly the operands of the maps the LayerNorms are folded into.
    bf16_t *la, *lb;             // lo parts belonging to x and x1
    float2 *sa, *sb;
    float2 *ps;                  // [rows][hidden / 64] per-row partial (sum, sum of squares) of the newest sums
    void *cls_a, *cls_g;         // per-request rows of the [CLS] refinement: [cls_rows][2H], [cls_rows][2F] bf16
    int64_t cls_rows;
    int64_t max_rows;            // rows every activation buffer holds (multiple of PS_ROW_TILE)
    int64_t max_qtiles;
    size_t bytes;
};

Workspace plan_workspace(const ps_model_info& info, int64_t n_tokens, int32_t n_req, void* base);

// ---- launchers (each enqueues on `s`; all pointers are device pointers) -------------------
void launch_prep(const ps_model* m, const int32_t* offsets, const int32_t* lengths, int32_t n_req, int64_t n_tokens,
                 const Workspace& ws, ps_status* st, hipStream_t s);
void launch_embed(const ps_model* m, const int32_t* token_ids, const int32_t* offsets, int32_t n_req,
                  const Workspace& ws, ps_status* st, hipStream_t s);
void launch_head(const ps_model* m, int32_t n_req, const Workspace& ws, float* pred_f, int32_t* pred_tokens,
                 ps_status* st, hipStream_t s);
void run_encoder_f32(const ps_model* m, int32_t n_req, const Workspace& ws, hipStream_t s);
void run_encoder_bf16(const ps_model* m, int32_t n_req, const Workspace& ws, hipStream_t s);

// bf16 kernels
enum GemmEpilogue {
    EPI_BIAS = 0, EPI_BIAS_GELU = 1, EPI_BIAS_RESIDUAL = 2, EPI_QKV = 3,
    EPI_GELU_SPLIT = 4,          // GELU, then the fp32 value stored as two bf16 (value ~ hi + lo) in [rows][2N]
    EPI_RESIDUAL_MAPPED = 5,     // EPI_BIAS_RESIDUAL with GEMM row r living at stream row row_map[r]
    EPI_KV = 6,                  // EPI_QKV without the query columns: W holds the key and value rows only
    EPI_Q_MAPPED = 7             // query columns only, GEMM row r stored at row row_map[r] of the [rows][2H] buffer
};
// The residual stream entering a sublayer: LayerNorm(y) with the row statistics already known.
struct ResidualSrc {
    const bf16_t* y_hi;      // [rows][hidden] pre-LayerNorm sums, value = hi + lo
    const bf16_t* y_lo;
    const float2* stats;     // [rows] (mean, 1 / sqrt(var + eps))
    const float* gamma;
    const float* beta;
    const int32_t* row_map;  // EPI_RESIDUAL_MAPPED: stream row of GEMM row r (the request's first row)
    const int32_t* seq_len;  //                       rows with seq_len[r] <= 0 are not stored
    // residual epilogues: the hi parts of the new sums (the lo parts go to the C argument); hi is also
    // the next map's operand.  Optional: every 64-column piece of a row leaves its (sum, sum of squares)
    // in pstats[row][N / 64]
    bf16_t* x_out;
    float2* pstats;
    // epilogues of the maps a LayerNorm is folded into (EPI_QKV, EPI_KV, EPI_Q_MAPPED, EPI_BIAS_GELU):
    // `stats` are the statistics of the operand's rows, colsum is c above and the bias argument is d
    const float* colsum;
};
// C[rows, N] = A[rows, K] * W^T (+ epilogue); W is [N][K]; rows = *total_rows (device).
// The residual epilogues write the new sums as hi (residual.x_out) + lo (C) bf16 pairs; all epilogues write bf16.  clk (device,
// may be null): workgroup 0 leaves {core clock cycles, constant-rate timer ticks} of its run there.
void launch_gemm_bf16(GemmEpilogue epi, const bf16_t* A, const bf16_t* W, const float* bias,
                      ResidualSrc res, void* C, bf16_t* vt, int64_t max_rows, int N, int K,
                      int hidden, const int32_t* total_rows, int64_t* clk, hipStream_t s);
// The per-request forms (EPI_GELU_SPLIT, EPI_RESIDUAL_MAPPED, EPI_Q_MAPPED) for calls of at most PS_SKINNY_ROWS
// requests: a stream over W with the contraction split among a workgroup's wavefronts.
#define PS_SKINNY_ROWS 16
void launch_skinny_gemm_bf16(GemmEpilogue epi, const bf16_t* A, const bf16_t* W, const float* bias, ResidualSrc residual,
                             void* C, int N, int K, int hidden, const int32_t* n_rows, hipStream_t s);
void launch_cls_gather(const ps_model* m, int32_t n_req, const Workspace& ws, const bf16_t* y_hi, const bf16_t* y_lo,
                       const float2* stats, const float* gamma, const float* beta, hipStream_t s);
// out[r][0:hidden] = x[first row of request r] for every request (zeros for faulty ones and padding rows).
void launch_cls_rows(const ps_model* m, int32_t n_req, const Workspace& ws, const bf16_t* x, bf16_t* out, hipStream_t s);
// stats[first row of request r] = LayerNorm statistics of that row of the sums hi + lo, for every request.
void launch_cls_stats(const ps_model* m, int32_t n_req, const Workspace& ws, const bf16_t* y_hi, const bf16_t* y_lo,
                      float2* stats, hipStream_t s);
// first_rows_only: compute (at least) the first query row of every request and nothing beyond its
// first 32 rows; the rest of the output buffer keeps its old contents.
void launch_attention_bf16(const ps_model* m, int32_t n_req, const Workspace& ws, bool first_rows_only, hipStream_t s);
// stats[row] = (mean, 1/std) of every live row from the partial sums the residual epilogues left.
void launch_ln_stats(const float2* pstats, float2* stats, float eps, int hidden, int64_t max_rows,
                     const int32_t* total_rows, hipStream_t s);

// Brackets the launches made during its lifetime with two events when profiling is on.
struct ProfScope {
    const ps_model* m;
    hipStream_t s;
    ProfRecord rec;
    bool live;
    ProfScope(const ps_model* model, int family, hipStream_t stream) : m(model), s(stream), live(false) {
        if (!m->profiling) return;
        hipEvent_t ev[2];
        for (int i = 0; i < 2; ++i) {
            if (!m->event_pool.empty()) {
                ev[i] = m->event_pool.back();
                m->event_pool.pop_back();
            } else if (hipEventCreate(&ev[i]) != hipSuccess) {
                return;
            }
        }
        rec = {family, ev[0], ev[1]};
        live = hipEventRecord(rec.start, s) == hipSuccess;
    }
    ~ProfScope() {
        if (!live) return;
        (void)hipEventRecord(rec.stop, s);
        m->prof.push_back(rec);
    }
};

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
