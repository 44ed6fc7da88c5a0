// bf16 encoder path: the per-layer sequence of MFMA GEMMs and attention launches.  There is no
// LayerNorm kernel: a residual epilogue writes the new sums of the residual stream as two bf16 values
// hi + lo (hi is the next map's operand) and leaves per-row partial sums; a small kernel turns those into (mean, 1/std),
// and the next map, which carries the LayerNorm's scale and shift in its weights, finishes the
// normalisation in its own epilogue.
#include "device_util.h"
#include "internal.h"

namespace {

// Row statistics from the partial sums the residual epilogues leave: 16 lanes per row, lane p taking
// the pieces p, p + 16, ...; the 16 partial results are added in a fixed order.  Biased variance as
// E[v^2] - mean^2 (the rows are residual-stream sums, whose mean is small against their spread).
__global__ __launch_bounds__(256) void ln_stats_kernel(const float2* __restrict__ pstats, float2* __restrict__ stats,
                                                       int pieces, float inv_n, float eps,
                                                       const int32_t* __restrict__ total_rows) {
    const int p = threadIdx.x & 15;
    const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    if (row >= *total_rows) return;                     // whole 16-lane groups leave together
    float sm = 0.f, sq = 0.f;
    for (int c = p; c < pieces; c += 16) {
        const float2 v = pstats[row * pieces + c];
        sm += v.x;
        sq += v.y;
    }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
        sm += __shfl_xor(sm, o, 16);
        sq += __shfl_xor(sq, o, 16);
    }
    const float mean = sm * inv_n;
    const float var = fmaxf(sq * inv_n - mean * mean, 0.f);
    if (p == 0) stats[row] = make_float2(mean, 1.0f / sqrtf(var + eps));
}

}  // namespace

void launch_ln_stats(const float2* pstats, float2* stats, float eps, int hidden, int64_t max_rows,
                     const int32_t* total_rows, hipStream_t s) {
    hipLaunchKernelGGL(ln_stats_kernel, dim3((unsigned)(max_rows / 16)), dim3(256), 0, s, pstats, stats, hidden / 64,
                       1.0f / (float)hidden, eps, total_rows);
}

void run_encoder_bf16(const ps_model* m, int32_t n_req, const Workspace& ws, hipStream_t s) {
    const ps_model_info& f = m->info;
    const int H = f.hidden, F = f.ffn;
    bf16_t *x = (bf16_t*)ws.x, *qk = (bf16_t*)ws.qkv, *vt = (bf16_t*)ws.vt, *att = (bf16_t*)ws.att,
           *x1 = (bf16_t*)ws.x1, *g = (bf16_t*)ws.g;
    const int32_t* rows = &ws.meta->total_rows;        // the rows that belong to requests
    const int32_t* qkv_rows = &ws.meta->qkv_rows;     // QKV projection: those plus the slack the key tiles read
    const ResidualSrc none = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    const int32_t* n_req_dev = &ws.meta->n_req;
    int64_t* clk = m->profiling ? m->clk_slot : nullptr;   // clock probe of the large GEMMs
    // the stream entering layer 0 is the embedding LayerNorm of the sums the embed kernel left in (x, la)
    const float *sg = m->lne_g, *sbeta = m->lne_b;
#define PS_TIMED(FAM, CALL) do { ProfScope p_(m, FAM, s); CALL; } while (0)
    // the per-request side maps: the tiled kernel, or for calls of a few requests the streaming one
    const bool skinny = n_req <= PS_SKINNY_ROWS;
    // (K = the map's contraction length; the hi | lo forms hold 2 K columns per row of A and of the repeated W)
    auto side_gemm = [&](GemmEpilogue epi, const bf16_t* A, const void* W, const float* bias, const ResidualSrc& r, void* C,
                         int N, int K) {
        const int k_cols = epi == EPI_Q_MAPPED ? K : 2 * K;
        if (skinny) launch_skinny_gemm_bf16(epi, A, (const bf16_t*)W, bias, r, C, N, K, H, n_req_dev, s);
        else launch_gemm_bf16(epi, A, (const bf16_t*)W, bias, r, C, nullptr, ws.cls_rows, N, k_cols, H, n_req_dev, nullptr, s);
    };
    for (int l = 0; l < f.layers; ++l) {
        const LayerWeights& w = m->layers[(size_t)l];
        // After the last layer only the first row of every request goes on (to the head), and within
        // that layer a row's output projection and feed-forward block depend on no other row: there the
        // all-row GEMMs and LayerNorms are skipped, attention computes the first rows only, and the
        // per-request side pass below, which every layer runs for accuracy, is all that is left.
        const bool last = l + 1 == f.layers;
        // the sums entering the layer are (x, la), those after the attention sublayer (x1, lb); the per-row
        // partial statistics are only needed where a map with a folded LayerNorm follows
        float2* ps = last ? nullptr : ws.ps;
        const ResidualSrc in = {x, ws.la, ws.sa, sg, sbeta, nullptr, nullptr, x1, ps, nullptr};
        const ResidualSrc mid = {x1, ws.lb, ws.sb, w.ln1_g, w.ln1_b, nullptr, nullptr, x, ps, nullptr};
        const ResidualSrc mid_cls = {x1, ws.lb, ws.sb, w.ln1_g, w.ln1_b, ws.row_start, ws.seq_len, x, ps, nullptr};
        // operands of the maps with a folded LayerNorm: row statistics and column sums
        const ResidualSrc fold_qkv = {nullptr, nullptr, ws.sa, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, w.c_qkv};
        const ResidualSrc fold_1 = {nullptr, nullptr, ws.sb, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, w.c_1};
        if (!last) {
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_QKV, x, (const bf16_t*)w.w_qkv, w.b_qkv, fold_qkv, qk, vt,
                                                   ws.max_rows, 3 * H, H, H, qkv_rows, clk, s));
        } else {
            // keys and values of all rows; queries of the requests' first rows only, by a side GEMM on
            // those rows gathered into the (not yet used) first-row buffer
            const ResidualSrc fold_kv = {nullptr, nullptr, ws.sa, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, w.c_qkv + H};
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_KV, x, (const bf16_t*)w.w_qkv + (size_t)H * H, w.b_qkv + H, fold_kv,
                                                   qk, vt, ws.max_rows, 2 * H, H, H, qkv_rows, clk, s));
            const ResidualSrc first_rows = {nullptr, nullptr, ws.sa, nullptr, nullptr, ws.row_start, ws.seq_len, nullptr, nullptr, w.c_qkv};
            PS_TIMED(PS_FAM_REFINE, launch_cls_rows(m, n_req, ws, x, (bf16_t*)ws.cls_a, s));
            PS_TIMED(PS_FAM_REFINE, side_gemm(EPI_Q_MAPPED, (const bf16_t*)ws.cls_a, w.w_qkv, w.b_qkv, first_rows, qk, H, H));
        }
        PS_TIMED(PS_FAM_ATTENTION, launch_attention_bf16(m, n_req, ws, last, s));
        if (!last)
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_BIAS_RESIDUAL, att, (const bf16_t*)w.w_o, w.b_o, in, ws.lb,
                                                   nullptr, ws.max_rows, H, H, H, rows, clk, s));
        // output projection again for each request's first row from the hi | lo pairs the attention
        // kernel left in cls_a (see the feed-forward refinement below)
        const ResidualSrc in_cls = {x, ws.la, ws.sa, sg, sbeta, ws.row_start, ws.seq_len, x1, ps, nullptr};
        PS_TIMED(PS_FAM_REFINE, side_gemm(EPI_RESIDUAL_MAPPED, (const bf16_t*)ws.cls_a, w.w_od, w.b_o, in_cls, ws.lb, H, H));
        if (!last) {
            PS_TIMED(PS_FAM_LAYERNORM, launch_ln_stats(ws.ps, ws.sb, m->ln_eps, H, ws.max_rows, rows, s));
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_BIAS_GELU, x1, (const bf16_t*)w.w_1, w.d_1, fold_1, g, nullptr,
                                                   ws.max_rows, F, H, H, rows, clk, s));
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_BIAS_RESIDUAL, g, (const bf16_t*)w.w_2, w.b_2, mid, ws.la,
                                                   nullptr, ws.max_rows, H, F, H, rows, clk, s));
        } else {
            PS_TIMED(PS_FAM_LAYERNORM, launch_cls_stats(m, n_req, ws, x1, ws.lb, ws.sb, s));
        }
        // The feed-forward block again for each request's first row, the one the head reads, with its
        // input and its GELU output carried as two bf16 values per element (contraction length doubled,
        // weights repeated): bf16 rounding of these two tensors is the dominant error of the prediction
        // and acts row by row, so the pass removes it where it matters at < 1 % of the block's cost.
        PS_TIMED(PS_FAM_REFINE, launch_cls_gather(m, n_req, ws, x1, ws.lb, ws.sb, w.ln1_g, w.ln1_b, s));
        PS_TIMED(PS_FAM_REFINE, side_gemm(EPI_GELU_SPLIT, (const bf16_t*)ws.cls_a, w.w_1d, w.b_1, none, ws.cls_g, F, H));
        PS_TIMED(PS_FAM_REFINE, side_gemm(EPI_RESIDUAL_MAPPED, (const bf16_t*)ws.cls_g, w.w_2d, w.b_2, mid_cls, ws.la, H, F));
        if (!last)
            PS_TIMED(PS_FAM_LAYERNORM, launch_ln_stats(ws.ps, ws.sa, m->ln_eps, H, ws.max_rows, rows, s));
        else
            PS_TIMED(PS_FAM_LAYERNORM, launch_cls_stats(m, n_req, ws, x, ws.la, ws.sa, s));   // what the head reads
        sg = w.ln2_g;
        sbeta = w.ln2_b;
    }
#undef PS_TIMED
}
