// bf16 encoder path: the per-layer sequence of MFMA GEMMs, attention and LayerNorm launches, and
// the row LayerNorm kernel.
#include "device_util.h"
#include "internal.h"

namespace {

// LayerNorm of one row of fp32 sums per wavefront (biased variance): writes the bf16 row the
// next GEMM reads and the row's (mean, 1/std), from which later epilogues recompute the fp32
// LayerNorm output.  A row is H = 256 * NCH floats; lane l holds the 4-element chunks l, l + 64, ...
// so every load and store of a wavefront is one contiguous run.
template <int NCH>
__global__ __launch_bounds__(256) void layernorm_bf16_kernel(const float* __restrict__ y, bf16_t* __restrict__ x,
                                                             float2* __restrict__ stats,
                                                             const float* __restrict__ gamma,
                                                             const float* __restrict__ beta, float eps,
                                                             const int32_t* __restrict__ total_rows) {
    constexpr int H = 256 * NCH;
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= *total_rows) return;
    const float4* src = (const float4*)(y + row * H);
    float4 v[NCH];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        v[c] = src[lane + 64 * c];
        sum += (v[c].x + v[c].y) + (v[c].z + v[c].w);
    }
    const float mean = wave_sum(sum) * (1.0f / H);
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        v[c].x -= mean; v[c].y -= mean; v[c].z -= mean; v[c].w -= mean;
        sq = fmaf(v[c].x, v[c].x, sq); sq = fmaf(v[c].y, v[c].y, sq);
        sq = fmaf(v[c].z, v[c].z, sq); sq = fmaf(v[c].w, v[c].w, sq);
    }
    const float rstd = 1.0f / sqrtf(wave_sum(sq) * (1.0f / H) + eps);
    if (lane == 0) stats[row] = make_float2(mean, rstd);
    uint2* dst = (uint2*)(x + row * H);
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const float4 g = ((const float4*)gamma)[lane + 64 * c];
        const float4 b = ((const float4*)beta)[lane + 64 * c];
        dst[lane + 64 * c] = make_uint2(pack_bf16x2(v[c].x * rstd * g.x + b.x, v[c].y * rstd * g.y + b.y),
                                        pack_bf16x2(v[c].z * rstd * g.z + b.z, v[c].w * rstd * g.w + b.w));
    }
}

}  // namespace

void launch_layernorm_bf16(const float* y, bf16_t* x, float2* stats, const float* gamma, const float* beta,
                           float eps, int hidden, int64_t max_rows, const int32_t* total_rows, hipStream_t s) {
    const dim3 grid((unsigned)(max_rows / 4)), block(256);
#define PS_LN(N) hipLaunchKernelGGL(layernorm_bf16_kernel<N>, grid, block, 0, s, y, x, stats, gamma, beta, eps, total_rows)
    switch (hidden / 256) {
        case 1: PS_LN(1); break;
        case 2: PS_LN(2); break;
        case 3: PS_LN(3); break;
        case 4: PS_LN(4); break;
        case 5: PS_LN(5); break;
        case 6: PS_LN(6); break;
        case 7: PS_LN(7); break;
        case 8: PS_LN(8); break;
    }
#undef PS_LN
}

void run_encoder_bf16(const ps_model* m, int32_t n_req, const Workspace& ws, hipStream_t s) {
    const ps_model_info& f = m->info;
    const int H = f.hidden, F = f.ffn;
    bf16_t *x = (bf16_t*)ws.x, *qk = (bf16_t*)ws.qkv, *vt = (bf16_t*)ws.vt, *att = (bf16_t*)ws.att,
           *x1 = (bf16_t*)ws.x1, *g = (bf16_t*)ws.g;
    const int32_t* rows = &ws.meta->total_rows;        // the rows that belong to requests
    const int32_t* qkv_rows = &ws.meta->qkv_rows;     // QKV projection: those plus the slack the key tiles read
    const ResidualSrc none = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    const int32_t* n_req_dev = &ws.meta->n_req;
    int64_t* clk = m->profiling ? m->clk_slot : nullptr;   // clock probe of the large GEMMs
    // the stream entering layer 0 is the embedding LayerNorm of the sums the embed kernel left in ya
    const float *sg = m->lne_g, *sbeta = m->lne_b;
#define PS_TIMED(FAM, CALL) do { ProfScope p_(m, FAM, s); CALL; } while (0)
    for (int l = 0; l < f.layers; ++l) {
        const LayerWeights& w = m->layers[(size_t)l];
        // After the last layer only the first row of every request goes on (to the head), and within
        // that layer a row's output projection and feed-forward block depend on no other row: there the
        // all-row GEMMs and LayerNorms are skipped, attention computes the first rows only, and the
        // per-request side pass below, which every layer runs for accuracy, is all that is left.
        const bool last = l + 1 == f.layers;
        const ResidualSrc in = {ws.ya, ws.sa, sg, sbeta, nullptr, nullptr};
        const ResidualSrc mid = {ws.yb, ws.sb, w.ln1_g, w.ln1_b, nullptr, nullptr};
        const ResidualSrc mid_cls = {ws.yb, ws.sb, w.ln1_g, w.ln1_b, ws.row_start, ws.seq_len};
        if (!last) {
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_QKV, x, (const bf16_t*)w.w_qkv, w.b_qkv, none, qk, vt,
                                                   ws.max_rows, 3 * H, H, H, qkv_rows, clk, s));
        } else {
            // keys and values of all rows; queries of the requests' first rows only, by a side GEMM on
            // those rows gathered into the (not yet used) first-row buffer
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_KV, x, (const bf16_t*)w.w_qkv + (size_t)H * H, w.b_qkv + H, none,
                                                   qk, vt, ws.max_rows, 2 * H, H, H, qkv_rows, clk, s));
            const ResidualSrc first_rows = {nullptr, nullptr, nullptr, nullptr, ws.row_start, ws.seq_len};
            PS_TIMED(PS_FAM_REFINE, launch_cls_rows(m, n_req, ws, x, (bf16_t*)ws.cls_a, s));
            PS_TIMED(PS_FAM_REFINE, launch_gemm_bf16(EPI_Q_MAPPED, (const bf16_t*)ws.cls_a, (const bf16_t*)w.w_qkv, w.b_qkv,
                                                     first_rows, qk, nullptr, ws.cls_rows, H, H, H, n_req_dev, nullptr, s));
        }
        PS_TIMED(PS_FAM_ATTENTION, launch_attention_bf16(m, n_req, ws, last, s));
        if (!last)
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_BIAS_RESIDUAL, att, (const bf16_t*)w.w_o, w.b_o, in, ws.yb,
                                                   nullptr, ws.max_rows, H, H, H, rows, clk, s));
        // output projection again for each request's first row from the hi | lo pairs the attention
        // kernel left in cls_a (see the feed-forward refinement below)
        const ResidualSrc in_cls = {ws.ya, ws.sa, sg, sbeta, ws.row_start, ws.seq_len};
        PS_TIMED(PS_FAM_REFINE, launch_gemm_bf16(EPI_RESIDUAL_MAPPED, (const bf16_t*)ws.cls_a, (const bf16_t*)w.w_od,
                                                 w.b_o, in_cls, ws.yb, nullptr, ws.cls_rows, H, 2 * H, H, n_req_dev, nullptr, s));
        if (!last) {
            PS_TIMED(PS_FAM_LAYERNORM, launch_layernorm_bf16(ws.yb, x1, ws.sb, w.ln1_g, w.ln1_b, m->ln_eps, H,
                                                             ws.max_rows, rows, s));
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_BIAS_GELU, x1, (const bf16_t*)w.w_1, w.b_1, none, g, nullptr,
                                                   ws.max_rows, F, H, H, rows, clk, s));
            PS_TIMED(PS_FAM_GEMM, launch_gemm_bf16(EPI_BIAS_RESIDUAL, g, (const bf16_t*)w.w_2, w.b_2, mid, ws.ya,
                                                   nullptr, ws.max_rows, H, F, H, rows, clk, s));
        } else {
            PS_TIMED(PS_FAM_LAYERNORM, launch_cls_stats(m, n_req, ws, ws.yb, ws.sb, s));
        }
        // The feed-forward block again for each request's first row, the one the head reads, with its
        // input and its GELU output carried as two bf16 values per element (contraction length doubled,
        // weights repeated): bf16 rounding of these two tensors is the dominant error of the prediction
        // and acts row by row, so the pass removes it where it matters at < 1 % of the block's cost.
        PS_TIMED(PS_FAM_REFINE, launch_cls_gather(m, n_req, ws, ws.yb, ws.sb, w.ln1_g, w.ln1_b, s));
        PS_TIMED(PS_FAM_REFINE, launch_gemm_bf16(EPI_GELU_SPLIT, (const bf16_t*)ws.cls_a, (const bf16_t*)w.w_1d, w.b_1,
                                                 none, ws.cls_g, nullptr, ws.cls_rows, F, 2 * H, H, n_req_dev, nullptr, s));
        PS_TIMED(PS_FAM_REFINE, launch_gemm_bf16(EPI_RESIDUAL_MAPPED, (const bf16_t*)ws.cls_g, (const bf16_t*)w.w_2d,
                                                 w.b_2, mid_cls, ws.ya, nullptr, ws.cls_rows, H, 2 * F, H, n_req_dev, nullptr, s));
        if (!last)
            PS_TIMED(PS_FAM_LAYERNORM, launch_layernorm_bf16(ws.ya, x, ws.sa, w.ln2_g, w.ln2_b, m->ln_eps, H,
                                                             ws.max_rows, rows, s));
        else
            PS_TIMED(PS_FAM_LAYERNORM, launch_cls_stats(m, n_req, ws, ws.ya, ws.sa, s));   // what the head reads
        sg = w.ln2_g;
        sbeta = w.ln2_b;
    }
#undef PS_TIMED
}
