// bf16 encoder path: the per-layer sequence of MFMA GEMMs, attention and LayerNorm launches, and
// the row LayerNorm kernel.
#include "device_util.h"
#include "internal.h"

namespace {

// LayerNorm of one row per wavefront (biased variance).  A row is H = 256 * NCH bf16; lane l holds
// the 4-element chunks l, l + 64, ... so every load and store of a wavefront is one contiguous
// 512-byte run.  Statistics in fp32 from the values held in registers; in == out is allowed.
template <int NCH>
__global__ __launch_bounds__(256) void layernorm_bf16_kernel(const bf16_t* __restrict__ in, bf16_t* __restrict__ out,
                                                             const float* __restrict__ gamma,
                                                             const float* __restrict__ beta, float eps,
                                                             const int32_t* __restrict__ total_rows) {
    constexpr int H = 256 * NCH;
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= *total_rows) return;
    const uint2* src = (const uint2*)(in + row * H);
    float x[NCH][4];
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const uint2 v = src[lane + 64 * c];
        x[c][0] = __uint_as_float(v.x << 16);
        x[c][1] = __uint_as_float(v.x & 0xffff0000u);
        x[c][2] = __uint_as_float(v.y << 16);
        x[c][3] = __uint_as_float(v.y & 0xffff0000u);
        sum += (x[c][0] + x[c][1]) + (x[c][2] + x[c][3]);
    }
    const float mean = wave_sum(sum) * (1.0f / H);
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[c][e] -= mean;
            sq = fmaf(x[c][e], x[c][e], sq);
        }
    const float rstd = 1.0f / sqrtf(wave_sum(sq) * (1.0f / H) + eps);
    uint2* dst = (uint2*)(out + row * H);
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const float4 g = ((const float4*)gamma)[lane + 64 * c];
        const float4 b = ((const float4*)beta)[lane + 64 * c];
        dst[lane + 64 * c] = make_uint2(pack_bf16x2(x[c][0] * rstd * g.x + b.x, x[c][1] * rstd * g.y + b.y),
                                        pack_bf16x2(x[c][2] * rstd * g.z + b.z, x[c][3] * rstd * g.w + b.w));
    }
}

}  // namespace

void launch_layernorm_bf16(const bf16_t* in, bf16_t* out, const float* gamma, const float* beta, float eps,
                           int hidden, int64_t max_rows, const int32_t* total_rows, hipStream_t s) {
    const dim3 grid((unsigned)(max_rows / 4)), block(256);
#define PS_LN(N) hipLaunchKernelGGL(layernorm_bf16_kernel<N>, grid, block, 0, s, in, out, gamma, beta, eps, total_rows)
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
           *y = (bf16_t*)ws.y, *x1 = (bf16_t*)ws.x1, *g = (bf16_t*)ws.g;
    const int32_t* rows = &ws.meta->total_rows;
    for (int l = 0; l < f.layers; ++l) {
        const LayerWeights& w = m->layers[(size_t)l];
        launch_gemm_bf16(EPI_QKV, x, (const bf16_t*)w.w_qkv, w.b_qkv, nullptr, qk, vt, ws.max_rows, 3 * H, H, H, rows, s);
        launch_attention_bf16(m, n_req, ws, s);
        launch_gemm_bf16(EPI_BIAS_RESIDUAL, att, (const bf16_t*)w.w_o, w.b_o, x, y, nullptr, ws.max_rows, H, H, H, rows, s);
        launch_layernorm_bf16(y, x1, w.ln1_g, w.ln1_b, m->ln_eps, H, ws.max_rows, rows, s);
        launch_gemm_bf16(EPI_BIAS_GELU, x1, (const bf16_t*)w.w_1, w.b_1, nullptr, g, nullptr, ws.max_rows, F, H, H, rows, s);
        launch_gemm_bf16(EPI_BIAS_RESIDUAL, g, (const bf16_t*)w.w_2, w.b_2, x1, y, nullptr, ws.max_rows, H, F, H, rows, s);
        launch_layernorm_bf16(y, x, w.ln2_g, w.ln2_b, m->ln_eps, H, ws.max_rows, rows, s);
    }
}
