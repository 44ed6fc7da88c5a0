// fp32 encoder path (models stored in fp32): plain LDS-tiled kernels in full single precision.
// It exists for small models whose results must track the fp64 definition to 1e-4; the bf16
// MFMA path in encoder_bf16.hip is the one built for throughput.
#include "device_util.h"
#include "internal.h"

namespace {

enum { F32_NONE = 0, F32_GELU = 1, F32_RESIDUAL = 2 };

// C[m, n] = sum_k A[m, k] W[k, n] + bias[n], then GELU or + residual[m, n].
// 64 x 64 output tile, 16-deep k slices staged in LDS, 4 x 4 outputs per thread.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W,
                                                       const float* __restrict__ bias,
                                                       const float* __restrict__ residual, float* __restrict__ C,
                                                       int N, int K, const BatchMeta* meta) {
    __shared__ float sA[16][64 + 1];
    __shared__ float sW[16][64 + 1];
    const int m0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    if (m0 >= meta->total_rows) return;
    const int tid = threadIdx.x;
    const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = tid; i < 64 * 16; i += 256) {
            const int r = i / 16, kk = i % 16;          // A: rows are always inside the padded buffer
            sA[kk][r] = (k0 + kk < K) ? A[(int64_t)(m0 + r) * K + k0 + kk] : 0.f;
            const int wk = i / 64, wn = i % 64;
            sW[wk][wn] = (k0 + wk < K && n0 + wn < N) ? W[(int64_t)(k0 + wk) * N + n0 + wn] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sA[kk][tm + i]; w[i] = sW[kk][tn + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tn + j;
            if (n >= N) continue;
            const int64_t at = (int64_t)(m0 + tm + i) * N + n;
            float v = acc[i][j] + bias[n];
            if (EPI == F32_GELU) v = 0.5f * v * (1.0f + erff(v * 0.70710678118654752f));
            if (EPI == F32_RESIDUAL) v += residual[at];
            C[at] = v;
        }
}

// One wavefront per (row, head): scores of the row against its request's keys go to LDS, then
// a max, an exponential pass and a weighted sum of the value rows, all in fp32.
__global__ __launch_bounds__(256) void attention_f32_kernel(const float* __restrict__ qkv, float* __restrict__ out,
                                                            int H, int d, int n_req, int max_pos,
                                                            const BatchMeta* meta, const int32_t* __restrict__ seq_len,
                                                            const int32_t* __restrict__ row_start) {
    extern __shared__ float lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    const int head = blockIdx.y;
    if (row >= meta->total_rows) return;          // whole wavefront leaves together
    int lo = 0, hi = n_req - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (row_start[mid] <= row) lo = mid; else hi = mid - 1;
    }
    const int base = row_start[lo], S = seq_len[lo];
    if (row - base >= S) return;
    float* sc = lds + wave * (max_pos + d);
    float* q = sc + max_pos;
    const int64_t ld = 3 * (int64_t)H;
    const float scale = 1.0f / sqrtf((float)d);
    for (int i = lane; i < d; i += 64) q[i] = qkv[row * ld + head * d + i];
    __builtin_amdgcn_wave_barrier();
    float mx = -INFINITY;
    for (int t = lane; t < S; t += 64) {
        const float* k = qkv + (base + t) * ld + H + head * d;
        float s = 0.f;
        for (int i = 0; i < d; ++i) s = fmaf(q[i], k[i], s);
        s *= scale;
        sc[t] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int t = lane; t < S; t += 64) {
        const float e = expf(sc[t] - mx);
        sc[t] = e;
        sum += e;
    }
    sum = wave_sum(sum);
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < d; i += 64) {
        const float* v = qkv + (int64_t)base * ld + 2 * H + head * d + i;
        float o = 0.f;
        for (int t = 0; t < S; ++t) o = fmaf(sc[t], v[t * ld], o);
        out[(int64_t)row * H + head * d + i] = o / sum;
    }
}

// LayerNorm of one row per wavefront (biased variance, two passes over the row).
__global__ __launch_bounds__(256) void layernorm_f32_kernel(const float* __restrict__ in, float* __restrict__ out,
                                                            const float* __restrict__ gamma,
                                                            const float* __restrict__ beta, float eps, int H,
                                                            const BatchMeta* meta) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= meta->total_rows) return;
    const float* x = in + row * H;
    float sum = 0.f;
    for (int i = lane; i < H; i += 64) sum += x[i];
    const float mean = wave_sum(sum) / (float)H;
    float sq = 0.f;
    for (int i = lane; i < H; i += 64) { const float t = x[i] - mean; sq += t * t; }
    const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)H + eps);
    for (int i = lane; i < H; i += 64) out[row * H + i] = (x[i] - mean) * rstd * gamma[i] + beta[i];
}

void gemm_f32(int epi, const float* A, const float* W, const float* bias, const float* res, float* C,
              int64_t max_rows, int N, int K, const BatchMeta* meta, hipStream_t s) {
    dim3 grid((unsigned)(max_rows / 64), (unsigned)((N + 63) / 64));
    if (epi == F32_NONE)
        hipLaunchKernelGGL(gemm_f32_kernel<F32_NONE>, grid, dim3(256), 0, s, A, W, bias, res, C, N, K, meta);
    else if (epi == F32_GELU)
        hipLaunchKernelGGL(gemm_f32_kernel<F32_GELU>, grid, dim3(256), 0, s, A, W, bias, res, C, N, K, meta);
    else
        hipLaunchKernelGGL(gemm_f32_kernel<F32_RESIDUAL>, grid, dim3(256), 0, s, A, W, bias, res, C, N, K, meta);
}

}  // namespace

void run_encoder_f32(const ps_model* m, int32_t n_req, const Workspace& ws, hipStream_t s) {
    const ps_model_info& f = m->info;
    const int H = f.hidden, F = f.ffn, d = H / f.heads;
    float *x = (float*)ws.x, *qkv = (float*)ws.qkv, *att = (float*)ws.att, *y = (float*)ws.y,
          *x1 = (float*)ws.x1, *g = (float*)ws.g;
    const unsigned row_blocks = (unsigned)(ws.max_rows / 4);
    const size_t att_lds = sizeof(float) * 4 * (size_t)(f.max_pos + d);
    for (int l = 0; l < f.layers; ++l) {
        const LayerWeights& w = m->layers[(size_t)l];
        gemm_f32(F32_NONE, x, (const float*)w.w_qkv, w.b_qkv, nullptr, qkv, ws.max_rows, 3 * H, H, ws.meta, s);
        hipLaunchKernelGGL(attention_f32_kernel, dim3(row_blocks, (unsigned)f.heads), dim3(256), att_lds, s,
                           qkv, att, H, d, n_req, f.max_pos, ws.meta, ws.seq_len, ws.row_start);
        gemm_f32(F32_RESIDUAL, att, (const float*)w.w_o, w.b_o, x, y, ws.max_rows, H, H, ws.meta, s);
        hipLaunchKernelGGL(layernorm_f32_kernel, dim3(row_blocks), dim3(256), 0, s, y, x1, w.ln1_g, w.ln1_b,
                           m->ln_eps, H, ws.meta);
        gemm_f32(F32_GELU, x1, (const float*)w.w_1, w.b_1, nullptr, g, ws.max_rows, F, H, ws.meta, s);
        gemm_f32(F32_RESIDUAL, g, (const float*)w.w_2, w.b_2, x1, y, ws.max_rows, H, F, ws.meta, s);
        hipLaunchKernelGGL(layernorm_f32_kernel, dim3(row_blocks), dim3(256), 0, s, y, x, w.ln2_g, w.ln2_b,
                           m->ln_eps, H, ws.meta);
    }
}
