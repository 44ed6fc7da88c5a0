// Online phase of the service workload predictor (Sec. 3.2, Alg. 2): per service, a multiplicative
// LSTM (Krause et al. 2016) for prompt tokens and one for response tokens forecast the current and
// then the next time window from the k past windows, and the forecasts give the number of instances
// N = max(P / mu_p, D / mu_d, (P + D) / mu_t).  A model sees its input sequence min-max normalised
// (Alg. 1's normalisation step): x = (v - min) / (max - min) over the sequence (a flat sequence takes
// the range as 1), and its output y goes back to token counts as min + (max - min) y, not below 0.
// The second step applies the model to the history extended by the first forecast: while that
// forecast lies inside the history's range the normalisation is unchanged and the recurrence simply
// goes on by one input; otherwise the k + 1 values are normalised afresh and the recurrence is run
// again from the start.  One wavefront per service, lane j owning hidden unit j (hidden <= 64); h and
// m are exchanged through the wavefront's LDS slots; fp32 arithmetic.  Matrices are stored input-major
// ([in][out]: element (out j, in i) at i * H + j), so the lanes of a wavefront read consecutive words.
// A model is packed as
//   w_mx[H] W_mh[H][H] w_hx[H] W_hm[H][H] b_h[H] w_ix[H] W_im[H][H] b_i[H] w_ox[H] W_om[H][H] b_o[H]
//   w_fx[H] W_fm[H][H] b_f[H] w_out[H] b_out
#include "device_util.h"
#include "internal.h"

namespace {

__device__ __forceinline__ float sigmoid_f(float z) { return 1.0f / (1.0f + expf(-z)); }

__global__ __launch_bounds__(256) void forecast_kernel(const float* __restrict__ weights, int hidden,
                                                       const float* __restrict__ hist_p,
                                                       const float* __restrict__ hist_d, int n_services, int k,
                                                       const float* __restrict__ mu, float* __restrict__ out) {
    __shared__ float s_h[4][64], s_m[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s = blockIdx.x * 4 + wave;
    const bool live = s < n_services;                       // whole wavefront; dead ones still meet the barriers
    const bool unit = lane < hidden;
    const int H = hidden;
    const size_t model_floats = (size_t)5 * H * H + 10 * H + 1;
    float y[2][2] = {{0.f, 0.f}, {0.f, 0.f}};               // [kind][step]
    for (int kind = 0; kind < 2; ++kind) {
        const float* w = weights + (size_t)(2 * (live ? s : 0) + kind) * model_floats;
        const float* w_mx = w;
        const float* W_mh = w_mx + H;
        const float* w_hx = W_mh + H * H;
        const float* W_hm = w_hx + H;
        const float* b_h = W_hm + H * H;
        const float* w_ix = b_h + H;
        const float* W_im = w_ix + H;
        const float* b_i = W_im + H * H;
        const float* w_ox = b_i + H;
        const float* W_om = w_ox + H;
        const float* b_o = W_om + H * H;
        const float* w_fx = b_o + H;
        const float* W_fm = w_fx + H;
        const float* b_f = W_fm + H * H;
        const float* w_out = b_f + H;
        const float b_out = w_out[H];
        const float* hist = (kind == 0 ? hist_p : hist_d) + (size_t)(live ? s : 0) * k;
        // minimum and maximum of the history (every lane scans it: the values are wave-uniform)
        float lo = hist[0], hi = hist[0];
        for (int t = 1; t < k; ++t) {
            lo = fminf(lo, hist[t]);
            hi = fmaxf(hi, hist[t]);
        }
        float span = hi > lo ? hi - lo : 1.0f;
        // pass 0: the k past windows, then (first forecast inside [lo, hi]) one more input.  pass 1, only if the
        // first forecast left that range: the k + 1 values again under their own normalisation.
        // The barriers below are met by all four wavefronts of the workgroup the same number of times whatever
        // their passes: if one of them needs the second pass, the others run it on their data all the same and
        // discard the result (needs_second false: y is not overwritten).
        bool needs_second = false;
        for (int pass = 0; pass < 2; ++pass) {
            float h = 0.f, c = 0.f;
            s_h[wave][lane] = 0.f;
            __syncthreads();
            for (int t = 0; t <= k; ++t) {
                const float v = t < k ? hist[t] : y[kind][0];
                const float x = (v - lo) / span;
                float a = 0.f;
                if (unit) {
#pragma unroll 16
                    for (int j = 0; j < H; ++j) a = fmaf(W_mh[j * H + lane], s_h[wave][j], a);
                }
                s_m[wave][lane] = unit ? (w_mx[lane] * x) * a : 0.f;
                __syncthreads();
                if (unit) {
                    float hh = fmaf(w_hx[lane], x, b_h[lane]), gi = fmaf(w_ix[lane], x, b_i[lane]);
                    float go = fmaf(w_ox[lane], x, b_o[lane]), gf = fmaf(w_fx[lane], x, b_f[lane]);
#pragma unroll 8
                    for (int j = 0; j < H; ++j) {
                        const float mj = s_m[wave][j];
                        hh = fmaf(W_hm[j * H + lane], mj, hh);
                        gi = fmaf(W_im[j * H + lane], mj, gi);
                        go = fmaf(W_om[j * H + lane], mj, go);
                        gf = fmaf(W_fm[j * H + lane], mj, gf);
                    }
                    c = sigmoid_f(gf) * c + sigmoid_f(gi) * tanhf(hh);
                    h = tanhf(c) * sigmoid_f(go);
                }
                s_h[wave][lane] = unit ? h : 0.f;
                __syncthreads();
                if (t >= k - 1) {                           // after the k-th input and after the extension
                    const float dot = wave_sum(unit ? w_out[lane] * h : 0.f);
                    const float f = fmaxf(0.f, fmaf(span, dot + b_out, lo));
                    if (pass == 0) {
                        y[kind][t - (k - 1)] = f;
                        if (t == k - 1) {
                            needs_second = f < lo || f > hi;
                        }
                    } else if (needs_second && t == k) {
                        y[kind][1] = f;
                    }
                }
            }
            // no wavefront of this workgroup needs the second pass (decided by all its threads together, so
            // every one of them leaves or stays)
            if (pass == 0 && !__syncthreads_or((int)needs_second)) break;
            // normalisation of the extended history for the second pass
            const float f1 = y[kind][0];
            if (needs_second) {
                lo = fminf(lo, f1);
                hi = fmaxf(hi, f1);
                span = hi > lo ? hi - lo : 1.0f;
            }
        }
    }
    if (live && lane == 0) {
        const float p2 = y[0][1], d2 = y[1][1];
        float* o = out + (size_t)s * 5;
        o[0] = y[0][0]; o[1] = y[1][0]; o[2] = p2; o[3] = d2;
        o[4] = fmaxf(fmaxf(p2 / mu[3 * s], d2 / mu[3 * s + 1]), (p2 + d2) / mu[3 * s + 2]);
    }
}

}  // namespace

extern "C" int ps_forecast(const float* weights, int32_t hidden, const float* hist_p, const float* hist_d,
                           int32_t n_services, int32_t k, const float* mu, float* out, void* hip_stream) {
    if (!weights || !hist_p || !hist_d || !mu || !out || n_services < 0 || k < 1) return PS_EINVAL;
    if (hidden < 1 || hidden > 64) return PS_EUNSUPPORTED;
    if (n_services == 0) return PS_OK;
    (void)hipGetLastError();
    hipLaunchKernelGGL(forecast_kernel, dim3((unsigned)((n_services + 3) / 4)), dim3(256), 0, (hipStream_t)hip_stream,
                       weights, hidden, hist_p, hist_d, n_services, k, mu, out);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}
