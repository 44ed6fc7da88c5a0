// In-window checks of the proactive instance scaler (Sec. 3.4.2) on the look-ahead maps: for each
// instance the number of the next `window` iterations whose usage exceeds over_pct % of its capacity,
// the peak over the window, and whether that count is more than share_pct % of the window; over all
// instances how many are potentially overloaded, whether all stay below idle_pct %, and the number
// to isolate in that case, N_c - sum(max U) / T_f.  Percent thresholds are integers and every
// comparison is done in integers (tokens * 100 against percent * capacity), so the flags are exact.
#include "device_util.h"
#include "internal.h"

namespace {

// one wavefront per instance
__global__ __launch_bounds__(256) void scaler_rows_kernel(const int32_t* __restrict__ kv_tokens,
                                                          const int32_t* __restrict__ capacity, int n_inst,
                                                          int map_len, int window, int over_pct, int share_pct,
                                                          int32_t* __restrict__ over_count,
                                                          int32_t* __restrict__ peak_tokens,
                                                          int32_t* __restrict__ overloaded) {
    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (k >= n_inst) return;
    const int w = min(window, map_len);
    const long long M = capacity[k];
    int cnt = 0, pk = (int)0x80000000;
    if (M >= 1) {
        const int32_t* row = kv_tokens + (int64_t)k * map_len;
        for (int t = lane; t < w; t += 64) {
            const int n = row[t];
            cnt += (long long)n * 100 > (long long)over_pct * M ? 1 : 0;
            pk = max(pk, n);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            cnt += __shfl_xor(cnt, o, 64);
            pk = max(pk, __shfl_xor(pk, o, 64));
        }
    } else {
        pk = 0;
    }
    if (lane == 0) {
        over_count[k] = cnt;
        peak_tokens[k] = w >= 1 ? pk : 0;
        overloaded[k] = (long long)cnt * 100 > (long long)share_pct * w ? 1 : 0;
    }
}

// one wavefront for the totals; the sum of the peak fractions is taken in instance order in fp64
__global__ __launch_bounds__(64) void scaler_summary_kernel(const int32_t* __restrict__ capacity,
                                                            const int32_t* __restrict__ peak_tokens,
                                                            const int32_t* __restrict__ overloaded, int n_inst,
                                                            int window, int idle_pct, int32_t* __restrict__ summary,
                                                            double* __restrict__ scale_down) {
    const int lane = threadIdx.x;
    int n_over = 0, idle = 1;
    for (int k = lane; k < n_inst; k += 64) {
        const long long M = capacity[k];
        n_over += overloaded[k];
        if (M < 1 || window < 1 || !((long long)peak_tokens[k] * 100 < (long long)idle_pct * M)) idle = 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        n_over += __shfl_xor(n_over, o, 64);
        idle &= __shfl_xor(idle, o, 64);
    }
    if (lane == 0) {
        double total = 0.0;
        if (window >= 1)
            for (int k = 0; k < n_inst; ++k)
                if (capacity[k] >= 1) total += (double)peak_tokens[k] / (double)capacity[k];
        summary[0] = n_over;
        summary[1] = idle;
        scale_down[0] = (double)n_inst - total / ((double)idle_pct / 100.0);
    }
}

}  // namespace

extern "C" int ps_scaler_scan(const int32_t* kv_tokens, const int32_t* capacity, int32_t n_inst, int32_t map_len,
                              int32_t window, int32_t over_pct, int32_t share_pct, int32_t idle_pct,
                              int32_t* over_count, int32_t* peak_tokens, int32_t* overloaded, int32_t* summary,
                              double* scale_down, void* hip_stream) {
    if (!kv_tokens || !capacity || !over_count || !peak_tokens || !overloaded || !summary || !scale_down) return PS_EINVAL;
    if (n_inst < 1 || map_len < 1 || window < 0 || over_pct < 0 || share_pct < 0 || idle_pct < 1) return PS_EINVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    (void)hipGetLastError();
    hipLaunchKernelGGL(scaler_rows_kernel, dim3((unsigned)((n_inst + 3) / 4)), dim3(256), 0, s, kv_tokens, capacity,
                       n_inst, map_len, window, over_pct, share_pct, over_count, peak_tokens, overloaded);
    hipLaunchKernelGGL(scaler_summary_kernel, dim3(1), dim3(64), 0, s, capacity, peak_tokens, overloaded, n_inst,
                       min(window, map_len), idle_pct, summary, scale_down);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}
