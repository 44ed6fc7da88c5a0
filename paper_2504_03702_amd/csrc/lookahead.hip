// Load-look-ahead map in the paper's own units (Sec. 3.4.1): per instance, the KV-cache tokens
// expected to be resident at each of the next map_len decoding iterations.
//
// A record (instance k, slot s, prompt P, i_begin, i_end, sign) adds sign * (P + i) to slot s + i
// for i in [i_begin, i_end): the admission of a request (i in [0, D), +1), the removal of the rest
// of one that finished early (i in [D', D), -1) or a virtual extension of one that runs long.  In
// terms of the slot t = s + i the amount is sign (P - s) + sign t, an offset and a slope that are
// constant over the record's slots [lo, hi) = [s + i_begin, s + i_end).  So with two difference
// arrays, dA[lo] += sign (P - s), dA[hi] -= sign (P - s) and dB[lo] += sign, dB[hi] -= sign,
// the map is N[t] = prefix(dA)[t] + t * prefix(dB)[t].  Both differences of a slot travel in one
// 64-bit word, offset * 2^24 + slope (sums of signed numbers add component-wise as long as the slope
// part stays below 2^23 in magnitude, i.e. fewer than 8 million records start or end in one slot), so a
// record costs two 64-bit integer atomic adds whatever its length.  Updates at or beyond map_len
// never reach a slot inside the map and are dropped; the tokens of iterations beyond the map go to
// overflow[] in closed form.  Rows here are long (thousands of iterations), so the differences live in
// an L2-resident global array rather than in LDS.  Kernels: clear the differences; one thread per
// record applies its updates; one workgroup per instance scans its row, accumulates into the
// caller's map and, if asked, writes the fraction of the instance's token capacity.  Integer
// arithmetic throughout: the result is exact and independent of record order.
#include "device_util.h"
#include "internal.h"

namespace {

__global__ __launch_bounds__(256) void lookahead_clear_kernel(ulonglong2* __restrict__ d2, int64_t n16) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256)
        d2[i] = make_ulonglong2(0ull, 0ull);
}

__global__ __launch_bounds__(256) void lookahead_scatter_kernel(
    const int32_t* __restrict__ instance_id, const int32_t* __restrict__ start_iter,
    const int32_t* __restrict__ prompt_tokens, const int32_t* __restrict__ i_begin,
    const int32_t* __restrict__ i_end, const int32_t* __restrict__ sign, int64_t n, int n_inst, int map_len,
    unsigned long long* __restrict__ d2, int64_t* __restrict__ overflow, ps_status* st) {
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < n; r += (int64_t)gridDim.x * 256) {
        const int k = instance_id[r], s = start_iter[r], P = prompt_tokens[r];
        const int b = i_begin[r], e = i_end[r], sg = sign[r];
        if ((unsigned)k >= (unsigned)n_inst || (unsigned)s >= (unsigned)map_len || (unsigned)P >= (1u << 20) || b < 0 ||
            e < b || e > PS_MAX_ITER || (sg != 1 && sg != -1)) {
            report_fault(st, PS_ST_BAD_RECORD, r);
            continue;
        }
        if (b == e) continue;
        const int64_t lo = (int64_t)s + b, hi = (int64_t)s + e;
        const long long word = (long long)sg * (P - s) * (1ll << 24) + sg;     // offset and slope, packed
        unsigned long long* row = d2 + (int64_t)k * map_len;
        if (lo < map_len) atomicAdd(row + lo, (unsigned long long)word);
        if (hi < map_len) atomicAdd(row + hi, (unsigned long long)(-word));
        if (hi > map_len && overflow) {
            // iterations io .. e - 1 fall beyond the map: c of them, sum of (P + i) in closed form
            const long long io = max((long long)b, (long long)map_len - s), c = e - io;
            const long long sum = c * P + (io + e - 1) * c / 2;
            atomicAdd((unsigned long long*)(overflow + k), (unsigned long long)((long long)sg * sum));
        }
    }
}

// One workgroup per instance.  Slots are taken 1024 at a time, thread t owning the four consecutive
// slots 4 t .. 4 t + 3; the two running sums (offsets, slopes) are scanned across the workgroup with
// wavefront shuffles (64-bit), carried from chunk to chunk.
__global__ __launch_bounds__(256) void lookahead_scan_kernel(const long long* __restrict__ d2, int n_inst, int map_len,
                                                             int32_t* __restrict__ kv_tokens,
                                                             const int32_t* __restrict__ capacity,
                                                             float* __restrict__ fraction, ps_status* st) {
    __shared__ long long s_w0[4], s_w1[4];
    const int k = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long* h = d2 + (int64_t)k * map_len;
    int32_t* out = kv_tokens + (int64_t)k * map_len;
    float* frow = fraction ? fraction + (int64_t)k * map_len : nullptr;
    const int cap = fraction ? capacity[k] : 1;
    const float cap_f = cap >= 1 ? (float)cap : __builtin_nanf("");      // no capacity: fractions are NaN
    long long carry0 = 0, carry1 = 0;
    for (int t0 = 0; t0 < map_len; t0 += 1024) {
        const int t = t0 + 4 * tid;
        long long a0[4], a1[4];                                 // offset differences, slope differences
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const long long v = t + c < map_len ? h[t + c] : 0;
            const long long slope = (long long)((unsigned long long)v << 40) >> 40;      // low 24 bits, signed
            a1[c] = slope;
            a0[c] = (v - slope) >> 24;                          // exact: the remainder is a multiple of 2^24
        }
#pragma unroll
        for (int c = 1; c < 4; ++c) { a0[c] += a0[c - 1]; a1[c] += a1[c - 1]; }
        long long i0 = a0[3], i1 = a1[3];                       // inclusive scans of the thread totals
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const long long u0 = __shfl_up(i0, o, 64), u1 = __shfl_up(i1, o, 64);
            if (lane >= o) { i0 += u0; i1 += u1; }
        }
        if (lane == 63) { s_w0[wave] = i0; s_w1[wave] = i1; }
        __syncthreads();
        long long before0 = carry0 + i0 - a0[3], before1 = carry1 + i1 - a1[3];
        for (int w = 0; w < wave; ++w) { before0 += s_w0[w]; before1 += s_w1[w]; }
        const long long tot0 = s_w0[0] + s_w0[1] + s_w0[2] + s_w0[3], tot1 = s_w1[0] + s_w1[1] + s_w1[2] + s_w1[3];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (t + c < map_len) {
                const long long nv = (long long)out[t + c] + (before0 + a0[c]) + (long long)(t + c) * (before1 + a1[c]);
                if (nv > 2147483647ll || nv < -2147483648ll) report_fault(st, PS_ST_RANGE, -1);
                out[t + c] = (int32_t)(uint32_t)(unsigned long long)nv;
                if (frow) frow[t + c] = (float)nv / cap_f;
            }
        }
        carry0 += tot0;
        carry1 += tot1;
        __syncthreads();
    }
}

}  // namespace

extern "C" size_t ps_lookahead_workspace_bytes(int32_t n_inst, int32_t map_len) {
    if (n_inst < 1 || map_len < 1 || map_len > PS_MAX_ITER + 1) return 0;
    return align_up((size_t)n_inst * (size_t)map_len * 8, 256);
}

extern "C" int ps_lookahead_update(const int32_t* instance_id, const int32_t* start_iter,
                                   const int32_t* prompt_tokens, const int32_t* i_begin, const int32_t* i_end,
                                   const int32_t* sign, int64_t n_rec, int32_t n_inst, int32_t map_len,
                                   int32_t* kv_tokens, int64_t* overflow, const int32_t* capacity, float* fraction,
                                   void* workspace, size_t workspace_bytes, ps_status* status, void* hip_stream) {
    if (n_rec < 0 || n_inst < 1 || map_len < 1 || !kv_tokens) return PS_EINVAL;
    if (fraction && !capacity) return PS_EINVAL;
    if (map_len > PS_MAX_ITER + 1) return PS_EUNSUPPORTED;
    if (n_rec > 0 && (!instance_id || !start_iter || !prompt_tokens || !i_begin || !i_end || !sign)) return PS_EINVAL;
    if (n_rec == 0 && !fraction) return PS_OK;
    const size_t need = ps_lookahead_workspace_bytes(n_inst, map_len);
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < need) return PS_EWORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    (void)hipGetLastError();
    const int64_t n16 = (int64_t)(need / 16);
    const unsigned clear_blocks = (unsigned)((n16 + 255) / 256 < 2048 ? (n16 + 255) / 256 : 2048);
    hipLaunchKernelGGL(lookahead_clear_kernel, dim3(clear_blocks), dim3(256), 0, s, (ulonglong2*)workspace, n16);
    if (n_rec > 0) {
        const int64_t want = (n_rec + 255) / 256;
        const unsigned blocks = (unsigned)(want < 8192 ? want : 8192);
        hipLaunchKernelGGL(lookahead_scatter_kernel, dim3(blocks), dim3(256), 0, s, instance_id, start_iter,
                           prompt_tokens, i_begin, i_end, sign, n_rec, n_inst, map_len,
                           (unsigned long long*)workspace, overflow, status);
    }
    hipLaunchKernelGGL(lookahead_scan_kernel, dim3((unsigned)n_inst), dim3(256), 0, s, (const long long*)workspace,
                       n_inst, map_len, kv_tokens, capacity, fraction, status);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}

// ------------------------------------------------------------------------------------------------
// In-window checks of the proactive instance scaler (Sec. 3.4.2) on the look-ahead maps: for each
// instance the number of the next `window` iterations whose usage exceeds over_pct % of its capacity,
// the peak over the window, and whether that count is more than share_pct % of the window; over all
// instances how many are potentially overloaded, whether all stay below idle_pct %, and the number
// to isolate in that case, N_c - sum(max U) / T_f.  Percent thresholds are integers and every
// comparison is done in integers (tokens * 100 against percent * capacity), so the flags are exact.
// ------------------------------------------------------------------------------------------------
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

// ------------------------------------------------------------------------------------------------
// Load-aware request router (Sec. 3.4.3): score every instance for each request of a micro-batch and
// dispatch to the smallest score,
//     100 L_i = 100 (queued_p_i + P + current_d_i + D) + beta * max(0, 100 peak_i - T_pct M_i),
// peak_i = the largest value, over the next `window` iterations, of instance i's look-ahead map with
// the request virtually added (P + t tokens at iteration t < D).  Decisions are sequential by
// definition (a dispatched request changes its instance's queue and map for the next one), so one
// workgroup walks the micro-batch with all state in LDS: TPI threads per instance scan its window, the
// scores are reduced to the minimum (lowest index on ties) with wavefront shuffles and one exchange
// through LDS, and the winner's threads add the request to its window.  Integer arithmetic
// throughout: the decisions are exact.
// ------------------------------------------------------------------------------------------------
namespace {

const int kRouteThreads = 1024;
const int kRouteLdsBytes = 160 * 1024;       // all of a compute unit's LDS

__global__ __launch_bounds__(kRouteThreads) void route_kernel(
    const int32_t* __restrict__ prompt_tokens, const int32_t* __restrict__ pred_tokens, int n_req, int n_inst,
    int window, int tpi, int32_t* __restrict__ window_tokens, const int32_t* __restrict__ capacity,
    int64_t* __restrict__ queued_p, int64_t* __restrict__ current_d, int t_mem_pct, int beta,
    int32_t* __restrict__ assigned, int64_t* __restrict__ score100, ps_status* st) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    long long* s_qp = (long long*)lds_raw;                       // [n_inst]
    long long* s_cd = s_qp + n_inst;                             // [n_inst]
    long long* s_best = s_cd + n_inst;                           // [2][16] per-wavefront minimum score
    int* s_best_i = (int*)(s_best + 32);                         // [2][16] and its instance
    int* s_cap = s_best_i + 32;                                  // [n_inst]
    int2* s_req = (int2*)(s_cap + n_inst + (n_inst & 1));         // [1024] (P, D) of the requests being walked
    long long* s_out_s = (long long*)(s_req + kRouteThreads);    // [1024] their scores
    int* s_out_i = (int*)(s_out_s + kRouteThreads);              // [1024] and instances, written out per chunk: a
                                                                 // global store per request would be waited for at
                                                                 // every barrier
    int* s_win = s_out_i + kRouteThreads;                        // [n_inst][window]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < n_inst; i += kRouteThreads) { s_qp[i] = queued_p[i]; s_cd[i] = current_d[i]; s_cap[i] = capacity[i]; }
    for (int i = tid; i < n_inst * window; i += kRouteThreads) s_win[i] = window_tokens[i];
    __syncthreads();
    const int inst = tid / tpi, sub = tid % tpi;
    const bool mine = inst < n_inst;
    int* row = s_win + (mine ? inst : 0) * window;
    const long long kNone = 0x7fffffffffffffffll;
    bool range_fault = false;
    for (int r = 0; r < n_req; ++r) {
        if ((r & (kRouteThreads - 1)) == 0) {
            // results of the last 1024 requests out, the next 1024 requests in
            __syncthreads();
            if (r > 0) { assigned[r - kRouteThreads + tid] = s_out_i[tid]; score100[r - kRouteThreads + tid] = s_out_s[tid]; }
            if (r + tid < n_req) s_req[tid] = make_int2(prompt_tokens[r + tid], pred_tokens[r + tid]);
            __syncthreads();
        }
        const int slot = r & (kRouteThreads - 1);
        const int2 pd = s_req[slot];
        const int P = pd.x, D = pd.y;                           // uniform
        if (P < 0 || D < 0) {
            if (tid == 0) { s_out_i[slot] = -1; s_out_s[slot] = 0; report_fault(st, PS_ST_BAD_RECORD, r); }
            __syncthreads();                                    // keeps the one-barrier-per-request rhythm of the exchange slots
            continue;
        }
        long long peak = -kNone;
        if (mine)
            for (int t = sub; t < window; t += tpi) peak = max(peak, (long long)row[t] + (t < D ? (long long)P + t : 0ll));
        for (int o = tpi >> 1; o > 0; o >>= 1) peak = max(peak, __shfl_xor(peak, o, 64));
        long long L = kNone;
        if (mine && sub == 0) {
            const long long pen = window > 0 ? max(0ll, 100 * peak - (long long)t_mem_pct * s_cap[inst]) : 0ll;
            L = 100 * (s_qp[inst] + P + s_cd[inst] + D) + (long long)beta * pen;
        }
        int bi = mine ? inst : 0x7fffffff;
        // minimum over the wavefront, lowest instance on ties
        for (int o = 32; o > 0; o >>= 1) {
            const long long oL = __shfl_xor(L, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (oL < L || (oL == L && oi < bi)) { L = oL; bi = oi; }
        }
        // the exchange slots alternate between requests, so one barrier per request is enough: a slot
        // is rewritten two requests later, after the barrier of the request in between
        const int par = (r & 1) * 16;
        if (lane == 0) { s_best[par + wave] = L; s_best_i[par + wave] = bi; }
        __syncthreads();
        long long bL = s_best[par];
        int bI = s_best_i[par];
        for (int w = 1; w < kRouteThreads / 64; ++w) {
            const long long oL = s_best[par + w];
            const int oi = s_best_i[par + w];
            if (oL < bL || (oL == bL && oi < bI)) { bL = oL; bI = oi; }
        }
        if (tid == 0) { s_out_i[slot] = bI; s_out_s[slot] = bL; }
        if (mine && inst == bI) {
            const int stop = min(D, window);
            for (int t = sub; t < stop; t += tpi) {
                const long long v = (long long)row[t] + P + t;
                if (v > 2147483647ll) range_fault = true;
                row[t] = (int)v;
            }
            if (sub == 0) { s_qp[inst] += P; s_cd[inst] += D; }
        }
        // no barrier here: an instance's window and counters are only ever touched by its own threads
    }
    __syncthreads();
    {   // results of the last, possibly partial, chunk
        const int done = n_req & ~(kRouteThreads - 1), first = done == n_req ? n_req - kRouteThreads : done;
        if (first + tid < n_req) { assigned[first + tid] = s_out_i[tid]; score100[first + tid] = s_out_s[tid]; }
    }
    if (range_fault) report_fault(st, PS_ST_RANGE, -1);
    for (int i = tid; i < n_inst; i += kRouteThreads) { queued_p[i] = s_qp[i]; current_d[i] = s_cd[i]; }
    for (int i = tid; i < n_inst * window; i += kRouteThreads) window_tokens[i] = s_win[i];
}

}  // namespace

extern "C" int ps_route(const int32_t* prompt_tokens, const int32_t* pred_tokens, int32_t n_req, int32_t n_inst,
                        int32_t window, int32_t* window_tokens, const int32_t* capacity, int64_t* queued_p,
                        int64_t* current_d, int32_t t_mem_pct, int32_t beta, int32_t* assigned, int64_t* score100,
                        ps_status* status, void* hip_stream) {
    if (n_req < 0 || n_inst < 1 || window < 0 || t_mem_pct < 0 || beta < 0) return PS_EINVAL;
    if (!capacity || !queued_p || !current_d || (window > 0 && !window_tokens)) return PS_EINVAL;
    if (n_req == 0) return PS_OK;
    if (!prompt_tokens || !pred_tokens || !assigned || !score100) return PS_EINVAL;
    if (n_inst > kRouteThreads) return PS_EUNSUPPORTED;
    const size_t lds = (size_t)n_inst * 20 + 32 * 12 + 20 * (size_t)kRouteThreads + (size_t)n_inst * window * 4 + 64;
    if (lds > (size_t)kRouteLdsBytes) return PS_EUNSUPPORTED;
    int tpi = 64;                                               // threads per instance: a power of two, <= 64
    while (tpi > 1 && (int64_t)tpi * n_inst > kRouteThreads) tpi >>= 1;
    hipStream_t s = (hipStream_t)hip_stream;
    (void)hipGetLastError();
    static bool lds_attr_set = false;     // raising the limit twice is harmless, so no lock
    if (!lds_attr_set) {
        if (hipFuncSetAttribute((const void*)route_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kRouteLdsBytes) != hipSuccess)
            return PS_EHIP;
        lds_attr_set = true;
    }
    hipLaunchKernelGGL(route_kernel, dim3(1), dim3(kRouteThreads), lds, s, prompt_tokens, pred_tokens, n_req, n_inst,
                       window, tpi, window_tokens, capacity, queued_p, current_d, t_mem_pct, beta, assigned, score100,
                       status);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}

// ------------------------------------------------------------------------------------------------
// Online phase of the service workload predictor (Sec. 3.2, Alg. 2): per service, a multiplicative
// LSTM (Krause et al. 2016) for prompt tokens and one for response tokens forecast the current and
// then the next time window from the k past windows (the recurrence goes on by one input, the first
// forecast), and the forecasts give the number of instances N = max(P / mu_p, D / mu_d,
// (P + D) / mu_t).  One wavefront per service, lane j owning hidden unit j (hidden <= 64); h and m
// are exchanged through the wavefront's LDS slots; fp32 arithmetic.  Matrices are stored input-major
// ([in][out]: element (out j, in i) at i * H + j), so the lanes of a wavefront read consecutive words.
// A model is packed as
//   w_mx[H] W_mh[H][H] w_hx[H] W_hm[H][H] b_h[H] w_ix[H] W_im[H][H] b_i[H] w_ox[H] W_om[H][H] b_o[H]
//   w_fx[H] W_fm[H][H] b_f[H] w_out[H] b_out scale
// ------------------------------------------------------------------------------------------------
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
    const size_t model_floats = (size_t)5 * H * H + 10 * H + 2;
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
        const float b_out = w_out[H], scale = w_out[H + 1];
        const float* hist = (kind == 0 ? hist_p : hist_d) + (size_t)(live ? s : 0) * k;
        float h = 0.f, c = 0.f;
        s_h[wave][lane] = 0.f;
        __syncthreads();
        for (int t = 0; t <= k; ++t) {
            const float x = (t < k ? hist[t] : y[kind][0]) / scale;
            float a = 0.f;
            if (unit) for (int j = 0; j < H; ++j) a = fmaf(W_mh[j * H + lane], s_h[wave][j], a);
            s_m[wave][lane] = unit ? (w_mx[lane] * x) * a : 0.f;
            __syncthreads();
            if (unit) {
                float hh = fmaf(w_hx[lane], x, b_h[lane]), gi = fmaf(w_ix[lane], x, b_i[lane]);
                float go = fmaf(w_ox[lane], x, b_o[lane]), gf = fmaf(w_fx[lane], x, b_f[lane]);
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
            if (t >= k - 1) {                               // after the k-th input and after the extension
                const float dot = wave_sum(unit ? w_out[lane] * h : 0.f);
                y[kind][t - (k - 1)] = fmaxf(0.f, scale * (dot + b_out));
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
