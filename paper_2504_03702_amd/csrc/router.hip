// Load-aware request router (Sec. 3.4.3): score every instance for each request of a micro-batch and
// dispatch to the smallest score,
//     100 L_i = 100 (queued_p_i + P + current_d_i + D) + beta * max(0, 100 peak_i - T_pct M_i),
// peak_i = the largest value, over the next `window` iterations, of instance i's look-ahead map with
// the request virtually added (P + t tokens at iteration t < D).  Decisions are sequential by
// definition (a dispatched request changes its instance's queue and map for the next one), so one
// workgroup walks the micro-batch with all state on chip (in the registers of the instances' threads where the
// windows are short enough, else in LDS): TPI threads per instance scan its window, the
// scores are reduced to the minimum (lowest index on ties) with wavefront shuffles and one exchange
// through LDS, and the winner's threads add the request to its window.  Integer arithmetic
// throughout: the decisions are exact.
#include "device_util.h"
#include "internal.h"

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

// The same walk with every instance's window in the registers of its TPI threads (thread `sub` of an instance
// owns iterations sub, sub + TPI, ...; at most kRegSlots each).  32-bit arithmetic: a running bound B on every
// window value is kept, and a request that could take a sum to 2^31 (B + P + window) is reported as a range
// fault before it is scored.  The sixteen wavefronts' minima are combined by every wavefront in parallel (one
// entry per lane, shuffles) instead of a serial scan.
const int kRegSlots = 32;

__global__ __launch_bounds__(kRouteThreads) void route_reg_kernel(
    const int32_t* __restrict__ prompt_tokens, const int32_t* __restrict__ pred_tokens, int n_req, int n_inst,
    int window, int tpi, int32_t* __restrict__ window_tokens, const int32_t* __restrict__ capacity,
    int64_t* __restrict__ queued_p, int64_t* __restrict__ current_d, int t_mem_pct, int beta,
    int32_t* __restrict__ assigned, int64_t* __restrict__ score100, ps_status* st) {
    __shared__ long long s_best[2][16];
    __shared__ int s_best_i[2][16];
    __shared__ int2 s_req[kRouteThreads];
    __shared__ long long s_out_s[kRouteThreads];
    __shared__ int s_out_i[kRouteThreads];
    __shared__ int s_max[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int inst = tid / tpi, sub = tid % tpi;
    const bool mine = inst < n_inst;
    const int kMin = (int)0x80000000;
    int r[kRegSlots];                            // dead slots (beyond the window, or no instance) hold the minimum
    int top = kMin;
#pragma unroll
    for (int i = 0; i < kRegSlots; ++i) {
        const int t = sub + tpi * i;
        r[i] = mine && t < window ? window_tokens[(int64_t)inst * window + t] : kMin;
        top = max(top, r[i]);
    }
    long long qp = 0, cd = 0, cap = 0;
    if (mine && sub == 0) { qp = queued_p[inst]; cd = current_d[inst]; cap = capacity[inst]; }
    // B: an upper bound on every window value, uniform over the workgroup
    for (int o = 32; o > 0; o >>= 1) top = max(top, __shfl_xor(top, o, 64));
    if (lane == 0) s_max[wave] = top;
    __syncthreads();
    long long B = kMin;
    for (int w = 0; w < 16; ++w) B = max(B, (long long)s_max[w]);
    const long long kNone = 0x7fffffffffffffffll;
    bool range_fault = false;
    for (int q = 0; q < n_req; ++q) {
        if ((q & (kRouteThreads - 1)) == 0) {
            // results of the last 1024 requests out, the next 1024 requests in
            __syncthreads();
            if (q > 0) { assigned[q - kRouteThreads + tid] = s_out_i[tid]; score100[q - kRouteThreads + tid] = s_out_s[tid]; }
            if (q + tid < n_req) s_req[tid] = make_int2(prompt_tokens[q + tid], pred_tokens[q + tid]);
            __syncthreads();
        }
        const int slot = q & (kRouteThreads - 1);
        const int2 pd = s_req[slot];
        const int P = pd.x, D = pd.y;                           // uniform
        if (P < 0 || D < 0) {
            if (tid == 0) { s_out_i[slot] = -1; s_out_s[slot] = 0; report_fault(st, PS_ST_BAD_RECORD, q); }
            __syncthreads();                                    // keeps the one-barrier-per-request rhythm of the exchange slots
            continue;
        }
        if (B + P + window >= 2147483647ll) range_fault = true; // a sum below may leave the int32 range
        int pk = kMin;
        const int Pt = P + sub;                                 // P + t of this thread's first iteration
#pragma unroll
        for (int i = 0; i < kRegSlots; ++i) {
            const int t = sub + tpi * i;
            const unsigned add = t < D ? (unsigned)(Pt + tpi * i) : 0u;
            pk = max(pk, (int)((unsigned)r[i] + add));          // (a dead slot stays far below any live one)
        }
        for (int o = tpi >> 1; o > 0; o >>= 1) pk = max(pk, __shfl_xor(pk, o, 64));
        long long L = kNone;
        if (mine && sub == 0) {
            const long long pen = max(0ll, 100 * (long long)pk - (long long)t_mem_pct * cap);
            L = 100 * (qp + P + cd + D) + (long long)beta * pen;
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
        const int par = q & 1;
        if (lane == 0) { s_best[par][wave] = L; s_best_i[par][wave] = bi; }
        __syncthreads();
        long long bL = lane < 16 ? s_best[par][lane] : kNone;
        int bI = lane < 16 ? s_best_i[par][lane] : 0x7fffffff;
        for (int o = 8; o > 0; o >>= 1) {
            const long long oL = __shfl_xor(bL, o, 64);
            const int oi = __shfl_xor(bI, o, 64);
            if (oL < bL || (oL == bL && oi < bI)) { bL = oL; bI = oi; }
        }
        bL = __shfl(bL, 0, 64);
        bI = __shfl(bI, 0, 64);
        if (tid == 0) { s_out_i[slot] = bI; s_out_s[slot] = bL; }
        if (mine && inst == bI) {
#pragma unroll
            for (int i = 0; i < kRegSlots; ++i) {
                const int t = sub + tpi * i;
                if (t < D && t < window) r[i] = (int)((unsigned)r[i] + (unsigned)(Pt + tpi * i));
            }
            if (sub == 0) { qp += P; cd += D; }
        }
        B += (long long)P + window;                             // every new value is at most an old one + P + window
    }
    __syncthreads();
    {   // results of the last, possibly partial, chunk
        const int done = n_req & ~(kRouteThreads - 1), first = done == n_req ? n_req - kRouteThreads : done;
        if (first + tid < n_req) { assigned[first + tid] = s_out_i[tid]; score100[first + tid] = s_out_s[tid]; }
    }
    if (range_fault && tid == 0) report_fault(st, PS_ST_RANGE, -1);
    if (mine && sub == 0) { queued_p[inst] = qp; current_d[inst] = cd; }
#pragma unroll
    for (int i = 0; i < kRegSlots; ++i) {
        const int t = sub + tpi * i;
        if (mine && t < window) window_tokens[(int64_t)inst * window + t] = r[i];
    }
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
    if (window >= 1 && (window + tpi - 1) / tpi <= kRegSlots)
        hipLaunchKernelGGL(route_reg_kernel, dim3(1), dim3(kRouteThreads), 0, s, prompt_tokens, pred_tokens, n_req, n_inst,
                           window, tpi, window_tokens, capacity, queued_p, current_d, t_mem_pct, beta, assigned,
                           score100, status);
    else
        hipLaunchKernelGGL(route_kernel, dim3(1), dim3(kRouteThreads), lds, s, prompt_tokens, pred_tokens, n_req, n_inst,
                           window, tpi, window_tokens, capacity, queued_p, current_d, t_mem_pct, beta, assigned, score100,
                           status);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}
