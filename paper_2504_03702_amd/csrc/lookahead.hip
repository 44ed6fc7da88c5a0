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
// 64-bit word, offset * 2^24 + slope, so a record costs two 64-bit integer atomic adds whatever its
// length.  Sums of signed numbers add component-wise as long as the slope part stays below 2^23 and the
// offset part below 2^39 in magnitude.  Nothing is assumed about where records fall (the paper admits
// every request at the map's origin, so all of them may start in one slot): a call is folded in parts
// of at most 2^22 records, each cleared, scattered and scanned into the caller's map on its own; with
// |offset| = |P - s| < 2^17 per record neither part of any word can leave its field.  Updates at or beyond map_len
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
    const int32_t* __restrict__ i_end, const int32_t* __restrict__ sign, int64_t n, int64_t first_index, int n_inst,
    int map_len, unsigned long long* __restrict__ d2, int64_t* __restrict__ overflow, ps_status* st) {
    for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < n; r += (int64_t)gridDim.x * 256) {
        const int k = instance_id[r], s = start_iter[r], P = prompt_tokens[r];
        const int b = i_begin[r], e = i_end[r], sg = sign[r];
        if ((unsigned)k >= (unsigned)n_inst || (unsigned)s >= (unsigned)map_len || (unsigned)P >= (unsigned)PS_MAX_PROMPT || b < 0 ||
            e < b || e > PS_MAX_ITER || (sg != 1 && sg != -1)) {
            report_fault(st, PS_ST_BAD_RECORD, first_index + r);
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
    // parts of at most kPart records: the packed differences of one slot cannot overflow their fields within a
    // part (see the top of this file); the map accumulates, so the parts add up to the whole
    const int64_t kPart = (int64_t)1 << 22;
    for (int64_t at = 0; at < n_rec || at == 0; at += kPart) {
        const int64_t n_part = n_rec - at < kPart ? n_rec - at : kPart;
        const bool last = at + kPart >= n_rec;
        hipLaunchKernelGGL(lookahead_clear_kernel, dim3(clear_blocks), dim3(256), 0, s, (ulonglong2*)workspace, n16);
        if (n_part > 0) {
            const int64_t want = (n_part + 255) / 256;
            const unsigned blocks = (unsigned)(want < 8192 ? want : 8192);
            hipLaunchKernelGGL(lookahead_scatter_kernel, dim3(blocks), dim3(256), 0, s, instance_id + at, start_iter + at,
                               prompt_tokens + at, i_begin + at, i_end + at, sign + at, n_part, at, n_inst, map_len,
                               (unsigned long long*)workspace, overflow, status);
        }
        // the fractions are written once, from the finished map
        hipLaunchKernelGGL(lookahead_scan_kernel, dim3((unsigned)n_inst), dim3(256), 0, s, (const long long*)workspace,
                           n_inst, map_len, kv_tokens, capacity, last ? fraction : nullptr, status);
    }
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}
