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
//
// Long record lists over maps whose rows fit a compute unit's LDS take another route, without global
// atomics: the records are first binned by instance.  A workgroup of the binning kernel takes a chunk of
// 8192 records, turns each into one 8-byte entry (first slot, slot after the last, offset, sign; tokens
// beyond the map are summed per instance in LDS and added to overflow[] at the end), ranks the chunk's
// entries per instance with an LDS counter each, and writes them to its own region of the workspace
// grouped by instance, with the region's per-instance boundaries in a table.  Then one workgroup per
// instance walks the table, applies its entries to an LDS row (offset differences in 64 bits, slope
// differences in 32: nothing can overflow) and scans the row into the caller's map itself.  Every record
// is read once (24 bytes), written once as an entry and read once more (8 bytes each).
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


// ---- binned route -----------------------------------------------------------------------------------
const int kBinThreads = 512;
const int kBinPerThread = 16;
const int kBinChunk = kBinThreads * kBinPerThread;       // records per binning workgroup
const int kBinMaxInst = 4096;                            // instance counters of a chunk live in LDS
const int kRowLdsBytes = 150 * 1024;                     // LDS a map row may take (12 bytes per slot)
const int64_t kBinMinRecords = 65536;                    // shorter lists do not pay for the extra pass
const int64_t kBinPart = (int64_t)1 << 26;               // records per part (bounds the workspace)

// entry: bits 0..16 first slot (map_len: none), 17..33 slot after the last (map_len: none),
//        34..52 offset + 2^18, bit 53 set for sign -1
__device__ __forceinline__ unsigned long long pack_entry(unsigned lo, unsigned hi, int offset, int sg) {
    return (unsigned long long)lo | ((unsigned long long)hi << 17) | ((unsigned long long)(unsigned)(offset + (1 << 18)) << 34) |
           ((unsigned long long)(sg < 0 ? 1u : 0u) << 53);
}

// VEC: the six arrays are 16-byte aligned, a thread takes four consecutive records per load.
template <bool VEC>
__global__ __launch_bounds__(kBinThreads) void lookahead_bin_kernel(
    const int32_t* __restrict__ instance_id, const int32_t* __restrict__ start_iter,
    const int32_t* __restrict__ prompt_tokens, const int32_t* __restrict__ i_begin,
    const int32_t* __restrict__ i_end, const int32_t* __restrict__ sign, int64_t n, int64_t first_index, int n_inst,
    int map_len, unsigned long long* __restrict__ entries, int32_t* __restrict__ table, int64_t n_chunks,
    int64_t* __restrict__ overflow, ps_status* st) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    unsigned long long* s_ent = (unsigned long long*)lds_raw;             // [kBinChunk] the chunk's entries, grouped by instance
    long long* s_ovf = (long long*)(s_ent + kBinChunk);                   // [n_inst] tokens beyond the map
    int* s_cnt = (int*)(s_ovf + n_inst);                                  // [n_inst] entries per instance, then their starts
    __shared__ int s_wave[kBinThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t chunk = blockIdx.x, base = chunk * kBinChunk;
    for (int i = tid; i < n_inst; i += kBinThreads) { s_ovf[i] = 0; s_cnt[i] = 0; }
    __syncthreads();
    unsigned long long ent[kBinPerThread];
    int inst[kBinPerThread], rank[kBinPerThread];
    // One record: checks, its tokens beyond the map, its entry and the entry's rank among its instance's
    auto take = [&](int u, int64_t r, int k, int s, int P, int b, int e, int sg) {
        inst[u] = -1;
        if ((unsigned)k >= (unsigned)n_inst || (unsigned)s >= (unsigned)map_len || (unsigned)P >= (unsigned)PS_MAX_PROMPT || b < 0 ||
            e < b || e > PS_MAX_ITER || (sg != 1 && sg != -1)) {
            report_fault(st, PS_ST_BAD_RECORD, first_index + r);
            return;
        }
        if (b == e) return;
        const int lo = s + b, hi = s + e;                                 // both below 2^17
        if (hi > map_len && overflow) {
            // iterations io .. e - 1 fall beyond the map: c of them, sum of (P + i) in closed form
            const long long io = max(b, map_len - s), c = e - io;
            const long long sum = c * P + (io + e - 1) * c / 2;
            atomicAdd((unsigned long long*)&s_ovf[k], (unsigned long long)((long long)sg * sum));
        }
        if (lo >= map_len) return;                                        // nothing of it inside the map
        ent[u] = pack_entry((unsigned)lo, (unsigned)min(hi, map_len), P - s, sg);
        inst[u] = k;
        rank[u] = atomicAdd(&s_cnt[k], 1);
    };
    if (VEC && base + kBinChunk <= n) {
        // whole chunk: a thread's u-th load covers records base + (u * kBinThreads + tid) * 4 .. + 3
        constexpr int NV = kBinPerThread / 4;
        int4 vk[NV], vs[NV], vp[NV], vb[NV], ve[NV], vg[NV];
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int64_t r = base + ((int64_t)u * kBinThreads + tid) * 4;
            vk[u] = load_stream_int4(instance_id + r); vs[u] = load_stream_int4(start_iter + r);
            vp[u] = load_stream_int4(prompt_tokens + r); vb[u] = load_stream_int4(i_begin + r);
            ve[u] = load_stream_int4(i_end + r); vg[u] = load_stream_int4(sign + r);
        }
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int64_t r = base + ((int64_t)u * kBinThreads + tid) * 4;
            take(4 * u, r, vk[u].x, vs[u].x, vp[u].x, vb[u].x, ve[u].x, vg[u].x);
            take(4 * u + 1, r + 1, vk[u].y, vs[u].y, vp[u].y, vb[u].y, ve[u].y, vg[u].y);
            take(4 * u + 2, r + 2, vk[u].z, vs[u].z, vp[u].z, vb[u].z, ve[u].z, vg[u].z);
            take(4 * u + 3, r + 3, vk[u].w, vs[u].w, vp[u].w, vb[u].w, ve[u].w, vg[u].w);
        }
    } else {
#pragma unroll
        for (int u = 0; u < kBinPerThread; ++u) {
            const int64_t r = base + (int64_t)u * kBinThreads + tid;
            inst[u] = -1;
            if (r < n) take(u, r, instance_id[r], start_iter[r], prompt_tokens[r], i_begin[r], i_end[r], sign[r]);
        }
    }
    __syncthreads();
    // exclusive scan of the per-instance counts: each thread a run of instances, the threads' totals by
    // wavefront shuffles, the wavefronts' totals through LDS
    const int per = (n_inst + kBinThreads - 1) / kBinThreads;
    const int k0 = min(tid * per, n_inst), k1 = min(k0 + per, n_inst);
    int run = 0;
    for (int k = k0; k < k1; ++k) run += s_cnt[k];
    int incl = run;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    int at = incl - run, total = 0;
    for (int w = 0; w < kBinThreads / 64; ++w) {
        if (w < wave) at += s_wave[w];
        total += s_wave[w];
    }
    // table[k][chunk] = where instance k's entries start in this chunk's region (row n_inst: where they all end);
    // instance-major, so that the workgroup that folds instance k reads two contiguous rows
    int32_t* tcol = table + chunk;
    for (int k = k0; k < k1; ++k) {
        const int c = s_cnt[k];
        s_cnt[k] = at;
        tcol[(int64_t)k * n_chunks] = at;
        at += c;
    }
    if (tid == 0) tcol[(int64_t)n_inst * n_chunks] = total;
    __syncthreads();
    // grouped in LDS first, so that the chunk's region is written with whole 16-byte pieces per lane
#pragma unroll
    for (int u = 0; u < kBinPerThread; ++u)
        if (inst[u] >= 0) s_ent[s_cnt[inst[u]] + rank[u]] = ent[u];
    __syncthreads();
    ulonglong2* out = (ulonglong2*)(entries + base);
    const ulonglong2* src = (const ulonglong2*)s_ent;
    for (int i = tid; i < (total + 1) / 2; i += kBinThreads) out[i] = src[i];
    if (overflow)
        for (int i = tid; i < n_inst; i += kBinThreads)
            if (s_ovf[i] != 0) atomicAdd((unsigned long long*)(overflow + i), (unsigned long long)s_ovf[i]);
}

// One workgroup per instance: its entries from every chunk into an LDS row, then the scan of that row
// into the caller's map (same arithmetic as lookahead_scan_kernel).
__global__ __launch_bounds__(1024) void lookahead_consume_kernel(
    const unsigned long long* __restrict__ entries, const int32_t* __restrict__ table, int64_t n_chunks, int n_inst,
    int map_len, int32_t* __restrict__ kv_tokens, const int32_t* __restrict__ capacity, float* __restrict__ fraction,
    ps_status* st) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    long long* s_off = (long long*)lds_raw;                               // [map_len] offset differences
    int* s_slp = (int*)(s_off + map_len);                                 // [map_len] slope differences
    __shared__ long long s_w0[16], s_w1[16];
    const int k = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < map_len; i += 1024) { s_off[i] = 0; s_slp[i] = 0; }
    __syncthreads();
    auto apply = [&](unsigned long long v) {
        const unsigned lo = (unsigned)(v & 0x1ffffu), hi = (unsigned)((v >> 17) & 0x1ffffu);
        const long long off = (long long)((v >> 34) & 0x7ffffu) - (1 << 18);
        const bool neg = (v >> 53) & 1u;
        const long long a = neg ? -off : off;                             // sign * (P - s)
        const int sl = neg ? -1 : 1;
        atomicAdd((unsigned long long*)&s_off[lo], (unsigned long long)a);
        atomicAdd(&s_slp[lo], sl);
        if (hi < (unsigned)map_len) {
            atomicAdd((unsigned long long*)&s_off[hi], (unsigned long long)(-a));
            atomicAdd(&s_slp[hi], -sl);
        }
    };
    // wavefront w takes chunks 64 w .. 64 w + 63, then 1024 further on; their bounds are fetched together (one chunk
    // per lane), and the first 64 entries of eight chunks are requested before any is applied
    for (int64_t c0 = (int64_t)wave * 64; c0 < n_chunks; c0 += 16 * 64) {
        const int64_t mine = c0 + lane;
        int seg_b = 0, seg_e = 0;
        if (mine < n_chunks) {
            seg_b = table[(int64_t)k * n_chunks + mine];
            seg_e = table[(int64_t)(k + 1) * n_chunks + mine];
        }
        constexpr int UC = 8;
        for (int j0 = 0; j0 < 64; j0 += UC) {
            if (c0 + j0 >= n_chunks) break;                               // uniform
            int b[UC], e[UC];
            unsigned long long first[UC];
#pragma unroll
            for (int u = 0; u < UC; ++u) {
                b[u] = __shfl(seg_b, j0 + u, 64);                          // (chunks past the end: empty segments)
                e[u] = __shfl(seg_e, j0 + u, 64);
                const unsigned long long* src = entries + (c0 + j0 + u) * kBinChunk;
                first[u] = b[u] + lane < e[u] ? src[b[u] + lane] : 0ull;
            }
#pragma unroll
            for (int u = 0; u < UC; ++u) {
                if (b[u] + lane < e[u]) apply(first[u]);
                const unsigned long long* src = entries + (c0 + j0 + u) * kBinChunk;
                for (int i = b[u] + 64 + lane; i < e[u]; i += 64) apply(src[i]);
            }
        }
    }
    __syncthreads();
    int32_t* out = kv_tokens + (int64_t)k * map_len;
    float* frow = fraction ? fraction + (int64_t)k * map_len : nullptr;
    const int cap = fraction ? capacity[k] : 1;
    const float cap_f = cap >= 1 ? (float)cap : __builtin_nanf("");      // no capacity: fractions are NaN
    long long carry0 = 0, carry1 = 0;
    for (int t0 = 0; t0 < map_len; t0 += 4096) {
        const int t = t0 + 4 * tid;
        long long a0[4], a1[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            a0[c] = t + c < map_len ? s_off[t + c] : 0;
            a1[c] = t + c < map_len ? (long long)s_slp[t + c] : 0;
        }
#pragma unroll
        for (int c = 1; c < 4; ++c) { a0[c] += a0[c - 1]; a1[c] += a1[c - 1]; }
        long long i0 = a0[3], i1 = a1[3];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const long long u0 = __shfl_up(i0, o, 64), u1 = __shfl_up(i1, o, 64);
            if (lane >= o) { i0 += u0; i1 += u1; }
        }
        if (lane == 63) { s_w0[wave] = i0; s_w1[wave] = i1; }
        __syncthreads();
        long long before0 = carry0 + i0 - a0[3], before1 = carry1 + i1 - a1[3];
        long long tot0 = 0, tot1 = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) { before0 += s_w0[w]; before1 += s_w1[w]; }
            tot0 += s_w0[w];
            tot1 += s_w1[w];
        }
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

// Layout of the workspace: the difference array of the atomic route, then the binned route's entries and table.
struct LookaheadPlan {
    bool binned;                 // the call qualifies for the binned route
    size_t diff_bytes, entries_at, entries_bytes, table_at, table_bytes, total_bytes;
    int64_t part;                // records per part of the route taken
};

LookaheadPlan plan_lookahead(int64_t n_rec, int n_inst, int map_len) {
    LookaheadPlan p;
    p.diff_bytes = align_up((size_t)n_inst * (size_t)map_len * 8, 256);
    p.binned = n_rec >= kBinMinRecords && n_inst <= kBinMaxInst && (int64_t)map_len * 12 <= kRowLdsBytes;
    p.part = p.binned ? kBinPart : (int64_t)1 << 22;
    p.entries_at = p.diff_bytes;
    p.entries_bytes = p.table_bytes = 0;
    if (p.binned) {
        const int64_t most = n_rec < kBinPart ? n_rec : kBinPart;
        const int64_t chunks = (most + kBinChunk - 1) / kBinChunk;
        p.entries_bytes = align_up((size_t)chunks * kBinChunk * 8, 256);
        p.table_bytes = align_up((size_t)chunks * (size_t)(n_inst + 1) * 4, 256);
    }
    p.table_at = p.entries_at + p.entries_bytes;
    p.total_bytes = p.table_at + p.table_bytes;
    return p;
}
}  // namespace

extern "C" size_t ps_lookahead_workspace_bytes(int64_t n_rec, int32_t n_inst, int32_t map_len) {
    if (n_rec < 0 || n_inst < 1 || map_len < 1 || map_len > PS_MAX_ITER + 1) return 0;
    return plan_lookahead(n_rec, n_inst, map_len).total_bytes;
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
    const LookaheadPlan plan = plan_lookahead(n_rec, n_inst, map_len);
    const size_t need = plan.total_bytes;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < need) return PS_EWORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    (void)hipGetLastError();
    const int64_t n16 = (int64_t)(plan.diff_bytes / 16);
    const unsigned clear_blocks = (unsigned)((n16 + 255) / 256 < 2048 ? (n16 + 255) / 256 : 2048);
    if (plan.binned) {
        static bool lds_attr_set = false;     // raising the limit twice is harmless, so no lock
        if (!lds_attr_set) {
            if (hipFuncSetAttribute((const void*)lookahead_consume_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kRowLdsBytes) != hipSuccess ||
                hipFuncSetAttribute((const void*)lookahead_bin_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kBinChunk * 8 + kBinMaxInst * 12) != hipSuccess ||
                hipFuncSetAttribute((const void*)lookahead_bin_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    kBinChunk * 8 + kBinMaxInst * 12) != hipSuccess)
                return PS_EHIP;
            lds_attr_set = true;
        }
        unsigned long long* entries = (unsigned long long*)((uint8_t*)workspace + plan.entries_at);
        int32_t* table = (int32_t*)((uint8_t*)workspace + plan.table_at);
        const bool vec = (((uintptr_t)instance_id | (uintptr_t)start_iter | (uintptr_t)prompt_tokens | (uintptr_t)i_begin |
                           (uintptr_t)i_end | (uintptr_t)sign) & 15) == 0;       // (parts start at multiples of 2^26 records)
        for (int64_t at = 0; at < n_rec; at += plan.part) {
            const int64_t n_part = n_rec - at < plan.part ? n_rec - at : plan.part;
            const bool last = at + plan.part >= n_rec;
            const int64_t chunks = (n_part + kBinChunk - 1) / kBinChunk;
            if (vec)
                hipLaunchKernelGGL(lookahead_bin_kernel<true>, dim3((unsigned)chunks), dim3(kBinThreads), (size_t)kBinChunk * 8 + (size_t)n_inst * 12, s,
                                   instance_id + at, start_iter + at, prompt_tokens + at, i_begin + at, i_end + at, sign + at,
                                   n_part, at, n_inst, map_len, entries, table, chunks, overflow, status);
            else
                hipLaunchKernelGGL(lookahead_bin_kernel<false>, dim3((unsigned)chunks), dim3(kBinThreads), (size_t)kBinChunk * 8 + (size_t)n_inst * 12, s,
                                   instance_id + at, start_iter + at, prompt_tokens + at, i_begin + at, i_end + at, sign + at,
                                   n_part, at, n_inst, map_len, entries, table, chunks, overflow, status);
            hipLaunchKernelGGL(lookahead_consume_kernel, dim3((unsigned)n_inst), dim3(1024), (size_t)map_len * 12, s, entries,
                               table, chunks, n_inst, map_len, kv_tokens, capacity, last ? fraction : nullptr, status);
        }
        return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
    }
    // parts of at most plan.part records: the packed differences of one slot cannot overflow their fields within
    // a part (see the top of this file); the map accumulates, so the parts add up to the whole
    const int64_t kPart = plan.part;
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
