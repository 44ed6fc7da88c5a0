// Load anticipator (paper Sec. 3.4.1): fold per-request predicted response lengths into the
// per-instance future-load curves load[instance][one-second bucket].
//
// A request is two range additions on its instance's row: buckets [a, a + rem) take q + 1 tokens
// and [a + rem, a + dur) take q, with q = D / dur, rem = D % dur.  Range additions are point
// updates of the row's difference array (+q+1 at a, -1 at a+rem, -q at a+dur), so a record costs
// three integer updates however long it decodes; the curve is the prefix sum of the differences.
//
// Kernel 1 (scatter): the map's rows are split into groups that fit one compute unit's LDS as
// difference arrays; the records are split into slices.  Workgroup (group, slice) streams its
// slice with coalesced 16-byte loads (four records per lane).  Each wavefront compacts the records
// whose instance is in its group into a small LDS queue (ballot + prefix count, no atomics) and,
// whenever 64 are queued, applies them with every lane busy: two exact divisions by float
// reciprocal and three LDS adds into the workgroup's private rows.  At the end the rows go to a
// partial buffer.  The groups of one slice are placed on the same XCD so the slice is fetched from
// HBM once and shared through that XCD's L2.
// Kernel 2 (reduce): one workgroup per instance sums the partial difference rows, takes the prefix
// sum over buckets and accumulates into load[]; overflow[] likewise.  No global atomics: every
// global word has exactly one writer; the only atomic operations are the LDS adds of kernel 1.  All arithmetic is integer, so the result is exact and
// independent of record order.
//
// Records in arrival order (a request log, the order requests are admitted in) allow a cheaper first
// kernel, tried first on long streams: a slice of such a stream touches few buckets, so its workgroup
// keeps a window of buckets for ALL instances in LDS (256 x 152 counters) instead of all buckets for a
// quarter of them.  Every record then belongs to the one workgroup that reads it: no second, third
// and fourth inspection by other groups, no compaction queue.  A workgroup that meets a record
// outside its window says so in place of its result; that makes the general kernel run after it
// (otherwise its workgroups leave at once) and tells the reduction which partial results to use, so
// the outcome is the same for any order.
#include <string.h>

#include <mutex>
#include <type_traits>

#include "device_util.h"
#include "internal.h"

namespace {

const int kLdsBytes = 160 * 1024;        // LDS of one gfx950 compute unit
const int kWaves = 16;                   // wavefronts per scatter workgroup
const int kScatterThreads = kWaves * 64;
const int kQueue = 128;                  // entries of a wavefront's compaction queue
const int kQueueBytes = kWaves * kQueue * 4;
const int64_t kMinSlice = 16384;         // records per slice below which more slices do not pay
const int kTargetWorkgroups = 256;       // one scatter workgroup per compute unit

const int64_t kWindowMinRecords = 262144;   // shorter streams do not pay for the extra launches
const int kWindowMaxHorizon = 4096;         // the reduction keeps one 64-bit row of the map in LDS
const int kGaveUp = -2;                     // a windowed workgroup's origin when a record fell outside its window

struct AntPlan {
    int rows_per_group, groups, slices;
    int64_t slice_len;
    size_t lds_bytes, partial_bytes, ovf_bytes, total_bytes;
    // windowed first kernel (records in arrival order); w_slices == 0: not used
    int w_slices, w_buckets;
    int64_t w_slice_len;
    size_t w_lds_bytes, w_partial_bytes, w_ovf_bytes, w_origin_bytes, w_partial_at, w_ovf_at, w_origin_at;
    bool ok;
};

AntPlan make_plan(int64_t n, int n_inst, int horizon) {
    AntPlan p;
    memset(&p, 0, sizeof(p));
    if (horizon > 65535) return p;
    const int64_t per_row = 4 * (int64_t)horizon + 8 + 8;      // difference row + overflow + (rate, 1/rate)
    int64_t fit = (kLdsBytes - kQueueBytes - 64) / per_row;
    if (fit < 1) return p;
    // a queued record names its difference cell (row * horizon + bucket) in 16 bits; LDS capacity
    // already keeps a group below 2^16 cells
    p.groups = (int)((n_inst + fit - 1) / fit);
    p.rows_per_group = (n_inst + p.groups - 1) / p.groups;
    int64_t s = (n + kMinSlice - 1) / kMinSlice;
    const int64_t cap = kTargetWorkgroups / p.groups > 0 ? kTargetWorkgroups / p.groups : 1;
    if (s > cap) s = cap;
    if (s < 1) s = 1;
    p.slices = (int)s;
    p.slice_len = (n + s - 1) / s;
    p.slice_len = (p.slice_len + 3) / 4 * 4;                    // slices start on 16-byte boundaries
    p.lds_bytes = (size_t)(p.rows_per_group * per_row + kQueueBytes + 64);
    p.partial_bytes = align_up((size_t)p.slices * n_inst * horizon * 4, 256);
    p.ovf_bytes = align_up((size_t)p.slices * n_inst * 8, 256);
    p.total_bytes = p.partial_bytes + p.ovf_bytes;
    p.ok = true;
    return p;
}

// Adds the windowed kernel's buffers behind the general ones when the call qualifies for it.
void plan_window(AntPlan& p, int64_t n, int n_inst, int horizon, bool with_rate) {
    p.w_slices = 0;
    if (!p.ok || !with_rate || n < kWindowMinRecords || horizon > kWindowMaxHorizon) return;
    const int64_t fixed = 64 + (int64_t)n_inst * 16;             // flag + overflow + (rate, 1/rate)
    int64_t wb = (kLdsBytes - fixed) / ((int64_t)n_inst * 4);
    if (wb > horizon) wb = horizon;
    if (wb < horizon) wb &= ~(int64_t)3;                          // whole 16-byte groups for the reduction's loads
    if (wb < 32) return;
    int64_t s = (n + kMinSlice - 1) / kMinSlice;
    if (s > kTargetWorkgroups) s = kTargetWorkgroups;
    p.w_slices = (int)s;
    p.w_buckets = (int)wb;
    p.w_slice_len = ((n + s - 1) / s + 3) / 4 * 4;
    p.w_lds_bytes = (size_t)(fixed + (int64_t)n_inst * wb * 4);
    p.w_partial_bytes = align_up((size_t)s * n_inst * wb * 4, 256);
    p.w_ovf_bytes = align_up((size_t)s * n_inst * 8, 256);
    p.w_origin_bytes = align_up((size_t)s * 4, 256);
    p.w_partial_at = p.total_bytes;
    p.w_ovf_at = p.w_partial_at + p.w_partial_bytes;
    p.w_origin_at = p.w_ovf_at + p.w_ovf_bytes;
    p.total_bytes = p.w_origin_at + p.w_origin_bytes;
}

// Exact integer division by float reciprocals.  All numerators here are below 2^20
// (pred_tokens <= PS_MAX_PRED < 2^16, rates clamped to PS_MAX_PRED, which changes no result because a
// rate above the prediction already gives a duration of one bucket; cell indices below 2^16).  For a numerator N < 2^20 and a
// divisor d, let x = N / d.  An estimate e with x < x (1 + 2.5 * 2^-23) <= e <= x (1 + 1.3 * 2^-20) has
// floor(e) = floor(x): e is never below x, and x is either an integer or at least 1/d below the
// next one, while e - x <= N * 1.3 * 2^-20 / d < 1/d.  Both estimates below stay inside that band:
//   - row reciprocal: fl(fl(1/r) * (1 + 2^-21)), then one multiply: factors (1 + 2^-21)(1 +- 2^-24)^3;
//   - v_rcp_f32 (1 ulp) times N times (1 + 2^-20): factors (1 + 2^-20)(1 +- 2^-23)(1 +- 2^-24)^2.
__device__ __forceinline__ unsigned div_by_row(unsigned num, float biased_rcp) {
    return (unsigned)((float)num * biased_rcp);
}
__device__ __forceinline__ unsigned div_exact(unsigned num, unsigned den) {
    return (unsigned)(((float)num * __builtin_amdgcn_rcpf((float)den)) * (1.0f + 0x1p-20f));
}

// True if some workgroup of the windowed kernel gave up.  Every wavefront looks through all the origins
// itself, so the answer is the same across the workgroup without a barrier or LDS.
__device__ __forceinline__ bool window_gave_up(const int32_t* __restrict__ worigin, int w_slices) {
    bool mine = false;
    for (int s = threadIdx.x & 63; s < w_slices; s += 64) mine |= worigin[s] == kGaveUp;
    return __any(mine) != 0;
}

__global__ __launch_bounds__(kScatterThreads) void anticipate_scatter_kernel(
    const int32_t* __restrict__ pred_tokens, const int32_t* __restrict__ instance_id,
    const int32_t* __restrict__ arrival_bucket, const int32_t* __restrict__ rate, int64_t n, int n_inst,
    int horizon, int rows_per_group, int groups, int slices, int64_t slice_len,
    int32_t* __restrict__ partial, int64_t* __restrict__ partial_ovf, const int32_t* __restrict__ worigin,
    int w_slices, ps_status* st) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    // launched behind the windowed kernel: needed only if that one gave up somewhere
    if (worigin && !window_gave_up(worigin, w_slices)) return;
    // blocks are dealt to the 8 XCDs round-robin: keep the groups of one slice on one XCD
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int g = j % groups;
    const int slice = (j / groups) * 8 + xcd;
    if (slice >= slices) return;
    const int k0 = g * rows_per_group;
    const int rows = min(rows_per_group, n_inst - k0);
    if (rows <= 0) return;
    uint32_t* s_queue = (uint32_t*)lds_raw;                                    // [kWaves][kQueue]
    int* s_flag = (int*)(lds_raw + kQueueBytes);                               // [1] some row has rate < 1
    unsigned long long* s_ovf = (unsigned long long*)(lds_raw + kQueueBytes + 64);  // [rows_per_group]
    int2* s_rr = (int2*)(s_ovf + rows_per_group);                              // (rate, biased 1/rate)
    int* s_diff = (int*)(s_rr + rows_per_group);                               // [rows_per_group][horizon]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) *s_flag = 0;
    __syncthreads();
    for (int i = tid; i < rows * horizon; i += kScatterThreads) s_diff[i] = 0;
    for (int i = tid; i < rows; i += kScatterThreads) {
        s_ovf[i] = 0;
        int r = rate ? rate[k0 + i] : 1;
        if (r < 1) { *s_flag = 1; r = 0; }
        r = min(r, PS_MAX_PRED);
        const float rcp = r > 0 ? (1.0f / (float)r) * (1.0f + 0x1p-21f) : 0.f;
        s_rr[i] = make_int2(r, __float_as_int(rcp));
    }
    __syncthreads();
    const bool bad_rate_rows = *s_flag != 0;                 // uniform; rare

    uint32_t* q = s_queue + wave * kQueue;
    const float rcp_horizon = (1.0f / (float)horizon) * (1.0f + 0x1p-21f);
    unsigned head = 0, tail = 0;                                // wave-uniform ring indices
    unsigned long long mass = 0;       // bound on the magnitude any difference cell can have reached

    // Apply up to 64 queued records (lane i takes entry head + i): all lanes busy on the divisions.
    auto consume = [&](unsigned count) {
        if ((unsigned)lane < count) {
            // entry: difference cell of the arrival bucket (row * horizon + bucket) | prediction
            const uint32_t e = q[(head + lane) & (kQueue - 1)];
            const unsigned D = e & 0xffffu, cell = e >> 16;
            const unsigned kk = div_by_row(cell, rcp_horizon), a = cell - kk * (unsigned)horizon;
            const int2 rr = s_rr[kk];
            unsigned dur;
            if (rate) dur = div_by_row(D + (unsigned)rr.x - 1u, __int_as_float(rr.y));
            else dur = (unsigned)horizon - a;
            const unsigned qq = div_exact(D, dur);
            const unsigned rem = D - qq * dur;
            int* row = s_diff + cell;
            const unsigned room = (unsigned)horizon - a;        // buckets from a to the end of the row
            atomicAdd(row, (int)(qq + 1));
            if (rem < room) atomicAdd(row + rem, -1);
            if (dur < room) {
                atomicAdd(row + dur, -(int)qq);
            } else if (dur > room) {
                const unsigned long long inside = (unsigned long long)room * qq + min(room, rem);
                atomicAdd(&s_ovf[kk], (unsigned long long)D - inside);
            }
            mass += qq + 1;
        }
    };

    const int64_t begin = (int64_t)slice * slice_len;
    const int64_t end = min(begin + slice_len, n);

    // Four consecutive records per lane, 256 per wavefront and block.  Loads run two blocks ahead of
    // the block being processed, so six 16-byte loads per lane are in flight while the wavefront works.
    // The last, partial block of a slice is read record by record.
    struct Block {
        int k[4], d[4], a[4];
        bool ragged;                                            // lane crosses the end of the slice
    };
    // Full blocks are loaded unconditionally (straight-line code keeps the memory counter exact, so
    // a block can be used while the two after it are still in flight); a prefetch past the last
    // full block is redirected to it and never used.
    const int64_t n_full = (end - begin) / 256;
    const int64_t last_full = begin + (n_full - 1) * 256;
    auto load_full = [&](int64_t blk) {
        Block b;
        const int64_t idx = min(blk, last_full) + lane * 4;
        // plain loads: the four row groups of a slice run on one XCD and share the slice through its L2 (with
        // the non-temporal hint the other three groups fetch it again: 0.258 against 0.225 ms on 44.1 M records)
        const int4 kv = *(const int4*)(instance_id + idx);
        const int4 dv = *(const int4*)(pred_tokens + idx);
        const int4 av = *(const int4*)(arrival_bucket + idx);
        b.k[0] = kv.x; b.k[1] = kv.y; b.k[2] = kv.z; b.k[3] = kv.w;
        b.d[0] = dv.x; b.d[1] = dv.y; b.d[2] = dv.z; b.d[3] = dv.w;
        b.a[0] = av.x; b.a[1] = av.y; b.a[2] = av.z; b.a[3] = av.w;
        b.ragged = false;
        return b;
    };
    auto load_ragged = [&](int64_t blk) {
        Block b;
        const int64_t idx = blk + lane * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool in = idx + c < end;
            b.k[c] = in ? instance_id[idx + c] : -1;            // -1 never matches a group
            b.d[c] = in ? pred_tokens[idx + c] : 0;
            b.a[c] = in ? arrival_bucket[idx + c] : 0;
        }
        b.ragged = idx < end;
        return b;
    };
    auto process_block = [&](const Block& b, int64_t blk) {
        const int64_t idx = blk + lane * 4;
        // validity of all four records at once; a block with a faulty record, or the ragged tail,
        // is checked record by record
        const unsigned dmax = max(max((unsigned)b.d[0], (unsigned)b.d[1]), max((unsigned)b.d[2], (unsigned)b.d[3]));
        const unsigned amax = max(max((unsigned)b.a[0], (unsigned)b.a[1]), max((unsigned)b.a[2], (unsigned)b.a[3]));
        const unsigned kmax = max(max((unsigned)b.k[0], (unsigned)b.k[1]), max((unsigned)b.k[2], (unsigned)b.k[3]));
        const bool suspect = b.ragged || dmax > (unsigned)PS_MAX_PRED || amax >= (unsigned)horizon ||
                             kmax >= (unsigned)n_inst;
        const bool slow = __any(suspect) || bad_rate_rows;      // uniform
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned kk = (unsigned)(b.k[c] - k0);
            bool m = kk < (unsigned)rows && b.d[c] != 0;
            if (slow) {
                const bool in = idx + c < end;
                const bool k_ok = (unsigned)b.k[c] < (unsigned)n_inst;
                bool ok = (unsigned)b.d[c] <= (unsigned)PS_MAX_PRED && (unsigned)b.a[c] < (unsigned)horizon;
                if (kk < (unsigned)rows && ok && s_rr[kk].x < 1) ok = false;
                // a record outside every group is reported by group 0, others by their own group
                if (in && ((!k_ok && g == 0) || (kk < (unsigned)rows && !ok))) report_fault(st, PS_ST_BAD_RECORD, idx + c);
                m = m && in && ok;
            }
            const unsigned long long mask = __ballot(m);
            if (mask) {
                const unsigned pos = tail + __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                                   __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
                if (m) q[pos & (kQueue - 1)] = ((kk * (unsigned)horizon + (unsigned)b.a[c]) << 16) | (unsigned)b.d[c];
                tail += (unsigned)__popcll(mask);
                if (tail - head >= 64u) {
                    consume(64u);
                    head += 64u;
                }
            }
        }
    };

    const int64_t stride = (int64_t)kWaves * 256;
    const int64_t blk0 = begin + (int64_t)wave * 256;
    const int64_t full_end = begin + n_full * 256;
    if (blk0 < full_end) {
        // three register sets used in rotation (unrolled, so no set is ever copied: a copy would
        // have to wait for the load it copies)
        Block b0 = load_full(blk0);
        Block b1 = load_full(blk0 + stride);
        Block b2 = load_full(blk0 + 2 * stride);
        for (int64_t blk = blk0;;) {
            process_block(b0, blk);
            b0 = load_full(blk + 3 * stride);
            if ((blk += stride) >= full_end) break;
            process_block(b1, blk);
            b1 = load_full(blk + 3 * stride);
            if ((blk += stride) >= full_end) break;
            process_block(b2, blk);
            b2 = load_full(blk + 3 * stride);
            if ((blk += stride) >= full_end) break;
        }
    }
    if (full_end < end && wave == (int)(n_full % kWaves)) process_block(load_ragged(full_end), full_end);
    if (tail != head) consume(tail - head);

    // a cell can only have wrapped if the updates of this workgroup's wavefronts add up to 2^31 or
    // more, i.e. if some wavefront contributed at least 2^31 / kWaves
    for (int o = 32; o > 0; o >>= 1) mass += __shfl_xor(mass, o, 64);
    if (lane == 0 && mass >= (1ull << 31) / kWaves) report_fault(st, PS_ST_RANGE, begin);
    __syncthreads();
    int32_t* out = partial + ((int64_t)slice * n_inst + k0) * horizon;
    for (int i = tid; i < rows * horizon; i += kScatterThreads) out[i] = s_diff[i];
    for (int i = tid; i < rows; i += kScatterThreads) partial_ovf[(int64_t)slice * n_inst + k0 + i] = (int64_t)s_ovf[i];
}

// Windowed scatter for records in arrival order: workgroup = slice of the records; LDS holds, for
// every instance, the difference counters of the buckets [a0, a0 + w_buckets), a0 = the arrival bucket
// of the slice's first record.  Each lane takes its own records straight through the two divisions and
// the three LDS adds.  A record that reaches outside the window (or before it) makes the workgroup
// leave kGaveUp in place of its origin; the general kernel then redoes the whole call.
__global__ __launch_bounds__(kScatterThreads) void anticipate_window_kernel(
    const int32_t* __restrict__ pred_tokens, const int32_t* __restrict__ instance_id,
    const int32_t* __restrict__ arrival_bucket, const int32_t* __restrict__ rate, int64_t n, int n_inst,
    int horizon, int w_buckets, int64_t slice_len, int32_t* __restrict__ wpartial,
    int64_t* __restrict__ wovf, int32_t* __restrict__ worigin, ps_status* st) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    int* s_flag = (int*)lds_raw;                                              // [0] a row has rate < 1, [1] gave up
    unsigned long long* s_ovf = (unsigned long long*)(lds_raw + 64);          // [n_inst]
    int2* s_rr = (int2*)(s_ovf + n_inst);                                      // (rate, biased 1/rate)
    int* s_diff = (int*)(s_rr + n_inst);                                       // [n_inst][w_buckets]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slice = blockIdx.x;
    const int64_t begin = (int64_t)slice * slice_len;
    const int64_t end = min(begin + slice_len, n);
    if (begin >= end) {
        if (tid == 0) worigin[slice] = -1;                    // nothing to add from this slice
        return;
    }
    // window origin: the slice's first arrival bucket; a faulty (negative) one must not shift the window the
    // slice's valid records are placed in, so the origin is never below bucket 0 (a first bucket at or beyond
    // the horizon leaves every valid record before the window: the workgroup gives up and the general kernel runs)
    const int a0 = max(arrival_bucket[begin], 0);
    if (tid < 2) s_flag[tid] = 0;
    __syncthreads();
    {
        // A look at the slice's first records before anything is set up: a stream in no particular order shows a
        // valid arrival bucket outside the window at once, and the workgroup leaves without clearing its counters.
        // (Invalid buckets are not counted: such records are skipped, not folded.)
        const int64_t probe = begin + (int64_t)tid * 4;
        bool far = false;
        if (probe + 4 <= end) {
            const int4 av = *(const int4*)(arrival_bucket + probe);
            const int aa[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                far |= (unsigned)aa[c] < (unsigned)horizon && (unsigned)(aa[c] - a0) >= (unsigned)w_buckets;
        }
        if (__any(far) && lane == 0) s_flag[1] = 1;
        __syncthreads();
        if (s_flag[1]) {                                      // uniform
            if (tid == 0) worigin[slice] = kGaveUp;
            return;
        }
    }
    for (int i = tid; i < n_inst * w_buckets; i += kScatterThreads) s_diff[i] = 0;
    for (int i = tid; i < n_inst; i += kScatterThreads) {
        s_ovf[i] = 0;
        int r = rate[i];
        if (r < 1) { s_flag[0] = 1; r = 0; }
        r = min(r, PS_MAX_PRED);
        const float rcp = r > 0 ? (1.0f / (float)r) * (1.0f + 0x1p-21f) : 0.f;
        s_rr[i] = make_int2(r, __float_as_int(rcp));
    }
    __syncthreads();
    const bool bad_rate_rows = s_flag[0] != 0;               // uniform; rare
    unsigned long long mass = 0;       // bound on the magnitude any difference cell can have reached
    unsigned mass32 = 0;               //   (a block's share, folded into it after the block)
    bool outside = false;

    // One record: (validity,) the two divisions, window test, three adds.  CHECKED is only used for
    // blocks that hold a record failing the cheap range test, rows without a usable rate, and the tail.
    // (rr = the instance's (rate, 1 / rate), read by the caller for all of a lane's records before the
    // first add, so that no read queues up behind another record's adds)
    auto take = [&](int k, int D, int a, int2 rr, int64_t idx, bool in, auto checked_tag) {
        constexpr bool CHECKED = decltype(checked_tag)::value;
        if (CHECKED) {
            bool ok = (unsigned)k < (unsigned)n_inst && (unsigned)D <= (unsigned)PS_MAX_PRED && (unsigned)a < (unsigned)horizon;
            if (ok && rr.x < 1) ok = false;
            if (in && !ok) report_fault(st, PS_ST_BAD_RECORD, idx);
            if (!(in && ok)) return;
        }
        const unsigned dur = div_by_row((unsigned)D + (unsigned)rr.x - 1u, __int_as_float(rr.y));
        const unsigned qq = div_exact((unsigned)D, max(dur, 1u));         // D == 0: dur == 0, nothing is added
        const unsigned rem = (unsigned)D - __umul24(qq, dur);        // both below 2^16
        const unsigned room = (unsigned)horizon - (unsigned)a;     // buckets from a to the end of the row
        const unsigned rel = (unsigned)(a - a0);                    // wraps to a huge value before the window
        const unsigned reach = min(dur, room - 1u);                 // furthest bucket touched, from a
        const bool out = rel >= (unsigned)w_buckets || rel + reach >= (unsigned)w_buckets;
        outside |= out && D != 0;
        if (!out && D != 0) {
            int* cell = s_diff + __umul24((unsigned)k, (unsigned)w_buckets) + rel;   // (LDS holds the rows: both small)
            atomicAdd(cell, (int)(qq + (rem != 0)));                // rem == 0: the +1 and the -1 fall on the same cell
            if (rem != 0 && rem < room) atomicAdd(cell + rem, -1);
            if (dur < room) {
                atomicAdd(cell + dur, -(int)qq);
            } else if (dur > room) {
                const unsigned long long inside = (unsigned long long)room * qq + min(room, rem);
                atomicAdd(&s_ovf[k], (unsigned long long)D - inside);
            }
            mass32 += qq + 1;
        }
    };
    using Checked = std::true_type;
    using Unchecked = std::false_type;

    // four consecutive records per lane, 256 per wavefront and block, loads two blocks ahead
    const int64_t n_full = (end - begin) / 256;
    const int64_t last_full = begin + (n_full - 1) * 256;
    struct Blk { int4 k, d, a; };
    auto load_full = [&](int64_t blk) {
        Blk b;
        const int64_t idx = min(blk, last_full) + lane * 4;
        b.k = load_stream_int4(instance_id + idx);
        b.d = load_stream_int4(pred_tokens + idx);
        b.a = load_stream_int4(arrival_bucket + idx);
        return b;
    };
    auto process = [&](const Blk& b, int64_t blk) {
        const int64_t idx = blk + lane * 4;
        // range test of all four records at once; a block with a suspect record is checked record by record
        const unsigned dmax = max(max((unsigned)b.d.x, (unsigned)b.d.y), max((unsigned)b.d.z, (unsigned)b.d.w));
        const unsigned amax = max(max((unsigned)b.a.x, (unsigned)b.a.y), max((unsigned)b.a.z, (unsigned)b.a.w));
        const unsigned kmax = max(max((unsigned)b.k.x, (unsigned)b.k.y), max((unsigned)b.k.z, (unsigned)b.k.w));
        const bool suspect = dmax > (unsigned)PS_MAX_PRED || amax >= (unsigned)horizon || kmax >= (unsigned)n_inst;
        const int kk[4] = {b.k.x, b.k.y, b.k.z, b.k.w}, dd[4] = {b.d.x, b.d.y, b.d.z, b.d.w}, aa[4] = {b.a.x, b.a.y, b.a.z, b.a.w};
        int2 rr[4];
        if (__any(suspect) || bad_rate_rows) {
#pragma unroll
            for (int c = 0; c < 4; ++c) rr[c] = (unsigned)kk[c] < (unsigned)n_inst ? s_rr[kk[c]] : make_int2(0, 0);
#pragma unroll
            for (int c = 0; c < 4; ++c) take(kk[c], dd[c], aa[c], rr[c], idx + c, true, Checked{});
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) rr[c] = s_rr[kk[c]];
#pragma unroll
            for (int c = 0; c < 4; ++c) take(kk[c], dd[c], aa[c], rr[c], idx + c, true, Unchecked{});
        }
        mass += mass32;
        mass32 = 0;
    };
    const int64_t stride = (int64_t)kWaves * 256;
    const int64_t blk0 = begin + (int64_t)wave * 256;
    const int64_t full_end = begin + n_full * 256;
    if (blk0 < full_end) {
        Blk b0 = load_full(blk0);
        Blk b1 = load_full(blk0 + stride);
        Blk b2 = load_full(blk0 + 2 * stride);
        for (int64_t blk = blk0;;) {
            process(b0, blk);
            b0 = load_full(blk + 3 * stride);
            if ((blk += stride) >= full_end || __any(outside)) break;
            process(b1, blk);
            b1 = load_full(blk + 3 * stride);
            if ((blk += stride) >= full_end || __any(outside)) break;
            process(b2, blk);
            b2 = load_full(blk + 3 * stride);
            if ((blk += stride) >= full_end || __any(outside)) break;
        }
    }
    if (full_end < end && wave == (int)(n_full % kWaves)) {
        const int64_t idx = full_end + lane * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool in = idx + c < end;
            const int k = in ? instance_id[idx + c] : 0;
            take(k, in ? pred_tokens[idx + c] : 0, in ? arrival_bucket[idx + c] : 0,
                 (unsigned)k < (unsigned)n_inst ? s_rr[k] : make_int2(0, 0), idx + c, in, Checked{});
        }
    }
    mass += mass32;
    if (__any(outside) && lane == 0) s_flag[1] = 1;
    for (int o = 32; o > 0; o >>= 1) mass += __shfl_xor(mass, o, 64);
    if (lane == 0 && mass >= (1ull << 31) / kWaves) report_fault(st, PS_ST_RANGE, begin);
    __syncthreads();
    if (s_flag[1]) {                                          // uniform: the general kernel takes over
        if (tid == 0) worigin[slice] = kGaveUp;
        return;
    }
    // instance-major: wpartial[instance][slice][bucket of the window], so that the reduction of an
    // instance reads one contiguous block
    const float inv_wb = 1.0f / (float)w_buckets;
    for (int i = tid; i < n_inst * w_buckets; i += kScatterThreads) {
        int k = (int)(((float)i + 0.5f) * inv_wb);
        int r = i - k * w_buckets;
        if (r < 0) { r += w_buckets; --k; }
        if (r >= w_buckets) { r -= w_buckets; ++k; }
        wpartial[((int64_t)k * gridDim.x + slice) * w_buckets + r] = s_diff[i];
    }
    for (int i = tid; i < n_inst; i += kScatterThreads) wovf[(int64_t)slice * n_inst + i] = (int64_t)s_ovf[i];
    if (tid == 0) worigin[slice] = a0;
}

// One workgroup per instance.  Where the horizon is short enough for a 64-bit row of the map in LDS, all
// 1024 threads first stream this instance's partial rows (one per slice: the whole horizon from the
// general kernel, a window at its origin from the windowed one) and add them into that row: the
// (slice, cell) pairs are dealt to the threads in order, so loads are contiguous runs, 16 in flight per
// thread, and the lanes of an LDS add hit different cells.  Longer horizons sum the general kernel's
// rows bucket by bucket.  Then buckets are taken 1024 at a time, thread t < 256 owning the four
// consecutive buckets 4 t .. 4 t + 3: it prefix-sums its four values, the 256 thread totals are scanned
// with wavefront shuffles, and the curve is accumulated into load[].  64-bit sums, so a bucket leaving
// the int32 range is seen exactly.
const int kReduceThreads = 1024;

__global__ __launch_bounds__(kReduceThreads) void anticipate_reduce_kernel(
    const int32_t* __restrict__ partial, const int64_t* __restrict__ partial_ovf, int slices, int n_inst, int horizon,
    const int32_t* __restrict__ wpartial, const int64_t* __restrict__ wovf, const int32_t* __restrict__ worigin,
    int w_slices, int w_buckets, int32_t* __restrict__ load, int64_t* __restrict__ overflow, ps_status* st) {
    __shared__ long long s_wave[4];
    __shared__ unsigned long long s_over;
    __shared__ int s_origin[kTargetWorkgroups];              // first bucket of every slice's row
    __shared__ unsigned long long s_row[kWindowMaxHorizon];  // this instance's difference row, 64-bit
    const int k = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // which first kernel produced the partial results: the windowed one unless it gave up
    const bool windowed = worigin && !window_gave_up(worigin, w_slices);
    const bool in_lds = horizon <= kWindowMaxHorizon;         // (the windowed kernel is only used then)
    if (tid == 0) s_over = 0;                                 // (a barrier follows before its first use)
    if (in_lds) {
        const int n_rows = windowed ? w_slices : slices, row_len = windowed ? w_buckets : horizon;
        for (int s = tid; s < n_rows; s += kReduceThreads) s_origin[s] = windowed ? worigin[s] : 0;
        for (int i = tid; i < horizon; i += kReduceThreads) s_row[i] = 0;
        __syncthreads();
        // general partials are [slice][instance][bucket], windowed ones [instance][slice][bucket of the window]
        const int32_t* rk = windowed ? wpartial + (int64_t)k * n_rows * row_len : partial + (int64_t)k * row_len;
        const int64_t rstride = windowed ? (int64_t)row_len : (int64_t)n_inst * row_len;
        const int total = n_rows * row_len;                   // at most 256 * 4096
        const float inv_len = 1.0f / (float)row_len;
        if ((row_len & 3) == 0) {
            // rows of whole 16-byte groups (every row then starts on a 16-byte boundary): four cells a load,
            // all of a thread's loads requested before the first is used
            const int groups = row_len >> 2, total4 = n_rows * groups;
            const float inv_groups = 1.0f / (float)groups;
            constexpr int NB = 12;
            for (int e0 = tid; e0 < total4; e0 += kReduceThreads * NB) {
                int4 v[NB];
                int cell[NB];
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    const int e = min(e0 + kReduceThreads * u, total4 - 1);
                    int sl = (int)(((float)e + 0.5f) * inv_groups);
                    int g4 = e - sl * groups;
                    if (g4 < 0) { g4 += groups; --sl; }
                    if (g4 >= groups) { g4 -= groups; ++sl; }
                    v[u] = *(const int4*)(rk + sl * rstride + 4 * g4);
                    const int a0 = s_origin[sl];              // -1: a slice that added nothing
                    cell[u] = (e0 + kReduceThreads * u < total4 && a0 >= 0) ? a0 + 4 * g4 : -1;
                }
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    if (cell[u] < 0) continue;
                    const int x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (x[c] != 0 && cell[u] + c < horizon) atomicAdd(&s_row[cell[u] + c], (unsigned long long)(long long)x[c]);
                }
            }
        } else {
            constexpr int NB = 16;                            // loads requested before the first is used
            for (int e0 = tid; e0 < total; e0 += kReduceThreads * NB) {
                int32_t v[NB];
                int cell[NB];
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    const int e = min(e0 + kReduceThreads * u, total - 1);
                    int sl = (int)(((float)e + 0.5f) * inv_len);
                    int i = e - sl * row_len;
                    if (i < 0) { i += row_len; --sl; }
                    if (i >= row_len) { i -= row_len; ++sl; }
                    v[u] = rk[sl * rstride + i];
                    const int a0 = s_origin[sl];              // -1: a slice that added nothing
                    cell[u] = (e0 + kReduceThreads * u < total && a0 >= 0 && a0 + i < horizon) ? a0 + i : -1;
                }
#pragma unroll
                for (int u = 0; u < NB; ++u)
                    if (cell[u] >= 0 && v[u] != 0) atomicAdd(&s_row[cell[u]], (unsigned long long)(long long)v[u]);
            }
        }
        __syncthreads();
    }
    const int64_t stride = (int64_t)n_inst * horizon;
    const int32_t* prow = partial + (int64_t)k * horizon;
    int32_t* lrow = load + (int64_t)k * horizon;
    const bool worker = tid < 256;                            // the scan is the first four wavefronts' work
    long long carry = 0;
    for (int b0 = 0; b0 < horizon; b0 += 1024) {
        const int b = b0 + 4 * (tid & 255);
        long long v[4] = {0, 0, 0, 0};
        if (worker) {
            if (in_lds) {
#pragma unroll
                for (int c = 0; c < 4; ++c) if (b + c < horizon) v[c] = (long long)s_row[b + c];
            } else {
                int s = 0;
                for (; s + 4 <= slices; s += 4) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int32_t* p = prow + (s + u) * stride;
#pragma unroll
                        for (int c = 0; c < 4; ++c) if (b + c < horizon) v[c] += p[b + c];
                    }
                }
                for (; s < slices; ++s) {
                    const int32_t* p = prow + s * stride;
#pragma unroll
                    for (int c = 0; c < 4; ++c) if (b + c < horizon) v[c] += p[b + c];
                }
            }
        }
        v[1] += v[0]; v[2] += v[1]; v[3] += v[2];
        // inclusive scan of the thread totals: within a wavefront by shuffles, then across the four
        long long incl = v[3];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const long long t = __shfl_up(incl, o, 64);
            if (lane >= o) incl += t;
        }
        if (worker && lane == 63) s_wave[wave] = incl;
        __syncthreads();
        long long before = carry + incl - v[3];
        for (int w = 0; w < (wave & 3); ++w) before += s_wave[w];
        const long long total = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
        if (worker) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (b + c < horizon) {
                    const long long nv = (long long)lrow[b + c] + before + v[c];
                    if (nv > 2147483647ll || nv < -2147483648ll) report_fault(st, PS_ST_RANGE, -1);
                    lrow[b + c] = (int32_t)(uint32_t)(unsigned long long)nv;
                }
            }
        }
        carry += total;
        __syncthreads();
    }
    // tokens past the horizon: one slice per thread, added up in LDS
    if (overflow) {
        const int n_rows = windowed ? w_slices : slices;
        for (int s2 = tid; s2 < n_rows; s2 += kReduceThreads) {
            long long o = 0;
            if (windowed) {
                if (worigin[s2] >= 0) o = wovf[(int64_t)s2 * n_inst + k];
            } else {
                o = partial_ovf[(int64_t)s2 * n_inst + k];
            }
            if (o) atomicAdd(&s_over, (unsigned long long)o);
        }
        __syncthreads();
        if (tid == 0 && s_over) overflow[k] += (long long)s_over;
    }
}

}  // namespace

extern "C" size_t ps_anticipate_workspace_bytes(int64_t n_req, int32_t n_inst, int32_t horizon) {
    if (n_req < 0 || n_inst < 1 || horizon < 1) return 0;
    AntPlan p = make_plan(n_req, n_inst, horizon);
    plan_window(p, n_req, n_inst, horizon, true);
    return p.ok ? p.total_bytes : 0;
}

namespace {

// Validates the arguments and enqueues the kernels of one call on `s`, with `workspace` (device memory of at
// least `workspace_bytes` bytes) for the partial curves.
int anticipate_enqueue(const int32_t* pred_tokens, const int32_t* instance_id, const int32_t* arrival_bucket,
                       const int32_t* rate, int64_t n_req, int32_t n_inst, int32_t horizon, int32_t* load,
                       int64_t* overflow, void* workspace, size_t workspace_bytes, ps_status* status, hipStream_t s) {
    if (n_req < 0 || n_inst < 1 || horizon < 1 || !load) return PS_EINVAL;
    if (rate && !overflow) return PS_EINVAL;
    if (n_req == 0) return PS_OK;
    if (!pred_tokens || !instance_id || !arrival_bucket || !workspace) return PS_EINVAL;
    if ((((uintptr_t)pred_tokens | (uintptr_t)instance_id | (uintptr_t)arrival_bucket) & 15) != 0) return PS_EINVAL;
    if ((int64_t)n_inst * horizon > (int64_t)0x7fffffff) return PS_EUNSUPPORTED;
    AntPlan p = make_plan(n_req, n_inst, horizon);
    if (!p.ok) return PS_EUNSUPPORTED;
    {
        // the workspace is sized for the windowed path whether or not this call takes it
        AntPlan sized = p;
        plan_window(sized, n_req, n_inst, horizon, true);
        if (((uintptr_t)workspace & 255) != 0 || workspace_bytes < sized.total_bytes) return PS_EWORKSPACE;
    }
    plan_window(p, n_req, n_inst, horizon, rate != nullptr);
    if (((uintptr_t)workspace & 255) != 0 || workspace_bytes < p.total_bytes) return PS_EWORKSPACE;
    (void)hipGetLastError();
    static bool lds_attr_set = false;     // raising the limit twice is harmless, so no lock
    if (!lds_attr_set) {
        if (hipFuncSetAttribute((const void*)anticipate_scatter_kernel,
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute((const void*)anticipate_window_kernel,
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
            return PS_EHIP;
        lds_attr_set = true;
    }
    uint8_t* wsb = (uint8_t*)workspace;
    int32_t* partial = (int32_t*)wsb;
    int64_t* partial_ovf = (int64_t*)(wsb + p.partial_bytes);
    int32_t* wpartial = nullptr;
    int64_t* wovf = nullptr;
    int32_t* worigin = nullptr;
    if (p.w_slices > 0) {
        wpartial = (int32_t*)(wsb + p.w_partial_at);
        wovf = (int64_t*)(wsb + p.w_ovf_at);
        worigin = (int32_t*)(wsb + p.w_origin_at);
        hipLaunchKernelGGL(anticipate_window_kernel, dim3((unsigned)p.w_slices), dim3(kScatterThreads), p.w_lds_bytes, s,
                           pred_tokens, instance_id, arrival_bucket, rate, n_req, n_inst, horizon, p.w_buckets,
                           p.w_slice_len, wpartial, wovf, worigin, status);
    }
    const unsigned blocks = 8u * (unsigned)p.groups * (unsigned)((p.slices + 7) / 8);
    hipLaunchKernelGGL(anticipate_scatter_kernel, dim3(blocks), dim3(kScatterThreads), p.lds_bytes, s,
                       pred_tokens, instance_id, arrival_bucket, rate, n_req, n_inst, horizon,
                       p.rows_per_group, p.groups, p.slices, p.slice_len, partial, partial_ovf, worigin, p.w_slices, status);
    hipLaunchKernelGGL(anticipate_reduce_kernel, dim3((unsigned)n_inst), dim3(kReduceThreads), 0, s, partial, partial_ovf, p.slices, n_inst, horizon,
                       wpartial, wovf, worigin, p.w_slices, p.w_buckets, load, overflow, status);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}

}  // namespace

extern "C" int ps_anticipate(const int32_t* pred_tokens, const int32_t* instance_id,
                             const int32_t* arrival_bucket, const int32_t* rate, int64_t n_req,
                             int32_t n_inst, int32_t horizon, int32_t* load, int64_t* overflow,
                             void* workspace, size_t workspace_bytes, ps_status* status, void* hip_stream) {
    return anticipate_enqueue(pred_tokens, instance_id, arrival_bucket, rate, n_req, n_inst, horizon, load, overflow,
                              workspace, workspace_bytes, status, (hipStream_t)hip_stream);
}

// ---- the variant for callers that cannot allocate ---------------------------------------------------------
// Its partial curves live in a file-scope device array instead of a caller-provided workspace.  Every GPU the
// library runs on holds its own copy of the array at its own address: the address is looked up once per
// device and kept; host code only ever uses that address, never the array's name.
static __device__ __align__(256) unsigned char scratch[PS_ANTICIPATE_STATIC_BYTES];

namespace {
const int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices];       // per device: device address of `scratch`, null until looked up
}  // namespace

extern "C" int ps_anticipate_static(const int32_t* pred_tokens, const int32_t* instance_id,
                                    const int32_t* arrival_bucket, const int32_t* rate, int64_t n_req,
                                    int32_t n_inst, int32_t horizon, int32_t* load, int64_t* overflow,
                                    ps_status* status, void* hip_stream) {
    if (n_req < 0 || n_inst < 1 || horizon < 1) return PS_EINVAL;
    // sizes beyond the array are refused before anything else is looked at
    const size_t need = ps_anticipate_workspace_bytes(n_req, n_inst, horizon);
    if (need == 0) return PS_EUNSUPPORTED;
    if (need > (size_t)PS_ANTICIPATE_STATIC_BYTES) return PS_EWORKSPACE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return PS_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return PS_EUNSUPPORTED;
    void* ptr;
    {
        std::lock_guard<std::mutex> hold(g_scratch_lock);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PS_EHIP;
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    // the kernels write every partial cell they later read, so the last call's contents need no clearing
    return anticipate_enqueue(pred_tokens, instance_id, arrival_bucket, rate, n_req, n_inst, horizon, load, overflow,
                              ptr, (size_t)PS_ANTICIPATE_STATIC_BYTES, status, (hipStream_t)hip_stream);
}
