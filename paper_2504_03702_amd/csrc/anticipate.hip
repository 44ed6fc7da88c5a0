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
// slice with coalesced loads and applies the updates of the records whose instance is in its
// group to its private LDS rows, then writes the rows to a partial buffer.  The groups of one
// slice are placed on the same XCD so the slice is fetched from HBM once and shared through L2.
// Kernel 2 (reduce): one workgroup per instance sums the partial difference rows, takes the prefix
// sum over buckets and accumulates into load[]; overflow[] likewise.  No global atomics: every
// global word has exactly one writer.  All arithmetic is integer, so the result is exact and
// independent of record order.
#include <string.h>

#include "device_util.h"
#include "internal.h"

namespace {

const int kLdsBytes = 160 * 1024;        // LDS of one gfx950 compute unit
const int kScatterThreads = 1024;
const int64_t kMinSlice = 16384;         // records per slice below which more slices do not pay
const int kTargetWorkgroups = 256;       // one scatter workgroup per compute unit

struct AntPlan {
    int rows_per_group, groups, slices;
    int64_t slice_len;
    size_t lds_bytes, partial_bytes, ovf_bytes, total_bytes;
    bool ok;
};

AntPlan make_plan(int64_t n, int n_inst, int horizon) {
    AntPlan p;
    memset(&p, 0, sizeof(p));
    const int64_t per_row = 4 * (int64_t)horizon + 8 + 4;      // difference row + overflow + rate
    const int64_t fit = (kLdsBytes - 64) / per_row;
    if (fit < 1) return p;
    p.groups = (int)((n_inst + fit - 1) / fit);
    p.rows_per_group = (n_inst + p.groups - 1) / p.groups;
    int64_t s = (n + kMinSlice - 1) / kMinSlice;
    const int64_t cap = kTargetWorkgroups / p.groups > 0 ? kTargetWorkgroups / p.groups : 1;
    if (s > cap) s = cap;
    if (s < 1) s = 1;
    p.slices = (int)s;
    p.slice_len = (n + s - 1) / s;
    p.slice_len = (p.slice_len + 3) / 4 * 4;
    p.lds_bytes = (size_t)(p.rows_per_group * per_row);
    p.partial_bytes = align_up((size_t)p.slices * n_inst * horizon * 4, 256);
    p.ovf_bytes = align_up((size_t)p.slices * n_inst * 8, 256);
    p.total_bytes = p.partial_bytes + p.ovf_bytes;
    p.ok = true;
    return p;
}

__global__ __launch_bounds__(kScatterThreads) void anticipate_scatter_kernel(
    const int32_t* __restrict__ pred_tokens, const int32_t* __restrict__ instance_id,
    const int32_t* __restrict__ arrival_bucket, const int32_t* __restrict__ rate, int64_t n, int n_inst,
    int horizon, int rows_per_group, int groups, int slices, int64_t slice_len,
    int32_t* __restrict__ partial, int64_t* __restrict__ partial_ovf, ps_status* st) {
    extern __shared__ __align__(8) unsigned char lds_raw[];
    // blocks are dealt to the 8 XCDs round-robin: keep the groups of one slice on one XCD
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int g = j % groups;
    const int slice = (j / groups) * 8 + xcd;
    if (slice >= slices) return;
    const int k0 = g * rows_per_group;
    const int rows = min(rows_per_group, n_inst - k0);
    if (rows <= 0) return;
    unsigned long long* s_ovf = (unsigned long long*)lds_raw;                  // [rows_per_group]
    int* s_rate = (int*)(s_ovf + rows_per_group);                              // [rows_per_group]
    int* s_diff = s_rate + rows_per_group;                                     // [rows_per_group][horizon]
    const int tid = threadIdx.x;
    for (int i = tid; i < rows * horizon; i += kScatterThreads) s_diff[i] = 0;
    for (int i = tid; i < rows; i += kScatterThreads) {
        s_ovf[i] = 0;
        s_rate[i] = rate ? rate[k0 + i] : 1;
    }
    __syncthreads();

    const int64_t begin = (int64_t)slice * slice_len;
    const int64_t end = min(begin + slice_len, n);
    unsigned long long mass = 0;      // bound on the magnitude any difference cell can have reached
    for (int64_t i = begin + tid; i < end; i += kScatterThreads) {
        const int k = instance_id[i];
        if ((unsigned)k >= (unsigned)n_inst) {
            if (g == 0) report_fault(st, PS_ST_BAD_RECORD, i);
            continue;
        }
        const int kk = k - k0;
        if ((unsigned)kk >= (unsigned)rows) continue;
        const int D = pred_tokens[i];
        const int a = arrival_bucket[i];
        const int r = s_rate[kk];
        if ((unsigned)D > (unsigned)PS_MAX_PRED || (unsigned)a >= (unsigned)horizon || r < 1) {
            report_fault(st, PS_ST_BAD_RECORD, i);
            continue;
        }
        if (D == 0) continue;
        const unsigned dur = rate ? ((unsigned)D + (unsigned)r - 1u) / (unsigned)r : (unsigned)(horizon - a);
        const unsigned q = (unsigned)D / dur;
        const unsigned rem = (unsigned)D - q * dur;
        int* row = s_diff + kk * horizon + a;
        const unsigned room = (unsigned)(horizon - a);      // buckets from a to the end of the row
        atomicAdd(row, (int)(q + 1));
        if (rem < room) atomicAdd(row + rem, -1);
        if (dur < room) {
            atomicAdd(row + dur, -(int)q);
        } else if (dur > room) {
            const unsigned long long inside = (unsigned long long)room * q + min(room, rem);
            atomicAdd(&s_ovf[kk], (unsigned long long)D - inside);
        }
        mass += q + 1;
    }
    // a cell can only have wrapped if the updates of this workgroup's 16 wavefronts add up to
    // 2^31 or more, i.e. if some wavefront contributed at least 2^27
    for (int o = 32; o > 0; o >>= 1) mass += __shfl_xor(mass, o, 64);
    if ((tid & 63) == 0 && mass >= (1ull << 27)) report_fault(st, PS_ST_RANGE, begin);
    __syncthreads();
    int32_t* out = partial + ((int64_t)slice * n_inst + k0) * horizon;
    for (int i = tid; i < rows * horizon; i += kScatterThreads) out[i] = s_diff[i];
    for (int i = tid; i < rows; i += kScatterThreads) partial_ovf[(int64_t)slice * n_inst + k0 + i] = (int64_t)s_ovf[i];
}

__global__ __launch_bounds__(256) void anticipate_reduce_kernel(const int32_t* __restrict__ partial,
                                                                const int64_t* __restrict__ partial_ovf,
                                                                int slices, int n_inst, int horizon,
                                                                int32_t* __restrict__ load,
                                                                int64_t* __restrict__ overflow, ps_status* st) {
    __shared__ long long s_scan[256];
    const int k = blockIdx.x, tid = threadIdx.x;
    const int64_t stride = (int64_t)n_inst * horizon;
    long long carry = 0;
    for (int b0 = 0; b0 < horizon; b0 += 256) {
        const int b = b0 + tid;
        long long v = 0;
        if (b < horizon) {
            const int32_t* p = partial + (int64_t)k * horizon + b;
            for (int s = 0; s < slices; ++s) v += p[s * stride];
        }
        s_scan[tid] = v;
        __syncthreads();
        for (int d = 1; d < 256; d <<= 1) {
            const long long t = tid >= d ? s_scan[tid - d] : 0;
            __syncthreads();
            s_scan[tid] += t;
            __syncthreads();
        }
        const long long incl = carry + s_scan[tid];
        if (b < horizon) {
            const long long nv = (long long)load[(int64_t)k * horizon + b] + incl;
            if (nv > 2147483647ll || nv < -2147483648ll) report_fault(st, PS_ST_RANGE, -1);
            load[(int64_t)k * horizon + b] = (int32_t)(uint32_t)(unsigned long long)nv;
        }
        carry += s_scan[255];
        __syncthreads();
    }
    if (tid == 0 && overflow) {
        long long o = 0;
        for (int s = 0; s < slices; ++s) o += partial_ovf[(int64_t)s * n_inst + k];
        if (o) overflow[k] += o;
    }
}

}  // namespace

extern "C" size_t ps_anticipate_workspace_bytes(int64_t n_req, int32_t n_inst, int32_t horizon) {
    if (n_req < 0 || n_inst < 1 || horizon < 1) return 0;
    AntPlan p = make_plan(n_req, n_inst, horizon);
    return p.ok ? p.total_bytes : 0;
}

extern "C" int ps_anticipate(const int32_t* pred_tokens, const int32_t* instance_id,
                             const int32_t* arrival_bucket, const int32_t* rate, int64_t n_req,
                             int32_t n_inst, int32_t horizon, int32_t* load, int64_t* overflow,
                             void* workspace, size_t workspace_bytes, ps_status* status, void* hip_stream) {
    if (n_req < 0 || n_inst < 1 || horizon < 1 || !load) return PS_EINVAL;
    if (rate && !overflow) return PS_EINVAL;
    if (n_req == 0) return PS_OK;
    if (!pred_tokens || !instance_id || !arrival_bucket || !workspace) return PS_EINVAL;
    if ((int64_t)n_inst * horizon > (int64_t)0x7fffffff) return PS_EUNSUPPORTED;
    AntPlan p = make_plan(n_req, n_inst, horizon);
    if (!p.ok) return PS_EUNSUPPORTED;
    if (((uintptr_t)workspace & 255) != 0 || workspace_bytes < p.total_bytes) return PS_EWORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    (void)hipGetLastError();
    static bool lds_attr_set = false;     // raising the limit twice is harmless, so no lock
    if (!lds_attr_set) {
        if (hipFuncSetAttribute((const void*)anticipate_scatter_kernel,
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
            return PS_EHIP;
        lds_attr_set = true;
    }
    int32_t* partial = (int32_t*)workspace;
    int64_t* partial_ovf = (int64_t*)((uint8_t*)workspace + p.partial_bytes);
    const unsigned blocks = 8u * (unsigned)p.groups * (unsigned)((p.slices + 7) / 8);
    hipLaunchKernelGGL(anticipate_scatter_kernel, dim3(blocks), dim3(kScatterThreads), p.lds_bytes, s,
                       pred_tokens, instance_id, arrival_bucket, rate, n_req, n_inst, horizon,
                       p.rows_per_group, p.groups, p.slices, p.slice_len, partial, partial_ovf, status);
    hipLaunchKernelGGL(anticipate_reduce_kernel, dim3((unsigned)n_inst), dim3(256), 0, s, partial, partial_ovf,
                       p.slices, n_inst, horizon, load, overflow, status);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}
