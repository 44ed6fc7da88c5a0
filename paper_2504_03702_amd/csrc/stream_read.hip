// Measurement hook: a kernel that does nothing but read a device buffer once, as fast as this library knows
// how (16-byte loads, eight in flight per lane, the load width and depth of the anticipator's record kernels).  The rate it reaches is the yardstick the record kernels' bandwidth is read
// against: the published HBM peak is not reachable by any kernel.  The buffer's 64-bit words are XOR-ed into
// *sink so that the reads cannot be dropped and the result can be checked.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace {

const int kReadThreads = 1024;
const int kReadUnroll = 8;

// 16 bytes that will not be read again: the non-temporal hint keeps them from displacing anything in the caches
// (measured on a 529 MB buffer: 6.7 TB/s with it, 6.0 without)
__device__ __forceinline__ uint4 load_once(const uint4* p) {
    uint4 v;
    v.x = __builtin_nontemporal_load(&p->x);
    v.y = __builtin_nontemporal_load(&p->y);
    v.z = __builtin_nontemporal_load(&p->z);
    v.w = __builtin_nontemporal_load(&p->w);
    return v;
}

__global__ __launch_bounds__(kReadThreads) void stream_read_kernel(const uint4* __restrict__ src, int64_t n16,
                                                                   unsigned long long* __restrict__ sink) {
    // workgroup b takes the 128 KB chunks b, b + grid, ...: at any moment the grid reads one contiguous window,
    // spread evenly over the memory channels
    constexpr int64_t kChunk = (int64_t)kReadThreads * kReadUnroll;          // 16-byte groups per chunk
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    for (int64_t c = (int64_t)blockIdx.x * kChunk; c < n16; c += (int64_t)gridDim.x * kChunk) {
        if (c + kChunk <= n16) {
            uint4 v[kReadUnroll];
#pragma unroll
            for (int u = 0; u < kReadUnroll; ++u) v[u] = load_once(src + c + (int64_t)u * kReadThreads + threadIdx.x);
#pragma unroll
            for (int u = 0; u < kReadUnroll; ++u) {
                acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w;
            }
        } else {
            for (int64_t i = c + threadIdx.x; i < n16; i += kReadThreads) {
                const uint4 v = load_once(src + i);
                acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
            }
        }
    }
    unsigned lo = acc.x ^ acc.z, hi = acc.y ^ acc.w;         // the two 64-bit words of a 16-byte group, folded
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        lo ^= __shfl_xor(lo, o, 64);
        hi ^= __shfl_xor(hi, o, 64);
    }
    // one atomic per workgroup: thousands of them on one address would take longer than the reads
    __shared__ unsigned long long part[kReadThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = (unsigned long long)lo | ((unsigned long long)hi << 32);
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long x = 0;
        for (int w = 0; w < kReadThreads / 64; ++w) x ^= part[w];
        atomicXor(sink, x);
    }
}

}  // namespace

extern "C" int ps_profile_stream_read(const void* data, int64_t bytes, uint64_t* sink, void* hip_stream) {
    if (!data || !sink || bytes < 0 || (bytes & 15) != 0 || ((uintptr_t)data & 15) != 0) return PS_EINVAL;
    if (bytes == 0) return PS_OK;
    const int64_t n16 = bytes >> 4;
    // one workgroup of 1024 threads per compute unit (128 KB requested per workgroup at a time), fewer for small buffers
    int64_t blocks = (n16 + (int64_t)kReadThreads * kReadUnroll - 1) / ((int64_t)kReadThreads * kReadUnroll);
    if (blocks > 256) blocks = 256;
    (void)hipGetLastError();
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(kReadThreads), 0, (hipStream_t)hip_stream,
                       (const uint4*)data, n16, (unsigned long long*)sink);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}
