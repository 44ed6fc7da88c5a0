// The per-request side maps (one row per request: the error-compensated output projection and feed-forward
// block of each request's first row, and the last layer's queries) for calls of at most 16 requests.
//
//   C[r, n] = sum_k A[r, k] * W[n, k]  for r < 16, then the same epilogues as the tiled GEMM's per-request forms.
//
// With so few rows the map is a stream over W: the tiled kernel would put one 128-row tile per 128 columns on
// a handful of compute units and walk the whole contraction there, slice after slice, each waiting out a trip to
// memory.  Here a workgroup owns 64 output columns and its 8 wavefronts split the contraction: each issues
// v_mfma_f32_16x16x32_bf16 on fragments loaded straight from global memory (A: request r = lane % 16, sixteen
// consecutive k per lane and 64-deep round; W the same with its row = output column), several rounds' loads
// requested before the first is used.  Where A carries each value as hi + lo, a W fragment serves both parts.  The wavefronts' partial 16 x 64 results are added through LDS in a fixed order; one wavefront applies
// the epilogue.  Results differ from the tiled kernel's in the last bits (another order of additions), so a
// request's prediction in a call of at most 16 requests need not be bit-equal to the same request's in a larger
// call.
#include "device_util.h"
#include "internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

const int kSkinnyWaves = 8;
const int kSkinnyCols = 64;      // output columns per workgroup: one piece of the rows' partial statistics

// sum over the 16 lanes that share lane / 16, every one of them gets it; fixed order
__device__ __forceinline__ float sum16(float v) {
    v += __shfl_xor(v, 1, 64);
    v += __shfl_xor(v, 2, 64);
    v += __shfl_xor(v, 4, 64);
    v += __shfl_xor(v, 8, 64);
    return v;
}

// DUAL: A holds each row as two bf16 values per element, hi in columns [0, K) and lo in [K, 2K) (row stride 2K),
// and W's rows are read over their first K columns only (row stride ldw): every W fragment serves two MFMAs.
template <int EPI, bool DUAL>
__global__ __launch_bounds__(kSkinnyWaves * 64) void skinny_gemm_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const float* __restrict__ bias, ResidualSrc res,
    void* __restrict__ Cv, int N, int K, int ldw, int hidden, const int32_t* __restrict__ n_rows) {
    __shared__ f32x4 s_part[kSkinnyWaves][4][64];      // [wavefront][column group][lane]: 16 rows x 16 columns each
    __shared__ f32x4 s_sum[4][64];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int frow = lane & 15, fq = lane >> 4;
    const int n0 = blockIdx.x * kSkinnyCols;

    // ---- what the epilogue will need from memory, requested before the contraction starts (wavefront 0) ------
    // Element e of column group g in a lane is C[4 * fq + e, n0 + 16 g + frow].
    const int rows = *n_rows;
    bool live[4] = {false, false, false, false};
    int64_t srow[4] = {0, 0, 0, 0};                     // first row of request 4 fq + e in the stream
    float2 st[4];
    float yprev[4][4];                                  // previous sums of the stream at (request e, column group g)
    float bv[4], cs[4] = {0.f, 0.f, 0.f, 0.f}, gm[4] = {0.f, 0.f, 0.f, 0.f}, bt[4] = {0.f, 0.f, 0.f, 0.f};
    if (wave == 0) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int c = n0 + 16 * g + frow;
            bv[g] = bias[c];
            if (EPI == EPI_Q_MAPPED) cs[g] = res.colsum[c];
            if (EPI == EPI_RESIDUAL_MAPPED) { gm[g] = res.gamma[c]; bt[g] = res.beta[c]; }
        }
        if (EPI != EPI_GELU_SPLIT) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int r = 4 * fq + e;               // the request; uniform over the 16 lanes that share fq
                live[e] = r < rows && res.seq_len[r] > 0;
                srow[e] = live[e] ? res.row_map[r] : 0;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                st[e] = res.stats[srow[e]];
                if (EPI == EPI_RESIDUAL_MAPPED) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int64_t at = srow[e] * N + n0 + 16 * g + frow;
                        yprev[e][g] = bf16_to_f32(res.y_hi[at]) + bf16_to_f32(res.y_lo[at]);
                    }
                }
            }
        }
    }

    // ---- contraction: this wavefront's share of k, 64 deep per round (two MFMA steps): a lane reads 32
    // consecutive bytes of its row, the four lanes of a row one whole 128-byte line ---------------------------
    const int total_rounds = K / 64;                    // dealt to the wavefronts as evenly as whole rounds allow
    const int r_begin = wave * total_rounds / kSkinnyWaves, rounds = (wave + 1) * total_rounds / kSkinnyWaves - r_begin;
    const int lda = DUAL ? 2 * K : K;
    const bf16_t* ap = A + (int64_t)frow * lda + 64 * r_begin + 16 * fq;
    const bf16_t* wp = W + (int64_t)(n0 + frow) * ldw + 64 * r_begin + 16 * fq;
    const int64_t wg = (int64_t)16 * ldw;               // next column group: 16 rows of W further
    f32x4 acc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int U = DUAL ? 3 : 4;                     // rounds whose loads are in flight together
    for (int t0 = 0; t0 < rounds; t0 += U) {
        bf16x8 fa[U][2], fl[DUAL ? U : 1][2], fw[U][4][2];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = min(t0 + u, rounds - 1);      // (past the end: the last round again, not used)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                fa[u][h] = *(const bf16x8*)(ap + 64 * t + 8 * h);
                if (DUAL) fl[u][h] = *(const bf16x8*)(ap + K + 64 * t + 8 * h);
#pragma unroll
                for (int g = 0; g < 4; ++g) fw[u][g][h] = *(const bf16x8*)(wp + g * wg + 64 * t + 8 * h);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (t0 + u < rounds) {
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[u][h], fw[u][g][h], acc[g], 0, 0, 0);
                        if (DUAL) acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fl[u][h], fw[u][g][h], acc[g], 0, 0, 0);
                    }
            }
        }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) s_part[wave][g][lane] = acc[g];
    __syncthreads();
    if (wave < 4) {                                     // column group `wave`: the eight partial results in order
        f32x4 t = s_part[0][wave][lane];
#pragma unroll
        for (int w = 1; w < kSkinnyWaves; ++w) {
            const f32x4 p = s_part[w][wave][lane];
            t[0] += p[0]; t[1] += p[1]; t[2] += p[2]; t[3] += p[3];
        }
        s_sum[wave][lane] = t;
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int g = 0; g < 4; ++g) acc[g] = s_sum[g][lane];
    if (EPI == EPI_GELU_SPLIT) {
        bf16_t* C = (bf16_t*)Cv;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t r = 4 * fq + e;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int c = n0 + 16 * g + frow;
                const float v = gelu_erf(acc[g][e] + bv[g]);
                const bf16_t hi = f32_to_bf16(v);
                C[r * 2 * N + c] = hi;
                C[r * 2 * N + N + c] = f32_to_bf16(v - bf16_to_f32(hi));
            }
        }
        return;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t row = srow[e];
        if (EPI == EPI_Q_MAPPED) {
            bf16_t* C = (bf16_t*)Cv;
            const float nm = -st[e].x * st[e].y;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float v = fmaf(acc[g][e], st[e].y, fmaf(nm, cs[g], bv[g]));
                if (live[e]) C[row * 2 * hidden + n0 + 16 * g + frow] = f32_to_bf16(v);
            }
        } else {
            bf16_t* Cl = (bf16_t*)Cv;
            float sm = 0.f, sq = 0.f;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int c = n0 + 16 * g + frow;
                const float o = acc[g][e] + bv[g] + ((yprev[e][g] - st[e].x) * st[e].y * gm[g] + bt[g]);
                sm += o;
                sq = fmaf(o, o, sq);
                if (live[e]) {
                    const bf16_t hi = f32_to_bf16(o);
                    res.x_out[row * N + c] = hi;
                    Cl[row * N + c] = f32_to_bf16(o - bf16_to_f32(hi));
                }
            }
            if (res.pstats) {
                sm = sum16(sm);
                sq = sum16(sq);
                if (live[e] && frow == 0) res.pstats[row * (N >> 6) + (n0 >> 6)] = make_float2(sm, sq);
            }
        }
    }
}

}  // namespace

// Requirements: at most 16 rows in use (A holds at least 16 rows, the unused ones finite), N % 64 == 0,
// K % 64 == 0 (both hold for every per-request map of a bf16 model: K is its hidden or feed-forward width).  EPI_GELU_SPLIT and
// EPI_RESIDUAL_MAPPED take A as [16][2K] (hi | lo) and W with row stride 2K (each row repeated: only its first
// half is read); EPI_Q_MAPPED takes A as [16][K] and W with row stride K.
void launch_skinny_gemm_bf16(GemmEpilogue epi, const bf16_t* A, const bf16_t* W, const float* bias, ResidualSrc residual,
                             void* C, int N, int K, int hidden, const int32_t* n_rows, hipStream_t s) {
    const dim3 grid((unsigned)(N / kSkinnyCols)), block(kSkinnyWaves * 64);
    switch (epi) {
        case EPI_GELU_SPLIT:
            hipLaunchKernelGGL((skinny_gemm_kernel<EPI_GELU_SPLIT, true>), grid, block, 0, s, A, W, bias, residual, C, N, K, 2 * K, hidden, n_rows);
            break;
        case EPI_RESIDUAL_MAPPED:
            hipLaunchKernelGGL((skinny_gemm_kernel<EPI_RESIDUAL_MAPPED, true>), grid, block, 0, s, A, W, bias, residual, C, N, K, 2 * K, hidden, n_rows);
            break;
        case EPI_Q_MAPPED:
            hipLaunchKernelGGL((skinny_gemm_kernel<EPI_Q_MAPPED, false>), grid, block, 0, s, A, W, bias, residual, C, N, K, K, hidden, n_rows);
            break;
        default:
            break;                                       // the other epilogues have no per-request form
    }
}
