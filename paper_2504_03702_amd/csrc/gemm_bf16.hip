// bf16 GEMM on the gfx950 matrix cores with fused epilogues.
//
//   C[m, n] = sum_k A[m, k] * W[n, k]   (A: activations [rows][K], W: weights [N][K], both bf16,
//                                        contraction index contiguous; fp32 accumulation)
//   epilogue: + bias[n], then one of: store | erf-GELU, store | + residual stream, store as hi + lo |
//             QKV split (query and key columns to [rows][2H], value columns transposed to
//             Vt[H][max_rows] so the attention kernel reads keys-contiguous value tiles), also as
//             keys and values only, and as the queries of mapped rows only.
//   A LayerNorm in front of a map is folded into it: the operand is the row before normalisation,
//   W carries the LayerNorm's scale, and the epilogue finishes with the row's (mean, 1/std):
//   rstd * (acc - mean * colsum[n]) + d[n].  The residual epilogues produce such operands: they write
//   the new sums as two bf16 values hi + lo (hi is the operand) and leave per-row partial sums for the
//   statistics.
//
// One workgroup computes a BM x BN tile.  Per 64-deep k slice the A and W sub-tiles are brought
// straight from global memory into LDS (global_load_lds, 16 bytes per lane, no register staging),
// double buffered; each wavefront then reads 32 x 16 fragments with ds_read_b128 and issues
// v_mfma_f32_32x32x16_bf16.  LDS rows are 128 bytes (64 bf16); the 16-byte chunks of a row are
// XOR-swizzled with the row index so that the 8 or 16 rows one ds_read_b128 phase touches fall in
// different banks.  The swizzle is applied on the global side of the DMA (each lane picks which
// chunk it fetches), since the LDS side of a DMA is always lane-linear.
//
// The kernel is persistent: one workgroup per compute unit walks a list of tiles, prefetching the
// first k slices of its next tile while the current one finishes, so only the very first tile pays
// the latency of filling LDS.  The number of rows is only known on the device (padded inputs are
// compacted); each workgroup derives its tile list from it.  Workgroups are dealt to the 8 XCDs
// round-robin by the hardware; the tile list is built so that the tiles in flight on one XCD are
// neighbours that share activation row panels and weight column panels through that XCD's L2.
#include <type_traits>

#include "device_util.h"
#include "internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define GLOBAL_AS __attribute__((address_space(1)))
#define LDS_AS __attribute__((address_space(3)))

// Sum over 8 consecutive lanes (lanes 8 r .. 8 r + 7) with DPP moves; every one of them gets the total.
// The order of the additions is fixed, so the result does not change from run to run.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row8_sum(float v) {
    v = dpp_add<0xB1>(v);      // quad_perm [1, 0, 3, 2]
    v = dpp_add<0x4E>(v);      // quad_perm [2, 3, 0, 1]
    return dpp_add<0x141>(v);  // row_half_mirror: lane i of each group of 8 takes lane 7 - i
}

template <int BM, int BN, int WM, int WN>
struct Tile {
    static constexpr int NW = WM * WN;               // wavefronts per workgroup
    static constexpr int THREADS = NW * 64;
    static constexpr int TM = BM / WM / 32;          // 32 x 32 accumulator tiles per wavefront
    static constexpr int TN = BN / WN / 32;
    static constexpr int A_BYTES = BM * 128;         // one 64-deep slice
    static constexpr int B_BYTES = BN * 128;
    static_assert(NW % 2 == 0 && BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile / wave split");
};

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const float* __restrict__ bias,
    ResidualSrc res, void* __restrict__ Cv, bf16_t* __restrict__ Vt, int64_t vt_ld,
    int N, int K, int hidden, const int32_t* __restrict__ total_rows, int64_t* __restrict__ clk) {
    using T = Tile<BM, BN, WM, WN>;
    constexpr int STAGE = T::A_BYTES + T::B_BYTES;      // an A slice followed by a W slice
    constexpr int EPI_BYTES = 4096;                     // per-wavefront transpose region of the epilogue
    static_assert(2 * STAGE + T::NW * EPI_BYTES <= 160 * 1024, "LDS budget");
    __shared__ __align__(1024) unsigned char smem[2 * STAGE + T::NW * EPI_BYTES];

    // the wavefront index is uniform; saying so keeps everything derived from it in scalar registers
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- this workgroup's tiles --------------------------------------------------------------
    // The grid is persistent (one workgroup per compute unit).  The hardware deals workgroups to the 8
    // XCDs round-robin, so workgroup b runs on XCD b % 8 as its slot b / 8.  Each XCD has its own L2:
    // the tiles in flight on one XCD should share operand panels, and panels should stay there.
    // A workgroup walks its tiles (tm, tn) by one rule: tn += step_n, tm += step_m, and when tn passes
    // the last tile column it wraps and tm += wrap_m.  Three walks use it:
    //  * large problems whose tile columns come in P groups of 4: the 32 workgroups of an XCD form an
    //    8 x 4 block of tiles, the fewest distinct panels for 32 tiles.
    //      - P divides 8: XCD x keeps column group x % P for the whole launch, so that group's weights
    //        (4 x 256 rows of W) stay in its L2, and walks down the row blocks x / P, x / P + 8 / P, ...;
    //        the P XCDs that need a row block work on it at the same time, so it comes from HBM once
    //        and from the memory-side cache for the others.
    //      - otherwise: XCD x takes row blocks x, x + 8, ... and visits the P column groups of each in
    //        turn (the row block is re-read from the memory-side cache, the weights rotate).
    //  * anything else (few tile rows, odd column counts, small grids): XCD x works through the contiguous
    //    run of tiles [x * per_xcd, (x + 1) * per_xcd), n fastest, its workgroups taking every slots-th.
    const int rows = *total_rows;
    const int n_tiles = N / BN, m_tiles = (rows + BM - 1) / BM;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
    int tm, tn, step_m, step_n, wrap_m, n_my;                // first tile, walk, number of tiles of this workgroup
    if (slots == 32 && m_tiles >= 64 && (n_tiles & 3) == 0) {
        const int P = n_tiles >> 2;
        if ((8 % P) == 0) {
            tm = (xcd / P) * 8 + (slot >> 2);
            tn = (xcd % P) * 4 + (slot & 3);
            step_m = 64 / P; step_n = 0; wrap_m = 0;
            n_my = tm < m_tiles ? (m_tiles - tm + step_m - 1) / step_m : 0;
        } else {
            tm = xcd * 8 + (slot >> 2);
            tn = slot & 3;
            step_m = 0; step_n = 4; wrap_m = 64;
            n_my = tm < m_tiles ? P * ((m_tiles - tm + 63) / 64) : 0;
        }
    } else {
        const int tiles = m_tiles * n_tiles;
        const int per_xcd = (tiles + 7) >> 3;
        const int first = xcd * per_xcd + slot, end = min((xcd + 1) * per_xcd, tiles);
        tm = first / n_tiles; tn = first % n_tiles;
        step_m = slots / n_tiles; step_n = slots % n_tiles; wrap_m = 1;
        n_my = first < end ? (end - first + slots - 1) / slots : 0;
    }
    if (n_my == 0) return;
    auto walk = [&](int& m, int& n) {
        n += step_n; m += step_m;
        const bool wrap = n >= n_tiles;
        n -= wrap ? n_tiles : 0;
        m += wrap ? wrap_m : 0;
    };
    // clock probe (profiling only): core cycles and constant-rate ticks over this workgroup's life
    const int64_t clk_c0 = clk ? (int64_t)clock64() : 0, clk_w0 = clk ? (int64_t)wall_clock64() : 0;

    // ---- DMA sources: lane i of a wavefront fetches chunk (i%8)^swz of row i/8 of its group ----
    const int dma_row = wave * 8 + (lane >> 3);
    const int dma_chunk = (lane & 7) ^ lds_swz(dma_row);
    const unsigned lane_off = (unsigned)(dma_row * K + dma_chunk * 8) * 2u;
    const int64_t ld_bytes = (int64_t)K * 2;

    // ---- fragment addresses: row (lane%32) of a 32-row tile, chunks 2*ks + lane/32 ----------
    const int frow = lane & 31, fhalf = lane >> 5;
    const int a_off = (wm * (BM / WM) + frow) * 128;
    const int b_off = (wn * (BN / WN) + frow) * 128;
    int koff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) koff[ks] = ((2 * ks + fhalf) ^ lds_swz(frow)) * 16;

    f32x16 acc[T::TM][T::TN];
    auto clear_acc = [&]() {
#pragma unroll
        for (int i = 0; i < T::TM; ++i)
#pragma unroll
            for (int j = 0; j < T::TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    };

    // Fragment double buffer: while the MFMAs of k-step s run, the ds_reads of step s+1 are in
    // flight.  The 64-deep slices of all this workgroup's tiles form one stream, slice g living in
    // stage g & 1.  Schedule per slice g:
    //   steps 0..2 : read fragments of the next step of this slice | MFMAs of the current step
    //   then       : wait for this wavefront's DMA of slice g+1, workgroup barrier (now every
    //                wavefront has read its last fragments of slice g and slice g+1 is visible),
    //                start the DMA of slice g+2 into the stage slice g occupied
    //   step 3     : read step-0 fragments of slice g+1 | MFMAs of step 3
    // Slices g+1 and g+2 may belong to the next tile: its first two slices land while this tile
    // finishes and runs its epilogue (which has an LDS region of its own), so a tile starts with
    // its operands already in LDS.
    bf16x8 fa0[T::TM], fb0[T::TN], fa1[T::TM], fb1[T::TN];
    auto read_frags = [&](bf16x8* fa, bf16x8* fb, const unsigned char* stage, int ks) {
        const unsigned char* sA = stage + a_off + koff[ks];
        const unsigned char* sB = stage + T::A_BYTES + b_off + koff[ks];
#pragma unroll
        for (int i = 0; i < T::TM; ++i) fa[i] = *(const bf16x8*)(sA + i * 4096);
#pragma unroll
        for (int j = 0; j < T::TN; ++j) fb[j] = *(const bf16x8*)(sB + j * 4096);
    };
    const int nk = K / 64;
    // Prefetch cursor: the next slice to fetch is slice pf_kt of tile (pf_m, pf_n), the pf_it-th of this
    // workgroup.  Once its tiles are used up the cursor parks on the first tile of the problem: the
    // DMAs stay unconditional (straight-line code the scheduler can interleave with the MFMAs) and the
    // parked ones refill LDS stages nobody reads any more.
    int pf_it = 0, pf_m = tm, pf_n = tn, pf_kt = 0, pf_stage = 0;
    const unsigned char* pf_a = (const unsigned char*)(A + (int64_t)pf_m * BM * K);
    const unsigned char* pf_w = (const unsigned char*)(W + (int64_t)pf_n * BN * K);
    // The DMA of a slice is issued in two halves, A rows then W rows, each spread among the MFMAs of
    // one k-step: a wavefront that queues all of a slice's DMA instructions at once waits at the
    // memory pipeline's issue queue and issues no MFMA meanwhile.
    auto prefetch_a = [&](int j) {        // DMA j of the slice's A rows
        const unsigned char* ub = pf_a + pf_kt * 128 + (int64_t)j * (T::NW * 8) * ld_bytes;    // wave-uniform
        __builtin_amdgcn_global_load_lds((const GLOBAL_AS void*)(ub + lane_off),
                                         (LDS_AS void*)(smem + pf_stage * STAGE + (j * T::NW + wave) * 1024), 16, 0, 0);
    };
    auto prefetch_w = [&](int j) {        // DMA j of the slice's W rows
        const unsigned char* ub = pf_w + pf_kt * 128 + (int64_t)j * (T::NW * 8) * ld_bytes;
        __builtin_amdgcn_global_load_lds((const GLOBAL_AS void*)(ub + lane_off),
                                         (LDS_AS void*)(smem + pf_stage * STAGE + T::A_BYTES + (j * T::NW + wave) * 1024), 16, 0, 0);
    };
    auto advance_cursor = [&]() {         // after the W rows: on to the next slice
        pf_stage ^= 1;
        const bool last = ++pf_kt == nk;
        pf_kt = last ? 0 : pf_kt;
        pf_it += last ? 1 : 0;
        int nm = pf_m, nn = pf_n;
        walk(nm, nn);
        const bool parked = pf_it >= n_my;
        pf_m = parked ? 0 : last ? nm : pf_m;
        pf_n = parked ? 0 : last ? nn : pf_n;
        pf_a = (const unsigned char*)(A + (int64_t)pf_m * BM * K);
        pf_w = (const unsigned char*)(W + (int64_t)pf_n * BN * K);
    };
    constexpr int NDMA_A = BM / 8 / T::NW, NDMA_W = BN / 8 / T::NW;

    // One k-step in exact issue order (the scheduler may not move anything across the fences): in
    // each of TM + TN rounds one fragment read for the next step, at most one DMA, and a share of this
    // step's MFMAs.  dma_tag: 0 none, 1 the slice's A rows, 2 its W rows.
    auto k_step = [&](const bf16x8* fa, const bf16x8* fb, bf16x8* na, bf16x8* nb, const unsigned char* rd_stage,
                      int rd_ks, auto dma_tag) {
        constexpr int DMA = decltype(dma_tag)::value;
        constexpr int nR = T::TM + T::TN, nM = T::TM * T::TN;
        static_assert(NDMA_A <= nR && NDMA_W <= nR, "one DMA per round");
        const unsigned char* sA = rd_stage + a_off + koff[rd_ks];
        const unsigned char* sB = rd_stage + T::A_BYTES + b_off + koff[rd_ks];
#pragma unroll
        for (int r = 0; r < nR; ++r) {
            if (r < T::TM) na[r] = *(const bf16x8*)(sA + r * 4096);
            else nb[r - T::TM] = *(const bf16x8*)(sB + (r - T::TM) * 4096);
            if (DMA == 1 && r < NDMA_A) prefetch_a(r);
            if (DMA == 2 && r < NDMA_W) prefetch_w(r);
            // MFMAs [r * nM / nR, (r + 1) * nM / nR) of the step, in row-major order of the wavefront's tiles
#pragma unroll
            for (int m = r * nM / nR; m < (r + 1) * nM / nR; ++m)
                acc[m / T::TN][m % T::TN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[m / T::TN], fb[m % T::TN],
                                                                                   acc[m / T::TN][m % T::TN], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using NoDma = std::integral_constant<int, 0>;
    using ADma = std::integral_constant<int, 1>;
    using WDma = std::integral_constant<int, 2>;

#pragma unroll
    for (int j = 0; j < NDMA_A; ++j) prefetch_a(j);
#pragma unroll
    for (int j = 0; j < NDMA_W; ++j) prefetch_w(j);
    advance_cursor();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NDMA_A; ++j) prefetch_a(j);
    read_frags(fa0, fb0, smem, 0);
    int stage = 0;
    float* stg = (float*)(smem + 2 * STAGE + wave * EPI_BYTES);
    constexpr int WTM = BM / WM, WTN = BN / WN;

    for (int it = 0; it < n_my; ++it, walk(tm, tn)) {
        clear_acc();
        for (int kt = 0; kt < nk; ++kt) {
            unsigned char* cur = smem + stage * STAGE;
            unsigned char* nxt = smem + (stage ^ 1) * STAGE;
            stage ^= 1;
            k_step(fa0, fb0, fa1, fb1, cur, 1, WDma{});       // + W half of the slice after this one
            advance_cursor();
            k_step(fa1, fb1, fa0, fb0, cur, 2, NoDma{});
            k_step(fa0, fb0, fa1, fb1, cur, 3, NoDma{});
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            // reads the step-0 fragments of the next slice, of this tile or of the next one (after the
            // last slice of all: of a stage nobody needs); + A half of the slice two after this one
            k_step(fa1, fb1, fa0, fb0, nxt, 0, ADma{});
        }

        // ---- epilogue -----------------------------------------------------------------------------
        // Accumulator element e of tile (i, j) is C[row, col] with row = 32 i + 8 (e / 4) + 4 (lane / 32)
        // + e % 4, col = 32 j + lane % 32: a lane holds one column.  Each wavefront transposes through
        // its private 4 KB of LDS: it writes a strip of accumulators, reads it back with 16 bytes of
        // consecutive output per lane, applies the epilogue there and issues 16-byte global accesses.
        const int m0 = tm * BM, n0 = tn * BN;
        const int m_base = m0 + wm * WTM, n_base = n0 + wn * WTN;

        // first value column of this launch's W: after the query and key columns, or after the key columns
        const int v_col0 = EPI == EPI_KV ? hidden : 2 * hidden;
        if ((EPI == EPI_QKV || EPI == EPI_KV) && n0 >= v_col0) {
            // Value columns go to Vt[feature][row].  One 32 x 32 accumulator tile at a time is staged as
            // [32 features][32 rows]; the 16-byte chunks of a feature's rows are XOR-swizzled with the
            // feature index so the 128-byte-strided writes of the 32 lanes spread over the banks.  Read
            // back, a lane holds 8 consecutive rows of one feature: the folded LayerNorm is finished there.
            const int rg = lane & 3;
            float cc[T::TN][2], dd[T::TN][2];
#pragma unroll
            for (int j = 0; j < T::TN; ++j)
#pragma unroll
                for (int it = 0; it < 2; ++it) {
                    const int c = n_base + 32 * j + (lane >> 2) + 16 * it;
                    cc[j][it] = res.colsum[c];
                    dd[j][it] = bias[c];
                }
            float2 sv[2][8];                         // statistics of the lane's 8 rows, tile row i and i + 1
            auto fetch_sv = [&](int i) {
#pragma unroll
                for (int r = 0; r < 8; ++r) sv[i & 1][r] = res.stats[m_base + 32 * i + 8 * rg + r];
            };
            fetch_sv(0);
#pragma unroll
            for (int i = 0; i < T::TM; ++i) {
                if (i + 1 < T::TM) fetch_sv(i + 1);
                float rs[8], nm[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    rs[r] = sv[i & 1][r].y;
                    nm[r] = -sv[i & 1][r].x * sv[i & 1][r].y;
                }
#pragma unroll
                for (int j = 0; j < T::TN; ++j) {
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        const f32x16& a = acc[i][j];
                        *(float4*)(stg + frow * 32 + 4 * ((2 * e4 + fhalf) ^ (frow & 7))) =
                            make_float4(a[4 * e4], a[4 * e4 + 1], a[4 * e4 + 2], a[4 * e4 + 3]);
                    }
#pragma unroll
                    for (int it = 0; it < 2; ++it) {
                        const int c = (lane >> 2) + 16 * it;
                        const float4 lo = *(const float4*)(stg + c * 32 + 4 * ((2 * rg) ^ (c & 7)));
                        const float4 hi = *(const float4*)(stg + c * 32 + 4 * ((2 * rg + 1) ^ (c & 7)));
                        const float a8[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                        float v[8];
#pragma unroll
                        for (int r = 0; r < 8; ++r) v[r] = fmaf(a8[r], rs[r], fmaf(nm[r], cc[j][it], dd[j][it]));
                        const uint4 o = make_uint4(cvt_pk_bf16(v[0], v[1]), cvt_pk_bf16(v[2], v[3]),
                                                   cvt_pk_bf16(v[4], v[5]), cvt_pk_bf16(v[6], v[7]));
                        *(uint4*)(Vt + (int64_t)(n_base - v_col0 + 32 * j + c) * vt_ld + m_base + 32 * i + 8 * rg) = o;
                    }
                }
            }
            continue;
        }

        // other epilogues: strips of 8 rows x WTN columns, row-major, padded rows
        constexpr int SW = WTN + 4;
        static_assert(8 * SW * 4 <= EPI_BYTES && 32 * 32 * 4 <= EPI_BYTES, "epilogue staging region");
        auto stage_strip = [&](int i, int e4) {      // rows 32 i + 8 e4 + 0..7 of the wavefront's tile
#pragma unroll
            for (int j = 0; j < T::TN; ++j)
#pragma unroll
                for (int t = 0; t < 4; ++t) stg[(4 * fhalf + t) * SW + 32 * j + frow] = acc[i][j][4 * e4 + t];
        };

        if (EPI == EPI_BIAS_RESIDUAL || EPI == EPI_RESIDUAL_MAPPED) {
            // New sums of the residual stream: v = acc + bias + LayerNorm(y_prev) recomputed from the
            // previous sums (kept as two bf16, hi + lo) and the row statistics, so the stream is never
            // rounded to 8 bits.  v goes out as hi + lo again: hi is what the next map reads.  A lane
            // handles 8 consecutive columns (16-byte accesses), 8 lanes a row of the strip.
            constexpr int LPR = WTN / 8, RPI = 64 / LPR, NIT = 8 / RPI, NS = 4 * T::TM;
            static_assert(LPR == 8 && NIT == 1, "8 lanes per 64-column row piece");
            const int cg = lane % LPR, r_in = lane / LPR;
            const int col = n_base + 8 * cg;
            float bv[8], rg[8], rb[8];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float4 b4 = *(const float4*)(bias + col + 4 * h);
                const float4 g4 = *(const float4*)(res.gamma + col + 4 * h);
                const float4 e4 = *(const float4*)(res.beta + col + 4 * h);
                bv[4 * h] = b4.x; bv[4 * h + 1] = b4.y; bv[4 * h + 2] = b4.z; bv[4 * h + 3] = b4.w;
                rg[4 * h] = g4.x; rg[4 * h + 1] = g4.y; rg[4 * h + 2] = g4.z; rg[4 * h + 3] = g4.w;
                rb[4 * h] = e4.x; rb[4 * h + 1] = e4.y; rb[4 * h + 2] = e4.z; rb[4 * h + 3] = e4.w;
            }
            bf16_t* Cl = (bf16_t*)Cv;
            const int piece = n_base >> 6, pieces = N >> 6;
            // one row of a strip: combine, store hi and lo, and (where asked for) leave the 64-column
            // piece's sum and sum of squares, added up over the row's 8 lanes
            auto finish_row = [&](int r, const uint4& h, const uint4& l, const float2& st, int64_t row, bool live) {
                const float4 a0 = *(const float4*)(stg + r * SW + 8 * cg);
                const float4 a1 = *(const float4*)(stg + r * SW + 8 * cg + 4);
                const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                const uint32_t hw[4] = {h.x, h.y, h.z, h.w}, lw[4] = {l.x, l.y, l.z, l.w};
                float o[8];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float y0 = __uint_as_float(hw[t] << 16) + __uint_as_float(lw[t] << 16);
                    const float y1 = __uint_as_float(hw[t] & 0xffff0000u) + __uint_as_float(lw[t] & 0xffff0000u);
                    o[2 * t] = a[2 * t] + bv[2 * t] + ((y0 - st.x) * st.y * rg[2 * t] + rb[2 * t]);
                    o[2 * t + 1] = a[2 * t + 1] + bv[2 * t + 1] + ((y1 - st.x) * st.y * rg[2 * t + 1] + rb[2 * t + 1]);
                }
                float sm = 0.f, sq = 0.f;
                if (res.pstats) {
                    sm = ((o[0] + o[1]) + (o[2] + o[3])) + ((o[4] + o[5]) + (o[6] + o[7]));
                    sq = (fmaf(o[0], o[0], o[1] * o[1]) + fmaf(o[2], o[2], o[3] * o[3])) +
                         (fmaf(o[4], o[4], o[5] * o[5]) + fmaf(o[6], o[6], o[7] * o[7]));
                    sm = row8_sum(sm);
                    sq = row8_sum(sq);
                }
                if (live) {
                    uint32_t ho[4], lo[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        ho[t] = cvt_pk_bf16(o[2 * t], o[2 * t + 1]);
                        lo[t] = cvt_pk_bf16(o[2 * t] - __uint_as_float(ho[t] << 16),
                                            o[2 * t + 1] - __uint_as_float(ho[t] & 0xffff0000u));
                    }
                    *(uint4*)(res.x_out + row * N + col) = make_uint4(ho[0], ho[1], ho[2], ho[3]);
                    *(uint4*)(Cl + row * N + col) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                    if (res.pstats && cg == 0) res.pstats[row * pieces + piece] = make_float2(sm, sq);
                }
            };
            if (EPI == EPI_BIAS_RESIDUAL) {
                // The previous sums and statistics of strip s + D are requested before strip s is worked
                // on, so the strips do not each wait out a trip to memory.  Strip s covers rows
                // 8 s .. 8 s + 7 of the wavefront's tile.
                constexpr int D = 3;
                const int64_t row0 = m_base + r_in;
                const bf16_t* yh = res.y_hi + row0 * N + col;
                const bf16_t* yl = res.y_lo + row0 * N + col;
                const float2* sb = res.stats + row0;
                uint4 ph[D + 1], pl[D + 1];
                float2 st[D + 1];
                auto fetch = [&](int s) {
                    ph[s % (D + 1)] = *(const uint4*)(yh + (int64_t)(8 * s) * N);
                    pl[s % (D + 1)] = *(const uint4*)(yl + (int64_t)(8 * s) * N);
                    st[s % (D + 1)] = sb[8 * s];
                };
#pragma unroll
                for (int s = 0; s < D; ++s) fetch(s);
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    if (s + D < NS) fetch(s + D);
                    stage_strip(s / 4, s % 4);
                    const int64_t row = row0 + 8 * s;
                    finish_row(r_in, ph[s % (D + 1)], pl[s % (D + 1)], st[s % (D + 1)], row, row < rows);
                }
                continue;
            }
            // rows mapped through the request table (a small side problem: no prefetch)
#pragma unroll
            for (int i = 0; i < T::TM; ++i)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    stage_strip(i, e4);
                    int64_t row = m_base + 32 * i + 8 * e4 + r_in;
                    // GEMM row = request; its stream row is the request's first row
                    if (row >= rows || res.seq_len[row] <= 0) continue;
                    row = res.row_map[row];
                    finish_row(r_in, *(const uint4*)(res.y_hi + row * N + col), *(const uint4*)(res.y_lo + row * N + col),
                               res.stats[row], row, true);
                }
            continue;
        }

        {
            // bf16 out (plain, GELU, or the query / key columns of the QKV projection): 8 columns per lane
            constexpr int LPR = WTN / 8, RPI = 64 / LPR, NIT = 8 / RPI;
            const int cg = lane % LPR, r_in = lane / LPR;
            const int col = n_base + 8 * cg;
            const float4 b0 = *(const float4*)(bias + col), b1 = *(const float4*)(bias + col + 4);
            // maps with a LayerNorm folded in: column sums, and the statistics of every row this lane
            // will touch, requested before the first strip
            constexpr bool FOLD = EPI == EPI_QKV || EPI == EPI_KV || EPI == EPI_Q_MAPPED || EPI == EPI_BIAS_GELU;
            float4 c0 = make_float4(0.f, 0.f, 0.f, 0.f), c1 = c0;
            float2 rst[FOLD ? T::TM * 4 * NIT : 1];
            if (FOLD) {
                c0 = *(const float4*)(res.colsum + col);
                c1 = *(const float4*)(res.colsum + col + 4);
#pragma unroll
                for (int s = 0; s < T::TM * 4; ++s)
#pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        int64_t row = m_base + 8 * s + r_in + RPI * it;
                        if (EPI == EPI_Q_MAPPED) row = (row < rows && res.seq_len[row] > 0) ? res.row_map[row] : 0;
                        rst[s * NIT + it] = res.stats[row];
                    }
            }
            const int64_t ldc = (EPI == EPI_QKV || EPI == EPI_KV || EPI == EPI_Q_MAPPED) ? 2 * (int64_t)hidden
                                : EPI == EPI_GELU_SPLIT ? 2 * (int64_t)N : (int64_t)N;
            const int c_col = col + (EPI == EPI_KV ? hidden : 0);   // key columns sit after the query columns
            bf16_t* C = (bf16_t*)Cv;
#pragma unroll
            for (int i = 0; i < T::TM; ++i)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    stage_strip(i, e4);
#pragma unroll
                    for (int it = 0; it < NIT; ++it) {
                        const int r = r_in + RPI * it;
                        int64_t row = m_base + 32 * i + 8 * e4 + r;
                        if (EPI == EPI_Q_MAPPED) {
                            // GEMM row = request; its queries belong to the request's first row
                            if (row >= rows || res.seq_len[row] <= 0) continue;
                            row = res.row_map[row];
                        }
                        const float4 lo = *(const float4*)(stg + r * SW + 8 * cg);
                        const float4 hi = *(const float4*)(stg + r * SW + 8 * cg + 4);
                        float v[8];
                        if (FOLD) {
                            const float2 st = rst[(4 * i + e4) * NIT + it];
                            const float nm = -st.x * st.y;
                            v[0] = fmaf(lo.x, st.y, fmaf(nm, c0.x, b0.x)); v[1] = fmaf(lo.y, st.y, fmaf(nm, c0.y, b0.y));
                            v[2] = fmaf(lo.z, st.y, fmaf(nm, c0.z, b0.z)); v[3] = fmaf(lo.w, st.y, fmaf(nm, c0.w, b0.w));
                            v[4] = fmaf(hi.x, st.y, fmaf(nm, c1.x, b1.x)); v[5] = fmaf(hi.y, st.y, fmaf(nm, c1.y, b1.y));
                            v[6] = fmaf(hi.z, st.y, fmaf(nm, c1.z, b1.z)); v[7] = fmaf(hi.w, st.y, fmaf(nm, c1.w, b1.w));
                        } else {
                            v[0] = lo.x + b0.x; v[1] = lo.y + b0.y; v[2] = lo.z + b0.z; v[3] = lo.w + b0.w;
                            v[4] = hi.x + b1.x; v[5] = hi.y + b1.y; v[6] = hi.z + b1.z; v[7] = hi.w + b1.w;
                        }
                        if (EPI == EPI_BIAS_GELU || EPI == EPI_GELU_SPLIT) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = gelu_erf(v[e]);
                        }
                        const uint4 o = make_uint4(cvt_pk_bf16(v[0], v[1]), cvt_pk_bf16(v[2], v[3]),
                                                   cvt_pk_bf16(v[4], v[5]), cvt_pk_bf16(v[6], v[7]));
                        *(uint4*)(C + row * ldc + c_col) = o;
                        if (EPI == EPI_GELU_SPLIT) {
                            // second half of the row: what the first rounding lost, as bf16 again
                            const uint32_t h[4] = {o.x, o.y, o.z, o.w};
                            uint32_t l[4];
#pragma unroll
                            for (int t = 0; t < 4; ++t)
                                l[t] = cvt_pk_bf16(v[2 * t] - __uint_as_float(h[t] << 16),
                                                   v[2 * t + 1] - __uint_as_float(h[t] & 0xffff0000u));
                            *(uint4*)(C + row * ldc + N + c_col) = make_uint4(l[0], l[1], l[2], l[3]);
                        }
                    }
                }
        }
    }
    // parked DMAs may still be in flight: they must land before the workgroup gives up its LDS
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (clk && blockIdx.x == 0 && threadIdx.x == 0) {
        clk[0] = (int64_t)clock64() - clk_c0;
        clk[1] = (int64_t)wall_clock64() - clk_w0;
    }
}

template <int BM, int BN, int WM, int WN>
void launch_cfg(GemmEpilogue epi, const bf16_t* A, const bf16_t* W, const float* bias, ResidualSrc residual,
                void* C, bf16_t* vt, int64_t max_rows, int N, int K, int hidden, const int32_t* total_rows,
                int64_t* clk, hipStream_t s) {
    // persistent: one workgroup per compute unit (fewer if there cannot be that many tiles); the small tiles
    // leave room for two workgroups per unit (LDS and registers), which then hide each other's waits
    const int64_t tiles = (max_rows + BM - 1) / BM * (N / BN);
    const int64_t most = BM * BN <= 128 * 128 ? 512 : 256;
    const int64_t wgs = tiles < most ? (tiles + 7) / 8 * 8 : most;
    const dim3 grid((unsigned)wgs), block(WM * WN * 64);
#define PS_LAUNCH(E)                                                                                       \
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, E>), grid, block, 0, s, A, W, bias, residual, C, vt, \
                       max_rows, N, K, hidden, total_rows, clk)
    switch (epi) {
        case EPI_BIAS: PS_LAUNCH(EPI_BIAS); break;
        case EPI_BIAS_GELU: PS_LAUNCH(EPI_BIAS_GELU); break;
        case EPI_BIAS_RESIDUAL: PS_LAUNCH(EPI_BIAS_RESIDUAL); break;
        case EPI_QKV: PS_LAUNCH(EPI_QKV); break;
        case EPI_GELU_SPLIT: PS_LAUNCH(EPI_GELU_SPLIT); break;
        case EPI_RESIDUAL_MAPPED: PS_LAUNCH(EPI_RESIDUAL_MAPPED); break;
        case EPI_KV: PS_LAUNCH(EPI_KV); break;
        case EPI_Q_MAPPED: PS_LAUNCH(EPI_Q_MAPPED); break;
    }
#undef PS_LAUNCH
}

}  // namespace

// Requirements (checked when the model is loaded): N % 256 == 0, K % 64 == 0; every buffer holds
// max_rows rows with max_rows % 256 == 0, so whole tiles are always in bounds.
void launch_gemm_bf16(GemmEpilogue epi, const bf16_t* A, const bf16_t* W, const float* bias,
                      ResidualSrc residual, void* C, bf16_t* vt, int64_t max_rows, int N, int K,
                      int hidden, const int32_t* total_rows, int64_t* clk, hipStream_t s) {
    // Problems with few 256 x 256 tiles (the per-request side problems: one row per request; whole calls on a
    // micro-batch of a few requests) would leave most compute units idle: 128 x 128 tiles give four times as
    // many workgroups to spread them over.
    const int64_t big_tiles = (max_rows + 255) / 256 * (N / 256);
    if (epi == EPI_RESIDUAL_MAPPED || epi == EPI_Q_MAPPED || big_tiles < 128)
        launch_cfg<128, 128, 2, 2>(epi, A, W, bias, residual, C, vt, max_rows, N, K, hidden, total_rows, clk, s);
    else
        launch_cfg<256, 256, 2, 4>(epi, A, W, bias, residual, C, vt, max_rows, N, K, hidden, total_rows, clk, s);
}
