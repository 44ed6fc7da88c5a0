// Varlen multi-head self-attention on the gfx950 matrix cores (head size 64, bf16 in, fp32
// softmax statistics and accumulation).
//
// One workgroup handles 128 consecutive query rows of one request and one head; each of its four
// wavefronts owns 32 of them.  Keys and values are streamed in tiles of 64 keys through LDS
// (global_load_lds, three stages) and shared by the four wavefronts.  Everything is computed
// transposed so that a query is a column, i.e. a lane:
//     S^T[key, q] = K[key, :] . Q[q, :]          (v_mfma_f32_32x32x16_bf16, A = K tile, B = Q^T)
//     O^T[d, q]  += V^T[d, key] . P^T[key, q]    (A = V^T tile, B = P^T taken from the S^T registers)
// so the running maximum, the running sum and the rescale factor of a query are per-lane scalars
// and the softmax needs one cross-lane exchange per tile (between the two half-wavefronts that
// hold different keys of the same query).  The accumulator layout of S^T is, up to the order of the
// contraction index (which A and B only have to agree on), the B-operand layout of the second
// product, so P never leaves registers.  Which key sits in which accumulator row is free too (it
// is just the LDS row a lane reads its K fragment from): rows are assigned so that the 8 scores a
// lane contributes to one step of the second product belong to 8 consecutive keys, and the
// matching value fragment is a single 16-byte LDS read.  The 1/sqrt(64) scale is folded into the
// query projection when the model is loaded.  The value tile is read keys-contiguous from the transposed copy Vt
// that the QKV projection's epilogue writes.
//
// Keys beyond the request's length in the last tile are excluded: their scores are set to -inf
// before the maximum, so their weights are exactly zero.  The value rows they multiply only have to
// be finite: the rows up to PS_KEY_SLACK past the last request are written by the same call's QKV
// projection (from zero-filled inputs) for that reason.
#include <type_traits>

#include "device_util.h"
#include "internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define GLOBAL_AS __attribute__((address_space(1)))
#define LDS_AS __attribute__((address_space(3)))

union Frag8 {
    bf16x8 v;
    uint32_t u[4];
    uint2 h[2];
};

constexpr int BK = 64;                 // keys per tile
constexpr int TILE_BYTES = BK * 128;   // K tile [64 keys][64 d] or V^T tile [64 d][64 keys]
constexpr int STAGES = 3;              // key/value tiles in LDS: one in use, two on their way
constexpr float LOG2E = 1.4426950408889634f;
constexpr float RESCALE_SLACK = 5.5f;  // e^5.5 = 245: how far a score may exceed the exponent's reference

__global__ __launch_bounds__(256) void attention_bf16_kernel(
    const bf16_t* __restrict__ qk,      // [rows][2H]: query columns then key columns
    const bf16_t* __restrict__ vt,      // [H][vt_ld]: value features x rows
    bf16_t* __restrict__ out,           // [rows][H]
    bf16_t* __restrict__ cls_out,       // [requests][2H]: first row of every request as hi | lo bf16 pairs
    int H, int64_t vt_ld, int n_req, const BatchMeta* __restrict__ meta,
    const int32_t* __restrict__ seq_len, const int32_t* __restrict__ row_start,
    const int32_t* __restrict__ qtile_start, int first_rows_only) {
    __shared__ __align__(1024) unsigned char smem[STAGES * 2 * TILE_BYTES];   // stages x (K, V^T)

    // heads vary fastest over the workgroups: the hardware deals consecutive workgroups to the 8 XCDs in
    // turn, so with 8 | heads all query tiles of one (request, head) run on one XCD and share that
    // request's keys and values through its L2 instead of fetching them once per XCD
    const int heads = H / 64;
    const int head = blockIdx.x % heads, qt = blockIdx.x / heads;
    if (qt >= meta->total_qtiles) return;
    int lo = 0, hi = n_req - 1;          // request of this query tile: largest r with qtile_start[r] <= qt
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (qtile_start[mid] <= qt) lo = mid; else hi = mid - 1;
    }
    const int S = seq_len[lo];
    const int base = row_start[lo];
    const int q0 = (qt - qtile_start[lo]) * PS_ATT_BQ;
    if (first_rows_only && q0 != 0) return;                 // whole workgroup: nothing to wait for
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int last_row = base + S - 1;
    const int64_t ld_qk = 2 * (int64_t)H;

    // ---- this wavefront's queries: B operand fragments, one per 16-deep slice of the head -------
    const int wq0 = q0 + 32 * wave;
    // wave-uniform; inactive wavefronts still move tiles and meet the barriers
    const bool active = wq0 < S && !(first_rows_only && wave != 0);
    const int my_q = base + wq0 + col;
    const bf16_t* qrow = qk + (int64_t)min(my_q, last_row) * ld_qk + head * 64;
    bf16x8 qf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[ks] = *(const bf16x8*)(qrow + (2 * ks + half) * 8);

    // ---- DMA addressing: 2 instructions per wavefront per tile for K, 2 for V^T ------------------
    // Each address is a wave-uniform base (scalar registers, advanced per tile) plus a per-lane byte
    // offset that never changes, so a tile's four DMAs cost no vector arithmetic.  Key rows past the
    // end of the request are loaded as they are (the next request's rows or the slack rows at the end
    // of the buffer, all inside it): their scores are replaced, not multiplied, by the mask.
    const int drow = lane >> 3;                               // row within an 8-row group
    unsigned k_off[2], v_off[2];                              // per-lane byte offsets
    const unsigned char *k_base[2], *v_base[2];               // wave-uniform, tile 0
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int grp = j * 4 + wave;
        const int r = grp * 8 + drow;                         // key row (K tile) / feature row (V^T tile)
        const int c = (lane & 7) ^ lds_swz(r);
        // LDS row r of the K tile holds the key with bits 2 and 3 of r swapped (see below)
        const int kr = (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1);
        const int kb = (grp * 8) & ~8;                        // wave-uniform; kr - kb is in 0..15
        k_off[j] = (unsigned)((kr - kb) * (int)ld_qk + c * 8) * 2u;
        v_off[j] = (unsigned)(drow * vt_ld + c * 8) * 2u;                      // vt_ld < 2^28 (checked by the host)
        k_base[j] = (const unsigned char*)(qk + (int64_t)(base + kb) * ld_qk + H + head * 64);
        v_base[j] = (const unsigned char*)(vt + (int64_t)(head * 64 + grp * 8) * vt_ld + base);
    }
    const int64_t k_step = (int64_t)BK * ld_qk * 2;          // bytes per key tile: 64 rows of qk / 64 columns of vt
    auto dma_tile = [&](int stage, int kt) {
        unsigned char* sK = smem + stage * 2 * TILE_BYTES;
        unsigned char* sV = sK + TILE_BYTES;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int grp = j * 4 + wave;
            const unsigned char* gk = k_base[j] + kt * k_step;            // wave-uniform
            const unsigned char* gv = v_base[j] + kt * (BK * 2);
            __builtin_amdgcn_global_load_lds((const GLOBAL_AS void*)(gk + k_off[j]), (LDS_AS void*)(sK + grp * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const GLOBAL_AS void*)(gv + v_off[j]), (LDS_AS void*)(sV + grp * 1024), 16, 0, 0);
        }
    };

    // ---- LDS fragment offsets ---------------------------------------------------------------------
    // K tile: the DMA stores key (r with bits 2 and 3 swapped) in LDS row r, so accumulator row r of a
    // 32-key block is that key.  Accumulator element e of half-wave h is row 8 (e / 4) + 4 h + e % 4,
    // hence key 16 (e / 8) + 8 h + e % 8 of the block: elements 8 j .. 8 j + 7 are the 8 consecutive
    // keys 16 j + 8 h + 0..7.  Lanes read rows in natural order, which keeps the reads conflict-free.
    int koff[4];                                              // chunk 2 ks + half of row col
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) koff[ks] = col * 128 + (((2 * ks + half) ^ lds_swz(col)) * 16);
    int voff[4];                                              // V^T tile: feature row col, key chunk 2 j + half
#pragma unroll
    for (int j = 0; j < 4; ++j) voff[j] = col * 128 + (((2 * j + half) ^ lds_swz(col)) * 16);

    f32x16 o[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[i][e] = 0.f;
    float m_run = -INFINITY;      // running maximum of this lane's query (same in both half-waves)
    // running sum of this lane's share of the weights of its query (the other half-wavefront holds the
    // other keys; the two are added once, at the end).  Summed in fp32 before the weights are rounded
    // to bf16 for the second product: the rounding errors of the numerator average out over the keys.
    float l_run = 0.f;

    auto process_tile = [&](int kt, auto partial_tag) {
        constexpr bool partial = decltype(partial_tag)::value;
        const unsigned char* sK = smem + (kt % STAGES) * 2 * TILE_BYTES;
        const unsigned char* sV = sK + TILE_BYTES;
        const int k0 = kt * BK;

        // S^T = K Q^T for the two 32-key blocks
        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
            for (int e = 0; e < 16; ++e) s[b][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 kf = *(const bf16x8*)(sK + b * 4096 + koff[ks]);
                s[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[b], 0, 0, 0);
            }
        }
        // element e of block b is key k0 + 32 b + 16 (e / 8) + 8 half + 4 ((e / 4) % 2) + e % 4
        if (partial) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = k0 + 32 * b + 16 * (e >> 3) + 8 * half + (e & 7);
                    if (key >= S) s[b][e] = -INFINITY;
                }
        }
        float mx = s[0][0];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[b][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));               // finite: every tile holds a valid key
        // The exponent's reference m_run follows the running maximum lazily: it moves only when a tile's
        // maximum exceeds it by more than RESCALE_SLACK, so weights may reach e^RESCALE_SLACK instead of
        // 1 (harmless in bf16 and fp32) and the accumulators are rescaled a few times per request
        // instead of at nearly every tile.  The first tile sets the reference; nothing to rescale yet.
        if (kt == 0) {
            m_run = mx;
        } else if (__any(mx > m_run + RESCALE_SLACK)) {
            const float m_new = mx > m_run + RESCALE_SLACK ? mx : m_run;
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * LOG2E);
            m_run = m_new;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[i][e] *= alpha;
            l_run *= alpha;
        }
        const float mb = m_run * LOG2E;
        Frag8 pf[2][2];                                       // P^T fragments: [key block][16-key step]
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(s[b][8 * j + 2 * t], LOG2E, -mb));
                    const float p1 = __builtin_amdgcn_exp2f(fmaf(s[b][8 * j + 2 * t + 1], LOG2E, -mb));
                    l_run += p0 + p1;
                    pf[b][j].u[t] = cvt_pk_bf16(p0, p1);
                }
        // O^T += V^T P^T.  Step (b, j) contracts keys 32 b + 16 j + 8 half + 0..7 in this lane, the keys
        // its P fragment holds in that order: the value fragment is key chunk 4 b + 2 j + half.
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    Frag8 vf;
                    vf.v = *(const bf16x8*)(sV + i * 4096 + voff[2 * b + j]);
                    o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf[b][j].v, o[i], 0, 0, 0);
                }
            }
    };

    const int nkt = (S + BK - 1) / BK;
    // Tile kt + 2 is requested while tile kt is worked on, so a DMA has two tile times to land.  The
    // memory counter is in order: with the 4 DMA instructions of the newest tile allowed to be
    // outstanding, everything older has arrived.
    dma_tile(0, 0);
    if (nkt > 1) dma_tile(1, 1);
    for (int kt = 0; kt < nkt; ++kt) {
        if (kt + 1 < nkt) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();                                      // tile kt landed; tile kt-1 no longer read
        if (kt + 2 < nkt) dma_tile((kt + 2) % STAGES, kt + 2);
        if (!active) continue;
        // the last tile of a request may be ragged; full tiles run the code without any masking
        if ((kt + 1) * BK > S) process_tile(kt, std::true_type{});
        else process_tile(kt, std::false_type{});
    }
    if (!active) return;

    // ---- normalise and store: element e of block i is feature 32 i + 8 (e / 4) + 4 half + e % 4 -----
    const float inv = 1.0f / (l_run + __shfl_xor(l_run, 32, 64));
    if (wq0 + col < S) {
        bf16_t* orow = out + (int64_t)my_q * H + head * 64;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const uint2 p = make_uint2(cvt_pk_bf16(o[i][4 * e4] * inv, o[i][4 * e4 + 1] * inv),
                                           cvt_pk_bf16(o[i][4 * e4 + 2] * inv, o[i][4 * e4 + 3] * inv));
                *(uint2*)(orow + 32 * i + 8 * e4 + 4 * half) = p;
                if (wq0 + col == 0) {
                    // the request's first row feeds the head: keep what the bf16 rounding lost as a
                    // second bf16 value, for the error-compensated output projection of these rows
                    bf16_t* c = cls_out + (int64_t)lo * 2 * H + head * 64 + 32 * i + 8 * e4 + 4 * half;
                    *(uint2*)c = p;
                    const float r0 = o[i][4 * e4] * inv - __uint_as_float(p.x << 16);
                    const float r1 = o[i][4 * e4 + 1] * inv - __uint_as_float(p.x & 0xffff0000u);
                    const float r2 = o[i][4 * e4 + 2] * inv - __uint_as_float(p.y << 16);
                    const float r3 = o[i][4 * e4 + 3] * inv - __uint_as_float(p.y & 0xffff0000u);
                    *(uint2*)(c + H) = make_uint2(cvt_pk_bf16(r0, r1), cvt_pk_bf16(r2, r3));
                }
            }
    } else if (wq0 + col < ((S + PS_ROW_ALIGN - 1) & ~(PS_ROW_ALIGN - 1))) {
        // alignment rows between this request and the next: nobody reads their results, but the layers
        // after this one carry them along and the next layer's key tiles load them, so they must stay
        // finite.  Zeros here keep every later tensor of these rows finite.
        bf16_t* orow = out + (int64_t)my_q * H + head * 64;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) *(uint2*)(orow + 32 * i + 8 * e4 + 4 * half) = make_uint2(0u, 0u);
    }
}

}  // namespace

void launch_attention_bf16(const ps_model* m, int32_t n_req, const Workspace& ws, bool first_rows_only, hipStream_t s) {
    const dim3 grid((unsigned)(m->info.heads * ws.max_qtiles));      // at most 2^27 / 128 * 32 workgroups
    hipLaunchKernelGGL(attention_bf16_kernel, grid, dim3(256), 0, s, (const bf16_t*)ws.qkv, (const bf16_t*)ws.vt,
                       (bf16_t*)ws.att, (bf16_t*)ws.cls_a, m->info.hidden, ws.max_rows, n_req, ws.meta, ws.seq_len, ws.row_start,
                       ws.qtile_start, first_rows_only ? 1 : 0);
}
