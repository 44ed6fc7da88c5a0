// Per-call bookkeeping, embedding gather + LayerNorm, and the pooling + regression head.
// These kernels are shared by the fp32 and the bf16 encoder paths.
#include "device_util.h"
#include "internal.h"

namespace {

// ------------------------------------------------------------------------------------------
// prep: one workgroup turns (offsets, lengths) into the packed row layout of this call.
// Request r occupies activation rows [row_start[r], row_start[r] + seq_len[r]); row_start is a
// multiple of PS_ROW_ALIGN.  A request with an impossible length, or whose span leaves the
// token array, gets seq_len 0.  The workspace was sized by the host for n_tokens token slots;
// offsets that overlap can ask for more rows than that: requests from the first one that does
// not fit onwards are dropped the same way, so no later kernel indexes past `row_capacity`.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void prep_kernel(const int32_t* __restrict__ offsets,
                                                    const int32_t* __restrict__ lengths, int n_req,
                                                    int n_soft, int max_pos, long long n_tokens,
                                                    long long row_capacity, BatchMeta* meta,
                                                    int32_t* seq_len, int32_t* row_start,
                                                    int32_t* qtile_start, int32_t* bad_req,
                                                    ps_status* st) {
    __shared__ long long s_rows[1024];
    __shared__ long long s_tiles[1024];
    __shared__ long long s_cut_rows, s_cut_tiles;     // rows / query tiles in front of the first request that does not fit
    const int tid = threadIdx.x;
    const int per = (n_req + 1023) / 1024;
    const int r0 = min(tid * per, n_req);
    const int r1 = min(r0 + per, n_req);
    long long rows = 0, tiles = 0;
    for (int r = r0; r < r1; ++r) {
        const long long o0 = offsets[r], o1 = offsets[r + 1];
        const long long span = o1 - o0;
        const long long len = lengths ? (long long)lengths[r] : span;
        const bool bad = o0 < 0 || o1 > n_tokens || span < 0 || len < 1 || len > span || len > max_pos - n_soft;
        const int S = bad ? 0 : (int)len + n_soft;
        if (bad) report_fault(st, PS_ST_BAD_LENGTH, r);
        seq_len[r] = S;
        bad_req[r] = 0;
        rows += (S + PS_ROW_ALIGN - 1) / PS_ROW_ALIGN * PS_ROW_ALIGN;
        tiles += (S + PS_ATT_BQ - 1) / PS_ATT_BQ;
    }
    s_rows[tid] = rows;
    s_tiles[tid] = tiles;
    __syncthreads();
    // inclusive scan over the 1024 per-thread sums
    for (int d = 1; d < 1024; d <<= 1) {
        long long a = 0, b = 0;
        if (tid >= d) { a = s_rows[tid - d]; b = s_tiles[tid - d]; }
        __syncthreads();
        s_rows[tid] += a;
        s_tiles[tid] += b;
        __syncthreads();
    }
    if (tid == 0) {
        s_cut_rows = s_rows[1023];
        s_cut_tiles = s_tiles[1023];
    }
    __syncthreads();
    // Row starts are non-decreasing, so the requests that do not fit the workspace are a suffix: the first of
    // them starts where the last fitting one ends.
    long long row = s_rows[tid] - rows, tile = s_tiles[tid] - tiles;
    bool cut_here = false;
    long long my_cut_rows = 0, my_cut_tiles = 0;
    for (int r = r0; r < r1; ++r) {
        const int S = seq_len[r];
        const long long sz = (S + PS_ROW_ALIGN - 1) / PS_ROW_ALIGN * PS_ROW_ALIGN;
        if (row + sz > row_capacity) {
            if (!cut_here && row <= row_capacity) { cut_here = true; my_cut_rows = row; my_cut_tiles = tile; }
            if (S > 0) report_fault(st, PS_ST_BAD_LENGTH, r);
            seq_len[r] = 0;
            row_start[r] = -1;                       // set below, once the cut is known
        } else {
            row_start[r] = (int32_t)row;
            qtile_start[r] = (int32_t)tile;
        }
        row += sz;
        tile += (S + PS_ATT_BQ - 1) / PS_ATT_BQ;
    }
    // at most one thread holds the first request that does not fit with a start inside the capacity
    if (cut_here) {
        s_cut_rows = my_cut_rows;
        s_cut_tiles = my_cut_tiles;
    }
    __syncthreads();
    const long long cut_rows = min(s_cut_rows, row_capacity), cut_tiles = s_cut_tiles;
    for (int r = r0; r < r1; ++r) {
        if (row_start[r] < 0) {
            row_start[r] = (int32_t)cut_rows;
            qtile_start[r] = (int32_t)cut_tiles;
        }
    }
    if (tid == 1023) {
        row_start[n_req] = (int32_t)cut_rows;
        qtile_start[n_req] = (int32_t)cut_tiles;
        meta->total_rows = (int32_t)cut_rows;
        meta->total_qtiles = (int32_t)cut_tiles;
        meta->n_req = n_req;
        meta->qkv_rows = (int32_t)cut_rows + PS_KEY_SLACK;
    }
}

template <typename T> __device__ inline float load_elem(const T* p, int64_t i);
template <> __device__ inline float load_elem<float>(const float* p, int64_t i) { return p[i]; }
template <> __device__ inline float load_elem<bf16_t>(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }
template <typename T> __device__ inline void store_elem(T* p, int64_t i, float v);
template <> __device__ inline void store_elem<float>(float* p, int64_t i, float v) { p[i] = v; }
template <> __device__ inline void store_elem<bf16_t>(bf16_t* p, int64_t i, float v) { p[i] = f32_to_bf16(v); }

// ------------------------------------------------------------------------------------------
// embed: one wavefront per activation row.  Text rows gather a token embedding, the last n_soft
// rows of a request take the learnable prompt vectors; both add the position embedding of the
// row's index within its request and go through the embedding LayerNorm.  Rows that belong to
// no request (alignment gaps, the tail up to the next row tile) are zero-filled so that every
// row a later tile touches holds finite numbers.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const int32_t* __restrict__ token_ids,
                                                    const int32_t* __restrict__ offsets, int n_req,
                                                    const T* __restrict__ e_tok, const T* __restrict__ e_pos,
                                                    const T* __restrict__ e_soft,
                                                    const float* __restrict__ gamma,
                                                    const float* __restrict__ beta, float eps, int H,
                                                    int vocab, int n_soft, const BatchMeta* meta,
                                                    const int32_t* __restrict__ seq_len,
                                                    const int32_t* __restrict__ row_start,
                                                    int32_t* bad_req, T* __restrict__ x,
                                                    bf16_t* __restrict__ lo_out, float2* __restrict__ stats_out,
                                                    ps_status* st) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int total = meta->total_rows;
    const int64_t live = ((int64_t)total + PS_KEY_SLACK + PS_ROW_TILE - 1) / PS_ROW_TILE * PS_ROW_TILE;
    if (row >= live) return;
    T* out = x + row * H;
    bf16_t* yrow = lo_out ? lo_out + row * H : nullptr;  // bf16 path: lo parts of the sums, and row statistics
    int r = -1, p = 0;
    if (row < total) {
        int lo = 0, hi = n_req - 1;          // largest r with row_start[r] <= row
        while (lo < hi) {
            int mid = (lo + hi + 1) >> 1;
            if (row_start[mid] <= row) lo = mid; else hi = mid - 1;
        }
        r = lo;
        p = (int)(row - row_start[r]);
    }
    const int S = r >= 0 ? seq_len[r] : 0;
    if (r < 0 || p >= S) {
        for (int i = lane; i < H; i += 64) {
            store_elem<T>(out, i, 0.f);
            if (yrow) yrow[i] = 0;
        }
        if (yrow && lane == 0) stats_out[row] = make_float2(0.f, 0.f);
        return;
    }
    const int n_text = S - n_soft;
    const T* src;
    if (p < n_text) {
        const int id = token_ids[offsets[r] + p];
        if (id < 0 || id >= vocab) {
            // faulty request: flagged here, its row zeroed; the head reports NaN / -1 for it
            if (lane == 0) {
                report_fault(st, PS_ST_BAD_TOKEN, r);
                bad_req[r] = 1;
            }
            for (int i = lane; i < H; i += 64) {
                store_elem<T>(out, i, 0.f);
                if (yrow) yrow[i] = 0;
            }
            if (yrow && lane == 0) stats_out[row] = make_float2(0.f, 0.f);
            return;
        }
        src = e_tok + (int64_t)id * H;
    } else {
        src = e_soft + (int64_t)(p - n_text) * H;
    }
    const T* pos = e_pos + (int64_t)p * H;
    if (sizeof(T) == 2 && yrow) {
        // bf16 models (H a multiple of 256, at most 2048): the row stays in registers, lane l holding the
        // 4-element chunks l, l + 64, ...; 8-byte loads, one pass over the tables
        const int nch = H >> 8;
        float4 e[8];
        float sum = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            if (c < nch) {
                const uint2 a = ((const uint2*)src)[lane + 64 * c], b = ((const uint2*)pos)[lane + 64 * c];
                e[c].x = __uint_as_float(a.x << 16) + __uint_as_float(b.x << 16);
                e[c].y = __uint_as_float(a.x & 0xffff0000u) + __uint_as_float(b.x & 0xffff0000u);
                e[c].z = __uint_as_float(a.y << 16) + __uint_as_float(b.y << 16);
                e[c].w = __uint_as_float(a.y & 0xffff0000u) + __uint_as_float(b.y & 0xffff0000u);
                sum += (e[c].x + e[c].y) + (e[c].z + e[c].w);
            }
        }
        const float mean = wave_sum(sum) / (float)H;
        float sq = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            if (c < nch) {
                const float dx = e[c].x - mean, dy = e[c].y - mean, dz = e[c].z - mean, dw = e[c].w - mean;
                sq += (dx * dx + dy * dy) + (dz * dz + dw * dw);
            }
        }
        const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)H + eps);
        // the sums as hi + lo; hi, not normalised, is the operand of the first QKV map, which has the
        // embedding LayerNorm folded into its weights and finishes it from the row statistics
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            if (c < nch) {
                const uint2 hi = make_uint2(pack_bf16x2(e[c].x, e[c].y), pack_bf16x2(e[c].z, e[c].w));
                ((uint2*)out)[lane + 64 * c] = hi;
                ((uint2*)yrow)[lane + 64 * c] =
                    make_uint2(pack_bf16x2(e[c].x - __uint_as_float(hi.x << 16), e[c].y - __uint_as_float(hi.x & 0xffff0000u)),
                               pack_bf16x2(e[c].z - __uint_as_float(hi.y << 16), e[c].w - __uint_as_float(hi.y & 0xffff0000u)));
            }
        }
        if (lane == 0) stats_out[row] = make_float2(mean, rstd);
        return;
    }
    float sum = 0.f;
    for (int i = lane; i < H; i += 64) sum += load_elem<T>(src, i) + load_elem<T>(pos, i);
    const float mean = wave_sum(sum) / (float)H;
    float sq = 0.f;
    for (int i = lane; i < H; i += 64) {
        const float dlt = load_elem<T>(src, i) + load_elem<T>(pos, i) - mean;
        sq += dlt * dlt;
    }
    const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)H + eps);
    for (int i = lane; i < H; i += 64) {
        const float e = load_elem<T>(src, i) + load_elem<T>(pos, i);
        store_elem<T>(out, i, (e - mean) * rstd * gamma[i] + beta[i]);
    }
    if (yrow && lane == 0) stats_out[row] = make_float2(mean, rstd);
}

// ------------------------------------------------------------------------------------------
// head: one workgroup of 16 wavefronts per request.  c = final state of the request's first row
// (bf16 path: the last LayerNorm recomputed in fp32 from the row's sums and statistics); wavefront w
// takes hidden units j = w, w + 16, ..., four of them at a time (their loads are all requested before
// the first is used: with few requests the kernel's time is the latency of these loads): 64-lane dot
// products of c with rows of W_h1^T reduced across the wavefront, ReLU, times w_h2[j]; the sixteen
// partial sums are added in a fixed order.  pred_tokens = clamp(rint(y), 0, d_max) with rint
// rounding half to even.
// ------------------------------------------------------------------------------------------
const int kHeadWaves = 16;

template <typename T>
__global__ __launch_bounds__(kHeadWaves * 64) void head_kernel(const T* __restrict__ x, const int32_t* __restrict__ seq_len,
                                                   const int32_t* __restrict__ row_start,
                                                   const int32_t* __restrict__ bad_req,
                                                   const bf16_t* __restrict__ y_lo, const float2* __restrict__ stats,
                                                   const float* __restrict__ ln_g, const float* __restrict__ ln_b,
                                                   int H, int Hh,
                                                   const float* __restrict__ w_h1t, const float* __restrict__ b_h1,
                                                   const float* __restrict__ w_h2, float b_h2, int d_max,
                                                   float* __restrict__ pred_f, int32_t* __restrict__ pred_tokens,
                                                   ps_status* st) {
    extern __shared__ float s_c[];           // [H] + kHeadWaves partial sums
    const int r = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (seq_len[r] <= 0 || bad_req[r]) {
        if (threadIdx.x == 0) {
            pred_f[r] = __builtin_nanf("");
            pred_tokens[r] = -1;
        }
        return;
    }
    const int64_t crow = row_start[r];
    if (y_lo) {
        // bf16 models: x holds the hi parts of the last sums
        const float2 st2 = stats[crow];
        const bf16_t* hi = (const bf16_t*)x + crow * H;
        const bf16_t* lo = y_lo + crow * H;
        for (int i = threadIdx.x; i < H; i += kHeadWaves * 64)
            s_c[i] = ((bf16_to_f32(hi[i]) + bf16_to_f32(lo[i])) - st2.x) * st2.y * ln_g[i] + ln_b[i];
    } else {
        const T* c = x + crow * H;
        for (int i = threadIdx.x; i < H; i += kHeadWaves * 64) s_c[i] = load_elem<T>(c, i);
    }
    __syncthreads();
    float acc = 0.f;
    const bool wide = (H & 255) == 0 && H <= 2048;       // rows of whole 16-byte pieces per lane (all bf16 models)
    for (int j0 = wave; j0 < Hh; j0 += 4 * kHeadWaves) {
        float dot[4] = {0.f, 0.f, 0.f, 0.f};
        if (wide) {
            // lane l holds the 4-element pieces l, l + 64, ... of a row; the loads of four units' rows are all
            // requested before the first product is taken, four pieces (1024 elements) at a time
            const int nch = H >> 8;
            for (int c0 = 0; c0 < nch; c0 += 4) {
                float4 wv[4][4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int j = min(j0 + u * kHeadWaves, Hh - 1);      // (a unit past the end re-reads the last row)
                    const float4* w = (const float4*)(w_h1t + (int64_t)j * H);
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        wv[u][c] = c0 + c < nch ? w[lane + 64 * (c0 + c)] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (c0 + c < nch) {
                        const float4 cv = ((const float4*)s_c)[lane + 64 * (c0 + c)];
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            dot[u] = fmaf(cv.x, wv[u][c].x, fmaf(cv.y, wv[u][c].y, fmaf(cv.z, wv[u][c].z, fmaf(cv.w, wv[u][c].w, dot[u]))));
                    }
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + u * kHeadWaves;
                if (j < Hh) {
                    const float* w = w_h1t + (int64_t)j * H;
                    for (int i = lane; i < H; i += 64) dot[u] = fmaf(s_c[i], w[i], dot[u]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = j0 + u * kHeadWaves;
            if (j < Hh) {
                const float d = wave_sum(dot[u]) + b_h1[j];
                acc += (d < 0.f ? 0.f : d) * w_h2[j];   // ReLU that lets a NaN through to the check below
            }
        }
    }
    if (lane == 0) s_c[H + wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float y = 0.f;
        for (int w = 0; w < kHeadWaves; ++w) y += s_c[H + w];
        y += b_h2;
        pred_f[r] = y;
        if (y != y) {
            pred_tokens[r] = -1;
            report_fault(st, PS_ST_NAN, r);
        } else {
            const float t = fminf(fmaxf(rintf(y), 0.f), (float)d_max);
            pred_tokens[r] = (int32_t)t;
        }
    }
}

// Gather for the [CLS] refinement: row r of the side matrix is the fp32 LayerNorm output of request
// r's first row, split into two bf16 values per element (x ~ hi + lo, |x - hi - lo| <= 2^-17 |x|),
// hi in columns [0, H), lo in [H, 2H).  Rows of faulty requests and padding rows are zero.
__global__ __launch_bounds__(256) void cls_gather_kernel(const bf16_t* __restrict__ y_hi, const bf16_t* __restrict__ y_lo,
                                                         const float2* __restrict__ stats,
                                                         const float* __restrict__ gamma, const float* __restrict__ beta,
                                                         int H, int n_req, const int32_t* __restrict__ seq_len,
                                                         const int32_t* __restrict__ row_start, bf16_t* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    bf16_t* o = out + (int64_t)r * 2 * H;
    if (r >= n_req || seq_len[r] <= 0) {
        for (int i = lane; i < 2 * H; i += 64) o[i] = 0;
        return;
    }
    const int64_t row = row_start[r];
    const float2 st = stats[row];
    for (int i = lane; i < H; i += 64) {
        const float x = ((bf16_to_f32(y_hi[row * H + i]) + bf16_to_f32(y_lo[row * H + i])) - st.x) * st.y * gamma[i] + beta[i];
        const bf16_t hi = f32_to_bf16(x);
        o[i] = hi;
        o[H + i] = f32_to_bf16(x - bf16_to_f32(hi));
    }
}

// LayerNorm statistics (mean, 1 / std; biased variance) of each request's first row of the sums hi + lo:
// one wavefront per request.  Used where only those rows go on (the last layer), in place of the
// LayerNorm over all rows.
__global__ __launch_bounds__(256) void cls_stats_kernel(const bf16_t* __restrict__ y_hi, const bf16_t* __restrict__ y_lo,
                                                        float2* __restrict__ stats, float eps,
                                                        int H, int n_req, const int32_t* __restrict__ seq_len,
                                                        const int32_t* __restrict__ row_start) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= n_req || seq_len[r] <= 0) return;
    const int64_t row = row_start[r];
    const bf16_t *yh = y_hi + row * H, *yl = y_lo + row * H;
    float sum = 0.f;
    for (int i = lane; i < H; i += 64) sum += bf16_to_f32(yh[i]) + bf16_to_f32(yl[i]);
    const float mean = wave_sum(sum) / (float)H;
    float sq = 0.f;
    for (int i = lane; i < H; i += 64) {
        const float d = (bf16_to_f32(yh[i]) + bf16_to_f32(yl[i])) - mean;
        sq = fmaf(d, d, sq);
    }
    const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)H + eps);
    if (lane == 0) stats[row] = make_float2(mean, rstd);
}

// The bf16 input rows of each request's first token, one per request, for the side GEMM that computes
// only those rows' queries (last layer).  Rows of faulty requests and padding rows are zero.
__global__ __launch_bounds__(256) void cls_rows_kernel(const bf16_t* __restrict__ x, int H, int n_req,
                                                       const int32_t* __restrict__ seq_len,
                                                       const int32_t* __restrict__ row_start, bf16_t* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    uint4* o = (uint4*)(out + (int64_t)r * H);
    const bool live = r < n_req && seq_len[r] > 0;
    const uint4* src = live ? (const uint4*)(x + (int64_t)row_start[r] * H) : nullptr;
    for (int i = lane; i < H / 8; i += 64) o[i] = live ? src[i] : make_uint4(0u, 0u, 0u, 0u);
}

}  // namespace

void launch_cls_rows(const ps_model* m, int32_t n_req, const Workspace& ws, const bf16_t* x, bf16_t* out, hipStream_t s) {
    hipLaunchKernelGGL(cls_rows_kernel, dim3((unsigned)(ws.cls_rows / 4)), dim3(256), 0, s, x, m->info.hidden, n_req,
                       ws.seq_len, ws.row_start, out);
}

void launch_cls_stats(const ps_model* m, int32_t n_req, const Workspace& ws, const bf16_t* y_hi, const bf16_t* y_lo,
                      float2* stats, hipStream_t s) {
    hipLaunchKernelGGL(cls_stats_kernel, dim3((unsigned)(ws.cls_rows / 4)), dim3(256), 0, s, y_hi, y_lo, stats, m->ln_eps,
                       m->info.hidden, n_req, ws.seq_len, ws.row_start);
}

void launch_cls_gather(const ps_model* m, int32_t n_req, const Workspace& ws, const bf16_t* y_hi, const bf16_t* y_lo,
                       const float2* stats, const float* gamma, const float* beta, hipStream_t s) {
    hipLaunchKernelGGL(cls_gather_kernel, dim3((unsigned)(ws.cls_rows / 4)), dim3(256), 0, s, y_hi, y_lo, stats, gamma, beta,
                       m->info.hidden, n_req, ws.seq_len, ws.row_start, (bf16_t*)ws.cls_a);
}

void launch_prep(const ps_model* m, const int32_t* offsets, const int32_t* lengths, int32_t n_req, int64_t n_tokens,
                 const Workspace& ws, ps_status* st, hipStream_t s) {
    hipLaunchKernelGGL(prep_kernel, dim3(1), dim3(1024), 0, s, offsets, lengths, n_req, m->info.n_soft,
                       m->info.max_pos, (long long)n_tokens, (long long)(ws.max_rows - PS_KEY_SLACK), ws.meta, ws.seq_len,
                       ws.row_start, ws.qtile_start, ws.bad_req, st);
}

void launch_embed(const ps_model* m, const int32_t* token_ids, const int32_t* offsets, int32_t n_req,
                  const Workspace& ws, ps_status* st, hipStream_t s) {
    const ps_model_info& f = m->info;
    const unsigned blocks = (unsigned)(ws.max_rows / 4);
    if (f.dtype == 1)
        hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, token_ids, offsets, n_req,
                           (const bf16_t*)m->e_tok, (const bf16_t*)m->e_pos, (const bf16_t*)m->e_soft,
                           m->lne_g, m->lne_b, m->ln_eps, f.hidden, f.vocab, f.n_soft, ws.meta, ws.seq_len,
                           ws.row_start, ws.bad_req, (bf16_t*)ws.x, ws.la, ws.sa, st);
    else
        hipLaunchKernelGGL(embed_kernel<float>, dim3(blocks), dim3(256), 0, s, token_ids, offsets, n_req,
                           (const float*)m->e_tok, (const float*)m->e_pos, (const float*)m->e_soft,
                           m->lne_g, m->lne_b, m->ln_eps, f.hidden, f.vocab, f.n_soft, ws.meta, ws.seq_len,
                           ws.row_start, ws.bad_req, (float*)ws.x, (bf16_t*)nullptr, (float2*)nullptr, st);
}

void launch_head(const ps_model* m, int32_t n_req, const Workspace& ws, float* pred_f, int32_t* pred_tokens,
                 ps_status* st, hipStream_t s) {
    const ps_model_info& f = m->info;
    const size_t lds = sizeof(float) * (size_t)(f.hidden + kHeadWaves);
    if (f.dtype == 1)
        hipLaunchKernelGGL(head_kernel<bf16_t>, dim3(n_req), dim3(kHeadWaves * 64), lds, s, (const bf16_t*)ws.x,
                           ws.seq_len, ws.row_start, ws.bad_req, (const bf16_t*)ws.la, (const float2*)ws.sa,
                           (const float*)m->layers.back().ln2_g, (const float*)m->layers.back().ln2_b, f.hidden, f.head_hidden, m->w_h1t, m->b_h1, m->w_h2,
                           m->b_h2, f.d_max, pred_f, pred_tokens, st);
    else
        hipLaunchKernelGGL(head_kernel<float>, dim3(n_req), dim3(kHeadWaves * 64), lds, s, (const float*)ws.x,
                           ws.seq_len, ws.row_start, ws.bad_req, (const bf16_t*)nullptr, (const float2*)nullptr,
                           (const float*)nullptr, (const float*)nullptr, f.hidden, f.head_hidden, m->w_h1t, m->b_h1, m->w_h2,
                           m->b_h2, f.d_max, pred_f, pred_tokens, st);
}
