// C-ABI entry points: model file loading and re-layout, workspace planning, and the sequence of
// kernel launches that makes up one ps_predict_load call.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "internal.h"

namespace {

const char kMagic[8] = {'P', 'S', 'L', 'P', '0', '0', '0', '1'};
const size_t kHeaderBytes = 64;

inline float bf16_to_float(bf16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

// Reads tensors of the model file one after the other.
struct FileCursor {
    const uint8_t* p;
    const uint8_t* end;
    int dtype;
    size_t elem() const { return dtype == 1 ? 2 : 4; }
    const uint8_t* take(size_t n) {
        const uint8_t* r = p;
        p += n * elem();
        return r;
    }
    float value(const uint8_t* base, size_t i) const {
        if (dtype == 1) {
            bf16_t b;
            memcpy(&b, base + 2 * i, 2);
            return bf16_to_float(b);
        }
        float f;
        memcpy(&f, base + 4 * i, 4);
        return f;
    }
};

// Bump allocator over the host staging copy of the device blob.
struct Carver {
    std::vector<uint8_t>* host;   // NULL on the sizing pass
    size_t off = 0;
    size_t take(size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    }
};

// dst[n][k] = scale * src[k][n] for a [K][N] file matrix, in the file's own element type.
template <typename T>
void transpose_into(T* dst, int64_t dst_ld, const T* src, int K, int N) {
    const int B = 32;
    for (int k0 = 0; k0 < K; k0 += B)
        for (int n0 = 0; n0 < N; n0 += B)
            for (int k = k0; k < k0 + B && k < K; ++k)
                for (int n = n0; n < n0 + B && n < N; ++n) dst[(int64_t)n * dst_ld + k] = src[(int64_t)k * N + n];
}

inline bf16_t float_to_bf16(float f) {      // round to nearest even; the weights hold no NaN worth keeping
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// Multiply a bf16 value by 2^-3 exactly (head size 64: 1/sqrt(64)); subnormal results flush
// towards zero by at most one unit of the smallest bf16 exponent, which N(0, 0.02)-scale
// weights never reach; zero stays zero.
inline bf16_t bf16_times_eighth(bf16_t b) {
    int e = (b >> 7) & 0xFF;
    if (e == 0xFF) return b;
    if (e > 3) return (bf16_t)(b - (3 << 7));
    return (bf16_t)(b & 0x8000);
}

}  // namespace

Workspace plan_workspace(const ps_model_info& info, int64_t n_tokens, int32_t n_req, void* base) {
    Workspace ws;
    memset(&ws, 0, sizeof(ws));
    const size_t es = info.dtype == 1 ? 2 : 4;
    const int64_t H = info.hidden, F = info.ffn;
    int64_t rows = n_tokens + (int64_t)n_req * (info.n_soft + PS_ROW_ALIGN - 1) + PS_KEY_SLACK;
    rows = (int64_t)align_up((size_t)(rows > 0 ? rows : 1), PS_ROW_TILE);
    ws.max_rows = rows;
    ws.max_qtiles = rows / PS_ATT_BQ + n_req;
    size_t off = 0;
    uint8_t* b = (uint8_t*)base;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes, 256);
        return b ? (void*)(b + at) : (void*)nullptr;
    };
    ws.meta = (BatchMeta*)take(sizeof(BatchMeta));
    ws.seq_len = (int32_t*)take(sizeof(int32_t) * (size_t)(n_req + 1));
    ws.row_start = (int32_t*)take(sizeof(int32_t) * (size_t)(n_req + 1));
    ws.qtile_start = (int32_t*)take(sizeof(int32_t) * (size_t)(n_req + 1));
    ws.bad_req = (int32_t*)take(sizeof(int32_t) * (size_t)(n_req + 1));
    ws.x = take(es * rows * H);
    ws.qkv = take(es * rows * 3 * H);
    ws.vt = info.dtype == 1 ? take(es * rows * H + 1024) : nullptr;   // + slack: the last key tile may read past a row end
    ws.att = take(es * rows * H);
    if (info.dtype == 1) {
        ws.la = (bf16_t*)take(2 * rows * H);
        ws.lb = (bf16_t*)take(2 * rows * H);
        ws.sa = (float2*)take(8 * rows);
        ws.sb = (float2*)take(8 * rows);
        ws.ps = (float2*)take(8 * rows * (H / 64));
        ws.cls_rows = (int64_t)align_up((size_t)(n_req > 0 ? n_req : 1), PS_ROW_TILE);
        ws.cls_a = take(2 * ws.cls_rows * 2 * H);
        ws.cls_g = take(2 * ws.cls_rows * 2 * F);
    } else {
        ws.y = take(es * rows * H);
    }
    ws.x1 = take(es * rows * H);
    ws.g = take(es * rows * F);
    ws.bytes = off;
    return ws;
}

extern "C" const char* ps_strerror(int code) {
    switch (code) {
        case PS_OK: return "ok";
        case PS_EINVAL: return "invalid argument";
        case PS_EIO: return "cannot read model file";
        case PS_EFORMAT: return "model file header or size is wrong";
        case PS_ENOMEM: return "out of memory";
        case PS_EWORKSPACE: return "workspace too small or misaligned";
        case PS_EUNSUPPORTED: return "shape not supported by the kernels";
        case PS_EHIP: return "HIP runtime call failed";
    }
    return "unknown error code";
}

extern "C" int ps_model_load(const char* path, int device, ps_model** out) {
    if (!path || !out) return PS_EINVAL;
    *out = nullptr;
    FILE* f = fopen(path, "rb");
    if (!f) return PS_EIO;
    std::vector<uint8_t> raw;
    {
        if (fseek(f, 0, SEEK_END) != 0) { fclose(f); return PS_EIO; }
        long sz = ftell(f);
        if (sz < 0) { fclose(f); return PS_EIO; }
        rewind(f);
        try { raw.resize((size_t)sz); } catch (const std::bad_alloc&) { fclose(f); return PS_ENOMEM; }
        size_t got = sz ? fread(raw.data(), 1, (size_t)sz, f) : 0;
        fclose(f);
        if (got != (size_t)sz) return PS_EIO;
    }
    if (raw.size() < kHeaderBytes || memcmp(raw.data(), kMagic, 8) != 0) return PS_EFORMAT;
    int32_t h[10];
    memcpy(h, raw.data() + 8, sizeof(h));
    double eps;
    memcpy(&eps, raw.data() + 48, 8);
    ps_model_info info = {h[0], h[1], h[2], h[3], h[4], h[5], h[6], h[7], h[8], h[9]};
    if (info.layers < 1 || info.hidden < 1 || info.heads < 1 || info.ffn < 1 || info.vocab < 1 ||
        info.max_pos < 1 || info.n_soft < 0 || info.head_hidden < 1 || info.d_max < 0 ||
        (info.dtype != 0 && info.dtype != 1) || info.hidden % info.heads != 0 || !(eps >= 0))
        return PS_EFORMAT;
    const int64_t L = info.layers, H = info.hidden, F = info.ffn, V = info.vocab, P = info.max_pos,
                  M = info.n_soft, Hh = info.head_hidden;
    const size_t fe = info.dtype == 1 ? 2 : 4;
    const uint64_t n_elems = (uint64_t)(V + P + M) * H + 2 * H +
                             (uint64_t)L * (4 * H * H + 4 * H + 2 * H * F + F + H + 4 * H) +
                             (uint64_t)H * Hh + 2 * Hh + 1;
    if (raw.size() != kHeaderBytes + n_elems * fe) return PS_EFORMAT;
    const int d = info.hidden / info.heads;
    if (info.dtype == 1 && (H % 256 != 0 || H > 2048 || F % 256 != 0 || d != 64)) return PS_EUNSUPPORTED;
    if (info.dtype == 0 && (d > 256 || H > 8192 || (P + d) * 16 > 60000 || 3 * H / 64 > 65535)) return PS_EUNSUPPORTED;

    if (hipSetDevice(device) != hipSuccess) return PS_EHIP;
    ps_model* m = new (std::nothrow) ps_model();
    if (!m) return PS_ENOMEM;
    m->info = info;
    m->ln_eps = (float)eps;
    m->device = device;
    m->blob = nullptr;
    m->clk_slot = nullptr;
    int lds = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess) lds = 65536;
    m->lds_max = lds;

    // Two passes over the same carving code: first sizes, then fills the staging buffer.
    std::vector<uint8_t> stage;
    size_t o_etok = 0, o_epos = 0, o_esoft = 0, o_lneg = 0, o_lneb = 0, o_h1 = 0, o_bh1 = 0, o_wh2 = 0;
    struct LayerOff { size_t wqkv, wo, w1, w2, wod, w1d, w2d, bqkv, bo, b1, b2, g1, be1, g2, be2, cqkv, c1, d1; };
    std::vector<LayerOff> lo((size_t)L);
    for (int pass = 0; pass < 2; ++pass) {
        Carver c;
        c.host = pass ? &stage : nullptr;
        FileCursor cur{raw.data() + kHeaderBytes, raw.data() + raw.size(), info.dtype};
        auto put_raw = [&](size_t n) {   // tensor kept in the file's dtype and layout
            size_t at = c.take(n * fe);
            const uint8_t* src = cur.take(n);
            if (pass) memcpy(stage.data() + at, src, n * fe);
            return at;
        };
        auto put_f32 = [&](size_t n) {   // vector widened to float
            size_t at = c.take(n * 4);
            const uint8_t* src = cur.take(n);
            if (pass) {
                float* dst = (float*)(stage.data() + at);
                for (size_t i = 0; i < n; ++i) dst[i] = cur.value(src, i);
            }
            return at;
        };
        o_etok = put_raw((size_t)V * H);
        o_epos = put_raw((size_t)P * H);
        o_esoft = put_raw((size_t)M * H);
        o_lneg = put_f32(H);
        o_lneb = put_f32(H);
        // Fold the LayerNorm (gamma, beta) in front of a bf16 map W [N][K] with bias b into it: W becomes
        // gamma W (rounded to bf16 again), c its column sums over the rounded values, d = b + beta W.
        auto fold_layernorm = [&](size_t w_at, int64_t N, int64_t K, size_t gamma_at, size_t beta_at, size_t b_at,
                                  size_t c_at, size_t d_at) {
            bf16_t* w = (bf16_t*)(stage.data() + w_at);
            const float* gamma = (const float*)(stage.data() + gamma_at);
            const float* beta = (const float*)(stage.data() + beta_at);
            const float* b = (const float*)(stage.data() + b_at);
            float* cs = (float*)(stage.data() + c_at);
            float* ds = (float*)(stage.data() + d_at);
            for (int64_t n = 0; n < N; ++n) {
                double c = 0.0, d = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    const float wv = bf16_to_float(w[n * K + k]);
                    d += (double)beta[k] * wv;
                    const bf16_t folded = float_to_bf16(gamma[k] * wv);
                    w[n * K + k] = folded;
                    c += bf16_to_float(folded);
                }
                cs[n] = (float)c;
                ds[n] = (float)((double)b[n] + d);
            }
        };
        for (int64_t l = 0; l < L; ++l) {
            LayerOff& t = lo[(size_t)l];
            // W_q b_q W_k b_k W_v b_v come one after the other; they become one [*, 3H] map.
            t.wqkv = c.take((size_t)3 * H * H * fe);
            t.bqkv = c.take((size_t)3 * H * 4);
            for (int part = 0; part < 3; ++part) {
                const uint8_t* w = cur.take((size_t)H * H);
                const uint8_t* b = cur.take(H);
                if (!pass) continue;
                float* bias = (float*)(stage.data() + t.bqkv) + part * H;
                for (int64_t i = 0; i < H; ++i) bias[i] = cur.value(b, i);
                if (info.dtype == 1) {
                    // [3H][H]: output feature major, contraction index contiguous
                    bf16_t* dst = (bf16_t*)(stage.data() + t.wqkv) + (size_t)part * H * H;
                    transpose_into<bf16_t>(dst, H, (const bf16_t*)w, (int)H, (int)H);
                    if (part == 0) {   // fold the 1/sqrt(64) score scale into the query map (exact)
                        for (int64_t i = 0; i < H * H; ++i) dst[i] = bf16_times_eighth(dst[i]);
                        for (int64_t i = 0; i < H; ++i) bias[i] *= 0.125f;
                    }
                } else {
                    float* dst = (float*)(stage.data() + t.wqkv);
                    const float* src = (const float*)w;
                    for (int64_t i = 0; i < H; ++i)
                        memcpy(dst + i * 3 * H + part * H, src + i * H, (size_t)H * 4);
                }
            }
            if (info.dtype == 1) {
                // the LayerNorm in front of the QKV map: the embedding's for the first layer, else the
                // previous layer's second one; d replaces the bias in place
                t.cqkv = c.take((size_t)3 * H * 4);
                if (pass)
                    fold_layernorm(t.wqkv, 3 * H, H, l ? lo[(size_t)l - 1].g2 : o_lneg, l ? lo[(size_t)l - 1].be2 : o_lneb,
                                   t.bqkv, t.cqkv, t.bqkv);
            }
            auto put_matrix = [&](int64_t K, int64_t N) {   // file [K][N]
                size_t at = c.take((size_t)K * N * fe);
                const uint8_t* w = cur.take((size_t)K * N);
                if (pass) {
                    if (info.dtype == 1)
                        transpose_into<bf16_t>((bf16_t*)(stage.data() + at), K, (const bf16_t*)w, (int)K, (int)N);
                    else
                        memcpy(stage.data() + at, w, (size_t)K * N * 4);
                }
                return at;
            };
            auto put_doubled = [&](size_t src_at, int64_t K, int64_t N) {   // [N][K] -> [N][2K], each row twice
                if (info.dtype != 1) return (size_t)0;
                size_t at = c.take((size_t)2 * K * N * 2);
                if (pass) {
                    const bf16_t* src = (const bf16_t*)(stage.data() + src_at);
                    bf16_t* dst = (bf16_t*)(stage.data() + at);
                    for (int64_t n = 0; n < N; ++n) {
                        memcpy(dst + n * 2 * K, src + n * K, (size_t)K * 2);
                        memcpy(dst + n * 2 * K + K, src + n * K, (size_t)K * 2);
                    }
                }
                return at;
            };
            t.wo = put_matrix(H, H);
            t.wod = put_doubled(t.wo, H, H);
            t.bo = put_f32(H);
            t.g1 = put_f32(H);
            t.be1 = put_f32(H);
            t.w1 = put_matrix(H, F);
            t.w1d = put_doubled(t.w1, H, F);
            t.b1 = put_f32(F);
            if (info.dtype == 1) {
                // the first LayerNorm goes into W_1 (after the plain copy for the first-row pass was taken)
                t.c1 = c.take((size_t)F * 4);
                t.d1 = c.take((size_t)F * 4);
                if (pass) fold_layernorm(t.w1, F, H, t.g1, t.be1, t.b1, t.c1, t.d1);
            }
            t.w2 = put_matrix(F, H);
            t.w2d = put_doubled(t.w2, F, H);
            t.b2 = put_f32(H);
            t.g2 = put_f32(H);
            t.be2 = put_f32(H);
        }
        {   // head: W_h1 [H][Hh] -> float [Hh][H]
            o_h1 = c.take((size_t)H * Hh * 4);
            const uint8_t* w = cur.take((size_t)H * Hh);
            if (pass) {
                float* dst = (float*)(stage.data() + o_h1);
                for (int64_t i = 0; i < H; ++i)
                    for (int64_t j = 0; j < Hh; ++j) dst[j * H + i] = cur.value(w, (size_t)(i * Hh + j));
            }
            o_bh1 = put_f32(Hh);
            o_wh2 = put_f32(Hh);
            const uint8_t* b2 = cur.take(1);
            if (pass) m->b_h2 = cur.value(b2, 0);
        }
        if (!pass) {
            m->blob_bytes = c.off;
            try { stage.assign(c.off, 0); } catch (const std::bad_alloc&) { delete m; return PS_ENOMEM; }
        }
    }
    if (hipMalloc(&m->blob, m->blob_bytes) != hipSuccess) { delete m; return PS_ENOMEM; }
    if (hipMemcpy(m->blob, stage.data(), m->blob_bytes, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(m->blob);
        delete m;
        return PS_EHIP;
    }
    if (hipMalloc((void**)&m->clk_slot, 2 * sizeof(int64_t)) != hipSuccess ||
        hipMemset(m->clk_slot, 0, 2 * sizeof(int64_t)) != hipSuccess) {
        (void)hipFree(m->blob);
        delete m;
        return PS_ENOMEM;
    }
    uint8_t* b = (uint8_t*)m->blob;
    m->e_tok = b + o_etok;
    m->e_pos = b + o_epos;
    m->e_soft = b + o_esoft;
    m->lne_g = (float*)(b + o_lneg);
    m->lne_b = (float*)(b + o_lneb);
    m->layers.resize((size_t)L);
    for (int64_t l = 0; l < L; ++l) {
        const LayerOff& t = lo[(size_t)l];
        LayerWeights& w = m->layers[(size_t)l];
        w.w_qkv = b + t.wqkv; w.w_o = b + t.wo; w.w_1 = b + t.w1; w.w_2 = b + t.w2;
        w.w_od = b + t.wod; w.w_1d = b + t.w1d; w.w_2d = b + t.w2d;
        w.b_qkv = (float*)(b + t.bqkv); w.b_o = (float*)(b + t.bo);
        w.b_1 = (float*)(b + t.b1); w.b_2 = (float*)(b + t.b2);
        w.ln1_g = (float*)(b + t.g1); w.ln1_b = (float*)(b + t.be1);
        w.ln2_g = (float*)(b + t.g2); w.ln2_b = (float*)(b + t.be2);
        w.c_qkv = (float*)(b + t.cqkv); w.c_1 = (float*)(b + t.c1); w.d_1 = (float*)(b + t.d1);
    }
    m->w_h1t = (float*)(b + o_h1);
    m->b_h1 = (float*)(b + o_bh1);
    m->w_h2 = (float*)(b + o_wh2);
    *out = m;
    return PS_OK;
}

extern "C" int ps_profile_enable(ps_model* m, int on) {
    if (!m) return PS_EINVAL;
    m->profiling = on != 0;
    return PS_OK;
}

extern "C" int ps_profile_read(ps_model* m, void* hip_stream, double* ms, int64_t* launches) {
    if (!m || !ms || !launches) return PS_EINVAL;
    if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return PS_EHIP;
    for (int i = 0; i < PS_N_FAMILIES; ++i) { ms[i] = 0; launches[i] = 0; }
    int rc = PS_OK;
    for (const ProfRecord& r : m->prof) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess) rc = PS_EHIP;
        ms[r.family] += t;
        launches[r.family] += 1;
        m->event_pool.push_back(r.start);
        m->event_pool.push_back(r.stop);
    }
    m->prof.clear();
    return rc;
}

extern "C" int ps_profile_clock(ps_model* m, void* hip_stream, double* core_ghz) {
    if (!m || !core_ghz) return PS_EINVAL;
    *core_ghz = 0.0;
    if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return PS_EHIP;
    int64_t v[2] = {0, 0};
    int khz = 0;
    if (hipMemcpy(v, m->clk_slot, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, m->device) != hipSuccess)
        return PS_EHIP;
    if (v[1] > 0 && khz > 0) *core_ghz = (double)v[0] / ((double)v[1] / ((double)khz * 1e3)) / 1e9;
    return PS_OK;
}

extern "C" void ps_model_free(ps_model* m) {
    if (!m) return;
    for (const ProfRecord& r : m->prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    for (hipEvent_t e : m->event_pool) (void)hipEventDestroy(e);
    if (m->blob) {
        (void)hipSetDevice(m->device);
        (void)hipFree(m->blob);
        if (m->clk_slot) (void)hipFree(m->clk_slot);
    }
    delete m;
}

extern "C" int ps_model_get_info(const ps_model* m, ps_model_info* out) {
    if (!m || !out) return PS_EINVAL;
    *out = m->info;
    return PS_OK;
}

extern "C" size_t ps_workspace_bytes(const ps_model* m, int64_t max_tokens, int32_t max_req) {
    if (!m || max_tokens < 0 || max_req < 0) return 0;
    if (max_tokens + (int64_t)max_req * (m->info.n_soft + PS_ROW_ALIGN) > PS_MAX_ROWS) return 0;
    return plan_workspace(m->info, max_tokens, max_req, nullptr).bytes;
}

extern "C" int ps_predict_load(ps_model* m, const int32_t* token_ids, const int32_t* offsets,
                               const int32_t* lengths, int32_t n_req, int64_t n_tokens, float* pred_f,
                               int32_t* pred_tokens, void* workspace, size_t workspace_bytes,
                               ps_status* status, void* hip_stream) {
    if (!m || n_req < 0 || n_tokens < 0) return PS_EINVAL;
    if (n_req == 0) return PS_OK;
    if (!offsets || !pred_f || !pred_tokens || !workspace || (n_tokens > 0 && !token_ids)) return PS_EINVAL;
    // activation row indices are 32-bit and 8 rows of the transposed values span a 32-bit byte offset
    if (n_tokens + (int64_t)n_req * (m->info.n_soft + PS_ROW_ALIGN) > PS_MAX_ROWS) return PS_EUNSUPPORTED;
    if (((uintptr_t)workspace & 255) != 0) return PS_EWORKSPACE;
    Workspace ws = plan_workspace(m->info, n_tokens, n_req, workspace);
    if (ws.bytes > workspace_bytes) return PS_EWORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    (void)hipGetLastError();
    {
        ProfScope p(m, PS_FAM_EMBED, s);
        launch_prep(m, offsets, lengths, n_req, n_tokens, ws, status, s);
        launch_embed(m, token_ids, offsets, n_req, ws, status, s);
    }
    if (m->info.dtype == 1) run_encoder_bf16(m, n_req, ws, s);
    else run_encoder_f32(m, n_req, ws, s);
    {
        ProfScope p(m, PS_FAM_HEAD, s);
        launch_head(m, n_req, ws, pred_f, pred_tokens, status, s);
    }
    return hipGetLastError() == hipSuccess ? PS_OK : PS_EHIP;
}

extern "C" int ps_status_read(const ps_status* status, void* hip_stream, ps_status* out) {
    if (!status || !out) return PS_EINVAL;
    if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return PS_EHIP;
    ps_status raw;
    if (hipMemcpy(&raw, status, sizeof(raw), hipMemcpyDeviceToHost) != hipSuccess) return PS_EHIP;
    // On the device first_bad holds (2^62 - index) so that a maximum finds the smallest index.
    out->flags = raw.flags;
    out->reserved = 0;
    out->first_bad = raw.first_bad > 0 ? ((int64_t)1 << 62) - raw.first_bad : -1;
    return PS_OK;
}
