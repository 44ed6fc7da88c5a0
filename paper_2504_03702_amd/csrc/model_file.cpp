// Host-only part of ps_model_load (see model_file.h): header checks, then two passes over the same carving code,
// the first sizing the image, the second filling it with the tensors re-laid for the kernels.
#include "model_file.h"

#include <stdlib.h>
#include <string.h>

#include <new>

typedef uint16_t bf16_t;   // raw bf16 bit pattern

static inline size_t align_up_sz(size_t v, size_t a) { return (v + a - 1) / a * a; }

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
        off = align_up_sz(off + bytes, 256);
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


int ps_build_model_image(const uint8_t* raw, size_t raw_bytes, ModelImage* out) {
    if (!out || (!raw && raw_bytes > 0)) return PS_EINVAL;
    if (raw_bytes < kHeaderBytes || memcmp(raw, kMagic, 8) != 0) return PS_EFORMAT;
    int32_t h[10];
    memcpy(h, raw + 8, sizeof(h));
    double eps;
    memcpy(&eps, raw + 48, 8);
    ps_model_info info = {h[0], h[1], h[2], h[3], h[4], h[5], h[6], h[7], h[8], h[9]};
    if (info.layers < 1 || info.hidden < 1 || info.heads < 1 || info.ffn < 1 || info.vocab < 1 ||
        info.max_pos < 1 || info.n_soft < 0 || info.head_hidden < 1 || info.d_max < 0 ||
        (info.dtype != 0 && info.dtype != 1) || info.hidden % info.heads != 0 || !(eps >= 0))
        return PS_EFORMAT;
    // bounds that keep every size below in 64 bits (no real model comes near them)
    if (info.layers > 4096 || info.hidden > (1 << 20) || info.ffn > (1 << 22) || info.vocab > (1 << 26) ||
        info.max_pos > (1 << 24) || info.n_soft > (1 << 20) || info.head_hidden > (1 << 20))
        return PS_EFORMAT;
    const int64_t L = info.layers, H = info.hidden, F = info.ffn, V = info.vocab, P = info.max_pos,
                  M = info.n_soft, Hh = info.head_hidden;
    const size_t fe = info.dtype == 1 ? 2 : 4;
    const uint64_t n_elems = (uint64_t)(V + P + M) * H + 2 * H +
                             (uint64_t)L * (4 * H * H + 4 * H + 2 * H * F + F + H + 4 * H) +
                             (uint64_t)H * Hh + 2 * Hh + 1;
    if (raw_bytes != kHeaderBytes + n_elems * fe) return PS_EFORMAT;
    const int d = info.hidden / info.heads;
    if (info.dtype == 1 && (H % 256 != 0 || H > 2048 || F % 256 != 0 || d != 64)) return PS_EUNSUPPORTED;
    if (info.dtype == 0 && (d > 256 || H > 8192 || (P + d) * 16 > 60000 || 3 * H / 64 > 65535)) return PS_EUNSUPPORTED;

    ModelImage& img = *out;
    img.info = info;
    img.ln_eps = (float)eps;
    img.b_h2 = 0.f;

    // Two passes over the same carving code: first sizes, then fills the staging buffer.
    std::vector<uint8_t>& stage = img.stage;
    size_t o_etok = 0, o_epos = 0, o_esoft = 0, o_lneg = 0, o_lneb = 0, o_h1 = 0, o_bh1 = 0, o_wh2 = 0;
    typedef ModelLayerOffsets LayerOff;
    std::vector<LayerOff>& lo = img.layers;
    try { lo.assign((size_t)L, LayerOff()); } catch (const std::bad_alloc&) { return PS_ENOMEM; }
    for (int pass = 0; pass < 2; ++pass) {
        Carver c;
        c.host = pass ? &stage : nullptr;
        FileCursor cur{raw + kHeaderBytes, raw + raw_bytes, info.dtype};
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
            if (pass) img.b_h2 = cur.value(b2, 0);
        }
        if (!pass) {
            try { stage.assign(c.off, 0); } catch (const std::bad_alloc&) { return PS_ENOMEM; }
        }
    }
    img.e_tok = o_etok; img.e_pos = o_epos; img.e_soft = o_esoft; img.lne_g = o_lneg; img.lne_b = o_lneb;
    img.w_h1t = o_h1; img.b_h1 = o_bh1; img.w_h2 = o_wh2;
    return PS_OK;
}
