// C-ABI entry points: model file loading and re-layout, workspace planning, and the sequence of
// kernel launches that makes up one ps_predict_load call.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "internal.h"
#include "model_file.h"

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
    ModelImage img;
    {
        const int rc = ps_build_model_image(raw.data(), raw.size(), &img);
        if (rc != PS_OK) return rc;
    }
    raw.clear();
    raw.shrink_to_fit();
    const ps_model_info& info = img.info;
    const int64_t L = info.layers;
    if (hipSetDevice(device) != hipSuccess) return PS_EHIP;
    ps_model* m = new (std::nothrow) ps_model();
    if (!m) return PS_ENOMEM;
    m->info = info;
    m->ln_eps = img.ln_eps;
    m->b_h2 = img.b_h2;
    m->device = device;
    m->blob = nullptr;
    m->clk_slot = nullptr;
    int lds = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, device) != hipSuccess) lds = 65536;
    m->lds_max = lds;
    m->blob_bytes = img.stage.size();
    const std::vector<uint8_t>& stage = img.stage;
    const std::vector<ModelLayerOffsets>& lo = img.layers;
    const size_t o_etok = img.e_tok, o_epos = img.e_pos, o_esoft = img.e_soft, o_lneg = img.lne_g, o_lneb = img.lne_b,
                 o_h1 = img.w_h1t, o_bh1 = img.b_h1, o_wh2 = img.w_h2;
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
        const ModelLayerOffsets& t = lo[(size_t)l];
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
