// Host-only part of ps_model_load: a model file's bytes -> the image that is copied to the device in one piece
// (weights re-laid for the kernels) and where each tensor sits in it.  No HIP here, so that this code can be
// built and run under the host compiler's sanitizers.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "preserve.h"

struct ModelLayerOffsets {
    size_t wqkv, wo, w1, w2, wod, w1d, w2d, bqkv, bo, b1, b2, g1, be1, g2, be2, cqkv, c1, d1;
};

struct ModelImage {
    ps_model_info info;
    float ln_eps;
    float b_h2;
    std::vector<uint8_t> stage;          // the device blob's contents
    size_t e_tok, e_pos, e_soft, lne_g, lne_b, w_h1t, b_h1, w_h2;      // byte offsets into `stage`
    std::vector<ModelLayerOffsets> layers;
};

// PS_OK, PS_EFORMAT (header, sizes), PS_EUNSUPPORTED (a shape the kernels are not built for) or PS_ENOMEM.
int ps_build_model_image(const uint8_t* raw, size_t raw_bytes, ModelImage* out);
