// Host-side sanitizer target: the model-file loader of the library and the two C oracles, built by
// tests/test_host_sanitizers.py with -fsanitize=address,undefined and run on files that test writes.
//   driver model <file>                  rc, then (if ok) image size, a checksum over every byte and the offsets
//   driver anticipate <in> <out>         the anticipator oracle on the arrays in <in>
//   driver lookahead <in> <out>          the look-ahead-map oracle on the arrays in <in>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "model_file.h"

extern "C" int pso_anticipate(const int32_t*, const int32_t*, const int32_t*, const int32_t*, int64_t, int32_t, int32_t,
                              int32_t*, int64_t*, int64_t*);
extern "C" int pso_lookahead_update(const int32_t*, const int32_t*, const int32_t*, const int32_t*, const int32_t*,
                                    const int32_t*, int64_t, int32_t, int32_t, int32_t*, int64_t*, int64_t*);

static bool read_file(const char* path, std::vector<uint8_t>& out) {
    FILE* f = fopen(path, "rb");
    if (!f) return false;
    fseek(f, 0, SEEK_END);
    long n = ftell(f);
    rewind(f);
    out.resize(n > 0 ? (size_t)n : 0);
    const bool ok = n <= 0 || fread(out.data(), 1, (size_t)n, f) == (size_t)n;
    fclose(f);
    return ok;
}

template <typename T>
static std::vector<T> take(const std::vector<uint8_t>& buf, size_t& at, size_t n) {
    std::vector<T> v(n);
    if (n) memcpy(v.data(), buf.data() + at, n * sizeof(T));
    at += n * sizeof(T);
    return v;
}

int main(int argc, char** argv) {
    if (argc < 3) return 2;
    std::vector<uint8_t> in;
    if (!read_file(argv[2], in)) return 3;
    if (!strcmp(argv[1], "model")) {
        ModelImage img;
        const int rc = ps_build_model_image(in.data(), in.size(), &img);
        printf("rc %d\n", rc);
        if (rc != 0) return 0;
        uint64_t sum = 1469598103934665603ull;
        for (uint8_t b : img.stage) sum = (sum ^ b) * 1099511628211ull;
        printf("bytes %zu checksum %llu layers %zu first %zu %zu %zu head %zu %zu %zu b_h2 %.9g\n", img.stage.size(),
               (unsigned long long)sum, img.layers.size(), img.e_tok, img.e_pos, img.e_soft, img.w_h1t, img.b_h1, img.w_h2,
               (double)img.b_h2);
        for (const ModelLayerOffsets& t : img.layers)
            printf("layer %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\n", t.wqkv, t.wo, t.w1, t.w2, t.wod, t.w1d, t.w2d, t.cqkv,
                   t.c1, t.d1);
        return 0;
    }
    if (argc < 4) return 2;
    size_t at = 0;
    const int64_t n = take<int64_t>(in, at, 1)[0];
    const std::vector<int32_t> dims = take<int32_t>(in, at, 4);      // n_inst, row length, flag, unused
    const int32_t n_inst = dims[0], len = dims[1];
    std::vector<int32_t> map = take<int32_t>(in, at, (size_t)n_inst * len);
    std::vector<int64_t> ovf = take<int64_t>(in, at, (size_t)n_inst);
    int64_t first_bad = -1;
    int rc;
    if (!strcmp(argv[1], "anticipate")) {
        std::vector<int32_t> pred = take<int32_t>(in, at, n), inst = take<int32_t>(in, at, n), arr = take<int32_t>(in, at, n);
        std::vector<int32_t> rate = take<int32_t>(in, at, dims[2] ? (size_t)n_inst : 0);
        rc = pso_anticipate(pred.data(), inst.data(), arr.data(), dims[2] ? rate.data() : nullptr, n, n_inst, len,
                            map.data(), ovf.data(), &first_bad);
    } else {
        std::vector<int32_t> c[6];
        for (auto& v : c) v = take<int32_t>(in, at, n);
        rc = pso_lookahead_update(c[0].data(), c[1].data(), c[2].data(), c[3].data(), c[4].data(), c[5].data(), n, n_inst,
                                  len, map.data(), ovf.data(), &first_bad);
    }
    FILE* f = fopen(argv[3], "wb");
    if (!f) return 3;
    const int64_t head[2] = {rc, first_bad};
    fwrite(head, sizeof(head), 1, f);
    fwrite(map.data(), sizeof(int32_t), map.size(), f);
    fwrite(ovf.data(), sizeof(int64_t), ovf.size(), f);
    fclose(f);
    return 0;
}
