// Host-side paths of the C ABI (include/int8t.h) in a build whose HOST code is compiled with
// -fsanitize=address,undefined: size queries, the code-unpacking aid, Eq.7, and the argument checks
// of every entry point, which must return an error code before anything is launched (so this runs
// on a machine without a GPU).  Prints "abi sanitize ok".
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/int8t.h"

static int bad = 0;
#define EXPECT(cond)                                                 \
    do {                                                             \
        if (!(cond)) { ++bad; std::printf("failed: %s (line %d)\n", #cond, __LINE__); } \
    } while (0)

int main() {
    const int d_act[4] = {2, 20, 3, 5}, d_w[4] = {33, 20, 3, 3}, d_bad[4] = {2, 0, 3, 5}, d_huge[4] = {65536, 65536, 2, 2};
    EXPECT(int8t_code_bytes(d_act, INT8T_ACT) == 2u * 3 * 5 * 32);
    EXPECT(int8t_code_bytes(d_bad, INT8T_ACT) == 0);
    EXPECT(int8t_code_bytes(d_huge, INT8T_ACT) == 0);
    EXPECT(int8t_code_bytes(d_act, (int8t_kind)9) == 0);
    EXPECT(int8t_quantize_workspace_bytes(d_act, INT8T_ACT) > 0);
    EXPECT(int8t_quantize_workspace_bytes(d_bad, INT8T_WGT) == 0);

    // unpack: fill the library layout by the header's formulas, expect the logical order back
    for (int kind = 0; kind < 4; ++kind) {
        const int* d = (kind == INT8T_WGT || kind == INT8T_WGT_PLANAR) ? d_w : d_act;
        const size_t nb = int8t_code_bytes(d, (int8t_kind)kind), n = (size_t)d[0] * d[1] * d[2] * d[3];
        std::vector<int8_t> codes(nb, 0), out(n, 99);
        const int plane = d[2] * d[3];
        auto val = [&](int a, int b, int p) { return (int8_t)((a * 31 + b * 7 + p * 3) % 255 - 127); };
        const int p0 = (d[1] + 15) & ~15, p1 = (d[0] + 15) & ~15;
        const size_t off2 = ((size_t)d[0] * plane * p0 + 255) & ~(size_t)255;
        for (int a = 0; a < d[0]; ++a)
            for (int b = 0; b < d[1]; ++b)
                for (int p = 0; p < plane; ++p) {
                    if (kind == INT8T_ACT_PLANAR || kind == INT8T_WGT_PLANAR) codes[((size_t)a * d[1] + b) * plane + p] = val(a, b, p);
                    else {
                        codes[((size_t)a * plane + p) * p0 + b] = val(a, b, p);
                        if (kind == INT8T_WGT) codes[off2 + ((size_t)b * plane + p) * p1 + a] = val(a, b, p);
                    }
                }
        for (int copy = 0; copy < (kind == INT8T_WGT ? 2 : 1); ++copy) {
            size_t padbad = 77;
            EXPECT(int8t_unpack_codes(codes.data(), d, (int8t_kind)kind, copy, out.data(), &padbad) == INT8T_OK);
            EXPECT(padbad == 0);
            size_t wrong = 0;
            for (int a = 0; a < d[0]; ++a)
                for (int b = 0; b < d[1]; ++b)
                    for (int p = 0; p < plane; ++p) wrong += out[((size_t)a * d[1] + b) * plane + p] != val(a, b, p);
            EXPECT(wrong == 0);
        }
        if (kind == INT8T_ACT) {
            codes[20] = 5;   // a padding byte (channel 20 of 32 at the first pixel)
            size_t padbad = 0;
            EXPECT(int8t_unpack_codes(codes.data(), d, INT8T_ACT, 0, out.data(), &padbad) == INT8T_OK && padbad == 1);
            EXPECT(int8t_unpack_codes(codes.data(), d, INT8T_ACT, 1, out.data(), nullptr) == INT8T_ERR_ARG);
        }
        EXPECT(int8t_unpack_codes(nullptr, d, (int8t_kind)kind, 0, out.data(), nullptr) == INT8T_ERR_NULL);
        EXPECT(int8t_unpack_codes(codes.data(), d_bad, (int8t_kind)kind, 0, out.data(), nullptr) == INT8T_ERR_SHAPE);
    }

    // workspace queries over a sweep of layer geometries (host plans: tile search, split counts)
    size_t total = 0;
    for (int C = 1; C <= 300; C += 37)
        for (int K = 1; K <= 300; K += 53)
            for (int R = 1; R <= 7; R += 2)
                for (int st = 1; st <= 3; ++st)
                    for (int hw = 1; hw <= 57; hw += 14) {
                        int8t_conv_desc d = {3, C, hw + R, hw + 2, K, R, (R == 7) ? 1 : R, st, st, R / 2, 0, 1};
                        for (int op = INT8T_OP_CONV_FWD; op <= INT8T_OP_CONV_BWD_WEIGHT; ++op) total += int8t_workspace_bytes((int8t_op)op, &d, 0, 0);
                        int8t_conv_desc dwise = {2, C, hw + R, hw + R, C, R, R, st, st, R / 2, R / 2, C};
                        total += int8t_workspace_bytes(INT8T_OP_CONV_BWD_WEIGHT, &dwise, 0, 0);
                    }
    EXPECT(total > 0);
    EXPECT(int8t_workspace_bytes(INT8T_OP_DSGC, nullptr, 1000, 32) > 0);
    EXPECT(int8t_workspace_bytes(INT8T_OP_CONV_FWD, nullptr, 0, 0) == 0);

    // argument errors of the entry points: nothing may be launched, nothing dereferenced
    alignas(16) static char fake[4096];
    float* f = reinterpret_cast<float*>(fake);
    int8_t* q = reinterpret_cast<int8_t*>(fake + 1024);
    double* dd = reinterpret_cast<double*>(fake + 2048);
    EXPECT(int8t_quantize(nullptr, d_act, INT8T_ACT, nullptr, INT8T_ROUND_NEAREST_EVEN, 0, q, f, nullptr, fake, 4096, nullptr) == INT8T_ERR_NULL);
    EXPECT(int8t_quantize(f, d_bad, INT8T_ACT, nullptr, INT8T_ROUND_NEAREST_EVEN, 0, q, f, nullptr, fake, 4096, nullptr) == INT8T_ERR_SHAPE);
    EXPECT(int8t_quantize(f, d_act, (int8t_kind)7, nullptr, INT8T_ROUND_NEAREST_EVEN, 0, q, f, nullptr, fake, 4096, nullptr) == INT8T_ERR_ARG);
    EXPECT(int8t_quantize(f, d_act, INT8T_ACT, nullptr, (int8t_round)5, 0, q, f, nullptr, fake, 4096, nullptr) == INT8T_ERR_ARG);
    EXPECT(int8t_quantize(f + 1, d_act, INT8T_ACT, nullptr, INT8T_ROUND_NEAREST_EVEN, 0, q, f, nullptr, fake, 4096, nullptr) == INT8T_ERR_ARG);
    EXPECT(int8t_quantize(f, d_act, INT8T_ACT, nullptr, INT8T_ROUND_NEAREST_EVEN, 0, q, f, nullptr, fake, 16, nullptr) == INT8T_ERR_WORKSPACE);
    EXPECT(int8t_quantize(f, d_act, INT8T_ACT, nullptr, INT8T_ROUND_NEAREST_EVEN, 0, q, f, nullptr, nullptr, 0, nullptr) == INT8T_ERR_NULL);
    int8t_quantize_item items[2];
    std::memset(items, 0, sizeof(items));
    EXPECT(int8t_quantize_batch(1, nullptr, fake, 4096, nullptr) == INT8T_ERR_NULL);
    EXPECT(int8t_quantize_batch(0, items, fake, 4096, nullptr) == INT8T_ERR_ARG);
    EXPECT(int8t_quantize_batch(INT8T_MAX_BATCH + 1, items, fake, 4096, nullptr) == INT8T_ERR_ARG);
    EXPECT(int8t_quantize_batch(2, items, fake, 4096, nullptr) == INT8T_ERR_NULL);
    EXPECT(int8t_quantize_batch_workspace_bytes(0, items) == 0);
    EXPECT(int8t_dsgc_clip(nullptr, 10, f, 4, INT8T_ROUND_STOCHASTIC, 0, f, dd, nullptr, fake, 4096, nullptr) == INT8T_ERR_NULL);
    EXPECT(int8t_dsgc_clip(f, 0, f, 4, INT8T_ROUND_STOCHASTIC, 0, f, dd, nullptr, fake, 4096, nullptr) == INT8T_ERR_SHAPE);
    EXPECT(int8t_dsgc_clip(f, 10, f, 0, INT8T_ROUND_STOCHASTIC, 0, f, dd, nullptr, fake, 4096, nullptr) == INT8T_ERR_ARG);
    EXPECT(int8t_dsgc_clip(f, 10, f, INT8T_MAX_CANDIDATES + 1, INT8T_ROUND_STOCHASTIC, 0, f, dd, nullptr, fake, 4096, nullptr) == INT8T_ERR_ARG);
    EXPECT(int8t_dsgc_clip(f, 10, f, 4, INT8T_ROUND_STOCHASTIC, 0, f, dd, nullptr, fake, 4096, nullptr) == INT8T_ERR_WORKSPACE);
    EXPECT(int8t_dsgc_prepare(f, 10, fake, 16, nullptr) == INT8T_ERR_WORKSPACE);
    EXPECT(int8t_dsgc_search(f, 10, f, 4, INT8T_ROUND_STOCHASTIC, 0, f, dd, nullptr, nullptr, 0, nullptr) == INT8T_ERR_NULL);
    int8t_conv_desc good = {2, 16, 8, 8, 16, 3, 3, 1, 1, 1, 1, 1}, neg = good, grp = good, tiny = good;
    neg.stride_h = 0;
    grp.groups = 4;
    tiny.H = 1; tiny.pad_h = 0;
    EXPECT(int8t_conv_fwd(nullptr, q, f, q, f, f, nullptr, nullptr, 0, nullptr) == INT8T_ERR_NULL);
    EXPECT(int8t_conv_fwd(&neg, q, f, q, f, f, nullptr, nullptr, 0, nullptr) == INT8T_ERR_SHAPE);
    EXPECT(int8t_conv_fwd(&grp, q, f, q, f, f, nullptr, nullptr, 0, nullptr) == INT8T_ERR_SHAPE);
    EXPECT(int8t_conv_fwd(&tiny, q, f, q, f, f, nullptr, nullptr, 0, nullptr) == INT8T_ERR_SHAPE);
    EXPECT(int8t_conv_fwd(&good, nullptr, f, q, f, f, nullptr, nullptr, 0, nullptr) == INT8T_ERR_NULL);
    EXPECT(int8t_conv_fwd(&good, q + 1, f, q, f, f, nullptr, nullptr, 0, nullptr) == INT8T_ERR_ARG);
    EXPECT(int8t_conv_bwd_data(&good, q, f, q, f, nullptr, nullptr, nullptr, 0, nullptr) == INT8T_ERR_NULL);
    EXPECT(int8t_conv_bwd_data(&neg, q, f, q, f, f, nullptr, nullptr, 0, nullptr) == INT8T_ERR_SHAPE);
    EXPECT(int8t_conv_bwd_weight(&good, q, f, q, f, f, nullptr, nullptr, 0, nullptr) == INT8T_ERR_NULL);
    EXPECT(int8t_conv_bwd_weight(&good, q, f, q, f, f, nullptr, fake, 16, nullptr) == INT8T_ERR_WORKSPACE);
    EXPECT(int8t_profile_start("no_such_kernel") == INT8T_ERR_ARG);
    EXPECT(int8t_profile_start_sampled("wgrad_kernel", 0) == INT8T_ERR_ARG);
    EXPECT(int8t_dclr_scale(0.0, 20.0, 0.1) == 1.0 && int8t_dclr_scale(1.0, 20.0, 0.1) == 0.1);
    for (int s = 0; s < 9; ++s) EXPECT(int8t_status_string((int8t_status)s) != nullptr);
    if (bad) return 1;
    std::printf("abi sanitize ok\n");
    return 0;
}
