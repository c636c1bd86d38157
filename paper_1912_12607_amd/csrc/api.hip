// C ABI of the library (see include/int8t.h): argument validation, scratch carving, dispatch.
// No device memory is allocated here and nothing synchronises with the host.
#include <math.h>

#include <array>
#include <map>
#include <mutex>

#include "../../include/int8t.h"
#include "kernels.h"
#include "device_common.h"

using namespace int8t;

// Scratch of int8t_dsgc_clip_static: the clip search's absmax partials, its 64-bit accumulator sets
// with the ticket word, and the sum-of-squares partials -- the same three areas int8t_dsgc_clip carves
// out of the caller's scratch.  One copy per GPU, held until the process ends.
#define INT8T_STATIC_A256(v) (((v) + 255) & ~(size_t)255)
constexpr size_t kStaticDsgcBytes = INT8T_STATIC_A256(kMaxPartials * sizeof(float)) +
                                    INT8T_STATIC_A256((kDsgcAccWords + 1) * sizeof(unsigned long long)) +
                                    INT8T_STATIC_A256(kMaxPartials * sizeof(double));
static __device__ __align__(256) unsigned char scratch[kStaticDsgcBytes];

namespace {

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline int pad16(int v) { return (v + 15) & ~15; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; }

constexpr size_t kMaxElems = 0x7FFFFFFFull;   // 32-bit indices inside the kernels

bool dims_ok(const int d[4], size_t* n) {
    if (!d) return false;
    size_t t = 1;
    for (int i = 0; i < 4; ++i) {
        if (d[i] <= 0) return false;
        t *= (size_t)d[i];
        if (t > kMaxElems) return false;
    }
    *n = t;
    return true;
}

struct Geo {
    int P, Q;
    bool depthwise;
};

int8t_status desc_ok(const int8t_conv_desc* d, Geo* g) {
    if (!d) return INT8T_ERR_NULL;
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 ||
        d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0 || d->groups <= 0)
        return INT8T_ERR_SHAPE;
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return INT8T_ERR_SHAPE;
    g->P = (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1;
    g->Q = (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
    if (d->groups == 1) g->depthwise = false;
    else if (d->groups == d->C && d->K == d->C) g->depthwise = true;
    else return INT8T_ERR_SHAPE;
    // element counts must fit the kernels' 32-bit indices (padded channel pitch included)
    const size_t nx = (size_t)d->N * pad16(d->C) * d->H * d->W;
    const size_t ny = (size_t)d->N * pad16(d->K) * g->P * g->Q;
    const size_t nw = (size_t)pad16(d->K) * pad16(d->C / d->groups) * d->R * d->S;
    if (nx > kMaxElems || ny > kMaxElems || nw > kMaxElems) return INT8T_ERR_SHAPE;
    if ((size_t)g->P * g->Q > (1u << 22) || (size_t)d->H * d->W > (1u << 22)) return INT8T_ERR_SHAPE;
    if (g->depthwise) {
        if (d->R * d->S > 64) return INT8T_ERR_SHAPE;
        if ((size_t)d->H * d->W + (size_t)g->P * g->Q > 48000) return INT8T_ERR_SHAPE;   // LDS planes
    }
    return INT8T_OK;
}

// scratch of int8t_quantize: [absmax partials][deviation partials]
size_t quant_ws_bytes(int blocks) { return align256(kMaxPartials * sizeof(float)) + align256((size_t)blocks * sizeof(DevPartial)); }

// The pass that writes a tensor's codes.  Channels-last codes of a 1 x 1 image whose channel count
// needs no padding (the input of a fully connected layer) are the tensor's own element order: the
// element-wise pass writes them, instead of the transposing one at one pixel per block.
int8t_kind pass_kind(const int d[4], int8t_kind kind) {
    if (kind == INT8T_ACT && d[2] * d[3] == 1 && (d[1] & 15) == 0) return INT8T_ACT_PLANAR;
    return kind;
}

int quant_blocks(const int d[4], int8t_kind kind) {
    switch (pass_kind(d, kind)) {
        case INT8T_ACT: return quant_blocks_act(d[0], pad16(d[1]), d[2] * d[3]);
        case INT8T_WGT: return quant_blocks_wgt(d[0], d[1], d[2], d[3]);
        default: return quant_blocks_planar((size_t)d[0] * d[1] * d[2] * d[3]);
    }
}

size_t dsgc_ws_bytes(size_t n) {
    (void)n;
    return align256(kMaxPartials * sizeof(float)) + align256((dsgc_acc_words() + 1) * sizeof(unsigned long long)) +
           align256(kMaxPartials * sizeof(double));
}

void fill_wgrad_geometry(WgradArgs* a, const int8t_conv_desc* d, const Geo& g) {
    a->N = d->N; a->C = d->C; a->Cp = pad16(d->C); a->H = d->H; a->W = d->W;
    a->K = d->K; a->Kp = pad16(d->K); a->P = g.P; a->Q = g.Q; a->R = d->R; a->S = d->S;
    a->stride_h = d->stride_h; a->stride_w = d->stride_w; a->pad_h = d->pad_h; a->pad_w = d->pad_w;
}

// geometry of the implicit GEMMs (pointers are set by the entry points)
void fill_igemm_fwd(IgemmArgs* a, const int8t_conv_desc* d, const Geo& g) {
    a->N = d->N; a->rows = d->K; a->Ca = pad16(d->C);
    a->IH = d->H; a->IW = d->W; a->OH = g.P; a->OW = g.Q; a->R = d->R; a->S = d->S;
    a->stride_h = d->stride_h; a->stride_w = d->stride_w; a->pad_h = d->pad_h; a->pad_w = d->pad_w;
    a->dgrad = 0;
    a->C = d->C;
}
void fill_igemm_bwd_data(IgemmArgs* a, const int8t_conv_desc* d, const Geo& g) {
    a->N = d->N; a->rows = d->C; a->Ca = pad16(d->K);
    a->IH = g.P; a->IW = g.Q; a->OH = d->H; a->OW = d->W; a->R = d->R; a->S = d->S;
    a->stride_h = d->stride_h; a->stride_w = d->stride_w; a->pad_h = d->pad_h; a->pad_w = d->pad_w;
    a->dgrad = 1;
}

// Kernel variants selected per (pass, layer) by int8t_conv_select_variant; everything else runs the
// library's own choice.  Process-wide, guarded by a mutex (a lookup per convolution call).
std::mutex g_variant_mutex;
std::map<std::array<int, 13>, int> g_variant_table;

std::array<int, 13> variant_key(int8t_op op, const int8t_conv_desc* d) {
    return {(int)op, d->N, d->C, d->H, d->W, d->K, d->R, d->S, d->stride_h, d->stride_w, d->pad_h, d->pad_w, d->groups};
}
int selected_variant(int8t_op op, const int8t_conv_desc* d) {
    std::lock_guard<std::mutex> lock(g_variant_mutex);
    if (g_variant_table.empty()) return VAR_AUTO;
    const auto it = g_variant_table.find(variant_key(op, d));
    return it == g_variant_table.end() ? VAR_AUTO : it->second;
}

// whether `variant` can run pass `op` of the layer
bool variant_ok(int8t_op op, const int8t_conv_desc* d, const Geo& g, int variant) {
    if (variant == VAR_AUTO) return true;
    if (g.depthwise) return false;
    if (op == INT8T_OP_CONV_BWD_WEIGHT) {
        if (variant == VAR_WGRAD_FEWER || variant == VAR_WGRAD_MORE || variant == VAR_WGRAD_IMAGES) return true;
        if (variant != VAR_WGRAD_LINES) return false;
        WgradArgs a{};
        fill_wgrad_geometry(&a, d, g);
        (void)wgrad_s2d(&a);
        return wgrad_lines_applies(a);
    }
    if (op != INT8T_OP_CONV_FWD && op != INT8T_OP_CONV_BWD_DATA) return false;
    IgemmArgs a{};
    if (op == INT8T_OP_CONV_FWD) fill_igemm_fwd(&a, d, g);
    else fill_igemm_bwd_data(&a, d, g);
    (void)igemm_s2d(&a);      // a layer that runs on its space-to-depth form is judged in that form
    return igemm_variant_ok(a, variant);
}

}  // namespace

extern "C" {

int int8t_conv_variant_ok(int8t_op op, const int8t_conv_desc* desc, int8t_variant variant) {
    Geo g;
    if (desc_ok(desc, &g) != INT8T_OK) return 0;
    if ((int)variant < 0 || (int)variant >= VAR_COUNT) return 0;
    return variant_ok(op, desc, g, (int)variant) ? 1 : 0;
}

int8t_status int8t_conv_select_variant(int8t_op op, const int8t_conv_desc* desc, int8t_variant variant) {
    Geo g;
    const int8t_status s = desc_ok(desc, &g);
    if (s != INT8T_OK) return s;
    if (op != INT8T_OP_CONV_FWD && op != INT8T_OP_CONV_BWD_DATA && op != INT8T_OP_CONV_BWD_WEIGHT) return INT8T_ERR_ARG;
    if ((int)variant < 0 || (int)variant >= VAR_COUNT || !variant_ok(op, desc, g, (int)variant)) return INT8T_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_variant_mutex);
    if (variant == INT8T_VARIANT_AUTO) g_variant_table.erase(variant_key(op, desc));
    else g_variant_table[variant_key(op, desc)] = (int)variant;
    return INT8T_OK;
}

int8t_variant int8t_conv_selected_variant(int8t_op op, const int8t_conv_desc* desc) {
    Geo g;
    if (desc_ok(desc, &g) != INT8T_OK) return INT8T_VARIANT_AUTO;
    return (int8t_variant)selected_variant(op, desc);
}

const char* int8t_status_string(int8t_status s) {
    switch (s) {
        case INT8T_OK: return "ok";
        case INT8T_ERR_NULL: return "required pointer is NULL";
        case INT8T_ERR_SHAPE: return "bad or unsupported shape";
        case INT8T_ERR_ARG: return "bad argument (enum value, alignment, candidate count)";
        case INT8T_ERR_WORKSPACE: return "workspace too small";
        case INT8T_ERR_RUNTIME: return "HIP launch failed";
        case INT8T_ERR_LIMIT: return "size beyond the limit of the allocation-free variant";
        default: break;
    }
    return "unknown status";
}

size_t int8t_code_bytes(const int dims[4], int8t_kind kind) {
    size_t n;
    if (!dims_ok(dims, &n)) return 0;
    switch (kind) {
        case INT8T_ACT: return (size_t)dims[0] * dims[2] * dims[3] * pad16(dims[1]);
        case INT8T_WGT:
            return align256((size_t)dims[0] * dims[2] * dims[3] * pad16(dims[1])) +
                   (size_t)dims[1] * dims[2] * dims[3] * pad16(dims[0]);
        case INT8T_ACT_PLANAR:
        case INT8T_WGT_PLANAR: return n;
        default: break;
    }
    return 0;
}

int8t_status int8t_unpack_codes(const int8_t* codes_host, const int dims[4], int8t_kind kind, int copy,
                                int8_t* out_host, size_t* pad_nonzero) {
    if (!codes_host || !dims || !out_host) return INT8T_ERR_NULL;
    size_t n;
    if (!dims_ok(dims, &n)) return INT8T_ERR_SHAPE;
    if (kind != INT8T_ACT && kind != INT8T_WGT && kind != INT8T_ACT_PLANAR && kind != INT8T_WGT_PLANAR) return INT8T_ERR_ARG;
    if (copy != 0 && !(kind == INT8T_WGT && copy == 1)) return INT8T_ERR_ARG;
    size_t bad = 0;
    if (kind == INT8T_ACT_PLANAR || kind == INT8T_WGT_PLANAR) {
        for (size_t i = 0; i < n; ++i) out_host[i] = codes_host[i];
    } else {
        // both dense layouts are [outer][plane position][inner padded to 16]: activations outer = N,
        // inner = C; weights, forward copy outer = K, inner = Cg; backward-data copy outer = Cg, inner = K
        const int plane = dims[2] * dims[3];
        const bool second = kind == INT8T_WGT && copy == 1;
        const int outer = second ? dims[1] : dims[0], inner = second ? dims[0] : dims[1];
        const int ip = pad16(inner);
        const int8_t* src = codes_host;
        if (second) src += align256((size_t)dims[0] * plane * pad16(dims[1]));
        for (int o = 0; o < outer; ++o)
            for (int p = 0; p < plane; ++p) {
                const int8_t* g = src + ((size_t)o * plane + p) * ip;
                for (int i = 0; i < inner; ++i) {
                    // logical index: [dims0][dims1][plane]
                    const size_t d0 = second ? (size_t)i : (size_t)o, d1 = second ? (size_t)o : (size_t)i;
                    out_host[(d0 * dims[1] + d1) * plane + p] = g[i];
                }
                for (int i = inner; i < ip; ++i) bad += g[i] != 0;
            }
    }
    if (pad_nonzero) *pad_nonzero = bad;
    return INT8T_OK;
}

size_t int8t_workspace_bytes(int8t_op op, const int8t_conv_desc* desc, size_t n, int n_cand) {
    (void)n_cand;
    switch (op) {
        case INT8T_OP_QUANTIZE: return 0;
        case INT8T_OP_DSGC: return dsgc_ws_bytes(n);
        case INT8T_OP_CONV_FWD:
        case INT8T_OP_CONV_BWD_DATA: {
            // optional: partial sums of a split reduction (layers with few output tiles)
            Geo g;
            if (desc_ok(desc, &g) != INT8T_OK || g.depthwise) return 0;
            // ... and, in the forward pass of a stride-2 layer with at most 4 channels, its rewritten codes
            IgemmArgs a{};
            if (op == INT8T_OP_CONV_FWD) fill_igemm_fwd(&a, desc, g);
            else fill_igemm_bwd_data(&a, desc, g);
            const size_t s2d_bytes = igemm_s2d(&a);   // (sized for the split variant whichever is selected)
            const int ks = igemm_ksplit(a);
            return s2d_bytes + (ks > 1 ? align256((size_t)ks * a.N * a.rows * a.OH * a.OW * 4) : 0);
        }
        case INT8T_OP_CONV_BWD_WEIGHT: {
            Geo g;
            if (desc_ok(desc, &g) != INT8T_OK) return 0;
            if (g.depthwise) {
                int threads, chunks, cg;
                dw_wgrad_shape(desc->N, desc->C, desc->H, desc->W, g.P, g.Q, desc->R, desc->S, desc->stride_h, desc->stride_w, &threads, &chunks, &cg);
                return align256((size_t)chunks * desc->C * desc->R * desc->S * 4);
            }
            WgradArgs a{};
            fill_wgrad_geometry(&a, desc, g);
            const size_t s2d_bytes = wgrad_s2d(&a);
            a.variant = selected_variant(INT8T_OP_CONV_BWD_WEIGHT, desc);
            wgrad_plan(&a);
            return align256((size_t)a.splits * a.K * a.R * a.S * a.Cp * 4) + align256(s2d_bytes);
        }
        default: break;
    }
    return 0;
}

size_t int8t_quantize_workspace_bytes(const int dims[4], int8t_kind kind) {
    size_t n;
    if (!dims_ok(dims, &n)) return 0;
    if (kind != INT8T_ACT && kind != INT8T_WGT && kind != INT8T_ACT_PLANAR && kind != INT8T_WGT_PLANAR) return 0;
    return quant_ws_bytes(quant_blocks(dims, kind));
}

int8t_status int8t_quantize(const float* x_dev, const int dims[4], int8t_kind kind,
                            const float* clip_dev, int8t_round mode, uint64_t seed, int8_t* q_dev,
                            float* scale_dev, double* deviation_dev, void* ws_dev, size_t ws_bytes,
                            void* stream) {
    if (!x_dev || !dims || !q_dev || !scale_dev) return INT8T_ERR_NULL;
    size_t n;
    if (!dims_ok(dims, &n)) return INT8T_ERR_SHAPE;
    if (kind != INT8T_ACT && kind != INT8T_WGT && kind != INT8T_ACT_PLANAR && kind != INT8T_WGT_PLANAR)
        return INT8T_ERR_ARG;
    if (mode != INT8T_ROUND_NEAREST_EVEN && mode != INT8T_ROUND_STOCHASTIC) return INT8T_ERR_ARG;
    if (!aligned16(x_dev) || !aligned16(q_dev) || !aligned4(scale_dev)) return INT8T_ERR_ARG;
    if (kind == INT8T_ACT && (size_t)dims[0] * pad16(dims[1]) * dims[2] * dims[3] > kMaxElems) return INT8T_ERR_SHAPE;
    if (kind == INT8T_ACT && dims[0] > 65535) return INT8T_ERR_SHAPE;   // grid.z
    const bool need_absmax = (clip_dev == nullptr);
    const bool need_dev = (deviation_dev != nullptr);
    const int blocks = quant_blocks(dims, kind);
    if (need_absmax || need_dev) {
        if (!ws_dev) return INT8T_ERR_NULL;
        if (ws_bytes < quant_ws_bytes(need_dev ? blocks : 0)) return INT8T_ERR_WORKSPACE;
        if (!aligned16(ws_dev)) return INT8T_ERR_ARG;
    }
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)ws_dev;
    float* absmax_part = (float*)ws;
    DevPartial* devpart = need_dev ? (DevPartial*)(ws + align256(kMaxPartials * sizeof(float))) : nullptr;

    int nparts = 0;
    if (need_absmax && launch_absmax(x_dev, n, absmax_part, &nparts, st) != hipSuccess) return INT8T_ERR_RUNTIME;
    QuantArgs a;
    a.x = x_dev;
    a.d0 = dims[0]; a.d1 = dims[1]; a.d2 = dims[2]; a.d3 = dims[3];
    a.clip = clip_dev;
    a.absmax_part = absmax_part;
    a.nparts = nparts;
    a.stochastic = (mode == INT8T_ROUND_STOCHASTIC);
    a.seed = seed;
    a.q = q_dev;
    a.scale = scale_dev;
    a.devpart = devpart;
    hipError_t e;
    const int8t_kind pk = pass_kind(dims, kind);
    if (pk == INT8T_ACT) e = launch_quantize_act(a, st);
    else if (pk == INT8T_WGT) e = launch_quantize_wgt(a, st);
    else e = launch_quantize_planar(a, st);
    if (e != hipSuccess) return INT8T_ERR_RUNTIME;
    if (need_dev && launch_deviation_finish(devpart, blocks, deviation_dev, st) != hipSuccess) return INT8T_ERR_RUNTIME;
    return INT8T_OK;
}

size_t int8t_quantize_batch_workspace_bytes(int count, const int8t_quantize_item* items) {
    if (count < 1 || count > INT8T_MAX_BATCH || !items) return 0;
    return (size_t)count * align256(kMaxPartials * sizeof(float));
}

}  // extern "C"

namespace {
DsgcWs dsgc_ws_layout(void* ws_dev);
// int8t_quantize_batch, and with g_dev also the first phase of a clip search on g in the same absmax launch
int8t_status quantize_batch_impl(int count, const int8t_quantize_item* items, void* ws_dev, size_t ws_bytes,
                                 const float* g_dev, size_t g_n, void* dsgc_ws_dev, size_t dsgc_ws_size, void* stream) {
    if (!items) return INT8T_ERR_NULL;
    if (count < 1 || count > INT8T_MAX_BATCH) return INT8T_ERR_ARG;
    if (g_dev) {
        if (!dsgc_ws_dev) return INT8T_ERR_NULL;
        if (g_n == 0 || g_n > kMaxElems) return INT8T_ERR_SHAPE;
        if (!aligned16(g_dev) || !aligned16(dsgc_ws_dev)) return INT8T_ERR_ARG;
        if (dsgc_ws_size < dsgc_ws_bytes(g_n)) return INT8T_ERR_WORKSPACE;
    }
    AbsmaxBatch ab{};
    QuantBatch qb{};
    qb.count = count;
    long long ablocks = 0, qblocks = 0;
    bool any_absmax = false;
    for (int i = 0; i < count; ++i) {
        const int8t_quantize_item& it = items[i];
        if (!it.x_dev || !it.q_dev || !it.scale_dev) return INT8T_ERR_NULL;
        size_t n;
        if (!dims_ok(it.dims, &n)) return INT8T_ERR_SHAPE;
        if (it.kind != INT8T_ACT && it.kind != INT8T_WGT && it.kind != INT8T_ACT_PLANAR && it.kind != INT8T_WGT_PLANAR)
            return INT8T_ERR_ARG;
        if (it.mode != INT8T_ROUND_NEAREST_EVEN && it.mode != INT8T_ROUND_STOCHASTIC) return INT8T_ERR_ARG;
        if (!aligned16(it.x_dev) || !aligned16(it.q_dev) || !aligned4(it.scale_dev) || !aligned4(it.clip_dev))
            return INT8T_ERR_ARG;
        if (it.kind == INT8T_ACT && (size_t)it.dims[0] * pad16(it.dims[1]) * it.dims[2] * it.dims[3] > kMaxElems)
            return INT8T_ERR_SHAPE;
        if (!it.clip_dev) any_absmax = true;
    }
    if (any_absmax) {
        if (!ws_dev) return INT8T_ERR_NULL;
        if (ws_bytes < int8t_quantize_batch_workspace_bytes(count, items)) return INT8T_ERR_WORKSPACE;
        if (!aligned16(ws_dev)) return INT8T_ERR_ARG;
    }
    // Block ranges are dealt smallest tensor first: the dispatcher hands out blocks in order, so the
    // few blocks of a small tensor run beside the first blocks of a large one instead of after its last.
    int order[INT8T_MAX_BATCH];
    size_t sizes[INT8T_MAX_BATCH];
    for (int i = 0; i < count; ++i) {
        order[i] = i;
        (void)dims_ok(items[i].dims, &sizes[i]);
    }
    for (int i = 1; i < count; ++i)
        for (int j = i; j > 0 && sizes[order[j]] < sizes[order[j - 1]]; --j) { const int t = order[j]; order[j] = order[j - 1]; order[j - 1] = t; }
    for (int oi = 0; oi < count; ++oi) {
        const int i = order[oi];
        const int8t_quantize_item& it = items[i];
        const size_t n = sizes[i];
        float* part = any_absmax ? (float*)((char*)ws_dev + (size_t)i * align256(kMaxPartials * sizeof(float))) : nullptr;
        const int nb = it.clip_dev ? 0 : absmax_blocks(n);
        if (nb) {
            AbsmaxBatchItem& a = ab.it[ab.count++];
            a.x = it.x_dev; a.n = n; a.part = part; a.block0 = (int)ablocks; a.nblocks = nb;
            ablocks += nb;
        }
        QuantBatchItem& q = qb.it[oi];
        q.x = it.x_dev; q.d0 = it.dims[0]; q.d1 = it.dims[1]; q.d2 = it.dims[2]; q.d3 = it.dims[3];
        q.clip = it.clip_dev; q.absmax_part = part; q.nparts = nb; q.q = it.q_dev; q.scale = it.scale_dev;
        const int8t_kind pk = pass_kind(it.dims, it.kind);
        q.kind = pk == INT8T_ACT ? 0 : pk == INT8T_WGT ? 1 : 2;
        q.stoch = it.mode == INT8T_ROUND_STOCHASTIC;
        q.seed_lo = seed_key_x(it.seed);
        q.seed_hi = seed_key_a(it.seed);
        quant_grid(q.kind, it.dims, &q.gx, &q.gy, &q.gz);
        q.block0 = (int)qblocks;
        qblocks += (long long)q.gx * q.gy * q.gz;
        if (qblocks > 0x7FFFFFFFll) return INT8T_ERR_SHAPE;
    }
    if (g_dev) {
        const DsgcWs dws = dsgc_ws_layout(dsgc_ws_dev);
        AbsmaxBatchItem& a = ab.it[ab.count++];
        a.x = g_dev; a.n = g_n; a.part = dws.absmax_part; a.block0 = (int)ablocks; a.nblocks = absmax_blocks(g_n);
        a.sumsq = dws.partG; a.zero = dws.acc; a.nzero = (int)dsgc_acc_words() + 1;
        ablocks += a.nblocks;
    }
    hipStream_t st = (hipStream_t)stream;
    if (ab.count && launch_absmax_batch(ab, (int)ablocks, st) != hipSuccess) return INT8T_ERR_RUNTIME;
    if (launch_quantize_batch(qb, (int)qblocks, st) != hipSuccess) return INT8T_ERR_RUNTIME;
    return INT8T_OK;
}
}  // namespace

extern "C" {

int8t_status int8t_quantize_batch(int count, const int8t_quantize_item* items, void* ws_dev, size_t ws_bytes,
                                  void* stream) {
    return quantize_batch_impl(count, items, ws_dev, ws_bytes, nullptr, 0, nullptr, 0, stream);
}

int8t_status int8t_quantize_batch_prepare(int count, const int8t_quantize_item* items, void* ws_dev, size_t ws_bytes,
                                          const float* g_dev, size_t n, void* dsgc_ws_dev, size_t dsgc_ws_size,
                                          void* stream) {
    if (!g_dev) return INT8T_ERR_NULL;
    return quantize_batch_impl(count, items, ws_dev, ws_bytes, g_dev, n, dsgc_ws_dev, dsgc_ws_size, stream);
}

namespace {
DsgcWs dsgc_ws_layout(void* ws_dev) {
    char* p = (char*)ws_dev;
    DsgcWs ws;
    const size_t nacc = dsgc_acc_words();
    ws.absmax_part = (float*)p;                 p += align256(kMaxPartials * sizeof(float));
    ws.acc = (unsigned long long*)p;
    ws.ticket = (unsigned int*)(ws.acc + nacc);  p += align256((nacc + 1) * sizeof(unsigned long long));
    ws.partG = (double*)p;
    return ws;
}
}  // namespace

int8t_status int8t_dsgc_prepare(const float* g_dev, size_t n, void* ws_dev, size_t ws_bytes, void* stream) {
    if (!g_dev || !ws_dev) return INT8T_ERR_NULL;
    if (n == 0 || n > kMaxElems) return INT8T_ERR_SHAPE;
    if (!aligned16(g_dev) || !aligned16(ws_dev)) return INT8T_ERR_ARG;
    if (ws_bytes < dsgc_ws_bytes(n)) return INT8T_ERR_WORKSPACE;
    const DsgcWs ws = dsgc_ws_layout(ws_dev);
    int nparts = 0;
    if (launch_absmax(g_dev, n, ws.absmax_part, &nparts, (hipStream_t)stream, ws.partG, ws.acc,
                      (int)dsgc_acc_words() + 1) != hipSuccess)
        return INT8T_ERR_RUNTIME;
    return INT8T_OK;
}

int8t_status int8t_dsgc_search(const float* g_dev, size_t n, const float* ratios_dev, int n_cand,
                               int8t_round mode, uint64_t seed, float* clip_dev, double* deviation_dev,
                               double* deviation_all_dev, void* ws_dev, size_t ws_bytes, void* stream) {
    if (!g_dev || !ratios_dev || !clip_dev || !deviation_dev || !ws_dev) return INT8T_ERR_NULL;
    if (n == 0 || n > kMaxElems) return INT8T_ERR_SHAPE;
    if (n_cand < 1 || n_cand > INT8T_MAX_CANDIDATES) return INT8T_ERR_ARG;
    if (mode != INT8T_ROUND_NEAREST_EVEN && mode != INT8T_ROUND_STOCHASTIC) return INT8T_ERR_ARG;
    if (!aligned16(g_dev) || !aligned16(ws_dev) || !aligned4(ratios_dev) || !aligned4(clip_dev) ||
        (reinterpret_cast<uintptr_t>(deviation_dev) & 7) || (reinterpret_cast<uintptr_t>(deviation_all_dev) & 7))
        return INT8T_ERR_ARG;
    if (ws_bytes < dsgc_ws_bytes(n)) return INT8T_ERR_WORKSPACE;
    const DsgcWs ws = dsgc_ws_layout(ws_dev);
    if (launch_dsgc(g_dev, n, ratios_dev, n_cand, mode == INT8T_ROUND_STOCHASTIC, seed, ws, absmax_blocks(n), clip_dev,
                    deviation_dev, deviation_all_dev, (hipStream_t)stream) != hipSuccess)
        return INT8T_ERR_RUNTIME;
    return INT8T_OK;
}

int8t_status int8t_dsgc_clip(const float* g_dev, size_t n, const float* ratios_dev, int n_cand,
                             int8t_round mode, uint64_t seed, float* clip_dev, double* deviation_dev,
                             double* deviation_all_dev, void* ws_dev, size_t ws_bytes, void* stream) {
    // argument checks of both phases first, so that nothing is launched on bad input
    if (!g_dev || !ratios_dev || !clip_dev || !deviation_dev || !ws_dev) return INT8T_ERR_NULL;
    if (n == 0 || n > kMaxElems) return INT8T_ERR_SHAPE;
    if (n_cand < 1 || n_cand > INT8T_MAX_CANDIDATES) return INT8T_ERR_ARG;
    if (mode != INT8T_ROUND_NEAREST_EVEN && mode != INT8T_ROUND_STOCHASTIC) return INT8T_ERR_ARG;
    if (!aligned16(g_dev) || !aligned16(ws_dev) || !aligned4(ratios_dev) || !aligned4(clip_dev) ||
        (reinterpret_cast<uintptr_t>(deviation_dev) & 7) || (reinterpret_cast<uintptr_t>(deviation_all_dev) & 7))
        return INT8T_ERR_ARG;
    if (ws_bytes < dsgc_ws_bytes(n)) return INT8T_ERR_WORKSPACE;
    int8t_status s = int8t_dsgc_prepare(g_dev, n, ws_dev, ws_bytes, stream);
    if (s != INT8T_OK) return s;
    return int8t_dsgc_search(g_dev, n, ratios_dev, n_cand, mode, seed, clip_dev, deviation_dev, deviation_all_dev,
                             ws_dev, ws_bytes, stream);
}

namespace {
// Device address of `scratch` on each GPU (every GPU holds its own copy of the array at its own
// address); looked up once per device, with that device current, by the first call on it.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_static_scratch[kMaxDevices];

int8t_status static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return INT8T_ERR_RUNTIME;
    void* p = g_static_scratch[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return INT8T_ERR_RUNTIME;
        g_static_scratch[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return INT8T_OK;
}
}  // namespace

int8t_status int8t_dsgc_clip_static(const float* g_dev, size_t n, const float* ratios_dev, int n_cand,
                                    int8t_round mode, uint64_t seed, float* clip_dev, double* deviation_dev,
                                    double* deviation_all_dev, void* stream) {
    if (!g_dev || !ratios_dev || !clip_dev || !deviation_dev) return INT8T_ERR_NULL;
    if (n == 0) return INT8T_ERR_SHAPE;
    if (n > INT8T_DSGC_STATIC_MAX_ELEMS || n_cand > INT8T_MAX_CANDIDATES) return INT8T_ERR_LIMIT;
    static_assert(INT8T_DSGC_STATIC_MAX_ELEMS <= kMaxElems, "the static variant's limit is the kernels' own");
    static_assert(kStaticDsgcBytes == INT8T_DSGC_STATIC_SCRATCH_BYTES, "size stated in the header");
    void* ws = nullptr;
    const int8t_status s = static_scratch(&ws);
    if (s != INT8T_OK) return s;
    if (dsgc_ws_bytes(n) > kStaticDsgcBytes) return INT8T_ERR_LIMIT;
    // the same two phases on the GPU's own array; the first pass clears the accumulators and the
    // ticket with its own stores (no memset node, so a caller may capture the call into a graph)
    return int8t_dsgc_clip(g_dev, n, ratios_dev, n_cand, mode, seed, clip_dev, deviation_dev, deviation_all_dev, ws,
                           kStaticDsgcBytes, stream);
}

int8t_status int8t_conv_fwd(const int8t_conv_desc* desc, const int8_t* xq_dev, const float* sx_dev,
                            const int8_t* wq_dev, const float* sw_dev, float* y_dev, int32_t* acc_dev,
                            void* ws_dev, size_t ws_bytes, void* stream) {
    Geo g;
    int8t_status s = desc_ok(desc, &g);
    if (s != INT8T_OK) return s;
    if (!xq_dev || !sx_dev || !wq_dev || !sw_dev || !y_dev) return INT8T_ERR_NULL;
    if (!aligned16(xq_dev) || !aligned16(wq_dev) || !aligned16(y_dev) || !aligned4(acc_dev) || !aligned16(ws_dev))
        return INT8T_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (g.depthwise) {
        DwArgs a{};
        a.a = xq_dev; a.b = wq_dev; a.sa = sx_dev; a.sb = sw_dev; a.out = y_dev; a.acc = acc_dev;
        a.N = desc->N; a.C = desc->C; a.IH = desc->H; a.IW = desc->W; a.OH = g.P; a.OW = g.Q;
        a.R = desc->R; a.S = desc->S; a.stride_h = desc->stride_h; a.stride_w = desc->stride_w;
        a.pad_h = desc->pad_h; a.pad_w = desc->pad_w; a.dgrad = 0;
        return launch_dw_conv(a, st) == hipSuccess ? INT8T_OK : INT8T_ERR_RUNTIME;
    }
    IgemmArgs a{};
    fill_igemm_fwd(&a, desc, g);
    a.variant = selected_variant(INT8T_OP_CONV_FWD, desc);
    a.act = xq_dev; a.wgt = wq_dev; a.sa = sx_dev; a.sb = sw_dev; a.out = y_dev; a.acc = acc_dev;
    a.partial = (int32_t*)ws_dev; a.partial_bytes = ws_dev ? ws_bytes : 0;
    {
        // the rewritten codes of a layer s2d.hip covers come first in the scratch; without it the layer runs as it is
        IgemmArgs t = a;
        const size_t s2d_bytes = igemm_s2d(&t);
        if (s2d_bytes && a.partial_bytes >= s2d_bytes) {
            a.s2d = (int8_t*)ws_dev;
            a.partial = (int32_t*)((int8_t*)ws_dev + s2d_bytes);
            a.partial_bytes -= s2d_bytes;
        }
    }
    return launch_igemm(a, st) == hipSuccess ? INT8T_OK : INT8T_ERR_RUNTIME;
}

int8t_status int8t_conv_fwd_fused(const int8t_conv_desc* desc, const float* x_dev, const float* clip_dev,
                                  const int8_t* wq_dev, const float* sw_dev, float* y_dev, int32_t* acc_dev,
                                  int8_t* xq_dev, float* sx_dev, void* ws_dev, size_t ws_bytes, void* stream) {
    Geo g;
    int8t_status s = desc_ok(desc, &g);
    if (s != INT8T_OK) return s;
    if (g.depthwise || desc->R != 1 || desc->S != 1 || desc->stride_h != 1 || desc->stride_w != 1 || desc->pad_h || desc->pad_w)
        return INT8T_ERR_SHAPE;
    if (!x_dev || !wq_dev || !sw_dev || !y_dev || !sx_dev) return INT8T_ERR_NULL;
    if (!aligned16(x_dev) || !aligned16(wq_dev) || !aligned16(y_dev) || !aligned4(acc_dev) || !aligned16(xq_dev) ||
        !aligned4(sx_dev) || !aligned4(clip_dev) || !aligned16(ws_dev))
        return INT8T_ERR_ARG;
    if (!clip_dev) {
        if (!ws_dev) return INT8T_ERR_NULL;
        if (ws_bytes < kMaxPartials * sizeof(float)) return INT8T_ERR_WORKSPACE;
    }
    hipStream_t st = (hipStream_t)stream;
    IgemmArgs a{};
    fill_igemm_fwd(&a, desc, g);
    a.xf = x_dev; a.xclip = clip_dev; a.xq_out = xq_dev; a.sx_out = sx_dev;
    a.wgt = wq_dev; a.sb = sw_dev; a.out = y_dev; a.acc = acc_dev;
    if (!clip_dev) {
        a.xabs_part = (const float*)ws_dev;
        if (launch_absmax(x_dev, (size_t)desc->N * desc->C * desc->H * desc->W, (float*)ws_dev, &a.xabs_nparts, st) != hipSuccess)
            return INT8T_ERR_RUNTIME;
    }
    return launch_igemm_fused(a, st) == hipSuccess ? INT8T_OK : INT8T_ERR_RUNTIME;
}

int8t_status int8t_conv_bwd_data(const int8t_conv_desc* desc, const int8_t* dyq_dev, const float* sdy_dev,
                                 const int8_t* wq_dev, const float* sw_dev, float* dx_dev, int32_t* acc_dev,
                                 void* ws_dev, size_t ws_bytes, void* stream) {
    Geo g;
    int8t_status s = desc_ok(desc, &g);
    if (s != INT8T_OK) return s;
    if (!dyq_dev || !sdy_dev || !wq_dev || !sw_dev || !dx_dev) return INT8T_ERR_NULL;
    if (!aligned16(dyq_dev) || !aligned16(wq_dev) || !aligned16(dx_dev) || !aligned4(acc_dev) || !aligned16(ws_dev))
        return INT8T_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (g.depthwise) {
        DwArgs a{};
        a.a = dyq_dev; a.b = wq_dev; a.sa = sdy_dev; a.sb = sw_dev; a.out = dx_dev; a.acc = acc_dev;
        a.N = desc->N; a.C = desc->C; a.IH = g.P; a.IW = g.Q; a.OH = desc->H; a.OW = desc->W;
        a.R = desc->R; a.S = desc->S; a.stride_h = desc->stride_h; a.stride_w = desc->stride_w;
        a.pad_h = desc->pad_h; a.pad_w = desc->pad_w; a.dgrad = 1;
        return launch_dw_conv(a, st) == hipSuccess ? INT8T_OK : INT8T_ERR_RUNTIME;
    }
    IgemmArgs a{};
    fill_igemm_bwd_data(&a, desc, g);
    a.variant = selected_variant(INT8T_OP_CONV_BWD_DATA, desc);
    a.act = dyq_dev;
    // second copy of the weight codes: [C][R][S][Kp]
    a.wgt = wq_dev + align256((size_t)desc->K * desc->R * desc->S * pad16(desc->C));
    a.sa = sdy_dev; a.sb = sw_dev; a.out = dx_dev; a.acc = acc_dev;
    a.partial = (int32_t*)ws_dev; a.partial_bytes = ws_dev ? ws_bytes : 0;
    return launch_igemm(a, st) == hipSuccess ? INT8T_OK : INT8T_ERR_RUNTIME;
}

int8t_status int8t_conv_bwd_weight(const int8t_conv_desc* desc, const int8_t* xq_dev, const float* sx_dev,
                                   const int8_t* dyq_dev, const float* sdy_dev, float* dw_dev, int32_t* acc_dev,
                                   void* ws_dev, size_t ws_bytes, void* stream) {
    Geo g;
    int8t_status s = desc_ok(desc, &g);
    if (s != INT8T_OK) return s;
    if (!xq_dev || !sx_dev || !dyq_dev || !sdy_dev || !dw_dev || !ws_dev) return INT8T_ERR_NULL;
    if (!aligned16(xq_dev) || !aligned16(dyq_dev) || !aligned16(dw_dev) || !aligned4(acc_dev) || !aligned16(ws_dev))
        return INT8T_ERR_ARG;
    if (ws_bytes < int8t_workspace_bytes(INT8T_OP_CONV_BWD_WEIGHT, desc, 0, 0)) return INT8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (g.depthwise) {
        DwArgs a{};
        a.a = xq_dev; a.b = dyq_dev; a.sa = sx_dev; a.sb = sdy_dev; a.out = dw_dev; a.acc = acc_dev;
        a.partial = (int32_t*)ws_dev;
        dw_wgrad_shape(desc->N, desc->C, desc->H, desc->W, g.P, g.Q, desc->R, desc->S, desc->stride_h, desc->stride_w, &a.threads, &a.chunks, &a.cg);
        a.N = desc->N; a.C = desc->C; a.IH = desc->H; a.IW = desc->W; a.OH = g.P; a.OW = g.Q;
        a.R = desc->R; a.S = desc->S; a.stride_h = desc->stride_h; a.stride_w = desc->stride_w;
        a.pad_h = desc->pad_h; a.pad_w = desc->pad_w; a.dgrad = 0;
        return launch_dw_wgrad(a, st) == hipSuccess ? INT8T_OK : INT8T_ERR_RUNTIME;
    }
    WgradArgs a{};
    fill_wgrad_geometry(&a, desc, g);
    wgrad_s2d(&a);
    a.variant = selected_variant(INT8T_OP_CONV_BWD_WEIGHT, desc);
    wgrad_plan(&a);
    a.x = xq_dev; a.dy = dyq_dev; a.sa = sx_dev; a.sb = sdy_dev; a.dw = dw_dev; a.acc = acc_dev;
    a.partial = (int32_t*)ws_dev;
    a.xs = (int8_t*)ws_dev + align256((size_t)a.splits * a.K * a.R * a.S * a.Cp * 4);
    return launch_wgrad(a, st) == hipSuccess ? INT8T_OK : INT8T_ERR_RUNTIME;
}

double int8t_dclr_scale(double d_c, double alpha, double beta) {
    const double e = exp(-alpha * d_c);
    return e > beta ? e : beta;
}

}  // extern "C"
