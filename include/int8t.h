/*
 * int8t.h -- C ABI of the MI355X (gfx950) INT8 training-convolution library.
 *
 * The calls are the per-layer steps of "Towards Unified INT8 Training for
 * Convolutional Neural Network":
 *
 *   int8t_quantize         Eq.1 (symmetric uniform quantizer, s = c/127) with
 *                          round-to-nearest for activations / weights and the
 *                          stochastic rounding of Eq.3 for output gradients;
 *                          optionally reports the direction deviation of Eq.6.
 *   int8t_dsgc_clip        Direction Sensitive Gradient Clipping (Sec.3.4): picks
 *                          the clip value of the output gradient that minimises
 *                          the cosine deviation d_c of Eq.6, as a search over
 *                          caller-supplied candidates; also returns d_c, the
 *                          scalar Eq.7 consumes.
 *   int8t_conv_fwd         z  = q_a (*) q_W          int8 x int8 -> int32, then Eq.2
 *   int8t_conv_bwd_data    g_a = q_gz (*)^T q_W      (Sec.3.4; Suppl. "INT8 Convolution")
 *   int8t_conv_bwd_weight  g_W = q_gz^T q_a          (Sec.3.4)
 *   int8t_dclr_scale       Eq.7, phi(d_c) = max(exp(-alpha d_c), beta)   (host)
 *
 * General conventions
 *   - Every pointer named *_dev is DEVICE memory owned by the caller.  The library
 *     never allocates, frees or keeps device memory between calls.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued asynchronously on it; no call synchronises with the host.
 *   - Scalars that flow between calls (clip, scale, deviation) stay in device
 *     memory, so the calls of one layer step chain without a host round trip.
 *   - fp32 tensors are dense, in PyTorch's logical order: activations and
 *     gradients N,C,H,W; weights K,C/groups,R,S.  They must be 16-byte aligned.
 *   - Errors are return codes.  Argument errors are detected before anything is
 *     launched; in that case no output is touched.
 *   - `ws_dev` is scratch the caller provides; ask int8t_workspace_bytes() how
 *     much a call needs.  Its contents need no initialisation and are
 *     unspecified afterwards.  Two calls that run concurrently (different
 *     streams) must not share scratch.
 *   - Inputs must be finite.  NaN quantizes to code 0; results derived from
 *     non-finite inputs are otherwise unspecified (but memory safe).
 *
 * Layout of int8 code tensors (the library's own; Suppl. "INT8 Convolution"
 * packs the reduction dimension innermost for the dot-product instruction, and
 * so do we, in granules of 16 bytes for the int8 MFMA):
 *   INT8T_ACT         dims {N,C,H,W}: codes[((n*H + h)*W + w)*Cp + c], Cp = C rounded up
 *                     to a multiple of 16, bytes c >= C are zero.  N*H*W*Cp bytes.
 *   INT8T_ACT_PLANAR  dims {N,C,H,W}: codes in logical N,C,H,W order (depthwise layers).
 *   INT8T_WGT         dims {K,Cg,R,S} (Cg = C/groups, groups == 1): two copies,
 *                       [0, K*R*S*Cp):             codes[((k*R + r)*S + s)*Cp + c]
 *                       [align256(K*R*S*Cp), ...): codes[((c*R + r)*S + s)*Kp + k]
 *                     (the second serves backward-data), Cp/Kp rounded up to 16, pad zero.
 *   INT8T_WGT_PLANAR  dims {K,Cg,R,S}: codes in logical order (depthwise layers).
 * int8t_code_bytes() returns the size of each.
 *
 * The stochastic draw of element i is a function of (seed, i) only, where i is
 * the element's linear index in LOGICAL order, so codes do not depend on the
 * code layout, the launch geometry or the clip search.
 */
#ifndef INT8T_H
#define INT8T_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    INT8T_OK = 0,
    INT8T_ERR_NULL = 1,       /* a required pointer is NULL */
    INT8T_ERR_SHAPE = 2,      /* non-positive or unsupported dimensions */
    INT8T_ERR_ARG = 3,        /* bad enum value, misaligned pointer, too many candidates */
    INT8T_ERR_WORKSPACE = 4,  /* ws_bytes smaller than int8t_workspace_bytes() */
    INT8T_ERR_RUNTIME = 5,    /* a HIP launch failed */
    INT8T_ERR_LIMIT = 6,      /* size beyond what an allocation-free variant (int8t_dsgc_clip_static) takes */
    INT8T_STATUS_MAX_ENUM = 0x7fffffff
} int8t_status;

/* (The *_MAX_ENUM enumerators only make every non-negative int a representable value of its enum, so
 * that a caller's out-of-range argument reaches the argument checks as a value, not as undefined
 * behaviour in the C++ implementation.  They are never returned and never valid as arguments.) */
typedef enum { INT8T_ROUND_NEAREST_EVEN = 0, INT8T_ROUND_STOCHASTIC = 1, INT8T_ROUND_MAX_ENUM = 0x7fffffff } int8t_round;

typedef enum {
    INT8T_ACT = 0,
    INT8T_WGT = 1,
    INT8T_ACT_PLANAR = 2,
    INT8T_WGT_PLANAR = 3,
    INT8T_KIND_MAX_ENUM = 0x7fffffff
} int8t_kind;

typedef enum {
    INT8T_OP_QUANTIZE = 0,
    INT8T_OP_DSGC = 1,
    INT8T_OP_CONV_FWD = 2,
    INT8T_OP_CONV_BWD_DATA = 3,
    INT8T_OP_CONV_BWD_WEIGHT = 4,
    INT8T_OP_MAX_ENUM = 0x7fffffff
} int8t_op;

/* Convolution geometry, PyTorch conventions: cross-correlation, zero padding,
 * P = floor((H + 2 pad_h - R)/stride_h) + 1, dilation 1.  groups must be 1
 * (dense; code layouts INT8T_ACT / INT8T_WGT) or C == K == groups (depthwise;
 * INT8T_ACT_PLANAR / INT8T_WGT_PLANAR). */
typedef struct {
    int N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups;
} int8t_conv_desc;

#define INT8T_MAX_CANDIDATES 64

const char *int8t_status_string(int8t_status s);

/* Bytes of the int8 code tensor of `kind` for logical dims; 0 on bad input. */
size_t int8t_code_bytes(const int dims[4], int8t_kind kind);

/*
 * Checking aid (HOST memory on both sides, plain loops, no GPU work): rewrites a code tensor from the
 * library's layout (see "Layout of int8 code tensors" above; Suppl. "INT8 Convolution" for why the
 * reduction dimension is packed innermost) into logical order, so that a caller can compare codes
 * with Eq.1 / Eq.3 evaluated element by element without knowing the layout.
 *   codes_host    int8t_code_bytes(dims, kind) bytes copied back from the device
 *   copy          INT8T_WGT only: 0 = the forward copy [K][R][S][Cp], 1 = the backward-data copy
 *                 [C][R][S][Kp]; must be 0 for the other kinds
 *   out_host      out: dims[0]*dims[1]*dims[2]*dims[3] codes in logical order (N,C,H,W or K,Cg,R,S)
 *   pad_nonzero   NULL, or out: number of padding bytes (channel positions >= C resp. >= K) of the
 *                 unpacked copy that are not zero -- the convolutions rely on their being zero
 * Returns INT8T_ERR_NULL / INT8T_ERR_SHAPE / INT8T_ERR_ARG on bad input and touches nothing then.
 */
int8t_status int8t_unpack_codes(const int8_t *codes_host, const int dims[4], int8t_kind kind, int copy,
                                int8_t *out_host, size_t *pad_nonzero);

/* Scratch a call needs.  DSGC: n = element count, n_cand = number of candidates, desc ignored.
 * CONV_*: desc required, n / n_cand ignored.  QUANTIZE: use int8t_quantize_workspace_bytes()
 * (this function returns 0 for it).  0 also means "bad arguments" for the CONV ops whose
 * descriptor is invalid; the call itself then reports the error.
 * CONV_BWD_WEIGHT and DSGC require their scratch.  CONV_FWD / CONV_BWD_DATA only use it as a
 * performance aid (layers with few output tiles and a long reduction split the reduction over
 * several workgroups and keep int32 partial sums there; the forward pass of a stride-2 layer with
 * at most 4 input channels -- the stem of an image network -- runs on a space-to-depth copy of its
 * codes kept there, four times the channels per 16-byte pixel and a quarter of the taps; integer
 * sums of the same products either way, so the result is the same bit for bit): ws_dev may be NULL
 * or smaller, the call then runs without them.  CONV_BWD_WEIGHT of such a layer holds the same
 * copy of the input codes in its (required) scratch. */
size_t int8t_workspace_bytes(int8t_op op, const int8t_conv_desc *desc, size_t n, int n_cand);

/* Scratch of int8t_quantize for a tensor of logical dims and code layout `kind`; covers both the
 * absmax pass (clip_dev == NULL) and the deviation output.  0 on bad input. */
size_t int8t_quantize_workspace_bytes(const int dims[4], int8t_kind kind);

/*
 * Eq.1 / Eq.3.  Per element (fp32, each operation rounded once, no fused multiply-add):
 *     inv = 127 / c
 *     nearest:    q = rint(min(max(x * inv, -127), 127))                 (ties to even)
 *     stochastic: m = min(127, floor((|x| * (inv * 2^24) + u) / 2^24)) in exact arithmetic,
 *                 q = sign(x) * m,  u = 24 uniform bits drawn from (seed, logical index)
 *                 ==> |q| = floor(|x|/s) + 1 with probability frac(|x|/s), resolved to 2^-24:
 *                 the distribution of Eq.3 (rounding the magnitude and restoring the sign keeps
 *                 the probabilities of floor and floor + 1 also for negative values).
 *   x_dev          fp32 tensor, logical order, dims[0]*dims[1]*dims[2]*dims[3] elements
 *   clip_dev       clip value c (1 float), or NULL: c = max|x| is computed first
 *   q_dev          out: int8 codes in the layout of `kind`, int8t_code_bytes() bytes
 *   scale_dev      out: 1 float, s = c / 127 (0 when c == 0, and then all codes are 0)
 *   deviation_dev  NULL, or out: 1 double, d_c of Eq.6 between x and q*s
 *                  (0 when x is all zero; 1 when every code is 0 but x is not)
 */
int8t_status int8t_quantize(const float *x_dev, const int dims[4], int8t_kind kind,
                            const float *clip_dev, int8t_round mode, uint64_t seed,
                            int8_t *q_dev, float *scale_dev, double *deviation_dev,
                            void *ws_dev, size_t ws_bytes, void *stream);

/*
 * Eq.1 / Eq.3 for several tensors at once (no deviation output): the result of each item is exactly
 * what int8t_quantize(..., mode, seed, ...) writes for it, but all absmax passes share one launch
 * and all quantize passes another.  Meant for the activations and the weights of a layer -- and, in
 * an iteration that keeps the clip value of an earlier search (Periodic Update, Sec.3.4), its
 * output gradient too -- or the weights of many layers: a small tensor no longer costs two kernel
 * launches of its own.
 *   items    host array of `count` (1 .. INT8T_MAX_BATCH) items, read before the call returns;
 *            fields as the arguments of the same names of int8t_quantize
 *   ws_dev   int8t_quantize_batch_workspace_bytes() bytes, 16-byte aligned; may be NULL when every
 *            item brings its clip value
 */
#define INT8T_MAX_BATCH 8
typedef struct int8t_quantize_item {
    const float *x_dev;
    int dims[4];
    int8t_kind kind;
    const float *clip_dev;
    int8_t *q_dev;
    float *scale_dev;
    int8t_round mode;
    uint64_t seed;             /* used by INT8T_ROUND_STOCHASTIC only */
} int8t_quantize_item;
size_t int8t_quantize_batch_workspace_bytes(int count, const int8t_quantize_item *items);
int8t_status int8t_quantize_batch(int count, const int8t_quantize_item *items,
                                  void *ws_dev, size_t ws_bytes, void *stream);

/*
 * Clip search of Sec.3.4.  Candidates c_j = fl32(max|g| * ratios[j]), j < n_cand
 * (1 <= n_cand <= INT8T_MAX_CANDIDATES).  For each, the tensor is quantized exactly
 * as int8t_quantize(mode, seed) would, and d_j = 1 - cos(g, q*s) (Eq.6) is evaluated;
 * the smallest d_j wins, ties go to the smallest j.
 *   g_dev              fp32 tensor, n elements (n < 2^31), logical order
 *   ratios_dev         n_cand floats in (0, 1]
 *   clip_dev           out: 1 float, the winning c_j
 *   deviation_dev      out: 1 double, its d_j
 *   deviation_all_dev  NULL, or out: n_cand doubles, every d_j
 */
int8t_status int8t_dsgc_clip(const float *g_dev, size_t n, const float *ratios_dev, int n_cand,
                             int8t_round mode, uint64_t seed,
                             float *clip_dev, double *deviation_dev, double *deviation_all_dev,
                             void *ws_dev, size_t ws_bytes, void *stream);

/*
 * The same search in its two phases, for callers that want to put something between them (an event
 * for a second stream, say): int8t_dsgc_prepare is the pass over g that finds max|g| and the sum of
 * squares of Eq.6 and clears the accumulators in the scratch; int8t_dsgc_search is the sweep over
 * the candidates, which needs the scratch exactly as the preceding int8t_dsgc_prepare on the same g,
 * n and ws_dev left it.  int8t_dsgc_clip is the two calls in a row; arguments as there.
 */
int8t_status int8t_dsgc_prepare(const float *g_dev, size_t n, void *ws_dev, size_t ws_bytes, void *stream);
/*
 * int8t_quantize_batch and int8t_dsgc_prepare in one call: the pass over g shares the launch of the items'
 * absmax passes (a step on one stream then has one launch fewer; Sec.3.4: max|.| of a, W and g_z are
 * independent of each other).  Writes what the two calls write, bit for bit; int8t_dsgc_search follows it
 * as it follows int8t_dsgc_prepare.
 *   count, items, ws_dev, ws_bytes   as for int8t_quantize_batch
 *   g_dev, n                         as for int8t_dsgc_prepare (required)
 *   dsgc_ws_dev, dsgc_ws_bytes       the search's scratch: int8t_workspace_bytes(INT8T_OP_DSGC, NULL, n, n_cand) bytes,
 *                                    16-byte aligned, not overlapping ws_dev
 * Errors as for the two calls; nothing is launched then.
 */
int8t_status int8t_quantize_batch_prepare(int count, const int8t_quantize_item *items, void *ws_dev, size_t ws_bytes,
                                          const float *g_dev, size_t n, void *dsgc_ws_dev, size_t dsgc_ws_bytes,
                                          void *stream);
int8t_status int8t_dsgc_search(const float *g_dev, size_t n, const float *ratios_dev, int n_cand,
                               int8t_round mode, uint64_t seed,
                               float *clip_dev, double *deviation_dev, double *deviation_all_dev,
                               void *ws_dev, size_t ws_bytes, void *stream);

/*
 * int8t_dsgc_clip for callers that cannot provide scratch because they cannot allocate: code under
 * HIP graph capture, tight serving / training loops, harnesses that forbid hipMalloc.  Same search,
 * same results bit for bit, same arguments minus ws_dev / ws_bytes: the scratch (absmax partials,
 * accumulator sets and ticket, sum-of-squares partials; INT8T_DSGC_STATIC_SCRATCH_BYTES = 61 696 bytes,
 * whatever n is) is an array inside the library's device image, one copy per GPU, held until the
 * process ends.  The call allocates and frees nothing -- no hipMalloc, no hipFree, no allocating
 * library routine -- and clears what must start at zero with a kernel's own stores, not a memset node.
 *   Limits: n <= INT8T_DSGC_STATIC_MAX_ELEMS and n_cand <= INT8T_MAX_CANDIDATES, else
 *   INT8T_ERR_LIMIT and nothing is launched (n == 0 is INT8T_ERR_SHAPE, n_cand < 1 INT8T_ERR_ARG).
 *   All calls on one GPU share that GPU's array, which keeps the previous call's contents: calls on
 *   the same stream are ordered and safe; calls that OVERLAP on one GPU (different streams, or
 *   several host threads on several streams) race on it and give wrong results.  Use
 *   int8t_dsgc_clip with separate scratch for concurrent searches.
 *   The first call on a GPU looks the array's device address up (hipGetSymbolAddress, with that GPU
 *   current); make that call outside stream capture.
 */
#define INT8T_DSGC_STATIC_SCRATCH_BYTES 61696
#define INT8T_DSGC_STATIC_MAX_ELEMS 0x7FFFFFFFull
int8t_status int8t_dsgc_clip_static(const float *g_dev, size_t n, const float *ratios_dev, int n_cand,
                                    int8t_round mode, uint64_t seed,
                                    float *clip_dev, double *deviation_dev, double *deviation_all_dev,
                                    void *stream);

/*
 * Forward convolution on codes: acc[n,k,p,q] = sum_{c,r,s} xq[n,c,p*sh+r-ph,q*sw+s-pw] * wq[k,c,r,s]
 * in int32 (two's-complement wrap), then Eq.2: y = (float)acc * (sx * sw).
 *   xq_dev   INT8T_ACT codes of dims {N,C,H,W}   (INT8T_ACT_PLANAR when depthwise)
 *   wq_dev   INT8T_WGT codes of dims {K,C/g,R,S} (INT8T_WGT_PLANAR when depthwise)
 *   sx_dev, sw_dev   1 float each (the scales int8t_quantize wrote)
 *   y_dev    out: fp32 N,K,P,Q
 *   acc_dev  NULL, or out: int32 N,K,P,Q, the raw accumulators
 *   ws_dev   NULL, or int8t_workspace_bytes(INT8T_OP_CONV_FWD, ...) bytes of scratch, 16-byte aligned
 *            (optional, see there; the same holds for int8t_conv_bwd_data)
 */
int8t_status int8t_conv_fwd(const int8t_conv_desc *desc,
                            const int8_t *xq_dev, const float *sx_dev,
                            const int8_t *wq_dev, const float *sw_dev,
                            float *y_dev, int32_t *acc_dev,
                            void *ws_dev, size_t ws_bytes, void *stream);

/*
 * The quantization-convolution fused kernel of the paper's Suppl. "INT8 Convolution" ("avoids one
 * extra global memory read and write"), for the layers where it saves traffic here: a 1 x 1 filter at
 * stride 1 without padding (dense).  int8t_quantize(a) + int8t_conv_fwd in one call: the forward pass
 * reads the fp32 activations, applies Eq.1 (round to nearest) in its load path with c = *clip_dev or
 * max|a| (found by a first pass when clip_dev is NULL), and multiplies the codes without their making
 * the round trip through memory.  Results are bit for bit those of the two separate calls.
 *   x_dev    fp32 N,C,H,W;  wq_dev / sw_dev as in int8t_conv_fwd
 *   xq_dev   NULL, or out: the INT8T_ACT codes of a, for the backward-weight pass (a forward-only
 *            caller leaves it out and saves their write as well)
 *   sx_dev   out: 1 float, the scale of a
 *   ws_dev   1024 floats of scratch when clip_dev is NULL, else unused
 * INT8T_ERR_SHAPE for any other filter, stride, padding or a depthwise layer.  A layer with more
 * than 128 filters reads (and quantizes) its activations once per 128 filters: the separate calls are
 * the better choice there.
 */
int8t_status int8t_conv_fwd_fused(const int8t_conv_desc *desc, const float *x_dev, const float *clip_dev,
                                  const int8_t *wq_dev, const float *sw_dev,
                                  float *y_dev, int32_t *acc_dev, int8_t *xq_dev, float *sx_dev,
                                  void *ws_dev, size_t ws_bytes, void *stream);

/*
 * Backward-data: acc[n,c,h,w] = sum over (k,r,s,p,q) with p*sh+r-ph = h, q*sw+s-pw = w of
 * dyq[n,k,p,q] * wq[k,c,r,s];  dx = (float)acc * (sdy * sw).
 *   dyq_dev  INT8T_ACT codes of dims {N,K,P,Q} (planar when depthwise);  wq_dev as in forward
 *   dx_dev   out: fp32 N,C,H,W;   acc_dev NULL or int32 N,C,H,W
 */
int8t_status int8t_conv_bwd_data(const int8t_conv_desc *desc,
                                 const int8_t *dyq_dev, const float *sdy_dev,
                                 const int8_t *wq_dev, const float *sw_dev,
                                 float *dx_dev, int32_t *acc_dev,
                                 void *ws_dev, size_t ws_bytes, void *stream);

/*
 * Backward-weight: acc[k,c,r,s] = sum_{n,p,q} dyq[n,k,p,q] * xq[n,c,p*sh+r-ph,q*sw+s-pw];
 * dw = (float)acc * (sdy * sx).  The forward's codes of x are re-used.
 *   dw_dev   out: fp32 K,C/g,R,S;   acc_dev NULL or int32 K,C/g,R,S
 */
int8t_status int8t_conv_bwd_weight(const int8t_conv_desc *desc,
                                   const int8_t *xq_dev, const float *sx_dev,
                                   const int8_t *dyq_dev, const float *sdy_dev,
                                   float *dw_dev, int32_t *acc_dev,
                                   void *ws_dev, size_t ws_bytes, void *stream);

/*
 * Choice of the kernel per layer by measurement "before training" (Suppl. "INT8 Convolution", last
 * paragraph: the paper picks between its two convolution algorithms per layer; here the choice is
 * among this library's kernels for a pass).  Every variant computes the same integer sums, so the
 * results are identical bit for bit; a caller times the variants int8t_conv_variant_ok() admits on
 * the layer's own buffers and selects the fastest.  The selection is kept in a process-wide table
 * keyed by (pass, descriptor) until it is changed; INT8T_VARIANT_AUTO (the default for every layer)
 * restores the library's own rules.  Thread-safe; not device-specific.
 *   forward / backward-data:  BAND, TILE, TILE_SPLIT, WIDE128, WIDE256, WIDE_SQ128, WIDE_SQ128_DEEP, WIDE_128X64;
 *   backward-data only:       WIDE_CELLS
 *   backward-weight:          WGRAD_IMAGES, WGRAD_LINES (the two kernels), WGRAD_FEWER, WGRAD_MORE (half / twice the
 *                             reduction shares of the cost model's choice); query int8t_workspace_bytes() again
 *                             after selecting any of them
 * Depthwise layers are served by the library's own choice among their kernels only.  A variant that needs scratch (TILE_SPLIT) and is not
 * given enough falls back to TILE.
 */
typedef enum {
    INT8T_VARIANT_AUTO = 0,
    INT8T_VARIANT_BAND = 1,          /* filter bank resident on chip, output rows streamed (small banks, stride 1) */
    INT8T_VARIANT_TILE = 2,          /* 64/128 x 128 implicit-GEMM tiles staged through registers */
    INT8T_VARIANT_TILE_SPLIT = 3,    /* ... with the reduction split over several blocks per tile */
    INT8T_VARIANT_WIDE128 = 4,       /* 128 x 256 tiles, operands loaded straight into a 3-stage LDS ring */
    INT8T_VARIANT_WIDE256 = 5,       /* 256 x 256 tiles, 2 stages of 128 reduction bytes */
    INT8T_VARIANT_WGRAD_FEWER = 6,
    INT8T_VARIANT_WGRAD_MORE = 7,
    INT8T_VARIANT_WGRAD_IMAGES = 8,  /* backward-weight: operands of 16 images per pixel, transposed in registers */
    INT8T_VARIANT_WGRAD_LINES = 9,   /* backward-weight, stride 1 with 1, 3 or 7 taps along an axis, 1x1 at any stride without
                                        padding, or 3x3 at stride 2 x 2: operands of 32 image lines per position through
                                        transposing LDS reads, gradient operands in a sliding window */
    INT8T_VARIANT_WIDE_SQ128 = 10,   /* forward / backward-data: 128 x 128 tiles from a 3-stage LDS ring, three blocks per
                                        compute unit: layers that have too few of the larger tiles to go round */
    INT8T_VARIANT_WIDE_SQ128_DEEP = 11,  /* ... with 2 stages of 128 reduction bytes: long reductions */
    INT8T_VARIANT_WIDE_128X64 = 12,      /* ... 128 x 64 tiles with 128-byte stages: few columns (7 x 7 images) */
    INT8T_VARIANT_WIDE_CELLS = 13,       /* backward-data of a layer with stride 2 x 2 and a filter of at least 2 x 2: tiles of 128
                                            rows x 64 cells of 2 x 2 pixels; a block runs the four pixel classes in turn and
                                            writes whole cells */
    INT8T_VARIANT_MAX_ENUM = 0x7fffffff
} int8t_variant;
#define INT8T_VARIANT_COUNT 14
/* 1 when `variant` can run pass `op` (INT8T_OP_CONV_*) of the layer, else 0 (also on a bad descriptor). */
int int8t_conv_variant_ok(int8t_op op, const int8t_conv_desc *desc, int8t_variant variant);
/* INT8T_ERR_ARG when the variant cannot run that pass of that layer; then nothing changes. */
int8t_status int8t_conv_select_variant(int8t_op op, const int8t_conv_desc *desc, int8t_variant variant);
int8t_variant int8t_conv_selected_variant(int8t_op op, const int8t_conv_desc *desc);

/*
 * Kernel timing (measurement aid, not part of the method).  Between int8t_profile_start and
 * int8t_profile_stop every launch of the selected kernel carries a pair of HIP events that take
 * the dispatch's own start and end time stamps on the launch stream.  A timed dispatch costs a few
 * microseconds of idle time before and after it; int8t_profile_start_sampled(kernel, every) times
 * only every `every`-th launch (every >= 1) of each selected kernel, so that a measured loop is
 * disturbed correspondingly less.
 *   kernel   host string: the kernel's name ("dsgc_sweep_kernel", "absmax_kernel",
 *            "absmax_batch_kernel", "quantize_batch_kernel", "quantize_act_kernel", "quantize_planar_kernel", "quantize_wgt_kernel",
 *            "deviation_finish_kernel", "igemm_kernel", "igemm_dma_kernel", "igemm_fused_kernel", "igemm_reduce_kernel",
 *            "band_kernel", "band_reg_kernel", "wgrad_kernel", "wgrad_lines_kernel", "wgrad_reduce_kernel", "s2d_repack_kernel",
 *            "s2d_weights_kernel", "dw_conv_kernel" (every depthwise forward / backward-data variant),
 *            "dw_wgrad_kernel" (every depthwise backward-weight variant), "dw_wgrad_reduce_kernel");
 *            NULL or "" selects every kernel.
 *            An unknown name returns INT8T_ERR_ARG and leaves timing off.
 * int8t_profile_stop waits for the recorded events, writes one entry per kernel that was
 * launched (name: static string owned by the library; launches; summed duration in ms) into
 * out[0..capacity), stores the number of kernels seen in *count (which may exceed capacity) and
 * switches timing off.  Host pointers throughout.  Not thread-safe; event objects are created
 * while timing is on, so keep it off under stream capture.
 */
typedef struct int8t_kernel_time {
    const char *name;
    int launches;
    double total_ms;
} int8t_kernel_time;
int8t_status int8t_profile_start(const char *kernel);
int8t_status int8t_profile_start_sampled(const char *kernel, int every);
int8t_status int8t_profile_stop(int8t_kernel_time *out, int capacity, int *count);

/*
 * Measurement aid: what the int8 matrix cores of the current GPU sustain.  Runs, on every compute
 * unit, eight waves of independent 32x32x32 int8 MFMAs (the wave tile of the wide convolution kernels)
 * for `iters` iterations of 16 MFMAs per wave, with operand bytes all zero (random_operands == 0) or
 * pseudo-random, held in registers (lds_reads == 0) or re-read from LDS before every eight MFMAs as
 * an implicit GEMM does.  Synchronises with the host.
 *   tops_out   host, out: int8 operations per second / 1e12 over the kernel's duration
 *   ghz_out    host, out: the shader clock the loop ran at (shader-clock counter against the constant
 *              100 MHz counter, both read inside the kernel)
 *   ws_dev     64 bytes of device scratch, 8-byte aligned
 * The published peak (5.0 POP/s at 2.4 GHz) is what zero operands reach; with random operands the
 * power limit lowers the clock, and that figure is the ceiling a convolution on real codes has.
 */
int8t_status int8t_profile_mfma_ceiling(int random_operands, int lds_reads, int iters,
                                        double *tops_out, double *ghz_out, void *ws_dev, void *stream);

/* Eq.7 on the host: max(exp(-alpha * d_c), beta).  The paper uses alpha = 20, beta = 0.1. */
double int8t_dclr_scale(double d_c, double alpha, double beta);

#ifdef __cplusplus
}
#endif
#endif /* INT8T_H */
