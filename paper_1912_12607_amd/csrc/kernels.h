// Internal launch interface between the C-ABI layer (api.hip) and the kernel files.
// Every launcher enqueues on `st` and returns the hipError_t of its last launch.
#pragma once
#include "profile.h"
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace int8t {

// Raises a kernel's dynamic-LDS limit (the default is 64 KB) the first time it is launched on a
// device; `done` is the call site's own bit mask of the devices already served.
inline hipError_t raise_dynamic_lds(const void* fn, int bytes, std::atomic<unsigned long long>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}


constexpr int kMaxPartials = 1024;   // per-block partial results of an absmax pass
constexpr int kAbsmaxPartials = 256;  // ... of which an absmax pass writes at most this many (its block count)

// Partial sums of Eq.6 left by one block: A = sum g*q, G = sum g^2, B = sum q^2.
struct DevPartial {
    double A;
    double G;
    unsigned long long B;
};

// ---- quantize.hip ---------------------------------------------------------------------------
// max|x| per block -> part[0..nparts); returns the number of partials through *nparts.
// sumsq: nullptr, or kMaxPartials doubles that receive per-block sums of squares; then the pass
// also clears the nzero 64-bit words at zero (the clip search's accumulators and ticket)
hipError_t launch_absmax(const float* x, size_t n, float* part, int* nparts, hipStream_t st, double* sumsq = nullptr,
                         unsigned long long* zero = nullptr, int nzero = 0);

struct QuantArgs {
    const float* x;
    int d0, d1, d2, d3;          // logical dims: N,C,H,W or K,Cg,R,S
    const float* clip;           // device scalar or nullptr (then absmax partials are reduced)
    const float* absmax_part;
    int nparts;
    int stochastic;
    uint64_t seed;
    int8_t* q;
    float* scale;
    DevPartial* devpart;         // nullptr: no deviation
};
// several tensors per launch (round-to-nearest, no deviation output)
constexpr int kMaxBatch = 8;
struct AbsmaxBatchItem {
    const float* x;
    size_t n;
    float* part;                 // this tensor's partials
    int block0, nblocks;         // its block range inside the launch (nblocks = 0: clip supplied)
    // the tensor of a clip search (at most one, the last item): its blocks also leave the sums of squares and clear
    // the search's accumulators, as absmax_kernel<true> does
    double* sumsq;
    unsigned long long* zero;
    int nzero;
};
struct AbsmaxBatch {
    int count;
    AbsmaxBatchItem it[kMaxBatch + 1];
};
struct QuantBatchItem {
    const float* x;
    int d0, d1, d2, d3;
    const float* clip;
    const float* absmax_part;
    int nparts;
    int8_t* q;
    float* scale;
    int kind;                    // 0 activations, 1 weights, 2 planar
    int block0, gx, gy, gz;      // its block range and virtual grid inside the launch
    int stoch;                   // Eq.3 instead of Eq.1
    uint32_t seed_lo, seed_hi;   // seed_key_x(seed), seed_key_a(seed): the draw's two keys
};
struct QuantBatch {
    int count;
    QuantBatchItem it[kMaxBatch];
};
int absmax_blocks(size_t n);
void quant_grid(int kind, const int d[4], int* gx, int* gy, int* gz);
hipError_t launch_absmax_batch(const AbsmaxBatch& b, int total_blocks, hipStream_t st);
hipError_t launch_quantize_batch(const QuantBatch& b, int total_blocks, hipStream_t st);
int quant_blocks_act(int N, int Cp, int HW);
int quant_blocks_planar(size_t n);
int quant_blocks_wgt(int K, int Cg, int R, int S);
hipError_t launch_quantize_act(const QuantArgs& a, hipStream_t st);
hipError_t launch_quantize_planar(const QuantArgs& a, hipStream_t st);
hipError_t launch_quantize_wgt(const QuantArgs& a, hipStream_t st);
hipError_t launch_deviation_finish(const DevPartial* part, int nparts, double* dev_out, hipStream_t st);

// ---- dsgc.hip -------------------------------------------------------------------------------
struct DsgcWs {
    float* absmax_part;          // kMaxPartials floats
    unsigned long long* acc;     // dsgc_acc_words() 64-bit accumulators, then the ticket word; cleared by the absmax pass
    unsigned int* ticket;
    double* partG;               // [kMaxPartials]: per-block sums of g^2 from the absmax pass
};
int dsgc_blocks(size_t n);
// 64-bit accumulator words of the sweep: 32 sets x 64 candidates x {sum H*m, sum L*m, sum m^2}
constexpr size_t kDsgcAccWords = (size_t)32 * 64 * 3;
size_t dsgc_acc_words();             // == kDsgcAccWords
hipError_t launch_dsgc(const float* g, size_t n, const float* ratios, int n_cand, int stochastic,
                       uint64_t seed, const DsgcWs& ws, int nparts_absmax, float* clip_out,
                       double* dev_out, double* dev_all_out, hipStream_t st);

// ---- conv_igemm.hip (dense forward and backward-data) -----------------------------------------
struct IgemmArgs {
    const int8_t* act;           // NHWC codes, channel pitch Ca
    const int8_t* wgt;           // [rows][R][S][Ca]
    const float* sa;
    const float* sb;
    float* out;                  // [N][rows][OH*OW]
    int32_t* acc;                // nullable, same order
    int N, rows, Ca;             // Ca: padded reduction channels (multiple of 16)
    int IH, IW, OH, OW, R, S;
    int stride_h, stride_w, pad_h, pad_w;
    int dgrad;                   // 0: ih = oh*stride + r - pad;  1: ih = (oh + pad - r)/stride
    int C;                       // forward: channels in use (<= Ca); lets the launch recognise a layer for s2d.hip
    int8_t* s2d;                 // nullable scratch of igemm_s2d_bytes() bytes for the rewritten codes
    int cell;                    // filled by launch_igemm(): 0, or 1 + the only residue class that has taps (cell form, conv_igemm.hip)
    int cls_h, cls_w;            // filled by launch_igemm(): strides of the residue classes a strided backward-data pass splits its pixels into (1 = not split)
    int32_t* partial;            // nullable scratch [ksplit][N][rows][OH*OW] of a split reduction
    size_t partial_bytes;
    int ksplit;                  // filled by launch_igemm(): blocks per output tile along the reduction
    int variant;                 // ConvVariant: VAR_AUTO, or the kernel the caller selected for this layer
    // Quantization fused into the forward pass of a 1 x 1, stride-1, unpadded layer (launch_igemm_fused):
    const float* xf;             // fp32 activations N,C,H,W (act is not read)
    const float* xclip;          // clip value of a, or nullptr: max|a| from xabs_part[0..xabs_nparts)
    const float* xabs_part;
    int xabs_nparts;
    int8_t* xq_out;              // nullable: the codes of a (N,H,W,Ca), written by the first row tile
    float* sx_out;               // the scale of a
};
// Kernel variants of the dense passes (values of INT8T_VARIANT_* in include/int8t.h).
enum ConvVariant : int {
    VAR_AUTO = 0,
    VAR_BAND = 1,          // forward / backward-data: filter bank resident on chip (conv_band.hip)
    VAR_TILE = 2,          // 64/128 x 128 tiles through registers, reduction whole
    VAR_TILE_SPLIT = 3,    // ... reduction split over several blocks per tile
    VAR_WIDE128 = 4,       // 128 x 256 tiles, operands straight into an LDS ring of 3 stages
    VAR_WIDE256 = 5,       // 256 x 256 tiles, ring of 2 stages of 128 reduction bytes
    VAR_WGRAD_FEWER = 6,   // backward-weight: half the reduction shares of the cost model's choice
    VAR_WGRAD_MORE = 7,    // backward-weight: twice as many
    VAR_WGRAD_IMAGES = 8,  // backward-weight: operands of 16 images per pixel, transposed in registers (conv_wgrad.hip)
    VAR_WGRAD_LINES = 9,   // backward-weight: operands of 32 image lines per position, transposing LDS reads (conv_wgrad_lines.hip)
    VAR_WIDE_SQ128 = 10,   // forward / backward-data: 128 x 128 tiles, ring of 3 stages, three blocks per compute unit
    VAR_WIDE_SQ128_DEEP = 11,   // ... 2 stages of 128 reduction bytes, two blocks per compute unit
    VAR_WIDE_128X64 = 12,       // ... 128 x 64 tiles: layers with few columns
    VAR_WIDE_CELLS = 13,        // backward-data under stride 2 x 2: 128 rows x 64 cells of 2 x 2 pixels, the four pixel classes in one block
    VAR_COUNT
};
int igemm_ksplit(const IgemmArgs& a);   // largest split a launch of this layer may use (1 = none): sizes the scratch
// whether `variant` can run this layer (VAR_AUTO always can); resolved = the variant VAR_AUTO stands for
bool igemm_variant_ok(const IgemmArgs& a, int variant);
int igemm_auto_variant(const IgemmArgs& a, bool allow_split = true);   // allow_split: the caller's scratch holds the partial sums of a split reduction
// Forward pass of a layer s2d.hip covers: rewrites the geometry and returns the scratch bytes of the
// rewritten input and filter codes (0: does not apply, the geometry is left alone).
size_t igemm_s2d(IgemmArgs* a);
hipError_t launch_igemm(const IgemmArgs& a, hipStream_t st);
// forward pass that quantizes fp32 activations in its load path; 1 x 1 filter, stride 1, no padding
hipError_t launch_igemm_fused(const IgemmArgs& a, hipStream_t st);
// conv_band.hip: LDS-resident variant for small filter banks; false = shape not covered
// (dry_run: only say whether the shape is covered, launch nothing)
bool launch_band(const IgemmArgs& a, hipStream_t st, hipError_t* err, bool dry_run = false);

// ---- s2d.hip ----------------------------------------------------------------------------------
// A stride-2 layer with at most 4 input channels (the stem of an image network) as the stride-1
// layer on the space-to-depth image: pixel (h', w') holds the 2 x 2 block of pixels (2h' + dy,
// 2w' + dx) as channel (2 dy + dx) * C + c.  Input row 2p + r - pad = 2 (p + r' - ph) + dy with
// ph = ceil(pad / 2) and r = 2 r' + dy - eh, eh = 2 ph - pad: the R x S filter becomes a
// ceil((R+eh)/2) x ceil((S+ew)/2) one whose taps outside the original filter are zero.  The 16-byte
// pixel granule then carries 4 C channels instead of C, and the taps shrink fourfold.  The output
// pixels stay the same.  An odd image gets a last block row / column whose missing pixels are zero, as
// the padding around the image is.
struct S2dGeo {
    int ph, pw, eh, ew, R2, S2;
};
inline bool s2d_applies(int C, int stride_h, int stride_w) { return stride_h == 2 && stride_w == 2 && C <= 4; }
inline S2dGeo s2d_geometry(int R, int S, int pad_h, int pad_w) {
    S2dGeo g;
    g.ph = (pad_h + 1) / 2;
    g.pw = (pad_w + 1) / 2;
    g.eh = 2 * g.ph - pad_h;
    g.ew = 2 * g.pw - pad_w;
    g.R2 = (R + g.eh + 1) / 2;
    g.S2 = (S + g.ew + 1) / 2;
    return g;
}
// input codes [N][H][W][16] -> [N][ceil(H/2)][ceil(W/2)][16]
hipError_t launch_s2d_repack(const int8_t* x, int8_t* xs, int N, int H, int W, int C, hipStream_t st);
// filter codes [K][R][S][16] -> [K][R2][S2][16]
hipError_t launch_s2d_weights(const int8_t* w, int8_t* ws, int K, int R, int S, int C, const S2dGeo& g, hipStream_t st);

// ---- conv_wgrad.hip (dense backward-weight) ---------------------------------------------------
struct WgradArgs {
    const int8_t* x;             // NHWC codes of a, pitch Cp
    const int8_t* dy;            // NHWC codes of g_z, pitch Kp
    const float* sa;
    const float* sb;
    float* dw;                   // [K][C][R][S]
    int32_t* acc;                // nullable
    int32_t* partial;            // scratch [splits][K][R*S*Cp]
    int N, C, Cp, H, W, K, Kp, P, Q, R, S;
    int stride_h, stride_w, pad_h, pad_w;
    // filled by wgrad_plan():
    int TB, CS;                  // taps per block, 32-channel slabs per wave
    int pk;                      // 1: a tensor of 16 channels, four taps per block packed side by side into the 64 columns
    int BP, BQ, ntp, ntq;        // output-pixel tile and tiles per image
    int ngrp, chunks, splits;    // groups of 16 images, reduction chunks, split-K factor
    int ktiles, ctiles, tapgroups;
    int xt_slots;                // 16-byte granules of the staged input window
    size_t lds_bytes;
    // filled by wgrad_s2d() when it rewrites the geometry above into the space-to-depth form:
    int s2d;                     // 1: C, Cp, H, W, R, S, strides and pads describe the rewritten problem
    int oC, oR, oS, oH, oW, eh, ew;   // the layer's own channels, filter and image; tap r = 2 r' + dy - eh, s = 2 s' + dx - ew
    int8_t* xs;                  // scratch: the input codes in space-to-depth form, [N][H][W][16]
    int variant;                 // VAR_AUTO or a VAR_WGRAD_*: set before wgrad_plan()
    int lines;                   // filled by wgrad_plan(): 1 = wgrad_lines_kernel runs (TB = taps along the line)
    int xgk, xgc;                // ... and its patches of output tiles per XCD: xgk x xgc = 8, or 0 0: tiles dealt by share
};
// Rewrites the geometry into the space-to-depth form (s2d.hip) when it applies.  Returns the bytes of
// the rewritten input codes (0: does not apply, the geometry is left alone).  Call before wgrad_plan().
size_t wgrad_s2d(WgradArgs* a);
void wgrad_plan(WgradArgs* a);   // needs the geometry fields above the first comment
hipError_t launch_wgrad(const WgradArgs& a, hipStream_t st);
// conv_wgrad_lines.hip: the kernel for stride-1 filters with 3 or 7 taps along an image axis
bool wgrad_lines_applies(const WgradArgs& a);    // geometry as wgrad_plan() takes it (after wgrad_s2d())
// lines are image rows and the taps of a block run along W (else: columns, along H)
__host__ __device__ inline bool wgrad_lines_along_w(int R, int S) { return S > 1 || R == 1; }
void wgrad_plan_lines(WgradArgs* a);
hipError_t launch_wgrad_lines(const WgradArgs& a, hipStream_t st);
// which kernel VAR_AUTO stands for: true = wgrad_lines_kernel
bool wgrad_auto_lines(const WgradArgs& a);
// Share z runs on XCD z mod 8 with all its output tiles (they read the same lines of both tensors, and every XCD fills
// its own L2) when the shares go round the XCDs evenly enough: the grid holds a multiple of 8 shares, the extra ones
// exit at once, and the XCDs with one share more take 8 / splits longer (at most 1/7 here).  Without it the tiles of a
// share land on all 8 XCDs and each L2 fetches the share's lines again (256 x 128 -> 128 3x3 at 28 x 28: 68 -> 47 us).
__host__ __device__ inline bool wgrad_xcd_mapping(int splits) {
    return splits >= 8 && (((splits + 7) & ~7) - splits) * 7 <= splits;
}

// ---- conv_dw.hip (depthwise, planar codes) ----------------------------------------------------
struct DwArgs {
    const int8_t* a;             // planar codes, input of the gather ([N][C][IH][IW])
    const int8_t* b;             // fwd/bwd-data: weights [C][R][S]; bwd-weight: dy codes [N][C][P][Q]
    const float* sa;
    const float* sb;
    float* out;
    int32_t* acc;                // nullable
    int32_t* partial;            // bwd-weight scratch [chunks][C*R*S]
    int chunks;                  // bwd-weight: shares of the batch, dw_wgrad_shape()
    int threads;                 // bwd-weight: block size, dw_wgrad_shape()
    int cg;                      // bwd-weight: consecutive channels per block (1: a block per channel), dw_wgrad_shape()
    int N, C, IH, IW, OH, OW, R, S;
    int stride_h, stride_w, pad_h, pad_w;
    int dgrad;
};
int dw_threads(int OH, int OW, bool quads);       // block size by plane size (quads: four results per task)
int dw_wgrad_threads(int P, int Q, int R, int S, int stride_h, int stride_w);
int dw_wgrad_chunks(int N, int C, int threads);
// launch shape of the depthwise backward-weight pass (its scratch is chunks * C * R * S int32)
void dw_wgrad_shape(int N, int C, int IH, int IW, int P, int Q, int R, int S, int stride_h, int stride_w,
                    int* threads, int* chunks, int* cg);
hipError_t launch_dw_conv(const DwArgs& a, hipStream_t st);
hipError_t launch_dw_wgrad(const DwArgs& a, hipStream_t st);

}  // namespace int8t
