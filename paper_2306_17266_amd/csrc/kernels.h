// Device kernels of the SubNet forward pass and their launchers (gfx950).
//
// Layouts
//   activations   [B][H][W][C]  channels fastest, C = active channels of the SubNet (compact)
//   dense weights [tap][channel group of 8][filter (padded to 16)][8 channels]
//                 so the slice (K' filters, C' channels) of a SubNet is, for every tap and channel
//                 group below C'/8, the contiguous prefix of K' * 8 elements; a 16-filter x 32-channel
//                 matrix-core operand is four 256-byte runs
//   depthwise     [tap in ring order][channel]: the 9 taps of the centre 3x3 first, then the 16 of
//                 the 5x5 ring, then the 24 of the 7x7 ring, so a centred k x k crop is the prefix
//                 of k*k taps
//   scale/shift   float32 prefixes of length K'
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace sushi {

struct ConvArgs {
    const void *x;       // input activations
    void *y;             // output activations
    const void *res;     // optional residual, same shape as y
    const void *w;       // packed weights of the layer
    const float *scale;  // may be null (= 1)
    const float *shift;  // shift or bias
    int B, H, W, C;      // input
    int P, Q, K;         // output
    int R, stride, pad;  // taps per side of the active kernel
    int Rmax;            // taps per side of the stored kernel (depthwise crops)
    int Kpad, CG;        // packed layout: padded filters, stored channel groups
    int act;             // sushi_act; applied after the residual add
    int hsigmoid;        // replace act by min(max(v+3,0),6)/6
    int out_f32;         // store float32 regardless of the activation type
    int in_f32;          // bf16 mode: the input is a float32 vector per image (pooled features, squeeze-excite and
                         // head vectors); the kernels split it into two bf16 terms (value = hi + lo) on the fly
};

// What an int8 layer needs beyond ConvArgs / PoolArgs (int8.hip).  Weights are then
// [tap][channel group of 16][filter (padded to 16)][16] and ConvArgs::CG counts the stored groups of 16.
struct QuantArgs {
    const int32_t *qmult;   // per filter: requantisation multiplier (classifier: bit pattern of a float32 factor)
    const int32_t *qshift;  // per filter: rounding right shift
    const int32_t *qbias;   // per filter: added to the accumulator
    const int32_t *wsum;    // per filter: sum of the active slice's weights over taps and channels (zero-point term)
    int zx, zy;             // zero points of the input and the output tensor (pooling: zx of the pooled map)
    int m_res, sh_res, z_res;  // residual: multiplier, shift, zero point
    int pool_hw;            // classifier: pixels the pooling before it summed over
};

struct PoolArgs {
    const void *x;
    void *y;
    const float *gate;  // OP_GATE: [B][C] multipliers
    int B, H, W, C, P, Q;
    int out_f32;        // OP_GAP in bf16 mode: store the averages as float32
};

// Kernel families, for per-kernel accounting.
enum KernelClass {
    KC_CONV_DIRECT = 0,   // conv_direct_kernel
    KC_CONV_MFMA = 1,     // conv_mfma_kernel (whole-reduction waves)
    KC_CONV_SPLITK = 2,   // conv_mfma_splitk_kernel
    KC_DWCONV = 3,
    KC_MAXPOOL = 4,
    KC_GAP = 5,
    KC_GATE = 6,
    KC_STREAM = 7,  // sushi_stream_kernel (one launch per query)
    KC_TEAM = 8,    // sushi_team_kernel (persistent; one launch serves many queries)
    KC_CONV_PATCH = 9,  // conv_patch_kernel (large pixel counts; the input patch of a tile staged in LDS)
    KC_CONV_I8 = 10,    // conv_i8_kernel / conv_i8_direct_kernel (int8 mode)
    KC_I8_OTHER = 11,   // int8 mode: max-pool, pooled sums, classifier
    KC_COUNT = 12
};
const char *kernel_class_name(int kc);

// Every launcher returns hipSuccess or the launch error.  bf16 = activations and weights are bf16.
// launch_conv reports the kernel family it picked in *kc (may be null).
// patch_min_pixels: dense 1x1 / 3x3 layers with at least that many output pixels (B * P * Q) go to the patch
// kernel (conv_patch.hip) where it covers the shape; 0 = never.
hipError_t launch_conv(const ConvArgs &a, bool bf16, hipStream_t s, int *kc, long patch_min_pixels);  // dense conv and FC

// Dense 1x1 (stride 1) and 3x3 (stride 1 or 2) convolution, bf16, C and K multiples of 8, tensors below 2 GiB: the
// patch kernel (conv_patch.hip).  Returns hipErrorNotSupported (nothing launched) for any other case.
hipError_t launch_conv_patch(const ConvArgs &a, hipStream_t s);
hipError_t launch_dwconv(const ConvArgs &a, bool bf16, hipStream_t s);
hipError_t launch_maxpool(const PoolArgs &a, bool bf16, hipStream_t s);   // 3x3 stride 2 pad 1
hipError_t launch_gap(const PoolArgs &a, bool bf16, hipStream_t s);       // [B][H][W][C] -> [B][C]
hipError_t launch_gate(const PoolArgs &a, bool bf16, hipStream_t s);      // y = x * gate[b][c]

// Depthwise k x k, k in {3, 5, 7}, stride 1 or 2, bf16, tensors below 2 GiB: the row-strip kernel (dwconv.hip).
// Returns hipErrorNotSupported (nothing launched) for any other case.
hipError_t launch_dwconv_rows(const ConvArgs &a, hipStream_t s);

// int8 mode (int8.hip): dense conv 1x1 / 3x3 on the int8 matrix cores (3 input channels: vector ALUs) with integer
// requantisation, 3x3/2 max-pool on codes, exact int32 pooled sums, int64 classifier with float32 logits.
hipError_t launch_conv_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s, long patch_min_pixels);
hipError_t launch_conv_patch_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s);  // conv_patch.hip
hipError_t launch_fc_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s);
hipError_t launch_maxpool_i8(const PoolArgs &a, hipStream_t s);
hipError_t launch_gap_i8(const PoolArgs &a, const QuantArgs &q, hipStream_t s);

// Streams `bytes` of `buf` through the caches (reads every 16-byte word once; `sink` receives one word that
// depends on all of them, so the reads cannot be dropped).  A measurement aid: see SUSHI_OPT_COLD_SWEEP_MIB.
hipError_t launch_cold_sweep(const void *buf, size_t bytes, void *sink, hipStream_t s);

// The library's static scratch buffer on the current device: STATIC_SCRATCH_BYTES of device memory that
// belong to the loaded code object (no allocation), for sushi_infer_static.  The address is looked up once
// per device, with that device current.
constexpr size_t STATIC_SCRATCH_BYTES = 16u << 20;
hipError_t static_scratch(int device, void **ptr);

// Ring order of depthwise taps: tap t of a 7x7 kernel sits at row/col offset (dr, ds) from the centre.
void dw_tap_offsets(int t, int *dr, int *ds);
hipError_t upload_tap_table();

}  // namespace sushi
