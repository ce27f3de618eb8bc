// int8 path (the paper's own precision: int8 weights, activations and zero points, int32 scale; Section 5.1
// footnote, Section 4.2.2) for the per-layer launch mode: dense convolution on the int8 matrix cores with integer
// requantisation, max-pool on codes, exact pooled sums, int64 classifier.  Every step is integer arithmetic with
// one right answer (see include/sushi.h: sushi_load_supernet_int8), so results are compared bit for bit.
//
// Layouts: activations [B][H][W][C] int8, C a multiple of 8 (3 for the network input); weights
// [tap][channel group of 16][filter, padded to 16][16 channels] int8, channels beyond the layer's width zero.
//
// conv_i8_kernel: v_mfma_i32_16x16x64_i8; filters are the rows, pixels the columns.  A lane supplies, for its
// filter (or pixel) lane & 15, the 16 channels of channel group lane >> 4 of the current 64-channel step: one
// 16-byte load per operand and step, straight from memory (which channel a lane holds does not matter as long as
// both operands agree: the instruction sums over all 64).  Zero points: the matrix cores multiply the raw codes,
// sum w * (x - z_x) = sum w * x - z_x * sum w.  Cells outside the image are filled with the code z_x (the real
// value 0), channels beyond the SubNet's width with the code 0, so the correction is z_x times the weight sum
// over the ACTIVE channels and all taps, which the host has as a prefix table per 8 channels.
#include "kernels.h"
#include "device_common.h"

#include <algorithm>

namespace sushi {

typedef __attribute__((ext_vector_type(4))) int i32x4_t;
constexpr int I8_OOB = 0x7FFFFFF0;

// (v + 2^(s-1)) >> s on 64-bit integers, arithmetic shift; 1 <= s <= 62
__device__ __forceinline__ long long rr64(long long v, int s) { return (v + (1ll << (s - 1))) >> s; }

// Requantises four accumulators of consecutive filters f .. f+3 of pixel m and stores four codes.
__device__ __forceinline__ void store_codes(const ConvArgs &a, const QuantArgs &q, const int acc[4], int f, long m) {
    if (f >= a.K) return;
    const int lo = a.act == 1 ? q.zy : -128;
    unsigned packed = 0;
    unsigned res = 0;
    if (a.res) res = *reinterpret_cast<const unsigned *>(static_cast<const int8_t *>(a.res) + m * a.K + f);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        long long t = rr64((long long)(acc[i] + q.qbias[f + i]) * (long long)q.qmult[f + i], q.qshift[f + i]);
        if (a.res) t += rr64((long long)((int)(int8_t)(res >> (8 * i)) - q.z_res) * (long long)q.m_res, q.sh_res);
        t += q.zy;
        const int v = (int)(t < lo ? lo : t > 127 ? 127 : t);
        packed |= (unsigned)(v & 0xFF) << (8 * i);
    }
    *reinterpret_cast<unsigned *>(static_cast<int8_t *>(a.y) + m * a.K + f) = packed;  // K is a multiple of 4
}

// One wave: FT x PT tiles of 16 filters x 16 pixels over the whole reduction; a workgroup is four waves on
// neighbouring pixel groups.
template <int FT, int PT>
__global__ __launch_bounds__(256) void conv_i8_kernel(ConvArgs a, QuantArgs q) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const long M = (long)a.B * a.P * a.Q;
    const long n_pgroups = (M + 16 * PT - 1) / (16 * PT);
    const long pg = (long)blockIdx.x * 4 + wave;
    if (pg >= n_pgroups) return;
    const int f0 = blockIdx.y * FT * 16;
    const long m0 = pg * PT * 16;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, (int)((long)a.B * a.H * a.W * a.C), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.w), 0, (int)((long)a.R * a.R * a.CG * a.Kpad * 16), 0x00020000);
    int pn[PT], ph[PT], pw[PT];
    bool pv[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        const long m = m0 + pt * 16 + l16;
        pv[pt] = m < M;
        const long mm = pv[pt] ? m : 0;
        const int qq = (int)(mm % a.Q), pp = (int)((mm / a.Q) % a.P);
        pn[pt] = (int)(mm / ((long)a.Q * a.P));
        ph[pt] = pp * a.stride - a.pad;
        pw[pt] = qq * a.stride - a.pad;
    }
    int fw[FT];
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) fw[ft] = (f0 + ft * 16 + l16 < a.Kpad) ? (f0 + ft * 16 + l16) * 16 : -1;
    const unsigned zfill = (unsigned)(q.zx & 0xFF) * 0x01010101u;
    i32x4_t acc[FT][PT];
#pragma unroll
    for (int ft = 0; ft < FT; ++ft)
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) acc[ft][pt] = i32x4_t{0, 0, 0, 0};
    const int csteps = (a.C + 63) >> 6;
    for (int tap = 0; tap < a.R * a.R; ++tap) {
        const int dr = tap / a.R, ds = tap - dr * a.R;
        for (int cs = 0; cs < csteps; ++cs) {
            const int c0 = cs * 64 + kg * 16;       // this lane's 16 channels
            const int cg = c0 >> 4;
            i32x4_t fa[FT], fb[PT];
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
                fa[ft] = __builtin_bit_cast(i32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                    rw, fw[ft] >= 0 && cg < a.CG ? ((tap * a.CG + cg) * a.Kpad) * 16 + fw[ft] : I8_OOB, 0, 0));
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                const int h = ph[pt] + dr, v = pw[pt] + ds;
                const bool inside = pv[pt] && h >= 0 && h < a.H && v >= 0 && v < a.W;
                const int off = inside && c0 < a.C ? ((pn[pt] * a.H + h) * a.W + v) * a.C + c0 : I8_OOB;
                i32x4_t b = __builtin_bit_cast(i32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 0));
                if (c0 + 8 >= a.C) b[2] = 0, b[3] = 0;     // the cell's upper half lies beyond the active channels
                if (!inside && c0 < a.C) {                   // a cell of the frame: the code of the real value 0
                    b[0] = (int)zfill, b[1] = (int)zfill;
                    if (c0 + 8 < a.C) b[2] = (int)zfill, b[3] = (int)zfill;
                }
                fb[pt] = b;
            }
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
                    acc[ft][pt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[ft], fb[pt], acc[ft][pt], 0, 0, 0);
        }
    }
    // the lane holds pixel l16 and filters 4 kg .. 4 kg + 3 of every tile
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) {
        const int f = f0 + ft * 16 + kg * 4;
        int corr[4] = {0, 0, 0, 0};
        if (f < a.K && q.zx != 0)
#pragma unroll
            for (int i = 0; i < 4; ++i) corr[i] = q.zx * q.wsum[f + i];
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            const long m = m0 + pt * 16 + l16;
            if (m >= M) continue;
            const int v[4] = {acc[ft][pt][0] - corr[0], acc[ft][pt][1] - corr[1], acc[ft][pt][2] - corr[2], acc[ft][pt][3] - corr[3]};
            store_codes(a, q, v, f, m);
        }
    }
}

// Fewer than 8 input channels (the network input): one thread per output pixel and four filters, plain integers.
__global__ __launch_bounds__(256) void conv_i8_direct_kernel(ConvArgs a, QuantArgs q) {
    const int groups = a.K >> 2;
    const long total = (long)a.B * a.P * a.Q * groups;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int fg = (int)(idx % groups);
    const long m = idx / groups;
    const int qq = (int)(m % a.Q), pp = (int)((m / a.Q) % a.P), n = (int)(m / ((long)a.Q * a.P));
    const int8_t *x = static_cast<const int8_t *>(a.x);
    const int8_t *w = static_cast<const int8_t *>(a.w);
    int acc[4] = {0, 0, 0, 0};
    for (int tap = 0; tap < a.R * a.R; ++tap) {
        const int h = pp * a.stride - a.pad + tap / a.R, v = qq * a.stride - a.pad + tap % a.R;
        if (h < 0 || h >= a.H || v < 0 || v >= a.W) continue;
        const int8_t *xp = x + (((long)n * a.H + h) * a.W + v) * a.C;
        for (int ch = 0; ch < a.C; ++ch) {
            const int xv = (int)xp[ch] - q.zx;
            const int8_t *wp = w + (((long)tap * a.CG + (ch >> 4)) * a.Kpad + fg * 4) * 16 + (ch & 15);
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] += xv * (int)wp[i * 16];
        }
    }
    store_codes(a, q, acc, fg * 4, m);
}

__global__ __launch_bounds__(256) void maxpool_i8_kernel(PoolArgs a) {
    const int cgs = a.C >> 3;
    const long total = (long)a.B * a.P * a.Q * cgs;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cg = (int)(idx % cgs);
    const long m = idx / cgs;
    const int qq = (int)(m % a.Q), pp = (int)((m / a.Q) % a.P), n = (int)(m / ((long)a.Q * a.P));
    const int8_t *x = static_cast<const int8_t *>(a.x);
    int best[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) best[j] = -128;
    for (int r = 0; r < 3; ++r) {
        const int h = pp * 2 - 1 + r;
        if (h < 0 || h >= a.H) continue;
        for (int s = 0; s < 3; ++s) {
            const int v = qq * 2 - 1 + s;
            if (v < 0 || v >= a.W) continue;
            const uint2 q = *reinterpret_cast<const uint2 *>(x + (((long)n * a.H + h) * a.W + v) * a.C + cg * 8);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = (int)(int8_t)((j < 4 ? q.x : q.y) >> (8 * (j & 3)));
                best[j] = c > best[j] ? c : best[j];
            }
        }
    }
    uint2 o = make_uint2(0, 0);
#pragma unroll
    for (int j = 0; j < 8; ++j) (j < 4 ? o.x : o.y) |= (unsigned)(best[j] & 0xFF) << (8 * (j & 3));
    *reinterpret_cast<uint2 *>(static_cast<int8_t *>(a.y) + m * a.C + cg * 8) = o;
}

// Exact sums of (code - z_x) over H x W: one thread per (image, channel); int32 out.
__global__ __launch_bounds__(256) void gap_i8_kernel(PoolArgs a, QuantArgs q) {
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)a.B * a.C) return;
    const int ch = (int)(idx % a.C), n = (int)(idx / a.C);
    const int8_t *x = static_cast<const int8_t *>(a.x) + (long)n * a.H * a.W * a.C + ch;
    int sum = 0;
    for (int p = 0; p < a.H * a.W; ++p) sum += (int)x[(long)p * a.C] - q.zx;
    static_cast<int *>(a.y)[idx] = sum;
}

// Classifier on the pooled sums: one thread per (image, class); int64 accumulator, float32 logit.
__global__ __launch_bounds__(256) void fc_i8_kernel(ConvArgs a, QuantArgs q) {
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)a.B * a.K) return;
    const int k = (int)(idx % a.K), n = (int)(idx / a.K);
    const int *sums = static_cast<const int *>(a.x) + (long)n * a.C;
    const int8_t *w = static_cast<const int8_t *>(a.w);
    long long acc = (long long)q.pool_hw * (long long)q.qbias[k];
    for (int ch = 0; ch < a.C; ++ch)
        acc += (long long)sums[ch] * (long long)w[(((long)(ch >> 4)) * a.Kpad + k) * 16 + (ch & 15)];
    const double base = (double)__int_as_float(q.qmult[k]);
    static_cast<float *>(a.y)[idx] = (float)((double)acc * (base / (double)q.pool_hw));
}

// ------------------------------------------------------------------ launchers

static inline unsigned i8_blocks(long total) { return (unsigned)((total + 255) / 256); }

template <int FT, int PT>
static hipError_t launch_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s) {
    const long M = (long)a.B * a.P * a.Q;
    const long n_pgroups = (M + 16 * PT - 1) / (16 * PT);
    const int n_fgroups = (a.K + 16 * FT - 1) / (16 * FT);
    hipLaunchKernelGGL((conv_i8_kernel<FT, PT>), dim3((unsigned)((n_pgroups + 3) / 4), n_fgroups), dim3(256), 0, s, a, q);
    return hipGetLastError();
}

hipError_t launch_conv_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s) {
    const long M = (long)a.B * a.P * a.Q;
    if ((a.K & 3) || M * a.K >= (1l << 31) - 256 || (long)a.B * a.H * a.W * a.C >= (1l << 31) - 256) return hipErrorInvalidValue;
    if ((long)a.R * a.R * a.CG * a.Kpad * 16 >= (1l << 31) - 256) return hipErrorInvalidValue;
    if (a.C < 8 || (a.C & 7)) {
        hipLaunchKernelGGL(conv_i8_direct_kernel, dim3(i8_blocks(M * (a.K >> 2))), dim3(256), 0, s, a, q);
        return hipGetLastError();
    }
    // more tiles per wave where that still leaves every SIMD a wave
    const long tiles = ((M + 15) / 16) * ((a.K + 15) / 16);
    if (tiles >= 16 * 1024 && a.K > 16) return launch_i8<2, 4>(a, q, s);
    if (tiles >= 4 * 1024) return launch_i8<1, 4>(a, q, s);
    return launch_i8<1, 1>(a, q, s);
}

hipError_t launch_fc_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s) {
    if (a.H * a.W != 1 || q.pool_hw < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fc_i8_kernel, dim3(i8_blocks((long)a.B * a.K)), dim3(256), 0, s, a, q);
    return hipGetLastError();
}

hipError_t launch_maxpool_i8(const PoolArgs &a, hipStream_t s) {
    if (a.C & 7) return hipErrorInvalidValue;
    hipLaunchKernelGGL(maxpool_i8_kernel, dim3(i8_blocks((long)a.B * a.P * a.Q * (a.C >> 3))), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gap_i8(const PoolArgs &a, const QuantArgs &q, hipStream_t s) {
    hipLaunchKernelGGL(gap_i8_kernel, dim3(i8_blocks((long)a.B * a.C)), dim3(256), 0, s, a, q);
    return hipGetLastError();
}

}  // namespace sushi
