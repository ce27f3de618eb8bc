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

// A workgroup of four waves computes FT x PT tiles of 16 filters x 16 pixels; the waves split the reduction steps
// (one tap, 64 channels) among them, each requests the operands of U of its steps before it multiplies them, and
// the partial sums meet in LDS.  Integer addition is exact in any order, so the split changes no result.
template <int FT, int PT, int U>
__global__ __launch_bounds__(256) void conv_i8_kernel(ConvArgs a, QuantArgs q) {
    __shared__ int red[4][FT * PT][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const long M = (long)a.B * a.P * a.Q;
    const int f0 = blockIdx.y * FT * 16;
    const long m0 = (long)blockIdx.x * PT * 16;
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
    const int nsteps = a.R * a.R * csteps;
    for (int base = wave; base < nsteps; base += 4 * U) {
        i32x4_t fa[U][FT], fb[U][PT];
        bool inside[U][PT];
        int c0s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int step = base + 4 * u;
            const bool live = step < nsteps;
            const int st = live ? step : 0;
            const int tap = st / csteps, cs = st - tap * csteps;
            const int dr = tap / a.R, ds = tap - dr * a.R;
            const int c0 = cs * 64 + kg * 16;       // this lane's 16 channels
            const int cg = c0 >> 4;
            c0s[u] = live ? c0 : a.C;               // (a step beyond the end: treated as channels beyond the SubNet's)
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
                fa[u][ft] = __builtin_bit_cast(i32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                    rw, live && fw[ft] >= 0 && cg < a.CG ? ((tap * a.CG + cg) * a.Kpad) * 16 + fw[ft] : I8_OOB, 0, 0));
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                const int h = ph[pt] + dr, v = pw[pt] + ds;
                inside[u][pt] = pv[pt] && h >= 0 && h < a.H && v >= 0 && v < a.W;
                const int off = live && inside[u][pt] && c0 < a.C ? ((pn[pt] * a.H + h) * a.W + v) * a.C + c0 : I8_OOB;
                fb[u][pt] = __builtin_bit_cast(i32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 0));
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c0 = c0s[u];
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                i32x4_t b = fb[u][pt];
                if (c0 + 8 >= a.C) b[2] = 0, b[3] = 0;        // the cell's upper half lies beyond the active channels
                if (!inside[u][pt] && c0 < a.C) {               // a cell of the frame: the code of the real value 0
                    b[0] = (int)zfill, b[1] = (int)zfill;
                    if (c0 + 8 < a.C) b[2] = (int)zfill, b[3] = (int)zfill;
                }
                fb[u][pt] = b;
            }
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
                    acc[ft][pt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[u][ft], fb[u][pt], acc[ft][pt], 0, 0, 0);
        }
    }
#pragma unroll
    for (int ft = 0; ft < FT; ++ft)
#pragma unroll
        for (int pt = 0; pt < PT; ++pt)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave][ft * PT + pt][i][lane] = acc[ft][pt][i];
    __syncthreads();
    // wave w finishes tiles w, w + 4, ...; the lane holds pixel l16 and filters 4 kg .. 4 kg + 3 of a tile
    for (int t = wave; t < FT * PT; t += 4) {
        const int ft = t / PT, pt = t - ft * PT;
        const int f = f0 + ft * 16 + kg * 4;
        const long m = m0 + pt * 16 + l16;
        if (f >= a.K || m >= M) continue;
        int v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[i] = red[0][t][i][lane] + red[1][t][i][lane] + red[2][t][i][lane] + red[3][t][i][lane];
            if (q.zx != 0) v[i] -= q.zx * q.wsum[f + i];
        }
        store_codes(a, q, v, f, m);
    }
}

// Fewer than 8 input channels (the network input): one thread per output pixel, all filters of a group of up to 32;
// the group's weights sit in LDS as int32 [tap * C + channel][32] (every thread reads the same word: a broadcast).
__global__ __launch_bounds__(256) void conv_i8_direct_kernel(ConvArgs a, QuantArgs q) {
    __shared__ int wl[49 * 4 * 32];
    const int f0 = blockIdx.y * 32;
    const int nf = min(32, a.K - f0);
    const int taps = a.R * a.R;
    const int8_t *w = static_cast<const int8_t *>(a.w);
    for (int i = threadIdx.x; i < taps * a.C * 32; i += 256) {
        const int f = i & 31, tc = i >> 5;
        const int tap = tc / a.C, ch = tc - tap * a.C;
        wl[i] = f < nf ? (int)w[(((long)tap * a.CG + (ch >> 4)) * a.Kpad + f0 + f) * 16 + (ch & 15)] : 0;
    }
    __syncthreads();
    const long M = (long)a.B * a.P * a.Q;
    const long m = (long)blockIdx.x * 256 + threadIdx.x;
    if (m >= M) return;
    const int qq = (int)(m % a.Q), pp = (int)((m / a.Q) % a.P), n = (int)(m / ((long)a.Q * a.P));
    const int8_t *x = static_cast<const int8_t *>(a.x);
    int acc[32];
#pragma unroll
    for (int f = 0; f < 32; ++f) acc[f] = 0;
    for (int tap = 0; tap < taps; ++tap) {
        const int h = pp * a.stride - a.pad + tap / a.R, v = qq * a.stride - a.pad + tap % a.R;
        if (h < 0 || h >= a.H || v < 0 || v >= a.W) continue;
        const int8_t *xp = x + (((long)n * a.H + h) * a.W + v) * a.C;
        for (int ch = 0; ch < a.C; ++ch) {
            const int xv = (int)xp[ch] - q.zx;
            const int4 *wr = reinterpret_cast<const int4 *>(wl + (tap * a.C + ch) * 32);
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const int4 wv = wr[g];
                acc[4 * g] += xv * wv.x, acc[4 * g + 1] += xv * wv.y, acc[4 * g + 2] += xv * wv.z, acc[4 * g + 3] += xv * wv.w;
            }
        }
    }
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        const int v[4] = {acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
        store_codes(a, q, v, f0 + 4 * g, m);
    }
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

// Exact sums of (code - z_x) over H x W: one thread per (image, group of 8 channels); int32 out.
__global__ __launch_bounds__(256) void gap_i8_kernel(PoolArgs a, QuantArgs q) {
    const int cgs = a.C >> 3;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)a.B * cgs) return;
    const int cg = (int)(idx % cgs), n = (int)(idx / cgs);
    const int8_t *x = static_cast<const int8_t *>(a.x) + (long)n * a.H * a.W * a.C + cg * 8;
    int sum[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) sum[j] = 0;
#pragma unroll 8
    for (int p = 0; p < a.H * a.W; ++p) {
        const uint2 v = *reinterpret_cast<const uint2 *>(x + (long)p * a.C);
#pragma unroll
        for (int j = 0; j < 8; ++j) sum[j] += (int)(int8_t)((j < 4 ? v.x : v.y) >> (8 * (j & 3))) - q.zx;
    }
    int *y = static_cast<int *>(a.y) + (long)n * a.C + cg * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) y[j] = sum[j];
}

// Classifier on the pooled sums: a workgroup serves 64 classes of one image; the image's sums sit in LDS, wave w
// takes the channel cells w, w + 4, ... (eight weight cells requested at a time), and the four partial sums are
// added in LDS (exact: integers).  int64 accumulator, float32 logit.
__global__ __launch_bounds__(256) void fc_i8_kernel(ConvArgs a, QuantArgs q) {
    extern __shared__ int fc_sums[];               // C sums, then 4 x 64 partial sums (two words each)
    const int n = blockIdx.y, kk = threadIdx.x & 63, part = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + kk;
    const int cpad = (a.C + 15) & ~15;
    const int *sums = static_cast<const int *>(a.x) + (long)n * a.C;
    for (int i = threadIdx.x; i < cpad; i += 256) fc_sums[i] = i < a.C ? sums[i] : 0;
    __syncthreads();
    long long acc = 0;
    if (k < a.K) {
        const uint4 *w = static_cast<const uint4 *>(a.w) + k;
        const int ncell = cpad >> 4;
#pragma unroll 1
        for (int c0 = part; c0 < ncell; c0 += 32) {
            uint4 cell[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) cell[u] = c0 + 4 * u < ncell ? w[(long)(c0 + 4 * u) * a.Kpad] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int cb = min(c0 + 4 * u, ncell - 1) * 16;
                const unsigned word[4] = {cell[u].x, cell[u].y, cell[u].z, cell[u].w};
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    acc += (long long)fc_sums[cb + j] * (long long)(int)(int8_t)(word[j >> 2] >> (8 * (j & 3)));
            }
        }
    }
    long long *part_sums = reinterpret_cast<long long *>(fc_sums + cpad);
    part_sums[part * 64 + kk] = acc;
    __syncthreads();
    if (part == 0 && k < a.K) {
        const long long total = part_sums[kk] + part_sums[64 + kk] + part_sums[128 + kk] + part_sums[192 + kk] +
                                (long long)q.pool_hw * (long long)q.qbias[k];
        const double base = (double)__int_as_float(q.qmult[k]);
        static_cast<float *>(a.y)[(long)n * a.K + k] = (float)((double)total * (base / (double)q.pool_hw));
    }
}

// ------------------------------------------------------------------ launchers

static inline unsigned i8_blocks(long total) { return (unsigned)((total + 255) / 256); }

template <int FT, int PT, int U>
static hipError_t launch_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s) {
    const long M = (long)a.B * a.P * a.Q;
    const long n_pgroups = (M + 16 * PT - 1) / (16 * PT);
    const int n_fgroups = (a.K + 16 * FT - 1) / (16 * FT);
    hipLaunchKernelGGL((conv_i8_kernel<FT, PT, U>), dim3((unsigned)n_pgroups, n_fgroups), dim3(256), 0, s, a, q);
    return hipGetLastError();
}

hipError_t launch_conv_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s, long patch_min_pixels) {
    const long M = (long)a.B * a.P * a.Q;
    if ((a.K & 3) || M * a.K >= (1l << 31) - 256 || (long)a.B * a.H * a.W * a.C >= (1l << 31) - 256) return hipErrorInvalidValue;
    if ((long)a.R * a.R * a.CG * a.Kpad * 16 >= (1l << 31) - 256) return hipErrorInvalidValue;
    if (patch_min_pixels > 0 && M >= patch_min_pixels && (M >= 4 * patch_min_pixels || (long)a.C * a.R * a.R >= 2048)) {
        const hipError_t e = launch_conv_patch_i8(a, q, s);
        if (e != hipErrorNotSupported) return e;
    }
    if (a.C < 8 || (a.C & 7)) {
        if (a.C > 4 || a.R * a.R > 49) return hipErrorInvalidValue;
        hipLaunchKernelGGL(conv_i8_direct_kernel, dim3(i8_blocks(M), (unsigned)((a.K + 31) / 32)), dim3(256), 0, s, a, q);
        return hipGetLastError();
    }
    // more tiles per workgroup where that still leaves every compute unit about two workgroups
    const long tiles = ((M + 15) / 16) * ((a.K + 15) / 16);
    if (tiles >= 8 * 512 && a.K > 16) return launch_i8<2, 4, 2>(a, q, s);
    if (tiles >= 4 * 512) return launch_i8<1, 4, 4>(a, q, s);
    if (tiles >= 2 * 512) return launch_i8<1, 2, 4>(a, q, s);
    return launch_i8<1, 1, 4>(a, q, s);
}

hipError_t launch_fc_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s) {
    if (a.H * a.W != 1 || q.pool_hw < 1) return hipErrorInvalidValue;
    const size_t lds = (size_t)((a.C + 15) & ~15) * 4 + 4 * 64 * 8;
    if (lds > 60 * 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fc_i8_kernel, dim3((unsigned)((a.K + 63) / 64), (unsigned)a.B), dim3(256), lds, s, a, q);
    return hipGetLastError();
}

hipError_t launch_maxpool_i8(const PoolArgs &a, hipStream_t s) {
    if (a.C & 7) return hipErrorInvalidValue;
    hipLaunchKernelGGL(maxpool_i8_kernel, dim3(i8_blocks((long)a.B * a.P * a.Q * (a.C >> 3))), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gap_i8(const PoolArgs &a, const QuantArgs &q, hipStream_t s) {
    if (a.C & 7) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gap_i8_kernel, dim3(i8_blocks((long)a.B * (a.C >> 3))), dim3(256), 0, s, a, q);
    return hipGetLastError();
}

}  // namespace sushi
