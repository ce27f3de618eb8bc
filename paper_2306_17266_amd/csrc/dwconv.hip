// Depthwise k x k convolution for the per-layer launch path (bf16, activations [B][H][W][C]).
//
// A thread produces a strip of DWR_T neighbouring outputs for one group of 8 channels: one below the other in a
// column (stride 1) or side by side in a row (stride 2).  For every tap line across the strip it requests, in
// one batch, the (DWR_T - 1) * stride + k input cells those outputs share (16 bytes each) and the line's k
// weight cells, so a thread waits for k load round trips instead of k * k, and an input cell is loaded once for
// all the outputs of the thread that use it.  Neighbouring lanes hold neighbouring channel groups, then
// neighbouring columns (column strips: every load and store of a wave is one contiguous run of cells, and what
// a load costs a compute unit follows the number of cache lines it touches) or neighbouring strips (row strips:
// at stride 2 a column strip would use every other cell of the lines it touches).  Cells outside the image are
// requested past the end of the buffer (a buffer load returns zeros there), which keeps the loads unconditional.
//
// Arithmetic: float32 multiply-add per (tap, channel), bf16 in and out.  Per output cell of 8 channels that is
// 8 k^2 multiply-adds plus the bf16 -> float32 unpacking of about k (k + (DWR_T - 1) stride) / DWR_T input
// cells plus the epilogue; for k = 7 the vector ALUs, not memory, bound the kernel.
#include "kernels.h"
#include "device_common.h"

namespace sushi {

typedef __attribute__((ext_vector_type(4))) unsigned dw_u32x4;
constexpr int DWR_T = 4;
constexpr int DWR_OOB = 0x7FFFFFF0;

__device__ __forceinline__ void dw_unpack(const dw_u32x4 q, float v[8]) {
    v[0] = bf2f(q.x & 0xFFFFu), v[1] = bf2f(q.x >> 16), v[2] = bf2f(q.y & 0xFFFFu), v[3] = bf2f(q.y >> 16);
    v[4] = bf2f(q.z & 0xFFFFu), v[5] = bf2f(q.z >> 16), v[6] = bf2f(q.w & 0xFFFFu), v[7] = bf2f(q.w >> 16);
}

// VERT: the strip runs down a column (outputs p0 .. p0 + T - 1 at column q), else along a row.
template <int R, int S, int ACT, bool VERT>
__global__ __launch_bounds__(256) void dwconv_rows_kernel(ConvArgs a) {
    constexpr int HALF = (R - 1) / 2, T = DWR_T, NS = (T - 1) * S + R;
    const int cgs = a.K >> 3;
    const int U = VERT ? a.P : a.Q, V = VERT ? a.Q : a.P;        // outputs along / across the strip direction
    const int IU = VERT ? a.H : a.W, IV = VERT ? a.W : a.H;      // the input's extents likewise
    const int ublocks = (U + T - 1) / T;
    const long total = (long)a.B * ublocks * V * cgs;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cg = (int)(idx % cgs);
    long rest = idx / cgs;
    int ub, v;
    if (VERT) {
        v = (int)(rest % V), rest /= V;
        ub = (int)(rest % ublocks), rest /= ublocks;
    } else {
        ub = (int)(rest % ublocks), rest /= ublocks;
        v = (int)(rest % V), rest /= V;
    }
    const int n = (int)rest;
    const int c = cg * 8;
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.x), 0, (int)((long)a.B * a.H * a.W * a.C * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(a.w), 0, a.Rmax * a.Rmax * a.Kpad * 2, 0x00020000);
    // byte steps of the input along and across the strip direction
    const int step_u = (VERT ? a.W : 1) * a.C * 2, step_v = (VERT ? 1 : a.W) * a.C * 2;
    const int u0 = ub * T * S - HALF, v0 = v * S - HALF;
    const int base = (n * a.H * a.W * a.C + c) * 2;
    int uoff[NS];  // byte offset of the window's cell i along the strip, or -1 outside the image
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int u = u0 + i;
        uoff[i] = (u >= 0 && u < IU) ? base + u * step_u : -1;
    }
    float acc[T][8];
#pragma unroll
    for (int k = 0; k < T; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[k][e] = 0.f;
    // (one tap line at a time: unrolled, the compiler would request every line's cells at once and run out of
    // registers)
#pragma unroll 1
    for (int dv = 0; dv < R; ++dv) {
        const int vv = v0 + dv;
        const bool v_ok = vv >= 0 && vv < IV;
        const int voff = vv * step_v;
        dw_u32x4 wq[R], xq[NS];
#pragma unroll
        for (int du = 0; du < R; ++du) {
            const int tap = VERT ? dw_tap_index(du - HALF, dv - HALF) : dw_tap_index(dv - HALF, du - HALF);
            wq[du] = __builtin_amdgcn_raw_buffer_load_b128(rw, (tap * a.Kpad + c) * 2, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < NS; ++i)
            xq[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, v_ok && uoff[i] >= 0 ? uoff[i] + voff : DWR_OOB, 0, 0);
        float wv[R][8];
#pragma unroll
        for (int du = 0; du < R; ++du) dw_unpack(wq[du], wv[du]);
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            float xv[8];
            dw_unpack(xq[i], xv);
#pragma unroll
            for (int k = 0; k < T; ++k) {
                const int du = i - k * S;  // (a constant once the loops are unrolled)
                if (du >= 0 && du < R) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[k][e] = fmaf(wv[du][e], xv[e], acc[k][e]);
                }
            }
        }
    }
    float sc[8], sh[8];
    load8(a.scale + c, sc);
    load8(a.shift + c, sh);
    uint16_t *y = static_cast<uint16_t *>(a.y);
#pragma unroll
    for (int k = 0; k < T; ++k) {
        const int u = ub * T + k;
        if (u >= U) break;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float t = acc[k][e] * sc[e] + sh[e];
            acc[k][e] = ACT == 1 ? fmaxf(t, 0.0f) : ACT == 2 ? t * fminf(fmaxf(t + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f) : t;
        }
        const int p = VERT ? u : v, q = VERT ? v : u;
        store8(y + (((long)n * a.P + p) * a.Q + q) * a.K + c, acc[k]);
    }
}

template <int R, int S>
static hipError_t launch_rows(const ConvArgs &a, hipStream_t s) {
    constexpr bool VERT = S == 1;
    const int U = VERT ? a.P : a.Q, V = VERT ? a.Q : a.P;
    const long total = (long)a.B * ((U + DWR_T - 1) / DWR_T) * V * (a.K >> 3);
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (a.act == 1)
        hipLaunchKernelGGL((dwconv_rows_kernel<R, S, 1, VERT>), grid, block, 0, s, a);
    else if (a.act == 2)
        hipLaunchKernelGGL((dwconv_rows_kernel<R, S, 2, VERT>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((dwconv_rows_kernel<R, S, 0, VERT>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_dwconv_rows(const ConvArgs &a, hipStream_t s) {
    if ((a.K & 7) != 0 || a.C != a.K || a.pad != (a.R - 1) / 2) return hipErrorNotSupported;
    if ((long)a.B * a.H * a.W * a.C * 2 >= (1l << 31) - 256) return hipErrorNotSupported;
    if (!a.scale) return hipErrorNotSupported;
    switch (a.R * 4 + a.stride) {
        case 3 * 4 + 1: return launch_rows<3, 1>(a, s);
        case 3 * 4 + 2: return launch_rows<3, 2>(a, s);
        case 5 * 4 + 1: return launch_rows<5, 1>(a, s);
        case 5 * 4 + 2: return launch_rows<5, 2>(a, s);
        case 7 * 4 + 1: return launch_rows<7, 1>(a, s);
        case 7 * 4 + 2: return launch_rows<7, 2>(a, s);
        default: return hipErrorNotSupported;
    }
}

}  // namespace sushi
