// Device-side helpers shared by the per-layer kernels and the stream kernel: bf16 <-> float32,
// 8-element vector access, activations, matrix-core operand types.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace sushi {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

#define DW_DR_LIST                                                                                                  \
    -1, -1, -1, 0, 0, 0, 1, 1, 1, -2, -2, -2, -2, -2, -1, -1, 0, 0, 1, 1, 2, 2, 2, 2, 2, -3, -3, -3, -3, -3, -3, -3, \
        -2, -2, -1, -1, 0, 0, 1, 1, 2, 2, 3, 3, 3, 3, 3, 3, 3
#define DW_DS_LIST                                                                                                 \
    -1, 0, 1, -1, 0, 1, -1, 0, 1, -2, -1, 0, 1, 2, -2, 2, -2, 2, -2, 2, -2, -1, 0, 1, 2, -3, -2, -1, 0, 1, 2, 3, -3, \
        3, -3, 3, -3, 3, -3, 3, -3, 3, -3, -2, -1, 0, 1, 2, 3

// Ring order of depthwise taps: offset of tap t from the centre (3x3 first, then the 5x5 ring, then 7x7).
static __constant__ signed char c_dw_dr[49] = {DW_DR_LIST};
static __constant__ signed char c_dw_ds[49] = {DW_DS_LIST};

union Frag {
    uint4 u;
    bf16x8_t v;
};

// ------------------------------------------------------------------ element helpers

__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint32_t f2bf(float f) {  // round to nearest even
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ void load8(const float *p, float v[8]) {
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x, v[1] = a.y, v[2] = a.z, v[3] = a.w, v[4] = b.x, v[5] = b.y, v[6] = b.z, v[7] = b.w;
}

__device__ __forceinline__ void load8(const uint16_t *p, float v[8]) {
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    v[0] = bf2f(a.x & 0xFFFFu), v[1] = bf2f(a.x >> 16), v[2] = bf2f(a.y & 0xFFFFu), v[3] = bf2f(a.y >> 16);
    v[4] = bf2f(a.z & 0xFFFFu), v[5] = bf2f(a.z >> 16), v[6] = bf2f(a.w & 0xFFFFu), v[7] = bf2f(a.w >> 16);
}

__device__ __forceinline__ void store8(float *p, const float v[8]) {
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}

__device__ __forceinline__ void store8(uint16_t *p, const float v[8]) {
    uint4 a;
    a.x = f2bf(v[0]) | (f2bf(v[1]) << 16), a.y = f2bf(v[2]) | (f2bf(v[3]) << 16);
    a.z = f2bf(v[4]) | (f2bf(v[5]) << 16), a.w = f2bf(v[6]) | (f2bf(v[7]) << 16);
    *reinterpret_cast<uint4 *>(p) = a;
}

__device__ __forceinline__ float ld1(const float *p) { return *p; }
__device__ __forceinline__ float ld1(const uint16_t *p) { return bf2f(*p); }
__device__ __forceinline__ void st1(float *p, float v) { *p = v; }
__device__ __forceinline__ void st1(uint16_t *p, float v) { *p = (uint16_t)f2bf(v); }

__device__ __forceinline__ float activate(float v, int act, int hsig) {
    if (hsig) return fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) / 6.0f;
    if (act == 1) return fmaxf(v, 0.0f);
    if (act == 2) return v * fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) / 6.0f;
    return v;
}

}  // namespace sushi
