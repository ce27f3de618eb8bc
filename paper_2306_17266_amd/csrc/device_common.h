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

// Position of the tap at offset (dr, ds) from the centre in the ring order of the stored taps.
__host__ __device__ constexpr int dw_tap_index(int dr, int ds) {
    const int ar = dr < 0 ? -dr : dr, as = ds < 0 ? -ds : ds;
    const int r = ar > as ? ar : as;
    if (r <= 1) return (dr + 1) * 3 + ds + 1;
    const int base = (2 * r - 1) * (2 * r - 1);
    if (dr == -r) return base + ds + r;
    if (dr == r) return base + (2 * r + 1) + 2 * (2 * r - 1) + ds + r;
    return base + (2 * r + 1) + (dr + r - 1) * 2 + (ds == r ? 1 : 0);
}

union Frag {
    uint4 u;
    bf16x8_t v;
};

// ------------------------------------------------------------------ element helpers

__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

// Two float32 values to one word of two bf16 (lo in bits 15:0), round to nearest even: the hardware's packed
// conversion (v_cvt_pk_bf16_f32), one instruction instead of about ten.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ uint32_t f2bf(float f) { return pack_bf16x2(f, 0.0f) & 0xFFFFu; }  // round to nearest even

// Eight float32 values (two 16-byte words) as two bf16 operands of eight: x = hi + lo, hi = bf16(x) rounded to
// nearest even, lo = bf16(x - hi); together they carry about 16 bits of x's mantissa.
__device__ __forceinline__ void split_f32x8(const uint4 a, const uint4 b, uint4 *hi, uint4 *lo) {
    const float x[8] = {__uint_as_float(a.x), __uint_as_float(a.y), __uint_as_float(a.z), __uint_as_float(a.w),
                        __uint_as_float(b.x), __uint_as_float(b.y), __uint_as_float(b.z), __uint_as_float(b.w)};
    unsigned h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        h[i] = pack_bf16x2(x[2 * i], x[2 * i + 1]);
        l[i] = pack_bf16x2(x[2 * i] - bf2f(h[i] & 0xFFFFu), x[2 * i + 1] - bf2f(h[i] >> 16));
    }
    *hi = make_uint4(h[0], h[1], h[2], h[3]);
    *lo = make_uint4(l[0], l[1], l[2], l[3]);
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
    a.x = pack_bf16x2(v[0], v[1]), a.y = pack_bf16x2(v[2], v[3]);
    a.z = pack_bf16x2(v[4], v[5]), a.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4 *>(p) = a;
}

__device__ __forceinline__ float ld1(const float *p) { return *p; }
__device__ __forceinline__ float ld1(const uint16_t *p) { return bf2f(*p); }
__device__ __forceinline__ void st1(float *p, float v) { *p = v; }
__device__ __forceinline__ void st1(uint16_t *p, float v) { *p = (uint16_t)f2bf(v); }

// (v + 2^(s-1)) >> s on 64-bit integers, arithmetic shift, 1 <= s <= 62: the rounding shift of the int8 path
__device__ __forceinline__ long long rr64(long long v, int s) { return (v + (1ll << (s - 1))) >> s; }

__device__ __forceinline__ float activate(float v, int act, int hsig) {
    if (hsig) return fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
    if (act == 1) return fmaxf(v, 0.0f);
    if (act == 2) return v * fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
    return v;
}

}  // namespace sushi
