// Dense 1x1 and 3x3 convolution for large pixel counts (batch 16 and up) on the matrix cores: an implicit GEMM
// whose activation operand is an input PATCH held in LDS (bf16, activations [B][H][W][C], float32 accumulation).
//
// A workgroup of four waves computes BN = 32 TF filters x BM = 128 TM consecutive output pixels (pixels counted
// through images, rows and columns); wave w owns pixels w * 32 TM .. + 32 TM - 1 and all BN filters, TF x TM
// accumulator tiles of v_mfma_f32_32x32x16_bf16.  The input is addressed in PADDED coordinates: image n, row
// h + pad, column w + pad of an (H + 2 pad) x (W + 2 pad) frame have the linear position
// u = (n (H + 2 pad) + h + pad)(W + 2 pad) + w + pad, so output pixel (n, p, q) reads, for tap (dr, ds), position
// base(n, p, q) + dr (W + 2 pad) + ds with base = (n (H + 2 pad) + p stride)(W + 2 pad) + q stride.  base grows with
// the pixel index, so the positions a tile needs are ONE contiguous range; the workgroup copies that range, for
// one chunk of CK channels at a time, from memory into LDS (frame cells and cells outside the tensor arrive as
// zeros: the loads are buffer loads aimed past the end of the buffer), and all R x R taps of the chunk are
// multiplied from the same copy.  A 3x3 layer therefore fetches an input cell once per chunk instead of nine
// times, and every wave load of the copy runs along contiguous pixels.
//
// LDS: the patch as [8-channel group][position] planes of 16-byte cells, double-buffered per chunk; the weights of
// one STAGE (the R taps of one tap row, one chunk) as [tap][group][filter] planes, double-buffered per stage.  A
// matrix-core operand read is then 32 consecutive cells per half-wave.  The global loads of the next stage's
// weights and of the next chunk's patch are in flight (registers) while the current stage is multiplied; one
// workgroup barrier per stage.
//
// Epilogue: every wave passes its outputs through LDS (its own region, no workgroup barrier) so that the residual
// is read and the result written as whole 16-byte cells along the channels, contiguous BN * 2 bytes per pixel,
// instead of 8-byte pieces per lane.  y = act(scale * acc + shift (+ res)), rounded to bf16 once.
#include "kernels.h"
#include "device_common.h"

#include <algorithm>
#include <type_traits>
#include <unordered_map>

namespace sushi {

typedef __attribute__((ext_vector_type(16))) float cp_f32x16;
typedef __attribute__((ext_vector_type(16))) int cp_i32x16;
typedef __attribute__((ext_vector_type(4))) int cp_i32x4;
typedef __attribute__((ext_vector_type(4))) unsigned cp_u32x4;
constexpr int CP_OOB = 0x7FFFFFF0;

// Division of a non-negative int below 2^31 by a fixed divisor d: n / d = mulhi(n, mul) >> shr for d > 1
// (mul = ceil(2^(31 + ceil(log2 d)) / d) fits 32 bits), n itself for d = 1.  The host prepares (mul, shr).
struct FastDiv {
    unsigned mul, shr;
    int d;
};

__host__ inline FastDiv make_fastdiv(int d) {
    FastDiv f{0u, 0u, d};
    if (d > 1) {
        int lg = 0;
        while ((1ll << lg) < d) ++lg;
        const int p = 31 + lg;
        f.mul = (unsigned)(((1ull << p) + (unsigned long long)d - 1) / (unsigned long long)d);
        f.shr = (unsigned)(p - 32);
    }
    return f;
}

__device__ __forceinline__ int fdiv(int n, const FastDiv &f) {
    return f.d == 1 ? n : (int)(__umulhi((unsigned)n, f.mul) >> f.shr);
}

struct PatchGeom {
    int tiles_f, tiles_m;
    int hp, wp;      // frame: H + 2 pad, W + 2 pad
    int ps;          // cells between the patch planes of neighbouring channel groups
    int M;           // B * P * Q
    int ss;          // cell offset of the scale / shift copies in LDS
    FastDiv dq, dp, dwp, dhp;  // division by Q, P, wp, hp
};

__device__ __forceinline__ int cp_base(const ConvArgs &a, const PatchGeom &g, int m) {
    const int t = fdiv(m, g.dq), q = m - t * a.Q;
    const int n = fdiv(t, g.dp), p = t - n * a.P;
    return (n * g.hp + p * a.stride) * g.wp + q * a.stride;
}

// I8: the int8 path (int8 codes, v_mfma_i32_32x32x32_i8, integer requantisation: see int8.hip for the arithmetic).
// A 16-byte cell then holds 16 channels instead of 8; everything that is counted in cells stays as it is.
template <int TF, int TM, int CK, int R, int MAXP, int MINB, int NW, bool I8>
__global__ __launch_bounds__(64 * NW, MINB) void conv_patch_kernel(ConvArgs a, PatchGeom g, QuantArgs q) {
    constexpr int NT = 64 * NW;  // threads
    constexpr int ES = I8 ? 1 : 2, CPC = 16 / ES;  // bytes per element, channels per cell
    constexpr int BN = 32 * TF, BM = 32 * NW * TM, NKG = CK / CPC, WPS = BN + 4;
    constexpr int PPW = NT / NKG;  // positions one pass of the workgroup's threads covers
    constexpr int WCELLS = R * NKG * BN, WPT = (WCELLS + NT - 1) / NT;
    constexpr int KSUB = NKG / 2;     // a matrix instruction takes two cells per lane pair
    constexpr int ROWC = BN / 8 + 1;  // epilogue: pieces per pixel row (one spare); a piece = 8 filters (16 bytes, int8: 8)
    extern __shared__ uint4 cp_lds[];
    uint4 *const patch = cp_lds;                         // [2][NKG * ps]
    uint4 *const wts = cp_lds + 2 * NKG * g.ps;          // [2][R * NKG * WPS]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kh = lane >> 5;
    const int ntiles = g.tiles_f * g.tiles_m;
    const int per_xcd = (ntiles + 7) >> 3;
    const int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (tile >= ntiles) return;
    const int tf = tile / g.tiles_m, tm = tile - tf * g.tiles_m;
    const int f0 = tf * BN, m0 = tm * BM;
    const int M = g.M;
    const int mlast = min(m0 + BM, M) - 1;
    const int u0 = cp_base(a, g, m0);
    const int npos = cp_base(a, g, mlast) + (R - 1) * (g.wp + 1) - u0 + 1;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.x), 0, (int)((long)a.B * a.H * a.W * a.C * ES), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.w), 0, (int)((long)R * R * a.CG * a.Kpad * 16), 0x00020000);

    // what this thread copies of a patch: cells (position pk + j * PPW, group kgp); byte offset at chunk 0 or -1
    const int kgp = tid % NKG, pk = tid / NKG;
    int poff[MAXP];
#pragma unroll
    for (int j = 0; j < MAXP; ++j) {
        const int pos = pk + j * PPW;
        const int u = u0 + pos;
        const int t = fdiv(u, g.dwp), n = fdiv(t, g.dhp);
        const int h = t - n * g.hp - a.pad, w = u - t * g.wp - a.pad;
        const bool ok = pos < npos && n < a.B && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
        poff[j] = ok ? (((n * a.H + h) * a.W + w) * a.C + kgp * CPC) * ES : -1;
    }
    // ... and of a stage's weights: cells (tap column t, group kg, filter f)
    int woff[WPT], wkg[WPT], wlds[WPT];
#pragma unroll
    for (int j = 0; j < WPT; ++j) {
        const int i = tid + NT * j;
        const int t = i / (NKG * BN), r = i - t * (NKG * BN);
        const int kg = r / BN, f = r - kg * BN;
        const bool ok = i < WCELLS && f0 + f < a.Kpad;
        woff[j] = ok ? ((t * a.CG + kg) * a.Kpad + f0 + f) * 16 : -1;
        wkg[j] = kg;
        wlds[j] = (t * NKG + kg) * WPS + f;
    }
    const int nchunks = (a.C + CK - 1) / CK;
    const int nstages = nchunks * R;
    // Register sets of the loads in flight: a stage's weights (and, for R = 1, its patch) are requested D = 3
    // stages before they are multiplied, the patch of a 3x3 chunk one chunk (three stages) ahead: about 1.5 us at
    // full matrix-core rate, the order of a load that misses the L2.  Stages run in groups of D, unrolled, so a
    // set's index is static.
    constexpr int D = 3;
    constexpr int NPS = R == 3 ? 1 : D;
    cp_u32x4 pr[NPS][MAXP], wr[D][WPT];
    auto load_patch = [&](int chunk, cp_u32x4 *regs) {
        const int c0 = chunk * CK;
        const bool cv = c0 + kgp * CPC < a.C;
#pragma unroll
        for (int j = 0; j < MAXP; ++j)
            if (j * PPW < npos)
                regs[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, cv && poff[j] >= 0 ? poff[j] + c0 * ES : CP_OOB, 0, 0);
    };
    // int8: a cell of the frame holds the code of the real value 0 (the input's zero point) in its active channels,
    // and the upper half of a cell that straddles the SubNet's channel count holds zeros (the load brought the next
    // pixel's bytes there).  `chunk` is the chunk the registers were loaded for.
    const unsigned zfill = (unsigned)(q.zx & 0xFF) * 0x01010101u;
    auto store_patch = [&](int buf, const cp_u32x4 *regs, int chunk) {
        uint4 *dst = patch + buf * NKG * g.ps + kgp * g.ps + pk;
        const int cc = chunk * CK + kgp * CPC;  // first channel of this thread's cells
#pragma unroll
        for (int j = 0; j < MAXP; ++j)
            if (pk + j * PPW < npos) {
                cp_u32x4 v = regs[j];
                if (I8) {
                    if (poff[j] < 0 && cc < a.C) v = cp_u32x4{zfill, zfill, zfill, zfill};
                    if (cc + 8 >= a.C) v[2] = 0u, v[3] = 0u;
                }
                dst[j * PPW] = __builtin_bit_cast(uint4, v);
            }
    };
    auto load_w = [&](int stage, cp_u32x4 *regs) {
        const int chunk = stage / R, dr = stage - chunk * R;
        const int cg0 = chunk * NKG;
        const int add = (dr * R * a.CG + cg0) * a.Kpad * 16;
#pragma unroll
        for (int j = 0; j < WPT; ++j)
            regs[j] = __builtin_amdgcn_raw_buffer_load_b128(rw, woff[j] >= 0 && cg0 + wkg[j] < a.CG ? woff[j] + add : CP_OOB, 0, 0);
    };
    auto store_w = [&](int buf, const cp_u32x4 *regs) {
        uint4 *dst = wts + buf * R * NKG * WPS;
#pragma unroll
        for (int j = 0; j < WPT; ++j)
            if (tid + NT * j < WCELLS) dst[wlds[j]] = __builtin_bit_cast(uint4, regs[j]);
    };

    // prologue: the loads of the first D stages; stage 0 into LDS.  The tile's scale and shift values go to LDS
    // as well (requested now, read in the epilogue).
    load_patch(0, pr[0]);
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < nstages) {
            load_w(d, wr[d]);
            if (R == 1 && d > 0) load_patch(d, pr[d % NPS]);
        }
    __builtin_amdgcn_sched_barrier(0);  // (everything below runs while those loads are on their way)
    // operand reads: position of this lane's pixel in tile column j, relative to the patch
    int boff[TM];
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = m0 + (wave * TM + j) * 32 + l32;
        boff[j] = m < M ? cp_base(a, g, m) - u0 : 0;
    }

    typename std::conditional<I8, cp_i32x16, cp_f32x16>::type acc[TF][TM];
#pragma unroll
    for (int i = 0; i < TF; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[i][j][k] = 0;

    if (I8) {
        // int8: multiplier, shift, and the bias with the zero-point term folded in (bias - z_x * sum of the active weights)
        if (tid < 3 * BN / 4) {
            const int which = tid / (BN / 4), f = f0 + (tid - which * (BN / 4)) * 4;
            int4 v = which == 1 ? make_int4(1, 1, 1, 1) : make_int4(0, 0, 0, 0);
            if (f < a.K) {
                v = *reinterpret_cast<const int4 *>((which == 0 ? q.qmult : which == 1 ? q.qshift : q.qbias) + f);
                if (which == 2) {
                    const int4 ws = *reinterpret_cast<const int4 *>(q.wsum + f);
                    v.x -= q.zx * ws.x, v.y -= q.zx * ws.y, v.z -= q.zx * ws.z, v.w -= q.zx * ws.w;
                }
            }
            reinterpret_cast<int4 *>(cp_lds + g.ss)[tid] = v;
        }
    } else if (tid < BN / 2) {
        const bool is_shift = tid >= BN / 4;
        const int f = f0 + (is_shift ? tid - BN / 4 : tid) * 4;
        float4 v = is_shift ? make_float4(0.f, 0.f, 0.f, 0.f) : make_float4(1.f, 1.f, 1.f, 1.f);
        if (f < a.K && (is_shift || a.scale)) v = *reinterpret_cast<const float4 *>((is_shift ? a.shift : a.scale) + f);
        reinterpret_cast<float4 *>(cp_lds + g.ss)[tid] = v;
    }
    store_patch(0, pr[0], 0);
    store_w(0, wr[0]);
    __syncthreads();
    for (int grp = 0; grp * D < nstages; ++grp) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int st = grp * D + d;
            if (st >= nstages) break;
            const int chunk = R == 3 ? grp : st, dr = R == 3 ? d : 0;
            const uint4 *pb = patch + (chunk & 1) * NKG * g.ps + dr * g.wp;
            const uint4 *wb = wts + (st & 1) * R * NKG * WPS;
            // Sub-steps (tap column t, 16 channels): the operands of sub-step s + 1 are requested from LDS before
            // the matrix instructions of sub-step s are issued (two operand register sets; a third set, two
            // sub-steps ahead, gains nothing: with one wave per SIMD the loop is bound by the rate at which one
            // wave gets LDS reads served, about one KiB per 50 clocks, not by their latency).
            constexpr int NSUB = R * KSUB, NFS = 2;
            Frag fa[NFS][TF], fb[NFS][TM];
            auto read_frags = [&](int s, Frag *qa, Frag *qb) {
                const int t = s / KSUB, kg = 2 * (s - t * KSUB) + kh;
#pragma unroll
                for (int i = 0; i < TF; ++i) qa[i].u = wb[(t * NKG + kg) * WPS + i * 32 + l32];
#pragma unroll
                for (int j = 0; j < TM; ++j) qb[j].u = pb[kg * g.ps + boff[j] + t];
            };
            read_frags(0, fa[0], fb[0]);
            __builtin_amdgcn_sched_barrier(0);
            // While the first operands are on their way: the register sets that the previous stage's hand-over
            // emptied take the loads of stage st + D (and of the next 3x3 chunk's patch).
            if (st + D < nstages) {
                load_w(st + D, wr[d]);
                if (R == 1) load_patch(st + D, pr[d % NPS]);
            }
            if (R == 3 && d == 0 && chunk + 1 < nchunks) load_patch(chunk + 1, pr[0]);
            const bool chunk_ends = R == 1 || d == D - 1;
            const int dn = (d + 1) % D;  // (static once the loop over d is unrolled)
#pragma unroll
            for (int s = 0; s < NSUB; ++s) {
                if (s + 1 < NSUB) read_frags(s + 1, fa[(s + 1) % NFS], fb[(s + 1) % NFS]);
                // before the last sub-step's matrix instructions: stage st + 1 (requested D stages ago) goes to
                // the LDS buffers that stage st - 1 used, so the stores run under those instructions
                if (s == NSUB - 1 && st + 1 < nstages) {
                    store_w((st + 1) & 1, wr[dn]);
                    if (chunk_ends) store_patch((chunk + 1) & 1, pr[dn % NPS], chunk + 1);
                }
                __builtin_amdgcn_sched_barrier(0);  // (the scheduler would otherwise sink the reads to their first use)
#pragma unroll
                for (int i = 0; i < TF; ++i)
#pragma unroll
                    for (int j = 0; j < TM; ++j)
                        if constexpr (I8)
                            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(cp_i32x4, fa[s % NFS][i].u),
                                                                                __builtin_bit_cast(cp_i32x4, fb[s % NFS][j].u), acc[i][j], 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s % NFS][i].v, fb[s % NFS][j].v, acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
        }
    }

    // ---- epilogue through this wave's own LDS region (the barrier above has released the buffers)
    if constexpr (I8) {
        // int8: pieces of 8 filters are 8 bytes; a lane's four filters are one 4-byte word
        typedef __attribute__((ext_vector_type(2))) unsigned cp_u32x2;
        const __amdgpu_buffer_rsrc_t rr8 = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<void *>(a.res ? a.res : a.y), 0, (int)((long)M * a.K), 0x00020000);
        uint2 *const ew2 = reinterpret_cast<uint2 *>(cp_lds) + wave * (TM * 32) * ROWC;
        const int mw0 = m0 + wave * TM * 32;
        constexpr int EPT = TM * 32 * (BN / 8) / 64;
        if (a.res) {
#pragma unroll
            for (int it = 0; it < EPT; ++it) {
                const int idx = lane + 64 * it;
                const int pix = idx / (BN / 8), cc = idx - pix * (BN / 8);
                const int m = mw0 + pix, f = f0 + cc * 8;
                const cp_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rr8, m < M && f < a.K ? m * a.K + f : CP_OOB, 0, 0);
                ew2[pix * ROWC + cc] = make_uint2(v[0], v[1]);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        const int4 *const ss = reinterpret_cast<const int4 *>(cp_lds + g.ss);
        const int lo = a.act == 1 ? q.zy : -128;
        const bool with_res = a.res != nullptr;
#pragma unroll
        for (int i = 0; i < TF; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int fl = i * 32 + 8 * jj + 4 * kh;  // first of this lane's four filters, within the tile
                const int4 mu = ss[fl >> 2], sh = ss[BN / 4 + (fl >> 2)], bi = ss[BN / 2 + (fl >> 2)];
                const int mu4[4] = {mu.x, mu.y, mu.z, mu.w}, sh4[4] = {sh.x, sh.y, sh.z, sh.w}, bi4[4] = {bi.x, bi.y, bi.z, bi.w};
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    unsigned *cell = reinterpret_cast<unsigned *>(ew2 + (j * 32 + l32) * ROWC) + (fl >> 2);
                    const unsigned r = with_res ? *cell : 0u;
                    unsigned packed = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        long long t = rr64((long long)(acc[i][j][4 * jj + e] + bi4[e]) * (long long)mu4[e], sh4[e]);
                        if (with_res) t += rr64((long long)((int)(int8_t)(r >> (8 * e)) - q.z_res) * (long long)q.m_res, q.sh_res);
                        t += q.zy;
                        const int v = (int)(t < lo ? lo : t > 127 ? 127 : t);
                        packed |= (unsigned)(v & 0xFF) << (8 * e);
                    }
                    *cell = packed;
                }
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const __amdgpu_buffer_rsrc_t ry8 = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, (int)((long)M * a.K), 0x00020000);
#pragma unroll
        for (int it = 0; it < EPT; ++it) {
            const int idx = lane + 64 * it;
            const int pix = idx / (BN / 8), cc = idx - pix * (BN / 8);
            const int m = mw0 + pix, f = f0 + cc * 8;
            const uint2 v = ew2[pix * ROWC + cc];
            __builtin_amdgcn_raw_buffer_store_b64(cp_u32x2{v.x, v.y}, ry8, m < M && f < a.K ? m * a.K + f : CP_OOB, 0, 0);
        }
        return;
    }
    if constexpr (!I8) {
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(a.res ? a.res : a.y), 0, (int)((long)M * a.K * 2), 0x00020000);
    uint4 *const ew = cp_lds + wave * (TM * 32) * ROWC;
    const int mw0 = m0 + wave * TM * 32;
    constexpr int ECELLS = TM * 32 * (BN / 8), EPT = ECELLS / 64;
    if (a.res) {
#pragma unroll
        for (int it = 0; it < EPT; ++it) {
            const int idx = lane + 64 * it;
            const int pix = idx / (BN / 8), cc = idx - pix * (BN / 8);
            const int m = mw0 + pix, f = f0 + cc * 8;
            const cp_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rr, m < M && f < a.K ? (m * a.K + f) * 2 : CP_OOB, 0, 0);
            ew[pix * ROWC + cc] = __builtin_bit_cast(uint4, v);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    // (the activation and the residual as compile-time switches: the loop below is straight-line code of a few
    // hundred instructions per variant, and only the variant in use is ever fetched)
    auto finish = [&](auto act_tag, auto res_tag) {
        constexpr int ACT = decltype(act_tag)::value;
        constexpr bool RES = decltype(res_tag)::value;
        uint2 *const e2 = reinterpret_cast<uint2 *>(ew);  // 8-byte pieces: pixel row = 2 ROWC of them
        const float4 *const ss = reinterpret_cast<const float4 *>(cp_lds + g.ss);
#pragma unroll
        for (int i = 0; i < TF; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int fl = i * 32 + 8 * jj + 4 * kh;  // first of this lane's four filters, within the tile
                const float4 sc = ss[fl >> 2], sh = ss[BN / 4 + (fl >> 2)];
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    uint2 *cell = e2 + (j * 32 + l32) * (2 * ROWC) + (fl >> 2);
                    float v[4] = {acc[i][j][4 * jj] * sc.x + sh.x, acc[i][j][4 * jj + 1] * sc.y + sh.y,
                                  acc[i][j][4 * jj + 2] * sc.z + sh.z, acc[i][j][4 * jj + 3] * sc.w + sh.w};
                    if (RES) {
                        const uint2 r = *cell;
                        v[0] += bf2f(r.x & 0xFFFFu), v[1] += bf2f(r.x >> 16), v[2] += bf2f(r.y & 0xFFFFu), v[3] += bf2f(r.y >> 16);
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (ACT == 1) v[e] = fmaxf(v[e], 0.0f);
                        if (ACT == 2) v[e] = v[e] * fminf(fmaxf(v[e] + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
                        if (ACT == 3) v[e] = fminf(fmaxf(v[e] + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
                    }
                    uint2 o;
                    o.x = pack_bf16x2(v[0], v[1]), o.y = pack_bf16x2(v[2], v[3]);
                    *cell = o;
                }
            }
    };
    {
        using std::integral_constant;
        const int code = (a.hsigmoid ? 3 : a.act) * 2 + (a.res ? 1 : 0);
        switch (code) {
            case 0: finish(integral_constant<int, 0>{}, integral_constant<bool, false>{}); break;
            case 1: finish(integral_constant<int, 0>{}, integral_constant<bool, true>{}); break;
            case 2: finish(integral_constant<int, 1>{}, integral_constant<bool, false>{}); break;
            case 3: finish(integral_constant<int, 1>{}, integral_constant<bool, true>{}); break;
            case 4: finish(integral_constant<int, 2>{}, integral_constant<bool, false>{}); break;
            case 5: finish(integral_constant<int, 2>{}, integral_constant<bool, true>{}); break;
            case 6: finish(integral_constant<int, 3>{}, integral_constant<bool, false>{}); break;
            default: finish(integral_constant<int, 3>{}, integral_constant<bool, true>{}); break;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const __amdgpu_buffer_rsrc_t ry =
        __builtin_amdgcn_make_buffer_rsrc(a.y, 0, (int)((long)M * a.K * 2), 0x00020000);
#pragma unroll
    for (int it = 0; it < EPT; ++it) {
        const int idx = lane + 64 * it;
        const int pix = idx / (BN / 8), cc = idx - pix * (BN / 8);
        const int m = mw0 + pix, f = f0 + cc * 8;
        const uint4 v = ew[pix * ROWC + cc];
        // (a store past the end of the buffer is dropped)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(cp_u32x4, v), ry, m < M && f < a.K ? (m * a.K + f) * 2 : CP_OOB, 0, 0);
    }
    }
}

// ------------------------------------------------------------------ host side

namespace {

struct PatchPlan {
    int npos_max;
};

// Largest number of frame positions any tile of BM consecutive output pixels spans.
int patch_positions(const ConvArgs &a, int BM) {
    struct Key {
        int v[9];
        bool operator==(const Key &o) const { return std::equal(v, v + 9, o.v); }
    };
    struct Hash {
        size_t operator()(const Key &k) const {
            size_t h = 1469598103934665603ull;
            for (int x : k.v) h = (h ^ (size_t)x) * 1099511628211ull;
            return h;
        }
    };
    thread_local std::unordered_map<Key, int, Hash> memo;
    const Key key{{a.B, a.H, a.W, a.P, a.Q, a.stride, a.R, a.pad, BM}};
    auto it = memo.find(key);
    if (it != memo.end()) return it->second;
    const int hp = a.H + 2 * a.pad, wp = a.W + 2 * a.pad;
    const long M = (long)a.B * a.P * a.Q;
    auto base = [&](long m) {
        const long q = m % a.Q, t = m / a.Q, p = t % a.P, n = t / a.P;
        return (n * hp + p * a.stride) * wp + q * a.stride;
    };
    long best = 0;
    for (long m0 = 0; m0 < M; m0 += BM) {
        const long ml = std::min(m0 + BM, M) - 1;
        best = std::max(best, base(ml) + (a.R - 1) * (wp + 1) - base(m0) + 1);
    }
    memo.emplace(key, (int)best);
    return (int)best;
}

template <int TF, int TM, int CK, int R, int MAXP, int MINB, int NW, bool I8 = false>
hipError_t launch_patch(const ConvArgs &a, hipStream_t s, const QuantArgs &q = QuantArgs{}) {
    constexpr int NT = 64 * NW, BN = 32 * TF, BM = 32 * NW * TM, NKG = CK / (I8 ? 16 : 8), WPS = BN + 4, ROWC = BN / 8 + 1;
    const int npos = patch_positions(a, BM);
    if ((long)npos * NKG > (long)MAXP * NT) return hipErrorNotSupported;
    // plane stride: congruent to 16 / NKG modulo 16 cells, so the NKG cells of a position fall into different banks
    int ps = npos;
    while (ps % 16 != 16 / NKG) ++ps;
    PatchGeom g;
    g.M = a.B * a.P * a.Q;
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_f = (a.K + BN - 1) / BN;
    g.hp = a.H + 2 * a.pad, g.wp = a.W + 2 * a.pad;
    g.ps = ps;
    const size_t cells = std::max<size_t>(2 * (size_t)NKG * ps + 2 * (size_t)R * NKG * WPS, (size_t)BM * ROWC);
    g.ss = (int)cells;
    g.dq = make_fastdiv(a.Q), g.dp = make_fastdiv(a.P), g.dwp = make_fastdiv(g.wp), g.dhp = make_fastdiv(g.hp);
    const size_t lds = (cells + 3 * BN / 4) * 16;
    if (lds > 160 * 1024) return hipErrorNotSupported;
    static bool attr_set = false;
    auto kern = conv_patch_kernel<TF, TM, CK, R, MAXP, MINB, NW, I8>;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int per_xcd = (g.tiles_m * g.tiles_f + 7) / 8;
    hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(NT), lds, s, a, g, q);
    return hipGetLastError();
}

template <int TM, int CK, int R, int MAXP, int MINB, int NW, bool I8 = false>
hipError_t launch_patch_tf(const ConvArgs &a, int tf, hipStream_t s, const QuantArgs &q = QuantArgs{}) {
    switch (tf) {
        case 2: return launch_patch<2, TM, CK, R, MAXP, MINB, NW, I8>(a, s, q);
        case 3: return launch_patch<3, TM, CK, R, MAXP, MINB, NW, I8>(a, s, q);
        default: return launch_patch<4, TM, CK, R, MAXP, MINB, NW, I8>(a, s, q);
    }
}

}  // namespace

// Returns hipErrorNotSupported (nothing launched) for shapes the patch kernel does not cover.
hipError_t launch_conv_patch(const ConvArgs &a, hipStream_t s) {
    if (a.in_f32 || a.out_f32 || (a.C & 7) || (a.K & 7) || a.K < 8) return hipErrorNotSupported;
    if (!(a.R == 1 || a.R == 3) || a.pad != (a.R - 1) / 2 || a.stride < 1 || a.stride > 2) return hipErrorNotSupported;
    if ((a.R == 1 && a.stride != 1) || a.Rmax != a.R) return hipErrorNotSupported;
    const long M = (long)a.B * a.P * a.Q;
    const long lim = (1l << 31) - 4096;
    if (M * a.K * 2 >= lim || (long)a.B * a.H * a.W * a.C * 2 >= lim) return hipErrorNotSupported;
    if ((long)a.B * (a.H + 2 * a.pad) * (a.W + 2 * a.pad) >= lim) return hipErrorNotSupported;
    if ((long)a.R * a.R * a.CG * a.Kpad * 16 >= lim) return hipErrorNotSupported;
    // filters per tile: the tile width (64, 96, 128) that wastes the fewest padded filters, the wider on a tie
    int tf = 4;
    long waste = -1;
    for (int t = 4; t >= 2; --t) {
        const long w = (long)((a.K + 32 * t - 1) / (32 * t)) * 32 * t - a.K;
        if (waste < 0 || w < waste) tf = t, waste = w;
    }
    if (a.R == 3) {
        if (a.stride == 2) return launch_patch_tf<1, 32, 3, 16, 1, 4>(a, tf, s);
        // 256-pixel tiles (eight waves of 32 pixels: two waves per SIMD get their LDS reads served at twice the
        // rate of one) while they still give most compute units a workgroup, else 128-pixel tiles of four waves
        const long tiles256 = ((M + 255) / 256) * ((a.K + 32 * tf - 1) / (32 * tf));
        if (tiles256 >= 160) return launch_patch_tf<1, 32, 3, 6, 1, 8>(a, tf, s);
        return launch_patch_tf<1, 32, 3, 12, 1, 4>(a, tf, s);
    }
    return launch_patch_tf<1, 64, 1, 4, 2, 4>(a, tf, s);
}

// The same for int8 codes (cells of 16 channels: chunks of 64 and 128 channels).  Returns hipErrorNotSupported
// (nothing launched) for shapes the patch kernel does not cover.
hipError_t launch_conv_patch_i8(const ConvArgs &a, const QuantArgs &q, hipStream_t s) {
    if ((a.C & 7) || a.C < 8 || (a.K & 7) || a.K < 8) return hipErrorNotSupported;
    if (!(a.R == 1 || a.R == 3) || a.pad != (a.R - 1) / 2 || a.stride < 1 || a.stride > 2) return hipErrorNotSupported;
    if ((a.R == 1 && a.stride != 1) || a.Rmax != a.R) return hipErrorNotSupported;
    const long M = (long)a.B * a.P * a.Q;
    const long lim = (1l << 31) - 4096;
    if (M * a.K >= lim || (long)a.B * a.H * a.W * a.C >= lim) return hipErrorNotSupported;
    if ((long)a.B * (a.H + 2 * a.pad) * (a.W + 2 * a.pad) >= lim) return hipErrorNotSupported;
    if ((long)a.R * a.R * a.CG * a.Kpad * 16 >= lim) return hipErrorNotSupported;
    int tf = 4;
    long waste = -1;
    for (int t = 4; t >= 2; --t) {
        const long w = (long)((a.K + 32 * t - 1) / (32 * t)) * 32 * t - a.K;
        if (waste < 0 || w < waste) tf = t, waste = w;
    }
    if (a.R == 3) {
        if (a.stride == 2) return launch_patch_tf<1, 64, 3, 16, 1, 4, true>(a, tf, s, q);
        const long tiles256 = ((M + 255) / 256) * ((a.K + 32 * tf - 1) / (32 * tf));
        if (tiles256 >= 160) return launch_patch_tf<1, 64, 3, 6, 1, 8, true>(a, tf, s, q);
        return launch_patch_tf<1, 64, 3, 12, 1, 4, true>(a, tf, s, q);
    }
    return launch_patch_tf<1, 128, 1, 4, 2, 4, true>(a, tf, s, q);
}

}  // namespace sushi
