// Device code shared by the stream kernel and the team kernels (see stream_kernel.h): the units that run one op of a
// query on a workgroup's share, and the team kernel itself as a template over the op set it contains.  Included by
// the translation units that instantiate a kernel (stream_kernel.hip, team_kernel_mobile.hip); bf16 mode.
#pragma once
#include "stream_kernel.h"

#include <algorithm>
#include <type_traits>

#include "device_common.h"
#include "model.h"

namespace sushi {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;
// Pointers read from a descriptor are generic to the compiler; weights are known to be in device memory.
typedef __attribute__((address_space(1))) u32x4_t global_u32x4;
typedef __attribute__((address_space(1))) uint16_t global_u16;
typedef __attribute__((address_space(1))) float global_f32;

// Cache policy bits of buffer accesses (gfx942/gfx950): sc0 = coherent within the XCD (skips the
// compute unit's vector L1, served by the XCD's L2), sc1 = coherent across the device's XCDs
// (stores write through the L2, loads do not hit stale lines there), both = system scope.
constexpr int AUX_PLAIN = 0, AUX_SC0 = 1, AUX_NT = 2, AUX_SC1 = 16, AUX_SYS = 17;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, long bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

template <int AUX>
__device__ __forceinline__ uint4 act_ld16(__amdgpu_buffer_rsrc_t r, int off) {
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, AUX);
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <int AUX>
__device__ __forceinline__ void act_st16(__amdgpu_buffer_rsrc_t r, int off, uint4 v) {
    const u32x4_t d = {v.x, v.y, v.z, v.w};
    __builtin_amdgcn_raw_buffer_store_b128(d, r, off, 0, AUX);
}

template <int AUX>
__device__ __forceinline__ void act_st8(__amdgpu_buffer_rsrc_t r, int off, uint2 v) {
    const u32x2_t d = {v.x, v.y};
    __builtin_amdgcn_raw_buffer_store_b64(d, r, off, 0, AUX);
}

__device__ __forceinline__ void unpack8(const uint4 a, float v[8]) {
    v[0] = bf2f(a.x & 0xFFFFu), v[1] = bf2f(a.x >> 16), v[2] = bf2f(a.y & 0xFFFFu), v[3] = bf2f(a.y >> 16);
    v[4] = bf2f(a.z & 0xFFFFu), v[5] = bf2f(a.z >> 16), v[6] = bf2f(a.w & 0xFFFFu), v[7] = bf2f(a.w >> 16);
}

__device__ __forceinline__ uint4 pack8(const float v[8]) {
    uint4 a;
    a.x = pack_bf16x2(v[0], v[1]), a.y = pack_bf16x2(v[2], v[3]);
    a.z = pack_bf16x2(v[4], v[5]), a.w = pack_bf16x2(v[6], v[7]);
    return a;
}

// ------------------------------------------------------------------ grid barrier
// sync[0] = abort, sync[16*(1+g)] = arrivals of group g, sync[16*40] = groups that arrived.
// Counters only grow: barrier number e (counted from the first launch on this area) is complete
// when the top counter reaches e * groups.  Returns false if the wait ran out or another
// workgroup gave up; the caller must leave the kernel then.
__device__ __forceinline__ bool grid_barrier(const StreamArgs &sa, unsigned long long e, int *lds_flag) {
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned nwg = gridDim.x;
        const unsigned g = blockIdx.x / BARRIER_GROUP;
        const unsigned gsize = min((unsigned)BARRIER_GROUP, nwg - g * BARRIER_GROUP);
        const unsigned ngroups = (nwg + BARRIER_GROUP - 1) / BARRIER_GROUP;
        unsigned long long *top = sa.sync + 16 * 40;
        const unsigned long long old =
            __hip_atomic_fetch_add(&sa.sync[16 * (1 + g)], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == e * gsize) __hip_atomic_fetch_add(top, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long target = e * ngroups;
        int spins = 0, good = 1;
        while (__hip_atomic_load(top, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (++spins > sa.spin_limit ||
                __hip_atomic_load(&sa.sync[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                __hip_atomic_store(&sa.sync[0], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(sa.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                good = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        *lds_flag = good;
    }
    __syncthreads();
    return *lds_flag != 0;
}

// ------------------------------------------------------------------ epilogue of one 16 x 16 tile

// LD / ST: cache policy of activation loads / stores; sys_out: the output is the caller's buffer and
// is written through to memory at system scope.
// Activation layout inside the stream and team kernels: [image][group of 8 channels][pixel][8 channels], one
// 16-byte cell per (group, pixel).  The 16 pixels x 4 channel groups a matrix-core operand takes are then four
// runs of 256 contiguous bytes (8 cache lines; 16 half-used lines if the channels of a pixel were contiguous,
// which costs a compute unit 2.5 times as long per load), and an output tile is written the same way.  With one
// pixel per image (pooled features, gates, logits) this is the plain [image][channel] order, for any channel
// count; with more pixels the channel count must be a multiple of 8.  The caller's input (3 channels) keeps its
// [image][pixel][channel] order and is read by the stem units only.
__device__ __forceinline__ int in_cell(const ConvArgs &a, int n, int cg, int h, int w) {  // byte offset
    return (((n * (a.C >> 3) + cg) * a.H + h) * a.W + w) * 16;
}
// Byte offset of the output cell (channel group cg, pixel pix of image n); the channel count is a multiple of 8.
__device__ __forceinline__ int out_cell(const ConvArgs &a, int n, int cg, int pix) {
    return ((n * (a.K >> 3) + cg) * (a.P * a.Q) + pix) * 16;
}
// Element offset of filter f of output pixel m (m counts pixels over the whole batch).
__device__ __forceinline__ long out_elem(const ConvArgs &a, int m, int f) {
    const int pq = a.P * a.Q;
    if (pq == 1) return (long)m * a.K + f;
    const int n = a.B == 1 ? 0 : m / pq, pix = m - n * pq;
    return (((long)n * (a.K >> 3) + (f >> 3)) * pq + pix) * 8 + (f & 7);
}
// The same in two parts for loops over tiles: out_elem = out_pixel_part(m) + out_filter_part(f).
__device__ __forceinline__ int out_pixel_part(const ConvArgs &a, int m) {
    const int pq = a.P * a.Q;
    if (pq == 1) return m * a.K;
    const int n = a.B == 1 ? 0 : m / pq, pix = m - n * pq;
    return (n * (a.K >> 3) * pq + pix) * 8;
}
__device__ __forceinline__ int out_filter_part(const ConvArgs &a, int f) {
    const int pq = a.P * a.Q;
    return pq == 1 ? f : (f >> 3) * pq * 8 + (f & 7);
}

// Scale and shift of the lane's four filters (and optionally the residual of one tile), fetched at
// the start of a unit so that their latency hides behind the reduction.
struct Epilogue {
    float sc[4], sh[4];
    u32x2_t res;
    bool have, have_res;
};

template <int LD>
__device__ __forceinline__ Epilogue fetch_epilogue(const ConvArgs &a, __amdgpu_buffer_rsrc_t rres, int fbase, int m,
                                                   int M, bool want_res) {
    Epilogue e;
    e.have = fbase + 4 <= a.K && (a.K & 3) == 0;
    e.have_res = false;
    e.res = u32x2_t{0u, 0u};
    if (e.have) {
        const float4 sh = *reinterpret_cast<const float4 *>(a.shift + fbase);
        float4 sc = make_float4(1.f, 1.f, 1.f, 1.f);
        if (a.scale) sc = *reinterpret_cast<const float4 *>(a.scale + fbase);
        e.sc[0] = sc.x, e.sc[1] = sc.y, e.sc[2] = sc.z, e.sc[3] = sc.w;
        e.sh[0] = sh.x, e.sh[1] = sh.y, e.sh[2] = sh.z, e.sh[3] = sh.w;
        if (want_res && a.res && m < M) {
            e.res = __builtin_amdgcn_raw_buffer_load_b64(rres, (int)(out_elem(a, m, fbase) * 2), 0, LD);
            e.have_res = true;
        }
    }
    return e;
}

template <int LD, int ST>
__device__ __forceinline__ void store_tile_coherent(const ConvArgs &a, __amdgpu_buffer_rsrc_t ry,
                                                    __amdgpu_buffer_rsrc_t rres, const f32x4_t acc, int fbase, int m,
                                                    int M, bool sys_out, const Epilogue &epi, bool epi_res) {
    if (fbase >= a.K || m >= M) return;
    const int nf = min(4, a.K - fbase);
    const bool vec = nf == 4 && (a.K & 3) == 0;
    const long o = out_elem(a, m, fbase);  // (the lane's filters never straddle a group of 8: fbase is a multiple of 4)
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float sc = epi.have ? epi.sc[i] : ((a.scale && i < nf) ? a.scale[fbase + i] : 1.0f);
        const float sh = epi.have ? epi.sh[i] : (i < nf ? a.shift[fbase + i] : 0.0f);
        v[i] = acc[i] * sc + sh;
    }
    if (a.res) {
        if (vec) {
            const u32x2_t r = (epi_res && epi.have_res) ? epi.res
                                                        : __builtin_amdgcn_raw_buffer_load_b64(rres, (int)(o * 2), 0, LD);
            v[0] += bf2f(r.x & 0xFFFFu), v[1] += bf2f(r.x >> 16), v[2] += bf2f(r.y & 0xFFFFu), v[3] += bf2f(r.y >> 16);
        } else {
            const uint16_t *rp = static_cast<const uint16_t *>(a.res) + o;
            for (int i = 0; i < nf; ++i)
                v[i] += bf2f(__hip_atomic_load(rp + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = activate(v[i], a.act, a.hsigmoid);
    if (a.out_f32) {
        if (vec) {
            const uint4 pk = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]),
                                        __float_as_uint(v[3]));
            if (sys_out)
                act_st16<AUX_SYS>(ry, (int)(o * 4), pk);
            else
                act_st16<ST>(ry, (int)(o * 4), pk);
        } else {
            float *yp = static_cast<float *>(a.y) + o;
            for (int i = 0; i < nf; ++i) __hip_atomic_store(yp + i, v[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    } else {
        if (vec) {
            const uint2 pk = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
            if (sys_out)
                act_st8<AUX_SYS>(ry, (int)(o * 2), pk);
            else
                act_st8<ST>(ry, (int)(o * 2), pk);
        } else {
            uint16_t *yp = static_cast<uint16_t *>(a.y) + o;
            for (int i = 0; i < nf; ++i)
                __hip_atomic_store(yp + i, (uint16_t)f2bf(v[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

// Straight-line epilogue for the common case (filters a multiple of 4, the lane's four filters inside
// K): ACT = 0 none, 1 ReLU, 2 h-swish, 3 h-sigmoid is a template parameter so that no per-element
// branch is left.
template <int ACT>
__device__ __forceinline__ float act_fast(float v) {
    if (ACT == 1) return fmaxf(v, 0.0f);
    if (ACT == 2) return v * fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
    if (ACT == 3) return fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f);
    return v;
}

template <int ACT, int ST>
__device__ __forceinline__ void store_tile_fast(const ConvArgs &a, __amdgpu_buffer_rsrc_t ry, const f32x4_t acc,
                                                const float4 sc, const float4 sh, const u32x2_t res, bool has_res,
                                                int fbase, int m, int M, bool sys_out) {
    if (fbase + 4 > a.K || m >= M) return;
    float v[4] = {acc[0] * sc.x + sh.x, acc[1] * sc.y + sh.y, acc[2] * sc.z + sh.z, acc[3] * sc.w + sh.w};
    if (has_res) v[0] += bf2f(res.x & 0xFFFFu), v[1] += bf2f(res.x >> 16), v[2] += bf2f(res.y & 0xFFFFu), v[3] += bf2f(res.y >> 16);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = act_fast<ACT>(v[i]);
    const int o = (int)out_elem(a, m, fbase);
    if (a.out_f32) {
        const uint4 pk = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
        if (sys_out)
            act_st16<AUX_SYS>(ry, o * 4, pk);
        else
            act_st16<ST>(ry, o * 4, pk);
    } else {
        const uint2 pk = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
        if (sys_out)
            act_st8<AUX_SYS>(ry, o * 2, pk);
        else
            act_st8<ST>(ry, o * 2, pk);
    }
}

// The same for a bf16 output inside the team's arena, without a branch: `offset` is the byte offset
// of the lane's four values or OOB_STORE, which the buffer store drops; `res` is zero when the op has
// no residual.
constexpr int OOB_STORE = 0x7FFFFFF0;
template <int ACT, int ST>
__device__ __forceinline__ void store_tile_bf16(__amdgpu_buffer_rsrc_t ry, const f32x4_t acc, const float4 sc,
                                                const float4 sh, const u32x2_t res, int offset) {
    float v[4] = {acc[0] * sc.x + sh.x, acc[1] * sc.y + sh.y, acc[2] * sc.z + sh.z, acc[3] * sc.w + sh.w};
    v[0] += bf2f(res.x & 0xFFFFu), v[1] += bf2f(res.x >> 16), v[2] += bf2f(res.y & 0xFFFFu), v[3] += bf2f(res.y >> 16);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = act_fast<ACT>(v[i]);
    act_st8<ST>(ry, offset, make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])));
}

// Calls f(std::integral_constant<int, ACT>) for the activation of the op.
template <typename F>
__device__ __forceinline__ void with_activation(const ConvArgs &a, F f) {
    const int mode = a.hsigmoid ? 3 : a.act;
    if (mode == 1)
        f(std::integral_constant<int, 1>{});
    else if (mode == 2)
        f(std::integral_constant<int, 2>{});
    else if (mode == 3)
        f(std::integral_constant<int, 3>{});
    else
        f(std::integral_constant<int, 0>{});
}

// ------------------------------------------------------------------ dense conv / FC on the matrix cores
// A unit = FT 16-filter tiles x PT 16-pixel tiles.  The workgroup's 8 waves form 8/wk slots of wk
// waves; a slot computes one unit, its waves splitting the reduction steps (tap x 32 channels).
// Partial sums meet in LDS in a fixed order.

// Residency (RES, team kernel only): an op that runs as one pixel group takes its filter tiles from
// a per-workgroup list instead: the tiles whose slab this workgroup holds in LDS, plus its share of
// the tiles nobody holds.  A resident tile reads the channel groups below cg_res from LDS and the
// rest (the part of the SubNet outside the cached SubGraph) from memory; the order of the
// reduction is the same either way, so the logits do not depend on what is cached.
struct ResView {
    const ResLayer *layer;    // null: the op has no resident tiles
    const ResEntry *entries;  // entries of this layer
    const char *store;        // this workgroup's LDS store
    int *list;                // LDS scratch for the unit list (>= 130 ints)
};

// Per-op tables in LDS, one entry per reduction step (tap, 32 channels) plus a null entry at index
// nsteps that every step past the end maps to:
//   steps[s] = {weight bytes to the step's first cell, activation bytes from tap (0, 0),
//               tap bit if the step is a full channel step, tap bit if it is the last of its tap}
//   slabs[s] = {byte offset of the step's first cell in a resident slab, first channel group}
struct StepTables {
    u32x4_t *steps;
    u32x2_t *slabs;
};
constexpr unsigned OOB_OFFSET = 0x7FFFFFF0u;  // past the end of any buffer: a buffer load there returns zeros

__device__ __forceinline__ void build_step_tables(const ConvArgs &a, int cg_stride, StepTables tb) {
    const int csteps = (a.C + 31) >> 5;
    const int nsteps = a.R * a.R * csteps;
    for (int st = threadIdx.x; st <= nsteps; st += STREAM_THREADS) {
        u32x4_t e = {OOB_OFFSET, 0u, 0u, 0u};
        u32x2_t r = {0u, OOB_OFFSET};
        if (st < nsteps) {
            const int tap = st / csteps, c = st - tap * csteps;
            const int dr = tap / a.R, ds = tap - dr * a.R;
            e.x = (unsigned)((tap * a.CG + c * 4) * a.Kpad * 16);
            e.y = (unsigned)(((dr * a.W + ds) + c * 4 * a.H * a.W) * 16);
            e.z = c == csteps - 1 ? 0u : 1u << tap;
            e.w = c == csteps - 1 ? 1u << tap : 0u;
            r.x = (unsigned)((tap * cg_stride + c * 4) * 256);
            r.y = (unsigned)(c * 4);
        }
        tb.steps[st] = e;
        tb.slabs[st] = r;
    }
    __syncthreads();
}

// x / d for 0 <= x < 2^22 from the reciprocal, corrected by one either way
__device__ __forceinline__ int div_small(int x, int d, float rcp) {
    int q = (int)((float)x * rcp);
    const int r = x - q * d;
    q += r >= d ? 1 : 0;
    q -= r < 0 ? 1 : 0;
    return q;
}

// The lane's activation cell of output pixel m: byte offset of (pixel, channel group kg) at tap (0, 0)
// and the mask whose bit t says that tap t falls inside the image (0 for m outside the output).
__device__ __forceinline__ void pixel_cell(const ConvArgs &a, int m, bool valid, int kg, float rcp_q, float rcp_pq,
                                           int *offset, unsigned *mask) {
    const int mm = valid ? m : 0;
    const int nn = div_small(mm, a.P * a.Q, rcp_pq);
    const int rem = mm - nn * a.P * a.Q;
    const int pp = div_small(rem, a.Q, rcp_q), qq = rem - pp * a.Q;
    const int h0 = pp * a.stride - a.pad, w0 = qq * a.stride - a.pad;
    *offset = in_cell(a, nn, kg, h0, w0);
    unsigned cols = 0, mk = 0;
    for (int ds = 0; ds < a.R; ++ds)
        if (w0 + ds >= 0 && w0 + ds < a.W) cols |= 1u << ds;
    for (int dr = 0; dr < a.R; ++dr)
        if (h0 + dr >= 0 && h0 + dr < a.H) mk |= cols << (dr * a.R);
    *mask = valid ? mk : 0u;
}

// The waves of a slot take the reduction steps ks, ks + wk, ...  Weight cells are requested DA steps
// ahead (they come from memory and take longest), activation cells DB steps ahead, both into
// register rings; the loop body is the same on every path, so the waits are exact.
// IN32: the input is a float32 vector per image (fully connected layers fed by pooled features, squeeze-excite
// or head vectors): a lane's eight channels are two 16-byte words, split on the fly into two bf16 operands
// (x = hi + lo) that are both multiplied with the step's weight fragment.
template <int FT, int PT, int LD, int ST, bool RES, bool IN32 = false>
__device__ __forceinline__ void conv_units(const DevOp &op, float *red, int rank, int nranks, const ResView rv,
                                           const StepTables tb) {
    constexpr int NT = FT * PT;   // 16 x 16 tiles of one unit (at most 4)
    constexpr int BW = IN32 ? 2 : 1;  // 16-byte words of one activation cell
    constexpr int DA = 8 / FT;    // weight steps in flight per wave
    constexpr int DB = 2;         // activation steps in flight per wave
    const ConvArgs &a = op.conv;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int wk = op.wk, slots = STREAM_WAVES / wk;
    const int slot = wave / wk, ks = wave - slot * wk;
    const int l16 = lane & 15, kg = lane >> 4;
    const int M = a.B * a.P * a.Q;
    const int taps = a.R * a.R;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (long)a.B * a.H * a.W * a.C * (IN32 ? 4 : 2));
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.w, (long)taps * a.CG * a.Kpad * 16);
    const long out_bytes = (long)M * a.K * (a.out_f32 ? 4 : 2);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, out_bytes);
    const __amdgpu_buffer_rsrc_t rres = make_rsrc(a.res ? a.res : a.y, (long)M * a.K * 2);
    const int csteps = (a.C + 31) >> 5;
    const int nsteps = taps * csteps;
    const int n_groups = (op.n_units + slots - 1) / slots;
    const int tail_active = ((a.C + 7) >> 3) - (csteps - 1) * 4;
    const int tail_stored = min(4, a.CG - (csteps - 1) * 4);
    const float rcp_q = 1.0f / (float)a.Q, rcp_pq = 1.0f / (float)(a.P * a.Q);
    const bool sys_out = op.out_patch != 0;

    // unit list of a resident op (FT <= 2): entries are (filter tile) | (resident ? 1 << 16 : 0); a
    // unit takes FT consecutive entries, which need not be neighbouring tiles
    constexpr bool CAN_LIST = RES && FT <= 2;
    const int ftiles = (a.K + 15) >> 4;
    const bool listed = CAN_LIST && rv.layer != nullptr && M <= 64;
    const int cg_res_op = listed ? __builtin_amdgcn_readfirstlane(rv.layer->cg_res) : 0;
    build_step_tables(a, listed ? __builtin_amdgcn_readfirstlane(rv.layer->cg_stride) : 0, tb);
    int n_listed = 0;
    if (listed) {
        if (wave == 0) {
            int count = 0;
            for (int base = 0; base < ftiles; base += 64) {
                const int f = base + lane;
                bool res = false, mine = false;
                if (f < ftiles) {
                    res = f < rv.layer->n_res && rv.entries[f].owner >= 0;
                    mine = res ? rv.entries[f].owner == rank : (f % nranks) == rank;
                }
                const unsigned long long mask = __ballot(mine);
                const int pos = __popcll(mask & ((1ull << lane) - 1ull));
                if (mine) rv.list[1 + count + pos] = f | (res ? 1 << 16 : 0);
                count += __popcll(mask);
            }
            if (lane == 0) rv.list[0] = count;
        }
        __syncthreads();
        n_listed = rv.list[0];
    }
    // a listed op: this workgroup's units are (FT entries of its list) x (pixel group)
    const int listed_units = ((n_listed + FT - 1) / FT) * op.n_p;
    const int first = listed ? 0 : rank, limit = listed ? (listed_units + slots - 1) / slots : n_groups,
              stride = listed ? 1 : nranks;
    for (int g = first; g < limit; g += stride) {
        // the unit's filter tiles
        int ftile[FT], cg_res[FT];
        bool fok[FT];
        const char *slab[FT];
        int pgroup = 0;
        if (listed) {
            const int unit = g * slots + slot;
            const int tgroup = unit / op.n_p;
            pgroup = unit - tgroup * op.n_p;
#pragma unroll
            for (int ft = 0; ft < FT; ++ft) {
                const int idx = tgroup * FT + ft;
                fok[ft] = unit < listed_units && idx < n_listed;
                const int entry = fok[ft] ? __builtin_amdgcn_readfirstlane(rv.list[1 + idx]) : 0;
                ftile[ft] = entry & 0xFFFF;
                const bool res = fok[ft] && (entry >> 16) != 0;
                cg_res[ft] = res ? cg_res_op : 0;
                slab[ft] = res ? rv.store + rv.entries[ftile[ft]].lds_off + (kg * 16 + l16) * 16 : nullptr;
            }
        } else {
            const int unit = g * slots + slot;
            const bool in_range = unit < op.n_units;
            const int fgroup = in_range ? unit / op.n_p : 0;
            pgroup = in_range ? unit - fgroup * op.n_p : 0;
#pragma unroll
            for (int ft = 0; ft < FT; ++ft) ftile[ft] = fgroup * FT + ft, fok[ft] = in_range, cg_res[ft] = 0, slab[ft] = nullptr;
        }
        const bool active = fok[0];
        const int m0 = pgroup * PT * 16;
        int b_lane[PT];
        unsigned mask_full[PT], mask_tail[PT];
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            const int m = m0 + pt * 16 + l16;
            pixel_cell(a, m, active && m < M, kg, rcp_q, rcp_pq, &b_lane[pt], &mask_full[pt]);
            mask_tail[pt] = kg < tail_active ? mask_full[pt] : 0u;
        }
        unsigned a_full[FT], a_tail[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
            const unsigned row = (unsigned)min(ftile[ft] * 16 + l16, a.Kpad - 1) * 16u;
            a_full[ft] = (unsigned)(kg * a.Kpad * 16) + row;
            a_tail[ft] = (unsigned)(min(kg, tail_stored - 1) * a.Kpad * 16) + row;
        }
        // scale/shift of every filter tile now, and the residual of the tile this wave finishes first
        const int t0 = wk == 1 ? 0 : ks;
        Epilogue epi[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
            epi[ft] = fetch_epilogue<LD>(a, rres, ftile[ft] * 16 + kg * 4, m0 + (t0 % PT) * 16 + l16, M,
                                         fok[ft] && t0 < NT && t0 / PT == ft);
        f32x4_t acc[FT][PT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) acc[ft][pt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        if (active) {
            const int per_wave = (nsteps - ks + wk - 1) / wk;  // steps ks, ks + wk, ... below nsteps
            u32x4_t ra[DA][FT], rb[DB][PT * BW];
            int ia = ks, ib = ks, ic = ks;  // step of the next weight request, activation request, product
            auto issue_a = [&](u32x4_t *q) {
                const int idx = min(ia, nsteps);
                ia += wk;
                const u32x4_t e = tb.steps[idx];
                unsigned cg_first = 0;
                if (CAN_LIST) cg_first = tb.slabs[idx].y;
#pragma unroll
                for (int ft = 0; ft < FT; ++ft) {
                    unsigned off = (e.w != 0u ? a_tail[ft] : a_full[ft]) + e.x;
                    // cells the slab holds are not fetched
                    if (CAN_LIST && cg_first + (unsigned)kg < (unsigned)cg_res[ft]) off = OOB_OFFSET;
                    q[ft] = __builtin_amdgcn_raw_buffer_load_b128(rw, (int)off, 0, 0);
                }
            };
            auto issue_b = [&](u32x4_t *q) {
                const int idx = min(ib, nsteps);
                ib += wk;
                const u32x4_t e = tb.steps[idx];
#pragma unroll
                for (int pt = 0; pt < PT; ++pt) {
                    const bool ok = ((mask_full[pt] & e.z) | (mask_tail[pt] & e.w)) != 0u;
                    const int off = ok ? (b_lane[pt] + (int)e.y) * BW : (int)OOB_OFFSET;
                    q[pt * BW] = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, LD);
                    if (IN32) q[pt * BW + BW - 1] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? off + 16 : (int)OOB_OFFSET, 0, LD);
                }
            };
#pragma unroll
            for (int d = 0; d < DA; ++d) issue_a(ra[d]);
#pragma unroll
            for (int d = 0; d < DB; ++d) issue_b(rb[d]);
            // Resident cells are read from the slab one step ahead of their product, so that the LDS round trip
            // (table entry, then the cell) lies behind the step before instead of in front of every product.
            uint4 sv[FT];
            bool sres[FT];
            auto fetch_slab = [&]() {
                const u32x2_t sl = tb.slabs[min(ic, nsteps)];
#pragma unroll
                for (int ft = 0; ft < FT; ++ft) {
                    sres[ft] = sl.y + (unsigned)kg < (unsigned)cg_res[ft];
                    if (sres[ft]) sv[ft] = *reinterpret_cast<const uint4 *>(slab[ft] + sl.x);
                }
            };
            if (CAN_LIST) fetch_slab();
            for (int i0 = 0; i0 < per_wave; i0 += DA) {
#pragma unroll
                for (int u = 0; u < DA; ++u) {
                    Frag fa[FT];
#pragma unroll
                    for (int ft = 0; ft < FT; ++ft) fa[ft].u = make_uint4(ra[u][ft].x, ra[u][ft].y, ra[u][ft].z, ra[u][ft].w);
                    if (CAN_LIST) {
#pragma unroll
                        for (int ft = 0; ft < FT; ++ft)
                            if (sres[ft]) fa[ft].u = sv[ft];
                    }
                    ic += wk;
                    if (CAN_LIST) fetch_slab();
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt) {
                        Frag fb;
                        const u32x4_t b = rb[u % DB][pt * BW];
                        fb.u = make_uint4(b.x, b.y, b.z, b.w);
                        if (IN32) {
                            const u32x4_t b2 = rb[u % DB][pt * BW + BW - 1];
                            Frag lo;
                            split_f32x8(fb.u, make_uint4(b2.x, b2.y, b2.z, b2.w), &fb.u, &lo.u);
#pragma unroll
                            for (int ft = 0; ft < FT; ++ft)
                                acc[ft][pt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[ft].v, lo.v, acc[ft][pt], 0, 0, 0);
                        }
#pragma unroll
                        for (int ft = 0; ft < FT; ++ft)
                            acc[ft][pt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[ft].v, fb.v, acc[ft][pt], 0, 0, 0);
                    }
                    issue_a(ra[u]);
                    issue_b(rb[u % DB]);
                }
            }
        }
        if (wk == 1) {
            if (active)
#pragma unroll
                for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt)
                        if (fok[ft])
                            store_tile_coherent<LD, ST>(a, ry, rres, acc[ft][pt], ftile[ft] * 16 + kg * 4, m0 + pt * 16 + l16,
                                                        M, sys_out, epi[ft], ft == 0 && pt == 0);
            continue;
        }
        if constexpr (NT <= 4) {
            // red[wave][NT][4][64]
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) red[((wave * NT + ft * PT + pt) * 4 + i) * 64 + lane] = acc[ft][pt][i];
            __syncthreads();
            if (active)
                for (int t = ks; t < NT; t += wk) {
                    f32x4_t s = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    for (int k = 0; k < wk; ++k)
#pragma unroll
                        for (int i = 0; i < 4; ++i) s[i] += red[(((slot * wk + k) * NT + t) * 4 + i) * 64 + lane];
                    const int ft = t / PT, pt = t - ft * PT;
                    Epilogue e = epi[0];
                    int tile = ftile[0];
                    bool ok = fok[0];
#pragma unroll
                    for (int k = 1; k < FT; ++k)
                        if (ft == k) e = epi[k], tile = ftile[k], ok = fok[k];
                    if (ok)
                        store_tile_coherent<LD, ST>(a, ry, rres, s, tile * 16 + kg * 4, m0 + pt * 16 + l16, M, sys_out, e,
                                                    t == ks);
                }
            __syncthreads();
        } else {
            // the scratch holds one filter tile's partial sums at a time: red[wave][PT][4][64]
#pragma unroll
            for (int ft = 0; ft < FT; ++ft) {
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) red[((wave * PT + pt) * 4 + i) * 64 + lane] = acc[ft][pt][i];
                __syncthreads();
                if (fok[ft])
                    for (int pt = ks; pt < PT; pt += wk) {
                        f32x4_t s = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        for (int k = 0; k < wk; ++k)
#pragma unroll
                            for (int i = 0; i < 4; ++i) s[i] += red[(((slot * wk + k) * PT + pt) * 4 + i) * 64 + lane];
                        store_tile_coherent<LD, ST>(a, ry, rres, s, ftile[ft] * 16 + kg * 4, m0 + pt * 16 + l16, M, sys_out,
                                                    epi[ft], false);
                    }
                __syncthreads();
            }
        }
    }
}

// ------------------------------------------------------------------ dense conv with many pixels: weight tile shared in LDS
// A unit = AT 16-filter tiles x (8 * BT) 16-pixel tiles.  The eight waves split the pixels; every
// wave multiplies its BT pixel tiles with all AT filter tiles, so an activation fragment (loaded
// straight from memory into the lane layout of the MFMA operand) is used AT times and the weight
// tile of a reduction step (one tap, 32 channels: AT KiB) is fetched once per workgroup, by waves
// 0 .. AT-1, and handed to the others through a two-stage LDS buffer.  The reduction advances in
// intervals of tile_ks(BT) steps with one workgroup barrier per interval; loads run TILE_SETS intervals
// ahead of the MFMAs in register sets.
// Activation cells outside the image, beyond the active channels or beyond the last pixel are
// requested at an offset past the end of the buffer, which a buffer load answers with zeros.
// Reduction steps per interval: two, or one where a wave holds four pixel tiles (the register sets
// of the activations are what limits the shape).
__host__ __device__ constexpr int tile_ks(int bt) { return bt >= 4 ? 1 : 2; }
constexpr int TILE_SETS = 3;  // register sets = intervals in flight

template <int AT, int BT, int LD, int ST>
__device__ __forceinline__ void conv_tile_units(const DevOp &op, u32x4_t *stage, int rank, int nranks) {
    constexpr int KS = tile_ks(BT);
    static_assert(TILE_SETS == 3, "the interval loop is written out for three register sets");
    constexpr int OOB = 0x7FFFFFF0;
    const ConvArgs &a = op.conv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, kg = lane >> 4;
    const int M = a.B * a.P * a.Q;
    const int taps = a.R * a.R;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (long)a.B * a.H * a.W * a.C * 2);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.w, (long)taps * a.CG * a.Kpad * 16);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (long)M * a.K * (a.out_f32 ? 4 : 2));
    const __amdgpu_buffer_rsrc_t rres = make_rsrc(a.res ? a.res : a.y, (long)M * a.K * 2);
    const int csteps = (a.C + 31) >> 5;
    const int nsteps = taps * csteps;
    const bool sys_out = op.out_patch != 0;
    // every wave passes its weight cell on to LDS: the waves beyond AT hold the last tile once more and
    // write it to the same place, so no wave branches around loads or stores (a branch there makes the
    // compiler move loads into it, and the counted waits then fall back to waiting for every load)
    const int st_cell = min(wave, AT - 1) * 64 + lane;
    // channel groups of the last 32-channel step of a tap: active ones (activations) and stored ones (weights)
    const int tail_active = ((a.C + 7) >> 3) - (csteps - 1) * 4;
    const int tail_stored = min(4, a.CG - (csteps - 1) * 4);
    // LDS behind the two weight stages: scale and shift of the unit's filters, then one entry per
    // reduction step {weight bytes to the step's first cell, activation bytes from tap (0, 0), tap bit
    // for a full channel step, tap bit for the last channel step of a tap}; steps past the end (the
    // loop runs whole rounds of intervals) have no tap bit and so multiply zeros
    float *epi_lds = reinterpret_cast<float *>(stage + 2 * KS * AT * 64);
    u32x4_t *table = stage + 2 * KS * AT * 64 + AT * 8;
    const int nsteps_pad = (nsteps + 3 * KS - 1) / (3 * KS) * (3 * KS);
    for (int st = tid; st < nsteps_pad + 3 * KS; st += STREAM_THREADS) {  // (the loads run one round past the end)
        const int tap = st / csteps, c = st - tap * csteps;
        const int dr = tap / a.R, ds = tap - dr * a.R;
        u32x4_t e = {0u, 0u, 0u, 0u};
        if (st < nsteps) {
            e.x = (unsigned)((tap * a.CG + c * 4) * a.Kpad * 16);
            e.y = (unsigned)(((dr * a.W + ds) + c * 4 * a.H * a.W) * 16);
            e.z = c == csteps - 1 ? 0u : 1u << tap;
            e.w = c == csteps - 1 ? 1u << tap : 0u;
        }
        table[st] = e;
    }
    __syncthreads();
    const float rcp_q = 1.0f / (float)a.Q, rcp_pq = 1.0f / (float)(a.P * a.Q);
    // x / d for 0 <= x < 2^22 from the reciprocal, corrected by one either way
    auto div_small = [](int x, int d, float rcp) {
        int q = (int)((float)x * rcp);
        const int r = x - q * d;
        q += r >= d ? 1 : 0;
        q -= r < 0 ? 1 : 0;
        return q;
    };

    for (int unit = rank; unit < op.n_units; unit += nranks) {
        const int fgroup = unit / op.n_p, pgroup = unit - fgroup * op.n_p;
        const int f0 = fgroup * AT * 16, m0 = (pgroup * STREAM_WAVES + wave) * BT * 16;
        // epilogue constants of filter f0 + tid: requested now, parked in LDS after the reduction
        float e_sc = 1.0f, e_sh = 0.0f;
        if (tid < AT * 16 && f0 + tid < a.K) {
            if (a.scale) e_sc = ((const global_f32 *)a.scale)[f0 + tid];
            e_sh = ((const global_f32 *)a.shift)[f0 + tid];
        }
        // Activation cell of this lane: byte offset of (pixel, channel group kg) at tap (0, 0); bit t
        // of the mask says whether tap t falls inside the image.  The mask of the last channel step
        // also drops the channel groups beyond the active channels.
        int b_lane[BT];
        unsigned mask_full[BT], mask_tail[BT];
#pragma unroll
        for (int j = 0; j < BT; ++j) {
            const int m = m0 + j * 16 + l16;
            const bool pv = m < M;
            const int mm = pv ? m : 0;
            const int nn = div_small(mm, a.P * a.Q, rcp_pq);
            const int rem = mm - nn * a.P * a.Q;
            const int pp = div_small(rem, a.Q, rcp_q), qq = rem - pp * a.Q;
            const int h0 = pp * a.stride - a.pad, w0 = qq * a.stride - a.pad;
            b_lane[j] = in_cell(a, nn, kg, h0, w0);
            unsigned cols = 0, mk = 0;
            for (int ds = 0; ds < a.R; ++ds)
                if (w0 + ds >= 0 && w0 + ds < a.W) cols |= 1u << ds;
            for (int dr = 0; dr < a.R; ++dr)
                if (h0 + dr >= 0 && h0 + dr < a.H) mk |= cols << (dr * a.R);
            mk = pv ? mk : 0u;
            mask_full[j] = mk;
            mask_tail[j] = kg < tail_active ? mk : 0u;
        }
        // Weight cell of this lane in the lane layout of the operand.  Every wave issues the load
        // (waves beyond AT repeat the last tile and drop the result): the load sequence is then the
        // same on every path through the loop, which lets the compiler wait for exactly the load a
        // step needs instead of for all of them.
        const int a_row = min(f0 + min(wave, AT - 1) * 16 + l16, a.Kpad - 1) * 16;
        const int a_full = kg * a.Kpad * 16 + a_row;
        const int a_tail = min(kg, tail_stored - 1) * a.Kpad * 16 + a_row;

        // register sets: weight cell and activation cells of the KS steps of an interval in flight
        u32x4_t ra0[KS], ra1[KS], ra2[KS];
        u32x4_t rb0[KS][BT], rb1[KS][BT], rb2[KS][BT];
        int i_step = 0;  // reduction step the next issue() fetches
        auto issue = [&](u32x4_t &qa, u32x4_t *qb) {
            const u32x4_t e = table[i_step++];
            qa = __builtin_amdgcn_raw_buffer_load_b128(rw, (e.w != 0u ? a_tail : a_full) + (int)e.x, 0, 0);
#pragma unroll
            for (int j = 0; j < BT; ++j) {
                const bool ok = ((mask_full[j] & e.z) | (mask_tail[j] & e.w)) != 0u;
                qb[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? b_lane[j] + (int)e.y : OOB, 0, LD);
            }
        };

        f32x4_t acc[AT][BT];
#pragma unroll
        for (int i = 0; i < AT; ++i)
#pragma unroll
            for (int j = 0; j < BT; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        // One interval: multiply the weight stage `par` with the activations of set `b`, pass the
        // next interval's weight cells (`a_next`, requested two intervals ago) to the other stage,
        // and reuse the registers of this interval (`a_free`, `b`) for the loads three intervals on.
        auto run_interval = [&](int par, u32x4_t *a_free, const u32x4_t *a_next, u32x4_t (*b)[BT]) {
            const u32x4_t *cur = stage + par * (KS * AT * 64);
            u32x4_t *nxt = stage + (par ^ 1) * (KS * AT * 64);
#pragma unroll
            for (int k = 0; k < KS; ++k) {
                u32x4_t fa[AT];
#pragma unroll
                for (int i = 0; i < AT; ++i) fa[i] = cur[(k * AT + i) * 64 + lane];
#pragma unroll
                for (int j = 0; j < BT; ++j) {
                    Frag fb;
                    fb.u = make_uint4(b[k][j].x, b[k][j].y, b[k][j].z, b[k][j].w);
#pragma unroll
                    for (int i = 0; i < AT; ++i) {
                        Frag f;
                        f.u = make_uint4(fa[i].x, fa[i].y, fa[i].z, fa[i].w);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.v, fb.v, acc[i][j], 0, 0, 0);
                    }
                }
            }
            // (the hand-over comes after the products: the wait for the next interval's weight cells then
            // falls behind this interval's matrix-core work instead of in front of it)
#pragma unroll
            for (int k = 0; k < KS; ++k) nxt[k * AT * 64 + st_cell] = a_next[k];
#pragma unroll
            for (int k = 0; k < KS; ++k) issue(a_free[k], b[k]);
            __syncthreads();
        };

#pragma unroll
        for (int k = 0; k < KS; ++k) issue(ra0[k], rb0[k]);
#pragma unroll
        for (int k = 0; k < KS; ++k) issue(ra1[k], rb1[k]);
#pragma unroll
        for (int k = 0; k < KS; ++k) issue(ra2[k], rb2[k]);
#pragma unroll
        for (int k = 0; k < KS; ++k) stage[k * AT * 64 + st_cell] = ra0[k];
        __syncthreads();
        // three intervals per round: the stage parity of a round's first interval alternates
        int par = 0;
        for (int s0 = 0; s0 < nsteps; s0 += 3 * KS) {
            run_interval(par, ra0, ra1, rb0);
            run_interval(par ^ 1, ra1, ra2, rb1);
            run_interval(par, ra2, ra0, rb2);
            par ^= 1;
        }
        // residuals are requested before the first store, so that they overlap instead of queueing
        // behind one another
        u32x2_t resid[AT][BT];
        const bool vec_k = (a.K & 3) == 0;
#pragma unroll
        for (int i = 0; i < AT; ++i) {
            const int fbase = f0 + i * 16 + kg * 4;
#pragma unroll
            for (int j = 0; j < BT; ++j) {
                const int m = m0 + j * 16 + l16;
                const bool want = a.res && vec_k && fbase + 4 <= a.K && m < M;  // else: past the end, reads zeros
                resid[i][j] = __builtin_amdgcn_raw_buffer_load_b64(rres, want ? (out_pixel_part(a, m) + out_filter_part(a, fbase)) * 2 : OOB_STORE, 0, LD);
            }
        }
        if (tid < AT * 16) epi_lds[tid] = e_sc, epi_lds[AT * 16 + tid] = e_sh;
        __syncthreads();
        if (vec_k && !a.out_f32 && !sys_out) {
            with_activation(a, [&](auto tag) {
                constexpr int ACT = decltype(tag)::value;
#pragma unroll
                for (int i = 0; i < AT; ++i) {
                    const int fbase = f0 + i * 16 + kg * 4;
                    const float4 sc = *reinterpret_cast<const float4 *>(epi_lds + i * 16 + kg * 4);
                    const float4 sh = *reinterpret_cast<const float4 *>(epi_lds + AT * 16 + i * 16 + kg * 4);
#pragma unroll
                    for (int j = 0; j < BT; ++j) {
                        const int m = m0 + j * 16 + l16;
                        const bool ok = fbase + 4 <= a.K && m < M;
                        store_tile_bf16<ACT, ST>(ry, acc[i][j], sc, sh, resid[i][j], ok ? (out_pixel_part(a, m) + out_filter_part(a, fbase)) * 2 : OOB_STORE);
                    }
                }
            });
        } else if (vec_k) {
            with_activation(a, [&](auto tag) {
                constexpr int ACT = decltype(tag)::value;
#pragma unroll
                for (int i = 0; i < AT; ++i) {
                    const int fbase = f0 + i * 16 + kg * 4;
                    const float4 sc = *reinterpret_cast<const float4 *>(epi_lds + i * 16 + kg * 4);
                    const float4 sh = *reinterpret_cast<const float4 *>(epi_lds + AT * 16 + i * 16 + kg * 4);
#pragma unroll
                    for (int j = 0; j < BT; ++j)
                        store_tile_fast<ACT, ST>(a, ry, acc[i][j], sc, sh, resid[i][j], a.res != nullptr, fbase,
                                                 m0 + j * 16 + l16, M, sys_out);
                }
            });
        } else {
#pragma unroll
            for (int i = 0; i < AT; ++i) {
                const int fbase = f0 + i * 16 + kg * 4;
                Epilogue e;
                e.have = false, e.have_res = false, e.res = u32x2_t{0u, 0u};
#pragma unroll
                for (int j = 0; j < BT; ++j)
                    store_tile_coherent<LD, ST>(a, ry, rres, acc[i][j], fbase, m0 + j * 16 + l16, M, sys_out, e, false);
            }
        }
        // (the next unit passes several barriers before it writes the constants in LDS again)
    }
}

// ------------------------------------------------------------------ dense conv with many pixels and few weights
// Units as in conv_tile_units (AT filter tiles x 8 * BT pixel tiles), for layers whose weights for one
// filter group fit in LDS whole (short reductions: the 1x1 convs of the early stages, the second and
// third stem conv).  A workgroup loads the filter group's weights for every reduction step once, in
// operand order, and keeps them while it works through the group's pixel blocks; inside a unit the
// waves run without any barrier, each with its own ring of activation cells ARES_D steps ahead.
constexpr int ARES_D = 4;

template <int AT, int BT, int LD, int ST>
__device__ __forceinline__ void conv_ares_units(const DevOp &op, u32x4_t *lds, int rank, int nranks) {
    constexpr int D = ARES_D;
    const ConvArgs &a = op.conv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, kg = lane >> 4;
    const int M = a.B * a.P * a.Q;
    const int taps = a.R * a.R;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (long)a.B * a.H * a.W * a.C * 2);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.w, (long)taps * a.CG * a.Kpad * 16);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (long)M * a.K * (a.out_f32 ? 4 : 2));
    const __amdgpu_buffer_rsrc_t rres = make_rsrc(a.res ? a.res : a.y, (long)M * a.K * 2);
    const int csteps = (a.C + 31) >> 5;
    const int nsteps = taps * csteps;
    const int nsteps_pad = (nsteps + D - 1) / D * D;
    const bool sys_out = op.out_patch != 0;
    const int tail_active = ((a.C + 7) >> 3) - (csteps - 1) * 4;
    const int tail_stored = min(4, a.CG - (csteps - 1) * 4);
    // LDS: [step][AT][64] weight cells, scale and shift of the group's filters, one table entry per step
    u32x4_t *wts = lds;
    float *epi_lds = reinterpret_cast<float *>(lds + nsteps * AT * 64);
    u32x4_t *table = lds + nsteps * AT * 64 + AT * 8;
    for (int st = tid; st < nsteps_pad; st += STREAM_THREADS) {
        const int tap = st / csteps, c = st - tap * csteps;
        const int dr = tap / a.R, ds = tap - dr * a.R;
        u32x4_t e = {0u, 0u, 0u, 0u};
        if (st < nsteps) {
            e.x = (unsigned)((tap * a.CG + c * 4) * a.Kpad * 16);
            e.y = (unsigned)(((dr * a.W + ds) + c * 4 * a.H * a.W) * 16);
            e.z = c == csteps - 1 ? 0u : 1u << tap;
            e.w = c == csteps - 1 ? 1u << tap : 0u;
        }
        table[st] = e;
    }
    __syncthreads();
    const float rcp_q = 1.0f / (float)a.Q, rcp_pq = 1.0f / (float)(a.P * a.Q);
    const bool vec_k = (a.K & 3) == 0;

    // Lane state of the unit whose activation cells are being requested, the ring of cells in flight and
    // the step the next request fetches.  The requests run ahead across units: while a unit's last D steps
    // are multiplied, the first D steps of the workgroup's next unit are requested, so they arrive during
    // this unit's epilogue (with one to three steps per unit the load round trip would otherwise be paid
    // once per unit).  A unit past the last one asks for nothing.
    int b_lane[BT];
    unsigned mask_full[BT], mask_tail[BT];
    auto aim_at = [&](int unit) {
        const bool live = unit < op.n_units;
        const int pgroup = unit % op.n_p;
        const int m0 = (pgroup * STREAM_WAVES + wave) * BT * 16;
#pragma unroll
        for (int j = 0; j < BT; ++j) {
            const int m = m0 + j * 16 + l16;
            pixel_cell(a, m, live && m < M, kg, rcp_q, rcp_pq, &b_lane[j], &mask_full[j]);
            mask_tail[j] = kg < tail_active ? mask_full[j] : 0u;
        }
    };
    u32x4_t rb[D][BT];
    int i_step = 0;
    auto issue = [&](u32x4_t *qb) {
        const u32x4_t e = table[min(i_step, nsteps_pad - 1)];
        ++i_step;
#pragma unroll
        for (int j = 0; j < BT; ++j) {
            const bool ok = ((mask_full[j] & e.z) | (mask_tail[j] & e.w)) != 0u;
            qb[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? b_lane[j] + (int)e.y : (int)OOB_OFFSET, 0, LD);
        }
    };
    aim_at(rank);
#pragma unroll
    for (int d = 0; d < D; ++d) issue(rb[d]);

    int loaded_group = -1;
    for (int unit = rank; unit < op.n_units; unit += nranks) {
        const int fgroup = unit / op.n_p, pgroup = unit - fgroup * op.n_p;
        const int f0 = fgroup * AT * 16, m0 = (pgroup * STREAM_WAVES + wave) * BT * 16;
        if (fgroup != loaded_group) {
            // (re)load the filter group: cell (step, tile, lane) in the lane layout of the MFMA operand
            loaded_group = fgroup;
            __syncthreads();
            const int cells = nsteps * AT * 64;
            for (int base = tid; base < cells; base += 4 * STREAM_THREADS) {
                u32x4_t v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = min(base + u * STREAM_THREADS, cells - 1);
                    const int st = i / (AT * 64), rem = i - st * (AT * 64);
                    const int tile = rem >> 6, ln = rem & 63;
                    const u32x4_t e = table[st];
                    const int kgx = e.w != 0u ? min(ln >> 4, tail_stored - 1) : (ln >> 4);
                    const int row = min(f0 + tile * 16 + (ln & 15), a.Kpad - 1);
                    v[u] = __builtin_amdgcn_raw_buffer_load_b128(rw, (int)e.x + (kgx * a.Kpad + row) * 16, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = base + u * STREAM_THREADS;
                    if (i < cells) wts[i] = v[u];
                }
            }
            if (tid < AT * 16) {
                float e_sc = 1.0f, e_sh = 0.0f;
                if (f0 + tid < a.K) {
                    if (a.scale) e_sc = ((const global_f32 *)a.scale)[f0 + tid];
                    e_sh = ((const global_f32 *)a.shift)[f0 + tid];
                }
                epi_lds[tid] = e_sc, epi_lds[AT * 16 + tid] = e_sh;
            }
            __syncthreads();
        }
        // residuals early: their latency hides behind the reduction
        u32x2_t resid[AT][BT];
#pragma unroll
        for (int i = 0; i < AT; ++i) {
            const int fbase = f0 + i * 16 + kg * 4;
#pragma unroll
            for (int j = 0; j < BT; ++j) {
                const int m = m0 + j * 16 + l16;
                const bool want = a.res && vec_k && fbase + 4 <= a.K && m < M;
                resid[i][j] = __builtin_amdgcn_raw_buffer_load_b64(rres, want ? (out_pixel_part(a, m) + out_filter_part(a, fbase)) * 2 : OOB_STORE, 0, LD);
            }
        }
        f32x4_t acc[AT][BT];
#pragma unroll
        for (int i = 0; i < AT; ++i)
#pragma unroll
            for (int j = 0; j < BT; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int s0 = 0; s0 < nsteps_pad; s0 += D) {
            if (s0 + D >= nsteps_pad) {  // the requests of the last D steps go to the next unit
                aim_at(unit + nranks);
                i_step = 0;
            }
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const int step = min(s0 + d, nsteps - 1);  // steps past the end multiply zeros with the last weights
                u32x4_t fa[AT];
#pragma unroll
                for (int i = 0; i < AT; ++i) fa[i] = wts[(step * AT + i) * 64 + lane];
#pragma unroll
                for (int j = 0; j < BT; ++j) {
                    Frag fb;
                    fb.u = make_uint4(rb[d][j].x, rb[d][j].y, rb[d][j].z, rb[d][j].w);
#pragma unroll
                    for (int i = 0; i < AT; ++i) {
                        Frag f;
                        f.u = make_uint4(fa[i].x, fa[i].y, fa[i].z, fa[i].w);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.v, fb.v, acc[i][j], 0, 0, 0);
                    }
                }
                issue(rb[d]);
            }
        }
        if (vec_k && !a.out_f32 && !sys_out) {
            with_activation(a, [&](auto tag) {
                constexpr int ACT = decltype(tag)::value;
#pragma unroll
                for (int i = 0; i < AT; ++i) {
                    const int fbase = f0 + i * 16 + kg * 4;
                    const float4 sc = *reinterpret_cast<const float4 *>(epi_lds + i * 16 + kg * 4);
                    const float4 sh = *reinterpret_cast<const float4 *>(epi_lds + AT * 16 + i * 16 + kg * 4);
#pragma unroll
                    for (int j = 0; j < BT; ++j) {
                        const int m = m0 + j * 16 + l16;
                        const bool ok = fbase + 4 <= a.K && m < M;
                        store_tile_bf16<ACT, ST>(ry, acc[i][j], sc, sh, resid[i][j], ok ? (out_pixel_part(a, m) + out_filter_part(a, fbase)) * 2 : OOB_STORE);
                    }
                }
            });
        } else {
            for (int i = 0; i < AT; ++i) {
                const int fbase = f0 + i * 16 + kg * 4;
                Epilogue e;
                e.have = false, e.have_res = false, e.res = u32x2_t{0u, 0u};
                for (int j = 0; j < BT; ++j)
                    store_tile_coherent<LD, ST>(a, ry, rres, acc[i][j], fbase, m0 + j * 16 + l16, M, sys_out, e, false);
            }
        }
    }
}

// ------------------------------------------------------------------ vector-ALU layers, grid-strided

// Dense conv with a channel count that is not a multiple of 8 (the 3-channel stem): one thread per
// output pixel x 4 filters.  The input is the caller's buffer (complete before the launch).
template <int ST>
__device__ __forceinline__ void conv_direct_units(const ConvArgs &a, int rank, int nranks) {
    const int groups = (a.K + 3) >> 2;
    const long total = (long)a.B * a.P * a.Q * groups;
    const uint16_t *x = static_cast<const uint16_t *>(a.x);
    const uint16_t *w = static_cast<const uint16_t *>(a.w);
    const int cgs = (a.C + 7) >> 3;
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (long)a.B * a.P * a.Q * a.K * 2);
    for (long idx = (long)rank * STREAM_THREADS + threadIdx.x; idx < total; idx += (long)nranks * STREAM_THREADS) {
        const int fg = (int)(idx % groups);
        const long m = idx / groups;
        const int qq = (int)(m % a.Q), pp = (int)((m / a.Q) % a.P), n = (int)(m / ((long)a.Q * a.P));
        const int fb = fg * 4;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int tap = 0; tap < a.R * a.R; ++tap) {
            const int h = pp * a.stride - a.pad + tap / a.R, v = qq * a.stride - a.pad + tap % a.R;
            if (h < 0 || h >= a.H || v < 0 || v >= a.W) continue;
            const uint16_t *xp = x + (((long)n * a.H + h) * a.W + v) * a.C;
            for (int cg = 0; cg < cgs; ++cg) {
                float xv[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int c = cg * 8 + j;
                    xv[j] = 0.f;
                    if (c < a.C) xv[j] = bf2f(__hip_atomic_load(xp + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM));
                }
                const uint16_t *wp = w + (((long)tap * a.CG + cg) * a.Kpad + fb) * 8;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (fb + i < a.Kpad) {
                        float wv[8];
                        load8(wp + i * 8, wv);
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[i] = fmaf(wv[j], xv[j], acc[i]);
                    }
            }
        }
        const long obase = out_elem(a, (int)m, fb);
        float v4[4];
        const int nf = min(4, a.K - fb);
        for (int i = 0; i < 4; ++i)
            v4[i] = i < nf ? activate(acc[i] * (a.scale ? a.scale[fb + i] : 1.0f) + a.shift[fb + i], a.act, a.hsigmoid)
                           : 0.f;
        uint16_t *yp = static_cast<uint16_t *>(a.y) + obase;
        if (nf == 4 && (a.K & 3) == 0) {
            act_st8<ST>(ry, (int)(obase * 2),
                        make_uint2(pack_bf16x2(v4[0], v4[1]), pack_bf16x2(v4[2], v4[3])));
        } else {
            for (int i = 0; i < nf; ++i)
                __hip_atomic_store(yp + i, (uint16_t)f2bf(v4[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// The stem on the matrix cores (wk == -1): a dense conv whose few input channels make the whole
// patch (taps x channels, at most 64 values) one or two reduction steps.  A unit is a band of
// op.pt output rows of one image: the workgroup copies the input rows the band needs into LDS with
// wide loads, then every wave gathers the patches of its 16-pixel tiles from LDS element by element
// (lane = pixel x 8 consecutive patch values) and multiplies them with weight fragments it gathered
// once.  SYS: the input is the caller's buffer and is read at system scope.
constexpr int STEM_MAX_FT = 4, STEM_MAX_KS = 2;
template <int LD, int ST, bool SYS>
__device__ __forceinline__ void stem_units(const DevOp &op, float *lds, int rank, int nranks) {
    constexpr int XLD = SYS ? AUX_SYS : LD;
    const ConvArgs &a = op.conv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, kg = lane >> 4;
    const int KK = a.R * a.R * a.C;      // patch length
    const int ksteps = (KK + 31) >> 5;   // <= STEM_MAX_KS
    const int ftiles = (a.K + 15) >> 4;  // <= STEM_MAX_FT
    const int M = a.B * a.P * a.Q;
    const int row_elems = a.W * a.C;     // even: rows are copied as 32-bit words
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (long)a.B * a.H * a.W * a.C * 2);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (long)M * a.K * 2);
    const global_u16 *wg = (const global_u16 *)a.w;
    uint16_t *rows = reinterpret_cast<uint16_t *>(lds);

    // patch value k = 32 * ks + 8 * kg + e of this lane: LDS element offset from the patch corner,
    // column offset (for the image border), or -1 beyond the patch
    int k_off[STEM_MAX_KS][8], k_ds[STEM_MAX_KS][8];
    Frag fa[STEM_MAX_FT][STEM_MAX_KS];
#pragma unroll
    for (int ks = 0; ks < STEM_MAX_KS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k = ks * 32 + kg * 8 + e;
            const int tap = k / a.C, c = k - tap * a.C;
            const int dr = tap / a.R, ds = tap - dr * a.R;
            const bool in = k < KK;
            k_off[ks][e] = in ? (dr * a.W + ds) * a.C + c : 0;
            k_ds[ks][e] = in ? ds : -0x10000;
        }
    // weight fragments: filter 16 * ft + l16, the same patch values (stored as [tap][filter][8 channels])
#pragma unroll
    for (int ft = 0; ft < STEM_MAX_FT; ++ft)
#pragma unroll
        for (int ks = 0; ks < STEM_MAX_KS; ++ks) {
            unsigned v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = ks * 32 + kg * 8 + e;
                const int tap = k / a.C, c = k - tap * a.C;
                const int f = min(ft * 16 + l16, a.Kpad - 1);
                v[e] = (ft < ftiles && ks < ksteps && k < KK) ? (unsigned)wg[((long)tap * a.CG * a.Kpad + f) * 8 + c] : 0u;
            }
            fa[ft][ks].u = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
        }

    const int bands = (a.P + op.pt - 1) / op.pt;
    for (int unit = rank; unit < op.n_units; unit += nranks) {
        const int n = unit / bands, band = unit - n * bands;
        const int p0 = band * op.pt, prows = min(op.pt, a.P - p0);
        const int h_first = p0 * a.stride - a.pad, rows_in = (prows - 1) * a.stride + a.R;
        // input rows h_first .. h_first + rows_in - 1 (zeros outside the image) -> LDS
        __syncthreads();
        if ((row_elems & 7) == 0) {
            // rows are multiples of 16 bytes: two 16-byte cells per thread and pass, requested together
            const int row_cells = row_elems >> 3, cells = rows_in * row_cells;
            for (int base = tid; base < cells; base += 2 * STREAM_THREADS) {
                u32x4_t v[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int i = base + u * STREAM_THREADS;
                    const int r = i / row_cells, cc = i - r * row_cells;
                    const int h = h_first + r;
                    const bool ok = i < cells && h >= 0 && h < a.H;
                    v[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? ((n * a.H + h) * row_elems + cc * 8) * 2 : (int)OOB_OFFSET, 0, XLD);
                }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int i = base + u * STREAM_THREADS;
                    if (i < cells) reinterpret_cast<u32x4_t *>(rows)[i] = v[u];
                }
            }
        } else {
            const int row_words = row_elems >> 1, words = rows_in * row_words;
            for (int base = tid; base < words; base += 8 * STREAM_THREADS) {
                unsigned v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = base + u * STREAM_THREADS;
                    const int r = i / row_words, cw = i - r * row_words;
                    const int h = h_first + r;
                    const bool ok = i < words && h >= 0 && h < a.H;
                    v[u] = __builtin_amdgcn_raw_buffer_load_b32(rx, ok ? ((n * a.H + h) * row_elems + cw * 2) * 2 : (int)OOB_OFFSET, 0, XLD);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int i = base + u * STREAM_THREADS;
                    if (i < words) reinterpret_cast<unsigned *>(rows)[i] = v[u];
                }
            }
        }
        __syncthreads();
        const int npix = prows * a.Q;
        for (int t = wave; t * 16 < npix; t += STREAM_WAVES) {
            const int i = t * 16 + l16;
            const bool pv = i < npix;
            const int pr = pv ? i / a.Q : 0, q = pv ? i - pr * a.Q : 0;
            const int w0 = q * a.stride - a.pad;
            const int corner = pr * a.stride * row_elems + w0 * a.C;
            f32x4_t acc[STEM_MAX_FT];
#pragma unroll
            for (int ft = 0; ft < STEM_MAX_FT; ++ft) acc[ft] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < STEM_MAX_KS; ++ks) {
                if (ks < ksteps) {
                    unsigned v[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int col = w0 + k_ds[ks][e];
                        const bool ok = pv && col >= 0 && col < a.W;
                        v[e] = ok ? (unsigned)rows[corner + k_off[ks][e]] : 0u;
                    }
                    Frag fb;
                    fb.u = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
#pragma unroll
                    for (int ft = 0; ft < STEM_MAX_FT; ++ft)
                        if (ft < ftiles) acc[ft] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[ft][ks].v, fb.v, acc[ft], 0, 0, 0);
                }
            }
            const int m = (n * a.P + p0) * a.Q + i;
            with_activation(a, [&](auto tag) {
                constexpr int ACT = decltype(tag)::value;
#pragma unroll
                for (int ft = 0; ft < STEM_MAX_FT; ++ft) {
                    const int fbase = ft * 16 + kg * 4;
                    if (ft < ftiles && fbase + 4 <= a.K && pv) {
                        const float4 sh = *reinterpret_cast<const float4 *>(a.shift + fbase);
                        float4 sc = make_float4(1.f, 1.f, 1.f, 1.f);
                        if (a.scale) sc = *reinterpret_cast<const float4 *>(a.scale + fbase);
                        store_tile_bf16<ACT, ST>(ry, acc[ft], sc, sh, u32x2_t{0u, 0u}, (int)(out_elem(a, m, fbase) * 2));
                    }
                }
            });
        }
    }
}

// Depthwise k x k: one thread per output pixel x 8 channels, taps in ring order.
template <int LD, int ST>
__device__ __forceinline__ void dwconv_units(const ConvArgs &a, int rank, int nranks) {
    const int cgs = a.K >> 3;
    const long total = (long)a.B * a.P * a.Q * cgs;
    const uint16_t *w = static_cast<const uint16_t *>(a.w);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (long)a.B * a.H * a.W * a.C * 2);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (long)a.B * a.P * a.Q * a.K * 2);
    const int ntaps = a.R * a.R;
    for (long idx = (long)rank * STREAM_THREADS + threadIdx.x; idx < total; idx += (long)nranks * STREAM_THREADS) {
        const int qq = (int)(idx % a.Q), pp = (int)((idx / a.Q) % a.P);
        const long plane = idx / ((long)a.Q * a.P);
        const int cg = (int)(plane % cgs), n = (int)(plane / cgs);
        const int c = cg * 8;
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        for (int t = 0; t < ntaps; ++t) {
            const int h = pp * a.stride + c_dw_dr[t], v = qq * a.stride + c_dw_ds[t];
            if (h < 0 || h >= a.H || v < 0 || v >= a.W) continue;
            float xv[8], wv[8];
            unpack8(act_ld16<LD>(rx, in_cell(a, n, cg, h, v)), xv);
            load8(w + (long)t * a.Kpad + c, wv);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = fmaf(wv[j], xv[j], acc[j]);
        }
        float sc[8], sh[8];
        load8(a.scale + c, sc);
        load8(a.shift + c, sh);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = activate(acc[j] * sc[j] + sh[j], a.act, 0);
        act_st16<ST>(ry, out_cell(a, n, cg, pp * a.Q + qq), pack8(acc));
    }
}

// Depthwise k x k through LDS (wk == -2), k in {3, 5, 7}, stride 1 or 2: a unit is op.ft channel groups
// (of 8 channels) x a band of op.pt output rows of one image.  The workgroup copies the input rows the
// band needs into LDS, in rows padded with zero cells left and right (and zero rows outside the image),
// so the inner loop has no bounds checks, and the taps' weights as fp32 in row-major tap order.  A
// thread computes DW_ITEMS neighbouring outputs of one row and channel group: for every tap row it
// reads the row's k weights and the (DW_ITEMS - 1) * stride + k input cells the outputs share, each
// cell once.  (An odd DW_ITEMS also keeps the lanes' 16-byte LDS reads on different banks at stride 1.)
constexpr int DW_ITEMS = 5;
__host__ __device__ constexpr int dw_padded_width(int W, int Q, int R, int stride) {
    const int need = (((Q + DW_ITEMS - 1) / DW_ITEMS) * DW_ITEMS - 1) * stride + R;  // last block's last column
    return need > W + (R - 1) ? need : W + (R - 1);
}
template <int R, int S, int LD, int ST>
__device__ __forceinline__ void dw_tiled_units(const DevOp &op, float *lds, int rank, int nranks) {
    constexpr int HALF = (R - 1) / 2, NT = R * R, IT = DW_ITEMS, NCOL = (IT - 1) * S + R;
    const ConvArgs &a = op.conv;
    const int tid = threadIdx.x;
    const int CB = op.ft, rows_out = op.pt;
    const int cgs = a.K >> 3, cblocks = (cgs + CB - 1) / CB, bands = (a.P + rows_out - 1) / rows_out;
    const int qblocks = (a.Q + IT - 1) / IT;
    const int Wp = dw_padded_width(a.W, a.Q, R, S);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (long)a.B * a.H * a.W * a.C * 2);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (long)a.B * a.P * a.Q * a.K * 2);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.w, (long)a.Rmax * a.Rmax * a.Kpad * 2);
    float4 *w_lds = reinterpret_cast<float4 *>(lds);                   // [tap row][tap column][CB][2]
    u32x4_t *x_lds = reinterpret_cast<u32x4_t *>(w_lds + NT * CB * 2);  // [row][padded column][CB]
    const int cb = tid % CB;  // STREAM_THREADS is a multiple of CB: fixed per thread
    for (int unit = rank; unit < op.n_units; unit += nranks) {
        const int band = unit % bands, rest = unit / bands;
        const int cblock = rest % cblocks, n = rest / cblocks;
        const int cg0 = cblock * CB;
        const int p0 = band * rows_out, prows = min(rows_out, a.P - p0);
        const int h_first = p0 * S - HALF, rows_in = (prows - 1) * S + R;
        __syncthreads();
        // taps are stored centre first, ring by ring; LDS takes them row by row
        for (int i = tid; i < NT * CB; i += STREAM_THREADS) {
            const int t = i / CB, ci = i - t * CB, c = cg0 + ci;
            const u32x4_t wq = __builtin_amdgcn_raw_buffer_load_b128(rw, c < cgs ? (t * a.Kpad + c * 8) * 2 : (int)OOB_OFFSET, 0, 0);
            float wv[8];
            unpack8(make_uint4(wq.x, wq.y, wq.z, wq.w), wv);
            const int slot = (((c_dw_dr[t] + HALF) * R + c_dw_ds[t] + HALF) * CB + ci) * 2;
            w_lds[slot] = make_float4(wv[0], wv[1], wv[2], wv[3]);
            w_lds[slot + 1] = make_float4(wv[4], wv[5], wv[6], wv[7]);
        }
        const int cells = rows_in * Wp * CB;
        for (int base = tid; base < cells; base += 4 * STREAM_THREADS) {
            u32x4_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * STREAM_THREADS;
                const int pix = i / CB, c = cg0 + (i - pix * CB);
                const int r = pix / Wp, col = pix - r * Wp - HALF;
                const int h = h_first + r;
                const bool ok = i < cells && h >= 0 && h < a.H && col >= 0 && col < a.W && c < cgs;
                v[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? in_cell(a, n, c, h, col) : (int)OOB_OFFSET, 0, LD);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * STREAM_THREADS;
                if (i < cells) x_lds[i] = v[u];
            }
        }
        __syncthreads();
        const int items = prows * qblocks * CB;
        const bool cvalid = cg0 + cb < cgs;
        const int c = (cg0 + cb) * 8;
        float sc[8], sh[8];
        if (cvalid) {
            load8(a.scale + c, sc);
            load8(a.shift + c, sh);
        }
        for (int it = tid; it < items; it += STREAM_THREADS) {
            const int blk = it / CB;  // (it % CB == cb)
            const int pr = blk / qblocks, qb = blk - pr * qblocks;
            float acc[IT][8];
#pragma unroll
            for (int k = 0; k < IT; ++k)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[k][j] = 0.f;
            const u32x4_t *xrow = x_lds + ((pr * S) * Wp + qb * IT * S) * CB + cb;
            const float4 *wrow = w_lds + cb * 2;
#pragma unroll 1
            for (int dr = 0; dr < R; ++dr) {
                float wv[R][8];
#pragma unroll
                for (int ds = 0; ds < R; ++ds) {
                    const float4 lo = wrow[ds * CB * 2], hi = wrow[ds * CB * 2 + 1];
                    wv[ds][0] = lo.x, wv[ds][1] = lo.y, wv[ds][2] = lo.z, wv[ds][3] = lo.w;
                    wv[ds][4] = hi.x, wv[ds][5] = hi.y, wv[ds][6] = hi.z, wv[ds][7] = hi.w;
                }
#pragma unroll
                for (int col = 0; col < NCOL; ++col) {
                    const u32x4_t xq = xrow[col * CB];
                    float xv[8];
                    unpack8(make_uint4(xq.x, xq.y, xq.z, xq.w), xv);
#pragma unroll
                    for (int k = 0; k < IT; ++k) {
                        const int ds = col - k * S;  // (a constant once the loops are unrolled)
                        if (ds >= 0 && ds < R) {
#pragma unroll
                            for (int j = 0; j < 8; ++j) acc[k][j] = fmaf(wv[ds][j], xv[j], acc[k][j]);
                        }
                    }
                }
                xrow += Wp * CB;
                wrow += R * CB * 2;
            }
            if (cvalid) {
#pragma unroll
                for (int k = 0; k < IT; ++k) {
                    const int q = qb * IT + k;
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[k][j] = activate(acc[k][j] * sc[j] + sh[j], a.act, 0);
                    act_st16<ST>(ry, q < a.Q ? out_cell(a, n, cg0 + cb, (p0 + pr) * a.Q + q) : (int)OOB_OFFSET, pack8(acc[k]));
                }
            }
        }
    }
}

// Depthwise k x k straight from memory (wk == -4), for layers whose bands in LDS would be too small to
// keep a workgroup's threads busy (wide maps, stride 2).  A thread computes DW_ITEMS outputs of one column
// and channel group, one below the other: for every tap column it loads the column's k weights and the
// (DW_ITEMS - 1) * stride + k input cells those outputs share, each once.  Neighbouring lanes take
// neighbouring columns, so every load and store of a wave is one contiguous run of cells; items are spread
// over all threads of the team; no LDS, no barriers.  Cells outside the image are requested past the end
// of the buffer and arrive as zeros.
template <int R, int S, int LD, int ST>
__device__ __forceinline__ void dw_direct_units(const DevOp &op, int rank, int nranks) {
    constexpr int HALF = (R - 1) / 2, IT = DW_ITEMS, NROW = (IT - 1) * S + R;
    const ConvArgs &a = op.conv;
    const int cgs = a.K >> 3, pblocks = (a.P + IT - 1) / IT;
    const long items = (long)a.B * cgs * pblocks * a.Q;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (long)a.B * a.H * a.W * a.C * 2);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (long)a.B * a.P * a.Q * a.K * 2);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.w, (long)a.Rmax * a.Rmax * a.Kpad * 2);
    for (long it = (long)rank * STREAM_THREADS + threadIdx.x; it < items; it += (long)nranks * STREAM_THREADS) {
        // items in storage order (image, channel group, block of rows, column)
        const int q = (int)(it % a.Q);
        const long rowi = it / a.Q;
        const int pb = (int)(rowi % pblocks);
        const long plane = rowi / pblocks;
        const int cg = (int)(plane % cgs), n = (int)(plane / cgs);
        const int c = cg * 8;
        const int row0 = pb * IT * S - HALF, col0 = q * S - HALF;
        float acc[IT][8];
#pragma unroll
        for (int k = 0; k < IT; ++k)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[k][j] = 0.f;
        int row_off[NROW];  // byte offset of the window's rows at column 0; -1 outside the image
#pragma unroll
        for (int r = 0; r < NROW; ++r) {
            const int h = row0 + r;
            row_off[r] = h >= 0 && h < a.H ? in_cell(a, n, cg, h, 0) : -1;
        }
#pragma unroll 1
        for (int ds = 0; ds < R; ++ds) {
            const int col = col0 + ds;
            const bool col_ok = col >= 0 && col < a.W;
            u32x4_t wq[R], xq[NROW];
#pragma unroll
            for (int dr = 0; dr < R; ++dr)
                wq[dr] = __builtin_amdgcn_raw_buffer_load_b128(rw, (dw_tap_index(dr - HALF, ds - HALF) * a.Kpad + c) * 2, 0, 0);
#pragma unroll
            for (int r = 0; r < NROW; ++r)
                xq[r] = __builtin_amdgcn_raw_buffer_load_b128(rx, col_ok && row_off[r] >= 0 ? row_off[r] + col * 16 : (int)OOB_OFFSET, 0, LD);
            float wv[R][8];
#pragma unroll
            for (int dr = 0; dr < R; ++dr) unpack8(make_uint4(wq[dr].x, wq[dr].y, wq[dr].z, wq[dr].w), wv[dr]);
#pragma unroll
            for (int r = 0; r < NROW; ++r) {
                float xv[8];
                unpack8(make_uint4(xq[r].x, xq[r].y, xq[r].z, xq[r].w), xv);
#pragma unroll
                for (int k = 0; k < IT; ++k) {
                    const int dr = r - k * S;  // (a constant once the loops are unrolled)
                    if (dr >= 0 && dr < R) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[k][j] = fmaf(wv[dr][j], xv[j], acc[k][j]);
                    }
                }
            }
        }
        float sc[8], sh[8];
        load8(a.scale + c, sc);
        load8(a.shift + c, sh);
#pragma unroll
        for (int k = 0; k < IT; ++k) {
            const int pr = pb * IT + k;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[k][j] = activate(acc[k][j] * sc[j] + sh[j], a.act, 0);
            act_st16<ST>(ry, pr < a.P ? out_cell(a, n, cg, pr * a.Q + q) : (int)OOB_OFFSET, pack8(acc[k]));
        }
    }
}

template <int LD, int ST>
__device__ __forceinline__ void maxpool_units(const PoolArgs &a, int rank, int nranks) {
    const int cgs = a.C >> 3;
    const long total = (long)a.B * a.P * a.Q * cgs;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (long)a.B * a.H * a.W * a.C * 2);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (long)a.B * a.P * a.Q * a.C * 2);
    for (long idx = (long)rank * STREAM_THREADS + threadIdx.x; idx < total; idx += (long)nranks * STREAM_THREADS) {
        // outputs in storage order (image, channel group, pixel): neighbouring lanes, neighbouring cells
        const int qq = (int)(idx % a.Q), pp = (int)((idx / a.Q) % a.P);
        const long plane = idx / ((long)a.Q * a.P);
        const int cg = (int)(plane % cgs), n = (int)(plane / cgs);
        // All nine cells are requested at once.  A row or column outside the image is replaced by the nearest one
        // inside, which belongs to the same window (the window's centre lies inside): the maximum does not change.
        uint4 cell[9];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int h = min(max(pp * 2 - 1 + r, 0), a.H - 1);
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const int v = min(max(qq * 2 - 1 + s, 0), a.W - 1);
                cell[r * 3 + s] = act_ld16<LD>(rx, (((n * cgs + cg) * a.H + h) * a.W + v) * 16);
            }
        }
        float best[8];
        unpack8(cell[0], best);
#pragma unroll
        for (int t = 1; t < 9; ++t) {
            float xv[8];
            unpack8(cell[t], xv);
#pragma unroll
            for (int j = 0; j < 8; ++j) best[j] = fmaxf(best[j], xv[j]);
        }
        act_st16<ST>(ry, (((n * cgs + cg) * a.P + pp) * a.Q + qq) * 16, pack8(best));
    }
}

// Global average: a workgroup takes (image, block of channel groups).  The threads are pixel lanes x channel groups
// (8 lanes per group when the groups fill the threads, up to 64 for few groups); a lane requests eight of its
// pixels at a time, the lanes' sums meet in LDS and one thread per channel group adds them up in a fixed order.
template <int LD, int ST>
__device__ __forceinline__ void gap_units(const PoolArgs &a, float *lds, int rank, int nranks) {
    const int t = threadIdx.x;
    const int cgs = a.C >> 3, hw = a.H * a.W;
    const int PLN = cgs > 32 ? 8 : cgs > 16 ? 16 : cgs > 8 ? 32 : 64, CGP = STREAM_THREADS / PLN, cstride = PLN * 8 + 8;
    const int passes = (cgs + CGP - 1) / CGP, n_blocks = a.B * passes;
    const int pl = t % PLN, cgl = t / PLN;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, (long)a.B * hw * a.C * 2);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, (long)a.B * a.C * (a.out_f32 ? 4 : 2));
    const float inv = 1.0f / (float)hw;
    for (int b = rank; b < n_blocks; b += nranks) {
        const int n = b / passes, cg0 = (b - n * passes) * CGP, cg = cg0 + cgl;
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        const int base = (n * cgs + cg) * hw;
        for (int p0 = pl; p0 < hw; p0 += 8 * PLN) {
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + u * PLN;
                v[u] = act_ld16<LD>(rx, cg < cgs && p < hw ? (base + p) * 16 : (int)OOB_OFFSET);  // (else zeros)
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                float xv[8];
                unpack8(v[u], xv);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] += xv[j];
            }
        }
        float4 *dst = reinterpret_cast<float4 *>(lds + cgl * cstride + pl * 8);
        dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
        __syncthreads();
        if (t < CGP && cg0 + t < cgs) {
            const float4 *src = reinterpret_cast<const float4 *>(lds + t * cstride);
            float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
            for (int q = 0; q < PLN; ++q) {
                const float4 x0 = src[q * 2], x1 = src[q * 2 + 1];
                lo.x += x0.x, lo.y += x0.y, lo.z += x0.z, lo.w += x0.w;
                hi.x += x1.x, hi.y += x1.y, hi.z += x1.z, hi.w += x1.w;
            }
            float o[8] = {lo.x * inv, lo.y * inv, lo.z * inv, lo.w * inv, hi.x * inv, hi.y * inv, hi.z * inv, hi.w * inv};
            const int c = (cg0 + t) * 8;
            if (a.out_f32) {  // (per-image vectors stay float32: the layers they feed split them into two bf16 terms)
                act_st16<ST>(ry, (n * a.C + c) * 4, make_uint4(__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3])));
                act_st16<ST>(ry, (n * a.C + c) * 4 + 16, make_uint4(__float_as_uint(o[4]), __float_as_uint(o[5]), __float_as_uint(o[6]), __float_as_uint(o[7])));
            } else {
                act_st16<ST>(ry, (n * a.C + c) * 2, pack8(o));
            }
        }
        __syncthreads();
    }
}

template <int LD, int ST>
__device__ __forceinline__ void gate_units(const PoolArgs &a, int rank, int nranks) {
    const int cgs = a.C >> 3;
    const long total = (long)a.B * a.H * a.W * cgs;
    const long bytes = (long)a.B * a.H * a.W * a.C * 2;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, bytes);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, bytes);
    const __amdgpu_buffer_rsrc_t rg = make_rsrc(a.gate, (long)a.B * a.C * 4);
    for (long idx = (long)rank * STREAM_THREADS + threadIdx.x; idx < total; idx += (long)nranks * STREAM_THREADS) {
        const long plane = idx / ((long)a.H * a.W);  // cells are taken in storage order: image, channel group, pixel
        const int cg = (int)(plane % cgs), n = (int)(plane / cgs);
        float xv[8];
        unpack8(act_ld16<LD>(rx, (int)(idx * 16)), xv);
        const uint4 g0 = act_ld16<LD>(rg, (n * a.C + cg * 8) * 4), g1 = act_ld16<LD>(rg, (n * a.C + cg * 8) * 4 + 16);
        xv[0] *= __uint_as_float(g0.x), xv[1] *= __uint_as_float(g0.y), xv[2] *= __uint_as_float(g0.z);
        xv[3] *= __uint_as_float(g0.w), xv[4] *= __uint_as_float(g1.x), xv[5] *= __uint_as_float(g1.y);
        xv[6] *= __uint_as_float(g1.z), xv[7] *= __uint_as_float(g1.w);
        act_st16<ST>(ry, (int)(idx * 16), pack8(xv));
    }
}

// ------------------------------------------------------------------ a squeeze-excite block as one op
// out[k] = f(sc[k] * sum_c w[k][c] * in[c] + sh[k]) for k < K, all vectors float32 in LDS; the workgroup's threads
// are KT filters x (512 / KT) slices of the channel groups, partial sums meet in `part`.  HSIG: f = hard sigmoid,
// else the activation `act`.
constexpr int SE_BATCH = 8;
template <bool HSIG>
__device__ __forceinline__ void se_gemv(const void *w, int Kpad, int K, int cgs_in, const float *in, float *out, float *part,
                                        const float *sc, const float *sh, int act) {
    const int t = threadIdx.x;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (long)cgs_in * Kpad * 16);
    const int KT = K <= 64 ? 64 : K <= 128 ? 128 : K <= 256 ? 256 : STREAM_THREADS;
    const int slots = STREAM_THREADS / KT;
    const int kk = t % KT, slot = t / KT;
    for (int k0 = 0; k0 < K; k0 += KT) {
        const int k = k0 + kk;
        float acc = 0.f;
        // (SE_BATCH cells per thread in flight: the op is a chain of load round trips, so few long ones)
        for (int cg0 = slot; cg0 < cgs_in; cg0 += slots * SE_BATCH) {
            u32x4_t v[SE_BATCH];
#pragma unroll
            for (int j = 0; j < SE_BATCH; ++j) {
                const int c = cg0 + j * slots;
                v[j] = __builtin_amdgcn_raw_buffer_load_b128(rw, c < cgs_in && k < Kpad ? (c * Kpad + k) * 16 : (int)OOB_OFFSET, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < SE_BATCH; ++j) {
                const int c = min(cg0 + j * slots, cgs_in - 1);  // (past the end the weights arrived as zeros)
                float wv[8];
                unpack8(make_uint4(v[j].x, v[j].y, v[j].z, v[j].w), wv);
                const float4 lo = *reinterpret_cast<const float4 *>(in + c * 8), hi = *reinterpret_cast<const float4 *>(in + c * 8 + 4);
                acc = fmaf(wv[0], lo.x, acc), acc = fmaf(wv[1], lo.y, acc), acc = fmaf(wv[2], lo.z, acc), acc = fmaf(wv[3], lo.w, acc);
                acc = fmaf(wv[4], hi.x, acc), acc = fmaf(wv[5], hi.y, acc), acc = fmaf(wv[6], hi.z, acc), acc = fmaf(wv[7], hi.w, acc);
            }
        }
        part[slot * KT + kk] = acc;
        __syncthreads();
        if (t < KT && k0 + t < K) {
            float v = 0.f;
            for (int sl = 0; sl < slots; ++sl) v += part[sl * KT + t];
            v = v * (sc ? sc[k0 + t] : 1.0f) + sh[k0 + t];
            out[k0 + t] = HSIG ? fminf(fmaxf(v + 3.0f, 0.0f), 6.0f) * (1.0f / 6.0f) : activate(v, act, 0);
        }
        __syncthreads();
    }
}

// Squeeze-excite block (DEV_SE).  The images are dealt to groups of workgroups; every workgroup of a group works
// out the image's gate on its own (average of the map over the pixels, FC, FC: the map and the weights come out of
// the XCD's L2, and the vectors never leave LDS), then the group's workgroups share the gating of the map.  The
// map is only read and the gated map is another buffer, so no workgroup waits for another inside the op.
constexpr int SE_PART = 4608;  // floats: pooling partials [<= 64 channel groups][pixel lanes * 8 + 8], then FC partials
static_assert((SE_PART + 2 * SE_MAX_C + SE_MAX_MID) * 4 <= RED_BYTES && SE_PART >= 64 * 72 && SE_PART >= 32 * 136 &&
                  SE_PART >= 16 * 264 && SE_PART >= 8 * 520 && SE_PART >= STREAM_THREADS,
              "the squeeze-excite op's vectors fit the scratch part of LDS");
// (a function of its own, not inlined: inside the kernel's body its registers count against those of the other
// units, which then run slower; and with 16 or more cells in flight per thread the function needs so many registers
// that the whole kernel slows down by almost half, measured, so SE_BATCH stays at 8)
template <int LD, int ST>
__device__ __attribute__((noinline)) void se_units(const SeArgs a, float *lds, int rank, int nranks) {
    const int t = threadIdx.x;
    float *part = lds, *mean = lds + SE_PART, *hid = mean + SE_MAX_C, *gate = hid + SE_MAX_MID;
    const int cgs = a.C >> 3, hw = a.HW;
    const long bytes = (long)a.B * hw * a.C * 2;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(a.x, bytes);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(a.y, bytes);
    const int ngroups = min(a.B, nranks), g = rank % ngroups, j_in = rank / ngroups;
    const int gsize = (nranks - g + ngroups - 1) / ngroups;  // workgroups with rank % ngroups == g
    // pixel lanes per channel group: as many as let all groups go in one pass, between 8 (a 128-byte line per lane
    // group) and 64
    const int PLN = cgs > 32 ? 8 : cgs > 16 ? 16 : cgs > 8 ? 32 : 64, CGP = STREAM_THREADS / PLN, cstride = PLN * 8 + 8;
    const int pl = t % PLN, cgl = t / PLN;
    const float inv = 1.0f / (float)hw;
    for (int n = g; n < a.B; n += ngroups) {
        for (int cg0 = 0; cg0 < cgs; cg0 += CGP) {
            const int cg = cg0 + cgl;
            float acc[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = 0.f;
            const int base = (n * cgs + cg) * hw;
            for (int p0 = pl; p0 < hw; p0 += SE_BATCH * PLN) {
                uint4 v[SE_BATCH];
#pragma unroll
                for (int j = 0; j < SE_BATCH; ++j) {
                    const int p = p0 + j * PLN;
                    v[j] = act_ld16<LD>(rx, cg < cgs && p < hw ? (base + p) * 16 : (int)OOB_OFFSET);
                }
#pragma unroll
                for (int j = 0; j < SE_BATCH; ++j) {
                    float xv[8];
                    unpack8(v[j], xv);
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[e] += xv[e];
                }
            }
            float4 *dst = reinterpret_cast<float4 *>(part + cgl * cstride + pl * 8);
            dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
            dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
            __syncthreads();
            if (t < CGP * 8 && cg0 + (t >> 3) < cgs) {
                const float *src = part + (t >> 3) * cstride + (t & 7);
                float sum = 0.f;
                for (int q = 0; q < PLN; ++q) sum += src[q * 8];
                mean[cg0 * 8 + t] = sum * inv;
            }
            __syncthreads();
        }
        se_gemv<false>(a.w1, a.Kpad1, a.mid, cgs, mean, hid, part, a.sc1, a.sh1, a.act1);
        se_gemv<true>(a.w2, a.Kpad2, a.C, a.mid >> 3, hid, gate, part, a.sc2, a.sh2, 0);
        // the image's cells in storage order (channel group, pixel), dealt to the group's workgroups in runs of 512
        const int cells = cgs * hw, first = n * cells;
        for (int i0 = j_in * STREAM_THREADS + t; i0 < cells; i0 += gsize * STREAM_THREADS * 8) {
            uint4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = i0 + j * gsize * STREAM_THREADS;
                v[j] = act_ld16<LD>(rx, i < cells ? (first + i) * 16 : (int)OOB_OFFSET);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = i0 + j * gsize * STREAM_THREADS;
                if (i < cells) {
                    const int cg = i / hw;
                    const float4 lo = *reinterpret_cast<const float4 *>(gate + cg * 8), hi = *reinterpret_cast<const float4 *>(gate + cg * 8 + 4);
                    float xv[8];
                    unpack8(v[j], xv);
                    xv[0] *= lo.x, xv[1] *= lo.y, xv[2] *= lo.z, xv[3] *= lo.w;
                    xv[4] *= hi.x, xv[5] *= hi.y, xv[6] *= hi.z, xv[7] *= hi.w;
                    act_st16<ST>(ry, (first + i) * 16, pack8(xv));
                }
            }
        }
        __syncthreads();  // the vectors in LDS are written again for the next image
    }
}

// The descriptor of the running op is staged in LDS, and what a lane reads from LDS counts as
// lane-varying for the compiler: buffer descriptors built from it would be resolved lane by lane.
// This copy moves every word to a scalar register.
__device__ __forceinline__ DevOp uniform_op(const DevOp &src) {
    constexpr int WORDS = (int)(sizeof(DevOp) / sizeof(int));
    union {
        DevOp o;
        int w[WORDS];
    } u;
    const int *p = reinterpret_cast<const int *>(&src);
#pragma unroll
    for (int k = 0; k < WORDS; ++k) u.w[k] = __builtin_amdgcn_readfirstlane(p[k]);
    return u.o;
}

// Tiled dense conv with the weights held in LDS (wk == -3): ft, pt as for wk == 0.
template <int LD, int ST>
__device__ __forceinline__ void run_ares(const DevOp &op, u32x4_t *lds, int rank, int nranks) {
    const int key = op.ft * 4 + op.pt;
    switch (key) {
        case 2 * 4 + 1: conv_ares_units<2, 1, LD, ST>(op, lds, rank, nranks); break;
        case 2 * 4 + 2: conv_ares_units<2, 2, LD, ST>(op, lds, rank, nranks); break;
        case 4 * 4 + 1: conv_ares_units<4, 1, LD, ST>(op, lds, rank, nranks); break;
        case 4 * 4 + 2: conv_ares_units<4, 2, LD, ST>(op, lds, rank, nranks); break;
        case 6 * 4 + 1: conv_ares_units<6, 1, LD, ST>(op, lds, rank, nranks); break;
        default: break;
    }
}

// Tiled dense conv (wk == 0): ft = filter tiles, pt = pixel tiles per wave of a unit.
template <int LD, int ST>
__device__ __forceinline__ void run_tiled(const DevOp &op, u32x4_t *stage, int rank, int nranks) {
    const int key = op.ft * 8 + op.pt;
    switch (key) {
        case 2 * 8 + 1: conv_tile_units<2, 1, LD, ST>(op, stage, rank, nranks); break;
        case 2 * 8 + 2: conv_tile_units<2, 2, LD, ST>(op, stage, rank, nranks); break;
        case 3 * 8 + 1: conv_tile_units<3, 1, LD, ST>(op, stage, rank, nranks); break;
        case 3 * 8 + 2: conv_tile_units<3, 2, LD, ST>(op, stage, rank, nranks); break;
        case 3 * 8 + 4: conv_tile_units<3, 4, LD, ST>(op, stage, rank, nranks); break;
        case 4 * 8 + 1: conv_tile_units<4, 1, LD, ST>(op, stage, rank, nranks); break;
        case 4 * 8 + 2: conv_tile_units<4, 2, LD, ST>(op, stage, rank, nranks); break;
        case 4 * 8 + 4: conv_tile_units<4, 4, LD, ST>(op, stage, rank, nranks); break;
        case 6 * 8 + 1: conv_tile_units<6, 1, LD, ST>(op, stage, rank, nranks); break;
        case 6 * 8 + 2: conv_tile_units<6, 2, LD, ST>(op, stage, rank, nranks); break;
        default: break;
    }
}

// A depthwise op: through LDS (wk == -2), straight from memory with neighbouring outputs per thread (wk == -4), or
// one output cell per thread.
template <int LD, int ST>
__device__ __forceinline__ void run_dw(const DevOp &op, float *lds, int rank, int nranks) {
    if (op.wk == -2) {
        const int key = op.conv.R * 4 + op.conv.stride;
        switch (key) {
            case 3 * 4 + 1: dw_tiled_units<3, 1, LD, ST>(op, lds, rank, nranks); break;
            case 3 * 4 + 2: dw_tiled_units<3, 2, LD, ST>(op, lds, rank, nranks); break;
            case 5 * 4 + 1: dw_tiled_units<5, 1, LD, ST>(op, lds, rank, nranks); break;
            case 5 * 4 + 2: dw_tiled_units<5, 2, LD, ST>(op, lds, rank, nranks); break;
            case 7 * 4 + 1: dw_tiled_units<7, 1, LD, ST>(op, lds, rank, nranks); break;
            case 7 * 4 + 2: dw_tiled_units<7, 2, LD, ST>(op, lds, rank, nranks); break;
            default: break;
        }
    } else if (op.wk == -4) {
        const int key = op.conv.R * 4 + op.conv.stride;
        switch (key) {
            case 3 * 4 + 1: dw_direct_units<3, 1, LD, ST>(op, rank, nranks); break;
            case 3 * 4 + 2: dw_direct_units<3, 2, LD, ST>(op, rank, nranks); break;
            case 5 * 4 + 1: dw_direct_units<5, 1, LD, ST>(op, rank, nranks); break;
            case 5 * 4 + 2: dw_direct_units<5, 2, LD, ST>(op, rank, nranks); break;
            case 7 * 4 + 1: dw_direct_units<7, 1, LD, ST>(op, rank, nranks); break;
            case 7 * 4 + 2: dw_direct_units<7, 2, LD, ST>(op, rank, nranks); break;
            default: break;
        }
    } else {
        dwconv_units<LD, ST>(op.conv, rank, nranks);
    }
}

// Runs one op on the calling workgroup's share (rank of nranks).  OPS says which kinds of op the kernel contains
// (a kernel holds one register allocation for all its units, so units that a network never uses are left out of
// the kernel that serves it): OPS_ALL, OPS_DENSE (no depthwise, gating or squeeze-excite ops), OPS_MOBILE (no
// max-pool).
constexpr int OPS_ALL = 0, OPS_DENSE = 1, OPS_MOBILE = 2;
template <int LD, int ST, bool RES, int OPS>
__device__ __forceinline__ void run_op(const DevOp &op, float *lds, int rank, int nranks, const ResView rv,
                                       const StepTables tb) {
    switch (op.kind) {
        case OP_CONV:
        case OP_FC:
            if (op.wk == -1 && op.in_patch)
                stem_units<LD, ST, true>(op, lds, rank, nranks);
            else if (op.wk == -1)
                stem_units<LD, ST, false>(op, lds, rank, nranks);
            else if ((op.conv.C & 7) != 0)
                conv_direct_units<ST>(op.conv, rank, nranks);
            else if (op.wk == 0)
                run_tiled<LD, ST>(op, reinterpret_cast<u32x4_t *>(lds), rank, nranks);
            else if (op.wk == -3)
                run_ares<LD, ST>(op, reinterpret_cast<u32x4_t *>(lds), rank, nranks);
            else if (op.conv.in_f32 && op.ft == 4)
                conv_units<4, 1, LD, ST, RES, true>(op, lds, rank, nranks, rv, tb);
            else if (op.conv.in_f32 && op.ft == 2)
                conv_units<2, 1, LD, ST, RES, true>(op, lds, rank, nranks, rv, tb);
            else if (op.conv.in_f32)
                conv_units<1, 1, LD, ST, RES, true>(op, lds, rank, nranks, rv, tb);
            else if (op.ft == 2 && op.pt == 4)
                conv_units<2, 4, LD, ST, RES>(op, lds, rank, nranks, rv, tb);
            else if (op.ft == 1 && op.pt == 4)
                conv_units<1, 4, LD, ST, RES>(op, lds, rank, nranks, rv, tb);
            else if (op.ft == 1 && op.pt == 2)
                conv_units<1, 2, LD, ST, RES>(op, lds, rank, nranks, rv, tb);
            else if (op.ft == 2 && op.pt == 2)
                conv_units<2, 2, LD, ST, RES>(op, lds, rank, nranks, rv, tb);
            else if (op.ft == 2 && op.pt == 1)
                conv_units<2, 1, LD, ST, RES>(op, lds, rank, nranks, rv, tb);
            else if (op.ft == 4 && op.pt == 1)
                conv_units<4, 1, LD, ST, RES>(op, lds, rank, nranks, rv, tb);
            else
                conv_units<1, 1, LD, ST, RES>(op, lds, rank, nranks, rv, tb);
            break;
        case OP_DW:
            if constexpr (OPS != OPS_DENSE) run_dw<LD, ST>(op, lds, rank, nranks);
            break;
        case OP_MAXPOOL:
            if constexpr (OPS != OPS_MOBILE) maxpool_units<LD, ST>(op.pool, rank, nranks);
            break;
        case OP_GAP:
            gap_units<LD, ST>(op.pool, lds, rank, nranks);
            break;
        case OP_GATE:
            if constexpr (OPS != OPS_DENSE) gate_units<LD, ST>(op.pool, rank, nranks);
            break;
        case DEV_SE:
            if constexpr (OPS == OPS_MOBILE) se_units<LD, ST>(op.se, lds, rank, nranks);  // (team programs only)
            break;
        default:
            break;
    }
}

// ------------------------------------------------------------------ the team kernel
// sync layout (64-bit words, 16 words apart): abort, workgroups that joined per XCD, barrier arrivals
// per team, workgroups that joined in total, go counter per team, broadcast slot per team (cmd/n_ops,
// prog, input, logits, seq), clock of the latest post any team received (a team leaves only when the
// whole kernel has been idle).
constexpr int SY_ABORT = 0;
__host__ __device__ constexpr int sy_xcd(int x) { return 16 * (1 + x); }
__host__ __device__ constexpr int sy_barrier(int t) { return 16 * (1 + MAX_XCDS + t); }
constexpr int SY_JOINED = 16 * (1 + MAX_XCDS + MAX_TEAMS);
__host__ __device__ constexpr int sy_go(int t) { return SY_JOINED + 16 * (1 + t); }
__host__ __device__ constexpr int sy_slot(int t) { return SY_JOINED + 16 * (1 + MAX_TEAMS + t); }
constexpr int SY_CLOCK = SY_JOINED + 16 * (1 + 2 * MAX_TEAMS);
static_assert(SY_CLOCK + 16 <= SYNC_WORDS, "the barrier area holds the team kernel's words");

__device__ __forceinline__ unsigned long long ld_agent(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(unsigned long long *p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_sys(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Why a workgroup gave up: which bounded wait ran out (the host reports it with the next call).
enum AbortWhy { ABORT_FORMATION = 1, ABORT_BARRIER = 2, ABORT_GO = 3, ABORT_POST = 4 };
__device__ __forceinline__ void raise_abort(const TeamArgs &ta, int why) {
    // the first reason stays: the waits that give up because somebody else did would overwrite it
    if (ld_agent(&ta.sync[SY_ABORT]) == 0)
        __hip_atomic_store(&ta.host->abort_flag, (unsigned)why, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    st_agent(&ta.sync[SY_ABORT], 1ull);
}

// Drops every line of this compute unit's vector L1.  A team's activations live in its XCD's L2:
// stores reach the L2 (the L1 is write-through), but ordinary loads may be served by the L1, which
// still holds the previous contents of a reused activation buffer.
__device__ __forceinline__ void invalidate_vector_l1() {
    asm volatile("buffer_inv sc1\n\ts_waitcnt vmcnt(0)" ::: "memory");
}

// Barrier among the workgroups of one team (all on one XCD).  With INV the compute unit's vector L1
// is empty on return, so that ordinary loads see what the team wrote; between the ops of a query the
// activations are instead loaded around the L1 (sc1), which costs less than emptying it.
// Returns false when the wait ran out.
template <bool INV = true>
__device__ __forceinline__ bool team_barrier(const TeamArgs &ta, int team, unsigned tsize, unsigned long long e,
                                             int *lds_flag) {
    // Every store of this wave has been acknowledged by the XCD's L2 (the vector L1 writes through) before the
    // wave reaches the workgroup barrier, hence before thread 0 counts the workgroup in at that same L2.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long *ctr = &ta.sync[sy_barrier(team)];
        __hip_atomic_fetch_add(ctr, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long target = e * tsize;
        int spins = 0, good = 1;
        while (ld_agent(ctr) < target) {
            if (++spins > ta.spin_limit || ld_agent(&ta.sync[SY_ABORT]) != 0) {
                raise_abort(ta, ABORT_BARRIER);
                good = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        if (INV) invalidate_vector_l1();
        *lds_flag = good;
    }
    __syncthreads();
    return *lds_flag != 0;
}

// Copies n 8-byte words from pinned host memory into device memory; the workgroups of a team share
// the work.  The team kernel takes everything the host hands it this way (programs, residency
// tables): it fills every compute unit, so a copy kernel of the runtime could not start beside it.
__device__ __forceinline__ void team_fetch(unsigned long long *dst, const unsigned long long *src, int n, int rank,
                                           int tsize) {
    for (int i = rank * STREAM_THREADS + (int)threadIdx.x; i < n; i += tsize * STREAM_THREADS) dst[i] = ld_sys(src + i);
}

// Brings the residency table `src` (pinned host memory) into the team's device memory `mem`; the
// workgroups of the team share the copy and meet at a barrier before anyone reads it.  Returns the
// device copy through `out`: null when there is no table or it was made for another team size.
// False: the barrier's wait ran out.
__device__ __forceinline__ bool fetch_table(const TeamArgs &ta, const ResTable *src, char *mem, int team, int rank,
                                            int tsize, unsigned long long &epoch, unsigned long long *hdr, int *lds_flag,
                                            const ResTable **out) {
    *out = nullptr;
    if (!src) return true;
    if (threadIdx.x < 4) hdr[threadIdx.x] = ld_sys(reinterpret_cast<const unsigned long long *>(src) + threadIdx.x);
    __syncthreads();
    const int n_layers = min((int)(hdr[0] & 0xFFFFFFFFull), RES_MAX_LAYERS), team_size = (int)(hdr[0] >> 32);
    const int n_entries = min((int)(hdr[1] & 0xFFFFFFFFull), RES_MAX_ENTRIES), geometry = (int)(hdr[1] >> 32);
    const unsigned long long *layers = reinterpret_cast<const unsigned long long *>(hdr[2]);
    const unsigned long long *entries = reinterpret_cast<const unsigned long long *>(hdr[3]);
    __syncthreads();  // hdr may be written again
    if (team_size != tsize) return true;
    ResTable *dst = reinterpret_cast<ResTable *>(mem);
    ResLayer *dst_layers = reinterpret_cast<ResLayer *>(mem + 64);
    ResEntry *dst_entries = reinterpret_cast<ResEntry *>(mem + 64 + (long)RES_MAX_LAYERS * sizeof(ResLayer));
    if (rank == 0 && threadIdx.x == 0) {
        dst->n_layers = n_layers, dst->team_size = team_size, dst->n_entries = n_entries, dst->geometry = geometry;
        dst->layers = dst_layers, dst->entries = dst_entries;
    }
    team_fetch(reinterpret_cast<unsigned long long *>(dst_layers), layers, n_layers * (int)(sizeof(ResLayer) / 8), rank, tsize);
    team_fetch(reinterpret_cast<unsigned long long *>(dst_entries), entries, n_entries, rank, tsize);
    epoch += 1;
    if (!team_barrier(ta, team, tsize, epoch, lds_flag)) return false;  // (empties the L1: an older table sat at these addresses)
    *out = dst;
    return true;
}

// Copies slab cells this workgroup owns from the packed weights into its LDS store: the valid cells of `tab`
// that the store does not hold yet.  `present` (device memory of the team, one word per table entry, cleared
// when the kernel starts) remembers for every slab how many channel groups of it have been copied, tagged
// with the geometry they were copied under; only the slab's owner reads and writes its word.  Cells stay in the store
// when a later SubGraph no longer covers them (they are still the SuperNet's weights), so a SubGraph that grows
// back finds them there.  `work` is LDS that is idle during an install (the partial-sum area).  The table sits
// in device memory and every dependent read costs a round trip, so nothing here walks it entry by entry: the
// layers come into LDS in one pass, the entries are searched by all threads at once, and the 16-byte pieces
// of all cells to copy form one index space that the threads share, eight loads each in flight.
struct InstallItem {
    int layer_f;      // layer << 16 | filter tile
    int lds_off;      // byte offset of the slab inside the store
    int first_piece;  // index of the item's first piece among all pieces of this workgroup
    int cg_from;      // first channel group to copy
};
constexpr int INSTALL_MAX_ITEMS = RES_STORE_BYTES / 256;  // a slab is at least one 256-byte cell row
static_assert(RES_MAX_LAYERS * sizeof(ResLayer) + INSTALL_MAX_ITEMS * sizeof(InstallItem) + 16 <= RED_BYTES,
              "the install work area must fit the partial-sum area");

__device__ void install_slabs(const ResTable *tab, unsigned *present, int rank, char *store, char *work, unsigned *layer_mask) {
    ResLayer *lay = reinterpret_cast<ResLayer *>(work);
    InstallItem *items = reinterpret_cast<InstallItem *>(work + RES_MAX_LAYERS * sizeof(ResLayer));
    int *cnt = reinterpret_cast<int *>(items + INSTALL_MAX_ITEMS);  // [0] items, [1] pieces
    const int tid = threadIdx.x;
    const int nl = min(tab->n_layers, RES_MAX_LAYERS), ne = min(tab->n_entries, RES_MAX_ENTRIES);
    const ResLayer *layers = tab->layers;
    const ResEntry *entries = tab->entries;
    // a slab's word: the geometry number (never 0) in the upper 23 bits, channel groups present in the lower 9;
    // the words are cleared when the kernel starts
    static_assert(RES_STORE_BYTES / 256 < 512, "a slab's channel groups fit 9 bits");
    const unsigned tag = ((unsigned)tab->geometry & 0x7FFFFFu) << 9;
    __syncthreads();  // the work area may still be read by the op before
    if (tid == 0) cnt[0] = 0, cnt[1] = 0;
    if (tid < RES_MAX_LAYERS / 32) layer_mask[tid] = 0u;
    __syncthreads();
    for (int l = tid; l < nl; l += STREAM_THREADS) {
        lay[l] = layers[l];
        if (lay[l].n_res > 0) atomicOr(&layer_mask[l >> 5], 1u << (l & 31));  // layers with valid slabs, for the op loop
    }
    __syncthreads();
    for (int i = tid; i < ne; i += STREAM_THREADS) {
        const ResEntry e = entries[i];
        if (e.owner != rank) continue;
        int l = 0;
        while (l < nl && !(lay[l].n_res > 0 && i >= lay[l].first_entry && i < lay[l].first_entry + lay[l].n_res)) ++l;
        if (l == nl) continue;
        const unsigned word = __hip_atomic_load(&present[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int cg_from = (word & 0xFFFFFE00u) == tag ? (int)(word & 0x1FFu) : 0;
        if (cg_from >= lay[l].cg_res) continue;  // everything this SubGraph wants of the tile is there already
        const int k = atomicAdd(&cnt[0], 1);
        if (k < INSTALL_MAX_ITEMS) {
            items[k] = InstallItem{(l << 16) | (i - lay[l].first_entry), e.lds_off, 0, cg_from};
            __hip_atomic_store(&present[i], tag | (unsigned)lay[l].cg_res, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    const int n = min(cnt[0], INSTALL_MAX_ITEMS);
    if (tid == 0) {
        int p = 0;
        for (int k = 0; k < n; ++k) {
            const ResLayer &L = lay[items[k].layer_f >> 16];
            items[k].first_piece = p;
            p += L.taps * (L.cg_res - items[k].cg_from) * 16;
        }
        cnt[1] = p;
    }
    __syncthreads();
    const int total = cnt[1];
    // (eight pieces in flight per thread, in named registers: arrays indexed inside the search loop would live in
    // scratch memory)
    auto fetch = [&](int p, uint4 &v, int &dst) {
        int lo = 0, hi = n - 1;  // the last item that starts at or before piece p
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (items[mid].first_piece <= p) lo = mid; else hi = mid - 1;
        }
        const InstallItem it = items[lo];
        const ResLayer &L = lay[it.layer_f >> 16];
        const int f = it.layer_f & 0xFFFF, i = p - it.first_piece;
        const int j = i & 15, tc = i >> 4;
        const int ncg = L.cg_res - it.cg_from;
        const int tap = tc / ncg, cg = it.cg_from + (tc - tap * ncg);
        v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(L.w) + (((long)tap * L.CG + cg) * L.Kpad + f * 16 + j) * 8);
        dst = it.lds_off + ((tap * L.cg_stride + cg) * 16 + j) * 16;
    };
    for (int p0 = tid; p0 < total; p0 += 8 * STREAM_THREADS) {
        uint4 v0, v1, v2, v3, v4, v5, v6, v7;
        int d0, d1, d2, d3, d4, d5, d6, d7;
        const int last = total - 1, T = STREAM_THREADS;
        fetch(min(p0, last), v0, d0), fetch(min(p0 + T, last), v1, d1), fetch(min(p0 + 2 * T, last), v2, d2);
        fetch(min(p0 + 3 * T, last), v3, d3), fetch(min(p0 + 4 * T, last), v4, d4), fetch(min(p0 + 5 * T, last), v5, d5);
        fetch(min(p0 + 6 * T, last), v6, d6), fetch(min(p0 + 7 * T, last), v7, d7);
        auto put = [&](int p, const uint4 &v, int dst) {
            if (p < total) *reinterpret_cast<uint4 *>(store + dst) = v;
        };
        put(p0, v0, d0), put(p0 + T, v1, d1), put(p0 + 2 * T, v2, d2), put(p0 + 3 * T, v3, d3);
        put(p0 + 4 * T, v4, d4), put(p0 + 5 * T, v5, d5), put(p0 + 6 * T, v6, d6), put(p0 + 7 * T, v7, d7);
    }
    __syncthreads();
}

// Two waves per SIMD (the 256-register budget): with one workgroup per compute unit there are never
// more, and under the smaller budget of three the op loops spill.  No other kernel fits beside this
// one while it runs.
template <int OPS>
__global__ __launch_bounds__(STREAM_THREADS, 2) void sushi_team_kernel(TeamArgs ta) {
    extern __shared__ __align__(16) char dyn_lds[];  // [RED_BYTES partial sums][RES_STORE_BYTES resident slabs]
    float *lds = reinterpret_cast<float *>(dyn_lds);
    char *store = dyn_lds + RED_BYTES;
    __shared__ int unit_list[132];
    __shared__ u32x4_t step_entries[STEP_TABLE_MAX];
    __shared__ u32x2_t slab_entries[STEP_TABLE_MAX];
    const StepTables tb{step_entries, slab_entries};
    __shared__ int flag;
    __shared__ int s_team, s_rank, s_size;
    __shared__ unsigned long long s_slot[7];
    __shared__ unsigned long long s_hdr[4];
    __shared__ unsigned s_layer_mask[RES_MAX_LAYERS / 32];  // bit l: layer l has valid slabs under the table in use

    // ---- team formation: which XCD am I on, how many of us are there
    if (threadIdx.x == 0) {
        const int xcc = (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 7);  // XCC_ID, bits 3:0
        const int per_xcd = ta.teams_per_xcd;
        const int arrival = (int)__hip_atomic_fetch_add(&ta.sync[sy_xcd(xcc)], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(&ta.sync[SY_JOINED], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int spins = 0, good = 1;
        while (ld_agent(&ta.sync[SY_JOINED]) < gridDim.x) {
            if (++spins > ta.spin_limit || ld_agent(&ta.sync[SY_ABORT]) != 0) {
                raise_abort(ta, ABORT_FORMATION);
                good = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        // arrival order inside the XCD deals the workgroups to its teams in turn
        const int on_xcd = (int)ld_agent(&ta.sync[sy_xcd(xcc)]);
        const int sub = arrival % per_xcd;
        s_team = xcc * per_xcd + sub;
        s_rank = arrival / per_xcd;
        s_size = (on_xcd - sub + per_xcd - 1) / per_xcd;
        flag = good;
        if (good && blockIdx.x == 0) {
            for (int t = 0; t < MAX_TEAMS; ++t) {
                const int x = t / per_xcd, k = t - x * per_xcd;
                unsigned size = 0;
                if (x < MAX_XCDS) {
                    const int n = (int)ld_agent(&ta.sync[sy_xcd(x)]);
                    size = (unsigned)((n - k + per_xcd - 1) / per_xcd);
                }
                __hip_atomic_store(&ta.host->team_size[t], size, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __hip_atomic_store(&ta.host->ready, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
    __syncthreads();
    if (!flag) return;
    const int team = s_team, rank = s_rank, tsize = s_size;
    char *arena = ta.arena + (long)team * ta.arena_bytes;
    char *team_mem = ta.team_mem + (long)team * TEAM_MEM_BYTES;
    DevOp *prog = reinterpret_cast<DevOp *>(team_mem);
    unsigned long long my_seq = ta.last_seq[team];
    unsigned long long epoch = 0;
    const ResTable *table = nullptr;   // the residency table in use (the team's device copy)
    unsigned long long table_seq = 0;  // its number (0: a fresh launch finds nothing in the LDS stores)
    unsigned *present = reinterpret_cast<unsigned *>(team_mem + TEAM_TABLE_OFFSET + TEAM_TABLE_BYTES);
    // (cleared by the whole team; the barrier inside the first table fetch comes before any of them is read)
    for (int i = rank * STREAM_THREADS + (int)threadIdx.x; i < RES_MAX_ENTRIES; i += tsize * STREAM_THREADS)
        __hip_atomic_store(&present[i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long *go = &ta.sync[sy_go(team)];
    unsigned long long *slot = &ta.sync[sy_slot(team)];
    const unsigned long long *posted = &ta.host->posted[team * 8];

    for (unsigned long long iter = 1;; ++iter) {
        // ---- wait for the next post: the leader polls the mailbox and hands the post to its team
        if (threadIdx.x == 0) {
            int good = 1;
            if (rank == 0) {
                const long long t0 = wall_clock64();
                unsigned long long cmd = TEAM_STOP, n_ops = 0, seq = my_seq;
                const TeamPost *post = &ta.host->post[team][0];
                for (;;) {
                    if (ld_sys(posted) > my_seq) {
                        // The host wrote the post (and, before that, the program and the table it names) ahead of
                        // the counter, with a release fence between; this thread has the counter's value in hand
                        // before it asks for the post, and every load of the post goes to host memory itself.
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");
                        st_agent(&ta.sync[SY_CLOCK], (unsigned long long)wall_clock64());  // any team's post keeps all teams alive
                        seq = my_seq + 1;
                        post = &ta.host->post[team][seq % POST_RING];
                        cmd = (unsigned long long)__hip_atomic_load(&post->cmd, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                        n_ops = (unsigned long long)__hip_atomic_load(&post->n_ops, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                        // (a slot is rewritten only after `done` has passed the post that sat in it, so the words
                        // belong to post `seq`; its first word says so)
                        if (ld_sys(&post->seq) != seq) {
                            raise_abort(ta, ABORT_POST);
                            cmd = TEAM_STOP;
                        }
                        break;
                    }
                    const long long last = std::max(t0, (long long)ld_agent(&ta.sync[SY_CLOCK]));
                    if (__hip_atomic_load(&ta.host->stop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0 ||
                        ld_agent(&ta.sync[SY_ABORT]) != 0 || wall_clock64() - last > ta.idle_ticks)
                        break;  // cmd stays TEAM_STOP
                    __builtin_amdgcn_s_sleep(8);
                }
                st_agent(&slot[0], cmd | (n_ops << 32));
                st_agent(&slot[1], ld_sys(reinterpret_cast<const unsigned long long *>(&post->prog)));
                st_agent(&slot[2], ld_sys(reinterpret_cast<const unsigned long long *>(&post->input)));
                st_agent(&slot[3], ld_sys(reinterpret_cast<const unsigned long long *>(&post->logits)));
                st_agent(&slot[4], seq);
                st_agent(&slot[5], ld_sys(reinterpret_cast<const unsigned long long *>(&post->table)));
                st_agent(&slot[6], ld_sys(&post->table_seq));
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the slot is in the L2 before go moves
                st_agent(go, iter);
            } else {
                const long long t0 = wall_clock64();
                while (ld_agent(go) < iter) {
                    // The leader polls for as long as any team of the kernel is at work or gets posts (they stamp the
                    // shared clock), which may be far longer than its own team has anything to do: the bound counts
                    // from the last stamp, after which the leader itself gives up within the idle limit.
                    const long long last = std::max(t0, (long long)ld_agent(&ta.sync[SY_CLOCK]));
                    if (ld_agent(&ta.sync[SY_ABORT]) != 0 || wall_clock64() - last > 4 * ta.idle_ticks + 100000000ll) {
                        raise_abort(ta, ABORT_GO);
                        good = 0;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(2);
                }
            }
            if (good)
                for (int k = 0; k < 7; ++k) s_slot[k] = ld_agent(&slot[k]);
            invalidate_vector_l1();
            flag = good;
        }
        __syncthreads();
        if (!flag) return;
        const int cmd = (int)(s_slot[0] & 0xFFFFFFFFull), n_ops = min((int)(s_slot[0] >> 32), TEAM_PROG_MAX_OPS);
        if (cmd != TEAM_RUN) return;
        // ---- the cached SubGraph this query runs under: bring the LDS stores up to its table if they hold another
        if (s_slot[6] != table_seq) {
            if (!fetch_table(ta, reinterpret_cast<const ResTable *>(s_slot[5]), team_mem + TEAM_TABLE_OFFSET, team, rank, tsize,
                             epoch, s_hdr, &flag, &table))
                return;
            if (table)
                install_slabs(table, present, rank, store, dyn_lds, s_layer_mask);
            else if (threadIdx.x < RES_MAX_LAYERS / 32)
                s_layer_mask[threadIdx.x] = 0u;
            __syncthreads();
            table_seq = s_slot[6];
        }
        const void *input = reinterpret_cast<const void *>(s_slot[2]);
        void *logits = reinterpret_cast<void *>(s_slot[3]);
        const unsigned long long seq = s_slot[4];
        // the query's program comes from the host's pinned pool into the team's memory
        team_fetch(reinterpret_cast<unsigned long long *>(prog), reinterpret_cast<const unsigned long long *>(s_slot[1]),
                   n_ops * (int)(sizeof(DevOp) / 8), rank, tsize);
        epoch += 1;
        if (!team_barrier<false>(ta, team, tsize, epoch, &flag)) return;

        // ---- run the query inside this XCD
        constexpr int OP_WORDS = (int)(sizeof(DevOp) / sizeof(int));
        static_assert(OP_WORDS <= 64, "one lane per descriptor word");
        // lane k of every wave carries word k of the next op's descriptor, fetched one op ahead; the
        // words then move to scalar registers lane by lane, without a trip through LDS
        const int dlane = (int)(threadIdx.x & 63);
        // (loaded around the L1, which may hold the previous query's program)
        auto prog_word = [&](int i, int k) {
            return __hip_atomic_load(reinterpret_cast<const int *>(prog + i) + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        int next_word = (dlane < OP_WORDS && n_ops > 0) ? prog_word(0, dlane) : 0;
        for (int i = 0; i < n_ops; ++i) {
            DevOp uop;
            {
                union {
                    DevOp o;
                    int w[OP_WORDS];
                } u;
#pragma unroll
                for (int k = 0; k < OP_WORDS; ++k) u.w[k] = __builtin_amdgcn_readlane(next_word, k);
                uop = u.o;
            }
            if (dlane < OP_WORDS && i + 1 < n_ops) next_word = prog_word(i + 1, dlane);
            {
                auto fix = [&](const void *p) -> const void * {
                    return p ? static_cast<const void *>(arena + (reinterpret_cast<long>(p) - 1)) : nullptr;
                };
                uop.conv.x = fix(uop.conv.x), uop.conv.y = const_cast<void *>(fix(uop.conv.y)), uop.conv.res = fix(uop.conv.res);
                uop.pool.x = fix(uop.pool.x), uop.pool.y = const_cast<void *>(fix(uop.pool.y));
                uop.pool.gate = static_cast<const float *>(fix(uop.pool.gate));
                if (uop.in_patch) uop.conv.x = input;
                if (uop.out_patch) uop.conv.y = logits;
            }
            uop = uniform_op(uop);  // the arena and the caller's buffers came through LDS
            if (ta.trace && i == 0 && rank == 0 && threadIdx.x == 0) ta.trace[team * TRACE_SLOTS] = wall_clock64();
            ResView rv{nullptr, nullptr, store, unit_list};
            // (asked of the mask in LDS: a look into the table costs a round trip to the L2 in front of every op)
            if (table && uop.layer >= 0 && uop.layer < RES_MAX_LAYERS &&
                ((__builtin_amdgcn_readfirstlane((int)s_layer_mask[uop.layer >> 5]) >> (uop.layer & 31)) & 1) != 0) {
                rv.layer = &table->layers[uop.layer];
                rv.entries = table->entries + rv.layer->first_entry;
            }
            if (uop.kind != DEV_NONE) {  // (the slot of an op that a fused op before it has already done)
                run_op<AUX_SC1, AUX_PLAIN, true, OPS>(uop, lds, rank, tsize, rv, tb);
                epoch += 1;
                if (!team_barrier<false>(ta, team, tsize, epoch, &flag)) return;
            }
            if (ta.trace && rank == 0 && threadIdx.x == 0 && i + 1 < TRACE_SLOTS)
                ta.trace[team * TRACE_SLOTS + i + 1] = wall_clock64();
            // a team at work keeps all teams alive: were the idle ones to leave during a query that takes
            // longer than the idle limit, a post to one of them would wait for the whole kernel to leave
            if (rank == 0 && threadIdx.x == 0) st_agent(&ta.sync[SY_CLOCK], (unsigned long long)wall_clock64());
        }
        // every workgroup's (write-through) logits stores have completed: report
        if (rank == 0 && threadIdx.x == 0)
            __hip_atomic_store(&ta.host->done[team * 8], seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        my_seq = seq;
    }
}

}  // namespace sushi
