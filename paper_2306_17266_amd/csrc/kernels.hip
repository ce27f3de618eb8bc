// Device kernels of the SubNet forward pass (gfx950 / CDNA4).  Layouts: see kernels.h.
//
// Dense convolutions and fully connected layers in bf16 run as implicit GEMMs on the matrix cores
// (v_mfma_f32_16x16x32_bf16, float32 accumulation): filters are the MFMA rows, output pixels the
// MFMA columns, so each lane ends up with four consecutive output channels of one pixel and the
// channels-last store is an 8-byte write.  Both operands are read straight from global memory
// in operand order (16 bytes per lane): the packed weight layout makes a 16 x 32 weight fragment
// four 256-byte runs, and a channels-last activation row supplies 64 contiguous bytes per pixel.
// Everything else (depthwise, pooling, squeeze-excite gating, the float32 mode) is bandwidth
// work on the vector ALUs with 16- or 32-byte accesses per lane.
#include "kernels.h"
#include "device_common.h"

#include <algorithm>

namespace sushi {

static const signed char h_dw_dr[49] = {DW_DR_LIST};
static const signed char h_dw_ds[49] = {DW_DS_LIST};

void dw_tap_offsets(int t, int *dr, int *ds) {
    *dr = h_dw_dr[t];
    *ds = h_dw_ds[t];
}

hipError_t upload_tap_table() { return hipSuccess; }

// ------------------------------------------------------------------ dense conv, vector ALUs
// One thread: one output pixel x 4 consecutive filters.  Serves the float32 mode, the 3-channel
// stem and fully connected layers in float32.  y = act(scale * conv + shift (+ res)).

template <typename T>
__global__ __launch_bounds__(256) void conv_direct_kernel(ConvArgs a) {
    const int groups = (a.K + 3) >> 2;
    const long total = (long)a.B * a.P * a.Q * groups;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int fg = (int)(idx % groups);
    const long m = idx / groups;
    const int qq = (int)(m % a.Q);
    const int pp = (int)((m / a.Q) % a.P);
    const int n = (int)(m / ((long)a.Q * a.P));
    const int fb = fg * 4;
    const T *x = static_cast<const T *>(a.x);
    const T *w = static_cast<const T *>(a.w);
    const int cgs = (a.C + 7) >> 3;
    const bool vec = (a.C & 7) == 0;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int tap = 0; tap < a.R * a.R; ++tap) {
        const int h = pp * a.stride - a.pad + tap / a.R;
        const int v = qq * a.stride - a.pad + tap % a.R;
        if (h < 0 || h >= a.H || v < 0 || v >= a.W) continue;
        const T *xp = x + (((long)n * a.H + h) * a.W + v) * a.C;
        for (int cg = 0; cg < cgs; ++cg) {
            float xv[8];
            if (vec) {
                load8(xp + cg * 8, xv);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) xv[j] = (cg * 8 + j < a.C) ? ld1(xp + cg * 8 + j) : 0.f;
            }
            const T *wp = w + (((long)tap * a.CG + cg) * a.Kpad + fb) * 8;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (fb + i < a.Kpad) {
                    float wv[8];
                    load8(wp + i * 8, wv);
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[i] = fmaf(wv[j], xv[j], acc[i]);
                }
            }
        }
    }
    const long obase = m * a.K + fb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (fb + i >= a.K) break;
        float v = acc[i] * (a.scale ? a.scale[fb + i] : 1.0f) + a.shift[fb + i];
        if (a.res) v += ld1(static_cast<const T *>(a.res) + obase + i);
        v = activate(v, a.act, a.hsigmoid);
        if (a.out_f32)
            static_cast<float *>(a.y)[obase + i] = v;
        else
            st1(static_cast<T *>(a.y) + obase + i, v);
    }
}

// ------------------------------------------------------------------ dense conv, bf16 matrix cores

// Epilogue of one 16 x 16 accumulator tile: the lane holds pixel m and filters fbase .. fbase+3.
// y = act(scale * acc + shift (+ res)), stored channels-last as bf16 or float32.
__device__ __forceinline__ void store_tile(const ConvArgs &a, const f32x4_t acc, int fbase, int m, int M) {
    if (fbase >= a.K || m >= M) return;
    const int nf = min(4, a.K - fbase);
    const bool vec = nf == 4 && (a.K & 3) == 0;
    const long o = (long)m * a.K + fbase;
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float sc = (a.scale && i < nf) ? a.scale[fbase + i] : 1.0f;
        const float sh = i < nf ? a.shift[fbase + i] : 0.0f;
        v[i] = acc[i] * sc + sh;
    }
    if (a.res) {
        const uint16_t *rp = static_cast<const uint16_t *>(a.res) + o;
        if (vec) {
            const uint2 r = *reinterpret_cast<const uint2 *>(rp);
            v[0] += bf2f(r.x & 0xFFFFu), v[1] += bf2f(r.x >> 16), v[2] += bf2f(r.y & 0xFFFFu), v[3] += bf2f(r.y >> 16);
        } else {
            for (int i = 0; i < nf; ++i) v[i] += bf2f(rp[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = activate(v[i], a.act, a.hsigmoid);
    if (a.out_f32) {
        float *yp = static_cast<float *>(a.y) + o;
        if (vec)
            *reinterpret_cast<float4 *>(yp) = make_float4(v[0], v[1], v[2], v[3]);
        else
            for (int i = 0; i < nf; ++i) yp[i] = v[i];
    } else {
        uint16_t *yp = static_cast<uint16_t *>(a.y) + o;
        if (vec) {
            uint2 r;
            r.x = pack_bf16x2(v[0], v[1]), r.y = pack_bf16x2(v[2], v[3]);
            *reinterpret_cast<uint2 *>(yp) = r;
        } else {
            for (int i = 0; i < nf; ++i) yp[i] = (uint16_t)f2bf(v[i]);
        }
    }
}

// Large problems (many pixels and filters; batch 16): the classic shared-memory tiling.  A workgroup
// of four waves (2 x 2) computes BN filters x BM pixels with 32 x 32 x 16 MFMAs.  Per reduction step
// (one tap, 32 channels) the BN x 32 weight tile and the BM x 32 activation tile are staged in LDS as
// [8-channel group][row] 16-byte cells, so a wave's operand read is four contiguous 512-byte runs;
// the next step's global loads are in flight (registers) while the current step is multiplied, and
// the two LDS buffers alternate with one barrier per step.  Consecutive workgroup ids land on
// different XCDs, so tile t is served by workgroup id (t % per_xcd) * 8 + t / per_xcd: tiles that
// share a weight tile run on the same XCD and meet in its L2.
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

template <int BN, int BM>
__global__ __launch_bounds__(256) void conv_mfma_kernel(ConvArgs a, int tiles_f, int tiles_m) {
    constexpr int TF = BN / 64, TM = BM / 64;  // 32 x 32 tiles per wave along filters / pixels
    constexpr int NA = BN / 64, NB = BM / 64;  // 16-byte cells each thread stages per step
    constexpr int SA = BN + 4, SB = BM + 4;    // padded row counts of one channel-group plane
    __shared__ uint4 sA[2][4 * SA];
    __shared__ uint4 sB[2][4 * SB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wf = wave >> 1, wm = wave & 1;
    const int M = a.B * a.P * a.Q;
    const int ntiles = tiles_f * tiles_m;
    const int per_xcd = (ntiles + 7) >> 3;
    int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)gridDim.x != per_xcd * 8) tile = blockIdx.x;
    if (tile >= ntiles) return;
    const int tf = tile / tiles_m, tm = tile - tf * tiles_m;
    const int f0 = tf * BN, m0 = tm * BM;
    const uint16_t *x = static_cast<const uint16_t *>(a.x);
    const uint16_t *w = static_cast<const uint16_t *>(a.w);

    // what this thread stages: weight cells (group akg, filter af[i]) and activation cells (group bkg, pixel i)
    int a_off[NA], a_kg[NA], a_lds[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int c = tid + 256 * i;
        a_kg[i] = c / BN;
        const int f = c - a_kg[i] * BN;
        a_off[i] = min(f0 + f, a.Kpad - 1) * 8;
        a_lds[i] = a_kg[i] * SA + f;
    }
    int b_kg[NB], b_lds[NB], pn[NB], ph[NB], pw[NB];
    bool pv[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int c = tid + 256 * i;
        b_kg[i] = c & 3;
        const int pix = c >> 2;
        b_lds[i] = b_kg[i] * SB + pix;
        const int m = m0 + pix;
        pv[i] = m < M;
        const int mm = pv[i] ? m : 0;
        const int qq = mm % a.Q, pp = (mm / a.Q) % a.P;
        pn[i] = mm / (a.Q * a.P);
        ph[i] = pp * a.stride - a.pad;
        pw[i] = qq * a.stride - a.pad;
    }
    const int csteps = (a.C + 31) >> 5;
    const int nsteps = a.R * a.R * csteps;
    // Register sets for the steps in flight: set j holds the cells of the steps congruent to j modulo PD.
    constexpr int PD = 1;
    uint4 ra[PD][NA], rb[PD][NB];
    auto gload = [&](int step, uint4 *qa, uint4 *qb) {
        const int tap = step / csteps;
        const int c0 = (step - tap * csteps) * 32;
        const int dr = tap / a.R, ds = tap - dr * a.R;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int cg = min((c0 >> 3) + a_kg[i], a.CG - 1);
            qa[i] = *reinterpret_cast<const uint4 *>(w + ((long)tap * a.CG + cg) * a.Kpad * 8 + a_off[i]);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int h = ph[i] + dr, v = pw[i] + ds, c = c0 + b_kg[i] * 8;
            const bool ok = pv[i] && c < a.C && h >= 0 && h < a.H && v >= 0 && v < a.W;
            const long off = (((long)pn[i] * a.H + (ok ? h : 0)) * a.W + (ok ? v : 0)) * a.C + (ok ? c : 0);
            qb[i] = *reinterpret_cast<const uint4 *>(x + off);
            if (!ok) qb[i] = make_uint4(0, 0, 0, 0);
        }
    };
    auto sstore = [&](int buf, const uint4 *qa, const uint4 *qb) {
#pragma unroll
        for (int i = 0; i < NA; ++i) sA[buf][a_lds[i]] = qa[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) sB[buf][b_lds[i]] = qb[i];
    };

    f32x16_t acc[TF][TM];
#pragma unroll
    for (int i = 0; i < TF; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[i][j][k] = 0.f;

    const int l32 = lane & 31, kh = lane >> 5;
    // prologue: step 0 into LDS, steps 1 .. PD-1 on their way
    gload(0, ra[0], rb[0]);
    sstore(0, ra[0], rb[0]);
#pragma unroll
    for (int j = 1; j < PD; ++j)
        if (j < nsteps) gload(j, ra[j], rb[j]);
    __syncthreads();
    for (int s0 = 0; s0 < nsteps; s0 += PD) {
#pragma unroll
        for (int j = 0; j < PD; ++j) {
            const int step = s0 + j;
            if (step >= nsteps) break;
            const int buf = step & 1;
            // set j is free (its step is in LDS): start the loads of step + PD
            if (step + PD < nsteps) gload(step + PD, ra[j], rb[j]);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                Frag fa[TF], fb[TM];
#pragma unroll
                for (int i = 0; i < TF; ++i) fa[i].u = sA[buf][(2 * h + kh) * SA + wf * (BN / 2) + i * 32 + l32];
#pragma unroll
                for (int jm = 0; jm < TM; ++jm) fb[jm].u = sB[buf][(2 * h + kh) * SB + wm * (BM / 2) + jm * 32 + l32];
#pragma unroll
                for (int i = 0; i < TF; ++i)
#pragma unroll
                    for (int jm = 0; jm < TM; ++jm)
                        acc[i][jm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[jm].v, acc[i][jm], 0, 0, 0);
            }
            // the next step's cells were requested PD-1 steps ago
            if (step + 1 < nsteps) sstore(buf ^ 1, ra[(j + 1) % PD], rb[(j + 1) % PD]);
            __syncthreads();
        }
    }
    // a 32 x 32 accumulator: lane holds pixel column l32 and, for jj = 0..3, filters 8*jj + 4*kh .. +3
#pragma unroll
    for (int i = 0; i < TF; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int m = m0 + wm * (BM / 2) + j * 32 + l32;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const f32x4_t v = {acc[i][j][4 * jj], acc[i][j][4 * jj + 1], acc[i][j][4 * jj + 2], acc[i][j][4 * jj + 3]};
                store_tile(a, v, f0 + wf * (BN / 2) + i * 32 + 8 * jj + 4 * kh, m, M);
            }
        }
}

// Small problems (batch-1 layers, FC): latency decides, so the reduction is split over the WK waves
// of the workgroup (WK = blockDim.x / 64, chosen by the host), every wave issues the loads of U steps
// before the first MFMA, and the partial sums are added in a fixed order through LDS.  One
// workgroup computes FT x PT tiles.  Loads are unconditional (addresses clamped into the tensor);
// masked activations are zeroed afterwards, which also covers the spatial zero padding.
// IN32: the input is a float32 vector per image (H = W = 1): every value is split into two bf16 terms,
// x = hi + lo with hi = bf16(x) and lo = bf16(x - hi), and both are multiplied with the same weight fragment, so
// the product carries about 16 bits of the input's mantissa instead of 8.
template <int FT, int PT, int U, int MAXT, bool IN32 = false>
__global__ __launch_bounds__(MAXT) void conv_mfma_splitk_kernel(ConvArgs a) {
    extern __shared__ float red[];  // [WK][FT*PT][4][64]
    const int WK = blockDim.x >> 6;
    const int lane = threadIdx.x & 63;
    const int wk = threadIdx.x >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const int M = a.B * a.P * a.Q;
    const int n_pgroups = (M + 16 * PT - 1) / (16 * PT);
    const int pgroup = blockIdx.x % n_pgroups, ftile = blockIdx.x / n_pgroups;
    const int f0 = ftile * FT * 16;
    const int m0 = pgroup * PT * 16;
    const uint16_t *x = static_cast<const uint16_t *>(a.x);
    const uint16_t *w = static_cast<const uint16_t *>(a.w);

    int pn[PT], ph[PT], pw[PT];
    bool pv[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        const int m = m0 + pt * 16 + l16;
        pv[pt] = m < M;
        const int mm = pv[pt] ? m : 0;
        const int qq = mm % a.Q, pp = (mm / a.Q) % a.P;
        pn[pt] = mm / (a.Q * a.P);
        ph[pt] = pp * a.stride - a.pad;
        pw[pt] = qq * a.stride - a.pad;
    }
    int fw[FT];
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) fw[ft] = min(f0 + ft * 16 + l16, a.Kpad - 1) * 8;

    f32x4_t acc[FT][PT];
#pragma unroll
    for (int ft = 0; ft < FT; ++ft)
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) acc[ft][pt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const int csteps = (a.C + 31) >> 5;
    const int nsteps = a.R * a.R * csteps;
    for (int base = wk; base < nsteps; base += WK * U) {
        Frag fa[U][FT], fb[U][PT];
        Frag fb2[IN32 ? U : 1][IN32 ? PT : 1];  // IN32: the second four floats of the lane's eight
        bool ok[U][PT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int step = base + u * WK;
            const bool live = step < nsteps;
            const int st = live ? step : 0;
            const int tap = st / csteps;
            const int c0 = (st - tap * csteps) * 32 + kg * 8;
            const int dr = tap / a.R, ds = tap - dr * a.R;
            const bool cv = live && c0 < a.C;
            const int cc = cv ? c0 : 0;
            const uint16_t *wp = w + ((long)tap * a.CG + (cc >> 3)) * a.Kpad * 8;
#pragma unroll
            for (int ft = 0; ft < FT; ++ft) fa[u][ft].u = *reinterpret_cast<const uint4 *>(wp + fw[ft]);
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                const int h = ph[pt] + dr, v = pw[pt] + ds;
                ok[u][pt] = cv && pv[pt] && h >= 0 && h < a.H && v >= 0 && v < a.W;
                const int hh = ok[u][pt] ? h : 0, vv = ok[u][pt] ? v : 0;
                const long e0 = (((long)pn[pt] * a.H + hh) * a.W + vv) * a.C + cc;
                if (IN32) {
                    const float *xf = static_cast<const float *>(a.x) + e0;
                    fb[u][pt].u = *reinterpret_cast<const uint4 *>(xf);
                    fb2[IN32 ? u : 0][IN32 ? pt : 0].u = *reinterpret_cast<const uint4 *>(xf + 4);
                } else {
                    fb[u][pt].u = *reinterpret_cast<const uint4 *>(x + e0);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int pt = 0; pt < PT; ++pt)
                if (!ok[u][pt]) {
                    fb[u][pt].u = make_uint4(0, 0, 0, 0);
                    if (IN32) fb2[IN32 ? u : 0][IN32 ? pt : 0].u = make_uint4(0, 0, 0, 0);
                }
            if (IN32) {
#pragma unroll
                for (int pt = 0; pt < PT; ++pt) {
                    Frag hi, lo;
                    split_f32x8(fb[u][pt].u, fb2[IN32 ? u : 0][IN32 ? pt : 0].u, &hi.u, &lo.u);
#pragma unroll
                    for (int ft = 0; ft < FT; ++ft) {
                        acc[ft][pt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[u][ft].v, hi.v, acc[ft][pt], 0, 0, 0);
                        acc[ft][pt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[u][ft].v, lo.v, acc[ft][pt], 0, 0, 0);
                    }
                }
            } else {
#pragma unroll
                for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt)
                        acc[ft][pt] =
                            __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[u][ft].v, fb[u][pt].v, acc[ft][pt], 0, 0, 0);
            }
        }
    }

    if (WK == 1) {
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) store_tile(a, acc[ft][pt], f0 + ft * 16 + kg * 4, m0 + pt * 16 + l16, M);
        return;
    }
    constexpr int NT = FT * PT;
#pragma unroll
    for (int ft = 0; ft < FT; ++ft)
#pragma unroll
        for (int pt = 0; pt < PT; ++pt)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[((wk * NT + ft * PT + pt) * 4 + i) * 64 + lane] = acc[ft][pt][i];
    __syncthreads();
    // wave t finishes tile t: partial sums of wave 0, 1, ... in that order
    for (int t = wk; t < NT; t += WK) {
        f32x4_t s = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < WK; ++k)
#pragma unroll
            for (int i = 0; i < 4; ++i) s[i] += red[((k * NT + t) * 4 + i) * 64 + lane];
        const int ft = t / PT, pt = t - ft * PT;
        store_tile(a, s, f0 + ft * 16 + kg * 4, m0 + pt * 16 + l16, M);
    }
}

// ------------------------------------------------------------------ depthwise k x k
// One thread: one output pixel x 8 channels, taps in ring order (prefix of the stored 7x7).

template <typename T>
__global__ __launch_bounds__(256) void dwconv_kernel(ConvArgs a) {
    const int cgs = a.K >> 3;
    const long total = (long)a.B * a.P * a.Q * cgs;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cg = (int)(idx % cgs);
    const long m = idx / cgs;
    const int qq = (int)(m % a.Q);
    const int pp = (int)((m / a.Q) % a.P);
    const int n = (int)(m / ((long)a.Q * a.P));
    const int c = cg * 8;
    const T *x = static_cast<const T *>(a.x);
    const T *w = static_cast<const T *>(a.w);
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    const int ntaps = a.R * a.R;
    for (int t = 0; t < ntaps; ++t) {
        const int h = pp * a.stride + c_dw_dr[t];
        const int v = qq * a.stride + c_dw_ds[t];
        if (h < 0 || h >= a.H || v < 0 || v >= a.W) continue;
        float xv[8], wv[8];
        load8(x + (((long)n * a.H + h) * a.W + v) * a.C + c, xv);
        load8(w + (long)t * a.Kpad + c, wv);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = fmaf(wv[j], xv[j], acc[j]);
    }
    float sc[8], sh[8];
    load8(a.scale + c, sc);
    load8(a.shift + c, sh);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = activate(acc[j] * sc[j] + sh[j], a.act, 0);
    store8(static_cast<T *>(a.y) + m * a.K + c, acc);
}

// ------------------------------------------------------------------ pooling and gating

template <typename T>
__global__ __launch_bounds__(256) void maxpool_kernel(PoolArgs a) {
    const int cgs = a.C >> 3;
    const long total = (long)a.B * a.P * a.Q * cgs;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cg = (int)(idx % cgs);
    const long m = idx / cgs;
    const int qq = (int)(m % a.Q);
    const int pp = (int)((m / a.Q) % a.P);
    const int n = (int)(m / ((long)a.Q * a.P));
    const T *x = static_cast<const T *>(a.x);
    float best[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) best[j] = -3.4028235e38f;
    for (int r = 0; r < 3; ++r) {
        const int h = pp * 2 - 1 + r;
        if (h < 0 || h >= a.H) continue;
        for (int s = 0; s < 3; ++s) {
            const int v = qq * 2 - 1 + s;
            if (v < 0 || v >= a.W) continue;
            float xv[8];
            load8(x + (((long)n * a.H + h) * a.W + v) * a.C + cg * 8, xv);
#pragma unroll
            for (int j = 0; j < 8; ++j) best[j] = fmaxf(best[j], xv[j]);
        }
    }
    store8(static_cast<T *>(a.y) + m * a.C + cg * 8, best);
}

// Global average over H x W.  Workgroup = 32 pixel lanes x 8 channel groups; partial sums are
// combined by a fixed binary tree, so the result does not depend on timing.
template <typename T>
__global__ __launch_bounds__(256) void gap_kernel(PoolArgs a) {
    __shared__ float part[32][8][9];
    const int cgs = a.C >> 3;
    const int blocks_per_image = (cgs + 7) >> 3;
    const int n = blockIdx.x / blocks_per_image;
    const int cgi = threadIdx.x & 7, pl = threadIdx.x >> 3;
    const int cg = (blockIdx.x % blocks_per_image) * 8 + cgi;
    const int hw = a.H * a.W;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    if (cg < cgs) {
        const T *x = static_cast<const T *>(a.x) + (long)n * hw * a.C + cg * 8;
        for (int p = pl; p < hw; p += 32) {
            float xv[8];
            load8(x + (long)p * a.C, xv);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += xv[j];
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) part[pl][cgi][j] = acc[j];
    __syncthreads();
    for (int s = 16; s > 0; s >>= 1) {
        if (pl < s)
#pragma unroll
            for (int j = 0; j < 8; ++j) part[pl][cgi][j] += part[pl + s][cgi][j];
        __syncthreads();
    }
    if (pl == 0 && cg < cgs) {
        float o[8];
        const float inv = 1.0f / (float)hw;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = part[0][cgi][j] * inv;
        if (a.out_f32)
            store8(static_cast<float *>(a.y) + (long)n * a.C + cg * 8, o);
        else
            store8(static_cast<T *>(a.y) + (long)n * a.C + cg * 8, o);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gate_kernel(PoolArgs a) {
    const int cgs = a.C >> 3;
    const long total = (long)a.B * a.H * a.W * cgs;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cg = (int)(idx % cgs);
    const long m = idx / cgs;
    const int n = (int)(m / ((long)a.H * a.W));
    float xv[8], g[8];
    load8(static_cast<const T *>(a.x) + m * a.C + cg * 8, xv);
    load8(a.gate + (long)n * a.C + cg * 8, g);
#pragma unroll
    for (int j = 0; j < 8; ++j) xv[j] *= g[j];
    store8(static_cast<T *>(a.y) + m * a.C + cg * 8, xv);
}

// ------------------------------------------------------------------ cache sweep

__global__ __launch_bounds__(256) void cold_sweep_kernel(const uint4 *buf, size_t n, uint4 *sink) {
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const uint4 v = buf[i];
        acc.x ^= v.x, acc.y ^= v.y, acc.z ^= v.z, acc.w ^= v.w;
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u && threadIdx.x == 0) sink[blockIdx.x] = acc;  // (never, for a zeroed buffer)
}

hipError_t launch_cold_sweep(const void *buf, size_t bytes, void *sink, hipStream_t s) {
    hipLaunchKernelGGL(cold_sweep_kernel, dim3(2048), dim3(256), 0, s, static_cast<const uint4 *>(buf), bytes / 16,
                       static_cast<uint4 *>(sink));
    return hipGetLastError();
}

// ------------------------------------------------------------------ static scratch

// Activation buffers of sushi_infer_static.  In host code the array's name only stands for the symbol; the
// device address (one per GPU that loaded this code object) comes from hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

hipError_t static_scratch(int device, void **ptr) {
    constexpr int MAX_DEVICES = 64;
    static void *ptrs[MAX_DEVICES] = {};
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (!ptrs[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        ptrs[device] = p;
    }
    *ptr = ptrs[device];
    return hipSuccess;
}

// ------------------------------------------------------------------ launchers

static inline unsigned blocks_for(long total) { return (unsigned)((total + 255) / 256); }

template <int BN, int BM>
static hipError_t launch_mfma(const ConvArgs &a, hipStream_t s) {
    const int M = a.B * a.P * a.Q;
    const int tiles_m = (M + BM - 1) / BM, tiles_f = (a.K + BN - 1) / BN;
    const int per_xcd = (tiles_m * tiles_f + 7) / 8;
    hipLaunchKernelGGL((conv_mfma_kernel<BN, BM>), dim3(per_xcd * 8), dim3(256), 0, s, a, tiles_f, tiles_m);
    return hipGetLastError();
}

template <int FT, int PT, int U, int MAXT, bool IN32 = false>
static hipError_t launch_splitk(const ConvArgs &a, int wk, hipStream_t s) {
    const int M = a.B * a.P * a.Q;
    const int n_pgroups = (M + 16 * PT - 1) / (16 * PT);
    const int n_ftiles = (a.K + 16 * FT - 1) / (16 * FT);
    wk = std::max(1, std::min(wk, MAXT / 64));
    const size_t lds = wk > 1 ? (size_t)wk * FT * PT * 256 * sizeof(float) : 0;
    hipLaunchKernelGGL((conv_mfma_splitk_kernel<FT, PT, U, MAXT, IN32>), dim3(n_pgroups * n_ftiles), dim3(64 * wk), lds, s, a);
    return hipGetLastError();
}

const char *kernel_class_name(int kc) {
    static const char *names[KC_COUNT] = {"conv_direct_kernel", "conv_mfma_kernel", "conv_mfma_splitk_kernel",
                                          "dwconv_rows_kernel", "maxpool_kernel",   "gap_kernel",
                                          "gate_kernel",        "sushi_stream_kernel", "sushi_team_kernel",
                                          "conv_patch_kernel",  "conv_i8_kernel",      "int8_pool_fc_kernels"};
    return kc >= 0 && kc < KC_COUNT ? names[kc] : "?";
}

hipError_t launch_conv(const ConvArgs &a, bool bf16, hipStream_t s, int *kc, long patch_min_pixels) {
    const long M = (long)a.B * a.P * a.Q;
    int dummy;
    if (!kc) kc = &dummy;
    *kc = KC_CONV_DIRECT;
    if (!bf16 || (a.C & 7) != 0) {
        const long total = M * ((a.K + 3) / 4);
        if (bf16)
            hipLaunchKernelGGL(conv_direct_kernel<uint16_t>, dim3(blocks_for(total)), dim3(256), 0, s, a);
        else
            hipLaunchKernelGGL(conv_direct_kernel<float>, dim3(blocks_for(total)), dim3(256), 0, s, a);
        return hipGetLastError();
    }
    const long ptiles = (M + 15) / 16, ftiles = (a.K + 15) / 16;
    if (a.in_f32) {  // a float32 vector per image (fully connected layers): always the latency-oriented kernel
        if (a.H * a.W != 1) return hipErrorInvalidValue;
        *kc = KC_CONV_SPLITK;
        return launch_splitk<1, 1, 4, 1024, true>(a, (a.R * a.R * ((a.C + 31) / 32) + 3) / 4, s);
    }
    // (at the threshold itself only long reductions: short ones are quicker in the kernels below)
    if (patch_min_pixels > 0 && M >= patch_min_pixels && (M >= 4 * patch_min_pixels || (long)a.C * a.R * a.R >= 1024)) {
        const hipError_t e = launch_conv_patch(a, s);
        if (e != hipErrorNotSupported) {
            *kc = KC_CONV_PATCH;
            return e;
        }
    }
    // Many tiles: LDS-tiled workgroups; the largest tile that still yields two workgroups per compute unit.
    *kc = KC_CONV_MFMA;
    if (a.K > 64 && ((M + 127) / 128) * ((a.K + 127) / 128) >= 512) return launch_mfma<128, 128>(a, s);
    if (((M + 127) / 128) * ((a.K + 63) / 64) >= 512) return launch_mfma<64, 128>(a, s);
    if (((M + 63) / 64) * ((a.K + 63) / 64) >= 384) return launch_mfma<64, 64>(a, s);
    *kc = KC_CONV_SPLITK;
    // Few tiles: the widest pixel group that still leaves about one workgroup per compute unit, and
    // about four reduction steps per wave.
    const int nsteps = a.R * a.R * ((a.C + 31) / 32);
    const int wk = (nsteps + 3) / 4;
    if (ftiles * ((ptiles + 3) / 4) >= 256) return launch_splitk<1, 4, 4, 512>(a, wk, s);
    if (ftiles * ((ptiles + 1) / 2) >= 256 || ptiles == 2) return launch_splitk<1, 2, 4, 1024>(a, wk, s);
    if (ptiles >= 3 && ptiles <= 4) return launch_splitk<1, 4, 4, 512>(a, wk, s);
    return launch_splitk<1, 1, 4, 1024>(a, wk, s);
}

hipError_t launch_dwconv(const ConvArgs &a, bool bf16, hipStream_t s) {
    const long total = (long)a.B * a.P * a.Q * (a.K >> 3);
    if (bf16) {
        const hipError_t e = launch_dwconv_rows(a, s);
        if (e != hipErrorNotSupported) return e;
    }
    if (bf16)
        hipLaunchKernelGGL(dwconv_kernel<uint16_t>, dim3(blocks_for(total)), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(dwconv_kernel<float>, dim3(blocks_for(total)), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_maxpool(const PoolArgs &a, bool bf16, hipStream_t s) {
    const long total = (long)a.B * a.P * a.Q * (a.C >> 3);
    if (bf16)
        hipLaunchKernelGGL(maxpool_kernel<uint16_t>, dim3(blocks_for(total)), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(maxpool_kernel<float>, dim3(blocks_for(total)), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gap(const PoolArgs &a, bool bf16, hipStream_t s) {
    const unsigned blocks = (unsigned)(a.B * (((a.C >> 3) + 7) >> 3));
    if (bf16)
        hipLaunchKernelGGL(gap_kernel<uint16_t>, dim3(blocks), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(gap_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gate(const PoolArgs &a, bool bf16, hipStream_t s) {
    const long total = (long)a.B * a.H * a.W * (a.C >> 3);
    if (bf16)
        hipLaunchKernelGGL(gate_kernel<uint16_t>, dim3(blocks_for(total)), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(gate_kernel<float>, dim3(blocks_for(total)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace sushi
