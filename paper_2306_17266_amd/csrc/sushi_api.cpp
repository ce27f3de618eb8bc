// C ABI of the library (include/sushi.h): context, SuperNet weight packer, SubGraph cache state,
// per-query plan cache and launch loop, counters.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/sushi.h"
#include "kernels.h"
#include "model.h"
#include "sched.h"
#include "stream_kernel.h"

using namespace sushi;

namespace {

struct Launch {
    int kind;
    ConvArgs conv{};
    PoolArgs pool{};
    QuantArgs quant{};  // int8 mode
    int in_patch = 0, out_patch = 0;  // 1 = pointer is the caller's input / logits buffer
};

struct CachedPlan {
    Plan plan;
    std::vector<Launch> launches;
    uint64_t weight_bytes = 0;
    double alg_bytes = 0.0, alg_flops = 0.0;  // algorithmic traffic and arithmetic of the whole query
    double vec_norm2 = 0.0;           // sum K^2 + C^2 over layers
    uint64_t g_version = ~0ull;       // cache state the two figures below were computed for
    uint64_t resident_bytes = 0;
    double hit_ratio = 0.0;
    // exec mode 1: the launch sequence recorded as a HIP graph, for one (input, logits) pointer pair
    hipGraphExec_t graph = nullptr;
    const void *graph_in = nullptr;
    void *graph_out = nullptr;
    // exec mode 2: the plan as a device program for the stream kernel
    DevOp *d_prog = nullptr;
    int n_dev_ops = 0;
    // exec mode 3: the same program with arena-relative activation pointers, for the team kernel
    DevOp *h_team_prog = nullptr;
    std::vector<DevOp> team_prog;     // host copy (tiling decides which ops can use resident slabs)
    uint64_t table_version = ~0ull;   // residency table the figure below was computed for
    uint64_t lds_bytes = 0;           // weight bytes this SubNet reads from resident LDS slabs
    ~CachedPlan() {
        if (graph) (void)hipGraphExecDestroy(graph);
        if (d_prog) (void)hipFree(d_prog);
    }
};

std::string g_create_error;

}  // namespace

struct sushi_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string err;
    bool loaded = false, bf16 = false;
    bool int8 = false;               // int8 weights and activations (sushi_load_supernet_int8): exec mode 0 only
    int32_t *d_qparams = nullptr;    // int8 mode: per layer mult[Kpad], rshift[Kpad], bias[Kpad]
    int32_t *d_wsum = nullptr;       // int8 mode: per conv layer [channel group of 8][Kpad] prefix sums of the weights
    SuperNet sn;
    void *d_weights = nullptr;
    float *d_params = nullptr;
    size_t weight_elems = 0;
    void *big[N_BIG_BUFS] = {};
    void *small_[N_SMALL_BUFS] = {};
    int arena_batch = 0;
    std::unordered_map<std::string, std::unique_ptr<CachedPlan>> plans;
    std::vector<sushi_layer_dims> G;  // cached SubGraph (empty = nothing cached)
    uint64_t g_version = 0;
    Scheduler sched;
    sushi_stats stats{};
    int exec_mode = 0;
    bool stream_dirty = false;  // work was enqueued on `stream` since the last synchronize
    hipStream_t capture_stream = nullptr;  // graphs are recorded here and replayed on `stream`
    // exec mode 2 (stream kernel): barrier area, abort flag in pinned host memory, barriers counted so far
    unsigned long long *d_sync = nullptr;
    unsigned *h_abort = nullptr;
    unsigned long long epoch_base = 0;
    int stream_wgs = 0, stream_wgs_override = 0;
    int team_wgs = 0, team_wgs_per_cu = 2;
    int teams_per_xcd = 1;  // teams each XCD's workgroups are dealt to (1, 2, 4, 8 or 16)
    int team_size() const { return team_wgs / (MAX_XCDS * teams_per_xcd); }  // workgroups of a team, if they spread evenly
    int spin_limit = 400000;
    void *static_buf = nullptr;  // this device's copy of the library's static scratch array (sushi_infer_static)
    long patch_min_pixels = 3136;  // SUSHI_OPT_PATCH_CONV_MIN_PIXELS
    void *d_sweep = nullptr;  // SUSHI_OPT_COLD_SWEEP_MIB: scratch streamed through the caches before every query
    size_t sweep_bytes = 0;
    // exec mode 3 (team kernel): mailboxes in pinned host memory, per-team arenas, private stream
    TeamHostState *th = nullptr;
    unsigned long long *d_tsync = nullptr;
    char *d_tarena = nullptr;
    long tarena_bytes = 0, tbig_bytes = 0, tsmall_bytes = 0;
    int tarena_batch = 0;
    hipStream_t pstream = nullptr;
    bool team_launched = false;
    unsigned long long posted[MAX_TEAMS] = {};
    int next_team = 0;
    long idle_ticks = 200000;  // 2 ms at 100 MHz
    // residency table of the cached SubGraph (host copies + pinned generations the teams copy from)
    struct ResGen {
        ResTable *table = nullptr;  // pinned HOST: header, then RES_MAX_LAYERS layers, then RES_MAX_ENTRIES entries
        ResLayer *layers = nullptr;
        ResEntry *entries = nullptr;
        unsigned long long last_ref[MAX_TEAMS] = {};  // last post to team t that names this generation
    };
    // While the team kernel runs it fills every compute unit, and hipMalloc / hipFree / hipMemcpy may
    // wait for it to leave.  What the host hands to a running kernel (programs, residency tables)
    // therefore lives in pinned host memory made up front; the teams copy it themselves.
    static constexpr size_t PROG_POOL_BYTES = 96u << 20;
    char *h_prog_pool = nullptr;  // pinned HOST
    size_t prog_pool_used = 0;
    char *d_team_mem = nullptr;   // DEVICE, MAX_TEAMS x TEAM_MEM_BYTES
    static constexpr int N_RES_GENS = 32;
    ResGen res_gens[N_RES_GENS];  // a generation stays untouched while an install post may still name it
    bool gen_valid[N_RES_GENS] = {};  // slot holds a table (false: nothing cached)
    int gen_cur = 0;
    std::vector<ResLayer> h_res_layers;   // the table in force: geometry + valid part per layer
    std::vector<ResEntry> h_res_entries;  // (empty: nothing resident)
    // slab geometry: per layer the tiles and channel groups slabs have room for (grow only), and the placement
    std::vector<int> geo_n, geo_cg;
    std::vector<ResLayer> geo_layers;
    std::vector<ResEntry> geo_entries;
    int geometry = 0, geometry_team_size = 0;
    std::vector<int> geo_present;  // per entry: channel groups a team that served under every table has copied (this geometry)
    uint64_t table_version = 0;
    unsigned long long table_seq = 1;  // number of the table in force, carried by every query post (see TeamPost)
    uint64_t table_bytes = 0;  // bytes of the cached SubGraph that sit in LDS (per team)
    unsigned long long *d_trace = nullptr;
    // per-kernel timing (SUSHI_OPT_KERNEL_TIMING): event pairs around every launch
    bool timing = false;
    struct Pending {
        hipEvent_t a, b;
        int kc;
        double bytes, flops;
        int op_index = -1;
    };
    std::vector<sushi_launch_record> records;  // per-launch durations of mode 0 since timing was switched on
    std::vector<Pending> pending;
    std::vector<hipEvent_t> free_events;
    sushi_kernel_stats kstats[KC_COUNT] = {};
    // the running team kernel's launch, when timed: its event pair and what has been posted to it
    bool team_timed = false;
    Pending team_pending{};
};

namespace {

int fail(sushi_ctx *c, int code, const std::string &msg) {
    if (c) c->err = msg;
    return code;
}

int hip_fail(sushi_ctx *c, hipError_t e, const char *what) {
    return fail(c, SUSHI_EDEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

inline uint16_t to_bf16(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

size_t elem_size(const sushi_ctx *c) { return c->int8 ? 1 : c->bf16 ? 2 : 4; }

// Lays the SuperNet out for the device.  Dense/FC layer: [tap][channel group][filter, padded to 16][8];
// depthwise: [tap in ring order][channel, padded to 16].  Scale/shift/bias: float32 runs, each
// starting on a 32-byte boundary.  Returns the two host staging buffers.
template <typename T, typename Cvt>
void pack_weights(SuperNet &sn, const float *blob, std::vector<T> &w, std::vector<float> &params, Cvt cvt) {
    size_t welems = 0, pfloats = 0;
    for (SuperLayer &L : sn.layers) {
        L.Kpad = (int)round_up(L.Kmax, 16);
        L.CG = L.type == L_DW ? 0 : (L.Cmax + 7) / 8;
        L.pk_w = welems;
        const size_t taps = (size_t)L.Rmax * L.Rmax;
        welems += L.type == L_DW ? taps * L.Kpad : taps * L.CG * L.Kpad * 8;
        welems = round_up(welems, 128);
        if (L.has_scale) {
            L.pk_scale = pfloats;
            pfloats += round_up(L.Kmax, 8);
        }
        L.pk_shift = pfloats;
        pfloats += round_up(L.Kmax, 8);
    }
    w.assign(welems, T(0));
    params.assign(pfloats, 0.f);
    for (const SuperLayer &L : sn.layers) {
        const float *src = blob + L.blob_w;
        T *dst = w.data() + L.pk_w;
        const int R = L.Rmax;
        if (L.type == L_DW) {
            for (int t = 0; t < R * R; ++t) {
                int dr, ds;
                if (R == 1)
                    dr = ds = 0;
                else
                    dw_tap_offsets(t, &dr, &ds);
                const int r = dr + R / 2, s = ds + R / 2;
                for (int k = 0; k < L.Kmax; ++k) dst[(size_t)t * L.Kpad + k] = cvt(src[((size_t)k * R + r) * R + s]);
            }
        } else {
            for (int k = 0; k < L.Kmax; ++k)
                for (int c = 0; c < L.Cmax; ++c)
                    for (int t = 0; t < R * R; ++t)
                        dst[(((size_t)t * L.CG + c / 8) * L.Kpad + k) * 8 + (c & 7)] =
                            cvt(src[((size_t)k * L.Cmax + c) * R * R + t]);
        }
        if (L.has_scale) std::memcpy(&params[L.pk_scale], blob + L.blob_scale, sizeof(float) * L.Kmax);
        std::memcpy(&params[L.pk_shift], blob + L.blob_shift, sizeof(float) * L.Kmax);
    }
}

void free_arena(sushi_ctx *c) {
    for (auto &p : c->big) {
        if (p) (void)hipFree(p);
        p = nullptr;
    }
    for (auto &p : c->small_) {
        if (p) (void)hipFree(p);
        p = nullptr;
    }
    c->arena_batch = 0;
}

sushi_subnet_cfg largest_cfg(const sushi_arch &a) {
    sushi_subnet_cfg m{};
    int res = a.res_choices[0];
    for (int i = 1; i < a.n_res; ++i) res = std::max(res, (int)a.res_choices[i]);
    m.resolution = res;
    auto argmax_d = [](const double *v, int n) {
        int b = 0;
        for (int i = 1; i < n; ++i)
            if (v[i] > v[b]) b = i;
        return b;
    };
    int mind = a.depth_drop_choices[0];
    for (int i = 1; i < a.n_depth_drop; ++i) mind = std::min(mind, (int)a.depth_drop_choices[i]);
    if (a.family == SUSHI_FAMILY_TINY)
        m.depth[0] = a.n_stages - mind;
    else
        for (int s = 0; s < a.n_stages; ++s) m.depth[s] = a.stage_max_depth[s] - mind;
    for (int s = 0; s <= a.n_stages; ++s) m.width_idx[s] = argmax_d(a.width_choices, a.n_width);
    int kb = 0;
    for (int i = 1; i < a.n_kernel; ++i)
        if (a.kernel_choices[i] > a.kernel_choices[kb]) kb = i;
    for (int b = 0; b < SUSHI_MAX_BLOCKS; ++b) {
        m.expand_idx[b] = argmax_d(a.expand_choices, a.n_expand);
        m.kernel_idx[b] = kb;
    }
    return m;
}

// Activation buffers for batches up to `batch`, sized by the largest SubNet at the largest resolution.
int ensure_arena(sushi_ctx *c, int batch) {
    if (batch <= c->arena_batch) return SUSHI_OK;
    Plan p;
    std::string err;
    int rc = plan_subnet(c->sn, largest_cfg(c->sn.arch), batch, p, err);
    if (rc) return fail(c, rc, "arena: " + err);
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
    free_arena(c);
    const size_t big_bytes = round_up(p.max_big_elems * elem_size(c), 256);
    const size_t small_bytes = round_up(std::max<size_t>(p.max_small_elems, 8) * 4, 256);
    for (auto &b : c->big)
        if ((e = hipMalloc(&b, big_bytes)) != hipSuccess) return fail(c, SUSHI_ENOMEM, "hipMalloc(activations)");
    for (auto &b : c->small_)
        if ((e = hipMalloc(&b, small_bytes)) != hipSuccess) return fail(c, SUSHI_ENOMEM, "hipMalloc(vectors)");
    c->arena_batch = batch;
    c->plans.clear();  // cached launches hold arena pointers
    return SUSHI_OK;
}

// Where a plan's activation buffers live: the context's arena, or one block cut into equal parts.
struct BufBase {
    char *block = nullptr;  // null: the context's arena
    size_t big_bytes = 0, small_bytes = 0;
};

void *buf_ptr(sushi_ctx *c, const BufBase &bb, int id, bool small) {
    if (id < 0) return nullptr;
    if (!bb.block) return small ? c->small_[id] : c->big[id];
    return small ? bb.block + N_BIG_BUFS * bb.big_bytes + id * bb.small_bytes : bb.block + id * bb.big_bytes;
}

// Turns a plan into launch records with device pointers bound.
void bind_plan(sushi_ctx *c, CachedPlan &cp, const BufBase &bb = BufBase()) {
    const size_t es = elem_size(c);
    for (const Op &op : cp.plan.ops) {
        Launch L;
        L.kind = op.kind;
        if (op.kind == OP_CONV || op.kind == OP_DW || op.kind == OP_FC) {
            const SuperLayer &S = c->sn.layers[op.layer];
            ConvArgs &a = L.conv;
            a.x = buf_ptr(c, bb, op.in_buf, op.in_small);
            a.y = buf_ptr(c, bb, op.out_buf, op.out_small);
            a.res = buf_ptr(c, bb, op.res_buf, false);
            a.w = static_cast<const char *>(c->d_weights) + S.pk_w * es;
            a.scale = S.has_scale ? c->d_params + S.pk_scale : nullptr;
            a.shift = c->d_params + S.pk_shift;
            a.B = op.B, a.H = op.H, a.W = op.W, a.C = op.C, a.P = op.P, a.Q = op.Q, a.K = op.K;
            a.R = op.r, a.stride = op.stride, a.pad = op.pad, a.Rmax = S.Rmax;
            a.Kpad = S.Kpad, a.CG = S.CG;
            a.act = op.act, a.hsigmoid = op.hsigmoid ? 1 : 0, a.out_f32 = op.out_f32 ? 1 : 0;
            a.in_f32 = (op.in_small && c->bf16) ? 1 : 0;
            if (c->int8) {
                a.scale = nullptr, a.shift = nullptr;
                QuantArgs &q = L.quant;
                q.qmult = c->d_qparams + S.pk_q, q.qshift = q.qmult + S.Kpad, q.qbias = q.qshift + S.Kpad;
                q.wsum = c->d_wsum + S.pk_wsum + (size_t)(std::max(op.C / 8, 1) - 1) * S.Kpad;
                a.CG = S.CG16;
                q.zx = S.qscalars[0], q.zy = S.qscalars[1];
                q.m_res = S.qscalars[2], q.sh_res = std::max(S.qscalars[3], 1), q.z_res = S.qscalars[4];
                q.pool_hw = 1;
                if (op.kind == OP_FC && !cp.launches.empty()) {  // the classifier works on the sums of the pooling before it
                    const PoolArgs &g = cp.launches.back().pool;
                    q.pool_hw = g.H * g.W;
                }
            }
            L.in_patch = op.in_buf == BUF_INPUT;
            L.out_patch = op.out_buf == BUF_LOGITS;
        } else {
            PoolArgs &a = L.pool;
            a.x = buf_ptr(c, bb, op.in_buf, op.in_small);
            a.y = buf_ptr(c, bb, op.out_buf, op.out_small);
            a.gate = static_cast<const float *>(buf_ptr(c, bb, op.gate_buf, true));
            a.B = op.B, a.H = op.H, a.W = op.W, a.C = op.C, a.P = op.P, a.Q = op.Q;
            a.out_f32 = (op.out_f32 && c->bf16) ? 1 : 0;
            if (c->int8 && op.kind == OP_GAP) {  // the zero point of the pooled map: first scalar of the classifier after it
                const size_t next = cp.launches.size() + 1;
                if (next < cp.plan.ops.size() && cp.plan.ops[next].layer >= 0)
                    L.quant.zx = c->sn.layers[cp.plan.ops[next].layer].qscalars[0];
            }
        }
        cp.launches.push_back(L);
    }
    cp.weight_bytes = 0;
    cp.vec_norm2 = 0.0;
    for (const sushi_layer_dims &d : cp.plan.dims) {
        cp.weight_bytes += (uint64_t)d.K * d.C * d.r * d.r * es;
        cp.vec_norm2 += (double)d.K * d.K + (double)d.C * d.C;
    }
}

// Bytes of the SubNet that lie inside the cached SubGraph, and the vector hit ratio (Appendix A.4).
void refresh_residency(sushi_ctx *c, CachedPlan &cp) {
    if (cp.g_version == c->g_version) return;
    cp.g_version = c->g_version;
    cp.resident_bytes = 0;
    cp.hit_ratio = 0.0;
    if (c->G.empty()) return;
    const size_t es = elem_size(c);
    double inter2 = 0.0;
    for (size_t i = 0; i < cp.plan.dims.size(); ++i) {
        const sushi_layer_dims &d = cp.plan.dims[i], &g = c->G[i];
        if (d.K == 0 || g.K == 0) continue;
        const uint64_t k = std::min(d.K, g.K), ch = std::min(d.C, g.C), r = std::min(d.r, g.r);
        cp.resident_bytes += k * ch * r * r * es;
        inter2 += (double)k * k + (double)ch * ch;
    }
    cp.hit_ratio = cp.vec_norm2 > 0 ? std::sqrt(inter2) / std::sqrt(cp.vec_norm2) : 0.0;
}

// Algorithmic traffic and arithmetic of one launch: every input, output, residual, weight and
// scale/shift element of the active slice counted once.
void launch_cost(const sushi_ctx *c, const Launch &L, double *bytes, double *flops) {
    const double es = c->int8 ? 1.0 : c->bf16 ? 2.0 : 4.0;
    if (L.kind == OP_CONV || L.kind == OP_FC || L.kind == OP_DW) {
        const ConvArgs &a = L.conv;
        const double in = (double)a.B * a.H * a.W * a.C, out = (double)a.B * a.P * a.Q * a.K;
        const double taps = (double)a.R * a.R;
        const double wts = L.kind == OP_DW ? a.K * taps : (double)a.K * a.C * taps;
        *bytes = in * (a.in_f32 ? 4.0 : es) + (wts + (a.res ? out : 0.0)) * es + out * (a.out_f32 ? 4.0 : es) + 8.0 * a.K;
        *flops = 2.0 * out * (L.kind == OP_DW ? taps : a.C * taps);
    } else {
        const PoolArgs &a = L.pool;
        const double in = (double)a.B * a.H * a.W * a.C;
        const double out = L.kind == OP_GATE ? in : (double)a.B * a.P * a.Q * a.C;
        *bytes = in * es + out * (a.out_f32 ? 4.0 : es) + (L.kind == OP_GATE ? 4.0 * a.B * a.C : 0.0);
        *flops = L.kind == OP_MAXPOOL ? 9.0 * out : in;
    }
}

hipError_t get_event(sushi_ctx *c, hipEvent_t *ev) {
    if (!c->free_events.empty()) {
        *ev = c->free_events.back();
        c->free_events.pop_back();
        return hipSuccess;
    }
    return hipEventCreate(ev);
}

// Waits for the recorded event pairs and adds their durations to the per-family totals.
hipError_t drain_timing(sushi_ctx *c) {
    hipError_t e = hipSuccess;
    for (sushi_ctx::Pending &p : c->pending) {
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventSynchronize(p.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, p.a, p.b);
        if (e == hipSuccess) {
            sushi_kernel_stats &k = c->kstats[p.kc];
            k.launches += 1, k.total_ms += ms, k.bytes += p.bytes, k.flops += p.flops;
            if (p.op_index >= 0 && c->records.size() < 65536)
                c->records.push_back(sushi_launch_record{p.op_index, p.kc, ms, 0.f, p.bytes, p.flops});
        }
        c->free_events.push_back(p.a);
        c->free_events.push_back(p.b);
    }
    c->pending.clear();
    return e;
}

hipError_t issue_launches(sushi_ctx *c, CachedPlan &cp, const void *input_dev, void *logits_dev, hipStream_t st) {
    const bool timed = c->timing && st == c->stream;
    hipError_t e = hipSuccess;
    int op_index = -1;
    for (Launch &L : cp.launches) {
        sushi_ctx::Pending pend{};
        pend.op_index = ++op_index;
        if (timed) {
            if ((e = get_event(c, &pend.a)) != hipSuccess || (e = get_event(c, &pend.b)) != hipSuccess) return e;
            if ((e = hipEventRecord(pend.a, st)) != hipSuccess) return e;
        }
        int kc = KC_COUNT;
        if (c->int8) {
            ConvArgs a = L.conv;
            PoolArgs pa = L.pool;
            switch (L.kind) {
                case OP_CONV:
                    if (L.in_patch) a.x = input_dev;
                    kc = KC_CONV_I8;
                    e = launch_conv_i8(a, L.quant, st, c->patch_min_pixels);
                    break;
                case OP_FC:
                    if (L.out_patch) a.y = logits_dev;
                    kc = KC_I8_OTHER;
                    e = launch_fc_i8(a, L.quant, st);
                    break;
                case OP_MAXPOOL:
                    kc = KC_I8_OTHER;
                    e = launch_maxpool_i8(pa, st);
                    break;
                case OP_GAP:
                    kc = KC_I8_OTHER;
                    e = launch_gap_i8(pa, L.quant, st);
                    break;
                default:
                    e = hipErrorNotSupported;
            }
        } else
        switch (L.kind) {
            case OP_CONV:
            case OP_FC: {
                ConvArgs a = L.conv;
                if (L.in_patch) a.x = input_dev;
                if (L.out_patch) a.y = logits_dev;
                e = launch_conv(a, c->bf16, st, &kc, c->patch_min_pixels);
                break;
            }
            case OP_DW:
                kc = KC_DWCONV;
                e = launch_dwconv(L.conv, c->bf16, st);
                break;
            case OP_MAXPOOL:
                kc = KC_MAXPOOL;
                e = launch_maxpool(L.pool, c->bf16, st);
                break;
            case OP_GAP:
                kc = KC_GAP;
                e = launch_gap(L.pool, c->bf16, st);
                break;
            case OP_GATE:
                kc = KC_GATE;
                e = launch_gate(L.pool, c->bf16, st);
                break;
            default:
                e = hipErrorInvalidValue;
        }
        if (e != hipSuccess) return e;
        if (timed) {
            if ((e = hipEventRecord(pend.b, st)) != hipSuccess) return e;
            pend.kc = kc;
            launch_cost(c, L, &pend.bytes, &pend.flops);
            c->pending.push_back(pend);
        }
    }
    if (timed && c->pending.size() >= 4096) return drain_timing(c);
    return hipSuccess;
}

// Exec mode 1: record the plan's launches once per (input, logits) pointer pair on a private stream,
// then replay the instantiated graph on the context's stream.  No memset nodes are recorded.
int replay_graph(sushi_ctx *c, CachedPlan &cp, const void *input_dev, void *logits_dev) {
    hipError_t e;
    if (!cp.graph || cp.graph_in != input_dev || cp.graph_out != logits_dev) {
        if (cp.graph) {
            (void)hipGraphExecDestroy(cp.graph);
            cp.graph = nullptr;
        }
        if (!c->capture_stream &&
            (e = hipStreamCreateWithFlags(&c->capture_stream, hipStreamNonBlocking)) != hipSuccess)
            return hip_fail(c, e, "hipStreamCreateWithFlags");
        if ((e = hipStreamBeginCapture(c->capture_stream, hipStreamCaptureModeThreadLocal)) != hipSuccess)
            return hip_fail(c, e, "hipStreamBeginCapture");
        hipError_t le = issue_launches(c, cp, input_dev, logits_dev, c->capture_stream);
        hipGraph_t g = nullptr;
        e = hipStreamEndCapture(c->capture_stream, &g);
        if (le != hipSuccess || e != hipSuccess) {
            if (g) (void)hipGraphDestroy(g);
            return hip_fail(c, le != hipSuccess ? le : e, "graph capture");
        }
        e = hipGraphInstantiate(&cp.graph, g, nullptr, nullptr, 0);
        (void)hipGraphDestroy(g);
        if (e != hipSuccess) {
            cp.graph = nullptr;
            return hip_fail(c, e, "hipGraphInstantiate");
        }
        cp.graph_in = input_dev, cp.graph_out = logits_dev;
    }
    if ((e = hipGraphLaunch(cp.graph, c->stream)) != hipSuccess) return hip_fail(c, e, "hipGraphLaunch");
    return SUSHI_OK;
}

// Exec mode 2: builds (once per plan) the device program and launches the stream kernel.
static bool planar_layout_fits(const DevOp &op);

int ensure_stream_state(sushi_ctx *c) {
    if (c->d_sync) return SUSHI_OK;
    hipError_t e;
    hipDeviceProp_t prop;
    if ((e = hipGetDeviceProperties(&prop, c->device)) != hipSuccess) return hip_fail(c, e, "hipGetDeviceProperties");
    c->stream_wgs = std::max(BARRIER_GROUP, prop.multiProcessorCount / BARRIER_GROUP * BARRIER_GROUP);
    if (c->stream_wgs_override) c->stream_wgs = c->stream_wgs_override;
    if ((e = hipMalloc(reinterpret_cast<void **>(&c->d_sync), SYNC_WORDS * 8)) != hipSuccess)
        return fail(c, SUSHI_ENOMEM, "hipMalloc(barrier area)");
    if ((e = hipMemset(c->d_sync, 0, SYNC_WORDS * 8)) != hipSuccess) return hip_fail(c, e, "hipMemset");
    if ((e = hipHostMalloc(reinterpret_cast<void **>(&c->h_abort), 64, hipHostMallocDefault)) != hipSuccess)
        return fail(c, SUSHI_ENOMEM, "hipHostMalloc(abort flag)");
    *c->h_abort = 0;
    c->epoch_base = 0;
    return SUSHI_OK;
}

int run_stream_kernel(sushi_ctx *c, CachedPlan &cp, const void *input_dev, void *logits_dev) {
    if (!c->bf16) return fail(c, SUSHI_ESTATE, "the stream kernel runs in bf16 mode only");
    int rc = ensure_stream_state(c);
    if (rc) return rc;
    hipError_t e;
    if (*c->h_abort) {
        // a wait inside an earlier launch ran out: drain, reset the barrier area, report
        (void)hipStreamSynchronize(c->stream);
        (void)hipMemset(c->d_sync, 0, SYNC_WORDS * 8);
        *c->h_abort = 0;
        c->epoch_base = 0;
        return fail(c, SUSHI_EDEVICE, "an earlier query timed out at a grid barrier; its logits are invalid");
    }
    if (!cp.d_prog) {
        std::vector<DevOp> prog;
        for (const Launch &L : cp.launches) {
            DevOp op{};
            op.kind = L.kind;
            op.conv = L.conv, op.pool = L.pool;
            op.in_patch = L.in_patch, op.out_patch = L.out_patch;
            op.pt = op.wk = op.ft = 1;
            op.layer = -1;
            if (!planar_layout_fits(op))
                return fail(c, SUSHI_ESTATE, "a layer's channel count does not fit the stream kernel's activation layout");
            if (L.kind == OP_CONV || L.kind == OP_FC) {
                if ((L.conv.C & 7) == 0 && !dense_op_fits(L.conv))
                    return fail(c, SUSHI_ESTATE, "a dense layer has too many reduction steps or taps for the stream kernel");
                if ((L.conv.C & 7) == 0)
                    tile_dev_op(op, c->stream_wgs, false);
                else
                    tile_stem_op(op, c->stream_wgs);
            } else if (L.kind == OP_DW) {
                tile_dw_op(op, c->stream_wgs);
            }
            prog.push_back(op);
        }
        if ((e = hipMalloc(reinterpret_cast<void **>(&cp.d_prog), prog.size() * sizeof(DevOp))) != hipSuccess)
            return fail(c, SUSHI_ENOMEM, "hipMalloc(program)");
        if ((e = hipMemcpy(cp.d_prog, prog.data(), prog.size() * sizeof(DevOp), hipMemcpyHostToDevice)) != hipSuccess)
            return hip_fail(c, e, "hipMemcpy(program)");
        cp.n_dev_ops = (int)prog.size();
    }
    StreamArgs sa{};
    sa.prog = cp.d_prog, sa.n_ops = cp.n_dev_ops;
    sa.input = input_dev, sa.logits = logits_dev;
    sa.sync = c->d_sync, sa.epoch_base = c->epoch_base, sa.spin_limit = c->spin_limit, sa.abort_flag = c->h_abort;
    sushi_ctx::Pending pend{};
    if (c->timing) {
        if ((e = get_event(c, &pend.a)) != hipSuccess || (e = get_event(c, &pend.b)) != hipSuccess ||
            (e = hipEventRecord(pend.a, c->stream)) != hipSuccess)
            return hip_fail(c, e, "kernel timing");
    }
    if ((e = launch_stream_kernel(sa, c->stream_wgs, c->stream)) != hipSuccess) return hip_fail(c, e, "stream kernel");
    if (c->timing) {
        if ((e = hipEventRecord(pend.b, c->stream)) != hipSuccess) return hip_fail(c, e, "kernel timing");
        pend.kc = KC_STREAM, pend.bytes = cp.alg_bytes, pend.flops = cp.alg_flops;
        c->pending.push_back(pend);
        if (c->pending.size() >= 4096 && (e = drain_timing(c)) != hipSuccess) return hip_fail(c, e, "kernel timing");
    }
    c->epoch_base += (unsigned long long)stream_barriers(cp.n_dev_ops);
    return SUSHI_OK;
}

// ---------------------------------------------------------------- SubGraph residency (team kernel)

bool team_kernel_running(sushi_ctx *c);
int launch_teams(sushi_ctx *c);

void free_res_gen(sushi_ctx::ResGen &g) {
    if (g.table) (void)hipHostFree(g.table);
    g = sushi_ctx::ResGen();
}

// Pools and table slots of the team mode; called once, before the kernel first runs.
int make_team_pools(sushi_ctx *c) {
    hipError_t e;
    if ((e = hipHostMalloc(reinterpret_cast<void **>(&c->h_prog_pool), sushi_ctx::PROG_POOL_BYTES, hipHostMallocDefault)) != hipSuccess)
        return fail(c, SUSHI_ENOMEM, "hipHostMalloc(program pool)");
    if ((e = hipMalloc(reinterpret_cast<void **>(&c->d_team_mem), (size_t)TEAM_MEM_BYTES * MAX_TEAMS)) != hipSuccess)
        return fail(c, SUSHI_ENOMEM, "hipMalloc(team memory)");
    const size_t gen_bytes = 64 + RES_MAX_LAYERS * sizeof(ResLayer) + RES_MAX_ENTRIES * sizeof(ResEntry);
    for (auto &g : c->res_gens) {
        char *base = nullptr;
        if ((e = hipHostMalloc(reinterpret_cast<void **>(&base), gen_bytes, hipHostMallocDefault)) != hipSuccess)
            return fail(c, SUSHI_ENOMEM, "hipHostMalloc(residency tables)");
        g.table = reinterpret_cast<ResTable *>(base);
        g.layers = reinterpret_cast<ResLayer *>(base + 64);
        g.entries = reinterpret_cast<ResEntry *>(base + 64 + RES_MAX_LAYERS * sizeof(ResLayer));
    }
    return SUSHI_OK;
}

// Slab geometry of the LDS stores: which 16-filter tile of which layer has a slab, how wide it is, which
// workgroup of a team holds it and where.  Layers from the last to the first (the late, few-pixel layers
// hold most weights and are the ones that use their slabs), tiles round-robin over the ranks, first rank
// with room wins.  A layer's slabs are as many (n_alloc) and as wide (cg_alloc) as the largest SubGraph
// cached since the SuperNet was loaded asked for, so the geometry changes only when a SubGraph outgrows
// it; between such changes a new SubGraph just moves the valid part of every slab, and the teams copy
// only the cells that were not valid before.
void rebuild_geometry(sushi_ctx *c) {
    const int team_size = c->team_size();
    const size_t n_layers = c->sn.layers.size();
    c->geo_layers.assign(n_layers, ResLayer{});
    c->geo_entries.clear();
    ++c->geometry;
    if (team_size < 1) return;
    std::vector<long> used(team_size, 0);
    int cursor = 0;
    for (int l = (int)n_layers - 1; l >= 0; --l) {
        const SuperLayer &L = c->sn.layers[l];
        if (L.type == L_DW || c->geo_n[l] == 0 || c->geo_cg[l] == 0) continue;
        const int taps = L.Rmax * L.Rmax;
        const long slab = (long)taps * c->geo_cg[l] * 256;
        if (c->geo_entries.size() + (size_t)c->geo_n[l] > (size_t)RES_MAX_ENTRIES) break;
        ResLayer &R = c->geo_layers[l];
        R.w = static_cast<const char *>(c->d_weights) + L.pk_w * 2;
        R.Kpad = L.Kpad, R.CG = L.CG, R.taps = taps, R.cg_stride = c->geo_cg[l];
        R.first_entry = (int)c->geo_entries.size();
        bool any = false;
        long most_free = RES_STORE_BYTES - *std::min_element(used.begin(), used.end());
        for (int f = 0; f < c->geo_n[l]; ++f) {
            ResEntry e{-1, 0};
            for (int k = 0; k < team_size && slab <= most_free; ++k) {
                const int r = (cursor + k) % team_size;
                if (used[r] + slab <= RES_STORE_BYTES) {
                    e.owner = r, e.lds_off = (int)used[r];
                    used[r] += slab;
                    cursor = (r + 1) % team_size;
                    any = true;
                    most_free = RES_STORE_BYTES - *std::min_element(used.begin(), used.end());
                    break;
                }
            }
            c->geo_entries.push_back(e);
        }
        R.n_res = any ? c->geo_n[l] : 0;  // (here: tiles the geometry lists; the table sets the valid count)
        if (!any) {  // no room for any slab of this layer: it takes no entries (the teams fetch the whole list)
            c->geo_entries.resize(R.first_entry);
            R = ResLayer{};
        }
    }
}

// The residency table of the cached SubGraph: the geometry with every layer's valid part set to what
// the SubGraph covers.  Returns true if it differs from the table in force (a team would then hold
// other cells than now).  Also counts the slab bytes that become valid (per team).
bool build_res_table(sushi_ctx *c, uint64_t *new_bytes) {
    const size_t n_layers = c->sn.layers.size();
    *new_bytes = 0;
    if (c->geo_n.size() != n_layers) c->geo_n.assign(n_layers, 0), c->geo_cg.assign(n_layers, 0), c->geometry_team_size = 0;
    bool grow = c->geometry_team_size != c->team_size();
    if (!c->G.empty())
        for (size_t l = 0; l < n_layers; ++l) {
            const SuperLayer &L = c->sn.layers[l];
            const sushi_layer_dims &g = c->G[l];
            if (L.type == L_DW || g.K == 0) continue;
            const int want_cg = std::min(g.C / 8, RES_STORE_BYTES / (L.Rmax * L.Rmax * 256)), want_n = (g.K + 15) / 16;
            if (want_cg > c->geo_cg[l]) c->geo_cg[l] = want_cg, grow = true;
            if (want_n > c->geo_n[l]) c->geo_n[l] = want_n, grow = true;
        }
    if (grow) {
        rebuild_geometry(c);
        c->geometry_team_size = c->team_size();
        c->geo_present.assign(c->geo_entries.size(), 0);
    }
    std::vector<ResLayer> layers = c->geo_layers;
    uint64_t bytes = 0;
    bool any = false;
    for (size_t l = 0; l < layers.size(); ++l) {
        ResLayer &R = layers[l];
        const int listed = R.n_res;
        R.n_res = 0, R.cg_res = 0;
        if (c->G.empty() || listed == 0 || c->G[l].K == 0) continue;
        R.n_res = std::min(listed, (c->G[l].K + 15) / 16);
        R.cg_res = std::min(c->G[l].C / 8, R.cg_stride);
        if (R.cg_res < 1) R.n_res = 0;
        for (int f = 0; f < R.n_res; ++f)
            if (c->geo_entries[R.first_entry + f].owner >= 0) {
                const uint64_t cells = (uint64_t)R.taps * 8 * std::min(16, c->G[l].K - 16 * f) * 2;
                bytes += cells * R.cg_res;
                any = true;
                // cells such a team's store does not hold yet
                int &have = c->geo_present[R.first_entry + f];
                if (R.cg_res > have) *new_bytes += cells * (R.cg_res - have), have = R.cg_res;
            }
    }
    bool changed = grow || layers.size() != c->h_res_layers.size() || any != !c->h_res_entries.empty();
    for (size_t l = 0; !changed && l < layers.size(); ++l)
        changed = layers[l].n_res != c->h_res_layers[l].n_res || layers[l].cg_res != c->h_res_layers[l].cg_res;
    if (!changed) return false;
    c->h_res_layers = std::move(layers);
    if (any) c->h_res_entries = c->geo_entries; else c->h_res_entries.clear();
    c->table_bytes = bytes;
    ++c->table_version;
    return true;
}

// Writes the table into the next of the pinned generations and makes it the one later posts name.  The slot
// it takes over held the table from N_RES_GENS - 1 changes ago; every post that still names that one must
// have been served first (with 32 generations and at most 32 posts per mailbox that wait never lasts).
int upload_res_table(sushi_ctx *c) {
    const int slot = (c->gen_cur + 1) % sushi_ctx::N_RES_GENS;
    sushi_ctx::ResGen &g = c->res_gens[slot];
    if (c->th)
        for (int t = 0; t < MAX_TEAMS; ++t) {
            const auto t0 = std::chrono::steady_clock::now();
            unsigned spins = 0;
            while (*(volatile unsigned long long *)&c->th->done[t * 8] < g.last_ref[t]) {
                if ((++spins & 0x3FF) != 0) continue;
                if (!team_kernel_running(c)) {  // the post is still in the mailbox: let a new launch serve it
                    int rc = launch_teams(c);
                    if (rc) return rc;
                }
                if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(20))
                    return fail(c, SUSHI_EDEVICE, "timed out waiting for a team");
            }
        }
    ++c->table_seq;
    c->gen_cur = slot;
    c->gen_valid[slot] = false;
    if (c->h_res_entries.empty()) return SUSHI_OK;
    if (c->h_res_layers.size() > (size_t)RES_MAX_LAYERS) return fail(c, SUSHI_ENOMEM, "too many layers for the table");
    if (c->h_res_entries.size() > (size_t)RES_MAX_ENTRIES) return fail(c, SUSHI_ENOMEM, "too many slabs for the table");
    std::memcpy(g.layers, c->h_res_layers.data(), c->h_res_layers.size() * sizeof(ResLayer));
    std::memcpy(g.entries, c->h_res_entries.data(), c->h_res_entries.size() * sizeof(ResEntry));
    ResTable t{};
    t.n_layers = (int)c->h_res_layers.size(), t.team_size = c->team_size(), t.n_entries = (int)c->h_res_entries.size();
    t.geometry = c->geometry;
    t.layers = g.layers, t.entries = g.entries;
    *g.table = t;
    c->gen_valid[slot] = true;
    return SUSHI_OK;
}

// Weight bytes of one SubNet that come out of resident slabs.
void refresh_lds_bytes(sushi_ctx *c, CachedPlan &cp) {
    if (cp.table_version == c->table_version) return;
    cp.table_version = c->table_version;
    cp.lds_bytes = 0;
    if (c->h_res_entries.empty()) return;
    for (const DevOp &op : cp.team_prog) {
        if ((op.kind != OP_CONV && op.kind != OP_FC) || op.wk <= 0 || op.ft > 2 || (long)op.conv.B * op.conv.P * op.conv.Q > 64 || op.layer < 0) continue;
        if ((op.conv.C & 7) != 0) continue;
        const ResLayer &R = c->h_res_layers[op.layer];
        const int n_f = (op.conv.K + 15) / 16;
        const int cgs = std::min(R.cg_res, op.conv.C / 8);
        for (int f = 0; f < std::min(R.n_res, n_f); ++f)
            if (c->h_res_entries[R.first_entry + f].owner >= 0)
                cp.lds_bytes += (uint64_t)R.taps * cgs * 8 * std::min(16, op.conv.K - 16 * f) * 2;
    }
}

// ---------------------------------------------------------------- exec mode 3: the team kernel

// Hands the finished (or finishing) team-kernel launch over to the timing totals.
void close_team_timing(sushi_ctx *c) {
    if (!c->team_timed) return;
    c->pending.push_back(c->team_pending);
    c->team_timed = false;
}

bool team_kernel_running(sushi_ctx *c) {
    return c->team_launched && hipStreamQuery(c->pstream) == hipErrorNotReady;
}

// Makes the team kernel leave (teams finish the post they are working on first) and waits for it.
int stop_team_kernel(sushi_ctx *c) {
    if (!c->team_launched) return SUSHI_OK;
    c->th->stop = 1;
    hipError_t e = hipStreamSynchronize(c->pstream);
    c->th->stop = 0;
    c->team_launched = false;
    close_team_timing(c);
    if (e != hipSuccess) return hip_fail(c, e, "team kernel");
    return SUSHI_OK;
}

int launch_teams(sushi_ctx *c) {
    hipError_t e;
    if (c->team_launched) {
        if ((e = hipStreamSynchronize(c->pstream)) != hipSuccess) return hip_fail(c, e, "team kernel");
        c->team_launched = false;
    }
    if (c->th->abort_flag) {
        static const char *const why[] = {"?", "not every workgroup of the launch became resident",
                                          "a workgroup did not reach a team barrier within the spin limit",
                                          "a team leader did not hand a post to its team in time",
                                          "a mailbox slot did not hold the post its counter announced"};
        const unsigned code = c->th->abort_flag;
        c->th->abort_flag = 0;
        for (int t = 0; t < MAX_TEAMS; ++t) c->th->done[t * 8] = c->posted[t];  // drop what was in flight
        return fail(c, SUSHI_EDEVICE, std::string("a wait inside the team kernel ran out (") + why[code < 5 ? code : 0] +
                                          "); queries in flight were dropped");
    }
    c->th->ready = 0;
    if ((e = hipMemsetAsync(c->d_tsync, 0, SYNC_WORDS * 8, c->pstream)) != hipSuccess) return hip_fail(c, e, "hipMemsetAsync");
    TeamArgs ta{};
    ta.host = c->th, ta.sync = c->d_tsync, ta.arena = c->d_tarena, ta.arena_bytes = c->tarena_bytes;
    ta.teams_per_xcd = c->teams_per_xcd;
    for (int t = 0; t < MAX_TEAMS; ++t) ta.last_seq[t] = c->th->done[t * 8];
    ta.idle_ticks = c->idle_ticks, ta.spin_limit = c->spin_limit;
    ta.trace = c->d_trace;
    ta.team_mem = c->d_team_mem;
    close_team_timing(c);
    if (c->timing) {
        sushi_ctx::Pending &tp = c->team_pending;
        tp = sushi_ctx::Pending{};
        if ((e = get_event(c, &tp.a)) != hipSuccess || (e = get_event(c, &tp.b)) != hipSuccess ||
            (e = hipEventRecord(tp.a, c->pstream)) != hipSuccess)
            return hip_fail(c, e, "kernel timing");
        tp.kc = KC_TEAM;
    }
    const bool mobile = c->sn.arch.family == SUSHI_FAMILY_MBV3;  // (a load of another SuperNet stops the kernel first)
    e = mobile ? launch_team_kernel_mobile(ta, c->team_wgs, c->pstream) : launch_team_kernel(ta, c->team_wgs, c->pstream);
    if (e != hipSuccess) return hip_fail(c, e, "team kernel launch");
    if (c->timing) {
        if ((e = hipEventRecord(c->team_pending.b, c->pstream)) != hipSuccess) return hip_fail(c, e, "kernel timing");
        c->team_timed = true;
    }
    c->team_launched = true;
    const auto t0 = std::chrono::steady_clock::now();
    while (!*(volatile unsigned *)&c->th->ready) {
        if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(5)) {
            (void)stop_team_kernel(c);
            return fail(c, SUSHI_EDEVICE, "the team kernel did not start");
        }
    }
    return SUSHI_OK;
}

int ensure_team_state(sushi_ctx *c, int batch) {
    hipError_t e;
    if (!c->th) {
        hipDeviceProp_t prop;
        if ((e = hipGetDeviceProperties(&prop, c->device)) != hipSuccess) return hip_fail(c, e, "hipGetDeviceProperties");
        if ((e = prepare_team_kernel()) != hipSuccess || (e = prepare_team_kernel_mobile()) != hipSuccess)
            return hip_fail(c, e, "hipFuncSetAttribute");
        // every workgroup must be resident at once (they wait for each other)
        int fit = 0, fit_mobile = 0;
        if ((e = team_kernel_blocks_per_cu(&fit)) != hipSuccess || (e = team_kernel_mobile_blocks_per_cu(&fit_mobile)) != hipSuccess)
            return hip_fail(c, e, "occupancy query");
        fit = std::min(fit, fit_mobile);
        const int per_cu = std::max(1, std::min(c->team_wgs_per_cu, fit));
        c->team_wgs = per_cu * std::max(BARRIER_GROUP, prop.multiProcessorCount / BARRIER_GROUP * BARRIER_GROUP);
        if ((e = hipHostMalloc(reinterpret_cast<void **>(&c->th), sizeof(TeamHostState), hipHostMallocDefault)) != hipSuccess)
            return fail(c, SUSHI_ENOMEM, "hipHostMalloc(mailboxes)");
        std::memset(c->th, 0, sizeof(TeamHostState));
        if ((e = hipMalloc(reinterpret_cast<void **>(&c->d_tsync), SYNC_WORDS * 8)) != hipSuccess)
            return fail(c, SUSHI_ENOMEM, "hipMalloc(team sync)");
        if ((e = hipStreamCreateWithFlags(&c->pstream, hipStreamNonBlocking)) != hipSuccess)
            return hip_fail(c, e, "hipStreamCreateWithFlags");
        int rc = make_team_pools(c);
        if (rc) return rc;
        uint64_t fresh = 0;
        if (build_res_table(c, &fresh) && (rc = upload_res_table(c)) != SUSHI_OK) return rc;  // a SubGraph may have been cached before the first query
        c->stats.cache_bytes_lds = c->table_bytes;
    }
    if (batch > c->tarena_batch) {
        int rc = stop_team_kernel(c);
        if (rc) return rc;
        Plan p;
        std::string err;
        rc = plan_subnet(c->sn, largest_cfg(c->sn.arch), batch, p, err);
        if (rc) return fail(c, rc, "arena: " + err);
        if (c->d_tarena) (void)hipFree(c->d_tarena);
        c->d_tarena = nullptr;
        c->tbig_bytes = (long)round_up(p.max_big_elems * 2, 256);
        c->tsmall_bytes = (long)round_up(std::max<size_t>(p.max_small_elems, 8) * 4, 256);
        c->tarena_bytes = N_BIG_BUFS * c->tbig_bytes + N_SMALL_BUFS * c->tsmall_bytes;
        // (one arena per team that can exist: the number of teams per XCD is fixed before the first query)
        if ((e = hipMalloc(reinterpret_cast<void **>(&c->d_tarena), (size_t)c->tarena_bytes * MAX_XCDS * c->teams_per_xcd)) != hipSuccess)
            return fail(c, SUSHI_ENOMEM, "hipMalloc(team arenas)");
        c->tarena_batch = batch;
        for (auto &kv : c->plans)
            if (kv.second->h_team_prog) {
                kv.second->h_team_prog = nullptr;
                kv.second->team_prog.clear();
            }
    }
    return SUSHI_OK;
}

// Blocks until team t has finished everything posted to it (relaunching the kernel if it has left).
int wait_team(sushi_ctx *c, int t) {
    const auto t0 = std::chrono::steady_clock::now();
    unsigned spins = 0;
    while (*(volatile unsigned long long *)&c->th->done[t * 8] != c->posted[t]) {
        if ((++spins & 0x3FF) == 0) {
            if (!team_kernel_running(c)) {
                int rc = launch_teams(c);
                if (rc) return rc;
            }
            if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(20))
                return fail(c, SUSHI_EDEVICE, "timed out waiting for a team");
        }
    }
    return SUSHI_OK;
}

// Blocks until team t's mailbox has room for one more post and returns that slot.
int reserve_post(sushi_ctx *c, int t, TeamPost **slot) {
    const auto t0 = std::chrono::steady_clock::now();
    unsigned spins = 0;
    while (c->posted[t] - *(volatile unsigned long long *)&c->th->done[t * 8] >= (unsigned long long)POST_RING) {
        if ((++spins & 0x3FF) == 0) {
            if (!team_kernel_running(c)) {
                int rc = launch_teams(c);
                if (rc) return rc;
            }
            if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(20))
                return fail(c, SUSHI_EDEVICE, "timed out waiting for a team");
        }
    }
    *slot = &c->th->post[t][(c->posted[t] + 1) % POST_RING];
    return SUSHI_OK;
}

void publish_post(sushi_ctx *c, int t, TeamPost *slot) {
    slot->seq = c->posted[t] + 1;
    __atomic_thread_fence(__ATOMIC_RELEASE);
    *(volatile unsigned long long *)&c->th->posted[t * 8] = ++c->posted[t];
}

int synchronize_teams(sushi_ctx *c);

// The stream and team kernels keep activations by groups of 8 channels (one 16-byte cell per group and pixel):
// every tensor with more than one pixel per image must have a multiple of 8 channels, except the caller's
// input, which only the stem units read (in its own order) and which therefore must not have one.
static bool planar_layout_fits(const DevOp &op) {
    if (op.kind == OP_CONV || op.kind == OP_DW || op.kind == OP_FC) {
        const ConvArgs &a = op.conv;
        if (a.P * a.Q > 1 && (a.K & 7) != 0) return false;
        if (op.in_patch) return (a.C & 7) != 0;
        return a.H * a.W == 1 || (a.C & 7) == 0;
    }
    return (op.pool.C & 7) == 0;
}

// Tiles one op of a plan for a team of nwg workgroups (dims only; the activation pointers stay as they are).
// False: a layer does not fit the team kernel.
static bool tile_team_op(DevOp &op, int nwg) {
    op.pt = op.wk = op.ft = 1;
    if (!planar_layout_fits(op)) return false;
    if (op.kind == OP_CONV || op.kind == OP_FC) {
        if ((op.conv.C & 7) == 0 && !dense_op_fits(op.conv)) return false;
        if ((op.conv.C & 7) == 0)
            tile_dev_op(op, nwg, true);
        else
            tile_stem_op(op, nwg);
    } else if (op.kind == OP_DW) {
        tile_dw_op(op, nwg);
    }
    return true;
}

int post_team_query(sushi_ctx *c, CachedPlan &cp, const void *input_dev, void *logits_dev, int batch) {
    if (!c->bf16) return fail(c, SUSHI_ESTATE, "the team kernel runs in bf16 mode only");
    int rc = ensure_team_state(c, batch);
    if (rc) return rc;
    hipError_t e;
    if (!cp.h_team_prog) {
        std::vector<DevOp> prog;
        for (size_t i = 0; i < cp.launches.size(); ++i) {
            const Launch &L = cp.launches[i];
            const Op &o = cp.plan.ops[i];
            DevOp op{};
            op.kind = L.kind;
            op.conv = L.conv, op.pool = L.pool;
            op.in_patch = L.in_patch, op.out_patch = L.out_patch;
            op.relative = 1;
            auto rel = [&](int id, bool small) -> void * {
                if (id < 0) return nullptr;
                const long off = small ? N_BIG_BUFS * c->tbig_bytes + id * c->tsmall_bytes : id * c->tbig_bytes;
                return reinterpret_cast<void *>(off + 1);
            };
            op.conv.x = rel(o.in_buf, o.in_small), op.conv.y = rel(o.out_buf, o.out_small);
            op.conv.res = rel(o.res_buf, false);
            op.pool.x = op.conv.x, op.pool.y = op.conv.y;
            op.pool.gate = static_cast<const float *>(rel(o.gate_buf, true));
            op.layer = (L.kind == OP_CONV || L.kind == OP_FC) ? o.layer : -1;
            if (!tile_team_op(op, c->team_size()))
                return fail(c, SUSHI_ESTATE, "a layer does not fit the team kernel (reduction steps, taps or channel counts)");
            // every activation tensor of the op must lie inside the buffer of the team arena it names
            {
                const bool conv = L.kind == OP_CONV || L.kind == OP_DW || L.kind == OP_FC;
                const long in_bytes = (long)o.B * o.H * o.W * o.C * (o.in_small ? 4 : 2);
                const long out_elems = (long)o.B * o.P * o.Q * (conv ? o.K : o.C);
                const long out_bytes = out_elems * (o.out_f32 ? 4 : 2);
                auto fits = [&](int id, bool small, long bytes) { return id < 0 || bytes <= (small ? c->tsmall_bytes : c->tbig_bytes); };
                if (!fits(o.in_buf, o.in_small, in_bytes) || !fits(o.out_buf, o.out_small, out_bytes) ||
                    !fits(o.res_buf, false, out_elems * 2) || !fits(o.gate_buf, true, (long)o.B * o.C * 4))
                    return fail(c, SUSHI_ESTATE, "internal: an activation tensor does not fit its team arena buffer");
            }
            prog.push_back(op);
        }
        if (prog.size() > (size_t)TEAM_PROG_MAX_OPS) return fail(c, SUSHI_ESTATE, "the SubNet has too many ops for the team kernel");
        fuse_se_blocks(prog, cp.plan);
        cp.team_prog = prog;
        cp.table_version = ~0ull;
        const size_t bytes = round_up(prog.size() * sizeof(DevOp), 256);
        if (c->prog_pool_used + bytes > sushi_ctx::PROG_POOL_BYTES) {
            // pool exhausted: forget every program (after the teams are done with them) and start over
            if ((rc = synchronize_teams(c)) != SUSHI_OK) return rc;
            for (auto &kv : c->plans) kv.second->h_team_prog = nullptr;
            c->prog_pool_used = 0;
        }
        DevOp *dst = reinterpret_cast<DevOp *>(c->h_prog_pool + c->prog_pool_used);
        std::memcpy(dst, prog.data(), prog.size() * sizeof(DevOp));
        c->prog_pool_used += bytes;
        cp.h_team_prog = dst;
        cp.n_dev_ops = (int)prog.size();
    }
    // The input must be complete before a team may read it.  Work still pending on the caller's stream may be
    // waiting for a compute unit, and the team kernel gives none up while it runs: make it leave first (the
    // teams finish what is in their mailboxes) instead of letting the stream wait for it to idle out.
    if (hipStreamQuery(c->stream) == hipErrorNotReady) {
        if (team_kernel_running(c) && (rc = stop_team_kernel(c)) != SUSHI_OK) return rc;
        if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
    }
    if (!c->team_launched && (rc = launch_teams(c)) != SUSHI_OK) return rc;
    int t = -1;
    for (int k = 0; k < MAX_TEAMS; ++k) {
        const int cand = (c->next_team + k) % MAX_TEAMS;
        if (c->th->team_size[cand] > 0) {
            t = cand;
            break;
        }
    }
    if (t < 0) return fail(c, SUSHI_EDEVICE, "no team has any workgroup");
    c->next_team = (t + 1) % MAX_TEAMS;
    TeamPost *slot = nullptr;
    if ((rc = reserve_post(c, t, &slot)) != SUSHI_OK) return rc;
    if (c->team_timed) c->team_pending.bytes += cp.alg_bytes, c->team_pending.flops += cp.alg_flops;
    refresh_lds_bytes(c, cp);
    c->stats.weight_bytes_lds += cp.lds_bytes;
    c->stats.last_lds_bytes = cp.lds_bytes;
    TeamPost &p = *slot;
    p.cmd = TEAM_RUN, p.n_ops = cp.n_dev_ops, p.prog = cp.h_team_prog, p.input = input_dev, p.logits = logits_dev;
    p.table = c->gen_valid[c->gen_cur] ? c->res_gens[c->gen_cur].table : nullptr;
    p.table_seq = c->table_seq;
    c->res_gens[c->gen_cur].last_ref[t] = c->posted[t] + 1;
    publish_post(c, t, slot);
    return SUSHI_OK;
}

// Rebuilds the residency table for the cached SubGraph.  If the teams would hold other cells than now, the
// table becomes a new generation; queries posted from here on name it, and a team brings its LDS stores up
// to it before the first such query it serves (queries posted earlier still run under the table they name).
int install_on_teams(sushi_ctx *c) {
    if (!c->th) return SUSHI_OK;  // the team kernel has never run: the table is built at its first start
    uint64_t fresh = 0;
    if (!build_res_table(c, &fresh)) return SUSHI_OK;  // the teams would hold exactly what they hold now
    int rc = upload_res_table(c);
    if (rc) return rc;
    c->stats.residency_changes += 1;
    c->stats.install_bytes_lds += fresh;
    return SUSHI_OK;
}

int synchronize_teams(sushi_ctx *c) {
    if (!c->th) return SUSHI_OK;
    for (int t = 0; t < MAX_TEAMS; ++t) {
        int rc = wait_team(c, t);
        if (rc) return rc;
    }
    return SUSHI_OK;
}

std::string plan_key(const sushi_subnet_cfg &cfg, int batch) {
    std::string k(reinterpret_cast<const char *>(&cfg), sizeof(cfg));
    k.append(reinterpret_cast<const char *>(&batch), sizeof(batch));
    return k;
}

}  // namespace

// Makes the context forget the SuperNet it holds (device weights, arenas, plans, cached SubGraph, residency state).
static int drop_loaded(sushi_ctx *c) {
    hipError_t e;
    if ((e = hipSetDevice(c->device)) != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
    if (c->th) {
        (void)synchronize_teams(c);
        (void)stop_team_kernel(c);
        // the team arenas were sized by the previous SuperNet's largest SubNet
        if (c->d_tarena) (void)hipFree(c->d_tarena);
        c->d_tarena = nullptr;
        c->tarena_batch = 0, c->tarena_bytes = 0, c->tbig_bytes = 0, c->tsmall_bytes = 0;
    }
    free_arena(c);
    c->plans.clear();
    if (c->d_weights) (void)hipFree(c->d_weights);
    if (c->d_params) (void)hipFree(c->d_params);
    c->d_weights = nullptr, c->d_params = nullptr, c->loaded = false;
    c->G.clear();
    ++c->g_version;
    for (bool &v : c->gen_valid) v = false;
    c->h_res_layers.clear(), c->h_res_entries.clear();
    c->geo_n.clear(), c->geo_cg.clear(), c->geo_layers.clear(), c->geo_entries.clear();
    ++c->geometry;
    ++c->table_seq;  // (teams drop the table they hold)
    c->geometry_team_size = 0;
    c->prog_pool_used = 0;
    ++c->table_version;
    c->stats = sushi_stats{};

    if (c->d_qparams) (void)hipFree(c->d_qparams);
    if (c->d_wsum) (void)hipFree(c->d_wsum);
    c->d_qparams = nullptr, c->d_wsum = nullptr, c->int8 = false;
    return SUSHI_OK;
}

extern "C" {

int sushi_synchronize(sushi_ctx *c);

int sushi_describe_supernet(const sushi_arch *arch, sushi_tensor_desc *out, int cap, int *n_out) {
    if (!arch || !n_out || cap < 0 || (cap > 0 && !out)) return SUSHI_EINVAL;
    SuperNet sn;
    std::string err;
    int rc = build_supernet(*arch, sn, err);
    if (rc) return rc;
    *n_out = (int)sn.tensors.size();
    for (int i = 0; i < cap && i < *n_out; ++i) out[i] = sn.tensors[i];
    return SUSHI_OK;
}

int sushi_subnet_layers(const sushi_arch *arch, const sushi_subnet_cfg *cfg, sushi_layer_dims *out, int cap,
                        int *n_out) {
    if (!arch || !cfg || !n_out || cap < 0 || (cap > 0 && !out)) return SUSHI_EINVAL;
    SuperNet sn;
    std::string err;
    int rc = build_supernet(*arch, sn, err);
    if (rc) return rc;
    std::vector<sushi_layer_dims> dims;
    rc = subnet_dims(sn, *cfg, dims, err);
    if (rc) return rc;
    *n_out = (int)dims.size();
    for (int i = 0; i < cap && i < *n_out; ++i) out[i] = dims[i];
    return SUSHI_OK;
}

int sushi_subgraph_overlap(const sushi_layer_dims *sn, const sushi_layer_dims *g, int n, int bytes_per_weight,
                           uint64_t *subnet_bytes, uint64_t *common_bytes, double *hit_ratio) {
    if (!sn || !g || n < 1 || bytes_per_weight < 1) return SUSHI_EINVAL;
    uint64_t total = 0, common = 0;
    double norm2 = 0.0, inter2 = 0.0;
    for (int i = 0; i < n; ++i) {
        const sushi_layer_dims &d = sn[i], &c = g[i];
        if (d.K <= 0) continue;
        total += (uint64_t)d.K * d.C * d.r * d.r * bytes_per_weight;
        norm2 += (double)d.K * d.K + (double)d.C * d.C;
        if (c.K <= 0) continue;
        const uint64_t k = std::min(d.K, c.K), ch = std::min(d.C, c.C), r = std::min(d.r, c.r);
        common += k * ch * r * r * bytes_per_weight;
        inter2 += (double)k * k + (double)ch * ch;
    }
    if (subnet_bytes) *subnet_bytes = total;
    if (common_bytes) *common_bytes = common;
    if (hit_ratio) *hit_ratio = norm2 > 0 ? std::sqrt(inter2) / std::sqrt(norm2) : 0.0;
    return SUSHI_OK;
}

int sushi_pack_supernet(const sushi_arch *arch, const void *weights, size_t nbytes, int dtype, void *packed,
                        size_t cap_bytes, size_t *n_bytes, sushi_packed_layer *layers, int cap_layers, int *n_layers) {
    if (!arch || !weights || !n_bytes || !n_layers || (cap_bytes > 0 && !packed) || cap_layers < 0 ||
        (cap_layers > 0 && !layers) || (dtype != SUSHI_FP32 && dtype != SUSHI_BF16))
        return SUSHI_EINVAL;
    SuperNet sn;
    std::string err;
    int rc = build_supernet(*arch, sn, err);
    if (rc) return rc;
    if (nbytes != sn.blob_floats * sizeof(float)) return SUSHI_EINVAL;
    const float *blob = static_cast<const float *>(weights);
    std::vector<float> params;
    std::vector<uint16_t> w16;
    std::vector<float> w32;
    const void *src = nullptr;
    try {
        if (dtype == SUSHI_BF16) {
            pack_weights<uint16_t>(sn, blob, w16, params, to_bf16);
            *n_bytes = w16.size() * 2, src = w16.data();
        } else {
            pack_weights<float>(sn, blob, w32, params, [](float f) { return f; });
            *n_bytes = w32.size() * 4, src = w32.data();
        }
    } catch (const std::bad_alloc &) {
        return SUSHI_ENOMEM;
    }
    *n_layers = (int)sn.layers.size();
    for (int i = 0; i < *n_layers && i < cap_layers; ++i) {
        const SuperLayer &L = sn.layers[i];
        layers[i] = sushi_packed_layer{(uint64_t)L.pk_w, L.type == L_DW ? 1 : 0, L.Kmax, L.Cmax, L.Rmax, L.Kpad, L.CG};
    }
    if (cap_bytes < *n_bytes) return packed || cap_bytes ? SUSHI_EINVAL : SUSHI_OK;
    std::memcpy(packed, src, *n_bytes);
    return SUSHI_OK;
}

int sushi_team_plan(const sushi_arch *arch, const sushi_subnet_cfg *cfg, int batch, int team_wgs, sushi_team_op *out,
                    int cap, int *n_out) {
    if (!arch || !cfg || !n_out || cap < 0 || (cap > 0 && !out) || batch < 1 || team_wgs < 1 || team_wgs > 32)
        return SUSHI_EINVAL;
    SuperNet sn;
    std::string err;
    int rc = build_supernet(*arch, sn, err);
    if (rc) return rc;
    Plan plan;
    rc = plan_subnet(sn, *cfg, batch, plan, err);
    if (rc) return rc;
    *n_out = (int)plan.ops.size();
    std::vector<DevOp> prog;
    for (int i = 0; i < *n_out; ++i) {
        const Op &o = plan.ops[i];
        DevOp op{};
        op.kind = o.kind;
        op.layer = (o.kind == OP_CONV || o.kind == OP_FC) ? o.layer : -1;
        op.in_patch = o.in_buf == BUF_INPUT, op.out_patch = o.out_buf == BUF_LOGITS;
        op.pool.B = o.B, op.pool.H = o.H, op.pool.W = o.W, op.pool.C = o.C, op.pool.P = o.P, op.pool.Q = o.Q;
        if (o.kind == OP_CONV || o.kind == OP_DW || o.kind == OP_FC) {
            const SuperLayer &S = sn.layers[o.layer];
            ConvArgs &a = op.conv;
            a.B = o.B, a.H = o.H, a.W = o.W, a.C = o.C, a.P = o.P, a.Q = o.Q, a.K = o.K;
            a.R = o.r, a.stride = o.stride, a.pad = o.pad, a.Rmax = S.Rmax;
            a.Kpad = S.Kpad, a.CG = S.CG;
            a.act = o.act, a.hsigmoid = o.hsigmoid ? 1 : 0, a.out_f32 = o.out_f32 ? 1 : 0;
            a.in_f32 = o.in_small ? 1 : 0;
            a.res = o.res_buf >= 0 ? &op : nullptr;  // (only whether there is one matters to the tiling)
        }
        if (!tile_team_op(op, team_wgs)) return SUSHI_ESTATE;
        op.conv.res = nullptr;
        prog.push_back(op);
    }
    fuse_se_blocks(prog, plan);
    for (int i = 0; i < *n_out && i < cap; ++i) {
        const Op &o = plan.ops[i];
        const DevOp &op = prog[i];
        sushi_team_op &t = out[i];
        t.kind = op.kind, t.layer = op.layer;
        t.B = o.B, t.H = o.H, t.W = o.W, t.C = o.C, t.P = o.P, t.Q = o.Q, t.K = o.K, t.R = o.r, t.stride = o.stride;
        t.ft = op.ft, t.pt = op.pt, t.wk = op.wk, t.n_units = op.n_units, t.n_p = op.n_p;
        t.lds_bytes = (int32_t)dev_op_lds_bytes(op);
        t.res = o.res_buf >= 0 ? 1 : 0, t.out_f32 = o.out_f32 ? 1 : 0;
        if (op.kind == DEV_SE) t.P = o.H, t.Q = o.W, t.K = op.se.mid, t.out_f32 = 0;  // (o is the block's pooling op)
    }
    return SUSHI_OK;
}

int sushi_create(sushi_ctx **out, int device_id, void *hip_stream) {
    if (!out) return SUSHI_EINVAL;
    *out = nullptr;
    if (device_id == -1) {  // host-only context: scheduler and planning calls, no device work
        sushi_ctx *h = new (std::nothrow) sushi_ctx();
        if (!h) return SUSHI_ENOMEM;
        h->device = -1;
        *out = h;
        return SUSHI_OK;
    }
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || device_id < 0 || device_id >= n) {
        g_create_error = e != hipSuccess ? std::string("hipGetDeviceCount: ") + hipGetErrorString(e)
                                         : "no such device";
        return e != hipSuccess ? SUSHI_EDEVICE : SUSHI_EINVAL;
    }
    if ((e = hipSetDevice(device_id)) != hipSuccess) {
        g_create_error = std::string("hipSetDevice: ") + hipGetErrorString(e);
        return SUSHI_EDEVICE;
    }
    sushi_ctx *c = new (std::nothrow) sushi_ctx();
    if (!c) return SUSHI_ENOMEM;
    c->device = device_id;
    c->stream = static_cast<hipStream_t>(hip_stream);
    // address of the static scratch array on this device (device_id is current), for sushi_infer_static
    if ((e = static_scratch(device_id, &c->static_buf)) != hipSuccess) {
        g_create_error = std::string("hipGetSymbolAddress(static scratch): ") + hipGetErrorString(e);
        delete c;
        return SUSHI_EDEVICE;
    }
    *out = c;
    return SUSHI_OK;
}

void sushi_destroy(sushi_ctx *c) {
    if (!c) return;
    if (c->device < 0) {
        delete c;
        return;
    }
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->stream);
    c->plans.clear();
    (void)drain_timing(c);
    for (hipEvent_t ev : c->free_events) (void)hipEventDestroy(ev);
    if (c->capture_stream) (void)hipStreamDestroy(c->capture_stream);
    if (c->th) {
        (void)stop_team_kernel(c);
        (void)hipStreamDestroy(c->pstream);
        (void)hipFree(c->d_tsync);
        if (c->d_trace) (void)hipFree(c->d_trace);
        for (auto &g : c->res_gens) free_res_gen(g);
        if (c->h_prog_pool) (void)hipHostFree(c->h_prog_pool);
        if (c->d_team_mem) (void)hipFree(c->d_team_mem);
        if (c->d_tarena) (void)hipFree(c->d_tarena);
        (void)hipHostFree(c->th);
    }
    if (c->d_sweep) (void)hipFree(c->d_sweep);
    if (c->d_sync) (void)hipFree(c->d_sync);
    if (c->h_abort) (void)hipHostFree(c->h_abort);
    free_arena(c);
    if (c->d_weights) (void)hipFree(c->d_weights);
    if (c->d_params) (void)hipFree(c->d_params);
    if (c->d_qparams) (void)hipFree(c->d_qparams);
    if (c->d_wsum) (void)hipFree(c->d_wsum);
    delete c;
}

const char *sushi_last_error(const sushi_ctx *c) { return c ? c->err.c_str() : g_create_error.c_str(); }

int sushi_load_supernet(sushi_ctx *c, const sushi_arch *arch, const void *weights, size_t nbytes, int dtype) {
    if (!c) return SUSHI_EINVAL;
    if (c->device < 0) return fail(c, SUSHI_ESTATE, "load: host-only context");
    if (!arch || !weights) return fail(c, SUSHI_EINVAL, "load: null argument");
    if (dtype != SUSHI_FP32 && dtype != SUSHI_BF16) return fail(c, SUSHI_EINVAL, "load: unknown compute dtype");
    SuperNet sn;
    std::string err;
    int rc = build_supernet(*arch, sn, err);
    if (rc) return fail(c, rc, err);
    if (nbytes != sn.blob_floats * sizeof(float))
        return fail(c, SUSHI_EINVAL, "load: blob holds " + std::to_string(nbytes) + " bytes, the SuperNet needs " +
                                         std::to_string(sn.blob_floats * sizeof(float)));
    hipError_t e;
    if ((rc = drop_loaded(c)) != SUSHI_OK) return rc;

    const float *blob = static_cast<const float *>(weights);
    std::vector<float> params;
    size_t wbytes = 0;
    const void *wsrc = nullptr;
    std::vector<uint16_t> w16;
    std::vector<float> w32;
    try {
        if (dtype == SUSHI_BF16) {
            pack_weights<uint16_t>(sn, blob, w16, params, to_bf16);
            wbytes = w16.size() * 2, wsrc = w16.data();
        } else {
            pack_weights<float>(sn, blob, w32, params, [](float f) { return f; });
            wbytes = w32.size() * 4, wsrc = w32.data();
        }
    } catch (const std::bad_alloc &) {
        return fail(c, SUSHI_ENOMEM, "load: host staging allocation failed");
    }
    if ((e = hipMalloc(&c->d_weights, std::max<size_t>(wbytes, 256))) != hipSuccess)
        return fail(c, SUSHI_ENOMEM, "load: hipMalloc(weights)");
    if ((e = hipMalloc(reinterpret_cast<void **>(&c->d_params), std::max<size_t>(params.size() * 4, 256))) !=
        hipSuccess)
        return fail(c, SUSHI_ENOMEM, "load: hipMalloc(params)");
    if ((e = hipMemcpy(c->d_weights, wsrc, wbytes, hipMemcpyHostToDevice)) != hipSuccess)
        return hip_fail(c, e, "hipMemcpy(weights)");
    if ((e = hipMemcpy(c->d_params, params.data(), params.size() * 4, hipMemcpyHostToDevice)) != hipSuccess)
        return hip_fail(c, e, "hipMemcpy(params)");
    c->sn = std::move(sn);
    c->bf16 = dtype == SUSHI_BF16;
    c->weight_elems = wbytes / (c->bf16 ? 2 : 4);
    c->loaded = true;
    return SUSHI_OK;
}

int sushi_load_supernet_int8(sushi_ctx *c, const sushi_arch *arch, const int8_t *weights, size_t n_weights,
                             const int32_t *qparams, size_t n_qparams) {
    if (!c) return SUSHI_EINVAL;
    if (c->device < 0) return fail(c, SUSHI_ESTATE, "load: host-only context");
    if (!arch || !weights || !qparams) return fail(c, SUSHI_EINVAL, "load: null argument");
    if (arch->family != SUSHI_FAMILY_TINY && arch->family != SUSHI_FAMILY_RESNET)
        return fail(c, SUSHI_EINVAL, "load: the int8 path covers the TINY and RESNET families");
    SuperNet sn;
    std::string err;
    int rc = build_supernet(*arch, sn, err);
    if (rc) return fail(c, rc, err);
    size_t need_w = 0, need_q = 0;
    for (const SuperLayer &L : sn.layers) {
        if (L.type == L_DW) return fail(c, SUSHI_EINVAL, "load: no int8 depthwise layers");
        need_w += (size_t)L.Kmax * L.Cmax * L.Rmax * L.Rmax;
        need_q += 3 * (size_t)L.Kmax + 8;
    }
    if (n_weights != need_w || n_qparams != need_q)
        return fail(c, SUSHI_EINVAL, "load: the SuperNet needs " + std::to_string(need_w) + " int8 weights and " +
                                         std::to_string(need_q) + " int32 parameter words");
    if ((rc = drop_loaded(c)) != SUSHI_OK) return rc;

    // Packed layout: [tap][channel group of 16][filter, padded to 16][16 channels], channels beyond Cmax zero; a
    // matrix-core operand of 16 filters x 64 channels is four runs of 256 bytes.  Parameter words per layer:
    // mult[Kpad], rshift[Kpad], bias[Kpad].  Prefix sums per conv layer: wsum[g][k] = sum of w_q[k][c][tap] over
    // all taps and the channels c < 8 (g + 1): the zero-point term of a SubNet that keeps 8 (g + 1) channels.
    std::vector<int8_t> w8;
    std::vector<int32_t> q, wsum;
    try {
        size_t welems = 0, qwords = 0, swords = 0;
        for (SuperLayer &L : sn.layers) {
            L.Kpad = (int)round_up(L.Kmax, 16);
            L.CG16 = (L.Cmax + 15) / 16;
            L.CG = (L.Cmax + 7) / 8;
            L.pk_w = welems;
            welems = round_up(welems + (size_t)L.Rmax * L.Rmax * L.CG16 * L.Kpad * 16, 256);
            L.pk_q = qwords;
            qwords += 3 * (size_t)L.Kpad;
            L.pk_wsum = swords;
            if (L.type == L_CONV && L.Cmax >= 8) swords += (size_t)L.CG * L.Kpad;
        }
        w8.assign(welems, 0);
        q.assign(std::max<size_t>(qwords, 64), 0);
        wsum.assign(std::max<size_t>(swords, 64), 0);
        const int8_t *src = weights;
        const int32_t *qs = qparams;
        for (SuperLayer &L : sn.layers) {
            const int R2 = L.Rmax * L.Rmax;
            int8_t *dst = w8.data() + L.pk_w;
            for (int k = 0; k < L.Kmax; ++k)
                for (int ch = 0; ch < L.Cmax; ++ch)
                    for (int t = 0; t < R2; ++t)
                        dst[(((size_t)t * L.CG16 + ch / 16) * L.Kpad + k) * 16 + (ch & 15)] = src[((size_t)k * L.Cmax + ch) * R2 + t];
            if (L.type == L_CONV && L.Cmax >= 8) {
                int32_t *ws = wsum.data() + L.pk_wsum;
                for (int k = 0; k < L.Kmax; ++k) {
                    int32_t run = 0;
                    for (int ch = 0; ch < L.Cmax; ++ch) {
                        for (int t = 0; t < R2; ++t) run += src[((size_t)k * L.Cmax + ch) * R2 + t];
                        if ((ch & 7) == 7 || ch == L.Cmax - 1) ws[(size_t)(ch / 8) * L.Kpad + k] = run;
                    }
                }
            }
            src += (size_t)L.Kmax * L.Cmax * R2;
            int32_t *qd = q.data() + L.pk_q;
            for (int k = 0; k < L.Kmax; ++k) {
                qd[k] = qs[k], qd[L.Kpad + k] = qs[L.Kmax + k], qd[2 * L.Kpad + k] = qs[2 * L.Kmax + k];
                if (L.type == L_CONV && (qd[L.Kpad + k] < 1 || qd[L.Kpad + k] > 62))
                    return fail(c, SUSHI_EINVAL, "load: shift of layer " + L.name + " outside 1 .. 62");
            }
            for (int k = L.Kmax; k < L.Kpad; ++k) qd[L.Kpad + k] = 1;
            for (int i = 0; i < 8; ++i) L.qscalars[i] = qs[3 * (size_t)L.Kmax + i];
            if (L.qscalars[0] < -128 || L.qscalars[0] > 127 || L.qscalars[1] < -128 || L.qscalars[1] > 127 ||
                L.qscalars[4] < -128 || L.qscalars[4] > 127 || L.qscalars[3] < 0 || L.qscalars[3] > 62 || L.qscalars[2] < 0)
                return fail(c, SUSHI_EINVAL, "load: scalars of layer " + L.name + " out of range");
            qs += 3 * (size_t)L.Kmax + 8;
        }
    } catch (const std::bad_alloc &) {
        return fail(c, SUSHI_ENOMEM, "load: host staging allocation failed");
    }
    hipError_t e;
    if (hipMalloc(&c->d_weights, std::max<size_t>(w8.size(), 256)) != hipSuccess) return fail(c, SUSHI_ENOMEM, "load: hipMalloc(weights)");
    if (hipMalloc(reinterpret_cast<void **>(&c->d_qparams), q.size() * 4) != hipSuccess) return fail(c, SUSHI_ENOMEM, "load: hipMalloc(parameter words)");
    if (hipMalloc(reinterpret_cast<void **>(&c->d_wsum), wsum.size() * 4) != hipSuccess) return fail(c, SUSHI_ENOMEM, "load: hipMalloc(weight sums)");
    if ((e = hipMemcpy(c->d_weights, w8.data(), w8.size(), hipMemcpyHostToDevice)) != hipSuccess) return hip_fail(c, e, "hipMemcpy(weights)");
    if ((e = hipMemcpy(c->d_qparams, q.data(), q.size() * 4, hipMemcpyHostToDevice)) != hipSuccess) return hip_fail(c, e, "hipMemcpy(parameter words)");
    if ((e = hipMemcpy(c->d_wsum, wsum.data(), wsum.size() * 4, hipMemcpyHostToDevice)) != hipSuccess) return hip_fail(c, e, "hipMemcpy(weight sums)");
    c->sn = std::move(sn);
    c->bf16 = false, c->int8 = true;
    c->weight_elems = w8.size();
    c->loaded = true;
    return SUSHI_OK;
}

int sushi_set_subgraph_cache(sushi_ctx *c, const sushi_subgraph_cfg *g, size_t budget_bytes) {
    if (!c) return SUSHI_EINVAL;
    if (!c->loaded) return fail(c, SUSHI_ESTATE, "set_subgraph_cache before load_supernet");
    if (!g || g->n_layers == 0) {
        c->G.clear();
        ++c->g_version;
        c->stats.cache_bytes = 0;
        c->stats.cache_bytes_lds = 0;
        return install_on_teams(c);
    }
    if (g->n_layers != (int)c->sn.layers.size() || !g->layers)
        return fail(c, SUSHI_EINVAL, "SubGraph must list all " + std::to_string(c->sn.layers.size()) + " layers");
    uint64_t bytes = 0;
    for (int i = 0; i < g->n_layers; ++i) {
        const sushi_layer_dims &d = g->layers[i];
        const SuperLayer &L = c->sn.layers[i];
        if (d.K == 0) continue;
        if (d.K < 0 || d.K > L.Kmax || d.C < 1 || d.C > L.Cmax || d.r < 1 || d.r > L.Rmax || (d.r & 1) == 0)
            return fail(c, SUSHI_EINVAL, "SubGraph box of layer " + L.name + " lies outside the SuperNet");
        bytes += (uint64_t)d.K * d.C * d.r * d.r * elem_size(c);
    }
    if (bytes > budget_bytes)
        return fail(c, SUSHI_EBUDGET, "SubGraph needs " + std::to_string(bytes) + " bytes, budget is " +
                                          std::to_string(budget_bytes));
    c->G.assign(g->layers, g->layers + g->n_layers);
    for (sushi_layer_dims &d : c->G)
        if (d.K == 0) d = sushi_layer_dims{0, 0, 0};
    ++c->g_version;
    c->stats.cache_installs += 1;
    c->stats.cache_bytes_installed += bytes;
    c->stats.cache_bytes = bytes;
    int rc = install_on_teams(c);
    c->stats.cache_bytes_lds = c->table_bytes;
    return rc;
}

int sushi_infer(sushi_ctx *c, const sushi_subnet_cfg *cfg, const void *input_dev, int batch, void *logits_dev) {
    if (!c) return SUSHI_EINVAL;
    if (!c->loaded) return fail(c, SUSHI_ESTATE, "infer before load_supernet");
    if (!cfg || !input_dev || !logits_dev || batch < 1) return fail(c, SUSHI_EINVAL, "infer: bad argument");
    if (c->int8 && c->exec_mode != 0) return fail(c, SUSHI_ESTATE, "infer: the int8 path runs in exec mode 0 only");
    hipError_t e;
    if ((e = hipSetDevice(c->device)) != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    CachedPlan *cp = nullptr;
    const std::string key = plan_key(*cfg, batch);
    auto it = c->plans.find(key);
    if (it != c->plans.end() && batch <= c->arena_batch) {
        cp = it->second.get();
        c->stats.plan_cache_hits++;
    } else {
        std::unique_ptr<CachedPlan> np(new (std::nothrow) CachedPlan());
        if (!np) return fail(c, SUSHI_ENOMEM, "infer: plan allocation failed");
        std::string err;
        int rc = plan_subnet(c->sn, *cfg, batch, np->plan, err);
        if (rc) return fail(c, rc, err);
        if ((rc = ensure_arena(c, batch)) != SUSHI_OK) return rc;
        bind_plan(c, *np);
        cp = np.get();
        c->plans[key] = std::move(np);
        c->stats.plan_cache_misses++;
    }
    refresh_residency(c, *cp);
    if (cp->alg_bytes == 0.0)
        for (const Launch &L : cp->launches) {
            double b = 0.0, f = 0.0;
            launch_cost(c, L, &b, &f);
            cp->alg_bytes += b, cp->alg_flops += f;
        }

    if (c->exec_mode != 3) c->stream_dirty = true;
    if (c->exec_mode != 3 && c->sweep_bytes) {
        if ((e = launch_cold_sweep(c->d_sweep, c->sweep_bytes, c->d_sweep, c->stream)) != hipSuccess)
            return hip_fail(c, e, "cache sweep");
    }
    if (c->exec_mode == 3) {
        int rc = post_team_query(c, *cp, input_dev, logits_dev, batch);
        if (rc) return rc;
    } else if (c->exec_mode == 2) {
        int rc = run_stream_kernel(c, *cp, input_dev, logits_dev);
        if (rc) return rc;
    } else if (c->exec_mode == 1) {
        int rc = replay_graph(c, *cp, input_dev, logits_dev);
        if (rc) return rc;
    } else {
        e = issue_launches(c, *cp, input_dev, logits_dev, c->stream);
        if (e != hipSuccess) return hip_fail(c, e, "kernel launch");
    }
    sushi_stats &s = c->stats;
    s.queries++;
    s.weight_bytes_total += cp->weight_bytes;
    s.weight_bytes_in_subgraph += cp->resident_bytes;
    s.last_weight_bytes = cp->weight_bytes;
    s.last_in_subgraph_bytes = cp->resident_bytes;
    s.last_hit_ratio = cp->hit_ratio;
    s.sum_hit_ratio += cp->hit_ratio;
    return SUSHI_OK;
}

int sushi_infer_static(sushi_ctx *c, const sushi_subnet_cfg *cfg, const void *input_dev, int batch, void *logits_dev) {
    if (!c) return SUSHI_EINVAL;
    if (!c->loaded) return fail(c, SUSHI_ESTATE, "infer before load_supernet");
    if (!cfg || !input_dev || !logits_dev || batch < 1) return fail(c, SUSHI_EINVAL, "infer: bad argument");
    hipError_t e;
    if ((e = hipSetDevice(c->device)) != hipSuccess) return hip_fail(c, e, "hipSetDevice");
    if (!c->static_buf) return fail(c, SUSHI_ESTATE, "the static scratch buffer was not found on this device");
    CachedPlan *cp = nullptr;
    std::string key = plan_key(*cfg, batch);
    key.push_back('S');  // (plans bound to the static buffer are kept apart from those bound to the arena)
    auto it = c->plans.find(key);
    if (it != c->plans.end()) {
        cp = it->second.get();
        c->stats.plan_cache_hits++;
    } else {
        std::unique_ptr<CachedPlan> np(new (std::nothrow) CachedPlan());
        if (!np) return fail(c, SUSHI_ENOMEM, "infer: plan allocation failed");
        std::string err;
        int rc = plan_subnet(c->sn, *cfg, batch, np->plan, err);
        if (rc) return fail(c, rc, err);
        // the activation buffers of THIS SubNet at this batch size and resolution, cut out of the static array
        BufBase bb;
        bb.block = static_cast<char *>(c->static_buf);
        bb.big_bytes = round_up(np->plan.max_big_elems * elem_size(c), 256);
        bb.small_bytes = round_up(std::max<size_t>(np->plan.max_small_elems, 8) * 4, 256);
        const size_t need = N_BIG_BUFS * bb.big_bytes + N_SMALL_BUFS * bb.small_bytes;
        if (need > STATIC_SCRATCH_BYTES)
            return fail(c, SUSHI_ENOMEM, "infer_static: this SubNet needs " + std::to_string(need) +
                                             " bytes of activation scratch at this batch size and resolution, the "
                                             "static buffer holds " + std::to_string(STATIC_SCRATCH_BYTES));
        bind_plan(c, *np, bb);
        cp = np.get();
        c->plans[key] = std::move(np);
        c->stats.plan_cache_misses++;
    }
    refresh_residency(c, *cp);
    c->stream_dirty = true;
    // one launch per op on the context's stream; no events, no allocation
    const bool timing = c->timing;
    c->timing = false;
    e = issue_launches(c, *cp, input_dev, logits_dev, c->stream);
    c->timing = timing;
    if (e != hipSuccess) return hip_fail(c, e, "kernel launch");
    sushi_stats &s = c->stats;
    s.queries++;
    s.weight_bytes_total += cp->weight_bytes;
    s.weight_bytes_in_subgraph += cp->resident_bytes;
    s.last_weight_bytes = cp->weight_bytes;
    s.last_in_subgraph_bytes = cp->resident_bytes;
    s.last_hit_ratio = cp->hit_ratio;
    s.sum_hit_ratio += cp->hit_ratio;
    return SUSHI_OK;
}

int sushi_sched_init(sushi_ctx *c, const sushi_sched_desc *d) {
    if (!c) return SUSHI_EINVAL;
    if (!d) return fail(c, SUSHI_EINVAL, "sched_init: null descriptor");
    std::string err;
    int rc = c->sched.init(*d, err);
    return rc ? fail(c, rc, err) : SUSHI_OK;
}

int sushi_sched_step(sushi_ctx *c, float acc_target, float lat_target, int *subnet_idx_out, int *new_cache_idx_out) {
    if (!c) return SUSHI_EINVAL;
    if (!c->sched.ready()) return fail(c, SUSHI_ESTATE, "sched_step before sched_init");
    if (!subnet_idx_out || !new_cache_idx_out) return fail(c, SUSHI_EINVAL, "sched_step: null output");
    const int i = c->sched.select(acc_target, lat_target);
    *subnet_idx_out = i;
    *new_cache_idx_out = c->sched.record(c->sched.subnet_vec(i));
    return SUSHI_OK;
}

int sushi_sched_record(sushi_ctx *c, const int32_t *vec, int *new_cache_idx_out) {
    if (!c) return SUSHI_EINVAL;
    if (!c->sched.ready()) return fail(c, SUSHI_ESTATE, "sched_record before sched_init");
    if (!vec || !new_cache_idx_out) return fail(c, SUSHI_EINVAL, "sched_record: null argument");
    *new_cache_idx_out = c->sched.record(vec);
    return SUSHI_OK;
}

int sushi_team_trace(sushi_ctx *c, int enable, uint64_t *out, int cap) {
    if (!c || c->device < 0) return SUSHI_EINVAL;
    hipError_t e;
    int rc = synchronize_teams(c);
    if (rc) return rc;
    if ((rc = stop_team_kernel(c)) != SUSHI_OK) return rc;
    if (out && c->d_trace && cap > 0) {
        const size_t n = std::min<size_t>((size_t)cap, (size_t)MAX_TEAMS * TRACE_SLOTS);
        if ((e = hipMemcpy(out, c->d_trace, n * 8, hipMemcpyDeviceToHost)) != hipSuccess) return hip_fail(c, e, "hipMemcpy(trace)");
    }
    if (enable && !c->d_trace) {
        if ((e = hipMalloc(reinterpret_cast<void **>(&c->d_trace), MAX_TEAMS * TRACE_SLOTS * 8)) != hipSuccess)
            return fail(c, SUSHI_ENOMEM, "hipMalloc(trace)");
        (void)hipMemset(c->d_trace, 0, MAX_TEAMS * TRACE_SLOTS * 8);
    } else if (!enable && c->d_trace) {
        (void)hipFree(c->d_trace);
        c->d_trace = nullptr;
    }
    return SUSHI_OK;
}

int sushi_quiesce(sushi_ctx *c) {
    if (!c) return SUSHI_EINVAL;
    if (c->device < 0) return SUSHI_OK;
    int rc = sushi_synchronize(c);
    if (rc) return rc;
    return c->th ? stop_team_kernel(c) : SUSHI_OK;
}

int sushi_synchronize(sushi_ctx *c) {
    if (!c) return SUSHI_EINVAL;
    if (c->device < 0) return SUSHI_OK;
    int rc = synchronize_teams(c);
    if (rc) return rc;
    // Nothing of this library runs on the context's stream in mode 3, and a wait on the default
    // stream may wait for the persistent kernel instead (until it idles out).
    if (c->exec_mode == 3 && !c->stream_dirty) return SUSHI_OK;
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
    c->stream_dirty = false;
    return SUSHI_OK;
}

int sushi_get_stats(sushi_ctx *c, sushi_stats *out) {
    if (!c || !out) return SUSHI_EINVAL;
    *out = c->stats;
    return SUSHI_OK;
}

int sushi_get_kernel_stats(sushi_ctx *c, sushi_kernel_stats *out, int cap, int *n_out) {
    if (!c || !n_out || cap < 0 || (cap > 0 && !out)) return SUSHI_EINVAL;
    if (c->device >= 0) {
        if (c->th) {
            int rc = synchronize_teams(c);
            if (rc == SUSHI_OK) rc = stop_team_kernel(c);
            if (rc) return rc;
        }
        hipError_t e = drain_timing(c);
        if (e != hipSuccess) return hip_fail(c, e, "kernel timing");
    }
    *n_out = KC_COUNT;
    for (int i = 0; i < cap && i < KC_COUNT; ++i) {
        out[i] = c->kstats[i];
        std::snprintf(out[i].name, sizeof(out[i].name), "%s", kernel_class_name(i));
    }
    return SUSHI_OK;
}

int sushi_get_launch_records(sushi_ctx *c, sushi_launch_record *out, int cap, int *n_out) {
    if (!c || !n_out || cap < 0 || (cap > 0 && !out)) return SUSHI_EINVAL;
    if (c->device >= 0) {
        hipError_t e = drain_timing(c);
        if (e != hipSuccess) return hip_fail(c, e, "kernel timing");
    }
    *n_out = (int)c->records.size();
    for (int i = 0; i < cap && i < *n_out; ++i) out[i] = c->records[i];
    return SUSHI_OK;
}

int sushi_set_option(sushi_ctx *c, int option, int64_t value) {
    if (!c) return SUSHI_EINVAL;
    if (option == SUSHI_OPT_KERNEL_TIMING && (value == 0 || value == 1)) {
        if (c->device >= 0) (void)drain_timing(c);
        if (value == 1) {
            for (auto &k : c->kstats) k = sushi_kernel_stats{};
            c->records.clear();
        }
        c->timing = value == 1;
        return SUSHI_OK;
    }
    if (option == SUSHI_OPT_SPIN_LIMIT && value >= 0 && value <= 100000000) {
        c->spin_limit = (int)value;
        return SUSHI_OK;
    }
    if (option == SUSHI_OPT_EXEC_MODE && value >= 0 && value <= 3) {
        if (c->exec_mode == 3 && value != 3 && c->th) {
            int rc = synchronize_teams(c);
            if (rc) return rc;
            if ((rc = stop_team_kernel(c)) != SUSHI_OK) return rc;
        }
        c->exec_mode = (int)value;
        return SUSHI_OK;
    }
    if (option == SUSHI_OPT_STREAM_WGS && value >= BARRIER_GROUP && value <= 1024 && value % BARRIER_GROUP == 0) {
        if (c->d_sync || c->th) return fail(c, SUSHI_ESTATE, "set the workgroup count before the first query");
        c->stream_wgs_override = (int)value;
        return SUSHI_OK;
    }
    if (option == SUSHI_OPT_TEAM_WGS_PER_CU && value >= 1 && value <= 2) {
        if (c->th) return fail(c, SUSHI_ESTATE, "set the workgroup count before the first query");
        c->team_wgs_per_cu = (int)value;
        return SUSHI_OK;
    }
    if (option == SUSHI_OPT_TEAMS_PER_XCD && (value == 1 || value == 2 || value == 4 || value == 8 || value == 16) && value <= MAX_TEAMS / MAX_XCDS) {
        if (c->th) return fail(c, SUSHI_ESTATE, "set the number of teams before the first query");
        c->teams_per_xcd = (int)value;
        return SUSHI_OK;
    }
    if (option == SUSHI_OPT_COLD_SWEEP_MIB && value >= 0 && value <= 4096) {
        if (c->device < 0) return fail(c, SUSHI_ESTATE, "set_option: host-only context");
        hipError_t e = hipStreamSynchronize(c->stream);
        if (e != hipSuccess) return hip_fail(c, e, "hipStreamSynchronize");
        if (c->d_sweep) (void)hipFree(c->d_sweep);
        c->d_sweep = nullptr, c->sweep_bytes = 0;
        if (value == 0) return SUSHI_OK;
        if (c->th) {  // an allocation may wait for the persistent kernel to leave
            int rc = synchronize_teams(c);
            if (rc == SUSHI_OK) rc = stop_team_kernel(c);
            if (rc) return rc;
        }
        const size_t bytes = (size_t)value << 20;
        if (hipMalloc(&c->d_sweep, bytes) != hipSuccess) return fail(c, SUSHI_ENOMEM, "hipMalloc(cache sweep buffer)");
        if ((e = hipMemset(c->d_sweep, 0, bytes)) != hipSuccess) return hip_fail(c, e, "hipMemset");
        c->sweep_bytes = bytes;
        return SUSHI_OK;
    }
    if (option == SUSHI_OPT_PATCH_CONV_MIN_PIXELS && value >= 0 && value <= (1l << 40)) {
        c->patch_min_pixels = (long)value;
        return SUSHI_OK;
    }
    if (option == SUSHI_OPT_IDLE_US && value >= 10 && value <= 10000000) {
        c->idle_ticks = (long)value * 100;
        return SUSHI_OK;
    }
    return fail(c, SUSHI_EINVAL, "set_option: unknown option or value");
}

}  // extern "C"
