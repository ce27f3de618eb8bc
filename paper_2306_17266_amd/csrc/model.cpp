// SuperNet tables and the per-query SubNet plan (host only).  See model.h.
#include "model.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>

namespace sushi {

int round_channels(double x) {
    int v = std::max(8, (int)std::floor(x / 8.0 + 0.5) * 8);
    if ((double)v < 0.9 * x) v += 8;
    return v;
}

int SuperNet::layer_index(const std::string &name) const {
    for (size_t i = 0; i < layers.size(); ++i)
        if (layers[i].name == name) return (int)i;
    return -1;
}

namespace {

bool in_list(const int32_t *list, int n, int v) {
    for (int i = 0; i < n; ++i)
        if (list[i] == v) return true;
    return false;
}

double max_of(const double *v, int n) {
    double m = v[0];
    for (int i = 1; i < n; ++i) m = std::max(m, v[i]);
    return m;
}

int check_arch(const sushi_arch &a, std::string &err) {
    auto bad = [&](const char *m) {
        err = std::string("arch: ") + m;
        return (int)SUSHI_EINVAL;
    };
    if (a.family < SUSHI_FAMILY_TINY || a.family > SUSHI_FAMILY_MBV3) return bad("unknown family");
    if (a.n_stages < 1 || a.n_stages > SUSHI_MAX_STAGES) return bad("n_stages out of range");
    if (a.n_classes < 1 || a.in_channels < 1 || a.in_channels > 8) return bad("n_classes / in_channels");
    auto cnt = [](int n) { return n >= 1 && n <= SUSHI_MAX_CHOICES; };
    if (!cnt(a.n_depth_drop) || !cnt(a.n_width) || !cnt(a.n_expand) || !cnt(a.n_kernel) || !cnt(a.n_res))
        return bad("choice list length");
    int slots = 0;
    for (int s = 0; s < a.n_stages; ++s) {
        if (a.stage_base_out[s] < 8 || a.stage_stride[s] < 1 || a.stage_stride[s] > 2 || a.stage_max_depth[s] < 1)
            return bad("stage parameters");
        if (a.family == SUSHI_FAMILY_TINY && a.stage_max_depth[s] != 1) return bad("TINY stages hold one layer");
        slots += a.stage_max_depth[s];
    }
    if (slots > SUSHI_MAX_BLOCKS) return bad("too many block slots");
    for (int i = 0; i < a.n_kernel; ++i)
        if (a.kernel_choices[i] < 1 || a.kernel_choices[i] > 7 || a.kernel_choices[i] % 2 == 0)
            return bad("kernel sizes must be odd and at most 7");
    for (int i = 0; i < a.n_width; ++i)
        if (!(a.width_choices[i] > 0.0)) return bad("width multipliers");
    for (int i = 0; i < a.n_expand; ++i)
        if (!(a.expand_choices[i] > 0.0)) return bad("expand ratios");
    for (int i = 0; i < a.n_depth_drop; ++i)
        if (a.depth_drop_choices[i] < 0) return bad("depth choices");
    for (int i = 0; i < a.n_res; ++i)
        if (a.res_choices[i] < 8) return bad("resolutions");
    if (a.family == SUSHI_FAMILY_RESNET && (a.stem_mid < 8 || a.stem_out < 8)) return bad("stem widths");
    if (a.family == SUSHI_FAMILY_MBV3 && (a.stem_out < 8 || a.head_mid < 8 || a.head_feat < 8 ||
                                          a.stem_out % 8 || a.head_mid % 8 || a.head_feat % 8))
        return bad("MBV3 stem/head widths must be multiples of 8");
    if (a.family == SUSHI_FAMILY_MBV3)
        for (int s = 0; s < a.n_stages; ++s)
            if (a.stage_base_out[s] % 8) return bad("MBV3 stage widths must be multiples of 8");
    return SUSHI_OK;
}

struct Builder {
    SuperNet &sn;
    size_t off = 0;
    void tensor(const std::string &name, int kind, std::initializer_list<int> shape) {
        sushi_tensor_desc d{};
        std::snprintf(d.name, sizeof(d.name), "%s", name.c_str());
        d.kind = kind;
        d.ndim = (int)shape.size();
        size_t n = 1;
        int i = 0;
        for (int s : shape) {
            d.shape[i++] = s;
            n *= (size_t)s;
        }
        sn.tensors.push_back(d);
        off += n;
    }
    void conv(const std::string &name, int k, int c, int r, bool res_scale = false, bool dw = false) {
        SuperLayer L;
        L.name = name;
        L.type = dw ? L_DW : L_CONV;
        L.Kmax = k;
        L.Cmax = dw ? 1 : c;
        L.Rmax = r;
        L.res_scale = res_scale;
        L.blob_w = off;
        tensor(name + ".w", dw ? SUSHI_T_DWCONV : SUSHI_T_CONV, {k, dw ? 1 : c, r, r});
        L.blob_scale = off;
        tensor(name + ".scale", res_scale ? SUSHI_T_SCALE_RES : SUSHI_T_SCALE, {k});
        L.blob_shift = off;
        tensor(name + ".shift", SUSHI_T_SHIFT, {k});
        sn.layers.push_back(L);
    }
    void fc(const std::string &name, int k, int c) {
        SuperLayer L;
        L.name = name;
        L.type = L_FC;
        L.Kmax = k;
        L.Cmax = c;
        L.Rmax = 1;
        L.has_scale = false;
        L.blob_w = off;
        tensor(name + ".w", SUSHI_T_FC, {k, c});
        L.blob_shift = off;
        tensor(name + ".b", SUSHI_T_BIAS, {k});
        sn.layers.push_back(L);
    }
};

std::string blk(int s, int j) { return "s" + std::to_string(s) + "b" + std::to_string(j); }

}  // namespace

int build_supernet(const sushi_arch &a, SuperNet &sn, std::string &err) {
    int rc = check_arch(a, err);
    if (rc) return rc;
    sn = SuperNet();
    sn.arch = a;
    Builder b{sn};
    const double wmax = max_of(a.width_choices, a.n_width), emax = max_of(a.expand_choices, a.n_expand);
    int kmax = 1;
    for (int i = 0; i < a.n_kernel; ++i) kmax = std::max(kmax, (int)a.kernel_choices[i]);

    if (a.family == SUSHI_FAMILY_TINY) {
        int cin = a.in_channels;
        for (int l = 0; l < a.n_stages; ++l) {
            int cout = round_channels(a.stage_base_out[l] * wmax);
            b.conv("conv" + std::to_string(l), cout, cin, 3);
            cin = cout;
        }
        b.fc("fc", a.n_classes, cin);
    } else if (a.family == SUSHI_FAMILY_RESNET) {
        int mid = round_channels(a.stem_mid * wmax), out = round_channels(a.stem_out * wmax);
        b.conv("stem0", mid, a.in_channels, 3);
        b.conv("stem1", mid, mid, 3);
        b.conv("stem2", out, mid, 3);
        int cin = out;
        for (int s = 0; s < a.n_stages; ++s) {
            int cout = round_channels(a.stage_base_out[s] * wmax);
            int cmid = round_channels(cout * emax);
            for (int j = 0; j < a.stage_max_depth[s]; ++j) {
                std::string n = blk(s, j);
                b.conv(n + ".conv1", cmid, cin, 1);
                b.conv(n + ".conv2", cmid, cmid, 3);
                b.conv(n + ".conv3", cout, cmid, 1, true);
                if (j == 0) b.conv(n + ".proj", cout, cin, 1);
                cin = cout;
            }
        }
        b.fc("fc", a.n_classes, cin);
    } else {
        int c0 = a.stem_out;
        b.conv("stem", c0, a.in_channels, 3);
        b.conv("first.dw", c0, 1, 3, false, true);
        b.conv("first.pw", c0, c0, 1, true);
        int cin = c0;
        for (int s = 0; s < a.n_stages; ++s) {
            int cout = a.stage_base_out[s];
            for (int j = 0; j < a.stage_max_depth[s]; ++j) {
                std::string n = blk(s, j);
                int stride = j == 0 ? a.stage_stride[s] : 1;
                int cmid = round_channels(cin * emax);
                b.conv(n + ".expand", cmid, cin, 1);
                b.conv(n + ".dw", cmid, 1, kmax, false, true);
                if (a.stage_se[s]) {
                    int red = round_channels(cmid / 4.0);
                    b.fc(n + ".se1", red, cmid);
                    b.fc(n + ".se2", cmid, red);
                }
                b.conv(n + ".project", cout, cmid, 1, stride == 1 && cin == cout);
                cin = cout;
            }
        }
        b.conv("head", a.head_mid, cin, 1);
        b.fc("feat", a.head_feat, a.head_mid);
        b.fc("fc", a.n_classes, a.head_feat);
    }
    sn.blob_floats = b.off;
    return SUSHI_OK;
}

namespace {

int check_cfg(const sushi_arch &a, const sushi_subnet_cfg &c, std::string &err) {
    auto bad = [&](const std::string &m) {
        err = "subnet cfg: " + m;
        return (int)SUSHI_EINVAL;
    };
    if (!in_list(a.res_choices, a.n_res, c.resolution)) return bad("resolution not offered");
    int slots = 0;
    if (a.family == SUSHI_FAMILY_TINY) {
        if (!in_list(a.depth_drop_choices, a.n_depth_drop, a.n_stages - c.depth[0])) return bad("depth not offered");
        slots = a.n_stages;
    } else {
        for (int s = 0; s < a.n_stages; ++s) {
            if (!in_list(a.depth_drop_choices, a.n_depth_drop, a.stage_max_depth[s] - c.depth[s]) || c.depth[s] < 1)
                return bad("depth of stage " + std::to_string(s) + " not offered");
            slots += a.stage_max_depth[s];
        }
    }
    for (int s = 0; s <= a.n_stages; ++s)
        if (c.width_idx[s] < 0 || c.width_idx[s] >= a.n_width) return bad("width index out of range");
    for (int b = 0; b < slots; ++b) {
        if (c.expand_idx[b] < 0 || c.expand_idx[b] >= a.n_expand) return bad("expand index out of range");
        if (c.kernel_idx[b] < 0 || c.kernel_idx[b] >= a.n_kernel) return bad("kernel index out of range");
    }
    return SUSHI_OK;
}

// Hands out feature-map buffers; a buffer is free when nobody holds it.
struct Bufs {
    bool busy[N_BIG_BUFS] = {};
    int get() {
        for (int i = 0; i < N_BIG_BUFS; ++i)
            if (!busy[i]) {
                busy[i] = true;
                return i;
            }
        return -1;
    }
    void put(int i) {
        if (i >= 0) busy[i] = false;
    }
};

struct Walker {
    const SuperNet &sn;
    Plan &plan;
    int B;
    Bufs bufs;
    int li = 0;  // next SuperNet layer

    int out_dim(int in, int r, int stride) { return (in + 2 * ((r - 1) / 2) - r) / stride + 1; }

    void note_big(size_t e) { plan.max_big_elems = std::max(plan.max_big_elems, e); }
    void note_small(size_t e) { plan.max_small_elems = std::max(plan.max_small_elems, e); }

    void skip(int n) {
        for (int i = 0; i < n; ++i) plan.dims[li++] = sushi_layer_dims{0, 0, 0};
    }

    // conv / depthwise layer `li` on feature map (buf, H, W, C) -> new buffer.
    int conv(int in_buf, int &H, int &W, int C, int K, int r, int stride, int act, int res_buf = BUF_NONE) {
        const SuperLayer &L = sn.layers[li];
        Op op;
        op.kind = L.type == L_DW ? OP_DW : OP_CONV;
        op.layer = li;
        op.B = B, op.H = H, op.W = W, op.C = C;
        op.r = r, op.stride = stride, op.pad = (r - 1) / 2;
        op.P = out_dim(H, r, stride), op.Q = out_dim(W, r, stride), op.K = K;
        op.act = act;
        op.in_buf = in_buf, op.res_buf = res_buf;
        op.out_buf = bufs.get();
        plan.ops.push_back(op);
        plan.dims[li++] = sushi_layer_dims{K, L.type == L_DW ? 1 : C, r};
        note_big((size_t)B * op.P * op.Q * K);
        H = op.P, W = op.Q;
        return op.out_buf;
    }

    void gap(int in_buf, int H, int W, int C, int out_small) {
        Op op;
        op.kind = OP_GAP;
        op.B = B, op.H = H, op.W = W, op.C = C, op.K = C, op.P = op.Q = 1;
        op.in_buf = in_buf, op.out_buf = out_small, op.out_small = true, op.out_f32 = true;
        plan.ops.push_back(op);
        note_small((size_t)B * C);
    }

    void fc(int in_small, int C, int K, int act, int out_buf, bool out_is_small, bool f32, bool hsig = false) {
        Op op;
        op.kind = OP_FC;
        op.layer = li;
        op.B = B, op.H = op.W = op.P = op.Q = 1, op.C = C, op.K = K;
        op.act = act, op.hsigmoid = hsig;
        op.in_buf = in_small, op.in_small = true;
        op.out_buf = out_buf, op.out_small = out_is_small, op.out_f32 = f32 || out_is_small;  // per-image vectors stay float32
        plan.ops.push_back(op);
        plan.dims[li++] = sushi_layer_dims{K, C, 1};
        if (out_is_small) note_small((size_t)B * K);
    }
};

}  // namespace

int plan_subnet(const SuperNet &sn, const sushi_subnet_cfg &c, int B, Plan &plan, std::string &err) {
    const sushi_arch &a = sn.arch;
    int rc = check_cfg(a, c, err);
    if (rc) return rc;
    if (B < 1) {
        err = "batch must be positive";
        return SUSHI_EINVAL;
    }
    plan = Plan();
    plan.dims.assign(sn.layers.size(), sushi_layer_dims{0, 0, 0});
    Walker w{sn, plan, B};
    int H = c.resolution, W = c.resolution;
    int x = BUF_INPUT, C = a.in_channels;

    if (a.family == SUSHI_FAMILY_TINY) {
        for (int l = 0; l < a.n_stages; ++l) {
            if (l >= c.depth[0]) {
                w.skip(1);
                continue;
            }
            int K = round_channels(a.stage_base_out[l] * a.width_choices[c.width_idx[1 + l]]);
            int y = w.conv(x, H, W, C, K, 3, 1, SUSHI_ACT_RELU);
            w.bufs.put(x);
            x = y, C = K;
        }
        w.gap(x, H, W, C, 0);
        w.fc(0, C, a.n_classes, SUSHI_ACT_NONE, BUF_LOGITS, false, true);
    } else if (a.family == SUSHI_FAMILY_RESNET) {
        const double w0 = a.width_choices[c.width_idx[0]];
        const int mid = round_channels(a.stem_mid * w0), out = round_channels(a.stem_out * w0);
        int y = w.conv(x, H, W, C, mid, 3, 2, SUSHI_ACT_RELU);
        x = y, C = mid;
        y = w.conv(x, H, W, C, mid, 3, 1, SUSHI_ACT_RELU);
        w.bufs.put(x), x = y;
        y = w.conv(x, H, W, C, out, 3, 1, SUSHI_ACT_RELU);
        w.bufs.put(x), x = y, C = out;
        {
            Op op;
            op.kind = OP_MAXPOOL;
            op.B = B, op.H = H, op.W = W, op.C = C, op.K = C;
            op.r = 3, op.stride = 2, op.pad = 1;
            op.P = w.out_dim(H, 3, 2), op.Q = w.out_dim(W, 3, 2);
            op.in_buf = x, op.out_buf = w.bufs.get();
            plan.ops.push_back(op);
            w.bufs.put(x);
            x = op.out_buf, H = op.P, W = op.Q;
        }
        int slot = 0;
        for (int s = 0; s < a.n_stages; ++s) {
            const int cout = round_channels(a.stage_base_out[s] * a.width_choices[c.width_idx[1 + s]]);
            for (int j = 0; j < a.stage_max_depth[s]; ++j, ++slot) {
                if (j >= c.depth[s]) {
                    w.skip(j == 0 ? 4 : 3);
                    continue;
                }
                const int stride = j == 0 ? a.stage_stride[s] : 1;
                const int cmid = round_channels(cout * a.expand_choices[c.expand_idx[slot]]);
                int h1H = H, h1W = W;
                int h1 = w.conv(x, h1H, h1W, C, cmid, 1, 1, SUSHI_ACT_RELU);
                int h2H = h1H, h2W = h1W;
                int h2 = w.conv(h1, h2H, h2W, cmid, cmid, 3, stride, SUSHI_ACT_RELU);
                w.bufs.put(h1);
                int sc = x;
                if (j == 0) {
                    // the projection is layer li+1 (after conv3) in blob order; emit it first so
                    // that conv3 can add it, then restore the order of the layer cursor
                    int save = w.li;
                    w.li = save + 1;
                    int pH = H, pW = W;
                    sc = w.conv(x, pH, pW, C, cout, 1, stride, SUSHI_ACT_NONE);
                    w.li = save;
                }
                int oH = h2H, oW = h2W;
                int o = w.conv(h2, oH, oW, cmid, cout, 1, 1, SUSHI_ACT_RELU, sc);
                if (j == 0) w.li += 1;
                w.bufs.put(h2);
                if (sc != x) w.bufs.put(sc);
                w.bufs.put(x);
                x = o, C = cout, H = oH, W = oW;
            }
        }
        w.gap(x, H, W, C, 0);
        w.fc(0, C, a.n_classes, SUSHI_ACT_NONE, BUF_LOGITS, false, true);
    } else {
        const int c0 = a.stem_out;
        int y = w.conv(x, H, W, C, c0, 3, 2, SUSHI_ACT_HSWISH);
        x = y, C = c0;
        int h = w.conv(x, H, W, C, c0, 3, 1, SUSHI_ACT_RELU);
        y = w.conv(h, H, W, c0, c0, 1, 1, SUSHI_ACT_NONE, x);
        w.bufs.put(h), w.bufs.put(x), x = y;
        int slot = 0;
        for (int s = 0; s < a.n_stages; ++s) {
            const int cout = a.stage_base_out[s];
            const int act = a.stage_act[s];
            for (int j = 0; j < a.stage_max_depth[s]; ++j, ++slot) {
                const int nl = a.stage_se[s] ? 5 : 3;
                if (j >= c.depth[s]) {
                    w.skip(nl);
                    continue;
                }
                const int stride = j == 0 ? a.stage_stride[s] : 1;
                const int cmid = round_channels(C * a.expand_choices[c.expand_idx[slot]]);
                const int k = a.kernel_choices[c.kernel_idx[slot]];
                int eH = H, eW = W;
                int e = w.conv(x, eH, eW, C, cmid, 1, 1, act);
                int dH = eH, dW = eW;
                int d = w.conv(e, dH, dW, cmid, cmid, k, stride, act);
                w.bufs.put(e);
                if (a.stage_se[s]) {
                    const int red = round_channels(cmid / 4.0);
                    w.gap(d, dH, dW, cmid, 0);
                    w.fc(0, cmid, red, SUSHI_ACT_RELU, 1, true, false);
                    w.fc(1, red, cmid, SUSHI_ACT_NONE, 2, true, true, true);
                    // The gated map goes to a buffer of its own (the expanded map's, free again): workgroups that
                    // still average d never see gated values, so pooling, both FC layers and the gating can run as
                    // one op without a barrier between them.
                    Op g;
                    g.kind = OP_GATE;
                    g.B = B, g.H = dH, g.W = dW, g.C = cmid, g.K = cmid, g.P = dH, g.Q = dW;
                    g.in_buf = d, g.out_buf = w.bufs.get(), g.gate_buf = 2;
                    plan.ops.push_back(g);
                    w.bufs.put(d);
                    d = g.out_buf;
                }
                const bool skip = stride == 1 && C == cout;
                int oH = dH, oW = dW;
                int o = w.conv(d, oH, oW, cmid, cout, 1, 1, SUSHI_ACT_NONE, skip ? x : BUF_NONE);
                w.bufs.put(d), w.bufs.put(x);
                x = o, C = cout, H = oH, W = oW;
            }
        }
        y = w.conv(x, H, W, C, a.head_mid, 1, 1, SUSHI_ACT_HSWISH);
        w.bufs.put(x), x = y, C = a.head_mid;
        w.gap(x, H, W, C, 0);
        w.fc(0, C, a.head_feat, SUSHI_ACT_HSWISH, 1, true, false);
        w.fc(1, a.head_feat, a.n_classes, SUSHI_ACT_NONE, BUF_LOGITS, false, true);
    }
    for (const Op &op : plan.ops)
        if ((op.kind == OP_CONV || op.kind == OP_DW || op.kind == OP_MAXPOOL || op.kind == OP_GATE) && op.out_buf < 0) {
            err = "internal: out of activation buffers";
            return SUSHI_EINVAL;
        }
    return SUSHI_OK;
}

int subnet_dims(const SuperNet &sn, const sushi_subnet_cfg &cfg, std::vector<sushi_layer_dims> &dims,
                std::string &err) {
    Plan p;
    int rc = plan_subnet(sn, cfg, 1, p, err);
    if (rc) return rc;
    dims = p.dims;
    return SUSHI_OK;
}

}  // namespace sushi
