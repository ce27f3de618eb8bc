// Host-side description of a weight-shared SuperNet and of the per-query SubNet plan.
//
// A SuperNet is a fixed list of weight-bearing layers at their largest size; a SubNet is the same
// list with every layer cut down to a prefix box (K leading filters, C leading input channels,
// centred r x r taps) or skipped (paper Section 2.1).  plan_subnet() walks the network for one
// SubNet and emits the device operations of the forward pass in execution order.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/sushi.h"

namespace sushi {

enum LayerType { L_CONV = 0, L_DW = 1, L_FC = 2 };

struct SuperLayer {
    std::string name;
    int type = L_CONV;
    int Kmax = 0, Cmax = 0, Rmax = 1;  // Cmax = 1 for depthwise
    bool res_scale = false;            // its scale tensor ends a residual branch
    // positions inside the canonical float32 blob (in floats)
    size_t blob_w = 0, blob_scale = 0, blob_shift = 0;  // FC: blob_scale unused, blob_shift = bias
    // packed device layout, filled by the packer
    int Kpad = 0, CG = 0;         // filters padded to 16, channel groups of 8
    size_t pk_w = 0;              // element offset of the packed weights
    size_t pk_scale = 0, pk_shift = 0;  // float offsets in the parameter buffer
    bool has_scale = true;
    // int8 mode: channel groups of 16 in the packed weights, offsets of the layer's parameter words
    // (mult[Kpad], rshift[Kpad], bias[Kpad]) and of its weight prefix sums ([Cmax/8][Kpad]), its eight scalars
    int CG16 = 0;
    size_t pk_q = 0, pk_wsum = 0;
    int32_t qscalars[8] = {};
};

struct SuperNet {
    sushi_arch arch{};
    std::vector<SuperLayer> layers;
    std::vector<sushi_tensor_desc> tensors;  // blob order
    size_t blob_floats = 0;
    int layer_index(const std::string &name) const;
};

// Activation buffer ids used by the plan.
enum BufId { BUF_INPUT = -2, BUF_LOGITS = -3, BUF_NONE = -1 };
constexpr int N_BIG_BUFS = 6;    // feature maps
constexpr int N_SMALL_BUFS = 4;  // per-image vectors (pooled features, SE gates)

enum OpKind { OP_CONV = 0, OP_DW = 1, OP_MAXPOOL = 2, OP_GAP = 3, OP_FC = 4, OP_GATE = 5 };

struct Op {
    int kind = OP_CONV;
    int layer = -1;                    // index into SuperNet::layers (conv, dw, fc)
    int B = 0, H = 0, W = 0, C = 0;    // input: batch, height, width, active channels
    int P = 0, Q = 0, K = 0;           // output: height, width, active channels
    int r = 1, stride = 1, pad = 0;
    int act = SUSHI_ACT_NONE;
    int in_buf = BUF_NONE, out_buf = BUF_NONE, res_buf = BUF_NONE, gate_buf = BUF_NONE;
    bool in_small = false, out_small = false;  // which buffer family the ids refer to
    bool out_f32 = false;              // float32 output even in bf16 mode (per-image vectors: pooled features,
                                       // squeeze-excite and head vectors, gates; logits)
    bool hsigmoid = false;             // FC epilogue: min(max(x+3,0),6)/6 instead of act
};

struct Plan {
    std::vector<Op> ops;
    std::vector<sushi_layer_dims> dims;  // per SuperNet layer: active slice
    size_t max_big_elems = 0, max_small_elems = 0;
};

int round_channels(double x);  // ch(x) of sushi.h

// Builds the layer and tensor tables.  Returns SUSHI_OK or SUSHI_EINVAL (message in err).
int build_supernet(const sushi_arch &arch, SuperNet &out, std::string &err);

// Checks cfg against arch and reports the active slice of every layer (K = 0 when skipped).
int subnet_dims(const SuperNet &sn, const sushi_subnet_cfg &cfg, std::vector<sushi_layer_dims> &dims,
                std::string &err);

// Emits the forward pass of SubNet cfg on a batch of B images.
int plan_subnet(const SuperNet &sn, const sushi_subnet_cfg &cfg, int B, Plan &plan, std::string &err);

}  // namespace sushi
