"""Seeded int8 model data for the quantised path (paper Section 5.1, footnote on number formats: weights, input
activations and zero points int8, scales int32; Section 4.2.2: the zero-point / scale buffer).

Turns the float32 tensors of `tensors.make_weights` into the INPUTS both sides of the int8 parity tests read:
int8 weights, and per weight-bearing layer the int32 words (multiplier, right shift, bias, zero points) that a
requantising layer is parameterised with.  This is input preparation only: how a layer USES these words (the
integer arithmetic of the forward pass) is written separately by the oracle and by the library.

The paper gives the formats, not the quantiser; the recipe here (stated in the design doc as a reading):

  weights       symmetric per output filter: s_w[k] = max|w[k]| / 127 over the SuperNet tensor (so a SubNet's
                slice is a slice of the same int8 tensor), w_q = clip(rint(w / s_w[k]), -127, 127)
  activations   one (scale, zero point) per tensor by role: network input (S_IN, 0); output of a ReLU layer
                (S_RELU, -128); output of a layer without activation (S_LIN, 0)
  conv layer    real y = scale[k] * s_x * s_w[k] * acc + shift[k]; in units of the output scale the factor
                M_k = scale[k] s_x s_w[k] / s_y is stored as an int32 multiplier m_k in [2^30, 2^31) and a right
                shift sh_k (M_k ~ m_k 2^-sh_k); bias_k = rint(shift[k] / (scale[k] s_x s_w[k])) joins the accumulator
  residual      M_res = s_res / s_y, stored the same way
  classifier    works on the exact int32 sums of the global pooling; base_k = s_x s_w[k] as float32 (its bit
                pattern in the multiplier word), bias_k = rint(b[k] / base_k)

Per layer the int32 words are laid out as mult[K], rshift[K], bias[K], then eight scalars
[z_x, z_y, m_res, sh_res, z_res, 0, 0, 0] (Q_SCALARS).
"""
import numpy as np

from .tensors import KIND_BIAS, KIND_CONV, KIND_FC, KIND_SCALE, KIND_SCALE_RES, KIND_SHIFT

S_IN = 4.0 / 127.0      # inputs are N(0,1): +-4 sigma
S_RELU = 32.0 / 255.0   # post-ReLU tensors, zero point -128 (the residual stream of the widest SubNets reaches about 30)
S_LIN = 32.0 / 127.0    # tensors without activation, zero point 0
Z_RELU = -128
Q_SCALARS = 8


def fixed_point(m):
    """Positive real m -> (mult, shift) with mult in [2^30, 2^31) and m ~ mult * 2^-shift; shift in [1, 62]."""
    assert m > 0
    e = int(np.floor(np.log2(m)))
    shift = 30 - e
    mult = int(np.rint(m * 2.0 ** shift))
    if mult >= 1 << 31:
        mult >>= 1
        shift -= 1
    assert (1 << 30) <= mult < (1 << 31) and 1 <= shift <= 62, (m, mult, shift)
    return mult, shift


def quantize_input(x):
    """float32 [B,H,W,3] -> int8, scale S_IN, zero point 0."""
    return np.clip(np.rint(np.asarray(x, dtype=np.float64) / S_IN), -128, 127).astype(np.int8)


def make_int8_model(names_shapes_kinds, tensors, layer_roles):
    """names_shapes_kinds: the SuperNet's tensor table (name, shape, kind) in blob order; tensors: the float32
    arrays of tensors.make_weights for it; layer_roles: dict layer name -> (in_role, out_role, res_role) with
    roles 'in', 'relu', 'lin' (res_role None when the layer adds no residual).

    Returns a list, in blob order of the weight tensors, of dicts
        name, wq (int8, shape of the float tensor), mult, rshift, bias (int32 [K]), scalars (int32 [8])."""
    role = {"in": (S_IN, 0), "relu": (S_RELU, Z_RELU), "lin": (S_LIN, 0)}
    by_name = {n: t for (n, _, _), t in zip(names_shapes_kinds, tensors)}
    out = []
    for (name, shape, kind) in names_shapes_kinds:
        if kind not in (KIND_CONV, KIND_FC):
            continue
        assert name.endswith(".w")
        base = name[:-2]
        w = by_name[name].astype(np.float64)
        K = shape[0]
        flat = np.abs(w.reshape(K, -1)).max(axis=1)
        s_w = np.maximum(flat, 1e-12) / 127.0
        wq = np.clip(np.rint(w / s_w.reshape((K,) + (1,) * (w.ndim - 1))), -127, 127).astype(np.int8)
        in_role, out_role, res_role = layer_roles[base]
        s_x, z_x = role[in_role]
        mult = np.zeros(K, dtype=np.int64)
        rshift = np.zeros(K, dtype=np.int64)
        bias = np.zeros(K, dtype=np.int64)
        scalars = np.zeros(Q_SCALARS, dtype=np.int64)
        if kind == KIND_CONV:
            s_y, z_y = role[out_role]
            scale = by_name[base + ".scale"].astype(np.float64)
            shift = by_name[base + ".shift"].astype(np.float64)
            for k in range(K):
                g = scale[k] * s_x * s_w[k]
                mult[k], rshift[k] = fixed_point(g / s_y)
                bias[k] = int(np.rint(shift[k] / g))
            scalars[0], scalars[1] = z_x, z_y
            if res_role is not None:
                s_r, z_r = role[res_role]
                scalars[2], scalars[3] = fixed_point(s_r / s_y)
                scalars[4] = z_r
        else:
            b = by_name[base + ".b"].astype(np.float64)
            for k in range(K):
                base_k = np.float32(s_x * s_w[k])
                mult[k] = int(np.array([base_k], dtype=np.float32).view(np.int32)[0])
                bias[k] = int(np.rint(b[k] / np.float64(base_k)))
            scalars[0] = z_x
        assert np.abs(bias).max() < (1 << 31)
        out.append(dict(name=base, wq=wq, mult=mult.astype(np.int32), rshift=rshift.astype(np.int32),
                        bias=bias.astype(np.int32), scalars=scalars.astype(np.int32)))
    return out


def flatten_int8(model):
    """(int8 weight blob, int32 parameter blob) in the layer order of `model`."""
    wq = np.concatenate([m["wq"].ravel() for m in model])
    q = np.concatenate([np.concatenate([m["mult"], m["rshift"], m["bias"], m["scalars"]]) for m in model])
    return np.ascontiguousarray(wq, dtype=np.int8), np.ascontiguousarray(q, dtype=np.int32)


def layer_roles(arch):
    """layer name -> (input role, output role, residual role) for the families the int8 path covers (the Tiny
    conv chain and the bottleneck SuperNet): which of the three activation formats a layer reads, writes and adds."""
    from .arch import FAMILY_RESNET, FAMILY_TINY
    roles = {}
    if arch.family == FAMILY_TINY:
        for l in range(arch.n_stages):
            roles["conv%d" % l] = ("in" if l == 0 else "relu", "relu", None)
        roles["fc"] = ("relu", None, None)
    elif arch.family == FAMILY_RESNET:
        roles["stem0"] = ("in", "relu", None)
        roles["stem1"] = roles["stem2"] = ("relu", "relu", None)
        for s in range(arch.n_stages):
            for j in range(arch.stage_max_depth[s]):
                n = "s%db%d" % (s, j)
                roles[n + ".conv1"] = roles[n + ".conv2"] = ("relu", "relu", None)
                roles[n + ".conv3"] = ("relu", "relu", "lin" if j == 0 else "relu")
                if j == 0:
                    roles[n + ".proj"] = ("relu", "lin", None)
        roles["fc"] = ("relu", None, None)
    else:
        raise ValueError("the int8 path covers the Tiny and the bottleneck families")
    return roles
