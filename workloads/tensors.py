"""Seeded synthetic weights and inputs.

`make_weights` fills a list of tensors whose shapes and kinds the caller
supplies (each side lists the SuperNet's tensors itself); tensor i is drawn
from its own stream derive(seed, i), so the values depend only on
(seed, position, shape, kind).  Recipe:

  CONV / FC   normal(0, sqrt(2 / fan_in)),  fan_in = C*R*S   (He initialisation)
  DWCONV      normal(0, sqrt(2 / (R*S)))
  SCALE       uniform(0.8, 1.2)
  SCALE_RES   uniform(0.25, 0.5)    last scale of a residual branch, keeps the skip stream O(1)
  SHIFT/BIAS  normal(0, 0.05)

With bf16=True the CONV/DWCONV/FC values (and the inputs) are rounded to the
nearest bf16-representable value (ties to even) and still returned as float32.
"""
import numpy as np

from . import rng

KIND_CONV = 0
KIND_DWCONV = 1
KIND_FC = 2
KIND_BIAS = 3
KIND_SCALE = 4
KIND_SHIFT = 5
KIND_SCALE_RES = 6


def round_to_bf16(a):
    """float32 array -> float32 array holding bf16-representable values (round to nearest even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).reshape(a.shape)


def make_weights(table, seed, bf16=False):
    """table: sequence of (shape, kind).  Returns a list of float32 arrays."""
    out = []
    for i, (shape, kind) in enumerate(table):
        n = int(np.prod(shape))
        s = rng.derive(seed, i)
        if kind in (KIND_CONV, KIND_FC):
            fan_in = int(np.prod(shape[1:]))
            v = rng.normal(s, n) * np.sqrt(2.0 / fan_in)
        elif kind == KIND_DWCONV:
            v = rng.normal(s, n) * np.sqrt(2.0 / (shape[-1] * shape[-2]))
        elif kind == KIND_SCALE:
            v = 0.8 + 0.4 * rng.uniform(s, 0, n)
        elif kind == KIND_SCALE_RES:
            v = 0.25 + 0.25 * rng.uniform(s, 0, n)
        elif kind in (KIND_SHIFT, KIND_BIAS):
            v = rng.normal(s, n) * 0.05
        else:
            raise ValueError("unknown tensor kind %r" % (kind,))
        v = v.astype(np.float32).reshape(shape)
        if bf16 and kind in (KIND_CONV, KIND_DWCONV, KIND_FC):
            v = round_to_bf16(v)
        out.append(v)
    return out


def flatten(tensors):
    """Concatenate tensors in order into one float32 blob."""
    return np.concatenate([np.ascontiguousarray(t, dtype=np.float32).ravel() for t in tensors])


def make_input(seed, t, batch, resolution, channels=3, bf16=False):
    """Query t's input, standard normal, layout [batch, H, W, channels] float32."""
    n = batch * resolution * resolution * channels
    x = rng.normal(rng.derive(seed, 1000003, t), n).astype(np.float32)
    x = x.reshape(batch, resolution, resolution, channels)
    return round_to_bf16(x) if bf16 else x
