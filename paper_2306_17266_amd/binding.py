"""ctypes binding of libsushi.so (include/sushi.h).  Argument marshalling only: every step of the
SubNet forward pass runs in the HIP library.  PyTorch supplies device memory and the stream."""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsushi.so")

MAX_STAGES, MAX_CHOICES, MAX_BLOCKS = 8, 4, 32
FP32, BF16 = 0, 1
STRICT_ACCURACY, STRICT_LATENCY = 0, 1
OPT_EXEC_MODE = 0
OPT_KERNEL_TIMING = 1
OPT_SPIN_LIMIT = 2
OPT_IDLE_US = 3
OPT_STREAM_WGS = 4
OPT_TEAM_WGS_PER_CU = 5
OPT_TEAMS_PER_XCD = 6
OPT_COLD_SWEEP_MIB = 7
OPT_PATCH_CONV_MIN_PIXELS = 8


class SushiError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("sushi error %d: %s" % (code, msg))
        self.code = code


class CArch(C.Structure):
    _fields_ = [("family", C.c_int32), ("n_classes", C.c_int32), ("in_channels", C.c_int32),
                ("n_stages", C.c_int32),
                ("stage_base_out", C.c_int32 * MAX_STAGES), ("stage_stride", C.c_int32 * MAX_STAGES),
                ("stage_max_depth", C.c_int32 * MAX_STAGES), ("stage_act", C.c_int32 * MAX_STAGES),
                ("stage_se", C.c_int32 * MAX_STAGES),
                ("n_depth_drop", C.c_int32), ("depth_drop_choices", C.c_int32 * MAX_CHOICES),
                ("n_width", C.c_int32), ("width_choices", C.c_double * MAX_CHOICES),
                ("n_expand", C.c_int32), ("expand_choices", C.c_double * MAX_CHOICES),
                ("n_kernel", C.c_int32), ("kernel_choices", C.c_int32 * MAX_CHOICES),
                ("n_res", C.c_int32), ("res_choices", C.c_int32 * MAX_CHOICES),
                ("stem_mid", C.c_int32), ("stem_out", C.c_int32),
                ("head_mid", C.c_int32), ("head_feat", C.c_int32)]


class CSubnetCfg(C.Structure):
    _fields_ = [("resolution", C.c_int32), ("depth", C.c_int32 * MAX_STAGES),
                ("width_idx", C.c_int32 * (MAX_STAGES + 1)),
                ("expand_idx", C.c_int32 * MAX_BLOCKS), ("kernel_idx", C.c_int32 * MAX_BLOCKS)]


class CTensorDesc(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("kind", C.c_int32), ("ndim", C.c_int32), ("shape", C.c_int32 * 4)]


class CLayerDims(C.Structure):
    _fields_ = [("K", C.c_int32), ("C", C.c_int32), ("r", C.c_int32)]


class CTeamOp(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "layer", "B", "H", "W", "C", "P", "Q", "K", "R", "stride",
                                          "ft", "pt", "wk", "n_units", "n_p", "lds_bytes", "res", "out_f32")]


class CPackedLayer(C.Structure):
    _fields_ = [("offset", C.c_uint64)] + [(n, C.c_int32) for n in ("depthwise", "K", "C", "R", "Kpad", "CG")]


class CSubgraphCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(CLayerDims))]


class CSchedDesc(C.Structure):
    _fields_ = [("n_subnets", C.c_int32), ("n_subgraphs", C.c_int32), ("vec_len", C.c_int32),
                ("subnet_vecs", C.POINTER(C.c_int32)), ("accuracy", C.POINTER(C.c_float)),
                ("subgraph_vecs", C.POINTER(C.c_int32)), ("table", C.POINTER(C.c_float)),
                ("Q", C.c_int32), ("policy", C.c_int32), ("initial_cache", C.c_int32)]


class CStats(C.Structure):
    _fields_ = [("queries", C.c_uint64), ("weight_bytes_total", C.c_uint64), ("weight_bytes_in_subgraph", C.c_uint64),
                ("last_weight_bytes", C.c_uint64), ("last_in_subgraph_bytes", C.c_uint64),
                ("cache_installs", C.c_uint64), ("cache_bytes_installed", C.c_uint64), ("cache_bytes", C.c_uint64),
                ("last_hit_ratio", C.c_double), ("sum_hit_ratio", C.c_double),
                ("plan_cache_hits", C.c_uint64), ("plan_cache_misses", C.c_uint64),
                ("weight_bytes_lds", C.c_uint64), ("last_lds_bytes", C.c_uint64), ("cache_bytes_lds", C.c_uint64),
                ("residency_changes", C.c_uint64), ("install_bytes_lds", C.c_uint64)]


class CKernelStats(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("launches", C.c_uint64), ("total_ms", C.c_double),
                ("bytes", C.c_double), ("flops", C.c_double)]


class CLaunchRecord(C.Structure):
    _fields_ = [("op_index", C.c_int32), ("kernel_class", C.c_int32), ("ms", C.c_float), ("pad", C.c_float),
                ("bytes", C.c_double), ("flops", C.c_double)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: build it with `python -m paper_2306_17266_amd.build` "
                           "(there is no fallback path)" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, ip = C.c_void_p, C.POINTER(C.c_int)
    L.sushi_describe_supernet.argtypes = [C.POINTER(CArch), C.POINTER(CTensorDesc), C.c_int, ip]
    L.sushi_subnet_layers.argtypes = [C.POINTER(CArch), C.POINTER(CSubnetCfg), C.POINTER(CLayerDims), C.c_int, ip]
    L.sushi_team_plan.argtypes = [C.POINTER(CArch), C.POINTER(CSubnetCfg), C.c_int, C.c_int, C.POINTER(CTeamOp), C.c_int, ip]
    L.sushi_pack_supernet.argtypes = [C.POINTER(CArch), vp, C.c_size_t, C.c_int, vp, C.c_size_t, C.POINTER(C.c_size_t),
                                      C.POINTER(CPackedLayer), C.c_int, ip]
    L.sushi_subgraph_overlap.argtypes = [C.POINTER(CLayerDims), C.POINTER(CLayerDims), C.c_int, C.c_int,
                                         C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_double)]
    L.sushi_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    L.sushi_destroy.argtypes = [vp]
    L.sushi_destroy.restype = None
    L.sushi_last_error.argtypes = [vp]
    L.sushi_last_error.restype = C.c_char_p
    L.sushi_load_supernet.argtypes = [vp, C.POINTER(CArch), vp, C.c_size_t, C.c_int]
    L.sushi_load_supernet_int8.argtypes = [vp, C.POINTER(CArch), vp, C.c_size_t, vp, C.c_size_t]
    L.sushi_set_subgraph_cache.argtypes = [vp, C.POINTER(CSubgraphCfg), C.c_size_t]
    L.sushi_infer.argtypes = [vp, C.POINTER(CSubnetCfg), vp, C.c_int, vp]
    L.sushi_infer_static.argtypes = [vp, C.POINTER(CSubnetCfg), vp, C.c_int, vp]
    L.sushi_sched_init.argtypes = [vp, C.POINTER(CSchedDesc)]
    L.sushi_sched_step.argtypes = [vp, C.c_float, C.c_float, ip, ip]
    L.sushi_sched_record.argtypes = [vp, C.POINTER(C.c_int32), ip]
    L.sushi_get_stats.argtypes = [vp, C.POINTER(CStats)]
    L.sushi_synchronize.argtypes = [vp]
    L.sushi_quiesce.argtypes = [vp]
    L.sushi_team_trace.argtypes = [vp, C.c_int, C.POINTER(C.c_uint64), C.c_int]
    L.sushi_set_option.argtypes = [vp, C.c_int, C.c_int64]
    L.sushi_get_kernel_stats.argtypes = [vp, C.POINTER(CKernelStats), C.c_int, ip]
    L.sushi_get_launch_records.argtypes = [vp, C.POINTER(CLaunchRecord), C.c_int, ip]
    _lib = L
    return L


def _fill(arr, values):
    for i, v in enumerate(values):
        arr[i] = v


def c_arch(a):
    """workloads.arch.Arch -> sushi_arch."""
    s = CArch()
    s.family, s.n_classes, s.in_channels, s.n_stages = a.family, a.n_classes, a.in_channels, a.n_stages
    _fill(s.stage_base_out, a.stage_base_out)
    _fill(s.stage_stride, a.stage_stride)
    _fill(s.stage_max_depth, a.stage_max_depth)
    _fill(s.stage_act, a.stage_act)
    _fill(s.stage_se, a.stage_se)
    s.n_depth_drop = len(a.depth_drop_choices)
    _fill(s.depth_drop_choices, a.depth_drop_choices)
    s.n_width = len(a.width_choices)
    _fill(s.width_choices, a.width_choices)
    s.n_expand = len(a.expand_choices)
    _fill(s.expand_choices, a.expand_choices)
    s.n_kernel = len(a.kernel_choices)
    _fill(s.kernel_choices, a.kernel_choices)
    s.n_res = len(a.res_choices)
    _fill(s.res_choices, a.res_choices)
    s.stem_mid, s.stem_out, s.head_mid, s.head_feat = a.stem_mid, a.stem_out, a.head_mid, a.head_feat
    return s


def c_cfg(cfg):
    """workloads.arch.SubnetCfg -> sushi_subnet_cfg."""
    s = CSubnetCfg()
    s.resolution = cfg.resolution
    _fill(s.depth, cfg.depth)
    _fill(s.width_idx, cfg.width_idx)
    _fill(s.expand_idx, cfg.expand_idx)
    _fill(s.kernel_idx, cfg.kernel_idx)
    return s


def _check(rc, ctx=None):
    if rc != 0:
        msg = lib().sushi_last_error(ctx) if ctx else b""
        raise SushiError(rc, (msg or b"").decode())


def sushi_describe_supernet(arch):
    """[(name, shape tuple, kind)] in weight-blob order."""
    a, n = c_arch(arch), C.c_int(0)
    _check(lib().sushi_describe_supernet(C.byref(a), None, 0, C.byref(n)))
    buf = (CTensorDesc * n.value)()
    _check(lib().sushi_describe_supernet(C.byref(a), buf, n.value, C.byref(n)))
    return [(d.name.decode(), tuple(d.shape[:d.ndim]), d.kind) for d in buf]


def sushi_subnet_layers(arch, cfg):
    """[(K, C, r)] per SuperNet layer for SubNet cfg."""
    a, s, n = c_arch(arch), c_cfg(cfg), C.c_int(0)
    buf = (CLayerDims * 256)()
    _check(lib().sushi_subnet_layers(C.byref(a), C.byref(s), buf, 256, C.byref(n)))
    return [(buf[i].K, buf[i].C, buf[i].r) for i in range(n.value)]


def sushi_pack_supernet(arch, weights, compute_dtype):
    """(packed image as a numpy array of uint16 (BF16) or float32 (FP32), [dict per weight-bearing layer]) - host only."""
    a = c_arch(arch)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    nb, nl = C.c_size_t(0), C.c_int(0)
    _check(lib().sushi_pack_supernet(C.byref(a), w.ctypes.data_as(C.c_void_p), w.nbytes, int(compute_dtype), None, 0,
                                     C.byref(nb), None, 0, C.byref(nl)))
    out = np.zeros(nb.value // (2 if compute_dtype == BF16 else 4), dtype=np.uint16 if compute_dtype == BF16 else np.float32)
    layers = (CPackedLayer * nl.value)()
    _check(lib().sushi_pack_supernet(C.byref(a), w.ctypes.data_as(C.c_void_p), w.nbytes, int(compute_dtype),
                                     out.ctypes.data_as(C.c_void_p), out.nbytes, C.byref(nb), layers, nl.value, C.byref(nl)))
    return out, [{f: getattr(layers[i], f) for f, _ in CPackedLayer._fields_} for i in range(nl.value)]


def sushi_team_plan(arch, cfg, batch, team_wgs):
    """[dict per op] of SubNet cfg as a team of team_wgs workgroups runs it (host only)."""
    a, s, n = c_arch(arch), c_cfg(cfg), C.c_int(0)
    buf = (CTeamOp * 512)()
    _check(lib().sushi_team_plan(C.byref(a), C.byref(s), int(batch), int(team_wgs), buf, 512, C.byref(n)))
    return [{f: getattr(buf[i], f) for f, _ in CTeamOp._fields_} for i in range(n.value)]


def marshal_box(box):
    """(K, C, r) triples -> sushi_layer_dims array."""
    return (CLayerDims * len(box))(*[CLayerDims(k, c, r) for (k, c, r) in box])


def sushi_subgraph_overlap(subnet_box, subgraph_box, bytes_per_weight=2):
    """(SubNet weight bytes, bytes inside the cached SubGraph, hit ratio of Appendix A.4).  The boxes may be
    lists of (K, C, r) or arrays from marshal_box."""
    a = subnet_box if isinstance(subnet_box, C.Array) else marshal_box(subnet_box)
    b = subgraph_box if isinstance(subgraph_box, C.Array) else marshal_box(subgraph_box)
    total, common, hit = C.c_uint64(0), C.c_uint64(0), C.c_double(0.0)
    _check(lib().sushi_subgraph_overlap(a, b, len(a), bytes_per_weight, C.byref(total), C.byref(common), C.byref(hit)))
    return total.value, common.value, hit.value


class Sushi:
    """One context (device + stream)."""

    def __init__(self, device=0, stream=None):
        if device < 0:
            stream = 0                      # host-only context: scheduler calls only
        elif stream is None:
            import torch
            stream = torch.cuda.current_stream(device).cuda_stream
        self._h = C.c_void_p()
        rc = lib().sushi_create(C.byref(self._h), device, C.c_void_p(stream))
        if rc != 0:
            raise SushiError(rc, (lib().sushi_last_error(None) or b"").decode())
        self.arch = None
        self.dtype = None
        self._cfg_cache = {}
        self._box_cache = {}
        self._j = C.c_int(0)

    def close(self):
        if self._h:
            lib().sushi_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def sushi_load_supernet(self, arch, blob, dtype):
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        a = c_arch(arch)
        _check(lib().sushi_load_supernet(self._h, C.byref(a), blob.ctypes.data_as(C.c_void_p), blob.nbytes, dtype),
               self._h)
        self.arch, self.dtype = arch, dtype
        self._cfg_cache = {}
        self._box_cache = {}

    def sushi_load_supernet_int8(self, arch, weights, qparams):
        """weights: int8 array (all weight tensors in blob order); qparams: int32 array (per weight tensor
        mult[K], rshift[K], bias[K] and eight scalars)."""
        w = np.ascontiguousarray(weights, dtype=np.int8)
        q = np.ascontiguousarray(qparams, dtype=np.int32)
        a = c_arch(arch)
        _check(lib().sushi_load_supernet_int8(self._h, C.byref(a), w.ctypes.data_as(C.c_void_p), w.size,
                                              q.ctypes.data_as(C.c_void_p), q.size), self._h)
        self.arch, self.dtype = arch, "int8"
        self._cfg_cache = {}
        self._box_cache = {}

    def sushi_set_subgraph_cache(self, box, budget_bytes):
        """box: list of (K, C, r) per layer, or None to empty the cache."""
        if not box:
            _check(lib().sushi_set_subgraph_cache(self._h, None, 0), self._h)
            return
        try:
            key = tuple(box)
            g = self._box_cache.get(key)
        except TypeError:  # layers given as lists: marshal every time
            key, g = None, None
        if g is None:
            arr = (CLayerDims * len(box))(*[CLayerDims(k, c, r) for (k, c, r) in box])
            g = CSubgraphCfg(len(box), arr)
            if key is not None and len(self._box_cache) < 1024:
                self._box_cache[key] = g
        _check(lib().sushi_set_subgraph_cache(self._h, C.byref(g), int(budget_bytes)), self._h)

    def sushi_infer(self, cfg, x, logits):
        """x: device tensor [B, res, res, C] (float32 or bfloat16); logits: float32 [B, classes]."""
        key = cfg.key()
        s = self._cfg_cache.get(key)
        if s is None:
            s = self._cfg_cache[key] = c_cfg(cfg)
        _check(lib().sushi_infer(self._h, C.byref(s), C.c_void_p(x.data_ptr()), x.shape[0],
                                 C.c_void_p(logits.data_ptr())), self._h)

    def sushi_infer_static(self, cfg, x, logits):
        """sushi_infer through the entry point that allocates nothing (activations in the library's static array)."""
        key = cfg.key()
        s = self._cfg_cache.get(key)
        if s is None:
            s = self._cfg_cache[key] = c_cfg(cfg)
        _check(lib().sushi_infer_static(self._h, C.byref(s), C.c_void_p(x.data_ptr()), x.shape[0],
                                        C.c_void_p(logits.data_ptr())), self._h)

    # Pre-marshalled arguments for callers that issue many queries: the same C calls, with the ctypes objects
    # built once instead of per call.
    def marshal_cfg(self, cfg):
        """A sushi_subnet_cfg for infer_marshalled."""
        return c_cfg(cfg)

    def marshal_subgraph(self, box):
        """A sushi_subgraph_cfg for set_subgraph_cache_marshalled (keeps its layer array alive)."""
        arr = (CLayerDims * len(box))(*[CLayerDims(k, c, r) for (k, c, r) in box])
        g = CSubgraphCfg(len(box), arr)
        g._keep = arr
        return g

    def marshal_vec(self, vec):
        """(int32 array, pointer) for sched_record_marshalled."""
        v = np.ascontiguousarray(vec, dtype=np.int32)
        return v, v.ctypes.data_as(C.POINTER(C.c_int32))

    def infer_marshalled(self, c_cfg_struct, x_ptr, batch, logits_ptr):
        rc = lib().sushi_infer(self._h, C.byref(c_cfg_struct), x_ptr, batch, logits_ptr)
        if rc != 0:
            _check(rc, self._h)

    def set_subgraph_cache_marshalled(self, g, budget_bytes):
        rc = lib().sushi_set_subgraph_cache(self._h, C.byref(g), budget_bytes)
        if rc != 0:
            _check(rc, self._h)

    def sched_record_marshalled(self, vec_pair):
        rc = lib().sushi_sched_record(self._h, vec_pair[1], C.byref(self._j))
        if rc != 0:
            _check(rc, self._h)
        return self._j.value

    def sushi_synchronize(self):
        _check(lib().sushi_synchronize(self._h), self._h)

    def sushi_quiesce(self):
        _check(lib().sushi_quiesce(self._h), self._h)

    def sushi_team_trace(self, enable):
        buf = (C.c_uint64 * (128 * 256))()
        _check(lib().sushi_team_trace(self._h, int(enable), buf, 128 * 256), self._h)
        return np.array(buf[:], dtype=np.uint64).reshape(128, 256)

    def sushi_sched_init(self, subnet_vecs, accuracy, subgraph_vecs, table, Q, policy, initial_cache=-1):
        sv = np.ascontiguousarray(subnet_vecs, dtype=np.int32)
        gv = np.ascontiguousarray(subgraph_vecs, dtype=np.int32).reshape(-1, sv.shape[1])
        acc = np.ascontiguousarray(accuracy, dtype=np.float32)
        tab = np.ascontiguousarray(table, dtype=np.float32)
        assert tab.shape == (sv.shape[0], gv.shape[0] + 1)
        d = CSchedDesc(sv.shape[0], gv.shape[0], sv.shape[1],
                       sv.ctypes.data_as(C.POINTER(C.c_int32)), acc.ctypes.data_as(C.POINTER(C.c_float)),
                       gv.ctypes.data_as(C.POINTER(C.c_int32)), tab.ctypes.data_as(C.POINTER(C.c_float)),
                       Q, policy, initial_cache)
        _check(lib().sushi_sched_init(self._h, C.byref(d)), self._h)

    def sushi_sched_step(self, acc_target, lat_target):
        i, j = C.c_int(0), C.c_int(0)
        _check(lib().sushi_sched_step(self._h, acc_target, lat_target, C.byref(i), C.byref(j)), self._h)
        return i.value, j.value

    def sushi_sched_record(self, vec):
        v = np.ascontiguousarray(vec, dtype=np.int32)
        j = C.c_int(0)
        _check(lib().sushi_sched_record(self._h, v.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(j)), self._h)
        return j.value

    def sushi_get_stats(self):
        s = CStats()
        _check(lib().sushi_get_stats(self._h, C.byref(s)), self._h)
        return {f: getattr(s, f) for f, _ in CStats._fields_}

    def sushi_set_option(self, option, value):
        _check(lib().sushi_set_option(self._h, option, value), self._h)

    def sushi_get_launch_records(self):
        n = C.c_int(0)
        _check(lib().sushi_get_launch_records(self._h, None, 0, C.byref(n)), self._h)
        buf = (CLaunchRecord * max(1, n.value))()
        _check(lib().sushi_get_launch_records(self._h, buf, n.value, C.byref(n)), self._h)
        return [(buf[i].op_index, buf[i].kernel_class, buf[i].ms, buf[i].bytes, buf[i].flops) for i in range(n.value)]

    def sushi_get_kernel_stats(self):
        buf, n = (CKernelStats * 16)(), C.c_int(0)
        _check(lib().sushi_get_kernel_stats(self._h, buf, 16, C.byref(n)), self._h)
        return [dict(name=buf[i].name.decode(), launches=buf[i].launches, total_ms=buf[i].total_ms,
                     bytes=buf[i].bytes, flops=buf[i].flops) for i in range(n.value)]
