"""Thin ctypes binding over libactorq.so (the C ABI in include/actorq.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch supplies device memory (tensors) and the current HIP stream, nothing else.
There is no fallback: if the library is not built, load() raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libactorq.so")
MAX_LAYERS = 8

OK, EINVAL, ESHAPE, ENONFINITE, ENOTQUANT, EHIP, ENOMEM, ERANGE, ETOOBIG = range(9)
STATIC_SCRATCH_BYTES = 16 << 20
KIND = {"fc": 0, "conv": 1}
ACT = {"none": 0, "relu": 1, "ln_tanh": 2}
HEAD = {"tanh": 0, "argmax": 1, "linear": 2}
WSCHEME = {"tensor_asym_u8": 0, "channel_sym_s8": 1}
INTYPE = {"f32": 0, "u8": 1}

EXPORTS = ["aq_policy_create", "aq_policy_destroy", "aq_policy_reserve", "aq_policy_set_path", "aq_policy_status",
           "aq_quantize_tensor", "aq_quantize_params", "aq_policy_export_layer", "aq_policy_export_act_qparams",
           "aq_policy_forward_int8", "aq_policy_forward_fp32", "aq_status_string",
           "aq_policy_blob_size", "aq_policy_export_blob", "aq_policy_import_blob", "aq_policy_explore", "aq_policy_step_int8",
           "aq_convert_params_fp16", "aq_policy_forward_fp16",
           "aq_policy_packed_blob_size", "aq_policy_export_packed_blob", "aq_policy_import_packed_blob",
           "aq_policy_conv_stack_layers", "aq_policy_fp16_conv_stack_layers", "aq_policy_fused_plan", "aq_policy_forward_int8_static",
           "aq_policy_set_params_fp32", "aq_calibrate_fp32", "aq_policy_forward_fp32_params", "aq_stream_reference",
           "aq_mfma_loop_reference", "aq_policy_subbyte_layers"]


class AqLayer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32), ("in_c", C.c_int32),
                ("out_c", C.c_int32), ("kh", C.c_int32), ("kw", C.c_int32), ("stride", C.c_int32),
                ("act", C.c_int32)]


class AqNet(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(AqLayer)), ("head", C.c_int32),
                ("wscheme", C.c_int32), ("in_type", C.c_int32), ("qdenom", C.c_int32), ("ln_eps", C.c_float),
                ("wbits", C.c_int32)]


class AqRange(C.Structure):
    _fields_ = [("lo", C.c_float), ("hi", C.c_float)]


class AqExplore(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("step", C.c_uint64), ("d_sigma", C.c_void_p), ("epsilon", C.c_float)]


class AqTaps(C.Structure):
    _fields_ = [("acc", C.POINTER(C.c_void_p)), ("act", C.POINTER(C.c_void_p)), ("ln_t", C.POINTER(C.c_void_p)),
                ("a0", C.c_void_p), ("y", C.c_void_p)]


class AqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = _lib.aq_status_string(status).decode() if _lib is not None else str(status)
        super().__init__(f"{where}: {msg} (aq_status {status})")


_lib = None


def load():
    """Loads libactorq.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1910_01055_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    pp = C.POINTER(C.c_void_p)
    lib.aq_status_string.restype = C.c_char_p
    lib.aq_status_string.argtypes = [C.c_int]
    lib.aq_policy_create.argtypes = [C.POINTER(AqNet), C.POINTER(vp)]
    lib.aq_policy_destroy.argtypes = [vp]
    lib.aq_policy_reserve.argtypes = [vp, i64]
    lib.aq_policy_set_path.argtypes = [vp, i32]
    lib.aq_policy_status.argtypes = [vp, vp]
    lib.aq_policy_conv_stack_layers.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.aq_policy_fp16_conv_stack_layers.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.aq_policy_subbyte_layers.argtypes = [vp, i64, C.POINTER(C.c_int32)]
    lib.aq_policy_fused_plan.argtypes = [vp, i64, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.aq_quantize_tensor.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp, vp]
    lib.aq_stream_reference.argtypes = [vp, i64, vp, vp]
    lib.aq_mfma_loop_reference.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    lib.aq_quantize_params.argtypes = [vp, pp, pp, pp, pp, C.POINTER(AqRange), vp]
    lib.aq_policy_export_layer.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.aq_policy_export_act_qparams.argtypes = [vp, vp, vp, vp]
    lib.aq_policy_forward_int8.argtypes = [vp, vp, i64, vp, C.POINTER(AqTaps), vp]
    lib.aq_policy_forward_int8_static.argtypes = [vp, vp, i64, vp, vp]
    lib.aq_policy_forward_fp32_params.argtypes = [vp, pp, pp, pp, pp, vp, i64, vp, vp, vp]
    lib.aq_policy_set_params_fp32.argtypes = [vp, pp, pp, pp, pp, vp]
    lib.aq_policy_forward_fp32.argtypes = [vp, vp, i64, vp, vp]
    lib.aq_calibrate_fp32.argtypes = [vp, vp, i64, C.POINTER(AqRange), vp]
    lib.aq_policy_blob_size.argtypes = [vp, C.POINTER(C.c_uint64)]
    lib.aq_policy_export_blob.argtypes = [vp, vp, C.c_uint64, vp]
    lib.aq_policy_import_blob.argtypes = [vp, vp, C.c_uint64, vp]
    lib.aq_policy_explore.argtypes = [vp, vp, i64, C.POINTER(AqExplore), vp]
    lib.aq_policy_step_int8.argtypes = [vp, vp, i64, vp, C.POINTER(AqExplore), C.POINTER(AqTaps), vp]
    for name in EXPORTS:
        if name != "aq_status_string":
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _ptr_array(tensors, n):
    arr = (C.c_void_p * n)()
    for i in range(n):
        t = tensors[i] if tensors is not None and i < len(tensors) else None
        arr[i] = 0 if t is None else t.data_ptr()
    return arr


def _check(status, where):
    if status != OK:
        raise AqError(status, where)


def make_net(net: dict):
    """dict description (see synth.CONFIGS) -> (AqNet, keep-alive layer array)."""
    n = len(net["layers"])
    arr = (AqLayer * n)()
    for i, l in enumerate(net["layers"]):
        if l["kind"] == "fc":
            arr[i] = AqLayer(KIND["fc"], 1, 1, l["in"], l["out"], 1, 1, 1, ACT[l["act"]])
        else:
            arr[i] = AqLayer(KIND["conv"], l["in_h"], l["in_w"], l["in_c"], l["out_c"], l["kh"], l["kw"],
                             l["stride"], ACT[l["act"]])
    cnet = AqNet(n, arr, HEAD[net["head"]], WSCHEME[net["wscheme"]], INTYPE[net["in_type"]], int(net["qdenom"]),
                 float(net["ln_eps"]), int(net.get("wbits", 0)))
    return cnet, arr


class Policy:
    """Owns one aq_policy handle.  Methods carry the C entry points' names."""

    def __init__(self, net: dict):
        lib = load()
        self.net = net
        self.n_layers = len(net["layers"])
        cnet, keep = make_net(net)
        h = C.c_void_p()
        _check(lib.aq_policy_create(C.byref(cnet), C.byref(h)), "aq_policy_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            load().aq_policy_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def policy_reserve(self, max_batch):
        _check(load().aq_policy_reserve(self._h, int(max_batch)), "aq_policy_reserve")

    def policy_set_path(self, path):
        _check(load().aq_policy_set_path(self._h, int(path)), "aq_policy_set_path")

    def policy_conv_stack_layers(self):
        n = C.c_int32(0)
        _check(load().aq_policy_conv_stack_layers(self._h, C.byref(n)), "aq_policy_conv_stack_layers")
        return int(n.value)

    def policy_fp16_conv_stack_layers(self):
        n = C.c_int32(0)
        _check(load().aq_policy_fp16_conv_stack_layers(self._h, C.byref(n)), "aq_policy_fp16_conv_stack_layers")
        return int(n.value)

    def policy_fused_plan(self, batch):
        """(rows per workgroup, feature tiles per wavefront, kernel: 0 general / 1 pipelined for wide layers /
        2 the kernel for small networks) of the fused launch at this batch; (0, 0, 0) = one launch per layer."""
        r, t, w = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        _check(load().aq_policy_fused_plan(self._h, int(batch), C.byref(r), C.byref(t), C.byref(w)), "aq_policy_fused_plan")
        return int(r.value), int(t.value), int(w.value)

    def policy_subbyte_layers(self, batch):
        """Layers of a forward pass at this batch that stream their weights as nibbles (policies of <= 4 bits)."""
        n = C.c_int32(0)
        _check(load().aq_policy_subbyte_layers(self._h, int(batch), C.byref(n)), "aq_policy_subbyte_layers")
        return int(n.value)

    def policy_status(self):
        return load().aq_policy_status(self._h, _stream())

    def policy_step_int8(self, obs, actions, seed, step, sigma=None, epsilon=0.0):
        """8-bit forward plus exploration in one call (fused into the forward kernel where possible)."""
        ex = AqExplore(int(seed), int(step), 0 if sigma is None else sigma.data_ptr(), float(epsilon))
        _check(load().aq_policy_step_int8(self._h, _ptr(obs), int(obs.shape[0]), _ptr(actions), C.byref(ex), None,
                                          _stream()), "aq_policy_step_int8")

    def policy_explore(self, actions, seed, step, sigma=None, epsilon=0.0):
        """In place on the actions of a forward: Gaussian noise with per-row sigma (device fp32 [batch]) for
        continuous heads, epsilon-greedy for argmax heads."""
        ex = AqExplore(int(seed), int(step), 0 if sigma is None else sigma.data_ptr(), float(epsilon))
        _check(load().aq_policy_explore(self._h, _ptr(actions), int(actions.shape[0]), C.byref(ex), _stream()),
               "aq_policy_explore")

    def policy_blob_size(self):
        n = C.c_uint64(0)
        _check(load().aq_policy_blob_size(self._h, C.byref(n)), "aq_policy_blob_size")
        return int(n.value)

    def policy_export_blob(self, blob):
        """blob: a uint8 device tensor of at least policy_blob_size() bytes."""
        _check(load().aq_policy_export_blob(self._h, _ptr(blob), blob.numel() * blob.element_size(), _stream()),
               "aq_policy_export_blob")

    def policy_import_blob(self, blob):
        _check(load().aq_policy_import_blob(self._h, _ptr(blob), blob.numel() * blob.element_size(), _stream()),
               "aq_policy_import_blob")

    def policy_packed_blob_size(self):
        n = C.c_uint64(0)
        _check(load().aq_policy_packed_blob_size(self._h, C.byref(n)), "aq_policy_packed_blob_size")
        return int(n.value)

    def policy_export_packed_blob(self, blob):
        _check(load().aq_policy_export_packed_blob(self._h, _ptr(blob), blob.numel() * blob.element_size(), _stream()),
               "aq_policy_export_packed_blob")

    def policy_import_packed_blob(self, blob):
        _check(load().aq_policy_import_packed_blob(self._h, _ptr(blob), blob.numel() * blob.element_size(), _stream()),
               "aq_policy_import_packed_blob")

    def quantize_params(self, w, b, gamma, beta, ranges):
        """w, b, gamma, beta: per-layer lists of device tensors (entries or lists may be None);
        ranges: n_layers (lo, hi) pairs."""
        n = self.n_layers
        r = (AqRange * n)()
        for i, (lo, hi) in enumerate(ranges):
            r[i] = AqRange(float(lo), float(hi))
        _check(load().aq_quantize_params(self._h, _ptr_array(w, n), _ptr_array(b, n), _ptr_array(gamma, n),
                                         _ptr_array(beta, n), r, _stream()), "aq_quantize_params")

    def policy_export_layer(self, layer, codes=None, w_scale=None, w_zp=None, bias_q=None, mult=None, rshift=None,
                            m=None):
        _check(load().aq_policy_export_layer(self._h, int(layer), _ptr(codes), _ptr(w_scale), _ptr(w_zp),
                                             _ptr(bias_q), _ptr(mult), _ptr(rshift), _ptr(m), _stream()),
               "aq_policy_export_layer")

    def policy_export_act_qparams(self, scale, zp):
        _check(load().aq_policy_export_act_qparams(self._h, _ptr(scale), _ptr(zp), _stream()),
               "aq_policy_export_act_qparams")

    def policy_forward_int8(self, obs, actions, taps=None):
        """taps: dict with optional keys acc/act/ln_t (per-layer lists of tensors or None), a0, y."""
        batch = int(obs.shape[0])
        ctaps = None
        if taps:
            n = self.n_layers
            keep = [_ptr_array(taps.get(k), n) for k in ("acc", "act", "ln_t")]
            ctaps = AqTaps(C.cast(keep[0], C.POINTER(C.c_void_p)), C.cast(keep[1], C.POINTER(C.c_void_p)),
                           C.cast(keep[2], C.POINTER(C.c_void_p)), _ptr(taps.get("a0")), _ptr(taps.get("y")))
        _check(load().aq_policy_forward_int8(self._h, _ptr(obs), batch, _ptr(actions),
                                             C.byref(ctaps) if ctaps is not None else None, _stream()),
               "aq_policy_forward_int8")

    def policy_forward_int8_static(self, obs, actions):
        """The 8-bit forward that allocates nothing (scratch in the library's static device buffer)."""
        _check(load().aq_policy_forward_int8_static(self._h, _ptr(obs), int(obs.shape[0]), _ptr(actions), _stream()),
               "aq_policy_forward_int8_static")

    def policy_forward_fp32_params(self, w, b, gamma, beta, obs, actions, ranges_out=None):
        n = self.n_layers
        _check(load().aq_policy_forward_fp32_params(self._h, _ptr_array(w, n), _ptr_array(b, n), _ptr_array(gamma, n),
                                                    _ptr_array(beta, n), _ptr(obs), int(obs.shape[0]), _ptr(actions),
                                                    _ptr(ranges_out), _stream()), "aq_policy_forward_fp32_params")

    def policy_set_params_fp32(self, w, b, gamma, beta):
        n = self.n_layers
        _check(load().aq_policy_set_params_fp32(self._h, _ptr_array(w, n), _ptr_array(b, n), _ptr_array(gamma, n),
                                                _ptr_array(beta, n), _stream()), "aq_policy_set_params_fp32")

    def policy_forward_fp32(self, obs, actions):
        _check(load().aq_policy_forward_fp32(self._h, _ptr(obs), int(obs.shape[0]), _ptr(actions), _stream()),
               "aq_policy_forward_fp32")

    def calibrate_fp32(self, obs):
        """(min, max) per activation tensor over this batch, as a list of n_layers pairs (waits for the stream)."""
        r = (AqRange * self.n_layers)()
        _check(load().aq_calibrate_fp32(self._h, _ptr(obs), int(obs.shape[0]), r, _stream()), "aq_calibrate_fp32")
        return [(float(x.lo), float(x.hi)) for x in r]

    def quantize_kept_params(self, ranges):
        """aq_quantize_params on the parameters kept by policy_set_params_fp32 (NULL parameter arrays)."""
        n = self.n_layers
        r = (AqRange * n)()
        for i, (lo, hi) in enumerate(ranges):
            r[i] = AqRange(float(lo), float(hi))
        _check(load().aq_quantize_params(self._h, None, None, None, None, r, _stream()), "aq_quantize_params")

    def convert_params_fp16(self, w, b, gamma, beta):
        n = self.n_layers
        _check(load().aq_convert_params_fp16(self._h, _ptr_array(w, n), _ptr_array(b, n), _ptr_array(gamma, n),
                                             _ptr_array(beta, n), _stream()), "aq_convert_params_fp16")

    def policy_forward_fp16(self, obs, actions, taps_out=None):
        taps = _ptr_array(taps_out, self.n_layers) if taps_out is not None else None
        _check(load().aq_policy_forward_fp16(self._h, _ptr(obs), int(obs.shape[0]), _ptr(actions), taps, _stream()),
               "aq_policy_forward_fp16")


def to_dev(a, device="cuda:0"):
    """numpy array (or None) -> contiguous device tensor (or None): device memory plumbing only."""
    import numpy as np
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(device)


def upload_params(params, device="cuda:0"):
    """Per-layer fp32 parameters (dicts with w, b, optional gamma, beta) -> four lists of device tensors."""
    return ([to_dev(p["w"], device) for p in params], [to_dev(p["b"], device) for p in params],
            [to_dev(p.get("gamma"), device) for p in params], [to_dev(p.get("beta"), device) for p in params])


def stream_reference(src, n, dst):
    _check(load().aq_stream_reference(_ptr(src), int(n), _ptr(dst), _stream()), "aq_stream_reference")


def mfma_loop_reference(weights, acts, ksteps, stream_weights, workgroups, acc):
    _check(load().aq_mfma_loop_reference(_ptr(weights), _ptr(acts), int(ksteps), int(bool(stream_weights)), int(workgroups),
                                         _ptr(acc), _stream()), "aq_mfma_loop_reference")


def quantize_tensor(w, rows, cols, wscheme, qdenom, codes, scale, zp, workspace):
    _check(load().aq_quantize_tensor(_ptr(w), int(rows), int(cols), WSCHEME[wscheme], int(qdenom), _ptr(codes),
                                     _ptr(scale), _ptr(zp), _ptr(workspace), _stream()), "aq_quantize_tensor")
