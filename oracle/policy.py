"""ctypes access to the C oracle and the layer-by-layer policy that strings its
functions together.  TEST INFRASTRUCTURE ONLY (never imported by the HIP path).

The order of operations is the one the method states (Sec. 3.1-3.2 of the
paper: quantize the learner's fp32 policy, then actors run the 8-bit policy):
quantize weights -> per-layer integer constants -> quantize the observation ->
for every layer: integer accumulator, then requantize / LayerNorm+tanh, or for
the last layer dequantize and apply the action head.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        # ACTORQ_ORACLE_LIB: a build of an altered copy of the C source, set only by the test that checks
        # that the pins notice planted mistakes
        path = os.environ.get("ACTORQ_ORACLE_LIB") or _build.build(force=False)
        _LIB = C.CDLL(path)
        _LIB.orc_num_threads.restype = C.c_int
        _LIB.orc_set_num_threads.restype = C.c_int
        _LIB.orc_set_num_threads.argtypes = [C.c_int]
    return _LIB


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


_f32, _f64, _i32, _i16, _i8, _u8, _i64 = (C.c_float, C.c_double, C.c_int32, C.c_int16, C.c_int8, C.c_uint8,
                                           C.c_int64)


def _chk(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def c_qparams_asym(w, qdenom=255.0, qmax=255):
    """qdenom = 2^n - 1 (default reading) or 2^n (literal); qmax = 2^n - 1 is the largest code."""
    w = np.ascontiguousarray(w, np.float32).ravel()
    s, z = _f32(), _i32()
    _chk(lib().orc_qparams_asym_n(_p(w, _f32), _i64(w.size), _f32(qdenom), _i32(qmax), C.byref(s), C.byref(z)),
         "qparams_asym")
    return np.float32(s.value), int(z.value)


def c_quantize_asym(w, scale, zp, qmax=255):
    w = np.ascontiguousarray(w, np.float32)
    q = np.empty(w.shape, np.uint8)
    lib().orc_quantize_asym_n(_p(w, _f32), _i64(w.size), _f32(scale), _i32(zp), _i32(qmax), _p(q, _u8))
    return q


def weight_levels(bits, qdenom=255):
    """(denominator of delta, largest unsigned code, largest symmetric code) of n-bit weights; the
    8-bit denominator says which reading of Sec. 3.2 is in force (255: 2^n - 1, 256: the literal 2^n)."""
    qmax = (1 << bits) - 1
    return float(qmax + 1 if int(qdenom) == 256 else qmax), qmax, (1 << (bits - 1)) - 1


def c_dequantize_asym(q, scale, zp):
    q = np.ascontiguousarray(q, np.uint8)
    w = np.empty(q.shape, np.float32)
    lib().orc_dequantize_asym(_p(q, _u8), _i64(q.size), _f32(scale), _i32(zp), _p(w, _f32))
    return w


def c_quantize_sym_rows(w2d, qw=127):
    w2d = np.ascontiguousarray(w2d, np.float32)
    rows, cols = w2d.shape
    s = np.empty(rows, np.float32)
    q = np.empty((rows, cols), np.int8)
    _chk(lib().orc_quantize_sym_rows_n(_p(w2d, _f32), _i64(rows), _i64(cols), _i32(qw), _p(s, _f32), _p(q, _i8)),
         "quantize_sym_rows")
    return q, s


def c_dequantize_sym_rows(q, s):
    q = np.ascontiguousarray(q, np.int8)
    w = np.empty(q.shape, np.float32)
    lib().orc_dequantize_sym_rows(_p(q, _i8), _i64(q.shape[0]), _i64(q.shape[1]), _p(np.ascontiguousarray(s, np.float32), _f32),
                                  _p(w, _f32))
    return w


def c_layer_consts(s_in, s_w, s_out, bias):
    s_w = np.ascontiguousarray(s_w, np.float32)
    bias = np.ascontiguousarray(bias, np.float32)
    n = s_w.size
    m = np.empty(n, np.float32)
    bq, M0, r = np.empty(n, np.int32), np.empty(n, np.int32), np.empty(n, np.int32)
    _chk(lib().orc_layer_consts(_f32(s_in), _p(s_w, _f32), _f32(s_out), _p(bias, _f32), _i64(n), _p(m, _f32),
                                _p(bq, _i32), _p(M0, _i32), _p(r, _i32)), "layer_consts")
    return m, bq, M0, r


def c_fc_acc(a, z_a, w_codes, z_w, bias_q):
    a = np.ascontiguousarray(a, np.uint8)
    B, K = a.shape
    w16 = np.ascontiguousarray(w_codes, np.int16)
    N = w16.shape[0]
    acc = np.empty((B, N), np.int32)
    _chk(lib().orc_fc_acc(_p(a, _u8), _i64(B), _i64(K), _i32(z_a), _p(w16, _i16), _i64(N),
                          _p(np.ascontiguousarray(z_w, np.int32), _i32), _p(np.ascontiguousarray(bias_q, np.int32), _i32),
                          _p(acc, _i32)), "fc_acc")
    return acc


def c_conv_acc(a, z_a, w_codes, stride, z_w, bias_q):
    a = np.ascontiguousarray(a, np.uint8)
    B, H, W, Cc = a.shape
    w16 = np.ascontiguousarray(w_codes, np.int16)
    Co, kh, kw, _ = w16.shape
    OH, OW = (H - kh) // stride + 1, (W - kw) // stride + 1
    acc = np.empty((B, OH, OW, Co), np.int32)
    _chk(lib().orc_conv_acc(_p(a, _u8), _i64(B), _i64(H), _i64(W), _i64(Cc), _i32(z_a), _p(w16, _i16), _i64(Co),
                            _i64(kh), _i64(kw), _i64(stride), _p(np.ascontiguousarray(z_w, np.int32), _i32),
                            _p(np.ascontiguousarray(bias_q, np.int32), _i32), _p(acc, _i32)), "conv_acc")
    return acc


def c_requant(acc, M0, r, z_out, relu):
    acc = np.ascontiguousarray(acc, np.int32)
    N = acc.shape[-1]
    rows = acc.size // N
    out = np.empty(acc.shape, np.uint8)
    lib().orc_requant(_p(acc, _i32), _i64(rows), _i64(N), _p(np.ascontiguousarray(M0, np.int32), _i32),
                      _p(np.ascontiguousarray(r, np.int32), _i32), _i32(z_out), _i32(1 if relu else 0), _p(out, _u8))
    return out


def c_dequant_acc(acc, m):
    acc = np.ascontiguousarray(acc, np.int32)
    N = acc.shape[-1]
    y = np.empty(acc.shape, np.float32)
    lib().orc_dequant_acc(_p(acc, _i32), _i64(acc.size // N), _i64(N), _p(np.ascontiguousarray(m, np.float32), _f32),
                          _p(y, _f32))
    return y


def c_ln_tanh(acc, m, gamma, beta, eps, s_out, z_out):
    acc = np.ascontiguousarray(acc, np.int32)
    N = acc.shape[-1]
    t = np.empty(acc.shape, np.float32)
    codes = np.empty(acc.shape, np.uint8)
    lib().orc_ln_tanh(_p(acc, _i32), _i64(acc.size // N), _i64(N), _p(np.ascontiguousarray(m, np.float32), _f32),
                      _p(np.ascontiguousarray(gamma, np.float32), _f32), _p(np.ascontiguousarray(beta, np.float32), _f32),
                      _f64(eps), _f32(s_out), _i32(z_out), _p(t, _f32), _p(codes, _u8))
    return t, codes


def c_tanh_f32(y):
    y = np.ascontiguousarray(y, np.float32)
    t = np.empty(y.shape, np.float32)
    lib().orc_tanh_f32(_p(y, _f32), _i64(y.size), _p(t, _f32))
    return t


def c_argmax_rows(y):
    y = np.ascontiguousarray(y, np.float32)
    N = y.shape[-1]
    idx = np.empty(y.size // N, np.int32)
    lib().orc_argmax_rows(_p(y, _f32), _i64(y.size // N), _i64(N), _p(idx, _i32))
    return idx


def c_philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(c.ctypes.data_as(C.c_void_p), k.ctypes.data_as(C.c_void_p), out.ctypes.data_as(C.c_void_p))
    return out


def c_explore_gaussian(actions, sigma, seed, step):
    """actions fp32 [rows][A] -> a copy with the exploration noise added (Sec. 4.1)."""
    a = np.array(actions, dtype=np.float32, order="C", copy=True)
    rows, A = a.shape
    sg = np.ascontiguousarray(sigma, dtype=np.float32)
    assert sg.shape == (rows,)
    lib().orc_explore_gaussian(_p(a, _f32), _i64(rows), _i64(A), _p(sg, _f32), C.c_uint64(seed), C.c_uint64(step))
    return a


def c_explore_eps_greedy(idx, A, epsilon, seed, step):
    i = np.array(idx, dtype=np.int32, order="C", copy=True)
    lib().orc_explore_eps_greedy(_p(i, _i32), _i64(i.size), _i64(A), _f32(epsilon), C.c_uint64(seed), C.c_uint64(step))
    return i


def c_fc_f64(x, w, b):
    x = np.ascontiguousarray(x, np.float64)
    B, K = x.shape
    w = np.ascontiguousarray(w, np.float32)
    N = w.shape[0]
    y = np.empty((B, N), np.float64)
    lib().orc_fc_f64(_p(x, _f64), _i64(B), _i64(K), _p(w, _f32), _p(np.ascontiguousarray(b, np.float32), _f32), _i64(N),
                     _p(y, _f64))
    return y


def c_conv_f64(x, w, b, stride):
    x = np.ascontiguousarray(x, np.float64)
    B, H, W, Cc = x.shape
    w = np.ascontiguousarray(w, np.float32)
    Co, kh, kw, _ = w.shape
    OH, OW = (H - kh) // stride + 1, (W - kw) // stride + 1
    y = np.empty((B, OH, OW, Co), np.float64)
    lib().orc_conv_f64(_p(x, _f64), _i64(B), _i64(H), _i64(W), _i64(Cc), _p(w, _f32),
                       _p(np.ascontiguousarray(b, np.float32), _f32), _i64(Co), _i64(kh), _i64(kw), _i64(stride), _p(y, _f64))
    return y


def c_relu_f64(x):
    x = np.ascontiguousarray(x, np.float64).copy()
    lib().orc_relu_f64(_p(x, _f64), _i64(x.size))
    return x


def c_tanh_f64(x):
    x = np.ascontiguousarray(x, np.float64).copy()
    lib().orc_tanh_f64(_p(x, _f64), _i64(x.size))
    return x


def c_layernorm_f64(x, gamma, beta, eps):
    x = np.ascontiguousarray(x, np.float64).copy()
    N = x.shape[-1]
    lib().orc_layernorm_f64(_p(x, _f64), _i64(x.size // N), _i64(N), _p(np.ascontiguousarray(gamma, np.float32), _f32),
                            _p(np.ascontiguousarray(beta, np.float32), _f32), _f64(eps))
    return x


def c_round_fp16(x):
    """IEEE binary16 rounding (nearest, ties to even) of fp64 values; returned widened to fp32."""
    x = np.ascontiguousarray(x, np.float64)
    out = np.empty(x.shape, np.float32)
    lib().orc_round_fp16(_p(x, _f64), _i64(x.size), _p(out, _f32))
    return out


class OraclePolicy:
    """The whole path, one layer at a time, every intermediate kept.

    `net` is a plain description (dict) of the policy: layer kinds and shapes,
    activation after each layer ("relu", "none", "ln_tanh"), head ("tanh",
    "argmax", "linear"), weight scheme ("tensor_asym_u8" | "channel_sym_s8"),
    input type ("f32" | "u8") and the quantizer's denominator.
    """

    def __init__(self, net):
        self.net = net
        self.layers = net["layers"]
        self.q = None

    # -- full-precision policy (Sec. 3.1: the learner's network) ------------------------------
    def forward_fp32(self, params, obs):
        """Returns (actions, ranges): ranges[i] = (min, max) of the network input (i = 0) and
        of each hidden layer's output (after its activation), as fp32."""
        x = np.asarray(obs, np.float64)
        ranges = [(np.float32(x.min()), np.float32(x.max()))]
        nl = len(self.layers)
        for i, (l, p) in enumerate(zip(self.layers, params)):
            if l["kind"] == "fc":
                x = c_fc_f64(x.reshape(x.shape[0], -1), p["w"], p["b"])
            else:
                x = c_conv_f64(x, p["w"], p["b"], l["stride"])
            if i == nl - 1:
                break
            if l["act"] == "relu":
                x = c_relu_f64(x)
            elif l["act"] == "ln_tanh":
                x = c_tanh_f64(c_layernorm_f64(x, p["gamma"], p["beta"], self.net["ln_eps"]))
            ranges.append((np.float32(x.min()), np.float32(x.max())))
        y = x.reshape(x.shape[0], -1)
        if self.net["head"] == "tanh":
            out = c_tanh_f64(y).astype(np.float32)
        elif self.net["head"] == "argmax":
            out = c_argmax_rows(y.astype(np.float32))
        else:
            out = y.astype(np.float32)
        return out, ranges

    # -- half-precision actor (Sec. 3.2 fp16 policies; actors at q = 16) ------------------------
    def forward_fp16(self, params, obs=None, start_layer=0, start_x=None, stop_layer=None):
        """Every parameter, the observation and every operator's output is a binary16 value;
        operators compute exactly (fp64) and round once.  Runs layers start_layer.. on `obs`
        (start_layer = 0) or on the given binary16-valued input of that layer; with stop_layer, stops
        before that layer and applies no head.  Returns
        dict(pre=[...], out=[...], actions): pre[i] is layer i's exact (unrounded, fp64) affine
        result, out[i] the binary16 tensor the layer hands on (after its activation), as fp32."""
        nl = len(self.layers)
        r16 = c_round_fp16
        x = r16(obs) if start_x is None else np.asarray(start_x, np.float32)
        taps = {"x0": x if start_layer == 0 else None, "pre": [None] * nl, "out": [None] * nl}
        for i in range(start_layer, nl if stop_layer is None else stop_layer):
            l, p = self.layers[i], params[i]
            w16, b16 = r16(p["w"]), r16(p["b"])
            if l["kind"] == "fc":
                pre = c_fc_f64(x.reshape(x.shape[0], -1), w16, b16)
            else:
                pre = c_conv_f64(x.reshape(x.shape[0], l["in_h"], l["in_w"], l["in_c"]), w16, b16, l["stride"])
            taps["pre"][i] = pre
            y = r16(pre)
            if i < nl - 1:
                if l["act"] == "relu":
                    y = r16(c_relu_f64(y))
                elif l["act"] == "ln_tanh":
                    y = r16(c_layernorm_f64(y, r16(p["gamma"]), r16(p["beta"]), self.net["ln_eps"]))
                    y = r16(c_tanh_f64(y))
            taps["out"][i] = x = y
        if stop_layer is not None:
            return taps
        y = x.reshape(x.shape[0], -1)
        if self.net["head"] == "tanh":
            taps["actions"] = r16(c_tanh_f64(y))
        elif self.net["head"] == "argmax":
            taps["actions"] = c_argmax_rows(y)
        else:
            taps["actions"] = y
        return taps

    # -- quantizer block (Sec. 3.2) ---------------------------------------------------------
    def quantize_params(self, params, act_ranges):
        """act_ranges[i] = (lo, hi) for the input (i = 0) and each hidden output."""
        qd = float(self.net["qdenom"])
        # weights at n bits (activations stay at 8): Sec. 3.2's Q_n with n below 8, codes in 8-bit containers
        wd, wmax, wsym = weight_levels(int(self.net.get("wbits", 8)), self.net["qdenom"])
        nl = len(self.layers)
        assert len(act_ranges) == nl
        act_q = []
        for i, (lo, hi) in enumerate(act_ranges):
            if i == 0 and self.net["in_type"] == "u8":
                act_q.append((np.float32(1.0), 0))  # raw frame codes are consumed as they are
            else:
                act_q.append(c_qparams_asym(np.array([lo, hi], np.float32), qd))
        q = []
        for i, (l, p) in enumerate(zip(self.layers, params)):
            w = p["w"]
            n_out = w.shape[0]
            if self.net["wscheme"] == "tensor_asym_u8":
                s, z = c_qparams_asym(w, wd, wmax)
                codes = c_quantize_asym(w, s, z, wmax)
                s_w = np.full(n_out, s, np.float32)
                z_w = np.full(n_out, z, np.int32)
            else:
                c2, s_w = c_quantize_sym_rows(w.reshape(n_out, -1), wsym)
                codes = c2.reshape(w.shape)
                z_w = np.zeros(n_out, np.int32)
            s_in, z_in = act_q[i]
            requant = (i < nl - 1) and l["act"] != "ln_tanh"
            s_out = act_q[i + 1][0] if requant else np.float32(0.0)
            m, bias_q, M0, r = c_layer_consts(s_in, s_w, s_out, p["b"])
            q.append({"codes": codes, "s_w": s_w, "z_w": z_w, "s_in": s_in, "z_in": z_in, "m": m, "bias_q": bias_q,
                      "M0": M0, "rshift": r, "gamma": p.get("gamma"), "beta": p.get("beta"),
                      "s_out": act_q[i + 1][0] if i < nl - 1 else None,
                      "z_out": act_q[i + 1][1] if i < nl - 1 else None})
        self.q = q
        self.act_q = act_q
        return q

    # -- actor inference on the 8-bit policy (Sec. 3.1) ----------------------------------------
    def quantize_obs(self, obs):
        if self.net["in_type"] == "u8":
            return np.ascontiguousarray(obs, np.uint8)
        s0, z0 = self.act_q[0]
        return c_quantize_asym(np.ascontiguousarray(obs, np.float32), s0, z0)

    def forward_int8(self, obs=None, start_layer=0, start_codes=None):
        """Runs layers start_layer.. on `obs` (start_layer = 0) or on the given
        unsigned activation codes.  Returns dict(acc=[...], act=[...], ln_t=[...], y, actions);
        lists are indexed by layer, entries before start_layer are None."""
        nl = len(self.layers)
        a = self.quantize_obs(obs) if start_codes is None else np.ascontiguousarray(start_codes, np.uint8)
        taps = {"a0": a if start_layer == 0 else None, "acc": [None] * nl, "act": [None] * nl, "ln_t": [None] * nl}
        for i in range(start_layer, nl):
            l, q = self.layers[i], self.q[i]
            if l["kind"] == "fc":
                acc = c_fc_acc(a.reshape(a.shape[0], -1), q["z_in"], q["codes"], q["z_w"], q["bias_q"])
            else:
                acc = c_conv_acc(a.reshape(a.shape[0], l["in_h"], l["in_w"], l["in_c"]), q["z_in"], q["codes"],
                                 l["stride"], q["z_w"], q["bias_q"])
            taps["acc"][i] = acc
            if i == nl - 1:
                y = c_dequant_acc(acc.reshape(acc.shape[0], -1), q["m"])
                taps["y"] = y
                if self.net["head"] == "tanh":
                    taps["actions"] = c_tanh_f32(y)
                elif self.net["head"] == "argmax":
                    taps["actions"] = c_argmax_rows(y)
                else:
                    taps["actions"] = y
            elif l["act"] == "ln_tanh":
                t, codes = c_ln_tanh(acc, q["m"], q["gamma"], q["beta"], self.net["ln_eps"], q["s_out"], q["z_out"])
                taps["ln_t"][i] = t
                taps["act"][i] = a = codes
            else:
                taps["act"][i] = a = c_requant(acc, q["M0"], q["rshift"], q["z_out"], l["act"] == "relu")
        return taps
