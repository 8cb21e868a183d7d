"""Seeded synthetic workloads shaped like the paper's policies and observations.

This module only *draws inputs* (network descriptions, fp32 parameters,
observations).  It holds none of the method's arithmetic: no quantization, no
forward pass.  It is the one module both the CPU oracle's tests and the HIP
path's tests/bench import, so both sides see identical arrays.

The shapes stand in for the paper's workloads (Sec. 4: D4PG actors on
continuous-control tasks with fully connected policies, DQN policies, a
three-layer CNN for Atari frames); no environment, dataset or trained weight
is reproduced, every array is drawn from numpy's PCG64 with a fixed seed.
"""
from __future__ import annotations

import copy
import math

import numpy as np


def _fc(k, n, act):
    return {"kind": "fc", "in": int(k), "out": int(n), "act": act}


def _conv(h, w, c, co, kh, kw, stride, act):
    return {"kind": "conv", "in_h": h, "in_w": w, "in_c": c, "out_c": co, "kh": kh, "kw": kw,
            "stride": stride, "act": act}


CONFIGS = {
    # tiny MLP, per-tensor asymmetric uint8 weights, calibrated on its own batch
    "cfg1": {"name": "cfg1", "in_type": "f32", "layers": [_fc(17, 256, "relu"), _fc(256, 256, "relu"),
                                                          _fc(256, 6, "none")],
             "head": "tanh", "wscheme": "tensor_asym_u8", "qdenom": 255, "ln_eps": 1e-5, "batch": 256,
             "init": "glorot_uniform", "obs_seed": 1001, "w_seed": 2001},
    # D4PG-style actor MLP (LayerNorm + tanh after the first layer)
    "cfg2": {"name": "cfg2", "in_type": "f32", "layers": [_fc(67, 256, "ln_tanh"), _fc(256, 256, "relu"),
                                                          _fc(256, 256, "relu"), _fc(256, 21, "none")],
             "head": "tanh", "wscheme": "channel_sym_s8", "qdenom": 255, "ln_eps": 1e-5, "batch": 4096,
             "init": "glorot_uniform", "obs_seed": 1002, "w_seed": 2101},
    # DQN-style conv policy on uint8 frames
    "cfg4": {"name": "cfg4", "in_type": "u8", "layers": [_conv(84, 84, 4, 32, 8, 8, 4, "relu"),
                                                         _conv(20, 20, 32, 64, 4, 4, 2, "relu"),
                                                         _conv(9, 9, 64, 64, 3, 3, 1, "relu"),
                                                         _fc(3136, 512, "relu"), _fc(512, 18, "none")],
             "head": "argmax", "wscheme": "channel_sym_s8", "qdenom": 255, "ln_eps": 1e-5, "batch": 256,
             "init": "he_normal", "obs_seed": 1004, "w_seed": 2401},
    # wide MLP, MFMA-bound
    "cfg5": {"name": "cfg5", "in_type": "f32", "layers": [_fc(256, 1024, "relu"), _fc(1024, 1024, "relu"),
                                                          _fc(1024, 1024, "relu"), _fc(1024, 64, "none")],
             "head": "tanh", "wscheme": "channel_sym_s8", "qdenom": 255, "ln_eps": 1e-5, "batch": 16384,
             "init": "glorot_uniform", "obs_seed": 1005, "w_seed": 2501},
    # the paper's own actor (Sec. 4.1: three hidden layers of 2048 units, plain fully connected) on a
    # 67-dimensional observation and 21-dimensional action; the paper runs it one observation at a time
    "paper_fc2048": {"name": "paper_fc2048", "in_type": "f32",
                     "layers": [_fc(67, 2048, "relu"), _fc(2048, 2048, "relu"), _fc(2048, 2048, "relu"),
                                _fc(2048, 21, "none")],
                     "head": "tanh", "wscheme": "channel_sym_s8", "qdenom": 255, "ln_eps": 1e-5, "batch": 16,
                     "init": "glorot_uniform", "obs_seed": 1006, "w_seed": 2601},
}
# batch sweep of cfg2's network
CONFIGS["cfg3"] = dict(copy.deepcopy(CONFIGS["cfg2"]), name="cfg3", batch=65536, obs_seed=1003)
CFG3_BATCHES = (1, 16, 256, 4096, 65536)
QUANT_TENSOR_SEED = 3003
QUANT_TENSOR_ELEMS = 4 * 1024 * 1024


def net_config(name: str) -> dict:
    return copy.deepcopy(CONFIGS[name])


def small_net(layers, head="tanh", wscheme="channel_sym_s8", in_type="f32", qdenom=255, init="glorot_uniform",
              name="custom") -> dict:
    """A network description for ad-hoc test shapes."""
    return {"name": name, "in_type": in_type, "layers": copy.deepcopy(layers), "head": head, "wscheme": wscheme,
            "qdenom": qdenom, "ln_eps": 1e-5, "batch": 0, "init": init, "obs_seed": 1, "w_seed": 2}


fc = _fc
conv = _conv


def layer_out_shape(layer) -> tuple:
    if layer["kind"] == "fc":
        return (layer["out"],)
    oh = (layer["in_h"] - layer["kh"]) // layer["stride"] + 1
    ow = (layer["in_w"] - layer["kw"]) // layer["stride"] + 1
    return (oh, ow, layer["out_c"])


def layer_weight_shape(layer) -> tuple:
    if layer["kind"] == "fc":
        return (layer["out"], layer["in"])
    return (layer["out_c"], layer["kh"], layer["kw"], layer["in_c"])


def obs_shape(net) -> tuple:
    l0 = net["layers"][0]
    return (l0["in"],) if l0["kind"] == "fc" else (l0["in_h"], l0["in_w"], l0["in_c"])


def action_dim(net) -> int:
    return int(np.prod(layer_out_shape(net["layers"][-1])))


def macs_per_sample(net) -> int:
    total = 0
    for l in net["layers"]:
        if l["kind"] == "fc":
            total += l["in"] * l["out"]
        else:
            oh, ow, co = layer_out_shape(l)
            total += oh * ow * co * l["kh"] * l["kw"] * l["in_c"]
    return total


def make_params(net, nonzero_bias=False, seed=None):
    """fp32 parameters per layer: dict(w, b, gamma, beta).  Benchmarks use zero
    biases and unit LayerNorm gain; parity runs can ask for seeded non-trivial
    biases, gains and offsets so that a dropped term cannot hide."""
    base = net["w_seed"] if seed is None else seed
    out = []
    for i, l in enumerate(net["layers"]):
        rng = np.random.Generator(np.random.PCG64(base + i))
        shape = layer_weight_shape(l)
        n_out = shape[0]
        fan_in = int(np.prod(shape[1:]))
        if net["init"] == "glorot_uniform":
            lim = math.sqrt(6.0 / (fan_in + n_out))
            w = rng.uniform(-lim, lim, size=shape)
        elif net["init"] == "he_normal":
            w = rng.normal(0.0, math.sqrt(2.0 / fan_in), size=shape)
        else:
            raise ValueError(net["init"])
        p = {"w": np.ascontiguousarray(w, dtype=np.float32), "b": np.zeros(n_out, np.float32)}
        if nonzero_bias:
            p["b"] = rng.uniform(-0.1, 0.1, size=n_out).astype(np.float32)
        if l["act"] == "ln_tanh":
            p["gamma"] = np.ones(n_out, np.float32)
            p["beta"] = np.zeros(n_out, np.float32)
            if nonzero_bias:
                p["gamma"] = rng.uniform(0.5, 1.5, size=n_out).astype(np.float32)
                p["beta"] = rng.uniform(-0.1, 0.1, size=n_out).astype(np.float32)
        out.append(p)
    return out


def make_obs(net, batch, seed=None):
    """Observations: N(0,1) fp32 vectors, or uniform uint8 frames (NHWC)."""
    rng = np.random.Generator(np.random.PCG64(net["obs_seed"] if seed is None else seed))
    shape = (int(batch),) + obs_shape(net)
    if net["in_type"] == "u8":
        return rng.integers(0, 256, size=shape, dtype=np.uint8)
    return rng.standard_normal(size=shape, dtype=np.float32)


def quant_tensor(n=QUANT_TENSOR_ELEMS, seed=QUANT_TENSOR_SEED, std=0.05):
    """The learner-to-actor weight tensor of the quantize-bandwidth test: N(0, std) fp32."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal(size=n, dtype=np.float32) * np.float32(std)).astype(np.float32)
