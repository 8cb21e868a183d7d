"""Helpers for the GPU parity tests: run the HIP library (through the C ABI) and the CPU oracle
on the same seeded inputs and compare stage by stage.

Bars: every integer stage bit-exact (weight codes, constants, quantized observation,
accumulators, requantized activations, argmax); floats (LayerNorm+tanh values, tanh actions)
within |g - o| <= 1e-4 |o| + 1e-6.  The one place where a float reduction decides an integer (the
8-bit code after LayerNorm+tanh) may differ by one step, only where the oracle's pre-rounding
value is within 1e-3 of a rounding tie; downstream of such a step the oracle is re-run from the
GPU's own codes and must again match bit for bit.
"""
import numpy as np
import torch

from oracle import policy as O
from paper_1910_01055_amd import synth

DEV = "cuda:0"
RTOL, ATOL = 1e-4, 1e-6


def close(g, o):
    g = np.asarray(g, np.float64)
    o = np.asarray(o, np.float64)
    return np.abs(g - o) <= RTOL * np.abs(o) + ATOL


def to_dev(a):
    from paper_1910_01055_amd import binding
    return binding.to_dev(a, DEV)


def upload_params(params):
    from paper_1910_01055_amd import binding
    return binding.upload_params(params, DEV)


def action_error_figures(a_q, a_f):
    """How far the 8-bit policy's actions are from the fp32 policy's on the same observations: largest and
    mean absolute difference, and the signal-to-quantization-noise ratio in dB."""
    a_q = np.asarray(a_q, np.float64)
    a_f = np.asarray(a_f, np.float64)
    d = a_q - a_f
    return {"max_abs": float(np.abs(d).max()), "mean_abs": float(np.abs(d).mean()),
            "sqnr_db": float(10.0 * np.log10((a_f ** 2).sum() / max((d ** 2).sum(), 1e-300)))}


def layer_rows_feats(net, batch):
    out = []
    for l in net["layers"]:
        shp = synth.layer_out_shape(l)
        out.append((batch * int(np.prod(shp[:-1])), shp[-1]))
    return out


def make_oracle(net, params, calib_obs):
    pol = O.OraclePolicy(net)
    _, ranges = pol.forward_fp32(params, calib_obs)
    pol.quantize_params(params, ranges)
    return pol, ranges


def gpu_quantize(aq, net, params, ranges):
    P = aq.Policy(net)
    d = upload_params(params)
    P.quantize_params(d[0], d[1], d[2], d[3], ranges)
    assert P.policy_status() == aq.OK
    return P, d


def check_quantized_params(aq, P, pol, net):
    """Exported weight codes and constants equal the oracle's, bit for bit."""
    nl = len(net["layers"])
    asym = net["wscheme"] == "tensor_asym_u8"
    s = torch.empty(nl, dtype=torch.float32, device=DEV)
    z = torch.empty(nl, dtype=torch.int32, device=DEV)
    P.policy_export_act_qparams(s, z)
    s, z = s.cpu().numpy(), z.cpu().numpy()
    for i, (so, zo) in enumerate(pol.act_q):
        assert s[i].view(np.uint32) == np.float32(so).view(np.uint32) and z[i] == zo, f"act qparams {i}"
    for l, q in enumerate(pol.q):
        n = q["codes"].shape[0]
        codes = torch.empty(q["codes"].shape, dtype=torch.uint8 if asym else torch.int8, device=DEV)
        fs = torch.empty(n, dtype=torch.float32, device=DEV)
        fm = torch.empty(n, dtype=torch.float32, device=DEV)
        iz, ib, iM, ir = (torch.empty(n, dtype=torch.int32, device=DEV) for _ in range(4))
        P.policy_export_layer(l, codes, fs, iz, ib, iM, ir, fm)
        assert np.array_equal(codes.cpu().numpy(), q["codes"]), f"layer {l} weight codes"
        assert np.array_equal(fs.cpu().numpy().view(np.uint32), q["s_w"].view(np.uint32)), f"layer {l} scales"
        assert np.array_equal(iz.cpu().numpy(), q["z_w"]), f"layer {l} zero-points"
        assert np.array_equal(ib.cpu().numpy(), q["bias_q"]), f"layer {l} bias_q"
        assert np.array_equal(iM.cpu().numpy(), q["M0"]), f"layer {l} multipliers"
        assert np.array_equal(ir.cpu().numpy(), q["rshift"]), f"layer {l} shifts"
        assert np.array_equal(fm.cpu().numpy().view(np.uint32), q["m"].view(np.uint32)), f"layer {l} m"


def gpu_forward(P, net, obs, taps=True, misalign=0):
    """misalign: place the observations this many elements past a fresh allocation's start, so that
    their address is not 16-byte aligned (the kernels' vector loads must then not be used)."""
    batch = obs.shape[0]
    d_obs = to_dev(obs)
    if misalign:
        flat = torch.empty(d_obs.numel() + misalign, dtype=d_obs.dtype, device=DEV)
        flat[misalign:].copy_(d_obs.reshape(-1))
        d_obs = flat[misalign:].reshape(d_obs.shape)
        assert d_obs.data_ptr() % 16 != 0 and d_obs.is_contiguous()
    nl = len(net["layers"])
    A = synth.action_dim(net)
    if net["head"] == "argmax":
        actions = torch.full((batch,), -7, dtype=torch.int32, device=DEV)
    else:
        actions = torch.full((batch, A), float("nan"), dtype=torch.float32, device=DEV)
    t = None
    if taps:
        rf = layer_rows_feats(net, batch)
        t = {"acc": [torch.zeros(r, n, dtype=torch.int32, device=DEV) for r, n in rf],
             "act": [torch.zeros(r, n, dtype=torch.uint8, device=DEV) if i < nl - 1 else None
                     for i, (r, n) in enumerate(rf)],
             "ln_t": [torch.zeros(r, n, dtype=torch.float32, device=DEV) if net["layers"][i]["act"] == "ln_tanh"
                      and i < nl - 1 else None for i, (r, n) in enumerate(rf)],
             "a0": torch.zeros(obs.reshape(batch, -1).shape, dtype=torch.uint8, device=DEV),
             "y": torch.zeros(batch, A, dtype=torch.float32, device=DEV)}
    P.policy_forward_int8(d_obs, actions, t)
    torch.cuda.synchronize()
    return actions.cpu().numpy(), t


def compare_forward(net, pol, obs, g_actions, t, rows=None):
    """rows: optional sample of batch rows the oracle is run on (rows are independent)."""
    nl = len(net["layers"])
    sel = np.arange(obs.shape[0]) if rows is None else np.asarray(rows)
    ref = pol.forward_int8(obs[sel])
    flips_total = 0

    def g(tensor, per_sample):
        a = tensor.cpu().numpy()
        a = a.reshape(obs.shape[0], per_sample, -1)[sel]
        return a.reshape(len(sel) * per_sample, -1)

    per = [int(np.prod(synth.layer_out_shape(l)[:-1])) for l in net["layers"]]
    assert np.array_equal(g(t["a0"], 1), ref["a0"].reshape(len(sel), -1)), "quantized observation"
    for l in range(nl):
        N = synth.layer_out_shape(net["layers"][l])[-1]
        assert np.array_equal(g(t["acc"][l], per[l]), ref["acc"][l].reshape(-1, N)), f"layer {l} accumulators"
        if l == nl - 1:
            break
        g_act = g(t["act"][l], per[l])
        o_act = ref["act"][l].reshape(-1, N)
        if net["layers"][l]["act"] == "ln_tanh":
            g_t = g(t["ln_t"][l], per[l])
            o_t = ref["ln_t"][l].reshape(-1, N)
            assert close(g_t, o_t).all(), f"layer {l} LayerNorm+tanh values"
            diff = g_act.astype(np.int64) - o_act
            flips = np.nonzero(diff)
            flips_total += len(flips[0])
            if len(flips[0]):
                assert np.abs(diff).max() <= 1
                s_out = pol.q[l]["s_out"]
                pre = o_t[flips].astype(np.float32) / np.float32(s_out)
                assert (np.abs(np.abs(pre - np.floor(pre)) - 0.5) <= 1e-3).all(), "flip away from a rounding tie"
                # downstream: the oracle continues from the GPU's own codes
                ref = dict(ref)
                shape = ref["act"][l].shape
                cont = pol.forward_int8(start_layer=l + 1, start_codes=g_act.reshape(shape))
                for k in ("acc", "act", "ln_t"):
                    ref[k] = [cont[k][i] if i > l else ref[k][i] for i in range(nl)]
                ref["y"], ref["actions"] = cont["y"], cont["actions"]
        else:
            assert np.array_equal(g_act, o_act), f"layer {l} requantized activations"
    gy = t["y"].cpu().numpy()[sel]
    assert np.array_equal(gy.view(np.uint32), ref["y"].view(np.uint32)), "dequantized last layer"
    ga = g_actions[sel]
    if net["head"] == "argmax":
        assert np.array_equal(ga, ref["actions"]), "argmax actions"
    else:
        assert close(ga, ref["actions"]).all(), "actions"
    return flips_total


def random_conv_stack(rng):
    """A random frame policy whose convolutions fit the single-launch kernel's shape rules (kernel rows of a
    multiple of 32 bytes, 16-byte aligned positions), found by rejection."""
    while True:
        nc = int(rng.integers(2, 4))
        c = int(rng.choice([4, 8, 16]))
        h, w = int(rng.integers(10, 41)), int(rng.integers(10, 41))
        layers, ok, tiles = [], True, 0
        for l in range(nc):
            kw, kh, st = int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 5))
            n = int(rng.choice([8, 16, 24, 32, 40, 48, 64, 72]))
            if (kw * c) % 32 or (st * c) % 16 or (w * c) % 16 or kh > h or kw > w:
                ok = False
                break
            layers.append(synth.conv(h, w, c, n, kh, kw, st, str(rng.choice(["relu", "relu", "none"]))))
            h, w, c = (h - kh) // st + 1, (w - kw) // st + 1, n
            tiles += (n + 31) // 32
        first = layers[0] if layers else None
        if not ok or tiles > 12 or h * w * c > 4000 or first["in_h"] * first["in_w"] * first["in_c"] > 32768 \
                or (first["in_h"] * first["in_w"] * first["in_c"]) % 16:
            continue
        hidden = int(rng.choice([20, 48]))
        layers += [synth.fc(h * w * c, hidden, "relu"), synth.fc(hidden, int(rng.integers(2, 19)), "none")]
        return synth.small_net(layers, head=str(rng.choice(["argmax", "tanh"])), in_type="u8", init="he_normal"), nc
