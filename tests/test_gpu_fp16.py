"""GPU parity of the half-precision actor (Sec. 3.2 fp16 policies) against the CPU oracle.

The oracle rounds each operator's exact result to binary16 once; the GPU accumulates in fp32 first.
Bars, per layer, with the oracle fed the GPU's own previous layer (so every layer is checked in
isolation):
  * affine layers: the GPU value is a binary16 value and lies within half a binary16 spacing plus the
    fp32 summation bound (K + 2) 2^-24 sum|x w| (plus one fp32 rounding of the result) of the exact
    result; at least 99 % of the values are identical to the oracle's;
  * a layer followed by LayerNorm + tanh hands on only the normalised tensor, so the GPU's affine result
    (which may differ from the oracle's by a rounding step in a few places) is not seen: the normalised
    values must be within 2e-3 (four binary16 spacings just below 1) and at least 97 % identical;
  * the tanh head (transcendental in fp32): at most one binary16 step from the oracle's value, at least
    98 % identical;
  * argmax: identical wherever the GPU's own logits have a unique maximum.
End to end (oracle alone vs GPU): tanh / linear actions within 5e-3 absolute on these networks."""
import numpy as np
import pytest
import torch

import gpu_util as U
from oracle import policy as O
from paper_1910_01055_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def aq():
    from paper_1910_01055_amd import binding
    binding.load()
    return binding


def _say(msg):
    print(f"[fp16] {msg}", flush=True)


def _ordered(a):
    """binary16 values -> integers in value order (one step = one unit)"""
    b = np.asarray(a, np.float32).astype(np.float16).view(np.int16).astype(np.int32)
    return np.where(b < 0, -(b & 0x7FFF), b)


def _spacing(v):
    e = np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -14)))
    return np.exp2(e - 10)


def _nets():
    fc, conv = synth.fc, synth.conv
    return {
        "cfg1": synth.net_config("cfg1"),
        "cfg2": synth.net_config("cfg2"),
        "cfg5": synth.net_config("cfg5"),
        "odd_ln": synth.small_net([fc(67, 200, "ln_tanh"), fc(200, 72, "relu"), fc(72, 21, "none")], head="tanh"),
        "ln_odd70": synth.small_net([fc(20, 70, "ln_tanh"), fc(70, 5, "none")], head="tanh"),
        "ln_wide": synth.small_net([fc(16, 1100, "ln_tanh"), fc(1100, 4, "none")], head="linear"),
        "wide_last": synth.small_net([fc(40, 64, "relu"), fc(64, 104, "none")], head="tanh"),
        "argmax_mlp": synth.small_net([fc(33, 64, "relu"), fc(64, 18, "none")], head="argmax"),
        "u8_mlp": synth.small_net([fc(48, 64, "relu"), fc(64, 5, "none")], head="linear", in_type="u8"),
        "long_k": synth.small_net([fc(20, 700, "relu"), fc(700, 10, "none")], head="tanh"),
        "conv_small": synth.small_net([conv(12, 12, 4, 16, 4, 4, 2, "relu"), conv(5, 5, 16, 32, 3, 3, 1, "relu"),
                                       fc(288, 48, "relu"), fc(48, 5, "none")], head="argmax", in_type="u8",
                                      init="he_normal"),
        "conv_odd": synth.small_net([conv(9, 10, 3, 5, 3, 2, 2, "relu"), fc(100, 24, "none"), fc(24, 7, "none")],
                                    head="tanh", in_type="u8", init="he_normal"),
    }


def _run_gpu(aq, net, params, obs):
    batch = obs.shape[0]
    P = aq.Policy(net)
    w, b, g, be = U.upload_params(params)
    P.convert_params_fp16(w, b, g, be)
    assert P.policy_status() == aq.OK
    rf = U.layer_rows_feats(net, batch)
    taps = [torch.zeros(r * n, dtype=torch.float16, device=U.DEV) for r, n in rf]
    A = synth.action_dim(net)
    if net["head"] == "argmax":
        actions = torch.full((batch,), -1, dtype=torch.int32, device=U.DEV)
    else:
        actions = torch.full((batch, A), float("nan"), dtype=torch.float32, device=U.DEV)
    P.policy_forward_fp16(U.to_dev(obs), actions, taps)
    torch.cuda.synchronize()
    a2 = actions.clone()
    P.policy_forward_fp16(U.to_dev(obs), a2, None)  # without taps: same actions
    torch.cuda.synchronize()
    assert torch.equal(a2, actions)
    P.close()
    return actions.cpu().numpy(), [t.cpu().numpy().astype(np.float32) for t in taps]


def _check(net, params, obs, actions, outs, end_to_end=True):
    pol = O.OraclePolicy(net)
    nl = len(net["layers"])
    r16 = O.c_round_fp16
    x = r16(obs)
    for i, l in enumerate(net["layers"]):
        t = pol.forward_fp16(params, start_layer=i, start_x=x.reshape(obs.shape[0], -1),
                             stop_layer=i + 1)
        pre, ref = t["pre"][i].reshape(-1), t["out"][i].reshape(-1)
        g = outs[i].reshape(-1)
        assert g.shape == ref.shape
        ln = i < nl - 1 and l["act"] == "ln_tanh"
        same = np.mean(g == ref)
        if ln:
            assert np.abs(g - ref).max() <= 2e-3, f"layer {i}"
            assert same >= 0.97, f"layer {i}: {same}"
        else:
            # |x| |w| sums bound the fp32 accumulation error
            p_abs = [{"w": np.abs(r16(p["w"])), "b": np.abs(r16(p["b"]))} for p in params]
            ta = pol.forward_fp16(p_abs, start_layer=i, start_x=np.abs(x).reshape(obs.shape[0], -1),
                                  stop_layer=i + 1)
            S = ta["pre"][i].reshape(-1)
            K = int(np.prod(params[i]["w"].shape[1:]))
            post = np.maximum(pre, 0.0) if (i < nl - 1 and l["act"] == "relu") else pre
            bound = 0.5 * _spacing(np.maximum(np.abs(g), np.abs(ref))) * (1 + 1e-6) + (K + 2) * 2.0 ** -24 * S + \
                2.0 ** -23 * np.abs(pre)
            assert (np.abs(g.astype(np.float64) - post) <= bound).all(), f"layer {i}"
            assert same >= 0.99, f"layer {i}: {same}"
        x = outs[i]
    y = outs[-1].reshape(obs.shape[0], -1)
    head = pol.forward_fp16(params, start_layer=nl, start_x=y)["actions"]
    if net["head"] == "argmax":
        top = np.sort(y, axis=1)
        clear = top[:, -1] > top[:, -2]
        assert np.array_equal(actions[clear], head[clear])
        assert np.array_equal(actions, head)  # ties: both take the lowest index
    else:
        assert np.abs(_ordered(actions) - _ordered(head)).max() <= 1
        assert np.mean(actions == head) >= 0.98
    if not end_to_end:
        return
    # end to end against the oracle alone (a criterion for the named configurations: layer-by-layer
    # rounding differences compound, and networks with saturating activations amplify them)
    full = pol.forward_fp16(params, obs)["actions"]
    if net["head"] == "argmax":
        assert np.mean(actions == full) >= 0.97
    else:
        assert np.abs(actions - full).max() <= 5e-3


@pytest.mark.parametrize("name", list(_nets().keys()))
@pytest.mark.parametrize("batch", [1, 77, 200])
def test_fp16_actor_every_layer(aq, name, batch):
    _say(f"fp16_actor_every_layer {name} batch={batch}")
    net = _nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    actions, outs = _run_gpu(aq, net, params, obs)
    _check(net, params, obs, actions, outs)


@pytest.mark.parametrize("name,batch", [("cfg5", 16384), ("cfg5", 4200), ("cfg2", 4096), ("cfg3", 65536),
                                        ("cfg4", 256), ("paper_fc2048", 16), ("paper_fc2048", 1)])
def test_fp16_actor_full_size(aq, name, batch):
    """The benchmark's shapes and tile configurations; the oracle checks a sample of the rows."""
    _say(f"fp16_actor_full_size {name} batch={batch}")
    net = synth.net_config(name)
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    actions, outs = _run_gpu(aq, net, params, obs)
    rng = np.random.default_rng(9)
    n_s = 6 if name == "cfg4" else 48
    rows = np.unique(np.concatenate([np.minimum([0, 31, 32, 127, 128, batch - 1], batch - 1),
                                     rng.integers(0, batch, n_s)]))
    _check(net, params, obs[rows], actions[rows], [o.reshape(batch, -1)[rows] for o in outs])


def _random_net(rng):
    fc = synth.fc
    n_layers = int(rng.integers(1, 5))
    widths = [int(rng.choice([1, 5, 17, 31, 32, 33, 64, 67, 100, 129, 200, 256, 300, 520]))]
    for _ in range(n_layers):
        widths.append(int(rng.choice([1, 3, 6, 18, 21, 32, 33, 64, 65, 96, 128, 200, 256, 288, 512, 1030])))
    layers = []
    for i in range(n_layers):
        last = i == n_layers - 1
        act = "none" if last else str(rng.choice(["relu", "relu", "none", "ln_tanh"]))
        if act == "ln_tanh" and widths[i + 1] < 32:  # (few features: one rounding step moves the statistics too far)
            act = "relu"
        layers.append(fc(widths[i], widths[i + 1], act))
    return synth.small_net(layers, head=str(rng.choice(["tanh", "linear", "argmax"])),
                           in_type=str(rng.choice(["f32", "f32", "u8"])))


@pytest.mark.parametrize("seed", list(range(24)))
def test_fp16_actor_random_mlp_shapes(aq, seed):
    rng = np.random.default_rng(9000 + seed)
    net = _random_net(rng)
    batch = int(rng.choice([1, 2, 31, 33, 64, 100, 257, 600]))
    desc = "-".join(str(l["in"]) for l in net["layers"]) + f"-{net['layers'][-1]['out']}"
    _say(f"fp16_actor_random_mlp_shapes seed={seed} {desc} acts={[l['act'] for l in net['layers']]} "
         f"head={net['head']} {net['in_type']} batch={batch}")
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    actions, outs = _run_gpu(aq, net, params, obs)
    _check(net, params, obs, actions, outs)


def test_fp16_actor_conv_policy(aq):
    _say("fp16_actor_conv_policy cfg4 batch=6")
    net = synth.net_config("cfg4")
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, 6)
    actions, outs = _run_gpu(aq, net, params, obs)
    _check(net, params, obs, actions, outs)


def _stack_nets():
    fc, conv = synth.fc, synth.conv
    return {
        "cfg4": (synth.net_config("cfg4"), 3),
        "conv_small": (_nets()["conv_small"], 2),
        "three_convs_tanh": (synth.small_net([conv(28, 28, 8, 48, 4, 4, 4, "relu"), conv(7, 7, 48, 32, 2, 2, 2, "none"),
                                              conv(3, 3, 32, 16, 2, 2, 1, "relu"), fc(64, 20, "relu"), fc(20, 6, "none")],
                                             head="tanh", in_type="u8", init="he_normal"), 3),
        "conv_odd": (_nets()["conv_odd"], 0),
    }


@pytest.mark.parametrize("name", list(_stack_nets().keys()))
@pytest.mark.parametrize("batch", [1, 5, 70])
def test_fp16_actor_convolutions_in_one_launch(aq, name, batch):
    """The leading convolutions as one launch (maps in LDS): the last convolution's map, every later layer
    and the actions must equal the per-layer launches bit for bit (same arithmetic in the same order), and
    pass the oracle's checks."""
    _say(f"fp16_actor_convolutions_in_one_launch {name} batch={batch}")
    net, nc = _stack_nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    P = aq.Policy(net)
    w, b, g, be = U.upload_params(params)
    P.convert_params_fp16(w, b, g, be)
    assert P.policy_fp16_conv_stack_layers() == nc
    rf = U.layer_rows_feats(net, batch)
    A = synth.action_dim(net)

    def run(first_tap):
        taps = [torch.zeros(r * n, dtype=torch.float16, device=U.DEV) if i >= first_tap else None
                for i, (r, n) in enumerate(rf)]
        if net["head"] == "argmax":
            actions = torch.full((batch,), -1, dtype=torch.int32, device=U.DEV)
        else:
            actions = torch.full((batch, A), float("nan"), dtype=torch.float32, device=U.DEV)
        P.policy_forward_fp16(U.to_dev(obs), actions, taps)
        torch.cuda.synchronize()
        return actions, taps

    a_layers, t_layers = run(0)                      # a tap on the first map: one launch per layer
    a_stack, t_stack = run(max(nc - 1, 0))           # taps from the last convolution on: the single launch
    assert torch.equal(a_stack, a_layers)
    for i in range(max(nc - 1, 0), len(rf)):
        assert torch.equal(t_stack[i], t_layers[i]), f"layer {i}"
    P.policy_set_path(3)
    assert P.policy_fp16_conv_stack_layers() == 0
    a3, _ = run(max(nc - 1, 0))
    assert torch.equal(a3, a_layers)
    P.close()
    outs = [(t_stack[i] if i >= max(nc - 1, 0) else t_layers[i]).cpu().numpy().astype(np.float32) for i in range(len(rf))]
    _check(net, params, obs, a_stack.cpu().numpy(), outs)


@pytest.mark.parametrize("seed", list(range(10)))
def test_fp16_actor_random_convolution_stacks(aq, seed):
    """Random frame policies (kernel rows of 32 to 384 values, strides 1-4, ragged tiles): the single launch
    against the per-layer launches, bit for bit, and against the oracle's checks."""
    rng = np.random.default_rng(7100 + seed)
    net, nc = U.random_conv_stack(rng)
    if nc > 4:
        pytest.skip("more convolutions than the half-precision stack takes")
    batch = int(rng.choice([1, 4, 33]))
    _say(f"fp16_actor_random_convolution_stacks seed={seed} batch={batch}")
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    P = aq.Policy(net)
    w, b, g, be = U.upload_params(params)
    P.convert_params_fp16(w, b, g, be)
    assert P.policy_fp16_conv_stack_layers() == nc
    rf = U.layer_rows_feats(net, batch)
    A = synth.action_dim(net)

    def run(first_tap):
        taps = [torch.zeros(r * n, dtype=torch.float16, device=U.DEV) if i >= first_tap else None
                for i, (r, n) in enumerate(rf)]
        if net["head"] == "argmax":
            actions = torch.full((batch,), -1, dtype=torch.int32, device=U.DEV)
        else:
            actions = torch.full((batch, A), float("nan"), dtype=torch.float32, device=U.DEV)
        P.policy_forward_fp16(U.to_dev(obs), actions, taps)
        torch.cuda.synchronize()
        return actions, taps

    a_layers, t_layers = run(0)
    a_stack, t_stack = run(nc - 1)
    P.close()
    assert torch.equal(a_stack, a_layers)
    for i in range(nc - 1, len(rf)):
        assert torch.equal(t_stack[i], t_layers[i]), f"layer {i}"
    outs = [(t_stack[i] if i >= nc - 1 else t_layers[i]).cpu().numpy().astype(np.float32) for i in range(len(rf))]
    _check(net, params, obs, a_stack.cpu().numpy(), outs, end_to_end=False)  # every layer from the previous one


@pytest.mark.parametrize("name", ["cfg5", "cfg2", "u8_mlp"])
def test_fp16_actor_unaligned_buffers(aq, name):
    """Observation and action buffers that start off a 16-byte boundary take the element-wise input path
    and the separate head kernel; the results must not change."""
    _say(f"fp16_actor_unaligned_buffers {name}")
    net = _nets()[name]
    batch = 130
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    ref, _ = _run_gpu(aq, net, params, obs)
    P = aq.Policy(net)
    w, b, g, be = U.upload_params(params)
    P.convert_params_fp16(w, b, g, be)
    flat = torch.from_numpy(np.ascontiguousarray(obs)).reshape(-1)
    pad = torch.zeros(flat.numel() + 8, dtype=flat.dtype, device=U.DEV)
    pad[1:1 + flat.numel()] = flat.to(U.DEV)
    d_obs = pad[1:1 + flat.numel()].view(obs.shape)
    A = synth.action_dim(net)
    abuf = torch.zeros(batch * A + 8, dtype=torch.float32, device=U.DEV)
    actions = abuf[1:1 + batch * A].view(batch, A)
    assert d_obs.data_ptr() % 16 != 0 and actions.data_ptr() % 16 != 0
    P.policy_forward_fp16(d_obs, actions, None)
    torch.cuda.synchronize()
    assert np.array_equal(actions.cpu().numpy(), ref)
    assert float(abuf[0]) == 0.0 and float(abuf[1 + batch * A]) == 0.0  # nothing written outside
    P.close()


@pytest.mark.parametrize("name", ["cfg2", "conv_small"])
def test_fp16_actor_graph_replays_match_eager(aq, name):
    """The benchmark replays conversion + forward from a HIP graph; every replay, with eager work of the
    program's own in between, must reproduce the eager actions bit for bit."""
    _say(f"fp16_actor_graph_replays {name}")
    net = _nets()[name]
    batch = 260
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    P = aq.Policy(net)
    w, b, g, be = U.upload_params(params)
    A = synth.action_dim(net)
    argmax = net["head"] == "argmax"
    shape, dt = ((batch,), torch.int32) if argmax else ((batch, A), torch.float32)
    d_obs = U.to_dev(obs)
    out = torch.zeros(shape, dtype=dt, device=U.DEV)

    def body():
        P.convert_params_fp16(w, b, g, be)
        P.policy_forward_fp16(d_obs, out, None)

    body()  # allocates the parameter storage and the activation buffers
    torch.cuda.synchronize()
    eager = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        body()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        body()
    for rep in range(3):
        out.zero_()
        scratch = torch.zeros(shape, dtype=dt, device=U.DEV)
        P.policy_forward_fp16(d_obs, scratch, None)
        torch.cuda.synchronize()
        gr.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep}"
        assert torch.equal(scratch, eager)
        assert P.policy_status() == aq.OK
    P.close()


def test_fp16_actor_errors_and_nonfinite(aq):
    _say("fp16_actor_errors")
    net = _nets()["argmax_mlp"]
    params = synth.make_params(net)
    P = aq.Policy(net)
    obs = U.to_dev(synth.make_obs(net, 4))
    actions = torch.zeros(4, dtype=torch.int32, device=U.DEV)
    with pytest.raises(aq.AqError):
        P.policy_forward_fp16(obs, actions, None)  # before the conversion
    params[0]["w"][0, 0] = 70000.0  # overflows binary16
    w, b, g, be = U.upload_params(params)
    P.convert_params_fp16(w, b, g, be)
    assert P.policy_status() == aq.ENONFINITE
    params[0]["w"][0, 0] = 65519.0  # rounds to the largest finite value
    w, b, g, be = U.upload_params(params)
    P.convert_params_fp16(w, b, g, be)
    assert P.policy_status() == aq.OK
    P.policy_forward_fp16(obs[:0], actions[:0], None)  # empty batch: no-op
    P.close()
