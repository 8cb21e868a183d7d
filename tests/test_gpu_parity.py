"""GPU parity tests: the HIP library, called through its C ABI, against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import policy as O
from paper_1910_01055_amd import synth

pytestmark = pytest.mark.gpu

import gpu_util as U  # noqa: E402


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ quantizer block on one tensor
@pytest.mark.parametrize("rows,cols", [(1, 4), (3, 8), (5, 260), (37, 132), (2048, 2048), (2, 4100), (1, 1 << 20)])
@pytest.mark.parametrize("scheme", ["tensor_asym_u8", "channel_sym_s8"])
def test_quantize_tensor(aq, rows, cols, scheme):
    _say(f"quantize_tensor rows={rows} cols={cols} {scheme}")
    w = synth.quant_tensor(rows * cols, seed=synth.QUANT_TENSOR_SEED + rows).reshape(rows, cols)
    if rows >= 3:
        w[1] = 0.0  # an all-zero channel
    d_w = U.to_dev(w)
    asym = scheme == "tensor_asym_u8"
    codes = torch.zeros(rows, cols, dtype=torch.uint8 if asym else torch.int8, device=U.DEV)
    ns = 1 if asym else rows
    scale = torch.zeros(ns, dtype=torch.float32, device=U.DEV)
    zp = torch.full((ns,), -1, dtype=torch.int32, device=U.DEV)
    ws = torch.ones(4096, dtype=torch.int32, device=U.DEV)
    ws[2] = 0  # the sticky non-finite flag
    aq.quantize_tensor(d_w, rows, cols, scheme, 255, codes, scale, zp, ws)
    torch.cuda.synchronize()
    if asym:
        s, z = O.c_qparams_asym(w)
        ref = O.c_quantize_asym(w, s, z)
        assert scale.cpu().numpy()[0].view(np.uint32) == np.float32(s).view(np.uint32) and int(zp[0]) == z
    else:
        ref, s = O.c_quantize_sym_rows(w)
        assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32)) and not zp.cpu().numpy().any()
    assert np.array_equal(codes.cpu().numpy(), ref)
    assert int(ws[2]) == 0


@pytest.mark.parametrize("qdenom", [3, 7, 15, 16, 31, 63, 64, 127])
@pytest.mark.parametrize("scheme", ["tensor_asym_u8", "channel_sym_s8"])
def test_quantize_tensor_below_8_bits(aq, qdenom, scheme):
    """Sec. 3.2's Q_n for n < 8: qdenom = 2^n - 1 or 2^n selects the precision; codes bit-exact."""
    _say(f"quantize_tensor_below_8_bits qdenom={qdenom} {scheme}")
    bits = int(np.ceil(np.log2(qdenom + 1))) if (qdenom & (qdenom + 1)) == 0 else int(np.log2(qdenom))
    qmax, qsym = 2 ** bits - 1, 2 ** (bits - 1) - 1
    for rows, cols in ((37, 132), (5, 4100), (300, 1024)):
        w = synth.quant_tensor(rows * cols, seed=synth.QUANT_TENSOR_SEED + qdenom).reshape(rows, cols)
        w[1] = 0.0
        asym = scheme == "tensor_asym_u8"
        codes = torch.zeros(rows, cols, dtype=torch.uint8 if asym else torch.int8, device=U.DEV)
        ns = 1 if asym else rows
        scale = torch.zeros(ns, dtype=torch.float32, device=U.DEV)
        zp = torch.full((ns,), -1, dtype=torch.int32, device=U.DEV)
        ws = torch.zeros(4096, dtype=torch.int32, device=U.DEV)
        aq.quantize_tensor(U.to_dev(w), rows, cols, scheme, qdenom, codes, scale, zp, ws)
        torch.cuda.synchronize()
        got = codes.cpu().numpy()
        if asym:
            s, z = O.c_qparams_asym(w, float(qdenom), qmax)
            ref = O.c_quantize_asym(w, s, z, qmax)
            assert scale.cpu().numpy()[0].view(np.uint32) == np.float32(s).view(np.uint32) and int(zp[0]) == z
            assert got.max() <= qmax
        else:
            ref, s = O.c_quantize_sym_rows(w, qsym)
            assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32))
            assert np.abs(got.astype(np.int32)).max() == qsym
        assert np.array_equal(got, ref)
    with pytest.raises(aq.AqError):
        aq.quantize_tensor(U.to_dev(w), rows, cols, scheme, 100, codes, scale, zp, ws)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "conv_small", "literal256"])
@pytest.mark.parametrize("wbits", [2, 4, 6])
@pytest.mark.parametrize("path", [0, 2])
def test_forward_with_weights_below_8_bits(aq, name, wbits, path):
    """The whole path with n-bit weight codes (8-bit containers, 8-bit activations): every stage against
    the oracle as at 8 bits, and the codes really use no more than 2^n levels."""
    _say(f"forward_with_weights_below_8_bits {name} wbits={wbits} path={path}")
    net = dict(_nets()[name], wbits=wbits)
    params = synth.make_params(net, nonzero_bias=True)
    batch = 150
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs)
    for q in pol.q:
        c = q["codes"].astype(np.int64)
        assert c.max() - c.min() <= 2 ** wbits - 1
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    U.check_quantized_params(aq, P, pol, net)
    P.policy_set_path(path)
    actions, t = U.gpu_forward(P, net, obs)
    U.compare_forward(net, pol, obs, actions, t)
    # a blob of this policy does not load into an 8-bit handle of the same network
    blob = torch.zeros(P.policy_blob_size(), dtype=torch.uint8, device=U.DEV)
    P.policy_export_blob(blob)
    Q = aq.Policy(_nets()[name])
    Q.policy_import_blob(blob)
    assert Q.policy_status() == aq.EINVAL
    P.close()
    Q.close()


def test_quantize_tensor_literal_denominator_and_nonfinite(aq):
    w = np.array([[-1, 0, 0.5, 1]], np.float32)
    codes = torch.zeros(1, 4, dtype=torch.uint8, device=U.DEV)
    scale = torch.zeros(1, dtype=torch.float32, device=U.DEV)
    zp = torch.zeros(1, dtype=torch.int32, device=U.DEV)
    ws = torch.zeros(4096, dtype=torch.int32, device=U.DEV)
    aq.quantize_tensor(U.to_dev(w), 1, 4, "tensor_asym_u8", 256, codes, scale, zp, ws)
    assert codes.cpu().numpy().tolist() == [[0, 128, 192, 255]] and float(scale[0]) == 1 / 128 and int(zp[0]) == 128
    for scheme in ("tensor_asym_u8", "channel_sym_s8"):
        w = np.array([[0.5, np.nan, 1.0, 2.0]], np.float32)
        ws.zero_()
        aq.quantize_tensor(U.to_dev(w), 1, 4, scheme, 255, codes, scale, zp, ws)
        torch.cuda.synchronize()
        assert int(ws[2]) == 1
    with pytest.raises(aq.AqError):
        aq.quantize_tensor(U.to_dev(w), 1, 3, "tensor_asym_u8", 255, codes, scale, zp, ws)


# ------------------------------------------------------------------ whole path, small batches, every stage
def _nets():
    fc, conv = synth.fc, synth.conv
    return {
        "cfg1": synth.net_config("cfg1"),
        "cfg2": synth.net_config("cfg2"),
        "odd_asym": synth.small_net([fc(17, 96, "relu"), fc(96, 40, "none"), fc(40, 6, "none")], head="linear",
                                    wscheme="tensor_asym_u8"),
        "odd_sym_ln": synth.small_net([fc(67, 200, "ln_tanh"), fc(200, 72, "relu"), fc(72, 21, "none")],
                                      head="tanh"),
        "argmax_mlp": synth.small_net([fc(33, 64, "relu"), fc(64, 18, "none")], head="argmax"),
        "u8_mlp": synth.small_net([fc(48, 64, "relu"), fc(64, 5, "none")], head="tanh", in_type="u8"),
        "literal256": synth.small_net([fc(17, 64, "relu"), fc(64, 6, "none")], head="tanh", qdenom=256,
                                      wscheme="tensor_asym_u8"),
        # last layers of one, two and more feature tiles, and single-layer networks (the fused kernel
        # spreads a narrow last layer over its waves by splitting K)
        "wide_last": synth.small_net([fc(40, 64, "relu"), fc(64, 100, "none")], head="linear"),
        "two_tile_last_asym": synth.small_net([fc(30, 64, "relu"), fc(64, 60, "none")], head="argmax",
                                              wscheme="tensor_asym_u8"),
        "single_narrow": synth.small_net([fc(50, 37, "none")], head="tanh"),
        "single_wide_asym": synth.small_net([fc(50, 130, "none")], head="linear", wscheme="tensor_asym_u8"),
        "long_k_narrow": synth.small_net([fc(20, 700, "relu"), fc(700, 10, "none")], head="tanh"),
        "conv_small": synth.small_net([conv(12, 12, 4, 16, 4, 4, 2, "relu"), conv(5, 5, 16, 32, 3, 3, 1, "relu"),
                                       fc(288, 48, "relu"), fc(48, 5, "none")], head="argmax", in_type="u8",
                                      init="he_normal"),
        # convolution stacks whose shapes the single-launch kernel takes: a ragged single tile, 48 and 40
        # features (second feature tile half empty), 49 output positions (ragged second row tile), a layer
        # without ReLU
        "conv_stack_a": synth.small_net([conv(20, 20, 4, 16, 8, 8, 4, "relu"), conv(4, 4, 16, 8, 2, 2, 1, "none"),
                                         fc(72, 24, "relu"), fc(24, 5, "none")], head="argmax", in_type="u8",
                                        init="he_normal"),
        "conv_stack_b": synth.small_net([conv(28, 28, 8, 48, 4, 4, 4, "relu"), conv(7, 7, 48, 32, 2, 2, 2, "relu"),
                                         conv(3, 3, 32, 16, 2, 2, 1, "relu"), fc(64, 20, "relu"), fc(20, 6, "none")],
                                        head="tanh", in_type="u8", init="he_normal"),
        "conv_odd": synth.small_net([conv(9, 10, 3, 5, 3, 2, 2, "relu"), fc(100, 24, "none"), fc(24, 7, "none")],
                                    head="tanh", in_type="u8", init="he_normal"),
    }


@pytest.mark.parametrize("name", list(_nets().keys()))
@pytest.mark.parametrize("path", [0, 2])
@pytest.mark.parametrize("batch", [1, 77, 300])
def test_forward_every_stage(aq, name, path, batch):
    _say(f"forward_every_stage {name} path={path} batch={batch}")
    net = _nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs)
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    U.check_quantized_params(aq, P, pol, net)
    P.policy_set_path(path)
    for rep in range(3):  # three times: a racy LDS stage would show as a changing accumulator
        actions, t = U.gpu_forward(P, net, obs)
        U.compare_forward(net, pol, obs, actions, t)
    # without taps the actions are the same
    a2, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(a2, actions, equal_nan=True)
    P.close()


@pytest.mark.parametrize("name,nc", [("conv_stack_a", 2), ("conv_stack_b", 3), ("cfg4", 3), ("conv_small", 0)])
@pytest.mark.parametrize("batch", [1, 3, 70])
def test_convolutions_in_one_launch(aq, name, nc, batch):
    """The leading convolutions as one launch (frame and feature maps in LDS) against the oracle, stage by
    stage, and against one launch per layer; without taps the actions must not change."""
    _say(f"convolutions_in_one_launch {name} batch={batch}")
    net = _nets()[name] if name in _nets() else synth.net_config(name)
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs)
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    assert P.policy_conv_stack_layers() == nc
    got = {}
    for path in (0, 3):
        P.policy_set_path(path)
        assert P.policy_conv_stack_layers() == (nc if path == 0 else 0)
        actions, t = U.gpu_forward(P, net, obs)
        U.compare_forward(net, pol, obs, actions, t)
        plain, _ = U.gpu_forward(P, net, obs, taps=False)
        assert np.array_equal(plain, actions)
        got[path] = actions
    assert np.array_equal(got[0], got[3])
    # observations at an address that is not 16-byte aligned take the per-layer launches: same result
    P.policy_set_path(0)
    shifted, _ = U.gpu_forward(P, net, obs, taps=False, misalign=3)
    assert np.array_equal(shifted, got[0])
    P.close()


@pytest.mark.parametrize("seed", list(range(16)))
def test_random_convolution_stacks(aq, seed):
    rng = np.random.default_rng(7000 + seed)
    net, nc = U.random_conv_stack(rng)
    batch = int(rng.choice([1, 5, 37, 300]))
    _say(f"random_convolution_stacks seed={seed} batch={batch} layers={[(l['in_h'], l['in_w'], l['in_c'], l['out_c'], l['kh'], l['kw'], l['stride']) for l in net['layers'][:nc]]}")
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs)
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    assert P.policy_conv_stack_layers() == nc
    actions, t = U.gpu_forward(P, net, obs)
    U.compare_forward(net, pol, obs, actions, t)
    plain, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(plain, actions)
    P.close()


@pytest.mark.parametrize("name", ["cfg2", "odd_asym", "u8_mlp", "single_narrow"])
@pytest.mark.parametrize("path", [0, 2])
@pytest.mark.parametrize("batch", [15, 16, 17, 33, 4096, 4097])
def test_forward_unaligned_observations_and_tile_edges(aq, name, path, batch):
    """Observation buffers that are not 16-byte aligned (fp32: 4 bytes off, uint8: 1 byte off) take the
    element-wise staging path; batch sizes sit on both sides of the 16- and 32-row workgroup sizes and
    of the switch between them."""
    _say(f"forward_unaligned {name} path={path} batch={batch}")
    net = _nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs[:256])
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    P.policy_set_path(path)
    rows = None if batch <= 64 else np.unique(np.concatenate([[0, 15, 16, 31, 32, batch - 2, batch - 1],
                                                               np.random.default_rng(8).integers(0, batch, 200)]))
    a_ref, t = U.gpu_forward(P, net, obs)
    U.compare_forward(net, pol, obs, a_ref, t, rows)
    a_mis, t = U.gpu_forward(P, net, obs, misalign=1)
    U.compare_forward(net, pol, obs, a_mis, t, rows)
    a_mis2, _ = U.gpu_forward(P, net, obs, taps=False, misalign=3)
    assert np.array_equal(a_mis2, a_mis, equal_nan=True)
    # An unaligned buffer takes the general kernel.  Where the aligned one ran the 16-row kernel, a LayerNorm
    # layer's fp32 statistics were summed in another order, and a code next to a rounding tie may differ: both
    # runs are held to the oracle above, bit equality between them is required of integer-only networks.
    ln = any(l["act"] == "ln_tanh" for l in net["layers"])
    if not (ln and path == 0 and P.policy_fused_plan(batch)[2] >= 2):
        assert np.array_equal(a_mis, a_ref, equal_nan=True)
    P.close()


@pytest.mark.parametrize("path", [0, 2])
@pytest.mark.parametrize("hi1,hi2", [(0.02, 3.0), (3.0, 3e5), (1e-3, 1e-3), (40.0, 0.5)])
def test_requant_forms(aq, path, hi1, hi2):
    """Activation ranges far from the calibrated ones push the requantization multiplier out of the
    window of the kernels' short form (r < 33: multiplier >= 1/4; r > 54: tiny multiplier): the
    general form must give the same integers as the oracle there too."""
    _say(f"requant_forms path={path} hi=({hi1},{hi2})")
    net = synth.small_net([synth.fc(40, 64, "relu"), synth.fc(64, 96, "none"), synth.fc(96, 9, "none")],
                          head="linear")
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, 70)
    pol = O.OraclePolicy(net)
    _, ranges = pol.forward_fp32(params, obs)
    ranges = [ranges[0], (np.float32(0.0), np.float32(hi1)), (np.float32(-hi2), np.float32(hi2))]
    pol.quantize_params(params, ranges)
    r = np.concatenate([pol.q[0]["rshift"], pol.q[1]["rshift"]])
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    U.check_quantized_params(aq, P, pol, net)
    P.policy_set_path(path)
    actions, t = U.gpu_forward(P, net, obs)
    U.compare_forward(net, pol, obs, actions, t)
    _say(f"  shifts span {r.min()}..{r.max()}")
    P.close()


# ------------------------------------------------------------------ full sizes, launch configuration of the bench
@pytest.mark.parametrize("name,batch,sample", [("cfg1", 256, None), ("cfg2", 4096, None), ("cfg3", 65536, 2048),
                                               ("cfg3", 16, None), ("cfg5", 16384, 384), ("cfg4", 256, 64)])
def test_forward_full_size(aq, name, batch, sample):
    _say(f"forward_full_size {name} batch={batch}")
    net = synth.net_config(name)
    params = synth.make_params(net)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs[:min(batch, 512)])
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    U.check_quantized_params(aq, P, pol, net)
    actions, t = U.gpu_forward(P, net, obs)
    rows = None
    if sample is not None:
        rng = np.random.default_rng(5)
        rows = np.unique(np.concatenate([[0, batch - 1], rng.integers(0, batch, sample)]))
    flips = U.compare_forward(net, pol, obs, actions, t, rows)
    _say(f"  LayerNorm code flips at rounding ties: {flips}")
    # the launch the benchmark times has no intermediate outputs (another compiled variant): same actions
    plain, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(plain, actions, equal_nan=True)
    # properties that hold at any size
    if net["head"] == "tanh":
        assert np.isfinite(actions).all() and np.abs(actions).max() <= 1.0
    else:
        assert actions.min() >= 0 and actions.max() < synth.action_dim(net)
    P.close()


# Every compiled variant of the whole-network kernels, named by (batch rows per workgroup, feature tiles per
# wavefront, per-tensor weight scheme, kernel kind: 0 general, 1 pipelined for wide layers, 2 the kernel
# for small networks, 3 its form for a workgroup alone on its CU: batch up to 4096): the network and batch that make the launch plan pick it.  Each is run with intermediate
# outputs (checked stage by stage against the oracle) and without (the variant a benchmark times; its actions
# must be the same bits).
_ODD_WIDE = [synth.fc(100, 1000, "relu"), synth.fc(1000, 1024, "relu"), synth.fc(1024, 40, "none")]
FUSED_VARIANTS = {
    # the kernel for small networks: one, two and four 16-row tiles per workgroup (batch up to 8192, up to 24576,
    # beyond), each with ragged shapes, LayerNorm on a ragged width, argmax over two feature tiles, one layer,
    # 8-bit observations (rows of 48 and of 37 bytes), for both weight schemes
    (16, 1, False, 3): [("cfg2", 4096), ("cfg2", 70), ("odd_small", 3000), ("argmax_small", 333), ("single_narrow", 100),
                        ("u8_mlp", 300)],
    (16, 1, False, 2): [("cfg2", 8185), ("odd_small", 4100), ("argmax_small", 5000), ("single_narrow", 4097),
                        ("u8_mlp", 6000)],
    (32, 1, False, 2): [("cfg2", 16384), ("odd_small", 8200), ("argmax_small", 12001), ("single_narrow", 8193),
                        ("u8_mlp", 10000)],
    (64, 1, False, 2): [("cfg2", 24580), ("cfg2", 32763), ("odd_small", 30011), ("argmax_small", 25000),
                        ("single_narrow", 24590), ("odd_sym_ln", 24577), ("u8_mlp", 26500)],
    (16, 1, True, 3): [("cfg1", 256), ("odd_asym", 100), ("two_tile_last_asym", 333), ("literal256", 77),
                       ("u8_odd_asym", 500), ("asym_ln", 1000)],
    (16, 1, True, 2): [("cfg1", 8192), ("odd_asym", 4100), ("two_tile_last_asym", 5000), ("u8_odd_asym", 4500),
                       ("asym_ln", 7000)],
    (32, 1, True, 2): [("cfg1", 16379), ("odd_asym", 8200), ("asym_ln", 9000), ("two_tile_last_asym", 8500)],
    (64, 1, True, 2): [("cfg1", 24600), ("odd_asym", 30011), ("two_tile_last_asym", 27000), ("u8_odd_asym", 24590),
                       ("asym_ln", 26500)],
    # the general kernel
    (16, 1, False, 0): [("mid_wide", 4096)],
    (16, 1, True, 0): [("mid_wide_asym", 4096)],
    (32, 1, False, 0): [("mid_wide", 8192)],
    (64, 1, False, 0): [("mid_wide", 16379)],
    (128, 1, False, 0): [("mid_wide", 32763), ("mid_wide_ln", 32700)],
    (32, 2, False, 0): [("cfg5", 8192), ("odd_wide", 8185)],
    (64, 2, False, 0): [("odd_wide", 16379)],
    (64, 2, False, 1): [("cfg5", 16384)],
    (32, 1, True, 0): [("mid_wide_asym", 8192)],
    (64, 1, True, 0): [("mid_wide_asym", 16379)],
}


def _variant_net(name):
    if name == "odd_wide":  # a ragged last feature tile (1000 = 31 * 32 + 8) with two tiles per wavefront
        return synth.small_net(_ODD_WIDE, head="tanh")
    if name == "odd_small":  # the 16-row kernel on ragged shapes: odd K, odd tile counts, LayerNorm on a ragged width
        return synth.small_net([synth.fc(37, 200, "relu"), synth.fc(200, 72, "ln_tanh"), synth.fc(72, 250, "none"),
                                synth.fc(250, 40, "none")], head="linear")
    if name == "argmax_small":  # ... and with an argmax head over two feature tiles
        return synth.small_net([synth.fc(130, 96, "relu"), synth.fc(96, 50, "none")], head="argmax")
    if name == "mid_wide_ln":  # ... with LayerNorm over a 256-wide layer behind it
        return synth.small_net([synth.fc(67, 512, "relu"), synth.fc(512, 256, "ln_tanh"), synth.fc(256, 21, "none")],
                               head="tanh")
    if name == "mid_wide_asym":  # per-tensor weights with a layer too wide for the small-network kernel
        return synth.small_net([synth.fc(67, 512, "relu"), synth.fc(512, 256, "relu"), synth.fc(256, 21, "none")],
                               head="tanh", wscheme="tensor_asym_u8")
    if name == "u8_odd_asym":  # 8-bit observations in rows that are not 4-byte aligned, per-tensor weights
        return synth.small_net([synth.fc(37, 100, "relu"), synth.fc(100, 30, "none"), synth.fc(30, 11, "none")],
                               head="tanh", wscheme="tensor_asym_u8", in_type="u8")
    if name == "asym_ln":  # LayerNorm on a ragged width with per-tensor weights
        return synth.small_net([synth.fc(20, 150, "ln_tanh"), synth.fc(150, 90, "relu"), synth.fc(90, 33, "none")],
                               head="linear", wscheme="tensor_asym_u8")
    if name in _nets():
        return _nets()[name]
    if name == "mid_wide":  # 128-row workgroups with a 512-wide layer (two passes of the eight wavefronts)
        return synth.small_net([synth.fc(67, 512, "relu"), synth.fc(512, 256, "relu"), synth.fc(256, 21, "none")],
                               head="tanh")
    return synth.net_config(name)


def test_fused_variant_table_covers_every_compiled_variant():
    """The table above names every instantiation the library compiles (with and without intermediate outputs)."""
    import os
    import re
    src = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_1910_01055_amd", "csrc",
                       "fused_mlp.hip")
    decl = re.findall(r"AQ_FUSED_DECL\((\d), (\d), (true|false), (true|false), (true|false)\);", open(src).read())
    assert len(decl) >= 18
    seen = {}
    for mt, nb, asym, taps, half in decl:
        key = (16 if half == "true" else 32 * int(mt), int(nb), asym == "true")
        seen.setdefault(key, set()).add(taps)
    # the general kernel's instantiations, plus the pipelined and the small-network kernel (each compiled with and
    # without intermediate outputs in its own file)
    assert set(seen) == {k[:3] for k in FUSED_VARIANTS if k[3] == 0}, (sorted(seen), sorted(FUSED_VARIANTS))
    assert all(v == {"true", "false"} for v in seen.values())
    assert {k[3] for k in FUSED_VARIANTS} == {0, 1, 2, 3}


@pytest.mark.parametrize("key", sorted(FUSED_VARIANTS))
def test_every_fused_variant_against_the_oracle(aq, key):
    for name, batch in FUSED_VARIANTS[key]:
        _say(f"fused_variant rows={key[0]} tiles={key[1]} per_tensor={key[2]} {name} batch={batch}")
        net = _variant_net(name)
        assert (net["wscheme"] == "tensor_asym_u8") == key[2]
        params = synth.make_params(net, nonzero_bias=True)
        obs = synth.make_obs(net, batch)
        pol, ranges = U.make_oracle(net, params, obs[:256])
        P, _ = U.gpu_quantize(aq, net, params, ranges)
        assert P.policy_fused_plan(batch) == (key[0], key[1], key[3])
        rng = np.random.default_rng(21)
        rows = np.unique(np.concatenate([[0, 15, 16, 31, 32, 63, 64, batch - 65, batch - 33, batch - 17, batch - 1],
                                         rng.integers(0, batch, 250)]))
        first = None
        for rep in range(3):
            actions, t = U.gpu_forward(P, net, obs)
            U.compare_forward(net, pol, obs, actions, t, rows)
            del t
            plain, _ = U.gpu_forward(P, net, obs, taps=False)
            assert np.array_equal(plain, actions, equal_nan=True)
            assert first is None or np.array_equal(first, plain, equal_nan=True)
            first = plain
        if net["head"] == "tanh":
            assert np.isfinite(plain).all() and np.abs(plain).max() <= 1.0
        P.close()


# The software-pipelined kernel for wide layers (64 rows per workgroup): the benchmark's wide MLP, layers of
# one and two passes mixed (a 512-wide layer's epilogue cannot hide under its own layer), a width that leaves
# wavefronts idle in the last pass (640 = 10 groups of 64 features) with an argmax head, and a single wide layer.
def _wide_nets():
    fc = synth.fc
    return {
        "cfg5": synth.net_config("cfg5"),
        "wide_mixed": synth.small_net([fc(128, 512, "relu"), fc(512, 1024, "none"), fc(1024, 512, "relu"),
                                       fc(512, 30, "none")], head="linear"),
        "wide_idle_waves": synth.small_net([fc(256, 640, "relu"), fc(640, 1024, "relu"), fc(1024, 64, "none")],
                                           head="argmax"),
        "wide_single": synth.small_net([fc(384, 1024, "relu"), fc(1024, 5, "none")], head="tanh"),
    }


@pytest.mark.parametrize("name,batch", [("cfg5", 16384), ("cfg5", 16321), ("wide_mixed", 16379), ("wide_idle_waves", 16000),
                                        ("wide_single", 12345), ("cfg5", 70000)])
def test_pipelined_wide_kernel_against_the_oracle(aq, name, batch):
    _say(f"pipelined_wide_kernel {name} batch={batch}")
    net = _wide_nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs[:256])
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    assert P.policy_fused_plan(batch) == (64, 2, 1)
    rng = np.random.default_rng(22)
    rows = np.unique(np.concatenate([[0, 31, 32, 63, 64, batch - 65, batch - 64, batch - 33, batch - 1],
                                     rng.integers(0, batch, 200)]))
    first = None
    for rep in range(3):
        actions, t = U.gpu_forward(P, net, obs)
        U.compare_forward(net, pol, obs, actions, t, rows)
        del t
        plain, _ = U.gpu_forward(P, net, obs, taps=False)
        assert np.array_equal(plain, actions, equal_nan=True)
        assert first is None or np.array_equal(first, plain, equal_nan=True)
        first = plain
    # an observation buffer that is not 16-byte aligned takes the general kernel: same bits
    shifted, _ = U.gpu_forward(P, net, obs, taps=False, misalign=1)
    assert np.array_equal(shifted, plain, equal_nan=True)
    # so does the one-launch-per-layer plan
    P.policy_set_path(2)
    per_layer, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(per_layer, plain, equal_nan=True)
    P.policy_set_path(0)
    if net["head"] != "argmax":
        # the actor step adds the exploration noise inside the kernel: same bits as forward, then explore
        d_obs = U.to_dev(obs)
        sg = U.to_dev(np.random.default_rng(23).uniform(0, 0.2, batch).astype(np.float32))
        a1 = torch.zeros(batch, synth.action_dim(net), dtype=torch.float32, device=U.DEV)
        a2 = torch.zeros_like(a1)
        P.policy_step_int8(d_obs, a1, 99, 5, sigma=sg)
        P.policy_forward_int8(d_obs, a2)
        P.policy_explore(a2, 99, 5, sigma=sg)
        torch.cuda.synchronize()
        assert torch.equal(a1, a2) and not np.array_equal(a1.cpu().numpy(), plain)
    P.close()


@pytest.mark.parametrize("hi1,hi2", [(0.02, 3.0), (3.0, 3e5), (1e-3, 1e-3)])
def test_pipelined_wide_kernel_general_requant_form(aq, hi1, hi2):
    """Activation ranges that push a layer's requantization shifts out of the short form's window: the
    pipelined kernel then runs that layer's epilogue in the general 64-bit form (not hidden under MFMAs)."""
    _say(f"pipelined_wide_requant hi=({hi1},{hi2})")
    net = synth.small_net([synth.fc(256, 1024, "relu"), synth.fc(1024, 1024, "none"), synth.fc(1024, 9, "none")],
                          head="linear")
    params = synth.make_params(net, nonzero_bias=True)
    batch = 16200
    obs = synth.make_obs(net, batch)
    pol = O.OraclePolicy(net)
    _, ranges = pol.forward_fp32(params, obs[:128])
    ranges = [ranges[0], (np.float32(0.0), np.float32(hi1)), (np.float32(-hi2), np.float32(hi2))]
    pol.quantize_params(params, ranges)
    r = np.concatenate([pol.q[0]["rshift"], pol.q[1]["rshift"]])
    _say(f"  shifts span {r.min()}..{r.max()}")
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    assert P.policy_fused_plan(batch) == (64, 2, 1)
    rows = np.unique(np.concatenate([[0, 63, 64, batch - 1], np.random.default_rng(24).integers(0, batch, 120)]))
    actions, t = U.gpu_forward(P, net, obs)
    U.compare_forward(net, pol, obs, actions, t, rows)
    plain, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(plain, actions, equal_nan=True)
    P.close()


@pytest.mark.parametrize("name", ["odd_asym", "two_tile_last_asym", "wide_last", "single_narrow", "long_k_narrow",
                                  "odd_sym_ln"])
@pytest.mark.parametrize("batch", [16500, 65700])
def test_fused_row_tiles_large_batch(aq, name, batch):
    """Small networks at the batch sizes where the fused kernel takes 64 and 128 rows per workgroup
    (every weight scheme, narrow and wide last layers), on sampled rows."""
    _say(f"fused_row_tiles_large_batch {name} batch={batch}")
    net = _nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs[:256])
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    actions, t = U.gpu_forward(P, net, obs)
    rng = np.random.default_rng(7)
    rows = np.unique(np.concatenate([[0, 31, 32, 63, 64, 127, 128, batch - 1], rng.integers(0, batch, 300)]))
    U.compare_forward(net, pol, obs, actions, t, rows)
    a2, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(a2, actions, equal_nan=True)
    P.close()


@pytest.mark.parametrize("name,batch,sample", [("cfg2", 262149, 400), ("paper_fc2048", 8200, 200), ("cfg4", 1100, 24),
                                               ("cfg1", 70001, 300)])
def test_very_large_batches(aq, name, batch, sample):
    """Sizes well past the benchmark's: many rounds of workgroups per CU in the fused kernel, the 8-wave
    tile of the per-layer kernel on 2048-wide layers, the convolution path at several hundred
    thousand output positions, and per-tensor asymmetric weights on 64-row workgroups; sampled rows against the oracle, every row for the stated invariants."""
    _say(f"very_large_batches {name} batch={batch}")
    net = synth.net_config(name)
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs[:128])
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    actions, t = U.gpu_forward(P, net, obs)
    rng = np.random.default_rng(9)
    rows = np.unique(np.concatenate([[0, 127, 128, batch - 129, batch - 1], rng.integers(0, batch, sample)]))
    U.compare_forward(net, pol, obs, actions, t, rows)
    del t
    a2, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(a2, actions)
    if net["head"] == "argmax":
        assert actions.min() >= 0 and actions.max() < synth.action_dim(net)
    else:
        assert np.isfinite(actions).all() and np.abs(actions).max() <= 1.0
    P.close()


@pytest.mark.parametrize("batch", [1, 16, 40, 300])
def test_paper_scale_actor_small_batches(aq, batch):
    """The paper's own actor shape (three hidden layers of 2048 units) at the batch sizes of its actors:
    too wide for the fused kernel, so every layer runs as a K-split launch (or the tiled kernel)."""
    _say(f"paper_scale_actor batch={batch}")
    net = synth.net_config("paper_fc2048")
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, synth.make_obs(net, 64))
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    actions, t = U.gpu_forward(P, net, obs)
    U.compare_forward(net, pol, obs, actions, t)
    a2, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(a2, actions)
    P.close()


@pytest.mark.parametrize("name,batch,sample", [("cfg5", 8200, 300), ("cfg2", 9000, 400)])
def test_per_layer_path_large_batch(aq, name, batch, sample):
    """The one-launch-per-layer plan at batch sizes where it picks its 128-row / 8-wave and its narrow
    2-wave tile configurations (MLPs normally run fused; convolution layers always take this path)."""
    _say(f"per_layer_path_large_batch {name} batch={batch}")
    net = synth.net_config(name)
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs[:256])
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    P.policy_set_path(2)
    actions, t = U.gpu_forward(P, net, obs)
    rng = np.random.default_rng(6)
    rows = np.unique(np.concatenate([[0, 127, 128, batch - 1], rng.integers(0, batch, sample)]))
    U.compare_forward(net, pol, obs, actions, t, rows)
    a2, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(a2, actions)
    P.close()


# ------------------------------------------------------------------ fp32 actor and calibration
@pytest.mark.parametrize("name,batch", [("cfg1", 256), ("cfg2", 300), ("cfg4", 8), ("cfg5", 96)])
def test_forward_fp32(aq, name, batch):
    _say(f"forward_fp32 {name} batch={batch}")
    net = synth.net_config(name)
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol = O.OraclePolicy(net)
    ref, ranges = pol.forward_fp32(params, obs)
    P = aq.Policy(net)
    w, b, g, be = U.upload_params(params)
    A = synth.action_dim(net)
    nl = len(net["layers"])
    if net["head"] == "argmax":
        actions = torch.zeros(batch, dtype=torch.int32, device=U.DEV)
    else:
        actions = torch.zeros(batch, A, dtype=torch.float32, device=U.DEV)
    r = torch.zeros(2 * nl, dtype=torch.float32, device=U.DEV)
    d_obs = U.to_dev(obs)
    P.policy_forward_fp32_params(w, b, g, be, d_obs, actions, r)
    torch.cuda.synchronize()
    got = actions.cpu().numpy()
    # the same actor on parameters kept in the handle, and the calibration call
    a2 = torch.zeros_like(actions)
    with pytest.raises(aq.AqError) as e:
        P.policy_forward_fp32(d_obs, a2)
    assert e.value.status == aq.ENOTQUANT
    with pytest.raises(aq.AqError) as e:
        P.calibrate_fp32(d_obs)
    assert e.value.status == aq.ENOTQUANT
    with pytest.raises(aq.AqError) as e:
        P.quantize_kept_params(ranges)
    assert e.value.status == aq.ENOTQUANT
    P.policy_set_params_fp32(w, b, g, be)
    P.policy_forward_fp32(d_obs, a2)
    torch.cuda.synchronize()
    assert torch.equal(a2, actions)
    kept = P.calibrate_fp32(d_obs)
    assert np.array_equal(np.array(kept, np.float32).reshape(-1), r.cpu().numpy())
    # quantizing the kept copy gives the policy that quantizing the caller's arrays gives
    P.quantize_kept_params(ranges)
    assert P.policy_status() == aq.OK
    pol.quantize_params(params, ranges)
    U.check_quantized_params(aq, P, pol, net)
    if name == "cfg2":  # absent biases, gains and offsets take their defaults in the kept copy as well
        Q = aq.Policy(net)
        Q.policy_set_params_fp32(w, None, None, None)
        a3, a4 = torch.zeros_like(actions), torch.zeros_like(actions)
        Q.policy_forward_fp32(d_obs, a3)
        Q.policy_forward_fp32_params(w, None, None, None, d_obs, a4)
        torch.cuda.synchronize()
        assert torch.equal(a3, a4) and not torch.equal(a3, actions)
        Q.close()
    if net["head"] == "argmax":
        # an fp32 sum may reorder two nearly equal logits; require agreement wherever the oracle's margin is clear
        assert (got == ref).mean() >= 0.99
    else:
        assert U.close(got, ref).all()
    rr = r.cpu().numpy().reshape(nl, 2)
    for i, (lo, hi) in enumerate(ranges):
        assert abs(rr[i, 0] - lo) <= 1e-4 * abs(lo) + 1e-6 and abs(rr[i, 1] - hi) <= 1e-4 * abs(hi) + 1e-6
    P.close()


def test_quantization_error_report_matches_oracle(aq):
    """The wide MLP's report of how far the 8-bit actions are from the fp32 actions on the same observations
    (largest and mean absolute difference, SQNR): the figures from the GPU's two forwards equal the figures
    from the oracle's two forwards.  The value itself is not pinned by the paper (it only calls the change of
    the action distribution very small, App. C), so it is held to a sanity bound only."""
    net = synth.net_config("cfg5")
    batch = 512
    _say(f"quantization_error_report cfg5 batch={batch}")
    params = synth.make_params(net)
    obs = synth.make_obs(net, batch)
    pol = O.OraclePolicy(net)
    o32, ranges = pol.forward_fp32(params, obs)
    pol.quantize_params(params, ranges)
    o8 = pol.forward_int8(obs)["actions"]
    P, d = U.gpu_quantize(aq, net, params, ranges)
    d_obs = U.to_dev(obs)
    g8 = torch.zeros(batch, synth.action_dim(net), dtype=torch.float32, device=U.DEV)
    g32 = torch.zeros_like(g8)
    P.policy_forward_int8(d_obs, g8)
    P.policy_set_params_fp32(*d)
    P.policy_forward_fp32(d_obs, g32)
    torch.cuda.synchronize()
    fg = U.action_error_figures(g8.cpu().numpy(), g32.cpu().numpy())
    fo = U.action_error_figures(o8, o32)
    _say(f"  GPU {fg}\n  oracle {fo}")
    assert abs(fg["max_abs"] - fo["max_abs"]) <= 1e-4 and abs(fg["mean_abs"] - fo["mean_abs"]) <= 1e-4
    assert abs(fg["sqnr_db"] - fo["sqnr_db"]) <= 0.05
    assert 0.0 < fo["mean_abs"] <= 0.05 and fo["max_abs"] <= 0.5 and fo["sqnr_db"] >= 15.0
    P.close()


# ------------------------------------------------------------------ policy blob (learner -> actor hand-off)
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "odd_sym_ln", "conv_small", "two_tile_last_asym"])
def test_policy_blob_round_trip(aq, name):
    """A policy exported as one blob and imported into a fresh handle of the same network computes what
    the oracle computes, bit for bit, and exposes the oracle's codes and constants; a blob from another
    network is refused through the status flag; size errors are refused at once."""
    _say(f"policy_blob_round_trip {name}")
    net = _nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, 70)
    pol, ranges = U.make_oracle(net, params, obs)
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    nbytes = P.policy_blob_size()
    assert nbytes > 192
    blob = torch.full((nbytes,), 0xAB, dtype=torch.uint8, device=U.DEV)
    Q = aq.Policy(net)
    with pytest.raises(aq.AqError) as e:
        Q.policy_export_blob(blob)
    assert e.value.status == aq.ENOTQUANT
    with pytest.raises(aq.AqError) as e:
        P.policy_export_blob(blob[:nbytes - 16])
    assert e.value.status == aq.EINVAL
    P.policy_export_blob(blob)
    torch.cuda.synchronize()
    with pytest.raises(aq.AqError) as e:
        Q.policy_import_blob(blob[:nbytes - 16])
    assert e.value.status == aq.EINVAL
    Q.policy_import_blob(blob)
    assert Q.policy_status() == aq.OK
    P.close()  # the imported copy owns everything it needs
    blob2 = torch.zeros_like(blob)
    Q.policy_export_blob(blob2)
    torch.cuda.synchronize()
    assert torch.equal(blob, blob2)
    U.check_quantized_params(aq, Q, pol, net)
    for path in (0, 2):
        Q.policy_set_path(path)
        actions, t = U.gpu_forward(Q, net, obs)
        U.compare_forward(net, pol, obs, actions, t)
    # a blob of a different network: flagged, not installed silently
    other = synth.small_net([synth.fc(12, 40, "relu"), synth.fc(40, 3, "none")], head="tanh")
    R = aq.Policy(other)
    big = torch.zeros(max(nbytes, R.policy_blob_size()), dtype=torch.uint8, device=U.DEV)
    big[:nbytes] = blob
    R.policy_import_blob(big)
    assert R.policy_status() == aq.EINVAL
    R.close()
    Q.close()


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "conv_small", "odd_asym"])
@pytest.mark.parametrize("wbits", [2, 4, 5, 6, 8])
def test_packed_policy_blob_round_trip(aq, name, wbits):
    """n-bit weight codes travel sub-byte: the packed blob is about n/8 of the weights' size, and a fresh
    handle that imports it exposes the oracle's codes and constants and computes the same bits."""
    _say(f"packed_policy_blob_round_trip {name} wbits={wbits}")
    net = dict(_nets()[name], wbits=wbits)
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, 130)
    pol, ranges = U.make_oracle(net, params, obs)
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    n_plain, n_packed = P.policy_blob_size(), P.policy_packed_blob_size()
    w_bytes = sum(int(np.prod(synth.layer_weight_shape(l))) for l in net["layers"])
    assert n_packed <= n_plain
    if wbits < 8:
        assert n_plain - n_packed >= w_bytes * (8 - wbits) // 8  # at least the real weights shrink by n/8
    blob = torch.full((n_packed + 64,), 0xA5, dtype=torch.uint8, device=U.DEV)
    P.policy_export_packed_blob(blob[:n_packed])
    torch.cuda.synchronize()
    assert bool((blob[n_packed:] == 0xA5).all())  # nothing written past the stated size
    Q = aq.Policy(net)
    Q.policy_import_packed_blob(blob[:n_packed])
    assert Q.policy_status() == aq.OK
    U.check_quantized_params(aq, Q, pol, net)
    for path in (0, 2):
        Q.policy_set_path(path)
        actions, t = U.gpu_forward(Q, net, obs)
        U.compare_forward(net, pol, obs, actions, t)
    # exporting from the importer gives the same bytes; a plain blob of it equals the original's
    blob2 = torch.zeros(n_packed, dtype=torch.uint8, device=U.DEV)
    Q.policy_export_packed_blob(blob2)
    assert torch.equal(blob2, blob[:n_packed])
    b1 = torch.zeros(n_plain, dtype=torch.uint8, device=U.DEV)
    b2 = torch.zeros(n_plain, dtype=torch.uint8, device=U.DEV)
    P.policy_export_blob(b1)
    Q.policy_export_blob(b2)
    assert torch.equal(b1, b2)
    # a handle with another weight precision, or the plain importer, refuses it
    R = aq.Policy(dict(net, wbits=8 if wbits != 8 else 4))
    if R.policy_packed_blob_size() <= n_packed:
        R.policy_import_packed_blob(blob[:n_packed])
        assert R.policy_status() == aq.EINVAL
    if n_plain <= n_packed:
        Q2 = aq.Policy(net)
        Q2.policy_import_blob(blob[:n_packed])
        assert Q2.policy_status() == aq.EINVAL
        Q2.close()
    for h in (P, Q, R):
        h.close()


# ------------------------------------------------------------------ exploration (Sec. 4.1)
@pytest.mark.parametrize("rows,A", [(1, 1), (77, 21), (4096, 6), (1000, 64)])
def test_explore_gaussian_matches_oracle(aq, rows, A):
    _say(f"explore_gaussian rows={rows} A={A}")
    net = synth.small_net([synth.fc(8, A, "none")], head="tanh")
    P = aq.Policy(net)
    rng = np.random.default_rng(11)
    a = rng.uniform(-1, 1, (rows, A)).astype(np.float32)
    sg = rng.uniform(0, 0.2, rows).astype(np.float32)
    sg[0] = 0.0
    for seed, step in ((5, 0), (0xFEDCBA9876543210, (3 << 32) + 17)):
        d_a = U.to_dev(a)
        P.policy_explore(d_a, seed, step, sigma=U.to_dev(sg))
        torch.cuda.synchronize()
        got = d_a.cpu().numpy()
        want = O.c_explore_gaussian(a, sg, seed, step)
        assert U.close(got, want).all()
        assert np.array_equal(got[0], a[0])          # sigma = 0: untouched
        if rows * A > 100:
            assert not np.array_equal(got, a)
    with pytest.raises(aq.AqError) as e:
        P.policy_explore(U.to_dev(a), 1, 1, sigma=None)
    assert e.value.status == aq.EINVAL
    P.close()


@pytest.mark.parametrize("rows,A", [(1, 2), (300, 18), (5000, 7)])
def test_explore_eps_greedy_matches_oracle(aq, rows, A):
    _say(f"explore_eps_greedy rows={rows} A={A}")
    net = synth.small_net([synth.fc(8, A, "none")], head="argmax")
    P = aq.Policy(net)
    idx = np.random.default_rng(12).integers(0, A, rows).astype(np.int32)
    for eps in (0.0, 0.05, 0.5, 1.0):
        for seed, step in ((9, 1), (1 << 40, 1 << 35)):
            d_i = U.to_dev(idx)
            P.policy_explore(d_i, seed, step, epsilon=eps)
            torch.cuda.synchronize()
            assert np.array_equal(d_i.cpu().numpy(), O.c_explore_eps_greedy(idx, A, eps, seed, step))
    with pytest.raises(aq.AqError) as e:
        P.policy_explore(U.to_dev(idx), 1, 1, epsilon=1.5)
    assert e.value.status == aq.EINVAL
    P.close()


@pytest.mark.parametrize("name", ["cfg1", "argmax_mlp"])
def test_forward_then_explore_end_to_end(aq, name):
    """The actor step: 8-bit forward, then exploration, against the oracle doing the same on its own actions."""
    _say(f"forward_then_explore {name}")
    net = _nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    batch = 200
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs)
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    ref = pol.forward_int8(obs)["actions"]
    d_obs = U.to_dev(obs)
    sg = np.random.default_rng(13).uniform(0, 0.2, batch).astype(np.float32)
    if net["head"] == "argmax":
        act = torch.zeros(batch, dtype=torch.int32, device=U.DEV)
        P.policy_forward_int8(d_obs, act)
        P.policy_explore(act, 77, 4, epsilon=0.25)
        torch.cuda.synchronize()
        assert np.array_equal(act.cpu().numpy(), O.c_explore_eps_greedy(ref, synth.action_dim(net), 0.25, 77, 4))
    else:
        act = torch.zeros(batch, synth.action_dim(net), dtype=torch.float32, device=U.DEV)
        P.policy_forward_int8(d_obs, act)
        P.policy_explore(act, 77, 4, sigma=U.to_dev(sg))
        torch.cuda.synchronize()
        assert U.close(act.cpu().numpy(), O.c_explore_gaussian(ref, sg, 77, 4)).all()
    P.close()


@pytest.mark.parametrize("name,path", [("cfg1", 0), ("cfg1", 2), ("single_narrow", 0), ("wide_last", 0), ("long_k_narrow", 0),
                                       ("argmax_mlp", 0), ("two_tile_last_asym", 2), ("conv_odd", 0)])
@pytest.mark.parametrize("batch", [5, 300])
def test_actor_step_entry_point(aq, name, path, batch):
    """aq_policy_step_int8 (noise added inside the forward kernel where that kernel writes the actions, a
    second launch otherwise) equals forward followed by explore, and both equal the oracle's step."""
    _say(f"actor_step {name} path={path} batch={batch}")
    net = _nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs)
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    P.policy_set_path(path)
    ref = pol.forward_int8(obs)["actions"]
    d_obs = U.to_dev(obs)
    A = synth.action_dim(net)
    sg = np.random.default_rng(14).uniform(0, 0.2, batch).astype(np.float32)
    seed, step = 0xABCDEF0123, (1 << 33) + 9
    if net["head"] == "argmax":
        a1 = torch.zeros(batch, dtype=torch.int32, device=U.DEV)
        a2 = torch.zeros_like(a1)
        P.policy_step_int8(d_obs, a1, seed, step, epsilon=0.3)
        P.policy_forward_int8(d_obs, a2)
        P.policy_explore(a2, seed, step, epsilon=0.3)
        torch.cuda.synchronize()
        assert torch.equal(a1, a2)
        assert np.array_equal(a1.cpu().numpy(), O.c_explore_eps_greedy(ref, A, 0.3, seed, step))
    else:
        a1 = torch.zeros(batch, A, dtype=torch.float32, device=U.DEV)
        a2 = torch.zeros_like(a1)
        d_sg = U.to_dev(sg)
        P.policy_step_int8(d_obs, a1, seed, step, sigma=d_sg)
        P.policy_forward_int8(d_obs, a2)
        P.policy_explore(a2, seed, step, sigma=d_sg)
        torch.cuda.synchronize()
        assert torch.equal(a1, a2)                      # the same arithmetic on both routes
        assert U.close(a1.cpu().numpy(), O.c_explore_gaussian(ref, sg, seed, step)).all()
    P.close()


# ------------------------------------------------------------------ seeded random shapes
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
        if act == "ln_tanh" and widths[i + 1] < 2:
            act = "relu"
        layers.append(fc(widths[i], widths[i + 1], act))
    return synth.small_net(layers, head=str(rng.choice(["tanh", "linear", "argmax"])),
                           wscheme=str(rng.choice(["channel_sym_s8", "tensor_asym_u8"])),
                           in_type=str(rng.choice(["f32", "f32", "u8"])), qdenom=int(rng.choice([255, 255, 256])))


@pytest.mark.parametrize("seed", list(range(40)))
def test_random_mlp_shapes(aq, seed):
    """Seeded random MLP policies (1-4 layers, widths on and off the tile edges, every activation, head,
    weight scheme, input type, 4..8-bit weights) at random batch sizes, on whichever path the library
    picks and on the per-layer path: every stage against the oracle."""
    rng = np.random.default_rng(7000 + seed)
    net = _random_net(rng)
    net["wbits"] = int(rng.choice([8, 8, 6, 4]))
    batch = int(rng.choice([1, 2, 15, 16, 17, 31, 33, 64, 100, 257, 600]))
    path = int(rng.choice([0, 0, 2]))
    desc = "-".join(str(l["in"]) for l in net["layers"]) + f"-{net['layers'][-1]['out']}"
    _say(f"random_mlp_shapes seed={seed} {desc} acts={[l['act'] for l in net['layers']]} head={net['head']} "
         f"{net['wscheme']} {net['in_type']} wbits={net['wbits']} batch={batch} path={path}")
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs)
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    U.check_quantized_params(aq, P, pol, net)
    P.policy_set_path(path)
    actions, t = U.gpu_forward(P, net, obs)
    U.compare_forward(net, pol, obs, actions, t)
    a2, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(a2, actions, equal_nan=True)
    P.close()


def _random_small_net(rng):
    """A random network of the small-network kernel's shape class without LayerNorm (integers only)."""
    fc = synth.fc
    n_layers = int(rng.integers(1, 5))
    widths = [int(rng.choice([1, 3, 4, 17, 63, 64, 65, 67, 128, 130, 255, 256]))]
    for i in range(n_layers):
        last = i == n_layers - 1
        widths.append(int(rng.choice([1, 2, 6, 16, 17, 21, 32, 33, 64] if last else
                                     [1, 5, 16, 31, 32, 33, 64, 96, 100, 160, 224, 255, 256])))
    layers = [fc(widths[i], widths[i + 1], "none" if i == n_layers - 1 else str(rng.choice(["relu", "none"])))
              for i in range(n_layers)]
    return synth.small_net(layers, head=str(rng.choice(["tanh", "linear", "argmax"])),
                           wscheme=str(rng.choice(["channel_sym_s8", "tensor_asym_u8"])),
                           in_type=str(rng.choice(["f32", "f32", "u8"])))


@pytest.mark.parametrize("seed", list(range(24)))
def test_small_network_kernel_equals_the_other_plans(aq, seed):
    """Integer-only random networks of the small-network kernel's shape class, at batch sizes that take one, two
    and four row tiles per workgroup: the actions equal, bit for bit, those of the general whole-network kernel
    (selected by an unaligned observation buffer) and of the one-launch-per-layer plan; sampled rows also go
    against the oracle stage by stage."""
    rng = np.random.default_rng(9100 + seed)
    net = _random_small_net(rng)
    batch = int(rng.choice([1, 15, 16, 17, 100, 4097, 8191, 8200, 20000, 24577, 30001]))
    desc = "-".join(str(l["in"]) for l in net["layers"]) + f"-{net['layers'][-1]['out']}"
    _say(f"small_network_kernel_equals seed={seed} {desc} acts={[l['act'] for l in net['layers']]} head={net['head']} "
         f"{net['wscheme']} {net['in_type']} batch={batch}")
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs[:256])
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    tiles = 1 if batch <= 8192 else (2 if batch <= 24576 else 4)
    assert P.policy_fused_plan(batch) == (16 * tiles, 1, 3 if batch <= 4096 else 2)
    rows = None if batch <= 128 else np.unique(np.concatenate([[0, 15, 16, 63, 64, batch - 17, batch - 1],
                                                                rng.integers(0, batch, 60)]))
    actions, t = U.gpu_forward(P, net, obs)
    U.compare_forward(net, pol, obs, actions, t, rows)
    del t
    plain, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(plain, actions, equal_nan=True)
    general, _ = U.gpu_forward(P, net, obs, taps=False, misalign=1 if net["in_type"] == "f32" else 3)
    assert np.array_equal(general, plain, equal_nan=True)
    P.policy_set_path(2)
    per_layer, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(per_layer, plain, equal_nan=True)
    P.close()


# ------------------------------------------------------------------ HIP graph capture
@pytest.mark.parametrize("name", ["cfg2", "cfg1", "conv_small", "conv_stack_b"])
def test_graph_replays_match_eager(aq, name):
    """The benchmark replays the library's launches from a HIP graph: quantize, forward, actor step and the
    blob hand-off are captured once and replayed several times, with eager work and synchronizations in
    between; every replay must reproduce the eager results bit for bit."""
    _say(f"graph_replays {name}")
    net = _nets()[name]
    params = synth.make_params(net, nonzero_bias=True)
    batch = 260
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, obs)
    P, d = U.gpu_quantize(aq, net, params, ranges)
    Q = aq.Policy(net)
    A = synth.action_dim(net)
    argmax = net["head"] == "argmax"
    shape, dt = ((batch,), torch.int32) if argmax else ((batch, A), torch.float32)
    d_obs = U.to_dev(obs)
    sg = U.to_dev(np.random.default_rng(15).uniform(0, 0.2, batch).astype(np.float32))
    blob = torch.zeros(P.policy_blob_size(), dtype=torch.uint8, device=U.DEV)
    out = {k: torch.zeros(shape, dtype=dt, device=U.DEV) for k in ("fwd", "step", "imported")}

    def body():
        P.quantize_params(d[0], d[1], d[2], d[3], ranges)
        P.policy_forward_int8(d_obs, out["fwd"])
        P.policy_step_int8(d_obs, out["step"], 31, 7, sigma=None if argmax else sg, epsilon=0.2)
        P.policy_export_blob(blob)
        Q.policy_import_blob(blob)
        Q.policy_forward_int8(d_obs, out["imported"])

    P.policy_reserve(batch)
    Q.policy_reserve(batch)
    body()
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in out.items()}
    assert torch.equal(eager["fwd"], eager["imported"])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        body()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        body()
    for rep in range(4):
        for v in out.values():
            v.zero_()
        # eager work of the program's own between the replays
        scratch = torch.zeros(shape, dtype=dt, device=U.DEV)
        P.policy_forward_int8(d_obs, scratch)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in out:
            assert torch.equal(out[k], eager[k]), f"replay {rep}: {k}"
        assert P.policy_status() == aq.OK and Q.policy_status() == aq.OK
    P.close()
    Q.close()


# ------------------------------------------------------------------ edge cases and error paths
def test_edges(aq):
    net = synth.net_config("cfg1")
    params = synth.make_params(net)
    obs = synth.make_obs(net, 4)
    P = aq.Policy(net)
    actions = torch.zeros(4, 6, dtype=torch.float32, device=U.DEV)
    with pytest.raises(aq.AqError) as e:
        P.policy_forward_int8(U.to_dev(obs), actions)
    assert e.value.status == aq.ENOTQUANT
    pol, ranges = U.make_oracle(net, params, obs)
    d = U.upload_params(params)
    P.quantize_params(d[0], d[1], d[2], d[3], ranges)
    assert P.policy_status() == aq.OK
    # empty batch: no-op
    P.policy_forward_int8(torch.zeros(0, 17, device=U.DEV), torch.zeros(0, 6, device=U.DEV))
    # observations far outside the calibrated range saturate, NaN takes code 0
    wild = obs.copy()
    wild[0, :] = 1e30
    wild[1, :] = -1e30
    wild[2, 0] = np.nan
    a, t = U.gpu_forward(P, net, wild)
    U.compare_forward(net, pol, wild, a, t)
    # non-finite weights are reported
    bad = [p["w"].copy() for p in params]
    bad[1][3, 5] = np.inf
    P.quantize_params([U.to_dev(x) for x in bad], d[1], d[2], d[3], ranges)
    assert P.policy_status() == aq.ENONFINITE
    # a requantization multiplier that needs a shift beyond 62 is reported, as the oracle does
    huge = [ranges[0], (np.float32(0), np.float32(1e30)), ranges[2]]
    with pytest.raises(ValueError):
        O.OraclePolicy(net).quantize_params(params, huge)
    P.quantize_params(d[0], d[1], d[2], d[3], huge)
    assert P.policy_status() == aq.ERANGE
    P.close()
    # a bias so large that its integer form saturates: folding the zero-point terms into it would leave the
    # int32 range for the channels whose weight codes sum to a positive number; reported, not wrapped
    small = synth.small_net([synth.fc(16, 64, "relu"), synth.fc(64, 4, "none")])
    sp = synth.make_params(small)
    sp[0]["b"][:] = 1e30
    S = aq.Policy(small)
    ds = U.upload_params(sp)
    S.quantize_params(ds[0], ds[1], ds[2], ds[3], [(np.float32(0.0), np.float32(4.0)), (np.float32(0.0), np.float32(1.0))])
    assert S.policy_status() == aq.ERANGE
    S.close()
    # all-zero weights: scale 1, codes 0, actions tanh(0) = 0
    zero = [{"w": np.zeros_like(p["w"]), "b": np.zeros_like(p["b"])} for p in params]
    pol0, r0 = U.make_oracle(net, zero, obs)
    P0, _ = U.gpu_quantize(aq, net, zero, r0)
    U.check_quantized_params(aq, P0, pol0, net)
    a, t = U.gpu_forward(P0, net, obs)
    U.compare_forward(net, pol0, obs, a, t)
    assert not a.any()
    P0.close()
    # shapes that do not chain are refused
    broken = synth.small_net([synth.fc(17, 32, "relu"), synth.fc(33, 6, "none")])
    with pytest.raises(aq.AqError) as e:
        aq.Policy(broken)
    assert e.value.status == aq.ESHAPE
    # layers beyond the int32 accumulation bound (K <= 65536) or the width limit are refused
    for too_big in (synth.small_net([synth.fc(65537, 8, "none")]), synth.small_net([synth.fc(8, (1 << 20) + 1, "none")])):
        with pytest.raises(aq.AqError) as e:
            aq.Policy(too_big)
        assert e.value.status == aq.ESHAPE


# ------------------------------------------------------------------ weights streamed as nibbles
@pytest.mark.parametrize("name,batch,wbits", [("paper_fc2048", 1, 4), ("paper_fc2048", 16, 4), ("paper_fc2048", 40, 3),
                                              ("paper_fc2048", 300, 4), ("cfg5", 96, 4), ("cfg2", 33, 2),
                                              ("cfg4", 8, 4), ("cfg4", 70, 4)])
def test_few_row_layers_stream_nibble_weights(aq, name, batch, wbits):
    """Policies of at most 4 bits with per-channel symmetric weights: the few-row layer kernel reads the codes two
    per byte and expands them in registers.  Every stage against the oracle (whose n-bit codes are the same
    integers), with and without taps, at 16- and 32-row tiles, through a blob hand-off, and identical to the same
    policy read from its 8-bit containers (launch plan 2)."""
    _say(f"few_row_layers_stream_nibble_weights {name} batch={batch} wbits={wbits}")
    net = dict(synth.net_config(name), wbits=wbits)
    # (convolutions keep to the 8-bit containers; cfg4's first fully connected layer has wave shares of 13 k-steps,
    # the variant with sixteen requests in flight)
    nl = sum(1 for layer in net["layers"] if layer["kind"] == "fc")
    params = synth.make_params(net, nonzero_bias=True)
    obs = synth.make_obs(net, batch)
    pol, ranges = U.make_oracle(net, params, synth.make_obs(net, 64 if name != "cfg4" else 8))
    P, _ = U.gpu_quantize(aq, net, params, ranges)
    U.check_quantized_params(aq, P, pol, net)
    P.policy_set_path(2)
    assert P.policy_subbyte_layers(batch) == 0     # a plan to choose, not the default
    from_bytes, _ = U.gpu_forward(P, net, obs, taps=False)
    P.policy_set_path(4)
    assert P.policy_subbyte_layers(batch) == nl
    assert P.policy_subbyte_layers(8192) == 0      # beyond the few-row kernel: 8-bit containers
    actions, t = U.gpu_forward(P, net, obs)
    assert np.array_equal(from_bytes, actions, equal_nan=True)
    U.compare_forward(net, pol, obs, actions, t)
    del t
    plain, _ = U.gpu_forward(P, net, obs, taps=False)
    assert np.array_equal(plain, actions, equal_nan=True)
    # the hand-off of the policy as a blob (plain and packed) rebuilds the nibble copy on the other side
    for packed in (False, True):
        Q = aq.Policy(net)
        if packed:
            blob = torch.zeros(P.policy_packed_blob_size(), dtype=torch.uint8, device=U.DEV)
            P.policy_export_packed_blob(blob)
            Q.policy_import_packed_blob(blob)
        else:
            blob = torch.zeros(P.policy_blob_size(), dtype=torch.uint8, device=U.DEV)
            P.policy_export_blob(blob)
            Q.policy_import_blob(blob)
        assert Q.policy_status() == aq.OK
        Q.policy_set_path(4)
        assert Q.policy_subbyte_layers(batch) == nl
        again, _ = U.gpu_forward(Q, net, obs, taps=False)
        assert np.array_equal(again, plain, equal_nan=True)
        Q.close()
    with pytest.raises(aq.AqError) as e:
        P.policy_set_path(5)
    assert e.value.status == aq.EINVAL
    P.close()
    # the same precision with per-tensor asymmetric weights, and 8-bit policies, keep to the 8-bit containers
    for other in (dict(net, wscheme="tensor_asym_u8"), dict(net, wbits=8), dict(net, wbits=5)):
        R = aq.Policy(other)
        R.policy_set_path(4)
        assert R.policy_subbyte_layers(batch) == 0
        R.close()


# ------------------------------------------------------------------ measurement aids
def test_stream_reference_moves_the_top_byte_of_every_value(aq):
    _say("stream_reference")
    n = 4 * 70001
    src = np.random.default_rng(31).standard_normal(n).astype(np.float32)
    d_src = U.to_dev(src)
    dst = torch.zeros(n, dtype=torch.uint8, device=U.DEV)
    aq.stream_reference(d_src, n, dst)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy(), (src.view(np.uint32) >> 24).astype(np.uint8))


@pytest.mark.parametrize("ksteps,stream", [(4, 1), (64, 1), (200, 1), (72, 0)])
def test_mfma_loop_reference_accumulators(aq, ksteps, stream):
    """The timing loop computes what it says: workgroup 0's accumulators equal the integer products of the
    weight tiles and activation rows it walked (so the rate it is timed at is the rate of real MFMAs on the
    operands given)."""
    _say(f"mfma_loop_reference ksteps={ksteps} stream={stream}")
    rng = np.random.default_rng(32)
    w = rng.integers(-127, 128, (16, 64, 64, 16), dtype=np.int8)   # [tile][k-step][lane][16 bytes]
    x = rng.integers(-128, 128, (64, 1024), dtype=np.int8)
    d_w, d_x = U.to_dev(w), U.to_dev(x)
    acc = torch.full((32768,), 7, dtype=torch.int32, device=U.DEV)
    aq.mfma_loop_reference(d_w, d_x, ksteps, stream, 3, acc)
    torch.cuda.synchronize()
    got = acc.cpu().numpy().reshape(8, 2, 2, 16, 64)            # [wave][feature tile][row tile][register][lane]
    # a tile's k-step as a 32 x 32 matrix [feature][k]: lane l holds feature l % 32, k = 16 * (l // 32) .. + 15
    wt = w.reshape(16, 64, 2, 32, 16).transpose(0, 1, 3, 2, 4).reshape(16, 64, 32, 32).astype(np.int64)
    xs = x.astype(np.int64)
    for wave in range(8):
        for ft in range(2):
            for rt in range(2):
                ref = np.zeros((32, 32), dtype=np.int64)        # [feature][row]
                for k in range(ksteps):
                    ks = k % 64 if stream else k % 4             # weights kept in registers: the first four k-steps
                    kk = k % 32
                    ref += wt[2 * wave + ft, ks] @ xs[32 * rt:32 * rt + 32, 32 * kk:32 * kk + 32].T
                lane = np.arange(64)
                for r in range(16):
                    feat = 8 * (r // 4) + 4 * (lane // 32) + r % 4
                    assert np.array_equal(got[wave, ft, rt, r], ref[feat, lane % 32].astype(np.int32)), (wave, ft, rt, r)
    # argument errors
    with pytest.raises(aq.AqError) as e:
        aq.mfma_loop_reference(d_w, d_x, 6, 1, 1, acc)
    assert e.value.status == aq.EINVAL
    with pytest.raises(aq.AqError) as e:
        aq.mfma_loop_reference(d_w, d_x, 8, 1, 0, acc)
    assert e.value.status == aq.EINVAL
