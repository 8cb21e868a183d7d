"""Do the oracle's pins notice a mistake?  Each case below plants one plausible slip (a dropped term, a
wrong sign, index, tie rule or constant) in a copy of the oracle's C source, builds that copy on the CPU
and runs tests/test_oracle_pins.py against it in a child process: the pins must fail.  The unaltered
copy must pass, so a failure comes from the planted mistake and not from the harness."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import build as orc_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text in the source (must occur exactly once), replacement)
MUTANTS = [
    ("unaltered", None, None),
    # Sec. 3.2 quantizer
    ("range_sign", "float s = (hi - lo) / qdenom;", "float s = (hi + lo) / qdenom;"),
    ("zero_point_sign", "*zp = rint_clamp(-lo / s, 0, qmax);", "*zp = rint_clamp(lo / s, 0, qmax);"),
    ("zero_point_dropped_from_codes", "q[i] = (uint8_t)(rint_clamp(w[i] / scale, -zp, qmax - zp) + zp);",
     "q[i] = (uint8_t)(rint_clamp(w[i] / scale, 0, qmax));"),
    ("ties_away_from_zero", "float r = rintf(v);", "float r = roundf(v);"),
    ("dequant_zero_point_sign", "w[i] = scale * (float)((int32_t)q[i] - zp);",
     "w[i] = scale * (float)((int32_t)q[i] + zp);"),
    ("channel_scale_128", "float s = m / (float)qw;", "float s = m / (float)(qw + 1);"),
    ("channel_abs_dropped", "float a = fabsf(v);", "float a = v;"),
    ("channel_dequant_scale_of_the_column", "w[r * cols + c] = scales[r] * (float)q[r * cols + c];",
     "w[r * cols + c] = scales[c % rows] * (float)q[r * cols + c];"),
    # layer constants
    ("multiplier_inverted", "double M = sw / (double)s_out;", "double M = sw * (double)s_out;"),
    ("shift_off_by_one", "int32_t r = 31 - e;", "int32_t r = 30 - e;"),
    ("bias_scale_single_factor", "double bq = rint((double)bias[n] / sw);",
     "double bq = rint((double)bias[n] / (double)s_in);"),
    # integer accumulators
    ("fc_input_zero_point_dropped", "s += (int64_t)((int32_t)a[b * K + k] - z_a) *",
     "s += (int64_t)((int32_t)a[b * K + k]) *"),
    ("fc_weight_zero_point_dropped", "(int64_t)((int32_t)w[n * K + k] - z_w[n]);", "(int64_t)((int32_t)w[n * K + k]);"),
    ("fc_weights_transposed", "(int64_t)((int32_t)w[n * K + k] - z_w[n]);",
     "(int64_t)((int32_t)w[k * N + n] - z_w[n]);"),
    ("fc_bias_dropped", "int64_t s = bias_q[n];", "int64_t s = 0;"),
    ("conv_stride_ignored_in_y", "int32_t av = a[((b * H + oy * stride + ky) * W + ox * stride + kx) * C + ci];",
     "int32_t av = a[((b * H + oy + ky) * W + ox * stride + kx) * C + ci];"),
    ("conv_kernel_axes_swapped", "int32_t wv = w[((co * kh + ky) * kw + kx) * C + ci];",
     "int32_t wv = w[((co * kw + kx) * kh + ky) * C + ci];"),
    ("conv_weight_zero_point_dropped", "s += (int64_t)(av - z_a) * (int64_t)(wv - z_w[co]);",
     "s += (int64_t)(av - z_a) * (int64_t)(wv);"),
    # requantization
    ("requant_truncates", "(int64_t)M0[n] + ((int64_t)1 << (rshift[n] - 1));", "(int64_t)M0[n] + 0;"),
    ("requant_relu_floor_dropped", "int64_t lo = relu ? z_out : 0;", "int64_t lo = 0;"),
    ("requant_zero_point_sign", "int64_t v = (p >> rshift[n]) + z_out;", "int64_t v = (p >> rshift[n]) - z_out;"),
    # LayerNorm + tanh on the 8-bit path
    ("ln_unbiased_variance", "        var /= (double)N;\n        double inv = 1.0 / sqrt(var + eps);\n        for (int64_t n = 0; n < N; ++n) {\n            double x = (double)((float)acc",
     "        var /= (double)(N - 1);\n        double inv = 1.0 / sqrt(var + eps);\n        for (int64_t n = 0; n < N; ++n) {\n            double x = (double)((float)acc"),
    ("ln_offset_dropped", "double y = (x - mu) * inv * (double)gamma[n] + (double)beta[n];",
     "double y = (x - mu) * inv * (double)gamma[n];"),
    ("ln_tanh_dropped", "float t = (float)tanh(y);", "float t = (float)y;"),
    # heads
    ("argmax_last_index_on_ties", "if (y[b * N + n] > y[b * N + best]) best = (int32_t)n;",
     "if (y[b * N + n] >= y[b * N + best]) best = (int32_t)n;"),
    # exploration
    ("philox_nine_rounds", "for (int round = 0; round < 10; ++round) {", "for (int round = 0; round < 9; ++round) {"),
    ("philox_key_schedule_from_round_0", "if (round > 0) {", "if (round >= 0) {"),
    ("philox_words_swapped", "const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;",
     "const uint32_t n0 = (uint32_t)(p0 >> 32) ^ c1 ^ k0;"),
    ("box_muller_halves_swapped", "(j % 2 == 0) ? rad * cos(two_pi * u2) : rad * sin(two_pi * u2);",
     "(j % 2 == 0) ? rad * sin(two_pi * u2) : rad * cos(two_pi * u2);"),
    ("box_muller_variance_halved", "const double rad = sqrt(-2.0 * log(u1));", "const double rad = sqrt(-1.0 * log(u1));"),
    ("box_muller_pairs_share_words", "const double u2 = (double)(r[2 * pair + 1] >> 8) / 16777216.0;",
     "const double u2 = (double)(r[1] >> 8) / 16777216.0;"),
    ("noise_not_scaled_per_actor", "(double)sigma[b] * z);", "(double)sigma[0] * z);"),
    ("eps_greedy_uses_wrong_word", "idx[b] = (int32_t)(((uint64_t)r[1] * (uint64_t)A) >> 32);",
     "idx[b] = (int32_t)(((uint64_t)r[0] * (uint64_t)A) >> 32);"),
    # fp32 / fp64 comparator network
    ("f64_fc_bias_dropped", "double s = (double)bias[n];", "double s = 0.0;"),
    ("f64_conv_stride_ignored_in_x", "s += x[((b * H + oy * stride + ky) * W + ox * stride + kx) * C + ci] *",
     "s += x[((b * H + oy * stride + ky) * W + ox + kx) * C + ci] *"),
    ("f64_relu_sign", "if (x[i] < 0.0) x[i] = 0.0;", "if (x[i] > 0.0) x[i] = 0.0;"),
    ("f64_ln_eps_outside_root", "        double inv = 1.0 / sqrt(var + eps);\n        for (int64_t n = 0; n < N; ++n) x[b * N + n] =",
     "        double inv = 1.0 / (sqrt(var) + eps);\n        for (int64_t n = 0; n < N; ++n) x[b * N + n] ="),
    # binary16 rounding
    ("fp16_ties_up", "return fmod(f, 2.0) == 0.0 ? f : f + 1.0;", "return f + 1.0;"),
    ("fp16_no_gradual_underflow", "if (exp2 < -14) exp2 = -14;", "if (exp2 < -24) exp2 = -24;"),
    ("fp16_overflow_threshold", "if (r >= 65520.0) r = INFINITY;", "if (r > 65536.0) r = INFINITY;"),
    ("fp16_eleven_fraction_bits", "double ulp = ldexp(1.0, exp2 - 10);", "double ulp = ldexp(1.0, exp2 - 11);"),
]


# The same for the layer-by-layer chain in oracle/policy.py (which operator follows which, which scale and
# zero-point go where, what is rounded to binary16): (name, text occurring exactly once, replacement)
CHAIN_MUTANTS = [
    ("chain_unaltered", None, None),
    ("fp32_relu_skipped", "                x = c_relu_f64(x)\n", "                pass\n"),
    ("fp32_tanh_after_layernorm_skipped",
     'x = c_tanh_f64(c_layernorm_f64(x, p["gamma"], p["beta"], self.net["ln_eps"]))',
     'x = c_layernorm_f64(x, p["gamma"], p["beta"], self.net["ln_eps"])'),
    ("fp32_tanh_head_skipped", "out = c_tanh_f64(y).astype(np.float32)", "out = y.astype(np.float32)"),
    ("fp16_weights_not_rounded", 'w16, b16 = r16(p["w"]), r16(p["b"])', 'w16, b16 = p["w"], r16(p["b"])'),
    ("fp16_bias_not_rounded", 'w16, b16 = r16(p["w"]), r16(p["b"])', 'w16, b16 = r16(p["w"]), p["b"]'),
    ("fp16_layer_output_not_rounded", "            y = r16(pre)\n", "            y = pre\n"),
    ("fp16_layernorm_output_not_rounded",
     'y = r16(c_layernorm_f64(y, r16(p["gamma"]), r16(p["beta"]), self.net["ln_eps"]))',
     'y = c_layernorm_f64(y, r16(p["gamma"]), r16(p["beta"]), self.net["ln_eps"])'),
    ("fp16_observation_not_rounded", "x = r16(obs) if start_x is None else", "x = np.asarray(obs, np.float32) if start_x is None else"),
    ("fp16_head_not_rounded", 'taps["actions"] = r16(c_tanh_f64(y))', 'taps["actions"] = c_tanh_f64(y)'),
    ("requant_uses_input_scale", "s_out = act_q[i + 1][0] if requant else np.float32(0.0)",
     "s_out = act_q[i][0] if requant else np.float32(0.0)"),
    ("requant_uses_input_zero_point", '"z_out": act_q[i + 1][1] if i < nl - 1 else None',
     '"z_out": act_q[i][1] if i < nl - 1 else None'),
    ("weights_quantized_at_8_bits_whatever_n", "codes = c_quantize_asym(w, s, z, wmax)", "codes = c_quantize_asym(w, s, z, 255)"),
    ("int8_fc_ignores_input_zero_point",
     'acc = c_fc_acc(a.reshape(a.shape[0], -1), q["z_in"], q["codes"], q["z_w"], q["bias_q"])',
     'acc = c_fc_acc(a.reshape(a.shape[0], -1), 0, q["codes"], q["z_w"], q["bias_q"])'),
    ("int8_relu_flag_dropped", 'c_requant(acc, q["M0"], q["rshift"], q["z_out"], l["act"] == "relu")',
     'c_requant(acc, q["M0"], q["rshift"], q["z_out"], False)'),
    ("int8_tanh_head_skipped", '                    taps["actions"] = c_tanh_f32(y)\n', '                    taps["actions"] = y\n'),
    ("int8_layernorm_uses_next_layers_gain", 'c_ln_tanh(acc, q["m"], q["gamma"], q["beta"], self.net["ln_eps"], q["s_out"], q["z_out"])',
     'c_ln_tanh(acc, q["m"], q["beta"], q["gamma"], self.net["ln_eps"], q["s_out"], q["z_out"])'),
]

# loaded by the child pytest with -p: installs the altered copy as oracle.policy before the pins import it
PLUGIN = '''
import importlib.util, os, sys
def pytest_configure(config):
    import oracle
    spec = importlib.util.spec_from_file_location("oracle.policy", os.environ["ACTORQ_ORACLE_POLICY_COPY"])
    m = importlib.util.module_from_spec(spec)
    sys.modules["oracle.policy"] = m
    spec.loader.exec_module(m)
    oracle.policy = m
'''


def _run_pins(lib, policy_copy=None, plugin_dir=None):
    env = dict(os.environ, OMP_NUM_THREADS="2")
    cmd = [sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q", "-p",
           "no:cacheprovider"]
    if lib:
        env["ACTORQ_ORACLE_LIB"] = lib
    if policy_copy:
        env["ACTORQ_ORACLE_POLICY_COPY"] = policy_copy
        env["PYTHONPATH"] = plugin_dir + os.pathsep + env.get("PYTHONPATH", "")
        cmd += ["-p", "actorq_policy_copy_plugin"]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return r.returncode, (r.stdout + r.stderr)[-1500:]


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Builds every altered copy and runs the pins on each, a few at a time."""
    work = tmp_path_factory.mktemp("mutants")
    src = open(orc_build.SRC).read()
    libs = {}
    for name, old, new in MUTANTS:
        text = src
        if old is not None:
            assert src.count(old) == 1, f"{name}: the text to alter occurs {src.count(old)} times"
            text = src.replace(old, new)
        c = str(work / f"{name}.c")
        open(c, "w").write(text)
        libs[name] = orc_build.build(True, c, str(work / f"{name}.so"))
    with ThreadPoolExecutor(max_workers=4) as pool:
        out = dict(zip(libs, pool.map(_run_pins, libs.values())))
    return out


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_pins_notice(outcomes, name):
    rc, tail = outcomes[name]
    if name == "unaltered":
        assert rc == 0, tail
    else:
        assert rc != 0, f"no pin fails when the oracle has the mistake '{name}'"


@pytest.fixture(scope="module")
def chain_outcomes(tmp_path_factory):
    work = tmp_path_factory.mktemp("chain_mutants")
    open(work / "actorq_policy_copy_plugin.py", "w").write(PLUGIN)
    src = open(os.path.join(ROOT, "oracle", "policy.py")).read()
    copies = {}
    for name, old, new in CHAIN_MUTANTS:
        text = src
        if old is not None:
            assert src.count(old) == 1, f"{name}: the text to alter occurs {src.count(old)} times"
            text = src.replace(old, new)
        copies[name] = str(work / f"{name}.py")
        open(copies[name], "w").write(text)
    with ThreadPoolExecutor(max_workers=4) as pool:
        out = dict(zip(copies, pool.map(lambda c: _run_pins(None, c, str(work)), copies.values())))
    return out


@pytest.mark.parametrize("name", [m[0] for m in CHAIN_MUTANTS])
def test_pins_notice_chain_mistakes(chain_outcomes, name):
    rc, tail = chain_outcomes[name]
    if name == "chain_unaltered":
        assert rc == 0, tail
    else:
        assert rc != 0, f"no pin fails when the oracle's chain has the mistake '{name}'"
