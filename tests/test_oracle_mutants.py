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


def _run_pins(lib):
    env = dict(os.environ, ACTORQ_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return r.returncode, r.stdout[-1500:]


@pytest.fixture(scope="module")
def verdicts(tmp_path_factory):
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
def test_pins_notice(verdicts, name):
    rc, tail = verdicts[name]
    if name == "unaltered":
        assert rc == 0, tail
    else:
        assert rc != 0, f"no pin fails when the oracle has the mistake '{name}'"
