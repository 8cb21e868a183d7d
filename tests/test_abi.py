"""CPU-side checks of the boundary: the C-ABI library loads and exports every symbol the header
declares; the binding's structs match the header's layout.  No compute call is made."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "actorq.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_1910_01055_amd import binding
    lib = binding.load()
    names = _declared()
    assert "aq_quantize_params" in names and "aq_policy_forward_int8" in names and "aq_policy_forward_fp32" in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in actorq.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_struct_layouts_match_header():
    from paper_1910_01055_amd import binding as b
    assert ctypes.sizeof(b.AqLayer) == 9 * 4
    assert ctypes.sizeof(b.AqRange) == 8
    assert ctypes.sizeof(b.AqNet) == 4 + 4 + 8 + 4 * 4 + 4 + 4  # int32, pad, pointer, 4 x int32, float, int32
    assert ctypes.sizeof(b.AqTaps) == 5 * 8
    assert b.MAX_LAYERS == int(re.search(r"#define AQ_MAX_LAYERS (\d+)", open(HEADER).read()).group(1))


def test_status_strings_and_argument_errors_without_gpu():
    from paper_1910_01055_amd import binding as b
    lib = b.load()
    assert lib.aq_status_string(0) == b"ok"
    assert lib.aq_policy_create(None, None) == b.EINVAL
    assert lib.aq_policy_destroy(None) == b.EINVAL
    assert lib.aq_quantize_tensor(None, 1, 4, 0, 255, None, None, None, None, None) == b.EINVAL
    assert lib.aq_policy_blob_size(None, None) == b.EINVAL
    assert lib.aq_policy_export_blob(None, None, 0, None) == b.EINVAL
    assert lib.aq_policy_import_blob(None, None, 0, None) == b.EINVAL
    assert lib.aq_stream_reference(None, 4, None, None) == b.EINVAL
    assert lib.aq_mfma_loop_reference(None, None, 4, 1, 1, None, None) == b.EINVAL
    assert lib.aq_calibrate_fp32(None, None, 1, None, None) == b.EINVAL
    assert lib.aq_policy_set_params_fp32(None, None, None, None, None, None) == b.EINVAL
    assert lib.aq_policy_forward_fp32(None, None, 1, None, None) == b.EINVAL
    assert lib.aq_policy_forward_int8_static(None, None, 1, None, None) == b.EINVAL
    assert lib.aq_policy_fused_plan(None, 1, None, None, None) == b.EINVAL
    assert lib.aq_policy_subbyte_layers(None, 1, None) == b.EINVAL
    assert lib.aq_status_string(8).startswith(b"needs more scratch")


def test_synth_configs_match_the_stated_workloads():
    from paper_1910_01055_amd import synth
    assert synth.macs_per_sample(synth.net_config("cfg1")) == 71424
    assert synth.macs_per_sample(synth.net_config("cfg2")) == 153600
    assert synth.macs_per_sample(synth.net_config("cfg4")) == 9352192
    assert synth.macs_per_sample(synth.net_config("cfg5")) == 2424832
    net = synth.net_config("cfg4")
    assert synth.layer_out_shape(net["layers"][2]) == (7, 7, 64) and net["layers"][3]["in"] == 3136
    a = synth.make_obs(synth.net_config("cfg2"), 4)
    b2 = synth.make_obs(synth.net_config("cfg2"), 4)
    assert (a == b2).all() and a.dtype.name == "float32"


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more exits with a message instead of running."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and not r.stdout.strip()
