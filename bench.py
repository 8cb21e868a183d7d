#!/usr/bin/env python3
"""Benchmark of the ActorQ 8-bit policy-inference path on one MI355X.

A step = one actor inference call on a batch of 4096 observations through the D4PG-style int8 MLP
(observation quantize -> 4 int8 layers with int32 accumulation, LayerNorm+tanh / requantize+ReLU
epilogues -> tanh actions), with the quantizer block (fp32 weights -> int8 policy) re-run once
every PULL_EVERY steps inside the timed region, as an actor that pulls a fresh policy from the
learner does.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

DEV = "cuda:0"
PULL_EVERY = 100           # actor steps between model pulls (the paper's smaller pull frequency)
INT8_PEAK_TOPS = 5000.0    # MI355X dense int8 MFMA, TOP/s
FP16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 MFMA, TFLOP/s
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the whole-network kernel on the headline workload, from the FETCH_SIZE and WRITE_SIZE
# hardware counters scaled by what they read on a plain 64 MiB copy (the rocprofv3 summary of this kernel under
# profiles/), together with the hash of the kernel's sources at the time the counters were taken: when the
# sources have changed since, the figure is reported as null.
FUSED_TRAFFIC = {"bytes_per_launch": 3154954,
                 "sources_sha256": "75b6ad5c7eaa211c0225db8b01d4072071b41805644b4b3b970418fafbee3eab"}
FUSED_SOURCES = ("rows16_mlp.hpp", "rows16_mlp.hip", "int8_device.hpp", "common.hpp", "explore_device.hpp")


def _fused_sources_hash():
    import hashlib
    h = hashlib.sha256()
    for f in FUSED_SOURCES:
        with open(os.path.join(ROOT, "paper_1910_01055_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def action_error_figures(a_q, a_f):
    """8-bit policy actions against fp32 policy actions on the same observations: largest and mean absolute
    difference and the signal-to-quantization-noise ratio in dB."""
    import numpy as np
    a_q = np.asarray(a_q, np.float64)
    a_f = np.asarray(a_f, np.float64)
    d = a_q - a_f
    return {"max_abs": float(np.abs(d).max()), "mean_abs": float(np.abs(d).mean()),
            "sqnr_db": float(10.0 * np.log10((a_f ** 2).sum() / max((d ** 2).sum(), 1e-300)))}


def _events_ms(torch, fn, n):
    """Average ms per fn() call, launched one by one from the host (includes host launch cost)."""
    st = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(n):
        fn()
    e1.record(st)
    e1.synchronize()
    return e0.elapsed_time(e1) / n


_USE_GRAPHS = True


def _capture(torch, body):
    """Records body() into a HIP graph (the library launches on torch's current stream, which is the
    capture stream inside torch.cuda.graph).  Returns None if capture is not possible."""
    if not _USE_GRAPHS:
        return None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            body()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            body()
        return g
    except Exception as e:  # noqa: BLE001
        print(f"bench.py: graph capture unavailable ({e}); timing eager launches", file=sys.stderr)
        return None


def _graph_ms(torch, fn, n, replays=5):
    """Average ms per fn() call with n calls replayed from one HIP graph: the device-side rate,
    free of per-launch host cost.  Falls back to eager launches."""
    g = _capture(torch, lambda: [fn() for _ in range(n)])
    if g is None:
        return _events_ms(torch, fn, n)
    g.replay()
    torch.cuda.synchronize()
    st = torch.cuda.current_stream()
    times = []
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(replays):
            g.replay()
        e1.record(st)
        e1.synchronize()
        times.append(e0.elapsed_time(e1) / (replays * n))
    return sorted(times)[2]  # median of 5 repeats


def forward_workload(torch, aq, synth, name, batch, iters, warm=20, report_error=False):
    """Average launch time of the 8-bit forward on `name` at `batch` (HIP events around back-to-back launches)."""
    net = synth.net_config(name)
    params = synth.make_params(net)
    obs = synth.make_obs(net, batch)
    P = aq.Policy(net)
    w, b, g, be = aq.upload_params(params, DEV)
    A = synth.action_dim(net)
    d_obs = aq.to_dev(obs, DEV)
    argmax = net["head"] == "argmax"
    new_actions = lambda: torch.zeros((batch,) if argmax else (batch, A), dtype=torch.int32 if argmax else torch.float32,
                                      device=DEV)
    act, act32, act16 = new_actions(), new_actions(), new_actions()
    calib = min(batch, 4096)
    P.policy_set_params_fp32(w, b, g, be)           # the learner's parameters, kept for the fp32 actor
    ranges = P.calibrate_fp32(d_obs[:calib])        # GPU min/max calibration of the activation ranges
    P.quantize_params(w, b, g, be, ranges)
    assert P.policy_status() == aq.OK
    P.policy_reserve(batch)
    fwd = lambda: P.policy_forward_int8(d_obs, act)
    for _ in range(warm):
        fwd()
    torch.cuda.synchronize()
    ms_eager = sorted(_events_ms(torch, fwd, iters) for _ in range(5))[2]
    ms = _graph_ms(torch, fwd, min(iters, 200))
    f32 = lambda: P.policy_forward_fp32(d_obs, act32)
    f32()
    torch.cuda.synchronize()
    ms32 = _events_ms(torch, f32, max(2, iters // 20))
    # the half-precision actor (q = 16 in the paper's run-time breakdown) on the same inputs
    P.convert_params_fp16(w, b, g, be)
    f16 = lambda: P.policy_forward_fp16(d_obs, act16)
    for _ in range(3):
        f16()
    torch.cuda.synchronize()
    ms16 = _graph_ms(torch, f16, min(iters, 50))
    ops = 2.0 * synth.macs_per_sample(net) * batch
    # algorithmic HBM bytes: observations in, actions out, 8-bit weights once
    n_w = sum(int(p["w"].size) for p in params)
    hbm = float(obs.nbytes + act.numel() * act.element_size() + n_w)
    rows, tiles, kind = P.policy_fused_plan(batch)
    kind_name = {0: "", 1: ", pipelined (k_mlp_wide)", 2: ", small-network kernel (k_mlp_rows16)",
                 3: ", small-network kernel (k_mlp_rows16, a workgroup alone on its CU)"}[kind]
    out = {"workload": f"{name} batch {batch}", "us_per_launch": ms * 1e3, "inferences_per_s": batch / (ms * 1e-3),
           "tops": ops / (ms * 1e-3) / 1e12, "frac_int8_mfma_peak": ops / (ms * 1e-3) / 1e12 / INT8_PEAK_TOPS,
           "GBps_algorithmic": hbm / (ms * 1e-3) / 1e9, "frac_hbm_peak": hbm / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "us_per_launch_eager": ms_eager * 1e3, "fp32_actor_us_per_launch": ms32 * 1e3,
           "fp16_actor_us_per_launch": ms16 * 1e3, "fp16_actor_tflops": ops / (ms16 * 1e-3) / 1e12,
           "fp16_actor_frac_fp16_mfma_peak": ops / (ms16 * 1e-3) / 1e12 / FP16_PEAK_TFLOPS,
           "launch_plan": f"fused kernel{kind_name}, {rows} rows per workgroup, {tiles} feature tile(s) per wavefront" if rows
           else "one launch per layer"}
    if report_error:
        # quantization error of the actions: the 8-bit and the half-precision actor against the fp32 actor on
        # the same observations (the paper gives this only qualitatively, App. C: the value is reported, not pinned)
        fwd()
        f32()
        f16()
        torch.cuda.synchronize()
        a8, a32, a16 = act.cpu().numpy(), act32.cpu().numpy(), act16.cpu().numpy()
        if argmax:
            out["action_agreement_int8_vs_fp32"] = float((a8 == a32).mean())
            out["action_agreement_fp16_vs_fp32"] = float((a16 == a32).mean())
        else:
            out["action_error_int8_vs_fp32"] = action_error_figures(a8, a32)
            out["action_error_fp16_vs_fp32"] = action_error_figures(a16, a32)
    return out, (P, w, b, g, be, ranges, d_obs, act, net, params, obs)


def quantize_workload(torch, aq, synth, scheme, iters=30, n_buf=40, repeat=1, reference=False):
    """Learner->actor weight quantize pass over 4M fp32 params (times `repeat`: the same values tiled
    into a larger tensor, for the asymptotic rate), rotating over distinct buffers so that the
    source comes from HBM, not from the 256 MB last-level cache."""
    n = synth.QUANT_TENSOR_ELEMS * repeat
    src = aq.to_dev(synth.quant_tensor(), DEV)
    if repeat > 1:
        src = src.reshape(-1).repeat(repeat)
    srcs = [src.clone() for _ in range(n_buf)]
    rows, cols = (1, n) if scheme == "tensor_asym_u8" else (2048 * repeat, 2048)
    dsts = [torch.empty(n, dtype=torch.uint8, device=DEV) for _ in range(n_buf)]
    scale = torch.empty(rows, dtype=torch.float32, device=DEV)
    zp = torch.empty(rows, dtype=torch.int32, device=DEV)
    ws = torch.zeros(4096, dtype=torch.int32, device=DEV)
    i = [0]

    def one():
        k = i[0] % n_buf
        i[0] += 1
        if reference:  # the same bytes moved with no arithmetic: the ceiling at this size
            aq.stream_reference(srcs[k], n, dsts[k])
        else:
            aq.quantize_tensor(srcs[k], rows, cols, scheme, 255, dsts[k], scale, zp, ws)
    for _ in range(n_buf):
        one()
    torch.cuda.synchronize()
    ms_eager = sorted(_events_ms(torch, one, iters) for _ in range(5))[2]
    i[0] = 0
    ms = _graph_ms(torch, one, n_buf)   # one pass over all the distinct buffers per replay
    gbs = 5.0 * n / (ms * 1e-3) / 1e9
    what = "plain streaming of the same bytes (no arithmetic)" if reference else scheme
    return {"workload": f"quantize {4 * repeat}M fp32 params, {what}, {n_buf} rotating buffers (HBM-resident source)",
            "us_per_call": ms * 1e3, "us_per_call_eager": ms_eager * 1e3, "GBps_algorithmic": gbs,
            "frac_hbm_peak": gbs / HBM_PEAK_GBS}


def mfma_loop_workload(torch, aq, operands, stream_weights=True, ksteps=2048):
    """What the matrix cores sustain in the wide whole-network kernel's k-step loop with nothing around it (no
    observation load, no epilogue, no barrier): one workgroup per CU, per CU and k-step 32 MFMAs on 16 KiB of
    streamed weights.  The clock under matrix load depends on the operand bits, so three operand sets: zeros,
    codes distributed like cfg5's (Gaussian weight codes, post-ReLU activations), uniformly random bytes."""
    import numpy as np
    rng = np.random.default_rng(41)
    if operands == "zeros":
        w = np.zeros(1 << 20, dtype=np.int8)
        x = np.zeros(64 * 1024, dtype=np.int8)
    elif operands == "cfg5-like codes":
        w = np.clip(np.rint(rng.standard_normal(1 << 20) * 38.0), -127, 127).astype(np.int8)
        x = (np.clip(np.rint(np.maximum(rng.standard_normal(64 * 1024), 0.0) * 64.0), 0, 255) - 128).astype(np.int8)
    else:
        w = rng.integers(-128, 128, 1 << 20, dtype=np.int8)
        x = rng.integers(-128, 128, 64 * 1024, dtype=np.int8)
    d_w, d_x = aq.to_dev(w, DEV), aq.to_dev(x, DEV)
    acc = torch.zeros(32768, dtype=torch.int32, device=DEV)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    ms = _graph_ms(torch, lambda: aq.mfma_loop_reference(d_w, d_x, ksteps, stream_weights, cus, acc), 4)
    tops = cus * ksteps * 32 * 65536.0 / (ms * 1e-3) / 1e12
    return {"workload": f"int8 MFMA k-step loop alone, {operands}, weights " +
                        ("streamed (16 KiB per CU and k-step)" if stream_weights else "kept in registers"),
            "us_per_call": ms * 1e3, "int8_TOPs": tops, "frac_int8_mfma_peak": tops / INT8_PEAK_TOPS}


def subbyte_workload(torch, aq, synth, name, batch, iters=200):
    """A 4-bit policy (per-channel symmetric codes in [-7, 7]) on the one-launch-per-layer plan: its weights read
    from the 8-bit containers (plan 2) against the same weights streamed as nibbles and expanded in registers
    (plan 4); identical integers, so the actions must be equal."""
    net = dict(synth.net_config(name), wbits=4)
    params = synth.make_params(net)
    obs = synth.make_obs(net, batch)
    P = aq.Policy(net)
    w, b, g, be = aq.upload_params(params, DEV)
    d_obs = aq.to_dev(obs, DEV)
    P.policy_set_params_fp32(w, b, g, be)
    P.quantize_params(w, b, g, be, P.calibrate_fp32(d_obs))
    P.policy_reserve(batch)
    acts, us = [], []
    for plan in (2, 4):
        P.policy_set_path(plan)
        act = torch.zeros(batch, synth.action_dim(net), dtype=torch.float32, device=DEV)
        fwd = lambda: P.policy_forward_int8(d_obs, act)
        for _ in range(10):
            fwd()
        torch.cuda.synchronize()
        us.append(_graph_ms(torch, fwd, iters) * 1e3)
        acts.append(act)
    out = {"workload": f"{name} batch {batch}, 4-bit weights, one launch per layer",
           "us_per_launch_8bit_containers": us[0], "us_per_launch_nibbles": us[1],
           "layers_streaming_nibbles": P.policy_subbyte_layers(batch), "actions_equal": bool(torch.equal(acts[0], acts[1]))}
    P.close()
    return out


def blob_workload(torch, aq, synth, name, wbits=8):
    """Learner -> actor hand-off of a quantized policy as one packed blob: export from one handle, import
    into another (device to device, no repacking), next to the cost of quantizing the fp32 parameters.
    With wbits < 8 the weight codes also travel sub-byte (n-bit fields, expanded on import)."""
    net = dict(synth.net_config(name), wbits=wbits)
    params = synth.make_params(net)
    obs = synth.make_obs(net, 512)
    P, Q = aq.Policy(net), aq.Policy(net)
    w, b, g, be = aq.upload_params(params, DEV)
    P.policy_set_params_fp32(w, b, g, be)
    ranges = P.calibrate_fp32(aq.to_dev(obs, DEV))
    P.quantize_params(w, b, g, be, ranges)
    assert P.policy_status() == aq.OK
    n = P.policy_blob_size()
    blob = torch.empty(n, dtype=torch.uint8, device=DEV)
    P.policy_export_blob(blob)
    Q.policy_import_blob(blob)
    assert Q.policy_status() == aq.OK
    ms_q = _graph_ms(torch, lambda: P.quantize_params(w, b, g, be, ranges), 20)
    ms_e = _graph_ms(torch, lambda: P.policy_export_blob(blob), 50)
    ms_i = _graph_ms(torch, lambda: Q.policy_import_blob(blob), 50)
    out = {"workload": f"{name} policy blob hand-off" + (f", {wbits}-bit weights" if wbits != 8 else ""), "blob_bytes": n,
           "us_export": ms_e * 1e3, "us_import": ms_i * 1e3, "us_quantize_params": ms_q * 1e3,
           "GBps_import": 2.0 * n / (ms_i * 1e-3) / 1e9}
    if wbits != 8:
        n_p = P.policy_packed_blob_size()
        pblob = torch.empty(n_p, dtype=torch.uint8, device=DEV)
        P.policy_export_packed_blob(pblob)
        Q.policy_import_packed_blob(pblob)
        assert Q.policy_status() == aq.OK
        out["packed_blob_bytes"] = n_p
        out["us_export_packed"] = _graph_ms(torch, lambda: P.policy_export_packed_blob(pblob), 50) * 1e3
        out["us_import_packed"] = _graph_ms(torch, lambda: Q.policy_import_packed_blob(pblob), 50) * 1e3
    P.close()
    Q.close()
    return out


def cpu_baseline(synth, net, params, obs, budget_s=10.0, budget_1t_s=4.0):
    """The CPU oracle, as it stands, on batches of the same workload: about budget_s seconds on all host
    cores, then budget_1t_s seconds on one."""
    from oracle import policy as O
    pol = O.OraclePolicy(net)
    _, own_ranges = pol.forward_fp32(params, obs[:512])   # the oracle calibrates itself
    pol.quantize_params(params, own_ranges)

    def rate(x, budget):
        n = 0
        t0 = time.perf_counter()
        while True:
            pol.forward_int8(x)
            n += x.shape[0]
            dt = time.perf_counter() - t0
            if dt >= budget:
                return n, dt
    cores = int(O.lib().orc_num_threads())
    n, dt = rate(obs, budget_s)
    O.lib().orc_set_num_threads(1)
    n1, dt1 = rate(obs[:512], budget_1t_s)
    O.lib().orc_set_num_threads(cores)
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"value": n / dt, "unit": "inferences/s", "cores": cores, "kind": "oracle",
            "one_thread_value": n1 / dt1, "cpu_model": model,
            "sample": f"{n} observations ({n // obs.shape[0]} batches of {obs.shape[0]}) of the same workload, "
                      f"{dt:.1f} s wall, OpenMP over batch rows on {cores} threads; then {n1} observations in batches "
                      f"of 512 on one thread, {dt1:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--eager", action="store_true", help="launch from the host instead of replaying HIP graphs "
                    "(for profiler runs)")
    ap.add_argument("--only", metavar="CFG:BATCH", help="time one secondary workload only: a forward pass, e.g. cfg5:16384, "
                    "or quantize4m for the 4 M-parameter quantize pass under both schemes (for profiler runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain 64 MiB device-to-device copies (reference for scaling HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path is measured on ONE GPU (the batch is the set of independent actors; "
              "more GPUs would each take a slice of it with no exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = 64 << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda:0").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_copy": n, "bytes_written_per_copy": n, "copies": 20}))
        return
    from paper_1910_01055_amd import binding as aq, synth
    aq.load()
    global _USE_GRAPHS
    _USE_GRAPHS = not args.eager

    if args.only == "quantize4m":
        print(json.dumps([quantize_workload(torch, aq, synth, sch) for sch in ("channel_sym_s8", "tensor_asym_u8")] +
                         [quantize_workload(torch, aq, synth, "channel_sym_s8", reference=True)]))
        return
    if args.only:
        name, bsz = args.only.split(":")
        o, c = forward_workload(torch, aq, synth, name, int(bsz), 100, report_error=True)
        c[0].close()
        print(json.dumps(o))
        return

    batch = 4096
    head, ctx = forward_workload(torch, aq, synth, "cfg2", batch, iters=500)
    P, w, b, g, be, ranges, d_obs, act, net, params, obs = ctx

    # The actor loop: one model pull (the quantizer block) every PULL_EVERY inference calls, counted over
    # warm-up and timed steps together, so that the ratio holds whatever --steps is.
    def step(i):
        if i % PULL_EVERY == 0:
            P.quantize_params(w, b, g, be, ranges)
        P.policy_forward_int8(d_obs, act)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    first = args.warmup
    # as HIP graphs: whole groups of PULL_EVERY steps share one graph (one pull + PULL_EVERY calls per replay,
    # aligned to the pull), the steps before and after them get graphs of their own
    lead = min((-first) % PULL_EVERY, args.steps)
    n_rep, rest = divmod(args.steps - lead, PULL_EVERY)
    g_lead = _capture(torch, lambda: [step(first + i) for i in range(lead)]) if lead else None
    g_main = _capture(torch, lambda: [step(i) for i in range(PULL_EVERY)]) if n_rep else None
    g_rest = _capture(torch, lambda: [step(i) for i in range(rest)]) if rest else None
    graphs_ok = (g_lead is not None or not lead) and (g_main is not None or not n_rep) and (g_rest is not None or not rest)
    pulls = sum(1 for i in range(first, first + args.steps) if i % PULL_EVERY == 0)
    if graphs_ok:
        for gr in (g_lead, g_main, g_rest):
            if gr is not None:
                gr.replay()
    torch.cuda.synchronize()
    st = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(st)
    if graphs_ok:
        if g_lead is not None:
            g_lead.replay()
        for _ in range(n_rep):
            g_main.replay()
        if g_rest is not None:
            g_rest.replay()
    else:
        for i in range(args.steps):
            step(first + i)
    e1.record(st)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    qp_ms = _events_ms(torch, lambda: P.quantize_params(w, b, g, be, ranges), 50)

    ops = 2.0 * synth.macs_per_sample(net) * batch
    achieved = ops / (head["us_per_launch"] * 1e-6) / 1e12
    traffic_ok = FUSED_TRAFFIC["sources_sha256"] == _fused_sources_hash()
    result = {
        "metric": "int8 policy inferences/sec at batch 4096 + % of int8 MFMA peak (1 GPU)",
        "value": batch * args.steps / wall, "unit": "inferences/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "cfg2: D4PG-style actor MLP 67-256(LN+tanh)-256-256-21(tanh), batch 4096, "
                               "per-channel symmetric int8 weights, static uint8 activations",
                   "batch": batch, "pull_every": PULL_EVERY, "model_pulls_in_timed_steps": pulls,
                   "quantize_params_us": qp_ms * 1e3,
                   "launch": "hip graph replay" if graphs_ok else "eager launches from the host (no graph)",
                   "launch_plan": head["launch_plan"],
                   "eager_us_per_launch": head["us_per_launch_eager"],
                   "device_ms_per_step": e0.elapsed_time(e1) / args.steps},
        "pct_int8_mfma_peak": 100.0 * achieved / INT8_PEAK_TOPS,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                     "frac": achieved / INT8_PEAK_TOPS,
                     "traffic": FUSED_TRAFFIC["bytes_per_launch"] if traffic_ok else None,
                     "traffic_unit": "bytes per launch (FETCH_SIZE + WRITE_SIZE counters, copy-calibrated)" if traffic_ok
                     else "null: the kernel's sources have changed since the counters were taken",
                     "kernel": "k_mlp_rows16 (whole-network int8 MLP, 16 batch rows per workgroup)", "us_per_launch": head["us_per_launch"],
                     "timing": "median of 5 repeats of HIP-graph replays of back-to-back launches, HIP events"},
        "fp32_actor_us_per_launch": head["fp32_actor_us_per_launch"],
        "fp16_actor_us_per_launch": head["fp16_actor_us_per_launch"],
    }
    if not args.no_extra:
        extra = []
        # the full actor step of Sec. 4.1: 8-bit forward, then Gaussian exploration noise with per-actor sigma
        sg = torch.rand(batch, device=DEV) * 0.2
        ctr = [0]

        def actor_step():
            ctr[0] += 1
            P.policy_step_int8(d_obs, act, 2024, ctr[0], sigma=sg)
        ms_step = _graph_ms(torch, actor_step, 100)
        extra.append({"workload": "cfg2 batch 4096 forward + exploration noise", "us_per_step": ms_step * 1e3,
                      "inferences_per_s": batch / (ms_step * 1e-3)})
        for name, bsz, it in (("cfg5", 16384, 100), ("cfg3", 65536, 100), ("cfg3", 256, 500), ("cfg3", 1, 500),
                              ("cfg1", 256, 500), ("cfg4", 256, 100), ("cfg4", 1, 200), ("paper_fc2048", 1, 200),
                              ("paper_fc2048", 16, 200)):
            o, c = forward_workload(torch, aq, synth, name, bsz, it, report_error=name in ("cfg5", "cfg4"))
            c[0].close()
            del c
            extra.append(o)
        for scheme in ("channel_sym_s8", "tensor_asym_u8"):
            extra.append(quantize_workload(torch, aq, synth, scheme))
        # the ceiling at that size: the same 16 MiB in / 4 MiB out per launch with no arithmetic at all
        extra.append(quantize_workload(torch, aq, synth, "channel_sym_s8", reference=True))
        # larger tensors: where the per-channel pass crosses 60 % of the HBM peak (launch and ramp amortised),
        # up to 64 M parameters (256 MB in, 64 MB out per call); the rotation always covers > 512 MB
        for rep_, nb_ in ((2, 20), (4, 10), (8, 6), (16, 4)):
            extra.append(quantize_workload(torch, aq, synth, "channel_sym_s8", iters=6, n_buf=nb_, repeat=rep_))
        extra.append(quantize_workload(torch, aq, synth, "channel_sym_s8", iters=6, n_buf=4, repeat=16, reference=True))
        # the ceiling of cfg5's kernel: its k-step loop with nothing around it, on three operand sets
        loops = [mfma_loop_workload(torch, aq, operands, streamed)
                 for operands, streamed in (("zeros", True), ("cfg5-like codes", True), ("cfg5-like codes", False),
                                            ("random bytes", True))]
        extra.extend(loops)
        # cfg5's whole forward pass against what its inner loop alone sustains on such operands (a second, measured
        # denominator beside the nominal peak)
        loop_tops = loops[1]["int8_TOPs"]  # cfg5-like codes, weights streamed
        for o in extra:
            if o.get("workload") == "cfg5 batch 16384":
                o["frac_of_kstep_loop_alone"] = o["tops"] / loop_tops
        for bsz in (1, 300):
            extra.append(subbyte_workload(torch, aq, synth, "paper_fc2048", bsz))
        for name in ("cfg2", "cfg5"):
            extra.append(blob_workload(torch, aq, synth, name))
        extra.append(blob_workload(torch, aq, synth, "cfg5", wbits=4))
        result["other_workloads"] = extra
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(synth, net, params, obs)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
