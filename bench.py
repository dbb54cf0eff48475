#!/usr/bin/env python3
"""Benchmark of the central inference step on one MI355X.

One "step" = one pass of the whole hot path (uint8 frames -> torso -> linear
-> LSTM -> heads -> action selection) over one batch of synthetic DMLab-shaped
input already resident in HBM.  The headline workload is the DMLab deep-ResNet
+ LSTM-256 agent at batch 4096 in bf16.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch B] [--no-extras] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16, published
HBM_PEAK_GBS = 8000.0


# model-size variants of Sections 4.1 (filters x2 / x4), 4.2 (medium and large minimaps) and 4.3 (Atari without
# frame stacking): name -> (label, base workload, overrides, batch)
VARIANTS = {
    "x2": ("DMLab filters x2", "C3", dict(sections=[32, 64, 64]), 1024),
    "x4": ("DMLab filters x4", "C3", dict(sections=[64, 128, 128]), 1024),
    "map120": ("Football map 120x90", "C4", dict(obs_h=90, obs_w=120), 1024),
    "map144": ("Football map 144x108", "C4", dict(obs_h=108, obs_w=144), 1024),
    "atari1": ("Atari without frame stacking", "C2", dict(obs_c=1), 256),
}


def variant_cfg(name):
    from paper_1910_06591_amd import workloads as wl
    label, base, over, b = VARIANTS[name]
    return dict(wl.CONFIGS[base], label=label, index=40, **over), b


def torso_macs_per_frame(cfg):
    from paper_1910_06591_amd import workloads as wl
    h, w, c = wl.torso_out_shape(cfg)
    tail = dict(cfg)
    full = wl.macs_per_frame(cfg)
    # everything after the torso: linear + core + heads
    fc = cfg["fc_units"]
    rest = h * w * c * fc
    core, A = fc, cfg["num_actions"]
    if cfg["lstm_units"]:
        rest += (fc + A + 1 + cfg["lstm_units"]) * 4 * cfg["lstm_units"]
        core = cfg["lstm_units"]
    rest += core * (A + 1) if cfg["head"] == 0 else 2 * core * cfg["head_hidden"] + cfg["head_hidden"] * (A + 1)
    return full - rest


def wake_device(launches=25):
    """Bring the clocks up from idle before a measurement: the host-side preparation of a workload (random frames,
    weight packing) leaves the device idle for up to a second, and the first tens of milliseconds of work after
    that run at reduced clocks whatever the number of warm-up steps.  25 launches of the MFMA probe loop, ~70 ms."""
    import torch
    from paper_1910_06591_amd import seedinf
    lib = seedinf.load_probe_library()
    sink = torch.zeros(4096, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    for _ in range(max(1, int(launches))):          # ~2.8 ms per launch
        rc = lib.seed_probe_mfma_bf16(2048, 400, sink.data_ptr(), st)
        assert rc == 0, rc
    torch.cuda.synchronize()


def time_config(cfg, B, steps, warmup, weights=None, profile=True):
    """Returns dict with ms_per_step (wall over K steps between syncs), p50 of
    per-step event pairs, and the torso kernel's mean duration."""
    import numpy as np
    import torch
    from paper_1910_06591_amd import seedinf, workloads as wl

    weights = wl.make_weights(cfg) if weights is None else weights
    batch = wl.make_batch(cfg, B)
    dev = {k: (None if v is None else torch.from_numpy(v).cuda()) for k, v in batch.items()}
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=B), weights)
    A, Hn = cfg["num_actions"], cfg["lstm_units"]
    out = {"action": torch.empty(B, dtype=torch.int32, device="cuda"),
           "logits": torch.empty(B, A, device="cuda"), "value": torch.empty(B, device="cuda")}
    if Hn:
        out["h"], out["c"] = torch.empty(B, Hn, device="cuda"), torch.empty(B, Hn, device="cuda")
    wake_device()
    for _ in range(warmup):
        net.step(out=out, **dev)
    torch.cuda.synchronize()
    if profile:
        net.set_profiling(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        net.step(out=out, **dev)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    res = {"ms_per_step": (t1 - t0) * 1e3 / steps}
    if profile:
        ms, n = net.profile_read()
        res["torso_ms"] = ms / max(n, 1)
        net.set_profiling(False)
    # per-step latency distribution (separate loop so the events do not sit in the timed region)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in evs:
        a.record()
        net.step(out=out, **dev)
        b.record()
    torch.cuda.synchronize()
    lat = np.sort(np.array([a.elapsed_time(b) for a, b in evs]))
    res.update(p10_ms=float(lat[int(0.1 * (steps - 1))]), p50_ms=float(lat[(steps - 1) // 2]),
               p90_ms=float(lat[int(0.9 * (steps - 1))]))
    net.close()
    return res


def time_extensions(cfg, B, weights):
    """The step with episode flags + epsilon-greedy, and the weight hot-swap between steps (extras, not `value`)."""
    import numpy as np
    import torch
    from paper_1910_06591_amd import seedinf, workloads as wl

    batch = wl.make_batch(cfg, B)
    dev = {k: (None if v is None else torch.from_numpy(v).cuda()) for k, v in batch.items()}
    done, eps, eu = wl.make_episode_inputs(cfg, B)
    ext = dict(done=torch.from_numpy(done).cuda(), epsilon=torch.from_numpy(eps).cuda(),
               explore_uniforms=torch.from_numpy(eu).cuda())
    net = seedinf.SeedInfer(seedinf.make_arch(cfg, max_batch=B), weights)
    out = net.step(**dev, **ext)
    torch.cuda.synchronize()

    def p50(fn, n=40):
        for _ in range(20):
            fn()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in evs:
            a.record(); fn(); b.record()
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in evs]))

    res = {"step_plain_p50_ms": p50(lambda: net.step(out=out, **dev)),
           "step_ext_p50_ms": p50(lambda: net.step(out=out, **dev, **ext))}
    # the same step captured once into a HIP graph (the step is kernel launches only) and replayed
    def graphed_p50(nb):
        sub = {k: (None if v is None else v[:nb].contiguous()) for k, v in dev.items()}
        o = net.step(**sub)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            net.step(out=o, **sub)
        return p50(g.replay), p50(lambda: net.step(out=o, **sub))
    res["graph_replay_vs_eager_p50_ms"] = {str(nb): list(graphed_p50(nb)) for nb in (64, 256, B) if nb <= B}
    # weight refresh: host time of the call (copy into pinned staging + enqueue; measured from an idle stream, as
    # between two training steps) and a step issued right behind it
    t = []
    for _ in range(7):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        net.set_weights(weights)
        t.append((time.perf_counter() - t0) * 1e3)
        net.step(out=out, **dev)
    torch.cuda.synchronize()
    res["set_weights_host_ms"] = float(np.median(t))
    res["step_after_set_weights_p50_ms"] = p50(lambda: (net.set_weights(weights), net.step(out=out, **dev)), n=5)
    res["weights_mb"] = weights.size * 4 / 1e6
    # sustained rate: about a second of back-to-back steps from whatever state the device is in (no wake-up loop in
    # front, one synchronisation at the end), with the torso kernel's own mean duration over the same steps
    n_sus = min(4000, max(2000, int(1.0 / max(res["step_plain_p50_ms"] * 1e-3, 1e-5))))
    net.set_profiling(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_sus):
        net.step(out=out, **dev)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tms, tn = net.profile_read()
    net.set_profiling(False)
    res["sustained_1s"] = {"steps": n_sus, "seconds": dt, "ms_per_step": dt * 1e3 / n_sus, "frames_per_s": n_sus * B / dt,
                           "torso_ms": tms / max(tn, 1),
                           "step_frac_of_bf16_peak": 2.0 * wl.macs_per_frame(cfg) * B * n_sus / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS}
    # T-step unroll over stored trajectories: T = 32 (the unroll length of the paper's V-trace agents), B / 32 rows
    if B % 32 == 0 and B >= 32:
        T, Bt = 32, B // 32
        r = lambda k, *tail: None if dev[k] is None else dev[k].reshape(T, Bt, *tail).contiguous()
        tdone = ext["done"].reshape(T, Bt).contiguous() if cfg["lstm_units"] else None
        h0 = None if dev["h_in"] is None else dev["h_in"][:Bt].contiguous()
        c0 = None if dev["c_in"] is None else dev["c_in"][:Bt].contiguous()
        args = (r("obs", cfg["obs_h"], cfg["obs_w"], cfg["obs_c"]), r("prev_action"), r("prev_reward"), h0, c0,
                r("uniforms", cfg["num_actions"]), tdone)
        ms = p50(lambda: net.unroll(*args), n=20)
        res["unroll_T32_p50_ms"] = ms
        res["unroll_T32_frames_per_s"] = B / ms * 1e3
    # host batching front-end: frames start in host memory; two batches in flight (PCIe-inclusive rate)
    bat = seedinf.Batcher(net, 2 * B)
    actors = [np.arange(B, dtype=np.int32), np.arange(B, 2 * B, dtype=np.int32)]
    rew = batch["prev_reward"]
    dn = np.zeros(B, np.uint8)
    rounds = 20
    for k in range(6):                                   # warm-up: first touches of the pinned staging sets
        bat.add_many(actors[k % 2], batch["obs"], rew, dn)
        bat.wait(bat.submit(batch["uniforms"]))
    tickets = []
    t0 = time.perf_counter()
    for k in range(rounds):
        bat.add_many(actors[k % 2], batch["obs"], rew, dn)
        tickets.append(bat.submit(batch["uniforms"]))
        if len(tickets) == 2:
            bat.wait(tickets.pop(0))
    for t in tickets:
        bat.wait(t)
    dt = time.perf_counter() - t0
    res["batcher_frames_per_s_pcie_inclusive"] = rounds * B / dt
    res["batcher_ms_per_round"] = dt * 1e3 / rounds
    bat.close()
    net.close()
    return res


def measure_peaks():
    """What this GPU sustains on the two rooflines: an MFMA-only bf16 loop and a plain streaming copy
    (libseedprobe.so), timed with events on the current stream."""
    import torch
    from paper_1910_06591_amd import seedinf
    lib = seedinf.load_probe_library()
    st = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(4096, dtype=torch.float32, device="cuda")
    blocks, iters = 2048, 400                       # 8 blocks per compute unit, ~1 ms per launch

    def timed(fn, n):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n * 1e-3

    def mfma():
        rc = lib.seed_probe_mfma_bf16(blocks, iters, sink.data_ptr(), st)
        assert rc == 0, rc
    t = timed(mfma, 10)
    tflops = lib.seed_probe_mfma_flops(blocks, iters) / t / 1e12
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)

    def copy():
        rc = lib.seed_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, st)
        assert rc == 0, rc
    t = timed(copy, 10)
    gbs = 2.0 * nbytes / t / 1e9
    return {"mfma_bf16_tflops": tflops, "mfma_frac_of_nominal": tflops / MFMA_BF16_PEAK_TFLOPS,
            "hbm_copy_gbs": gbs, "hbm_copy_frac_of_nominal": gbs / HBM_PEAK_GBS,
            "how": "MFMA-only loop (2048 blocks x 8 wavefronts x 25600 v_mfma_f32_16x16x32_bf16); streaming copy of 1 GiB "
                   "(four 16-byte non-temporal loads in flight per lane), read + write bytes"}


def cpu_baseline(cfg, rows):
    """The CPU oracle as it stands, on `rows` rows of the same workload."""
    import oracle
    from paper_1910_06591_amd import workloads as wl
    orc = oracle.Oracle("f32")
    weights = wl.make_weights(cfg)
    b = wl.make_batch(cfg, rows)
    kw = {k: b[k] for k in ("prev_action", "prev_reward", "h_in", "c_in", "uniforms")}
    arch = oracle.make_arch(cfg)
    orc.forward(arch, weights, b["obs"][:2], **{k: (None if v is None else v[:2]) for k, v in kw.items()})
    t0 = time.perf_counter()
    orc.forward(arch, weights, b["obs"], **kw)
    dt = time.perf_counter() - t0
    # one core: the oracle spreads rows over threads, so one-row calls run on a single thread
    one = {k: (None if v is None else v[:1]) for k, v in kw.items()}
    t1 = time.perf_counter()
    for _ in range(8):
        orc.forward(arch, weights, b["obs"][:1], **one)
    d1 = (time.perf_counter() - t1) / 8
    return {"value": rows / dt, "unit": "frames/s", "cores": int(orc.lib.oracle_num_threads()), "kind": "oracle",
            "sample": f"{rows} rows of the same workload, one oracle_forward call ({dt:.1f} s wall)",
            "one_core_value": 1.0 / d1}


def read_traffic(key="traffic_bytes_per_launch"):
    """HBM bytes per launch of the torso kernel (or, key = "step_traffic_bytes", of all the step's kernels) from
    the committed rocprofv3 counter summary (profiles/), or None."""
    path = os.path.join(ROOT, "profiles", "resnet_torso_c5_b4096_pmc.txt")
    try:
        for line in open(path):
            if line.startswith(key):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--batch", type=int, default=None, help="rows per step (default: 4096 for C5, the workload's own batch otherwise)")
    ap.add_argument("--workload", default="C5", choices=["C1", "C2", "C3", "C4", "C5"],
                    help="C5 (default) is the headline line; any other name times that workload alone and prints a "
                         "short line for it (used to profile the other workloads' kernels)")
    ap.add_argument("--variant", default=None, choices=sorted(VARIANTS),
                    help="time one model-size variant (Sections 4.1 / 4.2 / 4.3) alone and print a short line for it")
    ap.add_argument("--no-extras", action="store_true", help="skip the batch sweep and the other configs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-rows", type=int, default=512)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (reference kernel for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU; --gpus must be 1 (the step shards by batch rows "
              "with no exchange, so N GPUs are N independent copies)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1910_06591_amd import seedinf, workloads as wl
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if not os.path.exists(seedinf.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()

    if args.copy_calibration:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.workload != "C5" or args.variant:
        if args.variant:
            c, b0 = variant_cfg(args.variant)
            args.workload = "variant " + args.variant
        else:
            c, b0 = wl.CONFIGS[args.workload], wl.CONFIGS[args.workload]["batch"]
        b = args.batch or b0
        s = time_config(c, b, args.steps, args.warmup)
        print(json.dumps({"metric": "batched inference frames/sec at batch B (1 GPU)", "value": b / (s["ms_per_step"] * 1e-3),
                          "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": s["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                          "dtype": c["precision"], "data": "synthetic",
                          "config": {"workload": f"{args.workload}: {c.get('label', args.workload)}", "batch": b},
                          "p50_ms": s["p50_ms"], "torso_ms": s.get("torso_ms"),
                          "step_tflops": 2.0 * wl.macs_per_frame(c) * b / (s["ms_per_step"] * 1e-3) / 1e12}))
        return
    cfg = wl.CONFIGS["C5"]
    B = args.batch or 4096
    weights = wl.make_weights(cfg)
    peaks = None if args.no_extras else measure_peaks()
    r = time_config(cfg, B, args.steps, args.warmup, weights)
    fps = B / (r["ms_per_step"] * 1e-3)
    flops_step = 2.0 * wl.macs_per_frame(cfg) * B
    torso_flops = 2.0 * torso_macs_per_frame(cfg) * B
    achieved = torso_flops / (r["torso_ms"] * 1e-3) / 1e12
    line = {
        "metric": "batched inference frames/sec at batch B (1 GPU)",
        "value": fps, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"C5: DMLab deep-ResNet (16/32/32) + LSTM-256 agent, 72x96x3 uint8 frames, batch {B}, "
                               "15 actions, Gumbel-max sampling", "batch": B},
        "p50_ms": r["p50_ms"], "p10_ms": r["p10_ms"], "p90_ms": r["p90_ms"],
        "step_tflops": flops_step / (r["ms_per_step"] * 1e-3) / 1e12,
        "step_frac_of_bf16_peak": flops_step / (r["ms_per_step"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": "resnet3_bf16_kernel (fused torso)", "achieved": achieved,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                     "kernel_ms": r["torso_ms"], "traffic": read_traffic()},
    }
    if not args.no_extras:
        line["measured_peaks"] = peaks
        line["roofline"]["frac_of_measured_peak"] = achieved / peaks["mfma_bf16_tflops"]
        sweep = []
        for b in cfg["sweep"]:
            k = max(20, min(args.steps, 200))
            s = time_config(cfg, b, k, args.warmup, weights)
            entry = {"batch": b, "frames_per_s": b / (s["p50_ms"] * 1e-3), "p50_ms": s["p50_ms"],
                     "frac_of_bf16_peak": 2.0 * wl.macs_per_frame(cfg) * b / (s["p50_ms"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                     "torso_ms": s["torso_ms"],
                     # HBM rate of the bytes every implementation must move (frame, state, outputs) ...
                     "hbm_gbs_algorithmic": wl.hbm_bytes_per_frame(cfg) * b / (s["p50_ms"] * 1e-3) / 1e9}
            # ... and, at the batch the counter profile was taken at, of the bytes this one does move
            step_bytes = read_traffic("step_traffic_bytes")
            if b == B and step_bytes:
                entry["hbm_gbs_counters"] = step_bytes / (s["p50_ms"] * 1e-3) / 1e9
            sweep.append(entry)
        line["sweep"] = sweep
        others = []
        for name in ("C1", "C2", "C3", "C4"):
            c = wl.CONFIGS[name]
            s = time_config(c, c["batch"], max(20, min(args.steps, 100)), args.warmup)
            others.append({"config": name, "batch": c["batch"], "dtype": c["precision"],
                           "frames_per_s": c["batch"] / (s["p50_ms"] * 1e-3), "p50_ms": s["p50_ms"],
                           "tflops": 2.0 * wl.macs_per_frame(c) * c["batch"] / (s["p50_ms"] * 1e-3) / 1e12})
        line["other_workloads"] = others
        line["extensions"] = time_extensions(cfg, B, weights)
        # model-size variants (Section 4.1: filters x2 / x4; Section 4.2: medium and large minimaps; Atari without
        # frame stacking): the layer-by-layer bf16 ResNet path; the Atari agent on single frames has the fused conv stack
        variants = []
        for name in ("x2", "x4", "map120", "map144", "atari1"):
            c, b = variant_cfg(name)
            label = c["label"]
            s = time_config(c, b, 20, 3, profile=False)
            variants.append({"config": label, "batch": b, "dtype": c["precision"], "frames_per_s": b / (s["p50_ms"] * 1e-3),
                             "p50_ms": s["p50_ms"], "tflops": 2.0 * wl.macs_per_frame(c) * b / (s["p50_ms"] * 1e-3) / 1e12})
        line["model_variants"] = variants
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(cfg, args.cpu_rows)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
