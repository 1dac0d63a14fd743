"""Benchmark of the H-CNN hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: neighbour / child index lists
by hash lookups, then a 5-level encoder (conv3x3x3 -> ReLU -> 2x2x2 max-pool per level,
256^3 -> 8^3, channels 4-16-32-64-128-256) forward and backward (weight and data gradients at
every level), on the 256^3 / batch 8 workload.  Inputs are resident in HBM before the timed
region; PSH construction is pre-processing and is not timed.

Prints ONE JSON line; README.md lists its fields.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3  # dense fp32 matrix
MFMA_BF16_PEAK_TFLOPS = 2500.0
CHANNELS = [4, 16, 32, 64, 128, 256]
ALGOS = {"fused": "HCH_ALGO_FUSED", "fused_dense": "HCH_ALGO_FUSED_DENSE", "columns": "HCH_ALGO_COLUMNS"}


def make_inputs(config, batch, u):
    import synth_shapes as S
    coords, offs, normals = S.config_batch(config, batch=batch, u=u, with_normals=True)
    X0 = S.normals_plus_one(normals)
    W = [S.he_weights(CHANNELS[l], CHANNELS[l + 1], 4000 + l) for l in range(5)]
    return coords, offs, X0, W


def cpu_baseline(coords, offs, X0, W, u, max_shapes, budget_s=16.0):
    """The oracle, as it stands, on the first shapes of the same batch: encoder forward and
    backward with the paper's algorithms in double precision, with all its threads and with one."""
    from oracle import oracle as O
    import synth_shapes as S

    def run(ns):
        c, o = coords[: offs[ns]], offs[: ns + 1]
        lv = O.build_hierarchy(c, o, u, 6)           # construction is pre-processing: not timed
        t0 = time.perf_counter()
        X = [O.to_paper_X(X0[: offs[ns]])]
        A, sw = [], []
        flops = 0
        for l in range(5):
            Wp = O.to_paper_W(W[l])
            Y = O.conv_fwd(lv[l], X[l], Wp)
            A.append(np.maximum(Y, 0.0))
            P, s = O.pool_max_fwd(lv[l], lv[l + 1], A[l])
            X.append(P); sw.append(s)
            flops += 3 * 2 * 27 * CHANNELS[l] * CHANNELS[l + 1] * lv[l].Ntot
        g = O.to_paper_X(S.gaussian((lv[5].Ntot, CHANNELS[5]), 1.0, 4100))
        for l in reversed(range(5)):
            dA = O.pool_max_bwd(lv[l].Ntot, g, sw[l])
            dY = np.where(A[l] > 0, dA, 0.0)
            O.conv_bwd_weight(lv[l], X[l], dY)
            g = O.conv_bwd_data(lv[l], dY, O.to_paper_W(W[l]), CHANNELS[l])
        return time.perf_counter() - t0, flops

    def sample(budget):
        # whole passes over a prefix of the batch until about `budget` seconds of CPU work are spent
        total_t, total_f, passes = 0.0, 0.0, 0
        dt, flops = run(1)
        ns = max_shapes if dt * max_shapes < budget else max(1, min(max_shapes, int(budget / max(dt, 1e-3))))
        while total_t < budget / 2 and passes < 20:
            dt, flops = run(ns)
            total_t += dt; total_f += flops; passes += 1
        return total_f / total_t / 1e12, f"first {ns} of {len(offs) - 1} shapes, {passes} fwd+bwd passes, {total_t:.1f} s"

    cores = O.threads()
    v_all, note_all = sample(budget_s)
    O.set_threads(1)
    try:
        v_one, note_one = sample(budget_s / 2)
    finally:
        O.set_threads(cores)
    return {"value": round(v_all, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle", "sample": note_all,
            "note": "plain loops in double precision in the paper's data layout: a correctness reference, not a tuned CPU code",
            "single_thread": {"value": round(v_one, 6), "unit": "TFLOP/s", "cores": 1, "sample": note_one}}


def time_calls(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def conv_products(torch, hch, S, cfg, algo_name, steps, warmup, tap_major=True):
    """The three products of ONE convolution on the finest level of a per-kernel workload:
    3 = 128^3 grid, batch 16, 32 -> 64, fp32; 5 = 512^3 grid, batch 4, 64 -> 64, bf16 inputs with
    fp32 sums and outputs.  Tables built on the device; time per product from HIP events."""
    u, ci, co, bf = {3: (128, 32, 64, False), 5: (512, 64, 64, True)}[cfg]
    coords, offs, _ = S.config_batch(cfg)
    lv = hch.hch_build_levels_device(coords, offs, u, 1)
    n = lv.n(0)
    algo = getattr(hch, ALGOS[algo_name])
    DT = hch.HCH_BF16 if bf else hch.HCH_F32
    if bf and tap_major:
        hch.hch_build_tap_major(lv, 0)        # the bf16 gathers read their indices tap by tap

    def put(a):
        if bf:
            return torch.from_numpy(S.bf16_bits(S.to_bf16_grid(a)).view(np.int16)).to("cuda")
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda")

    seed = 1000 * cfg
    X, G = put(S.gaussian((n, ci), 1.0, seed + 1)), put(S.gaussian((n, co), 1.0, seed + 3))
    W = put(S.he_weights(ci, co, seed + 2))
    Y = torch.empty((n, co), dtype=torch.float32, device="cuda")
    dX = torch.empty((n, ci), dtype=torch.float32, device="cuda")
    dW = torch.empty((27, ci, co), dtype=torch.float32, device="cuda")
    need = max(hch.hch_conv_workspace_bytes(lv, 0, ci, co, DT, k, algo)
               for k in (hch.HCH_WS_FWD, hch.HCH_WS_BWD_DATA, hch.HCH_WS_BWD_WEIGHT))
    buf = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    off = (-buf.data_ptr()) % 256
    ws = buf[off: off + need]
    calls = (("forward", lambda: hch.hch_conv_fwd(lv, 0, DT, X, W, Y, ci, co, ws, algo)),
             ("data_gradient", lambda: hch.hch_conv_bwd_data(lv, 0, DT, G, W, dX, ci, co, ws, algo)),
             ("weight_gradient", lambda: hch.hch_conv_bwd_weight(lv, 0, DT, X, G, dW, ci, co, ws, algo)))
    occupied = lv.info(0).nbr_valid
    flop, useful = 2.0 * n * 27 * ci * co, 2.0 * occupied * ci * co
    peak = MFMA_BF16_PEAK_TFLOPS if bf else MFMA_F32_PEAK_TFLOPS
    out = {}
    for name, fn in calls:
        ms = time_calls(torch, fn, steps, warmup)
        out[name] = {"ms": round(ms, 4), "tflops": round(flop / ms / 1e9, 1),
                     "useful_tflops": round(useful / ms / 1e9, 1),
                     "frac_of_mfma_peak": round(flop / ms / 1e9 / peak, 4)}
    return {"metric": f"one 3x3x3 convolution {ci} -> {co}: time per product", "unit": "ms",
            "products": out, "calls_timed": steps, "higher_is_better": False,
            "dtype": "bf16" if bf else "f32", "data": "synthetic", "algo": algo_name,
            "flop_count": "tflops: paper-method 2*27*c_in*c_out*N; useful_tflops: occupied taps only",
            "mfma_peak_tflops": peak,
            "config": {"workload": f"{u}^3 grid, batch {len(offs) - 1}, random-primitive surfaces, {n} voxels, "
                                   f"{occupied / n:.2f} of 27 taps occupied per voxel"}}


def measured_roofs(torch, hch):
    """What this GPU delivers on a plain copy (the library's ReLU kernel over 2^26 floats: 256 MiB
    read, 256 MiB written) and on loops of nothing but matrix instructions."""
    n = 1 << 26
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    ms = time_calls(torch, lambda: hch.hch_relu_fwd(src, dst, n), 10, 3)
    copy = 8.0 * n / ms / 1e6
    del src, dst
    wgs, iters = 256 * 16, 4000
    sink = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    out = {"copy_GBs": round(copy, 1), "copy_frac_of_hbm_peak": round(copy / HBM_PEAK_GBS, 4)}
    for name, dt, per, peak in (("mfma_f32", hch.HCH_F32, 2048.0, MFMA_F32_PEAK_TFLOPS),
                                ("mfma_bf16", hch.HCH_BF16, 16384.0, MFMA_BF16_PEAK_TFLOPS)):
        ms = time_calls(torch, lambda: hch.hch_probe_mfma(dt, iters, wgs, sink), 5, 2)
        tf = wgs * 4 * iters * 8 * per / ms / 1e9
        out[name + "_TFLOPs"] = round(tf, 1)
        out[name + "_frac_of_peak"] = round(tf / peak, 4)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--resolution", type=int, default=256, help="finest grid side (256 = the headline workload)")
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-all", action="store_true", help="time every kernel in the timed region (adds event overhead)")
    ap.add_argument("--no-kernel-pass", action="store_true", help="skip the fully timed pass of the benchmarked algorithm")
    ap.add_argument("--no-other-algo", action="store_true", help="skip the fully timed pass of the other algorithm")
    ap.add_argument("--no-extra", action="store_true", help="skip the measured roofs and the two per-kernel workloads")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="before the warm-up, run the library's ReLU kernel three times over 2^24 floats (reads "
                         "64 MiB, writes 64 MiB): the known-size copy that scales the FETCH_SIZE / WRITE_SIZE "
                         "counters of a rocprofv3 --pmc run")
    ap.add_argument("--two-streams", action="store_true",
                    help="timed region with the weight gradients and the coarse index lists on a second "
                         "stream (faster; kernels then share the chip, so per-kernel times are not clean)")
    ap.add_argument("--no-overlap-pass", action="store_true", help="skip the extra two-stream pass")
    ap.add_argument("--build-bench", action="store_true",
                    help="time only the construction of the hash tables of the workload, on the host "
                         "(hch_build_levels) and on the device (hch_build_levels_device), and print that")
    ap.add_argument("--conv-bench", type=int, choices=[3, 5], default=0,
                    help="time only the three products of one convolution on a per-kernel workload and print "
                         "that: 3 = 128^3 grid, batch 16, 32 -> 64, fp32; 5 = 512^3 grid, batch 4, 64 -> 64, bf16")
    ap.add_argument("--no-tap-major", action="store_true", help="--conv-bench 5 without the tap-major index copy")
    ap.add_argument("--algo", choices=sorted(ALGOS), default="fused",
                    help="columns: hash2col -> GEMM -> col2hash through memory; fused: gathered GEMM operand, taps "
                         "that a tile of voxels lacks left out; fused_dense: the same without leaving taps out")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1803_11385_amd as hch
    from paper_1803_11385_amd.pipeline import Encoder
    import synth_shapes as S

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.conv_bench:
        print(json.dumps(conv_products(torch, hch, S, args.conv_bench, args.algo, args.steps, args.warmup,
                                       tap_major=not args.no_tap_major)))
        return
    u, b = args.resolution, args.batch
    t0 = time.perf_counter()
    coords, offs, X0, W = make_inputs(4, b, u)
    t_gen = time.perf_counter() - t0

    def timed_build(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        lv = fn(coords, offs, u, 6)
        torch.cuda.synchronize()
        return lv, time.perf_counter() - t0

    if args.build_bench:
        res = {"host": [], "device": []}
        for _ in range(max(1, args.warmup // 2) + max(1, args.steps // 4)):
            for name, fn in (("host", hch.hch_build_levels), ("device", hch.hch_build_levels_device)):
                lv, dt = timed_build(fn)
                res[name].append(dt)
                del lv
        skip = max(1, args.warmup // 2)
        print(json.dumps({"metric": "construction of the 6-level hash tables, index lists included", "unit": "ms",
                          "host_ms": round(1e3 * float(np.median(res["host"][skip:])), 2),
                          "device_ms": round(1e3 * float(np.median(res["device"][skip:])), 2),
                          "calls_timed": len(res["host"]) - skip, "higher_is_better": False,
                          "config": {"workload": f"{u}^3 grid, batch {b}, random-primitive surfaces"}}))
        return
    levels, t_build = timed_build(hch.hch_build_levels)
    lv_dev, t_build_dev = timed_build(hch.hch_build_levels_device)
    del lv_dev
    algo = getattr(hch, ALGOS[args.algo])
    G5 = None

    def new_encoder(algo_id, two_streams=False):
        nonlocal G5
        enc = Encoder(levels, CHANNELS, algo_id, two_streams=two_streams)
        if G5 is None:
            G5 = torch.from_numpy(S.gaussian((enc.n[5], CHANNELS[5]), 1.0, 4100))
        enc.X[0].copy_(torch.from_numpy(X0))
        for l in range(5):
            enc.W[l].copy_(torch.from_numpy(W[l]))
        enc.dX[5].copy_(G5)
        torch.cuda.synchronize()
        return enc

    enc = new_encoder(algo, args.two_streams)

    def kernel_table():
        out = {}
        for i in range(hch.hch_kernel_count()):
            st = hch.hch_profile_read(i)
            if st["launches"]:
                out[hch.hch_kernel_name(i)] = (i, st)
        return out

    from paper_1803_11385_amd.build import source_digest
    digest = source_digest()

    def load_traffic(algo_name):
        """kernel -> HBM bytes per launch, from the committed rocprofv3 --pmc summary of this
        workload (FETCH_SIZE + WRITE_SIZE, calibrated on a copy kernel); the counters cannot be
        read from inside this process.  The summary names the digest of the sources it ran on."""
        db, src = {}, {"file": None, "sources_sha256_16": None, "stale": None}
        path = os.path.join(ROOT, "profiles", f"hbm_traffic_encoder_{u}x{b}_{algo_name}.txt")
        if os.path.exists(path):
            src["file"] = os.path.relpath(path, ROOT)
            for line in open(path):
                if line.startswith("# sources sha256/16:"):
                    src["sources_sha256_16"] = line.split(":", 1)[1].strip()
                parts = [x.strip() for x in line.split("|")]
                if line.startswith("#") or len(parts) != 5:
                    continue
                try:
                    db[parts[0]] = float(parts[4])
                except ValueError:
                    pass
            src["stale"] = src["sources_sha256_16"] != digest
        return db, src

    traffic = {a: load_traffic(a) for a in ("fused", "columns")}

    def traffic_key(algo_name):
        return "columns" if algo_name == "columns" else "fused"

    def roofline_of(name, st, steps, algo_name):
        """achieved = algorithmic bytes (or flops) of the timed launches / their event-measured
        time; a kernel counts as MFMA-bound when its arithmetic intensity is above the ridge.
        traffic = counter-measured HBM bytes per launch from the committed summary; null when
        that summary was measured on other sources than the ones running now."""
        ai = st["flops"] / max(1.0, st["bytes"])
        product = any(t in name for t in ("gemm", "conv_direct", "conv_narrow4"))
        if product and ai >= MFMA_F32_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
            bound, achieved, peak, unit = "mfma", st["flops"] / (st["ms"] * 1e-3) / 1e12, MFMA_F32_PEAK_TFLOPS, "TFLOP/s"
        else:
            bound, achieved, peak, unit = "hbm", st["bytes"] / (st["ms"] * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
        db, src = traffic[traffic_key(algo_name)]
        return {"kernel": name, "bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": None if src["stale"] else db.get(name),
                "launches_per_step": st["launches"] / steps,
                "avg_launch_ms": round(st["ms"] / max(1, st["launches"]), 5),
                "algorithmic_bytes_per_launch": round(st["bytes"] / max(1, st["launches"])),
                "flops_per_launch": round(st["flops"] / max(1, st["launches"]))}

    if args.copy_calibration:
        src = torch.ones(1 << 24, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            hch.hch_relu_fwd(src, dst, src.numel())
        torch.cuda.synchronize()
        del src, dst

    # warm-up; the first warm-up step times every kernel to find the dominant one
    hch.hch_profile_reset()
    hch.hch_profile_enable(-1, True)
    enc.step()
    torch.cuda.synchronize()
    first = kernel_table()
    dom_name = max(first, key=lambda k: first[k][1]["ms"])
    dominant = first[dom_name][0]
    if not args.profile_all:
        hch.hch_profile_enable(-1, False)
        hch.hch_profile_enable(dominant, True)
    for _ in range(max(0, args.warmup - 1)):
        enc.step()
    torch.cuda.synchronize()
    hch.hch_profile_reset()

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        enc.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    hch.hch_profile_enable(-1, False)

    ms_per_step = dt / args.steps * 1e3
    flops = enc.flops_per_step()
    # the same three products per level counted on the occupied taps only: what is left of the
    # paper's count once the products with zero rows of the column matrix are taken out
    occupied = [levels.info(l).nbr_valid for l in range(5)]
    useful = sum(3 * 2 * occupied[l] * CHANNELS[l] * CHANNELS[l + 1] for l in range(5))
    value = flops / (ms_per_step * 1e-3) / 1e12
    roofline = roofline_of(dom_name, hch.hch_profile_read(dominant), args.steps, args.algo)
    roofline["traffic_source"] = traffic[traffic_key(args.algo)][1]

    out = {
        "metric": "sparse conv fwd+bwd TFLOP/s and gather/scatter HBM GB/s, 256^3 grid, batch 8",
        "value": round(value, 4), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"5-level encoder fwd+bwd, {u}^3 grid, batch {b}, random-primitive surfaces, "
                               f"channels 4-16-32-64-128-256, N per level = {enc.n}",
                   "algo": args.algo,
                   "flop_count": "value: paper-method 3 * 2*27*c_in*c_out*N_l per level; "
                                 "useful_value: 3 * 2*c_in*c_out*(occupied taps of level l)",
                   "gflop_per_step": round(flops / 1e9, 3), "useful_gflop_per_step": round(useful / 1e9, 3),
                   "occupied_taps_per_voxel": [round(occupied[l] / max(1, enc.n[l]), 2) for l in range(5)],
                   "psh_build_s": round(t_build, 3), "psh_build_device_s": round(t_build_dev, 3),
                   "shape_gen_s": round(t_gen, 2), "sources_sha256_16": digest},
        "useful_value": round(useful / (ms_per_step * 1e-3) / 1e12, 4),
        "roofline": roofline,
        "kernels_ms_first_step": {k: round(v[1]["ms"], 4) for k, v in first.items()},
    }

    def timed_pass(algo_name):
        """`steps` steps of an algorithm with EVERY kernel timed (the events' overhead is in the
        step time): per-kernel rooflines, slowest kernel first."""
        e = new_encoder(getattr(hch, ALGOS[algo_name]))
        for _ in range(2):
            e.step()
        torch.cuda.synchronize()
        hch.hch_profile_reset()
        hch.hch_profile_enable(-1, True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            e.step()
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t0
        hch.hch_profile_enable(-1, False)
        tab = kernel_table()
        return dt2, [roofline_of(k, v[1], args.steps, algo_name)
                     for k, v in sorted(tab.items(), key=lambda kv: -kv[1][1]["ms"])]

    if not args.no_kernel_pass:
        dt2, ks = timed_pass(args.algo)
        out[f"{traffic_key(args.algo)}_kernels"] = {
            "algo": args.algo, "ms_per_step_all_kernels_timed": round(dt2 / args.steps * 1e3, 4), "kernels": ks}

    if not args.two_streams and not args.no_overlap_pass:
        # the same steps with the weight gradients and the coarse levels' index lists on a second
        # stream: whole-step throughput when independent kernels share the chip
        enc3 = new_encoder(algo, True)
        for _ in range(max(1, args.warmup)):
            enc3.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            enc3.step()
        torch.cuda.synchronize()
        dt3 = time.perf_counter() - t0
        out["two_streams"] = {"ms_per_step": round(dt3 / args.steps * 1e3, 4),
                              "value": round(flops / (dt3 / args.steps) / 1e12, 4),
                              "useful_value": round(useful / (dt3 / args.steps) / 1e12, 4), "unit": "TFLOP/s"}
        del enc3

    if not args.no_other_algo:
        # the other algorithm on the same inputs (by default the paper's own three-step path
        # hash2col -> GEMM -> col2hash): rooflines of its gather, GEMM and scatter kernels
        other = "columns" if args.algo != "columns" else "fused"
        dt2, ks = timed_pass(other)
        out["other_algo"] = {
            "algo": other, "ms_per_step_all_kernels_timed": round(dt2 / args.steps * 1e3, 4),
            "value": round(flops / (dt2 / args.steps) / 1e12, 4), "unit": "TFLOP/s",
            "kernels": [k for k in ks if any(t in k["kernel"] for t in ("hash2col", "col2hash", "gemm", "neighbour", "conv_"))],
            "traffic_source": traffic[traffic_key(other)][1],
        }
    del enc
    if not args.no_extra:
        roofs = measured_roofs(torch, hch)
        measured = roofs["mfma_f32_TFLOPs"] if roofline["bound"] == "mfma" else roofs["copy_GBs"]
        roofs["dominant_kernel_frac_of_measured"] = round(roofline["achieved"] / measured, 4)
        out["roofline_measured"] = roofs
        out["per_kernel_benches"] = {
            "config3": conv_products(torch, hch, S, 3, "fused", args.steps, args.warmup),
            "config5": conv_products(torch, hch, S, 5, "fused", args.steps, args.warmup),
        }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(coords, offs, X0, W, u, b)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
