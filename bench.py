"""Benchmark of the H-CNN hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: neighbour / child index lists
by hash lookups, then a 5-level encoder (conv3x3x3 -> ReLU -> 2x2x2 max-pool per level,
256^3 -> 8^3, channels 4-16-32-64-128-256) forward and backward (weight and data gradients at
every level), on the 256^3 / batch 8 workload.  Inputs are resident in HBM before the timed
region; PSH construction is pre-processing and is not timed.

Prints ONE JSON line (see README / DESIGN for the fields).
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
CHANNELS = [4, 16, 32, 64, 128, 256]


def make_inputs(config, batch, u):
    import synth_shapes as S
    coords, offs, normals = S.config_batch(config, batch=batch, u=u, with_normals=True)
    X0 = S.normals_plus_one(normals)
    W = [S.he_weights(CHANNELS[l], CHANNELS[l + 1], 4000 + l) for l in range(5)]
    return coords, offs, X0, W


def cpu_baseline(coords, offs, X0, W, u, max_shapes, budget_s=24.0):
    """The oracle, as it stands, on the first shapes of the same batch: encoder forward and
    backward with the paper's algorithms in double precision.  Returns (TFLOP/s, cores, note)."""
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

    # whole passes over a growing prefix of the batch until about budget_s of CPU work is spent
    ns, total_t, total_f, passes = 1, 0.0, 0.0, 0
    dt, flops = run(ns)
    if dt * max_shapes / ns < budget_s:
        ns = max_shapes
    else:
        ns = max(1, min(max_shapes, int(ns * budget_s / max(dt, 1e-3))))
    while total_t < budget_s / 2 and passes < 20:
        dt, flops = run(ns)
        total_t += dt; total_f += flops; passes += 1
    return (total_f / total_t / 1e12, O.threads(),
            f"first {ns} of {len(offs) - 1} shapes, {passes} fwd+bwd passes, {total_t:.1f} s")


def conv_bench(args, torch, hch, S):
    """The three products of ONE convolution on the finest level of a per-kernel workload:
    3 = 128^3 grid, batch 16, 32 -> 64, fp32; 5 = 512^3 grid, batch 4, 64 -> 64, bf16 inputs with
    fp32 sums and outputs.  Tables built on the device; time per product from HIP events."""
    cfg = args.conv_bench
    u, ci, co, bf = {3: (128, 32, 64, False), 5: (512, 64, 64, True)}[cfg]
    coords, offs, _ = S.config_batch(cfg)
    lv = hch.hch_build_levels_device(coords, offs, u, 1)
    n = lv.n(0)
    algo = {"fused": hch.HCH_ALGO_FUSED, "fused_dense": hch.HCH_ALGO_FUSED_DENSE, "columns": hch.HCH_ALGO_COLUMNS}[args.algo]
    DT = hch.HCH_BF16 if bf else hch.HCH_F32
    if bf and not args.no_tap_major:
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
    flop = 2.0 * n * 27 * ci * co
    out = {}
    for name, fn in calls:
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        out[name] = {"ms": round(ms, 4), "tflops": round(flop / ms / 1e9, 1)}
    print(json.dumps({"metric": f"one 3x3x3 convolution {ci} -> {co}: time per product", "unit": "ms",
                      "products": out, "calls_timed": args.steps, "higher_is_better": False,
                      "dtype": "bf16" if bf else "f32", "data": "synthetic", "algo": args.algo,
                      "config": {"workload": f"{u}^3 grid, batch {len(offs) - 1}, random-primitive surfaces, {n} voxels"}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--resolution", type=int, default=256, help="finest grid side (256 = the headline workload)")
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-all", action="store_true", help="time every kernel (adds event overhead)")
    ap.add_argument("--no-other-algo", action="store_true", help="skip the second, fully timed pass")
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
    ap.add_argument("--algo", choices=["columns", "fused", "fused_dense"], default="fused",
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
        conv_bench(args, torch, hch, S)
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
    algo = {"fused": hch.HCH_ALGO_FUSED, "fused_dense": hch.HCH_ALGO_FUSED_DENSE, "columns": hch.HCH_ALGO_COLUMNS}[args.algo]
    enc = Encoder(levels, CHANNELS, algo, two_streams=args.two_streams)
    enc.X[0].copy_(torch.from_numpy(X0))
    for l in range(5):
        enc.W[l].copy_(torch.from_numpy(W[l]))
    enc.dX[5].copy_(torch.from_numpy(S.gaussian((enc.n[5], CHANNELS[5]), 1.0, 4100)))
    torch.cuda.synchronize()

    def kernel_table():
        out = {}
        for i in range(hch.hch_kernel_count()):
            st = hch.hch_profile_read(i)
            if st["launches"]:
                out[hch.hch_kernel_name(i)] = (i, st)
        return out

    def roofline_of(name, st, steps):
        """achieved = algorithmic bytes (or flops) of the timed launches / their event-measured
        time; a kernel counts as MFMA-bound when its arithmetic intensity is above the ridge."""
        ai = st["flops"] / max(1.0, st["bytes"])
        if "gemm" in name and ai >= MFMA_F32_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
            bound, achieved, peak, unit = "mfma", st["flops"] / (st["ms"] * 1e-3) / 1e12, MFMA_F32_PEAK_TFLOPS, "TFLOP/s"
        else:
            bound, achieved, peak, unit = "hbm", st["bytes"] / (st["ms"] * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
        return {"kernel": name, "bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": traffic_of(name),
                "launches_per_step": st["launches"] / steps,
                "avg_launch_ms": round(st["ms"] / max(1, st["launches"]), 5),
                "algorithmic_bytes_per_launch": round(st["bytes"] / max(1, st["launches"])),
                "flops_per_launch": round(st["flops"] / max(1, st["launches"]))}

    def load_traffic(algo_name):
        """kernel -> HBM bytes per launch, from the committed rocprofv3 --pmc summary of this
        workload (FETCH_SIZE + WRITE_SIZE, calibrated on a copy kernel); the counters cannot be
        read from inside this process."""
        db = {}
        path = os.path.join(ROOT, "profiles", f"hbm_traffic_encoder_{u}x{b}_{algo_name}.txt")
        if os.path.exists(path):
            for line in open(path):
                parts = [x.strip() for x in line.split("|")]
                if line.startswith("#") or len(parts) != 5:
                    continue
                try:
                    db[parts[0]] = float(parts[4])
                except ValueError:
                    pass
        return db

    traffic_db = {a: load_traffic(a) for a in ("fused", "columns")}

    def traffic_of(name):
        return traffic_db.get(args.algo, {}).get(name)

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
    value = flops / (ms_per_step * 1e-3) / 1e12
    roofline = roofline_of(dom_name, hch.hch_profile_read(dominant), args.steps)

    out = {
        "metric": "sparse conv fwd+bwd TFLOP/s and gather/scatter HBM GB/s, 256^3 grid, batch 8",
        "value": round(value, 4), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"5-level encoder fwd+bwd, {u}^3 grid, batch {b}, random-primitive surfaces, "
                               f"channels 4-16-32-64-128-256, N per level = {enc.n}",
                   "algo": args.algo, "flop_count": "paper-method 3 * 2*27*c_in*c_out*N_l per level",
                   "gflop_per_step": round(flops / 1e9, 3), "psh_build_s": round(t_build, 3), "psh_build_device_s": round(t_build_dev, 3),
                   "shape_gen_s": round(t_gen, 2)},
        "roofline": roofline,
        "kernels_ms_first_step": {k: round(v[1]["ms"], 4) for k, v in first.items()},
    }

    if not args.two_streams and not args.no_overlap_pass:
        # the same steps with the weight gradients and the coarse levels' index lists on a second
        # stream: whole-step throughput when independent kernels share the chip
        enc3 = Encoder(levels, CHANNELS, algo, two_streams=True)
        enc3.X[0].copy_(enc.X[0]); enc3.dX[5].copy_(enc.dX[5])
        for l in range(5):
            enc3.W[l].copy_(enc.W[l])
        for _ in range(max(1, args.warmup)):
            enc3.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            enc3.step()
        torch.cuda.synchronize()
        dt3 = time.perf_counter() - t0
        out["two_streams"] = {"ms_per_step": round(dt3 / args.steps * 1e3, 4),
                              "value": round(flops / (dt3 / args.steps) / 1e12, 4), "unit": "TFLOP/s"}
        del enc3

    if not args.no_other_algo:
        # the other algorithm on the same inputs, every kernel timed (event overhead included in
        # its step time): per-kernel rooflines of the gather, GEMM and scatter kernels
        other = "columns" if args.algo == "fused" else "fused"
        enc2 = Encoder(levels, CHANNELS, hch.HCH_ALGO_COLUMNS if other == "columns" else hch.HCH_ALGO_FUSED)
        enc2.X[0].copy_(enc.X[0]); enc2.dX[5].copy_(enc.dX[5])
        for l in range(5):
            enc2.W[l].copy_(enc.W[l])
        for _ in range(2):
            enc2.step()
        torch.cuda.synchronize()
        hch.hch_profile_reset()
        hch.hch_profile_enable(-1, True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            enc2.step()
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t0
        hch.hch_profile_enable(-1, False)
        save_algo, args.algo = args.algo, other
        tab = kernel_table()
        out["other_algo"] = {
            "algo": other, "ms_per_step_all_kernels_timed": round(dt2 / args.steps * 1e3, 4),
            "value": round(flops / (dt2 / args.steps) / 1e12, 4), "unit": "TFLOP/s",
            "kernels": [roofline_of(k, v[1], args.steps) for k, v in
                        sorted(tab.items(), key=lambda kv: -kv[1][1]["ms"])
                        if any(t in k for t in ("hash2col", "col2hash", "gemm", "neighbour"))],
        }
        args.algo = save_algo
    if not args.no_cpu_baseline:
        v, cores, note = cpu_baseline(coords, offs, X0, W, u, b)
        out["cpu_baseline"] = {"value": round(v, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                               "sample": note}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
