#!/usr/bin/env python3
"""Benchmark of the table-lookup conv2d hot path on one MI355X.

One "step" is one pass over the ResNet-50-shaped workload (53 convolutions + the 2048x1000
classifier, batch 32, every layer on its own seeded synthetic input resident in HBM, the
truncated-multiplier table with the 6 low partial-product columns removed; filters and table
prepared once per layer, as they do not change between batches).  Prints ONE JSON line:
whole-job LUT-MACs/s, the roofline of the dominant kernel (measured live with HIP events
around that kernel on the launch stream) and the CPU oracle timed on a bounded sample of the
same workload.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def kernel_sources_hash():
    """sha256 over the HIP sources of the library, in name order."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2002_09481_amd", "csrc", "*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--cpu-batch", type=int, default=32, help="images per layer for the oracle timing (0 = skip)")
    ap.add_argument("--no-check", action="store_true", help="skip the sampled parity check")
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary workloads (configs 2, 4, 5)")
    ap.add_argument("--probe", action="store_true", help="only run the LDS / copy micro-benchmarks and print a table")
    ap.add_argument("--per-layer", action="store_true", help="only time every layer of the workload and print a table")
    return ap.parse_args()


def probe_table(ax, torch):
    """LDS gather rates (the denominators of the roofline) and copy bandwidth, as markdown."""
    a = torch.randn(4096, 4096, device="cuda")
    t = time.time()
    while time.time() - t < 1.0:  # let the clocks ramp up
        (a @ a).sum().item()
    names = {0: "consecutive (conflict-free)", 1: "uniform random", 2: "random, half of the lanes on entry 0",
             3: "random entries of 16 interleaved tables, table = lane % 16",
             4: "random entries of 16 interleaved tables, table = (lane / 4) % 16",
             5: "random entries of 16 interleaved tables, table = lane % 8 + 8 * ((lane / 32) % 2)",
             6: "random entries of 16 interleaved tables, table = lane % 4 + 4 * ((lane / 16) % 4)"}
    print("| read width | pattern | table | T lanes/s | TB/s | lookups per lane |")
    print("|---|---|---|---|---|---|")
    for width in (2, 4, 8, 16):
        for pat in (0, 1, 2) + ((3, 4, 5, 6) if width == 16 else ()):
            for tb in ((32768,) if pat == 0 else (65536,) if pat >= 3 else (4096, 131072)):
                r = ax.ax_probe_lds_gather(width, pat, tb, 1024, 20000 if width < 16 else 10000)
                lanes = r["wave_reads"] * r["workgroups"] * 64 / r["seconds"]
                print("| %d B | %s | %d KiB | %.2f | %.1f | %d |" % (width, names[pat], tb // 1024, lanes / 1e12,
                                                                  lanes * width / 1e12, max(1, width // 2)))
    nb = 1 << 30
    x = torch.empty(nb, dtype=torch.uint8, device="cuda")
    y = torch.empty(nb, dtype=torch.uint8, device="cuda")
    ax.ax_probe_copy(y, x)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        ax.ax_probe_copy(y, x)
    e1.record()
    torch.cuda.synchronize()
    print("\ncopy kernel, 1 GiB: %.1f GB/s (read + write)" % (2 * nb * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2002_09481_amd import binding as ax
    from paper_2002_09481_amd import inputs as I

    if not os.path.exists(ax.LIB_PATH):
        from paper_2002_09481_amd import build as hip_build
        hip_build.build()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.probe:
        probe_table(ax, torch)
        return

    layers = I.config_resnet50(args.batch)
    lut = I.lut_truncated(6)
    lut_d = ax.lut_to_device(lut)

    # ---- operands resident in HBM, filters and table prepared, before anything is timed -----
    # Every layer is a handle: its filters and the multiplier table do not change from batch to
    # batch, so the re-laid-out table, the packed filters and their sums are made once
    # (ax_layer_prepare) and a step only runs what depends on the activations.
    t_gen = time.time()
    calls = []
    host = []
    for idx, l in enumerate(layers):
        x, w, q = I.make_operands(l, I.layer_seed(3, idx))
        xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
        if l.dense:
            xd, wd = xd.view(l.N, l.K), wd.view(l.K, l.Cout)
            desc = ax._dense_desc(l.N, l.K, l.Cout)
        else:
            desc = ax._conv_desc(x.shape, w.shape, l.stride, l.pad)
        h = ax.AxLayer(desc, q)
        h.prepare(wd, lut_d)
        acc = torch.empty(h.out_shape(), dtype=torch.int32, device=dev)
        y = torch.empty(acc.shape, dtype=torch.float32, device=dev)
        ws = torch.empty(max(256, h.workspace_bytes), dtype=torch.uint8, device=dev)
        calls.append((l, h, xd, wd, q, acc, y, ws))
        host.append((x, w, q) if not args.no_check else None)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen
    total_macs = sum(l.macs for l in layers)

    def step():
        for l, h, xd, wd, q, acc, y, ws in calls:
            h.run(xd, acc, y, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = e0.elapsed_time(e1) / args.steps
    value = total_macs / (ms_per_step * 1e-3)

    # the same step through the one-call entry points, which prepare the constants in every call
    def step_one_call():
        for l, h, xd, wd, q, acc, y, ws1 in calls1:
            if l.dense:
                ax.ax_dense(xd, wd, lut_d, q, acc, y, ws1)
            else:
                ax.ax_conv2d(xd, wd, lut_d, l.stride, l.pad, q, acc, y, ws1)

    calls1 = []
    for l, h, xd, wd, q, acc, y, ws in calls:
        need = ax.ax_dense_workspace_bytes(l.N, l.K, l.Cout) if l.dense else \
            ax.ax_conv2d_workspace_bytes((l.N, l.H, l.W, l.Cin), (l.KH, l.KW, l.Cin, l.Cout), l.stride, l.pad)
        calls1.append((l, h, xd, wd, q, acc, y, torch.empty(max(256, need), dtype=torch.uint8, device=dev)))
    step_one_call()
    torch.cuda.synchronize()
    o0, o1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    o0.record()
    for _ in range(max(1, args.steps // 2)):
        step_one_call()
    o1.record()
    torch.cuda.synchronize()
    ms_one_call = o0.elapsed_time(o1) / max(1, args.steps // 2)
    del calls1

    # ---- dominant kernel: HIP events around the main kernel of every layer (measurement helper
    # of the library: eight launches between the two events, so that their own cost is diluted) ---
    kern_ms = []
    for rep in range(3):
        kern_ms.append([h.kernel_ms(xd, acc, y, ws, reps=8) for l, h, xd, wd, q, acc, y, ws in calls])
    kern_ms = np.median(np.array(kern_ms), axis=0)
    main_ms = float(kern_ms.sum())
    n_launch = len(calls)

    if args.per_layer:
        # every layer on its own: whole call (per-call preparation, main kernel, fix-up) and main kernel
        print("| layer | M | K | Cout | lookups (G) | plan (variant, tile, workgroups, pieces, combine, tables) | call us | main kernel us | "
              "T lookups/s (call) | T lookups/s (kernel) |")
        print("|---|---|---|---|---|---|---|---|---|---|")
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        tot_call = 0.0
        for (l, h, xd, wd, q, acc, y, ws), km in zip(calls, kern_ms):
            for _ in range(3):
                h.run(xd, acc, y, ws)
            torch.cuda.synchronize()
            a0.record()
            for _ in range(20):
                h.run(xd, acc, y, ws)
            a1.record()
            torch.cuda.synchronize()
            cm = a0.elapsed_time(a1) / 20
            tot_call += cm
            p = h.plan()
            print("| %s | %d | %d | %d | %.3f | %d, %d, %d, %d, %d, %d | %.1f | %.1f | %.2f | %.2f |" % (
                l.name, l.M, l.K, l.Cout, l.macs / 1e9, p["variant"], p["tile"], p["workgroups"], p["pieces"],
                p["combine"], p["tables"], cm * 1e3,
                km * 1e3, l.macs / cm / 1e9, l.macs / km / 1e9))
        print("\nsum of the calls timed one layer at a time: %.3f ms; the same 54 calls back to back in a step: %.3f ms; "
              "main kernels: %.3f ms" % (tot_call, ms_per_step, main_ms))
        return

    # measured denominators: LDS lookup rates and copy bandwidth on this device
    r_cf = ax.ax_probe_lds_gather(2, 0, 131072, 1024, 20000)
    r_rand = ax.ax_probe_lds_gather(2, 1, 131072, 1024, 8000)
    r_cf16 = ax.ax_probe_lds_gather(16, 0, 32768, 1024, 20000)
    r_rand16 = ax.ax_probe_lds_gather(16, 1, 4096, 1024, 8000)
    lookups = lambda r: r["wave_reads"] * r["workgroups"] * 64 / r["seconds"]
    lds_peak, lds_rand = lookups(r_cf), lookups(r_rand)
    lds_wide, lds_wide_rand = 8 * lookups(r_cf16), 8 * lookups(r_rand16)  # a 16-byte entry holds 8 products
    nb = 1 << 30
    a = torch.empty(nb, dtype=torch.uint8, device=dev)
    b = torch.empty(nb, dtype=torch.uint8, device=dev)
    ax.ax_probe_copy(b, a)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        ax.ax_probe_copy(b, a)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * nb * 5 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del a, b

    alg_bytes = sum(l.algorithmic_bytes for l in layers)
    kern_rate = total_macs / (main_ms * 1e-3)  # lookup-MACs per second inside the dominant kernel
    # Vector-instruction issue.  In the K loop of the compiled kernel a wave executes, per 16-tap
    # chunk, 1200 vector instructions for 1024 lookups per lane (32-column tile; 614 of them in
    # 64-bit encodings: v_sad_u16, v_perm_b32 ...) or 652 for 512 lookups (16-column tile; 326 in
    # 64-bit encodings).  Issue rates measured on this machine with every SIMD full (4 waves each):
    # 60.9 T lane-instructions/s for a 32-bit encoded add, 32.5 T/s for the 64-bit encoded forms.
    # valu_issue.frac = time those rates need for the K loops of all layers / measured kernel time.
    r32, r64 = 60.9e12, 32.5e12
    per_lookup = {3: (586 / 1024.0, 614 / 1024.0), 5: (326 / 512.0, 326 / 512.0)}
    need_s = 0.0
    for l, h, xd, wd, q, acc, y, ws in calls:
        n32, n64 = per_lookup.get(h.plan()["tile"], per_lookup[5])
        need_s += l.macs * (n32 / r32 + n64 / r64)
    valu_issue = {"frac": need_s / (main_ms * 1e-3),
                  "lane_instructions_per_lookup": {"tile_3": sum(per_lookup[3]), "tile_5": sum(per_lookup[5])},
                  "measured_issue_T_per_s": {"32_bit_encoded": r32 / 1e12, "64_bit_encoded": r64 / 1e12},
                  "note": "time the K loops of all main kernels need at the vector issue rates measured on this "
                          "machine, over the measured kernel time; the rest is barrier rendezvous, table building "
                          "waits, prologues and epilogues"}
    # HBM-side traffic of the dominant kernel comes from two rocprofv3 counter runs (FETCH_SIZE,
    # WRITE_SIZE) and cannot be read inside this process; the committed figure is only reported
    # while it belongs to the kernel sources that are running (it records their hash).
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            tj = json.load(open(tpath))
            if tj.get("kernel_sources_sha256") == kernel_sources_hash():
                traffic = tj.get("bytes_per_launch")
        except Exception:
            traffic = None
    # Bound of the kernel: the LDS.  A lookup-MAC reads 2 bytes of a 16-byte table entry and takes
    # one integer add; the measured conflict-free rate of 16-byte LDS gathers (8 products each)
    # gives fewer lookups per second than the integer-add peak, so it is the roofline.
    roofline = {
        "kernel": "tab_kernel (table-tile lookup-MAC kernel), %d launches per step" % n_launch,
        "bound": "lds",
        "achieved": kern_rate * 2 / 1e9,
        "peak": lds_wide * 2 / 1e9,
        "unit": "GB/s",
        "frac": kern_rate / lds_wide,
        "peak_source": "measured on this device: conflict-free 16-byte LDS gathers (ds_read_b128, one workgroup of "
                       "1024 threads per compute unit); a 16-byte entry holds 8 products, 2 bytes per lookup-MAC",
        "achieved_Glookup_s": kern_rate / 1e9,
        "peak_Glookup_s": lds_wide / 1e9,
        "avg_launch_ms": main_ms / n_launch,
        "algorithmic_lookups_per_launch": total_macs / n_launch,
        "algorithmic_lds_bytes_per_launch": 2 * total_macs / n_launch,
        "traffic": traffic,
        "frac_of_random_code_16_byte_gathers": kern_rate / lds_wide_rand,
        "whole_step_frac": value / lds_wide,
        "ratio_to_2_byte_gather_rate": {
            "value": kern_rate / lds_peak, "conflict_free_2_byte_Glookup_s": lds_peak / 1e9,
            "random_2_byte_Glookup_s": lds_rand / 1e9,
            "note": "a ratio, not a bound: one-product (2-byte) gathers, what a kernel with the whole table in LDS "
                    "would issue; this kernel fetches eight products per gather"},
        # 256 CUs x 4 SIMDs x 32 lanes per clock x 2.4 GHz (the 157.3 TFLOP/s fp32 vector figure is
        # two flops on each of these lanes); one integer add per lookup-MAC is the algorithmic minimum
        "alu": {"achieved": kern_rate / 1e12, "peak": 78.64, "unit": "Tint32-add/s", "frac": kern_rate / 78.64e12},
        "valu_issue": valu_issue,
        "hbm": {"achieved": alg_bytes / (main_ms * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                "frac": alg_bytes / (main_ms * 1e-3) / 8e12, "measured_copy_GBps": copy_gbs,
                "algorithmic_bytes_per_launch": alg_bytes / n_launch},
    }

    # ---- sampled parity against the oracle, in the configuration that was timed -------------
    parity = None
    if not args.no_check:
        from oracle import oracle
        rng = np.random.default_rng(0)
        parity = True
        for (l, h, xd, wd, q, acc, y, ws), (x, w, qq) in zip(calls, host):
            n_out = l.M * l.Cout
            idx = rng.integers(0, n_out, size=48)
            a_s, y_s = oracle.conv2d_sample(x, w, lut, l.stride, l.pad, qq, idx)
            ti = torch.from_numpy(idx).to(dev)
            a_g = acc.view(-1)[ti].cpu().numpy()
            y_g = y.view(-1)[ti].cpu().numpy()
            ok = np.array_equal(a_g, a_s) and np.all(np.abs(y_g.astype(np.float64) - y_s) <= 1e-5 * np.abs(y_s) + 1e-6)
            if not ok:
                parity = False
                print("bench.py: PARITY FAILURE in layer %s" % l.name, file=sys.stderr)

    # ---- the oracle, as it stands, on the host cores (bounded sample) ------------------------
    cpu = None
    if args.cpu_batch > 0:
        from oracle import oracle
        cl = I.config_resnet50(args.cpu_batch)
        if args.cpu_batch == args.batch and not args.no_check:
            ops = host  # the very tensors the GPU consumed
        else:
            ops = [I.make_operands(l, I.layer_seed(3, idx)) for idx, l in enumerate(cl)]
        t = time.perf_counter()
        for l, (x, w, q) in zip(cl, ops):
            if l.dense:
                oracle.dense(x.reshape(l.N, l.K), w.reshape(l.K, l.Cout), lut, q)
            else:
                oracle.conv2d(x, w, lut, l.stride, l.pad, q)
        dt = time.perf_counter() - t
        cmacs = sum(l.macs for l in cl)
        cpu = {"value": cmacs / dt, "unit": "LUT-MAC/s", "cores": oracle.threads(), "kind": "oracle",
               "per_core": cmacs / dt / max(1, oracle.threads()),
               "gpu_over_oracle": (total_macs / (ms_per_step * 1e-3)) / (cmacs / dt),
               "sample": "all 54 layers of the same workload at batch %d (%.2f G lookups, %.1f s)" % (
                   args.cpu_batch, cmacs / 1e9, dt),
               "images_per_s": args.cpu_batch / dt}

    # ---- secondary workloads (context; the headline stays the ResNet-50 sweep) ----------------
    extra = None
    if not args.no_extra:
        extra = {}

        def time_calls(fns, reps):
            for f in fns:
                f()
            torch.cuda.synchronize()
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record()
            for _ in range(reps):
                for f in fns:
                    f()
            a1.record()
            torch.cuda.synchronize()
            return a0.elapsed_time(a1) / reps

        def make_call(l, seed, lut_dev):
            x, w, q = I.make_operands(l, seed)
            xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
            if l.dense:
                xd, wd = xd.view(l.N, l.K), wd.view(l.K, l.Cout)
                acc = torch.empty((l.N, l.Cout), dtype=torch.int32, device=dev)
                ws = torch.empty(max(256, ax.ax_dense_workspace_bytes(l.N, l.K, l.Cout)), dtype=torch.uint8, device=dev)
                y = torch.empty(acc.shape, dtype=torch.float32, device=dev)
                return lambda lt=lut_dev: ax.ax_dense(xd, wd, lt, q, acc, y, ws)
            acc = torch.empty((l.N, l.OH, l.OW, l.Cout), dtype=torch.int32, device=dev)
            ws = torch.empty(max(256, ax.ax_conv2d_workspace_bytes(x.shape, w.shape, l.stride, l.pad)),
                             dtype=torch.uint8, device=dev)
            y = torch.empty(acc.shape, dtype=torch.float32, device=dev)
            return lambda lt=lut_dev: ax.ax_conv2d(xd, wd, lt, l.stride, l.pad, q, acc, y, ws)

        kept = []  # handles of the secondary workloads (freed with the process)

        def make_handle_call(l, seed, lut_dev):
            # the layer as a prepared handle, like the headline: constants laid out once, outside the timing
            x, w, q = I.make_operands(l, seed)
            xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
            h = ax.AxLayer(ax._conv_desc(x.shape, w.shape, l.stride, l.pad), q)
            h.prepare(wd, lut_dev)
            acc = torch.empty(h.out_shape(), dtype=torch.int32, device=dev)
            y = torch.empty(acc.shape, dtype=torch.float32, device=dev)
            ws = torch.empty(max(256, h.workspace_bytes), dtype=torch.uint8, device=dev)
            kept.append(h)
            return lambda: h.run(xd, acc, y, ws)

        # config 2: CIFAR-shaped stack, batch 128, random-error table
        l2 = I.config_resnet8_cifar(128)
        lut2 = ax.lut_to_device(I.lut_random_error(2000))
        ms = time_calls([make_handle_call(l, I.layer_seed(2, i), lut2) for i, l in enumerate(l2)], 50)
        ms_1c = time_calls([make_call(l, I.layer_seed(2, i), lut2) for i, l in enumerate(l2)], 50)
        m2 = sum(l.macs for l in l2)
        extra["config2_cifar_stack_b128"] = {"ms": ms, "lut_macs_per_s": m2 / ms * 1e3, "images_per_s": 128 / ms * 1e3,
                                             "ms_one_call_entry_points": ms_1c}
        # the same stack at the batch size the paper used for its CIFAR-10 runs (1000 images)
        l2k = I.config_resnet8_cifar(1000)
        ms_k = time_calls([make_handle_call(l, I.layer_seed(2, i), lut2) for i, l in enumerate(l2k)], 10)
        m2k = sum(l.macs for l in l2k)
        extra["config2_cifar_stack_b1000"] = {
            "ms": ms_k, "lut_macs_per_s": m2k / ms_k * 1e3, "images_per_s": 1000 / ms_k * 1e3,
            "context": "the paper's ResNet-8 (7 conv layers, 21 M MACs per image) took 1.5 s for 10^4 CIFAR-10 images "
                       "on a GTX 1080, about 0.14 T lookup-MAC/s; another network, machine and decade: context only"}
        # the stack chained from float tensors: every layer takes the ranges of its input (after
        # ReLU) and of its filters, quantizes both, runs the lookup-MAC convolution and hands its
        # float output to the next layer; nothing returns to the host in between
        try:
            xf0, _ = I.make_float_operands(l2k[0], I.layer_seed(2, 0))
            xf = torch.from_numpy(xf0).to(dev)
            wf = [torch.from_numpy(I.make_float_operands(l, I.layer_seed(2, i))[1]).to(dev) for i, l in enumerate(l2k)]
            yf = [torch.empty((l.N, l.OH, l.OW, l.Cout), dtype=torch.float32, device=dev) for l in l2k]
            wsf = [torch.empty(ax.ax_conv2d_f32_workspace_bytes((l.N, l.H, l.W, l.Cin), (l.KH, l.KW, l.Cin, l.Cout),
                                                                l.stride, l.pad), dtype=torch.uint8, device=dev)
                   for l in l2k]

            def chained():
                cur = xf
                for i, l in enumerate(l2k):
                    ax.ax_conv2d_f32(cur, wf[i], lut2, l.stride, l.pad, None, None, relu=i > 0, acc_out=False,
                                     y_out=yf[i], workspace=wsf[i])
                    cur = yf[i]
            ms_c = time_calls([chained], 10)
            extra["config2_cifar_stack_b1000_chained_float"] = {
                "ms": ms_c, "lut_macs_per_s": m2k / ms_c * 1e3, "images_per_s": 1000 / ms_c * 1e3,
                "note": "float32 in, seven chained layers with ReLU, ranges and quantization on the device"}
        except Exception as e:  # never lose the main line
            extra["config2_cifar_stack_b1000_chained_float"] = {"error": repr(e)}
        # the same seven calls captured once into a HIP graph and replayed (the calls only enqueue
        # kernels, so nothing but launch overhead changes)
        try:
            c2 = [make_handle_call(l, I.layer_seed(2, i), lut2) for i, l in enumerate(l2)]
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for f in c2:
                    f()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                for f in c2:
                    f()
            ms_g = time_calls([g2.replay], 50)
            extra["config2_cifar_stack_b128"]["ms_hip_graph_replay"] = ms_g
            del g2, c2
        except Exception as e:  # capture support is not needed for any other number
            extra["config2_cifar_stack_b128"]["ms_hip_graph_replay"] = "capture failed: %s" % e
        # config 4: two layers against 64 tables back to back (tables resident in HBM; every call
        # re-lays-out and re-stages its table)
        l4 = I.config_lut_sweep(64)
        luts = [ax.lut_to_device(I.lut_random_error(sd)) for sd in range(64)]
        c4 = [make_call(l, I.layer_seed(4, i), luts[0]) for i, l in enumerate(l4)]
        fns = [(lambda lt=lt, c=c: c(lt)) for lt in luts for c in c4]
        ms = time_calls(fns, 3)
        m4 = sum(l.macs for l in l4) * 64
        extra["config4_lut_sweep_64_tables"] = {"ms": ms, "lut_macs_per_s": m4 / ms * 1e3, "tables_per_s": 64 / ms * 1e3}
        # the same, with every table's 128 KB host-to-device copy (from page-locked host memory) inside
        # the timed region: (a) enqueued on the compute stream in front of the table's two layers,
        # (b) on a second stream, overlapping the layers that run on the previous table
        # (sweep.TableSweep: two staging buffers, event-ordered).  Both go through layer handles
        # (prepare + run per table and layer), like (c), the tables resident in device memory.
        from paper_2002_09481_amd.sweep import TableSweep
        host_all = torch.from_numpy(np.stack([np.ascontiguousarray(I.lut_random_error(sd)).reshape(-1)
                                              for sd in range(64)]).view(np.int16).copy()).pin_memory()
        sw_layers = []
        for i, l in enumerate(l4):
            x, w, q = I.make_operands(l, I.layer_seed(4, i))
            sw_layers.append((ax._conv_desc(x.shape, w.shape, l.stride, l.pad), q, torch.from_numpy(x).to(dev),
                              torch.from_numpy(w).to(dev)))
        for chunk, tag in ((1, "per_table"), (8, "eight_tables_per_call")):
            sw = TableSweep(sw_layers, chunk=chunk)
            acc_sw = [torch.empty(sw.out_shape(li, 64), dtype=torch.int32, device=dev) for li in range(len(l4))]
            y_sw = [torch.empty(sw.out_shape(li, 64), dtype=torch.float32, device=dev) for li in range(len(l4))]
            ms_ser = time_calls([lambda: sw.run(host_all, acc_sw, y_sw, overlap=False)], 3)
            ms_ovl = time_calls([lambda: sw.run(host_all, acc_sw, y_sw, overlap=True)], 3)
            # tables already in device memory: the same handles, prepare + run per chunk
            resident = host_all.to(dev)

            def run_resident():
                for t0 in range(0, 64, chunk):
                    for li in range(len(l4)):
                        h = sw._handle(li, chunk)
                        h.prepare(sw_layers[li][3], resident[t0:t0 + chunk], prepared=sw._blocks[(li, chunk, 0)])
                        a, yy = acc_sw[li][t0:t0 + chunk], y_sw[li][t0:t0 + chunk]
                        h.run(sw_layers[li][2], a[0] if chunk == 1 else a, yy[0] if chunk == 1 else yy,
                              workspace=sw._ws[(li, chunk)])
            ms_res = time_calls([run_resident], 3)
            extra["config4_lut_sweep_64_tables_handles_" + tag] = {
                "ms_tables_resident": ms_res, "ms_upload_on_compute_stream": ms_ser, "ms_upload_overlapped": ms_ovl,
                "overlapped_over_resident": ms_ovl / ms_res, "lut_macs_per_s_overlapped": m4 / ms_ovl * 1e3,
                "tables_per_s_overlapped": 64 / ms_ovl * 1e3}
            sw.close()
            del acc_sw, y_sw, resident
        host_luts = [host_all[sd] for sd in range(64)]
        stage = torch.empty(65536, dtype=torch.int16, device=dev)

        def with_upload(h):
            stage.copy_(h, non_blocking=True)
            for c in c4:
                c(stage)

        ms = time_calls([(lambda h=h: with_upload(h)) for h in host_luts], 3)
        extra["config4_lut_sweep_64_tables_upload_in_timing"] = {"ms": ms, "lut_macs_per_s": m4 / ms * 1e3,
                                                                 "tables_per_s": 64 / ms * 1e3}
        # the same sweep through ax_conv2d_multi_lut: one call per layer for all 64 tables (operands
        # prepared once, the tiles of all tables share one grid)
        luts_all = torch.stack(luts)
        mcalls = []
        for i, l in enumerate(l4):
            x, w, q = I.make_operands(l, I.layer_seed(4, i))
            xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
            acc = torch.empty((64, l.N, l.OH, l.OW, l.Cout), dtype=torch.int32, device=dev)
            y = torch.empty(acc.shape, dtype=torch.float32, device=dev)
            ws = torch.empty(ax.ax_conv2d_multi_lut_workspace_bytes(x.shape, w.shape, 64, l.stride, l.pad),
                             dtype=torch.uint8, device=dev)
            mcalls.append(lambda xd=xd, wd=wd, q=q, acc=acc, y=y, ws=ws, l=l: ax.ax_conv2d_multi_lut(
                xd, wd, luts_all, l.stride, l.pad, q, acc, y, ws))
        ms = time_calls(mcalls, 3)
        extra["config4_lut_sweep_64_tables_one_call_per_layer"] = {"ms": ms, "lut_macs_per_s": m4 / ms * 1e3,
                                                                   "tables_per_s": 64 / ms * 1e3}
        del mcalls
        # config 5: GEMM-shaped layers, truncated table
        l5 = I.config_gemm_shaped()
        ms = time_calls([make_call(l, I.layer_seed(5, i), lut_d) for i, l in enumerate(l5)], 20)
        m5 = sum(l.macs for l in l5)
        extra["config5_gemm_shaped"] = {"ms": ms, "lut_macs_per_s": m5 / ms * 1e3}
        # run time must not depend on the table's content, but it does depend on the operands'
        # distribution (LDS bank conflicts): the same two layers with the exact table, and one 3x3
        # layer with uniform codes against ReLU-distributed codes (about half of them equal)
        lut_exact_d = ax.lut_to_device(I.lut_exact())
        ms_exact = time_calls([make_call(l, I.layer_seed(5, i), lut_exact_d) for i, l in enumerate(l5)], 20)
        extra["config5_gemm_shaped"]["ms_exact_table"] = ms_exact
        dep = {}
        for dist in ("uniform", "relu"):
            ld = I.Layer("dep." + dist, args.batch, 28, 28, 128, 3, 3, 128, 1, 1, x_dist=dist,
                         w_dist="uniform" if dist == "uniform" else "normal")
            dep[dist] = time_calls([make_call(ld, 99, lut_d)], 20)
        extra["operand_distribution_3x3_28x28x128"] = {"ms_uniform_codes": dep["uniform"], "ms_relu_codes": dep["relu"]}

        # operator variants: one ResNet-50 3x3 layer in unsigned, signed and dilated form, and two
        # depthwise layers of MobileNet size (whole table in LDS, HBM-bound on the outputs)
        def time_ex(x, w, lut_np, stride, pad, q, dilation=1, depthwise=False, reps=20):
            xd, wd, ld = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev), ax.lut_to_device(lut_np)
            acc, y = ax.ax_conv2d_ex(xd, wd, ld, stride, pad, q, dilation=dilation, depthwise=depthwise)
            wsz = ax.lib().ax_conv2d_ex_workspace_bytes(ax.ax_conv_desc_t(
                x.shape[0], x.shape[1], x.shape[2], x.shape[3], w.shape[0], w.shape[1],
                x.shape[3] * w.shape[3] if depthwise else w.shape[3], stride, stride, pad, pad, dilation, dilation,
                int(depthwise), int(x.dtype == np.int8)), None)
            ws = torch.empty(max(256, int(wsz)), dtype=torch.uint8, device=dev)
            return time_calls([lambda: ax.ax_conv2d_ex(xd, wd, ld, stride, pad, q, dilation=dilation,
                                                       depthwise=depthwise, acc_out=acc, y_out=y, workspace=ws)], reps)

        vr = np.random.default_rng(77)
        var = {}
        shp = (args.batch, 56, 56, 64)
        xu = vr.integers(0, 256, shp).astype(np.uint8)
        wu = vr.integers(0, 256, (3, 3, 64, 64)).astype(np.uint8)
        xs_ = (xu.astype(np.int16) - 128).astype(np.int8)
        ws_ = (wu.astype(np.int16) - 128).astype(np.int8)
        macs = args.batch * 56 * 56 * 64 * 64 * 9
        for name, ms in (("conv3x3_56x56x64_unsigned", time_ex(xu, wu, I.lut_random_error(1), 1, 1, I.Quant(0.02, 3, 0.01, 128, None))),
                         ("conv3x3_56x56x64_signed", time_ex(xs_, ws_, I.lut_signed_random_error(1), 1, 1, I.Quant(0.02, -125, 0.01, 0, None))),
                         ("conv3x3_56x56x64_dilation2", time_ex(xu, wu, I.lut_random_error(1), 1, 2, I.Quant(0.02, 3, 0.01, 128, None), dilation=2))):
            var[name] = {"ms": ms, "lut_macs_per_s": macs / ms * 1e3}
        for hw, c in ((112, 32), (56, 128)):
            xdw = vr.integers(0, 256, (args.batch, hw, hw, c)).astype(np.uint8)
            wdw = vr.integers(0, 256, (3, 3, c, 1)).astype(np.uint8)
            ms = time_ex(xdw, wdw, I.lut_random_error(1), 1, 1, I.Quant(0.02, 3, 0.01, 128, None), depthwise=True)
            n_out = args.batch * hw * hw * c
            byts = xdw.size + wdw.size + 131072 + 8 * n_out
            var["depthwise3x3_%dx%dx%d" % (hw, hw, c)] = {
                "ms": ms, "lut_macs_per_s": n_out * 9 / ms * 1e3,
                "roofline": {"bound": "hbm", "achieved": byts / ms / 1e6, "peak": 8000.0, "unit": "GB/s",
                             "frac": byts / ms / 1e6 / 8000.0, "algorithmic_bytes": byts,
                             "lds_random_gather_Glookup_s": lds_rand / 1e9,
                             "frac_of_lds_random_2_byte_gather_rate": n_out * 9 / ms * 1e3 / lds_rand}}
        extra["variants_batch%d" % args.batch] = var

        # backward pass (straight-through: gradients of the exact convolution of the dequantized
        # tensors) of the 53 convolutions of the sweep, both gradients, on the matrix cores
        bw = []
        for l, h, xd, wd, q, acc, y, ws in calls:
            if l.dense:
                continue
            desc = ax._conv_desc((l.N, l.H, l.W, l.Cin), (l.KH, l.KW, l.Cin, l.Cout), l.stride, l.pad)
            gy = torch.randn((l.N, l.OH, l.OW, l.Cout), device=dev)
            gx = torch.empty((l.N, l.H, l.W, l.Cin), dtype=torch.float32, device=dev)
            gw = torch.empty((l.KH, l.KW, l.Cin, l.Cout), dtype=torch.float32, device=dev)
            wsb = torch.empty(int(ax.lib().ax_conv2d_backward_workspace_bytes(desc)), dtype=torch.uint8, device=dev)
            bw.append((l, xd, wd, q, gy, gx, gw, wsb))

        def bstep():
            for l, xd, wd, q, gy, gx, gw, wsb in bw:
                ax.ax_conv2d_backward(xd, wd, gy, l.stride, l.pad, q, gx_out=gx, gw_out=gw, workspace=wsb)
        ms_b = time_calls([bstep], 3)

        def bstep_net():  # as a network's backward pass runs: the images need no gradient
            for i, (l, xd, wd, q, gy, gx, gw, wsb) in enumerate(bw):
                ax.ax_conv2d_backward(xd, wd, gy, l.stride, l.pad, q, gx_out=False if i == 0 else gx, gw_out=gw, workspace=wsb)
        ms_bn = time_calls([bstep_net], 3)
        flops_b = sum(4.0 * l.macs for l, *_ in bw)  # two gradients, two flops per multiply-add
        extra["backward_resnet50_convs_batch%d" % args.batch] = {
            "ms": ms_b, "useful_TFLOP_s": flops_b / ms_b / 1e9,
            "ms_without_the_input_gradient_of_the_first_layer": ms_bn,
            "roofline": {"bound": "mfma", "achieved": flops_b / ms_b / 1e9, "peak": 2500.0 / 3.0, "unit": "TFLOP/s",
                         "frac": flops_b / ms_b / 1e9 / (2500.0 / 3.0),
                         "note": "useful float32-equivalent flops; every product takes three bf16 matrix "
                                 "instructions (gy split into three exact bf16 pieces), so the bound is a third of "
                                 "the dense bf16 peak of 2.5 PFLOP/s"},
            "forward_ms_same_layers": ms_per_step}
        del bw

    # ---- float-in / float-out form of the same sweep (range + quantization glue included) ------
    float_layer = None
    if not args.no_extra:
        fcalls = []
        n_x = n_w = 0
        for l, h, xd, wd, q, acc, y, ws in calls:
            # real-valued tensors with the sweep's distributions: the dequantized operands
            xf = ((xd.float() - q.x_zp) * q.x_scale).contiguous()
            wf = ((wd.float() - q.w_zp) * q.w_scale).contiguous()
            n_x += xf.numel()
            n_w += wf.numel()
            if l.dense:
                need = ax.ax_dense_f32_workspace_bytes(l.N, l.K, l.Cout)
            else:
                need = ax.ax_conv2d_f32_workspace_bytes((l.N, l.H, l.W, l.Cin), (l.KH, l.KW, l.Cin, l.Cout), l.stride, l.pad)
            wsf = torch.empty(need, dtype=torch.uint8, device=dev)
            fcalls.append((l, xf, wf, acc, y, wsf))

        def fstep():  # ranges of both tensors are taken inside the layer call, once per call
            for l, xf, wf, acc, y, wsf in fcalls:
                if l.dense:
                    ax.ax_dense_f32(xf, wf, lut_d, None, None, False, 0, acc, y, wsf)
                else:
                    ax.ax_conv2d_f32(xf, wf, lut_d, l.stride, l.pad, None, None, False, 0, acc, y, wsf)

        for _ in range(2):
            fstep()
        torch.cuda.synchronize()
        f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        freps = max(1, args.steps // 2)
        f0.record()
        for _ in range(freps):
            fstep()
        f1.record()
        torch.cuda.synchronize()
        fms = f0.elapsed_time(f1) / freps
        del fcalls
        # the two glue kernels alone on one large tensor (HBM-bound: 4 B/element read for the
        # range, 4 B read + 1 B written for the quantization)
        nbig = 1 << 28
        big = torch.empty(nbig, dtype=torch.float32, device=dev).normal_()
        codes = torch.empty(nbig, dtype=torch.uint8, device=dev)
        rr = torch.empty(2, dtype=torch.float32, device=dev)
        cc = torch.empty(2, dtype=torch.int32, device=dev)
        rws = torch.empty(ax.ax_range_workspace_bytes(nbig), dtype=torch.uint8, device=dev)

        def timed(fn, reps=10):
            fn()
            torch.cuda.synchronize()
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            g0.record()
            for _ in range(reps):
                fn()
            g1.record()
            torch.cuda.synchronize()
            return g0.elapsed_time(g1) / reps

        r_ms = timed(lambda: ax.ax_range_f32(big, False, rr, rws))
        q_ms = timed(lambda: ax.ax_quantize_f32(big, rr, False, 0, codes, cc))
        del big, codes
        glue_bytes = 2 * 4 * (n_x + n_w) + (n_x + n_w)  # range pass + quantization pass over both operands
        float_layer = {
            "workload": "the same 54 layers with float32 activations and filters: per layer the range and the "
                        "quantization of both tensors (one launch each), the lookup-MAC convolution and dequantization",
            "ms_per_step": fms,
            "lut_macs_per_s": total_macs / (fms * 1e-3),
            "images_per_s": args.batch / (fms * 1e-3),
            "glue_ms_per_step": fms - ms_per_step,
            "glue_algorithmic_bytes_per_step": glue_bytes,
            "range_kernel": {"bound": "hbm", "achieved": 4 * nbig / (r_ms * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                             "frac": 4 * nbig / (r_ms * 1e-3) / 8e12, "elements": nbig, "ms": r_ms},
            "quantize_kernel": {"bound": "hbm", "achieved": 5 * nbig / (q_ms * 1e-3) / 1e9, "peak": 8000.0,
                                "unit": "GB/s", "frac": 5 * nbig / (q_ms * 1e-3) / 8e12, "elements": nbig, "ms": q_ms},
            "measured_copy_GBps": copy_gbs,
        }

    out = {
        "metric": "LUT-MACs/s (ResNet-50 shapes)",
        "value": value,
        "unit": "LUT-MAC/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8 codes x u16 table -> int32",
        "data": "synthetic",
        "config": {"workload": "configs[2]: ResNet-50-shaped inference, 53 conv + FC, batch %d, 224x224x3, "
                               "truncated-multiplier table (6 low partial-product columns removed)" % args.batch,
                   "global_batch": args.batch, "layers": len(layers), "lut_macs_per_step": total_macs},
        "images_per_s": args.batch / (ms_per_step * 1e-3),
        "frac_of_lds_roofline": value / lds_wide,
        "ms_per_step_one_call_entry_points": ms_one_call,
        "main_kernel_ms_per_step": main_ms,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity_sampled": parity,
        "paper_context": "the paper reports about 200x for its GPU version (GTX 1080) over its optimized CPU version "
                         "(Xeon E5-2620) on CIFAR-10 ResNets; other hardware and workload, not a target",
        "other_workloads": extra,
        "float_layer": float_layer,
        "wall_s_timed_region": wall,
        "input_generation_s": t_gen,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
