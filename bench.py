#!/usr/bin/env python3
"""Benchmark of the sparse pointwise convolution path on one MI355X.

Workload (config.workload): the 13 pointwise 1x1 convolutions of a MobileNetV1-shaped
network at 224x224 input, batch 32, V=4, 90 % of the 4x1 weight blocks dropped
(exact count per layer, seeded), weights N(0, 0.1), inputs ReLU(N(0, 1)), fp32.
One "step" = one alcs_sparse_conv launch per layer, all 13 layers, inputs and packed
weights already resident in HBM.  value = dense-equivalent GFLOP/s of the whole step
(2*N*Ho*Wo*Cout*Cin per layer, as if nothing were pruned, divided by the step time).

Prints one JSON line on stdout; a per-layer table goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_FP32_PEAK_TFLOPS = 157.3  # MI355X dense fp32 matrix peak, published


def layer_bytes(L, nnzb):
    """Algorithmic bytes of one call: X once, Y once, the grouped CSR once."""
    packed = 4 * (L.G + 1) + 4 * nnzb + 4 * L.V * nnzb
    return L.x_bytes() + L.y_bytes() + packed


def layer_flops(L, nnzb):
    """Algorithmic flops: two per multiply-accumulate of a kept weight."""
    return 2.0 * L.N * L.Ho * L.Wo * L.V * nnzb


def kernel_symbol(L, info):
    """Name of the kernel template instance a launch used, as rocprofv3 prints it."""
    b = lambda x: "true" if x else "false"
    mf = info["path"] == 2
    vec = L.stride == 1 and (L.Ho * L.Wo) % 4 == 0
    if info["mode"] == 1:
        return "alcs::k_pw_resident<%d, %d, %s, %s, %d>" % (L.V, info["pv"], b(mf), b(vec), info["group_slots"])
    if info["mode"] == 2:
        return "alcs::k_pw_chunked<%d, %d, 4, %s, %s>" % (L.V, info["pv"], b(mf), b(vec))
    if info["mode"] in (3, 7):
        return "alcs::k_conv3<%d, %d" % (L.V, L.stride)          # prefix: tile shape and flags follow
    if info["mode"] == 5:
        return "alcs::k_pw_pipe<%d" % L.V
    return "alcs::k_pw_stream<%d, %d, 8>" % (L.V, info["pv"])


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_mobilenetv1_pointwise_b32.txt")


KERNEL_SOURCES = ("alcs_sparse.hip", "alcs_pack.cpp", "alcs_internal.h")


def kernel_sources_digest():
    """SHA-256 over the sources that decide the 1x1 kernels and their weight layout: the stamp the
    traffic profile carries, so that a profile taken before a kernel change is not quoted after it."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2109_00170_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def read_traffic(symbol):
    """HBM bytes per launch of `symbol` from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy of known size), or None - also when the
    summary was taken with other kernel sources than the ones in the tree (its `# sources:` stamp)."""
    try:
        with open(TRAFFIC_FILE) as f:
            lines = f.read().splitlines()
        stamp = [l.split(":", 1)[1].strip() for l in lines if l.startswith("# sources:")]
        if not stamp or stamp[0] != kernel_sources_digest():
            return None
        with open(TRAFFIC_FILE) as f:
            for line in f:
                if line.startswith("#") or "|" not in line:
                    continue
                name, fetch_b, write_b = [t.strip() for t in line.split("|")[:3]]
                if name == symbol:
                    return int(float(fetch_b) + float(write_b))
    except OSError:
        pass
    return None


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown CPU"


def cpu_oracle_us(np, d, L, images=None):
    """cpu_baseline leg: the oracle (oracle_conv on the masked weights, all host threads) on the
    layer's inputs.  images: run the first `images` of the batch only and scale linearly (images
    are independent); returns (microseconds for the whole batch, "measured" | "extrapolated")."""
    import oracle
    nb = L.N if images is None else max(1, min(images, L.N))
    Wd = oracle.densify(d.W, d.mask, L.V)
    xs = np.ascontiguousarray(d.X[:nb])
    t0 = time.perf_counter()
    oracle.conv(Wd, xs, stride=L.stride, nthreads=oracle.max_threads())
    t = time.perf_counter() - t0
    return t * 1e6 * L.N / nb, ("measured" if nb == L.N else "extrapolated from %d images" % nb)


def cpu_header(pr):
    import oracle
    pr("CPU oracle column: oracle_conv (plain C, double accumulation, zero weights skipped) on %d threads of: %s\n"
       % (oracle.max_threads(), cpu_model()))


def time_layer(alcs, torch, np, workloads, L, seed, dense=False, iters=10, tuning=None, cpu_images=0):
    """Median kernel time of one layer (kernel time stamps), optionally with the dense conv
    (then the two results are compared with each other; parity with the CPU oracle is the
    business of the tests)."""
    d = workloads.make_layer(L, seed)
    p = alcs.alcs_pack_weights(d.W, d.mask, L.V, options=tuning or None)
    X = torch.from_numpy(d.X).cuda()
    Y = torch.empty((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.float32, device="cuda")
    # rotate over enough copies that more than 600 MB is touched before a buffer comes round
    # again (the Infinity Cache holds 256 MB)
    R = max(1, min(8, int(600e6 // (L.x_bytes() + L.y_bytes())) + 1))
    Xr = [X] + [X.clone() for _ in range(R - 1)]
    Yr = [Y] + [torch.empty_like(Y) for _ in range(R - 1)]
    for _ in range(2):
        alcs.alcs_sparse_conv(p, X, None, Y, stride=L.stride)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    iters = max(iters, R + 1)
    ev = alcs.HipEvents(iters)
    for i in range(iters):
        alcs.alcs_sparse_conv(p, Xr[(i + 1) % R], None, Yr[(i + 1) % R], stride=L.stride, events=ev.pairs[i])
    torch.cuda.synchronize()
    t = float(np.median([ev.elapsed_us(i) for i in range(iters)]))
    ev.close()
    td = tl = None
    err = float("nan")
    if dense:
        # dense weights of the pruned layer: kept blocks as they are, dropped blocks zero
        keep = np.repeat(d.mask, L.V, axis=0)[:L.Cout] if d.mask is not None else 1
        Wd = torch.from_numpy(np.ascontiguousarray(d.W * keep, dtype=np.float32)).cuda()
        Ys = Y.clone()
        for _ in range(2):
            alcs.alcs_dense_conv(Wd, X, None, Y, stride=L.stride)
        torch.cuda.synchronize()
        err = float((Ys - Y).abs().max() / Y.abs().max().clamp_min(1e-30))
        del Ys
        e = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        for a, b in e:
            a.record()
            alcs.alcs_dense_conv(Wd, X, None, Y, stride=L.stride)
            b.record()
        torch.cuda.synchronize()
        td = float(np.median([a.elapsed_time(b) * 1e3 for a, b in e]))
        # the vendor library's dense convolution (PyTorch -> MIOpen, float32) on the same tensors: context
        # for the speed-up columns, which would otherwise rest on this repository's own dense kernel alone
        import torch.nn.functional as F
        pad = (L.k - 1) // 2
        for _ in range(3):
            Yl = F.conv2d(X, Wd, stride=L.stride, padding=pad)
        torch.cuda.synchronize()
        e = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        for a, b in e:
            a.record()
            Yl = F.conv2d(X, Wd, stride=L.stride, padding=pad)
            b.record()
        torch.cuda.synchronize()
        tl = float(np.median([a.elapsed_time(b) * 1e3 for a, b in e]))
        del Yl
    nn = p.nnzb
    by, fl = layer_bytes(L, nn), layer_flops(L, nn)
    p.free()
    cpu_us = cpu_how = None
    if cpu_images != 0:
        cpu_us, cpu_how = cpu_oracle_us(np, d, L, None if cpu_images < 0 else cpu_images)
    roof = max(by / (HBM_PEAK_GBS * 1e9), fl / (MFMA_FP32_PEAK_TFLOPS * 1e12)) * 1e6
    bound = "hbm" if by / (HBM_PEAK_GBS * 1e9) >= fl / (MFMA_FP32_PEAK_TFLOPS * 1e12) else "mfma"
    return {"us": t, "dense_us": td, "lib_us": tl, "roof_us": roof, "bound": bound, "bytes": by, "flops": fl, "err": err,
            "info": info, "cpu_us": cpu_us, "cpu_how": cpu_how}


def report(kind, alcs, workloads, torch, np):
    """Per-layer tables for configurations 3, 4, 5 and the MFMA / FMA comparison (markdown on stdout)."""
    pr = lambda *a: print(*a, flush=True)
    if kind == "sweep":
        cpu_header(pr)
        pr("| sparsity | sparse us | kernel | dense us | speed-up | PyTorch dense us | vs PyTorch | dense-equiv TFLOP/s | actual TFLOP/s | bound | roofline frac | max diff vs dense | CPU oracle ms (whole batch) |")
        pr("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
        for s in workloads.SWEEP_SPARSITIES:
            L = workloads.sweep_layer(s)
            r = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(4, int(round(s * 100))), dense=True, cpu_images=-1)
            pr("| %.2f | %.1f | mode %d | %.1f | %.2f | %.1f | %.2f | %.1f | %.1f | %s | %.3f | %.1e | %.0f (%s) |" %
               (s, r["us"], r["info"]["mode"], r["dense_us"], r["dense_us"] / r["us"], r["lib_us"], r["lib_us"] / r["us"], L.dense_flops() / r["us"] / 1e6,
                r["flops"] / r["us"] / 1e6, r["bound"], r["roof_us"] / r["us"], r["err"], r["cpu_us"] / 1e3, r["cpu_how"]))
    elif kind == "config1":
        cpu_header(pr)
        L = workloads.config1()
        r = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(1, 0), dense=True, cpu_images=-1, iters=50)
        pr("| layer | sparse us | dense us | PyTorch dense us | roofline us | roofline frac | max diff vs dense | CPU oracle ms |")
        pr("|---|---|---|---|---|---|---|---|")
        pr("| %s %d->%d @%d, batch %d, %d %% of the blocks kept | %.2f | %.2f | %.2f | %.2f | %.3f | %.1e | %.2f |" %
           (L.name, L.Cin, L.Cout, L.H, L.N, round(100 * (1 - L.sparsity)), r["us"], r["dense_us"], r["lib_us"], r["roof_us"],
            r["roof_us"] / r["us"], r["err"], r["cpu_us"] / 1e3))
        pr("\n(a launch-bound layer: its roofline is 0.2 us, an empty kernel takes 3.9 us by its own time stamps)")
    elif kind == "floor":
        # What bounds a layer apart from its roofline: (a) a vendor copy kernel that moves the layer's
        # algorithmic bytes (X read once, Y written once) on the same rotating, cache-cold buffers;
        # (b) the multiply alone at the rate the LDS-fed 4x4x1 inner loop reaches on this chip
        # (72.5 TFLOP/s of kept weights with two pixels per lane, measured with a register-and-LDS-only
        # loop of the same instructions), spread over all SIMDs; (c) the time stamps of an empty kernel.
        MUL_TFLOPS = 72.5
        EMPTY_US = 3.9
        pr("| layer | Cin->Cout | HxW | roofline us (8 TB/s) | copy of the same bytes us | multiply alone us | empty kernel us | "
           "measured us | measured / roofline | copy / measured | at least 50 % of the roofline |")
        pr("|---|---|---|---|---|---|---|---|---|---|---|")
        tot = tcopy = troof = 0.0
        for i, L in enumerate(workloads.mobilenet_v1_pointwise(32, 0.9)):
            r = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(2, i))
            R = max(2, min(8, int(600e6 // (L.x_bytes() + L.y_bytes())) + 1))
            Xr = [torch.randn((L.N, L.Cin, L.H, L.W), device="cuda") for _ in range(R)]
            Yr = [torch.empty((L.N, L.Cout, L.Ho, L.Wo), device="cuda") for _ in range(R)]
            rep = L.Cout // L.Cin

            def copy(j):
                if rep == 1:
                    Yr[j % R].copy_(Xr[j % R])
                else:
                    torch.cat([Xr[j % R]] * rep, dim=1, out=Yr[j % R])
            for j in range(R):
                copy(j)
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(3 * R)]
            for j, (a, b) in enumerate(evs):
                a.record()
                copy(j)
                b.record()
            torch.cuda.synchronize()
            c_us = float(np.median([a.elapsed_time(b) * 1e3 for a, b in evs]))
            m_us = r["flops"] / (MUL_TFLOPS * 1e12) * 1e6
            tot += r["us"]
            tcopy += c_us
            troof += r["roof_us"]
            pr("| %s | %d->%d | %d | %.2f | %.2f | %.2f | %.1f | %.2f | %.2f | %.2f | %s |" %
               (L.name, L.Cin, L.Cout, L.H, r["roof_us"], c_us, m_us, EMPTY_US, r["us"], r["us"] / r["roof_us"], c_us / r["us"],
                "yes" if 2 * r["roof_us"] >= r["us"] else "no"))
            del Xr, Yr
            torch.cuda.empty_cache()
        pr("\n13 layers: measured %.0f us, copies of the same bytes %.0f us, rooflines %.0f us" % (tot, tcopy, troof))
    elif kind == "resnet":
        cpu_header(pr)
        pr("| layer | Cin->Cout | k/s | HxW | x | sparse us | dense us | speed-up | PyTorch dense us | vs PyTorch | actual TFLOP/s | eff GB/s | bound | roofline frac | max diff vs dense | CPU oracle ms (batch 64, extrapolated from 2 images) |")
        pr("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
        tot = troof = tdense = tlib = tcpu = 0.0
        for i, L in enumerate(workloads.resnet50_bottlenecks(64)):
            r = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(3, i), dense=True, cpu_images=2)
            tcpu += r["cpu_us"] * L.repeats
            tot += r["us"] * L.repeats
            troof += r["roof_us"] * L.repeats
            tdense += r["dense_us"] * L.repeats
            tlib += r["lib_us"] * L.repeats
            pr("| %s | %d->%d | %d/%d | %d | %d | %.1f | %.1f | %.2f | %.1f | %.2f | %.1f | %.0f | %s | %.3f | %.1e | %.0f |" %
               (L.name, L.Cin, L.Cout, L.k, L.stride, L.H, L.repeats, r["us"], r["dense_us"],
                r["dense_us"] / r["us"], r["lib_us"], r["lib_us"] / r["us"], r["flops"] / r["us"] / 1e6,
                r["bytes"] / r["us"] / 1e3, r["bound"], r["roof_us"] / r["us"], r["err"], r["cpu_us"] / 1e3))
        pr("\nall 48 convs, batch 64: sparse %.0f us, dense %.0f us (%.2fx), PyTorch dense %.0f us (%.2fx), sum of rooflines %.0f us (%.3f), CPU oracle %.0f ms (extrapolated)" %
           (tot, tdense, tdense / tot, tlib, tlib / tot, troof, troof / tot, tcpu / 1e3))
    elif kind == "mbv2":
        cpu_header(pr)
        for V in (1, 4, 8, 16):
            pr("\nV = %d" % V)
            pr("| layer | sparse us | eff GB/s | bound | roofline frac | longest/mean group | CPU oracle ms (batch 128, extrapolated from 2 images) |")
            pr("|---|---|---|---|---|---|---|")
            tot = troof = tcpu = 0.0
            for i, L in enumerate(workloads.mobilenet_v2_pointwise(128, V)):
                r = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(5, 100 * V + i), cpu_images=2)
                tot += r["us"] * L.repeats
                troof += r["roof_us"] * L.repeats
                tcpu += r["cpu_us"] * L.repeats
                cnt = workloads.zipf_counts(L.G, L.K, 1.0 - L.sparsity)
                pr("| %s | %.1f | %.0f | %s | %.3f | %.1f | %.1f |" %
                   (L.name, r["us"], r["bytes"] / r["us"] / 1e3, r["bound"], r["roof_us"] / r["us"],
                    cnt.max() / max(cnt.mean(), 1e-9), r["cpu_us"] / 1e3))
            pr("total (with repeats) %.0f us, sum of rooflines %.0f us (%.3f), CPU oracle %.0f ms (extrapolated)" % (tot, troof, troof / tot, tcpu / 1e3))
    elif kind == "mbv1":
        cpu_header(pr)
        for N, sp, label in ((32, 0.9, "batch 32, block sparsity 0.9 in every layer"),
                             (32, None, "batch 32, per-layer block sparsity drawn from U(0.7, 0.9)"),
                             (1, None, "batch 1, per-layer block sparsity drawn from U(0.7, 0.9)")):
            pr("\n%s" % label)
            pr("| layer | Cin->Cout | HxW | sparsity | sparse us | dense us | speed-up | PyTorch dense us | vs PyTorch | eff GB/s | bound | roofline us | roofline frac | max diff vs dense | CPU oracle ms (whole batch) |")
            pr("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
            tot = troof = tdense = tlib = tcpu = 0.0
            for i, L in enumerate(workloads.mobilenet_v1_pointwise(N, sp)):
                r = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(2, i), dense=True, cpu_images=-1)
                tcpu += r["cpu_us"]
                tot += r["us"]
                troof += r["roof_us"]
                tdense += r["dense_us"]
                tlib += r["lib_us"]
                pr("| %s | %d->%d | %d | %.3f | %.1f | %.1f | %.2f | %.1f | %.2f | %.0f | %s | %.2f | %.3f | %.1e | %.1f |" %
                   (L.name, L.Cin, L.Cout, L.H, L.sparsity, r["us"], r["dense_us"], r["dense_us"] / r["us"],
                    r["lib_us"], r["lib_us"] / r["us"], r["bytes"] / r["us"] / 1e3, r["bound"], r["roof_us"],
                    r["roof_us"] / r["us"], r["err"], r["cpu_us"] / 1e3))
            pr("13 layers: sparse %.0f us, dense %.0f us (%.2fx), PyTorch dense %.0f us (%.2fx), sum of rooflines %.0f us (%.3f), CPU oracle %.0f ms" %
               (tot, tdense, tdense / tot, tlib, tlib / tot, troof, troof / tot, tcpu / 1e3))
    elif kind == "fused":
        # the element-wise layers behind a convolution folded into its epilogue, against the plain
        # convolution followed by PyTorch's in-place element-wise kernels on the same buffers
        def one(L, seed, act, residual):
            d = workloads.make_layer(L, seed, with_bias=True)
            p = alcs.alcs_pack_weights(d.W, d.mask, L.V)
            X = torch.from_numpy(d.X).cuda()
            b = torch.from_numpy(d.bias).cuda()
            R = max(2, min(8, int(600e6 // (L.x_bytes() + (2 if residual else 1) * L.y_bytes())) + 1))
            Xr = [X] + [X.clone() for _ in range(R - 1)]
            Yr = [torch.empty((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.float32, device="cuda") for _ in range(R)]
            Rr = [torch.randn_like(Yr[0]) for _ in range(R)] if residual else [None] * R

            def fused(i):
                alcs.alcs_sparse_conv_fused(p, Xr[i % R], b, Rr[i % R], Yr[i % R], stride=L.stride, activation=act)

            def unfused(i):
                alcs.alcs_sparse_conv(p, Xr[i % R], b, Yr[i % R], stride=L.stride)
                if residual:
                    Yr[i % R].add_(Rr[i % R])
                if act == "relu":
                    Yr[i % R].relu_()
                elif act == "relu6":
                    Yr[i % R].clamp_(0.0, 6.0)

            res = []
            for fn in (fused, unfused):
                for i in range(3):
                    fn(i)
                torch.cuda.synchronize()
                n = 3 * R
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(n):
                    fn(i)
                e1.record()
                torch.cuda.synchronize()
                res.append(e0.elapsed_time(e1) * 1e3 / n)
            fused(0)
            unf = Yr[0].clone()
            unfused(0)
            torch.cuda.synchronize()
            diff = float((unf - Yr[0]).abs().max() / Yr[0].abs().max().clamp_min(1e-30))
            by = layer_bytes(L, p.nnzb) + 4 * L.Cout + (L.y_bytes() if residual else 0)
            p.free()
            return res[0], res[1], by, diff

        pr("| layer | epilogue | fused us | conv + element-wise kernels us | ratio | fused eff GB/s | max diff |")
        pr("|---|---|---|---|---|---|---|")
        tf = tu = 0.0
        for i, L in enumerate(workloads.mobilenet_v1_pointwise(32, 0.9)):
            f, u, by, diff = one(L, workloads.seed_for(2, i), "relu", False)
            tf += f
            tu += u
            pr("| %s %d->%d @%d | bias + ReLU | %.1f | %.1f | %.2f | %.0f | %.1e |" %
               (L.name, L.Cin, L.Cout, L.H, f, u, u / f, by / f / 1e3, diff))
        pr("| 13 MobileNetV1-shaped layers, batch 32 | | %.0f | %.0f | %.2f | | |" % (tf, tu, tu / tf))
        tf = tu = 0.0
        for i, L in enumerate(workloads.mobilenet_v2_pointwise(128, 4)):
            if not L.name.startswith("proj") or L.Cin != 6 * L.Cout:
                continue   # shortcut connections exist where a block keeps its width
            f, u, by, diff = one(L, workloads.seed_for(5, 400 + i), None, True)
            tf += f
            tu += u
            pr("| %s | bias + shortcut | %.1f | %.1f | %.2f | %.0f | %.1e |" % (L.name, f, u, u / f, by / f / 1e3, diff))
        pr("| MobileNetV2-shaped projections with a shortcut, batch 128 | | %.0f | %.0f | %.2f | | |" % (tf, tu, tu / tf))
    elif kind == "block":
        # depthwise 3x3 + bias + ReLU -> sparse pointwise + bias + ReLU: one kernel against two
        def one(L, dws, seed):
            d = workloads.make_layer(L, seed, with_bias=True)
            p = alcs.alcs_pack_weights(d.W, d.mask, L.V)
            rng = np.random.Generator(np.random.PCG64(seed + 17))
            Hin, Win = L.H * dws, L.W * dws
            D = torch.from_numpy((rng.standard_normal((L.Cin, 3, 3)) * 0.3).astype(np.float32)).cuda()
            b1 = torch.from_numpy(rng.standard_normal(L.Cin).astype(np.float32)).cuda()
            b2 = torch.from_numpy(d.bias).cuda()
            xin = 4 * L.N * L.Cin * Hin * Win
            R = max(2, min(8, int(600e6 // (xin + L.x_bytes() + L.y_bytes())) + 1))
            X0 = torch.from_numpy(workloads.draw_x((L.N, L.Cin, Hin, Win), "relu", rng)).cuda()
            Xr = [X0] + [X0.clone() for _ in range(R - 1)]
            Zr = [torch.empty((L.N, L.Cin, L.H, L.W), dtype=torch.float32, device="cuda") for _ in range(R)]
            Yr = [torch.empty((L.N, L.Cout, L.H, L.W), dtype=torch.float32, device="cuda") for _ in range(R)]

            def fused(i):
                alcs.alcs_dw_sparse_conv_fused(p, D, b1, Xr[i % R], b2, None, Yr[i % R], dw_stride=dws,
                                               dw_activation="relu", activation="relu")

            def auto(i):
                alcs.alcs_dw_sparse_conv_fused(p, D, b1, Xr[i % R], b2, None, Yr[i % R], dw_stride=dws,
                                               dw_activation="relu", activation="relu", workspace=Zr[i % R])

            def two(i):
                alcs.alcs_depthwise_conv(D, Xr[i % R], b1, Zr[i % R], stride=dws, activation="relu")
                alcs.alcs_sparse_conv_fused(p, Zr[i % R], b2, None, Yr[i % R], activation="relu")

            def dw_only(i):
                alcs.alcs_depthwise_conv(D, Xr[i % R], b1, Zr[i % R], stride=dws, activation="relu")

            def pw_only(i):
                alcs.alcs_sparse_conv_fused(p, Zr[i % R], b2, None, Yr[i % R], activation="relu")

            res = []
            for fn in (fused, two, dw_only, pw_only, auto):
                for i in range(3):
                    fn(i)
                torch.cuda.synchronize()
                n = 3 * R
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(n):
                    fn(i)
                e1.record()
                torch.cuda.synchronize()
                res.append(e0.elapsed_time(e1) * 1e3 / n)
            fused(0)
            info = alcs.alcs_last_launch()
            yf = Yr[0].clone()
            two(0)
            torch.cuda.synchronize()
            diff = float((yf - Yr[0]).abs().max() / Yr[0].abs().max().clamp_min(1e-30))
            by_f = xin + L.y_bytes()
            by_u = xin + 2 * L.x_bytes() + L.y_bytes()
            p.free()
            return res, by_f, by_u, diff, info

        for N in (32, 1):
            pr("\nbatch %d\n" % N)
            pr("| block | depthwise | pointwise | one kernel us | two kernels us | ratio | with workspace us | depthwise alone us | "
               "pointwise alone us | one kernel eff GB/s | bytes saved | max diff | launch |")
            pr("|---|---|---|---|---|---|---|---|---|---|---|---|---|")
            tf = tu = ta = 0.0
            for i, (L, dws) in enumerate(workloads.mobilenet_v1_blocks(N, 0.9)):
                (f, u, t_dw, t_pw, t_auto), by_f, by_u, diff, info = one(L, dws, workloads.seed_for(2, 300 + i))
                tf += f
                tu += u
                ta += t_auto
                pr("| %d | %d ch 3x3/%d @%d | %d->%d @%d | %.1f | %.1f | %.2f | %.1f | %.1f | %.1f | %.0f | %.0f %% | %.1e | pv%d w%d wg%d |" %
                   (i + 1, L.Cin, dws, L.H * dws, L.Cin, L.Cout, L.H, f, u, u / f, t_auto, t_dw, t_pw, by_f / f / 1e3,
                    100.0 * (by_u - by_f) / by_u, diff, info["pv"], info["waves"], info["workgroups"]))
            pr("| 13 MobileNetV1-shaped blocks, 90 %% block sparsity | | | %.0f | %.0f | %.2f | %.0f | | | | | | |" % (tf, tu, tu / tf, ta))
    elif kind == "bf16":
        # the same layers with X and Y stored as bfloat16 against float32 tensors (both through the
        # fused-epilogue entry points with bias + ReLU; stream events over rotated buffers)
        def one(L, seed):
            d = workloads.make_layer(L, seed, with_bias=True)
            p = alcs.alcs_pack_weights(d.W, d.mask, L.V)
            b = torch.from_numpy(d.bias).cuda()
            X = torch.from_numpy(d.X).cuda()
            R = max(2, min(8, int(600e6 // (L.x_bytes() + L.y_bytes())) + 1))
            X32 = [X] + [X.clone() for _ in range(R - 1)]
            Y32 = [torch.empty((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.float32, device="cuda") for _ in range(R)]
            X16 = [x.to(torch.bfloat16) for x in X32] + [X.to(torch.bfloat16) for _ in range(R)]   # same bytes in rotation
            Y16 = [torch.empty((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.bfloat16, device="cuda") for _ in range(2 * R)]

            def f32(i):
                alcs.alcs_sparse_conv_fused(p, X32[i % R], b, None, Y32[i % R], stride=L.stride, activation="relu")

            def f16(i):
                alcs.alcs_sparse_conv_bf16(p, X16[i % (2 * R)], b, None, Y16[i % (2 * R)], stride=L.stride, activation="relu")

            res = []
            for fn in (f32, f16):
                for i in range(3):
                    fn(i)
                torch.cuda.synchronize()
                n = 6 * R
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(n):
                    fn(i)
                e1.record()
                torch.cuda.synchronize()
                res.append(e0.elapsed_time(e1) * 1e3 / n)
            f32(0)
            f16(0)
            torch.cuda.synchronize()
            diff = float((Y32[0] - Y16[0].float()).abs().max() / Y32[0].abs().max().clamp_min(1e-30))
            wb = layer_bytes(L, p.nnzb) - L.x_bytes() - L.y_bytes()
            by32 = layer_bytes(L, p.nnzb) + 4 * L.Cout
            by16 = (L.x_bytes() + L.y_bytes()) // 2 + wb + 4 * L.Cout
            p.free()
            return res[0], res[1], by32, by16, diff

        pr("| layer | float32 us | bfloat16 us | ratio | bfloat16 bytes MB | bfloat16 eff GB/s | bfloat16 HBM roofline frac | max diff (of max) |")
        pr("|---|---|---|---|---|---|---|---|")
        t32 = t16 = roof = 0.0
        for i, L in enumerate(workloads.mobilenet_v1_pointwise(32, 0.9)):
            a, b_, by32, by16, diff = one(L, workloads.seed_for(2, i))
            t32 += a
            t16 += b_
            roof += by16 / (HBM_PEAK_GBS * 1e3)
            pr("| %s %d->%d @%d | %.1f | %.1f | %.2f | %.1f | %.0f | %.3f | %.1e |" %
               (L.name, L.Cin, L.Cout, L.H, a, b_, a / b_, by16 / 1e6, by16 / b_ / 1e3, by16 / (HBM_PEAK_GBS * 1e3) / b_, diff))
        pr("| 13 MobileNetV1-shaped layers, batch 32, 90 %% block sparsity | %.0f | %.0f | %.2f | | | %.3f | |" %
           (t32, t16, t32 / t16, roof / t16))
    elif kind == "math16":
        # 16-bit arithmetic (alcs_sparse_conv_bf16_mfma: bfloat16 tensors and weights on the 16-bit matrix
        # instruction) against the float32 path and against bfloat16 storage with float32 arithmetic;
        # bias + ReLU in all three; stream events over rotated buffers of the same number of bytes
        import dataclasses

        def one(L, seed):
            d = workloads.make_layer(L, seed, with_bias=True)
            p = alcs.alcs_pack_weights(d.W, d.mask, L.V)
            p16 = None
            try:
                p.add_bf16_weights()                       # the same handle serves all three entry points
                p16 = p
            except alcs.AlcsError:
                pass                                       # more input channels than one 16-bit tile holds
            b = torch.from_numpy(d.bias).cuda()
            X = torch.from_numpy(d.X).cuda()
            R = max(2, min(8, int(600e6 // (L.x_bytes() + L.y_bytes())) + 1))
            X32 = [X] + [X.clone() for _ in range(R - 1)]
            Y32 = [torch.empty((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.float32, device="cuda") for _ in range(R)]
            X16 = [x.to(torch.bfloat16) for x in X32] + [X.to(torch.bfloat16) for _ in range(R)]
            Y16 = [torch.empty((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.bfloat16, device="cuda") for _ in range(2 * R)]

            def f32(i):
                alcs.alcs_sparse_conv_fused(p, X32[i % R], b, None, Y32[i % R], stride=L.stride, activation="relu")

            def f16(i):
                alcs.alcs_sparse_conv_bf16(p, X16[i % (2 * R)], b, None, Y16[i % (2 * R)], stride=L.stride, activation="relu")

            def m16(i):
                alcs.alcs_sparse_conv_bf16_mfma(p16, X16[i % (2 * R)], b, None, Y16[i % (2 * R)], stride=L.stride, activation="relu")

            res = []
            for fn in (f32, f16, m16):
                if fn is m16 and p16 is None:
                    res.append(float("nan"))
                    continue
                for i in range(3):
                    fn(i)
                torch.cuda.synchronize()
                n = 6 * R
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(n):
                    fn(i)
                e1.record()
                torch.cuda.synchronize()
                res.append(e0.elapsed_time(e1) * 1e3 / n)
            diff = float("nan")
            if p16 is not None:
                f32(0)
                m16(0)
                torch.cuda.synchronize()
                diff = float((Y32[0] - Y16[0].float()).abs().max() / Y32[0].abs().max().clamp_min(1e-30))
            wb = layer_bytes(L, p.nnzb) - L.x_bytes() - L.y_bytes()
            by16 = (L.x_bytes() + L.y_bytes()) // 2 + wb // 2 + 4 * L.Cout
            p.free()
            return res, by16, diff

        for V in (8, 16, 4):
            pr("")
            pr("V = %d" % V)
            pr("")
            pr("| layer | float32 us | bfloat16 storage us | 16-bit arithmetic us | float32 / 16-bit | storage / 16-bit | "
               "16-bit bytes MB | eff GB/s | HBM roofline frac | max diff to float32 (of max) |")
            pr("|---|---|---|---|---|---|---|---|---|---|")
            tot = [0.0, 0.0, 0.0]
            for i, L0 in enumerate(workloads.mobilenet_v1_pointwise(32, 0.9)):
                L = dataclasses.replace(L0, V=V)
                (a, b_, c), by16, diff = one(L, workloads.seed_for(2, i))
                if c == c:
                    tot = [tot[0] + a, tot[1] + b_, tot[2] + c]
                    pr("| %s %d->%d @%d | %.1f | %.1f | %.1f | %.2f | %.2f | %.1f | %.0f | %.3f | %.1e |" %
                       (L.name, L.Cin, L.Cout, L.H, a, b_, c, a / c, b_ / c, by16 / 1e6, by16 / c / 1e3,
                        by16 / (HBM_PEAK_GBS * 1e3) / c, diff))
                else:
                    pr("| %s %d->%d @%d | %.1f | %.1f | n/a (more than 1278 input channels) | | | | | | |" %
                       (L.name, L.Cin, L.Cout, L.H, a, b_))
            pr("| layers with a 16-bit time | %.0f | %.0f | %.0f | %.2f | %.2f | | | | |" %
               (tot[0], tot[1], tot[2], tot[0] / tot[2], tot[1] / tot[2]))
    elif kind == "project":
        # Algorithm 1 on the GPU: block scores, top-N selection, the bisection; times are wall-clock
        # around synchronised calls (the bisection synchronises once per step by design)
        import time

        def net(name):
            if name == "mbv1":
                return [(L.Cout, L.Cin, 1) for L in workloads.mobilenet_v1_pointwise(1, 0.0)]
            return [(L.Cout, L.Cin, L.k) for L in workloads.resnet50_bottlenecks(1, 0.0, distinct=False)]

        notes = []
        pr("| network | weights | blocks (V=4) | scores us | scores eff GB/s | select N = half us | select eff GB/s | "
           "projection ms | bisection steps | kept blocks | estimate vs budget |")
        pr("|---|---|---|---|---|---|---|---|---|---|---|")
        for name, title in (("mbv1", "13 MobileNetV1-shaped pointwise layers"), ("resnet", "48 ResNet-50-shaped convs")):
            rng = np.random.Generator(np.random.PCG64(workloads.seed_for(2, 700)))
            shapes = net(name)
            Ws = [torch.from_numpy((rng.standard_normal((co, ci, k, k), dtype=np.float32) *
                                    np.float32(0.05 + 0.2 * rng.random()))).cuda() for co, ci, k in shapes]
            V = 4
            sizes = [((co + V - 1) // V) * ci * k * k for co, ci, k in shapes]
            starts = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
            allsc = torch.empty((int(starts[-1]),), dtype=torch.float32, device="cuda")
            views = [allsc[int(a):int(b)].view((co + V - 1) // V, ci, k, k) for (co, ci, k), a, b in zip(shapes, starts, starts[1:])]

            def scores():
                for W, v in zip(Ws, views):
                    alcs.alcs_block_scores(W, V, scores=v)
            for _ in range(2):
                scores()
            torch.cuda.synchronize()
            reps = 10
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                scores()
            e1.record()
            torch.cuda.synchronize()
            t_sc = e0.elapsed_time(e1) * 1e3 / reps
            nw = sum(co * ci * k * k for co, ci, k in shapes)
            by_sc = 4 * nw + 4 * int(starts[-1])
            n = int(starts[-1])
            alcs.alcs_topn_mask(allsc, n // 2, seg_starts=starts)
            t0 = time.perf_counter()
            for _ in range(reps):
                alcs.alcs_topn_mask(allsc, n // 2, seg_starts=starts)
            t_sel = (time.perf_counter() - t0) * 1e6 / reps
            by_sel = 9 * 4 * n + n
            # latency tables of the shape measured on this GPU: a floor plus a slope per kept weight
            tables = []
            for co, ci, k in shapes:
                kk = np.arange(11) * 0.1 * (co * ci * k * k)
                tables.append((kk, 9.0 + 60.0 * np.arange(11) / 10.0 * (k * k) ** 0.5))
            t_none = sum(t[0] for _, t in tables)
            t_all = sum(t[-1] for _, t in tables)
            budget = t_none + 0.3 * (t_all - t_none)
            alcs.alcs_project_latency(allsc, starts, [V] * len(shapes), tables, 0.0, budget, 1e-3)
            t0 = time.perf_counter()
            N, mask, lo, hi = alcs.alcs_project_latency(allsc, starts, [V] * len(shapes), tables, 0.0, budget, 1e-3)
            t_proj = (time.perf_counter() - t0) * 1e3
            steps = int(np.ceil(np.log2(max(n, 2))))
            pr("| %s | %.2f M | %.2f M | %.1f | %.0f | %.0f | %.0f | %.2f | <= %d | %d (%.1f %%) | %.1f <= %.1f <= %.1f |" %
               (title, nw / 1e6, n / 1e6, t_sc, by_sc / t_sc / 1e3, t_sel, by_sel / t_sel / 1e3, t_proj, steps, N,
                100.0 * N / n, lo, budget, hi))
            # from the projection's flags to handles: storage format built on the device against the
            # host packer (which needs the dense weights and the flags in host memory)
            masks = [mask[int(a):int(b)] for a, b in zip(starts, starts[1:])]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            csr = [alcs.alcs_pack_csr_device(W, m, V) for W, m in zip(Ws, masks)]
            torch.cuda.synchronize()
            t_csr = (time.perf_counter() - t0) * 1e3
            t0 = time.perf_counter()
            hs = [alcs.alcs_pack_from_csr(r.cpu().numpy(), c.cpu().numpy(), v.cpu().numpy(), co, ci, k, V)
                  for (r, c, v), (co, ci, k) in zip(csr, shapes)]
            t_from = (time.perf_counter() - t0) * 1e3
            for h in hs:
                h.free()
            t0 = time.perf_counter()
            Wh = [W.cpu().numpy() for W in Ws]
            mh = [m.cpu().numpy().reshape((co + V - 1) // V, ci, k, k) for m, (co, ci, k) in zip(masks, shapes)]
            t_down = (time.perf_counter() - t0) * 1e3
            t0 = time.perf_counter()
            hs = [alcs.alcs_pack_weights(W, m, V) for W, m in zip(Wh, mh)]
            t_host = (time.perf_counter() - t0) * 1e3
            for h in hs:
                h.free()
            # everything on the device: weights + flags -> arrays -> layout -> handle (alcs_pack_weights_device)
            m8 = [m.contiguous() for m in masks]
            hs = [alcs.alcs_pack_weights_device(W, m, V) for W, m in zip(Ws, m8)]      # warm-up
            for h in hs:
                h.free()
            torch.cuda.synchronize()
            t_dev = []
            for _ in range(5):
                t0 = time.perf_counter()
                hs = [alcs.alcs_pack_weights_device(W, m, V) for W, m in zip(Ws, m8)]
                torch.cuda.synchronize()
                t_dev.append((time.perf_counter() - t0) * 1e3)
                for h in hs:
                    h.free()
            ws = torch.empty((alcs.alcs_pack_workspace_bytes(Ws, m8, V),), dtype=torch.uint8, device="cuda")
            t_net = []
            for _ in range(6):
                t0 = time.perf_counter()
                hs = alcs.alcs_pack_network_device(Ws, m8, V, workspace=ws)
                torch.cuda.synchronize()
                t_net.append((time.perf_counter() - t0) * 1e3)
                for h in hs:
                    h.free()
            t_net = t_net[1:]
            notes.append("%s: weights + flags on the device -> handles, all layers in one call "
                         "(alcs_pack_network_device, caller's workspace of %.1f MB) **%.2f ms** (median of 5, min %.2f); "
                         "layer by layer with alcs_pack_weights_device %.2f ms "
                         "(median of 5, min %.2f; %d layers); in steps through the host: storage format on the device "
                         "%.2f ms (2 calls a layer), arrays to the host + layout + upload %.2f ms; all on the host: "
                         "weights and flags to the host %.2f ms, alcs_pack_weights %.2f ms." %
                         (title, ws.numel() / 1e6, float(np.median(t_net)), min(t_net), float(np.median(t_dev)), min(t_dev),
                          len(shapes), t_csr, t_from, t_down, t_host))
        pr("")
        for line in notes:
            pr(line)
    elif kind == "latency":
        # Section 3.3 of the paper on this GPU: time every layer at block densities 0, 0.1, ..., 1
        # (eleven runs per layer), interpolate linearly in the number of non-zero weights
        # (alcs_latency_estimate / alcs_network_latency), and compare estimate and measurement on
        # randomly drawn sparse networks.
        def layer_timer(L, seed):
            rng = np.random.Generator(np.random.PCG64(seed))
            W = rng.standard_normal(size=(L.Cout, L.Cin, L.k, L.k), dtype=np.float32) * np.float32(L.w_std)
            X = torch.from_numpy(workloads.draw_x((L.N, L.Cin, L.H, L.W), L.x_dist, rng)).cuda()
            R = max(2, min(8, int(600e6 // (L.x_bytes() + L.y_bytes())) + 1))
            Xr = [X] + [X.clone() for _ in range(R - 1)]
            Yr = [torch.empty((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.float32, device="cuda") for _ in range(R)]
            iters = max(7, R + 1)
            ev = alcs.HipEvents(iters)

            def timed(density):
                mask = workloads.mask_exact(L.G, L.Cin, L.k, 1.0 - density, rng, tap_shared=L.tap_shared)
                p = alcs.alcs_pack_weights(W, mask, L.V)
                alcs.alcs_sparse_conv(p, Xr[0], None, Yr[0], stride=L.stride)
                for i in range(iters):
                    alcs.alcs_sparse_conv(p, Xr[(i + 1) % R], None, Yr[(i + 1) % R], stride=L.stride,
                                          events=ev.pairs[i])
                torch.cuda.synchronize()
                t = float(np.median([ev.elapsed_us(i) for i in range(iters)]))
                nnz = float(p.nnzb) * L.V
                p.free()
                return nnz, t
            return timed, ev

        nets = (("13 MobileNetV1-shaped pointwise convs, batch 32", workloads.mobilenet_v1_pointwise(32, 0.0), 2, 100),
                ("ResNet-50-shaped bottleneck convs (1x1 and 3x3), batch 16", workloads.resnet50_bottlenecks(16, 0.0), 3, 40))
        for title, layers, cfg, n_models in nets:
            pr("\n## %s\n" % title)
            pr("Run time in us at block density 0, 0.1, ..., 1.0 (kernel time stamps, median of 7 or more cold launches):\n")
            pr("| layer | shape | " + " | ".join("%.1f" % (0.1 * j) for j in range(11)) + " |")
            pr("|---|---|" + "---|" * 11)
            draw = np.random.Generator(np.random.PCG64(workloads.seed_for(cfg, 900)))
            dens = draw.random((n_models, len(layers)))          # every layer's density, per sampled network
            real = np.zeros(n_models)
            est = np.zeros(n_models)
            layer_err = []
            for li, L in enumerate(layers):
                timed, ev = layer_timer(L, workloads.seed_for(cfg, 500 + li))
                pts = [timed(0.1 * j) for j in range(11)]
                k = [a for a, _ in pts]
                t = [b for _, b in pts]
                pr("| %s | %d->%d %dx%d/%d @%d | " % (L.name, L.Cin, L.Cout, L.k, L.k, L.stride, L.H) +
                   " | ".join("%.1f" % v for v in t) + " |")
                errs = []
                for m in range(n_models):
                    nnz, tm = timed(float(dens[m, li]))
                    te = alcs.alcs_latency_estimate(k, t, nnz)
                    real[m] += tm * L.repeats
                    est[m] += te * L.repeats
                    errs.append(abs(te - tm) / tm)
                layer_err.append((L.name, float(np.mean(errs)), float(np.max(errs))))
                ev.close()
            rel = np.abs(est - real) / real
            pr("\n%d sampled networks (every layer's block density drawn from U(0, 1), fresh random mask):"
               " measured total %.0f-%.0f us; estimate off by %.2f %% on average, %.2f %% at most; "
               "correlation %.5f." % (n_models, real.min(), real.max(), 100 * rel.mean(), 100 * rel.max(),
                                      float(np.corrcoef(est, real)[0, 1])))
            pr("Per layer, mean / largest relative error of the estimate: " +
               ", ".join("%s %.1f / %.1f %%" % (n, 100 * a, 100 * b) for n, a, b in layer_err) + ".")
    elif kind == "paths":
        pr("| layer | MFMA us | FMA us | FMA / MFMA |")
        pr("|---|---|---|---|")
        for i, L in enumerate(workloads.mobilenet_v1_pointwise(32, 0.9)):
            if L.Cin > 639:
                continue    # wider inputs need several groups per wavefront, which only the MFMA form does
            # one group per wavefront for both forms (the default layout pairs groups from 512 channels on)
            a = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(2, i), tuning={"path": 2, "group_slots": 1})
            b = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(2, i), tuning={"path": 1, "group_slots": 1})
            pr("| %s | %.1f | %.1f | %.2f |" % (L.name, a["us"], b["us"], b["us"] / a["us"]))
        for s in (0.5, 0.9):
            L = workloads.sweep_layer(s)
            a = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(4, int(s * 100)), tuning={"path": 2, "group_slots": 1})
            b = time_layer(alcs, torch, np, workloads, L, workloads.seed_for(4, int(s * 100)), tuning={"path": 1, "group_slots": 1})
            pr("| sweep s=%.2f | %.1f | %.1f | %.2f |" % (s, a["us"], b["us"], b["us"] / a["us"]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--sparsity", type=float, default=0.9,
                    help="block sparsity of every layer; a negative value draws U(0.7,0.9) per layer")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-batch", type=int, default=32)
    ap.add_argument("--layers-json", default=None, help="also write the per-layer table to this file")
    ap.add_argument("--report", choices=["sweep", "resnet", "mbv2", "paths", "mbv1", "fused", "latency", "block", "project", "bf16", "math16", "config1", "floor"], default=None,
                    help="instead of the benchmark line, print a per-layer table for another configuration: "
                         "the sparsity sweep with the same-GPU dense conv (config 4), the ResNet-50-shaped "
                         "bottleneck convs (config 3), the MobileNetV2-shaped pointwise convs for V in "
                         "{1,4,8,16} (config 5), MFMA against plain-FMA inner loops (V=4), or the "
                         "MobileNetV1-shaped pointwise convs at batch 1 and 32 with fixed and drawn "
                         "sparsities, beside the dense conv (config 2), or the fused epilogue "
                         "(alcs_sparse_conv_fused) against the convolution followed by separate "
                         "element-wise kernels")
    ap.add_argument("--calib-copy", action="store_true",
                    help="for rocprofv3 --pmc runs only: put a plain 256 MiB device copy in front of every "
                         "step, so that the HBM byte counters can be scaled by a kernel of known traffic "
                         "(the printed timings are then not a benchmark result)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path needs no exchange between GPUs); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2109_00170_amd as alcs
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    alcs.load_library()

    if args.report:
        report(args.report, alcs, workloads, torch, np)
        return

    sp = None if args.sparsity < 0 else args.sparsity
    layers = workloads.mobilenet_v1_pointwise(args.batch, sp)
    data, packed, Xs, Ys, nnzb = [], [], [], [], []
    for i, L in enumerate(layers):
        d = workloads.make_layer(L, workloads.seed_for(2, i))
        data.append(d)
        p = alcs.alcs_pack_weights(d.W, d.mask, L.V)
        assert p.on_device
        packed.append(p)
        nnzb.append(p.nnzb)
        Xs.append(torch.from_numpy(d.X).to(dev))
        Ys.append(torch.empty((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.float32, device=dev))
    stream = torch.cuda.current_stream()
    stream_ptr = stream.cuda_stream

    def run_layer(i):
        alcs.alcs_sparse_conv(packed[i], Xs[i], None, Ys[i], stride=layers[i].stride, stream=stream_ptr)

    def run_step():
        for i in range(len(layers)):
            run_layer(i)

    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()

    def run_layer_timed(i, pair):
        alcs.alcs_sparse_conv(packed[i], Xs[i], None, Ys[i], stride=layers[i].stride, stream=stream_ptr,
                              events=pair)

    launch = []
    for i in range(len(layers)):
        run_layer(i)
        launch.append(alcs.alcs_last_launch())
    torch.cuda.synchronize()
    symbols = [kernel_symbol(layers[i], launch[i]) for i in range(len(layers))]

    calib = None
    if args.calib_copy:
        calib = (torch.zeros(64 * 1024 * 1024, device=dev), torch.empty(64 * 1024 * 1024, device=dev))

    # ---- timed region: exactly `steps` steps, nothing but the 13 launches per step ----
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        if calib is not None:
            calib[1].copy_(calib[0])
        run_step()
    t_submitted = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    host_submit_ms_per_step = (t_submitted - t0) * 1e3 / args.steps  # the host's share: all launches queued

    # ---- the same `steps` steps once more, every launch carrying a pair of HIP events that
    # take the kernel's own begin/end time stamps (alcs_sparse_conv_timed): per-launch
    # durations in the launch order and on the buffers of the timed steps ----
    evs = alcs.HipEvents(args.steps * len(layers))
    torch.cuda.synchronize()
    for s in range(args.steps):
        for i in range(len(layers)):
            run_layer_timed(i, evs.pairs[s * len(layers) + i])
    torch.cuda.synchronize()
    dur = np.array([[evs.elapsed_us(s * len(layers) + i) for i in range(len(layers))]
                    for s in range(args.steps)])
    evs.close()
    layer_us = [float(np.mean(dur[:, i])) for i in range(len(layers))]

    # ---- labelled extra, not part of `value`: every layer launched back to back on its own
    # buffers, so that inputs, weights and translations are cache-warm (the timed steps above
    # walk through 594 MB between two launches of a layer and find nothing of it cached) ----
    n_warm = 12
    evw = alcs.HipEvents(n_warm)
    warm_us = []
    for i in range(len(layers)):
        for j in range(n_warm):
            run_layer_timed(i, evw.pairs[j])
        torch.cuda.synchronize()
        warm_us.append(float(np.median([evw.elapsed_us(j) for j in range(2, n_warm)])))
    evw.close()
    # the dominant kernel: the kernel symbol (template instance) with the largest total time per step
    per_symbol = {}
    for i, sname in enumerate(symbols):
        per_symbol[sname] = per_symbol.get(sname, 0.0) + layer_us[i]
    dom_symbol = max(per_symbol, key=per_symbol.get)
    dom_layers = [i for i, sname in enumerate(symbols) if sname == dom_symbol]
    dom_us = float(np.mean(dur[:, dom_layers]))

    dense_flops = sum(L.dense_flops() for L in layers)
    alg_flops = sum(layer_flops(L, n) for L, n in zip(layers, nnzb))
    alg_bytes = sum(layer_bytes(L, n) for L, n in zip(layers, nnzb))
    value = dense_flops / (ms_per_step * 1e-3) / 1e9

    # ---- per-layer table ----
    rows = []
    roof_sum = 0.0
    for i, L in enumerate(layers):
        b = layer_bytes(L, nnzb[i])
        f = layer_flops(L, nnzb[i])
        t_hbm = b / (HBM_PEAK_GBS * 1e9)
        t_mfma = f / (MFMA_FP32_PEAK_TFLOPS * 1e12)
        t_roof = max(t_hbm, t_mfma)
        roof_sum += t_roof
        us = layer_us[i]
        rows.append({"layer": L.name, "Cin": L.Cin, "Cout": L.Cout, "HW": L.H, "N": L.N,
                     "sparsity": round(L.sparsity, 4), "nnzb": nnzb[i], "us": round(us, 2),
                     "dense_equiv_gflops": round(L.dense_flops() / us / 1e3, 1),
                     "actual_gflops": round(f / us / 1e3, 1),
                     "effective_gbs": round(b / us / 1e3, 1),
                     "bound": "hbm" if t_hbm >= t_mfma else "mfma",
                     "roofline_us": round(t_roof * 1e6, 2),
                     "roofline_frac": round(t_roof * 1e6 / us, 3),
                     "cache_warm_us": round(warm_us[i], 2), "launch": launch[i]})
    print("%-6s %-10s %4s %8s %8s %9s %10s %9s %6s %6s  launch" %
          ("layer", "Cin->Cout", "HW", "us", "warm us", "denseGF/s", "actGF/s", "effGB/s", "bound", "frac"),
          file=sys.stderr)
    for r in rows:
        print("%-6s %-10s %4d %8.2f %8.2f %9.0f %10.0f %9.0f %6s %6.3f  %s" %
              (r["layer"], "%d->%d" % (r["Cin"], r["Cout"]), r["HW"], r["us"], r["cache_warm_us"],
               r["dense_equiv_gflops"],
               r["actual_gflops"], r["effective_gbs"], r["bound"], r["roofline_frac"],
               "m%d pv%d w%d wg%d lds%d gt%d" % (r["launch"]["mode"], r["launch"]["pv"], r["launch"]["waves"],
                                                  r["launch"]["workgroups"], r["launch"]["lds_bytes"],
                                                  r["launch"]["group_tiles"])), file=sys.stderr)
    sum_us = sum(layer_us)
    print("sum of per-launch kernel times %.1f us; step %.1f us; sum of rooflines %.1f us (%.3f of step)" %
          (sum_us, ms_per_step * 1e3, roof_sum * 1e6, roof_sum * 1e3 / ms_per_step), file=sys.stderr)
    if args.layers_json:
        with open(args.layers_json, "w") as f:
            json.dump(rows, f, indent=1)

    dom_bytes = float(np.mean([layer_bytes(layers[i], nnzb[i]) for i in dom_layers]))
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": read_traffic(dom_symbol),
                "kernel": dom_symbol,
                "layers": [layers[i].name for i in dom_layers],
                "algorithmic_bytes_per_launch": int(dom_bytes), "avg_launch_us": round(dom_us, 2),
                "share_of_step": round(per_symbol[dom_symbol] / sum(layer_us), 3)}

    out = {
        "metric": "dense-equiv GFLOP/s + achieved HBM GB/s, sparse pointwise conv, 1 MI355X",
        "value": round(value, 1),
        "unit": "GFLOP/s (dense-equivalent)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "MobileNetV1-shaped 13 pointwise 1x1 convs @224, batch %d, V=4, block sparsity %s"
                               % (args.batch, "0.9 fixed" if sp is not None and abs(sp - 0.9) < 1e-9 else
                                  ("%.2f fixed" % sp if sp is not None else "U(0.7,0.9) per layer")),
                   "batch": args.batch, "layers": len(layers)},
        "effective_gbs": round(alg_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "actual_gflops": round(alg_flops / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline_frac_step": round(roof_sum * 1e3 / ms_per_step, 4),
        "host_submit_ms_per_step": round(host_submit_ms_per_step, 5),
        "sum_of_kernel_us": round(sum(layer_us), 1),
        "roofline": roofline,
        "cache_warm": {"sum_of_kernel_us": round(sum(warm_us), 1),
                       "roofline_frac": round(roof_sum * 1e6 / sum(warm_us), 4),
                       "note": "each layer relaunched on the same buffers (inputs, weights and address "
                               "translations cached); kernel time stamps; not part of value"},
    }

    if not args.no_cpu_baseline:
        # The oracle as it stands, on the host cores, on the first nb images of every layer;
        # its outputs are also what the timed GPU buffers are checked against.
        import oracle
        nb = max(1, min(args.cpu_sample_batch, args.batch))
        threads = oracle.max_threads()
        t_cpu = 0.0
        fl = 0.0
        max_err = 0.0
        for i, L in enumerate(layers):
            Wd = oracle.densify(data[i].W, data[i].mask, L.V)
            xs = np.ascontiguousarray(data[i].X[:nb])
            c0 = time.perf_counter()
            ref = oracle.conv(Wd, xs, stride=L.stride, nthreads=threads)
            t_cpu += time.perf_counter() - c0
            fl += L.dense_flops() * nb / L.N
            got = Ys[i][:nb].cpu().numpy()
            max_err = max(max_err, float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30)))
        out["cpu_baseline"] = {"value": round(fl / t_cpu / 1e9, 2), "unit": "GFLOP/s (dense-equivalent)",
                               "cores": threads, "kind": "oracle", "cpu": cpu_model(),
                               "sample": "same 13 layers and weights, first %d of %d images, %.1f s of CPU time"
                                         % (nb, args.batch, t_cpu)}
        out["max_rel_err_vs_oracle"] = float("%.3g" % max_err)
    if args.calib_copy:
        out["calibration_run"] = True
    print(json.dumps(out))


if __name__ == "__main__":
    main()
