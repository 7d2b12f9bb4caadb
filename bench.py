#!/usr/bin/env python3
"""Benchmark of the structured-tensor hot path on one MI355X.

One *step* is one pass of the whole hot path over the five synthetic
workloads: symmetric MTTKRP (n=64, R=16), upper-triangular BATAX (n=8192),
band TTM (512^3, w=8, R=64), symmetric MTTKRP (n=512, R=64), third-moment
accumulation (N=2e6, n=64) followed by the expansion of its result.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]

Per-call figures are MEDIANS of event pairs on the launch stream over the timed steps (the mean is kept beside
them); `kernels[*].kernel_us` and `kernels[*].traffic` come from the committed rocprofv3 summary
profiles/bench_step_counters.txt and are null once the kernel's source has changed since it was taken.
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

import st_workloads as W  # noqa: E402

# published MI355X peaks
HBM_PEAK_GBS = 8000.0
MFMA_FP32_PEAK_TFLOPS = 157.3
# plain (unpacked) fp32 vector rate: 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz; packed fp32 is compiled out
ALU_FP32_PEAK_TFLOPS = 78.6


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def tri(n):
    return n * (n + 1) // 2


def tet(n):
    return n * (n + 1) * (n + 2) // 6


def workloads():
    """Algorithmic flops (unique-element convention) and bytes per launch."""
    c1, c2, c3, c4, c5 = (W.CONFIGS[i] for i in range(1, 6))
    out = {}
    n, R = c1["n"], c1["R"]
    out["mttkrp_sym3_n64_R16"] = dict(flops=6 * R * tet(n), bytes=4 * (tet(n) + 2 * n * R), bound="mfma")
    n = c2["n"]
    out["batax_utri_n8192"] = dict(flops=4 * tri(n), bytes=4 * (tri(n) + 2 * n), bound="hbm")
    rows, nl, R = c3["band_pairs"], c3["nl"], c3["R"]
    out["ttm_band_n512_w8_R64"] = dict(flops=2 * rows * nl * R, bytes=4 * (rows * nl + nl * R + rows * R),
                                       bound="mfma")
    n, R = c4["n"], c4["R"]
    out["mttkrp_sym3_n512_R64"] = dict(flops=6 * R * tet(n), bytes=4 * (tet(n) + 2 * n * R), bound="mfma")
    N, n = c5["N"], c5["n"]
    out["moment3_sym_N2e6_n64"] = dict(flops=N * (2 * tet(n) + tri(n)), bytes=4 * (N * n + tet(n)), bound="mfma")
    out["expand_sym_n64"] = dict(flops=0, bytes=4 * (tet(n) + n ** 3), bound="hbm")
    return out


# entry point of the step -> source file of its kernels (for the hash guard of the recorded counters)
SOURCES = {
    "mttkrp_sym3_n64_R16": "st_mttkrp.hip", "batax_utri_n8192": "st_batax.hip", "ttm_band_n512_w8_R64": "st_ttm.hip",
    "mttkrp_sym3_n512_R64": "st_mttkrp.hip", "moment3_sym_N2e6_n64": "st_moment3.hip", "expand_sym_n64": "st_expand.hip",
}


def recorded_counters():
    """Per call of the step: kernel time (sum of the average durations of its kernels, rocprofv3 kernel trace)
    and HBM bytes (FETCH_SIZE + WRITE_SIZE, scaled by the copy probe) from the committed summary -- or None for
    a call whose kernel source has changed since the counters were taken."""
    import hashlib
    rec = os.path.join(ROOT, "profiles", "bench_step_counters.txt")
    out = {}
    try:
        with open(rec) as f:
            for line in f:
                parts = line.split()
                if len(parts) != 6 or line.startswith("#"):
                    continue
                call, src, sha, kus, fetch, write = parts
                with open(os.path.join(ROOT, "paper_2211_10482_amd", "csrc", src), "rb") as g:
                    if hashlib.sha256(g.read()).hexdigest() != sha:
                        continue
                out[call] = dict(kernel_us=float(kus), traffic=float(fetch) + float(write))
    except (OSError, ValueError):
        pass
    return out


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def errors(got, ref):
    """Norm-wise error max|got-ref| / max|ref| and floored element-wise error max |got-ref| / max(|ref|, 1e-3 max|ref|)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = float(np.abs(ref).max())
    d = np.abs(got - ref)
    if scale == 0.0:
        return float(d.max()), float(d.max())
    return float(d.max() / scale), float((d / np.maximum(np.abs(ref), 1e-3 * scale)).max())


def cpu_baseline(inputs, gpu_out):
    """The oracle as it stands, timed on a bounded sample of the same step: on all host cores and on ONE
    thread (the paper's protocol, "Experimental Setup"); its results are also what `parity` compares the GPU
    outputs of the timed step with."""
    import oracle

    def timed(f):
        t0 = time.perf_counter()
        r = f()
        return r, time.perf_counter() - t0

    Tc1, B1 = inputs["c1"]
    Ap, x = inputs["c2"]
    Tc3, U = inputs["c3"]
    Tc4, B4 = inputs["c4"]
    X = inputs["c5"]
    Sc = W.uniform(7, tet(64))
    total_flops = sum(w["flops"] for w in workloads().values())
    legs, parity = {}, {}
    all_cores = oracle.num_threads()
    # (threads, rows of the n=512 MTTKRP, samples of the third moment): about 10-20 s of CPU work per leg
    for label, threads, nrows, ns in (("all_cores", all_cores, 512, 250_000), ("one_thread", 1, 48, 24_000)):
        oracle.set_num_threads(threads)
        t_est, parts = 0.0, []
        r1, t = timed(lambda: oracle.mttkrp_sym3(Tc1, B1))
        t_est += t
        parts.append("mttkrp n=64 full %.2fs" % t)
        r2, t = timed(lambda: oracle.batax_utri(Ap, x, 0.5))
        t_est += t
        parts.append("batax n=8192 full %.2fs" % t)
        r3, t = timed(lambda: oracle.ttm_band(Tc3, U, 512, 8))
        t_est += t
        parts.append("ttm full %.2fs" % t)
        rows = np.linspace(0, 511, nrows).round().astype(np.int64) if nrows < 512 else np.arange(512, dtype=np.int64)
        r4, t = timed(lambda: oracle.mttkrp_sym3(Tc4, B4, rows=rows))
        t_est += t * (512 / rows.size)
        parts.append("mttkrp n=512: %d of 512 rows %.2fs" % (rows.size, t))
        r5, t = timed(lambda: oracle.moment3_dense(X[:ns]))
        t_est += t * (X.shape[0] / ns)
        parts.append("moment3: %d of %d samples %.2fs" % (ns, X.shape[0], t))
        r6, t = timed(lambda: oracle.expand_sym(Sc, 64, 3))
        t_est += t
        parts.append("expand full %.3fs" % t)
        legs[label] = dict(value=total_flops / t_est / 1e9, cores=threads,
                           sample="; ".join(parts) + "; scaled to one full step = %.1fs" % t_est)
        if label == "all_cores" and gpu_out is not None:
            lst = oracle.list_sym3(64).astype(np.int64)
            for name, got, ref in (("mttkrp_sym3_n64_R16", gpu_out["M1"], r1), ("batax_utri_n8192", gpu_out["y"], r2),
                                   ("ttm_band_n512_w8_R64", gpu_out["Yc"], r3), ("mttkrp_sym3_n512_R64", gpu_out["M4"], r4),
                                   ("moment3_sym_first_%d_samples_n64" % ns, gpu_out["moment3_sample"](ns),
                                    r5[lst[:, 0], lst[:, 1], lst[:, 2]])):
                e, ee = errors(got, ref)
                parity[name] = dict(normwise=float("%.3e" % e), elementwise_floored=float("%.3e" % ee))
            Sd = gpu_out["S"]
            parity["expand_sym_n64"] = dict(bit_exact=bool(np.array_equal(
                Sd.view(np.uint32), oracle.expand_sym(gpu_out["Sc"], 64, 3).view(np.uint32))))
    oracle.set_num_threads(all_cores)
    a = legs["all_cores"]
    out = dict(value=a["value"], unit="GFLOP/s", cores=a["cores"], kind="oracle", sample=a["sample"],
               cpu_model=cpu_model(),
               one_thread=dict(value=legs["one_thread"]["value"], unit="GFLOP/s", cores=1,
                               sample=legs["one_thread"]["sample"]))
    return out, parity


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next", action="store_true", help="skip the rows beyond the step (moment2, moment4, expand 4, kernel table)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed region, run one plain 256 MiB device copy (a kernel of known "
                         "traffic for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the library runs on one GPU only (--gpus 1); nothing here uses a second GPU")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible (there is no CPU fallback)")
    import paper_2211_10482_amd as st
    st.lib()
    dev = torch.device("cuda:0")

    log("generating inputs ...")
    c1, c2, c3, c4, c5 = (W.CONFIGS[i] for i in range(1, 6))
    host = {
        "c1": W.mttkrp_inputs(c1["n"], c1["R"], c1["entries"], c1["b_dist"], 1),
        "c2": W.batax_inputs(c2["n"], c2["entries"]),
        "c3": W.ttm_inputs(c3["band_pairs"], c3["nl"], c3["R"]),
        "c4": W.mttkrp_inputs(c4["n"], c4["R"], c4["entries"], c4["b_dist"], 4),
        "c5": W.moment_inputs(c5["N"], c5["n"]),
    }
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    Tc1, B1 = map(up, host["c1"])
    Ap, x = map(up, host["c2"])
    Tc3, U = map(up, host["c3"])
    Tc4, B4 = map(up, host["c4"])
    X = up(host["c5"])

    # outputs and workspaces are allocated once, outside the timed region
    f32 = dict(dtype=torch.float32, device=dev)
    M1 = torch.empty((c1["n"], c1["R"]), **f32)
    y = torch.empty(c2["n"], **f32)
    Yc = torch.empty((c3["band_pairs"], c3["R"]), **f32)
    M4 = torch.empty((c4["n"], c4["R"]), **f32)
    Sc = torch.empty(c5["entries"], **f32)
    S = torch.empty((c5["n"],) * 3, **f32)
    wsb = max(st.workspace_bytes("mttkrp_sym3", n=c1["n"], R=c1["R"]),
              st.workspace_bytes("batax_utri", n=c2["n"]),
              st.workspace_bytes("ttm_band", n=c3["n"], w=c3["w"], nl=c3["nl"], R=c3["R"]),
              st.workspace_bytes("mttkrp_sym3", n=c4["n"], R=c4["R"]),
              st.workspace_bytes("moment3_sym", N=c5["N"], n=c5["n"]))
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)

    calls = [
        ("mttkrp_sym3_n64_R16", lambda: st.mttkrp_sym3(Tc1, B1, M=M1, ws=ws)),
        ("batax_utri_n8192", lambda: st.batax_utri(Ap, x, c2["beta"], y=y, ws=ws)),
        ("ttm_band_n512_w8_R64", lambda: st.ttm_band(Tc3, U, c3["n"], c3["w"], Yc=Yc, ws=ws)),
        ("mttkrp_sym3_n512_R64", lambda: st.mttkrp_sym3(Tc4, B4, M=M4, ws=ws)),
        ("moment3_sym_N2e6_n64", lambda: st.moment3_sym(X, Sc=Sc, ws=ws)),
        ("expand_sym_n64", lambda: st.expand_sym(Sc, c5["n"], 3, S=S)),
    ]

    def step(events=None):
        for name, f in calls:
            if events is not None:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                f()
                e1.record()
                events[name].append((e0, e1))
            else:
                f()

    log("warmup ...")
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # the timed region: exactly `steps` steps, nothing but the six calls between the two synchronisations
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # per-call durations: the same steps once more with an event pair around every call (the twelve event records
    # cost about 50 us per step, which is why they are kept out of the timed region)
    events = {name: [] for name, _ in calls}
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()

    if args.copy_probe:
        src = torch.empty(64 * 1024 * 1024, **f32)
        src.fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # the same calls back to back (operands that fit the last-level cache stay in it): reported beside the
    # step's figures, which see cold operands because a step touches more than the cache holds
    warm = {}
    ba = torch.randn((2048, 2048), **f32)
    bc = torch.empty_like(ba)
    for name, f in calls:
        f()
        torch.cuda.synchronize()
        # keep the GPU busy (a few small matrix products, 48 MB in all) while the timed calls are enqueued,
        # so that the events see kernels running back to back, not the host's launch latency
        for _ in range(6):
            torch.mm(ba, ba, out=bc)
        evs = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            f()
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        warm[name] = float(np.median([a.elapsed_time(b) for a, b in evs]))

    # floors of the short calls: an empty launch, and a plain streaming read of the operand, in the launch shape
    # of the kernel (event pairs like everything else; the kernel-trace durations are in profiles/)
    floors = {}
    sink = torch.zeros(16, **f32)
    def timed_median(f, reps=30):
        f()
        torch.cuda.synchronize()
        evs = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            f()
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in evs])) * 1e3
    # (not in a --copy-probe run: the copies made here would be counted with the probe's)
    floor_cases = () if args.copy_probe else (("ttm_operand_17.7MB", Tc3, (256, 1024)), ("mttkrp_operand_90MB", Tc4, (4096, 256)),
                                              ("batax_operand_134MB", Ap, (8192, 256)))
    floors["empty_launch_256x1024_us"] = round(timed_median(lambda: st.probe_empty(256, 1024)), 2)
    for tag, buf, shape in floor_cases:
        copies = [buf] + [buf.clone() for _ in range(max(2, int(600e6 // (buf.numel() * 4))))]
        k = [0]
        def f(copies=copies, shape=shape):
            k[0] += 1
            st.probe_stream(copies[k[0] % len(copies)], shape[0], shape[1], sink)
        floors["stream_read_%s_cold_%dx%d_us" % ((tag,) + shape)] = round(timed_median(f), 2)
        del copies

    # matrix-core floor of the single-precision kernels: 23 MFMAs 16x16x4 per block from registers, alone and with
    # the 9 cross-lane multiplies per block that the third-moment kernel needs for its pair products (on this
    # chip the fp32 MFMA and the vector ALU do not overlap, so the second figure is that kernel's ceiling)
    msink = torch.empty(256 * 512, **f32)
    for valu, tag in ((0, "mfma_f32_registers_only_tflops"), (9, "mfma_f32_with_9_valu_per_23_mfma_tflops")):
        fl = [0]
        def f(valu=valu):
            fl[0] = st.probe_mfma_f32(valu, 4000, msink)
        floors[tag] = round(fl[0] / 1e6 / timed_median(f, reps=10) if timed_median(f, reps=3) and fl[0] else 0.0, 2)

    wl = workloads()
    rec = recorded_counters()
    kernels = {}
    for name, _ in calls:
        t = np.array([a.elapsed_time(b) for a, b in events[name]])
        ms, ms_mean = float(np.median(t)), float(t.mean())
        w = wl[name]
        gflops = w["flops"] / (ms * 1e-3) / 1e9
        gbs = w["bytes"] / (ms * 1e-3) / 1e9
        peak = HBM_PEAK_GBS if w["bound"] == "hbm" else MFMA_FP32_PEAK_TFLOPS * 1e3
        frac = (gbs if w["bound"] == "hbm" else gflops) / peak
        r = rec.get(name)
        kus = r["kernel_us"] if r else None
        kfrac = ((w["bytes"] if w["bound"] == "hbm" else w["flops"]) / (kus * 1e-6) / 1e9 / peak) if kus else None
        kernels[name] = dict(ms=round(ms, 5), ms_mean=round(ms_mean, 5), unique_gflops=round(gflops, 2),
                             alg_gbs=round(gbs, 2), bound=w["bound"], frac=round(frac, 4), warm_ms=round(warm[name], 5),
                             kernel_us=kus, frac_kernel_trace=round(kfrac, 4) if kfrac else None,
                             alg_bytes=w["bytes"], traffic=r["traffic"] if r else None)
    total_flops = sum(w["flops"] for w in wl.values())
    value = total_flops / (ms_per_step * 1e-3) / 1e9

    dom = "moment3_sym_N2e6_n64"
    dom_ms = kernels[dom]["ms"]
    achieved = wl[dom]["flops"] / (dom_ms * 1e-3) / 1e12
    roofline = dict(kernel=dom, bound="mfma", achieved=round(achieved, 3), peak=MFMA_FP32_PEAK_TFLOPS,
                    unit="TFLOP/s", frac=round(achieved / MFMA_FP32_PEAK_TFLOPS, 4),
                    frac_kernel_trace=kernels[dom]["frac_kernel_trace"], traffic=kernels[dom]["traffic"],
                    measured_ceiling=dict(mfma_only=floors["mfma_f32_registers_only_tflops"],
                                          with_pair_products=floors["mfma_f32_with_9_valu_per_23_mfma_tflops"],
                                          unit="TFLOP/s (matrix-core flops of the probe; the kernel's padded tiles do "
                                               "47104/45760 of its unique flops on the matrix cores)"),
                    timing="median of %d event pairs around the call (main kernel + its partial-sum kernel); "
                           "frac_kernel_trace = the same flops over the rocprofv3 kernel durations in profiles/" % args.steps)

    # Rows beyond the step (order-2 and order-4 moments of the same samples, order-4 reconstruction): timed
    # on their own after the step, reported for information, not part of `value`.
    next_rows = None
    if not args.no_next:
        log("next rows (moment2, moment4, expand order 4) ...")
        n5, N5 = c5["n"], c5["N"]
        pent = n5 * (n5 + 1) * (n5 + 2) * (n5 + 3) // 24
        Sc2 = torch.empty(tri(n5), **f32)
        Sc4 = torch.empty(pent, **f32)
        S4 = torch.empty((n5,) * 4, **f32)
        ws2 = torch.empty(max(16, st.workspace_bytes("moment2_sym", N=N5, n=n5)), dtype=torch.uint8, device=dev)
        ws4 = torch.empty(max(16, st.workspace_bytes("moment4_sym", N=N5, n=n5)), dtype=torch.uint8, device=dev)
        extra = [
            ("moment2_sym_N2e6_n64", lambda: st.moment2_sym(X, Sc=Sc2, ws=ws2),
             dict(flops=N5 * 2 * tri(n5), bytes=4 * (N5 * n5 + tri(n5)), bound="hbm")),
            ("moment4_sym_N2e6_n64", lambda: st.moment4_sym(X, Sc=Sc4, ws=ws4),
             dict(flops=N5 * (2 * pent + tri(n5)), bytes=4 * (N5 * n5 + pent), bound="mfma")),
            ("expand_sym_order4_n64", lambda: st.expand_sym(Sc4, n5, 4, S=S4),
             dict(flops=0, bytes=4 * (pent + n5 ** 4), bound="hbm")),
        ]
        # the second moment at 128 and 1024 features (linear-regression covariance of wide data): strips of 64
        # columns on the matrix cores
        for Nw, nw, tag in ((1_000_000, 128, "N1e6_n128"), (100_000, 1024, "N1e5_n1024")):
            Xw = torch.randn((Nw, nw), **f32)
            Scw = torch.empty(tri(nw), **f32)
            wsw = torch.empty(max(16, st.workspace_bytes("moment2_sym", N=Nw, n=nw)), dtype=torch.uint8, device=dev)
            extra.append(("moment2_sym_" + tag, lambda Xw=Xw, Scw=Scw, wsw=wsw: st.moment2_sym(Xw, Sc=Scw, ws=wsw),
                          dict(flops=Nw * 2 * tri(nw), bytes=4 * (Nw * nw + tri(nw)), bound="mfma")))
        S1c, S2c, S3c = torch.empty(tri(n5), **f32), torch.empty(tet(n5), **f32), torch.empty(pent, **f32)
        wsc = torch.empty(max(16, st.workspace_bytes("covar_pr2", N=N5, n=n5)), dtype=torch.uint8, device=dev)
        extra += [
            ("covar_pr2_N2e6_n64", lambda: st.covar_pr2(X, S=(S1c, S2c, S3c), ws=wsc),
             dict(flops=N5 * (2 * tri(n5) + 2 * tet(n5) + tri(n5) + 2 * pent + tri(n5)),
                  bytes=4 * (3 * N5 * n5 + tri(n5) + tet(n5) + pent), bound="mfma")),
        ]
        # the same covariance at 200 features (the widest the paper's comparison systems reach), 10,000 samples
        nf, Nf = 200, 10_000
        pent_f = nf * (nf + 1) * (nf + 2) * (nf + 3) // 24
        Xf = torch.randn((Nf, nf), **f32)
        Sf = (torch.empty(tri(nf), **f32), torch.empty(tet(nf), **f32), torch.empty(pent_f, **f32))
        wsf = torch.empty(max(16, st.workspace_bytes("covar_pr2", N=Nf, n=nf)), dtype=torch.uint8, device=dev)
        extra += [
            ("covar_pr2_N1e4_n200", lambda: st.covar_pr2(Xf, S=Sf, ws=wsf),
             dict(flops=Nf * (2 * tri(nf) + 2 * tet(nf) + tri(nf) + 2 * pent_f + tri(nf)),
                  bytes=4 * (3 * Nf * nf + tri(nf) + tet(nf) + pent_f), bound="mfma")),
        ]
        # and at 6 and 13 features (the feature counts of the paper's end-to-end data sets), as many samples as config 5;
        # up to sixteen features the call is ONE pass over the samples
        ns, Ns = 13, N5
        pent_s = ns * (ns + 1) * (ns + 2) * (ns + 3) // 24
        Xs = torch.randn((Ns, ns), **f32)
        Ss = (torch.empty(tri(ns), **f32), torch.empty(tet(ns), **f32), torch.empty(pent_s, **f32))
        wss = torch.empty(max(16, st.workspace_bytes("covar_pr2", N=Ns, n=ns)), dtype=torch.uint8, device=dev)
        n6 = 6
        pent_6 = n6 * (n6 + 1) * (n6 + 2) * (n6 + 3) // 24
        X6 = torch.randn((Ns, n6), **f32)
        S6 = (torch.empty(tri(n6), **f32), torch.empty(tet(n6), **f32), torch.empty(pent_6, **f32))
        ws6 = torch.empty(max(16, st.workspace_bytes("covar_pr2", N=Ns, n=n6)), dtype=torch.uint8, device=dev)
        extra += [
            ("covar_pr2_N2e6_n6", lambda: st.covar_pr2(X6, S=S6, ws=ws6),
             dict(flops=Ns * (2 * tri(n6) + 2 * tet(n6) + tri(n6) + 2 * pent_6 + tri(n6)),
                  bytes=4 * (Ns * n6 + tri(n6) + tet(n6) + pent_6), bound="hbm")),
        ]
        extra += [
            ("covar_pr2_N2e6_n13", lambda: st.covar_pr2(Xs, S=Ss, ws=wss),
             dict(flops=Ns * (2 * tri(ns) + 2 * tet(ns) + tri(ns) + 2 * pent_s + tri(ns)),
                  bytes=4 * (Ns * ns + tri(ns) + tet(ns) + pent_s), bound="alu")),
        ]
        # the kernel table's structures at the size of the band workload (512 x 512 x 512, R = 64)
        nt, Rt = c3["n"], c3["R"]
        up_pairs = st.count_struct(st.STRUCT_UPPER, nt, nt)
        Bu = torch.empty((up_pairs, nt), **f32).uniform_(-1.0, 1.0)
        Cd = torch.empty((nt, nt, nt), **f32).uniform_(-1.0, 1.0)
        Au = torch.empty((up_pairs, Rt), **f32)
        Hu = torch.empty((up_pairs, nt), **f32)
        Tdense = torch.empty((nt, nt, c3["nl"]), **f32)
        Afk = torch.empty((nt, Rt), **f32)
        wsk = torch.empty(max(16, st.workspace_bytes("mttkrp_fixed", kind=st.MTTKRP_FIXED_K, ni=nt, nk=nt, nl=nt,
                                                     R=Rt)), dtype=torch.uint8, device=dev)
        extra += [
            ("ttm_struct_upper_n512_R64", lambda: st.ttm_struct(st.STRUCT_UPPER, Bu, U, nt, nt, Ac=Au),
             dict(flops=2 * up_pairs * nt * Rt, bytes=4 * (up_pairs * nt + nt * Rt + up_pairs * Rt), bound="mfma")),
            ("thp_struct_upper_n512", lambda: st.thp_struct(st.STRUCT_UPPER, Bu, Cd, Ac=Hu),
             dict(flops=up_pairs * nt, bytes=4 * 3 * up_pairs * nt, bound="hbm")),
            ("mttkrp_fixed_k_n512_R64", lambda: st.mttkrp_fixed(st.MTTKRP_FIXED_K, Bu[:nt], B4, U, nt, 7, A=Afk,
                                                                ws=wsk),
             dict(flops=2 * nt * nt * Rt + nt * Rt, bytes=4 * (nt * nt + 3 * nt * Rt), bound="mfma")),
            ("expand_band_n512_w8", lambda: st.expand_band(Tc3, c3["n"], c3["w"], c3["nl"], T=Tdense),
             dict(flops=0, bytes=4 * (c3["band_pairs"] * c3["nl"] + nt * nt * c3["nl"]), bound="hbm")),
        ]
        # kernels generated from a textual descriptor of the same structures (compiled at first use, which the
        # untimed first call below absorbs)
        dsym = st.Descriptor("T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)", (n5, n5, n5), "sort", n=n5)
        dband = st.Descriptor("B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)", (nt, nt, c3["nl"]), n=nt, w=c3["w"],
                              m=c3["nl"])
        Hb = torch.empty(c3["band_pairs"] * c3["nl"], **f32)
        Tc3f = Tc3.reshape(-1)
        extra += [
            ("desc_expand_sym3_n64", lambda: dsym.expand(Sc, T=S),
             dict(flops=0, bytes=4 * (tet(n5) + n5 ** 3), bound="hbm")),
            ("desc_expand_band_n512_w8", lambda: dband.expand(Tc3f, T=Tdense),
             dict(flops=0, bytes=4 * (c3["band_pairs"] * c3["nl"] + nt * nt * c3["nl"]), bound="hbm")),
            ("desc_thp_band_n512_w8", lambda: dband.thp(Tc3f, Cd, Ac=Hb),
             dict(flops=c3["band_pairs"] * c3["nl"], bytes=4 * 3 * c3["band_pairs"] * c3["nl"], bound="hbm")),
        ]
        # moment accumulation generated from a descriptor: the symmetric third moment again (vector ALUs here,
        # matrix cores in the hand-written kernel) and one only a descriptor gives: features at most 8 apart
        dnear = st.Descriptor("T(i,j,k): (0<=i<=j<n)*(j<=k<=i+w)", (n5, n5, n5), None, n=n5, w=8)
        near_count = dnear.count
        Scn, Scd = torch.empty(max(near_count, 4), **f32), torch.empty(tet(n5), **f32)
        extra += [
            ("desc_moment_sym3_N2e6_n64", lambda: dsym.moment(X, Sc=Scd),
             dict(flops=N5 * 2 * tet(n5), bytes=4 * (N5 * n5 + tet(n5)), bound="alu")),
            ("desc_moment_near3_N2e6_n64_w8", lambda: dnear.moment(X, Sc=Scn),
             dict(flops=N5 * 2 * near_count, bytes=4 * (N5 * n5 + near_count), bound="alu")),
        ]
        # the kernel table's MTTKRP generated for a sparsity structure no hand-written kernel has: the tetrahedron
        # i <= j <= l as a pattern of non-zeros (not a symmetry), 256 indices, 64 columns
        nm, Rm = 256, 64
        dtet = st.Descriptor("B(i,j,l): (0<=i<n)*(i<=j<n)*(j<=l<n)", (nm, nm, nm), None, n=nm)
        Bm = torch.randn(dtet.count, **f32)
        Cm, Dm, Am = torch.randn((nm, Rm), **f32), torch.randn((nm, Rm), **f32), torch.empty((nm, Rm), **f32)
        # ... and for the upper half cube at 512^3 (last variable free: the contraction over it runs on the matrix cores,
        # a generated kernel combines the runs of every row with the rows of C)
        dup = st.Descriptor("B(i,k,l): (0<=i<n)*(i<=k<n)*(0<=l<m)", (nt, nt, c3["nl"]), None, n=nt, m=c3["nl"])
        Bq = torch.randn(dup.count, **f32)
        Cq, Dq, Aq = torch.randn((nt, Rt), **f32), torch.randn((c3["nl"], Rt), **f32), torch.empty((nt, Rt), **f32)
        wsq = torch.empty(max(16, int(st.lib().st_desc_mttkrp_workspace(dup._h, Rt))), dtype=torch.uint8, device=dev)
        extra += [
            ("desc_mttkrp_tetra_n256_R64", lambda: dtet.mttkrp(Bm, Cm, Dm, A=Am),
             dict(flops=3 * Rm * dtet.count, bytes=4 * (dtet.count + 3 * nm * Rm), bound="alu")),
            ("desc_mttkrp_upper_n512_R64", lambda: dup.mttkrp(Bq, Cq, Dq, A=Aq, ws=wsq),
             dict(flops=2 * Rt * dup.count + 2 * Rt * dup.runs, bytes=4 * (dup.count + 3 * nt * Rt), bound="mfma")),
        ]
        next_rows = {}
        for name, f, w in extra:
            f()
            torch.cuda.synchronize()
            # a busy queue in front of the timed calls (as for the warm figures above): the events then see the
            # kernels back to back and not the host's launch path, which for the short rows is longer than the kernel
            for _ in range(6):
                torch.mm(ba, ba, out=bc)
            evs = []
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                f()
                e1.record()
                evs.append((e0, e1))
            torch.cuda.synchronize()
            ms = float(np.median([a.elapsed_time(b) for a, b in evs]))
            gflops = w["flops"] / (ms * 1e-3) / 1e9
            gbs = w["bytes"] / (ms * 1e-3) / 1e9
            frac = (gbs / HBM_PEAK_GBS if w["bound"] == "hbm" else
                    gflops / 1e3 / (ALU_FP32_PEAK_TFLOPS if w["bound"] == "alu" else MFMA_FP32_PEAK_TFLOPS))
            next_rows[name] = dict(ms=round(ms, 5), unique_gflops=round(gflops, 2), alg_gbs=round(gbs, 2),
                                   bound=w["bound"], frac=round(frac, 4))

    result = {
        "metric": "unique-element GFLOP/s over the five structured kernels, 1xMI355X",
        "value": round(value, 2),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "all five configs per step: mttkrp_sym3 n=64 R=16; batax_utri n=8192; "
                               "ttm_band n=512 w=8 nl=512 R=64; mttkrp_sym3 n=512 R=64; "
                               "moment3_sym N=2e6 n=64 + expand_sym n=64"},
        "roofline": roofline,
        "kernels": kernels,
        "floors": floors,
        "next_rows": next_rows,
    }
    if not args.no_cpu_baseline:
        log("cpu baseline (oracle on a bounded sample, all cores and one thread) and parity of the step's outputs ...")
        gpu_out = dict(M1=M1.cpu().numpy(), y=y.cpu().numpy(), Yc=Yc.cpu().numpy(), M4=M4.cpu().numpy(),
                       Sc=Sc.cpu().numpy(), S=S.cpu().numpy(),
                       moment3_sample=lambda ns: st.moment3_sym(X[:ns]).cpu().numpy())
        result["cpu_baseline"], result["parity"] = cpu_baseline(host, gpu_out)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
