#!/usr/bin/env python3
"""Benchmark of the mesh-convolution hot path on one MI355X.

One "step" = facet2vertex forward + backward (dh and dW) over the whole config-3 mesh (1024x1024
height-field, 2,093,058 facets, L=3, 64->64, bf16 features with fp32 accumulation), everything resident
in HBM, adjacency and workspaces prepared before the timed region.  Prints ONE JSON line with the
facets/s figure, the roofline position of the dominant kernel (timed with HIP events inside the library
on the launch stream) and the fp64 CPU oracle timed on the same box on a bounded sample.
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

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="untimed load before the warm-up steps: after idling (set-up, uploads) the board's power "
                         "management needs about 40 ms of this load before clocks and step times are steady "
                         "(steps 0-9 after an idle second: 1.1-1.5 ms, 10-19: 1.02, 20-29: 0.98, from 40 on: 0.955)")
    ap.add_argument("--grid", type=int, default=1024, help="height-field side (1024 = the benchmark config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--oracle-rows", type=int, default=0,
                    help="grid rows of the mesh the oracle is timed on (0 = the whole mesh, about 40 s on 16 cores)")
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5],
                    help="3 (default): the benchmark step.  1, 2, 4, 5: the op set of that configuration, one JSON line "
                         "with per-operator times, rates and roofline fractions (not the driver's line)")
    ap.add_argument("--ops", action="store_true",
                    help="instead of the benchmark step: time every operator (F2V, V2F, F2F, forward and backward) on the "
                         "same mesh and print one JSON line with per-kernel times")
    ap.add_argument("--ops-dtype", default="bf16", choices=["bf16", "f32"])
    return ap.parse_args()


def settle(fn, torch, ms):
    """Run `fn` back to back for `ms` milliseconds (untimed): brings the device from idle to its steady clocks."""
    if ms <= 0:
        return 0
    n, t0 = 0, time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(4):
            fn()
        n += 4
        torch.cuda.synchronize()
    return n


def kernel_models(F, V, K, cin, cout, e):
    """Algorithmic work per launch of each kernel of the step: flop of the contraction, bytes each array once."""
    flop = 2.0 * K * cin * cout * F
    w_bytes = K * cin * cout * e
    geom = F * 12 + V * 12                       # corner ids + vertex positions, each touched once
    return {
        # row-wise contraction: read h (and geometry), write the facet summands (feature dtype)
        "f2v/k_conv_rows": dict(bound="mfma", flop=flop, bytes=F * cin * e + geom + w_bytes + F * cout * e),
        # segmented mean: read the summands once + CSR, write g
        "f2v/k_segreduce": dict(bound="hbm", flop=F * cout * 3.0, bytes=F * cout * e + 12 * F + 4 * V + V * cout * e),
        # dh: read the gathered rows dy the weight-gradient kernel left (bf16), geometry, write dh
        "f2v_bwd/k_conv_rows": dict(bound="mfma", flop=flop, bytes=F * cout * e + geom + w_bytes + F * cin * e),
        # dW: read h, gather dg, geometry; write dy for the pass above; the dW partial sums are tiny
        "f2v_bwd/k_wgrad": dict(bound="mfma", flop=flop, bytes=F * cin * e + V * cout * e + geom + 4 * V + F * cout * e),
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the hot path is a single-GPU kernel pipeline); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2112_01801_amd import binding as pm
    from paper_2112_01801_amd import meshgen as mg

    assert torch.cuda.is_available(), "bench.py needs a GPU (there is no CPU fallback)"
    torch.cuda.set_device(0)
    pm.lib()

    if args.config != 3:
        print(json.dumps(config_ops(args, pm, mg, torch)))
        return
    cfg = mg.config3(args.grid)
    b = cfg.batch
    if args.ops:
        print(json.dumps(all_ops(args, cfg, pm, mg, torch)))
        return
    F, V, K, cin, cout = b.n_facet, b.n_vert, cfg.K, cfg.cin, cfg.cout
    rng = mg.rng_for(3, 1)
    h = mg.round_to_bf16(mg.normal_features(rng, F, cin))
    W = mg.round_to_bf16(mg.glorot_coeffs(rng, K, cin, cout))
    dg = mg.round_to_bf16(mg.normal_features(rng, V, cout))

    mesh = pm.mesh_to_device(b)
    bf = lambda x: torch.from_numpy(x).cuda().to(torch.bfloat16)
    h_d, W_d, dg_d = bf(h), bf(W), bf(dg)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    adj = pm.pm_build_vf_adjacency(mesh)
    torch.cuda.synchronize()
    setup_ms = (time.perf_counter() - t0) * 1e3

    DT = pm.PM_BF16
    ws_f = pm.alloc_workspace(pm.pm_workspace_bytes(pm.PM_OP_F2V, V, F, 0, cfg.L, cin, cout, DT))
    ws_b = pm.alloc_workspace(pm.pm_workspace_bytes(pm.PM_OP_F2V_BWD, V, F, 0, cfg.L, cin, cout, DT))
    g = torch.empty((V, cout), dtype=torch.bfloat16, device="cuda")
    dh = torch.empty((F, cin), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((K, cin, cout), dtype=torch.float32, device="cuda")

    def step():
        pm.pm_f2v(mesh, adj, cfg.L, h_d, W_d, DT, out=g, ws=ws_f)
        pm.pm_f2v_bwd(mesh, adj, cfg.L, h_d, W_d, dg_d, DT, dh=dh, dW=dW, ws=ws_b)

    models = kernel_models(F, V, K, cin, cout, 2)

    def kernel_table(recs, n_steps):
        agg = {}
        for name, ms in recs:
            a = agg.setdefault(name, [0.0, 0])
            a[0] += ms
            a[1] += 1
        rows = []
        for name, (tot, cnt) in agg.items():
            avg = tot / cnt
            ent = {"kernel": name, "launches_per_step": cnt / n_steps, "avg_ms": round(avg, 5),
                   "ms_per_step": round(tot / n_steps, 5)}
            m = models.get(name)
            if m:
                if m["bound"] == "mfma":
                    ach = m["flop"] / (avg * 1e-3) / 1e12
                    ent.update(bound="mfma", achieved=round(ach, 2), peak=PEAK_MFMA_TFLOPS["bf16"], unit="TFLOP/s",
                               frac=round(ach / PEAK_MFMA_TFLOPS["bf16"], 4),
                               hbm_gbs_algorithmic=round(m["bytes"] / (avg * 1e-3) / 1e9, 1))
                else:
                    ach = m["bytes"] / (avg * 1e-3) / 1e9
                    ent.update(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                               frac=round(ach / PEAK_HBM_GBS, 4))
            rows.append(ent)
        rows.sort(key=lambda k: -k["ms_per_step"])
        return rows

    # Warm-up.  Every kernel of the warm-up steps is bracketed by HIP events (the `kernels` table); that finds
    # the dominant kernel.  A pair of events costs the stream a few microseconds (14 pairs a step: ~5 % of this
    # step), so the timed region brackets the dominant kernel alone, whose durations give `roofline`.
    settled = settle(step, torch, args.settle_ms)
    pm.pm_profile_filter("")
    pm.pm_profile_reset()
    pm.pm_profile_enable(True)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    pm.pm_profile_enable(False)
    wrecs = pm.pm_profile_read()
    wsteps = args.warmup
    if args.warmup >= 2:                              # the first step pays one-time costs (code load, cold caches)
        per = len(wrecs) // args.warmup
        wrecs, wsteps = wrecs[per:], args.warmup - 1
    warm = kernel_table(wrecs, max(wsteps, 1))
    pm.pm_profile_reset()
    dom_name = next((k["kernel"] for k in warm if "bound" in k), "")

    pm.pm_profile_filter(dom_name)
    pm.pm_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    pm.pm_profile_enable(False)
    recs = pm.pm_profile_read()
    pm.pm_profile_reset()
    pm.pm_profile_filter("")
    assert torch.isfinite(g.float()).all() and torch.isfinite(dW).all()

    ms_per_step = elapsed * 1e3 / args.steps
    value = F * args.steps / elapsed

    timed = kernel_table(recs, args.steps)            # the dominant kernel over the timed region (all kernels if W = 0)
    if warm:
        # the other kernels: the same number of steps once more, untimed, every kernel bracketed
        pm.pm_profile_enable(True)
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        pm.pm_profile_enable(False)
        post = kernel_table(pm.pm_profile_read(), args.steps)
        pm.pm_profile_reset()
        kernels = [next((t for t in timed if t["kernel"] == k["kernel"]), k) for k in post]
        kernels_from = "an untimed repeat of the timed steps with every kernel bracketed"
    else:
        kernels, kernels_from = timed, "timed steps"
    dom = next((k for k in timed if "bound" in k), None)
    roofline = None
    if dom:
        traffic = read_traffic(dom["kernel"], args.grid)
        roofline = {"kernel": dom["kernel"], "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                    "unit": dom["unit"], "frac": dom["frac"], "traffic": traffic,
                    "traffic_source": None if traffic is None else
                    "stored, not measured in this run: profiles/hbm_traffic_c3.txt (rocprofv3 --pmc FETCH_SIZE and "
                    "WRITE_SIZE runs of this command, bytes per launch of this kernel)",
                    "avg_ms": dom["avg_ms"]}

    # board power while the same step runs back to back for ~1.5 s (untimed; the sensor is slow).  The
    # published matrix peak assumes the top clock; under the board's power cap the clock drops with activity.
    power = board_power(step, torch)

    # what this device sustains in short issue loops, beside the published peaks
    pws = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    peaks = {}
    for key, kind in (("mfma_bf16_ones", pm.PM_PEAK_MFMA_BF16_ONES), ("mfma_bf16_random", pm.PM_PEAK_MFMA_BF16_RANDOM),
                      ("hbm_copy", pm.PM_PEAK_HBM_COPY)):
        rate, clk = pm.pm_peak_probe(kind, pws)
        peaks[key] = {"value": round(rate, 1), "unit": "GB/s" if key == "hbm_copy" else "TFLOP/s",
                      "shader_clock_mhz": round(clk)}
    del pws
    if roofline:
        ref = peaks["mfma_bf16_random"]["value"] if roofline["bound"] == "mfma" else peaks["hbm_copy"]["value"]
        roofline["frac_of_measured_peak"] = round(roofline["achieved"] / ref, 4)
        roofline["measured_peak"] = ref

    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = oracle_baseline(cfg, min(args.oracle_rows, args.grid) if args.oracle_rows > 0 else args.grid, h, W, dg)

    out = {
        "metric": "mesh-conv facets/sec (fwd+bwd) at 1 MI355X",
        "value": value, "unit": "facets/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": settled,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 3: %dx%d height-field, F=%d V=%d, L=3 (K=16), 64->64, bf16 in / fp32 "
                               "accumulate, facet2vertex forward + backward (dh, dW)" % (args.grid, args.grid, F, V),
                   "ops": ["pm_f2v", "pm_f2v_bwd"], "adjacency_setup_ms": round(setup_ms, 3)},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "measured_peaks": peaks,
        "board_power": power,
        "kernels_measured_over": kernels_from + " (the roofline kernel: timed steps)",
        "kernels": kernels,
    }
    print(json.dumps(out))


def op_model(op, F, V, P, K, cin, cout, e):
    """Algorithmic work of one operator call: matrix flop as executed, and the bytes of every array touched once
    (ids 12 B per facet, positions 12 B per vertex, CSR 12 B per facet + 4 B per vertex, features e bytes per element)."""
    kcc = K * cin * cout
    csr = 12 * F + 4 * V
    geom = 12 * F + 12 * V
    m = {
        "f2v": (2 * kcc * F, geom + F * cin * e + csr + V * cout * e),
        "f2v_bwd": (4 * kcc * F, geom + 4 * V + V * cout * e + 2 * F * cin * e + kcc * 4),
        "v2f": (2 * 3 * cin * cout * F, 12 * F + V * cin * e + F * cout * e),
        "v2f_bwd": (4 * 3 * cin * cout * F, 12 * F + csr + F * cout * e + 2 * V * cin * e + kcc * 4),
        "f2f": (2 * kcc * P, P * (12 + cin * e) + 4 * F + F * cout * e),
        "f2f_bwd": (4 * kcc * P, P * (12 + 2 * cin * e) + 4 * F + F * cout * e + kcc * 4),
    }
    flop, byts = m[op]
    return float(flop), float(byts)


def config_ops(args, pm, mg, torch):
    """The op set of configuration 1, 2, 4 or 5 on its own synthetic meshes: per operator the kernel time (HIP events
    inside the library), rows/s, matrix TFLOP/s and algorithmic GB/s with their fractions of the published peaks."""
    n = args.config
    if n == 1:
        c = mg.config1()
        runs = [("config 1", c.batch, c.L, "f32", [("f2v", c.cin, c.cout), ("v2f", c.cin, c.cout)])]
    elif n == 2:
        c = mg.config2(16)
        both = lambda op: [(op, c.cin, c.cout), (op + "_bwd", c.cin, c.cout)]
        runs = [("config 2", c.batch, c.L, "f32", both("f2v") + both("v2f") + both("f2f"))]
    elif n == 4:
        c = mg.config4()
        ops = [("v2f", 32, 128), ("v2f_bwd", 32, 128), ("f2v", 128, 128), ("f2v_bwd", 128, 128), ("f2f", 32, 128),
               ("f2f_bwd", 32, 128)]
        runs = [("config 4", c.batch, c.L, "f32", ops)]
    else:
        runs = []
        for lvl, c in enumerate(mg.config5_levels()):
            ops = [(op + sfx, c.cin, c.cout) for op in ("f2v", "v2f", "f2f") for sfx in ("", "_bwd")]
            runs.append(("config 5 level %d" % lvl, c.batch, c.L, "bf16", ops))
    out = {"metric": "mesh-conv facets/sec (fwd+bwd) at 1 MI355X", "unit": "facets/s", "config": n, "steps": args.steps,
           "note": "kernel times from HIP events inside the library; one operator at a time, inputs resident in HBM; "
                   "adjacency and workspaces prepared before; an extra row times facet2facet at the paper's own "
                   "shape (3 colour channels in, Eq. 7)", "runs": []}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20211201 + n)
    tot_ms_all, tot_F_all = 0.0, 0
    for name, b, L, dtype, ops in runs:
        F, V, K = b.n_facet, b.n_vert, (L + 1) ** 2
        DT = pm.PM_BF16 if dtype == "bf16" else pm.PM_F32
        tdt, e = (torch.bfloat16, 2) if dtype == "bf16" else (torch.float32, 4)
        peak = PEAK_MFMA_TFLOPS[dtype]
        rnd = lambda *sh: torch.randn(*sh, device="cuda", generator=gen).to(tdt)
        mesh = pm.mesh_to_device(b)
        adj = pm.pm_build_vf_adjacency(mesh)
        tex_off, bary = mg.texture_layout(b, 3, 1)
        P = int(tex_off[-1])
        t_off, t_bary = torch.from_numpy(tex_off).cuda(), torch.from_numpy(bary).cuda()
        rows = []
        for op, cin, cout in ops + [("f2f", 3, 32), ("f2f_bwd", 3, 32)]:
            W = ((torch.rand(K, cin, cout, device="cuda", generator=gen) * 2 - 1) * (6.0 / (K * cin + cout)) ** 0.5).to(tdt)
            if op == "f2v":
                x = rnd(F, cin); fn = lambda: pm.pm_f2v(mesh, adj, L, x, W, DT)
            elif op == "f2v_bwd":
                x, d = rnd(F, cin), rnd(V, cout); fn = lambda: pm.pm_f2v_bwd(mesh, adj, L, x, W, d, DT)
            elif op == "v2f":
                x = rnd(V, cin); fn = lambda: pm.pm_v2f(mesh, L, x, W, DT)
            elif op == "v2f_bwd":
                x, d = rnd(V, cin), rnd(F, cout); fn = lambda: pm.pm_v2f_bwd(mesh, adj, L, x, W, d, DT)
            elif op == "f2f":
                x = rnd(P, cin); fn = lambda: pm.pm_f2f(t_off, t_bary, L, x, W, DT)
            else:
                x, d = rnd(P, cin), rnd(F, cout); fn = lambda: pm.pm_f2f_bwd(t_off, t_bary, L, x, W, d, DT)
            settle(fn, torch, args.settle_ms)
            for _ in range(max(1, args.warmup)):
                fn()
            torch.cuda.synchronize()
            pm.pm_profile_reset()
            pm.pm_profile_enable(True)
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            pm.pm_profile_enable(False)
            kern = {}
            for label, ms in pm.pm_profile_read():
                k = label.split("/", 1)[1]
                kern[k] = kern.get(k, 0.0) + ms / args.steps
            pm.pm_profile_reset()
            ms = sum(kern.values())
            flop, byts = op_model(op, F, V, P, K, cin, cout, e)
            tf, gbs = flop / (ms * 1e-3) / 1e12, byts / (ms * 1e-3) / 1e9
            extra = cin == 3
            rows.append({"op": op + (" (paper shape)" if extra else ""), "cin": cin, "cout": cout, "ms": round(ms, 4),
                         "facets_per_s": round(F / (ms * 1e-3)), "tflops": round(tf, 2), "frac_mfma": round(tf / peak, 4),
                         "gbs_algorithmic": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4),
                         "kernels_ms": {k: round(v, 4) for k, v in sorted(kern.items(), key=lambda kv: -kv[1])}})
            del x
            if not extra:
                tot_ms_all += ms
        tot_F_all += F
        named = [r for r in rows if "paper shape" not in r["op"]]
        out["runs"].append({"workload": "%s: F=%d V=%d meshes=%d texture points=%d, L=%d, %s" %
                                        (name, F, V, b.n_mesh, P, L, dtype),
                            "facets_per_s_op_set": round(F / (sum(r["ms"] for r in named) * 1e-3)),
                            "ms_op_set": round(sum(r["ms"] for r in named), 4), "peak_tflops": peak, "ops": rows})
    out["value"] = tot_F_all / (tot_ms_all * 1e-3)
    out["ms_per_step"] = tot_ms_all
    return out


def all_ops(args, cfg, pm, mg, torch):
    """Per-kernel event times of every operator on the benchmark mesh (textures of Eq. 8 with (alpha, beta) = (3, 1))."""
    b = cfg.batch
    F, V, K, cin, cout, L = b.n_facet, b.n_vert, cfg.K, cfg.cin, cfg.cout, cfg.L
    DT = pm.PM_BF16 if args.ops_dtype == "bf16" else pm.PM_F32
    tdt = torch.bfloat16 if DT == pm.PM_BF16 else torch.float32
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20211201 + 3)
    rnd = lambda *sh: torch.randn(*sh, device="cuda", generator=gen).to(tdt)
    W = ((torch.rand(K, cin, cout, device="cuda", generator=gen) * 2 - 1) * (6.0 / (K * cin + cout)) ** 0.5).to(tdt)
    mesh = pm.mesh_to_device(b)
    adj = pm.pm_build_vf_adjacency(mesh)
    tex_off, bary = mg.texture_layout(b, 3, 1)
    P = int(tex_off[-1])
    t_off, t_bary = torch.from_numpy(tex_off).cuda(), torch.from_numpy(bary).cuda()
    hF, hV, hP, dgV, dgF = rnd(F, cin), rnd(V, cin), rnd(P, cin), rnd(V, cout), rnd(F, cout)
    # separable form: W[k, ci, co] = alpha[k, ci] * Pw[ci, co]
    alpha = (torch.rand(K, cin, device="cuda", generator=gen) * 2 - 1) / K ** 0.5
    Pw = ((torch.rand(cin, cout, device="cuda", generator=gen) * 2 - 1) * (3.0 / cin) ** 0.5).to(tdt)
    _, zV = pm.pm_f2v_sep(mesh, adj, L, hF, alpha, Pw, DT, save_z=True)
    ops = {
        "f2v": (lambda: pm.pm_f2v(mesh, adj, L, hF, W, DT), F),
        "f2v_bwd": (lambda: pm.pm_f2v_bwd(mesh, adj, L, hF, W, dgV, DT), F),
        "v2f": (lambda: pm.pm_v2f(mesh, L, hV, W, DT), F),
        "v2f_bwd": (lambda: pm.pm_v2f_bwd(mesh, adj, L, hV, W, dgF, DT), F),
        "f2f": (lambda: pm.pm_f2f(t_off, t_bary, L, hP, W, DT), P),
        "f2f_bwd": (lambda: pm.pm_f2f_bwd(t_off, t_bary, L, hP, W, dgF, DT), P),
        "f2v_sep": (lambda: pm.pm_f2v_sep(mesh, adj, L, hF, alpha, Pw, DT), F),
        "f2v_sep_bwd": (lambda: pm.pm_f2v_sep_bwd(mesh, adj, L, hF, alpha, Pw, dgV, DT), F),
        "f2v_sep_bwd_saved_z": (lambda: pm.pm_f2v_sep_bwd(mesh, adj, L, hF, alpha, Pw, dgV, DT, z_saved=zV), F),
        "v2f_sep": (lambda: pm.pm_v2f_sep(mesh, L, hV, alpha, Pw, DT), F),
        "v2f_sep_bwd": (lambda: pm.pm_v2f_sep_bwd(mesh, adj, L, hV, alpha, Pw, dgF, DT), F),
    }
    if cin == cout:
        # separable vertex2vertex block (vertex2facet -> affine, ReLU -> facet2vertex -> affine, ReLU), C -> C -> C
        ep = pm.Epilogue(torch.rand(cout, device="cuda", generator=gen) + 0.5,
                         torch.randn(cout, device="cuda", generator=gen) * 0.3, True)
        oV, gF, zV2 = pm.pm_v2v_sep(mesh, adj, L, hV, alpha, Pw, ep, alpha, Pw, ep, DT, save=True)
        ops["v2v_sep"] = (lambda: pm.pm_v2v_sep(mesh, adj, L, hV, alpha, Pw, ep, alpha, Pw, ep, DT), F)
        ops["v2v_sep_saving"] = (lambda: pm.pm_v2v_sep(mesh, adj, L, hV, alpha, Pw, ep, alpha, Pw, ep, DT, save=True), F)
        ops["v2v_sep_bwd"] = (lambda: pm.pm_v2v_sep_bwd(mesh, adj, L, hV, alpha, Pw, ep, alpha, Pw, ep, gF, zV2, oV,
                                                        dgV, DT), F)
    if args.grid >= 4:
        # point-cloud convolution on the vertices of the level two decimations down (the resolution the paper's
        # dual blocks use it at), neighbours of a range search of about six grid spacings
        import numpy as np
        gn = args.grid // 2
        pv, _ = mg.heightfield(gn, gn, np.random.default_rng(20211201 + 4))
        rho = 5.5 / (gn - 1)
        nptr, nidx = mg.range_neighbors(pv, pv, rho)
        pts = torch.from_numpy(np.ascontiguousarray(pv, dtype=np.float32)).cuda()
        nb = pm.Neighbors(pts, pts, torch.from_numpy(nptr).cuda(), torch.from_numpy(nidx).cuda(), rho)
        c0 = torch.rand(cin, device="cuda", generator=gen) * 2 - 1
        hN, dgN = rnd(gn * gn, cin), rnd(gn * gn, cout)
        nb_rev = pm.pm_build_reverse_neighbors(nb)
        _, yN = pm.pm_pcloud_conv(nb, L, hN, alpha, c0, Pw, DT, save_y=True)
        ops.update({
            "pcloud_conv": (lambda: pm.pm_pcloud_conv(nb, L, hN, alpha, c0, Pw, DT), int(nidx.shape[0])),
            "pcloud_conv_bwd": (lambda: pm.pm_pcloud_conv_bwd(nb, L, hN, alpha, c0, Pw, dgN, DT), int(nidx.shape[0])),
            "pcloud_conv_bwd_saved": (lambda: pm.pm_pcloud_conv_bwd(nb_rev, L, hN, alpha, c0, Pw, dgN, DT, y_saved=yN),
                                      int(nidx.shape[0])),
        })
    ops.update({
        "facet_geometry": (lambda: pm.pm_facet_geometry(mesh, DT, True), F),
        "texture_layout": (lambda: pm.pm_texture_layout(mesh, 3, 1), F),
    })
    if args.grid % 2 == 0:
        # pooling between this mesh and its 2x2-clustered coarse level (the hierarchy of config 5)
        vc, io = mg.grid_cluster_maps(args.grid, args.grid)
        Vc = (args.grid // 2) ** 2
        cm = pm.pm_build_cluster_map(torch.from_numpy(vc).cuda(), torch.from_numpy(io).cuda(), Vc)
        hC = rnd(Vc, cin)
        _, amax = pm.pm_pool(cm, pm.PM_POOL_MAX, hV, DT)
        ops.update({
            "cluster_map": (lambda: pm.pm_build_cluster_map(cm_in[0], cm_in[1], Vc), V),
            "pool_max": (lambda: pm.pm_pool(cm, pm.PM_POOL_MAX, hV, DT), V),
            "pool_max_bwd": (lambda: pm.pm_pool_bwd(cm, pm.PM_POOL_MAX, hC, DT, argmax=amax), V),
            "pool_avg": (lambda: pm.pm_pool(cm, pm.PM_POOL_AVG, hV, DT), V),
            "pool_avg_bwd": (lambda: pm.pm_pool_bwd(cm, pm.PM_POOL_AVG, hC, DT), V),
            "unpool": (lambda: pm.pm_unpool(cm, hC, DT), V),
            "unpool_bwd": (lambda: pm.pm_unpool_bwd(cm, hV, DT), V),
        })
        cm_in = (torch.from_numpy(vc).cuda(), torch.from_numpy(io).cuda())
    out = {"workload": "config 3 mesh %dx%d: F=%d V=%d texture points=%d, L=%d, %d->%d, %s" %
                       (args.grid, args.grid, F, V, P, L, cin, cout, args.ops_dtype),
           "steps": args.steps, "ops": {}}
    for name, (fn, rows) in ops.items():
        settle(fn, torch, args.settle_ms)
        for _ in range(max(1, args.warmup)):
            fn()
        torch.cuda.synchronize()
        pm.pm_profile_reset()
        pm.pm_profile_enable(True)
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        pm.pm_profile_enable(False)
        agg = {}
        for label, ms in pm.pm_profile_read():
            agg[label] = agg.get(label, 0.0) + ms / args.steps
        pm.pm_profile_reset()
        tot = sum(agg.values())
        kern = {}
        for k, v in agg.items():        # an operator built from other entry points carries their labels: by kernel
            kern[k.split("/", 1)[1]] = round(kern.get(k.split("/", 1)[1], 0.0) + v, 4)
        out["ops"][name] = {"kernel_ms": round(tot, 4), "rows": rows, "rows_per_s": round(rows / (tot * 1e-3)),
                            "kernels": kern}
    return out


def board_power(step, torch):
    """Mean of the board power sensor (W) while `step` runs in a loop, or None when no sensor is readable."""
    import glob
    import threading
    paths = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") + \
        glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")
    if not paths:
        return None

    def read():
        try:
            with open(paths[0]) as f:
                return int(f.read()) / 1e6
        except (OSError, ValueError):
            return None
    idle = read()
    if idle is None:
        return None
    samples, stop = [], [False]

    def sampler():
        while not stop[0]:
            v = read()
            if v is not None:
                samples.append(v)
            time.sleep(0.05)
    th = threading.Thread(target=sampler)
    th.start()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 1.5:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    stop[0] = True
    th.join()
    tail = samples[len(samples) // 3:]
    if not tail:
        return None
    return {"step_loop_w": round(sum(tail) / len(tail)), "before_w": round(idle), "sensor": paths[0]}


def read_traffic(kernel, grid):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if one covers this kernel."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_c3.txt")
    if grid != 1024 or not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == kernel:
            try:
                return float(parts[1])
            except ValueError:
                return None
    return None


def oracle_baseline(cfg, rows, h, W, dg):
    """The fp64 oracle, as it stands, on the first `rows` grid rows of the same mesh (a bounded sample)."""
    import numpy as np
    import oracle
    from paper_2112_01801_amd import meshgen as mg
    nx = cfg.info["ny"]
    b = cfg.batch
    Vs = rows * nx
    Fs = 2 * (rows - 1) * (nx - 1)
    sub = mg.pack_batch([(b.vert[:Vs], b.facet[:Fs])])
    assert int(sub.facet.max()) < Vs
    hs, dgs = h[:Fs], dg[:Vs]
    t0 = time.perf_counter()
    oracle.f2v(sub.vert, sub.facet, cfg.L, hs, W)
    oracle.f2v_bwd(sub.vert, sub.facet, cfg.L, hs, W, dgs)
    dt = time.perf_counter() - t0
    what = "the whole mesh" if rows == nx else "the first %d of %d grid rows of the same mesh" % (rows, nx)
    return {"value": Fs / dt, "unit": "facets/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "facet2vertex forward + backward (dh, dW) in fp64 on %s (%d facets), %.1f s" % (what, Fs, dt)}


if __name__ == "__main__":
    main()
