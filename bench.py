#!/usr/bin/env python3
"""Benchmark of the ECC hot path on one MI355X.

A step is one ecc_hard call (batch-global range, thresholds, coefficient sweep,
histogram, merge, scan) over workload C2: a batch of 16 2D 4096x4096 float32
smoothed Gaussian random fields, 1024 equal-width bins over the batch-global
[min, max] computed on the device.  Inputs are resident in HBM before the
timed region.  The same run also times, as extra fields of the one JSON line,
the 3D 512^3 float32 volume (C4), the hard path with the range supplied, the
two integer workloads (C1, C3), directional curves (16 directions over one
4096^2 field, ecc_hard_dir), soft forward + backward over the 32 x 512^2
batch (C5) and over one 256^3 volume, and the CPU oracle on the host cores (a baseline, not the target).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--quick]
    python bench.py --only c2|c2r|c4|c5|dir|calib   one workload (profiling runs)
    python bench.py --sweep                         the grid sizes of the paper's Tables 1-2
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_steps(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3  # ms per step


# "New" kernel times of the paper's Tables 1 and 2 (ms, one RTX A6000; dtype, bins and timing
# method not stated there): context beside the sizes below, not a target.
PAPER_MS = {(128, 128): 0.0165, (256, 256): 0.0174, (512, 512): 0.021, (1024, 1024): 0.032,
            (2048, 2048): 0.11, (4096, 4096): 0.408, (8192, 8192): 1.6, (128, 128, 128): 0.1,
            (256, 256, 256): 0.71, (512, 512, 512): 5.61, (1024, 1024, 1024): 48.47}


def run_sweep(args, np, torch, api, synth):
    """One float32 smoothed random field of each size of the paper's Tables 1-2, 1024 bins over
    the range found on the device (the whole hot path per call).  The 1024^3 volume is the
    periodic 512^3 field tiled 2x2x2 (the generator smooths with wrap-around, so the tiling is
    seamless); exact duplicates across tiles are ties like any other."""
    rows = []
    for shape in PAPER_MS:
        nd = len(shape)
        if shape == (1024, 1024, 1024):
            X = np.tile(synth.grf((512, 512, 512), 3.0, 4242), (2, 2, 2))
        else:
            X = synth.grf(shape, 4.0 if nd == 2 else 3.0, 4242)
        g = torch.from_numpy(X[None]).cuda()
        ws = torch.empty(api.ecc_workspace_bytes(shape, 1, 1024), dtype=torch.uint8, device="cuda")
        cv = torch.empty((1, 1024), dtype=torch.int64, device="cuda")
        fn = lambda: api.ecc_hard(g, nd, 1024, curve=cv, workspace=ws)
        ms = time_steps(fn, args.steps, args.warmup)
        assert int(cv[0, -1]) == 1  # the full grid is contractible
        n = int(np.prod(shape))
        rows.append({"shape": "x".join(map(str, shape)), "ms": round(ms, 4), "gvoxel_per_s": round(n / ms / 1e6, 1),
                     "paper_ms_rtx_a6000": PAPER_MS[shape]})
        log(f"[bench] sweep {rows[-1]['shape']:>14}: {ms:8.4f} ms  {rows[-1]['gvoxel_per_s']:8.1f} Gvoxel/s"
            f"   (paper, RTX A6000: {PAPER_MS[shape]} ms)")
        del g, ws, cv, X
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "hard_ecc_size_sweep", "unit": "ms", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": "one float32 smoothed random field per size of the paper's "
                                             "Tables 1-2, 1024 bins, range found on the device"},
                      "rows": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--quick", action="store_true", help="skip the extra workloads and the CPU baseline")
    ap.add_argument("--sweep", action="store_true",
                    help="time one grid of every size of the paper's Tables 1-2 instead (own JSON line)")
    ap.add_argument("--only", default="", help="profiling aid: run only 'c2', 'c2r' (range supplied), 'c4', 'c5', 'dir' or 'calib' (a plain 1 GiB copy), no JSON")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (the path shards by batch item / "
              "z-slab with one all-reduce of the histogram, which this single-GPU build does not include)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_20271_amd import _lib, api, synth

    _lib.load()  # fails loudly when the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.only == "calib":
        # counter calibration: a plain device copy of exactly 1 GiB read + 1 GiB written per launch
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("[bench] calib: copied 1 GiB x %d" % args.steps)
        return
    BINS = 1024
    extra = {}
    if args.sweep:
        run_sweep(args, np, torch, api, synth)
        return

    # ---------------- C2: the headline workload --------------------------------
    if args.only in ("", "c2", "c2r"):
        t0 = time.perf_counter()
        X2 = synth.config_c2()
        log(f"[bench] generated C2 {X2.shape} in {time.perf_counter() - t0:.1f}s")
        g2 = torch.from_numpy(X2).cuda()
        ws2 = torch.empty(api.ecc_workspace_bytes(X2.shape[1:], X2.shape[0], BINS), dtype=torch.uint8, device="cuda")
        curve2 = torch.empty((X2.shape[0], BINS), dtype=torch.int64, device="cuda")
        step = lambda: api.ecc_hard(g2, 2, BINS, curve=curve2, workspace=ws2)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        api.ecc_profile_begin(args.steps)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        sweep_ms, nl = api.ecc_profile_end()
        nvox = X2.size
        value = nvox / (ms * 1e-3) / 1e9
        alg_bytes = 4.0 * nvox  # one float32 read per vertex per sweep launch
        achieved = alg_bytes / (sweep_ms * 1e-3) / 1e9
        traffic = None
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
        if os.path.exists(tpath):
            traffic = json.load(open(tpath)).get("c2_sweep_bytes_per_launch")
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                    "kernel": "sweep2d_list_kernel (coefficient sweep + range + critical-vertex lists)", "kernel_ms": round(sweep_ms, 4),
                    "launches_timed": nl, "algorithmic_bytes_per_launch": alg_bytes}
        log(f"[bench] C2: {ms:.3f} ms/step, {value:.1f} Gvoxel/s, sweep kernel {sweep_ms:.3f} ms")
        if args.only == "c2":
            return
        if args.only == "c2r":  # profiling aid: the histogram-mode sweep (range supplied)
            rng2 = (float(X2.min()), float(X2.max()))
            ms_r = time_steps(lambda: api.ecc_hard(g2, 2, BINS, range=rng2, curve=curve2, workspace=ws2),
                              args.steps, args.warmup)
            log(f"[bench] C2, range supplied: {ms_r:.3f} ms/step")
            return
        if not args.quick:
            rng2 = (float(X2.min()), float(X2.max()))
            ms_r = time_steps(lambda: api.ecc_hard(g2, 2, BINS, range=rng2, curve=curve2, workspace=ws2),
                              args.steps, args.warmup)
            extra["c2_range_supplied"] = {"ms_per_step": round(ms_r, 4), "gvoxel_per_s": round(nvox / ms_r / 1e6, 1),
                                          "hbm_frac_one_pass": round(alg_bytes / (ms_r * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
            # CPU oracle on the same batch, as it stands
            from oracle import ecc_oracle as O
            from oracle import ecc_oracle_c as OC
            nitem = X2.shape[0]  # the whole batch: a couple of seconds on the host cores
            t0 = time.perf_counter()
            lo, hi = X2.min(), X2.max()
            ref = OC.ecc_hard_batch(X2[:nitem], O.thresholds_equal_width(lo, hi, BINS))
            dt = time.perf_counter() - t0
            cpu = {"value": round(nitem * X2[0].size / dt / 1e9, 4), "unit": "Gvoxel/s", "cores": OC.threads(),
                   "kind": "oracle", "sample": f"the whole C2 batch, {nitem} items, thresholds from its min/max "
                   f"({dt:.1f} s of host time)"}
            got = curve2[:nitem].cpu().numpy()
            extra["c2_sample_matches_oracle"] = bool(np.array_equal(got, ref))
        del g2, X2
        torch.cuda.empty_cache()

    # ---------------- C4: 3D 512^3 float32 -------------------------------------
    if args.only in ("", "c4") and (not args.quick or args.only == "c4"):
        t0 = time.perf_counter()
        X4 = synth.config_c4()[None]
        log(f"[bench] generated C4 {X4.shape} in {time.perf_counter() - t0:.1f}s")
        g4 = torch.from_numpy(X4).cuda()
        ws4 = torch.empty(api.ecc_workspace_bytes(X4.shape[1:], 1, BINS), dtype=torch.uint8, device="cuda")
        curve4 = torch.empty((1, BINS), dtype=torch.int64, device="cuda")
        step4 = lambda: api.ecc_hard(g4, 3, BINS, curve=curve4, workspace=ws4)
        for _ in range(args.warmup):
            step4()
        torch.cuda.synchronize()
        api.ecc_profile_begin(args.steps)
        ms4 = time_steps(step4, args.steps, 0)
        sweep4, _ = api.ecc_profile_end()
        rng4 = (float(X4.min()), float(X4.max()))
        ms4r = time_steps(lambda: api.ecc_hard(g4, 3, BINS, range=rng4, curve=curve4, workspace=ws4),
                          args.steps, args.warmup)
        b4 = 4.0 * X4.size
        extra["c4"] = {"workload": "C4: 3D 512^3 float32 GRF sigma=3, 1024 bins",
                       "ms_per_step_auto_range": round(ms4, 4), "ms_per_step_range_supplied": round(ms4r, 4),
                       "gvoxel_per_s_auto_range": round(X4.size / ms4 / 1e6, 1),
                       "gvoxel_per_s_range_supplied": round(X4.size / ms4r / 1e6, 1),
                       "sweep_kernel_ms": round(sweep4, 4),
                       "sweep_hbm_frac": round(b4 / (sweep4 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        log(f"[bench] C4: {ms4:.3f} ms/step (range supplied {ms4r:.3f}), sweep kernel {sweep4:.3f} ms")
        if args.only == "c4":
            return
        del g4, X4
        torch.cuda.empty_cache()

    # ---------------- C1 / C3: integer levels, one bin per level ----------------
    if (args.only == "" and not args.quick) or args.only in ("c1", "c3"):
        for name, X, nd, bins in (("c1", synth.config_c1()[None], 2, 256), ("c3", synth.config_c3()[None], 3, 4096)):
            if args.only and args.only != name:
                continue
            if X.dtype == np.uint16:
                gi = torch.from_numpy(X.view(np.int16)).cuda().view(torch.uint16)
            else:
                gi = torch.from_numpy(X).cuda()
            wsi = torch.empty(api.ecc_workspace_bytes(X.shape[1:], 1, bins), dtype=torch.uint8, device="cuda")
            cvi = torch.empty((1, bins), dtype=torch.int64, device="cuda")
            fn = lambda: api.ecc_hard(gi, nd, bins, curve=cvi, workspace=wsi)
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            api.ecc_profile_begin(args.steps)
            msi = time_steps(fn, args.steps, 0)
            swi, _ = api.ecc_profile_end()
            extra[name] = {"workload": {"c1": "C1: 2D 256^2 uint8 i.i.d., 256 levels (launch-latency bound, 3 launches)",
                                        "c3": "C3: 3D 256^3 uint16 i.i.d., 4096 levels"}[name],
                           "us_per_step": round(msi * 1e3, 2), "sweep_kernel_us": round(swi * 1e3, 2),
                           "gvoxel_per_s": round(X.size / msi / 1e6, 2)}
            log(f"[bench] {name}: {msi * 1e3:.1f} us/step, sweep {swi * 1e3:.1f} us")
            del gi
        if args.only in ("c1", "c3"):
            return

    # ---------------- directional curves: 16 directions of one 4096^2 field --------
    if args.only in ("", "dir") and (not args.quick or args.only == "dir"):
        Xd = synth.grf((4096, 4096), 4.0, 2002)[None]
        th = np.linspace(0.0, np.pi, 16, endpoint=False)
        Ud = np.stack([np.cos(th), np.sin(th)], 1).astype(np.float32)
        gd, ud = torch.from_numpy(Xd).cuda(), torch.from_numpy(Ud).cuda()
        wsd = torch.empty(api.ecc_workspace_bytes_dir(Xd.shape[1:], 1, 16, BINS), dtype=torch.uint8, device="cuda")
        cvd = torch.empty((16, 1, BINS), dtype=torch.int64, device="cuda")
        fnd = lambda: api.ecc_hard_dir(gd, 2, ud, 1e-4, BINS, curve=cvd, workspace=wsd)
        for _ in range(args.warmup):
            fnd()
        torch.cuda.synchronize()
        api.ecc_profile_begin(args.steps)
        msd = time_steps(fnd, args.steps, 0)
        swd, _ = api.ecc_profile_end()
        extra["directional"] = {"workload": "16 directions x one 2D 4096^2 float32 GRF (alpha = 1e-4 per pixel), 1024 "
                                            "bins over the range of all tilted fields, found on the device",
                                "ms_per_step": round(msd, 4), "sweep_kernel_ms": round(swd, 4),
                                "gvoxel_per_s": round(16 * Xd.size / msd / 1e6, 1),
                                "note": "the field (64 MiB) is read once per direction; re-reads are served by "
                                        "the L2 / Infinity Cache, so vertices/s may pass the HBM roofline of a "
                                        "single read"}
        log(f"[bench] directional: {msd:.3f} ms/step (16 x 4096^2), sweep kernel {swd:.3f} ms")
        del gd, Xd
        torch.cuda.empty_cache()
        if args.only == "dir":
            return

    # ---------------- C5: soft forward + backward -------------------------------
    if args.only in ("", "c5") and (not args.quick or args.only == "c5"):
        X5 = synth.config_c5()
        p = synth.soft_params_c5(X5)
        T = len(p["tau"])
        g5 = torch.from_numpy(X5).cuda()
        u5, tau5 = torch.from_numpy(p["u"]).cuda(), torch.from_numpy(p["tau"]).cuda()
        G5 = torch.from_numpy(synth.upstream_grad(X5.shape[0], T)).cuda()
        ws5 = torch.empty(api.ecc_workspace_bytes(X5.shape[1:], X5.shape[0], T), dtype=torch.uint8, device="cuda")
        chi = torch.empty((X5.shape[0], T), dtype=torch.float32, device="cuda")
        gx = torch.empty_like(g5)
        dt_ = torch.empty_like(chi)
        du_ = torch.empty((X5.shape[0], T, 2), dtype=torch.float32, device="cuda")

        def step5():
            api.ecc_soft_fwd(g5, 2, u5, p["alpha"], tau5, p["lam"], chi=chi, workspace=ws5)
            api.ecc_soft_bwd(g5, 2, u5, p["alpha"], tau5, p["lam"], grad_chi=G5, grad_X=gx, dchi_dtau=dt_,
                             dchi_du=du_, workspace=ws5)
        st5 = torch.empty(api.ecc_soft_state_bytes(X5.shape[1:], X5.shape[0]), dtype=torch.uint8, device="cuda")

        def step5s():
            api.ecc_soft_fwd_save(g5, 2, u5, p["alpha"], tau5, p["lam"], chi=chi, dchi_dtau=dt_, dchi_du=du_, state=st5,
                                  workspace=ws5)
            api.ecc_soft_bwd_saved(g5, 2, u5, p["alpha"], tau5, p["lam"], st5, grad_chi=G5, grad_X=gx, workspace=ws5)
        ms5s = time_steps(step5s, args.steps, args.warmup)
        ms5sf = time_steps(lambda: api.ecc_soft_fwd_save(g5, 2, u5, p["alpha"], tau5, p["lam"], chi=chi, dchi_dtau=dt_,
                                                         dchi_du=du_, state=st5, workspace=ws5), args.steps, args.warmup)
        log(f"[bench] C5 soft saved-state: fwd_save+bwd_saved {ms5s:.4f} ms, fwd_save {ms5sf:.4f} ms")
        ms5 = time_steps(step5, args.steps, args.warmup)
        ms5f = time_steps(lambda: api.ecc_soft_fwd(g5, 2, u5, p["alpha"], tau5, p["lam"], chi=chi, workspace=ws5),
                          args.steps, args.warmup)
        K = int((api.ecc_coeff(g5, 2) != 0).sum().item())
        extra["c5_soft"] = {"workload": "C5: soft fwd+bwd, 32 x 512^2 float32, T=128, lambda=20, alpha=0.01",
                            "ms_fwd_plus_bwd": round(ms5, 4), "ms_fwd": round(ms5f, 4),
                            "critical_vertices": K, "pairs_evaluated": K * T * 3,
                            "dense_pairs": int(X5.size) * T}
        log(f"[bench] C5 soft: fwd+bwd {ms5:.3f} ms, fwd {ms5f:.3f} ms, K={K}")
        if args.only == "c5":
            return
        if not args.quick:
            from oracle import ecc_oracle as O
            t0 = time.perf_counter()
            O.soft_fwd_batch(X5[:2], p["u"], p["alpha"], p["tau"], p["lam"])
            O.soft_bwd_batch(X5[:2], p["u"], p["alpha"], p["tau"], p["lam"], G5[:2].cpu().numpy())
            dt = time.perf_counter() - t0
            extra["c5_soft"]["cpu_oracle_ms_full_batch_extrapolated"] = round(dt / 2 * X5.shape[0] * 1e3, 1)
            extra["c5_soft"]["cpu_oracle_sample"] = "2 of 32 items, numpy float64"

    # ---------------- soft forward + backward on a volume (fused 3D path) ---------
    if args.only == "" and not args.quick:
        V = synth.grf((256, 256, 256), 3.0, 5151)[None]
        T3 = 64
        gv = torch.from_numpy(V).cuda()
        uv = torch.tensor([0.48, -0.6, 0.64], dtype=torch.float32, device="cuda")
        tv = torch.linspace(float(V.min()), float(V.max()), T3, device="cuda")
        Gv = torch.from_numpy(synth.upstream_grad(1, T3)).cuda()
        wsv = torch.empty(api.ecc_workspace_bytes(V.shape[1:], 1, T3), dtype=torch.uint8, device="cuda")
        gxv = torch.empty_like(gv)

        def stepv():
            api.ecc_soft_fwd(gv, 3, uv, 0.01, tv, 20.0, workspace=wsv)
            api.ecc_soft_bwd(gv, 3, uv, 0.01, tv, 20.0, grad_chi=Gv, grad_X=gxv, workspace=wsv)
        msv = time_steps(stepv, args.steps, args.warmup)
        extra["soft_3d"] = {"workload": "soft fwd+bwd, one 256^3 float32 GRF sigma=3, T=64, lambda=20, alpha=0.01",
                            "ms_fwd_plus_bwd": round(msv, 4)}
        log(f"[bench] soft 3D 256^3: fwd+bwd {msv:.3f} ms")
        del gv, gxv, wsv

    line = {
        "metric": "hard_ecc_throughput", "value": round(value, 2), "unit": "Gvoxel/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "C2: hard ECC, batch 16 of 2D 4096x4096 float32 smoothed Gaussian random fields "
                               "(sigma=4 px), 1024 equal-width bins over the batch-global [min,max] found on the "
                               "device (single read pass: the sweep tracks the range and lists the critical "
                               "vertices, which are binned afterwards)", "bins": BINS, "batch": 16},
        "roofline": roofline,
    }
    if not args.quick:
        line["cpu_baseline"] = cpu
    line["extra"] = extra
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
