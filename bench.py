#!/usr/bin/env python3
"""Benchmark of the projector pair on one MI355X.

One "step" is one pass of the whole hot path over one synthetic input: y = A x followed by x' = A^T y on
the 512^3 circular cone-beam workload (720 views, 512x512 detector), inputs resident in HBM.  Prints ONE
JSON line.  value = voxel-view updates per second over the step (both operators: 2 * nviews*nx*ny*nz per
step); the literal ray-voxel (nonzero-weight) rate is value * nnz_per_update.
"""
from __future__ import annotations

import argparse
import json
import re
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

PEAK_FP32_TFLOPS = 157.3      # MI355X published vector fp32 (packed); 78.6 without packed instructions
PEAK_HBM_GBPS = 8000.0

# Traffic beyond L2 per operator call, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this very command (summaries
# under profiles/), scaled by a 512 MiB device copy in the same run (FETCH_SIZE x 2 KiB, WRITE_SIZE x 1 KiB).  These are
# NOT measured in this run and they are NOT HBM bytes alone: FETCH_SIZE counts what leaves L2, part of which the 256 MB
# memory-side cache serves.  Each entry names the kernel instance it was measured on; when leap_geometry_describe no
# longer shows that instance the entry is ignored and the fields print null.
MEASURED_TRAFFIC = {
    ("c3_cone_512", "A"): {"instance": "A=columns(nq=12/16,nkp=5,rg=4,cw=4,slab=60)", "launches": 18,
                           "fetch_bytes": 3.74159e7 * 2048, "write_bytes": 9.93274e6 * 1024,
                           "source": "profiles/sf_project_columns_c3_cone_512.md"},
    ("c3_cone_512", "AT"): {"instance": "AT=tiled(nc=3,nv=2,zc=64,window=24x63)", "launches": 1,
                            "fetch_bytes": 6.36848e6 * 2048, "write_bytes": 524288 * 1024,
                            "source": "profiles/sf_backproject_tiled_c3_cone_512.md"},
    ("c2_parallel3d_256", "A"): {"instance": "A=columns(nq=8/8,nkp=3,rg=2,cw=4,slab=256)", "launches": 2,
                                 "fetch_bytes": 1.72456e6 * 2048, "write_bytes": 72767 * 1024,
                                 "source": "profiles/sf_pair_c2_parallel_256.md"},
    ("c2_parallel3d_256", "AT"): {"instance": "AT=tiled(nc=3,nv=2,zc=64,window=25x67)", "launches": 1,
                                  "fetch_bytes": 178849 * 2048, "write_bytes": 65536 * 1024,
                                  "source": "profiles/sf_pair_c2_parallel_256.md"},
    ("c4_cone_limited_batch8_256", "A"): {"instance": "A=columns(nq=8/8,nkp=3,rg=3,cw=4,slab=256)", "launches": 10,
                                          "fetch_bytes": 4.58747e6 * 2048, "write_bytes": 1.85073e6 * 1024,
                                          "source": "profiles/sf_pair_c4_training_batch.md"},
    ("c4_cone_limited_batch8_256", "AT"): {"instance": "AT=tiled(nc=4,nv=3,zc=16,window=49x46)", "launches": 1,
                                           "fetch_bytes": 1.65103e6 * 2048, "write_bytes": 524288 * 1024,
                                           "source": "profiles/sf_pair_c4_training_batch.md"},
    ("c5_cone_1024", "A"): {"instance": "A=columns(nq=11/16,nkp=4,rg=4,cw=4,slab=124)", "launches": 18,
                            "fetch_bytes": 9.98654e8 * 2048, "write_bytes": 9.88812e7 * 1024,
                            "source": "profiles/sf_pair_c5_cone_1024.md"},
    ("c5_cone_1024", "AT"): {"instance": "AT=tiled(nc=3,nv=3,zc=64,window=31x86)", "launches": 1,
                             "fetch_bytes": 7.15103e8 * 2048, "write_bytes": 4.1943e6 * 1024,
                             "source": "profiles/sf_pair_c5_cone_1024.md"},
    ("c3_cone_512:siddon", "A"): {"instance": "A=columns(rg=8,slab=124)", "launches": 10,
                                  "fetch_bytes": 8.21501e7 * 2048, "write_bytes": 9.42225e6 * 1024,
                                  "source": "profiles/sd_project_columns_c3_cone_512.md"},
    ("c3_cone_512:siddon", "AT"): {"instance": "AT=tiled(nc=2,zc=32,window=21x32)", "launches": 1,
                                   "fetch_bytes": 2.19946e7 * 2048, "write_bytes": 524288 * 1024,
                                   "source": "profiles/sd_backproject_tiled_c3_cone_512.md"},
}


def algorithmic_flops_per_update(n_u: float, n_v: float, nz: int) -> float:
    """Cheapest known evaluation of the separable weights, per voxel-view pair: 40 flops per (view, voxel
    column) for knots and magnification, 15 per transaxial weight, 5 per axial weight, 3 per nonzero
    (ray, voxel) pair (two multiplies to combine, one add to accumulate)."""
    return 40.0 / nz + 15.0 * n_u / nz + 5.0 * n_v + 3.0 * n_u * n_v


def siddon_flops_per_update(cfg) -> tuple:
    """Cheapest known evaluation of the Siddon weights, per voxel-view pair.  Per (ray, slab): 10 flops for the two
    positions at the slab's exit face, the in-plane and the axial crossing parameter; per nonzero (ray, voxel) pair 3
    (difference of two parameters, multiply, accumulate).  A ray meets 1 + |m| + |m_z| voxels per slab (|m| averages
    2 ln(2)/pi... taken as 0.44 over a full turn, |m_z| as a quarter of the cone's half angle slope), and there are
    nrows*ncols rays per view against ny*nz voxel columns per slab.  Returns (flops per update, nonzeros per update)."""
    rays_per_column = (cfg.nrows * cfg.ncols) / float(cfg.ny * cfg.nz)
    mz = 0.0 if cfg.geom not in (2, 4) else 0.25 * (0.5 * cfg.nrows * cfg.pixel_v / cfg.sdd) * cfg.voxel_xy / cfg.voxel_z
    per_slab = 1.0 + 0.44 + mz
    return rays_per_column * (10.0 + 3.0 * per_slab), rays_per_column * per_slab


def footprint_counts(cfg) -> tuple:
    """Mean pixels per voxel in u and v from the scanner's magnification (volume average at the axis)."""
    if cfg.geom == 0:
        mag = 1.0
    else:
        mag = cfg.sdd / cfg.sod
    # mean transaxial footprint width over view angles: T * mag * mean(|cos|+|sin|) = T mag 4/pi
    n_u = 1.0 + cfg.voxel_xy * mag * (4.0 / np.pi) / cfg.pixel_u
    n_v = 1.0 if cfg.geom == 1 else 1.0 + cfg.voxel_z * mag / cfg.pixel_v
    return n_u, n_v


def cpu_baseline(cfg, x, seconds_target: float, model: str = "sf"):
    """Times the CPU oracle, as it stands, on a bounded sample of the same workload."""
    import oracle
    if model == "siddon":
        oracle = oracle.siddon
        oracle.build()
    threads = oracle.num_threads()
    nview_sample = max(threads, 8)
    views = [int(v) for v in np.linspace(0, cfg.nviews, nview_sample, endpoint=False)]
    sub = cfg.with_views(views)
    t0 = time.perf_counter()
    ax = oracle.project(sub, x)
    t_a = time.perf_counter() - t0
    rate_a = sub.voxel_views / t_a
    # A^T: sample voxels over all views; size the sample from a probe
    rng = np.random.default_rng(7)
    nvox = cfg.nx * cfg.ny * cfg.nz
    y = rng.random(cfg.sino_shape, dtype=np.float32)
    probe = rng.integers(0, nvox, 2000)
    t0 = time.perf_counter()
    oracle.backproject_voxels(cfg, y, probe)
    t_probe = time.perf_counter() - t0
    n = int(min(nvox, max(2000, 2000 * (0.5 * seconds_target) / max(t_probe, 1e-3))))
    vox = rng.integers(0, nvox, n)
    t0 = time.perf_counter()
    oracle.backproject_voxels(cfg, y, vox)
    t_at = time.perf_counter() - t0
    rate_at = n * cfg.nviews / t_at
    step_rate = 2.0 / (1.0 / rate_a + 1.0 / rate_at)          # updates/s of a whole A + A^T step
    return {
        "value": step_rate, "unit": "voxel-view updates/s", "cores": threads, "kind": "oracle",
        "sample": f"A on {len(views)} of {cfg.nviews} views ({t_a:.1f} s), A^T on {n} random voxels over all views "
                  f"({t_at:.1f} s); rates combined as for one A + A^T step",
        "A_updates_per_s": rate_a, "AT_updates_per_s": rate_at,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="benchmark case number (3 = the headline 512^3 cone-beam)")
    ap.add_argument("--model", choices=["sf", "siddon"], default="sf",
                    help="projector model: sf = separable footprint (the headline), siddon = thin rays")
    ap.add_argument("--detector", choices=["flat", "curved"], default="flat",
                    help="cone-beam cases only: flat panel (the headline) or cylindrical detector of the same pixel pitch")
    ap.add_argument("--tilted-modules", type=float, default=0.0, metavar="RAD",
                    help="cone-beam cases only: the same scan as a modular geometry whose every source and detector is moved "
                         "by up to 5 mm and whose every module is turned by up to RAD about each of its axes (seeded)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="CPU time budget of the oracle baseline; 0 skips it")
    ap.add_argument("--no-transfer-leg", action="store_true",
                    help="skip the extra leg that times the host-memory entry points (upload + run + download)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed region, run one device-to-device copy of the volume (a plain copy kernel of "
                         "known size) so that a rocprofv3 --pmc run of this command can scale FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from synthetic import config, standard_volume
    from paper_2307_05801_amd import Geometry

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    cfg = config(args.config)
    if args.detector == "curved":
        if cfg.geom != 2:
            print("bench.py: --detector curved needs a cone-beam case", file=sys.stderr)
            return 2
        cfg = cfg.replace(geom=3, name=cfg.name + "_curved")
    if args.tilted_modules > 0.0:
        if cfg.geom != 2:
            print("bench.py: --tilted-modules needs a flat-panel cone-beam case", file=sys.stderr)
            return 2
        from synthetic import perturbed_poses
        cfg = perturbed_poses(cfg, 3, shift_mm=5.0, tilt_rad=args.tilted_modules)
    batch = cfg.batch
    x_np = np.stack([standard_volume(args.config, cfg, item=b) for b in range(batch)])
    torch.cuda.synchronize()
    t_create = time.perf_counter()
    geo = Geometry(cfg, device="cuda:0", model=args.model)       # blocking: validation, tables, scratch
    create_ms = 1e3 * (time.perf_counter() - t_create)
    y = torch.empty((batch,) + cfg.sino_shape, dtype=torch.float32, device="cuda")
    y_meas = None
    if args.config == 4:
        # training step: current estimate x, photon-noise measurement of A x_true (input preparation, untimed)
        from synthetic import measured_sinogram, perturbed_volume
        geo.project(torch.from_numpy(x_np).cuda(), out=y)
        ideal = y.cpu().numpy()
        y_meas = torch.from_numpy(np.stack([measured_sinogram(ideal[b], 1004 + b) for b in range(batch)])).cuda()
        x_np = np.stack([perturbed_volume(x_np[b], 1004 + b) for b in range(batch)])
    x = torch.from_numpy(x_np).cuda()
    xb = torch.empty_like(x)

    def step(ev=None):
        if ev:
            ev[0].record()
        geo.project(x, out=y)
        if ev:
            ev[1].record()
        if y_meas is not None:
            y.sub_(y_meas)                       # residual r = A x - y_meas; the gradient is A^T r
        geo.backproject(y, out=xb)
        if ev:
            ev[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_a = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    ms_at = float(np.mean([e[1].elapsed_time(e[2]) for e in events]))
    ms_step = 1e3 * wall / args.steps
    updates = 2.0 * batch * cfg.voxel_views
    value = updates / (ms_step * 1e-3)

    if args.model == "siddon":
        fl, nnz_per_update = siddon_flops_per_update(cfg)
    else:
        n_u, n_v = footprint_counts(cfg)
        fl = algorithmic_flops_per_update(n_u, n_v, cfg.nz)
        nnz_per_update = n_u * n_v
    describe = geo.describe()
    found = re.search(r"scratch=(\d+)", describe)
    scratch_bytes = int(found.group(1)) if found else None      # device memory the handle owns beyond its tables
    flops_call = fl * batch * cfg.voxel_views
    alg_bytes = 4.0 * batch * (cfg.nx * cfg.ny * cfg.nz + cfg.nviews * cfg.nrows * cfg.ncols)
    workload = cfg.name if args.model == "sf" else cfg.name + ":" + args.model

    def operator_report(op, ms):
        """Roofline figures of one operator call (A or AT): the vector-ALU fraction that bounds it, and what is known of
        its traffic."""
        rec = MEASURED_TRAFFIC.get((workload, op))
        if rec is not None and rec["instance"] not in describe:
            rec = None
        tflops = flops_call / (ms * 1e-3) / 1e12
        out = {
            "ms": ms, "updates_per_s": batch * cfg.voxel_views / (ms * 1e-3),
            "alu_TFLOPs": tflops, "alu_frac_of_fp32_peak": tflops / PEAK_FP32_TFLOPS,
            "alu_frac_of_unpacked_fp32_peak": tflops / (PEAK_FP32_TFLOPS / 2),
            "algorithmic_bytes": alg_bytes, "algorithmic_GBps": alg_bytes / (ms * 1e-3) / 1e9,
            "beyond_l2_bytes": None, "beyond_l2_GBps": None, "restream_factor": None, "traffic_source": None,
        }
        if rec is not None:
            total = rec["fetch_bytes"] + rec["write_bytes"]
            out.update({"beyond_l2_bytes": total, "beyond_l2_GBps": total / (ms * 1e-3) / 1e9,
                        "restream_factor": total / alg_bytes, "traffic_source": rec["source"],
                        "kernel_launches": rec["launches"]})
        return out

    per_op = {"A": operator_report("A", ms_a), "AT": operator_report("AT", ms_at)}
    dom_op = "A" if ms_a >= ms_at else "AT"
    dom = per_op[dom_op]
    # the forward operator walks the volume slab by slab: one call is several launches of the same kernel (plus the slab
    # copies, about 1 % of the time); the roofline is stated per launch, as one launch's share of the call
    launches = dom.get("kernel_launches") or 1
    roofline = {
        "bound": "alu", "kernel": "leap_project (A)" if dom_op == "A" else "leap_backproject (A^T)",
        "achieved": dom["alu_TFLOPs"], "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s", "frac": dom["alu_frac_of_fp32_peak"],
        "traffic": None if dom["beyond_l2_bytes"] is None else dom["beyond_l2_bytes"] / launches,
        "traffic_note": "bytes leaving L2 per kernel launch (FETCH_SIZE + WRITE_SIZE of an earlier rocprofv3 run on this "
                        "kernel instance, not of this run); they include hits in the memory-side cache, so they bound HBM "
                        "traffic from above",
        "flops_per_update": fl, "launch_ms": dom["ms"] / launches, "launches_per_call": launches, "call_ms": dom["ms"],
        "frac_of_unpacked_fp32_peak": dom["alu_frac_of_unpacked_fp32_peak"],
        "hbm_target_note": "the path is bound by vector-ALU issue, not by HBM: its algorithmic traffic is %.2f GB per operator "
                           "call (%.0f GB/s, %.1f %% of the 8 TB/s peak); the metric's 50 %%-of-HBM-peak mark is reachable "
                           "only by re-streaming the input, which is waste" % (
                               alg_bytes / 1e9, dom["algorithmic_GBps"], 100 * dom["algorithmic_GBps"] / PEAK_HBM_GBPS),
    }
    out = {
        "metric": "ray-voxel updates/s for A and A^T (voxel-view pairs, both operators per step)"
                  + (" at 512^3 cone-beam" if args.config == 3 else f" on case {args.config}")
                  + ("" if args.model == "sf" else ", Siddon model"),
        "value": value, "unit": "voxel-view updates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload, "model": args.model, "nviews": cfg.nviews, "volume": list(cfg.vol_shape),
                   "detector": [cfg.nrows, cfg.ncols], "batch": batch, "kernels": describe},
        "A_ms": ms_a, "AT_ms": ms_at,
        "A_updates_per_s": per_op["A"]["updates_per_s"], "AT_updates_per_s": per_op["AT"]["updates_per_s"],
        "nnz_per_update": nnz_per_update,
        "geometry_create_ms": create_ms,
        "scratch_bytes": scratch_bytes,
        "roofline": roofline,
        "operators": per_op,
    }
    if not args.no_transfer_leg:
        # the same operators with their arrays in (pinned) host memory: upload, run, download, the three overlapped over
        # the items of a batch.  Reported beside the resident figures, never as `value`.
        hx = torch.from_numpy(x_np).pin_memory()
        hy = torch.empty((batch,) + cfg.sino_shape, dtype=torch.float32).pin_memory()
        hxb = torch.empty_like(hx).pin_memory()
        geo.project_host(hx, hy)                 # first call: the handle allocates its staging and device buffers
        geo.backproject_host(hy, hxb)
        t0 = time.perf_counter()
        geo.project_host(hx, hy)
        t1 = time.perf_counter()
        geo.backproject_host(hy, hxb)
        t2 = time.perf_counter()
        out["with_transfer"] = {
            "A_ms": 1e3 * (t1 - t0), "AT_ms": 1e3 * (t2 - t1), "host_memory": "pinned",
            "bytes_moved_per_operator": alg_bytes,
            "updates_per_s": updates / (t2 - t0),
            "note": "leap_project_host + leap_backproject_host, one call each: input uploaded, output downloaded, "
                    "PCIe-inclusive; not the headline value",
        }
        del hx, hy, hxb
    if args.calibration_copy:
        xb.copy_(x)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = int(x.numel() * 4)
    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, x_np[0], args.cpu_seconds, args.model)
    print(json.dumps(out))
    geo.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
