#!/usr/bin/env python3
"""Benchmark of the CORE hot path on one MI355X.

A step is one `core_round` (projection of n client gradients onto m common Gaussian vectors,
cross-chunk sum + client mean, reconstruction) over one batch of synthetic gradients that is
already resident in HBM.  The default workload is the ResNet-50-sized configuration
(d = 25,557,032, m = 1024, n = 8, bf16 storage, fp32 arithmetic).

Prints ONE JSON line with the whole-job throughput (projected coordinates per second,
d*m*n / t), a roofline object for the dominant kernel, the CPU oracle timed on a bounded sample
of the same workload (one thread, and the same code over all host cores), and, under
`other_workloads`, the round time of the four other configurations.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2309_13307_amd as core  # noqa: E402
from paper_2309_13307_amd import build as hip_build, workloads  # noqa: E402

# Peak of the plain vector ALU: 256 CUs x 4 SIMDs x 32 fp32 lanes per clock x 2.4 GHz.  It is the
# published 157.3 TFLOP/s fp32 vector figure divided by the 2 flops of an FMA; measured on this
# chip, a wave64 two-operand VALU instruction issues in ~2 cycles, i.e. 32 lanes per clock.
PEAK_LANE_OPS = 256 * 4 * 32 * 2.4e9
PEAK_FLOPS = 157.3e12

# Algorithmic lane-operations per (coordinate, vector) pair: one Philox4x32-10 call is 20 wide
# multiplies + 20 key/xor steps for 4 outputs -> 20 per output counting half-products and xors;
# uniform map + Box-Muller ~6 per output; then n projection FMAs, or 1 reconstruction FMA.
OPS_GENERATE = 26

# Hardware counters cannot be read from inside this process.  The figures below were read with
# rocprofv3 --pmc for the two large workloads (per launch of each kernel; FETCH_SIZE x 2.000 and
# WRITE_SIZE x 1.000 KiB after calibration with a 1 GiB copy) and are static properties of the
# compiled kernels at those shapes: they are reported only while the kernel sources still hash to
# `kernel_id`, and as null otherwise.
COUNTERS = {
    "kernel_id": "4c4a63965e3b77c1",
    "config4": {
        "source": "profiles/core_round_config4.md", "date": "2026-11-27",
        "project": {"SQ_INSTS_VALU": 9.13251e9, "fetch_bytes": 200631 * 2 * 1024, "write_bytes": 65216 * 1024},
        "reconstruct": {"SQ_INSTS_VALU": 6.10726e9, "fetch_bytes": 41 * 2 * 1024, "write_bytes": 99832.2 * 1024},
    },
    "config5": {
        "source": "profiles/core_round_config5.md", "date": "2026-11-27",
        "project": {"SQ_INSTS_VALU": 1.48462e11, "fetch_bytes": 1.94443e6 * 2 * 1024, "write_bytes": 131072 * 1024},
        "reconstruct": {"SQ_INSTS_VALU": 1.18894e11, "fetch_bytes": 90 * 2 * 1024, "write_bytes": 486093 * 1024},
    },
}


def kernel_id() -> str:
    """Hash of the sources of the kernels the counters were read for: the projection for whole tiles of
    256 vectors, the reconstruction and the generator (the host side and the other kernel families do
    not change their instruction counts)."""
    h = hashlib.sha256()
    for name in ("core_common.hpp", "core_rng.hpp", "core_project.hpp", "core_reconstruct.hpp"):
        with open(os.path.join(hip_build.CSRC, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config4", choices=["config1", "config2", "config3", "config4", "config5"],
                    help="config4 is the headline; config1/config2 are single rounds of those small shapes "
                         "(launch-bound), config2's full CORE-GD run lives in the tests")
    ap.add_argument("--variant", default="regenerate", choices=["regenerate", "materialized"],
                    help="materialized = the comparison variant that stores Xi while projecting and "
                         "reads it back to reconstruct (needs 4*d*m bytes of HBM)")
    ap.add_argument("--clients", type=int, default=None,
                    help="override the number of clients n of config4 / config5 (same recipe, more or fewer "
                         "rows of G); the workload name in the output says so")
    ap.add_argument("--vectors", type=int, default=None,
                    help="override the number of common vectors m of config4 / config5; the workload name "
                         "in the output says so")
    ap.add_argument("--graph", action="store_true",
                    help="time the K rounds as one replay of a HIP graph that holds them (distinct round "
                         "counters by value): removes the host's launch cost, which is what the two "
                         "launch-bound workloads (config1, config2) otherwise measure")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the four other configurations")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device-to-device copy (3x) and exit; used to scale "
                         "the FETCH_SIZE / WRITE_SIZE counters of a profiler run")
    return ap.parse_args()


def _host_cores() -> int:
    """Cores this process may use: the affinity mask, capped by the thread budget the environment
    states (OMP_NUM_THREADS is the per-GPU CPU share on shared boxes)."""
    cores = len(os.sched_getaffinity(0))
    try:
        cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    except ValueError:
        pass
    return max(1, cores)


def cpu_baseline(case, d_s=1 << 20, m_s=256):
    """The oracle as it stands on the first d_s coordinates x m_s vectors x all clients of the same G:
    one thread (one call of its round routine), then the same routines over all host cores."""
    import oracle
    d_s = min(d_s, case.d)
    m_s = min(m_s, case.m)
    G_host = np.ascontiguousarray(workloads.to_host(case.G[:, :d_s]))
    oracle.lib()
    t0 = time.perf_counter()
    _, pbar_ref, gt_ref = oracle.core_round(case.seed, 0, G_host, m_s)
    dt = time.perf_counter() - t0

    # all cores: the compression split by vector range and the reconstruction by coordinate range,
    # one range per thread (the C routines run without the interpreter lock; no oracle code changes)
    cores = _host_cores()
    jr = [np.arange(a, b, dtype=np.uint32) for a, b in
          zip(np.linspace(0, m_s, cores + 1).astype(int)[:-1], np.linspace(0, m_s, cores + 1).astype(int)[1:]) if b > a]
    nblk = (d_s + 3) // 4
    cuts = (np.linspace(0, nblk, cores + 1).astype(int) * 4).clip(max=d_s)
    ir = [(int(a), int(b - a)) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as pool:
        cols = list(pool.map(lambda jj: oracle.compress(case.seed, 0, G_host, jidx=jj), jr))
        pbar_all = oracle.client_mean(np.concatenate(cols, axis=1))
        parts = list(pool.map(lambda r: oracle.reconstruct(case.seed, 0, pbar_all, 1.0 / m_s, r[0], r[1]), ir))
    dt_all = time.perf_counter() - t0
    gt_all = np.concatenate(parts)
    same = bool(np.array_equal(pbar_all, pbar_ref) and np.array_equal(gt_all, gt_ref))

    # the same slice through the HIP path: the oracle's result is at hand, so report the parity too
    G_s = case.G[:, :d_s].contiguous()
    pbar, gtilde = core.core_round(case.seed, 0, G_s, m_s)
    torch.cuda.synchronize()
    if G_host.dtype == np.uint16:
        G_f = (G_host.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    else:
        G_f = G_host.astype(np.float64)
    norm = float(np.sqrt((G_f ** 2).sum(axis=1)).mean())
    parity = {
        "pbar_max_abs_err_over_norm_g": float(np.abs(pbar.cpu().numpy() - pbar_ref).max() / norm),
        "gtilde_rel_l2": float(np.linalg.norm(gtilde.cpu().numpy() - gt_ref) / np.linalg.norm(gt_ref)),
    }
    units = d_s * m_s * case.n
    return {
        "parity_on_sample": parity,
        "value": units / dt,
        "unit": "coords/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"one full oracle round on the first {d_s} coordinates x first {m_s} vectors x all "
                  f"{case.n} clients of the same G ({dt:.1f} s on one thread; the BASELINE plan's slice had 64 "
                  f"vectors, 256 are used so that the all-cores leg gives every core several vectors)",
        "all_cores": {
            "value": units / dt_all,
            "unit": "coords/s",
            "cores": cores,
            "seconds": dt_all,
            "how": "same oracle routines, compression split by vector range and reconstruction by coordinate "
                   "range over one thread per core of the affinity mask",
            "bit_identical_to_one_thread": same,
        },
    }


def time_rounds(case, steps, warmup, graph=False, mat=False, first_round=0):
    """Whole-round time (K rounds back to back, host clock around a synchronised region) and the
    durations of the two halves (HIP events on the launch stream) for one workload."""
    dev = case.G.device
    d, m, n, G = case.d, case.m, case.n, case.G
    ws = core.alloc_workspace(d, m, n, dev)
    pbar = torch.empty(m, dtype=torch.float32, device=dev)
    gtilde = torch.empty(d, dtype=torch.float32, device=dev)
    xi = core.alloc_xi(d, m, dev) if mat else None
    torch.cuda.synchronize()

    def one_round(r):
        if mat:
            core.core_round_materialized(case.seed, r, G, m, xi, pbar=pbar, gtilde=gtilde, ws=ws)
        else:
            core.core_round(case.seed, r, G, m, pbar=pbar, gtilde=gtilde, ws=ws)

    rnd = first_round
    for _ in range(warmup):
        one_round(rnd)
        rnd += 1
    torch.cuda.synchronize()

    if graph:
        # the K rounds recorded once, replayed once untimed, then replayed once inside the timed region
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for k in range(steps):
                one_round(rnd + k)
        rnd += steps
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        # timed region: exactly K rounds with distinct round counters, nothing else on the stream
        t0 = time.perf_counter()
        for k in range(steps):
            one_round(rnd)
            rnd += 1
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0

    # per-kernel durations with events on the launch stream (the binding launches on torch's
    # current stream).  core_round is exactly these two calls back to back.
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    for k in range(steps):
        ev[k][0].record()
        if mat:
            _, pb = core.core_compress_batched_store_xi(case.seed, rnd, G, m, xi, ws=ws, want_P=False)
            ev[k][1].record()
            core.core_reconstruct_from_xi(d, pb, 1.0 / m, xi, gtilde=gtilde)
        else:
            core.core_compress_batched(case.seed, rnd, G, m, pbar=pbar, ws=ws, want_P=False)
            ev[k][1].record()
            core.core_reconstruct(case.seed, rnd, d, pbar, 1.0 / m, gtilde=gtilde)
        ev[k][2].record()
        rnd += 1
    torch.cuda.synchronize()
    per_round = sorted(e[0].elapsed_time(e[2]) for e in ev)
    t_proj = float(np.mean([e[0].elapsed_time(e[1]) for e in ev])) * 1e-3
    t_recon = float(np.mean([e[1].elapsed_time(e[2]) for e in ev])) * 1e-3
    pairs = float(d) * m
    s_per_step = elapsed / steps
    return {
        "s_per_step": s_per_step, "per_round_ms": per_round, "t_proj": t_proj, "t_recon": t_recon,
        "pairs": pairs, "ops_proj": pairs * (OPS_GENERATE + n), "ops_recon": pairs * (OPS_GENERATE + 1),
        "next_round": rnd,
    }


def other_workload(name, make, dev, steps, warmup, with_graph):
    """Round time and whole-round fraction of the lane-op peak for one of the other configurations."""
    case = make(dev)
    r = time_rounds(case, steps, warmup)
    ops = r["ops_proj"] + r["ops_recon"]
    out = {
        "d": case.d, "m": case.m, "n": case.n, "steps": steps, "warmup": warmup,
        "ms_per_round": r["s_per_step"] * 1e3,
        "coords_per_s": case.d * case.m * case.n / r["s_per_step"],
        "whole_round_frac": ops / r["s_per_step"] / PEAK_LANE_OPS,
        "compress_ms": r["t_proj"] * 1e3, "reconstruct_ms": r["t_recon"] * 1e3,
    }
    if with_graph:
        g = time_rounds(case, steps, warmup, graph=True, first_round=r["next_round"])
        out["ms_per_round_graph_replay"] = g["s_per_step"] * 1e3
        out["whole_round_frac_graph_replay"] = ops / g["s_per_step"] / PEAK_LANE_OPS
    del case
    torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1.", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": dst.numel() * 4,
                          "launches": 3}))
        return 0
    core.load_library()

    makers = {"config1": workloads.config1, "config2": workloads.config2_round, "config3": workloads.config3,
              "config4": workloads.config4, "config5": workloads.config5}
    make = makers[args.workload]
    if args.clients is not None:
        if args.workload not in ("config4", "config5") or args.clients < 1:
            print("bench.py: --clients applies to config4 and config5 and must be >= 1", file=sys.stderr)
            return 2
        case = make(dev, n=args.clients)
        case.name += f" with n overridden to {args.clients}"
    else:
        case = make(dev)
    if args.vectors is not None:
        if args.workload not in ("config4", "config5") or args.vectors < 1:
            print("bench.py: --vectors applies to config4 and config5 and must be >= 1", file=sys.stderr)
            return 2
        case.m = args.vectors
        case.name += f" with m overridden to {args.vectors}"
    d, m, n = case.d, case.m, case.n
    mat = args.variant == "materialized"

    r = time_rounds(case, args.steps, args.warmup, graph=args.graph, mat=mat)
    s_per_step, t_proj, t_recon = r["s_per_step"], r["t_proj"], r["t_recon"]
    ms_per_step = s_per_step * 1e3
    per_round = r["per_round_ms"]
    pairs, ops_proj, ops_recon = r["pairs"], r["ops_proj"], r["ops_recon"]
    value = float(d) * m * n / s_per_step
    ach_proj = ops_proj / t_proj
    ach_recon = ops_recon / t_recon
    ach_round = (ops_proj + ops_recon) / s_per_step
    esize = 2 if case.G.dtype == torch.bfloat16 else 4
    algo_bytes = float(n) * d * esize + 4.0 * d

    # counter-derived figures, only for the workloads they were collected on and only while the
    # kernels are the ones they were collected from
    ctr = COUNTERS.get(args.workload) if (not mat and args.clients is None and args.vectors is None
                                          and not args.graph) else None
    if ctr is not None and COUNTERS["kernel_id"] != kernel_id():
        ctr = None

    def issue_frac(which, t):
        return ctr[which]["SQ_INSTS_VALU"] * 64.0 / t / PEAK_LANE_OPS if ctr else None

    def traffic(which):
        return ctr[which]["fetch_bytes"] + ctr[which]["write_bytes"] if ctr else None

    out = {
        "metric": "projected coords/sec (d*m*n/s) for compress+reconstruct",
        "value": value,
        "unit": "coords/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{case.name}: one core_round, d={d}, m={m}, n={n}, G stored "
                        f"{'bf16' if esize == 2 else 'fp32'}, fp32 arithmetic, inputs resident in HBM",
            "d": d, "m": m, "n": n, "variant": args.variant,
            "launch": "one replay of a HIP graph holding the K rounds" if args.graph else "K eager calls",
        },
        # spread of single rounds, from events around each round in a separate pass
        "ms_per_round_median": per_round[len(per_round) // 2],
        "ms_per_round_min": per_round[0],
        "pct_fp32_valu_peak": 100.0 * ach_round / PEAK_LANE_OPS,
        # for context: the same work counted in flops (an FMA as 2, every other lane-op as 1)
        # against the published 157.3 TFLOP/s, which only packed-fp32 FMAs can reach
        "flop_equivalent_TFLOPs": pairs * (52 + 2 * (n + 1)) / s_per_step / 1e12,
        "roofline": {
            "bound": "alu",
            "kernel": ("project_kernel" if n <= 8 or mat else "project_mfma_kernel")
                      + " (core_compress_batched: projection + cross-chunk sum)",
            "achieved": ach_proj / 1e12,
            "peak": PEAK_LANE_OPS / 1e12,
            "unit": "Tlaneop/s",
            # three readings of the same launch time.  frac: algorithmic lane-operations (26 per
            # generated normal + n FMAs; a 64-bit multiply-add and a three-input xor each do the work
            # of two).  issue_frac: vector instructions the kernel actually issues x 64 lanes.
            # flop_equiv_frac: an FMA as 2 flops, everything else as 1, against 157.3 TFLOP/s.
            "frac": ach_proj / PEAK_LANE_OPS,
            "issue_frac": issue_frac("project", t_proj),
            "flop_equiv_frac": pairs * (OPS_GENERATE + 2 * n) / t_proj / PEAK_FLOPS,
            "traffic": traffic("project"),
            "traffic_source": (f"{ctr['source']} ({ctr['date']}): rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE per launch, "
                               "scaled by the same counters on a 1 GiB copy; a constant of the compiled kernel at "
                               "this shape, not read during this run") if ctr else None,
            "ms": t_proj * 1e3,
            "lane_ops_per_pair": OPS_GENERATE + n,
            "second_kernel": {
                "kernel": "reconstruct_kernel (core_reconstruct)",
                "achieved": ach_recon / 1e12,
                "frac": ach_recon / PEAK_LANE_OPS,
                "issue_frac": issue_frac("reconstruct", t_recon),
                "flop_equiv_frac": pairs * (OPS_GENERATE + 2) / t_recon / PEAK_FLOPS,
                "traffic": traffic("reconstruct"),
                "ms": t_recon * 1e3,
                "lane_ops_per_pair": OPS_GENERATE + 1,
            },
            "whole_round_frac": ach_round / PEAK_LANE_OPS,
            "whole_round_flop_equiv_frac": pairs * (52 + 2 * (n + 1)) / s_per_step / PEAK_FLOPS,
            "hbm_algorithmic_bytes": algo_bytes,
            "hbm_achieved_GBps": algo_bytes / s_per_step / 1e9,
            "hbm_peak_GBps": 8000.0,
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(case)
    if (not args.no_other_workloads and args.workload == "config4" and not mat and args.clients is None
            and args.vectors is None):
        del case
        torch.cuda.empty_cache()
        others = {}
        # warm-up long enough for the clocks to settle: at config 3 three rounds are 1 ms of work, and the
        # first 30 rounds after them run 10 % slower than the 200 that follow
        for name, steps, warmup, with_graph in (("config1", 200, 50, True), ("config2", 200, 50, True),
                                                ("config3", 200, 50, True), ("config5", 3, 1, False)):
            others[name] = other_workload(name, makers[name], dev, steps, warmup, with_graph)
        out["other_workloads"] = others
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
