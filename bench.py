#!/usr/bin/env python3
"""Benchmark of the contraction hot path on ONE MI355X.

A "step" is one execution of the planned contraction over resident device buffers
(default workload: configuration 2, the fp64 particle-particle ladder
D[a,b,i,j] += sum_{c,d} V[a,b,c,d] T[c,d,i,j], v = 192, o = 64: 1.1133e13 flop).
Prints ONE JSON line: whole-job GFLOP/s, the dominant kernel's roofline figure measured
with HIP events inside the timed region, and the CPU oracle timed on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg1|cfg3|cfg4|cfg5]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3, "c128": 78.6}     # MI355X dense matrix peaks
PEAK_HBM_GBS = 8000.0
# L2 <-> fabric bytes per STEP from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same
# command, scaled by a streaming probe kernel (profiles/); keyed by (workload, path, variant) so a
# figure is only reported for the kernel it was taken on.  The JSON line reports it per launch.
MEASURED_TRAFFIC_BYTES = {
    ("cfg2_f64_ppladder_v192_o64", 1, 0): 110.21e9 + 1.34e9,               # 18 launches (rounds) per step
    ("cfg5_f64_network_e4_k5_f5_p7832", 1, 10): 52.2e6 + 8.39e6,
    ("cfg5_f64_network_e4_k1_f7_p7832", 2, 1): 31.2e6 + 2147.48e6,         # s1
    ("cfg5_f64_network_e4_k0_f7_p7832", 2, 1): 5.7e6 + 2147.48e6,          # s2
    ("hadamard_f64_4x128", 2, 0): None,                                     # s3 / s3b differ by beta: see profiles/
}
DT = {"f32": 0, "f64": 1, "c128": 3}


def _gemm(m, n, k, dtype="f64") -> W.Problem:
    """Plain column-major matrix product (calibration shape)."""
    e = dict(m=m, n=n, k=k)
    return W.Problem("gemm_%s_%dx%dx%d" % (dtype, m, n, k), dtype, W.tensor("mk", e), W.tensor("kn", e), W.tensor("mn", e),
                     alpha=1.0, beta=0.0, seed=W.BASE_SEED + 20)


def make_problem(name: str) -> W.Problem:
    table = {"cfg1": W.config1, "cfg2": W.config2, "cfg3": W.config3, "cfg4": W.config4, "cfg5": W.config5,
             "cfg3r2": lambda: W.config3(d_layout="R2"), "cfg4hs": lambda: W.config4(h_slowest=True),
             "gemm1k": lambda: W.config2(v=32, o=32),      # contiguous 1024^3 product, same size as cfg5
             "gemmk16": lambda: _gemm(1024, 1024, 16), "gemmk256": lambda: _gemm(1024, 1024, 256),
             # large plain products in both real dtypes (fp32 has no large configuration of its own)
             "gemm8k": lambda: _gemm(8192, 8192, 16384), "gemm8kf": lambda: _gemm(8192, 8192, 16384, "f32"),
             # supplementary HBM-bound shapes
             "s1": lambda: W.config5(extent=4, nshared=1, nfree=7), "s2": lambda: W.config5(extent=4, nshared=0, nfree=7),
             "s3": lambda: W.hadamard(4, 128), "s3p": lambda: W.hadamard(4, 128, permuted=True),
             "s3b": lambda: W.hadamard(4, 128, beta=0.5), "s4": lambda: W.config4(h=512, n=96, k=4)}
    return table[name]()


def _device_tensor(spec: W.TensorSpec, seed, tag, torch, tdtype, dist):
    """Strided tensor generated on the device: values keyed on the logical index, placed by strides."""
    dev = "cuda:0"
    if tdtype == torch.complex128:
        flat = torch.view_as_complex(W.torch_uniform_pm1(seed, tag, 0, 2 * spec.count, torch.float64, dev, dist=dist).view(-1, 2))
    else:
        flat = W.torch_uniform_pm1(seed, tag, 0, spec.count, tdtype, dev, dist=dist)
    contiguous = list(spec.strides) == [int(np.prod(spec.extents[:i], dtype=np.int64)) for i in range(len(spec.extents))]
    if contiguous and spec.size == spec.count:
        return flat
    buf = torch.full((spec.size,), -777.0, dtype=tdtype, device=dev)
    n = len(spec.extents)
    logical = flat.view(*reversed(spec.extents)).permute(*reversed(range(n)))      # index [i0, i1, ..], i0 fastest
    buf.as_strided(spec.extents, spec.strides, spec.base).copy_(logical)
    return buf


def device_operands(p: W.Problem, torch, dist: str = "uniform"):
    """Inputs resident in HBM, generated on the device with the torch twin of the counter-based
    generator (bit-identical to the host generator for uniform and integer values)."""
    tdt = {"f32": torch.float32, "f64": torch.float64, "c128": torch.complex128}[p.dtype]
    a = _device_tensor(p.A, p.seed, W.TAG_A, torch, tdt, dist)
    b = _device_tensor(p.B, p.seed, W.TAG_B, torch, tdt, dist)
    d = _device_tensor(p.D, p.seed, W.TAG_C, torch, tdt, dist)
    return a, b, d, None


def cpu_baseline(p: W.Problem):
    """The oracle's storage-precision loop nest on the host cores, on a bounded sample."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import oracle
    from helpers import run_oracle
    if p.name.startswith("cfg2"):
        sm, sn = 4096, 192
        sub, a, b, c = W.config2_sample(p, np.arange(sm), np.arange(sn))
        sample = "rows m<%d of V, columns n<%d of T, all %d contracted terms (%.2e of %.2e flop)" % (
            sm, sn, p.sizes()[3], sub.real_flops(), p.real_flops())
    else:
        sub = p
        a, b, c = W.make_operands(p)
        sample = "the whole workload"
    t0 = time.perf_counter()
    run_oracle(sub, a, b, c, oracle.MODE_TIMED)
    dt = time.perf_counter() - t0
    return {"value": sub.real_flops() / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": sample, "seconds": dt}


def parity_after_run(p: W.Problem, dD, steps_done: int, torch, dist: str = "uniform"):
    """Sampled check of the timed output of config 2 against the oracle: with beta = 1 and D
    updated in place, after s steps D = D0 + s * (V T) exactly in exact arithmetic."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import oracle
    from helpers import run_oracle
    _, M, N, K = p.sizes()
    rng = np.random.default_rng(p.seed)
    # tile-boundary rows/columns (multiples of the macro-tile extents +-1, first, last) and random ones
    m_idx = np.unique(np.concatenate([[0, 1, 63, 64, 255, 256, 257, M - 257, M - 256, M - 1], rng.integers(0, M, 22)]))
    n_idx = np.unique(np.concatenate([[0, 1, 127, 128, 129, N - 129, N - 128, N - 1], rng.integers(0, N, 8)]))
    sub, a, b, c = W.config2_sample(p, m_idx, n_idx, dist)
    one = W.Problem("ab", "f64", sub.A, sub.B, sub.D, alpha=1.0, beta=0.0)
    ab, S = run_oracle(one, a, b, c, oracle.MODE_TRUTH, want_S=True)
    expect = c + steps_done * ab
    lin = (m_idx[:, None] + M * n_idx[None, :]).T.reshape(-1)          # column-major over (x, y)
    got = dD[torch.from_numpy(lin.astype(np.int64)).to(dD.device)].cpu().numpy()
    err = np.abs(got - expect) / np.maximum(steps_done * S + np.abs(c), 1e-300)
    return {"samples": int(lin.size), "max_normalised_error": float(err.max()), "tolerance": 1e-12,
            "ok": bool(err.max() <= 1e-12), "bit_exact": bool(np.array_equal(got, expect))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variant", type=int, default=None, help="force a tiled-kernel instantiation")
    ap.add_argument("--path", type=int, default=None, help="force a kernel path (0 generic, 1 tiled MFMA, 2 streaming)")
    ap.add_argument("--split-k", type=int, default=None, help="force the number of parts of the contracted range (tiled path)")
    ap.add_argument("--perm-seeds", type=int, default=0,
                    help="cfg5 only: also time this many other permutation seeds (its speed depends on the draw)")
    ap.add_argument("--cold", type=int, default=0,
                    help="rotate through this many distinct copies of the operands (choose enough to exceed the "
                         "256 MB Infinity Cache) so that every step reads its inputs from HBM")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB streaming kernel (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    import paper_2601_07827_amd as T          # raises if libtcx.so is not built: no fallback

    p = make_problem(args.workload)
    torch.cuda.set_device(0)
    dA, dB, dD, _ = device_operands(p, torch)
    torch.cuda.synchronize()

    h = T.tcx_create_handle()
    if not T.tcx_handle_has_device(h):
        sys.exit("bench.py: no gfx950 device")
    stream = torch.cuda.current_stream()
    ex = T.tcx_create_executor(h, stream.cuda_stream)
    ids = W.label_ids(p)
    infos = [T.tcx_create_tensor_info(h, DT[p.dtype], t.extents, t.strides) for t in (p.A, p.B, p.D)]
    labs = [[ids[l] for l in t.labels] for t in (p.A, p.B, p.D)]
    t0 = time.perf_counter()
    prod = T.tcx_create_product(h, p.opA, infos[0], labs[0], p.opB, infos[1], labs[1], p.opC, infos[2], labs[2],
                                0, infos[2], labs[2])
    plan_ms = (time.perf_counter() - t0) * 1e3
    if args.path is not None:
        T.tcx_product_set(prod, T.TCX_KEY_FORCE_PATH, args.path)
    if args.variant is not None:
        T.tcx_product_set(prod, T.TCX_KEY_VARIANT, args.variant)
    if args.split_k is not None:
        T.tcx_product_set(prod, T.TCX_KEY_SPLIT_K, args.split_k)
    item = dD.element_size()
    pA, pB, pD = (t.data_ptr() + s.base * item for t, s in ((dA, p.A), (dB, p.B), (dD, p.D)))

    sets = [(pA, pB, pD)]
    keep = []
    for _ in range(max(0, args.cold - 1)):                # device-side copies: same values, other addresses
        cA, cB, cD = dA.clone(), dB.clone(), dD.clone()
        keep.append((cA, cB, cD))
        sets.append(tuple(t.data_ptr() + s.base * item for t, s in ((cA, p.A), (cB, p.B), (cD, p.D))))
    counter = [0]

    def step():
        a, b, d = sets[counter[0] % len(sets)]
        counter[0] += 1
        T.tcx_execute_product(prod, ex, DT[p.dtype], p.alpha, a, b, p.beta, d, d)

    if args.copy_probe:
        src = torch.ones(1 << 27, dtype=torch.float64, device="cuda:0")     # fill kernel: 1 GiB written
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)                                        # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events on the stream the kernels are launched on: one pair around the whole timed
    # region (launches are back to back, so total / steps is the average launch duration
    # including the gap to the next launch), plus one event per step boundary for the spread.
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(args.steps):
        step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]
    region_ms = marks[0].elapsed_time(marks[-1])
    ms_per_step = wall * 1e3 / args.steps
    flops = p.real_flops()
    value = flops / (ms_per_step * 1e-3) / 1e9

    avg_kernel_s = region_ms / args.steps * 1e-3
    ai = flops / p.algorithmic_bytes()
    ridge = PEAK_TFLOPS[p.dtype] * 1e12 / (PEAK_HBM_GBS * 1e9)
    if ai >= ridge:
        achieved = flops / avg_kernel_s / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS[p.dtype], "unit": "TFLOP/s",
                    "frac": achieved / PEAK_TFLOPS[p.dtype], "traffic": None}
    else:
        achieved = p.algorithmic_bytes() / avg_kernel_s / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    # A step may be several launches of the dominant kernel (a long-tile product is enqueued round
    # by round); the per-launch figures are the step's divided by that count.
    launches = max(1, T.tcx_product_get(prod, T.TCX_KEY_LAUNCHES) - (1 if T.tcx_product_get(prod, T.TCX_KEY_SPLIT_K) > 1 else 0))
    step_traffic = MEASURED_TRAFFIC_BYTES.get(
        (p.name, T.tcx_product_get(prod, T.TCX_KEY_PATH), T.tcx_product_get(prod, T.TCX_KEY_VARIANT)))
    roofline["traffic"] = None if step_traffic is None else step_traffic / launches
    roofline["launches_per_step"] = launches
    roofline["launch_ms_avg"] = region_ms / args.steps / launches
    roofline["algorithmic_per_launch"] = (flops if roofline["bound"] == "mfma" else p.algorithmic_bytes()) / launches
    roofline["kernel_ms_avg"] = region_ms / args.steps
    roofline["kernel_ms_min"] = float(np.min(kern_ms))
    roofline["kernel_ms_median"] = float(np.median(kern_ms))

    cfg = {"workload": p.name, "sizes_HMNK": list(p.sizes()), "alpha": complex(p.alpha).real, "beta": complex(p.beta).real,
           "path": T.tcx_product_get(prod, T.TCX_KEY_PATH), "variant": T.tcx_product_get(prod, T.TCX_KEY_VARIANT),
           "tile": [T.tcx_product_get(prod, k) for k in (T.TCX_KEY_TILE_M, T.TCX_KEY_TILE_N, T.TCX_KEY_TILE_K)],
           "split_k": T.tcx_product_get(prod, T.TCX_KEY_SPLIT_K),
           "grid": T.tcx_product_get(prod, T.TCX_KEY_GRID), "launches_per_step": T.tcx_product_get(prod, T.TCX_KEY_LAUNCHES),
           "gather_width": T.tcx_product_get(prod, T.TCX_KEY_GATHER_WIDTH),
           "plan_ms": plan_ms,
           "flop_per_step": flops, "algorithmic_bytes_per_step": p.algorithmic_bytes()}

    cfg["buffers"] = "cache-resident (one operand set)" if len(sets) == 1 else \
        "cold: rotating over %d operand sets, %.0f MB in total" % (len(sets), len(sets) * p.algorithmic_bytes() / 1e6)
    if avg_kernel_s < 1e-3:
        # what a back-to-back launch of an (almost) empty kernel costs on this stream: the floor
        # under any sub-millisecond figure above
        one = torch.zeros(1, device="cuda:0")
        for _ in range(20):
            one.zero_()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(200):
            one.zero_()
        e1.record(stream)
        torch.cuda.synchronize()
        roofline["launch_floor_us"] = e0.elapsed_time(e1) / 200 * 1e3

    if args.perm_seeds and args.workload == "cfg5":
        times = []
        for ps in range(args.perm_seeds):
            q = W.config5(perm_seed=1000 + ps)
            qa, qb, qd, _ = device_operands(q, torch)
            qi = [T.tcx_create_tensor_info(h, DT[q.dtype], t.extents, t.strides) for t in (q.A, q.B, q.D)]
            ql = [[W.label_ids(q)[l] for l in t.labels] for t in (q.A, q.B, q.D)]
            qp = T.tcx_create_product(h, 0, qi[0], ql[0], 0, qi[1], ql[1], 0, qi[2], ql[2], 0, qi[2], ql[2])
            for _ in range(3):
                T.tcx_execute_product(qp, ex, DT[q.dtype], q.alpha, qa.data_ptr(), qb.data_ptr(), q.beta, 0, qd.data_ptr())
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(51)]
            ev[0].record(stream)
            for it in range(50):
                T.tcx_execute_product(qp, ex, DT[q.dtype], q.alpha, qa.data_ptr(), qb.data_ptr(), q.beta, 0, qd.data_ptr())
                ev[it + 1].record(stream)
            torch.cuda.synchronize()
            # the median launch: a single stall of the box (tens of ms, now and then) would own a mean
            times.append(float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(50)])) * 1e3)
            T.tcx_destroy_product(qp)
        cfg["perm_seed_us"] = {"min": float(np.min(times)), "median": float(np.median(times)), "max": float(np.max(times)),
                               "n": len(times)}

    out = {"metric": "contraction GFLOP/s (fp64/fp32/c128) and % MFMA peak; GB/s for low-AI shapes",
           "value": value, "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": p.dtype, "data": "synthetic", "config": cfg, "roofline": roofline}
    if not args.no_cpu_baseline:
        # the only leg that runs the oracle: its timing, and (config 2) its values on sampled
        # elements of the buffer the timed steps have just written
        out["cpu_baseline"] = cpu_baseline(p)
        if p.name.startswith("cfg2"):
            out["cpu_baseline"]["parity_of_timed_output"] = parity_after_run(p, dD, args.warmup + args.steps, torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
