#!/usr/bin/env python3
"""Benchmark of the contraction hot path on ONE MI355X.

A "step" is one execution of the planned contraction over resident device buffers.  The headline
(`value`, `ms_per_step`, `roofline`, `cpu_baseline` at the top level of the JSON line) is
configuration 2, the fp64 particle-particle ladder D[a,b,i,j] += sum_{c,d} V[a,b,c,d] T[c,d,i,j]
with v = 192, o = 64 (1.1133e13 flop), timed over exactly --steps steps after --warmup steps.
The same line carries a `configs` array with the other four configurations and the supplementary
memory-bound shapes: per workload the plan, warm (one operand set) and cold (rotating operand sets
beyond the 256 MB memory-side cache) time per step, the roofline figure, the oracle's time on the
host cores, and the parity of the buffer the timed steps wrote.  `peaks` holds the specification
figures and what single-purpose probe kernels sustain on this chip.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|cfg2|cfg1|...]
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

PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3, "c128": 78.6, "c64": 157.3}     # MI355X dense matrix peaks
PEAK_HBM_GBS = 8000.0
CACHE_BYTES = 256e6                                       # memory-side cache: cold runs rotate over more than twice this
TOLERANCE = {"f32": 1e-5, "f64": 1e-12, "c128": 1e-12, "c64": 1e-5}
DT = {"f32": 0, "f64": 1, "c64": 2, "c128": 3, "f16": 4}
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")

# workloads of the default run besides the headline, in the order they are reported
SUITE = ["cfg1", "cfg3", "cfg3r2", "cfg4", "cfg4hs", "cfg5", "s1", "s2", "s3", "s3b", "s3p", "s4"]
HOST_LIMIT = 1 << 26          # operands up to this many elements are generated on the host and checked in full


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
             "s3b": lambda: W.hadamard(4, 128, beta=0.5), "s4": lambda: W.config4(h=512, n=96, k=4),
             # s3p with 128 bytes added to every tensor's slowest stride (diagnostic: not all strides powers of two)
             "s3pp": lambda: W.hadamard(4, 128, permuted=True, pad_slowest=16)}
    return table[name]()


# ---- operands -------------------------------------------------------------------------------------
def _torch_dtype(p, torch):
    return {"f32": torch.float32, "f64": torch.float64, "c128": torch.complex128, "c64": torch.complex64}[p.dtype]


def _device_tensor(spec: W.TensorSpec, seed, tag, torch, tdtype, dist):
    """Strided tensor generated on the device: values keyed on the logical index, placed by strides."""
    dev = "cuda:0"
    if tdtype in (torch.complex128, torch.complex64):
        real = torch.float64 if tdtype == torch.complex128 else torch.float32
        flat = torch.view_as_complex(W.torch_uniform_pm1(seed, tag, 0, 2 * spec.count, real, dev, dist=dist).view(-1, 2))
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
    tdt = _torch_dtype(p, torch)
    a = _device_tensor(p.A, p.seed, W.TAG_A, torch, tdt, dist)
    b = _device_tensor(p.B, p.seed, W.TAG_B, torch, tdt, dist)
    d = _device_tensor(p.D, p.seed, W.TAG_C, torch, tdt, dist)
    return a, b, d, None


class Operands:
    """Device buffers of one problem (and host copies when they were generated there)."""

    def __init__(self, p: W.Problem, torch):
        self.p, self.host = p, None
        small = max(p.A.size, p.B.size, p.D.size) <= HOST_LIMIT
        if p.beta == 0 and p.D.size > HOST_LIMIT and max(p.A.size, p.B.size) <= HOST_LIMIT:
            a = W.fill(p.A, p.seed, W.TAG_A, p.np_dtype, p.dist)      # a large output of small operands that is never read
            b = W.fill(p.B, p.seed, W.TAG_B, p.np_dtype, p.dist)
            self.dA, self.dB = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
            self.dC = torch.full((p.D.size,), -777.0, dtype=_torch_dtype(p, torch), device="cuda:0")
        elif small or p.dist == "normal":
            a, b, c = W.make_operands(p)
            self.host = (a, b, c)
            self.dA, self.dB, self.dC = (torch.from_numpy(x).cuda() for x in (a, b, c))
        else:
            self.dA, self.dB, self.dC, _ = device_operands(p, torch)
        # C is its own buffer (the steps are then idempotent: D = alpha A B + beta C every time)
        self.dD = self.dC.clone() if p.beta != 0 else self.dC
        torch.cuda.synchronize()

    def pointers(self, dA=None, dB=None, dC=None, dD=None):
        p = self.p
        item = self.dD.element_size()
        A, B, C, D = (self.dA if dA is None else dA, self.dB if dB is None else dB,
                      self.dC if dC is None else dC, self.dD if dD is None else dD)
        return (A.data_ptr() + p.A.base * item, B.data_ptr() + p.B.base * item,
                C.data_ptr() + p.D.base * item, D.data_ptr() + p.D.base * item)


# ---- plan -------------------------------------------------------------------------------------------
class Plan:
    def __init__(self, T, h, ex, p: W.Problem, path=None, variant=None, split_k=None):
        self.T, self.p, self.ex = T, p, ex
        ids = W.label_ids(p)
        infos = [T.tcx_create_tensor_info(h, DT[p.dtype], t.extents, t.strides) for t in (p.A, p.B, p.D)]
        labs = [[ids[l] for l in t.labels] for t in (p.A, p.B, p.D)]
        t0 = time.perf_counter()
        self.prod = T.tcx_create_product(h, p.opA, infos[0], labs[0], p.opB, infos[1], labs[1], p.opC, infos[2], labs[2],
                                         0, infos[2], labs[2])
        self.plan_ms = (time.perf_counter() - t0) * 1e3
        for i in infos:
            T.tcx_destroy_tensor_info(i)
        if path is not None:
            T.tcx_product_set(self.prod, T.TCX_KEY_FORCE_PATH, path)
        if variant is not None:
            T.tcx_product_set(self.prod, T.TCX_KEY_VARIANT, variant)
        if split_k is not None:
            T.tcx_product_set(self.prod, T.TCX_KEY_SPLIT_K, split_k)

    def get(self, key):
        return self.T.tcx_product_get(self.prod, key)

    def run(self, ptrs):
        a, b, c, d = ptrs
        self.T.tcx_execute_product(self.prod, self.ex, DT[self.p.dtype], self.p.alpha, a, b, self.p.beta, c, d)

    def describe(self):
        T, p = self.T, self.p
        launches = self.get(T.TCX_KEY_LAUNCHES)
        return {"workload": p.name, "sizes_HMNK": list(p.sizes()), "alpha": complex(p.alpha).real, "beta": complex(p.beta).real,
                "path": self.get(T.TCX_KEY_PATH), "variant": self.get(T.TCX_KEY_VARIANT),
                "tile": [self.get(k) for k in (T.TCX_KEY_TILE_M, T.TCX_KEY_TILE_N, T.TCX_KEY_TILE_K)],
                "split_k": self.get(T.TCX_KEY_SPLIT_K), "grid": self.get(T.TCX_KEY_GRID), "launches_per_step": launches,
                "gather_width": self.get(T.TCX_KEY_GATHER_WIDTH), "plan_ms": self.plan_ms,
                "flop_per_step": p.real_flops(), "algorithmic_bytes_per_step": p.algorithmic_bytes()}

    def close(self):
        self.T.tcx_destroy_product(self.prod)


# ---- timing -------------------------------------------------------------------------------------------
def timed_region(torch, stream, step, steps):
    """`steps` back-to-back steps between two HIP events recorded on the launch stream, plus one
    event per step boundary for the spread.  Returns (region ms, per-step ms list, wall seconds)."""
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(steps):
        step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return marks[0].elapsed_time(marks[-1]), [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)], wall


def region_us(torch, stream, step, launches, reps=5):
    """Median over `reps` regions of (time of `launches` back-to-back steps) / launches, in us:
    two events per region, none between the steps."""
    out = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(launches):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) / launches * 1e3)
    return float(np.median(out)), float(np.min(out))


def launch_floor_us(torch, stream):
    """Back-to-back launch cost of an (almost) empty kernel on the same stream."""
    one = torch.zeros(1, device="cuda:0")
    for _ in range(20):
        one.zero_()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(200):
        one.zero_()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / 200 * 1e3


def roofline_of(p: W.Problem, seconds_per_step: float):
    flops, nbytes = p.real_flops(), p.algorithmic_bytes()
    ridge = PEAK_TFLOPS[p.dtype] * 1e12 / (PEAK_HBM_GBS * 1e9)
    if flops / nbytes >= ridge:
        achieved = flops / seconds_per_step / 1e12
        return {"bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS[p.dtype], "unit": "TFLOP/s",
                "frac": achieved / PEAK_TFLOPS[p.dtype], "traffic": None}
    achieved = nbytes / seconds_per_step / 1e9
    return {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
            "traffic": None}


def measured_traffic(desc):
    """HBM bytes per step of this (workload, path, tile shape, split) from the last counter run
    summarised into profiles/traffic.json (see --pmc-summary); None if that run used another plan."""
    try:
        table = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None
    row = table.get(desc.get("alias", desc["workload"]))
    if not row or [row.get("path"), row.get("variant"), row.get("split_k")] != [desc["path"], desc["variant"], desc["split_k"]]:
        return None
    return row["fetch_bytes_per_step"] + row["write_bytes_per_step"]


# ---- parity of the timed output and the CPU baseline ---------------------------------------------------
def _oracle():
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import oracle
    from helpers import normalised_error, run_oracle
    return oracle, run_oracle, normalised_error


def full_parity_and_baseline(p: W.Problem, ops: Operands, want_baseline: bool):
    """Whole output of the timed buffer against the oracle's truth; the oracle's storage-precision
    loop nest over the whole workload is the CPU baseline."""
    oracle, run_oracle, normalised_error = _oracle()
    a, b, c = ops.host
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    got = ops.dD.cpu().numpy()
    err = normalised_error(p, got, truth, S, c)
    parity = {"compared": "every element of D", "elements": int(p.D.count), "max_normalised_error": err,
              "tolerance": TOLERANCE[p.dtype], "ok": bool(err <= TOLERANCE[p.dtype])}
    base = None
    if want_baseline:
        t0 = time.perf_counter()
        run_oracle(p, a, b, c, oracle.MODE_TIMED)
        dt = time.perf_counter() - t0
        base = {"value": p.real_flops() / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.max_threads(), "kind": "oracle",
                "sample": "the whole workload", "seconds": dt}
    return parity, base


def sampled_parity_and_baseline(p: W.Problem, ops: Operands, torch, nsamples: int, want_baseline: bool):
    """Sampled outputs of the timed buffer: for `nsamples` index tuples of D (first, last and seeded
    random ones) the operand rows they depend on are fetched from the device buffers and handed to
    the oracle as a batch of independent sums  D_s[x] = alpha sum_k A_s[k, x] B_s[k, x] + beta C_s[x]."""
    oracle, run_oracle, _ = _oracle()
    assert all(len(set(t.labels)) == len(t.labels) for t in (p.A, p.B, p.D))
    H, M, N, K = p.groups()
    ext = p.extent_of()
    rng = np.random.default_rng(p.seed)
    dlabels = list(p.D.labels)
    idx = {l: rng.integers(0, ext[l], nsamples) for l in dlabels}
    for l in dlabels:
        idx[l][0], idx[l][1] = 0, ext[l] - 1
    nk = int(np.prod([ext[l] for l in K], dtype=np.int64)) if K else 1
    kgrid, run = {}, np.arange(nk, dtype=np.int64)
    for l in K:                                       # first contracted label fastest
        kgrid[l] = run % ext[l]
        run = run // ext[l]

    def offsets(spec):
        off = np.full((nsamples, nk), spec.base, dtype=np.int64)
        for l, s in zip(spec.labels, spec.strides):
            off += (idx[l][:, None] if l in idx else kgrid[l][None, :]) * s
        return off

    dev = ops.dD.device

    def fetch(buf, off):
        return buf[torch.from_numpy(off.reshape(-1)).to(dev)].cpu().numpy()

    offD = np.full(nsamples, p.D.base, dtype=np.int64)
    for l, s in zip(p.D.labels, p.D.strides):
        offD += idx[l] * s
    a, b = fetch(ops.dA, offsets(p.A)), fetch(ops.dB, offsets(p.B))
    c = fetch(ops.dC, offD) if p.beta != 0 else np.zeros(nsamples, dtype=p.np_dtype)
    got = fetch(ops.dD, offD)
    e = dict(k=nk, x=nsamples)
    sub = W.Problem(p.name + "_sampled", p.dtype, W.tensor("kx", e), W.tensor("kx", e), W.tensor("x", e),
                    alpha=p.alpha, beta=p.beta, opA=p.opA, opB=p.opB, opC=p.opC, seed=p.seed)
    truth, S = run_oracle(sub, a, b, c, oracle.MODE_TRUTH, want_S=True)
    den = abs(p.alpha) * S + abs(p.beta) * np.abs(c)
    err = float(np.max(np.abs(got - truth) / np.maximum(den, np.finfo(np.float64).tiny)))
    parity = {"compared": "%d sampled elements of D (first, last, seeded random), each a full sum over %d terms" % (nsamples, nk),
              "elements": nsamples, "max_normalised_error": err, "tolerance": TOLERANCE[p.dtype], "ok": bool(err <= TOLERANCE[p.dtype])}
    base = None
    if want_baseline:
        t0 = time.perf_counter()
        run_oracle(sub, a, b, c, oracle.MODE_TIMED)
        dt = time.perf_counter() - t0
        base = {"value": sub.real_flops() / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.max_threads(), "kind": "oracle",
                "sample": "%d sampled elements of D with their operand rows (%.2e of %.2e flop)" % (nsamples, sub.real_flops(), p.real_flops()),
                "seconds": dt}
    return parity, base


def cpu_baseline(p: W.Problem):
    """Configuration 2: the oracle's storage-precision loop nest on a bounded slab."""
    oracle, run_oracle, _ = _oracle()
    sm, sn = 1024, 192           # about 20 s of the oracle on 16 host threads
    sub, a, b, c = W.config2_sample(p, np.arange(sm), np.arange(sn))
    sample = "rows m<%d of V, columns n<%d of T, all %d contracted terms (%.2e of %.2e flop)" % (
        sm, sn, p.sizes()[3], sub.real_flops(), p.real_flops())
    t0 = time.perf_counter()
    run_oracle(sub, a, b, c, oracle.MODE_TIMED)
    dt = time.perf_counter() - t0
    return {"value": sub.real_flops() / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": sample, "seconds": dt}


def config2_sample_indices(p: W.Problem, tile_m: int, tile_n: int, rng, rows=384, cols=192):
    """Rows and columns whose grid of samples (rows x cols of them, 73 728 by default) reaches every
    launch round and, inside a round, the stretch of tiles of every XCD: tiles wider than high are walked
    in bands of 4 tile rows (one round of 256 workgroups is two bands of 4 x 32 tiles), and an XCD's
    stretch is 8 tile columns of a band.  The last row / column of every tile and the first of the next
    (every tile boundary), the first and last two of the tensor, one seeded random row in every band and
    column in every group of 8 tile columns, and seeded random ones up to the requested count."""
    _, M, N, _ = p.sizes()
    band, group = 4 * tile_m, 8 * tile_n

    def pick(extent, tile, stretch, want):
        idx = [0, 1, extent - 2, extent - 1]
        for edge in range(tile, extent, tile):
            idx += [edge - 1, edge]
        idx += [int(lo + rng.integers(0, min(stretch, extent - lo))) for lo in range(0, extent, stretch)]
        idx = np.unique(np.clip(np.asarray(idx, dtype=np.int64), 0, extent - 1))
        if len(idx) < want:
            idx = np.unique(np.concatenate([idx, rng.integers(0, extent, want - len(idx))]))
        return idx
    return pick(M, tile_m, band, rows), pick(N, tile_n, group, cols)


def parity_after_run(p: W.Problem, dD, steps_done: int, torch, dist: str = "uniform", tile=(256, 128)):
    """Sampled check of the timed output of config 2 against the oracle: with beta = 1 and D
    updated in place, after s steps D = D0 + s * (V T) exactly in exact arithmetic."""
    oracle, run_oracle, _ = _oracle()
    _, M, N, K = p.sizes()
    rng = np.random.default_rng(p.seed)
    m_idx, n_idx = config2_sample_indices(p, tile[0], tile[1], rng)
    sub, a, b, c = W.config2_sample(p, m_idx, n_idx, dist)
    one = W.Problem("ab", "f64", sub.A, sub.B, sub.D, alpha=1.0, beta=0.0)
    ab, S = run_oracle(one, a, b, c, oracle.MODE_TRUTH, want_S=True)
    expect = c + steps_done * ab
    lin = (m_idx[:, None] + M * n_idx[None, :]).T.reshape(-1)          # column-major over (x, y)
    got = dD[torch.from_numpy(lin.astype(np.int64)).to(dD.device)].cpu().numpy()
    err = np.abs(got - expect) / np.maximum(steps_done * S + np.abs(c), 1e-300)
    return {"samples": int(lin.size), "rows": [int(v) for v in m_idx], "columns": [int(v) for v in n_idx],
            "max_normalised_error": float(err.max()), "tolerance": 1e-12,
            "ok": bool(err.max() <= 1e-12), "bit_exact": bool(np.array_equal(got, expect))}


# ---- what the chip sustains (probe kernels) -------------------------------------------------------------
def measured_peaks(T, ex, torch, stream):
    """Specification figures beside what single-purpose kernels reach on this chip."""
    buf = torch.empty(1 << 28, dtype=torch.float64, device="cuda:0")          # 2 GiB
    out = {"spec": {"mfma_f64_TFLOPs": PEAK_TFLOPS["f64"], "mfma_f32_TFLOPs": PEAK_TFLOPS["f32"], "hbm_GBs": PEAK_HBM_GBS}}

    def rate(kind, nbytes, iters):
        T.tcx_probe_launch(ex, kind, buf.data_ptr(), nbytes, iters)           # warm-up
        best = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            work = T.tcx_probe_launch(ex, kind, buf.data_ptr(), nbytes, iters)
            e1.record(stream)
            torch.cuda.synchronize()
            best = max(best, work / (e0.elapsed_time(e1) * 1e-3))
        return best

    out["measured"] = {"mfma_f64_TFLOPs": rate(T.TCX_PROBE_MFMA_F64, 4096, 20000) / 1e12,
                       "mfma_f32_TFLOPs": rate(T.TCX_PROBE_MFMA_F32, 4096, 20000) / 1e12,
                       "store_GBs": rate(T.TCX_PROBE_STORE, buf.numel() * 8, 0) / 1e9,
                       "copy_GBs": rate(T.TCX_PROBE_COPY, buf.numel() * 8, 0) / 1e9}
    out["how"] = ("back-to-back independent 16x16x4 MFMAs from 8 waves per CU; 16-byte stores over 2 GiB; "
                  "copy of 1 GiB to 1 GiB (bytes read + written)")
    del buf
    return out


# ---- one workload of the suite ------------------------------------------------------------------------------
def measure(name, T, h, ex, torch, stream, want_baseline=True, path=None, variant=None, split_k=None):
    p = make_problem(name)
    ops = Operands(p, torch)
    plan = Plan(T, h, ex, p, path, variant, split_k)
    desc = dict(plan.describe(), alias=name)
    warm_ptrs = ops.pointers()
    plan.run(warm_ptrs)
    torch.cuda.synchronize()
    # launches per timed region: about 20 ms of work, at least 10
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(3):
        plan.run(warm_ptrs)
    e1.record(stream)
    torch.cuda.synchronize()
    est_ms = max(e0.elapsed_time(e1) / 3, 1e-3)
    launches = int(min(400, max(10, 20.0 / est_ms)))
    warm_us, warm_min = region_us(torch, stream, lambda: plan.run(warm_ptrs), launches)
    # the same steps with an event between every two: nothing of one step's launch overlaps the
    # end of the step before it, so this is the time of a step issued alone
    _, apart, _ = timed_region(torch, stream, lambda: plan.run(warm_ptrs), min(launches, 100))
    torch.cuda.synchronize()
    # parity of the buffer the timed steps wrote
    if ops.host is not None:
        parity, base = full_parity_and_baseline(p, ops, want_baseline)
    else:
        parity, base = sampled_parity_and_baseline(p, ops, torch, 4096, want_baseline)
    # cold: rotate over operand sets that together exceed twice the memory-side cache
    nbytes = p.algorithmic_bytes()
    if nbytes >= 2 * CACHE_BYTES:
        cold_us, cold_note = warm_us, "one operand set of %.0f MB exceeds the cache: warm is cold" % (nbytes / 1e6)
    else:
        nsets = int(np.ceil(2 * CACHE_BYTES / nbytes)) + 1
        sets, keep = [], []
        for _ in range(nsets):
            cA, cB, cC = ops.dA.clone(), ops.dB.clone(), ops.dC.clone()
            cD = cC.clone() if p.beta != 0 else cC
            keep.append((cA, cB, cC, cD))
            sets.append(ops.pointers(cA, cB, cC, cD))
        counter = [0]

        def cold_step():
            plan.run(sets[counter[0] % nsets])
            counter[0] += 1
        for _ in range(nsets):
            cold_step()
        cold_us, _ = region_us(torch, stream, cold_step, max(launches, nsets))
        cold_note = "rotating over %d operand sets, %.0f MB in total" % (nsets, nsets * nbytes / 1e6)
        del keep
    roof = roofline_of(p, warm_us * 1e-6)
    roof["frac_cold"] = roofline_of(p, cold_us * 1e-6)["frac"]
    roof["traffic"] = measured_traffic(desc)
    out = {"workload": name, "dtype": p.dtype, "config": desc, "warm_us": warm_us, "warm_us_min": warm_min,
           "warm_us_apart": float(np.median(apart)) * 1e3, "cold_us": cold_us,
           "launches_per_region": launches, "buffers_cold": cold_note, "roofline": roof, "parity_of_timed_output": parity}
    if base is not None:
        out["cpu_baseline"] = base
    plan.close()
    del ops
    torch.cuda.empty_cache()
    return out


def pmc_summary(args):
    """Fold the counter files of two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE) of
    `bench.py --workload W --copy-probe` into profiles/traffic.json: bytes per step of the library's
    kernels, each counter scaled by what it reads for the probe kernels of known size in the same run."""
    import csv
    import glob
    work = json.loads(open(args.pmc_summary[0]).read().strip().splitlines()[-1])
    desc = work["config"]
    steps = work["steps"] + work["warmup"]
    row = {"path": desc["path"], "variant": desc["variant"], "split_k": desc["split_k"], "steps_profiled": steps}
    for counter, folder in (("FETCH_SIZE", args.pmc_summary[1]), ("WRITE_SIZE", args.pmc_summary[2])):
        files = glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True)
        lib = probe_copy = 0.0
        for r in csv.DictReader(open(files[0])):
            if r["Counter_Name"] != counter:
                continue
            v = float(r["Counter_Value"]) * 1024.0                     # KiB
            if "copy_probe_kernel" in r["Kernel_Name"]:
                probe_copy += v
            elif "probe_kernel" not in r["Kernel_Name"] and "tcx::" in r["Kernel_Name"]:
                lib += v
        # the copy probe, run once, reads 1 GiB and writes 1 GiB
        scale = float(1 << 30) / probe_copy if probe_copy > 0 else 1.0
        row["%s_scale" % counter.lower()] = scale
        row["%s_bytes_per_step" % ("fetch" if counter == "FETCH_SIZE" else "write")] = lib * scale / steps
    try:
        table = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        table = {}
    table[desc.get("alias", desc["workload"])] = row
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps({desc.get("alias", desc["workload"]): row}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="all",
                    help="'all': configuration 2 as the headline plus the `configs` array; a name: that workload alone as the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variant", type=int, default=None, help="force a tiled-kernel instantiation")
    ap.add_argument("--path", type=int, default=None, help="force a kernel path (0 generic, 1 tiled MFMA, 2 streaming)")
    ap.add_argument("--split-k", type=int, default=None, help="force the number of parts of the contracted range (tiled path)")
    ap.add_argument("--perm-seeds", type=int, default=0,
                    help="cfg5 only: also time this many other permutation seeds (its speed depends on the draw)")
    ap.add_argument("--cold", type=int, default=0,
                    help="rotate through this many distinct copies of the operands (choose enough to exceed the "
                         "256 MB memory-side cache) so that every step reads its inputs from HBM")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run the store and copy probe kernels once each (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--pmc-summary", nargs=3, metavar=("BENCH_JSON", "FETCH_DIR", "WRITE_DIR"),
                    help="no GPU work: fold two rocprofv3 --pmc output folders into profiles/traffic.json")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")
    if args.pmc_summary:
        return pmc_summary(args)

    import torch
    import __graft_entry__
    __graft_entry__.ensure_built()            # compiles only where no library is there yet
    import paper_2601_07827_amd as T          # raises if libtcx.so is missing: no fallback

    torch.cuda.set_device(0)
    h = T.tcx_create_handle()
    if not T.tcx_handle_has_device(h):
        sys.exit("bench.py: no gfx950 device")
    stream = torch.cuda.current_stream()
    ex = T.tcx_create_executor(h, stream.cuda_stream)
    suite = args.workload == "all"
    head = "cfg2" if suite else args.workload

    p = make_problem(head)
    in_place = p.name.startswith("cfg2")           # configuration 2 is stated as an update of D in place
    if in_place:
        dA, dB, dD, _ = device_operands(p, torch)
        dC = dD
        ops = None
    else:
        ops = Operands(p, torch)
        dA, dB, dC, dD = ops.dA, ops.dB, ops.dC, ops.dD
    torch.cuda.synchronize()
    plan = Plan(T, h, ex, p, args.path, args.variant, args.split_k)
    item = dD.element_size()
    ptr = lambda t, s: t.data_ptr() + s.base * item
    sets = [(ptr(dA, p.A), ptr(dB, p.B), ptr(dC, p.D), ptr(dD, p.D))]
    keep = []
    for _ in range(max(0, args.cold - 1)):                # device-side copies: same values, other addresses
        cA, cB, cC = dA.clone(), dB.clone(), dC.clone()
        cD = cC if (in_place or p.beta == 0) else cC.clone()
        keep.append((cA, cB, cC, cD))
        sets.append((ptr(cA, p.A), ptr(cB, p.B), ptr(cC, p.D), ptr(cD, p.D)))
    counter = [0]

    def step():
        plan.run(sets[counter[0] % len(sets)])
        counter[0] += 1

    if args.copy_probe:
        probe = torch.empty(1 << 28, dtype=torch.float64, device="cuda:0")
        T.tcx_probe_launch(ex, T.TCX_PROBE_STORE, probe.data_ptr(), probe.numel() * 8)      # 2 GiB written
        T.tcx_probe_launch(ex, T.TCX_PROBE_COPY, probe.data_ptr(), probe.numel() * 8)       # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        del probe
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    region_ms, kern_ms, wall = timed_region(torch, stream, step, args.steps)
    ms_per_step = wall * 1e3 / args.steps
    flops = p.real_flops()
    value = flops / (ms_per_step * 1e-3) / 1e9

    cfg = dict(plan.describe(), alias=head)
    roofline = roofline_of(p, region_ms / args.steps * 1e-3)
    # A step may be several launches of the dominant kernel (a long-tile product is enqueued round
    # by round); the per-launch figures are the step's divided by that count.
    launches = max(1, cfg["launches_per_step"] - (1 if plan.get(T.TCX_KEY_WORKSPACE_BYTES) > 0 else 0))
    step_traffic = measured_traffic(cfg)
    roofline["traffic"] = None if step_traffic is None else step_traffic / launches
    roofline["launches_per_step"] = launches
    roofline["launch_ms_avg"] = region_ms / args.steps / launches
    roofline["algorithmic_per_launch"] = (flops if roofline["bound"] == "mfma" else p.algorithmic_bytes()) / launches
    roofline["kernel_ms_avg"] = region_ms / args.steps
    roofline["kernel_ms_min"] = float(np.min(kern_ms))
    roofline["kernel_ms_median"] = float(np.median(kern_ms))
    total_bytes = len(sets) * p.algorithmic_bytes()
    if len(sets) > 1:
        cfg["buffers"] = "cold: rotating over %d operand sets, %.0f MB in total" % (len(sets), total_bytes / 1e6)
    elif total_bytes > 2 * CACHE_BYTES:
        cfg["buffers"] = "one operand set of %.0f MB, far beyond the 256 MB memory-side cache: read from HBM every step" % (total_bytes / 1e6)
    else:
        cfg["buffers"] = "cache-resident (one operand set of %.0f MB)" % (total_bytes / 1e6)
    if region_ms / args.steps < 1.0:
        roofline["launch_floor_us"] = launch_floor_us(torch, stream)

    if args.perm_seeds and head == "cfg5":
        times = []
        for ps in range(args.perm_seeds):
            q = W.config5(perm_seed=1000 + ps)
            qo = Operands(q, torch)
            qp = Plan(T, h, ex, q)
            qptr = qo.pointers()
            for _ in range(3):
                qp.run(qptr)
            times.append(region_us(torch, stream, lambda: qp.run(qptr), 400)[0])      # as many steps per region as `configs` uses
            qp.close()
        cfg["perm_seed_us"] = {"min": float(np.min(times)), "median": float(np.median(times)), "max": float(np.max(times)),
                               "n": len(times)}

    out = {"metric": "contraction GFLOP/s (fp64/fp32/c128) and % MFMA peak; GB/s for low-AI shapes",
           "value": value, "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": p.dtype, "data": "synthetic", "config": cfg, "roofline": roofline}
    if not args.no_cpu_baseline:
        # the only leg that runs the oracle: its timing, and its values on the buffer the timed
        # steps have just written
        if in_place:
            out["cpu_baseline"] = cpu_baseline(p)
            out["cpu_baseline"]["parity_of_timed_output"] = parity_after_run(
                p, dD, args.warmup + args.steps, torch, tile=(cfg["tile"][0] or 256, cfg["tile"][1] or 128))
        elif ops.host is not None:
            parity, base = full_parity_and_baseline(p, ops, True)
            out["cpu_baseline"] = dict(base, parity_of_timed_output=parity)
        else:
            parity, base = sampled_parity_and_baseline(p, ops, torch, 4096, True)
            out["cpu_baseline"] = dict(base, parity_of_timed_output=parity)
    plan.close()
    del dA, dB, dC, dD, ops, keep
    torch.cuda.empty_cache()
    if suite:
        out["peaks"] = measured_peaks(T, ex, torch, stream)
        out["launch_floor_us"] = launch_floor_us(torch, stream)
        out["configs"] = []
        for name in SUITE:
            sys.stderr.write("[bench] %s\n" % name)
            sys.stderr.flush()
            out["configs"].append(measure(name, T, h, ex, torch, stream, want_baseline=not args.no_cpu_baseline))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
