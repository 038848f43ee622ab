"""Glue shared by the tests: run the oracle on a workloads.Problem, the error measure,
and a random problem generator.  Holds no contraction arithmetic of its own."""
from __future__ import annotations

import numpy as np

import oracle
import workloads as W


def desc(spec: W.TensorSpec, ids):
    return (list(spec.extents), list(spec.strides), [ids[l] for l in spec.labels])


def run_oracle(p: W.Problem, bufA, bufB, bufC, mode=oracle.MODE_TRUTH, want_S=False, alpha=None, beta=None):
    """Returns (bufD, S).  bufC is not modified."""
    ids = W.label_ids(p)
    bufD = bufC.copy()
    al = p.alpha if alpha is None else alpha
    be = p.beta if beta is None else beta
    st, S = oracle.contract(desc(p.A, ids), desc(p.B, ids), desc(p.D, ids), desc(p.D, ids),
                            (p.opA, p.opB, p.opC), al, be, bufA, bufB, bufC, bufD,
                            base=(p.A.base, p.B.base, p.D.base, p.D.base), mode=mode, want_S=want_S)
    assert st == oracle.V_OK, oracle.V_NAMES[st]
    return bufD, S


UNIT_ROUNDOFF = {"f32": 2.0 ** -24, "f64": 2.0 ** -53, "c128": 2.0 ** -53, "c64": 2.0 ** -24, "f16": 2.0 ** -11,
                 "bf16": 2.0 ** -8}
# Gate of the error measure |d - d_truth| / (|alpha| S + |beta| |c|), S = sum |a||b|.
# 16-bit tensors are computed in 32-bit (or 64-bit) arithmetic and rounded to storage once: the
# error is one 16-bit rounding of d, at most 2^-11 |d| <= 2^-11 (|alpha| S + |beta||c|), plus the
# 32-bit accumulation error (|K| + 2) 2^-24 S; the gate is twice the rounding bound.
# bfloat16 (unit roundoff 2^-8): the same bound; where a label lives in one operand only the reduced
# operand is rounded to storage as well (a second 2^-8, against |alpha| S), and with the 32-bit
# accumulation error of up to 2^11 terms the two stay below 2^-7 (1 + 2^-5).
TOLERANCE = {"f32": 1e-5, "f64": 1e-12, "c128": 1e-12, "c64": 1e-5, "f16": 2.0 ** -10, "bf16": 2.0 ** -7 * (1 + 2.0 ** -5)}
# 32-bit tensors computed with TCX_PREC_F64: sums are exact to 64-bit rounding, D is rounded to
# storage once: |error| <= 2^-24 |d| (1 + small) <= 2^-24 (|alpha| S + |beta||c|); gate at twice that.
TOLERANCE_WIDENED = 2.0 ** -23


def values_of(p: W.Problem, buf, spec):
    """The tensor `spec` inside `buf` as numbers (bfloat16 buffers hold bit patterns)."""
    v = W.strided_view(buf, spec)
    return W.bf16_values(v) if p.dtype == "bf16" else v


def normalised_error(p: W.Problem, got, truth, S, bufC, alpha=None, beta=None):
    """max over the addressed elements of D of |got - truth| / (|alpha| S + |beta||c|)."""
    al = abs(p.alpha if alpha is None else alpha)
    be = abs(p.beta if beta is None else beta)
    g = values_of(p, got, p.D).astype(np.complex128 if p.dtype in ("c128", "c64") else np.float64)
    t = values_of(p, truth, p.D).astype(g.dtype)
    s = W.strided_view(S, p.D)
    c = np.abs(values_of(p, bufC, p.D).astype(g.dtype)) if be != 0 else 0.0
    den = al * s + be * c
    num = np.abs(g - t)
    tiny = np.finfo(np.float64).tiny
    ok_zero = (den == 0) & (num == 0)
    ratio = np.where(ok_zero, 0.0, num / np.maximum(den, tiny))
    return float(ratio.max()) if ratio.size else 0.0


def gaps_untouched(p: W.Problem, before, after) -> bool:
    """True iff every buffer element that (extents, strides) does not address is bit-identical."""
    mask = np.zeros(before.shape[0], dtype=bool)
    W.strided_view(mask, p.D)[...] = True
    return bool(np.array_equal(before[~mask].view(np.uint8), after[~mask].view(np.uint8)))


def random_problem(rng: np.random.Generator, dtype="f64", max_group=2, max_extent=4, allow_neg=False,
                   pad=True, min_k=0, name="rand", isolated=False) -> W.Problem:
    """A random valid Case-1/2 problem: random numbers of H, M, N, K labels, random extents,
    random label order per tensor, random memory order, optional padding / negative strides.
    isolated: also labels that live in A only, in B only (Case 4) and in D only (Case 5)."""
    while True:
        nh, nm, nn = (int(rng.integers(0, max_group + 1)) for _ in range(3))
        nk = int(rng.integers(min_k, max_group + 1))
        if nh + nm + nn + nk > 0:
            break
    H = ["h%d" % i for i in range(nh)]
    M = ["m%d" % i for i in range(nm)]
    N = ["n%d" % i for i in range(nn)]
    K = ["k%d" % i for i in range(nk)]
    IA = ["x%d" % i for i in range(int(rng.integers(0, 3)))] if isolated else []
    IB = ["y%d" % i for i in range(int(rng.integers(0, 3)))] if isolated else []
    IC = ["z%d" % i for i in range(int(rng.integers(0, 2)))] if isolated else []
    ext = {l: int(rng.integers(1, max_extent + 1)) for l in H + M + N + K + IA + IB + IC}

    def layout(labels):
        labels = list(labels)
        rng.shuffle(labels)
        order = list(labels)
        rng.shuffle(order)
        strides, run = {}, 1
        for l in order:
            if pad and rng.random() < 0.3:
                run *= int(rng.integers(2, 4))
            strides[l] = run
            run *= ext[l]
        if allow_neg:
            for l in order:
                if rng.random() < 0.4:
                    strides[l] = -strides[l]
        return W.tensor(labels, ext, strides=strides)

    A, B, D = layout(H + M + K + IA), layout(H + N + K + IB), layout(H + M + N + IC)
    cplx = dtype in ("c128", "c64")
    alpha = complex(rng.integers(-2, 3), rng.integers(-2, 3) if cplx else 0) or 1.0
    beta = complex(rng.integers(-2, 3), rng.integers(-2, 3) if cplx else 0)
    if not cplx:
        alpha, beta = alpha.real, beta.real
    return W.Problem(name, dtype, A, B, D, alpha=alpha, beta=beta,
                     opA=int(rng.integers(0, 2)), opB=int(rng.integers(0, 2)), opC=int(rng.integers(0, 2)),
                     seed=int(rng.integers(1, 1 << 30)))
