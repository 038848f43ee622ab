"""Pins of the CPU oracle against things other than itself (no GPU needed).

What each group fixes is stated at its head.  The paper prints no numeric worked example,
so the pins are: exact rational brute force on tiny tensors, numpy.einsum as an
independent library evaluation, closed forms (all-ones, one-hot), invariants of the
definition, and agreement of the three evaluation orders within the rounding bound.
"""
import dataclasses
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads as W
from helpers import UNIT_ROUNDOFF, desc, gaps_untouched, normalised_error, random_problem, run_oracle, values_of

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------------------
# an evaluator that shares nothing with the oracle: exact rationals, scatter into a dict
# --------------------------------------------------------------------------------------
def _frac(z):
    z = complex(z)
    return (Fraction(z.real), Fraction(z.imag))


def _cmul(x, y):
    return (x[0] * y[0] - x[1] * y[1], x[0] * y[1] + x[1] * y[0])


def _cadd(x, y):
    return (x[0] + y[0], x[1] + y[1])


def _conj(x, op):
    return (x[0], -x[1]) if op else x


def brute_exact(p: W.Problem, bufA, bufB, bufC):
    """Exact D as {D index tuple: (Fraction re, Fraction im)}: one pass over the whole index
    space of all distinct labels, each term scattered to its D entry (Eq. case2, read as
    "for every assignment of the labels")."""
    vA, vB, vC = values_of(p, bufA, p.A), values_of(p, bufB, p.B), values_of(p, bufC, p.D)
    ext = p.extent_of()
    labels = sorted(ext)
    out = {}
    for assign in itertools.product(*[range(ext[l]) for l in labels]):
        at = dict(zip(labels, assign))
        a = _conj(_frac(vA[tuple(at[l] for l in p.A.labels)]), p.opA)
        b = _conj(_frac(vB[tuple(at[l] for l in p.B.labels)]), p.opB)
        key = tuple(at[l] for l in p.D.labels)
        out[key] = _cadd(out.get(key, (Fraction(0), Fraction(0))), _cmul(a, b))
    al, be = _frac(p.alpha), _frac(p.beta)
    res = {}
    for key, acc in out.items():
        d = _cmul(al, acc)
        if p.beta != 0:
            d = _cadd(d, _cmul(be, _conj(_frac(vC[key]), p.opC)))
        res[key] = d
    return res


def _as_complex(x):
    return complex(float(x[0]), float(x[1]))      # float(Fraction) rounds correctly, once


# ---- P1: brute force on tiny tensors --------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32", "c128", "c64", "f16"])
@pytest.mark.parametrize("seed", range(12))
def test_brute_force_integer_inputs_exact(dtype, seed):
    """Integer-valued inputs: every partial sum is exactly representable, so the oracle (all
    three evaluation orders) must equal the rational result bit for bit.  Fixes label
    classification, offsets, op, alpha/beta handling for arbitrary label patterns."""
    rng = np.random.default_rng(1000 + seed)
    p = random_problem(rng, dtype, allow_neg=(seed % 2 == 1))
    a, b, c = W.make_operands(p, "ints")
    exact = brute_exact(p, a, b, c)
    for mode in (oracle.MODE_TRUTH, oracle.MODE_TIMED, oracle.MODE_LITERAL):
        d, _ = run_oracle(p, a, b, c, mode)
        v = W.strided_view(d, p.D)
        for key, val in exact.items():
            assert complex(v[key]) == _as_complex(val), (p, key, mode)
        assert gaps_untouched(p, c, d)


@pytest.mark.parametrize("dtype", ["f64", "c128"])
@pytest.mark.parametrize("seed", range(8))
def test_brute_force_uniform_inputs_one_rounding(dtype, seed):
    """Uniform inputs: the long-double truth must sit within one storage rounding (plus the
    80-bit accumulation error) of the exact rational value."""
    rng = np.random.default_rng(2000 + seed)
    p = random_problem(rng, dtype, max_extent=3)
    a, b, c = W.make_operands(p, "uniform")
    exact = brute_exact(p, a, b, c)
    d, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    v, s = W.strided_view(d, p.D), W.strided_view(S, p.D)
    vc = W.strided_view(c, p.D)
    for key, val in exact.items():
        ref = _as_complex(val)
        scale = abs(p.alpha) * s[key] + abs(p.beta) * abs(vc[key])
        assert abs(complex(v[key]) - ref) <= 2.0 ** -52 * abs(ref) + 2.0 ** -58 * scale + 1e-300


# ---- 16-bit storage: the oracle's own conversions, pinned to numpy's float16 ----------------
def test_half_to_double_on_every_bit_pattern():
    """All 65 536 patterns: zeros, subnormals, normals, infinities, NaNs."""
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    for b in range(65536):
        got = oracle.half_to_double(b)
        if np.isnan(ref[b]):
            assert np.isnan(got)
        else:
            assert got == ref[b] and np.signbit(got) == np.signbit(ref[b]), hex(b)


def test_half_from_double_rounds_to_nearest_even():
    """numpy converts float64 to float16 with one correct rounding: random doubles over the whole
    range (normal, subnormal, overflowing), every midpoint between neighbouring 16-bit values
    (ties go to the even neighbour), and the values just beside those midpoints."""
    rng = np.random.default_rng(16)
    xs = [0.0, -0.0, 65504.0, 65519.999, 65520.0, 65536.0, 1e6, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * (1 + 2.0 ** -40), 3 * 2.0 ** -25,
          2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -40, float("inf")]
    xs += list(rng.uniform(-1, 1, 2000) * 10.0 ** rng.integers(-9, 6, 2000))
    pos = np.arange(0, 0x7c00, dtype=np.uint16).view(np.float16).astype(np.float64)      # every finite non-negative value
    mid = (pos[:-1] + pos[1:]) / 2                                                       # exact in float64
    xs += list(mid[::7]) + list(np.nextafter(mid[::11], np.inf)) + list(np.nextafter(mid[::13], -np.inf))
    with np.errstate(over="ignore"):
        for x in xs:
            for v in (x, -x):
                want = int(np.array([v], dtype=np.float64).astype(np.float16).view(np.uint16)[0])
                assert oracle.half_from_double(v) == want, (v, hex(want))


def test_f16_uniform_inputs_round_once():
    """float16 tensors with uniform entries (multiples of 2^-10) and a handful of terms: every
    product and sum is exact in any wider type, so the truth is the exact rational result rounded
    ONCE to 16 bits, and the storage-type evaluation orders differ from it by their own roundings
    only (timed: float sums, exact here as well)."""
    for seed in range(8):
        rng = np.random.default_rng(2600 + seed)
        p = random_problem(rng, "f16", max_extent=3)
        p = dataclasses.replace(p, alpha=0.5, beta=-2.0)
        a, b, c = W.make_operands(p, "uniform")
        exact = brute_exact(p, a, b, c)
        for mode in (oracle.MODE_TRUTH, oracle.MODE_TIMED):
            d, _ = run_oracle(p, a, b, c, mode)
            v = W.strided_view(d, p.D)
            for key, val in exact.items():
                want = np.float16(float(val[0]))          # float(Fraction) is exact here (few terms of 20-bit products)
                assert v[key] == want, (p, key, mode, v[key], want)


# ---- bfloat16 storage: pinned to the format's definition (the upper half of a binary32) -------
def test_bfloat16_to_double_on_every_bit_pattern():
    with np.errstate(invalid="ignore"):
        ref = W.bf16_values(np.arange(65536, dtype=np.uint16)).astype(np.float64)
    for b in range(65536):
        got = oracle.bfloat16_to_double(b)
        if np.isnan(ref[b]):
            assert np.isnan(got)
        else:
            assert got == ref[b] and np.signbit(got) == np.signbit(ref[b]), hex(b)


def _nearest_bfloat16(x: float) -> int:
    """Round to nearest, ties to the even bit pattern, by exact rational comparison with the
    two neighbouring values out of the table of all finite ones; past the midpoint between the
    largest value and 2^128: infinity."""
    pos = W.bf16_values(np.arange(0, 0x7f80, dtype=np.uint16)).astype(np.float64)
    sign, a = (0x8000 if np.signbit(x) else 0), abs(x)
    if a == float("inf"):
        return sign | 0x7f80
    hi = int(np.searchsorted(pos, a, side="left"))          # first value >= a
    if hi < len(pos) and pos[hi] == a:
        return sign | hi
    lo = hi - 1
    top = Fraction(float(pos[hi])) if hi < len(pos) else Fraction(2) ** 128
    dl, dh = Fraction(a) - Fraction(float(pos[lo])), top - Fraction(a)
    pick = lo if dl < dh else hi if dh < dl else (lo if lo % 2 == 0 else hi)
    return sign | pick          # pick == 0x7f80 is the pattern of infinity


def test_bfloat16_from_double_rounds_to_nearest_even():
    """Random doubles over the whole range (normal, subnormal, overflowing), every 5th midpoint
    between neighbouring values (ties to even) and the doubles just beside midpoints; and, on
    float32 inputs, torch's own float32 -> bfloat16 conversion."""
    import torch
    rng = np.random.default_rng(17)
    big = float(W.bf16_values(np.array([0x7f7f], dtype=np.uint16))[0])
    xs = [0.0, -0.0, big, big * (1 + 2.0 ** -9), big * (1 + 2.0 ** -8), 2.0 ** 128, 1e39, 2.0 ** -133, 2.0 ** -134, 2.0 ** -134 * (1 + 2.0 ** -40),
          3 * 2.0 ** -134, 2.0 ** -126, 2.0 ** -126 - 2.0 ** -134, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -40, float("inf")]
    xs += list(rng.uniform(-1, 1, 2000) * 10.0 ** rng.integers(-42, 39, 2000))
    pos = W.bf16_values(np.arange(0, 0x7f80, dtype=np.uint16)).astype(np.float64)
    mid = (pos[:-1] + pos[1:]) / 2
    xs += list(mid[::5]) + list(np.nextafter(mid[::11], np.inf)) + list(np.nextafter(mid[::13], -np.inf))
    for x in xs:
        for v in (float(x), -float(x)):
            assert oracle.bfloat16_from_double(v) == _nearest_bfloat16(v), v
    f = (rng.uniform(-1, 1, 4000) * 10.0 ** rng.integers(-40, 38, 4000)).astype(np.float32)
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for v, w in zip(f, want):
        assert oracle.bfloat16_from_double(float(v)) == int(w), v


@pytest.mark.parametrize("seed", range(10))
def test_bfloat16_brute_force(seed):
    """bfloat16 tensors (buffers of bit patterns).  Integer inputs: all three evaluation orders
    equal the rational result bit for bit.  Uniform inputs (multiples of 2^-7, a handful of
    terms: every product and sum exact in any wider type): the truth and the float-sum order are
    the exact result rounded ONCE to 8 significant bits."""
    rng = np.random.default_rng(2700 + seed)
    p = random_problem(rng, "bf16", allow_neg=(seed % 2 == 1))
    a, b, c = W.make_operands(p, "ints")
    exact = brute_exact(p, a, b, c)
    for mode in (oracle.MODE_TRUTH, oracle.MODE_TIMED, oracle.MODE_LITERAL):
        d, _ = run_oracle(p, a, b, c, mode)
        v = values_of(p, d, p.D)
        for key, val in exact.items():
            assert float(v[key]) == float(val[0]), (p, key, mode)
        assert gaps_untouched(p, c, d)
    p = dataclasses.replace(random_problem(rng, "bf16", max_extent=3), alpha=0.5, beta=-2.0)
    a, b, c = W.make_operands(p, "uniform")
    exact = brute_exact(p, a, b, c)
    for mode in (oracle.MODE_TRUTH, oracle.MODE_TIMED):
        d, _ = run_oracle(p, a, b, c, mode)
        v = W.strided_view(d, p.D)
        for key, val in exact.items():
            assert int(v[key]) == _nearest_bfloat16(float(val[0])), (p, key, mode)      # float(Fraction) exact: few terms of 16-bit products


def test_S_is_sum_of_moduli():
    """The normaliser returned by the truth mode is sum |a||b| (checked exactly on integers)."""
    rng = np.random.default_rng(5)
    p = random_problem(rng, "f64", min_k=1)
    a, b, c = W.make_operands(p, "ints")
    pa = W.Problem("abs", "f64", p.A, p.B, p.D, alpha=1.0, beta=0.0)
    d_abs, _ = run_oracle(pa, np.abs(a), np.abs(b), c)
    _, S = run_oracle(p, a, b, c, want_S=True)
    assert np.array_equal(W.strided_view(S, p.D), W.strided_view(d_abs, p.D))


# Gaussian integers whose moduli are integers (Pythagorean triples): |3+4i| = 5, |5+12i| = 13, ...
_PYTHAGOREAN = [(3, 4, 5), (5, 12, 13), (8, 15, 17), (7, 24, 25), (20, 21, 29), (12, 35, 37), (9, 40, 41)]


@pytest.mark.parametrize("mode", [oracle.MODE_TRUTH, oracle.MODE_TIMED], ids=["truth", "timed"])
@pytest.mark.parametrize("dtype", ["c128", "c64", "f64", "f32", "f16", "bf16"])
def test_normaliser_on_exact_moduli(dtype, mode):
    """S = sum_P |op(a)||op(b)| with the complex MODULUS (the error measure's denominator).
    Complex operands are drawn from Gaussian integers with integer moduli, in all sign, swap and
    conjugation variants, so S is an integer that plain integer arithmetic gives exactly; a
    squared norm, |re| + |im| or max(|re|, |im|) in place of the modulus gives another integer.
    Real operands are signed integers (modulus = absolute value)."""
    rng = np.random.default_rng(17 + len(dtype))
    ext = dict(h=2, m=3, n=4, k=5, l=3)
    A = W.tensor("mhkl", ext, memory_order="khlm")
    B = W.tensor("lnkh", ext)
    D = W.tensor("nhm", ext, strides=dict(n=2, h=8, m=-16))
    p = W.Problem("moduli", dtype, A, B, D, alpha=2.0, beta=0.5, opA=1, opB=0, opC=1)

    def draw(spec):
        """(buffer, integer moduli shaped like the tensor)."""
        buf = np.zeros(spec.size, dtype=p.np_dtype)
        mod = np.zeros(spec.extents, dtype=object)
        v = W.strided_view(buf, spec)
        for at in itertools.product(*[range(e) for e in spec.extents]):
            if dtype in ("c128", "c64"):
                x, y, r = _PYTHAGOREAN[int(rng.integers(len(_PYTHAGOREAN)))]
                if rng.random() < 0.5:
                    x, y = y, x
                v[at] = complex(x * int(rng.choice([-1, 1])), y * int(rng.choice([-1, 1])))
            else:
                r = int(rng.integers(0, 9))
                x = r * int(rng.choice([-1, 1]))
                v[at] = W.bf16_bits(np.float32(x)).reshape(())[()] if dtype == "bf16" else x
            mod[at] = r
        return buf, mod

    a, ma = draw(A)
    b, mb = draw(B)
    c = W.fill(D, 3, W.TAG_C, p.np_dtype, "ints")
    _, S = run_oracle(p, a, b, c, mode, want_S=True)
    vs = W.strided_view(S, D)
    for n, h, m in itertools.product(range(4), range(2), range(3)):
        expect = sum(ma[m, h, k, l] * mb[l, n, k, h] for k in range(5) for l in range(3))
        assert vs[n, h, m] == float(expect), (dtype, mode, (n, h, m))


# ---- P2: numpy.einsum as an independent library evaluation ----------------------------
def einsum_reference(p: W.Problem, bufA, bufB, bufC):
    letters = {}
    for t in (p.A, p.B, p.D):
        for l in t.labels:
            letters.setdefault(l, "abcdefghijklmnopqrstuvwxyzABCDEFGHIJKLMNOPQRSTUVWXYZ"[len(letters)])
    sub = lambda t: "".join(letters[l] for l in t.labels)
    hi = np.complex128 if p.dtype in ("c128", "c64") else np.float64
    vA = values_of(p, bufA, p.A).astype(hi)
    vB = values_of(p, bufB, p.B).astype(hi)
    vC = values_of(p, bufC, p.D).astype(hi)
    if p.opA:
        vA = np.conj(vA)
    if p.opB:
        vB = np.conj(vB)
    if p.opC:
        vC = np.conj(vC)
    out = p.alpha * np.einsum("%s,%s->%s" % (sub(p.A), sub(p.B), sub(p.D)), vA, vB)
    if p.beta != 0:
        out = out + p.beta * vC
    return out


@pytest.mark.parametrize("dtype", ["f64", "f32", "c128", "c64", "f16", "bf16"])
@pytest.mark.parametrize("seed", range(10))
def test_einsum_random_problems(dtype, seed):
    rng = np.random.default_rng(3000 + seed)
    p = random_problem(rng, dtype, max_group=3, max_extent=5, allow_neg=(seed % 3 == 0))
    a, b, c = W.make_operands(p)
    ref = einsum_reference(p, a, b, c)
    for mode in (oracle.MODE_TRUTH, oracle.MODE_TIMED, oracle.MODE_LITERAL):
        d, _ = run_oracle(p, a, b, c, mode)
        _, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
        k = p.sizes()[3]
        bound = (k + 4) * UNIT_ROUNDOFF[p.dtype] * (abs(p.alpha) * W.strided_view(S, p.D)
                                                    + abs(p.beta) * np.abs(values_of(p, c, p.D))) * 4
        assert np.all(np.abs(values_of(p, d, p.D) - ref) <= bound + 1e-300), (p, mode)


@pytest.mark.parametrize("p", W.configs_reduced(), ids=lambda p: p.name)
def test_einsum_reduced_configs(p):
    """The five benchmark label structures and layouts (reduced sizes) against einsum."""
    a, b, c = W.make_operands(p)
    ref = einsum_reference(p, a, b, c)
    d, S = run_oracle(p, a, b, c, want_S=True)
    k = p.sizes()[3]
    bound = (k + 4) * 2.0 ** -53 * (abs(p.alpha) * W.strided_view(S, p.D) + abs(p.beta) * np.abs(W.strided_view(c, p.D)))
    got = W.strided_view(d, p.D).astype(ref.dtype)
    slack = 2.0 ** -23 * np.abs(ref) if p.dtype == "f32" else 0.0       # storage rounding of the f32 result
    assert np.all(np.abs(got - ref) <= bound * 4 + slack + 1e-300)
    assert gaps_untouched(p, c, d)


def test_config2_is_a_column_major_gemm():
    """After grouping (a,b), (c,d), (i,j) config 2 is the plain matrix product of the
    column-major matrices V (|M| x |K|) and T (|K| x |N|)."""
    p = W.config2(v=12, o=5)
    a, b, c = W.make_operands(p)
    m, n, k = 144, 25, 144
    ref = a.reshape((m, k), order="F") @ b.reshape((k, n), order="F") + c.reshape((m, n), order="F")
    d, _ = run_oracle(p, a, b, c)
    assert np.allclose(d.reshape((m, n), order="F"), ref, rtol=0, atol=1e-12)


def test_config4_hslowest_is_batched_AhB():
    p = W.config4(h=4, n=9, h_slowest=True)
    a, b, c = W.make_operands(p)
    A3 = a.reshape((9, 9, 4), order="F")      # [k, i, h]
    B3 = b.reshape((9, 9, 4), order="F")      # [k, j, h]
    C3 = c.reshape((9, 9, 4), order="F")      # [i, j, h]
    d, _ = run_oracle(p, a, b, c)
    D3 = d.reshape((9, 9, 4), order="F")
    for h in range(4):
        assert np.allclose(D3[:, :, h], A3[:, :, h].conj().T @ B3[:, :, h] + 0.5 * C3[:, :, h], atol=1e-13)


# ---- the paper's symbolic examples (label strings only; it prints no values) -----------
def _paper_examples():
    rows = []
    with open(os.path.join(GOLDEN, "paper_label_examples.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                case, A, B, D, supported = line.split()
                rows.append((case, A, B, D, supported == "yes"))
    return rows


@pytest.mark.parametrize("row", _paper_examples(), ids=lambda r: r[0])
def test_paper_label_examples(row):
    case, la, lb, ld, supported = row
    ext = dict(a=3, b=4, g=2, d=5, e=2)       # alpha, beta, gamma, delta, epsilon
    p = W.Problem(case, "f64", _rep_tensor(la, ext), _rep_tensor(lb, ext), _rep_tensor(ld, ext), alpha=2.0, beta=-1.0)
    ids = W.label_ids(p)
    st = oracle.validate(desc(p.A, ids), desc(p.B, ids), desc(p.D, ids), desc(p.D, ids))
    assert st == oracle.V_OK              # also the cases the standard does not require (Note 7): their equations define the result
    a, b, c = W.make_operands(p, "ints")
    exact = brute_exact(p, a, b, c)
    d, _ = run_oracle(p, a, b, c)
    v = W.strided_view(d, p.D)
    for key, val in exact.items():
        assert complex(v[key]) == _as_complex(val)


def _rep_tensor(labels, ext):
    """Column-major tensor whose label string repeats a label (each position its own stride)."""
    strides, run = [], 1
    for l in labels:
        strides.append(run)
        run *= ext[l]
    e = tuple(ext[l] for l in labels)
    base, size = W.span_of(e, strides)
    return W.TensorSpec(tuple(labels), e, tuple(strides), base, size)


def test_repeated_label_equals_summed_stride():
    """Note 6: A[k,i,k] with strides (s0,s1,s2) is A'[k,i] with strides (s0+s2, s1)."""
    ext = dict(k=4, i=3, j=5)
    A3 = _rep_tensor("kik", ext)
    A2 = W.TensorSpec(("k", "i"), (4, 3), (A3.strides[0] + A3.strides[2], A3.strides[1]), 0, A3.size)
    B, D = W.tensor("kj", ext), W.tensor("ji", ext)
    p3 = W.Problem("rep", "f64", A3, B, D, alpha=1.5, beta=0.25)
    p2 = W.Problem("sum", "f64", A2, B, D, alpha=1.5, beta=0.25)
    a, b, c = W.make_operands(p3)
    d3, _ = run_oracle(p3, a, b, c)
    d2, _ = run_oracle(p2, a, b, c)
    assert np.array_equal(d3, d2)
    # and against einsum's own diagonal handling
    ref = 1.5 * np.einsum("kik,kj->ji", a.reshape((4, 3, 4), order="F"), b.reshape((4, 5), order="F")) \
        + 0.25 * c.reshape((5, 3), order="F")
    assert np.allclose(d3.reshape((5, 3), order="F"), ref, atol=1e-14)


# ---- P3: all-ones closed form ----------------------------------------------------------
@pytest.mark.parametrize("p", W.configs_reduced(), ids=lambda p: p.name)
def test_all_ones_gives_product_of_contracted_extents(p):
    """A = B = 1  =>  every D element is alpha*|K| + beta*op(c), exactly when alpha, beta
    are powers of two."""
    p = W.Problem(p.name, p.dtype, p.A, p.B, p.D, alpha=2.0, beta=0.5, opA=p.opA, opB=p.opB, opC=p.opC, seed=p.seed)
    a = W.fill(p.A, 0, 0, p.np_dtype, "ones")
    b = W.fill(p.B, 0, 0, p.np_dtype, "ones")
    c = W.fill(p.D, p.seed, W.TAG_C, p.np_dtype, "ints")
    K = p.sizes()[3]
    for mode in (oracle.MODE_TRUTH, oracle.MODE_TIMED, oracle.MODE_LITERAL):
        d, _ = run_oracle(p, a, b, c, mode)
        vc = W.strided_view(c, p.D)
        expect = 2.0 * K + 0.5 * (np.conj(vc) if p.opC else vc)
        assert np.array_equal(W.strided_view(d, p.D), expect.astype(p.np_dtype))


def test_all_ones_config1_value():
    """Config 1 at full size with its own scalars: 1.3*576 + 0.7*c (one rounding)."""
    p = W.config1()
    a = W.fill(p.A, 0, 0, p.np_dtype, "ones")
    b = W.fill(p.B, 0, 0, p.np_dtype, "ones")
    c = W.fill(p.D, p.seed, W.TAG_C, p.np_dtype)
    idx = np.array([0, 1, 577, 331775, 100000])
    # evaluate a handful of elements only (the full loop nest takes seconds; see the gpu tests)
    sub = W.Problem("sub", "f64", p.A, p.B, p.D, alpha=1.3, beta=0.7)
    d, _ = run_oracle(sub, a, b, c)
    expect = np.longdouble(1.3) * 576 + np.longdouble(0.7) * c.astype(np.longdouble)
    assert np.array_equal(d[idx], expect.astype(np.float64)[idx])
    assert np.array_equal(d, expect.astype(np.float64))


# ---- P4: one-hot operand => pure gather / permutation, bit exact -----------------------
@pytest.mark.parametrize("dtype", ["f64", "f32", "c128", "c64", "f16", "bf16"])
def test_delta_operand_reproduces_permutation(dtype):
    """B[k..., n...] = prod delta(k_i, n_i)  =>  D[m..., n...] = A[m..., k... = n...]: each
    sum has exactly one non-zero term, so D is a bit-exact re-layout of A."""
    ext = dict(m0=3, m1=4, k0=5, k1=2, n0=5, n1=2)
    A = W.tensor(["m0", "k1", "m1", "k0"], ext, memory_order=["k0", "m1", "m0", "k1"])
    B = W.tensor(["n1", "k0", "k1", "n0"], ext)
    D = W.tensor(["n0", "m1", "n1", "m0"], ext, memory_order=["m0", "n1", "n0", "m1"])
    p = W.Problem("delta", dtype, A, B, D, alpha=1.0, beta=0.0)
    a = W.fill(p.A, 11, 0, p.np_dtype)
    b = np.zeros(B.size, dtype=p.np_dtype)
    vb = W.strided_view(b, B)
    for k0 in range(5):
        for k1 in range(2):
            vb[k1, k0, k1, k0] = 0x3f80 if dtype == "bf16" else 1.0
    c = np.full(D.size, 0x7fc0 if dtype == "bf16" else np.nan, dtype=p.np_dtype)          # NaN; beta == 0: never read
    d, _ = run_oracle(p, a, b, c)
    vA, vD = W.strided_view(a, A), W.strided_view(d, D)
    for m0, m1, k0, k1 in itertools.product(range(3), range(4), range(5), range(2)):
        assert vD[k0, m1, k1, m0].tobytes() == vA[m0, k1, m1, k0].tobytes()


# ---- P6: invariants ---------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(6))
def test_relabelling_and_mode_permutation_leave_D_unchanged(seed):
    rng = np.random.default_rng(4000 + seed)
    p = random_problem(rng, "f64", max_group=2, max_extent=4, min_k=1)
    a, b, c = W.make_operands(p)
    d0, _ = run_oracle(p, a, b, c)

    # (i) a bijection on the labels
    ren = {l: "z" + l for l in p.extent_of()}
    rn = lambda t: W.TensorSpec(tuple(ren[l] for l in t.labels), t.extents, t.strides, t.base, t.size)
    p1 = W.Problem("ren", p.dtype, rn(p.A), rn(p.B), rn(p.D), p.alpha, p.beta, p.opA, p.opB, p.opC)
    d1, _ = run_oracle(p1, a, b, c)
    assert np.array_equal(d0, d1)

    # (ii) permute (label, extent, stride) triples of each tensor together: same memory, same D.
    #      Summation order may change with A's label order, so compare within rounding.
    def perm(t):
        o = rng.permutation(len(t.labels))
        return W.TensorSpec(tuple(t.labels[i] for i in o), tuple(t.extents[i] for i in o),
                            tuple(t.strides[i] for i in o), t.base, t.size)
    p2 = W.Problem("perm", p.dtype, perm(p.A), perm(p.B), perm(p.D), p.alpha, p.beta, p.opA, p.opB, p.opC)
    d2, S = run_oracle(p2, a, b, c, want_S=True)
    assert normalised_error(p, d2, d0, S, c) <= 4 * 2.0 ** -53

    # (iii) commutativity: swap (A, opA) with (B, opB)
    p3 = W.Problem("swap", p.dtype, p.B, p.A, p.D, p.alpha, p.beta, p.opB, p.opA, p.opC)
    d3, _ = run_oracle(p3, b, a, c)
    assert np.array_equal(d0, d3)


def test_permuting_D_labels_with_memory_order_gives_permuted_values():
    """Writing D's labels in another order with column-major strides of that order yields the
    transposed array (the appendix's 'changing around the indices for D')."""
    ext = dict(a=3, b=4, c=5, k=6)
    A, B = W.tensor("ak", ext), W.tensor("kbc", ext)
    p0 = W.Problem("d0", "f64", A, B, W.tensor("abc", ext), alpha=1.0, beta=0.0)
    p1 = W.Problem("d1", "f64", A, B, W.tensor("cab", ext), alpha=1.0, beta=0.0)
    a, b, _ = W.make_operands(p0)
    c = np.zeros(60)
    d0, _ = run_oracle(p0, a, b, c)
    d1, _ = run_oracle(p1, a, b, c)
    assert np.array_equal(d0.reshape((3, 4, 5), order="F").transpose(2, 0, 1), d1.reshape((5, 3, 4), order="F"))
    assert not np.array_equal(d0, d1)


@pytest.mark.parametrize("dtype", ["f64", "c128", "c64"])
def test_linearity_in_alpha_and_beta(dtype):
    rng = np.random.default_rng(77)
    p = random_problem(rng, dtype, max_group=2, max_extent=4, min_k=1)
    a, b, c = W.make_operands(p)
    al, be = (0.75 - 0.5j, -1.25 + 2j) if dtype != "f64" else (0.75, -1.25)
    d, S = run_oracle(p, a, b, c, want_S=True, alpha=al, beta=be)
    d10, _ = run_oracle(p, a, b, c, alpha=1.0, beta=0.0)
    d01, _ = run_oracle(p, a, b, c, alpha=0.0, beta=1.0)
    combo = (al * d10 + be * d01).astype(p.np_dtype)
    assert normalised_error(p, combo, d, S, c, alpha=al, beta=be) <= 8 * UNIT_ROUNDOFF[dtype]
    # alpha = 0, beta = 1 returns op(C) exactly
    vc = W.strided_view(c, p.D)
    assert np.array_equal(W.strided_view(d01, p.D), np.conj(vc) if p.opC else vc)


def test_conjugation_symmetry_and_op_equals_preconjugated_copy():
    rng = np.random.default_rng(99)
    p = random_problem(rng, "c128", max_group=2, max_extent=4, min_k=1)
    a, b, c = W.make_operands(p)
    al, be = 0.5 + 1.5j, -0.25 + 0.75j
    d, _ = run_oracle(p, a, b, c, alpha=al, beta=be)
    dc, _ = run_oracle(p, np.conj(a), np.conj(b), np.conj(c), alpha=np.conj(al), beta=np.conj(be))
    mask = np.zeros(c.shape[0], dtype=bool)
    W.strided_view(mask, p.D)[...] = True
    assert np.array_equal(np.conj(d)[mask], dc[mask])
    # opA = conj on A  ==  identity on a conjugated copy, bit for bit
    pc = W.Problem("c", "c128", p.A, p.B, p.D, opA=1, opB=0, opC=1)
    pi = W.Problem("i", "c128", p.A, p.B, p.D, opA=0, opB=0, opC=0)
    d1, _ = run_oracle(pc, a, b, c, alpha=al, beta=be)
    d2, _ = run_oracle(pi, np.conj(a), b, np.conj(c), alpha=al, beta=be)
    assert np.array_equal(d1[mask], d2[mask])
    # and conj really changes the answer
    d3, _ = run_oracle(pi, a, b, c, alpha=al, beta=be)
    assert not np.array_equal(d1[mask], d3[mask])


def test_conj_on_real_dtype_is_identity():
    rng = np.random.default_rng(3)
    p = random_problem(rng, "f64", min_k=1)
    a, b, c = W.make_operands(p)
    p0 = W.Problem("i", "f64", p.A, p.B, p.D, p.alpha, p.beta, 0, 0, 0)
    p1 = W.Problem("c", "f64", p.A, p.B, p.D, p.alpha, p.beta, 1, 1, 1)
    assert np.array_equal(run_oracle(p0, a, b, c)[0], run_oracle(p1, a, b, c)[0])


# ---- P9: the three evaluation orders agree within the rounding bound --------------------
@pytest.mark.parametrize("p", W.configs_reduced(), ids=lambda p: p.name)
def test_three_modes_agree(p):
    a, b, c = W.make_operands(p)
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    k = p.sizes()[3]
    for mode in (oracle.MODE_TIMED, oracle.MODE_LITERAL):
        d, _ = run_oracle(p, a, b, c, mode)
        assert normalised_error(p, d, truth, S, c) <= (k + 2) * UNIT_ROUNDOFF[p.dtype] * 2


# ---- beta == 0 / alpha == 0 never read ---------------------------------------------------
def test_beta_zero_does_not_read_C_and_alpha_zero_does_not_read_AB():
    ext = dict(m=3, n=4, k=5)
    p = W.Problem("b0", "f64", W.tensor("mk", ext), W.tensor("kn", ext), W.tensor("mn", ext), alpha=1.0, beta=0.0)
    a, b, _ = W.make_operands(p)
    c = np.full(12, np.nan)
    d, _ = run_oracle(p, a, b, c)
    assert np.all(np.isfinite(d))
    d, _ = run_oracle(p, np.full(15, np.nan), np.full(20, np.inf), np.ones(12), alpha=0.0, beta=2.0)
    assert np.array_equal(d, np.full(12, 2.0))


# ---- degenerate shapes (Note 4; appendix tests 6, 7, 8, 9) -------------------------------
def test_degenerate_shapes():
    ext = dict(m=3, n=4, k=5)
    # outer product: no contracted label
    p = W.Problem("outer", "f64", W.tensor("m", ext), W.tensor("n", ext), W.tensor("mn", ext), alpha=1.0)
    a, b, c = W.make_operands(p)
    d, _ = run_oracle(p, a, b, c)
    assert np.array_equal(d.reshape((3, 4), order="F"), np.outer(a, b))
    # everything contracted: D has rank zero
    p = W.Problem("dot", "f64", W.tensor("k", ext), W.tensor("k", ext), W.tensor("", ext), alpha=1.0)
    a, b, c = W.make_operands(p, "ints")
    d, _ = run_oracle(p, a, b, c)
    assert d.shape == (1,) and d[0] == float(np.dot(a, b))
    # rank-zero A: scaling of B
    p = W.Problem("scale", "f64", W.tensor("", ext), W.tensor("n", ext), W.tensor("n", ext), alpha=1.0)
    a, b, c = W.make_operands(p, "ints")
    d, _ = run_oracle(p, a, b, c)
    assert np.array_equal(d, a[0] * b)
    # pure Hadamard product
    p = W.Problem("had", "f64", W.tensor("mn", ext), W.tensor("nm", ext), W.tensor("mn", ext), alpha=1.0)
    a, b, c = W.make_operands(p, "ints")
    d, _ = run_oracle(p, a, b, c)
    assert np.array_equal(d.reshape((3, 4), order="F"), a.reshape((3, 4), order="F") * b.reshape((4, 3), order="F").T)


# ---- validation (appendix tests 26-28, Eq. FreeD, Note 7) --------------------------------
def test_validation_classes():
    ext = dict(m=3, n=4, k=5, x=2)
    ids = dict(m=1, n=2, k=3, x=4)
    t = lambda labels, **kw: desc(W.tensor(labels, ext, **kw), ids)
    A, B, D = t("mk"), t("kn"), t("mn")
    assert oracle.validate(A, B, D, D) == oracle.V_OK
    bad = ([3, 6], [1, 3], [1, 3])                                    # k has extent 6 in A
    assert oracle.validate(bad, B, D, D) == oracle.V_EXTENT_MISMATCH
    assert oracle.validate(A, B, t("nm"), D) == oracle.V_CD_MISMATCH    # C transposed in memory
    assert oracle.validate(A, B, t("nm", strides=dict(m=1, n=3)), D) == oracle.V_OK   # same layout, modes listed in another order
    assert oracle.validate(A, B, t("mn", strides=dict(m=1, n=4)), D) == oracle.V_CD_MISMATCH
    assert oracle.validate(A, B, t("mn", strides=dict(m=1, n=2)), t("mn", strides=dict(m=1, n=2))) == oracle.V_D_ALIASING
    assert oracle.validate(A, B, t("mn", strides=dict(m=0, n=1)), t("mn", strides=dict(m=0, n=1))) == oracle.V_D_ALIASING
    assert oracle.validate(t("mkx"), B, D, D) == oracle.V_OK            # Case 4: x is summed inside A
    assert oracle.validate(A, B, t("mnx"), t("mnx")) == oracle.V_OK        # Case 5: x broadcasts
    assert oracle.validate(([0, 5], [1, 1], [1, 3]), B, D, D) == oracle.V_BAD_ARG


def test_config3_literal_stride_reading_aliases():
    """'a=1, b=37, c=2' (unit-stride a AND stride 2 in c) collides: (a=2,c=0) and (a=0,c=1)."""
    ext = dict(a=37, b=53, c=61)
    ids = dict(a=1, b=2, c=3, d=4, e=5)
    D = desc(W.tensor("abc", ext, strides=dict(a=1, b=37, c=2)), ids)
    p = W.config3()
    A, B = desc(p.A, W.label_ids(p)), desc(p.B, W.label_ids(p))
    lab = W.label_ids(p)
    D = (D[0], D[1], [lab[l] for l in "abc"])
    assert oracle.validate(A, B, D, D) == oracle.V_D_ALIASING
    Dok = desc(p.D, lab)
    assert oracle.validate(A, B, Dok, Dok) == oracle.V_OK


# ---- Cases 4 and 5: reductions inside A, B and broadcast into D ------------------------------
@pytest.mark.parametrize("dtype", ["f64", "c128", "f32"])
@pytest.mark.parametrize("seed", range(10))
def test_isolated_labels_brute_force(dtype, seed):
    """Labels in A only or in B only are summed inside that tensor before the product, labels in D
    only repeat the product (Secs. "Case 4", "Case 5").  The rational evaluator sums A * B over
    every assignment of ALL labels and scatters to D's entry, which equals the sum of products of
    the reduced operands by distributivity: an independent form of the same definition.  Integer
    inputs, exact in all three evaluation orders."""
    rng = np.random.default_rng(7000 + seed)
    p = random_problem(rng, dtype, allow_neg=(seed % 2 == 1), isolated=True)
    a, b, c = W.make_operands(p, "ints")
    exact = brute_exact(p, a, b, c)
    for mode in (oracle.MODE_TRUTH, oracle.MODE_TIMED, oracle.MODE_LITERAL):
        d, _ = run_oracle(p, a, b, c, mode)
        v = W.strided_view(d, p.D)
        for key, val in exact.items():
            assert complex(v[key]) == _as_complex(val), (p, key, mode)


def test_case4_example_is_a_reduction_then_a_contraction():
    """The paper's Case 4 example D[d,a] = A[b,a,b] B[b,g,d,g,a] + C[d,a]: summing B's diagonal over
    g first and contracting the result is the same computation; einsum agrees."""
    ext = dict(a=3, b=4, g=2, d=5)
    A, B, D = _rep_tensor("bab", ext), _rep_tensor("bgdga", ext), _rep_tensor("da", ext)
    p = W.Problem("case4", "f64", A, B, D, alpha=2.0, beta=-1.0)
    a, b, c = W.make_operands(p, "ints")
    d, S = run_oracle(p, a, b, c, want_S=True)
    va, vb = W.strided_view(a, A), W.strided_view(b, B)
    ref = 2.0 * np.einsum("bab,bgdga->da", va, vb) - c.reshape((5, 3), order="F")
    assert np.array_equal(d.reshape((5, 3), order="F"), ref)
    # the normaliser: sum over b of (|A[b,a,b]|) (sum over g |B[b,g,d,g,a]|)
    refS = np.einsum("bab,bgdga->da", np.abs(va), np.abs(vb))
    assert np.array_equal(S.reshape((5, 3), order="F"), refS)


def test_case5_broadcasts_the_product():
    ext = dict(m=3, n=4, k=5, x=6)
    p = W.Problem("case5", "f64", W.tensor("mk", ext), W.tensor("kn", ext), W.tensor("mxn", ext), alpha=1.0, beta=0.5)
    a, b, c = W.make_operands(p, "ints")
    d, _ = run_oracle(p, a, b, c)
    prod = a.reshape((3, 5), order="F") @ b.reshape((5, 4), order="F")
    D3, C3 = d.reshape((3, 6, 4), order="F"), c.reshape((3, 6, 4), order="F")
    for x in range(6):
        assert np.array_equal(D3[:, x, :], prod + 0.5 * C3[:, x, :])
