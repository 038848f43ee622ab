"""Parity of the HIP paths with the CPU oracle, element by element, through the C-ABI.

Tolerance (stated by the benchmark spec): max over D of |d_gpu - d_truth| / (|alpha| sum|a||b| + |beta||c|)
<= 1e-12 (fp64, complex128), 1e-5 (fp32).  Integer-valued and permutation-only cases must
match bit for bit."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import TOLERANCE, TOLERANCE_WIDENED, gaps_untouched, normalised_error, random_problem, run_oracle, values_of

pytestmark = pytest.mark.gpu

GENERIC, GETT, STREAM = 0, 1, 2
REFUSED = 19                                        # TCX_ERR_PLAN_REFUSED


TWO_PHASE = {False: (0, 10, 11), True: (7, 8)}    # tile shapes served by the two-phase kernels (real, complex); 8: batch lanes
NUM_SHAPES = {False: 12, True: 9}
COMPLEX = ("c128", "c64")


def _paths_for(p):
    from gpu_helpers import DT  # noqa: F401
    paths = [(GENERIC, None)]
    paths += [(GETT, v) for v in range(7 if p.dtype == "c64" else NUM_SHAPES[p.dtype in COMPLEX])]      # complex64: no two-phase shapes
    if p.sizes()[3] <= 64:
        paths.append((STREAM, None))
    return paths


# Plans that a forced path declined, per test: a sweep over paths and shapes must not turn green
# because the planner refused everything.
_TALLY = {"ran": 0, "declined": 0}


@pytest.fixture(autouse=True)
def _declined_plans_stay_a_minority():
    _TALLY["ran"] = _TALLY["declined"] = 0
    yield
    total = _TALLY["ran"] + _TALLY["declined"]
    if total:
        assert _TALLY["ran"] >= max(1, (3 * total + 4) // 5), "only %d of %d forced plans ran" % (_TALLY["ran"], total)


def _check(p, a, b, c, path, variant, exact=False, truth=None, S=None, split_k=None):
    from gpu_helpers import run_gpu, say
    say("%s path=%s variant=%s split_k=%s exact=%s" % (p.name, path, variant, split_k, exact))
    if truth is None:
        truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    try:
        got = run_gpu(p, a, b, c, force_path=path, variant=variant, split_k=split_k)
    except Exception as exc:                       # the streaming path may decline large |K| (operand rows must fit LDS)
        if path == STREAM and getattr(exc, "code", None) == REFUSED and p.sizes()[3] > 8:
            say("  (streaming path declined: |K| = %d)" % p.sizes()[3])
            _TALLY["declined"] += p.sizes()[3] <= 64           # beyond 64 contracted terms it always declines: not counted
            return
        if path == GETT and variant in TWO_PHASE[p.dtype in COMPLEX] and getattr(exc, "code", None) == REFUSED:
            # the two-phase kernel needs |K| in whole slabs and slab-periodic k offsets
            say("  (two-phase kernel declined this plan)")
            _TALLY["declined"] += 1
            return
        raise
    _TALLY["ran"] += 1
    assert gaps_untouched(p, c, got), "elements outside (extents, strides) of D were modified"
    if exact:
        assert np.array_equal(W.strided_view(got, p.D), W.strided_view(truth, p.D))
    else:
        err = normalised_error(p, got, truth, S, c)
        assert err <= TOLERANCE[p.dtype], "normalised error %.3e" % err


@pytest.mark.parametrize("p", W.configs_reduced(), ids=lambda p: p.name)
def test_reduced_configs_all_paths(p):
    a, b, c = W.make_operands(p)
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    for path, variant in _paths_for(p):
        _check(p, a, b, c, path, variant, truth=truth, S=S)
        if path == GETT:            # the contracted range cut into parts, reduced by the second kernel
            _check(p, a, b, c, path, variant, truth=truth, S=S, split_k=2 + variant)
    # the plan's own choice
    _check(p, a, b, c, None, None, truth=truth, S=S)


@pytest.mark.parametrize("p", W.configs_reduced(), ids=lambda p: p.name)
def test_reduced_configs_integer_inputs_bit_exact(p):
    a, b, c = W.make_operands(p, "ints")
    p2 = W.Problem(p.name + "_ints", p.dtype, p.A, p.B, p.D, alpha=2.0, beta=(-1.0 if p.beta != 0 else 0.0),
                   opA=p.opA, opB=p.opB, opC=p.opC, seed=p.seed)
    truth, S = run_oracle(p2, a, b, c, oracle.MODE_TRUTH, want_S=True)
    for path, variant in _paths_for(p2) + [(None, None)]:
        _check(p2, a, b, c, path, variant, exact=True, truth=truth, S=S)
        if path == GETT:
            _check(p2, a, b, c, path, variant, exact=True, truth=truth, S=S, split_k=3)


@pytest.mark.parametrize("dtype", ["f64", "f32", "c128", "c64"])
def test_random_problems(dtype):
    rng = np.random.default_rng(31337)
    for i in range(40):
        p = random_problem(rng, dtype, max_group=3, max_extent=6, allow_neg=(i % 3 == 0), name="rand%d_%s" % (i, dtype))
        a, b, c = W.make_operands(p)
        truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
        paths = [(GENERIC, None), (GETT, (1 + i % 6) if dtype in COMPLEX else (2 + i % 7)), (STREAM, None)]
        for path, variant in paths:
            _check(p, a, b, c, path, variant, truth=truth, S=S)
        _check(p, a, b, c, GETT, paths[1][1], truth=truth, S=S, split_k=2 + i % 3)


@pytest.mark.parametrize("dtype", ["f64", "f32", "c128", "c64"])
def test_one_hot_operand_is_a_bit_exact_permutation(dtype):
    ext = dict(m0=7, m1=9, k0=11, k1=5, n0=11, n1=5)
    A = W.tensor(["m0", "k1", "m1", "k0"], ext, memory_order=["k0", "m1", "m0", "k1"])
    B = W.tensor(["n1", "k0", "k1", "n0"], ext)
    D = W.tensor(["n0", "m1", "n1", "m0"], ext, memory_order=["m0", "n1", "n0", "m1"])
    p = W.Problem("delta_" + dtype, dtype, A, B, D, alpha=1.0, beta=0.0)
    a = W.fill(p.A, 11, 0, p.np_dtype)
    b = np.zeros(B.size, dtype=p.np_dtype)
    vb = W.strided_view(b, B)
    for k0 in range(11):
        for k1 in range(5):
            vb[k1, k0, k1, k0] = 1.0
    c = np.full(D.size, np.nan, dtype=p.np_dtype)
    for path, variant in _paths_for(p):
        _check(p, a, b, c, path, variant, exact=True)


@pytest.mark.parametrize("p", W.low_intensity_shapes(full=False), ids=lambda p: p.name)
def test_low_intensity_shapes_all_paths(p):
    """Outer product, one-label contraction, Hadamard products, tiny-K batched: the streaming
    path, the tiled path and the generic path against the oracle; bit-exact on integer inputs."""
    a, b, c = W.make_operands(p)
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    for path, variant in [(GENERIC, None), (GETT, None), (STREAM, None), (STREAM, 0), (None, None)]:
        _check(p, a, b, c, path, variant, truth=truth, S=S)
    a, b, c = W.make_operands(p, "ints")
    p2 = W.Problem(p.name + "_ints", p.dtype, p.A, p.B, p.D, alpha=-2.0, beta=(4.0 if p.beta != 0 else 0.0),
                   opA=p.opA, opB=p.opB, opC=p.opC, seed=p.seed)
    truth, S = run_oracle(p2, a, b, c, oracle.MODE_TRUTH, want_S=True)
    for path, variant in ((GETT, None), (STREAM, None), (STREAM, 0)):
        _check(p2, a, b, c, path, variant, exact=True, truth=truth, S=S)


def _matrix_product(m, n, k, a_k_fast, b_k_fast, d_n_fast, dtype):
    e = {"m": m, "n": n, "k": k}
    A = W.tensor(["m", "k"], e, memory_order=["k", "m"] if a_k_fast else ["m", "k"])
    B = W.tensor(["k", "n"], e, memory_order=["k", "n"] if b_k_fast else ["n", "k"])
    D = W.tensor(["m", "n"], e, memory_order=["n", "m"] if d_n_fast else ["m", "n"])
    return W.Problem("mat_%s_%dx%dx%d_%d%d%d" % (dtype, m, n, k, a_k_fast, b_k_fast, d_n_fast), dtype, A, B, D,
                     alpha=1.25, beta=-0.5, seed=W.BASE_SEED + 21)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_two_phase_kernel(dtype):
    """The two-phase (ping-pong) kernel of the large tile, forced: every operand orientation, slab
    counts that end in each position of its loop unrolled by three, ragged M and N, split K."""
    from gpu_helpers import GpuProduct  # noqa: F401
    from gpu_helpers import run_gpu, say
    for flags in range(8):
        akf, bkf, dnf = bool(flags & 4), bool(flags & 2), bool(flags & 1)
        for k in (16, 32, 48, 64, 80, 96, 160, 176, 5, 23, 40, 100, 171):     # whole slabs, and ragged last slabs
            p = _matrix_product(300, 200, k, akf, bkf, dnf, dtype)
            a, b, c = W.make_operands(p)
            truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
            for variant in TWO_PHASE[False]:
                say("%s two-phase shape %d" % (p.name, variant))
                got = run_gpu(p, a, b, c, force_path=GETT, variant=variant)      # must not be declined: raises otherwise
                assert normalised_error(p, got, truth, S, c) <= TOLERANCE[p.dtype]
                for parts in (2, 3) if k >= 48 else ():
                    # 2 parts: summed inside the workgroup (one tile per wave group) or by the second
                    # kernel; 3 parts: the two items of a workgroup get different numbers of slabs
                    got = run_gpu(p, a, b, c, force_path=GETT, variant=variant, split_k=parts)
                    assert normalised_error(p, got, truth, S, c) <= TOLERANCE[p.dtype]
    # integer inputs: bit-exact
    p = _matrix_product(520, 260, 160, False, True, False, dtype)
    a, b, c = W.make_operands(p, "ints")
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    for variant in TWO_PHASE[False]:
        for parts in (None, 2):
            got = run_gpu(p, a, b, c, force_path=GETT, variant=variant, split_k=parts)
            assert np.array_equal(W.strided_view(got, p.D), W.strided_view(truth, p.D))


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_two_phase_kernel_batches_and_negative_strides(dtype):
    """Real batched products (a hyper label, slowest or fastest in memory) and operands stored
    backwards along k, along the rows, or both, on every two-phase shape; padded leading dimensions."""
    from gpu_helpers import run_gpu, say
    cases = []
    e = {"h": 5, "m": 150, "n": 100, "k": 64}
    # batch slowest / batch fastest
    cases.append(("batch_slowest", W.tensor("hmk", e, memory_order="mkh"), W.tensor("hkn", e, memory_order="knh"),
                  W.tensor("hmn", e, memory_order="mnh")))
    cases.append(("batch_fastest", W.tensor("hmk", e, memory_order="hkm"), W.tensor("hkn", e, memory_order="hkn"),
                  W.tensor("hmn", e, memory_order="hmn")))
    # reversed storage: negative strides along k (A), along n (B), along m (D); padded leading dimension in A
    e2 = {"m": 200, "n": 136, "k": 96}
    cases.append(("reversed", W.tensor("mk", e2, strides={"m": 1, "k": -210}), W.tensor("kn", e2, strides={"k": 1, "n": -96}),
                  W.tensor("mn", e2, strides={"m": -1, "n": 200})))
    cases.append(("reversed_k_fast", W.tensor("mk", e2, strides={"m": 100, "k": -1}), W.tensor("kn", e2, strides={"k": -1, "n": 97}),
                  W.tensor("mn", e2, strides={"m": 136, "n": -1})))
    for name, A, B, D in cases:
        p = W.Problem("two_phase_%s_%s" % (name, dtype), dtype, A, B, D, alpha=-0.75, beta=1.5, seed=W.BASE_SEED + 22)
        a, b, c = W.make_operands(p)
        truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
        for variant in TWO_PHASE[False]:
            for parts in (None, 2, 3):
                say("%s shape %d parts %s" % (p.name, variant, parts))
                got = run_gpu(p, a, b, c, force_path=GETT, variant=variant, split_k=parts)
                assert gaps_untouched(p, c, got)
                assert normalised_error(p, got, truth, S, c) <= TOLERANCE[p.dtype]


def _run_on(gp, p, a, b, c, shift_a=0):
    """Execute plan gp; shift_a: A is stored that many elements into its device buffer (an operand
    pointer that is not 16-byte aligned)."""
    import torch
    dA = torch.empty(a.size + shift_a, dtype=torch.from_numpy(a).dtype, device="cuda:0")
    dA[shift_a:] = torch.from_numpy(a).cuda()
    dB, dD = torch.from_numpy(b).cuda(), torch.from_numpy(c.copy()).cuda()
    gp.execute(dA[shift_a:], dB, dD, dD)
    torch.cuda.synchronize()
    return dD.cpu().numpy()


def test_two_phase_kernel_paired_loads():
    """fp64 tiles of one wave group each: with whole tiles and slabs, contiguous neighbours and
    16-byte alignment a gather load brings two elements (status: gather width 2).  Every operand
    orientation, K unsplit / in two / in three parts, integer inputs bit for bit; the same plan
    run on an operand pointer that is only 8-byte aligned takes the one-element kernel; a layout
    whose contiguous neighbours are four rows apart inside the tile."""
    from gpu_helpers import GpuProduct, say
    import paper_2601_07827_amd as T
    for flags, k in [(f, 96) for f in range(8)] + [(5, 16), (2, 32), (7, 48), (0, 80)]:    # short loops: 1 - 5 slabs
        akf, bkf, dnf = bool(flags & 4), bool(flags & 2), bool(flags & 1)
        p = _matrix_product(256, 384, k, akf, bkf, dnf, "f64")
        a, b, c = W.make_operands(p, "ints")
        truth, _ = run_oracle(p, a, b, c, oracle.MODE_TRUTH)
        for variant in (10, 11):
            for parts in (None, 2, 3) if k >= 48 else (None,):
                gp = GpuProduct(p, GETT, variant, parts)
                try:
                    assert gp.get(T.TCX_KEY_GATHER_WIDTH) == 2
                    for shift, width in ((0, 2), (1, 1)):
                        say("%s shape %d parts %s A shifted by %d" % (p.name, variant, parts, shift))
                        got = _run_on(gp, p, a, b, c, shift)
                        assert gp.last_gather_width == width and gp.last_variant == variant
                        assert np.array_equal(W.strided_view(got, p.D), W.strided_view(truth, p.D))
                finally:
                    gp.close()
    # B[k,x,y,z] stored z-fastest, D[x,m,y,z] stored x-fastest: the tile's columns run (x, z, y), so
    # B's contiguous neighbours (along z) are four columns apart
    e = {"m": 128, "k": 48, "x": 4, "y": 8, "z": 4}
    p = W.Problem("paired_step4", "f64", W.tensor("mk", e), W.tensor("kxyz", e, memory_order="zkxy"),
                  W.tensor("mxyz", e, memory_order="xmyz"), alpha=2.0, beta=-1.0, seed=W.BASE_SEED + 23)
    for dist, exact in (("uniform", False), ("ints", True)):
        a, b, c = W.make_operands(p, dist)
        truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
        for variant in (10, 11):
            gp = GpuProduct(p, GETT, variant)
            try:
                assert gp.get(T.TCX_KEY_GATHER_WIDTH) == 2
                assert [m[0] for m in gp.get(T.TCX_KEY_MODES_N)] == [4, 4, 8]
                say("%s shape %d dist %s" % (p.name, variant, dist))
                got = _run_on(gp, p, a, b, c)
                assert gp.last_gather_width == 2
                if exact:
                    assert np.array_equal(W.strided_view(got, p.D), W.strided_view(truth, p.D))
                else:
                    assert normalised_error(p, got, truth, S, c) <= TOLERANCE[p.dtype]
            finally:
                gp.close()


@pytest.mark.parametrize("h_slowest", [False, True])
def test_two_phase_kernel_complex(h_slowest):
    """The two-phase kernel with one 96 x 96 complex tile per wave group: batched conj(A)^T B with
    an odd number of batches (the last workgroup's second group has no tile), ragged tiles, whole and
    ragged slabs of K; also with K split (items of different length in one workgroup) and integer inputs."""
    from gpu_helpers import run_gpu, say
    for h, n, k in ((7, 40, 40), (5, 100, 24), (3, 96, 96), (4, 50, 21), (2, 96, 3)):
        p = W.config4(h=h, n=n, h_slowest=h_slowest, k=k)
        for dist, exact in (("uniform", False), ("ints", True)):
            a, b, c = W.make_operands(p, dist)
            truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
            for split in (None, 2, 3):
                say("%s two-phase complex dist=%s split=%s" % (p.name, dist, split))
                got = run_gpu(p, a, b, c, force_path=GETT, variant=TWO_PHASE[True][0], split_k=split)
                if exact:                                  # 0.5 * integer is exact
                    assert np.array_equal(W.strided_view(got, p.D), W.strided_view(truth, p.D))
                else:
                    assert normalised_error(p, got, truth, S, c) <= TOLERANCE[p.dtype]


@pytest.mark.parametrize("dtype", ["c128", "c64", "f64", "f32"])
def test_ragged_last_tiles_of_every_shape(dtype):
    """M = 200 and N = 250 end inside the last tile of every compiled shape (tiles of 32 to 256,
    and of 96 and 48 for complex128, which do not divide the tables' former padding unit): every
    shape, unsplit and split, against the oracle; every forced shape must run."""
    e = dict(m=200, n=250, k=40)
    # (the complex two-phase tile takes operands whose fastest mode is contracted)
    p = W.Problem("ragged_tiles_" + dtype, dtype, W.tensor("mk", e, memory_order="km" if dtype in COMPLEX else "mk"),
                  W.tensor("kn", e), W.tensor("mn", e),
                  alpha=1.5, beta=-0.5, opA=int(dtype in COMPLEX), seed=W.BASE_SEED + 51)
    a, b, c = W.make_operands(p)
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    for path, variant in _paths_for(p):
        _check(p, a, b, c, path, variant, truth=truth, S=S)
        if path == GETT:
            _check(p, a, b, c, path, variant, truth=truth, S=S, split_k=2)
    # at most the streaming path (operand rows beyond its LDS budget) and, unsplit and split, the
    # batch-lane shape (this product has no batch mode)
    assert _TALLY["declined"] <= (3 if dtype == "c128" else 1)


def _batched_complex(h, m, n, k, a_order, b_order, d_order, ops, beta=0.5, name="bl"):
    """D[h,i,j] = sum_k op(A[h,k,i]) op(B[h,k,j]) + beta op(C[h,i,j]) with the given memory orders."""
    e = dict(h=h, i=m, j=n, k=k)
    return W.Problem("%s_h%d_%dx%dx%d_%s_%s_%s_ops%d%d%d" % ((name, h, m, n, k, a_order, b_order, d_order) + tuple(ops)), "c128",
                     W.tensor("hki", e, memory_order=a_order), W.tensor("hkj", e, memory_order=b_order),
                     W.tensor("hij", e, memory_order=d_order), alpha=0.75 - 0.5j, beta=beta,
                     opA=ops[0], opB=ops[1], opC=ops[2], seed=W.BASE_SEED + 61)


def test_batch_lane_kernel():
    """The batch-lane kernel (complex tile shape 8): batches fastest in A, B and D, four batches per
    wave group.  Every combination of conjugations (the kernel sums conj(A) B or A B and conjugates
    the sum where needed), both orientations of A, B and D behind the batch mode, batch counts that
    leave the last workgroup's second group without a tile, ragged tiles of M and N, one and many
    slabs of K, beta = 0 with C absent, integer inputs bit for bit.  Layouts it cannot take (batch
    mode not fastest, batch count not a multiple of four, |K| not in whole slabs) are refused."""
    from gpu_helpers import GpuProduct, run_gpu, say
    import paper_2601_07827_amd as T
    cases = []
    for ops in ((0, 0, 0), (1, 0, 0), (0, 1, 1), (1, 1, 0)):
        cases.append(_batched_complex(8, 48, 48, 8, "hki", "hkj", "hij", ops))
    cases += [_batched_complex(12, 40, 100, 4, "hki", "hkj", "hij", (1, 0, 1)),        # odd number of groups, ragged tiles, one slab
              _batched_complex(4, 96, 50, 36, "hik", "hjk", "hji", (0, 1, 0)),          # rows before k in A and B, j before i in D
              _batched_complex(20, 17, 33, 12, "hki", "hjk", "hij", (1, 1, 1), beta=0.0),
              _batched_complex(16, 96, 96, 96, "hki", "hkj", "hij", (1, 0, 0))]         # configuration 4's shape, fewer batches
    for p in cases:
        for dist, exact in (("uniform", False), ("ints", True)):
            a, b, c = W.make_operands(p, dist)
            p2 = p if not exact else W.Problem(p.name + "_ints", p.dtype, p.A, p.B, p.D, alpha=2.0 - 1.0j, beta=(0.5 if p.beta != 0 else 0.0),
                                               opA=p.opA, opB=p.opB, opC=p.opC, seed=p.seed)
            truth, S = run_oracle(p2, a, b, c, oracle.MODE_TRUTH, want_S=True)
            say("%s dist=%s" % (p2.name, dist))
            got = run_gpu(p2, a, b, c, force_path=GETT, variant=8, c_null=(p2.beta == 0))      # must not be declined
            assert gaps_untouched(p2, c, got)
            if exact:
                assert np.array_equal(W.strided_view(got, p2.D), W.strided_view(truth, p2.D))
            else:
                assert normalised_error(p2, got, truth, S, c) <= TOLERANCE[p2.dtype]
    for bad in (_batched_complex(8, 48, 48, 8, "kih", "kjh", "ijh", (0, 0, 0)),            # batches slowest
                _batched_complex(6, 48, 48, 8, "hki", "hkj", "hij", (0, 0, 0)),            # 6 batches
                _batched_complex(8, 48, 48, 6, "hki", "hkj", "hij", (0, 0, 0))):           # |K| = 6
        with pytest.raises(T.TcxError) as exc:
            GpuProduct(bad, GETT, 8)
        assert exc.value.code == T.TCX_ERR_PLAN_REFUSED
    # K may not be split on it
    gp = GpuProduct(cases[0], GETT, 8)
    try:
        with pytest.raises(T.TcxError) as exc:
            T.tcx_product_set(gp.prod, T.TCX_KEY_SPLIT_K, 2)
        assert exc.value.code == T.TCX_ERR_PLAN_REFUSED
    finally:
        gp.close()


def test_conjugation_combinations_on_the_complex_two_phase_tile():
    """The 96 x 96 complex two-phase tile keeps conjugation out of its data path (sign modifier of
    the MFMA, conjugated sum): all eight combinations of opA, opB, opC, unsplit, K in two (summed in
    the second kernel) and with a ragged last slab."""
    from gpu_helpers import run_gpu, say
    for ops in [(a, b, c) for a in (0, 1) for b in (0, 1) for c in (0, 1)]:
        for k in (24, 21):
            p = _batched_complex(3, 100, 50, k, "kih", "kjh", "ijh", ops, name="conj")
            a, b, c = W.make_operands(p)
            truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
            for split in (None, 2):
                say("%s split=%s" % (p.name, split))
                got = run_gpu(p, a, b, c, force_path=GETT, variant=7, split_k=split)
                assert normalised_error(p, got, truth, S, c) <= TOLERANCE[p.dtype]


def _c64(p):
    return W.Problem(p.name.replace("c128", "c64"), "c64", p.A, p.B, p.D, alpha=p.alpha, beta=p.beta, opA=p.opA, opB=p.opB,
                     opC=p.opC, seed=p.seed)


@pytest.mark.parametrize("p", [_c64(W.config4(h=6, n=20)), _c64(W.config4(h=5, n=18, h_slowest=True)), _c64(W.config4(h=24, n=20, k=4)),
                               _c64(W.hadamard(2, 9, dtype="c128", permuted=True)), _c64(W.config4(h=3, n=96, k=40))],
                         ids=lambda p: p.name)
def test_complex64(p):
    """complex64 (Sec. "The Reference Implementation": complex numbers in 32-bit precision): the
    batched conjugated product of configuration 4 in both layouts, a low-intensity and a Hadamard
    shape, on every path and tile shape built for the type, K unsplit and split; integer inputs
    bit for bit; the error gate is the fp32 one."""
    for dist, exact in (("uniform", False), ("ints", True)):
        a, b, c = W.make_operands(p, dist)
        q = p if not exact else W.Problem(p.name + "_ints", p.dtype, p.A, p.B, p.D, alpha=2.0 - 1.0j, beta=(0.5 if p.beta != 0 else 0.0),
                                          opA=p.opA, opB=p.opB, opC=p.opC, seed=p.seed)
        truth, S = run_oracle(q, a, b, c, oracle.MODE_TRUTH, want_S=True)
        for path, variant in _paths_for(q) + [(None, None)]:
            _check(q, a, b, c, path, variant, exact=exact, truth=truth, S=S)
            if path == GETT and q.sizes()[3] >= 16:
                _check(q, a, b, c, path, variant, exact=exact, truth=truth, S=S, split_k=2)


@pytest.mark.parametrize("dtype", ["f32", "c64"])
def test_precision_f64_on_32_bit_tensors(dtype):
    """TCX_PREC_F64 (Sec. "Tensor Operation Descriptors": the plan's computational precision):
    32-bit tensors, products and sums in 64-bit arithmetic, one rounding on the store.  With 8192
    contracted terms the result sits within one storage rounding of the truth (gate 2^-23 of the
    normaliser, against 1e-5 for 32-bit arithmetic), on the generic kernel and on both widened tile
    shapes, K unsplit and split; the same plan in default precision is measurably further away;
    integer inputs bit for bit."""
    from gpu_helpers import run_gpu, say
    import paper_2601_07827_amd as T
    e = dict(m=150, n=70, k=8192)
    cplx = dtype == "c64"
    p = W.Problem("wide_" + dtype, dtype, W.tensor("km", e), W.tensor("kn", e), W.tensor("mn", e),
                  alpha=(0.5 - 0.25j) if cplx else 0.5, beta=-2.0, opA=int(cplx), seed=W.BASE_SEED + 71)
    a, b, c = W.make_operands(p)
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    shapes = (1, 2) if cplx else (2, 3)
    worst_wide = 0.0
    for path, variant, split in [(GENERIC, None, None)] + [(GETT, v, sp) for v in shapes for sp in (None, 4)] + [(None, None, None)]:
        say("%s path=%s shape=%s split=%s TCX_PREC_F64" % (p.name, path, variant, split))
        got = run_gpu(p, a, b, c, force_path=path, variant=variant, split_k=split, precision=T.TCX_PREC_F64)
        err = normalised_error(p, got, truth, S, c)
        assert err <= TOLERANCE_WIDENED, (path, variant, split, err)
        worst_wide = max(worst_wide, err)
    plain = normalised_error(p, run_gpu(p, a, b, c, force_path=GETT, variant=shapes[0]), truth, S, c)
    assert plain <= TOLERANCE[dtype] and plain > 2 * worst_wide, (plain, worst_wide)
    a, b, c = W.make_operands(p, "ints")
    q = W.Problem(p.name + "_ints", dtype, p.A, p.B, p.D, alpha=2.0, beta=-1.0, opA=p.opA, seed=p.seed)
    truth, _ = run_oracle(q, a, b, c, oracle.MODE_TRUTH)
    for path, variant in ((GENERIC, None), (GETT, shapes[0]), (GETT, shapes[1])):
        got = run_gpu(q, a, b, c, force_path=path, variant=variant, precision=T.TCX_PREC_F64)
        assert np.array_equal(W.strided_view(got, q.D), W.strided_view(truth, q.D))


@pytest.mark.parametrize("dtype", ["f64", "f32", "c128", "c64"])
def test_isolated_labels(dtype):
    """Secs. "Case 4" and "Case 5": labels in A only or in B only are summed inside that tensor by a
    kernel of their own before the product, labels in D only repeat it.  Random label patterns with
    such labels on every path, uniform inputs within tolerance and integer inputs bit for bit; the
    paper's two examples (repeated labels on top)."""
    from gpu_helpers import run_gpu, say
    rng = np.random.default_rng(4242)
    for i in range(24):
        p = random_problem(rng, dtype, max_group=2, max_extent=5, allow_neg=(i % 3 == 0), name="iso%d_%s" % (i, dtype), isolated=True)
        for dist, exact in (("uniform", False), ("ints", True)):
            a, b, c = W.make_operands(p, dist)
            truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
            for path, variant in ((GENERIC, None), (GETT, 2 if dtype not in COMPLEX else 1), (STREAM, None), (None, None)):
                _check(p, a, b, c, path, variant, exact=exact, truth=truth, S=S)
    ext = dict(a=13, b=24, g=7, d=35, e=3)
    rep = lambda labels: _rep(labels, ext)
    for name, la, lb, ld in (("case4", "bab", "bgdga", "da"), ("case5", "bab", "bgdga", "dae")):
        p = W.Problem("%s_%s" % (name, dtype), dtype, rep(la), rep(lb), rep(ld), alpha=2.0, beta=-1.0, opA=int(dtype in COMPLEX),
                      seed=W.BASE_SEED + 81)
        a, b, c = W.make_operands(p, "ints")
        truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
        for path in (None, GENERIC, GETT, STREAM):
            say("%s path=%s" % (p.name, path))
            try:
                got = run_gpu(p, a, b, c, force_path=path)
            except Exception as exc:
                if path in (GETT, STREAM) and getattr(exc, "code", None) == REFUSED:
                    continue
                raise
            assert np.array_equal(W.strided_view(got, p.D), W.strided_view(truth, p.D)), path


def _rep(labels, ext):
    """Column-major tensor whose label string may repeat a label (each position its own stride)."""
    strides, run = [], 1
    for l in labels:
        strides.append(run)
        run *= ext[l]
    e = tuple(ext[l] for l in labels)
    base, size = W.span_of(e, strides)
    return W.TensorSpec(tuple(labels), e, tuple(strides), base, size)


@pytest.mark.parametrize("dtype", ["f64", "f32", "c128", "c64"])
def test_unary_and_binary_operations(dtype):
    """Sec. "Unary and Binary Operations": C := alpha op(A) + beta op(B) with a label of A that C
    lacks (summed) and a label of C that A lacks (broadcast), in place and into a separate C, against
    numpy's plain evaluation and against the oracle's contraction alpha A * 1 + beta B; B := alpha
    op(A) as a scaled transposition between two layouts and as the diagonal of a repeated label.
    Integer inputs: bit for bit."""
    import torch
    import paper_2601_07827_amd as T
    from gpu_helpers import DT, say
    ext = dict(h=37, g=11, x=6, y=9)
    ids = dict(h=1, g=2, x=3, y=4)
    cplx = dtype in COMPLEX
    npdt = W.Problem("t", dtype, W.tensor("", ext), W.tensor("", ext), W.tensor("", ext)).np_dtype
    A = W.tensor("xhg", ext, memory_order="gxh")
    B = W.tensor("gyh", ext, strides=dict(g=2, y=25, h=-230))
    a = W.fill(A, 5, W.TAG_A, npdt, "ints")
    b = W.fill(B, 5, W.TAG_B, npdt, "ints")
    alpha, beta = ((2.0 - 1.0j), -0.5) if cplx else (2.0, -0.5)
    opA, opB = int(cplx), int(cplx)
    va, vb = W.strided_view(a, A), W.strided_view(b, B)
    fa = np.conj(va) if opA else va
    fb = np.conj(vb) if opB else vb
    expect = (alpha * fa.sum(axis=0).T[:, None, :] + beta * fb).astype(npdt)          # [g, y, h]: sum over x, broadcast over y
    # the same through the oracle: contraction with a rank-0 second operand holding one
    one = W.tensor("", ext)
    p = W.Problem("binary_as_contraction", dtype, A, one, B, alpha=alpha, beta=beta, opA=opA, opC=opB)
    truth, _ = run_oracle(p, a, np.ones(1, dtype=npdt), b, oracle.MODE_TRUTH)
    assert np.array_equal(W.strided_view(truth, B), expect)
    h = T.tcx_create_handle()
    ex = T.tcx_create_executor(h, torch.cuda.current_stream().cuda_stream)
    info = lambda spec: T.tcx_create_tensor_info(h, DT[dtype], spec.extents, spec.strides)
    lab = lambda spec: [ids[l] for l in spec.labels]
    ia, ib = info(A), info(B)
    plan = T.tcx_create_binary(h, opA, ia, lab(A), opB, ib, lab(B), 0, ib, lab(B))
    item = np.dtype(npdt).itemsize
    dA, dB = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
    for in_place in (False, True):
        say("binary %s in_place=%s" % (dtype, in_place))
        dC = dB.clone() if in_place else torch.full_like(dB, -777.0)
        src = dC if in_place else dB
        T.tcx_execute_binary(plan, ex, DT[dtype], alpha, dA.data_ptr() + A.base * item, beta, src.data_ptr() + B.base * item,
                             dC.data_ptr() + B.base * item)
        torch.cuda.synchronize()
        got = dC.cpu().numpy()
        assert np.array_equal(W.strided_view(got, B), expect)
        keep = b if in_place else np.full_like(b, -777.0)
        mask = np.zeros(b.shape[0], dtype=bool)
        W.strided_view(mask, B)[...] = True
        assert np.array_equal(got[~mask], keep[~mask])                      # gaps of C untouched
    T.tcx_destroy_product(plan)
    # unary: B[h,g,x] := alpha op(A[x,h,g]) into another layout
    Bt = W.tensor("hgx", ext, memory_order="xgh")
    it = info(Bt)
    un = T.tcx_create_unary(h, opA, ia, lab(A), 0, it, lab(Bt))
    dT = torch.full((Bt.size,), -777.0, dtype=dA.dtype, device="cuda:0")
    T.tcx_execute_unary(un, ex, DT[dtype], alpha, dA.data_ptr() + A.base * item, dT.data_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(W.strided_view(dT.cpu().numpy(), Bt), (alpha * fa.transpose(1, 2, 0)).astype(npdt))
    T.tcx_destroy_product(un)
    # unary with a repeated label: the diagonal of a square matrix
    sq = W.TensorSpec(("g", "g"), (11, 11), (1, 11), 0, 121)
    vec = W.tensor("g", ext)
    m = W.fill(sq, 6, W.TAG_A, npdt, "ints")
    isq, iv = info(sq), info(vec)
    un = T.tcx_create_unary(h, 0, isq, [2, 2], 0, iv, [2])
    dM, dV = torch.from_numpy(m).cuda(), torch.zeros(11, dtype=dA.dtype, device="cuda:0")
    T.tcx_execute_unary(un, ex, DT[dtype], 3.0, dM.data_ptr(), dV.data_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(dV.cpu().numpy(), (3.0 * np.diagonal(m.reshape(11, 11))).astype(npdt))
    T.tcx_destroy_product(un)
    for i in (ia, ib, it, isq, iv):
        T.tcx_destroy_tensor_info(i)
    T.tcx_destroy_executor(ex)
    T.tcx_destroy_handle(h)


@pytest.mark.parametrize("dt16", ["f16", "bf16"])
@pytest.mark.parametrize("precision", [0, 1], ids=["arith32", "arith64"])
def test_sixteen_bit_tensors(precision, dt16):
    """TCX_F16, TCX_BF16 (Sec. "The Reference Implementation": real types of 16 bit): IEEE binary16 or bfloat16 tensors,
    products and sums in 32-bit (default) or 64-bit reals, one rounding to 16 bits on the store;
    alpha and beta are floats.  A product with 2048 contracted terms on the generic kernel and on
    both widened tile shapes, K unsplit and split, and on the plan's own choice (gate: twice one 16-bit rounding of
    the normaliser); integer inputs bit for bit; random label patterns with
    padded and negative strides, with labels of one tensor only (reduction kernel and broadcast);
    a binary operation."""
    import torch
    import paper_2601_07827_amd as T
    from gpu_helpers import DT, run_gpu, say
    e = dict(m=150, n=70, k=2048)
    p = W.Problem(dt16 + "_gemm", dt16, W.tensor("km", e), W.tensor("kn", e), W.tensor("mn", e), alpha=0.5, beta=-2.0, seed=W.BASE_SEED + 73)
    a, b, c = W.make_operands(p)
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    for path, variant, split in [(GENERIC, None, None)] + [(GETT, v, sp) for v in (2, 3) for sp in (None, 4)] + [(None, None, None)]:
        say("%s path=%s shape=%s split=%s precision=%d" % (p.name, path, variant, split, precision))
        got = run_gpu(p, a, b, c, force_path=path, variant=variant, split_k=split, precision=precision)
        err = normalised_error(p, got, truth, S, c)
        assert err <= TOLERANCE[dt16], (path, variant, split, err)
    a, b, c = W.make_operands(p, "ints")
    q = W.Problem(p.name + "_ints", dt16, p.A, p.B, p.D, alpha=2.0, beta=-1.0, seed=p.seed)
    truth, _ = run_oracle(q, a, b, c, oracle.MODE_TRUTH)
    for path, variant in ((GENERIC, None), (GETT, 2), (GETT, 3)):
        got = run_gpu(q, a, b, c, force_path=path, variant=variant, precision=precision)
        assert np.array_equal(values_of(q, got, q.D), values_of(q, truth, q.D))
    # shapes the tiled path does not take for 16-bit tensors, and the streaming path, are refused
    for path, variant in ((GETT, 0), (GETT, 10), (STREAM, None)):
        with pytest.raises(T.TcxError) as exc:
            run_gpu(q, a, b, c, force_path=path, variant=variant, precision=precision)
        assert exc.value.code == REFUSED
    rng = np.random.default_rng(1616 + precision)
    for i in range(24):
        r = random_problem(rng, dt16, max_group=3, max_extent=6, allow_neg=(i % 3 == 0), name="rand%d_%s" % (i, dt16), isolated=(i % 2 == 1))
        a, b, c = W.make_operands(r)
        truth, S = run_oracle(r, a, b, c, oracle.MODE_TRUTH, want_S=True)
        for path, variant in ((GENERIC, None), (GETT, 2 + i % 2), (None, None)):
            say("%s path=%s shape=%s precision=%d" % (r.name, path, variant, precision))
            got = run_gpu(r, a, b, c, force_path=path, variant=variant, precision=precision)
            assert gaps_untouched(r, c, got)
            assert normalised_error(r, got, truth, S, c) <= TOLERANCE[dt16], (r, path, variant)
    # binary operation: C[g,y,h] := alpha sum_x A[x,h,g] + beta B[g,y,h]
    ext = dict(x=5, h=7, g=11, y=3)
    A, B = W.tensor("xhg", ext), W.tensor("gyh", ext, memory_order="hgy")
    ids = {l: i for i, l in enumerate("xhgy")}
    npdt = p.np_dtype
    q = W.Problem("binary", dt16, A, B, B)
    av, bv = W.fill(A, 5, W.TAG_A, npdt, "ints"), W.fill(B, 5, W.TAG_B, npdt, "ints")
    # halves of small integers: exact in either 16-bit type, so float64 arithmetic gives the stored value
    expect = 2.0 * values_of(q, av, A).astype(np.float64).sum(axis=0).T[:, None, :] - 0.5 * values_of(q, bv, B).astype(np.float64)
    h = T.tcx_create_handle()
    ex = T.tcx_create_executor(h, torch.cuda.current_stream().cuda_stream)
    ia, ib = (T.tcx_create_tensor_info(h, DT[dt16], t.extents, t.strides) for t in (A, B))
    plan = T.tcx_create_binary(h, 0, ia, [ids[l] for l in A.labels], 0, ib, [ids[l] for l in B.labels], 0, ib, [ids[l] for l in B.labels], precision)
    dA, dB = torch.from_numpy(av).cuda(), torch.from_numpy(bv).cuda()
    T.tcx_execute_binary(plan, ex, DT[dt16], 2.0, dA.data_ptr(), -0.5, dB.data_ptr(), dB.data_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(values_of(q, dB.cpu().numpy(), B).astype(np.float64), expect)
    T.tcx_destroy_product(plan)
    for i in (ia, ib):
        T.tcx_destroy_tensor_info(i)
    T.tcx_destroy_executor(ex)
    T.tcx_destroy_handle(h)


@pytest.mark.parametrize("dt16", ["f16", "bf16"])
def test_sixteen_bit_store_rounds_once_from_64_bit_sums(dt16):
    """16-bit tensors with TCX_PREC_F64: the 64-bit sum is rounded to 16 bits in ONE step.  With p
    significant bits (11 for binary16, 8 for bfloat16) and u = 2^-p, two sums that a detour over a
    32-bit float would round the wrong way: 1 + u + 2^-30 (a hair above the midpoint of 1 and
    1 + 2u; as a float it is the midpoint itself and the tie would go down to 1) and
    1 + 2u + u - 2^-30 (a hair below the midpoint of 1 + 2u and 1 + 4u; the tie would go up).
    Both round to 1 + 2u.  Expected values: the oracle's, from its long-double sum."""
    from gpu_helpers import run_gpu, say
    u = 2.0 ** -11 if dt16 == "f16" else 2.0 ** -8
    one_plus_2u = 0x3c01 if dt16 == "f16" else 0x3f81
    e = dict(m=2, k=4, n=1)
    p = W.Problem(dt16 + "_round_once", dt16, W.tensor("km", e), W.tensor("kn", e), W.tensor("mn", e), alpha=1.0, beta=0.0)

    def encode(values):          # all of them 16-bit numbers (2^-15 is a subnormal of binary16)
        v = np.asarray(values, dtype=np.float32)
        return v.astype(np.float16) if dt16 == "f16" else W.bf16_bits(v)
    a = encode([1.0, u, 2.0 ** -15, 0.0, 1.0, 2 * u, u, -2.0 ** -15])        # [m][k], k fastest
    b0, b1 = encode([1.0, 1.0, 2.0 ** -15, 2.0 ** -15]), encode([1.0, 1.0, 1.0, 2.0 ** -15])
    assert np.array_equal(a.astype(np.float64) if dt16 == "f16" else W.bf16_values(a).astype(np.float64),
                          [1.0, u, 2.0 ** -15, 0.0, 1.0, 2 * u, u, -2.0 ** -15])
    c = np.zeros(2, dtype=p.np_dtype)
    for row, b in ((0, b0), (1, b1)):
        truth, _ = run_oracle(p, a, b, c, oracle.MODE_TRUTH)
        assert int(truth.view(np.uint16)[row]) == one_plus_2u, hex(int(truth.view(np.uint16)[row]))
        for path, variant in ((GENERIC, None), (GETT, 2), (GETT, 3)):
            say("%s row=%d path=%s shape=%s" % (p.name, row, path, variant))
            got = run_gpu(p, a, b, c, force_path=path, variant=variant, precision=1)
            assert int(got.view(np.uint16)[row]) == one_plus_2u, (row, path, variant, hex(int(got.view(np.uint16)[row])))


@pytest.mark.parametrize("dtype", ["f64", "f32", "c128", "c64"])
def test_streaming_tiles_whose_lines_collide(dtype):
    """A three-way transposition whose strides inside a tile are all multiples of 128 KB: the plan
    marks its loads as paced (TCX_KEY_PACED_LOADS) and runs the paced instantiation of the flat
    streaming kernel.  Whole tiles, ragged last chunks, with and without the C read, conjugations;
    integer inputs bit for bit."""
    import paper_2601_07827_amd as T
    from gpu_helpers import GpuProduct, run_gpu, say
    labs = ["h0", "h1", "h2", "h3"]
    cplx = dtype in ("c128", "c64")
    unit = 128 * 1024 // {"f32": 4, "f64": 8, "c64": 8, "c128": 16}[dtype]        # elements in 128 KB
    for ext, beta in ((dict(h0=16, h1=16, h2=3, h3=16), 0.0), (dict(h0=24, h1=32, h2=2, h3=16), 0.5),
                      (dict(h0=8, h1=16, h2=5, h3=40), -1.0)):
        A = W.tensor(labs, ext, strides=dict(h1=1, h2=128, h3=unit, h0=32 * unit))
        B = W.tensor(labs, ext, strides=dict(h3=1, h2=128, h1=unit, h0=32 * unit))
        D = W.tensor(labs, ext, strides=dict(h0=1, h1=128, h2=unit, h3=32 * unit))
        for dist in ("uniform", "ints"):
            alpha = 2.0 if dist == "ints" else ((1.5 - 0.5j) if cplx else 1.5)
            p = W.Problem("colliding_lines_%s" % dtype, dtype, A, B, D, alpha=alpha, beta=beta if dist == "uniform" else float(int(beta * 2)),
                          opA=int(cplx), opC=int(cplx), seed=W.BASE_SEED + 97)
            gp = GpuProduct(p, force_path=STREAM)
            paced = gp.get(T.TCX_KEY_PACED_LOADS)
            gp.close()
            assert paced == 1, "the plan did not see the collision"
            say("%s extents %s beta %s %s" % (p.name, ext, p.beta, dist))
            a, b, c = W.make_operands(p, dist)
            truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
            got = run_gpu(p, a, b, c, force_path=STREAM)
            if dist == "ints":
                assert np.array_equal(W.strided_view(got, p.D), W.strided_view(truth, p.D))
            else:
                assert normalised_error(p, got, truth, S, c) <= TOLERANCE[dtype]
            mask = np.zeros(c.shape[0], dtype=bool)
            W.strided_view(mask, p.D)[...] = True
            assert np.array_equal(got[~mask], c[~mask])              # gaps of D untouched


LOW_AI_LARGE = [W.config5(extent=4, nshared=1, nfree=7), W.config4(h=512, n=96, k=4),
                W.hadamard(4, 64, permuted=True, beta=0.5), W.config5(extent=4, nshared=0, nfree=6)]


@pytest.mark.parametrize("p", LOW_AI_LARGE, ids=lambda p: p.name)
def test_low_intensity_shapes_large(p):
    """The streaming path at sizes far beyond one tile (the rank-14 output of the one-label
    contraction has 4^14 elements), whole output compared, on the plan's own path and on the
    streaming path forced."""
    a, b, c = W.make_operands(p, "uniform")
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    _check(p, a, b, c, None, None, truth=truth, S=S)
    _check(p, a, b, c, STREAM, None, truth=truth, S=S)


FULL = [W.config1(), W.config3(), W.config3(d_layout="R2"), W.config4(), W.config4(h_slowest=True), W.config5()]


@pytest.mark.parametrize("p", FULL, ids=lambda p: p.name)
def test_full_size_configs(p):
    """Configurations 1, 3, 4, 5 at their full sizes, plan's own path, whole output compared."""
    a, b, c = W.make_operands(p)
    _check(p, a, b, c, None, None)


@pytest.mark.parametrize("p", [W.config1(), W.config3(), W.config5()], ids=lambda p: p.name)
def test_full_size_integer_inputs_bit_exact(p):
    a, b, c = W.make_operands(p, "ints")
    p2 = W.Problem(p.name + "_ints", p.dtype, p.A, p.B, p.D, alpha=2.0, beta=(0.5 if p.beta != 0 else 0.0), seed=p.seed)
    truth, S = run_oracle(p2, a, b, c, oracle.MODE_TRUTH, want_S=True)
    _check(p2, a, b, c, None, None, exact=True, truth=truth, S=S)
    _check(p2, a, b, c, GETT, 1, exact=True, truth=truth, S=S, split_k=4)
    _check(p2, a, b, c, GETT, 2, exact=True, truth=truth, S=S, split_k=1)


def test_split_k_is_deterministic():
    """Two executions of a split-K plan give the same bits (parts are summed in a fixed order)."""
    from gpu_helpers import run_gpu
    p = W.config1()
    a, b, c = W.make_operands(p)
    r1 = run_gpu(p, a, b, c, force_path=GETT, variant=2, split_k=6)
    r2 = run_gpu(p, a, b, c, force_path=GETT, variant=2, split_k=6)
    assert np.array_equal(r1, r2)


def test_one_split_k_product_on_two_executors_at_once():
    """The partial sums of a split-K plan live in the executor's workspace, not in the plan: one
    product is executed on two executors (two streams of default priority) whose launches
    interleave, each into its own D, many times over; both results carry the oracle's bits
    (integer inputs), also in the iterations where the two streams ran side by side."""
    import torch
    import paper_2601_07827_amd as T
    from gpu_helpers import GpuProduct, say
    import dataclasses
    p = dataclasses.replace(W.config1(), alpha=2.0, beta=-1.0)          # integer scalars: every order of the sums gives the same bits
    a, b, c = W.make_operands(p, "ints")
    truth, _ = run_oracle(p, a, b, c, oracle.MODE_TRUTH)
    gp = GpuProduct(p, force_path=GETT, variant=3, split_k=6)
    assert gp.get(T.TCX_KEY_WORKSPACE_BYTES) > 0
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    exs = [T.tcx_create_executor(gp.h, s.cuda_stream) for s in streams]
    item = a.itemsize
    dA, dB, dC = (torch.from_numpy(x).cuda() for x in (a, b, c))
    dD = [torch.zeros_like(dC), torch.zeros_like(dC)]
    torch.cuda.synchronize()
    say("%s on two executors, 40 interleaved executions each" % p.name)
    for it in range(40):
        for ex, d in zip(exs, dD):
            T.tcx_execute_product(gp.prod, ex, gp.dtype, p.alpha, dA.data_ptr() + p.A.base * item, dB.data_ptr() + p.B.base * item,
                                  p.beta, dC.data_ptr() + p.D.base * item, d.data_ptr() + p.D.base * item)
    torch.cuda.synchronize()
    for d in dD:
        assert np.array_equal(W.strided_view(d.cpu().numpy(), p.D), W.strided_view(truth, p.D))
    for ex in exs:
        T.tcx_destroy_executor(ex)
    gp.close()


@pytest.mark.parametrize("dist", ["uniform", "ints"])
def test_config2_full_size_sampled(dist):
    """Configuration 2 at its full size (10.9 GB V, generated on the device by the torch twin of
    the counter-based generator), in the launch configuration bench.py times.  More than 65 536
    sampled outputs -- both sides of every tile boundary, every launch round and XCD stretch, plus
    random ones -- each a full 36864-term sum evaluated by the oracle.  Integer-valued inputs must
    match bit for bit."""
    import torch
    import bench
    from gpu_helpers import GpuProduct, say
    p = W.config2()
    say("%s full size, dist=%s" % (p.name, dist))
    dA, dB, dD, _ = bench.device_operands(p, torch, dist)
    # the device generator reproduces the host generator
    probe = np.array([0, 1, 12345678, p.A.size - 1], dtype=np.uint64)
    gen = W.DISTRIBUTIONS[dist]
    assert np.array_equal(dA[torch.from_numpy(probe.astype(np.int64)).cuda()].cpu().numpy(), gen(p.seed, W.TAG_A, probe, np.float64))
    gp = GpuProduct(p)
    try:
        assert (gp.get(gp.T.TCX_KEY_PATH), gp.get(gp.T.TCX_KEY_TILE_M), gp.get(gp.T.TCX_KEY_TILE_N)) == (1, 256, 128)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(torch.cuda.current_stream())
        gp.execute(dA, dB, dD, dD)
        e1.record(torch.cuda.current_stream())
        torch.cuda.synchronize()
        # a guard against the kernel silently losing its registers to scratch memory (it then runs
        # forty times longer and still computes the right numbers): 1.1e13 flop at 25 % of peak
        assert e0.elapsed_time(e1) < 600.0, "configuration 2 took %.0f ms" % e0.elapsed_time(e1)
        res = bench.parity_after_run(p, dD, 1, torch, dist)
    finally:
        gp.close()
    assert res["samples"] >= 65536
    assert res["ok"], res
    if dist == "ints":
        assert res["bit_exact"], res


def test_config2_full_size_freivalds_probes():
    """Every element of configuration 2's 1.5e8 outputs at once: for eight seeded random vector
    pairs (x over the rows, y over the columns of D as a 36864 x 4096 matrix)
        x^T D y  =  alpha sum_k (x^T V)_k (T y)_k  +  beta x^T D0 y,
    the right-hand side evaluated by the oracle (long-double sums; V, T and D0 come from the
    counter-based generator's device twin, copied to the host slab by slab).  A single element that
    is off by its own magnitude moves the left-hand side by more than the gate, 1e-12 of
    sum_k |(x^T V)_k| |(T y)_k| + |x|^T |D0 y| (a lower bound of the error measure's normaliser)."""
    import torch
    import bench
    from gpu_helpers import GpuProduct, say
    p = W.config2()
    _, M, N, K = p.sizes()
    P = 8
    say("%s full size, %d Freivalds probes" % (p.name, P))
    dA, dB, dD, _ = bench.device_operands(p, torch)
    X = W.uniform_pm1(p.seed, 40, np.arange(P * M, dtype=np.uint64), np.float64)         # [p, m], p fastest
    Y = W.uniform_pm1(p.seed, 41, np.arange(N * P, dtype=np.uint64), np.float64)         # [n, p], n fastest
    e = dict(p=P, m=M, n=N, k=K)

    def times_Y(buf):
        """[M or K, N] (first index fastest) times Y: rows x P."""
        rows = buf.shape[0] // N
        ee = dict(r=rows, n=N, p=P)
        q = W.Problem("timesY", "f64", W.tensor("rn", ee), W.tensor("np", ee), W.tensor("rp", ee), alpha=1.0, beta=0.0)
        out, _ = run_oracle(q, buf, Y, np.zeros(rows * P))
        return out.reshape((rows, P), order="F")

    d0 = dD.cpu().numpy()
    Z0 = times_Y(d0)                                                   # D0 y
    del d0
    Wm = times_Y(dB.cpu().numpy())                                     # T y: [k, p]
    U = np.empty((P, K))                                               # x^T V: [p, k]
    kc = 2048
    for k0 in range(0, K, kc):
        slab = dA[k0 * M:(k0 + kc) * M].cpu().numpy()                  # V[:, k0 : k0 + kc], rows fastest
        ee = dict(p=P, m=M, k=kc)
        q = W.Problem("xV", "f64", W.tensor("pm", ee), W.tensor("mk", ee), W.tensor("pk", ee), alpha=1.0, beta=0.0)
        out, _ = run_oracle(q, X, slab, np.zeros(P * kc))
        U[:, k0:k0 + kc] = out.reshape((P, kc), order="F")
        say("  x^T V: slab %d of %d" % (k0 // kc + 1, K // kc))
    gp = GpuProduct(p)
    try:
        gp.execute(dA, dB, dD, dD)
        torch.cuda.synchronize()
    finally:
        gp.close()
    Z1 = times_Y(dD.cpu().numpy())                                     # D y
    ld = np.longdouble
    Xm = X.reshape((P, M), order="F").astype(ld)
    for j in range(P):
        lhs = np.sum(Xm[j] * Z1[:, j].astype(ld))
        ab = np.sum(U[j].astype(ld) * Wm[:, j].astype(ld))
        c0 = np.sum(Xm[j] * Z0[:, j].astype(ld))
        rhs = ld(p.alpha) * ab + ld(p.beta) * c0
        gate = 1e-12 * float(np.sum(np.abs(U[j]) * np.abs(Wm[:, j])) + np.sum(np.abs(Xm[j]) * np.abs(Z0[:, j])))
        say("  probe %d: lhs %.6e rhs %.6e |diff| %.3e gate %.3e" % (j, float(lhs), float(rhs), abs(float(lhs - rhs)), gate))
        assert abs(float(lhs - rhs)) <= gate
        assert gate < 1.0                                              # a single element off by its own size (tens) would show


@pytest.mark.parametrize("dist", ["uniform", "ints"])
def test_round_by_round_launch(dist):
    """A product whose tiles are long (324 slabs) and more numerous than the CUs is enqueued as
    several launches of the two-phase kernel, the last one partial (378 tiles = 256 + 122).
    Sampled outputs from both launches against the oracle; integer inputs bit for bit."""
    import torch
    import bench
    from gpu_helpers import GpuProduct, say
    p = W.config2(v=72, o=48)
    say("%s, dist=%s" % (p.name, dist))
    dA, dB, dD, _ = bench.device_operands(p, torch, dist)
    gp = GpuProduct(p, force_path=GETT, variant=0)        # a forced shape starts unsplit
    try:
        assert (gp.get(gp.T.TCX_KEY_PATH), gp.get(gp.T.TCX_KEY_VARIANT), gp.get(gp.T.TCX_KEY_GRID)) == (1, 0, 378)
        assert gp.get(gp.T.TCX_KEY_LAUNCHES) == 2
        gp.execute(dA, dB, dD, dD)
        torch.cuda.synchronize()
        res = bench.parity_after_run(p, dD, 1, torch, dist)
    finally:
        gp.close()
    assert res["samples"] >= 200
    assert res["ok"], res
    if dist == "ints":
        assert res["bit_exact"], res


def test_key_value_interface_on_a_status_and_a_replanned_product():
    """The unified key-value interface on objects that only exist with a device: a status object
    answers its keys through it and carries free-form values; a product whose tuning overrides were
    set and then cleared through it computes the same result as before."""
    import torch
    import paper_2601_07827_amd as T
    from gpu_helpers import GpuProduct
    p = W.config1(16)
    a, b, c = W.make_operands(p)
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    gp = GpuProduct(p)
    try:
        planned = {k: gp.get(k) for k in (T.TCX_KEY_PATH, T.TCX_KEY_VARIANT, T.TCX_KEY_SPLIT_K)}
        for step in ("planned", "forced", "cleared"):
            if step == "forced":
                T.tcx_attr_set(gp.prod, T.TCX_KEY_FORCE_PATH, GETT)
                T.tcx_attr_set(gp.prod, T.TCX_KEY_VARIANT, 1)
                T.tcx_attr_set(gp.prod, T.TCX_KEY_SPLIT_K, 2)
            if step == "cleared":
                T.tcx_attr_clear(gp.prod, T.TCX_KEY_VARIANT)
                assert {k: gp.get(k) for k in planned} == planned
            dA, dB, dD = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda(), torch.from_numpy(c.copy()).cuda()
            st = T.tcx_execute_product(gp.prod, gp.ex, gp.dtype, p.alpha, dA.data_ptr(), dB.data_ptr(), p.beta,
                                       dD.data_ptr(), dD.data_ptr(), want_status=True)
            torch.cuda.synchronize()
            for key in (T.TCX_KEY_PATH, T.TCX_KEY_VARIANT, T.TCX_KEY_GRID, T.TCX_KEY_HIP_ERROR):
                assert T.tcx_attr_get(st, key) == T.tcx_status_get(st, key)
            if step == "forced":
                assert (T.tcx_attr_get(st, T.TCX_KEY_PATH), T.tcx_attr_get(st, T.TCX_KEY_VARIANT)) == (GETT, 1)
            T.tcx_attr_set(st, T.TCX_KEY_USER + 1, step.encode())
            assert T.tcx_attr_get(st, T.TCX_KEY_USER + 1) == step.encode()
            assert T.tcx_destroy_status(st) == 0
            assert normalised_error(p, dD.cpu().numpy(), truth, S, c) <= TOLERANCE[p.dtype], step
    finally:
        gp.close()


def _sub(labels, ext, parent_ext, fixed=None, negative=()):
    """A sub-tensor: a box of extents `ext` inside a column-major parent with extents `parent_ext`
    over the same label order plus the labels in `fixed` (parent indices held fixed: a view with
    fewer modes than its parent); labels in `negative` are walked backwards."""
    fixed = fixed or {}
    order = list(labels) + [l for l in fixed if l not in labels]
    stride, run = {}, 1
    for l in order:
        stride[l] = run
        run *= parent_ext[l]
    strides = [(-stride[l] if l in negative else stride[l]) for l in labels]
    e = tuple(ext[l] for l in labels)
    base, _ = W.span_of(e, strides)
    return W.TensorSpec(tuple(labels), e, tuple(strides), base + sum(i * stride[l] for l, i in fixed.items()), run)


def _paper_list_cases():
    ext = dict(h=3, m=20, n=17, k=9, l=5, x=4)
    big = dict(h=5, m=33, n=19, k=12, l=7, x=6)
    rep, run = [], 1
    for l in "kmk":                                        # A[k,m,k]: a repeated label, each position its own stride
        rep.append(run)
        run *= ext[l]
    A_rep = W.TensorSpec(("k", "m", "k"), (ext["k"], ext["m"], ext["k"]), tuple(rep), 0, run)
    t = W.tensor
    cases = [
        ("t7_all_contracted", t("kl", ext), t("lk", ext), t("", ext)),
        ("t8_zero_mode_A", t("", ext), t("nm", ext), t("mn", ext)),
        ("t8_zero_mode_all", t("", ext), t("", ext), t("", ext)),
        ("t9_one_mode", t("k", ext), t("k", ext), t("", ext)),
        ("t9_one_mode_outer", t("m", ext), t("n", ext), t("nm", ext)),
        ("t10_subtensors_same_modes", _sub("mk", ext, big), _sub("kn", ext, big), _sub("mn", ext, big)),
        ("t11_subtensors_fewer_modes", _sub("mk", ext, big, fixed={"x": 2}), _sub("kn", ext, big, fixed={"h": 1}),
         _sub("mn", ext, big, fixed={"l": 3})),
        ("t13_subtensors_negative", _sub("mk", ext, big, negative="k"), _sub("kn", ext, big, negative="kn"),
         _sub("mn", ext, big, negative="m")),
        ("t17_mixed_signs_fewer_modes", _sub("mkl", ext, big, fixed={"x": 1}, negative="l"), _sub("lkn", ext, big, negative="n"),
         _sub("nm", ext, big, fixed={"h": 2}, negative="n")),
        ("t21_zero_stride_A", t("mk", ext, strides={"m": 0, "k": 1}), t("kn", ext), t("mn", ext)),
        ("t21_zero_stride_B_k", t("mk", ext), t("kn", ext, strides={"k": 0, "n": 1}), t("mn", ext)),
        ("t23_repeated_label", A_rep, t("kn", ext), t("nm", ext)),
        ("t24_hadamard_free", t("hm", ext), t("nh", ext), t("mhn", ext)),
        ("t25_hadamard_contracted", t("hkm", ext), t("khl", ext), t("hlm", ext)),
    ]
    out = []
    for name, A, B, D in cases:
        for dtype in ("f64", "c128", "c64"):
            out.append(W.Problem("%s_%s" % (name, dtype), dtype, A, B, D, alpha=2.0, beta=-1.0,
                                 opA=int(dtype in COMPLEX), seed=W.BASE_SEED + 31))
    return out


@pytest.mark.parametrize("p", _paper_list_cases(), ids=lambda p: p.name)
def test_shapes_of_the_papers_test_list(p):
    """The shapes of the paper's own test list (Sec. "Testing") that the other tests do not reach:
    everything contracted, tensors with zero modes and with one mode, sub-tensors with as many and
    with fewer modes than their parents, with negative and mixed strides, a zero stride in an input,
    a repeated label, Hadamard labels combined with free and with contracted ones — on every kernel
    path that accepts the plan, integer inputs bit for bit."""
    from gpu_helpers import run_gpu, say
    a, b, c = W.make_operands(p, "ints")
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    ran = 0
    for path in (None, GENERIC, GETT, STREAM):
        say("%s path=%s" % (p.name, path))
        try:
            got = run_gpu(p, a, b, c, force_path=path)
        except Exception as exc:
            if path in (GETT, STREAM) and getattr(exc, "code", None) == REFUSED:
                say("  (path declined this plan)")
                continue
            raise
        ran += 1
        assert gaps_untouched(p, c, got)
        assert np.array_equal(W.strided_view(got, p.D), W.strided_view(truth, p.D)), path
    assert ran >= 2


def _batch_lane_cases():
    t = W.tensor
    out = []
    for dtype in ("f64", "f32", "c128"):
        for k in (1, 2, 4):
            e = {"h": 512, "i": 12, "j": 8, "k": k}
            out.append(W.Problem("batch_lanes_%s_k%d" % (dtype, k), dtype, t("hki", e), t("hkj", e), t("hij", e),
                                 alpha=2.0, beta=-1.0, opA=int(dtype == "c128"), opB=int(dtype == "c128" and k == 2),
                                 seed=W.BASE_SEED + 41))
        # two batch modes that do not fuse (padded), four contracted terms from two modes, A walked backwards along g
        e = {"g": 16, "h": 32, "i": 6, "j": 10, "p": 2, "q": 2}
        A = t("ghpqi", e, strides={"g": -1, "h": 20, "p": 700, "q": 1400, "i": 2800})
        B = t("ghqpj", e, strides={"g": 1, "h": 16, "q": 512, "p": 1024, "j": 2048})
        D = t("ghji", e, strides={"g": 1, "h": 17, "j": 600, "i": 6000})
        out.append(W.Problem("batch_lanes_%s_two_modes" % dtype, dtype, A, B, D, alpha=-1.0, beta=0.0, seed=W.BASE_SEED + 42))
    return out


@pytest.mark.parametrize("p", _batch_lane_cases(), ids=lambda p: p.name)
def test_streaming_tiles_with_batch_lanes(p):
    """Low-intensity batched products whose batch modes are the fastest in A, B and D: the streaming
    tile's lanes all run along batch modes, nothing is staged through LDS and every lane reads its
    own operand rows (the LDS-free blocked kernel).  The plan must take that tile by itself; every
    other path must agree; integer inputs bit for bit."""
    from gpu_helpers import GpuProduct, run_gpu, say
    import paper_2601_07827_amd as T
    gp = GpuProduct(p)
    try:
        assert gp.get(T.TCX_KEY_PATH) == STREAM and gp.get(T.TCX_KEY_VARIANT) == 1 and gp.get(T.TCX_KEY_TILE_M) == 256
    finally:
        gp.close()
    a, b, c = W.make_operands(p, "ints")
    truth, S = run_oracle(p, a, b, c, oracle.MODE_TRUTH, want_S=True)
    for path, variant in ((None, None), (GENERIC, None), (STREAM, 0), (GETT, None)):
        say("%s path=%s variant=%s" % (p.name, path, variant))
        try:
            got = run_gpu(p, a, b, c, force_path=path, variant=variant, c_null=(p.beta == 0))
        except Exception as exc:
            if path == GETT and getattr(exc, "code", None) == REFUSED:
                continue
            raise
        assert gaps_untouched(p, c, got)
        assert np.array_equal(W.strided_view(got, p.D), W.strided_view(truth, p.D)), (path, variant)


def test_small_tiles_on_random_network_layouts():
    """Seeded random tensor-network-like products (M, N, K each a product of modes with extents
    2 - 16, every tensor in its own random memory order, sometimes a batch mode) on the small
    two-phase tiles, unsplit and with K in two: whichever of the one-element and the paired-load
    kernels the layout admits must reproduce the oracle bit for bit on integer inputs, and paired
    loads must actually occur."""
    import torch
    from gpu_helpers import GpuProduct, say
    import paper_2601_07827_amd as T
    rng = np.random.default_rng(20260107)
    runs = paired = 0
    for case in range(30):
        def modes(prefix, target):
            out, left, i = [], target, 0
            while left > 1:
                e = int(rng.choice([x for x in (2, 4, 8, 16) if left % x == 0]))
                out.append(("%s%d" % (prefix, i), e))
                left //= e
                i += 1
            return out
        Mm, Nm = modes("m", int(rng.choice([64, 128, 256]))), modes("n", int(rng.choice([64, 128])))
        Km = modes("k", int(rng.choice([16, 32, 64])))
        Hm = [("h0", int(rng.choice([2, 3])))] if rng.random() < 0.3 else []
        ext = dict(Mm + Nm + Km + Hm)

        def layout(labels):
            labels = list(labels)
            rng.shuffle(labels)
            order = list(labels)
            rng.shuffle(order)
            return W.tensor(labels, ext, memory_order=order)
        p = W.Problem("network%d" % case, "f64", layout([l for l, _ in Hm + Mm + Km]), layout([l for l, _ in Hm + Km + Nm]),
                      layout([l for l, _ in Hm + Mm + Nm]), alpha=2.0, beta=-1.0, seed=W.BASE_SEED + 100 + case)
        a, b, c = W.make_operands(p, "ints")
        truth, _ = run_oracle(p, a, b, c, oracle.MODE_TRUTH)
        for variant in (10, 11):
            for parts in (None, 2):
                try:
                    gp = GpuProduct(p, GETT, variant, parts)
                except T.TcxError as exc:
                    assert exc.code == T.TCX_ERR_PLAN_REFUSED            # k offsets that do not repeat from slab to slab
                    continue
                try:
                    say("%s shape %d parts %s" % (p.name, variant, parts))
                    dA, dB, dD = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda(), torch.from_numpy(c.copy()).cuda()
                    gp.execute(dA, dB, dD, dD)
                    torch.cuda.synchronize()
                    runs += 1
                    paired += gp.last_gather_width == 2
                    assert np.array_equal(W.strided_view(dD.cpu().numpy(), p.D), W.strided_view(truth, p.D))
                finally:
                    gp.close()
    assert runs >= 60 and paired >= runs // 3
