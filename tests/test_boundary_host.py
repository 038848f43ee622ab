"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, reports each error class before any HIP call, follows the paper's
conventions (Sec. "Error Handling": codes + text, outputs by pointer, destroy nulls the
handle), agrees with the oracle's independent validation, and the index analyser produces
the expected fused shapes.  No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2601_07827_amd as T
import workloads as W
from helpers import desc, random_problem

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "tcx.h")).read()


def test_library_exports_every_declared_symbol():
    declared = sorted(set(re.findall(r"^(?:tcx_error_t|int|size_t)\s+(tcx_[a-z_]+)\s*\(", HEADER, re.M)))
    assert len(declared) >= 17
    lib = ctypes.CDLL(T.binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), "libtcx.so lacks %s" % name
    assert sorted(T.binding.EXPORTS) == declared


def test_header_constants_match_binding():
    for name, value in re.findall(r"\b(TCX_[A-Z0-9_]+)\s*=\s*(\d+)", HEADER):
        assert getattr(T, name) == int(value), name


def test_explain_error_and_check_success():
    assert T.tcx_check_success(0) and not T.tcx_check_success(T.TCX_ERR_D_ALIASING)
    texts = {T.tcx_explain_error(c) for c in range(21)}
    assert len(texts) == 21 and all(texts)
    assert "unknown" in T.tcx_explain_error(12345)
    # truncation keeps a NUL and returns the full length
    buf = ctypes.create_string_buffer(8)
    need = T.raw().tcx_explain_error(T.TCX_ERR_CD_MISMATCH, 8, buf)
    assert need > 8 and len(buf.value) == 7


@pytest.fixture()
def handle():
    h = T.tcx_create_handle()
    yield h
    T.tcx_destroy_handle(h)


def _code(fn, *a):
    try:
        fn(*a)
    except T.TcxError as e:
        return e.code
    return 0


def test_handle_lifecycle_and_null_conventions(handle):
    lib = T.raw()
    assert lib.tcx_create_handle(None) == T.TCX_ERR_NULL_ARG
    assert lib.tcx_destroy_handle(None) == T.TCX_ERR_NULL_ARG
    h2 = ctypes.c_ssize_t(T.tcx_create_handle())
    assert lib.tcx_destroy_handle(ctypes.byref(h2)) == 0 and h2.value == 0        # destroy nulls the handle
    assert lib.tcx_destroy_handle(ctypes.byref(h2)) == T.TCX_ERR_INVALID_HANDLE
    stale = ctypes.c_ssize_t(123456)
    assert lib.tcx_destroy_handle(ctypes.byref(stale)) == T.TCX_ERR_INVALID_HANDLE
    # a tensor-info handle is not a library handle
    ti = T.tcx_create_tensor_info(handle, T.TCX_F64, [2], [1])
    assert _code(T.tcx_create_executor, ti, 0) == T.TCX_ERR_INVALID_HANDLE
    assert _code(T.tcx_destroy_product, ti) == T.TCX_ERR_INVALID_HANDLE
    assert T.tcx_destroy_tensor_info(ti) == 0


def test_tensor_info_errors_and_roundtrip(handle):
    assert _code(T.tcx_create_tensor_info, handle, 7, [2], [1]) == T.TCX_ERR_BAD_DTYPE
    assert _code(T.tcx_create_tensor_info, handle, 6, [2], [1]) == T.TCX_ERR_BAD_DTYPE
    assert _code(T.tcx_create_tensor_info, handle, -1, [2], [1]) == T.TCX_ERR_BAD_DTYPE
    assert _code(T.tcx_create_tensor_info, handle, T.TCX_F64, [1] * 33, [1] * 33) == T.TCX_ERR_BAD_NMODE
    assert _code(T.tcx_create_tensor_info, handle, T.TCX_F64, [3, 0], [1, 3]) == T.TCX_ERR_BAD_EXTENT
    assert _code(T.tcx_create_tensor_info, handle, T.TCX_F64, [3, -2], [1, 3]) == T.TCX_ERR_BAD_EXTENT
    assert _code(T.tcx_create_tensor_info, 0, T.TCX_F64, [3], [1]) == T.TCX_ERR_INVALID_HANDLE
    ti = T.tcx_create_tensor_info(handle, T.TCX_C128, [3, 4, 5], [20, -5, 1])
    assert T.tcx_tensor_info_get(ti) == (T.TCX_C128, [3, 4, 5], [20, -5, 1])
    scalar = T.tcx_create_tensor_info(handle, T.TCX_F32, [], [])
    assert T.tcx_tensor_info_get(scalar) == (T.TCX_F32, [], [])
    T.tcx_destroy_tensor_info(ti)
    T.tcx_destroy_tensor_info(scalar)


def _product_code(handle, A, B, C, D, ops=(0, 0, 0, 0), dtypes=(1, 1, 1, 1), prec=0):
    infos = [T.tcx_create_tensor_info(handle, dt, t[0], t[1]) for dt, t in zip(dtypes, (A, B, C, D))]
    try:
        p = T.tcx_create_product(handle, ops[0], infos[0], A[2], ops[1], infos[1], B[2], ops[2], infos[2], C[2],
                                 ops[3], infos[3], D[2], prec)
        T.tcx_destroy_product(p)
        return 0
    except T.TcxError as e:
        return e.code
    finally:
        for i in infos:
            T.tcx_destroy_tensor_info(i)


def test_product_validation_errors(handle):
    ext = dict(m=3, n=4, k=5, x=2)
    ids = dict(m=1, n=2, k=3, x=4)
    t = lambda labels, **kw: desc(W.tensor(labels, ext, **kw), ids)
    A, B, D = t("mk"), t("kn"), t("mn")
    assert _product_code(handle, A, B, D, D) == 0
    assert _product_code(handle, ([3, 6], [1, 3], [1, 3]), B, D, D) == T.TCX_ERR_EXTENT_MISMATCH       # appendix test 26
    assert _product_code(handle, A, B, t("nm"), D) == T.TCX_ERR_CD_MISMATCH                           # appendix test 27
    assert _product_code(handle, A, B, t("mn", strides=dict(m=1, n=4)), D) == T.TCX_ERR_CD_MISMATCH
    assert _product_code(handle, A, B, t("nm", strides=dict(m=1, n=3)), D) == 0                        # same layout, listed differently
    al = t("mn", strides=dict(m=1, n=2))
    assert _product_code(handle, A, B, al, al) == T.TCX_ERR_D_ALIASING                                # appendix test 28
    z = t("mn", strides=dict(m=0, n=1))
    assert _product_code(handle, A, B, z, z) == T.TCX_ERR_D_ALIASING
    assert _product_code(handle, t("mkx"), B, D, D) == 0                                              # Case 4: x summed inside A
    assert _product_code(handle, A, B, t("mnx"), t("mnx")) == 0                                       # Case 5: x broadcasts
    assert _product_code(handle, A, B, D, D, dtypes=(1, 0, 1, 1)) == T.TCX_ERR_DTYPE_MIX
    assert _product_code(handle, A, B, D, D, ops=(0, 0, 0, 1)) == T.TCX_ERR_UNSUPPORTED_OP            # opD must be identity
    assert _product_code(handle, A, B, D, D, ops=(5, 0, 0, 0)) == T.TCX_ERR_UNSUPPORTED_OP
    assert _product_code(handle, A, B, D, D, prec=3) == T.TCX_ERR_UNSUPPORTED_PRECISION
    # zero stride in an input is a broadcast and is legal
    assert _product_code(handle, t("mk", strides=dict(m=0, k=1)), B, D, D) == 0
    # repeated label inside a tensor (Case 3) is accepted; with unequal extents it is not
    assert _product_code(handle, ([5, 3, 5], [1, 5, 15], [3, 1, 3]), B, D, D) == 0
    assert _product_code(handle, ([5, 3, 4], [1, 5, 15], [3, 1, 3]), B, D, D) == T.TCX_ERR_EXTENT_MISMATCH


def test_config3_literal_stride_reading_is_rejected_as_aliasing(handle):
    p = W.config3()
    ids = W.label_ids(p)
    bad = ([37, 53, 61], [1, 37, 2], [ids[l] for l in "abc"])
    assert _product_code(handle, desc(p.A, ids), desc(p.B, ids), bad, bad, dtypes=(0, 0, 0, 0)) == T.TCX_ERR_D_ALIASING


ORACLE_TO_TCX = {oracle.V_OK: 0, oracle.V_EXTENT_MISMATCH: T.TCX_ERR_EXTENT_MISMATCH,
                 oracle.V_CD_MISMATCH: T.TCX_ERR_CD_MISMATCH, oracle.V_D_ALIASING: T.TCX_ERR_D_ALIASING}


def test_library_and_oracle_agree_on_validity(handle):
    """Random problems, each possibly broken in one way; the two independent validators must
    put it in the same class."""
    rng = np.random.default_rng(2601)
    seen = set()
    for i in range(300):
        p = random_problem(rng, "f64", max_group=2, max_extent=4, allow_neg=(i % 2 == 0))
        ids = W.label_ids(p)
        A, B, D = [list(map(list, desc(t, ids))) for t in (p.A, p.B, p.D)]
        C = [list(D[0]), list(D[1]), list(D[2])]
        kind = i % 6
        if kind == 1 and A[0]:
            A[0][int(rng.integers(len(A[0])))] += 1                      # extent mismatch (or isolated if unique)
        elif kind == 2 and D[0]:
            j = int(rng.integers(len(D[0])))
            C[1][j] = C[1][j] * 2 + 1                                    # C laid out differently
        elif kind == 3 and len(D[0]) >= 2:
            D[1][0] = D[1][1]
            C[1][0] = C[1][1]                                            # two modes of D share a stride
        elif kind == 4:
            A[0].append(2); A[1].append(1000); A[2].append(999)          # label only in A: a reduction (Case 4), valid
        elif kind == 5:
            for t_ in (C, D):
                t_[0].append(2); t_[1].append(5000); t_[2].append(998)   # label only in D: a broadcast (Case 5), valid
        v = oracle.validate(tuple(A), tuple(B), tuple(C), tuple(D))
        code = _product_code(handle, A, B, C, D)
        assert code == ORACLE_TO_TCX[v], (i, kind, A, B, C, D, oracle.V_NAMES[v], code)
        seen.add(v)
    assert seen == set(ORACLE_TO_TCX)


def test_execute_argument_checks_without_a_device(handle):
    ext = dict(m=3, n=4, k=5)
    ids = dict(m=1, n=2, k=3)
    infos = [T.tcx_create_tensor_info(handle, T.TCX_F64, *desc(W.tensor(l, ext), ids)[:2]) for l in ("mk", "kn", "mn")]
    labs = [[ids[c] for c in l] for l in ("mk", "kn", "mn")]
    prod = T.tcx_create_product(handle, 0, infos[0], labs[0], 0, infos[1], labs[1], 0, infos[2], labs[2], 0, infos[2], labs[2])
    ex = T.tcx_create_executor(handle, 0)
    lib = T.raw()
    one = ctypes.c_double(1.0)
    zero = ctypes.c_double(0.0)
    p1, p0 = ctypes.cast(ctypes.pointer(one), ctypes.c_void_p), ctypes.cast(ctypes.pointer(zero), ctypes.c_void_p)
    fake = ctypes.c_void_p(4096)
    assert lib.tcx_execute_product(prod, ex, None, None, fake, fake, p0, None, fake) == T.TCX_ERR_NULL_ARG   # alpha
    assert lib.tcx_execute_product(prod, ex, None, p1, fake, fake, p0, None, None) == T.TCX_ERR_NULL_ARG     # D
    assert lib.tcx_execute_product(prod, ex, None, p1, None, fake, p0, None, fake) == T.TCX_ERR_NULL_ARG     # A with alpha != 0
    assert lib.tcx_execute_product(prod, ex, None, p1, fake, fake, p1, None, fake) == T.TCX_ERR_NULL_ARG     # C with beta != 0
    assert lib.tcx_execute_product(prod, 0, None, p1, fake, fake, p0, None, fake) == T.TCX_ERR_INVALID_HANDLE
    assert lib.tcx_execute_product(ex, ex, None, p1, fake, fake, p0, None, fake) == T.TCX_ERR_INVALID_HANDLE
    if not T.tcx_handle_has_device(handle):
        # beta == 0 with C == NULL is legal; without a GPU the call stops at NO_DEVICE, before any launch
        assert lib.tcx_execute_product(prod, ex, None, p1, fake, fake, p0, None, fake) == T.TCX_ERR_NO_DEVICE
    for i in infos:
        T.tcx_destroy_tensor_info(i)
    assert T.tcx_destroy_product(prod) == 0 and T.tcx_destroy_executor(ex) == 0


def test_product_get_conventions(handle):
    p = W.config1()
    ids = W.label_ids(p)
    infos = [T.tcx_create_tensor_info(handle, T.TCX_F64, t.extents, t.strides) for t in (p.A, p.B, p.D)]
    labs = [[ids[l] for l in t.labels] for t in (p.A, p.B, p.D)]
    prod = T.tcx_create_product(handle, 0, infos[0], labs[0], 0, infos[1], labs[1], 0, infos[2], labs[2], 0, infos[2], labs[2])
    lib = T.raw()
    v = ctypes.c_int64(0)
    n = ctypes.c_size_t(4)
    assert lib.tcx_product_get(prod, T.TCX_KEY_SIZE_M, ctypes.byref(v), ctypes.byref(n)) == T.TCX_ERR_BUFFER_TOO_SMALL
    assert n.value == 8
    assert lib.tcx_product_get(prod, 999, ctypes.byref(v), ctypes.byref(n)) == T.TCX_ERR_BAD_KEY
    assert lib.tcx_product_get(prod, T.TCX_KEY_SIZE_M, ctypes.byref(v), None) == T.TCX_ERR_NULL_ARG
    assert T.tcx_product_get(prod, T.TCX_KEY_SIZE_M) == 576
    assert _code(T.tcx_product_set, prod, T.TCX_KEY_VARIANT, 99) == T.TCX_ERR_PLAN_REFUSED
    T.tcx_destroy_product(prod)
    for i in infos:
        T.tcx_destroy_tensor_info(i)


# ---- the analyser's fused shapes for the five configurations -----------------------------------
def _plan(handle, p):
    ids = W.label_ids(p)
    dt = {"f32": 0, "f64": 1, "c128": 3}[p.dtype]
    infos = [T.tcx_create_tensor_info(handle, dt, t.extents, t.strides) for t in (p.A, p.B, p.D)]
    labs = [[ids[l] for l in t.labels] for t in (p.A, p.B, p.D)]
    prod = T.tcx_create_product(handle, p.opA, infos[0], labs[0], p.opB, infos[1], labs[1], p.opC, infos[2], labs[2],
                                0, infos[2], labs[2])
    for i in infos:
        T.tcx_destroy_tensor_info(i)
    out = {k: T.tcx_product_get(prod, getattr(T, "TCX_KEY_" + k)) for k in
           ("PATH", "SIZE_H", "SIZE_M", "SIZE_N", "SIZE_K", "MODES_H", "MODES_M", "MODES_N", "MODES_K",
            "A_K_FASTEST", "B_K_FASTEST", "D_N_FASTEST", "TILE_M", "TILE_N", "TILE_K", "GRID", "BLOCK", "VARIANT",
            "SPLIT_K", "LAUNCHES", "GATHER_WIDTH")}
    T.tcx_destroy_product(prod)
    return out


def test_analyser_config1(handle):
    a = _plan(handle, W.config1())
    # nothing fuses: (a,i), (b,j), (c,d); modes are (extent, strideA, strideB, strideD), fastest first
    assert a["MODES_M"] == [(24, 1, 0, 1), (24, 576, 0, 576)]
    assert a["MODES_N"] == [(24, 0, 24, 24), (24, 0, 13824, 13824)]
    assert a["MODES_K"] == [(24, 24, 1, 0), (24, 13824, 576, 0)]
    assert (a["A_K_FASTEST"], a["B_K_FASTEST"], a["D_N_FASTEST"]) == (0, 1, 0)
    assert a["PATH"] == T.TCX_PATH_GETT_MFMA


def test_analyser_config2_is_one_gemm(handle):
    a = _plan(handle, W.config2())
    assert a["MODES_M"] == [(36864, 1, 0, 1)]
    assert a["MODES_K"] == [(36864, 36864, 1, 0)]
    assert a["MODES_N"] == [(4096, 0, 36864, 36864)]
    assert a["MODES_H"] == []
    assert (a["A_K_FASTEST"], a["B_K_FASTEST"], a["D_N_FASTEST"]) == (0, 1, 0)
    assert (a["TILE_M"], a["TILE_N"], a["TILE_K"], a["GRID"]) == (256, 128, 16, 4608)


def test_analyser_config3(handle):
    a = _plan(handle, W.config3())
    # A: e=1, b=41, a=2173, d=80401; B: e=1, c=41, d=2501; D: c=2, a=122, b=4514.  Nothing fuses.
    assert a["MODES_K"] == [(41, 1, 1, 0), (29, 80401, 2501, 0)]
    assert a["MODES_N"] == [(61, 0, 41, 2)]
    assert sorted(a["MODES_M"]) == sorted([(37, 2173, 0, 122), (53, 41, 0, 4514)])
    assert (a["A_K_FASTEST"], a["B_K_FASTEST"], a["D_N_FASTEST"]) == (1, 1, 1)
    assert (a["SIZE_M"], a["SIZE_N"], a["SIZE_K"]) == (1961, 61, 1189)


def test_analyser_config4(handle):
    a = _plan(handle, W.config4())
    assert a["MODES_H"] == [(512, 1, 1, 1)]
    assert a["MODES_M"] == [(96, 49152, 0, 512)]
    assert a["MODES_N"] == [(96, 0, 49152, 49152)]
    assert a["MODES_K"] == [(96, 512, 512, 0)]
    b = _plan(handle, W.config4(h_slowest=True))
    assert b["MODES_H"] == [(512, 9216, 9216, 9216)]
    assert b["MODES_K"] == [(96, 1, 1, 0)] and b["MODES_M"] == [(96, 96, 0, 1)]


def test_analyser_config5_fuses_only_where_the_layouts_agree(handle):
    p = W.config5()
    a = _plan(handle, p)
    assert (a["SIZE_M"], a["SIZE_N"], a["SIZE_K"]) == (1024, 1024, 1024)
    for key, tensors in (("MODES_M", (1, 3)), ("MODES_N", (2, 3)), ("MODES_K", (1, 2))):
        modes = a[key]
        prod = 1
        for m in modes:
            prod *= m[0]
            assert m[0] in (4, 16, 64, 256, 1024)
            for t in tensors:
                assert m[t] != 0
        assert prod == 1024
        # no fusable pair is left
        for x in modes:
            for y in modes:
                if x is not y:
                    assert not all(y[t] == x[t] * x[0] for t in (1, 2, 3))


def test_analyser_drops_extent_one_and_merges_repeated_labels(handle):
    ids = dict(k=1, i=2, j=3, u=4)
    # A[k,i,k,u] with u of extent 1; strides (1, 4, 12, 48) -> merged k stride 13
    A = ([4, 3, 4, 1], [1, 4, 12, 48], [1, 2, 1, 4])
    B = ([4, 5, 1], [1, 4, 20], [1, 3, 4])
    D = ([5, 3], [1, 5], [3, 2])
    infos = [T.tcx_create_tensor_info(handle, T.TCX_F64, t[0], t[1]) for t in (A, B, D)]
    prod = T.tcx_create_product(handle, 0, infos[0], A[2], 0, infos[1], B[2], 0, infos[2], D[2], 0, infos[2], D[2])
    assert T.tcx_product_get(prod, T.TCX_KEY_MODES_K) == [(4, 13, 1, 0)]
    assert T.tcx_product_get(prod, T.TCX_KEY_MODES_M) == [(3, 4, 0, 5)]
    assert T.tcx_product_get(prod, T.TCX_KEY_MODES_N) == [(5, 0, 4, 1)]
    assert T.tcx_product_get(prod, T.TCX_KEY_MODES_H) == []
    T.tcx_destroy_product(prod)
    for i in infos:
        T.tcx_destroy_tensor_info(i)


def test_planner_routes_each_configuration(handle):
    """Which kernel form the plan takes (a plan-only handle assumes 256 CUs).  The two-phase kernel
    needs, for an operand whose lanes run along k, the same relative k offsets in every whole slab;
    plans that fail this fall back to the classic staged kernel."""
    c2 = _plan(handle, W.config2())
    # one 256x128 tile per workgroup, eight waves, 4608 workgroups enqueued in 18 rounds of 256
    assert (c2["VARIANT"], c2["BLOCK"], c2["GRID"], c2["SPLIT_K"], c2["LAUNCHES"]) == (0, 512, 4608, 1, 18)
    c5 = _plan(handle, W.config5())
    # 256 tiles of 64x64, K in two halves = 512 items, two per workgroup, summed inside it: one launch
    assert (c5["TILE_M"], c5["TILE_N"], c5["BLOCK"], c5["GRID"], c5["SPLIT_K"], c5["LAUNCHES"]) == (64, 64, 512, 256, 2, 1)
    c4 = _plan(handle, W.config4())
    # batches fastest in memory: tiles of four consecutive batches x 48 x 48 (128 groups of batches x 4 tiles),
    # two per workgroup, K whole
    assert (c4["TILE_M"], c4["TILE_N"], c4["TILE_K"], c4["BLOCK"], c4["GRID"], c4["SPLIT_K"], c4["LAUNCHES"]) == (48, 48, 4, 512, 256, 1, 1)
    c4s = _plan(handle, W.config4(h_slowest=True))
    # batches slowest: 512 contiguous matrices, one 96x96 complex tile each, two per workgroup
    assert (c4s["TILE_M"], c4s["TILE_N"], c4s["TILE_K"], c4s["BLOCK"], c4s["GRID"], c4s["LAUNCHES"]) == (96, 96, 8, 512, 256, 1)
    c1 = _plan(handle, W.config1())
    # B's lanes run along k = (c, d) with extent 24: slabs of 16 do not repeat -> classic kernel; its 324
    # short tiles of 32 x 32 already give every CU a workgroup: one launch, K whole, no workspace
    assert (c1["TILE_M"], c1["BLOCK"], c1["SPLIT_K"], c1["LAUNCHES"], c1["GRID"]) == (32, 256, 1, 1, 324)
    c3 = _plan(handle, W.config3())
    # K = (e41, d29): slabs of 16 do not repeat; 124 tiles do not fill the chip: K is cut, plus the reduction launch
    assert c3["BLOCK"] == 256 and c3["SPLIT_K"] > 1 and c3["LAUNCHES"] == 2


def test_tile_modes_cover_a_cache_line_of_every_tensor(handle):
    """Order of the modes inside a group: a tile's rows are the first modes of M (columns: of N, slab:
    of K).  For a tensor network with random mode orders the fastest modes of D *and* of the operand
    must both come first, or every access to one of them touches a 128-byte line for one element.
    (Modes are (extent, strideA, strideB, strideD).)"""
    for seed in range(1000, 1008):
        p = W.config5(perm_seed=seed)
        a = _plan(handle, p)
        line = 16                                             # fp64 elements per 128 bytes

        def line_strides(which):
            modes = [m for g in ("MODES_M", "MODES_N", "MODES_K") for m in a[g] if m[which] != 0]
            out, have = [], 1
            for m in sorted(modes, key=lambda m: abs(m[which])):
                if have >= line:
                    break
                out.append(abs(m[which]))
                have *= m[0]
            return out

        def first_modes(group, count):
            got, have = [], 1
            for m in a[group]:
                if have >= count:
                    break
                got.append(m)
                have *= m[0]
            return got

        tile = {"MODES_M": first_modes("MODES_M", a["TILE_M"]), "MODES_N": first_modes("MODES_N", a["TILE_N"]),
                "MODES_K": first_modes("MODES_K", a["TILE_K"])}
        for which, groups in ((1, ("MODES_M", "MODES_K")), (2, ("MODES_N", "MODES_K")), (3, ("MODES_M", "MODES_N"))):
            inside = [abs(m[which]) for g in groups for m in tile[g]]
            # the fastest mode always; the rest of the line unless the other tensor's line has
            # used up the tile (a slab holds only 16 contracted indices)
            assert line_strides(which)[0] in inside, (seed, which, tile)
        # ... and then both operands can be gathered two contiguous elements per load
        assert a["GATHER_WIDTH"] == 2, seed
    assert _plan(handle, W.config5())["GATHER_WIDTH"] == 2
    assert _plan(handle, W.config2())["GATHER_WIDTH"] == 1      # the 256 x 128 tile has no paired twin
    assert _plan(handle, W.config4())["GATHER_WIDTH"] == 1      # 16-byte elements


def test_forcing_a_shape_the_plan_cannot_take_is_refused(handle):
    p = W.config1()
    ids = W.label_ids(p)
    infos = [T.tcx_create_tensor_info(handle, 1, t.extents, t.strides) for t in (p.A, p.B, p.D)]
    labs = [[ids[l] for l in t.labels] for t in (p.A, p.B, p.D)]
    prod = T.tcx_create_product(handle, 0, infos[0], labs[0], 0, infos[1], labs[1], 0, infos[2], labs[2], 0, infos[2], labs[2])
    before = T.tcx_product_get(prod, T.TCX_KEY_VARIANT)
    with pytest.raises(T.TcxError) as e:
        T.tcx_product_set(prod, T.TCX_KEY_VARIANT, 0)            # two-phase 256x128: needs slab-periodic k offsets
    assert e.value.code == T.TCX_ERR_PLAN_REFUSED and "plan cannot take" in str(e.value)
    assert T.tcx_product_get(prod, T.TCX_KEY_VARIANT) == before   # the plan is unchanged
    T.tcx_product_set(prod, T.TCX_KEY_VARIANT, 2)                # a classic shape is fine
    assert T.tcx_product_get(prod, T.TCX_KEY_VARIANT) == 2 and T.tcx_product_get(prod, T.TCX_KEY_SPLIT_K) == 1
    T.tcx_destroy_product(prod)


def test_key_value_stores_on_every_object(handle):
    """Sec. "Virtual Key-Value Stores": one set/get/clear interface on every object and on a bare
    store; free-form keys hold arbitrary binary values; the library's own keys are a layer over
    state kept elsewhere (the plan, the status)."""
    p = W.config1()
    ids = W.label_ids(p)
    infos = [T.tcx_create_tensor_info(handle, 1, t.extents, t.strides) for t in (p.A, p.B, p.D)]
    labs = [[ids[l] for l in t.labels] for t in (p.A, p.B, p.D)]
    prod = T.tcx_create_product(handle, 0, infos[0], labs[0], 0, infos[1], labs[1], 0, infos[2], labs[2], 0, infos[2], labs[2])
    ex = T.tcx_create_executor(handle, 0)
    bare = T.tcx_create_attr(handle)
    U = T.TCX_KEY_USER
    objects = [handle, ex, infos[0], prod, bare]
    for n, obj in enumerate(objects):
        assert _code(T.tcx_attr_get, obj, U + 7) == T.TCX_ERR_BAD_KEY                   # never set
        blob = bytes(range(n, n + 40)) + b"\x00tail"
        T.tcx_attr_set(obj, U + 7, blob)
        T.tcx_attr_set(obj, U + 8, b"")                                                # an empty value is a value
    for n, obj in enumerate(objects):                                                   # stores are per object
        assert T.tcx_attr_get(obj, U + 7) == bytes(range(n, n + 40)) + b"\x00tail"
        assert T.tcx_attr_get(obj, U + 8) == b""
    T.tcx_attr_set(bare, U + 7, b"replaced")
    assert T.tcx_attr_get(bare, U + 7) == b"replaced"
    # the two-call protocol of the C interface: size query, short buffer, exact buffer
    n = ctypes.c_size_t(0)
    assert T.raw().tcx_attr_get(bare, U + 7, None, ctypes.byref(n)) == T.TCX_ERR_NULL_ARG and n.value == 8
    buf = ctypes.create_string_buffer(4)
    n = ctypes.c_size_t(4)
    assert T.raw().tcx_attr_get(bare, U + 7, buf, ctypes.byref(n)) == T.TCX_ERR_BUFFER_TOO_SMALL and n.value == 8
    assert T.raw().tcx_attr_get(bare, U + 7, buf, None) == T.TCX_ERR_NULL_ARG
    assert T.raw().tcx_attr_set(bare, U + 9, None, 3) == T.TCX_ERR_NULL_ARG
    T.tcx_attr_clear(bare, U + 7)
    assert _code(T.tcx_attr_get, bare, U + 7) == T.TCX_ERR_BAD_KEY
    assert _code(T.tcx_attr_clear, bare, U + 7) == T.TCX_ERR_BAD_KEY
    assert T.tcx_attr_get(bare, U + 8) == b""                                           # other keys stay
    # the library's own keys: on a product they are the plan's
    assert T.tcx_attr_get(prod, T.TCX_KEY_SIZE_K) == 576 == T.tcx_product_get(prod, T.TCX_KEY_SIZE_K)
    assert T.tcx_attr_get(prod, T.TCX_KEY_MODES_K) == T.tcx_product_get(prod, T.TCX_KEY_MODES_K)
    planned = {k: T.tcx_product_get(prod, k) for k in (T.TCX_KEY_PATH, T.TCX_KEY_VARIANT, T.TCX_KEY_SPLIT_K)}
    T.tcx_attr_set(prod, T.TCX_KEY_VARIANT, 2)                                          # a tuning override ...
    T.tcx_attr_set(prod, T.TCX_KEY_SPLIT_K, 2)
    assert (T.tcx_product_get(prod, T.TCX_KEY_VARIANT), T.tcx_product_get(prod, T.TCX_KEY_SPLIT_K)) == (2, 2)
    T.tcx_attr_set(prod, T.TCX_KEY_FORCE_PATH, T.TCX_PATH_GENERIC)
    assert T.tcx_product_get(prod, T.TCX_KEY_PATH) == T.TCX_PATH_GENERIC
    T.tcx_attr_clear(prod, T.TCX_KEY_FORCE_PATH)                                        # ... and back to the analyser's choice
    assert {k: T.tcx_product_get(prod, k) for k in planned} == planned
    assert _code(T.tcx_attr_clear, prod, T.TCX_KEY_SIZE_K) == T.TCX_ERR_BAD_KEY         # not something that can be cleared
    assert _code(T.tcx_attr_set, prod, T.TCX_KEY_SIZE_K, 5) == T.TCX_ERR_BAD_KEY
    assert _code(T.tcx_attr_get, handle, T.TCX_KEY_SIZE_K) == T.TCX_ERR_BAD_KEY         # a handle has no such key
    assert _code(T.tcx_attr_set, ex, T.TCX_KEY_VARIANT, 1) == T.TCX_ERR_BAD_KEY
    # destroyed objects: invalid handle, and their values are gone with them
    assert T.tcx_destroy_attr(bare) == 0
    assert _code(T.tcx_attr_get, bare, U + 8) == T.TCX_ERR_INVALID_HANDLE
    assert _code(T.tcx_attr_set, 0, U, b"x") == T.TCX_ERR_INVALID_HANDLE
    assert _code(T.tcx_destroy_attr, bare) == T.TCX_ERR_INVALID_HANDLE
    assert _code(T.tcx_destroy_attr, prod) == T.TCX_ERR_INVALID_HANDLE                  # wrong object type
    T.tcx_destroy_product(prod)
    T.tcx_destroy_executor(ex)
    for i in infos:
        T.tcx_destroy_tensor_info(i)


# ---- padding of the plan's offset tables ----------------------------------------------------------
def _matrix_product(handle, dtype, m, n, k, a_kfast=False, b_kfast=True):
    e = dict(m=m, n=n, k=k)
    A = W.tensor("mk", e, memory_order="km" if a_kfast else "mk")
    B = W.tensor("kn", e, memory_order="kn" if b_kfast else "nk")
    D = W.tensor("mn", e)
    infos = [T.tcx_create_tensor_info(handle, dtype, t.extents, t.strides) for t in (A, B, D)]
    prod = T.tcx_create_product(handle, 0, infos[0], [1, 3], 0, infos[1], [3, 2], 0, infos[2], [1, 2], 0, infos[2], [1, 2])
    for i in infos:
        T.tcx_destroy_tensor_info(i)
    return prod


def _tile_shapes(handle, dtype):
    """(tile rows, tile columns, slab) of every compiled tile shape of a dtype, read through the
    plan interface on products that each shape accepts (both operand orientations)."""
    shapes = {}
    for a_kfast, b_kfast in ((False, True), (True, True), (False, False), (True, False)):
        prod = _matrix_product(handle, dtype, 768, 768, 64, a_kfast, b_kfast)
        T.tcx_product_set(prod, T.TCX_KEY_FORCE_PATH, T.TCX_PATH_GETT_MFMA)
        for v in range(32):
            try:
                T.tcx_product_set(prod, T.TCX_KEY_VARIANT, v)
            except T.TcxError as exc:
                assert exc.code == T.TCX_ERR_PLAN_REFUSED
                continue
            shapes[v] = tuple(T.tcx_product_get(prod, k) for k in (T.TCX_KEY_TILE_M, T.TCX_KEY_TILE_N, T.TCX_KEY_TILE_K))
        T.tcx_destroy_product(prod)
    return shapes


@pytest.mark.parametrize("dtype", [T.TCX_F64, T.TCX_F32, T.TCX_C128, T.TCX_C64])
def test_offset_tables_hold_a_whole_number_of_tiles_of_every_shape(handle, dtype):
    """The tiled kernels index the rows and columns of a ragged last tile without a mask, so the
    padded tables must reach the end of the last tile of EVERY compiled shape (tiles of 96 and 48
    do not divide a padding unit of 256), for every size of M, N and K."""
    shapes = _tile_shapes(handle, dtype)
    # (the batch-lane shape needs a batch mode; complex64 has no two-phase shapes)
    assert len(shapes) >= {T.TCX_C128: 8, T.TCX_C64: 7}.get(dtype, 12), shapes
    assert {s[0] for s in shapes.values()} >= ({96, 48} if dtype in (T.TCX_C128, T.TCX_C64) else {256, 32})
    for size in list(range(1, 1101)) + [36864, 4096]:
        m, n, k = size, max(2, 1101 - size if size <= 1100 else 4096), 2 + size % 71
        if m * n < 256:
            n = 256
        prod = _matrix_product(handle, dtype, m, n, k)
        T.tcx_product_set(prod, T.TCX_KEY_FORCE_PATH, T.TCX_PATH_GETT_MFMA)
        lenM, lenN, lenK = T.tcx_product_get(prod, T.TCX_KEY_TABLE_ENTRIES)
        for v, (tm, tn, tk) in shapes.items():
            assert -(-m // tm) * tm <= lenM, (m, v, tm, lenM)
            assert -(-n // tn) * tn <= lenN, (n, v, tn, lenN)
            assert -(-k // tk) * tk <= lenK, (k, v, tk, lenK)
        T.tcx_destroy_product(prod)


def test_keys_of_handle_and_executor(handle):
    """Sec. "Virtual Key-Value Stores": the library's own keys on a handle and on an executor."""
    assert T.tcx_attr_get(handle, T.TCX_KEY_DEVICE) == (-1 if not T.tcx_handle_has_device(handle) else T.tcx_attr_get(handle, T.TCX_KEY_DEVICE))
    assert T.tcx_attr_get(handle, T.TCX_KEY_NUM_CU) >= 0
    assert _code(T.tcx_attr_get, handle, T.TCX_KEY_STREAM) == T.TCX_ERR_BAD_KEY
    assert _code(T.tcx_attr_set, handle, T.TCX_KEY_NUM_CU, 5) == T.TCX_ERR_BAD_KEY
    ex = T.tcx_create_executor(handle, 0)
    assert T.tcx_attr_get(ex, T.TCX_KEY_STREAM) == 0
    T.tcx_attr_set(ex, T.TCX_KEY_STREAM, 0x1230)
    assert T.tcx_attr_get(ex, T.TCX_KEY_STREAM) == 0x1230
    T.tcx_attr_set(ex, T.TCX_KEY_STREAM, 0)
    assert T.tcx_attr_get(ex, T.TCX_KEY_WORKSPACE_BYTES) == 0
    if not T.tcx_handle_has_device(handle):
        assert _code(T.tcx_attr_set, ex, T.TCX_KEY_WORKSPACE_BYTES, 4096) == T.TCX_ERR_NO_DEVICE
    assert _code(T.tcx_attr_get, ex, T.TCX_KEY_NUM_CU) == T.TCX_ERR_BAD_KEY
    T.tcx_destroy_executor(ex)


def test_split_products_report_their_workspace(handle):
    """A plan cut along K says how many bytes of partial sums an execution writes; an unsplit plan
    and a two-part split summed inside the workgroup write none."""
    prod = _matrix_product(handle, T.TCX_F64, 64, 64, 4096)
    T.tcx_product_set(prod, T.TCX_KEY_FORCE_PATH, T.TCX_PATH_GETT_MFMA)
    T.tcx_product_set(prod, T.TCX_KEY_VARIANT, 3)                     # 32 x 32 tiles: 4 of them
    T.tcx_product_set(prod, T.TCX_KEY_SPLIT_K, 8)
    assert T.tcx_product_get(prod, T.TCX_KEY_SPLIT_K) == 8
    assert T.tcx_product_get(prod, T.TCX_KEY_WORKSPACE_BYTES) == 4 * 8 * 32 * 32 * 8
    T.tcx_product_set(prod, T.TCX_KEY_SPLIT_K, 1)
    assert T.tcx_product_get(prod, T.TCX_KEY_WORKSPACE_BYTES) == 0
    T.tcx_destroy_product(prod)


def test_plan_precision(handle):
    """Sec. "Tensor Operation Descriptors": the plan carries a desired computational precision.
    TCX_PREC_F64 widens 32-bit tensors to 64-bit arithmetic: such plans take the generic kernel or
    one of the two widened tile shapes, never the streaming path; on 64-bit dtypes it changes nothing."""
    e = dict(m=300, n=200, k=64)
    A, B, D = W.tensor("mk", e), W.tensor("kn", e), W.tensor("mn", e)
    for dtype in (T.TCX_F32, T.TCX_C64, T.TCX_F64):
        infos = [T.tcx_create_tensor_info(handle, dtype, t.extents, t.strides) for t in (A, B, D)]
        args = (handle, 0, infos[0], [1, 3], 0, infos[1], [3, 2], 0, infos[2], [1, 2], 0, infos[2], [1, 2])
        assert _code(T.tcx_create_product, *args, 7) == T.TCX_ERR_UNSUPPORTED_PRECISION
        plain, wide = T.tcx_create_product(*args), T.tcx_create_product(*args, T.TCX_PREC_F64)
        assert T.tcx_product_get(plain, T.TCX_KEY_PRECISION) == 0 and T.tcx_product_get(wide, T.TCX_KEY_PRECISION) == 1
        assert T.tcx_product_get(wide, T.TCX_KEY_PATH) == T.TCX_PATH_GETT_MFMA
        if dtype == T.TCX_F64:
            assert T.tcx_product_get(wide, T.TCX_KEY_VARIANT) == T.tcx_product_get(plain, T.TCX_KEY_VARIANT)
        else:
            assert T.tcx_product_get(wide, T.TCX_KEY_VARIANT) in ((2, 3) if dtype == T.TCX_F32 else (1, 2))
            assert _code(T.tcx_product_set, wide, T.TCX_KEY_VARIANT, 0) == T.TCX_ERR_PLAN_REFUSED
            assert _code(T.tcx_product_set, wide, T.TCX_KEY_FORCE_PATH, T.TCX_PATH_BANDWIDTH) == T.TCX_ERR_PLAN_REFUSED
        for prod in (plain, wide):
            T.tcx_destroy_product(prod)
        for i in infos:
            T.tcx_destroy_tensor_info(i)


@pytest.mark.parametrize("dt16", [T.TCX_F16, T.TCX_BF16], ids=["f16", "bf16"])
def test_sixteen_bit_plans(handle, dt16):
    """TCX_F16, TCX_BF16 (Sec. "The Reference Implementation": real types of 16 bit): storage is always
    narrower than the arithmetic, so both precisions plan on the generic kernel or the two widened
    tile shapes and never on the streaming path; a low-intensity product falls to them as well;
    the four tensors must share the dtype."""
    e = dict(m=300, n=200, k=64)
    A, B, D = W.tensor("mk", e), W.tensor("kn", e), W.tensor("mn", e)
    infos = [T.tcx_create_tensor_info(handle, dt16, t.extents, t.strides) for t in (A, B, D)]
    args = (handle, 0, infos[0], [1, 3], 0, infos[1], [3, 2], 0, infos[2], [1, 2], 0, infos[2], [1, 2])
    for prec in (T.TCX_PREC_DEFAULT, T.TCX_PREC_F64):
        plan = T.tcx_create_product(*args, prec)
        assert T.tcx_product_get(plan, T.TCX_KEY_PRECISION) == prec
        assert T.tcx_product_get(plan, T.TCX_KEY_PATH) == T.TCX_PATH_GETT_MFMA
        assert T.tcx_product_get(plan, T.TCX_KEY_VARIANT) in (2, 3)
        assert _code(T.tcx_product_set, plan, T.TCX_KEY_VARIANT, 0) == T.TCX_ERR_PLAN_REFUSED
        assert _code(T.tcx_product_set, plan, T.TCX_KEY_FORCE_PATH, T.TCX_PATH_BANDWIDTH) == T.TCX_ERR_PLAN_REFUSED
        T.tcx_product_set(plan, T.TCX_KEY_SPLIT_K, 2)
        # partial sums are kept in the arithmetic's reals: 4 or 8 bytes each
        assert T.tcx_product_get(plan, T.TCX_KEY_WORKSPACE_BYTES) % (8 if prec else 4) == 0
        T.tcx_destroy_product(plan)
    f32 = T.tcx_create_tensor_info(handle, T.TCX_F32, D.extents, D.strides)
    assert _code(T.tcx_create_product, handle, 0, infos[0], [1, 3], 0, infos[1], [3, 2], 0, f32, [1, 2], 0, f32, [1, 2]) == T.TCX_ERR_DTYPE_MIX
    T.tcx_destroy_tensor_info(f32)
    # the two 16-bit formats do not mix either
    other = T.tcx_create_tensor_info(handle, T.TCX_BF16 if dt16 == T.TCX_F16 else T.TCX_F16, B.extents, B.strides)
    assert _code(T.tcx_create_product, handle, 0, infos[0], [1, 3], 0, other, [3, 2], 0, infos[2], [1, 2], 0, infos[2], [1, 2]) == T.TCX_ERR_DTYPE_MIX
    T.tcx_destroy_tensor_info(other)
    for i in infos:
        T.tcx_destroy_tensor_info(i)
    # an outer product of 16-bit vectors: not streamed, planned on the tiled or generic kernel
    e = dict(m=4096, n=4096)
    u, v, O = W.tensor("m", e), W.tensor("n", e), W.tensor("mn", e)
    infos = [T.tcx_create_tensor_info(handle, dt16, t.extents, t.strides) for t in (u, v, O)]
    plan = T.tcx_create_product(handle, 0, infos[0], [1], 0, infos[1], [2], 0, infos[2], [1, 2], 0, infos[2], [1, 2])
    assert T.tcx_product_get(plan, T.TCX_KEY_PATH) in (T.TCX_PATH_GETT_MFMA, T.TCX_PATH_GENERIC)
    T.tcx_destroy_product(plan)
    for i in infos:
        T.tcx_destroy_tensor_info(i)


def test_isolated_labels_are_planned_as_reductions_and_broadcasts(handle):
    """Sec. "Case 4": a label in A only is summed inside A by a launch of its own into workspace
    memory, and the plan then sees the dense reduced operand; Sec. "Case 5": a label in D only is a
    free mode that neither operand moves along."""
    ext = dict(m=30, n=20, k=16, x=5, y=3, z=4)
    ids = dict(m=1, n=2, k=3, x=4, y=5, z=6)
    t = lambda labels, **kw: W.tensor(labels, ext, **kw)
    A, B, D = t("xmky"), t("kn"), t("mzn")
    infos = [T.tcx_create_tensor_info(handle, T.TCX_F64, s.extents, s.strides) for s in (A, B, D)]
    labs = [[ids[l] for l in s.labels] for s in (A, B, D)]
    prod = T.tcx_create_product(handle, 0, infos[0], labs[0], 0, infos[1], labs[1], 0, infos[2], labs[2], 0, infos[2], labs[2])
    assert T.tcx_product_get(prod, T.TCX_KEY_SIZE_K) == 16 and T.tcx_product_get(prod, T.TCX_KEY_SIZE_M) == 30 * 4
    # A reduced over x and y is a dense 30 x 16 matrix: m keeps the smaller stride
    assert sorted(T.tcx_product_get(prod, T.TCX_KEY_MODES_M)) == [(4, 0, 0, 30), (30, 1, 0, 1)]
    assert T.tcx_product_get(prod, T.TCX_KEY_MODES_K) == [(16, 30, 1, 0)]
    assert T.tcx_product_get(prod, T.TCX_KEY_WORKSPACE_BYTES) >= 30 * 16 * 8
    launches = T.tcx_product_get(prod, T.TCX_KEY_LAUNCHES)
    T.tcx_product_set(prod, T.TCX_KEY_FORCE_PATH, T.TCX_PATH_GENERIC)
    assert T.tcx_product_get(prod, T.TCX_KEY_LAUNCHES) == 2 and launches >= 2
    T.tcx_destroy_product(prod)
    for i in infos:
        T.tcx_destroy_tensor_info(i)


def test_unary_and_binary_plans(handle):
    """Sec. "Unary and Binary Operations": C := alpha A + beta B is planned as the contraction
    alpha A * 1 + beta B (labels of A that C lacks are summed, labels of C that A lacks broadcast);
    B := alpha A needs the same label set on both sides.  Each plan answers only to its own execute call."""
    ext = dict(h=6, x=4, y=5)
    ids = dict(h=1, x=2, y=3)
    t = lambda labels, **kw: W.tensor(labels, ext, **kw)
    info = lambda spec: T.tcx_create_tensor_info(handle, T.TCX_F64, spec.extents, spec.strides)
    lab = lambda spec: [ids[l] for l in spec.labels]
    A, B = t("hx"), t("yh")
    ia, ib = info(A), info(B)
    plan = T.tcx_create_binary(handle, 0, ia, lab(A), 0, ib, lab(B), 0, ib, lab(B))
    assert T.tcx_product_get(plan, T.TCX_KEY_SIZE_K) == 1 and T.tcx_product_get(plan, T.TCX_KEY_SIZE_H) == 1
    assert T.tcx_product_get(plan, T.TCX_KEY_SIZE_M) == 30              # h (carried by A) and y (broadcast)
    assert T.tcx_product_get(plan, T.TCX_KEY_WORKSPACE_BYTES) >= 6 * 8   # A summed over x
    ex = T.tcx_create_executor(handle, 0)
    lib = T.raw()
    one = ctypes.c_double(1.0)
    args = (ctypes.byref(one), ctypes.c_void_p(16), ctypes.c_void_p(16), ctypes.byref(one), ctypes.c_void_p(16), ctypes.c_void_p(16))
    assert lib.tcx_execute_product(plan, ex, None, *args) == T.TCX_ERR_INVALID_HANDLE      # a binary plan is not a contraction
    assert lib.tcx_execute_unary(plan, ex, None, ctypes.byref(one), ctypes.c_void_p(16), ctypes.c_void_p(16)) == T.TCX_ERR_INVALID_HANDLE
    # C laid out differently from B
    ic = info(t("yh", memory_order="hy"))
    assert _code(T.tcx_create_binary, handle, 0, ia, lab(A), 0, ib, lab(B), 0, ic, lab(B)) == T.TCX_ERR_CD_MISMATCH
    assert _code(T.tcx_create_binary, handle, 0, ia, lab(A), 0, ib, lab(B), 1, ib, lab(B)) == T.TCX_ERR_UNSUPPORTED_OP
    # unary: same label set on both sides
    assert _code(T.tcx_create_unary, handle, 0, ia, lab(A), 0, ib, lab(B)) == T.TCX_ERR_ISOLATED_INDEX
    it = info(t("xh"))
    un = T.tcx_create_unary(handle, 0, ia, lab(A), 0, it, lab(t("xh")))
    assert lib.tcx_execute_binary(un, ex, None, ctypes.byref(one), ctypes.c_void_p(16), ctypes.byref(one), ctypes.c_void_p(16),
                                  ctypes.c_void_p(16)) == T.TCX_ERR_INVALID_HANDLE
    if not T.tcx_handle_has_device(handle):
        assert lib.tcx_execute_unary(un, ex, None, ctypes.byref(one), ctypes.c_void_p(16), ctypes.c_void_p(16)) == T.TCX_ERR_NO_DEVICE
    for prod in (plan, un):
        T.tcx_destroy_product(prod)
    T.tcx_destroy_executor(ex)
    for i in (ia, ib, ic, it):
        T.tcx_destroy_tensor_info(i)
