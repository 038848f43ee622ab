"""Seeded synthetic workloads: problem descriptions and input generators.

This module serves the tests, the bench and the smoke check.  It holds none of the
contraction's arithmetic: it only says which tensors exist (labels, extents, strides,
dtype, scalars) and fills buffers with counter-based pseudo-random values.  Neither the
oracle nor the GPU library imports it.

Values are a pure function of (seed, tensor tag, logical linear index), where the
logical linear index runs over the tensor's labels in the order they are written in
the problem statement, first label fastest -- NOT over memory order.  Re-laying a tensor
out in memory therefore moves values but does not change them.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 7827

# --------------------------------------------------------------------------------------
# counter-based generator
# --------------------------------------------------------------------------------------
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix64_block(key, z):
    """In place on a uint64 block (fresh pages are expensive on some hosts, so no temporaries
    beyond one block-sized scratch)."""
    t = np.empty_like(z)
    with np.errstate(over="ignore"):
        z += key
        np.right_shift(z, np.uint64(30), out=t); z ^= t; z *= _M1
        np.right_shift(z, np.uint64(27), out=t); z ^= t; z *= _M2
        np.right_shift(z, np.uint64(31), out=t); z ^= t
    return z


def _hashed(seed: int, tag: int, idx: np.ndarray, out_dtype, finish) -> np.ndarray:
    """finish(hash block) evaluated block by block over idx; returns an array shaped like idx."""
    with np.errstate(over="ignore"):
        key = np.uint64((int(seed) * 8 + int(tag) + 1) & 0xFFFFFFFFFFFFFFFF) * _GOLD
    idx = np.asarray(idx)
    out = np.empty(idx.shape, dtype=out_dtype)
    flat_in, flat_out = idx.reshape(-1), out.reshape(-1)
    if flat_in.shape[0] and not np.shares_memory(flat_out, out):
        raise ValueError("index array must be reshapeable without a copy")
    block = 1 << 20
    for lo in range(0, flat_in.shape[0], block):
        z = flat_in[lo:lo + block].astype(np.uint64)          # a copy
        flat_out[lo:lo + block] = finish(_mix64_block(key, z))
    return out


def mix64(seed: int, tag: int, idx: np.ndarray) -> np.ndarray:
    """64-bit hash of (seed, tag, idx); idx is an integer array (any shape)."""
    return _hashed(seed, tag, idx, np.uint64, lambda h: h)


# numpy has no bfloat16.  A bfloat16 is the upper half of a float32, so buffers of that type are
# uint16 arrays of bit patterns (dtype "bf16" <-> np.uint16 throughout this module), and the two
# functions below only move bits: no rounding happens here, a value that is not a bfloat16 is an error.
BF16 = np.dtype(np.uint16)


def bf16_bits(x) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xffff)), "not a bfloat16 value"
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_values(bits) -> np.ndarray:
    return (np.asarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32)


def uniform_pm1(seed: int, tag: int, idx: np.ndarray, dtype) -> np.ndarray:
    """Uniform on [-1, 1): 53 random bits for float64, 24 for float32, 11 for float16, 8 for
    bfloat16 (all exact)."""
    dtype = np.dtype(dtype)
    if dtype == BF16:            # 8 random bits: multiples of 2^-7, all of them bfloat16 values
        return bf16_bits(_hashed(seed, tag, idx, np.float32,
                                 lambda h: (h >> np.uint64(56)).astype(np.float32) * np.float32(2.0 ** -7) - np.float32(1.0)))
    if dtype in (np.complex128, np.complex64):
        real = np.float64 if dtype == np.complex128 else np.float32
        out = np.empty(np.shape(idx), dtype=dtype)
        two = np.asarray(idx).astype(np.uint64) * np.uint64(2)
        out.real = uniform_pm1(seed, tag, two, real)
        out.imag = uniform_pm1(seed, tag, two + np.uint64(1), real)
        return out
    if dtype == np.float64:
        return _hashed(seed, tag, idx, np.float64,
                       lambda h: (h >> np.uint64(11)).astype(np.float64) * 2.0 ** -52 - 1.0)
    if dtype == np.float32:
        return _hashed(seed, tag, idx, np.float32,
                       lambda h: (h >> np.uint64(40)).astype(np.float32) * np.float32(2.0 ** -23) - np.float32(1.0))
    if dtype == np.float16:      # 11 random bits: multiples of 2^-10, all of them 16-bit values
        return _hashed(seed, tag, idx, np.float16,
                       lambda h: ((h >> np.uint64(53)).astype(np.float32) * np.float32(2.0 ** -10) - np.float32(1.0)).astype(np.float16))
    raise ValueError(dtype)


def normal01(seed: int, tag: int, idx: np.ndarray, dtype) -> np.ndarray:
    """Standard normal by Box-Muller on two hashed uniforms (host only)."""
    dtype = np.dtype(dtype)
    if dtype == BF16:
        raise ValueError("normal entries are not bfloat16 values; use uniform, ints or ones")
    if dtype in (np.complex128, np.complex64):
        re = normal01(seed, tag, idx.astype(np.uint64) * np.uint64(2), np.float64)
        im = normal01(seed, tag, idx.astype(np.uint64) * np.uint64(2) + np.uint64(1), np.float64)
        return (re + 1j * im).astype(dtype)
    h1 = mix64(seed, tag, idx)
    h2 = mix64(seed, tag + 101, idx)
    u1 = ((h1 >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53      # (0, 1]
    u2 = (h2 >> np.uint64(11)).astype(np.float64) * 2.0 ** -53              # [0, 1)
    return (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(dtype)


def small_ints(seed: int, tag: int, idx: np.ndarray, dtype, lo: int = -4, hi: int = 4) -> np.ndarray:
    """Integer-valued entries in [lo, hi]: every partial sum of products is exact."""
    dtype = np.dtype(dtype)
    if dtype == BF16:
        return bf16_bits(small_ints(seed, tag, idx, np.float32, lo, hi))
    span = np.uint64(hi - lo + 1)
    if dtype in (np.complex128, np.complex64):
        re = small_ints(seed, tag, idx.astype(np.uint64) * np.uint64(2), np.float64, lo, hi)
        im = small_ints(seed, tag, idx.astype(np.uint64) * np.uint64(2) + np.uint64(1), np.float64, lo, hi)
        return (re + 1j * im).astype(dtype)
    h = mix64(seed, tag, idx) >> np.uint64(33)
    return ((h % span).astype(np.int64) + lo).astype(dtype)


def ones(seed, tag, idx, dtype):
    if np.dtype(dtype) == BF16:
        return bf16_bits(np.ones(idx.shape, dtype=np.float32))
    return np.ones(idx.shape, dtype=dtype)


DISTRIBUTIONS = {"uniform": uniform_pm1, "normal": normal01, "ints": small_ints, "ones": ones}

# --------------------------------------------------------------------------------------
# problem description
# --------------------------------------------------------------------------------------


@dataclass(frozen=True)
class TensorSpec:
    labels: Tuple[str, ...]
    extents: Tuple[int, ...]
    strides: Tuple[int, ...]          # elements
    base: int = 0                     # buffer index of the element with all indices zero
    size: int = 0                     # buffer length in elements

    @property
    def count(self) -> int:
        n = 1
        for e in self.extents:
            n *= e
        return n


def span_of(extents: Sequence[int], strides: Sequence[int]) -> Tuple[int, int]:
    """(base, size) of the smallest buffer that holds a strided tensor."""
    lo = sum(s * (e - 1) for e, s in zip(extents, strides) if s < 0)
    hi = sum(s * (e - 1) for e, s in zip(extents, strides) if s > 0)
    return -lo, hi - lo + 1


def tensor(labels: Sequence[str], extent_of: Dict[str, int], memory_order: Optional[Sequence[str]] = None,
           strides: Optional[Dict[str, int]] = None, size: Optional[int] = None) -> TensorSpec:
    """Describe a tensor.  Default layout: column-major over `labels` as written (glossary,
    "Column-major layout": s_k = prod_{l<k} e_l).  `memory_order` lists the labels from
    fastest to slowest instead; `strides` gives them outright."""
    labels = tuple(labels)
    ext = tuple(int(extent_of[l]) for l in labels)
    if strides is None:
        order = tuple(memory_order) if memory_order is not None else labels
        assert sorted(order) == sorted(labels)
        st, run = {}, 1
        for l in order:
            st[l] = run
            run *= extent_of[l]
        strides = st
    sv = tuple(int(strides[l]) for l in labels)
    base, need = span_of(ext, sv)
    return TensorSpec(labels, ext, sv, base, int(size) if size is not None else need)


@dataclass(frozen=True)
class Problem:
    name: str
    dtype: str                        # "f32" | "f64" | "c64" | "c128" | "f16" | "bf16"
    A: TensorSpec
    B: TensorSpec
    D: TensorSpec                     # C shares D's description
    alpha: complex = 1.0
    beta: complex = 0.0
    opA: int = 0                      # 0 identity, 1 conjugate
    opB: int = 0
    opC: int = 0
    seed: int = BASE_SEED
    dist: str = "uniform"
    note: str = ""

    @property
    def np_dtype(self):
        return {"f32": np.float32, "f64": np.float64, "c64": np.complex64, "c128": np.complex128, "f16": np.float16,
                "bf16": np.uint16}[self.dtype]

    def extent_of(self) -> Dict[str, int]:
        out: Dict[str, int] = {}
        for t in (self.A, self.B, self.D):
            out.update(dict(zip(t.labels, t.extents)))
        return out

    def groups(self):
        """Label groups by set membership: (H, M = F_A, N = F_B, K = P)."""
        a, b, d = set(self.A.labels), set(self.B.labels), set(self.D.labels)
        seen, order = set(), []
        for l in self.D.labels + self.A.labels + self.B.labels:
            if l not in seen:
                seen.add(l)
                order.append(l)
        H = [l for l in order if l in a and l in b and l in d]
        M = [l for l in order if l in a and l in d and l not in b]
        N = [l for l in order if l in b and l in d and l not in a]
        K = [l for l in order if l in a and l in b and l not in d]
        return H, M, N, K

    def sizes(self):
        e = self.extent_of()
        out = []
        for g in self.groups():
            n = 1
            for l in g:
                n *= e[l]
            out.append(n)
        return tuple(out)            # |H|, |M|, |N|, |K|

    def real_flops(self) -> int:
        h, m, n, k = self.sizes()
        return (8 if self.dtype in ("c128", "c64") else 2) * h * m * n * k

    def algorithmic_bytes(self) -> int:
        item = np.dtype(self.np_dtype).itemsize
        return item * (self.A.count + self.B.count + self.D.count * (2 if self.beta != 0 else 1))


def label_ids(p: Problem) -> Dict[str, int]:
    """Map label strings to the integer labels the C interfaces take."""
    ids: Dict[str, int] = {}
    for t in (p.A, p.B, p.D):
        for l in t.labels:
            ids.setdefault(l, 100 + len(ids))
    return ids


# --------------------------------------------------------------------------------------
# filling buffers
# --------------------------------------------------------------------------------------
TAG_A, TAG_B, TAG_C = 0, 1, 2


def logical_values(spec: TensorSpec, seed: int, tag: int, dtype, dist: str = "uniform") -> np.ndarray:
    """Values as an array of shape `extents`; entry [i0,i1,..] is keyed on i0 + e0*(i1 + e1*(...))."""
    idx = np.arange(spec.count, dtype=np.uint64)
    vals = DISTRIBUTIONS[dist](seed, tag, idx, dtype)
    return vals.reshape(spec.extents, order="F") if spec.extents else vals.reshape(())


def strided_view(buf: np.ndarray, spec: TensorSpec) -> np.ndarray:
    """View of a 1-D buffer as the tensor `spec` describes (read/write)."""
    item = buf.dtype.itemsize
    assert buf.ndim == 1 and buf.shape[0] >= spec.size
    return np.lib.stride_tricks.as_strided(buf[spec.base:], shape=spec.extents,
                                           strides=tuple(s * item for s in spec.strides), writeable=True)


def fill(spec: TensorSpec, seed: int, tag: int, dtype, dist: str = "uniform", background=None) -> np.ndarray:
    """New 1-D buffer of spec.size elements holding the tensor; gaps hold `background`
    (default: a recognisable sentinel so that tests can see gaps stay untouched)."""
    dtype = np.dtype(dtype)
    if background is None:
        background = -777.0
    if dtype == BF16:
        background = bf16_bits(np.float32(-768.0 if background == -777.0 else background)).reshape(())[()]
    buf = np.full(spec.size, background, dtype=dtype)
    strided_view(buf, spec)[...] = logical_values(spec, seed, tag, dtype, dist)
    return buf


def make_operands(p: Problem, dist: Optional[str] = None):
    """(bufA, bufB, bufC) for a problem; bufC is what D holds before the call."""
    d = dist or p.dist
    a = fill(p.A, p.seed, TAG_A, p.np_dtype, d)
    b = fill(p.B, p.seed, TAG_B, p.np_dtype, d)
    c = fill(p.D, p.seed, TAG_C, p.np_dtype, "uniform" if d == "normal" else d)
    return a, b, c


# --------------------------------------------------------------------------------------
# the five benchmark-shaped configurations (sizes can be scaled down for quick parity)
# --------------------------------------------------------------------------------------

def config1(n: int = 24) -> Problem:
    """fp64 rank-4: D[a,b,i,j] = 1.3 * sum_{c,d} A[a,c,i,d] B[c,b,d,j] + 0.7 C[a,b,i,j]."""
    e = dict.fromkeys("abcdij", n)
    return Problem("cfg1_f64_rank4_n%d" % n, "f64", tensor("acid", e), tensor("cbdj", e), tensor("abij", e),
                   alpha=1.3, beta=0.7, seed=BASE_SEED + 1)


def config2(v: int = 192, o: int = 64) -> Problem:
    """fp64 particle-particle ladder: D[a,b,i,j] = sum_{c,d} V[a,b,c,d] T[c,d,i,j] + D[a,b,i,j]."""
    e = dict(a=v, b=v, c=v, d=v, i=o, j=o)
    return Problem("cfg2_f64_ppladder_v%d_o%d" % (v, o), "f64", tensor("abcd", e), tensor("cdij", e),
                   tensor("abij", e), alpha=1.0, beta=1.0, seed=BASE_SEED + 2)


def config3(scale: float = 1.0, d_layout: str = "R1") -> Problem:
    """fp32 permuted, non-unit-stride: D[a,b,c] = sum_{d,e} A[a,d,e,b] B[e,c,d]; A is stored
    with e fastest, then b, a, d.  D is an interleaved buffer: "R1" gives c stride 2 (c is
    D's fastest mode, every other float is a gap); "R2" keeps a fastest and skips every
    other c-slab."""
    base = dict(a=37, b=53, c=61, d=29, e=41)
    e = {k: max(2, int(round(v * scale))) for k, v in base.items()}
    A = tensor("adeb", e, memory_order="ebad")
    B = tensor("ecd", e)
    nD = e["a"] * e["b"] * e["c"]
    if d_layout == "R1":
        D = tensor("abc", e, strides=dict(c=2, a=2 * e["c"], b=2 * e["c"] * e["a"]), size=2 * nD)
    else:
        D = tensor("abc", e, strides=dict(a=1, b=e["a"], c=2 * e["a"] * e["b"]), size=2 * nD)
    return Problem("cfg3_f32_permuted_%s_x%g" % (d_layout, scale), "f32", A, B, D, alpha=1.0, beta=0.0,
                   seed=BASE_SEED + 3)


def config4(h: int = 512, n: int = 96, h_slowest: bool = False, k: Optional[int] = None) -> Problem:
    """complex128 batched: D[h,i,j] = sum_k conj(A[h,k,i]) B[h,k,j] + 0.5 C[h,i,j]."""
    e = dict(h=h, i=n, j=n, k=n if k is None else k)
    if h_slowest:
        A, B, D = tensor("hki", e, memory_order="kih"), tensor("hkj", e, memory_order="kjh"), \
            tensor("hij", e, memory_order="ijh")
    else:
        A, B, D = tensor("hki", e), tensor("hkj", e), tensor("hij", e)
    return Problem("cfg4_c128_batched_h%d_n%d%s%s" % (h, n, "_hslow" if h_slowest else "", "" if k is None else "_k%d" % k),
                   "c128", A, B, D,
                   alpha=1.0, beta=0.5, opA=1, seed=BASE_SEED + 4)


def config5(extent: int = 4, nshared: int = 5, nfree: int = 5, perm_seed: Optional[int] = None) -> Problem:
    """fp64 tensor-network style: A and B of rank nshared+nfree, every extent `extent`,
    `nshared` contracted labels; each tensor's memory order is its own seeded
    Fisher-Yates permutation of its labels; values normal(0,1)."""
    seed = BASE_SEED + 5
    ms = ["m%d" % i for i in range(nfree)]
    ns = ["n%d" % i for i in range(nfree)]
    ks = ["k%d" % i for i in range(nshared)]
    e = dict.fromkeys(ms + ns + ks, extent)
    pseed = seed if perm_seed is None else perm_seed

    def shuffled(labels, tag):
        labels = list(labels)
        for i in range(len(labels) - 1, 0, -1):
            j = int(mix64(pseed, 50 + tag, np.array([i], dtype=np.uint64))[0] % np.uint64(i + 1))
            labels[i], labels[j] = labels[j], labels[i]
        return labels

    A = tensor(ms + ks, e, memory_order=shuffled(ms + ks, 0))
    B = tensor(ks + ns, e, memory_order=shuffled(ks + ns, 1))
    D = tensor(ms + ns, e, memory_order=shuffled(ms + ns, 2))
    return Problem("cfg5_f64_network_e%d_k%d_f%d_p%d" % (extent, nshared, nfree, pseed), "f64", A, B, D,
                   alpha=1.0, beta=0.0, seed=seed, dist="normal")


def hadamard(nmodes: int = 4, extent: int = 128, permuted: bool = False, dtype: str = "f64", beta: float = 0.0,
             pad_slowest: int = 0) -> Problem:
    """Pure Hadamard product D[h..] = A[h..] * B[h..] (+ beta C): every label in all three tensors.
    `permuted`: A, B and D each store the modes in a different order.  `pad_slowest`: elements added
    to the stride of each tensor's slowest mode (a layout whose strides are not all powers of two
    when the extent is one)."""
    labs = ["h%d" % i for i in range(nmodes)]
    e = dict.fromkeys(labs, extent)

    def laid_out(order):
        st, run = {}, 1
        for i, l in enumerate(order):
            st[l] = run + (pad_slowest if i == nmodes - 1 and nmodes > 1 else 0)
            run *= extent
        return tensor(labs, e, strides=st)
    if permuted:
        A, B, D = laid_out(labs[1:] + labs[:1]), laid_out(labs[::-1]), laid_out(labs)
    else:
        A, B, D = laid_out(labs), laid_out(labs), laid_out(labs)
    return Problem("hadamard_%s_%dx%d%s%s" % (dtype, nmodes, extent, "_perm" if permuted else "",
                                              "_pad%d" % pad_slowest if pad_slowest else ""), dtype, A, B, D,
                   alpha=1.0, beta=beta, seed=BASE_SEED + 13)


def low_intensity_shapes(full: bool = True) -> List[Problem]:
    """Supplementary shapes whose algorithmic flop/byte is far below the ridge, so HBM bounds them:
    a one-label contraction and an outer product of high-rank small-extent tensors (random
    mode orders, as configuration 5), a pure Hadamard product, and configuration 4 with 4
    contracted terms."""
    if full:
        return [config5(extent=4, nshared=1, nfree=7), config5(extent=4, nshared=0, nfree=7),
                hadamard(4, 128), hadamard(4, 128, permuted=True), config4(h=512, n=96, k=4)]
    return [config5(extent=4, nshared=1, nfree=3), config5(extent=3, nshared=0, nfree=4),
            hadamard(3, 20), hadamard(3, 17, permuted=True, beta=0.5), hadamard(2, 9, dtype="c128", permuted=True),
            config4(h=24, n=20, k=4), config4(h=5, n=33, k=2, h_slowest=True), config3(0.3)]


def configs_full() -> List[Problem]:
    return [config1(), config2(), config3(), config4(), config5()]


def configs_reduced() -> List[Problem]:
    """Same label structure and layouts, sizes the CPU oracle finishes in about a second."""
    return [config1(12), config2(v=20, o=7), config3(0.45), config3(0.45, "R2"), config4(h=6, n=20),
            config4(h=5, n=18, h_slowest=True), config5(extent=3, nshared=3, nfree=3),
            config5(extent=4, nshared=3, nfree=3)]


# --------------------------------------------------------------------------------------
# the same generator on a torch device (for tensors too large to build on the host)
# --------------------------------------------------------------------------------------
def _as_i64(u: int) -> int:
    u &= 0xFFFFFFFFFFFFFFFF
    return u - (1 << 64) if u >= (1 << 63) else u


def torch_uniform_pm1(seed: int, tag: int, start: int, count: int, dtype, device, out=None, dist="uniform"):
    """uniform_pm1 (or small_ints for dist="ints") of (seed, tag, arange(start, start+count)) as a
    torch tensor on `device`, bit-identical to the numpy version (wrapping 64-bit integer
    arithmetic, exact conversion)."""
    import torch
    assert dtype in (torch.float64, torch.float32)
    key = _as_i64(((int(seed) * 8 + int(tag) + 1) & 0xFFFFFFFFFFFFFFFF) * 0x9E3779B97F4A7C15)
    if out is None:
        out = torch.empty(count, dtype=dtype, device=device)
    chunk = 1 << 26
    for lo in range(0, count, chunk):
        n = min(chunk, count - lo)
        z = torch.arange(start + lo, start + lo + n, dtype=torch.int64, device=device) + key

        def lsr(x, s):
            return (x >> s) & ((1 << (64 - s)) - 1)
        z = (z ^ lsr(z, 30)) * _as_i64(0xBF58476D1CE4E5B9)
        z = (z ^ lsr(z, 27)) * _as_i64(0x94D049BB133111EB)
        z = z ^ lsr(z, 31)
        if dist == "ints":
            out[lo:lo + n] = (torch.remainder(lsr(z, 33), 9) - 4).to(dtype)
        elif dtype == torch.float64:
            out[lo:lo + n] = lsr(z, 11).to(torch.float64) * 2.0 ** -52 - 1.0
        else:
            out[lo:lo + n] = lsr(z, 40).to(torch.float32) * 2.0 ** -23 - 1.0
    return out


# --------------------------------------------------------------------------------------
# sampled sub-problems of config 2 (the full tensors never exist on the host)
# --------------------------------------------------------------------------------------
def config2_sample(p: Problem, m_idx: np.ndarray, n_idx: np.ndarray, dist: str = "uniform"):
    """Rows m_idx of V (as an |m_idx| x |K| matrix), columns n_idx of T and the matching
    entries of the initial D of a config-2 style problem, generated straight from the
    counter-based generator.  Returns (sub_problem, bufA, bufB, bufC); the sub-problem is
    D_s[x,y] = alpha * sum_k A_s[x,k] B_s[k,y] + beta * C_s[x,y], column-major, k running
    over the fused (c,d) index in V's order."""
    _, M, N, K = p.sizes()
    m_idx = np.asarray(m_idx, dtype=np.uint64)
    n_idx = np.asarray(n_idx, dtype=np.uint64)
    k = np.arange(K, dtype=np.uint64)
    # logical linear indices: V[m, k] -> m + M*k ; T[k, n] -> k + K*n ; D[m, n] -> m + M*n.
    # Index arrays are built slow-index-first so that their C-order flattening is the
    # column-major buffer of the sub-tensor.
    gen = DISTRIBUTIONS[dist]
    a = gen(p.seed, TAG_A, np.uint64(M) * k[:, None] + m_idx[None, :], np.float64).reshape(-1)
    b = gen(p.seed, TAG_B, np.uint64(K) * n_idx[:, None] + k[None, :], np.float64).reshape(-1)
    c = gen(p.seed, TAG_C, np.uint64(M) * n_idx[:, None] + m_idx[None, :], np.float64).reshape(-1)
    e = dict(x=len(m_idx), y=len(n_idx), k=K)
    sub = Problem(p.name + "_sample", "f64", tensor("xk", e), tensor("ky", e), tensor("xy", e),
                  alpha=p.alpha, beta=p.beta, seed=p.seed)
    return sub, a, b, c
