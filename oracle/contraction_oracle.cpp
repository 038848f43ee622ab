// CPU ORACLE for the binary tensor contraction  D := alpha * op(A) * op(B) + beta * op(C).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
// library is checked against.  It shares no code with the library, is never linked
// into it, and only tests, the smoke check and the bench's cpu_baseline leg call it.
//
// What it computes (paper, Sec. "Mathematical Definitions"):
//   * Eq. (binary_contraction):  D := alpha A B + beta C.
//   * Case 1 / Eq. (case1): labels shared by A and B only (P) are summed; labels
//     shared by A and D (F_A) or by B and D (F_B) are free.
//   * Case 2 / Eq. (case2): labels present in A, B and D (H) are element-wise.
//   * Case 3 + Note 6: a label repeated inside one tensor addresses a diagonal; the
//     strides of all its occurrences are added.
//   * Case 4 / its equation: a label in A only (I_A) or in B only (I_B) is summed inside
//     that tensor before the product:  sum_P (sum_{I_A} A) (sum_{I_B} B).
//   * Case 5 / its equation: a label in D (and C) only (I_C) broadcasts the product: the
//     same alpha * sum is written for every value of the label, plus beta * C at that place.
//     (The standard does not require Cases 4 and 5 (Note 7); their definitions are still the
//     paper's, so the oracle states them.)
// How it computes it (paper, Sec. "Algorithm Structure"): every index tuple over the
// distinct labels of D, first label fastest; for each, every tuple over the contracted
// labels, again first label fastest; per term one displacement sum(index*stride) per
// tensor.  Strides are in ELEMENTS, measured from the element whose indices
// are all zero (glossary, "Strided layout"); absent labels get stride 0.
//
// Readings where the paper is silent:
//   * op() is identity or complex conjugation applied to the element as it is read;
//     on real types it is the identity.
//   * beta == 0 means C is never read (so C may hold NaN or be a null pointer);
//     alpha == 0 means A and B are never read.  (The paper-literal mode below is the
//     exception: it follows the figure, which always reads C.)
//   * C has exactly D's extents, labels and strides (Note 5) and is addressed with
//     D's offset, as in the figure.
//
// Three evaluation modes of the same loop nest:
//   MODE_TRUTH   accumulator is long double (x87 80-bit), one rounding to the storage
//                type at the end; also returns S = sum |op(a)||op(b)| per D element,
//                the normaliser of the error measure.
//   MODE_TIMED   accumulator in the storage type's own precision: what a plain CPU
//                code does; this is the instantiation the bench times.
//   MODE_LITERAL the figure's order of operations: D <- beta*C, then
//                D <- D + alpha*a*b for every term, read-modify-write on D in storage
//                precision.
//
// Build:  g++ -O2 -fopenmp -shared -fPIC contraction_oracle.cpp -o liboracle.so

#include <complex>
#include <cstdint>
#include <cstdlib>
#include <cmath>
#include <vector>
#include <algorithm>

namespace {

enum { DT_F32 = 0, DT_F64 = 1, DT_C64 = 2, DT_C128 = 3, DT_F16 = 4, DT_BF16 = 5 };
enum { MODE_TRUTH = 0, MODE_TIMED = 1, MODE_LITERAL = 2 };
enum { OP_IDENTITY = 0, OP_CONJ = 1 };

// validation outcomes (classes, not the library's numeric codes)
enum {
    V_OK = 0,
    V_EXTENT_MISMATCH = 1,   // same label, different extent (Preliminaries: Id(i)=Id(j) only if d_i=d_j)
    V_CD_MISMATCH = 2,       // C is not laid out exactly as D (Note 5)
    V_D_ALIASING = 3,        // two index tuples of D address the same element
    V_ISOLATED = 4,          // (no longer produced: Cases 4 and 5 are defined and evaluated)
    V_BAD_ARG = 5            // non-positive extent, bad rank
};

struct Tensor {
    int n;
    const int64_t* extent;
    const int64_t* stride;
    const int64_t* label;
};

// One entry per distinct label of the whole operation (paper: "pre-processing").
struct Loop {
    int64_t label;
    int64_t extent;
    int64_t sA, sB, sD;   // summed strides (Note 6); 0 where the label is absent
};

bool has_label(const Tensor& t, int64_t lab) {
    for (int i = 0; i < t.n; ++i) if (t.label[i] == lab) return true;
    return false;
}

int64_t summed_stride(const Tensor& t, int64_t lab) {
    int64_t s = 0;
    for (int i = 0; i < t.n; ++i) if (t.label[i] == lab) s += t.stride[i];
    return s;
}

// Distinct labels of `t`, in order of first appearance.
std::vector<int64_t> distinct_labels(const Tensor& t) {
    std::vector<int64_t> out;
    for (int i = 0; i < t.n; ++i)
        if (std::find(out.begin(), out.end(), t.label[i]) == out.end()) out.push_back(t.label[i]);
    return out;
}

int validate(const Tensor& A, const Tensor& B, const Tensor& C, const Tensor& D) {
    const Tensor* all[4] = {&A, &B, &C, &D};
    for (const Tensor* t : all) {
        if (t->n < 0) return V_BAD_ARG;
        for (int i = 0; i < t->n; ++i) if (t->extent[i] <= 0) return V_BAD_ARG;
    }
    // equal labels carry equal extents, within and across tensors
    for (const Tensor* t : all)
        for (int i = 0; i < t->n; ++i)
            for (const Tensor* u : all)
                for (int j = 0; j < u->n; ++j)
                    if (t->label[i] == u->label[j] && t->extent[i] != u->extent[j])
                        return V_EXTENT_MISMATCH;
    // C must be D (Note 5: identical memory layout).  Compared label by label on the
    // distinct labels (extent and summed stride), so writing C's modes in another order
    // with the strides moved along is the same layout and is accepted.
    {
        std::vector<int64_t> lc = distinct_labels(C), ld = distinct_labels(D);
        if (lc.size() != ld.size()) return V_CD_MISMATCH;
        for (int64_t lab : ld) {
            if (!has_label(C, lab)) return V_CD_MISMATCH;
            int64_t ec = 0, ed = 0;
            for (int i = 0; i < C.n; ++i) if (C.label[i] == lab) ec = C.extent[i];
            for (int i = 0; i < D.n; ++i) if (D.label[i] == lab) ed = D.extent[i];
            if (ec != ed) return V_CD_MISMATCH;
            if (ed > 1 && summed_stride(C, lab) != summed_stride(D, lab)) return V_CD_MISMATCH;
        }
    }
    // Aliasing inside D.  Work on distinct labels with summed strides, drop extent 1,
    // sort by |stride| and require each stride to clear the span of the smaller ones.
    // Sufficient for "no two tuples collide"; conservative for exotic layouts.
    std::vector<std::pair<int64_t, int64_t>> se;   // (|stride|, extent)
    for (int64_t lab : distinct_labels(D)) {
        int64_t e = 0;
        for (int i = 0; i < D.n; ++i) if (D.label[i] == lab) e = D.extent[i];
        if (e == 1) continue;
        int64_t s = summed_stride(D, lab);
        se.push_back({s < 0 ? -s : s, e});
    }
    std::sort(se.begin(), se.end());
    int64_t span = 0;               // largest |offset| reachable with the modes so far
    for (auto& p : se) {
        if (p.first <= span) return V_D_ALIASING;   // also catches stride 0
        span += p.first * (p.second - 1);
    }
    return V_OK;
}

// ---- 16-bit storage (Sec. "The Reference Implementation": real types of 64, 32 and 16 bit) ----
// IEEE 754 binary16: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits; exponent field 0
// holds zero and the subnormals (multiples of 2^-24), 31 holds infinities and NaNs.  The host
// compiler has no such type, so the two conversions are written out: to a wider type exactly, from
// a wider type with ONE rounding to nearest, ties to even.
struct half16 {
    uint16_t bits;
    half16() : bits(0) {}
    // One rounding from the exact value of x.  float and double arguments promote exactly.
    half16(long double x) {
        const uint16_t sign = std::signbit(x) ? 0x8000u : 0u;
        long double a = fabsl(x);
        if (std::isnan(x)) { bits = sign | 0x7e00u; return; }
        if (a == 0.0L) { bits = sign; return; }
        if (std::isinf(x)) { bits = sign | 0x7c00u; return; }
        // the grid the result lies on: 2^(e-10) for a leading exponent e, never finer than 2^-24
        int e = ilogbl(a);
        if (e < -14) e = -14;
        const long double quantum = ldexpl(1.0L, e - 10);
        const long double n = nearbyintl(a / quantum);          // exact division; rounds to nearest, ties to even
        a = n * quantum;                                         // may have moved up to the next power of two
        if (a >= 65536.0L) { bits = sign | 0x7c00u; return; }    // beyond the largest finite value 65504 after rounding
        if (a == 0.0L) { bits = sign; return; }
        const int e2 = ilogbl(a);
        if (e2 < -14) bits = sign | (uint16_t)(a / ldexpl(1.0L, -24));
        else bits = sign | (uint16_t)((e2 + 15) << 10) | (uint16_t)((long long)(a / ldexpl(1.0L, e2 - 10)) - 1024);
    }
    half16(double x) : half16((long double)x) {}
    half16(float x) : half16((long double)x) {}
    half16(int x) : half16((long double)x) {}
    // exact
    operator long double() const {
        const int ef = (bits >> 10) & 31, frac = bits & 1023;
        long double a;
        if (ef == 31) a = frac ? (long double)NAN : (long double)INFINITY;
        else if (ef == 0) a = ldexpl((long double)frac, -24);
        else a = ldexpl((long double)(1024 + frac), ef - 25);
        return (bits & 0x8000u) ? -a : a;
    }
};
// Arithmetic "in the storage type" (the figure-literal mode): the exact result of one operation
// on two 16-bit values fits a long double, and is rounded once.
inline half16 operator*(half16 a, half16 b) { return half16((long double)a * (long double)b); }
inline half16 operator+(half16 a, half16 b) { return half16((long double)a + (long double)b); }
inline bool operator==(half16 a, half16 b) { return (long double)a == (long double)b; }

// bfloat16: the upper half of an IEEE binary32 -- 1 sign bit, 8 exponent bits (bias 127), 7 fraction
// bits; exponent field 0 holds zero and the subnormals (multiples of 2^-133), 255 infinities and
// NaNs.  Same two conversions: widening exact, narrowing ONE rounding to nearest, ties to even.
struct bfloat16 {
    uint16_t bits;
    bfloat16() : bits(0) {}
    bfloat16(long double x) {
        const uint16_t sign = std::signbit(x) ? 0x8000u : 0u;
        long double a = fabsl(x);
        if (std::isnan(x)) { bits = sign | 0x7fc0u; return; }
        if (a == 0.0L) { bits = sign; return; }
        if (std::isinf(x)) { bits = sign | 0x7f80u; return; }
        int e = ilogbl(a);
        if (e < -126) e = -126;
        const long double quantum = ldexpl(1.0L, e - 7);
        a = nearbyintl(a / quantum) * quantum;
        if (a >= ldexpl(1.0L, 128)) { bits = sign | 0x7f80u; return; }
        if (a == 0.0L) { bits = sign; return; }
        const int e2 = ilogbl(a);
        if (e2 < -126) bits = sign | (uint16_t)(a / ldexpl(1.0L, -133));
        else bits = sign | (uint16_t)((e2 + 127) << 7) | (uint16_t)((long long)(a / ldexpl(1.0L, e2 - 7)) - 128);
    }
    bfloat16(double x) : bfloat16((long double)x) {}
    bfloat16(float x) : bfloat16((long double)x) {}
    bfloat16(int x) : bfloat16((long double)x) {}
    operator long double() const {
        const int ef = (bits >> 7) & 255, frac = bits & 127;
        long double a;
        if (ef == 255) a = frac ? (long double)NAN : (long double)INFINITY;
        else if (ef == 0) a = ldexpl((long double)frac, -133);
        else a = ldexpl((long double)(128 + frac), ef - 134);
        return (bits & 0x8000u) ? -a : a;
    }
};
inline bfloat16 operator*(bfloat16 a, bfloat16 b) { return bfloat16((long double)a * (long double)b); }
inline bfloat16 operator+(bfloat16 a, bfloat16 b) { return bfloat16((long double)a + (long double)b); }
inline bool operator==(bfloat16 a, bfloat16 b) { return (long double)a == (long double)b; }

// ---- element access helpers -------------------------------------------------------
template <class T> struct Real { using type = T; };
template <class R> struct Real<std::complex<R>> { using type = R; };

template <class T> inline T apply_op(T x, int) { return x; }
template <class R> inline std::complex<R> apply_op(std::complex<R> x, int op) {
    return op == OP_CONJ ? std::conj(x) : x;
}

template <class Acc, class T> struct Widen { static Acc of(T x) { return (Acc)x; } };
template <class RA, class R> struct Widen<std::complex<RA>, std::complex<R>> {
    static std::complex<RA> of(std::complex<R> x) { return {(RA)x.real(), (RA)x.imag()}; }
};

template <class T, class Acc> struct Narrow { static T of(Acc x) { return (T)x; } };
template <class R, class RA> struct Narrow<std::complex<R>, std::complex<RA>> {
    static std::complex<R> of(std::complex<RA> x) { return {(R)x.real(), (R)x.imag()}; }
};

inline long double modulus(long double x) { return fabsl(x); }
inline long double modulus(std::complex<long double> x) { return hypotl(x.real(), x.imag()); }
inline double modulus(double x) { return std::fabs(x); }
inline float modulus(float x) { return std::fabs(x); }
inline double modulus(std::complex<double> x) { return std::hypot(x.real(), x.imag()); }
inline float modulus(std::complex<float> x) { return std::hypot(x.real(), x.imag()); }

// Complex multiply written out (no library special-casing of inf/nan).
template <class R> inline R mul(R a, R b) { return a * b; }
template <class R> inline std::complex<R> mul(std::complex<R> a, std::complex<R> b) {
    return {a.real() * b.real() - a.imag() * b.imag(), a.real() * b.imag() + a.imag() * b.real()};
}

template <class X> inline bool is_zero(X x) { return x == X(0); }

// Next index tuple in the order "first index fastest" (Sec. "Algorithm Structure": the free and
// the contracted index spaces are each walked in reverse lexicographical order).  A position
// that has reached its extent goes back to zero and hands a carry to the next one; the tuple
// after the last one is all zeros again.
inline void advance(std::vector<int64_t>& idx, const std::vector<int64_t>& shape) {
    size_t k = 0;
    while (k < shape.size() && ++idx[k] == shape[k]) idx[k++] = 0;
}
// Position of an index tuple relative to the all-zero element (glossary, "Strided layout":
// base + sum_k i_k * s_k), in elements.
inline int64_t displacement(const std::vector<int64_t>& idx, const std::vector<int64_t>& strides) {
    int64_t d = 0;
    for (size_t k = 0; k < idx.size(); ++k) d += strides[k] * idx[k];
    return d;
}

// The sum over one tensor's isolated labels (Case 4: a reduction inside the tensor) of the
// elements at base + displacement, each passed through op.  With no isolated label it is the one
// element at base.  *mod receives the sum of the moduli (for the normaliser).
template <class Acc, class T>
Acc reduced(const T* X, int64_t base, const std::vector<int64_t>& shape, const std::vector<int64_t>& strides, int op,
            long double* mod) {
    if (shape.empty()) {                       // nothing to sum over: the element itself
        const Acc x = Widen<Acc, T>::of(apply_op(X[base], op));
        *mod = (long double)modulus(x);
        return x;
    }
    int64_t count = 1;
    for (int64_t e : shape) count *= e;
    std::vector<int64_t> I(shape.size(), 0);
    Acc sum = Acc(0);
    *mod = 0.0L;
    for (int64_t n = 0; n < count; ++n, advance(I, shape)) {
        const Acc x = Widen<Acc, T>::of(apply_op(X[base + displacement(I, strides)], op));
        sum = sum + x;
        *mod += (long double)modulus(x);
    }
    return sum;
}

template <class T, class Acc>
void contract(int mode, const std::vector<Loop>& free_loops, const std::vector<Loop>& sum_loops,
              const std::vector<Loop>& only_A, const std::vector<Loop>& only_B,
              int opA, int opB, int opC, Acc alpha, Acc beta,
              const T* A, const T* B, const T* C, T* D, double* S) {
    std::vector<int64_t> dshape, dsA, dsB, dsD, pshape, psA, psB, iashape, iasA, ibshape, ibsB;
    int64_t size_D = 1, size_P = 1;
    for (const Loop& l : free_loops) {
        dshape.push_back(l.extent); dsA.push_back(l.sA); dsB.push_back(l.sB); dsD.push_back(l.sD);
        size_D *= l.extent;
    }
    for (const Loop& l : sum_loops) {
        pshape.push_back(l.extent); psA.push_back(l.sA); psB.push_back(l.sB);
        size_P *= l.extent;
    }
    for (const Loop& l : only_A) { iashape.push_back(l.extent); iasA.push_back(l.sA); }
    for (const Loop& l : only_B) { ibshape.push_back(l.extent); ibsB.push_back(l.sB); }
    const bool read_ab = !is_zero(alpha);
    const bool read_c = !is_zero(beta);

    // The paper runs three nested odometers over H, F_A, F_B and notes that its own
    // implementation folds them into one loop over the labels of D; so does this.
    // Each iteration rebuilds its multi-index from the linear counter, so the result
    // does not depend on how OpenMP cuts the range.
#pragma omp parallel for schedule(static)
    for (int64_t lin = 0; lin < size_D; ++lin) {
        std::vector<int64_t> I(dshape.size());
        int64_t rem = lin;
        for (size_t k = 0; k < dshape.size(); ++k) { I[k] = rem % dshape[k]; rem /= dshape[k]; }
        const int64_t off_D = displacement(I, dsD);
        const int64_t baseA = displacement(I, dsA);
        const int64_t baseB = displacement(I, dsB);
        std::vector<int64_t> K(pshape.size(), 0);

        if (mode == MODE_LITERAL) {
            // The order of operations of Fig. "implementation": D starts as beta*C and every
            // term alpha*a*b is added to it as it comes, all in the storage type.  The running
            // value is kept in a variable of the storage type and stored once, which rounds
            // exactly like a read-modify-write of D per term.  C is read even when beta is 0.
            const T al = Narrow<T, Acc>::of(alpha), be = Narrow<T, Acc>::of(beta);
            T running = mul(be, apply_op(C[off_D], opC));
            long double unused;
            for (int64_t k = 0; k < size_P; ++k, advance(K, pshape)) {
                const T a = reduced<T, T>(A, baseA + displacement(K, psA), iashape, iasA, opA, &unused);
                const T b = reduced<T, T>(B, baseB + displacement(K, psB), ibshape, ibsB, opB, &unused);
                running = running + mul(al, mul(a, b));
            }
            D[off_D] = running;
            continue;
        }

        Acc acc = Acc(0);
        long double s = 0.0L;
        if (read_ab) {
            for (int64_t k = 0; k < size_P; ++k) {
                const int64_t off_A = baseA + displacement(K, psA);
                const int64_t off_B = baseB + displacement(K, psB);
                long double ma, mb;
                const Acc a = reduced<Acc, T>(A, off_A, iashape, iasA, opA, &ma);      // Case 4: sum over I_A
                const Acc b = reduced<Acc, T>(B, off_B, ibshape, ibsB, opB, &mb);      // Case 4: sum over I_B
                acc = acc + mul(a, b);
                if (S) s += ma * mb;
                advance(K, pshape);
            }
        }
        Acc d = mul(alpha, acc);
        if (read_c) d = d + mul(beta, Widen<Acc, T>::of(apply_op(C[off_D], opC)));
        D[off_D] = Narrow<T, Acc>::of(d);
        if (S) S[off_D] = (double)s;
    }
}

}  // namespace

extern "C" {

// Validation by the rules of the paper, independent of the library's.  Returns a V_* class.
int oracle_validate(int nA, const int64_t* extA, const int64_t* strA, const int64_t* labA,
                    int nB, const int64_t* extB, const int64_t* strB, const int64_t* labB,
                    int nC, const int64_t* extC, const int64_t* strC, const int64_t* labC,
                    int nD, const int64_t* extD, const int64_t* strD, const int64_t* labD) {
    Tensor A{nA, extA, strA, labA}, B{nB, extB, strB, labB}, C{nC, extC, strC, labC}, D{nD, extD, strD, labD};
    return validate(A, B, C, D);
}

// The contraction.  alpha/beta: {re, im} as long double is awkward over ctypes, so they
// come as double pairs (every test scalar is a double or float value anyway).
// A, B, C, D point at the element with all indices zero.  S (may be null) has D's
// layout but element type double.  Returns a V_* class; nothing is written unless V_OK.
int oracle_contract(int dtype, int mode,
                    int nA, const int64_t* extA, const int64_t* strA, const int64_t* labA, int opA,
                    int nB, const int64_t* extB, const int64_t* strB, const int64_t* labB, int opB,
                    int nC, const int64_t* extC, const int64_t* strC, const int64_t* labC, int opC,
                    int nD, const int64_t* extD, const int64_t* strD, const int64_t* labD,
                    const double* alpha, const double* beta,
                    const void* A, const void* B, const void* C, void* D, double* S) {
    Tensor tA{nA, extA, strA, labA}, tB{nB, extB, strB, labB}, tC{nC, extC, strC, labC}, tD{nD, extD, strD, labD};
    const int v = validate(tA, tB, tC, tD);
    if (v != V_OK) return v;

    // classification by set membership (Secs. Case 1, Case 2): D's labels drive the
    // outer odometer (H, F_A, F_B together, in D's order); A∩B minus D is P.
    std::vector<Loop> free_loops, sum_loops;
    for (int64_t lab : distinct_labels(tD)) {
        Loop l{};
        l.label = lab;
        for (int i = 0; i < nD; ++i) if (labD[i] == lab) l.extent = extD[i];
        l.sA = summed_stride(tA, lab); l.sB = summed_stride(tB, lab); l.sD = summed_stride(tD, lab);
        free_loops.push_back(l);
    }
    std::vector<Loop> only_A, only_B;
    for (int64_t lab : distinct_labels(tA)) {
        if (has_label(tD, lab)) continue;
        Loop l{};
        l.label = lab;
        for (int i = 0; i < nA; ++i) if (labA[i] == lab) l.extent = extA[i];
        l.sA = summed_stride(tA, lab); l.sB = summed_stride(tB, lab); l.sD = 0;
        if (has_label(tB, lab)) sum_loops.push_back(l);       // P
        else only_A.push_back(l);                             // I_A
    }
    for (int64_t lab : distinct_labels(tB)) {
        if (has_label(tD, lab) || has_label(tA, lab)) continue;
        Loop l{};
        l.label = lab;
        for (int i = 0; i < nB; ++i) if (labB[i] == lab) l.extent = extB[i];
        l.sA = 0; l.sB = summed_stride(tB, lab); l.sD = 0;
        only_B.push_back(l);                                  // I_B
    }

    using cld = std::complex<long double>;
    using cd = std::complex<double>;
    using cf = std::complex<float>;
    if (dtype == DT_F64) {
        if (mode == MODE_TRUTH)
            contract<double, long double>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, alpha[0], beta[0],
                                          (const double*)A, (const double*)B, (const double*)C, (double*)D, S);
        else
            contract<double, double>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, alpha[0], beta[0],
                                     (const double*)A, (const double*)B, (const double*)C, (double*)D, S);
    } else if (dtype == DT_F32) {
        if (mode == MODE_TRUTH)
            contract<float, long double>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, alpha[0], beta[0],
                                         (const float*)A, (const float*)B, (const float*)C, (float*)D, S);
        else
            contract<float, float>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, (float)alpha[0], (float)beta[0],
                                   (const float*)A, (const float*)B, (const float*)C, (float*)D, S);
    } else if (dtype == DT_C128) {
        if (mode == MODE_TRUTH)
            contract<cd, cld>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, cld(alpha[0], alpha[1]), cld(beta[0], beta[1]),
                              (const cd*)A, (const cd*)B, (const cd*)C, (cd*)D, S);
        else
            contract<cd, cd>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, cd(alpha[0], alpha[1]), cd(beta[0], beta[1]),
                             (const cd*)A, (const cd*)B, (const cd*)C, (cd*)D, S);
    } else if (dtype == DT_C64) {
        if (mode == MODE_TRUTH)
            contract<cf, cld>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, cld(alpha[0], alpha[1]), cld(beta[0], beta[1]),
                              (const cf*)A, (const cf*)B, (const cf*)C, (cf*)D, S);
        else
            contract<cf, cf>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, cf((float)alpha[0], (float)alpha[1]),
                             cf((float)beta[0], (float)beta[1]), (const cf*)A, (const cf*)B, (const cf*)C, (cf*)D, S);
    } else if (dtype == DT_F16) {
        // truth: long-double sums, one rounding to 16 bits; timed: products and sums in float (what a
        // plain CPU code does with 16-bit data), one rounding; literal: every operation rounded to 16 bits
        if (mode == MODE_TRUTH)
            contract<half16, long double>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, alpha[0], beta[0],
                                          (const half16*)A, (const half16*)B, (const half16*)C, (half16*)D, S);
        else
            contract<half16, float>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, (float)alpha[0], (float)beta[0],
                                    (const half16*)A, (const half16*)B, (const half16*)C, (half16*)D, S);
    } else if (dtype == DT_BF16) {
        if (mode == MODE_TRUTH)
            contract<bfloat16, long double>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, alpha[0], beta[0],
                                            (const bfloat16*)A, (const bfloat16*)B, (const bfloat16*)C, (bfloat16*)D, S);
        else
            contract<bfloat16, float>(mode, free_loops, sum_loops, only_A, only_B, opA, opB, opC, (float)alpha[0], (float)beta[0],
                                      (const bfloat16*)A, (const bfloat16*)B, (const bfloat16*)C, (bfloat16*)D, S);
    } else {
        return V_BAD_ARG;
    }
    return V_OK;
}

// The two 16-bit conversions on their own, for the tests that pin them.
uint16_t oracle_half_from_double(double x) { return half16(x).bits; }
double oracle_half_to_double(uint16_t bits) { half16 h; h.bits = bits; return (double)(long double)h; }
uint16_t oracle_bfloat16_from_double(double x) { return bfloat16(x).bits; }
double oracle_bfloat16_to_double(uint16_t bits) { bfloat16 h; h.bits = bits; return (double)(long double)h; }

int oracle_max_threads(void);
}

#ifdef _OPENMP
#include <omp.h>
extern "C" int oracle_max_threads(void) { return omp_get_max_threads(); }
#else
extern "C" int oracle_max_threads(void) { return 1; }
#endif
