// Generic strided contraction kernel: one thread per element of D, a loop over the whole
// contracted index space, 64-bit element offsets.  It mirrors the structure of the paper's
// loop nest (Sec. "Algorithm Structure", Fig. "implementation": the H, F_A and F_B loops
// folded into one index over D, the P loop innermost) with the outer index spread over
// the grid.  It handles every dtype, op, stride sign and rank the analyser accepts and is
// the fallback for shapes the tiled kernels do not take.
#include <hip/hip_runtime.h>

#include "bf16.hpp"
#include "tcx_internal.hpp"

namespace tcx {
namespace {

// Arithmetic policies: `stor` is what memory holds, `acc_t` what products and sums are formed in
// (the storage type itself, its 64-bit widening when the plan asks for TCX_PREC_F64, 32-bit or
// 64-bit reals for 16-bit storage; the conversion back on the store rounds to nearest even).
template <class R> struct cplx_of {
    R re, im;
};

template <class S, class R> struct RealNum {
    using stor = S;
    using acc_t = R;
    static __device__ __forceinline__ R load(const S* p, int64_t off, int) { return (R)p[off]; }
    static __device__ __forceinline__ R zero() { return (R)0; }
    static __device__ __forceinline__ R fma(R a, R b, R c) {
        if constexpr (sizeof(R) == 4) return __builtin_fmaf(a, b, c);
        else return __builtin_fma(a, b, c);
    }
    static __device__ __forceinline__ R scale(const Scalars& s, bool alpha, R x) { return (R)(alpha ? s.alpha_re : s.beta_re) * x; }
    static __device__ __forceinline__ R add(R a, R b) { return a + b; }
    static __device__ __forceinline__ S narrow(R x) { return (S)x; }
};

template <class S, class R> struct ComplexNum {
    using stor = cplx_of<S>;
    using acc_t = cplx_of<R>;
    static __device__ __forceinline__ acc_t load(const stor* p, int64_t off, int op) {
        const stor v = p[off];
        return {(R)v.re, op == TCX_OP_CONJ ? -(R)v.im : (R)v.im};
    }
    static __device__ __forceinline__ acc_t zero() { return {(R)0, (R)0}; }
    static __device__ __forceinline__ R f(R a, R b, R c) {
        if constexpr (sizeof(R) == 4) return __builtin_fmaf(a, b, c);
        else return __builtin_fma(a, b, c);
    }
    static __device__ __forceinline__ acc_t fma(acc_t a, acc_t b, acc_t c) {
        c.re = f(a.re, b.re, c.re);
        c.re = f(-a.im, b.im, c.re);
        c.im = f(a.re, b.im, c.im);
        c.im = f(a.im, b.re, c.im);
        return c;
    }
    static __device__ __forceinline__ acc_t scale(const Scalars& s, bool alpha, acc_t x) {
        const R sr = (R)(alpha ? s.alpha_re : s.beta_re), si = (R)(alpha ? s.alpha_im : s.beta_im);
        return {sr * x.re - si * x.im, sr * x.im + si * x.re};
    }
    static __device__ __forceinline__ acc_t add(acc_t a, acc_t b) { return {a.re + b.re, a.im + b.im}; }
    static __device__ __forceinline__ stor narrow(acc_t x) { return {(S)x.re, (S)x.im}; }
};

template <class N_>
__global__ __launch_bounds__(256) void generic_contract(GenericArgs g) {
    using T = typename N_::stor;
    const int64_t lin = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (lin >= g.sizeD) return;
    // decode the D index, D-fastest mode first
    int64_t rem = lin, offA = 0, offB = 0, offD = 0;
    for (int i = 0; i < g.nD; ++i) {
        const int64_t e = g.dExt[i];
        const int64_t q = rem / e, idx = rem - q * e;
        rem = q;
        offA += idx * g.dSA[i];
        offB += idx * g.dSB[i];
        offD += idx * g.dSD[i];
    }
    const T* A = (const T*)g.A;
    const T* B = (const T*)g.B;
    typename N_::acc_t acc = N_::zero();
    if (g.read_ab) {
        // odometer over the contracted modes, first mode fastest
        int64_t kidx[kMaxGenericModes];
        for (int i = 0; i < g.nK; ++i) kidx[i] = 0;
        int64_t oa = offA, ob = offB;
        for (int64_t k = 0; k < g.sizeK; ++k) {
            acc = N_::fma(N_::load(A, oa, g.opA), N_::load(B, ob, g.opB), acc);
            for (int i = 0; i < g.nK; ++i) {
                if (++kidx[i] < g.kExt[i]) { oa += g.kSA[i]; ob += g.kSB[i]; break; }
                oa -= g.kSA[i] * (g.kExt[i] - 1);
                ob -= g.kSB[i] * (g.kExt[i] - 1);
                kidx[i] = 0;
            }
        }
    }
    typename N_::acc_t d = N_::scale(g.s, true, acc);
    if (g.read_c) d = N_::add(d, N_::scale(g.s, false, N_::load((const T*)g.C, offD, g.opC)));
    ((T*)g.D)[offD] = N_::narrow(d);
}

// Pre-reduction of an operand over its isolated labels (paper, Sec. "Case 4"): one thread per
// element of the reduced operand, which is dense (the linear index is the offset), a loop over
// the summed index space.  Sums are formed in the plan's arithmetic, stored in the storage type.
template <class N_>
__global__ __launch_bounds__(256) void reduce_operand(ReduceArgs g) {
    using T = typename N_::stor;
    const int64_t lin = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (lin >= g.count) return;
    int64_t rem = lin, off = 0;
    for (int i = 0; i < g.nKeep; ++i) {
        const int64_t e = g.keepExt[i];
        const int64_t q = rem / e;
        off += (rem - q * e) * g.keepSrc[i];
        rem = q;
    }
    const T* src = (const T*)g.src;
    typename N_::acc_t acc = N_::zero();
    int64_t idx[kMaxGenericModes];
    for (int i = 0; i < g.nSum; ++i) idx[i] = 0;
    for (int64_t k = 0; k < g.sumCount; ++k) {
        acc = N_::add(acc, N_::load(src, off, TCX_OP_IDENTITY));
        for (int i = 0; i < g.nSum; ++i) {
            if (++idx[i] < g.sumExt[i]) { off += g.sumSrc[i]; break; }
            off -= g.sumSrc[i] * (g.sumExt[i] - 1);
            idx[i] = 0;
        }
    }
    ((T*)g.dst)[lin] = N_::narrow(acc);
}

}  // namespace

int launch_reduce(int dtype, int precision, const ReduceArgs& args, void* stream) {
    const int64_t blocks = (args.count + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffff) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    const dim3 gr((unsigned)blocks), bl(256);
    const bool wide = is_widened(dtype, precision);
    switch (dtype) {
        case TCX_F64: reduce_operand<RealNum<double, double>><<<gr, bl, 0, st>>>(args); break;
        case TCX_F32:
            if (wide) reduce_operand<RealNum<float, double>><<<gr, bl, 0, st>>>(args);
            else reduce_operand<RealNum<float, float>><<<gr, bl, 0, st>>>(args);
            break;
        case TCX_F16:
            if (precision == TCX_PREC_F64) reduce_operand<RealNum<_Float16, double>><<<gr, bl, 0, st>>>(args);
            else reduce_operand<RealNum<_Float16, float>><<<gr, bl, 0, st>>>(args);
            break;
        case TCX_BF16:
            if (precision == TCX_PREC_F64) reduce_operand<RealNum<bf16_t, double>><<<gr, bl, 0, st>>>(args);
            else reduce_operand<RealNum<bf16_t, float>><<<gr, bl, 0, st>>>(args);
            break;
        case TCX_C128: reduce_operand<ComplexNum<double, double>><<<gr, bl, 0, st>>>(args); break;
        case TCX_C64:
            if (wide) reduce_operand<ComplexNum<float, double>><<<gr, bl, 0, st>>>(args);
            else reduce_operand<ComplexNum<float, float>><<<gr, bl, 0, st>>>(args);
            break;
        default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

int launch_generic(int dtype, int precision, const GenericArgs& args, void* stream, int64_t* grid, int* block) {
    const int64_t blocks = (args.sizeD + 255) / 256;
    *grid = blocks;
    *block = 256;
    if (blocks > 0x7fffffff) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    const dim3 gr((unsigned)blocks), bl(256);
    const bool wide = is_widened(dtype, precision);
    switch (dtype) {
        case TCX_F64: generic_contract<RealNum<double, double>><<<gr, bl, 0, st>>>(args); break;
        case TCX_F32:
            if (wide) generic_contract<RealNum<float, double>><<<gr, bl, 0, st>>>(args);
            else generic_contract<RealNum<float, float>><<<gr, bl, 0, st>>>(args);
            break;
        case TCX_F16:
            if (precision == TCX_PREC_F64) generic_contract<RealNum<_Float16, double>><<<gr, bl, 0, st>>>(args);
            else generic_contract<RealNum<_Float16, float>><<<gr, bl, 0, st>>>(args);
            break;
        case TCX_BF16:
            if (precision == TCX_PREC_F64) generic_contract<RealNum<bf16_t, double>><<<gr, bl, 0, st>>>(args);
            else generic_contract<RealNum<bf16_t, float>><<<gr, bl, 0, st>>>(args);
            break;
        case TCX_C128: generic_contract<ComplexNum<double, double>><<<gr, bl, 0, st>>>(args); break;
        case TCX_C64:
            if (wide) generic_contract<ComplexNum<float, double>><<<gr, bl, 0, st>>>(args);
            else generic_contract<ComplexNum<float, float>><<<gr, bl, 0, st>>>(args);
            break;
        default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

}  // namespace tcx
