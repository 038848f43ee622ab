// Generic strided contraction kernel: one thread per element of D, a loop over the whole
// contracted index space, 64-bit element offsets.  It mirrors the structure of the paper's
// loop nest (Sec. "Algorithm Structure", Fig. "implementation": the H, F_A and F_B loops
// folded into one index over D, the P loop innermost) with the outer index spread over
// the grid.  It handles every dtype, op, stride sign and rank the analyser accepts and is
// the fallback for shapes the tiled kernels do not take.
#include <hip/hip_runtime.h>

#include "tcx_internal.hpp"

namespace tcx {
namespace {

struct cplx {
    double re, im;
};

template <class T> struct Num;
template <> struct Num<double> {
    using acc_t = double;
    static __device__ __forceinline__ double load(const double* p, int64_t off, int) { return p[off]; }
    static __device__ __forceinline__ double zero() { return 0.0; }
    static __device__ __forceinline__ double fma(double a, double b, double c) { return __builtin_fma(a, b, c); }
    static __device__ __forceinline__ double scale(const Scalars& s, bool alpha, double x) {
        return (alpha ? s.alpha_re : s.beta_re) * x;
    }
    static __device__ __forceinline__ double add(double a, double b) { return a + b; }
};
template <> struct Num<float> {
    using acc_t = float;
    static __device__ __forceinline__ float load(const float* p, int64_t off, int) { return p[off]; }
    static __device__ __forceinline__ float zero() { return 0.0f; }
    static __device__ __forceinline__ float fma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
    static __device__ __forceinline__ float scale(const Scalars& s, bool alpha, float x) {
        return (float)(alpha ? s.alpha_re : s.beta_re) * x;
    }
    static __device__ __forceinline__ float add(float a, float b) { return a + b; }
};
template <> struct Num<cplx> {
    using acc_t = cplx;
    static __device__ __forceinline__ cplx load(const cplx* p, int64_t off, int op) {
        cplx v = p[off];
        if (op == TCX_OP_CONJ) v.im = -v.im;
        return v;
    }
    static __device__ __forceinline__ cplx zero() { return {0.0, 0.0}; }
    static __device__ __forceinline__ cplx fma(cplx a, cplx b, cplx c) {
        c.re = __builtin_fma(a.re, b.re, c.re);
        c.re = __builtin_fma(-a.im, b.im, c.re);
        c.im = __builtin_fma(a.re, b.im, c.im);
        c.im = __builtin_fma(a.im, b.re, c.im);
        return c;
    }
    static __device__ __forceinline__ cplx scale(const Scalars& s, bool alpha, cplx x) {
        const double sr = alpha ? s.alpha_re : s.beta_re, si = alpha ? s.alpha_im : s.beta_im;
        return {sr * x.re - si * x.im, sr * x.im + si * x.re};
    }
    static __device__ __forceinline__ cplx add(cplx a, cplx b) { return {a.re + b.re, a.im + b.im}; }
};

template <class T>
__global__ __launch_bounds__(256) void generic_contract(GenericArgs g) {
    using N_ = Num<T>;
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
    T d = N_::scale(g.s, true, acc);
    if (g.read_c) d = N_::add(d, N_::scale(g.s, false, N_::load((const T*)g.C, offD, g.opC)));
    ((T*)g.D)[offD] = d;
}

}  // namespace

int launch_generic(int dtype, const GenericArgs& args, void* stream, int64_t* grid, int* block) {
    const int64_t blocks = (args.sizeD + 255) / 256;
    *grid = blocks;
    *block = 256;
    if (blocks > 0x7fffffff) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    switch (dtype) {
        case TCX_F64: generic_contract<double><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(args); break;
        case TCX_F32: generic_contract<float><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(args); break;
        case TCX_C128: generic_contract<cplx><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(args); break;
        default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

}  // namespace tcx
