// Bandwidth (streaming) contraction kernel for shapes of low arithmetic intensity: few
// contracted terms per output, output (and C) dominating the traffic -- outer products,
// Hadamard products, tiny-|K| contractions of high-rank small-extent tensors.
//
// Output-stationary.  A workgroup walks over tiles of D; a tile is made of D's fastest modes,
// so a wave's stores cover one contiguous stretch of D, however the modes of D map to
// modes of A and B.  Per tile the needed elements of A and B (rows x K) are staged through LDS
// by a plan-time list sorted by source address -- loads follow A's and B's own memory order,
// LDS does the permutation.  Then every thread forms its outputs from LDS:
//     D[e] = alpha * sum_k A_s[rowA(e)][k] * B_s[rowB(e)][k] + beta * op(C[e])
// (paper, Eq. case2, with the hyper, free and contracted labels all folded into the row/k
// lookup tables), with FMAs on the vector ALUs.
#include <hip/hip_runtime.h>

#include "tcx_internal.hpp"

namespace tcx {
namespace {

template <class T> struct SNum;
template <> struct SNum<double> {
    static __device__ __forceinline__ double ld(const double* p, int64_t o, int) { return p[o]; }
    static __device__ __forceinline__ double zero() { return 0.0; }
    static __device__ __forceinline__ double fma(double a, double b, double c) { return __builtin_fma(a, b, c); }
    static __device__ __forceinline__ double out(const Scalars& s, double acc, bool rc, const double* C, int64_t o, int) {
        double d = s.alpha_re * acc;
        if (rc) d += s.beta_re * C[o];
        return d;
    }
};
template <> struct SNum<float> {
    static __device__ __forceinline__ float ld(const float* p, int64_t o, int) { return p[o]; }
    static __device__ __forceinline__ float zero() { return 0.0f; }
    static __device__ __forceinline__ float fma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
    static __device__ __forceinline__ float out(const Scalars& s, float acc, bool rc, const float* C, int64_t o, int) {
        float d = (float)s.alpha_re * acc;
        if (rc) d += (float)s.beta_re * C[o];
        return d;
    }
};
template <> struct SNum<double2> {
    static __device__ __forceinline__ double2 ld(const double2* p, int64_t o, int op) {
        double2 v = p[o];
        if (op == TCX_OP_CONJ) v.y = -v.y;
        return v;
    }
    static __device__ __forceinline__ double2 zero() { return double2{0.0, 0.0}; }
    static __device__ __forceinline__ double2 fma(double2 a, double2 b, double2 c) {
        c.x = __builtin_fma(a.x, b.x, c.x);
        c.x = __builtin_fma(-a.y, b.y, c.x);
        c.y = __builtin_fma(a.x, b.y, c.y);
        c.y = __builtin_fma(a.y, b.x, c.y);
        return c;
    }
    static __device__ __forceinline__ double2 out(const Scalars& s, double2 acc, bool rc, const double2* C, int64_t o, int opC) {
        double2 d{s.alpha_re * acc.x - s.alpha_im * acc.y, s.alpha_re * acc.y + s.alpha_im * acc.x};
        if (rc) {
            double2 c = C[o];
            if (opC == TCX_OP_CONJ) c.y = -c.y;
            d.x += s.beta_re * c.x - s.beta_im * c.y;
            d.y += s.beta_re * c.y + s.beta_im * c.x;
        }
        return d;
    }
};

// KC > 0: the number of contracted terms is the compile-time constant KC (inner loop unrolled);
// KC == 0: any K.
template <class T, int KC>
__global__ __launch_bounds__(kStreamThreads) void stream_kernel(StreamArgs g) {
    using N_ = SNum<T>;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    T* sA = (T*)lds_raw;
    T* sB = sA + (size_t)g.rowsA * g.K;
    const int K = KC > 0 ? KC : g.K;
    const int tid = threadIdx.x;

    for (int64_t tile = blockIdx.x; tile < g.num_tiles; tile += gridDim.x) {
        // outer index -> base offsets of this tile (uniform over the workgroup)
        int64_t rem = tile, baseA = 0, baseB = 0, baseD = 0, first = 0;
        for (int i = 0; i < g.n_outer; ++i) {
            const int64_t q = rem / g.oExt[i], idx = rem - q * g.oExt[i];
            rem = q;
            if (i == 0) first = idx;
            baseA += idx * g.oSA[i];
            baseB += idx * g.oSB[i];
            baseD += idx * g.oSD[i];
        }
        // the split mode's last chunk may be ragged
        const int64_t left = g.split_extent - first * g.chunk;
        const unsigned digits = (unsigned)(left < g.chunk ? left : g.chunk);
        const int valid = g.inner * (int)digits;

        __syncthreads();          // the previous tile's reads of LDS are done
        const T* A = (const T*)g.A + baseA;
        const T* B = (const T*)g.B + baseB;
        for (int p = tid; p < g.nItemsA; p += kStreamThreads) {
            const StreamItem it = g.itemsA[p];
            if (it.digit < digits) sA[it.slot] = N_::ld(A, it.src, g.opA);
        }
        for (int p = tid; p < g.nItemsB; p += kStreamThreads) {
            const StreamItem it = g.itemsB[p];
            if (it.digit < digits) sB[it.slot] = N_::ld(B, it.src, g.opB);
        }
        __syncthreads();

        const T* C = (const T*)g.C + baseD;
        T* D = (T*)g.D + baseD;
        for (int e = tid; e < valid; e += kStreamThreads) {
            const unsigned rab = g.rowAB[e];
            const int64_t off = g.dD[e];
            const T* a = sA + (size_t)(rab & 0xffffu) * K;
            const T* b = sB + (size_t)(rab >> 16) * K;
            T acc = N_::zero();
            if (KC > 0) {
#pragma unroll
                for (int k = 0; k < KC; ++k) acc = N_::fma(a[k], b[k], acc);
            } else {
                for (int k = 0; k < K; ++k) acc = N_::fma(a[k], b[k], acc);
            }
            D[off] = N_::out(g.s, acc, g.read_c != 0, C, off, g.opC);
        }
    }
}

template <class T>
hipError_t launch_k(const StreamArgs& a, size_t lds, unsigned blocks, hipStream_t st) {
    switch (a.K) {
        case 1: stream_kernel<T, 1><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
        case 2: stream_kernel<T, 2><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
        case 4: stream_kernel<T, 4><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
        case 8: stream_kernel<T, 8><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
        default: stream_kernel<T, 0><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
    }
    return hipGetLastError();
}

}  // namespace

int launch_stream(int dtype, const StreamArgs& args, size_t lds_bytes, int num_cu, void* stream, int64_t* grid,
                  int* block) {
    // persistent-style grid: enough workgroups to fill every CU several times over, each
    // walking the tile list with a grid stride
    const int64_t cap = (int64_t)(num_cu > 0 ? num_cu : 256) * 8;
    const int64_t blocks = args.num_tiles < cap ? args.num_tiles : cap;
    *grid = blocks;
    *block = kStreamThreads;
    if (blocks <= 0) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    switch (dtype) {
        case TCX_F64: return (int)launch_k<double>(args, lds_bytes, (unsigned)blocks, st);
        case TCX_F32: return (int)launch_k<float>(args, lds_bytes, (unsigned)blocks, st);
        case TCX_C128: return (int)launch_k<double2>(args, lds_bytes, (unsigned)blocks, st);
        default: return (int)hipErrorInvalidValue;
    }
}

}  // namespace tcx
