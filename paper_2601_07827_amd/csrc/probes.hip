// Measurement aids: plain kernels that do one kind of work only, so that a benchmark can print
// what this chip sustains next to its specification figures -- back-to-back MFMAs from every wave
// (the matrix pipes' achievable rate), a store loop and a copy loop (the memory system's achievable
// rate for a perfectly coalesced stream).  Nothing in the contraction path uses them.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "tcx_internal.hpp"

namespace tcx {
namespace {

typedef double double4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef double plain_double2 __attribute__((ext_vector_type(2)));

constexpr int kProbeAcc = 16;        // independent accumulators per wave: no MFMA waits for another
constexpr int kProbeThreads = 512;   // two waves per SIMD

template <class T, class V> __device__ __forceinline__ V probe_mac(T a, T b, V c);
template <> __device__ __forceinline__ double4_t probe_mac<double, double4_t>(double a, double b, double4_t c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}
template <> __device__ __forceinline__ float4_t probe_mac<float, float4_t>(float a, float b, float4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

template <class T, class V>
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(T* out, int64_t iters) {
    const T a = (T)(threadIdx.x & 7), b = (T)1;
    V acc[kProbeAcc];
#pragma unroll
    for (int i = 0; i < kProbeAcc; ++i) acc[i] = V{0, 0, 0, 0};
    for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kProbeAcc; ++i) acc[i] = probe_mac<T, V>(a, b, acc[i]);
    }
    T s = 0;
#pragma unroll
    for (int i = 0; i < kProbeAcc; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == (T)-1) out[0] = s;          // never true (sums of non-negative products): keeps the loop alive, stores nothing
}

// A workgroup moves tiles of 2048 consecutive 16-byte items (32 KB), eight items per thread with
// consecutive lanes on consecutive items, all eight accesses issued before any is waited for.
constexpr int kProbeTile = 2048;
__global__ __launch_bounds__(256) void store_probe_kernel(plain_double2* dst, int64_t tiles) {
    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
        plain_double2* p = dst + t * kProbeTile + threadIdx.x;
#pragma unroll
        for (int r = 0; r < 8; ++r) p[r * 256] = plain_double2{1.0, (double)r};
    }
}
__global__ __launch_bounds__(256) void copy_probe_kernel(const plain_double2* __restrict__ src, plain_double2* __restrict__ dst, int64_t tiles) {
    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
        const plain_double2* s = src + t * kProbeTile + threadIdx.x;
        plain_double2* p = dst + t * kProbeTile + threadIdx.x;
        plain_double2 v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = s[r * 256];
#pragma unroll
        for (int r = 0; r < 8; ++r) p[r * 256] = v[r];
    }
}

}  // namespace

int launch_probe(int kind, void* buffer, size_t bytes, int64_t iters, int num_cu, void* stream, double* work) {
    hipStream_t st = (hipStream_t)stream;
    const int cus = num_cu > 0 ? num_cu : 256;
    *work = 0;
    if (kind == TCX_PROBE_MFMA_F64 || kind == TCX_PROBE_MFMA_F32) {
        if (iters <= 0 || !buffer || bytes < 16) return (int)hipErrorInvalidValue;
        if (kind == TCX_PROBE_MFMA_F64)
            mfma_probe_kernel<double, double4_t><<<dim3((unsigned)cus), dim3(kProbeThreads), 0, st>>>((double*)buffer, iters);
        else
            mfma_probe_kernel<float, float4_t><<<dim3((unsigned)cus), dim3(kProbeThreads), 0, st>>>((float*)buffer, iters);
        // a 16 x 16 x 4 MFMA is 2 * 16 * 16 * 4 flop
        *work = (double)cus * (kProbeThreads / 64) * (double)iters * kProbeAcc * 2048.0;
    } else if (kind == TCX_PROBE_STORE || kind == TCX_PROBE_COPY) {
        // whole tiles only: what is left of the buffer beyond them is not touched
        const int64_t tiles = (int64_t)(kind == TCX_PROBE_COPY ? bytes / 2 : bytes) / 16 / kProbeTile;
        if (!buffer || tiles <= 0) return (int)hipErrorInvalidValue;
        const int64_t blocks = std::min<int64_t>(tiles, (int64_t)cus * 64);
        if (kind == TCX_PROBE_STORE) {
            store_probe_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>((plain_double2*)buffer, tiles);
            *work = (double)tiles * kProbeTile * 16.0;
        } else {
            copy_probe_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>((const plain_double2*)buffer,
                                                                           (plain_double2*)buffer + tiles * kProbeTile, tiles);
            *work = (double)tiles * kProbeTile * 32.0;      // read + written
        }
    } else {
        return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

}  // namespace tcx
