// Tiled, stride-aware contraction kernels for gfx950 (fp64, fp32, and complex128 as real pairs).
//
// The contraction is treated as |H| independent products of an |M| x |K| by |K| x |N|
// operand pair (paper, Eqs. case1, case2: M = F_A, N = F_B, K = P), but no operand is ever
// transposed or packed in memory: a workgroup gathers its MT_M x KT slab of A and KT x MT_N
// slab of B straight from the strided tensors into LDS.  Element addresses are additively
// separable -- offset(m, k) = oM[m] + oK[k], because the paper's `offset` helper
// (Fig. "helper-functions") is linear in the indices -- so two small tables per operand,
// built at plan time, replace the per-term index arithmetic of the reference loop nest.
// Lanes run along whichever of the operand's two index groups holds its smallest stride, so
// global loads are coalesced for either orientation, and LDS keeps that orientation
// ([k][m] or [m][k]); only the MFMA fragment read differs.  Accumulation is register
// blocked over 16x16x4 MFMA tiles; the alpha/beta epilogue scatters to strided D with lanes
// along D's fastest group (the MFMA operand roles are swapped to make that so).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "tcx_internal.hpp"

namespace tcx {
namespace {

typedef double double4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// 16x16x4 MFMA: the row operand is held as (row = lane % 16, k = lane / 16), the column
// operand as (col = lane % 16, k = lane / 16); the result register v of a lane holds column
// lane % 16 and the row given by row_of().
template <class T> struct Mfma;
template <> struct Mfma<double> {
    using vec = double4_t;
    static __device__ __forceinline__ vec mac(double rowop, double colop, vec c) {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(rowop, colop, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_of(int lane, int v) { return 4 * v + (lane >> 4); }
};
template <> struct Mfma<float> {
    using vec = float4_t;
    static __device__ __forceinline__ vec mac(float rowop, float colop, vec c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(rowop, colop, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_of(int lane, int v) { return 4 * (lane >> 4) + v; }
};

// ---- arithmetic policies: what an element is, how a 16x16x4 block is accumulated, and how
// the epilogue combines alpha, beta, the accumulator and op(C) --------------------------------
template <class R> struct RealPolicy {
    using elem = R;
    using MF = Mfma<R>;
    using vec = typename MF::vec;
    struct acc_t {
        vec v;
    };
    static __device__ __forceinline__ void clear(acc_t& c) { c.v = vec{0, 0, 0, 0}; }
    static __device__ __forceinline__ elem zero() { return R(0); }
    static __device__ __forceinline__ elem load(const elem* p, int64_t off, unsigned) { return p[off]; }
    template <bool DNF> static __device__ __forceinline__ void mac(elem a, elem b, acc_t& c) {
        c.v = DNF ? MF::mac(a, b, c.v)      // rows = m, lanes along n
                  : MF::mac(b, a, c.v);     // rows = n, lanes along m
    }
    static __device__ __forceinline__ void store(elem* D, const elem* C, int64_t off, const acc_t& c, int v,
                                                 const Scalars& s, bool read_c, int) {
        R d = (R)s.alpha_re * c.v[v];
        if (read_c) d += (R)s.beta_re * C[off];
        D[off] = d;
    }
};

// complex128 as pairs of reals: four real MFMAs per complex 16x16x4 block,
//   re += ar*br - ai*bi,  im += ar*bi + ai*br.
// Conjugation is applied once, as the element is gathered (the sign bit of the imaginary part
// is flipped), so the main loop does not depend on the ops.
struct ComplexPolicy {
    using elem = double2;
    using MF = Mfma<double>;
    using vec = double4_t;
    struct acc_t {
        vec re, im;
    };
    static __device__ __forceinline__ void clear(acc_t& c) { c.re = vec{0, 0, 0, 0}; c.im = vec{0, 0, 0, 0}; }
    static __device__ __forceinline__ elem zero() { return double2{0.0, 0.0}; }
    static __device__ __forceinline__ elem load(const elem* p, int64_t off, unsigned conj_mask_hi) {
        elem v = p[off];
        unsigned long long bits = __builtin_bit_cast(unsigned long long, v.y) ^ ((unsigned long long)conj_mask_hi << 32);
        v.y = __builtin_bit_cast(double, bits);
        return v;
    }
    template <bool DNF> static __device__ __forceinline__ void mac(elem a, elem b, acc_t& c) {
        const double nai = -a.y;
        if (DNF) {
            c.re = MF::mac(a.x, b.x, c.re);
            c.re = MF::mac(nai, b.y, c.re);
            c.im = MF::mac(a.x, b.y, c.im);
            c.im = MF::mac(a.y, b.x, c.im);
        } else {
            c.re = MF::mac(b.x, a.x, c.re);
            c.re = MF::mac(b.y, nai, c.re);
            c.im = MF::mac(b.y, a.x, c.im);
            c.im = MF::mac(b.x, a.y, c.im);
        }
    }
    static __device__ __forceinline__ void store(elem* D, const elem* C, int64_t off, const acc_t& c, int v,
                                                 const Scalars& s, bool read_c, int opC) {
        const double re = c.re[v], im = c.im[v];
        double dr = s.alpha_re * re - s.alpha_im * im;
        double di = s.alpha_re * im + s.alpha_im * re;
        if (read_c) {
            elem cc = C[off];
            if (opC == TCX_OP_CONJ) cc.y = -cc.y;
            dr += s.beta_re * cc.x - s.beta_im * cc.y;
            di += s.beta_re * cc.y + s.beta_im * cc.x;
        }
        D[off] = double2{dr, di};
    }
};

constexpr int kPadMN = 16;   // [k][mn] rows: the four k-rows of a fragment land on distinct banks
constexpr int kPadK = 1;     // [mn][k] rows: odd row pitch spreads the 16 rows of a fragment

// One operand's slab: MT rows (m or n) by KT contracted indices.
template <class T, int MT, int KT, int NT, bool KF>
struct Slab {
    static constexpr int PER = MT * KT / NT;                       // elements per thread per slab
    static constexpr int LD = KF ? KT + kPadK : MT + kPadMN;
    static constexpr int ELEMS = KF ? MT * LD : KT * LD;
    static_assert(MT * KT % NT == 0, "slab must divide evenly over the workgroup");
    // lanes run along the rows and a wave covers whole rows' worth: one k index per wave
    static constexpr bool UNIFORM_K = !KF && MT % 64 == 0 && (NT % MT == 0 || MT % NT == 0);

    static __device__ __forceinline__ int row(int e) { return KF ? e / KT : e % MT; }
    static __device__ __forceinline__ int kin(int e) { return KF ? e % KT : e / MT; }
    static __device__ __forceinline__ int lds_index(int e) { return KF ? row(e) * LD + kin(e) : kin(e) * LD + row(e); }
    // fragment element for (row r of the slab, k index kk of the slab)
    static __device__ __forceinline__ int frag_index(int r, int kk) { return KF ? r * LD + kk : kk * LD + r; }
};

template <class P, int MT_M, int MT_N, int KT, int WGM, int WGN, bool AKF, bool BKF, bool DNF>
__global__ __launch_bounds__(WGM* WGN * 64) void gett_kernel(GettArgs g) {
    using T = typename P::elem;
    using acc_t = typename P::acc_t;
    constexpr int NT = WGM * WGN * 64;
    constexpr int WT_M = MT_M / WGM, WT_N = MT_N / WGN;
    constexpr int FM = WT_M / 16, FN = WT_N / 16;
    using SA = Slab<T, MT_M, KT, NT, AKF>;
    using SB = Slab<T, MT_N, KT, NT, BKF>;
    using MF = typename P::MF;
    static_assert(KT % 4 == 0 && WT_M % 16 == 0 && WT_N % 16 == 0, "tile shape");

    __shared__ T lds[2 * (SA::ELEMS + SB::ELEMS)];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;

    // ---- which tile: consecutive workgroup ids go round-robin over the 8 XCDs, so give
    // each XCD one contiguous stretch of the tile order (its own L2 then sees neighbouring
    // tiles), and walk tiles in bands of 8 tile-rows.
    int64_t lid = blockIdx.x;
    {
        const int64_t nb = gridDim.x, per = nb / 8;
        if (lid < per * 8) lid = (lid % 8) * per + lid / 8;
    }
    const int64_t tiles_per_h = (int64_t)g.tilesM * g.tilesN;
    const int64_t h = lid / tiles_per_h;
    const int t = (int)(lid - h * tiles_per_h);
    constexpr int BAND = 8;
    const int band = t / (BAND * g.tilesN);
    const int first_m = band * BAND;
    const int band_rows = min(BAND, g.tilesM - first_m);
    const int in_band = t - band * BAND * g.tilesN;
    const int tm = first_m + in_band % band_rows;
    const int tn = in_band / band_rows;
    const int64_t m0 = (int64_t)tm * MT_M, n0 = (int64_t)tn * MT_N;

    // ---- hyper index -> base offsets (Eq. case2: an independent product per value of H)
    int64_t hA = 0, hB = 0, hD = 0;
    {
        int64_t rem = h;
        for (int i = 0; i < g.nH; ++i) {
            const int64_t q = rem / g.hExt[i], idx = rem - q * g.hExt[i];
            rem = q;
            hA += idx * g.hSA[i];
            hB += idx * g.hSB[i];
            hD += idx * g.hSD[i];
        }
    }
    const T* __restrict__ A = (const T*)g.A + hA;
    const T* __restrict__ B = (const T*)g.B + hB;

    // ---- loop-invariant part of the gather: this thread's row offsets.  Rows past the end of
    // M or N read a valid (padded) table entry; what they accumulate is never stored.
    int64_t offA[SA::PER], offB[SB::PER];
#pragma unroll
    for (int i = 0; i < SA::PER; ++i) offA[i] = g.oAM[m0 + SA::row(tid + i * NT)];
#pragma unroll
    for (int i = 0; i < SB::PER; ++i) offB[i] = g.oBN[n0 + SB::row(tid + i * NT)];

    // Offsets along K come from the tables one slab ahead of the data loads that use them,
    // so a data load never waits on a table load issued in the same iteration.  Where the
    // k index is the same for a whole wave it is made scalar, which turns the table read
    // into a scalar load.
    const int nk = g.tilesK;
    unsigned kinA[SA::PER], kinB[SB::PER];       // this thread's k index inside a slab, per element
#pragma unroll
    for (int i = 0; i < SA::PER; ++i) {
        kinA[i] = (unsigned)SA::kin(tid + i * NT);
        if (SA::UNIFORM_K) kinA[i] = __builtin_amdgcn_readfirstlane(kinA[i]);
    }
#pragma unroll
    for (int i = 0; i < SB::PER; ++i) {
        kinB[i] = (unsigned)SB::kin(tid + i * NT);
        if (SB::UNIFORM_K) kinB[i] = __builtin_amdgcn_readfirstlane(kinB[i]);
    }
    int64_t kA[SA::PER], kB[SB::PER];
    auto k_offsets = [&](int kt) {
        const int64_t* __restrict__ ta = g.oAK + (int64_t)min(kt, nk - 1) * KT;
        const int64_t* __restrict__ tb = g.oBK + (int64_t)min(kt, nk - 1) * KT;
#pragma unroll
        for (int i = 0; i < SA::PER; ++i) kA[i] = ta[kinA[i]];
#pragma unroll
        for (int i = 0; i < SB::PER; ++i) kB[i] = tb[kinB[i]];
    };

    T ra[SA::PER], rb[SB::PER];
    const unsigned conjA = g.opA == TCX_OP_CONJ ? 0x80000000u : 0u;
    const unsigned conjB = g.opB == TCX_OP_CONJ ? 0x80000000u : 0u;
    // Data loads of slab kt; k_offsets(kt) must have been issued before.  Unconditional: the
    // tables are padded with offsets of valid elements.
    auto gather = [&]() {
#pragma unroll
        for (int i = 0; i < SA::PER; ++i) ra[i] = P::load(A, offA[i] + kA[i], conjA);
#pragma unroll
        for (int i = 0; i < SB::PER; ++i) rb[i] = P::load(B, offB[i] + kB[i], conjB);
    };
    // The last slab of a ragged K holds padded k entries whose (valid, arbitrary) values must
    // not be summed: zero them after the load.
    auto mask_last = [&]() {
        const unsigned kleft = (unsigned)(g.sizeK - (int64_t)(nk - 1) * KT);
#pragma unroll
        for (int i = 0; i < SA::PER; ++i) ra[i] = kinA[i] < kleft ? ra[i] : P::zero();
#pragma unroll
        for (int i = 0; i < SB::PER; ++i) rb[i] = kinB[i] < kleft ? rb[i] : P::zero();
    };
    auto stage = [&](int buf) {
        T* sa = lds + buf * (SA::ELEMS + SB::ELEMS);
        T* sb = sa + SA::ELEMS;
#pragma unroll
        for (int i = 0; i < SA::PER; ++i) sa[SA::lds_index(tid + i * NT)] = ra[i];
#pragma unroll
        for (int i = 0; i < SB::PER; ++i) sb[SB::lds_index(tid + i * NT)] = rb[i];
    };

    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) P::clear(acc[i][j]);

    const int fr = lane & 15, fq = lane >> 4;
    auto compute = [&](int buf) {
        const T* sa = lds + buf * (SA::ELEMS + SB::ELEMS);
        const T* sb = sa + SA::ELEMS;
#pragma unroll
        for (int ks = 0; ks < KT; ks += 4) {
            T fa[FM], fb[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) fa[i] = sa[SA::frag_index(wm * WT_M + i * 16 + fr, ks + fq)];
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[j] = sb[SB::frag_index(wn * WT_N + j * 16 + fr, ks + fq)];
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) P::template mac<DNF>(fa[i], fb[j], acc[i][j]);
        }
    };

    // ---- main loop: the data loads of slab kt+1 and the table loads of slab kt+2 are in
    // flight while the MFMAs run on slab kt.  The last two slabs are peeled so that the loop
    // body is one straight path.
    const bool ragged_k = g.sizeK % KT != 0;
    k_offsets(0);
    gather();
    k_offsets(1);
    if (ragged_k && nk == 1) mask_last();
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int kt = 0; kt + 2 < nk; ++kt) {
        gather();                 // slab kt+1
        k_offsets(kt + 2);
        compute(buf);
        stage(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    if (nk >= 2) {
        gather();                 // slab nk-1
        compute(buf);
        if (ragged_k) mask_last();
        stage(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
    compute(buf);

    // ---- epilogue: D = alpha * acc + beta * C, scattered through D's offset tables
    const T* __restrict__ C = (const T*)g.C + hD;
    T* __restrict__ D = (T*)g.D + hD;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int rr = MF::row_of(lane, v);
                const int ml = wm * WT_M + i * 16 + (DNF ? rr : fr);
                const int nl = wn * WT_N + j * 16 + (DNF ? fr : rr);
                if (m0 + ml < g.sizeM && n0 + nl < g.sizeN)
                    P::store(D, C, g.oDM[m0 + ml] + g.oDN[n0 + nl], acc[i][j], v, g.s, g.read_c != 0, g.opC);
            }
}

// ---- instantiation tables -------------------------------------------------------------------
struct Shape {
    int mt_m, mt_n, kt, wgm, wgn;
    float efficiency;      // relative speed of the main loop per unit of tile area (planner's cost model)
};
constexpr Shape kRealShapes[] = {
    {256, 128, 16, 4, 2, 1.00f},
    {128, 128, 16, 2, 2, 0.80f},
    {64, 64, 16, 2, 2, 0.55f},
    {32, 32, 16, 2, 2, 0.25f},
};
constexpr Shape kComplexShapes[] = {
    {96, 96, 8, 2, 2, 1.00f},
    {64, 64, 8, 2, 2, 0.85f},
    {32, 32, 8, 2, 2, 0.40f},
};
constexpr int kNumRealShapes = sizeof(kRealShapes) / sizeof(Shape);
constexpr int kNumComplexShapes = sizeof(kComplexShapes) / sizeof(Shape);

template <class P, int S, bool AKF, bool BKF, bool DNF>
hipError_t launch_one(const GettArgs& a, int64_t blocks, hipStream_t st) {
    constexpr Shape s = std::is_same<P, ComplexPolicy>::value ? kComplexShapes[S] : kRealShapes[S];
    gett_kernel<P, s.mt_m, s.mt_n, s.kt, s.wgm, s.wgn, AKF, BKF, DNF>
        <<<dim3((unsigned)blocks), dim3(s.wgm * s.wgn * 64), 0, st>>>(a);
    return hipGetLastError();
}

template <class P, int S>
hipError_t launch_flags(bool akf, bool bkf, bool dnf, const GettArgs& a, int64_t blocks, hipStream_t st) {
    const int f = (akf ? 4 : 0) | (bkf ? 2 : 0) | (dnf ? 1 : 0);
    switch (f) {
        case 0: return launch_one<P, S, false, false, false>(a, blocks, st);
        case 1: return launch_one<P, S, false, false, true>(a, blocks, st);
        case 2: return launch_one<P, S, false, true, false>(a, blocks, st);
        case 3: return launch_one<P, S, false, true, true>(a, blocks, st);
        case 4: return launch_one<P, S, true, false, false>(a, blocks, st);
        case 5: return launch_one<P, S, true, false, true>(a, blocks, st);
        case 6: return launch_one<P, S, true, true, false>(a, blocks, st);
        default: return launch_one<P, S, true, true, true>(a, blocks, st);
    }
}

template <class P>
hipError_t launch_real_shape(int variant, bool akf, bool bkf, bool dnf, const GettArgs& a, int64_t blocks, hipStream_t st) {
    switch (variant) {
        case 0: return launch_flags<P, 0>(akf, bkf, dnf, a, blocks, st);
        case 1: return launch_flags<P, 1>(akf, bkf, dnf, a, blocks, st);
        case 2: return launch_flags<P, 2>(akf, bkf, dnf, a, blocks, st);
        case 3: return launch_flags<P, 3>(akf, bkf, dnf, a, blocks, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_complex_shape(int variant, bool akf, bool bkf, bool dnf, const GettArgs& a, int64_t blocks, hipStream_t st) {
    switch (variant) {
        case 0: return launch_flags<ComplexPolicy, 0>(akf, bkf, dnf, a, blocks, st);
        case 1: return launch_flags<ComplexPolicy, 1>(akf, bkf, dnf, a, blocks, st);
        case 2: return launch_flags<ComplexPolicy, 2>(akf, bkf, dnf, a, blocks, st);
        default: return hipErrorInvalidValue;
    }
}

const Shape* shapes_of(int dtype, int* n) {
    if (dtype == TCX_C128) { *n = kNumComplexShapes; return kComplexShapes; }
    if (dtype == TCX_F64 || dtype == TCX_F32) { *n = kNumRealShapes; return kRealShapes; }
    *n = 0;
    return nullptr;
}

}  // namespace

int gett_num_variants(int dtype) {
    int n = 0;
    shapes_of(dtype, &n);
    return n;
}

GettVariant gett_variant(int dtype, int variant) {
    int n = 0;
    const Shape* t = shapes_of(dtype, &n);
    const Shape s = t[variant];
    return {s.mt_m, s.mt_n, s.kt, s.wgm * s.wgn * 64, s.efficiency};
}

int launch_gett(int dtype, int variant, bool a_kf, bool b_kf, bool d_nf, const GettArgs& args, void* stream,
                int64_t* grid, int* block) {
    if (variant < 0 || variant >= gett_num_variants(dtype)) return (int)hipErrorInvalidValue;
    const int64_t blocks = (int64_t)args.tilesM * args.tilesN * args.sizeH;
    *grid = blocks;
    *block = gett_variant(dtype, variant).threads;
    if (blocks <= 0 || blocks > 0x7fffffff) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == TCX_F64) return (int)launch_real_shape<RealPolicy<double>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
    if (dtype == TCX_F32) return (int)launch_real_shape<RealPolicy<float>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
    if (dtype == TCX_C128) return (int)launch_complex_shape(variant, a_kf, b_kf, d_nf, args, blocks, st);
    return (int)hipErrorInvalidValue;
}

}  // namespace tcx
