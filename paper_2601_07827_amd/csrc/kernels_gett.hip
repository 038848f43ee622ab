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
//
// Three kernels share the pieces above:
//   gett_pingpong_kernel  two wave groups alternate a memory phase and a compute phase, the
//                         memory phase free of vector-ALU instructions (the fast one; needs |K|
//                         in whole slabs and slab-periodic k offsets);
//   gett_kernel           one barrier per slab in the middle of its MFMAs, register ring of
//                         global loads (every plan the first cannot take);
//   gett_direct_kernel    no LDS, no barrier (few short tiles);
// plus gett_reduce_kernel, which sums split-K parts in a fixed order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "bf16.hpp"
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
    // The fp64 MFMA reads its last immediate as sign modifiers (bit 0: first source, bit 1: second,
    // bit 2: accumulator input): c - rowop * colop without a vector-ALU instruction.
    static __device__ __forceinline__ vec mac_minus(double rowop, double colop, vec c) {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(rowop, colop, c, 0, 0, 1);
    }
    static __device__ __forceinline__ int row_of(int lane, int v) { return 4 * v + (lane >> 4); }
};
template <> struct Mfma<float> {
    using vec = float4_t;
    static __device__ __forceinline__ vec mac(float rowop, float colop, vec c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(rowop, colop, c, 0, 0, 0);
    }
    // (the fp32 MFMA has no sign modifiers: the operand is negated on the vector ALU)
    static __device__ __forceinline__ vec mac_minus(float rowop, float colop, vec c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(-rowop, colop, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row_of(int lane, int v) { return 4 * (lane >> 4) + v; }
};

// ---- arithmetic policies: what an element is, how a 16x16x4 block is accumulated, and how
// the epilogue combines alpha, beta, the accumulator and op(C) --------------------------------
// `elem` is what the kernels compute on and keep in LDS, `stor` what memory holds: the same type,
// or its 32-bit form when a plan widens 32-bit tensors to 64-bit arithmetic (elements are widened
// as they are gathered, D is rounded once on the store).
template <class R, class S = R> struct RealPolicy {
    using elem = R;
    using stor = S;
    using real = R;
    static constexpr bool is_complex = false;
    static constexpr bool two_phase = std::is_same<R, S>::value;       // the two-phase kernels move raw storage
    template <int FM, int FN> static constexpr int acc_reals() { return FM * FN * 4; }
    template <int FM, int FN, class A> static __device__ __forceinline__ void spill(const A (&acc)[FM][FN], R* dst, int pitch) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) dst[(size_t)((i * FN + j) * 4 + v) * pitch] = acc[i][j].v[v];
    }
    template <int FM, int FN, class A> static __device__ __forceinline__ void accumulate(A (&acc)[FM][FN], const R* src, int pitch) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][j].v[v] += src[(size_t)((i * FN + j) * 4 + v) * pitch];
    }
    using MF = Mfma<R>;
    using vec = typename MF::vec;
    struct acc_t {
        vec v;
    };
    static __device__ __forceinline__ void clear(acc_t& c) { c.v = vec{0, 0, 0, 0}; }
    static __device__ __forceinline__ elem zero() { return R(0); }
    static __device__ __forceinline__ elem load(const stor* p, int64_t off, unsigned) { return (R)p[off]; }
    static __device__ __forceinline__ elem load_at(const char* base, uint32_t byte_off, unsigned) {
        return (R) * (const stor*)(base + byte_off);
    }
    template <bool DNF, bool MIXED = false> static __device__ __forceinline__ void mac(elem a, elem b, acc_t& c) {
        c.v = DNF ? MF::mac(a, b, c.v)      // rows = m, lanes along n
                  : MF::mac(b, a, c.v);     // rows = n, lanes along m
    }
    static __device__ __forceinline__ stor combine(const acc_t& c, int v, const Scalars& s, bool read_c, stor cc, int, bool = false) {
        R d = (R)s.alpha_re * c.v[v];
        if (read_c) d += (R)s.beta_re * (R)cc;
        return (S)d;
    }
};

// Complex numbers as pairs of reals: four real MFMAs per complex 16x16x4 block,
//   re += ar*br - ai*bi,  im += ar*bi + ai*br.
template <class R> struct pair_of;
template <> struct pair_of<double> { using type = double2; };
template <> struct pair_of<float> { using type = float2; };

template <class R, class S = R> struct ComplexPolicyT {
    using elem = typename pair_of<R>::type;
    using stor = typename pair_of<S>::type;
    using real = R;
    static constexpr bool is_complex = true;
    static constexpr bool two_phase = std::is_same<R, double>::value && std::is_same<S, double>::value;
    template <int FM, int FN> static constexpr int acc_reals() { return FM * FN * 8; }
    template <int FM, int FN, class A> static __device__ __forceinline__ void spill(const A (&acc)[FM][FN], R* dst, int pitch) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    dst[(size_t)((i * FN + j) * 8 + v) * pitch] = acc[i][j].re[v];
                    dst[(size_t)((i * FN + j) * 8 + 4 + v) * pitch] = acc[i][j].im[v];
                }
    }
    template <int FM, int FN, class A> static __device__ __forceinline__ void accumulate(A (&acc)[FM][FN], const R* src, int pitch) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    acc[i][j].re[v] += src[(size_t)((i * FN + j) * 8 + v) * pitch];
                    acc[i][j].im[v] += src[(size_t)((i * FN + j) * 8 + 4 + v) * pitch];
                }
    }
    using MF = Mfma<R>;
    using vec = typename MF::vec;
    struct acc_t {
        vec re, im;
    };
    static __device__ __forceinline__ void clear(acc_t& c) { c.re = vec{0, 0, 0, 0}; c.im = vec{0, 0, 0, 0}; }
    static __device__ __forceinline__ elem zero() { return elem{R(0), R(0)}; }
    // Kernels that conjugate as they gather pass the sign bit to flip (0 or 0x80000000).
    static __device__ __forceinline__ elem widen(stor v, unsigned conj_mask_hi) {
        elem e{(R)v.x, (R)v.y};
        if constexpr (sizeof(R) == 8) {
            const unsigned long long bits = __builtin_bit_cast(unsigned long long, e.y) ^ ((unsigned long long)conj_mask_hi << 32);
            e.y = __builtin_bit_cast(double, bits);
        } else {
            e.y = __builtin_bit_cast(float, __builtin_bit_cast(unsigned, e.y) ^ conj_mask_hi);
        }
        return e;
    }
    static __device__ __forceinline__ elem load(const stor* p, int64_t off, unsigned conj_mask_hi) { return widen(p[off], conj_mask_hi); }
    static __device__ __forceinline__ elem load_at(const char* base, uint32_t byte_off, unsigned conj_mask_hi) {
        return widen(*(const stor*)(base + byte_off), conj_mask_hi);
    }
    // MIXED = false: the product a * b.  MIXED = true: conj(a) * b, for kernels that leave
    // conjugation out of their data path: with both operands conjugated they sum a * b, with one
    // conj(a) * b, and the epilogue conjugates the sum where the conjugated operand was B
    // (a * conj(b) = conj(conj(a) * b)).  The one minus sign of either form rides on the MFMA
    // (fp64: its sign modifier).
    template <bool DNF, bool MIXED = false> static __device__ __forceinline__ void mac(elem a, elem b, acc_t& c) {
        if (DNF) {
            c.re = MF::mac(a.x, b.x, c.re);
            c.re = MIXED ? MF::mac(a.y, b.y, c.re) : MF::mac_minus(a.y, b.y, c.re);
            c.im = MF::mac(a.x, b.y, c.im);
            c.im = MIXED ? MF::mac_minus(a.y, b.x, c.im) : MF::mac(a.y, b.x, c.im);
        } else {
            c.re = MF::mac(b.x, a.x, c.re);
            c.re = MIXED ? MF::mac(b.y, a.y, c.re) : MF::mac_minus(b.y, a.y, c.re);
            c.im = MF::mac(b.y, a.x, c.im);
            c.im = MIXED ? MF::mac_minus(b.x, a.y, c.im) : MF::mac(b.x, a.y, c.im);
        }
    }
    static __device__ __forceinline__ stor combine(const acc_t& c, int v, const Scalars& s, bool read_c, stor cs, int opC,
                                                   bool conj_acc = false) {
        const R re = c.re[v], im = conj_acc ? -c.im[v] : c.im[v];
        const R ar = (R)s.alpha_re, ai = (R)s.alpha_im;
        R dr = ar * re - ai * im;
        R di = ar * im + ai * re;
        if (read_c) {
            const R br = (R)s.beta_re, bi = (R)s.beta_im;
            const R cx = (R)cs.x, cy = opC == TCX_OP_CONJ ? -(R)cs.y : (R)cs.y;
            dr += br * cx - bi * cy;
            di += br * cy + bi * cx;
        }
        return stor{(S)dr, (S)di};
    }
};
using ComplexPolicy = ComplexPolicyT<double>;

constexpr int kPadMN = 16;   // [k][mn] rows: the four k-rows of a fragment land on distinct banks
constexpr int kPadK = 1;     // [mn][k] rows: odd row pitch spreads the 16 rows of a fragment

// One operand's slab: MT rows (m or n) by KT contracted indices.  A thread stages PER items of
// VEC elements each (VEC = 2: the kernel pairs the elements up itself and does not use row(),
// kin() and lds_index()).
template <class T, int MT, int KT, int NT, bool KF, int VEC = 1>
struct Slab {
    static constexpr int PER = MT * KT / NT / VEC;                 // items per thread per slab
    static constexpr int LD = KF ? KT + kPadK : MT + kPadMN;
    static constexpr int ELEMS = KF ? MT * LD : KT * LD;
    static_assert(MT * KT % (NT * VEC) == 0 && MT % VEC == 0 && KT % VEC == 0, "slab must divide evenly over the workgroup");
    // lanes run along the rows and a wave covers whole rows' worth: one k index per wave
    static constexpr bool UNIFORM_K = !KF && MT % 64 == 0 && (NT % MT == 0 || MT % NT == 0);

    static __device__ __forceinline__ int row(int e) { return KF ? e / KT : e % MT; }
    static __device__ __forceinline__ int kin(int e) { return KF ? e % KT : e / MT; }
    static __device__ __forceinline__ int lds_index(int e) { return KF ? row(e) * LD + kin(e) : kin(e) * LD + row(e); }
    // fragment element for (row r of the slab, k index kk of the slab)
    static __device__ __forceinline__ int frag_index(int r, int kk) { return KF ? r * LD + kk : kk * LD + r; }
};

// Keeps reads of an accumulator away from the MFMA that wrote it last.  On gfx950 a 16x16x4
// fp64 MFMA writes its result registers over 16 passes; the wait states this compiler inserts
// between such an MFMA and a following non-MFMA read of its result assume 8 (the last-written
// quarter of the accumulator was observed stale when a wave owns a single accumulator and the
// compiler moves it between register files right after the MFMA).  With several accumulators
// per wave the other MFMAs provide the distance; where a wave has only one or two, and once
// before every epilogue, 24 idle issue slots are inserted by hand.  They idle only this wave.
__device__ __forceinline__ void settle_accumulators() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// Values that are the same for every lane of a wave but were computed by vector instructions
// (divisions, table reads): moved to scalar registers, so that what is derived from them (loop
// counters, base addresses, table reads) is scalar work too.
__device__ __forceinline__ int wave_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t wave_uniform(int64_t v) {
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)(uint64_t)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Read-only plan tables indexed by a wave-uniform number: viewed through the constant address
// space their reads are scalar loads whatever else the kernel stores.
template <class T> using const_table = const __attribute__((address_space(4))) T*;
template <class T> __device__ __forceinline__ const_table<T> scalar_table(const T* p) { return (const_table<T>)(uintptr_t)p; }

// Consecutive workgroup ids go round-robin over the 8 XCDs; remap so that each XCD (private
// 4 MB L2) works on one contiguous stretch of the tile order.
__device__ __forceinline__ int64_t xcd_contiguous(int64_t id, int64_t nb) {
    const int64_t per = nb / 8;
    return id < per * 8 ? (id % 8) * per + id / 8 : id;
}

// Quotient of two non-negative numbers.  A 64-bit division costs a few hundred cycles on this
// chip (no hardware divider); tile and item numbers nearly always fit 32 bits, where it costs a
// fraction of that, and a workgroup does several before its first load can go out.
__device__ __forceinline__ int64_t quotient(int64_t a, int64_t b) {
    return ((uint64_t)(a | b) >> 32) == 0 ? (int64_t)((uint32_t)a / (uint32_t)b) : a / b;
}

struct Tile {
    int64_t m0, n0;          // first row / column of the tile in the linearised M, N index
    int64_t hA, hB, hD;      // base offsets from the hyper index
};

// Tile number -> tile coordinates.  Tiles are walked in bands of tile-rows, column by column
// inside a band, so that the 32 consecutive tiles an XCD receives form a block that shares
// operand panels through that XCD's L2: 8 rows x 4 columns of square tiles, 4 rows x 8 columns
// of tiles that are higher than wide (the block's A panels + B panels are then fewest bytes).
// The hyper index is the slowest (Eq. case2: an independent product per value of H).
template <bool FAST = false>
__device__ __forceinline__ Tile locate_tile(int64_t t_all, const GettArgs& g, int mt_m, int mt_n) {
    const int64_t tiles_per_h = (int64_t)g.tilesM * g.tilesN;
    const int64_t h = FAST ? quotient(t_all, tiles_per_h) : t_all / tiles_per_h;
    const int t = (int)(t_all - h * tiles_per_h);
    const int BAND = mt_m > mt_n ? 4 : 8;
    const int band = t / (BAND * g.tilesN);
    const int first_m = band * BAND;
    const int band_rows = min(BAND, g.tilesM - first_m);
    const int in_band = t - band * BAND * g.tilesN;
    Tile r;
    r.m0 = (int64_t)(first_m + in_band % band_rows) * mt_m;
    r.n0 = (int64_t)(in_band / band_rows) * mt_n;
    r.hA = r.hB = r.hD = 0;
    int64_t rem = h;
    for (int i = 0; i < g.nH; ++i) {
        const int64_t q = FAST ? quotient(rem, g.hExt[i]) : rem / g.hExt[i], idx = rem - q * g.hExt[i];
        rem = q;
        r.hA += idx * g.hSA[i];
        r.hB += idx * g.hSB[i];
        r.hD += idx * g.hSD[i];
    }
    return r;
}

// alpha/beta epilogue of one thread's accumulators: strided scatter through D's offset tables.
// The reads of C for a whole row of fragments are issued together before any of them is used,
// so a thread pays the memory latency FM times rather than once per element.
// Small real tiles read D's offsets before the main loop (registers are plentiful there), so
// that the epilogue starts with its stores instead of with a table read per row of fragments.
template <class P, int FM, int FN> struct DOffsets {
    int64_t off[FM][FN][4];
    bool ok[FM][FN][4];
};
template <class P, int FM, int FN, int WT_M, int WT_N, bool DNF>
__device__ __forceinline__ void d_offsets(DOffsets<P, FM, FN>& o, const GettArgs& g, const Tile& tile, int wm, int wn, int lane) {
    using MF = typename P::MF;
    const int fr = lane & 15;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int rr = MF::row_of(lane, v);
                const int ml = wm * WT_M + i * 16 + (DNF ? rr : fr);
                const int nl = wn * WT_N + j * 16 + (DNF ? fr : rr);
                o.ok[i][j][v] = tile.m0 + ml < g.sizeM && tile.n0 + nl < g.sizeN;
                o.off[i][j][v] = tile.hD + g.oDM[tile.m0 + ml] + g.oDN[tile.n0 + nl];      // padded tables: always a valid entry
            }
}
template <class P, int FM, int FN>
__device__ __forceinline__ void scatter_at(const typename P::acc_t (&acc)[FM][FN], const GettArgs& g, const DOffsets<P, FM, FN>& o) {
    using T = typename P::stor;
    const T* __restrict__ C = (const T*)g.C;
    T* __restrict__ D = (T*)g.D;
    const bool read_c = g.read_c != 0;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        T cval[FN][4];
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                cval[j][v] = T{};
                if (read_c && o.ok[i][j][v]) cval[j][v] = C[o.off[i][j][v]];
            }
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (o.ok[i][j][v]) D[o.off[i][j][v]] = P::combine(acc[i][j], v, g.s, read_c, cval[j][v], g.opC, g.conj_acc != 0);
    }
}

template <class P, int FM, int FN, int WT_M, int WT_N, bool DNF>
__device__ __forceinline__ void scatter(const typename P::acc_t (&acc)[FM][FN], const GettArgs& g, const Tile& tile,
                                        int wm, int wn, int lane) {
    using T = typename P::stor;
    using MF = typename P::MF;
    const T* __restrict__ C = (const T*)g.C + tile.hD;
    T* __restrict__ D = (T*)g.D + tile.hD;
    const int fr = lane & 15;
    const bool read_c = g.read_c != 0;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        int64_t off[FN][4];
        bool ok[FN][4];
        T cval[FN][4];
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int rr = MF::row_of(lane, v);
                const int ml = wm * WT_M + i * 16 + (DNF ? rr : fr);
                const int nl = wn * WT_N + j * 16 + (DNF ? fr : rr);
                ok[j][v] = tile.m0 + ml < g.sizeM && tile.n0 + nl < g.sizeN;
                off[j][v] = g.oDM[tile.m0 + ml] + g.oDN[tile.n0 + nl];      // padded tables: always a valid entry
                cval[j][v] = T{};
            }
        if (read_c) {
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (ok[j][v]) cval[j][v] = C[off[j][v]];
        }
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (ok[j][v]) D[off[j][v]] = P::combine(acc[i][j], v, g.s, read_c, cval[j][v], g.opC, g.conj_acc != 0);
    }
}

// DEPTH: how many slabs ahead of the MFMAs the global loads run (a ring of DEPTH register sets).
// Large tiles spend longer on a slab than a load takes and need 1; small tiles need more bytes
// in flight to cover the same latency.
template <class P, int MT_M, int MT_N, int KT, int WGM, int WGN, bool AKF, bool BKF, bool DNF, int DEPTH>
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

    // three slabs of LDS: see the main loop
    __shared__ T lds[3 * (SA::ELEMS + SB::ELEMS)];
    static_assert(sizeof(T) * 3 * (SA::ELEMS + SB::ELEMS) <= 160 * 1024, "LDS budget of a CU");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;

    // ---- which tile, and which part of K (split-K: consecutive ids are the parts of one tile)
    const int64_t lid = g.lid_base + xcd_contiguous(blockIdx.x, gridDim.x);
    const int split = wave_uniform((int)(lid % g.splitK));
    const Tile tile = locate_tile(lid / g.splitK, g, MT_M, MT_N);
    const int64_t m0 = wave_uniform(tile.m0), n0 = wave_uniform(tile.n0);
    // ---- gather addressing.  An element's address is a wave-uniform 64-bit base plus a 32-bit
    // per-lane byte offset (the plan's tile-relative tables), which the hardware adds itself: no
    // 64-bit vector arithmetic in the loop and one register per offset.
    const char* const Ab = (const char*)g.A + wave_uniform(tile.hA * (int64_t)sizeof(typename P::stor) + scalar_table(g.rbA)[m0 / MT_M]);
    const char* const Bb = (const char*)g.B + wave_uniform(tile.hB * (int64_t)sizeof(typename P::stor) + scalar_table(g.rbB)[n0 / MT_N]);
    // Row offsets are loop-invariant.  Rows past the end of M or N repeat a valid row of the
    // tile; what they accumulate is never stored.
    uint32_t rrA[SA::PER], rrB[SB::PER];
#pragma unroll
    for (int i = 0; i < SA::PER; ++i) rrA[i] = g.rrA[m0 + SA::row(tid + i * NT)];
#pragma unroll
    for (int i = 0; i < SB::PER; ++i) rrB[i] = g.rrB[n0 + SB::row(tid + i * NT)];

    // Offsets along K come from the tables one slab ahead of the data loads that use them,
    // so a data load never waits on a table load issued in the same iteration.  Where the
    // k index is the same for a whole wave its offset is a scalar that goes into the base;
    // otherwise the slab's base is the scalar and each lane adds its k's relative offset.
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
    int64_t kqA[SA::PER], kqB[SB::PER];          // uniform-k operands: scalar byte offset per element
    uint32_t krA[SA::PER], krB[SB::PER];         // others: per-lane offset relative to the slab's base
    int64_t kbA = 0, kbB = 0;
    auto k_offsets = [&](int kt) {
        const int kc = min(kt, nk - 1);
        const int64_t at = (int64_t)kc * KT;
        if (SA::UNIFORM_K) {
            const const_table<int64_t> q = scalar_table(g.kqA + at);
#pragma unroll
            for (int i = 0; i < SA::PER; ++i) kqA[i] = q[kinA[i]];
        } else {
            const uint32_t* __restrict__ t = g.krA + at;
            kbA = scalar_table(g.kbA)[kc];
#pragma unroll
            for (int i = 0; i < SA::PER; ++i) krA[i] = t[kinA[i]];
        }
        if (SB::UNIFORM_K) {
            const const_table<int64_t> q = scalar_table(g.kqB + at);
#pragma unroll
            for (int i = 0; i < SB::PER; ++i) kqB[i] = q[kinB[i]];
        } else {
            const uint32_t* __restrict__ t = g.krB + at;
            kbB = scalar_table(g.kbB)[kc];
#pragma unroll
            for (int i = 0; i < SB::PER; ++i) krB[i] = t[kinB[i]];
        }
    };

    T ra[DEPTH][SA::PER], rb[DEPTH][SB::PER];
    const unsigned conjA = g.opA == TCX_OP_CONJ ? 0x80000000u : 0u;
    const unsigned conjB = g.opB == TCX_OP_CONJ ? 0x80000000u : 0u;
    // Data loads of one slab into ring slot `slot`; its k_offsets() must have been issued
    // before.  Unconditional: the tables are padded with offsets of valid elements.
    auto gather = [&](int slot) {
#pragma unroll
        for (int i = 0; i < SA::PER; ++i) {
            if (SA::UNIFORM_K) {
                // the empty statement keeps the compiler from folding the loop-invariant row
                // offset into a 64-bit per-lane pointer (which would undo the scalar base)
                asm("" : "+v"(rrA[i]));
                ra[slot][i] = P::load_at(Ab + kqA[i], rrA[i], conjA);
            } else {
                ra[slot][i] = P::load_at(Ab + kbA, rrA[i] + krA[i], conjA);
            }
        }
#pragma unroll
        for (int i = 0; i < SB::PER; ++i) {
            if (SB::UNIFORM_K) {
                asm("" : "+v"(rrB[i]));
                rb[slot][i] = P::load_at(Bb + kqB[i], rrB[i], conjB);
            } else {
                rb[slot][i] = P::load_at(Bb + kbB, rrB[i] + krB[i], conjB);
            }
        }
    };
    // The last slab of a ragged K holds padded k entries whose (valid, arbitrary) values must
    // not be summed: zero them after the load.
    auto mask_last = [&](int slot) {
        const unsigned kleft = (unsigned)(g.sizeK - (int64_t)(nk - 1) * KT);
#pragma unroll
        for (int i = 0; i < SA::PER; ++i) ra[slot][i] = kinA[i] < kleft ? ra[slot][i] : P::zero();
#pragma unroll
        for (int i = 0; i < SB::PER; ++i) rb[slot][i] = kinB[i] < kleft ? rb[slot][i] : P::zero();
    };
    auto stage = [&](int slot, int buf) {
        T* sa = lds + buf * (SA::ELEMS + SB::ELEMS);
        T* sb = sa + SA::ELEMS;
#pragma unroll
        for (int i = 0; i < SA::PER; ++i) sa[SA::lds_index(tid + i * NT)] = ra[slot][i];
#pragma unroll
        for (int i = 0; i < SB::PER; ++i) sb[SB::lds_index(tid + i * NT)] = rb[slot][i];
    };

    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) P::clear(acc[i][j]);

    // MFMA fragments are read from LDS one k-step (4 contracted indices) ahead of the MFMAs
    // that consume them, into two register sets used alternately; the last step of a slab reads
    // the first fragments of the next slab.  A wave's MFMAs then follow each other without
    // waiting on LDS, whatever the other wave of its SIMD is doing.
    const int fr = lane & 15, fq = lane >> 4;
    constexpr int STEPS = KT / 4;
    static_assert(STEPS % 2 == 0, "fragment sets alternate per k-step and must line up across slabs");
    T fa[2][FM], fb[2][FN];
    auto frag_load = [&](int buf, int step, int set) {
        const T* sa = lds + buf * (SA::ELEMS + SB::ELEMS);
        const T* sb = sa + SA::ELEMS;
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[set][i] = sa[SA::frag_index(wm * WT_M + i * 16 + fr, step * 4 + fq)];
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[set][j] = sb[SB::frag_index(wn * WT_N + j * 16 + fr, step * 4 + fq)];
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) P::template mac<DNF>(fa[set][i], fb[set][j], acc[i][j]);
        if (FM * FN <= 2) settle_accumulators();
    };

    // ---- main loop.  Global loads run DEPTH slabs ahead in registers.  LDS holds three slabs
    // and the workgroup barrier sits in the MIDDLE of a slab's MFMAs: slab kt+1 is written to
    // LDS after the first half of slab kt and is first read (by the fragment prefetch of slab
    // kt's last step) half a slab after the barrier, so a wave that waits at the barrier does
    // so with its next fragments already in registers.  The third buffer makes that safe: the
    // buffer being written was last read two slabs ago, which every wave finished before it
    // reached the previous barrier.
    const bool ragged_k = g.sizeK % KT != 0;
    const int per_split = (nk + g.splitK - 1) / g.splitK;
    const int kb = wave_uniform(split * per_split), ke = wave_uniform(min(nk, kb + per_split));   // this workgroup's slabs [kb, ke)
    // Prologue: fill the ring with slabs kb .. kb+DEPTH-1 (slab numbers past the end are clamped
    // by k_offsets to the last slab: harmless loads that are never staged).
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        k_offsets(kb + d);
        gather(d);
    }
    k_offsets(kb + DEPTH);
    if (ragged_k && kb == nk - 1) mask_last(0);
    stage(0, 0);
    __syncthreads();
    int buf = 0;
    frag_load(0, 0, 0);
    // Steady state, unrolled by DEPTH so that ring slots are compile-time register names.  In
    // iteration kt slot u holds slab kt (already staged), so it is refilled with slab kt+DEPTH;
    // slot u+1 holds slab kt+1, issued DEPTH-1 iterations ago, and is staged for the next one.
    // `last_group` is a compile-time flag: only the final group of iterations can meet the end
    // of the range or the ragged slab, so the steady-state body is one straight path.
    auto iteration = [&](int kt, int u, auto last_group) {
        const int next = buf == 2 ? 0 : buf + 1;
        gather(u);                                       // slab kt+u+DEPTH
        k_offsets(kt + u + DEPTH + 1);
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            if (st + 1 < STEPS) frag_load(buf, st + 1, (st + 1) & 1);
            else frag_load(next, 0, 0);                  // slab kt+u+1, complete since this slab's barrier
            mfmas(st & 1);
            if (st == STEPS / 2 - 1) {
                if (decltype(last_group)::value && ragged_k && kt + u + 1 == nk - 1) mask_last((u + 1) % DEPTH);
                stage((u + 1) % DEPTH, next);            // slab kt+u+1
                __syncthreads();
            }
        }
        buf = next;
    };
    int kt = kb;
    for (; kt + DEPTH < ke - 1; kt += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) iteration(kt, u, std::false_type{});
    }
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
        if (kt + u >= ke - 1) break;
        iteration(kt, u, std::true_type{});
    }
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {                 // slab ke-1
        if (st + 1 < STEPS) frag_load(buf, st + 1, (st + 1) & 1);
        mfmas(st & 1);
    }
    settle_accumulators();

    // ---- epilogue.  With split-K the raw accumulators go to the workspace, one coalesced
    // stretch per accumulator register; the reduction kernel sums the parts in a fixed order
    // and applies alpha, beta and the scatter.
    if (g.splitK > 1) {
        typename P::real* ws = (typename P::real*)g.workspace + (size_t)lid * (NT * P::template acc_reals<FM, FN>());
        P::template spill<FM, FN>(acc, ws + tid, NT);
    } else {
        scatter<P, FM, FN, WT_M, WT_N, DNF>(acc, g, tile, wm, wn, lane);
    }
}

// ---- two-phase ("ping-pong") kernel for the large tile -----------------------------------------
// Measured on gfx950: while one wave issues MFMAs back to back, the other waves of its SIMD cannot
// issue ANY vector-ALU instruction (integer adds for addresses included); scalar instructions, LDS
// accesses and global loads of those waves proceed at full speed.  A workgroup barrier once per
// slab, on the other hand, puts all waves into the same phase: they then do their memory work at
// the same time and the matrix pipe idles meanwhile.  This kernel therefore
//  * splits the waves into two groups with one wave of each on every SIMD (wave w and w + half
//    share a SIMD).  An iteration is a MEMORY phase (copy the slab that has arrived in registers
//    to LDS, issue the global loads of the slab after it, read the first MFMA fragments) and a
//    COMPUTE phase (all MFMAs of a slab), each ended by a workgroup barrier; the second group
//    runs one phase behind the first, so one group is always streaming MFMAs while the other
//    does its memory work in that shadow;
//  * keeps the memory phase free of vector-ALU instructions: every per-lane address (global
//    offsets, LDS write and read addresses for each of the three LDS slabs) is computed once
//    before the loop; what changes per slab is scalar (base pointers from the plan's tables);
//    the loop is unrolled by three so that the LDS slab in use is a compile-time constant.
// Preconditions, checked by the host: an operand whose lanes run along k has the same relative k
// offsets in every whole slab, and an operand whose lanes run along the rows has a tile extent
// that is a multiple of 64.
// A slab's global loads have a whole iteration to arrive.  Three LDS slabs: slab i+1 is written
// in phase 2i by the first group and in phase 2i+1 by the second; the buffer it goes to held slab
// i-2, last read in phase 2i-2; it is first read in phase 2i+2.
template <class T> __device__ __forceinline__ void lds_store(unsigned byte_addr, T v) {
    *(__attribute__((address_space(3))) T*)(uintptr_t)byte_addr = v;
}
template <class T> __device__ __forceinline__ T lds_load(unsigned byte_addr) {
    return *(const __attribute__((address_space(3))) T*)(uintptr_t)byte_addr;
}
// complex elements travel as a plain 16-byte vector (one ds_write_b128 / ds_read_b128)
typedef double plain_double2 __attribute__((ext_vector_type(2)));
template <> __device__ __forceinline__ void lds_store<double2>(unsigned byte_addr, double2 v) {
    *(__attribute__((address_space(3))) plain_double2*)(uintptr_t)byte_addr = plain_double2{v.x, v.y};
}
template <> __device__ __forceinline__ double2 lds_load<double2>(unsigned byte_addr) {
    const plain_double2 t = *(const __attribute__((address_space(3))) plain_double2*)(uintptr_t)byte_addr;
    return double2{t.x, t.y};
}

// what one gather load brings: an element, or two neighbouring real elements
template <class T, int VEC> struct staged_item { using type = T; };
template <> struct staged_item<double, 2> { using type = plain_double2; };
template <> struct staged_item<float, 2> { typedef float type __attribute__((ext_vector_type(2))); };

// DUAL: each of the two wave groups owns a tile of its own (WGM x WGN waves per tile, twice that
// per workgroup) and stages only its own operands; the groups meet at the phase barriers alone.
// This brings the schedule to small tiles: a workgroup of eight waves works on two 64 x 64 or
// 96 x 96 tiles.  Two LDS slabs per group are enough then (a group writes slab i+1 one phase
// after it last read the buffer).  A workgroup's two items may have different numbers of slabs
// (split K) or the second may not exist (odd count): both groups run the phase barriers of the
// longer one.
// One predicate, used by the kernel, its launcher and the planner alike: the partial sums of a
// tile (one group's accumulators) fit into the LDS slabs of a dual workgroup.  The slabs' pitch
// padding is left out, so it can only err towards "does not fit".
constexpr bool pair_fits_lds(size_t elem_bytes, size_t real_bytes, int planes, int mt_m, int mt_n, int kt) {
    return real_bytes * planes * mt_m * mt_n <= elem_bytes * 4 * (size_t)(mt_m + mt_n) * kt;
}

template <int MT, int NTG, bool KF> constexpr bool pingpong_operand_ok() {
    // lanes along k, or lanes along the rows with one k per wave and rows that repeat per thread
    return KF || (MT % 64 == 0 && NTG % MT == 0);
}

template <int I, int N, class F> __device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// DEPTH: slabs of global loads in flight in registers.  The large tile spends 3.6 us on a slab and
// needs one; an iteration of the small tiles is shorter than a load takes.
// LATE (small tiles, DEPTH >= 2): a slab's global loads are issued in the compute phase, between
// the MFMAs, instead of in the memory phase.  A CU's address unit takes about 16 cycles per
// gather load of 64 addresses; for a 64 x 64 x 16 tile that made the memory phase longer than
// the compute phase (about 1300 against 1000 cycles).  Loads need no vector-ALU slot, and the
// matrix pipe works off the MFMAs already issued while the wave waits for the address unit.
// RAGGED: |K| is not a multiple of KT.  A separate instantiation, so that the steady state of
// the common case carries none of it: the last slab's lanes along k take their offsets from the
// table (padded entries address a valid element) instead of the slab-periodic ones, and what the
// padded entries load is zeroed before it goes to LDS -- vector-ALU work in a memory phase, once
// per tile.
// VEC = 2 (8-byte elements, whole tiles and slabs only): a gather load brings two elements that
// are neighbours in memory.  Along the direction its lanes run (k if the operand is K-fastest,
// else the tile's rows) element x is paired with x + ps, where ps (GettArgs::psA / psB, a power
// of two) is the step at which the host found every such pair contiguous and 16-byte aligned:
// 1 if the operand's fastest mode comes first in the tile, more if other modes of the tile lie
// in between.  The two halves go to LDS with one write each.  The address unit of a CU takes a
// gather load of 64 different addresses in about 16 cycles whatever its width, so on small
// tiles, whose memory phase is as long as the compute phase, the number of load instructions is
// what counts.  Both operands take the slab-periodic form of the k offsets (one scalar base per
// slab), whichever way their lanes run.
template <class P, int MT_M, int MT_N, int KT, int WGM, int WGN, bool AKF, bool BKF, bool DNF, bool DUAL, int DEPTH, bool RAGGED, bool LATE = false, int VEC = 1, bool MIXED = false>
__global__ __launch_bounds__(WGM* WGN * 64 * (DUAL ? 2 : 1)) void gett_pingpong_kernel(GettArgs g) {
    using T = typename P::elem;
    using V = typename staged_item<T, VEC>::type;
    using acc_t = typename P::acc_t;
    constexpr bool PAIR = VEC > 1;
    constexpr bool ALANES_K = AKF || PAIR, BLANES_K = BKF || PAIR;      // per-lane k offsets, one scalar base per slab
    static_assert(P::two_phase, "this kernel moves raw storage and (complex) uses the fp64 MFMA's sign modifier");
    static_assert(!(PAIR && RAGGED), "paired loads need whole slabs");
    static_assert(!LATE || DEPTH >= 2, "loads issued in a compute phase need a phase more to arrive");
    constexpr int NTG = WGM * WGN * 64;                   // threads that work on one tile
    constexpr int GROUPS_PER_TILE = DUAL ? 1 : 2;
    constexpr int NB = DUAL ? 2 : 3;                      // LDS slabs per tile
    constexpr int WT_M = MT_M / WGM, WT_N = MT_N / WGN;
    constexpr int FM = WT_M / 16, FN = WT_N / 16;
    using SA = Slab<T, MT_M, KT, NTG, AKF, VEC>;
    using SB = Slab<T, MT_N, KT, NTG, BKF, VEC>;
    constexpr int STEPS = KT / 4;
    constexpr int SLAB = SA::ELEMS + SB::ELEMS;
    constexpr unsigned ES = sizeof(T);
    static_assert(KT % 8 == 0 && WT_M % 16 == 0 && WT_N % 16 == 0, "tile shape");
    static_assert((NTG / 64 * (DUAL ? 2 : 1)) % 8 == 0, "two groups with a wave on each of the four SIMDs");
    static_assert(NTG % KT == 0, "a thread's slab elements differ by a constant LDS offset");
    static_assert(PAIR || (pingpong_operand_ok<MT_M, NTG, AKF>() && pingpong_operand_ok<MT_N, NTG, BKF>()), "operand orientation");
    static_assert(!PAIR || ((AKF || NTG % (MT_M / VEC) == 0) && (BKF || NTG % (MT_N / VEC) == 0)), "a thread's items differ by a constant LDS offset");
    static_assert(ES * SLAB < 65536, "LDS offsets inside a slab must fit the instruction's immediate");

    __shared__ __attribute__((aligned(16))) T lds[(DUAL ? 2 : 1) * NB * SLAB];
    static_assert(sizeof(T) * (DUAL ? 2 : 1) * NB * SLAB <= 160 * 1024, "LDS budget of a CU");

    const int wave_all = wave_uniform((int)threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const bool second_group = wave_all >= NTG / 64 * (DUAL ? 2 : 1) / 2;
    const int tid = DUAL ? (int)threadIdx.x % NTG : (int)threadIdx.x;      // thread number inside the tile's group(s)
    const int wave = DUAL ? wave_all % (NTG / 64) : wave_all;
    const int wm = wave % WGM, wn = wave / WGM;

    // ---- which item (tile, part of K) this group works on, and how many slabs both items have
    const int64_t items = (int64_t)g.tilesM * g.tilesN * g.sizeH * g.splitK;
    const int64_t wg = g.lid_base + xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t lid = DUAL ? 2 * wg + (second_group ? 1 : 0) : wg;
    const int nk = g.tilesK;
    const int per_split = (nk + g.splitK - 1) / g.splitK;
    auto slabs_of = [&](int64_t item, int* first) __attribute__((always_inline)) {
        if (item >= items) { *first = 0; return 0; }
        const int sp = DUAL ? (int)(item - quotient(item, g.splitK) * g.splitK) : (int)(item % g.splitK);
        *first = sp * per_split;
        return max(0, min(nk, *first + per_split) - *first);
    };
    int kb = 0, kb_other = 0;
    const int n = wave_uniform(slabs_of(lid, &kb));
    const int n_all = DUAL ? wave_uniform(max(n, slabs_of(lid ^ 1, &kb_other))) : n;
    kb = wave_uniform(kb);
    // (the short divisions only in the small-tile instantiations, whose prologue matters; the
    // large tile's steady state is sensitive to any change of its code and keeps what it had)
    const Tile tile = DUAL ? locate_tile<true>(quotient(min(lid, items - 1), g.splitK), g, MT_M, MT_N)
                           : locate_tile(min(lid, items - 1) / g.splitK, g, MT_M, MT_N);
    const int64_t m0 = wave_uniform(tile.m0), n0 = wave_uniform(tile.n0);
    const char* const Ab = (const char*)g.A + wave_uniform(tile.hA * (int64_t)sizeof(T) + scalar_table(g.rbA)[m0 / MT_M]);
    const char* const Bb = (const char*)g.B + wave_uniform(tile.hB * (int64_t)sizeof(T) + scalar_table(g.rbB)[n0 / MT_N]);

    // ---- everything per-lane, once.  Global byte offsets of this thread's slab elements
    // relative to the slab's scalar base: the row part, plus (lanes along k) the k part, which
    // the host guarantees to be the same in every slab.
    uint32_t voA[SA::PER], voB[SB::PER];
    unsigned kinA[SA::PER], kinB[SB::PER];
    // (row, k) of item e of a slab; paired items: x-th pair along the lanes -> its first element
    const int psA = PAIR ? g.psA : 1, psB = PAIR ? g.psB : 1;
    auto first_of_pair = [](int x, int ps) __attribute__((always_inline)) { return x % ps + 2 * ps * (x / ps); };
    auto rowA_of = [&](int e) __attribute__((always_inline)) { return !PAIR ? SA::row(e) : AKF ? e / (KT / 2) : first_of_pair(e % (MT_M / 2), psA); };
    auto kinA_of = [&](int e) __attribute__((always_inline)) { return !PAIR ? SA::kin(e) : AKF ? first_of_pair(e % (KT / 2), psA) : e / (MT_M / 2); };
    auto rowB_of = [&](int e) __attribute__((always_inline)) { return !PAIR ? SB::row(e) : BKF ? e / (KT / 2) : first_of_pair(e % (MT_N / 2), psB); };
    auto kinB_of = [&](int e) __attribute__((always_inline)) { return !PAIR ? SB::kin(e) : BKF ? first_of_pair(e % (KT / 2), psB) : e / (MT_N / 2); };
#pragma unroll
    for (int i = 0; i < SA::PER; ++i) {
        const int e = tid + i * NTG;
        voA[i] = g.rrA[m0 + rowA_of(e)] + (ALANES_K ? g.krA[kinA_of(e)] : 0u);
        kinA[i] = ALANES_K ? 0u : (unsigned)__builtin_amdgcn_readfirstlane(SA::kin(e));
    }
#pragma unroll
    for (int i = 0; i < SB::PER; ++i) {
        const int e = tid + i * NTG;
        voB[i] = g.rrB[n0 + rowB_of(e)] + (BLANES_K ? g.krB[kinB_of(e)] : 0u);
        kinB[i] = BLANES_K ? 0u : (unsigned)__builtin_amdgcn_readfirstlane(SB::kin(e));
    }
    // small real tiles: D's offsets too, in the same round trip to the tables
    constexpr bool D_AHEAD = DUAL && sizeof(T) <= 8 && FM * FN <= 8;
    DOffsets<P, D_AHEAD ? FM : 1, D_AHEAD ? FN : 1> d_at;
    if constexpr (D_AHEAD) d_offsets<P, FM, FN, WT_M, WT_N, DNF>(d_at, g, tile, wm, wn, lane);
    // LDS byte addresses, per LDS slab: where this thread writes its first element of A and of
    // B, and where it reads its first fragment of A and of B.  Further elements / fragments are
    // at compile-time offsets from these.
    const int fr = lane & 15, fq = lane >> 4;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) T*)lds +
                          (DUAL && second_group ? ES * NB * SLAB : 0u);
    unsigned wA[NB], wB[NB], fA[NB], fB[NB];
    unsigned wA2[NB], wB2[NB];                            // paired items: where the second element goes
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        wA[b] = lds0 + ES * (unsigned)(b * SLAB + SA::frag_index(rowA_of(tid), kinA_of(tid)));
        wB[b] = lds0 + ES * (unsigned)(b * SLAB + SA::ELEMS + SB::frag_index(rowB_of(tid), kinB_of(tid)));
        wA2[b] = wA[b] + ES * (unsigned)psA;
        wB2[b] = wB[b] + ES * (unsigned)psB;
        if constexpr (PAIR) asm volatile("" : "+v"(wA2[b]), "+v"(wB2[b]));
        fA[b] = lds0 + ES * (unsigned)(b * SLAB + SA::frag_index(wm * WT_M + fr, fq));
        fB[b] = lds0 + ES * (unsigned)(b * SLAB + SA::ELEMS + SB::frag_index(wn * WT_N + fr, fq));
        // opaque to the compiler from here on: kept in registers instead of being recomputed
        // (with vector-ALU instructions) inside the loop
        asm volatile("" : "+v"(wA[b]), "+v"(wB[b]), "+v"(fA[b]), "+v"(fB[b]));
    }
    constexpr unsigned dWA = ES * (AKF ? (NTG * VEC / KT) * SA::LD : (NTG * VEC / MT_M) * SA::LD);   // item i+1 minus item i
    constexpr unsigned dWB = ES * (BKF ? (NTG * VEC / KT) * SB::LD : (NTG * VEC / MT_N) * SB::LD);
    constexpr unsigned dFA_row = ES * (AKF ? 16 * SA::LD : 16), dFA_step = ES * (AKF ? 4 : 4 * SA::LD);
    constexpr unsigned dFB_row = ES * (BKF ? 16 * SB::LD : 16), dFB_step = ES * (BKF ? 4 : 4 * SB::LD);

    // ---- per slab, scalar: the base of each load
    int64_t kqA[SA::PER], kqB[SB::PER];          // lanes along the rows: one byte offset per element's k
    int64_t kbA = 0, kbB = 0;                    // lanes along k: the slab's base
    auto k_offsets = [&](int kt) __attribute__((always_inline)) {
        const int kc = min(kt, nk - 1);
        if (ALANES_K) {
            kbA = scalar_table(g.kbA)[kc];
        } else {
            const const_table<int64_t> q = scalar_table(g.kqA + (int64_t)kc * KT);
#pragma unroll
            for (int i = 0; i < SA::PER; ++i) kqA[i] = q[kinA[i]];
        }
        if (BLANES_K) {
            kbB = scalar_table(g.kbB)[kc];
        } else {
            const const_table<int64_t> q = scalar_table(g.kqB + (int64_t)kc * KT);
#pragma unroll
            for (int i = 0; i < SB::PER; ++i) kqB[i] = q[kinB[i]];
        }
    };
    // conjugation is applied to the MFMA fragments in the compute phase (a vector-ALU operation)
    V ra[DEPTH][SA::PER], rb[DEPTH][SB::PER];     // slab kb+j waits in ring slot j % DEPTH
    const unsigned kleft = (unsigned)(g.sizeK - (int64_t)(nk - 1) * KT);          // valid indices of the last slab
    // `part` of `parts`: the loads are issued in portions (item i belongs to portion i % parts)
    auto gather = [&](auto SLOT, int slab, int part, int parts) __attribute__((always_inline)) {
        constexpr int sl = decltype(SLOT)::value;
        if constexpr (RAGGED) {
            if (slab >= nk - 1) {
                // the ragged slab (or a clamped slab past the end): offsets of lanes along k from the table
#pragma unroll
                for (int i = 0; i < SA::PER; ++i) {
                    if (i % parts != part) continue;
                    uint32_t vo = voA[i];
                    if (AKF) vo += g.krA[(int64_t)(nk - 1) * KT + SA::kin(tid + i * NTG)] - g.krA[SA::kin(tid + i * NTG)];
                    ra[sl][i] = P::load_at(Ab + (AKF ? kbA : kqA[i]), vo, 0u);
                }
#pragma unroll
                for (int i = 0; i < SB::PER; ++i) {
                    if (i % parts != part) continue;
                    uint32_t vo = voB[i];
                    if (BKF) vo += g.krB[(int64_t)(nk - 1) * KT + SB::kin(tid + i * NTG)] - g.krB[SB::kin(tid + i * NTG)];
                    rb[sl][i] = P::load_at(Bb + (BKF ? kbB : kqB[i]), vo, 0u);
                }
                return;
            }
        }
        // steady state: no vector-ALU instruction
#pragma unroll
        for (int i = 0; i < SA::PER; ++i) {
            if (i % parts != part) continue;
            asm("" : "+v"(voA[i]));              // keeps "scalar base + 32-bit lane offset" from being folded into a 64-bit lane address
            if constexpr (PAIR) ra[sl][i] = *(const V*)(Ab + kbA + voA[i]);
            else ra[sl][i] = P::load_at(Ab + (AKF ? kbA : kqA[i]), voA[i], 0u);
        }
#pragma unroll
        for (int i = 0; i < SB::PER; ++i) {
            if (i % parts != part) continue;
            asm("" : "+v"(voB[i]));
            if constexpr (PAIR) rb[sl][i] = *(const V*)(Bb + kbB + voB[i]);
            else rb[sl][i] = P::load_at(Bb + (BKF ? kbB : kqB[i]), voB[i], 0u);
        }
    };
    auto stage = [&](auto BUF, auto SLOT, int slab) __attribute__((always_inline)) {
        constexpr int b = decltype(BUF)::value, sl = decltype(SLOT)::value;
        if constexpr (RAGGED) {
            if (slab == nk - 1) {
#pragma unroll
                for (int i = 0; i < SA::PER; ++i)
                    if ((unsigned)SA::kin(tid + i * NTG) >= kleft) ra[sl][i] = P::zero();
#pragma unroll
                for (int i = 0; i < SB::PER; ++i)
                    if ((unsigned)SB::kin(tid + i * NTG) >= kleft) rb[sl][i] = P::zero();
            }
        }
#pragma unroll
        for (int i = 0; i < SA::PER; ++i) {
            if constexpr (PAIR) {
                lds_store<T>(wA[b] + i * dWA, ra[sl][i].x);
                lds_store<T>(wA2[b] + i * dWA, ra[sl][i].y);
            } else {
                lds_store<T>(wA[b] + i * dWA, ra[sl][i]);
            }
        }
#pragma unroll
        for (int i = 0; i < SB::PER; ++i) {
            if constexpr (PAIR) {
                lds_store<T>(wB[b] + i * dWB, rb[sl][i].x);
                lds_store<T>(wB2[b] + i * dWB, rb[sl][i].y);
            } else {
                lds_store<T>(wB[b] + i * dWB, rb[sl][i]);
            }
        }
    };

    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) P::clear(acc[i][j]);
    T fa[2][FM], fb[2][FN];
    auto frag_load = [&](auto BUF, int step, int set) __attribute__((always_inline)) {
        constexpr int b = decltype(BUF)::value;
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[set][i] = lds_load<T>(fA[b] + i * dFA_row + step * dFA_step);
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[set][j] = lds_load<T>(fB[b] + j * dFB_row + step * dFB_step);
    };
    // Conjugation never touches the data here: with exactly one operand conjugated (MIXED) the
    // blocks sum conj(a) * b (one sign moves inside the complex product, on the MFMA's own sign
    // modifier), and the launcher asks the epilogue to conjugate the sum if that operand was B.
    auto mfmas = [&](int set) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) P::template mac<DNF, MIXED>(fa[set][i], fb[set][j], acc[i][j]);
    };

    // Prologue: slab kb to LDS, slabs kb+1 .. kb+DEPTH into the ring (slab numbers past the end
    // are clamped: harmless loads that are never staged).  With a ring of two or more the second
    // slab's loads go out before the wait for the first (its slot is free), so that the first
    // iteration does not meet a second load latency.
    if (n > 0) {
        constexpr int EARLY = DEPTH >= 2 ? 1 : 0;
        k_offsets(kb);
        gather(std::integral_constant<int, 0>{}, kb, 0, 1);
        k_offsets(kb + 1);
        if constexpr (EARLY) {
            gather(std::integral_constant<int, 1 % DEPTH>{}, kb + 1, 0, 1);
            k_offsets(kb + 2);
        }
        stage(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, kb);
        static_for<EARLY, DEPTH>([&](auto D) __attribute__((always_inline)) {
            gather(std::integral_constant<int, (1 + decltype(D)::value) % DEPTH>{}, kb + 1 + decltype(D)::value, 0, 1);
            k_offsets(kb + 2 + decltype(D)::value);
        });
    }
    __syncthreads();
    if (second_group) __builtin_amdgcn_s_barrier();       // one phase behind the first group

    // A phase ends with the workgroup barrier; the compiler may move nothing across it (MFMAs
    // only touch registers, so the barrier alone would not hold them in their phase).
    auto phase_end = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    };
    // The loop is unrolled so that the LDS slab and the ring slot are compile-time constants:
    // iteration i has IDX = i % UNROLL.
    constexpr int UNROLL = NB * DEPTH / (NB % DEPTH == 0 ? DEPTH : DEPTH % NB == 0 ? NB : 1);
    static_assert(UNROLL % NB == 0 && UNROLL % DEPTH == 0, "unroll factor");
    // FULL: the caller guarantees i + 1 < n, and the round has no branch.  (With the loads under
    // a condition the compiler cannot count how many younger loads are in flight when a slab is
    // staged, and waits for all of them.)
    auto round = [&](int i, auto IDX, auto FULL) __attribute__((always_inline)) {
        constexpr bool full = decltype(FULL)::value;
        using BUF = std::integral_constant<int, decltype(IDX)::value % NB>;
        using NEXT_BUF = std::integral_constant<int, (decltype(IDX)::value + 1) % NB>;
        using NEXT_SLOT = std::integral_constant<int, (decltype(IDX)::value + 1) % DEPTH>;
        // memory phase: no vector-ALU instruction in here
        if (full || i + 1 < n) {
            if constexpr (LATE) {
                k_offsets(kb + i + 1 + DEPTH);           // for the loads of the coming compute phase
                stage(NEXT_BUF{}, NEXT_SLOT{}, kb + i + 1);
            } else {
                stage(NEXT_BUF{}, NEXT_SLOT{}, kb + i + 1);
                gather(NEXT_SLOT{}, kb + i + 1 + DEPTH, 0, 1);
                k_offsets(kb + i + 2 + DEPTH);
            }
        }
        if (full || i < n) frag_load(BUF{}, 0, 0);
        phase_end();
        // compute phase
        if (full || i < n) {
#pragma unroll
            for (int st = 0; st < STEPS; ++st) {
                if (st + 1 < STEPS) frag_load(BUF{}, st + 1, (st + 1) & 1);
                mfmas(st & 1);
                // LATE: the slab's loads go out a few per k-step behind MFMAs that keep the matrix
                // pipe busy while the address unit takes them
                if constexpr (LATE) {
                    // pinned behind this step's MFMAs: hoisted to the start of the phase the loads
                    // would hold up the first MFMA for as long as the address unit takes them
                    __builtin_amdgcn_sched_barrier(0);
                    if (full || i + 1 < n) gather(NEXT_SLOT{}, kb + i + 1 + DEPTH, st, STEPS);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        phase_end();
    };
    int i = 0;
    if constexpr (LATE)
        for (; i + UNROLL < n; i += UNROLL)
            static_for<0, UNROLL>([&](auto IDX) __attribute__((always_inline)) { round(i + decltype(IDX)::value, IDX, std::true_type{}); });
    for (; i + UNROLL <= n_all; i += UNROLL)
        static_for<0, UNROLL>([&](auto IDX) __attribute__((always_inline)) { round(i + decltype(IDX)::value, IDX, std::false_type{}); });
    static_for<0, UNROLL - 1>([&](auto IDX) __attribute__((always_inline)) {
        if (i + decltype(IDX)::value < n_all) round(i + decltype(IDX)::value, IDX, std::false_type{});
    });
    if (!second_group) __builtin_amdgcn_s_barrier();      // pairs with the second group's last barrier
    settle_accumulators();

    // ---- epilogue.  K in two parts with one tile per group: the two items of a workgroup are
    // the two parts of ONE tile, and the partial sums meet in LDS (first group's + second
    // group's, a fixed order) instead of going through the workspace and a second kernel.
    constexpr bool PAIR_FITS = DUAL && pair_fits_lds(sizeof(T), sizeof(typename P::real), sizeof(T) / sizeof(typename P::real), MT_M, MT_N, KT);
    static_assert(!PAIR_FITS || sizeof(typename P::real) * NTG * P::template acc_reals<FM, FN>() <= sizeof(T) * 2 * NB * SLAB, "partial sums must fit the slabs");
    if (PAIR_FITS && g.splitK == 2) {
        typename P::real* part = (typename P::real*)lds;
        __syncthreads();                                  // every wave has left the main loop: the slabs are free
        if (second_group) P::template spill<FM, FN>(acc, part + tid, NTG);
        __syncthreads();
        if (!second_group) {
            P::template accumulate<FM, FN>(acc, part + tid, NTG);
            if constexpr (D_AHEAD) scatter_at<P, FM, FN>(acc, g, d_at);
            else scatter<P, FM, FN, WT_M, WT_N, DNF>(acc, g, tile, wm, wn, lane);
        }
        return;
    }
    if (n == 0) return;                                   // a second group without an item
    if (g.splitK > 1) {
        typename P::real* ws = (typename P::real*)g.workspace + (size_t)lid * (NTG * P::template acc_reals<FM, FN>());
        P::template spill<FM, FN>(acc, ws + tid, NTG);
    } else {
        if constexpr (D_AHEAD) scatter_at<P, FM, FN>(acc, g, d_at);
        else scatter<P, FM, FN, WT_M, WT_N, DNF>(acc, g, tile, wm, wn, lane);
    }
}

// Second kernel of a split-K product: one workgroup per tile, same thread-to-element mapping as
// the main kernel.  Parts are summed in the order 0, 1, ..., splitK-1, so the result does not
// depend on scheduling.
template <class P, int MT_M, int MT_N, int WGM, int WGN, bool DNF>
__global__ __launch_bounds__(WGM* WGN * 64) void gett_reduce_kernel(GettArgs g) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int WT_M = MT_M / WGM, WT_N = MT_N / WGN;
    constexpr int FM = WT_M / 16, FN = WT_N / 16;
    using acc_t = typename P::acc_t;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    const int64_t t_all = blockIdx.x;
    const Tile tile = locate_tile(t_all, g, MT_M, MT_N);
    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) P::clear(acc[i][j]);
    constexpr size_t PART = (size_t)NT * P::template acc_reals<FM, FN>();
    const typename P::real* ws = (const typename P::real*)g.workspace + (size_t)t_all * g.splitK * PART + tid;
    for (int sp = 0; sp < g.splitK; ++sp) P::template accumulate<FM, FN>(acc, ws + (size_t)sp * PART, NT);
    scatter<P, FM, FN, WT_M, WT_N, DNF>(acc, g, tile, wm, wn, lane);
}

// ---- direct kernel for small tiles --------------------------------------------------------------
// When a product has few tiles the LDS pipeline above spends most of its time in barriers and
// in the latency between a slab's global loads and its use.  This kernel has no LDS and no
// barrier: every wave loads its own MFMA fragments from the strided tensors straight into
// registers -- lane (row = lane % 16, q = lane / 16) of a 16x16x4 block holds one element of a
// row of the tile, which is exactly one gathered load -- two chunks of K ahead of the MFMAs
// that consume them.  Waves that share rows of A or columns of B re-read them through the L1.
// Inside a chunk of 4*CH contracted indices lane group q owns the CH consecutive indices
// q*CH .. q*CH+CH-1 (the order in which a contraction index is summed is free as long as both
// operands agree), so an operand whose fastest mode is contracted is read in short runs.
template <class P, int FM, int FN, int CH, bool DNF>
__global__ __launch_bounds__(256) void gett_direct_kernel(GettArgs g) {
    using T = typename P::elem;
    using acc_t = typename P::acc_t;
    constexpr int WGM = 2, WGN = 2, NT = 256;
    constexpr int WT_M = FM * 16, WT_N = FN * 16, MT_M = WGM * WT_M, MT_N = WGN * WT_N;
    constexpr int KC = 4 * CH;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;
    const int fr = lane & 15, fq = lane >> 4;

    const int64_t lid = g.lid_base + xcd_contiguous(blockIdx.x, gridDim.x);
    const int split = (int)(lid % g.splitK);
    const Tile tile = locate_tile(lid / g.splitK, g, MT_M, MT_N);
    const typename P::stor* __restrict__ A = (const typename P::stor*)g.A + tile.hA;
    const typename P::stor* __restrict__ B = (const typename P::stor*)g.B + tile.hB;
    const unsigned conjA = g.opA == TCX_OP_CONJ ? 0x80000000u : 0u;
    const unsigned conjB = g.opB == TCX_OP_CONJ ? 0x80000000u : 0u;

    int64_t rowA[FM], rowB[FN];
#pragma unroll
    for (int i = 0; i < FM; ++i) rowA[i] = g.oAM[tile.m0 + wm * WT_M + i * 16 + fr];
#pragma unroll
    for (int j = 0; j < FN; ++j) rowB[j] = g.oBN[tile.n0 + wn * WT_N + j * 16 + fr];

    const int nk = g.tilesK;                                   // chunks of KC contracted indices
    const int per_split = (nk + g.splitK - 1) / g.splitK;
    const int kb = split * per_split, ke = min(nk, kb + per_split);
    const bool ragged_k = g.sizeK % KC != 0;

    int64_t ka[2][CH], kbo[2][CH];       // K offsets of this lane's indices, two chunks
    T da[2][CH][FM], db[2][CH][FN];      // fragments, two chunks
    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) P::clear(acc[i][j]);

    auto koffs = [&](int buf, int c) {
        const int64_t base = (int64_t)min(c, nk - 1) * KC + fq * CH;
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            ka[buf][j] = g.oAK[base + j];
            kbo[buf][j] = g.oBK[base + j];
        }
    };
    auto loads = [&](int buf) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
#pragma unroll
            for (int i = 0; i < FM; ++i) da[buf][j][i] = P::load(A, rowA[i] + ka[buf][j], conjA);
#pragma unroll
            for (int i = 0; i < FN; ++i) db[buf][j][i] = P::load(B, rowB[i] + kbo[buf][j], conjB);
        }
    };
    auto mask = [&](int buf, int c) {          // last chunk of a ragged K: padded indices must add nothing
#pragma unroll
        for (int j = 0; j < CH; ++j)
            if ((int64_t)c * KC + fq * CH + j >= g.sizeK) {
#pragma unroll
                for (int i = 0; i < FM; ++i) da[buf][j][i] = P::zero();
#pragma unroll
                for (int i = 0; i < FN; ++i) db[buf][j][i] = P::zero();
            }
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int j = 0; j < CH; ++j)
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int jn = 0; jn < FN; ++jn) P::template mac<DNF>(da[buf][j][i], db[buf][j][jn], acc[i][jn]);
        if (FM * FN <= 2) settle_accumulators();
    };

    // register pipeline: fragments of chunk c+1 and K offsets of chunk c+2 are in flight while
    // the MFMAs of chunk c run; the loop is unrolled by two so that buffer indices are static
    koffs(0, kb);
    koffs(1, kb + 1);
    loads(0);
    if (ragged_k && kb == nk - 1) mask(0, kb);
    int c = kb;
    while (true) {
        if (c + 1 < ke) {
            loads(1);
            koffs(0, c + 2);
            if (ragged_k && c + 1 == nk - 1) mask(1, c + 1);
        }
        mfmas(0);
        if (++c >= ke) break;
        if (c + 1 < ke) {
            loads(0);
            koffs(1, c + 2);
            if (ragged_k && c + 1 == nk - 1) mask(0, c + 1);
        }
        mfmas(1);
        if (++c >= ke) break;
    }
    settle_accumulators();

    if (g.splitK > 1) {
        typename P::real* ws = (typename P::real*)g.workspace + (size_t)lid * (NT * P::template acc_reals<FM, FN>());
        P::template spill<FM, FN>(acc, ws + tid, NT);
    } else {
        scatter<P, FM, FN, WT_M, WT_N, DNF>(acc, g, tile, wm, wn, lane);
    }
}

// ---- batch-lane kernel: batched products whose batch mode is the fastest mode of A, B and D ------
// When consecutive memory holds consecutive BATCHES (D[h, i, j] with h fastest), an operand row of
// one batch is one element out of every 128-byte line, and a tile of D for one batch writes one
// element per line.  This kernel turns the tile around: a wave group of four waves owns FOUR
// consecutive batches x MT_M x MT_N, wave w computing batch w of them.  Global loads run with four
// neighbouring lanes on the four batches of a row (64 contiguous bytes of 16-byte elements; the
// other half of the line belongs to the workgroup's other group, one phase later), LDS keeps one
// region per batch in [row][k] order, and each wave reads its MFMA fragments from its own region:
// LDS is the transposition between "lanes along the batches" (memory) and "one batch per wave"
// (MFMA).  The epilogue goes back the same way: accumulators of a 16 x 16 block to LDS per batch,
// read back with lanes along the batches, so C is read and D written in 64-byte pieces.
// The schedule is the two-phase one of gett_pingpong_kernel with one tile per group: memory phase
// (registers -> LDS, next global loads, fragment reads: no vector-ALU instruction) and compute
// phase (MFMAs only: conjugation rides on the MFMA sign modifier), the groups one phase apart.
// Preconditions (host): the fastest hyper mode has stride 1 in A, B and D and an extent that is a
// multiple of 4; |K| is a multiple of KT; the relative k offsets repeat from slab to slab; K unsplit.
constexpr int kBatchLanes = 4;

template <class P, int MT_M, int MT_N, int KT, bool DNF, int DEPTH, bool MIXED>
__global__ __launch_bounds__(512) void gett_hlane_kernel(GettArgs g) {
    using T = typename P::elem;
    using acc_t = typename P::acc_t;
    constexpr int HL = kBatchLanes, NTG = 256, NB = 2;
    constexpr int FM = MT_M / 16, FN = MT_N / 16;
    constexpr int QT = NTG / HL;                          // threads of a group per batch
    constexpr int PER_A = MT_M * KT / QT, PER_B = MT_N * KT / QT;
    constexpr int LD = KT + kPadK;                        // [row][k] pitch
    constexpr int REGION = (MT_M + MT_N) * LD + 4;        // elements of one batch's slab; + 64 bytes so the four
                                                          // batches of a row land in different banks
    constexpr int SLAB = HL * REGION;
    constexpr unsigned ES = sizeof(T);
    static_assert(sizeof(T) == 16 && P::two_phase, "four batches of 16-byte elements make a 64-byte piece");
    static_assert(KT == 4, "one MFMA k-step per slab");
    static_assert(MT_M % 16 == 0 && MT_N % 16 == 0 && (MT_M * KT) % QT == 0 && (MT_N * KT) % QT == 0 && QT % KT == 0, "tile shape");
    static_assert(NB % DEPTH == 0 || DEPTH % NB == 0, "ring and LDS slabs cycle together");
    constexpr int EPI = HL * (256 + 4);                   // epilogue: a 16 x 16 block per batch, regions 64 bytes apart in the banks
    static_assert(2 * EPI <= NB * SLAB, "the epilogue's exchange buffers live in the slabs");

    __shared__ __attribute__((aligned(16))) T lds[2 * NB * SLAB];
    static_assert(sizeof(T) * 2 * NB * SLAB <= 160 * 1024, "LDS budget of a CU");

    const int wave_all = wave_uniform((int)threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const bool second_group = wave_all >= 4;
    const int tid = (int)threadIdx.x % NTG;
    const int wave = wave_all % 4;                        // = the batch of the group's four this wave computes
    const int hl = tid % HL, q = tid / HL;                // staging: batch and slot of this thread

    // ---- which item: (group of four batches, tile of M x N).  A group past the end repeats the last
    // item and stores nothing, so that every wave runs the same barriers.
    const int64_t items = (int64_t)g.tilesM * g.tilesN * g.sizeH;          // sizeH: groups of four batches
    const int64_t wg = g.lid_base + xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t lid = 2 * wg + (second_group ? 1 : 0);
    const bool active = lid < items;
    const Tile tile = locate_tile<true>(min(lid, items - 1), g, MT_M, MT_N);
    const int64_t m0 = wave_uniform(tile.m0), n0 = wave_uniform(tile.n0);
    const char* const Ab = (const char*)g.A + wave_uniform(tile.hA * (int64_t)ES + scalar_table(g.rbA)[m0 / MT_M]);
    const char* const Bb = (const char*)g.B + wave_uniform(tile.hB * (int64_t)ES + scalar_table(g.rbB)[n0 / MT_N]);
    const int nk = g.tilesK;

    // ---- per lane, once: global byte offsets of this thread's slab elements relative to the slab's
    // scalar base (row part + slab-periodic k part + batch), LDS write and fragment-read addresses.
    // Item e of the batch's QT-thread slice is (row e / KT, k e % KT); a thread's items are QT apart.
    uint32_t voA[PER_A], voB[PER_B];
#pragma unroll
    for (int i = 0; i < PER_A; ++i) voA[i] = g.rrA[m0 + (q + i * QT) / KT] + g.krA[q % KT] + (uint32_t)hl * ES;
#pragma unroll
    for (int i = 0; i < PER_B; ++i) voB[i] = g.rrB[n0 + (q + i * QT) / KT] + g.krB[q % KT] + (uint32_t)hl * ES;
    const int fr = lane & 15, fq = lane >> 4;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) T*)lds + (second_group ? ES * NB * SLAB : 0u);
    unsigned wA[NB], wB[NB], fA[NB], fB[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        wA[b] = lds0 + ES * (unsigned)(b * SLAB + hl * REGION + (q / KT) * LD + q % KT);
        wB[b] = wA[b] + ES * (unsigned)(MT_M * LD);
        fA[b] = lds0 + ES * (unsigned)(b * SLAB + wave * REGION + fr * LD + fq);
        fB[b] = fA[b] + ES * (unsigned)(MT_M * LD);
        asm volatile("" : "+v"(wA[b]), "+v"(wB[b]), "+v"(fA[b]), "+v"(fB[b]));     // kept, not recomputed in the loop
    }
    constexpr unsigned dW = ES * (QT / KT) * LD;          // a thread's next item: QT / KT rows further
    constexpr unsigned dF = ES * 16 * LD;                 // next block of 16 rows

    int64_t kbA = 0, kbB = 0;                             // per slab, scalar: the base of each load
    auto k_offsets = [&](int slab) __attribute__((always_inline)) {
        const int kc = min(slab, nk - 1);                 // slabs past the end repeat the last: loads that nothing uses
        kbA = scalar_table(g.kbA)[kc];
        kbB = scalar_table(g.kbB)[kc];
    };
    T ra[DEPTH][PER_A], rb[DEPTH][PER_B];                 // slab j waits in ring slot j % DEPTH
    auto gather = [&](auto SLOT) __attribute__((always_inline)) {
        constexpr int sl = decltype(SLOT)::value;
#pragma unroll
        for (int i = 0; i < PER_A; ++i) {
            asm("" : "+v"(voA[i]));                       // "scalar base + 32-bit lane offset" stays that way
            ra[sl][i] = P::load_at(Ab + kbA, voA[i], 0u);
        }
#pragma unroll
        for (int i = 0; i < PER_B; ++i) {
            asm("" : "+v"(voB[i]));
            rb[sl][i] = P::load_at(Bb + kbB, voB[i], 0u);
        }
    };
    auto stage = [&](auto BUF, auto SLOT) __attribute__((always_inline)) {
        constexpr int b = decltype(BUF)::value, sl = decltype(SLOT)::value;
#pragma unroll
        for (int i = 0; i < PER_A; ++i) lds_store<T>(wA[b] + i * dW, ra[sl][i]);
#pragma unroll
        for (int i = 0; i < PER_B; ++i) lds_store<T>(wB[b] + i * dW, rb[sl][i]);
    };
    acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) P::clear(acc[i][j]);
    T fa[FM], fb[FN];
    auto frag_load = [&](auto BUF) __attribute__((always_inline)) {
        constexpr int b = decltype(BUF)::value;
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[i] = lds_load<T>(fA[b] + i * dF);
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[j] = lds_load<T>(fB[b] + j * dF);
    };
    auto mfmas = [&]() __attribute__((always_inline)) {       // MIXED: see ComplexPolicy::mac
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) P::template mac<DNF, MIXED>(fa[i], fb[j], acc[i][j]);
    };

    // Prologue: slab 0 to LDS, slabs 1 .. DEPTH into the ring.
    k_offsets(0);
    gather(std::integral_constant<int, 0>{});
    k_offsets(1);
    if constexpr (DEPTH >= 2) {
        gather(std::integral_constant<int, 1>{});
        k_offsets(2);
    }
    stage(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    gather(std::integral_constant<int, DEPTH % DEPTH>{});               // slab DEPTH into the slot slab 0 has left
    k_offsets(DEPTH + 1);
    __syncthreads();
    if (second_group) __builtin_amdgcn_s_barrier();       // one phase behind the first group

    auto phase_end = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    };
    // Round i works on slab i (LDS buffer i % NB); its memory phase stages slab i + 1 from ring slot
    // (i + 1) % DEPTH and refills that slot with slab i + 1 + DEPTH.  No branch inside: slabs past the
    // end are clamped loads and LDS writes that nothing reads.
    constexpr int UNROLL = NB > DEPTH ? NB : DEPTH;
    auto round = [&](int i, auto IDX) __attribute__((always_inline)) {
        using BUF = std::integral_constant<int, decltype(IDX)::value % NB>;
        using NEXT_BUF = std::integral_constant<int, (decltype(IDX)::value + 1) % NB>;
        using NEXT_SLOT = std::integral_constant<int, (decltype(IDX)::value + 1) % DEPTH>;
        stage(NEXT_BUF{}, NEXT_SLOT{});
        gather(NEXT_SLOT{});
        k_offsets(i + 2 + DEPTH);
        frag_load(BUF{});
        phase_end();
        mfmas();
        phase_end();
    };
    int i = 0;
    for (; i + UNROLL <= nk; i += UNROLL)
        static_for<0, UNROLL>([&](auto IDX) __attribute__((always_inline)) { round(i + decltype(IDX)::value, IDX); });
    static_for<0, UNROLL - 1>([&](auto IDX) __attribute__((always_inline)) {
        if (i + decltype(IDX)::value < nk) round(i + decltype(IDX)::value, IDX);
    });
    if (!second_group) __builtin_amdgcn_s_barrier();      // pairs with the second group's last barrier
    settle_accumulators();

    // ---- epilogue: block by block through LDS.  Wave w writes the 16 x 16 block of its batch in
    // register order (element 64 v + lane, consecutive lanes on consecutive 16 bytes); after a barrier
    // thread (batch hl, slot q) reads elements q, q + 64, .. of batch hl, so four neighbouring lanes
    // hold one element of the four batches: 64 contiguous bytes of C and of D.  Two exchange buffers
    // alternate, so one barrier per block is enough.
    const T* __restrict__ C = (const T*)g.C + tile.hD + hl;
    T* __restrict__ D = (T*)g.D + tile.hD + hl;
    const bool read_c = g.read_c != 0;
    const bool conj_acc = g.conj_acc != 0;
    // element e = 64 r + q of a block is (row 4 r + q / 16 of the MFMA result, lane column q % 16):
    // rows run along n and columns along m, or the other way round (DNF)
    int64_t off_col[DNF ? FN : FM], off_row[DNF ? FM : FN][4];
    bool ok_col[DNF ? FN : FM], ok_row[DNF ? FM : FN][4];
    {
        const int col = q % 16, row = q / 16;
#pragma unroll
        for (int b = 0; b < (DNF ? FN : FM); ++b) {
            const int64_t x = (DNF ? n0 : m0) + b * 16 + col;
            ok_col[b] = x < (DNF ? g.sizeN : g.sizeM);
            off_col[b] = (DNF ? g.oDN : g.oDM)[x];                     // padded tables: always a valid entry
        }
#pragma unroll
        for (int b = 0; b < (DNF ? FM : FN); ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t x = (DNF ? m0 : n0) + b * 16 + 4 * r + row;
                ok_row[b][r] = x < (DNF ? g.sizeM : g.sizeN);
                off_row[b][r] = (DNF ? g.oDM : g.oDN)[x];
            }
    }
    const unsigned ew = lds0 + ES * (unsigned)(wave * (256 + 4) + lane);       // where this lane writes element 64 v + lane
    const unsigned er = lds0 + ES * (unsigned)(hl * (256 + 4) + q);            // where this thread reads element 64 r + q
    T cval[2][4];
    auto c_loads = [&](int blk, int slot) __attribute__((always_inline)) {
        const int bi = blk % FM, bj = blk / FM;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int bc = DNF ? bj : bi, br = DNF ? bi : bj;
            cval[slot][r] = P::zero();
            if (read_c && active && ok_col[bc] && ok_row[br][r]) cval[slot][r] = C[off_col[bc] + off_row[br][r]];
        }
    };
    __syncthreads();                                      // every wave has left the main loop: the slabs are free
    c_loads(0, 0);
#pragma unroll
    for (int blk = 0; blk < FM * FN; ++blk) {
        const int bi = blk % FM, bj = blk / FM;
        const unsigned buf = (blk & 1) * ES * EPI;
#pragma unroll
        for (int v = 0; v < 4; ++v) lds_store<T>(ew + buf + ES * 64 * v, T{acc[bi][bj].re[v], acc[bi][bj].im[v]});
        if (blk + 1 < FM * FN) c_loads(blk + 1, (blk + 1) & 1);
        __syncthreads();
        const int bc = DNF ? bj : bi, br = DNF ? bi : bj;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const T sum = lds_load<T>(er + buf + ES * 64 * r);
            typename P::acc_t one;
            one.re[0] = sum.x;
            one.im[0] = sum.y;
            if (active && ok_col[bc] && ok_row[br][r])
                D[off_col[bc] + off_row[br][r]] = P::combine(one, 0, g.s, read_c, cval[blk & 1][r], g.opC, conj_acc);
        }
    }
}

// ---- instantiation tables -------------------------------------------------------------------
struct Shape {
    int mt_m, mt_n, kt, wgm, wgn;
    float efficiency;      // relative speed of the main loop per unit of tile area (planner's cost model)
    int ch;                // 0: LDS-staged kernel; > 0: direct kernel with chunks of 4*ch contracted indices
    int depth;             // LDS-staged kernel: slabs of global loads in flight
    bool narrow;           // LDS-staged kernel: gather through the 32-bit tile-relative tables
    bool pingpong = false; // two-phase kernel (needs |K| % kt == 0 and slab-periodic k offsets)
    int fallback = -1;     // shape to use instead when this one's preconditions fail (-1: any)
    bool dual = false;     // two-phase kernel: one tile per wave group (two per workgroup)
    int hl = 0;            // batch-lane kernel: batches per tile (0: the tile belongs to one batch)
};
// `efficiency`: measured fraction of a CU's matrix peak that the shape's main loop sustains on
// MI355X with the CU saturated (256x128: config 2; the others: a 1024^3 product, 576^3, 96^3 x 512).
constexpr Shape kRealShapes[] = {
    {256, 128, 16, 4, 2, 0.95f, 0, 1, true, true, 9},
    {128, 128, 16, 2, 2, 0.46f, 0, 2, true},
    {64, 64, 16, 2, 2, 0.36f, 0, 3, true},
    {32, 32, 16, 2, 2, 0.30f, 0, 3, true},
    {128, 64, 16, 2, 2, 0.33f, 4, 0, false},
    {64, 64, 16, 2, 2, 0.30f, 4, 0, false},
    {32, 32, 16, 2, 2, 0.20f, 4, 0, false},
    {64, 64, 16, 2, 4, 0.36f, 0, 2, true},
    {64, 64, 16, 4, 4, 0.41f, 0, 2, true},
    {256, 128, 16, 4, 2, 0.80f, 0, 1, true, false, -1},
    {64, 64, 16, 2, 2, 0.80f, 0, 1, true, true, -1, true},
    {128, 64, 16, 2, 2, 0.85f, 0, 2, true, true, -1, true},
};
constexpr Shape kComplexShapes[] = {
    {96, 96, 8, 2, 2, 0.45f, 0, 2, true},
    {64, 64, 8, 2, 2, 0.30f, 0, 2, true},
    {32, 32, 8, 2, 2, 0.20f, 0, 3, true},
    {96, 96, 8, 2, 2, 0.45f, 2, 0, false},
    {64, 64, 8, 2, 2, 0.25f, 2, 0, false},
    {96, 48, 8, 2, 1, 0.45f, 0, 2, true},
    {48, 96, 8, 1, 2, 0.45f, 0, 2, true},
    {96, 96, 8, 2, 2, 0.85f, 0, 1, true, true, 5, true},
    {48, 48, 4, 2, 2, 0.90f, 0, 2, true, true, 7, true, kBatchLanes},
};
constexpr int kNumRealShapes = sizeof(kRealShapes) / sizeof(Shape);
constexpr int kNumComplexShapes = sizeof(kComplexShapes) / sizeof(Shape);

constexpr Shape shape_at(bool complex_table, int i) {
    return complex_table ? kComplexShapes[i < kNumComplexShapes ? i : 0] : kRealShapes[i < kNumRealShapes ? i : 0];
}

template <class P, int S, bool AKF, bool BKF, bool DNF>
hipError_t launch_one(const GettArgs& a_in, int64_t blocks, hipStream_t st) {
    constexpr Shape s = shape_at(P::is_complex, S);
    GettArgs a = a_in;
    // the two-phase and batch-lane kernels sum conj(A) * B or A * B and leave the rest of the
    // conjugation to the epilogue (ComplexPolicy::mac); the others conjugate as they gather
    a.conj_acc = (s.ch == 0 && s.pingpong && a.opB == TCX_OP_CONJ) ? 1 : 0;
    if constexpr (s.hl > 0) {
        // lanes run along the batches whatever the operands' orientation: one instantiation per DNF
        if constexpr (!AKF && !BKF && P::is_complex && P::two_phase) {
            if (!a.periodicA || !a.periodicB || a.sizeK % s.kt != 0 || a.splitK != 1) return hipErrorInvalidValue;
            const int64_t wgs = (blocks + 1) / 2;
            auto launch = [&](const GettArgs& r, int64_t count) {
                if (r.opA != r.opB)
                    gett_hlane_kernel<P, s.mt_m, s.mt_n, s.kt, DNF, s.depth, true><<<dim3((unsigned)count), dim3(512), 0, st>>>(r);
                else
                    gett_hlane_kernel<P, s.mt_m, s.mt_n, s.kt, DNF, s.depth, false><<<dim3((unsigned)count), dim3(512), 0, st>>>(r);
            };
            if (a.round_size > 0 && wgs > a.round_size) {
                GettArgs r = a;
                for (int64_t at = 0; at < wgs; at += a.round_size) {
                    r.lid_base = at;
                    launch(r, std::min<int64_t>(a.round_size, wgs - at));
                }
            } else {
                launch(a, wgs);
            }
            return hipGetLastError();
        } else if constexpr (P::is_complex && P::two_phase) {
            return launch_one<P, S, false, false, DNF>(a_in, blocks, st);
        } else {
            return hipErrorInvalidValue;
        }
    } else if constexpr (s.ch > 0) {
        // the direct kernel gathers per lane; the operands' orientation does not enter
        if constexpr (!AKF && !BKF)
            gett_direct_kernel<P, s.mt_m / 32, s.mt_n / 32, s.ch, DNF><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(a);
        else
            return launch_one<P, S, false, false, DNF>(a_in, blocks, st);
    } else if constexpr (s.pingpong) {
        constexpr int NTG = s.wgm * s.wgn * 64;
        if constexpr (!P::two_phase) {
            return hipErrorInvalidValue;      // not built for this element type / precision: the plan must not choose it
        } else if constexpr (pingpong_operand_ok<s.mt_m, NTG, AKF>() && pingpong_operand_ok<s.mt_n, NTG, BKF>()) {
            if ((AKF && !a.periodicA) || (BKF && !a.periodicB)) return hipErrorInvalidValue;
            constexpr int threads = NTG * (s.dual ? 2 : 1);
            const int64_t wgs = s.dual ? (blocks + 1) / 2 : blocks;
            const bool ragged = a.sizeK % s.kt != 0;
            constexpr bool PAIRED = s.dual && std::is_same<typename P::elem, double>::value;      // the shapes that have a paired-load twin
            auto launch = [&](const GettArgs& r, int64_t count) {
                if constexpr (PAIRED) {
                    if (r.pair && !ragged) {
                        gett_pingpong_kernel<P, s.mt_m, s.mt_n, s.kt, s.wgm, s.wgn, AKF, BKF, DNF, s.dual, (s.depth < 2 ? 2 : s.depth), false, true, 2>
                            <<<dim3((unsigned)count), dim3(threads), 0, st>>>(r);
                        return;
                    }
                }
                if constexpr (P::is_complex) {
                    if (r.opA != r.opB) {             // exactly one operand conjugated
                        if (ragged)
                            gett_pingpong_kernel<P, s.mt_m, s.mt_n, s.kt, s.wgm, s.wgn, AKF, BKF, DNF, s.dual, s.depth, true, false, 1, true>
                                <<<dim3((unsigned)count), dim3(threads), 0, st>>>(r);
                        else
                            gett_pingpong_kernel<P, s.mt_m, s.mt_n, s.kt, s.wgm, s.wgn, AKF, BKF, DNF, s.dual, s.depth, false, false, 1, true>
                                <<<dim3((unsigned)count), dim3(threads), 0, st>>>(r);
                        return;
                    }
                }
                if (ragged)
                    gett_pingpong_kernel<P, s.mt_m, s.mt_n, s.kt, s.wgm, s.wgn, AKF, BKF, DNF, s.dual, s.depth, true>
                        <<<dim3((unsigned)count), dim3(threads), 0, st>>>(r);
                else
                    gett_pingpong_kernel<P, s.mt_m, s.mt_n, s.kt, s.wgm, s.wgn, AKF, BKF, DNF, s.dual, s.depth, false>
                        <<<dim3((unsigned)count), dim3(threads), 0, st>>>(r);
            };
            // Long tiles are launched round by round (one workgroup per CU each): workgroups of a
            // round that share operand panels through an XCD's L2 start together, whereas in one big
            // launch the 0.5 - 1 % differences in tile duration between CUs add up from round to
            // round until the sharers are further apart than the L2 holds.
            if (a.round_size > 0 && a.splitK == 1 && wgs > a.round_size) {
                GettArgs r = a;
                for (int64_t at = 0; at < wgs; at += a.round_size) {
                    r.lid_base = at;
                    launch(r, std::min<int64_t>(a.round_size, wgs - at));
                }
            } else {
                launch(a, wgs);
            }
        } else {
            return hipErrorInvalidValue;      // this orientation is not built for the shape: the plan must not choose it
        }
    } else {
        gett_kernel<P, s.mt_m, s.mt_n, s.kt, s.wgm, s.wgn, AKF, BKF, DNF, s.depth>
            <<<dim3((unsigned)blocks), dim3(s.wgm * s.wgn * 64), 0, st>>>(a);
    }
    hipError_t err = hipGetLastError();
    bool reduced = false;
    if constexpr (s.ch == 0 && s.pingpong)
        reduced = a.splitK == 2 && s.dual &&
                  pair_fits_lds(sizeof(typename P::elem), sizeof(typename P::real), sizeof(typename P::elem) / sizeof(typename P::real), s.mt_m, s.mt_n, s.kt);
    if (err == hipSuccess && a.splitK > 1 && !reduced) {
        gett_reduce_kernel<P, s.mt_m, s.mt_n, s.wgm, s.wgn, DNF>
            <<<dim3((unsigned)(blocks / a.splitK)), dim3(s.wgm * s.wgn * 64), 0, st>>>(a);
        err = hipGetLastError();
    }
    return err;
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
        case 4: return launch_flags<P, 4>(akf, bkf, dnf, a, blocks, st);
        case 5: return launch_flags<P, 5>(akf, bkf, dnf, a, blocks, st);
        case 6: return launch_flags<P, 6>(akf, bkf, dnf, a, blocks, st);
        case 7: return launch_flags<P, 7>(akf, bkf, dnf, a, blocks, st);
        case 8: return launch_flags<P, 8>(akf, bkf, dnf, a, blocks, st);
        case 9: return launch_flags<P, 9>(akf, bkf, dnf, a, blocks, st);
        case 10: return launch_flags<P, 10>(akf, bkf, dnf, a, blocks, st);
        case 11: return launch_flags<P, 11>(akf, bkf, dnf, a, blocks, st);
        default: return hipErrorInvalidValue;
    }
}

template <class P>
hipError_t launch_complex_shape(int variant, bool akf, bool bkf, bool dnf, const GettArgs& a, int64_t blocks, hipStream_t st) {
    switch (variant) {
        case 0: return launch_flags<P, 0>(akf, bkf, dnf, a, blocks, st);
        case 1: return launch_flags<P, 1>(akf, bkf, dnf, a, blocks, st);
        case 2: return launch_flags<P, 2>(akf, bkf, dnf, a, blocks, st);
        case 3: return launch_flags<P, 3>(akf, bkf, dnf, a, blocks, st);
        case 4: return launch_flags<P, 4>(akf, bkf, dnf, a, blocks, st);
        case 5: return launch_flags<P, 5>(akf, bkf, dnf, a, blocks, st);
        case 6: return launch_flags<P, 6>(akf, bkf, dnf, a, blocks, st);
        default: break;
    }
    if constexpr (P::two_phase) {
        if (variant == 7) return launch_flags<P, 7>(akf, bkf, dnf, a, blocks, st);
        if (variant == 8) return launch_flags<P, 8>(akf, bkf, dnf, a, blocks, st);
    }
    return hipErrorInvalidValue;
}

// Tensors whose storage is narrower than the arithmetic (32-bit in 64-bit arithmetic, 16-bit in
// 32- or 64-bit arithmetic): two staged shapes each (64 x 64 and 32 x 32)
constexpr int kWideRealShapes[] = {2, 3};
constexpr int kWideComplexShapes[] = {1, 2};
template <class P>
hipError_t launch_wide_shape(int variant, bool akf, bool bkf, bool dnf, const GettArgs& a, int64_t blocks, hipStream_t st) {
    constexpr int v0 = P::is_complex ? kWideComplexShapes[0] : kWideRealShapes[0];
    constexpr int v1 = P::is_complex ? kWideComplexShapes[1] : kWideRealShapes[1];
    if (variant == v0) return launch_flags<P, v0>(akf, bkf, dnf, a, blocks, st);
    if (variant == v1) return launch_flags<P, v1>(akf, bkf, dnf, a, blocks, st);
    return hipErrorInvalidValue;
}

const Shape* shapes_of(int dtype, int* n) {
    if (dtype == TCX_C128 || dtype == TCX_C64) { *n = kNumComplexShapes; return kComplexShapes; }
    if (dtype == TCX_F64 || dtype == TCX_F32 || dtype == TCX_F16 || dtype == TCX_BF16) { *n = kNumRealShapes; return kRealShapes; }
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
    const int planes = is_complex(dtype) ? 2 : 1;
    return {s.mt_m, s.mt_n, s.kt, s.wgm * s.wgn * 64, s.efficiency, s.mt_m * s.mt_n * planes, s.ch == 0 && s.narrow, s.pingpong, s.fallback, s.dual,
            s.hl == 0 && s.dual && pair_fits_lds(elem_bytes_of(dtype), real_bytes_of(dtype), planes, s.mt_m, s.mt_n, s.kt),
            s.hl > 0 ? s.hl : 1};
}

bool gett_available(int dtype, int precision, int variant) {
    if (variant < 0 || variant >= gett_num_variants(dtype)) return false;
    if (is_widened(dtype, precision)) {
        const int* ok = is_complex(dtype) ? kWideComplexShapes : kWideRealShapes;
        return variant == ok[0] || variant == ok[1];
    }
    if (dtype == TCX_C64) return !gett_variant(dtype, variant).pingpong;      // the two-phase complex kernels are fp64 only
    return true;
}

int launch_gett(int dtype, int precision, int variant, bool a_kf, bool b_kf, bool d_nf, const GettArgs& args, void* stream,
                int64_t* grid, int* block) {
    if (!gett_available(dtype, precision, variant)) return (int)hipErrorInvalidValue;
    if (args.splitK < 1) return (int)hipErrorInvalidValue;
    if (args.splitK > 1 && !args.workspace && !(args.splitK == 2 && gett_variant(dtype, variant).pair_in_lds))
        return (int)hipErrorInvalidValue;
    const int64_t blocks = (int64_t)args.tilesM * args.tilesN * args.sizeH * args.splitK;      // sizeH: in units of the shape's batches per tile
    const GettVariant gv = gett_variant(dtype, variant);
    *grid = gv.dual ? (blocks + 1) / 2 : blocks;
    *block = gv.threads * (gv.dual ? 2 : 1);
    if (blocks <= 0 || blocks > 0x7fffffff) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    const bool wide = is_widened(dtype, precision);
    switch (dtype) {
        case TCX_F64: return (int)launch_real_shape<RealPolicy<double>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
        case TCX_F32:
            if (wide) return (int)launch_wide_shape<RealPolicy<double, float>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
            return (int)launch_real_shape<RealPolicy<float>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
        case TCX_F16:        // 16-bit storage is always widened: fp32 MFMAs by default, fp64 on request
            if (precision == TCX_PREC_F64) return (int)launch_wide_shape<RealPolicy<double, _Float16>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
            return (int)launch_wide_shape<RealPolicy<float, _Float16>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
        case TCX_BF16:
            if (precision == TCX_PREC_F64) return (int)launch_wide_shape<RealPolicy<double, bf16_t>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
            return (int)launch_wide_shape<RealPolicy<float, bf16_t>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
        case TCX_C128: return (int)launch_complex_shape<ComplexPolicyT<double>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
        case TCX_C64:
            if (wide) return (int)launch_wide_shape<ComplexPolicyT<double, float>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
            return (int)launch_complex_shape<ComplexPolicyT<float>>(variant, a_kf, b_kf, d_nf, args, blocks, st);
        default: return (int)hipErrorInvalidValue;
    }
}

}  // namespace tcx
