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
    static __device__ __forceinline__ double out(const Scalars& s, double acc, bool rc, double c, int) {
        double d = s.alpha_re * acc;
        if (rc) d += s.beta_re * c;
        return d;
    }
};
template <> struct SNum<float> {
    static __device__ __forceinline__ float ld(const float* p, int64_t o, int) { return p[o]; }
    static __device__ __forceinline__ float zero() { return 0.0f; }
    static __device__ __forceinline__ float fma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
    static __device__ __forceinline__ float out(const Scalars& s, float acc, bool rc, float c, int) {
        float d = (float)s.alpha_re * acc;
        if (rc) d += (float)s.beta_re * c;
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
    static __device__ __forceinline__ double2 out(const Scalars& s, double2 acc, bool rc, double2 c, int opC) {
        double2 d{s.alpha_re * acc.x - s.alpha_im * acc.y, s.alpha_re * acc.y + s.alpha_im * acc.x};
        if (rc) {
            if (opC == TCX_OP_CONJ) c.y = -c.y;
            d.x += s.beta_re * c.x - s.beta_im * c.y;
            d.y += s.beta_re * c.y + s.beta_im * c.x;
        }
        return d;
    }
};

template <> struct SNum<float2> {
    static __device__ __forceinline__ float2 ld(const float2* p, int64_t o, int op) {
        float2 v = p[o];
        if (op == TCX_OP_CONJ) v.y = -v.y;
        return v;
    }
    static __device__ __forceinline__ float2 zero() { return float2{0.0f, 0.0f}; }
    static __device__ __forceinline__ float2 fma(float2 a, float2 b, float2 c) {
        c.x = __builtin_fmaf(a.x, b.x, c.x);
        c.x = __builtin_fmaf(-a.y, b.y, c.x);
        c.y = __builtin_fmaf(a.x, b.y, c.y);
        c.y = __builtin_fmaf(a.y, b.x, c.y);
        return c;
    }
    static __device__ __forceinline__ float2 out(const Scalars& s, float2 acc, bool rc, float2 c, int opC) {
        const float ar = (float)s.alpha_re, ai = (float)s.alpha_im, br = (float)s.beta_re, bi = (float)s.beta_im;
        float2 d{ar * acc.x - ai * acc.y, ar * acc.y + ai * acc.x};
        if (rc) {
            if (opC == TCX_OP_CONJ) c.y = -c.y;
            d.x += br * c.x - bi * c.y;
            d.y += br * c.y + bi * c.x;
        }
        return d;
    }
};

// KC > 0: the number of contracted terms is the compile-time constant KC (inner loop unrolled);
// KC == 0: any K.
//
// Every tile has the same shape, so a thread's share of the lookup tables (which elements it
// stages, which outputs it forms) is the same for every tile: it is read once into registers
// before the tile loop.  Inside the loop a thread issues all its global loads back to back.
//
// PACED: a plan whose operand lines collide in the L2 (stream_plan.cpp) issues a tile's loads in
// pairs (one of A, one of B) and lets at most one older pair stay in flight behind each new one,
// instead of sending all of a tile's misses to one L2 set at once.
template <class T, int KC, bool PACED>
__global__ __launch_bounds__(kStreamThreads) void stream_kernel(StreamArgs g) {
    using N_ = SNum<T>;
    constexpr int PER = kStreamPerThread;
    constexpr unsigned NEVER = 0xffffu;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    T* sA = (T*)lds_raw;
    T* sB = sA + (size_t)g.rowsA * g.K;
    const int K = KC > 0 ? KC : g.K;
    const int tid = threadIdx.x;

    int64_t srcA[PER], srcB[PER], offD[PER];
    unsigned packA[PER], packB[PER], rab[PER];       // pack = digit << 16 | LDS slot
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int p = tid + i * kStreamThreads;
        srcA[i] = 0; srcB[i] = 0; offD[i] = 0;
        packA[i] = packB[i] = NEVER << 16;
        rab[i] = 0;
        if (p < g.nItemsA) { const StreamItem it = g.itemsA[p]; srcA[i] = it.src; packA[i] = it.digit << 16 | it.slot; }
        if (p < g.nItemsB) { const StreamItem it = g.itemsB[p]; srcB[i] = it.src; packB[i] = it.digit << 16 | it.slot; }
        if (p < g.tile) { rab[i] = g.rowAB[p]; offD[i] = g.dD[p]; }
    }

    // Tile index -> base offsets through two small plan-time tables (low / high part of the
    // outer index), one division per tile instead of one per outer mode.
    struct Where {
        int64_t a, b, d;
        unsigned digits;      // valid indices along the split mode (the last chunk may be ragged)
    };
    auto locate = [&](int64_t tile) {
        const int64_t hi = tile / g.outer_lo, lo = tile - hi * g.outer_lo;
        const int64_t* pl = g.tabLo + lo * 4;
        const int64_t* ph = g.tabHi + hi * 4;
        return Where{pl[0] + ph[0], pl[1] + ph[1], pl[2] + ph[2], (unsigned)pl[3]};
    };
    T va[PER], vb[PER], vc[PER];
    auto fetch = [&](const Where& w) {       // global loads of a tile's operands (and its C), all in flight together
        const T* A = (const T*)g.A + w.a;
        const T* B = (const T*)g.B + w.b;
        if constexpr (PACED) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                if ((packA[i] >> 16) < w.digits) va[i] = N_::ld(A, srcA[i], g.opA);
                if ((packB[i] >> 16) < w.digits) vb[i] = N_::ld(B, srcB[i], g.opB);
                // in-order return: "at most two outstanding" = the pair before this one has arrived
                // (earlier stores of D count too, which only makes the wait longer)
                asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
            }
        } else {
#pragma unroll
            for (int i = 0; i < PER; ++i)
                if ((packA[i] >> 16) < w.digits) va[i] = N_::ld(A, srcA[i], g.opA);
#pragma unroll
            for (int i = 0; i < PER; ++i)
                if ((packB[i] >> 16) < w.digits) vb[i] = N_::ld(B, srcB[i], g.opB);
        }
        if (g.read_c) {
            const T* C = (const T*)g.C + w.d;
            const int valid = g.inner * (int)w.digits;
#pragma unroll
            for (int i = 0; i < PER; ++i)
                if (tid + i * kStreamThreads < valid) vc[i] = C[offD[i]];
        }
    };

    // Three tiles are in flight per workgroup: `cur` is computed from LDS, the operands of
    // `nxt` travel from memory, and the table rows of the tile after that are being fetched.
    int64_t tile = blockIdx.x;
    if (tile >= g.num_tiles) return;
    const int64_t step = gridDim.x;
    Where cur = locate(tile);
    fetch(cur);
    Where nxt = cur;
    if (tile + step < g.num_tiles) nxt = locate(tile + step);
    while (true) {
        __syncthreads();          // the previous tile's reads of LDS are done
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if ((packA[i] >> 16) < cur.digits) sA[packA[i] & 0xffffu] = va[i];
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if ((packB[i] >> 16) < cur.digits) sB[packB[i] & 0xffffu] = vb[i];
        __syncthreads();

        // C of this tile arrived with its operands; keep it while the next tile's loads reuse vc
        T cv[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) cv[i] = vc[i];
        const bool more = tile + step < g.num_tiles;
        Where after = nxt;
        if (more) {
            fetch(nxt);
            if (tile + 2 * step < g.num_tiles) after = locate(tile + 2 * step);
        }

        const int valid = g.inner * (int)cur.digits;
        T* D = (T*)g.D + cur.d;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int e = tid + i * kStreamThreads;
            if (e < valid) {
                const T* a = sA + (size_t)(rab[i] & 0xffffu) * K;
                const T* b = sB + (size_t)(rab[i] >> 16) * K;
                T acc = N_::zero();
                if (KC > 0) {
#pragma unroll
                    for (int k = 0; k < KC; ++k) acc = N_::fma(a[k], b[k], acc);
                } else {
                    for (int k = 0; k < K; ++k) acc = N_::fma(a[k], b[k], acc);
                }
                D[offD[i]] = N_::out(g.s, acc, g.read_c != 0, cv[i], g.opC);
            }
        }
        if (!more) break;
        tile += step;
        cur = nxt;
        nxt = after;
    }
}

// Blocked tiles: thread `tid` owns lane index tid of the tile and a regA x regB block of outputs
// (free indices of A times free indices of B held in registers): regA + regB operand rows are
// read from LDS for regA * regB outputs.  No chunk is ragged here (the planner takes divisors).
// PER: staged operand elements per thread and operand the instantiation has registers for (the
// launcher picks the smallest that holds the plan's item lists: a tile that stages few elements
// then runs three waves per SIMD instead of two).
template <class T, int KC, int PER>
__global__ __launch_bounds__(kStreamThreads) void stream_blocked_kernel(StreamArgs g) {
    using N_ = SNum<T>;
    static_assert(PER <= kStreamPerThread, "the planner's cap");
    constexpr int RB = kStreamRegBlock;
    constexpr unsigned NEVER = 0xffffu;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    T* sA = (T*)lds_raw;
    T* sB = sA + (size_t)g.rowsA * KC;
    const int tid = threadIdx.x;

    int64_t srcA[PER], srcB[PER];
    unsigned slotA[PER], slotB[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int p = tid + i * kStreamThreads;
        srcA[i] = 0; srcB[i] = 0;
        slotA[i] = slotB[i] = NEVER;
        if (p < g.nItemsA) { const StreamItem it = g.itemsA[p]; srcA[i] = it.src; slotA[i] = it.slot; }
        if (p < g.nItemsB) { const StreamItem it = g.itemsB[p]; srcB[i] = it.src; slotB[i] = it.slot; }
    }
    const bool lane_ok = tid < g.tile;
    const unsigned rab = lane_ok ? g.rowAB[tid] : 0u;
    const int64_t offL = lane_ok ? g.dD[tid] : 0;

    struct Where {
        int64_t a, b, d;
    };
    auto locate = [&](int64_t tile) {
        const int64_t hi = tile / g.outer_lo, lo = tile - hi * g.outer_lo;
        const int64_t* pl = g.tabLo + lo * 4;
        const int64_t* ph = g.tabHi + hi * 4;
        return Where{pl[0] + ph[0], pl[1] + ph[1], pl[2] + ph[2]};
    };
    T va[PER], vb[PER];
    auto fetch = [&](const Where& w) {
        const T* A = (const T*)g.A + w.a;
        const T* B = (const T*)g.B + w.b;
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (slotA[i] != NEVER) va[i] = N_::ld(A, srcA[i], g.opA);
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (slotB[i] != NEVER) vb[i] = N_::ld(B, srcB[i], g.opB);
    };

    int64_t tile = blockIdx.x;
    if (tile >= g.num_tiles) return;
    const int64_t step = gridDim.x;
    Where cur = locate(tile);
    fetch(cur);
    Where nxt = cur;
    if (tile + step < g.num_tiles) nxt = locate(tile + step);
    while (true) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (slotA[i] != NEVER) sA[slotA[i]] = va[i];
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (slotB[i] != NEVER) sB[slotB[i]] = vb[i];
        __syncthreads();

        const bool more = tile + step < g.num_tiles;
        Where after = nxt;
        if (more) {
            fetch(nxt);
            if (tile + 2 * step < g.num_tiles) after = locate(tile + 2 * step);
        }

        if (lane_ok) {
            const T* C = (const T*)g.C + cur.d + offL;
            T* D = (T*)g.D + cur.d + offL;
            T a[RB][KC], b[RB][KC];
            // (register indices beyond the block re-read its last row: no branch around the reads)
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const T* row = sA + (size_t)((rab & 0xffffu) + min(r, g.regA - 1) * g.rowStepA) * KC;
#pragma unroll
                for (int k = 0; k < KC; ++k) a[r][k] = row[k];
            }
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const T* row = sB + (size_t)((rab >> 16) + min(r, g.regB - 1) * g.rowStepB) * KC;
#pragma unroll
                for (int k = 0; k < KC; ++k) b[r][k] = row[k];
            }
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                if (rb < g.regB) {
                    T cv[RB];
                    if (g.read_c) {
#pragma unroll
                        for (int ra = 0; ra < RB; ++ra)
                            if (ra < g.regA) cv[ra] = C[g.dRegA[ra] + g.dRegB[rb]];
                    }
#pragma unroll
                    for (int ra = 0; ra < RB; ++ra)
                        if (ra < g.regA) {
                            T acc = N_::zero();
#pragma unroll
                            for (int k = 0; k < KC; ++k) acc = N_::fma(a[ra][k], b[rb][k], acc);
                            D[g.dRegA[ra] + g.dRegB[rb]] = N_::out(g.s, acc, g.read_c != 0, cv[ra], g.opC);
                        }
                }
        }
        if (!more) break;
        tile += step;
        cur = nxt;
        nxt = after;
    }
}

// Blocked tiles whose lanes all run along hyper (batch) modes: no lane shares an operand element
// with another, so there is nothing to stage.  Every lane reads the regA + regB operand rows of
// its own batch index straight from memory, contracted index by contracted index, and keeps the
// regA x regB accumulators in registers; loads and stores coalesce along the batch modes.  No
// LDS, no barrier; the waves of a CU cover each other's load latency.
template <class T, int KC>
__global__ __launch_bounds__(kStreamThreads) void stream_direct_kernel(StreamArgs g) {
    using N_ = SNum<T>;
    constexpr int RB = kStreamRegBlock;
    const int tid = threadIdx.x;
    if (tid >= g.tile) return;
    const int64_t offA = g.laneA[tid], offB = g.laneB[tid], offD = g.dD[tid];
    const int64_t step = gridDim.x;
    for (int64_t tile = blockIdx.x; tile < g.num_tiles; tile += step) {
        const int64_t hi = tile / g.outer_lo, lo = tile - hi * g.outer_lo;
        const int64_t* pl = g.tabLo + lo * 4;
        const int64_t* ph = g.tabHi + hi * 4;
        const T* A = (const T*)g.A + pl[0] + ph[0] + offA;
        const T* B = (const T*)g.B + pl[1] + ph[1] + offB;
        const T* C = (const T*)g.C + pl[2] + ph[2] + offD;
        T* D = (T*)g.D + pl[2] + ph[2] + offD;
        // Straight-line code: register indices beyond the block repeat its last row (a load that
        // hits the cache, an unused product) instead of branching around the loads, so that the
        // loads of a tile are issued together and waited for once.
        T acc[RB][RB];
#pragma unroll
        for (int ra = 0; ra < RB; ++ra)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[ra][rb] = N_::zero();
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            T a[RB], b[RB];
#pragma unroll
            for (int r = 0; r < RB; ++r) a[r] = N_::ld(A, g.aReg[min(r, g.regA - 1)] + g.aK[k], g.opA);
#pragma unroll
            for (int r = 0; r < RB; ++r) b[r] = N_::ld(B, g.bReg[min(r, g.regB - 1)] + g.bK[k], g.opB);
#pragma unroll
            for (int ra = 0; ra < RB; ++ra)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) acc[ra][rb] = N_::fma(a[ra], b[rb], acc[ra][rb]);
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int64_t col = g.dRegB[min(rb, g.regB - 1)];
            T cv[RB];
#pragma unroll
            for (int ra = 0; ra < RB; ++ra) cv[ra] = N_::zero();
            if (g.read_c) {
#pragma unroll
                for (int ra = 0; ra < RB; ++ra) cv[ra] = C[g.dRegA[min(ra, g.regA - 1)] + col];
            }
#pragma unroll
            for (int ra = 0; ra < RB; ++ra)
                if (ra < g.regA && rb < g.regB) D[g.dRegA[ra] + col] = N_::out(g.s, acc[ra][rb], g.read_c != 0, cv[ra], g.opC);
        }
    }
}

template <class T>
hipError_t launch_k(bool blocked, bool direct, const StreamArgs& a, size_t lds, unsigned blocks, hipStream_t st) {
    if (blocked && direct) {
        switch (a.K) {
            case 1: stream_direct_kernel<T, 1><<<dim3(blocks), dim3(kStreamThreads), 0, st>>>(a); break;
            case 2: stream_direct_kernel<T, 2><<<dim3(blocks), dim3(kStreamThreads), 0, st>>>(a); break;
            case 4: stream_direct_kernel<T, 4><<<dim3(blocks), dim3(kStreamThreads), 0, st>>>(a); break;
            default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    if (blocked) {
        const int need = (std::max(a.nItemsA, a.nItemsB) + kStreamThreads - 1) / kStreamThreads;
        if (need > kStreamPerThread) return hipErrorInvalidValue;
        auto go = [&](auto KC_) {
            constexpr int KC = decltype(KC_)::value;
            if (need <= 2) stream_blocked_kernel<T, KC, 2><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a);
            else if (need <= 4) stream_blocked_kernel<T, KC, 4><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a);
            else stream_blocked_kernel<T, KC, kStreamPerThread><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a);
        };
        switch (a.K) {
            case 1: go(std::integral_constant<int, 1>{}); break;
            case 2: go(std::integral_constant<int, 2>{}); break;
            case 4: go(std::integral_constant<int, 4>{}); break;
            default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    auto flat = [&](auto PACED_) {
        constexpr bool PACED = decltype(PACED_)::value;
        switch (a.K) {
            case 1: stream_kernel<T, 1, PACED><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
            case 2: stream_kernel<T, 2, PACED><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
            case 4: stream_kernel<T, 4, PACED><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
            case 8: stream_kernel<T, 8, PACED><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
            default: stream_kernel<T, 0, PACED><<<dim3(blocks), dim3(kStreamThreads), lds, st>>>(a); break;
        }
    };
    if (a.paced) flat(std::true_type{});
    else flat(std::false_type{});
    return hipGetLastError();
}

}  // namespace

// Workgroups launched for a streaming plan; each walks the tile list with a grid stride.  A
// workgroup reads its share of the plan's lookup tables once, so the flat kernels (a dozen table
// entries per thread) run as a persistent grid of 8 workgroups per CU.  The blocked kernels read
// few entries, and for them the memory system does better the shorter a workgroup lives
// (workgroups dispatched in order keep the chip's stores inside a narrow window of D): measured on
// 2 GB outputs, 4^14 elements, 8 / 32 / 64 per CU / one tile each: 411 / 373 / 374 / 426 us with
// four staged elements per thread, 403 / 396 / 388 / 372 us with two.
int64_t stream_grid(bool blocked, bool direct, int items_per_thread, int64_t num_tiles, int num_cu) {
    const int64_t cus = num_cu > 0 ? num_cu : 256;
    int64_t cap = cus * 8;
    if (direct || (blocked && items_per_thread <= 2)) cap = num_tiles;
    else if (blocked) cap = cus * 64;
    if (cap > 0x7fffffff) cap = 0x7fffffff;          // the grid stride covers what the grid does not
    return num_tiles < cap ? num_tiles : cap;
}

int launch_stream(int dtype, bool blocked, bool direct, const StreamArgs& args, size_t lds_bytes, int num_cu, void* stream,
                  int64_t* grid, int* block) {
    const int need = (std::max(args.nItemsA, args.nItemsB) + kStreamThreads - 1) / kStreamThreads;
    const int64_t blocks = stream_grid(blocked, direct, need, args.num_tiles, num_cu);
    *grid = blocks;
    *block = kStreamThreads;
    if (blocks <= 0) return (int)hipErrorInvalidConfiguration;
    hipStream_t st = (hipStream_t)stream;
    switch (dtype) {
        case TCX_F64: return (int)launch_k<double>(blocked, direct, args, lds_bytes, (unsigned)blocks, st);
        case TCX_F32: return (int)launch_k<float>(blocked, direct, args, lds_bytes, (unsigned)blocks, st);
        case TCX_C128: return (int)launch_k<double2>(blocked, direct, args, lds_bytes, (unsigned)blocks, st);
        case TCX_C64: return (int)launch_k<float2>(blocked, direct, args, lds_bytes, (unsigned)blocks, st);
        default: return (int)hipErrorInvalidValue;
    }
}

}  // namespace tcx
