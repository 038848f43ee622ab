// C-ABI layer of libtcx: opaque objects, argument checking, plan construction (analyser +
// offset tables + kernel choice) and the execute call.  See include/tcx.h for the contract.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <unordered_map>

#include "tcx_internal.hpp"

// Fixed scratch buffer of tcx_execute_product_noalloc: device memory that exists from the moment
// the library's code is loaded on a GPU until the process ends, so that an execution which needs
// room for split-K partial sums does not have to allocate it.  Every GPU holds its own copy at its
// own address; in host code the array's name only identifies the symbol.  The address on a device
// is asked for once, with that device current, when a handle is created on it, and kept.
static __device__ __align__(256) unsigned char scratch[TCX_SCRATCH_BYTES];

// The number one in 64-bit and in 32-bit (complex: 1 + 0i): the second operand of the contraction
// that a unary or binary operation is planned as (C := alpha A + beta B  is  alpha A * 1 + beta B).
static __device__ __align__(16) double one_in_64_bits[2] = {1.0, 0.0};
static __device__ __align__(16) float one_in_32_bits[2] = {1.0f, 0.0f};
static __device__ __align__(16) unsigned short one_in_16_bits[16] = {0x3c00u, 0, 0, 0, 0, 0, 0, 0,       // 1.0 as IEEE binary16
                                                                     0x3f80u, 0, 0, 0, 0, 0, 0, 0};      // 16 bytes on: as bfloat16

namespace tcx {
namespace {

enum : uint32_t { MAGIC_HANDLE = 0x74637801, MAGIC_EXEC, MAGIC_INFO, MAGIC_PRODUCT, MAGIC_STATUS, MAGIC_ATTR };

struct Handle {
    int device = -1;
    bool has_device = false;
    int num_cu = 0;
    void* scratch = nullptr;   // this device's copy of the fixed scratch buffer (tcx_execute_product_noalloc)
    const void* one64 = nullptr;   // ... of the constants 1 (unary and binary operations)
    const void* one32 = nullptr;
    const void* one16 = nullptr;
};
struct Executor {
    Handle handle;
    hipStream_t stream = nullptr;
    // Partial sums of split-K products executed through this executor.  Work on one stream runs
    // in order, so successive executions may share the buffer; other executors have their own.
    void* workspace = nullptr;
    size_t workspace_bytes = 0;
    std::mutex mu;
};
struct Info {
    TensorDesc desc;
};
enum { KIND_CONTRACTION = 0, KIND_BINARY = 1, KIND_UNARY = 2 };
struct Product {
    Handle handle;
    int kind = KIND_CONTRACTION;     // which execute call the plan belongs to
    Analysis an;
    int variant = 0;                 // index into the tiled kernel instantiations
    int splitK = 1;                  // parts the K slabs are divided into (tiled path)
    // offset tables, host copies and one device allocation holding all six
    std::vector<int64_t> tables[6];  // oAM oAK oBN oBK oDM oDN
    int64_t* dev_tables = nullptr;
    size_t dev_offset[6] = {0, 0, 0, 0, 0, 0};
    // tile-relative 32-bit gather tables of the LDS-staged tiled kernels (built for the plan's
    // tile shape; one device allocation): per operand rowrel, rowbase, kofs, krel, kbase
    unsigned char* dev_narrow = nullptr;
    size_t narrow_off[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    int narrow_variant = -1;         // tile shape the narrow tables were built for (-1: none)
    int analysed_path = TCX_PATH_GENERIC; // the analyser's verdict, before routing and overrides
    bool periodic[2] = {false, false};   // A, B: relative k offsets repeat from slab to slab
    bool pairs = false;                  // both operands can be gathered two neighbouring elements at a time
    int pair_step[2] = {0, 0};           // ... element x along the lanes is paired with x + step
    GenericArgs generic{};
    // bandwidth path: plan and its device tables (one allocation)
    StreamPlan stream;
    unsigned char* dev_stream = nullptr;
    size_t stream_off[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // rowAB, dD, itemsA, itemsB, tabLo, tabHi, laneA, laneB
};
struct Status {
    int64_t path = 0, variant = 0, grid = 0, block = 0, tile_m = 0, tile_n = 0, tile_k = 0, hip_error = 0, gather_width = 1;
};

// Workgroups per launch when a product's grid is enqueued round by round (0: one launch).  Rounds
// pay off when a tile runs for milliseconds (hundreds of slabs): see the launcher.
int64_t round_size_of(const Product& p, const GettVariant& s) {
    const int64_t nk = (p.an.sizeK + s.kt - 1) / s.kt;
    return (s.pingpong && nk >= 256) ? (p.handle.num_cu > 0 ? p.handle.num_cu : 256) : 0;   // a plan-only handle assumes 256 CUs
}

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};
void* g_one64_ptr[kMaxDevices] = {};
void* g_one32_ptr[kMaxDevices] = {};
void* g_one16_ptr[kMaxDevices] = {};
bool g_scratch_asked[kMaxDevices] = {};

// Address of `scratch` on `device`, which must be the current device.  nullptr if the runtime
// cannot tell (the no-alloc entry point then refuses split products).
void* scratch_on(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_asked[device]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            ptr = nullptr;
        }
        g_scratch_ptr[device] = ptr;
        if (hipGetSymbolAddress(&g_one64_ptr[device], HIP_SYMBOL(one_in_64_bits)) != hipSuccess) { (void)hipGetLastError(); g_one64_ptr[device] = nullptr; }
        if (hipGetSymbolAddress(&g_one32_ptr[device], HIP_SYMBOL(one_in_32_bits)) != hipSuccess) { (void)hipGetLastError(); g_one32_ptr[device] = nullptr; }
        if (hipGetSymbolAddress(&g_one16_ptr[device], HIP_SYMBOL(one_in_16_bits)) != hipSuccess) { (void)hipGetLastError(); g_one16_ptr[device] = nullptr; }
        g_scratch_asked[device] = true;
    }
    return g_scratch_ptr[device];
}

std::mutex g_mu;
std::unordered_map<intptr_t, uint32_t> g_live;   // handle value -> object type
// free-form key-value pairs of every live object (Sec. "Virtual Key-Value Stores")
std::unordered_map<intptr_t, std::map<int32_t, std::vector<unsigned char>>> g_kv;
struct Attr {};                                  // a bare store: all it has lives in g_kv

template <class T> intptr_t publish(T* obj, uint32_t magic) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_live[(intptr_t)obj] = magic;
    return (intptr_t)obj;
}
template <class T> T* lookup(intptr_t h, uint32_t magic) {
    if (h == 0) return nullptr;
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_live.find(h);
    return (it != g_live.end() && it->second == magic) ? (T*)h : nullptr;
}
template <class T> tcx_error_t retire(intptr_t* h, uint32_t magic) {
    if (!h) return TCX_ERR_NULL_ARG;
    T* obj = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_live.find(*h);
        if (*h == 0 || it == g_live.end() || it->second != magic) return TCX_ERR_INVALID_HANDLE;
        obj = (T*)*h;
        g_live.erase(it);
        g_kv.erase(*h);
    }
    delete obj;
    *h = 0;
    return TCX_SUCCESS;
}

int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

int64_t tiles_of(const Analysis& an, const GettVariant& s) {
    return ((an.sizeM + s.mt_m - 1) / s.mt_m) * ((an.sizeN + s.mt_n - 1) / s.mt_n) * (an.sizeH / s.hl);
}

// The batch-lane kernel takes plans whose fastest hyper mode is the fastest mode of A, B and D
// (stride 1) with an extent it can cut into whole groups of s.hl batches.
bool batch_lanes_ok(const Analysis& an, const GettVariant& s) {
    if (s.hl <= 1) return true;
    if (an.H.empty()) return false;
    const Mode& h = an.H[0];
    return h.sA == 1 && h.sB == 1 && h.sD == 1 && h.extent % s.hl == 0;
}

// Cost model for tile shape and split-K, in microseconds.  A workgroup's time is its slabs at
// the shape's fraction of the CU's matrix peak plus a fixed prologue/epilogue; the grid runs
// in rounds over the CUs; split-K adds a second launch and the traffic of the partial
// accumulators, and writing D (about 4 TB/s) is exposed in full where a CU holds one workgroup,
// so that every CU stores at the same time, and half hidden behind other workgroups' main
// loops otherwise.  Large tiles win when there are enough of them; small problems are cut
// along K to fill the chip.
struct PlanChoice {
    double us;
    int variant, splitK;
};

// Every tile shape with its best split count, cheapest first.
std::vector<PlanChoice> rank_plans(const Analysis& an, int num_cu) {
    std::vector<PlanChoice> ranked;
    const int n = gett_num_variants(an.dtype);
    const double cus = num_cu > 0 ? num_cu : 256;
    const double cu_flops = (compute_real_bytes(an.dtype, an.precision) == 4 ? 157.3e12 : 78.6e12) / 256.0;
    const double flop_per_mac = is_complex(an.dtype) ? 8.0 : 2.0;
    const int ebytes = elem_bytes_of(an.dtype);
    const double store_us = (double)an.sizeH * an.sizeM * an.sizeN * ebytes / 4e12 * 1e6;
    for (int v = 0; v < n; ++v) {
        const GettVariant s = gett_variant(an.dtype, v);
        if (!gett_available(an.dtype, an.precision, v) || !batch_lanes_ok(an, s)) continue;
        double best = -1;
        int bestS = 1;
        const double tiles = (double)tiles_of(an, s);
        const int64_t nk = (an.sizeK + s.kt - 1) / s.kt;
        const double slab_us = flop_per_mac * s.mt_m * s.mt_n * s.kt / (cu_flops * s.efficiency) * 1e6;
        for (int64_t want : {1, 2, 3, 4, 6, 8}) {
            if (want > nk || (want > 1 && s.hl > 1)) break;
            const int64_t per = (nk + want - 1) / want;
            const int64_t S = (nk + per - 1) / per;
            // small tiles leave room for several workgroups per CU, which then share its matrix
            // pipe: the time of a round does not shrink, but a partial last round costs less
            const double resident = s.dual ? 2.0   // one workgroup per CU, two tiles in it
                                           : std::max(1.0, std::min(4.0, 65536.0 / ((double)s.mt_m * s.mt_n * (ebytes > 8 ? 2 : 1))));
            const double slots = cus * resident;
            const double rounds = std::ceil(tiles * (double)S / slots);
            double us = rounds * resident * (double)per * slab_us + 6.0 + store_us * (s.pingpong ? 1.0 : 0.5);
            if (S > 1 && !(S == 2 && s.pair_in_lds))
                us += 3.0 + (2.0 * S + 1.0) * tiles * s.acc_reals * (ebytes > 8 ? 8 : ebytes) / 6e12 * 1e6;
            if (best < 0 || us < best) { best = us; bestS = (int)S; }
        }
        // Short tiles that already give every CU a workgroup are not cut along K: such a product
        // is bound by latency, not by the matrix pipe, and the model above overrates the split.
        // Measured on a 576^3 product in 324 tiles of 32 x 32 (36 slabs each): one launch of the
        // unsplit tiles 21.3 us; K in 2, 3, 4, 6 parts plus the reduction launch 21.3, 21.0, 22.5,
        // 22.0 us, with four times the memory traffic (partial sums written and read back).
        if (bestS > 1 && !(bestS == 2 && s.pair_in_lds) && nk <= 64 && tiles >= cus) bestS = 1;
        ranked.push_back({best, v, bestS});
    }
    std::stable_sort(ranked.begin(), ranked.end(), [](const PlanChoice& x, const PlanChoice& y) { return x.us < y.us; });
    return ranked;
}

void choose_plan(const Analysis& an, int num_cu, int* variant, int* splitK) {
    const std::vector<PlanChoice> r = rank_plans(an, num_cu);
    if (r.empty()) return;
    *variant = r[0].variant;
    *splitK = r[0].splitK;
}

void fill_generic(const Analysis& an, GenericArgs* g) {
    // every mode that indexes D, D-fastest first, so neighbouring threads write neighbouring elements
    std::vector<Mode> d;
    d.insert(d.end(), an.H.begin(), an.H.end());
    d.insert(d.end(), an.M.begin(), an.M.end());
    d.insert(d.end(), an.N.begin(), an.N.end());
    std::stable_sort(d.begin(), d.end(), [](const Mode& a, const Mode& b) {
        return (a.sD < 0 ? -a.sD : a.sD) < (b.sD < 0 ? -b.sD : b.sD);
    });
    g->nD = (int)d.size();
    g->nK = (int)an.K.size();
    g->sizeD = an.sizeH * an.sizeM * an.sizeN;
    g->sizeK = an.sizeK;
    for (int i = 0; i < g->nD; ++i) {
        g->dExt[i] = d[i].extent; g->dSA[i] = d[i].sA; g->dSB[i] = d[i].sB; g->dSD[i] = d[i].sD;
    }
    for (int i = 0; i < g->nK; ++i) {
        g->kExt[i] = an.K[i].extent; g->kSA[i] = an.K[i].sA; g->kSB[i] = an.K[i].sB;
    }
    g->opA = an.opA; g->opB = an.opB; g->opC = an.opC;
}

// The wide tables are padded so that every compiled tile shape finds a whole number of its tiles
// in them (kernels index rows and columns of a ragged last tile without a mask): the padding unit
// is the least common multiple of the shapes' extents (tiles of 256 and of 96: 768).
void table_units(int dtype, int64_t* unitM, int64_t* unitN, int64_t* unitK) {
    auto lcm = [](int64_t a, int64_t b) {
        int64_t x = a, y = b;
        while (y) { const int64_t t = x % y; x = y; y = t; }
        return a / x * b;
    };
    *unitM = *unitN = 256;
    *unitK = 64;
    for (int v = 0; v < gett_num_variants(dtype); ++v) {
        const GettVariant s = gett_variant(dtype, v);
        *unitM = lcm(*unitM, s.mt_m);
        *unitN = lcm(*unitN, s.mt_n);
        *unitK = lcm(*unitK, s.kt);
    }
}

tcx_error_t build_tables(Product* p) {
    const Analysis& an = p->an;
    int64_t unitM, unitN, unitK;
    table_units(an.dtype, &unitM, &unitN, &unitK);
    const int64_t padM = round_up(an.sizeM, unitM), padN = round_up(an.sizeN, unitN), padK = round_up(an.sizeK, unitK);
    try {
        p->tables[0] = offset_table(an.M, 0, padM);
        p->tables[1] = offset_table(an.K, 0, padK);
        p->tables[2] = offset_table(an.N, 1, padN);
        p->tables[3] = offset_table(an.K, 1, padK);
        p->tables[4] = offset_table(an.M, 2, padM);
        p->tables[5] = offset_table(an.N, 2, padN);
    } catch (const std::bad_alloc&) {
        return TCX_ERR_ALLOC;
    }
    if (!p->handle.has_device) return TCX_SUCCESS;
    size_t total = 0;
    for (int i = 0; i < 6; ++i) { p->dev_offset[i] = total; total += p->tables[i].size(); }
    if (hipMalloc((void**)&p->dev_tables, total * sizeof(int64_t)) != hipSuccess) {
        p->dev_tables = nullptr;
        (void)hipGetLastError();
        return TCX_ERR_ALLOC;
    }
    for (int i = 0; i < 6; ++i)
        if (hipMemcpy(p->dev_tables + p->dev_offset[i], p->tables[i].data(), p->tables[i].size() * sizeof(int64_t),
                      hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(p->dev_tables);
            p->dev_tables = nullptr;
            return TCX_ERR_LAUNCH;
        }
    return TCX_SUCCESS;
}

// Bytes of partial sums one execution of the plan writes (0: none, or summed inside the workgroup).
size_t partials_need(const Product& p) {
    if (p.an.path != TCX_PATH_GETT_MFMA || p.splitK <= 1) return 0;
    const GettVariant s = gett_variant(p.an.dtype, p.variant);
    if (p.splitK == 2 && s.pair_in_lds) return 0;
    const size_t real_bytes = (size_t)compute_real_bytes(p.an.dtype, p.an.precision);
    return (size_t)tiles_of(p.an, s) * (size_t)p.splitK * (size_t)s.acc_reals * real_bytes;
}
size_t align256(size_t n) { return (n + 255) / 256 * 256; }
// Bytes of a pre-reduced operand (Sec. "Case 4"), 0 if the operand is read as it is.
size_t reduced_bytes(const Product& p, const Reduction& r) {
    return r.active ? align256((size_t)r.count * (size_t)elem_bytes_of(p.an.dtype)) : 0;
}
// Workspace of one execution: [partial sums][reduced A][reduced B], each part 256-byte aligned.
size_t workspace_need(const Product& p) {
    return align256(partials_need(p)) + reduced_bytes(p, p.an.redA) + reduced_bytes(p, p.an.redB);
}

// Grow the executor's workspace to `need` bytes.  hipFree waits for the work that still uses the
// old buffer.  Caller holds e->mu.
tcx_error_t grow_workspace(Executor* e, size_t need) {
    if (need <= e->workspace_bytes) return TCX_SUCCESS;
    if (e->workspace) { (void)hipFree(e->workspace); e->workspace = nullptr; e->workspace_bytes = 0; }
    if (hipMalloc(&e->workspace, need) != hipSuccess) {
        (void)hipGetLastError();
        e->workspace = nullptr;
        return TCX_ERR_ALLOC;
    }
    e->workspace_bytes = need;
    return TCX_SUCCESS;
}

int elem_bytes(int dtype) { return elem_bytes_of(dtype); }

// Gather tables of the LDS-staged tiled kernels.  An operand element's address is split as
//   base(workgroup) + rowbase[tile] + { kofs[k]  |  kbase[slab] + krel[k] } + rowrel[row],
// all in bytes, where rowbase / kbase are the smallest offsets inside a tile's rows / a slab's
// contracted indices.  rowrel and krel are then small non-negative numbers and fit 32 bits
// (checked here), so a load is "64-bit scalar base + 32-bit per-lane offset": no 64-bit vector
// arithmetic and half the registers per offset.  kofs serves operands whose lanes run along the
// rows (one k per wave: its offset is a scalar); kbase + krel serves lanes that run along k.
struct NarrowOperand {
    std::vector<uint32_t> rowrel, krel;
    std::vector<int64_t> rowbase, kofs, kbase;
    bool periodic = true;      // every whole slab has the relative k offsets of the first
};

bool narrow_operand(const std::vector<int64_t>& rows, int64_t nrows, int mt, const std::vector<int64_t>& ks, int64_t nk,
                    int kt, int64_t esize, NarrowOperand* out) {
    const int64_t tiles = (nrows + mt - 1) / mt, slabs = (nk + kt - 1) / kt;
    out->rowrel.assign((size_t)(tiles * mt), 0);
    out->rowbase.assign((size_t)tiles, 0);
    out->krel.assign((size_t)(slabs * kt), 0);
    out->kbase.assign((size_t)slabs, 0);
    out->kofs.assign((size_t)(slabs * kt), 0);
    uint64_t max_row = 0, max_k = 0;
    for (int64_t t = 0; t < tiles; ++t) {
        const int64_t lo = t * mt, hi = std::min(nrows, lo + mt);
        int64_t base = rows[(size_t)lo];
        for (int64_t r = lo; r < hi; ++r) base = std::min(base, rows[(size_t)r]);
        out->rowbase[(size_t)t] = base * esize;
        for (int64_t r = lo; r < lo + mt; ++r) {                 // rows past the end repeat the tile's first row
            const uint64_t rel = (uint64_t)(rows[(size_t)(r < hi ? r : lo)] - base) * (uint64_t)esize;
            if (rel > 0xffffffffull) return false;
            out->rowrel[(size_t)r] = (uint32_t)rel;
            max_row = std::max(max_row, rel);
        }
    }
    for (int64_t sl = 0; sl < slabs; ++sl) {
        const int64_t lo = sl * kt, hi = std::min(nk, lo + kt);
        int64_t base = ks[(size_t)lo];
        for (int64_t k = lo; k < hi; ++k) base = std::min(base, ks[(size_t)k]);
        out->kbase[(size_t)sl] = base * esize;
        for (int64_t k = lo; k < lo + kt; ++k) {                 // indices past the end repeat the slab's first
            const int64_t off = ks[(size_t)(k < hi ? k : lo)];
            const uint64_t rel = (uint64_t)(off - base) * (uint64_t)esize;
            if (rel > 0xffffffffull) return false;
            out->krel[(size_t)k] = (uint32_t)rel;
            out->kofs[(size_t)k] = off * esize;
            max_k = std::max(max_k, rel);
        }
    }
    out->periodic = true;
    for (int64_t k = kt; k < nk / kt * kt && out->periodic; ++k)        // whole slabs only
        if (out->krel[(size_t)k] != out->krel[(size_t)(k % kt)]) out->periodic = false;
    return max_row + max_k <= 0xffffffffull;                     // the kernel adds the two in 32 bits
}

// Builds the narrow tables for tile shape `variant`; TCX_ERR_PLAN_REFUSED if a tile of that
// shape spans 4 GB or more of an operand.
tcx_error_t build_narrow(Product* p, int variant) {
    const GettVariant s = gett_variant(p->an.dtype, variant);
    if (!gett_available(p->an.dtype, p->an.precision, variant) || !batch_lanes_ok(p->an, s)) return TCX_ERR_PLAN_REFUSED;
    if (p->narrow_variant == variant) return TCX_SUCCESS;
    const int64_t es = elem_bytes(p->an.dtype);
    NarrowOperand a, b;
    try {
        if (!narrow_operand(p->tables[0], p->an.sizeM, s.mt_m, p->tables[1], p->an.sizeK, s.kt, es, &a) ||
            !narrow_operand(p->tables[2], p->an.sizeN, s.mt_n, p->tables[3], p->an.sizeK, s.kt, es, &b))
            return TCX_ERR_PLAN_REFUSED;
        // the two-phase kernel precomputes the per-lane k offsets of an operand whose lanes run along k
        auto operand_ok = [&](bool k_fastest, bool periodic, int mt) {
            return k_fastest ? periodic : (mt % 64 == 0 && s.threads % mt == 0);
        };
        if (s.hl > 1) {
            // lanes run along the batches: both operands in the slab-periodic form, whole slabs of K
            if (!a.periodic || !b.periodic || p->an.sizeK % s.kt != 0) return TCX_ERR_PLAN_REFUSED;
        } else if (s.pingpong && (!operand_ok(p->an.a_k_fastest, a.periodic, s.mt_m) || !operand_ok(p->an.b_k_fastest, b.periodic, s.mt_n))) {
            return TCX_ERR_PLAN_REFUSED;
        }
        p->periodic[0] = a.periodic;
        p->periodic[1] = b.periodic;
        // Paired gather loads (8-byte elements, two-phase kernel with one tile per wave group):
        // whole tiles and slabs, slab-periodic k offsets, and a step ps (a power of two) along the
        // direction the operand's lanes run such that every element x with (x / ps) even and its
        // partner x + ps are contiguous, x being 16-byte aligned relative to the operand's pointer
        // (whose own alignment is looked at when the product is executed).  Returns ps, 0 if none.
        auto pair_step = [&](const NarrowOperand& o, bool k_fastest, int64_t nrows, int mt, int which) -> int {
            if (!o.periodic || nrows % mt != 0 || p->an.sizeK % s.kt != 0) return 0;
            for (const Mode& h : p->an.H)
                if ((which == 0 ? h.sA : h.sB) % 2 != 0) return 0;
            for (int64_t v : o.rowbase) if (v % 16 != 0) return 0;
            for (int64_t v : o.kbase) if (v % 16 != 0) return 0;
            const std::vector<uint32_t>& along = k_fastest ? o.krel : o.rowrel;
            const std::vector<uint32_t>& across = k_fastest ? o.rowrel : o.krel;
            for (uint32_t v : across) if (v % 16 != 0) return 0;
            const int unit = k_fastest ? s.kt : mt;               // pairs stay inside a slab / a tile
            for (int ps = 1; 2 * ps <= unit; ps *= 2) {
                if (unit % (2 * ps) != 0) break;
                bool ok = true;
                for (size_t x = 0; x < along.size() && ok; ++x)
                    if ((x / (size_t)ps) % 2 == 0) ok = along[x] % 16 == 0 && along[x + (size_t)ps] == along[x] + 8;
                if (ok) return ps;
            }
            return 0;
        };
        p->pair_step[0] = pair_step(a, p->an.a_k_fastest, p->an.sizeM, s.mt_m, 0);
        p->pair_step[1] = pair_step(b, p->an.b_k_fastest, p->an.sizeN, s.mt_n, 1);
        p->pairs = s.pingpong && s.dual && s.hl == 1 && es == 8 && p->pair_step[0] > 0 && p->pair_step[1] > 0;
    } catch (const std::bad_alloc&) {
        return TCX_ERR_ALLOC;
    }
    p->narrow_variant = -1;
    if (!p->handle.has_device) return TCX_SUCCESS;
    if (p->dev_narrow) { (void)hipFree(p->dev_narrow); p->dev_narrow = nullptr; }
    const void* src[10] = {a.rowrel.data(), a.rowbase.data(), a.kofs.data(), a.krel.data(), a.kbase.data(),
                           b.rowrel.data(), b.rowbase.data(), b.kofs.data(), b.krel.data(), b.kbase.data()};
    const size_t bytes[10] = {a.rowrel.size() * 4, a.rowbase.size() * 8, a.kofs.size() * 8, a.krel.size() * 4, a.kbase.size() * 8,
                              b.rowrel.size() * 4, b.rowbase.size() * 8, b.kofs.size() * 8, b.krel.size() * 4, b.kbase.size() * 8};
    size_t total = 0;
    for (int i = 0; i < 10; ++i) { p->narrow_off[i] = total; total += (bytes[i] + 255) / 256 * 256; }
    if (hipMalloc((void**)&p->dev_narrow, total) != hipSuccess) {
        p->dev_narrow = nullptr;
        (void)hipGetLastError();
        return TCX_ERR_ALLOC;
    }
    for (int i = 0; i < 10; ++i)
        if (bytes[i] && hipMemcpy(p->dev_narrow + p->narrow_off[i], src[i], bytes[i], hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(p->dev_narrow);
            p->dev_narrow = nullptr;
            return TCX_ERR_LAUNCH;
        }
    p->narrow_variant = variant;
    return TCX_SUCCESS;
}

// Everything the tiled path needs for the plan's current tile shape.  If a tile of that shape
// spans too much of an operand for 32-bit relative offsets, smaller shapes are tried.
tcx_error_t prepare_tiled(Product* p) {
    if (p->tables[0].empty()) {
        const tcx_error_t err = build_tables(p);
        if (err != TCX_SUCCESS) return err;
    }
    // order: the plan's shape, the shape it names as its stand-in, then the others as the cost
    // model ranks them (each with its own best split count)
    tcx_error_t err = TCX_ERR_PLAN_REFUSED;
    const int first = p->variant, second = gett_variant(p->an.dtype, first).fallback;
    std::vector<PlanChoice> order = {{0.0, first, p->splitK}};
    if (second >= 0) order.push_back({0.0, second, 1});
    for (const PlanChoice& c : rank_plans(p->an, p->handle.num_cu))
        if (c.variant != first && c.variant != second) order.push_back(c);
    for (const PlanChoice& c : order) {
        err = !gett_available(p->an.dtype, p->an.precision, c.variant) ? TCX_ERR_PLAN_REFUSED
              : gett_variant(p->an.dtype, c.variant).staged                ? build_narrow(p, c.variant)
                                                                           : TCX_SUCCESS;
        if (err == TCX_SUCCESS) {
            if (c.variant != p->variant) { p->variant = c.variant; p->splitK = c.splitK; }
            break;
        }
        if (err != TCX_ERR_PLAN_REFUSED) break;
    }
    if (err != TCX_SUCCESS) return err;
    p->an.variant = p->variant;
    return TCX_SUCCESS;
}

tcx_error_t build_stream(Product* p, bool allow_blocked = true) {
    if (p->dev_stream) { (void)hipFree(p->dev_stream); p->dev_stream = nullptr; }
    try {
        p->stream = plan_stream(p->an, elem_bytes(p->an.dtype), allow_blocked);
    } catch (const std::bad_alloc&) {
        return TCX_ERR_ALLOC;
    }
    if (!p->stream.ok) return TCX_ERR_PLAN_REFUSED;
    if (!p->handle.has_device) return TCX_SUCCESS;
    const StreamPlan& sp = p->stream;
    const size_t bytes[8] = {sp.rowAB.size() * sizeof(uint32_t), sp.dD.size() * sizeof(int64_t),
                             sp.itemsA.size() * sizeof(StreamItem), sp.itemsB.size() * sizeof(StreamItem),
                             sp.tabLo.size() * sizeof(int64_t), sp.tabHi.size() * sizeof(int64_t),
                             sp.laneA.size() * sizeof(int64_t), sp.laneB.size() * sizeof(int64_t)};
    const void* src[8] = {sp.rowAB.data(), sp.dD.data(), sp.itemsA.data(), sp.itemsB.data(), sp.tabLo.data(), sp.tabHi.data(),
                          sp.laneA.data(), sp.laneB.data()};
    size_t total = 0;
    for (int i = 0; i < 8; ++i) { p->stream_off[i] = total; total += (bytes[i] + 255) / 256 * 256; }
    if (hipMalloc((void**)&p->dev_stream, total) != hipSuccess) {
        p->dev_stream = nullptr;
        (void)hipGetLastError();
        return TCX_ERR_ALLOC;
    }
    for (int i = 0; i < 8; ++i)
        if (bytes[i] && hipMemcpy(p->dev_stream + p->stream_off[i], src[i], bytes[i], hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(p->dev_stream);
            p->dev_stream = nullptr;
            return TCX_ERR_LAUNCH;
        }
    return TCX_SUCCESS;
}

tcx_error_t put(const void* src, size_t need, void* value, size_t* nbytes) {
    if (!nbytes) return TCX_ERR_NULL_ARG;
    if (!value || *nbytes < need) { *nbytes = need; return value ? TCX_ERR_BUFFER_TOO_SMALL : TCX_ERR_NULL_ARG; }
    std::memcpy(value, src, need);
    *nbytes = need;
    return TCX_SUCCESS;
}
tcx_error_t put_i64(int64_t v, void* value, size_t* nbytes) { return put(&v, sizeof v, value, nbytes); }
tcx_error_t put_modes(const std::vector<Mode>& m, void* value, size_t* nbytes) {
    std::vector<int64_t> flat;
    for (const Mode& x : m) { flat.push_back(x.extent); flat.push_back(x.sA); flat.push_back(x.sB); flat.push_back(x.sD); }
    if (flat.empty()) { if (!nbytes) return TCX_ERR_NULL_ARG; *nbytes = 0; return TCX_SUCCESS; }
    return put(flat.data(), flat.size() * sizeof(int64_t), value, nbytes);
}

const char* const kMessages[] = {
    "success",
    "a required pointer argument is NULL",
    "invalid, destroyed or mistyped object handle",
    "unsupported data type",
    "number of modes is negative or exceeds TCX_MAX_MODES",
    "an extent is not positive",
    "modes that share a label have different extents",
    "tensor C does not have tensor D's labels, extents and strides",
    "two index tuples of tensor D address the same element",
    "a label occurs in only one of A, B, D (isolated index: reduction or broadcast is not supported)",
    "the four tensors do not share one data type",
    "unsupported element-wise operation (op value unknown, or opD is not the identity)",
    "unsupported computational precision",
    "memory allocation failed",
    "the HIP runtime reported an error; query TCX_KEY_HIP_ERROR on the status object",
    "the handle has no usable gfx950 device; plans can be built but not executed",
    "an index range or offset exceeds what the kernels can address",
    "unknown key",
    "value buffer too small",
    "this plan cannot take the requested kernel path, tile shape or split of the contracted range",
    "the product needs more scratch memory than the library's fixed buffer holds",
};

}  // namespace
}  // namespace tcx

using namespace tcx;

extern "C" {

tcx_error_t tcx_create_handle(tcx_handle_t* out) {
    if (!out) return TCX_ERR_NULL_ARG;
    Handle* h = new (std::nothrow) Handle;
    if (!h) return TCX_ERR_ALLOC;
    int count = 0;
    if (hipGetDeviceCount(&count) == hipSuccess && count > 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
            std::strncmp(prop.gcnArchName, "gfx950", 6) == 0) {
            h->device = dev;
            h->has_device = true;
            h->num_cu = prop.multiProcessorCount;
            h->scratch = scratch_on(dev);
            h->one64 = g_one64_ptr[dev];
            h->one32 = g_one32_ptr[dev];
            h->one16 = g_one16_ptr[dev];
        }
    }
    (void)hipGetLastError();
    *out = publish(h, MAGIC_HANDLE);
    return TCX_SUCCESS;
}

tcx_error_t tcx_destroy_handle(tcx_handle_t* handle) { return retire<Handle>(handle, MAGIC_HANDLE); }

tcx_error_t tcx_handle_has_device(tcx_handle_t handle, int32_t* out) {
    if (!out) return TCX_ERR_NULL_ARG;
    Handle* h = lookup<Handle>(handle, MAGIC_HANDLE);
    if (!h) return TCX_ERR_INVALID_HANDLE;
    *out = h->has_device ? 1 : 0;
    return TCX_SUCCESS;
}

tcx_error_t tcx_create_executor(tcx_handle_t handle, void* hip_stream, tcx_executor_t* out) {
    if (!out) return TCX_ERR_NULL_ARG;
    Handle* h = lookup<Handle>(handle, MAGIC_HANDLE);
    if (!h) return TCX_ERR_INVALID_HANDLE;
    Executor* e = new (std::nothrow) Executor;
    if (!e) return TCX_ERR_ALLOC;
    e->handle = *h;
    e->stream = (hipStream_t)hip_stream;
    *out = publish(e, MAGIC_EXEC);
    return TCX_SUCCESS;
}

tcx_error_t tcx_destroy_executor(tcx_executor_t* executor) {
    if (!executor) return TCX_ERR_NULL_ARG;
    Executor* e = lookup<Executor>(*executor, MAGIC_EXEC);
    if (!e) return TCX_ERR_INVALID_HANDLE;
    if (e->workspace) { (void)hipFree(e->workspace); e->workspace = nullptr; e->workspace_bytes = 0; }
    return retire<Executor>(executor, MAGIC_EXEC);
}

tcx_error_t tcx_create_tensor_info(tcx_handle_t handle, tcx_dtype_t dtype, int32_t nmode, const int64_t* extents,
                                   const int64_t* strides, tcx_tensor_info_t* out) {
    if (!out) return TCX_ERR_NULL_ARG;
    if (!lookup<Handle>(handle, MAGIC_HANDLE)) return TCX_ERR_INVALID_HANDLE;
    if (!valid_dtype((int)dtype)) return TCX_ERR_BAD_DTYPE;
    if (nmode < 0 || nmode > TCX_MAX_MODES) return TCX_ERR_BAD_NMODE;
    if (nmode > 0 && (!extents || !strides)) return TCX_ERR_NULL_ARG;
    for (int i = 0; i < nmode; ++i)
        if (extents[i] <= 0) return TCX_ERR_BAD_EXTENT;
    Info* t = new (std::nothrow) Info;
    if (!t) return TCX_ERR_ALLOC;
    t->desc.dtype = dtype;
    t->desc.extent.assign(extents, extents + nmode);
    t->desc.stride.assign(strides, strides + nmode);
    *out = publish(t, MAGIC_INFO);
    return TCX_SUCCESS;
}

tcx_error_t tcx_destroy_tensor_info(tcx_tensor_info_t* info) { return retire<Info>(info, MAGIC_INFO); }

tcx_error_t tcx_tensor_info_get(tcx_tensor_info_t info, tcx_dtype_t* dtype, int32_t* nmode, int64_t* extents,
                                int64_t* strides) {
    Info* t = lookup<Info>(info, MAGIC_INFO);
    if (!t) return TCX_ERR_INVALID_HANDLE;
    if (dtype) *dtype = (tcx_dtype_t)t->desc.dtype;
    if (nmode) *nmode = (int32_t)t->desc.extent.size();
    for (size_t i = 0; i < t->desc.extent.size(); ++i) {
        if (extents) extents[i] = t->desc.extent[i];
        if (strides) strides[i] = t->desc.stride[i];
    }
    return TCX_SUCCESS;
}

// Routing.  Low arithmetic intensity goes to the streaming path when its tile re-reads little
// operand data per output; otherwise the tiled MFMA path if the free index space can fill MFMA
// tiles; otherwise streaming if it applies at all; else generic.
tcx_error_t route(Product* p) {
    tcx_error_t err = TCX_SUCCESS;
    p->an.path = p->analysed_path;
    const bool low_ai = stream_preferred(p->an, elem_bytes(p->an.dtype));
    const bool stream_ok = low_ai && build_stream(p) == TCX_SUCCESS;
    if (stream_ok && (p->stream.staged_per_output <= 0.5 || p->an.path != TCX_PATH_GETT_MFMA)) {
        p->an.path = TCX_PATH_BANDWIDTH;
    } else if (p->an.path == TCX_PATH_GETT_MFMA) {
        choose_plan(p->an, p->handle.num_cu, &p->variant, &p->splitK);
        err = prepare_tiled(p);
        if (err == TCX_ERR_PLAN_REFUSED) { err = TCX_SUCCESS; p->an.path = TCX_PATH_GENERIC; }
    }
    p->an.variant = p->variant;
    return err;
}

tcx_error_t tcx_create_product(tcx_handle_t handle, tcx_op_t opA, tcx_tensor_info_t A, const int64_t* labelsA,
                               tcx_op_t opB, tcx_tensor_info_t B, const int64_t* labelsB, tcx_op_t opC,
                               tcx_tensor_info_t C, const int64_t* labelsC, tcx_op_t opD, tcx_tensor_info_t D,
                               const int64_t* labelsD, tcx_prec_t precision, tcx_product_t* out) {
    if (!out) return TCX_ERR_NULL_ARG;
    Handle* h = lookup<Handle>(handle, MAGIC_HANDLE);
    Info* a = lookup<Info>(A, MAGIC_INFO);
    Info* b = lookup<Info>(B, MAGIC_INFO);
    Info* c = lookup<Info>(C, MAGIC_INFO);
    Info* d = lookup<Info>(D, MAGIC_INFO);
    if (!h || !a || !b || !c || !d) return TCX_ERR_INVALID_HANDLE;
    if ((!labelsA && !a->desc.extent.empty()) || (!labelsB && !b->desc.extent.empty()) ||
        (!labelsC && !c->desc.extent.empty()) || (!labelsD && !d->desc.extent.empty()))
        return TCX_ERR_NULL_ARG;
    Product* p = new (std::nothrow) Product;
    if (!p) return TCX_ERR_ALLOC;
    p->handle = *h;
    tcx_error_t err = analyse(a->desc, labelsA, b->desc, labelsB, c->desc, labelsC, d->desc, labelsD, (int)opA,
                              (int)opB, (int)opC, (int)opD, (int)precision, &p->an);
    if (err == TCX_SUCCESS) {
        fill_generic(p->an, &p->generic);
        p->analysed_path = p->an.path;
        err = route(p);
    }
    if (err != TCX_SUCCESS) { delete p; return err; }
    *out = publish(p, MAGIC_PRODUCT);
    return TCX_SUCCESS;
}

// Sec. "Unary and Binary Operations": C := alpha opA(A) + beta opB(B) read as the contraction
// alpha A * 1 + beta B with a rank-0 second operand, so labels of A that C lacks are summed
// (Case 4) and labels of C that A lacks broadcast (Case 5) through the same analysis and kernels.
tcx_error_t tcx_create_binary(tcx_handle_t handle, tcx_op_t opA, tcx_tensor_info_t A, const int64_t* labelsA, tcx_op_t opB,
                              tcx_tensor_info_t B, const int64_t* labelsB, tcx_op_t opC, tcx_tensor_info_t C,
                              const int64_t* labelsC, tcx_prec_t precision, tcx_product_t* out) {
    if (!out) return TCX_ERR_NULL_ARG;
    Handle* h = lookup<Handle>(handle, MAGIC_HANDLE);
    Info* a = lookup<Info>(A, MAGIC_INFO);
    Info* b = lookup<Info>(B, MAGIC_INFO);
    Info* c = lookup<Info>(C, MAGIC_INFO);
    if (!h || !a || !b || !c) return TCX_ERR_INVALID_HANDLE;
    if ((!labelsA && !a->desc.extent.empty()) || (!labelsB && !b->desc.extent.empty()) || (!labelsC && !c->desc.extent.empty()))
        return TCX_ERR_NULL_ARG;
    Product* p = new (std::nothrow) Product;
    if (!p) return TCX_ERR_ALLOC;
    p->handle = *h;
    p->kind = KIND_BINARY;
    TensorDesc one;
    one.dtype = a->desc.dtype;
    tcx_error_t err = analyse(a->desc, labelsA, one, nullptr, b->desc, labelsB, c->desc, labelsC, (int)opA, TCX_OP_IDENTITY,
                              (int)opB, (int)opC, (int)precision, &p->an);
    if (err == TCX_SUCCESS) {
        fill_generic(p->an, &p->generic);
        p->analysed_path = p->an.path;
        err = route(p);
    }
    if (err != TCX_SUCCESS) { delete p; return err; }
    *out = publish(p, MAGIC_PRODUCT);
    return TCX_SUCCESS;
}

// B := alpha opA(A): the binary operation with beta = 0; a unary operation has no distinct label
// subsets (A and B carry the same set of labels; repeated labels address diagonals).
tcx_error_t tcx_create_unary(tcx_handle_t handle, tcx_op_t opA, tcx_tensor_info_t A, const int64_t* labelsA, tcx_op_t opB,
                             tcx_tensor_info_t B, const int64_t* labelsB, tcx_prec_t precision, tcx_product_t* out) {
    if (!out) return TCX_ERR_NULL_ARG;
    Info* a = lookup<Info>(A, MAGIC_INFO);
    Info* b = lookup<Info>(B, MAGIC_INFO);
    if (!a || !b) return TCX_ERR_INVALID_HANDLE;
    if ((!labelsA && !a->desc.extent.empty()) || (!labelsB && !b->desc.extent.empty())) return TCX_ERR_NULL_ARG;
    for (size_t i = 0; i < a->desc.extent.size(); ++i)
        if (std::find(labelsB, labelsB + b->desc.extent.size(), labelsA[i]) == labelsB + b->desc.extent.size()) return TCX_ERR_ISOLATED_INDEX;
    for (size_t i = 0; i < b->desc.extent.size(); ++i)
        if (std::find(labelsA, labelsA + a->desc.extent.size(), labelsB[i]) == labelsA + a->desc.extent.size()) return TCX_ERR_ISOLATED_INDEX;
    const tcx_error_t err = tcx_create_binary(handle, opA, A, labelsA, TCX_OP_IDENTITY, B, labelsB, opB, B, labelsB, precision, out);
    if (err == TCX_SUCCESS) ((Product*)*out)->kind = KIND_UNARY;
    return err;
}

tcx_error_t tcx_destroy_product(tcx_product_t* product) {
    if (!product) return TCX_ERR_NULL_ARG;
    Product* p = lookup<Product>(*product, MAGIC_PRODUCT);
    if (!p) return TCX_ERR_INVALID_HANDLE;
    if (p->dev_tables) { (void)hipFree(p->dev_tables); p->dev_tables = nullptr; }
    if (p->dev_narrow) { (void)hipFree(p->dev_narrow); p->dev_narrow = nullptr; }
    if (p->dev_stream) { (void)hipFree(p->dev_stream); p->dev_stream = nullptr; }
    return retire<Product>(product, MAGIC_PRODUCT);
}

tcx_error_t tcx_product_get(tcx_product_t product, int32_t key, void* value, size_t* nbytes) {
    Product* p = lookup<Product>(product, MAGIC_PRODUCT);
    if (!p) return TCX_ERR_INVALID_HANDLE;
    const Analysis& an = p->an;
    const bool tiled = an.path == TCX_PATH_GETT_MFMA;
    const GettVariant s = tiled ? gett_variant(an.dtype, p->variant) : GettVariant{0, 0, 0, 256, 0.f, 0, false, false, -1, false, false, 1};
    switch (key) {
        case TCX_KEY_PATH: return put_i64(an.path, value, nbytes);
        case TCX_KEY_SIZE_H: return put_i64(an.sizeH, value, nbytes);
        case TCX_KEY_SIZE_M: return put_i64(an.sizeM, value, nbytes);
        case TCX_KEY_SIZE_N: return put_i64(an.sizeN, value, nbytes);
        case TCX_KEY_SIZE_K: return put_i64(an.sizeK, value, nbytes);
        case TCX_KEY_NMODES_H: return put_i64((int64_t)an.H.size(), value, nbytes);
        case TCX_KEY_NMODES_M: return put_i64((int64_t)an.M.size(), value, nbytes);
        case TCX_KEY_NMODES_N: return put_i64((int64_t)an.N.size(), value, nbytes);
        case TCX_KEY_NMODES_K: return put_i64((int64_t)an.K.size(), value, nbytes);
        case TCX_KEY_TILE_M: return put_i64(an.path == TCX_PATH_BANDWIDTH ? p->stream.tile : s.mt_m, value, nbytes);
        case TCX_KEY_TILE_N: return put_i64(an.path == TCX_PATH_BANDWIDTH ? p->stream.regA * p->stream.regB : s.mt_n, value, nbytes);
        case TCX_KEY_TILE_K: return put_i64(s.kt, value, nbytes);
        case TCX_KEY_GRID:
            if (an.path == TCX_PATH_BANDWIDTH) {
                const int need = (int)((std::max(p->stream.itemsA.size(), p->stream.itemsB.size()) + kStreamThreads - 1) / kStreamThreads);
                return put_i64(stream_grid(p->stream.blocked, p->stream.direct, need, p->stream.num_tiles, p->handle.num_cu), value, nbytes);
            }
            return put_i64(tiled ? (s.dual ? (tiles_of(an, s) * p->splitK + 1) / 2 : tiles_of(an, s) * p->splitK)
                                 : (an.sizeH * an.sizeM * an.sizeN + 255) / 256, value, nbytes);
        case TCX_KEY_BLOCK: return put_i64(s.threads * (tiled && s.dual ? 2 : 1), value, nbytes);
        case TCX_KEY_A_K_FASTEST: return put_i64(an.a_k_fastest, value, nbytes);
        case TCX_KEY_B_K_FASTEST: return put_i64(an.b_k_fastest, value, nbytes);
        case TCX_KEY_D_N_FASTEST: return put_i64(an.d_n_fastest, value, nbytes);
        case TCX_KEY_SPLIT_K: return put_i64(tiled ? p->splitK : 1, value, nbytes);
        case TCX_KEY_PACED_LOADS: return put_i64(an.path == TCX_PATH_BANDWIDTH && p->stream.paced ? 1 : 0, value, nbytes);
        case TCX_KEY_LAUNCHES: {
            const int64_t reductions = (an.redA.active ? 1 : 0) + (an.redB.active ? 1 : 0);      // Case 4 pre-reductions
            if (!tiled) return put_i64(1 + reductions, value, nbytes);
            const int64_t items = tiles_of(an, s) * p->splitK;
            const int64_t blocks = s.dual ? (items + 1) / 2 : items;
            const int64_t round = round_size_of(*p, s);
            const bool second_kernel = p->splitK > 1 && !(p->splitK == 2 && s.pair_in_lds);
            return put_i64((round > 0 && p->splitK == 1 && blocks > round ? (blocks + round - 1) / round : 1) + (second_kernel ? 1 : 0) + reductions,
                           value, nbytes);
        }
        case TCX_KEY_GATHER_WIDTH: return put_i64(tiled && s.pingpong && s.dual && p->pairs ? 2 : 1, value, nbytes);
        case TCX_KEY_WORKSPACE_BYTES: return put_i64((int64_t)workspace_need(*p), value, nbytes);
        case TCX_KEY_PRECISION: return put_i64(an.precision, value, nbytes);
        case TCX_KEY_TABLE_ENTRIES: {
            const int64_t n[3] = {(int64_t)p->tables[0].size(), (int64_t)p->tables[2].size(), (int64_t)p->tables[1].size()};
            return put(n, sizeof n, value, nbytes);
        }
        case TCX_KEY_VARIANT:
            return put_i64(tiled ? p->variant : (an.path == TCX_PATH_BANDWIDTH && p->stream.blocked) ? 1 : 0, value, nbytes);
        case TCX_KEY_MODES_M: return put_modes(an.M, value, nbytes);
        case TCX_KEY_MODES_N: return put_modes(an.N, value, nbytes);
        case TCX_KEY_MODES_K: return put_modes(an.K, value, nbytes);
        case TCX_KEY_MODES_H: return put_modes(an.H, value, nbytes);
        default: return TCX_ERR_BAD_KEY;
    }
}

tcx_error_t tcx_product_set(tcx_product_t product, int32_t key, const void* value, size_t nbytes) {
    Product* p = lookup<Product>(product, MAGIC_PRODUCT);
    if (!p) return TCX_ERR_INVALID_HANDLE;
    if (!value) return TCX_ERR_NULL_ARG;
    if (nbytes != sizeof(int64_t)) return TCX_ERR_BUFFER_TOO_SMALL;
    int64_t v;
    std::memcpy(&v, value, sizeof v);
    if (key == TCX_KEY_FORCE_PATH) {
        if (v == TCX_PATH_GENERIC) { p->an.path = TCX_PATH_GENERIC; return TCX_SUCCESS; }
        if (v == TCX_PATH_GETT_MFMA) {
            if (gett_num_variants(p->an.dtype) == 0 || (int)p->an.H.size() > kMaxHModes) return TCX_ERR_PLAN_REFUSED;
            if (p->tables[0].empty()) choose_plan(p->an, p->handle.num_cu, &p->variant, &p->splitK);
            const tcx_error_t err = prepare_tiled(p);
            if (err != TCX_SUCCESS) return err;
            p->an.path = TCX_PATH_GETT_MFMA;
            return TCX_SUCCESS;
        }
        if (v == TCX_PATH_BANDWIDTH) {
            if (!p->stream.ok) {
                const tcx_error_t err = build_stream(p);
                if (err != TCX_SUCCESS) return err;
            }
            p->an.path = TCX_PATH_BANDWIDTH;
            return TCX_SUCCESS;
        }
        return TCX_ERR_PLAN_REFUSED;
    }
    if (key == TCX_KEY_VARIANT && p->an.path == TCX_PATH_BANDWIDTH) {
        // 0: flat tiles only, 1: register-blocked tiles where the shape allows them
        if (v != 0 && v != 1) return TCX_ERR_PLAN_REFUSED;
        return build_stream(p, v == 1);
    }
    if (key == TCX_KEY_VARIANT) {
        if (p->an.path != TCX_PATH_GETT_MFMA || v < 0 || v >= gett_num_variants(p->an.dtype)) return TCX_ERR_PLAN_REFUSED;
        if (!gett_available(p->an.dtype, p->an.precision, (int)v)) return TCX_ERR_PLAN_REFUSED;
        if (gett_variant(p->an.dtype, (int)v).staged) {
            const tcx_error_t err = build_narrow(p, (int)v);
            if (err != TCX_SUCCESS) return err;
        }
        p->variant = (int)v;
        p->an.variant = (int)v;
        p->splitK = 1;                       // a forced shape starts unsplit; set TCX_KEY_SPLIT_K afterwards
        return TCX_SUCCESS;
    }
    if (key == TCX_KEY_SPLIT_K) {
        if (p->an.path != TCX_PATH_GETT_MFMA || v < 1 || v > 64) return TCX_ERR_PLAN_REFUSED;
        const GettVariant sh = gett_variant(p->an.dtype, p->variant);
        if (sh.hl > 1 && v > 1) return TCX_ERR_PLAN_REFUSED;          // the batch-lane kernel keeps K whole
        const int64_t nk = (p->an.sizeK + sh.kt - 1) / sh.kt;
        const int64_t per = (nk + v - 1) / v;
        p->splitK = (int)((nk + per - 1) / per);        // no part may be empty
        return TCX_SUCCESS;
    }
    return TCX_ERR_BAD_KEY;
}

}  // extern "C"

namespace {
// Body of both execute calls.  fixed_scratch: partial sums go to the library's fixed per-device
// buffer and nothing is allocated, neither on the device nor (no status object) on the host.
tcx_error_t run_product(tcx_product_t product, tcx_executor_t executor, tcx_status_t* status, const void* alpha,
                        const void* A, const void* B, const void* beta, const void* C, void* D, bool fixed_scratch,
                        int kind = KIND_CONTRACTION) {
    Product* p = lookup<Product>(product, MAGIC_PRODUCT);
    Executor* e = lookup<Executor>(executor, MAGIC_EXEC);
    if (!p || !e || p->kind != kind) return TCX_ERR_INVALID_HANDLE;
    if (!alpha || !beta || !D) return TCX_ERR_NULL_ARG;
    if (kind != KIND_CONTRACTION) {
        const int rb = real_bytes_of(p->an.dtype);
        B = rb == 4 ? e->handle.one32 : rb == 8 ? e->handle.one64 : e->handle.one16;
        if (B && p->an.dtype == TCX_BF16) B = (const char*)B + 16;
    }
    Scalars s{0, 0, 0, 0};
    switch (p->an.dtype) {
        case TCX_F32:
        case TCX_F16:
        case TCX_BF16:                       // 16-bit tensors take their scalars as floats
            s.alpha_re = *(const float*)alpha; s.beta_re = *(const float*)beta; break;
        case TCX_F64: s.alpha_re = *(const double*)alpha; s.beta_re = *(const double*)beta; break;
        case TCX_C64:
            s.alpha_re = ((const float*)alpha)[0]; s.alpha_im = ((const float*)alpha)[1];
            s.beta_re = ((const float*)beta)[0]; s.beta_im = ((const float*)beta)[1];
            break;
        default:
            s.alpha_re = ((const double*)alpha)[0]; s.alpha_im = ((const double*)alpha)[1];
            s.beta_re = ((const double*)beta)[0]; s.beta_im = ((const double*)beta)[1];
    }
    const bool read_ab = s.alpha_re != 0 || s.alpha_im != 0;
    const bool read_c = s.beta_re != 0 || s.beta_im != 0;
    if ((read_ab && (!A || (!B && kind == KIND_CONTRACTION))) || (read_c && !C)) return TCX_ERR_NULL_ARG;
    if (!p->handle.has_device || !e->handle.has_device) return TCX_ERR_NO_DEVICE;
    if (read_ab && !B) return TCX_ERR_LAUNCH;                 // the device constant 1 could not be located when the handle was made

    Status st;
    int hip_err = 0;
    int64_t grid = 0;
    int block = 0;
    // Workspace of this execution: leased from the executor (executions on its stream run in order
    // and may share it) or, for the call that may not allocate, the library's fixed buffer.
    char* ws = nullptr;
    bool split_ok = true;
    std::unique_lock<std::mutex> lease;      // held until every launch that uses the workspace is enqueued
    const size_t need_partials = align256(partials_need(*p));
    const size_t need_red = read_ab ? reduced_bytes(*p, p->an.redA) + reduced_bytes(*p, p->an.redB) : 0;
    if (need_partials + need_red > 0) {
        if (fixed_scratch) {
            if (need_partials + need_red > (size_t)TCX_SCRATCH_BYTES || !e->handle.scratch) return TCX_ERR_SCRATCH_TOO_SMALL;
            ws = (char*)e->handle.scratch;                   // every byte read is written first by this execution
        } else {
            // Two host threads may execute through one executor: the one that grows the workspace
            // frees the old buffer (hipFree waits for the work already enqueued), so the other must
            // not be between taking the pointer and enqueuing its kernels.  The lock also makes the
            // order of enqueuing the order in which executions pass the buffer on.
            lease = std::unique_lock<std::mutex>(e->mu);
            if (grow_workspace(e, need_partials + need_red) == TCX_SUCCESS) ws = (char*)e->workspace;
            else if (need_red > 0) return TCX_ERR_ALLOC;     // a reduced operand has to live somewhere
            else split_ok = false;                           // no memory for partial sums: run unsplit
        }
    }
    // Sec. "Case 4": operands with isolated labels are summed over them first; the contraction
    // reads the dense result.
    if (read_ab && ws) {
        char* at = ws + need_partials;
        for (int which = 0; which < 2; ++which) {
            const Reduction& r = which == 0 ? p->an.redA : p->an.redB;
            if (!r.active) continue;
            ReduceArgs ra{};
            ra.src = which == 0 ? A : B;
            ra.dst = at;
            ra.nKeep = (int32_t)r.keepExt.size(); ra.nSum = (int32_t)r.sumExt.size();
            ra.count = r.count; ra.sumCount = 1;
            for (int i = 0; i < ra.nKeep; ++i) { ra.keepExt[i] = r.keepExt[i]; ra.keepSrc[i] = r.keepSrc[i]; }
            for (int i = 0; i < ra.nSum; ++i) { ra.sumExt[i] = r.sumExt[i]; ra.sumSrc[i] = r.sumSrc[i]; ra.sumCount *= r.sumExt[i]; }
            const int err = launch_reduce(p->an.dtype, p->an.precision, ra, (void*)e->stream);
            if (err != 0) {
                st.hip_error = err;
                if (status) { Status* so = new (std::nothrow) Status(st); *status = so ? publish(so, MAGIC_STATUS) : 0; }
                return TCX_ERR_LAUNCH;
            }
            (which == 0 ? A : B) = at;
            at += reduced_bytes(*p, r);
        }
    }
    const bool tiled = p->an.path == TCX_PATH_GETT_MFMA && read_ab && p->dev_tables &&
                       (!gett_variant(p->an.dtype, p->variant).staged || (p->dev_narrow && p->narrow_variant == p->variant));
    const bool streamed = p->an.path == TCX_PATH_BANDWIDTH && read_ab && p->dev_stream;
    if (streamed) {
        const StreamPlan& sp = p->stream;
        StreamArgs g{};
        g.A = A; g.B = B; g.C = C; g.D = D;
        g.rowAB = (const uint32_t*)(p->dev_stream + p->stream_off[0]);
        g.dD = (const int64_t*)(p->dev_stream + p->stream_off[1]);
        g.itemsA = (const StreamItem*)(p->dev_stream + p->stream_off[2]);
        g.itemsB = (const StreamItem*)(p->dev_stream + p->stream_off[3]);
        g.laneA = (const int64_t*)(p->dev_stream + p->stream_off[6]);
        g.laneB = (const int64_t*)(p->dev_stream + p->stream_off[7]);
        for (int i = 0; i < kStreamRegBlock; ++i) { g.aReg[i] = sp.aReg[i]; g.bReg[i] = sp.bReg[i]; g.aK[i] = sp.aK[i]; g.bK[i] = sp.bK[i]; }
        g.nItemsA = (int32_t)sp.itemsA.size(); g.nItemsB = (int32_t)sp.itemsB.size();
        g.tile = sp.tile; g.inner = sp.inner; g.chunk = sp.chunk; g.K = sp.K; g.rowsA = sp.rowsA; g.rowsB = sp.rowsB;
        g.regA = sp.regA; g.regB = sp.regB; g.rowStepA = sp.rowStepA; g.rowStepB = sp.rowStepB;
        for (int i = 0; i < kStreamRegBlock; ++i) { g.dRegA[i] = sp.dRegA[i]; g.dRegB[i] = sp.dRegB[i]; }
        g.split_extent = sp.split_extent; g.num_tiles = sp.num_tiles; g.outer_lo = sp.outer_lo;
        g.paced = sp.paced ? 1 : 0;
        g.tabLo = (const int64_t*)(p->dev_stream + p->stream_off[4]);
        g.tabHi = (const int64_t*)(p->dev_stream + p->stream_off[5]);
        g.s = s;
        g.opA = p->an.opA; g.opB = p->an.opB; g.opC = p->an.opC;
        g.read_c = read_c;
        hip_err = launch_stream(p->an.dtype, sp.blocked, sp.direct, g, sp.lds_bytes, p->handle.num_cu, (void*)e->stream, &grid, &block);
        st.path = TCX_PATH_BANDWIDTH;
        st.variant = sp.blocked ? 1 : 0;
        st.tile_m = sp.tile; st.tile_n = sp.regA * sp.regB; st.tile_k = sp.K;
    } else if (tiled) {
        const GettVariant v = gett_variant(p->an.dtype, p->variant);
        GettArgs g{};
        g.A = A; g.B = B; g.C = C; g.D = D;
        g.oAM = p->dev_tables + p->dev_offset[0]; g.oAK = p->dev_tables + p->dev_offset[1];
        g.oBN = p->dev_tables + p->dev_offset[2]; g.oBK = p->dev_tables + p->dev_offset[3];
        g.oDM = p->dev_tables + p->dev_offset[4]; g.oDN = p->dev_tables + p->dev_offset[5];
        if (p->dev_narrow) {
            const unsigned char* nb = p->dev_narrow;
            const size_t* o = p->narrow_off;
            g.rrA = (const uint32_t*)(nb + o[0]); g.rbA = (const int64_t*)(nb + o[1]); g.kqA = (const int64_t*)(nb + o[2]);
            g.krA = (const uint32_t*)(nb + o[3]); g.kbA = (const int64_t*)(nb + o[4]);
            g.rrB = (const uint32_t*)(nb + o[5]); g.rbB = (const int64_t*)(nb + o[6]); g.kqB = (const int64_t*)(nb + o[7]);
            g.krB = (const uint32_t*)(nb + o[8]); g.kbB = (const int64_t*)(nb + o[9]);
            g.periodicA = p->periodic[0]; g.periodicB = p->periodic[1];
            g.pair = p->pairs && (((uintptr_t)A | (uintptr_t)B) & 15) == 0;
            g.psA = p->pair_step[0]; g.psB = p->pair_step[1];
        }
        g.sizeM = p->an.sizeM; g.sizeN = p->an.sizeN; g.sizeK = p->an.sizeK; g.sizeH = p->an.sizeH;
        g.tilesM = (int32_t)((g.sizeM + v.mt_m - 1) / v.mt_m);
        g.tilesN = (int32_t)((g.sizeN + v.mt_n - 1) / v.mt_n);
        g.tilesK = (int32_t)((g.sizeK + v.kt - 1) / v.kt);
        g.nH = (int32_t)p->an.H.size();
        for (int i = 0; i < g.nH; ++i) {
            g.hExt[i] = p->an.H[i].extent; g.hSA[i] = p->an.H[i].sA; g.hSB[i] = p->an.H[i].sB; g.hSD[i] = p->an.H[i].sD;
        }
        if (v.hl > 1) {
            // a tile holds v.hl consecutive batches of the fastest hyper mode: the kernel decodes groups of them
            g.sizeH /= v.hl;
            g.hExt[0] /= v.hl; g.hSA[0] *= v.hl; g.hSB[0] *= v.hl; g.hSD[0] *= v.hl;
        }
        g.s = s;
        g.opA = p->an.opA; g.opB = p->an.opB; g.opC = p->an.opC;
        g.read_c = read_c;
        g.splitK = p->splitK;
        if (need_partials > 0) {
            if (split_ok) g.workspace = ws;                  // fully written by the parts before the reduction kernel reads it
            else g.splitK = 1;
        }
        g.lid_base = 0;
        // rounds pay off when a tile runs for milliseconds (hundreds of slabs) and there are several rounds
        g.round_size = (int32_t)round_size_of(*p, v);
        hip_err = launch_gett(p->an.dtype, p->an.precision, p->variant, p->an.a_k_fastest, p->an.b_k_fastest, p->an.d_n_fastest, g,
                              (void*)e->stream, &grid, &block);
        st.path = TCX_PATH_GETT_MFMA; st.variant = p->variant;
        st.gather_width = g.pair && v.pingpong && v.dual && g.sizeK % v.kt == 0 ? 2 : 1;
        st.tile_m = v.mt_m; st.tile_n = v.mt_n; st.tile_k = v.kt;
    } else {
        GenericArgs g = p->generic;
        g.A = A; g.B = B; g.C = C; g.D = D;
        g.s = s;
        g.read_c = read_c; g.read_ab = read_ab;
        hip_err = launch_generic(p->an.dtype, p->an.precision, g, (void*)e->stream, &grid, &block);
        st.path = TCX_PATH_GENERIC;
    }
    st.grid = grid; st.block = block; st.hip_error = hip_err;
    if (status) {
        Status* so = new (std::nothrow) Status(st);
        *status = so ? publish(so, MAGIC_STATUS) : 0;
    }
    return hip_err == 0 ? TCX_SUCCESS : TCX_ERR_LAUNCH;
}
}  // namespace

extern "C" {

tcx_error_t tcx_execute_product(tcx_product_t product, tcx_executor_t executor, tcx_status_t* status, const void* alpha,
                                const void* A, const void* B, const void* beta, const void* C, void* D) {
    return run_product(product, executor, status, alpha, A, B, beta, C, D, false);
}

tcx_error_t tcx_execute_binary(tcx_product_t plan, tcx_executor_t executor, tcx_status_t* status, const void* alpha, const void* A,
                               const void* beta, const void* B, void* C) {
    return run_product(plan, executor, status, alpha, A, nullptr, beta, B, C, false, KIND_BINARY);
}

tcx_error_t tcx_execute_unary(tcx_product_t plan, tcx_executor_t executor, tcx_status_t* status, const void* alpha, const void* A,
                              void* B) {
    const double zero[2] = {0.0, 0.0};                       // beta = 0 in every dtype: B is never read
    return run_product(plan, executor, status, alpha, A, nullptr, zero, nullptr, B, false, KIND_UNARY);
}

tcx_error_t tcx_execute_product_noalloc(tcx_product_t product, tcx_executor_t executor, const void* alpha, const void* A,
                                        const void* B, const void* beta, const void* C, void* D) {
    return run_product(product, executor, nullptr, alpha, A, B, beta, C, D, true);
}

tcx_error_t tcx_probe_launch(tcx_executor_t executor, int32_t kind, void* buffer, size_t bytes, int64_t iters, double* work) {
    Executor* e = lookup<Executor>(executor, MAGIC_EXEC);
    if (!e) return TCX_ERR_INVALID_HANDLE;
    if (!buffer || !work) return TCX_ERR_NULL_ARG;
    if (!e->handle.has_device) return TCX_ERR_NO_DEVICE;
    if (((uintptr_t)buffer & 15) != 0) return TCX_ERR_TOO_LARGE;
    return launch_probe(kind, buffer, bytes, iters, e->handle.num_cu, (void*)e->stream, work) == 0 ? TCX_SUCCESS : TCX_ERR_LAUNCH;
}

tcx_error_t tcx_status_get(tcx_status_t status, int32_t key, void* value, size_t* nbytes) {
    Status* s = lookup<Status>(status, MAGIC_STATUS);
    if (!s) return TCX_ERR_INVALID_HANDLE;
    switch (key) {
        case TCX_KEY_PATH: return put_i64(s->path, value, nbytes);
        case TCX_KEY_VARIANT: return put_i64(s->variant, value, nbytes);
        case TCX_KEY_GRID: return put_i64(s->grid, value, nbytes);
        case TCX_KEY_BLOCK: return put_i64(s->block, value, nbytes);
        case TCX_KEY_TILE_M: return put_i64(s->tile_m, value, nbytes);
        case TCX_KEY_TILE_N: return put_i64(s->tile_n, value, nbytes);
        case TCX_KEY_TILE_K: return put_i64(s->tile_k, value, nbytes);
        case TCX_KEY_HIP_ERROR: return put_i64(s->hip_error, value, nbytes);
        case TCX_KEY_GATHER_WIDTH: return put_i64(s->gather_width, value, nbytes);
        default: return TCX_ERR_BAD_KEY;
    }
}

tcx_error_t tcx_destroy_status(tcx_status_t* status) { return retire<Status>(status, MAGIC_STATUS); }

tcx_error_t tcx_create_attr(tcx_handle_t handle, tcx_attr_t* out) {
    if (!out) return TCX_ERR_NULL_ARG;
    if (!lookup<Handle>(handle, MAGIC_HANDLE)) return TCX_ERR_INVALID_HANDLE;
    Attr* a = new (std::nothrow) Attr;
    if (!a) return TCX_ERR_ALLOC;
    *out = publish(a, MAGIC_ATTR);
    return TCX_SUCCESS;
}

tcx_error_t tcx_destroy_attr(tcx_attr_t* attr) { return retire<Attr>(attr, MAGIC_ATTR); }

namespace {
uint32_t type_of(intptr_t object) {
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_live.find(object);
    return object != 0 && it != g_live.end() ? it->second : 0u;
}
}  // namespace

tcx_error_t tcx_attr_set(tcx_object_t object, int32_t key, const void* value, size_t nbytes) {
    const uint32_t type = type_of(object);
    if (!type) return TCX_ERR_INVALID_HANDLE;
    if (key < TCX_KEY_USER) {
        if (type == MAGIC_PRODUCT) return tcx_product_set(object, key, value, nbytes);
        if (type == MAGIC_EXEC && (key == TCX_KEY_STREAM || key == TCX_KEY_WORKSPACE_BYTES)) {
            Executor* e = lookup<Executor>(object, MAGIC_EXEC);
            if (!e) return TCX_ERR_INVALID_HANDLE;
            if (!value) return TCX_ERR_NULL_ARG;
            if (nbytes != sizeof(int64_t)) return TCX_ERR_BUFFER_TOO_SMALL;
            int64_t v;
            std::memcpy(&v, value, sizeof v);
            std::lock_guard<std::mutex> lk(e->mu);
            if (key == TCX_KEY_STREAM) { e->stream = (hipStream_t)(intptr_t)v; return TCX_SUCCESS; }
            if (v < 0) return TCX_ERR_TOO_LARGE;
            if (!e->handle.has_device) return TCX_ERR_NO_DEVICE;
            return grow_workspace(e, (size_t)v);              // reserve ahead of the first execution
        }
        return TCX_ERR_BAD_KEY;
    }
    if (!value && nbytes) return TCX_ERR_NULL_ARG;
    try {
        std::vector<unsigned char> copy((const unsigned char*)value, (const unsigned char*)value + nbytes);
        std::lock_guard<std::mutex> lk(g_mu);
        if (!g_live.count(object)) return TCX_ERR_INVALID_HANDLE;       // destroyed meanwhile
        g_kv[object][key] = std::move(copy);
    } catch (const std::bad_alloc&) {
        return TCX_ERR_ALLOC;
    }
    return TCX_SUCCESS;
}

tcx_error_t tcx_attr_get(tcx_object_t object, int32_t key, void* value, size_t* nbytes) {
    const uint32_t type = type_of(object);
    if (!type) return TCX_ERR_INVALID_HANDLE;
    if (key < TCX_KEY_USER) {
        if (type == MAGIC_PRODUCT) return tcx_product_get(object, key, value, nbytes);
        if (type == MAGIC_STATUS) return tcx_status_get(object, key, value, nbytes);
        if (type == MAGIC_HANDLE) {
            Handle* h = lookup<Handle>(object, MAGIC_HANDLE);
            if (!h) return TCX_ERR_INVALID_HANDLE;
            if (key == TCX_KEY_DEVICE) return put_i64(h->has_device ? h->device : -1, value, nbytes);
            if (key == TCX_KEY_NUM_CU) return put_i64(h->num_cu, value, nbytes);
            return TCX_ERR_BAD_KEY;
        }
        if (type == MAGIC_EXEC) {
            Executor* e = lookup<Executor>(object, MAGIC_EXEC);
            if (!e) return TCX_ERR_INVALID_HANDLE;
            if (key == TCX_KEY_DEVICE) return put_i64(e->handle.has_device ? e->handle.device : -1, value, nbytes);
            if (key == TCX_KEY_STREAM) return put_i64((int64_t)(intptr_t)e->stream, value, nbytes);
            if (key == TCX_KEY_WORKSPACE_BYTES) {
                std::lock_guard<std::mutex> lk(e->mu);
                return put_i64((int64_t)e->workspace_bytes, value, nbytes);
            }
            return TCX_ERR_BAD_KEY;
        }
        return TCX_ERR_BAD_KEY;
    }
    if (!nbytes) return TCX_ERR_NULL_ARG;
    std::lock_guard<std::mutex> lk(g_mu);
    auto obj = g_kv.find(object);
    if (obj == g_kv.end()) return TCX_ERR_BAD_KEY;
    auto it = obj->second.find(key);
    if (it == obj->second.end()) return TCX_ERR_BAD_KEY;
    const std::vector<unsigned char>& v = it->second;
    if (v.empty()) { *nbytes = 0; return TCX_SUCCESS; }
    return put(v.data(), v.size(), value, nbytes);
}

tcx_error_t tcx_attr_clear(tcx_object_t object, int32_t key) {
    const uint32_t type = type_of(object);
    if (!type) return TCX_ERR_INVALID_HANDLE;
    if (key < TCX_KEY_USER) {
        if (type != MAGIC_PRODUCT || (key != TCX_KEY_FORCE_PATH && key != TCX_KEY_VARIANT && key != TCX_KEY_SPLIT_K))
            return TCX_ERR_BAD_KEY;
        Product* p = lookup<Product>(object, MAGIC_PRODUCT);
        return p ? route(p) : TCX_ERR_INVALID_HANDLE;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    auto obj = g_kv.find(object);
    if (obj == g_kv.end() || !obj->second.erase(key)) return TCX_ERR_BAD_KEY;
    return TCX_SUCCESS;
}

int tcx_check_success(tcx_error_t error) { return error == TCX_SUCCESS ? 1 : 0; }

size_t tcx_explain_error(tcx_error_t error, size_t maxlen, char* msg) {
    const int n = (int)(sizeof(kMessages) / sizeof(kMessages[0]));
    const char* text = (error >= 0 && error < n) ? kMessages[error] : "unknown error code";
    const size_t need = std::strlen(text);
    if (msg && maxlen > 0) {
        const size_t ncopy = need < maxlen - 1 ? need : maxlen - 1;
        std::memcpy(msg, text, ncopy);
        msg[ncopy] = '\0';
    }
    return need;
}

}  // extern "C"
