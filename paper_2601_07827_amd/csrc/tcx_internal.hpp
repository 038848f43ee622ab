// Internal declarations of libtcx: the result of the index analysis, the kernel argument
// blocks, and the launch entry points each kernel file exports to the API layer.
#pragma once

#include <cstdint>
#include <vector>

#include "tcx.h"

namespace tcx {

// One fused mode of a label group.  A stride is 0 where the tensor does not carry the mode
// (paper, Sec. "Algorithm Structure": strides of absent indices are set to zero).
struct Mode {
    int64_t extent;
    int64_t sA, sB, sD;
};

// ---- element types --------------------------------------------------------------------
inline int elem_bytes_of(int dtype) { return dtype == TCX_F16 || dtype == TCX_BF16 ? 2 : dtype == TCX_F32 ? 4 : dtype == TCX_C128 ? 16 : 8; }
inline int real_bytes_of(int dtype) { return dtype == TCX_F16 || dtype == TCX_BF16 ? 2 : dtype == TCX_F32 || dtype == TCX_C64 ? 4 : 8; }   // of the storage type
inline bool is_complex(int dtype) { return dtype == TCX_C64 || dtype == TCX_C128; }
inline bool valid_dtype(int dtype) {
    return dtype == TCX_F32 || dtype == TCX_F64 || dtype == TCX_C64 || dtype == TCX_C128 || dtype == TCX_F16 || dtype == TCX_BF16;
}
// Reals that products and sums are formed in: the storage type's own, 32 bits for 16-bit storage,
// 64 bits for every plan in TCX_PREC_F64.
inline int compute_real_bytes(int dtype, int precision) {
    return precision == TCX_PREC_F64 ? 8 : real_bytes_of(dtype) == 2 ? 4 : real_bytes_of(dtype);
}
// storage narrower than the arithmetic: elements are widened as they are read, D is rounded once
inline bool is_widened(int dtype, int precision) { return compute_real_bytes(dtype, precision) > real_bytes_of(dtype); }

struct TensorDesc {
    int32_t dtype = 0;
    std::vector<int64_t> extent, stride;
};

// Sum over an operand's isolated labels (paper, Sec. "Case 4": labels in A only, or in B only,
// are reduced inside that tensor before the product).  The reduced operand is written densely,
// column-major over the kept modes in `keep` order, into workspace memory; the contraction then
// reads it in place of the tensor.
struct Reduction {
    bool active = false;
    std::vector<int64_t> keepExt, keepSrc;     // kept modes, fastest of the reduced operand first: extent, stride in the tensor
    std::vector<int64_t> sumExt, sumSrc;       // summed modes: extent, stride in the tensor
    int64_t count = 1;                         // elements of the reduced operand
};

// Result of validation + classification + merging + fusion + sorting.
struct Analysis {
    int32_t dtype = 0;
    int32_t precision = 0;                  // tcx_prec_t
    int32_t opA = 0, opB = 0, opC = 0;
    std::vector<Mode> H, M, N, K;           // fastest mode first
    int64_t sizeH = 1, sizeM = 1, sizeN = 1, sizeK = 1;
    bool a_k_fastest = false;               // A's smallest |stride| over M and K modes is a K mode
    bool b_k_fastest = false;
    bool d_n_fastest = false;               // D's smallest |stride| over M and N modes is an N mode
    int32_t path = TCX_PATH_GENERIC;
    int32_t variant = 0;
    Reduction redA, redB;                   // Case 4: the strides sA / sB above then address the reduced operand
};

// Host part of the planner (analyser.cpp).  Pure host code: no HIP calls.
tcx_error_t analyse(const TensorDesc& A, const int64_t* labA, const TensorDesc& B, const int64_t* labB,
                    const TensorDesc& C, const int64_t* labC, const TensorDesc& D, const int64_t* labD,
                    int opA, int opB, int opC, int opD, int precision, Analysis* out);

// offsets[g] = sum_i idx_i * stride_i for the linear index g over `modes` (first mode fastest);
// which: 0 = A, 1 = B, 2 = D.  The table is padded with zeros up to `padded` entries.
std::vector<int64_t> offset_table(const std::vector<Mode>& modes, int which, int64_t padded);

// ---- kernel argument blocks (plain data, passed by value) ------------------------------
constexpr int kMaxHModes = 8;      // hyper modes decoded inside the tiled kernels
constexpr int kMaxGenericModes = 32;

struct Scalars {
    double alpha_re, alpha_im, beta_re, beta_im;
};

// Tiled (GETT) kernels.  Offsets are in elements.  Tables are padded to a whole number of
// tiles with entries that address a valid element, so unmasked loads stay in bounds.
struct GettArgs {
    const void* A;
    const void* B;
    const void* C;
    void* D;
    const int64_t* oAM;  // [tilesM * MT_M]
    const int64_t* oAK;  // [tilesK * KT]
    const int64_t* oBN;  // [tilesN * MT_N]
    const int64_t* oBK;  // [tilesK * KT]
    const int64_t* oDM;  // [tilesM * MT_M]
    const int64_t* oDN;  // [tilesN * MT_N]
    // LDS-staged kernels gather through tile-relative byte offsets: element address =
    // operand + hyper offset + rowbase[tile] + (kofs[k] | kbase[slab] + krel[k]) + rowrel[row]
    const uint32_t* rrA;   // rowrel  [tilesM * MT_M]
    const int64_t* rbA;    // rowbase [tilesM]
    const int64_t* kqA;    // kofs    [tilesK * KT]   (lanes along the rows: one scalar per k)
    const uint32_t* krA;   // krel    [tilesK * KT]   (lanes along k)
    const int64_t* kbA;    // kbase   [tilesK]
    const uint32_t* rrB;
    const int64_t* rbB;
    const int64_t* kqB;
    const uint32_t* krB;
    const int64_t* kbB;
    int32_t periodicA, periodicB;   // krel is the same in every slab (two-phase kernel, lanes along k)
    int64_t lid_base;      // first tile number of this launch (a product may be launched in rounds)
    int32_t round_size;    // > 0: launch the grid in rounds of this many workgroups (two-phase kernel)
    int32_t pair;          // two-phase kernel, 8-byte elements: a gather load brings two elements that the host found contiguous and 16-byte aligned
    int32_t psA, psB;      // ... element x along the lanes' direction is paired with x + ps
    int64_t sizeM, sizeN, sizeK, sizeH;
    int32_t tilesM, tilesN, tilesK;
    int32_t nH;
    int64_t hExt[kMaxHModes], hSA[kMaxHModes], hSB[kMaxHModes], hSD[kMaxHModes];
    Scalars s;
    int32_t opA, opB, opC;
    int32_t read_c;      // beta != 0
    int32_t conj_acc;    // set by the launcher: the kernel sums the conjugate of the wanted product (complex two-phase kernels)
    int32_t splitK;      // >= 1: number of parts the K slabs are divided into
    void* workspace;     // splitK > 1: [tiles * splitK][accumulator reals of a tile], owned by the plan
};

struct GettVariant {
    int mt_m, mt_n, kt, threads;   // threads: per TILE (a dual workgroup has twice as many)
    float efficiency;    // relative main-loop speed per unit tile area, for the planner's cost model
    int acc_reals;       // real accumulator values per tile (split-K workspace per part)
    bool staged;         // kernel gathers through the narrow (32-bit, tile-relative) tables
    bool pingpong;       // two-phase kernel: needs |K| % kt == 0 and slab-periodic relative k offsets
    int fallback;        // shape to try first when this one cannot serve the plan (-1: none)
    bool dual;           // two-phase kernel with one tile per wave group: a workgroup takes two items
    bool pair_in_lds;    // ... and reduces a two-part split of K inside the workgroup (no workspace, no second kernel)
    int hl;              // batches per tile (> 1: batch-lane kernel; the fastest hyper mode is cut into groups of hl; K unsplit)
};

// Generic fallback: every mode of D (H, M, N together, D-fastest first) and every K mode.
struct GenericArgs {
    const void* A;
    const void* B;
    const void* C;
    void* D;
    int32_t nD, nK;
    int64_t dExt[kMaxGenericModes], dSA[kMaxGenericModes], dSB[kMaxGenericModes], dSD[kMaxGenericModes];
    int64_t kExt[kMaxGenericModes], kSA[kMaxGenericModes], kSB[kMaxGenericModes];
    int64_t sizeD, sizeK;
    Scalars s;
    int32_t opA, opB, opC;
    int32_t read_c, read_ab;
};

// Pre-reduction of an operand (Sec. "Case 4"): dst[lin] = sum over the summed modes of src.
struct ReduceArgs {
    const void* src;
    void* dst;
    int32_t nKeep, nSum;
    int64_t keepExt[kMaxGenericModes], keepSrc[kMaxGenericModes];
    int64_t sumExt[kMaxGenericModes], sumSrc[kMaxGenericModes];
    int64_t count, sumCount;
};

// Launchers (defined in the .hip files).  `stream` is a hipStream_t.  Return a hipError_t.
int launch_reduce(int dtype, int precision, const ReduceArgs& args, void* stream);
int launch_generic(int dtype, int precision, const GenericArgs& args, void* stream, int64_t* grid, int* block);

int gett_num_variants(int dtype);
GettVariant gett_variant(int dtype, int variant);
// Is tile shape `variant` built for this element type and precision?  (The two-phase kernels exist
// for fp32, fp64 and complex128 in their own precision; widened 32-bit types have two shapes each.)
bool gett_available(int dtype, int precision, int variant);
int launch_gett(int dtype, int precision, int variant, bool a_kf, bool b_kf, bool d_nf, const GettArgs& args, void* stream,
                int64_t* grid, int* block);

}  // namespace tcx

// ---- bandwidth (streaming) path ---------------------------------------------------------------
// Output-stationary: a workgroup owns a tile made of D's fastest modes (so its stores are one
// contiguous stretch of D wherever D is), stages the few elements of A and B that the tile
// needs through LDS with loads that follow A's and B's own memory order, and streams D out.
namespace tcx {

constexpr int kStreamThreads = 256;
constexpr int kStreamRegBlock = 4;    // a thread's register block is at most 4 x 4 outputs
constexpr int kStreamPerThread = 8;   // table entries a thread keeps in registers: tile, staged items <= 2048

struct StreamItem {        // one element to stage: where it comes from and where it goes
    int64_t src;           // element offset relative to the tile's base in A (or B)
    uint32_t slot;         // LDS slot = row * K + k
    uint32_t digit;        // index along the split mode (for masking the ragged last chunk)
};

struct StreamPlan {
    bool ok = false;
    bool blocked = false;      // threads own a regA x regB register block of outputs
    bool direct = false;       // blocked tile whose lanes all run along hyper modes: every lane has operand rows of its own, read straight from memory
    bool paced = false;        // flat tile whose operand lines collide in the L2 (see stream_plan.cpp): loads go out a few at a time
    int32_t tile = 0;          // lane indices per tile (flat: outputs per full tile = inner * chunk)
    int32_t inner = 0;         // flat tiles: product of the tile modes below the split mode
    int32_t chunk = 1;         // flat tiles: indices of the split mode per tile
    int64_t split_extent = 1;  // flat tiles: extent of the split mode (1 if none)
    int32_t rowsA = 0, rowsB = 0, K = 0;
    int32_t regA = 1, regB = 1;            // register block (blocked tiles)
    int32_t rowStepA = 0, rowStepB = 0;    // row increment per register index
    int64_t dRegA[kStreamRegBlock], dRegB[kStreamRegBlock];   // D offset per register index
    int64_t num_tiles = 0;
    // host tables
    std::vector<uint32_t> rowAB;     // [tile]: rowA | rowB << 16 of a lane index
    std::vector<int64_t> dD;         // [tile]: D offset of a lane index relative to the tile base
    std::vector<int64_t> laneA, laneB;   // direct tiles, [tile]: A / B offset of a lane index
    int64_t aReg[kStreamRegBlock], bReg[kStreamRegBlock];   // direct tiles: A / B offset per register index
    int64_t aK[kStreamRegBlock], bK[kStreamRegBlock];       // direct tiles: A / B offset per contracted index (K <= 4)
    std::vector<StreamItem> itemsA, itemsB;
    // tile index -> base offsets: tile = lo + outer_lo * hi; rows are (offA, offB, offD, digits)
    int64_t outer_lo = 1;
    std::vector<int64_t> tabLo, tabHi;
    size_t lds_bytes = 0;
    double staged_per_output = 0;    // operand elements staged per output element (traffic overhead)
};

struct StreamArgs {
    const void* A;
    const void* B;
    const void* C;
    void* D;
    const uint32_t* rowAB;
    const int64_t* dD;
    const StreamItem* itemsA;
    const StreamItem* itemsB;
    const int64_t* laneA;      // direct tiles
    const int64_t* laneB;
    int64_t aReg[kStreamRegBlock], bReg[kStreamRegBlock], aK[kStreamRegBlock], bK[kStreamRegBlock];
    int32_t nItemsA, nItemsB;
    int32_t tile, inner, chunk, K, rowsA, rowsB;
    int32_t regA, regB, rowStepA, rowStepB;
    int64_t dRegA[kStreamRegBlock], dRegB[kStreamRegBlock];
    int64_t split_extent;
    int64_t num_tiles;
    int64_t outer_lo;          // number of rows of tabLo
    const int64_t* tabLo;      // [outer_lo][4]
    const int64_t* tabHi;      // [num_tiles / outer_lo][4]
    Scalars s;
    int32_t opA, opB, opC;
    int32_t read_c;
    int32_t paced;
};

// Host: lay out the streaming plan for an analysed product (stream_plan.cpp).
StreamPlan plan_stream(const Analysis& an, int elem_bytes, bool allow_blocked = true);
// Arithmetic intensity test + size limits: should this product take the streaming path?
bool stream_preferred(const Analysis& an, int elem_bytes);

// Measurement aid (probes.hip): one launch of a single-purpose kernel; *work = flop or bytes it does.
int launch_probe(int kind, void* buffer, size_t bytes, int64_t iters, int num_cu, void* stream, double* work);

// Number of workgroups launch_stream starts for a plan (items_per_thread: staged operand elements per thread).
int64_t stream_grid(bool blocked, bool direct, int items_per_thread, int64_t num_tiles, int num_cu);
int launch_stream(int dtype, bool blocked, bool direct, const StreamArgs& args, size_t lds_bytes, int num_cu, void* stream,
                  int64_t* grid, int* block);

}  // namespace tcx
