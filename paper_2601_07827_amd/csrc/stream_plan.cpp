// Planner of the bandwidth (streaming) path: picks the output tile from D's fastest modes and
// builds the per-tile lookup tables.  Pure host code.
#include <algorithm>
#include <cstdlib>

#include "tcx_internal.hpp"

namespace tcx {
namespace {

struct DMode {
    Mode m;
    bool inA, inB;
};

inline int64_t iabs64(int64_t x) { return x < 0 ? -x : x; }

}  // namespace

bool stream_preferred(const Analysis& an, int elem_bytes) {
    // Flop per byte if every operand moved exactly once (beta taken as 0: an upper bound).
    const double flop = (an.dtype == TCX_C128 ? 8.0 : 2.0) * (double)an.sizeH * an.sizeM * an.sizeN * an.sizeK;
    const double bytes = (double)elem_bytes * ((double)an.sizeH * an.sizeM * an.sizeK + (double)an.sizeH * an.sizeN * an.sizeK +
                                               (double)an.sizeH * an.sizeM * an.sizeN);
    const double ridge = an.dtype == TCX_F32 ? 19.7 : 9.8;     // peak matrix flop/s over peak HBM byte/s
    return an.sizeK <= 32 && flop / bytes < ridge;
}

StreamPlan plan_stream(const Analysis& an, int elem_bytes) {
    StreamPlan p;
    if (an.sizeK > 64) return p;
    // every mode that indexes D, D-fastest first
    std::vector<DMode> dm;
    for (const Mode& m : an.H) dm.push_back({m, true, true});
    for (const Mode& m : an.M) dm.push_back({m, true, false});
    for (const Mode& m : an.N) dm.push_back({m, false, true});
    std::stable_sort(dm.begin(), dm.end(), [](const DMode& a, const DMode& b) { return iabs64(a.m.sD) < iabs64(b.m.sD); });
    const int K = (int)an.sizeK;

    for (int target = 2048; target >= 64 && !p.ok; target /= 2) {
        // whole modes while they fit, then a chunk of the next one
        size_t nfull = 0;
        int64_t inner = 1;
        while (nfull < dm.size() && inner * dm[nfull].m.extent <= target) inner *= dm[nfull++].m.extent;
        int64_t chunk = 1, split_extent = 1;
        const bool has_split = nfull < dm.size() && inner < target;
        if (has_split) {
            split_extent = dm[nfull].m.extent;
            chunk = std::min<int64_t>(split_extent, std::max<int64_t>(1, target / inner));
        }
        int64_t rowsA = 1, rowsB = 1;
        for (size_t i = 0; i < nfull; ++i) {
            if (dm[i].inA) rowsA *= dm[i].m.extent;
            if (dm[i].inB) rowsB *= dm[i].m.extent;
        }
        if (has_split && dm[nfull].inA) rowsA *= chunk;
        if (has_split && dm[nfull].inB) rowsB *= chunk;
        const int64_t tile = inner * chunk;
        const size_t lds = (size_t)(rowsA + rowsB) * K * elem_bytes;
        if (lds > 60 * 1024 || rowsA > 65535 || rowsB > 65535) continue;

        p.tile = (int32_t)tile; p.inner = (int32_t)inner; p.chunk = (int32_t)chunk; p.split_extent = split_extent;
        p.rowsA = (int32_t)rowsA; p.rowsB = (int32_t)rowsB; p.K = K;
        p.split_in_A = has_split && dm[nfull].inA; p.split_in_B = has_split && dm[nfull].inB;
        p.lds_bytes = lds;

        // tile-local tables: walk the tile in D order (first tile mode fastest)
        std::vector<DMode> tm(dm.begin(), dm.begin() + (long)nfull);
        if (has_split) { DMode s = dm[nfull]; s.m.extent = chunk; tm.push_back(s); }
        p.rowAB.assign((size_t)tile, 0);
        p.dD.assign((size_t)tile, 0);
        std::vector<int64_t> rowSrcA((size_t)rowsA, 0), rowSrcB((size_t)rowsB, 0);
        std::vector<uint32_t> rowDigA((size_t)rowsA, 0), rowDigB((size_t)rowsB, 0);
        std::vector<int64_t> idx(tm.size(), 0);
        for (int64_t e = 0; e < tile; ++e) {
            int64_t ra = 0, rb = 0, wa = 1, wb = 1, offA = 0, offB = 0, offD = 0;
            for (size_t i = 0; i < tm.size(); ++i) {
                offD += idx[i] * tm[i].m.sD;
                if (tm[i].inA) { ra += idx[i] * wa; wa *= tm[i].m.extent; offA += idx[i] * tm[i].m.sA; }
                if (tm[i].inB) { rb += idx[i] * wb; wb *= tm[i].m.extent; offB += idx[i] * tm[i].m.sB; }
            }
            p.rowAB[(size_t)e] = (uint32_t)ra | ((uint32_t)rb << 16);
            p.dD[(size_t)e] = offD;
            rowSrcA[(size_t)ra] = offA; rowSrcB[(size_t)rb] = offB;
            const uint32_t dig = has_split ? (uint32_t)idx.back() : 0;
            if (p.split_in_A) rowDigA[(size_t)ra] = dig;
            if (p.split_in_B) rowDigB[(size_t)rb] = dig;
            for (size_t i = 0; i < tm.size(); ++i) {
                if (++idx[i] < tm[i].m.extent) break;
                idx[i] = 0;
            }
        }
        // staging lists: (row, k) -> source offset; sorted by source so neighbouring lanes read
        // neighbouring addresses whatever the operand's own mode order is
        const std::vector<int64_t> kA = offset_table(an.K, 0, 0), kB = offset_table(an.K, 1, 0);
        auto items = [&](const std::vector<int64_t>& rowSrc, const std::vector<uint32_t>& dig, const std::vector<int64_t>& kOff) {
            std::vector<StreamItem> v;
            v.reserve(rowSrc.size() * (size_t)K);
            for (size_t r = 0; r < rowSrc.size(); ++r)
                for (int k = 0; k < K; ++k) v.push_back({rowSrc[r] + kOff[(size_t)k], (uint32_t)(r * (size_t)K + (size_t)k), dig[r]});
            std::stable_sort(v.begin(), v.end(), [](const StreamItem& a, const StreamItem& b) { return a.src < b.src; });
            return v;
        };
        p.itemsA = items(rowSrcA, rowDigA, kA);
        p.itemsB = items(rowSrcB, rowDigB, kB);

        // outer loop modes: chunks of the split mode, then the rest of D's modes
        p.n_outer = 0;
        p.num_tiles = 1;
        auto push_outer = [&](int64_t ext, int64_t sA, int64_t sB, int64_t sD) {
            p.oExt[p.n_outer] = ext; p.oSA[p.n_outer] = sA; p.oSB[p.n_outer] = sB; p.oSD[p.n_outer] = sD;
            ++p.n_outer;
            p.num_tiles *= ext;
        };
        if (has_split) {
            const Mode& s = dm[nfull].m;
            push_outer((split_extent + chunk - 1) / chunk, s.sA * chunk, s.sB * chunk, s.sD * chunk);
        }
        for (size_t i = nfull + (has_split ? 1 : 0); i < dm.size(); ++i) push_outer(dm[i].m.extent, dm[i].m.sA, dm[i].m.sB, dm[i].m.sD);
        p.ok = p.n_outer <= kMaxOuterModes;
    }
    return p;
}

}  // namespace tcx
