// Planner of the bandwidth (streaming) path: picks the output tile from D's fastest modes and
// builds the per-tile lookup tables.  Pure host code.
//
// A tile is a list of pieces.  A piece takes `count` consecutive indices of one D mode.  LANE
// pieces (D's fastest modes) form the index that runs across the threads, so stores are
// contiguous in D; REG_A / REG_B pieces are free modes of A / of B that each thread walks in
// registers, so an operand row fetched from LDS is reused for several outputs ("blocked"
// tiles).  What a piece leaves of its mode becomes an outer mode that the grid walks.
#include <algorithm>
#include <cstdlib>

#include "tcx_internal.hpp"

namespace tcx {
namespace {

struct DMode {
    Mode m;
    bool inA, inB;
};

enum Role { LANE = 0, REG_A = 1, REG_B = 2 };

struct Piece {
    int mode;        // index into the D-ordered mode list
    int64_t count;   // indices taken per tile
    int64_t mult;    // index = digit * mult (+ what other pieces / the outer loop add)
    int role;
};

inline int64_t iabs64(int64_t x) { return x < 0 ? -x : x; }

int64_t largest_divisor_at_most(int64_t n, int64_t cap) {
    for (int64_t c = std::min(n, cap); c > 1; --c)
        if (n % c == 0) return c;
    return 1;
}

// Fill every table of `p` from the chosen pieces.  `ragged`: the last LANE piece may not divide
// its mode (flat tiles only); its digit is recorded so the kernel can mask the last chunk.
bool build(const std::vector<DMode>& dm, const std::vector<Piece>& pieces, bool ragged, const Analysis& an, int elem_bytes,
           StreamPlan* out) {
    StreamPlan p;
    const int K = (int)an.sizeK;
    p.K = K;
    // sizes
    int64_t lanes = 1, ra = 1, rb = 1, rowsA_lane = 1, rowsB_lane = 1;
    for (const Piece& pc : pieces) {
        if (pc.role == LANE) {
            lanes *= pc.count;
            if (dm[(size_t)pc.mode].inA) rowsA_lane *= pc.count;
            if (dm[(size_t)pc.mode].inB) rowsB_lane *= pc.count;
        } else if (pc.role == REG_A) {
            ra *= pc.count;
        } else {
            rb *= pc.count;
        }
    }
    const int64_t rowsA = rowsA_lane * ra, rowsB = rowsB_lane * rb;
    const int64_t cap = (int64_t)kStreamThreads * kStreamPerThread;      // what a workgroup's registers hold
    const size_t lds = (size_t)(rowsA + rowsB) * (size_t)K * (size_t)elem_bytes;
    const bool blocked = ra * rb > 1;
    // Lanes that all run along hyper modes share no operand element: staging through LDS would
    // only add traffic, and every lane reads its own rows straight from memory instead (the
    // loads coalesce as the stores do when the hyper modes are the operands' fastest too).
    bool direct = blocked && K <= kStreamRegBlock;
    for (const Piece& pc : pieces)
        if (pc.role == LANE && !(dm[(size_t)pc.mode].inA && dm[(size_t)pc.mode].inB)) direct = false;
    if (!direct && (lds > 64 * 1024 || rowsA * K > cap || rowsB * K > cap || rowsA > 65535 || rowsB > 65535)) return false;
    if (blocked ? lanes > kStreamThreads : lanes > cap) return false;
    if (ra > kStreamRegBlock || rb > kStreamRegBlock) return false;

    p.blocked = blocked;
    p.direct = direct;
    p.tile = (int32_t)lanes;
    p.regA = (int32_t)ra; p.regB = (int32_t)rb;
    p.rowsA = (int32_t)rowsA; p.rowsB = (int32_t)rowsB;
    p.rowStepA = (int32_t)rowsA_lane; p.rowStepB = (int32_t)rowsB_lane;
    p.lds_bytes = direct ? 0 : lds;

    // the ragged piece, if any, is the last LANE piece
    int last_lane = -1;
    for (size_t i = 0; i < pieces.size(); ++i)
        if (pieces[i].role == LANE) last_lane = (int)i;
    const bool has_split = ragged && last_lane >= 0 && pieces[(size_t)last_lane].count < dm[(size_t)pieces[(size_t)last_lane].mode].m.extent;
    p.chunk = has_split ? (int32_t)pieces[(size_t)last_lane].count : 1;
    p.split_extent = has_split ? dm[(size_t)pieces[(size_t)last_lane].mode].m.extent : 1;
    p.inner = (int32_t)(lanes / p.chunk);

    // lane tables: walk the LANE pieces, first fastest
    std::vector<const Piece*> lp, apieces, bpieces;
    for (const Piece& pc : pieces) if (pc.role == LANE) lp.push_back(&pc);
    p.rowAB.assign((size_t)lanes, 0);
    p.dD.assign((size_t)lanes, 0);
    if (direct) { p.laneA.assign((size_t)lanes, 0); p.laneB.assign((size_t)lanes, 0); }
    {
        std::vector<int64_t> idx(lp.size(), 0);
        for (int64_t l = 0; l < lanes; ++l) {
            int64_t rA = 0, rB = 0, wa = 1, wb = 1, offD = 0;
            for (size_t i = 0; i < lp.size(); ++i) {
                const DMode& d = dm[(size_t)lp[i]->mode];
                offD += idx[i] * lp[i]->mult * d.m.sD;
                if (direct) {
                    p.laneA[(size_t)l] += idx[i] * lp[i]->mult * d.m.sA;
                    p.laneB[(size_t)l] += idx[i] * lp[i]->mult * d.m.sB;
                }
                if (d.inA) { rA += idx[i] * wa; wa *= lp[i]->count; }
                if (d.inB) { rB += idx[i] * wb; wb *= lp[i]->count; }
            }
            p.rowAB[(size_t)l] = (uint32_t)rA | ((uint32_t)rB << 16);
            p.dD[(size_t)l] = offD;
            for (size_t i = 0; i < lp.size(); ++i) {
                if (++idx[i] < lp[i]->count) break;
                idx[i] = 0;
            }
        }
    }
    // register-block offsets in D
    auto reg_offsets = [&](int role, int64_t n, int64_t* dst, int64_t Mode::*stride) {
        std::vector<const Piece*> rp;
        for (const Piece& pc : pieces) if (pc.role == role) rp.push_back(&pc);
        std::vector<int64_t> idx(rp.size(), 0);
        for (int64_t r = 0; r < n; ++r) {
            int64_t off = 0;
            for (size_t i = 0; i < rp.size(); ++i) off += idx[i] * rp[i]->mult * (dm[(size_t)rp[i]->mode].m.*stride);
            dst[r] = off;
            for (size_t i = 0; i < rp.size(); ++i) {
                if (++idx[i] < rp[i]->count) break;
                idx[i] = 0;
            }
        }
    };
    for (int i = 0; i < kStreamRegBlock; ++i) p.dRegA[i] = p.dRegB[i] = p.aReg[i] = p.bReg[i] = p.aK[i] = p.bK[i] = 0;
    reg_offsets(REG_A, ra, p.dRegA, &Mode::sD);
    reg_offsets(REG_B, rb, p.dRegB, &Mode::sD);
    if (direct) {
        reg_offsets(REG_A, ra, p.aReg, &Mode::sA);
        reg_offsets(REG_B, rb, p.bReg, &Mode::sB);
    }

    // staging lists.  Rows are numbered over the pieces the operand carries: LANE pieces first
    // (as in the lane tables), then its REG pieces.
    const std::vector<int64_t> kA = offset_table(an.K, 0, 0), kB = offset_table(an.K, 1, 0);
    if (direct)
        for (int k = 0; k < K; ++k) { p.aK[k] = kA[(size_t)k]; p.bK[k] = kB[(size_t)k]; }
    auto items = [&](bool forA, int64_t rows, const std::vector<int64_t>& kOff) {
        std::vector<const Piece*> op;
        for (const Piece& pc : pieces)
            if (pc.role == LANE && (forA ? dm[(size_t)pc.mode].inA : dm[(size_t)pc.mode].inB)) op.push_back(&pc);
        for (const Piece& pc : pieces)
            if (pc.role == (forA ? REG_A : REG_B)) op.push_back(&pc);
        std::vector<StreamItem> v;
        v.reserve((size_t)rows * (size_t)K);
        std::vector<int64_t> idx(op.size(), 0);
        for (int64_t r = 0; r < rows; ++r) {
            int64_t src = 0;
            uint32_t digit = 0;
            for (size_t i = 0; i < op.size(); ++i) {
                const Mode& m = dm[(size_t)op[i]->mode].m;
                src += idx[i] * op[i]->mult * (forA ? m.sA : m.sB);
                if (has_split && op[i] == &pieces[(size_t)last_lane]) digit = (uint32_t)idx[i];
            }
            for (int k = 0; k < K; ++k) v.push_back({src + kOff[(size_t)k], (uint32_t)(r * K + k), digit});
            for (size_t i = 0; i < op.size(); ++i) {
                if (++idx[i] < op[i]->count) break;
                idx[i] = 0;
            }
        }
        // sorted by source so that neighbouring lanes read neighbouring addresses whatever the
        // operand's own mode order is
        std::stable_sort(v.begin(), v.end(), [](const StreamItem& a, const StreamItem& b) { return a.src < b.src; });
        return v;
    };
    if (!direct) {
        p.itemsA = items(true, rowsA, kA);
        p.itemsB = items(false, rowsB, kB);
    }

    // LDS bank conflicts of a flat tile.  Rows are numbered in D's lane order, so the lanes read
    // consecutive rows; the staging writes go in the operand's own address order, which for a
    // permuted operand is a large power-of-two stride in row numbers: every lane of a quarter
    // wave would hit the same bank.  Rows are therefore spread out, r -> r + (r >> s1) * p1 +
    // (r >> s2) * p2, with the pair of skews that a simulation of both access patterns (16
    // lanes per cycle, 32 banks of 4 bytes) finds cheapest; LDS grows by at most a quarter.
    if (!blocked) {
        const int words = std::max(1, elem_bytes / 4);
        auto cost_of = [&](const std::vector<uint32_t>& rows_in_issue_order) {
            // rows_in_issue_order: the row each consecutive lane touches, instruction after instruction
            int64_t cycles = 0;
            int hits[32];
            for (size_t at = 0; at < rows_in_issue_order.size(); at += 16) {
                for (int b = 0; b < 32; ++b) hits[b] = 0;
                int worst = 0;
                for (size_t l = at; l < std::min(at + 16, rows_in_issue_order.size()); ++l) {
                    const int b = (int)(((int64_t)rows_in_issue_order[l] * K * words) % 32);
                    worst = std::max(worst, ++hits[b]);
                }
                cycles += worst;
            }
            return cycles;
        };
        auto spread = [&](std::vector<StreamItem>& its, bool forA, int64_t* rows) {
            std::vector<uint32_t> readers((size_t)lanes), writers(its.size());
            auto remap = [](uint32_t r, int s1, int p1, int s2, int p2) {
                return r + (s1 >= 0 ? (r >> s1) * (uint32_t)p1 : 0u) + (s2 >= 0 ? (r >> s2) * (uint32_t)p2 : 0u);
            };
            int best[4] = {-1, 0, -1, 0};
            int64_t best_cost = -1;
            static const int kShift[] = {-1, 2, 3, 4, 5, 6, 7, 8};
            for (int s1 : kShift)
                for (int s2 : kShift) {
                    if (s2 >= 0 && s2 <= s1) continue;
                    for (int p1 = (s1 >= 0 ? 1 : 0); p1 <= (s1 >= 0 ? 2 : 0); ++p1)
                        for (int p2 = (s2 >= 0 ? 1 : 0); p2 <= (s2 >= 0 ? 2 : 0); ++p2) {
                            const uint32_t top = remap((uint32_t)*rows - 1, s1, p1, s2, p2) + 1;
                            if (top > 65535 || (int64_t)top * 4 > *rows * 5) continue;
                            for (int64_t l = 0; l < lanes; ++l) {
                                const uint32_t r = forA ? (p.rowAB[(size_t)l] & 0xffffu) : (p.rowAB[(size_t)l] >> 16);
                                readers[(size_t)l] = remap(r, s1, p1, s2, p2);
                            }
                            for (size_t i = 0; i < its.size(); ++i) writers[i] = remap(its[i].slot / (uint32_t)K, s1, p1, s2, p2);
                            const int64_t c = cost_of(readers) + cost_of(writers);
                            if (best_cost < 0 || c < best_cost) { best_cost = c; best[0] = s1; best[1] = p1; best[2] = s2; best[3] = p2; }
                        }
                }
            if (best[0] < 0 && best[2] < 0) return;
            for (StreamItem& it : its) it.slot = remap(it.slot / (uint32_t)K, best[0], best[1], best[2], best[3]) * (uint32_t)K + it.slot % (uint32_t)K;
            for (int64_t l = 0; l < lanes; ++l) {
                uint32_t& w = p.rowAB[(size_t)l];
                const uint32_t a = w & 0xffffu, b = w >> 16;
                w = forA ? (remap(a, best[0], best[1], best[2], best[3]) | (b << 16)) : (a | (remap(b, best[0], best[1], best[2], best[3]) << 16));
            }
            *rows = remap((uint32_t)*rows - 1, best[0], best[1], best[2], best[3]) + 1;
        };
        int64_t padA = rowsA, padB = rowsB;
        spread(p.itemsA, true, &padA);
        spread(p.itemsB, false, &padB);
        p.rowsA = (int32_t)padA; p.rowsB = (int32_t)padB;
        p.lds_bytes = (size_t)(padA + padB) * (size_t)K * (size_t)elem_bytes;
        if (p.lds_bytes > 64 * 1024) return false;
    }

    // Lines that collide in the L2.  When every stride of an operand inside the tile is a multiple
    // of 128 KB (power-of-two extents, the operand's fastest mode a different one from D's), the
    // cache lines a tile reads from it agree in all address bits 7 .. 16 -- the bits that pick the
    // L2 channel and the set.  A hundred such misses in flight at once overflow the set's ways and
    // stall the channel's tag pipeline for everybody (measured: ten times the tag stalls, 2.9 TB/s
    // chip-wide where the same tile on strides padded by one line streams at 4.0).  Such a plan is
    // marked `paced`: its kernel keeps only a few of a tile's loads in flight per thread.
    if (!blocked) {
        auto collides = [&](const std::vector<StreamItem>& its) {
            std::vector<int64_t> lines, classes;
            for (const StreamItem& it : its) {
                const int64_t line = (it.src * (int64_t)elem_bytes) >> 7;
                lines.push_back(line);
                classes.push_back(line & 1023);
            }
            auto distinct = [](std::vector<int64_t>& v) {
                std::sort(v.begin(), v.end());
                return (int64_t)(std::unique(v.begin(), v.end()) - v.begin());
            };
            const int64_t nl = distinct(lines), nc = distinct(classes);
            return nl >= 64 && nl >= 64 * nc;
        };
        p.paced = collides(p.itemsA) || collides(p.itemsB);
    }

    // outer modes: what the pieces leave of every D mode, the ragged mode first (its chunk index
    // decides how much of the last tile is valid)
    std::vector<int64_t> taken(dm.size(), 1);
    for (const Piece& pc : pieces) taken[(size_t)pc.mode] *= pc.count;
    struct Outer { int64_t ext, sA, sB, sD; };
    std::vector<Outer> outer;
    auto push_outer = [&](size_t i) {
        const Mode& m = dm[i].m;
        const int64_t ext = (m.extent + taken[i] - 1) / taken[i];
        if (ext > 1 || (has_split && (int)i == pieces[(size_t)last_lane].mode)) outer.push_back({ext, m.sA * taken[i], m.sB * taken[i], m.sD * taken[i]});
    };
    if (has_split) push_outer((size_t)pieces[(size_t)last_lane].mode);
    for (size_t i = 0; i < dm.size(); ++i)
        if (!(has_split && (int)i == pieces[(size_t)last_lane].mode)) push_outer(i);
    p.num_tiles = 1;
    for (const Outer& o : outer) p.num_tiles *= o.ext;

    // two-level table of tile base offsets: the first outer modes (product near the square
    // root of the tile count) form the low part, the rest the high part
    size_t nlo = 0;
    p.outer_lo = 1;
    while (nlo < outer.size() && p.outer_lo * p.outer_lo < p.num_tiles) p.outer_lo *= outer[nlo++].ext;
    if (has_split && nlo == 0) { nlo = 1; p.outer_lo = outer[0].ext; }
    auto table = [&](size_t first, size_t last, bool with_digits) {
        int64_t n = 1;
        for (size_t i = first; i < last; ++i) n *= outer[i].ext;
        std::vector<int64_t> t((size_t)n * 4, 0);
        std::vector<int64_t> ix(std::max<size_t>(1, last - first), 0);
        for (int64_t r = 0; r < n; ++r) {
            for (size_t i = first; i < last; ++i) {
                t[(size_t)r * 4 + 0] += ix[i - first] * outer[i].sA;
                t[(size_t)r * 4 + 1] += ix[i - first] * outer[i].sB;
                t[(size_t)r * 4 + 2] += ix[i - first] * outer[i].sD;
            }
            if (with_digits) t[(size_t)r * 4 + 3] = has_split ? std::min<int64_t>(p.chunk, p.split_extent - ix[0] * p.chunk) : 1;
            for (size_t i = first; i < last; ++i) {
                if (++ix[i - first] < outer[i].ext) break;
                ix[i - first] = 0;
            }
        }
        return t;
    };
    p.tabLo = table(0, nlo, true);
    p.tabHi = table(nlo, outer.size(), false);
    p.staged_per_output = (double)(p.itemsA.size() + p.itemsB.size()) / (double)(lanes * ra * rb);
    p.ok = true;
    *out = std::move(p);
    return true;
}

}  // namespace

bool stream_preferred(const Analysis& an, int elem_bytes) {
    // Flop per byte if every operand moved exactly once (beta taken as 0: an upper bound).
    if (is_widened(an.dtype, an.precision)) return false;       // the streaming kernels compute in the storage type
    const double flop = (is_complex(an.dtype) ? 8.0 : 2.0) * (double)an.sizeH * an.sizeM * an.sizeN * an.sizeK;
    const double bytes = (double)elem_bytes * ((double)an.sizeH * an.sizeM * an.sizeK + (double)an.sizeH * an.sizeN * an.sizeK +
                                               (double)an.sizeH * an.sizeM * an.sizeN);
    const double ridge = real_bytes_of(an.dtype) == 4 ? 19.7 : 9.8;     // peak matrix flop/s over peak HBM byte/s
    return an.sizeK <= 32 && flop / bytes < ridge;
}

StreamPlan plan_stream(const Analysis& an, int elem_bytes, bool allow_blocked) {
    StreamPlan p;
    if (an.sizeK > 64 || is_widened(an.dtype, an.precision)) return p;
    // every mode that indexes D, D-fastest first
    std::vector<DMode> dm;
    for (const Mode& m : an.H) dm.push_back({m, true, true});
    for (const Mode& m : an.M) dm.push_back({m, true, false});
    for (const Mode& m : an.N) dm.push_back({m, false, true});
    std::stable_sort(dm.begin(), dm.end(), [](const DMode& a, const DMode& b) { return iabs64(a.m.sD) < iabs64(b.m.sD); });
    const int K = (int)an.sizeK;

    // ---- blocked tile: up to 256 lanes along D's fastest modes (whole modes or divisors, so no
    // chunk is ragged), then up to 4 x 4 register-blocked indices of free modes of A and of B.
    // If the operand rows of such a tile do not fit a workgroup's registers / LDS, smaller
    // lane counts and register blocks are tried, most operand reuse first.
    if (allow_blocked && (K == 1 || K == 2 || K == 4)) {
        static const int kTry[][2] = {{256, 4}, {128, 4}, {256, 2}, {64, 4}, {128, 2}};
        for (const auto& t : kTry) {
            const int64_t lane_cap = t[0], reg_cap = t[1];
            std::vector<Piece> pieces;
            std::vector<int64_t> left(dm.size());       // what is still untaken of each mode
            std::vector<int64_t> mult(dm.size(), 1);
            for (size_t i = 0; i < dm.size(); ++i) left[i] = dm[i].m.extent;
            int64_t lanes = 1;
            size_t pos = 0;
            for (; pos < dm.size(); ++pos) {
                const int64_t c = largest_divisor_at_most(left[pos], lane_cap / lanes);
                if (c <= 1) break;
                pieces.push_back({(int)pos, c, 1, LANE});
                lanes *= c; left[pos] /= c; mult[pos] *= c;
                if (left[pos] > 1) break;
            }
            int64_t ra = 1, rb = 1;
            for (size_t i = pos; i < dm.size() && i < pos + 8; ++i) {
                if (left[i] <= 1 || dm[i].inA == dm[i].inB) continue;      // hyper modes give no reuse
                int64_t& r = dm[i].inA ? ra : rb;
                const int64_t c = largest_divisor_at_most(left[i], reg_cap / r);
                if (c <= 1) continue;
                pieces.push_back({(int)i, c, mult[i], dm[i].inA ? REG_A : REG_B});
                r *= c; left[i] /= c; mult[i] *= c;
            }
            if (ra * rb > 1 && lanes >= 64 && build(dm, pieces, false, an, elem_bytes, &p)) return p;
        }
    }

    // ---- flat tile.  It starts with a run of D's fastest mode; if A's or B's own fastest mode is
    // a different mode of D, a run of that mode is taken too, so that all three tensors are
    // touched in runs of whole cache lines (LDS does the transposition).  The rest of the tile
    // is filled with D's next modes; only the last piece may be ragged.
    const int64_t run = std::max<int64_t>(4, 128 / elem_bytes);
    auto fastest_of = [&](bool forA) {
        int best = -1;
        for (size_t i = 0; i < dm.size(); ++i) {
            if (!(forA ? dm[i].inA : dm[i].inB)) continue;
            const int64_t s = iabs64(forA ? dm[i].m.sA : dm[i].m.sB);
            if (s == 0) continue;
            if (best < 0 || s < iabs64(forA ? dm[(size_t)best].m.sA : dm[(size_t)best].m.sB)) best = (int)i;
        }
        // a contracted mode may be faster still; then the operand is read in runs along K anyway
        for (const Mode& k : an.K)
            if (best >= 0 && iabs64(forA ? k.sA : k.sB) != 0 &&
                iabs64(forA ? k.sA : k.sB) < iabs64(forA ? dm[(size_t)best].m.sA : dm[(size_t)best].m.sB) && an.sizeK >= 4)
                return -1;
        return best;
    };
    std::vector<int> fast;          // distinct D modes that must contribute a run
    if (!dm.empty()) fast.push_back(0);
    for (int f : {fastest_of(true), fastest_of(false)})
        if (f >= 0 && std::find(fast.begin(), fast.end(), f) == fast.end()) fast.push_back(f);
    for (int target = kStreamThreads * kStreamPerThread; target >= 64; target /= 2) {
        std::vector<Piece> pieces;
        std::vector<int64_t> left(dm.size());
        for (size_t i = 0; i < dm.size(); ++i) left[i] = dm[i].m.extent;
        int64_t lanes = 1;
        if (fast.size() > 1) {
            // equal shares of the tile for each run, at least a cache line where the extent allows
            int64_t share = 1;
            while ((share * 2) * (share * 2) * (fast.size() > 2 ? share * 2 : 1) <= target) share *= 2;
            share = std::max(share, std::min<int64_t>(run, target));
            // Sizes are handed out to the operands' runs first and to D's run last: a read
            // that covers half a 128-byte line still fetches the whole line, whereas 64-byte
            // stores cost nothing extra.  The pieces keep D's run first (consecutive lanes write
            // consecutive elements).
            std::vector<int64_t> size(fast.size(), 1);
            for (size_t q = 0; q < fast.size(); ++q) {
                const size_t at = (q + 1) % fast.size();          // order: the operands' runs, then D's run (index 0)
                const int f = fast[at];
                const int64_t c = largest_divisor_at_most(left[(size_t)f], std::min<int64_t>(share, target / lanes));
                if (c <= 1) continue;
                size[at] = c;
                lanes *= c; left[(size_t)f] /= c;
            }
            for (size_t q = 0; q < fast.size(); ++q)
                if (size[q] > 1) pieces.push_back({fast[q], size[q], 1, LANE});
        }
        for (size_t i = 0; i < dm.size() && lanes < target; ++i) {
            if (left[i] <= 1) continue;
            const bool untouched = left[i] == dm[i].m.extent;
            if (untouched && lanes * left[i] <= target) {
                pieces.push_back({(int)i, left[i], 1, LANE});
                lanes *= left[i]; left[i] = 1;
            } else if (untouched) {
                const int64_t chunk = std::min<int64_t>(left[i], std::max<int64_t>(1, target / lanes));
                if (chunk > 1) { pieces.push_back({(int)i, chunk, 1, LANE}); lanes *= chunk; }
                break;          // a ragged piece must be the last one
            }
        }
        if (build(dm, pieces, true, an, elem_bytes, &p)) return p;
    }
    return p;
}

}  // namespace tcx
