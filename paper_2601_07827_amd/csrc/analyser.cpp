// Index analyser: validation, classification of labels into Hadamard / free / contracted
// groups (paper, Secs. "Case 1", "Case 2"), merging of repeated labels (Sec. "Case 3",
// Note 6), removal of extent-1 modes, fusion of modes that are contiguous in every tensor
// that carries them, and ordering of each group so that tiles follow the tensors' own
// fastest modes.  Pure host code.
#include <algorithm>
#include <cstdlib>
#include <map>

#include "tcx_internal.hpp"

namespace tcx {
namespace {

struct Merged {            // one distinct label of one tensor
    int64_t extent = 0;
    int64_t stride = 0;    // sum over the label's occurrences (Note 6)
    bool present = false;
};

using LabelMap = std::map<int64_t, Merged>;

// Collapse repeated labels.  Fails if one label carries two extents inside the tensor.
bool merge_labels(const TensorDesc& t, const int64_t* lab, LabelMap* out) {
    for (size_t i = 0; i < t.extent.size(); ++i) {
        Merged& m = (*out)[lab[i]];
        if (m.present && m.extent != t.extent[i]) return false;
        m.present = true;
        m.extent = t.extent[i];
        m.stride += t.stride[i];
    }
    return true;
}

inline int64_t iabs(int64_t x) { return x < 0 ? -x : x; }

// Fuse y into x when, in every tensor that carries the group, y continues x's run:
// stride(y) == stride(x) * extent(x).  A tensor that does not carry the group has
// stride 0 for both, which satisfies the same equation.
void fuse(std::vector<Mode>* g) {
    bool changed = true;
    while (changed) {
        changed = false;
        for (size_t x = 0; x < g->size() && !changed; ++x)
            for (size_t y = 0; y < g->size() && !changed; ++y) {
                if (x == y) continue;
                Mode& a = (*g)[x];
                const Mode& b = (*g)[y];
                if (b.sA == a.sA * a.extent && b.sB == a.sB * a.extent && b.sD == a.sD * a.extent) {
                    a.extent *= b.extent;
                    g->erase(g->begin() + (long)y);
                    changed = true;
                }
            }
    }
}

int64_t Mode::*const kStride[3] = {&Mode::sA, &Mode::sB, &Mode::sD};

void sort_by(std::vector<Mode>* g, int which) {
    std::stable_sort(g->begin(), g->end(), [which](const Mode& a, const Mode& b) {
        return iabs(a.*kStride[which]) < iabs(b.*kStride[which]);
    });
}

// Smallest non-zero |stride| of tensor `which` over a group; INT64_MAX if none.
int64_t min_stride(const std::vector<Mode>& g, int which) {
    int64_t best = INT64_MAX;
    for (const Mode& m : g) {
        const int64_t s = iabs(m.*kStride[which]);
        if (s != 0 && s < best) best = s;
    }
    return best;
}

int64_t product(const std::vector<Mode>& g) {
    int64_t p = 1;
    for (const Mode& m : g) p *= m.extent;
    return p;
}

}  // namespace

tcx_error_t analyse(const TensorDesc& A, const int64_t* labA, const TensorDesc& B, const int64_t* labB,
                    const TensorDesc& C, const int64_t* labC, const TensorDesc& D, const int64_t* labD,
                    int opA, int opB, int opC, int opD, int precision, Analysis* out) {
    // ---- a0: validation ------------------------------------------------------------------
    if (A.dtype != B.dtype || A.dtype != C.dtype || A.dtype != D.dtype) return TCX_ERR_DTYPE_MIX;
    for (int op : {opA, opB, opC, opD})
        if (op != TCX_OP_IDENTITY && op != TCX_OP_CONJ) return TCX_ERR_UNSUPPORTED_OP;
    if (opD != TCX_OP_IDENTITY) return TCX_ERR_UNSUPPORTED_OP;
    if (!valid_dtype(A.dtype)) return TCX_ERR_BAD_DTYPE;
    if (precision != TCX_PREC_DEFAULT && precision != TCX_PREC_F64) return TCX_ERR_UNSUPPORTED_PRECISION;

    LabelMap a, b, c, d;
    if (!merge_labels(A, labA, &a) || !merge_labels(B, labB, &b) || !merge_labels(C, labC, &c) ||
        !merge_labels(D, labD, &d))
        return TCX_ERR_EXTENT_MISMATCH;
    // one label, one extent, across tensors (Sec. Preliminaries)
    for (const LabelMap* x : {&a, &b, &c, &d})
        for (const LabelMap* y : {&a, &b, &c, &d})
            for (const auto& kv : *x) {
                auto it = y->find(kv.first);
                if (it != y->end() && it->second.extent != kv.second.extent) return TCX_ERR_EXTENT_MISMATCH;
            }
    // C is D: same label set, and per label the same extent and (merged) stride (Note 5)
    if (c.size() != d.size()) return TCX_ERR_CD_MISMATCH;
    for (const auto& kv : d) {
        auto it = c.find(kv.first);
        if (it == c.end() || it->second.extent != kv.second.extent) return TCX_ERR_CD_MISMATCH;
        if (kv.second.extent > 1 && it->second.stride != kv.second.stride) return TCX_ERR_CD_MISMATCH;
    }
    // no two index tuples of D may share an address: with modes sorted by |stride| each
    // stride has to clear everything the smaller ones can reach
    {
        std::vector<std::pair<int64_t, int64_t>> se;
        for (const auto& kv : d)
            if (kv.second.extent > 1) se.push_back({iabs(kv.second.stride), kv.second.extent});
        std::sort(se.begin(), se.end());
        int64_t reach = 0;
        for (const auto& p : se) {
            if (p.first <= reach) return TCX_ERR_D_ALIASING;
            if (p.first > (INT64_MAX - reach) / p.second) return TCX_ERR_TOO_LARGE;
            reach += p.first * (p.second - 1);
        }
    }

    // ---- a1: classification by set membership ----------------------------------------------
    Analysis r;
    r.dtype = D.dtype;
    r.precision = precision;
    r.opA = opA; r.opB = opB; r.opC = opC;
    if (!is_complex(r.dtype)) r.opA = r.opB = r.opC = TCX_OP_IDENTITY;   // conj of a real number
    auto stride_in = [](const LabelMap& m, int64_t lab) {
        auto it = m.find(lab);
        return it == m.end() ? (int64_t)0 : it->second.stride;
    };
    LabelMap all = a;
    all.insert(b.begin(), b.end());
    all.insert(d.begin(), d.end());
    std::vector<Mode> onlyA, onlyB;
    for (const auto& kv : all) {
        const int64_t lab = kv.first;
        const bool inA = a.count(lab), inB = b.count(lab), inD = d.count(lab);
        Mode m{kv.second.extent, stride_in(a, lab), stride_in(b, lab), stride_in(d, lab)};
        if (m.extent == 1) continue;                       // a2: extent-1 modes address nothing
        if (inA && inB && inD) r.H.push_back(m);
        else if (inA && inB) r.K.push_back(m);
        else if (inA && inD) r.M.push_back(m);
        else if (inB && inD) r.N.push_back(m);
        else if (inA) onlyA.push_back(m);                  // Sec. "Case 4": summed inside A
        else if (inB) onlyB.push_back(m);                  // ... inside B
        else r.M.push_back(m);                             // Sec. "Case 5": in D (and C) only -- a free mode that neither
                                                           // operand moves along (strides 0): the product is repeated
    }
    // Case 4: the operand is reduced over its isolated labels first (one pass over it, into
    // workspace memory); from here on sA / sB of the other modes address that dense result.
    auto pre_reduce = [&](const std::vector<Mode>& only, int which, Reduction* red) {
        if (only.empty()) return;
        red->active = true;
        for (const Mode& m : only) { red->sumExt.push_back(m.extent); red->sumSrc.push_back(m.*kStride[which]); }
        std::vector<Mode*> kept;
        for (std::vector<Mode>* g : {&r.H, &r.M, &r.N, &r.K})
            for (Mode& m : *g)
                if (m.*kStride[which] != 0) kept.push_back(&m);
        std::stable_sort(kept.begin(), kept.end(), [which](const Mode* x, const Mode* y) {
            return iabs(x->*kStride[which]) < iabs(y->*kStride[which]);
        });
        int64_t run = 1;
        for (Mode* m : kept) {
            red->keepExt.push_back(m->extent);
            red->keepSrc.push_back(m->*kStride[which]);
            m->*kStride[which] = run;
            run *= m->extent;
        }
        red->count = run;
    };
    pre_reduce(onlyA, 0, &r.redA);
    pre_reduce(onlyB, 1, &r.redB);
    if ((int)(r.redA.keepExt.size()) > kMaxGenericModes || (int)r.redA.sumExt.size() > kMaxGenericModes ||
        (int)(r.redB.keepExt.size()) > kMaxGenericModes || (int)r.redB.sumExt.size() > kMaxGenericModes)
        return TCX_ERR_TOO_LARGE;

    // ---- a2: fuse, then order each group -----------------------------------------------------
    fuse(&r.H); fuse(&r.M); fuse(&r.N); fuse(&r.K);
    r.sizeH = product(r.H); r.sizeM = product(r.M); r.sizeN = product(r.N); r.sizeK = product(r.K);

    // Which group holds each tensor's fastest (smallest-stride) mode, hyper modes aside.
    const int64_t aM = min_stride(r.M, 0), aK = min_stride(r.K, 0);
    const int64_t bN = min_stride(r.N, 1), bK = min_stride(r.K, 1);
    const int64_t dM = min_stride(r.M, 2), dN = min_stride(r.N, 2);
    r.a_k_fastest = aK < aM;
    r.b_k_fastest = bK < bN;
    r.d_n_fastest = dN < dM;
    // Order inside each group.  A tile takes the first modes of M and of N as its rows and
    // columns, a slab the first modes of K, so what matters is which modes come first: the
    // fastest modes of each tensor that make up a 128-byte line should lie inside the tile, or
    // every access to that tensor touches a line for one element.  M: D's line modes first (by
    // D's stride: consecutive lanes store consecutive elements), then A's line modes, then the
    // rest by the stride of the tensor whose fastest mode the group holds (D if D's fastest mode
    // is an M mode, else A).  N likewise with B.  K: the line modes of whichever input is
    // K-fastest (both: the larger operand first), then the rest by that input's stride.
    const int64_t line = 128 / elem_bytes_of(r.dtype);
    auto line_strides = [&](int which) {
        // strides (in tensor `which`) of its fastest modes, up to a line's worth of elements
        std::vector<std::pair<int64_t, int64_t>> se;
        for (const std::vector<Mode>* g : {&r.H, &r.M, &r.N, &r.K})
            for (const Mode& m : *g)
                if (m.*kStride[which] != 0) se.push_back({iabs(m.*kStride[which]), m.extent});
        std::sort(se.begin(), se.end());
        std::vector<int64_t> out;
        int64_t have = 1;
        for (const auto& p : se) {
            if (have >= line) break;
            out.push_back(p.first);
            have *= p.second;
        }
        return out;
    };
    auto order = [&](std::vector<Mode>* g, std::initializer_list<int> first, int rest) {
        std::vector<Mode> left = *g, done;
        for (int which : first) {
            const std::vector<int64_t> ls = line_strides(which);
            sort_by(&left, which);
            for (size_t i = 0; i < left.size();) {
                if (std::find(ls.begin(), ls.end(), iabs(left[i].*kStride[which])) != ls.end()) {
                    done.push_back(left[i]);
                    left.erase(left.begin() + (long)i);
                } else {
                    ++i;
                }
            }
        }
        sort_by(&left, rest);
        done.insert(done.end(), left.begin(), left.end());
        *g = done;
    };
    order(&r.M, {2, 0}, !r.d_n_fastest ? 2 : 0);
    order(&r.N, {2, 1}, r.d_n_fastest ? 2 : 1);
    int k_anchor = 0;
    if (r.a_k_fastest && r.b_k_fastest) {
        const int64_t sizeA = r.sizeM * r.sizeK, sizeB = r.sizeN * r.sizeK;
        k_anchor = sizeA >= sizeB ? 0 : 1;
    } else if (r.b_k_fastest) {
        k_anchor = 1;
    }
    if (k_anchor == 0) order(&r.K, {0, 1}, 0);
    else order(&r.K, {1, 0}, 1);
    sort_by(&r.H, 2);

    if ((int)(r.H.size() + r.M.size() + r.N.size()) > kMaxGenericModes || (int)r.K.size() > kMaxGenericModes)
        return TCX_ERR_TOO_LARGE;

    // ---- a3: path ------------------------------------------------------------------------------
    // The tiled MFMA path needs offset tables over M, N and K and pays off once a tile has
    // real work; everything else runs on the generic kernel.
    const int64_t table_limit = (int64_t)1 << 27;
    const bool tables_ok = r.sizeM <= table_limit && r.sizeN <= table_limit && r.sizeK <= table_limit;
    const bool tiled = tables_ok && (int)r.H.size() <= kMaxHModes && r.sizeM * r.sizeN >= 256 && r.sizeK >= 2;
    r.path = tiled ? TCX_PATH_GETT_MFMA : TCX_PATH_GENERIC;
    r.variant = -1;   // chosen by the API layer from the compiled instantiations
    *out = r;
    return TCX_SUCCESS;
}

std::vector<int64_t> offset_table(const std::vector<Mode>& modes, int which, int64_t padded) {
    int64_t n = 1;
    for (const Mode& m : modes) n *= m.extent;
    std::vector<int64_t> t((size_t)std::max(n, padded), 0);
    std::vector<int64_t> idx(modes.size(), 0);
    int64_t off = 0;
    for (int64_t g = 0; g < n; ++g) {
        t[(size_t)g] = off;
        for (size_t k = 0; k < modes.size(); ++k) {      // odometer, first mode fastest
            const int64_t s = modes[k].*kStride[which];
            if (++idx[k] < modes[k].extent) { off += s; break; }
            off -= s * (modes[k].extent - 1);
            idx[k] = 0;
        }
    }
    return t;
}

}  // namespace tcx
