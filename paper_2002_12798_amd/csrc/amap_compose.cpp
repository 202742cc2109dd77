// Host-side map composer: builds, for "operator applied to the tensor a map
// describes", the composed map (paper Section 2.1, eq. 3 and eq. 4; with the
// operators written in gather form the store map is the identity and the
// composition is  g' = g o f  where f is the operator's own index function).
//
// The paper delegates reverse and composition of (quasi-)affine functions to
// a Presburger-arithmetic library.  Here the algebra is written out for the
// operator set at hand, on the strided normal form described in amap_map.hpp:
// every operator only re-labels, clips, shifts or re-digits the dst side of a
// piece, while the source strides ride along with the loops.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <numeric>

#include "amap_map.hpp"
#include "amap_plan.hpp"

using namespace amap_detail;

namespace amap_detail {

std::vector<int64_t> row_major_strides(const std::vector<int64_t> &shape) {
    std::vector<int64_t> s(shape.size(), 1);
    for (int k = (int)shape.size() - 2; k >= 0; --k) s[k] = s[k + 1] * shape[k + 1];
    return s;
}

static inline int64_t fdiv(int64_t a, int64_t b) {  // floor(a / b), b > 0
    int64_t q = a / b;
    return (a % b != 0 && a < 0) ? q - 1 : q;
}
static inline int64_t cdiv(int64_t a, int64_t b) {  // ceil(a / b), b > 0
    return -fdiv(-a, b);
}

static void sort_iter(Piece &p) {
    p.it.erase(std::remove_if(p.it.begin(), p.it.end(), [](const IterDim &d) { return d.extent == 1; }),
               p.it.end());
    std::stable_sort(p.it.begin(), p.it.end(), [](const IterDim &a, const IterDim &b) {
        if (a.dim != b.dim) return a.dim < b.dim;
        return a.mult > b.mult;
    });
}

// ---------------------------------------------------------------- program

bool eval_program(const PNode *n, const int64_t *idx_in, int *src, int64_t *off, uint32_t *fill) {
    int64_t idx[kMaxRank], tmp[kMaxRank];
    int rank = (int)n->shape.size();
    for (int k = 0; k < rank; ++k) idx[k] = idx_in[k];
    for (;;) {
        switch (n->kind) {
        case PNode::SOURCE: {
            int64_t o = 0;
            for (int k = 0; k < rank; ++k) o = o * n->shape[k] + idx[k];
            *src = n->src_id;
            *off = o;
            return true;
        }
        case PNode::TRANSPOSE: {
            for (int k = 0; k < rank; ++k) tmp[n->perm[k]] = idx[k];
            for (int k = 0; k < rank; ++k) idx[k] = tmp[k];
            n = n->kids[0].get();
            break;
        }
        case PNode::RESHAPE: {
            int64_t L = 0;
            for (int k = 0; k < rank; ++k) L = L * n->shape[k] + idx[k];
            const PNode *c = n->kids[0].get();
            int cr = (int)c->shape.size();
            for (int k = cr - 1; k >= 0; --k) {
                idx[k] = L % c->shape[k];
                L /= c->shape[k];
            }
            n = c;
            rank = cr;
            break;
        }
        case PNode::SLICE:
            idx[n->axis] = n->begin + idx[n->axis] * n->step;
            n = n->kids[0].get();
            break;
        case PNode::REPEAT:
            idx[n->axis] /= n->count;
            n = n->kids[0].get();
            break;
        case PNode::TILE:
            idx[n->axis] %= n->count;
            n = n->kids[0].get();
            break;
        case PNode::PAD: {
            const PNode *c = n->kids[0].get();
            for (int k = 0; k < rank; ++k) {
                idx[k] -= n->lo[k];
                if (idx[k] < 0 || idx[k] >= c->shape[k]) {
                    *fill = n->fill;
                    return false;
                }
            }
            n = c;
            break;
        }
        case PNode::CONCAT: {
            int64_t o = 0;
            size_t m = 0;
            while (idx[n->axis] >= o + n->kids[m]->shape[n->axis]) {
                o += n->kids[m]->shape[n->axis];
                ++m;
            }
            idx[n->axis] -= o;
            n = n->kids[m].get();
            break;
        }
        }
    }
}

// ---------------------------------------------------------------- finalise

std::vector<KDim> merge_loops(std::vector<KDim> dims) {
    std::stable_sort(dims.begin(), dims.end(), [](const KDim &a, const KDim &b) { return a.ds > b.ds; });
    std::vector<KDim> out;
    for (const KDim &d : dims) {
        if (!out.empty() && out.back().ds == d.ds * d.extent && out.back().ss == d.ss * d.extent) {
            out.back().extent *= d.extent;
            out.back().ds = d.ds;
            out.back().ss = d.ss;
        } else {
            out.push_back(d);
        }
    }
    return out;
}

void finalise(amap &m) {
    m.kpieces.clear();
    m.plan.reset();
    if (!m.strided) return;
    auto R = row_major_strides(m.shape);
    int rank = (int)m.shape.size();
    for (const Piece &p : m.pieces) {
        KPiece k;
        k.fill = p.fill;
        k.fill_bits = p.fill_bits;
        k.src = p.src;
        k.sbase = p.sbase;
        k.dbase = 0;
        for (int d = 0; d < rank; ++d) k.dbase += p.lo[d] * R[d];
        for (const IterDim &it : p.it) k.dims.push_back({it.extent, it.mult * R[it.dim], p.fill ? 0 : it.sstride});
        k.dims = merge_loops(std::move(k.dims));
        m.kpieces.push_back(std::move(k));
    }
}

}  // namespace amap_detail

// every builder ends here: derive the kernel-form pieces and the launch plan
// ---- merging of pieces
//
// A split followed by a concat of the parts, a tensor cut into slices that are processed the same
// way and put together again: composition leaves one piece per part although the parts continue
// one another.  Two pieces that are the same box displaced along ONE dst dimension, reading the
// same source (or writing the same constant), are one piece with a longer, or a new, outermost
// loop in that dimension.

static bool same_loops(const std::vector<IterDim> &a, size_t a0, const std::vector<IterDim> &b, size_t b0, bool fill) {
    if (a.size() - a0 != b.size() - b0) return false;
    for (size_t i = a0, j = b0; i < a.size(); ++i, ++j)
        if (a[i].extent != b[j].extent || a[i].mult != b[j].mult || (!fill && a[i].sstride != b[j].sstride)) return false;
    return true;
}

// b lies after a along one dimension: extend a by b if the two form one box
static bool absorb(Piece &a, const Piece &b, int rank) {
    if (a.fill != b.fill || (a.fill ? a.fill_bits != b.fill_bits : a.src != b.src)) return false;
    int d = -1;
    for (int k = 0; k < rank; ++k)
        if (a.lo[k] != b.lo[k]) {
            if (d >= 0) return false;
            d = k;
        }
    if (d < 0) return false;
    const int64_t dlo = b.lo[d] - a.lo[d], ds = a.fill ? 0 : b.sbase - a.sbase;
    if (dlo <= 0) return false;
    std::vector<IterDim> ao, bo, ad, bd;  // loops outside dimension d, loops in it (outermost first)
    for (const IterDim &it : a.it) (it.dim == d ? ad : ao).push_back(it);
    for (const IterDim &it : b.it) (it.dim == d ? bd : bo).push_back(it);
    if (!same_loops(ao, 0, bo, 0, a.fill)) return false;
    for (size_t i = 0; i < ao.size(); ++i)
        if (ao[i].dim != bo[i].dim) return false;
    const bool f = a.fill;
    if (!ad.empty() && ad.size() == bd.size() && same_loops(ad, 1, bd, 1, f) && ad[0].mult == bd[0].mult &&
        (f || ad[0].sstride == bd[0].sstride) && dlo == ad[0].extent * ad[0].mult && ds == ad[0].extent * ad[0].sstride) {
        ad[0].extent += bd[0].extent;  // b continues a's outermost loop
    } else if (ad.size() == bd.size() + 1 && same_loops(ad, 1, bd, 0, f) && dlo == ad[0].extent * ad[0].mult &&
               ds == ad[0].extent * ad[0].sstride) {
        ad[0].extent += 1;             // b is one more iteration of it
    } else if (bd.size() == ad.size() + 1 && same_loops(bd, 1, ad, 0, f) && dlo == bd[0].mult && ds == bd[0].sstride) {
        ad.insert(ad.begin(), IterDim{bd[0].extent + 1, d, bd[0].mult, f ? 0 : bd[0].sstride});  // a is iteration 0 of b's loop
    } else if (same_loops(ad, 0, bd, 0, f)) {
        int64_t span = 0;
        for (const IterDim &it : ad) span += (it.extent - 1) * it.mult;
        if (dlo <= span) return false;  // interleaved boxes: not a loop nest
        if ((int)a.it.size() >= kMaxRank) return false;  // one more loop than the kernels' loop nests hold
        ad.insert(ad.begin(), IterDim{2, d, dlo, ds});  // two copies of the same box: a loop of two
    } else {
        return false;
    }
    a.it = ao;
    a.it.insert(a.it.end(), ad.begin(), ad.end());
    sort_iter(a);
    return true;
}

static void merge_pieces(amap &m) {
    const int rank = (int)m.shape.size();
    std::vector<Piece> &P = m.pieces;
    if (P.size() < 2 || P.size() > 1024) return;
    // neighbours first: by source, then by origin
    std::stable_sort(P.begin(), P.end(), [rank](const Piece &a, const Piece &b) {
        if (a.fill != b.fill) return a.fill < b.fill;
        if (!a.fill && a.src != b.src) return a.src < b.src;
        for (int k = 0; k < rank; ++k)
            if (a.lo[k] != b.lo[k]) return a.lo[k] < b.lo[k];
        return false;
    });
    bool changed = true;
    while (changed) {
        changed = false;
        for (size_t i = 0; i < P.size(); ++i)
            for (size_t j = 0; j < P.size(); ++j) {
                if (i == j || !absorb(P[i], P[j], rank)) continue;
                P.erase(P.begin() + (ptrdiff_t)j);
                if (j < i) --i;
                j = (size_t)-1;  // the grown piece may now reach pieces it could not before
                changed = true;
            }
    }
}

static void finish(amap &m) {
    if (m.strided) merge_pieces(m);
    // a source that no piece reads any more (sliced away, say) is no longer an
    // argument of the map: the caller need not supply it
    if (m.strided && !m.pieces.empty()) {
        std::vector<char> used(m.src_shapes.size(), 0);
        for (const Piece &p : m.pieces)
            if (!p.fill) used[(size_t)p.src] = 1;
        for (size_t i = 0; i < used.size(); ++i)
            if (!used[i]) m.src_shapes[i].clear();
        while (!m.src_shapes.empty() && m.src_shapes.back().empty()) m.src_shapes.pop_back();
    }
    finalise(m);
    attach_plan(m);
}

// ---------------------------------------------------------------- helpers

static amap *clone_header(const amap *m) {
    amap *r = new (std::nothrow) amap();
    if (!r) return nullptr;
    r->elem = m->elem;
    r->src_shapes = m->src_shapes;
    r->injective = m->injective;
    return r;
}

static std::shared_ptr<PNode> unary_node(PNode::Kind k, const amap *m, std::vector<int64_t> shape) {
    auto n = std::make_shared<PNode>();
    n->kind = k;
    n->shape = std::move(shape);
    n->kids.push_back(m->prog);
    return n;
}

static bool valid_shape(int rank, const int64_t *shape) {
    if (rank < 1 || rank > kMaxRank || !shape) return false;
    for (int k = 0; k < rank; ++k)
        if (shape[k] < 0) return false;
    return true;
}

#define GUARD_BEGIN try {
#define GUARD_END                     \
    }                                 \
    catch (const std::bad_alloc &) {  \
        return AMAP_E_NOMEM;          \
    }                                 \
    catch (...) {                     \
        return AMAP_E_INVALID;        \
    }

// ---------------------------------------------------------------- source

extern "C" amap_status amap_source(int src_id, int rank, const int64_t *shape, amap_elem es, amap_t **out) {
    GUARD_BEGIN
    if (!out || src_id < 0 || src_id > 4095 || !valid_shape(rank, shape)) return AMAP_E_INVALID;
    if (es != AMAP_B16 && es != AMAP_B32) return AMAP_E_INVALID;
    amap *m = new amap();
    m->elem = (int)es;
    m->shape.assign(shape, shape + rank);
    m->src_shapes.resize(src_id + 1);
    m->src_shapes[src_id] = m->shape;
    auto n = std::make_shared<PNode>();
    n->kind = PNode::SOURCE;
    n->shape = m->shape;
    n->src_id = src_id;
    m->prog = n;
    m->strided = true;
    if (volume_of(m->shape) > 0) {
        Piece p;
        p.src = src_id;
        auto R = row_major_strides(m->shape);
        for (int k = 0; k < rank; ++k)
            if (shape[k] > 1) p.it.push_back({shape[k], k, 1, R[k]});
        m->pieces.push_back(std::move(p));
    }
    finish(*m);
    *out = m;
    return AMAP_OK;
    GUARD_END
}

// ---------------------------------------------------------------- transpose

extern "C" amap_status amap_transpose(const amap_t *m, const int32_t *perm, amap_t **out) {
    GUARD_BEGIN
    if (!m || !perm || !out) return AMAP_E_INVALID;
    int rank = (int)m->shape.size();
    int inv[kMaxRank];
    bool seen[kMaxRank] = {false};
    for (int k = 0; k < rank; ++k) {
        if (perm[k] < 0 || perm[k] >= rank || seen[perm[k]]) return AMAP_E_INVALID;
        seen[perm[k]] = true;
        inv[perm[k]] = k;
    }
    amap *r = clone_header(m);
    if (!r) return AMAP_E_NOMEM;
    std::unique_ptr<amap> hold(r);
    r->shape.resize(rank);
    for (int k = 0; k < rank; ++k) r->shape[k] = m->shape[perm[k]];
    auto n = unary_node(PNode::TRANSPOSE, m, r->shape);
    n->perm.assign(perm, perm + rank);
    r->prog = n;
    r->strided = m->strided;
    if (m->strided) {
        for (const Piece &p : m->pieces) {
            Piece q = p;
            for (int k = 0; k < rank; ++k) q.lo[k] = p.lo[perm[k]];
            for (auto &d : q.it) d.dim = inv[d.dim];
            sort_iter(q);
            r->pieces.push_back(std::move(q));
        }
    }
    finish(*r);
    *out = hold.release();
    return AMAP_OK;
    GUARD_END
}

// ---------------------------------------------------------------- slice

namespace {

struct SliceCtx {
    int axis;
    int64_t b, e, s;
    std::vector<Piece> *out;
    bool ok = true;
};

// Slice one piece whose loops on the axis are `p.it` entries with dim == axis.
void slice_piece(SliceCtx &c, const Piece &p) {
    if (!c.ok) return;
    if ((int64_t)c.out->size() > kMaxPieces) {
        c.ok = false;
        return;
    }
    std::vector<int> on;  // indices of loops on the axis, outermost first
    for (int k = 0; k < (int)p.it.size(); ++k)
        if (p.it[k].dim == c.axis) on.push_back(k);
    const int64_t lo = p.lo[c.axis];
    if (on.empty()) {
        if (lo >= c.b && lo < c.e && (lo - c.b) % c.s == 0) {
            Piece q = p;
            q.lo[c.axis] = (lo - c.b) / c.s;
            c.out->push_back(std::move(q));
        }
        return;
    }
    if (on.size() == 1) {
        // index = lo + i*m must equal b + j*s inside [b, e)
        const IterDim &d = p.it[on[0]];
        const int64_t m = d.mult, n = d.extent;
        const int64_t g = std::gcd(m, c.s);
        const int64_t period = c.s / g;  // spacing of admissible i
        int64_t i_min = std::max<int64_t>(0, cdiv(c.b - lo, m));
        int64_t i_max = std::min<int64_t>(n - 1, fdiv(c.e - 1 - lo, m));
        int64_t i0 = -1;
        for (int64_t i = i_min; i <= i_max && i < i_min + period; ++i)
            if ((lo + i * m - c.b) % c.s == 0) {
                i0 = i;
                break;
            }
        if (i0 < 0) return;
        int64_t cnt = (i_max - i0) / period + 1;
        Piece q = p;
        q.lo[c.axis] = (lo + i0 * m - c.b) / c.s;
        q.sbase += i0 * d.sstride;
        IterDim &qd = q.it[on[0]];
        qd.extent = cnt;
        qd.mult = m / g;
        qd.sstride = d.sstride * period;
        sort_iter(q);
        c.out->push_back(std::move(q));
        return;
    }
    // several loops on the axis and a step: if every loop but the innermost
    // moves by whole steps, the residue class is decided by the innermost loop
    // alone.  Keep its admissible iterations, divide the axis by the step, and
    // what is left is a unit-step slice (this is how slice(repeat(x, r), step r)
    // and slice(reshape(x), step) lose their division).
    if (c.s > 1) {
        bool outer_whole = true;
        for (size_t t = 0; t + 1 < on.size(); ++t) outer_whole = outer_whole && p.it[on[t]].mult % c.s == 0;
        if (outer_whole) {
            const IterDim &d = p.it[on.back()];
            const int64_t g = std::gcd(d.mult, c.s), period = c.s / g;
            int64_t i0 = -1;
            for (int64_t i = 0; i < d.extent && i < period; ++i)
                if ((lo + i * d.mult - c.b) % c.s == 0) {
                    i0 = i;
                    break;
                }
            if (i0 < 0) return;
            Piece q = p;
            q.sbase += i0 * d.sstride;
            IterDim &qd = q.it[on.back()];
            qd.extent = (d.extent - 1 - i0) / period + 1;
            qd.mult = d.mult * period / c.s;
            qd.sstride = d.sstride * period;
            for (size_t t = 0; t + 1 < on.size(); ++t) q.it[on[t]].mult /= c.s;
            q.lo[c.axis] = (lo + i0 * d.mult - c.b) / c.s;  // exact; may be negative until clipped below
            sort_iter(q);
            SliceCtx unit{c.axis, 0, cdiv(c.e - c.b, c.s), 1, c.out};
            slice_piece(unit, q);
            c.ok = c.ok && unit.ok;
            return;
        }
    }
    // several loops on the axis: peel the outermost one
    const IterDim d = p.it[on[0]];
    int64_t inner_span = 0;
    for (size_t t = 1; t < on.size(); ++t) inner_span += (p.it[on[t]].extent - 1) * p.it[on[t]].mult;
    auto fixed_at = [&](int64_t i) {
        Piece q = p;
        q.it.erase(q.it.begin() + on[0]);
        q.lo[c.axis] += i * d.mult;
        q.sbase += i * d.sstride;
        slice_piece(c, q);
    };
    // outer values whose inner range meets [b, e) at all
    int64_t i_first = std::max<int64_t>(0, cdiv(c.b - inner_span - lo, d.mult));
    int64_t i_last = std::min<int64_t>(d.extent - 1, fdiv(c.e - 1 - lo, d.mult));
    if (i_first > i_last) return;
    if (c.s == 1) {
        // outer values whose whole inner range lies inside [b, e)
        int64_t u = std::max<int64_t>(i_first, cdiv(c.b - lo, d.mult));
        int64_t v = std::min<int64_t>(i_last + 1, fdiv(c.e - 1 - inner_span - lo, d.mult) + 1);
        if (u < v) {
            for (int64_t i = i_first; i < u && c.ok; ++i) fixed_at(i);
            Piece q = p;
            q.lo[c.axis] = lo + u * d.mult - c.b;
            q.sbase += u * d.sstride;
            q.it[on[0]].extent = v - u;
            sort_iter(q);
            c.out->push_back(std::move(q));
            for (int64_t i = v; i <= i_last && c.ok; ++i) fixed_at(i);
            return;
        }
    }
    if (i_last - i_first + 1 > kMaxPieces) {
        c.ok = false;
        return;
    }
    for (int64_t i = i_first; i <= i_last && c.ok; ++i) fixed_at(i);
}

}  // namespace

// The same piece with one dst axis of extent E reversed: position x becomes
// E - 1 - x.  Every loop on the axis runs backwards (i -> n - 1 - i), which
// moves the origin to the far end and negates the source stride.
static Piece flip_piece(const Piece &p, int axis, int64_t E) {
    Piece q = p;
    int64_t span = 0;
    for (IterDim &d : q.it) {
        if (d.dim != axis) continue;
        span += (d.extent - 1) * d.mult;
        q.sbase += (d.extent - 1) * d.sstride;
        d.sstride = -d.sstride;
    }
    q.lo[axis] = E - 1 - p.lo[axis] - span;
    return q;
}

extern "C" amap_status amap_slice(const amap_t *m, int axis, int64_t begin, int64_t end, int64_t step,
                                  amap_t **out) {
    GUARD_BEGIN
    if (!m || !out) return AMAP_E_INVALID;
    int rank = (int)m->shape.size();
    if (axis < 0 || axis >= rank) return AMAP_E_INVALID;
    const int64_t E = m->shape[axis];
    int64_t count;
    if (step >= 1) {
        if (begin < 0 || begin >= end || end > E) return AMAP_E_SHAPE;
        count = (end - begin + step - 1) / step;
    } else if (step <= -1) {
        if (end < -1 || end >= begin || begin > E - 1) return AMAP_E_SHAPE;
        count = (begin - end + (-step) - 1) / (-step);
    } else {
        return AMAP_E_SHAPE;
    }
    amap *r = clone_header(m);
    if (!r) return AMAP_E_NOMEM;
    std::unique_ptr<amap> hold(r);
    r->shape = m->shape;
    r->shape[axis] = count;
    auto n = unary_node(PNode::SLICE, m, r->shape);
    n->axis = axis;
    n->begin = begin;
    n->step = step;
    r->prog = n;
    r->strided = m->strided;
    if (m->strided) {
        // a negative step is the positive step on the reversed axis:
        // in[begin + i step] = flipped[(E - 1 - begin) + i |step|]
        SliceCtx c{axis, begin, end, step, &r->pieces};
        if (step < 0) c = SliceCtx{axis, E - 1 - begin, E - 1 - end, -step, &r->pieces};
        for (const Piece &p : m->pieces) slice_piece(c, step < 0 ? flip_piece(p, axis, E) : p);
        if (!c.ok) {
            r->strided = false;
            r->pieces.clear();
        }
    }
    finish(*r);
    *out = hold.release();
    return AMAP_OK;
    GUARD_END
}

// ---------------------------------------------------------------- repeat, tile

extern "C" amap_status amap_repeat(const amap_t *m, int axis, int64_t count, amap_t **out) {
    GUARD_BEGIN
    if (!m || !out) return AMAP_E_INVALID;
    int rank = (int)m->shape.size();
    if (axis < 0 || axis >= rank) return AMAP_E_INVALID;
    if (count < 1) return AMAP_E_SHAPE;
    amap *r = clone_header(m);
    if (!r) return AMAP_E_NOMEM;
    std::unique_ptr<amap> hold(r);
    r->shape = m->shape;
    r->shape[axis] *= count;
    auto n = unary_node(PNode::REPEAT, m, r->shape);
    n->axis = axis;
    n->count = count;
    r->prog = n;
    r->strided = m->strided;
    if (count > 1 && volume_of(m->shape) > 0) r->injective = false;
    if (m->strided) {
        // new index = old index * count + j: every loop on the axis steps count
        // times as far in dst, and a new innermost loop j re-reads the element
        for (const Piece &p : m->pieces) {
            Piece q = p;
            q.lo[axis] *= count;
            for (IterDim &d : q.it)
                if (d.dim == axis) d.mult *= count;
            if (count > 1) q.it.push_back({count, axis, 1, 0});
            sort_iter(q);
            r->pieces.push_back(std::move(q));
        }
    }
    finish(*r);
    *out = hold.release();
    return AMAP_OK;
    GUARD_END
}

extern "C" amap_status amap_tile(const amap_t *m, int axis, int64_t count, amap_t **out) {
    GUARD_BEGIN
    if (!m || !out) return AMAP_E_INVALID;
    int rank = (int)m->shape.size();
    if (axis < 0 || axis >= rank) return AMAP_E_INVALID;
    if (count < 1) return AMAP_E_SHAPE;
    const int64_t E = m->shape[axis];
    amap *r = clone_header(m);
    if (!r) return AMAP_E_NOMEM;
    std::unique_ptr<amap> hold(r);
    r->shape = m->shape;
    r->shape[axis] *= count;
    auto n = unary_node(PNode::TILE, m, r->shape);
    n->axis = axis;
    n->count = E;
    n->step = count;
    r->prog = n;
    r->strided = m->strided;
    if (count > 1 && volume_of(m->shape) > 0) r->injective = false;
    if (m->strided) {
        for (const Piece &p : m->pieces) {
            int64_t span = 0;
            for (const IterDim &d : p.it)
                if (d.dim == axis) span += (d.extent - 1) * d.mult;
            if (count == 1) {
                r->pieces.push_back(p);
            } else if (p.lo[axis] == 0 && span == E - 1) {
                // the piece covers the whole axis: one more (outermost) loop over the copies
                Piece q = p;
                q.it.push_back({count, axis, E, 0});
                sort_iter(q);
                r->pieces.push_back(std::move(q));
            } else {
                for (int64_t k = 0; k < count; ++k) {
                    Piece q = p;
                    q.lo[axis] += k * E;
                    r->pieces.push_back(std::move(q));
                }
            }
            if ((int64_t)r->pieces.size() > kMaxPieces) break;
        }
        if ((int64_t)r->pieces.size() > kMaxPieces) {
            r->strided = false;
            r->pieces.clear();
        }
    }
    finish(*r);
    *out = hold.release();
    return AMAP_OK;
    GUARD_END
}

// ---------------------------------------------------------------- pad

extern "C" amap_status amap_pad(const amap_t *m, const int64_t *lo, const int64_t *hi, uint32_t fill_bits,
                                amap_t **out) {
    GUARD_BEGIN
    if (!m || !lo || !hi || !out) return AMAP_E_INVALID;
    int rank = (int)m->shape.size();
    for (int k = 0; k < rank; ++k)
        if (lo[k] < 0 || hi[k] < 0) return AMAP_E_SHAPE;
    amap *r = clone_header(m);
    if (!r) return AMAP_E_NOMEM;
    std::unique_ptr<amap> hold(r);
    r->shape.resize(rank);
    for (int k = 0; k < rank; ++k) r->shape[k] = lo[k] + m->shape[k] + hi[k];
    if (m->elem == 2) fill_bits &= 0xFFFFu;
    auto n = unary_node(PNode::PAD, m, r->shape);
    n->lo.assign(lo, lo + rank);
    n->fill = fill_bits;
    r->prog = n;
    r->strided = m->strided;
    if (m->strided) {
        for (const Piece &p : m->pieces) {
            Piece q = p;
            for (int k = 0; k < rank; ++k) q.lo[k] += lo[k];
            r->pieces.push_back(std::move(q));
        }
        // complement of the inner box, as at most 2*rank boxes: for dim d, the
        // slabs below / above the inner range, with dims before d restricted
        // to the inner range and dims after d unrestricted.
        if (volume_of(r->shape) > 0) {
            for (int d = 0; d < rank; ++d) {
                for (int side = 0; side < 2; ++side) {
                    int64_t a = side == 0 ? 0 : lo[d] + m->shape[d];
                    int64_t b = side == 0 ? lo[d] : r->shape[d];
                    if (a >= b) continue;
                    Piece f;
                    f.fill = true;
                    f.fill_bits = fill_bits;
                    bool empty = false;
                    for (int k = 0; k < rank; ++k) {
                        int64_t s, e;
                        if (k < d) {
                            s = lo[k];
                            e = lo[k] + m->shape[k];
                        } else if (k == d) {
                            s = a;
                            e = b;
                        } else {
                            s = 0;
                            e = r->shape[k];
                        }
                        if (e <= s) empty = true;
                        f.lo[k] = s;
                        if (e - s > 1) f.it.push_back({e - s, k, 1, 0});
                    }
                    if (!empty) r->pieces.push_back(std::move(f));
                }
            }
        }
        if ((int64_t)r->pieces.size() > kMaxPieces) {
            r->strided = false;
            r->pieces.clear();
        }
    }
    finish(*r);
    *out = hold.release();
    return AMAP_OK;
    GUARD_END
}

// ---------------------------------------------------------------- concat

extern "C" amap_status amap_concat(const amap_t *const *ms, int n, int axis, amap_t **out) {
    GUARD_BEGIN
    if (!ms || n < 1 || !out) return AMAP_E_INVALID;
    for (int i = 0; i < n; ++i)
        if (!ms[i]) return AMAP_E_INVALID;
    int rank = (int)ms[0]->shape.size();
    if (axis < 0 || axis >= rank) return AMAP_E_INVALID;
    amap *r = new amap();
    std::unique_ptr<amap> hold(r);
    r->elem = ms[0]->elem;
    r->shape = ms[0]->shape;
    r->shape[axis] = 0;
    auto node = std::make_shared<PNode>();
    node->kind = PNode::CONCAT;
    node->axis = axis;
    r->strided = true;
    for (int i = 0; i < n; ++i) {
        const amap *m = ms[i];
        if ((int)m->shape.size() != rank || m->elem != r->elem) return AMAP_E_INVALID;
        for (int k = 0; k < rank; ++k)
            if (k != axis && m->shape[k] != r->shape[k]) return AMAP_E_SHAPE;
        // merge source tables
        if (m->src_shapes.size() > r->src_shapes.size()) r->src_shapes.resize(m->src_shapes.size());
        for (size_t s = 0; s < m->src_shapes.size(); ++s) {
            if (m->src_shapes[s].empty()) continue;
            if (r->src_shapes[s].empty())
                r->src_shapes[s] = m->src_shapes[s];
            else if (r->src_shapes[s] != m->src_shapes[s])
                return AMAP_E_SHAPE;  // same id, different tensors
            else
                r->injective = false;  // two inputs read the same source
        }
        r->strided = r->strided && m->strided;
        r->injective = r->injective && m->injective;
        if (r->strided) {
            for (const Piece &p : m->pieces) {
                Piece q = p;
                q.lo[axis] += r->shape[axis];
                r->pieces.push_back(std::move(q));
            }
        }
        node->kids.push_back(m->prog);
        r->shape[axis] += m->shape[axis];
    }
    node->shape = r->shape;
    r->prog = node;
    if (!r->strided || (int64_t)r->pieces.size() > kMaxPieces) {
        r->strided = false;
        r->pieces.clear();
    }
    finish(*r);
    *out = hold.release();
    return AMAP_OK;
    GUARD_END
}

// ---------------------------------------------------------------- reshape

namespace {

struct LinDim {
    int64_t extent, ds, ss;
};

// Loops (sorted by ds descending) that continue one another on both sides become one loop:
// a tensor that is contiguous where it is read can then be re-split along any new shape.
void merge_contiguous(std::vector<LinDim> &dims) {
    for (size_t i = 0; i + 1 < dims.size();) {
        const LinDim &a = dims[i], &b = dims[i + 1];
        if (a.ds == b.ds * b.extent && a.ss == b.ss * b.extent) {
            dims[i] = {a.extent * b.extent, b.ds, b.ss};
            dims.erase(dims.begin() + i + 1);
        } else {
            ++i;
        }
    }
}

struct Redigit {
    std::vector<int64_t> shape, R;  // new shape and its row-major strides
    std::vector<int> cand;          // new dims with extent > 1, outermost first
    const Piece *proto;             // fill / src come from here
    std::vector<Piece> *out;
    bool ok = true;

    // Express the set { L0 + sum_j i_j * ds_j } (dims sorted by ds descending,
    // each ds larger than the span of the dims after it) in the digits of the
    // new shape, splitting into several pieces where a loop would carry from
    // one new dimension into the next.
    void rec(int64_t L0, int64_t sbase, std::vector<LinDim> dims) {
        if (!ok) return;
        if ((int64_t)out->size() > kMaxPieces) {
            ok = false;
            return;
        }
        dims.erase(std::remove_if(dims.begin(), dims.end(), [](const LinDim &d) { return d.extent == 1; }),
                   dims.end());
        const int nd = (int)dims.size();
        std::vector<int> where(nd);
        std::vector<int64_t> mult(nd);
        for (int j = 0; j < nd; ++j) {
            int d = -1;
            for (int c : cand)
                if (R[c] <= dims[j].ds) {
                    d = c;
                    break;
                }
            if (d < 0 || dims[j].ds % R[d] != 0) {
                // this loop's step is not a whole number of steps of any new
                // dimension: no box form, one piece per iteration
                if (dims[j].extent > kMaxPieces) {
                    ok = false;
                    return;
                }
                LinDim dj = dims[j];
                std::vector<LinDim> rest = dims;
                rest.erase(rest.begin() + j);
                for (int64_t i = 0; i < dj.extent && ok; ++i) rec(L0 + i * dj.ds, sbase + i * dj.ss, rest);
                return;
            }
            where[j] = d;
            mult[j] = dims[j].ds / R[d];
        }
        const int rank = (int)shape.size();
        int64_t lo[kMaxRank];
        for (int d = 0; d < rank; ++d) lo[d] = shape[d] > 0 ? (L0 / R[d]) % shape[d] : 0;
        for (int ci = (int)cand.size() - 1; ci >= 0; --ci) {
            const int d = cand[ci];
            const int64_t E = shape[d];
            int64_t acc = lo[d];
            // innermost loop of this dim first
            for (int j = nd - 1; j >= 0; --j) {
                if (where[j] != d) continue;
                const int64_t m = mult[j], n = dims[j].extent;
                if (acc + (n - 1) * m < E) {
                    acc += (n - 1) * m;
                    continue;
                }
                // loop j carries out of dimension d.  If it steps through whole multiples of the
                // dimension (everything inside it stays below one step, the dimension is a whole
                // number of steps, the loop a whole number of dimensions) it is two loops: one
                // inside d and one that counts d's wrap-arounds, i.e. runs in an outer dimension.
                if (acc < m && E % m == 0 && n % (E / m) == 0) {
                    const int64_t q = E / m;
                    std::vector<LinDim> two(dims.begin(), dims.begin() + j);
                    two.push_back({n / q, dims[j].ds * q, dims[j].ss * q});
                    two.push_back({q, dims[j].ds, dims[j].ss});
                    two.insert(two.end(), dims.begin() + j + 1, dims.end());
                    rec(L0, sbase, two);
                    return;
                }
                // otherwise cut its range into blocks
                split(L0, sbase, dims, j, lo[d], acc - lo[d], m, E);
                return;
            }
        }
        Piece p;
        p.fill = proto->fill;
        p.fill_bits = proto->fill_bits;
        p.src = proto->src;
        p.sbase = sbase;
        for (int d = 0; d < rank; ++d) p.lo[d] = lo[d];
        for (int j = 0; j < nd; ++j) p.it.push_back({dims[j].extent, where[j], mult[j], dims[j].ss});
        sort_iter(p);
        out->push_back(std::move(p));
    }

    // Loop j (step m in new dim d of extent E, starting digit lo, loops inside
    // it in the same dim spanning s_in < m) leaves [0, E): cut i into runs that
    // stay inside one block of E.
    void split(int64_t L0, int64_t sbase, const std::vector<LinDim> &dims, int j, int64_t lo, int64_t s_in,
               int64_t m, int64_t E) {
        const LinDim dj = dims[j];
        auto with_j = [&](int64_t i_a, std::vector<LinDim> repl) {
            std::vector<LinDim> nd(dims.begin(), dims.begin() + j);
            nd.insert(nd.end(), repl.begin(), repl.end());
            nd.insert(nd.end(), dims.begin() + j + 1, dims.end());
            rec(L0 + i_a * dj.ds, sbase + i_a * dj.ss, nd);
        };
        // run [i_a, i_a + len): all inside one block; its clean prefix keeps
        // loop j, the rest (inner loops would carry) fixes i one at a time
        auto run = [&](int64_t i_a, int64_t len) {
            if (len <= 0) return;
            int64_t pos = (lo + i_a * m) % E;
            // clean: pos + k*m + s_in < E
            int64_t clean = (E - 1 - s_in - pos) >= 0 ? std::min(len, (E - 1 - s_in - pos) / m + 1) : 0;
            if (clean > 0) with_j(i_a, {{clean, dj.ds, dj.ss}});
            for (int64_t i = i_a + clean; i < i_a + len && ok; ++i) with_j(i, {});
        };
        const int64_t n = dj.extent;
        // iterations before the first carry; none are set apart when the
        // first block is already a full one of the uniform pattern below
        const bool aligned = E % m == 0 && lo < m;
        const int64_t head = aligned ? 0 : std::min(n, cdiv(E - lo, m));
        run(0, head);
        int64_t i = head;
        if (E % m == 0) {
            const int64_t q = E / m;
            const int64_t full = (n - i) / q;
            if (full > 0) {
                // every full block starts at the same digit r0 < m
                const int64_t r0 = (lo + i * m) % E;
                int64_t clean = (E - 1 - s_in - r0) >= 0 ? std::min(q, (E - 1 - s_in - r0) / m + 1) : 0;
                if (clean > 0) with_j(i, {{full, dj.ds * q, dj.ss * q}, {clean, dj.ds, dj.ss}});
                for (int64_t t = clean; t < q && ok; ++t) with_j(i + t, {{full, dj.ds * q, dj.ss * q}});
                i += full * q;
            }
            run(i, n - i);
        } else {
            while (i < n && ok) {
                int64_t pos = (lo + i * m) % E;
                int64_t len = std::min(n - i, cdiv(E - pos, m));
                run(i, len);
                i += len;
                if ((int64_t)out->size() > kMaxPieces) ok = false;
            }
        }
    }
};

// sorted by ds descending and each ds exceeds the span of the loops after it
bool nested(const std::vector<LinDim> &dims) {
    int64_t span = 0;
    for (int j = (int)dims.size() - 1; j >= 0; --j) {
        if (dims[j].ds <= span && dims[j].extent > 1) return false;
        span += (dims[j].extent - 1) * dims[j].ds;
    }
    return true;
}

}  // namespace

extern "C" amap_status amap_reshape(const amap_t *m, int rank, const int64_t *shape, amap_t **out) {
    GUARD_BEGIN
    if (!m || !out || !valid_shape(rank, shape)) return AMAP_E_INVALID;
    std::vector<int64_t> ns(shape, shape + rank);
    if (volume_of(ns) != volume_of(m->shape)) return AMAP_E_SHAPE;
    amap *r = clone_header(m);
    if (!r) return AMAP_E_NOMEM;
    std::unique_ptr<amap> hold(r);
    r->shape = ns;
    r->prog = unary_node(PNode::RESHAPE, m, ns);
    r->strided = m->strided;
    if (m->strided && !m->pieces.empty()) {
        auto Rold = row_major_strides(m->shape);
        Redigit rd;
        rd.shape = ns;
        rd.R = row_major_strides(ns);
        for (int d = 0; d < rank; ++d)
            if (ns[d] > 1) rd.cand.push_back(d);
        rd.out = &r->pieces;
        for (const Piece &p : m->pieces) {
            int64_t L0 = 0;
            for (size_t d = 0; d < m->shape.size(); ++d) L0 += p.lo[d] * Rold[d];
            std::vector<LinDim> dims;
            for (const IterDim &it : p.it) dims.push_back({it.extent, it.mult * Rold[it.dim], it.sstride});
            std::stable_sort(dims.begin(), dims.end(), [](const LinDim &a, const LinDim &b) { return a.ds > b.ds; });
            if (!nested(dims)) {
                rd.ok = false;
                break;
            }
            merge_contiguous(dims);
            rd.proto = &p;
            rd.rec(L0, p.sbase, dims);
            if (!rd.ok) break;
        }
        if (!rd.ok) {
            r->strided = false;
            r->pieces.clear();
        }
    }
    finish(*r);
    *out = hold.release();
    return AMAP_OK;
    GUARD_END
}

// ---------------------------------------------------------------- inverse

extern "C" amap_status amap_inverse(const amap_t *m, amap_t **out) {
    GUARD_BEGIN
    if (!m || !out) return AMAP_E_INVALID;
    // Only a single affine piece that is a bijection between dst and the whole
    // of one source can be reversed here (Section 2.1 reverses affine store
    // maps); anything else is refused.
    if (!m->strided || m->pieces.size() != 1 || m->pieces[0].fill) return AMAP_E_UNSUPPORTED;
    const Piece &p = m->pieces[0];
    const std::vector<int64_t> &sshape = m->src_shapes[p.src];
    if (p.volume() != volume_of(m->shape) || p.volume() != volume_of(sshape)) return AMAP_E_UNSUPPORTED;
    auto Rd = row_major_strides(m->shape);
    int64_t dbase = 0;
    for (size_t d = 0; d < m->shape.size(); ++d) dbase += p.lo[d] * Rd[d];
    // the loops with the roles of the two sides exchanged
    std::vector<LinDim> dims;
    int64_t sbase = p.sbase;
    for (const IterDim &it : p.it) {
        if (it.sstride == 0) return AMAP_E_UNSUPPORTED;  // an element read more than once
        if (it.sstride > 0) {
            dims.push_back({it.extent, it.sstride, it.mult * Rd[it.dim]});
        } else {
            // a loop that walks the source backwards: run it the other way round
            sbase += (it.extent - 1) * it.sstride;
            dbase += (it.extent - 1) * it.mult * Rd[it.dim];
            dims.push_back({it.extent, -it.sstride, -it.mult * Rd[it.dim]});
        }
    }
    std::stable_sort(dims.begin(), dims.end(), [](const LinDim &a, const LinDim &b) { return a.ds > b.ds; });
    if (!nested(dims)) return AMAP_E_UNSUPPORTED;  // not injective on the source side
    amap *r = new amap();
    std::unique_ptr<amap> hold(r);
    r->elem = m->elem;
    r->shape = sshape;
    r->src_shapes.resize(1);
    r->src_shapes[0] = m->shape;
    Piece proto;
    proto.src = 0;
    Redigit rd;
    rd.shape = sshape;
    rd.R = row_major_strides(sshape);
    for (int d = 0; d < (int)sshape.size(); ++d)
        if (sshape[d] > 1) rd.cand.push_back(d);
    rd.out = &r->pieces;
    rd.proto = &proto;
    rd.rec(sbase, dbase, dims);
    if (!rd.ok) return AMAP_E_UNSUPPORTED;
    r->strided = true;
    // program: source(dst shape) -> reshape to the loop extents in dst order ->
    // transpose into source order -> reshape to the source shape
    {
        std::vector<LinDim> by_dst;  // {extent, old dst stride, old src stride}
        for (const IterDim &it : p.it) by_dst.push_back({it.extent, it.mult * Rd[it.dim], it.sstride});
        std::stable_sort(by_dst.begin(), by_dst.end(), [](const LinDim &a, const LinDim &b) { return a.ds > b.ds; });
        if ((int)by_dst.size() > kMaxRank) return AMAP_E_UNSUPPORTED;
        if (by_dst.empty()) by_dst.push_back({1, 1, 1});
        int n = (int)by_dst.size();
        std::vector<int> order(n);
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(),
                         [&](int a, int b) { return std::llabs(by_dst[a].ss) > std::llabs(by_dst[b].ss); });
        auto s0 = std::make_shared<PNode>();
        s0->kind = PNode::SOURCE;
        s0->shape = m->shape;
        s0->src_id = 0;
        auto r1 = std::make_shared<PNode>();
        r1->kind = PNode::RESHAPE;
        for (auto &d : by_dst) r1->shape.push_back(d.extent);
        r1->kids.push_back(s0);
        // loops that walk the source backwards: reverse that axis
        std::shared_ptr<PNode> below = r1;
        for (int k = 0; k < n; ++k) {
            if (by_dst[k].ss >= 0) continue;
            auto f = std::make_shared<PNode>();
            f->kind = PNode::SLICE;
            f->shape = r1->shape;
            f->axis = k;
            f->begin = by_dst[k].extent - 1;
            f->step = -1;
            f->kids.push_back(below);
            below = f;
        }
        auto t = std::make_shared<PNode>();
        t->kind = PNode::TRANSPOSE;
        t->perm = order;
        for (int k = 0; k < n; ++k) t->shape.push_back(by_dst[order[k]].extent);
        t->kids.push_back(below);
        auto r2 = std::make_shared<PNode>();
        r2->kind = PNode::RESHAPE;
        r2->shape = sshape;
        r2->kids.push_back(t);
        r->prog = r2;
    }
    finish(*r);
    *out = hold.release();
    return AMAP_OK;
    GUARD_END
}

// ---------------------------------------------------------------- compose

extern "C" amap_status amap_compose(const amap_src_desc *srcs, int n_src, const amap_op *ops, int n_ops,
                                    amap_t **out) {
    GUARD_BEGIN
    if (!srcs || n_src < 1 || n_ops < 0 || (n_ops > 0 && !ops) || !out) return AMAP_E_INVALID;
    std::vector<amap *> cur;
    auto cleanup = [&]() {
        for (amap *p : cur) delete p;
        cur.clear();
    };
    for (int i = 0; i < n_src; ++i) {
        amap *s = nullptr;
        amap_status st = amap_source(i, srcs[i].rank, srcs[i].shape, srcs[i].es, &s);
        if (st != AMAP_OK) {
            cleanup();
            return st;
        }
        cur.push_back(s);
    }
    for (int k = 0; k < n_ops; ++k) {
        const amap_op &op = ops[k];
        amap *next = nullptr;
        amap_status st = AMAP_E_INVALID;
        if (op.kind == AMAP_CONCAT) {
            if (k == 0) st = amap_concat(cur.data(), (int)cur.size(), op.axis, &next);
        } else if (cur.size() == 1) {
            const amap *m = cur[0];
            int rank = (int)m->shape.size();
            switch (op.kind) {
            case AMAP_TRANSPOSE: {
                if (!op.a || op.n != rank) break;
                int32_t perm[kMaxRank];
                for (int t = 0; t < rank; ++t) perm[t] = (int32_t)op.a[t];
                st = amap_transpose(m, perm, &next);
                break;
            }
            case AMAP_RESHAPE:
                st = amap_reshape(m, op.n, op.a, &next);
                break;
            case AMAP_SLICE:
                if (!op.a) break;
                st = amap_slice(m, op.axis, op.a[0], op.a[1], op.a[2], &next);
                break;
            case AMAP_PAD:
                if (op.n != rank) break;
                st = amap_pad(m, op.a, op.b, op.fill_bits, &next);
                break;
            case AMAP_REPEAT:
                if (!op.a) break;
                st = amap_repeat(m, op.axis, op.a[0], &next);
                break;
            case AMAP_TILE:
                if (!op.a) break;
                st = amap_tile(m, op.axis, op.a[0], &next);
                break;
            default:
                break;
            }
        }
        if (st != AMAP_OK) {
            cleanup();
            return st;
        }
        cleanup();
        cur.push_back(next);
    }
    if (cur.size() != 1) {
        cleanup();
        return AMAP_E_INVALID;
    }
    *out = cur[0];
    return AMAP_OK;
    GUARD_END
}

extern "C" void amap_free(amap_t *m) { delete m; }

extern "C" const char *amap_status_str(amap_status s) {
    switch (s) {
    case AMAP_OK: return "ok";
    case AMAP_E_INVALID: return "invalid argument";
    case AMAP_E_SHAPE: return "shape mismatch or index out of range";
    case AMAP_E_UNSUPPORTED: return "unsupported map";
    case AMAP_E_NOMEM: return "out of host memory";
    case AMAP_E_ALIAS: return "dst overlaps a source";
    case AMAP_E_HIP: return "HIP runtime error";
    }
    return "unknown status";
}
