// Data-movement elimination over an operator graph (paper Section 2.1).
//
// The paper walks a program of loop nests, finds load/store pairs whose load
// feeds the store directly, and rewrites every load of the stored tensor t_s
// into a load of the original tensor t_l through g' = f_l o f_s' o f_l'
// (eq. 3, eq. 4), until no pair is left.  Here the program is a graph whose
// layout operators are exactly such pairs.  Every load is kept as a composed
// map over tensor ids; one rewrite step replaces, in one load, the tensor t_s
// by the map that defines it.  The composition itself is done by re-applying
// the load's operator program on top of the defining map, i.e. by the same
// builders that normalise a single chain.
#include <algorithm>
#include <functional>
#include <memory>
#include <new>
#include <vector>

#include "amap_map.hpp"

using namespace amap_detail;

namespace {

struct GTensor {
    enum Kind { INPUT, COMPUTE, LAYOUT } kind = INPUT;
    std::vector<int64_t> shape;
    int elem = 2;
    std::unique_ptr<amap> def;  // LAYOUT: the operator as a map over its input tensors (source id = tensor id)
    std::vector<int> inputs;    // COMPUTE: tensors read, by slot
    int pairs = 0;              // LAYOUT: load/store pairs of the operator
    bool output = false;
};

struct GLoad {
    int consumer, slot;
    std::unique_ptr<amap> map;  // over tensor ids
};

using Leaf = std::function<amap_status(int id, const std::vector<int64_t> &shape, int elem, amap **out)>;

// Re-apply an operator program with its SOURCE leaves replaced by leaf(id).
amap_status replay(const PNode *n, int elem, const Leaf &leaf, amap **out) {
    if (n->kind == PNode::SOURCE) return leaf(n->src_id, n->shape, elem, out);
    std::vector<amap *> kids;
    auto drop = [&]() {
        for (amap *k : kids) delete k;
    };
    for (const auto &c : n->kids) {
        amap *k = nullptr;
        amap_status st = replay(c.get(), elem, leaf, &k);
        if (st != AMAP_OK) {
            drop();
            return st;
        }
        kids.push_back(k);
    }
    amap_status st = AMAP_E_INVALID;
    const int rank = (int)n->shape.size();
    switch (n->kind) {
    case PNode::TRANSPOSE: {
        int32_t perm[kMaxRank];
        for (int k = 0; k < rank; ++k) perm[k] = n->perm[k];
        st = amap_transpose(kids[0], perm, out);
        break;
    }
    case PNode::RESHAPE:
        st = amap_reshape(kids[0], rank, n->shape.data(), out);
        break;
    case PNode::SLICE: {
        // the node keeps begin and step; any end that yields the node's extent will do
        const int64_t cnt = n->shape[n->axis];
        const int64_t end = n->begin + (cnt - 1) * n->step + (n->step > 0 ? 1 : -1);
        st = amap_slice(kids[0], n->axis, n->begin, end, n->step, out);
        break;
    }
    case PNode::PAD: {
        int64_t hi[kMaxRank];
        for (int k = 0; k < rank; ++k) hi[k] = n->shape[k] - n->lo[k] - kids[0]->shape[k];
        st = amap_pad(kids[0], n->lo.data(), hi, n->fill, out);
        break;
    }
    case PNode::CONCAT:
        st = amap_concat(kids.data(), (int)kids.size(), n->axis, out);
        break;
    case PNode::REPEAT:
        st = amap_repeat(kids[0], n->axis, n->count, out);
        break;
    case PNode::TILE:
        st = amap_tile(kids[0], n->axis, n->step, out);
        break;
    case PNode::SOURCE:
        break;
    }
    drop();
    return st;
}

std::vector<int> sources_of(const amap &m) {
    std::vector<int> ids;
    for (size_t i = 0; i < m.src_shapes.size(); ++i)
        if (!m.src_shapes[i].empty()) ids.push_back((int)i);
    return ids;
}

// bytes read + written when the map is executed on its own
int64_t moved_bytes(const amap &m) {
    amap_info info;
    if (amap_describe(&m, &info) != AMAP_OK) return 0;
    return info.min_read_bytes + info.write_bytes;
}

// the identity of exactly one whole tensor, element for element in memory order (its shape may
// differ: a reshape of a whole tensor is a view): executing it would be a plain copy
bool is_identity(const amap &m, const std::vector<int64_t> &src_shape) {
    if (!m.strided || m.kpieces.size() != 1 || m.kpieces[0].fill || volume_of(m.shape) != volume_of(src_shape)) return false;
    const KPiece &k = m.kpieces[0];
    if (k.dbase != 0 || k.sbase != 0) return false;
    if (volume_of(m.shape) <= 1) return true;
    return k.dims.size() == 1 && k.dims[0].ds == 1 && k.dims[0].ss == 1 && k.dims[0].extent == volume_of(m.shape);
}

}  // namespace

struct amap_graph {
    std::vector<GTensor> t;
    std::vector<GLoad> loads;
    bool done = false;
};

#define GUARD_BEGIN try {
#define GUARD_END                     \
    }                                 \
    catch (const std::bad_alloc &) {  \
        return AMAP_E_NOMEM;          \
    }                                 \
    catch (...) {                     \
        return AMAP_E_INVALID;        \
    }

extern "C" amap_status amap_graph_create(amap_graph_t **out) {
    GUARD_BEGIN
    if (!out) return AMAP_E_INVALID;
    *out = new amap_graph();
    return AMAP_OK;
    GUARD_END
}

extern "C" void amap_graph_free(amap_graph_t *g) { delete g; }

static bool valid_tensor(const amap_graph *g, int id) { return id >= 0 && id < (int)g->t.size(); }

extern "C" amap_status amap_graph_input(amap_graph_t *g, int rank, const int64_t *shape, amap_elem es, int *tensor) {
    GUARD_BEGIN
    if (!g || !tensor || g->done) return AMAP_E_INVALID;
    if (g->t.size() >= 4096) return AMAP_E_UNSUPPORTED;
    amap *probe = nullptr;  // validates rank / shape / element size
    amap_status st = amap_source((int)g->t.size(), rank, shape, es, &probe);
    if (st != AMAP_OK) return st;
    delete probe;
    GTensor x;
    x.kind = GTensor::INPUT;
    x.shape.assign(shape, shape + rank);
    x.elem = (int)es;
    g->t.push_back(std::move(x));
    *tensor = (int)g->t.size() - 1;
    return AMAP_OK;
    GUARD_END
}

extern "C" amap_status amap_graph_op(amap_graph_t *g, const amap_op *op, const int *inputs, int n_inputs, int *tensor) {
    GUARD_BEGIN
    if (!g || !op || !inputs || n_inputs < 1 || !tensor || g->done) return AMAP_E_INVALID;
    if (g->t.size() >= 4096) return AMAP_E_UNSUPPORTED;
    if (op->kind != AMAP_CONCAT && n_inputs != 1) return AMAP_E_INVALID;
    std::vector<amap *> ins;
    auto drop = [&]() {
        for (amap *k : ins) delete k;
    };
    for (int i = 0; i < n_inputs; ++i) {
        if (!valid_tensor(g, inputs[i])) {
            drop();
            return AMAP_E_INVALID;
        }
        const GTensor &x = g->t[inputs[i]];
        amap *s = nullptr;
        amap_status st = amap_source(inputs[i], (int)x.shape.size(), x.shape.data(), (amap_elem)x.elem, &s);
        if (st != AMAP_OK) {
            drop();
            return st;
        }
        ins.push_back(s);
    }
    amap *def = nullptr;
    amap_status st = AMAP_E_INVALID;
    const int rank = (int)ins[0]->shape.size();
    switch (op->kind) {
    case AMAP_CONCAT:
        st = amap_concat(ins.data(), n_inputs, op->axis, &def);
        break;
    case AMAP_TRANSPOSE: {
        if (!op->a || op->n != rank) break;
        int32_t perm[kMaxRank];
        for (int k = 0; k < rank; ++k) perm[k] = (int32_t)op->a[k];
        st = amap_transpose(ins[0], perm, &def);
        break;
    }
    case AMAP_RESHAPE:
        st = amap_reshape(ins[0], op->n, op->a, &def);
        break;
    case AMAP_SLICE:
        if (op->a) st = amap_slice(ins[0], op->axis, op->a[0], op->a[1], op->a[2], &def);
        break;
    case AMAP_PAD:
        if (op->n == rank) st = amap_pad(ins[0], op->a, op->b, op->fill_bits, &def);
        break;
    case AMAP_REPEAT:
        if (op->a) st = amap_repeat(ins[0], op->axis, op->a[0], &def);
        break;
    case AMAP_TILE:
        if (op->a) st = amap_tile(ins[0], op->axis, op->a[0], &def);
        break;
    }
    drop();
    if (st != AMAP_OK) return st;
    GTensor x;
    x.kind = GTensor::LAYOUT;
    x.shape = def->shape;
    x.elem = def->elem;
    x.def.reset(def);
    x.pairs = n_inputs;
    g->t.push_back(std::move(x));
    *tensor = (int)g->t.size() - 1;
    return AMAP_OK;
    GUARD_END
}

extern "C" amap_status amap_graph_map(amap_graph_t *g, const amap_t *m, const int *inputs, int n_inputs, int *tensor) {
    GUARD_BEGIN
    if (!g || !m || !m->prog || !inputs || n_inputs < 1 || !tensor || g->done) return AMAP_E_INVALID;
    if (g->t.size() >= 4096) return AMAP_E_UNSUPPORTED;
    for (int i = 0; i < n_inputs; ++i)
        if (!valid_tensor(g, inputs[i])) return AMAP_E_INVALID;
    // the operator's own program, re-applied on top of the graph tensors it reads
    int used = 0;
    const Leaf leaf = [&](int id, const std::vector<int64_t> &shape, int elem, amap **out) -> amap_status {
        if (id < 0 || id >= n_inputs) return AMAP_E_INVALID;
        const GTensor &x = g->t[inputs[id]];
        if (x.shape != shape || x.elem != elem) return AMAP_E_SHAPE;
        ++used;
        return amap_source(inputs[id], (int)shape.size(), shape.data(), (amap_elem)elem, out);
    };
    amap *def = nullptr;
    amap_status st = replay(m->prog.get(), m->elem, leaf, &def);
    if (st != AMAP_OK) return st;
    GTensor x;
    x.kind = GTensor::LAYOUT;
    x.shape = def->shape;
    x.elem = def->elem;
    x.pairs = std::max<int>(1, (int)sources_of(*def).size());
    x.def.reset(def);
    g->t.push_back(std::move(x));
    *tensor = (int)g->t.size() - 1;
    return AMAP_OK;
    GUARD_END
}

extern "C" amap_status amap_graph_store(amap_graph_t *g, const amap_t *store_map, int input, int *tensor) {
    GUARD_BEGIN
    if (!g || !store_map || !tensor || g->done || !valid_tensor(g, input)) return AMAP_E_INVALID;
    if (store_map->shape != g->t[input].shape || store_map->elem != g->t[input].elem) return AMAP_E_SHAPE;
    // t_s[f_s(i)] = t_l[i]: reverse the store map (Section 2.1) and the operator is a load like the others
    amap *rev = nullptr;
    amap_status st = amap_inverse(store_map, &rev);
    if (st != AMAP_OK) return st;
    std::unique_ptr<amap> hold(rev);
    return amap_graph_map(g, rev, &input, 1, tensor);
    GUARD_END
}

extern "C" amap_status amap_graph_compute(amap_graph_t *g, const int *inputs, int n_inputs, int rank,
                                          const int64_t *shape, amap_elem es, int *tensor) {
    GUARD_BEGIN
    if (!g || n_inputs < 0 || (n_inputs > 0 && !inputs) || !tensor || g->done) return AMAP_E_INVALID;
    for (int i = 0; i < n_inputs; ++i)
        if (!valid_tensor(g, inputs[i])) return AMAP_E_INVALID;
    int id = -1;
    amap_status st = amap_graph_input(g, rank, shape, es, &id);
    if (st != AMAP_OK) return st;
    g->t[id].kind = GTensor::COMPUTE;
    g->t[id].inputs.assign(inputs, inputs + n_inputs);
    *tensor = id;
    return AMAP_OK;
    GUARD_END
}

extern "C" amap_status amap_graph_output(amap_graph_t *g, int tensor) {
    if (!g || g->done || !valid_tensor(g, tensor)) return AMAP_E_INVALID;
    g->t[tensor].output = true;
    return AMAP_OK;
}

extern "C" amap_status amap_graph_eliminate(amap_graph_t *g, amap_graph_report *rep) {
    GUARD_BEGIN
    if (!g || !rep || g->done) return AMAP_E_INVALID;
    amap_graph_report r{};
    // every load starts as the identity of the tensor it reads
    auto identity = [&](int id, amap **out) {
        const GTensor &x = g->t[id];
        return amap_source(id, (int)x.shape.size(), x.shape.data(), (amap_elem)x.elem, out);
    };
    for (int c = 0; c < (int)g->t.size(); ++c) {
        const GTensor &x = g->t[c];
        if (x.kind == GTensor::LAYOUT) {
            ++r.n_layout_ops;
            r.n_pairs += x.pairs;
            r.moved_bytes_before += moved_bytes(*x.def);
            r.intermediate_bytes += volume_of(x.shape) * x.elem;
        }
        if (x.kind == GTensor::COMPUTE) {
            for (int s = 0; s < (int)x.inputs.size(); ++s) {
                amap *m = nullptr;
                amap_status st = identity(x.inputs[s], &m);
                if (st != AMAP_OK) return st;
                g->loads.push_back(GLoad{c, s, std::unique_ptr<amap>(m)});
            }
        }
        if (x.output) {
            amap *m = nullptr;
            amap_status st = identity(c, &m);
            if (st != AMAP_OK) return st;
            g->loads.push_back(GLoad{-1, c, std::unique_ptr<amap>(m)});
        }
    }
    // fixed point: while some load still reads a tensor t_s defined by a pair,
    // rewrite that load to read what t_s was copied from (eq. 4)
    for (GLoad &L : g->loads) {
        for (;;) {
            int ts = -1;
            for (int id : sources_of(*L.map))
                if (g->t[id].kind == GTensor::LAYOUT) {
                    ts = id;
                    break;
                }
            if (ts < 0) break;
            const amap *def = g->t[ts].def.get();
            Leaf leaf = [&](int id, const std::vector<int64_t> &shape, int elem, amap **out) -> amap_status {
                if (id == ts) {
                    *out = new amap(*def);
                    return AMAP_OK;
                }
                return amap_source(id, (int)shape.size(), shape.data(), (amap_elem)elem, out);
            };
            amap *next = nullptr;
            amap_status st = replay(L.map->prog.get(), L.map->elem, leaf, &next);
            if (st != AMAP_OK) return st;
            L.map.reset(next);
            ++r.n_rewrites;
        }
    }
    r.n_loads = (int)g->loads.size();
    for (const GLoad &L : g->loads) {
        if (L.consumer >= 0) {
            // a compute operator that cannot take a map in its own operand load
            // needs this load materialised by one composed copy
            const std::vector<int> ids = sources_of(*L.map);
            if (!(ids.size() == 1 && is_identity(*L.map, g->t[ids[0]].shape))) {
                ++r.n_mapped_loads;
                r.mapped_load_bytes += moved_bytes(*L.map);
            }
            continue;
        }
        if (g->t[L.slot].kind != GTensor::LAYOUT) continue;
        const std::vector<int> ids = sources_of(*L.map);
        if (ids.size() == 1 && is_identity(*L.map, g->t[ids[0]].shape)) {
            ++r.n_alias_outputs;
            continue;
        }
        r.n_pairs_left += std::max<int>(1, (int)ids.size());
        r.moved_bytes_after += moved_bytes(*L.map);
        r.intermediate_bytes -= volume_of(g->t[L.slot].shape) * g->t[L.slot].elem;  // this one still exists
    }
    g->done = true;
    *rep = r;
    return AMAP_OK;
    GUARD_END
}

extern "C" amap_status amap_graph_load(const amap_graph_t *g, int index, int *consumer, int *slot, amap_t **map,
                                       int *src_tensors, int *n_src) {
    GUARD_BEGIN
    if (!g || !g->done || index < 0 || index >= (int)g->loads.size() || !consumer || !slot || !map || !src_tensors ||
        !n_src)
        return AMAP_E_INVALID;
    const GLoad &L = g->loads[index];
    const std::vector<int> ids = sources_of(*L.map);
    if (ids.size() > 16) return AMAP_E_UNSUPPORTED;
    // renumber the tensors the map reads to 0 .. n-1
    // (a leaf that no piece reads gets a number past the end and drops out of the new map)
    int spare = (int)ids.size();
    Leaf leaf = [&](int id, const std::vector<int64_t> &shape, int elem, amap **out) -> amap_status {
        const auto at = std::find(ids.begin(), ids.end(), id);
        const int k = at != ids.end() ? (int)(at - ids.begin()) : spare++;
        return amap_source(k, (int)shape.size(), shape.data(), (amap_elem)elem, out);
    };
    amap *m = nullptr;
    amap_status st = replay(L.map->prog.get(), L.map->elem, leaf, &m);
    if (st != AMAP_OK) return st;
    *consumer = L.consumer;
    *slot = L.slot;
    *map = m;
    *n_src = (int)ids.size();
    for (size_t k = 0; k < ids.size(); ++k) src_tensors[k] = ids[k];
    return AMAP_OK;
    GUARD_END
}
