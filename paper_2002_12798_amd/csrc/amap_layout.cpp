// Global layout assignment: the GPU counterpart of the paper's global
// memory-bank mapping (Section 2.2).  The paper derives bank mappings for the
// operators that restrict them, propagates the mappings across the network
// along the data dependencies with a fixed-point iteration, and inserts a
// tensor t' and a copy t -> t' only where a tensor meets conflicting
// requirements; its baseline ("local mapping") decides inside each operator.
// On a GPU the analogous per-tensor property is the order of the dimensions in
// HBM (which one is contiguous, i.e. coalesced); a conflict costs a relayout
// copy, which is a transpose map for amap_execute.
#include <algorithm>
#include <memory>
#include <new>
#include <vector>

#include "amap_map.hpp"

using namespace amap_detail;

namespace {

using Order = std::vector<int32_t>;

struct LTensor {
    std::vector<int64_t> shape;
    int elem = 2;
    bool fixed = false;
    Order order;  // empty = not assigned yet
    int producer = -1;
};

struct LOperand {
    int tensor;
    bool output;
    Order req;  // empty = free
};

struct LOp {
    std::vector<LOperand> x;
    bool same_layout;
};

struct LCopy {
    int op, slot, tensor;
    Order from, to;  // orders of the source and of the destination of the copy
};

bool valid_order(const int32_t *o, int rank) {
    bool seen[kMaxRank] = {false};
    for (int k = 0; k < rank; ++k) {
        if (o[k] < 0 || o[k] >= rank || seen[o[k]]) return false;
        seen[o[k]] = true;
    }
    return true;
}

Order canonical(int rank) {
    Order o(rank);
    for (int k = 0; k < rank; ++k) o[k] = k;
    return o;
}

int64_t bytes_of(const LTensor &t) { return volume_of(t.shape) * t.elem; }

}  // namespace

struct amap_layout_graph {
    std::vector<LTensor> t;
    std::vector<LOp> ops;
    std::vector<LCopy> copies;
    bool solved = false;
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

extern "C" amap_status amap_layout_create(amap_layout_graph_t **out) {
    GUARD_BEGIN
    if (!out) return AMAP_E_INVALID;
    *out = new amap_layout_graph();
    return AMAP_OK;
    GUARD_END
}

extern "C" void amap_layout_free(amap_layout_graph_t *g) { delete g; }

extern "C" amap_status amap_layout_tensor(amap_layout_graph_t *g, int rank, const int64_t *shape, amap_elem es,
                                          const int32_t *fixed_order, int *tensor) {
    GUARD_BEGIN
    if (!g || !shape || !tensor || g->solved || rank < 1 || rank > kMaxRank) return AMAP_E_INVALID;
    if (es != AMAP_B16 && es != AMAP_B32) return AMAP_E_INVALID;
    for (int k = 0; k < rank; ++k)
        if (shape[k] < 0) return AMAP_E_INVALID;
    if (fixed_order && !valid_order(fixed_order, rank)) return AMAP_E_INVALID;
    LTensor x;
    x.shape.assign(shape, shape + rank);
    x.elem = (int)es;
    if (fixed_order) {
        x.fixed = true;
        x.order.assign(fixed_order, fixed_order + rank);
    }
    g->t.push_back(std::move(x));
    *tensor = (int)g->t.size() - 1;
    return AMAP_OK;
    GUARD_END
}

extern "C" amap_status amap_layout_op(amap_layout_graph_t *g, const int *operands, const int *is_output,
                                      const int32_t *const *req_orders, int n, int same_layout, int *op) {
    GUARD_BEGIN
    if (!g || !operands || !is_output || n < 1 || !op || g->solved) return AMAP_E_INVALID;
    LOp o;
    o.same_layout = same_layout != 0;
    for (int i = 0; i < n; ++i) {
        if (operands[i] < 0 || operands[i] >= (int)g->t.size()) return AMAP_E_INVALID;
        LTensor &x = g->t[operands[i]];
        LOperand a;
        a.tensor = operands[i];
        a.output = is_output[i] != 0;
        if (req_orders && req_orders[i]) {
            if (!valid_order(req_orders[i], (int)x.shape.size())) return AMAP_E_INVALID;
            a.req.assign(req_orders[i], req_orders[i] + x.shape.size());
        }
        if (a.output) {
            if (x.producer >= 0) return AMAP_E_INVALID;  // one producer per tensor
            x.producer = (int)g->ops.size();
        }
        o.x.push_back(std::move(a));
    }
    g->ops.push_back(std::move(o));
    *op = (int)g->ops.size() - 1;
    return AMAP_OK;
    GUARD_END
}

extern "C" amap_status amap_layout_solve(amap_layout_graph_t *g, amap_layout_report *rep) {
    GUARD_BEGIN
    if (!g || !rep || g->solved) return AMAP_E_INVALID;
    amap_layout_report r{};

    // ---- local assignment: every operator decides for itself.  A restricted operand is in the
    // order its operator asks for, anything else in the canonical order; a copy wherever what the
    // producer wrote is not what a consumer reads.
    auto local_order = [&](const LOperand &a) { return a.req.empty() ? canonical((int)g->t[a.tensor].shape.size()) : a.req; };
    for (size_t ti = 0; ti < g->t.size(); ++ti) {
        const LTensor &x = g->t[ti];
        Order written = x.fixed ? x.order : canonical((int)x.shape.size());
        bool produced_fixed_mismatch = false;
        if (x.producer >= 0)
            for (const LOperand &a : g->ops[x.producer].x)
                if (a.output && a.tensor == (int)ti) {
                    const Order w = local_order(a);
                    if (x.fixed && w != x.order) produced_fixed_mismatch = true;  // copy into the required order
                    if (!x.fixed) written = w;
                }
        if (produced_fixed_mismatch) {
            ++r.n_copies_local;
            r.copy_bytes_local += 2 * bytes_of(x);
        }
        for (const LOp &o : g->ops)
            for (const LOperand &a : o.x)
                if (!a.output && a.tensor == (int)ti && local_order(a) != written) {
                    ++r.n_copies_local;
                    r.copy_bytes_local += 2 * bytes_of(x);
                }
    }

    // ---- global assignment.  Seeds: fixed tensors, then what restricted operators write, then
    // what restricted operators read.
    for (int pass = 0; pass < 2; ++pass)
        for (const LOp &o : g->ops)
            for (const LOperand &a : o.x)
                if (!a.req.empty() && a.output == (pass == 0) && g->t[a.tensor].order.empty()) g->t[a.tensor].order = a.req;
    // Propagation through the unrestricted operators, in both directions, to a fixed point.
    for (bool changed = true; changed;) {
        changed = false;
        ++r.n_sweeps;
        for (const LOp &o : g->ops) {
            if (!o.same_layout) continue;
            for (int rank = 1; rank <= kMaxRank; ++rank) {
                const Order *have = nullptr;
                for (const LOperand &a : o.x)  // inputs first: data flows forwards
                    if (a.req.empty() && !a.output && (int)g->t[a.tensor].shape.size() == rank && !g->t[a.tensor].order.empty()) {
                        have = &g->t[a.tensor].order;
                        break;
                    }
                if (!have)
                    for (const LOperand &a : o.x)
                        if (a.req.empty() && (int)g->t[a.tensor].shape.size() == rank && !g->t[a.tensor].order.empty()) {
                            have = &g->t[a.tensor].order;
                            break;
                        }
                if (!have) continue;
                const Order pick = *have;
                for (const LOperand &a : o.x)
                    if (a.req.empty() && (int)g->t[a.tensor].shape.size() == rank && g->t[a.tensor].order.empty()) {
                        g->t[a.tensor].order = pick;
                        changed = true;
                    }
            }
        }
    }
    for (LTensor &x : g->t)
        if (x.order.empty()) x.order = canonical((int)x.shape.size());

    // ---- cost of an assignment, and the order an unrestricted operator works in
    const size_t nt = g->t.size();
    // the order of the free operands of one rank that leaves the fewest bytes to convert
    auto work_order = [&](const LOp &o, size_t rank, const std::vector<Order> &ord) {
        Order best;
        int64_t best_cost = -1;
        for (const LOperand &c : o.x) {
            if (!c.req.empty() || g->t[c.tensor].shape.size() != rank) continue;
            const Order &cand = ord[c.tensor];
            int64_t cost = 0;
            for (const LOperand &b : o.x)
                if (b.req.empty() && g->t[b.tensor].shape.size() == rank && ord[b.tensor] != cand) cost += 2 * bytes_of(g->t[b.tensor]);
            if (best_cost < 0 || cost < best_cost) {
                best_cost = cost;
                best = cand;
            }
        }
        return best;
    };
    auto need_of = [&](const LOp &o, const LOperand &a, const std::vector<Order> &ord) {
        if (!a.req.empty()) return a.req;
        return o.same_layout ? work_order(o, g->t[a.tensor].shape.size(), ord) : Order();
    };
    auto cost_of = [&](const std::vector<Order> &ord) {
        int64_t c = 0;
        for (const LOp &o : g->ops)
            for (const LOperand &a : o.x) {
                const Order need = need_of(o, a, ord);
                if (!need.empty() && need != ord[a.tensor]) c += 2 * bytes_of(g->t[a.tensor]);
            }
        return c;
    };
    std::vector<Order> ord(nt);
    for (size_t ti = 0; ti < nt; ++ti) ord[ti] = g->t[ti].order;
    // The propagation is a heuristic.  The per-operator assignment is an assignment too (every
    // tensor stored the way its producer writes it): start from whichever of the two is cheaper ...
    {
        std::vector<Order> loc(nt);
        for (size_t ti = 0; ti < nt; ++ti) {
            const LTensor &x = g->t[ti];
            loc[ti] = x.fixed ? x.order : canonical((int)x.shape.size());
            if (!x.fixed && x.producer >= 0)
                for (const LOperand &a : g->ops[x.producer].x)
                    if (a.output && a.tensor == (int)ti && !a.req.empty()) loc[ti] = a.req;
        }
        if (cost_of(loc) < cost_of(ord)) ord = loc;
    }
    // ... and let every free tensor try the orders its operators ask for or its neighbours have,
    // one tensor at a time, for as long as the total shrinks.
    for (int sweep = 0; sweep < 16; ++sweep) {
        bool better = false;
        for (size_t ti = 0; ti < nt; ++ti) {
            if (g->t[ti].fixed) continue;
            std::vector<Order> cands;
            for (const LOp &o : g->ops) {
                bool mine = false;
                for (const LOperand &a : o.x) mine = mine || a.tensor == (int)ti;
                if (!mine) continue;
                for (const LOperand &a : o.x) {
                    if (a.tensor == (int)ti && !a.req.empty()) cands.push_back(a.req);
                    if (a.tensor != (int)ti && a.req.empty() && o.same_layout &&
                        g->t[a.tensor].shape.size() == g->t[ti].shape.size())
                        cands.push_back(ord[a.tensor]);
                }
            }
            int64_t cur = cost_of(ord);
            for (const Order &c : cands) {
                if (c == ord[ti]) continue;
                const Order keep = ord[ti];
                ord[ti] = c;
                const int64_t now = cost_of(ord);
                if (now < cur) {
                    cur = now;
                    better = true;
                } else {
                    ord[ti] = keep;
                }
            }
        }
        if (!better) break;
    }
    for (size_t ti = 0; ti < nt; ++ti) g->t[ti].order = ord[ti];
    // Conflicts: an operand whose operator needs another order than the tensor has.
    for (size_t oi = 0; oi < g->ops.size(); ++oi) {
        const LOp &o = g->ops[oi];
        for (size_t si = 0; si < o.x.size(); ++si) {
            const LOperand &a = o.x[si];
            const LTensor &x = g->t[a.tensor];
            const Order need = need_of(o, a, ord);
            if (need.empty() || need == x.order) continue;
            LCopy c;
            c.op = (int)oi;
            c.slot = (int)si;
            c.tensor = a.tensor;
            c.from = a.output ? need : x.order;
            c.to = a.output ? x.order : need;
            g->copies.push_back(std::move(c));
            ++r.n_copies_global;
            r.copy_bytes_global += 2 * bytes_of(x);
        }
    }
    g->solved = true;
    *rep = r;
    return AMAP_OK;
    GUARD_END
}

extern "C" amap_status amap_layout_order(const amap_layout_graph_t *g, int tensor, int32_t *order) {
    if (!g || !g->solved || !order || tensor < 0 || tensor >= (int)g->t.size()) return AMAP_E_INVALID;
    const Order &o = g->t[tensor].order;
    for (size_t k = 0; k < o.size(); ++k) order[k] = o[k];
    return AMAP_OK;
}

extern "C" amap_status amap_layout_copy(const amap_layout_graph_t *g, int index, int *op, int *slot, int *tensor,
                                        amap_t **map) {
    GUARD_BEGIN
    if (!g || !g->solved || index < 0 || index >= (int)g->copies.size() || !op || !slot || !tensor || !map)
        return AMAP_E_INVALID;
    const LCopy &c = g->copies[index];
    const LTensor &x = g->t[c.tensor];
    const int rank = (int)x.shape.size();
    // source: the tensor with its dimensions in order `from`; dst dimension k is logical dimension
    // to[k], which sits at position pos_from[to[k]] of the source
    int64_t sshape[kMaxRank];
    int32_t pos[kMaxRank], perm[kMaxRank];
    for (int k = 0; k < rank; ++k) {
        sshape[k] = x.shape[c.from[k]];
        pos[c.from[k]] = k;
    }
    for (int k = 0; k < rank; ++k) perm[k] = pos[c.to[k]];
    amap *s = nullptr;
    amap_status st = amap_source(0, rank, sshape, (amap_elem)x.elem, &s);
    if (st != AMAP_OK) return st;
    std::unique_ptr<amap> hold(s);
    amap *m = nullptr;
    st = amap_transpose(s, perm, &m);
    if (st != AMAP_OK) return st;
    *op = c.op;
    *slot = c.slot;
    *tensor = c.tensor;
    *map = m;
    return AMAP_OK;
    GUARD_END
}
