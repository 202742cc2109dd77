// Host-side inspection (amap_describe, the text behind the last error) and the host evaluator of a
// map.  The evaluator exists so that the composer can be tested on machines without a GPU; the device
// entry points never call it.  Nothing in this file touches the GPU runtime.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include <cstdio>

#include "amap_map.hpp"
#include "amap_plan.hpp"

using namespace amap_detail;

namespace {

template <class F>
void for_each_index(const std::vector<int64_t> &shape, F &&f) {
    if (volume_of(shape) == 0) return;
    const int rank = (int)shape.size();
    int64_t idx[kMaxRank] = {0};
    for (;;) {
        f(idx);
        int k = rank - 1;
        for (; k >= 0; --k) {
            if (++idx[k] < shape[k]) break;
            idx[k] = 0;
        }
        if (k < 0) return;
    }
}

// visit (dst offset, src offset) of every iteration of a kernel-form piece
template <class F>
void for_each_iteration(const KPiece &p, F &&f) {
    const int nd = (int)p.dims.size();
    std::vector<int64_t> i(nd, 0);
    int64_t d = p.dbase, s = p.sbase;
    for (;;) {
        f(d, s);
        int k = nd - 1;
        for (; k >= 0; --k) {
            d += p.dims[k].ds;
            s += p.dims[k].ss;
            if (++i[k] < p.dims[k].extent) break;
            d -= p.dims[k].ds * p.dims[k].extent;
            s -= p.dims[k].ss * p.dims[k].extent;
            i[k] = 0;
        }
        if (k < 0) return;
    }
}

inline void put(void *dst, int64_t off, const void *src, int64_t soff, int es) {
    std::memcpy((char *)dst + off * es, (const char *)src + soff * es, (size_t)es);
}

}  // namespace

namespace {

// Elements a piece reads when no two of its iterations (stride-0 loops removed) meet in the
// source: with the loops sorted by |stride|, every stride is larger than the span of all
// smaller ones.  -1 if that test fails (the loops may still be injective; the caller then counts).
int64_t injective_read_count(const KPiece &p) {
    std::vector<KDim> d;
    for (const KDim &k : p.dims)
        if (k.ss != 0 && k.extent > 1) d.push_back(k);
    std::sort(d.begin(), d.end(), [](const KDim &x, const KDim &y) { return std::llabs(x.ss) < std::llabs(y.ss); });
    int64_t span = 0, n = 1;
    for (const KDim &k : d) {
        if (std::llabs(k.ss) <= span) return -1;
        span += std::llabs(k.ss) * (k.extent - 1);
        n *= k.extent;
    }
    return n;
}

}  // namespace

int64_t amap_detail::distinct_source_elements(const amap &m) {
    if (m.distinct_reads >= 0) return m.distinct_reads;
    int64_t n = 0;
    // the common cases need no walk: a source read by ONE piece whose moving loops do not overlap
    // (repeat, tile, broadcast: loops that stand still in the source drop out)
    std::vector<int> readers(m.src_shapes.size(), 0);
    bool counted = m.strided;
    if (m.strided) {
        for (const KPiece &p : m.kpieces)
            if (!p.fill) ++readers[(size_t)p.src];
        for (const KPiece &p : m.kpieces) {
            if (p.fill) continue;
            const int64_t c = readers[(size_t)p.src] == 1 ? injective_read_count(p) : -1;
            if (c < 0) {
                counted = false;
                break;
            }
            n += c;
        }
    }
    if (!counted) {
        // one bit per source element; refused beyond kMaxDistinctBits (the caller reports AMAP_E_NOMEM)
        int64_t bits = 0;
        for (const auto &sh : m.src_shapes)
            if (!sh.empty()) bits += volume_of(sh);
        if (bits > kMaxDistinctBits) throw std::bad_alloc();
        n = 0;
        std::vector<std::vector<uint8_t>> seen(m.src_shapes.size());
        for (size_t i = 0; i < m.src_shapes.size(); ++i)
            if (!m.src_shapes[i].empty()) seen[i].assign((size_t)((volume_of(m.src_shapes[i]) + 7) / 8), 0);
        auto mark = [&](int sid, int64_t off) {
            uint8_t &b = seen[(size_t)sid][(size_t)(off >> 3)];
            const uint8_t bit = (uint8_t)(1u << (off & 7));
            n += !(b & bit);
            b |= bit;
        };
        if (m.strided) {
            for (const KPiece &p : m.kpieces) {
                if (p.fill) continue;
                KPiece q = p;  // loops that do not move in the source add nothing
                q.dims.erase(std::remove_if(q.dims.begin(), q.dims.end(), [](const KDim &d) { return d.ss == 0; }),
                             q.dims.end());
                for_each_iteration(q, [&](int64_t, int64_t s) { mark(p.src, s); });
            }
        } else {
            for_each_index(m.shape, [&](const int64_t *idx) {
                int sid = -1;
                int64_t off = 0;
                uint32_t fill = 0;
                if (eval_program(m.prog.get(), idx, &sid, &off, &fill)) mark(sid, off);
            });
        }
    }
    m.distinct_reads = n;
    return n;
}

extern "C" amap_status amap_eval_host(const amap_t *m, const void *const *src, void *dst, int mode) {
    if (!m || !dst || mode < 0 || mode > 2) return AMAP_E_INVALID;
    if (volume_of(m->shape) == 0) return AMAP_OK;
    if (!src && !m->src_shapes.empty()) return AMAP_E_INVALID;
    const int es = m->elem;
    const bool use_pieces = mode == 2 || (mode == 0 && m->strided);
    if (use_pieces) {
        if (!m->strided) return AMAP_E_UNSUPPORTED;
        for (const KPiece &p : m->kpieces) {
            if (p.fill) {
                uint32_t f32 = p.fill_bits;
                uint16_t f16 = (uint16_t)p.fill_bits;
                const void *f = es == 2 ? (const void *)&f16 : (const void *)&f32;
                for_each_iteration(p, [&](int64_t d, int64_t) { put(dst, d, f, 0, es); });
            } else {
                if (!src[p.src]) return AMAP_E_INVALID;
                const void *s = src[p.src];
                for_each_iteration(p, [&](int64_t d, int64_t so) { put(dst, d, s, so, es); });
            }
        }
        return AMAP_OK;
    }
    int64_t L = 0;
    amap_status st = AMAP_OK;
    for_each_index(m->shape, [&](const int64_t *idx) {
        int sid = -1;
        int64_t off = 0;
        uint32_t fill = 0;
        if (eval_program(m->prog.get(), idx, &sid, &off, &fill)) {
            if (!src[sid])
                st = AMAP_E_INVALID;
            else
                put(dst, L, src[sid], off, es);
        } else {
            uint16_t f16 = (uint16_t)fill;
            put(dst, L, es == 2 ? (const void *)&f16 : (const void *)&fill, 0, es);
        }
        ++L;
    });
    return st;
}

extern "C" amap_status amap_source_shape(const amap_t *m, int src_id, int *rank, int64_t *shape) {
    if (!m || !rank || !shape || src_id < 0 || src_id >= (int)m->src_shapes.size()) return AMAP_E_INVALID;
    const auto &s = m->src_shapes[src_id];
    if (s.empty()) return AMAP_E_INVALID;
    *rank = (int)s.size();
    for (size_t k = 0; k < s.size(); ++k) shape[k] = s[k];
    return AMAP_OK;
}

// Number of dst elements written zero times / more than once by the pieces:
// both must be 0 for a well-formed strided map (every dst element has exactly
// one writer).  Diagnostic for tests; costs one byte per dst element.
extern "C" amap_status amap_check_cover(const amap_t *m, int64_t *unwritten, int64_t *overwritten) {
    if (!m || !unwritten || !overwritten) return AMAP_E_INVALID;
    if (!m->strided) return AMAP_E_UNSUPPORTED;
    const int64_t vol = volume_of(m->shape);
    std::vector<uint8_t> cnt((size_t)vol, 0);
    int64_t over = 0, bad = 0;
    for (const KPiece &p : m->kpieces) {
        int64_t svol = p.fill ? 0 : volume_of(m->src_shapes[p.src]);
        for_each_iteration(p, [&](int64_t d, int64_t s) {
            if (d < 0 || d >= vol || (!p.fill && (s < 0 || s >= svol))) {
                ++bad;
                return;
            }
            if (cnt[(size_t)d] == 1) ++over;
            if (cnt[(size_t)d] < 2) ++cnt[(size_t)d];
        });
    }
    int64_t un = 0;
    for (uint8_t c : cnt) un += c == 0;
    *unwritten = un;
    *overwritten = over + bad;
    return AMAP_OK;
}

// ---- the text behind the last AMAP_E_HIP / AMAP_E_UNSUPPORTED of this thread
namespace {
thread_local char g_last_error[256] = "";
}

void amap_detail::set_last_error(const char *what, const char *detail) {
    if (detail)
        std::snprintf(g_last_error, sizeof(g_last_error), "%s: %s", what, detail);
    else
        std::snprintf(g_last_error, sizeof(g_last_error), "%s", what);
}

extern "C" const char *amap_last_error(void) { return g_last_error; }

extern "C" amap_status amap_describe(const amap_t *m, amap_info *out) {
    if (!m || !out) return AMAP_E_INVALID;
    try {
    amap_info o;
    std::memset(&o, 0, sizeof(o));
    o.rank = (int)m->shape.size();
    for (int k = 0; k < o.rank; ++k) o.shape[k] = m->shape[k];
    o.elem_size = m->elem;
    o.n_src = (int)m->src_shapes.size();
    o.strided = m->strided ? 1 : 0;
    o.write_bytes = volume_of(m->shape) * m->elem;
    if (m->strided) {
        o.n_pieces = (int)m->kpieces.size();
        for (const KPiece &p : m->kpieces) {
            if (p.fill) {
                ++o.n_fill_pieces;
                o.fill_bytes += p.volume() * m->elem;
            } else {
                o.min_read_bytes += p.volume() * m->elem;
            }
        }
    } else {
        // count the data elements by walking the program over dst
        int64_t idx[kMaxRank] = {0};
        const int rank = o.rank;
        int64_t data = 0, vol = volume_of(m->shape);
        for (int64_t L = 0; L < vol; ++L) {
            int sid;
            int64_t off;
            uint32_t fill;
            data += eval_program(m->prog.get(), idx, &sid, &off, &fill) ? 1 : 0;
            for (int k = rank - 1; k >= 0; --k) {
                if (++idx[k] < m->shape[k]) break;
                idx[k] = 0;
            }
        }
        o.min_read_bytes = data * m->elem;
        o.fill_bytes = (vol - data) * m->elem;
    }
    if (!m->injective) o.min_read_bytes = distinct_source_elements(*m) * m->elem;
    const Plan *plan = plan_of(*m);
    o.kernel_id = plan ? plan->main_kernel : AMAP_K_PROGRAM;
    o.vec_bytes = plan ? plan->min_vec_bytes : m->elem;
    *out = o;
    return AMAP_OK;
    } catch (...) {
        return AMAP_E_NOMEM;   // the marks of a non-injective map over very large sources, or the plan
    }
}
