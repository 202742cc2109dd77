// Host replay of a launch plan: walks every workgroup and every lane of every
// launch with the same index functions the kernels use (amap_index.hpp),
// checks that every address is in bounds, that LDS slots stay inside the
// tile, and that the routing  dst element <- source element  equals the map's
// pieces with exactly one writer per dst element.  It moves no tensor data and
// is never called by the device entry points; tests run it on machines
// without a GPU before any kernel is launched.
#include <cstring>
#include <vector>

#include "amap_index.hpp"
#include "amap_plan.hpp"

using namespace amap_dev;
using namespace amap_detail;

namespace {

constexpr int64_t kUnwritten = -1, kFill = -2;

struct Replay {
    const amap &m;
    std::vector<int64_t> got;      // per dst element: source id * 2^40 + source offset, kFill, kUnwritten
    std::vector<int64_t> src_vol;  // by source id
    int64_t errors = 0;

    explicit Replay(const amap &mm) : m(mm), got((size_t)volume_of(mm.shape), kUnwritten) {
        for (const auto &s : m.src_shapes) src_vol.push_back(s.empty() ? 0 : volume_of(s));
    }

    void write(int64_t d, int64_t code) {
        if (d < 0 || d >= (int64_t)got.size()) {
            ++errors;
            return;
        }
        if (got[(size_t)d] != kUnwritten) ++errors;  // second writer
        got[(size_t)d] = code;
    }
    int64_t code_of(int sid, int64_t soff) {
        if (sid < 0) return kFill;
        if (soff < 0 || soff >= src_vol[(size_t)sid]) {
            ++errors;
            return kFill;
        }
        return ((int64_t)sid << 40) + soff;
    }

    // alone: the launch runs in one of the kernels that decode plain row pieces through all loop slots
    void rows(const DevPiece &P, int sid, uint32_t blk, bool alone) {
        // the expanding, reversing, gathered and interleaving forms are written for 16-byte vectors whatever
        // vlog says: replay what the kernel does, so that a plan with another width shows up as errors
        const bool fixed16 = P.rev || P.rep_log || P.gather || P.inter;
        const uint32_t V = fixed16 ? 16u / (uint32_t)m.elem : 1u << P.vlog;
        const uint32_t threads = 64u << P.nwlog;
        for (uint32_t tid = 0; tid < threads; ++tid)
            for (int u = 0; u < kRowsUnroll; ++u) {
                const uint32_t r = blk * (threads * kRowsUnroll) + tid + u * threads;
                uint32_t d, s;
                {
                    if (r >= P.n_units) continue;
                    if (alone && rows_is_plain(P, m.elem))
                        rows_offsets_fixed(P, r, d, s);
                    else
                        rows_offsets(P, r, d, s);
                }
                if (P.inter >= 3) {
                    // one plane kept: position q reads element q * eP (+ eP - 1 for the last-of-group form)
                    for (uint32_t q = 0; q < V; ++q) {
                        const uint32_t ss = s + q * P.eP + (P.inter == 4 ? P.eP - 1 : 0u);
                        write((int64_t)P.dwin + d + q, code_of(sid, (int64_t)P.swin + (int64_t)(int32_t)ss));
                    }
                    // the rest of the window is loaded too and must exist
                    const int64_t first = (int64_t)P.swin + (int64_t)(int32_t)s, last = first + (int64_t)V * P.eP - 1;
                    if (first < 0 || last >= src_vol[(size_t)sid]) ++errors;
                    continue;
                }
                if (P.inter) {
                    // V positions q of eP planes: interleaved side at q * eP + p, planar side at p * plane + q
                    for (uint32_t pl = 0; pl < P.eP; ++pl)
                        for (uint32_t q = 0; q < V; ++q) {
                            const uint32_t il = q * P.eP + pl, pn = pl * (uint32_t)P.ssP + q;
                            const uint32_t dd = P.inter == 1 ? d + il : d + pn, ss = P.inter == 1 ? s + pn : s + il;
                            write((int64_t)P.dwin + dd, code_of(sid, (int64_t)P.swin + (int64_t)(int32_t)ss));
                        }
                    continue;
                }
                if (P.gather) {
                    const uint32_t rv = r - fdiv(r, P.loops[0].fd) * P.loops[0].extent;
                    GatherCursor c = P.nq == 1 ? gather_begin<1>(P, rv * V) : P.nq == 2 ? gather_begin<2>(P, rv * V) : P.nq == 3 ? gather_begin<3>(P, rv * V) : gather_begin<4>(P, rv * V);
                    for (uint32_t e = 0; e < V; ++e) {
                        write((int64_t)P.dwin + d + e, code_of(sid, (int64_t)P.swin + (int64_t)(int32_t)(s + c.off)));
                        if (P.nq == 1)
                            gather_next<1>(P, c);
                        else if (P.nq == 2)
                            gather_next<2>(P, c);
                        else if (P.nq == 3)
                            gather_next<3>(P, c);
                        else
                            gather_next<4>(P, c);
                    }
                    continue;
                }
                for (uint32_t e = 0; e < V; ++e)
                    write((int64_t)P.dwin + d + e, code_of(sid, P.rev ? (int64_t)P.swin + s - e : (int64_t)P.swin + s + (e >> P.rep_log)));
            }
    }

    // the column-blocked form of a flat tile
    void rag(const DevPiece &P, int sid, uint32_t t, uint32_t lds_bytes) {
        const uint32_t V = 16u / (uint32_t)m.elem, vlog = V == 8 ? 3 : 2, rvlog = P.lqlog - vlog;
        if (P.lqlog != 6 || P.vlog != vlog || (P.flat != 1 && P.flat != 2) || (P.flat == 1 && P.EQ % V) || t >= P.n_blocks || P.nq < 1 || P.nq > 4 ||
            P.nloops + P.nq > (uint32_t)kMaxLoops || P.rag_cb % V || P.rag_s != P.rag_cb / V + 1 || P.rag_w < P.rag_cb || (P.rag_w * m.elem) % 4 ||
            (uint64_t)P.rag_w * 64 * m.elem > lds_bytes || (uint64_t)P.tilesQ * P.rag_cb < P.eP) {
            ++errors;
            return;
        }
        const RagUnit U = rag_unit(P, t);
        const uint32_t C = P.eP, W = P.rag_w, S = P.rag_s, threads = 64u << P.nwlog;
        const uint32_t nrag = U.rcount * S, nstr = U.ccount << rvlog;
        std::vector<int64_t> lds((size_t)lds_bytes / (size_t)m.elem, kUnwritten);
        auto lds_put = [&](uint64_t e, int64_t code) {
            if (e >= lds.size() || lds[e] != kUnwritten)
                ++errors;
            else
                lds[e] = code;
        };
        auto lds_get = [&](uint64_t e) -> int64_t {
            if (e >= lds.size() || lds[e] == kUnwritten) {
                ++errors;
                return kFill;
            }
            return lds[e];
        };
        for (int phase = 0; phase < 2; ++phase)
            for (uint32_t tid = 0; tid < threads; ++tid) {
                const bool rag_side = (phase == 0) == (P.flat == 1);
                if (!rag_side) {
                    for (uint32_t vi = tid; vi < nstr; vi += threads) {
                        const uint32_t rv = vi & ((1u << rvlog) - 1), c = vi >> rvlog;
                        if (rv * V >= U.rcount) continue;
                        for (uint32_t k = 0; k < V && rv * V + k < U.rcount; ++k) {
                            const uint32_t e = (rv * V + k) * W + c, off = flat_c_offset(P, U.c0 + c) + rv * V + k;
                            if (P.flat == 1 && k == 0 && (P.dwin + (uint32_t)(U.doff + off)) % V) ++errors;
                            if (P.flat == 1)
                                write((int64_t)P.dwin + (uint32_t)(U.doff + off), lds_get(e));
                            else
                                lds_put(e, code_of(sid, (int64_t)P.swin + (int64_t)(int32_t)(U.soff + off)));
                        }
                    }
                } else if (P.flat == 1) {
                    for (uint32_t item = tid; item < nrag; item += threads) {
                        const uint32_t r = fdiv(item, P.fd_rag_s), col = (item - r * S) * V;
                        if (col >= U.ccount) continue;
                        const uint32_t a = U.soff + r * C + col, at = r * W + col;
                        if ((at * (uint32_t)m.elem) % 4) ++errors;  // dword LDS stores
                        for (uint32_t i = 0; i < V && col + i < U.ccount; ++i)
                            lds_put(at + i, code_of(sid, (int64_t)P.swin + (int64_t)(int32_t)(a + i)));
                    }
                } else {
                    for (uint32_t item = tid; item < nrag; item += threads) {
                        const uint32_t r = fdiv(item, P.fd_rag_s), s = item - r * S;
                        const uint32_t a = U.doff + r * C, x = (a & ~(V - 1)) + s * V;
                        const uint32_t lo = x > a ? x : a, hi = x + V < a + U.ccount ? x + V : a + U.ccount;
                        if (lo >= hi) continue;
                        if (hi - lo == V && (P.dwin + x) % V) ++errors;
                        for (uint32_t p = lo; p < hi; ++p) write((int64_t)P.dwin + p, lds_get(r * W + (p - a)));
                    }
                }
            }
    }

    // the two phases of a flat tile, lane by lane, with LDS as an array of codes
    void flat(const DevPiece &P, int sid, uint32_t t, uint32_t lds_bytes) {
        const uint32_t V = 16u / (uint32_t)m.elem, vlog = V == 8 ? 3 : 2, rvlog = P.lqlog - vlog;
        if (P.lqlog < 4 || P.lqlog > 6 || P.vlog != vlog || (P.flat != 1 && P.flat != 2) || P.EQ % V || t >= P.n_blocks || P.nq < 1 || P.nq > 4 || P.nloops + P.nq > (uint32_t)kMaxLoops) {
            ++errors;
            return;
        }
        const FlatUnit U = flat_unit(P, t);
        const uint32_t C = P.eP, threads = 64u << P.nwlog;
        const uint32_t nflat = (U.rcount * C) >> vlog, nstr = C << rvlog;
        if ((uint64_t)nflat * 16 > lds_bytes) {
            ++errors;
            return;
        }
        std::vector<int64_t> lds((size_t)lds_bytes / (size_t)m.elem, kUnwritten);
        auto lds_put = [&](uint64_t e, int64_t code) {
            if (e >= lds.size() || lds[e] != kUnwritten)
                ++errors;
            else
                lds[e] = code;
        };
        auto lds_get = [&](uint64_t e) -> int64_t {
            if (e >= lds.size() || lds[e] == kUnwritten) {
                ++errors;
                return kFill;
            }
            return lds[e];
        };
        for (int phase = 0; phase < 2; ++phase)
            for (uint32_t tid = 0; tid < threads; ++tid) {
                const bool flat_side = (phase == 0) == (P.flat == 1);
                if (flat_side) {
                    for (uint32_t i = tid; i < nflat; i += threads)
                        for (uint32_t k = 0; k < V; ++k) {
                            const uint32_t e = i * V + k;
                            if (P.flat == 2 && k == 0 && (P.dwin + U.doff + e) % V) ++errors;  // aligned dst vectors
                            if (P.flat == 1)
                                lds_put(e, code_of(sid, (int64_t)P.swin + (int64_t)(int32_t)(U.soff + e)));
                            else
                                write((int64_t)P.dwin + U.doff + e, lds_get(e));
                        }
                } else {
                    for (uint32_t vi = tid; vi < nstr; vi += threads) {
                        const uint32_t rv = vi & ((1u << rvlog) - 1), c = vi >> rvlog;
                        if (rv * V >= U.rcount) continue;
                        for (uint32_t k = 0; k < V; ++k) {
                            const uint32_t e = (rv * V + k) * C + c, off = flat_c_offset(P, c) + rv * V + k;
                            if (P.flat == 1 && k == 0 && (P.dwin + (uint32_t)(U.doff + off)) % V) ++errors;
                            if (P.flat == 1)
                                write((int64_t)P.dwin + (uint32_t)(U.doff + off), lds_get(e));
                            else
                                lds_put(e, code_of(sid, (int64_t)P.swin + (int64_t)(int32_t)(U.soff + off)));
                        }
                    }
                }
            }
    }

    // cross-lane form: lane k of a unit stores, at Q position w0 + k, element k of the vector that each of
    // the unit's V lanes (xl_npv lanes apart, lane j holding P index + j) has loaded
    void xlane(const DevPiece &P, uint32_t blk) {
        const uint32_t vlog = P.vlog, V = 1u << vlog;
        if (V * (uint32_t)m.elem != 16 || P.xl_npv < 1 || P.xl_rows < V || P.xl_rows % V || P.xl_rows * P.xl_npv > 64 || P.tilesP != 1) {
            ++errors;
            return;
        }
        for (uint32_t wave = 0; wave < (1u << P.nwlog); ++wave) {
            const uint32_t t = (blk << P.nwlog) + wave;
            if (t >= P.n_units) continue;
            const TileGeom G = tile_geometry(P, vlog, t);
            XlaneLane L[64];
            for (uint32_t lane = 0; lane < 64; ++lane) L[lane] = xlane_lane(P, G, vlog, lane);
            for (uint32_t lane = 0; lane < 64; ++lane) {
                if (!L[lane].ok) continue;
                for (uint32_t j = 0; j < V; ++j) {
                    const uint32_t from = L[lane].lane0 + j * P.xl_npv;   // the unit's lane that loaded P index + j
                    if (from >= 64 || !L[from].ok || L[from].k != j || L[from].lane0 != L[lane].lane0 || L[from].sub != L[lane].sub) {
                        ++errors;
                        continue;
                    }
                    const int sid = (int)(uintptr_t)L[from].src - 1;
                    write((int64_t)P.dwin + L[lane].doff + j, code_of(sid, (int64_t)(&P)[L[from].sub].swin + L[from].soff + L[lane].k));
                }
            }
        }
    }

    void tile(const DevPiece &P, uint32_t t, uint32_t lds_bytes) {
        const uint32_t vlog = P.vlog, V = 1u << vlog;
        const TileGeom G = tile_geometry(P, vlog, t);
        const bool use_lds = P.kind == PK_TILE;
        std::vector<int64_t> lds;
        if (use_lds) {
            if ((uint64_t)G.TP * G.TQ * m.elem > lds_bytes) {
                ++errors;
                return;
            }
            lds.assign((size_t)G.TP * G.TQ, kUnwritten);
        }
        for (uint32_t tid = 0; tid < (64u << P.nwlog); ++tid) {
            const TileLane L = tile_lane(P, G, vlog, tid);
            if (!L.valid) continue;
            const int sid = (int)(uintptr_t)L.src - 1;
            for (uint32_t j = 0; j < V; ++j) {
                // out[j] = elements along P (i = 0..V-1) at Q position w0 + j: in[i].elem[j]
                for (uint32_t i = 0; i < V; ++i) {
                    const int64_t code = code_of(sid, (int64_t)(&P)[L.sub].swin + L.soff + (int64_t)i * L.ssP + j);
                    if (use_lds) {
                        const uint64_t slot = tile_lds_slot(G, vlog, L.r0 + j, L.pvl);
                        const uint64_t at = slot * V + i;
                        if (at >= lds.size() || lds[at] != kUnwritten)
                            ++errors;
                        else
                            lds[at] = code;
                    } else {
                        write((int64_t)P.dwin + G.db + q_chain_offset(P, L.w0 + j) + L.p + i, code);
                    }
                }
            }
        }
        if (!use_lds) return;
        const uint32_t nvec = G.TQ << G.ncvlog;
        for (uint32_t vi = 0; vi < nvec; ++vi) {
            const TileStore S = tile_store(P, G, vlog, vi);
            if (!S.ok) continue;
            for (uint32_t i = 0; i < V; ++i) {
                const uint64_t at = (uint64_t)S.slot * V + i;
                if (at >= lds.size() || lds[at] == kUnwritten) {
                    ++errors;
                    continue;
                }
                write((int64_t)P.dwin + S.doff + i, lds[at]);
            }
        }
    }
};

}  // namespace

// Replays the plan of `m` for the given kernel family (-1 = planned) on the
// host.  *n_errors = out-of-bounds accesses + dst elements with no or several
// writers + dst elements routed from the wrong source element.
extern "C" amap_status amap_plan_selfcheck(const amap_t *m, int kernel_id, int64_t *n_errors) {
    if (!m || !n_errors) return AMAP_E_INVALID;
    try {
        Plan forced;
        const Plan *plan = nullptr;
        if (kernel_id < 0) {
            plan = plan_of(*m);
        } else {
            if (!plan_strided(*m, kernel_id, forced)) return AMAP_E_UNSUPPORTED;
            plan = &forced;
        }
        if (!plan || !plan->strided_ok) return AMAP_E_UNSUPPORTED;
        Replay R(*m);
        for (size_t li = 0; li < plan->launches.size(); ++li) {
            const LaunchArgs &A = plan->launches[li];
            std::vector<uint8_t> seen(plan->grid[li], 0);
            for (uint32_t hw = 0; hw < plan->grid[li]; ++hw) {
                const uint32_t b = logical_block(A, hw, plan->grid[li]);
                if (b >= plan->grid[li] || seen[b]++) {
                    ++R.errors;
                    continue;
                }
                uint32_t pi = 0;
                for (uint32_t k = 1; k < A.n_pieces; ++k)
                    if (A.p[k].n_blocks && b >= A.p[k].first_block) pi = k;
                const DevPiece &P = A.p[pi];
                if (P.nwlog != A.nwlog || P.nwplog > P.nwlog || P.group_n < 1 || pi + P.group_n > A.n_pieces) ++R.errors;
                const int sid = (int)(uintptr_t)P.src - 1;
                const uint32_t local = b - P.first_block;
                if (local >= P.n_blocks) {
                    ++R.errors;
                    continue;
                }
                if (P.kind == PK_ROWS)
                    R.rows(P, sid, local, A.n_pieces == 1 || launch_is_tile16(A, m->elem) || launch_is_plain_rows(A, m->elem));
                else if (P.kind == PK_FLAT && P.rag_cb)
                    R.rag(P, sid, local, plan->lds_bytes[li]);
                else if (P.kind == PK_FLAT)
                    R.flat(P, sid, local, plan->lds_bytes[li]);
                else if (P.kind == PK_XLANE)
                    R.xlane(P, local);
                else
                    R.tile(P, local, plan->lds_bytes[li]);
            }
        }
        // expected routing straight from the pieces
        std::vector<int64_t> want(R.got.size(), kUnwritten);
        for (const KPiece &p : m->kpieces) {
            const int nd = (int)p.dims.size();
            std::vector<int64_t> i(nd, 0);
            int64_t d = p.dbase, s = p.sbase;
            for (;;) {
                if (d >= 0 && d < (int64_t)want.size()) want[(size_t)d] = p.fill ? kFill : (((int64_t)p.src << 40) + s);
                int k = nd - 1;
                for (; k >= 0; --k) {
                    d += p.dims[k].ds;
                    s += p.dims[k].ss;
                    if (++i[k] < p.dims[k].extent) break;
                    d -= p.dims[k].ds * p.dims[k].extent;
                    s -= p.dims[k].ss * p.dims[k].extent;
                    i[k] = 0;
                }
                if (k < 0) break;
            }
        }
        for (size_t d = 0; d < want.size(); ++d)
            if (want[d] != R.got[d]) ++R.errors;
        *n_errors = R.errors;
        return AMAP_OK;
    } catch (...) {
        return AMAP_E_NOMEM;
    }
}
