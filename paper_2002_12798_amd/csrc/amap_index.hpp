// Index arithmetic of the piece kernels, written once and compiled both for
// the GPU (used by the kernels) and for the host (used by the plan checker,
// which replays every lane of every launch on the CPU and verifies that all
// addresses are in bounds and that every dst element has exactly one writer).
#pragma once

#include "amap_device.hpp"

#if defined(__HIPCC__)
#define AMAP_HD __host__ __device__ __forceinline__
#else
#define AMAP_HD inline
#endif

namespace amap_dev {

AMAP_HD uint32_t fdiv(uint32_t n, FastDiv f) {
#if defined(__HIP_DEVICE_COMPILE__)
    return (__umulhi(n, f.mul) + n) >> f.shift;
#else
    return (uint32_t)((((uint64_t)n * f.mul) >> 32) + n) >> f.shift;
#endif
}

// Workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD
// b % 8), and each XCD has its own L2.  Remap the hardware workgroup index so
// that every XCD works on one contiguous eighth of the logical tile sequence:
// tiles that are neighbours in memory (and may share a cache line at their
// edges) then meet in the same L2.  A bijection on [0, grid).
AMAP_HD uint32_t xcd_remap(uint32_t b, uint32_t grid) {
    const uint32_t x = b & 7, idx = b >> 3;
    const uint32_t q = grid >> 3, r = grid & 7;
    return x * q + (x < r ? x : r) + idx;
}

AMAP_HD uint32_t logical_block(const LaunchArgs &a, uint32_t hw, uint32_t grid) {
    return a.xcd_remap ? xcd_remap(hw, grid) : hw;
}

// ---- row kernel: vector r of the piece (dst order) -> element offsets
// Up to four loops (the common case) are decoded with a fixed trip count: the loop descriptors are then
// read once, side by side, instead of one dependent scalar load per loop and vector (a 25 MB row copy:
// 7.7 -> 6.8 us).  A descriptor past nloops is all zero there (the forms that keep loops at the END of
// loops[] use slots 4 and up): its divider hands r on unchanged and its strides add nothing.
AMAP_HD void rows_offsets(const DevPiece &P, uint32_t r, uint32_t &doff, uint32_t &soff) {
    uint32_t d = P.dbase, s = P.sbase;
    if (P.nloops <= 4) {
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            const uint32_t q = fdiv(r, P.loops[k].fd);
            const uint32_t dig = r - q * P.loops[k].extent;
            d += dig * (uint32_t)P.loops[k].ds;
            s += dig * (uint32_t)P.loops[k].ss;
            r = q;
        }
    } else {
        for (uint32_t k = 0; k < P.nloops; ++k) {
            const uint32_t q = fdiv(r, P.loops[k].fd);
            const uint32_t dig = r - q * P.loops[k].extent;
            d += dig * (uint32_t)P.loops[k].ds;
            s += dig * (uint32_t)P.loops[k].ss;
            r = q;
        }
    }
    doff = d;
    soff = s;
}

// ---- a launch of one plain row piece (16-byte vectors copied or filled, nothing reshuffled in registers) runs
// in a kernel of its own, which decodes through all kMaxLoops descriptors with a fixed trip count: they are
// read once, side by side, and a descriptor past nloops is all zero (it hands r on and adds nothing).
AMAP_HD bool rows_is_plain(const DevPiece &P, int es) {
    return P.kind == PK_ROWS && !P.rep_log && !P.rev && !P.gather && !P.inter && (es << P.vlog) == 16;
}
// ---- a launch whose first piece is an LDS-staged tile piece (or group) of 16-byte vectors and whose other
// pieces are plain row pieces (the fills around a padded tensor) runs in a kernel of its own as well
AMAP_HD bool launch_is_tile16(const LaunchArgs &a, int es) {
    if (a.n_pieces == 0) return false;
    const DevPiece &H = a.p[0];
    if (H.kind != PK_TILE || (es << H.vlog) != 16 || H.group_n < 1 || H.group_n > a.n_pieces || H.n_blocks == 0) return false;
    for (uint32_t k = 1; k < H.group_n; ++k)
        if (a.p[k].n_blocks) return false;
    for (uint32_t k = H.group_n; k < a.n_pieces; ++k)
        if (!rows_is_plain(a.p[k], es)) return false;
    return true;
}
// ---- a launch of several plain row pieces (the outputs of one multi-output call, a copy with its fills)
AMAP_HD bool launch_is_plain_rows(const LaunchArgs &a, int es) {
    for (uint32_t k = 0; k < a.n_pieces; ++k)
        if (!rows_is_plain(a.p[k], es) || a.p[k].n_blocks == 0) return false;
    return a.n_pieces > 0 && !a.xcd_remap;
}
AMAP_HD void rows_offsets_fixed(const DevPiece &P, uint32_t r, uint32_t &doff, uint32_t &soff) {
    uint32_t d = P.dbase, s = P.sbase;
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
#endif
    for (uint32_t k = 0; k < (uint32_t)kMaxLoops; ++k) {
        const uint32_t q = fdiv(r, P.loops[k].fd);
        const uint32_t dig = r - q * P.loops[k].extent;
        d += dig * (uint32_t)P.loops[k].ds;
        s += dig * (uint32_t)P.loops[k].ss;
        r = q;
    }
    doff = d;
    soff = s;
}

// ---- flat tiles (see DevPiece::flat): workgroup t -> element offsets of its block on both sides
// (of row r0, c = 0), and the number of rows in the block
// rows per block = 1 << P.lqlog (16, 32 or 64: as many as fit LDS)
struct FlatUnit {
    uint32_t doff, soff, rcount;
};
AMAP_HD FlatUnit flat_unit(const DevPiece &P, uint32_t t) {
    uint32_t rest = fdiv(t, P.fdTP);
    const uint32_t r0 = (t - rest * P.tilesP) << P.lqlog;
    uint32_t d = P.dbase, s = P.sbase;
    for (uint32_t k = 0; k < P.nloops; ++k) {
        const uint32_t q = fdiv(rest, P.loops[k].fd);
        const uint32_t dig = rest - q * P.loops[k].extent;
        d += dig * (uint32_t)P.loops[k].ds;
        s += dig * (uint32_t)P.loops[k].ss;
        rest = q;
    }
    FlatUnit u;
    u.doff = d + (P.flat == 1 ? r0 : r0 * P.eP);
    u.soff = s + (P.flat == 1 ? r0 * P.eP : r0);
    const uint32_t left = P.EQ - r0;
    u.rcount = left < (1u << P.lqlog) ? left : (1u << P.lqlog);
    return u;
}

// column-blocked form: workgroup t -> block (rows from r0, columns from c0), offsets of (r0, c0)
struct RagUnit {
    uint32_t doff, soff, rcount, c0, ccount;
};
AMAP_HD RagUnit rag_unit(const DevPiece &P, uint32_t t) {
    uint32_t rest = fdiv(t, P.fdTQ);
    const uint32_t c0 = (t - rest * P.tilesQ) * P.rag_cb;
    const uint32_t t2 = rest;
    rest = fdiv(t2, P.fdTP);
    const uint32_t r0 = (t2 - rest * P.tilesP) << P.lqlog;
    uint32_t d = P.dbase, s = P.sbase;
    for (uint32_t k = 0; k < P.nloops; ++k) {
        const uint32_t q = fdiv(rest, P.loops[k].fd);
        const uint32_t dig = rest - q * P.loops[k].extent;
        d += dig * (uint32_t)P.loops[k].ds;
        s += dig * (uint32_t)P.loops[k].ss;
        rest = q;
    }
    RagUnit u;
    u.doff = d + (P.flat == 1 ? r0 : r0 * P.eP + c0);
    u.soff = s + (P.flat == 1 ? r0 * P.eP + c0 : r0);
    const uint32_t rleft = P.EQ - r0, cleft = P.eP - c0;
    u.rcount = rleft < (1u << P.lqlog) ? rleft : (1u << P.lqlog);
    u.c0 = c0;
    u.ccount = cleft < P.rag_cb ? cleft : P.rag_cb;
    return u;
}

// position c of a row -> element offset on the side where the row is not contiguous: the row's loops
// sit at the end of loops[] (loops[kMaxLoops - 1 - j], j < nq, innermost first)
AMAP_HD uint32_t flat_c_offset(const DevPiece &P, uint32_t c) {
    uint32_t off = 0;
    for (uint32_t j = 0; j < P.nq; ++j) {
        const Loop &l = P.loops[kMaxLoops - 1 - j];
        const uint32_t stride = (uint32_t)(P.flat == 1 ? l.ds : l.ss);
        if (j + 1 == P.nq) {
            off += c * stride;
        } else {
            const uint32_t q = fdiv(c, l.fd);
            off += (c - q * l.extent) * stride;
            c = q;
        }
    }
    return off;
}

// ---- gather rows: position p of a run (see DevPiece::gather) -> source offset relative to the
// offset rows_offsets returns, kept as a cursor that steps to the next position with carries
struct GatherCursor {
    uint32_t dig[4];
    uint32_t off;
};

// NQ = number of loops of the run (P.nq, 1..4), a compile-time constant so that a run of one
// loop steps with a single addition and a run of two with one carry.
template <int NQ>
AMAP_HD GatherCursor gather_begin(const DevPiece &P, uint32_t p) {
    GatherCursor c;
    c.off = 0;
    c.dig[0] = c.dig[1] = c.dig[2] = c.dig[3] = 0;
    for (int j = 0; j < NQ; ++j) {
        const Loop &l = P.loops[kMaxLoops - 1 - j];
        if (j == NQ - 1) {  // the outermost loop of the run never wraps
            c.dig[j] = p;
        } else {
            const uint32_t q = fdiv(p, l.fd);
            c.dig[j] = p - q * l.extent;
            p = q;
        }
        c.off += c.dig[j] * (uint32_t)l.ss;
    }
    return c;
}

template <int NQ>
AMAP_HD void gather_next(const DevPiece &P, GatherCursor &c) {
    bool carry = true;
    for (int j = 0; j < NQ; ++j) {
        if (!carry) continue;
        const Loop &l = P.loops[kMaxLoops - 1 - j];
        c.off += (uint32_t)l.ss;
        if (j == NQ - 1) break;
        carry = ++c.dig[j] == l.extent;
        if (carry) {
            c.dig[j] = 0;
            c.off -= l.extent * (uint32_t)l.ss;
        }
    }
}

// ---- tile kernels
struct TileGeom {
    uint32_t tp, tq;      // tile coordinates along P and Q
    uint32_t db;          // dst element offset of the tile's batch point
    uint32_t sb;          // source element offset of the batch point in the head entry
    uint32_t dig[kMaxLoops];  // batch loop indices of the tile; dig[i] belongs to loop nq + i
    uint32_t TP, TQ;      // tile extents in elements
    uint32_t ncvlog;      // log2(vectors along P per tile row)
    uint32_t lqlog, lplog, nwplog;
    uint32_t swz_bits, swz_shift;
};

AMAP_HD TileGeom tile_geometry(const DevPiece &P, uint32_t vlog, uint32_t t) {
    TileGeom G;
    uint32_t q = fdiv(t, P.fdTP);
    G.tp = t - q * P.tilesP;
    t = q;
    q = fdiv(t, P.fdTQ);
    G.tq = t - q * P.tilesQ;
    t = q;
    G.db = P.dbase;
    G.sb = P.sbase;
    // fixed trip count and constant subscripts: dig[] stays in registers
#pragma unroll
    for (uint32_t i = 0; i < (uint32_t)kMaxLoops; ++i) {
        G.dig[i] = 0;
        const uint32_t k = P.nq + i;
        if (k < P.nloops) {
            q = fdiv(t, P.loops[k].fd);
            G.dig[i] = t - q * P.loops[k].extent;
            G.db += G.dig[i] * (uint32_t)P.loops[k].ds;
            G.sb += G.dig[i] * (uint32_t)P.loops[k].ss;
            t = q;
        }
    }
    G.lqlog = P.lqlog;
    G.lplog = 6 - P.lqlog;
    G.nwplog = P.nwplog;
    G.swz_bits = P.swz_bits;
    G.swz_shift = P.swz_shift;
    G.TP = ((1u << G.nwplog) << G.lplog) << vlog;
    G.TQ = (((1u << P.nwlog) >> G.nwplog) << G.lqlog) << vlog;
    G.ncvlog = G.nwplog + G.lplog;
    return G;
}

// what one lane loads: V vectors along Q at P indices p .. p+V-1, Q position w0
struct TileLane {
    bool valid;
    uint32_t pvl;     // vector index along P inside the tile
    uint32_t r0;      // first row (Q position) inside the tile
    uint32_t p, w0;   // the same in piece coordinates (elements)
    uint32_t sub;     // which entry of the piece group the lane reads from
    const void *src;  // that entry's source (null: constant), P stride and fill pattern
    int32_t ssP;
    uint32_t fill;
    uint32_t soff;    // source element offset of the first vector
};

// P is the head of a piece group ((&P)[0 .. group_n) are its entries).  The
// entries are walked with a wave-uniform index and each lane keeps the fields
// of the entry its P index falls into: indexing the kernel arguments with a
// per-lane index would force the whole argument block into scratch memory.
// `grouped` = false promises group_n == 1 (everything stays in scalar registers).
AMAP_HD TileLane tile_lane(const DevPiece &P, const TileGeom &G, uint32_t vlog, uint32_t tid, bool grouped = true) {
    TileLane L;
    const uint32_t wave = tid >> 6, lane = tid & 63;
    const uint32_t wp = wave & ((1u << G.nwplog) - 1), wq = wave >> G.nwplog;
    const uint32_t lq = lane & ((1u << G.lqlog) - 1), lp = lane >> G.lqlog;
    L.pvl = (wp << G.lplog) + lp;
    L.r0 = ((wq << G.lqlog) + lq) << vlog;
    L.p = G.tp * G.TP + (L.pvl << vlog);
    L.w0 = G.tq * G.TQ + L.r0;
    L.valid = L.p < P.eP && L.w0 < P.EQ;
    L.sub = 0;
    L.src = P.src;
    L.ssP = P.ssP;
    L.fill = P.fill;
    L.soff = G.sb + L.p * (uint32_t)P.ssP + L.w0;
    if (!grouped) return L;
    const uint32_t n = P.group_n;
    for (uint32_t k = 1; k < n; ++k) {
        const DevPiece &S = (&P)[k];
        uint32_t sb = S.sbase;
#pragma unroll
        for (uint32_t i = 0; i < (uint32_t)kMaxLoops; ++i)
            if (P.nq + i < P.nloops) sb += G.dig[i] * (uint32_t)S.loops[P.nq + i].ss;
        if (L.p >= S.p_begin) {  // entries are in increasing p_begin order: the last match wins
            L.sub = k;
            L.src = S.src;
            L.ssP = S.ssP;
            L.fill = S.fill;
            L.soff = sb + (L.p - S.p_begin) * (uint32_t)S.ssP + L.w0;
        }
    }
    return L;
}

// dst offset contributed by position w of the merged Q chain
AMAP_HD uint32_t q_chain_offset(const DevPiece &P, uint32_t w) {
    uint32_t off = 0;
    for (uint32_t k = 0; k + 1 < P.nq; ++k) {
        const uint32_t q = fdiv(w, P.loops[k].fd);
        off += (w - q * P.loops[k].extent) * (uint32_t)P.loops[k].ds;
        w = q;
    }
    return off + w * (uint32_t)P.loops[P.nq - 1].ds;
}

// ---- cross-lane form (PK_XLANE): what one lane loads and stores.
// The V lanes of a unit sit xl_npv lanes apart (same P vector pv, Q positions w0 .. w0 + V - 1): lane k
// of the unit LOADS the V elements along Q at P index pv * V + k and, after the V x V block has been
// transposed across the unit, STORES the V elements along P at Q position w0 + k.
struct XlaneLane {
    bool ok;          // the lane's unit lies inside the piece (all V lanes of a unit agree)
    uint32_t doff;    // dst element offset of the vector the lane stores
    uint32_t k;       // the lane's place in its unit
    uint32_t lane0;   // first lane of the unit; the others follow xl_npv lanes apart
    uint32_t sub;     // entry of the piece group the unit reads (all of a unit's P indices lie in one entry)
    const void *src;  // that entry's source (null: constant) and fill pattern
    uint32_t fill;
    uint32_t soff;    // source element offset of the vector the lane loads
};

AMAP_HD XlaneLane xlane_lane(const DevPiece &P, const TileGeom &G, uint32_t vlog, uint32_t lane, bool grouped = true) {
    XlaneLane L;
    const uint32_t V = 1u << vlog;
    const uint32_t ql = fdiv(lane, P.fd_npv), pv = lane - ql * P.xl_npv;
    const uint32_t a = ql >> vlog;
    L.k = ql & (V - 1);
    L.lane0 = (a << vlog) * P.xl_npv + pv;
    const uint32_t w0 = G.tq * P.xl_rows + (a << vlog), q = w0 + L.k;
    L.ok = ql < P.xl_rows && w0 < P.EQ;
    const uint32_t p = pv << vlog;  // first P index of the unit
    L.doff = G.db + q_chain_offset(P, L.ok ? q : 0) + p;
    L.sub = 0;
    L.src = P.src;
    L.fill = P.fill;
    L.soff = G.sb + (p + L.k) * (uint32_t)P.ssP + w0;
    if (!grouped) return L;
    const uint32_t n = P.group_n;
    for (uint32_t j = 1; j < n; ++j) {
        const DevPiece &S = (&P)[j];
        uint32_t sb = S.sbase;
#pragma unroll
        for (uint32_t i = 0; i < (uint32_t)kMaxLoops; ++i)
            if (P.nq + i < P.nloops) sb += G.dig[i] * (uint32_t)S.loops[P.nq + i].ss;
        if (p >= S.p_begin) {  // entries are in increasing p_begin order: the last match wins
            L.sub = j;
            L.src = S.src;
            L.fill = S.fill;
            L.soff = sb + (p + L.k - S.p_begin) * (uint32_t)S.ssP + w0;
        }
    }
    return L;
}

// LDS slot (in vectors) of the vector at (row, column cv) of the tile.  The tile
// is kept in dst order (one row per Q position, pitch = the tile's P extent),
// so the store phase reads whole rows.  In the load phase the lanes of a
// wavefront that are served together (16 lanes for 16-byte accesses) sit at
// different rows of ONE column, or of a few neighbouring columns: the column
// is XOR-ed with the low bits of the lane's Q coordinate, shifted above the
// column bits that already differ inside such a lane group, so that the group
// covers all 64 banks.
AMAP_HD uint32_t tile_lds_slot(const TileGeom &G, uint32_t vlog, uint32_t row, uint32_t cv) {
    const uint32_t lqv = (row >> vlog) & ((1u << G.lqlog) - 1);
    const uint32_t ncv = 1u << G.ncvlog;
    const uint32_t swz = ((lqv & ((1u << G.swz_bits) - 1)) << G.swz_shift) & (ncv - 1);
    return (row << G.ncvlog) + (cv ^ swz);
}

// store phase of the LDS tile: vector vi of the tile in dst order
struct TileStore {
    bool ok;
    uint32_t slot;
    uint32_t doff;
};

AMAP_HD TileStore tile_store(const DevPiece &P, const TileGeom &G, uint32_t vlog, uint32_t vi) {
    TileStore S;
    const uint32_t row = vi >> G.ncvlog, cv = vi & ((1u << G.ncvlog) - 1);
    const uint32_t w = G.tq * G.TQ + row, pp = G.tp * G.TP + (cv << vlog);
    S.ok = w < P.EQ && pp < P.eP;
    S.slot = tile_lds_slot(G, vlog, row, cv);
    S.doff = S.ok ? G.db + q_chain_offset(P, w) + pp : 0;
    return S;
}

}  // namespace amap_dev
