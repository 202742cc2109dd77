// Host planner: chooses, for every strided piece, the kernel family and the
// tile geometry, and packs the pieces into launches.
//
// Vocabulary (per piece, loops in linearised form):
//   P  = the loop with dst stride 1 (the dst-contiguous direction),
//   Q  = the loop with source stride 1 (the source-contiguous direction),
//        extended to the chain of loops that continue it contiguously in the
//        source, so that a tile can span several short source rows;
//   batch = all other loops.
// P == Q: both sides are contiguous along the same loop -> vector row copy.
// P != Q: the composed map permutes the contiguous dimension -> the tile is
//   read along Q, transposed in registers in V x V blocks, and written along P
//   (through LDS for long dst runs, straight from registers for small P).
#include <algorithm>
#include <climits>
#include <cstdint>
#include <cstdlib>
#include <cstring>

#include "amap_plan.hpp"

#include <cstdio>

using namespace amap_dev;

namespace amap_detail {

static int env_int(const char *name, int def) {
    const char *v = std::getenv(name);
    return v && *v ? std::atoi(v) : def;
}

static uint32_t pow2ceil(uint64_t x) {
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}
static uint32_t ilog2(uint32_t x) {
    uint32_t l = 0;
    while ((1u << l) < x) ++l;
    return l;
}

// largest power of two <= vmax dividing every number in xs
static uint32_t common_pow2(uint32_t vmax, std::initializer_list<int64_t> xs, const std::vector<int64_t> &more) {
    uint32_t v = vmax;
    auto fit = [&](int64_t x) {
        if (x < 0) x = -x;
        while (v > 1 && x % v != 0) v >>= 1;
    };
    for (int64_t x : xs) fit(x);
    for (int64_t x : more) fit(x);
    return v;
}

// true if every number, taken in elements of es bytes, is a multiple of a 128-byte line
static bool line_aligned(int es, std::initializer_list<int64_t> xs, const std::vector<int64_t> &more) {
    for (int64_t x : xs)
        if ((x * es) % 128 != 0) return false;
    for (int64_t x : more)
        if ((x * es) % 128 != 0) return false;
    return true;
}

static uint32_t replicate_fill(uint32_t bits, int es) {
    if (es == 2) return (bits & 0xFFFFu) | (bits << 16);
    return bits;
}

static void fill_rows(DevPiece &dp, const KPiece &kp, uint32_t V, uint32_t nwlog) {
    const int64_t chunk = (int64_t)(64u << nwlog) * kRowsUnroll;
    dp.nwlog = nwlog;
    dp.kind = PK_ROWS;
    dp.vlog = ilog2(V);
    dp.nloops = (uint32_t)kp.dims.size();
    int64_t vol = 1;
    for (size_t k = 0; k < kp.dims.size(); ++k) {
        const KDim &d = kp.dims[kp.dims.size() - 1 - k];  // innermost first
        Loop &l = dp.loops[k];
        l.extent = (uint32_t)d.extent;
        l.ds = (int32_t)d.ds;
        l.ss = (int32_t)d.ss;
        if (k == 0 && V > 1) {
            l.extent = (uint32_t)(d.extent / V);
            l.ds = (int32_t)V;
            l.ss = kp.fill ? 0 : (int32_t)V;
        }
        l.fd = make_fastdiv(l.extent);
        vol *= l.extent;
    }
    dp.n_units = (uint32_t)vol;
    dp.n_blocks = (uint32_t)((vol + chunk - 1) / chunk);
}

// Short rows in a blocked order.  In dst order a workgroup of the row kernel writes one long run of dst
// but fetches every row from another place of the source (one 128-byte line here, one there) when the
// loop that continues a row in dst is not the one that continues it in the source (a head split or
// merge, a permutation of outer dimensions): memory pages are opened for a single line.  The unit index
// is decoded loop by loop with both strides of every loop, so any order and any split of the loops is a
// valid schedule: the low part of the loop that continues the row in the source comes first, then the
// low part of the loop that continues it in dst, each sized so that neighbouring wavefronts cover about
// `run` contiguous bytes on both sides, then the other loops in dst order.
static void block_rows(DevPiece &dp, int es) {
    // Measured with 128-byte rows of 2-byte elements (a head split and a head merge of [b,512,2304]): 75 MB moved
    // 15.2 -> 14.5 us, 600 MB 108.6 -> 99.3 us, 805 MB 131.4 -> 128.8 us; 25 MB 5.5 -> 5.7 us, hence the floor.
    const int64_t run = env_int("AMAP_ROWS_RUN", 1024);  // bytes; 0 keeps the dst order
    const uint32_t floor_units = 1u << std::min(31, std::max(0, env_int("AMAP_ROWS_BLOCK_MIN_LOG2", 21)));  // tests lower it
    if (run <= 0 || dp.n_units < floor_units || dp.nloops < 3 || dp.rep_log || dp.rev || dp.gather || dp.inter) return;
    const int64_t row = (int64_t)dp.loops[0].extent << dp.vlog, row_bytes = row * es;
    if (row_bytes >= run || row_bytes < 64) return;
    int jd = -1, js = -1;
    for (int j = 1; j < (int)dp.nloops; ++j) {
        const Loop &l = dp.loops[j];
        if (l.extent < 2) continue;
        if (l.ds >= row && l.ds <= 2 * row && (jd < 0 || l.ds < dp.loops[jd].ds)) jd = j;
        if (l.ss >= row && l.ss <= 2 * row && (js < 0 || l.ss < dp.loops[js].ss)) js = j;
    }
    if (jd < 0 || js < 0 || jd == js) return;
    const int64_t want = (run + row_bytes - 1) / row_bytes;
    auto low_part = [&](uint32_t ext) {  // a divisor of ext: the smallest that reaches `want` rows, else the largest below
        uint32_t best = 1;
        for (uint32_t d = 1; d <= ext && d <= 4 * want; ++d)
            if (ext % d == 0) {
                if (d >= want) return d;
                best = d;
            }
        return best;
    };
    const uint32_t a = low_part(dp.loops[js].extent), b = low_part(dp.loops[jd].extent);
    if (a < 2 || b < 2) return;
    std::vector<Loop> order;
    auto part = [](const Loop &l, uint32_t ext, int32_t mult) {
        return Loop{ext, l.ds * mult, l.ss * mult, make_fastdiv(ext)};
    };
    order.push_back(dp.loops[0]);
    order.push_back(part(dp.loops[js], a, 1));
    order.push_back(part(dp.loops[jd], b, 1));
    for (int j = 1; j < (int)dp.nloops; ++j) {
        const Loop &l = dp.loops[j];
        const uint32_t lo = j == js ? a : j == jd ? b : 1;
        if ((int64_t)l.ds * lo >= (1ll << 31) || (int64_t)l.ss * lo >= (1ll << 31) || (int64_t)l.ss * lo <= -(1ll << 31)) return;
        if (l.extent / lo > 1) order.push_back(part(l, l.extent / lo, (int32_t)lo));
    }
    if (order.size() > (size_t)kMaxLoops) return;
    for (size_t j = 0; j < (size_t)kMaxLoops; ++j) dp.loops[j] = j < order.size() ? order[j] : Loop{};
    dp.nloops = (uint32_t)order.size();
}

// Streaming (non-temporal) accesses a piece may use.  A loop that stands still in the source
// (repeat, tile, broadcast) reads the same lines again and again: those loads must stay
// cached (a [1,1,1,256] row tiled 100,352 times ran 14.0 us with streaming loads, 11.0 us without).
static uint32_t nt_mask(const KPiece &kp) {
    uint32_t mask = PF_NT_LOAD | PF_NT_STORE;
    if (!kp.fill)
        for (const KDim &d : kp.dims)
            if (d.ss == 0 && d.extent > 1) mask &= ~(uint32_t)PF_NT_LOAD;
    return mask;
}

// Gather rows: the innermost loops of the piece (up to four) continue one another in dst, so
// together they cover one long contiguous run, but the source is not contiguous along it: an
// innermost extent of 3 (channels of an image), a repeat by 3, a source stride of 5.  The run is
// written in aligned 16-byte vectors whose elements are fetched one by one.
static bool plan_gather(const KPiece &kp, int es, uint32_t nwlog, DevPiece &dp) {
    const int n = (int)kp.dims.size();
    if (kp.fill || n == 0 || kp.dims[n - 1].ds != 1) return false;
    int first = n - 1;  // the run's loops are dims[first .. n-1]
    int64_t R = kp.dims[n - 1].extent;
    while (first > 0 && n - first < 4 && kp.dims[first - 1].ds == R) {
        --first;
        R *= kp.dims[first].extent;
    }
    const uint32_t V = 16u / (uint32_t)es;
    std::vector<int64_t> pre_ds;
    for (int k = 0; k < first; ++k) pre_ds.push_back(kp.dims[k].ds);
    if (common_pow2(V, {R, kp.dbase}, pre_ds) != V) return false;
    if (1 + first + (n - first) > kMaxLoops) return false;
    const int64_t chunk = (int64_t)(64u << nwlog) * kRowsUnroll;
    dp.nwlog = nwlog;
    dp.kind = PK_ROWS;
    dp.vlog = ilog2(V);
    dp.gather = 1;
    dp.nq = (uint32_t)(n - first);
    dp.nloops = 1 + (uint32_t)first;
    int64_t vol = R / V;
    dp.loops[0] = Loop{(uint32_t)(R / V), (int32_t)V, 0, make_fastdiv((uint32_t)(R / V))};
    for (int k = 0; k < first; ++k) {
        const KDim &d = kp.dims[first - 1 - k];  // innermost first
        dp.loops[1 + k] = Loop{(uint32_t)d.extent, (int32_t)d.ds, (int32_t)d.ss, make_fastdiv((uint32_t)d.extent)};
        vol *= d.extent;
    }
    for (int j = 0; j < n - first; ++j) {
        const KDim &d = kp.dims[n - 1 - j];
        dp.loops[kMaxLoops - 1 - j] = Loop{(uint32_t)d.extent, (int32_t)d.ds, (int32_t)d.ss, make_fastdiv((uint32_t)d.extent)};
    }
    if (vol >= (1ll << 31)) return false;
    dp.n_units = (uint32_t)vol;
    dp.n_blocks = (uint32_t)((vol + chunk - 1) / chunk);
    if (line_aligned(es, {R, kp.dbase}, pre_ds)) dp.flags |= PF_NT_STORE;
    dp.flags &= nt_mask(kp);
    return true;
}

// Interleave / de-interleave rows: a small number of planes (3 channels of an image, the 2 x 2
// sub-pixels of a pixel shuffle) is the
// innermost dimension on one side and an outer one on the other, and the positions inside a plane
// are contiguous on both sides.  Both sides then move whole 16-byte vectors: E per unit, shuffled
// in registers (see DevPiece::inter).
// One plane of an interleaved source (a slice with step E along the contiguous dimension): the lane
// loads the E vectors that hold V kept elements and stores one.  The window of E * V elements starts
// at the first kept element (inter = 3) unless that would leave the source behind its last kept
// element; then it ends at the last kept element (inter = 4), which must not leave it at the front.
static bool plan_keep_plane(const KPiece &kp, int es, uint32_t nwlog, int64_t svol, DevPiece &dp) {
    const int n = (int)kp.dims.size();
    const int64_t V = 16 / es;
    const KDim &Q = kp.dims[n - 1];
    const int64_t E = Q.ss;
    // Measured on 2-byte elements: step 2 runs 38.5 us against 64.0 us for gathered rows (128 MiB read);
    // steps 3 and 4 are slower than gathered rows (33.4 / 27.9 and 49.1 / 39.4 us), and 4-byte elements gain nothing.
    if (E != 2 || es != 2 || Q.extent % V || kp.dbase % V || n > kMaxLoops) return false;
    int64_t lo = kp.sbase, hi = kp.sbase + (Q.extent - 1) * E;  // offsets of kept elements, relative to the window
    std::vector<int64_t> ds_o, ss_o;
    for (int k = 0; k < n - 1; ++k) {
        const KDim &d = kp.dims[k];
        if (d.ds % V) return false;
        (d.ss < 0 ? lo : hi) += (d.extent - 1) * d.ss;
        ds_o.push_back(d.ds);
        ss_o.push_back(d.ss);
    }
    int64_t shift = 0;
    if (kp.swin + hi + E - 1 >= svol) {
        shift = E - 1;
        if (lo - shift < 0) return false;
    }
    if (lo < 0 || kp.swin + hi - shift + V * E - 1 - (V - 1) * E >= svol) return false;
    if (hi + E >= (1ll << 32)) return false;
    const int64_t chunk = (int64_t)(64u << nwlog) * kRowsUnroll;
    dp.nwlog = nwlog;
    dp.kind = PK_ROWS;
    dp.vlog = ilog2((uint32_t)V);
    dp.inter = shift ? 4u : 3u;
    dp.eP = (uint32_t)E;
    dp.ssP = 0;
    dp.sbase = (uint32_t)(kp.sbase - shift);
    const uint32_t units = (uint32_t)(Q.extent / V);
    dp.loops[0] = Loop{units, (int32_t)V, (int32_t)(V * E), make_fastdiv(units)};
    int64_t vol = units;
    uint32_t nl = 1;
    for (int k = n - 2; k >= 0; --k) {  // innermost first
        const KDim &d = kp.dims[k];
        dp.loops[nl++] = Loop{(uint32_t)d.extent, (int32_t)d.ds, (int32_t)d.ss, make_fastdiv((uint32_t)d.extent)};
        vol *= d.extent;
    }
    dp.nloops = nl;
    if (vol >= (1ll << 31)) return false;
    dp.n_units = (uint32_t)vol;
    dp.n_blocks = (uint32_t)((vol + chunk - 1) / chunk);
    if (line_aligned(es, {Q.extent, kp.dbase}, ds_o)) dp.flags |= PF_NT_STORE;
    if (line_aligned(es, {Q.extent * E, kp.sbase - shift}, ss_o)) dp.flags |= PF_NT_LOAD;
    dp.flags &= nt_mask(kp);
    return true;
}

static bool plan_inter(const KPiece &kp, int es, uint32_t nwlog, int64_t svol, DevPiece &dp) {
    const int n = (int)kp.dims.size();
    if (kp.fill || n < 1 || kp.dims[n - 1].ds != 1) return false;
    if (n < 2) return plan_keep_plane(kp, es, nwlog, svol, dp);
    const int64_t V = 16 / es;
    auto planes_ok = [](int64_t e) { return e >= 2 && e <= 7; };
    int iQ = -1, iP = -1, dir = 0;
    const KDim &last = kp.dims[n - 1];
    if (planes_ok(last.extent) && kp.dims[n - 2].ds == last.extent && kp.dims[n - 2].ss == 1) {
        dir = 1, iP = n - 1, iQ = n - 2;  // dst interleaved
    } else if (planes_ok(last.ss)) {
        for (int k = 0; k < n - 1; ++k)
            if (kp.dims[k].ss == 1 && kp.dims[k].extent == last.ss) iP = k;
        if (iP >= 0) dir = 2, iQ = n - 1;  // dst planar
        if (!dir) return plan_keep_plane(kp, es, nwlog, svol, dp);
    }
    if (!dir) return false;
    // 4-byte elements towards the interleaved side: a vector holds 4 elements only, and the gathered
    // form (contiguous stores, 4 loads per vector) measured faster there (18.2 against 25.2 us)
    if (dir == 1 && es == 4) return false;
    const KDim &P = kp.dims[iP], &Q = kp.dims[iQ];
    const int64_t E = P.extent;
    if (Q.extent % V || kp.dbase % V) return false;
    if (dir == 2 && P.ds % V) return false;
    std::vector<int64_t> ds_o, ss_o;
    for (int k = 0; k < n; ++k)
        if (k != iP && k != iQ) {
            if (kp.dims[k].ds % V) return false;
            ds_o.push_back(kp.dims[k].ds);
            ss_o.push_back(kp.dims[k].ss);
        }
    if ((int)ds_o.size() + 1 > kMaxLoops) return false;
    const int64_t chunk = (int64_t)(64u << nwlog) * kRowsUnroll;
    dp.nwlog = nwlog;
    dp.kind = PK_ROWS;
    dp.vlog = ilog2((uint32_t)V);
    dp.inter = (uint32_t)dir;
    dp.eP = (uint32_t)E;
    dp.ssP = (int32_t)(dir == 1 ? P.ss : P.ds);
    const uint32_t units = (uint32_t)(Q.extent / V);
    dp.loops[0] = Loop{units, (int32_t)(dir == 1 ? V * E : V), (int32_t)(dir == 1 ? V : V * E), make_fastdiv(units)};
    int64_t vol = units;
    uint32_t nl = 1;
    for (int k = n - 1; k >= 0; --k) {  // innermost first
        if (k == iP || k == iQ) continue;
        const KDim &d = kp.dims[k];
        dp.loops[nl++] = Loop{(uint32_t)d.extent, (int32_t)d.ds, (int32_t)d.ss, make_fastdiv((uint32_t)d.extent)};
        vol *= d.extent;
    }
    dp.nloops = nl;
    if (vol >= (1ll << 31)) return false;
    dp.n_units = (uint32_t)vol;
    dp.n_blocks = (uint32_t)((vol + chunk - 1) / chunk);
    if (dir == 1) {
        if (line_aligned(es, {Q.extent * E, kp.dbase}, ds_o)) dp.flags |= PF_NT_STORE;
        if (line_aligned(es, {Q.extent, kp.sbase, P.ss}, ss_o)) dp.flags |= PF_NT_LOAD;
    } else {
        if (line_aligned(es, {Q.extent, kp.dbase, P.ds}, ds_o)) dp.flags |= PF_NT_STORE;
        if (line_aligned(es, {Q.extent * E, kp.sbase}, ss_o)) dp.flags |= PF_NT_LOAD;
    }
    dp.flags &= nt_mask(kp);
    return true;
}

// Flat tiles: a transposing piece whose P x Q matrix is contiguous on one side (rows follow one
// another without a gap) while the extent C along that side's contiguous loop offers no 16-byte
// vectors (49 = 7 x 7 positions of an image in channel-major order).  A workgroup takes 64 rows (32 or 16 where
// 64 do not fit LDS) of the other loop: on the flat side that is ONE contiguous run of rows * C elements, moved in
// whole vectors whatever C is; LDS holds the run, and the other side is served with 16-byte vectors
// along its own contiguous loop, its elements picked from / put into LDS one by one.
//   dir 1: the source is the flat side (P's source stride == Q's extent): r = P, c = Q
//   dir 2: dst is the flat side (Q's dst stride == P's extent): r = Q, c = P
constexpr uint32_t kFlatLdsBytes = 65536;  // rows of 289 (17 x 17): 32.9 us as whole-vector part + tail, 24.8 us as flat tiles of 37 KiB
constexpr uint32_t kFlatMinRows = 16;      // 48 channels of 7 x 7 images: 23.6 -> 12.5 us; 16 channels: 21.4 -> 11.6 us

// The loops that continue the source-contiguous loop iQ in the source (x, then y of an image: one run of
// H * W elements), innermost first, and the length of that run.  A tile vector along Q may straddle the
// loops of the chain (every Q position gets its dst offset through the chain), so only the run's
// length has to be a whole number of vectors.
static std::vector<int> q_chain(const KPiece &kp, int iP, int iQ, int64_t &EQ) {
    const int n = (int)kp.dims.size();
    std::vector<int> chain{iQ};
    EQ = kp.dims[iQ].extent;
    for (bool grown = true; grown && chain.size() < 3;) {
        grown = false;
        for (int k = 0; k < n; ++k) {
            if (k == iP || std::find(chain.begin(), chain.end(), k) != chain.end()) continue;
            if (kp.dims[k].ss == EQ && EQ * kp.dims[k].extent < (1ll << 31)) {
                chain.push_back(k);
                EQ *= kp.dims[k].extent;
                grown = true;
                break;
            }
        }
    }
    return chain;
}

struct FlatShape {
    int dir = 0;             // 0: the piece has no flat form
    int iR = -1;             // the loop that is cut into blocks of rows
    std::vector<int> chain;  // the loops that make up a row of the flat side, innermost first
    int64_t C = 0, ER = 0;
    uint32_t rlog = 6;       // log2(rows per block)
    int64_t cb = 0;          // > 0: column-blocked form with this many columns per block
};

// The row of the flat side may be several loops that continue one another on that side only (the
// y and x loops of a 7 x 7 image that lands inside a padded image, or comes from a crop): on the other
// side every loop of the chain has a stride of its own.
static FlatShape flat_shape(const KPiece &kp, int es) {
    FlatShape none, f;
    if (kp.fill || (es != 2 && es != 4)) return none;
    const int n = (int)kp.dims.size();
    int iP = -1, iQ = -1;
    for (int k = 0; k < n; ++k) {
        if (kp.dims[k].ds == 1) iP = k;
        if (kp.dims[k].ss == 1) iQ = k;
    }
    if (iP < 0 || iQ < 0 || iP == iQ) return none;
    const int64_t V = 16 / es;
    const KDim &P = kp.dims[iP], &Q = kp.dims[iQ];
    // only where the tile forms would move vectors of less than 16 bytes (with 8-byte vectors: 14.4 -> 10.4 us for
    // 196 positions under 1024 channels, 33.0 -> 21.2 us for rows of 100)
    int64_t EQc = Q.extent;
    if (env_int("AMAP_TILE_CHAIN_VEC", 1)) q_chain(kp, iP, iQ, EQc);
    const int64_t tile_bytes = (int64_t)common_pow2((uint32_t)V, {P.extent, EQc}, {}) * es;
    if (tile_bytes >= 16) return none;
    for (int dir = 1; dir <= 2; ++dir) {
        // dir 1: rows are contiguous in the source, from Q outwards, until P's source stride is reached;
        // dir 2: in dst, from P outwards, until Q's dst stride is reached
        const int first = dir == 1 ? iQ : iP, iR = dir == 1 ? iP : iQ;
        auto flat_stride = [&](int k) { return dir == 1 ? kp.dims[k].ss : kp.dims[k].ds; };
        std::vector<int> chain{first};
        int64_t C = kp.dims[first].extent;
        while (flat_stride(iR) != C && chain.size() < 4) {
            int next = -1;
            for (int k = 0; k < n; ++k)
                if (k != iR && std::find(chain.begin(), chain.end(), k) == chain.end() && kp.dims[k].extent > 1 && flat_stride(k) == C) next = k;
            if (next < 0) break;
            chain.push_back(next);
            C *= kp.dims[next].extent;
        }
        if (flat_stride(iR) != C) continue;
        const int64_t ER = kp.dims[iR].extent;
        // rows of 2 .. 7 elements belong to the interleaving row forms (a block of 64 such rows is too little work)
        if (C < 8 || ER < (int64_t)kFlatMinRows) continue;
        if (n - 1 > kMaxLoops) continue;  // batch loops + chain
        // whole 16-byte vectors on the dst side and along the rows?  If not, only the blocked form with dst as
        // the contiguous side remains: its stores take any alignment and its loads along the rows end element by element
        // (a transposition of 4097 x 4099 elements: 74.8 us element by element)
        bool aligned = kp.dbase % V == 0 && ER % V == 0;
        for (int k = 0; k < n; ++k) {
            const bool in_chain = std::find(chain.begin(), chain.end(), k) != chain.end();
            if (k == iP || k == iR) continue;            // dst stride 1; in dir 2 the block loop walks dst in steps of C
            if (dir == 2 && in_chain) continue;          // inside the flat dst run
            if (kp.dims[k].ds % V) aligned = false;      // batch loops on both sides, the chain's dst strides in dir 1
        }
        if (!aligned) {
            if (dir == 1) continue;
            // where dst still offers vectors along P, the tile forms (cut into whole-vector part + tail) keep the piece
            std::vector<int64_t> ds_all;
            for (int k = 0; k < n; ++k)
                if (k != iP) ds_all.push_back(kp.dims[k].ds);
            if (common_pow2((uint32_t)V, {kp.dbase}, ds_all) >= 2) continue;
        }
        // as many rows per block as fit LDS: 64, 32 or 16 (rows of 1225 = 35 x 35 positions: 16 at a time)
        const int64_t lds_limit = (int64_t)kFlatLdsBytes;
        uint32_t rlog = 6;
        // 16 rows at a time only against forms with vectors of less than 8 bytes (rows of 1225: 216.2 -> 27.8 us);
        // against tiles with 8-byte vectors they lose (rows of 1444: 13.2 -> 21.1 us), 32 rows still win (676: 17.6 -> 15.6 us)
        const uint32_t rlog_min = tile_bytes >= 8 ? 5 : 4;
        while (rlog > rlog_min && C * std::min<int64_t>(ER, 1ll << rlog) * es > lds_limit) --rlog;
        int64_t cb = 0;
        // 128 2-byte columns per block (55 x 55 positions under 96 channels, towards channel-major: 24.4 us; 256 columns: 26.6 us;
        // gathered rows: 178.8 us).  With the source as the contiguous side and a row of one loop, the cut into a
        // whole-vector part and a one-element tail is as fast or faster (23.7 against 23.8 us; 75 x 75 fp32: 11.9 against
        // 17.4 us), so there the blocked form is left to rows of several loops (padded or cropped images).
        const int64_t cb_env = 256 / es;  // 256-byte row segments (fp32: 64 columns 15.5 us, 128 columns 17.2 us)
        const bool rag_ok = cb_env >= V && cb_env % V == 0 && tile_bytes < 8 && ER >= 64;
        // long rows of one loop under few channels, the source contiguous: the cut into a whole-vector part and a
        // one-element tail is faster there (concat of 64 + 64 + 96 + 32 channels of 35 x 35 positions: 26.8 against 34.6 us)
        if (dir == 1 && chain.size() == 1 && rlog == 4 && ER < 128) continue;
        const bool fits = aligned && C * std::min<int64_t>(ER, 1ll << rlog) * es <= lds_limit;
        if (!fits) {
            // rows too long for LDS: blocks of 64 rows x cb columns whose row segments start at any element
            if (!rag_ok || !(dir == 2 || chain.size() > 1)) continue;
            rlog = 6;
            cb = cb_env;
        } else if (rag_ok && rlog == 4 && dir == 1) {
            // 16 rows at a time with the source as the contiguous side: the blocked form is faster
            // (35 x 35 positions under 288 channels: 26.3 against 30.7 us; into a padded image 29.1 against 32.1 us)
            rlog = 6;
            cb = cb_env;
        }
        f.dir = dir, f.iR = iR, f.chain = chain, f.C = C, f.ER = ER, f.rlog = rlog, f.cb = cb;
        return f;
    }
    return none;
}

static bool plan_flat(const KPiece &kp, int es, uint32_t nwlog, DevPiece &dp, uint32_t &lds) {
    const FlatShape f = flat_shape(kp, es);
    if (!f.dir) return false;
    const int n = (int)kp.dims.size();
    const int64_t V = 16 / es;
    dp.kind = PK_FLAT;
    dp.nwlog = nwlog;
    dp.vlog = ilog2((uint32_t)V);
    dp.inter = 0;
    dp.flat = (uint32_t)f.dir;
    dp.eP = (uint32_t)f.C;
    dp.EQ = (uint32_t)f.ER;
    const int64_t rows = 1ll << f.rlog;
    dp.lqlog = f.rlog;
    dp.tilesP = (uint32_t)((f.ER + rows - 1) / rows);
    dp.fdTP = make_fastdiv(dp.tilesP);
    int64_t nb = dp.tilesP;
    uint32_t nl = 0;
    std::vector<int64_t> ds_o, ss_o, chain_other;
    for (int k = n - 1; k >= 0; --k) {  // batch loops, innermost first
        if (k == f.iR || std::find(f.chain.begin(), f.chain.end(), k) != f.chain.end()) continue;
        const KDim &d = kp.dims[k];
        dp.loops[nl++] = Loop{(uint32_t)d.extent, (int32_t)d.ds, (int32_t)d.ss, make_fastdiv((uint32_t)d.extent)};
        nb *= d.extent;
        ds_o.push_back(d.ds);
        ss_o.push_back(d.ss);
    }
    dp.nloops = nl;
    dp.nq = (uint32_t)f.chain.size();
    if (nl + dp.nq > (uint32_t)kMaxLoops) return false;
    for (size_t j = 0; j < f.chain.size(); ++j) {  // the row's loops at the end of loops[], innermost first
        const KDim &d = kp.dims[f.chain[j]];
        dp.loops[kMaxLoops - 1 - j] = Loop{(uint32_t)d.extent, (int32_t)d.ds, (int32_t)d.ss, make_fastdiv((uint32_t)d.extent)};
        chain_other.push_back(f.dir == 1 ? d.ds : d.ss);
    }
    if (nb >= (1ll << 31)) return false;
    dp.n_blocks = (uint32_t)nb;
    dp.n_units = dp.n_blocks;
    lds = (uint32_t)(f.C * std::min<int64_t>(f.ER, rows) * es);
    if (f.cb) {
        dp.rag_cb = (uint32_t)f.cb;
        dp.rag_w = (uint32_t)(f.cb + (es == 2 ? 2 : 1));  // LDS row stride: an odd number of dwords
        dp.rag_s = (uint32_t)(f.cb / V + 1);
        dp.fd_rag_s = make_fastdiv(dp.rag_s);
        dp.tilesQ = (uint32_t)((f.C + f.cb - 1) / f.cb);
        dp.fdTQ = make_fastdiv(dp.tilesQ);
        nb *= dp.tilesQ;
        if (nb >= (1ll << 31)) return false;
        dp.n_blocks = (uint32_t)nb;
        dp.n_units = dp.n_blocks;
        lds = (uint32_t)(rows * dp.rag_w * es);
        dp.flags = 0;
        return true;
    }
    // streaming accesses where every block covers whole lines on that side
    if (f.ER % rows == 0) {
        const bool flat_dst = line_aligned(es, {kp.dbase, rows * f.C}, ds_o), flat_src = line_aligned(es, {kp.sbase, rows * f.C}, ss_o);
        const bool rows_ok = line_aligned(es, {rows}, chain_other);
        const bool rows_dst = rows_ok && line_aligned(es, {kp.dbase}, ds_o), rows_src = rows_ok && line_aligned(es, {kp.sbase}, ss_o);
        if (f.dir == 1 ? rows_dst : flat_dst) dp.flags |= PF_NT_STORE;
        if (f.dir == 1 ? flat_src : rows_src) dp.flags |= PF_NT_LOAD;
    }
    dp.flags &= nt_mask(kp);
    return true;
}

// returns the family used (amap_kernel_id) or -1 if the forced family cannot run the piece
static int plan_piece(const amap &m, const KPiece &kp, int family, uint32_t nwlog, DevPiece &dp, uint32_t &lds,
                      int &vec_bytes, std::vector<int> *slot_dim = nullptr) {
    const int es = m.elem;
    const uint32_t vmax = (uint32_t)std::min(16, std::max(es, env_int("AMAP_VEC_BYTES", 16))) / es;
    std::memset(&dp, 0, sizeof(dp));
    dp.src = kp.fill ? nullptr : reinterpret_cast<const void *>((uintptr_t)(kp.src + 1));
    dp.fill = replicate_fill(kp.fill_bits, es);
    dp.dbase = (uint32_t)kp.dbase;
    dp.sbase = (uint32_t)kp.sbase;
    dp.dwin = (uint64_t)kp.dwin;
    dp.swin = (uint64_t)kp.swin;
    dp.group_n = 1;
    lds = 0;
    const int n = (int)kp.dims.size();
    int iP = -1, iQ = -1;
    for (int k = 0; k < n; ++k) {
        if (kp.dims[k].ds == 1) iP = k;
        if (!kp.fill && kp.dims[k].ss == 1) iQ = k;
    }
    std::vector<int64_t> ds_others, ss_others;
    for (int k = 0; k < n; ++k) {
        if (k != iP) ds_others.push_back(kp.dims[k].ds);
        if (k != iQ && !kp.fill) ss_others.push_back(kp.dims[k].ss);
    }
    // A repeat along the contiguous dimension: the innermost loop (dst stride 1)
    // does not move in the source and the loop around it walks the source
    // contiguously, so a dst row is the source row with every element written r
    // times.  For r a power of two that fits a 16-byte vector the row kernel
    // handles both loops as one loop over dst vectors.
    if (family < 0 || family == AMAP_K_ROWS) {
        const int inner = n - 1;
        if (!kp.fill && n >= 2 && kp.dims[inner].ds == 1 && kp.dims[inner].ss == 0 && kp.dims[inner - 1].ss == 1 &&
            kp.dims[inner - 1].ds == kp.dims[inner].extent) {
            const int64_t r = kp.dims[inner].extent, cnt = kp.dims[inner - 1].extent;
            // the expanding row form always writes 16-byte dst vectors: not available under a narrower cap
            const uint32_t V = 16u / (uint32_t)es;
            const bool pow2 = (r & (r - 1)) == 0 && vmax == V;
            std::vector<int64_t> dso, sso;
            for (int k = 0; k < n - 2; ++k) {
                dso.push_back(kp.dims[k].ds);
                sso.push_back(kp.dims[k].ss);
            }
            if (pow2 && r >= 2 && r <= (int64_t)V && common_pow2(V, {cnt * r, kp.dbase}, dso) == V &&
                common_pow2(V, {cnt * r}, {}) == V && (int64_t)common_pow2(V, {kp.sbase * r, cnt * r}, {}) == V) {
                const int64_t sv = V / r;  // source elements per dst vector
                bool ok = kp.sbase % sv == 0 && cnt % sv == 0;
                for (int64_t x : sso) ok = ok && x % sv == 0;
                if (ok) {
                    KPiece merged = kp;
                    merged.dims.pop_back();
                    merged.dims.back() = KDim{cnt * r, 1, 1};
                    fill_rows(dp, merged, V, nwlog);
                    dp.loops[0].ss = (int32_t)sv;
                    dp.rep_log = ilog2((uint32_t)r);
                    vec_bytes = (int)(sv * es);
                    if (line_aligned(es, {cnt * r, kp.dbase}, dso)) dp.flags |= PF_NT_STORE;
                    if (line_aligned(es, {cnt, kp.sbase}, sso)) dp.flags |= PF_NT_LOAD;
                    dp.flags &= nt_mask(kp);
                    return AMAP_K_ROWS;
                }
            }
        }
    }
    // A reversed contiguous axis: the dst-contiguous loop walks the source backwards one element
    // at a time.  With whole 16-byte dst vectors the row kernel loads the mirrored vector and
    // reverses it in registers.
    if ((family < 0 || family == AMAP_K_ROWS) && !kp.fill && n >= 1 && kp.dims[n - 1].ds == 1 && kp.dims[n - 1].ss == -1) {
        std::vector<int64_t> dso;
        for (int k = 0; k < n - 1; ++k) dso.push_back(kp.dims[k].ds);
        // the reversing row form always moves 16-byte vectors: not available under a narrower cap
        const uint32_t V16 = 16u / (uint32_t)es;
        if (vmax == V16 && common_pow2(V16, {kp.dims[n - 1].extent, kp.dbase}, dso) == V16) {
            fill_rows(dp, kp, V16, nwlog);
            dp.loops[0].ss = -(int32_t)V16;
            dp.rev = 1;
            vec_bytes = 16;
            if (line_aligned(es, {kp.dims[n - 1].extent, kp.dbase}, dso)) dp.flags |= PF_NT_STORE;
            dp.flags &= nt_mask(kp);
            return AMAP_K_ROWS;
        }
    }
    const bool rows_ok = iP >= 0 && (kp.fill || iP == iQ);
    const bool tile_shape = !kp.fill && iP >= 0 && iQ >= 0 && iP != iQ;
    // The vector width follows from the dst side (aligned 16-byte stores) and from
    // the extents; source runs may start at any element (under-aligned loads).
    uint32_t Vt = 1;
    if (tile_shape) {
        int64_t EQc = 0;
        q_chain(kp, iP, iQ, EQc);
        Vt = common_pow2(vmax, {kp.dims[iP].extent, env_int("AMAP_TILE_CHAIN_VEC", 1) ? EQc : kp.dims[iQ].extent, kp.dbase}, ds_others);
    }
    const bool tile_ok = tile_shape && Vt * es >= 4;

    int fam = family;
    if (fam < 0) {
        if (rows_ok)
            fam = AMAP_K_ROWS;
        else if (tile_ok)
            fam = (int64_t)kp.dims[iP].extent * es <= 64 ? AMAP_K_WAVE : AMAP_K_TILE;
        else
            fam = AMAP_K_ELEMENT;
    }
    if (kp.fill && (fam == AMAP_K_TILE || fam == AMAP_K_WAVE)) fam = AMAP_K_ROWS;  // constants need no transpose
    // Where the planned family would move 2- or 4-byte vectors only (or single elements), gathered
    // 16-byte dst vectors are the better row form; a forced row family may use them as well.
    if (!kp.fill && env_int("AMAP_GATHER", 1) && vmax * (uint32_t)es == 16) {  // both forms move 16-byte vectors only
        int64_t narrow = es;
        if (fam == AMAP_K_ROWS && rows_ok) narrow = (int64_t)common_pow2(vmax, {kp.dims[iP].extent, kp.dbase}, ds_others) * es;
        if ((fam == AMAP_K_TILE || fam == AMAP_K_WAVE) && tile_ok) narrow = (int64_t)Vt * es;
        const bool planned_narrow = family < 0 && narrow < 8;
        const bool forced_rows = family == AMAP_K_ROWS && (!rows_ok || narrow < 8);
        const int64_t svol = kp.src >= 0 && (size_t)kp.src < m.src_shapes.size() ? volume_of(m.src_shapes[(size_t)kp.src]) : 0;
        if ((planned_narrow || forced_rows) && env_int("AMAP_INTER", 1) && plan_inter(kp, es, nwlog, svol, dp)) {
            vec_bytes = 16;
            return AMAP_K_ROWS;
        }
        dp.inter = 0;
        dp.flags = 0;
        dp.sbase = (uint32_t)kp.sbase;
        const bool forced_tile = family == AMAP_K_TILE && (!tile_ok || narrow < 8);
        const bool planned_flat = family < 0 && narrow < 16;
        // (slot_dim: the caller plans a group of pieces as one tile piece and needs the tile geometry proper)
        if ((planned_flat || forced_tile) && !slot_dim && env_int("AMAP_FLAT", 1) && plan_flat(kp, es, nwlog, dp, lds)) {
            vec_bytes = 16;
            return AMAP_K_TILE;
        }
        dp.flat = 0;
        dp.rag_cb = 0;
        dp.nq = 0;
        dp.flags = 0;
        lds = 0;
        if ((planned_narrow || forced_rows) && plan_gather(kp, es, nwlog, dp)) {
            vec_bytes = 16;
            return AMAP_K_ROWS;
        }
        // the attempts may have touched dp before giving up
        dp.gather = 0;
        dp.nq = 0;
        dp.flags = 0;
    }

    if (fam == AMAP_K_ELEMENT) {
        fill_rows(dp, kp, 1, nwlog);
        vec_bytes = es;
        return fam;
    }
    if (fam == AMAP_K_ROWS) {
        if (!rows_ok) return -1;
        uint32_t V = common_pow2(vmax, {kp.dims[iP].extent, kp.dbase}, ds_others);
        fill_rows(dp, kp, V, nwlog);
        if (!kp.fill && V * (uint32_t)es == 16) block_rows(dp, es);
        vec_bytes = (int)V * es;
        // streaming accesses where the piece touches only whole lines
        if (line_aligned(es, {kp.dims[iP].extent, kp.dbase}, ds_others)) dp.flags |= PF_NT_STORE;
        // a fill piece loads nothing, so it never vetoes streaming loads for its launch
        if (kp.fill || line_aligned(es, {kp.dims[iP].extent, kp.sbase}, ss_others)) dp.flags |= PF_NT_LOAD;
        dp.flags &= nt_mask(kp);
        return fam;
    }
    if (fam != AMAP_K_TILE && fam != AMAP_K_WAVE) return -1;
    if (!tile_ok) return -1;

    // ---- tile geometry
    const uint32_t V = Vt;
    dp.kind = fam == AMAP_K_TILE ? PK_TILE : PK_WAVE;
    dp.vlog = ilog2(V);
    dp.eP = (uint32_t)kp.dims[iP].extent;
    dp.ssP = (int32_t)kp.dims[iP].ss;
    int64_t EQ = 0;
    const std::vector<int> chain = q_chain(kp, iP, iQ, EQ);
    dp.EQ = (uint32_t)EQ;
    dp.nq = (uint32_t)chain.size();
    uint32_t nl = 0;
    if (slot_dim) slot_dim->clear();
    for (int k : chain) {
        if (slot_dim) slot_dim->push_back(k);
        Loop &l = dp.loops[nl++];
        l.extent = (uint32_t)kp.dims[k].extent;
        l.ds = (int32_t)kp.dims[k].ds;
        l.ss = (int32_t)kp.dims[k].ss;
        l.fd = make_fastdiv(l.extent);
    }
    int64_t batch = 1;
    for (int k = n - 1; k >= 0; --k) {
        if (k == iP || std::find(chain.begin(), chain.end(), k) != chain.end()) continue;
        if (slot_dim) slot_dim->push_back(k);
        Loop &l = dp.loops[nl++];
        l.extent = (uint32_t)kp.dims[k].extent;
        l.ds = (int32_t)kp.dims[k].ds;
        l.ss = (int32_t)kp.dims[k].ss;
        l.fd = make_fastdiv(l.extent);
        batch *= l.extent;
    }
    dp.nloops = nl;
    const uint64_t pv = dp.eP / V, qv = (uint64_t)EQ / V;  // vectors along P / Q
    uint32_t LP = std::min<uint32_t>(64, pow2ceil(pv)), LQ = std::min<uint32_t>(64, pow2ceil(qv));
    while (LP * LQ > 64) {
        if (LP > LQ)
            LP >>= 1;
        else
            LQ >>= 1;
    }
    if (LP * LQ < 64) LQ = 64 / LP;
    const uint64_t remP = (pv + LP - 1) / LP, remQ = (qv + LQ - 1) / LQ;
    const uint32_t NW = 1u << nwlog;
    uint32_t NWP;
    if (NW >= 4 && remP >= 4 && remP % 4 == 0)
        NWP = 4;  // the wavefronts of a workgroup side by side along P: longest dst runs (measured +2 %)
    else if (NW >= 4 && remP >= 2 && remQ >= 2)
        NWP = 2;
    else if (remQ < 2)
        NWP = std::min<uint32_t>(NW, pow2ceil(remP));
    else
        NWP = 1;
    // dst rows that are not a whole number of 128-byte lines: a tile boundary
    // inside the row would leave partial lines to two workgroups, so let one
    // tile span the whole row if the workgroup is large enough
    if ((dp.eP * (uint64_t)es) % 128 != 0) NWP = std::min<uint32_t>(NW, pow2ceil(remP));
    dp.lqlog = ilog2(LQ);
    dp.nwplog = ilog2(NWP);
    dp.nwlog = nwlog;
    {
        // lanes served together by one LDS access of V * es bytes: 256 bytes' worth
        const uint32_t group_log = 8 - ilog2((uint32_t)(V * es));
        const uint32_t ncvlog = ilog2(NWP * LP);
        dp.swz_bits = std::min(group_log, dp.lqlog);
        const uint32_t span = std::min(group_log, ncvlog);
        dp.swz_shift = span > dp.swz_bits ? span - dp.swz_bits : 0;
    }
    const uint32_t TP = NWP * LP * V, TQ = (NW / NWP) * LQ * V;
    dp.tilesP = (dp.eP + TP - 1) / TP;
    dp.tilesQ = (uint32_t)((EQ + TQ - 1) / TQ);
    dp.fdTP = make_fastdiv(dp.tilesP);
    dp.fdTQ = make_fastdiv(dp.tilesQ);
    int64_t nb = (int64_t)dp.tilesP * dp.tilesQ * batch;
    if (nb >= (1ll << 31)) return -1;
    dp.n_blocks = (uint32_t)nb;
    if (dp.kind == PK_TILE) lds = TP * TQ * es;
    {
        std::vector<int64_t> batch_ds, batch_ss;
        for (uint32_t k = dp.nq; k < dp.nloops; ++k) {
            batch_ds.push_back(dp.loops[k].ds);
            batch_ss.push_back(dp.loops[k].ss);
        }
        for (uint32_t k = 0; k < dp.nq; ++k) batch_ds.push_back(dp.loops[k].ds);
        if (line_aligned(es, {dp.eP, (int64_t)LP * V, kp.dbase}, batch_ds)) dp.flags |= PF_NT_STORE;
        if (line_aligned(es, {EQ, (int64_t)LQ * V, kp.sbase, dp.ssP}, batch_ss)) dp.flags |= PF_NT_LOAD;
        dp.flags &= nt_mask(kp);
    }
    vec_bytes = (int)V * es;
    // ---- short P runs: the cross-lane form.  A dst row (fills beside it included, when this is the head of
    // a piece group) of at most 128 bytes; one 16-byte vector per lane each way, stores of a wavefront contiguous.
    {
        const uint32_t npv = dp.eP / V;
        const uint32_t R = npv ? ((64u / npv) / V) * V : 0;
        // Measured at 1 GiB per launch: ahead of the register micro-transpose only where a wavefront still covers
        // 64 bytes or more of every source row it touches, i.e. for 2-byte elements in dst rows of one or two
        // vectors (5.0 against 4.1 and 4.8 TB/s); behind it for longer rows and for 4-byte elements
        // (3.5 against 5.7 TB/s on 80-byte rows).  AMAP_XLANE=2 plans it wherever it applies, 0 nowhere.
        const int xl = env_int("AMAP_XLANE", 1);
        const bool xl_pays = xl >= 2 || (es == 2 && npv <= 2);
        if (xl && xl_pays && V * (uint32_t)es == 16 && dp.eP % V == 0 && (uint64_t)dp.eP * es <= 128 && npv >= 1 && npv <= 8 &&
            R >= V && EQ % V == 0) {
            dp.kind = PK_XLANE;
            dp.xl_npv = npv;
            dp.xl_rows = R;
            dp.fd_npv = make_fastdiv(npv);
            dp.tilesP = 1;
            dp.fdTP = make_fastdiv(1);
            dp.tilesQ = (uint32_t)((EQ + R - 1) / R);
            dp.fdTQ = make_fastdiv(dp.tilesQ);
            const int64_t tiles = (int64_t)dp.tilesQ * batch;
            if (tiles >= (1ll << 31)) return -1;
            dp.n_units = (uint32_t)tiles;
            dp.n_blocks = (uint32_t)((tiles + NW - 1) / NW);
            dp.lqlog = dp.nwplog = dp.swz_bits = dp.swz_shift = 0;
            lds = 0;
            // streaming stores where every wavefront's run of dst is whole lines; the loads of a wavefront are
            // short pieces of many source rows and stay cached
            std::vector<int64_t> ds_all;
            for (uint32_t k = 0; k < dp.nloops; ++k) ds_all.push_back(k == 0 ? (int64_t)dp.loops[0].ds * R : (int64_t)dp.loops[k].ds);
            dp.flags = line_aligned(es, {(int64_t)dp.eP * R, kp.dbase}, ds_all) && dp.loops[0].ds == (int32_t)dp.eP ? PF_NT_STORE : 0;
            dp.flags &= nt_mask(kp);
        }
    }
    return fam;
}

// ---------------------------------------------------------------- piece groups
//
// Pieces that tile the dst-contiguous dimension P between them (concat on the
// innermost dst dimension, padding of it) are planned as ONE tile piece whose
// P extent is the sum: tiles then follow the 128-byte lines of dst instead of
// the piece boundaries, and no workgroup writes a fraction of a line that some
// other workgroup completes much later (measured: 3.3 vs 5.4 TB/s).

namespace {

struct Member {
    const KPiece *kp;
    std::vector<KDim> dims;  // loops in the order of the group's first copy piece
    int64_t p_extent;
};

int p_loop(const std::vector<KDim> &dims) {
    for (size_t k = 0; k < dims.size(); ++k)
        if (dims[k].ds == 1) return (int)k;
    return -1;
}

// Can piece x continue anchor a along P, starting at dst offset `at`?  On
// success returns x's loops in a's loop order.
bool continues(const KPiece &a, int iP, const KPiece &x, int64_t at, Member &out) {
    if (x.dbase != at) return false;
    out.kp = &x;
    if (!x.fill) {
        if (x.dims.size() != a.dims.size() || p_loop(x.dims) != iP) return false;
        for (size_t k = 0; k < a.dims.size(); ++k) {
            if ((int)k == iP) continue;
            if (x.dims[k].extent != a.dims[k].extent || x.dims[k].ds != a.dims[k].ds) return false;
        }
        out.dims = x.dims;
        out.p_extent = x.dims[iP].extent;
        return true;
    }
    // a fill piece merges more loops than a copy piece: rebuild it in a's loop
    // structure and check that this is the same box
    int64_t vol_rest = 1;
    for (size_t k = 0; k < a.dims.size(); ++k)
        if ((int)k != iP) vol_rest *= a.dims[k].extent;
    if (x.volume() % vol_rest != 0) return false;
    const int64_t pe = x.volume() / vol_rest;
    if (pe < 1) return false;
    std::vector<KDim> cand = a.dims;
    for (auto &d : cand) d.ss = 0;
    cand[iP].extent = pe;
    std::vector<KDim> nontrivial;
    for (const auto &d : cand)
        if (d.extent > 1) nontrivial.push_back(d);
    const std::vector<KDim> merged = merge_loops(nontrivial);
    if (merged.size() != x.dims.size()) return false;
    for (size_t k = 0; k < merged.size(); ++k)
        if (merged[k].extent != x.dims[k].extent || merged[k].ds != x.dims[k].ds) return false;
    out.dims = cand;
    out.p_extent = pe;
    return true;
}

// Greedy grouping: every copy piece with a P loop anchors a group and absorbs
// the pieces that follow / precede it along P.
std::vector<std::vector<Member>> find_groups(const amap &m, std::vector<char> &grouped) {
    std::vector<std::vector<Member>> groups;
    const auto &ks = m.kpieces;
    grouped.assign(ks.size(), 0);
    for (size_t a = 0; a < ks.size(); ++a) {
        if (grouped[a] || ks[a].fill) continue;
        const int iP = p_loop(ks[a].dims);
        if (iP < 0) continue;
        std::vector<Member> g;
        g.push_back(Member{&ks[a], ks[a].dims, ks[a].dims[iP].extent});
        std::vector<size_t> idx{a};
        int64_t lo = ks[a].dbase, hi = ks[a].dbase + ks[a].dims[iP].extent;
        // the run of P must stay inside one dst row of the anchor's loop structure:
        // the next larger dst stride bounds it
        int64_t row = INT64_MAX;
        for (size_t k = 0; k < ks[a].dims.size(); ++k)
            if ((int)k != iP) row = std::min(row, ks[a].dims[k].ds);
        for (bool grown = true; grown;) {
            grown = false;
            for (size_t x = 0; x < ks.size(); ++x) {
                if (grouped[x] || std::find(idx.begin(), idx.end(), x) != idx.end()) continue;
                Member mem;
                if (continues(ks[a], iP, ks[x], hi, mem) && hi - lo + mem.p_extent <= row) {
                    g.push_back(mem);
                    idx.push_back(x);
                    hi += mem.p_extent;
                    grown = true;
                } else if (ks[x].fill && continues(ks[a], iP, ks[x], ks[x].dbase, mem) &&
                           ks[x].dbase + mem.p_extent == lo && hi - lo + mem.p_extent <= row) {
                    g.insert(g.begin(), mem);
                    idx.push_back(x);
                    lo -= mem.p_extent;
                    grown = true;
                }
            }
        }
        if (g.size() >= 2 && g.size() <= (size_t)kMaxPiecesPerLaunch) {
            for (size_t x : idx) grouped[x] = 1;
            groups.push_back(std::move(g));
        }
    }
    return groups;
}

}  // namespace

// Plan a group as one tile piece: out[0] is the head (geometry, total P
// extent), out[i] the entry of member i.  False if the members do not share
// one vector width / source chain, in which case they are planned one by one.
static bool plan_group(const amap &m, const std::vector<Member> &g, int family, uint32_t nwlog,
                       std::vector<DevPiece> &out, uint32_t &lds, int &vec_bytes) {
    const int es = m.elem;
    const Member *first_copy = nullptr;
    for (const Member &mem : g)
        if (!mem.kp->fill && !first_copy) first_copy = &mem;
    if (!first_copy) return false;
    const int iP = p_loop(first_copy->dims);
    int64_t total = 0;
    for (const Member &mem : g) total += mem.p_extent;
    // synthetic piece: the first copy member's loops with the whole P run
    KPiece H = *first_copy->kp;
    H.dims = first_copy->dims;
    H.dims[iP].extent = total;
    H.dbase = g[0].kp->dbase;
    DevPiece head;
    std::vector<int> slot_dim;
    int fam = family < 0 ? AMAP_K_TILE : family;
    if (fam != AMAP_K_TILE && fam != AMAP_K_WAVE) return false;
    if (plan_piece(m, H, fam, nwlog, head, lds, vec_bytes, &slot_dim) != fam) return false;
    const int64_t V = 1ll << head.vlog;
    bool nt_load = true;
    int64_t at = 0;
    out.clear();
    for (const Member &mem : g) {
        DevPiece s = head;
        const KPiece &kp = *mem.kp;
        if (at % V != 0 || mem.p_extent % V != 0) return false;
        s.p_begin = (uint32_t)at;
        s.n_blocks = 0;
        s.group_n = 1;
        s.fill = replicate_fill(kp.fill_bits, es);
        if (kp.fill) {
            s.src = nullptr;
            s.sbase = 0;
            s.ssP = 0;
            for (uint32_t k = 0; k < s.nloops; ++k) s.loops[k].ss = 0;
        } else {
            s.src = reinterpret_cast<const void *>((uintptr_t)(kp.src + 1));
            s.sbase = (uint32_t)kp.sbase;
            s.swin = (uint64_t)kp.swin;
            s.ssP = (int32_t)mem.dims[iP].ss;
            std::vector<int64_t> bss;
            for (uint32_t k = 0; k < s.nloops; ++k) {
                const int64_t ss = mem.dims[slot_dim[k]].ss;
                // the Q chain must be the same contiguous chain in every source
                if (k < s.nq && ss != head.loops[k].ss) return false;
                s.loops[k].ss = (int32_t)ss;
                if (k >= s.nq) bss.push_back(ss);
            }
            nt_load = nt_load && line_aligned(es, {kp.sbase, mem.dims[iP].ss}, bss);
        }
        out.push_back(s);
        at += mem.p_extent;
    }
    // the head entry is member 0 with the group's geometry
    out[0].n_blocks = head.n_blocks;
    out[0].group_n = (uint32_t)g.size();
    uint32_t flags = head.flags & PF_NT_STORE;
    if ((head.flags & PF_NT_LOAD) && nt_load) flags |= PF_NT_LOAD;
    for (DevPiece &s : out) s.flags = flags;
    return true;
}

static bool plan_strided_nw(const amap &m, int family, int nw_forced, Plan &out, bool &split_rows) {
    split_rows = false;
    out.launches.clear();
    out.grid.clear();
    out.lds_bytes.clear();
    out.strided_ok = false;
    out.fits32 = volume_of(m.shape) < (1ll << 31);
    for (const auto &s : m.src_shapes)
        if (!s.empty() && volume_of(s) >= (1ll << 31)) out.fits32 = false;
    if (!m.strided) return false;
    // workgroup size: single wavefronts balance small problems over the
    // 256 compute units and keep the tail short; large problems amortise
    // dispatch with 4 wavefronts per workgroup
    uint32_t nwlog = volume_of(m.shape) * m.elem < env_int("AMAP_SMALL_BYTES_MB", 256) * (1ll << 20) ? 0 : 2;
    if (nw_forced >= 0) nwlog = (uint32_t)nw_forced;
    int64_t best_vol = -1;
    out.min_vec_bytes = 16;
    LaunchArgs cur;
    std::memset(&cur, 0, sizeof(cur));
    cur.nwlog = nwlog;
    uint32_t blocks = 0, lds_max = 0;
    auto flush = [&]() {
        if (cur.n_pieces == 0) return;
        // XCD-aware order only where it pays: tile pieces whose source segments
        // are not line-aligned share lines between neighbouring tiles, and those
        // neighbours should meet in one L2 (measured +6..11 %); for aligned
        // streaming pieces the plain round-robin order is faster
        uint32_t xr = 0;
        for (uint32_t k = 0; k < cur.n_pieces; ++k)
            if (cur.p[k].kind != PK_ROWS && cur.p[k].src && !(cur.p[k].flags & PF_NT_LOAD)) xr = 1;
        cur.xcd_remap = xr;
        out.launches.push_back(cur);
        out.grid.push_back(blocks);
        out.lds_bytes.push_back(lds_max);
        std::memset(&cur, 0, sizeof(cur));
        cur.nwlog = nwlog;
        blocks = 0;
        lds_max = 0;
    };
    const bool trace = env_int("AMAP_PLAN_TRACE", 0) != 0;  // one line per planned piece on stderr
    if (trace) std::fprintf(stderr, "amap plan: begin (%zu pieces, family %d)\n", m.kpieces.size(), family);
    auto emit = [&](const std::vector<DevPiece> &dps, uint32_t lds, int vb, int fam, int64_t vol) {
        if (trace)
            for (const DevPiece &d : dps) {
                const char *form = d.kind == PK_TILE ? "tile" : d.kind == PK_WAVE ? "wave" : d.kind == PK_XLANE ? "xlane" : "rows";
                if (d.kind == PK_FLAT && d.rag_cb) form = d.flat == 1 ? "flat-blocked-src" : "flat-blocked-dst";
                if (d.kind == PK_FLAT && !d.rag_cb) form = d.flat == 1 ? "flat-src" : "flat-dst";
                if (d.kind == PK_ROWS) {
                    if (!d.src) form = "rows-fill";
                    if (d.rep_log) form = "rows-expand";
                    if (d.rev) form = "rows-reverse";
                    if (d.gather) form = "rows-gather";
                    if (d.inter) form = d.inter == 1 ? "rows-interleave" : d.inter == 2 ? "rows-deinterleave" : "rows-keep-plane";
                }
                std::fprintf(stderr, "amap plan: %s vec_bytes=%d workgroups=%u lds=%u lanes=%u elements=%lld\n", form, vb, d.n_blocks, lds,
                             64u << nwlog, (long long)vol);
            }
        uint32_t nb = 0;
        for (const DevPiece &d : dps) nb += d.n_blocks;
        if (cur.n_pieces + dps.size() > (size_t)kMaxPiecesPerLaunch || (uint64_t)blocks + nb >= (1u << 31)) flush();
        for (DevPiece d : dps) {
            // a flat tile of 8 KiB and more: few workgroups fit a compute unit, so each should bring 4 wavefronts
            // (rows of 81 elements: 9.1 -> 7.8 us, of 169: 10.9 -> 6.8 us; of 49 and fewer a single wavefront is faster)
            if (d.kind == PK_FLAT && ((uint64_t)d.eP * std::min(d.EQ, 1u << d.lqlog) * m.elem >= 8192 || d.rag_cb)) split_rows = true;
            if (d.kind != PK_ROWS && d.kind != PK_FLAT && d.n_blocks && d.tilesP > 1 && (d.eP * (uint64_t)m.elem) % 128 != 0) split_rows = true;
            d.first_block = blocks;
            cur.nt = cur.n_pieces == 0 ? d.flags : (cur.nt & d.flags);
            cur.p[cur.n_pieces++] = d;
        }
        blocks += nb;
        lds_max = std::max(lds_max, lds);
        out.min_vec_bytes = std::min(out.min_vec_bytes, vb);
        if (vol > best_vol) {
            best_vol = vol;
            out.main_kernel = fam;
        }
    };
    // groups of pieces that are neighbours along the dst-contiguous dimension
    std::vector<char> grouped(m.kpieces.size(), 0);
    if ((family < 0 || family == AMAP_K_TILE || family == AMAP_K_WAVE) && !out.windowed) {
        std::vector<char> in_group;
        for (const auto &g : find_groups(m, in_group)) {
            std::vector<DevPiece> dps;
            uint32_t lds = 0;
            int vb = 0;
            bool fits = true;
            for (const Member &mem : g) fits = fits && (int)mem.dims.size() <= kMaxLoops;
            if (!fits || !plan_group(m, g, family, nwlog, dps, lds, vb)) continue;
            int64_t vol = 0;
            for (const Member &mem : g) vol += mem.kp->volume();
            emit(dps, lds, vb, dps[0].kind == PK_TILE ? AMAP_K_TILE : AMAP_K_WAVE, vol);
            for (const Member &mem : g) grouped[mem.kp - m.kpieces.data()] = 1;
        }
    }
    // then the remaining copy pieces, fill pieces last (measured: constant
    // stores at the head of the launch delay the first loads more than they gain)
    std::vector<const KPiece *> order;
    for (size_t i = 0; i < m.kpieces.size(); ++i)
        if (!grouped[i] && !m.kpieces[i].fill) order.push_back(&m.kpieces[i]);
    for (size_t i = 0; i < m.kpieces.size(); ++i)
        if (!grouped[i] && m.kpieces[i].fill) order.push_back(&m.kpieces[i]);
    for (const KPiece *kpp : order) {
        const KPiece &kp = *kpp;
        if ((int)kp.dims.size() > kMaxLoops) return false;
        DevPiece dp;
        uint32_t lds = 0;
        int vb = 0;
        int fam = plan_piece(m, kp, family, nwlog, dp, lds, vb);
        if (fam < 0) return false;
        emit({dp}, lds, vb, fam, kp.volume());
    }
    flush();
    out.strided_ok = true;
    return true;
}

// A transposing piece whose P or Q extent is not a whole number of vectors would
// have to run element by element.  Cut it into a main part with whole vectors
// and a thin tail (fewer than one vector wide), planned on their own.
static std::vector<KPiece> split_ragged(const KPiece &kp, int es) {
    std::vector<KPiece> out{kp};
    if (kp.fill) return out;
    const int64_t vmax = 16 / es;
    int iP = -1, iQ = -1;
    for (int k = 0; k < (int)kp.dims.size(); ++k) {
        if (kp.dims[k].ds == 1) iP = k;
        if (kp.dims[k].ss == 1) iQ = k;
    }
    if (iP < 0 || iQ < 0 || iP == iQ) return out;
    // a flat tile takes the piece whole (under the same switches as in plan_piece)
    const bool flat_on = env_int("AMAP_FLAT", 1) && env_int("AMAP_GATHER", 1) && env_int("AMAP_VEC_BYTES", 16) >= 16;
    if (flat_on && flat_shape(kp, es).dir) return out;
    std::vector<int64_t> ds_others;
    for (int k = 0; k < (int)kp.dims.size(); ++k)
        if (k != iP) ds_others.push_back(kp.dims[k].ds);
    const int64_t V = common_pow2((uint32_t)vmax, {kp.dbase}, ds_others);  // what the dst side allows
    if (V < 2) return out;
    int64_t EQc = 0;
    q_chain(kp, iP, iQ, EQc);
    const bool chain_whole = env_int("AMAP_TILE_CHAIN_VEC", 1) && EQc % V == 0;  // vectors may straddle the chain's loops
    for (int dim : {iQ, iP}) {
        std::vector<KPiece> next;
        for (const KPiece &p : out) {
            const int64_t E = p.dims[dim].extent, tail = E % V;
            if (tail == 0 || E < 2 * V || (dim == iQ && chain_whole)) {
                next.push_back(p);
                continue;
            }
            KPiece a = p, b = p;
            a.dims[dim].extent = E - tail;
            b.dims[dim].extent = tail;
            b.dbase += (E - tail) * p.dims[dim].ds;
            b.sbase += (E - tail) * p.dims[dim].ss;
            next.push_back(std::move(a));
            next.push_back(std::move(b));
        }
        out = std::move(next);
    }
    for (KPiece &p : out) {
        std::vector<KDim> d;
        for (const KDim &x : p.dims)
            if (x.extent > 1) d.push_back(x);
        p.dims = merge_loops(std::move(d));
    }
    return out;
}

// Largest span (in elements) a piece may cover on either side: offsets inside a
// piece are 32-bit.  Lowering it (tests) makes small tensors take the path of
// tensors with 2^31 elements and more.
static int64_t span_limit() {
    const int bits = env_int("AMAP_MAX_SPAN_LOG2", 31);
    return 1ll << std::min(31, std::max(8, bits));
}

// Give every piece a window (a 64-bit origin on each side, multiples of 64
// elements so that vector and line alignment are unchanged) and cut pieces
// that span more than the limit along the loop that contributes most.
static bool window_pieces(std::vector<KPiece> &ks, int64_t limit) {
    std::vector<KPiece> out;
    std::vector<KPiece> work(ks.rbegin(), ks.rend());
    while (!work.empty()) {
        KPiece p = std::move(work.back());
        work.pop_back();
        int64_t dspan = 0, s_lo = 0, s_hi = 0, worst = -1;
        int at = -1;
        for (int k = 0; k < (int)p.dims.size(); ++k) {
            const KDim &d = p.dims[k];
            const int64_t dd = (d.extent - 1) * d.ds, ss = (d.extent - 1) * d.ss;
            dspan += dd;
            (ss < 0 ? s_lo : s_hi) += ss;
            const int64_t c = std::max(dd, ss < 0 ? -ss : ss);
            if (d.extent > 1 && c > worst) {
                worst = c;
                at = k;
            }
        }
        // 64 elements of slack for the rounding of the window origin, one vector for masked lanes
        if (dspan + 128 < limit && (p.fill || s_hi - s_lo + 128 < limit)) {
            p.dwin = p.dbase / 64 * 64;
            p.dbase -= p.dwin;
            if (!p.fill) {
                const int64_t lo = p.sbase + s_lo;
                p.swin = lo / 64 * 64;
                p.sbase -= p.swin;
            }
            out.push_back(std::move(p));
            continue;
        }
        if (at < 0 || out.size() + work.size() > 100000) return false;
        // cut loop `at` in two; keep the first part a whole number of vectors where it is the row loop
        const KDim d = p.dims[at];
        int64_t half = d.extent / 2;
        if (half > 64) half = half / 64 * 64;
        KPiece a = p, b = p;
        a.dims[at].extent = half;
        b.dims[at].extent = d.extent - half;
        b.dbase += half * d.ds;
        b.sbase += half * d.ss;
        for (KPiece *q : {&b, &a}) {
            std::vector<KDim> dd;
            for (const KDim &x : q->dims)
                if (x.extent > 1) dd.push_back(x);
            q->dims = merge_loops(std::move(dd));
            work.push_back(std::move(*q));
        }
    }
    ks = std::move(out);
    return true;
}

bool plan_strided(const amap &m0, int family, Plan &out) {
    amap m = m0;  // the planner's own piece list: ragged pieces cut into main part + tails
    m.plan.reset();
    if (m.strided) {
        std::vector<KPiece> ks;
        for (const KPiece &kp : m0.kpieces)
            for (KPiece &p : split_ragged(kp, m.elem)) ks.push_back(std::move(p));
        if (ks.size() <= 4 * m0.kpieces.size() + 8) m.kpieces = std::move(ks);
    }
    out.windowed = false;
    if (m.strided) {
        const int64_t limit = span_limit();
        bool big = volume_of(m.shape) >= limit;
        for (const auto &s : m.src_shapes)
            if (!s.empty() && volume_of(s) >= limit) big = true;
        if (big) {
            if (!window_pieces(m.kpieces, limit)) {
                out.strided_ok = false;
                out.fits32 = false;
                return false;
            }
            out.windowed = true;
        }
    }
    const int nw_env = env_int("AMAP_WAVES_LOG", -1);
    bool split_rows = false;
    if (nw_env >= 0 && nw_env <= 2) return plan_strided_nw(m, family, nw_env, out, split_rows);
    if (!plan_strided_nw(m, family, -1, out, split_rows)) return false;
    // rows that are not whole lines were split between workgroups: larger
    // workgroups can span them (large flat tiles ask for them as well)
    if (split_rows && !out.launches.empty() && out.launches[0].nwlog < 2) {
        Plan wide = out;
        bool still = false;
        if (plan_strided_nw(m, family, 2, wide, still)) out = wide;
    }
    return true;
}

// ---------------------------------------------------------------- program

namespace {

struct Flattener {
    Program &P;
    bool ok = true;
    int64_t max_src = -1;

    int alloc() {
        if (P.n >= kMaxInstr) {
            ok = false;
            return -1;
        }
        std::memset(&P.ins[P.n], 0, sizeof(Instr));
        return P.n++;
    }

    void concat_group(const PNode *n, size_t lo, size_t hi) {
        if (volume_of(n->shape) >= (1ll << 31)) {   // as in emit: 32-bit intermediate indices
            ok = false;
            return;
        }
        // one CONCAT instruction over at most 8 children or groups of children
        int at = alloc();
        if (at < 0) return;
        const size_t count = hi - lo;
        const size_t per = (count + 7) / 8;  // children per slot
        Instr &I = P.ins[at];
        I.kind = I_CONCAT;
        I.rank = (int32_t)n->shape.size();
        I.a = n->axis;
        std::vector<std::pair<size_t, size_t>> slots;
        for (size_t s = lo; s < hi; s += per) slots.push_back({s, std::min(hi, s + per)});
        P.ins[at].b = (int32_t)slots.size();
        for (size_t t = 0; t < slots.size(); ++t) {
            int64_t ext = 0;
            for (size_t c = slots[t].first; c < slots[t].second; ++c) ext += n->kids[c]->shape[n->axis];
            P.ins[at].v[t] = (int32_t)ext;
        }
        for (size_t t = 0; t < slots.size() && ok; ++t) {
            P.ins[at].w[t] = P.n;
            if (slots[t].second - slots[t].first == 1)
                emit(n->kids[slots[t].first].get());
            else
                concat_group(n, slots[t].first, slots[t].second);
        }
    }

    void emit(const PNode *n) {
        while (ok) {
            if (n->kind == PNode::CONCAT) {
                concat_group(n, 0, n->kids.size());
                return;
            }
            // the interpreter linearises every intermediate index in 32 bits: a chain that passes
            // through a tensor of 2^31 elements or more (a repeat or tile that a later slice cuts
            // down again) has no program form, however small its source and dst are
            if (volume_of(n->shape) >= (1ll << 31) || std::llabs(n->begin) >= (1ll << 31) || std::llabs(n->step) >= (1ll << 31) ||
                n->count >= (1ll << 31)) {
                ok = false;
                return;
            }
            int at = alloc();
            if (at < 0) return;
            Instr &I = P.ins[at];
            const int rank = (int)n->shape.size();
            I.rank = rank;
            switch (n->kind) {
            case PNode::SOURCE:
                I.kind = I_SOURCE;
                I.a = n->src_id;
                for (int k = 0; k < rank; ++k) I.v[k] = (int32_t)n->shape[k];
                max_src = std::max<int64_t>(max_src, n->src_id);
                return;
            case PNode::TRANSPOSE:
                I.kind = I_TRANSPOSE;
                for (int k = 0; k < rank; ++k) I.v[k] = n->perm[k];
                break;
            case PNode::RESHAPE: {
                I.kind = I_RESHAPE;
                const auto &cs = n->kids[0]->shape;
                I.a = (int32_t)cs.size();
                for (int k = 0; k < rank; ++k) I.v[k] = (int32_t)n->shape[k];
                for (size_t k = 0; k < cs.size(); ++k) I.w[k] = (int32_t)cs[k];
                break;
            }
            case PNode::SLICE:
                I.kind = I_SLICE;
                I.a = n->axis;
                I.v[0] = (int32_t)n->begin;
                I.v[1] = (int32_t)n->step;
                break;
            case PNode::REPEAT:
            case PNode::TILE:
                I.kind = n->kind == PNode::REPEAT ? I_REPEAT : I_TILE;
                I.a = n->axis;
                I.b = (int32_t)n->count;
                break;
            case PNode::PAD: {
                I.kind = I_PAD;
                I.b = (int32_t)n->fill;
                const auto &cs = n->kids[0]->shape;
                for (int k = 0; k < rank; ++k) {
                    I.v[k] = (int32_t)n->lo[k];
                    I.w[k] = (int32_t)cs[k];
                }
                break;
            }
            default:
                ok = false;
                return;
            }
            n = n->kids[0].get();
        }
    }
};

}  // namespace

bool plan_program(const amap &m, Plan &out) {
    out.program_ok = false;
    if (!m.prog || !out.fits32) return false;
    std::memset(&out.prog, 0, sizeof(out.prog));
    out.prog.rank = (int32_t)m.shape.size();
    for (size_t k = 0; k < m.shape.size(); ++k) out.prog.shape[k] = (int32_t)m.shape[k];
    Flattener f{out.prog};
    f.emit(m.prog.get());
    if (!f.ok || f.max_src >= 16) return false;
    out.n_prog_src = (int)f.max_src + 1;
    out.program_ok = true;
    return true;
}

void attach_plan(amap &m) {
    auto p = std::make_shared<Plan>();
    plan_strided(m, -1, *p);
    plan_program(m, *p);
    if (!p->strided_ok) {
        p->main_kernel = AMAP_K_PROGRAM;
        p->min_vec_bytes = m.elem;
    }
    m.plan = p;
}

}  // namespace amap_detail
