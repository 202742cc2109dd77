// Host-side representation of a composed access map.
//
// Two representations of the same function  dst index -> (source, offset) | fill
// are kept side by side:
//
//  * the operator program: the chain (or tree, with concat) of per-operator
//    index functions, applied one after the other to a dst multi-index.  It
//    represents ANY composition of the supported operators (piecewise
//    quasi-affine in general) and is what the element-wise fallback executes;
//
//  * the strided normal form: a list of disjoint pieces.  A piece is a loop
//    nest (its iteration dims) with an affine store address into dst and an
//    affine load address into one source - the paper's pair
//    (v = t_l[f_l(i)], t_s[f_s(i)] = v) of Section 2.1 with both maps in
//    linearised form - or a constant fill.  It exists whenever composition
//    can cancel every floor-div / mod, which is what the fast kernels need.
#pragma once

#include <cstdint>
#include <memory>
#include <vector>

#include "amap.h"

namespace amap_detail {

constexpr int kMaxRank = AMAP_MAX_RANK;
constexpr int kMaxPieces = 4096;  // beyond this the strided form is dropped

struct PNode {
    enum Kind { SOURCE, TRANSPOSE, RESHAPE, SLICE, PAD, CONCAT, REPEAT, TILE } kind = SOURCE;
    std::vector<int64_t> shape;  // shape of this node's output tensor
    int src_id = -1;             // SOURCE
    std::vector<int> perm;       // TRANSPOSE
    int axis = 0;                // SLICE, CONCAT, REPEAT, TILE
    int64_t count = 1;           // REPEAT: r;  TILE: extent of the child's axis
    int64_t begin = 0, step = 1; // SLICE; TILE keeps its number of copies in step
    std::vector<int64_t> lo;     // PAD
    uint32_t fill = 0;           // PAD
    std::vector<std::shared_ptr<const PNode>> kids;
};

// One loop of a piece's loop nest.  The loop variable i in [0, extent)
// contributes i * mult to the dst index of dimension `dim` and i * sstride
// to the source element offset.
struct IterDim {
    int64_t extent;
    int dim;
    int64_t mult;
    int64_t sstride;
};

struct Piece {
    bool fill = false;
    uint32_t fill_bits = 0;
    int src = -1;
    int64_t sbase = 0;
    int64_t lo[kMaxRank] = {0};  // dst index of the piece's origin, per dst dim
    std::vector<IterDim> it;     // sorted by (dim ascending, mult descending); extents > 1
    int64_t volume() const {
        int64_t v = 1;
        for (const auto &d : it) v *= d.extent;
        return v;
    }
};

// Linearised loop of a piece: dst and src element strides.
struct KDim {
    int64_t extent, ds, ss;
};

// A piece ready for a kernel: loops sorted by dst stride descending, loops
// that are contiguous on both sides merged.
struct KPiece {
    bool fill = false;
    uint32_t fill_bits = 0;
    int src = -1;
    int64_t dbase = 0, sbase = 0;
    // Set by the launch planner only: element offsets of the piece's window on
    // either side.  Once set, dbase / sbase are relative to them, so that every
    // offset inside the piece fits 32 bits even in tensors of 2^31 elements and more.
    int64_t dwin = 0, swin = 0;
    std::vector<KDim> dims;
    int64_t volume() const {
        int64_t v = 1;
        for (const auto &d : dims) v *= d.extent;
        return v;
    }
};

}  // namespace amap_detail

struct amap {
    int elem = 2;
    std::vector<int64_t> shape;                    // dst shape
    std::vector<std::vector<int64_t>> src_shapes;  // by source id; empty vector = id not used
    std::shared_ptr<const amap_detail::PNode> prog;
    bool strided = false;
    bool injective = true;                         // false once repeat / tile / a repeated concat source may read an element twice
    std::vector<amap_detail::Piece> pieces;
    std::vector<amap_detail::KPiece> kpieces;      // derived from pieces when strided
    std::shared_ptr<void> plan;                    // device launch plan (owned by the executor)
    mutable int64_t distinct_reads = -1;           // distinct source elements read, once counted (see distinct_source_elements)
};

namespace amap_detail {

inline int64_t volume_of(const std::vector<int64_t> &s) {
    int64_t v = 1;
    for (auto e : s) v *= e;
    return v;
}

std::vector<int64_t> row_major_strides(const std::vector<int64_t> &shape);

// Sort loops by dst stride (descending) and merge neighbours that are
// contiguous on both sides.
std::vector<KDim> merge_loops(std::vector<KDim> dims);

// Recompute m.kpieces from m.pieces (no-op if not strided).
void finalise(amap &m);

// Number of distinct source elements a map reads (exact).  Closed form when every source is read by
// one piece whose moving loops cannot meet; otherwise one bit per source element is marked while the
// pieces (or, without a strided form, the program) are walked: throws std::bad_alloc when the sources
// hold more than kMaxDistinctBits elements.  The count is kept in the map.
constexpr int64_t kMaxDistinctBits = int64_t(1) << 33;   // 1 GiB of marks
int64_t distinct_source_elements(const amap &m);

// Evaluate the operator program for one dst multi-index.
// Returns true and sets (src, off) for a data element, false for fill (sets fill).
bool eval_program(const PNode *n, const int64_t *idx, int *src, int64_t *off, uint32_t *fill);

}  // namespace amap_detail
