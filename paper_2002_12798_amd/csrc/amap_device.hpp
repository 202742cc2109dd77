// Plain-data descriptors shared by the host planner and the gfx950 kernels.
// A launch carries up to kMaxPiecesPerLaunch pieces by value in its kernel
// arguments, so executing a map needs no device allocation and no copy.
#pragma once

#include <cstdint>

namespace amap_dev {

constexpr int kMaxLoops = 8;             // loops per piece after merging
constexpr int kMaxPiecesPerLaunch = 11;  // keeps the argument block under 4 KiB
constexpr int kMaxThreads = 256;         // up to 4 wavefronts per workgroup
constexpr int kProgramThreads = 256;
constexpr int kRowsUnroll = 4;           // vectors per lane in the row kernel

// n / d for n < 2^31:  q = (umulhi(n, mul) + n) >> shift
struct FastDiv {
    uint32_t mul, shift;
};

inline FastDiv make_fastdiv(uint32_t d) {
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    uint64_t m = ((1ull << 32) * ((1ull << l) - d)) / d + 1;
    return FastDiv{(uint32_t)m, l};
}

inline uint32_t fastdiv_host(uint32_t n, FastDiv f) {
    return (uint32_t)((((uint64_t)n * f.mul) >> 32) + n) >> f.shift;
}

struct Loop {
    uint32_t extent;
    int32_t ds, ss;  // element strides on the dst / source side
    FastDiv fd;      // division by extent
};

enum PieceKind : uint32_t {
    PK_ROWS = 0,  // one lane per vector, dst order (also fill pieces and the element-wise form)
    PK_TILE = 1,  // P x Q tile, register micro-transpose, staged through LDS
    PK_WAVE = 2,  // P x Q tile per wavefront, register micro-transpose, no LDS
    PK_FLAT = 3,  // block of rows that is one contiguous run on one side, staged through LDS
    PK_XLANE = 4  // short P runs: one vector per lane, V x V blocks transposed across V lanes (ds_bpermute)
};

enum PieceFlags : uint32_t {
    PF_NT_LOAD = 1,   // source accesses of a wavefront cover whole 128-byte lines
    PF_NT_STORE = 2   // dst accesses of a wavefront cover whole 128-byte lines
};

struct DevPiece {
    uint32_t kind;
    uint32_t flags;
    uint32_t first_block;  // first workgroup of this piece within the launch
    uint32_t n_blocks;
    uint32_t n_units;      // ROWS: vectors in the piece
    const void *src;       // device pointer of the piece's source (patched in at launch); null = fill
    uint32_t fill;         // fill pattern replicated to 32 bits
    uint32_t dbase, sbase; // element offsets
    uint32_t vlog;         // log2(elements per vector)
    uint32_t nloops;
    // ROWS: loops[0..nloops) innermost first; loop 0 counts vectors.
    // TILE/WAVE: loops[0..nq) = Q chain innermost first (ds used, contiguous in the source),
    //            loops[nq..nloops) = batch loops.
    Loop loops[kMaxLoops];
    uint32_t nq;
    uint32_t eP, EQ;       // extents in elements along P (dst-contiguous) and the merged Q chain
    int32_t ssP;           // source stride of P
    uint32_t tilesP, tilesQ;
    FastDiv fdTP, fdTQ;
    uint32_t lqlog;        // log2(lanes along Q); lanes along P = 64 >> lqlog
    uint32_t nwplog;       // log2(wavefronts along P); wavefronts along Q = (1 << nwlog) >> nwplog
    uint32_t nwlog;        // log2(wavefronts per workgroup), the same for every piece of a launch
    // LDS column swizzle of the staged tile: column ^= (lq & ((1 << swz_bits) - 1)) << swz_shift
    uint32_t swz_bits, swz_shift;
    // Pieces that are neighbours along P (concat on the dst-contiguous dimension,
    // padding of it) are executed as one tile piece so that tiles follow the dst
    // lines, not the piece boundaries: the head entry carries the geometry and
    // the total P extent, it and the group_n - 1 entries after it carry their own
    // source, source strides and first P index.  group_n = 1: a plain piece.
    uint32_t group_n;
    uint32_t p_begin;
    // ROWS only: every source element of the row is written 1 << rep_log times in
    // a row (a repeat along the contiguous dimension); a lane then loads
    // 1 / (1 << rep_log) of a vector and spreads it over a whole one.
    uint32_t rep_log;
    // ROWS only: the row walks the source backwards (a reversed contiguous axis).  Loop 0 has
    // source stride -V; the lane loads the V elements that END at its source offset and
    // reverses them in registers.
    uint32_t rev;
    // ROWS only: gather.  The dst vectors tile a run that several loops cover jointly (they
    // continue one another in dst), but the source is not contiguous along it (an innermost
    // extent of 3, a repeat by 3, ...).  Loop 0 counts the 16-byte dst vectors of the run and does
    // not move in the source; the run's own loops sit at the END of loops[] (loops[kMaxLoops - 1 - j],
    // j < nq, innermost first) and give, element by element, the source offset of a dst position.
    uint32_t gather;
    // ROWS only: interleave (1) / de-interleave (2) of eP = 2 .. 7 planes (a planar image made
    // interleaved and back, a pixel shuffle).  A unit is one 16-byte vector of positions q per plane.  1: the lane
    // loads one vector from each of the eP planes (ssP elements apart in the source) and writes eP
    // consecutive dst vectors holding the positions' plane values side by side.  2: the reverse,
    // eP consecutive source vectors taken apart into one vector per plane, ssP elements apart in dst.
    // Loop 0 counts the units and carries the strides of a unit on both sides.
    // 3 / 4: one plane only is kept (a slice with step eP = 2 along the contiguous dimension, 2-byte elements):
    // the lane loads eP consecutive vectors and keeps the first (3) or the last (4) element of every
    // group of eP; the window lies so that it never leaves the source.
    uint32_t inter;
    // FLAT only.  An r x c matrix (r: EQ values, blocks of 1 << lqlog = 16, 32 or 64; c: eP values, any number) is contiguous
    // on one side (offset r * eP + c) and has rows along r on the other (offset f(c) + r, where c runs
    // over the nq loops at the END of loops[], loops[kMaxLoops - 1 - j], innermost first, each with
    // its own stride on that side).  1: the source is the contiguous side, 2: dst is.
    // tilesP = blocks along r; loops[0..nloops) = batch loops.  A workgroup moves the contiguous run of its block in 16-byte vectors into / out of LDS
    // and serves the other side with 16-byte vectors along r whose elements it picks one by one.
    uint32_t flat;
    // FLAT, column-blocked ("ragged") form, for rows too long for LDS: rag_cb > 0.  A workgroup takes
    // rows x rag_cb elements (tilesQ blocks along c, the fastest-running part of the workgroup index).  On
    // the contiguous side a row segment starts at any element: loads take 16-byte vectors from the segment's
    // start (under-aligned) and single elements at its end; stores take the aligned 16-byte slots the
    // segment covers (rag_s = rag_cb / V + 1 of them), whole where the slot lies inside the segment and
    // element by element at the two ends.  LDS rows are rag_w elements apart.
    uint32_t rag_cb, rag_w, rag_s;
    FastDiv fd_rag_s;
    // XLANE only.  A dst row (the whole P run, fills beside it included) is xl_npv vectors long; a wavefront
    // takes xl_rows consecutive Q positions (a multiple of V, xl_rows * xl_npv <= 64): lane l stores vector
    // l % xl_npv of row l / xl_npv, so the stores of a wavefront are one contiguous run of dst.  n_units =
    // wavefront tiles of the piece (tilesQ per batch point); loops as for TILE.
    uint32_t xl_npv, xl_rows;
    FastDiv fd_npv;
    // Window of the piece in tensors too large for 32-bit offsets: dbase and every
    // dst offset are relative to element dwin of dst; swin likewise for the source
    // (the host folds it into `src` at launch).  0 for ordinary tensors.
    uint64_t dwin, swin;
};

struct LaunchArgs {
    uint32_t n_pieces;
    uint32_t nwlog;      // workgroup size = 64 << nwlog
    uint32_t nt;         // PieceFlags every piece of the launch agrees on
    uint32_t xcd_remap;  // 1: remap workgroup indices so each XCD gets a contiguous range
    DevPiece p[kMaxPiecesPerLaunch];
};

static_assert(sizeof(LaunchArgs) <= 4000, "kernel argument block too large");

// ---- operator program for the element-wise interpreter ----
constexpr int kMaxInstr = 24;
enum InstrKind : int32_t { I_SOURCE = 0, I_TRANSPOSE, I_RESHAPE, I_SLICE, I_PAD, I_CONCAT, I_REPEAT, I_TILE };

struct Instr {
    int32_t kind;
    int32_t rank;  // rank of the index the instruction receives
    int32_t a;     // SOURCE: src id; SLICE/CONCAT/REPEAT/TILE: axis; RESHAPE: child rank
    int32_t b;     // PAD: fill bits; CONCAT: number of children; REPEAT: count; TILE: extent of the child's axis
    int32_t v[8];  // SOURCE: shape; TRANSPOSE: perm; RESHAPE: own shape; SLICE: {begin, step}; PAD: lo; CONCAT: child extents
    int32_t w[8];  // RESHAPE/PAD: child shape; CONCAT: jump targets
};

struct Program {
    int32_t n;
    int32_t rank;          // dst rank
    int32_t shape[8];      // dst shape
    Instr ins[kMaxInstr];
};

static_assert(sizeof(Program) <= 2048, "program too large");

struct SrcTable {
    const void *p[16];
};

}  // namespace amap_dev
