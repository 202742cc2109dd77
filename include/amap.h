/*
 * amap - composed access maps for chains of layout operators, and their
 * single-kernel execution on gfx950.
 *
 * Model (paper Section 2, equations "load" and "store"): every tensor access
 * is an element-wise load v = t[f(i)] or store t[f(i)] = v inside a loop nest
 * i, with f(i) = C i + b.  A layout operator (transpose, reshape, slice, pad,
 * concat) is one load/store pair whose load feeds its store directly
 * (Section 2.1).  Data-movement elimination reverses the store map, composes
 * it with the load map (eq. 3) and rewrites every consumer load to read the
 * original tensor through the composed function (eq. 4), so the intermediate
 * tensor and the copy that defined it disappear.
 *
 * An amap_t is such a composed function for a whole chain: it maps every
 * index of the chain's final tensor ("dst") either to (source tensor id,
 * element offset in that source) or to a constant fill pattern.  Reshape
 * makes the function quasi-affine (floor-div / mod by constants) and pad /
 * concat make it piecewise, so the normal form is a list of disjoint pieces,
 * each a loop nest with an affine store address into dst and an affine load
 * address into one source (or a constant).
 *
 * All tensors are dense, row-major, offset 0.  Elements are opaque bit
 * patterns of 2 or 4 bytes; data movement never interprets them.
 *
 * Conventions: every call returns an amap_status and never aborts; on error
 * the out-parameter is left untouched.  amap_t objects are immutable after
 * creation, live in host memory, may be shared between threads, and are
 * released by the caller with amap_free.  The library never owns tensor
 * memory.  Pointers named src / dst / A_src / W / out in the device entry
 * points are DEVICE pointers; everything else is a host pointer.
 */
#ifndef AMAP_H
#define AMAP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AMAP_MAX_RANK 8

typedef struct amap amap_t;

typedef enum {
    AMAP_OK = 0,
    AMAP_E_INVALID = 1,      /* null pointer, bad rank / axis / perm / element size / source id */
    AMAP_E_SHAPE = 2,        /* reshape volume mismatch, slice or pad out of range, concat extents */
    AMAP_E_UNSUPPORTED = 3,  /* e.g. reverse of a map that is not a bijection */
    AMAP_E_NOMEM = 4,
    AMAP_E_ALIAS = 5,        /* dst overlaps a source */
    AMAP_E_HIP = 6           /* the HIP runtime reported an error at launch */
} amap_status;

typedef enum { AMAP_B16 = 2, AMAP_B32 = 4 } amap_elem; /* element size in bytes */

/* ---- map construction (host only) --------------------------------------
 * Each builder returns a NEW map for "operator applied to the tensor that m
 * describes": the operator's own index function (its f in v = in[f(i)]) is
 * composed with m (eq. 4 with identity store maps) and normalised.  Inputs
 * are unchanged. */

/* The identity map of source tensor number src_id with the given shape. */
amap_status amap_source(int src_id, int rank, const int64_t *shape, amap_elem es, amap_t **out);

/* out axis k = in axis perm[k] (numpy / torch permute convention). */
amap_status amap_transpose(const amap_t *m, const int32_t *perm, amap_t **out);

/* Row-major reshape; the volume must be preserved. */
amap_status amap_reshape(const amap_t *m, int rank, const int64_t *shape, amap_t **out);

/* One axis strided (strided_slice in the paper's Section 2.1 operator list).
 * step >= 1: keep indices begin, begin+step, ... < end; needs 0 <= begin < end <= extent.
 * step <= -1: keep begin, begin+step, ... > end, walking the axis downwards;
 * needs -1 <= end < begin <= extent - 1 (end = -1 reaches index 0). */
amap_status amap_slice(const amap_t *m, int axis, int64_t begin, int64_t end, int64_t step,
                       amap_t **out);

/* Section 2.1 operator list, "repeat": every index of one axis r >= 1 times in
 * a row, out[.., i, ..] = in[.., i / r, ..].  A load that is not injective. */
amap_status amap_repeat(const amap_t *m, int axis, int64_t r, amap_t **out);

/* Section 2.1 operator list, "tile": the whole axis t >= 1 times one after the
 * other, out[.., i, ..] = in[.., i % extent, ..].  Broadcasting an extent-1
 * axis to t is the case extent = 1. */
amap_status amap_tile(const amap_t *m, int axis, int64_t t, amap_t **out);

/* lo[k] / hi[k] >= 0 fill elements before / after axis k; fill_bits is the
 * constant (its low 16 bits for 2-byte elements). */
amap_status amap_pad(const amap_t *m, const int64_t *lo, const int64_t *hi, uint32_t fill_bits,
                     amap_t **out);

/* Join n maps along axis; all other extents and the element size must agree.
 * The maps may read different sources, or the same ones. */
amap_status amap_concat(const amap_t *const *ms, int n, int axis, amap_t **out);

/* The paper's "reverse" (Section 2.1): for a map that is a bijection between
 * dst and one source, the map from that source's index space back to dst,
 * expressed as a map whose source 0 has dst's shape. */
amap_status amap_inverse(const amap_t *m, amap_t **out);

/* One-shot form: fold a linear operator list over n_src sources.  A CONCAT
 * may only come first and joins all n_src sources; otherwise n_src must be 1. */
typedef struct {
    int rank;
    const int64_t *shape;
    amap_elem es;
} amap_src_desc;

typedef enum {
    AMAP_TRANSPOSE = 0, AMAP_RESHAPE = 1, AMAP_SLICE = 2, AMAP_PAD = 3, AMAP_CONCAT = 4,
    AMAP_REPEAT = 5, AMAP_TILE = 6
} amap_op_kind;

typedef struct {
    amap_op_kind kind;
    int axis;           /* SLICE, CONCAT, REPEAT, TILE */
    int n;              /* TRANSPOSE: rank; RESHAPE: new rank; PAD: rank; SLICE: 3; REPEAT, TILE: 1 */
    const int64_t *a;   /* TRANSPOSE: perm[n]; RESHAPE: shape[n]; SLICE: {begin,end,step}; PAD: lo[n];
                           REPEAT, TILE: {count} */
    const int64_t *b;   /* PAD: hi[n] */
    uint32_t fill_bits; /* PAD */
} amap_op;

amap_status amap_compose(const amap_src_desc *srcs, int n_src, const amap_op *ops, int n_ops,
                         amap_t **out);

void amap_free(amap_t *m);

/* ---- inspection (host only) -------------------------------------------- */

typedef enum {
    AMAP_K_PROGRAM = 0, /* element-wise interpreter of the operator program (any map)      */
    AMAP_K_ELEMENT = 1, /* element-wise over the strided pieces                             */
    AMAP_K_ROWS = 2,    /* both sides share their contiguous dimension: vector row copy     */
    AMAP_K_TILE = 3,    /* contiguous dimension permuted: LDS-staged tile transpose (also the
                           flat tiles: blocks of rows that are contiguous on one side)      */
    AMAP_K_WAVE = 4     /* small permute without LDS, one tile per wavefront.  Two forms: the
                           register micro-transpose (every lane loads V source vectors and
                           reorders its V x V block in its own registers), and, for 2-byte
                           elements in dst rows of 16 or 32 bytes, the cross-lane form (one
                           vector per lane, the V x V block exchanged between V lanes with
                           ds_bpermute), which is ahead only there (4.7 against 4.0 TB/s at
                           1 GiB per launch; 3.4 against 5.9 TB/s on 80-byte rows of 4-byte
                           elements).  Environment AMAP_XLANE=0 plans the first form
                           everywhere, 2 the second wherever it applies.                    */
} amap_kernel_id;

typedef struct {
    int rank;                        /* of dst */
    int64_t shape[AMAP_MAX_RANK];    /* of dst */
    int elem_size;
    int n_src;                       /* length of the src[] array amap_execute expects */
    int strided;                     /* 1 if the normal form is a list of affine pieces */
    int n_pieces;                    /* copy + fill pieces (0 if not strided) */
    int n_fill_pieces;
    int kernel_id;                   /* amap_kernel_id the planner chose for the largest piece */
    int vec_bytes;                   /* smallest access width planned over all pieces, both sides */
    int64_t min_read_bytes;          /* distinct source elements needed x elem size (an element that
                                        repeat / tile / overlapping concat inputs read several times counts once) */
    int64_t write_bytes;             /* volume(dst) x elem size */
    int64_t fill_bytes;              /* part of write_bytes that is constant fill */
} amap_info;

amap_status amap_describe(const amap_t *m, amap_info *out);
/* With AMAP_PLAN_TRACE=1 in the environment the planner also prints, on stderr, one line per
 * planned piece (its form, vector bytes, workgroups, LDS bytes) whenever it plans a map. */

/* Shape of source src_id as recorded in the map (rank returned in *rank). */
amap_status amap_source_shape(const amap_t *m, int src_id, int *rank, int64_t *shape);

/* Evaluate the map on HOST memory: dst[i] = src[g(i)] or the fill.  For tests
 * of the composer on machines without a GPU; the device path never calls it.
 * mode 0: as the map is represented (pieces if strided, else the program);
 * mode 1: operator program; mode 2: pieces (AMAP_E_UNSUPPORTED if not strided). */
amap_status amap_eval_host(const amap_t *m, const void *const *src, void *dst, int mode);

/* Diagnostic: number of dst elements written by no piece / by more than one
 * piece of a strided map (both 0 for a well-formed map; out-of-range
 * addresses count as overwritten).  Costs one byte of host memory per dst
 * element. */
amap_status amap_check_cover(const amap_t *m, int64_t *unwritten, int64_t *overwritten);

/* Diagnostic: replay on the host, lane by lane, the launches that
 * amap_execute_kernel(.., kernel_id) would make (kernel_id -1 = planned) and
 * count out-of-bounds accesses, dst elements with no or several writers, and
 * dst elements routed from the wrong source element.  Moves no tensor data;
 * lets the device indexing be verified on a machine without a GPU. */
amap_status amap_plan_selfcheck(const amap_t *m, int kernel_id, int64_t *n_errors);

/* Diagnostic: the same for the 256 x 256-tile kernel of amap_gemm_fused / amap_gemm_fused_store
 * (see amap_gemm_fused for the shapes it takes): replays on the host, with the kernel's own address
 * functions, the loads of every workgroup (for a device of n_workgroups compute units: the kernel
 * launches as many workgroups, at most one per compute unit, as give every one the same number of
 * tiles; a small number makes workgroups walk many tiles) and the stores of every tile
 * for the product A_map x W (W row-major [K,N] when W_map is NULL, else read through W_map as in
 * amap_gemm_mapped; stored through out_map when it is not NULL), and counts loads
 * outside A's source or W, k-steps that fetch anything but their own block of A and W, fetches out
 * of the order of use, stores outside out and elements of out written never or twice.
 * AMAP_E_UNSUPPORTED when the product would run in the general kernel (no replay for that one). */
amap_status amap_gemm_selfcheck(const amap_t *A_map, const amap_t *W_map, int64_t N, const amap_t *out_map,
                                int n_workgroups, int64_t *n_errors);

/* ---- data-movement elimination over an operator graph (host only) ---------
 * Section 2.1 applied to a whole program: tensors are either materialised
 * (graph inputs, results of compute operators) or defined by a layout operator,
 * i.e. by a load/store pair whose load feeds its store.  amap_graph_eliminate
 * repeats the rewrite of eq. 3 / eq. 4 until no load reads a tensor defined by
 * such a pair: every load of a compute operator, and every graph output, ends
 * up reading materialised tensors through one composed map, and the
 * intermediate tensors and the copies that defined them disappear.
 * Compute operators are opaque here: the graph records only what they read
 * and the shape of what they produce. */
typedef struct amap_graph amap_graph_t;

amap_status amap_graph_create(amap_graph_t **out);
void amap_graph_free(amap_graph_t *g);

/* A tensor that exists in memory before the graph runs.  *tensor receives its id. */
amap_status amap_graph_input(amap_graph_t *g, int rank, const int64_t *shape, amap_elem es, int *tensor);

/* tensor = op(inputs): a layout operator (CONCAT takes n_inputs >= 1 tensors, every other kind one). */
amap_status amap_graph_op(amap_graph_t *g, const amap_op *op, const int *inputs, int n_inputs, int *tensor);

/* A layout operator given as a map in load (gather) form: tensor[i] = inputs[src][map(i)], any
 * composed map over n_inputs sources (source id k of the map reads inputs[k]; shapes and
 * element size must agree with the graph tensors, else AMAP_E_SHAPE). */
amap_status amap_graph_map(amap_graph_t *g, const amap_t *map, const int *inputs, int n_inputs, int *tensor);

/* A layout operator given in store (scatter) form, the paper's t_s[f_s(i)] = t_l[i]: store_map
 * has the shape of `input` as its dst shape and ONE source, whose shape is the shape of the tensor
 * the operator writes; store_map(i) is where element i of the input goes.  The map is reversed on
 * entry (Section 2.1), so it must be a bijection between the two tensors (AMAP_E_UNSUPPORTED
 * otherwise, as for amap_inverse); from then on the operator is eliminated like the others. */
amap_status amap_graph_store(amap_graph_t *g, const amap_t *store_map, int input, int *tensor);

/* An opaque compute operator reading n_inputs tensors (in this order: input slot k = inputs[k])
 * and producing one materialised tensor of the given shape. */
amap_status amap_graph_compute(amap_graph_t *g, const int *inputs, int n_inputs, int rank, const int64_t *shape,
                               amap_elem es, int *tensor);

/* The tensor must exist in memory when the graph has run. */
amap_status amap_graph_output(amap_graph_t *g, int tensor);

typedef struct {
    int n_layout_ops;            /* layout operators in the graph */
    int n_pairs;                 /* load/store pairs they stand for (a concat of k inputs is k pairs) */
    int n_pairs_left;            /* pairs still executed afterwards: one per source of every graph output
                                    that has to be materialised through a composed map */
    int n_loads;                 /* loads of compute operators + graph outputs, = composed maps produced */
    int n_rewrites;              /* applications of eq. 4 (one load rewritten past one eliminated tensor) */
    int n_alias_outputs;         /* graph outputs whose composed map is the identity of one tensor: no copy left */
    int64_t moved_bytes_before;  /* bytes read + written by all layout operators, one at a time */
    int64_t moved_bytes_after;   /* bytes read + written by the composed maps of the graph outputs */
    int64_t intermediate_bytes;  /* storage of the tensors that no longer exist */
    int n_mapped_loads;          /* compute-operator loads whose composed map is not the identity of a tensor */
    int64_t mapped_load_bytes;   /* bytes read + written if each of those is materialised by one composed copy
                                    (a consumer that fuses the map into its operand load moves none of them) */
} amap_graph_report;

/* Run data-movement elimination to its fixed point.  Call once, after the graph is complete. */
amap_status amap_graph_eliminate(amap_graph_t *g, amap_graph_report *report);

/* Load number `index` (0 .. n_loads-1) after elimination.  consumer = tensor id of the compute
 * operator that issues it, slot = which of its inputs; for a graph output consumer = -1 and
 * slot = the output tensor's id.  *map is a NEW map (caller frees) whose source ids 0 .. *n_src-1
 * stand for the materialised tensors src_tensors[0 .. *n_src-1] (room for 16 entries; maps that
 * read more are refused with AMAP_E_UNSUPPORTED). */
amap_status amap_graph_load(const amap_graph_t *g, int index, int *consumer, int *slot, amap_t **map,
                            int *src_tensors, int *n_src);

/* ---- global layout assignment (host only) --------------------------------
 * The GPU counterpart of the paper's global memory-bank mapping (Section 2.2).
 * There the property propagated through the network is which tensor dimension
 * is spread over the on-chip banks; here it is the order of a tensor's
 * dimensions in HBM (which one is contiguous).  Operators with a restriction
 * (matrix products, convolutions) seed the layouts of their operands,
 * the layouts are propagated along the data dependencies through the
 * unrestricted operators to a fixed point, and only where a tensor meets
 * conflicting requirements is a copy t -> t' inserted, as a relayout map that
 * amap_execute runs.  The propagated assignment is then refined tensor by tensor
 * for as long as the total copy bytes shrink (starting from the cheaper of it and
 * the local assignment), so the result never costs more than the local assignment
 * (every operator on its own, unrestricted operators in the canonical order), with
 * which it is compared. */
typedef struct amap_layout_graph amap_layout_graph_t;

amap_status amap_layout_create(amap_layout_graph_t **out);
void amap_layout_free(amap_layout_graph_t *g);

/* A logical tensor.  An order lists the logical dimensions from the outermost to the
 * innermost (contiguous) one in memory; {0,1,..} is the canonical order.
 * fixed_order = NULL: free; else the order the tensor must have (graph inputs / outputs). */
amap_status amap_layout_tensor(amap_layout_graph_t *g, int rank, const int64_t *shape, amap_elem es,
                               const int32_t *fixed_order, int *tensor);

/* An operator over n operands.  is_output[i] != 0 marks the tensors it produces.
 * req_orders[i] = NULL: the operand is free; else the order this operator needs it in.
 * same_layout != 0: all free operands of equal rank must share one order (element-wise
 * operators, pooling); the operator takes whatever order reaches it. */
amap_status amap_layout_op(amap_layout_graph_t *g, const int *operands, const int *is_output,
                           const int32_t *const *req_orders, int n, int same_layout, int *op);

typedef struct {
    int n_copies_local;          /* copies the per-operator assignment needs */
    int64_t copy_bytes_local;    /* bytes they read + write */
    int n_copies_global;         /* copies left after propagation */
    int64_t copy_bytes_global;
    int n_sweeps;                /* sweeps over the operators until the propagation reached its fixed point */
} amap_layout_report;

amap_status amap_layout_solve(amap_layout_graph_t *g, amap_layout_report *report);

/* After amap_layout_solve: the order assigned to a tensor (rank entries). */
amap_status amap_layout_order(const amap_layout_graph_t *g, int tensor, int32_t *order);

/* Copy number `index` (0 .. n_copies_global-1) of the global assignment: operator `op` reads or
 * writes operand `slot` (tensor `tensor`) in another order than the tensor has in memory.
 * *map is a NEW map (caller frees) from the tensor as stored (source 0, its dimensions in the
 * assigned order) to the order the operator needs; for an output operand the copy runs the other
 * way and *map goes from what the operator wrote to the tensor as stored. */
amap_status amap_layout_copy(const amap_layout_graph_t *g, int index, int *op, int *slot, int *tensor,
                             amap_t **map);

/* ---- execution (device pointers; asynchronous on `stream`) --------------
 * `stream` is a hipStream_t passed as void* (NULL = the default stream).
 * No allocation, no synchronisation, no host access to device memory. */

/* dst[i] = src[src_id][g(i)] or fill, for every index i of dst: the rewritten
 * load v' = t_l[g'(i')] of eq. 4 executed for the whole chain by one kernel
 * per group of pieces (one launch for every map in the five workloads).
 * src has n_src entries, indexed by source id (entries of ids the map no longer
 * reads may be NULL).  dst must not overlap any source (AMAP_E_ALIAS).  dst is
 * fully overwritten.  Tensors may exceed 2^31 elements when the map has a
 * strided form; AMAP_E_UNSUPPORTED if such a map needs the element-wise
 * interpreter. */
amap_status amap_execute(const void *const *src, void *dst, const amap_t *map, void *stream);

/* Several maps over ONE source table executed together (a split: one tensor feeding
 * several outputs, e.g. Q, K and V; eq. 4 applied to every consumer of the same t_l):
 * dst[i] receives maps[i].  The pieces of all maps share launches, so n small outputs
 * cost one launch, not n.  All maps must have the same element size; the dst buffers
 * must not overlap each other or a source. */
amap_status amap_execute_multi(const void *const *src, void *const *dst, const amap_t *const *maps, int n,
                               void *stream);

/* Same, with the kernel family forced (amap_kernel_id) instead of planned:
 * for A/B measurements and for tests of every family on every map.
 * AMAP_E_UNSUPPORTED if that family cannot execute the map. */
amap_status amap_execute_kernel(const void *const *src, void *dst, const amap_t *map,
                                void *stream, int kernel_id);

/* out[M,N] = bf16( A[M,K] x W[K,N] ) with A[m,k] = A_src[g(m,k)] loaded through
 * the map in the operand-load prologue (the consumer load of eq. 4); A is never
 * materialised.  A_map: dst shape [M,K], 2-byte elements (bf16), one source;
 * either no fill pieces, or fill pieces of ONE constant around ONE data piece
 * (A padded along m and / or k, e.g. a zero-padded activation; along k in
 * multiples of 8 elements): the constant is supplied in the operand load.
 * W: [K,N] row-major bf16.  out: [M,N] row-major bf16,
 * fp32 accumulation, round-to-nearest-even on output.
 * Needs N % 8 == 0, K % 8 == 0 and 8-element aligned contiguous source runs in
 * the map, either along k (a row-major operand behind permutes and reshapes) or,
 * with M % 8 == 0, along m (an operand kept transposed, a channel-major activation
 * read as the [N*H*W, C] matrix of a pointwise convolution: 4 k x 8 m blocks are
 * transposed on their way to the matrix cores), else AMAP_E_UNSUPPORTED; M, N and K
 * need not be whole numbers of the 256 x 128 x 64 tiles (edge tiles are clamped on
 * load, masked on store).  Shapes with K % 64 == 0, K >= 128, no padding and
 * source runs of 64 elements and more along k that do not straddle a block of
 * 256 rows (the rows of A one run of evenly spaced source rows, or split into
 * blocks that are multiples of 256) run a kernel with 256 x 256 x 64 tiles whose
 * operands go straight from L2 into LDS, M and N being whole numbers of tiles
 * or not (environment AMAP_GEMM_TILE256=0: the general kernel for these too);
 * both add the same products in the same order, so their results are
 * bit-identical.  Operands and sources of 2^31 elements and more (an A of
 * [1048832, 2048], 4.3 GB) are taken by that kernel only, with a plain store;
 * every other product over such tensors is AMAP_E_UNSUPPORTED. */
amap_status amap_gemm_fused(const void *A_src, const amap_t *A_map, const void *W, int64_t N,
                            void *out, void *stream);

/* The same product with its store rewritten as well (the store side t_s[f_s(i)] = v of
 * Section 2): out_map is the layout chain that would be applied to the product, as a map
 * whose single source is the [M,N] product and whose dst is the final tensor.  It must be
 * a bijection (amap_inverse turns it into the store map) with 8-element aligned contiguous
 * runs along n; element (m, n) is written straight to its place in `out` (the final tensor,
 * M*N elements) and the row-major product never exists.  Example: a QKV projection that
 * writes the head-split layout [3, b, heads, seq, 64] directly. */
amap_status amap_gemm_fused_store(const void *A_src, const amap_t *A_map, const void *W, int64_t N,
                                  const amap_t *out_map, void *out, void *stream);

/* All three accesses of the product rewritten: A through A_map, W through W_map
 * (dst shape [K,N], bf16, one source, no fill; its contiguous runs of a multiple of 8
 * elements may lie along n, as in a row-major weight, or along k, as in a transposed
 * [N,K] weight, which then needs no transposition on its way to the matrix cores), and
 * the product stored through out_map if that is not NULL (as in amap_gemm_fused_store).
 * A [N,K] weight with whole 64-element runs along k and evenly spaced rows also runs in
 * the 256 x 256-tile kernel when A and K are as described for amap_gemm_fused. */
amap_status amap_gemm_mapped(const void *A_src, const amap_t *A_map, const void *W_src, const amap_t *W_map,
                             const amap_t *out_map, void *out, void *stream);

/* The product with A gathered from several sources: a concat along the reduction dimension
 * (channel concat of the branches of an inception block in front of a pointwise convolution,
 * skip connections) rewritten into the consumer load, eq. 4 once per concat operand, so the
 * concatenated tensor never exists.  A_map may have up to 8 sources and one piece per range
 * of k; A_srcs is indexed by the map's source ids (device pointers, 16-byte aligned).  Every
 * piece must span all of m, the pieces must follow one another along k, all with their
 * 8-element runs the same way round: along k, then every range but the last must end at a
 * multiple of 64, or along m, then at a multiple of 32 (a k-step, or half of one, reads one
 * source).  W_map NULL: W_src is the row-major [K,N] weight and N its width; else as in
 * amap_gemm_mapped and N is ignored.  out_map as in amap_gemm_fused_store, or NULL.
 * A single-piece A_map is accepted as well.  AMAP_E_UNSUPPORTED for any other piece structure. */
amap_status amap_gemm_gather(const void *const *A_srcs, const amap_t *A_map, const void *W_src, const amap_t *W_map,
                             int64_t N, const amap_t *out_map, void *out, void *stream);

const char *amap_status_str(amap_status s);

/* Text of the HIP error behind the last AMAP_E_HIP returned on this thread, or the reason
 * why a device entry point (amap_execute*, amap_gemm_*) last returned AMAP_E_UNSUPPORTED on
 * this thread (which requirement the maps did not meet); empty string if none. */
const char *amap_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* AMAP_H */
