/*
 * CPU oracle for layout-operator chains and the consumer GEMM.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that the GPU results can be checked against an independent,
 * plain and slow implementation, and so that a CPU baseline can be timed.
 * It shares no code with the HIP library.
 *
 * Every layout operator is one load/store pair in the sense of the paper's
 * Section 2 (equations "load" and "store"): a loop nest over the index space
 * of the output tensor, a load  v = in[f(i)]  and a store  out[i] = v  with
 * identity store map (Section 2.1, the pair pattern that data-movement
 * elimination looks for).  Each function below writes that loop nest out
 * literally: enumerate every output multi-index, apply the operator's index
 * function f, move one element.  The output is always a freshly materialised
 * dense row-major tensor; nothing is fused, blocked or reordered.
 *
 * Elements are opaque bit patterns of elem_size bytes (2 or 4).
 * All functions return 0 on success and a negative code on a bad argument.
 *
 * Pins (tests/test_oracle_*.py): numpy library routines on iota tensors,
 * operator inverse identities, hand-derived closed-form address formulas of
 * the composed workloads, permutation/fill-count invariants, a hand-worked
 * fixture, and for the GEMM exact-arithmetic special cases plus a float64
 * library matmul.  No function here is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MAX_RANK 8

static int g_threads = 1;

/* Number of threads used for the outermost loop (1 = plain serial loops). */
void oracle_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int oracle_get_threads(void) { return g_threads; }

static int64_t volume(int rank, const int64_t *shape)
{
    int64_t v = 1;
    for (int k = 0; k < rank; ++k) v *= shape[k];
    return v;
}

/* row-major linear offset of multi-index idx in a tensor of the given shape */
static int64_t linearise(int rank, const int64_t *shape, const int64_t *idx)
{
    int64_t off = 0;
    for (int k = 0; k < rank; ++k) off = off * shape[k] + idx[k];
    return off;
}

static void move_elem(const void *in, int64_t in_off, void *out, int64_t out_off, int es)
{
    memcpy((char *)out + out_off * es, (const char *)in + in_off * es, (size_t)es);
}

/* advance idx[1..rank-1] (all dims but the outermost) like an odometer;
 * returns 0 when it wraps around */
static int next_inner(int rank, const int64_t *shape, int64_t *idx)
{
    for (int k = rank - 1; k >= 1; --k) {
        if (++idx[k] < shape[k]) return 1;
        idx[k] = 0;
    }
    return 0;
}

static int inner_nonempty(int rank, const int64_t *shape)
{
    for (int k = 1; k < rank; ++k)
        if (shape[k] <= 0) return 0;
    return 1;
}

static int check_common(int rank, const int64_t *shape, int es)
{
    if (rank < 1 || rank > ORACLE_MAX_RANK) return -1;
    if (es != 2 && es != 4) return -1;
    for (int k = 0; k < rank; ++k)
        if (shape[k] < 0) return -1;
    return 0;
}

/*
 * transpose: out shape e[k] = d[perm[k]];  out[i] = in[j] with j[perm[k]] = i[k].
 * In the paper's affine form f(i) = C i + b, C is a permutation matrix, b = 0.
 */
int oracle_transpose(const void *in, void *out, int rank, const int64_t *d,
                     const int32_t *perm, int es)
{
    if (check_common(rank, d, es)) return -1;
    int seen[ORACLE_MAX_RANK] = {0};
    int64_t e[ORACLE_MAX_RANK];
    for (int k = 0; k < rank; ++k) {
        if (perm[k] < 0 || perm[k] >= rank || seen[perm[k]]) return -2;
        seen[perm[k]] = 1;
        e[k] = d[perm[k]];
    }
    if (volume(rank, e) == 0) return 0;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t i0 = 0; i0 < e[0]; ++i0) {
        int64_t i[ORACLE_MAX_RANK] = {0}, j[ORACLE_MAX_RANK];
        i[0] = i0;
        if (!inner_nonempty(rank, e)) continue;
        do {
            for (int k = 0; k < rank; ++k) j[perm[k]] = i[k];
            move_elem(in, linearise(rank, d, j), out, linearise(rank, e, i), es);
        } while (next_inner(rank, e, i));
    }
    return 0;
}

/*
 * reshape: prod(e) == prod(d).  L = sum_k i_k * prod_{t>k} e[t];
 * j_k = (L div prod_{t>k} d[t]) mod d[k];  out[i] = in[j].
 * A quasi-affine map (floor-div and mod by constants).
 */
int oracle_reshape(const void *in, void *out, int in_rank, const int64_t *d,
                   int out_rank, const int64_t *e, int es)
{
    if (check_common(in_rank, d, es) || check_common(out_rank, e, es)) return -1;
    if (volume(in_rank, d) != volume(out_rank, e)) return -3;
    if (volume(out_rank, e) == 0) return 0;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t i0 = 0; i0 < e[0]; ++i0) {
        int64_t i[ORACLE_MAX_RANK] = {0}, j[ORACLE_MAX_RANK];
        i[0] = i0;
        do {
            int64_t L = linearise(out_rank, e, i);
            int64_t below = 1; /* prod_{t>k} d[t] */
            for (int k = in_rank - 1; k >= 0; --k) {
                j[k] = (L / below) % d[k];
                below *= d[k];
            }
            move_elem(in, linearise(in_rank, d, j), out, L, es);
        } while (next_inner(out_rank, e, i));
    }
    return 0;
}

/*
 * slice on one axis (strided_slice in the paper's operator list, Section 2.1).
 * step >= 1:  0 <= begin < end <= d[axis],  e[axis] = ceil((end - begin) / step);
 * step <= -1: -1 <= end < begin <= d[axis] - 1, e[axis] = ceil((begin - end) / -step)
 * (the axis is walked downwards from begin and stops before end; end = -1
 * means "down to and including index 0").
 * out[.., i, ..] = in[.., begin + i*step, ..].
 * Affine: C = diag(1, .., step, .., 1), b = begin on that axis.
 */
int oracle_slice(const void *in, void *out, int rank, const int64_t *d, int axis,
                 int64_t begin, int64_t end, int64_t step, int es)
{
    if (check_common(rank, d, es)) return -1;
    if (axis < 0 || axis >= rank) return -2;
    int64_t e[ORACLE_MAX_RANK];
    for (int k = 0; k < rank; ++k) e[k] = d[k];
    if (step >= 1) {
        if (begin < 0 || begin >= end || end > d[axis]) return -3;
        e[axis] = (end - begin + step - 1) / step;
    } else if (step <= -1) {
        if (end < -1 || end >= begin || begin > d[axis] - 1) return -3;
        e[axis] = (begin - end + (-step) - 1) / (-step);
    } else {
        return -3;
    }
    if (volume(rank, e) == 0) return 0;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t i0 = 0; i0 < e[0]; ++i0) {
        int64_t i[ORACLE_MAX_RANK] = {0}, j[ORACLE_MAX_RANK];
        i[0] = i0;
        do {
            for (int k = 0; k < rank; ++k) j[k] = i[k];
            j[axis] = begin + i[axis] * step;
            move_elem(in, linearise(rank, d, j), out, linearise(rank, e, i), es);
        } while (next_inner(rank, e, i));
    }
    return 0;
}

/*
 * repeat (Section 2.1 operator list): every index of one axis appears r times
 * in a row.  e[axis] = d[axis] * r;  out[.., i, ..] = in[.., i div r, ..].
 * A non-injective load: the map has a floor-division by the constant r.
 */
int oracle_repeat(const void *in, void *out, int rank, const int64_t *d, int axis,
                  int64_t r, int es)
{
    if (check_common(rank, d, es)) return -1;
    if (axis < 0 || axis >= rank) return -2;
    if (r < 1) return -3;
    int64_t e[ORACLE_MAX_RANK];
    for (int k = 0; k < rank; ++k) e[k] = d[k];
    e[axis] = d[axis] * r;
    if (volume(rank, e) == 0) return 0;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t i0 = 0; i0 < e[0]; ++i0) {
        int64_t i[ORACLE_MAX_RANK] = {0}, j[ORACLE_MAX_RANK];
        i[0] = i0;
        do {
            for (int k = 0; k < rank; ++k) j[k] = i[k];
            j[axis] = i[axis] / r;
            move_elem(in, linearise(rank, d, j), out, linearise(rank, e, i), es);
        } while (next_inner(rank, e, i));
    }
    return 0;
}

/*
 * tile (Section 2.1 operator list): the whole axis is laid out t times one
 * after the other.  e[axis] = d[axis] * t;  out[.., i, ..] = in[.., i mod d[axis], ..].
 * A non-injective load: the map has a remainder by the constant d[axis].
 * Broadcasting an extent-1 axis to t is the case d[axis] = 1.
 */
int oracle_tile(const void *in, void *out, int rank, const int64_t *d, int axis,
                int64_t t, int es)
{
    if (check_common(rank, d, es)) return -1;
    if (axis < 0 || axis >= rank) return -2;
    if (t < 1) return -3;
    int64_t e[ORACLE_MAX_RANK];
    for (int k = 0; k < rank; ++k) e[k] = d[k];
    e[axis] = d[axis] * t;
    if (volume(rank, e) == 0) return 0;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t i0 = 0; i0 < e[0]; ++i0) {
        int64_t i[ORACLE_MAX_RANK] = {0}, j[ORACLE_MAX_RANK];
        i[0] = i0;
        do {
            for (int k = 0; k < rank; ++k) j[k] = i[k];
            j[axis] = i[axis] % d[axis];
            move_elem(in, linearise(rank, d, j), out, linearise(rank, e, i), es);
        } while (next_inner(rank, e, i));
    }
    return 0;
}

/*
 * pad: e[k] = lo[k] + d[k] + hi[k];
 * out[i] = in[i - lo] if lo[k] <= i_k < lo[k] + d[k] for all k, else the fill
 * pattern.  Two store statements into one tensor with disjoint domains: a
 * copy and a constant.
 */
int oracle_pad(const void *in, void *out, int rank, const int64_t *d, const int64_t *lo,
               const int64_t *hi, uint32_t fill_bits, int es)
{
    if (check_common(rank, d, es)) return -1;
    int64_t e[ORACLE_MAX_RANK];
    for (int k = 0; k < rank; ++k) {
        if (lo[k] < 0 || hi[k] < 0) return -3;
        e[k] = lo[k] + d[k] + hi[k];
    }
    if (volume(rank, e) == 0) return 0;
    uint16_t fill16 = (uint16_t)fill_bits;
    const void *fill = es == 2 ? (const void *)&fill16 : (const void *)&fill_bits;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t i0 = 0; i0 < e[0]; ++i0) {
        int64_t i[ORACLE_MAX_RANK] = {0}, j[ORACLE_MAX_RANK];
        i[0] = i0;
        do {
            int inside = 1;
            for (int k = 0; k < rank; ++k) {
                j[k] = i[k] - lo[k];
                if (j[k] < 0 || j[k] >= d[k]) inside = 0;
            }
            int64_t o = linearise(rank, e, i);
            if (inside)
                move_elem(in, linearise(rank, d, j), out, o, es);
            else
                move_elem(fill, 0, out, o, es);
        } while (next_inner(rank, e, i));
    }
    return 0;
}

/*
 * concat of n tensors on one axis: all other extents equal;
 * off_m = sum_{t<m} d_t[axis];  out[.., i, ..] = in_m[.., i - off_m, ..]
 * for off_m <= i < off_{m+1}.  n load/store pairs with disjoint store domains.
 * shapes is an n x rank row-major table.
 */
int oracle_concat(const void *const *ins, int n, void *out, int rank, const int64_t *shapes,
                  int axis, int es)
{
    if (n < 1 || axis < 0 || axis >= rank || rank > ORACLE_MAX_RANK) return -2;
    int64_t e[ORACLE_MAX_RANK];
    for (int k = 0; k < rank; ++k) e[k] = shapes[k];
    e[axis] = 0;
    for (int m = 0; m < n; ++m) {
        const int64_t *d = shapes + (int64_t)m * rank;
        if (check_common(rank, d, es)) return -1;
        for (int k = 0; k < rank; ++k)
            if (k != axis && d[k] != e[k]) return -3;
        e[axis] += d[axis];
    }
    if (volume(rank, e) == 0) return 0;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t i0 = 0; i0 < e[0]; ++i0) {
        int64_t i[ORACLE_MAX_RANK] = {0}, j[ORACLE_MAX_RANK];
        i[0] = i0;
        do {
            int m = 0;
            int64_t off = 0;
            while (i[axis] >= off + shapes[(int64_t)m * rank + axis]) {
                off += shapes[(int64_t)m * rank + axis];
                ++m;
            }
            for (int k = 0; k < rank; ++k) j[k] = i[k];
            j[axis] = i[axis] - off;
            move_elem(ins[m], linearise(rank, shapes + (int64_t)m * rank, j), out,
                      linearise(rank, e, i), es);
        } while (next_inner(rank, e, i));
    }
    return 0;
}

/* bf16 storage bits -> value (bf16 is the upper half of an IEEE binary32) */
static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/*
 * double -> bf16 storage bits, round to nearest, ties to even, done in one
 * step from the double so there is no double rounding.  bf16 has 8
 * significand bits (7 stored) and binary32's exponent range.
 */
static uint16_t double_to_bf16(double x)
{
    if (isnan(x)) return 0x7FC0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7F80;
    int ex;
    (void)frexp(a, &ex);                /* a = m * 2^ex, 0.5 <= m < 1 */
    int e = ex - 1;                     /* a = (2m) * 2^e, 1 <= 2m < 2 */
    if (e < -126) e = -126;             /* subnormal range: fixed quantum 2^-133 */
    double q = ldexp(a, 7 - e);         /* in units of the last place */
    double r = nearbyint(q);            /* default rounding mode: ties to even */
    /* r in [0, 256]; 256 means carry into the next binade */
    int64_t ri = (int64_t)r;
    int64_t bits;
    if (e == -126 && ri < 128) {
        bits = ri;                      /* subnormal (or zero) */
    } else {
        bits = ((int64_t)(e + 127) << 7) + (ri - 128);  /* carry propagates into exponent */
    }
    if (bits >= 0x7F80) bits = 0x7F80;  /* overflow to infinity */
    return sign | (uint16_t)bits;
}

uint16_t oracle_double_to_bf16(double x) { return double_to_bf16(x); }
double oracle_bf16_to_double(uint16_t b) { return bf16_to_double(b); }

/*
 * Consumer GEMM of the rewritten load (Section 2.1): A is the materialised
 * chain output [M,K] (bf16 bits), W is [K,N] row-major (bf16 bits),
 * C[m,n] = bf16_rne( sum_{k=0}^{K-1} A[m,k] * W[k,n] ), products and the sum
 * in float64 in index order k = 0..K-1 (bf16 x bf16 is exact in float64).
 */
int oracle_gemm_bf16(const uint16_t *A, const uint16_t *W, uint16_t *C, int64_t M, int64_t K,
                     int64_t N)
{
    if (M < 0 || K < 0 || N < 0) return -1;
    if (M == 0 || N == 0) return 0;
    int fail = 0;
#pragma omp parallel num_threads(g_threads)
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)N);
        if (!acc) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t m = 0; m < M; ++m) {
                for (int64_t n = 0; n < N; ++n) acc[n] = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    double a = bf16_to_double(A[m * K + k]);
                    for (int64_t n = 0; n < N; ++n) acc[n] += a * bf16_to_double(W[k * N + n]);
                }
                for (int64_t n = 0; n < N; ++n) C[m * N + n] = double_to_bf16(acc[n]);
            }
        }
        free(acc);
    }
    return fail ? -4 : 0;
}

/* one output element of the same GEMM, for sampled checks at full size */
double oracle_gemm_bf16_point(const uint16_t *A, const uint16_t *W, int64_t K, int64_t N,
                              int64_t m, int64_t n)
{
    double acc = 0.0;
    for (int64_t k = 0; k < K; ++k) acc += bf16_to_double(A[m * K + k]) * bf16_to_double(W[k * N + n]);
    return acc;
}
