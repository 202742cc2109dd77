// bf16 GEMM whose A operand is fetched through a composed access map:
//     out[m,n] = bf16( sum_k A[m,k] * W[k,n] ),   A[m,k] = A_src[g(m,k)].
// This is the consumer side of the paper's eq. 4: the load of the GEMM that
// used to read the materialised chain output t_s reads the chain's source t_l
// through g' instead, in its operand-load prologue, and t_s never exists.
//
// Two kernels.  amap_gemm_tile256_kernel (further down) takes the common case of whole 64-element runs along k;
// the general one:
// Kernel shape (gfx950): 256 x 128 output tile per workgroup of 4 wavefronts,
// each wavefront 128 x 64 = 4 x 2 MFMA tiles of v_mfma_f32_32x32x16_bf16 (fp32
// accumulate in 128 AGPRs), K stepped by 64 through one LDS stage with the
// next step prefetched into registers.  Registers (<= 256 per lane) and LDS
// (68 KiB) are sized so that TWO workgroups share a compute unit: while one
// waits at a barrier, refills LDS or runs its epilogue, the other one keeps the
// MFMA pipes busy.  K = 1024 means only 16 steps per tile, so hiding the
// per-tile prologue and epilogue matters as much as the steady-state loop.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>

#include "amap_index.hpp"
#include "amap_plan.hpp"

using namespace amap_dev;
using namespace amap_detail;

namespace {

constexpr int BM = 256, BN = 128, BK = 64;
constexpr int kGemmThreads = 256;
constexpr int kATileBytes = BM * BK * 2;  // 32 KiB
constexpr int kCPitch = BN * 2 + 16;      // bytes per row of the staged output tile (padded against bank conflicts)
constexpr int kLdsBytes = BM * kCPitch;   // 69,632 B: covers the operand stage (48 KiB) and the output stage
constexpr int kMaxDigits = 4;
constexpr int kMaxSeg = 8;  // sources of an A operand gathered along k

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// One dst dimension of the A map written as mixed-radix digits of its index:
// digit j = (x / mult[j]) % ext[j] contributes digit * ss[j] source elements.
struct Digits {
    uint32_t n;
    uint32_t mult[kMaxDigits], ext[kMaxDigits];
    int32_t ss[kMaxDigits];
    FastDiv fmult[kMaxDigits], fext[kMaxDigits];
};

// The k-steps of an operand of the 256 x 256-tile kernel as an odometer over the digits of k, so that the kernel
// moves from one step to the next with a few scalar additions instead of decoding k: level 0 counts the
// 64-element blocks of the contiguous lowest digit, level j >= 1 is digit j.  A step that carries into level j
// (levels below j return to 0, level j goes up by one) moves the operand's address by dl[j] bytes.
struct T2Steps {
    uint32_t e[kMaxDigits - 1];   // extents of levels 0 .. 2 (the top level ends with K)
    int64_t dl[kMaxDigits];
};

// A padded operand (Section 2.1: the load of a pad operator composed into the consumer load): the one
// data piece covers, per dimension, index lo + sum_j i_j * mult[j] with i_j < ext[j]; an index is decoded
// in the radices rad[j] = mult[j + 1] / mult[j] of the PADDED tensor and lies in the piece iff every
// digit stays below the piece's extent.  Everything else reads the pad constant.
struct PadBox {
    uint32_t lo;
    uint32_t rad[kMaxDigits];   // rad of the outermost digit: 0 = unbounded
    FastDiv frad[kMaxDigits];
};

struct GemmArgs {
    const uint16_t *A_src;
    const uint16_t *W;
    uint16_t *C;
    uint32_t M, N, K;
    uint32_t sbase;
    uint32_t tiles_m, tiles_n;
    uint32_t a_row_ss;  // tile256 kernel: source elements between consecutive m inside a 256-row tile
    int64_t a_base;     // tile256 kernel: sbase in 64 bits (its tile and k-step offsets are 64-bit: operands of 2^31 elements and more)
    uint32_t w_row_ss;  // tile256 kernel, W with runs along k (a weight kept as [N,K]): source elements between consecutive n
    T2Steps a_steps, w_steps;   // tile256 kernel: the k-steps of A (and of a W with runs along k) as odometers over the digits of k
    Digits dm, dk;
    // store side (Section 2, eq. "store"): element (m, n) of the product goes to
    // out[obase + om(m) + on(n)]; store_mapped = 0 means the plain row-major C
    uint32_t store_mapped, obase;
    Digits om, on;
    // W read through a map as well: element (k, n) of W is W[wbase + wk(k) + wn(n)]
    uint32_t wbase;
    Digits wk, wn;
    // A gathered from several sources, one per range of k (a concat along the reduction
    // dimension that is never materialised): segment j covers k in [seg_kend[j-1], seg_kend[j])
    // and reads seg_src[j] at seg_sbase[j] + seg_dm[j](m) + seg_dk[j](k - seg_kend[j-1]).
    // n_seg <= 1: the single-source fields above are used instead.
    // A with padding: padded = 1, the data piece's box per dimension, the pad constant (two bf16 per word)
    uint32_t padded, pad_word;
    PadBox pm, pk;
    uint32_t n_seg;
    uint32_t seg_kend[kMaxSeg];
    uint32_t seg_sbase[kMaxSeg];
    const uint16_t *seg_src[kMaxSeg];
    Digits seg_dm[kMaxSeg], seg_dk[kMaxSeg];
};

// How the W operand is fetched: plain row-major [K,N]; through a map whose
// contiguous runs lie along n (same 4 x 8 blocks, transposed in registers); or
// through a map whose runs lie along k (a transposed weight: vectors go to LDS
// as they are, like the A operand).
enum WMode { W_PLAIN = 0, W_MAPPED_N = 1, W_MAPPED_K = 2 };

// How the A operand is fetched: 16-byte runs of the source along k (vectors go to
// LDS as they are), or along m (an operand kept transposed, or a channel-major
// activation feeding a pointwise convolution: 4 k x 8 m blocks, transposed in
// registers like the W operand whose runs lie along n).
enum AMode { A_RUNS_K = 0, A_RUNS_M = 1 };

__device__ __forceinline__ uint32_t digits_offset(const Digits &d, uint32_t x) {
    uint32_t off = 0;
    for (uint32_t j = 0; j < d.n; ++j) {
        const uint32_t q = fdiv(x, d.fmult[j]);
        const uint32_t dig = q - fdiv(q, d.fext[j]) * d.ext[j];
        off += dig * (uint32_t)d.ss[j];
    }
    return off;
}

// index x of a padded dimension -> inside the data piece? and its source offset along that dimension
__device__ __forceinline__ bool padded_offset(const Digits &d, const PadBox &b, uint32_t x, uint32_t &off) {
    off = 0;
    if (x < b.lo) return false;
    const uint32_t y = x - b.lo;
    bool in = true;
    for (uint32_t j = 0; j < d.n; ++j) {
        uint32_t q = fdiv(y, d.fmult[j]);
        if (b.rad[j]) q -= fdiv(q, b.frad[j]) * b.rad[j];
        in = in && q < d.ext[j];
        off += q * (uint32_t)d.ss[j];
    }
    return in;
}

// Byte offset inside an operand tile kept as [row][64 k] bf16 (128 B per row,
// eight 16-byte chunks).  The chunk index is XOR-swizzled with the row so
// that (a) the 32 rows a wavefront reads for one MFMA operand and (b) the
// rows 8 apart that the W transposition writes both spread over the banks.
__device__ __forceinline__ uint32_t tile_offset(uint32_t row, uint32_t chunk) {
    return row * 128u + ((chunk ^ (row & 7u) ^ ((row >> 3) & 7u)) << 4);
}

// r[i] = eight consecutive rows (m or n) of the operand at k = 4 kq + i.  The MFMA wants, per
// row, consecutive k: transpose the 4 x 8 block of 16-bit values in registers and write
// 8 bytes (4 k) per row of the stage.
__device__ __forceinline__ void store_transposed(char *stage, const u32x4 *r, uint32_t row0, uint32_t kq) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t a0 = r[0][j >> 1], a1 = r[1][j >> 1], a2 = r[2][j >> 1], a3 = r[3][j >> 1];
        u32x2 o;
        o.x = (j & 1) ? ((a0 >> 16) | (a1 & 0xFFFF0000u)) : ((a0 & 0xFFFFu) | (a1 << 16));
        o.y = (j & 1) ? ((a2 >> 16) | (a3 & 0xFFFF0000u)) : ((a2 & 0xFFFFu) | (a3 << 16));
        *reinterpret_cast<u32x2 *>(stage + tile_offset(row0 + j, kq >> 1) + (kq & 1u) * 8u) = o;
    }
}

// two fp32 -> two bf16 (round to nearest even; the hardware conversion of gfx950)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Workgroup index -> output tile.  Workgroups go to the 8 XCDs round-robin;
// each XCD gets a compact 2-D block of tiles so that the A rows and W columns
// its workgroups share are fetched into that XCD's L2 once.
__host__ __device__ __forceinline__ void tile_of_block(uint32_t b, uint32_t tiles_m, uint32_t tiles_n, uint32_t &tm, uint32_t &tn) {
    if ((tiles_m & 3u) == 0 && (tiles_n & 1u) == 0) {
        const uint32_t xcd = b & 7u, j = b >> 3;        // j-th tile of this XCD
        const uint32_t rm = tiles_m >> 2, rn = tiles_n >> 1;  // region extents: 4 x 2 regions
        const uint32_t xm = xcd >> 1, xn = xcd & 1u;
        tm = xm * rm + j % rm;
        tn = xn * rn + j / rm;
    } else {
        tm = b % tiles_m;
        tn = b / tiles_m;
    }
}

// EDGE: M, N or K is not a whole number of tiles.  Rows past M are clamped for the
// loads and skipped by the stores, vectors past K or N are replaced by zeros, so the
// extra lanes neither read outside the operands nor contribute to a kept result.
// SEG: A is gathered from several sources along k (its own instances: the extra
// bookkeeping in the load path costs the single-source kernels 4-6 % when it is a run-time branch).
template <int AM, int WM, bool EDGE, bool SEG>
__global__ __launch_bounds__(kGemmThreads, 2) void amap_gemm_kernel(const GemmArgs g) {
    extern __shared__ uint4 smem_v[];
    char *smem = reinterpret_cast<char *>(smem_v);
    char *const sa = smem;                // A stage: [256 rows][64 k]
    char *const sw = smem + kATileBytes;  // W stage: [128 n][64 k], 16 KiB
    const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    uint32_t tm, tn;
    tile_of_block(blockIdx.x, g.tiles_m, g.tiles_n, tm, tn);
    const uint32_t m0 = tm * BM, n0 = tn * BN;

    // ---- A prologue assignment.  Runs along k: 8 vectors of 8 k per lane and step,
    // vector v = tid + 256 i -> row v / 8 of the tile, k chunk v % 8.  Runs along m: two
    // 4 k x 8 m blocks per lane and step, m block tid % 32, k rows 4 (tid / 32 + 8 h) + i.
    const uint32_t a_chunk = tid & 7u;
    const uint32_t a_mb = tid & 31u, a_kq = tid >> 5;
    const bool a_m_ok = !EDGE || m0 + a_mb * 8u < g.M;  // this lane's 8 m of A exist
    uint32_t a_soff[8];
    constexpr bool segmented = SEG;
    // state of the segmented load stream (runs along k): current segment, its first k, its source
    uint32_t cur_seg = 0, seg_klo = 0;
    const uint16_t *a_base = segmented ? g.seg_src[0] : g.A_src;
    auto a_rows_of_segment = [&](uint32_t sg) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t row = m0 + (tid >> 3) + 32u * i;
            if constexpr (EDGE) row = row < g.M ? row : g.M - 1;
            if (EDGE && !segmented && g.padded) {
                uint32_t off;   // (a source of < 2^31 elements: no offset reaches the mark of a row outside the data piece)
                a_soff[i] = padded_offset(g.dm, g.pm, row, off) ? g.sbase + off : 0xFFFFFFFFu;
            } else {
                a_soff[i] = segmented ? g.seg_sbase[sg] + digits_offset(g.seg_dm[sg], row) : g.sbase + digits_offset(g.dm, row);
            }
        }
    };
    if constexpr (AM == A_RUNS_K) {
        a_rows_of_segment(0);
    } else if constexpr (!segmented) {
        a_soff[0] = g.sbase + digits_offset(g.dm, a_m_ok ? m0 + a_mb * 8u : 0u);
    }
    // ---- W assignment: one 4 k x 8 n block per lane and step (runs along n), or
    // four vectors of 8 k for n rows tid / 8 + 32 i (runs along k)
    const uint32_t w_nb = tid & 15u, w_kq = tid >> 4;
    const uint16_t *w_ptr = g.W + (size_t)(w_kq * 4u) * g.N + n0 + w_nb * 8u;
    uint32_t w_noff[4] = {0, 0, 0, 0};
    const bool w_n_ok = !EDGE || n0 + w_nb * 8u < g.N;  // this lane's 8 n of W exist
    if constexpr (WM == W_MAPPED_N) w_noff[0] = g.wbase + digits_offset(g.wn, w_n_ok ? n0 + w_nb * 8u : 0u);
    if constexpr (WM == W_MAPPED_K) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t n = n0 + (tid >> 3) + 32u * i;
            if constexpr (EDGE) n = n < g.N ? n : g.N - 1;
            w_noff[i] = g.wbase + digits_offset(g.wn, n);
        }
    }

    u32x4 ra[8], rw[4];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    auto load_step = [&](uint32_t k0) {
        const uint32_t kc = k0 + a_chunk * 8u;
        const bool kc_ok = !EDGE || kc < g.K;
        if constexpr (AM == A_RUNS_K) {
            uint32_t koff;
            if constexpr (segmented) {
                // segment ends are multiples of BK, so a whole step reads one source; steps come in
                // increasing k, so the segment index only moves forward
                uint32_t sg = cur_seg;
                while (sg + 1 < g.n_seg && k0 >= g.seg_kend[sg]) ++sg;
                if (sg != cur_seg) {
                    cur_seg = sg;
                    seg_klo = g.seg_kend[sg - 1];
                    a_base = g.seg_src[sg];
                    a_rows_of_segment(sg);
                }
                koff = digits_offset(g.seg_dk[sg], kc_ok ? kc - seg_klo : 0u);
            } else if (EDGE && g.padded) {
                // vectors past K are zero (they meet zero rows of W); vectors outside the data piece hold the pad constant
                // (every lane loads: one outside the piece reads the piece's first vector and drops it)
                const bool k_in = padded_offset(g.dk, g.pk, kc_ok ? kc : 0u, koff) && kc_ok;
                const uint32_t c = kc_ok ? g.pad_word : 0u;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const bool in = k_in && a_soff[i] != 0xFFFFFFFFu;
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(a_base + (size_t)(in ? a_soff[i] + koff : g.sbase));
                    ra[i] = in ? v : u32x4{c, c, c, c};
                }
                koff = 0;
            } else {
                koff = digits_offset(g.dk, kc_ok ? kc : 0u);
            }
            if (!(EDGE && !segmented && g.padded)) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    ra[i] = kc_ok ? *reinterpret_cast<const u32x4 *>(a_base + (size_t)(a_soff[i] + koff)) : zero4;
            }
        } else if constexpr (!segmented) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t k = k0 + 4u * (a_kq + 8u * (i >> 2)) + (i & 3);
                const bool ok = !EDGE || (a_m_ok && k < g.K);
                ra[i] = ok ? *reinterpret_cast<const u32x4 *>(g.A_src + (size_t)(a_soff[0] + digits_offset(g.dk, ok ? k : 0u))) : zero4;
            }
        } else {
            // segment ends are multiples of 32: each half of the step (h) reads one source
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t kb = k0 + 32u * h;
                uint32_t sg = 0;
                while (sg + 1 < g.n_seg && kb >= g.seg_kend[sg]) ++sg;
                const uint32_t klo = sg ? g.seg_kend[sg - 1] : 0u;
                const uint16_t *base = g.seg_src[sg];
                // this lane's 8 m in that source (decoded per half-step: registers are short here)
                const uint32_t off = g.seg_sbase[sg] + digits_offset(g.seg_dm[sg], a_m_ok ? m0 + a_mb * 8u : 0u);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t k = kb + 4u * a_kq + i;
                    const bool ok = !EDGE || (a_m_ok && k < g.K);
                    ra[4 * h + i] =
                        ok ? *reinterpret_cast<const u32x4 *>(base + (size_t)(off + digits_offset(g.seg_dk[sg], ok ? k - klo : 0u))) : zero4;
                }
            }
        }
        if constexpr (WM == W_PLAIN) {
            const uint16_t *w = w_ptr + (size_t)k0 * g.N;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool ok = !EDGE || (w_n_ok && k0 + w_kq * 4u + i < g.K);
                rw[i] = ok ? *reinterpret_cast<const u32x4 *>(w + (size_t)i * g.N) : zero4;
            }
        } else if constexpr (WM == W_MAPPED_N) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t k = k0 + w_kq * 4u + i;
                const bool ok = !EDGE || (w_n_ok && k < g.K);
                rw[i] = ok ? *reinterpret_cast<const u32x4 *>(g.W + (size_t)(w_noff[0] + digits_offset(g.wk, k))) : zero4;
            }
        } else {
            const uint32_t wkoff = digits_offset(g.wk, kc_ok ? kc : 0u);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                rw[i] = kc_ok ? *reinterpret_cast<const u32x4 *>(g.W + (size_t)(w_noff[i] + wkoff)) : zero4;
        }
    };
    auto store_step = [&]() {
        if constexpr (AM == A_RUNS_K) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                *reinterpret_cast<u32x4 *>(sa + tile_offset((tid >> 3) + 32u * i, a_chunk)) = ra[i];
        } else {
            store_transposed(sa, ra, a_mb * 8u, a_kq);
            store_transposed(sa, ra + 4, a_mb * 8u, a_kq + 8u);
        }
        if constexpr (WM == W_MAPPED_K) {
            // already 8 consecutive k per n row: straight into the stage
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *reinterpret_cast<u32x4 *>(sw + tile_offset((tid >> 3) + 32u * i, a_chunk)) = rw[i];
            return;
        }
        // rw[i] = W[k = 4 kq + i][n = 8 nb .. 8 nb + 7]
        store_transposed(sw, rw, w_nb * 8u, w_kq);
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const uint32_t wm = wave >> 1, wn = wave & 1u;
    const uint32_t frag_row = lane & 31u, frag_half = lane >> 5;
    const uint32_t steps = (g.K + BK - 1) / BK;

    load_step(0);
    store_step();
    __syncthreads();
    if (steps > 1) load_step(BK);
    for (uint32_t s = 0; s < steps; ++s) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 fa[4], fb[2];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                fa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(
                                                       sa + tile_offset(wm * 128u + i * 32u + frag_row, 2u * kk + frag_half)));
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(
                                                       sw + tile_offset(wn * 64u + j * 32u + frag_row, 2u * kk + frag_half)));
            // W fragment as the row operand, A fragment as the column operand:
            // the 32 x 32 result tile is C^T, so that a lane ends up with four
            // consecutive n of one output row m (8 contiguous bytes of C)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
        __syncthreads();  // every wavefront is done reading this step's stage
        if (s + 1 < steps) {
            store_step();
            if (s + 2 < steps) load_step((s + 2) * BK);
            __syncthreads();
        }
    }

    // ---- epilogue: round to bf16 and stage the 256 x 128 tile in LDS, then
    // write whole 256-byte rows with 16-byte stores.
    // Accumulator v of a transposed 32 x 32 tile in lane l: m = l % 32,
    // n = 8 (v / 4) + 4 (l / 32) + v % 4.
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t row = wm * 128u + i * 32u + frag_row;
                const uint32_t col = wn * 64u + j * 32u + 8u * q + 4u * frag_half;
                u32x2 o;
                o.x = pack_bf16(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
                o.y = pack_bf16(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                *reinterpret_cast<u32x2 *>(smem + row * kCPitch + col * 2) = o;
            }
    __syncthreads();
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const uint32_t v = tid + 256u * i, row = v >> 4, cv = v & 15u;
        const u32x4 x = *reinterpret_cast<const u32x4 *>(smem + row * kCPitch + cv * 16);
        if constexpr (EDGE) {
            if (m0 + row >= g.M || n0 + cv * 8u >= g.N) continue;
        }
        size_t off = (size_t)(m0 + row) * g.N + n0 + cv * 8u;
        if (g.store_mapped) off = g.obase + digits_offset(g.om, m0 + row) + digits_offset(g.on, n0 + cv * 8u);
        __builtin_nontemporal_store(x, reinterpret_cast<u32x4 *>(g.C + off));
    }
}

// ---------------------------------------------------------------------------------------------
// The common case: K % 64 = 0, K >= 128, one source with its runs along k, a tile's 256 rows inside one
// digit of m and a k-step inside one digit of k, W row-major or kept as [N,K] with the same properties
// (W_KM); M and N whole numbers of tiles or not (EDGE).
// Same consumer load of eq. 4, different machine mapping:
//   * 256 x 256 output tile per workgroup of 4 wavefronts (128 x 128 each: 16 MFMA tiles, 256
//     accumulator registers), one workgroup per compute unit, persistent over its tiles;
//   * both operands go from global memory straight into LDS (global_load_lds, 16 bytes per lane,
//     no staging registers, no LDS-write instructions); the lane -> address permutation applies the
//     bank swizzle on the global side because such a load always fills 1 KiB of LDS in lane order;
//   * W stays [k][n] in LDS and is read with the transposing LDS read (ds_read_b64_tr_b16), which
//     hands every lane four consecutive k of one n: the MFMA operand layout without a register transpose;
//   * two LDS stages of 64 k whose halves (A, W) are refilled half a step apart: W's fragments are read
//     three quarters of a step ahead of the MFMAs, A's one quarter, so W of step s + 2 goes out after the
//     first quarter of step s and A of step s + 2 after the third, two batches are in flight at any time,
//     and the first loads of the workgroup's next tile are in flight while the current tile is written out;
//   * every memory instruction sits at a fixed place between two MFMAs (scheduling barriers pin the
//     order): one LDS read, or one LDS read and one load, per MFMA.
constexpr int T2M = 256, T2N = 256, T2K = 64;
constexpr int kT2Stage = 65536;            // A [256 rows][64 k] + W [64 k][256 n]
constexpr int kT2WOff = 32768;             // W part of a stage
constexpr int kT2Scratch = 2 * kT2Stage;   // output staging, 8 KiB per wavefront
constexpr int kT2Lds = kT2Scratch + 32768; // 160 KiB: all of a compute unit's LDS

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const u32x4 lds_u32x4;

// all digits of one dimension, fixed trip count (unused digits have extent 1 and stride 0)
__host__ __device__ __forceinline__ uint32_t digits_offset4(const Digits &d, uint32_t x) {
    uint32_t off = 0;
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
#endif
    for (uint32_t j = 0; j < (uint32_t)kMaxDigits; ++j) {
        const uint32_t q = fdiv(x, d.fmult[j]);
        const uint32_t dig = q - fdiv(q, d.fext[j]) * d.ext[j];
        off += dig * (uint32_t)d.ss[j];
    }
    return off;
}

// 16 bytes per lane from global memory straight into LDS: lane i lands at lds_base + 16 i
__device__ __forceinline__ void load_to_lds16(const void *base, uint32_t byte_off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_base) : "memory");
}

#define AMAP_PIN() __builtin_amdgcn_sched_barrier(0)

// ---- global addressing of amap_gemm_tile256_kernel, shared with its host replay (amap_gemm_selfcheck)
// The load cursor: the (tile, k-step) the next batch of 16 loads per wavefront fetches.  It runs two k-steps
// ahead of the MFMAs and crosses into the workgroup's next tile (tile + number of workgroups) on its own.
struct T2Cursor {
    uint32_t tile, k0;
};
__host__ __device__ __forceinline__ bool t2_cursor_advance(T2Cursor &c, uint32_t K, uint32_t n_workgroups) {
    c.k0 += (uint32_t)T2K;
    if (c.k0 < K) return false;
    c.k0 = 0;
    c.tile += n_workgroups;
    return true;  // a new tile: its bases must be recomputed (if it exists)
}
// Per-lane byte offsets inside a tile and k-step, for the load blocks of even / odd index (par).
// A stage: 1 KiB block b = rows 8 b .. 8 b + 7, 128 B each; lane i of the load holds row 8 b + i / 8,
// physical chunk i % 8 = logical chunk ^ ((row >> 1) & 7).  W stage: block b = k rows 2 b, 2 b + 1,
// 512 B each; lane i holds row 2 b + i / 32, physical chunk i % 32 = logical chunk ^ ((k & 3) << 2).
// Wavefront w issues blocks 8 w .. 8 w + 7 of both.
__host__ __device__ __forceinline__ uint32_t t2_a_lane(const GemmArgs &g, uint32_t wave, uint32_t lane, uint32_t par) {
    const uint32_t a_chunk0 = (lane & 7u) ^ (lane >> 4);
    return 2u * ((64u * wave + (lane >> 3)) * g.a_row_ss + 8u * (a_chunk0 ^ (par << 2)));
}
// (W_KM: W's runs lie along k, a weight kept as [N,K] read through a transpose map: its stage is laid out like A's, rows = n)
template <bool W_KM>
__host__ __device__ __forceinline__ uint32_t t2_w_lane(const GemmArgs &g, uint32_t wave, uint32_t lane, uint32_t par) {
    if constexpr (W_KM) {
        const uint32_t chunk0 = (lane & 7u) ^ (lane >> 4);
        return 2u * ((64u * wave + (lane >> 3)) * g.w_row_ss + 8u * (chunk0 ^ (par << 2)));
    }
    const uint32_t w_kr = lane >> 5;
    return 2u * ((16u * wave + w_kr) * g.N + 8u * ((lane & 31u) ^ (w_kr << 2) ^ (par << 3)));
}
// Wave-uniform byte offsets of a tile, and of a k-step inside it: 64-bit, added to the operand's pointer in
// scalar registers, so that operands of 2^31 elements and more are within reach; what a lane adds (below) is a
// non-negative 32-bit offset inside the tile's rows of one k-step.
__host__ __device__ __forceinline__ int64_t digits_offset4_wide(const Digits &d, uint32_t x) {
    int64_t off = 0;
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
#endif
    for (uint32_t j = 0; j < (uint32_t)kMaxDigits; ++j) {
        const uint32_t q = fdiv(x, d.fmult[j]);
        const uint32_t dig = q - fdiv(q, d.fext[j]) * d.ext[j];
        off += (int64_t)dig * (int64_t)d.ss[j];
    }
    return off;
}
template <bool W_KM>
__host__ __device__ __forceinline__ void t2_tile_bases(const GemmArgs &g, uint32_t tile, int64_t &a_tile, int64_t &w_tile) {
    uint32_t tm, tn;
    tile_of_block(tile, g.tiles_m, g.tiles_n, tm, tn);
    a_tile = 2 * (g.a_base + digits_offset4_wide(g.dm, tm * (uint32_t)T2M));
    if constexpr (W_KM)
        w_tile = 2 * ((int64_t)g.wbase + digits_offset4_wide(g.wn, tn * (uint32_t)T2N));
    else
        w_tile = 2 * (int64_t)(tn * (uint32_t)T2N);
}
// the odometer of an operand whose lowest digit of k is contiguous and a whole number of 64-element steps
__host__ inline T2Steps t2_steps_of(const Digits &d) {
    T2Steps s;
    const int64_t st[kMaxDigits] = {(int64_t)T2K, d.ss[1], d.ss[2], d.ss[3]};
    const uint32_t e[kMaxDigits] = {d.ext[0] / (uint32_t)T2K, d.ext[1], d.ext[2], d.ext[3]};
    int64_t back = 0;   // from the last step of the levels below to their first one
    for (int j = 0; j < kMaxDigits; ++j) {
        s.dl[j] = 2 * (st[j] - back);
        back += (int64_t)(e[j] - 1u) * st[j];
        if (j + 1 < kMaxDigits) s.e[j] = e[j];
    }
    return s;
}
// plain row-major W[K,N]: one level, 64 rows of N elements per step
__host__ inline T2Steps t2_steps_plain_w(uint32_t K, uint32_t N) {
    T2Steps s;
    s.e[0] = K / (uint32_t)T2K;
    s.e[1] = s.e[2] = 1;
    for (int j = 0; j < kMaxDigits; ++j) s.dl[j] = 2 * (int64_t)T2K * (int64_t)N;
    return s;
}
// counters of levels 0 .. 2 of one operand's odometer; all 0 at the first k-step of a tile
struct T2Odo {
    uint32_t c0, c1, c2;
};
// one k-step on: the byte delta to the next step's base (not called at the last step of a tile)
__host__ __device__ __forceinline__ int64_t t2_odo_advance(T2Odo &o, const T2Steps &s) {
    if (++o.c0 < s.e[0]) return s.dl[0];
    o.c0 = 0;
    if (++o.c1 < s.e[1]) return s.dl[1];
    o.c1 = 0;
    if (++o.c2 < s.e[2]) return s.dl[2];
    o.c2 = 0;
    return s.dl[3];
}
// The load stream of a workgroup: its cursor, the byte offsets of the cursor's tile in both operands and of the
// cursor's k-step inside the tile's rows, and the odometers that move the latter.
struct T2Stream {
    T2Cursor c;
    int64_t a_tile, w_tile, a_step, w_step;
    T2Odo ao, wo;
};
// the cursor's tile has changed (and exists): its bases, first k-step
template <bool W_KM>
__host__ __device__ __forceinline__ void t2_stream_tile(const GemmArgs &g, T2Stream &st) {
    t2_tile_bases<W_KM>(g, st.c.tile, st.a_tile, st.w_tile);
    st.a_step = st.w_step = 0;
    st.ao = st.wo = T2Odo{0, 0, 0};
}
// one k-step on, into the workgroup's next tile after the last step of a tile; true if that was a tile change.
// (g_tile: the same arguments as g, for what only the start of a tile reads; see t2_args_again)
template <bool W_KM>
__host__ __device__ __forceinline__ bool t2_stream_next(const GemmArgs &g, const GemmArgs &g_tile, T2Stream &st, uint32_t n_workgroups, uint32_t ntiles) {
    if (t2_cursor_advance(st.c, g.K, n_workgroups)) {
        if (st.c.tile < ntiles) t2_stream_tile<W_KM>(g_tile, st);
        return true;
    }
    st.a_step += t2_odo_advance(st.ao, g.a_steps);
    st.w_step += t2_odo_advance(st.wo, g.w_steps);
    return false;
}
// a lane's byte offset for load block j (0 .. 7) of its wavefront, from the k-step's base
__host__ __device__ __forceinline__ uint32_t t2_a_load(const GemmArgs &g, uint32_t a_lane_par, uint32_t j) {
    return a_lane_par + 16u * j * g.a_row_ss;
}
template <bool W_KM>
__host__ __device__ __forceinline__ uint32_t t2_w_load(const GemmArgs &g, uint32_t w_lane_par, uint32_t j) {
    if constexpr (W_KM) return w_lane_par + 16u * j * g.w_row_ss;
    return w_lane_par + 4u * j * g.N;
}
// EDGE instances (M or N no multiple of 256): the rows / columns of a tile that exist; a lane whose row or column
// lies past them loads the last existing one instead (its LDS slot then holds a copy of valid data, which only
// reaches accumulators of rows / columns that are never stored), so no load leaves the operands.
__host__ __device__ __forceinline__ uint32_t t2_rows_valid(const GemmArgs &g, uint32_t tm) {
    const uint32_t left = g.M - tm * (uint32_t)T2M;
    return left < (uint32_t)T2M ? left : (uint32_t)T2M;
}
__host__ __device__ __forceinline__ uint32_t t2_cols_valid(const GemmArgs &g, uint32_t tn) {
    const uint32_t left = g.N - tn * (uint32_t)T2N;
    return left < (uint32_t)T2N ? left : (uint32_t)T2N;
}
// rv: t2_rows_valid of the tile
__host__ __device__ __forceinline__ uint32_t t2_a_load_edge(const GemmArgs &g, uint32_t wave, uint32_t lane, uint32_t j, uint32_t rv) {
    uint32_t row = 64u * wave + (lane >> 3) + 8u * j;
    row = row < rv ? row : rv - 1u;
    const uint32_t chunk = (lane & 7u) ^ (lane >> 4) ^ ((j & 1u) << 2);
    return 2u * (row * g.a_row_ss + 8u * chunk);
}
// cv: t2_cols_valid of the tile (a multiple of 8)
template <bool W_KM>
__host__ __device__ __forceinline__ uint32_t t2_w_load_edge(const GemmArgs &g, uint32_t wave, uint32_t lane, uint32_t j, uint32_t cv) {
    if constexpr (W_KM) {
        uint32_t row = 64u * wave + (lane >> 3) + 8u * j;
        row = row < cv ? row : cv - 1u;
        const uint32_t chunk = (lane & 7u) ^ (lane >> 4) ^ ((j & 1u) << 2);
        return 2u * (row * g.w_row_ss + 8u * chunk);
    }
    const uint32_t w_kr = lane >> 5;
    uint32_t chunk = (lane & 31u) ^ (w_kr << 2) ^ ((j & 1u) << 3);
    const uint32_t last = (cv >> 3) - 1u;
    chunk = chunk < last ? chunk : last;
    return 2u * ((16u * wave + w_kr + 2u * j) * g.N + 8u * chunk);
}
// epilogue: element offset in out of the 8 values a lane stores for row m, first column n_lane
template <bool MAPPED>
__host__ __device__ __forceinline__ size_t t2_store_col(const GemmArgs &g, uint32_t n_lane) {
    if constexpr (MAPPED) return (size_t)(g.obase + digits_offset4(g.on, n_lane));
    return (size_t)n_lane;
}
template <bool MAPPED>
__host__ __device__ __forceinline__ size_t t2_store_off(const GemmArgs &g, size_t col_off, uint32_t m) {
    if constexpr (MAPPED) return col_off + digits_offset4(g.om, m);
    return (size_t)m * g.N + col_off;
}

// Workgroups of the persistent grid: as many as give every one the same number of tiles (288 tiles on 256 compute
// units: 144 workgroups of two tiles each, not 256 of which 32 run a second tile while the others idle; the product
// runs at the power limit, and the busy part of the chip then clocks higher: 46.9 -> 44.4 us on that shape).
inline uint32_t t2_workgroups(uint32_t ntiles, uint32_t n_compute_units) {
    const uint32_t rounds = (ntiles + n_compute_units - 1) / n_compute_units;
    return (ntiles + rounds - 1) / rounds;
}

// The kernel's argument block, read from the argument segment again at the place of use: what only the start of a
// tile or its epilogue needs (the digits of m and n of both operands and of the store) then occupies no scalar
// registers during the k-loop.  Left to itself the compiler loads every field once at the top of the kernel and
// keeps it, and spills scalar registers inside the loop.  (The block is the kernel's only argument: offset 0.)
__device__ __forceinline__ const GemmArgs &t2_args_again() {
    auto p = (const __attribute__((address_space(4))) GemmArgs *)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(p));
    return *(const GemmArgs *)p;
}

template <bool STORE_MAPPED, bool W_KM, bool EDGE>
__global__ __launch_bounds__(kGemmThreads, 1) void amap_gemm_tile256_kernel(const GemmArgs g) {
    const uint32_t tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t wm = wave >> 1, wn = wave & 1u;
    const uint32_t steps = g.K / T2K;  // >= 2
    const uint32_t ntiles = g.tiles_m * g.tiles_n;

    // ---- load stream (see T2Stream) and the per-lane parts of the load addresses
    T2Stream ld = {};
    ld.c = T2Cursor{blockIdx.x, 0};
    uint32_t a_lane[2], w_lane[2];   // per-lane byte offsets, block parity 0 / 1
#pragma unroll
    for (uint32_t par = 0; par < 2; ++par) {
        a_lane[par] = t2_a_lane(g, wave, lane, par);
        w_lane[par] = t2_w_lane<W_KM>(g, wave, lane, par);
    }
    uint32_t ld_rv = (uint32_t)T2M, ld_cv = (uint32_t)T2N;   // EDGE: existing rows / columns of the cursor's tile
    auto cursor_edges = [&]() __attribute__((always_inline)) {
        if constexpr (EDGE) {
            uint32_t tm, tn;
            tile_of_block(ld.c.tile, g.tiles_m, g.tiles_n, tm, tn);
            ld_rv = t2_rows_valid(g, tm);
            ld_cv = t2_cols_valid(g, tn);
        }
    };
    const char *ka = nullptr, *wk = nullptr;   // the operands at the cursor's tile and k-step
    auto loads_begin = [&]() __attribute__((always_inline)) {
        ka = reinterpret_cast<const char *>(g.A_src) + (ld.a_tile + ld.a_step);
        wk = reinterpret_cast<const char *>(g.W) + (ld.w_tile + ld.w_step);
    };
    auto load_one = [&](uint32_t stage_base, int j, int which) __attribute__((always_inline)) {
        if (which == 0)
            load_to_lds16(ka, EDGE ? t2_a_load_edge(g, wave, lane, (uint32_t)j, ld_rv) : t2_a_load(g, a_lane[j & 1], (uint32_t)j),
                          stage_base + (wave * 8u + j) * 1024u);
        else
            load_to_lds16(wk, EDGE ? t2_w_load_edge<W_KM>(g, wave, lane, (uint32_t)j, ld_cv) : t2_w_load<W_KM>(g, w_lane[j & 1], (uint32_t)j),
                          stage_base + kT2WOff + (wave * 8u + j) * 1024u);
    };
    // the stream moves on by one k-step (a few scalar additions); in a new tile that exists its bases are recomputed
    auto cursor_next = [&]() __attribute__((always_inline)) {
        if (t2_stream_next<W_KM>(g, t2_args_again(), ld, gridDim.x, ntiles) && ld.c.tile < ntiles) cursor_edges();
    };

    // ---- fragment addresses (bytes from the start of a stage)
    // A: row 128 wm + 32 i + lane % 32, logical chunk 2 kk + lane / 32
    const uint32_t fa_addr0 = wm * 16384u + (lane & 31u) * 128u + (((lane >> 5) ^ ((lane >> 1) & 7u)) << 4);
    // W: lane = 16 g + s supplies the 8 bytes at k = 16 kk + 8 (g >> 1) + s / 4 (+ 4), n = 128 wn + 32 jn + 16 (g & 1) + 4 (s % 4)
    // and receives k = 16 kk + 8 (lane / 32) .. + 3 (+ 4) of n = 128 wn + 32 jn + lane % 32
    const uint32_t gq = lane >> 4, sq = lane & 15u;
    const uint32_t fw_base = kT2WOff + (8u * (gq >> 1) + (sq >> 2)) * 512u + wn * 256u + (2u * (gq & 1u) + ((sq >> 1) & 1u)) * 16u + (sq & 1u) * 8u;
    uint32_t fw_addr[4];
#pragma unroll
    for (int jn = 0; jn < 4; ++jn) fw_addr[jn] = fw_base + (((uint32_t)jn ^ ((sq >> 2) & 3u)) << 6);

    // W with runs along k: its stage is laid out like A's (row = n), and so are its fragments:
    // row 128 wn + 32 jn + lane % 32, logical chunk 2 kk + lane / 32
    const uint32_t fb_addr0 = kT2WOff + wn * 16384u + (lane & 31u) * 128u + (((lane >> 5) ^ ((lane >> 1) & 7u)) << 4);

    f32x16 acc[4][4];
    bf16x8 fa[2][4];                      // A fragments: two sets, read one k sub-step ahead
    bf16x4 fbl[4][4], fbh[4][4];          // W fragments: four sets, read three sub-steps ahead (see the k-loop)
    bf16x8 fbk[4][4];
    auto mf = [&](int aset, int wset, int i, int jn) __attribute__((always_inline)) {
        bf16x8 b;
        if constexpr (W_KM)
            b = fbk[wset][jn];
        else
            b = __builtin_shufflevector(fbl[wset][jn], fbh[wset][jn], 0, 1, 2, 3, 4, 5, 6, 7);
        // W fragment as the row operand: the 32 x 32 result is C^T, a lane holds four consecutive n of one row m
        acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, fa[aset][i], acc[i][jn], 0, 0, 0);
    };
    // the fragment reads of a k sub-step: 4 of A, 8 of W (4 of W when its runs lie along k)
    auto rd_a = [&](int set, uint32_t stage_base, int kk, int r) __attribute__((always_inline)) {
        fa[set][r] = __builtin_bit_cast(bf16x8, *reinterpret_cast<lds_u32x4 *>(stage_base + (fa_addr0 ^ ((uint32_t)kk << 5)) + r * 4096u));
    };
    auto rd_w = [&](int set, uint32_t stage_base, int kk, int r) __attribute__((always_inline)) {
        if constexpr (W_KM) {
            if (r < 4)
                fbk[set][r] = __builtin_bit_cast(bf16x8, *reinterpret_cast<lds_u32x4 *>(stage_base + (fb_addr0 ^ ((uint32_t)kk << 5)) + r * 4096u));
        } else {
            const uint32_t a = stage_base + fw_addr[r >> 1] + kk * 8192u + ((r & 1) ? 2048u : 0u);
            const bf16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(reinterpret_cast<__attribute__((address_space(3))) bf16x4 *>(a));
            if (r & 1)
                fbh[set][r >> 1] = v;
            else
                fbl[set][r >> 1] = v;
        }
    };
    // 16 MFMAs of one k sub-step on A set `aset` and W set `wset`.  Under them, one per MFMA: the 4 reads of A's
    // next sub-step (into the other A set), the 8 reads of the W sub-step three ahead (into the W set before
    // `wset`), and, with `which` = 1 / 2, the 8 loads per wavefront of the stream's k-step of W / of A.
    // (One code path for all cases: an MFMA sequence in two arms of a branch makes the compiler copy the
    // accumulators; and no branch around a load: 16 branches per k-step cost more than the loads.)
    auto phase = [&](int aset, int wset, uint32_t a_stage, int a_kk, uint32_t w_stage, int w_kk, uint32_t ld_stage, int which) __attribute__((always_inline)) {
        if (which == 1) wk = reinterpret_cast<const char *>(g.W) + (ld.w_tile + ld.w_step);
        if (which == 2) ka = reinterpret_cast<const char *>(g.A_src) + (ld.a_tile + ld.a_step);
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            mf(aset, wset, s >> 2, s & 3);
            if (s < 4) rd_a(aset ^ 1, a_stage, a_kk, s);
            if (s >= 4 && s < 12) rd_w((wset + 3) & 3, w_stage, w_kk, s - 4);
            if (which != 0 && (s & 1) == 0) load_one(ld_stage, s >> 1, which == 1 ? 1 : 0);
            AMAP_PIN();
        }
    };
    uint32_t cur = 0;
    if (ld.c.tile < ntiles) {
        t2_stream_tile<W_KM>(t2_args_again(), ld);
        cursor_edges();
        // the first two k-steps (K >= 2 steps: both lie in the first tile); of the second one W first, then A:
        // the order in which the k-loop waits for them
        loads_begin();
#pragma unroll
        for (int s = 0; s < 16; ++s) load_one(0, s >> 1, s & 1);
        // (with K = 2 k-steps the second advance already moves the cursor to the workgroup's next tile;
        // a cursor left at k = K would fetch weight rows past the end of W)
        cursor_next();
        loads_begin();
#pragma unroll
        for (int j = 0; j < 8; ++j) load_one(kT2Stage, j, 1);
#pragma unroll
        for (int j = 0; j < 8; ++j) load_one(kT2Stage, j, 0);
        cursor_next();
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");   // the first step is there, the second may still be on its way
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int r = 0; r < 4; ++r) rd_a(0, 0, 0, r);
#pragma unroll
        for (int kk = 0; kk < 3; ++kk)
#pragma unroll
            for (int r = 0; r < 8; ++r) rd_w(kk, 0, kk, r);
    }
    for (uint32_t c_tile = blockIdx.x; c_tile < ntiles; c_tile += gridDim.x) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        for (uint32_t ks = 0; ks < steps; ++ks) {
            // One k-step (four sub-steps of 16 k) on stage `cur`; `oth` holds the next step.  The two operands of a
            // stage are released, refilled and waited for half a step apart, so that two batches of loads are in
            // flight at any time (one batch at a time left the step waiting for the latency of its loads plus
            // their transfer): A's fragments are read one sub-step ahead, W's three sub-steps ahead, hence
            //   sub-step 0: last reads of W in `cur`                     -> W of the stream's step goes into `cur`
            //   sub-step 2: last reads of A in `cur`                     -> A of the stream's step goes into `cur`
            // The stream's step is two ahead of this one, possibly in the workgroup's next tile.  Each wavefront
            // has 8 loads per operand and step; vmcnt(8) therefore waits for the older of the two batches in flight.
            // Once the stream has passed the workgroup's last tile it stands still: the loads of the last two
            // k-steps fetch that tile's last step again, into stages nobody reads any more.
            const uint32_t oth = kT2Stage - cur;
            AMAP_PIN();
            phase(0, 0, cur, 1, cur, 3, 0, 0);
            // W of the next step has landed (A of it may still be on its way), and every wavefront is done with W in `cur`
            // (the loads only count in vmcnt; the compiler does not know of them)
            asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            AMAP_PIN();
            phase(1, 1, cur, 2, oth, 0, cur, 1);
            phase(0, 2, cur, 3, oth, 1, 0, 0);
            // A of the next step has landed, and every wavefront is done with A in `cur`
            asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            AMAP_PIN();
            // (after the workgroup's last step the fragments read ahead are stale and unused)
            phase(1, 3, oth, 0, oth, 2, cur, 2);
            if (ld.c.tile < ntiles) cursor_next();
            cur = oth;
        }

        // ---- epilogue: this wavefront's 128 x 128 block, 32 rows at a time: rounded to bf16, through its
        // own 8 KiB of LDS (16-byte chunks XOR-swizzled by the row, the 8-byte halves by row bit 4), then
        // whole 256-byte row segments to memory.  Accumulator v of a tile in lane l: m = l % 32,
        // n = 8 (v / 4) + 4 (l / 32) + v % 4.
        uint32_t tm, tn;
        tile_of_block(c_tile, g.tiles_m, g.tiles_n, tm, tn);
        const uint32_t scr = kT2Scratch + wave * 8192u;
        const uint32_t row_w = lane & 31u, half_w = lane >> 5;
        const uint32_t m_base = tm * T2M + wm * 128u, n_lane = tn * T2N + wn * 128u + (lane & 15u) * 8u;
        const GemmArgs &gs = t2_args_again();   // the store map's digits
        const size_t col_off = t2_store_col<STORE_MAPPED>(gs, n_lane);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int jn = 0; jn < 4; ++jn)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    u32x2 o;
                    o.x = pack_bf16(acc[i][jn][4 * q], acc[i][jn][4 * q + 1]);
                    o.y = pack_bf16(acc[i][jn][4 * q + 2], acc[i][jn][4 * q + 3]);
                    const uint32_t chunk = (uint32_t)(jn * 4 + q) ^ (row_w & 15u);
                    *reinterpret_cast<__attribute__((address_space(3))) u32x2 *>(scr + row_w * 256u + (chunk << 4) + ((half_w ^ (row_w >> 4)) << 3)) = o;
                }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const uint32_t row = 4u * p + (lane >> 4), chunk = lane & 15u;
                u32x4 x = *reinterpret_cast<lds_u32x4 *>(scr + row * 256u + ((chunk ^ (row & 15u)) << 4));
                if (p >= 4) x = u32x4{x.z, x.w, x.x, x.y};
                const uint32_t m = m_base + i * 32u + row;
                const size_t off = t2_store_off<STORE_MAPPED>(gs, col_off, m);
                if (!EDGE || (m < g.M && n_lane < g.N)) __builtin_nontemporal_store(x, reinterpret_cast<u32x4 *>(g.C + off));
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the loads of the last two k-steps land in LDS before the wavefront ends
}

// Split the loops of one dst dimension of a piece into digits.  The piece must start at
// index `lo` of that dimension and cover `extent` indices.
bool make_digits(const Piece &p, int dim, int64_t extent, Digits &d, int64_t lo = 0) {
    std::memset(&d, 0, sizeof(d));
    std::vector<IterDim> its;
    for (const IterDim &it : p.it)
        if (it.dim == dim) its.push_back(it);
    // loops that continue one another on both sides (h and w of an image plane kept whole)
    // count as one digit: fewer divisions, and longer contiguous runs for the vector check
    std::sort(its.begin(), its.end(), [](const IterDim &x, const IterDim &y) { return x.mult < y.mult; });
    for (size_t i = 0; i + 1 < its.size();) {
        const IterDim &in = its[i], &out = its[i + 1];
        if (out.mult == in.mult * in.extent && out.sstride == in.sstride * in.extent) {
            its[i].extent *= out.extent;
            its.erase(its.begin() + i + 1);
        } else {
            ++i;
        }
    }
    if (its.size() > (size_t)kMaxDigits) return false;
    int64_t covered = 1;
    for (const IterDim &it : its) covered *= it.extent;
    if (covered != extent || p.lo[dim] != lo) return false;
    for (const IterDim &it : its)   // what the 32-bit fields below (and the dividers, good below 2^31) hold
        if (it.mult >= (1ll << 31) || it.extent >= (1ll << 31) || it.sstride >= (1ll << 31) || it.sstride <= -(1ll << 31)) return false;
    for (const IterDim &it : its) {
        const uint32_t j = d.n++;
        d.mult[j] = (uint32_t)it.mult;
        d.ext[j] = (uint32_t)it.extent;
        d.ss[j] = (int32_t)it.sstride;
        d.fmult[j] = make_fastdiv(d.mult[j]);
        d.fext[j] = make_fastdiv(d.ext[j]);
    }
    // the rest as digits that contribute nothing, for decoders with a fixed trip count
    for (uint32_t j = d.n; j < (uint32_t)kMaxDigits; ++j) {
        d.mult[j] = d.ext[j] = 1;
        d.ss[j] = 0;
        d.fmult[j] = d.fext[j] = make_fastdiv(1);
    }
    return true;
}


// The loops of one dst dimension of a data piece that padding surrounds: digits as in make_digits plus
// the box (origin and, per digit, the radix of the padded tensor) that tells inside from outside.
bool make_pad_digits(const Piece &p, int dim, Digits &d, PadBox &b) {
    std::memset(&d, 0, sizeof(d));
    std::memset(&b, 0, sizeof(b));
    std::vector<IterDim> its;
    for (const IterDim &it : p.it)
        if (it.dim == dim) its.push_back(it);
    std::sort(its.begin(), its.end(), [](const IterDim &x, const IterDim &y) { return x.mult < y.mult; });
    for (size_t i = 0; i + 1 < its.size();) {   // loops that continue one another on both sides are one digit
        const IterDim &in = its[i], &out = its[i + 1];
        if (out.mult == in.mult * in.extent && out.sstride == in.sstride * in.extent) {
            its[i].extent *= out.extent;
            its.erase(its.begin() + i + 1);
        } else {
            ++i;
        }
    }
    if (its.empty()) its.push_back(IterDim{1, dim, 1, 0});   // a single index of this dimension
    if (its.size() > (size_t)kMaxDigits || its[0].mult != 1 || p.lo[dim] < 0 || p.lo[dim] >= (1ll << 31)) return false;
    b.lo = (uint32_t)p.lo[dim];
    for (size_t j = 0; j < its.size(); ++j) {
        const IterDim &it = its[j];
        if (it.extent >= (1ll << 31) || it.mult >= (1ll << 31)) return false;
        d.mult[j] = (uint32_t)it.mult;
        d.ext[j] = (uint32_t)it.extent;
        d.ss[j] = (int32_t)it.sstride;
        d.fmult[j] = make_fastdiv(d.mult[j]);
        d.fext[j] = make_fastdiv(d.ext[j]);
        if (j + 1 < its.size()) {
            if (its[j + 1].mult % it.mult) return false;
            const int64_t rad = its[j + 1].mult / it.mult;
            if (rad < it.extent) return false;
            b.rad[j] = (uint32_t)rad;
            b.frad[j] = make_fastdiv(b.rad[j]);
        }
    }
    d.n = (uint32_t)its.size();
    return true;
}

}  // namespace

namespace {

// 16-byte vectors along a dimension: its innermost digit must be contiguous on
// the other side in runs of a multiple of 8 elements, everything else 8-aligned
bool vector_runs(const Digits &inner, const Digits &outer, int64_t base) {
    bool inner_ok = false;
    for (uint32_t j = 0; j < inner.n; ++j) {
        if (inner.mult[j] == 1)
            inner_ok = inner.ss[j] == 1 && inner.ext[j] % 8 == 0;
        else if (inner.ss[j] % 8 != 0 || inner.mult[j] % 8 != 0)
            return false;
    }
    for (uint32_t j = 0; j < outer.n; ++j)
        if (outer.ss[j] % 8 != 0) return false;
    return inner_ok && base % 8 == 0;
}

bool overlaps(const void *a, int64_t an, const void *b, int64_t bn) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + (uintptr_t)bn && b0 < a0 + (uintptr_t)an;
}

// AMAP_E_UNSUPPORTED with the reason left for amap_last_error
amap_status unsupported(const char *why) {
    set_last_error("unsupported", why);
    return AMAP_E_UNSUPPORTED;
}

// extent of a piece along one dst dimension
int64_t piece_extent(const Piece &p, int dim) {
    int64_t e = 1;
    for (const IterDim &it : p.it)
        if (it.dim == dim) e *= it.extent;
    return e;
}

// A_srcs: by source id of A_map when `by_id`, else the one source of a single-piece map
// dry / dry_kernel: plan only, for the host replay: the kernel arguments and which kernel would run
// (1: 256 x 256 tiles, 0: the general kernel); nothing is launched and no HIP call is made.
amap_status gemm_launch(const void *const *A_srcs, bool by_id, const amap_t *A_map, const void *W, int64_t N,
                        const amap_t *W_map, const amap_t *out_map, void *out, void *stream, GemmArgs *dry = nullptr,
                        int *dry_kernel = nullptr) {
    if (W_map) {
        if (W_map->shape.size() != 2) return AMAP_E_INVALID;
        N = W_map->shape[1];
    }
    if (!A_srcs || !A_map || !W || !out || N <= 0) return AMAP_E_INVALID;
    if (((uintptr_t)W | (uintptr_t)out) & 15) return AMAP_E_INVALID;
    if (A_map->shape.size() != 2 || A_map->elem != 2) return AMAP_E_INVALID;
    const int64_t M = A_map->shape[0], K = A_map->shape[1];
    if (M == 0 || K == 0) return unsupported("empty product");
    if (N % 8 || K % 8) return unsupported("N and K must be multiples of 8");
    bool edge = M % BM || N % BN || K % BK;
    if (!A_map->strided || A_map->pieces.empty()) return unsupported("the A map has no strided form");
    if (M >= (1ll << 31) || N >= (1ll << 24) || K >= (1ll << 31) || M * N >= (1ll << 40)) return unsupported("operand too large");
    // Operands or sources of 2^31 elements and more: only the 256 x 256-tile kernel reaches them (64-bit tile bases);
    // every other product is refused further down, once it is known which kernel it would take.
    bool wide = M * K >= (1ll << 31) || K * N >= (1ll << 31);
    if (out_map && M * N >= (1ll << 31)) return unsupported("product too large for a mapped store");
    const int64_t cbytes = M * N * 2;
    GemmArgs g;
    std::memset(&g, 0, sizeof(g));
    // ---- the A operand: one piece, or one piece per range of k (segments, sorted by k)
    // A piece whose k indices are not one interval (one source feeding two ranges of k is kept
    // as one piece with an outer loop over the two) is taken apart along that loop.
    // Padding (Section 2.1, a pad operator in front of the product): fill pieces of one constant around
    // ONE data piece are folded into the operand load; the pieces of a map partition its index space, so
    // whatever the data piece does not cover reads the constant.
    std::vector<Piece> parts;
    bool padded = false;
    uint32_t pad_bits = 0;
    for (const Piece &q : A_map->pieces) {
        if (!q.fill) {
            parts.push_back(q);
        } else if (padded && (q.fill_bits & 0xFFFFu) != pad_bits) {
            return unsupported("the A map pads with more than one constant");
        } else {
            padded = true;
            pad_bits = q.fill_bits & 0xFFFFu;
        }
    }
    if (padded && (parts.size() != 1 || by_id)) return unsupported("padding around an A operand of several pieces");
    for (size_t i = 0; !padded && i < parts.size() && parts.size() <= (size_t)kMaxSeg; ++i) {
        for (;;) {
            std::vector<IterDim> kl;
            for (const IterDim &it : parts[i].it)
                if (it.dim == 1) kl.push_back(it);
            std::sort(kl.begin(), kl.end(), [](const IterDim &x, const IterDim &y) { return x.mult < y.mult; });
            int64_t run = 1;
            bool dense = true;
            for (const IterDim &it : kl) {
                dense = dense && it.mult == run;
                run *= it.extent;
            }
            if (dense || kl.back().extent + parts.size() - 1 > (size_t)kMaxSeg) break;
            const IterDim outer = kl.back();
            Piece rest = parts[i];
            rest.it.erase(std::remove_if(rest.it.begin(), rest.it.end(),
                                         [&](const IterDim &it) { return it.dim == 1 && it.mult == outer.mult; }),
                          rest.it.end());
            parts[i] = rest;
            for (int64_t c = 1; c < outer.extent; ++c) {
                Piece q = rest;
                q.lo[1] += c * outer.mult;
                q.sbase += c * outer.sstride;
                parts.push_back(q);
            }
        }
    }
    std::vector<const Piece *> segs;
    for (const Piece &q : parts) segs.push_back(&q);
    if (segs.size() > (size_t)kMaxSeg || (segs.size() > 1 && !by_id)) return unsupported("the A map has several pieces (amap_gemm_gather takes up to 8, one per range of k)");
    std::sort(segs.begin(), segs.end(), [](const Piece *x, const Piece *y) { return x->lo[1] < y->lo[1]; });
    int amode = -1;
    int64_t k_at = 0;
    for (size_t j = 0; j < segs.size(); ++j) {
        const Piece &p = *segs[j];
        const void *src = A_srcs[by_id ? p.src : 0];
        if (!src || ((uintptr_t)src & 15)) return AMAP_E_INVALID;
        const int64_t svol = volume_of(A_map->src_shapes[p.src]);
        if (svol >= (1ll << 31) || p.sbase >= (1ll << 31)) wide = true;
        if (overlaps(out, cbytes, src, svol * 2)) return AMAP_E_ALIAS;
        const int64_t kext = piece_extent(p, 1);
        Digits dm, dk;
        if (padded) {
            if (!make_pad_digits(p, 0, dm, g.pm) || !make_pad_digits(p, 1, dk, g.pk)) return unsupported("the padded A map does not decode into digits");
            // whole 16-byte vectors along k lie inside or outside the data piece
            if (!vector_runs(dk, dm, p.sbase) || g.pk.lo % 8 || (g.pk.rad[0] && g.pk.rad[0] % 8)) return unsupported("the padded A map has no 8-element aligned runs along k inside 8-element aligned padding");
            g.padded = 1;
            g.pad_word = pad_bits | (pad_bits << 16);
            amode = A_RUNS_K;
            g.A_src = static_cast<const uint16_t *>(src);
            g.sbase = (uint32_t)p.sbase;
            g.dm = dm;
            g.dk = dk;
            k_at = K;
            break;
        }
        // every segment spans all of m and continues k where the one before ended
        if (!make_digits(p, 0, M, dm) || !make_digits(p, 1, kext, dk, k_at)) return unsupported("a piece of the A map does not span all of m, or the pieces do not follow one another along k");
        int mode = A_RUNS_K;
        if (!vector_runs(dk, dm, p.sbase)) {
            if (M % 8 || !vector_runs(dm, dk, p.sbase)) return unsupported("the A map has no 8-element aligned source runs along k or along m");
            mode = A_RUNS_M;
        }
        if (amode >= 0 && mode != amode) return unsupported("the sources of A have their runs along different dimensions");
        amode = mode;
        k_at += kext;
        // a k-step (64, runs along k) or half of one (32, runs along m) reads one source
        if (j + 1 < segs.size() && k_at % (mode == A_RUNS_K ? BK : BK / 2)) return unsupported("a source of A ends inside a k-step (ranges must end at multiples of 64, or 32 with runs along m)");
        if (segs.size() == 1) {
            g.A_src = static_cast<const uint16_t *>(src);
            g.sbase = (uint32_t)p.sbase;
            g.a_base = p.sbase;
            g.dm = dm;
            g.dk = dk;
        } else {
            g.seg_src[j] = static_cast<const uint16_t *>(src);
            g.seg_sbase[j] = (uint32_t)p.sbase;
            g.seg_kend[j] = (uint32_t)k_at;
            g.seg_dm[j] = dm;
            g.seg_dk[j] = dk;
        }
    }
    if (k_at != K) return unsupported("the pieces of the A map do not cover k");
    g.n_seg = (uint32_t)segs.size();
    if (g.n_seg > 1) g.A_src = g.seg_src[0];
    int wmode = W_PLAIN;
    int64_t wvol = K * N;
    if (W_map) {
        // W[k,n] = W_src[g_w(k,n)]: the second consumer load of the product, rewritten like the first
        if (W_map->elem != 2 || W_map->shape[0] != K) return AMAP_E_INVALID;
        if (!W_map->strided || W_map->pieces.size() != 1 || W_map->pieces[0].fill) return unsupported("the W map is not one fill-free strided piece");
        const Piece &q = W_map->pieces[0];
        wvol = volume_of(W_map->src_shapes[q.src]);
        if (wvol >= (1ll << 31)) return unsupported("W source too large for 32-bit offsets");
        if (!make_digits(q, 0, K, g.wk) || !make_digits(q, 1, N, g.wn)) return unsupported("the W map does not span [K,N]");
        if (vector_runs(g.wn, g.wk, q.sbase))
            wmode = W_MAPPED_N;
        else if (vector_runs(g.wk, g.wn, q.sbase))
            wmode = W_MAPPED_K;
        else
            return unsupported("the W map has no 8-element aligned source runs along n or along k");
        g.wbase = (uint32_t)q.sbase;
    }
    if (overlaps(out, cbytes, W, wvol * 2)) return AMAP_E_ALIAS;
    if (out_map) {
        // the layout chain applied to the product, turned into a store map: the
        // reverse of the chain's load map (Section 2.1), C index -> index of out
        if (out_map->elem != 2 || out_map->src_shapes.size() != 1 || out_map->src_shapes[0].size() != 2 ||
            out_map->src_shapes[0][0] != M || out_map->src_shapes[0][1] != N)
            return AMAP_E_INVALID;
        amap_t *rev = nullptr;
        amap_status st = amap_inverse(out_map, &rev);
        if (st != AMAP_OK) {  // not a bijection between the product and out
            set_last_error("unsupported", "the store map is not a bijection between the product and out");
            return st;
        }
        std::unique_ptr<amap> hold(rev);
        if (!rev->strided || rev->pieces.size() != 1 || rev->pieces[0].fill) return unsupported("the reversed store map is not one strided piece");
        const Piece &q = rev->pieces[0];
        if (!make_digits(q, 0, M, g.om) || !make_digits(q, 1, N, g.on)) return unsupported("the store map does not span [M,N]");
        if (!vector_runs(g.on, g.om, q.sbase)) return unsupported("the store map has no 8-element aligned runs along n");
        g.store_mapped = 1;
        g.obase = (uint32_t)q.sbase;
    }

    g.W = static_cast<const uint16_t *>(W);
    g.C = static_cast<uint16_t *>(out);
    g.M = (uint32_t)M;
    g.N = (uint32_t)N;
    g.K = (uint32_t)K;
    g.tiles_m = (uint32_t)((M + BM - 1) / BM);
    g.tiles_n = (uint32_t)((N + BN - 1) / BN);
    hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
    // ---- the common case runs on 256 x 256 tiles (see amap_gemm_tile256_kernel)
    const char *t256 = std::getenv("AMAP_GEMM_TILE256");   // 0: always the general kernel (tests compare the two)
    const bool tile256_on = !(t256 && t256[0] == '0');
    if (g.padded) edge = true;   // the instances that test every vector also take the padding
    // W: row-major [K,N], or kept as [N,K] and read through a transpose map (whole 64-element runs along k, rows of n evenly
    // spaced inside every 256-row block: blocks that never straddle a digit, or one digit for all of n)
    const bool edge256 = M % T2M != 0 || N % T2N != 0;   // partial last tiles: the EDGE instances
    const bool w_km = wmode == W_MAPPED_K && g.wk.mult[0] == 1 && g.wk.ss[0] == 1 && g.wk.ext[0] % T2K == 0 && g.wn.mult[0] == 1 &&
                      (g.wn.ext[0] % T2N == 0 || g.wn.n == 1) && g.wn.ss[0] >= 0 && g.wn.ss[0] < (1 << 23);
    if (tile256_on && !g.padded && amode == A_RUNS_K && segs.size() == 1 && (wmode == W_PLAIN || w_km) && K % T2K == 0 &&
        K >= 2 * T2K && g.dm.mult[0] == 1 && (g.dm.ext[0] % T2M == 0 || g.dm.n == 1) && g.dm.ss[0] >= 0 && g.dm.ss[0] < (1 << 23) && g.dk.mult[0] == 1 &&
        g.dk.ss[0] == 1 && g.dk.ext[0] % T2K == 0 && (!wide || !out_map)) {
        g.w_row_ss = w_km ? (uint32_t)g.wn.ss[0] : 0u;
        g.a_steps = t2_steps_of(g.dk);
        g.w_steps = w_km ? t2_steps_of(g.wk) : t2_steps_plain_w(g.K, g.N);
        if (dry) {
            g.a_row_ss = (uint32_t)g.dm.ss[0];
            g.tiles_m = (uint32_t)((M + T2M - 1) / T2M);
            g.tiles_n = (uint32_t)((N + T2N - 1) / T2N);
            *dry = g;
            *dry_kernel = (w_km ? 2 : 1) + (edge256 ? 2 : 0);
            return AMAP_OK;
        }
        static thread_local int n_cu = 0;
        if (n_cu == 0) {
            int dev = 0;
            if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) {
                (void)hipGetLastError();
                n_cu = 0;
                set_last_error("amap_gemm_tile256_kernel: cannot query the device");
                return AMAP_E_HIP;
            }
#define AMAP_T2_FNS(E)                                                                                                                                     \
    reinterpret_cast<const void *>(amap_gemm_tile256_kernel<false, false, E>), reinterpret_cast<const void *>(amap_gemm_tile256_kernel<true, false, E>), \
        reinterpret_cast<const void *>(amap_gemm_tile256_kernel<false, true, E>), reinterpret_cast<const void *>(amap_gemm_tile256_kernel<true, true, E>)
            for (const void *fn : {AMAP_T2_FNS(false), AMAP_T2_FNS(true)})
                if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kT2Lds) != hipSuccess) {
                    (void)hipGetLastError();
                    n_cu = 0;
                    set_last_error("amap_gemm_tile256_kernel: cannot reserve its LDS stages");
                    return AMAP_E_HIP;
                }
        }
        if (const char *tr = std::getenv("AMAP_PLAN_TRACE"); tr && tr[0] != '0')
            std::fprintf(stderr, "amap gemm: 256 x 256 tiles%s%s, %lld x %lld x %lld\n", w_km ? " (W runs along k)" : "", edge256 ? " (partial last tiles)" : "",
                         (long long)M, (long long)N, (long long)K);
        g.a_row_ss = (uint32_t)g.dm.ss[0];
        g.tiles_m = (uint32_t)((M + T2M - 1) / T2M);
        g.tiles_n = (uint32_t)((N + T2N - 1) / T2N);
        const uint32_t ntiles = g.tiles_m * g.tiles_n;
        const dim3 grid2(t2_workgroups(ntiles, (uint32_t)n_cu)), block2(kGemmThreads);
        (void)hipGetLastError();   // an earlier, unrelated error on this thread is not this launch's
#define AMAP_T2_LAUNCH(E)                                                                                   \
    do {                                                                                                    \
        if (g.store_mapped && w_km)                                                                         \
            hipLaunchKernelGGL((amap_gemm_tile256_kernel<true, true, E>), grid2, block2, kT2Lds, hs, g);    \
        else if (g.store_mapped)                                                                            \
            hipLaunchKernelGGL((amap_gemm_tile256_kernel<true, false, E>), grid2, block2, kT2Lds, hs, g);   \
        else if (w_km)                                                                                      \
            hipLaunchKernelGGL((amap_gemm_tile256_kernel<false, true, E>), grid2, block2, kT2Lds, hs, g);   \
        else                                                                                                \
            hipLaunchKernelGGL((amap_gemm_tile256_kernel<false, false, E>), grid2, block2, kT2Lds, hs, g);  \
    } while (0)
        if (edge256)
            AMAP_T2_LAUNCH(true);
        else
            AMAP_T2_LAUNCH(false);
#undef AMAP_T2_LAUNCH
        const hipError_t e2 = hipGetLastError();
        if (e2 != hipSuccess) {
            set_last_error("amap_gemm_tile256_kernel", hipGetErrorString(e2));
            return AMAP_E_HIP;
        }
        return AMAP_OK;
    }
    if (wide) return unsupported("an operand or source of 2^31 elements and more: only the 256 x 256-tile kernel (see amap_gemm_fused) with a plain store reaches it");
    if (dry) {
        *dry = g;
        *dry_kernel = 0;
        return AMAP_OK;
    }
    if (const char *tr = std::getenv("AMAP_PLAN_TRACE"); tr && tr[0] != '0')
        std::fprintf(stderr, "amap gemm: 256 x 128 tiles, %lld x %lld x %lld\n", (long long)M, (long long)N, (long long)K);
    const size_t lds = kLdsBytes;
    static thread_local bool attr_done = false;
    if (!attr_done) {
#define AMAP_GEMM_FN(AM, WM, E) \
    reinterpret_cast<const void *>(amap_gemm_kernel<AM, WM, E, false>), reinterpret_cast<const void *>(amap_gemm_kernel<AM, WM, E, true>)
        for (const void *fn :
             {AMAP_GEMM_FN(A_RUNS_K, W_PLAIN, false), AMAP_GEMM_FN(A_RUNS_K, W_MAPPED_N, false),
              AMAP_GEMM_FN(A_RUNS_K, W_MAPPED_K, false), AMAP_GEMM_FN(A_RUNS_K, W_PLAIN, true),
              AMAP_GEMM_FN(A_RUNS_K, W_MAPPED_N, true), AMAP_GEMM_FN(A_RUNS_K, W_MAPPED_K, true),
              AMAP_GEMM_FN(A_RUNS_M, W_PLAIN, false), AMAP_GEMM_FN(A_RUNS_M, W_MAPPED_N, false),
              AMAP_GEMM_FN(A_RUNS_M, W_MAPPED_K, false), AMAP_GEMM_FN(A_RUNS_M, W_PLAIN, true),
              AMAP_GEMM_FN(A_RUNS_M, W_MAPPED_N, true), AMAP_GEMM_FN(A_RUNS_M, W_MAPPED_K, true)}) {
#undef AMAP_GEMM_FN
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
                (void)hipGetLastError();
                set_last_error("amap_gemm_kernel: cannot reserve its LDS stage");
                return AMAP_E_HIP;
            }
        }
        attr_done = true;
    }
    const dim3 grid(g.tiles_m * g.tiles_n), block(kGemmThreads);
    const bool seg = g.n_seg > 1;
    (void)hipGetLastError();   // an earlier, unrelated error on this thread is not this launch's
#define AMAP_GEMM_AWE(AM, WM, E)                                                                       \
    do {                                                                                               \
        if (seg)                                                                                       \
            hipLaunchKernelGGL((amap_gemm_kernel<AM, WM, E, true>), grid, block, lds, hs, g);          \
        else                                                                                           \
            hipLaunchKernelGGL((amap_gemm_kernel<AM, WM, E, false>), grid, block, lds, hs, g);         \
    } while (0)
#define AMAP_GEMM(WM)                                                                                  \
    do {                                                                                               \
        if (amode == A_RUNS_K && edge)                                                                 \
            AMAP_GEMM_AWE(A_RUNS_K, WM, true);                                                         \
        else if (amode == A_RUNS_K)                                                                    \
            AMAP_GEMM_AWE(A_RUNS_K, WM, false);                                                        \
        else if (edge)                                                                                 \
            AMAP_GEMM_AWE(A_RUNS_M, WM, true);                                                         \
        else                                                                                           \
            AMAP_GEMM_AWE(A_RUNS_M, WM, false);                                                        \
    } while (0)
    if (wmode == W_PLAIN)
        AMAP_GEMM(W_PLAIN);
    else if (wmode == W_MAPPED_N)
        AMAP_GEMM(W_MAPPED_N);
    else
        AMAP_GEMM(W_MAPPED_K);
#undef AMAP_GEMM_AWE
#undef AMAP_GEMM
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_last_error("amap_gemm_kernel", hipGetErrorString(e));
        return AMAP_E_HIP;
    }
    return AMAP_OK;
}

}  // namespace

extern "C" amap_status amap_gemm_fused(const void *A_src, const amap_t *A_map, const void *W, int64_t N, void *out,
                                       void *stream) {
    try {
        return gemm_launch(&A_src, false, A_map, W, N, nullptr, nullptr, out, stream);
    } catch (...) {
        return AMAP_E_NOMEM;
    }
}

extern "C" amap_status amap_gemm_fused_store(const void *A_src, const amap_t *A_map, const void *W, int64_t N,
                                             const amap_t *out_map, void *out, void *stream) {
    if (!out_map) return AMAP_E_INVALID;
    try {
        return gemm_launch(&A_src, false, A_map, W, N, nullptr, out_map, out, stream);
    } catch (...) {
        return AMAP_E_NOMEM;
    }
}

extern "C" amap_status amap_gemm_mapped(const void *A_src, const amap_t *A_map, const void *W_src, const amap_t *W_map,
                                        const amap_t *out_map, void *out, void *stream) {
    if (!W_map) return AMAP_E_INVALID;
    try {
        return gemm_launch(&A_src, false, A_map, W_src, 0, W_map, out_map, out, stream);
    } catch (...) {
        return AMAP_E_NOMEM;
    }
}

extern "C" amap_status amap_gemm_gather(const void *const *A_srcs, const amap_t *A_map, const void *W_src,
                                        const amap_t *W_map, int64_t N, const amap_t *out_map, void *out, void *stream) {
    if (!A_srcs || !A_map) return AMAP_E_INVALID;
    for (const Piece &q : A_map->pieces)
        if (!q.fill && (q.src < 0 || (size_t)q.src >= A_map->src_shapes.size())) return AMAP_E_INVALID;
    try {
        return gemm_launch(A_srcs, true, A_map, W_src, W_map ? 0 : N, W_map, out_map, out, stream);
    } catch (...) {
        return AMAP_E_NOMEM;
    }
}

// Host replay of the global accesses of amap_gemm_tile256_kernel for the product A_map x W[K,N] (-> out_map):
// every workgroup's load cursor is walked through its prologue and its k-loop exactly as the kernel walks it,
// with the kernel's own address functions, and every store of the epilogue is enumerated.  Counted as errors:
// a load outside the A source or outside W; a k-step that does not fetch exactly the 256 x 64 block of A and the
// 64 x 256 block of W it is for; fetches that are not in the order the MFMAs consume them; a store outside out,
// and elements of out written never or twice.  AMAP_E_UNSUPPORTED if the product would run in the general kernel.
namespace {
template <bool W_KM, bool EDGE>
amap_status replay_tile256(const GemmArgs &g, int64_t a_bytes, int64_t w_bytes, int n_workgroups, int64_t *n_errors);
}

extern "C" amap_status amap_gemm_selfcheck(const amap_t *A_map, const amap_t *W_map, int64_t N, const amap_t *out_map,
                                           int n_workgroups, int64_t *n_errors) {
    if (!A_map || !n_errors || n_workgroups < 1) return AMAP_E_INVALID;
    try {
        GemmArgs g;
        int kernel = 0;
        const void *fake_a = reinterpret_cast<const void *>((uintptr_t)1 << 40);
        amap_status st = gemm_launch(&fake_a, false, A_map, reinterpret_cast<const void *>((uintptr_t)2 << 40), N, W_map, out_map,
                                     reinterpret_cast<void *>((uintptr_t)3 << 40), nullptr, &g, &kernel);
        if (st != AMAP_OK) return st;
        if (kernel == 0) return unsupported("no host replay for the general GEMM kernel");
        int src = -1;
        for (const Piece &q : A_map->pieces)
            if (!q.fill) src = q.src;
        if (src < 0 || (size_t)src >= A_map->src_shapes.size()) return AMAP_E_INVALID;
        const int64_t a_bytes = volume_of(A_map->src_shapes[(size_t)src]) * 2;
        const int64_t w_bytes = (W_map ? volume_of(W_map->src_shapes[(size_t)W_map->pieces[0].src]) : (int64_t)g.K * g.N) * 2;
        switch (kernel) {
        case 1: return replay_tile256<false, false>(g, a_bytes, w_bytes, n_workgroups, n_errors);
        case 2: return replay_tile256<true, false>(g, a_bytes, w_bytes, n_workgroups, n_errors);
        case 3: return replay_tile256<false, true>(g, a_bytes, w_bytes, n_workgroups, n_errors);
        default: return replay_tile256<true, true>(g, a_bytes, w_bytes, n_workgroups, n_errors);
        }
    } catch (...) {
        return AMAP_E_NOMEM;
    }
}

namespace {
template <bool W_KM, bool EDGE>
amap_status replay_tile256(const GemmArgs &g, int64_t a_bytes, int64_t w_bytes, int n_workgroups, int64_t *n_errors) {
    {
        const int64_t c_elems = (int64_t)g.M * g.N;
        int64_t errors = 0;
        const uint32_t ntiles = g.tiles_m * g.tiles_n, steps = g.K / (uint32_t)T2K;
        const uint32_t nwg = t2_workgroups(ntiles, (uint32_t)n_workgroups);
        std::vector<uint8_t> written((size_t)(c_elems / 8), 0);   // per 8-element vector of out
        std::vector<int64_t> got_a, got_w, want_a, want_w;
        for (uint32_t blk = 0; blk < nwg; ++blk) {
            std::vector<T2Cursor> fetched, consumed;
            // one batch of loads of all four wavefronts for the cursor's k-step
            auto fetch = [&](const T2Stream &st) {
                const T2Cursor &c = st.c;
                fetched.push_back(c);
                if (c.tile >= ntiles || c.k0 + (uint32_t)T2K > g.K) {
                    ++errors;
                    return;
                }
                const int64_t ka = st.a_tile + st.a_step, wk = st.w_tile + st.w_step;
                got_a.clear(), got_w.clear(), want_a.clear(), want_w.clear();
                uint32_t tm, tn;
                tile_of_block(c.tile, g.tiles_m, g.tiles_n, tm, tn);
                const uint32_t rv = EDGE ? t2_rows_valid(g, tm) : (uint32_t)T2M, cv = EDGE ? t2_cols_valid(g, tn) : (uint32_t)T2N;
                for (uint32_t wave = 0; wave < 4; ++wave)
                    for (uint32_t j = 0; j < 8; ++j)
                        for (uint32_t lane = 0; lane < 64; ++lane) {
                            const int64_t ao = ka + (int64_t)(EDGE ? t2_a_load_edge(g, wave, lane, j, rv) : t2_a_load(g, t2_a_lane(g, wave, lane, j & 1u), j));
                            const int64_t wo = wk + (int64_t)(EDGE ? t2_w_load_edge<W_KM>(g, wave, lane, j, cv)
                                                                   : t2_w_load<W_KM>(g, t2_w_lane<W_KM>(g, wave, lane, j & 1u), j));
                            if (ao < 0 || ao + 16 > a_bytes) ++errors;
                            if (wo < 0 || wo + 16 > w_bytes) ++errors;
                            got_a.push_back(ao);
                            got_w.push_back(wo);
                        }
                // what the k-step is for: the existing rows (columns) of the tile, every 16-byte vector of them once
                for (uint32_t r = 0; r < rv; ++r)
                    for (uint32_t ch = 0; ch < 8; ++ch)
                        want_a.push_back(2 * (g.a_base + digits_offset4_wide(g.dm, tm * (uint32_t)T2M + r) + digits_offset4_wide(g.dk, c.k0 + 8u * ch)));
                if constexpr (W_KM) {
                    for (uint32_t r = 0; r < cv; ++r)
                        for (uint32_t ch = 0; ch < 8; ++ch)
                            want_w.push_back(2 * ((int64_t)g.wbase + digits_offset4_wide(g.wn, tn * (uint32_t)T2N + r) + digits_offset4_wide(g.wk, c.k0 + 8u * ch)));
                } else {
                    for (uint32_t kr = 0; kr < (uint32_t)T2K; ++kr)
                        for (uint32_t ch = 0; ch < cv / 8; ++ch)
                            want_w.push_back(2 * ((int64_t)(c.k0 + kr) * (int64_t)g.N + (int64_t)(tn * (uint32_t)T2N + 8u * ch)));
                }
                std::sort(got_a.begin(), got_a.end()), std::sort(want_a.begin(), want_a.end());
                std::sort(got_w.begin(), got_w.end()), std::sort(want_w.begin(), want_w.end());
                if (EDGE) {  // lanes past the last row / column repeat existing vectors: compare the sets
                    got_a.erase(std::unique(got_a.begin(), got_a.end()), got_a.end());
                    got_w.erase(std::unique(got_w.begin(), got_w.end()), got_w.end());
                }
                if (got_a != want_a) ++errors;
                if (got_w != want_w) ++errors;
            };
            // loads issued after the stream has passed the workgroup's last tile: bounds only (nobody reads them)
            auto stale = [&](const T2Stream &st) {
                const int64_t ka = st.a_tile + st.a_step, wk = st.w_tile + st.w_step;
                uint32_t tm, tn;
                tile_of_block(st.c.tile - nwg, g.tiles_m, g.tiles_n, tm, tn);   // the tile whose state the stream kept
                const uint32_t rv = EDGE ? t2_rows_valid(g, tm) : (uint32_t)T2M, cv = EDGE ? t2_cols_valid(g, tn) : (uint32_t)T2N;
                for (uint32_t wave = 0; wave < 4; ++wave)
                    for (uint32_t j = 0; j < 8; ++j)
                        for (uint32_t lane = 0; lane < 64; ++lane) {
                            const int64_t ao = ka + (int64_t)(EDGE ? t2_a_load_edge(g, wave, lane, j, rv) : t2_a_load(g, t2_a_lane(g, wave, lane, j & 1u), j));
                            const int64_t wo = wk + (int64_t)(EDGE ? t2_w_load_edge<W_KM>(g, wave, lane, j, cv)
                                                                   : t2_w_load<W_KM>(g, t2_w_lane<W_KM>(g, wave, lane, j & 1u), j));
                            if (ao < 0 || ao + 16 > a_bytes) ++errors;
                            if (wo < 0 || wo + 16 > w_bytes) ++errors;
                        }
            };
            T2Stream ld = {};
            ld.c = T2Cursor{blk, 0};
            if (ld.c.tile < ntiles) {
                t2_stream_tile<W_KM>(g, ld);
                for (int p = 0; p < 2; ++p) {
                    fetch(ld);
                    t2_stream_next<W_KM>(g, g, ld, nwg, ntiles);
                }
            }
            for (uint32_t c_tile = blk; c_tile < ntiles; c_tile += nwg) {
                for (uint32_t ks = 0; ks < steps; ++ks) {
                    consumed.push_back(T2Cursor{c_tile, ks * (uint32_t)T2K});
                    if (ld.c.tile < ntiles) {
                        fetch(ld);
                        t2_stream_next<W_KM>(g, g, ld, nwg, ntiles);
                    } else {
                        stale(ld);   // the stream stands still past the last tile; its loads are issued all the same
                    }
                }
                // epilogue of this tile
                uint32_t tm, tn;
                tile_of_block(c_tile, g.tiles_m, g.tiles_n, tm, tn);
                for (uint32_t wave = 0; wave < 4; ++wave) {
                    const uint32_t wm = wave >> 1, wn = wave & 1u;
                    for (uint32_t lane = 0; lane < 64; ++lane) {
                        const uint32_t m_base = tm * (uint32_t)T2M + wm * 128u, n_lane = tn * (uint32_t)T2N + wn * 128u + (lane & 15u) * 8u;
                        const size_t col_off = g.store_mapped ? t2_store_col<true>(g, n_lane) : t2_store_col<false>(g, n_lane);
                        for (uint32_t i = 0; i < 4; ++i)
                            for (uint32_t pp = 0; pp < 8; ++pp) {
                                const uint32_t m = m_base + i * 32u + 4u * pp + (lane >> 4);
                                if (EDGE && !(m < g.M && n_lane < g.N)) continue;   // the kernel's store mask
                                const size_t off = g.store_mapped ? t2_store_off<true>(g, col_off, m) : t2_store_off<false>(g, col_off, m);
                                if (off % 8 || (int64_t)off + 8 > c_elems) {
                                    ++errors;
                                    continue;
                                }
                                if (written[off / 8]++) ++errors;
                            }
                    }
                }
            }
            if (fetched.size() != consumed.size()) ++errors;
            for (size_t i = 0; i < std::min(fetched.size(), consumed.size()); ++i)
                if (fetched[i].tile != consumed[i].tile || fetched[i].k0 != consumed[i].k0) ++errors;
        }
        for (uint8_t w : written)
            if (w != 1) ++errors;
        *n_errors = errors;
        return AMAP_OK;
    }
}
}  // namespace
