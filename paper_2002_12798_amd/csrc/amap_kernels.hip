// gfx950 kernels that execute a composed access map, and the device entry
// points amap_execute / amap_execute_kernel.
//
// Every kernel performs the rewritten load of the paper's eq. 4,
//     dst[i] = src[g(i)]      (or the fill constant outside every copy piece),
// for all i of the final tensor of a chain, without materialising any
// intermediate tensor.  Data are moved as opaque integers of 2..16 bytes.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <type_traits>

#include "amap_index.hpp"
#include "amap_plan.hpp"

using namespace amap_dev;
using namespace amap_detail;

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// VB-byte LDS accesses (VB = 4, 8, 16 go through dword vectors)
template <int VB>
__device__ __forceinline__ void ld(uint32_t (&r)[VB / 4], const void *p) {
    if constexpr (VB == 16) {
        u32x4 v = *reinterpret_cast<const u32x4 *>(p);
        r[0] = v.x, r[1] = v.y, r[2] = v.z, r[3] = v.w;
    } else if constexpr (VB == 8) {
        u32x2 v = *reinterpret_cast<const u32x2 *>(p);
        r[0] = v.x, r[1] = v.y;
    } else {
        r[0] = *reinterpret_cast<const uint32_t *>(p);
    }
}
template <int VB>
__device__ __forceinline__ void st(void *p, const uint32_t (&r)[VB / 4]) {
    if constexpr (VB == 16) {
        u32x4 v = {r[0], r[1], r[2], r[3]};
        *reinterpret_cast<u32x4 *>(p) = v;
    } else if constexpr (VB == 8) {
        u32x2 v = {r[0], r[1]};
        *reinterpret_cast<u32x2 *>(p) = v;
    } else {
        *reinterpret_cast<uint32_t *>(p) = r[0];
    }
}

// VB-byte global accesses.  Every source element is read once and every dst
// element written once, so where a wavefront covers whole 128-byte lines the
// accesses are issued non-temporal (streaming; a compile-time choice, since
// a run-time choice between the two forms is merged back into a plain access): the lines do not linger in the
// per-XCD L2s, which shortens the write-back at the end of the kernel.
// Loads may start at any element: the pointee types below carry 2-byte
// alignment only, and the hardware (in the unaligned access mode every HSA
// queue runs in) serves a 16-byte load from such an address with the same
// instruction.  A composed map often reads a source run that is shifted by a
// few elements against the 16-byte grid of dst (a slice offset, a dilated
// tap); dst vectors stay aligned, so only the loads need this.
typedef u32x4 u32x4_u __attribute__((aligned(2)));
typedef u32x2 u32x2_u __attribute__((aligned(2)));
typedef uint32_t u32_u __attribute__((aligned(2)));
template <int VB, bool NT>
__device__ __forceinline__ void gld(uint32_t (&r)[VB / 4], const void *p) {
    if constexpr (VB == 16) {
        u32x4 v;
        if constexpr (NT)
            v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
        else
            v = *reinterpret_cast<const u32x4_u *>(p);
        r[0] = v.x, r[1] = v.y, r[2] = v.z, r[3] = v.w;
    } else if constexpr (VB == 8) {
        u32x2 v;
        if constexpr (NT)
            v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
        else
            v = *reinterpret_cast<const u32x2_u *>(p);
        r[0] = v.x, r[1] = v.y;
    } else {
        if constexpr (NT)
            r[0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p));
        else
            r[0] = *reinterpret_cast<const u32_u *>(p);
    }
}
template <int VB, bool NT>
__device__ __forceinline__ void gst(void *p, const uint32_t (&r)[VB / 4]) {
    if constexpr (NT) {
        if constexpr (VB == 16) {
            u32x4 v = {r[0], r[1], r[2], r[3]};
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
        } else if constexpr (VB == 8) {
            u32x2 v = {r[0], r[1]};
            __builtin_nontemporal_store(v, reinterpret_cast<u32x2 *>(p));
        } else {
            __builtin_nontemporal_store(r[0], reinterpret_cast<uint32_t *>(p));
        }
    } else {
        st<VB>(p, r);
    }
}

// ------------------------------------------------------------------ rows
// One lane per vector of VB bytes, vectors enumerated in dst order, so the
// stores of a wavefront are contiguous; loads are contiguous per source run.
template <int VB, int NT>
__device__ __forceinline__ void rows_move(const DevPiece &P, char *dst, int es, const uint32_t (&doff)[kRowsUnroll],
                                          const uint32_t (&soff)[kRowsUnroll], const bool (&ok)[kRowsUnroll]) {
    if constexpr (VB == 2) {
        uint16_t v[kRowsUnroll];
#pragma unroll
        for (int u = 0; u < kRowsUnroll; ++u)
            v[u] = P.src && ok[u] ? *reinterpret_cast<const uint16_t *>((const char *)P.src + (size_t)soff[u] * es)
                                  : (uint16_t)P.fill;
#pragma unroll
        for (int u = 0; u < kRowsUnroll; ++u)
            if (ok[u]) *reinterpret_cast<uint16_t *>(dst + (size_t)doff[u] * es) = v[u];
    } else {
        uint32_t v[kRowsUnroll][VB / 4];
#pragma unroll
        for (int u = 0; u < kRowsUnroll; ++u) {
            if (P.src && ok[u]) {
                gld<VB, (NT & PF_NT_LOAD) != 0>(v[u], (const char *)P.src + (size_t)soff[u] * es);
            } else {
#pragma unroll
                for (int k = 0; k < VB / 4; ++k) v[u][k] = P.fill;
            }
        }
#pragma unroll
        for (int u = 0; u < kRowsUnroll; ++u)
            if (ok[u]) gst<VB, (NT & PF_NT_STORE) != 0>(dst + (size_t)doff[u] * es, v[u]);
    }
}

// The same for a row whose source elements are each repeated REP times in dst
// (REP a power of two): the lane loads 16 / REP bytes and spreads them over
// one 16-byte dst vector in registers.
template <int ES, int REP, int NT>
__device__ __forceinline__ void rows_expand(const DevPiece &P, char *dst, const uint32_t (&doff)[kRowsUnroll],
                                            const uint32_t (&soff)[kRowsUnroll], const bool (&ok)[kRowsUnroll]) {
    constexpr int SB = 16 / REP;           // source bytes per dst vector
    constexpr int SW = SB >= 4 ? SB / 4 : 1;
    uint32_t in[kRowsUnroll][SW];
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) {
        const char *s = (const char *)P.src + (size_t)soff[u] * ES;
        if (!ok[u]) {
#pragma unroll
            for (int k = 0; k < SW; ++k) in[u][k] = 0;
        } else if constexpr (SB >= 4) {
            gld<SB, (NT & PF_NT_LOAD) != 0>(in[u], s);
        } else {
            in[u][0] = *reinterpret_cast<const uint16_t *>(s);
        }
    }
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) {
        uint32_t out[4] = {0, 0, 0, 0};
        if constexpr (ES == 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i) out[i] = in[u][i / REP];
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = i / REP;  // source element of dst element i
                const uint32_t v = (in[u][e / 2] >> (16 * (e & 1))) & 0xFFFFu;
                out[i / 2] |= v << (16 * (i & 1));
            }
        }
        if (ok[u]) gst<16, (NT & PF_NT_STORE) != 0>(dst + (size_t)doff[u] * ES, out);
    }
}

// The same for a row read backwards: the lane loads the 16 bytes that end at its
// source element and reverses the elements in registers.
template <int ES, int NT>
__device__ __forceinline__ void rows_reverse(const DevPiece &P, char *dst, const uint32_t (&doff)[kRowsUnroll],
                                             const uint32_t (&soff)[kRowsUnroll], const bool (&ok)[kRowsUnroll]) {
    constexpr uint32_t V = 16 / ES;
    uint32_t in[kRowsUnroll][4];
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) {
        if (ok[u]) {
            gld<16, false>(in[u], (const char *)P.src + ((size_t)soff[u] - (V - 1)) * ES);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) in[u][k] = 0;
        }
    }
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) {
        uint32_t out[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t w = in[u][3 - k];
            out[k] = ES == 4 ? w : ((w >> 16) | (w << 16));
        }
        if (ok[u]) gst<16, (NT & PF_NT_STORE) != 0>(dst + (size_t)doff[u] * ES, out);
    }
}

// Gather rows: 16-byte dst vectors, every element fetched on its own through the run's loops.
// The loads of neighbouring lanes and elements share cache lines, so they stay temporal.
template <int ES, int NT, int NQ>
__device__ __forceinline__ void rows_gather(const DevPiece &P, char *dst, uint32_t base, uint32_t threads,
                                            const uint32_t (&doff)[kRowsUnroll], const uint32_t (&soff)[kRowsUnroll],
                                            const bool (&ok)[kRowsUnroll]) {
    constexpr int V = 16 / ES;
    uint32_t out[kRowsUnroll][4];
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) {
#pragma unroll
        for (int k = 0; k < 4; ++k) out[u][k] = 0;
        if (!ok[u]) continue;
        const uint32_t r = base + u * threads;
        const uint32_t rv = r - fdiv(r, P.loops[0].fd) * P.loops[0].extent;
        GatherCursor c = gather_begin<NQ>(P, rv * V);
        const char *s = (const char *)P.src;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const uint32_t at = soff[u] + c.off;  // 32-bit wrap-around: strides may be negative
            if constexpr (ES == 4) {
                out[u][e] = *reinterpret_cast<const uint32_t *>(s + (size_t)at * 4);
            } else {
                const uint32_t v = *reinterpret_cast<const uint16_t *>(s + (size_t)at * 2);
                out[u][e / 2] |= v << (16 * (e & 1));
            }
            if (e + 1 < V) gather_next<NQ>(P, c);
        }
    }
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u)
        if (ok[u]) gst<16, (NT & PF_NT_STORE) != 0>(dst + (size_t)doff[u] * ES, out[u]);
}

// Interleave / de-interleave rows (DevPiece::inter): E vectors in, E vectors out, shuffled in
// registers.  With a[p][q] the value of plane p at position q of the unit (V positions), the
// interleaved side holds a[p][q] at flat element q * E + p, the planar side at vector p, element q.
template <int ES, int NT, int E, int DIR>
__device__ __forceinline__ void rows_inter(const DevPiece &P, char *dst, const uint32_t (&doff)[kRowsUnroll],
                                           const uint32_t (&soff)[kRowsUnroll], const bool (&ok)[kRowsUnroll]) {
    constexpr int V = 16 / ES;
    const uint32_t plane = (uint32_t)P.ssP;
    auto get = [](const uint32_t (&r)[E][4], int flat) -> uint32_t {  // element `flat` of E consecutive vectors
        const uint32_t w = r[flat / V][(flat % V) * ES / 4];
        return ES == 4 ? w : ((w >> (16 * (flat & 1))) & 0xFFFFu);
    };
    auto put = [](uint32_t (&r)[E][4], int flat, uint32_t v) {
        if constexpr (ES == 4)
            r[flat / V][flat % V] = v;
        else
            r[flat / V][(flat % V) / 2] |= v << (16 * (flat & 1));
    };
    // one unit at a time: issuing the loads of two units before the first shuffle measured slower
    // (16.9 against 13.1 us on a batch of 3-channel images) and costs registers of every other path
#pragma unroll 1
    for (int u = 0; u < kRowsUnroll; ++u) {
        if (!ok[u]) continue;
        uint32_t in[E][4], out[E][4];
#pragma unroll
        for (int p = 0; p < E; ++p) {
            const uint32_t at = DIR == 1 ? soff[u] + (uint32_t)p * plane : soff[u] + (uint32_t)p * V;
            gld<16, (NT & PF_NT_LOAD) != 0>(in[p], (const char *)P.src + (size_t)at * ES);
#pragma unroll
            for (int k = 0; k < 4; ++k) out[p][k] = 0;
        }
        if constexpr (DIR >= 3) {  // one plane kept: the first (3) or the last (4) element of every group of E
#pragma unroll
            for (int q = 0; q < V; ++q) put(out, q, get(in, q * E + (DIR == 3 ? 0 : E - 1)));
            gst<16, (NT & PF_NT_STORE) != 0>(dst + (size_t)doff[u] * ES, out[0]);
            continue;
        }
#pragma unroll
        for (int p = 0; p < E; ++p)
#pragma unroll
            for (int q = 0; q < V; ++q) {
                if constexpr (DIR == 1)
                    put(out, q * E + p, get(in, p * V + q));
                else
                    put(out, p * V + q, get(in, q * E + p));
            }
#pragma unroll
        for (int p = 0; p < E; ++p) {
            const uint32_t at = DIR == 1 ? doff[u] + (uint32_t)p * V : doff[u] + (uint32_t)p * plane;
            gst<16, (NT & PF_NT_STORE) != 0>(dst + (size_t)at * ES, out[p]);
        }
    }
}

template <int ES, int NT>
__device__ __forceinline__ void rows_body(const DevPiece &P, char *dst, uint32_t blk, uint32_t tid) {
    uint32_t doff[kRowsUnroll], soff[kRowsUnroll];
    bool ok[kRowsUnroll];
    const uint32_t threads = 64u << P.nwlog;
    const uint32_t base = blk * (threads * kRowsUnroll) + tid;
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) {
        const uint32_t r = base + u * threads;
        ok[u] = r < P.n_units;
        rows_offsets(P, r, doff[u], soff[u]);
    }
    if (P.inter) {  // set only together with 16-byte vectors on both sides and a source
#define AMAP_INTER(E)                                                     \
    case E:                                                               \
        if (P.inter == 1)                                                 \
            rows_inter<ES, NT, E, 1>(P, dst, doff, soff, ok);             \
        else                                                              \
            rows_inter<ES, NT, E, 2>(P, dst, doff, soff, ok);             \
        break;
#define AMAP_INTER_KEEP(E)                                                \
    case E:                                                               \
        if (P.inter == 1)                                                 \
            rows_inter<ES, NT, E, 1>(P, dst, doff, soff, ok);             \
        else if (P.inter == 2)                                            \
            rows_inter<ES, NT, E, 2>(P, dst, doff, soff, ok);             \
        else if (P.inter == 3)                                            \
            rows_inter<ES, NT, E, 3>(P, dst, doff, soff, ok);             \
        else                                                              \
            rows_inter<ES, NT, E, 4>(P, dst, doff, soff, ok);             \
        break;
        switch (P.eP) {
            AMAP_INTER_KEEP(2)
            AMAP_INTER(3)
            AMAP_INTER(4)
            AMAP_INTER(5)
            AMAP_INTER(6)
            AMAP_INTER(7)
        default: break;
        }
#undef AMAP_INTER
#undef AMAP_INTER_KEEP
        return;
    }
    if (P.gather) {  // set only together with 16-byte dst vectors and a source
        switch (P.nq) {
        case 1: rows_gather<ES, NT, 1>(P, dst, base, threads, doff, soff, ok); break;
        case 2: rows_gather<ES, NT, 2>(P, dst, base, threads, doff, soff, ok); break;
        case 3: rows_gather<ES, NT, 3>(P, dst, base, threads, doff, soff, ok); break;
        default: rows_gather<ES, NT, 4>(P, dst, base, threads, doff, soff, ok); break;
        }
        return;
    }
    if (P.rev) {  // set only together with 16-byte dst vectors and a source
        rows_reverse<ES, NT>(P, dst, doff, soff, ok);
        return;
    }
    if (P.rep_log) {  // the planner only sets it together with 16-byte dst vectors and a source
        switch (P.rep_log) {
        case 1: rows_expand<ES, 2, NT>(P, dst, doff, soff, ok); break;
        case 2: rows_expand<ES, 4, NT>(P, dst, doff, soff, ok); break;
        default:
            if constexpr (ES == 2) rows_expand<2, 8, NT>(P, dst, doff, soff, ok);
            break;
        }
        return;
    }
    switch (ES << P.vlog) {
    case 16: rows_move<16, NT>(P, dst, ES, doff, soff, ok); break;
    case 8: rows_move<8, NT>(P, dst, ES, doff, soff, ok); break;
    case 4: rows_move<4, NT>(P, dst, ES, doff, soff, ok); break;
    default:
        if constexpr (ES == 2) rows_move<2, 0>(P, dst, ES, doff, soff, ok);
        break;
    }
}

// ------------------------------------------------------------------ tile
// Register micro-transpose: in[i] holds V elements along Q for P index i;
// out[j] holds V elements along P for Q index j.
template <int ES, int V>
__device__ __forceinline__ void micro_transpose(const uint32_t (&in)[V][ES * V / 4], uint32_t (&out)[V][ES * V / 4]) {
    if constexpr (ES == 4) {
#pragma unroll
        for (int i = 0; i < V; ++i)
#pragma unroll
            for (int j = 0; j < V; ++j) out[j][i] = in[i][j];
    } else {
#pragma unroll
        for (int j = 0; j < V; ++j)
#pragma unroll
            for (int i2 = 0; i2 < V / 2; ++i2) {
                const uint32_t a = in[2 * i2][j / 2], b = in[2 * i2 + 1][j / 2];
                out[j][i2] = (j & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
            }
    }
}

template <int ES, int V, bool USE_LDS, int NT, bool GROUPED>
__device__ __forceinline__ void tile_body(const DevPiece &P, char *dst, uint32_t t, uint32_t tid, char *smem) {
    constexpr int VB = ES * V;
    constexpr int NW = VB / 4;
    constexpr uint32_t VLOG = V == 8 ? 3 : V == 4 ? 2 : V == 2 ? 1 : 0;
    const TileGeom G = tile_geometry(P, VLOG, t);
    const TileLane L = tile_lane(P, G, VLOG, tid, GROUPED);

    uint32_t in[V][NW], out[V][NW];
    if (L.valid && L.src) {
        const char *s = (const char *)L.src + (size_t)L.soff * ES;
        const size_t pitch = (size_t)L.ssP * ES;
#pragma unroll
        for (int i = 0; i < V; ++i) gld<VB, (NT & PF_NT_LOAD) != 0>(in[i], s + i * pitch);
    } else {
        // lanes outside the piece, and lanes of a constant (fill) entry
#pragma unroll
        for (int i = 0; i < V; ++i)
#pragma unroll
            for (int k = 0; k < NW; ++k) in[i][k] = L.fill;
    }
    micro_transpose<ES, V>(in, out);

    if constexpr (!USE_LDS) {
        if (L.valid) {
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const uint32_t doff = G.db + q_chain_offset(P, L.w0 + j) + L.p;
                gst<VB, (NT & PF_NT_STORE) != 0>(dst + (size_t)doff * ES, out[j]);
            }
        }
    } else {
        if (L.valid) {
#pragma unroll
            for (int j = 0; j < V; ++j)
                st<VB>(smem + (size_t)tile_lds_slot(G, VLOG, L.r0 + j, L.pvl) * VB, out[j]);
        }
        __syncthreads();
        const uint32_t nvec = G.TQ << G.ncvlog;
        for (uint32_t vi = tid; vi < nvec; vi += (64u << P.nwlog)) {
            const TileStore S = tile_store(P, G, VLOG, vi);
            if (S.ok) {
                uint32_t v[NW];
                ld<VB>(v, smem + (size_t)S.slot * VB);
                gst<VB, (NT & PF_NT_STORE) != 0>(dst + (size_t)S.doff * ES, v);
            }
        }
    }
}

// ------------------------------------------------------------------ cross-lane tiles
// Short P runs (a dst row of at most 128 bytes, fills beside it included).  Every lane loads ONE 16-byte
// vector along Q and stores ONE 16-byte vector along P; in between, the V x V block held by the V lanes of
// a unit is transposed across those lanes with ds_bpermute (no LDS memory, no barrier).  Lane l stores
// vector l of the wavefront's tile in dst order, so a store instruction covers one contiguous run of dst
// whatever the row length: with the register micro-transpose the same stores are 16-byte pieces a row apart.
//   4-byte elements: 4 x 4 block over 4 lanes, three exchanges of one dword (round s: lane k sends its
//   element (k - s) % 4 to lane (k - s) % 4 ... i.e. reads from lane (k + s) % 4 what that lane holds for it).
//   2-byte elements: 8 x 8 block over 8 lanes: first the two lanes of a pair swap halves so that a dword holds
//   one element of each (4 exchanges), then the 4 x 4 transposition of dwords among the pairs (3 exchanges).
// v_i of four values held in registers (scalars on purpose: a select between elements of a local array is
// turned into an indexed load, which sends the array to scratch memory)
__device__ __forceinline__ uint32_t pick4(uint32_t v0, uint32_t v1, uint32_t v2, uint32_t v3, uint32_t i) {
    const uint32_t lo = (i & 1u) ? v1 : v0, hi = (i & 1u) ? v3 : v2;
    return (i & 2u) ? hi : lo;
}

// out D = value K (the reader's place) of the lane D places on in the ring of four lanes lane_of(0 .. 3)
template <class LaneOf>
__device__ __forceinline__ void ring_transpose4(uint32_t i0, uint32_t i1, uint32_t i2, uint32_t i3, uint32_t &o0, uint32_t &o1, uint32_t &o2,
                                                uint32_t &o3, uint32_t K, LaneOf lane_of) {
    const uint32_t g0 = pick4(i0, i1, i2, i3, K);
    const uint32_t g1 = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(lane_of((K + 1u) & 3u) << 2), (int)pick4(i0, i1, i2, i3, (K - 1u) & 3u));
    const uint32_t g2 = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(lane_of((K + 2u) & 3u) << 2), (int)pick4(i0, i1, i2, i3, (K - 2u) & 3u));
    const uint32_t g3 = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(lane_of((K + 3u) & 3u) << 2), (int)pick4(i0, i1, i2, i3, (K - 3u) & 3u));
    o0 = pick4(g0, g1, g2, g3, (0u - K) & 3u);
    o1 = pick4(g0, g1, g2, g3, (1u - K) & 3u);
    o2 = pick4(g0, g1, g2, g3, (2u - K) & 3u);
    o3 = pick4(g0, g1, g2, g3, (3u - K) & 3u);
}

template <int ES, int NT, bool GROUPED>
__device__ __forceinline__ void xlane_body(const DevPiece &P, char *dst, uint32_t blk, uint32_t tid) {
    constexpr uint32_t VLOG = ES == 2 ? 3 : 2;
    const uint32_t wave = tid >> 6, lane = tid & 63;
    const uint32_t t = (blk << P.nwlog) + wave;
    if (t >= P.n_units) return;  // the whole wavefront: no exchange partner is lost
    const TileGeom G = tile_geometry(P, VLOG, t);
    const XlaneLane L = xlane_lane(P, G, VLOG, lane, GROUPED);
    uint32_t in[4], out[4];
    if (L.ok && L.src) {
        gld<16, (NT & PF_NT_LOAD) != 0>(in, (const char *)L.src + (size_t)L.soff * ES);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) in[i] = L.fill;
    }
    const uint32_t npv = P.xl_npv;
    if constexpr (ES == 4) {
        ring_transpose4(in[0], in[1], in[2], in[3], out[0], out[1], out[2], out[3], L.k, [&](uint32_t j) { return L.lane0 + j * npv; });
    } else {
        // the pair (k, k ^ 1): afterwards dword d of the even lane holds element 2 d of both, of the odd lane element 2 d + 1
        const uint32_t partner = (L.lane0 + (L.k ^ 1u) * npv) << 2;
        uint32_t t2[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t o = (uint32_t)__builtin_amdgcn_ds_bpermute((int)partner, (int)in[d]);
            t2[d] = (L.k & 1u) ? ((o >> 16) | (in[d] & 0xFFFF0000u)) : ((in[d] & 0xFFFFu) | (o << 16));
        }
        const uint32_t r = L.k & 1u;
        ring_transpose4(t2[0], t2[1], t2[2], t2[3], out[0], out[1], out[2], out[3], L.k >> 1, [&](uint32_t j) { return L.lane0 + (2u * j + r) * npv; });
    }
    if (L.ok) gst<16, (NT & PF_NT_STORE) != 0>(dst + (size_t)L.doff * ES, out);
}

// ------------------------------------------------------------------ flat tiles
// A block of 64 rows that is one contiguous run on one side (see DevPiece::flat).  The run passes
// through LDS unchanged, in whole 16-byte vectors whatever the row length C is; the other side is
// served with 16-byte vectors along r (8 or 16 lanes per row of 64 elements, so a wavefront covers
// whole 128-byte row segments), whose elements are LDS accesses C elements apart.
template <int ES, int NT>
__device__ __forceinline__ void flat_body(const DevPiece &P, char *dst, uint32_t t, uint32_t tid, char *smem) {
    constexpr int V = 16 / ES;
    constexpr uint32_t VLOG = ES == 2 ? 3 : 2;
    const uint32_t RVLOG = P.lqlog - VLOG;  // log2(vectors per row of the block)
    constexpr int kBatch = 4;  // loads a lane has in flight
    typedef typename std::conditional<ES == 2, uint16_t, uint32_t>::type elem_t;
    const FlatUnit U = flat_unit(P, t);
    const uint32_t C = P.eP, threads = 64u << P.nwlog;
    const uint32_t nflat = (U.rcount * C) >> VLOG, nstr = C << RVLOG;
    elem_t *const lds = reinterpret_cast<elem_t *>(smem);
    const char *const src = (const char *)P.src;

    if (P.flat == 1) {
        for (uint32_t i0 = tid; i0 < nflat; i0 += kBatch * threads) {
            uint32_t v[kBatch][4];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const uint32_t i = i0 + b * threads;
                if (i < nflat) gld<16, (NT & PF_NT_LOAD) != 0>(v[b], src + (size_t)(U.soff + i * V) * ES);
            }
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const uint32_t i = i0 + b * threads;
                if (i < nflat) st<16>(smem + (size_t)i * 16, v[b]);
            }
        }
        __syncthreads();
        for (uint32_t vi = tid; vi < nstr; vi += threads) {
            const uint32_t rv = vi & ((1u << RVLOG) - 1), c = vi >> RVLOG;
            if (rv * V >= U.rcount) continue;
            uint32_t v[4] = {0, 0, 0, 0};
#pragma unroll
            for (int k = 0; k < V; ++k) {
                const uint32_t x = lds[(rv * V + k) * C + c];
                if constexpr (ES == 2)
                    v[k / 2] |= x << (16 * (k & 1));
                else
                    v[k] = x;
            }
            gst<16, (NT & PF_NT_STORE) != 0>(dst + (size_t)(U.doff + flat_c_offset(P, c) + rv * V) * ES, v);
        }
    } else {
        for (uint32_t v0 = tid; v0 < nstr; v0 += kBatch * threads) {
            uint32_t v[kBatch][4];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const uint32_t vi = v0 + b * threads, rv = vi & ((1u << RVLOG) - 1), c = vi >> RVLOG;
                if (vi < nstr && rv * V < U.rcount)
                    gld<16, (NT & PF_NT_LOAD) != 0>(v[b], src + (size_t)(U.soff + flat_c_offset(P, c) + rv * V) * ES);
            }
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const uint32_t vi = v0 + b * threads, rv = vi & ((1u << RVLOG) - 1), c = vi >> RVLOG;
                if (vi < nstr && rv * V < U.rcount) {
#pragma unroll
                    for (int k = 0; k < V; ++k) {
                        if constexpr (ES == 2)
                            lds[(rv * V + k) * C + c] = (uint16_t)(v[b][k / 2] >> (16 * (k & 1)));
                        else
                            lds[(rv * V + k) * C + c] = v[b][k];
                    }
                }
            }
        }
        __syncthreads();
        for (uint32_t i = tid; i < nflat; i += threads) {
            uint32_t v[4];
            ld<16>(v, smem + (size_t)i * 16);
            gst<16, (NT & PF_NT_STORE) != 0>(dst + (size_t)(U.doff + i * V) * ES, v);
        }
    }
}

// The same for rows too long for LDS: blocks of rows x rag_cb columns (see DevPiece::rag_cb).
template <int ES, int NT>
__device__ __forceinline__ void rag_body(const DevPiece &P, char *dst, uint32_t t, uint32_t tid, char *smem) {
    constexpr uint32_t V = 16 / ES;
    constexpr uint32_t VLOG = ES == 2 ? 3 : 2;
    const uint32_t RVLOG = P.lqlog - VLOG;
    constexpr int kBatch = 4;
    typedef typename std::conditional<ES == 2, uint16_t, uint32_t>::type elem_t;
    const RagUnit U = rag_unit(P, t);
    const uint32_t C = P.eP, W = P.rag_w, S = P.rag_s, threads = 64u << P.nwlog;
    const uint32_t nrag = U.rcount * S, nstr = U.ccount << RVLOG;
    elem_t *const lds = reinterpret_cast<elem_t *>(smem);
    const char *const src = (const char *)P.src;

    if (P.flat == 1) {
        for (uint32_t item = tid; item < nrag; item += threads) {
            const uint32_t r = fdiv(item, P.fd_rag_s), col = (item - r * S) * V;
            if (col >= U.ccount) continue;
            const uint32_t a = U.soff + r * C + col, at = r * W + col;
            if (col + V <= U.ccount) {
                uint32_t v[4];
                gld<16, false>(v, src + (size_t)a * ES);
#pragma unroll
                for (int k = 0; k < 4; ++k) reinterpret_cast<uint32_t *>(smem)[(at * ES) / 4 + k] = v[k];
            } else {
                for (uint32_t i = 0; col + i < U.ccount; ++i) lds[at + i] = reinterpret_cast<const elem_t *>(src)[a + i];
            }
        }
        __syncthreads();
        for (uint32_t vi = tid; vi < nstr; vi += threads) {
            const uint32_t rv = vi & ((1u << RVLOG) - 1), c = vi >> RVLOG;
            if (rv * V >= U.rcount) continue;
            uint32_t v[4] = {0, 0, 0, 0};
#pragma unroll
            for (uint32_t k = 0; k < V; ++k) {
                const uint32_t x = lds[(rv * V + k) * W + c];
                if constexpr (ES == 2)
                    v[k / 2] |= x << (16 * (k & 1));
                else
                    v[k] = x;
            }
            gst<16, (NT & PF_NT_STORE) != 0>(dst + (size_t)(U.doff + flat_c_offset(P, U.c0 + c) + rv * V) * ES, v);
        }
    } else {
        for (uint32_t v0 = tid; v0 < nstr; v0 += kBatch * threads) {
            uint32_t v[kBatch][4];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const uint32_t vi = v0 + b * threads, rv = vi & ((1u << RVLOG) - 1), c = vi >> RVLOG;
                if (vi < nstr && rv * V < U.rcount) {
                    const uint32_t a = U.soff + flat_c_offset(P, U.c0 + c) + rv * V;
                    if (rv * V + V <= U.rcount) {
                        gld<16, (NT & PF_NT_LOAD) != 0>(v[b], src + (size_t)a * ES);
                    } else {  // the last rows of a row count that is no whole number of vectors
#pragma unroll
                        for (int k = 0; k < 4; ++k) v[b][k] = 0;
                        for (uint32_t k = 0; rv * V + k < U.rcount; ++k) {
                            const uint32_t e = reinterpret_cast<const elem_t *>(src)[a + k];
                            if constexpr (ES == 2)
                                v[b][k / 2] |= e << (16 * (k & 1));
                            else
                                v[b][k] = e;
                        }
                    }
                }
            }
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const uint32_t vi = v0 + b * threads, rv = vi & ((1u << RVLOG) - 1), c = vi >> RVLOG;
                if (vi < nstr && rv * V < U.rcount) {
#pragma unroll
                    for (uint32_t k = 0; k < V; ++k) {
                        if (rv * V + k >= U.rcount) break;
                        if constexpr (ES == 2)
                            lds[(rv * V + k) * W + c] = (uint16_t)(v[b][k / 2] >> (16 * (k & 1)));
                        else
                            lds[(rv * V + k) * W + c] = v[b][k];
                    }
                }
            }
        }
        __syncthreads();
        for (uint32_t item = tid; item < nrag; item += threads) {
            const uint32_t r = fdiv(item, P.fd_rag_s), s = item - r * S;
            const uint32_t a = U.doff + r * C;                 // first dst element of the row segment
            const uint32_t x = (a & ~(V - 1)) + s * V;         // the aligned slot
            const uint32_t lo = x > a ? x : a, hi = x + V < a + U.ccount ? x + V : a + U.ccount;
            if (lo >= hi) continue;
            if (hi - lo == V) {
                uint32_t v[4] = {0, 0, 0, 0};
#pragma unroll
                for (uint32_t k = 0; k < V; ++k) {
                    const uint32_t e = lds[r * W + (x - a) + k];
                    if constexpr (ES == 2)
                        v[k / 2] |= e << (16 * (k & 1));
                    else
                        v[k] = e;
                }
                gst<16, false>(dst + (size_t)x * ES, v);
            } else {
                for (uint32_t p = lo; p < hi; ++p) reinterpret_cast<elem_t *>(dst)[p] = lds[r * W + (p - a)];
            }
        }
    }
}

template <int ES, bool USE_LDS, int NT, bool GROUPED>
__device__ __forceinline__ void tile_dispatch(const DevPiece &P, char *dst, uint32_t t, uint32_t tid, char *smem) {
    if constexpr (ES == 2) {
        switch (P.vlog) {
        case 3: tile_body<2, 8, USE_LDS, NT, GROUPED>(P, dst, t, tid, smem); break;
        case 2: tile_body<2, 4, USE_LDS, NT, GROUPED>(P, dst, t, tid, smem); break;
        default: tile_body<2, 2, USE_LDS, NT, GROUPED>(P, dst, t, tid, smem); break;
        }
    } else {
        switch (P.vlog) {
        case 2: tile_body<4, 4, USE_LDS, NT, GROUPED>(P, dst, t, tid, smem); break;
        case 1: tile_body<4, 2, USE_LDS, NT, GROUPED>(P, dst, t, tid, smem); break;
        default: tile_body<4, 1, USE_LDS, NT, GROUPED>(P, dst, t, tid, smem); break;
        }
    }
}

// One launch executes up to kMaxPiecesPerLaunch pieces: each workgroup finds
// its piece from the block ranges and runs that piece's body.  GROUPED is set
// by the host when some tile piece of the launch is a group of more than one
// entry; the two forms are separate kernels so that each stays small enough
// for the compiler to read the argument block in place (scalar loads) instead
// of copying it to private memory.
template <int ES, int NT, bool GROUPED>
__global__ __launch_bounds__(kMaxThreads) void amap_pieces_kernel(const LaunchArgs args, char *dst) {
    extern __shared__ uint4 smem_v[];
    const uint32_t b = logical_block(args, blockIdx.x, gridDim.x);
    uint32_t pi = 0;
    for (uint32_t k = 1; k < args.n_pieces; ++k)
        if (args.p[k].n_blocks && b >= args.p[k].first_block) pi = k;
    const DevPiece &P = args.p[pi];
    const uint32_t local = b - P.first_block;
    char *const d = dst + (size_t)P.dwin * ES;
    if (P.kind == PK_ROWS)
        rows_body<ES, NT>(P, d, local, threadIdx.x);
    else if (P.kind == PK_XLANE)
        xlane_body<ES, NT, GROUPED>(P, d, local, threadIdx.x);
    else if (P.kind == PK_TILE)
        tile_dispatch<ES, true, NT, GROUPED>(P, d, local, threadIdx.x, reinterpret_cast<char *>(smem_v));
    else if (P.kind == PK_FLAT && P.rag_cb)
        rag_body<ES, NT>(P, d, local, threadIdx.x, reinterpret_cast<char *>(smem_v));
    else if (P.kind == PK_FLAT)
        flat_body<ES, NT>(P, d, local, threadIdx.x, reinterpret_cast<char *>(smem_v));
    else
        tile_dispatch<ES, false, NT, GROUPED>(P, d, local, threadIdx.x, nullptr);
}

// ------------------------------------------------------------------ one plain row piece
// The launch that most row maps come down to (a head split or merge, a permutation of outer
// dimensions, a broadcast, a plain copy): one piece, 16-byte vectors, nothing to reshuffle.  Same
// schedule as rows_body (one lane per vector in dst order, kRowsUnroll vectors per lane), without the
// piece search and the dispatch over forms in front of it.
template <int ES, int NT>
__global__ __launch_bounds__(kMaxThreads) void amap_rows_kernel(const DevPiece P, char *dst) {
    uint32_t doff[kRowsUnroll], soff[kRowsUnroll];
    bool ok[kRowsUnroll];
    const uint32_t threads = blockDim.x;
    const uint32_t base = blockIdx.x * (threads * kRowsUnroll) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) {
        const uint32_t r = base + u * threads;
        ok[u] = r < P.n_units;
        rows_offsets_fixed(P, r, doff[u], soff[u]);
    }
    rows_move<16, NT>(P, dst + (size_t)P.dwin * ES, ES, doff, soff, ok);
}

// The same for a launch of several plain row pieces: the piece is looked up, the rest is alike.
template <int ES, int NT>
__global__ __launch_bounds__(kMaxThreads) void amap_rows_multi_kernel(const LaunchArgs args, char *dst) {
    const uint32_t b = blockIdx.x;
    uint32_t pi = 0;
    for (uint32_t k = 1; k < args.n_pieces; ++k)
        if (b >= args.p[k].first_block) pi = k;
    const DevPiece &P = args.p[pi];
    uint32_t doff[kRowsUnroll], soff[kRowsUnroll];
    bool ok[kRowsUnroll];
    const uint32_t threads = blockDim.x;
    const uint32_t base = (b - P.first_block) * (threads * kRowsUnroll) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) {
        const uint32_t r = base + u * threads;
        ok[u] = r < P.n_units;
        rows_offsets_fixed(P, r, doff[u], soff[u]);
    }
    rows_move<16, NT>(P, dst + (size_t)P.dwin * ES, ES, doff, soff, ok);
}

// ------------------------------------------------------------------ one tile piece + plain rows
// The launch of a transposing map (NCHW -> NHWC with or without padding, a concat in front of it):
// piece 0 is known without a search and its fields sit at fixed places of the argument block; only
// the workgroups behind it (constant borders) look their piece up.
template <int ES, int NT, bool GROUPED>
__global__ __launch_bounds__(kMaxThreads) void amap_tile16_kernel(const LaunchArgs args, char *dst) {
    extern __shared__ uint4 smem_v[];
    const uint32_t b = logical_block(args, blockIdx.x, gridDim.x);
    if (b < args.p[0].n_blocks) {
        tile_body<ES, 16 / ES, true, NT, GROUPED>(args.p[0], dst + (size_t)args.p[0].dwin * ES, b, threadIdx.x,
                                                   reinterpret_cast<char *>(smem_v));
        return;
    }
    uint32_t pi = args.p[0].group_n;
    for (uint32_t k = pi + 1; k < args.n_pieces; ++k)
        if (b >= args.p[k].first_block) pi = k;
    const DevPiece &P = args.p[pi];
    uint32_t doff[kRowsUnroll], soff[kRowsUnroll];
    bool ok[kRowsUnroll];
    const uint32_t threads = blockDim.x;
    const uint32_t base = (b - P.first_block) * (threads * kRowsUnroll) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < kRowsUnroll; ++u) {
        const uint32_t r = base + u * threads;
        ok[u] = r < P.n_units;
        rows_offsets_fixed(P, r, doff[u], soff[u]);
    }
    rows_move<16, NT>(P, dst + (size_t)P.dwin * ES, ES, doff, soff, ok);
}

// ------------------------------------------------------------------ program
// Element-wise interpreter of the operator program: applies the index
// function of every operator of the chain in turn (eq. 4 evaluated lazily).
// Handles any map, at one dst element per lane.
template <int ES>
__global__ __launch_bounds__(kProgramThreads) void amap_program_kernel(const Program prog, const SrcTable srcs, char *dst,
                                                               uint32_t total) {
    const uint32_t L = blockIdx.x * kProgramThreads + threadIdx.x;
    if (L >= total) return;
    int32_t idx[8], tmp[8];
    {
        uint32_t r = L;
        for (int k = prog.rank - 1; k >= 0; --k) {
            idx[k] = (int32_t)(r % (uint32_t)prog.shape[k]);
            r /= (uint32_t)prog.shape[k];
        }
    }
    int pc = 0;
    uint32_t value = 0;
    for (;;) {
        const Instr &I = prog.ins[pc];
        if (I.kind == I_SOURCE) {
            uint32_t off = 0;
            for (int k = 0; k < I.rank; ++k) off = off * (uint32_t)I.v[k] + (uint32_t)idx[k];
            const char *s = (const char *)srcs.p[I.a];
            value = ES == 2 ? *reinterpret_cast<const uint16_t *>(s + (size_t)off * 2)
                            : *reinterpret_cast<const uint32_t *>(s + (size_t)off * 4);
            break;
        } else if (I.kind == I_TRANSPOSE) {
            for (int k = 0; k < I.rank; ++k) tmp[I.v[k]] = idx[k];
            for (int k = 0; k < I.rank; ++k) idx[k] = tmp[k];
            ++pc;
        } else if (I.kind == I_RESHAPE) {
            uint32_t r = 0;
            for (int k = 0; k < I.rank; ++k) r = r * (uint32_t)I.v[k] + (uint32_t)idx[k];
            for (int k = I.a - 1; k >= 0; --k) {
                idx[k] = (int32_t)(r % (uint32_t)I.w[k]);
                r /= (uint32_t)I.w[k];
            }
            ++pc;
        } else if (I.kind == I_SLICE) {
            idx[I.a] = I.v[0] + idx[I.a] * I.v[1];
            ++pc;
        } else if (I.kind == I_REPEAT) {
            idx[I.a] = (int32_t)((uint32_t)idx[I.a] / (uint32_t)I.b);
            ++pc;
        } else if (I.kind == I_TILE) {
            idx[I.a] = (int32_t)((uint32_t)idx[I.a] % (uint32_t)I.b);
            ++pc;
        } else if (I.kind == I_PAD) {
            bool inside = true;
            for (int k = 0; k < I.rank; ++k) {
                idx[k] -= I.v[k];
                inside = inside && idx[k] >= 0 && idx[k] < I.w[k];
            }
            if (!inside) {
                value = (uint32_t)I.b;
                break;
            }
            ++pc;
        } else {  // I_CONCAT
            int32_t x = idx[I.a];
            int m = 0;
            while (m + 1 < I.b && x >= I.v[m]) {
                x -= I.v[m];
                ++m;
            }
            idx[I.a] = x;
            pc = I.w[m];
        }
    }
    if (ES == 2)
        *reinterpret_cast<uint16_t *>(dst + (size_t)L * 2) = (uint16_t)value;
    else
        *reinterpret_cast<uint32_t *>(dst + (size_t)L * 4) = value;
}

// ------------------------------------------------------------------ host side

// An error left on this thread by an earlier, unrelated HIP call must not be read as the failure
// of the launch that follows: called right before every launch, launch_failed right after it.
void clear_stale_error() { (void)hipGetLastError(); }

// true if the launch just made left an error
bool launch_failed(const char *what) {
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return false;
    char detail[200];
    std::snprintf(detail, sizeof(detail), "%s (%s)", hipGetErrorString(e), hipGetErrorName(e));
    set_last_error(what, detail);
    return true;
}

bool overlaps(const void *a, int64_t an, const void *b, int64_t bn) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + (uintptr_t)bn && b0 < a0 + (uintptr_t)an;
}

amap_status check_pointers(const amap *m, const void *const *src, const void *dst) {
    const int es = m->elem;
    const int64_t dbytes = volume_of(m->shape) * es;
    if (!dst || ((uintptr_t)dst & 15)) return AMAP_E_INVALID;
    for (size_t i = 0; i < m->src_shapes.size(); ++i) {
        if (m->src_shapes[i].empty()) continue;
        if (!src[i] || ((uintptr_t)src[i] & 15)) return AMAP_E_INVALID;
        if (overlaps(dst, dbytes, src[i], volume_of(m->src_shapes[i]) * es)) return AMAP_E_ALIAS;
    }
    return AMAP_OK;
}

// one launch of the piece kernel; args.p[].src must already hold device pointers
amap_status launch_pieces(const LaunchArgs &args, uint32_t blocks, size_t lds, int es, char *d, hipStream_t stream) {
    bool grouped = false;
    for (uint32_t k = 0; k < args.n_pieces; ++k)
        grouped = grouped || (args.p[k].kind != PK_ROWS && args.p[k].group_n > 1);
    const dim3 grid(blocks), block(64u << args.nwlog);
    clear_stale_error();
    const char *tr = std::getenv("AMAP_PLAN_TRACE");
    const bool trace = tr && tr[0] && tr[0] != '0';   // one line per launch on stderr: the kernel that takes it
    auto say = [&](const char *kernel) {
        if (trace) std::fprintf(stderr, "amap launch: %s, %u workgroups of %u lanes, %u pieces\n", kernel, blocks, 64u << args.nwlog, args.n_pieces);
    };
    if (args.n_pieces == 1 && rows_is_plain(args.p[0], es)) {
        say("amap_rows_kernel");
        const DevPiece &P = args.p[0];
#define AMAP_LAUNCH_ROWS(ES, NT) hipLaunchKernelGGL((amap_rows_kernel<ES, NT>), grid, block, 0, stream, P, d)
        switch ((es == 2 ? 0 : 4) + (int)(args.nt & 3)) {
        case 0: AMAP_LAUNCH_ROWS(2, 0); break;
        case 1: AMAP_LAUNCH_ROWS(2, 1); break;
        case 2: AMAP_LAUNCH_ROWS(2, 2); break;
        case 3: AMAP_LAUNCH_ROWS(2, 3); break;
        case 4: AMAP_LAUNCH_ROWS(4, 0); break;
        case 5: AMAP_LAUNCH_ROWS(4, 1); break;
        case 6: AMAP_LAUNCH_ROWS(4, 2); break;
        default: AMAP_LAUNCH_ROWS(4, 3); break;
        }
#undef AMAP_LAUNCH_ROWS
        return launch_failed("amap_rows_kernel") ? AMAP_E_HIP : AMAP_OK;
    }
    if (launch_is_plain_rows(args, es)) {
        say("amap_rows_multi_kernel");
#define AMAP_LAUNCH_ROWSM(ES, NT) hipLaunchKernelGGL((amap_rows_multi_kernel<ES, NT>), grid, block, 0, stream, args, d)
        switch ((es == 2 ? 0 : 4) + (int)(args.nt & 3)) {
        case 0: AMAP_LAUNCH_ROWSM(2, 0); break;
        case 1: AMAP_LAUNCH_ROWSM(2, 1); break;
        case 2: AMAP_LAUNCH_ROWSM(2, 2); break;
        case 3: AMAP_LAUNCH_ROWSM(2, 3); break;
        case 4: AMAP_LAUNCH_ROWSM(4, 0); break;
        case 5: AMAP_LAUNCH_ROWSM(4, 1); break;
        case 6: AMAP_LAUNCH_ROWSM(4, 2); break;
        default: AMAP_LAUNCH_ROWSM(4, 3); break;
        }
#undef AMAP_LAUNCH_ROWSM
        return launch_failed("amap_rows_multi_kernel") ? AMAP_E_HIP : AMAP_OK;
    }
    if (launch_is_tile16(args, es)) {
        say("amap_tile16_kernel");
#define AMAP_LAUNCH_T16(ES, NT)                                                                              \
    do {                                                                                                     \
        if (grouped)                                                                                         \
            hipLaunchKernelGGL((amap_tile16_kernel<ES, NT, true>), grid, block, lds, stream, args, d);       \
        else                                                                                                 \
            hipLaunchKernelGGL((amap_tile16_kernel<ES, NT, false>), grid, block, lds, stream, args, d);      \
    } while (0)
        switch ((es == 2 ? 0 : 4) + (int)(args.nt & 3)) {
        case 0: AMAP_LAUNCH_T16(2, 0); break;
        case 1: AMAP_LAUNCH_T16(2, 1); break;
        case 2: AMAP_LAUNCH_T16(2, 2); break;
        case 3: AMAP_LAUNCH_T16(2, 3); break;
        case 4: AMAP_LAUNCH_T16(4, 0); break;
        case 5: AMAP_LAUNCH_T16(4, 1); break;
        case 6: AMAP_LAUNCH_T16(4, 2); break;
        default: AMAP_LAUNCH_T16(4, 3); break;
        }
#undef AMAP_LAUNCH_T16
        return launch_failed("amap_tile16_kernel") ? AMAP_E_HIP : AMAP_OK;
    }
    say("amap_pieces_kernel");
#define AMAP_LAUNCH(ES, NT)                                                                                  \
    do {                                                                                                     \
        if (grouped)                                                                                         \
            hipLaunchKernelGGL((amap_pieces_kernel<ES, NT, true>), grid, block, lds, stream, args, d);       \
        else                                                                                                 \
            hipLaunchKernelGGL((amap_pieces_kernel<ES, NT, false>), grid, block, lds, stream, args, d);      \
    } while (0)
    switch ((es == 2 ? 0 : 4) + (int)(args.nt & 3)) {
    case 0: AMAP_LAUNCH(2, 0); break;
    case 1: AMAP_LAUNCH(2, 1); break;
    case 2: AMAP_LAUNCH(2, 2); break;
    case 3: AMAP_LAUNCH(2, 3); break;
    case 4: AMAP_LAUNCH(4, 0); break;
    case 5: AMAP_LAUNCH(4, 1); break;
    case 6: AMAP_LAUNCH(4, 2); break;
    default: AMAP_LAUNCH(4, 3); break;
    }
#undef AMAP_LAUNCH
    return launch_failed("amap_pieces_kernel") ? AMAP_E_HIP : AMAP_OK;
}

void patch_sources(LaunchArgs &args, const void *const *src, int es) {
    for (uint32_t k = 0; k < args.n_pieces; ++k) {
        const uintptr_t id = (uintptr_t)args.p[k].src;
        args.p[k].src = id ? (const char *)src[id - 1] + (size_t)args.p[k].swin * (size_t)es : nullptr;
    }
}

amap_status launch_strided(const amap *m, const Plan &plan, const void *const *src, void *dst, hipStream_t stream) {
    for (size_t i = 0; i < plan.launches.size(); ++i) {
        LaunchArgs args = plan.launches[i];
        patch_sources(args, src, m->elem);
        amap_status st = launch_pieces(args, plan.grid[i], plan.lds_bytes[i], m->elem, (char *)dst, stream);
        if (st != AMAP_OK) return st;
    }
    return AMAP_OK;
}

// AMAP_E_UNSUPPORTED with the reason left for amap_last_error
amap_status refuse(const char *why) {
    set_last_error("unsupported", why);
    return AMAP_E_UNSUPPORTED;
}

amap_status launch_program(const amap *m, const Plan &plan, const void *const *src, void *dst, hipStream_t stream) {
    if (!plan.program_ok)
        return refuse("the map has no strided form and its operator program exceeds the interpreter (16 sources, 24 operators)");
    SrcTable t;
    std::memset(&t, 0, sizeof(t));
    // leaves of the program that no dst index reaches are not arguments of the map
    for (int i = 0; i < plan.n_prog_src && i < (int)m->src_shapes.size(); ++i) t.p[i] = src[i];
    const uint32_t total = (uint32_t)volume_of(m->shape);
    const uint32_t grid = (total + kProgramThreads - 1) / kProgramThreads;
    clear_stale_error();
    if (m->elem == 2)
        hipLaunchKernelGGL(amap_program_kernel<2>, dim3(grid), dim3(kProgramThreads), 0, stream, plan.prog, t, (char *)dst, total);
    else
        hipLaunchKernelGGL(amap_program_kernel<4>, dim3(grid), dim3(kProgramThreads), 0, stream, plan.prog, t, (char *)dst, total);
    return launch_failed("amap_program_kernel") ? AMAP_E_HIP : AMAP_OK;
}

}  // namespace

extern "C" amap_status amap_execute_kernel(const void *const *src, void *dst, const amap_t *map, void *stream,
                                           int kernel_id) {
    if (!map || kernel_id < -1 || kernel_id > AMAP_K_WAVE) return AMAP_E_INVALID;
    if (volume_of(map->shape) == 0) return AMAP_OK;
    if (!src && !map->src_shapes.empty()) return AMAP_E_INVALID;
    amap_status st = check_pointers(map, src, dst);
    if (st != AMAP_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    try {
        if (kernel_id < 0) {
            const Plan *plan = plan_of(*map);
            if (!plan) return refuse("no launch plan");
            if (plan->strided_ok) return launch_strided(map, *plan, src, dst, s);
            if (!plan->fits32) return refuse("the map has no strided form and a tensor of 2^31 elements or more (the interpreter works in 32-bit indices)");
            return launch_program(map, *plan, src, dst, s);
        }
        Plan forced;
        if (kernel_id == AMAP_K_PROGRAM) {
            plan_strided(*map, -1, forced);  // sets fits32
            if (!forced.fits32 || !plan_program(*map, forced)) return refuse("the operator program exceeds the interpreter");
            return launch_program(map, forced, src, dst, s);
        }
        if (!plan_strided(*map, kernel_id, forced)) return refuse("the forced kernel family cannot execute this map");
        return launch_strided(map, forced, src, dst, s);
    } catch (...) {
        return AMAP_E_NOMEM;
    }
}

// Several maps over one source table, each with its own dst, in as few launches
// as their pieces fit: the pieces of all maps are packed into shared launches,
// every piece carrying the offset of its own dst from the lowest dst address.
extern "C" amap_status amap_execute_multi(const void *const *src, void *const *dst, const amap_t *const *maps, int n,
                                          void *stream) {
    if (!dst || !maps || n < 1) return AMAP_E_INVALID;
    for (int i = 0; i < n; ++i)
        if (!maps[i] || !dst[i]) return AMAP_E_INVALID;
    const int es = maps[0]->elem;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    try {
        uintptr_t base = UINTPTR_MAX;
        for (int i = 0; i < n; ++i) {
            const amap *m = maps[i];
            if (m->elem != es) return AMAP_E_INVALID;
            if (volume_of(m->shape) == 0) continue;
            if (!src && !m->src_shapes.empty()) return AMAP_E_INVALID;
            amap_status st = check_pointers(m, src, dst[i]);
            if (st != AMAP_OK) return st;
            for (int j = 0; j < i; ++j)
                if (volume_of(maps[j]->shape) > 0 &&
                    overlaps(dst[i], volume_of(m->shape) * es, dst[j], volume_of(maps[j]->shape) * es))
                    return AMAP_E_ALIAS;
            base = std::min(base, (uintptr_t)dst[i]);
        }
        if (base == UINTPTR_MAX) return AMAP_OK;  // nothing to write
        LaunchArgs cur;
        uint32_t blocks = 0, lds = 0;
        std::memset(&cur, 0, sizeof(cur));
        auto flush = [&]() -> amap_status {
            if (cur.n_pieces == 0) return AMAP_OK;
            amap_status st = launch_pieces(cur, blocks, lds, es, reinterpret_cast<char *>(base), s);
            std::memset(&cur, 0, sizeof(cur));
            blocks = 0;
            lds = 0;
            return st;
        };
        for (int i = 0; i < n; ++i) {
            const amap *m = maps[i];
            if (volume_of(m->shape) == 0) continue;
            const Plan *plan = plan_of(*m);
            if (!plan) return refuse("no launch plan");
            if (!plan->strided_ok) {  // no strided form: this one runs on its own, through the interpreter
                amap_status st = flush();
                if (st != AMAP_OK) return st;
                if (!plan->fits32) return refuse("a map without strided form over a tensor of 2^31 elements or more");
                st = launch_program(m, *plan, src, dst[i], s);
                if (st != AMAP_OK) return st;
                continue;
            }
            const uint64_t shift = ((uintptr_t)dst[i] - base) / (uint64_t)es;  // dst pointers are 16-byte aligned
            for (size_t j = 0; j < plan->launches.size(); ++j) {
                LaunchArgs a = plan->launches[j];
                patch_sources(a, src, es);
                const bool fits = cur.n_pieces == 0 ||
                                  (cur.nwlog == a.nwlog && cur.n_pieces + a.n_pieces <= (uint32_t)kMaxPiecesPerLaunch &&
                                   (uint64_t)blocks + plan->grid[j] < (1u << 31));
                if (!fits) {
                    amap_status st = flush();
                    if (st != AMAP_OK) return st;
                }
                if (cur.n_pieces == 0) {
                    cur.nwlog = a.nwlog;
                    cur.nt = a.nt;
                } else {
                    cur.nt &= a.nt;
                }
                cur.xcd_remap |= a.xcd_remap;
                for (uint32_t k = 0; k < a.n_pieces; ++k) {
                    DevPiece p = a.p[k];
                    p.first_block += blocks;
                    p.dwin += shift;
                    cur.p[cur.n_pieces++] = p;
                }
                blocks += plan->grid[j];
                lds = std::max<uint32_t>(lds, plan->lds_bytes[j]);
            }
        }
        return flush();
    } catch (...) {
        return AMAP_E_NOMEM;
    }
}

extern "C" amap_status amap_execute(const void *const *src, void *dst, const amap_t *map, void *stream) {
    return amap_execute_kernel(src, dst, map, stream, -1);
}

