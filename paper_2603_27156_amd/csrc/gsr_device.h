// Device-side building blocks for gfx950 (wave64): storage conversion, sub-wave reductions,
// the exact top-k select of the GS operator, neighbour gathers and 16x16x4 float32 MFMA tiles.
//
// Thread layout used everywhere ("row layout"): a row of a group has DG = 32 or 64 columns;
// lane c of a (sub-)wave owns column c.  With DG = 64 a wave holds one row, with DG = 32 it
// holds two rows (lanes 0..31 and 32..63, `sub` = lane / DG).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gsr {

struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

template <typename T>
__device__ __forceinline__ T from_float(float v);
template <>
__device__ __forceinline__ float from_float<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float v) {
    // round to nearest even; inputs are finite by contract
    uint32_t b = __float_as_uint(v);
    b = b + 0x7FFFu + ((b >> 16) & 1u);
    bf16_t r;
    r.bits = (uint16_t)(b >> 16);
    return r;
}

// value as it will read back after a store of type T
template <typename T>
__device__ __forceinline__ float stored(float v) { return to_float(from_float<T>(v)); }

template <int DG>
struct MaskOf;
template <>
struct MaskOf<32> { using type = uint32_t; };
template <>
struct MaskOf<64> { using type = uint64_t; };

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Orders this wave's LDS traffic: everything before is complete and visible to the other lanes
// of the wave before anything after is issued.  (A wave runs in lock step; only the compiler
// and the LDS queue need to be told.)
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ uint64_t ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// bits of a wave-wide ballot that belong to this lane's row
template <int DG>
__device__ __forceinline__ typename MaskOf<DG>::type sub_bits(uint64_t m, int sub) {
    if constexpr (DG == 64) return m;
    else return (uint32_t)(m >> (32 * sub));
}

template <int DG>
__device__ __forceinline__ int popc(typename MaskOf<DG>::type m) {
    if constexpr (DG == 64) return __popcll(m);
    else return __popc(m);
}

// sum over the DG lanes of this lane's row, same value (and same order) in every lane
template <int DG>
__device__ __forceinline__ float sub_sum(float v) {
#pragma unroll
    for (int off = DG / 2; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ---- GS: exact top-k of a row ----------------------------------------------------------------
// The Group-Sparse operator of Section 4.1 of the paper keeps, per row, the k largest entries by
// signed value.  The row's k-th largest value is found by bisection on an order-preserving
// 32-bit image of the floats, one bit per round: count = popcount(ballot(key >= candidate)).
// As soon as a candidate splits off exactly k entries the search is over.  Ties at the
// threshold go to the lowest columns, -0 equals +0.  Returns whether this lane's column is kept
// and the row's column bit mask.
template <int DG>
__device__ __forceinline__ bool topk_select(float x, int k, int c, int sub, typename MaskOf<DG>::type* mask_out) {
    using M = typename MaskOf<DG>::type;
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;
    const uint32_t key = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    uint32_t thr = 0u;
    bool done = (k >= DG);
    for (int bit = 31; bit >= 0; --bit) {
        if (ballot(!done) == 0ull) break;
        const uint32_t cand = thr | (1u << bit);
        const int cnt = popc<DG>(sub_bits<DG>(ballot(key >= cand), sub));
        if (cnt >= k) thr = cand;
        done = done || (cnt == k);
    }
    const M gt = sub_bits<DG>(ballot(key > thr), sub);
    const M eq = sub_bits<DG>(ballot(key == thr), sub);
    const int need = k - popc<DG>(gt);
    const M below = ((M)1 << c) - 1;
    const bool sel = (key > thr) || (key == thr && popc<DG>(eq & below) < need);
    *mask_out = sub_bits<DG>(ballot(sel), sub);
    return sel;
}

// ---- CSR views -------------------------------------------------------------------------------
struct CsrView {
    const int32_t* rp;
    const int32_t* ci;
    const float* av;
    // split plan of very long rows
    const int32_t* hub_rows;
    const int32_t* hub_cptr;
    int32_t n_hub;
    int32_t hub_threshold;
};

__device__ __forceinline__ int find_hub(const CsrView& g, int row) {
    int lo = 0, hi = g.n_hub - 1;
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (g.hub_rows[mid] < row) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// sum of the first-pass partial rows of hub row `row`, in chunk order
template <int DG>
__device__ __forceinline__ float hub_row_sum(const CsrView& g, const float* __restrict__ part, int row, int c) {
    const int h = find_hub(g, row);
    float acc = 0.f;
    for (int q = g.hub_cptr[h]; q < g.hub_cptr[h + 1]; ++q) acc += part[(size_t)q * DG + c];
    return acc;
}

// One row of  A * scatter(V, I)  (Section 4.1, eq. (10)): for every stored neighbour j of `row`
// lane c adds a_ij * V[j][slot] if j recorded column c.  The record of j is its k values in
// ascending column order plus a DG-bit column mask, so slot = popcount(mask below c).
// e0/e1: edge range to visit (the whole row, or one chunk of a hub row).
template <int DG, typename T>
__device__ __forceinline__ float gather_records(const CsrView& g, const T* __restrict__ vals,
                                                const typename MaskOf<DG>::type* __restrict__ masks, int k,
                                                int e0, int e1, int c, int stride = 1) {
    using M = typename MaskOf<DG>::type;
    const M below = ((M)1 << c) - 1;
    float acc = 0.f;
    constexpr int U = 4;
    for (int e = e0; ballot(e < e1) != 0ull; e += U * stride) {
        int j[U]; float a[U]; M m[U]; float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = e + u * stride < e1;
            j[u] = ok ? g.ci[e + u * stride] : -1;
            a[u] = ok ? g.av[e + u * stride] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) m[u] = j[u] >= 0 ? masks[j[u]] : (M)0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool hit = (m[u] >> c) & 1;
            v[u] = hit ? to_float(vals[(size_t)j[u] * k + popc<DG>(m[u] & below)]) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc += a[u] * v[u];
    }
    return acc;
}

// One row of  A * X  for a dense plane X (row stride ld): lane c adds a_ij * X[j][c].
template <int DG, typename T>
__device__ __forceinline__ float gather_dense(const CsrView& g, const T* __restrict__ x, int64_t ld,
                                              int e0, int e1, int c, int stride = 1) {
    float acc = 0.f;
    constexpr int U = 4;
    for (int e = e0; ballot(e < e1) != 0ull; e += U * stride) {
        int j[U]; float a[U]; float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = e + u * stride < e1;
            j[u] = ok ? g.ci[e + u * stride] : -1;
            a[u] = ok ? g.av[e + u * stride] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = j[u] >= 0 ? to_float(x[(size_t)j[u] * ld + c]) : 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) acc += a[u] * v[u];
    }
    return acc;
}

// ---- 16-row MFMA tiles -------------------------------------------------------------------------
// A wave multiplies its 16 x DG tile (staged in LDS, row stride DG+1) by a DG x DG matrix held
// in registers as v_mfma_f32_16x16x4_f32 B-operands:
//   A[i][kk]: lane = kk*16 + i;  B[kk][j]: lane = kk*16 + j;  D[4*(lane/16)+r][lane%16] in reg r.
using f32x4 = __attribute__((__vector_size__(4 * sizeof(float)))) float;

template <int DG>
struct WFrag {
    float b[DG / 4][DG / 16];
};

// transposed = false: B = W (tile * W);  true: B = W^T (tile * W^T)
template <int DG>
__device__ __forceinline__ void load_wfrag(const float* __restrict__ w, bool transposed, WFrag<DG>& f) {
    const int lane = lane_id();
#pragma unroll
    for (int s = 0; s < DG / 4; ++s)
#pragma unroll
        for (int cb = 0; cb < DG / 16; ++cb) {
            const int kk = 4 * s + (lane >> 4), j = 16 * cb + (lane & 15);
            f.b[s][cb] = transposed ? w[j * DG + kk] : w[kk * DG + j];
        }
}

template <int DG>
__device__ __forceinline__ void mfma_tile(const float* st, const WFrag<DG>& f, f32x4 (&acc)[DG / 16]) {
    const int lane = lane_id();
#pragma unroll
    for (int cb = 0; cb < DG / 16; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < DG / 4; ++s) {
        const float a = st[(lane & 15) * (DG + 1) + 4 * s + (lane >> 4)];
#pragma unroll
        for (int cb = 0; cb < DG / 16; ++cb)
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, f.b[s][cb], acc[cb], 0, 0, 0);
    }
}

template <int DG>
__device__ __forceinline__ void store_tile(float* st, const f32x4 (&acc)[DG / 16]) {
    const int lane = lane_id();
#pragma unroll
    for (int cb = 0; cb < DG / 16; ++cb)
#pragma unroll
        for (int r = 0; r < 4; ++r) st[(4 * (lane >> 4) + r) * (DG + 1) + 16 * cb + (lane & 15)] = acc[cb][r];
}

// dW += H^T dY over the 16 rows of the tile: D[m][o] += sum_n H[n][m] dY[n][o]
template <int DG>
__device__ __forceinline__ void mfma_outer(const float* st_h, const float* st_g, f32x4 (&acc)[DG / 16][DG / 16]) {
    const int lane = lane_id();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int nrow = 4 * ks + (lane >> 4);
        float bop[DG / 16];
#pragma unroll
        for (int ob = 0; ob < DG / 16; ++ob) bop[ob] = st_g[nrow * (DG + 1) + 16 * ob + (lane & 15)];
#pragma unroll
        for (int mb = 0; mb < DG / 16; ++mb) {
            const float a = st_h[nrow * (DG + 1) + 16 * mb + (lane & 15)];
#pragma unroll
            for (int ob = 0; ob < DG / 16; ++ob)
                acc[mb][ob] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bop[ob], acc[mb][ob], 0, 0, 0);
        }
    }
}

// ---- persistent row-tile schedule ---------------------------------------------------------------
// Workgroups are dealt to the 8 XCDs round-robin by the hardware; each XCD has its own L2.  Every
// XCD therefore sweeps one contiguous eighth of the row tiles, its resident waves working on
// adjacent tiles, so that neighbour records (circuit graphs connect nearby levels) stay in that L2.
struct TileSweep {
    int first, end, step;
};
__device__ __forceinline__ TileSweep tile_sweep(int tiles) {
    const int xcd = blockIdx.x & 7, local_wg = blockIdx.x >> 3, wg_per_xcd = gridDim.x >> 3;
    const int waves_per_wg = blockDim.x >> 6;
    const int slot = local_wg * waves_per_wg + (threadIdx.x >> 6);
    TileSweep t;
    const int t0 = (int)((int64_t)tiles * xcd / 8), t1 = (int)((int64_t)tiles * (xcd + 1) / 8);
    t.first = t0 + slot;
    t.end = t1;
    t.step = wg_per_xcd * waves_per_wg;
    return t;
}

// ---- first pass over the chunks of very long rows ------------------------------------------------
// One wave per chunk.  With DG = 32 the two half-waves take alternate neighbours of the chunk and
// their sums are added (lower half first).  part[chunk][DG] receives the un-scaled partial row.
struct HubChunks {
    const int32_t* ce0;
    const int32_t* ce1;
    int32_t n_chunks;
};

template <int DG, typename T>
__global__ __launch_bounds__(256) void k_hub_records(CsrView g, HubChunks h, const T* __restrict__ vals,
                                                     const typename MaskOf<DG>::type* __restrict__ masks, int k,
                                                     float* __restrict__ part) {
    constexpr int G = 64 / DG;
    const int lane = lane_id(), c = lane % DG, sub = lane / DG;
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int q = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; q < h.n_chunks; q += nwaves) {
        float acc = gather_records<DG, T>(g, vals, masks, k, h.ce0[q] + sub, h.ce1[q], c, G);
        if constexpr (G == 2) acc = __shfl(acc, c, 64) + __shfl(acc, c + 32, 64);
        if (sub == 0) part[(size_t)q * DG + c] = acc;
    }
}

template <int DG, typename T>
__global__ __launch_bounds__(256) void k_hub_dense(CsrView g, HubChunks h, const T* __restrict__ x, int64_t ld,
                                                   float* __restrict__ part) {
    constexpr int G = 64 / DG;
    const int lane = lane_id(), c = lane % DG, sub = lane / DG;
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int q = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; q < h.n_chunks; q += nwaves) {
        float acc = gather_dense<DG, T>(g, x, ld, h.ce0[q] + sub, h.ce1[q], c, G);
        if constexpr (G == 2) acc = __shfl(acc, c, 64) + __shfl(acc, c + 32, 64);
        if (sub == 0) part[(size_t)q * DG + c] = acc;
    }
}

// Row `row` of A * scatter(V, I): direct gather, or the sum of its first-pass partials.
template <int DG, typename T>
__device__ __forceinline__ float row_records(const CsrView& g, const T* __restrict__ vals,
                                             const typename MaskOf<DG>::type* __restrict__ masks, int k,
                                             const float* __restrict__ hub_part, int row, bool ok, int c) {
    int e0 = 0, e1 = 0;
    if (ok) { e0 = g.rp[row]; e1 = g.rp[row + 1]; }
    const bool hub = (e1 - e0) > g.hub_threshold;
    float acc = gather_records<DG, T>(g, vals, masks, k, e0, hub ? e0 : e1, c);
    if (hub) acc = hub_row_sum<DG>(g, hub_part, row, c);
    return acc;
}

template <int DG, typename T>
__device__ __forceinline__ float row_dense(const CsrView& g, const T* __restrict__ x, int64_t ld,
                                           const float* __restrict__ hub_part, int row, bool ok, int c) {
    int e0 = 0, e1 = 0;
    if (ok) { e0 = g.rp[row]; e1 = g.rp[row + 1]; }
    const bool hub = (e1 - e0) > g.hub_threshold;
    float acc = gather_dense<DG, T>(g, x, ld, e0, hub ? e0 : e1, c);
    if (hub) acc = hub_row_sum<DG>(g, hub_part, row, c);
    return acc;
}

}  // namespace gsr
