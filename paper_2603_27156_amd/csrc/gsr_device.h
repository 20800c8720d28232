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

// Orders this wave's LDS traffic for the compiler.  The hardware executes the LDS instructions of
// one wave in issue order, so a write followed by another lane's read needs no wait, only the
// guarantee that the compiler keeps the two in program order.
__device__ __forceinline__ void wave_sync() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_wave_barrier();
}

// LDS += v without a return value (ds_add_f32).  Only used where no two lanes of the same
// instruction address the same word and one wave owns the buffer: the additions then happen in
// program order and the result does not depend on timing.
__device__ __forceinline__ void lds_add(float* p, float v) {
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
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

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true);
    return v + __builtin_bit_cast(float, moved);
}

__device__ __forceinline__ float read_lane(float v, int l) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}

// Sum over the DG lanes of this lane's row, the same value (same association) in every lane:
// butterfly inside each group of 16 lanes with DPP (xor 1, xor 2, half-row mirror, row mirror),
// then the four group sums are combined as (g0 + g1) + (g2 + g3).
template <int DG>
__device__ __forceinline__ float sub_sum(float v) {
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror
    v = dpp_add<0x140>(v);   // row_mirror
    const float lo = read_lane(v, 0) + read_lane(v, 16), hi = read_lane(v, 32) + read_lane(v, 48);
    if constexpr (DG == 64) return lo + hi;
    else return (threadIdx.x & 32) ? hi : lo;
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

// The same search for R rows at once (independent bisections interleaved so that their
// dependent ballot -> popcount -> compare chains overlap).  With one row per wave (DG = 64) every
// quantity of the search is wave-uniform and lives in scalar registers.
template <int DG, int R>
__device__ __forceinline__ void topk_select_multi(const float (&x)[R], int k, int c, int sub, bool (&sel)[R],
                                                  typename MaskOf<DG>::type (&mask_out)[R]) {
    using M = typename MaskOf<DG>::type;
    uint32_t key[R], thr[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        uint32_t u = __float_as_uint(x[r]);
        if (u == 0x80000000u) u = 0u;
        key[r] = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
        thr[r] = 0u;
    }
    if constexpr (DG == 64) {
        // Interval bisection with a data-driven start.  Invariant per row: at least k keys are
        // >= lo and fewer than k are >= hi.  hi starts just above the row maximum; lo starts 4
        // binades below it (16x in value), which holds the k-th largest of almost every row, and
        // falls back to 0 when a count says it does not.  A row is closed as soon as a candidate
        // splits off exactly k keys.
        uint32_t lo[R], hi[R];
        uint32_t open = 0u;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            uint32_t m = key[r];
            m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0xB1, 0xF, 0xF, true));
            m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x4E, 0xF, 0xF, true));
            m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x141, 0xF, 0xF, true));
            m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x140, 0xF, 0xF, true));
            const uint32_t m01 = max((uint32_t)__builtin_amdgcn_readlane((int)m, 0), (uint32_t)__builtin_amdgcn_readlane((int)m, 16));
            const uint32_t m23 = max((uint32_t)__builtin_amdgcn_readlane((int)m, 32), (uint32_t)__builtin_amdgcn_readlane((int)m, 48));
            const uint32_t top = max(m01, m23);
            const uint32_t guess = top > (4u << 23) ? top - (4u << 23) : 0u;
            const int cnt = __popcll(ballot(key[r] >= guess));
            lo[r] = cnt >= k ? guess : 0u;
            hi[r] = top + 1u;
            if (cnt != k && k < DG) open |= 1u << r;
            if (k >= DG) lo[r] = 0u;
        }
        // 33 halvings bring any 32-bit interval down to one value (rows with a tie at the k-th
        // position never see an exact count and run the full course)
        for (int round = 0; round < 33 && open != 0u; ++round) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t mid = lo[r] + ((hi[r] - lo[r]) >> 1);
                const int cnt = __popcll(ballot(key[r] >= mid));
                lo[r] = cnt >= k ? mid : lo[r];
                hi[r] = cnt >= k ? hi[r] : mid;
                open = cnt == k ? open & ~(1u << r) : open;
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) thr[r] = lo[r];
    } else {
        bool done[R];
#pragma unroll
        for (int r = 0; r < R; ++r) done[r] = (k >= DG);
        for (int bit = 31; bit >= 0; --bit) {
            bool all = true;
#pragma unroll
            for (int r = 0; r < R; ++r) all = all && done[r];
            if (ballot(!all) == 0ull) break;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t cand = thr[r] | (1u << bit);
                const int cnt = popc<DG>(sub_bits<DG>(ballot(key[r] >= cand), sub));
                thr[r] = cnt >= k ? cand : thr[r];
                done[r] = done[r] || (cnt == k);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool ge = key[r] >= thr[r];
        const M ge_m = sub_bits<DG>(ballot(ge), sub);
        bool exact = popc<DG>(ge_m) == k;       // no tie at the threshold: the set is {key >= thr}
        if constexpr (DG != 64) exact = ballot(!exact) == 0ull;
        if (exact) {
            sel[r] = ge;
            mask_out[r] = ge_m;
        } else {
            const M below = ((M)1 << c) - 1;
            const M gt = sub_bits<DG>(ballot(key[r] > thr[r]), sub);
            const M eq = sub_bits<DG>(ballot(key[r] == thr[r]), sub);
            const int need = k - popc<DG>(gt);
            sel[r] = (key[r] > thr[r]) || (key[r] == thr[r] && popc<DG>(eq & below) < need);
            mask_out[r] = sub_bits<DG>(ballot(sel[r]), sub);
        }
    }
}

// number of set bits of this row's mask below this lane's column
template <int DG>
__device__ __forceinline__ int rank_in_mask(typename MaskOf<DG>::type m, uint64_t wave_mask, int sub) {
    const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(wave_mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)wave_mask, 0));
    if constexpr (DG == 64) return below;
    else return sub ? below - __popc((uint32_t)wave_mask) : below;
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
    constexpr int U = 8;
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
    constexpr int U = 8;
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

// ---- tile-staged gathers ----------------------------------------------------------------------------
// A wave owns 16 consecutive rows.  Their neighbour lists are one contiguous edge range, so the
// dependent chain row pointer -> column index -> neighbour data is walked once per tile, 64 edges
// per step, instead of once per row: lane l loads edge l of the chunk, finds the row it belongs
// to, and parks (column, value, row) in LDS.  The neighbour data of many edges is then in flight
// at once, and every contribution is added into the LDS tile H[row][col] in edge order.
struct EdgeRec {
    int j;      // neighbour (column of A)
    float a;    // a_ij
    int r;      // row of the tile, 0..15
    int pad;
};

// Row pointers of the tile's 17 row boundaries (clamped at n) into s_rp.  Returns whether one of
// the rows is a split ("hub") row.
__device__ __forceinline__ bool tile_begin(const CsrView& g, int r0, int n, int* s_rp, int lane) {
    int rpv = 0;
    if (lane < 17) {
        const int row = r0 + lane < n ? r0 + lane : n;
        rpv = g.rp[row];
        s_rp[lane] = rpv;
    }
    wave_sync();
    const bool hub = lane < 16 && (s_rp[lane + 1] - rpv) > g.hub_threshold;
    return ballot(hub) != 0ull;
}

// stage up to 64 edges [eb, min(eb+64, e_b)) into ebuf; returns how many
__device__ __forceinline__ int stage_edges(const CsrView& g, int eb, int e_b, const int* s_rp, EdgeRec* ebuf, int lane) {
    const int e = eb + lane;
    const bool ok = e < e_b;
    EdgeRec me;
    me.j = ok ? g.ci[e] : 0;
    me.a = ok ? g.av[e] : 0.f;
    int r = 0;
#pragma unroll
    for (int step = 8; step >= 1; step >>= 1)
        if (s_rp[r + step] <= e) r += step;
    me.r = r;
    me.pad = 0;
    wave_sync();          // readers of the previous chunk are done
    ebuf[lane] = me;
    wave_sync();
    return e_b - eb < 64 ? e_b - eb : 64;
}

// One staged edge of a record gather: where neighbour j's k values start, a_ij, and j's column mask.
struct RecEdge {
    uint32_t off0;   // j * k
    float a;
    uint32_t mlo, mhi;
};

// H[r][c] += a_ij * V[j][slot of c] for every edge in [e_a, e_b): lane c of a (sub-)wave owns
// column c.  The record of j is its k kept values in ascending column order plus a DG-bit column
// mask, so lane c finds its value at popcount(mask below c) if bit c is set.  All 64 lanes load
// from inside the 4k-byte record (lanes whose column is absent read a neighbouring slot and
// contribute 0), so the loads of a batch of edges are unconditional and in flight together.  The
// edges of one row are summed in a register; the sum goes to the LDS tile when the row changes.
// With two rows per wave (DG = 32) the half-waves take alternate edges and flush one after the
// other.  n * k must stay below 2^32.
template <int DG, typename T>
__device__ __forceinline__ void range_gather_records(const CsrView& g, const T* __restrict__ vals,
                                                     const typename MaskOf<DG>::type* __restrict__ masks, int k, int e_a,
                                                     int e_b, const int* s_rp, RecEdge* ebuf, uint8_t* rbuf, float* st_h,
                                                     int lane) {
    using M = typename MaskOf<DG>::type;
    constexpr int LR = DG + 1, G = 64 / DG, GB = 16;
    const int c = lane % DG, sub = lane / DG;
    const uint32_t bit_lo = c < 32 ? 1u << c : 0u, bit_hi = c >= 32 ? 1u << (c - 32) : 0u;
    const uint32_t below_lo = c < 32 ? bit_lo - 1u : 0xFFFFFFFFu, below_hi = c >= 32 ? bit_hi - 1u : 0u;
    float acc = 0.f;
    int cur = 16;                      // row being summed; 16 = the dump row
    auto flush = [&](int next) {
#pragma unroll
        for (int s2 = 0; s2 < G; ++s2)
            if (s2 == sub && next != cur) st_h[cur * LR + c] += acc;
        if (next != cur) { acc = 0.f; cur = next; }
    };
    for (int eb = e_a; eb < e_b; eb += 64) {
        // stage up to 64 edges: lane l takes edge eb + l
        const int e = eb + lane;
        const bool eok = e < e_b;
        const int j = eok ? g.ci[e] : 0;
        RecEdge me;
        me.a = eok ? g.av[e] : 0.f;
        me.off0 = (uint32_t)j * (uint32_t)k;
        const M m = masks[j];
        me.mlo = (uint32_t)m;
        if constexpr (DG == 64) me.mhi = (uint32_t)(m >> 32);
        else me.mhi = 0u;
        int r = 0;
#pragma unroll
        for (int step = 8; step >= 1; step >>= 1)
            if (s_rp[r + step] <= e) r += step;
        wave_sync();          // readers of the previous chunk are done
        ebuf[lane] = me;
        rbuf[lane] = (uint8_t)r;
        wave_sync();
        const int cnt = e_b - eb < 64 ? e_b - eb : 64;
        const int nit = (cnt + G - 1) / G;
        for (int i0 = 0; i0 < nit; i0 += GB) {
            float v[GB];
            int rr[GB];
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                const int ei = (i0 + u) * G + sub;
                const bool ok = ei < cnt;
                const int eu = ok ? ei : cnt - 1;
                const RecEdge er = ebuf[eu];
                const bool hit = ((er.mlo & bit_lo) | (er.mhi & bit_hi)) != 0u;
                int pos = __popc(er.mlo & below_lo) + __popc(er.mhi & below_hi);
                pos = pos < k ? pos : k - 1;
                const float val = to_float(vals[er.off0 + (uint32_t)pos]);
                v[u] = (ok && hit) ? er.a * val : 0.f;
                const int rrow = (int)rbuf[eu];
                rr[u] = ok ? rrow : -1;
            }
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                flush(rr[u] >= 0 ? rr[u] : cur);
                acc += v[u];
            }
        }
    }
    flush(16);
}

// Q[r][c] += a_ij * X[j][c] for every edge in [e_a, e_b): lane c of a (sub-)wave owns column c and
// sums the edges of one row in a register; the sum goes to the LDS tile when the row changes.
// With two rows per wave (DG = 32) the half-waves take alternate edges and flush one after the
// other, so two partial sums of the same row never meet in one instruction.
template <int DG, typename T>
__device__ __forceinline__ void range_gather_dense(const CsrView& g, const T* __restrict__ x, int64_t ld, int e_a, int e_b,
                                                   const int* s_rp, EdgeRec* ebuf, float* st, int lane) {
    constexpr int LR = DG + 1, G = 64 / DG, GB = 16;
    const int c = lane % DG, sub = lane / DG;
    float acc = 0.f;
    int cur = 16;                      // row being summed; 16 = the dump row
    auto flush = [&](int next) {
#pragma unroll
        for (int s2 = 0; s2 < G; ++s2)
            if (s2 == sub && next != cur) st[cur * LR + c] += acc;
        if (next != cur) { acc = 0.f; cur = next; }
    };
    for (int eb = e_a; eb < e_b; eb += 64) {
        const int cnt = stage_edges(g, eb, e_b, s_rp, ebuf, lane);
        const int nit = (cnt + G - 1) / G;
        for (int i0 = 0; i0 < nit; i0 += GB) {
            float v[GB];
            int rr[GB];
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                const int ei = (i0 + u) * G + sub;
                const bool ok = ei < cnt;
                const EdgeRec er = ebuf[ok ? ei : cnt - 1];
                const float val = to_float(x[(size_t)er.j * ld + c]);
                v[u] = ok ? er.a * val : 0.f;
                rr[u] = ok ? er.r : -1;
            }
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                flush(rr[u] >= 0 ? rr[u] : cur);
                acc += v[u];
            }
        }
    }
    flush(16);
}

// Walks the tile's rows: maximal runs of ordinary rows go through `range(e_a, e_b)`, split rows
// receive the sum of their first-pass partial rows.  st must be zero on entry; it is 16 rows of
// DG+1 floats followed by 64 dump words.
template <int DG, typename Range>
__device__ __forceinline__ void tile_gather(const CsrView& g, const float* __restrict__ hub_part, bool has_hub, int r0,
                                            const int* s_rp, float* st, int lane, Range range) {
    constexpr int LR = DG + 1;
    if (!has_hub) {
        range(s_rp[0], s_rp[16]);
        return;
    }
    int run = 0;
    for (int r = 0; r <= 16; ++r) {
        const bool hub = r < 16 && (s_rp[r + 1] - s_rp[r]) > g.hub_threshold;
        if (r == 16 || hub) {
            if (s_rp[r] > s_rp[run]) range(s_rp[run], s_rp[r]);
            run = r + 1;
        }
        if (hub && lane < DG) st[r * LR + lane] = hub_row_sum<DG>(g, hub_part, r0 + r, lane);
    }
}

template <int DG>
__device__ __forceinline__ void zero_tile(float* st, int lane) {
#pragma unroll
    for (int i = lane; i < 16 * (DG + 1); i += 64) st[i] = 0.f;
}

// ---- 16-row MFMA tiles -------------------------------------------------------------------------
// A wave multiplies its 16 x DG tile (staged in LDS, row stride DG+1) by a DG x DG matrix with
// v_mfma_f32_16x16x4_f32:
//   A[i][kk]: lane = kk*16 + i;  B[kk][j]: lane = kk*16 + j;  D[4*(lane/16)+r][lane%16] in reg r.
using f32x4 = __attribute__((__vector_size__(4 * sizeof(float)))) float;

// The DG x DG weight matrix sits in LDS (row stride DG + 8, which spreads the four k-rows of a
// B operand over different banks), loaded once per workgroup; transposed = true stores W^T.
template <int DG>
struct WLds {
    static constexpr int WP = DG + 8;
    float w[DG * WP];
};

template <int DG>
__device__ __forceinline__ void load_w_lds(const float* __restrict__ w, bool transposed, WLds<DG>& l) {
    for (int i = threadIdx.x; i < DG * DG; i += blockDim.x) {
        const int r = i / DG, cc = i % DG;
        l.w[r * WLds<DG>::WP + cc] = transposed ? w[cc * DG + r] : w[i];
    }
    __syncthreads();
}

// acc = tile (16 x DG, LDS, row stride DG+1) * B (DG x DG, LDS)
template <int DG>
__device__ __forceinline__ void mfma_tile(const float* st, const WLds<DG>& wl, f32x4 (&acc)[DG / 16]) {
    const int lane = lane_id();
#pragma unroll
    for (int cb = 0; cb < DG / 16; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < DG / 4; ++s) {
        const float a = st[(lane & 15) * (DG + 1) + 4 * s + (lane >> 4)];
#pragma unroll
        for (int cb = 0; cb < DG / 16; ++cb) {
            const float b = wl.w[(4 * s + (lane >> 4)) * WLds<DG>::WP + 16 * cb + (lane & 15)];
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[cb], 0, 0, 0);
        }
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
