// Device-side building blocks for gfx950 (wave64): storage conversion, sub-wave reductions,
// the exact top-k select of the GS operator, neighbour gathers and 16x16x4 float32 MFMA tiles.
//
// Three thread layouts appear.  "Row layout" (operators exposed on their own, first pass over split
// rows, head): a row of a group has DG = 32 or 64 columns and lane c of a (sub-)wave owns column
// c; with DG = 64 a wave holds one row, with DG = 32 two (lanes 0..31 and 32..63, `sub` = lane /
// DG).  "Tile register layout" (layer kernels: what the MFMA leaves in the accumulators for a
// 16-row tile; four rows per memory instruction) and "quarter layout" (GS of a 16-row tile: lane
// = (row, quarter of its columns)) are described where they are introduced below.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

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

// (a & m) | (b & ~m)
__device__ __forceinline__ uint32_t bit_select(uint32_t m, uint32_t a, uint32_t b) { return (a & m) | (b & ~m); }

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

// ---- "quarter layout": lane = (row r = lane % 16, quarter q = lane / 16) ------------------------
// The four lanes r, r+16, r+32, r+48 share a row of a 16-row tile, each holding a quarter of its
// columns.  v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the even
// rows of its second, v_permlane32_swap the upper half of the first with the lower half of the
// second; fed the same register twice they hand every lane its partner quarters.

// q[i] = v of the lane of quarter i in this lane's row
__device__ __forceinline__ void quarter_all(uint32_t v, uint32_t (&q)[4]) {
    const auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);        // quarters {0|2}, {1|3} of my half
    const auto b = __builtin_amdgcn_permlane32_swap(a[0], a[0], false, false);  // quarter 0, quarter 2
    const auto d = __builtin_amdgcn_permlane32_swap(a[1], a[1], false, false);  // quarter 1, quarter 3
    q[0] = b[0]; q[1] = d[0]; q[2] = b[1]; q[3] = d[1];
}
__device__ __forceinline__ uint32_t quarter_sum(uint32_t v) {
    const auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    const uint32_t s = a[0] + a[1];
    const auto b = __builtin_amdgcn_permlane32_swap(s, s, false, false);
    return b[0] + b[1];
}
__device__ __forceinline__ uint32_t quarter_max(uint32_t v) {
    const auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    const uint32_t s = max(a[0], a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(s, s, false, false);
    return max(b[0], b[1]);
}
// (q0 + q1) + (q2 + q3), the same value in the four lanes
__device__ __forceinline__ float quarter_sum(float v) {
    const uint32_t u = __float_as_uint(v);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const float s = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const uint32_t su = __float_as_uint(s);
    const auto b = __builtin_amdgcn_permlane32_swap(su, su, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

__device__ __forceinline__ float quarter_fmax(float v) {
    const uint32_t u = __float_as_uint(v);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const float s = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const uint32_t su = __float_as_uint(s);
    const auto b = __builtin_amdgcn_permlane32_swap(su, su, false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quarter_fmin(float v) { return -quarter_fmax(-v); }

// ---- GS: exact top-k of a row ----------------------------------------------------------------
// The Group-Sparse operator of Section 4.1 of the paper keeps, per row, the k largest entries by
// signed value.  The row's k-th largest value is found by bisection on an order-preserving
// 32-bit image of the floats, one bit per round: count = popcount(ballot(key >= candidate)).
// As soon as a candidate splits off exactly k entries the search is over.  Ties at the
// threshold go to the lowest columns, -0 equals +0.  Row layout (lane c of a (sub-)wave owns
// column c), R rows at once: the independent bisections are interleaved so that their dependent
// ballot -> popcount -> compare chains overlap.  sel[r]: this lane's column of row r is kept;
// mask_out[r]: the row's column bit mask.  With one row per wave (DG = 64) every quantity of the
// search is wave-uniform and lives in scalar registers.  (The layer kernels select in the
// quarter layout instead, 16 rows at once in vector registers.)
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

// ---- CSR views -------------------------------------------------------------------------------
struct CsrView {
    const int32_t* rp;
    const int32_t* ci;
    const float* av;
    // split plan of very long rows
    const int32_t* hub_rows;
    const int32_t* hub_cptr;
    const int32_t* hub_tile0;     // [tiles + 1]: split rows before row 16 t
    int32_t n_hub;
    int32_t hub_threshold;
    // tiles with more than heavy_edges stored entries, ascending (see TileDeal)
    const int32_t* heavy;
    int32_t n_heavy;
    int32_t heavy_edges;
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
    // sixteen partial rows in flight at a time; added in chunk order, so the sum does not depend
    // on the unrolling
    const int q1 = g.hub_cptr[h + 1];
    int q = g.hub_cptr[h];
    float acc = 0.f;
    for (; q + 16 <= q1; q += 16) {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = part[(size_t)(q + u) * DG + c];
#pragma unroll
        for (int u = 0; u < 16; ++u) acc += v[u];
    }
    for (; q < q1; ++q) acc += part[(size_t)q * DG + c];
    return acc;
}

// ---- tile gathers on the matrix cores ------------------------------------------------------------------
// A wave owns 16 consecutive rows.  Their neighbour lists are one contiguous edge range, so the
// dependent chain row pointer -> column index -> neighbour data is walked once per tile, 64 edges
// per step: lane l loads edge l, finds the tile row it belongs to, and parks (neighbour, a_ij, row)
// in LDS.  The aggregation itself is the product  H = P * X  of the tile's 16 x E selection
// matrix (P[r][e] = a_e if edge e belongs to row r, else 0) with the E x DG matrix of neighbour
// rows, taken four edges at a time by v_mfma_f32_16x16x4_f32:
//   A operand  lane (i = lane % 16, kk = lane / 16):  P[i][edge kk of the four]
//   B operand  lane (j = lane % 16, kk = lane / 16):  X[neighbour of edge kk][column of (j, cb)]
// One MFMA covers 16 columns; the DG / 16 column blocks cb are interleaved, column = CPL * j + cb
// with CPL = DG / 16, so that a lane's CPL columns are adjacent in memory and arrive in one load
// of CPL values.  One load instruction thus fetches the rows of four edges, nothing is predicated
// (edges past the end are staged with a_ij = 0 and neighbour 0) and the sum over a row's edges is
// taken in edge order inside the accumulators, which hold H as D[4 * (lane / 16) + reg][j].
using f32x4 = __attribute__((__vector_size__(4 * sizeof(float)))) float;
typedef uint32_t u32x2a __attribute__((ext_vector_type(2), aligned(4)));
typedef uint32_t u32x3a __attribute__((ext_vector_type(3), aligned(4)));
typedef uint32_t u32x4a __attribute__((ext_vector_type(4), aligned(4)));

template <int NW>
__device__ __forceinline__ void load_words(const void* p, uint32_t (&w)[NW]) {
    if constexpr (NW == 1) {
        w[0] = *reinterpret_cast<const uint32_t*>(p);
    } else if constexpr (NW == 2) {
        const u32x2a v = *reinterpret_cast<const u32x2a*>(p);
        w[0] = v[0]; w[1] = v[1];
    } else if constexpr (NW == 3) {
        const u32x3a v = *reinterpret_cast<const u32x3a*>(p);
        w[0] = v[0]; w[1] = v[1]; w[2] = v[2];
    } else {
        static_assert(NW == 4, "1 to 4 words");
        const u32x4a v = *reinterpret_cast<const u32x4a*>(p);
        w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
    }
}

// ---- tile register layout ---------------------------------------------------------------------------
// What the MFMA leaves in a wave's accumulators for a 16 x DG tile when the A operand takes tile
// row 4 (i % 4) + i / 4 as its row i and the B operand takes column CPL j + cb as column j of
// block cb (CPL = DG / 16): lane (g = lane / 16, j = lane % 16) holds, in acc[cb][reg],
//     tile row 4 reg + g,  column CPL j + cb.
// For a fixed reg the 16 lanes of a group cover one whole row with CPL adjacent elements each, so
// a row moves between registers and memory with one fully coalesced access of CPL elements per
// lane, four rows per instruction.  Sums over a row are sums over the 16 lanes of a group.
template <int CPL, typename T>
__device__ __forceinline__ void load_cols(const T* p, float (&v)[CPL]) {       // non-temporal
    constexpr int NW = CPL * (int)sizeof(T) / 4;
    uint32_t w[NW];
    if constexpr (NW == 1) {
        w[0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
    } else if constexpr (NW == 2) {
        const u32x2a t = __builtin_nontemporal_load(reinterpret_cast<const u32x2a*>(p));
        w[0] = t[0]; w[1] = t[1];
    } else {
        const u32x4a t = __builtin_nontemporal_load(reinterpret_cast<const u32x4a*>(p));
        w[0] = t[0]; w[1] = t[1]; w[2] = t[2]; w[3] = t[3];
    }
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        if constexpr (sizeof(T) == 4) v[c] = __uint_as_float(w[c]);
        else v[c] = __uint_as_float((c & 1) ? (w[c >> 1] & 0xFFFF0000u) : (w[c >> 1] << 16));
    }
}
// v must hold values representable in T (as stored<T>() returns them)
template <int CPL, typename T>
__device__ __forceinline__ void store_cols(T* p, const float (&v)[CPL]) {      // non-temporal
    constexpr int NW = CPL * (int)sizeof(T) / 4;
    uint32_t w[NW];
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        if constexpr (sizeof(T) == 4) w[i] = __float_as_uint(v[i]);
        else w[i] = (__float_as_uint(v[2 * i]) >> 16) | (__float_as_uint(v[2 * i + 1]) & 0xFFFF0000u);
    }
    if constexpr (NW == 1) {
        __builtin_nontemporal_store(w[0], reinterpret_cast<uint32_t*>(p));
    } else if constexpr (NW == 2) {
        u32x2a t; t[0] = w[0]; t[1] = w[1];
        __builtin_nontemporal_store(t, reinterpret_cast<u32x2a*>(p));
    } else {
        u32x4a t; t[0] = w[0]; t[1] = w[1]; t[2] = w[2]; t[3] = w[3];
        __builtin_nontemporal_store(t, reinterpret_cast<u32x4a*>(p));
    }
}
// sum over the 16 lanes of this lane's group, the same value in all of them
__device__ __forceinline__ float group16_sum(float v) {
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror
    v = dpp_add<0x140>(v);   // row_mirror
    return v;
}

// ---- bf16 operands for the gathers of the bf16-storage variant --------------------------------------
// With 16-bit stored values the product P * X runs on v_mfma_f32_16x16x16_bf16: sixteen edges per
// instruction instead of four.  The K index is permuted so that nothing has to move between
// lanes: K slot 4 kk + u of lane group kk is edge kk of staged group u (u = 0..3), which is what
// the lane already holds after four loads.  X is exact in bf16; a_ij is split into two bf16 terms
// (a = hi + lo + O(2^-17 a)), one MFMA each, float32 accumulation.
typedef short bf16x4 __attribute__((ext_vector_type(4)));

// upper halves of four float32 words as four bf16
__device__ __forceinline__ bf16x4 pack_upper4(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3) {
    const uint32_t lo = __builtin_amdgcn_perm(w1, w0, 0x07060302u), hi = __builtin_amdgcn_perm(w3, w2, 0x07060302u);
    return __builtin_bit_cast(bf16x4, (uint64_t)lo | ((uint64_t)hi << 32));
}
// lower halves of four words as four bf16
__device__ __forceinline__ bf16x4 pack_lower4(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3) {
    const uint32_t lo = __builtin_amdgcn_perm(w1, w0, 0x05040100u), hi = __builtin_amdgcn_perm(w3, w2, 0x05040100u);
    return __builtin_bit_cast(bf16x4, (uint64_t)lo | ((uint64_t)hi << 32));
}
// the selection operand of four groups as three bf16 terms: p = hi + mid + lo exactly
__device__ __forceinline__ void split_p4(const float* p, bf16x4& hi, bf16x4& mid, bf16x4& lo) {
    uint32_t h[4], m[4], l[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        h[u] = __float_as_uint(p[u]) & 0xFFFF0000u;
        const float r1 = p[u] - __uint_as_float(h[u]);
        m[u] = __float_as_uint(r1) & 0xFFFF0000u;
        l[u] = __float_as_uint(r1 - __uint_as_float(m[u]));
    }
    hi = pack_upper4(h[0], h[1], h[2], h[3]);
    mid = pack_upper4(m[0], m[1], m[2], m[3]);
    lo = pack_upper4(l[0], l[1], l[2], l[3]);
}

struct EdgeRec {
    int j;      // neighbour (column of A)
    float a;    // a_ij
    int r;      // row of the tile, 0..15
    int pad;
};

// Row pointer of row r0 + lane (clamped at n) for the 17 row boundaries of a tile, in lanes 0..16.
// Split from tile_begin so that a kernel can request its other per-tile data before it waits.
__device__ __forceinline__ int tile_rp_load(const CsrView& g, int r0, int n, int lane) {
    int rpv = 0;
    if (lane < 17) rpv = g.rp[r0 + lane < n ? r0 + lane : n];
    return rpv;
}

// Publishes the tile's row pointers (rpv as tile_rp_load returned it) in s_rp.  Returns whether
// one of the rows is a split ("hub") row.
__device__ __forceinline__ bool tile_begin(const CsrView& g, int rpv, int* s_rp, int lane) {
    if (lane < 17) s_rp[lane] = rpv;
    wave_sync();
    const bool hub = lane < 16 && (s_rp[lane + 1] - rpv) > g.hub_threshold;
    return ballot(hub) != 0ull;
}
__device__ __forceinline__ bool tile_begin(const CsrView& g, int r0, int n, int* s_rp, int lane) {
    return tile_begin(g, tile_rp_load(g, r0, n, lane), s_rp, lane);
}

// tile row of edge e: the last row boundary at or below e
__device__ __forceinline__ int tile_row_of(const int* s_rp, int e) {
    int r = 0;
#pragma unroll
    for (int step = 8; step >= 1; step >>= 1)
        if (s_rp[r + step] <= e) r += step;
    return r;
}

// Runs `batch(GB, i0)` over the nit <= 16 groups of four staged edges in as few batches as
// possible: all sixteen at once if MAXB allows, else eight, then the rest as one batch of eight
// or four (a batch may overrun nit by up to three groups, which stay inside the 64 staged edges
// and contribute zero).
template <int MAXB, typename Batch>
__device__ __forceinline__ void edge_batches(int nit, Batch batch) {
    int i0 = 0;
    if constexpr (MAXB >= 16) {
        if (nit > 12) {
            batch(std::integral_constant<int, 16>{}, 0);
            return;
        }
    }
    if (nit > 8) {
        batch(std::integral_constant<int, 8>{}, 0);
        i0 = 8;
    }
    if (nit - i0 > 4) batch(std::integral_constant<int, 8>{}, i0);
    else if (nit - i0 > 0) batch(std::integral_constant<int, 4>{}, i0);
}

// acc += P * X over the edges [e_a, e_b) of ordinary rows; X is a dense plane, row stride ld.
// ONE_ROW: every edge belongs to tile row 0 (a chunk of a split row).  The matrix product would then spend
// fifteen of its sixteen rows on zeros; instead lane (kk, j) adds a_e * X[e][its columns] for the edges kk,
// kk + 4, .. in ordinary arithmetic into acc[cb][0], and the caller adds the four lane groups up.
template <int DG, typename T, int MAXB, bool ONE_ROW = false>
__device__ __forceinline__ void gather_dense_mfma(const CsrView& g, const T* __restrict__ x, int64_t ld, int e_a, int e_b,
                                                  const int* s_rp, EdgeRec* ebuf, int lane, f32x4 (&acc)[DG / 16]) {
    constexpr int CPL = DG / 16, NW = CPL * (int)sizeof(T) / 4;
    const int i16 = lane & 15, kk = lane >> 4;
    const T* xl = x + CPL * i16;
    const uint32_t ldu = (uint32_t)ld;
    for (int eb = e_a; eb < e_b; eb += 64) {
        const int e = eb + lane;
        const bool ok = e < e_b;
        EdgeRec me;
        me.j = ok ? __builtin_nontemporal_load(g.ci + e) : 0;
        me.a = ok ? __builtin_nontemporal_load(g.av + e) : 0.f;
        me.r = tile_row_of(s_rp, e);
        me.pad = 0;
        wave_sync();          // readers of the previous chunk are done
        ebuf[lane] = me;
        wave_sync();
        const int cnt = e_b - eb < 64 ? e_b - eb : 64;
        edge_batches<MAXB>((cnt + 3) >> 2, [&](auto gbc, int i0) {
            constexpr int GB = decltype(gbc)::value;
            uint32_t w[GB][NW];
            float p[GB];
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                const EdgeRec er = ebuf[4 * (i0 + u) + kk];
                load_words<NW>(xl + (size_t)(uint32_t)er.j * ldu, w[u]);
                p[u] = (ONE_ROW || er.r == i16) ? er.a : 0.f;
            }
            if constexpr (ONE_ROW) {
#pragma unroll
                for (int u = 0; u < GB; ++u)
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) {
                        uint32_t bits;
                        if constexpr (sizeof(T) == 4) bits = w[u][cb];
                        else bits = (cb & 1) ? (w[u][cb >> 1] & 0xFFFF0000u) : (w[u][cb >> 1] << 16);
                        acc[cb][0] = __builtin_fmaf(p[u], __uint_as_float(bits), acc[cb][0]);
                    }
            } else if constexpr (sizeof(T) == 4) {
#pragma unroll
                for (int u = 0; u < GB; ++u)
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb)
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(p[u], __uint_as_float(w[u][cb]), acc[cb], 0, 0, 0);
            } else {
#pragma unroll
                for (int u = 0; u < GB; u += 4) {
                    bf16x4 ph, pm, pl;
                    split_p4(p + u, ph, pm, pl);
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) {
                        const int d = cb >> 1;
                        const bf16x4 b = (cb & 1) ? pack_upper4(w[u][d], w[u + 1][d], w[u + 2][d], w[u + 3][d])
                                                  : pack_lower4(w[u][d], w[u + 1][d], w[u + 2][d], w[u + 3][d]);
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ph, b, acc[cb], 0, 0, 0);
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pm, b, acc[cb], 0, 0, 0);
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pl, b, acc[cb], 0, 0, 0);
                    }
                }
            }
        });
    }
}

// One staged edge of a record gather: where neighbour j's k values start, a_ij, and j's column mask.
struct RecEdge {
    uint32_t off0;   // j * k
    float a;
    uint32_t mlo, mhi;
};

// Dealing 16-bit record values to a lane's four columns with two byte permutes.  The window of four slots is two
// words (slot t in bytes 2t, 2t+1); column c takes slot popcount(mask bits below c) if its bit is set, else zero.
// For each of the 16 values of the lane's four mask bits a table holds the two v_perm_b32 selectors that build
// (column 0 | column 1 << 16) and (column 2 | column 3 << 16) from the window (selector byte 0x0c yields zero).
// The table sits in LDS (16 entries of 8 bytes, one ds_read_b64 per staged edge and lane).
struct DealLut {
    uint2 sel[16];
};
__device__ __forceinline__ void deal_lut_fill(DealLut& l) {
    if (threadIdx.x < 16) {
        const uint32_t nib = threadIdx.x;
        uint32_t s[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t t = (uint32_t)__popc(nib & ((1u << c) - 1u));
            s[c] = ((nib >> c) & 1u) ? ((2u * t + 1u) << 8 | (2u * t)) : 0x0c0cu;
        }
        l.sel[nib] = make_uint2(s[0] | s[1] << 16, s[2] | s[3] << 16);
    }
    __syncthreads();
}

// The same for float32 records and four columns per lane: the window is four words, column c takes word
// popcount(mask bits below c) if its bit is set.  A word moves whole, so a v_perm_b32 over two words of the window
// with a selector that copies the lower word, the upper word or zeros does it: column 0 from word 0, column 1 from
// words (0, 1), columns 2 and 3 from words (0, 1) or-ed with (2, -) and (2, 3).  Six selectors per value of the four
// mask bits, eight instructions per staged edge and lane instead of a chain of some twenty-five bitwise selects.
struct alignas(32) DealLutF {
    uint32_t sel[16][8];      // s0, s1, s2 over (0,1), s2 over (2,-), s3 over (0,1), s3 over (2,3), unused
};
__device__ __forceinline__ void deal_lutf_fill(DealLutF& l) {
    if (threadIdx.x < 16) {
        constexpr uint32_t LOW = 0x03020100u, HIGH = 0x07060504u, ZERO = 0x0c0c0c0cu;
        const uint32_t nib = threadIdx.x;
        const uint32_t p1 = nib & 1u, p2 = (uint32_t)__popc(nib & 3u), p3 = (uint32_t)__popc(nib & 7u);
        const bool b0 = nib & 1u, b1 = nib & 2u, b2 = nib & 4u, b3 = nib & 8u;
        uint32_t* e = l.sel[nib];
        e[0] = b0 ? LOW : ZERO;
        e[1] = b1 ? (p1 ? HIGH : LOW) : ZERO;
        e[2] = (b2 && p2 < 2u) ? (p2 ? HIGH : LOW) : ZERO;
        e[3] = (b2 && p2 == 2u) ? LOW : ZERO;
        e[4] = (b3 && p3 < 2u) ? (p3 ? HIGH : LOW) : ZERO;
        e[5] = (b3 && p3 >= 2u) ? (p3 == 3u ? HIGH : LOW) : ZERO;
        e[6] = ZERO; e[7] = ZERO;
    }
    __syncthreads();
}

// acc += P * scatter(V, I) over the edges [e_a, e_b) of ordinary rows (Section 4.1, eq. (10)).
// The record of neighbour j is its k kept values in ascending column order plus a DG-bit column
// mask.  A lane's CPL adjacent columns occupy adjacent slots of the record, starting at
// popcount(mask below its first column): the lane loads CPL values from there (the tail of the
// window may belong to the next record, or to the padding that follows the last one) and deals
// them out to the columns whose mask bit is set.  16-bit values are loaded from the even slot at
// or below the start.  n * k must stay below 2^32.
template <int DG, typename T, int MAXB, bool ONE_ROW = false>
__device__ __forceinline__ void gather_records_mfma(const CsrView& g, const T* __restrict__ vals,
                                                    const typename MaskOf<DG>::type* __restrict__ masks, int k, int e_a,
                                                    int e_b, const int* s_rp, RecEdge* ebuf, uint8_t* rbuf, int lane,
                                                    f32x4 (&acc)[DG / 16], const DealLut* lut = nullptr,
                                                    const DealLutF* lutf = nullptr) {
    constexpr bool PERM = sizeof(T) == 2 && !ONE_ROW;     // (callers of that case pass the table)
    constexpr bool PERMF = sizeof(T) == 4 && ONE_ROW && DG == 64;   // float32 chunk sums: the table of DealLutF (passed too)
    using M = typename MaskOf<DG>::type;
    constexpr int CPL = DG / 16, NW = sizeof(T) == 4 ? CPL : CPL / 2 + 1;
    const int i16 = lane & 15, kk = lane >> 4, bp = CPL * i16;
    const uint32_t sh = bp & 31;
    const bool upper = bp >= 32;
    const uint32_t below_lo = upper ? 0xFFFFFFFFu : (1u << sh) - 1u, below_hi = upper ? (1u << sh) - 1u : 0u;
    for (int eb = e_a; eb < e_b; eb += 64) {
        const int e = eb + lane;
        const bool ok = e < e_b;
        const int j = ok ? __builtin_nontemporal_load(g.ci + e) : 0;
        RecEdge me;
        me.a = ok ? __builtin_nontemporal_load(g.av + e) : 0.f;
        me.off0 = (uint32_t)j * (uint32_t)k;
        const M m = masks[j];
        me.mlo = (uint32_t)m;
        if constexpr (DG == 64) me.mhi = (uint32_t)(m >> 32);
        else me.mhi = 0u;
        const int r = tile_row_of(s_rp, e);
        wave_sync();          // readers of the previous chunk are done
        ebuf[lane] = me;
        rbuf[lane] = (uint8_t)r;
        wave_sync();
        const int cnt = e_b - eb < 64 ? e_b - eb : 64;
        edge_batches<MAXB>((cnt + 3) >> 2, [&](auto gbc, int i0) {
            constexpr int GB = decltype(gbc)::value;
            uint32_t w[GB][NW];
            uint32_t nib[GB];     // mask bits of this lane's CPL columns (bit 31: odd 16-bit start)
            float p[GB];
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                const int ei = 4 * (i0 + u) + kk;
                const RecEdge er = ebuf[ei];
                const uint32_t word = upper ? er.mhi : er.mlo;
                const uint32_t at = er.off0 + (uint32_t)__popc(er.mlo & below_lo) + (uint32_t)__popc(er.mhi & below_hi);
                nib[u] = (word >> sh) & ((1u << CPL) - 1u);
                if constexpr (sizeof(T) == 4) {
                    load_words<NW>(vals + (size_t)at, w[u]);
                } else {
                    load_words<NW>(vals + (size_t)(at & ~1u), w[u]);
                    nib[u] |= at << 31;
                }
                p[u] = (ONE_ROW || (int)rbuf[ei] == i16) ? er.a : 0.f;
            }
            if constexpr (PERM) {
                // columns (0 | 1 << 16) and, with four columns per lane, (2 | 3 << 16) of every staged edge, as bf16
                uint32_t o01[GB], o23[CPL == 4 ? GB : 1];
#pragma unroll
                for (int u = 0; u < GB; ++u) {
                    const uint32_t shift = (nib[u] >> 31) * 16u;
                    const uint32_t lo = __builtin_amdgcn_alignbit(w[u][1], w[u][0], shift);
                    const uint2 sel = lut->sel[nib[u] & 15u];
                    if constexpr (CPL == 4) {
                        const uint32_t hi = __builtin_amdgcn_alignbit(w[u][2], w[u][1], shift);
                        o01[u] = __builtin_amdgcn_perm(hi, lo, sel.x);
                        o23[u] = __builtin_amdgcn_perm(hi, lo, sel.y);
                    } else {
                        o01[u] = __builtin_amdgcn_perm(0u, lo, sel.x);      // (two mask bits: the window is one word)
                    }
                }
#pragma unroll
                for (int u = 0; u < GB; u += 4) {
                    bf16x4 ph, pm, pl;
                    split_p4(p + u, ph, pm, pl);
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) {
                        const uint32_t* o = cb < 2 ? o01 : o23;
                        const bf16x4 b = (cb & 1) ? pack_upper4(o[u], o[u + 1], o[u + 2], o[u + 3])
                                                  : pack_lower4(o[u], o[u + 1], o[u + 2], o[u + 3]);
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ph, b, acc[cb], 0, 0, 0);
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pm, b, acc[cb], 0, 0, 0);
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pl, b, acc[cb], 0, 0, 0);
                    }
                }
                return;
            }
            if constexpr (PERMF) {
#pragma unroll
                for (int u = 0; u < GB; ++u) {
                    const uint4 sa = *reinterpret_cast<const uint4*>(lutf->sel[nib[u]]);
                    const uint2 sb = *reinterpret_cast<const uint2*>(lutf->sel[nib[u]] + 4);
                    const uint32_t b0 = __builtin_amdgcn_perm(0u, w[u][0], sa.x);
                    const uint32_t b1 = __builtin_amdgcn_perm(w[u][1], w[u][0], sa.y);
                    const uint32_t b2 = __builtin_amdgcn_perm(w[u][1], w[u][0], sa.z) | __builtin_amdgcn_perm(0u, w[u][2], sa.w);
                    const uint32_t b3 = __builtin_amdgcn_perm(w[u][1], w[u][0], sb.x) | __builtin_amdgcn_perm(w[u][3], w[u][2], sb.y);
                    acc[0][0] = __builtin_fmaf(p[u], __uint_as_float(b0), acc[0][0]);
                    acc[1][0] = __builtin_fmaf(p[u], __uint_as_float(b1), acc[1][0]);
                    acc[2][0] = __builtin_fmaf(p[u], __uint_as_float(b2), acc[2][0]);
                    acc[3][0] = __builtin_fmaf(p[u], __uint_as_float(b3), acc[3][0]);
                }
                return;
            }
            uint32_t bq[sizeof(T) == 4 ? 1 : GB][CPL];   // dealt-out values (float bits) of the 16-bit variant
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                uint32_t q[CPL];  // the window (float bits): slot start + t
                if constexpr (sizeof(T) == 4) {
#pragma unroll
                    for (int t = 0; t < CPL; ++t) q[t] = w[u][t];
                } else {
                    const uint32_t shift = (nib[u] >> 31) * 16u;
#pragma unroll
                    for (int t = 0; t < CPL / 2; ++t) {
                        const uint32_t pair = __builtin_amdgcn_alignbit(w[u][t + 1], w[u][t], shift);
                        q[2 * t] = pair << 16;
                        q[2 * t + 1] = pair & 0xFFFF0000u;
                    }
                }
                // a set column takes the head of the window and advances it; all-ones / all-zero
                // words from a signed bit extract drive bitwise selects, no condition codes
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) {
                    const uint32_t m = (uint32_t)__builtin_amdgcn_sbfe((int)nib[u], cb, 1);
                    const uint32_t b = q[0] & m;
#pragma unroll
                    for (int t = 0; t + 1 < CPL - cb; ++t) q[t] = bit_select(m, q[t + 1], q[t]);
                    if constexpr (ONE_ROW) acc[cb][0] = __builtin_fmaf(p[u], __uint_as_float(b), acc[cb][0]);
                    else if constexpr (sizeof(T) == 4) acc[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(p[u], __uint_as_float(b), acc[cb], 0, 0, 0);
                    else bq[u][cb] = b;
                }
            }
            if constexpr (sizeof(T) != 4 && !ONE_ROW) {
#pragma unroll
                for (int u = 0; u < GB; u += 4) {
                    bf16x4 ph, pm, pl;
                    split_p4(p + u, ph, pm, pl);
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) {
                        const bf16x4 b = pack_upper4(bq[u][cb], bq[u + 1][cb], bq[u + 2][cb], bq[u + 3][cb]);
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ph, b, acc[cb], 0, 0, 0);
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pm, b, acc[cb], 0, 0, 0);
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pl, b, acc[cb], 0, 0, 0);
                    }
                }
            }
        });
    }
}

// The same sums in ordinary arithmetic, for float32 records (Section 4.1, eq. (10)): on this chip float32 matrix
// instructions do not hide under vector work, and a 16-row product spends fifteen rows of every edge on zeros.
// The staged edges of a round are cut into four equal runs, one per group of sixteen lanes; a group walks its run
// in order (rows do not decrease along it), lane j of the group keeping a running sum of its CPL columns for the
// run's present row and adding it to the row of the LDS tile `st` (zeroed by the caller, row stride DG + 1) when
// the row changes and at the end of the round.  Two groups never add to one row in the same instruction: inside a
// round only the last run that holds a row sees it end; the sums left at the end of the round are added group by
// group.  The order of the additions is fixed by the edge list alone.
template <int DG, int GB, bool LUT = false>
__device__ __forceinline__ void gather_records_rows(const CsrView& g, const float* __restrict__ vals,
                                                    const typename MaskOf<DG>::type* __restrict__ masks, int k, int e_a,
                                                    int e_b, const int* s_rp, RecEdge* ebuf, uint8_t* rbuf, int lane,
                                                    float* st, const DealLutF* lut = nullptr) {
    using M = typename MaskOf<DG>::type;
    constexpr int CPL = DG / 16, LR = DG + 1;
    const int i16 = lane & 15, kk = lane >> 4, bp = CPL * i16;
    const uint32_t sh = bp & 31;
    const bool upper = bp >= 32;
    const uint32_t below_lo = upper ? 0xFFFFFFFFu : (1u << sh) - 1u, below_hi = upper ? (1u << sh) - 1u : 0u;
    float* mine = st + bp;
    for (int eb = e_a; eb < e_b; eb += 64) {
        const int e = eb + lane;
        const bool ok = e < e_b;
        const int ec = ok ? e : e_b - 1;
        const int j = __builtin_nontemporal_load(g.ci + ec);
        RecEdge me;
        me.a = ok ? __builtin_nontemporal_load(g.av + ec) : 0.f;
        const M m = masks[j];
        me.off0 = (uint32_t)j * (uint32_t)k;
        me.mlo = (uint32_t)m;
        if constexpr (DG == 64) me.mhi = (uint32_t)(m >> 32);
        else me.mhi = 0u;
        // The places of the round past its last edge are staged too: the last edge once more with a_ij = 0.
        // A run is a whole number of batches, so every place a lane group reads is staged and adds what it should: no
        // test per edge for the end of the run or of the round.
        const int r = tile_row_of(s_rp, ec);
        wave_sync();          // readers of the previous round are done
        ebuf[lane] = me;
        rbuf[lane] = (uint8_t)r;
        wave_sync();
        const int cnt = e_b - eb < 64 ? e_b - eb : 64;     // wave-uniform
        const int steps = (((cnt + 3) >> 2) + GB - 1) / GB * GB;      // edges per run (at most 16: GB divides 16)
        static_assert(16 % GB == 0, "a run must end inside the 64 staged places");
        const int first = kk * steps;
        int cur = (int)rbuf[first];
        float run[CPL];
#pragma unroll
        for (int cb = 0; cb < CPL; ++cb) run[cb] = 0.f;
        for (int s0 = 0; s0 < steps; s0 += GB) {
            uint32_t w[GB][CPL], nib[GB];
            float p[GB];
            int row[GB];
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                const int ei = first + s0 + u;
                const RecEdge er = ebuf[ei];
                const uint32_t word = upper ? er.mhi : er.mlo;
                const uint32_t at = er.off0 + (uint32_t)__popc(er.mlo & below_lo) + (uint32_t)__popc(er.mhi & below_hi);
                nib[u] = (word >> sh) & ((1u << CPL) - 1u);
                load_words<CPL>(vals + (size_t)at, w[u]);
                p[u] = er.a;
                row[u] = (int)rbuf[ei];
            }
            constexpr bool PERM = LUT && CPL == 4;
            uint4 sa_next = make_uint4(0u, 0u, 0u, 0u);      // selectors of the edge after the present one
            uint2 sb_next = make_uint2(0u, 0u);
            if constexpr (PERM) {
                sa_next = *reinterpret_cast<const uint4*>(lut->sel[nib[0]]);
                sb_next = *reinterpret_cast<const uint2*>(lut->sel[nib[0]] + 4);
            }
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                const uint4 sa = sa_next;
                const uint2 sb = sb_next;
                if constexpr (PERM) {
                    if (u + 1 < GB) {
                        sa_next = *reinterpret_cast<const uint4*>(lut->sel[nib[u + 1 < GB ? u + 1 : u]]);
                        sb_next = *reinterpret_cast<const uint2*>(lut->sel[nib[u + 1 < GB ? u + 1 : u]] + 4);
                    }
                }
                if (row[u] != cur) {     // the row of this run has ended: its sum joins the tile
                    float was[CPL];            // (all reads before the writes: one LDS round trip, not one per pair)
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) was[cb] = mine[cur * LR + cb];
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) {
                        mine[cur * LR + cb] = was[cb] + run[cb];
                        run[cb] = 0.f;
                    }
                    cur = row[u];
                }
                if constexpr (PERM) {
                    const uint32_t b0 = __builtin_amdgcn_perm(0u, w[u][0], sa.x);
                    const uint32_t b1 = __builtin_amdgcn_perm(w[u][1], w[u][0], sa.y);
                    const uint32_t b2 = __builtin_amdgcn_perm(w[u][1], w[u][0], sa.z) | __builtin_amdgcn_perm(0u, w[u][2], sa.w);
                    const uint32_t b3 = __builtin_amdgcn_perm(w[u][1], w[u][0], sb.x) | __builtin_amdgcn_perm(w[u][3], w[u][2], sb.y);
                    run[0] = __builtin_fmaf(p[u], __uint_as_float(b0), run[0]);
                    run[1] = __builtin_fmaf(p[u], __uint_as_float(b1), run[1]);
                    run[2] = __builtin_fmaf(p[u], __uint_as_float(b2), run[2]);
                    run[3] = __builtin_fmaf(p[u], __uint_as_float(b3), run[3]);
                    continue;
                }
                uint32_t q[CPL];
#pragma unroll
                for (int t = 0; t < CPL; ++t) q[t] = w[u][t];
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) {
                    const uint32_t mbit = (uint32_t)__builtin_amdgcn_sbfe((int)nib[u], cb, 1);
                    const uint32_t b = q[0] & mbit;
#pragma unroll
                    for (int t = 0; t + 1 < CPL - cb; ++t) q[t] = bit_select(mbit, q[t + 1], q[t]);
                    run[cb] = __builtin_fmaf(p[u], __uint_as_float(b), run[cb]);
                }
            }
        }
        // what the runs still hold, one group after the other (neighbouring runs may end in the same row)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            wave_sync();
            if (kk == gq) {
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) mine[cur * LR + cb] += run[cb];
            }
        }
    }
}

// The same for a dense float32 plane X (row stride ld): st += P * X over the edges [e_a, e_b) of ordinary rows.
template <int DG, int GB>
__device__ __forceinline__ void gather_dense_rows(const CsrView& g, const float* __restrict__ x, int64_t ld, int e_a, int e_b,
                                                  const int* s_rp, EdgeRec* ebuf, int lane, float* st) {
    constexpr int CPL = DG / 16, LR = DG + 1;
    const int i16 = lane & 15, kk = lane >> 4;
    const float* xl = x + CPL * i16;
    const uint32_t ldu = (uint32_t)ld;
    float* mine = st + CPL * i16;
    for (int eb = e_a; eb < e_b; eb += 64) {
        const int e = eb + lane;
        const bool ok = e < e_b;
        EdgeRec me;
        const int ec = ok ? e : e_b - 1;                 // (places past the last edge: the last edge once more with a_ij = 0)
        me.j = __builtin_nontemporal_load(g.ci + ec);
        me.a = ok ? __builtin_nontemporal_load(g.av + ec) : 0.f;
        me.r = tile_row_of(s_rp, ec);
        me.pad = 0;
        wave_sync();          // readers of the previous round are done
        ebuf[lane] = me;
        wave_sync();
        const int cnt = e_b - eb < 64 ? e_b - eb : 64;
        const int steps = (((cnt + 3) >> 2) + GB - 1) / GB * GB;
        static_assert(16 % GB == 0, "a run must end inside the 64 staged places");
        const int first = kk * steps;
        int cur = ebuf[first].r;
        float run[CPL];
#pragma unroll
        for (int cb = 0; cb < CPL; ++cb) run[cb] = 0.f;
        for (int s0 = 0; s0 < steps; s0 += GB) {
            uint32_t w[GB][CPL];
            float p[GB];
            int row[GB];
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                const EdgeRec er = ebuf[first + s0 + u];
                load_words<CPL>(xl + (size_t)(uint32_t)er.j * ldu, w[u]);
                p[u] = er.a;
                row[u] = er.r;
            }
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                if (row[u] != cur) {
                    float was[CPL];            // (all reads before the writes: one LDS round trip, not one per pair)
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) was[cb] = mine[cur * LR + cb];
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) {
                        mine[cur * LR + cb] = was[cb] + run[cb];
                        run[cb] = 0.f;
                    }
                    cur = row[u];
                }
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) run[cb] = __builtin_fmaf(p[u], __uint_as_float(w[u][cb]), run[cb]);
            }
        }
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            wave_sync();
            if (kk == gq) {
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) mine[cur * LR + cb] += run[cb];
            }
        }
    }
}

template <int DG, bool FAST = true>
__device__ __forceinline__ void hub_rows_fill(const CsrView& g, const float* __restrict__ hub_part, int r0, const int* s_rp,
                                              float* st, int lane);

// H of the tile into st through gather_records_rows: st is cleared, the runs of ordinary rows are added into it,
// split rows receive the sum of their first-pass partial rows afterwards.
template <int DG, bool FAST = true, typename Range>
__device__ __forceinline__ void tile_gather_rows(const CsrView& g, const float* __restrict__ hub_part, bool has_hub, int r0,
                                                 const int* s_rp, float* st, int lane, Range range) {
    for (int i = lane; i < 16 * (DG + 1); i += 64) st[i] = 0.f;
    wave_sync();
    tile_ranges(g, has_hub, s_rp, range);
    wave_sync();
    if (has_hub) hub_rows_fill<DG, FAST>(g, hub_part, r0, s_rp, st, lane);
}

// sum of the first-pass partial rows of every split row of the tile into st, each row's in chunk order.  On a graph of
// long rows every row of every tile is split, into one or two chunks, and a tile is all a wave has to do in a launch:
// what counts is the number of memory round trips in a row.  So the sixteen rows find their places in the list of
// split rows from one number per tile (split rows before the tile) and a count over the lanes before them, not by a
// search each; the first partial rows of all sixteen are requested together, then the second ones, up to the fourth;
// and only rows of more than four chunks go on one by one, sixteen loads in flight (Table-1-shaped graph: forward
// kernel 43 -> 38 us per launch, fused inverse + dW 51 -> 46 us).  The additions of a row are 0 + p_0 + p_1 + .. in this
// order whatever the batching.
constexpr int HUB_FILL_ROWS = 16;     // rows whose partial rows are requested together
constexpr int HUB_FILL_DEPTH = 4;     // partial rows per row taken that way (the launch of a long-row graph ends with the
                                      // tile whose rows go on one by one: 26 us against a median of 6)
template <int DG, bool FAST>
__device__ __forceinline__ void hub_rows_fill(const CsrView& g, const float* __restrict__ hub_part, int r0, const int* s_rp,
                                              float* st, int lane) {
    // (FAST = false: a search per row and the rows one by one - for kernels that have no register to spare; same
    // additions)
    if constexpr (!FAST) {
        int q0s = 0, q1s = 0;
        if (lane < 16 && (s_rp[lane + 1] - s_rp[lane]) > g.hub_threshold) {
            const int h = find_hub(g, r0 + lane);
            q0s = g.hub_cptr[h];
            q1s = g.hub_cptr[h + 1];
        }
        for (int r = 0; r < 16; ++r) {
            int q = __builtin_amdgcn_readlane(q0s, r);
            const int q1 = __builtin_amdgcn_readlane(q1s, r);
            if (q1 <= q) continue;                 // not a split row
            const int cc = lane < DG ? lane : 0;
            float acc = 0.f;
            for (; q + 16 <= q1; q += 16) {
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = hub_part[(size_t)(q + u) * DG + cc];
#pragma unroll
                for (int u = 0; u < 16; ++u) acc += v[u];
            }
            for (; q < q1; ++q) acc += hub_part[(size_t)q * DG + cc];
            if (lane < DG) st[r * (DG + 1) + lane] = acc;
        }
        return;
    }
    const bool split = lane < 16 && (s_rp[lane + 1] - s_rp[lane]) > g.hub_threshold;
    const uint64_t splits = __builtin_amdgcn_ballot_w64(split);
    int q0v = 0, q1v = 0;
    if (split) {
        const int h = g.hub_tile0[r0 >> 4] + __popcll(splits & (((uint64_t)1 << lane) - 1));
        q0v = g.hub_cptr[h];
        q1v = g.hub_cptr[h + 1];
    }
    const int c = lane < DG ? lane : 0;
    // partial row j of every row that has one, j = 0 .. HUB_FILL_DEPTH - 1, while any row has one
    for (int j = 0; j < HUB_FILL_DEPTH; ++j) {
        if (__builtin_amdgcn_ballot_w64(q1v - q0v > j) == 0) break;
#pragma unroll
        for (int rb = 0; rb < 16; rb += HUB_FILL_ROWS) {
            float v[HUB_FILL_ROWS];
#pragma unroll
            for (int u = 0; u < HUB_FILL_ROWS; ++u) {
                const int q = __builtin_amdgcn_readlane(q0v, rb + u) + j, q1 = __builtin_amdgcn_readlane(q1v, rb + u);
                v[u] = hub_part[(size_t)(q < q1 ? q : 0) * DG + c];        // (no chunk j: any row, not used)
            }
#pragma unroll
            for (int u = 0; u < HUB_FILL_ROWS; ++u) {
                const int r = rb + u;
                const int q = __builtin_amdgcn_readlane(q0v, r) + j, q1 = __builtin_amdgcn_readlane(q1v, r);
                if (q < q1 && lane < DG) st[r * (DG + 1) + lane] = (j == 0 ? 0.f : st[r * (DG + 1) + lane]) + v[u];
            }
        }
    }
    // rows of more chunks than that go on one by one, sixteen loads in flight
    for (int r = 0; r < 16; ++r) {
        int q = __builtin_amdgcn_readlane(q0v, r) + HUB_FILL_DEPTH;
        const int q1 = __builtin_amdgcn_readlane(q1v, r);
        if (q1 <= q) continue;
        float acc = st[r * (DG + 1) + c];
        for (; q + 16 <= q1; q += 16) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = hub_part[(size_t)(q + u) * DG + c];
#pragma unroll
            for (int u = 0; u < 16; ++u) acc += v[u];
        }
        for (; q < q1; ++q) acc += hub_part[(size_t)q * DG + c];
        if (lane < DG) st[r * (DG + 1) + lane] = acc;
    }
}

// Calls `range(e_a, e_b)` for every maximal run of ordinary (not split) rows of the tile.
template <typename Range>
__device__ __forceinline__ void tile_ranges(const CsrView& g, bool has_hub, const int* s_rp, Range range) {
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
    }
}

// H of the tile into st (16 rows of DG+1 floats): the runs of ordinary rows go through
// `range(e_a, e_b)`, which accumulates into acc (D[4 (lane / 16) + reg][j] of column block cb,
// column = CPL j + cb); split rows receive the sum of their first-pass partial rows afterwards.
template <int DG, bool FAST = true, typename Range>
__device__ __forceinline__ void tile_gather(const CsrView& g, const float* __restrict__ hub_part, bool has_hub, int r0,
                                            const int* s_rp, float* st, int lane, f32x4 (&acc)[DG / 16], Range range) {
    constexpr int CPL = DG / 16, LR = DG + 1;
#pragma unroll
    for (int cb = 0; cb < CPL; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    tile_ranges(g, has_hub, s_rp, range);
#pragma unroll
    for (int cb = 0; cb < CPL; ++cb)
#pragma unroll
        for (int r = 0; r < 4; ++r) st[(4 * (lane >> 4) + r) * LR + CPL * (lane & 15) + cb] = acc[cb][r];
    if (has_hub) hub_rows_fill<DG, FAST>(g, hub_part, r0, s_rp, st, lane);
}

// ---- 16-row MFMA tiles -------------------------------------------------------------------------
// A wave multiplies its 16 x DG tile (staged in LDS, row stride DG+1) by a DG x DG matrix with
// v_mfma_f32_16x16x4_f32:
//   A[i][kk]: lane = kk*16 + i;  B[kk][j]: lane = kk*16 + j;  D[4*(lane/16)+r][lane%16] in reg r.
// The DG x DG weight matrix (row stride ldw in memory: DG, or more when it is a block of a wider matrix) sits in LDS (odd row stride DG + 1, which spreads the four k-rows of a
// B operand over different banks), loaded once per workgroup; transposed = true stores W^T.
template <int DG>
struct WLds {
    static constexpr int WP = DG + 1;
    float w[DG * WP];
};

template <int DG>
__device__ __forceinline__ void load_w_lds(const float* __restrict__ w, int ldw, bool transposed, WLds<DG>& l) {
    // eight loads of a thread in flight at a time: on a graph where a launch is one short tile per wave this
    // prologue is a good part of the launch, and one load after the other is a round trip to memory each
    // (the transposed form, whose loads touch a cache line per lane, was a tenth slower that way and keeps the plain loop)
    constexpr int NL = 8;
    const int nt = blockDim.x;
    if (transposed) {
        for (int i = threadIdx.x; i < DG * DG; i += nt) {
            const int r = i / DG, cc = i % DG;
            l.w[r * WLds<DG>::WP + cc] = w[cc * ldw + r];
        }
    } else {
        for (int i0 = threadIdx.x; i0 < DG * DG; i0 += NL * nt) {
            float v[NL];
#pragma unroll
            for (int u = 0; u < NL; ++u) {
                const int i = i0 + u * nt < DG * DG ? i0 + u * nt : 0;
                v[u] = w[(i / DG) * ldw + i % DG];
            }
#pragma unroll
            for (int u = 0; u < NL; ++u) {
                const int i = i0 + u * nt;
                if (i < DG * DG) l.w[(i / DG) * WLds<DG>::WP + i % DG] = v[u];
            }
        }
    }
    __syncthreads();
}

// acc = tile (16 x DG, LDS, row stride DG+1) * B (DG x DG, LDS), left in the tile register
// layout: acc[cb][reg] = product[row 4 reg + lane / 16][column CPL (lane % 16) + cb].
template <int DG>
__device__ __forceinline__ void mfma_tile(const float* st, const WLds<DG>& wl, f32x4 (&acc)[DG / 16]) {
    constexpr int CPL = DG / 16;
    const int lane = lane_id(), i = lane & 15, kk = lane >> 4;
    const int arow = 4 * (i & 3) + (i >> 2);
#pragma unroll
    for (int cb = 0; cb < CPL; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < DG / 4; ++s) {
        const float a = st[arow * (DG + 1) + 4 * s + kk];
#pragma unroll
        for (int cb = 0; cb < CPL; ++cb) {
            const float b = wl.w[(4 * s + kk) * WLds<DG>::WP + CPL * i + cb];
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[cb], 0, 0, 0);
        }
    }
}

// ---- the same products on the bf16 matrix pipe, exact to float32 rounding --------------------------------
// A float32 value is the exact sum of three bf16 terms (8 + 8 + 8 significant bits: hi = the value truncated to bf16,
// mid = the remainder truncated, lo = what is left).  A product a b is then the sum of nine exact bf16 products, of
// which the six with the largest weights (hi hi, hi mid, mid hi, hi lo, mid mid, lo hi) carry it to 2^-24 relative:
// what a float32 multiply would round away.  v_mfma_f32_16x16x16_bf16 forms such products exactly and adds them in
// float32, takes 16 K-slots per instruction and, unlike the float32 matrix instructions of this chip, runs beside
// the vector pipe, so the six products of a 16-deep step cost less than the one float32 instruction sequence they
// replace and hide under the vector work of the other waves.
// W is kept in LDS already split and laid out as B operands: entry [term][s][cb][lane] holds, for lane (kk = lane / 16,
// j = lane % 16), the four bf16 of rows 16 s + 4 kk .. + 3 of column CPL j + cb (of W, or of W^T).
template <int DG>
struct WLdsB3 {
    uint64_t w[3][DG / 16][DG / 16][64];
};

__device__ __forceinline__ uint64_t as_u64(bf16x4 v) { return __builtin_bit_cast(uint64_t, v); }
__device__ __forceinline__ bf16x4 as_bf16x4(uint64_t v) { return __builtin_bit_cast(bf16x4, v); }

template <int DG>
__device__ __forceinline__ void load_w_lds_b3(const float* __restrict__ w, int ldw, bool transposed, WLdsB3<DG>& l) {
    constexpr int CPL = DG / 16, NB = DG / 16;
    // (the loads of two of a thread's items in flight at a time, as in load_w_lds; not for the transposed form)
    constexpr int NI = 2, ITEMS = NB * NB * 64;
    const int nt = blockDim.x;
    if (transposed) {
        for (int e = threadIdx.x; e < ITEMS; e += nt) {
            const int lane = e & 63, cb = (e >> 6) % NB, s = (e >> 6) / NB;
            const int kk = lane >> 4, j = lane & 15, col = CPL * j + cb;
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = w[col * ldw + 16 * s + 4 * kk + u];
            bf16x4 hi, mid, lo;
            split_p4(v, hi, mid, lo);
            l.w[0][s][cb][lane] = as_u64(hi);
            l.w[1][s][cb][lane] = as_u64(mid);
            l.w[2][s][cb][lane] = as_u64(lo);
        }
        __syncthreads();
        return;
    }
    for (int e0 = threadIdx.x; e0 < ITEMS; e0 += NI * nt) {
        float v[NI][4];
#pragma unroll
        for (int t = 0; t < NI; ++t) {
            const int e = e0 + t * nt < ITEMS ? e0 + t * nt : 0;
            const int lane = e & 63, cb = (e >> 6) % NB, s = (e >> 6) / NB;
            const int kk = lane >> 4, j = lane & 15, col = CPL * j + cb;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int row = 16 * s + 4 * kk + u;
                v[t][u] = w[row * ldw + col];
            }
        }
#pragma unroll
        for (int t = 0; t < NI; ++t) {
            const int e = e0 + t * nt;
            if (e < ITEMS) {
                const int lane = e & 63, cb = (e >> 6) % NB, s = (e >> 6) / NB;
                bf16x4 hi, mid, lo;
                split_p4(v[t], hi, mid, lo);
                l.w[0][s][cb][lane] = as_u64(hi);
                l.w[1][s][cb][lane] = as_u64(mid);
                l.w[2][s][cb][lane] = as_u64(lo);
            }
        }
    }
    __syncthreads();
}

// acc = tile (16 x DG float32, LDS, row stride DG+1) * W, in the tile register layout of mfma_tile.
template <int DG>
__device__ __forceinline__ void mfma_tile_b3(const float* st, const WLdsB3<DG>& wl, f32x4 (&acc)[DG / 16]) {
    constexpr int CPL = DG / 16;
    const int lane = lane_id(), i = lane & 15, kk = lane >> 4;
    const int arow = 4 * (i & 3) + (i >> 2);
#pragma unroll
    for (int cb = 0; cb < CPL; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < DG / 16; ++s) {
        float a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a[u] = st[arow * (DG + 1) + 16 * s + 4 * kk + u];
        bf16x4 ah, am, al;
        split_p4(a, ah, am, al);
#pragma unroll
        for (int cb = 0; cb < CPL; ++cb) {
            const bf16x4 bh = as_bf16x4(wl.w[0][s][cb][lane]), bm = as_bf16x4(wl.w[1][s][cb][lane]),
                         bl = as_bf16x4(wl.w[2][s][cb][lane]);
            // smallest terms first
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(al, bh, acc[cb], 0, 0, 0);
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(am, bm, acc[cb], 0, 0, 0);
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bl, acc[cb], 0, 0, 0);
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(am, bh, acc[cb], 0, 0, 0);
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bm, acc[cb], 0, 0, 0);
            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bh, acc[cb], 0, 0, 0);
        }
    }
}

// dW += H^T dY over the 16 rows of the tile, as mfma_outer, on the bf16 pipe.  The 16 rows are the 16 K-slots of one
// instruction; K-slot 4 kk + u stands for tile row 4 u + kk, so that the B operand of lane (kk, j) is what the lane
// already holds of dY (gy[u][ob], rows 4 u + kk) and the A operand is H[4 u + kk][16 mb + j] from the LDS tile.
template <int DG>
__device__ __forceinline__ void mfma_outer_b3(const float* st_h, const float (&gy)[4][DG / 16], f32x4 (&acc)[DG / 16][DG / 16]) {
    const int lane = lane_id(), kk = lane >> 4, j = lane & 15;
    bf16x4 bh[DG / 16], bm[DG / 16], bl[DG / 16];
#pragma unroll
    for (int ob = 0; ob < DG / 16; ++ob) {
        const float b[4] = {gy[0][ob], gy[1][ob], gy[2][ob], gy[3][ob]};
        split_p4(b, bh[ob], bm[ob], bl[ob]);
    }
#pragma unroll
    for (int mb = 0; mb < DG / 16; ++mb) {
        float a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a[u] = st_h[(4 * u + kk) * (DG + 1) + 16 * mb + j];
        bf16x4 ah, am, al;
        split_p4(a, ah, am, al);
#pragma unroll
        for (int ob = 0; ob < DG / 16; ++ob) {
            acc[mb][ob] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(al, bh[ob], acc[mb][ob], 0, 0, 0);
            acc[mb][ob] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(am, bm[ob], acc[mb][ob], 0, 0, 0);
            acc[mb][ob] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bl[ob], acc[mb][ob], 0, 0, 0);
            acc[mb][ob] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(am, bh[ob], acc[mb][ob], 0, 0, 0);
            acc[mb][ob] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bm[ob], acc[mb][ob], 0, 0, 0);
            acc[mb][ob] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ah, bh[ob], acc[mb][ob], 0, 0, 0);
        }
    }
}

// dW += H^T dY over the 16 rows of the tile: D[m][o] += sum_n H[n][m] dY[n][o].  H comes from the
// LDS tile; dY is held in the tile register layout (gy[reg][cb] = dY[row 4 reg + lane / 16]
// [column CPL (lane % 16) + cb]), which is the B operand as it stands.  The result has its
// columns interleaved the same way: acc[mb][ob][r] = dW[16 mb + 4 (lane / 16) + r][CPL (lane % 16) + ob].
template <int DG>
__device__ __forceinline__ void mfma_outer(const float* st_h, const float (&gy)[4][DG / 16], f32x4 (&acc)[DG / 16][DG / 16]) {
    const int lane = lane_id();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int nrow = 4 * ks + (lane >> 4);
#pragma unroll
        for (int mb = 0; mb < DG / 16; ++mb) {
            const float a = st_h[nrow * (DG + 1) + 16 * mb + (lane & 15)];
#pragma unroll
            for (int ob = 0; ob < DG / 16; ++ob)
                acc[mb][ob] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, gy[ks][ob], acc[mb][ob], 0, 0, 0);
        }
    }
}

// ---- GS of a 16-row tile --------------------------------------------------------------------------
// Compressed record of a row ("CBSR" of Section 4.3): the k kept values in ascending column
// order (already RMS-scaled) and the row's column bit mask.
template <int DG, typename T>
struct Record {
    using M = typename MaskOf<DG>::type;
    T* vals;        // [n][k]
    M* mask;        // [n]
};

// ---- the k-th largest key of a row when k is a quarter of its width -------------------------------
// (k = 16 of 64 columns, k = 8 of 32: the shapes of the benchmark configurations.)  A selection network of fixed
// cost instead of a search whose length depends on the data (Section 4.1: the k largest entries of a row).
// Lane (r, q) holds QW = k keys of row r.
//   1. every lane sorts its keys (Batcher's odd-even merge sort): even quarters descending, odd quarters ascending
//      in register order;
//   2. quarters (0,1) and (2,3): u[i] = max(even[i], odd[i]) pairs the i-th largest of one with the i-th smallest of
//      the other, so u is the set of the k largest of the two quarters, and a bitonic sequence; the even lane keeps
//      u[0 .. k/2), the odd lane the rest;
//   3. a bitonic merge sorts u over the two lanes: quarters (0,1) descending, quarters (2,3) ascending;
//   4. the same pairing over the halves leaves the k largest of the whole row; their minimum is the answer.
// A compare-exchange whose direction depends on the lane is two v_med3_u32 with a third operand of all ones
// (the median is then the larger of the two) or zero (the smaller).
constexpr int SORT8[19][2] = {{0, 1}, {2, 3}, {4, 5}, {6, 7}, {0, 2}, {1, 3}, {4, 6}, {5, 7}, {1, 2}, {5, 6},
                              {0, 4}, {1, 5}, {2, 6}, {3, 7}, {2, 4}, {3, 5}, {1, 2}, {3, 4}, {5, 6}};
constexpr int SORT16[63][2] = {
    {0, 1}, {2, 3}, {4, 5}, {6, 7}, {8, 9}, {10, 11}, {12, 13}, {14, 15}, {0, 2}, {1, 3}, {4, 6}, {5, 7}, {8, 10},
    {9, 11}, {12, 14}, {13, 15}, {1, 2}, {5, 6}, {9, 10}, {13, 14}, {0, 4}, {1, 5}, {2, 6}, {3, 7}, {8, 12}, {9, 13},
    {10, 14}, {11, 15}, {2, 4}, {3, 5}, {10, 12}, {11, 13}, {1, 2}, {3, 4}, {5, 6}, {9, 10}, {11, 12}, {13, 14}, {0, 8},
    {1, 9}, {2, 10}, {3, 11}, {4, 12}, {5, 13}, {6, 14}, {7, 15}, {4, 8}, {5, 9}, {6, 10}, {7, 11}, {2, 4}, {3, 5},
    {6, 8}, {7, 9}, {10, 12}, {11, 13}, {1, 2}, {3, 4}, {5, 6}, {7, 8}, {9, 10}, {11, 12}, {13, 14}};

__device__ __forceinline__ uint32_t med3_u32(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t d;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}
// a <- the larger of (a, b) where up is all ones, the smaller where it is zero; b <- the other one
__device__ __forceinline__ void compare_exchange(uint32_t& a, uint32_t& b, uint32_t up) {
    const uint32_t hi = med3_u32(a, b, up), lo = med3_u32(a, b, ~up);
    a = hi; b = lo;
}

template <int QW>
__device__ __forceinline__ uint32_t kth_largest_quarter(const uint32_t (&key)[QW], int q) {
    static_assert(QW == 8 || QW == 16, "selection network for 8 or 16 keys per lane");
    constexpr int H = QW / 2, NCE = QW == 16 ? 63 : 19;
    uint32_t s[QW];
#pragma unroll
    for (int j = 0; j < QW; ++j) s[j] = key[j];
    const uint32_t up1 = (q & 1) ? 0u : 0xFFFFFFFFu;
#pragma unroll
    for (int c = 0; c < NCE; ++c) {
        if constexpr (QW == 16) compare_exchange(s[SORT16[c][0]], s[SORT16[c][1]], up1);
        else compare_exchange(s[SORT8[c][0]], s[SORT8[c][1]], up1);
    }
    uint32_t t[H];
#pragma unroll
    for (int i = 0; i < H; ++i) {
        const auto a = __builtin_amdgcn_permlane16_swap(s[i], s[i + H], false, false);
        t[i] = max(a[0], a[1]);
    }
    const uint32_t up3 = (q == 0 || q == 3) ? 0xFFFFFFFFu : 0u, upl = q < 2 ? 0xFFFFFFFFu : 0u;
#pragma unroll
    for (int i = 0; i < H; ++i) {
        const auto a = __builtin_amdgcn_permlane16_swap(t[i], t[i], false, false);
        t[i] = med3_u32(a[0], a[1], up3);
    }
#pragma unroll
    for (int d = H / 2; d >= 1; d >>= 1) {
#pragma unroll
        for (int i = 0; i < H; ++i)
            if ((i & d) == 0) compare_exchange(t[i], t[i + d], upl);
    }
    uint32_t m = 0xFFFFFFFFu;
#pragma unroll
    for (int i = 0; i < H / 2; ++i) {
        const auto a = __builtin_amdgcn_permlane32_swap(t[i], t[i + H / 2], false, false);
        m = min(m, max(a[0], a[1]));
    }
    const auto a = __builtin_amdgcn_permlane16_swap(m, m, false, false);
    const uint32_t m2 = min(a[0], a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(m2, m2, false, false);
    return min(b[0], b[1]);
}

// Bits of the quarter's columns that belong to the row's k largest entries (x: the quarter's QW
// values; valid: the row exists; q: the quarter).  All four lanes of a row must call it together.
template <int DG, int KS>
__device__ __forceinline__ uint32_t select_quarter(const float (&x)[DG / 4], int k, bool valid, int q) {
    constexpr int QW = DG / 4;
    uint32_t key[QW];
#pragma unroll
    for (int j = 0; j < QW; ++j) {
        const uint32_t u = __float_as_uint(x[j] + 0.0f);    // -0 -> +0, every other value as it is
        const uint32_t kk = u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
        key[j] = kk >> KS;
    }
    uint32_t lo;
    if (k == QW) {
        lo = kth_largest_quarter<QW>(key, q);          // the k-th largest key itself
    } else {
        uint32_t top = 0u;
#pragma unroll
        for (int j = 0; j < QW; ++j) top = max(top, key[j]);
        top = quarter_max(top);
        auto count_ge = [&](uint32_t t) {
            uint32_t cnt = 0u;
#pragma unroll
            for (int j = 0; j < QW; ++j) cnt += key[j] >= t ? 1u : 0u;
            return quarter_sum(cnt);
        };
        constexpr uint32_t span = (4u << 23) >> KS;
        const uint32_t uk = (uint32_t)k;
        uint32_t hi = top + 1u;
        lo = top > span ? top - span : 0u;
        const uint32_t cnt = count_ge(lo);
        lo = (cnt >= uk && k < DG) ? lo : 0u;
        uint32_t open = (cnt != uk && k < DG && valid) ? 1u : 0u;
        for (int round = 0; round < 33 && ballot(open != 0u) != 0ull; ++round) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            const uint32_t c2 = count_ge(mid);
            lo = c2 >= uk ? mid : lo;
            hi = c2 >= uk ? hi : mid;
            open = (c2 == uk || hi - lo <= 1u) ? 0u : open;
        }
    }
    // Column set of this quarter at or above the threshold, built as a shift register (a compare and an add with
    // carry per key).  It is the answer unless the row has more than k keys there: then several keys equal the
    // threshold (which is a key of the row in that case) and the lowest columns among them win.
    uint32_t mge = 0u;
#pragma unroll
    for (int j = QW - 1; j >= 0; --j) mge = mge + mge + (key[j] >= lo ? 1u : 0u);
    uint32_t msel = mge;
    if (ballot(quarter_sum((uint32_t)__popc(mge)) != (uint32_t)k) != 0ull) {
        uint32_t mgt = 0u;
#pragma unroll
        for (int j = QW - 1; j >= 0; --j) mgt = mgt + mgt + (key[j] > lo ? 1u : 0u);
        const uint32_t meq = mge & ~mgt;
        const uint32_t cg = __popc(mgt), ce = __popc(meq);
        uint32_t all[4];
        quarter_all(cg | ce << 8, all);
        const int need = k - (int)((all[0] & 255u) + (all[1] & 255u) + (all[2] & 255u) + (all[3] & 255u));
        int before = 0;   // ties in lower quarters
#pragma unroll
        for (int i = 0; i < 3; ++i) before += i < q ? (int)(all[i] >> 8) : 0;
        int take = min(max(need - before, 0), (int)ce);
        msel = mgt;
#pragma unroll
        for (int j = 0; j < QW; ++j) {
            const uint32_t s1 = ((meq >> j) & 1u) & (take > 0 ? 1u : 0u);
            msel |= s1 << j;
            take -= (int)s1;
        }
    }
    return msel;
}

// Rows whose column set is kept because they selected at a near-tie (a selective form of the save of Section 4.2):
// one segment per application of GS in the forward sweep.  A row is listed iff k < DG and, with v_k the smallest
// kept and v_(k+1) the largest dropped value, v_k - v_(k+1) <= tol * max|row| in float32 (exact ties always are).
// The inverse sweep selects again on the rebuilt rows and then gives the listed rows their kept sets back.
// The list of a segment is kept as TIE_SUB sub-lists, each with its own counter on its own cache line: a tile appends
// to sub-list (tile number mod TIE_SUB).  (All appends of a launch on one counter - 15 thousand at 1M rows - are served
// one after the other by the memory side: 36 us on a 172 us kernel.)
constexpr int TIE_SUB = 16, TIE_COUNTER_STRIDE = 32;
template <int DG>
struct TieSeg {
    using M = typename MaskOf<DG>::type;
    int* count;        // [TIE_SUB] counters, TIE_COUNTER_STRIDE ints apart: rows listed so far in each sub-list (may run
                       // past cap: the excess is not kept); NULL: nothing is listed
    uint32_t* rows;    // [TIE_SUB][cap]
    M* masks;          // [TIE_SUB][cap]
    int cap;           // places per sub-list
    float tol;
};

// The factor GS applies to the kept values of a row held in the quarter layout (x: this lane's quarter); the same
// value in the four lanes of the row.
template <int DG>
__device__ __forceinline__ float record_scale(const float (&x)[DG / 4], int norm, float eps) {
    float scale = 1.f;
    if (norm == GSR_NORM_RMS) {
        float ss = 0.f;
#pragma unroll
        for (int j = 0; j < DG / 4; ++j) ss += x[j] * x[j];
        ss = quarter_sum(ss);
        scale = __builtin_amdgcn_rsqf(ss * (1.0f / (float)DG) + eps);
    }
    return scale;
}

// GS of the 16 rows of an LDS tile and their records (Section 4.1; record layout of Section 4.3).
// st holds the rows as they read back from memory (16 x (DG+1) floats, rows past the end zero).
// Lane (r, q) takes the quarter q of row r into registers, so the 16 searches for the k-th largest
// key run side by side in vector registers on an order-preserving integer image of the values
// (select_quarter): a selection network when k is a quarter of the width, else interval bisection,
// count = own compares + the three partner quarters.  Invariant per row of the bisection: at
// least k keys are >= lo and fewer than k are >= hi; hi starts just above the row maximum, lo four
// binades below it (0 when a count says that is too high).  A row closes when a candidate splits
// off exactly k keys or the interval is down to one value (a tie at the k-th position); ties go
// to the lowest columns, -0 equals +0.  The kept values (RMS-scaled) are compacted in LDS in
// column order and leave as one contiguous block, since rows r0..r0+15 are adjacent in [n][k].
// With `given` the column set is not searched for: out.mask already holds the set an earlier
// application selected (Section 4.2 keeps the indices of the forward pass) and only the values
// are taken, from the present rows.  st is overwritten.  With idx_out (and ist, 16 * DG words of
// LDS scratch) the kept column numbers are written as well, [n][k] in ascending order, and
// out.mask may be NULL.
template <int DG, typename T>
__device__ __forceinline__ void emit_tile(float* st, int r0, int n, int k, int norm, float eps, const Record<DG, T>& out,
                                          bool given, int lane, int32_t* idx_out = nullptr, int* ist = nullptr,
                                          TieSeg<DG> tie = TieSeg<DG>{nullptr, nullptr, nullptr, 0, 0.f}) {
    using M = typename MaskOf<DG>::type;
    constexpr int QW = DG / 4, LR = DG + 1;
    constexpr int KS = sizeof(T) == 2 ? 16 : 0;   // bf16 values: the low 16 key bits are zero
    const int r = lane & 15, q = lane >> 4;
    float x[QW];
#pragma unroll
    for (int j = 0; j < QW; ++j) x[j] = st[r * LR + q * QW + j];
    uint32_t msel;
    if (given) {
        const M m = out.mask[r0 + r < n ? r0 + r : n - 1];
        msel = (uint32_t)(m >> (QW * q)) & ((1u << QW) - 1u);
    } else {
        msel = select_quarter<DG, KS>(x, k, r0 + r < n, q);
    }
    uint32_t all[4];
    quarter_all(msel | (uint32_t)__popc(msel) << 16, all);
    int slot = r * k;
#pragma unroll
    for (int i = 0; i < 3; ++i) slot += i < q ? (int)(all[i] >> 16) : 0;
    M mask;
    if constexpr (DG == 64)
        mask = (M)(all[0] & 0xFFFFu) | (M)(all[1] & 0xFFFFu) << 16 | (M)(all[2] & 0xFFFFu) << 32 | (M)(all[3] & 0xFFFFu) << 48;
    else
        mask = (all[0] & 0xFFu) | (all[1] & 0xFFu) << 8 | (all[2] & 0xFFu) << 16 | (all[3] & 0xFFu) << 24;
    if (tie.count && !given) {
        // near-tie test on the row's values: smallest kept, largest dropped, largest magnitude
        float vk = __builtin_huge_valf(), vr = -__builtin_huge_valf(), am = 0.f;
#pragma unroll
        for (int j = 0; j < QW; ++j) {
            const bool bit = (msel >> j) & 1u;
            vk = bit ? fminf(vk, x[j]) : vk;
            vr = bit ? vr : fmaxf(vr, x[j]);
            am = fmaxf(am, fabsf(x[j]));
        }
        vk = quarter_fmin(vk); vr = quarter_fmax(vr); am = quarter_fmax(am);
        const float gap = vk - vr, bar = tie.tol * am;
        if (q == 0 && r0 + r < n && k < DG && gap <= bar) {
            const int sub = (r0 >> 4) & (TIE_SUB - 1);
            const int pos = atomicAdd(tie.count + sub * TIE_COUNTER_STRIDE, 1);
            if (pos < tie.cap) { tie.rows[sub * tie.cap + pos] = (uint32_t)(r0 + r); tie.masks[sub * tie.cap + pos] = mask; }
        }
    }
    const float scale = record_scale<DG>(x, norm, eps);
    wave_sync();   // every lane holds its quarter: the tile can be reused for the compacted values
    // a kept value goes to its slot, a dropped one to the lane's dump word: word number = dump + bit * (slot - dump)
    const int dump = 16 * LR + lane;
    int ahead = slot - dump;
#pragma unroll
    for (int j = 0; j < QW; ++j) {
        const int bit = (int)((msel >> j) & 1u);
        st[dump + __mul24(bit, ahead)] = x[j] * scale;
        if (idx_out && bit) ist[dump + ahead] = q * QW + j;
        ahead += bit;
    }
    wave_sync();
    const int rows = min(16, n - r0), total = rows * k;
    T* dst = out.vals + (size_t)r0 * k;
    for (int i = lane; i < total; i += 64) dst[i] = from_float<T>(st[i]);
    if (idx_out)
        for (int i = lane; i < total; i += 64) idx_out[(size_t)r0 * k + i] = ist[i];
    if (!given && out.mask && q == 0 && r < rows) out.mask[r0 + r] = mask;
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
    // the wave index through readfirstlane: everything derived from the tile number then lives in scalar registers
    const int slot = local_wg * waves_per_wg + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    TileSweep t;
    const int t0 = (int)((int64_t)tiles * xcd / 8), t1 = (int)((int64_t)tiles * (xcd + 1) / 8);
    t.first = t0 + slot;
    t.end = t1;
    t.step = wg_per_xcd * waves_per_wg;
    return t;
}

// Dynamic form of the sweep.  Tiles differ a lot in cost (a few rows have hundreds of neighbours),
// and with a fixed assignment the kernel ends when the unluckiest wave does.  Here the tiles of an
// XCD's eighth are dealt to nq = TILE_NQ queues (queue q owns tiles t0 + q + nq v); a wave serves
// queue (its slot mod nq) and draws the queue's next tile from a counter, so a wave that drew
// long rows draws fewer tiles.  The active window still moves through the rows in order.  Many
// queues rather than one keep the atomics on different addresses: one counter for the 512 waves
// of an XCD serialises and costs more than the balance gains.  The next draw is requested at
// the start of a tile and read at its end.  A launch leaves the counters as it found them (all
// zero): every wave signs off when it has drawn its last tile, and the wave that signs off last
// clears them (tile_finish), so launches need no clearing step and may be replayed from a
// captured graph in any number.  Which wave processes which tile varies between runs; kernels
// that sum over the tiles a wave has seen must keep the fixed sweep.
constexpr int TILE_NQ = 64, TILE_QSTRIDE = 32;              // counters sit 128 bytes apart
constexpr int TILE_COUNTERS = 8 * TILE_NQ * TILE_QSTRIDE;   // ints of the counter set (the host allocates kTileCounters)
struct TileDraws {
    int* ctr;      // this wave's queue counter
    int base;      // first tile of the queue
    int nq;        // queues in use: TILE_NQ, or the number of waves of the XCD if that is smaller
    int end;       // one past the XCD's last tile
    int* set;      // the whole counter set
    int* done;     // waves that have signed off
};
__device__ __forceinline__ TileDraws tile_draws(int tiles, int* set, int* done) {
    const int xcd = blockIdx.x & 7;
    const int slot = (blockIdx.x >> 3) * (blockDim.x >> 6) + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int waves = (gridDim.x >> 3) * (blockDim.x >> 6);
    TileDraws d;
    d.nq = waves < TILE_NQ ? waves : TILE_NQ;
    const int q = slot % d.nq;
    d.ctr = set + (xcd * TILE_NQ + q) * TILE_QSTRIDE;
    d.base = (int)((int64_t)tiles * xcd / 8) + q;
    d.end = (int)((int64_t)tiles * (xcd + 1) / 8);
    d.set = set;
    d.done = done;
    return d;
}
// requests a draw; the value is valid in lane 0 once the wave waits for it (tile_drawn)
__device__ __forceinline__ int tile_request(const TileDraws& d) {
    int v = 0;
    if (lane_id() == 0) v = atomicAdd(d.ctr, 1);
    return v;
}
__device__ __forceinline__ int tile_drawn(const TileDraws& d, int requested) {
    return d.base + d.nq * __builtin_amdgcn_readfirstlane(requested);
}
// Every wave of the grid calls this once, after its last tile_drawn (all its draws have returned).
// Sign-off in two levels, an XCD's waves on the XCD's counter and the last wave of each XCD on a
// common one, keeps the atomics on one address few.  d.done: 9 counters, 128 bytes apart.
__device__ __forceinline__ void tile_finish(const TileDraws& d) {
    int last = 0;
    if (lane_id() == 0) {
        // no fence: this wave's own draws have returned, and nothing but the counters is handed over
        const int waves = (int)((gridDim.x >> 3) * (blockDim.x >> 6));
        if (atomicAdd(d.done + (blockIdx.x & 7) * TILE_QSTRIDE, 1) == waves - 1)
            last = atomicAdd(d.done + 8 * TILE_QSTRIDE, 1) == 7 ? 1 : 0;
    }
    if (__builtin_amdgcn_readfirstlane(last)) {
        for (int i = lane_id(); i < 8 * TILE_NQ; i += 64) d.set[i * TILE_QSTRIDE] = 0;
        if (lane_id() < 9) d.done[lane_id() * TILE_QSTRIDE] = 0;
    }
}

// ---- the long tiles first -----------------------------------------------------------------------------
// A tile with many stored entries takes many times longer than a median one.  Met late in a sweep it makes
// the kernel's tail; met twice by one wave of a fixed sweep it makes that wave the last.  The layer kernels
// therefore deal the listed heavy tiles out first, wave w of the grid taking entries w, w + waves, .. of the
// list, and pass them over in the sweep that follows (a tile is heavy by its row pointers alone, so the sweep
// needs no flag; the check sits after the tile's own rows have been requested, which costs a few wasted loads).  The assignment is the same on every run.
struct TileDeal {
    int at;        // this wave's next entry of the list
    int waves;     // waves of the grid
    bool on;       // still dealing
};
__device__ __forceinline__ TileDeal tile_deal(const CsrView& g) {
    TileDeal d;
    d.waves = (int)(gridDim.x * (blockDim.x >> 6));
    d.at = (int)(blockIdx.x * (blockDim.x >> 6)) + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    d.on = d.at < g.n_heavy;
    return d;
}
// s_rp: the tile's row pointers as tile_begin published them.  Rows that are split do not count: their
// neighbours are summed by the first pass.
__device__ __forceinline__ bool tile_is_heavy(const CsrView& g, int rpv, const int* s_rp, bool has_hub) {
    int e = __builtin_amdgcn_readlane(rpv, 16) - __builtin_amdgcn_readlane(rpv, 0);   // rpv: as tile_rp_load returned it
    if (e <= g.heavy_edges) return false;
    if (has_hub)
        for (int r = 0; r < 16; ++r) {
            const int d = s_rp[r + 1] - s_rp[r];
            e -= d > g.hub_threshold ? d : 0;
        }
    return e > g.heavy_edges;
}

// Per-wave LDS of the tile operators: staged edges, the tile's row pointers, rows of the staged records.
struct TileLds {
    EdgeRec ebuf[64];
    int rp[20];
    uint8_t rbuf[64];
};

// The order in which a wave of these kernels visits tiles: its share of the listed heavy tiles first (DEAL, see
// TileDeal), then tiles drawn from the counters, with the next draw requested a tile ahead.  (Walking one tile
// further ahead, so that the next tile's row pointers and first edges arrive during the present tile, was
// measured on the dense product: 233 us against 224, so it is not done.)
template <bool DEAL>
struct TileWalk {
    TileDraws td;
    TileDeal deal;
    int requested, t, t_end;
    __device__ __forceinline__ TileWalk(const CsrView& g, int tiles, int* set, int* done) {
        td = tile_draws(tiles, set, done);
        deal = TileDeal{0, 0, false};
        if constexpr (DEAL) deal = tile_deal(g);
        requested = tile_request(td);
        if (DEAL && deal.on) { t = g.heavy[deal.at]; t_end = tiles; }
        else { t = tile_drawn(td, requested); t_end = td.end; }
    }
    __device__ __forceinline__ bool more() const { return t < t_end; }
    // at the top of a tile: ask for the next draw (while dealing, the one asked for at the start is still out)
    __device__ __forceinline__ void ahead() { if (!DEAL || !deal.on) requested = tile_request(td); }
    // in the sweep, a heavy tile has been dealt out already
    __device__ __forceinline__ bool dealt(const CsrView& g, int rpv, const int* s_rp, bool has_hub) const {
        if constexpr (DEAL) return !deal.on && tile_is_heavy(g, rpv, s_rp, has_hub);
        return false;
    }
    __device__ __forceinline__ void next(const CsrView& g) {
        if (DEAL && deal.on) {
            deal.at += deal.waves;
            deal.on = deal.at < g.n_heavy;
            if (deal.on) { t = g.heavy[deal.at]; return; }
            t_end = td.end;
        }
        t = tile_drawn(td, requested);
    }
    __device__ __forceinline__ void finish() { tile_finish(td); }
};

// ---- first pass over the chunks of very long rows ------------------------------------------------
// One wave per chunk, through the staging and the wide loads of the tile gathers: the chunk is
// treated as a tile whose row 0 owns every edge, so all of a chunk's neighbours are in flight at
// once (a chain of one row pointer, the edges, the masks and the values instead of one such chain
// per edge).  The sums form in ordinary arithmetic (ONE_ROW of the gathers): lane (kk, j) adds the
// edges kk, kk + 4, .. for its columns, the four lane groups are added at the end.
// part[chunk][DG] receives the un-scaled partial row.
struct HubChunks {
    const int32_t* ce0;
    const int32_t* ce1;
    int32_t n_chunks;
    int32_t banded = 0;      // every XCD takes a contiguous eighth of the list (hub_sweep)
};

// Which chunks a wave takes; what a chunk's partial row holds does not depend on the wave that sums it.  The chunks
// are listed in row order and the hardware deals workgroups to the XCDs round-robin.  On a graph of long rows (nearly
// every row split, chunks alike in cost, neighbours within a few thousand rows) the sweep is banded: XCD x takes the
// x-th eighth of the list and its waves walk that eighth side by side, so the rows its L2 has to hold are the
// neighbourhood of a narrow band of rows and not that of every row in flight on the chip.  Elsewhere the split rows are
// few and unlike (a handful of rows with tens of thousands of neighbours from all over the graph, listed first, then
// rows of a few hundred): there the chunks go to the waves of the whole grid in turn, which shares the costly ones out
// (banded, the 8M-node workload's first passes took 117 us against 88).  Any grid is covered (banded with fewer than
// eight workgroups: one part each).
struct HubSweep {
    int q, end, step;
};
__device__ __forceinline__ HubSweep hub_sweep(const HubChunks& h) {
    const int wpw = (int)blockDim.x >> 6;
    HubSweep w;
    if (!h.banded) {
        w.q = (int)blockIdx.x * wpw + ((int)threadIdx.x >> 6);
        w.end = h.n_chunks;
        w.step = (int)gridDim.x * wpw;
        return w;
    }
    const int parts = gridDim.x < 8 ? (int)gridDim.x : 8;
    const int part = (int)blockIdx.x % parts, wg = (int)blockIdx.x / parts;
    const int wgs = ((int)gridDim.x - part + parts - 1) / parts;
    w.q = (int)((int64_t)h.n_chunks * part / parts) + wg * wpw + ((int)threadIdx.x >> 6);
    w.end = (int)((int64_t)h.n_chunks * (part + 1) / parts);
    w.step = wgs * wpw;
    return w;
}

struct HubLds {
    EdgeRec ebuf[64];
    int rp[20];
    uint8_t rbuf[64];
};
// row pointers of the pretended tile: row 0 spans [e0, e1), rows 1..15 are empty
__device__ __forceinline__ void hub_chunk_begin(HubLds& L, int e0, int e1, int lane) {
    wave_sync();
    if (lane < 17) L.rp[lane] = lane == 0 ? e0 : e1;
    wave_sync();
}
template <int DG>
__device__ __forceinline__ void hub_chunk_store(const f32x4 (&acc)[DG / 16], float* __restrict__ part, int lane) {
    constexpr int CPL = DG / 16;
    if (lane < 16) {
#pragma unroll
        for (int cb = 0; cb < CPL; ++cb) part[CPL * lane + cb] = acc[cb][0];
    }
}

template <int DG, typename T>
__device__ __forceinline__ void hub_records_pass(const CsrView& g, const HubChunks& h, const T* __restrict__ vals,
                                                 const typename MaskOf<DG>::type* __restrict__ masks, int k,
                                                 float* __restrict__ part, HubLds& L, const HubSweep w,
                                                 const DealLutF* lutf) {
    const int lane = lane_id();
    for (int q = w.q; q < w.end; q += w.step) {
        const int e0 = __builtin_amdgcn_readfirstlane(h.ce0[q]), e1 = __builtin_amdgcn_readfirstlane(h.ce1[q]);
        hub_chunk_begin(L, e0, e1, lane);
        f32x4 acc[DG / 16];
#pragma unroll
        for (int cb = 0; cb < DG / 16; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
        gather_records_mfma<DG, T, 16, true>(g, vals, masks, k, e0, e1, L.rp, reinterpret_cast<RecEdge*>(L.ebuf), L.rbuf, lane, acc,
                                             nullptr, lutf);
#pragma unroll
        for (int cb = 0; cb < DG / 16; ++cb) acc[cb][0] = quarter_sum(acc[cb][0]);
        hub_chunk_store<DG>(acc, part + (size_t)q * DG, lane);
    }
}
template <int DG, typename T>
__device__ __forceinline__ void hub_dense_pass(const CsrView& g, const HubChunks& h, const T* __restrict__ x, int64_t ld,
                                               float* __restrict__ part, HubLds& L, const HubSweep w) {
    const int lane = lane_id();
    for (int q = w.q; q < w.end; q += w.step) {
        const int e0 = __builtin_amdgcn_readfirstlane(h.ce0[q]), e1 = __builtin_amdgcn_readfirstlane(h.ce1[q]);
        hub_chunk_begin(L, e0, e1, lane);
        f32x4 acc[DG / 16];
#pragma unroll
        for (int cb = 0; cb < DG / 16; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
        gather_dense_mfma<DG, T, 16, true>(g, x, ld, e0, e1, L.rp, L.ebuf, lane, acc);
#pragma unroll
        for (int cb = 0; cb < DG / 16; ++cb) acc[cb][0] = quarter_sum(acc[cb][0]);
        hub_chunk_store<DG>(acc, part + (size_t)q * DG, lane);
    }
}

template <int DG, typename T>
__global__ __launch_bounds__(256) void k_hub_records(CsrView g, HubChunks h, const T* __restrict__ vals,
                                                     const typename MaskOf<DG>::type* __restrict__ masks, int k,
                                                     float* __restrict__ part) {
    __shared__ HubLds lds[4];
    __shared__ DealLutF dlut;
    deal_lutf_fill(dlut);
    hub_records_pass<DG, T>(g, h, vals, masks, k, part, lds[threadIdx.x >> 6], hub_sweep(h), &dlut);
}

template <int DG, typename T>
__global__ __launch_bounds__(256) void k_hub_dense(CsrView g, HubChunks h, const T* __restrict__ x, int64_t ld,
                                                   float* __restrict__ part) {
    __shared__ HubLds lds[4];
    hub_dense_pass<DG, T>(g, h, x, ld, part, lds[threadIdx.x >> 6], hub_sweep(h));
}

// Both first passes of one block's backward in one launch: blockIdx.y = 0 takes the records over A (for the
// inverse), blockIdx.y = 1 the dense gradient rows over A^T (for the data gradient).
template <int DG, typename T>
__global__ __launch_bounds__(256) void k_hub_both(CsrView ga, HubChunks ha, const T* __restrict__ vals,
                                                  const typename MaskOf<DG>::type* __restrict__ masks, int k,
                                                  float* __restrict__ part_a, CsrView gt, HubChunks ht,
                                                  const T* __restrict__ x, int64_t ld, float* __restrict__ part_t) {
    __shared__ HubLds lds[4];
    __shared__ DealLutF dlut;
    deal_lutf_fill(dlut);
    if (blockIdx.y == 0) hub_records_pass<DG, T>(ga, ha, vals, masks, k, part_a, lds[threadIdx.x >> 6], hub_sweep(ha), &dlut);
    else hub_dense_pass<DG, T>(gt, ht, x, ld, part_t, lds[threadIdx.x >> 6], hub_sweep(ht));
}

// ---- first pass over the chunks, value by value (float32 records) ---------------------------------
// On graphs where nearly every row is split the first pass is the step, and dealing a record to the lanes that own
// its columns (sixteen lanes, a four-slot window each: four times the record's bytes through the vector cache, some
// thirty instructions per four edges) is what it spends.  Here a lane owns a *value* instead: LPE = 2^LG lanes per
// edge, lane t of them loads value t (+ LPE, + 2 LPE .. below k) of the record and the number of its column - one
// byte per value, written from the column mask by k_record_columns before the pass (0xFF for a slot the record does
// not use: a column block of a wide group keeps between 0 and k values) - and adds a_ij * value to that
// column of its edge place's row in LDS (64 / LPE places, each a row of DG floats; the places of one instruction are
// different rows and the values of one record different columns, so no two lanes meet): the sum is read, added to
// and written back by the lane, and stays in the row for the whole chunk.  Even and odd instructions of a batch keep
// rows of their own, so two such chains are in flight.  At the end of a chunk the rows of the places are added in
// place order and cleared.  Scattering into zeroed rows, reading them back sixteen bytes wide into running sums and
// clearing them again was 3 % slower; LDS float atomics were four times slower than the dealing (one such
// instruction takes some 140 cycles).  The order of the additions is fixed by the edge list and the lane layout.
template <int DG>
__global__ __launch_bounds__(256) void k_record_columns(int n, int k, const typename MaskOf<DG>::type* __restrict__ masks,
                                                        uint8_t* __restrict__ cols) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    uint64_t m = (uint64_t)masks[j];
    uint8_t* o = cols + (size_t)j * k;
    if ((k & 3) == 0) {
        for (int t = 0; t < k; t += 4) {
            uint32_t w = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t c = m ? (uint32_t)__builtin_ctzll(m) : 0xFFu;
                m &= m - 1;
                w |= c << (8 * b);
            }
            *reinterpret_cast<uint32_t*>(o + t) = w;
        }
    } else {
        for (int t = 0; t < k; ++t) {
            o[t] = m ? (uint8_t)__builtin_ctzll(m) : (uint8_t)0xFF;
            m &= m - 1;
        }
    }
}

// The same for a group of S column blocks of 64 (S = 2 or 3: a column number must fit a byte beside the 0xFF of an
// unused slot): the k values a row keeps over its whole width, taken out of the S records of its column blocks into
// one list [n][k] with the column in the whole row beside each, so that one first pass serves all S blocks and every
// lane of it has a value (a pass per column block walks the edges S times with room for k values in each).
template <int S>
struct WideRecords {
    const float* vals[S];
    const uint64_t* mask[S];
};
template <int S>
__global__ __launch_bounds__(256) void k_record_columns_wide(int n, int k, WideRecords<S> r, float* __restrict__ vals,
                                                             uint8_t* __restrict__ cols) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    float* v = vals + (size_t)j * k;
    uint8_t* o = cols + (size_t)j * k;
    int pos = 0;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        uint64_t m = r.mask[s][j];
        const float* src = r.vals[s] + (size_t)j * k;
        for (int t = 0; m && pos < k; ++t, ++pos) {
            v[pos] = src[t];
            o[pos] = (uint8_t)(64 * s + __builtin_ctzll(m));
            m &= m - 1;
        }
    }
    for (; pos < k; ++pos) { v[pos] = 0.f; o[pos] = (uint8_t)0xFF; }
}

template <int DG, int LG>
struct HubValLds {
    uint2 ebuf[64];                   // (j * k, a_ij) of the staged edges
    float rows[2][(64 >> LG) * DG];   // two rows of sums per edge place (even and odd instructions of a batch)
    float spare[64];                  // where a lane without a value adds its zero
};

template <int DG, int LG, int KQ>
__device__ __forceinline__ void hub_values_pass(const CsrView& g, const HubChunks& h, const float* __restrict__ vals,
                                                const uint8_t* __restrict__ cols, int k, float* __restrict__ part,
                                                HubValLds<DG, LG>& L, const HubSweep w) {
    constexpr int LPE = 1 << LG, NE = 64 >> LG;          // lanes per edge, edges per instruction
    constexpr int MAXS = 64 / NE;                        // instructions per round of 64 staged edges
    constexpr int GB = KQ == 1 ? (MAXS < 8 ? MAXS : 8) : KQ == 2 ? 4 : 2;
    constexpr int TOT = NE * DG;
    static_assert(MAXS % GB == 0 && GB % 2 == 0, "a round is a whole number of batches, a batch of pairs");
    const int lane = lane_id();
    const int place = lane >> LG, t = lane & (LPE - 1);
    float* base = &L.rows[0][0];
    const int spare = (int)(&L.spare[lane] - base);
    for (int i = lane; i < 2 * TOT; i += 64) base[i] = 0.f;
    for (int q = w.q; q < w.end; q += w.step) {
        const int e0 = __builtin_amdgcn_readfirstlane(h.ce0[q]), e1 = __builtin_amdgcn_readfirstlane(h.ce1[q]);
        for (int eb = e0; eb < e1; eb += 64) {
            // places past the last edge: the last edge once more with a_ij = 0
            // (with sixteen lanes per edge a place is a row of sixteen lanes, and an instruction could take its edge
            // from a lane of the row by a DPP row broadcast instead of from LDS: measured 2.5 % slower)
            const int e = eb + lane;
            const bool ok = e < e1;
            const int ec = ok ? e : e1 - 1;
            const int j = __builtin_nontemporal_load(g.ci + ec);
            const float a = ok ? __builtin_nontemporal_load(g.av + ec) : 0.f;
            wave_sync();          // readers of the previous round are done
            L.ebuf[lane] = make_uint2((uint32_t)j * (uint32_t)k, __float_as_uint(a));
            wave_sync();
            const int cnt = e1 - eb < 64 ? e1 - eb : 64;
            const int steps = ((cnt + NE - 1) / NE + GB - 1) / GB * GB;
            for (int s0 = 0; s0 < steps; s0 += GB) {
                float v[GB][KQ];
                uint32_t c[GB][KQ];
#pragma unroll
                for (int u = 0; u < GB; ++u) {
                    const uint2 er = L.ebuf[(s0 + u) * NE + place];
#pragma unroll
                    for (int w = 0; w < KQ; ++w) {
                        // (a lane past the record's last slot takes slot 0 again: with one value per lane it writes
                        // what slot 0's lane writes)
                        const int tt = t + w * LPE;
                        const uint32_t at = er.x + (uint32_t)(tt < k ? tt : 0);
                        v[u][w] = vals[at] * __uint_as_float(er.y);
                        c[u][w] = cols[at];
                    }
                }
                // sum += value, read and written back: the lanes of an instruction hold different places or different
                // columns of one record, so no two of them meet; even and odd instructions keep rows of their own so
                // that two read - add - write chains are in flight
#pragma unroll
                for (int u = 0; u < GB; u += 2) {
#pragma unroll
                    for (int w = 0; w < KQ; ++w) {
                        const bool has = KQ == 1 || t + w * LPE < k;      // (else slot 0 once more: not added again)
                        const bool h0 = has && c[u][w] != 0xFFu, h1 = has && c[u + 1][w] != 0xFFu;
                        const int i0 = h0 ? place * DG + (int)c[u][w] : spare;
                        const int i1 = h1 ? TOT + place * DG + (int)c[u + 1][w] : spare;
                        const float o0 = base[i0];
                        const float o1 = base[i1];
                        wave_sync();
                        base[i0] = o0 + (h0 ? v[u][w] : 0.f);
                        base[i1] = o1 + (h1 ? v[u + 1][w] : 0.f);
                        wave_sync();
                    }
                }
            }
        }
        // the sums of the places are added in place order, even rows before odd rows, and the rows cleared
        // (DG > 64, a group of column blocks: part is [DG / 64][n_chunks][64], one array of partial rows per block)
        wave_sync();
#pragma unroll
        for (int c0 = 0; c0 < DG; c0 += 64) {
            const int c = c0 + lane;
            if (c < DG) {
                float s = 0.f;
#pragma unroll
                for (int pl = 0; pl < 2 * NE; ++pl) {
                    s += base[pl * DG + c];
                    base[pl * DG + c] = 0.f;
                }
                if (DG > 64) part[((size_t)(c0 >> 6) * h.n_chunks + q) * 64 + lane] = s;
                else part[(size_t)q * DG + lane] = s;
            }
        }
        wave_sync();
    }
}

// Lanes per edge and values per lane for k kept values: (4, 1), (8, 1), (16, 1), (16, 2), (16, 4).
template <typename F>
inline void hub_values_variant(int k, F&& f) {
    if (k <= 4) f(std::integral_constant<int, 2>{}, std::integral_constant<int, 1>{});
    else if (k <= 8) f(std::integral_constant<int, 3>{}, std::integral_constant<int, 1>{});
    else if (k <= 16) f(std::integral_constant<int, 4>{}, std::integral_constant<int, 1>{});
    else if (k <= 32) f(std::integral_constant<int, 4>{}, std::integral_constant<int, 2>{});
    else f(std::integral_constant<int, 4>{}, std::integral_constant<int, 4>{});
}

// The same for a group of column blocks (rows of 128 or 192 sums per edge place in LDS): at least eight lanes per edge.
template <typename F>
inline void hub_values_variant_wide(int k, F&& f) {
    if (k <= 8) f(std::integral_constant<int, 3>{}, std::integral_constant<int, 1>{});
    else if (k <= 16) f(std::integral_constant<int, 4>{}, std::integral_constant<int, 1>{});
    else if (k <= 32) f(std::integral_constant<int, 4>{}, std::integral_constant<int, 2>{});
    else f(std::integral_constant<int, 4>{}, std::integral_constant<int, 4>{});
}

template <int DG, int LG, int KQ>
__global__ __launch_bounds__(256) void k_hub_values(CsrView g, HubChunks h, const float* __restrict__ vals,
                                                    const uint8_t* __restrict__ cols, int k, float* __restrict__ part) {
    __shared__ HubValLds<DG, LG> lds[4];
    hub_values_pass<DG, LG, KQ>(g, h, vals, cols, k, part, lds[threadIdx.x >> 6], hub_sweep(h));
}

}  // namespace gsr
